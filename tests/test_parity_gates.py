"""The acceptance criteria of the GPU parity tests (tests/parity_gates.py) against mistakes planted
on the oracle side: each gate must accept the reference and reject a result with a lost, mis-scaled
or misplaced update."""
import copy

import numpy as np
import pytest

import cdp_workloads as wl
from oracle import cdp_oracle as O
from precision_standins import Bf16Storage, Fp32Accumulation
import parity_gates as G


@pytest.fixture(scope="module")
def runs():
    cfg = wl.get_config("cfg2_mini")
    T = 3
    xs, ys = wl.make_data(cfg, T, 0)
    p0 = wl.init_params(cfg, 0)
    ref = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, keep_versions=False)
    emu = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, keep_versions=False, stage_impl=Bf16Storage)
    return cfg, p0, xs, ys, ref, emu


def test_reference_and_emulation_pass(runs):
    cfg, p0, xs, ys, ref, emu = runs
    assert G.f32_gate(ref.params, ref.params)[0]
    ok, rep = G.bf16_gate(emu.params, ref.params, emu.params, p0)
    assert ok and rep["worst_ratio"] <= 1.0 / G.BF16_K + 1e-12 and 0 < rep["emu_median"] < 0.2


def test_unchanged_initial_weights_fail_both_gates(runs):
    cfg, p0, xs, ys, ref, emu = runs
    assert not G.f32_gate(p0, ref.params)[0]
    ok, rep = G.bf16_gate(p0, ref.params, emu.params, p0)
    assert not ok
    # every tensor fails, not just one: the update error of theta_0 is exactly 1
    assert sum(1 for f in rep["failed"] if f[0] == "tensor") == sum(len(st) for st in p0)


def test_one_tensor_without_its_update_fails(runs):
    cfg, p0, xs, ys, ref, emu = runs
    for j, t in [(0, 1), (cfg.S - 1, 0), (1, 1)]:      # a bias, the classifier's weight, another bias
        got = copy.deepcopy(emu.params)
        got[j][t] = np.asarray(p0[j][t], dtype=np.float64)
        ok, rep = G.bf16_gate(got, ref.params, emu.params, p0)
        assert not ok and any(f[:3] == ("tensor", j, t) for f in rep["failed"])
        got = copy.deepcopy(ref.params)
        got[j][t] = np.asarray(p0[j][t], dtype=np.float64)
        assert not G.f32_gate(got, ref.params)[0]


def test_wrong_rule_and_wrong_scale_fail_the_fp32_gates(runs):
    """What the fp32 runs of every configuration are there for: a wrong weight version (v1 read where v2
    is due, the lock-step rule) or a gradient sum scaled by (N-1)/N fails the strict gate and the
    yardstick gate with the fp32 stand-in."""
    cfg, p0, xs, ys, ref, emu = runs
    emu32 = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, keep_versions=False, stage_impl=Fp32Accumulation(1)).params
    assert G.yardstick_gate(emu32, ref.params, emu32, p0, 3, bf16=False)[0]
    v1 = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V1, keep_versions=False)
    scaled = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, keep_versions=False, lr=cfg.lr * (cfg.N - 1) / cfg.N)
    dp = O.train_schedule(cfg, p0, xs, ys, wl.RULE_DP, keep_versions=False)
    for wrong in (v1, scaled, dp):
        assert not G.f32_gate(wrong.params, ref.params)[0]
        ok, rep = G.yardstick_gate(wrong.params, ref.params, emu32, p0, 3, bf16=False)
        assert not ok and any(f[0] == "tensor" for f in rep["failed"])


def test_fp32_master_resolution_is_allowed_for(runs):
    """A tensor whose update is smaller than what an fp32 master copy resolves (a gamma near 1 that barely
    moves): rounding the result to fp32 must pass the yardstick gate."""
    cfg, p0, xs, ys, ref, emu = runs
    p0b = [[np.asarray(w, dtype=np.float64) for w in st] for st in p0]
    refb = [[np.asarray(w, dtype=np.float64).copy() for w in st] for st in ref.params]
    p0b[0][1] = np.ones_like(p0b[0][1])
    refb[0][1] = 1.0 + 3e-7 * wl.random_normal(3, 1, refb[0][1].size)       # an update of a few ulp of 1.0f
    got = [[a.astype(np.float32).astype(np.float64) for a in st] for st in refb]
    ok, rep = G.yardstick_gate(got, refb, refb, p0b, 3, bf16=False)
    assert ok and G.update_err(got[0][1], refb[0][1], p0b[0][1]) > 0.05


def test_update_twice_as_large_fails_the_bf16_gate(runs):
    cfg, p0, xs, ys, ref, emu = runs
    got = [[2.0 * np.asarray(r) - np.asarray(w0, dtype=np.float64) for r, w0 in zip(rs, ws)] for rs, ws in zip(ref.params, p0)]
    assert not G.bf16_gate(got, ref.params, emu.params, p0)[0]


def test_stage_impl_hook_with_the_oracle_s_own_functions_changes_nothing(runs):
    from oracle import layers as L
    cfg, p0, xs, ys, ref, emu = runs

    class Own:
        prepare_input = staticmethod(lambda x: x)
        forward = staticmethod(L.stage_forward)
        backward = staticmethod(L.stage_backward)

    again = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, keep_versions=False, stage_impl=Own)
    for a, b in zip(again.params, ref.params):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    # and the equation form agrees with the timeline form under the bf16-storage stand-in as well
    eq = O.train_equation(cfg, p0, xs, ys, wl.RULE_V2, stage_impl=Bf16Storage)
    assert O.max_rel_err([t for st in eq.params for t in st], [t for st in emu.params for t in st]) < 1e-12


def test_stand_in_rounding_equals_the_oracle_s():
    import precision_standins as PS
    from oracle import layers as L
    x = np.concatenate([wl.random_normal(5, 1, 100000) * 10.0 ** wl.random_normal(5, 2, 100000),
                        [0.0, -0.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 3.0e38, -3.0e38, 1e-40]])
    assert np.array_equal(PS.round_bf16(x), L.round_bf16(x))
