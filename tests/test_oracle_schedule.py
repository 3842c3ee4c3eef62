"""Pins of the oracle's schedule and version rules against what the paper prints.

No GPU.  Each test cites the passage that fixes the expected value.
"""
import itertools

import numpy as np
import pytest

import cdp_workloads as wl
from oracle import cdp_oracle as O
from conftest import read_golden

SN = [(3, 3), (4, 4), (8, 8), (8, 4), (16, 8), (24, 16), (4, 1), (4, 2), (4, 8), (6, 4), (5, 2), (5, 10)]


def _cfg(S, N):
    stages = [[wl.Layer(wl.LINEAR, (2, 2)), wl.Layer(wl.RELU)] for _ in range(S)]
    return wl.Config("t", stages, (2,), 2, N=N, B=1, dtype=wl.F32, lr=0.1, steps=1)


def _run(S, N, rule, T):
    return O.train_schedule(_cfg(S, N), None, [None] * T, [None] * T, rule, compute=False)


def test_fig1_dp_timeline():
    """Sec. 3.1: 2N ticks per step, activation peak at tick 2, barrier between ticks 5 and 6."""
    g = read_golden("fig1_timeline_n3.txt")
    N, S = int(g["n_workers"]), int(g["n_stages"])
    r = _run(S, N, wl.RULE_DP, 2)
    peak = int(g["dp_activation_peak_tick"])
    assert r.live_inputs[peak] == N * S == max(r.live_inputs)
    assert all(v < N * S for v in r.live_inputs[:peak])
    last = int(g["dp_barrier_after_tick"])
    assert int(g["ticks_per_training_step"]) == 2 * N == last + 1
    # every stage holds theta_1 once the barrier tick is over (per-stage writes may land earlier:
    # nothing reads them before the next step, so the arithmetic is that of a barrier update)
    assert max(tick for (tick, j, v) in r.updates if v == 1) == last
    assert min(tick for (tick, i, t, j, d, v) in r.trace if t == 1) == last + 1
    assert max(tick for (tick, i, t, j, d, v) in r.trace if t == 0) == last


def test_fig1_cdp_timeline():
    """Fig. 1 caption: delay of 2 ticks between workers; Sec. 3.2: the N-th micro-batch
    finishes at tick 9, where CDP-v1 places its barrier."""
    g = read_golden("fig1_timeline_n3.txt")
    N, S = int(g["n_workers"]), int(g["n_stages"])
    for rule in (wl.RULE_V1, wl.RULE_V2):
        r = _run(S, N, rule, 2)
        starts = {i: min(tick for (tick, ii, t, j, d, v) in r.trace if ii == i and t == 0) for i in range(N)}
        assert [starts[i + 1] - starts[i] for i in range(N - 1)] == [int(g["cdp_delay_ticks"])] * (N - 1)
        end = max(tick for (tick, i, t, j, d, v) in r.trace if t == 0)
        assert end == int(g["cdp_v1_barrier_tick"])
        # all of theta_1 exists once that tick is over, none of theta_2 before
        assert max(tick for (tick, j, v) in r.updates if v == 1) == end


def test_v2_rule_table_from_paper():
    """Sec. 3.2: u_{i,j} = a iff j >= N - i + 1 (1-indexed), spelled out for N = 3."""
    g = read_golden("cdp_v2_rule.txt")
    N = int(g["n"])
    r = _run(N, N, wl.RULE_V2, 4)
    used = {(t, i, j): v for (tick, i, t, j, d, v) in r.trace if d == O.FWD}
    for i1 in range(1, N + 1):
        row = [int(s) for s in g["row_i%d" % i1].split()]
        for j1 in range(1, N + 1):
            assert row[j1 - 1] == int(j1 >= N - i1 + 1)
            for t in range(1, 4):
                assert used[(t, i1 - 1, j1 - 1)] == (t if row[j1 - 1] else t - 1)
            assert O.fresh_closed_form(wl.RULE_V2, N, N, 2, i1 - 1, j1 - 1) == bool(row[j1 - 1])


@pytest.mark.parametrize("S,N", SN)
def test_v2_freshest_equals_closed_form(S, N):
    """Operational rule (Sec. 3.2: whatever parameters are in memory are the freshest ones) ==
    closed form d(i+1)+2j >= 2S, which is the paper's predicate when S = N."""
    T = 4
    r = _run(S, N, wl.RULE_V2, T)
    d = 2 * S // N
    for (tick, i, t, j, dr, v) in r.trace:
        want = t if (O.fresh_closed_form(wl.RULE_V2, S, N, d, i, j) or t == 0) else t - 1
        assert v == want
        if S == N and t > 0:
            assert (v == t) == ((j + 1) >= N - (i + 1) + 1)


@pytest.mark.parametrize("S,N", SN)
def test_v1_and_dp_versions(S, N):
    """Eq. (CDP-v1): every gradient of step t at theta_{t-1}; Eq. (DP): at theta_t."""
    for rule in (wl.RULE_V1, wl.RULE_DP):
        r = _run(S, N, rule, 4)
        for (tick, i, t, j, dr, v) in r.trace:
            assert v == (max(t - 1, 0) if rule == wl.RULE_V1 else t)


@pytest.mark.parametrize("S,N", SN)
def test_backward_uses_forward_version_and_chain_order(S, N):
    r = _run(S, N, wl.RULE_V2, 3)
    fwd = {(t, i, j): (tick, v) for (tick, i, t, j, dr, v) in r.trace if dr == O.FWD}
    bwd = {(t, i, j): (tick, v) for (tick, i, t, j, dr, v) in r.trace if dr == O.BWD}
    assert set(fwd) == set(bwd) == set(itertools.product(range(3), range(N), range(S)))
    d = 2 * S // N
    for (t, i, j), (tick, v) in fwd.items():
        assert tick == 2 * S * t + d * i + j
        assert bwd[(t, i, j)] == (2 * S * t + d * i + 2 * S - 1 - j, v)


@pytest.mark.parametrize("S,N", SN)
def test_live_stage_inputs_constant(S, N):
    """Table 1 "+ Cyclic": (N+1)/2 B Psi_A against N B Psi_A for DP; Sec. 4.1: "nearly
    constant across time steps".  In stage-input units the in-tick count is N(S+1)/2 in
    every steady-state tick; DP peaks at N*S."""
    T = 4
    d = 2 * S // N
    r = _run(S, N, wl.RULE_V2, T)
    steady = r.live_inputs[d * (N - 1):2 * S * T]
    assert abs(np.mean(steady) - O.cdp_live_inputs(S, N)) < 1e-9
    if N >= 2:       # a single micro-batch cannot be constant: it ramps 1..S..1
        assert set(steady) == {N * (S + 1) // 2}
    assert max(_run(S, N, wl.RULE_DP, 2).live_inputs) == O.dp_peak_live_inputs(S, N)
    if S == N:       # the paper's case, Table 1 literally: (N+1)/2 of N stage inputs vs N of N
        assert max(steady) * 2 == (N + 1) * S


def test_live_counts_baseline_configs():
    """The values for the worked example and the five benchmark configurations."""
    want = {(3, 3): 6, (4, 4): 10, (8, 8): 36, (8, 4): 18, (16, 8): 68, (24, 16): 200}
    for (S, N), n in want.items():
        r = _run(S, N, wl.RULE_V2, 3)
        d = 2 * S // N
        steady = r.live_inputs[d * (N - 1):2 * S * 3]
        assert max(steady) == n, (S, N, max(steady))
        assert n == N * (S + 1) // 2


@pytest.mark.parametrize("S,N", [(3, 3), (4, 4), (8, 8), (8, 4), (16, 8), (4, 2)])
def test_each_stage_one_pass_per_tick_even_delay(S, N):
    """Sec. 3.2: each stage performs either a forward or a backward on a single, distinct
    micro-batch per tick (holds when the delay is even)."""
    r = _run(S, N, wl.RULE_V2, 3)
    seen = {}
    for (tick, i, t, j, dr, v) in r.trace:
        assert (tick, j) not in seen
        seen[(tick, j)] = i
    if S == N:  # steady state: every stage is busy every tick
        for tick in range(2 * (N - 1), 2 * S * 3):
            assert sum(1 for (tk, j) in seen if tk == tick) == S


def test_odd_delay_same_stage_fwd_and_bwd_never_two_bwd():
    """With an odd delay a stage may see one forward and one backward in a tick, but
    never two backwards (accumulation order stays well defined)."""
    r = _run(24, 16, wl.RULE_V2, 3)
    per = {}
    for (tick, i, t, j, dr, v) in r.trace:
        per.setdefault((tick, j, dr), []).append(i)
    assert all(len(v) == 1 for v in per.values())
    assert any((tick, j, O.BWD) in per for (tick, j, dr) in per if dr == O.FWD)


@pytest.mark.parametrize("S,N", SN)
def test_updates_once_per_step_per_stage(S, N):
    T = 3
    for rule in (wl.RULE_V1, wl.RULE_V2, wl.RULE_DP):
        r = _run(S, N, rule, T)
        assert sorted((j, v) for (_, j, v) in r.updates) == sorted(itertools.product(range(S), range(1, T + 1)))
