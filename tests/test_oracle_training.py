"""Pins of the oracle's trainers: equation == timeline, reductions to textbook SGD,
delayed-gradient recurrences re-derived with PyTorch autograd.  No GPU."""
import numpy as np
import pytest
import torch

import cdp_workloads as wl
from oracle import cdp_oracle as O
from oracle import layers as L
from test_oracle_layers import torch_forward, to_torch_params, to_torch_x
from precision_standins import Bf16Storage, Fp32Accumulation

RULES = [wl.RULE_DP, wl.RULE_V1, wl.RULE_V2]


def _setup(name, T, seed=0, N=None):
    cfg = wl.get_config(name)
    if N is not None:
        cfg.N = N
    xs, ys = wl.make_data(cfg, T, seed)
    return cfg, wl.init_params(cfg, seed), xs, ys


def _torch_grads(cfg, params, x, y):
    tp = to_torch_params(params)
    loss = torch_forward(cfg.stages, tp, to_torch_x(x), torch.tensor(np.asarray(y), dtype=torch.long))
    loss.backward()
    return float(loss), [[t.grad.numpy() for t in st] for st in tp]


def _close(a, b, tol=1e-10):
    return O.max_rel_err(a, b) <= tol


@pytest.mark.parametrize("name", ["mlp_mini", "mlp_odd", "resnet18_mini", "vit_mini", "vit_odd"])
@pytest.mark.parametrize("rule", RULES)
def test_equation_oracle_equals_timeline_oracle(name, rule):
    """Eq. (CDP) with the closed-form selector == tick-by-tick execution with the ring."""
    cfg, p0, xs, ys = _setup(name, 4 if name in ("mlp_mini", "mlp_odd") else 3)
    a = O.train_equation(cfg, p0, xs, ys, rule)
    b = O.train_schedule(cfg, p0, xs, ys, rule)
    for j in range(cfg.S):
        assert _close(b.params[j], a.params[j], 1e-12)
        for t in range(len(xs) + 1):
            assert _close(b.versions[(j, t)], a.history[t][j], 1e-12)
    assert np.abs(a.losses - b.losses).max() < 1e-12


@pytest.mark.parametrize("name", ["mlp_mini", "resnet18_mini", "vit_mini"])
def test_first_step_is_textbook_minibatch_sgd_under_every_rule(name):
    """theta_{-1} := theta_0, so theta_1 = theta_0 - lr * grad of the mean loss over all
    N*B samples (Eq. (DP)) whatever the rule; the gradient comes from torch autograd."""
    cfg, p0, xs, ys = _setup(name, 1)
    _, g = _torch_grads(cfg, p0, xs[0], ys[0])        # mean over N*B samples
    want = [[np.asarray(w, dtype=np.float64) - cfg.lr * gw for w, gw in zip(ws, gs)] for ws, gs in zip(p0, g)]
    for rule in RULES:
        r = O.train_schedule(cfg, p0, xs, ys, rule)
        for j in range(cfg.S):
            assert _close(r.params[j], want[j], 1e-10)


@pytest.mark.parametrize("rule", [wl.RULE_DP, wl.RULE_V2])
def test_single_microbatch_is_plain_sgd(rule):
    """Sec. 3.2: with one micro-batch, j >= N-i+1 holds for every stage, so CDP-v2 is SGD."""
    cfg, p0, xs, ys = _setup("mlp_odd", 5, N=1)
    tp = to_torch_params(p0)
    opt = torch.optim.SGD([t for st in tp for t in st], lr=cfg.lr)
    for t in range(5):
        opt.zero_grad()
        torch_forward(cfg.stages, tp, to_torch_x(xs[t]), torch.tensor(ys[t], dtype=torch.long)).backward()
        opt.step()
    r = O.train_schedule(cfg, p0, xs, ys, rule)
    for j in range(cfg.S):
        assert _close(r.params[j], [t.detach().numpy() for t in tp[j]], 1e-10)


def test_single_microbatch_v1_is_delay_one_sgd():
    """Eq. (CDP-v1) with N = 1: theta_{t+1} = theta_t - lr * grad f_t(theta_{t-1})."""
    cfg, p0, xs, ys = _setup("mlp_odd", 5, N=1)
    hist = [[[np.asarray(w, dtype=np.float64) for w in st] for st in p0]]
    for t in range(5):
        _, g = _torch_grads(cfg, hist[max(t - 1, 0)], xs[t], ys[t])
        hist.append([[w - cfg.lr * gw for w, gw in zip(ws, gs)] for ws, gs in zip(hist[t], g)])
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V1)
    for j in range(cfg.S):
        assert _close(r.params[j], hist[-1][j], 1e-10)


@pytest.mark.parametrize("rule", RULES)
def test_zero_learning_rate_freezes_weights(rule):
    cfg, p0, xs, ys = _setup("mlp_mini", 3)
    r = O.train_schedule(cfg, p0, xs, ys, rule, lr=0.0)
    for j in range(cfg.S):
        for a, b in zip(r.params[j], p0[j]):
            assert np.array_equal(a, np.asarray(b, dtype=np.float64))


def test_v2_applied_gradient_is_gradient_at_paper_mixed_point():
    """Eq. (CDP-v2), literally and 1-indexed: micro-batch i is differentiated at
    (theta^1_{t-1},...,theta^{N-i}_{t-1}, theta^{N-i+1}_t,...,theta^N_t).  Gradients from
    torch autograd, versions from the timeline oracle's own history."""
    cfg, p0, xs, ys = _setup("mlp_mini", 4)
    N, B = cfg.N, cfg.B
    assert cfg.S == N
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2)
    for t in range(4):
        gsum = None
        for i1 in range(1, N + 1):
            mix = [r.versions[(j1 - 1, t if j1 >= N - i1 + 1 else max(t - 1, 0))] for j1 in range(1, N + 1)]
            sl = slice((i1 - 1) * B, i1 * B)
            loss, g = _torch_grads(cfg, mix, xs[t][sl], ys[t][sl])
            assert abs(loss - r.losses[t, i1 - 1]) < 1e-10
            gsum = g if gsum is None else [[a + b for a, b in zip(x, y)] for x, y in zip(gsum, g)]
        for j in range(N):
            want = [w - cfg.lr / N * gw for w, gw in zip(r.versions[(j, t)], gsum[j])]
            assert _close(r.versions[(j, t + 1)], want, 1e-10)


def test_v1_is_delay_one_minibatch_sgd_with_autograd():
    """Eq. (CDP-v1): all N micro-batch gradients of step t at theta_{t-1}."""
    cfg, p0, xs, ys = _setup("mlp_mini", 4)
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V1)
    for t in range(4):
        prev = [r.versions[(j, max(t - 1, 0))] for j in range(cfg.S)]
        _, g = _torch_grads(cfg, prev, xs[t], ys[t])       # mean over N*B == (1/N) sum_i grad f_i
        for j in range(cfg.S):
            want = [w - cfg.lr * gw for w, gw in zip(r.versions[(j, t)], g[j])]
            assert _close(r.versions[(j, t + 1)], want, 1e-10)


def test_rules_differ_after_the_first_step():
    """A dropped or swapped selector would make two rules coincide."""
    cfg, p0, xs, ys = _setup("mlp_mini", 3)
    res = {rule: O.train_schedule(cfg, p0, xs, ys, rule) for rule in RULES}
    for a in RULES:
        for b in RULES:
            if a < b:
                assert O.max_rel_err(res[a].params[0], res[b].params[0]) > 1e-6


def test_bf16_emulation_stays_close_to_fp64():
    cfg, p0, xs, ys = _setup("cfg2_mini", 3)
    a = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2)
    b = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, stage_impl=Bf16Storage)
    for j in range(cfg.S):
        # per stage vector theta^j; single tensors that start at zero (biases) see O(10%) of
        # their own small range from isolated ReLU sign flips, so they are not the gate
        e = O.stage_rel_err(b.params[j], a.params[j])
        assert 0 < e < 2e-2


# --- momentum and weight decay (the optimiser the paper trained with, Sec. 5) -----------------
@pytest.mark.parametrize("rule", [wl.RULE_DP, wl.RULE_V2])
def test_momentum_weight_decay_single_microbatch_is_torch_sgd(rule):
    cfg, p0, xs, ys = _setup("mlp_odd", 5, N=1)
    tp = to_torch_params(p0)
    opt = torch.optim.SGD([t for st in tp for t in st], lr=cfg.lr, momentum=0.9, weight_decay=5e-4)
    for t in range(5):
        opt.zero_grad()
        torch_forward(cfg.stages, tp, to_torch_x(xs[t]), torch.tensor(ys[t], dtype=torch.long)).backward()
        opt.step()
    r = O.train_schedule(cfg, p0, xs, ys, rule, momentum=0.9, weight_decay=5e-4)
    for j in range(cfg.S):
        assert _close(r.params[j], [t.detach().numpy() for t in tp[j]], 1e-10)


def test_momentum_dp_minibatch_is_torch_sgd():
    """Eq. (DP) with N micro-batches: the summed gradient / N is the mini-batch mean gradient."""
    cfg, p0, xs, ys = _setup("mlp_mini", 4)
    tp = to_torch_params(p0)
    opt = torch.optim.SGD([t for st in tp for t in st], lr=cfg.lr, momentum=0.9, weight_decay=1e-3)
    for t in range(4):
        opt.zero_grad()
        torch_forward(cfg.stages, tp, to_torch_x(xs[t]), torch.tensor(ys[t], dtype=torch.long)).backward()
        opt.step()
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_DP, momentum=0.9, weight_decay=1e-3)
    for j in range(cfg.S):
        assert _close(r.params[j], [t.detach().numpy() for t in tp[j]], 1e-10)


@pytest.mark.parametrize("rule", RULES)
def test_momentum_equation_equals_timeline(rule):
    cfg, p0, xs, ys = _setup("mlp_odd", 4)
    a = O.train_equation(cfg, p0, xs, ys, rule, momentum=0.9, weight_decay=5e-4)
    b = O.train_schedule(cfg, p0, xs, ys, rule, momentum=0.9, weight_decay=5e-4)
    for j in range(cfg.S):
        assert _close(b.params[j], a.params[j], 1e-12)
    plain = O.train_schedule(cfg, p0, xs, ys, rule)
    assert O.max_rel_err(b.params[0], plain.params[0]) > 1e-6


# ---------------------------------------------------------------------------
# rules between v1 and v2 (Sec. 3.2, "Update rules"), and the backward that reads the
# freshest parameters
# ---------------------------------------------------------------------------
def _rand_mask(cfg, seed):
    return np.random.default_rng(seed).integers(0, 2, (cfg.N, cfg.S))


@pytest.mark.parametrize("name", ["mlp_mini", "mlp_odd", "resnet18_mini"])
def test_mask_rule_with_constant_masks_is_v1_and_v2(name):
    cfg, p0, xs, ys = _setup(name, 3)
    for const, rule in ((1, wl.RULE_V2), (0, wl.RULE_V1)):
        m = np.full((cfg.N, cfg.S), const)
        a = O.train_schedule(cfg, p0, xs, ys, wl.RULE_MASK, mask=m)
        b = O.train_schedule(cfg, p0, xs, ys, rule)
        assert a.trace == b.trace and a.live_inputs == b.live_inputs
        assert np.array_equal(a.losses, b.losses)
        for j in range(cfg.S):
            for u, v in zip(a.params[j], b.params[j]):
                assert np.array_equal(u, v)


@pytest.mark.parametrize("name", ["mlp_mini", "mlp_odd", "resnet18_mini"])
@pytest.mark.parametrize("seed", [1, 2])
def test_mask_rule_equation_equals_timeline(name, seed):
    cfg, p0, xs, ys = _setup(name, 3)
    m = _rand_mask(cfg, seed)
    a = O.train_equation(cfg, p0, xs, ys, wl.RULE_MASK, mask=m)
    b = O.train_schedule(cfg, p0, xs, ys, wl.RULE_MASK, mask=m)
    for j in range(cfg.S):
        assert _close(b.params[j], a.params[j], 1e-12)
    assert np.abs(a.losses - b.losses).max() < 1e-12


def test_mask_rule_gradient_point_with_autograd():
    """Micro-batch i is differentiated at theta^j_t where the mask allows it AND the v2
    condition j >= N-i+1 (1-indexed, S = N) holds, at theta^j_{t-1} elsewhere."""
    cfg, p0, xs, ys = _setup("mlp_mini", 4)
    N, B = cfg.N, cfg.B
    m = _rand_mask(cfg, 5)
    assert 0 < m.sum() < m.size
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_MASK, mask=m)
    for t in range(4):
        gsum = None
        for i1 in range(1, N + 1):
            mix = [r.versions[(j1 - 1, t if (m[i1 - 1][j1 - 1] and j1 >= N - i1 + 1) else max(t - 1, 0))]
                   for j1 in range(1, N + 1)]
            sl = slice((i1 - 1) * B, i1 * B)
            _, g = _torch_grads(cfg, mix, xs[t][sl], ys[t][sl])
            gsum = g if gsum is None else [[a + b for a, b in zip(x, y)] for x, y in zip(gsum, g)]
        for j in range(N):
            want = [w - cfg.lr / N * gw for w, gw in zip(r.versions[(j, t)], gsum[j])]
            assert _close(r.versions[(j, t + 1)], want, 1e-10)
    v1 = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V1)
    v2 = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2)
    assert not _close(r.params[1], v1.params[1], 1e-6) and not _close(r.params[1], v2.params[1], 1e-6)


def test_bwd_fresh_degenerate_cases_are_the_exact_rules():
    """One micro-batch, the lock-step rule and the first step never see two versions."""
    cfg, p0, xs, ys = _setup("mlp_odd", 3, N=1)
    a = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, bwd_fresh=True)
    b = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2)
    assert a.trace == b.trace
    for j in range(cfg.S):
        assert all(np.array_equal(u, v) for u, v in zip(a.params[j], b.params[j]))
    cfg, p0, xs, ys = _setup("mlp_mini", 3)
    a = O.train_schedule(cfg, p0, xs, ys, wl.RULE_DP, bwd_fresh=True)
    b = O.train_schedule(cfg, p0, xs, ys, wl.RULE_DP)
    for j in range(cfg.S):
        assert all(np.array_equal(u, v) for u, v in zip(a.params[j], b.params[j]))
    a = O.train_schedule(cfg, p0, xs[:1], ys[:1], wl.RULE_V2, bwd_fresh=True)
    b = O.train_schedule(cfg, p0, xs[:1], ys[:1], wl.RULE_V2)
    for j in range(cfg.S):
        assert all(np.array_equal(u, v) for u, v in zip(a.params[j], b.params[j]))


def test_bwd_fresh_reads_the_freshest_version_and_matches_autograd_surrogate():
    """(a) every backward record carries the number of updates its stage has received before
    that tick; (b) the applied gradient equals backpropagation in which the Jacobian with
    respect to a layer's input is taken with the backward's parameters and everything else
    (values, ReLU masks, weight gradients) with the forward's.  Built with torch autograd:
    linear(x) = linear(x.detach(); W_f) + (x W_b^T - (x W_b^T).detach())."""
    cfg, p0, xs, ys = _setup("mlp_mini", 4)
    N, B, S = cfg.N, cfg.B, cfg.S
    r = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, bwd_fresh=True)
    exact = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2)
    assert not _close(r.params[1], exact.params[1], 1e-6)       # it is a different iteration
    n_upd = {}
    for (tick, i, t, j, dr, v) in r.trace:
        if dr == O.BWD:
            assert v == sum(1 for (ut, uj, _) in r.updates if uj == j and ut < tick)
    vf = {(t, i, j): v for (_, i, t, j, dr, v) in r.trace if dr == O.FWD}
    vb = {(t, i, j): v for (_, i, t, j, dr, v) in r.trace if dr == O.BWD}
    assert any(vf[k] != vb[k] for k in vf)

    def surrogate(t, i):
        pf = [to_torch_params([r.versions[(j, vf[(t, i, j)])]])[0] for j in range(S)]
        pb = [[torch.tensor(np.asarray(a)) for a in r.versions[(j, vb[(t, i, j)])]] for j in range(S)]
        h = to_torch_x(xs[t][i * B:(i + 1) * B])
        y = torch.tensor(np.asarray(ys[t][i * B:(i + 1) * B]), dtype=torch.long)
        for j in range(S):
            k = 0
            for layer in cfg.stages[j]:
                if layer.kind == wl.LINEAR:
                    Wf, bf, Wb = pf[j][k], pf[j][k + 1], pb[j][k]
                    lin_b = h @ Wb.T
                    h = torch.nn.functional.linear(h.detach(), Wf, bf) + (lin_b - lin_b.detach())
                    k += 2
                elif layer.kind == wl.RELU:
                    h = torch.relu(h)
                else:
                    assert layer.kind == wl.CE_HEAD
                    h = torch.nn.functional.cross_entropy(h, y)
        h.backward()
        return [[p.grad.numpy() for p in st] for st in pf]

    for t in range(4):
        gsum = None
        for i in range(N):
            g = surrogate(t, i)
            gsum = g if gsum is None else [[a + b for a, b in zip(x, y)] for x, y in zip(gsum, g)]
        for j in range(S):
            want = [w - cfg.lr / N * gw for w, gw in zip(r.versions[(j, t)], gsum[j])]
            assert _close(r.versions[(j, t + 1)], want, 1e-10)
