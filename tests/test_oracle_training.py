"""Pins of the oracle's trainers: equation == timeline, reductions to textbook SGD,
delayed-gradient recurrences re-derived with PyTorch autograd.  No GPU."""
import numpy as np
import pytest
import torch

import cdp_workloads as wl
from oracle import cdp_oracle as O
from oracle import layers as L
from test_oracle_layers import torch_forward, to_torch_params, to_torch_x

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


@pytest.mark.parametrize("name", ["mlp_mini", "mlp_odd", "resnet18_mini"])
@pytest.mark.parametrize("rule", RULES)
def test_equation_oracle_equals_timeline_oracle(name, rule):
    """Eq. (CDP) with the closed-form selector == tick-by-tick execution with the ring."""
    cfg, p0, xs, ys = _setup(name, 4 if name != "resnet18_mini" else 3)
    a = O.train_equation(cfg, p0, xs, ys, rule)
    b = O.train_schedule(cfg, p0, xs, ys, rule)
    for j in range(cfg.S):
        assert _close(b.params[j], a.params[j], 1e-12)
        for t in range(len(xs) + 1):
            assert _close(b.versions[(j, t)], a.history[t][j], 1e-12)
    assert np.abs(a.losses - b.losses).max() < 1e-12


@pytest.mark.parametrize("name", ["mlp_mini", "resnet18_mini"])
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
    b = O.train_schedule(cfg, p0, xs, ys, wl.RULE_V2, rnd=L.round_bf16)
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
