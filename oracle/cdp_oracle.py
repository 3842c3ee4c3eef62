"""The CDP oracle: schedule, update rules and two independent trainers.

TEST INFRASTRUCTURE ONLY (see package docstring).

Notation (0-indexed; the paper is 1-indexed and takes #stages = #micro-batches):
  S  number of stages, N number of micro-batches, B micro-batch size,
  d  start delay between consecutive micro-batches in ticks ("time steps").
     The paper fixes d = 2 for S = N (Sec. 3.2, "Algorithmic description"); here
     d = 2S/N so that the cycle closes for S != N (a reading of the paper's
     "uniform delay"; it requires N | 2S).
  tick   one forward or one backward of one stage (Sec. 3.1, "Disadvantages of DP")
  step t indexes theta_t; one step = 2S ticks.
  phase p of a micro-batch in its own pass: p < S forward of stage p,
     p >= S backward of stage 2S-1-p.

Two trainers:
  * ``train_equation``  -- Eq. (CDP) evaluated literally from the full history
    theta_0..theta_t with the closed-form selector u_{i,j} (Eq. (CDP-v1), Eq.
    (CDP-v2), Eq. (DP)); an ordinary whole-network forward/backward per
    micro-batch.
  * ``train_schedule``  -- the tick-by-tick execution timeline of Fig. 1 with a
    two-slot weight ring per stage, gradient accumulators and activation
    bookkeeping; the selector is *operational* (v2: the freshest version held in
    memory, Sec. 3.2).  It also records the tick trace and live-buffer counts.
Their agreement is one of the pins; the others are in tests/test_oracle_*.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

import cdp_workloads as wl
from . import layers as L

FWD, BWD = 0, 1


# ---------------------------------------------------------------------------
# schedule (integers only)
# ---------------------------------------------------------------------------
def delay_for(S: int, N: int, rule: int) -> int:  # every cyclic rule (v1, v2, masks) shares the delay
    """Uniform start delay.  DP: all micro-batches in lock-step (Fig. 1a)."""
    if rule == wl.RULE_DP:
        return 0
    if (2 * S) % N != 0:
        raise ValueError("N must divide 2S")
    return 2 * S // N


def active_set(tick: int, S: int, N: int, d: int, T: int) -> List[Tuple[int, int, int, int]]:
    """(micro-batch i, step t, stage j, direction) for every micro-batch that works
    at ``tick``, i ascending.  Micro-batch i of step t starts at tick 2S*t + d*i."""
    out = []
    for i in range(N):
        rel = tick - d * i
        if rel < 0:
            continue
        t, p = divmod(rel, 2 * S)
        if t >= T:
            continue
        out.append((i, t, p, FWD) if p < S else (i, t, 2 * S - 1 - p, BWD))
    return out


def total_ticks(S: int, N: int, d: int, T: int) -> int:
    return 2 * S * T + d * (N - 1) if T > 0 else 0


def fresh_closed_form(rule: int, S: int, N: int, d: int, i: int, j: int, mask=None) -> bool:
    """u_{i,j} = a (use theta_t) iff this returns True, else b (theta_{t-1}).

    DP: always theta_t (Eq. (DP)).  v1: always theta_{t-1} (Eq. (CDP-v1)).
    v2: paper (1-indexed, S = N, d = 2): j >= N - i + 1.  General form derived
    from the timeline: stage j receives its N-th gradient of step t-1 at tick
    2S*t + 2S - d - 1 - j, micro-batch i of step t reads stage j at tick
    2S*t + d*i + j, hence fresh iff d*(i+1) + 2*j >= 2S.
    RULE_MASK (the rules "in between" of Sec. 3.2, "Update rules"): theta_t where
    mask[i][j] is set AND theta_t is already in memory (the v2 condition), else theta_{t-1};
    an all-ones mask is v2, an all-zeros mask is v1.
    """
    if rule == wl.RULE_DP:
        return True
    if rule == wl.RULE_V1:
        return False
    avail = d * (i + 1) + 2 * j >= 2 * S
    if rule == wl.RULE_MASK:
        return bool(mask[i][j]) and avail
    return avail


# ---------------------------------------------------------------------------
# results
# ---------------------------------------------------------------------------
@dataclass
class Result:
    params: List[List[np.ndarray]]                    # final theta_T per stage
    losses: np.ndarray                                # [T, N] micro-batch objectives f_i
    history: Optional[List[List[List[np.ndarray]]]] = None   # theta_0..theta_T (equation oracle)
    trace: List[Tuple[int, int, int, int, int, int]] = field(default_factory=list)  # (tick,i,t,j,dir,version)
    live_inputs: List[int] = field(default_factory=list)     # in-tick count of retained stage inputs
    updates: List[Tuple[int, int, int]] = field(default_factory=list)              # (tick, stage, new version)
    versions: Dict[Tuple[int, int], List[np.ndarray]] = field(default_factory=dict)  # (stage, version) -> params


def _copy_params(p):
    return [[np.array(a, dtype=np.float64) for a in st] for st in p]


# ---------------------------------------------------------------------------
# Oracle A: the update equation, literally
# ---------------------------------------------------------------------------
def sgd_update(w: np.ndarray, gsum: np.ndarray, v: Optional[np.ndarray], lr: float, N: int,
               momentum: float, weight_decay: float):
    """One SGD step on the summed micro-batch gradients.  Plain SGD (Eq. (CDP)):
    w - (lr/N) gsum.  With momentum / weight decay (the optimiser of Sec. 5
    "Hyperparameters", in the usual convention): g = gsum/N + wd*w, v = mu*v + g,
    w - lr*v.  Returns (w_new, v_new)."""
    if momentum == 0.0 and weight_decay == 0.0:
        return w - (lr / N) * gsum, v
    g = gsum / N + weight_decay * w
    v_new = g if v is None else momentum * v + g
    return w - lr * v_new, v_new


def train_equation(cfg: wl.Config, params0, xs: Sequence[np.ndarray], ys: Sequence[np.ndarray],
                   rule: int, lr: Optional[float] = None, stage_impl=None,
                   momentum: float = 0.0, weight_decay: float = 0.0, mask=None) -> Result:
    """theta_{t+1} = theta_t - (lr/N) sum_i grad f_i(theta_hat_{i,t}),
    theta_hat^j_{i,t} = theta^j_t if fresh(i,j) else theta^j_{t-1}, theta_{-1} := theta_0.
    ``stage_impl``: see train_schedule."""
    S, N, B = cfg.S, cfg.N, cfg.B
    lr = cfg.lr if lr is None else lr
    d = delay_for(S, N, rule)
    T = len(xs)
    hist = [_copy_params(params0)]
    vel = [[None for _ in st] for st in hist[0]]
    losses = np.zeros((T, N))
    for t in range(T):
        cur, prev = hist[t], hist[max(t - 1, 0)]
        gsum = [[np.zeros_like(a) for a in st] for st in cur]
        for i in range(N):
            mix = [cur[j] if fresh_closed_form(rule, S, N, d, i, j, mask) else prev[j] for j in range(S)]
            x = np.asarray(xs[t][i * B:(i + 1) * B], dtype=np.float64)
            y = np.asarray(ys[t][i * B:(i + 1) * B])
            loss, grads = L.model_forward_backward(cfg.stages, mix, x, y, stage_impl)
            losses[t, i] = loss
            for j in range(S):
                for a, g in zip(gsum[j], grads[j]):
                    a += g
        new = []
        for j in range(S):
            stage_new = []
            for k, (w, g) in enumerate(zip(cur[j], gsum[j])):
                w2, vel[j][k] = sgd_update(w, g, vel[j][k], lr, N, momentum, weight_decay)
                stage_new.append(w2)
            new.append(stage_new)
        hist.append(new)
    return Result(params=hist[-1], losses=losses, history=hist)


# ---------------------------------------------------------------------------
# Oracle B: the execution timeline, tick by tick
# ---------------------------------------------------------------------------
def train_schedule(cfg: wl.Config, params0, xs: Sequence[np.ndarray], ys: Sequence[np.ndarray],
                   rule: int, lr: Optional[float] = None, stage_impl=None,
                   compute: bool = True, keep_versions: bool = True,
                   progress: Optional[Callable[[int, int], None]] = None,
                   momentum: float = 0.0, weight_decay: float = 0.0, mask=None, bwd_fresh: bool = False) -> Result:
    """Per tick: every active micro-batch runs one stage forward or backward with the
    weight version the rule assigns (forward) or the one its own forward used
    (backward); a backward adds its gradient to the stage accumulator; at the end of
    the tick every stage holding N gradients is updated into the other ring slot and
    the new version becomes visible from the next tick.  ``compute=False`` runs the
    integer bookkeeping only (trace, versions, live counts); ``keep_versions=False`` does
    not retain superseded weight versions (large models); ``progress(tick, n_ticks)`` is
    called after every tick.

    ``stage_impl`` (tests only): an object with prepare_input(x), forward(stage, params, x,
    labels) and backward(stage, params, saved, dy) that stands in for the identity and for
    layers.stage_forward / layers.stage_backward, e.g. a copy of them that rounds stored
    tensors to a storage format.  The timeline, the rule and the update stay the ones here.

    ``mask`` (RULE_MASK): N x S array; forward (i, j) reads the freshest version where
    mask[i][j] is set, theta_{t-1} elsewhere.
    ``bwd_fresh``: the variant Sec. 3.2 alludes to when it says that no second copy of
    the parameters is needed: the backward reads the parameters that are freshest in
    memory at ITS tick (every parameter the backward formulas touch), on the activations
    its forward saved.  The applied gradient is then no longer the gradient of f_i at one
    point, so this variant has no counterpart in the equation oracle; the trace records the
    version the backward read."""
    S, N, B = cfg.S, cfg.N, cfg.B
    lr = cfg.lr if lr is None else lr
    d = delay_for(S, N, rule)
    T = len(xs)
    stage_fwd = L.stage_forward if stage_impl is None else stage_impl.forward
    stage_bwd = L.stage_backward if stage_impl is None else stage_impl.backward
    ring = [[_copy_params([params0[j]])[0], _copy_params([params0[j]])[0]] for j in range(S)] if compute \
        else [[None, None] for _ in range(S)]
    ring_ver = [[0, 0] for _ in range(S)]        # which version each slot currently holds
    ver = [0] * S                                # freshest version of each stage
    G = [[np.zeros_like(a) for a in ring[j][0]] for j in range(S)] if compute else [None] * S
    vel = [[None for _ in ring[j][0]] for j in range(S)] if compute else [None] * S
    cnt = [0] * S
    used: Dict[Tuple[int, int, int], int] = {}   # (t, i, j) -> version read by the forward
    saved: Dict[Tuple[int, int, int], object] = {}
    carry: Dict[Tuple[int, int], object] = {}    # (t, i) -> activation / gradient travelling between stages
    res = Result(params=[], losses=np.zeros((T, N)))
    if compute and keep_versions:
        for j in range(S):
            res.versions[(j, 0)] = ring[j][0]
    for tick in range(total_ticks(S, N, d, T)):
        act = active_set(tick, S, N, d, T)
        # retained stage inputs while this tick's kernels run: a forward has already
        # stored its input, a backward has not yet released it
        live = len(saved) + sum(1 for (_, _, _, dr) in act if dr == FWD)
        res.live_inputs.append(live)
        for (i, t, j, dr) in act:
            if dr == FWD:
                if rule == wl.RULE_V2 or (rule == wl.RULE_MASK and mask[i][j]):
                    v = ver[j]                      # freshest parameters in memory
                elif rule == wl.RULE_V1 or rule == wl.RULE_MASK:
                    v = max(t - 1, 0)               # theta_{t-1}
                else:
                    v = t                           # theta_t
                assert ring_ver[j][v % 2] == v, "ring depth 2 violated (fwd)"
                used[(t, i, j)] = v
                if compute:
                    if j == 0:
                        carry[(t, i)] = np.asarray(xs[t][i * B:(i + 1) * B], dtype=np.float64)
                        if stage_impl is not None:
                            carry[(t, i)] = stage_impl.prepare_input(carry[(t, i)])
                    lab = np.asarray(ys[t][i * B:(i + 1) * B]) if j == S - 1 else None
                    out, sv = stage_fwd(cfg.stages[j], ring[j][v % 2], carry[(t, i)], lab)
                    saved[(t, i, j)] = sv
                    if j == S - 1:
                        res.losses[t, i] = out
                        carry[(t, i)] = None
                    else:
                        carry[(t, i)] = out
                else:
                    saved[(t, i, j)] = True
            else:
                v = used.pop((t, i, j))
                if bwd_fresh:
                    v = ver[j]
                assert ring_ver[j][v % 2] == v, "ring depth 2 violated (bwd)"
                sv = saved.pop((t, i, j))
                if compute:
                    dx, grads = stage_bwd(cfg.stages[j], ring[j][v % 2], sv, carry[(t, i)])
                    carry[(t, i)] = dx
                    if j == 0:
                        del carry[(t, i)]
                    for a, g in zip(G[j], grads):
                        a += g
                cnt[j] += 1
            res.trace.append((tick, i, t, j, dr, v))
        for j in range(S):
            if cnt[j] == N:
                new = ver[j] + 1
                if compute:
                    stage_new = []
                    for k, (w, g) in enumerate(zip(ring[j][ver[j] % 2], G[j])):
                        w2, vel[j][k] = sgd_update(w, g, vel[j][k], lr, N, momentum, weight_decay)
                        stage_new.append(w2)
                    ring[j][new % 2] = stage_new
                    for a in G[j]:
                        a[...] = 0.0
                    if keep_versions:
                        res.versions[(j, new)] = ring[j][new % 2]
                ring_ver[j][new % 2] = new
                ver[j] = new
                cnt[j] = 0
                res.updates.append((tick, j, new))
        if progress is not None:
            progress(tick, total_ticks(S, N, d, T))
    assert not saved and not used and all(c == 0 for c in cnt)
    assert all(v == T for v in ver)
    if compute:
        res.params = [ring[j][ver[j] % 2] for j in range(S)]
    return res


# ---------------------------------------------------------------------------
# helpers shared by the tests
# ---------------------------------------------------------------------------
def max_rel_err(got: Sequence[np.ndarray], ref: Sequence[np.ndarray]) -> float:
    """Per tensor max|got-ref| / max|ref|; the maximum over tensors."""
    worst = 0.0
    for g, r in zip(got, ref):
        r = np.asarray(r, dtype=np.float64)
        den = float(np.abs(r).max()) if r.size else 0.0
        num = float(np.abs(np.asarray(g, dtype=np.float64) - r).max()) if r.size else 0.0
        if den == 0.0:
            worst = max(worst, 0.0 if num == 0.0 else float("inf"))
        else:
            worst = max(worst, num / den)
    return worst


def stage_rel_err(got: Sequence[np.ndarray], ref: Sequence[np.ndarray]) -> float:
    """max|got-ref| / max|ref| over the whole parameter vector theta^j of one stage."""
    g = np.concatenate([np.asarray(a, dtype=np.float64).ravel() for a in got])
    r = np.concatenate([np.asarray(a, dtype=np.float64).ravel() for a in ref])
    return float(np.abs(g - r).max() / np.abs(r).max())


def dp_peak_live_inputs(S: int, N: int) -> int:
    """Lock-step DP retains every stage input of every micro-batch at the end of the
    forward pass (Table 1, row "Single-GPU DP": N*B*Psi_A)."""
    return N * S


def cdp_live_inputs(S: int, N: int) -> float:
    """Table 1, row "+ Cyclic": (N+1)/2 * B*Psi_A with Psi_A = S stage units when S = N;
    for general S, N the in-tick count is N(S+1)/2."""
    return N * (S + 1) / 2
