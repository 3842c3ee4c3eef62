"""Seeded synthetic workloads for Cyclic Data Parallelism (CDP) training.

This module is the only code shared by the CPU oracle and the HIP library's
tests/bench.  It holds *no* arithmetic of the method: only

  * the layer-kind vocabulary (integer codes equal to the ``cdp_layer_kind``
    enum of ``include/cdp.h``),
  * the five model configurations named by the benchmark (stage partitions as
    lists of layer descriptors),
  * a counter-based random generator (splitmix64 -> Box-Muller) that is
    specified bit-exactly here, so the same host arrays are handed to both the
    oracle and the library,
  * the initial-parameter recipe (Kaiming-normal weights, zero biases).

Inputs stand in for CIFAR-10 / ImageNet records (paper Sec. 5,
"Hyperparameters"): same shapes and label cardinalities, values i.i.d. N(0,1),
labels i.i.d. uniform.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# layer vocabulary (must equal enum cdp_layer_kind in include/cdp.h)
# ---------------------------------------------------------------------------
LINEAR = 1    # p = (in_features, out_features)              params: W[out,in], b[out]
RELU = 2      # p = ()
CONV2D = 3    # p = (cin, cout, ksize, stride, pad)          params: W[cout,k,k,cin]
AFFINE = 4    # p = (channels,)                              params: gamma[c], beta[c]
ADD = 5       # p = (src2,)   y = tensor[src] + tensor[src2]
MAXPOOL = 6   # p = (ksize, stride, pad)
GAP = 7       # p = ()   global average pool NHWC -> [B, C]
CE_HEAD = 8   # p = (classes,)  mean softmax cross-entropy over the micro-batch
LAYERNORM = 9   # p = (channels,)  over the channel axis of every position     params: gamma[c], beta[c]
GELU = 10       # p = ()   x * Phi(x), exact (erf) form
TOKENS = 12     # p = ()   [H, W, C] -> [1, H*W, C]: the patch grid read as one row of tokens (no data movement)
ATTENTION = 11  # p = (heads,)  self-attention core on tokens [B, 1, T, 3*D] = (q | k | v) per token,
                #              each D = heads * dh wide: out[B, 1, T, D] = softmax(q k^T / sqrt(dh)) v per head

KIND_NAMES = {LINEAR: "linear", RELU: "relu", CONV2D: "conv2d", AFFINE: "affine",
              ADD: "add", MAXPOOL: "maxpool", GAP: "gap", CE_HEAD: "ce_head", LAYERNORM: "layernorm",
              GELU: "gelu", ATTENTION: "attention", TOKENS: "tokens"}

# update rules (must equal enum cdp_rule)
RULE_DP = 0
RULE_V1 = 1
RULE_V2 = 2
RULE_MASK = 3   # per (micro-batch, stage) choice between the v2 and the v1 selector
RULE_NAMES = {RULE_DP: "dp", RULE_V1: "cdp_v1", RULE_V2: "cdp_v2", RULE_MASK: "cdp_mask"}

# compute dtypes (must equal enum cdp_dtype)
F32 = 0
BF16 = 1


@dataclass(frozen=True)
class Layer:
    """One layer of a stage.

    Tensor numbering inside a stage: tensor 0 is the stage input, tensor k+1 is
    the output of layer k.  ``src`` is the tensor the layer reads (-1 = output
    of the previous layer, i.e. tensor k for layer k).
    """
    kind: int
    p: Tuple[int, ...] = ()
    src: int = -1


@dataclass
class Config:
    name: str
    stages: List[List[Layer]]
    in_shape: Tuple[int, ...]      # per-sample input shape (features,) or (H, W, C)
    classes: int
    N: int                         # micro-batches per mini-batch
    B: int                         # micro-batch size
    dtype: int                     # F32 or BF16
    lr: float
    steps: int                     # steps for the parity run
    init_gain_last_affine: float = 1.0
    init_gain_head: float = 1.0    # scale on the classifier weights (the LINEAR feeding CE_HEAD)
    notes: str = ""

    @property
    def S(self) -> int:
        return len(self.stages)

    @property
    def delay(self) -> int:
        assert (2 * self.S) % self.N == 0
        return 2 * self.S // self.N


# ---------------------------------------------------------------------------
# shape inference / parameter shapes (pure bookkeeping)
# ---------------------------------------------------------------------------
def layer_param_shapes(layer: Layer) -> List[Tuple[int, ...]]:
    k, p = layer.kind, layer.p
    if k == LINEAR:
        return [(p[1], p[0]), (p[1],)]
    if k == CONV2D:
        cin, cout, ks = p[0], p[1], p[2]
        return [(cout, ks, ks, cin)]
    if k in (AFFINE, LAYERNORM):
        return [(p[0],), (p[0],)]
    return []


def layer_out_shape(layer: Layer, in_shape: Tuple[int, ...],
                    shapes: Sequence[Tuple[int, ...]]) -> Tuple[int, ...]:
    """Per-sample output shape of ``layer`` given its per-sample input shape."""
    k, p = layer.kind, layer.p
    if k == LINEAR:
        n_in = int(np.prod(in_shape))
        assert n_in == p[0], (in_shape, p)
        return (p[1],)
    if k in (RELU, AFFINE, GELU):
        return tuple(in_shape)
    if k == LAYERNORM:
        assert in_shape[-1] == p[0], (in_shape, p)
        return tuple(in_shape)
    if k == TOKENS:
        h, w, c = in_shape
        return (1, h * w, c)
    if k == ATTENTION:
        h, w, c = in_shape
        assert h == 1 and c % (3 * p[0]) == 0, (in_shape, p)
        return (1, w, c // 3)
    if k == ADD:
        assert tuple(shapes[p[0]]) == tuple(in_shape), (shapes[p[0]], in_shape)
        return tuple(in_shape)
    if k == CONV2D:
        h, w, c = in_shape
        cin, cout, ks, st, pad = p
        assert c == cin, (in_shape, p)
        return ((h + 2 * pad - ks) // st + 1, (w + 2 * pad - ks) // st + 1, cout)
    if k == MAXPOOL:
        h, w, c = in_shape
        ks, st, pad = p
        return ((h + 2 * pad - ks) // st + 1, (w + 2 * pad - ks) // st + 1, c)
    if k == GAP:
        return (in_shape[2],)
    if k == CE_HEAD:
        assert in_shape == (p[0],)
        return ()
    raise ValueError(k)


def stage_tensor_shapes(stage: Sequence[Layer], in_shape: Tuple[int, ...]) -> List[Tuple[int, ...]]:
    shapes = [tuple(in_shape)]
    for idx, layer in enumerate(stage):
        src = idx if layer.src < 0 else layer.src
        shapes.append(layer_out_shape(layer, shapes[src], shapes))
    return shapes


def config_stage_in_shapes(cfg: Config) -> List[Tuple[int, ...]]:
    out = []
    shp = tuple(cfg.in_shape)
    for st in cfg.stages:
        out.append(shp)
        shp = stage_tensor_shapes(st, shp)[-1]
    return out


def stage_param_shapes(stage: Sequence[Layer]) -> List[Tuple[int, ...]]:
    out: List[Tuple[int, ...]] = []
    for layer in stage:
        out.extend(layer_param_shapes(layer))
    return out


def stage_param_count(stage: Sequence[Layer]) -> int:
    return int(sum(int(np.prod(s)) for s in stage_param_shapes(stage)))


# ---------------------------------------------------------------------------
# model builders
# ---------------------------------------------------------------------------
def _mlp(in_dim: int, width: int, n_stages: int, classes: int, stem: bool) -> List[List[Layer]]:
    stages: List[List[Layer]] = []
    for j in range(n_stages):
        st: List[Layer] = []
        if j == 0 and stem:
            st += [Layer(LINEAR, (in_dim, width)), Layer(RELU)]
        cin = in_dim if (j == 0 and not stem) else width
        st += [Layer(LINEAR, (cin, width)), Layer(RELU)]
        if j == n_stages - 1:
            st += [Layer(LINEAR, (width, classes)), Layer(CE_HEAD, (classes,))]
        stages.append(st)
    return stages


def _conv_affine(cin, cout, ks, stride, pad, src=-1) -> List[Layer]:
    return [Layer(CONV2D, (cin, cout, ks, stride, pad), src), Layer(AFFINE, (cout,))]


def _basic_block(cin: int, cout: int, stride: int, base: int) -> List[Layer]:
    """ResNet BasicBlock; ``base`` = tensor index of the block input inside the stage."""
    layers: List[Layer] = []
    t = base  # running tensor index of the last produced tensor
    if stride != 1 or cin != cout:
        layers += _conv_affine(cin, cout, 1, stride, 0, src=base)
        t += 2
        short = t
    else:
        short = base
    layers += _conv_affine(cin, cout, 3, stride, 1, src=base) + [Layer(RELU)]
    layers += _conv_affine(cout, cout, 3, 1, 1)
    layers += [Layer(ADD, (short,)), Layer(RELU)]
    return layers


def _bottleneck(cin: int, width: int, stride: int, base: int) -> List[Layer]:
    cout = 4 * width
    layers: List[Layer] = []
    t = base
    if stride != 1 or cin != cout:
        layers += _conv_affine(cin, cout, 1, stride, 0, src=base)
        t += 2
        short = t
    else:
        short = base
    layers += _conv_affine(cin, width, 1, 1, 0, src=base) + [Layer(RELU)]
    layers += _conv_affine(width, width, 3, stride, 1) + [Layer(RELU)]
    layers += _conv_affine(width, cout, 1, 1, 0)
    layers += [Layer(ADD, (short,)), Layer(RELU)]
    return layers


def _resnet18_cifar(classes: int, widths=(64, 128, 256, 512)) -> List[List[Layer]]:
    stages: List[List[Layer]] = []
    cin = widths[0]
    blocks = []
    for gi, w in enumerate(widths):
        for bi in range(2):
            stride = 2 if (gi > 0 and bi == 0) else 1
            blocks.append((cin, w, stride))
            cin = w
    for j, (ci, co, s) in enumerate(blocks):
        st: List[Layer] = []
        if j == 0:
            st += _conv_affine(3, widths[0], 3, 1, 1) + [Layer(RELU)]
        st += _basic_block(ci, co, s, base=len(st))
        if j == len(blocks) - 1:
            st += [Layer(GAP), Layer(LINEAR, (co, classes)), Layer(CE_HEAD, (classes,))]
        stages.append(st)
    return stages


def _resnet50(classes: int, widths=(64, 128, 256, 512), depths=(3, 4, 6, 3)) -> List[List[Layer]]:
    stages: List[List[Layer]] = []
    cin = widths[0]
    blocks = []
    for gi, (w, dep) in enumerate(zip(widths, depths)):
        for bi in range(dep):
            stride = 2 if (gi > 0 and bi == 0) else 1
            blocks.append((cin, w, stride))
            cin = 4 * w
    for j, (ci, w, s) in enumerate(blocks):
        st: List[Layer] = []
        if j == 0:
            st += _conv_affine(3, widths[0], 7, 2, 3) + [Layer(RELU), Layer(MAXPOOL, (3, 2, 1))]
        st += _bottleneck(ci, w, s, base=len(st))
        if j == len(blocks) - 1:
            st += [Layer(GAP), Layer(LINEAR, (4 * w, classes)), Layer(CE_HEAD, (classes,))]
        stages.append(st)
    return stages


def _vit(image: int, patch: int, dim: int, heads: int, depth: int, classes: int) -> List[List[Layer]]:
    """ViT-shaped stages on tokens kept as a [1, T, D] "image": patch embedding (a patch x patch /
    patch convolution, then the patch grid is read as one row of T tokens), one pre-norm
    transformer block per stage, mean pooling over the tokens and a linear classifier.  A
    token-wise linear map is a 1x1 convolution followed by a per-channel affine (scale and bias;
    the scale is an extra parameter a plain ViT does not have, initialised to 1)."""
    def block(base: int) -> List[Layer]:
        ls = [Layer(LAYERNORM, (dim,), src=base)]
        ls += _conv_affine(dim, 3 * dim, 1, 1, 0) + [Layer(ATTENTION, (heads,))]
        ls += _conv_affine(dim, dim, 1, 1, 0) + [Layer(ADD, (base,))]
        mid = base + len(ls)
        ls += [Layer(LAYERNORM, (dim,))]
        ls += _conv_affine(dim, 4 * dim, 1, 1, 0) + [Layer(GELU)]
        ls += _conv_affine(4 * dim, dim, 1, 1, 0) + [Layer(ADD, (mid,))]
        return ls
    stages: List[List[Layer]] = []
    for j in range(depth):
        st: List[Layer] = []
        if j == 0:
            st += _conv_affine(3, dim, patch, patch, 0) + [Layer(TOKENS)]
        st += block(len(st))
        if j == depth - 1:
            st += [Layer(LAYERNORM, (dim,)), Layer(GAP), Layer(LINEAR, (dim, classes)), Layer(CE_HEAD, (classes,))]
        stages.append(st)
    return stages


def get_config(name: str) -> Config:
    """The five benchmark configurations plus reduced "mini" variants for tests."""
    if name == "cfg1":
        return Config("cfg1", _mlp(64, 64, 4, 10, stem=False), (64,), 10, N=4, B=8,
                      dtype=F32, lr=0.05, steps=20, notes="Tiny MLP")
    if name == "cfg2":
        return Config("cfg2", _mlp(3072, 1024, 8, 10, stem=True), (3072,), 10, N=8, B=32,
                      dtype=BF16, lr=0.05, steps=50, notes="CIFAR-shaped MLP")
    if name == "cfg3":
        return Config("cfg3", _resnet18_cifar(10), (32, 32, 3), 10, N=4, B=32,
                      dtype=BF16, lr=0.05, steps=10, init_gain_last_affine=0.25, init_gain_head=0.05,
                      notes="CIFAR-shaped ResNet-18")
    if name == "cfg4":
        return Config("cfg4", _resnet50(1000), (224, 224, 3), 1000, N=8, B=32,
                      dtype=BF16, lr=0.01, steps=4, init_gain_last_affine=0.25, init_gain_head=0.05,
                      notes="ImageNet-shaped ResNet-50")
    if name == "cfg5":
        return Config("cfg5", _mlp(4096, 4096, 24, 1000, stem=False), (4096,), 1000, N=16, B=64,
                      dtype=BF16, lr=0.05, steps=10, notes="Deep wide MLP stress")
    # ---- reduced variants (same structure, small enough for the CPU suite) ----
    if name == "mlp_mini":       # S=3, N=3: the paper's worked example size (Fig. 1)
        return Config("mlp_mini", _mlp(12, 16, 3, 5, stem=False), (12,), 5, N=3, B=4,
                      dtype=F32, lr=0.1, steps=6)
    if name == "mlp_odd":        # odd delay d=3, ragged sizes, stem + 2-layer head
        return Config("mlp_odd", _mlp(40, 72, 6, 7, stem=True), (40,), 7, N=4, B=5,
                      dtype=F32, lr=0.05, steps=6)
    if name == "mlp_longk":      # long, ragged reduction in the stem (1100 inputs), 40-wide layers, B = 5
        return Config("mlp_longk", _mlp(1100, 40, 4, 7, stem=True), (1100,), 7, N=4, B=5,
                      dtype=F32, lr=0.05, steps=4)
    if name == "mlp_longk_b40":  # the same stem with micro-batches of 40 rows: 64-row tiles
        c = get_config("mlp_longk")
        c.name, c.B = "mlp_longk_b40", 40
        return c
    if name == "mlp_longk_bf16":  # 2120 inputs: 34 slabs of 64, the last one partial
        return Config("mlp_longk_bf16", _mlp(2120, 136, 4, 10, stem=True), (2120,), 10, N=4, B=24,
                      dtype=BF16, lr=0.02, steps=4)
    if name == "cfg2_mini":      # bf16, several tiles + ragged tail
        return Config("cfg2_mini", _mlp(200, 136, 4, 10, stem=True), (200,), 10, N=4, B=24,
                      dtype=BF16, lr=0.05, steps=8)
    if name == "cfg5_mini":      # bf16, d=3, N=16
        return Config("cfg5_mini", _mlp(320, 320, 24, 100, stem=False), (320,), 100, N=16, B=40,
                      dtype=BF16, lr=0.05, steps=5)
    if name == "resnet18_mini":  # 8 BasicBlock stages at 1/8 width, 8x8 images
        return Config("resnet18_mini", _resnet18_cifar(10, widths=(8, 16, 32, 64)), (8, 8, 3), 10,
                      N=4, B=4, dtype=BF16, lr=0.05, steps=5, init_gain_last_affine=0.25)
    if name == "resnet18_mini_f32":
        c = get_config("resnet18_mini")
        c.name, c.dtype = "resnet18_mini_f32", F32
        return c
    if name == "resnet18_odd_f32":  # 9x9 images: image rows of 27 elements are not whole 16-byte pieces, maps of 9, 5, 3, 2
        c = get_config("resnet18_mini")
        c.name, c.dtype, c.in_shape, c.B = "resnet18_odd_f32", F32, (9, 9, 3), 3
        return c
    if name == "resnet18_odd":
        c = get_config("resnet18_odd_f32")
        c.name, c.dtype = "resnet18_odd", BF16
        return c
    if name == "resnet50_mini":  # 16 bottleneck stages at 1/8 width, 32x32 images
        return Config("resnet50_mini", _resnet50(20, widths=(8, 16, 32, 64)), (32, 32, 3), 20,
                      N=8, B=2, dtype=BF16, lr=0.05, steps=4, init_gain_last_affine=0.25)
    if name == "vit_mini":       # 4 transformer-block stages, 16 tokens of width 32, 4 heads
        return Config("vit_mini", _vit(16, 4, 32, 4, 4, 10), (16, 16, 3), 10, N=4, B=4, dtype=BF16, lr=0.05, steps=5,
                      init_gain_last_affine=0.25, init_gain_head=0.2)
    if name == "vit_mini_f32":
        c = get_config("vit_mini")
        c.name, c.dtype = "vit_mini_f32", F32
        return c
    if name == "vit_odd":        # 9 tokens of width 20, heads of width 5: no multiple of four, rows not whole 16-byte chunks in bf16
        return Config("vit_odd", _vit(12, 4, 20, 4, 2, 5), (12, 12, 3), 5, N=4, B=3, dtype=F32, lr=0.05, steps=4,
                      init_gain_last_affine=0.25, init_gain_head=0.2)
    if name == "vit_odd_bf16":
        c = get_config("vit_odd")
        c.name, c.dtype = "vit_odd_bf16", BF16
        return c
    if name == "vit_long":       # 324 tokens of width 16 in 2 heads
        return Config("vit_long", _vit(36, 2, 16, 2, 2, 5), (36, 36, 3), 5, N=2, B=2, dtype=F32, lr=0.05, steps=3,
                      init_gain_last_affine=0.25, init_gain_head=0.2)
    if name == "vit_b16":        # ViT-B/16-shaped: 196 tokens of width 768, 12 heads, 12 block stages
        return Config("vit_b16", _vit(224, 16, 768, 12, 12, 1000), (224, 224, 3), 1000, N=8, B=32, dtype=BF16, lr=0.01,
                      steps=2, init_gain_last_affine=0.25, init_gain_head=0.2, notes="ViT-B/16-shaped")
    if name == "cfg4_s64":       # the ResNet-50 configuration with 64x64 inputs: every stage at its real channel widths,
        c = get_config("cfg4")   # N = 8 micro-batches of 32, at 1/12 of the oracle's cost
        c.name, c.in_shape, c.steps = "cfg4_s64", (64, 64, 3), 3
        return c
    if name == "resnet50_mini_f32":
        c = get_config("resnet50_mini")
        c.name, c.dtype = "resnet50_mini_f32", F32
        return c
    raise KeyError(name)


# ---------------------------------------------------------------------------
# counter-based random numbers: splitmix64 hash of (seed, stream, counter)
# ---------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z += np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def random_u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words: word c = mix(mix(seed*2^32 + stream) + c)."""
    key = _splitmix64(np.array([(seed << 32) ^ (stream & 0xFFFFFFFF)], dtype=np.uint64))[0]
    ctr = np.arange(offset, offset + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _splitmix64(ctr + key)


def random_uniform(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """float64 uniform in (0, 1): (top 53 bits + 0.5) / 2^53."""
    u = random_u64(seed, stream, n, offset) >> np.uint64(11)
    return (u.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def random_normal(seed: int, stream: int, n: int) -> np.ndarray:
    """float64 N(0,1) by Box-Muller on consecutive uniform pairs."""
    m = (n + 1) // 2
    u = random_uniform(seed, stream, 2 * m)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    th = (2.0 * math.pi) * u[1::2]
    out = np.empty(2 * m, dtype=np.float64)
    out[0::2] = r * np.cos(th)
    out[1::2] = r * np.sin(th)
    return out[:n]


def random_labels(seed: int, stream: int, n: int, classes: int) -> np.ndarray:
    return (random_u64(seed, stream, n) % np.uint64(classes)).astype(np.int32)


# ---------------------------------------------------------------------------
# data and initial parameters
# ---------------------------------------------------------------------------
_STREAM_X = 1
_STREAM_Y = 2
_STREAM_W = 1000


def make_batch(cfg: Config, step: int, seed: int = 0):
    """Mini-batch ``step``: x float32 [N*B, *in_shape] ~ N(0,1), y int32 [N*B] uniform."""
    rows = cfg.N * cfg.B
    per = int(np.prod(cfg.in_shape))
    x = random_normal(seed, _STREAM_X + 16 * step, rows * per).astype(np.float32)
    y = random_labels(seed, _STREAM_Y + 16 * step, rows, cfg.classes)
    return x.reshape((rows,) + tuple(cfg.in_shape)), y


def make_data(cfg: Config, steps: int, seed: int = 0):
    xs, ys = zip(*(make_batch(cfg, t, seed) for t in range(steps)))
    return list(xs), list(ys)


def init_params(cfg: Config, seed: int = 0) -> List[List[np.ndarray]]:
    """theta_0: per stage, the list of float32 parameter tensors in layer order.

    Linear / conv weights ~ N(0, 2/fan_in); biases 0; affine gamma 1, beta 0,
    except the affine that feeds a residual ADD, whose gamma is
    ``cfg.init_gain_last_affine`` (keeps activations bounded without
    normalisation layers), and the classifier weights, which are scaled by
    ``cfg.init_gain_head`` (the pooled features are all positive, so a
    Kaiming-scaled classifier would start with logits of std ~5).
    """
    out: List[List[np.ndarray]] = []
    stream = _STREAM_W
    for st in cfg.stages:
        plist: List[np.ndarray] = []
        for li, layer in enumerate(st):
            if layer.kind == LINEAR:
                fan_in = layer.p[0]
                w = random_normal(seed, stream, layer.p[0] * layer.p[1]) * math.sqrt(2.0 / fan_in)
                if li + 1 < len(st) and st[li + 1].kind == CE_HEAD:
                    w = w * cfg.init_gain_head
                stream += 1
                plist.append(w.astype(np.float32).reshape(layer.p[1], layer.p[0]))
                plist.append(np.zeros(layer.p[1], dtype=np.float32))
            elif layer.kind == CONV2D:
                cin, cout, ks = layer.p[0], layer.p[1], layer.p[2]
                fan_in = cin * ks * ks
                w = random_normal(seed, stream, cout * fan_in) * math.sqrt(2.0 / fan_in)
                stream += 1
                plist.append(w.astype(np.float32).reshape(cout, ks, ks, cin))
            elif layer.kind == LAYERNORM:
                plist.append(np.ones(layer.p[0], dtype=np.float32))
                plist.append(np.zeros(layer.p[0], dtype=np.float32))
            elif layer.kind == AFFINE:
                feeds_add = li + 1 < len(st) and st[li + 1].kind == ADD
                g = cfg.init_gain_last_affine if feeds_add else 1.0
                plist.append(np.full(layer.p[0], g, dtype=np.float32))
                plist.append(np.zeros(layer.p[0], dtype=np.float32))
        out.append(plist)
    return out


def flatten_params(plist: Sequence[np.ndarray]) -> np.ndarray:
    if not plist:
        return np.zeros(0, dtype=np.float32)
    return np.concatenate([np.asarray(p, dtype=np.float32).ravel() for p in plist])


def unflatten_params(flat: np.ndarray, stage: Sequence[Layer]) -> List[np.ndarray]:
    out, off = [], 0
    for shp in stage_param_shapes(stage):
        n = int(np.prod(shp))
        out.append(np.asarray(flat[off:off + n]).reshape(shp))
        off += n
    assert off == flat.size
    return out
