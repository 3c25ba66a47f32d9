"""Seeded synthetic workloads for the Two-Branch Swin Block.

This module only draws inputs: feature maps, int8 weights with their
per-channel scales, LayerNorm parameters, biases, a relative-position-bias
tensor and quantizer (scale, zero point) pairs.  It holds none of the block's
arithmetic, so the HIP path and the test oracle can both be fed from it.

The shapes follow the Swin-T / Swin-B stages at detection scale (800x1344 and
1024x1024 images); the maps stand in for COCO-derived feature maps, which are
not available here.  Quantizer ranges are closed-form constants per tensor
(normalised activations have known spread), not a calibration pass.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

WINDOW = 7
TOKENS = WINDOW * WINDOW


@dataclass
class BlockSpec:
    """Shape and precision of one block (the fields of the C descriptor)."""
    B: int
    H: int
    W: int
    C: int
    heads: int
    shift: int = 0
    mlp_ratio: int = 4
    act_bits_high: int = 8
    act_bits_low: int = 4
    weight_bits: int = 8
    score_mode: int = 0
    ln_eps: float = 1e-5
    window: int = WINDOW

    @property
    def Hp(self):
        return -(-self.H // self.window) * self.window

    @property
    def Wp(self):
        return -(-self.W // self.window) * self.window

    @property
    def nW(self):
        return (self.Hp // self.window) * (self.Wp // self.window)


@dataclass
class BranchParams:
    ln1_gamma: np.ndarray
    ln1_beta: np.ndarray
    ln2_gamma: np.ndarray
    ln2_beta: np.ndarray
    b_qkv: np.ndarray
    b_proj: np.ndarray
    b_fc1: np.ndarray
    b_fc2: np.ndarray
    # name -> (scale, zero_point); names: a_qkv_in a_q a_k a_v a_p a_proj_in a_fc1_in a_fc2_in
    q: Dict[str, tuple] = field(default_factory=dict)


@dataclass
class SharedParams:
    w_qkv: np.ndarray
    w_proj: np.ndarray
    w_fc1: np.ndarray
    w_fc2: np.ndarray
    s_qkv: np.ndarray
    s_proj: np.ndarray
    s_fc1: np.ndarray
    s_fc2: np.ndarray
    rel_pos_bias: np.ndarray
    score_gamma: Optional[np.ndarray] = None
    score_beta: Optional[np.ndarray] = None


@dataclass
class BlockInputs:
    spec: BlockSpec
    shared: SharedParams
    branches: List[BranchParams]


QNAMES = ("a_qkv_in", "a_q", "a_k", "a_v", "a_p", "a_proj_in", "a_fc1_in", "a_fc2_in")

# Clip ranges [lo, hi] of each quantized activation, in real units.  LayerNorm
# outputs have unit spread times gamma (<= 2) plus beta; q/k/v and the attention
# output are sums of C products of N(0, 0.02^2) weights with such values; p is a
# probability; the GELU output is bounded below by -0.17.
DEFAULT_RANGES = {
    "a_qkv_in": (-4.0, 4.5),
    "a_q": (-1.0, 1.0),
    "a_k": (-1.125, 1.125),          # q, k and v each get a range of their own, so that an exchanged quantizer shows
    "a_v": (-0.875, 0.875),
    "a_p": (0.0, 0.3),
    "a_proj_in": (-0.4, 0.45),
    "a_fc1_in": (-4.5, 4.0),
    "a_fc2_in": (-0.17, 0.8),
}


def _rng(seed, stream):
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(stream)]))


def qparam_for_range(lo, hi, bits, symmetric=False):
    """(scale, zero_point) of a b-bit signed-container grid covering [lo, hi]."""
    qmin, qmax = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    if symmetric:
        m = max(abs(lo), abs(hi))
        return float(np.float32(m / qmax)), 0
    scale = np.float32((hi - lo) / (qmax - qmin))
    zp = int(np.clip(np.rint(qmin - lo / float(scale)), qmin, qmax))
    return float(scale), zp


def quantize_weights(w, bits):
    """Symmetric per-output-channel codes in an int8 container and fp32 scales."""
    qmax = (1 << (bits - 1)) - 1
    s = (np.abs(w).max(axis=1) / qmax).astype(np.float32)
    s = np.maximum(s, np.float32(1e-8))
    codes = np.clip(np.rint(w / s[:, None].astype(np.float64)), -qmax, qmax).astype(np.int8)
    return codes, s


def expand_rel_pos_bias(table, heads, window=WINDOW):
    """[heads,(2w-1)^2] table -> [heads, w*w, w*w] with Swin's relative index."""
    coords = np.stack(np.meshgrid(np.arange(window), np.arange(window), indexing="ij")).reshape(2, -1)
    rel = coords[:, :, None] - coords[:, None, :] + (window - 1)
    idx = rel[0] * (2 * window - 1) + rel[1]
    return np.ascontiguousarray(table[:, idx]).astype(np.float32)


def make_feature_map(spec, seed, blobs=False, outlier_channels=False):
    rng = _rng(seed, 1)
    x = rng.standard_normal((spec.B, spec.H, spec.W, spec.C)).astype(np.float32)
    if blobs:
        # elliptical high-magnitude regions until their union covers ~30 % of the map
        brng = _rng(seed, 2)
        rr, cc = np.meshgrid(np.arange(spec.H), np.arange(spec.W), indexing="ij")
        for b in range(spec.B):
            cover = np.zeros((spec.H, spec.W), dtype=bool)
            rejected = 0                     # on a map of a few pixels no further region may fit under the limit: give up then
            while cover.mean() < 0.30 and rejected < 200:
                cy, cx = brng.uniform(0, spec.H), brng.uniform(0, spec.W)
                ay = brng.uniform(0.04, 0.12) * spec.H + 2
                ax = brng.uniform(0.04, 0.12) * spec.W + 2
                m = ((rr - cy) / ay) ** 2 + ((cc - cx) / ax) ** 2 <= 1.0
                m &= ~cover
                if cover.mean() + m.mean() > 0.31:
                    rejected += 1
                    continue
                rejected = rejected + 1 if not m.any() else 0    # a region that adds no pixel is no progress either
                u = brng.standard_normal(spec.C).astype(np.float32)
                x[b][m] = np.float32(4.0) * x[b][m] + np.float32(3.0) * u
                cover |= m
    if outlier_channels:
        orng = _rng(seed, 3)
        n_out = max(1, int(round(0.03 * spec.C)))
        ch = orng.choice(spec.C, size=n_out, replace=False)
        fac = np.exp(orng.uniform(np.log(8.0), np.log(32.0), size=n_out)).astype(np.float32)
        x[..., ch] *= fac
    return np.ascontiguousarray(x)


def make_block_inputs(spec, seed, ranges=None, asymmetric=True, per_branch_bias=False, bias_std=0.02):
    """Weights, LayerNorm parameters, biases and quantizers of one block.

    per_branch_bias=False: both branches carry the same bias arrays (the QAT setting, shadow layers
    share weights and biases); True: the low branch gets biases of its own, drawn independently
    (the PTQ setting, where the biases are made independent per branch)."""
    rng = _rng(seed, 10)
    C, F = spec.C, spec.C * spec.mlp_ratio
    ranges = dict(DEFAULT_RANGES, **(ranges or {}))

    def lin(n_out, n_in):
        w = rng.standard_normal((n_out, n_in)) * 0.02
        return quantize_weights(w, spec.weight_bits)

    w_qkv, s_qkv = lin(3 * C, C)
    w_proj, s_proj = lin(C, C)
    w_fc1, s_fc1 = lin(F, C)
    w_fc2, s_fc2 = lin(C, F)
    table = rng.standard_normal((spec.heads, (2 * spec.window - 1) ** 2)) * 0.5
    rpb = expand_rel_pos_bias(table, spec.heads, spec.window)

    def ln_pair():
        g = np.clip(1.0 + 0.25 * rng.standard_normal(C), 0.25, 2.0).astype(np.float32)
        b = (0.1 * rng.standard_normal(C)).astype(np.float32)
        return g, b

    shared_bias = [(bias_std * rng.standard_normal(n)).astype(np.float32) for n in (3 * C, C, F, C)]
    brng = _rng(seed, 11)                               # a stream of its own: the other draws do not move
    own_bias = [(bias_std * brng.standard_normal(n)).astype(np.float32) for n in (3 * C, C, F, C)]
    branches = []
    for br, bits in enumerate((spec.act_bits_high, spec.act_bits_low)):
        g1, b1 = ln_pair()
        g2, b2 = ln_pair()
        q = {}
        for name in QNAMES:
            lo, hi = ranges[name]
            if br == 1:                                   # each branch calibrates its own step sizes (Sec. 3.2): the low
                lo, hi = lo * 0.9375, hi * 0.9375         # branch's ranges differ also where the bit widths are equal
            sym = name in ("a_q", "a_k", "a_v") or not asymmetric
            if name == "a_p":
                sym = False
            q[name] = qparam_for_range(lo, hi, bits, symmetric=sym)
        # shadow layers share weights and (unless per_branch_bias) biases across the branches
        branches.append(BranchParams(g1, b1, g2, b2, *(own_bias if per_branch_bias and br == 1 else shared_bias), q=q))
    srng = _rng(seed, 12)                               # the scoring LayerNorm (score mode 1) has parameters of its own
    score_gamma = np.clip(1.0 + 0.25 * srng.standard_normal(C), 0.25, 2.0).astype(np.float32)
    score_beta = (0.1 * srng.standard_normal(C)).astype(np.float32)
    shared = SharedParams(w_qkv, w_proj, w_fc1, w_fc2, s_qkv, s_proj, s_fc1, s_fc2, rpb,
                          score_gamma=score_gamma, score_beta=score_beta)
    return BlockInputs(spec, shared, branches)


@dataclass
class DownSpec:
    """Shape and precision of a layer between stages (the fields of the C descriptor):
    kind 0 = patch embedding (patch x patch x C_in values per token), kind 1 = patch merging."""
    kind: int
    B: int
    H: int
    W: int
    C_in: int
    N: int
    patch: int = 4
    act_bits: int = 8
    weight_bits: int = 8
    ln_eps: float = 1e-5

    @property
    def P(self):
        return self.patch if self.kind == 0 else 2

    @property
    def K(self):
        return self.P * self.P * self.C_in

    @property
    def Ho(self):
        return -(-self.H // self.P)

    @property
    def Wo(self):
        return -(-self.W // self.P)


@dataclass
class DownInputs:
    spec: DownSpec
    w: np.ndarray            # [N,K] int8 codes
    s_w: np.ndarray          # [N]
    bias: Optional[np.ndarray]
    ln_gamma: np.ndarray     # kind 0: [N]; kind 1: [K]
    ln_beta: np.ndarray
    a_in: tuple              # (scale, zero_point)


def make_image(B, H, W, seed, channels=3):
    """Smooth noise (N(0,1) box-filtered over 16 pixels, rescaled to unit spread) plus a few
    object-like elliptical blobs of raised magnitude; stands in for a detection-scale photograph."""
    rng = _rng(seed, 20)
    n = rng.standard_normal((B, H + 15, W + 15, channels))
    c = np.cumsum(np.cumsum(n, axis=1), axis=2)
    c = np.pad(c, ((0, 0), (1, 0), (1, 0), (0, 0)))
    box = c[:, 16:, 16:] - c[:, :-16, 16:] - c[:, 16:, :-16] + c[:, :-16, :-16]
    img = (box[:, :H, :W] / 16.0).astype(np.float32)
    rr, cc = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    for b in range(B):
        for _ in range(12):
            cy, cx = rng.uniform(0, H), rng.uniform(0, W)
            ay, ax = rng.uniform(0.03, 0.10) * H + 4, rng.uniform(0.03, 0.10) * W + 4
            m = ((rr - cy) / ay) ** 2 + ((cc - cx) / ax) ** 2 <= 1.0
            img[b][m] = np.float32(2.0) * img[b][m] + rng.standard_normal(channels).astype(np.float32)
    return np.ascontiguousarray(img)


def make_downsample_inputs(spec, seed, in_range=(-4.0, 4.5)):
    """Weights ~ N(0, 0.02^2) (patch embedding: N(0, 0.2^2), its inputs are few), LayerNorm parameters,
    bias (patch embedding only) and the input quantizer of a layer between stages."""
    rng = _rng(seed, 30)
    std = 0.2 if spec.kind == 0 else 0.02
    w, s_w = quantize_weights(rng.standard_normal((spec.N, spec.K)) * std, spec.weight_bits)
    n_ln = spec.N if spec.kind == 0 else spec.K
    g = np.clip(1.0 + 0.25 * rng.standard_normal(n_ln), 0.25, 2.0).astype(np.float32)
    b = (0.1 * rng.standard_normal(n_ln)).astype(np.float32)
    bias = (0.02 * rng.standard_normal(spec.N)).astype(np.float32) if spec.kind == 0 else None
    return DownInputs(spec, w, s_w, bias, g, b, qparam_for_range(in_range[0], in_range[1], spec.act_bits))


def backbone(name="cfg4"):
    """The whole backbone of a workload as a chain: patch embedding, then every stage, with a patch
    merging between stages.  Returns dict(image=(B,H,W), embed=DownSpec, stages=[...], merges=[DownSpec...])."""
    wl = workload(name)
    st = wl["stages"]
    s0 = st[0]["spec"]
    bits, wbits = s0.act_bits_high, s0.weight_bits
    embed = DownSpec(0, s0.B, s0.H * 4, s0.W * 4, 3, s0.C, patch=4, act_bits=bits, weight_bits=wbits)
    merges = [DownSpec(1, a["spec"].B, a["spec"].H, a["spec"].W, a["spec"].C, b["spec"].C, act_bits=bits, weight_bits=wbits)
              for a, b in zip(st[:-1], st[1:])]
    for m, nxt in zip(merges, st[1:]):
        assert (m.Ho, m.Wo, m.N) == (nxt["spec"].H, nxt["spec"].W, nxt["spec"].C)
    return dict(wl, image=(s0.B, s0.H * 4, s0.W * 4), embed=embed, merges=merges)


# The five benchmark workloads, as lists of stages; every stage is a run of
# blocks with alternating shift on one feature map.
def workload(name):
    """Returns dict(stages=[dict(spec=BlockSpec, blocks=n, keep=[...])], blobs=..., outliers=..., seed=...)."""
    if name == "cfg1":
        return dict(seed=1001, blobs=False, outliers=False, keep=[0.5],
                    stages=[dict(spec=BlockSpec(1, 56, 56, 96, 3), shifts=[0])])
    if name == "cfg2":
        return dict(seed=1002, blobs=True, outliers=False, keep=[0.5],
                    stages=[dict(spec=BlockSpec(1, 200, 336, 96, 3), shifts=[0, 3])])
    if name == "cfg3":
        return dict(seed=1003, blobs=False, outliers=False, keep=[0.25, 0.5, 0.75],
                    stages=[dict(spec=BlockSpec(2, 50, 84, 384, 12), shifts=[0, 3, 0, 3, 0, 3])])
    if name == "cfg4":
        mk = lambda H, W, C, h: BlockSpec(1, H, W, C, h, act_bits_high=4, act_bits_low=2, weight_bits=4)
        return dict(seed=1004, blobs=True, outliers=False, keep=[0.5],
                    stages=[dict(spec=mk(200, 336, 96, 3), shifts=[0, 3]),
                            dict(spec=mk(100, 168, 192, 6), shifts=[0, 3]),
                            dict(spec=mk(50, 84, 384, 12), shifts=[0, 3, 0, 3, 0, 3]),
                            dict(spec=mk(25, 42, 768, 24), shifts=[0, 3])])
    if name == "cfg5":
        return dict(seed=1005, blobs=False, outliers=True, keep=[0.4],
                    ranges={"a_qkv_in": (-12.0, 13.5), "a_fc1_in": (-11.0, 10.0)},
                    stages=[dict(spec=BlockSpec(4, 256, 256, 128, 4), shifts=[0, 3]),
                            dict(spec=BlockSpec(4, 128, 128, 256, 8), shifts=[0, 3])])
    raise KeyError(name)
