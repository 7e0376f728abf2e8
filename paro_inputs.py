"""Seeded synthetic inputs for the rotated-W4A16 linear hot path.

This module only DRAWS random tensors and lays them out in the interchange
formats of the C ABI.  It holds none of the method's arithmetic (no rotation,
no dequantisation, no contraction), so both the CPU oracle's tests and the GPU
tests can use it without sharing any code of the method itself.

Workloads stand in for the reasoning-LLM decoder layers the paper evaluates
(its Section 5 and Appendix A.5 use LLaMA-3-8B / Qwen3-class models, group size
128, K = 8 rotation layers of up to 64 pairs, Section 5 "Implementation").
Real weights and calibrated transforms are not available, so every tensor is
drawn from a documented distribution:

  X         fp16 of N(0,1) [T x C]; `n_outlier` channels (chosen without
            replacement) have their whole column multiplied by 50
  pairs     per group, per layer: an independent uniformly random perfect
            matching of the 128 local channels -> int16 [G][K][64][2]
  theta     fp32 uniform[-pi, pi)               [G][K][64]
  ch_scale  fp16 of exp(N(0, 0.3))              [C]
  codes     uniform integers 0..15              [N][C]  -> packed 8 per uint32
  scales    fp16 of uniform[0.005, 0.02]        [G][N]
  zeros     uniform integers 0..15              [G][N]  -> packed 8 per uint32

One numpy Generator(PCG64(seed)) per tensor, seed = 10000*config + 100*linear
+ tensor_id, so any tensor can be regenerated alone.  X for T tokens is a
prefix of X for more tokens (row-major fill from the same stream).
"""
from __future__ import annotations

import dataclasses
import numpy as np

GROUP = 128
N_LAYERS = 8
PAIRS_PER_LAYER = GROUP // 2

# tensor ids inside one linear's seed block
_TID_X, _TID_OUTLIER, _TID_PAIRS, _TID_THETA, _TID_CHSCALE, _TID_CODES, _TID_SCALES, _TID_ZEROS, _TID_BIAS = range(9)


@dataclasses.dataclass(frozen=True)
class LinearShape:
    name: str
    c_in: int
    c_out: int


@dataclasses.dataclass(frozen=True)
class Config:
    index: int
    name: str
    linears: tuple
    tokens: tuple          # token counts this config is run at
    n_outlier_fixed: int | None = None   # config 0 uses exactly 4 outlier channels

    def n_outlier(self, c_in: int) -> int:
        if self.n_outlier_fixed is not None:
            return self.n_outlier_fixed
        return int(round(0.005 * c_in))


_L8B = (
    LinearShape("qkv", 4096, 6144),
    LinearShape("o", 4096, 4096),
    LinearShape("gate_up", 4096, 28672),
    LinearShape("down", 14336, 4096),
)
_L32B = (
    LinearShape("qkv", 5120, 7168),
    LinearShape("o", 5120, 5120),
    LinearShape("gate_up", 5120, 55296),
    LinearShape("down", 27648, 5120),
)

CONFIGS = (
    Config(0, "tiny", (LinearShape("tiny", 512, 512),), (1,), n_outlier_fixed=4),
    Config(1, "8b_decode_b1", _L8B, (1,)),
    Config(2, "8b_decode_b16", _L8B, (16,)),
    Config(3, "8b_prefill_2048", _L8B, (2048,)),
    Config(4, "32b_layer", _L32B, (1, 4096)),
)


def _rng(config: int, linear: int, tid: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(10_000 * config + 100 * linear + tid))


def pack_nibbles_u32(codes: np.ndarray) -> np.ndarray:
    """Pack the last axis 8 codes per uint32, code k of a word in bits 4k..4k+3."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    assert codes.shape[-1] % 8 == 0
    c = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // 8, 8)).astype(np.uint32)
    out = np.zeros(c.shape[:-1], dtype=np.uint32)
    for k in range(8):
        out |= c[..., k] << np.uint32(4 * k)
    return out


def draw_matchings(rng: np.random.Generator, n_groups: int, n_layers: int, group: int = GROUP) -> np.ndarray:
    """Independent uniformly random perfect matchings: permute, pair consecutive."""
    pairs = np.empty((n_groups, n_layers, group // 2, 2), dtype=np.int16)
    for g in range(n_groups):
        for t in range(n_layers):
            pairs[g, t] = rng.permutation(group).astype(np.int16).reshape(group // 2, 2)
    return pairs


@dataclasses.dataclass
class LinearInputs:
    """All tensors of one linear, in the C ABI's interchange layouts (numpy, host)."""
    shape: LinearShape
    tokens: int
    x: np.ndarray          # fp16 [T][C]
    pairs: np.ndarray      # int16 [G][K][P][2]
    theta: np.ndarray      # fp32 [G][K][P]
    ch_scale: np.ndarray   # fp16 [C]
    codes: np.ndarray | None   # uint8 [N][C] (dropped for the big cases to save memory)
    qweight: np.ndarray    # uint32 [N][C/8]
    scales: np.ndarray     # fp16 [G][N]
    zeros: np.ndarray | None   # uint8 [G][N]
    qzeros: np.ndarray     # uint32 [G][N/8]
    outlier_channels: np.ndarray

    @property
    def c_in(self) -> int:
        return self.shape.c_in

    @property
    def c_out(self) -> int:
        return self.shape.c_out

    @property
    def n_groups(self) -> int:
        return self.shape.c_in // GROUP


def make_x(config: int, linear: int, tokens: int, c_in: int, n_outlier: int):
    rng = _rng(config, linear, _TID_X)
    x = rng.standard_normal((tokens, c_in), dtype=np.float32)
    out_ch = np.sort(_rng(config, linear, _TID_OUTLIER).choice(c_in, size=n_outlier, replace=False))
    x[:, out_ch] *= 50.0
    return x.astype(np.float16), out_ch


def make_rotation(config: int, linear: int, c_in: int, n_layers: int = N_LAYERS):
    g = c_in // GROUP
    pairs = draw_matchings(_rng(config, linear, _TID_PAIRS), g, n_layers)
    theta = _rng(config, linear, _TID_THETA).uniform(-np.pi, np.pi, size=(g, n_layers, PAIRS_PER_LAYER)).astype(np.float32)
    ch_scale = np.exp(_rng(config, linear, _TID_CHSCALE).normal(0.0, 0.3, size=c_in)).astype(np.float16)
    return pairs, theta, ch_scale


def make_weight(config: int, linear: int, c_in: int, c_out: int, keep_codes: bool = True):
    g = c_in // GROUP
    codes = _rng(config, linear, _TID_CODES).integers(0, 16, size=(c_out, c_in), dtype=np.uint8)
    qweight = pack_nibbles_u32(codes)
    scales = _rng(config, linear, _TID_SCALES).uniform(0.005, 0.02, size=(g, c_out)).astype(np.float16)
    zeros = _rng(config, linear, _TID_ZEROS).integers(0, 16, size=(g, c_out), dtype=np.uint8)
    qzeros = pack_nibbles_u32(zeros)
    if not keep_codes:
        codes = None
    return codes, qweight, scales, zeros, qzeros


def make_bias(config: int, linear: int, c_out: int) -> np.ndarray:
    return _rng(config, linear, _TID_BIAS).normal(0.0, 1.0, size=c_out).astype(np.float16)


def make_linear(config: int, linear: int, tokens: int | None = None, keep_codes: bool = True) -> LinearInputs:
    cfg = CONFIGS[config]
    shp = cfg.linears[linear]
    t = cfg.tokens[0] if tokens is None else tokens
    x, out_ch = make_x(config, linear, t, shp.c_in, cfg.n_outlier(shp.c_in))
    pairs, theta, ch_scale = make_rotation(config, linear, shp.c_in)
    codes, qweight, scales, zeros, qzeros = make_weight(config, linear, shp.c_in, shp.c_out, keep_codes)
    return LinearInputs(shp, t, x, pairs, theta, ch_scale, codes, qweight, scales, zeros, qzeros, out_ch)


def make_custom(seed: int, tokens: int, c_in: int, c_out: int, n_layers: int = N_LAYERS,
                pairs_per_layer: int = PAIRS_PER_LAYER, n_outlier: int = 0) -> LinearInputs:
    """Off-config shapes for edge-case tests (ragged tails, partial matchings).

    With pairs_per_layer < 64 the remaining channels of each layer stay unpaired;
    the last unused slot of every layer is additionally filled with an explicit
    (i, i) no-op sentinel when there is room, so both spellings are exercised.
    """
    assert c_in % GROUP == 0 and c_out % 8 == 0
    g = c_in // GROUP
    rs = np.random.Generator(np.random.PCG64(seed))
    x = rs.standard_normal((tokens, c_in), dtype=np.float32)
    out_ch = np.sort(rs.choice(c_in, size=n_outlier, replace=False)) if n_outlier else np.zeros(0, dtype=np.int64)
    x[:, out_ch] *= 50.0
    full = draw_matchings(rs, g, n_layers)
    pairs = np.ascontiguousarray(full[:, :, :pairs_per_layer, :])
    if 0 < pairs_per_layer < PAIRS_PER_LAYER:
        # turn the last kept slot into an (i, i) sentinel on odd layers
        pairs[:, 1::2, -1, 1] = pairs[:, 1::2, -1, 0]
    theta = rs.uniform(-np.pi, np.pi, size=(g, n_layers, pairs_per_layer)).astype(np.float32)
    ch_scale = np.exp(rs.normal(0.0, 0.3, size=c_in)).astype(np.float16)
    codes = rs.integers(0, 16, size=(c_out, c_in), dtype=np.uint8)
    scales = rs.uniform(0.005, 0.02, size=(g, c_out)).astype(np.float16)
    zeros = rs.integers(0, 16, size=(g, c_out), dtype=np.uint8)
    return LinearInputs(LinearShape(f"custom{seed}", c_in, c_out), tokens, x.astype(np.float16), pairs, theta,
                        ch_scale, codes, pack_nibbles_u32(codes), scales, zeros, pack_nibbles_u32(zeros), out_ch)


def make_dense_weight(seed: int, c_out: int, c_in: int, sigma: float = 0.02, outlier_frac: float = 0.005,
                      outlier_mult: float = 20.0) -> np.ndarray:
    """Dense fp16 weight [c_out][c_in] for the weight-side quantiser: N(0, sigma) with a fraction of
    isolated elements multiplied by ``outlier_mult`` (stands in for the outlier-heavy pre-trained
    weights the method targets; real checkpoints are not available)."""
    rs = np.random.Generator(np.random.PCG64(seed))
    w = rs.standard_normal((c_out, c_in), dtype=np.float32) * np.float32(sigma)
    n_out = int(round(outlier_frac * w.size))
    if n_out:
        idx = rs.choice(w.size, size=n_out, replace=False)
        w.reshape(-1)[idx] *= np.float32(outlier_mult)
    return w.astype(np.float16)


def make_pair_order(seed: int, group: int = GROUP) -> np.ndarray:
    """The shuffle that Algorithm A1 draws: a seeded permutation of the g(g-1)/2 pair numbers."""
    rs = np.random.Generator(np.random.PCG64(seed))
    return rs.permutation(group * (group - 1) // 2).astype(np.int32)
