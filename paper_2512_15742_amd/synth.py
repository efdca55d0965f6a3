"""Seeded synthetic inputs for the VQ-KAN forward pass.

This module only draws random parameters and inputs with the shapes, dtypes
and distributions of the benchmark configurations; it contains none of the
method's arithmetic (no spline evaluation, no reconstruction, no summation),
so both the CPU oracle's tests and the GPU tests may use it.  numpy only.

Stand-in note: the paper evaluates on detection heads fed by backbone features
of real images.  Those datasets and weights are not available; the cost of the
forward pass depends only on shapes, dtypes and the index distribution, so
seeded synthetic tensors of the stated shapes stand in for them.  Uniform
random indices are the worst case for gather locality.

Draw order per layer (fixed): codebook, idx, gain, bias.  Inputs x are drawn
from their own generator.  "N(0, s)" means standard deviation s.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

G = 10


@dataclass
class VQLayerParams:
    n_in: int
    n_out: int
    K: int
    codebook: np.ndarray      # [K][10] float32, float16 or int8
    scale: np.float32         # Int8: value = scale * q; 1.0 for float codebooks
    idx: np.ndarray           # [in][out] uint16 or uint32
    gain: np.ndarray          # [in][out] float32 or float16, or uint8 codes (byte-coded format)
    bias: np.ndarray          # [in][out] float32 or float16, or int8 codes
    gb_params: tuple = None   # byte-coded format only: (gain_log2_lo, gain_log2_step, bias_scale) as float32

    def as_dict(self):
        d = {"codebook": self.codebook, "scale": self.scale, "idx": self.idx,
             "gain": self.gain, "bias": self.bias}
        if self.gb_params is not None:
            d["gb_params"] = self.gb_params
        return d

    @property
    def metadata_bytes(self) -> int:
        return self.idx.nbytes + self.gain.nbytes + self.bias.nbytes

    @property
    def edges(self) -> int:
        return self.n_in * self.n_out


def make_shapes(rng: np.random.Generator, K: int) -> np.ndarray:
    """K rows of N(0,1)^10, made zero-mean and unit-L2-norm, as float32."""
    s = rng.standard_normal((K, G))
    s -= s.mean(axis=1, keepdims=True)
    s /= np.linalg.norm(s, axis=1, keepdims=True)
    return s.astype(np.float32)


def quantise_shapes(shapes: np.ndarray):
    """Int8 codebook with one scale per layer: scale = max|shape| / 127,
    q = clip(rint(shape / scale), -127, 127)."""
    scale = np.float32(np.abs(shapes).max() / 127.0)
    q = np.clip(np.rint(shapes.astype(np.float64) / np.float64(scale)), -127, 127).astype(np.int8)
    return q, scale


def quantise_shapes_bfp8(shapes: np.ndarray) -> np.ndarray:
    """Block-floating-point codebook, one block per row: int8 [K][12] = ten mantissas, the row's
    exponent, a zero byte.  Encoder only: exponent e = the smallest integer with
    max|row| <= 127 * 2**e (clamped to -126..127; an all-zero row gets -126),
    mantissas rint(row / 2**e) in -127..127."""
    s = shapes.astype(np.float64)
    m = np.abs(s).max(axis=1)
    e = np.where(m > 0, np.ceil(np.log2(np.maximum(m, 1e-300) / 127.0)), -126.0)
    e = np.clip(e, -126, 127)
    q = np.clip(np.rint(s / np.exp2(e)[:, None]), -127, 127)
    out = np.zeros((s.shape[0], G + 2), dtype=np.int8)
    out[:, :G] = q.astype(np.int8)
    out[:, G] = e.astype(np.int8)
    return out


def encode_gain_bias_q8(gain: np.ndarray, bias: np.ndarray):
    """One byte each (the 16 bits per edge of the fully quantised format): gains on a
    logarithmic grid, biases on a linear one.  Encoder only - what the codes MEAN is the
    method's business (oracle and kernels each state it):
        gain code 0 for a zero gain, else rint((log2 g - lo) / step) in 1..255, where
        step = (log2 of the largest gain - log2 of the smallest positive one) / 254 and
        lo = log2 of the smallest positive gain - step (so that it gets code 1);
        bias code rint(b / bias_scale) in -127..127, bias_scale = max|b| / 127.
    Returns (gain codes uint8, bias codes int8, (lo, step, bias_scale) as float32)."""
    g = gain.astype(np.float64)
    pos = g > 0
    lg = np.log2(g[pos]) if pos.any() else np.array([0.0])
    step = np.float32(max((lg.max() - lg.min()) / 254.0, 1e-6))
    lo = np.float32(lg.min() - float(step))
    qg = np.zeros(g.shape, dtype=np.uint8)
    qg[pos] = np.clip(np.rint((np.log2(g[pos]) - float(lo)) / float(step)), 1, 255).astype(np.uint8)
    b = bias.astype(np.float64)
    bscale = np.float32(max(np.abs(b).max() / 127.0, 1e-30))
    qb = np.clip(np.rint(b / float(bscale)), -127, 127).astype(np.int8)
    return qg, qb, (lo, step, bscale)


def draw_idx(rng: np.random.Generator, K: int, shape, dist: str = "uniform", zipf_s: float = 1.0) -> np.ndarray:
    """Codeword of every edge, int64.  'uniform': every codeword equally likely (the worst case
    for gather locality; the draw the configurations name).  'zipf': a trained-like skewed
    histogram, P(rank r) ~ 1 / r**zipf_s, the ranks scattered over the codebook by a random
    permutation.  'zipf-sorted': the same histogram with the popular codewords at the low ids
    (what a compiler that orders the codebook by use would emit)."""
    if dist == "uniform":
        return rng.integers(0, K, size=shape, dtype=np.int64)
    if dist not in ("zipf", "zipf-sorted"):
        raise ValueError(dist)
    p = 1.0 / np.arange(1, K + 1, dtype=np.float64) ** zipf_s
    p /= p.sum()
    ranks = rng.choice(K, size=shape, p=p)
    if dist == "zipf-sorted":
        return ranks.astype(np.int64)
    return rng.permutation(K)[ranks].astype(np.int64)


def make_layer(seed: int, n_in: int, n_out: int, K: int, *, cb_dtype="f32",
               gb_dtype="f32", idx_dtype=None, idx_dist="uniform", zipf_s=1.0) -> VQLayerParams:
    rng = np.random.default_rng(seed)
    shapes = make_shapes(rng, K)
    if cb_dtype == "i8":
        codebook, scale = quantise_shapes(shapes)
    elif cb_dtype == "f32":
        codebook, scale = shapes, np.float32(1.0)
    elif cb_dtype == "f16":
        codebook, scale = shapes.astype(np.float16), np.float32(1.0)
    elif cb_dtype == "bfp8":
        codebook, scale = quantise_shapes_bfp8(shapes), np.float32(1.0)
    else:
        raise ValueError(cb_dtype)
    if idx_dtype is None:
        idx_dtype = "u16" if K <= 65536 else "u32"
    np_idx = {"u16": np.uint16, "u32": np.uint32}[idx_dtype]
    if idx_dtype == "u16" and K > 65536:
        raise ValueError("K does not fit a 16-bit index")
    idx = draw_idx(rng, K, (n_in, n_out), idx_dist, zipf_s).astype(np_idx)
    np_gb = {"f32": np.float32, "f16": np.float16, "q8": np.float64}[gb_dtype]
    gain = np.abs(rng.normal(0.0, 0.1, size=(n_in, n_out))).astype(np_gb)
    bias = rng.normal(0.0, 0.01, size=(n_in, n_out)).astype(np_gb)
    if gb_dtype == "q8":
        qg, qb, params = encode_gain_bias_q8(gain, bias)
        return VQLayerParams(n_in, n_out, K, codebook, scale, idx, qg, qb, params)
    return VQLayerParams(n_in, n_out, K, codebook, scale, idx, gain, bias)


def make_x(seed: int, B: int, n_in: int, dist: str = "uniform") -> np.ndarray:
    """Inputs [B][in] float32: 'uniform' = U[-1,1]; 'normal' = clamp(N(0,0.4),-1,1)."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=(B, n_in))
    elif dist == "normal":
        x = np.clip(rng.normal(0.0, 0.4, size=(B, n_in)), -1.0, 1.0)
    else:
        raise ValueError(dist)
    return x.astype(np.float32)


def make_dense_grids(seed: int, n_in: int, n_out: int, K: int, noise: float = 0.05):
    """A dense layer to compress, with the codebook to compress it against:
    coef[i][j] = g * shape[k] + b + noise * g * N(0,1)^10 with the draws of make_layer
    (shapes zero-mean unit-norm, k uniform, g ~ |N(0,0.1)|, b ~ N(0,0.01)); returns
    (coef float32 [in][out][10], codebook float32 [K][10], k int64 [in][out])."""
    rng = np.random.default_rng(seed)
    shapes = make_shapes(rng, K)
    k = rng.integers(0, K, size=(n_in, n_out), dtype=np.int64)
    g = np.abs(rng.normal(0.0, 0.1, size=(n_in, n_out))) + 1e-3
    b = rng.normal(0.0, 0.01, size=(n_in, n_out))
    coef = g[..., None] * (shapes[k].astype(np.float64) + noise * rng.standard_normal((n_in, n_out, G))) + b[..., None]
    return coef.astype(np.float32), shapes, k


# ---- the five benchmark configurations ------------------------------------
# Seeds: configuration n, layer l -> 1000*n + l; x -> 1000*n + 900 + variant.
# Configuration 4: head h uses seed h for its first layer and h + 100 for its
# second.

def config1():
    """Single fp32 layer 64 -> 32, K = 256, batch 16."""
    return [make_layer(1000, 64, 32, 256)], make_x(1900, 16, 64, "uniform")


def config2(B: int):
    """Backbone-feature head layer 2048 -> 512, fp32 codebook K = 65,536."""
    return [make_layer(2000, 2048, 512, 65536)], make_x(2900 + B, B, 2048, "normal")


def config3_layers(gb_dtype: str = "f16", cb_dtype: str = "i8", idx_dist: str = "uniform"):
    """Two-layer Int8 head 2048 -> 1024 -> 256, fp16 gain/bias, K = 65,536 each.
    gb_dtype="q8": the same draws with gain and bias encoded in one byte each (the
    4-bytes-per-edge format of the paper, section 4.2).  cb_dtype and idx_dist vary the
    codebook precision and the assignment histogram on the same shapes (studies, not the
    configuration itself)."""
    return [make_layer(3000, 2048, 1024, 65536, cb_dtype=cb_dtype, gb_dtype=gb_dtype, idx_dist=idx_dist),
            make_layer(3001, 1024, 256, 65536, cb_dtype=cb_dtype, gb_dtype=gb_dtype, idx_dist=idx_dist)]


def config3(B: int):
    return config3_layers(), make_x(3900 + B, B, 2048, "uniform")


def config4_head(h: int):
    """Task head h of the multi-expert deployment: 2048 -> 256 -> 21, Int8."""
    return [make_layer(h, 2048, 256, 65536, cb_dtype="i8", gb_dtype="f16"),
            make_layer(h + 100, 256, 21, 65536, cb_dtype="i8", gb_dtype="f16")]


def config4(n_heads: int = 50, B: int = 64):
    return [config4_head(h) for h in range(n_heads)], make_x(4900, B, 2048, "uniform")


def config5(variant: str = "i8", B: int = 8192, n_in: int = 4096, n_out: int = 4096):
    """Large layer, K = 262,144, uint32 indices; 'i8' (fp16 gain/bias) or 'f32'."""
    if variant == "i8":
        L = make_layer(5000, n_in, n_out, 262144, cb_dtype="i8", gb_dtype="f16", idx_dtype="u32")
    else:
        L = make_layer(5001, n_in, n_out, 262144, cb_dtype="f32", gb_dtype="f32", idx_dtype="u32")
    return [L], make_x(5900, B, n_in, "uniform")
