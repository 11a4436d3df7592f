"""Seeded synthetic inputs for the quantized-linear hot path.

This module only draws random numbers and lays them out the way the layer's
inputs are defined; it holds none of the layer's arithmetic (no rotation, no
activation quantizer, no GEMM, no epilogue).  Both the CPU oracle's tests and
the GPU tests / benchmark take their inputs from here, so the two sides always
see identical bytes.

The five workloads are video-DiT linear-layer shapes: token counts come from
latent patch grids (21x30x52 and 33x45x80), channel widths from the attention
and FFN projections.  Values follow what the method section says about the
tensors it quantizes: Gaussian-like weights (Sec. 3.1) and activations with a
few massive outlier channels plus token-wise magnitude variation (Sec. 3.2).
They stand in for the real model's activations and weights, which are not
available offline.

Randomness is chunked so that any row range can be produced without drawing
the whole tensor: rows [c*CHUNK, (c+1)*CHUNK) of X come from
``default_rng([seed, TAG_X, c])`` and likewise for W.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "workload", "make_x_rows", "make_x", "make_weights",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "pack_w4", "sample_rows",
]

X_CHUNK = 1024   # token rows per independent random stream
W_CHUNK = 256    # weight rows per independent random stream
_TAG_X, _TAG_TOK, _TAG_OUT, _TAG_W, _TAG_CLIP = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    M: int            # tokens
    K: int            # input channels
    N: int            # output channels
    had_block: int    # Hadamard block size along K
    act_bits: int     # activation code width
    x_kind: str       # "gauss" | "postgelu"
    token_lognormal_sigma: float   # 0 -> no per-token scale
    outlier_frac: float
    outlier_gain: float
    w_sigma: float


WORKLOADS = (
    Workload("tiny_qlinear", 0, 128, 256, 256, 256, 4, "gauss", 0.0, 0.02, 30.0, 0.02),
    Workload("small_dit_qkv_w4a4", 1, 32760, 1536, 4608, 256, 4, "gauss", 0.5, 0.01, 50.0, 0.02),
    Workload("small_dit_ffn_up_w4a6", 2, 32760, 1536, 8960, 256, 6, "gauss", 0.5, 0.01, 50.0, 0.02),
    Workload("large_dit_proj_w4a4", 3, 118800, 3072, 3072, 256, 4, "gauss", 0.5, 0.01, 50.0, 0.02),
    Workload("large_dit_ffn_down_w4a4", 4, 32760, 13824, 5120, 512, 4, "postgelu", 0.0, 0.005, 80.0, 0.015),
)


def workload(i: int) -> Workload:
    return WORKLOADS[i]


# ---------------------------------------------------------------- bf16 casts
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- activations
def _outlier_channels(wl: Workload) -> np.ndarray:
    n = int(round(wl.outlier_frac * wl.K))
    rng = np.random.default_rng([wl.seed, _TAG_OUT])
    return np.sort(rng.choice(wl.K, size=n, replace=False))


def _token_scales(wl: Workload) -> np.ndarray | None:
    if wl.token_lognormal_sigma == 0.0:
        return None
    rng = np.random.default_rng([wl.seed, _TAG_TOK])
    return rng.lognormal(0.0, wl.token_lognormal_sigma, size=wl.M).astype(np.float32)


def _x_chunk(wl: Workload, c: int, tok: np.ndarray | None, out_ch: np.ndarray) -> np.ndarray:
    r0 = c * X_CHUNK
    rows = min(X_CHUNK, wl.M - r0)
    rng = np.random.default_rng([wl.seed, _TAG_X, c])
    x = rng.standard_normal((rows, wl.K), dtype=np.float32)
    if wl.x_kind == "postgelu":
        np.abs(x, out=x)
        x -= np.float32(0.2)
        np.maximum(x, np.float32(-0.17), out=x)
    if tok is not None:
        x *= tok[r0:r0 + rows, None]
    x[:, out_ch] *= np.float32(wl.outlier_gain)
    return f32_to_bf16_bits(x)


def make_x_rows(wl: Workload, rows: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of the requested token rows, shape [len(rows), K]."""
    rows = np.asarray(rows, dtype=np.int64)
    tok, out_ch = _token_scales(wl), _outlier_channels(wl)
    out = np.empty((rows.size, wl.K), dtype=np.uint16)
    chunk_of = rows // X_CHUNK
    for c in np.unique(chunk_of):
        blk = _x_chunk(wl, int(c), tok, out_ch)
        sel = np.nonzero(chunk_of == c)[0]
        out[sel] = blk[rows[sel] - int(c) * X_CHUNK]
    return out


def make_x(wl: Workload) -> np.ndarray:
    """All activations as bf16 bit patterns, shape [M, K], row-major."""
    tok, out_ch = _token_scales(wl), _outlier_channels(wl)
    out = np.empty((wl.M, wl.K), dtype=np.uint16)
    for c in range((wl.M + X_CHUNK - 1) // X_CHUNK):
        blk = _x_chunk(wl, c, tok, out_ch)
        out[c * X_CHUNK:c * X_CHUNK + blk.shape[0]] = blk
    return out


# ---------------------------------------------------------------- weights
def pack_w4(codes: np.ndarray) -> np.ndarray:
    """int8 codes [N, K] in [-8, 7] -> canonical packed bytes [N, K/2]:
    byte j of a row holds code[2j] in its low nibble and code[2j+1] in its
    high nibble, both as 4-bit two's complement."""
    c = np.ascontiguousarray(codes, dtype=np.int8).view(np.uint8)
    lo = c[:, 0::2] & np.uint8(0x0F)
    hi = (c[:, 1::2] & np.uint8(0x0F)) << np.uint8(4)
    return (lo | hi).astype(np.uint8)


def make_weights(wl: Workload):
    """Offline-quantized weights as the layer receives them.

    The drawn matrix is taken to be already expressed in the rotated basis (an
    i.i.d. Gaussian matrix keeps its distribution under an orthogonal change of
    basis).  Per output channel: scale = clip * max|w| / 7 with clip ~ U(0.8, 1),
    code = clamp(rint(w / scale), -7, 7).

    Returns (w_packed uint8 [N, K/2], w_scale float32 [N], w_codes int8 [N, K]).
    """
    clip = np.random.default_rng([wl.seed, _TAG_CLIP]).uniform(0.8, 1.0, size=wl.N)
    codes = np.empty((wl.N, wl.K), dtype=np.int8)
    scale = np.empty(wl.N, dtype=np.float32)
    for c in range((wl.N + W_CHUNK - 1) // W_CHUNK):
        r0 = c * W_CHUNK
        rows = min(W_CHUNK, wl.N - r0)
        rng = np.random.default_rng([wl.seed, _TAG_W, c])
        w = rng.standard_normal((rows, wl.K), dtype=np.float32).astype(np.float64) * wl.w_sigma
        s = (clip[r0:r0 + rows] * np.abs(w).max(axis=1) / 7.0).astype(np.float32)
        q = np.clip(np.rint(w / s.astype(np.float64)[:, None]), -7, 7)
        codes[r0:r0 + rows] = q.astype(np.int8)
        scale[r0:r0 + rows] = s
    return pack_w4(codes), scale, codes


def sample_rows(M: int, n_edge: int = 256) -> np.ndarray:
    """Deterministic token subset used when the oracle cannot afford all M rows:
    the first and the last ``n_edge`` rows (the last ones cover the ragged tail
    tile of the GPU launch)."""
    if M <= 2 * n_edge:
        return np.arange(M, dtype=np.int64)
    return np.concatenate([np.arange(n_edge), np.arange(M - n_edge, M)]).astype(np.int64)
