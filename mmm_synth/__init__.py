"""Seeded synthetic inputs for Masked Matrix Multiplication, C = M(X) x N(Y).

This module only *draws inputs*: dense X and Y, and the keep-bitmaps that
parameterise the mask functions M and N.  It contains none of the method's
arithmetic (no mask evaluation, no zero detection, no multiplication), so both
the CPU oracle and the HIP path can be fed from it without sharing code.

Workloads follow the paper's evaluation: seeded random matrices with a chosen
fraction of zeros in A and of zero vectors in B (section 4, "Random Matrices"),
and MLP-shaped activation x weight products with ReLU sparsity and contextual
row/block selection standing in for the Deja Vu matrices (section 4, "Matrices
from ML workloads"), which are not redistributable here.

Bitmap layout used everywhere in this repository: LSB-first little-endian
64-bit words, row-major, each row padded to a whole number of words with zero
bits: bit (c mod 64) of word (c div 64) of row r describes column c.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

PRED_NONZERO = 0  # keep iff x != 0
PRED_GT = 1       # keep iff x > threshold   (ReLU is threshold 0)
PRED_ABS_GT = 2   # keep iff |x| > threshold

DT_F32 = 0
DT_BF16 = 1
DT_F16 = 2
DT_F64 = 3        # X, Y (and C) in double: X and Y of the workload are float64 arrays


def pack_bits(flags: np.ndarray) -> np.ndarray:
    """Pack a 2-D boolean array into uint64 words, LSB-first, rows padded."""
    flags = np.ascontiguousarray(flags, dtype=bool)
    if flags.ndim == 1:
        flags = flags[None, :]
    rows, cols = flags.shape
    words = (cols + 63) // 64
    padded = np.zeros((rows, words * 64), dtype=bool)
    padded[:, :cols] = flags
    by = np.packbits(padded, axis=1, bitorder="little")
    return np.ascontiguousarray(by).view("<u8").reshape(rows, words)


def unpack_bits(words: np.ndarray, cols: int) -> np.ndarray:
    """Inverse of pack_bits: uint64 [rows, W] -> bool [rows, cols]."""
    words = np.ascontiguousarray(words, dtype="<u8")
    rows = words.shape[0]
    by = words.view(np.uint8).reshape(rows, -1)
    return np.unpackbits(by, axis=1, bitorder="little")[:, :cols].astype(bool)


def round_to_bf16(x: np.ndarray):
    """Round fp32 to bfloat16 (nearest-even).  Returns (bits uint16, value fp32).

    Input preparation only: the same bits go to the oracle (as the widened fp32
    value) and to the device (as the 16-bit pattern).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint32)
    # NaN stays NaN (inputs here are finite; kept for completeness)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = 0x7FC0
    bits = r.astype(np.uint16)
    val = (bits.astype(np.uint32) << 16).view(np.float32)
    return bits, val


def round_to_f16(x: np.ndarray):
    """Round fp32 to IEEE half (nearest-even).  Returns (bits uint16, value fp32).  Input preparation only."""
    h = np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)
    return h.view(np.uint16), h.astype(np.float32)


def _narrow(w):
    """Round the inputs of a workload to its 16-bit element type and keep the bit patterns."""
    if w.dtype == DT_BF16:
        w.X_bits, w.X = round_to_bf16(w.X)
        w.Y_bits, w.Y = round_to_bf16(w.Y)
    elif w.dtype == DT_F16:
        w.X_bits, w.X = round_to_f16(w.X)
        w.Y_bits, w.Y = round_to_f16(w.Y)
    return w


@dataclass
class Workload:
    """One MMM problem instance; everything the C ABI needs, as host arrays."""
    name: str
    M: int
    K: int
    N: int
    bw: int
    dtype: int                       # DT_F32, DT_BF16 or DT_F16
    X: np.ndarray                    # fp32 [M,K]  (representable in the 16-bit type if dtype is one)
    Y: np.ndarray                    # fp32 [K,N]
    pred: int = PRED_NONZERO
    threshold: float = 0.0
    keep_a: Optional[np.ndarray] = None       # uint64 [M, ceil(K/64)] or None
    keep_rows: Optional[np.ndarray] = None    # uint64 [ceil(K/64)] or None
    keep_blocks: Optional[np.ndarray] = None  # uint64 [K, ceil(NB/64)] or None
    X_bits: Optional[np.ndarray] = None       # uint16 [M,K] when dtype is 16-bit
    Y_bits: Optional[np.ndarray] = None       # uint16 [K,N] when dtype is 16-bit
    p_a: float = float("nan")
    p_b: float = float("nan")
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def NB(self) -> int:
        return self.N // self.bw


def _values(rng: np.random.Generator, shape, dist: str, a: float, b: float, f64: bool = False) -> np.ndarray:
    if f64:   # double-precision workloads draw doubles
        if dist == "uniform":
            return rng.uniform(a, b, size=shape)
        if dist == "normal":
            return rng.standard_normal(size=shape) * b + a
        if dist == "smallint":
            return rng.choice(np.array([-2.0, -1.0, 1.0, 2.0]), size=shape)
        raise ValueError(dist)
    if dist == "uniform":
        return rng.uniform(a, b, size=shape).astype(np.float32)
    if dist == "normal":
        out = rng.standard_normal(size=shape, dtype=np.float32)
        out *= np.float32(b)
        out += np.float32(a)
        return out
    if dist == "smallint":   # values in {-2,-1,1,2}: every product and partial sum is exact
        return rng.choice(np.array([-2.0, -1.0, 1.0, 2.0], dtype=np.float32), size=shape)
    raise ValueError(dist)


def random_masked(M: int, K: int, N: int, bw: int, p_a: float, p_b: float, seed: int,
                  dist: str = "uniform", lo: float = -1.0, hi: float = 1.0,
                  name: str = "random", dtype: int = DT_F32,
                  p_rows: Optional[float] = None) -> Workload:
    """Random element sparsity in A, block-random sparsity in B (Fig. 'Types of
    sparsity'; section 4 'Random Matrices').  Draw order: X, Y, A keep-uniforms,
    B row-keep uniforms (only if p_rows is given), B block-keep uniforms.
    keep = (u < p)."""
    assert N % bw == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    X = _values(rng, (M, K), dist, lo, hi, dtype == DT_F64)
    Y = _values(rng, (K, N), dist, lo, hi, dtype == DT_F64)
    ua = rng.random(size=(M, K), dtype=np.float32)
    keep_rows = None
    if p_rows is not None:
        ur = rng.random(size=(K,), dtype=np.float32)
        keep_rows = pack_bits(ur < np.float32(p_rows))[0]
    ub = rng.random(size=(K, N // bw), dtype=np.float32)
    w = Workload(name=name, M=M, K=K, N=N, bw=bw, dtype=dtype, X=X, Y=Y,
                 pred=PRED_NONZERO, threshold=0.0,
                 keep_a=pack_bits(ua < np.float32(p_a)),
                 keep_rows=keep_rows,
                 keep_blocks=pack_bits(ub < np.float32(p_b)),
                 p_a=p_a, p_b=p_b, seed=seed)
    return _narrow(w)


def relu_mlp(tokens: int, d_ff: int, d_model: int, bw: int, mu: float, p_rows: Optional[float],
             p_blocks: float, seed: int, name: str, dtype: int = DT_F32,
             w_std: float = 0.02) -> Workload:
    """MLP down-projection shape: A = ReLU(X) with X ~ N(mu,1) (no keep bitmap:
    the mask is the predicate x > 0), B = W2 ~ N(0, w_std) with contextual
    selection of whole rows (p_rows) and of 1 x bw blocks inside kept rows
    (p_blocks).  Draw order: X, Y, row-keep uniforms, block-keep uniforms."""
    assert d_model % bw == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    X = _values(rng, (tokens, d_ff), "normal", mu, 1.0)
    Y = _values(rng, (d_ff, d_model), "normal", 0.0, w_std)
    keep_rows = None
    if p_rows is not None:
        ur = rng.random(size=(d_ff,), dtype=np.float32)
        keep_rows = pack_bits(ur < np.float32(p_rows))[0]
    ub = rng.random(size=(d_ff, d_model // bw), dtype=np.float32)
    w = Workload(name=name, M=tokens, K=d_ff, N=d_model, bw=bw, dtype=dtype, X=X, Y=Y,
                 pred=PRED_GT, threshold=0.0, keep_a=None, keep_rows=keep_rows,
                 keep_blocks=pack_bits(ub < np.float32(p_blocks)),
                 p_a=float("nan"), p_b=(p_rows if p_rows is not None else 1.0) * p_blocks,
                 seed=seed, meta={"mu": mu})
    return _narrow(w)


def column_sparse(M: int, K: int, N: int, bw: int, p_cols: float, p_in: float, p_blocks: float, seed: int,
                  name: Optional[str] = None, dtype: int = DT_F32) -> Workload:
    """Column-structured A (the random-column form of the paper's Fig. "Matrix forms"): a set of columns of X, each
    chosen with probability p_cols, is switched on, the same set of rows of Y is switched on (the contextual selection
    of neurons of an MLP), elements inside a kept column survive with probability p_in, blocks inside a kept row of Y
    with probability p_blocks.  Draw order: X, Y, column uniforms, element uniforms, block uniforms."""
    assert N % bw == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    X = _values(rng, (M, K), "normal", 0.0, 1.0)
    Y = _values(rng, (K, N), "normal", 0.0, 1.0)
    cols = rng.random(size=(K,), dtype=np.float32) < np.float32(p_cols)
    ue = rng.random(size=(M, K), dtype=np.float32)
    ub = rng.random(size=(K, N // bw), dtype=np.float32)
    w = Workload(name=name or f"colsparse_{M}x{K}x{N}_c{int(round(p_cols * 100))}_bw{bw}", M=M, K=K, N=N, bw=bw,
                 dtype=dtype, X=X, Y=Y, pred=PRED_NONZERO, threshold=0.0,
                 keep_a=pack_bits((ue < np.float32(p_in)) & cols[None, :]), keep_rows=pack_bits(cols)[0],
                 keep_blocks=pack_bits(ub < np.float32(p_blocks)), p_a=p_cols * p_in, p_b=p_cols * p_blocks,
                 seed=seed, meta={"p_cols": p_cols})
    return _narrow(w)


SWEEP_P = (0.40, 0.30, 0.20, 0.10, 0.05)


def config(n: int, i_a: int = 3, i_b: Optional[int] = None, scale: int = 1) -> Workload:
    """The five benchmark workloads (1-based).  `scale` > 1 divides every matrix
    dimension (kept a multiple of what the block width needs) to give a small
    instance of the same recipe for CPU-side tests."""
    if i_b is None:
        i_b = i_a
    s = scale
    if n == 1:
        d = 256 // s
        return random_masked(d, d, d, 8, 0.2, 0.2, 1001, "uniform", -1.0, 1.0, name="cfg1_256_p20_bw8")
    if n == 2:
        d = 2048 // s
        return random_masked(d, d, d, 16, 0.1, 0.1, 1002, "normal", 0.0, 1.0, name="cfg2_2048_p10_bw16")
    if n == 3:
        d = 4096 // s
        pa, pb = SWEEP_P[i_a], SWEEP_P[i_b]
        return random_masked(d, d, d, 16, pa, pb, 3000 + 10 * i_a + i_b, "uniform", -1.0, 1.0,
                             name=f"cfg3_4096_pa{int(pa*100):02d}_pb{int(pb*100):02d}_bw16")
    if n == 4:
        return relu_mlp(2048 // s, 16384 // s, 4096 // s, 32, -1.3, 0.1, 0.5, 1004,
                        name="cfg4_mlp_2048x16384x4096_relu_bw32")
    if n == 5:
        return relu_mlp(max(32 // s, 1), 16384 // s, 4096 // s, 16, -1.65, None, 0.1, 1005,
                        name="cfg5_decode_32x16384x4096_bf16_bw16", dtype=DT_BF16)
    raise ValueError(f"no config {n}")
