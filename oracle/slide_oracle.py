"""CPU oracle for the SlideSparse (2N-2):2N structured-sparse linear layer.

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, obviously-correct
statement of what the GPU library must compute.  It shares no code with the HIP
path and is imported only by tests, the smoke check and the benchmark's
cpu_baseline leg.  Nothing in the product package may import it.

Notation (fixed for the whole repository; the paper reuses letters):
    M   tokens                      K   input features
    O   output features             N   pattern parameter, pattern is (2N-2):2N
    nw = N-1 windows per 2N block   K' = ceil(K/2N) * 4(N-1)  lifted width (= K * 2(N-1)/N when 2N | K)
    X[M,K], W[O,K], Y[M,O] all row-major;  Y = X . W^T

Every function cites the passage of the paper that defines it.  Floating-point
steps that decide an integer code (quantisation) are taken in fp32, the
precision the kernels use; exact sums are taken in int64 / fp64.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
invariants, closed forms, the paper's worked 6:8 example, brute force over all
block masks and library routines.  Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# Cost model (Sec. 3.4 "Cost Analysis", expansion-factor equation; App. C.1.5 table)
# ----------------------------------------------------------------------------

def n_windows(N: int) -> int:
    """Windows per 2N block: stride-2 size-4 windows, N-1 of them (Theorem 1)."""
    _check_N(N)
    return N - 1


def gamma(N: int) -> float:
    """Expansion factor gamma = 4(N-1)/(2N) = 2 - 2/N (Sec. 3.4)."""
    _check_N(N)
    return 4.0 * (N - 1) / (2.0 * N)


def s_eff(N: int, alpha: float = 2.0) -> float:
    """Speedup bound alpha/gamma = N/(N-1) for alpha = 2 (Corollary 1.2)."""
    return alpha / gamma(N)


def n_groups(K: int, N: int) -> int:
    """n_g = ceil(K / 2N): the last block is completed with zeros when 2N does not
    divide K (Alg. 1, the line that sets n_g and n_w)."""
    _check_N(N)
    if K <= 0:
        raise ValueError(f"K={K} is not positive")
    return -(-K // (2 * N))


def lifted_k(K: int, N: int) -> int:
    """K' = 4 n_w = n_g * 4(N-1) (Alg. 1: Y has 4 n_w columns)."""
    return n_groups(K, N) * 4 * (N - 1)


def pad_blocks(A: np.ndarray, N: int) -> np.ndarray:
    """A[R, K] -> A[R, n_g * 2N] with zero columns appended: the zero-completed last
    block that Alg. 1's n_g = ceil(K/2N) implies.  Zero of every storage type here
    is the all-zero bit pattern."""
    A = np.asarray(A)
    R, K = A.shape
    Kb = n_groups(K, N) * 2 * N
    if Kb == K:
        return A
    out = np.zeros((R, Kb), dtype=A.dtype)
    out[:, :K] = A
    return out


def _check_N(N: int) -> None:
    if not (isinstance(N, (int, np.integer)) and 2 <= N <= 8):
        raise ValueError(f"pattern parameter N={N} outside 2..8")


# ----------------------------------------------------------------------------
# Storage formats: bf16 and OCP fp8 e4m3 (the paper's "FP8 (E4M3)", App. D.1)
# ----------------------------------------------------------------------------

def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even.  NaN not in contract."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = u + 0x7FFF + lsb
    return (u >> 16).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> fp32, exact."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def fp16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE binary16 bit pattern (uint16), round-to-nearest-even (numpy's conversion);
    values beyond +-65504 are not in contract."""
    return np.asarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def fp16_to_f32(b: np.ndarray) -> np.ndarray:
    """binary16 bit pattern (uint16) -> fp32, exact."""
    return np.asarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def fp8_e4m3_decode(code: np.ndarray) -> np.ndarray:
    """OCP e4m3fn byte -> fp64 value.  1 sign, 4 exponent (bias 7), 3 mantissa bits;
    no infinities; exponent 15 with mantissa 7 is NaN; largest finite value 448."""
    c = np.asarray(code, dtype=np.uint8).astype(np.int64)
    sign = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    sub = m.astype(np.float64) * 2.0 ** (-9)               # e == 0: m/8 * 2^-6
    nor = (1.0 + m.astype(np.float64) / 8.0) * np.exp2((e - 7).astype(np.float64))
    v = np.where(e == 0, sub, nor)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return sign * v


def fp8_e4m3_encode(x: np.ndarray) -> np.ndarray:
    """fp32 -> OCP e4m3fn byte, round-to-nearest-even, saturating at +-448.

    Written as a search over the 127 non-negative finite codes' values so that it
    does not share bit tricks with any other encoder: the nearest representable
    magnitude is chosen, ties go to the code with even mantissa (= even code)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    mag = np.abs(x.astype(np.float64))
    codes = np.arange(0, 127, dtype=np.uint8)               # 0x00 .. 0x7E  (0x7F is NaN)
    vals = fp8_e4m3_decode(codes)                          # strictly increasing
    mag = np.minimum(mag, vals[-1])
    hi = np.searchsorted(vals, mag, side="left")            # first code with value >= mag
    hi = np.clip(hi, 0, 126)
    lo = np.clip(hi - 1, 0, 126)                            # last code with value < mag
    d_hi = vals[hi] - mag                                   # >= 0
    d_lo = mag - vals[lo]                                   # >= 0
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & ((lo & 1) == 0))
    out = np.where(pick_lo, lo, hi).astype(np.uint8)
    neg = np.signbit(x)
    return (out | np.where(neg, np.uint8(0x80), np.uint8(0))).astype(np.uint8)


QMAX = {"i8": 127.0, "fp8": 448.0}
DTYPES = ("i8", "fp8", "bf16", "fp16")
UNSCALED = ("bf16", "fp16")          # 16-bit operands carry no scales (App. D.1 lists BF16 and FP16 side by side)


def to_real(q: np.ndarray, dtype: str) -> np.ndarray:
    """Stored operand (int8 / fp8 byte / bf16 bits) -> its exact value in fp64."""
    if dtype == "i8":
        return np.asarray(q, dtype=np.int8).astype(np.float64)
    if dtype == "fp8":
        return fp8_e4m3_decode(q)
    if dtype == "bf16":
        return bf16_to_f32(q).astype(np.float64)
    if dtype == "fp16":
        return fp16_to_f32(q).astype(np.float64)
    raise ValueError(dtype)


def is_zero(q: np.ndarray, dtype: str) -> np.ndarray:
    """Zero test on the storage type handed to the packer (Alg. 2's 'w != 0');
    for fp8 and bf16 both +0 and -0 count as zero."""
    if dtype == "i8":
        return np.asarray(q) == 0
    if dtype == "fp8":
        return (np.asarray(q, dtype=np.uint8) & 0x7F) == 0
    if dtype in UNSCALED:
        return (np.asarray(q, dtype=np.uint16) & 0x7FFF) == 0
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# (2N-2):2N magnitude pruning  (Sec. 3.1 constraint C_Alg; App. E "magnitude pruning")
# ----------------------------------------------------------------------------

def prune_2n(W: np.ndarray, N: int) -> np.ndarray:
    """Keep the 2N-2 largest-|w| entries of every aligned run of 2N along K, zero
    the other two.  Ties in |w|: the lower index is kept.  A last run shorter than
    2N is completed with zeros first (they are the first to be dropped) and cut
    back afterwards."""
    _check_N(N)
    W = np.asarray(W)
    O, K = W.shape
    Wb = pad_blocks(W, N)
    blk = Wb.reshape(O, Wb.shape[1] // (2 * N), 2 * N)
    order = np.argsort(-np.abs(blk), axis=-1, kind="stable")   # descending |w|, stable
    drop = order[..., 2 * N - 2:]                              # the two smallest
    out = blk.copy()
    np.put_along_axis(out, drop, 0, axis=-1)
    return out.reshape(O, -1)[:, :K]


# ----------------------------------------------------------------------------
# Per-row dynamic symmetric quantisation  (Alg. 1, pass 1 and the Clamp line)
# ----------------------------------------------------------------------------

def row_scales(V: np.ndarray, dtype: str):
    """a = max_k |v|, r = Qmax / a, s = a / Qmax, all in fp32 (Alg. 1 pass 1).
    An all-zero row takes r = 0 and s = 1 (the paper is silent; q is then 0)."""
    V = np.asarray(V, dtype=np.float32)
    qmax = np.float32(QMAX[dtype])
    a = np.max(np.abs(V), axis=1).astype(np.float32)
    safe = np.where(a > 0, a, np.float32(1.0)).astype(np.float32)
    r = np.where(a > 0, qmax / safe, np.float32(0.0)).astype(np.float32)
    s = np.where(a > 0, safe / qmax, np.float32(1.0)).astype(np.float32)
    return r, s


def quantize_rows(V: np.ndarray, dtype: str):
    """q = Clamp(round(v * r), -Qmax, Qmax) per row (Alg. 1).  Rounding is to
    nearest-even on the single fp32 product v*r.  Returns (q, s):
       i8   -> int8 array, fp32 scales
       fp8  -> uint8 e4m3 codes, fp32 scales
       bf16 -> uint16 bf16 bits of v itself, scales None (no scaling in bf16)."""
    V = np.asarray(V, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits(V), None
    if dtype == "fp16":
        return fp16_bits(V), None
    r, s = row_scales(V, dtype)
    prod = (V * r[:, None]).astype(np.float32)                 # one rounded fp32 multiply
    qmax = np.float32(QMAX[dtype])
    if dtype == "i8":
        q = np.clip(np.rint(prod), -qmax, qmax).astype(np.int8)
    elif dtype == "fp8":
        q = fp8_e4m3_encode(np.clip(prod, -qmax, qmax))
    else:
        raise ValueError(dtype)
    return q, s


# ----------------------------------------------------------------------------
# Sliding Window Decomposition Phi  (Alg. 2 "Greedy Residual Allocation")
# ----------------------------------------------------------------------------

def slide_decompose(Wq: np.ndarray, N: int, dtype: str = "i8") -> np.ndarray:
    """Alg. 2 applied to every row: returns the dense slided matrix W'[O, K'].

    Window (g, l) of a row reads source positions b = 2N g + 2 l + delta,
    delta = 0..3, takes the first (lowest delta) at most two non-zeros not yet
    used by an earlier window, and writes each at offset delta of output window
    (N-1) g + l.  Vectorised over rows and groups g only; the l and delta loops
    and the `used` array are the algorithm's own.
    A block holding more than 2N-2 non-zeros violates the precondition: raise."""
    _check_N(N)
    Wq = np.asarray(Wq)
    O, K = Wq.shape
    Kp = lifted_k(K, N)
    ng = n_groups(K, N)
    blk = pad_blocks(Wq, N).reshape(O, ng, 2 * N)       # last block zero-completed
    nz = ~is_zero(blk, dtype)
    if np.any(nz.sum(axis=-1) > 2 * N - 2):
        raise ValueError("a 2N block holds more than 2N-2 non-zeros")
    used = np.zeros_like(nz)
    out = np.zeros((O, ng, N - 1, 4), dtype=Wq.dtype)
    for l in range(N - 1):
        cnt = np.zeros((O, ng), dtype=np.int64)
        for delta in range(4):
            p = 2 * l + delta
            take = nz[..., p] & ~used[..., p] & (cnt < 2)
            out[..., l, delta] = np.where(take, blk[..., p], 0)
            used[..., p] |= take
            cnt += take
    assert np.array_equal(used, nz), "greedy left a non-zero unassigned"
    return out.reshape(O, Kp)


def compress_24(Wp: np.ndarray, dtype: str = "i8"):
    """Canonical 2:4 compression of a slided matrix (Sec. 4.3: non-zeros plus
    compact metadata).  For every window of 4: two stored values and their two
    2-bit offsets i0 < i1, one byte per window = i0 | i1 << 2.  A window with
    fewer than two non-zeros pads with value 0 at the lowest offsets not holding
    a non-zero.  Returns (vals[O, K'/2], idx[O, K'/4] uint8)."""
    Wp = np.asarray(Wp)
    O, Kp = Wp.shape
    win = Wp.reshape(O, Kp // 4, 4)
    nz = ~is_zero(win, dtype)
    if np.any(nz.sum(axis=-1) > 2):
        raise ValueError("window with more than 2 non-zeros")
    # rank offsets: non-zeros first is wrong (order must be ascending offset); choose the
    # set = nz offsets plus lowest free offsets until two are chosen, then sort ascending.
    chosen = nz.copy()
    need = 2 - nz.sum(axis=-1)
    for delta in range(4):
        add = (~chosen[..., delta]) & (need > 0)
        chosen[..., delta] |= add
        need = need - add
    assert np.all(chosen.sum(axis=-1) == 2)
    offs = np.argsort(~chosen, axis=-1, kind="stable")[..., :2]   # ascending chosen offsets
    i0, i1 = offs[..., 0], offs[..., 1]
    vals = np.take_along_axis(win, offs, axis=-1)
    vals = np.where(np.take_along_axis(nz, offs, axis=-1), vals, 0).astype(Wp.dtype)
    idx = (i0 | (i1 << 2)).astype(np.uint8)
    return vals.reshape(O, Kp // 2), idx


def decompress_24(vals: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Inverse of compress_24: scatter the two stored values of each window to
    their offsets; everything else is zero."""
    O, half = vals.shape
    nwin = half // 2
    v = vals.reshape(O, nwin, 2)
    out = np.zeros((O, nwin, 4), dtype=vals.dtype)
    i0 = (idx & 3).astype(np.int64)
    i1 = ((idx >> 2) & 3).astype(np.int64)
    np.put_along_axis(out, i0[..., None], v[..., 0:1], axis=-1)
    # i1 != i0 in every valid encoding; write second after first
    np.put_along_axis(out, i1[..., None], v[..., 1:2], axis=-1)
    return out.reshape(O, nwin * 4)


# ----------------------------------------------------------------------------
# Activation lifting Psi  (Sec. 3.3 lifting operator; Alg. 1 pass 2 index formula)
# ----------------------------------------------------------------------------

def lift(Xq: np.ndarray, N: int) -> np.ndarray:
    """X'[i, 4 j + t] = X[i, 2N g + 2 l + t],  j = g (N-1) + l,  t = 0..3; source
    columns at or beyond K (last block when 2N does not divide K) read as zero."""
    _check_N(N)
    Xq = np.asarray(Xq)
    M, K = Xq.shape
    Kp = lifted_k(K, N)
    Xq = pad_blocks(Xq, N)
    out = np.empty((M, Kp), dtype=Xq.dtype)
    for j in range(Kp // 4):
        g, l = divmod(j, N - 1)
        b = 2 * N * g + 2 * l
        out[:, 4 * j:4 * j + 4] = Xq[:, b:b + 4]
    return out


def act_lift_quant(X: np.ndarray, N: int, dtype: str):
    """Alg. 1, fused quantisation + slide: per-row scale (pass 1), then for each
    output window quantise the four source elements and store them (pass 2).
    Returns (X'[M, K'], s[M] or None for bf16)."""
    q, s = quantize_rows(X, dtype)
    return lift(q, N), s


# ----------------------------------------------------------------------------
# Reference GEMM and epilogue  (Sec. 3.1 goal: w^T x = Phi(w)^T Psi(x))
# ----------------------------------------------------------------------------

def gemm_exact(Xq: np.ndarray, Wq: np.ndarray, dtype: str) -> np.ndarray:
    """acc[m, o] = sum_k X[m, k] * W[o, k]: int64 for i8, fp64 for fp8 / bf16
    (operands converted exactly).  Used for both the unlifted (K) and the lifted
    (K') product."""
    if dtype == "i8":
        return np.asarray(Xq, dtype=np.int8).astype(np.int64) @ \
            np.asarray(Wq, dtype=np.int8).astype(np.int64).T
    return to_real(Xq, dtype) @ to_real(Wq, dtype).T


def epilogue(acc: np.ndarray, s_x, s_w, dtype: str) -> np.ndarray:
    """Y = bf16( (fp32(acc) * s_x[m]) * s_w[o] ), two rounded fp32 multiplies in
    that order; bf16 operands carry no scales: Y = bf16(fp32(acc)).
    Returns bf16 bit patterns (uint16)."""
    if dtype == "i8":
        a = np.asarray(acc)
        assert np.all(np.abs(a) < 2 ** 31), "accumulator exceeds int32"
    f = np.asarray(acc).astype(np.float32)
    if dtype not in UNSCALED:
        f = (f * np.asarray(s_x, dtype=np.float32)[:, None]).astype(np.float32)
        f = (f * np.asarray(s_w, dtype=np.float32)[None, :]).astype(np.float32)
    return bf16_bits(f)


def prepare_weights(W: np.ndarray, N: int, dtype: str):
    """Offline step: prune fp32 weights to (2N-2):2N, then quantise per output
    channel.  Returns (Wq, s_w)."""
    return quantize_rows(prune_2n(np.asarray(W, dtype=np.float32), N), dtype)


def linear_reference(X: np.ndarray, W: np.ndarray, N: int, dtype: str):
    """The plain definition of the layer's result: quantise, multiply at the
    original K, rescale.  Returns dict with every intermediate."""
    Wq, s_w = prepare_weights(W, N, dtype)
    Xq, s_x = quantize_rows(X, dtype)
    acc = gemm_exact(Xq, Wq, dtype)
    Y = epilogue(acc, s_x, s_w, dtype)
    return dict(Wq=Wq, s_w=s_w, Xq=Xq, s_x=s_x, acc=acc, Y=Y)
