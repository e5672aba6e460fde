"""Pins for the CPU oracle: every function is checked against something other than
itself -- values the paper prints, hand-worked blocks, closed forms, invariants, brute
force over all block masks, and library routines (numpy sort / matmul, torch casts)."""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import slide_oracle as so
from oracle import gemm_ref
from paper_2603_05232_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLD, name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


# ---------------------------------------------------------------- cost model
def test_cost_model_matches_printed_table():
    for line in _lines("cost_model_table.txt"):
        pat, N, g, s = line.split()
        N = int(N)
        z, l = map(int, pat.split(":"))
        assert (z, l) == (2 * N - 2, 2 * N)
        assert abs(so.gamma(N) - float(g)) <= 0.005 + 1e-12
        assert abs(so.s_eff(N) - float(s)) <= 0.005 + 1e-12
        assert so.n_windows(N) == N - 1
        assert abs(so.s_eff(N) - l / z) < 1e-12          # bound equals 1/density (Thm 3)
    assert so.gamma(2) == 1.0 and so.s_eff(2) == 2.0      # native 2:4 row of the table


def test_lifted_k_of_benchmark_shapes():
    assert so.lifted_k(512, 4) == 768
    assert so.lifted_k(3584, 4) == 5376 and so.lifted_k(18944, 4) == 28416
    assert so.lifted_k(6144, 3) == 8192 and so.lifted_k(4096, 4) == 6144 and so.lifted_k(5120, 5) == 8192
    for N in range(2, 9):
        assert so.lifted_k(2 * N * 7, N) == 7 * 4 * (N - 1)
        # Alg. 1: n_g = ceil(K / 2N), so a partial last block counts as a whole one
        assert so.lifted_k(2 * N * 7 + 2, N) == 8 * 4 * (N - 1)
        assert so.lifted_k(1, N) == 4 * (N - 1)
    assert so.lifted_k(3584, 3) == 598 * 8 and so.lifted_k(4096, 3) == 683 * 8 and so.lifted_k(6912, 5) == 692 * 16
    with pytest.raises(ValueError):
        so.lifted_k(0, 4)
    for bad in (1, 9, 0, -1):
        with pytest.raises(ValueError):
            so.lifted_k(64, bad)


# ---------------------------------------------------------------- storage formats
def test_fp8_codec_roundtrip_and_torch_cast():
    codes = np.arange(256, dtype=np.uint8)
    vals = so.fp8_e4m3_decode(codes)
    tv = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    finite = ~np.isnan(tv)
    assert np.array_equal(np.isnan(vals), np.isnan(tv))
    assert np.array_equal(vals[finite], tv[finite])
    assert np.nanmax(vals) == 448.0
    enc = so.fp8_e4m3_encode(vals[finite].astype(np.float32))
    assert np.array_equal(enc, codes[finite])                       # every code round-trips
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * s for s in (0.01, 1, 50, 300)])
    x = np.clip(x, -448, 448)
    mids = ((vals[1:126] + vals[2:127]) / 2).astype(np.float32)    # exact ties between codes
    x = np.concatenate([x, mids, -mids, np.float32([0.0, -0.0, 448, -448, 2 ** -10, 2 ** -9, 1e-8])])
    ours = so.fp8_e4m3_encode(x)
    theirs = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(ours, theirs)
    assert np.array_equal(so.fp8_e4m3_encode(np.float32([1e6, -1e6])), np.uint8([0x7E, 0xFE]))  # saturates


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(300000) * np.exp(rng.uniform(-20, 20, 300000))).astype(np.float32)
    x = np.concatenate([x, np.float32([0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38])])
    ours = so.bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    assert np.array_equal(so.bf16_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_fp16_rounding_matches_torch_and_the_format():
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(300000) * np.exp(rng.uniform(-18, 10, 300000))).astype(np.float32)
    x = np.clip(x, -65504, 65504)
    x = np.concatenate([x, np.float32([0, -0.0, 1.0, 1.00048828125, 1.0009765625, 65504.0, 6.0e-8, 5.96e-8, 2.0e-8])])
    ours = so.fp16_bits(x)
    theirs = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    # format facts: 1 + 2^-11 is a tie and goes to even (1.0); 1 + 2^-10 is representable; the largest finite value
    assert ours[-7] == 0x3C00 and ours[-6] == 0x3C00 and ours[-5] == 0x3C01 and ours[-4] == 0x7BFF
    assert so.fp16_to_f32(np.uint16([0x3C00, 0xC000, 0x0001, 0x7BFF])).tolist() == [1.0, -2.0, 2.0 ** -24, 65504.0]
    # every finite code survives a round trip
    codes = np.arange(0x7C00, dtype=np.uint16)
    assert np.array_equal(so.fp16_bits(so.fp16_to_f32(codes)), codes)


# ---------------------------------------------------------------- pruning
@pytest.mark.parametrize("N", [2, 3, 4, 5, 8])
def test_prune_keeps_top_2n_minus_2(N):
    rng = np.random.default_rng(N)
    W = rng.standard_normal((13, 2 * N * 9)).astype(np.float32)
    P = so.prune_2n(W, N)
    b0, b1 = W.reshape(13, 9, 2 * N), P.reshape(13, 9, 2 * N)
    for r in range(13):
        for g in range(9):
            src, dst = b0[r, g], b1[r, g]
            keep = sorted(range(2 * N), key=lambda k: (-abs(src[k]), k))[:2 * N - 2]   # brute force
            exp = np.zeros_like(src)
            exp[keep] = src[keep]
            assert np.array_equal(dst, exp)
            assert (dst != 0).sum() == 2 * N - 2
            assert np.abs(src[dst == 0]).max() <= np.abs(dst[dst != 0]).min()


def test_prune_ties_keep_lower_index():
    W = np.float32([[1, -1, 1, 1, -1, 1, 1, 1]])
    assert np.array_equal(so.prune_2n(W, 4), np.float32([[1, -1, 1, 1, -1, 1, 0, 0]]))
    W = np.float32([[2, 1, 2, 1, 2, 1]])
    assert np.array_equal(so.prune_2n(W, 3), np.float32([[2, 1, 2, 0, 2, 0]]))


# ---------------------------------------------------------------- quantisation
def test_int8_quantisation_properties():
    X = synth.activations(32, 512, seed=3, n_outliers=4)
    X[7] = 0.0                                                    # all-zero token
    X[9, 100] = -np.abs(X[9]).max() * 2                           # negative extreme
    q, s = so.quantize_rows(X, "i8")
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert q.min() >= -127 and q.max() <= 127
    amax = np.abs(X).max(axis=1)
    for m in range(32):
        if amax[m] == 0:
            assert s[m] == 1.0 and not q[m].any()
            continue
        k = np.argmax(np.abs(X[m]))
        assert abs(int(q[m, k])) == 127 and np.sign(q[m, k]) == np.sign(X[m, k])
        assert s[m] == np.float32(amax[m]) / np.float32(127)
    err = np.abs(X.astype(np.float64) - q.astype(np.float64) * s[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * s[:, None] * (1 + 1e-5))          # within half a step
    assert q[9, 100] == -127
    # an independent fp64 evaluation agrees except at fp32-rounding ties
    q64 = np.clip(np.rint(X.astype(np.float64) * (127.0 / np.where(amax > 0, amax, 1))[:, None]), -127, 127)
    assert np.mean(q64 != q) < 1e-3 and np.abs(q64 - q).max() <= 1


def test_int8_rounding_is_nearest_even():
    # row max 127 -> r == 1 exactly, so the products are the inputs themselves
    X = np.float32([[127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, 126.5, -126.5, 0.49999, 63.5]])
    q, s = so.quantize_rows(X, "i8")
    assert s[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3, 126, -126, 0, 64]


def test_fp8_and_bf16_quantisation():
    X = synth.activations(8, 256, seed=4, n_outliers=2)
    X[3] = 0
    q, s = so.quantize_rows(X, "fp8")
    assert q.dtype == np.uint8
    v = so.fp8_e4m3_decode(q)
    assert np.nanmax(np.abs(v)) == 448.0 and not np.isnan(v).any()
    for m in range(8):
        if m == 3:
            assert s[m] == 1 and not (q[m] & 0x7F).any()
            continue
        k = np.argmax(np.abs(X[m]))
        assert abs(v[m, k]) == 448.0
    # library cross-check: torch cast of the same fp32 products
    r, _ = so.row_scales(X, "fp8")
    prod = torch.from_numpy((X * r[:, None]).astype(np.float32)).clamp(-448, 448)
    assert np.array_equal(q, prod.to(torch.float8_e4m3fn).view(torch.uint8).numpy())
    b, sb = so.quantize_rows(X, "bf16")
    assert sb is None
    assert np.array_equal(b, torch.from_numpy(X).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    h, sh = so.quantize_rows(X, "fp16")
    assert sh is None
    assert np.array_equal(h, torch.from_numpy(X).to(torch.float16).view(torch.int16).numpy().view(np.uint16))


# ---------------------------------------------------------------- Phi (Alg. 2)
def _alg2_literal_row(w, N):
    """Alg. 2 for one row, scalar loops (second implementation, test-only)."""
    K = len(w)
    out = [0] * (K // (2 * N) * 4 * (N - 1))
    used = [False] * K
    for g in range(K // (2 * N)):
        for l in range(N - 1):
            b, cnt = 2 * N * g + 2 * l, 0
            for d in range(4):
                if w[b + d] != 0 and not used[b + d] and cnt < 2:
                    out[(N - 1) * 4 * g + 4 * l + d] = w[b + d]
                    used[b + d] = True
                    cnt += 1
    return out


def _carry_recurrence_row(w, N):
    """Independent formulation: window j takes the still-unused non-zeros of its first
    two positions (the carry) before the new ones, at most two in total; only a 2-bit
    carry mask moves between windows."""
    K = len(w)
    out = []
    for g in range(K // (2 * N)):
        blk = w[2 * N * g:2 * N * (g + 1)]
        carry = [blk[0] != 0, blk[1] != 0]            # unused non-zeros at positions 2j, 2j+1
        for j in range(N - 1):
            cand = [2 * j + t for t in (0, 1) if carry[t]] + [2 * j + 2 + t for t in (0, 1) if blk[2 * j + 2 + t] != 0]
            take = cand[:2]
            win = [0, 0, 0, 0]
            for p in take:
                win[p - 2 * j] = blk[p]
            out += win
            carry = [(2 * j + 2 + t) in cand and (2 * j + 2 + t) not in take for t in (0, 1)]
    return out


def test_alg2_hand_worked_blocks():
    for line in _lines("alg2_worked_blocks.txt"):
        n, blk, exp = [p.strip() for p in line.split("|")]
        N = int(n)
        blk = np.int8([int(v) for v in blk.split()])[None, :]
        exp = np.int8([int(v) for v in exp.split()])[None, :]
        assert exp.shape[1] == 4 * (N - 1)
        assert np.array_equal(so.slide_decompose(blk, N), exp), line


def _all_masks(N, max_pop):
    L = 2 * N
    rows = []
    for mask in range(1 << L):
        if bin(mask).count("1") <= max_pop:
            rows.append([(k + 1) if (mask >> k) & 1 else 0 for k in range(L)])
    return np.int8(rows)


@pytest.mark.parametrize("N,count,count_full", [(2, 11, 6), (3, 57, 15), (4, 247, 28), (5, 1013, 45), (6, 4083, 66)])
def test_alg2_brute_force_all_masks(N, count, count_full):
    B = _all_masks(N, 2 * N - 2)                         # distinct values 1..2N mark positions
    assert len(B) == count
    assert (np.count_nonzero(B, axis=1) == 2 * N - 2).sum() == count_full   # C(2N, 2N-2)
    Wp = so.slide_decompose(B, N)
    win = Wp.reshape(len(B), N - 1, 4)
    assert np.count_nonzero(win, axis=-1).max() <= 2     # every window is 2:4
    back = np.zeros_like(B, dtype=np.int64)
    hits = np.zeros_like(B, dtype=np.int64)
    for l in range(N - 1):
        back[:, 2 * l:2 * l + 4] += win[:, l]
        hits[:, 2 * l:2 * l + 4] += win[:, l] != 0
    assert np.array_equal(back, B)                       # windows sum back exactly
    assert np.array_equal(hits, (B != 0).astype(np.int64))   # each non-zero in exactly one window
    for r in range(0, len(B), max(1, len(B) // 300)):
        row = B[r].tolist()
        assert Wp[r].tolist() == _alg2_literal_row(row, N) == _carry_recurrence_row(row, N)


def test_alg2_multi_group_rows_and_identity():
    rng = np.random.default_rng(11)
    for N in (2, 3, 4, 5, 7, 8):
        W = so.prune_2n(rng.integers(-127, 128, size=(9, 2 * N * 6)).astype(np.float32), N).astype(np.int8)
        W[rng.random(W.shape) < 0.2] = 0                 # fewer than 2N-2 non-zeros is allowed
        Wp = so.slide_decompose(W, N)
        assert Wp.shape == (9, so.lifted_k(W.shape[1], N))
        for r in range(9):
            assert Wp[r].tolist() == _alg2_literal_row(W[r].tolist(), N) == _carry_recurrence_row(W[r].tolist(), N)
        if N == 2:
            assert np.array_equal(Wp, W)                 # one window per block: identity
    with pytest.raises(ValueError):
        so.slide_decompose(np.int8([[1, 2, 3, 4, 5, 6, 7, 0]]), 4)   # 7 non-zeros in a 6:8 block
    # fp8 / bf16: -0 counts as zero
    Wb = np.uint16([[0x8000, 0x3F80, 0, 0x3F80, 0x3F80, 0x8000]])
    assert so.slide_decompose(Wb, 3, "bf16").tolist() == [[0, 0x3F80, 0, 0x3F80, 0, 0, 0x3F80, 0]]
    Wh = np.uint16([[0x8000, 0x3C00, 0, 0x3C00, 0x3C00, 0x8000]])     # -0, 1, 0, 1, 1, -0 in binary16
    assert so.slide_decompose(Wh, 3, "fp16").tolist() == [[0, 0x3C00, 0, 0x3C00, 0, 0, 0x3C00, 0]]


# ---------------------------------------------------------------- canonical 2:4 compression
def test_compress_roundtrip_and_padding_rule():
    wins = [w for w in itertools.product([0, 5, -3], repeat=4) if sum(v != 0 for v in w) <= 2]
    Wp = np.int8(wins).reshape(1, -1)
    vals, idx = so.compress_24(Wp)
    assert vals.shape == (1, Wp.shape[1] // 2) and idx.shape == (1, Wp.shape[1] // 4)
    i0, i1 = idx & 3, (idx >> 2) & 3
    assert np.all(i0 < i1) and np.all(idx < 16)
    assert np.array_equal(so.decompress_24(vals, idx), Wp)
    table = {(0, 0, 0, 0): (0, 1, 0, 0), (0, 0, 0, 5): (0, 3, 0, 5), (0, 5, 0, 0): (0, 1, 0, 5),
             (5, 0, 0, 0): (0, 1, 5, 0), (0, 0, 5, -3): (2, 3, 5, -3), (0, 0, -3, 0): (0, 2, 0, -3),
             (5, 0, 0, -3): (0, 3, 5, -3)}
    for w, (e0, e1, v0, v1) in table.items():
        v, i = so.compress_24(np.int8([w]))
        assert (int(i[0, 0] & 3), int(i[0, 0] >> 2), int(v[0, 0]), int(v[0, 1])) == (e0, e1, v0, v1)
    with pytest.raises(ValueError):
        so.compress_24(np.int8([[1, 2, 3, 0]]))
    X, W = synth.config1()
    Wq, _ = so.prepare_weights(W, 4, "i8")
    Wp = so.slide_decompose(Wq, 4)
    vals, idx = so.compress_24(Wp)
    assert vals.shape == (512, 384) and idx.shape == (512, 192)
    assert np.array_equal(so.decompress_24(vals, idx), Wp)


# ---------------------------------------------------------------- Psi
def test_lifting_matches_printed_matrix_and_multiplicity():
    exp = np.array([[int(v) for v in l.split()] for l in _lines("lifting_6_8.txt")])
    x = np.arange(8)[None, :]
    assert np.array_equal(so.lift(x, 4).reshape(3, 4), exp)
    for N in range(2, 9):
        K = 2 * N * 5
        src = np.arange(K)[None, :]
        L = so.lift(src, N)[0]
        assert len(L) == so.lifted_k(K, N)
        mult = np.bincount(L, minlength=K).reshape(5, 2 * N)
        want = np.full(2 * N, 2)
        want[[0, 1, 2 * N - 2, 2 * N - 1]] = 1
        assert np.all(mult == want)
        if N == 2:
            assert np.array_equal(L, src[0])


def test_act_lift_quant_commutes_with_lifting():
    X = synth.activations(8, 240, seed=9, n_outliers=2)
    for N in (2, 3, 4, 5):
        for dt in so.DTYPES:
            Xl, s = so.act_lift_quant(X, N, dt)
            q, s2 = so.quantize_rows(X, dt)
            assert np.array_equal(Xl, so.lift(q, N))
            assert (s is None and s2 is None) or np.array_equal(s, s2)


# ---------------------------------------------------------------- GEMM and epilogue
def test_lifted_product_equals_unlifted_int8():
    for N, seed in ((3, 0), (4, 1), (5, 2), (2, 3)):
        K = 2 * N * 16
        X = synth.activations(12, K, seed, n_outliers=2)
        W = synth.weights(24, K, seed)
        ref = so.linear_reference(X, W, N, "i8")
        Wp = so.slide_decompose(ref["Wq"], N)
        Xl, s = so.act_lift_quant(X, N, "i8")
        acc = so.gemm_exact(Xl, Wp, "i8")
        assert acc.dtype == np.int64 and np.array_equal(acc, ref["acc"])
        vals, idx = so.compress_24(Wp)
        assert np.array_equal(so.gemm_exact(Xl, so.decompress_24(vals, idx), "i8"), ref["acc"])
        # library / brute-force pins for the unlifted sum
        assert np.array_equal(ref["acc"], gemm_ref.gemm_i8_i64(ref["Xq"], ref["Wq"]))
        assert np.array_equal(ref["acc"], (ref["Xq"].astype(np.float64) @ ref["Wq"].astype(np.float64).T).astype(np.int64))
        m, o = 5, 7
        assert ref["acc"][m, o] == sum(int(a) * int(b) for a, b in zip(ref["Xq"][m], ref["Wq"][o]))


@pytest.mark.parametrize("dt", ["fp8", "bf16", "fp16"])
def test_lifted_product_equals_unlifted_float(dt):
    N, K = 4, 256
    X = synth.activations(10, K, 2, n_outliers=2)
    W = synth.weights(20, K, 2)
    ref = so.linear_reference(X, W, N, dt)
    Wp = so.slide_decompose(ref["Wq"], N, dt)
    Xl, _ = so.act_lift_quant(X, N, dt)
    acc = so.gemm_exact(Xl, Wp, dt)
    scale = np.abs(ref["acc"]).max()
    assert np.abs(acc - ref["acc"]).max() <= 1e-12 * scale
    c = gemm_ref.gemm_f64(so.to_real(ref["Xq"], dt), so.to_real(ref["Wq"], dt))
    assert np.abs(c - ref["acc"]).max() <= 1e-12 * scale


def test_epilogue_against_torch():
    rng = np.random.default_rng(3)
    acc = rng.integers(-3_000_000, 3_000_000, size=(9, 17))
    sx = rng.uniform(0.001, 0.2, 9).astype(np.float32)
    sw = rng.uniform(1e-4, 1e-3, 17).astype(np.float32)
    ours = so.epilogue(acc, sx, sw, "i8")
    t = (torch.from_numpy(acc).to(torch.float32) * torch.from_numpy(sx)[:, None]) * torch.from_numpy(sw)[None, :]
    assert np.array_equal(ours, t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    f = rng.standard_normal((4, 6))
    assert np.array_equal(so.epilogue(f, None, None, "bf16"),
                          torch.from_numpy(f).float().to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    with pytest.raises(AssertionError):
        so.epilogue(np.int64([[2 ** 31]]), np.float32([1]), np.float32([1]), "i8")


def test_config1_end_to_end_consistency():
    X, W = synth.config1()
    ref = so.linear_reference(X, W, 4, "i8")
    assert ref["Wq"].shape == (512, 512) and ref["Y"].shape == (16, 512)
    nzb = np.count_nonzero(ref["Wq"].reshape(512, 64, 8), axis=-1)
    assert nzb.max() <= 6
    Xl, s = so.act_lift_quant(X, 4, "i8")
    assert Xl.shape == (16, 768)
    Wp = so.slide_decompose(ref["Wq"], 4)
    Y2 = so.epilogue(so.gemm_exact(Xl, Wp, "i8"), s, ref["s_w"], "i8")
    assert np.array_equal(Y2, ref["Y"])
    # dequantised result tracks the fp64 product of the pruned fp32 operands
    Yf = so.bf16_to_f32(ref["Y"]).astype(np.float64)
    exact = X.astype(np.float64) @ so.prune_2n(W, 4).astype(np.float64).T
    rel = np.linalg.norm(Yf - exact) / np.linalg.norm(exact)
    assert rel < 0.1


# ---------------------------------------------------------------- K not a multiple of 2N
@pytest.mark.parametrize("N", [2, 3, 4, 5, 8])
def test_partial_last_block_equals_explicit_zero_padding(N):
    """Alg. 1 sets n_g = ceil(K/2N): every step on a row whose length is not a multiple of
    2N must equal the same step on the row completed with zeros (checked by padding
    explicitly with numpy and calling the functions at a multiple of 2N), and the
    lifted product must still equal the plain product over the original K."""
    rng = np.random.default_rng(100 + N)
    for r in range(1, 2 * N):
        K = 2 * N * 3 + r
        Kb = 2 * N * 4
        W = rng.standard_normal((5, K)).astype(np.float32)
        X = rng.standard_normal((4, K)).astype(np.float32)
        Wpad = np.zeros((5, Kb), np.float32); Wpad[:, :K] = W
        Xpad = np.zeros((4, Kb), np.float32); Xpad[:, :K] = X
        # pruning: pads are dropped first, the result is the padded call cut back
        P = so.prune_2n(W, N)
        assert np.array_equal(P, so.prune_2n(Wpad, N)[:, :K])
        tail = P[:, 2 * N * 3:]
        kept = (tail != 0).sum(axis=1)
        assert np.all(kept == min(r, 2 * N - 2))           # only a tail of 2N-1 loses a real entry
        if r == 2 * N - 1:
            lost = np.argmax(tail == 0, axis=1)
            assert np.array_equal(lost, np.argmin(np.abs(W[:, 2 * N * 3:]), axis=1))
        for dt in ("i8", "bf16"):
            Wq, _ = so.quantize_rows(P, dt)
            Wq_pad = np.zeros((5, Kb), Wq.dtype); Wq_pad[:, :K] = Wq
            Wp = so.slide_decompose(Wq, N, dt)
            assert Wp.shape == (5, 4 * 4 * (N - 1))
            assert np.array_equal(Wp, so.slide_decompose(Wq_pad, N, dt))
            Xl, sx = so.act_lift_quant(X, N, dt)
            Xl_pad, sx_pad = so.act_lift_quant(Xpad, N, dt)
            assert np.array_equal(Xl, Xl_pad)
            assert sx is None or np.array_equal(sx, sx_pad)
            Xq, _ = so.quantize_rows(X, dt)
            lifted = so.gemm_exact(Xl, Wp, dt)
            plain = so.gemm_exact(Xq, Wq, dt)
            if dt == "i8":
                assert np.array_equal(lifted, plain)
            else:
                assert np.allclose(lifted, plain, rtol=1e-12, atol=1e-12)


def test_partial_last_block_hand_worked():
    # 4:6 (N = 3), K = 8: one full block and a block of two real elements.
    # block 1 = (7, 9, 0, 0, 0, 0) after zero completion; windows of block 1 read
    # positions 6..9 and 8..11 -> (7, 9, 0, 0) and (0, 0, 0, 0)
    W = np.int8([[1, 0, 2, 3, 0, 4, 7, 9]])
    Wp = so.slide_decompose(W, 3, "i8")
    assert Wp.tolist() == [[1, 0, 2, 0, 0, 3, 0, 4, 7, 9, 0, 0, 0, 0, 0, 0]]
    X = np.int8([[10, 11, 12, 13, 14, 15, 16, 17]])
    assert so.lift(X, 3).tolist() == [[10, 11, 12, 13, 12, 13, 14, 15, 16, 17, 0, 0, 0, 0, 0, 0]]
