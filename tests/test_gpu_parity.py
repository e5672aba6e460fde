"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.
Integer / byte / index results must be bit-exact."""
import numpy as np
import pytest
import torch

from oracle import slide_oracle as so
from oracle import gemm_ref
from paper_2603_05232_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def bits16(t):
    return host(t.view(torch.int16)).view(np.uint16)


def to_dev_q(q, dtype):
    """oracle storage array -> torch tensor of the binding's storage dtype"""
    if dtype == "i8":
        return dev(q.astype(np.int8))
    if dtype == "fp8":
        return dev(q.astype(np.uint8))
    return dev(q.astype(np.uint16).view(np.int16)).view(torch.float16 if dtype == "fp16" else torch.bfloat16)


def from_dev_q(t, dtype):
    if dtype in ("bf16", "fp16"):
        return bits16(t)
    return host(t)


def check_lifted(got, exp, dtype):
    """X_lifted rows are stored K' rounded up to whole 128-byte units wide: the first K' columns
    are the oracle's lifted row, the rest is zero padding."""
    got = from_dev_q(got, dtype)
    per = 128 // got.dtype.itemsize
    Kp = exp.shape[1]
    assert got.shape == (exp.shape[0], (Kp + per - 1) // per * per)
    assert np.array_equal(got[:, :Kp], exp)
    assert not got[:, Kp:].any()


# ------------------------------------------------------------------ act_lift_quant
@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,M,K", [(4, 16, 512), (2, 7, 64), (3, 5, 6 * 37), (4, 33, 3584), (5, 3, 5120), (8, 4, 16 * 9),
                                   (4, 2, 18944), (3, 9, 6144), (4, 3, 8 * 3001),
                                   # K not a multiple of 2N: the last block is completed with zeros (Alg. 1, n_g = ceil(K / 2N))
                                   (3, 5, 100), (4, 7, 3001), (5, 3, 6912), (2, 4, 63), (8, 3, 17), (4, 2, 1), (3, 6, 3584),
                                   (7, 3, 4099)])
def test_act_lift_quant_fp32(dtype, N, M, K):
    X = synth.activations(M, K, seed=N * 100 + M, n_outliers=min(4, K // 8))
    if M > 2:
        X[1] = 0.0                                           # an all-zero token
        X[2, K // 2] = -3.0 * np.abs(X[2]).max()              # negative extreme
    exp, s = so.act_lift_quant(X, N, dtype)
    got, gs = binding.act_lift_quant(dev(X), N, dtype)
    check_lifted(got, exp, dtype)
    if dtype in ("bf16", "fp16"):
        assert gs is None
    else:
        assert np.array_equal(host(gs), s)


@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
def test_act_lift_quant_bf16_input_and_row_stride(dtype):
    M, K, N = 19, 1024, 4
    Xf = synth.activations(M, K, seed=5)
    Xb = so.bf16_bits(Xf)                                    # bf16 input tensor, exact fp32 value of it for the oracle
    exp, s = so.act_lift_quant(so.bf16_to_f32(Xb), N, dtype)
    xt = dev(Xb.view(np.int16)).view(torch.bfloat16)
    got, gs = binding.act_lift_quant(xt, N, dtype)
    check_lifted(got, exp, dtype)
    if dtype not in ("bf16", "fp16"):
        assert np.array_equal(host(gs), s)
    # strided rows (a column slice of a wider matrix), fp32
    wide = np.zeros((M, K + 64), dtype=np.float32)
    wide[:, 32:32 + K] = Xf
    exp2, s2 = so.act_lift_quant(Xf, N, dtype)
    got2, gs2 = binding.act_lift_quant(dev(wide)[:, 32:32 + K], N, dtype)
    check_lifted(got2, exp2, dtype)
    # bf16 input whose length is neither a multiple of 2N nor of the vector width
    K3 = 1003
    exp3, s3 = so.act_lift_quant(so.bf16_to_f32(Xb[:, :K3]), N, dtype)
    got3, gs3 = binding.act_lift_quant(xt[:, :K3], N, dtype)
    check_lifted(got3, exp3, dtype)
    if dtype not in ("bf16", "fp16"):
        assert np.array_equal(host(gs3), s3)


# ------------------------------------------------------------------ slide_prune_quant
@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,O,K", [(4, 512, 512), (2, 9, 64), (3, 17, 6 * 50), (5, 6, 5120), (8, 5, 16 * 11),
                                   (3, 17, 100), (4, 9, 3001), (4, 5, 7), (8, 6, 15 + 32), (2, 3, 5), (5, 4, 6912)])
def test_prune_quant(dtype, N, O, K):
    W = synth.weights(O, K, seed=N)
    W[0, : min(K, 2 * N)] = 0.5                               # ties: the lower indices survive
    if O > 3:
        W[3] = 0.0
    expq, exps = so.prepare_weights(W, N, dtype)
    gq, gs = binding.slide_prune_quant(dev(W), N, dtype)
    assert np.array_equal(from_dev_q(gq, dtype), expq)
    if dtype not in ("bf16", "fp16"):
        assert np.array_equal(host(gs), exps)


@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,O,K", [(4, 33, 512), (3, 7, 100), (8, 5, 1000)])
def test_prune_quant_bf16_weights(dtype, N, O, K):
    """Weights handed over as bf16 (in_dtype = SS_IN_BF16): the oracle sees their exact fp32 values."""
    Wb = so.bf16_bits(synth.weights(O, K, seed=20 + N))
    Wb[0, : min(K, 2 * N)] = 0x3F00                          # ties (0.5): the lower indices survive
    expq, exps = so.prepare_weights(so.bf16_to_f32(Wb), N, dtype)
    gq, gs = binding.slide_prune_quant(dev(Wb.view(np.int16)).view(torch.bfloat16), N, dtype)
    assert np.array_equal(from_dev_q(gq, dtype), expq)
    if dtype not in ("bf16", "fp16"):
        assert np.array_equal(host(gs), exps)


# ------------------------------------------------------------------ slide_decompose (canonical form)
@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,O,K", [(4, 512, 512), (2, 5, 64), (3, 33, 6 * 21), (5, 7, 200), (6, 3, 120), (7, 2, 14 * 5), (8, 4, 160),
                                   (3, 9, 100), (4, 5, 3001), (8, 3, 17), (2, 4, 63), (5, 2, 1), (6, 7, 131)])
def test_decompose_canonical(dtype, N, O, K):
    W = synth.weights(O, K, seed=10 + N)
    Wq, _ = so.prepare_weights(W, N, dtype)
    rng = np.random.default_rng(N)
    Wq = Wq.copy()
    Wq[rng.random(Wq.shape) < 0.15] = 0                       # blocks with fewer than 2N-2 non-zeros
    if dtype != "i8":
        neg0 = 0x80 if dtype == "fp8" else 0x8000
        Wq[rng.random(Wq.shape) < 0.05] = neg0               # -0 must count as zero
    Wp = so.slide_decompose(Wq, N, dtype)
    ev, ei = so.compress_24(Wp, dtype)
    gv, gi, viol = binding.slide_decompose_canonical(to_dev_q(Wq, dtype), N, dtype)
    gv, gi = from_dev_q(gv, dtype), host(gi)
    assert int(host(viol)[0]) == 0
    assert np.all((gi & 3) < ((gi >> 2) & 3)) and np.all(gi < 16)
    # what is unique: the densified windows; -0 inputs never surface as stored values
    dense = so.decompress_24(gv, gi)
    assert np.array_equal(~so.is_zero(dense, dtype), ~so.is_zero(Wp, dtype))
    assert np.array_equal(np.where(so.is_zero(dense, dtype), 0, dense), Wp)
    # and this library follows the same padding rule as the oracle's canonical form
    assert np.array_equal(gi, ei)
    assert np.array_equal(np.where(so.is_zero(gv, dtype), 0, gv), ev)


def test_decompose_counts_pattern_violations():
    N, O, K = 4, 4, 64
    Wq = np.zeros((O, K), dtype=np.int8)
    Wq[1, 8:15] = 1                                          # 7 non-zeros in one 6:8 block
    Wq[2, 0:8] = 2                                           # 8 non-zeros
    Wq[3, 16:22] = 3                                         # 6: allowed
    _, _, viol = binding.slide_decompose_canonical(dev(Wq), N, "i8")
    assert int(host(viol)[0]) == 2
    _, _, viol_packed = binding.slide_decompose(dev(Wq), N, "i8", count_violations=True)
    assert int(host(viol_packed)[0]) == 2                    # the packed form counts the same blocks, once each
    Wh = np.zeros((3, 24), dtype=np.uint16)                  # 16-bit elements, 4:6, row length not a multiple of 128 bytes
    Wh[0, 0:5] = 0x3C00                                      # 5 non-zeros in a block of 6
    Wh[1, 6:10] = 0x3C00                                     # 4: allowed
    Wh[2, 18:24] = 0xBC00                                    # 6 non-zeros
    Wh[2, 3] = 0x8000                                        # -0 is not a non-zero
    _, _, v16 = binding.slide_decompose(to_dev_q(Wh, "fp16"), 3, "fp16", count_violations=True)
    assert int(host(v16)[0]) == 2


# ------------------------------------------------------------------ GEMMs
def _gemm_case(M, O, K, N, seed):
    X = synth.activations(M, K, seed)
    W = synth.weights(O, K, seed)
    ref = so.linear_reference(X, W, N, "i8")
    return X, W, ref


def _acc_big(Xq, Wq):
    return gemm_ref.gemm_i8_i64(Xq, Wq)


@pytest.mark.parametrize("N,M,O,K", [(4, 16, 512, 512),          # the anchor case
                                     (4, 300, 640, 1024),        # several tiles, ragged tokens and channels
                                     (3, 257, 130, 768),         # K' = 1024, one ragged panel
                                     (5, 64, 256, 640),          # K' = 1024
                                     (2, 40, 128, 256),          # native 2:4
                                     (4, 1, 384, 512)])          # a single token
def test_sparse_and_dense_gemm_int8(N, M, O, K):
    X, W, ref = _gemm_case(M, O, K, N, seed=M + O)
    Xd, Wd = dev(X), dev(W)
    Wq, s_w = binding.slide_prune_quant(Wd, N, "i8")
    assert np.array_equal(host(Wq), ref["Wq"]) and np.array_equal(host(s_w), ref["s_w"])
    w_vals, w_meta, viol = binding.slide_decompose(Wq, N, "i8", count_violations=True)
    XL, s_x = binding.act_lift_quant(Xd, N, "i8")
    Y = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, "i8")
    assert int(host(viol)[0]) == 0
    assert np.array_equal(bits16(Y), ref["Y"])
    # dense baseline at the original K (N = 2 lifting is plain quantisation)
    Xq, s_x2 = binding.act_lift_quant(Xd, 2, "i8")
    assert np.array_equal(host(Xq), ref["Xq"]) and np.array_equal(host(s_x2), ref["s_x"])
    Yd = binding.dense_gemm(Xq, s_x2, Wq, s_w, "i8")
    assert np.array_equal(bits16(Yd), ref["Y"])


def test_gemm_strided_output_and_random_sparse_weights():
    # weights that are not the product of pruning: random values with random (<= 6 of 8) supports,
    # so windows with 0, 1 and 2 stored values all occur; output written into a wider buffer
    rng = np.random.default_rng(77)
    M, O, K, N = 70, 256, 512, 4
    Wq = rng.integers(-127, 128, size=(O, K)).astype(np.int8)
    keep = np.argsort(rng.random((O, K // 8, 8)), axis=-1) < rng.integers(0, 7, size=(O, K // 8, 1))
    Wq = (Wq.reshape(O, K // 8, 8) * keep).reshape(O, K).astype(np.int8)
    Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    s_x = rng.uniform(0.01, 0.1, M).astype(np.float32)
    s_w = rng.uniform(1e-4, 1e-3, O).astype(np.float32)
    exp = so.epilogue(so.gemm_exact(Xq, Wq, "i8"), s_x, s_w, "i8")
    w_vals, w_meta = binding.slide_decompose(dev(Wq), N, "i8")
    XL = dev(so.lift(Xq, N))
    buf = torch.full((M, O + 64), -1.0, dtype=torch.bfloat16, device=DEV)
    binding.slide_sparse_gemm(XL, dev(s_x), w_vals, w_meta, dev(s_w), O, "i8", out=buf[:, :O])
    assert np.array_equal(bits16(buf[:, :O].contiguous()), exp)
    assert torch.all(buf[:, O:] == -1.0)
    buf2 = torch.full((M, O + 64), -1.0, dtype=torch.bfloat16, device=DEV)
    binding.dense_gemm(dev(Xq), dev(s_x), dev(Wq), dev(s_w), "i8", out=buf2[:, :O])
    assert np.array_equal(bits16(buf2[:, :O].contiguous()), exp)
    assert torch.all(buf2[:, O:] == -1.0)


# ------------------------------------------------------------------ FP8 / BF16 GEMMs
def _float_gemm_check(Ybits, ref, dtype):
    """Floating-point bar: max |Y - Y_ref| / (||Xd[m]||_2 ||Wd[o]||_2) <= 1e-2 with Xd, Wd the dequantised
    operands and Y_ref the fp64 result before the bf16 rounding.  On top of it a bound derived from the
    arithmetic (fp32 accumulation over K terms + one bf16 rounding):
    |Y - Y_ref| <= 2^-8 |Y_ref| + K 2^-23 ||Xd[m]|| ||Wd[o]||.
    FP8 adds 2^-9 ||Xd[m]|| ||Wd[o]||: the fp8 matrix instructions of gfx950 (sparse and dense) add the products of
    an instruction in small groups aligned to the group's largest product and keep 14 bits below it (measured: beside
    a product of 2^8, products of 2^-6 in the same group of 8 are dropped, 2^-5 survive; bf16 products keep all 24
    bits), so each product loses less than 2^-13 of its group's largest, and the group maxima sum to at most
    sum |x w| <= ||x|| ||w||: at most 8 (16 allowed for) x 2^-13 of that in total.  Operand placement is pinned
    separately by the exact small-integer cases, where every product survives."""
    Xd = so.to_real(ref["Xq"], dtype)
    Wd = so.to_real(ref["Wq"], dtype)
    if dtype not in ("bf16", "fp16"):
        Xd = Xd * ref["s_x"].astype(np.float64)[:, None]
        Wd = Wd * ref["s_w"].astype(np.float64)[:, None]
    Yref = Xd @ Wd.T
    Y = so.bf16_to_f32(Ybits).astype(np.float64)
    norm = np.linalg.norm(Xd, axis=1)[:, None] * np.linalg.norm(Wd, axis=1)[None, :]
    norm = np.where(norm == 0, 1.0, norm)
    err = np.abs(Y - Yref)
    assert np.max(err / norm) <= 1e-2
    K = Xd.shape[1]
    group_truncation = 2.0 ** -9 if dtype == "fp8" else 0.0
    assert np.all(err <= 2.0 ** -8 * np.abs(Yref) + (K * 2.0 ** -23 + group_truncation) * norm + 1e-30)


@pytest.mark.parametrize("dtype", ["fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,M,O,K", [(4, 16, 512, 512),           # the anchor shape
                                     (4, 300, 640, 1024),         # several tiles, ragged tokens and channels
                                     (3, 257, 130, 768),          # one ragged panel
                                     (5, 64, 256, 640),
                                     (2, 40, 128, 256),           # native 2:4
                                     (4, 1, 384, 512)])           # a single token
def test_sparse_and_dense_gemm_float(dtype, N, M, O, K):
    X = synth.activations(M, K, seed=M + O)
    W = synth.weights(O, K, seed=M + O)
    if M > 2:
        X[1] = 0.0                                               # an all-zero token
    ref = so.linear_reference(X, W, N, dtype)
    Xd, Wd = dev(X), dev(W)
    Wq, s_w = binding.slide_prune_quant(Wd, N, dtype)
    assert np.array_equal(from_dev_q(Wq, dtype), ref["Wq"])
    w_vals, w_meta, viol = binding.slide_decompose(Wq, N, dtype, count_violations=True)
    XL, s_x = binding.act_lift_quant(Xd, N, dtype)
    Y = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype)
    assert int(host(viol)[0]) == 0
    _float_gemm_check(bits16(Y), ref, dtype)
    Xq, s_x2 = binding.act_lift_quant(Xd, 2, dtype)
    assert np.array_equal(from_dev_q(Xq, dtype), ref["Xq"])
    Yd = binding.dense_gemm(Xq, s_x2, Wq, s_w, dtype)
    _float_gemm_check(bits16(Yd), ref, dtype)
    # small integers make every product and partial sum exact in fp32: then both kernels must return
    # exactly the rounded exact result, whatever their summation order
    rng = np.random.default_rng(K + M)
    Xi = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
    Wi = so.prune_2n(rng.integers(-4, 5, size=(O, K)).astype(np.float32), N)
    if dtype == "fp8":
        Xq_i, Wq_i = so.fp8_e4m3_encode(Xi), so.fp8_e4m3_encode(Wi)
        sx = np.ones(M, np.float32); sw = np.ones(O, np.float32)
    else:
        to_bits = so.bf16_bits if dtype == "bf16" else so.fp16_bits
        Xq_i, Wq_i = to_bits(Xi), to_bits(Wi)
        sx = sw = None
    exp = so.epilogue(so.gemm_exact(Xq_i, Wq_i, dtype), sx, sw, dtype)
    Wq_t = to_dev_q(Wq_i, dtype)
    w_vals, w_meta = binding.slide_decompose(Wq_t, N, dtype)
    XL_t = to_dev_q(so.lift(Xq_i, N), dtype)
    sxd = None if sx is None else dev(sx)
    swd = None if sw is None else dev(sw)
    Ys = binding.slide_sparse_gemm(XL_t, sxd, w_vals, w_meta, swd, O, dtype)
    assert np.array_equal(bits16(Ys), exp)
    Yd = binding.dense_gemm(to_dev_q(Xq_i, dtype), sxd, Wq_t, swd, dtype)
    assert np.array_equal(bits16(Yd), exp)


# ------------------------------------------------------------------ kernel selection boundaries
@pytest.mark.parametrize("M,O", [(32, 128), (33, 160), (64, 8192), (65, 8192), (65, 128 * 320), (65, 128 * 321), (128, 512), (129, 512),
                                 (128, 128 * 320), (129, 128 * 161), (256, 128 * 160), (257, 128 * 107)])
def test_gemm_kernel_selection_boundaries_int8(M, O):
    """Shapes around the switches between the few-token kernels (M <= 64), the 128 x 128-tile kernels (up to 320
    such tiles) and the 256 x 256 tile kernels: the result must not depend on which one runs."""
    N, K = 4, 256
    rng = np.random.default_rng(M * 7 + O)
    Wq = rng.integers(-127, 128, size=(O, K)).astype(np.int8)
    keep = np.argsort(rng.random((O, K // 8, 8)), axis=-1) < 6
    Wq = (Wq.reshape(O, K // 8, 8) * keep).reshape(O, K).astype(np.int8)
    Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    s_x = rng.uniform(0.01, 0.1, M).astype(np.float32)
    s_w = rng.uniform(1e-4, 1e-3, O).astype(np.float32)
    exp = so.epilogue(_acc_big(Xq, Wq), s_x, s_w, "i8")
    w_vals, w_meta = binding.slide_decompose(dev(Wq), N, "i8")
    Ys = binding.slide_sparse_gemm(dev(so.lift(Xq, N)), dev(s_x), w_vals, w_meta, dev(s_w), O, "i8")
    assert np.array_equal(bits16(Ys), exp)
    Yd = binding.dense_gemm(dev(Xq), dev(s_x), dev(Wq), dev(s_w), "i8")
    assert np.array_equal(bits16(Yd), exp)


# ------------------------------------------------------------------ split k range with a caller-owned workspace
def _workspace(M, O, Kp, dtype, fill, scale=1.0):
    need = binding.slide_gemm_workspace_bytes(M, O, Kp, dtype)
    n = max(16, int(need * scale) // 16 * 16)
    return need, torch.full((n,), fill, dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("dtype", ["i8", "fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,M,O,K", [(4, 100, 384, 2048),       # 3 tiles of 128 x 128, K' = 3072: 24 units
                                     (4, 48, 200, 8192),        # 32 < M <= 64 with long rows
                                     (3, 300, 130, 3072),       # ragged tokens and channels, K' = 4096
                                     (2, 129, 257, 4096),       # native 2:4
                                     (5, 64, 128, 10240),       # K' = 16384
                                     (5, 16, 200, 10240),       # few-token kernels, k range split in two
                                     (4, 24, 130, 16384)])      # ... in three (K' = 24576)
def test_gemm_split_k_with_workspace(dtype, N, M, O, K):
    """The 128 x 128-tile kernels (and, for few tokens on long rows, the few-token kernels) with the k range split
    over several workgroups: partial sums go through the caller's workspace and are added in a fixed order.  INT8 must equal the oracle bit for bit (and
    so the call without workspace); floats stay within the GEMM tolerance and are reproducible bit for bit."""
    X = synth.activations(M, K, seed=M + K, n_outliers=2)
    W = synth.weights(O, K, seed=O + N)
    ref = so.linear_reference(X, W, N, dtype)
    Xd, Wd = dev(X), dev(W)
    Wq, s_w = binding.slide_prune_quant(Wd, N, dtype)
    w_vals, w_meta = binding.slide_decompose(Wq, N, dtype)
    XL, s_x = binding.act_lift_quant(Xd, N, dtype)
    Xq, s_x2 = binding.act_lift_quant(Xd, 2, dtype)
    need, ws = _workspace(M, O, XL.shape[1], dtype, fill=0xFF)             # 0xFF..: NaN patterns, contents must not matter
    assert need > 0, "shape chosen so that the k range is split"
    Ys = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype, workspace=ws)
    need_d, ws_d = _workspace(M, O, K, dtype, fill=0x7F)
    Yd = binding.dense_gemm(Xq, s_x2, Wq, s_w, dtype, workspace=ws_d)
    if dtype == "i8":
        assert np.array_equal(bits16(Ys), ref["Y"]) and np.array_equal(bits16(Yd), ref["Y"])
        assert torch.equal(Ys, binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype))
    else:
        _float_gemm_check(bits16(Ys), ref, dtype)
        _float_gemm_check(bits16(Yd), ref, dtype)
    # same bits on a second run over the used workspace, and with a workspace that only holds fewer ranges
    assert torch.equal(Ys, binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype, workspace=ws))
    assert torch.equal(Yd, binding.dense_gemm(Xq, s_x2, Wq, s_w, dtype, workspace=ws_d))
    _, small = _workspace(M, O, XL.shape[1], dtype, fill=0x11, scale=0.6)
    Y2 = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype, workspace=small)
    if dtype == "i8":
        assert torch.equal(Y2, Ys)
    else:
        _float_gemm_check(bits16(Y2), ref, dtype)
    tiny = torch.zeros((16,), dtype=torch.uint8, device=DEV)                # too small for any split: plain path
    Y3 = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype, workspace=tiny)
    assert torch.equal(Y3, binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype))


# ------------------------------------------------------------------ seeded random shapes
def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        N = int(rng.integers(2, 9))
        K = 128 * N * int(rng.integers(1, 3))                # K and K' = 256 (N-1) r are whole numbers of 128-byte units
        M = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 256, 257, 300, 511]))
        O = int(rng.choice([1, 31, 32, 33, 127, 128, 129, 255, 256, 257, 384, 513, 700]))
        cases.append((N, M, O, K))
    return cases


def _ragged_k_cases(n, seed):
    """K neither a multiple of 2N nor of the 128-byte unit (last block completed with zeros, Alg. 1's
    n_g = ceil(K / 2N); lifted rows padded to whole units), plus two layer shapes of that kind."""
    rng = np.random.default_rng(seed)
    cases = [(3, 64, 96, 3584), (5, 130, 160, 6912)]        # 4:6 on a 3584-wide layer, 8:10 on a 6912-wide one
    for _ in range(n):
        N = int(rng.integers(2, 9))
        K = int(rng.integers(2, 1500))
        M = int(rng.choice([1, 17, 64, 65, 128, 129, 300]))
        O = int(rng.choice([1, 33, 128, 257, 513]))
        cases.append((N, M, O, K))
    return cases


@pytest.mark.parametrize("N,M,O,K", _random_cases(24, seed=2024) + _ragged_k_cases(14, seed=31))
def test_random_shapes_int8_end_to_end(N, M, O, K):
    """The whole path on ragged shapes around every tile, fragment and token-block boundary, for every
    pattern N = 2..8: prune + quantise, decompose, lift + quantise, sparse GEMM, dense GEMM; all bit-exact."""
    X = synth.activations(M, K, seed=M + O + K, n_outliers=2)
    W = synth.weights(O, K, seed=M + O + N)
    ref = so.linear_reference(X, W, N, "i8")
    Xd, Wd = dev(X), dev(W)
    Wq, s_w = binding.slide_prune_quant(Wd, N, "i8")
    assert np.array_equal(host(Wq), ref["Wq"]) and np.array_equal(host(s_w), ref["s_w"])
    w_vals, w_meta, viol = binding.slide_decompose(Wq, N, "i8", count_violations=True)
    XL, s_x = binding.act_lift_quant(Xd, N, "i8")
    check_lifted(XL, so.lift(ref["Xq"], N), "i8")
    assert np.array_equal(host(s_x), ref["s_x"])
    Y = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, "i8")
    assert int(host(viol)[0]) == 0
    assert np.array_equal(bits16(Y), ref["Y"])
    if K % 128 == 0:                                         # the dense baseline wants whole 128-byte rows
        Xq, s_x2 = binding.act_lift_quant(Xd, 2, "i8")
        Yd = binding.dense_gemm(Xq, s_x2, Wq, s_w, "i8")
        assert np.array_equal(bits16(Yd), ref["Y"])


@pytest.mark.parametrize("dtype", ["fp8", "bf16", "fp16"])
@pytest.mark.parametrize("N,M,O,K", _random_cases(8, seed=77) + _ragged_k_cases(6, seed=32) +
                         [(4, 1100, 2100, 103)])         # short rows, many outputs that cancel to ~0: tightest for the derived bound
def test_random_shapes_float_end_to_end(dtype, N, M, O, K):
    X = synth.activations(M, K, seed=M + O + K, n_outliers=2)
    W = synth.weights(O, K, seed=M + O + N)
    ref = so.linear_reference(X, W, N, dtype)
    Xd, Wd = dev(X), dev(W)
    Wq, s_w = binding.slide_prune_quant(Wd, N, dtype)
    assert np.array_equal(from_dev_q(Wq, dtype), ref["Wq"])
    w_vals, w_meta = binding.slide_decompose(Wq, N, dtype)
    XL, s_x = binding.act_lift_quant(Xd, N, dtype)
    check_lifted(XL, so.lift(ref["Xq"], N), dtype)
    _float_gemm_check(bits16(binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, dtype)), ref, dtype)
    if K * XL.element_size() % 128 == 0:
        Xq, s_x2 = binding.act_lift_quant(Xd, 2, dtype)
        _float_gemm_check(bits16(binding.dense_gemm(Xq, s_x2, Wq, s_w, dtype)), ref, dtype)


# ------------------------------------------------------------------ capture into a HIP graph
@pytest.mark.parametrize("M,use_ws", [(16, False), (128, True)])
def test_hip_graph_replay(M, use_ws):
    """The per-call path (lift + quantise, sparse GEMM; with M = 128 the split-k kernels and their reduction) records
    into a HIP graph: the library allocates nothing and never synchronises.  Every replay is checked against the
    oracle, with new activations written into the captured input buffer between replays."""
    N, K, O = 4, 2048, 640
    W = synth.weights(O, K, seed=3)
    Wq, s_w = binding.slide_prune_quant(dev(W), N, "i8")
    w_vals, w_meta = binding.slide_decompose(Wq, N, "i8")
    Xs = [synth.activations(M, K, seed=50 + i, n_outliers=2) for i in range(3)]
    x_in = dev(Xs[0]).clone()
    XL, s_x = binding.act_lift_quant(x_in, N, "i8")              # warm-up outside the capture (first-use set-up)
    Y = torch.empty((M, O), dtype=torch.bfloat16, device=DEV)
    ws = None
    if use_ws:
        n = binding.slide_gemm_workspace_bytes(M, O, XL.shape[1], "i8")
        assert n > 0
        ws = torch.empty((n,), dtype=torch.uint8, device=DEV)
    binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, "i8", out=Y, workspace=ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.act_lift_quant(x_in, N, "i8", out=XL, s_x=s_x)
        binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, "i8", out=Y, workspace=ws)
    for i in (1, 2, 0, 2):
        x_in.copy_(dev(Xs[i]))
        Y.fill_(7.0)                                             # eager work between the replays
        g.replay()
        ref = so.linear_reference(Xs[i], W, N, "i8")
        assert np.array_equal(bits16(Y), ref["Y"]), f"replay with input {i}"


# ------------------------------------------------------------------ the fp8 accumulation model behind the tolerance
@pytest.mark.parametrize("kernel", ["dense", "sparse"])
def test_fp8_products_keep_14_bits_below_the_largest_of_their_group(kernel):
    """The extra 2^-9 ||x|| ||w|| the FP8 tolerance allows rests on how the fp8 matrix instructions of gfx950 add an
    instruction's products: aligned to the largest product of a small group, 14 bits kept below it.  One token, one
    instruction's worth of k: products +256 and -256 (they cancel exactly) next to 22 products of 2^e.  With e >= -5
    the small products survive whole and the result is exact; from e = -6 down they are cut off (seen on the dense
    instruction; the sparse one must at least not exceed the exact sum); bf16 products keep all 24 bits.  Every case stays inside the bound the parity tests use."""
    N, M, O, K = 4, 1, 128, 256
    cols = [c for c in range(2, 32) if c % 8 < 6]                # a 6:8-compliant support inside one instruction's k range (lifted too)
    def run(dtype, e):
        x = np.zeros((M, K), np.float32)
        w = np.zeros((O, K), np.float32)
        x[:, 0], x[:, 1] = 16.0, -16.0
        x[:, cols] = 2.0 ** (e // 2)
        w[:, [0, 1]] = 16.0
        w[:, cols] = 2.0 ** (e - e // 2)
        if dtype == "fp8":
            xq, wq = so.fp8_e4m3_encode(x), so.fp8_e4m3_encode(w)
            sx, sw = dev(np.ones(M, np.float32)), dev(np.ones(O, np.float32))
        else:
            xq, wq = so.bf16_bits(x), so.bf16_bits(w)
            sx = sw = None
        assert np.array_equal(so.to_real(xq, dtype), x) and np.array_equal(so.to_real(wq, dtype), w)   # all values exact in the format
        if kernel == "dense":
            Y = binding.dense_gemm(to_dev_q(xq, dtype), sx, to_dev_q(wq, dtype), sw, dtype)
        else:
            w_vals, w_meta = binding.slide_decompose(to_dev_q(wq, dtype), N, dtype)
            Y = binding.slide_sparse_gemm(to_dev_q(so.lift(xq, N), dtype), sx, w_vals, w_meta, sw, O, dtype)
        got = so.bf16_to_f32(bits16(Y)).astype(np.float64)
        assert np.all(got == got[0, 0])
        return float(got[0, 0]), len(cols) * 2.0 ** e, float(np.linalg.norm(x) * np.linalg.norm(w[0]))
    for e in (-2, -4, -5):
        got, exact, _ = run("fp8", e)
        assert got == exact, (e, got, exact)
    for e in (-6, -8):
        got, exact, norm = run("fp8", e)
        assert got < exact if kernel == "dense" else got <= exact, (e, got, exact)     # cut off below 2^8 x 2^-14 = 2^-6 ...
        assert abs(got - exact) <= 2.0 ** -9 * norm              # ... and inside the allowance
    for e in (-6, -10, -14):
        got, exact, _ = run("bf16", e)
        assert got == exact, (e, got, exact)
