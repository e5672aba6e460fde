"""GPU parity of the fused-lifting path (slide_decompose_fused + slide_sparse_gemm_fused, 6:8 only): the GEMM takes the
unlifted quantised activations and must give the oracle's linear layer, bit-exact for INT8."""
import numpy as np
import pytest
import torch

from oracle import slide_oracle as so
from oracle import gemm_ref
from paper_2603_05232_amd import binding, synth
from test_gpu_parity import dev, host, bits16, to_dev_q, from_dev_q, _float_gemm_check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N = 4


@pytest.mark.parametrize("M,O,K", [(16, 512, 512),         # the anchor case
                                   (300, 640, 1024),       # ragged tokens and channels
                                   (1, 384, 128),          # one token, one super-unit
                                   (257, 130, 256),        # two super-units, one ragged panel
                                   (64, 256, 384),         # three super-units (no steady iteration)
                                   (40, 128, 512),         # four: one steady iteration
                                   (513, 300, 896)])       # seven, three token tiles
def test_fused_gemm_int8(M, O, K):
    X = synth.activations(M, K, seed=M + O)
    W = synth.weights(O, K, seed=M + O)
    ref = so.linear_reference(X, W, N, "i8")
    Wq, s_w = binding.slide_prune_quant(dev(W), N, "i8")
    w_vals, w_meta, viol = binding.slide_decompose_fused(Wq, N, "i8", count_violations=True)
    Xq, s_x = binding.act_lift_quant(dev(X), 2, "i8")          # plain per-token quantisation: K bytes per token
    assert np.array_equal(host(Xq)[:, :K], ref["Xq"])
    Y = binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, "i8")
    assert int(host(viol)[0]) == 0
    assert np.array_equal(bits16(Y), ref["Y"])


# shapes that take the few-token kernels (M <= 64: one and two token blocks, single fragments, whole panels, eight
# wavefronts) and the 128 x 128-tile kernels, with and without a workspace (k range split through it)
SMALL = [(1, 384, 128), (1, 4608, 3584), (7, 640, 1024), (16, 37888 // 8, 512), (32, 130, 2048), (33, 3584, 1024), (64, 260, 18944 // 2),
         (16, 3584, 18944), (64, 3584, 18944), (65, 512, 512), (100, 256, 128), (129, 300, 256), (70, 130, 384), (128, 4608, 3584), (200, 700, 1152), (256, 3584, 4736), (1024, 1100, 640)]


@pytest.mark.parametrize("with_ws", [False, True])
@pytest.mark.parametrize("M,O,K", SMALL)
def test_fused_gemm_small_and_mid_int8(M, O, K, with_ws):
    rng = np.random.default_rng(M * 7 + O)
    Wq = rng.integers(-127, 128, size=(O, K)).astype(np.int8)
    keep = np.argsort(rng.random((O, K // 8, 8)), axis=-1) < rng.integers(0, 7, size=(O, K // 8, 1))
    Wq = (Wq.reshape(O, K // 8, 8) * keep).reshape(O, K).astype(np.int8)
    Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    s_x = rng.uniform(0.01, 0.1, M).astype(np.float32)
    s_w = rng.uniform(1e-4, 1e-3, O).astype(np.float32)
    exp = so.epilogue(gemm_ref.gemm_i8_i64(Xq, Wq), s_x, s_w, "i8")
    w_vals, w_meta = binding.slide_decompose_fused(dev(Wq), N, "i8")
    ws = None
    if with_ws:
        nbytes = binding.slide_gemm_workspace_bytes(M, O, K, "i8")
        ws = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=DEV)
    Y = binding.slide_sparse_gemm_fused(dev(Xq), dev(s_x), w_vals, w_meta, dev(s_w), O, K, N, "i8", workspace=ws)
    assert np.array_equal(bits16(Y), exp)


@pytest.mark.parametrize("dtype", ["fp8", "bf16", "fp16"])
@pytest.mark.parametrize("M,O,K", [(1, 640, 1024), (16, 3584, 4096), (48, 260, 2048), (128, 1100, 1152), (300, 256, 8192)])
def test_fused_gemm_small_and_mid_float(dtype, M, O, K):
    X = synth.activations(M, K, seed=M + O)
    W = synth.weights(O, K, seed=M + O)
    ref = so.linear_reference(X, W, N, dtype)
    Wq, s_w = binding.slide_prune_quant(dev(W), N, dtype)
    w_vals, w_meta = binding.slide_decompose_fused(Wq, N, dtype)
    Xq, s_x = binding.act_lift_quant(dev(X), 2, dtype)
    nbytes = binding.slide_gemm_workspace_bytes(M, O, K, dtype)
    ws = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=DEV)
    for w in (None, ws):
        Y = binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, dtype, workspace=w)
        _float_gemm_check(bits16(Y), ref, dtype)


def test_fused_gemm_two_rounds_full_output_and_strides():
    """More tiles than compute units (17 x 18 = 306 tiles of 256 x 256: two persistent rounds), ragged edges, random
    sparse supports (windows with 0, 1 and 2 stored values), strided X and Y; every output element against the C oracle."""
    rng = np.random.default_rng(5)
    M, O, K = 4300, 4400, 256
    Wq = rng.integers(-127, 128, size=(O, K)).astype(np.int8)
    keep = np.argsort(rng.random((O, K // 8, 8)), axis=-1) < rng.integers(0, 7, size=(O, K // 8, 1))
    Wq = (Wq.reshape(O, K // 8, 8) * keep).reshape(O, K).astype(np.int8)
    Xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    s_x = rng.uniform(0.01, 0.1, M).astype(np.float32)
    s_w = rng.uniform(1e-4, 1e-3, O).astype(np.float32)
    exp = so.epilogue(gemm_ref.gemm_i8_i64(Xq, Wq), s_x, s_w, "i8")
    w_vals, w_meta = binding.slide_decompose_fused(dev(Wq), N, "i8")
    xbuf = torch.zeros((M, K + 128), dtype=torch.int8, device=DEV)
    xbuf[:, :K] = dev(Xq)
    ybuf = torch.full((M, O + 64), -1.0, dtype=torch.bfloat16, device=DEV)
    binding.slide_sparse_gemm_fused(xbuf, dev(s_x), w_vals, w_meta, dev(s_w), O, K, N, "i8", out=ybuf[:, :O])
    assert np.array_equal(bits16(ybuf[:, :O].contiguous()), exp)
    assert torch.all(ybuf[:, O:] == -1.0)


@pytest.mark.parametrize("dtype", ["fp8", "bf16", "fp16"])
@pytest.mark.parametrize("M,O,K", [(16, 512, 512), (300, 640, 1024), (257, 130, 256)])
def test_fused_gemm_float(dtype, M, O, K):
    X = synth.activations(M, K, seed=M + O)
    W = synth.weights(O, K, seed=M + O)
    if M > 2:
        X[1] = 0.0
    ref = so.linear_reference(X, W, N, dtype)
    Wq, s_w = binding.slide_prune_quant(dev(W), N, dtype)
    w_vals, w_meta = binding.slide_decompose_fused(Wq, N, dtype)
    Xq, s_x = binding.act_lift_quant(dev(X), 2, dtype)
    Y = binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, dtype)
    _float_gemm_check(bits16(Y), ref, dtype)
    # small integers: every product and partial sum is exact, so the result must be the rounded exact one
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
    w_vals, w_meta = binding.slide_decompose_fused(to_dev_q(Wq_i, dtype), N, dtype)
    sxd = None if sx is None else dev(sx)
    swd = None if sw is None else dev(sw)
    Ys = binding.slide_sparse_gemm_fused(to_dev_q(Xq_i, dtype), sxd, w_vals, w_meta, swd, O, K, N, dtype)
    assert np.array_equal(bits16(Ys), exp)


def test_fused_rejects_other_patterns_and_ragged_k():
    Wq = torch.zeros((128, 256), dtype=torch.int8, device=DEV)
    with pytest.raises(binding.SlideSparseError) as e:
        binding.slide_decompose_fused(Wq, 3, "i8")
    assert e.value.code == 2
    w_vals, w_meta = binding.slide_decompose_fused(Wq, 4, "i8")
    Xq = torch.zeros((4, 256), dtype=torch.int8, device=DEV)
    s = torch.ones((128,), dtype=torch.float32, device=DEV)
    with pytest.raises(binding.SlideSparseError) as e:
        binding.slide_sparse_gemm_fused(Xq, s[:4], w_vals, w_meta, s, 128, 200, 4, "i8")     # K * es not a multiple of 128
    assert e.value.code == 3


def _random_fused_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 256, 257, 300, 511, 700]))
        O = int(rng.choice([1, 31, 32, 33, 127, 128, 129, 255, 256, 257, 384, 513, 700, 1300]))
        K = 128 * int(rng.integers(1, 20))
        out.append((M, O, K, bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("M,O,K,with_ws", _random_fused_cases(28, seed=606))
def test_fused_random_shapes_int8_end_to_end(M, O, K, with_ws):
    """The fused path from fp32 inputs on shapes around every token-block, fragment, tile and kernel-family boundary:
    prune + quantise, fused packing, quantisation, fused GEMM; bit-exact against the oracle's linear layer."""
    X = synth.activations(M, K, seed=M + O + K, n_outliers=2)
    W = synth.weights(O, K, seed=M + O)
    ref = so.linear_reference(X, W, N, "i8")
    Wq, s_w = binding.slide_prune_quant(dev(W), N, "i8")
    w_vals, w_meta = binding.slide_decompose_fused(Wq, N, "i8")
    Xq, s_x = binding.act_lift_quant(dev(X), 2, "i8")
    ws = None
    if with_ws:
        ws = torch.empty((max(binding.slide_gemm_workspace_bytes(M, O, K, "i8"), 16),), dtype=torch.uint8, device=DEV)
    Y = binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, "i8", workspace=ws)
    assert np.array_equal(bits16(Y), ref["Y"])


@pytest.mark.parametrize("dtype", ["fp8", "bf16", "fp16"])
@pytest.mark.parametrize("M,O,K,with_ws", _random_fused_cases(8, seed=909))
def test_fused_random_shapes_float_end_to_end(dtype, M, O, K, with_ws):
    es = 1 if dtype == "fp8" else 2
    K = K if (K * es) % 128 == 0 else K + 64
    X = synth.activations(M, K, seed=M + O + K, n_outliers=2)
    W = synth.weights(O, K, seed=M + O)
    ref = so.linear_reference(X, W, N, dtype)
    Wq, s_w = binding.slide_prune_quant(dev(W), N, dtype)
    w_vals, w_meta = binding.slide_decompose_fused(Wq, N, dtype)
    Xq, s_x = binding.act_lift_quant(dev(X), 2, dtype)
    ws = None
    if with_ws:
        ws = torch.empty((max(binding.slide_gemm_workspace_bytes(M, O, K, dtype), 16),), dtype=torch.uint8, device=DEV)
    Y = binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, dtype, workspace=ws)
    _float_gemm_check(bits16(Y), ref, dtype)


@pytest.mark.parametrize("M", [16, 128, 600])
def test_fused_hip_graph_replay(M):
    """Quantisation + fused GEMM (few-token kernel; 128 x 128 tiles with split k and their reduction; persistent tiles)
    recorded into a HIP graph: nothing is allocated and nothing synchronises.  Every replay is checked against the oracle,
    with new activations written into the captured input buffer between replays."""
    K, O = 2048, 640
    W = synth.weights(O, K, seed=3)
    Wq, s_w = binding.slide_prune_quant(dev(W), N, "i8")
    w_vals, w_meta = binding.slide_decompose_fused(Wq, N, "i8")
    Xs = [synth.activations(M, K, seed=50 + i, n_outliers=2) for i in range(3)]
    x_in = dev(Xs[0]).clone()
    Xq, s_x = binding.act_lift_quant(x_in, 2, "i8")              # warm-up outside the capture (first-use set-up)
    Y = torch.empty((M, O), dtype=torch.bfloat16, device=DEV)
    n = binding.slide_gemm_workspace_bytes(M, O, K, "i8")
    ws = torch.empty((max(n, 16),), dtype=torch.uint8, device=DEV)
    binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, "i8", out=Y, workspace=ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.act_lift_quant(x_in, 2, "i8", out=Xq, s_x=s_x)
        binding.slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O, K, N, "i8", out=Y, workspace=ws)
    for i in (1, 2, 0, 1):
        x_in.copy_(dev(Xs[i]))
        Y.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits16(Y), so.linear_reference(Xs[i], W, N, "i8")["Y"])
