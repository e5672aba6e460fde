"""slide_sparse_gemm_static (scratch in a static device array, nothing allocated) against slide_sparse_gemm_ws on the
same inputs: calls in a row, the later ones on smaller inputs, all bit for bit.  (Named to be collected last.)"""
import pytest
import torch

from paper_2603_05232_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(M, O, K, N, seed):
    X = torch.from_numpy(synth.activations(M, K, seed=seed)).to(DEV)
    W = torch.from_numpy(synth.weights(O, K, seed=seed)).to(DEV)
    Wq, s_w = binding.slide_prune_quant(W, N, "i8")
    w_vals, w_meta = binding.slide_decompose(Wq, N, "i8")
    XL, s_x = binding.act_lift_quant(X, N, "i8")
    n = binding.slide_gemm_workspace_bytes(M, O, XL.shape[1], "i8")
    assert 0 < n <= binding.slide_static_scratch_bytes(), "the case must split its k range"
    ws = torch.empty((n,), dtype=torch.uint8, device=DEV)
    Y_ws = binding.slide_sparse_gemm(XL, s_x, w_vals, w_meta, s_w, O, "i8", workspace=ws)
    Y_st = torch.full((M, O), -1.0, dtype=torch.bfloat16, device=DEV)
    binding.slide_sparse_gemm_static(XL, s_x, w_vals, w_meta, s_w, O, "i8", out=Y_st)
    torch.cuda.synchronize()
    assert torch.equal(Y_st.view(torch.int16), Y_ws.view(torch.int16))


def test_static_scratch_matches_workspace_call_twice():
    assert binding.slide_static_scratch_bytes() == 16 << 20
    _case(300, 640, 2048, 4, seed=1)        # 15 tiles of 128 x 128, k range split
    _case(130, 384, 2048, 4, seed=2)        # smaller: reuses the start of the same scratch array
    _case(16, 3584, 18944, 4, seed=3)       # few-token kernels with split k (long rows)


def test_static_scratch_rejects_bad_arguments():
    Y = torch.empty((4, 128), dtype=torch.bfloat16, device=DEV)
    x = torch.zeros((4, 100), dtype=torch.int8, device=DEV)
    s = torch.ones((128,), dtype=torch.float32, device=DEV)
    with pytest.raises(binding.SlideSparseError) as e:
        binding.slide_sparse_gemm_static(x, s[:4], x, x, s, 128, "i8", out=Y)      # K' not a multiple of 128
    assert e.value.code == 3
