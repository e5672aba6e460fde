"""The Llama-3-8B-shaped block forward (M = 4096, 6:8 INT8): every linear of the chained run is checked against the
oracle on the activations that linear actually received (sampled tokens x channels, whole rows of K), for the fused,
the lifted and the dense path.  Attention / RMSNorm / gating are torch reference ops and need no oracle."""
import numpy as np
import pytest
import torch

from oracle import slide_oracle as so
from paper_2603_05232_amd import synth
from paper_2603_05232_amd.block import LlamaBlock, HIDDEN
from test_gpu_parity import bits16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def block():
    return LlamaBlock(torch.device(DEV))


@pytest.mark.parametrize("path", ["fused", "lifted", "dense"])
def test_block_linears_against_oracle(block, path):
    M = 4096
    x = torch.from_numpy(synth.activations(M, HIDDEN, seed=5)).to(DEV).to(torch.bfloat16)
    rec = {}
    y = block.forward(x, path, record=rec)
    assert y.shape == (M, HIDDEN) and bool(torch.isfinite(y.float()).all())
    rng = np.random.default_rng(17)
    for i, (name, K, O) in enumerate(synth.LLAMA3_8B):
        inp, out = rec[name]
        assert inp.shape == (M, K) and out.shape == (M, O)
        rows = np.sort(rng.choice(M, size=48, replace=False)); rows[-1] = M - 1
        cols = np.sort(rng.choice(O, size=64, replace=False)); cols[-1] = O - 1
        ri, ci = torch.from_numpy(rows).to(DEV), torch.from_numpy(cols).to(DEV)
        Xs = inp[ri].float().cpu().numpy()                       # bf16 activations are exact in fp32
        ref = so.linear_reference(Xs, synth.weights(O, K, block.lin[name].seed)[cols], 4, "i8")
        assert np.array_equal(bits16(out[ri][:, ci].contiguous()), ref["Y"]), name
