"""Transformer-block driver for the Llama-3-8B-shaped configuration (model mode of the paper's kernel benchmarks, Sec. 5 /
App. D.3: the latencies of Wqkv, Wo, W13 and W2 summed): the four linear layers run through the library, chained through
plain torch reference ops (RMSNorm, grouped-query causal attention, SiLU gating, residuals) that are not timed.

Only the linear layers are the method; every one of them is: per-token quantisation (act_lift_quant), then
  "fused"  slide_sparse_gemm_fused on the unlifted activations (lifting inside the GEMM), or
  "lifted" act_lift_quant with N = 4 + slide_sparse_gemm, or
  "dense"  dense_gemm at the original K (the speed-up denominator).
Weights are random-init (synth.weights), magnitude-pruned 6:8 and quantised by the library."""
from __future__ import annotations

import torch

from . import binding, synth

HIDDEN, N_Q_HEADS, N_KV_HEADS, HEAD_DIM, MLP = 4096, 32, 8, 128, 14336
N = 4


class Linear:
    def __init__(self, name: str, K: int, O: int, seed: int, dev):
        self.name, self.K, self.O, self.seed = name, K, O, seed
        W = torch.from_numpy(synth.weights(O, K, seed)).to(dev)
        self.Wq, self.s_w = binding.slide_prune_quant(W, N, "i8")
        self.w_vals, self.w_meta = binding.slide_decompose(self.Wq, N, "i8")
        self.fw_vals, self.fw_meta = binding.slide_decompose_fused(self.Wq, N, "i8")

    def __call__(self, x: torch.Tensor, path: str, timer=None):
        """x[M, K] bf16 -> y[M, O] bf16; timer(name, stage) is called around the two kernels if given."""
        mark = (lambda stage: timer(self.name, stage)) if timer else (lambda stage: None)
        mark("start")
        if path == "lifted":
            xq, s_x = binding.act_lift_quant(x, N, "i8")
            mark("quantised")
            y = binding.slide_sparse_gemm(xq, s_x, self.w_vals, self.w_meta, self.s_w, self.O, "i8")
        else:
            xq, s_x = binding.act_lift_quant(x, 2, "i8")
            mark("quantised")
            if path == "fused":
                y = binding.slide_sparse_gemm_fused(xq, s_x, self.fw_vals, self.fw_meta, self.s_w, self.O, self.K, N, "i8")
            elif path == "dense":
                y = binding.dense_gemm(xq, s_x, self.Wq, self.s_w, "i8")
            else:
                raise ValueError(path)
        mark("done")
        return y


def rms_norm(x: torch.Tensor, eps: float = 1e-5) -> torch.Tensor:
    xf = x.float()
    return (xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + eps)).to(torch.bfloat16)


class LlamaBlock:
    """One block; `layers` follows synth.LLAMA3_8B (qkv, o, gate_up, down)."""

    def __init__(self, dev, seed: int = 0):
        self.dev = dev
        self.lin = {name: Linear(name, K, O, seed + i, dev) for i, (name, K, O) in enumerate(synth.LLAMA3_8B)}

    def forward(self, x: torch.Tensor, path: str = "fused", timer=None, record=None):
        """x[M, HIDDEN] bf16, one causal sequence of M tokens.  record: dict that receives (input, output) per linear."""
        M = x.shape[0]

        def run(name, inp):
            inp = inp.contiguous()
            out = self.lin[name](inp, path, timer)
            if record is not None:
                record[name] = (inp, out)
            return out

        qkv = run("qkv", rms_norm(x))
        q, k, v = qkv.split([N_Q_HEADS * HEAD_DIM, N_KV_HEADS * HEAD_DIM, N_KV_HEADS * HEAD_DIM], dim=1)
        q = q.view(M, N_Q_HEADS, HEAD_DIM).transpose(0, 1).unsqueeze(0)
        k = k.view(M, N_KV_HEADS, HEAD_DIM).transpose(0, 1).unsqueeze(0)
        v = v.view(M, N_KV_HEADS, HEAD_DIM).transpose(0, 1).unsqueeze(0)
        a = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
        a = a.squeeze(0).transpose(0, 1).reshape(M, N_Q_HEADS * HEAD_DIM)
        x = x + run("o", a)
        gate, up = run("gate_up", rms_norm(x)).split([MLP, MLP], dim=1)
        act = (torch.nn.functional.silu(gate.float()) * up.float()).to(torch.bfloat16)
        return x + run("down", act)
