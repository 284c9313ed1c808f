"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds input recipes only: random draws, outlier channels and the
cast to bf16.  None of the quantization method's arithmetic lives here, so
both the CPU oracle's callers and the HIP path's callers may use it.

The tensors stand in for the LLM activations and weights the paper profiles
(Section 3.1, block-level profiling): a Gaussian-like bulk, block maxima that
spread over a binade, and channel-wise outliers (a few columns of an
activation matrix scaled up for every token).  Shapes are LLaMA-3-8B /
LLaMA-2-7B layer shapes.  Values are drawn in fp32 on the CPU with a fixed
seed and rounded to bf16 once; the same bf16 bits feed both sides.
"""
import numpy as np
import torch


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def gaussian(rows, cols, std=1.0, seed=0):
    """bf16 [rows, cols], N(0, std^2)."""
    x = torch.randn(rows, cols, generator=_gen(seed), dtype=torch.float32) * std
    return x.to(torch.bfloat16)


def gaussian_outlier_channels(rows, cols, n_outlier, factor, std=1.0, seed=0):
    """bf16 [rows, cols], N(0, std^2) with n_outlier columns (a seeded random
    choice, the same for every row) multiplied by factor."""
    g = _gen(seed)
    x = torch.randn(rows, cols, generator=g, dtype=torch.float32) * std
    ch = torch.randperm(cols, generator=g)[:n_outlier]
    x[:, ch] *= factor
    return x.to(torch.bfloat16)


def student_t(rows, cols, df=3.0, seed=0):
    """bf16 [rows, cols], heavy-tailed Student-t(df)."""
    x = np.random.default_rng(int(seed)).standard_t(df, size=(rows, cols)).astype(np.float32)
    return torch.from_numpy(x).to(torch.bfloat16)


def softmax_rows(rows, cols, seed=0):
    """bf16 [rows, cols]: softmax over the last dim of N(0,1) logits (attention
    probabilities, computed in fp32)."""
    z = torch.randn(rows, cols, generator=_gen(seed), dtype=torch.float32)
    return torch.softmax(z, dim=-1).to(torch.bfloat16)


def single_linear(seed=0, M=32, K=4096, N=4096):
    """Small parity case: A [M,K] ~N(0,1) with 8 outlier channels x30,
    W [N,K] ~N(0, 0.02^2)."""
    a = gaussian_outlier_channels(M, K, 8, 30.0, 1.0, seed)
    w = gaussian(N, K, 0.02, seed + 1000)
    return a, w


def llama3_8b_mlp(seed=2, M=2048, hidden=4096, inter=14336):
    """LLaMA-3-8B MLP prefill operands.  Activations have 0.5 % outlier
    channels x50; weights ~N(0, 0.02^2).  Returns a dict of bf16 tensors:
    x [M,hidden], w_gate/w_up [inter,hidden], h [M,inter], w_down [hidden,inter]."""
    return {
        "x": gaussian_outlier_channels(M, hidden, round(0.005 * hidden), 50.0, 1.0, seed),
        "w_gate": gaussian(inter, hidden, 0.02, seed + 1),
        "w_up": gaussian(inter, hidden, 0.02, seed + 2),
        "h": gaussian_outlier_channels(M, inter, round(0.005 * inter), 50.0, 1.0, seed + 3),
        "w_down": gaussian(hidden, inter, 0.02, seed + 4),
    }


def llama2_7b_linears(seed=4, M=4096, hidden=4096, inter=11008):
    """LLaMA-2-7B decoder linear operands at M tokens (same recipe as the MLP
    case).  w_qkv [3*hidden,hidden], w_o [hidden,hidden], w_gate/w_up
    [inter,hidden], w_down [hidden,inter]."""
    return {
        "x": gaussian_outlier_channels(M, hidden, round(0.005 * hidden), 50.0, 1.0, seed),
        "w_qkv": gaussian(3 * hidden, hidden, 0.02, seed + 1),
        "w_o": gaussian(hidden, hidden, 0.02, seed + 2),
        "w_gate": gaussian(inter, hidden, 0.02, seed + 3),
        "w_up": gaussian(inter, hidden, 0.02, seed + 4),
        "h": gaussian_outlier_channels(M, inter, round(0.005 * inter), 50.0, 1.0, seed + 5),
        "w_down": gaussian(hidden, inter, 0.02, seed + 6),
    }


def quantizer_streams(seed=3):
    """The two quantizer-only streaming tensors (Student-t, df=3)."""
    return {
        "act_8192x4096": student_t(8192, 4096, 3.0, seed),
        "act_4096x14336": student_t(4096, 14336, 3.0, seed + 1),
    }


def attention_operands(seed=5, B=4, H=32, S=2048, D=128):
    """Attention matmul operands: Q, K [B*H, S, D] blocked along D; P [B*H, S, S]
    (softmax rows) and V^T [B*H, D, S] blocked along the sequence.  Q/K/V are
    N(0,1) with 2 outlier head dims x30."""
    bh = B * H
    q = gaussian_outlier_channels(bh * S, D, 2, 30.0, 1.0, seed).view(bh, S, D)
    k = gaussian_outlier_channels(bh * S, D, 2, 30.0, 1.0, seed + 1).view(bh, S, D)
    v = gaussian_outlier_channels(bh * S, D, 2, 30.0, 1.0, seed + 2).view(bh, S, D)
    return {"q": q, "k": k, "vt": v.transpose(1, 2).contiguous()}


def to_f64(x_bf16):
    """Exact float64 NumPy view of a bf16 tensor (for the oracle's callers)."""
    return x_bf16.detach().cpu().to(torch.float64).numpy()


def all_bf16_bit_patterns():
    """Every finite bf16 value (65280 bit patterns, in bit-pattern order) as a
    [2040, 32] tensor; used for exhaustive element-level checks."""
    bits = np.arange(65536, dtype=np.uint32)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF].astype(np.uint16)
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).view(-1, 32)
