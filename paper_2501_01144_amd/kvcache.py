"""Value cache with a high-precision residual chunk (paper, Appendix C).

Values are multiplied over the token axis (P V), so they are quantized along it:
the cache holds the quantized transpose V^T [head_dim, capacity] in blocks of 32
tokens.  A block can only be quantized when all its 32 tokens are known, and
requantizing it for every new token would repeat work and compound errors, so
the most recent, incomplete chunk (fewer than 32 tokens) stays in bf16 and is
quantized once, when it is full.  Keys are multiplied over the head dimension
and need no such care: each new key row is quantized on its own (dfp4.quantize).

Host-side bookkeeping only; the arithmetic is in the library's kernels
(dfp4_quantize_t_at).  Unwritten blocks of the cache are zero (code 0, exponent
byte 0), so a product over the whole capacity with zero-padded probabilities
equals the product over the tokens present.
"""
import torch

from . import dfp4

BLOCK = 32


class ValueCache:
    def __init__(self, head_dim, capacity_tokens, device):
        assert capacity_tokens % BLOCK == 0 and head_dim % 8 == 0
        self.head_dim, self.capacity = head_dim, capacity_tokens
        self.q = dfp4.QTensor(
            torch.zeros((head_dim, capacity_tokens // 2), dtype=torch.uint8, device=device),
            torch.zeros((head_dim, capacity_tokens // BLOCK), dtype=torch.uint8, device=device),
            torch.zeros((head_dim, capacity_tokens // BLOCK), dtype=torch.uint8, device=device),
            head_dim, capacity_tokens)
        self.residual = torch.zeros((BLOCK, head_dim), dtype=torch.bfloat16, device=device)
        self.n_quantized = 0           # tokens held in 4-bit form (a multiple of 32)
        self.n_residual = 0            # tokens held in bf16 (< 32)

    @property
    def n_tokens(self):
        return self.n_quantized + self.n_residual

    def append(self, v):
        """v: bf16 [t, head_dim], the values of t new tokens."""
        assert v.dtype == torch.bfloat16 and v.dim() == 2 and v.shape[1] == self.head_dim
        assert self.n_tokens + v.shape[0] <= self.capacity, "value cache full"
        pos = 0
        while pos < v.shape[0]:
            if self.n_residual == 0 and v.shape[0] - pos >= BLOCK:
                # whole chunks go straight to 4 bits
                rows = (v.shape[0] - pos) // BLOCK * BLOCK
                dfp4.quantize_t_at(v[pos:pos + rows].contiguous(), self.q, self.n_quantized)
                self.n_quantized += rows
                pos += rows
                continue
            take = min(BLOCK - self.n_residual, v.shape[0] - pos)
            self.residual[self.n_residual:self.n_residual + take] = v[pos:pos + take]
            self.n_residual += take
            pos += take
            if self.n_residual == BLOCK:
                dfp4.quantize_t_at(self.residual, self.q, self.n_quantized)
                self.n_quantized += BLOCK
                self.n_residual = 0

    def residual_values(self):
        """bf16 [n_residual, head_dim]: the tokens not yet quantized."""
        return self.residual[:self.n_residual]
