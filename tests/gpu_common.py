"""Shared helpers of the GPU parity tests: run a stack through the C ABI, run the oracle on the
same seeded inputs, compare."""
import numpy as np

from oracle import forward as F
from paper_2605_11678_amd import configs as CFG
from paper_2605_11678_amd.harness import Engine


def rel_err(got, want):
    """max |got - want| / max |want| (element-wise ratios are meaningless near zero)."""
    return float(np.max(np.abs(got.astype(np.float64) - want)) / np.max(np.abs(want)))


def oracle_cfg(c):
    return c.as_dict()


class GpuStack:
    """One module on a fresh engine, weights from the seeded recipe (or a given generator)."""

    def __init__(self, c, max_tokens, cap_bytes=2 << 30, max_ctx=0, weights=None, head=None):
        self.c = c
        self.eng = Engine(cap_bytes, device=0)
        self.weights = weights or (lambda l: CFG.make_layer_weights(c, l))
        self.head = head if head is not None else (CFG.make_head(c) if c.vocab > 0 else None)
        self.mid = self.eng.add_module(c, max_tokens, max_ctx, weights=self.weights, head=self.head)
        self.max_tokens = max_tokens
        self.xp, self.xv = self.eng.alloc_f32(max_tokens * c.d_model)
        self.yp, self.yv = self.eng.alloc_f32(max_tokens * c.d_model)
        self.np_, self.nv = self.eng.alloc_f32(max_tokens * c.d_model)
        self.cp = self.cv = None
        if max_ctx:
            self.cp, self.cv = self.eng.alloc_f32(max_ctx * c.d_ctx)

    def close(self):
        self.eng.close()

    def forward(self, x, pos0=0, ctx=None, final_norm=False):
        T, d = x.shape
        self.eng.upload(self.xv[:T * d], x)
        n_ctx = 0
        if ctx is not None:
            n_ctx = ctx.shape[0]
            self.eng.upload(self.cv[:ctx.size], ctx)
        self.eng.ctx.forward(self.mid, self.xp, self.yp, T, pos0, self.cp if ctx is not None else None, n_ctx)
        if final_norm:
            self.eng.ctx.final_norm(self.mid, self.yp, self.np_, T)
            return self.eng.download(self.nv[:T * d]).reshape(T, d)
        return self.eng.download(self.yv[:T * d]).reshape(T, d)

    def forward_bits(self, x, pos0=0, ctx=None):
        return self.forward(x, pos0, ctx).view(np.uint32).copy()
