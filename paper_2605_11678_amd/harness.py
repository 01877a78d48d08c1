"""Glue between the workloads (configs.py), PyTorch (device memory, streams) and the C-ABI
binding.  Plumbing only: allocates the capped arena as one torch tensor, creates the two
streams, registers a layer stack with seeded weights, and moves activations in and out.
No step of the forward pass, planner or predictor is computed here.
"""
import numpy as np

from . import binding as B
from . import configs as CFG


def desc_fields(c: CFG.ModuleConfig, max_tokens: int, max_ctx: int = 0):
    f = c.as_dict()
    f["max_tokens"] = max_tokens
    f["max_ctx"] = max_ctx
    return f


class Engine:
    """One context on one device (device=-1: host-only accounting context, no GPU)."""

    def __init__(self, cap_bytes: int, device: int = 0):
        self.device = device
        self.cap_bytes = int(cap_bytes)
        self.ctx = B.Context(device)
        self.torch = None
        if device >= 0:
            import torch
            self.torch = torch
            self.dev = torch.device("cuda", device)
            torch.cuda.set_device(self.dev)
            self.arena = torch.empty(self.cap_bytes, dtype=torch.uint8, device=self.dev)
            self.ctx.set_arena(self.arena.data_ptr(), self.cap_bytes, keep=self.arena)
            self.s_compute = torch.cuda.Stream(device=self.dev)
            self.s_copy = torch.cuda.Stream(device=self.dev)
            self.ctx.set_streams(self.s_compute.cuda_stream, self.s_copy.cuda_stream, keep=(self.s_compute, self.s_copy))
        else:
            self.ctx.set_arena(0, self.cap_bytes)
        self.modules = {}

    def close(self):
        self.ctx.destroy()
        self.arena = None

    # ---- registration ----
    def add_module(self, c: CFG.ModuleConfig, max_tokens: int, max_ctx: int = 0, weights=None, head=None):
        """weights: callable layer -> {tensor id: uint16 array}; default: the seeded recipe of configs.py."""
        mid = self.ctx.module_create(**desc_fields(c, max_tokens, max_ctx))
        gen = weights or (lambda l: CFG.make_layer_weights(c, l))
        for l in range(c.n_layers):
            for tid, arr in gen(l).items():
                self.ctx.layer_set_tensor(mid, l, tid, np.ascontiguousarray(arr).reshape(-1))
        if c.vocab > 0:
            hd = head if head is not None else CFG.make_head(c)
            for which, arr in hd.items():
                self.ctx.set_resident_tensor(mid, which, np.ascontiguousarray(arr).reshape(-1))
        self.ctx.module_finalize(mid)
        self.modules[mid] = c
        return mid

    def pick_copy_stream(self, mid, n_tokens, x_ptr, y_ptr, pos0=0, candidates=6, passes=3):
        """HIP maps streams onto a handful of hardware queues; two streams that land on the same queue do
        not overlap.  Which pairs collide cannot be queried, so it is measured: every candidate copy stream
        runs a few fully streamed passes back to back and the fastest one is kept.  Returns the
        (stream index, ms per pass) list."""
        import time
        c = self.modules[mid]
        keep_res = self.ctx.get_residency(mid, c.n_layers)
        self.ctx.set_residency(mid, [])
        tried = []
        cands = [self.s_copy] + [self.torch.cuda.Stream(device=self.dev) for _ in range(candidates - 1)]
        for i, st in enumerate(cands):
            if st.cuda_stream == self.s_compute.cuda_stream:
                continue
            self.ctx.set_streams(self.s_compute.cuda_stream, st.cuda_stream, keep=st)
            self.ctx.forward(mid, x_ptr, y_ptr, n_tokens, pos0)
            self.ctx.sync()
            t = time.perf_counter()
            for _ in range(passes):
                self.ctx.forward(mid, x_ptr, y_ptr, n_tokens, pos0)
            self.ctx.sync()
            tried.append((i, (time.perf_counter() - t) * 1e3 / passes))
        best = min(tried, key=lambda r: r[1])[0]
        self.s_copy = cands[best]
        self.ctx.set_streams(self.s_compute.cuda_stream, self.s_copy.cuda_stream, keep=self.s_copy)
        self.ctx.set_residency(mid, keep_res)
        return tried

    # ---- activations (fp32, carved from the arena so that they count against the cap) ----
    def alloc_f32(self, n_elems: int):
        ptr = self.ctx.arena_alloc(4 * int(n_elems))
        if self.device < 0:
            return ptr, None
        off = ptr - self.arena.data_ptr()
        view = self.arena[off: off + 4 * int(n_elems)].view(self.torch.float32)
        return ptr, view

    def upload(self, view, host_f32: np.ndarray):
        t = self.torch.from_numpy(np.ascontiguousarray(host_f32, dtype=np.float32).reshape(-1))
        with self.torch.cuda.stream(self.s_compute):
            view.copy_(t, non_blocking=False)
        self.s_compute.synchronize()

    def download(self, view) -> np.ndarray:
        self.ctx.sync()
        return view.cpu().numpy().copy()
