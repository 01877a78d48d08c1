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

    def __init__(self, cap_bytes: int, device: int = 0, fence_slack_bytes=None):
        """cap_bytes: the emulated VRAM cap = size of the arena every byte of the path is carved from.
        fence_slack_bytes: second fence around the cap: PyTorch's caching allocator may not hold more than
        cap + slack on this device (slack covers measurement buffers that are not part of the path) until close().
        The limit is per process, so only one fenced engine can be alive at a time; None (default): no fence."""
        self.device = device
        self.cap_bytes = int(cap_bytes)
        self.ctx = B.Context(device)
        self.torch = None
        if device >= 0:
            import torch
            self.torch = torch
            self.dev = torch.device("cuda", device)
            torch.cuda.set_device(self.dev)
            self.fenced = fence_slack_bytes is not None
            if self.fenced:
                total = torch.cuda.get_device_properties(self.dev).total_memory
                torch.cuda.set_per_process_memory_fraction(min(1.0, (self.cap_bytes + fence_slack_bytes) / total), self.dev)
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
        if self.torch is not None and getattr(self, "fenced", False):
            self.torch.cuda.set_per_process_memory_fraction(1.0, self.dev)
            self.fenced = False

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


class VlaPipeline:
    """The five-stage pipeline (vision encoder, merger, decoder prefill, decoder decode, action head with
    Euler steps) wired from C-ABI calls.  One context, one slot pair shared by the three layer stacks.
    Plumbing only: it registers the parts, owns the buffers and calls dl_vla_infer."""

    def __init__(self, eng: Engine, vit: CFG.ModuleConfig, dec: CFG.ModuleConfig, act: CFG.ModuleConfig,
                 n_patches: int, n_text: int, n_actions: int = 64, pool: int = 4, out_dim: int = 3,
                 seeds=(11, 12, 13, 14, 15), matrix_gain: float = 0.0):
        """matrix_gain: see configs.make_layer_weights (0 = the stated N(0, 0.02) recipe)."""
        self.eng, self.vit, self.dec, self.act = eng, vit, dec, act
        self.n_patches, self.n_text, self.n_actions, self.pool = n_patches, n_text, n_actions, pool
        self.n_vis = n_patches // pool
        self.n_prefill = self.n_vis + n_text
        ctx = eng.ctx
        gen = (lambda c: (lambda l: CFG.make_layer_weights(c, l, matrix_gain)))
        self.m_vit = eng.add_module(vit, max_tokens=n_patches, weights=gen(vit))
        self.m_dec = eng.add_module(dec, max_tokens=self.n_prefill, weights=gen(dec))
        self.m_act = eng.add_module(act, max_tokens=n_actions, max_ctx=self.n_prefill, weights=gen(act))
        inp = CFG.make_pipeline_inputs(vit, dec, act, n_patches, n_text, n_actions, out_dim, seeds, matrix_gain)
        self.proj_w, self.out_w = inp["proj_w"], inp["out_w"]
        self.mlp_proj = ctx.mlp_create(vit.d_model, dec.d_model, dec.d_model, *self.proj_w, max_tokens=n_patches)
        self.mlp_out = ctx.mlp_create(act.d_model, 0, out_dim, None, None, self.out_w[2], self.out_w[3],
                                      max_tokens=n_actions)
        self.patches, self.text, self.a0 = inp["patches"], inp["text"], inp["a0"]
        A = eng.alloc_f32
        self.p_patch, self.v_patch = A(n_patches * vit.d_model)
        self.p_vit, self.v_vit = A(n_patches * vit.d_model)
        self.p_proj, self.v_proj = A(n_patches * dec.d_model)
        self.p_seq, self.v_seq = A(self.n_prefill * dec.d_model)
        self.p_h, self.v_h = A(self.n_prefill * dec.d_model)
        self.p_ctx, self.v_ctx = A(self.n_prefill * dec.d_model)
        self.p_x1, self.v_x1 = A(dec.d_model)
        self.p_y1, self.v_y1 = A(dec.d_model)
        self.p_tok, self.v_tok = A(256)
        self.p_a, self.v_a = A(n_actions * act.d_model)
        self.p_ain, self.v_ain = A(n_actions * act.d_model)
        self.p_vel, self.v_vel = A(n_actions * act.d_model)
        self.p_traj, self.v_traj = A(n_actions * out_dim)
        self.out_dim = out_dim
        eng.upload(self.v_patch, self.patches)

    def run(self, n_decode: int, n_euler: int = 10):
        """Enqueues one whole inference; returns after the final synchronisation."""
        e, ctx = self.eng, self.eng.ctx
        d = self.dec.d_model
        # text embeddings and the initial action noise are inputs: (re)upload them untimed by the caller if needed
        e.upload(self.v_seq[self.n_vis * d:], self.text)
        e.upload(self.v_a, self.a0)
        self.enqueue(n_decode, n_euler)
        ctx.sync()

    def enqueue(self, n_decode: int, n_euler: int = 10):
        """One whole inference as ONE library call (dl_vla_infer sequences the five stages natively)."""
        self.eng.ctx.vla_infer(
            dict(m_vit=self.m_vit, m_dec=self.m_dec, m_act=self.m_act, mlp_proj=self.mlp_proj, mlp_out=self.mlp_out,
                 n_patches=self.n_patches, pool=self.pool, n_text=self.n_text, n_actions=self.n_actions,
                 n_decode=n_decode, n_euler=n_euler, out_dim=self.out_dim),
            dict(patches=self.p_patch, vit_out=self.p_vit, proj_out=self.p_proj, seq=self.p_seq, hidden=self.p_h,
                 hidden_ctx=self.p_ctx, x1=self.p_x1, y1=self.p_y1, tokens=self.p_tok, actions=self.p_a,
                 act_in=self.p_ain, velocity=self.p_vel, trajectory=self.p_traj))

    def enqueue_glue(self, n_euler: int = 10):
        """Only the launches of `enqueue` that belong to no layer and not to the greedy head: projector, pooling,
        final norm, time embeddings, Euler updates, output projection (what a latency model has to add as a constant)."""
        ctx = self.eng.ctx
        d, da = self.dec.d_model, self.act.d_model
        ctx.mlp_forward(self.mlp_proj, self.p_vit, self.p_proj, self.n_patches)
        ctx.mean_pool(self.p_proj, self.p_seq, self.n_vis, self.pool, d)
        ctx.final_norm(self.m_dec, self.p_h, self.p_ctx, self.n_prefill)
        for s in range(n_euler):
            ctx.add_time_embedding(self.p_a, self.p_ain, s / n_euler, self.n_actions, da)
            ctx.axpy(self.p_a, 1.0 / n_euler, self.p_vel, self.n_actions * da)
        ctx.mlp_forward(self.mlp_out, self.p_a, self.p_traj, self.n_actions)

    def results(self, n_decode: int):
        e = self.eng
        toks = e.download(self.v_tok[:min(n_decode, 256)]).view(np.int32).tolist() if n_decode else []
        return dict(tokens=toks,
                    hidden_ctx=e.download(self.v_ctx).reshape(self.n_prefill, self.dec.d_model),
                    actions=e.download(self.v_a).reshape(self.n_actions, self.act.d_model),
                    trajectory=e.download(self.v_traj).reshape(self.n_actions, self.out_dim))
