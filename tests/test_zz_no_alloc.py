"""dl_greedy_step_static (the greedy head for callers that cannot allocate: its scratch is a static device array)
against dl_greedy_step, through the C ABI: identical token and identical next-step input, on two calls in a row, the
second with a smaller head (the array keeps the first call's logits, which the second must not see)."""
import numpy as np
import pytest

from paper_2605_11678_amd import binding as B
from paper_2605_11678_amd import configs as CFG
from tests.gpu_common import GpuStack


def _run(c, T, seed, torch):
    x = CFG.make_tokens(T, c.d_model, seed=seed)
    g = GpuStack(c, max_tokens=T, cap_bytes=256 << 20)
    try:
        eng, ctx, d = g.eng, g.eng.ctx, c.d_model
        eng.upload(g.xv[:T * d], x)
        ctx.forward(g.mid, g.xp, g.yp, T, 0)
        h_ptr = g.yp + 4 * (T - 1) * d
        # the existing entry point: token and next-step input through the module's arena workspace
        tp, tv = eng.alloc_f32(2)
        ctx.greedy_step(g.mid, h_ptr, tp, g.xp)
        want_tok = int(eng.download(tv).view(np.int32)[0])
        want_x = eng.download(g.xv[:d]).copy()
        # the same head in the caller's own device memory (torch tensors), nothing from the context
        dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).reshape(-1).copy()).to(eng.dev)
        head, emb = dev(g.head[CFG.R_HEAD]), dev(g.head[CFG.R_EMBED])
        ng = dev(g.head[CFG.R_FINAL_NORM_G])
        nb = dev(g.head[CFG.R_FINAL_NORM_B]) if c.norm == CFG.NORM_LN else None
        tok = torch.full((1,), -1, dtype=torch.int32, device=eng.dev)
        xo = torch.full((d,), float("nan"), dtype=torch.float32, device=eng.dev)
        torch.cuda.synchronize()
        B.greedy_step_static(0, eng.s_compute.cuda_stream, h_ptr, head.data_ptr(), emb.data_ptr(), ng.data_ptr(),
                             nb.data_ptr() if nb is not None else None, c.norm, c.norm_eps, d, c.vocab,
                             tok.data_ptr(), xo.data_ptr())
        eng.s_compute.synchronize()
        assert int(tok.cpu()[0]) == want_tok, (int(tok.cpu()[0]), want_tok)
        assert np.array_equal(xo.cpu().numpy().view(np.uint32), want_x.view(np.uint32))
        # token only (no embedding table): same token
        tok.fill_(-1)
        torch.cuda.synchronize()
        B.greedy_step_static(0, eng.s_compute.cuda_stream, h_ptr, head.data_ptr(), None, ng.data_ptr(),
                             nb.data_ptr() if nb is not None else None, c.norm, c.norm_eps, d, c.vocab, tok.data_ptr(), None)
        eng.s_compute.synchronize()
        assert int(tok.cpu()[0]) == want_tok
        return want_tok
    finally:
        g.close()


@pytest.mark.gpu
def test_static_greedy_step_matches_greedy_step_twice_second_smaller():
    import torch
    big = CFG.tiny_decoder()                                    # RMSNorm, d = 256, vocab 1024
    small = CFG.ModuleConfig("ln_head_small", 1, 128, 2, 2, 64, 256, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0,
                             seed_base=8100, vocab=320)         # LayerNorm (bias), d = 128, vocab 320
    t_big = _run(big, 96, 51, torch)
    t_small = _run(small, 40, 52, torch)
    assert 0 <= t_big < big.vocab and 0 <= t_small < small.vocab
    # sizes beyond the static array are refused with a message, before anything is launched
    with pytest.raises(B.DLError) as e:
        B.greedy_step_static(0, None, 1, 1, 1, 1, None, CFG.NORM_RMS, 1e-6, 256, 131073, 1, 1)
    assert e.value.code == B.DL_ERR_INVALID_ARG and "131072" in str(e.value)
    with pytest.raises(B.DLError):
        B.greedy_step_static(0, None, 1, 1, 1, 1, None, CFG.NORM_LN, 1e-6, 256, 1024, 1, 1)   # LayerNorm without bias
