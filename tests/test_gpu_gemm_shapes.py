"""GPU parity of the GEMM kernels over the tile shapes the dispatcher can pick, through the C-ABI's two-layer
perceptron (dl_mlp_forward: y = GELU(x W1^T + b1) W2^T + b2, Sec. II-A stage 2).  The first product takes the
fast MFMA path with the GELU epilogue in every tile shape (128x128, 128x144 on four LDS stages with both loop tails, 128x192, 192x192, 192x256, 256x192, 256x256, and 256x256
with the last half round split into 128x256 halves), the generic kernel, or, with at most 64 rows and K a multiple
of 64, the few-rows kernel; the second one (fp32 output) takes the generic or the few-rows kernel.  Rows are independent, so the oracle evaluates a sample of rows that covers the first and
last row, tile borders and the ragged tail."""
import numpy as np
import pytest

from oracle import pipeline as PL
from paper_2605_11678_amd import configs as CFG
from paper_2605_11678_amd.harness import Engine
from tests.gpu_common import rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2

# (tokens, d_in, d_hidden, d_out, what the dispatcher picks for the first product)
SHAPES = [
    (50, 200, 264, 40, "generic kernel: few rows, K not a multiple of 128"),
    (64, 1024, 4096, 1024, "few-rows kernel: both products, every wavefront has chunks"),
    (13, 256, 320, 96, "few-rows kernel: ragged rows, half of the wavefronts without a chunk"),
    (33, 64, 64, 32, "few-rows kernel: a single K chunk"),
    (97, 256, 384, 64, "128x128, a single ragged row tile"),
    (300, 1152, 1152, 96, "128x128, narrow output, ragged last row tile"),
    (4000, 1152, 4352, 64, "128x192, short reduction, ragged last row tile"),
    (1000, 2304, 1152, 64, "128x144 of 160, four stages, 36 k-tiles (tail of four), ragged last row tile"),
    (300, 2176, 1096, 64, "128x144 of 160, four stages, 34 k-tiles (tail of six), last column tile cut by the matrix edge"),
    (1000, 2304, 4096, 64, "192x192"),
    (3072, 2176, 4096, 64, "192x256"),
    (4096, 2176, 3072, 64, "256x192"),
    (4096, 2176, 4096, 64, "256x256, exactly one round"),
    (3072, 2176, 24576, 128, "256x256 with the last half round split into 128x256 halves"),
]


@pytest.mark.parametrize("T,d_in,d_hid,d_out,what", SHAPES, ids=[s[4].split(",")[0].split(":")[0] + "-%d" % i for i, s in enumerate(SHAPES)])
def test_mlp_matches_oracle_on_sampled_rows(T, d_in, d_hid, d_out, what):
    w = CFG.make_mlp(d_in, d_hid, d_out, seed=4242 + d_hid)
    x = CFG.make_tokens(T, d_in, seed=17)
    act_bytes = 4 * T * (d_in + d_out) + 2 * T * (d_in + d_hid)
    w_bytes = 2 * (d_hid * d_in + d_out * d_hid + d_hid + d_out)
    eng = Engine(act_bytes + w_bytes + (64 << 20), device=0)
    try:
        ctx = eng.ctx
        m = ctx.mlp_create(d_in, d_hid, d_out, *w, max_tokens=T)
        xp, xv = eng.alloc_f32(T * d_in)
        yp, yv = eng.alloc_f32(T * d_out)
        eng.upload(xv, x)
        ctx.mlp_forward(m, xp, yp, T)
        got = eng.download(yv).reshape(T, d_out)
        rows = sorted({0, 1, T // 2, T - 1, T - 2} | {r for b in (96, 127, 128, 191, 192, 255, 256, 383, 384) for r in (b - 1, b, b + 1) if 0 <= r < T}
                      | set(np.random.default_rng(5).integers(0, T, 12).tolist()))
        want = PL.mlp(x[rows], *w)
        assert np.all(np.isfinite(got))
        assert rel_err(got[rows], want) <= TOL, (what, rel_err(got[rows], want))
        # a second call with fewer rows leaves the rows it does not touch alone and reproduces the others bit for bit
        if T > 8:
            yv.zero_()
            eng.torch.cuda.synchronize()
            ctx.mlp_forward(m, xp, yp, T - 7)
            again = eng.download(yv).reshape(T, d_out)
            assert np.array_equal(again[:T - 7].view(np.uint32), got[:T - 7].view(np.uint32))
            assert not again[T - 7:].any()
    finally:
        eng.close()
