// BF16 GEMM on gfx950 matrix cores: C[M,N] = A[M,K] * B[N,K]^T with fused epilogues.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants for A and
// for B alike (a lane supplies 8 consecutive k of one row / one column), so no tile is ever
// transposed on its way to the matrix core.  Weights are stored [N,K] by the packer for exactly this reason.
//
// Three kernels share the epilogues:
//
//  * gemm_fast<BM,BN,EPI,WM,BNR,NS> — the production path for K % 128 == 0.  256 threads = 4 wavefronts, 2x2 (WM = 2:
//    each owns a (BM/2)x(BN/2) tile, up to 4x4 MFMA tiles = 256 fp32 accumulators per lane) or stacked 4x1 (WM = 4);
//    one workgroup per CU for the 192- and 256-row tiles, two for 128x192 and 128x128.  BNR <= BN columns are stored
//    (128x144 of a 128x160 tile puts exactly one workgroup on every CU for N = 1152).  k-tile 64: a row of a tile is
//    one 128-byte cache line.  Tiles go global -> LDS directly (buffer_load_dwordx4 ... lds, no staging registers) into
//    NS = 2 (4 for the small tile with long reductions) LDS stages that are separate arrays, so the compiler can tell
//    the stage being filled from the one being read; the wait for a copy is an explicit s_waitcnt.  LDS rows are
//    128 bytes, unpadded (a wavefront's copy fills 1 KB = 8 rows contiguously); the 16-byte chunk index is
//    XOR-swizzled with (row/2)%8 on both sides, which keeps the b128 fragment reads conflict-free.  Per k-tile four
//    phases of up to 16 MFMAs, each interleaved with the fragment reads of the next phase through
//    sched_group_barrier, ONE bare s_barrier, and the copy of the k-tile NS ahead spread over the two phases that
//    follow the barrier (a whole k-tile of time to land).
//  * gemm_generic<EPI> — any shape (K % 8 == 0): 128x128 tile, 64x64 per wavefront, staged through registers.
//  * gemm_few_rows<EPI> — M <= 64: 64x32 output per workgroup, reduction split over its 8 wavefronts.
//
// Accumulator layout of a 32x32 tile: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4.
#include <type_traits>

#include "kernels.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_LD = BK + 8;   // row stride in elements: 144 bytes keeps 16-byte alignment and staggers banks

// x * sigmoid(x); the quotient is a multiplication with the hardware reciprocal (1 ulp), not an IEEE division
__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
// tanh form of GELU: 0.5 x (1 + tanh u) = x * sigmoid(2u), u = sqrt(2/pi) (x + 0.044715 x^3): one exponential and
// one reciprocal instead of a library tanh (which dominated the epilogue of the encoder's MLP GEMM)
__device__ __forceinline__ float gelu_tanh_f(float x) {
    const float c2 = 2.0f * 0.7978845608028654f;
    const float u2 = c2 * (x + 0.044715f * x * x * x);
    return x * __builtin_amdgcn_rcpf(1.0f + __expf(-u2));
}
__device__ __forceinline__ float bf16_to_f(bf16_t v) { return __uint_as_float(uint32_t(v) << 16); }
__device__ __forceinline__ bf16_t f_to_bf16(float f) {
    __bf16 b = (__bf16)f;   // hardware round-to-nearest-even
    return *reinterpret_cast<bf16_t*>(&b);
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm_generic(GemmArgs p) {
    __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles_n = (p.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tiles_n) * BM, n0 = (blockIdx.x % tiles_n) * BN;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = (c & 7) * 8;
            const int k = k0 + kc;
            u32x4 z = {0u, 0u, 0u, 0u};
            ra[i] = z;
            rb[i] = z;
            if (m0 + row < p.M && k < p.K)
                ra[i] = *reinterpret_cast<const u32x4*>(p.A + size_t(m0 + row) * p.lda + k);
            if (n0 + row < p.N && k < p.K)
                rb[i] = *reinterpret_cast<const u32x4*>(p.B + size_t(n0 + row) * p.ldb + k);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = (c & 7) * 8;
            *reinterpret_cast<u32x4*>(&sA[row * LDS_LD + kc]) = ra[i];
            *reinterpret_cast<u32x4*>(&sB[row * LDS_LD + kc]) = rb[i];
        }
    };

    const int nk = (p.K + BK - 1) / BK;
    fetch(0);
    for (int kt = 0; kt < nk; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * BK);
        const int lr = lane & 31, lk = (lane >> 5) * 8;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = *reinterpret_cast<const bf16x8*>(&sA[(64 * wm + 32 * i + lr) * LDS_LD + 16 * kk + lk]);
                b[i] = *reinterpret_cast<const bf16x8*>(&sB[(64 * wn + 32 * i + lr) * LDS_LD + 16 * kk + lk]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue ----
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
    if (EPI == EPI_SWIGLU_BF16) {
        // tile column j = 0 holds gate rows, j = 1 the matching up rows (packed in groups of 32)
        const int pn = n0 + 64 * wn + col_in;           // packed column of the gate value
        if (pn + 32 < p.N) {
            const int f = (n0 + 64 * wn) / 2 + col_in;  // feature index
            bf16_t* out = static_cast<bf16_t*>(p.out);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + 64 * wm + 32 * i + 8 * (r >> 2) + row_in + (r & 3);
                    if (m < p.M) out[size_t(m) * p.ldo + f] = f_to_bf16(silu_f(acc[i][0][r]) * acc[i][1][r]);
                }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + 64 * wn + 32 * j + col_in;
        if (n >= p.N) continue;
        const float bias = p.bias ? bf16_to_f(p.bias[n]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 64 * wm + 32 * i + 8 * (r >> 2) + row_in + (r & 3);
                if (m >= p.M) continue;
                const float v = acc[i][j][r] + bias;
                if (EPI == EPI_BF16) {
                    static_cast<bf16_t*>(p.out)[size_t(m) * p.ldo + n] = f_to_bf16(v);
                } else if (EPI == EPI_GELU_BF16) {
                    static_cast<bf16_t*>(p.out)[size_t(m) * p.ldo + n] = f_to_bf16(gelu_tanh_f(v));
                } else if (EPI == EPI_RESID_F32) {
                    static_cast<float*>(p.out)[size_t(m) * p.ldo + n] = p.resid[size_t(m) * p.ldr + n] + v;
                } else {
                    static_cast<float*>(p.out)[size_t(m) * p.ldo + n] = v;
                }
            }
    }
}


// ---- few rows (M <= 64): the work is tiny and the launch is bound by memory latency, so it is spread as widely as a
// deterministic sum allows.  One 512-thread workgroup per 32 output columns; its 8 wavefronts take the 64-wide K chunks
// round-robin and each computes the whole 64 x 32 tile over its chunks.  A wavefront fetches a chunk (64 + 32 rows of
// 128 bytes) with 8 lanes per row, so a load instruction touches 8 cache lines (fragment-shaped loads touch 32 and
// were bound by the L1's tag rate: 15 us for K = 1024), parks it in its own piece of LDS and reads MFMA fragments
// back from there; two chunks are in flight per wavefront, row addresses are clamped to M - 1, nothing is predicated.
// The 8 partial tiles meet in LDS and are summed in wavefront order, then every thread finishes 4 adjacent columns of
// one row.  Needs K % 64 == 0, N % 32 == 0, 16-byte aligned rows.
constexpr int SK_WAVES = 8, SK_DEPTH = 2;
constexpr int SK_LD = 72;                            // staged row stride (elements): 144 bytes staggers the banks
constexpr int SK_STAGE = (64 + 32) * SK_LD;          // elements per wavefront
template <int EPI>
__global__ __launch_bounds__(512) void gemm_few_rows(GemmArgs p) {
    // the staging area of the main loop and the partial tiles of the reduction share the same memory
    __shared__ __attribute__((aligned(16))) char smem[SK_WAVES * SK_STAGE * 2];
    static_assert(SK_WAVES * SK_STAGE * 2 >= SK_WAVES * 64 * 32 * 4, "partial tiles must fit the staging area");
    bf16_t* stage = reinterpret_cast<bf16_t*>(smem) + (threadIdx.x >> 6) * SK_STAGE;
    float (*part)[64 * 32] = reinterpret_cast<float (*)[64 * 32]>(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * 32;
    const int lr = lane & 31, g2 = lane >> 5;
    const int n_chunks = p.K >> 6;
    const int n_my = wave < n_chunks ? (n_chunks - wave + SK_WAVES - 1) / SK_WAVES : 0;
    // fetch mapping: load j covers rows 8 j .. 8 j + 7, lane l row 8 j + l / 8, bytes 16 (l % 8) of the chunk
    const int frow = lane >> 3, fcol = (lane & 7) * 8;
    const bf16_t* asrc[8];
    const bf16_t* bsrc[4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int m = 8 * j + frow;
        asrc[j] = p.A + size_t(m < p.M ? m : p.M - 1) * p.lda + fcol;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) bsrc[j] = p.B + size_t(n0 + 8 * j + frow) * p.ldb + fcol;

    u32x4 ra[SK_DEPTH][8], rb[SK_DEPTH][4];
    auto request = [&](int d, int idx) {
        // chunks past the wavefront's last one repeat it (in bounds, never used)
        const int ii = idx < n_my ? idx : (n_my > 0 ? n_my - 1 : 0);
        const int k0 = (n_my > 0 ? wave + SK_WAVES * ii : 0) * 64;
#pragma unroll
        for (int j = 0; j < 8; ++j) ra[d][j] = *reinterpret_cast<const u32x4*>(asrc[j] + k0);
#pragma unroll
        for (int j = 0; j < 4; ++j) rb[d][j] = *reinterpret_cast<const u32x4*>(bsrc[j] + k0);
    };
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
#pragma unroll
    for (int d = 0; d < SK_DEPTH; ++d) request(d, d);
    for (int base = 0; base < n_my; base += SK_DEPTH) {
#pragma unroll
        for (int d = 0; d < SK_DEPTH; ++d) {
            if (base + d < n_my) {
                // LDS operations of one wavefront execute in order: the fragment reads of the previous chunk are
                // done before these writes land, and the reads below see them
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    *reinterpret_cast<u32x4*>(stage + (8 * j + frow) * SK_LD + fcol) = ra[d][j];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4*>(stage + (64 + 8 * j + frow) * SK_LD + fcol) = rb[d][j];
            }
            request(d, base + d + SK_DEPTH);
            if (base + d < n_my) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    // read with the type the chunk was written with (the same accesses, as far as the compiler's
                    // alias rules go), reinterpret in registers
                    u32x4 fb = *reinterpret_cast<const u32x4*>(stage + (64 + lr) * SK_LD + 16 * s + 8 * g2);
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        u32x4 fa = *reinterpret_cast<const u32x4*>(stage + (32 * i + lr) * SK_LD + 16 * s + 8 * g2);
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&fa),
                                                                         *reinterpret_cast<bf16x8*>(&fb), acc[i], 0, 0, 0);
                    }
                }
            }
        }
    }
    __syncthreads();                                  // everybody is done with the staging area
    // accumulator (tile i, lane, register r) -> row 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32
    const int row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            part[wave][(32 * i + 8 * (r >> 2) + row_in + (r & 3)) * 32 + lr] = acc[i][r];
    __syncthreads();
    const int row = tid >> 3, c4 = (tid & 7) * 4;
    float4 sum = *reinterpret_cast<const float4*>(&part[0][row * 32 + c4]);
#pragma unroll
    for (int w = 1; w < SK_WAVES; ++w) {
        const float4 t = *reinterpret_cast<const float4*>(&part[w][row * 32 + c4]);
        sum.x += t.x;
        sum.y += t.y;
        sum.z += t.z;
        sum.w += t.w;
    }
    if (row >= p.M) return;
    const int n = n0 + c4;
    float v[4] = {sum.x, sum.y, sum.z, sum.w};
    if (p.bias) {
        const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + n);
        v[0] += __uint_as_float(bb.x << 16);
        v[1] += __uint_as_float(bb.x & 0xFFFF0000u);
        v[2] += __uint_as_float(bb.y << 16);
        v[3] += __uint_as_float(bb.y & 0xFFFF0000u);
    }
    if (EPI == EPI_BF16 || EPI == EPI_GELU_BF16) {
        if (EPI == EPI_GELU_BF16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = gelu_tanh_f(v[e]);
        }
        uint2 pk;
        pk.x = uint32_t(f_to_bf16(v[0])) | (uint32_t(f_to_bf16(v[1])) << 16);
        pk.y = uint32_t(f_to_bf16(v[2])) | (uint32_t(f_to_bf16(v[3])) << 16);
        *reinterpret_cast<uint2*>(static_cast<bf16_t*>(p.out) + size_t(row) * p.ldo + n) = pk;
    } else {
        float4 o = make_float4(v[0], v[1], v[2], v[3]);
        if (EPI == EPI_RESID_F32) {
            const float4 rs = *reinterpret_cast<const float4*>(p.resid + size_t(row) * p.ldr + n);
            o = make_float4(rs.x + v[0], rs.y + v[1], rs.z + v[2], rs.w + v[3]);
        }
        *reinterpret_cast<float4*>(static_cast<float*>(p.out) + size_t(row) * p.ldo + n) = o;
    }
}


// epilogue shared by both kernels: accumulator tile (i, j) of a wavefront whose tile starts at (mw, nw)
// n_end: first column past the tile's own columns (the matrix edge, or the start of the next tile when the tile's
// LDS width is padded beyond its stride)
template <int EPI, int TM, int TN>
__device__ __forceinline__ void store_tiles(const GemmArgs& p, f32x16 (&acc)[TM][TN], int mw, int nw, int lane, int n_end) {
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
    if (EPI == EPI_SWIGLU_BF16) {
        // even tile columns hold gate rows, the next odd one the matching up rows (packed in groups of 32)
        bf16_t* out = static_cast<bf16_t*>(p.out);
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
            const int pn = nw + 32 * j + col_in;            // packed column of the gate value
            if (pn + 32 >= p.N) continue;
            const int f = (nw + 32 * j) / 2 + col_in;        // feature index
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mw + 32 * i + 8 * (r >> 2) + row_in + (r & 3);
                    if (m < p.M) out[size_t(m) * p.ldo + f] = f_to_bf16(silu_f(acc[i][j][r]) * acc[i][j + 1][r]);
                }
        }
        return;
    }
    if (EPI == EPI_RESID_F32) {
        // out may be the same buffer as resid: every element is read and then written by the same lane only, so the
        // pointers are declared non-aliasing.  The residual values of a batch of accumulator tiles are all requested
        // before the first one is used - unpredicated, rows and columns clamped into the matrix - so that the
        // wavefront pays one memory round trip per batch instead of one per tile; only the stores are predicated.
        const float* __restrict__ resid = p.resid;
        float* __restrict__ out = static_cast<float*>(p.out);
        // column tiles per batch: what fits next to the accumulators without spilling (TM = 3: all of them)
        constexpr int JFIT = (352 - TM * TN * 16) / (TM * 16);
        constexpr int JB = TM == 3 ? TN : (JFIT < 1 ? 1 : (JFIT > TN ? TN : JFIT));
#pragma unroll
        for (int j0 = 0; j0 < TN; j0 += JB) {
            float rv[JB][TM][16];
            float bias[JB];
#pragma unroll
            for (int jj = 0; jj < JB; ++jj) {
                const int j = j0 + jj;
                if (j >= TN) continue;
                const int nc = min(nw + 32 * j + col_in, n_end - 1);
                bias[jj] = p.bias ? bf16_to_f(p.bias[nc]) : 0.0f;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int mc = min(mw + 32 * i + 8 * (r >> 2) + row_in + (r & 3), p.M - 1);
                        rv[jj][i][r] = resid[uint32_t(mc) * uint32_t(p.ldr) + uint32_t(nc)];   // < 2^31 elements (host checks)
                    }
            }
#pragma unroll
            for (int jj = 0; jj < JB; ++jj) {
                const int j = j0 + jj;
                if (j >= TN) continue;
                const int n = nw + 32 * j + col_in;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = mw + 32 * i + 8 * (r >> 2) + row_in + (r & 3);
                        if (m < p.M && n < n_end) out[uint32_t(m) * uint32_t(p.ldo) + uint32_t(n)] = rv[jj][i][r] + acc[i][j][r] + bias[jj];
                    }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = nw + 32 * j + col_in;
        if (n >= n_end) continue;
        const float bias = p.bias ? bf16_to_f(p.bias[n]) : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = mw + 32 * i + 8 * (r >> 2) + row_in + (r & 3);
                if (m >= p.M) continue;
                const float v = acc[i][j][r] + bias;
                if (EPI == EPI_BF16) {
                    static_cast<bf16_t*>(p.out)[size_t(m) * p.ldo + n] = f_to_bf16(v);
                } else if (EPI == EPI_GELU_BF16) {
                    static_cast<bf16_t*>(p.out)[size_t(m) * p.ldo + n] = f_to_bf16(gelu_tanh_f(v));
                } else {
                    static_cast<float*>(p.out)[size_t(m) * p.ldo + n] = v;
                }
            }
    }
}

// The same epilogues for a wavefront tile that lies wholly inside the matrix (every tile of the 8B shapes): nothing is
// predicated, and an element's address is a wavefront-uniform pointer (tile origin + row and column of the accumulator
// register, kept in scalar registers) plus one per-lane 32-bit offset computed once, so an element costs its
// arithmetic and one store instead of a 64-bit multiply-add, an exec-mask save/restore and a branch as well.
template <int EPI, int TM, int TN>
__device__ __forceinline__ void store_tiles_full(const GemmArgs& p, f32x16 (&acc)[TM][TN], int mw, int nw, int lane) {
    const uint32_t col_in = lane & 31, row_in = (lane >> 5) * 4;
    const uint32_t lane_o = row_in * uint32_t(p.ldo) + col_in;          // output element offset of this lane
    auto urow = [&](int i, int r) { return mw + 32 * i + 8 * (r >> 2) + (r & 3); };   // uniform part of the row
    if (EPI == EPI_SWIGLU_BF16) {
        bf16_t* out = static_cast<bf16_t*>(p.out);
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
            const int f0 = (nw + 32 * j) / 2;                             // first feature of this column-tile pair
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    bf16_t* pu = out + size_t(urow(i, r)) * p.ldo + f0;
                    pu[lane_o] = f_to_bf16(silu_f(acc[i][j][r]) * acc[i][j + 1][r]);
                }
        }
        return;
    }
    float bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bias[j] = p.bias ? bf16_to_f(p.bias[nw + 32 * j + col_in]) : 0.0f;
    if (EPI == EPI_RESID_F32) {
        // one base pointer each for resid and out, per-lane 32-bit element offsets that advance row by row with
        // additions (no scalar pointer per row: 48-64 of them next to the accumulators made the loads slower)
        const float* __restrict__ resid = p.resid + size_t(mw) * p.ldr + nw;
        float* __restrict__ out = static_cast<float*>(p.out) + size_t(mw) * p.ldo + nw;
        const uint32_t lane_r = row_in * uint32_t(p.ldr) + col_in;
        constexpr int JFIT = (352 - TM * TN * 16) / (TM * 16);
        constexpr int JB = TM == 3 ? TN : (JFIT < 1 ? 1 : (JFIT > TN ? TN : JFIT));
#pragma unroll
        for (int j0 = 0; j0 < TN; j0 += JB) {
            float rv[JB][TM][16];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t ro = lane_r + uint32_t(32 * i + 8 * (r >> 2) + (r & 3)) * uint32_t(p.ldr);
#pragma unroll
                    for (int jj = 0; jj < JB; ++jj)
                        if (j0 + jj < TN) rv[jj][i][r] = resid[ro + 32 * (j0 + jj)];
                }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t oo = lane_o + uint32_t(32 * i + 8 * (r >> 2) + (r & 3)) * uint32_t(p.ldo);
#pragma unroll
                    for (int jj = 0; jj < JB; ++jj)
                        if (j0 + jj < TN) out[oo + 32 * (j0 + jj)] = rv[jj][i][r] + acc[i][j0 + jj][r] + bias[j0 + jj];
                }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v = acc[i][j][r] + bias[j];
                const size_t uo = size_t(urow(i, r)) * p.ldo + (nw + 32 * j);
                if (EPI == EPI_BF16) {
                    (static_cast<bf16_t*>(p.out) + uo)[lane_o] = f_to_bf16(v);
                } else if (EPI == EPI_GELU_BF16) {
                    (static_cast<bf16_t*>(p.out) + uo)[lane_o] = f_to_bf16(gelu_tanh_f(v));
                } else {
                    (static_cast<float*>(p.out) + uo)[lane_o] = v;
                }
            }
}

// blockIdx -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): XCD x gets a
// contiguous range of the tile order, and inside it 8 row-tiles x consecutive column-tiles run together,
// so the tiles resident on one XCD share their A and B slabs in that XCD's L2.
__device__ __forceinline__ bool tile_of(int bid, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    const int xcd = bid % 8, idx = bid / 8;
    const int per = (total + 7) / 8;
    const int lin = xcd * per + idx;
    if (idx >= per || lin >= total) return false;
    constexpr int GM = 8;
    const int grp = lin / (GM * tiles_n), r = lin % (GM * tiles_n);
    const int gm = min(GM, tiles_m - grp * GM);
    *tm = grp * GM + r % gm;
    *tn = r / gm;
    return true;
}

// 16 bytes per lane from a buffer straight into LDS (buffer_load_dwordx4 ... offen lds): the address is the buffer's
// base (four scalar registers, set up once) + a per-lane 32-bit offset that never changes + a scalar offset that
// advances with the k-tile, so a copy costs the vector unit nothing (a flat 64-bit address per lane cost 1.5 vector
// additions per copy instruction, which a wavefront cannot overlap with its own MFMAs).  Offsets past the buffer's
// size read zeros.
#define DL_BLL16(rsrc, voff, soff, l)                                                                    \
    __builtin_amdgcn_raw_ptr_buffer_load_lds((rsrc), (__attribute__((address_space(3))) void*)(l), 16,  \
                                             int(voff), int(soff), 0, 0)
// third dword of a raw buffer resource on gfx9: 32-bit data format, no swizzle, offsets checked against the size
constexpr int kBufferFlags = 0x00020000;

// s_waitcnt with an explicit vector-memory count (6 bits, split 4 + 2 in the gfx9 encoding); expcnt is left
// unconstrained, lgkmcnt is either unconstrained or zero
#define DL_WAIT_VM(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
#define DL_WAIT_VM_LGKM0(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0x0 << 8))

// scheduling request for one phase of a k-tile: NM MFMAs with the NR fragment reads spread evenly over all but the
// last RT of them (those cover the latency of the last read) and the NC global->LDS copies spread over all of them
template <int NM, int NR, int NC, int RT, int M>
struct SchedEven {
    static __device__ __forceinline__ void run() {
        if constexpr (M < NM) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            constexpr int span = NM - RT;
            constexpr int r = M < span ? ((M + 1) * NR / span - M * NR / span) : 0;
            if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
            constexpr int c = (M + 1) * NC / NM - M * NC / NM;
            if constexpr (c > 0) __builtin_amdgcn_sched_group_barrier(0x020, c, 0);
            SchedEven<NM, NR, NC, RT, M + 1>::run();
        }
    }
};

// One output tile with its top-left corner at (m0, n0).  S0 .. S(NS-1) are the LDS stages; they must be distinct
// __shared__ arrays of at least (BM + BN) * 64 elements each.  The four wavefronts form a WM x (4 / WM) grid.  BNR is
// the number of columns the tile really owns (its stride in N): with BNR < BN the last BN - BNR columns are computed
// from the next tile's weight rows and never stored (128 x 144 of 160: 4096 x 1152 outputs are then exactly 256 tiles).
template <int BM, int BN, int EPI, int WM = 2, int BNR = BN, int NS = 2>
__device__ __forceinline__ void fast_tile(const GemmArgs& p, int m0, int n0, bf16_t* S0, bf16_t* S1, bf16_t* S2 = nullptr,
                                          bf16_t* S3 = nullptr) {
    constexpr int BK = 64, WN = 4 / WM;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int JA = BM / 32, JB = BN / 32;            // 1 KB copy blocks (8 rows x 128 B) per wavefront and k-tile
    constexpr int RT = TM * TN / 4;
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "whole MFMA tiles per wavefront");
    // the wavefront index is the same in every lane: as a scalar it keeps the LDS addresses of the copies (M0) and
    // everything else derived from it out of the vector unit
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // copy sources: block b = wave + 4*j of a tile holds rows 8b..8b+7, 128 bytes (one cache line, 64 k) each;
    // lane L lands at row 8b + L/8, physical 16-byte chunk L%8, and therefore fetches logical chunk
    // (L%8) ^ ((row/2)%8): a b128 fragment read serves 16 lanes (16 consecutive rows, 256 bytes of banks) at a time,
    // two rows fill the 64 banks once, so the swizzle has to differ between the 8 row PAIRS (with row%8 the counters
    // showed every second LDS cycle of the kernel as a bank conflict).  Rows past the matrix edge are clamped: they produce values that the epilogue never stores.
    uint32_t offA[JA], offB[JB];
#pragma unroll
    for (int j = 0; j < JA; ++j) {
        const int row = 8 * (wave + 4 * j) + (lane >> 3), lc = (lane & 7) ^ ((row >> 1) & 7);
        offA[j] = uint32_t((size_t(min(m0 + row, p.M - 1)) * p.lda + lc * 8) * 2);
    }
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        const int row = 8 * (wave + 4 * j) + (lane >> 3), lc = (lane & 7) ^ ((row >> 1) & 7);
        offB[j] = uint32_t((size_t(min(n0 + row, p.N - 1)) * p.ldb + lc * 8) * 2);
    }
    // the host only takes this path for operands below 4 GB
    const __amdgpu_buffer_rsrc_t gA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.A), 0, int(uint32_t(size_t(p.M) * p.lda * 2)), kBufferFlags);
    const __amdgpu_buffer_rsrc_t gB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.B), 0, int(uint32_t(size_t(p.N) * p.ldb * 2)), kBufferFlags);
    // fragment read offsets (elements) inside a stage, one per 16-wide k step
    const int lr = lane & 31, g2 = lane >> 5;
    int rdA[4], rdB[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int pc = (2 * kk + g2) ^ ((lr >> 1) & 7);
        rdA[kk] = ((BM / WM) * wm + lr) * BK + pc * 8;
        rdB[kk] = BM * BK + ((BN / WN) * wn + lr) * BK + pc * 8;
    }

    bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
    auto copyA = [&](bf16_t* S, int kt) {
#pragma unroll
        for (int j = 0; j < JA; ++j) DL_BLL16(gA, offA[j], kt * (BK * 2), S + (wave + 4 * j) * 512);
    };
    auto copyB = [&](bf16_t* S, int kt) {
#pragma unroll
        for (int j = 0; j < JB; ++j) DL_BLL16(gB, offB[j], kt * (BK * 2), S + BM * BK + (wave + 4 * j) * 512);
    };
    auto ldfrag = [&](bf16x8* a, bf16x8* b, const bf16_t* S, int kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(S + rdA[kk] + 32 * i * BK);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(S + rdB[kk] + 32 * j * BK);
    };
    // serpentine order over the accumulator tiles: from one MFMA to the next exactly one operand changes
    auto mma = [&](const bf16x8* a, const bf16x8* b) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jj = 0; jj < TN; ++jj) {
                const int j = (i & 1) ? TN - 1 - jj : jj;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
            }
    };
    auto interleave = [&](auto ncopy_c) {
        SchedEven<TM * TN, TM + TN, decltype(ncopy_c)::value, RT, 0>::run();
        __builtin_amdgcn_sched_barrier(0);
    };

    const int nk = p.K / BK;                             // host guarantees K % 128 == 0: nk is even and >= 2

    // One k-tile = four phases of TM*TN MFMAs (16-wide k steps), each overlapped with the fragment reads of the next
    // phase.  Before the last phase the wavefront waits for its own copies of k-tile kt+1 and for all of its LDS reads
    // and meets the others at the one barrier of the k-tile; past it (a) k-tile kt+1 has landed for everyone and
    // (b) nobody reads stage kt any more, so the copy of k-tile kt+NS into that stage starts right there: its A half
    // is spread over the last phase, its B half over the first phase of the next k-tile.  With NS = 2 stages a copy has
    // one k-tile of MFMAs to land (64 per wavefront for the large tiles: enough); a small tile's k-tile is 16-20 MFMAs,
    // so it runs NS = 4 stages and its copies have three k-tiles.
    // REM = k-tiles after this one, capped at NS (the steady state): with fewer than NS - 1 left the copy's B half has
    // nothing to fetch, with fewer than NS its A half; the wait leaves the copies younger than k-tile kt+1 in flight.
    auto ktile = [&](bf16_t* cur, bf16_t* nxt, bf16_t* prv, int kt, auto rem_c) {
        constexpr int REM = decltype(rem_c)::value;
        constexpr bool kB = REM >= NS - 1, kA = REM >= NS;
        ldfrag(a1, b1, cur, 1);
        if (kB) copyB(prv, kt + NS - 1);                 // second half of the copy begun in the previous k-tile
        mma(a0, b0);
        interleave(std::integral_constant<int, (kB ? JB : 0)>{});
        ldfrag(a0, b0, cur, 2);
        mma(a1, b1);
        interleave(std::integral_constant<int, 0>{});
        ldfrag(a1, b1, cur, 3);
        mma(a0, b0);
        interleave(std::integral_constant<int, 0>{});
        if constexpr (REM >= 1) {
            constexpr int younger = (REM - 1 < NS - 2 ? REM - 1 : NS - 2) * (JA + JB);
            DL_WAIT_VM_LGKM0(younger);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            ldfrag(a0, b0, nxt, 0);
            if (kA) copyA(cur, kt + NS);
            mma(a1, b1);
            interleave(std::integral_constant<int, (kA ? JA : 0)>{});
        } else {
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::integral_constant;
    if constexpr (NS == 2) {
        copyA(S0, 0); copyB(S0, 0);
        copyA(S1, 1);
        DL_WAIT_VM(JA);                                  // k-tile 0 has landed (this wavefront's share)
        __builtin_amdgcn_s_barrier();
        ldfrag(a0, b0, S0, 0);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + 2 < nk; kt += 2) {
            ktile(S0, S1, S1, kt, integral_constant<int, 2>{});
            ktile(S1, S0, S0, kt + 1, integral_constant<int, 2>{});
        }
        ktile(S0, S1, S1, kt, integral_constant<int, 1>{});
        ktile(S1, S0, S0, kt + 1, integral_constant<int, 0>{});
    } else {
        static_assert(NS == 4, "two or four stages");
        // the host takes this path only for nk >= 4; nk is even, so nk % 4 is 0 or 2
        copyA(S0, 0); copyB(S0, 0);
        copyA(S1, 1); copyB(S1, 1);
        copyA(S2, 2); copyB(S2, 2);
        copyA(S3, 3);
        DL_WAIT_VM(2 * (JA + JB) + JA);                  // k-tile 0 has landed (this wavefront's share)
        __builtin_amdgcn_s_barrier();
        ldfrag(a0, b0, S0, 0);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + 8 <= nk; kt += 4) {                  // whole groups of four in the steady state
            ktile(S0, S1, S3, kt, integral_constant<int, 4>{});
            ktile(S1, S2, S0, kt + 1, integral_constant<int, 4>{});
            ktile(S2, S3, S1, kt + 2, integral_constant<int, 4>{});
            ktile(S3, S0, S2, kt + 3, integral_constant<int, 4>{});
        }
        if (nk - kt == 4) {
            ktile(S0, S1, S3, kt, integral_constant<int, 3>{});
            ktile(S1, S2, S0, kt + 1, integral_constant<int, 2>{});
            ktile(S2, S3, S1, kt + 2, integral_constant<int, 1>{});
            ktile(S3, S0, S2, kt + 3, integral_constant<int, 0>{});
        } else {                                         // six left: two more in the steady state, then the last four
            ktile(S0, S1, S3, kt, integral_constant<int, 4>{});
            ktile(S1, S2, S0, kt + 1, integral_constant<int, 4>{});
            ktile(S2, S3, S1, kt + 2, integral_constant<int, 3>{});
            ktile(S3, S0, S2, kt + 3, integral_constant<int, 2>{});
            ktile(S0, S1, S3, kt + 4, integral_constant<int, 1>{});
            ktile(S1, S2, S0, kt + 5, integral_constant<int, 0>{});
        }
    }

    // wavefront tile wholly inside the matrix (SwiGLU: inside the packed gate/up columns): unpredicated epilogue
    const int mw = m0 + (BM / WM) * wm, nw = n0 + (BN / WN) * wn;
    const int n_end = min(p.N, n0 + BNR);
    if (mw + BM / WM <= p.M && nw + BN / WN <= n_end) store_tiles_full<EPI, TM, TN>(p, acc, mw, nw, lane);
    else store_tiles<EPI, TM, TN>(p, acc, mw, nw, lane, n_end);
}

// 128-row tiles leave room for two workgroups per compute unit (at most 80 KB of LDS and 128 accumulators each): one's
// prologue and epilogue hide under the other's main loop.
template <int BM, int BN, int EPI, int WM = 2, int BNR = BN, int NS = 2>
__global__ __launch_bounds__(256, (BM == 128 && BN <= 192 && NS == 2) ? 2 : 1) void gemm_fast(GemmArgs p) {
    __shared__ __attribute__((aligned(1024))) bf16_t S0[(BM + BN) * 64];
    __shared__ __attribute__((aligned(1024))) bf16_t S1[(BM + BN) * 64];
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BNR - 1) / BNR;
    int tm, tn;
    if (!tile_of(blockIdx.x, tiles_m, tiles_n, &tm, &tn)) return;
    if constexpr (NS == 4) {
        __shared__ __attribute__((aligned(1024))) bf16_t S2[(BM + BN) * 64];
        __shared__ __attribute__((aligned(1024))) bf16_t S3[(BM + BN) * 64];
        fast_tile<BM, BN, EPI, WM, BNR, 4>(p, tm * BM, tn * BNR, S0, S1, S2, S3);
    } else {
        fast_tile<BM, BN, EPI, WM, BNR, 2>(p, tm * BM, tn * BNR, S0, S1);
    }
}

// 256x256 tiles whose count is r full rounds of 256 workgroups plus a remainder of at most half a round: the last
// `n_split` tiles are computed as two 128x256 halves each, so the final round holds twice as many workgroups of
// half the work and ends in half the time instead of leaving most compute units idle for a whole tile time.
// Block b < n_big computes whole tile b (in the XCD-aware order), block n_big + 2 j + h half h of tile n_big + j.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_fast_split_tail(GemmArgs p, int n_big) {
    __shared__ __attribute__((aligned(1024))) bf16_t S0[512 * 64];
    __shared__ __attribute__((aligned(1024))) bf16_t S1[512 * 64];
    const int tiles_m = (p.M + 255) / 256, tiles_n = (p.N + 255) / 256;
    const int b = blockIdx.x;
    const int v = b < n_big ? b : n_big + ((b - n_big) >> 1);
    int tm, tn;
    if (!tile_of(v, tiles_m, tiles_n, &tm, &tn)) return;
    if (b < n_big) {
        fast_tile<256, 256, EPI>(p, tm * 256, tn * 256, S0, S1);
    } else {
        const int m0 = tm * 256 + 128 * ((b - n_big) & 1);
        if (m0 < p.M) fast_tile<128, 256, EPI>(p, m0, tn * 256, S0, S1);
    }
}

template <int BM, int BN, int EPI, int WM = 2, int BNR = BN, int NS = 2>
void launch_fast(const GemmArgs& a, hipStream_t st) {
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BNR - 1) / BNR);
    if (BM == 256 && BN == 256) {
        // tile_of deals tiles to 8 XCDs in equal shares: the split needs every virtual index below `tiles` to be valid
        const int rem = tiles % 256;
        if (tiles > 256 && tiles % 8 == 0 && rem > 0 && rem <= 128) {
            const int n_big = tiles - rem;
            hipLaunchKernelGGL((gemm_fast_split_tail<EPI>), dim3(n_big + 2 * rem), dim3(256), 0, st, a, n_big);
            return;
        }
    }
    const int grid = (tiles + 7) / 8 * 8;
    hipLaunchKernelGGL((gemm_fast<BM, BN, EPI, WM, BNR, NS>), dim3(grid), dim3(256), 0, st, a);
}

// tile shape for the fast path: 0 = 256x256, 1 = 192x256, 2 = 256x192, 3 = 192x192, 4 = 128x192, 5 = 128x128, 6 = 128x144.  Cost of
// a shape = rounds of workgroup slots x tile area / relative efficiency, the efficiencies fitted to measured launch
// times.  Shapes 0-3 hold one workgroup per compute unit (256 slots).  128x192 and 128x128 need at most 80 KB of LDS,
// so two workgroups share a compute unit (512 slots at half speed each, but one's prologue and epilogue hide under the
// other's main loop); they are considered only for short reductions or narrow outputs (the encoder's K = 1152 and
// N = 1152 GEMMs), where the large tiles leave compute units idle or spend their time outside the main loop.
int pick_tile(int M, int N, int K, bool need_even_cols) {
    const int bm[6] = {256, 192, 256, 192, 128, 128}, bn[6] = {256, 256, 192, 192, 192, 128};
    const double eff[6] = {1.0, 0.93, 0.93, 0.90, 1.34, 1.0};
    const bool small_ok = K <= 2048 || N <= 1536;
    int best = 0;
    double best_cost = 1e300;
    // 6 = 128x144 (stored columns; 160 in LDS), four wavefronts stacked in M: taken when it gives every compute unit at
    // most one tile (4096 x 1152 outputs = exactly 256 tiles), where the 128x128 tiles put two on some compute units
    // and all of them are bound by the global -> LDS rate (a 128x128 tile moves 32 KB per 16 MFMAs of a wavefront)
    if (!need_even_cols && small_ok) {
        const long tiles6 = long((M + 127) / 128) * ((N + 143) / 144);
        if (tiles6 <= 256 && K >= 2048) { best = 6; best_cost = 128.0 * 144.0 / 0.9; }
    }
    for (int c = 0; c < 6; ++c) {
        if (need_even_cols && bn[c] % 128 != 0) continue;   // gate/up pairs need an even number of 32-wide column tiles
        if (c >= 4 && !small_ok) continue;
        const long tiles = long((M + bm[c] - 1) / bm[c]) * ((N + bn[c] - 1) / bn[c]);
        const long slots = c >= 4 ? 512 : 256;
        const double rounds = tiles >= 3 * slots ? double(tiles) / double(slots) : double((tiles + slots - 1) / slots);
        const double cost = rounds * (c >= 4 ? 2.0 : 1.0) * bm[c] * bn[c] / eff[c];
        if (cost < best_cost) { best_cost = cost; best = c; }
    }
    return best;
}

template <int EPI>
void dispatch_fast(const GemmArgs& a, hipStream_t st) {
    const int t = pick_tile(a.M, a.N, a.K, EPI == EPI_SWIGLU_BF16);
    if (t == 0) launch_fast<256, 256, EPI>(a, st);
    else if (t == 1) launch_fast<192, 256, EPI>(a, st);
    else if (t == 5) launch_fast<128, 128, EPI>(a, st);
    else if constexpr (EPI != EPI_SWIGLU_BF16) {
        // odd numbers of 32-wide tile columns per wavefront cannot pair gate/up rows: never chosen for SwiGLU
        if (t == 2) launch_fast<256, 192, EPI>(a, st);
        else if (t == 3) launch_fast<192, 192, EPI>(a, st);
        else if (t == 6) launch_fast<128, 160, EPI, 4, 144, 4>(a, st);
        else launch_fast<128, 192, EPI>(a, st);
    }
}

}  // namespace

void gemm(const GemmArgs& a, hipStream_t st) {
    if (a.M <= 0 || a.N <= 0) return;
    // the residual epilogue addresses out and resid with 32-bit element offsets: split the rows of larger outputs
    if (a.epi == EPI_RESID_F32 && a.M > 1 &&
        (size_t(a.M) * size_t(a.ldo) >= (1ull << 31) || size_t(a.M) * size_t(a.ldr) >= (1ull << 31))) {
        const int m1 = a.M / 2;
        GemmArgs lo = a, hi = a;
        lo.M = m1;
        hi.M = a.M - m1;
        hi.A = a.A + size_t(m1) * a.lda;
        hi.out = static_cast<float*>(a.out) + size_t(m1) * a.ldo;
        hi.resid = a.resid + size_t(m1) * a.ldr;
        gemm(lo, st);
        gemm(hi, st);
        return;
    }
    // fast path: K in whole pairs of 64-wide steps, 16-byte aligned rows, enough rows to fill a tile
    const bool fast = a.K >= 128 && a.K % 128 == 0 && a.lda % 8 == 0 && a.ldb % 8 == 0 && a.M >= 96 && a.N >= 128 &&
                      a.epi != EPI_F32 &&
                      size_t(a.M) * a.lda * 2 < (1ull << 32) && size_t(a.N) * a.ldb * 2 < (1ull << 32);
    if (fast) {
        switch (a.epi) {
            case EPI_BF16: dispatch_fast<EPI_BF16>(a, st); return;
            case EPI_RESID_F32: dispatch_fast<EPI_RESID_F32>(a, st); return;
            case EPI_SWIGLU_BF16: dispatch_fast<EPI_SWIGLU_BF16>(a, st); return;
            case EPI_GELU_BF16: dispatch_fast<EPI_GELU_BF16>(a, st); return;
            default: break;
        }
    }
    // few rows: latency-bound, spread over N / 32 workgroups with the reduction split over 8 wavefronts
    const bool aligned_out = a.epi == EPI_BF16 || a.epi == EPI_GELU_BF16
                                 ? (a.ldo % 4 == 0 && reinterpret_cast<uintptr_t>(a.out) % 8 == 0)
                                 : (a.ldo % 4 == 0 && reinterpret_cast<uintptr_t>(a.out) % 16 == 0 &&
                                    (a.epi != EPI_RESID_F32 ||
                                     (a.ldr % 4 == 0 && reinterpret_cast<uintptr_t>(a.resid) % 16 == 0)));
    const bool few_rows = a.M <= 64 && a.K >= 64 && a.K % 64 == 0 && a.N % 32 == 0 && a.lda % 8 == 0 && a.ldb % 8 == 0 &&
                          a.epi != EPI_SWIGLU_BF16 && aligned_out &&
                          (!a.bias || reinterpret_cast<uintptr_t>(a.bias) % 8 == 0) &&
                          reinterpret_cast<uintptr_t>(a.A) % 16 == 0 && reinterpret_cast<uintptr_t>(a.B) % 16 == 0;
    if (few_rows) {
        dim3 grid(a.N / 32), block(512);
        switch (a.epi) {
            case EPI_BF16: hipLaunchKernelGGL(gemm_few_rows<EPI_BF16>, grid, block, 0, st, a); return;
            case EPI_RESID_F32: hipLaunchKernelGGL(gemm_few_rows<EPI_RESID_F32>, grid, block, 0, st, a); return;
            case EPI_GELU_BF16: hipLaunchKernelGGL(gemm_few_rows<EPI_GELU_BF16>, grid, block, 0, st, a); return;
            default: hipLaunchKernelGGL(gemm_few_rows<EPI_F32>, grid, block, 0, st, a); return;
        }
    }
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    dim3 grid(tiles), block(256);
    switch (a.epi) {
        case EPI_BF16: hipLaunchKernelGGL(gemm_generic<EPI_BF16>, grid, block, 0, st, a); break;
        case EPI_RESID_F32: hipLaunchKernelGGL(gemm_generic<EPI_RESID_F32>, grid, block, 0, st, a); break;
        case EPI_SWIGLU_BF16: hipLaunchKernelGGL(gemm_generic<EPI_SWIGLU_BF16>, grid, block, 0, st, a); break;
        case EPI_GELU_BF16: hipLaunchKernelGGL(gemm_generic<EPI_GELU_BF16>, grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL(gemm_generic<EPI_F32>, grid, block, 0, st, a); break;
    }
}

}  // namespace dlk
