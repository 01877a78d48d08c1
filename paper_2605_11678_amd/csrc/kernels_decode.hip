// Single-token (decode) linear maps: out[N] = B[N,K] * x[K].  The work is one pass over the weight
// bytes, so it is bound by HBM: one wavefront owns whole rows, every lane streams 16-byte pieces of
// the row and multiplies them with the activation vector held in LDS, then the 64 partial sums are
// folded with cross-lane shuffles.  Same epilogues as the GEMM.
#include "kernels.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }
__device__ __forceinline__ float gelu_tanh_f(float x) {
    const float c = 0.7978845608028654f;
    return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float bf16_to_f(bf16_t v) { return __uint_as_float(uint32_t(v) << 16); }
__device__ __forceinline__ bf16_t f_to_bf16(float f) {
    __bf16 b = (__bf16)f;
    return *reinterpret_cast<bf16_t*>(&b);
}
__device__ __forceinline__ float lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

__device__ __forceinline__ float dot8(u32x4 w, u32x4 x) {
    float s = lo(w[0]) * lo(x[0]);
    s = fmaf(hi(w[0]), hi(x[0]), s);
    s = fmaf(lo(w[1]), lo(x[1]), s);
    s = fmaf(hi(w[1]), hi(x[1]), s);
    s = fmaf(lo(w[2]), lo(x[2]), s);
    s = fmaf(hi(w[2]), hi(x[2]), s);
    s = fmaf(lo(w[3]), lo(x[3]), s);
    s = fmaf(hi(w[3]), hi(x[3]), s);
    return s;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sum over a 256-thread block; every thread gets the result
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

constexpr int UNITS_PER_WAVE = 2;

// a "unit" is one output element; for SwiGLU it needs two weight rows (gate and up)
template <int EPI>
__global__ __launch_bounds__(256) void gemv_kernel(GemvArgs p) {
    extern __shared__ __attribute__((aligned(16))) bf16_t sx[];
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nchunk = p.K >> 3;
    if (p.xf) {
        // fused normalisation: every workgroup normalises the (small) input vector for itself
        float mean = 0.0f;
        if (p.norm_kind == 1) {
            float s = 0.0f;
            for (int i = tid; i < p.K; i += 256) s += p.xf[i];
            mean = block_sum_256(s, red) / float(p.K);
        }
        float ss = 0.0f;
        for (int i = tid; i < p.K; i += 256) {
            const float c = p.xf[i] - mean;
            ss += c * c;
        }
        const float inv = rsqrtf(block_sum_256(ss, red) / float(p.K) + p.eps);
        for (int i = tid; i < p.K; i += 256) {
            float v = (p.xf[i] - mean) * inv * bf16_to_f(p.ng[i]);
            if (p.norm_kind == 1) v += bf16_to_f(p.nb[i]);
            sx[i] = f_to_bf16(v);
        }
    } else {
        for (int c = tid; c < nchunk; c += 256)
            reinterpret_cast<u32x4*>(sx)[c] = reinterpret_cast<const u32x4*>(p.x)[c];
    }
    __syncthreads();

    const int n_units = (EPI == EPI_SWIGLU_BF16) ? p.N / 2 : p.N;
    const int u0 = (blockIdx.x * 4 + wave) * UNITS_PER_WAVE;
    constexpr int ROWS = (EPI == EPI_SWIGLU_BF16) ? 2 * UNITS_PER_WAVE : UNITS_PER_WAVE;
    const bf16_t* rows[ROWS];
    bool valid[UNITS_PER_WAVE];
#pragma unroll
    for (int u = 0; u < UNITS_PER_WAVE; ++u) {
        const int unit = u0 + u;
        valid[u] = unit < n_units;
        const int uu = valid[u] ? unit : 0;
        if (EPI == EPI_SWIGLU_BF16) {
            const int pr = (uu / 32) * 64 + (uu % 32);
            rows[2 * u] = p.B + size_t(pr) * p.ldb;
            rows[2 * u + 1] = p.B + size_t(pr + 32) * p.ldb;
        } else {
            rows[u] = p.B + size_t(uu) * p.ldb;
        }
    }
    float acc[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = 0.0f;
    for (int c = lane; c < nchunk; c += 64) {
        const u32x4 xv = reinterpret_cast<const u32x4*>(sx)[c];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const u32x4 w = reinterpret_cast<const u32x4*>(rows[r])[c];
            acc[r] += dot8(w, xv);
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = wave_sum(acc[r]);
    if (lane != 0) return;
#pragma unroll
    for (int u = 0; u < UNITS_PER_WAVE; ++u) {
        if (!valid[u]) continue;
        const int n = u0 + u;
        if (EPI == EPI_SWIGLU_BF16) {
            static_cast<bf16_t*>(p.out)[n] = f_to_bf16(silu_f(acc[2 * u]) * acc[2 * u + 1]);
        } else {
            const float v = acc[u] + (p.bias ? bf16_to_f(p.bias[n]) : 0.0f);
            if (EPI == EPI_BF16) static_cast<bf16_t*>(p.out)[n] = f_to_bf16(v);
            else if (EPI == EPI_GELU_BF16) static_cast<bf16_t*>(p.out)[n] = f_to_bf16(gelu_tanh_f(v));
            else if (EPI == EPI_RESID_F32) static_cast<float*>(p.out)[n] = p.resid[n] + v;
            else static_cast<float*>(p.out)[n] = v;
        }
    }
}


typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// One wavefront = one KV head x one 64-position tile.  Transposed formulation as in the prefill kernel:
// S^T = K Q^T with the query heads of the group as MFMA columns (columns >= group are zero),
// O^T = V^T P^T.  Every K / V element is used by exactly one wavefront, so operands are loaded from global
// memory straight into MFMA fragment layout; no LDS.
template <int DHP>
__global__ __launch_bounds__(64) void decode_attn_partial(DecodeAttnArgs p, float scale_log2, int n_tiles) {
    const int lane = threadIdx.x, lq = lane & 31, g2 = lane >> 5;
    const int tile = blockIdx.x, kvh = blockIdx.y;
    const int group = p.Hq / p.Hkv;
    const int j0 = tile * 64;
    const int h = kvh * group + lq;                    // this lane's query head (valid if lq < group)
    bf16x8 qf[DHP / 16];
#pragma unroll
    for (int kk = 0; kk < DHP / 16; ++kk) {
        const int e = 16 * kk + 8 * g2;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (lq < group && e < p.dh) v = *reinterpret_cast<const u32x4*>(p.q + size_t(h) * p.dh + e);
        qf[kk] = *reinterpret_cast<bf16x8*>(&v);
    }
    const bf16_t* kbase = p.k + size_t(kvh) * p.k_head_stride;
    const bf16_t* vbase = p.vt + size_t(kvh) * p.v_head_stride;
    f32x16 accS[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[i][r] = 0.0f;
        const int row = j0 + 32 * i + lq;
        const bf16_t* krow = kbase + size_t(min(row, p.S - 1)) * p.ldk;
#pragma unroll
        for (int kk = 0; kk < DHP / 16; ++kk) {
            const int e = 16 * kk + 8 * g2;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row < p.S && e < p.dh) v = *reinterpret_cast<const u32x4*>(krow + e);
            accS[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&v), qf[kk], accS[i], 0, 0, 0);
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kv = j0 + 32 * i + 8 * (r >> 2) + 4 * g2 + (r & 3);
            accS[i][r] = kv < p.S ? accS[i][r] : -INFINITY;
            mx = fmaxf(mx, accS[i][r]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));            // the tile holds at least one valid position
    const float ms = mx * scale_log2;
    float psum = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(accS[i][8 * t2 + j], scale_log2, -ms));
                psum += pv;
                pf[i][t2][j] = (__bf16)pv;
            }
    psum += __shfl_xor(psum, 32, 64);
    f32x16 accO[DHP / 32];
#pragma unroll
    for (int dt = 0; dt < DHP / 32; ++dt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[dt][r] = 0.0f;
        const int e = 32 * dt + lq;
        const bf16_t* vrow = vbase + size_t(min(e, p.dh - 1)) * p.ldv + j0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                const int o = 32 * i + 16 * t2 + 4 * g2;
                u32x2 lo = {0u, 0u}, hi = {0u, 0u};
                if (e < p.dh) {                        // rows of the cache are padded to whole tiles: in bounds
                    lo = *reinterpret_cast<const u32x2*>(vrow + o);
                    hi = *reinterpret_cast<const u32x2*>(vrow + o + 8);
                    // positions >= S hold stale memory: zero them (their probabilities are zero, but 0 * NaN is not)
                    const int n_lo = p.S - (j0 + o), n_hi = n_lo - 8;
                    if (n_lo < 4) { if (n_lo <= 0) lo[0] = 0u; else if (n_lo == 1) lo[0] &= 0xFFFFu; if (n_lo <= 2) lo[1] = 0u; else if (n_lo == 3) lo[1] &= 0xFFFFu; }
                    if (n_hi < 4) { if (n_hi <= 0) hi[0] = 0u; else if (n_hi == 1) hi[0] &= 0xFFFFu; if (n_hi <= 2) hi[1] = 0u; else if (n_hi == 3) hi[1] &= 0xFFFFu; }
                }
                u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
                accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&av), pf[i][t2], accO[dt], 0, 0, 0);
            }
    }
    if (lq >= group) return;
    float* dst = p.partial + (size_t(h) * n_tiles + tile) * (p.dh + 2);
    if (g2 == 0) { dst[0] = mx; dst[1] = psum; }
#pragma unroll
    for (int dt = 0; dt < DHP / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int e = 32 * dt + 8 * (r >> 2) + 4 * g2 + (r & 3);
            if (e < p.dh) dst[2 + e] = accO[dt][r];
        }
}

// merges the tiles of one head: out[e] = sum_t w_t o_t[e] / sum_t w_t l_t, w_t = 2^((m_t - M) * scale)
__global__ __launch_bounds__(128) void decode_attn_merge(DecodeAttnArgs p, float scale_log2, int n_tiles) {
    const int h = blockIdx.x, e = threadIdx.x;
    const float* src = p.partial + size_t(h) * n_tiles * (p.dh + 2);
    float M = -INFINITY;
    for (int t = 0; t < n_tiles; ++t) M = fmaxf(M, src[size_t(t) * (p.dh + 2)]);
    float l = 0.0f, o = 0.0f;
    for (int t = 0; t < n_tiles; ++t) {
        const float* s = src + size_t(t) * (p.dh + 2);
        const float w = __builtin_amdgcn_exp2f((s[0] - M) * scale_log2);
        l += w * s[1];
        if (e < p.dh) o += w * s[2 + e];
    }
    if (e < p.dh) p.out[size_t(h) * p.dh + e] = f_to_bf16(o / l);
}

}  // namespace

void gemv(const GemvArgs& a, hipStream_t st) {
    if (a.N <= 0) return;
    const int n_units = (a.epi == EPI_SWIGLU_BF16) ? a.N / 2 : a.N;
    const int per_block = 4 * UNITS_PER_WAVE;
    dim3 grid((n_units + per_block - 1) / per_block), block(256);
    const size_t lds = size_t(a.K) * 2;
    switch (a.epi) {
        case EPI_BF16: hipLaunchKernelGGL(gemv_kernel<EPI_BF16>, grid, block, lds, st, a); break;
        case EPI_RESID_F32: hipLaunchKernelGGL(gemv_kernel<EPI_RESID_F32>, grid, block, lds, st, a); break;
        case EPI_SWIGLU_BF16: hipLaunchKernelGGL(gemv_kernel<EPI_SWIGLU_BF16>, grid, block, lds, st, a); break;
        case EPI_GELU_BF16: hipLaunchKernelGGL(gemv_kernel<EPI_GELU_BF16>, grid, block, lds, st, a); break;
        default: hipLaunchKernelGGL(gemv_kernel<EPI_F32>, grid, block, lds, st, a); break;
    }
}

uint64_t decode_attention_workspace_bytes(int max_seq, int Hq, int dh) {
    const uint64_t n_tiles = (uint64_t(max_seq) + 63) / 64;
    return uint64_t(Hq) * n_tiles * uint64_t(dh + 2) * 4;
}

void decode_attention(const DecodeAttnArgs& a, hipStream_t st) {
    if (a.S <= 0) return;
    const int n_tiles = (a.S + 63) / 64;
    const float scale_log2 = 1.4426950408889634f / sqrtf(float(a.dh));
    dim3 grid(n_tiles, a.Hkv), block(64);
    if (a.dh <= 64) hipLaunchKernelGGL(decode_attn_partial<64>, grid, block, 0, st, a, scale_log2, n_tiles);
    else if (a.dh <= 96) hipLaunchKernelGGL(decode_attn_partial<96>, grid, block, 0, st, a, scale_log2, n_tiles);
    else hipLaunchKernelGGL(decode_attn_partial<128>, grid, block, 0, st, a, scale_log2, n_tiles);
    hipLaunchKernelGGL(decode_attn_merge, dim3(a.Hq), dim3(128), 0, st, a, scale_log2, n_tiles);
}

}  // namespace dlk
