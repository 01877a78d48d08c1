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

constexpr int UNITS_PER_WAVE = 2;

// a "unit" is one output element; for SwiGLU it needs two weight rows (gate and up)
template <int EPI>
__global__ __launch_bounds__(256) void gemv_kernel(GemvArgs p) {
    extern __shared__ __attribute__((aligned(16))) bf16_t sx[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nchunk = p.K >> 3;
    for (int c = tid; c < nchunk; c += 256)
        reinterpret_cast<u32x4*>(sx)[c] = reinterpret_cast<const u32x4*>(p.x)[c];
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

}  // namespace dlk
