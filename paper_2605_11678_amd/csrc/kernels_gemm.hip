// BF16 GEMM on gfx950 matrix cores: C[M,N] = A[M,K] * B[N,K]^T with fused epilogues.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants for A and
// for B alike (a lane supplies 8 consecutive k of one row / one column), so tiles go
// global -> registers -> LDS -> MFMA without any transposition.  Weights are stored [N,K]
// by the packer for exactly this reason.
//
// Tiling: 256 threads = 4 wavefronts of 64 lanes in a 2x2 grid; block tile 128x128, K step 64;
// each wavefront owns 64x64 = 2x2 MFMA tiles of 32x32 (4 x 16 fp32 accumulators per lane).
// The next K tile is fetched into registers while the current one is multiplied out of LDS.
// Accumulator layout of a 32x32 tile: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4.
#include "kernels.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_LD = BK + 8;   // row stride in elements: 144 bytes keeps 16-byte alignment and staggers banks

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }
__device__ __forceinline__ float gelu_tanh_f(float x) {
    const float c = 0.7978845608028654f;   // sqrt(2/pi)
    return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float bf16_to_f(bf16_t v) { return __uint_as_float(uint32_t(v) << 16); }
__device__ __forceinline__ bf16_t f_to_bf16(float f) {
    __bf16 b = (__bf16)f;   // hardware round-to-nearest-even
    return *reinterpret_cast<bf16_t*>(&b);
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs p) {
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

}  // namespace

void gemm(const GemmArgs& a, hipStream_t st) {
    if (a.M <= 0 || a.N <= 0) return;
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    dim3 grid(tiles), block(256);
    switch (a.epi) {
        case EPI_BF16: hipLaunchKernelGGL(gemm_kernel<EPI_BF16>, grid, block, 0, st, a); break;
        case EPI_RESID_F32: hipLaunchKernelGGL(gemm_kernel<EPI_RESID_F32>, grid, block, 0, st, a); break;
        case EPI_SWIGLU_BF16: hipLaunchKernelGGL(gemm_kernel<EPI_SWIGLU_BF16>, grid, block, 0, st, a); break;
        case EPI_GELU_BF16: hipLaunchKernelGGL(gemm_kernel<EPI_GELU_BF16>, grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL(gemm_kernel<EPI_F32>, grid, block, 0, st, a); break;
    }
}

}  // namespace dlk
