// Row-wise kernels that move activations once through HBM: normalisation (wavefront reductions),
// rotary embedding + KV scatter after the QKV projection, embedding lookup, greedy argmax.
#include "kernels.hpp"
#include "norm_device.hpp"

namespace dlk {

namespace {

__device__ __forceinline__ float bf16_to_f(bf16_t v) { return __uint_as_float(uint32_t(v) << 16); }
__device__ __forceinline__ bf16_t f_to_bf16(float f) {
    __bf16 b = (__bf16)f;
    return *reinterpret_cast<bf16_t*>(&b);
}

// One 256-thread workgroup per row; rows are read as float4 (d % 4 == 0) and kept in registers between the
// reduction and the scaling pass when they fit (d <= 4096), so a row is read from memory once.
template <int KIND, bool OUT_F32>
__global__ __launch_bounds__(256) void norm_kernel(const float* __restrict__ x, const bf16_t* __restrict__ g,
                                                   const bf16_t* __restrict__ b, void* __restrict__ out, int d,
                                                   float eps) {
    __shared__ float red[4];
    const float4* row = reinterpret_cast<const float4*>(x + size_t(blockIdx.x) * d);
    normdev::RowPieces<KIND> rp;
    rp.request(row, g, b, d >> 2);
    normdev::norm_row<KIND>(rp, row, g, b, d, eps, red, [&](int i, float o0, float o1, float o2, float o3) {
        if (OUT_F32) {
            reinterpret_cast<float4*>(static_cast<float*>(out) + size_t(blockIdx.x) * d)[i] = make_float4(o0, o1, o2, o3);
        } else {
            uint2 pk;
            pk.x = uint32_t(f_to_bf16(o0)) | (uint32_t(f_to_bf16(o1)) << 16);
            pk.y = uint32_t(f_to_bf16(o2)) | (uint32_t(f_to_bf16(o3)) << 16);
            reinterpret_cast<uint2*>(static_cast<bf16_t*>(out) + size_t(blockIdx.x) * d)[i] = pk;
        }
    });
}

// Rows of at most 2048 elements: one WAVEFRONT per row (four rows per workgroup), the row and its gains held in
// registers, both reductions done with cross-lane shuffles only - no LDS, no workgroup barrier.  With one workgroup per
// row a 1152-element row (the encoder's) leaves most threads one piece each and spends its time in the two barriers of
// every reduction: 12.1 us per launch (between events) at 4096 x 1152 against 9.6 us this way.
template <int KIND, bool OUT_F32>
__global__ __launch_bounds__(256) void norm_wave_kernel(const float* __restrict__ x, const bf16_t* __restrict__ g,
                                                        const bf16_t* __restrict__ b, void* __restrict__ out, int T, int d,
                                                        float eps) {
    constexpr int MAXV = 8;                            // float4 pieces per lane
    const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= T) return;
    const int nv = d >> 2;
    const float4* row = reinterpret_cast<const float4*>(x + size_t(r) * d);
    float4 v[MAXV];
    uint2 gk[MAXV], bk[MAXV];
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {                   // everything requested before anything is used; index clamped
        const int i = lane + 64 * j, ic = i < nv ? i : 0;
        v[j] = row[ic];
        gk[j] = reinterpret_cast<const uint2*>(g)[ic];
        if (KIND == 1) bk[j] = reinterpret_cast<const uint2*>(b)[ic];
    }
    float mean = 0.0f;
    if (KIND == 1) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < MAXV; ++j)
            if (lane + 64 * j < nv) s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
        mean = normdev::wave_sum(s) / float(d);
    }
    float ss = 0.0f;
#pragma unroll
    for (int j = 0; j < MAXV; ++j)
        if (lane + 64 * j < nv) {
            const float a0 = v[j].x - mean, a1 = v[j].y - mean, a2 = v[j].z - mean, a3 = v[j].w - mean;
            ss += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    const float inv = rsqrtf(normdev::wave_sum(ss) / float(d) + eps);
#pragma unroll
    for (int j = 0; j < MAXV; ++j) {
        const int i = lane + 64 * j;
        if (i >= nv) continue;
        float o0 = (v[j].x - mean) * inv * __uint_as_float(gk[j].x << 16);
        float o1 = (v[j].y - mean) * inv * __uint_as_float(gk[j].x & 0xFFFF0000u);
        float o2 = (v[j].z - mean) * inv * __uint_as_float(gk[j].y << 16);
        float o3 = (v[j].w - mean) * inv * __uint_as_float(gk[j].y & 0xFFFF0000u);
        if (KIND == 1) {
            o0 += __uint_as_float(bk[j].x << 16);
            o1 += __uint_as_float(bk[j].x & 0xFFFF0000u);
            o2 += __uint_as_float(bk[j].y << 16);
            o3 += __uint_as_float(bk[j].y & 0xFFFF0000u);
        }
        if (OUT_F32) {
            reinterpret_cast<float4*>(static_cast<float*>(out) + size_t(r) * d)[i] = make_float4(o0, o1, o2, o3);
        } else {
            uint2 pk;
            pk.x = uint32_t(f_to_bf16(o0)) | (uint32_t(f_to_bf16(o1)) << 16);
            pk.y = uint32_t(f_to_bf16(o2)) | (uint32_t(f_to_bf16(o3)) << 16);
            reinterpret_cast<uint2*>(static_cast<bf16_t*>(out) + size_t(r) * d)[i] = pk;
        }
    }
}

__global__ __launch_bounds__(256) void cast_kernel(const float* __restrict__ x, bf16_t* __restrict__ out, uint64_t n) {
    for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += uint64_t(gridDim.x) * 256)
        out[i] = f_to_bf16(x[i]);
}

__global__ __launch_bounds__(256) void mean_pool_kernel(const float* __restrict__ x, float* __restrict__ y, int group,
                                                        int d) {
    const int t = blockIdx.x;
    const float inv = 1.0f / float(group);
    for (int i = threadIdx.x; i < d; i += 256) {
        float s = 0.0f;
        for (int j = 0; j < group; ++j) s += x[(size_t(t) * group + j) * d + i];
        y[size_t(t) * d + i] = s * inv;
    }
}

__global__ __launch_bounds__(256) void axpy_kernel(float* __restrict__ y, float alpha, const float* __restrict__ x,
                                                   uint64_t n) {
    for (uint64_t i = uint64_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += uint64_t(gridDim.x) * 256)
        y[i] = fmaf(alpha, x[i], y[i]);
}

__global__ __launch_bounds__(256) void time_embed_kernel(const float* __restrict__ x, float* __restrict__ y, float tval,
                                                         int d) {
    const int t = blockIdx.x, half = d >> 1;
    for (int i = threadIdx.x; i < d; i += 256) {
        const int j = i < half ? i : i - half;
        const float ang = 1000.0f * tval * exp2f(-float(j) / float(half) * 13.287712379549449f);   // log2(10000)
        y[size_t(t) * d + i] = x[size_t(t) * d + i] + (i < half ? sinf(ang) : cosf(ang));
    }
}

// Rotary embedding of q (in place) and k (to the cache, or in place): one workgroup per token.  The angle
// depends on (position, i) only, so each thread evaluates one sin/cos pair and reuses it for every head.
// FUSE_V (single-token passes): the block also scatters its token's V row into the transposed cache, which
// saves the second launch where there is nothing to tile.
template <bool FUSE_V>
__global__ __launch_bounds__(256) void rope_kernel(QkvPostArgs p) {
    const int t = blockIdx.x, pos = p.pos0 + t;
    bf16_t* row = p.qkv + size_t(t) * p.n_qkv;
    const int half = p.dh >> 1;
    const int lanes = half < 256 ? half : 256;            // threads that own a frequency index
    const int i = threadIdx.x % lanes, hg = threadIdx.x / lanes, n_hg = 256 / lanes;
    if (FUSE_V) {
        const int ncol = p.Hkv * p.dh;
        for (int col = threadIdx.x; col < ncol; col += 256) {
            const int g = col / p.dh, e = col % p.dh;
            p.vt_out[size_t(g) * p.vt_head_stride + size_t(e) * p.vt_ld + pos] = row[p.v_off + col];
        }
    }
    if (!FUSE_V && (half & 7) == 0 && half <= 128) {
        // multi-token passes: the token's sin/cos table goes to LDS once (one evaluation per frequency), then every
        // thread rotates 8 pairs per step with 16-byte loads and stores: (i..i+7) and (i+half..i+half+7) of one head
        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
        __shared__ float s_cs[128], s_sn[128];
        if (int(threadIdx.x) < half) {
            float sn = 0.0f, cs = 1.0f;
            if (p.theta > 0.0f)
                sincosf(float(pos) * exp2f(-2.0f * float(threadIdx.x) / float(p.dh) * log2f(p.theta)), &sn, &cs);
            s_cs[threadIdx.x] = cs;
            s_sn[threadIdx.x] = sn;
        }
        __syncthreads();
        const int per_head = half >> 3;
        const int nq = (p.theta > 0.0f && p.q_off >= 0) ? p.Hq : 0;
        const int nk = (p.k_out || p.theta > 0.0f) ? p.Hkv : 0;
        for (int task = threadIdx.x; task < (nq + nk) * per_head; task += 256) {
            const int hh = task / per_head, c = (task - hh * per_head) * 8;
            const bf16_t* src;
            bf16_t* dst;
            if (hh < nq) {
                dst = row + p.q_off + hh * p.dh;
                src = dst;
            } else {
                const int g = hh - nq;
                src = row + p.k_off + g * p.dh;
                dst = p.k_out ? p.k_out + size_t(g) * p.k_head_stride + size_t(pos) * p.dh : row + p.k_off + g * p.dh;
            }
            const u32x4 lo = *reinterpret_cast<const u32x4*>(src + c), hi = *reinterpret_cast<const u32x4*>(src + c + half);
            u32x4 olo, ohi;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float a0 = __uint_as_float(lo[w] << 16), a1 = __uint_as_float(lo[w] & 0xFFFF0000u);
                const float b0 = __uint_as_float(hi[w] << 16), b1 = __uint_as_float(hi[w] & 0xFFFF0000u);
                const float c0 = s_cs[c + 2 * w], c1 = s_cs[c + 2 * w + 1], n0 = s_sn[c + 2 * w], n1 = s_sn[c + 2 * w + 1];
                olo[w] = uint32_t(f_to_bf16(a0 * c0 - b0 * n0)) | (uint32_t(f_to_bf16(a1 * c1 - b1 * n1)) << 16);
                ohi[w] = uint32_t(f_to_bf16(a0 * n0 + b0 * c0)) | (uint32_t(f_to_bf16(a1 * n1 + b1 * c1)) << 16);
            }
            *reinterpret_cast<u32x4*>(dst + c) = olo;
            *reinterpret_cast<u32x4*>(dst + c + half) = ohi;
        }
        return;
    }
    float sn = 0.0f, cs = 1.0f;
    if (p.theta > 0.0f) {
        const float ang = float(pos) * exp2f(-2.0f * float(i) / float(p.dh) * log2f(p.theta));
        sincosf(ang, &sn, &cs);
    }
    if (hg >= n_hg) return;
    if (p.theta > 0.0f && p.q_off >= 0) {
        for (int h = hg; h < p.Hq; h += n_hg) {
            bf16_t* q = row + p.q_off + h * p.dh;
            for (int ii = i; ii < half; ii += lanes) {
                const float a = bf16_to_f(q[ii]), b = bf16_to_f(q[ii + half]);
                q[ii] = f_to_bf16(a * cs - b * sn);
                q[ii + half] = f_to_bf16(a * sn + b * cs);
            }
        }
    }
    if (p.k_out || p.theta > 0.0f) {
        for (int g = hg; g < p.Hkv; g += n_hg) {
            const bf16_t* k = row + p.k_off + g * p.dh;
            bf16_t* dst = p.k_out ? p.k_out + size_t(g) * p.k_head_stride + size_t(pos) * p.dh : row + p.k_off + g * p.dh;
            for (int ii = i; ii < half; ii += lanes) {
                const float a = bf16_to_f(k[ii]), b = bf16_to_f(k[ii + half]);
                dst[ii] = f_to_bf16(a * cs - b * sn);
                dst[ii + half] = f_to_bf16(a * sn + b * cs);
            }
        }
    }
}

// V -> V^T: a 64-token x 64-feature tile goes through LDS so that both the reads (token rows) and the
// writes (feature rows of the transposed cache, 64 consecutive positions = 128 bytes) are contiguous.  Both sides move
// 16 bytes per thread and instruction: two unpredicated loads per thread (token and column clamped into the matrix, so
// nothing waits between them), and one store of 8 consecutive positions gathered from LDS; positions past T and a
// destination that is not 16-byte aligned (pos0 not a multiple of 8) fall back to 2-byte stores.
__global__ __launch_bounds__(256) void v_transpose_kernel(QkvPostArgs p) {
    __shared__ __attribute__((aligned(16))) bf16_t tile[64][72];     // 144-byte rows: 16-byte aligned, staggered banks
    const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;          // first token / first column of V (= g*dh + e)
    const int ncol = p.Hkv * p.dh;                                  // a multiple of 8
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    u32x4 v[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int idx = threadIdx.x + 256 * k, r = idx >> 3, cc = (idx & 7) * 8;
        const int tr = min(t0 + r, p.T - 1), col = c0 + cc < ncol ? c0 + cc : 0;
        v[k] = *reinterpret_cast<const u32x4*>(p.qkv + size_t(tr) * p.n_qkv + p.v_off + col);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int idx = threadIdx.x + 256 * k, r = idx >> 3, cc = (idx & 7) * 8;
        *reinterpret_cast<u32x4*>(&tile[r][cc]) = v[k];
    }
    __syncthreads();
    const bool aligned = (p.pos0 & 7) == 0 && (p.vt_ld & 7) == 0 && (p.vt_head_stride & 7) == 0;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int idx = threadIdx.x + 256 * k, c = idx >> 3, rc = (idx & 7) * 8;   // feature, first of 8 positions
        const int col = c0 + c;
        if (col >= ncol || t0 + rc >= p.T) continue;
        const int g = col / p.dh, e = col % p.dh;
        bf16_t* dst = p.vt_out + size_t(g) * p.vt_head_stride + size_t(e) * p.vt_ld + p.pos0 + t0 + rc;
        if (aligned && t0 + rc + 8 <= p.T) {
            u32x4 o;
#pragma unroll
            for (int w = 0; w < 4; ++w) o[w] = uint32_t(tile[rc + 2 * w][c]) | (uint32_t(tile[rc + 2 * w + 1][c]) << 16);
            *reinterpret_cast<u32x4*>(dst) = o;
        } else {
            for (int j = 0; j < 8 && t0 + rc + j < p.T; ++j) dst[j] = tile[rc + j][c];
        }
    }
}

__global__ __launch_bounds__(256) void embed_kernel(const bf16_t* __restrict__ table, int d,
                                                    const int32_t* __restrict__ token_dev, int token_host,
                                                    float* __restrict__ x_out) {
    const int tok = token_dev ? *token_dev : token_host;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d; i += gridDim.x * 256)
        x_out[i] = bf16_to_f(table[size_t(tok) * d + i]);
}

// Greedy choice and the next input in one launch: index of the largest of v[0..n) (lowest index on ties) written to
// out0 and, if given, out1; then, if a table is given, row `index` of the bf16 table [*, d] widened to fp32 into
// x_out.  One 1024-thread workgroup; a thread's values are requested eight at a time with clamped indices before
// any is compared.
__device__ __forceinline__ void take_better(float& best, int& bi, float x, int i) {
    if (x > best || (x == best && i < bi)) { best = x; bi = i; }
}
__global__ __launch_bounds__(1024) void argmax_embed_kernel(const float* __restrict__ v, int n, int32_t* __restrict__ out0,
                                                            int32_t* __restrict__ out1, const bf16_t* __restrict__ table,
                                                            int d, float* __restrict__ x_out) {
    __shared__ float sv[16];
    __shared__ int si[16];
    __shared__ int s_tok;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float best = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int base = 0; base < n; base += 8 * 1024) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = base + tid + 1024 * j;
            x[j] = v[i < n ? i : n - 1];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = base + tid + 1024 * j;
            if (i < n) take_better(best, bi, x[j], i);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        take_better(best, bi, ob, oi);
    }
    if (lane == 0) {
        sv[wave] = best;
        si[wave] = bi;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < 16; ++w) take_better(best, bi, sv[w], si[w]);
        const int tok = bi == 0x7FFFFFFF ? 0 : bi;
        *out0 = tok;
        if (out1) *out1 = tok;
        s_tok = tok;
    }
    if (!table) return;
    __syncthreads();
    const bf16_t* row = table + size_t(s_tok) * d;
    for (int i = tid; i < d; i += 1024) x_out[i] = bf16_to_f(row[i]);
}

}  // namespace

void norm_rows(int kind, const float* x, const bf16_t* g, const bf16_t* b, void* out, bool out_f32, int T, int d,
               float eps, hipStream_t st) {
    if (T <= 0) return;
    if (d <= 2048 && T >= 4) {
        // short rows, several of them: one wavefront per row
        dim3 grid((T + 3) / 4), block(256);
        if (kind == 0) {
            if (out_f32) hipLaunchKernelGGL((norm_wave_kernel<0, true>), grid, block, 0, st, x, g, b, out, T, d, eps);
            else hipLaunchKernelGGL((norm_wave_kernel<0, false>), grid, block, 0, st, x, g, b, out, T, d, eps);
        } else {
            if (out_f32) hipLaunchKernelGGL((norm_wave_kernel<1, true>), grid, block, 0, st, x, g, b, out, T, d, eps);
            else hipLaunchKernelGGL((norm_wave_kernel<1, false>), grid, block, 0, st, x, g, b, out, T, d, eps);
        }
        return;
    }
    dim3 grid(T), block(256);
    if (kind == 0) {
        if (out_f32) hipLaunchKernelGGL((norm_kernel<0, true>), grid, block, 0, st, x, g, b, out, d, eps);
        else hipLaunchKernelGGL((norm_kernel<0, false>), grid, block, 0, st, x, g, b, out, d, eps);
    } else {
        if (out_f32) hipLaunchKernelGGL((norm_kernel<1, true>), grid, block, 0, st, x, g, b, out, d, eps);
        else hipLaunchKernelGGL((norm_kernel<1, false>), grid, block, 0, st, x, g, b, out, d, eps);
    }
}

void cast_f32_bf16(const float* x, bf16_t* out, uint64_t n, hipStream_t st) {
    if (n == 0) return;
    const uint64_t blocks = (n + 255) / 256;
    dim3 grid(unsigned(blocks < 4096 ? blocks : 4096)), block(256);
    hipLaunchKernelGGL(cast_kernel, grid, block, 0, st, x, out, n);
}

void mean_pool_rows(const float* x, float* y, int T_out, int group, int d, hipStream_t st) {
    if (T_out <= 0) return;
    hipLaunchKernelGGL(mean_pool_kernel, dim3(T_out), dim3(256), 0, st, x, y, group, d);
}

// Register-only MFMA loop: every wavefront keeps 16 independent 32x32 accumulator tiles busy with operands that
// never leave registers.  pattern 0: all-zero operands; 1: values in [1, 2) with hashed mantissa and sign.
namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t probe_u32x4;
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters, int pattern) {
    probe_bf16x8 a[4], b[4];
    uint32_t s = threadIdx.x * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        probe_u32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s = s * 1664525u + 1013904223u;
            const uint32_t lo = 0x3F80u | ((s >> 9) & 0x7Fu) | ((s >> 3) & 0x8000u);
            s = s * 1664525u + 1013904223u;
            const uint32_t hi = 0x3F80u | ((s >> 9) & 0x7Fu) | ((s >> 3) & 0x8000u);
            w[j] = pattern ? (lo | (hi << 16)) : 0u;
        }
        if (i < 4) a[i] = *reinterpret_cast<probe_bf16x8*>(&w);
        else b[i - 4] = *reinterpret_cast<probe_bf16x8*>(&w);
    }
    probe_f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = sum;
}
}  // namespace

double mfma_rate_probe(float* out, int blocks, int iters, int pattern, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, st, out, iters, pattern);
    return double(blocks) * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
}

void axpy_f32(float* y, float alpha, const float* x, uint64_t n, hipStream_t st) {
    if (n == 0) return;
    const uint64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(axpy_kernel, dim3(unsigned(blocks < 4096 ? blocks : 4096)), dim3(256), 0, st, y, alpha, x, n);
}

void add_time_embedding(const float* x, float* y, float tval, int T, int d, hipStream_t st) {
    if (T <= 0) return;
    hipLaunchKernelGGL(time_embed_kernel, dim3(T), dim3(256), 0, st, x, y, tval, d);
}

void qkv_post(const QkvPostArgs& a, hipStream_t st) {
    if (a.T <= 0) return;
    if (a.T <= 4) {
        hipLaunchKernelGGL(rope_kernel<true>, dim3(a.T), dim3(256), 0, st, a);
        return;
    }
    // without a rotary embedding and without a cache to append K to there is nothing for the first kernel to do
    if (a.theta > 0.0f || a.k_out)
        hipLaunchKernelGGL(rope_kernel<false>, dim3(a.T), dim3(256), 0, st, a);
    hipLaunchKernelGGL(v_transpose_kernel, dim3((a.T + 63) / 64, (a.Hkv * a.dh + 63) / 64), dim3(256), 0, st, a);
}

void embed_row(const bf16_t* table, int d, const int32_t* token_dev, int token_host, float* x_out, hipStream_t st) {
    hipLaunchKernelGGL(embed_kernel, dim3((d + 255) / 256), dim3(256), 0, st, table, d, token_dev, token_host, x_out);
}

void argmax_f32(const float* logits, int n, int32_t* token_dev, int32_t* token_copy, const bf16_t* table, int d,
                float* x_out, hipStream_t st) {
    if (n <= 0) return;
    hipLaunchKernelGGL(argmax_embed_kernel, dim3(1), dim3(1024), 0, st, logits, n, token_dev, token_copy, table, d, x_out);
}

}  // namespace dlk
