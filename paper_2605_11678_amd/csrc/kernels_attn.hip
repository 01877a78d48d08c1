// Flash-style attention on gfx950 matrix cores (online softmax, no score matrix in memory).
//
// Works on the TRANSPOSED problem so that nothing has to change layout between the two matrix
// products: a wavefront owns 32 queries and computes S^T = K * Q^T (keys are MFMA rows, queries
// MFMA columns).  In the 32x32 accumulator layout a lane then holds 16 scores of ONE query
// (column l%32; rows 8*(r/4) + 4*(l/32) + r%4), so the softmax row reductions are in-lane plus one
// exchange with lane l^32, the running max / sum / rescale are per-lane scalars, and the
// probabilities P^T are already in B-operand position for O^T = V^T * P^T (8 consecutive
// accumulator registers = the 8 k-values a lane supplies).  V is kept transposed in memory
// ([feature][position]) so V^T tiles are plain row loads.
//
// Block: 4 wavefronts x 32 queries = 128 queries of one head; K/V tiles of 64 positions in LDS.
// Head dims 64 / 72 / 128 run as DHP = 64 / 96 / 128 with zero padding (exact zeros contribute nothing).
#include "kernels.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

namespace {

constexpr int BQ = 128, BKV = 64;

template <int DHP>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs p, float scale_log2) {
    constexpr int KLD = DHP + 8;     // sK row stride (elements)
    constexpr int VLD = BKV + 8;     // sV row stride
    __shared__ __attribute__((aligned(16))) bf16_t sK[BKV * KLD];
    __shared__ __attribute__((aligned(16))) bf16_t sV[DHP * VLD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, g2 = lane >> 5;
    const int h = blockIdx.y, kvh = h / (p.Hq / p.Hkv);
    const int q0 = blockIdx.x * BQ;
    const int tq = q0 + 32 * wave + lq;               // this lane's query (token index)
    const int qpos = p.q_pos0 + tq;

    // Q fragments (B operand): 8 consecutive features per lane and k-step
    bf16x8 qf[DHP / 16];
    {
        const bf16_t* qrow = p.q + size_t(tq) * p.ldq + size_t(h) * p.dh;
#pragma unroll
        for (int kk = 0; kk < DHP / 16; ++kk) {
            const int e = 16 * kk + 8 * g2;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (tq < p.T && e < p.dh) v = *reinterpret_cast<const u32x4*>(qrow + e);
            qf[kk] = *reinterpret_cast<bf16x8*>(&v);
        }
    }

    f32x16 accO[DHP / 32];
#pragma unroll
    for (int dt = 0; dt < DHP / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[dt][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const bf16_t* kbase = p.k + size_t(kvh) * p.k_head_stride;
    const bf16_t* vbase = p.vt + size_t(kvh) * p.v_head_stride;
    int kv_end = p.S;
    if (p.causal) {
        const int last_q = p.q_pos0 + min(q0 + BQ, p.T);   // one past the last query position of the block
        kv_end = min(p.S, last_q);
    }

    for (int j0 = 0; j0 < kv_end; j0 += BKV) {
        __syncthreads();
        // K tile: 64 positions x DHP features
        for (int c = tid; c < BKV * (DHP / 8); c += 256) {
            const int row = c / (DHP / 8), kc = (c % (DHP / 8)) * 8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (j0 + row < p.S && kc < p.dh)
                v = *reinterpret_cast<const u32x4*>(kbase + size_t(j0 + row) * p.ldk + kc);
            *reinterpret_cast<u32x4*>(&sK[row * KLD + kc]) = v;
        }
        // V^T tile: DHP features x 64 positions; positions >= S are zeroed (stale memory must not reach the MFMA)
        for (int c = tid; c < DHP * (BKV / 8); c += 256) {
            const int e = c / (BKV / 8), jc = (c % (BKV / 8)) * 8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (e < p.dh && j0 + jc < p.S) {
                v = *reinterpret_cast<const u32x4*>(vbase + size_t(e) * p.ldv + j0 + jc);
                const int nvalid = p.S - (j0 + jc);          // > 0
                if (nvalid < 8) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        if (2 * w >= nvalid) v[w] = 0u;
                        else if (2 * w + 1 >= nvalid) v[w] &= 0x0000FFFFu;
                    }
                }
            }
            *reinterpret_cast<u32x4*>(&sV[e * VLD + jc]) = v;
        }
        __syncthreads();

        // S^T tile: 64 keys x 32 queries per wavefront
        f32x16 accS[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[i][r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < DHP / 16; ++kk) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sK[(32 * i + lq) * KLD + 16 * kk + 8 * g2]);
                accS[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], accS[i], 0, 0, 0);
            }
        }

        // mask, online softmax (base-2 exponent; scale_log2 = log2(e) / sqrt(dh))
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = j0 + 32 * i + 8 * (r >> 2) + 4 * g2 + (r & 3);
                const bool ok = kv < p.S && (!p.causal || kv <= qpos);
                const float s = ok ? accS[i][r] * scale_log2 : -INFINITY;
                accS[i][r] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
        const float alpha = exp2f(m_run - m_use);
        m_run = m_new;
        float psum = 0.0f;
        bf16x8 pf[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float pv = exp2f(accS[i][8 * t + j] - m_use);
                    psum += pv;
                    pf[i][t][j] = (__bf16)pv;
                }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < DHP / 32; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) accO[dt][r] *= alpha;

        // O^T += V^T * P^T
#pragma unroll
        for (int dt = 0; dt < DHP / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const bf16_t* vr = &sV[(32 * dt + lq) * VLD + 32 * i + 16 * t + 4 * g2];
                    const u32x2 lo = *reinterpret_cast<const u32x2*>(vr);
                    const u32x2 hi = *reinterpret_cast<const u32x2*>(vr + 8);
                    u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
                    accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&av), pf[i][t],
                                                                       accO[dt], 0, 0, 0);
                }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (tq >= p.T) return;
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    bf16_t* orow = p.out + size_t(tq) * p.ldo + size_t(h) * p.dh;
#pragma unroll
    for (int dt = 0; dt < DHP / 32; ++dt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int e0 = 32 * dt + 8 * rg + 4 * g2;
            if (e0 < p.dh) {
                bf16x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = (__bf16)(accO[dt][4 * rg + j] * inv);
                *reinterpret_cast<bf16x4*>(orow + e0) = o;
            }
        }
}

}  // namespace

void attention(const AttnArgs& a, hipStream_t st) {
    if (a.T <= 0 || a.S <= 0) return;
    dim3 grid((a.T + BQ - 1) / BQ, a.Hq), block(256);
    const float scale_log2 = 1.4426950408889634f / sqrtf(float(a.dh));
    if (a.dh <= 64) hipLaunchKernelGGL(attn_kernel<64>, grid, block, 0, st, a, scale_log2);
    else if (a.dh <= 96) hipLaunchKernelGGL(attn_kernel<96>, grid, block, 0, st, a, scale_log2);
    else hipLaunchKernelGGL(attn_kernel<128>, grid, block, 0, st, a, scale_log2);
}

}  // namespace dlk
