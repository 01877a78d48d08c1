// Single-token (decode) linear maps: out[N] = B[N,K] * x[K].  The work is one pass over the weight
// bytes, so it is bound by HBM: one wavefront owns whole rows, every lane streams 16-byte pieces of
// the row and multiplies them with the activation vector held in LDS, then the 64 partial sums are
// folded with cross-lane shuffles.  Same epilogues as the GEMM.
#include "kernels.hpp"
#include "norm_device.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

// same forms as in the GEMM epilogues, so that a single-token pass rounds like a multi-token one
__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float gelu_tanh_f(float x) {
    const float c2 = 2.0f * 0.7978845608028654f;
    const float u2 = c2 * (x + 0.044715f * x * x * x);
    return x * __builtin_amdgcn_rcpf(1.0f + __expf(-u2));
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


// a "unit" is one output element; for SwiGLU it needs two weight rows (gate and up)
// ROWS: rows a wavefront streams together (4: two SwiGLU units = 2 gate + 2 up rows, or four plain units; 2 for
// matrices with so few rows that 4 would leave compute units without a workgroup)
// NORM: -1 the input vector is p.x (bf16); 0 / 1: it is RMSNorm / LayerNorm of the fp32 row p.norm_x, computed by
// every workgroup for itself (the row and its gains sit in L2; this saves a launch per product)
template <int EPI, int ROWS, int NORM>
__global__ __launch_bounds__(256) void gemv_kernel(GemvArgs p) {
    extern __shared__ __attribute__((aligned(16))) bf16_t sx[];
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nchunk = p.K >> 3;

    constexpr bool PAIRED = EPI == EPI_SWIGLU_BF16 || EPI == EPI_QKV_POST;     // a unit needs two weight rows
    const int n_units = PAIRED ? p.N / 2 : p.N;
    constexpr int UNITS_PER_WAVE = PAIRED ? ROWS / 2 : ROWS;
    const int u0 = (blockIdx.x * 4 + wave) * UNITS_PER_WAVE;
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
        } else if (EPI == EPI_QKV_POST) {
            // unit = rotary pair: features i and i + dh/2 of one head
            const int half = p.post.dh >> 1, r0 = (uu / half) * p.post.dh + (uu % half);
            rows[2 * u] = p.B + size_t(r0) * p.ldb;
            rows[2 * u + 1] = p.B + size_t(r0 + half) * p.ldb;
        } else {
            rows[u] = p.B + size_t(uu) * p.ldb;
        }
    }
    // Weight pieces are fetched 4 rows x CU pieces (of 64 chunks = 1 KB) at a time = 16 independent 16-byte loads
    // per lane, double-buffered, and the FIRST group is requested before the input vector is copied to LDS.  Wavefronts start at different pieces of their rows (rotation).
    // Every weight byte is used exactly once per launch: the loads carry the non-temporal hint, so the stream does not
    // displace what the caches hold for the small operands (8B-class layer, single token: 88.1 -> 83.6 us; the same
    // hint on the K / V^T loads of the single-token attention made that kernel slower and is not used there).
    constexpr int CU = 4;
    const int n_it = nchunk >> 6;
    const bool piped = (nchunk & 63) == 0 && (n_it % CU) == 0;
    const int rot = piped ? (blockIdx.x * 4 + wave) % n_it : 0;
    auto chunk_of = [&](int it) {
        int idx = it + rot;
        idx = idx >= n_it ? idx - n_it : idx;
        return lane + 64 * idx;
    };
    auto load_group = [&](int it, u32x4 (&w)[ROWS][CU]) {
#pragma unroll
        for (int u = 0; u < CU; ++u) {
            const int c = chunk_of(it + u);
#pragma unroll
            for (int r = 0; r < ROWS; ++r) w[r][u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rows[r]) + c);
        }
    };
    u32x4 wA[ROWS][CU], wB[ROWS][CU];
    if constexpr (NORM >= 0) {
        // the row is requested first and the first weight group right behind it: memory returns loads in order, so
        // the normalisation runs while the weights are still on their way
        const float4* row = reinterpret_cast<const float4*>(p.norm_x);
        normdev::RowPieces<NORM> rp;
        rp.request(row, p.norm_g, p.norm_b, p.K >> 2);
        if (piped) load_group(0, wA);
        normdev::norm_row<NORM>(rp, row, p.norm_g, p.norm_b, p.K, p.norm_eps, red,
                                [&](int i, float o0, float o1, float o2, float o3) {
                                    uint2 pk;
                                    pk.x = uint32_t(f_to_bf16(o0)) | (uint32_t(f_to_bf16(o1)) << 16);
                                    pk.y = uint32_t(f_to_bf16(o2)) | (uint32_t(f_to_bf16(o3)) << 16);
                                    reinterpret_cast<uint2*>(sx)[i] = pk;
                                });
    } else {
        if (piped) load_group(0, wA);
        for (int c = tid; c < nchunk; c += 256)
            reinterpret_cast<u32x4*>(sx)[c] = reinterpret_cast<const u32x4*>(p.x)[c];
    }
    __syncthreads();

    float acc[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) acc[r] = 0.0f;
    auto consume = [&](int it, const u32x4 (&w)[ROWS][CU]) {
#pragma unroll
        for (int u = 0; u < CU; ++u) {
            const u32x4 xv = reinterpret_cast<const u32x4*>(sx)[chunk_of(it + u)];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) acc[r] += dot8(w[r][u], xv);
        }
    };
    if (piped) {
        int it = 0;
        while (true) {
            if (it + CU < n_it) load_group(it + CU, wB);
            consume(it, wA);
            it += CU;
            if (it >= n_it) break;
            if (it + CU < n_it) load_group(it + CU, wA);
            consume(it, wB);
            it += CU;
            if (it >= n_it) break;
        }
    } else {
        for (int c = lane; c < nchunk; c += 64) {
            const u32x4 xv = reinterpret_cast<const u32x4*>(sx)[c];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rows[r]) + c);
                acc[r] += dot8(w, xv);
            }
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
        } else if (EPI == EPI_QKV_POST) {
            const QkvPostArgs& q = p.post;
            const int half = q.dh >> 1, hh = n / half, i = n % half, r0 = hh * q.dh + i, r1 = r0 + half;
            // the projection is rounded to bf16 first, like the stand-alone product whose output the rotary kernel reads
            const float a = bf16_to_f(f_to_bf16(acc[2 * u] + (p.bias ? bf16_to_f(p.bias[r0]) : 0.0f)));
            const float b = bf16_to_f(f_to_bf16(acc[2 * u + 1] + (p.bias ? bf16_to_f(p.bias[r1]) : 0.0f)));
            bf16_t* row = static_cast<bf16_t*>(p.out);
            const int pos = q.pos0, dq = q.Hq * q.dh, dkv = q.Hkv * q.dh;
            if (r0 >= dq + dkv) {                         // V: into the transposed cache, no rotation
                const int g = (r0 - dq - dkv) / q.dh;
                bf16_t* dst = q.vt_out + size_t(g) * q.vt_head_stride + pos;
                dst[size_t(i) * q.vt_ld] = f_to_bf16(a);
                dst[size_t(i + half) * q.vt_ld] = f_to_bf16(b);
            } else {
                float sn = 0.0f, cs = 1.0f;
                if (q.theta > 0.0f) sincosf(float(pos) * exp2f(-2.0f * float(i) / float(q.dh) * log2f(q.theta)), &sn, &cs);
                bf16_t* dst = row + r0;                   // Q (q_off = 0) or K kept in the row
                if (r0 >= dq && q.k_out) dst = q.k_out + size_t((r0 - dq) / q.dh) * q.k_head_stride + size_t(pos) * q.dh + i;
                dst[0] = f_to_bf16(a * cs - b * sn);
                dst[half] = f_to_bf16(a * sn + b * cs);
            }
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

// One wavefront = one KV head x one 64-position tile.  Transposed formulation as in the prefill kernel:
// S^T = K Q^T with the query heads of the group as MFMA columns (columns >= group are zero),
// O^T = V^T P^T.  Every K / V element is used by exactly one wavefront, so operands are loaded from global
// memory straight into MFMA fragment layout; no LDS.  All loads of the tile (K and V) are issued before the
// first MFMA and nothing tests a loaded value before it is used, so the wavefront pays one memory latency,
// not one per fragment.  Key rows sit on MFMA rows with bits 2 and 3 swapped (as in the prefill kernel), which
// makes every V^T fragment one 16-byte load.  Addresses are clamped instead of predicated: K rows past S
// repeat row S-1 and are masked to -inf; V^T positions past S are stale but finite (the cache is zeroed when
// the module is finalised and its rows are padded to whole tiles) and meet zero probabilities.
template <int DHP>
__global__ __launch_bounds__(64) void decode_attn_partial(DecodeAttnArgs p, float scale_log2, int n_tiles) {
    const int lane = threadIdx.x, lq = lane & 31, g2 = lane >> 5;
    const int krow = (lq & 0x13) | ((lq & 4) << 1) | ((lq & 8) >> 1);
    const int tile = blockIdx.x, kvh = blockIdx.y;
    const int group = p.Hq / p.Hkv;
    const int j0 = tile * 64;
    const int h = kvh * group + lq;                    // this lane's query head (valid if lq < group)
    const bf16_t* kbase = p.k + size_t(kvh) * p.k_head_stride;
    const bf16_t* vbase = p.vt + size_t(kvh) * p.v_head_stride;
    u32x4 kf[2][DHP / 16], vf[DHP / 32][4], qv[DHP / 16];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const bf16_t* kr = kbase + size_t(min(j0 + 32 * i + krow, p.S - 1)) * p.ldk;
#pragma unroll
        for (int kk = 0; kk < DHP / 16; ++kk) {
            const int e = 16 * kk + 8 * g2;
            kf[i][kk] = *reinterpret_cast<const u32x4*>(kr + (e < p.dh ? e : 0));
        }
    }
#pragma unroll
    for (int kk = 0; kk < DHP / 16; ++kk) {
        const int e = 16 * kk + 8 * g2;
        qv[kk] = *reinterpret_cast<const u32x4*>(p.q + size_t(min(h, p.Hq - 1)) * p.dh + (e < p.dh ? e : 0));
    }
#pragma unroll
    for (int dt = 0; dt < DHP / 32; ++dt) {
        const bf16_t* vr = vbase + size_t(min(32 * dt + lq, p.dh - 1)) * p.ldv + j0 + 8 * g2;
#pragma unroll
        for (int q = 0; q < 4; ++q) vf[dt][q] = *reinterpret_cast<const u32x4*>(vr + 16 * q);   // q = 2*i + t2
    }
    // keep every load above this line: left alone, the scheduler sinks the V^T loads below the score MFMAs and the
    // wavefront pays a second memory latency for them
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 qf[DHP / 16];
#pragma unroll
    for (int kk = 0; kk < DHP / 16; ++kk) {
        const int e = 16 * kk + 8 * g2;
        const u32x4 z = {0u, 0u, 0u, 0u};
        const u32x4 v = (lq < group && e < p.dh) ? qv[kk] : z;     // padding columns and padding features are zero
        qf[kk] = *reinterpret_cast<const bf16x8*>(&v);
    }
    f32x16 accS[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[i][r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < DHP / 16; ++kk)
            accS[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&kf[i][kk]), qf[kk], accS[i], 0, 0, 0);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // accumulator row 8*(r/4) + 4*g2 + r%4 holds key 16*(r/8) + 8*g2 + r%8
            const int kv = j0 + 32 * i + 16 * (r >> 3) + 8 * g2 + (r & 7);
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
#pragma unroll
        for (int q = 0; q < 4; ++q)
            accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&vf[dt][q]), pf[q >> 1][q & 1],
                                                               accO[dt], 0, 0, 0);
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

// merges the tiles of one head: out[e] = sum_t w_t o_t[e] / sum_t w_t l_t, w_t = 2^((m_t - M) * scale).
// 4 x 128 threads: thread (e, part) folds the tiles t = part, part + 4, ... with a running maximum (its loads do
// not depend on one another, so they are in flight together), then the four parts are folded through LDS in
// fixed order.  Every tile holds at least one valid position, so every m_t is finite.
__global__ __launch_bounds__(512) void decode_attn_merge(DecodeAttnArgs p, float scale_log2, int n_tiles) {
    __shared__ float s_m[4], s_l[4], s_o[4][128];
    const int h = blockIdx.x, e = threadIdx.x & 127, part = threadIdx.x >> 7;
    const float* src = p.partial + size_t(h) * n_tiles * (p.dh + 2);
    float M = -INFINITY, l = 0.0f, o = 0.0f;
#pragma unroll 4
    for (int t = part; t < n_tiles; t += 4) {
        const float* s = src + size_t(t) * (p.dh + 2);
        const float m = s[0], lt = s[1], ot = e < p.dh ? s[2 + e] : 0.0f;
        const float Mn = fmaxf(M, m);
        const float a = __builtin_amdgcn_exp2f((M - Mn) * scale_log2), b = __builtin_amdgcn_exp2f((m - Mn) * scale_log2);
        l = l * a + lt * b;
        o = o * a + ot * b;
        M = Mn;
    }
    if (e == 0) { s_m[part] = M; s_l[part] = l; }
    s_o[part][e] = o;
    __syncthreads();
    if (part != 0 || e >= p.dh) return;
    float Mt = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float L = 0.0f, O = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float w = __builtin_amdgcn_exp2f((s_m[k] - Mt) * scale_log2);   // a part without tiles has m = -inf: w = 0
        L += w * s_l[k];
        O += w * s_o[k][e];
    }
    p.out[size_t(h) * p.dh + e] = f_to_bf16(O / L);
}

}  // namespace

template <int EPI, int NORM>
void launch_gemv_n(const GemvArgs& a, int n_units, hipStream_t st) {
    const size_t lds = size_t(a.K) * 2;
    constexpr bool SW = EPI == EPI_SWIGLU_BF16 || EPI == EPI_QKV_POST;     // two rows per unit
    // 4 rows per wavefront unless that gives fewer than two workgroups per compute unit
    const int blocks4 = (n_units + (SW ? 8 : 16) - 1) / (SW ? 8 : 16);
    if (EPI == EPI_SWIGLU_BF16 || blocks4 >= 512) {
        hipLaunchKernelGGL((gemv_kernel<EPI, 4, NORM>), dim3(blocks4), dim3(256), lds, st, a);
    } else {
        hipLaunchKernelGGL((gemv_kernel<EPI, 2, NORM>), dim3((n_units + (SW ? 4 : 8) - 1) / (SW ? 4 : 8)), dim3(256), lds,
                           st, a);
    }
}

template <int EPI>
void launch_gemv(const GemvArgs& a, int n_units, hipStream_t st) {
    // the products that follow a normalisation: QKV, the feed-forward's first map, the output head
    constexpr bool kAfterNorm = EPI == EPI_QKV_POST || EPI == EPI_SWIGLU_BF16 || EPI == EPI_GELU_BF16 || EPI == EPI_F32;
    if constexpr (kAfterNorm) {
        if (a.norm_x && a.norm_kind == 0) return launch_gemv_n<EPI, 0>(a, n_units, st);
        if (a.norm_x) return launch_gemv_n<EPI, 1>(a, n_units, st);
    }
    launch_gemv_n<EPI, -1>(a, n_units, st);
}

void gemv(const GemvArgs& a, hipStream_t st) {
    if (a.N <= 0) return;
    const int n_units = (a.epi == EPI_SWIGLU_BF16 || a.epi == EPI_QKV_POST) ? a.N / 2 : a.N;
    switch (a.epi) {
        case EPI_QKV_POST: launch_gemv<EPI_QKV_POST>(a, n_units, st); break;
        case EPI_BF16: launch_gemv<EPI_BF16>(a, n_units, st); break;
        case EPI_RESID_F32: launch_gemv<EPI_RESID_F32>(a, n_units, st); break;
        case EPI_SWIGLU_BF16: launch_gemv<EPI_SWIGLU_BF16>(a, n_units, st); break;
        case EPI_GELU_BF16: launch_gemv<EPI_GELU_BF16>(a, n_units, st); break;
        default: launch_gemv<EPI_F32>(a, n_units, st); break;
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
    hipLaunchKernelGGL(decode_attn_merge, dim3(a.Hq), dim3(512), 0, st, a, scale_log2, n_tiles);
}

}  // namespace dlk
