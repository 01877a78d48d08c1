// Device code of the row normalisation, shared by the stand-alone kernel (one workgroup per row) and the
// single-token matrix-vector kernel, which normalises its input vector itself instead of reading the output of
// a separate launch.  Both therefore round identically.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace dlk {
namespace normdev {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sum over a 256-thread block; every thread gets the result
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();               // red may still be read from a previous call
    if (lane == 0) red[wave] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// The first KEEP float4 pieces of a thread's share of the row, with their gains (and biases): all requested
// before anything is used, with the index clamped instead of a predicate, so the workgroup pays one memory
// round trip for a row of up to 4096 elements.
constexpr int KEEP = 4;
template <int KIND>
struct RowPieces {
    float4 v[KEEP];
    uint2 gk[KEEP], bk[KEEP];
    __device__ __forceinline__ void request(const float4* row, const uint16_t* g, const uint16_t* b, int nv) {
        const int tid = threadIdx.x;
#pragma unroll
        for (int j = 0; j < KEEP; ++j) {
            const int i = tid + 256 * j, ic = i < nv ? i : 0;
            v[j] = row[ic];
            gk[j] = reinterpret_cast<const uint2*>(g)[ic];
            if (KIND == 1) bk[j] = reinterpret_cast<const uint2*>(b)[ic];
        }
    }
};

// KIND 0: RMSNorm (g); 1: LayerNorm (g, b).  256 threads, d % 4 == 0.  emit(i, o0, o1, o2, o3) receives the four
// normalised elements 4i .. 4i+3.  `red` is 4 floats of LDS.
template <int KIND, typename Emit>
__device__ __forceinline__ void norm_row(RowPieces<KIND>& rp, const float4* row, const uint16_t* g, const uint16_t* b,
                                         int d, float eps, float* red, Emit emit) {
    const int tid = threadIdx.x, nv = d >> 2;
#pragma unroll
    for (int j = 0; j < KEEP; ++j)
        if (tid + 256 * j >= nv) rp.v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    float mean = 0.0f;
    if (KIND == 1) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < KEEP; ++j) s += (rp.v[j].x + rp.v[j].y) + (rp.v[j].z + rp.v[j].w);
        for (int i = tid + 256 * KEEP; i < nv; i += 256) {
            const float4 t = row[i];
            s += (t.x + t.y) + (t.z + t.w);
        }
        mean = block_sum_256(s, red) / float(d);
    }
    float ss = 0.0f;
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
        if (tid + 256 * j < nv) {
            const float a0 = rp.v[j].x - mean, a1 = rp.v[j].y - mean, a2 = rp.v[j].z - mean, a3 = rp.v[j].w - mean;
            ss += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    }
    for (int i = tid + 256 * KEEP; i < nv; i += 256) {
        const float4 t = row[i];
        const float a0 = t.x - mean, a1 = t.y - mean, a2 = t.z - mean, a3 = t.w - mean;
        ss += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
    const float inv = rsqrtf(block_sum_256(ss, red) / float(d) + eps);
    auto scale = [&](int i, const float4& t, const uint2& gg, const uint2& bb) {
        float o0 = (t.x - mean) * inv * __uint_as_float(gg.x << 16);
        float o1 = (t.y - mean) * inv * __uint_as_float(gg.x & 0xFFFF0000u);
        float o2 = (t.z - mean) * inv * __uint_as_float(gg.y << 16);
        float o3 = (t.w - mean) * inv * __uint_as_float(gg.y & 0xFFFF0000u);
        if (KIND == 1) {
            o0 += __uint_as_float(bb.x << 16);
            o1 += __uint_as_float(bb.x & 0xFFFF0000u);
            o2 += __uint_as_float(bb.y << 16);
            o3 += __uint_as_float(bb.y & 0xFFFF0000u);
        }
        emit(i, o0, o1, o2, o3);
    };
#pragma unroll
    for (int j = 0; j < KEEP; ++j)
        if (tid + 256 * j < nv) scale(tid + 256 * j, rp.v[j], rp.gk[j], rp.bk[j]);
    for (int i = tid + 256 * KEEP; i < nv; i += 256) {
        uint2 bb = make_uint2(0u, 0u);
        if (KIND == 1) bb = reinterpret_cast<const uint2*>(b)[i];
        scale(i, row[i], reinterpret_cast<const uint2*>(g)[i], bb);
    }
}

}  // namespace normdev
}  // namespace dlk
