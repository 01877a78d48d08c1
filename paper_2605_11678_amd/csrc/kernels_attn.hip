// Flash-style attention on gfx950 matrix cores (online softmax, no score matrix in memory).
//
// Works on the TRANSPOSED problem so that nothing has to change layout between the two matrix
// products: a wavefront owns 32 queries and computes S^T = K * Q^T (keys are MFMA rows, queries
// MFMA columns).  In the 32x32 accumulator layout a lane then holds 16 scores of ONE query
// (column l%32; rows 8*(r/4) + 4*(l/32) + r%4), so the softmax row reductions are in-lane plus one
// exchange with lane l^32, the running max / sum / rescale are per-lane scalars, and the
// probabilities P^T are already in B-operand position for O^T = V^T * P^T (8 consecutive
// accumulator registers = the 8 k-values a lane supplies).  The keys of a score tile are assigned to
// MFMA rows with bits 2 and 3 of the row index swapped, which makes those 8 k-values 8 consecutive keys.
// V is kept transposed in memory ([feature][position]) so V^T tiles are plain row loads.
//
// Block: 4 wavefronts, K/V tiles of 64 positions in LDS, two stages; the next tile is copied global -> LDS
// directly (no staging registers) while the current one is multiplied.  Two work splits:
//   HEADS = true  (grouped-query attention, group size a multiple of 4): the four wavefronts are four
//                  query heads of ONE KV head on the same 32 query positions, so a K/V tile is loaded once
//                  for four heads;
//   HEADS = false: the four wavefronts are four 32-query slices of one head (128 queries per block).
// The score product runs over DK = the head dimension rounded up to 16 features, the output product over DV = the head
// dimension rounded up to 32 rows (64 / 72 / 128 run as 64x64 / 80x96 / 128x128; exact zeros contribute nothing).
// When the output tile has a padding row (dh < DV), the last one is fed with ones instead of V^T: its accumulator is
// then the sum of the (bf16-rounded) probabilities, i.e. the softmax denominator comes out of the matrix core and the
// vector unit does not add the probabilities up.
// Softmax runs on raw scores: the 1/sqrt(dh) * log2(e) scale is folded into one FMA in front of the
// base-2 exponential, masking is skipped on tiles that cannot need it, and the reference maximum of the
// online softmax moves lazily (only past a 2^8 margin), so the running output is rescaled about once.
#include "kernels.hpp"

namespace dlk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int BKV = 64;

__device__ __forceinline__ bf16_t f_to_bf16_attn(float f) {
    __bf16 b = (__bf16)f;
    return *reinterpret_cast<bf16_t*>(&b);
}

// 16 bytes per lane from a buffer straight into LDS (buffer_load_dwordx4 ... offen lds): buffer base in four scalar
// registers, a per-lane 32-bit offset that is the same for every tile, a scalar offset that advances with the tile.
// Offsets past the buffer's size read zeros.
#define DL_ATT_BLL16(rsrc, voff, soff, l)                                                                \
    __builtin_amdgcn_raw_ptr_buffer_load_lds((rsrc), (__attribute__((address_space(3))) void*)(l), 16,  \
                                             int(voff), int(soff), 0, 0)
constexpr int kAttnBufferFlags = 0x00020000;   // raw buffer, 32-bit data format, offsets checked against the size

// K / V^T tiles sit in LDS without padding, filled by global -> LDS copies (a wavefront instruction lands 64 chunks of
// 16 bytes contiguously).  A b128 fragment read serves 16 lanes = 16 rows of one logical chunk per cycle across 64
// banks (256 bytes), so the physical chunk is the logical one XORed with a function of the row that makes those 16
// slots distinct: rows of 128 bytes (8 chunks): (row / 2) % 8; 160 bytes (10): (row / 8) % 2; 192 bytes (12):
// (row / 4) % 4; 256 bytes (16): row % 16.
template <int CPR>
__device__ __forceinline__ int chunk_swizzle(int row) {
    return CPR == 8 ? (row >> 1) & 7 : (CPR == 10 ? (row >> 3) & 1 : (CPR == 12 ? (row >> 2) & 3 : row & 15));
}

// SPLIT: the launch's z dimension divides the K/V tiles into runs of `tps` tiles; a workgroup handles one run and
// writes, per query and head, its unnormalised output, reference maximum and sum to p.split_ws
// ([run][head][query][DV + 4] floats) for attn_merge_kernel.  Used for few queries over many keys (cross-attention
// of a short sequence), where a launch would otherwise consist of a handful of workgroups walking the whole key range.
template <int DK, int DV, bool HEADS, bool SPLIT, bool ONES>
__global__ __launch_bounds__(256, 2) void attn_kernel(AttnArgs p, float scale_log2, int tps) {
    constexpr int QB = HEADS ? 32 : 128;
    constexpr int KCPR = DK / 8;                        // 16-byte chunks per K row; a K tile is KCPR copy instructions
    constexpr int NKI = (KCPR + 3) / 4, NVI = DV / 32;  // copy instructions per wavefront and tile (K, V^T)
    static_assert(KCPR == 8 || KCPR == 10 || KCPR == 12 || KCPR == 16, "swizzle defined for these row lengths");
    // two stages as separate arrays: the compiler can tell the stage being filled from the one being read
    __shared__ __attribute__((aligned(1024))) bf16_t sK0[BKV * DK];
    __shared__ __attribute__((aligned(1024))) bf16_t sK1[BKV * DK];
    __shared__ __attribute__((aligned(1024))) bf16_t sV0[DV * BKV];
    __shared__ __attribute__((aligned(1024))) bf16_t sV1[DV * BKV];

    // the wavefront index as a scalar: the head, the K / V^T base and the LDS addresses of the copies stay out of
    // the vector unit
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31, g2 = lane >> 5;
    // MFMA row lq of a score tile holds key krow: bits 2 and 3 swapped.  With that order the 8 accumulator
    // registers a lane turns into one B-operand fragment of P^T belong to 8 CONSECUTIVE keys
    // (16*t2 + 8*g2 + 0..7), so the matching V^T fragment is one 16-byte read.
    const int krow = (lq & 0x13) | ((lq & 4) << 1) | ((lq & 8) >> 1);
    const int group = p.Hq / p.Hkv;
    // Workgroups are dispatched in blockIdx order, x fastest.  x is the head (group) and y the query block, taken
    // from the last one down in causal passes: the whole launch runs its longest jobs (most visible keys) first, in
    // every head at once, so the tail of the launch is made of the shortest ones.  (With the query block in x, each
    // head's short blocks were dispatched before the next head's long ones.)  Consecutive workgroups go to
    // consecutive XCDs, so with 8 heads (groups) a head's K and V stay in one XCD's L2.
    const int q0 = (p.causal ? int(gridDim.y) - 1 - int(blockIdx.y) : int(blockIdx.y)) * QB;
    const int h = HEADS ? blockIdx.x * 4 + wave : blockIdx.x;
    const int kvh = h / group;
    const int wq0 = HEADS ? q0 : q0 + 32 * wave;       // first query of this wavefront
    const int tq = wq0 + lq;                           // this lane's query (token index)
    const int qpos = p.q_pos0 + tq;

    // Q fragments (B operand): 8 consecutive features per lane and k-step.  All of them are requested here, with
    // clamped addresses and no predicate, and turned into fragments only after the first K/V tile has been requested
    // as well: the wavefront pays one memory round trip for Q and the first tile together, not one per fragment.
    u32x4 qv[DK / 16];
    {
        const bf16_t* qrow = p.q + size_t(min(tq, p.T - 1)) * p.ldq + size_t(h) * p.dh;
#pragma unroll
        for (int kk = 0; kk < DK / 16; ++kk) {
            const int e = 16 * kk + 8 * g2;
            qv[kk] = *reinterpret_cast<const u32x4*>(qrow + (e < p.dh ? e : 0));
        }
    }

    f32x16 accO[DV / 32];
#pragma unroll
    for (int dt = 0; dt < DV / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[dt][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;             // running maximum (raw score units) and sum

    // K of this KV head: S rows of ldk elements (what lies behind row S - 1 is out of range and reads zeros);
    // V^T: dh rows of ldv positions.  The host keeps both below 4 GB.
    const __amdgpu_buffer_rsrc_t kbuf = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.k + size_t(kvh) * p.k_head_stride), 0, int(uint32_t(size_t(p.S) * p.ldk * 2)), kAttnBufferFlags);
    const __amdgpu_buffer_rsrc_t vbuf = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(p.vt + size_t(kvh) * p.v_head_stride), 0, int(uint32_t(size_t(p.dh) * p.ldv * 2)), kAttnBufferFlags);
    int kv_end = p.S;                                  // block-uniform: keys any query of the block may see
    if (p.causal) kv_end = min(p.S, p.q_pos0 + min(q0 + QB, p.T));
    const int wave_last = p.q_pos0 + min(wq0 + 31, p.T - 1);   // last query position of this wavefront
    const int nt_all = (kv_end + BKV - 1) / BKV;
    const int t_begin = SPLIT ? int(blockIdx.z) * tps : 0;
    const int nt = SPLIT ? min(nt_all, t_begin + tps) : nt_all;      // tiles t_begin .. nt - 1

    // Copies are unconditional; a lane's offset inside its buffer is the same for every tile (computed once here)
    // plus the tile's scalar offset:
    //  * K rows past S lie outside the buffer and read zeros; those keys are masked to -inf (a tile that contains
    //    them is always masked);
    //  * feature chunks past dh (zero padding of the head dimension) re-read chunk 0: they meet zero Q features;
    //  * V^T rows past dh repeat row dh-1 (they produce output features nobody stores); V^T positions past S are
    //    read as they are (rows are padded to a multiple of 64 positions): their probabilities are exact zeros and
    //    the buffers hold finite numbers everywhere (zeroed when the module is finalised), what would lie past the
    //    last row's end reads zeros;
    //  * ONES: the last V^T row of a stage (a padding row) holds ones, written once below; the copies skip it.
    // Copy instruction ii of a K tile lands chunks 64 ii .. 64 ii + 63 of the row-major tile (row = id / KCPR); of a
    // V^T tile rows 8 ii .. 8 ii + 7.  A lane fetches the LOGICAL chunk that belongs at its physical position.
    uint32_t koff[NKI], voff[NVI];
#pragma unroll
    for (int i = 0; i < NKI; ++i) {
        const int id = 64 * (wave + 4 * i) + lane, row = id / KCPR, c = (id % KCPR) ^ chunk_swizzle<KCPR>(row);
        koff[i] = uint32_t((size_t(row) * p.ldk + (8 * c < p.dh ? 8 * c : 0)) * 2);
    }
#pragma unroll
    for (int i = 0; i < NVI; ++i) {
        const int row = 8 * (wave + 4 * i) + (lane >> 3), c = (lane & 7) ^ chunk_swizzle<8>(row);
        voff[i] = uint32_t((size_t(min(row, p.dh - 1)) * p.ldv + 8 * c) * 2);
    }
    const int k_tile_bytes = BKV * p.ldk * 2;
    auto copy_tile = [&](int t, bf16_t* sKd, bf16_t* sVd) {
#pragma unroll
        for (int i = 0; i < NKI; ++i) {
            const int ii = wave + 4 * i;
            if (KCPR % 4 != 0 && ii >= KCPR) continue;           // wavefront-uniform
            DL_ATT_BLL16(kbuf, koff[i], t * k_tile_bytes, sKd + 512 * ii);
        }
#pragma unroll
        for (int i = 0; i < NVI; ++i) {
            const int ii = wave + 4 * i;
            if (ONES && ii == DV / 8 - 1) {                      // the last row of the tile keeps its ones
                if (lane < 56) DL_ATT_BLL16(vbuf, voff[i], t * (BKV * 2), sVd + 512 * ii);
            } else {
                DL_ATT_BLL16(vbuf, voff[i], t * (BKV * 2), sVd + 512 * ii);
            }
        }
    };
    if (ONES && tid < 16) {
        const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};            // bf16 1.0 pairs
        *reinterpret_cast<u32x4*>((tid < 8 ? sV0 : sV1) + (DV - 1) * BKV + 8 * (tid & 7)) = ones;
    }

    copy_tile(t_begin, sK0, sV0);                      // range-checked by the buffers: safe for any S >= 1 (the host rejects S <= 0)
    bf16x8 qf[DK / 16];
#pragma unroll
    for (int kk = 0; kk < DK / 16; ++kk) {
        const int e = 16 * kk + 8 * g2;
        const u32x4 z = {0u, 0u, 0u, 0u};
        u32x4 v = (tq < p.T && e < p.dh) ? qv[kk] : z;      // queries past T and padding features are zero
        // pass the words through a register move: inside the tile loop the fragments are then results of vector
        // instructions, and the compiler does not put a wait for ALL outstanding loads (the copy of the next
        // K/V tile included) in front of the first MFMA that reads them
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t y;
            asm volatile("v_mov_b32 %0, %1" : "=v"(y) : "v"(v[w]));
            v[w] = y;
        }
        qf[kk] = *reinterpret_cast<bf16x8*>(&v);
    }
    __builtin_amdgcn_s_waitcnt(0);                     // the first tile and the ones rows are in place
    __builtin_amdgcn_s_barrier();
    // one K/V tile: cK / cV the stage it is read from, nK / nV the stage the next tile is copied into meanwhile
    auto tile_step = [&](int t, const bf16_t* cK, const bf16_t* cV, bf16_t* nK, bf16_t* nV) {
        const int j0 = t * BKV;
        if (t + 1 < nt) copy_tile(t + 1, nK, nV);
        // a wavefront whose queries all lie before this tile has nothing to add (causal)
        const bool active = !p.causal || j0 <= wave_last;
        if (active) {
            // S^T tile: 64 keys x 32 queries.  LDS fragments are requested AHEAD MFMAs early so that an MFMA does
            // not wait for the read issued right in front of it.
            constexpr int NS = 2 * (DK / 16), AHEAD = 3;
            f32x16 accS[2];
            {
                bf16x8 fr[NS];
                auto kfrag = [&](int n) {
                    const int i = n / (DK / 16), kk = n % (DK / 16);
                    const int row = 32 * i + krow, pc = (2 * kk + g2) ^ chunk_swizzle<KCPR>(row);
                    return *reinterpret_cast<const bf16x8*>(cK + row * DK + 8 * pc);
                };
#pragma unroll
                for (int n = 0; n < AHEAD; ++n) fr[n] = kfrag(n);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accS[i][r] = 0.0f;
#pragma unroll
                for (int n = 0; n < NS; ++n) {
                    if (n + AHEAD < NS) fr[n + AHEAD] = kfrag(n + AHEAD);
                    const int i = n / (DK / 16), kk = n % (DK / 16);
                    accS[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n], qf[kk], accS[i], 0, 0, 0);
                }
                // keep that order: AHEAD reads, then one read per MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
                for (int n = 0; n < NS; ++n) {
                    if (n + AHEAD < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // masking only where it can bite: the diagonal tiles of a causal pass and the ragged last tile
            const bool need_mask = (j0 + BKV > p.S) || (p.causal && j0 + BKV - 1 > p.q_pos0 + wq0);
            if (need_mask) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        // accumulator row 8*(r/4) + 4*g2 + r%4 holds key 16*(r/8) + 8*g2 + r%8
                        const int kv = j0 + 32 * i + 16 * (r >> 3) + 8 * g2 + (r & 7);
                        const bool ok = kv < p.S && (!p.causal || kv <= qpos);
                        accS[i][r] = ok ? accS[i][r] : -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, accS[i][r]);
            {
                // exchange with lane l^32 (the other 16 keys of the same query) without going through the LDS
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            }
            // Lazy reference maximum: m_run moves only when the tile maximum exceeds it by more than 2^LAZY in the
            // exponent, so probabilities stay below 2^LAZY (no overflow in bf16 / fp32) and the running output is
            // rescaled on the first tile and almost never again.  Any reference gives the same softmax.
            constexpr float LAZY = 8.0f;
            const bool move = (mx - m_run) * scale_log2 > LAZY;   // false for NaN (-inf minus -inf: nothing visible yet)
            const float m_use = move ? mx : (m_run == -INFINITY ? 0.0f : m_run);
            if (__any(move)) {
                const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2) : 1.0f;
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < DV / 32; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accO[dt][r] *= alpha;
                m_run = move ? mx : m_run;
            }
            const float ms = m_use * scale_log2;
            float psum = 0.0f;
            bf16x8 pf[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float pv = __builtin_amdgcn_exp2f(fmaf(accS[i][8 * t2 + j], scale_log2, -ms));
                        if (!ONES) psum += pv;
                        pf[i][t2][j] = (__bf16)pv;
                    }
            l_run += psum;
            // O^T += V^T * P^T
            {
                constexpr int NP = (DV / 32) * 4;
                bf16x8 fr[NP];
                auto vfrag = [&](int n) {
                    const int dt = n / 4, i = (n / 2) % 2, t2 = n % 2;
                    const int row = 32 * dt + lq, pc = (4 * i + 2 * t2 + g2) ^ chunk_swizzle<8>(row);
                    return *reinterpret_cast<const bf16x8*>(cV + row * BKV + 8 * pc);
                };
#pragma unroll
                for (int n = 0; n < AHEAD; ++n) fr[n] = vfrag(n);
#pragma unroll
                for (int n = 0; n < NP; ++n) {
                    if (n + AHEAD < NP) fr[n + AHEAD] = vfrag(n + AHEAD);
                    const int dt = n / 4, i = (n / 2) % 2, t2 = n % 2;
                    accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n], pf[i][t2], accO[dt], 0, 0, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
                for (int n = 0; n < NP; ++n) {
                    if (n + AHEAD < NP) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // this wavefront's copies of the next tile have landed and its fragment reads are done; past the barrier that
        // holds for the whole workgroup
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_s_barrier();
    };
    for (int t = t_begin; t < nt; t += 2) {
        tile_step(t, sK0, sV0, sK1, sV1);
        if (t + 1 < nt) tile_step(t + 1, sK1, sV1, sK0, sV0);
    }

    // ONES: output row DV - 1 (tile DV/32 - 1, register 15 of the lanes 32..63) holds the sum of the probabilities
    const float l_tot = ONES ? __shfl(accO[DV / 32 - 1][15], 32 + lq, 64) : l_run + __shfl_xor(l_run, 32, 64);
    if (tq >= p.T) return;
    if constexpr (SPLIT) {
        float* prow = p.split_ws + ((size_t(blockIdx.z) * p.Hq + h) * p.T + tq) * (DV + 4);
#pragma unroll
        for (int dt = 0; dt < DV / 32; ++dt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int e0 = 32 * dt + 8 * rg + 4 * g2;
                *reinterpret_cast<float4*>(prow + e0) =
                    make_float4(accO[dt][4 * rg], accO[dt][4 * rg + 1], accO[dt][4 * rg + 2], accO[dt][4 * rg + 3]);
            }
        if (g2 == 0) {
            prow[DV] = m_run * scale_log2;             // reference of this run's exponentials, base-2 units
            prow[DV + 1] = l_tot;
        }
        return;
    }
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    bf16_t* orow = p.out + size_t(tq) * p.ldo + size_t(h) * p.dh;
#pragma unroll
    for (int dt = 0; dt < DV / 32; ++dt)
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

// out[query, head] = sum_z w_z O_z / sum_z w_z l_z with w_z = 2^(m_z - max m), runs z taken in order.  At most 16
// runs; every run's values are requested before the first is used (index clamped to the last run, weight zero).
template <int DHP>
__global__ __launch_bounds__(128) void attn_merge_kernel(AttnArgs p, int n_runs) {
    constexpr int MAXR = 16;
    const int tq = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    const size_t run_stride = size_t(p.Hq) * p.T * (DHP + 4);
    const float* base = p.split_ws + (size_t(h) * p.T + tq) * (DHP + 4);
    const int ec = e < DHP ? e : DHP - 1;
    float mz[MAXR], lz[MAXR], oz[MAXR];
#pragma unroll
    for (int z = 0; z < MAXR; ++z) {
        const float* r = base + size_t(z < n_runs ? z : n_runs - 1) * run_stride;
        mz[z] = r[DHP];
        lz[z] = r[DHP + 1];
        oz[z] = r[ec];
    }
    float m = -INFINITY;
#pragma unroll
    for (int z = 0; z < MAXR; ++z) m = fmaxf(m, mz[z]);
    float num = 0.0f, den = 0.0f;
#pragma unroll
    for (int z = 0; z < MAXR; ++z) {
        const float w = (z < n_runs && mz[z] != -INFINITY) ? __builtin_amdgcn_exp2f(mz[z] - m) : 0.0f;
        num = fmaf(w, oz[z], num);
        den = fmaf(w, lz[z], den);
    }
    if (e < p.dh) p.out[size_t(tq) * p.ldo + size_t(h) * p.dh + e] = f_to_bf16_attn(den > 0.0f ? num / den : 0.0f);
}

template <int DK, int DV, bool ONES>
void launch_attn(const AttnArgs& a, float scale_log2, hipStream_t st) {
    const int group = a.Hq / a.Hkv;
    const bool heads = group % 4 == 0;
    const dim3 grid = heads ? dim3(a.Hq / 4, (a.T + 31) / 32) : dim3(a.Hq, (a.T + 127) / 128);
    // few queries over many keys: split the key range over the launch's z dimension
    const int nt = (a.S + BKV - 1) / BKV;
    if (a.split_ws && !a.causal && a.T <= 128 && nt >= 8) {
        int n_runs = nt / 2 < 16 ? nt / 2 : 16;
        const int tps = (nt + n_runs - 1) / n_runs;
        n_runs = (nt + tps - 1) / tps;                       // every run has at least one tile
        if (uint64_t(n_runs) * a.Hq * a.T * (DV + 4) * 4 <= a.split_ws_bytes) {
            const dim3 g3(grid.x, grid.y, n_runs);
            if (heads) hipLaunchKernelGGL((attn_kernel<DK, DV, true, true, ONES>), g3, dim3(256), 0, st, a, scale_log2, tps);
            else hipLaunchKernelGGL((attn_kernel<DK, DV, false, true, ONES>), g3, dim3(256), 0, st, a, scale_log2, tps);
            hipLaunchKernelGGL(attn_merge_kernel<DV>, dim3(a.T, a.Hq), dim3(128), 0, st, a, n_runs);
            return;
        }
    }
    if (heads) hipLaunchKernelGGL((attn_kernel<DK, DV, true, false, ONES>), grid, dim3(256), 0, st, a, scale_log2, 0);
    else hipLaunchKernelGGL((attn_kernel<DK, DV, false, false, ONES>), grid, dim3(256), 0, st, a, scale_log2, 0);
}

}  // namespace

uint64_t attention_split_workspace_bytes(int T, int Hq, int dh) {
    const int dhp = dh <= 64 ? 64 : (dh <= 96 ? 96 : 128);
    const uint64_t t = T < 128 ? T : 128;
    return 16ull * uint64_t(Hq) * t * uint64_t(dhp + 4) * 4;
}

void attention(const AttnArgs& a, hipStream_t st) {
    if (a.T <= 0 || a.S <= 0) return;
    const float scale_log2 = 1.4426950408889634f / sqrtf(float(a.dh));
    // a padding row in the output tile (dh below its multiple of 32) carries the softmax denominator
    if (a.dh < 64) launch_attn<64, 64, true>(a, scale_log2, st);
    else if (a.dh == 64) launch_attn<64, 64, false>(a, scale_log2, st);
    else if (a.dh <= 80) launch_attn<80, 96, true>(a, scale_log2, st);
    else if (a.dh < 96) launch_attn<96, 96, true>(a, scale_log2, st);
    else if (a.dh == 96) launch_attn<96, 96, false>(a, scale_log2, st);
    else if (a.dh < 128) launch_attn<128, 128, true>(a, scale_log2, st);
    else launch_attn<128, 128, false>(a, scale_log2, st);
}

}  // namespace dlk
