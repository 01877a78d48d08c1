// Launch wrappers of the hand-written gfx950 kernels.  Every function enqueues on `st` and
// returns; none allocates or synchronises.  bf16 data is addressed as uint16_t on the host side.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace dlk {

typedef uint16_t bf16_t;

// ---- GEMM: C[M,N] = A[M,K] * B[N,K]^T, BF16 operands, FP32 accumulation on MFMA -------------
enum GemmEpilogue {
    EPI_BF16 = 0,        // out bf16 [M,N]           = acc + bias
    EPI_RESID_F32 = 1,   // out f32  [M,N]           = resid + acc + bias         (out may alias resid)
    EPI_SWIGLU_BF16 = 2, // out bf16 [M,N/2]: B rows interleave gate/up in groups of 32; out = silu(gate) * up
    EPI_GELU_BF16 = 3,   // out bf16 [M,N]           = gelu_tanh(acc + bias)
    EPI_F32 = 4,         // out f32  [M,N]           = acc + bias
    EPI_QKV_POST = 5     // matrix-vector only: QKV projection of ONE token followed by what qkv_post does for it
};
struct GemmArgs {
    const bf16_t* A; int lda;     // [M,K], row stride lda (elements); 16-byte aligned rows
    const bf16_t* B; int ldb;     // [N,K]
    const bf16_t* bias;           // [N] or nullptr
    void* out; int ldo;
    const float* resid; int ldr;
    int M, N, K;                  // K % 8 == 0
    int epi;
};
void gemm(const GemmArgs& a, hipStream_t st);

// ---- after the QKV projection: rotary embedding and scatter -------------------------------------
// qkv bf16 [T, n_qkv] = [q | k | v] per token.  Rotates q in place (if theta > 0); writes k (rotated)
// to k_out[(g*k_head_stride) + (pos0+t)*dh + e] when k_out != nullptr, else rotates k in place;
// writes v transposed to vt_out[g*vt_head_stride + e*vt_ld + (pos0+t)].
struct QkvPostArgs {
    bf16_t* qkv; int n_qkv;
    int T, pos0, Hq, Hkv, dh;
    float theta;
    bf16_t* k_out; uint64_t k_head_stride;
    bf16_t* vt_out; uint64_t vt_head_stride; int vt_ld;
    int q_off, k_off, v_off;      // column offsets of q, k, v inside a qkv row (q_off < 0: no q part)
};
void qkv_post(const QkvPostArgs& a, hipStream_t st);

// ---- matrix-vector for single-token passes: out[N] = B[N,K] * x[K], same epilogues ----------
struct GemvArgs {
    const bf16_t* x;              // [K] bf16
    const bf16_t* B; int ldb;     // [N,K]
    const bf16_t* bias;
    void* out;
    const float* resid;
    int N, K;
    int epi;
    // EPI_QKV_POST: `out` is the token's qkv row (= post.qkv, T = 1); q and k are rotated, k goes to the cache (or
    // stays in the row), v goes to the transposed cache, exactly as qkv_post would do after an EPI_BF16 product
    QkvPostArgs post;
    // When norm_x != nullptr (epilogues QKV_POST, SWIGLU, GELU and F32 only) the input vector is not x but the
    // normalisation of the fp32 row norm_x[K] (kind as in norm_rows), computed inside the kernel; x is ignored.
    const float* norm_x;
    const bf16_t* norm_g;
    const bf16_t* norm_b;
    int norm_kind;
    float norm_eps;
};
void gemv(const GemvArgs& a, hipStream_t st);

// ---- normalisation: fp32 rows in, bf16 (or fp32) rows out -------------------------------------
// kind: 0 RMSNorm (g), 1 LayerNorm (g, b).  x [T, d] fp32, row stride d.
void norm_rows(int kind, const float* x, const bf16_t* g, const bf16_t* b, void* out, bool out_f32,
               int T, int d, float eps, hipStream_t st);
// fp32 -> bf16 elementwise (cross-attention source)
void cast_f32_bf16(const float* x, bf16_t* out, uint64_t n, hipStream_t st);

// ---- attention (flash-style, online softmax, MFMA) ------------------------------------------------
// The V^T rows must be readable up to S rounded up to 8 positions and hold finite numbers there (stale values are
// fine: they meet zero probabilities); K rows and V^T rows are read in 16-byte pieces (ldk, ldv multiples of 8).
struct AttnArgs {
    const bf16_t* q; int ldq;                         // token t, head h: q + t*ldq + h*dh
    const bf16_t* k; int ldk; uint64_t k_head_stride; // kv head g, position j: k + g*k_head_stride + j*ldk
    const bf16_t* vt; int ldv; uint64_t v_head_stride;// kv head g, feature e, position j: vt + g*v_head_stride + e*ldv + j
    bf16_t* out; int ldo;                             // out + t*ldo + h*dh
    int T, S, q_pos0, Hq, Hkv, dh, causal;
    // optional scratch for non-causal calls with at most 128 queries and at least 512 keys: the key range is then
    // split over more workgroups and the pieces are merged by a second launch (fixed order).  nullptr: never split.
    float* split_ws;
    uint64_t split_ws_bytes;
};
// bytes of split_ws that let a call with T queries (T <= 128) split its key range
uint64_t attention_split_workspace_bytes(int T, int Hq, int dh);
void attention(const AttnArgs& a, hipStream_t st);

// Single-query attention over a KV cache (decode), split over the key range: one wavefront per
// (KV head, 64-position tile) writes a partial (max, sum, output) per query head into `partial`
// ([Hq][n_tiles][dh + 2] floats), a second kernel merges the tiles.  S = number of cached positions.
struct DecodeAttnArgs {
    const bf16_t* q;                                   // [Hq * dh] (already rotated)
    const bf16_t* k; int ldk; uint64_t k_head_stride;
    const bf16_t* vt; int ldv; uint64_t v_head_stride;
    bf16_t* out;                                       // [Hq * dh]
    float* partial;
    int S, Hq, Hkv, dh;
};
uint64_t decode_attention_workspace_bytes(int max_seq, int Hq, int dh);
void decode_attention(const DecodeAttnArgs& a, hipStream_t st);

// ---- small elementwise helpers of the multi-module pipeline (fp32 activations) ----------------------
// y[t, :] = mean over j < group of x[t*group + j, :]
void mean_pool_rows(const float* x, float* y, int T_out, int group, int d, hipStream_t st);
// y[i] += alpha * x[i]
void axpy_f32(float* y, float alpha, const float* x, uint64_t n, hipStream_t st);
// y[t, i] = x[t, i] + (i < d/2 ? sin : cos)(1000 * tval * 10000^(-(i mod d/2) / (d/2)))
void add_time_embedding(const float* x, float* y, float tval, int T, int d, hipStream_t st);

// ---- diagnostic: register-only BF16 MFMA loop on `blocks` workgroups of 4 wavefronts; out holds blocks*256 floats.
// Returns the flop the launch performs.
double mfma_rate_probe(float* out, int blocks, int iters, int pattern, hipStream_t st);

// ---- head --------------------------------------------------------------------------------------------
void embed_row(const bf16_t* table, int d, const int32_t* token_dev, int token_host, float* x_out, hipStream_t st);
// token_dev (and token_copy, if not null) = index of the largest logit, lowest index on ties; if table != nullptr also
// x_out[0..d) = row `token` of the bf16 table [*, d] as fp32 (the next step's input), in the same launch
void argmax_f32(const float* logits, int n, int32_t* token_dev, int32_t* token_copy, const bf16_t* table, int d,
                float* x_out, hipStream_t st);

}  // namespace dlk
