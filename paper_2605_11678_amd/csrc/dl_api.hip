// C ABI of the library: context, pinned parameter store, residency, the pipelined forward pass
// (Sec. IV-C), profiling (Table III procedure) and run statistics.  HIP backend: one copy stream,
// one compute stream, event fences between them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "dl_internal.hpp"
#include "kernels.hpp"

using dl::PackLayout;

// Scratch of dl_greedy_step_static (the logits of one step and the chosen token): device memory that exists once per
// GPU for the life of the process, so that the call never allocates.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels are given is looked up once per device (static_scratch_ptr below).
constexpr int32_t kStaticMaxVocab = 131072;
constexpr size_t kStaticScratchBytes = size_t(kStaticMaxVocab) * 4 + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kStaticMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kStaticMaxDevices] = {};
thread_local std::string g_static_err;     // message of the last failed context-free call on this thread

// Device address of `scratch` on `device`, which must be the current device.  Looked up on first use per device.
hipError_t static_scratch_ptr(int32_t device, void** out) {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_static_ptr[device] = p;
    }
    *out = g_static_ptr[device];
    return hipSuccess;
}

struct Module {
    dl_module_desc d{};
    PackLayout L;
    dl::WorkspaceLayout W;
    dl::KvLayout KV;
    uint8_t* store = nullptr;            // n_layers blobs, pinned (or plain malloc in a host-only context)
    std::vector<uint32_t> set_mask;      // per layer: which tensors have been provided
    bool finalized = false;
    std::vector<uint8_t> resident;       // per layer
    std::vector<uint64_t> res_off;       // arena offset of the resident copy
    uint64_t ws_off = 0, kv_off = 0;
    uint64_t rt_off[DL_R_COUNT] = {0, 0, 0, 0};
    bool rt_set[DL_R_COUNT] = {false, false, false, false};
};

struct Mlp {
    int32_t d_in = 0, d_hidden = 0, d_out = 0, max_tokens = 0;
    uint64_t w1 = 0, b1 = 0, w2 = 0, b2 = 0, xin = 0, hid = 0;   // arena offsets
    bool has_b1 = false, has_b2 = false;
};

struct TimedOp {
    hipEvent_t e0, e1;
    int32_t module, layer, slot;
    int32_t copy_index;                  // for EXEC of a streamed layer: index into copies, else -1
};

}  // namespace

struct dl_ctx {
    int32_t device = -1;
    std::string err;
    dl::Arena arena;
    uint8_t* base = nullptr;
    hipStream_t s_compute = nullptr, s_copy = nullptr;
    bool streams_set = false;
    std::vector<Module> mods;
    std::vector<Mlp> mlps;
    uint64_t slot_bytes = 0;
    uint64_t slot_off[dl::kMaxSlots] = {0, 0, 0, 0};
    int32_t n_slots = 2;          // device slots in use: 1 .. kMaxSlots
    int32_t slots_held = 0;       // how many of slot_off[] are allocated right now
    bool slots_alloc = false;
    // Arena discipline.  Blocks that never move (KV caches, resident non-layer tensors, MLPs, the caller's blocks)
    // are stacked at the TOP of the arena, the activation workspaces right below them; slots and resident layer
    // copies fill the arena from the BOTTOM and may be moved (re-uploaded from the pinned store) whenever a change
    // does not fit between the holes: what slots and resident layers can use is exactly what lies below the top stack.
    std::vector<uint64_t> perms;  // offsets of the blocks that never move
    bool poisoned = false;        // a device copy failed after the state was committed: the context is unusable
    dl::SlotBook book;
    hipEvent_t ev_dma[dl::kMaxSlots] = {}, ev_comp[dl::kMaxSlots] = {}, ev_pass = nullptr;
    bool events_made = false;
    static constexpr int kMaxRunAhead = 8;
    hipEvent_t ev_inflight[kMaxRunAhead] = {};   // start of the last layer of the most recent streaming passes (host throttle)
    uint64_t n_passes = 0;                       // streaming passes enqueued so far
    int32_t run_ahead = 1;                        // streaming passes that may be unfinished; 0 = unlimited
    int32_t mode = DL_MODE_PIPELINED, wrap = 0;
    bool tracing = false;
    std::vector<dl_trace_op> trace;
    bool timing = false;
    std::vector<TimedOp> copies, execs;
    int32_t last_copy_in_slot[dl::kMaxSlots] = {-1, -1, -1, -1};
    std::vector<hipEvent_t> ev_pool;
    size_t ev_next = 0;
    uint32_t ktiming = 0;   // bit k set: launches of kernel class k are bracketed with events
    struct KRec { int32_t kind; hipEvent_t e0, e1; double flops, bytes; };
    std::vector<KRec> krecs;
};

namespace {

int32_t fail(dl_ctx* c, int32_t code, const std::string& msg) {
    if (c) c->err = msg;
    return code;
}

#define DL_HIP(c, call)                                                                              \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return fail((c), DL_ERR_DEVICE, std::string(#call) + ": " + hipGetErrorString(e_));      \
    } while (0)

bool on_gpu(const dl_ctx* c) { return c->device >= 0; }

int32_t enter(dl_ctx* c) {
    if (!c) return DL_ERR_INVALID_ARG;
    if (c->poisoned) return fail(c, DL_ERR_DEVICE, "the context is unusable: an earlier device copy failed after its state change was committed");
    if (on_gpu(c)) DL_HIP(c, hipSetDevice(c->device));
    return DL_OK;
}

Module* get_module(dl_ctx* c, int32_t m) {
    if (m < 0 || size_t(m) >= c->mods.size()) return nullptr;
    return &c->mods[size_t(m)];
}

int32_t make_events(dl_ctx* c) {
    if (c->events_made || !on_gpu(c)) return DL_OK;
    for (int s = 0; s < dl::kMaxSlots; ++s) {
        DL_HIP(c, hipEventCreateWithFlags(&c->ev_dma[s], hipEventDisableTiming));
        DL_HIP(c, hipEventCreateWithFlags(&c->ev_comp[s], hipEventDisableTiming));
    }
    DL_HIP(c, hipEventCreateWithFlags(&c->ev_pass, hipEventDisableTiming));
    for (int s = 0; s < dl_ctx::kMaxRunAhead; ++s) DL_HIP(c, hipEventCreateWithFlags(&c->ev_inflight[s], hipEventDisableTiming));
    c->events_made = true;
    return DL_OK;
}

int32_t timing_event(dl_ctx* c, hipEvent_t* out) {
    if (c->ev_next == c->ev_pool.size()) {
        hipEvent_t e;
        DL_HIP(c, hipEventCreate(&e));
        c->ev_pool.push_back(e);
    }
    *out = c->ev_pool[c->ev_next++];
    return DL_OK;
}

int32_t sync_streams(dl_ctx* c) {
    if (on_gpu(c) && c->streams_set) {
        DL_HIP(c, hipStreamSynchronize(c->s_copy));
        DL_HIP(c, hipStreamSynchronize(c->s_compute));
    }
    return DL_OK;
}

// ---- placement of everything the library keeps in the arena ------------------------------------------
// A proposed change: residency per module, workspace size per module, slot count, and blocks that never move to add.
struct Proposal {
    std::vector<std::vector<uint8_t>> resident;   // [module][layer]
    std::vector<uint64_t> ws_bytes;               // [module]; 0: the module has no workspace (not finalized)
    std::vector<uint8_t> counted;                 // [module]: finalized, or being finalized by this change
    int32_t n_slots = 2;
    std::vector<uint64_t> new_perm;               // sizes of blocks to add to the top stack, in order
};

struct Placement {
    dl::Arena arena;
    std::vector<std::vector<uint64_t>> res_off;
    std::vector<uint64_t> ws_off;
    std::vector<uint8_t> ws_moved;
    uint64_t slot_off[dl::kMaxSlots] = {0, 0, 0, 0};
    uint64_t slot_bytes = 0;
    int32_t slots_held = 0;
    std::vector<uint64_t> perm_off;
};

Proposal current_proposal(const dl_ctx* c) {
    Proposal p;
    p.n_slots = c->n_slots;
    for (const Module& M : c->mods) {
        p.resident.push_back(M.resident);
        p.ws_bytes.push_back(M.finalized ? M.W.bytes : 0);
        p.counted.push_back(M.finalized ? 1 : 0);
    }
    return p;
}

// Places the proposal on a copy of the arena.  repack == false: blocks that stay keep their place, new ones go
// first-fit.  repack == true: every slot, resident copy and workspace is released and placed again (top stack first,
// then slots and resident copies from the bottom, largest layers first), which leaves no hole below the top stack.
bool place(const dl_ctx* c, const Proposal& p, bool repack, Placement* out, std::string* why) {
    dl::Arena A = c->arena;
    const size_t nm = c->mods.size();
    out->res_off.assign(nm, {});
    out->ws_off.assign(nm, 0);
    out->ws_moved.assign(nm, 0);
    out->perm_off.clear();
    bool touch_ws = repack || !p.new_perm.empty();
    for (size_t m = 0; m < nm; ++m) {
        const Module& M = c->mods[m];
        out->res_off[m] = M.res_off;
        out->ws_off[m] = M.ws_off;
        const uint64_t old_ws = M.finalized ? M.W.bytes : 0;
        touch_ws = touch_ws || old_ws != p.ws_bytes[m];
    }
    // 1. release
    for (size_t m = 0; m < nm; ++m) {
        const Module& M = c->mods[m];
        for (int32_t i = 0; i < M.d.n_layers; ++i)
            if (M.resident[size_t(i)] && (repack || !p.resident[m][size_t(i)])) A.free(M.res_off[size_t(i)]);
        if (touch_ws && M.finalized) A.free(M.ws_off);
    }
    uint64_t need_bytes = 0;
    bool any_streamed = false;
    for (size_t m = 0; m < nm; ++m) {
        if (!p.counted[m]) continue;
        bool streams = false;
        for (uint8_t v : p.resident[m]) streams |= !v;
        if (streams) need_bytes = std::max(need_bytes, c->mods[m].L.bytes);
        any_streamed |= streams;
    }
    const bool keep_slots = !repack && c->slots_alloc && any_streamed && c->slot_bytes == need_bytes && c->slots_held == p.n_slots;
    if (c->slots_alloc && !keep_slots)
        for (int32_t k = 0; k < c->slots_held; ++k) A.free(c->slot_off[k]);
    // 2. the top stack: blocks that never move, then the workspaces.  Each must land inside the stack (a hole left by
    // a released block) or directly below it; anything else would strand it among the movable blocks.
    uint64_t top = A.capacity();
    for (uint64_t off : c->perms) top = std::min(top, off);
    if (!touch_ws)
        for (size_t m = 0; m < nm; ++m)
            if (c->mods[m].finalized) top = std::min(top, c->mods[m].ws_off);
    auto stack_block = [&](uint64_t bytes, uint64_t* off) {
        if (!A.alloc_top(bytes, off)) return false;
        const uint64_t sz = dl::align_up(bytes ? bytes : 1);
        if (*off < top && *off + sz != top) return false;
        top = std::min(top, *off);
        return true;
    };
    for (uint64_t bytes : p.new_perm) {
        uint64_t off = 0;
        if (!stack_block(bytes, &off)) { *why = "arena cannot hold the block below its top stack"; return false; }
        out->perm_off.push_back(off);
    }
    if (touch_ws)
        for (size_t m = 0; m < nm; ++m) {
            if (!p.ws_bytes[m]) continue;
            uint64_t off = 0;
            if (!stack_block(p.ws_bytes[m], &off)) { *why = "arena cannot hold the activation workspace"; return false; }
            out->ws_moved[m] = 1;
            out->ws_off[m] = off;
        }
    // 3. slots, then resident copies, from the bottom
    out->slot_bytes = any_streamed ? need_bytes : 0;
    out->slots_held = 0;
    if (keep_slots) {
        for (int32_t k = 0; k < c->slots_held; ++k) out->slot_off[k] = c->slot_off[k];
        out->slots_held = c->slots_held;
    } else if (any_streamed) {
        for (int32_t k = 0; k < p.n_slots; ++k)
            if (!A.alloc(need_bytes, &out->slot_off[k])) { *why = "arena cannot hold the layer slots"; return false; }
        out->slots_held = p.n_slots;
    }
    std::vector<size_t> order(nm);
    for (size_t m = 0; m < nm; ++m) order[m] = m;
    if (repack)
        std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b2) { return c->mods[a].L.bytes > c->mods[b2].L.bytes; });
    for (size_t m : order) {
        const Module& M = c->mods[m];
        for (int32_t i = 0; i < M.d.n_layers; ++i) {
            if (!p.resident[m][size_t(i)] || (!repack && M.resident[size_t(i)])) continue;
            if (!A.alloc(M.L.bytes, &out->res_off[m][size_t(i)])) {
                char buf[200];
                snprintf(buf, sizeof buf, "arena cannot hold resident layer %d of module %d (%llu bytes each, %llu of %llu used)", i,
                         int(m), (unsigned long long)M.L.bytes, (unsigned long long)A.used(), (unsigned long long)A.capacity());
                *why = buf;
                return false;
            }
        }
    }
    out->arena = A;
    return true;
}

// Applies a proposal: first-fit next to what is there, and if that does not fit, with everything movable placed
// again.  Commits only if it fits (DL_ERR_BUDGET_EXCEEDED otherwise, nothing changed); new_perm_out receives the
// offsets of the added blocks.  The streams must be idle.
int32_t relayout(dl_ctx* c, const Proposal& p, std::vector<uint64_t>* new_perm_out = nullptr) {
    Placement P;
    std::string why;
    if (!place(c, p, false, &P, &why) && !place(c, p, true, &P, &why)) return fail(c, DL_ERR_BUDGET_EXCEEDED, why);
    // layer copies to (re)fill from the pinned store: newly resident ones and those that moved
    struct Up { size_t m; int32_t i; uint64_t off; };
    std::vector<Up> ups;
    bool reuses_live_copy = false;
    for (size_t m = 0; m < c->mods.size(); ++m) {
        const Module& M = c->mods[m];
        for (int32_t i = 0; i < M.d.n_layers; ++i) {
            if (!p.resident[m][size_t(i)]) continue;
            if (!M.resident[size_t(i)] || M.res_off[size_t(i)] != P.res_off[m][size_t(i)]) ups.push_back({m, i, P.res_off[m][size_t(i)]});
        }
    }
    // does an upload land on memory that holds a resident copy in the CURRENT state (one dropped or moved by this call)?
    for (const Up& u : ups) {
        const uint64_t u0 = u.off, u1 = u.off + c->mods[u.m].L.bytes;
        for (size_t m = 0; m < c->mods.size() && !reuses_live_copy; ++m) {
            const Module& M = c->mods[m];
            for (int32_t i = 0; i < M.d.n_layers; ++i)
                if (M.resident[size_t(i)] && u0 < M.res_off[size_t(i)] + M.L.bytes && M.res_off[size_t(i)] < u1) { reuses_live_copy = true; break; }
        }
    }
    auto upload = [&](const Up& u) -> hipError_t {
        const Module& M = c->mods[u.m];
        return hipMemcpy(c->base + u.off, M.store + size_t(u.i) * M.L.bytes, M.L.bytes, hipMemcpyHostToDevice);
    };
    // what the slots hold is gone either way (a copy issued ahead for the next pass is simply issued again)
    c->book = dl::SlotBook();
    c->book.n_slots = c->n_slots;
    if (on_gpu(c) && !reuses_live_copy) {
        // the new copies only touch memory that is free or transient in the current state: fill them first, so that a
        // failed copy leaves the context exactly as it was
        for (const Up& u : ups) DL_HIP(c, upload(u));
    }
    c->arena = P.arena;
    c->n_slots = p.n_slots;
    c->book.n_slots = p.n_slots;
    c->slots_alloc = P.slots_held > 0;
    c->slots_held = P.slots_held;
    c->slot_bytes = P.slot_bytes;
    for (int32_t k = 0; k < dl::kMaxSlots; ++k) c->slot_off[k] = P.slot_off[k];
    for (size_t m = 0; m < c->mods.size(); ++m) {
        c->mods[m].resident = p.resident[m];
        c->mods[m].res_off = P.res_off[m];
        c->mods[m].ws_off = P.ws_off[m];
    }
    for (uint64_t off : P.perm_off) c->perms.push_back(off);
    if (new_perm_out) *new_perm_out = P.perm_off;
    if (on_gpu(c)) {
        hipError_t e = hipSuccess;
        if (reuses_live_copy)
            for (const Up& u : ups)
                if (e == hipSuccess) e = upload(u);
        // stale bytes in the transposed-V areas of a workspace must be finite numbers: a placed workspace starts as zeros
        for (size_t m = 0; m < c->mods.size(); ++m)
            if (P.ws_moved[m] && e == hipSuccess) e = hipMemset(c->base + P.ws_off[m], 0, p.ws_bytes[m]);
        if (e != hipSuccess) {
            c->poisoned = true;
            return fail(c, DL_ERR_DEVICE, std::string("device copy failed after the new placement was committed: ") + hipGetErrorString(e));
        }
    }
    return DL_OK;
}

// adds one block to the top stack (see dl_ctx::perms); synchronises, because the workspaces move
int32_t add_permanent(dl_ctx* c, uint64_t bytes, uint64_t* off) {
    int32_t rc = sync_streams(c);
    if (rc) return rc;
    Proposal p = current_proposal(c);
    p.new_perm.push_back(bytes);
    std::vector<uint64_t> offs;
    rc = relayout(c, p, &offs);
    if (rc) return rc;
    *off = offs[0];
    return DL_OK;
}

// ---- one layer on the compute stream -------------------------------------------------------------
using dlk::bf16_t;

// A single-token product may take its input as "the normalisation of an fp32 row" instead of a bf16 vector.
struct NormSrc {
    const float* x = nullptr;
    const bf16_t* g = nullptr;
    const bf16_t* b = nullptr;
    int kind = 0;
    float eps = 0.0f;
};
void with_norm(dlk::GemvArgs& g, const NormSrc& n) {
    g.norm_x = n.x;
    g.norm_g = n.g;
    g.norm_b = n.b;
    g.norm_kind = n.kind;
    g.norm_eps = n.eps;
}

void linear(hipStream_t st, int T, const bf16_t* A, int lda, const bf16_t* B, int K, int N, const bf16_t* bias,
            int epi, void* out, int ldo, const float* resid, int ldr, const NormSrc& nsrc = NormSrc()) {
    if (T == 1) {
        dlk::GemvArgs g{A, B, K, bias, out, resid, N, K, epi};
        with_norm(g, nsrc);
        dlk::gemv(g, st);
    } else {
        dlk::GemmArgs g{A, lda, B, K, bias, out, ldo, resid, ldr, T, N, K, epi};
        dlk::gemm(g, st);
    }
}

void run_layer(dl_ctx* c, Module& M, int32_t layer, const uint8_t* w, const float* in, float* out, int32_t T,
               int32_t pos0, const float* ctx, int32_t n_ctx) {
    const dl_module_desc& d = M.d;
    const PackLayout& L = M.L;
    hipStream_t st = c->s_compute;
    auto P = [&](uint64_t off) -> const bf16_t* {
        return off == PackLayout::kNone ? nullptr : reinterpret_cast<const bf16_t*>(w + off);
    };
    uint8_t* ws = c->base + M.ws_off;
    bf16_t* nbuf = reinterpret_cast<bf16_t*>(ws + M.W.nbuf);
    bf16_t* qkv = reinterpret_cast<bf16_t*>(ws + M.W.qkv);
    bf16_t* attn = reinterpret_cast<bf16_t*>(ws + M.W.attn);
    bf16_t* mid = reinterpret_cast<bf16_t*>(ws + M.W.mid);
    const int dm = d.d_model, dh = d.d_head, Hq = d.n_q_heads, Hkv = d.n_kv_heads;
    const int dq = Hq * dh, dkv = Hkv * dh;
    const bool cache = d.max_seq > 0;
    const double Td = double(T);
    // optional per-kernel timing: events around each launch, work counted algorithmically
    dl_ctx::KRec* open_rec = nullptr;
    auto kbegin = [&](int32_t kind, double flops, double bytes) {
        if (!((c->ktiming >> kind) & 1u)) return;
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (timing_event(c, &e0) != DL_OK || timing_event(c, &e1) != DL_OK) return;
        c->krecs.push_back({kind, e0, e1, flops, bytes});
        open_rec = &c->krecs.back();
        (void)hipEventRecord(e0, st);
    };
    auto kend = [&]() {
        if (open_rec) (void)hipEventRecord(open_rec->e1, st);
        open_rec = nullptr;
    };
    auto lin_work = [&](double M_, double N_, double K_, double* fl, double* by) {
        *fl = 2.0 * M_ * N_ * K_;
        *by = 2.0 * (M_ * K_ + N_ * K_ + M_ * N_);
    };
    double fl, by;

    // attention sub-block.  A single-token pass has no normalisation launches: the matrix-vector kernels of the
    // QKV projection and of the feed-forward's first map normalise their input row themselves.
    const bool fused_norm = T == 1;
    if (!fused_norm) {
        kbegin(DL_K_NORM, 0, Td * dm * 6.0);
        dlk::norm_rows(d.norm, in, P(L.norm1_g), P(L.norm1_b), nbuf, false, T, dm, d.norm_eps, st);
        kend();
    }
    bf16_t* kc = nullptr;
    bf16_t* vt;
    uint64_t k_hs, v_hs;
    int ldk, ldv;
    if (cache) {
        uint8_t* kvb = c->base + M.kv_off + uint64_t(layer) * (M.KV.k_layer_bytes + M.KV.v_layer_bytes);
        kc = reinterpret_cast<bf16_t*>(kvb);
        vt = reinterpret_cast<bf16_t*>(kvb + M.KV.k_layer_bytes);
        k_hs = uint64_t(d.max_seq) * dh;
        ldk = dh;
        ldv = M.KV.v_ld;
        v_hs = uint64_t(dh) * ldv;
    } else {
        vt = reinterpret_cast<bf16_t*>(ws + M.W.vt);
        k_hs = uint64_t(dh);
        ldk = L.n_qkv;
        ldv = M.W.vt_ld;
        v_hs = uint64_t(dh) * ldv;
    }
    dlk::QkvPostArgs qp{qkv, L.n_qkv, T, pos0, Hq, Hkv, dh, d.rope_theta, kc, k_hs, vt, v_hs, ldv, 0, dq, dq + dkv};
    lin_work(Td, L.n_qkv, dm, &fl, &by);
    kbegin(DL_K_GEMM_QKV, fl, by);
    if (T == 1) {
        // single token: rotary embedding and the append to the K / V^T caches happen in the product's epilogue
        dlk::GemvArgs g{nullptr, P(L.w_qkv), dm, P(L.b_qkv), qkv, nullptr, L.n_qkv, dm, dlk::EPI_QKV_POST, qp};
        with_norm(g, NormSrc{in, P(L.norm1_g), P(L.norm1_b), d.norm, d.norm_eps});
        dlk::gemv(g, st);
        kend();
    } else {
        linear(st, T, nbuf, dm, P(L.w_qkv), dm, L.n_qkv, P(L.b_qkv), dlk::EPI_BF16, qkv, L.n_qkv, nullptr, 0);
        kend();
        kbegin(DL_K_QKV_POST, 0, Td * L.n_qkv * 4.0);
        dlk::qkv_post(qp, st);
        kend();
    }
    dlk::AttnArgs aa{qkv, L.n_qkv, cache ? kc : qkv + dq, ldk, k_hs, vt, ldv, v_hs, attn, dq,
                     T, pos0 + T, pos0, Hq, Hkv, dh, d.causal};
    {
        const double pairs = d.causal ? Td * pos0 + Td * (Td + 1.0) / 2.0 : Td * double(pos0 + T);
        kbegin(DL_K_ATTN, 4.0 * dh * Hq * pairs, 2.0 * (2.0 * Td * dq + 2.0 * double(pos0 + T) * dkv));
    }
    if (T == 1 && cache) {
        dlk::DecodeAttnArgs da{qkv, kc, ldk, k_hs, vt, ldv, v_hs, attn, reinterpret_cast<float*>(ws + M.W.dec_part),
                               pos0 + 1, Hq, Hkv, dh};
        dlk::decode_attention(da, st);
    } else {
        dlk::attention(aa, st);
    }
    kend();
    lin_work(Td, dm, dq, &fl, &by);
    kbegin(DL_K_GEMM_O, fl, by + 8.0 * Td * dm);
    linear(st, T, attn, dq, P(L.w_o), dq, dm, P(L.b_o), dlk::EPI_RESID_F32, out, dm, in, dm);
    kend();

    // cross-attention sub-block
    if (d.d_ctx > 0) {
        bf16_t* ctxn = reinterpret_cast<bf16_t*>(ws + M.W.ctxn);
        bf16_t* kvc = reinterpret_cast<bf16_t*>(ws + M.W.kvc);
        bf16_t* vtc = reinterpret_cast<bf16_t*>(ws + M.W.vtc);
        kbegin(DL_K_CROSS, 2.0 * (2.0 * Td * dq * dm + 2.0 * double(n_ctx) * dkv * d.d_ctx) + 4.0 * dh * Hq * Td * n_ctx,
               2.0 * (2.0 * double(dq) * dm + 2.0 * double(dkv) * d.d_ctx));
        dlk::norm_rows(d.norm, out, P(L.normc_g), P(L.normc_b), nbuf, false, T, dm, d.norm_eps, st);
        linear(st, T, nbuf, dm, P(L.w_qc), dm, dq, P(L.b_qc), dlk::EPI_BF16, qkv, dq, nullptr, 0);
        // the context is the same for every layer of a pass: layer 0 converts it to bf16 for all of them (a pass
        // always starts at layer 0, and nothing else writes this buffer)
        if (layer == 0) dlk::cast_f32_bf16(ctx, ctxn, uint64_t(n_ctx) * d.d_ctx, st);
        linear(st, n_ctx, ctxn, d.d_ctx, P(L.w_kvc), d.d_ctx, 2 * dkv, P(L.b_kvc), dlk::EPI_BF16, kvc, 2 * dkv,
               nullptr, 0);
        dlk::QkvPostArgs cp{kvc, 2 * dkv, n_ctx, 0, Hq, Hkv, dh, 0.0f, nullptr, 0, vtc,
                            uint64_t(dh) * M.W.vtc_ld, M.W.vtc_ld, -1, 0, dkv};
        dlk::qkv_post(cp, st);
        dlk::AttnArgs ca{qkv, dq, kvc, 2 * dkv, uint64_t(dh), vtc, M.W.vtc_ld, uint64_t(dh) * M.W.vtc_ld, attn, dq,
                         T, n_ctx, 0, Hq, Hkv, dh, 0,
                         M.W.att_part_bytes ? reinterpret_cast<float*>(ws + M.W.att_part) : nullptr, M.W.att_part_bytes};
        dlk::attention(ca, st);
        linear(st, T, attn, dq, P(L.w_oc), dq, dm, P(L.b_oc), dlk::EPI_RESID_F32, out, dm, out, dm);
        kend();
    }

    // feed-forward sub-block
    NormSrc n2;
    if (fused_norm) {
        n2 = NormSrc{out, P(L.norm2_g), P(L.norm2_b), d.norm, d.norm_eps};
    } else {
        kbegin(DL_K_NORM, 0, Td * dm * 6.0);
        dlk::norm_rows(d.norm, out, P(L.norm2_g), P(L.norm2_b), nbuf, false, T, dm, d.norm_eps, st);
        kend();
    }
    lin_work(Td, L.n_up, dm, &fl, &by);
    kbegin(DL_K_GEMM_UP, fl, 2.0 * (Td * dm + double(L.n_up) * dm + Td * d.d_ff));
    if (d.act == DL_ACT_SWIGLU)
        linear(st, T, nbuf, dm, P(L.w_up), dm, L.n_up, nullptr, dlk::EPI_SWIGLU_BF16, mid, L.ffp, nullptr, 0, n2);
    else
        linear(st, T, nbuf, dm, P(L.w_up), dm, L.n_up, P(L.b_up), dlk::EPI_GELU_BF16, mid, L.ffp, nullptr, 0, n2);
    kend();
    lin_work(Td, dm, d.d_ff, &fl, &by);
    kbegin(DL_K_GEMM_DOWN, fl, by + 8.0 * Td * dm);
    linear(st, T, mid, L.ffp, P(L.w_down), L.ffp, dm, P(L.b_down), dlk::EPI_RESID_F32, out, dm, out, dm);
    kend();
}

hipEvent_t event_of(dl_ctx* c, const dl_trace_op& o) {
    if (o.event_kind == DL_EV_DMA_DONE) return c->ev_dma[o.slot];
    if (o.event_kind == DL_EV_COMPUTE_DONE) return c->ev_comp[o.slot];
    return c->ev_pass;
}

// Enqueues one pass.  force_all: every layer goes through a slot (profiling).
int32_t run_pass(dl_ctx* c, int32_t mi, const float* x, float* y, int32_t T, int32_t pos0, const float* ctx,
                 int32_t n_ctx, bool force_all) {
    Module& M = c->mods[size_t(mi)];
    std::vector<dl_trace_op> ops;
    dl::build_pass(mi, M.d.n_layers, M.resident.data(), c->mode, c->wrap, force_all, &c->book, &ops);
    if (c->tracing || !on_gpu(c)) c->trace.insert(c->trace.end(), ops.begin(), ops.end());
    if (!on_gpu(c)) return DL_OK;
    // Bounded run-ahead for passes that stream: by default the host enqueues such a pass only once the previous
    // streaming pass has finished (inside the pass it still runs far ahead of the GPU: enqueuing takes a tenth of
    // the pass time or less).  Every further pass of short streamed layers kept in flight made copies and kernels
    // slower on MI355X (27-layer encoder, fully streamed: 15.4 ms per pass with one pass in flight, 16.0 with two,
    // 17.7 with three, 19 with four; waiting only for the previous pass's copies instead of its end cost 5 % on
    // the five-stage pipeline).  Passes without copies are never held back.
    bool has_copy = false;
    for (const dl_trace_op& o : ops) has_copy = has_copy || o.op == DL_OP_COPY;
    if (has_copy && c->run_ahead > 0 && c->n_passes >= uint64_t(c->run_ahead))
        DL_HIP(c, hipEventSynchronize(c->ev_inflight[(c->n_passes - uint64_t(c->run_ahead)) % dl_ctx::kMaxRunAhead]));
    // The throttle's event goes in front of the pass's last layer, not behind it: the host then has that layer's
    // execution time to enqueue the head of the next pass, and the GPU does not sit idle between two streaming passes
    // while the host wakes up and launches (70 us per pass of the 27-layer encoder).
    const dl_trace_op* last_exec = nullptr;
    for (const dl_trace_op& o : ops)
        if (o.op == DL_OP_EXEC) last_exec = &o;
    for (const dl_trace_op& o : ops) {
        hipStream_t st = o.queue == 0 ? c->s_compute : c->s_copy;
        if (has_copy && &o == last_exec)
            DL_HIP(c, hipEventRecord(c->ev_inflight[c->n_passes % dl_ctx::kMaxRunAhead], c->s_compute));
        switch (o.op) {
            case DL_OP_WAIT:
                DL_HIP(c, hipStreamWaitEvent(st, event_of(c, o), 0));
                break;
            case DL_OP_RECORD:
                DL_HIP(c, hipEventRecord(event_of(c, o), st));
                break;
            case DL_OP_COPY: {
                TimedOp t{nullptr, nullptr, o.module, o.layer, o.slot, -1};
                if (c->timing) {
                    int32_t rc = timing_event(c, &t.e0);
                    if (rc) return rc;
                    rc = timing_event(c, &t.e1);
                    if (rc) return rc;
                    DL_HIP(c, hipEventRecord(t.e0, st));
                }
                DL_HIP(c, hipMemcpyAsync(c->base + c->slot_off[o.slot], M.store + size_t(o.layer) * M.L.bytes,
                                         M.L.bytes, hipMemcpyHostToDevice, st));
                if (c->timing) {
                    DL_HIP(c, hipEventRecord(t.e1, st));
                    c->last_copy_in_slot[o.slot] = int32_t(c->copies.size());
                    c->copies.push_back(t);
                }
                break;
            }
            case DL_OP_EXEC: {
                const uint8_t* w = o.slot >= 0 ? c->base + c->slot_off[o.slot]
                                               : c->base + M.res_off[size_t(o.layer)];
                TimedOp t{nullptr, nullptr, o.module, o.layer, o.slot, o.slot >= 0 ? c->last_copy_in_slot[o.slot] : -1};
                if (c->timing) {
                    int32_t rc = timing_event(c, &t.e0);
                    if (rc) return rc;
                    rc = timing_event(c, &t.e1);
                    if (rc) return rc;
                    DL_HIP(c, hipEventRecord(t.e0, st));
                }
                run_layer(c, M, o.layer, w, o.layer == 0 ? x : y, y, T, pos0, ctx, n_ctx);
                DL_HIP(c, hipGetLastError());
                if (c->timing) {
                    DL_HIP(c, hipEventRecord(t.e1, st));
                    c->execs.push_back(t);
                }
                break;
            }
            default: break;
        }
    }
    if (has_copy) ++c->n_passes;
    return DL_OK;
}

int32_t check_forward_args(dl_ctx* c, Module* M, const void* x, void* y, int32_t T, int32_t pos0, const void* ctx,
                           int32_t n_ctx) {
    if (!M) return fail(c, DL_ERR_INVALID_ARG, "no such module");
    if (!M->finalized) return fail(c, DL_ERR_BAD_STATE, "module not finalized");
    if (on_gpu(c) && !c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    if (on_gpu(c) && (!x || !y)) return fail(c, DL_ERR_INVALID_ARG, "null activation pointer");
    if (T < 1 || T > M->d.max_tokens) return fail(c, DL_ERR_INVALID_ARG, "n_tokens outside [1, max_tokens]");
    if (pos0 < 0) return fail(c, DL_ERR_INVALID_ARG, "pos0 < 0");
    if (M->d.max_seq == 0 && pos0 != 0) return fail(c, DL_ERR_INVALID_ARG, "pos0 must be 0 without a KV cache");
    if (M->d.max_seq > 0 && pos0 + T > M->d.max_seq) return fail(c, DL_ERR_INVALID_ARG, "pos0 + n_tokens exceeds max_seq");
    if (M->d.d_ctx > 0) {
        if (n_ctx < 1 || n_ctx > M->d.max_ctx) return fail(c, DL_ERR_INVALID_ARG, "n_ctx outside [1, max_ctx]");
        if (on_gpu(c) && !ctx) return fail(c, DL_ERR_INVALID_ARG, "cross-attention source missing");
    }
    return DL_OK;
}

}  // namespace

extern "C" {

int32_t dl_create(dl_ctx** out, int32_t device) {
    if (!out || device < -1) return DL_ERR_INVALID_ARG;
    if (device >= 0) {
        int n = 0;
        if (hipGetDeviceCount(&n) != hipSuccess || device >= n) return DL_ERR_DEVICE;
        if (hipSetDevice(device) != hipSuccess) return DL_ERR_DEVICE;
    }
    if (device >= 0 && device < kStaticMaxDevices) {
        void* p = nullptr;                        // set-up time: resolve the static scratch of this device once
        if (static_scratch_ptr(device, &p) != hipSuccess) return DL_ERR_DEVICE;
    }
    dl_ctx* c = new dl_ctx();
    c->device = device;
    *out = c;
    return DL_OK;
}

int32_t dl_destroy(dl_ctx* c) {
    if (!c) return DL_ERR_INVALID_ARG;
    if (on_gpu(c)) {
        (void)hipSetDevice(c->device);
        if (c->streams_set) {
            (void)hipStreamSynchronize(c->s_copy);
            (void)hipStreamSynchronize(c->s_compute);
        }
        if (c->events_made) {
            for (int s = 0; s < dl::kMaxSlots; ++s) {
                (void)hipEventDestroy(c->ev_dma[s]);
                (void)hipEventDestroy(c->ev_comp[s]);
            }
            (void)hipEventDestroy(c->ev_pass);
            for (int s = 0; s < dl_ctx::kMaxRunAhead; ++s) (void)hipEventDestroy(c->ev_inflight[s]);
        }
        for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    }
    for (Module& M : c->mods) {
        if (!M.store) continue;
        if (on_gpu(c)) (void)hipHostFree(M.store);
        else free(M.store);
    }
    delete c;
    return DL_OK;
}

const char* dl_last_error(const dl_ctx* c) { return c ? c->err.c_str() : g_static_err.c_str(); }

int32_t dl_set_arena(dl_ctx* c, void* dev_base, uint64_t bytes) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena already set");
    if (bytes < dl::kAlign) return fail(c, DL_ERR_INVALID_ARG, "arena too small");
    if (on_gpu(c) && (!dev_base || (reinterpret_cast<uintptr_t>(dev_base) % dl::kAlign)))
        return fail(c, DL_ERR_INVALID_ARG, "arena base must be a 256-byte aligned device pointer");
    c->base = static_cast<uint8_t*>(dev_base);
    c->arena.reset(bytes);
    return DL_OK;
}

int32_t dl_arena_alloc(dl_ctx* c, uint64_t bytes, void** out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!out || bytes == 0) return fail(c, DL_ERR_INVALID_ARG, "bad arguments");
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    uint64_t off = 0;
    rc = add_permanent(c, bytes, &off);
    if (rc) return rc;
    *out = c->base + off;
    return DL_OK;
}

int32_t dl_arena_free(dl_ctx* c, void* p) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    const uint64_t off = uint64_t(static_cast<uint8_t*>(p) - c->base);
    auto it = std::find(c->perms.begin(), c->perms.end(), off);
    if (!p || it == c->perms.end() || !c->arena.free(off)) return fail(c, DL_ERR_INVALID_ARG, "pointer is not a live arena block of the caller");
    c->perms.erase(it);
    return DL_OK;
}

int32_t dl_arena_stats(const dl_ctx* c, uint64_t* used, uint64_t* peak, uint64_t* cap) {
    if (!c) return DL_ERR_INVALID_ARG;
    if (used) *used = c->arena.used();
    if (peak) *peak = c->arena.peak();
    if (cap) *cap = c->arena.capacity();
    return DL_OK;
}

int32_t dl_residency_budget(const dl_ctx* c, uint64_t* bytes) {
    if (!c || !bytes) return DL_ERR_INVALID_ARG;
    uint64_t top = c->arena.capacity();
    for (uint64_t off : c->perms) top = std::min(top, off);
    for (const Module& M : c->mods)
        if (M.finalized) top = std::min(top, M.ws_off);
    *bytes = top;
    return DL_OK;
}

int32_t dl_set_streams(dl_ctx* c, void* compute_stream, void* copy_stream) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!on_gpu(c)) return DL_OK;
    if (compute_stream == copy_stream) return fail(c, DL_ERR_INVALID_ARG, "the two streams must be distinct");
    rc = sync_streams(c);
    if (rc) return rc;
    c->s_compute = static_cast<hipStream_t>(compute_stream);
    c->s_copy = static_cast<hipStream_t>(copy_stream);
    c->streams_set = true;
    c->book = dl::SlotBook();
    c->book.n_slots = c->n_slots;
    return make_events(c);
}

int32_t dl_module_create(dl_ctx* c, const dl_module_desc* desc, int32_t* module_out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!desc || !module_out) return fail(c, DL_ERR_INVALID_ARG, "null argument");
    std::string why;
    if (!dl::validate_desc(*desc, &why)) return fail(c, DL_ERR_INVALID_ARG, why);
    Module M;
    M.d = *desc;
    M.L = dl::make_layout(*desc);
    M.W = dl::make_workspace(*desc);
    M.KV = dl::make_kv(*desc);
    const uint64_t total = uint64_t(desc->n_layers) * M.L.bytes;
    if (on_gpu(c)) {
        void* p = nullptr;
        if (hipHostMalloc(&p, total, hipHostMallocDefault) != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(c, DL_ERR_HOST_ALLOC, "pinned host allocation failed");
        }
        M.store = static_cast<uint8_t*>(p);
    } else {
        M.store = static_cast<uint8_t*>(malloc(total));
        if (!M.store) return fail(c, DL_ERR_HOST_ALLOC, "host allocation failed");
    }
    memset(M.store, 0, total);    // alignment gaps and K padding must be exact zeros
    M.set_mask.assign(size_t(desc->n_layers), 0u);
    M.resident.assign(size_t(desc->n_layers), 0);
    M.res_off.assign(size_t(desc->n_layers), 0);
    c->mods.push_back(M);
    *module_out = int32_t(c->mods.size() - 1);
    return DL_OK;
}

int32_t dl_layer_set_tensor(dl_ctx* c, int32_t module, int32_t layer, int32_t tid, const void* host, uint64_t n) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M) return fail(c, DL_ERR_INVALID_ARG, "no such module");
    if (M->finalized) return fail(c, DL_ERR_BAD_STATE, "module already finalized");
    if (layer < 0 || layer >= M->d.n_layers) return fail(c, DL_ERR_INVALID_ARG, "layer out of range");
    if (tid < 0 || tid >= DL_T_COUNT || !host) return fail(c, DL_ERR_INVALID_ARG, "bad tensor id or null data");
    const uint64_t want = dl::tensor_elems(M->d, tid);
    if (want == 0) return fail(c, DL_ERR_INVALID_ARG, "this module has no such tensor");
    if (want != n) return fail(c, DL_ERR_INVALID_ARG, "tensor has the wrong number of elements");
    dl::pack_tensor(M->d, M->L, tid, static_cast<const uint16_t*>(host), M->store + size_t(layer) * M->L.bytes);
    M->set_mask[size_t(layer)] |= 1u << tid;
    return DL_OK;
}

int32_t dl_set_resident_tensor(dl_ctx* c, int32_t module, int32_t which, const void* host, uint64_t n) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M) return fail(c, DL_ERR_INVALID_ARG, "no such module");
    if (which < 0 || which >= DL_R_COUNT || !host) return fail(c, DL_ERR_INVALID_ARG, "bad tensor id or null data");
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    uint64_t want = 0;
    if (which == DL_R_EMBED || which == DL_R_HEAD) want = uint64_t(M->d.vocab) * M->d.d_model;
    else if (which == DL_R_FINAL_NORM_G) want = M->d.d_model;
    else want = M->d.norm == DL_NORM_LN ? M->d.d_model : 0;
    if (want == 0 || want != n) return fail(c, DL_ERR_INVALID_ARG, "resident tensor has the wrong size for this module");
    rc = sync_streams(c);
    if (rc) return rc;
    if (!M->rt_set[which]) {
        uint64_t off = 0;
        rc = add_permanent(c, 2 * n, &off);
        if (rc) return rc;
        M = get_module(c, module);
        M->rt_off[which] = off;
        M->rt_set[which] = true;
    }
    if (on_gpu(c)) DL_HIP(c, hipMemcpy(c->base + M->rt_off[which], host, 2 * n, hipMemcpyHostToDevice));
    return DL_OK;
}

int32_t dl_module_finalize(dl_ctx* c, int32_t module) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M) return fail(c, DL_ERR_INVALID_ARG, "no such module");
    if (M->finalized) return fail(c, DL_ERR_BAD_STATE, "module already finalized");
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    const uint32_t need = dl::required_tensor_mask(M->d);
    for (int32_t i = 0; i < M->d.n_layers; ++i)
        if ((M->set_mask[size_t(i)] & need) != need) {
            char buf[96];
            snprintf(buf, sizeof buf, "layer %d is missing tensors (have mask 0x%x, need 0x%x)", i,
                     M->set_mask[size_t(i)], need);
            return fail(c, DL_ERR_BAD_STATE, buf);
        }
    rc = sync_streams(c);
    if (rc) return rc;
    // KV cache (never moves) on the top stack, the workspace below it, the slots from the bottom: all or nothing
    Proposal p = current_proposal(c);
    p.counted[size_t(module)] = 1;
    p.ws_bytes[size_t(module)] = M->W.bytes;
    if (M->KV.bytes) p.new_perm.push_back(M->KV.bytes);
    std::vector<uint64_t> offs;
    rc = relayout(c, p, &offs);
    if (rc) return rc;
    M = get_module(c, module);
    M->kv_off = M->KV.bytes ? offs[0] : 0;
    if (on_gpu(c) && M->KV.bytes) DL_HIP(c, hipMemset(c->base + M->kv_off, 0, M->KV.bytes));
    M->finalized = true;
    return DL_OK;
}

int32_t dl_module_layer_bytes(const dl_ctx* c, int32_t module, uint64_t* packed, uint64_t* params) {
    if (!c || module < 0 || size_t(module) >= c->mods.size()) return DL_ERR_INVALID_ARG;
    if (packed) *packed = c->mods[size_t(module)].L.bytes;
    if (params) *params = c->mods[size_t(module)].L.param_bytes;
    return DL_OK;
}

int32_t dl_set_residency(dl_ctx* c, int32_t module, const int32_t* idx, int32_t n) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M) return fail(c, DL_ERR_INVALID_ARG, "no such module");
    if (!M->finalized) return fail(c, DL_ERR_BAD_STATE, "module not finalized");
    if (n < 0 || n > M->d.n_layers || (n > 0 && !idx)) return fail(c, DL_ERR_INVALID_ARG, "bad resident count");
    std::vector<uint8_t> res(size_t(M->d.n_layers), 0);
    for (int32_t i = 0; i < n; ++i) {
        if (idx[i] < 0 || idx[i] >= M->d.n_layers) return fail(c, DL_ERR_INVALID_ARG, "resident layer index out of range");
        if (res[size_t(idx[i])]) return fail(c, DL_ERR_INVALID_ARG, "duplicate resident layer index");
        res[size_t(idx[i])] = 1;
    }
    rc = sync_streams(c);
    if (rc) return rc;
    Proposal p = current_proposal(c);
    p.resident[size_t(module)] = res;
    return relayout(c, p);
}

int32_t dl_get_residency(const dl_ctx* c, int32_t module, int32_t* idx_out, int32_t* n_out) {
    if (!c || module < 0 || size_t(module) >= c->mods.size() || !n_out) return DL_ERR_INVALID_ARG;
    const Module& M = c->mods[size_t(module)];
    int32_t n = 0;
    for (int32_t i = 0; i < M.d.n_layers; ++i)
        if (M.resident[size_t(i)]) {
            if (idx_out) idx_out[n] = i;
            ++n;
        }
    *n_out = n;
    return DL_OK;
}

int32_t dl_set_mode(dl_ctx* c, int32_t mode, int32_t wrap) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (mode != DL_MODE_PIPELINED && mode != DL_MODE_SEQUENTIAL) return fail(c, DL_ERR_INVALID_ARG, "unknown mode");
    c->mode = mode;
    c->wrap = wrap ? 1 : 0;
    return DL_OK;
}

int32_t dl_forward(dl_ctx* c, int32_t module, const void* x, void* y, int32_t T, int32_t pos0, const void* ctx,
                   int32_t n_ctx) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    rc = check_forward_args(c, M, x, y, T, pos0, ctx, n_ctx);
    if (rc) return rc;
    return run_pass(c, module, static_cast<const float*>(x), static_cast<float*>(y), T, pos0,
                    static_cast<const float*>(ctx), n_ctx, false);
}

int32_t dl_embed_token(dl_ctx* c, int32_t module, int32_t token, void* x_dev) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M || !M->finalized) return fail(c, DL_ERR_BAD_STATE, "module missing or not finalized");
    if (!M->rt_set[DL_R_EMBED]) return fail(c, DL_ERR_BAD_STATE, "embedding table not set");
    if (token < 0 || token >= M->d.vocab) return fail(c, DL_ERR_INVALID_ARG, "token out of range");
    if (!on_gpu(c)) return DL_OK;
    if (!x_dev) return fail(c, DL_ERR_INVALID_ARG, "null output");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    dlk::embed_row(reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_EMBED]), M->d.d_model, nullptr, token,
                   static_cast<float*>(x_dev), c->s_compute);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_final_norm(dl_ctx* c, int32_t module, const void* h, void* out, int32_t T) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M || !M->finalized) return fail(c, DL_ERR_BAD_STATE, "module missing or not finalized");
    if (!M->rt_set[DL_R_FINAL_NORM_G] || (M->d.norm == DL_NORM_LN && !M->rt_set[DL_R_FINAL_NORM_B]))
        return fail(c, DL_ERR_BAD_STATE, "final norm parameters not set");
    if (T < 1) return fail(c, DL_ERR_INVALID_ARG, "n_tokens < 1");
    if (!on_gpu(c)) return DL_OK;
    if (!h || !out) return fail(c, DL_ERR_INVALID_ARG, "null pointer");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    dlk::norm_rows(M->d.norm, static_cast<const float*>(h),
                   reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_FINAL_NORM_G]),
                   M->rt_set[DL_R_FINAL_NORM_B] ? reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_FINAL_NORM_B]) : nullptr,
                   out, true, T, M->d.d_model, M->d.norm_eps, c->s_compute);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

// final norm + head + greedy choice; with x_next != nullptr the chosen token's embedding row is written there (and the
// token to token_copy, if given) by the same launch that picks it
static int32_t head_common(dl_ctx* c, Module* M, const void* h, int32_t* token_copy = nullptr, float* x_next = nullptr) {
    if (!M || !M->finalized) return fail(c, DL_ERR_BAD_STATE, "module missing or not finalized");
    if (M->d.vocab <= 0 || !M->rt_set[DL_R_HEAD] || !M->rt_set[DL_R_FINAL_NORM_G] ||
        (M->d.norm == DL_NORM_LN && !M->rt_set[DL_R_FINAL_NORM_B]))
        return fail(c, DL_ERR_BAD_STATE, "head or final norm parameters not set");
    if (x_next && !M->rt_set[DL_R_EMBED]) return fail(c, DL_ERR_BAD_STATE, "embedding table not set");
    if (!on_gpu(c)) return DL_OK;
    if (!h) return fail(c, DL_ERR_INVALID_ARG, "null hidden state");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    uint8_t* ws = c->base + M->ws_off;
    float* logits = reinterpret_cast<float*>(ws + M->W.logits);
    int32_t* tok = reinterpret_cast<int32_t*>(ws + M->W.token);
    hipStream_t st = c->s_compute;
    // the final normalisation happens inside the matrix-vector kernel
    dlk::GemvArgs g{nullptr, reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_HEAD]), M->d.d_model, nullptr,
                    logits, nullptr, M->d.vocab, M->d.d_model, dlk::EPI_F32};
    g.norm_x = static_cast<const float*>(h);
    g.norm_g = reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_FINAL_NORM_G]);
    g.norm_b = M->rt_set[DL_R_FINAL_NORM_B] ? reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_FINAL_NORM_B]) : nullptr;
    g.norm_kind = M->d.norm;
    g.norm_eps = M->d.norm_eps;
    dlk::gemv(g, st);
    dlk::argmax_f32(logits, M->d.vocab, tok, token_copy,
                    x_next ? reinterpret_cast<const bf16_t*>(c->base + M->rt_off[DL_R_EMBED]) : nullptr, M->d.d_model, x_next,
                    st);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_logits_argmax(dl_ctx* c, int32_t module, const void* h, int32_t* token_out, float* logits_out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!token_out) return fail(c, DL_ERR_INVALID_ARG, "null token_out");
    rc = head_common(c, M, h);
    if (rc) return rc;
    if (!on_gpu(c)) { *token_out = 0; return DL_OK; }
    uint8_t* ws = c->base + M->ws_off;
    DL_HIP(c, hipMemcpyAsync(token_out, ws + M->W.token, 4, hipMemcpyDeviceToHost, c->s_compute));
    if (logits_out)
        DL_HIP(c, hipMemcpyAsync(logits_out, ws + M->W.logits, 4 * size_t(M->d.vocab), hipMemcpyDeviceToHost, c->s_compute));
    DL_HIP(c, hipStreamSynchronize(c->s_compute));
    return DL_OK;
}

int32_t dl_greedy_step(dl_ctx* c, int32_t module, const void* h, int32_t* token_dev, void* x_dev) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (M && M->finalized && !M->rt_set[DL_R_EMBED]) return fail(c, DL_ERR_BAD_STATE, "embedding table not set");
    if (on_gpu(c) && !x_dev) return fail(c, DL_ERR_INVALID_ARG, "null x_dev");
    return head_common(c, M, h, token_dev, static_cast<float*>(x_dev));
}

int32_t dl_greedy_step_static(int32_t device, void* stream, const void* h_dev, const void* head_dev, const void* embed_dev,
                              const void* norm_g_dev, const void* norm_b_dev, int32_t norm, float norm_eps,
                              int32_t d_model, int32_t vocab, int32_t* token_dev, void* x_dev) {
    auto bad = [&](int32_t code, const std::string& msg) { g_static_err = msg; return code; };
    if (device < 0 || device >= kStaticMaxDevices) return bad(DL_ERR_INVALID_ARG, "device ordinal outside [0, 64)");
    if (vocab < 1 || vocab > kStaticMaxVocab) {
        char buf[128];
        snprintf(buf, sizeof buf, "vocab %d outside [1, %d]: the static scratch holds at most %d logits", vocab, kStaticMaxVocab, kStaticMaxVocab);
        return bad(DL_ERR_INVALID_ARG, buf);
    }
    if (d_model < 8 || d_model % 8 || d_model > 16384) return bad(DL_ERR_INVALID_ARG, "d_model must be a multiple of 8 in [8, 16384]");
    if (norm != DL_NORM_RMS && norm != DL_NORM_LN) return bad(DL_ERR_INVALID_ARG, "unknown norm");
    if (!(norm_eps >= 0)) return bad(DL_ERR_INVALID_ARG, "norm_eps < 0");
    if (!h_dev || !head_dev || !norm_g_dev || !token_dev || (norm == DL_NORM_LN && !norm_b_dev))
        return bad(DL_ERR_INVALID_ARG, "null device pointer");
    if ((x_dev == nullptr) != (embed_dev == nullptr)) return bad(DL_ERR_INVALID_ARG, "x_dev and embed_dev go together");
    // the call runs with `device` current and leaves the caller's current device as it found it
    struct DeviceGuard {
        int prev = -1;
        ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
    } guard;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) {
        e = hipSetDevice(device);
        if (e == hipSuccess) guard.prev = cur;
    }
    void* sp = nullptr;
    if (e == hipSuccess) e = static_scratch_ptr(device, &sp);
    if (e != hipSuccess) return bad(DL_ERR_DEVICE, std::string("static scratch of the device: ") + hipGetErrorString(e));
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every logit of this call is written before the argmax reads it: nothing in the scratch has to start at zero,
    // and what a larger earlier call left beyond `vocab` is never read
    float* logits = static_cast<float*>(sp);
    int32_t* tok = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(sp) + size_t(kStaticMaxVocab) * 4);
    dlk::GemvArgs g{nullptr, static_cast<const bf16_t*>(head_dev), d_model, nullptr, logits, nullptr, vocab, d_model, dlk::EPI_F32};
    g.norm_x = static_cast<const float*>(h_dev);
    g.norm_g = static_cast<const bf16_t*>(norm_g_dev);
    g.norm_b = norm == DL_NORM_LN ? static_cast<const bf16_t*>(norm_b_dev) : nullptr;
    g.norm_kind = norm;
    g.norm_eps = norm_eps;
    dlk::gemv(g, st);
    dlk::argmax_f32(logits, vocab, tok, token_dev, static_cast<const bf16_t*>(embed_dev), d_model, static_cast<float*>(x_dev), st);
    e = hipGetLastError();
    if (e != hipSuccess) return bad(DL_ERR_DEVICE, std::string("launch failed: ") + hipGetErrorString(e));
    return DL_OK;
}

int32_t dl_mlp_create(dl_ctx* c, int32_t d_in, int32_t d_hidden, int32_t d_out, const void* w1, const void* b1,
                      const void* w2, const void* b2, int32_t max_tokens, int32_t* mlp_out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!mlp_out || !w2 || d_in < 8 || d_in % 8 || d_hidden < 0 || d_hidden % 8 || d_out < 1 || max_tokens < 1 ||
        (d_hidden > 0 && !w1))
        return fail(c, DL_ERR_INVALID_ARG, "bad MLP description");
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    Mlp m;
    m.d_in = d_in; m.d_hidden = d_hidden; m.d_out = d_out; m.max_tokens = max_tokens;
    m.has_b1 = d_hidden > 0 && b1 != nullptr;
    m.has_b2 = b2 != nullptr;
    const uint64_t k2 = d_hidden > 0 ? d_hidden : d_in;
    struct Part { uint64_t* off; uint64_t bytes; const void* src; };
    std::vector<Part> parts;
    if (d_hidden > 0) parts.push_back({&m.w1, 2ull * d_hidden * d_in, w1});
    if (m.has_b1) parts.push_back({&m.b1, 2ull * d_hidden, b1});
    parts.push_back({&m.w2, 2ull * d_out * k2, w2});
    if (m.has_b2) parts.push_back({&m.b2, 2ull * d_out, b2});
    parts.push_back({&m.xin, 2ull * max_tokens * d_in, nullptr});
    if (d_hidden > 0) parts.push_back({&m.hid, 2ull * max_tokens * d_hidden, nullptr});
    rc = sync_streams(c);
    if (rc) return rc;
    Proposal prop = current_proposal(c);          // all or nothing
    for (Part& p : parts) prop.new_perm.push_back(p.bytes);
    std::vector<uint64_t> offs;
    rc = relayout(c, prop, &offs);
    if (rc) return rc;
    for (size_t i = 0; i < parts.size(); ++i) *parts[i].off = offs[i];
    if (on_gpu(c))
        for (Part& p : parts)
            if (p.src) DL_HIP(c, hipMemcpy(c->base + *p.off, p.src, p.bytes, hipMemcpyHostToDevice));
    c->mlps.push_back(m);
    *mlp_out = int32_t(c->mlps.size() - 1);
    return DL_OK;
}

int32_t dl_mlp_forward(dl_ctx* c, int32_t mlp, const void* x, void* y, int32_t T) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (mlp < 0 || size_t(mlp) >= c->mlps.size()) return fail(c, DL_ERR_INVALID_ARG, "no such MLP");
    const Mlp& m = c->mlps[size_t(mlp)];
    if (T < 1 || T > m.max_tokens) return fail(c, DL_ERR_INVALID_ARG, "n_tokens outside [1, max_tokens]");
    if (!on_gpu(c)) return DL_OK;
    if (!x || !y) return fail(c, DL_ERR_INVALID_ARG, "null pointer");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    hipStream_t st = c->s_compute;
    auto P = [&](uint64_t off) { return reinterpret_cast<bf16_t*>(c->base + off); };
    dlk::cast_f32_bf16(static_cast<const float*>(x), P(m.xin), uint64_t(T) * m.d_in, st);
    const bf16_t* a2 = P(m.xin);
    int k2 = m.d_in;
    if (m.d_hidden > 0) {
        dlk::GemmArgs g1{P(m.xin), m.d_in, P(m.w1), m.d_in, m.has_b1 ? P(m.b1) : nullptr, P(m.hid), m.d_hidden, nullptr, 0,
                         T, m.d_hidden, m.d_in, dlk::EPI_GELU_BF16};
        dlk::gemm(g1, st);
        a2 = P(m.hid);
        k2 = m.d_hidden;
    }
    dlk::GemmArgs g2{a2, k2, P(m.w2), k2, m.has_b2 ? P(m.b2) : nullptr, y, m.d_out, nullptr, 0, T, m.d_out, k2, dlk::EPI_F32};
    dlk::gemm(g2, st);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_mean_pool(dl_ctx* c, const void* x, void* y, int32_t n_out, int32_t group, int32_t d) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (n_out < 1 || group < 1 || d < 1) return fail(c, DL_ERR_INVALID_ARG, "bad sizes");
    if (!on_gpu(c)) return DL_OK;
    if (!x || !y || x == y) return fail(c, DL_ERR_INVALID_ARG, "null or aliasing pointers");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    dlk::mean_pool_rows(static_cast<const float*>(x), static_cast<float*>(y), n_out, group, d, c->s_compute);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_axpy(dl_ctx* c, void* y, float alpha, const void* x, uint64_t n) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!on_gpu(c) || n == 0) return DL_OK;
    if (!x || !y) return fail(c, DL_ERR_INVALID_ARG, "null pointer");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    dlk::axpy_f32(static_cast<float*>(y), alpha, static_cast<const float*>(x), n, c->s_compute);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_add_time_embedding(dl_ctx* c, const void* x, void* y, float tval, int32_t T, int32_t d) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (T < 1 || d < 2 || d % 2) return fail(c, DL_ERR_INVALID_ARG, "bad sizes");
    if (!on_gpu(c)) return DL_OK;
    if (!x || !y) return fail(c, DL_ERR_INVALID_ARG, "null pointer");
    if (!c->streams_set) return fail(c, DL_ERR_BAD_STATE, "streams not set");
    dlk::add_time_embedding(static_cast<const float*>(x), static_cast<float*>(y), tval, T, d, c->s_compute);
    DL_HIP(c, hipGetLastError());
    return DL_OK;
}

int32_t dl_vla_infer(dl_ctx* c, const dl_vla_desc* v, const dl_vla_buffers* b) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!v || !b) return fail(c, DL_ERR_INVALID_ARG, "null description or buffers");
    Module* vit = get_module(c, v->m_vit);
    Module* dec = get_module(c, v->m_dec);
    Module* act = get_module(c, v->m_act);
    if (!vit || !dec || !act || !vit->finalized || !dec->finalized || !act->finalized)
        return fail(c, DL_ERR_BAD_STATE, "the three modules must exist and be finalized");
    if (v->mlp_proj < 0 || size_t(v->mlp_proj) >= c->mlps.size() || v->mlp_out < 0 || size_t(v->mlp_out) >= c->mlps.size())
        return fail(c, DL_ERR_INVALID_ARG, "no such MLP");
    const Mlp& proj = c->mlps[size_t(v->mlp_proj)];
    const Mlp& outp = c->mlps[size_t(v->mlp_out)];
    if (v->pool < 1 || v->n_patches < v->pool || v->n_patches % v->pool || v->n_text < 0 || v->n_actions < 1 || v->n_decode < 0 ||
        v->n_euler < 1 || v->out_dim < 1)
        return fail(c, DL_ERR_INVALID_ARG, "bad token counts");
    const int32_t n_vis = v->n_patches / v->pool, n_prefill = n_vis + v->n_text;
    const int32_t dv = vit->d.d_model, dd = dec->d.d_model, da = act->d.d_model;
    if (proj.d_in != dv || proj.d_out != dd || outp.d_in != da || outp.d_out != v->out_dim || outp.d_hidden != 0)
        return fail(c, DL_ERR_INVALID_ARG, "MLP shapes do not match the modules");
    if (act->d.d_ctx != dd) return fail(c, DL_ERR_INVALID_ARG, "the action stack's d_ctx must equal the decoder's d_model");
    if (dec->d.max_seq < n_prefill + v->n_decode || dec->d.vocab <= 0)
        return fail(c, DL_ERR_INVALID_ARG, "the decoder needs a head and a KV cache of n_prefill + n_decode positions");
    if (v->n_patches > vit->d.max_tokens || v->n_patches > proj.max_tokens || n_prefill > dec->d.max_tokens ||
        v->n_actions > act->d.max_tokens || v->n_actions > outp.max_tokens || n_prefill > act->d.max_ctx)
        return fail(c, DL_ERR_INVALID_ARG, "token counts exceed what the modules were sized for");
    if (on_gpu(c) && (!b->patches || !b->vit_out || !b->proj_out || !b->seq || !b->hidden || !b->hidden_ctx || !b->x1 || !b->y1 ||
                      (v->n_decode > 0 && !b->tokens) || !b->actions || !b->act_in || !b->velocity || !b->trajectory))
        return fail(c, DL_ERR_INVALID_ARG, "null buffer");
#define DL_STEP(call) do { rc = (call); if (rc) return rc; } while (0)
    // stages 1-2: encoder, merger
    DL_STEP(dl_forward(c, v->m_vit, b->patches, b->vit_out, v->n_patches, 0, nullptr, 0));
    DL_STEP(dl_mlp_forward(c, v->mlp_proj, b->vit_out, b->proj_out, v->n_patches));
    DL_STEP(dl_mean_pool(c, b->proj_out, b->seq, n_vis, v->pool, dd));
    // stage 3: prefill over [visual tokens ; text embeddings]
    DL_STEP(dl_forward(c, v->m_dec, b->seq, b->hidden, n_prefill, 0, nullptr, 0));
    DL_STEP(dl_final_norm(c, v->m_dec, b->hidden, b->hidden_ctx, n_prefill));
    // stage 4: greedy decode; the un-normed state goes into the head, which normalises it itself
    const void* h = on_gpu(c) ? static_cast<const char*>(b->hidden) + size_t(n_prefill - 1) * dd * 4 : nullptr;
    for (int32_t s = 0; s < v->n_decode; ++s) {
        DL_STEP(dl_greedy_step(c, v->m_dec, h, on_gpu(c) ? b->tokens + s : nullptr, b->x1));
        DL_STEP(dl_forward(c, v->m_dec, b->x1, b->y1, 1, n_prefill + s, nullptr, 0));
        h = b->y1;
    }
    // stage 5: Euler steps of the action stack against the fixed context, then the trajectory head
    for (int32_t s = 0; s < v->n_euler; ++s) {
        DL_STEP(dl_add_time_embedding(c, b->actions, b->act_in, float(s) / float(v->n_euler), v->n_actions, da));
        DL_STEP(dl_forward(c, v->m_act, b->act_in, b->velocity, v->n_actions, 0, b->hidden_ctx, n_prefill));
        DL_STEP(dl_axpy(c, b->actions, 1.0f / float(v->n_euler), b->velocity, uint64_t(v->n_actions) * da));
    }
    DL_STEP(dl_mlp_forward(c, v->mlp_out, b->actions, b->trajectory, v->n_actions));
#undef DL_STEP
    return DL_OK;
}

int32_t dl_sync(dl_ctx* c) {
    int32_t rc = enter(c);
    if (rc) return rc;
    return sync_streams(c);
}

int32_t dl_set_timing(dl_ctx* c, int32_t on) {
    int32_t rc = enter(c);
    if (rc) return rc;
    c->timing = on != 0;
    return DL_OK;
}

int32_t dl_collect_stats(dl_ctx* c, dl_run_stats* stats, dl_layer_record* recs, int32_t cap) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!stats) return fail(c, DL_ERR_INVALID_ARG, "null stats");
    memset(stats, 0, sizeof *stats);
    stats->hidden_frac = 1.0;
    stats->arena_peak = c->arena.peak();
    if (!on_gpu(c)) return DL_OK;
    rc = sync_streams(c);
    if (rc) return rc;
    if (c->execs.empty()) {
        c->copies.clear();
        if (c->krecs.empty()) c->ev_next = 0;
        return DL_OK;
    }
    // origin: the earlier of the first copy start and the first exec start
    hipEvent_t origin = c->execs[0].e0;
    if (!c->copies.empty()) {
        float ms = 0;
        DL_HIP(c, hipEventElapsedTime(&ms, c->copies[0].e0, c->execs[0].e0));
        if (ms > 0) origin = c->copies[0].e0;
    }
    auto rel = [&](hipEvent_t e, float* out) -> hipError_t { return hipEventElapsedTime(out, origin, e); };
    std::vector<float> c0(c->copies.size()), c1(c->copies.size());
    for (size_t i = 0; i < c->copies.size(); ++i) {
        DL_HIP(c, rel(c->copies[i].e0, &c0[i]));
        DL_HIP(c, rel(c->copies[i].e1, &c1[i]));
    }
    double dma = 0, exe = 0, exposed = 0, last_end = 0;
    uint64_t bytes = 0;
    float prev_exe_end = 0;
    for (size_t i = 0; i < c->execs.size(); ++i) {
        const TimedOp& t = c->execs[i];
        float e0, e1;
        DL_HIP(c, rel(t.e0, &e0));
        DL_HIP(c, rel(t.e1, &e1));
        exe += double(e1) - e0;
        dl_layer_record r{t.module, t.layer, t.slot >= 0 ? 1 : 0, t.slot, 0, 0, e0, e1};
        if (t.copy_index >= 0) {
            const float d0 = c0[size_t(t.copy_index)], d1 = c1[size_t(t.copy_index)];
            r.dma_start_ms = d0;
            r.dma_end_ms = d1;
            dma += double(d1) - d0;
            bytes += c->mods[size_t(t.module)].L.bytes;
            exposed += std::max(0.0, double(d1) - std::max(double(prev_exe_end), double(d0)));
        }
        prev_exe_end = e1;
        last_end = std::max(last_end, double(e1));
        if (recs && int32_t(i) < cap) recs[i] = r;
    }
    stats->total_ms = last_end;
    stats->dma_ms = dma;
    stats->exe_ms = exe;
    stats->exposed_ms = exposed;
    stats->hidden_frac = dma > 0 ? 1.0 - exposed / dma : 1.0;
    stats->bytes_streamed = bytes;
    stats->h2d_gbps = dma > 0 ? double(bytes) / (dma * 1e6) : 0.0;
    stats->n_layer_records = int32_t(c->execs.size());
    c->copies.clear();
    c->execs.clear();
    for (int s = 0; s < dl::kMaxSlots; ++s) c->last_copy_in_slot[s] = -1;
    if (c->krecs.empty()) c->ev_next = 0;
    return DL_OK;
}

int32_t dl_profile(dl_ctx* c, int32_t module, int32_t T, int32_t pos0, const void* x, const void* ctx, int32_t n_ctx,
                   int32_t iters, dl_layer_profile* out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!out || iters < 2) return fail(c, DL_ERR_INVALID_ARG, "need an output array and at least 2 iterations");
    if (!on_gpu(c)) return fail(c, DL_ERR_BAD_STATE, "profiling needs a device context");
    float* scratch = nullptr;
    {
        // validated against a placeholder output pointer; the real one is carved below
        rc = check_forward_args(c, M, x, const_cast<void*>(x), T, pos0, ctx, n_ctx);
        if (rc) return rc;
    }
    if (!c->slots_alloc || c->slot_bytes < M->L.bytes)
        return fail(c, DL_ERR_BAD_STATE, "the slots cannot hold this module's layers (it is fully resident): profile with at least one of its layers streamed");
    rc = sync_streams(c);
    if (rc) return rc;
    if (!c->copies.empty() || !c->execs.empty()) return fail(c, DL_ERR_BAD_STATE, "collect pending statistics first");
    // temporaries of this call (its output row block, weight copies for the continuous run) come from the bottom of
    // the arena and are gone when it returns; the peak they reach is not the path's
    const uint64_t peak_before = c->arena.peak();
    uint64_t tmp_off = 0;
    if (!c->arena.alloc(uint64_t(T) * M->d.d_model * 4, &tmp_off))
        return fail(c, DL_ERR_BUDGET_EXCEEDED, "arena cannot hold the profiling run's activation block");
    scratch = reinterpret_cast<float*>(c->base + tmp_off);
    const int32_t mode0 = c->mode, wrap0 = c->wrap;
    const bool timing0 = c->timing, tracing0 = c->tracing;
    c->mode = DL_MODE_SEQUENTIAL;
    c->wrap = 0;
    c->timing = true;
    c->tracing = false;
    c->book = dl::SlotBook();
    c->book.n_slots = c->n_slots;
    const int32_t Ln = M->d.n_layers;
    std::vector<double> dma(size_t(Ln), 0.0), exe(size_t(Ln), 0.0), hot(size_t(Ln), 0.0), fence(size_t(Ln), 0.0);
    double timed_span = 0.0;         // first copy start -> last kernel end of the passes with timing events, summed
    double fence_excess = 0.0;       // per layer: what the timing events added to a sequential pass
    double cont_scale = 1.0;         // copy time inside a train of copies / isolated copy time
    double hot_total = 0.0;          // the uninterrupted run of all layers, median
    double fence_hot = 0.0;          // per layer: what the event protocol of a streamed layer adds to that run
    double load_scale = 1.0;         // that run next to a train of copies / that run alone
    for (int32_t it = 0; it < iters && rc == DL_OK; ++it) {
        rc = run_pass(c, module, static_cast<const float*>(x), scratch, T, pos0, static_cast<const float*>(ctx), n_ctx, true);
        if (rc) break;
        dl_run_stats st;
        std::vector<dl_layer_record> recs;
        recs.resize(size_t(Ln));
        rc = dl_collect_stats(c, &st, recs.data(), Ln);
        if (rc) break;
        if (it == 0) continue;       // the first iteration is discarded
        for (int32_t i = 0; i < Ln; ++i) {
            dma[size_t(i)] += double(recs[size_t(i)].dma_end_ms) - recs[size_t(i)].dma_start_ms;
            exe[size_t(i)] += double(recs[size_t(i)].exe_end_ms) - recs[size_t(i)].exe_start_ms;
            // hand-offs: copy end -> first kernel, last kernel -> next copy (the last layer has no next copy: its
            // first hand-off is counted twice)
            const double in = double(recs[size_t(i)].exe_start_ms) - recs[size_t(i)].dma_end_ms;
            const double outw = i + 1 < Ln ? double(recs[size_t(i + 1)].dma_start_ms) - recs[size_t(i)].exe_end_ms : in;
            fence[size_t(i)] += std::max(0.0, in) + std::max(0.0, outw);
        }
        timed_span += double(recs[size_t(Ln - 1)].exe_end_ms) - recs[0].dma_start_ms;
    }
    // The event pair around every copy and every layer costs a few microseconds each, and in a sequential pass all
    // of it lands in the gaps between the operations, i.e. in the hand-off figure.  Passes that are timed
    // in one piece (first copy enqueued -> last kernel done) show what a pass costs without those events; the
    // difference, spread over the layers, is taken off the hand-offs.
    // Copies are also faster when the next one is already queued as one ends (pipelined runs that are bound by
    // the copies keep the copy queue full) than each one is with an idle queue on both sides: a train of all
    // layers' copies into the slots, timed in one piece, gives the ratio.
    if (rc == DL_OK) {
        constexpr int32_t kReps = 3;
        double whole[kReps] = {0, 0, 0}, train[kReps] = {0, 0, 0};
        c->timing = false;
        for (int32_t rep = 0; rep < kReps && rc == DL_OK; ++rep) {
            hipEvent_t e0 = nullptr, e1 = nullptr;
            rc = timing_event(c, &e0);
            if (rc == DL_OK) rc = timing_event(c, &e1);
            if (rc) break;
            c->book = dl::SlotBook();
            c->book.n_slots = c->n_slots;
            if (hipEventRecord(e0, c->s_copy) != hipSuccess) { rc = fail(c, DL_ERR_DEVICE, "event record failed"); break; }
            rc = run_pass(c, module, static_cast<const float*>(x), scratch, T, pos0, static_cast<const float*>(ctx), n_ctx, true);
            if (rc) break;
            float ms = 0.0f;
            if (hipEventRecord(e1, c->s_compute) != hipSuccess || hipStreamSynchronize(c->s_compute) != hipSuccess ||
                hipStreamSynchronize(c->s_copy) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
                rc = fail(c, DL_ERR_DEVICE, "timing the sequential pass in one piece failed");
                break;
            }
            whole[rep] = double(ms);
        }
        for (int32_t rep = 0; rep < kReps && rc == DL_OK; ++rep) {
            hipEvent_t e0 = nullptr, e1 = nullptr;
            rc = timing_event(c, &e0);
            if (rc == DL_OK) rc = timing_event(c, &e1);
            if (rc) break;
            // every copy sits between a wait on a (long completed) event of the compute stream and a record, as the
            // copies of a pass do: the packets these put into the copy queue are part of what a copy in a train costs
            hipEvent_t released = nullptr, copied = nullptr;
            rc = timing_event(c, &released);
            if (rc == DL_OK) rc = timing_event(c, &copied);
            if (rc) break;
            bool ok = hipEventRecord(released, c->s_compute) == hipSuccess && hipStreamSynchronize(c->s_compute) == hipSuccess &&
                      hipEventRecord(e0, c->s_copy) == hipSuccess;
            for (int32_t i = 0; i < Ln && ok; ++i)
                ok = hipStreamWaitEvent(c->s_copy, released, 0) == hipSuccess &&
                     hipMemcpyAsync(c->base + c->slot_off[i % c->slots_held], M->store + size_t(i) * M->L.bytes, M->L.bytes,
                                    hipMemcpyHostToDevice, c->s_copy) == hipSuccess &&
                     hipEventRecord(copied, c->s_copy) == hipSuccess;
            float ms = 0.0f;
            ok = ok && hipEventRecord(e1, c->s_copy) == hipSuccess && hipStreamSynchronize(c->s_copy) == hipSuccess &&
                 hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            if (!ok) { rc = fail(c, DL_ERR_DEVICE, "timing the train of copies failed"); break; }
            train[rep] = double(ms);
        }
        c->timing = true;
        if (rc == DL_OK) {
            std::sort(whole, whole + kReps);
            std::sort(train, train + kReps);
            double dma_sum = 0.0;
            for (int32_t i = 0; i < Ln; ++i) dma_sum += dma[size_t(i)];
            dma_sum /= double(iters - 1);
            fence_excess = std::max(0.0, timed_span / double(iters - 1) - whole[kReps / 2]) / double(Ln);
            if (dma_sum > 0.0 && train[kReps / 2] > 0.0) cont_scale = std::min(1.0, train[kReps / 2] / dma_sum);
        }
    }
    // all layers back to back, no copies: execution time under continuous load.  The last of kHotReps runs counts:
    // the chip is power-limited, and the first passes after an idle spell still run at a higher clock than a
    // sustained sequence of passes does.
    // Resident layers read weights that have long left the caches and whose pages have left the TLBs (a whole stack is
    // far larger than the 256 MB memory-side cache), so the run must not keep re-reading one slot: the layers rotate
    // through the two slots plus temporary copies, one buffer per layer if the arena can spare that much (re-reading
    // three 386 MB buffers made single-token passes look 7 % faster than passes over 36 resident layers are).
    std::vector<uint64_t> rot(c->slot_off, c->slot_off + c->slots_held);
    std::vector<uint64_t> rot_tmp;
    {
        for (uint64_t j = 0; int64_t(j) + 2 < Ln; ++j) {
            uint64_t off = 0;
            if (!c->arena.alloc(M->L.bytes, &off)) break;
            if (hipMemcpyAsync(c->base + off, M->store + size_t(j % uint64_t(Ln)) * M->L.bytes, M->L.bytes,
                               hipMemcpyHostToDevice, c->s_compute) != hipSuccess) {
                c->arena.free(off);
                rc = fail(c, DL_ERR_DEVICE, "copy of a temporary weight block failed");
                break;
            }
            rot_tmp.push_back(off);
            rot.push_back(off);
        }
    }
    constexpr int32_t kHotReps = 4;
    for (int32_t rep = 0; rep < kHotReps && rc == DL_OK; ++rep) {
        for (int32_t i = 0; i < Ln && rc == DL_OK; ++i) {
            TimedOp t{nullptr, nullptr, module, i, -1, -1};
            rc = timing_event(c, &t.e0);
            if (rc == DL_OK) rc = timing_event(c, &t.e1);
            if (rc) break;
            if (hipEventRecord(t.e0, c->s_compute) != hipSuccess) { rc = fail(c, DL_ERR_DEVICE, "event record failed"); break; }
            run_layer(c, *M, i, c->base + rot[size_t(i) % rot.size()], i == 0 ? static_cast<const float*>(x) : scratch, scratch, T, pos0,
                      static_cast<const float*>(ctx), n_ctx);
            if (hipEventRecord(t.e1, c->s_compute) != hipSuccess) { rc = fail(c, DL_ERR_DEVICE, "event record failed"); break; }
            c->execs.push_back(t);
        }
        if (rc) break;
        dl_run_stats st;
        std::vector<dl_layer_record> recs;
        recs.resize(size_t(Ln));
        rc = dl_collect_stats(c, &st, recs.data(), Ln);
        if (rc == DL_OK && rep == kHotReps - 1) {
            // start-to-start spacing, so that launch gaps between layers are part of the figure
            double gap = 0;
            for (int32_t i = 0; i + 1 < Ln; ++i) {
                hot[size_t(i)] = double(recs[size_t(i + 1)].exe_start_ms) - recs[size_t(i)].exe_start_ms;
                gap += double(recs[size_t(i + 1)].exe_start_ms) - recs[size_t(i)].exe_end_ms;
            }
            hot[size_t(Ln - 1)] = double(recs[size_t(Ln - 1)].exe_end_ms) - recs[size_t(Ln - 1)].exe_start_ms +
                                  (Ln > 1 ? gap / (Ln - 1) : 0.0);
        }
    }
    // The event pairs between the layers drain the queue (a few microseconds per layer, which is percents for short
    // layers): runs with events only around the whole stack give the true total, and the per-layer figures are scaled
    // to it.  Three variants of that run, each taken in turn with a plain one (three rounds,
    // medians) because the part's clock under sustained load drifts by a percent or two over the tens of passes of a
    // profile, which is as much as the two effects the variants are there to measure:
    //  * plain: all layers back to back;
    //  * with what a streamed layer puts on the compute stream when its copy is done before the layer's turn: in
    //    front of the layer a wait on an event that the copy stream records behind a (tiny) copy of its own - a fresh
    //    event per layer, so that the wait is a real one with its acquire of what the copy wrote, not one the runtime
    //    can drop because the event is known to be complete - and behind the layer an event record that the copy
    //    stream waits for (a record nobody waits for costs a third: 7 against 24 us per 27-layer-encoder layer).  The
    //    difference to the plain run, per layer, is the hand-off cost of a streamed layer in a pass that is bound by
    //    execution;
    //  * next to a train of copies that lasts at least as long as the run: host-to-device copies write to HBM
    //    through the same fabric the kernels read through, and a pass that streams some layers while it is bound by
    //    execution runs its kernels a few percent slower than this profile's copy-free runs.  The layers read the
    //    temporary weight copies only (the train overwrites the slots); without any they share the slots, which
    //    changes values, not times.
    if (rc == DL_OK) {
        constexpr int32_t kRounds = 3;
        double plain[kRounds] = {0, 0, 0}, with_ops[kRounds] = {0, 0, 0}, loaded[kRounds] = {0, 0, 0};
        std::vector<hipEvent_t> fresh(size_t(Ln), nullptr);
        std::vector<hipEvent_t> released(size_t(Ln), nullptr);
        for (int32_t i = 0; i < Ln && rc == DL_OK; ++i) rc = timing_event(c, &fresh[size_t(i)]);
        for (int32_t i = 0; i < Ln && rc == DL_OK; ++i) rc = timing_event(c, &released[size_t(i)]);
        double dma_mean = 0.0, hot_sum = 0.0;
        for (int32_t i = 0; i < Ln; ++i) { dma_mean += dma[size_t(i)]; hot_sum += hot[size_t(i)]; }
        dma_mean = dma_mean / double(iters - 1) / double(Ln) * cont_scale;
        const int32_t n_train = dma_mean > 0.0 ? int32_t(std::min(4096.0, std::ceil(1.15 * hot_sum / dma_mean) + 1.0)) : 0;
        std::vector<uint64_t> rot2(rot_tmp.begin(), rot_tmp.end());
        if (rot2.empty()) rot2 = rot;
        // variant 0 plain, 1 with the event protocol, 2 next to the train of copies
        auto whole_run = [&](int32_t variant, double* ms_out) -> int32_t {
            hipEvent_t e0 = nullptr, e1 = nullptr;
            int32_t r = timing_event(c, &e0);
            if (r == DL_OK) r = timing_event(c, &e1);
            if (r) return r;
            bool ok = true;
            if (variant == 2)
                for (int32_t i = 0; i < n_train && ok; ++i)
                    ok = hipMemcpyAsync(c->base + c->slot_off[i % c->slots_held], M->store + size_t(i % Ln) * M->L.bytes,
                                        M->L.bytes, hipMemcpyHostToDevice, c->s_copy) == hipSuccess;
            const std::vector<uint64_t>& from = variant == 2 ? rot2 : rot;
            ok = ok && hipEventRecord(e0, c->s_compute) == hipSuccess;
            for (int32_t i = 0; i < Ln && ok; ++i) {
                if (variant == 1)
                    ok = hipMemcpyAsync(c->base + c->slot_off[0], M->store + size_t(i) * M->L.bytes, 256, hipMemcpyHostToDevice,
                                        c->s_copy) == hipSuccess &&
                         hipEventRecord(fresh[size_t(i)], c->s_copy) == hipSuccess &&
                         hipStreamWaitEvent(c->s_compute, fresh[size_t(i)], 0) == hipSuccess;
                run_layer(c, *M, i, c->base + from[size_t(i) % from.size()], i == 0 ? static_cast<const float*>(x) : scratch,
                          scratch, T, pos0, static_cast<const float*>(ctx), n_ctx);
                if (variant == 1)
                    ok = ok && hipEventRecord(released[size_t(i)], c->s_compute) == hipSuccess &&
                         hipStreamWaitEvent(c->s_copy, released[size_t(i)], 0) == hipSuccess;
            }
            float total = 0.0f;
            ok = ok && hipEventRecord(e1, c->s_compute) == hipSuccess;
            if (hipStreamSynchronize(c->s_compute) != hipSuccess || hipStreamSynchronize(c->s_copy) != hipSuccess || !ok ||
                hipEventElapsedTime(&total, e0, e1) != hipSuccess)
                return fail(c, DL_ERR_DEVICE, "timing an uninterrupted run failed");
            *ms_out = double(total);
            return DL_OK;
        };
        // the runs next to copies come last and have plain runs of their own to be compared with: the copy engines add
        // to the board's power, and the plain run right behind such a run is 2-4 % slower than one in a copy-free
        // sequence (which is what a pass over resident layers is)
        double plain_b[kRounds] = {0, 0, 0};
        for (int32_t round = 0; round < kRounds && rc == DL_OK; ++round) {
            rc = whole_run(0, &plain[round]);
            if (rc == DL_OK) rc = whole_run(1, &with_ops[round]);
        }
        for (int32_t round = 0; round < kRounds && rc == DL_OK && n_train > 0; ++round) {
            rc = whole_run(0, &plain_b[round]);
            if (rc == DL_OK) rc = whole_run(2, &loaded[round]);
        }
        if (rc == DL_OK) {
            std::sort(plain, plain + kRounds);
            std::sort(with_ops, with_ops + kRounds);
            std::sort(plain_b, plain_b + kRounds);
            std::sort(loaded, loaded + kRounds);
            hot_total = plain[kRounds / 2];
            if (hot_sum > 0.0 && hot_total > 0.0)
                for (int32_t i = 0; i < Ln; ++i) hot[size_t(i)] *= hot_total / hot_sum;
            if (hot_total > 0.0) fence_hot = std::max(0.0, with_ops[kRounds / 2] - hot_total) / double(Ln);
            if (n_train > 0 && plain_b[kRounds / 2] > 0.0) load_scale = std::max(1.0, loaded[kRounds / 2] / plain_b[kRounds / 2]);
        }
    }
    // The continuous runs executed every layer on rotated parameters and appended THOSE keys and values at pos0..:
    // one more sequential pass with every layer's own parameters leaves the cache rows as a real pass over this
    // input writes them.
    if (rc == DL_OK && M->d.max_seq > 0) {
        c->timing = false;
        c->book = dl::SlotBook();
        c->book.n_slots = c->n_slots;
        rc = run_pass(c, module, static_cast<const float*>(x), scratch, T, pos0, static_cast<const float*>(ctx), n_ctx, true);
    }
    c->mode = mode0;
    c->wrap = wrap0;
    c->timing = timing0;
    c->tracing = tracing0;
    c->book = dl::SlotBook();
    c->book.n_slots = c->n_slots;
    sync_streams(c);
    for (uint64_t off : rot_tmp) c->arena.free(off);
    c->copies.clear();
    c->execs.clear();
    if (c->krecs.empty()) c->ev_next = 0;
    c->arena.free(tmp_off);
    c->arena.restore_peak(peak_before);
    if (rc) return rc;
    for (int32_t i = 0; i < Ln; ++i) {
        out[i].c_dma_ms = dma[size_t(i)] / (iters - 1);
        out[i].c_dma_cont_ms = out[i].c_dma_ms * cont_scale;
        out[i].c_exe_ms = exe[size_t(i)] / (iters - 1);
        out[i].c_exe_hot_ms = hot[size_t(i)];
        out[i].c_exe_loaded_ms = hot[size_t(i)] * load_scale;
        out[i].c_fence_ms = std::max(0.0, fence[size_t(i)] / (iters - 1) - fence_excess);
        out[i].c_fence_hot_ms = fence_hot;
        out[i].bytes = M->L.bytes;
    }
    return DL_OK;
}

int32_t dl_set_run_ahead(dl_ctx* c, int32_t passes) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (passes < 0 || passes > dl_ctx::kMaxRunAhead) return fail(c, DL_ERR_INVALID_ARG, "run-ahead outside [0, 8]");
    c->run_ahead = passes;
    return DL_OK;
}

int32_t dl_set_slot_count(dl_ctx* c, int32_t n_slots) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (n_slots < 1 || n_slots > dl::kMaxSlots) return fail(c, DL_ERR_INVALID_ARG, "slot count must be 1 .. 4");
    if (n_slots == c->n_slots) return DL_OK;
    rc = sync_streams(c);
    if (rc) return rc;
    Proposal p = current_proposal(c);
    p.n_slots = n_slots;
    return relayout(c, p);
}

int32_t dl_module_set_max_tokens(dl_ctx* c, int32_t module, int32_t max_tokens) {
    int32_t rc = enter(c);
    if (rc) return rc;
    Module* M = get_module(c, module);
    if (!M || !M->finalized) return fail(c, DL_ERR_BAD_STATE, "module missing or not finalized");
    if (max_tokens < 1) return fail(c, DL_ERR_INVALID_ARG, "max_tokens < 1");
    if (M->d.max_seq > 0 && max_tokens > M->d.max_seq) return fail(c, DL_ERR_INVALID_ARG, "max_tokens exceeds max_seq");
    if (max_tokens == M->d.max_tokens) return DL_OK;
    rc = sync_streams(c);
    if (rc) return rc;
    dl_module_desc d2 = M->d;
    d2.max_tokens = max_tokens;
    const dl::WorkspaceLayout W2 = dl::make_workspace(d2);
    Proposal p = current_proposal(c);
    p.ws_bytes[size_t(module)] = W2.bytes;
    rc = relayout(c, p);
    if (rc) return rc;
    M = get_module(c, module);
    M->W = W2;
    M->d = d2;
    return DL_OK;
}

int32_t dl_probe_mfma_rate(dl_ctx* c, int32_t pattern, int32_t iters, double* tflops_out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!tflops_out || iters < 1 || iters > (1 << 20) || pattern < 0 || pattern > 1) return fail(c, DL_ERR_INVALID_ARG, "bad probe arguments");
    if (!on_gpu(c)) return fail(c, DL_ERR_BAD_STATE, "the MFMA probe needs a device context");
    if (!c->arena.is_set()) return fail(c, DL_ERR_BAD_STATE, "arena not set");
    hipDeviceProp_t prop;
    DL_HIP(c, hipGetDeviceProperties(&prop, c->device));
    const int blocks = prop.multiProcessorCount;
    uint64_t off = 0;
    if (!c->arena.alloc(uint64_t(blocks) * 1024, &off)) return fail(c, DL_ERR_BUDGET_EXCEEDED, "arena cannot hold the probe's output");
    float* out = reinterpret_cast<float*>(c->base + off);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t he = hipEventCreate(&e0);
    if (he == hipSuccess) he = hipEventCreate(&e1);
    double flop = 0.0;
    float ms = 0.0f;
    if (he == hipSuccess) {
        dlk::mfma_rate_probe(out, blocks, iters, pattern, c->s_compute);          // warm-up launch
        (void)hipEventRecord(e0, c->s_compute);
        flop = dlk::mfma_rate_probe(out, blocks, iters, pattern, c->s_compute);
        (void)hipEventRecord(e1, c->s_compute);
        he = hipStreamSynchronize(c->s_compute);
        if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    c->arena.free(off);
    DL_HIP(c, he);
    *tflops_out = ms > 0.0f ? flop / (double(ms) * 1e-3) / 1e12 : 0.0;
    return DL_OK;
}

int32_t dl_set_kernel_timing(dl_ctx* c, int32_t on) {
    int32_t rc = enter(c);
    if (rc) return rc;
    c->ktiming = uint32_t(on);
    return DL_OK;
}

int32_t dl_collect_kernel_times(dl_ctx* c, dl_kernel_time* out) {
    int32_t rc = enter(c);
    if (rc) return rc;
    if (!out) return fail(c, DL_ERR_INVALID_ARG, "null output");
    for (int32_t k = 0; k < DL_K_COUNT; ++k) out[k] = dl_kernel_time{k, 0, 0.0, 0.0, 0.0};
    if (!on_gpu(c)) return DL_OK;
    rc = sync_streams(c);
    if (rc) return rc;
    for (const dl_ctx::KRec& r : c->krecs) {
        float ms = 0;
        DL_HIP(c, hipEventElapsedTime(&ms, r.e0, r.e1));
        dl_kernel_time& o = out[r.kind];
        o.launches += 1;
        o.total_ms += ms;
        o.flops += r.flops;
        o.bytes += r.bytes;
    }
    c->krecs.clear();
    if (c->copies.empty() && c->execs.empty()) c->ev_next = 0;
    return DL_OK;
}

int32_t dl_trace_enable(dl_ctx* c, int32_t on) {
    if (!c) return DL_ERR_INVALID_ARG;
    c->tracing = on != 0;
    return DL_OK;
}

int32_t dl_trace_read(dl_ctx* c, dl_trace_op* out, int32_t cap, int32_t* n_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !out)) return DL_ERR_INVALID_ARG;
    const int32_t n = int32_t(c->trace.size());
    for (int32_t i = 0; i < n && i < cap; ++i) out[i] = c->trace[size_t(i)];
    *n_out = n;
    c->trace.clear();
    return DL_OK;
}

}  // extern "C"
