// Host core: arena accounting, packed-blob layout, the per-pass schedule (slot protocol),
// and the planner / predictor.  No HIP call in this file: everything here also runs in a
// host-only context.
#include "dl_internal.hpp"

#include <algorithm>
#include <utility>
#include <cmath>
#include <cstring>

namespace dl {

// ------------------------------------------------------------------------------------------
// Arena
// ------------------------------------------------------------------------------------------
void Arena::reset(uint64_t capacity) {
    blocks_.clear();
    cap_ = capacity / kAlign * kAlign;
    used_ = peak_ = 0;
    if (cap_) blocks_.push_back({0, cap_, false});
}

bool Arena::alloc(uint64_t bytes, uint64_t* off_out) {
    uint64_t need = align_up(bytes ? bytes : 1);
    for (size_t i = 0; i < blocks_.size(); ++i) {
        Block& b = blocks_[i];
        if (b.used || b.size < need) continue;
        if (b.size > need) {
            Block rest{b.off + need, b.size - need, false};
            b.size = need;
            b.used = true;
            *off_out = b.off;
            blocks_.insert(blocks_.begin() + i + 1, rest);
        } else {
            b.used = true;
            *off_out = b.off;
        }
        used_ += need;
        peak_ = std::max(peak_, used_);
        return true;
    }
    return false;
}

bool Arena::alloc_top(uint64_t bytes, uint64_t* off_out) {
    const uint64_t need = align_up(bytes ? bytes : 1);
    for (size_t i = blocks_.size(); i-- > 0;) {
        Block& b = blocks_[i];
        if (b.used || b.size < need) continue;
        if (b.size > need) {
            const Block top{b.off + b.size - need, need, true};
            b.size -= need;
            *off_out = top.off;
            blocks_.insert(blocks_.begin() + i + 1, top);
        } else {
            b.used = true;
            *off_out = b.off;
        }
        used_ += need;
        peak_ = std::max(peak_, used_);
        return true;
    }
    return false;
}

bool Arena::free(uint64_t off) {
    for (size_t i = 0; i < blocks_.size(); ++i) {
        if (blocks_[i].off != off || !blocks_[i].used) continue;
        blocks_[i].used = false;
        used_ -= blocks_[i].size;
        if (i + 1 < blocks_.size() && !blocks_[i + 1].used) {
            blocks_[i].size += blocks_[i + 1].size;
            blocks_.erase(blocks_.begin() + i + 1);
        }
        if (i > 0 && !blocks_[i - 1].used) {
            blocks_[i - 1].size += blocks_[i].size;
            blocks_.erase(blocks_.begin() + i);
        }
        return true;
    }
    return false;
}

uint64_t Arena::size_of(uint64_t off) const {
    for (const Block& b : blocks_)
        if (b.off == off && b.used) return b.size;
    return 0;
}

// ------------------------------------------------------------------------------------------
// Descriptor checks and the packed layout
// ------------------------------------------------------------------------------------------
bool validate_desc(const dl_module_desc& d, std::string* why) {
    auto bad = [&](const char* m) { *why = m; return false; };
    if (d.n_layers < 1 || d.n_layers > 4096) return bad("n_layers out of range");
    if (d.d_model < 8 || d.d_model % 8) return bad("d_model must be a positive multiple of 8");
    if (d.n_q_heads < 1 || d.n_kv_heads < 1 || d.n_q_heads % d.n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
    if (d.d_head < 8 || d.d_head % 8 || d.d_head > 128) return bad("d_head must be a multiple of 8 in [8, 128]");
    if (d.norm != DL_NORM_RMS && d.norm != DL_NORM_LN) return bad("unknown norm");
    if (d.act != DL_ACT_SWIGLU && d.act != DL_ACT_GELU) return bad("unknown activation");
    if (d.d_ff < 8 || d.d_ff % 8) return bad("d_ff must be a positive multiple of 8");
    if (d.act == DL_ACT_SWIGLU && d.d_ff % 32) return bad("d_ff must be a multiple of 32 for SwiGLU");
    if (d.rope_theta < 0 || (d.rope_theta > 0 && d.d_head % 2)) return bad("bad rope_theta");
    if (d.d_ctx < 0 || d.d_ctx % 8) return bad("d_ctx must be a multiple of 8");
    if (d.d_ctx > 0 && d.max_ctx < 1) return bad("max_ctx must be positive when d_ctx > 0");
    if (d.max_seq < 0 || d.max_tokens < 1) return bad("max_seq >= 0 and max_tokens >= 1 required");
    if (d.max_seq > 0 && !d.causal) return bad("a KV cache needs a causal module");
    if (d.max_seq > 0 && d.max_tokens > d.max_seq) return bad("max_tokens exceeds max_seq");
    // the single-token attention kernel maps the query heads of one KV head onto the 32 columns of one MFMA tile
    if (d.max_seq > 0 && d.n_q_heads / d.n_kv_heads > 32)
        return bad("with a KV cache at most 32 query heads may share one KV head");
    // the kernels address an operand (an activation matrix, the keys or values of one head) with 32-bit byte offsets
    {
        const uint64_t positions = uint64_t(std::max(std::max(d.max_seq, d.max_tokens), d.max_ctx));
        const uint64_t widest = std::max(uint64_t(d.n_q_heads + 2 * d.n_kv_heads) * uint64_t(d.d_head),
                                         std::max(uint64_t(d.d_ff) * (d.act == DL_ACT_SWIGLU ? 2u : 1u), uint64_t(std::max(d.d_model, d.d_ctx))));
        if (positions * widest * 4 >= (1ull << 32)) return bad("max_seq / max_tokens / max_ctx times the widest row exceeds 4 GB");
    }
    if (d.vocab < 0) return bad("vocab < 0");
    if (!(d.norm_eps >= 0)) return bad("norm_eps < 0");
    return true;
}

PackLayout make_layout(const dl_module_desc& d) {
    PackLayout L;
    const uint64_t dm = d.d_model, dq = uint64_t(d.n_q_heads) * d.d_head, dkv = uint64_t(d.n_kv_heads) * d.d_head;
    const uint64_t f = d.d_ff;
    const bool ln = d.norm == DL_NORM_LN, b = d.has_bias != 0, cross = d.d_ctx > 0, glu = d.act == DL_ACT_SWIGLU;
    uint64_t off = 0, params = 0;
    auto put = [&](uint64_t* field, uint64_t elems) {
        *field = off;
        off = align_up(off + 2 * elems);
        params += elems;
    };
    L.n_qkv = int32_t(dq + 2 * dkv);
    L.n_up = int32_t(glu ? 2 * f : f);
    L.ffp = int32_t(align_up(f, 128));
    put(&L.norm1_g, dm);
    if (ln) put(&L.norm1_b, dm);
    put(&L.w_qkv, (dq + 2 * dkv) * dm);
    if (b) put(&L.b_qkv, dq + 2 * dkv);
    put(&L.w_o, dm * dq);
    if (b) put(&L.b_o, dm);
    if (cross) {
        put(&L.normc_g, dm);
        if (ln) put(&L.normc_b, dm);
        put(&L.w_qc, dq * dm);
        if (b) put(&L.b_qc, dq);
        put(&L.w_kvc, 2 * dkv * uint64_t(d.d_ctx));
        if (b) put(&L.b_kvc, 2 * dkv);
        put(&L.w_oc, dm * dq);
        if (b) put(&L.b_oc, dm);
    }
    put(&L.norm2_g, dm);
    if (ln) put(&L.norm2_b, dm);
    put(&L.w_up, uint64_t(L.n_up) * dm);
    if (b) put(&L.b_up, f);
    put(&L.w_down, dm * uint64_t(L.ffp));
    params -= dm * (uint64_t(L.ffp) - f);      // the zero padding is not a parameter
    if (b) put(&L.b_down, dm);
    L.bytes = off;
    L.param_bytes = 2 * params;
    return L;
}

uint64_t tensor_elems(const dl_module_desc& d, int32_t tid) {
    const uint64_t dm = d.d_model, dq = uint64_t(d.n_q_heads) * d.d_head, dkv = uint64_t(d.n_kv_heads) * d.d_head;
    const uint64_t f = d.d_ff, dc = d.d_ctx;
    const bool ln = d.norm == DL_NORM_LN, b = d.has_bias != 0, cross = d.d_ctx > 0, glu = d.act == DL_ACT_SWIGLU;
    switch (tid) {
        case DL_T_NORM1_G: case DL_T_NORM2_G: return dm;
        case DL_T_NORM1_B: case DL_T_NORM2_B: return ln ? dm : 0;
        case DL_T_WQ: return dq * dm;
        case DL_T_WK: case DL_T_WV: return dkv * dm;
        case DL_T_BQ: return b ? dq : 0;
        case DL_T_BK: case DL_T_BV: return b ? dkv : 0;
        case DL_T_WO: return dm * dq;
        case DL_T_BO: return b ? dm : 0;
        case DL_T_W_GATE: return glu ? f * dm : 0;
        case DL_T_W_UP: return f * dm;
        case DL_T_B_UP: return b ? f : 0;
        case DL_T_W_DOWN: return dm * f;
        case DL_T_B_DOWN: return b ? dm : 0;
        case DL_T_NORMC_G: return cross ? dm : 0;
        case DL_T_NORMC_B: return cross && ln ? dm : 0;
        case DL_T_WQ_C: return cross ? dq * dm : 0;
        case DL_T_WK_C: case DL_T_WV_C: return cross ? dkv * dc : 0;
        case DL_T_BQ_C: return cross && b ? dq : 0;
        case DL_T_BK_C: case DL_T_BV_C: return cross && b ? dkv : 0;
        case DL_T_WO_C: return cross ? dm * dq : 0;
        case DL_T_BO_C: return cross && b ? dm : 0;
        default: return 0;
    }
}

uint32_t required_tensor_mask(const dl_module_desc& d) {
    uint32_t m = 0;
    for (int32_t t = 0; t < DL_T_COUNT; ++t)
        if (tensor_elems(d, t)) m |= 1u << t;
    return m;
}

void pack_tensor(const dl_module_desc& d, const PackLayout& L, int32_t tid, const uint16_t* src, uint8_t* blob) {
    const uint64_t dm = d.d_model, dq = uint64_t(d.n_q_heads) * d.d_head, dkv = uint64_t(d.n_kv_heads) * d.d_head;
    const uint64_t f = d.d_ff, dc = d.d_ctx;
    const uint64_t n = tensor_elems(d, tid);
    auto plain = [&](uint64_t off, uint64_t elem_off) { std::memcpy(blob + off + 2 * elem_off, src, 2 * n); };
    switch (tid) {
        case DL_T_NORM1_G: plain(L.norm1_g, 0); break;
        case DL_T_NORM1_B: plain(L.norm1_b, 0); break;
        case DL_T_NORM2_G: plain(L.norm2_g, 0); break;
        case DL_T_NORM2_B: plain(L.norm2_b, 0); break;
        case DL_T_NORMC_G: plain(L.normc_g, 0); break;
        case DL_T_NORMC_B: plain(L.normc_b, 0); break;
        // fused QKV: rows [0,dq) = Q, [dq,dq+dkv) = K, [dq+dkv, dq+2dkv) = V
        case DL_T_WQ: plain(L.w_qkv, 0); break;
        case DL_T_WK: plain(L.w_qkv, dq * dm); break;
        case DL_T_WV: plain(L.w_qkv, (dq + dkv) * dm); break;
        case DL_T_BQ: plain(L.b_qkv, 0); break;
        case DL_T_BK: plain(L.b_qkv, dq); break;
        case DL_T_BV: plain(L.b_qkv, dq + dkv); break;
        case DL_T_WO: plain(L.w_o, 0); break;
        case DL_T_BO: plain(L.b_o, 0); break;
        case DL_T_WQ_C: plain(L.w_qc, 0); break;
        case DL_T_BQ_C: plain(L.b_qc, 0); break;
        case DL_T_WK_C: plain(L.w_kvc, 0); break;
        case DL_T_WV_C: plain(L.w_kvc, dkv * dc); break;
        case DL_T_BK_C: plain(L.b_kvc, 0); break;
        case DL_T_BV_C: plain(L.b_kvc, dkv); break;
        case DL_T_WO_C: plain(L.w_oc, 0); break;
        case DL_T_BO_C: plain(L.b_oc, 0); break;
        case DL_T_B_UP: plain(L.b_up, 0); break;
        case DL_T_W_DOWN:
            // rows padded to ffp elements; the padding stays zero (the store is zero-initialised)
            for (uint64_t r = 0; r < dm; ++r) std::memcpy(blob + L.w_down + 2 * r * uint64_t(L.ffp), src + r * f, 2 * f);
            break;
        case DL_T_B_DOWN: plain(L.b_down, 0); break;
        case DL_T_W_GATE:
        case DL_T_W_UP:
            if (d.act == DL_ACT_SWIGLU) {
                // gate and up rows interleaved in groups of 32: packed row (f/32)*64 + f%32 is gate row f,
                // 32 rows further is up row f; the GEMM epilogue then finds both in one wave
                const uint64_t shift = (tid == DL_T_W_UP) ? 32 : 0;
                for (uint64_t r = 0; r < f; ++r) {
                    uint64_t pr = (r / 32) * 64 + (r % 32) + shift;
                    std::memcpy(blob + L.w_up + 2 * pr * dm, src + r * dm, 2 * dm);
                }
            } else {
                plain(L.w_up, 0);
            }
            break;
        default: break;
    }
}

WorkspaceLayout make_workspace(const dl_module_desc& d) {
    WorkspaceLayout W;
    const uint64_t T = d.max_tokens, dm = d.d_model, dq = uint64_t(d.n_q_heads) * d.d_head,
                   dkv = uint64_t(d.n_kv_heads) * d.d_head, f = d.d_ff;
    uint64_t off = 0;
    auto put = [&](uint64_t* field, uint64_t bytes) { *field = off; off = align_up(off + bytes); };
    put(&W.nbuf, 2 * T * dm);
    put(&W.qkv, 2 * T * (dq + 2 * dkv));
    put(&W.attn, 2 * T * dq);
    put(&W.mid, 2 * T * align_up(f, 128));
    if (d.max_seq == 0) {
        W.vt_ld = int32_t(align_up(T, 64));
        put(&W.vt, 2 * dkv * uint64_t(W.vt_ld));
    } else {
        // partial results of the split single-token attention: [Hq][tiles of 64 positions][d_head + 2] floats
        put(&W.dec_part, uint64_t(d.n_q_heads) * ((uint64_t(d.max_seq) + 63) / 64) * uint64_t(d.d_head + 2) * 4);
    }
    if (d.d_ctx > 0) {
        const uint64_t C = d.max_ctx;
        W.vtc_ld = int32_t(align_up(C, 64));
        put(&W.ctxn, 2 * C * uint64_t(d.d_ctx));
        put(&W.kvc, 2 * C * 2 * dkv);
        put(&W.vtc, 2 * dkv * uint64_t(W.vtc_ld));
        // few queries attending to a long context: partial results of the key-range split, 16 runs x heads x
        // queries x (padded head dim + 4) floats (the attention launcher's layout)
        if (T <= 128) {
            const uint64_t dhp = d.d_head <= 64 ? 64 : (d.d_head <= 96 ? 96 : 128);
            W.att_part_bytes = 16ull * uint64_t(d.n_q_heads) * T * (dhp + 4) * 4;
            put(&W.att_part, W.att_part_bytes);
        }
    }
    if (d.vocab > 0) {
        put(&W.logits, 4 * uint64_t(d.vocab));
        put(&W.token, 256);
    }
    W.bytes = off;
    return W;
}

KvLayout make_kv(const dl_module_desc& d) {
    KvLayout K;
    if (d.max_seq <= 0) return K;
    const uint64_t dkv = uint64_t(d.n_kv_heads) * d.d_head;
    K.v_ld = int32_t(align_up(uint64_t(d.max_seq), 64));
    K.k_layer_bytes = align_up(2 * dkv * uint64_t(d.max_seq));
    K.v_layer_bytes = align_up(2 * dkv * uint64_t(K.v_ld));
    K.bytes = uint64_t(d.n_layers) * (K.k_layer_bytes + K.v_layer_bytes);
    return K;
}

// ------------------------------------------------------------------------------------------
// One pass as a list of queue operations (Sec. IV-C(ii): slots, DMA-done / compute-done events)
// ------------------------------------------------------------------------------------------
namespace {
constexpr int32_t QC = 0, QD = 1;   // compute queue, copy (DMA) queue
dl_trace_op mk(int32_t q, int32_t op, int32_t ev, int32_t slot, int32_t module, int32_t layer) {
    return dl_trace_op{q, op, ev, slot, module, layer, 0};
}
}  // namespace

void build_pass(int32_t module, int32_t n_layers, const uint8_t* resident, int32_t mode, int32_t wrap_prefetch,
                bool force_stream_all, SlotBook* book, std::vector<dl_trace_op>* ops) {
    std::vector<int32_t> streamed;
    for (int32_t i = 0; i < n_layers; ++i)
        if (force_stream_all || !resident[i]) streamed.push_back(i);
    std::vector<int32_t> slot_of(n_layers, -1);

    auto drop_pending = [&]() { book->n_pending = 0; book->pending_module = -1; };

    if (mode == DL_MODE_SEQUENTIAL) {
        // Sec. IV-B: the copy of a layer starts only when the previous layer has finished
        drop_pending();
        size_t si = 0;
        for (int32_t i = 0; i < n_layers; ++i) {
            const bool st = si < streamed.size() && streamed[si] == i;
            int32_t s = -1;
            if (st) {
                ++si;
                s = int32_t(book->ordinal++ % uint64_t(book->n_slots));
                if (book->pass_recorded) ops->push_back(mk(QD, DL_OP_WAIT, DL_EV_PASS_DONE, -1, module, i));
                ops->push_back(mk(QD, DL_OP_COPY, -1, s, module, i));
                ops->push_back(mk(QD, DL_OP_RECORD, DL_EV_DMA_DONE, s, module, i));
                book->dma_recorded[s] = true;
                ops->push_back(mk(QC, DL_OP_WAIT, DL_EV_DMA_DONE, s, module, i));
            }
            ops->push_back(mk(QC, DL_OP_EXEC, -1, s, module, i));
            if (st) {
                ops->push_back(mk(QC, DL_OP_RECORD, DL_EV_COMPUTE_DONE, s, module, i));
                book->compute_recorded[s] = true;
            }
            ops->push_back(mk(QC, DL_OP_RECORD, DL_EV_PASS_DONE, -1, module, i));
            book->pass_recorded = true;
        }
        return;
    }

    auto issue_copy = [&](int32_t layer, bool gate_on_pass, int32_t passes_ahead) -> int32_t {
        const int32_t s = int32_t(book->ordinal++ % uint64_t(book->n_slots));
        if (gate_on_pass && book->pass_recorded) ops->push_back(mk(QD, DL_OP_WAIT, DL_EV_PASS_DONE, -1, module, layer));
        // the slot may be overwritten only after the layer that last used it has executed
        if (book->compute_recorded[s]) ops->push_back(mk(QD, DL_OP_WAIT, DL_EV_COMPUTE_DONE, s, module, layer));
        dl_trace_op cp = mk(QD, DL_OP_COPY, -1, s, module, layer);
        cp.flags = passes_ahead;
        ops->push_back(cp);
        ops->push_back(mk(QD, DL_OP_RECORD, DL_EV_DMA_DONE, s, module, layer));
        book->dma_recorded[s] = true;
        return s;
    };

    // The streamed layers of this pass and of the passes after it form one sequence q = 0, 1, 2, ...:
    // q < n_str is streamed layer q of this pass, q >= n_str is layer streamed[q % n_str] of pass q / n_str ahead
    // (copied ahead only with cross-pass prefetch, and only while the next passes run the same module).
    const size_t n_str = streamed.size();
    size_t issued = 0;                          // copies q < issued have been issued
    // copies issued ahead by earlier passes: consumed in order as long as they are the copies this pass needs
    if (n_str > 0 && book->pending_module == module) {
        bool match = true;
        for (int32_t j = 0; j < book->n_pending; ++j) match = match && book->pending_layer[j] == streamed[size_t(j) % n_str];
        if (match) {
            for (int32_t j = 0; j < book->n_pending; ++j) {
                if (size_t(j) < n_str) slot_of[streamed[size_t(j)]] = book->pending_slot[j];
                ++issued;
            }
            // entries beyond this pass's own layers stay pending for the passes after it
            const int32_t used = int32_t(std::min(n_str, size_t(book->n_pending)));
            for (int32_t j = used; j < book->n_pending; ++j) {
                book->pending_layer[j - used] = book->pending_layer[j];
                book->pending_slot[j - used] = book->pending_slot[j];
            }
            book->n_pending -= used;
            if (book->n_pending == 0) book->pending_module = -1;
        } else {
            drop_pending();
        }
    } else {
        drop_pending();
    }
    auto issue_until = [&](size_t limit) {
        while (issued < limit) {
            const size_t q = issued;
            if (q < n_str) {
                slot_of[streamed[q]] = issue_copy(streamed[q], /*gate_on_pass=*/q == 0 && !wrap_prefetch, 0);
            } else {
                if (!wrap_prefetch || n_str == 0 || book->n_pending >= kMaxSlots) return;
                const int32_t layer = streamed[q % n_str];
                const int32_t s = issue_copy(layer, false, int32_t(q / n_str));
                book->pending_module = module;
                book->pending_layer[book->n_pending] = layer;
                book->pending_slot[book->n_pending] = s;
                ++book->n_pending;
            }
            ++issued;
        }
    };
    // With n slots, n - 1 copies run ahead of the streamed layer that executes: the copy into a slot is issued when
    // the layer that used the slot n streamed layers earlier has long recorded its compute-done event, so it overlaps
    // the execution of the layers before it.  With one slot the following copy overwrites THIS layer's parameters,
    // so it is issued after this layer's compute-done record (a wait refers to the latest record issued before it)
    // and overlaps only the resident layers that follow.
    const bool one_slot = book->n_slots == 1;
    const size_t ahead = one_slot ? 0 : size_t(book->n_slots - 1);
    if (n_str > 0) issue_until(one_slot ? 1 : std::min(ahead, n_str));
    size_t si = 0;
    for (int32_t i = 0; i < n_layers; ++i) {
        const bool st = si < n_str && streamed[si] == i;
        int32_t s = -1;
        if (st) {
            s = slot_of[i];
            // a layer never executes before its parameters have arrived
            ops->push_back(mk(QC, DL_OP_WAIT, DL_EV_DMA_DONE, s, module, i));
            ++si;
            if (!one_slot) issue_until(si + ahead);
        }
        ops->push_back(mk(QC, DL_OP_EXEC, -1, s, module, i));
        if (st) {
            ops->push_back(mk(QC, DL_OP_RECORD, DL_EV_COMPUTE_DONE, s, module, i));
            book->compute_recorded[s] = true;
            if (one_slot) issue_until(si + 1);
        }
    }
    ops->push_back(mk(QC, DL_OP_RECORD, DL_EV_PASS_DONE, -1, module, n_layers - 1));
    book->pass_recorded = true;
}

}  // namespace dl

// ------------------------------------------------------------------------------------------
// Planner and predictor: pure functions of the C ABI
// ------------------------------------------------------------------------------------------
extern "C" {

int32_t dl_place_interleaved(int32_t n_layers, int32_t k, int32_t* idx_out) {
    if (n_layers < 1 || k < 0 || k > n_layers || (k > 0 && !idx_out)) return DL_ERR_INVALID_ARG;
    if (k == n_layers) {
        for (int32_t i = 0; i < k; ++i) idx_out[i] = i;
        return DL_OK;
    }
    for (int32_t i = 0; i < k; ++i) idx_out[i] = int32_t((int64_t(i) * (n_layers - 1)) / k);
    return DL_OK;
}

int32_t dl_benefit(double c_dma_ms, double m_mib, int32_t n_phases, const double* c_exe_ms, const int32_t* reps,
                   double* out3) {
    if (!(c_dma_ms >= 0) || !(m_mib > 0) || n_phases < 1 || !c_exe_ms || !reps || !out3) return DL_ERR_INVALID_ARG;
    double first = 0, mid = 0, last = 0;
    for (int32_t p = 0; p < n_phases; ++p) {
        if (reps[p] < 0 || !(c_exe_ms[p] >= 0)) return DL_ERR_INVALID_ARG;
        const double R = reps[p];
        if (c_dma_ms <= c_exe_ms[p]) {
            // EXE-intensive phase (Table IV): only the exposed leading copy of each pass is saved
            first += R * c_dma_ms;
        } else {
            // DMA-intensive phase (Table V): every copy is on the critical path; removing the last one
            // leaves a new trailing execution behind
            first += R * c_dma_ms;
            mid += R * c_dma_ms;
            last += R * (c_dma_ms - c_exe_ms[p]);
        }
    }
    out3[0] = first / m_mib;
    out3[1] = mid / m_mib;
    out3[2] = last / m_mib;
    return DL_OK;
}

int32_t dl_consecutive_limit(double c_dma_ms, double c_exe_ms, int32_t* out) {
    if (!(c_dma_ms >= 0) || !(c_exe_ms > 0) || !out) return DL_ERR_INVALID_ARG;
    *out = int32_t(std::floor(c_dma_ms / c_exe_ms));
    return DL_OK;
}

int32_t dl_predict_linear(double c_total0_ms, double slope_ms_per_layer, int32_t k, double* out) {
    if (k < 0 || !out) return DL_ERR_INVALID_ARG;
    *out = c_total0_ms - double(k) * slope_ms_per_layer;
    return DL_OK;
}

int32_t dl_timeline(const double* c_dma_ms, const double* c_dma_cont_ms, const double* c_exe_ms,
                    const double* c_exe_idle_ms, const double* c_exe_loaded_ms, const double* c_fence_ms,
                    const double* c_fence_hot_ms, const uint8_t* streamed, const uint8_t* pass_start, const int32_t* module_id, int32_t n,
                    int32_t mode, int32_t wrap_prefetch, int32_t n_slots, double overhead_ms,
                    double* total_ms, double* hidden_frac, double* exposed_ms) {
    if (n < 0 || (n > 0 && (!c_dma_ms || !c_exe_ms || !streamed || !pass_start))) return DL_ERR_INVALID_ARG;
    if (n_slots < 1 || n_slots > dl::kMaxSlots) return DL_ERR_INVALID_ARG;
    if (mode != DL_MODE_PIPELINED && mode != DL_MODE_SEQUENTIAL) return DL_ERR_INVALID_ARG;
    if (n > 0 && !pass_start[0]) return DL_ERR_INVALID_ARG;
    // Replays the very schedule a pass enqueues (build_pass) on two in-order queues.
    struct Pass { int32_t j0, j1, module; };
    std::vector<Pass> passes;
    for (int32_t j = 0; j < n;) {
        int32_t j1 = j + 1;
        while (j1 < n && !pass_start[j1]) ++j1;
        passes.push_back({j, j1, module_id ? module_id[j] : 0});
        j = j1;
    }
    dl::SlotBook book;
    book.n_slots = n_slots;
    double t[2] = {0, 0};                       // queue clocks: [0] compute, [1] copy
    double ev_dma[dl::kMaxSlots] = {0, 0, 0, 0}, ev_comp[dl::kMaxSlots] = {0, 0, 0, 0}, ev_pass = 0;
    double copy_start[dl::kMaxSlots] = {0, 0, 0, 0}, copy_dur[dl::kMaxSlots] = {0, 0, 0, 0};
    double exposed = 0, dma_sum = 0;
    std::vector<std::pair<double, double>> copy_busy;   // [start, end) of every copy placed so far, in queue order
    size_t first_live = 0;                               // copies before this index ended before the compute queue's clock
    double last_copy_end = -1.0;                 // copy-queue clock when its latest copy ended (no copy yet: none)
    bool idled = false;                          // the compute queue waited for the copy of the next layer
    std::vector<dl_trace_op> ops;
    std::vector<uint8_t> resident;
    for (size_t p = 0; p < passes.size(); ++p) {
        const Pass& P = passes[p];
        resident.assign(size_t(P.j1 - P.j0), 0);
        for (int32_t j = P.j0; j < P.j1; ++j) resident[size_t(j - P.j0)] = streamed[j] ? 0 : 1;
        ops.clear();
        dl::build_pass(P.module, P.j1 - P.j0, resident.data(), mode, wrap_prefetch, false, &book, &ops);
        for (const dl_trace_op& o : ops) {
            const int32_t q = o.queue;
            const int32_t j = P.j0 + o.layer;
            switch (o.op) {
                case DL_OP_WAIT: {
                    const double e = o.event_kind == DL_EV_DMA_DONE ? ev_dma[o.slot]
                                   : o.event_kind == DL_EV_COMPUTE_DONE ? ev_comp[o.slot] : ev_pass;
                    if (q == 0 && o.event_kind == DL_EV_DMA_DONE) {
                        // time the compute queue idles while the copy it needs is in flight
                        exposed += std::max(0.0, e - std::max(t[0], copy_start[o.slot]));
                        dma_sum += copy_dur[o.slot];
                        idled = e > t[0];
                    }
                    t[q] = std::max(t[q], e);
                    break;
                }
                case DL_OP_RECORD:
                    if (o.event_kind == DL_EV_DMA_DONE) ev_dma[o.slot] = t[q];
                    else if (o.event_kind == DL_EV_COMPUTE_DONE) ev_comp[o.slot] = t[q];
                    else ev_pass = t[q];
                    break;
                case DL_OP_COPY: {
                    int32_t jj = j;
                    if (o.flags > 0) {
                        // copied ahead for a later pass: takes that pass's copy time when it runs the same module
                        const size_t pp = p + size_t(o.flags);
                        if (pp < passes.size() && passes[pp].module == P.module && o.layer < passes[pp].j1 - passes[pp].j0)
                            jj = passes[pp].j0 + o.layer;
                    }
                    // a copy that starts the instant the previous one ended runs at the rate of a train of copies
                    const double dur = (c_dma_cont_ms && t[q] == last_copy_end) ? c_dma_cont_ms[jj] : c_dma_ms[jj];
                    copy_start[o.slot] = t[q];
                    copy_dur[o.slot] = dur;
                    copy_busy.emplace_back(t[q], t[q] + dur);
                    t[q] += dur;
                    last_copy_end = t[q];
                    break;
                }
                case DL_OP_EXEC: {
                    const double exe = (idled && c_exe_idle_ms) ? c_exe_idle_ms[j] : c_exe_ms[j];
                    const double rest = overhead_ms +
                        ((o.slot >= 0 && c_fence_ms) ? ((!idled && c_fence_hot_ms) ? c_fence_hot_ms[j] : c_fence_ms[j]) : 0.0);
                    const double slow = (c_exe_loaded_ms && c_exe_ms[j] > 0.0) ? std::max(1.0, c_exe_loaded_ms[j] / c_exe_ms[j]) : 1.0;
                    double now = t[q], left = exe;
                    if (slow > 1.0) {
                        // the execution advances at 1 / slow while a copy is in flight
                        while (first_live < copy_busy.size() && copy_busy[first_live].second <= now) ++first_live;
                        for (size_t ci = first_live; ci < copy_busy.size() && left > 0.0; ++ci) {
                            const double cs = copy_busy[ci].first, ce = copy_busy[ci].second;
                            if (ce <= now) continue;
                            if (cs > now) {
                                const double free_run = std::min(left, cs - now);
                                now += free_run;
                                left -= free_run;
                                if (left <= 0.0) break;
                            }
                            const double under = (ce - now) / slow;        // work done until this copy ends
                            if (under >= left) { now += left * slow; left = 0.0; }
                            else { now = ce; left -= under; }
                        }
                    }
                    t[q] = now + left + rest;
                    idled = false;
                    break;
                }
                default: break;
            }
        }
    }
    if (total_ms) *total_ms = t[0];
    if (exposed_ms) *exposed_ms = exposed;
    if (hidden_frac) *hidden_frac = dma_sum > 0 ? 1.0 - exposed / dma_sum : 1.0;
    return DL_OK;
}

int32_t dl_plan(int32_t n_modules, const int32_t* n_layers, const uint64_t* layer_bytes, const double* b3,
                uint64_t budget_bytes, int32_t* k_out) {
    if (n_modules < 1 || !n_layers || !layer_bytes || !b3 || !k_out) return DL_ERR_INVALID_ARG;
    // candidate groups: a module's first layer, its middle layers, its last layer (Tables IV-VI rank them
    // first >= middle >= last inside a module); groups are taken in order of benefit per MiB
    struct Group { double b; int32_t module, order, count; };
    std::vector<Group> groups;
    for (int32_t m = 0; m < n_modules; ++m) {
        if (n_layers[m] < 1 || layer_bytes[m] == 0) return DL_ERR_INVALID_ARG;
        const double* b = b3 + 3 * m;
        if (!(b[0] >= 0) || !(b[1] >= 0) || !(b[2] >= 0)) return DL_ERR_INVALID_ARG;
        k_out[m] = 0;
        if (n_layers[m] == 1) {
            groups.push_back({b[0], m, 0, 1});
            continue;
        }
        groups.push_back({b[0], m, 0, 1});
        if (n_layers[m] > 2) groups.push_back({std::min(b[1], b[0]), m, 1, n_layers[m] - 2});
        groups.push_back({std::min(b[2], std::min(b[1], b[0])), m, 2, 1});
    }
    std::stable_sort(groups.begin(), groups.end(), [](const Group& a, const Group& c) {
        if (a.b != c.b) return a.b > c.b;
        if (a.module != c.module) return a.module < c.module;
        return a.order < c.order;
    });
    uint64_t left = budget_bytes;
    std::vector<int32_t> next_order(size_t(n_modules), 0);
    for (const Group& g : groups) {
        if (!(g.b > 0)) break;                              // no time to win: keep the memory
        if (g.order != next_order[size_t(g.module)]) continue;   // never skip ahead inside a module
        const uint64_t each = layer_bytes[g.module];
        const int32_t take = int32_t(std::min<uint64_t>(uint64_t(g.count), left / each));
        k_out[g.module] += take;
        left -= uint64_t(take) * each;
        if (take == g.count) next_order[size_t(g.module)] = g.order + 1;
        else next_order[size_t(g.module)] = 99;             // group cut short: nothing further from this module
    }
    return DL_OK;
}

int32_t dl_plan_shared_slots(int32_t n_modules, const int32_t* n_layers, const uint64_t* layer_bytes, const double* b3,
                             uint64_t budget_bytes, int32_t n_slots, int32_t* k_out) {
    if (n_modules < 1 || n_modules > 12 || !n_layers || !layer_bytes || !b3 || !k_out || n_slots < 1) return DL_ERR_INVALID_ARG;
    for (int32_t m = 0; m < n_modules; ++m) {
        if (n_layers[m] < 1 || layer_bytes[m] == 0) return DL_ERR_INVALID_ARG;
        const double* b = b3 + 3 * m;
        if (!(b[0] >= 0) || !(b[1] >= 0) || !(b[2] >= 0)) return DL_ERR_INVALID_ARG;
    }
    const double MiB = 1048576.0;
    // benefit (ms) of the first j resident layers of module m in dl_plan's order: first, middles, last
    auto value_of = [&](int32_t m, int32_t j) {
        const double* b = b3 + 3 * m;
        const double mib = double(layer_bytes[m]) / MiB;
        const int32_t L = n_layers[m];
        double v = 0.0;
        if (j >= 1) v += b[0] * mib;
        if (L > 2) v += std::min(b[1], b[0]) * mib * double(std::min(std::max(j - 1, 0), L - 2));
        if (L >= 2 && j >= L) v += std::min(b[2], std::min(b[1], b[0])) * mib;
        return v;
    };
    bool found = false;
    double best_v = -1.0;
    uint64_t best_bytes = 0;
    std::vector<int32_t> best(size_t(n_modules), 0), cur(size_t(n_modules), 0);
    std::vector<int32_t> sub_layers;
    std::vector<uint64_t> sub_bytes;
    std::vector<double> sub_b3;
    std::vector<int32_t> sub_index, sub_k;
    for (uint32_t F = 0; F < (1u << n_modules); ++F) {
        uint64_t fixed = 0, slot = 0;
        bool overflow = false;
        for (int32_t m = 0; m < n_modules; ++m) {
            if ((F >> m) & 1u) {
                fixed += uint64_t(n_layers[m]) * layer_bytes[m];
                if (fixed > budget_bytes) { overflow = true; break; }
            } else {
                slot = std::max(slot, layer_bytes[m]);
            }
        }
        if (overflow) continue;
        fixed += uint64_t(n_slots) * slot;
        if (fixed > budget_bytes) continue;
        // the modules outside F keep at least their last layer streamed: hand dl_plan a stack without it
        sub_layers.clear(); sub_bytes.clear(); sub_b3.clear(); sub_index.clear();
        for (int32_t m = 0; m < n_modules; ++m) {
            if ((F >> m) & 1u) { cur[size_t(m)] = n_layers[m]; continue; }
            cur[size_t(m)] = 0;
            if (n_layers[m] < 2) continue;                 // its only layer is the streamed one
            sub_index.push_back(m);
            sub_layers.push_back(n_layers[m] - 1);
            sub_bytes.push_back(layer_bytes[m]);
            // a stack of L - 1 layers whose "last" group is one more middle layer (or the first, if L == 2)
            const double* b = b3 + 3 * m;
            const double mid = std::min(b[1], b[0]);
            sub_b3.push_back(b[0]);
            sub_b3.push_back(mid);
            sub_b3.push_back(n_layers[m] - 1 >= 2 ? mid : b[0]);
        }
        if (!sub_index.empty()) {
            sub_k.assign(sub_index.size(), 0);
            const int32_t rc = dl_plan(int32_t(sub_index.size()), sub_layers.data(), sub_bytes.data(), sub_b3.data(),
                                       budget_bytes - fixed, sub_k.data());
            if (rc != DL_OK) return rc;
            for (size_t i = 0; i < sub_index.size(); ++i) cur[size_t(sub_index[i])] = sub_k[i];
        }
        double v = 0.0;
        uint64_t bytes = 0;
        for (int32_t m = 0; m < n_modules; ++m) {
            v += value_of(m, cur[size_t(m)]);
            bytes += uint64_t(cur[size_t(m)]) * layer_bytes[m];
        }
        if (!found || v > best_v || (v == best_v && bytes < best_bytes)) {
            found = true;
            best_v = v;
            best_bytes = bytes;
            best = cur;
        }
    }
    if (!found) return DL_ERR_BUDGET_EXCEEDED;
    for (int32_t m = 0; m < n_modules; ++m) k_out[m] = best[size_t(m)];
    return DL_OK;
}

}  // extern "C"
