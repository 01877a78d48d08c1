// Internal declarations shared by the host core (dl_host.cpp) and the HIP backend (dl_api.hip).
// Nothing here crosses the C ABI.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "demand_layering.h"

namespace dl {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v, uint64_t a = kAlign) { return (v + a - 1) / a * a; }

// ---- arena: first-fit free list over [0, capacity), offsets only (works without a device) ----
class Arena {
public:
    void reset(uint64_t capacity);
    // returns false if no free range of that size exists
    bool alloc(uint64_t bytes, uint64_t* off_out);
    // same, but takes the END of the HIGHEST free range that is large enough.  For blocks that get re-sized later
    // (activation workspaces): kept at the top, what they give back joins the free range below them instead of
    // leaving a hole between longer-lived blocks.
    bool alloc_top(uint64_t bytes, uint64_t* off_out);
    bool free(uint64_t off);
    uint64_t used() const { return used_; }
    uint64_t peak() const { return peak_; }
    uint64_t capacity() const { return cap_; }
    bool is_set() const { return cap_ > 0; }
    uint64_t size_of(uint64_t off) const;
    // forget a peak reached by temporaries (profiling): the peak becomes max(peak_before, current use)
    void restore_peak(uint64_t peak_before) { peak_ = peak_before > used_ ? peak_before : used_; }
private:
    struct Block { uint64_t off, size; bool used; };
    std::vector<Block> blocks_;
    uint64_t cap_ = 0, used_ = 0, peak_ = 0;
};

// ---- byte layout of one layer's packed blob (what one host-to-device copy moves) ----
struct PackLayout {
    static constexpr uint64_t kNone = ~0ull;
    // byte offsets of each section inside the blob; kNone when the section does not exist
    uint64_t norm1_g = kNone, norm1_b = kNone, w_qkv = kNone, b_qkv = kNone, w_o = kNone, b_o = kNone;
    uint64_t normc_g = kNone, normc_b = kNone, w_qc = kNone, b_qc = kNone, w_kvc = kNone, b_kvc = kNone,
             w_oc = kNone, b_oc = kNone;
    uint64_t norm2_g = kNone, norm2_b = kNone, w_up = kNone, b_up = kNone, w_down = kNone, b_down = kNone;
    uint64_t bytes = 0;        // blob size, multiple of kAlign
    uint64_t param_bytes = 0;  // 2 * number of parameters
    int32_t n_qkv = 0;         // rows of the fused QKV matrix
    int32_t n_up = 0;          // rows of the first FFN matrix (2*d_ff interleaved for SwiGLU)
    int32_t ffp = 0;           // d_ff rounded up to 128: row length of the second FFN matrix and of the
                               // activation between the two (zero padding keeps the GEMM K a multiple of 128)
};

bool validate_desc(const dl_module_desc& d, std::string* why);
PackLayout make_layout(const dl_module_desc& d);
// bit t set <=> tensor id t must be provided for every layer
uint32_t required_tensor_mask(const dl_module_desc& d);
// number of BF16 elements tensor `tid` must have, 0 if the tensor does not exist for this descriptor
uint64_t tensor_elems(const dl_module_desc& d, int32_t tid);
// copies one caller tensor into its place in the blob (fusing Q/K/V rows, interleaving gate/up rows)
void pack_tensor(const dl_module_desc& d, const PackLayout& L, int32_t tid, const uint16_t* src, uint8_t* blob);

// ---- activation workspace / KV cache sizes of a module, in bytes ----
struct WorkspaceLayout {
    uint64_t nbuf = 0, qkv = 0, attn = 0, mid = 0, vt = 0, ctxn = 0, kvc = 0, vtc = 0, logits = 0, token = 0,
             dec_part = 0, att_part = 0;  // offsets
    uint64_t att_part_bytes = 0;  // scratch of the split cross-attention (0: none)
    uint64_t bytes = 0;
    int32_t vt_ld = 0;      // row length (positions) of the transposed-V scratch
    int32_t vtc_ld = 0;     // same for the cross-attention V scratch
};
WorkspaceLayout make_workspace(const dl_module_desc& d);
struct KvLayout {
    uint64_t k_layer_bytes = 0, v_layer_bytes = 0, bytes = 0;
    int32_t v_ld = 0;       // positions per row of the transposed V cache (max_seq rounded up to 64)
};
KvLayout make_kv(const dl_module_desc& d);

// ---- the schedule of one pass as data (Sec. IV-C(ii)) ----
constexpr int32_t kMaxSlots = 4;
struct SlotBook {
    // persistent across passes
    int32_t n_slots = 2;                  // device slots, 1 .. kMaxSlots
    uint64_t ordinal = 0;                 // count of copies issued so far; slot = ordinal % n_slots
    bool dma_recorded[kMaxSlots] = {false, false, false, false};
    bool compute_recorded[kMaxSlots] = {false, false, false, false};
    bool pass_recorded = false;
    // copies issued ahead for the first streamed layers of coming passes and not consumed yet, oldest first
    int32_t n_pending = 0;
    int32_t pending_module = -1;
    int32_t pending_layer[kMaxSlots] = {-1, -1, -1, -1}, pending_slot[kMaxSlots] = {-1, -1, -1, -1};
};
// Appends the ops of one pass over a module to `ops`.  resident[i] != 0: layer i executes from its
// resident copy.  force_stream_all: every layer is copied (profiling).  Updates `book`.
void build_pass(int32_t module, int32_t n_layers, const uint8_t* resident, int32_t mode, int32_t wrap_prefetch,
                bool force_stream_all, SlotBook* book, std::vector<dl_trace_op>* ops);

}  // namespace dl
