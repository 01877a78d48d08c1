"""CPU oracle for the residency planner and the latency predictor — TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this file.  It shares no code with the product library and imports nothing
from it.  Plain Python floats (float64), the paper's notation:

    C_DMA, C_EXE   per-layer transfer / execution time          (Sec. II-C)
    L              layers in a module;  R (or N) repetitions per inference
    M              layer footprint (the paper's "MB" are MiB)
    B              residency benefit, time saved per unit of memory (Eq. 4)

Functions follow, in the paper's order: Eq. 1, Eq. 2, Eq. 3 (Sec. II-C, III-A);
Eq. 4 and the per-position Tables IV, V, VI with the module times Eq. 5, 6, 7
(Sec. IV-D); the consecutive residency limit; the interleaved placement Eq. 8;
the value and the device bytes of a residency over several modules that share
the slots, with an exhaustive search for the best one (small stacks);
the linear prediction model Eq. 9 (Sec. IV-E).  `timeline` is the two-event
protocol of Sec. IV-C(ii) written as arithmetic: every closed form above is
a special case of it, which is how it is pinned
(tests/test_oracle_planner.py, with the values the paper prints in
Sec. IV-D and Table VIII stored under tests/golden/).
"""
import math


# ---- Sec. II-C ---------------------------------------------------------------
def time_exe_intensive(C_DMA, C_EXE):
    """Eq. 1: lists of per-layer times, every layer with C_DMA < C_EXE: the first transfer
    is exposed, the rest hide under execution."""
    return C_DMA[0] + sum(C_EXE)


def time_dma_intensive(C_DMA, C_EXE):
    """Eq. 2: every layer with C_DMA > C_EXE: the transfers chain, only the last execution trails."""
    return sum(C_DMA) + C_EXE[-1]


def lower_bound(C_EXE):
    """Eq. 3: C_opt, all parameters preloaded."""
    return sum(C_EXE)


# ---- Sec. IV-D ---------------------------------------------------------------
def delta_C(C_DMA, C_EXE):
    """Per-invocation time saved by keeping one layer resident (text under Eq. 4)."""
    return C_DMA - min(C_DMA, C_EXE)


def residency_benefit(R, C_DMA, C_EXE, M):
    """Eq. 4."""
    return R * delta_C(C_DMA, C_EXE) / M


def module_time_exe_intensive(R, L, C_DMA, C_EXE):
    """Eq. 5."""
    return R * (C_DMA + L * C_EXE)


def module_time_dma_intensive(R, L, C_DMA, C_EXE):
    """Eq. 6."""
    return R * (L * C_DMA + C_EXE)


def module_time_hybrid(N, L, C_DMA, C_prefill, C_decode):
    """Eq. 7: one EXE-intensive pass (prefill) then N DMA-intensive passes (decode) over the same layers."""
    return C_DMA + L * C_prefill + N * (L * C_DMA + C_decode)


def benefit_exe_intensive(R, C_DMA, M):
    """Table IV: (first, middle, last)."""
    return (R * C_DMA / M, 0.0, 0.0)


def benefit_dma_intensive(R, C_DMA, C_EXE, M):
    """Table V: (first, middle, last); first and middle are equal."""
    return (R * C_DMA / M, R * C_DMA / M, R * (C_DMA - C_EXE) / M)


def benefit_hybrid(N, C_DMA, C_decode, M):
    """Table VI: (first, middle, last)."""
    return ((N + 1) * C_DMA / M, N * C_DMA / M, N * (C_DMA - C_decode) / M)


def consecutive_residency_limit(C_DMA, C_EXE):
    """Largest run of resident layers whose execution hides inside one transfer (Sec. IV-D)."""
    return math.floor(C_DMA / C_EXE)


def interleaved_placement(k, L=36):
    """Eq. 8, R(k) = { floor(i*(L-1)/k) : i = 0..k-1 } over layers 0..L-2 (first in, last out);
    the paper prints it for L = 36.  Outside the printed range: k = 0 gives the empty set and
    k = L gives every layer (the only way to include the last one)."""
    if k == 0:
        return []
    if k == L:
        return list(range(L))
    assert 1 <= k <= L - 1
    return [(i * (L - 1)) // k for i in range(k)]


# ---- Sec. IV-D over several modules that share the slots (Sec. IV-C(i)) ------------------
def residency_value(k, L, M_bytes, b3):
    """Time saved (ms) by keeping k of a module's L layers resident, taken in the order the per-position tables
    rank them (first, then the middle layers, the last one last): sum of B * M over those layers, B in ms/MiB,
    middle and last capped by the ranks before them as the ranking requires."""
    b_first, b_mid, b_last = b3
    b_mid = min(b_mid, b_first)
    b_last = min(b_last, b_mid)
    mib = M_bytes / 1048576.0
    v = 0.0
    for j in range(k):                       # j-th layer taken
        if j == 0:
            v += b_first * mib
        elif j == L - 1:
            v += b_last * mib
        else:
            v += b_mid * mib
    return v


def residency_bytes(k, L, M_bytes, n_slots=2):
    """Device bytes of a residency (k_m) over modules with L_m layers of M_m bytes: the resident copies plus
    n_slots slots of the largest layer among the modules that still stream one (none if nothing streams)."""
    streaming = [M_bytes[m] for m in range(len(k)) if k[m] < L[m]]
    return sum(k[m] * M_bytes[m] for m in range(len(k))) + (n_slots * max(streaming) if streaming else 0)


def plan_shared_slots_exhaustive(L, M_bytes, b3, budget_bytes, n_slots=2):
    """The residency (k_m) with the largest total residency_value among all that fit the budget, found by trying every
    vector of counts (small stacks only).  Ties: fewer resident bytes.  Returns (k, value) or None if nothing fits."""
    best = None
    def rec(m, k):
        nonlocal best
        if m == len(L):
            if residency_bytes(k, L, M_bytes, n_slots) > budget_bytes:
                return
            v = sum(residency_value(k[i], L[i], M_bytes[i], b3[i]) for i in range(len(L)))
            by = sum(k[i] * M_bytes[i] for i in range(len(L)))
            if best is None or v > best[1] + 1e-12 or (abs(v - best[1]) <= 1e-12 and by < best[2]):
                best = (list(k), v, by)
            return
        for j in range(L[m] + 1):
            rec(m + 1, k + [j])
    rec(0, [])
    return None if best is None else (best[0], best[1])


# ---- Sec. IV-E ---------------------------------------------------------------
def predict_linear(C_total_0, k, B_VLM, M_VLM):
    """Eq. 9."""
    return C_total_0 - k * B_VLM * M_VLM


# ---- Sec. IV-C(ii) as arithmetic -----------------------------------------------
def _layer_terms(rec):
    """A layer record is (C_DMA, C_EXE, streamed) or, with the measured corrections of the MI355X build,
    (C_DMA, C_EXE, streamed, C_EXE_idle, C_fence):
      C_EXE_idle  execution time of the layer when the compute queue had to wait for its transfer
                  (the GPU was idle just before; the paper's profiling run measures exactly this);
      C_fence     time the two cross-queue hand-offs of a streamed layer add on the compute queue."""
    if len(rec) == 3:
        C_DMA, C_EXE, streamed = rec
        return C_DMA, C_EXE, streamed, C_EXE, 0.0
    return rec


def timeline(invocations, wrap_prefetch=False, n_slots=2, overhead=0.0):
    """invocations: list of passes over a layer stack, each a list of layer records (see _layer_terms).
    One copy queue and one compute queue; the j-th streamed layer uses slot j mod n_slots (ordinal among
    streamed layers, counted across passes).

      DMA-done:      a streamed layer starts executing only after its transfer ended;
      compute-done:  a transfer into a slot starts only after the layer that last
                     used that slot finished executing;
      each queue runs its items in order.

    Without wrap_prefetch the first transfer of a pass is issued when the pass begins
    (after the previous pass's last layer ended) — the per-pass restart that Eq. 6
    and the "last" rows of Tables V and VI assume.  With it, the transfer is issued as soon
    as the queues allow.

    A layer occupies the compute queue for C_EXE (C_EXE_idle if the queue waited for its transfer)
    + C_fence (streamed layers only) + overhead (every layer).

    Returns dict(total, exposed, dma, hidden): total time, summed exposed transfer time (time
    the compute queue sat idle waiting for a transfer), summed transfer time, 1 - exposed/dma."""
    dma_end_prev = 0.0          # end of the previous transfer on the copy queue
    exe_end_prev = 0.0          # end of the previous layer on the compute queue
    slot_free = [0.0] * n_slots  # exe_end of the streamed layer that last used each slot
    ordinal = 0
    exposed = 0.0
    dma_sum = 0.0
    for layers in invocations:
        pass_begin = exe_end_prev
        first_streamed = True
        for rec in layers:
            C_DMA, C_EXE, streamed, C_EXE_idle, C_fence = _layer_terms(rec)
            if streamed:
                s = ordinal % n_slots
                ordinal += 1
                dma_start = max(dma_end_prev, slot_free[s])
                if first_streamed and not wrap_prefetch:
                    dma_start = max(dma_start, pass_begin)
                first_streamed = False
                dma_end = dma_start + C_DMA
                dma_end_prev = dma_end
                dma_sum += C_DMA
                exposed += max(0.0, dma_end - max(exe_end_prev, dma_start))
                waited = dma_end > exe_end_prev
                exe_start = max(exe_end_prev, dma_end)
                exe_end_prev = exe_start + (C_EXE_idle if waited else C_EXE) + C_fence + overhead
                slot_free[s] = exe_end_prev
            else:
                exe_end_prev = exe_end_prev + C_EXE + overhead
    hidden = 1.0 - exposed / dma_sum if dma_sum > 0 else 1.0
    return dict(total=exe_end_prev, exposed=exposed, dma=dma_sum, hidden=hidden)


def sequential_time(invocations, overhead=0.0):
    """Sequential Demand Layering (Sec. IV-B): transfer and execution strictly alternate, so every streamed
    layer finds the compute queue waiting for it."""
    total = 0.0
    for layers in invocations:
        for rec in layers:
            C_DMA, C_EXE, streamed, C_EXE_idle, C_fence = _layer_terms(rec)
            total += (C_DMA + C_EXE_idle + C_fence if streamed else C_EXE) + overhead
    return total
