"""Pins for oracle/planner.py: values the paper prints, its closed forms, and a brute-force
discrete-event simulation of the two-event protocol (Sec. IV-C(ii))."""
import itertools
import json
import math
import os
import random

import pytest

from oracle import planner as P
from tests.des_sim import simulate

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
T3 = GOLD["table3_profile_rtx5070ti"]
MS = GOLD["module_shapes"]


def test_table7_printed_benefits():
    vit = P.benefit_exe_intensive(MS["vit"]["R"], T3["vision"]["C_DMA"], MS["vit"]["M"])
    vlm = P.benefit_hybrid(MS["vlm"]["N"], T3["vlm_decode"]["C_DMA"], T3["vlm_decode"]["C_EXE"], MS["vlm"]["M"])
    exp = P.benefit_dma_intensive(MS["expert"]["R"], T3["diffusion"]["C_DMA"], T3["diffusion"]["C_EXE"], MS["expert"]["M"])
    for got, want in ((vit, GOLD["table7_benefit_ms_per_MB"]["vit"]),
                      (vlm, GOLD["table7_benefit_ms_per_MB"]["vlm"]),
                      (exp, GOLD["table7_benefit_ms_per_MB"]["expert"])):
        for g, w in zip(got, want):
            assert abs(g - w) < 1e-3, (got, want)   # three printed decimals; 22*10.9/368.0 = 0.6516 is printed as 0.651


def test_eq4_matches_tables_for_middle_layers():
    # Eq. 4 with delta C = C_DMA - min(C_DMA, C_EXE): zero for an EXE-intensive layer,
    # C_DMA - C_EXE for a DMA-intensive one (the "last" rows of Tables V/VI)
    assert P.residency_benefit(1, 0.9, 8.3, 29.1) == 0.0
    assert P.residency_benefit(21, 10.9, 0.9, 368.0) == pytest.approx(21 * 10.0 / 368.0)
    assert P.delta_C(3.6, 1.0) == pytest.approx(2.6)


def test_ratio_r_and_consecutive_limit():
    for row in ("vision", "vlm_prefill", "vlm_decode", "diffusion"):
        r = T3[row]["C_DMA"] / T3[row]["C_EXE"]
        # r is printed from unrounded times: 3.6/1.0 shows as 3.5, 10.9/16.6 = 0.657 as 0.66
        assert abs(r - T3[row]["r"]) / T3[row]["r"] < 0.1
    assert P.consecutive_residency_limit(T3["vlm_decode"]["C_DMA"], T3["vlm_decode"]["C_EXE"]) == \
        GOLD["consecutive_limit_vlm_decode"]["value"]


def test_eq8_placement_properties():
    L = 36
    assert P.interleaved_placement(5, L) == [0, 7, 14, 21, 28]
    for k in range(1, L):
        idx = P.interleaved_placement(k, L)
        assert len(idx) == k and len(set(idx)) == k
        assert idx[0] == 0 and (L - 1) not in idx
        gaps = [b - a for a, b in zip(idx, idx[1:])]
        assert all(g >= (L - 1) // k for g in gaps)
    assert P.interleaved_placement(0, L) == []
    assert P.interleaved_placement(L, L) == list(range(L))
    for L2 in (4, 8, 27):
        for k in range(1, L2):
            idx = P.interleaved_placement(k, L2)
            assert len(set(idx)) == k and idx[0] == 0 and max(idx) <= L2 - 2


def test_eq9_table8_rows():
    t8 = GOLD["table8_prediction"]
    c0 = t8["C_total_0_s"] * 1e3
    step = -t8["slope_ms_per_layer"]
    for row in t8["rows"]:
        # slope = B_VLM * M_VLM; feed Eq. 9 with B = step / M
        pred = P.predict_linear(c0, row["k"], step / 368.0, 368.0) / 1e3
        assert abs(pred - row["predicted_s"]) < 6e-4
        err = (row["predicted_s"] - row["measured_s"]) / row["measured_s"] * 100
        assert abs(err - row["error_pct"]) < 0.02   # the error column is printed from unrounded times
    # the profiled slope equals N * C_DMA (Table VI middle row times M) up to the rounding of Table III
    assert abs(21 * 10.9 - step) / step < 0.004


def test_closed_forms_vs_paper_measurement():
    # Eq. 5 + Eq. 7 + Eq. 6 with Table III values land near the measured 10.482 s (sanity, not exact)
    vit = P.module_time_exe_intensive(1, 27, 0.9, 8.3)
    vlm = P.module_time_hybrid(21, 36, 10.9, 16.6, 0.9)
    exp = P.module_time_dma_intensive(10, 36, 3.6, 1.0)
    assert vit == pytest.approx(225.0) and vlm == pytest.approx(8867.8) and exp == pytest.approx(1306.0)
    assert abs((vit + vlm + exp) / 1e3 - 10.482) / 10.482 < 0.02


def _uniform(L, c_dma, c_exe, resident=()):
    return [(c_dma, c_exe, i not in resident) for i in range(L)]


def test_timeline_reduces_to_eq1_eq2_eq3():
    rnd = random.Random(1)
    L = 9
    # Eq. 1: every layer EXE-intensive (and each transfer shorter than the previous execution)
    dma = [rnd.uniform(0.5, 1.0) for _ in range(L)]
    exe = [rnd.uniform(2.0, 3.0) for _ in range(L)]
    tl = P.timeline([[(d, e, True) for d, e in zip(dma, exe)]])
    assert tl["total"] == pytest.approx(P.time_exe_intensive(dma, exe))
    # Eq. 2: every layer DMA-intensive
    dma = [rnd.uniform(2.0, 3.0) for _ in range(L)]
    exe = [rnd.uniform(0.5, 1.0) for _ in range(L)]
    tl = P.timeline([[(d, e, True) for d, e in zip(dma, exe)]])
    assert tl["total"] == pytest.approx(P.time_dma_intensive(dma, exe))
    # Eq. 3: nothing streamed
    tl = P.timeline([[(d, e, False) for d, e in zip(dma, exe)]])
    assert tl["total"] == pytest.approx(P.lower_bound(exe)) and tl["hidden"] == 1.0


@pytest.mark.parametrize("R", [1, 3, 10])
def test_timeline_reduces_to_eq5_eq6_eq7(R):
    L = 7
    assert P.timeline([_uniform(L, 0.9, 8.3)] * R)["total"] == pytest.approx(P.module_time_exe_intensive(R, L, 0.9, 8.3))
    assert P.timeline([_uniform(L, 3.6, 1.0)] * R)["total"] == pytest.approx(P.module_time_dma_intensive(R, L, 3.6, 1.0))
    hybrid = [_uniform(L, 10.9, 16.6)] + [_uniform(L, 10.9, 0.9)] * R
    assert P.timeline(hybrid)["total"] == pytest.approx(P.module_time_hybrid(R, L, 10.9, 16.6, 0.9))


def test_timeline_single_layer_residency_matches_tables_4_5_6():
    L, M = 8, 100.0
    first, mid, last = 0, 3, L - 1

    def saved(build, pos):
        return P.timeline(build(()))["total"] - P.timeline(build((pos,)))["total"]

    for R in (1, 4):
        exe_int = lambda res: [_uniform(L, 0.9, 8.3, res)] * R
        want = P.benefit_exe_intensive(R, 0.9, M)
        assert [saved(exe_int, p) / M for p in (first, mid, last)] == pytest.approx(list(want), abs=1e-12)
        dma_int = lambda res: [_uniform(L, 3.6, 1.0, res)] * R
        want = P.benefit_dma_intensive(R, 3.6, 1.0, M)
        assert [saved(dma_int, p) / M for p in (first, mid, last)] == pytest.approx(list(want))
        hyb = lambda res: [_uniform(L, 10.9, 16.6, res)] + [_uniform(L, 10.9, 0.9, res)] * R
        want = P.benefit_hybrid(R, 10.9, 0.9, M)
        assert [saved(hyb, p) / M for p in (first, mid, last)] == pytest.approx(list(want))


def protocol_ops(invocations, wrap_prefetch):
    """Host-ordered queue ops of the two-event protocol as the paper words it: the compute queue
    waits on DMA-done before a streamed layer and records compute-done after it; the copy queue
    waits on compute-done of the slot before overwriting it and records DMA-done after the copy;
    the copy for the next streamed layer is issued while the current one executes."""
    flat = [(p, i) + tuple(rec) for p, layers in enumerate(invocations) for i, rec in enumerate(layers)]
    streamed = [n for n, r in enumerate(flat) if r[4]]
    ordinal = {n: j for j, n in enumerate(streamed)}
    ops = []
    issued = set()

    def issue(n, barrier_pass=None):
        s = ordinal[n] % 2
        if barrier_pass is not None:
            ops.append(("copy", ("wait", ("pass_end", barrier_pass))))
        ops.append(("copy", ("wait", ("compute_done", s))))
        ops.append(("copy", ("copy", flat[n][2], n)))
        ops.append(("copy", ("record", ("dma_done", s))))
        issued.add(n)

    for n, (p, i, c_dma, c_exe, st) in enumerate(flat):
        first_of_pass = i == 0
        if first_of_pass and p > 0:
            ops.append(("compute", ("record", ("pass_end", p - 1))))
        if first_of_pass:
            # the first streamed layer of this pass, unless a previous pass prefetched it
            nxt = [m for m in streamed if flat[m][0] == p]
            if nxt and nxt[0] not in issued:
                issue(nxt[0], barrier_pass=(p - 1) if (p > 0) else None)
        if st:
            ops.append(("compute", ("wait", ("dma_done", ordinal[n] % 2))))
            j = ordinal[n] + 1
            if j < len(streamed):
                m = streamed[j]
                if flat[m][0] == p or wrap_prefetch:
                    issue(m)
        ops.append(("compute", ("exec", c_exe, n)))
        if st:
            ops.append(("compute", ("record", ("compute_done", ordinal[n] % 2))))
    return ops, flat


def des_total(invocations, wrap_prefetch):
    ops, flat = protocol_ops(invocations, wrap_prefetch)
    times = simulate(ops)
    # safety properties of the protocol (Sec. IV-C(ii)): never execute before the parameters arrive,
    # never overwrite a slot that is still in use
    copy_span, exec_span = {}, {}
    for (q, op), (t0, t1) in zip(ops, times):
        if op[0] == "copy":
            copy_span[op[2]] = (t0, t1)
        if op[0] == "exec":
            exec_span[op[2]] = (t0, t1)
    streamed = sorted(copy_span)
    for j, n in enumerate(streamed):
        assert exec_span[n][0] >= copy_span[n][1] - 1e-12
        if j >= 2:
            assert copy_span[n][0] >= exec_span[streamed[j - 2]][1] - 1e-12
    return max(t1 for _, t1 in times)


@pytest.mark.parametrize("wrap", [False, True])
def test_timeline_equals_discrete_event_simulation_all_residency_sets(wrap):
    rnd = random.Random(7)
    for L in (1, 2, 3, 5, 6):
        dma = [rnd.uniform(0.2, 4.0) for _ in range(L)]
        exe_a = [rnd.uniform(0.2, 4.0) for _ in range(L)]
        exe_b = [rnd.uniform(0.1, 1.0) for _ in range(L)]
        for mask in itertools.product([False, True], repeat=L):
            inv = [[(dma[i], exe_a[i], mask[i]) for i in range(L)]] + \
                  [[(dma[i], exe_b[i], mask[i]) for i in range(L)]] * 2
            assert P.timeline(inv, wrap_prefetch=wrap)["total"] == pytest.approx(des_total(inv, wrap), rel=1e-12)


def test_hidden_fraction_limits():
    # EXE-intensive: only the first transfer is exposed; DMA-intensive: everything but what hides under EXE
    L = 10
    tl = P.timeline([_uniform(L, 1.0, 5.0)])
    assert tl["exposed"] == pytest.approx(1.0) and tl["hidden"] == pytest.approx(1 - 1.0 / L)
    tl = P.timeline([_uniform(L, 5.0, 1.0)])
    assert tl["exposed"] == pytest.approx(5.0 + (L - 1) * 4.0)
    assert P.sequential_time([_uniform(L, 5.0, 1.0)]) == pytest.approx(L * 6.0)


def test_timeline_corrections_closed_forms():
    """the measured corrections against hand-derived totals: one pass of L identical streamed layers"""
    L, f, ov = 9, 0.25, 0.125
    # execution-bound (C_EXE > C_DMA): only the first layer waits for its transfer and runs at the idle time
    exe_bound = [[(1.0, 4.0, True, 5.0, f)] * L]
    assert P.timeline(exe_bound, overhead=ov)["total"] == pytest.approx(1.0 + 5.0 + (L - 1) * 4.0 + L * (f + ov))
    # transfer-bound (C_DMA > C_EXE_idle + fence + overhead): every layer waits; total = all transfers + last layer
    dma_bound = [[(4.0, 1.0, True, 1.5, f)] * L]
    assert P.timeline(dma_bound, overhead=ov)["total"] == pytest.approx(L * 4.0 + 1.5 + f + ov)
    # resident layers carry neither the idle time nor the fence
    res = [[(4.0, 1.0, False, 1.5, f)] * L]
    assert P.timeline(res, overhead=ov)["total"] == pytest.approx(L * (1.0 + ov))
    # sequential: transfer + idle execution + fence per streamed layer
    assert P.sequential_time(dma_bound, overhead=ov) == pytest.approx(L * (4.0 + 1.5 + f + ov))
    # three-field records are the five-field ones with C_EXE_idle = C_EXE and no fence
    a = [[(2.0, 3.0, True), (1.0, 0.5, False), (2.5, 0.7, True)]] * 3
    b = [[(d, e, s, e, 0.0) for (d, e, s) in layers] for layers in a]
    assert P.timeline(a)["total"] == P.timeline(b)["total"]


def test_shared_slot_residency_bytes_and_value_closed_forms():
    M = [3 << 20, 7 << 20]
    L = [4, 5]
    # bytes: copies + two slots of the largest layer that still streams; none when nothing streams
    assert P.residency_bytes([0, 0], L, M) == 2 * M[1]
    assert P.residency_bytes([4, 2], L, M) == 4 * M[0] + 2 * M[1] + 2 * M[1]
    assert P.residency_bytes([1, 5], L, M) == M[0] + 5 * M[1] + 2 * M[0]
    assert P.residency_bytes([4, 5], L, M) == 4 * M[0] + 5 * M[1]
    assert P.residency_bytes([1, 5], L, M, n_slots=3) == M[0] + 5 * M[1] + 3 * M[0]
    # value: Table VI's positions, first + middles + last, in MiB
    b3 = P.benefit_hybrid(N=21, C_DMA=11.0, C_decode=0.9, M=7.0)
    full = P.residency_value(5, 5, M[1], b3)
    assert full == pytest.approx((b3[0] + 3 * b3[1] + b3[2]) * 7.0)
    # all resident removes exactly what Eq. 7 pays for transfers beyond the last decode's trailing execution
    assert full == pytest.approx((21 + 1) * 11.0 + 3 * 21 * 11.0 + 21 * (11.0 - 0.9))
    assert P.residency_value(0, 5, M[1], b3) == 0.0
    assert P.residency_value(3, 5, M[1], b3) == pytest.approx((b3[0] + 2 * b3[1]) * 7.0)


def test_shared_slot_exhaustive_search_single_module_closed_form():
    M = 1 << 20
    b3 = [(1.0, 0.8, 0.3)]
    for L in (1, 2, 5):
        for budget in range(0, (L + 3) * M + 1, M // 2):
            got = P.plan_shared_slots_exhaustive([L], [M], b3, budget)
            if budget >= L * M:
                assert got[0] == [L]                 # no slots once everything is resident
            elif budget < 2 * M:
                assert got is None                   # not even the two slots fit
            else:
                assert got[0] == [min(L - 1, (budget - 2 * M) // M)]
