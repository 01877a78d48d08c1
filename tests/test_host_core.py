"""CPU tests of the library's host logic through the C ABI: exports, packing sizes, planner and
predictor against the oracle, the slot protocol on a host-only context, budget accounting."""
import itertools
import json
import os
import random
import re

import numpy as np
import pytest

from oracle import planner as P
from paper_2605_11678_amd import binding as B
from paper_2605_11678_amd import build, configs as CFG
from paper_2605_11678_amd.harness import Engine, desc_fields
from tests.des_sim import simulate

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_values.json")))


@pytest.fixture(scope="module", autouse=True)
def _built():
    build.ensure_built()


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "demand_layering.h")).read()
    names = set(re.findall(r"\b(dl_[a-z_0-9]+)\s*\(", hdr))
    assert len(names) >= 30
    lib = B.lib()
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert names == set(B.SIGNATURES), names ^ set(B.SIGNATURES)


def tiny_weights(c, rng):
    def gen(l):
        return {tid: rng.integers(0, 2 ** 16, size=shape, dtype=np.uint16) for tid, shape, _ in CFG.layer_tensors(c)}
    return gen


def small_cfg(n_layers=4, **kw):
    c = CFG.tiny_decoder()
    c.n_layers = n_layers
    c.vocab = 0
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_packed_layer_sizes_match_paper():
    eng = Engine(1 << 40, device=-1)
    for c, want_mib in ((CFG.decoder_8b(n_layers=1), GOLD["layer_sizes_MiB"]["vlm"]),
                        (CFG.vit_encoder(n_layers=1), GOLD["layer_sizes_MiB"]["vit"])):
        c.vocab = 0
        mid = eng.ctx.module_create(**desc_fields(c, 16))
        packed, params = eng.ctx.module_layer_bytes(mid)
        assert params == 2 * CFG.layer_param_count(c)
        assert abs(params / 2 ** 20 - want_mib) < 0.05          # Sec. IV-D prints 368.0 and 29.1 (MiB)
        # sections are 256-byte aligned; the second FFN matrix pads its rows (K) to a multiple of 128 with zeros
        pad = 2 * c.d_model * ((-c.d_ff) % 128)
        assert params <= packed <= params + pad + 64 * 256
    eng.close()


def test_placement_matches_eq8():
    for L in (1, 4, 8, 27, 36):
        for k in range(0, L + 1):
            assert B.place_interleaved(L, k) == P.interleaved_placement(k, L)
    with pytest.raises(B.DLError):
        B.place_interleaved(4, 5)


def test_benefit_tables_and_limit():
    rnd = random.Random(3)
    for _ in range(50):
        c_dma, m = rnd.uniform(0.5, 12), rnd.uniform(20, 400)
        lo, hi = c_dma * rnd.uniform(0.05, 0.9), c_dma * rnd.uniform(1.1, 4)
        R = rnd.randint(1, 30)
        assert B.benefit(c_dma, m, [hi], [R]) == pytest.approx(P.benefit_exe_intensive(R, c_dma, m))
        assert B.benefit(c_dma, m, [lo], [R]) == pytest.approx(P.benefit_dma_intensive(R, c_dma, lo, m))
        assert B.benefit(c_dma, m, [hi, lo], [1, R]) == pytest.approx(P.benefit_hybrid(R, c_dma, lo, m))
    t7 = GOLD["table7_benefit_ms_per_MB"]
    assert B.benefit(10.9, 368.0, [16.6, 0.9], [1, 21]) == pytest.approx(t7["vlm"], abs=1e-3)
    assert B.benefit(3.6, 120.8, [1.0], [10]) == pytest.approx(t7["expert"], abs=1e-3)
    assert B.benefit(0.9, 29.1, [8.3], [1]) == pytest.approx(t7["vit"], abs=1e-3)
    assert B.consecutive_limit(10.9, 0.9) == P.consecutive_residency_limit(10.9, 0.9) == 12


def test_predict_linear_table8():
    t8 = GOLD["table8_prediction"]
    for row in t8["rows"]:
        got = B.predict_linear(t8["C_total_0_s"] * 1e3, -t8["slope_ms_per_layer"], row["k"]) / 1e3
        assert abs(got - row["predicted_s"]) < 6e-4


def _flatten(invocations):
    dma, exe, st, ps = [], [], [], []
    for layers in invocations:
        for i, (d, e, s) in enumerate(layers):
            dma.append(d), exe.append(e), st.append(s), ps.append(i == 0)
    return dma, exe, st, ps


@pytest.mark.parametrize("wrap", [0, 1])
def test_timeline_matches_oracle_recurrence(wrap):
    rnd = random.Random(11)
    for trial in range(200):
        L = rnd.randint(1, 7)
        n_pass = rnd.randint(1, 4)
        mask = [rnd.random() < 0.6 for _ in range(L)]
        dma = [rnd.uniform(0.1, 5) for _ in range(L)]
        inv = [[(dma[i], rnd.uniform(0.1, 5), mask[i]) for i in range(L)] for _ in range(n_pass)]
        want = P.timeline(inv, wrap_prefetch=bool(wrap))
        got = B.timeline(*_flatten(inv), wrap_prefetch=wrap)
        assert got["total"] == pytest.approx(want["total"], rel=1e-12)
        assert got["exposed"] == pytest.approx(want["exposed"], rel=1e-9, abs=1e-12)
        assert got["hidden"] == pytest.approx(want["hidden"], rel=1e-9, abs=1e-12)
        seq = B.timeline(*_flatten(inv), mode=B.DL_MODE_SEQUENTIAL)
        assert seq["total"] == pytest.approx(P.sequential_time(inv), rel=1e-12)


def _flatten5(invocations):
    dma, exe, st, ps, idle, fence = [], [], [], [], [], []
    for layers in invocations:
        for i, (d, e, s, ei, f) in enumerate(layers):
            dma.append(d), exe.append(e), st.append(s), ps.append(i == 0), idle.append(ei), fence.append(f)
    return (dma, exe, st, ps), dict(c_exe_idle_ms=idle, c_fence_ms=fence)


@pytest.mark.parametrize("wrap", [0, 1])
def test_timeline_with_measured_corrections_matches_oracle(wrap):
    """idle-execution time, per-streamed-layer fence cost and per-layer overhead: library replay vs the
    oracle's recurrence on random schedules"""
    rnd = random.Random(23)
    for trial in range(200):
        L = rnd.randint(1, 7)
        n_pass = rnd.randint(1, 4)
        mask = [rnd.random() < 0.6 for _ in range(L)]
        inv = [[(rnd.uniform(0.1, 5), rnd.uniform(0.1, 5), mask[i], rnd.uniform(0.1, 6), rnd.uniform(0, 0.5))
                for i in range(L)] for _ in range(n_pass)]
        ov = rnd.choice([0.0, 0.07])
        pos, kw = _flatten5(inv)
        want = P.timeline(inv, wrap_prefetch=bool(wrap), overhead=ov)
        got = B.timeline(*pos, wrap_prefetch=wrap, overhead_ms=ov, **kw)
        assert got["total"] == pytest.approx(want["total"], rel=1e-12)
        assert got["exposed"] == pytest.approx(want["exposed"], rel=1e-9, abs=1e-12)
        seq = B.timeline(*pos, mode=B.DL_MODE_SEQUENTIAL, overhead_ms=ov, **kw)
        assert seq["total"] == pytest.approx(P.sequential_time(inv, overhead=ov), rel=1e-12)


def test_timeline_copy_trains_take_the_continuous_copy_time():
    """c_dma_cont_ms applies to a copy exactly when the copy queue did not wait since the previous copy ended:
    closed forms for the two regimes of Sec. IV-C, and NULL / equal arrays change nothing"""
    L = 9
    st, ps = [True] * L, [i == 0 for i in range(L)]
    # copy-bound (C_DMA > C_EXE, two slots): every copy after the first follows its predecessor at once
    d, dc, e = 4.0, 3.5, 1.0
    got = B.timeline([d] * L, [e] * L, st, ps, c_dma_cont_ms=[dc] * L)
    assert got["total"] == pytest.approx(d + (L - 1) * dc + e)
    # execution-bound: the first two copies form a train, every later one waits for its slot to be released
    d, dc, e = 1.0, 0.6, 5.0
    got = B.timeline([d] * L, [e] * L, st, ps, c_dma_cont_ms=[dc] * L)
    assert got["total"] == pytest.approx(d + L * e)
    assert got["exposed"] == pytest.approx(d)
    # one slot: a copy always waits for the execution before it, so no copy is part of a train
    got = B.timeline([4.0] * L, [1.0] * L, st, ps, c_dma_cont_ms=[3.5] * L, n_slots=1)
    assert got["total"] == pytest.approx(L * 5.0)
    # sequential mode never forms trains either
    got = B.timeline([4.0] * L, [1.0] * L, st, ps, c_dma_cont_ms=[3.5] * L, mode=B.DL_MODE_SEQUENTIAL)
    assert got["total"] == pytest.approx(L * 5.0)
    # per-invocation values: the train time used is the one of the copy that runs, not of its predecessor
    dma = [4.0, 5.0, 6.0]
    cont = [0.1, 4.5, 5.5]
    got = B.timeline(dma, [1.0] * 3, [True] * 3, [True, False, False], c_dma_cont_ms=cont)
    assert got["total"] == pytest.approx(4.0 + 4.5 + 5.5 + 1.0)
    # a resident layer between streamed ones does not break a train on the copy queue
    got = B.timeline([4.0] * 4, [1.0] * 4, [True, False, True, True], [True, False, False, False], c_dma_cont_ms=[3.0] * 4)
    assert got["total"] == pytest.approx(4.0 + 3.0 + 3.0 + 1.0)
    rnd = random.Random(5)
    for trial in range(100):
        n = rnd.randint(1, 8)
        dma = [rnd.uniform(0.1, 5) for _ in range(n)]
        exe = [rnd.uniform(0.1, 5) for _ in range(n)]
        mask = [rnd.random() < 0.7 for _ in range(n)]
        ps = [i == 0 for i in range(n)]
        base = B.timeline(dma, exe, mask, ps, wrap_prefetch=trial % 2)
        same = B.timeline(dma, exe, mask, ps, wrap_prefetch=trial % 2, c_dma_cont_ms=list(dma))
        assert base == same
        faster = B.timeline(dma, exe, mask, ps, wrap_prefetch=trial % 2, c_dma_cont_ms=[0.8 * v for v in dma])
        assert faster["total"] <= base["total"] + 1e-12
        assert faster["total"] >= B.timeline([0.8 * v for v in dma], exe, mask, ps, wrap_prefetch=trial % 2)["total"] - 1e-12


def test_timeline_hand_off_cost_depends_on_whether_the_copy_was_exposed():
    """c_fence_hot_ms is charged to a streamed layer whose copy was complete when the compute queue reached it,
    c_fence_ms to one the queue had to wait for; NULL keeps one figure for both."""
    L = 8
    st, ps = [True] * L, [i == 0 for i in range(L)]
    f, fh = 0.3, 0.1
    # execution-bound (two slots): only the first layer waits for its copy
    d, e = 1.0, 5.0
    got = B.timeline([d] * L, [e] * L, st, ps, c_fence_ms=[f] * L, c_fence_hot_ms=[fh] * L)
    assert got["total"] == pytest.approx(d + L * e + f + (L - 1) * fh)
    # copy-bound: every layer waits for its copy
    d, e = 4.0, 1.0
    got = B.timeline([d] * L, [e] * L, st, ps, c_fence_ms=[f] * L, c_fence_hot_ms=[fh] * L)
    assert got["total"] == pytest.approx(L * d + e + f)
    # resident layers carry neither
    got = B.timeline([d] * L, [e] * L, [False] * L, ps, c_fence_ms=[f] * L, c_fence_hot_ms=[fh] * L)
    assert got["total"] == pytest.approx(L * e)
    # without the second array the first one is used throughout (the oracle's recurrence)
    a = B.timeline([1.0] * L, [5.0] * L, st, ps, c_fence_ms=[f] * L)
    b = B.timeline([1.0] * L, [5.0] * L, st, ps, c_fence_ms=[f] * L, c_fence_hot_ms=[f] * L)
    assert a == b and a["total"] == pytest.approx(1.0 + L * 5.0 + L * f)


def test_timeline_execution_slows_down_under_a_copy():
    """c_exe_loaded_ms: an execution advances at c_exe / c_exe_loaded while a copy is in flight.  Closed forms for
    the execution-bound and the copy-bound pass, partial overlap, and no effect without copies or with equal arrays."""
    L = 6
    st, ps = [True] * L, [i == 0 for i in range(L)]
    # execution-bound, two slots: every layer but the last runs next to the whole copy of its successor (1.0 of wall
    # time does 1 / 1.2 of work), the last one next to none
    d, e, k = 1.0, 5.0, 1.2
    got = B.timeline([d] * L, [e] * L, st, ps, c_exe_loaded_ms=[k * e] * L)
    assert got["total"] == pytest.approx(d + (L - 1) * (e + d * (1 - 1 / k)) + e)
    # copy-bound: a layer runs entirely under the next copy (e * k < d), the last one alone
    d, e = 4.0, 1.0
    got = B.timeline([d] * L, [e] * L, st, ps, c_exe_loaded_ms=[k * e] * L)
    assert got["total"] == pytest.approx(L * d + e)
    assert B.timeline([d] * 1, [e] * 1, [True], [True], c_exe_loaded_ms=[k * e])["total"] == pytest.approx(d + e)
    # a resident layer behind a streamed one runs under the copy of the streamed layer after it:
    # copies [0,2) and [2,4); layer 0 runs 2 -> 3.2 (1 of work under a copy), layer 1 (resident, 3 of work): 0.8 of wall
    # under the copy does 2/3 of work, the other 7/3 alone -> 6.3333; layer 2 alone
    got = B.timeline([2.0, 9.9, 2.0], [1.0, 3.0, 1.0], [True, False, True], [True, False, False],
                     c_exe_loaded_ms=[1.2, 3.6, 1.2])
    assert got["total"] == pytest.approx(3.2 + 0.8 + (3.0 - 0.8 / 1.2) + 1.0)
    # no copies: nothing changes; equal arrays: nothing changes
    a = B.timeline([d] * L, [e] * L, [False] * L, ps, c_exe_loaded_ms=[k * e] * L)
    assert a["total"] == pytest.approx(L * e)
    rnd = random.Random(9)
    for trial in range(60):
        n = rnd.randint(1, 8)
        dma = [rnd.uniform(0.1, 5) for _ in range(n)]
        exe = [rnd.uniform(0.1, 5) for _ in range(n)]
        mask = [rnd.random() < 0.7 for _ in range(n)]
        p2 = [i == 0 for i in range(n)]
        base = B.timeline(dma, exe, mask, p2)
        assert B.timeline(dma, exe, mask, p2, c_exe_loaded_ms=list(exe)) == base
        slower = B.timeline(dma, exe, mask, p2, c_exe_loaded_ms=[1.3 * v for v in exe])
        assert base["total"] - 1e-12 <= slower["total"] <= B.timeline(dma, [1.3 * v for v in exe], mask, p2)["total"] + 1e-12


def test_timeline_closed_forms_eq5_eq6_eq7():
    L, R = 36, 21
    uni = lambda d, e: [(d, e, True)] * L
    assert B.timeline(*_flatten([uni(0.9, 8.3)]))["total"] == pytest.approx(P.module_time_exe_intensive(1, L, 0.9, 8.3))
    assert B.timeline(*_flatten([uni(3.6, 1.0)] * 10))["total"] == pytest.approx(P.module_time_dma_intensive(10, L, 3.6, 1.0))
    hyb = [uni(10.9, 16.6)] + [uni(10.9, 0.9)] * R
    assert B.timeline(*_flatten(hyb))["total"] == pytest.approx(P.module_time_hybrid(R, L, 10.9, 16.6, 0.9))


def _host_engine_with_module(c, cap=1 << 34, max_tokens=8):
    eng = Engine(cap, device=-1)
    rng = np.random.default_rng(0)
    mid = eng.add_module(c, max_tokens, weights=tiny_weights(c, rng))
    return eng, mid


def _ops_for_des(trace, dma, exe):
    ops = []
    for o in trace:
        q = "compute" if o["queue"] == 0 else "copy"
        if o["op"] == B.DL_OP_WAIT:
            ops.append((q, ("wait", (o["event_kind"], o["slot"]))))
        elif o["op"] == B.DL_OP_RECORD:
            ops.append((q, ("record", (o["event_kind"], o["slot"]))))
        elif o["op"] == B.DL_OP_COPY:
            ops.append((q, ("copy", dma[o["layer"]], o)))
        else:
            ops.append((q, ("exec", exe[o["layer"]], o)))
    return ops


@pytest.mark.parametrize("n_slots", [2, 1, 3, 4])
@pytest.mark.parametrize("wrap", [0, 1])
def test_slot_protocol_on_recorded_schedule_all_residency_sets(wrap, n_slots):
    """The schedule dl_forward enqueues (recorded by a host-only context) is replayed on an independent
    two-queue simulator: a layer never executes before its copy ended, a slot is never overwritten while
    the layer that used it is still running (Sec. IV-C(ii)), and the end time equals both predictors."""
    rnd = random.Random(5)
    for L in (1, 2, 3, 5, 6):
        c = small_cfg(L)
        eng, mid = _host_engine_with_module(c)
        eng.ctx.set_mode(B.DL_MODE_PIPELINED, wrap)
        eng.ctx.set_slot_count(n_slots)
        dma = [rnd.uniform(0.2, 4) for _ in range(L)]
        exe = [rnd.uniform(0.2, 4) for _ in range(L)]
        for mask in itertools.product([0, 1], repeat=L):
            resident = [i for i in range(L) if mask[i]]
            eng.ctx.set_residency(mid, resident)
            assert eng.ctx.get_residency(mid, L) == resident
            n_pass = 3
            for _ in range(n_pass):
                eng.ctx.forward(mid, 0, 0, 1, 0)
            trace = eng.ctx.trace_read()
            execs = [o for o in trace if o["op"] == B.DL_OP_EXEC]
            assert [o["layer"] for o in execs] == list(range(L)) * n_pass
            for o in execs:
                assert (o["slot"] < 0) == (o["layer"] in resident)
                assert o["slot"] < n_slots
            ops = _ops_for_des(trace, dma, exe)
            times = simulate(ops)
            # safety: pair every streamed exec with the last copy into its slot
            last_copy = {}
            busy_until = {s: 0.0 for s in range(4)}
            for (q, op), (t0, t1) in zip(ops, times):
                if op[0] == "copy":
                    s = op[2]["slot"]
                    assert t0 >= busy_until[s] - 1e-12, "slot overwritten while in use"
                    last_copy[s] = (op[2]["layer"], t1)
                elif op[0] == "exec" and op[2]["slot"] >= 0:
                    s = op[2]["slot"]
                    assert last_copy[s][0] == op[2]["layer"], "layer executed from a slot holding another layer"
                    assert t0 >= last_copy[s][1] - 1e-12, "layer executed before its parameters arrived"
                    busy_until[s] = t1
            total = max(t1 for (q, op), (t0, t1) in zip(ops, times) if q == "compute")
            inv = [[(dma[i], exe[i], not mask[i]) for i in range(L)]] * n_pass
            assert total == pytest.approx(P.timeline(inv, wrap_prefetch=bool(wrap), n_slots=n_slots)["total"], rel=1e-12)
            assert total == pytest.approx(B.timeline(*_flatten(inv), wrap_prefetch=wrap, n_slots=n_slots)["total"], rel=1e-12)
        eng.close()


def test_sequential_schedule_never_overlaps():
    L = 4
    c = small_cfg(L)
    eng, mid = _host_engine_with_module(c)
    eng.ctx.set_mode(B.DL_MODE_SEQUENTIAL, 0)
    eng.ctx.set_residency(mid, [1])
    for _ in range(2):
        eng.ctx.forward(mid, 0, 0, 1, 0)
    trace = eng.ctx.trace_read()
    dma, exe = [1.0, 2.0, 3.0, 4.0], [0.5, 0.25, 0.125, 1.5]
    ops = _ops_for_des(trace, dma, exe)
    times = simulate(ops)
    spans = sorted((t0, t1) for (q, op), (t0, t1) in zip(ops, times) if op[0] in ("copy", "exec"))
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert b0 >= a1 - 1e-12
    assert spans[-1][1] == pytest.approx(2 * (sum(exe) + dma[0] + dma[2] + dma[3]))
    eng.close()


def test_budget_two_slots_plus_one_resident_layer():
    """Tiny-decoder budget: room for the workspace, the KV cache, two slots and ONE resident layer."""
    c = small_cfg(4)
    probe, mid = _host_engine_with_module(c, cap=1 << 30, max_tokens=128)
    packed, _ = probe.ctx.module_layer_bytes(mid)
    base = probe.ctx.arena_stats()["used"]          # workspace + KV cache + two slots
    probe.close()
    eng, mid = _host_engine_with_module(c, cap=base + packed + 256, max_tokens=128)
    eng.ctx.set_residency(mid, [0])
    used1 = eng.ctx.arena_stats()["used"]
    assert used1 == base + packed
    with pytest.raises(B.DLError) as e:
        eng.ctx.set_residency(mid, [0, 2])
    assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
    # the failed call changed nothing
    assert eng.ctx.get_residency(mid, 4) == [0] and eng.ctx.arena_stats()["used"] == used1
    eng.ctx.set_residency(mid, [3])
    assert eng.ctx.get_residency(mid, 4) == [3] and eng.ctx.arena_stats()["used"] == used1
    eng.ctx.set_residency(mid, [])
    assert eng.ctx.arena_stats()["used"] == base
    eng.close()


def test_shrinking_the_workspace_makes_room_for_a_resident_layer():
    """Sec. IV-D: activations and parameters share one memory.  A workspace sized for the prefill, shrunk to the
    single-token passes that follow, frees what one more resident layer needs; growing it back is refused while
    that layer is resident, and the refusal changes nothing."""
    c = small_cfg(4, d_ff=1024, max_seq=640)
    probe, mid = _host_engine_with_module(c, cap=1 << 30, max_tokens=512)
    packed, _ = probe.ctx.module_layer_bytes(mid)
    base_long = probe.ctx.arena_stats()["used"]     # workspace for 512 tokens + KV cache + two slots
    probe.ctx.module_set_max_tokens(mid, 1)
    base_short = probe.ctx.arena_stats()["used"]
    probe.close()
    freed = base_long - base_short
    assert freed > packed                           # the long workspace is worth more than a layer here
    # room for ONE resident layer next to the long workspace
    eng, mid = _host_engine_with_module(c, cap=base_long + packed + 256, max_tokens=512)
    eng.ctx.forward(mid, 0, 0, 512, 0)              # a long pass is accepted ...
    with pytest.raises(B.DLError) as e:
        eng.ctx.set_residency(mid, [0, 2])
    assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
    eng.ctx.module_set_max_tokens(mid, 1)
    assert eng.ctx.arena_stats()["used"] == base_short
    eng.ctx.set_residency(mid, [0, 2])              # ... and after the shrink a second layer fits
    used2 = eng.ctx.arena_stats()["used"]
    assert used2 == base_short + 2 * packed
    eng.ctx.forward(mid, 0, 0, 1, 512)
    with pytest.raises(B.DLError) as e:
        eng.ctx.forward(mid, 0, 0, 2, 0)            # longer passes are refused now
    assert e.value.code == B.DL_ERR_INVALID_ARG
    with pytest.raises(B.DLError) as e:
        eng.ctx.module_set_max_tokens(mid, 512)     # no room to grow back while two layers are resident
    assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
    assert eng.ctx.arena_stats()["used"] == used2 and eng.ctx.get_residency(mid, 4) == [0, 2]
    eng.ctx.forward(mid, 0, 0, 1, 513)              # still works as before the refused call
    eng.ctx.set_residency(mid, [])                  # release first: the grown block then finds one free range
    eng.ctx.module_set_max_tokens(mid, 512)
    eng.ctx.set_residency(mid, [0])
    assert eng.ctx.arena_stats()["used"] == base_long + packed
    for bad in (0, 641):                            # below one token, beyond the KV cache
        with pytest.raises(B.DLError) as e:
            eng.ctx.module_set_max_tokens(mid, bad)
        assert e.value.code == B.DL_ERR_INVALID_ARG
    eng.close()


def test_all_resident_releases_slots_and_bigger_module_resizes_them():
    c = small_cfg(3)
    eng, mid = _host_engine_with_module(c, cap=1 << 30)
    packed, _ = eng.ctx.module_layer_bytes(mid)
    base = eng.ctx.arena_stats()["used"]
    eng.ctx.set_residency(mid, [0, 1, 2])
    assert eng.ctx.arena_stats()["used"] == base - 2 * packed + 3 * packed
    eng.ctx.forward(mid, 0, 0, 1, 0)
    assert all(o["op"] in (B.DL_OP_EXEC, B.DL_OP_RECORD) and o["queue"] == 0 for o in eng.ctx.trace_read())
    eng.ctx.set_residency(mid, [])
    assert eng.ctx.arena_stats()["used"] == base
    big = small_cfg(2, d_ff=1536)
    rng = np.random.default_rng(1)
    mid2 = eng.add_module(big, 8, weights=tiny_weights(big, rng))
    packed2, _ = eng.ctx.module_layer_bytes(mid2)
    assert packed2 > packed
    ws_kv2 = eng.ctx.arena_stats()["used"] - base - 2 * (packed2 - packed)
    assert ws_kv2 > 0            # slots grew to the largest layer over all modules (2 x M_max), plus module 2's workspace
    eng.close()


def test_one_slot_gives_a_layer_back_and_only_overlaps_resident_layers():
    c = small_cfg(4)
    eng, mid = _host_engine_with_module(c, cap=1 << 30)
    packed, _ = eng.ctx.module_layer_bytes(mid)
    used2 = eng.ctx.arena_stats()["used"]
    eng.ctx.set_slot_count(1)
    assert eng.ctx.arena_stats()["used"] == used2 - packed
    # all streamed through one slot: copy j+1 cannot start before layer j has executed, so nothing overlaps
    dma, exe = [3.0, 1.0, 2.0, 5.0], [0.5, 0.25, 1.5, 1.0]
    inv = [[(dma[i], exe[i], True) for i in range(4)]]
    assert B.timeline(*_flatten(inv), n_slots=1)["total"] == pytest.approx(sum(dma) + sum(exe))
    assert P.timeline(inv, n_slots=1)["total"] == pytest.approx(sum(dma) + sum(exe))
    # layers 1 and 2 resident: the copy of layer 3 overlaps their execution
    inv = [[(dma[0], exe[0], True), (9.0, exe[1], False), (9.0, exe[2], False), (dma[3], exe[3], True)]]
    want = dma[0] + exe[0] + max(dma[3], exe[1] + exe[2]) + exe[3]
    assert B.timeline(*_flatten(inv), n_slots=1)["total"] == pytest.approx(want)
    assert P.timeline(inv, n_slots=1)["total"] == pytest.approx(want)
    eng.ctx.set_slot_count(2)
    assert eng.ctx.arena_stats()["used"] == used2
    # three and four slots: one more layer of memory each (deeper prefetch)
    for n in (3, 4):
        eng.ctx.set_slot_count(n)
        assert eng.ctx.arena_stats()["used"] == used2 + (n - 2) * packed
    eng.ctx.set_slot_count(2)
    for bad in (0, 5):
        with pytest.raises(B.DLError) as e:
            eng.ctx.set_slot_count(bad)
        assert e.value.code == B.DL_ERR_INVALID_ARG
    eng.close()


def test_fully_resident_module_does_not_size_the_slots():
    """Sec. IV-C(i) with several modules: the slot pair holds the largest layer that can still be copied into it."""
    small, big = small_cfg(3), small_cfg(2, d_ff=1536)
    eng, m_small = _host_engine_with_module(small, cap=1 << 30)
    p_small, _ = eng.ctx.module_layer_bytes(m_small)
    rng = np.random.default_rng(1)
    m_big = eng.add_module(big, 8, weights=tiny_weights(big, rng))
    p_big, _ = eng.ctx.module_layer_bytes(m_big)
    assert p_big > p_small
    used_all_streamed = eng.ctx.arena_stats()["used"]
    fixed = used_all_streamed - 2 * p_big                      # workspaces and KV caches of both modules
    # the big module fully resident: its two copies, and the pair shrinks to the small module's layers
    eng.ctx.set_residency(m_big, [0, 1])
    assert eng.ctx.arena_stats()["used"] == fixed + 2 * p_big + 2 * p_small
    eng.ctx.trace_read()                                       # drop what has been recorded so far
    eng.ctx.forward(m_small, 0, 0, 1, 0)                       # still streams, through the smaller slots
    assert sum(o["op"] == B.DL_OP_COPY for o in eng.ctx.trace_read()) == 3
    eng.ctx.forward(m_big, 0, 0, 1, 0)
    # one layer of the big module streams again: the pair grows back before anything else is placed
    eng.ctx.set_residency(m_big, [1])
    assert eng.ctx.arena_stats()["used"] == fixed + p_big + 2 * p_big
    # both fully resident: no slots at all
    eng.ctx.set_residency(m_big, [0, 1])
    eng.ctx.set_residency(m_small, [0, 1, 2])
    assert eng.ctx.arena_stats()["used"] == fixed + 2 * p_big + 3 * p_small
    eng.close()


def _fits(k, L, M, budget, n_slots=2):
    return P.residency_bytes(k, L, M, n_slots) <= budget


def test_plan_shared_slots_against_exhaustive_search():
    rng = np.random.default_rng(5)
    for trial in range(60):
        n = int(rng.integers(1, 4))
        L = [int(rng.integers(1, 7)) for _ in range(n)]
        equal = trial % 2 == 0
        M = [4096 * int(rng.integers(1, 9))] * n if equal else [4096 * int(rng.integers(1, 9)) for _ in range(n)]
        b3 = []
        for _ in range(n):
            first = float(rng.uniform(0.0, 2.0))
            mid = first * float(rng.uniform(0.3, 1.0))
            b3.append([first, mid, mid * float(rng.uniform(0.0, 1.0))])
        total = sum(L[m] * M[m] for m in range(n))
        budget = int(rng.integers(2 * max(M), total + 2 * max(M) + 1))
        k = B.plan_shared_slots(L, M, b3, budget)
        assert all(0 <= k[m] <= L[m] for m in range(n)) and _fits(k, L, M, budget)
        v = sum(P.residency_value(k[m], L[m], M[m], b3[m]) for m in range(n))
        k_best, v_best = P.plan_shared_slots_exhaustive(L, M, b3, budget)
        assert v <= v_best + 1e-9
        if equal:
            # equal layer sizes: ranking by benefit per MiB is ranking by benefit, the greedy choice is optimal
            assert v == pytest.approx(v_best, rel=1e-12, abs=1e-12)
        # never worse than planning with the slots fixed at the largest layer of all modules
        k_fixed = B.plan(L, M, b3, budget - 2 * max(M))
        assert v >= sum(P.residency_value(k_fixed[m], L[m], M[m], b3[m]) for m in range(n)) - 1e-9


def test_plan_shared_slots_special_cases():
    M = 1 << 20
    b = [[1.0, 1.0, 0.5]]
    assert B.plan_shared_slots([10], [M], b, 10 * M) == [10]              # everything fits once the slots are gone
    assert B.plan_shared_slots([10], [M], b, 10 * M - 1) == [7]            # else two slots come off the budget
    assert B.plan_shared_slots([10], [M], b, 2 * M) == [0]
    with pytest.raises(B.DLError) as e:
        B.plan_shared_slots([10], [M], b, 2 * M - 1)
    assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
    # the module with the large layers goes fully resident and the pair shrinks to the small module's layers
    L, Ms, b3 = [4, 6], [1 * M, 8 * M], [[0.2, 0.2, 0.1], [1.0, 1.0, 0.9]]
    assert B.plan_shared_slots(L, Ms, b3, 6 * 8 * M + 2 * M + 1 * M) == [1, 6]
    assert B.plan(L, Ms, b3, 6 * 8 * M + 3 * M - 2 * 8 * M) == [3, 4]      # with fixed 2 x 8 MiB slots: two big layers less
    assert B.plan_shared_slots(L, Ms, b3, 6 * 8 * M + 4 * M) == [4, 6]     # everything resident, no slots
    # a benefit of zero buys nothing
    assert B.plan_shared_slots([3], [M], [[0.0, 0.0, 0.0]], 100 * M) == [0]


def test_error_paths():
    c = small_cfg(2)
    eng = Engine(1 << 30, device=-1)
    mid = eng.ctx.module_create(**desc_fields(c, 8))
    with pytest.raises(B.DLError) as e:
        eng.ctx.forward(mid, 0, 0, 1, 0)
    assert e.value.code == B.DL_ERR_BAD_STATE
    with pytest.raises(B.DLError) as e:
        eng.ctx.module_finalize(mid)           # tensors missing
    assert e.value.code == B.DL_ERR_BAD_STATE
    rng = np.random.default_rng(2)
    w = tiny_weights(c, rng)
    with pytest.raises(B.DLError) as e:
        eng.ctx.layer_set_tensor(mid, 0, CFG.T_WQ, np.zeros(7, np.uint16))      # wrong size
    assert e.value.code == B.DL_ERR_INVALID_ARG
    with pytest.raises(B.DLError):
        eng.ctx.layer_set_tensor(mid, 0, CFG.T_BQ, np.zeros(256, np.uint16))    # tensor the module does not have
    with pytest.raises(B.DLError):
        eng.ctx.layer_set_tensor(mid, 5, CFG.T_WQ, np.zeros(256 * 256, np.uint16))
    for l in range(2):
        for tid, arr in w(l).items():
            eng.ctx.layer_set_tensor(mid, l, tid, arr.reshape(-1))
    eng.ctx.module_finalize(mid)
    for bad in ([2], [-1], [0, 0]):
        with pytest.raises(B.DLError) as e:
            eng.ctx.set_residency(mid, bad)
        assert e.value.code == B.DL_ERR_INVALID_ARG
    with pytest.raises(B.DLError):
        eng.ctx.forward(mid, 0, 0, 9, 0)       # more tokens than max_tokens
    with pytest.raises(B.DLError):
        eng.ctx.forward(mid, 0, 0, 1, 160)     # beyond max_seq
    with pytest.raises(B.DLError):
        eng.ctx.module_create(**desc_fields(small_cfg(2, d_head=12), 8))
    eng.close()
    # a slot pair that does not fit the arena is refused at finalize, and nothing stays allocated
    small = Engine(600_000, device=-1)
    mid = small.ctx.module_create(**desc_fields(c, 8))
    for l in range(2):
        for tid, arr in w(l).items():
            small.ctx.layer_set_tensor(mid, l, tid, arr.reshape(-1))
    with pytest.raises(B.DLError) as e:
        small.ctx.module_finalize(mid)
    assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED and small.ctx.arena_stats()["used"] == 0
    small.close()


def test_plan_follows_benefit_ranking():
    t7 = GOLD["table7_benefit_ms_per_MB"]
    MiB = 1 << 20
    n_layers = [27, 36, 36]
    sizes = [int(29.1 * MiB), int(368.0 * MiB), int(120.8 * MiB)]
    b3 = [t7["vit"], t7["vlm"], t7["expert"]]
    # Sec. IV-D: with the RTX 5070 Ti numbers the budget goes to VLM layers only
    assert B.plan(n_layers, sizes, b3, 28 * sizes[1] + 1000) == [0, 28, 0]
    # an unlimited budget takes everything that saves time: VLM, expert, and only the first ViT layer
    assert B.plan(n_layers, sizes, b3, 1 << 50) == [1, 36, 36]
    # budget runs out inside the VLM middle group
    assert B.plan(n_layers, sizes, b3, 10 * sizes[1]) == [0, 10, 0]
    # after all VLM layers, the expert layers come next (0.298 > 0.031)
    assert B.plan(n_layers, sizes, b3, 36 * sizes[1] + 5 * sizes[2] + 10) == [0, 36, 5]


def test_fits_by_bytes_means_accepted():
    """Sec. IV-D's budget as the library takes it: whatever is resident now, a residency whose resident copies plus
    the slots of the largest layer that still streams sum to at most dl_residency_budget is accepted (slots and
    resident copies are placed again when first-fit leaves holes), and one that needs a byte more is refused whole."""
    rnd = random.Random(11)
    cfgs = [small_cfg(5), small_cfg(3, d_ff=1536), small_cfg(6, d_ff=512)]
    probe = Engine(1 << 32, device=-1)
    rng = np.random.default_rng(3)
    sizes = []
    for c in cfgs:
        m = probe.add_module(c, 16, weights=tiny_weights(c, rng))
        sizes.append(probe.ctx.module_layer_bytes(m)[0])
    top_stack = (1 << 32) - probe.ctx.residency_budget()
    probe.close()
    Ls = [c.n_layers for c in cfgs]
    full = sum(L * s for L, s in zip(Ls, sizes))
    for n_slots in (2, 1, 3):
        cap = top_stack + full * 2 // 3 + 256 * rnd.randint(0, 4000)     # room for about two thirds of all layers
        eng = Engine(cap, device=-1)
        rng = np.random.default_rng(3)
        mods = [eng.add_module(c, 16, weights=tiny_weights(c, rng)) for c in cfgs]
        eng.ctx.set_slot_count(n_slots)
        xp = eng.ctx.arena_alloc(4096)                                    # a caller block joins the top stack
        budget = eng.ctx.residency_budget()
        assert budget == cap // 256 * 256 - top_stack - 4096
        cur = [[] for _ in cfgs]

        def need(res):
            stream = [sizes[m] for m in range(3) if len(res[m]) < Ls[m]]
            return sum(len(res[m]) * sizes[m] for m in range(3)) + (n_slots * max(stream) if stream else 0)
        accepted = refused = 0
        for step in range(300):
            m = rnd.randrange(3)
            new = sorted(rnd.sample(range(Ls[m]), rnd.randint(0, Ls[m])))
            trial = list(cur)
            trial[m] = new
            if need(trial) <= budget:
                eng.ctx.set_residency(mods[m], new)
                cur = trial
                accepted += 1
            else:
                used = eng.ctx.arena_stats()["used"]
                with pytest.raises(B.DLError) as e:
                    eng.ctx.set_residency(mods[m], new)
                assert e.value.code == B.DL_ERR_BUDGET_EXCEEDED
                assert eng.ctx.arena_stats()["used"] == used
                refused += 1
            assert [eng.ctx.get_residency(mods[i], Ls[i]) for i in range(3)] == cur
            assert eng.ctx.arena_stats()["used"] == top_stack + 4096 + need(cur)
            assert eng.ctx.residency_budget() == budget                   # nothing movable ever strands the top stack
        assert accepted > 50 and refused > 20, (accepted, refused)
        # the tightest fit: fill the budget to the last layer
        for m in range(3):
            eng.ctx.set_residency(mods[m], [])
        k = B.plan_shared_slots(Ls, sizes, [[1.0, 1.0, 0.5]] * 3, budget, n_slots)
        for m in range(3):
            eng.ctx.set_residency(mods[m], B.place_interleaved(Ls[m], k[m]))
        eng.ctx.arena_free(xp)
        eng.close()


def test_head_needs_the_final_norm_bias_of_a_layernorm_module():
    """A LayerNorm module whose final-norm bias was never set must be refused by the greedy head (the kernel would
    read it), as dl_final_norm refuses it."""
    c = CFG.ModuleConfig("ln_head", 1, 64, 2, 2, 32, 64, CFG.NORM_LN, CFG.ACT_GELU, 1, 0, 0.0, vocab=32)
    eng = Engine(1 << 26, device=-1)
    head = CFG.make_head(c)
    del head[CFG.R_FINAL_NORM_B]
    rng = np.random.default_rng(0)
    mid = eng.add_module(c, 4, weights=tiny_weights(c, rng), head=head)
    for call in (lambda: eng.ctx.logits_argmax(mid, 0), lambda: eng.ctx.greedy_step(mid, 0, 0, 0),
                 lambda: eng.ctx.final_norm(mid, 0, 0, 1)):
        with pytest.raises(B.DLError) as e:
            call()
        assert e.value.code == B.DL_ERR_BAD_STATE
    eng.ctx.set_resident_tensor(mid, CFG.R_FINAL_NORM_B, np.zeros(64, np.uint16))
    eng.ctx.logits_argmax(mid, 0)
    eng.close()


def test_kv_cache_module_limits_query_heads_per_kv_head():
    """The single-token attention kernel puts the query heads of one KV head on the 32 columns of an MFMA tile."""
    eng = Engine(1 << 26, device=-1)
    wide = small_cfg(1, n_q_heads=64, n_kv_heads=1, d_head=8, d_model=64)
    with pytest.raises(B.DLError) as e:
        eng.ctx.module_create(**desc_fields(wide, 8))
    assert e.value.code == B.DL_ERR_INVALID_ARG and "32 query heads" in str(e.value)
    wide.max_seq = 0                                   # without a cache (prefill kernels only) the shape is fine
    eng.ctx.module_create(**desc_fields(wide, 8))
    ok = small_cfg(1, n_q_heads=32, n_kv_heads=1, d_head=8, d_model=64)
    eng.ctx.module_create(**desc_fields(ok, 8))
    eng.close()


def test_module_whose_operands_would_pass_4_gb_is_refused():
    """The kernels address an operand (an activation matrix, one head's keys) with 32-bit byte offsets; a descriptor
    whose longest pass times its widest row does not fit them is refused when the module is created."""
    eng = Engine(1 << 26, device=-1)
    c = CFG.decoder_8b(n_layers=1, vocab=0)
    ok = desc_fields(c, 16384)
    ok["max_seq"] = 16384
    eng.ctx.module_create(**ok)                        # 16384 x 24576 x 4 B = 1.6 GB: fine
    too_long = dict(ok)
    too_long["max_seq"] = too_long["max_tokens"] = 65536
    with pytest.raises(B.DLError) as e:
        eng.ctx.module_create(**too_long)
    assert e.value.code == B.DL_ERR_INVALID_ARG and "4 GB" in str(e.value)
    eng.close()


def test_vla_infer_records_the_five_stages_and_checks_shapes():
    """dl_vla_infer on a host-only context: the recorded schedule is one encoder pass, one prefill pass, n_decode
    single-token passes and n_euler action passes, in that order; mismatching shapes are refused before anything is
    enqueued."""
    from tests import parity_cases as PC
    vit, dec, act = PC.pipe_small_modules()
    eng = Engine(1 << 30, device=-1)
    rng = np.random.default_rng(4)
    m_vit = eng.add_module(vit, 256, weights=tiny_weights(vit, rng))
    m_dec = eng.add_module(dec, 104, weights=tiny_weights(dec, rng))
    m_act = eng.add_module(act, 64, 104, weights=tiny_weights(act, rng))
    z = lambda *shape: np.zeros(shape, np.uint16)
    proj = eng.ctx.mlp_create(vit.d_model, dec.d_model, dec.d_model, z(dec.d_model, vit.d_model), z(dec.d_model),
                              z(dec.d_model, dec.d_model), z(dec.d_model), max_tokens=256)
    outp = eng.ctx.mlp_create(act.d_model, 0, 3, None, None, z(3, act.d_model), z(3), max_tokens=64)
    desc = dict(m_vit=m_vit, m_dec=m_dec, m_act=m_act, mlp_proj=proj, mlp_out=outp, n_patches=256, pool=4, n_text=40,
                n_actions=64, n_decode=3, n_euler=5, out_dim=3)
    bufs = {k: 0 for k, _ in B.dl_vla_buffers._fields_}
    eng.ctx.trace_read()
    eng.ctx.vla_infer(desc, bufs)
    execs = [(o["module"], o["layer"]) for o in eng.ctx.trace_read() if o["op"] == B.DL_OP_EXEC]
    want = [(m_vit, l) for l in range(vit.n_layers)] + [(m_dec, l) for l in range(dec.n_layers)] * (1 + 3) + \
           [(m_act, l) for l in range(act.n_layers)] * 5
    assert execs == want
    for bad in (dict(n_patches=255), dict(n_decode=100), dict(n_text=41), dict(mlp_out=proj), dict(out_dim=4),
                dict(n_euler=0), dict(m_act=m_vit)):
        with pytest.raises(B.DLError) as e:
            eng.ctx.vla_infer({**desc, **bad}, bufs)
        assert e.value.code == B.DL_ERR_INVALID_ARG, bad
        assert eng.ctx.trace_read() == []                    # nothing was enqueued
    eng.close()
