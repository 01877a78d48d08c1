#!/usr/bin/env python3
"""Benchmark of the pipelined Demand Layering hot path on one MI355X.

Workload (configs[2] of the task description): 8B-class decoder prefill — 36 layers, d=4096,
32 query / 8 KV heads x 128, SwiGLU 12288, RMSNorm, RoPE theta=1e6, 3072 tokens, batch 1, BF16
weights ~N(0,0.02) (seeded, synthetic), all device memory inside one 16e9-byte arena.

A "step" is one inference: one pass over all 36 layers (copies of the streamed layers on the copy
stream overlapped with compute, resident layers read in place), at the largest resident count the
arena holds.  Besides the contract line it reports a residency sweep with the predictor's error,
the fraction of transfer time hidden, achieved host-to-device GB/s, MFMA utilisation and the CPU
oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense BF16 MFMA
PEAK_HBM_GBPS = 8000.0
LINK_GBPS_THEORY = 63.0            # PCIe Gen5 x16 after 128b/130b


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class ClockSampler:
    """Samples the shader clock the driver reports (the starred level of pp_dpm_sclk) and the board power (hwmon
    power1_input, with its cap) on a host thread while a region runs; the paper locks clocks (Sec. V-A), an ordinary
    user on this machine cannot, so the observed clock and power are recorded next to the result instead."""

    def __init__(self, period_s=0.02):
        import glob
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.power_paths = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.period, self.samples, self.power, self._stop, self._th = period_s, [], [], False, None

    def _read_power(self):
        for p in self.power_paths:
            try:
                return float(open(p).read()) * 1e-6          # microwatts
            except Exception:
                pass
        return None

    def power_cap_w(self):
        for p in self.power_paths:
            try:
                return float(open(p.replace("power1_input", "power1_cap")).read()) * 1e-6
            except Exception:
                pass
        return None

    def _read(self):
        for p in self.paths:
            try:
                for line in open(p).read().splitlines():
                    if line.strip().endswith("*"):
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
            except Exception:
                pass
        return None

    def __enter__(self):
        import threading
        self._stop = False

        def loop():
            while not self._stop:
                v = self._read()
                if v is not None:
                    self.samples.append(v)
                w = self._read_power()
                if w is not None:
                    self.power.append(w)
                time.sleep(self.period)
        self._th = threading.Thread(target=loop, daemon=True)
        self._th.start()
        return self

    def __exit__(self, *a):
        self._stop = True
        self._th.join()

    def summary(self):
        if not self.samples:
            return None
        v = np.array(self.samples)
        out = {"sclk_mhz_median": float(np.median(v)), "sclk_mhz_min": float(v.min()), "sclk_mhz_max": float(v.max()),
               "samples": int(v.size), "source": "pp_dpm_sclk (current level), sampled on the host during the timed region"}
        if self.power:
            w = np.array(self.power)
            out.update({"power_w_median": float(np.median(w)), "power_w_max": float(w.max()),
                        "power_cap_w": self.power_cap_w(), "power_source": "hwmon power1_input / power1_cap"})
        return out


def decode_leg(eng, ctx, mid, c, T, L, xp, yp, packed, B, torch, log):
    """64 greedy steps at batch 1 after the T-token prefill.  Caps: the arena itself (16e9 B) and 12e9 B
    (emulated by parking a ballast block in the arena).  Policies: nothing resident; the largest count
    that fits placed by Eq. 8; the same count as the first k consecutive layers."""
    import numpy as np
    d = c.d_model
    tp, tv = eng.alloc_f32(64)
    # per-phase profile of the single-token pass (Table III's "VLM decode" row)
    ctx.set_residency(mid, [])
    prof = ctx.profile(mid, L, 1, T, xp, iters=3)
    c_dma = [p["c_dma_ms"] for p in prof]
    c_cont = [p["c_dma_cont_ms"] for p in prof]
    c_exe = [p["c_exe_ms"] for p in prof]
    c_hot = [p["c_exe_hot_ms"] for p in prof]
    c_fence = [p["c_fence_ms"] for p in prof]
    c_fhot = [p["c_fence_hot_ms"] for p in prof]
    c_load = [p["c_exe_loaded_ms"] for p in prof]
    res = {"profile": {"c_dma_ms": round(float(np.mean(c_dma)), 4), "c_dma_cont_ms": round(float(np.mean(c_cont)), 4),
                       "c_exe_ms": round(float(np.mean(c_exe)), 4),
                       "c_exe_hot_ms": round(float(np.mean(c_hot)), 4),
                       "r": round(float(np.mean(c_dma) / np.mean(c_exe)), 1),
                       "consecutive_limit": B.consecutive_limit(float(np.mean(c_dma)), float(np.mean(c_exe)))},
           "runs": []}

    # the greedy head (final norm, 4096x32768 GEMV, argmax, embedding row) runs once per token, always resident
    ctx.forward(mid, xp, yp, T, 0)
    ctx.sync()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(50):
        ctx.greedy_step(mid, yp, tp, xp + 4 * d)
    ctx.sync()
    head_ms = (time.perf_counter() - t) * 1e3 / 50
    res["head_ms"] = round(head_ms, 4)

    def run(resident, steps, wrap, shrink=False):
        ctx.set_mode(B.DL_MODE_PIPELINED, wrap)
        h_ptr = yp + 4 * (T - 1) * d
        if shrink:
            # the prefill streams everything under the long workspace; the single-token passes that follow need a
            # workspace for one token, and the difference goes to resident layers
            ctx.set_residency(mid, [])
            ctx.forward(mid, xp, yp, T, 0)
            ctx.greedy_step(mid, h_ptr, tp, xp + 4 * d)
            ctx.sync()
            ctx.module_set_max_tokens(mid, 1)
            ctx.set_residency(mid, resident)
        else:
            ctx.set_residency(mid, resident)
            ctx.forward(mid, xp, yp, T, 0)                   # refresh the KV cache (untimed)
            ctx.greedy_step(mid, h_ptr, tp, xp + 4 * d)      # next input lives behind row 0 so that xp's prefill rows stay intact
        ctx.forward(mid, xp + 4 * d, yp, 1, T)               # one untimed step: first-use effects stay out of the figure
        ctx.sync()
        # median over three groups of consecutive steps: the host link is shared with other tenants of the machine,
        # and one slow spell would otherwise decide a streamed figure
        samples, s = [], 0
        for _ in range(3):
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(steps // 3):
                ctx.forward(mid, xp + 4 * d, yp, 1, T + s)
                ctx.greedy_step(mid, yp, tp + 4 * ((s + 1) % 64), xp + 4 * d)
                s += 1
            ctx.sync()
            torch.cuda.synchronize()
            samples.append((time.perf_counter() - t) * 1e3 / (steps // 3))
        ms = float(np.median(samples))
        # per-layer statistics from a few more steps with timing events on (the event pairs cost ~7 us per layer,
        # 7 % of a resident single-token pass, so they stay out of the timed loop)
        ctx.set_timing(True)
        for s in range(min(steps, 4)):
            ctx.forward(mid, xp + 4 * d, yp, 1, T + s)
            ctx.greedy_step(mid, yp, tp + 4 * ((s + 1) % 64), xp + 4 * d)
        st = ctx.collect_stats()
        ctx.set_timing(False)
        return ms, st

    def predict(resident, steps, wrap, n_slots=2):
        rs = set(resident)
        streamed = [i not in rs for i in range(L)] * steps
        starts = [i == 0 for i in range(L)] * steps
        return B.timeline(c_dma * steps, c_hot * steps, streamed, starts, wrap_prefetch=wrap, n_slots=n_slots,
                          c_exe_idle_ms=c_exe * steps, c_fence_ms=c_fence * steps,
                          c_dma_cont_ms=c_cont * steps, c_fence_hot_ms=c_fhot * steps, c_exe_loaded_ms=c_load * steps)["total"] / steps + head_ms

    def fit_count():
        for k in range(L, -1, -1):
            try:
                ctx.set_residency(mid, B.place_interleaved(L, k))
                return k
            except B.DLError as e:
                if e.code != B.DL_ERR_BUDGET_EXCEEDED:
                    raise
        return 0

    for cap_name, ballast_bytes in (("16e9", 0), ("12e9", 4_000_000_000)):
        ctx.set_residency(mid, [])
        ballast = ctx.arena_alloc(ballast_bytes) if ballast_bytes else None
        try:
            kfit = fit_count()
            policies = [("none", [], 2, False), ("interleaved_eq8", B.place_interleaved(L, kfit), 2, False)]
            if 0 < kfit < L:
                policies.append(("first_k_consecutive", list(range(kfit)), 2, False))
                # a copy takes ~60 x longer than a single-token layer executes: the overlap a second slot buys is worth
                # less than the resident layer its memory holds
                ctx.set_residency(mid, [])
                ctx.set_slot_count(1)
                kfit1 = fit_count()
                ctx.set_residency(mid, [])
                ctx.set_slot_count(2)
                policies.append(("interleaved_eq8_one_slot", B.place_interleaved(L, kfit1), 1, False))
                # three slots (two copies ahead of the executing layer): one resident layer less; it can only pay where
                # the copy queue would otherwise wait for a slot, i.e. for runs of consecutive streamed layers whose
                # execution outlasts a copy - never in single-token passes, measured here for the record
                ctx.set_slot_count(3)
                kfit3 = fit_count()
                ctx.set_residency(mid, [])
                ctx.set_slot_count(2)
                policies.append(("interleaved_eq8_three_slots", B.place_interleaved(L, kfit3), 3, False))
                policies.append(("first_k_consecutive_three_slots", list(range(kfit3)), 3, False))
                # ... and with the activation workspace shrunk from the prefill's T tokens to one token
                ctx.set_slot_count(1)
                ctx.module_set_max_tokens(mid, 1)
                kfit1s = fit_count()
                ctx.set_residency(mid, [])
                ctx.module_set_max_tokens(mid, T)
                ctx.set_slot_count(2)
                if kfit1s > kfit1:
                    policies.append(("interleaved_eq8_one_slot_decode_workspace", B.place_interleaved(L, kfit1s), 1, True))
            for name, resident, n_slots, shrink in policies:
                streamed_n = L - len(resident)
                steps = 63 if streamed_n * float(np.mean(c_dma)) < 40 else 6        # three timed groups of steps / 3
                ctx.set_residency(mid, [])
                ctx.set_slot_count(n_slots)
                for wrap in ((0, 1) if streamed_n else (0,)):
                    try:
                        ms, st = run(resident, steps, wrap, shrink)
                        arena_used = ctx.arena_stats()["used"]
                    finally:
                        if shrink:
                            ctx.set_residency(mid, [])
                            ctx.module_set_max_tokens(mid, T)
                    pred = predict(resident, steps // 3, wrap, n_slots)
                    row = {"cap": cap_name, "policy": name, "k": len(resident), "slots": n_slots, "wrap_prefetch": wrap, "steps": steps,
                           "ms_per_token": round(ms, 3), "predicted_ms_per_token": round(pred, 3),
                           "pred_err_pct": round((pred - ms) / ms * 100, 2), "hidden_frac": round(st["hidden_frac"], 4),
                           "h2d_gbps": round(st["h2d_gbps"], 2),
                           "arena_gb": round(arena_used / 1e9 - ballast_bytes / 1e9, 3)}
                    if not streamed_n:
                        row["weight_stream_gbps"] = round(L * packed / (ms * 1e-3) / 1e9, 1)   # HBM-bound resident pass
                    res["runs"].append(row)
                    log("decode cap %s %-20s k=%2d wrap=%d: %.3f ms/token (predicted %.3f, %.2f%%) hidden %.3f" %
                        (cap_name, name, len(resident), wrap, ms, pred, row["pred_err_pct"], st["hidden_frac"]))
        finally:
            ctx.set_residency(mid, [])
            ctx.module_set_max_tokens(mid, T)
            ctx.set_slot_count(2)
            if ballast:
                ctx.arena_free(ballast)
    # the planner's choice per cap = the candidate (placement, slot count, prefetch setting) with the lowest PREDICTED
    # time, taken from the one profiling run above; reported next to what that candidate measured
    res["planner_choice"] = []
    for cap_name in ("16e9", "12e9"):
        cand = [r for r in res["runs"] if r["cap"] == cap_name and r["policy"].startswith("interleaved_eq8")]
        if cand:
            best = min(cand, key=lambda r: r["predicted_ms_per_token"])
            res["planner_choice"].append({k: best[k] for k in ("cap", "policy", "k", "slots", "wrap_prefetch",
                                                               "predicted_ms_per_token", "ms_per_token", "pred_err_pct")})
    return res


def vit_leg(B, CFG, Engine, torch, log):
    """configs[1]: 27-layer d=1152 encoder, 4096 tokens, bidirectional; two slots; residency sweep."""
    import numpy as np
    c = CFG.vit_encoder()
    T, L = 4096, c.n_layers
    eng = Engine(int(2e9), device=0)
    mid = eng.add_module(c, max_tokens=T)
    ctx = eng.ctx
    packed, params = ctx.module_layer_bytes(mid)
    x = CFG.make_tokens(T, c.d_model, seed=7)
    xp, xv = eng.alloc_f32(T * c.d_model)
    yp, yv = eng.alloc_f32(T * c.d_model)
    eng.upload(xv, x)
    tried = eng.pick_copy_stream(mid, T, xp, yp)
    log("vit copy-stream candidates (ms per fully streamed pass): " + ", ".join("%.2f" % t for _, t in tried))
    prof = ctx.profile(mid, L, T, 0, xp, iters=4)
    c_dma = [p["c_dma_ms"] for p in prof]
    c_cont = [p["c_dma_cont_ms"] for p in prof]
    c_exe = [p["c_exe_ms"] for p in prof]
    c_hot = [p["c_exe_hot_ms"] for p in prof]
    c_fence = [p["c_fence_ms"] for p in prof]
    c_fhot = [p["c_fence_hot_ms"] for p in prof]
    c_load = [p["c_exe_loaded_ms"] for p in prof]
    rows = []
    for k in (0, 7, 14, 20, 24, 27):
        res = B.place_interleaved(L, k)
        ctx.set_residency(mid, res)
        ctx.forward(mid, xp, yp, T, 0)
        ctx.sync()
        samples = []
        for _ in range(5):                                   # median of groups of back-to-back passes: the host link is shared
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(4):
                ctx.forward(mid, xp, yp, T, 0)
            ctx.sync()
            samples.append((time.perf_counter() - t) * 1e3 / 4)
        ms = float(np.median(samples))
        ctx.set_timing(True)
        ctx.forward(mid, xp, yp, T, 0)
        st = ctx.collect_stats()
        ctx.set_timing(False)
        rs = set(res)
        pred = B.timeline(c_dma, c_hot, [i not in rs for i in range(L)], [i == 0 for i in range(L)],
                          c_exe_idle_ms=c_exe, c_fence_ms=c_fence, c_dma_cont_ms=c_cont, c_fence_hot_ms=c_fhot, c_exe_loaded_ms=c_load)["total"]
        rows.append({"k": k, "measured_ms": round(ms, 3), "predicted_ms": round(pred, 3),
                     "pred_err_pct": round((pred - ms) / ms * 100, 2), "hidden_frac": round(st["hidden_frac"], 4),
                     "h2d_gbps": round(st["h2d_gbps"], 2)})
        log("vit k=%2d measured %.3f ms predicted %.3f ms (%.2f%%) hidden %.3f H2D %.1f GB/s" %
            (k, ms, pred, rows[-1]["pred_err_pct"], st["hidden_frac"], st["h2d_gbps"]))
    flops_layer = 2.0 * T * c.d_model * 3 * c.d_model + 2.0 * T * c.d_model * c.d_model + 4.0 * T * c.d_model * c.d_ff \
        + 4.0 * c.d_head * c.n_q_heads * float(T) * T
    # slot count x placement at a partial residency (r = C_DMA / C_EXE is closest to 1 for this module, so this is
    # where deeper prefetch or the placement could matter): 1 .. 4 slots, Eq. 8 placement against the first k layers
    slot_rows = []
    for k in (0, 14):
        for name, res in (("interleaved_eq8", B.place_interleaved(L, k)), ("first_k_consecutive", list(range(k)))):
            if k == 0 and name != "interleaved_eq8":
                continue
            for n_slots in (1, 2, 3, 4):
                ctx.set_residency(mid, [])
                ctx.set_slot_count(n_slots)
                ctx.set_residency(mid, res)
                ctx.forward(mid, xp, yp, T, 0)
                ctx.sync()
                samples = []
                for _ in range(5):
                    torch.cuda.synchronize()
                    t = time.perf_counter()
                    for _ in range(4):
                        ctx.forward(mid, xp, yp, T, 0)
                    ctx.sync()
                    samples.append((time.perf_counter() - t) * 1e3 / 4)
                ms = float(np.median(samples))
                rs = set(res)
                pred = B.timeline(c_dma, c_hot, [i not in rs for i in range(L)], [i == 0 for i in range(L)],
                                  c_exe_idle_ms=c_exe, c_fence_ms=c_fence, n_slots=n_slots, c_dma_cont_ms=c_cont, c_fence_hot_ms=c_fhot, c_exe_loaded_ms=c_load)["total"]
                slot_rows.append({"k": k, "placement": name, "slots": n_slots, "measured_ms": round(ms, 3),
                                  "predicted_ms": round(pred, 3), "pred_err_pct": round((pred - ms) / ms * 100, 2)})
                log("vit k=%2d %-20s slots=%d measured %.3f ms predicted %.3f ms" % (k, name, n_slots, ms, pred))
    ctx.set_residency(mid, [])
    ctx.set_slot_count(2)
    # per-kernel-class times of the fully resident pass
    ctx.set_residency(mid, list(range(L)))
    ctx.forward(mid, xp, yp, T, 0)
    ctx.set_kernel_timing(True)
    for _ in range(5):
        ctx.forward(mid, xp, yp, T, 0)
    kt = ctx.collect_kernel_times()
    ctx.set_kernel_timing(False)
    kernels = {k: {"us_per_layer": round(v["total_ms"] * 1e3 / v["launches"] * (2 if k == "norm" else 1), 2),
                   "tflops": round(v["flops"] / (v["total_ms"] * 1e-3) / 1e12, 1) if v["flops"] > 0 else None}
               for k, v in kt.items() if v["launches"]}
    resident_ms = rows[-1]["measured_ms"]
    out = {"workload": "configs[1]: 27-layer d=1152 encoder (16x72 heads, GELU MLP 4304, LayerNorm, biases), T=4096",
           "layer_bytes": packed, "kernels_resident_pass": kernels, "slots_x_placement": slot_rows,
           "roofline_ms_resident": round(flops_layer * L / (PEAK_BF16_TFLOPS * 1e9), 3),
           "roofline_frac_resident": round(flops_layer * L / (PEAK_BF16_TFLOPS * 1e9) / resident_ms, 4),
           "roofline_frac_streamed_k0": round(L * packed / (LINK_GBPS_THEORY * 1e6) / rows[0]["measured_ms"], 4),
           "profile": {"c_dma_ms": round(float(np.mean(c_dma)), 4), "c_dma_cont_ms": round(float(np.mean(c_cont)), 4),
                       "c_exe_ms": round(float(np.mean(c_exe)), 4),
                       "c_exe_hot_ms": round(float(np.mean(c_hot)), 4), "c_exe_loaded_ms": round(float(np.mean(c_load)), 4),
                       "c_fence_ms": round(float(np.mean(c_fence)), 4), "c_fence_hot_ms": round(float(np.mean(c_fhot)), 4),
                       "r": round(float(np.mean(c_dma) / np.mean(c_exe)), 2)},
           "sweep": rows, "layer_flop": flops_layer,
           "resident_tflops": round(flops_layer * L / (rows[-1]["measured_ms"] * 1e-3) / 1e12, 1)}
    eng.close()
    return out

def long_prefill_leg(B, CFG, Engine, torch, log, cap, which="decoder"):
    """The execution-intensive regime of Sec. IV-C (Eq. 5, Table IV) on this part: the 36-layer 8B-class decoder over
    a 16384-token prompt, or the 27-layer encoder over 8192 patches, where a layer executes for longer than its copy
    takes (at the paper's 3072 / 4096 tokens the copy takes 5.7x / 1.8x the execution, so most of it CANNOT be
    hidden).  Everything streamed, pipelined against sequential, the first layer resident, and the largest residency
    the arena holds; hidden fraction from the per-layer event records; predictor from one profiling run; streamed
    and partially resident outputs compared bit for bit on the device."""
    import numpy as np
    if which == "decoder":
        T = 16384
        c = CFG.decoder_8b(max_seq=T, vocab=0)
        name = "8B-class decoder prefill, 36 layers"
    else:
        T, cap = 8192, 2e9
        c = CFG.vit_encoder()
        name = "27-layer encoder"
    L = c.n_layers
    eng = Engine(int(cap), device=0)
    try:
        mid = eng.add_module(c, max_tokens=T)
        ctx = eng.ctx
        packed, _ = ctx.module_layer_bytes(mid)
        xp, xv = eng.alloc_f32(T * c.d_model)
        yp, yv = eng.alloc_f32(T * c.d_model)
        eng.upload(xv, CFG.make_tokens(T, c.d_model, seed=7))
        tried = eng.pick_copy_stream(mid, T, xp, yp, passes=1 if which == "decoder" else 3)
        log("long %s copy-stream candidates (ms per fully streamed pass): " % which + ", ".join("%.1f" % t for _, t in tried))
        prof = ctx.profile(mid, L, T, 0, xp, iters=2 if which == "decoder" else 4)
        col = lambda key: [p_[key] for p_ in prof]
        c_dma, c_cont, c_exe, c_hot, c_fence, c_fhot, c_load = (col(k_) for k_ in ("c_dma_ms", "c_dma_cont_ms", "c_exe_ms", "c_exe_hot_ms",
                                                                                  "c_fence_ms", "c_fence_hot_ms", "c_exe_loaded_ms"))
        pairs = T * (T + 1) / 2.0 if c.causal else float(T) * T
        ff = 6.0 if c.act == CFG.ACT_SWIGLU else 4.0
        flops_layer = 2.0 * T * c.d_model * (c.n_q_heads * c.d_head + 2 * c.n_kv_heads * c.d_head) \
            + 2.0 * T * c.d_model * c.n_q_heads * c.d_head + ff * T * c.d_model * c.d_ff \
            + 4.0 * c.d_head * c.n_q_heads * pairs
        roof_layer_ms = max(packed / (LINK_GBPS_THEORY * 1e6), flops_layer / (PEAK_BF16_TFLOPS * 1e9))

        def measure(k, mode):
            ctx.set_mode(mode, 0)
            ctx.set_residency(mid, B.place_interleaved(L, k))
            ctx.forward(mid, xp, yp, T, 0)
            ctx.sync()
            samples = []
            n_rep = 1 if which == "decoder" else 4
            for _ in range(5):
                torch.cuda.synchronize()
                t = time.perf_counter()
                for _ in range(n_rep):
                    ctx.forward(mid, xp, yp, T, 0)
                ctx.sync()
                samples.append((time.perf_counter() - t) * 1e3 / n_rep)
            ctx.set_timing(True)
            ctx.forward(mid, xp, yp, T, 0)
            st = ctx.collect_stats()
            ctx.set_timing(False)
            rs = set(B.place_interleaved(L, k))
            pred = B.timeline(c_dma, c_hot, [i not in rs for i in range(L)], [i == 0 for i in range(L)], mode=mode,
                              c_exe_idle_ms=c_exe, c_fence_ms=c_fence, c_dma_cont_ms=c_cont, c_fence_hot_ms=c_fhot, c_exe_loaded_ms=c_load)["total"]
            ms = float(np.median(samples))
            return {"k": k, "mode": "sequential" if mode == B.DL_MODE_SEQUENTIAL else "pipelined",
                    "measured_ms": round(ms, 2), "predicted_ms": round(pred, 2), "pred_err_pct": round((pred - ms) / ms * 100, 2),
                    "hidden_frac": round(st["hidden_frac"], 4), "h2d_gbps": round(st["h2d_gbps"], 2),
                    "roofline_frac": round(roof_layer_ms * L / ms, 4), "arena_gb": round(ctx.arena_stats()["used"] / 1e9, 3)}

        rows = [measure(0, B.DL_MODE_SEQUENTIAL), measure(0, B.DL_MODE_PIPELINED)]
        ctx.sync()
        torch.cuda.synchronize()
        ref = yv.clone()
        k_fit = 0
        for k in range(L, 0, -1):
            try:
                ctx.set_residency(mid, B.place_interleaved(L, k))
                k_fit = k
                break
            except B.DLError as e:
                if e.code != B.DL_ERR_BUDGET_EXCEEDED:
                    raise
        identical = None
        # Table IV (execution-intensive): only the first layer's copy is exposed, so making it resident saves one
        # C_DMA and any further resident layer saves nothing but its hand-offs
        rows.append(measure(1, B.DL_MODE_PIPELINED))
        b3 = B.benefit(float(np.mean(c_dma)), packed / 2.0 ** 20, [float(np.mean(c_hot))], [1])
        table4 = {"first_layer_saving_ms_measured": round(rows[1]["measured_ms"] - rows[2]["measured_ms"], 2),
                  "first_layer_saving_ms_eq4": round(b3[0] * packed / 2.0 ** 20, 2),
                  "middle_layer_saving_ms_eq4": round(b3[1] * packed / 2.0 ** 20, 2)}
        if k_fit > 1:
            rows.append(measure(k_fit, B.DL_MODE_PIPELINED))
            ctx.sync()
            torch.cuda.synchronize()
            identical = bool(torch.equal(yv.view(torch.int32), ref.view(torch.int32)))
        del ref
        for r in rows:
            log("long %s T=%d k=%2d %-10s %.2f ms (predicted %.2f, %+.2f%%) hidden %.3f H2D %.1f GB/s roofline frac %.3f" %
                (which, T, r["k"], r["mode"], r["measured_ms"], r["predicted_ms"], r["pred_err_pct"], r["hidden_frac"], r["h2d_gbps"],
                 r["roofline_frac"]))
        return {"workload": "%s, T=%d, cap %.3g B" % (name, T, cap), "layer_bytes": packed,
                "layer_flop": flops_layer,
                "profile": {"c_dma_ms": round(float(np.mean(c_dma)), 4), "c_dma_cont_ms": round(float(np.mean(c_cont)), 4),
                            "c_exe_ms": round(float(np.mean(c_exe)), 4), "c_exe_hot_ms": round(float(np.mean(c_hot)), 4),
                            "c_fence_ms": round(float(np.mean(c_fence)), 4), "c_fence_hot_ms": round(float(np.mean(c_fhot)), 4),
                            "r": round(float(np.mean(c_dma) / np.mean(c_exe)), 3)},
                "runs": rows, "table4_check": table4, "streamed_vs_partially_resident_bit_identical": identical}
    finally:
        eng.close()


def vla_leg(B, CFG, Engine, torch, log, cap, n_decode=64):
    """configs[4]: vision encoder -> merger -> 8B decoder prefill + 64 decode steps -> action head (10 Euler
    steps, 64 tokens cross-attending to the decoder's hidden states), all under one arena; one slot pair shared
    by the three stacks; residency per module chosen by the planner from one profiling run."""
    import numpy as np
    from paper_2605_11678_amd.harness import VlaPipeline
    vit, dec, act = CFG.vit_encoder(), CFG.decoder_8b(max_seq=3072 + n_decode), CFG.action_head()
    eng = Engine(int(cap), device=0)
    t0 = time.time()
    pipe = VlaPipeline(eng, vit, dec, act, n_patches=4096, n_text=2048, n_actions=64)
    ctx = eng.ctx
    mods = [pipe.m_vit, pipe.m_dec, pipe.m_act]
    cfgs = [vit, dec, act]
    Ls = [c.n_layers for c in cfgs]
    sizes = [ctx.module_layer_bytes(m)[0] for m in mods]
    log("vla setup %.1f s; layer bytes %s; arena used %.3f GB (everything streamed)" %
        (time.time() - t0, sizes, ctx.arena_stats()["used"] / 1e9))
    ctx.set_mode(B.DL_MODE_PIPELINED, 1)
    pipe.run(1)                                              # warm every kernel once, fills the KV cache and ctx
    eng.pick_copy_stream(pipe.m_vit, 4096, pipe.p_patch, pipe.p_vit)
    # ---- one profiling run per module and phase ----
    P = {}
    P["vit"] = ctx.profile(pipe.m_vit, Ls[0], 4096, 0, pipe.p_patch, iters=3)
    P["prefill"] = ctx.profile(pipe.m_dec, Ls[1], pipe.n_prefill, 0, pipe.p_seq, iters=3)
    P["decode"] = ctx.profile(pipe.m_dec, Ls[1], 1, pipe.n_prefill, pipe.p_x1, iters=3)
    P["action"] = ctx.profile(pipe.m_act, Ls[2], 64, 0, pipe.p_ain, iters=3, ctx_ptr=pipe.p_ctx, n_ctx=pipe.n_prefill)
    mean = lambda rows, key: float(np.mean([r[key] for r in rows]))
    prof = {k: {"c_dma_ms": round(mean(v, "c_dma_ms"), 4), "c_exe_ms": round(mean(v, "c_exe_ms"), 4),
                "c_exe_hot_ms": round(mean(v, "c_exe_hot_ms"), 4), "c_fence_ms": round(mean(v, "c_fence_ms"), 4)}
            for k, v in P.items()}
    MiB = float(1 << 20)
    b3 = [B.benefit(prof["vit"]["c_dma_ms"], sizes[0] / MiB, [prof["vit"]["c_exe_ms"]], [1]),
          B.benefit(prof["prefill"]["c_dma_ms"], sizes[1] / MiB, [prof["prefill"]["c_exe_ms"], prof["decode"]["c_exe_ms"]],
                    [1, n_decode]),
          B.benefit(prof["action"]["c_dma_ms"], sizes[2] / MiB, [prof["action"]["c_exe_ms"]], [10])]
    # Sec. IV-D's budget as the library accepts it: every residency whose resident copies and slots sum to at most
    # this many bytes is taken, so the planner's choice never has to be re-tried with head-room
    budget = ctx.residency_budget()
    # the ranking when the budget also covers the slots and these are sized by the modules that still stream:
    # a fully resident decoder shrinks the pair from 2 x 386 MB to the small stacks' layers
    k_shared = B.plan_shared_slots(Ls, sizes, [list(b) for b in b3], budget)
    # ... against the paper's reading: two slots of the largest layer of all modules, fixed
    k_plan = B.plan(Ls, sizes, [list(b) for b in b3], budget - 2 * max(sizes))
    log("vla benefit (ms/MiB) first/mid/last: vit %s, decoder %s, action %s; budget %.3f GB -> k = %s (slots fixed at 2 x M_max), "
        "%s (slots sized by the streaming modules)" %
        (np.round(b3[0], 4).tolist(), np.round(b3[1], 4).tolist(), np.round(b3[2], 4).tolist(), budget / 1e9, k_plan, k_shared))

    # benefit per MiB as a function of the decode length N and of the number of Euler steps (Sec. IV-D: the
    # ranking of the modules, and with it the plan, depends on how often each module's layers are invoked)
    def b3_for(n_dec, n_eul):
        return [B.benefit(prof["vit"]["c_dma_ms"], sizes[0] / MiB, [prof["vit"]["c_exe_ms"]], [1]),
                B.benefit(prof["prefill"]["c_dma_ms"], sizes[1] / MiB,
                          [prof["prefill"]["c_exe_ms"], prof["decode"]["c_exe_ms"]], [1, n_dec]),
                B.benefit(prof["action"]["c_dma_ms"], sizes[2] / MiB, [prof["action"]["c_exe_ms"]], [n_eul])]
    crossover = []
    for n_dec, n_eul in [(0, 10), (1, 10), (4, 10), (15, 10), (21, 10), (64, 10), (256, 10), (1024, 10), (64, 1), (64, 4), (64, 20), (64, 50)]:
        bb = b3_for(n_dec, n_eul)
        crossover.append({"n_decode": n_dec, "n_euler": n_eul, "b_mid_ms_per_MiB_vit_dec_act": [round(float(b[1]), 5) for b in bb],
                          "k_vit_dec_act": B.plan_shared_slots(Ls, sizes, [list(b) for b in bb], budget),
                          "k_with_slots_2x_largest_layer": B.plan(Ls, sizes, [list(b) for b in bb], budget - 2 * max(sizes))})

    # greedy head per token (resident, outside the layer passes)
    ctx.sync()
    t = time.perf_counter()
    for _ in range(30):
        ctx.greedy_step(pipe.m_dec, pipe.p_y1, pipe.p_tok, pipe.p_x1)
    ctx.sync()
    head_ms = (time.perf_counter() - t) * 1e3 / 30

    # the launches that belong to no layer (projector, pooling, final norm, Euler updates, output projection)
    ctx.sync()
    t = time.perf_counter()
    for _ in range(10):
        pipe.enqueue_glue()
    ctx.sync()
    glue_ms = (time.perf_counter() - t) * 1e3 / 10

    def predict(ks, wrap):
        dma, cont, hot, idle, fence, fhot, load, streamed, starts, mids = [], [], [], [], [], [], [], [], [], []
        def add_pass(mi, rows, res):
            for i, r in enumerate(rows):
                dma.append(r["c_dma_ms"]); cont.append(r["c_dma_cont_ms"]); hot.append(r["c_exe_hot_ms"]); idle.append(r["c_exe_ms"]); fence.append(r["c_fence_ms"]); fhot.append(r["c_fence_hot_ms"]); load.append(r["c_exe_loaded_ms"])
                streamed.append(i not in res); starts.append(i == 0); mids.append(mi)
        rs = [set(B.place_interleaved(Ls[m], ks[m])) for m in range(3)]
        add_pass(0, P["vit"], rs[0])
        add_pass(1, P["prefill"], rs[1])
        for _ in range(n_decode):
            add_pass(1, P["decode"], rs[1])
        for _ in range(10):
            add_pass(2, P["action"], rs[2])
        return B.timeline(dma, hot, streamed, starts, module_id=mids, wrap_prefetch=wrap, c_exe_idle_ms=idle,
                          c_fence_ms=fence, c_dma_cont_ms=cont, c_fence_hot_ms=fhot, c_exe_loaded_ms=load)["total"] \
            + head_ms * n_decode + glue_ms

    def measure(ks, wrap, reps):
        for m in range(3):
            ctx.set_residency(mods[m], [])                   # release first: the new plan may not fit next to the old one
        for m in range(3):
            ctx.set_residency(mods[m], B.place_interleaved(Ls[m], ks[m]))
        ctx.set_mode(B.DL_MODE_PIPELINED, wrap)
        eng.upload(pipe.v_seq[pipe.n_vis * dec.d_model:], pipe.text)
        samples = []
        for _ in range(reps):
            eng.upload(pipe.v_a, pipe.a0)
            torch.cuda.synchronize()
            t = time.perf_counter()
            pipe.enqueue(n_decode)
            ctx.sync()
            samples.append((time.perf_counter() - t) * 1e3)
        return float(np.median(samples)), pipe.results(n_decode)

    rows, ref = [], None
    # second policy of the comparison: small modules fully resident first, the decoder gets what is left
    left = budget - 2 * max(sizes) - Ls[0] * sizes[0] - Ls[2] * sizes[2]
    k_alt = [Ls[0], max(0, min(Ls[1], int(left // sizes[1]))), Ls[2]]
    for name, ks, reps in (("planner_slots_sized_by_streaming_modules", k_shared, 3), ("planner_slots_2x_largest_layer", k_plan, 3),
                           ("vit_and_action_resident_first", k_alt, 3), ("all_streamed", [0, 0, 0], 1)):
        try:
            ms, out = measure(ks, 1, reps)
        except B.DLError as e:
            rows.append({"policy": name, "k": ks, "error": str(e)})
            continue
        pred = predict(ks, 1)
        same = None
        if ref is None:
            ref = out
        else:
            same = bool(np.array_equal(out["trajectory"].view(np.uint32), ref["trajectory"].view(np.uint32))
                        and out["tokens"] == ref["tokens"])
        rows.append({"policy": name, "k_vit_dec_act": ks, "ms_per_inference": round(ms, 2), "predicted_ms": round(pred, 2),
                     "pred_err_pct": round((pred - ms) / ms * 100, 2), "arena_gb": round(ctx.arena_stats()["used"] / 1e9, 3),
                     "bit_identical_to_first": same})
        log("vla %-30s k=%s: %.1f ms/inference (predicted %.1f, %.2f%%) identical=%s" % (name, ks, ms, pred, rows[-1]["pred_err_pct"], same))
    res = {"workload": "configs[4]: ViT 27L T=4096 -> merger -> 8B decoder prefill 3072 + %d decode steps -> action head 8L x 10 Euler "
                       "steps on 64 tokens; cap %.3g B" % (n_decode, cap),
           "layer_bytes": sizes, "profile": prof, "benefit_ms_per_MiB": [np.round(b, 5).tolist() for b in b3],
           "budget_gb": round(budget / 1e9, 3), "budget_source": "dl_residency_budget (what slots and resident layers may use; every set within it is accepted)", "head_ms": round(head_ms, 4), "glue_ms": round(glue_ms, 4), "runs": rows,
           "benefit_vs_decode_length_and_euler_steps": crossover,
           "trajectory_finite": bool(np.all(np.isfinite(ref["trajectory"]))) if ref else None}
    eng.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=36, help="debug: fewer layers (invalidates the number)")
    ap.add_argument("--tokens", type=int, default=3072)
    ap.add_argument("--cap", type=float, default=16e9)
    ap.add_argument("--sweep", type=str, default="0,9,18,27,33,35,36")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the decode, ViT and pipeline legs")
    ap.add_argument("--extras", default="decode,vit,vla,long", help="which of the extra legs to run (comma list)")
    ap.add_argument("--only", default="", help="profiling aid: run just one of the extra legs (vit | vla | long) and print its "
                                                "record instead of the contract line")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE), then "
                         "the timed steps at full residency; no sweep, no extras, no CPU leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build is single-GPU by design (one process, one MI355X, no collectives); "
            "run it with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2605_11678_amd import binding as B, build, configs as CFG
    from paper_2605_11678_amd.harness import Engine

    build.ensure_built()
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)

    if args.only:
        leg = {"vit": lambda: vit_leg(B, CFG, Engine, torch, log),
               "vla": lambda: vla_leg(B, CFG, Engine, torch, log, int(args.cap)),
               "long": lambda: long_prefill_leg(B, CFG, Engine, torch, log, int(args.cap)),
               "long_encoder": lambda: long_prefill_leg(B, CFG, Engine, torch, log, int(args.cap), which="encoder")}[args.only]
        print(json.dumps({"only": args.only, "record": leg()}), flush=True)
        return

    c = CFG.decoder_8b(n_layers=args.layers)            # with the 4096x32768 head and embedding (decode leg)
    T, L = args.tokens, c.n_layers
    cap = int(args.cap)
    t0 = time.time()
    eng = Engine(cap, device=0, fence_slack_bytes=3 << 30)     # allocator limit as a second fence around the cap
    mid = eng.add_module(c, max_tokens=T)
    packed, params = eng.ctx.module_layer_bytes(mid)
    log("setup: %d layers x %.1f MiB packed (%.1f MiB parameters) in %.1f s" % (L, packed / 2 ** 20, params / 2 ** 20, time.time() - t0))
    x = CFG.make_tokens(T, c.d_model, seed=7)
    xp, xv = eng.alloc_f32(T * c.d_model)
    yp, yv = eng.alloc_f32(T * c.d_model)
    eng.upload(xv, x)
    ctx = eng.ctx
    ctx.set_mode(B.DL_MODE_PIPELINED, 0)
    tried = eng.pick_copy_stream(mid, T, xp, yp, passes=2)
    log("copy-stream candidates (ms per fully streamed pass): " + ", ".join("%.2f" % t for _, t in tried))

    # ---- one profiling run in sequential mode (Table III procedure) ----
    prof = ctx.profile(mid, L, T, 0, xp, iters=3)
    c_dma = [p["c_dma_ms"] for p in prof]
    c_cont = [p["c_dma_cont_ms"] for p in prof]        # the same copy inside a train of copies (copy queue never dry)
    c_exe = [p["c_exe_ms"] for p in prof]              # right after the copy (GPU was idle): the paper's C_EXE
    c_hot = [p["c_exe_hot_ms"] for p in prof]          # the same layer re-run at once (GPU busy)
    c_fence = [p["c_fence_ms"] for p in prof]          # cross-stream hand-offs of a streamed layer
    c_fhot = [p["c_fence_hot_ms"] for p in prof]       # the same when the copy is long done as the layer starts
    c_load = [p["c_exe_loaded_ms"] for p in prof]      # c_hot while copies run the whole time
    log("profile: C_DMA %.3f ms  C_EXE %.3f ms (%.3f ms when compute is continuous) per layer (means), r = %.2f" %
        (np.mean(c_dma), np.mean(c_exe), np.mean(c_hot), np.mean(c_dma) / np.mean(c_exe)))

    def set_k(k):
        ctx.set_residency(mid, B.place_interleaved(L, k))

    def run_once():
        ctx.forward(mid, xp, yp, T, 0)

    def timed(n):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            run_once()
        ctx.sync()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n

    def predict(k, mode=B.DL_MODE_PIPELINED):
        res = set(B.place_interleaved(L, k))
        streamed = [i not in res for i in range(L)]
        return B.timeline(c_dma, c_hot, streamed, [i == 0 for i in range(L)], mode=mode, c_exe_idle_ms=c_exe,
                          c_fence_ms=c_fence, c_dma_cont_ms=c_cont, c_fence_hot_ms=c_fhot, c_exe_loaded_ms=c_load)

    # ---- largest resident count the arena holds ----
    k_best = None
    for k in range(L, -1, -1):
        try:
            set_k(k)
            k_best = k
            break
        except B.DLError as e:
            if e.code != B.DL_ERR_BUDGET_EXCEEDED:
                raise
    arena = ctx.arena_stats()
    log("headline residency: k = %d of %d, arena %.3f of %.3f GB" % (k_best, L, arena["used"] / 1e9, arena["capacity"] / 1e9))

    if args.pmc_probe:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        dst.copy_(src)                                       # known traffic: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        args.sweep, args.no_extras, args.no_cpu_baseline = "", True, True

    # ---- the timed region: exactly K steps ----
    # Inside it only the dominant kernel class (the gate/up projection GEMM, ~40 % of a pass) is bracketed
    # with events: an event pair drains the queue between kernels, and bracketing all eight classes costs
    # ~3 % of the pass.  The full per-class breakdown comes from a second region of the same K steps.
    for _ in range(args.warmup):
        run_once()
    ctx.sync()
    ctx.set_kernel_timing(True, kinds=[B.DL_K_NAMES.index("gemm_up")])
    with ClockSampler() as clk:
        ms_per_step = timed(args.steps)
    clock = clk.summary()
    dom = ctx.collect_kernel_times()["gemm_up"]
    ctx.set_kernel_timing(True)
    ms_per_step_all_events = timed(args.steps)
    kt = ctx.collect_kernel_times()
    ctx.set_kernel_timing(False)

    gemm_kinds = ["gemm_qkv", "gemm_o", "gemm_up", "gemm_down"]
    g_ms = sum(kt[k]["total_ms"] for k in gemm_kinds)
    g_fl = sum(kt[k]["flops"] for k in gemm_kinds)
    a_ms, a_fl = kt["attn"]["total_ms"], kt["attn"]["flops"]
    achieved = dom["flops"] / (dom["total_ms"] * 1e-3) / 1e12 if dom["total_ms"] > 0 else 0.0
    family = g_fl / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    # bytes per launch between L2 and the fabric, from the committed rocprofv3 --pmc summary of this same workload
    # (hardware counters cannot be read from inside this process; the figure is the one of the committed counter run
    # of this same command line, and says so)
    traffic, traffic_source = None, None
    tj = os.path.join(ROOT, "profiles", "traffic_gemm_up_decoder8b_prefill.json")
    if os.path.exists(tj) and L == 36 and T == 3072:
        traffic = round(json.load(open(tj))["bytes_per_launch"])
        traffic_source = "profiles/hbm_traffic_decoder8b_prefill_T3072.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE over `bench.py --pmc-probe`, not measured in this run)"
    roofline = {"bound": "mfma", "kernel": "gemm_fast_split_tail<SwiGLU>: 256x256 tiles, last half round as 128x256 (gate/up projection, M=%d N=%d K=%d)" % (T, 2 * c.d_ff, c.d_model),
                "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "launches": dom["launches"],
                "avg_launch_ms": round(dom["total_ms"] / max(dom["launches"], 1), 4),
                "flop_per_launch": dom["flops"] / max(dom["launches"], 1),
                "gemm_family_tflops": round(family, 2), "ms_per_step_with_all_classes_timed": round(ms_per_step_all_events, 3)}
    mfma_util = (g_fl + a_fl) / ((g_ms + a_ms) * 1e-3) / (PEAK_BF16_TFLOPS * 1e12) if g_ms + a_ms > 0 else 0.0
    kernels = {k: {"ms_per_step": round(v["total_ms"] / args.steps, 4),
                   "tflops": round(v["flops"] / (v["total_ms"] * 1e-3) / 1e12, 2) if v["total_ms"] > 0 and v["flops"] > 0 else None,
                   "gbps": round(v["bytes"] / (v["total_ms"] * 1e-3) / 1e9, 1) if v["total_ms"] > 0 else None}
               for k, v in kt.items() if v["launches"]}

    # ---- the box's own ceilings, measured in this run ----
    # register-only MFMA rate (zero operands and hashed +-[1,2) operands: the chip is power-limited, the rate depends
    # on operand toggling), and the best pinned host-to-device copy of 1 GiB on the copy stream
    peaks = {}
    try:
        peaks["mfma_zero_operands_tflops"] = round(ctx.probe_mfma_rate(0), 1)
        peaks["mfma_random_operands_tflops"] = round(ctx.probe_mfma_rate(1), 1)
        hsrc = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
        hsrc.zero_()
        ddst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        best = 1e30
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(eng.s_copy):
                e0.record()
                ddst.copy_(hsrc, non_blocking=True)
                e1.record()
            eng.s_copy.synchronize()
            best = min(best, e0.elapsed_time(e1))
        peaks["h2d_1gib_gbps"] = round((1 << 30) / (best * 1e6), 2)
        del hsrc, ddst
    except B.DLError as e:
        peaks["error"] = str(e)
    log("box ceilings: %s" % peaks)

    flops_layer = 2.0 * T * c.d_model * (c.n_q_heads * c.d_head + 2 * c.n_kv_heads * c.d_head) \
        + 2.0 * T * c.d_model * c.n_q_heads * c.d_head + 6.0 * T * c.d_model * c.d_ff \
        + 4.0 * c.d_head * c.n_q_heads * (T * (T + 1) / 2.0)
    roof_dma = [packed / (LINK_GBPS_THEORY * 1e6)] * L          # ms per layer at the link's theoretical rate
    roof_exe = [flops_layer / (PEAK_BF16_TFLOPS * 1e9)] * L     # ms per layer at the vendor MFMA peak

    # ---- residency sweep: measured vs predicted, hidden fraction, link rate ----
    sweep = []
    ks = sorted({min(max(int(s), 0), L) for s in args.sweep.split(",") if s.strip() != ""})
    if args.pmc_probe:
        ks = []
    c_total0 = None
    for k in ks:
        try:
            set_k(k)
        except B.DLError as e:
            if e.code == B.DL_ERR_BUDGET_EXCEEDED:
                sweep.append({"k": k, "error": "does not fit the arena"})
                continue
            raise
        run_once()
        ctx.sync()
        reps = 3
        meas = timed(reps)
        ctx.set_timing(True)
        run_once()
        st = ctx.collect_stats()
        ctx.set_timing(False)
        pred = predict(k)
        if k == 0:
            c_total0 = meas
        streamed_dma = sum(c_dma[i] for i in range(L) if i not in set(B.place_interleaved(L, k)))
        hideable = min(1.0, sum(c_hot) / streamed_dma) if streamed_dma > 0 else 1.0
        # per-layer roofline max(bytes / link, flops / MFMA peak), composed through the same timeline
        link = max(st["h2d_gbps"], 1e-9)
        row = {"k": k, "measured_ms": round(meas, 3), "predicted_ms": round(pred["total"], 3),
               "pred_err_pct": round((pred["total"] - meas) / meas * 100, 2),
               "hidden_frac": round(st["hidden_frac"], 4), "hideable_frac": round(hideable, 4),
               "h2d_gbps": round(st["h2d_gbps"], 2), "timed_pass_ms": round(st["total_ms"], 3),
               "exe_ms_per_layer": round(st["exe_ms"] / L, 4), "arena_gb": round(ctx.arena_stats()["used"] / 1e9, 3)}
        res_k = set(B.place_interleaved(L, k))
        roof = B.timeline(roof_dma, roof_exe, [i not in res_k for i in range(L)], [i == 0 for i in range(L)])["total"]
        row["roofline_ms"] = round(roof, 3)
        row["roofline_frac"] = round(roof / meas, 4)
        if c_total0 is not None:
            # Eq. 9 with the slope taken from the profile alone (DMA-intensive, R = 1: one C_DMA per layer)
            lin = B.predict_linear(c_total0, float(np.mean(c_dma)), k)
            row["eq9_ms"] = round(lin, 3)
        sweep.append(row)
        log("k=%2d measured %.2f ms predicted %.2f ms (%.2f%%) hidden %.3f (hideable %.3f) H2D %.1f GB/s" %
            (k, meas, pred["total"], row["pred_err_pct"], st["hidden_frac"], hideable, link))

    # sequential vs pipelined at k = 0 (Sec. IV-B vs IV-C)
    progress = {}
    try:
        if args.pmc_probe:
            raise B.DLError(0, "skipped in --pmc-probe mode")
        set_k(0)
        ctx.set_mode(B.DL_MODE_SEQUENTIAL, 0)
        run_once()
        progress["sequential_k0_ms"] = round(timed(2), 3)
        ctx.set_mode(B.DL_MODE_PIPELINED, 0)
        run_once()
        progress["pipelined_k0_ms"] = round(timed(2), 3)
        progress["resident_best_ms"] = round(ms_per_step, 3)
    except B.DLError as e:
        progress["error"] = str(e)


    # ---- decode leg (configs[3]): same stack, KV cache from the 3072-token prefill, greedy steps ----
    extras = {}
    legs = set() if args.no_extras else {x.strip() for x in args.extras.split(",") if x.strip()}
    if "decode" in legs:
        try:
            extras["decode"] = decode_leg(eng, ctx, mid, c, T, L, xp, yp, packed, B, torch, log)
        except B.DLError as e:
            extras["decode"] = {"error": str(e)}

    # ---- CPU oracle on bounded samples (a reported baseline, not the target) ----
    # the headline workload: one layer of the same stack at the same T, scaled to the stack (labelled extrapolated);
    # beside it the tiny workload in full, four encoder layers scaled to 27, and single-token steps of one 8B layer
    # scaled to 36 layers
    cpu, cpu_other = None, []
    if not args.no_cpu_baseline:
        from oracle import forward as F
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        n_samp = 1
        w0 = CFG.make_layer_weights(c, 0)
        W0 = {t: F.widen(a) for t, a in w0.items()}          # widened once: the steps below time the arithmetic
        oc = c.as_dict()
        oc["n_layers"] = n_samp
        kvc = F.new_kv_cache(oc)
        tc = time.perf_counter()
        F.stack_forward(oc, lambda l: W0, x, 0, kvc)
        dt = time.perf_counter() - tc
        cpu = {"value": round(dt / n_samp * L * 1e3, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
               "extrapolated": True,
               "sample": "%d of %d layers at T=%d in fp64 numpy (%.1f s), scaled to %d layers" % (n_samp, L, T, dt, L)}
        tc = time.perf_counter()
        n_tok = 4
        for s_ in range(n_tok):
            F.stack_forward(oc, lambda l: W0, x[s_:s_ + 1], T + s_, kvc)
        dt = time.perf_counter() - tc
        cpu_other.append({"workload": "configs[3] decode: ms per token", "value": round(dt / n_tok * L * 1e3, 1), "unit": "ms",
                          "cores": int(cores), "kind": "oracle", "extrapolated": True,
                          "sample": "%d single-token steps of 1 layer over a %d-entry cache (%.2f s), scaled to %d layers" % (n_tok, T, dt, L)})
        del W0, w0, kvc
        tiny = CFG.tiny_decoder()
        xt = CFG.make_tokens(128, tiny.d_model, seed=7)
        tc = time.perf_counter()
        F.generate_greedy(tiny.as_dict(), lambda l: CFG.make_layer_weights(tiny, l), CFG.make_head(tiny), xt, 8)
        cpu_other.append({"workload": "configs[0] in full: prefill 128 + 8 greedy steps", "value": round((time.perf_counter() - tc) * 1e3, 1),
                          "unit": "ms", "cores": int(cores), "kind": "oracle", "extrapolated": False, "sample": "the whole workload"})
        vit = CFG.vit_encoder(n_layers=4)
        xv_ = CFG.make_tokens(4096, vit.d_model, seed=7)
        tc = time.perf_counter()
        F.stack_forward(vit.as_dict(), lambda l: CFG.make_layer_weights(vit, l), xv_)
        dt = time.perf_counter() - tc
        cpu_other.append({"workload": "configs[1]: 27-layer encoder, T=4096", "value": round(dt / 4 * 27 * 1e3, 1), "unit": "ms",
                          "cores": int(cores), "kind": "oracle", "extrapolated": True,
                          "sample": "4 of 27 layers at T=4096 (%.1f s), scaled to 27 layers" % dt})

    # ---- the streamed path next to the resident headline ----
    row_k0 = next((r for r in sweep if r.get("k") == 0 and "measured_ms" in r), None)
    row_top = next((r for r in sweep if r.get("k") == k_best and "measured_ms" in r), None)
    # per-layer roofline max(bytes / link, flops / MFMA peak) composed over the pass (all layers resident: L x flops / peak)
    path_roof_ms = L * flops_layer / (PEAK_BF16_TFLOPS * 1e9) if (k_best == L or not row_top) else row_top["roofline_ms"]
    roofline["path_roofline_ms_k%d" % k_best] = round(path_roof_ms, 3)
    roofline["path_roofline_frac_k%d" % k_best] = round(path_roof_ms / ms_per_step, 4)
    streamed = None
    if row_k0:
        streamed = {"k": 0, "ms": row_k0["measured_ms"], "h2d_gbps": row_k0["h2d_gbps"],
                    "link_roofline_frac": row_k0["roofline_frac"], "hidden_frac": row_k0["hidden_frac"],
                    "hideable_frac": row_k0["hideable_frac"],
                    "hidden_over_hideable": round(row_k0["hidden_frac"] / row_k0["hideable_frac"], 4) if row_k0["hideable_frac"] > 0 else None,
                    "pred_err_pct": row_k0["pred_err_pct"]}
        roofline["streamed_k0_ms"] = row_k0["measured_ms"]
        roofline["streamed_k0_h2d_gbps"] = row_k0["h2d_gbps"]
        roofline["streamed_k0_link_roofline_frac"] = row_k0["roofline_frac"]
        roofline["streamed_k0_hidden_over_hideable"] = streamed["hidden_over_hideable"]

    out = {
        "metric": "ms/inference under VRAM cap", "value": round(ms_per_step, 3), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[2]: 8B-class decoder prefill, %d layers d=4096 GQA 32/8x128 SwiGLU 12288, "
                               "T=%d, batch 1, cap %.3g B, resident layers k=%d (largest that fits)" % (L, T, cap, k_best),
                   "layer_bytes": packed, "mode": "pipelined, 2 slots", "seed": "weights 3000+layer, tokens 7"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "cpu_baseline_other_workloads": cpu_other,
        "streamed": streamed,
        "clock": clock,
        "mfma_util": round(mfma_util, 4),
        "mfma_util_vs_measured_peak": round(mfma_util * PEAK_BF16_TFLOPS / peaks["mfma_random_operands_tflops"], 4)
        if peaks.get("mfma_random_operands_tflops") else None,
        "box_ceilings": peaks,
        "layer_flop": flops_layer,
        "inference_tflops": round(flops_layer * L / (ms_per_step * 1e-3) / 1e12, 2),
        "kernels": kernels,
        "profile": {"c_dma_ms": round(float(np.mean(c_dma)), 4), "c_dma_cont_ms": round(float(np.mean(c_cont)), 4),
                    "c_exe_ms": round(float(np.mean(c_exe)), 4),
                    "c_exe_hot_ms": round(float(np.mean(c_hot)), 4),
                    "c_fence_ms": round(float(np.mean(c_fence)), 4),
                    "c_fence_hot_ms": round(float(np.mean(c_fhot)), 4),
                    "r": round(float(np.mean(c_dma) / np.mean(c_exe)), 3),
                    "h2d_gbps": round(packed / (float(np.mean(c_dma)) * 1e6), 2),
                    "h2d_frac_of_63GBps": round(packed / (float(np.mean(c_dma)) * 1e6) / LINK_GBPS_THEORY, 3)},
        "sweep": sweep,
        "progression": progress,
        "max_pred_err_pct": max([abs(r["pred_err_pct"]) for r in sweep if "pred_err_pct" in r] or [None]),
        "extras": extras,
    }
    eng.close()
    if "vit" in legs:
        try:
            out["extras"]["vit"] = vit_leg(B, CFG, Engine, torch, log)
        except B.DLError as e:
            out["extras"]["vit"] = {"error": str(e)}
    if "vla" in legs:
        try:
            out["extras"]["vla"] = vla_leg(B, CFG, Engine, torch, log, cap)
        except B.DLError as e:
            out["extras"]["vla"] = {"error": str(e)}
    if "long" in legs:
        try:
            out["extras"]["long_prefill"] = long_prefill_leg(B, CFG, Engine, torch, log, cap)
            out["extras"]["long_encoder"] = long_prefill_leg(B, CFG, Engine, torch, log, cap, which="encoder")
            # the execution-intensive regime next to the streamed headline figures (what a record of the line's
            # top-level objects keeps)
            lp = [r for r in out["extras"]["long_prefill"]["runs"] if r["k"] == 0 and r["mode"] == "pipelined"]
            if lp and isinstance(out.get("streamed"), dict):
                out["streamed"]["T16384_k0"] = {k_: lp[0][k_] for k_ in ("measured_ms", "predicted_ms", "pred_err_pct",
                                                                         "hidden_frac", "h2d_gbps", "roofline_frac")}
        except B.DLError as e:
            out["extras"]["long_prefill"] = {"error": str(e)}
    # the residency sweep of the headline workload once more, last on stderr (what a truncated log keeps)
    log("---- summary: 8B decoder prefill T=%d under %.3g B ----" % (T, cap))
    for r in sweep:
        if "measured_ms" in r:
            log("k=%2d  %.2f ms  predicted %.2f ms (%+.2f%%)  hidden %.3f of hideable %.3f  H2D %.1f GB/s  roofline frac %.3f" %
                (r["k"], r["measured_ms"], r["predicted_ms"], r["pred_err_pct"], r["hidden_frac"], r["hideable_frac"],
                 r["h2d_gbps"], r["roofline_frac"]))
    log("headline k=%d: %.2f ms/inference, gate/up GEMM %.0f TFLOP/s (%.3f of peak), whole path %.3f of its MFMA roofline; clock %s" %
        (k_best, ms_per_step, achieved, achieved / PEAK_BF16_TFLOPS, path_roof_ms / ms_per_step, clock))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
