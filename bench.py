#!/usr/bin/env python3
"""Benchmark of the TLI draft-and-verify hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input already resident in HBM:
tli_draft_sample on all B*K drafter rows, then tli_verify on the B sequences.  The workload is the
large-vocabulary batch (B=256, K=8, Vt=256000, Vd=128256, ~90000 shared ids, bf16 logits, temperature
0.7).  Prints ONE JSON line: `ms_per_step` of the whole step, `value` = verified draft positions per second of
tli_verify (the metric), the step's own rate beside it, the roofline figures of the dominant kernel (the
target-row normaliser scan of tli_verify) measured with HIP events on the launch stream inside the timed
region and of the whole tli_verify call, and the CPU oracle timed on a bounded sample of the same batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per launch of the dominant kernel as read by rocprofv3 (FETCH_SIZE + WRITE_SIZE, each scaled by
# what the same counter reads for the library's plain copy kernel); from profiles/*_hbm_traffic_pmc.md.
# Counters cannot be read from inside this process, so the figure is carried here per workload.
_PMC_NOTE = (" (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, of a separate run of this command, scaled by the copy "
             "kernel's reading; carried here, not measured by this run)")
MEASURED_TRAFFIC = {  # fetched + written bytes per launch of the dominant kernel
    "large_vocab": dict(bytes=1049.24e6 + 2.19e6, source="profiles/large_vocab_all_kernels_hbm_traffic_pmc.md" + _PMC_NOTE),
    "mismatch": dict(bytes=517.35e6 + 1.16e6, source="profiles/mismatch_all_kernels_hbm_traffic_pmc.md" + _PMC_NOTE),
    "batched": dict(bytes=97.42e6 + 0.32e6, source="profiles/batched_all_kernels_hbm_traffic_pmc.md" + _PMC_NOTE),
}
DOMINANT_KERNEL = {  # what the library launches for the target rows' log-normalisers, by batch size
    True: "k_lse_accept_seq (log-normalisers of the K target rows of every sequence, accept tests as the rows complete)",
    False: "k_lse (target-row log-normalisers)",
}


def _cpu_model() -> str:
    try:
        for l in open("/proc/cpuinfo"):
            if l.startswith("model name"):
                return l.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", type=int, default=4, help="1..5 (default 4 = the headline configuration)")
    ap.add_argument("--spinup-ms", type=float, default=300.0,
                    help="untimed steps for this long before the declared warm-up (clocks settle); reported in the line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=0, help="sequences in the oracle's sample (0 = auto)")
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel in a second pass")
    ap.add_argument("--next", action="store_true",
                    help="also time the neighbouring entry points (union algorithm, acceptance rates, exact-match tail, "
                         "temperature zero) on the same batch")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent: N GPUs would each take "
              "B/N sequences with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2502_05202_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load_library()  # raises if the HIP library is missing: there is no fallback
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    inp = synth.make_inputs(w, dev)
    code = binding.TLI_F32 if w.dtype == "f32" else binding.TLI_BF16
    esz = 4 if w.dtype == "f32" else 2
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    ws = binding.alloc_workspace(w.B, w.K, m, code, dev)
    u_draft = inp["u_draft"].reshape(-1).contiguous()
    u_acc = inp["u_acc"].reshape(-1).contiguous()
    R = w.B * w.K
    d_out = dict(tok_d=torch.empty(R, dtype=torch.int32, device=dev), tok_t=torch.empty(R, dtype=torch.int32, device=dev),
                 q_tok=torch.empty(R, dtype=torch.float64, device=dev), lse_q=torch.empty(R, dtype=torch.float64, device=dev),
                 status=torch.empty(R, dtype=torch.int32, device=dev))
    v_out = binding.alloc_verify_outputs(w.B, w.K, dev)

    # The chip keeps 256 MB of what it touched last (Infinity Cache), and tli_verify's last kernels re-read one target
    # row and one drafter row per sequence: called again on the same tensors, the next call would find those rows in
    # the cache (13 us of 219 on the large-vocabulary batch).  A serving loop gets new logits every step, so every
    # timed call below takes the next of several identical copies of the inputs, together more than twice the cache:
    # every row comes from HBM.  (The same-set figure is reported beside it, as cache.same_set_*.)
    set_bytes = (inp["logits_t"].numel() + inp["logits_d"].numel()) * esz
    cache_bytes = 256 << 20
    n_sets = max(3, -(-2 * cache_bytes // set_bytes) + 1)
    if n_sets > 64:
        n_sets = 1  # a few MB per set: latency figures, warm only
    sets = [(inp["logits_t"], inp["logits_d"])] + [(inp["logits_t"].clone(), inp["logits_d"].clone())
                                                    for _ in range(n_sets - 1)]
    turn = [0]

    def next_set():
        turn[0] += 1
        return sets[turn[0] % n_sets]

    def step():
        lt, ld = next_set()
        binding.tli_draft_sample(m, ld, w.tau_d, u_draft, ws, out=d_out)
        binding.tli_verify(m, lt, ld, w.tau_t, w.tau_d, d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws, out=v_out)

    # one plain copy of known size (256 MiB read + 256 MiB written): the yardstick for rocprofv3's byte counters
    calib_src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib_src)
    binding.tli_calib_copy(calib_src, calib_dst)
    torch.cuda.synchronize()
    del calib_src, calib_dst

    # untimed spin-up, reported on its own: a short invocation (a few milliseconds of timed work) would otherwise run
    # on clocks that have not settled; the declared warm-up and the timed steps below are exactly as passed
    spin_t0 = time.perf_counter()
    spin_steps = 0
    while time.perf_counter() - spin_t0 < args.spinup_ms * 1e-3:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        spin_steps += 20
    spinup_ms = 1e3 * (time.perf_counter() - spin_t0)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps; HIP events around the dominant kernel on the launch stream
    # (an event pair costs ~10 us of idle GPU, so one step in five carries it)
    binding.tli_profile_enable(["lse"], args.steps, every=5)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    lse_ms, lse_n = binding.tli_profile_collect("lse")
    binding.tli_profile_disable()
    total_s = t1 - t0
    ms_per_step = 1e3 * total_s / args.steps
    positions = w.B * w.K
    step_value = positions * args.steps / total_s

    # ---- the metric itself: verified draft positions per second of tli_verify -- the same number of calls, timed
    # the same way (wall clock around the loop, device idle before and after), drafts and normalisers as the last
    # step left them
    def verify_call():
        lt, ld = next_set()
        binding.tli_verify(m, lt, ld, w.tau_t, w.tau_d, d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws, out=v_out)

    def draft_call():
        binding.tli_draft_sample(m, next_set()[1], w.tau_d, u_draft, ws, out=d_out)

    torch.cuda.synchronize()
    v0 = time.perf_counter()
    for _ in range(args.steps):
        verify_call()
    torch.cuda.synchronize()
    v1 = time.perf_counter()
    verify_wall_ms = 1e3 * (v1 - v0) / args.steps
    value = positions * args.steps / (v1 - v0)

    # ---- separate timings of the two calls (outside the timed region)
    def time_call(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def time_each(fn, n):
        """one HIP-event pair per call: (median, min) in ms"""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        torch.cuda.synchronize()
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ts = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return ts[len(ts) // 2], ts[0]

    n_sep = max(5, args.steps // 2)
    draft_ms = time_call(draft_call, n_sep)
    verify_ms = time_call(verify_call, n_sep)
    verify_med_ms, verify_min_ms = time_each(verify_call, max(50, n_sep // 2))

    # the mode that is never the headline: no lse_q from the draft call, the library rescans the K drafter rows
    def verify_no_lse_q():
        lt, ld = next_set()
        binding.tli_verify(m, lt, ld, w.tau_t, w.tau_d, d_out["tok_d"], None, u_acc, inp["u_fin"], ws, out=v_out)

    verify_no_lse_q_ms = time_call(verify_no_lse_q, max(5, n_sep // 4))
    draft_med_ms, draft_min_ms = time_each(draft_call, max(50, n_sep // 2))
    # the same two calls on one set of tensors, back to back (what the cache returns of the last call's rows)
    same_draft_ms = time_call(lambda: binding.tli_draft_sample(m, inp["logits_d"], w.tau_d, u_draft, ws, out=d_out), n_sep)
    same_verify_ms = time_call(lambda: binding.tli_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d,
                                                          d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws,
                                                          out=v_out), n_sep)
    # ---- the drafting loop at its real shape: one tli_draft_sample call per lookahead position on the B rows
    # logits_d[:, k, :] (as after each drafter forward), then tli_verify; eager, and captured in a HIP graph
    def iteration(which=None):
        lt, ld = next_set() if which is None else sets[which]
        for k in range(w.K):
            binding.tli_draft_sample(m, ld[:, k, :], w.tau_d, u_draft, ws, out=d_out, column=(k, w.K))
        binding.tli_verify(m, lt, ld, w.tau_t, w.tau_d, d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws, out=v_out)

    per_step_eager_ms = time_call(iteration, n_sep)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graphs = []  # one captured iteration per input set, replayed in turn
    for i in range(n_sets):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            iteration(i)
        graphs.append(g)

    def replay():
        turn[0] += 1
        graphs[turn[0] % n_sets].replay()

    per_step_graph_ms = time_call(replay, n_sep)
    del graphs

    cache = dict(input_mb=round(set_bytes / 1e6, 1), rotated_sets=n_sets, same_set_draft_ms=round(same_draft_ms, 4),
                 same_set_verify_ms=round(same_verify_ms, 4),
                 note="every timed call takes the next of `rotated_sets` identical copies of the inputs (more than twice "
                      "the 256 MB cache together), so no row of the previous call is still cached; same_set_*: the two "
                      "calls back to back on one copy" if n_sets > 1 else
                      "the inputs are a few MB: latency figures, everything cached")

    # ---- the neighbouring steps on the same batch (each timed on its own; algorithmic bytes = rows read once)
    next_rows = {}
    if args.next:
        n_nx = max(3, n_sep // 3)
        rows_t = w.B * (w.K + 1)
        u_rows = torch.rand(rows_t, device=dev, dtype=torch.float32)
        draft_t = d_out["tok_t"].clone()
        ws_em = torch.empty(int(binding.load_library().tli_exact_match_workspace_bytes(w.B, w.K, w.Vt, code)),
                            dtype=torch.uint8, device=dev)
        em_out = binding.tli_exact_match_verify(inp["logits_t"], w.tau_t, draft_t, u_rows, ws_em)

        def timed(name, fn, nbytes):
            fn()
            ms = time_call(fn, n_nx)
            next_rows[name] = dict(ms=round(ms, 4), algorithmic_gbs=round(nbytes / (1e-3 * ms) / 1e9, 1),
                                   frac_of_peak=round(nbytes / (1e-3 * ms) / 1e9 / HBM_PEAK_GBS, 4))

        timed("exact_match_verify_sampled", lambda: binding.tli_exact_match_verify(
            inp["logits_t"], w.tau_t, draft_t, u_rows, ws_em, out=em_out), rows_t * w.Vt * esz)
        timed("exact_match_verify_argmax", lambda: binding.tli_exact_match_verify(
            inp["logits_t"], 0.0, draft_t, None, ws_em, out=em_out), rows_t * w.Vt * esz)
        timed("greedy_draft", lambda: binding.tli_greedy_draft(m, inp["logits_d"], ws), R * w.Vd * esz)
        timed("union_draft_sample", lambda: binding.tli_union_draft_sample(m, inp["logits_d"], w.tau_d, u_draft, ws, out=d_out),
              R * w.Vd * esz)
        timed("union_verify", lambda: binding.tli_union_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d,
                                                               d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws,
                                                               out=v_out), positions * w.Vt * esz + w.B * w.Vd * esz)
        ar = binding.tli_acceptance_rates(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d)
        timed("acceptance_rates", lambda: binding.tli_acceptance_rates(m, inp["logits_t"], inp["logits_d"], w.tau_t,
                                                                       w.tau_d, workspace=ar["workspace"]),
              positions * (w.Vt + 2 * w.Vd) * esz)
        ok = ar["status"] == 0
        next_rows["mean_alpha_tli"] = round(float(ar["alpha_tli"][ok].mean()), 4)
        next_rows["mean_alpha_union"] = round(float(ar["alpha_union"][ok].mean()), 4)
        # top-k / top-p warp of the target rows (sweeps for the thresholds + the rewrite; bytes = rows read once)
        warped = torch.empty_like(inp["logits_t"]).reshape(rows_t, w.Vt)
        lt_rows = inp["logits_t"].reshape(rows_t, w.Vt)
        timed("warp_rows_top_k50_top_p0.9", lambda: binding.tli_warp_rows(lt_rows, w.tau_t, 50, 0.9, out=warped),
              rows_t * w.Vt * esz)
        del warped
        wws = torch.empty(int(binding.load_library().tli_warp_workspace_bytes(rows_t, w.Vt, code)), dtype=torch.uint8,
                          device=dev)
        timed("warp_thresholds_top_k50_top_p0.9", lambda: binding.tli_warp_rows(lt_rows, w.tau_t, 50, 0.9, rewrite=False,
                                                                               workspace=wws),
              rows_t * w.Vt * esz)
        timed("warp_thresholds_top_k50", lambda: binding.tli_warp_rows(lt_rows, w.tau_t, 50, 1.0, rewrite=False,
                                                                      workspace=wws), rows_t * w.Vt * esz)
        timed("warp_thresholds_top_p0.9", lambda: binding.tli_warp_rows(lt_rows, w.tau_t, 0, 0.9, rewrite=False,
                                                                       workspace=wws), rows_t * w.Vt * esz)
        # compact drafter layout: rows hold only the shared tokens' logits (a head pruned to the intersection)
        sh_x = torch.from_numpy(np.nonzero(inp["d2t"] >= 0)[0]).to(dev)
        epv = 16 // esz
        c_stride = (w.S + epv - 1) // epv * epv
        cbuf = torch.zeros((w.B, w.K, c_stride), dtype=inp["logits_d"].dtype, device=dev)
        cbuf[:, :, : w.S] = inp["logits_d"].index_select(2, sh_x)
        ldc = cbuf[:, :, : w.S]
        step()
        timed("draft_sample_compact", lambda: binding.tli_draft_sample_compact(
            m, cbuf.reshape(R, c_stride)[:, : w.S], w.tau_d, u_draft, ws, out=d_out), R * w.S * esz)
        timed("verify_compact", lambda: binding.tli_verify_compact(
            m, inp["logits_t"], ldc, w.tau_t, w.tau_d, d_out["tok_d"], d_out["lse_q"], u_acc, inp["u_fin"], ws, out=v_out),
            positions * w.Vt * esz + w.B * w.S * esz)
        del cbuf, ldc
        # restore the TLI drafts for the figures below
        step()
        torch.cuda.synchronize()

    breakdown = None
    if args.breakdown:
        binding.tli_profile_enable(binding.KERNELS, n_sep)
        for _ in range(n_sep):
            step()
        torch.cuda.synchronize()
        breakdown = {}
        for k in binding.KERNELS:
            ms, n = binding.tli_profile_collect(k)
            breakdown[k + "_us"] = round(1e3 * ms / max(n, 1), 2)
        binding.tli_profile_disable()

    # ---- algorithmic bytes
    n_acc = v_out["n_accepted"].cpu().numpy()
    lse_bytes = positions * w.Vt * esz                       # K target rows per sequence, once
    n_bonus = int((n_acc == w.K).sum())
    verify_bytes = lse_bytes + n_bonus * w.Vt * esz + (w.B - n_bonus) * w.Vd * esz
    draft_bytes = R * w.Vd * esz
    lse_avg_s = 1e-3 * lse_ms / max(lse_n, 1)
    achieved = lse_bytes / lse_avg_s / 1e9
    call_gbs = verify_bytes / (1e-3 * verify_wall_ms) / 1e9
    traffic = MEASURED_TRAFFIC.get(w.name)
    roofline = dict(bound="hbm", kernel=DOMINANT_KERNEL[w.B >= 200], achieved=round(achieved, 1),
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=traffic["bytes"] if traffic else None,
                    traffic_source=traffic["source"] if traffic else None,
                    bytes_per_launch=lse_bytes, avg_launch_us=round(1e6 * lse_avg_s, 2), launches=lse_n,
                    # the whole tli_verify call (every kernel of it) against the same peak: the figure the 70 % target
                    # of the large-vocabulary batch is defined on
                    call=dict(entry="tli_verify", algorithmic_bytes=verify_bytes, ms=round(verify_wall_ms, 4),
                              achieved=round(call_gbs, 1), frac=round(call_gbs / HBM_PEAK_GBS, 4)))
    # the second yardstick: a read-only pass with plain 16-byte loads over the very rows k_lse reads (the target
    # tensor, a workgroup per row as in k_lse; the row's tail beyond whole 4 KB chunks is left out)
    row_bytes = w.Vt * esz // 4096 * 4096
    if row_bytes and (w.Vt * esz) % 16 == 0:
        flat = inp["logits_t"].reshape(-1)
        rd_out = torch.zeros(flat.numel() * esz // row_bytes + 1, dtype=torch.int32, device=dev)
        n_rd = max(5, args.steps // 8)
        read_gbs = {}
        for nt in (0, 1):
            if (w.Vt * esz) % 4096 == 0:  # rows are whole chunks: read the tensor as it lies
                fn = lambda: binding.tli_calib_read(flat, row_bytes, bool(nt), rd_out)
                nbytes = flat.numel() * esz
            else:  # read whole chunks of a contiguous stretch of the same size
                nbytes = flat.numel() * esz // row_bytes * row_bytes
                fn = lambda: binding.tli_calib_read(flat, row_bytes, bool(nt), rd_out, nbytes=nbytes)
            fn()
            read_gbs["nontemporal" if nt else "plain"] = round(nbytes / (1e-3 * time_call(fn, n_rd)) / 1e9, 1)
        roofline["read_kernel_gbs"] = read_gbs
        roofline["frac_of_read_kernel"] = round(achieved / max(read_gbs.values()), 4)
    # what the runtime reports for this device, beside the vendor's 8 TB/s: an HBM3 pin moves 4 bits per cycle of the
    # reported clock (data strobe at twice the clock, both edges)
    info = binding.tli_device_info()
    info["bus_gbs_at_4_bits_per_clock"] = round(4.0 * info["memory_clock_khz"] * 1e3 * info["memory_bus_bits"] / 8 / 1e9, 1)
    roofline["device_reported"] = info
    extra = dict(
        draft_ms=round(draft_ms, 4), verify_ms=round(verify_ms, 4),
        verify_ms_median_min=[round(verify_med_ms, 4), round(verify_min_ms, 4)],
        draft_ms_median_min=[round(draft_med_ms, 4), round(draft_min_ms, 4)],
        verify_without_lse_q_ms=round(verify_no_lse_q_ms, 4),
        verify_only_positions_per_s=round(positions / (1e-3 * verify_ms), 1),
        verify_algorithmic_gbs=round(verify_bytes / (1e-3 * verify_ms) / 1e9, 1),
        verify_frac_of_peak=round(verify_bytes / (1e-3 * verify_ms) / 1e9 / HBM_PEAK_GBS, 4),
        draft_rows_per_s=round(R / (1e-3 * draft_ms), 1),
        draft_algorithmic_gbs=round(draft_bytes / (1e-3 * draft_ms) / 1e9, 1),
        mean_accepted=round(float(n_acc.mean()), 3), cache=cache,
        per_step_iteration=dict(calls=f"{w.K} x tli_draft_sample(R={w.B}) + tli_verify", eager_ms=round(per_step_eager_ms, 4),
                                hip_graph_ms=round(per_step_graph_ms, 4)),
    )
    if breakdown:
        extra["kernel_breakdown"] = breakdown
    if next_rows:
        extra["next_rows"] = next_rows

    # ---- CPU oracle on a bounded sample of the same batch
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        oracle.build()
        cores = min(16, len(os.sched_getaffinity(0)))
        tau_t, tau_d = float(np.float32(w.tau_t)), float(np.float32(w.tau_d))  # the C ABI's temperatures are fp32
        per_seq_s = 0.12 * (w.K * (w.Vt + w.Vd)) / (8 * (256000 + 128256))  # rough single-thread cost
        nseq = args.cpu_seqs or int(max(1, min(w.B, 20.0 * cores / max(per_seq_s, 1e-6))))
        nseq = max(min(nseq, w.B), 1)
        lt = synth.logits_to_numpy(inp["logits_t"][:nseq])
        ld = synth.logits_to_numpy(inp["logits_d"][:nseq])
        ud = inp["u_draft"][:nseq].cpu().numpy().astype(np.float64)
        ua = inp["u_acc"][:nseq].cpu().numpy().astype(np.float64)
        uf = inp["u_fin"][:nseq].cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ds = oracle.draft_sample(ld.reshape(nseq * w.K, w.Vd), tau_d, inp["d2t"], ud, threads=cores)
        oracle.verify(lt, ld, tau_t, tau_d, inp["d2t"], ds["tok_d"], ua, uf, threads=cores)
        c1 = time.perf_counter()
        n1 = max(1, min(nseq, 8))
        s0 = time.perf_counter()
        ds1 = oracle.draft_sample(ld[:n1].reshape(n1 * w.K, w.Vd), tau_d, inp["d2t"], ud[:n1], threads=1)
        oracle.verify(lt[:n1], ld[:n1], tau_t, tau_d, inp["d2t"], ds1["tok_d"], ua[:n1], uf[:n1], threads=1)
        s1 = time.perf_counter()
        cpu = dict(value=round(nseq * w.K / (c1 - c0), 2), unit="positions/s", cores=cores, kind="oracle",
                   sample=f"first {nseq} of {w.B} sequences of the same batch, draft+verify, {cores} threads, "
                          f"{c1 - c0:.1f} s",
                   single_thread_value=round(n1 * w.K / (s1 - s0), 2), single_thread_sample=f"first {n1} sequences",
                   host_cpus=os.cpu_count(), cpu_model=_cpu_model())

    line = dict(
        metric="verified_draft_positions_per_s (tli_verify)", value=round(value, 1), unit="positions/s", n_gpus=1,
        steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=True, scaling="weak",
        vs_baseline=None, spinup_ms=round(spinup_ms, 1), spinup_steps=spin_steps,
        value_is="B*K positions / wall time of one tli_verify call (`steps` calls timed after the timed steps)",
        step_positions_per_s=round(step_value, 1),
        dtype="f32", data="synthetic",
        config=dict(workload=w.name, B=w.B, K=w.K, Vt=w.Vt, Vd=w.Vd, shared=w.S, storage=w.dtype, temp_t=w.tau_t,
                    temp_d=w.tau_d, step="tli_draft_sample(B*K rows) + tli_verify(B sequences)"),
        roofline=roofline, cpu_baseline=cpu, **extra,
    )
    print(json.dumps(line))


if __name__ == "__main__":
    main()
