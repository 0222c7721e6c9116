"""Throughput of the BlockBatch denoising path on one MI355X (LLaDA-8B-shaped synthetic model).

A "step" is one pass of the whole hot path: bb_denoise_step (pack, batched block forward, LM
head, vocabulary reduction) + bb_merge_commit (Eq. 1 commit, merge, sync), plus the periodic
full-sequence refresh whenever R block forwards have run.  `value` is steps/s of a free-running
decode (refreshes included, inputs and weights resident in HBM; a request that finishes inside the
timed region is opened again, so every counted step is a real block forward).  Beside it:

  * the steady-state step (bb_denoise_step + bb_merge_commit at a frozen state with every window fully
    masked, the worst case): median and mean over the timed iterations, each bracketed by events on the
    library's stream; the block forward alone; the periodic refresh alone; the committed-token rate;
  * `roofline`: the weight-streaming MFMA GEMM launches of the block forward against the HBM peak, from
    per-launch HIP events on the library's stream (raw, and with the measured cost of the event packets
    taken off), with the HBM traffic per launch that rocprofv3 counters gave for the same kernels;
  * `roofline_kv`: the block forward's attention launches against the HBM peak (K,V streamed per step);
  * `measured_peaks`: what a plain 16-byte-per-lane copy and a pure MFMA loop reach on this very GPU;
  * `other_workloads`: steady step, refresh and both rooflines for the long-context and 16-request shapes;
  * `cpu_baseline`: the CPU oracle timed on the host for reference.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def stored_gemm_traffic(workload_name):
    """HBM bytes per GEMM launch of a block forward from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each
    scaled by what the counter reads for a plain copy of known size).  Counters cannot be read from inside this
    process, so the figure is the one stored with the profile summary, which names the commit it was measured at:
    a line `gemm_traffic_bytes_per_launch[<workload>] = <bytes> @ <commit>` in profiles/llada_hbm_traffic_pmc.md."""
    try:
        text = open(os.path.join(ROOT, "profiles", "llada_hbm_traffic_pmc.md")).read()
    except OSError:
        return None, None
    m = re.search(r"gemm_traffic_bytes_per_launch\[%s\]\s*=\s*([0-9.eE+]+)\s*@\s*(\w+)" % re.escape(workload_name), text)
    return (float(m.group(1)), m.group(2)) if m else (None, None)


def make_context(w, torch):
    from workload import gen_weights
    from paper_2605_29233_amd import BlockBatch, Limits
    m = w.model
    L = max(w.prompt_lens) + w.gen_len
    step_rows = w.n_requests * sum(min(b, w.gen_len) for b in w.block_sizes)
    bb = BlockBatch(m, w.decode, Limits(w.n_requests, len(w.block_sizes), L, w.gen_len, step_rows))
    bb.load_weights(gen_weights(m, w.seed, device="cuda:0"))
    if os.environ.get("BB_WIDE_FORMAT", "1") == "0":       # measurements: two bf16 activation terms in every GEMM
        bb.wide_format(False)
    torch.cuda.empty_cache()
    return bb, step_rows


def open_all(bb, w):
    from workload import gen_prompt
    from paper_2605_29233_amd import BB_INIT
    ids = [bb.request_open(gen_prompt(w.model, w.seed, r, lp), w.gen_len, w.block_sizes) for r, lp in enumerate(w.prompt_lens)]
    for r in ids:
        bb.refresh([r], BB_INIT)
    return ids


def steady_state(bb, w, ids, steps, warmup, profile_steps, torch):
    """Frozen state right after the initial forward (every window fully masked).  Returns the timings of the
    block forward alone, of denoise + commit per step, the per-class kernel times and the two rooflines."""
    from paper_2605_29233_amd import BB_PERIODIC
    m = w.model
    frozen = [(bb.get_tokens(r).copy(), list(bb.get_stats(r).branch)[:len(w.block_sizes)]) for r in ids]
    for _ in range(warmup):
        bb.denoise_step(ids, want_view=False)
    bb.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        bb.denoise_step(ids, want_view=False)
    bb.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / steps

    # denoise + commit, one pair of events per step on the library's stream (= torch's current stream here);
    # the state is put back between steps, outside the events
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        bb.denoise_step(ids, want_view=False)
        bb.merge_commit(ids, want_stats=False)
        b.record()
        bb.synchronize()
        for r, (X, br) in zip(ids, frozen):
            bb.set_state(r, X, br)
    step_ms = [a.elapsed_time(b) for a, b in ev]

    # per-kernel-class timing of the frozen block forward (HIP events around every launch)
    bb.profile_enable(True)
    for _ in range(profile_steps):
        bb.denoise_step(ids, want_view=False)
    prof = bb.profile_read()
    bb.profile_enable(False)
    g = prof["gemm_skinny"] if prof["gemm_skinny"]["launches"] else prof["gemm_wide"]
    # the event packet after every launch lengthens the profiled forward; its cost per launch is what the
    # profiled forward takes beyond the unprofiled one, spread over the launches
    all_launches = sum(v["launches"] for v in prof.values())
    all_ms = sum(v["total_ms"] for v in prof.values())
    ev_ms = max(0.0, (all_ms - fwd_ms * profile_steps) / max(all_launches, 1))
    n = max(g["launches"], 1)
    raw_ms, corr_ms = g["total_ms"], max(g["total_ms"] - ev_ms * g["launches"], 1e-9)
    per_step = {k: v["total_ms"] / profile_steps for k, v in prof.items()}
    per_step_corr = {k: (v["total_ms"] - ev_ms * v["launches"]) / profile_steps for k, v in prof.items()}
    hbm_bound = g is prof["gemm_skinny"]
    work = 2.0 if os.environ.get("BB_WIDE_FORMAT", "1") == "0" else 1.5
    traffic, commit = stored_gemm_traffic(w.name)
    gbs = g["bytes"] / 1e9 / (raw_ms / 1e3)
    tfl = g["flops"] / 1e12 / (raw_ms / 1e3)
    roof = {"bound": "hbm" if hbm_bound else "mfma",
            "kernel": "gemm_wide_kernel and the LM head's gemm_kernel (MFMA GEMM launches of the block forward: %s)"
                      % ("weight streaming" if hbm_bound else "many rows"),
            "achieved": gbs if hbm_bound else tfl, "peak": HBM_PEAK_GBS if hbm_bound else MFMA_BF16_PEAK_TFLOPS,
            "unit": "GB/s" if hbm_bound else "TFLOP/s",
            "frac": gbs / HBM_PEAK_GBS if hbm_bound else tfl / MFMA_BF16_PEAK_TFLOPS,
            "traffic": traffic, "traffic_unit": "bytes/launch", "traffic_measured_at_commit": commit,
            "algorithmic_bytes_per_launch": g["bytes"] / n, "algorithmic_flops_per_launch": g["flops"] / n,
            "avg_launch_ms": raw_ms / n, "launches": g["launches"],
            "avg_launch_ms_event_corrected": corr_ms / n, "event_packet_ms_per_launch": ev_ms,
            "frac_event_corrected": (g["bytes"] / 1e9 / (corr_ms / 1e3) / HBM_PEAK_GBS) if hbm_bound
            else (g["flops"] / 1e12 / (corr_ms / 1e3) / MFMA_BF16_PEAK_TFLOPS),
            "hbm_gbs": gbs, "mfma_tflops_nominal": tfl, "mfma_work_factor": work, "mfma_tflops_issued": work * tfl,
            "note": "nominal flops 2*M*N*K; issued = matrix-pipe work in bf16-MFMA equivalents: x1.5 with the fp16 + double-rate "
                    "fp8 terms of the layer GEMMs (x2 for the LM head, which keeps two bf16 activation terms)"}
    # attention of the block forward: K and V of every active branch row are streamed once per layer.  Algorithmic
    # bytes = 2 B per cached element (n_kv_heads * head_dim keys + as many values per token); the cache holds two
    # fp16 terms per element, so the kernel actually streams twice that.
    at = prof["attention"]
    rows_tokens = sum(lp + w.gen_len for lp in w.prompt_lens) * len(w.block_sizes)
    kv_bytes = 2.0 * m.n_kv_heads * m.head_dim * 2 * rows_tokens * m.n_layers
    at_ms = at["total_ms"] / profile_steps
    kv = {"bound": "hbm", "kernel": "attention_kernel (block forward, paged K,V of every branch row)",
          "achieved": kv_bytes / 1e9 / (at_ms / 1e3), "peak": HBM_PEAK_GBS, "unit": "GB/s",
          "frac": kv_bytes / 1e9 / (at_ms / 1e3) / HBM_PEAK_GBS,
          "algorithmic_bytes_per_forward": kv_bytes, "streamed_bytes_per_forward": 2 * kv_bytes,
          "frac_of_streamed_bytes": 2 * kv_bytes / 1e9 / (at_ms / 1e3) / HBM_PEAK_GBS,
          "attention_ms_per_forward": at_ms, "launches_per_forward": at["launches"] / profile_steps}

    # refresh alone
    bb.merge_commit(ids, want_stats=False)
    bb.refresh(ids, BB_PERIODIC)
    bb.synchronize()
    t0 = time.perf_counter()
    bb.refresh(ids, BB_PERIODIC)
    bb.synchronize()
    refresh_ms = (time.perf_counter() - t0) * 1e3
    return {"block_forward_ms_steady": fwd_ms, "step_ms_steady_median": statistics.median(step_ms),
            "step_ms_steady_mean": statistics.fmean(step_ms), "steps_per_s_steady_median": 1e3 / statistics.median(step_ms),
            "refresh_ms": refresh_ms, "kernel_ms_per_block_forward": per_step,
            "kernel_ms_per_block_forward_event_corrected": per_step_corr, "roofline": roof, "roofline_kv": kv}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="llada")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--refresh-interval", type=int, default=0, help="override the workload's R (App. E.3 sweeps)")
    ap.add_argument("--tau-sync", type=int, default=-1, help="override the workload's tau_sync (App. E.3 sweeps)")
    ap.add_argument("--profile-steps", type=int, default=8)
    ap.add_argument("--other-workloads", default="llada_long,llada_x16",
                    help="comma-separated workloads whose steady step, refresh and rooflines are reported beside the main one ('' = none)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from workload import workload, gen_weights, gen_prompt
    from paper_2605_29233_amd import BB_INIT, BB_PERIODIC

    w = workload(args.workload)
    if args.refresh_interval > 0 or args.tau_sync >= 0:
        import dataclasses
        d = w.decode
        d = dataclasses.replace(d, refresh_interval=args.refresh_interval if args.refresh_interval > 0 else d.refresh_interval,
                                tau_sync=args.tau_sync if args.tau_sync >= 0 else d.tau_sync)
        w = dataclasses.replace(w, decode=d)
    m = w.model
    torch.cuda.set_device(0)
    bb, step_rows = make_context(w, torch)
    R = w.decode.refresh_interval

    # ---- 1.-3. steady state, per-kernel-class timing, refresh alone -----------------------------------
    ids = open_all(bb, w)
    steady = steady_state(bb, w, ids, args.steps, args.warmup, args.profile_steps, torch)

    # ---- measured peaks on this GPU: a plain copy with the library's access width, a pure MFMA loop ----
    src = torch.ones(1 << 28, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    bb.debug_copy16(src, dst)
    bb.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(8):
        bb.debug_copy16(src, dst)
    e1.record()
    bb.synchronize()
    copy_gbs = 8 * 2 * src.numel() / 1e9 / (e0.elapsed_time(e1) / 1e3)
    if args.copy_calibration:
        assert bool((dst == 1).all())
    del src, dst
    mfma_tflops = bb.debug_mfma_rate()
    peaks = {"copy_read_plus_write_GBps": copy_gbs, "mfma_bf16_32x32x16_TFLOPs": mfma_tflops,
             "copy_frac_of_hbm_peak": copy_gbs / HBM_PEAK_GBS, "mfma_frac_of_nominal_peak": mfma_tflops / MFMA_BF16_PEAK_TFLOPS}
    steady["roofline"]["frac_of_measured_copy"] = steady["roofline"]["hbm_gbs"] / copy_gbs
    steady["roofline"]["issued_mfma_frac_of_measured_rate"] = steady["roofline"]["mfma_tflops_issued"] / mfma_tflops

    # ---- 4. free-running decode: the timed region ---------------------------------------------------
    # Every timed step is a real block forward.  The loop is the library's own driver loop (bb_generate) written out:
    # while no listed request can need a refresh, block forwards and commits are enqueued back to back without reading
    # anything back; then the per-request summaries are read (one synchronisation), a refresh runs for the requests
    # that say it is due, and a request that has finished is closed and opened again (its initial full forward and
    # first commit then fall inside the timed region as extra work, not as a step).  Steps are counted from the
    # device's own forward counters, and the refresh cadence is asserted at every read.
    tally = {"committed": 0, "refresh": 0, "init": 0, "completed": 0}
    prev = {}
    fwd_at_refresh = {}                 # request -> nfe_block when its cache was last rebuilt

    def account(r, st):
        d = sum(st.branch[k].tokens_decoded for k in range(st.n_branches))
        a = prev.get(r, (0, 0))
        tally["committed"] += d - a[0]
        tally["refresh"] += st.nfe_refresh - a[1]
        fwd_at_refresh.setdefault(r, st.nfe_block)       # a request that was just opened: its initial forward built the cache
        prev[r] = (d, st.nfe_refresh)

    def restart(i):
        bb.request_close(ids[i])
        prev.pop(ids[i], None)
        fwd_at_refresh.pop(ids[i], None)
        ids[i] = bb.request_open(gen_prompt(m, w.seed, i, w.prompt_lens[i]), w.gen_len, w.block_sizes)
        bb.refresh([ids[i]], BB_INIT)
        st = bb.merge_commit([ids[i]])[0]
        prev.pop(ids[i], None)
        fwd_at_refresh.pop(ids[i], None)
        tally["init"] += 1
        return st

    stats = [restart(i) for i in range(len(ids))]
    for i, st in enumerate(stats):
        account(ids[i], st)

    def run_steps(n_steps):
        """Runs exactly n_steps batched block forwards (with the refreshes and restarts that fall between them)."""
        done = 0
        while done < n_steps:
            due = [r for r, st in zip(ids, stats) if st.refresh_due and not st.finished]
            if due:
                bb.refresh(due, BB_PERIODIC)
                for r, st in zip(ids, stats):
                    if r in due:
                        fwd_at_refresh[r] = st.nfe_block
            # forwards that may run before any request needs a refresh (a refreshed request has a whole interval)
            quiet = min(R if r in due else R - (st.nfe_block - fwd_at_refresh[r]) for r, st in zip(ids, stats))
            assert quiet >= 1, quiet
            k = min(quiet, 8, n_steps - done)        # (read at least every 8 forwards: one that finishes is then not stepped in vain for long)
            before = [st.nfe_block for st in stats]
            for _ in range(k):
                bb.denoise_step(ids, want_view=False)
                bb.merge_commit(ids, want_stats=False)
            new = [bb.get_stats(r) for r in ids]            # (the first of these waits for the stream)
            done += max(st.nfe_block - b0 for st, b0 in zip(new, before))      # a request that finished on the way ran fewer
            for i, st in enumerate(new):
                account(ids[i], st)
                since = st.nfe_block - fwd_at_refresh[ids[i]]
                assert st.finished or (since <= R and bool(st.refresh_due) == (since >= R)), (since, st.refresh_due, R)
                if st.finished:
                    tally["completed"] += 1
                    st = restart(i)
                    account(ids[i], st)
                stats[i] = st

    run_steps(args.warmup)
    for k in tally:
        tally[k] = 0
    bb.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps)
    bb.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_refresh = tally["refresh"] // max(len(ids), 1)
    committed = tally["committed"]
    ms_per_step = dt * 1e3 / args.steps

    out = {
        "metric": "branch-batched denoise steps/s (free-running, refreshes included), LLaDA-8B shape, 1 MI355X",
        "value": args.steps / dt, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x two-term activations (fp16 + fp8 remainder in the layer GEMMs, bf16 hi+lo in the LM head), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "model_shape": m.name, "requests": w.n_requests, "prompt_len": list(w.prompt_lens),
                   "gen_len": w.gen_len, "block_sizes": list(w.block_sizes), "packed_rows": step_rows,
                   "refresh_interval": R, "tau_dec": w.decode.tau_dec, "tau_sync": w.decode.tau_sync},
        "committed_tokens_per_s": committed / dt, "committed_tokens": committed, "refreshes_in_timed_region": int(n_refresh),
        "requests_completed_in_timed_region": tally["completed"], "initial_forwards_in_timed_region": tally["init"],
        "measured_peaks": peaks,
    }
    out.update(steady)
    bb.close()
    del bb
    torch.cuda.empty_cache()

    # ---- other workloads: steady step, refresh, rooflines (no free-running loop) -----------------------
    others = {}
    for name in [n for n in args.other_workloads.split(",") if n and n != w.name]:
        wo = workload(name)
        bo, rows_o = make_context(wo, torch)
        ido = open_all(bo, wo)
        so = steady_state(bo, wo, ido, max(4, args.steps // 4), 2, 2, torch)
        so["config"] = {"workload": wo.name, "requests": wo.n_requests, "packed_rows": rows_o, "gen_len": wo.gen_len,
                        "prompt_len": [min(wo.prompt_lens), max(wo.prompt_lens)], "block_sizes": list(wo.block_sizes)}
        so["roofline"]["issued_mfma_frac_of_measured_rate"] = so["roofline"]["mfma_tflops_issued"] / mfma_tflops
        others[name] = so
        bo.close()
        del bo
        torch.cuda.empty_cache()
    if others:
        out["other_workloads"] = others

    # ---- 5. the CPU oracle on the host cores (reported baseline, bounded sample) ----------------------
    if not args.no_cpu_baseline:
        from oracle.model import OracleModel
        from oracle.blockbatch import OracleRequest
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        host = {k: v.cpu() for k, v in gen_weights(m, w.seed, device="cuda:0")}
        om = OracleModel(m, host, np.float32)
        del host
        rq = OracleRequest(om, gen_prompt(m, w.seed, 0, w.prompt_lens[0]), w.gen_len, w.block_sizes, w.decode)
        rq.init_forward()
        rq.commit_merge()
        n_cpu, t0 = 0, time.perf_counter()
        while n_cpu < 3 or (time.perf_counter() - t0 < 10 and n_cpu < 12):
            rq.block_forward()
            rq.commit_merge()
            n_cpu += 1
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n_cpu / cdt, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{n_cpu} block steps (block forward + commit/merge, no refresh) of request 0 "
                                         f"after the initial forward, fp32 numpy oracle"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
