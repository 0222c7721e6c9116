"""Throughput of the BlockBatch denoising path on one MI355X (LLaDA-8B-shaped synthetic model).

A "step" is one pass of the whole hot path: bb_denoise_step (pack, batched block forward, LM
head, vocabulary reduction) + bb_merge_commit (Eq. 1 commit, merge, sync), plus the periodic
full-sequence refresh whenever R block forwards have run.  `value` is steps/s of a free-running
decode (refreshes included, inputs and weights resident in HBM; a request that finishes inside the
timed region is opened again, so every counted step is a real block forward); the steady-state block forward,
the refresh and the committed-token rate are reported beside it.  The roofline figure is for the
weight-streaming MFMA GEMM launches of the block forward at a frozen, fully masked state, timed
with HIP events on the library's stream; the CPU oracle is timed on the host for reference.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


# HBM bytes per GEMM launch of a block forward from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), each scaled
# by what the counter reads for a plain 16-byte-per-lane copy of known size (FETCH_SIZE x 2.000, WRITE_SIZE x
# 1.000); the per-kernel table and the commands are in profiles/llada_hbm_traffic_pmc.md.  Counters cannot be
# read from inside this process, so the figure is the stored one for the workload it was measured on.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {"llada": 152.8e6}


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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from workload import workload, gen_weights, gen_prompt
    from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT, BB_PERIODIC

    w = workload(args.workload)
    if args.refresh_interval > 0 or args.tau_sync >= 0:
        import dataclasses
        d = w.decode
        d = dataclasses.replace(d, refresh_interval=args.refresh_interval if args.refresh_interval > 0 else d.refresh_interval,
                                tau_sync=args.tau_sync if args.tau_sync >= 0 else d.tau_sync)
        w = dataclasses.replace(w, decode=d)
    m = w.model
    L = max(w.prompt_lens) + w.gen_len
    step_rows = w.n_requests * sum(min(b, w.gen_len) for b in w.block_sizes)
    torch.cuda.set_device(0)
    bb = BlockBatch(m, w.decode, Limits(w.n_requests, len(w.block_sizes), L, w.gen_len, step_rows))
    bb.load_weights(gen_weights(m, w.seed, device="cuda:0"))
    torch.cuda.empty_cache()

    def open_all():
        ids = [bb.request_open(gen_prompt(m, w.seed, r, lp), w.gen_len, w.block_sizes) for r, lp in enumerate(w.prompt_lens)]
        for r in ids:
            bb.refresh([r], BB_INIT)
        return ids

    def decoded(stats):
        return sum(st.branch[k].tokens_decoded for st in stats for k in range(st.n_branches))

    R = w.decode.refresh_interval

    # ---- 1. steady state at a frozen, fully masked state: block forward only --------------------
    ids = open_all()
    for _ in range(args.warmup):
        bb.denoise_step(ids, want_view=False)
    bb.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        bb.denoise_step(ids, want_view=False)
    bb.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- 2. per-kernel-class timing of the same frozen block forward (HIP events) ---------------
    bb.profile_enable(True)
    for _ in range(args.profile_steps):
        bb.denoise_step(ids, want_view=False)
    prof = bb.profile_read()
    bb.profile_enable(False)
    g = prof["gemm_skinny"] if prof["gemm_skinny"]["launches"] else prof["gemm_wide"]
    # The event packet after every launch lengthens the profiled forward; its cost per launch is what the profiled
    # forward takes beyond the unprofiled one (measured just above), spread over the launches, and is taken off.
    all_launches = sum(v["launches"] for v in prof.values())
    all_ms = sum(v["total_ms"] for v in prof.values())
    ev_ms = max(0.0, (all_ms - fwd_ms * args.profile_steps) / max(all_launches, 1))
    gemm_raw_ms = g["total_ms"] / max(g["launches"], 1)
    gemm_total_ms = max(g["total_ms"] - ev_ms * g["launches"], 1e-9)
    gemm_ms = gemm_total_ms / max(g["launches"], 1)
    gemm_gbs = g["bytes"] / 1e9 / (gemm_total_ms / 1e3)
    gemm_tflops = g["flops"] / 1e12 / (gemm_total_ms / 1e3)
    per_step = {k: (v["total_ms"] - ev_ms * v["launches"]) / args.profile_steps for k, v in prof.items()}

    # ---- 3. refresh alone --------------------------------------------------------------------------
    bb.merge_commit(ids, want_stats=False)
    bb.refresh(ids, BB_PERIODIC)
    bb.synchronize()
    t0 = time.perf_counter()
    bb.refresh(ids, BB_PERIODIC)
    bb.synchronize()
    refresh_ms = (time.perf_counter() - t0) * 1e3

    # ---- 4. free-running decode: the timed region ---------------------------------------------------
    # Every timed step is a real block forward: the per-request flags are read back after each commit (one
    # small copy; the launches of the next step still run ahead of the GPU), a refresh runs when a request
    # says it is due, and a request that has finished is closed and opened again (its initial full forward
    # and first commit then fall inside the timed region as extra work, not as a step).
    tally = {"committed": 0, "refresh": 0, "init": 0, "completed": 0}
    prev = {}

    def account(r, st):
        d = sum(st.branch[k].tokens_decoded for k in range(st.n_branches))
        a = prev.get(r, (0, 0))
        tally["committed"] += d - a[0]
        tally["refresh"] += st.nfe_refresh - a[1]
        prev[r] = (d, st.nfe_refresh)

    def restart(i):
        bb.request_close(ids[i])
        ids[i] = bb.request_open(gen_prompt(m, w.seed, i, w.prompt_lens[i]), w.gen_len, w.block_sizes)
        bb.refresh([ids[i]], BB_INIT)
        st = bb.merge_commit([ids[i]])[0]
        prev.pop(ids[i], None)
        tally["init"] += 1
        return st

    stats = [restart(i) for i in range(len(ids))]

    def one_step():
        due = [r for r, st in zip(ids, stats) if st.refresh_due and not st.finished]
        if due:
            bb.refresh(due, BB_PERIODIC)
        bb.denoise_step(ids, want_view=False)
        new = bb.merge_commit(ids)
        for i, st in enumerate(new):
            account(ids[i], st)
            if st.finished:
                tally["completed"] += 1
                st = restart(i)
                account(ids[i], st)
            stats[i] = st

    for _ in range(args.warmup):
        one_step()
    for k in tally:
        tally[k] = 0
    bb.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
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
        "dtype": "bf16 weights x (bf16 hi+lo) activations, fp32 accumulate", "data": "synthetic",
        "config": {"workload": w.name, "model_shape": m.name, "requests": w.n_requests, "prompt_len": list(w.prompt_lens),
                   "gen_len": w.gen_len, "block_sizes": list(w.block_sizes), "packed_rows": step_rows,
                   "refresh_interval": R, "tau_dec": w.decode.tau_dec, "tau_sync": w.decode.tau_sync},
        "committed_tokens_per_s": committed / dt, "committed_tokens": committed, "refreshes_in_timed_region": int(n_refresh),
        "requests_completed_in_timed_region": tally["completed"], "initial_forwards_in_timed_region": tally["init"],
        "block_forward_ms_steady": fwd_ms, "block_forward_steps_per_s_steady": 1e3 / fwd_ms, "refresh_ms": refresh_ms,
        "kernel_ms_per_block_forward": per_step,
        "roofline": {"bound": "hbm", "kernel": "gemm_kernel (weight-streaming MFMA GEMM, block forward)",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(w.name), "traffic_unit": "bytes/launch",
                     "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1),
                     "avg_launch_ms": gemm_ms, "avg_launch_ms_with_event_packets": gemm_raw_ms,
                     "event_packet_ms_per_launch": ev_ms, "launches": g["launches"],
                     "mfma_tflops": gemm_tflops, "mfma_frac_of_bf16_peak": gemm_tflops / MFMA_BF16_PEAK_TFLOPS},
    }
    if args.copy_calibration:
        # one plain copy of known size (256 MiB in, 256 MiB out, 16 bytes per lane like the library's kernels)
        src = torch.ones(1 << 28, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        bb.debug_copy16(src, dst)
        bb.synchronize()
        assert bool((dst == 1).all())
        del src, dst
    bb.close()
    del bb
    torch.cuda.empty_cache()

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
