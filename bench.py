#!/usr/bin/env python3
"""Benchmark of the S2D2 hot path on one MI355X: accepted tokens/s per draft+verify step.

One "step" = s2d2_draft + s2d2_verify + s2d2_accept + s2d2_kv_append + s2d2_block_advance on the whole batch,
replayed as a HIP graph.  The headline workload is the largest single-GPU configuration, config 4 (dense bf16
8B-shaped decoder: 36 layers, hidden 4096, 32/8 heads of 128, FFN 12288, vocab 151936; batch 16, prefix 8192,
block 16, threshold 0.9, paged cache with 16-token pages), on synthetic random-init weights with the prefix cache
prefilled through the library.  Everything is resident in HBM before the timed region.  The other bf16
configurations (2, 3, 5) are measured the same way and reported under "configs".  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import dataclasses
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # dense MFMA peak of the arithmetic type (f16 and bf16 MFMA run at the same rate)
HEADLINE, OTHERS = 4, (2, 3, 5)
# HBM-side bytes (L2 misses, both directions) per launch of the dominant GEMM kernel of a configuration and per
# step, from the FETCH_SIZE / WRITE_SIZE counter runs summarised under profiles/ (rocprofv3 --pmc on this file with
# the default operand mode; a plain copy of 1 GiB reads FETCH_SIZE = 524300 KiB and WRITE_SIZE = 1048576 KiB, so
# bytes = FETCH_SIZE KiB * 2048 + WRITE_SIZE KiB * 1024).  Averages over all GEMM launches of two steps.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {2: 31224525, 3: 89565184, 4: 199932416, 5: 340076037}
STEP_TRAFFIC_BYTES = {   # all kernels of a step: (FETCH_SIZE KiB * 2048 + WRITE_SIZE KiB * 1024) summed over the step's launches
    2: (1690673.1 + 3417419.0 + 3216.1) * 2048 + (44688.0 + 56515.1 + 649.7) * 1024,
    3: (3967161.5 + 10775508.1 + 41642.3) * 2048 + (1853479.4 + 3814144.6 + 10579.1) * 1024,
    4: (20326794.5 + 23919422.5 + 159398.6) * 2048 + (3800861.3 + 8782625.1 + 29411.1) * 1024,
    5: (4899233.2 + 278935.0 + 29215321.8 + 2673974.5) * 2048 + (2783471.0 + 14287.5 + 8082510.8 + 839212.4) * 1024,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bench_config(args, cfg_id: int, K: int, Wm: int, cpu_baseline: bool) -> dict:
    import numpy as np
    import torch

    import s2d2_inputs as I
    from paper_2603_25702_amd import Params
    from paper_2603_25702_amd.runner import Session

    wl = I.CONFIGS[cfg_id]
    cfg = wl.cfg if not args.layers else I.shrink(wl.cfg, n_layers=args.layers)
    if args.right_shifted:
        cfg = dataclasses.replace(cfg, right_shifted=True)
    N, B = wl.batch, wl.block
    dev = "cuda:0"
    t0 = time.time()
    weights = I.gen_weights(cfg, args.seed)
    log(f"[bench] config {cfg_id}: weights generated in {time.time() - t0:.1f}s ({cfg.n_params() / 1e6:.0f} M params)")
    lens = I.gen_prefix_lengths(wl, args.seed)
    ids = [I.gen_prefix_ids(cfg, int(lens[n]), args.seed, n) for n in range(N)]
    max_seq = int(lens.max()) + (max(K, Wm) + 2) * B + 64
    table = I.gen_page_table(N, (max_seq + wl.page_size - 1) // wl.page_size, args.seed)
    ses = Session(cfg, weights, N, B, max_seq, wl.page_size, dev, page_table=table, act_planes=args.act_planes)
    t0 = time.time()
    last = [int(x[-1]) for x in ids]
    ses.prefill(ids)
    log(f"[bench] prefix cache of {int(lens.min())}-{int(lens.max())} tokens x {N} prefilled on the GPU in {time.time() - t0:.2f}s")

    tau = wl.taus[-1] if len(wl.taus) == 1 else 0.9
    prm = Params(tau=tau, seed=args.seed, step=0, step_dev=ses.step_dev)
    i32 = torch.int32
    acc_buf = torch.zeros((max(K, Wm), N), dtype=i32, device=dev)
    com_buf = torch.zeros((max(K, Wm), N), dtype=i32, device=dev)

    def run(steps):
        for s in range(steps):
            ses.step(prm, acc_buf[s], com_buf[s])

    run(Wm)
    torch.cuda.synchronize()
    graph = None
    if args.no_graph:
        ses.reset_blocks(lens, last)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(K)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        committed = int(com_buf[:K].sum().item())
        accepted = int(acc_buf[:K].sum().item())
    else:
        # one step = one HIP graph (every kernel of draft, verify, accept, append, advance); K replays are timed
        graph = ses.capture_step(prm)
        ses.reset_blocks(lens, last)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        committed = int(ses.tot_commit.sum().item())
        accepted = int(ses.tot_accept.sum().item())
    assert int(ses.kv.status.abs().sum().item()) == 0, "a sequence ran out of cache pages"
    ses.eng.s2d2_status()   # raises if a bounded device-side wait ran out during the timed steps (results would be invalid)
    value = committed / elapsed
    log(f"[bench] config {cfg_id}: {K} steps in {elapsed * 1e3:.2f} ms: {committed} tokens committed ({accepted} accepted drafts)")

    # ---- instrumented pass: HIP events stamped by every dispatch, on the library's stream ----------------
    roofline, phases = None, {}
    if not args.no_profile_pass:
        Kp = min(K, 8)
        ses.reset_blocks(lens, last)
        per_fwd = cfg.n_layers * 10 + 16
        ses.eng.s2d2_profile_start(2 * Kp * per_fwd + 64)
        run(Kp)
        prof = ses.eng.s2d2_profile_stop()
        mfma_peak = MFMA_PEAK_TFLOPS["bf16" if cfg.dtype == "bf16" else "f32"]
        tot = sum(prof[c]["ms"] for c in ("gemm", "attention", "vocab", "other"))
        for name, c in prof.items():
            if not c["launches"]:
                continue
            phases[name] = {"ms_per_step": round(c["ms"] / Kp, 4), "launches_per_step": c["launches"] // Kp,
                            "share": round(c["ms"] / tot, 4)}
            if name.startswith("gemm"):   # weight bytes once per launch; the method's flops counted once
                phases[name]["hbm_GBs"] = round(c["bytes"] / (c["ms"] * 1e-3) / 1e9, 1)
                phases[name]["mfma_TFLOPs"] = round(c["flops"] / (c["ms"] * 1e-3) / 1e12, 1)
                phases[name]["hbm_frac"] = round(phases[name]["hbm_GBs"] / HBM_PEAK_GBS, 4)
                phases[name]["mfma_frac"] = round(phases[name]["mfma_TFLOPs"] / mfma_peak, 4)
        # attention and vocabulary phases from the workload's shapes (nominal rows of fresh blocks: N*B draft rows,
        # 2*N*B verifier rows; cached lengths = mean of before and after the pass)
        es = 2 if cfg.dtype == "bf16" else 4
        S_mean = 0.5 * (float(np.sum(lens)) + float(ses.kv.seq_len.sum().item()))
        kv_bytes = 2 * cfg.n_layers * S_mean * 2 * cfg.n_kv_heads * cfg.head_dim * es          # both forwards, K and V once
        attn_flops = cfg.n_layers * 3 * B * 4.0 * cfg.n_q_heads * cfg.head_dim * S_mean
        vocab_bytes = 2 * N * B * cfg.vocab * 4.0                                                # draft and verifier logits read once
        if prof["attention"]["launches"]:
            t = prof["attention"]["ms"] * 1e-3 / Kp
            phases["attention"].update(hbm_GBs=round(kv_bytes / t / 1e9, 1), hbm_frac=round(kv_bytes / t / 1e9 / HBM_PEAK_GBS, 4),
                                       mfma_TFLOPs=round(attn_flops / t / 1e12, 1), kv_bytes_per_step=round(kv_bytes))
        if prof["vocab"]["launches"]:
            t = prof["vocab"]["ms"] * 1e-3 / Kp
            phases["vocab"].update(hbm_GBs=round(vocab_bytes / t / 1e9, 1), hbm_frac=round(vocab_bytes / t / 1e9 / HBM_PEAK_GBS, 4))
        # dominant kernel: the GEMM kernel of this window width (all its launches of a step).  It is bound by the
        # matrix pipes when the method's flops at the MFMA peak take longer than its weight bytes at the HBM peak.
        g = prof["gemm"]
        wide = 3 * N * B > 32                     # windows above 32 rows run the LDS-tiled kernel (launch_gemm_stream)
        t_mfma, t_hbm = g["flops"] / (mfma_peak * 1e12), g["bytes"] / (HBM_PEAK_GBS * 1e9)
        common = {"kernel": "gemm_tile_kernel" if wide else "gemm_stream_kernel",
                  "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(cfg_id) if not (args.layers or args.right_shifted) else None,
                  "avg_launch_us": round(g["ms"] * 1e3 / g["launches"], 3), "launches_per_step": g["launches"] // Kp,
                  "bytes_per_launch": round(g["bytes"] / g["launches"]), "flops_per_launch": round(g["flops"] / g["launches"])}
        if t_mfma > t_hbm:
            ach = g["flops"] / (g["ms"] * 1e-3) / 1e12
            roofline = {"bound": "mfma", "achieved": round(ach, 1), "peak": mfma_peak, "unit": "TFLOP/s",
                        "frac": round(ach / mfma_peak, 4), **common}
        else:
            ach = g["bytes"] / (g["ms"] * 1e-3) / 1e9
            roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(ach / HBM_PEAK_GBS, 4), **common}
        # the step against its own bound: weights of both forwards + cached K/V + logits at the HBM peak
        step_bytes = g["bytes"] / Kp + kv_bytes + vocab_bytes
        roofline["step_hbm_bound_ms"] = round(step_bytes / (HBM_PEAK_GBS * 1e9) * 1e3, 3)
        roofline["step_hbm_frac"] = round(step_bytes / (HBM_PEAK_GBS * 1e9) / (elapsed / K), 4)
        if common["traffic"] is not None:   # counters: what the whole step moved over what it must move at least once
            roofline["step_traffic"] = round(STEP_TRAFFIC_BYTES[cfg_id])
            roofline["step_traffic_over_algorithmic"] = round(STEP_TRAFFIC_BYTES[cfg_id] / step_bytes, 3)
        log(f"[bench] config {cfg_id}: profile pass ({Kp} steps): {json.dumps(phases)}")

    # ---- the fp64 oracle on the host cores: a bounded sample of full steps of the same workload -----
    cpu = None
    if cpu_baseline:
        from oracle import s2d2_oracle as O  # test infrastructure, used for the reported CPU baseline only
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        ses.reset_blocks(lens, last)
        torch.cuda.synchronize()
        n = int(np.argmax(lens))           # the sequence with the longest prefix
        tb = ses.kv.page_table.cpu().numpy()
        ps = wl.page_size
        S = int(lens[n])
        pages = torch.as_tensor(tb[n, :(S + ps - 1) // ps].astype(np.int64), device=dev)
        ck = [ses.kv.k[l][pages].permute(0, 2, 1, 3).reshape(-1, cfg.n_kv_heads, cfg.head_dim)[:S].cpu() for l in range(cfg.n_layers)]
        cv = [ses.kv.v[l][pages].permute(0, 3, 1, 2).reshape(-1, cfg.n_kv_heads, cfg.head_dim)[:S].cpu() for l in range(cfg.n_layers)]
        st = O.SeqState(S, S, np.full(B, cfg.mask_id, dtype=np.int64))
        if args.right_shifted:
            st = O.shifted_prefill_state(S, last[n], B, cfg.mask_id)
            ck, cv = [x[:S - 1] for x in ck], [x[:S - 1] for x in cv]
        w64 = O.LazyF64Weights(weights) if cfg.is_moe else weights   # same stored values; expert up-casts cached per layer
        t0 = time.perf_counter()
        tokens, n_steps = 0, 0   # bounded sample: one sequence, consecutive steps until about 10 s have been spent (at most 4)
        while True:
            _, _, a = O.step(cfg, w64, st, ck, cv, prm.tau, args.seed, n_steps, n)
            tokens += a.n_commit
            n_steps += 1
            log(f"[bench] config {cfg_id}: oracle step {n_steps} done after {time.perf_counter() - t0:.1f}s")
            if time.perf_counter() - t0 >= 10.0 or n_steps >= 4:
                break
        dt = time.perf_counter() - t0
        cpu = {"value": round(tokens / dt * N, 4), "unit": "accepted tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"1 of {N} sequence(s) (the longest prefix) x {n_steps} consecutive draft+verify+accept+append step(s) of the "
                         f"same workload (fp64 numpy, {dt:.1f}s)" + (f"; sequences are independent: rate extrapolated x{N}" if N > 1 else "")}
        log(f"[bench] config {cfg_id}: oracle: {n_steps} step(s) of one sequence in {dt:.1f}s, {tokens} tokens")

    rec = {
        "value": round(value, 2), "unit": "tokens/s", "steps": K, "warmup": Wm, "ms_per_step": round(elapsed * 1e3 / K, 4),
        "dtype": ("f16" if args.act_planes in (0, 3) else "bf16") if cfg.dtype == "bf16" else cfg.dtype,
        "operands": {0: "GEMM inputs as IEEE half against a half copy of the bf16 weights (f16 MFMA, fp32 accumulate); queries, keys, values and the KV cache bf16",
                     3: "GEMM inputs as IEEE half against a half copy of the bf16 weights (f16 MFMA, fp32 accumulate); queries, keys, values and the KV cache bf16",
                     2: "GEMM inputs as bf16 hi + lo planes against the bf16 weights (bf16 MFMA issued twice, fp32 accumulate)",
                     1: "GEMM inputs as one bf16 plane (outside the logit tolerance on the 36-layer configurations)"}[args.act_planes] if cfg.dtype == "bf16" else "fp32",
        "launch": "host calls" if args.no_graph else "hip graph of one step, replayed",
        "config": {"workload": f"config {cfg_id}: {cfg.name} {cfg.n_layers}L d{cfg.d_model} V{cfg.vocab}, batch {N}, "
                               f"prefix {int(lens.min())}-{int(lens.max())}, block {B}, tau {prm.tau}, {K} consecutive steps"
                               + (", right-shifted model" if args.right_shifted else "")
                               + (f", act_planes={args.act_planes}" if args.act_planes else ""),
                   "tokens_committed": committed, "drafts_accepted": accepted},
        "roofline": roofline, "cpu_baseline": cpu, "phases": phases,
    }
    ses.eng.close()
    del ses, weights, graph
    gc.collect()
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0, help="measure only this workload id (default: config 4 as the headline, "
                                                           "then configs 2, 3 and 5 under \"configs\")")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; result is labelled)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-cpu-baselines", action="store_true", help="time the oracle for the configurations under \"configs\" too (about 15 s each)")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every call of a step from the host instead of replaying a HIP graph of one step")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--act-planes", type=int, default=0, help="operand mode of the GEMMs (s2d2_model_desc.act_planes): 0/3 half "
                                                               "values (default), 2 two bf16 planes, 1 one bf16 plane; the result is labelled")
    ap.add_argument("--right-shifted", action="store_true",
                    help="treat the synthetic model as right-shifted (output at position i-1 scores token i): plain causal "
                         "verifier rows instead of the 2L window; the result is labelled")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="counter calibration: first run a plain elementwise copy kernel over this many MiB "
                         "(read once, written once) so that a rocprofv3 --pmc run of this command holds a kernel of "
                         "known HBM traffic next to the library's kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (sequences are independent, so more GPUs would be plain "
                 "data parallelism with no exchange); run with --gpus 1")

    import torch

    if args.calibrate_copy_mib > 0:
        n = args.calibrate_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)  # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst

    head_id = args.config or HEADLINE
    head = bench_config(args, head_id, args.steps, args.warmup, not args.no_cpu_baseline)
    out = {
        "metric": "accepted tokens/s per draft+verify step", "value": head["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "operands": head["operands"], "data": "synthetic",
        "launch": head["launch"], "config": head["config"], "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"], "phases": head["phases"],
    }
    if not args.config:   # the other bf16 configurations, same measurement each
        out["configs"] = {}
        for cid in OTHERS:
            try:
                out["configs"][str(cid)] = bench_config(args, cid, args.steps, args.warmup, args.all_cpu_baselines)
            except Exception as e:   # the headline line is still printed
                log(f"[bench] config {cid} failed: {type(e).__name__}: {e}")
                out["configs"][str(cid)] = {"error": f"{type(e).__name__}: {e}"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
