#!/usr/bin/env python3
"""Benchmark of the S2D2 hot path on one MI355X: accepted tokens/s per draft+verify step.

One "step" = s2d2_draft + s2d2_verify + s2d2_accept + s2d2_kv_append + s2d2_block_advance on the
whole batch.  The workload is the dense bf16 1.7B-shaped decoder (28 layers, hidden 2048, 16/8
heads of 128, FFN 6144, vocab 151936), batch 1, prefix 512 random tokens, block size 4,
threshold 0.9, consecutive steps on synthetic random-init weights.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per launch of the streaming GEMM on this workload, from the FETCH_SIZE / WRITE_SIZE counter runs
# recorded in profiles/gemm_stream_kernel_config2.md (31.16 MB fetched + 0.26 MB written; 30.45 MB algorithmic)
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 31.4e6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", type=int, default=2, help="workload id (2 is the benchmark configuration)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; result is labelled)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every call of a step from the host instead of replaying a HIP graph of one step")
    ap.add_argument("--seed", type=int, default=0)
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

    import numpy as np
    import torch

    import s2d2_inputs as I
    from paper_2603_25702_amd import Params
    from paper_2603_25702_amd.runner import Session

    if args.calibrate_copy_mib > 0:
        n = args.calibrate_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)  # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst

    wl = I.CONFIGS[args.config]
    cfg = wl.cfg if not args.layers else I.shrink(wl.cfg, n_layers=args.layers)
    if args.right_shifted:
        cfg = dataclasses.replace(cfg, right_shifted=True)
    N, B, K, Wm = wl.batch, wl.block, args.steps, args.warmup
    dev = "cuda:0"
    t0 = time.time()
    weights = I.gen_weights(cfg, args.seed)
    log(f"[bench] weights generated in {time.time() - t0:.1f}s ({cfg.n_params() / 1e6:.0f} M params)")
    lens = I.gen_prefix_lengths(wl, args.seed)
    ids = [I.gen_prefix_ids(cfg, int(lens[n]), args.seed, n) for n in range(N)]
    max_seq = int(lens.max()) + (max(K, Wm) + 2) * B + 64
    table = I.gen_page_table(N, (max_seq + wl.page_size - 1) // wl.page_size, args.seed)
    ses = Session(cfg, weights, N, B, max_seq, wl.page_size, dev, page_table=table)
    t0 = time.time()
    last = [int(x[-1]) for x in ids]
    ses.prefill(ids)
    log(f"[bench] prefix cache of {lens.tolist()} tokens prefilled on the GPU in {time.time() - t0:.2f}s")

    prm = Params(tau=wl.taus[-1] if len(wl.taus) == 1 else 0.9, seed=args.seed, step=0, step_dev=ses.step_dev)
    i32 = torch.int32
    acc_buf = torch.zeros((max(K, Wm), N), dtype=i32, device=dev)
    com_buf = torch.zeros((max(K, Wm), N), dtype=i32, device=dev)

    def run(steps):
        for s in range(steps):
            ses.step(prm, acc_buf[s], com_buf[s])

    run(Wm)
    torch.cuda.synchronize()
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
    log(f"[bench] {K} steps in {elapsed * 1e3:.2f} ms: {committed} tokens committed ({accepted} accepted drafts)")

    # ---- instrumented pass: HIP events around every launch, on the library's stream ----------------
    roofline, phases = None, {}
    if not args.no_profile_pass:
        Kp = min(K, 8)
        ses.reset_blocks(lens, last)
        per_fwd = cfg.n_layers * 8 + 16
        ses.eng.s2d2_profile_start(2 * Kp * per_fwd + 64)
        run(Kp)
        prof = ses.eng.s2d2_profile_stop()
        # dominant kernel: the fused forward (all layer weights of one forward per launch) when the window is narrow
        # enough for it, else the streaming GEMM launches; algorithmic bytes = the weight matrices once per launch
        fused = prof["forward"]["launches"] > 0
        g = prof["forward"] if fused else prof["gemm"]
        ach = g["bytes"] / (g["ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "forward_fused_kernel" if fused else "gemm_stream_kernel",
                    "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH if (args.config == 2 and not fused and not args.layers) else None,
                    "avg_launch_us": round(g["ms"] * 1e3 / g["launches"], 3),
                    "bytes_per_launch": round(g["bytes"] / g["launches"])}
        tot = sum(c["ms"] for c in prof.values())
        for name, c in prof.items():
            phases[name] = {"ms_per_step": round(c["ms"] / Kp, 4), "launches_per_step": c["launches"] // Kp,
                            "share": round(c["ms"] / tot, 4)}
        for name in ("gemm", "forward"):
            if prof[name]["launches"]:
                phases[name]["hbm_GBs"] = round(prof[name]["bytes"] / (prof[name]["ms"] * 1e-3) / 1e9, 1)
        # Per-phase HBM rate and MFMA use from the workload's shapes (nominal rows of fresh blocks: N*B draft rows,
        # 2*N*B verifier rows, N*B logit rows per forward; cached lengths = mean of before and after the pass)
        es = 2 if cfg.dtype == "bf16" else 4
        S_mean = 0.5 * (float(np.sum(lens)) + float(ses.kv.seq_len.sum().item()))
        kv_bytes = 2 * cfg.n_layers * S_mean * 2 * cfg.n_kv_heads * cfg.head_dim * es          # both forwards, K and V once
        attn_flops = cfg.n_layers * (N * B + 2 * N * B) / N * 4.0 * cfg.n_q_heads * cfg.head_dim * S_mean
        per_layer = cfg.d_model * (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim + cfg.n_q_heads * cfg.head_dim * cfg.d_model
        per_layer += (cfg.top_k * 3 * cfg.d_model * cfg.d_expert + cfg.d_model * cfg.n_experts) if cfg.is_moe else 3 * cfg.d_model * cfg.d_ffn
        gemm_flops = 2.0 * (3 * N * B * cfg.n_layers * per_layer + 2 * N * B * cfg.d_model * cfg.vocab)
        vocab_bytes = 2 * N * B * cfg.vocab * 4.0                                                # draft and verifier logits read once
        MFMA_PEAK = 2.5e15 if cfg.dtype == "bf16" else 157.3e12
        if prof["attention"]["launches"]:
            t = prof["attention"]["ms"] * 1e-3 / Kp
            phases["attention"]["hbm_GBs"] = round(kv_bytes / t / 1e9, 1)
            phases["attention"]["mfma_pct"] = round(100 * attn_flops / t / MFMA_PEAK, 2)
        if prof["gemm"]["launches"]:
            phases["gemm"]["mfma_pct"] = round(100 * gemm_flops / (prof["gemm"]["ms"] * 1e-3 / Kp) / MFMA_PEAK, 2)
        if prof["vocab"]["launches"]:
            phases["vocab"]["hbm_GBs"] = round(vocab_bytes / (prof["vocab"]["ms"] * 1e-3 / Kp) / 1e9, 1)
        log(f"[bench] profile pass ({Kp} steps): {json.dumps(phases)}")

    # ---- the fp64 oracle on the host cores: a bounded sample of full steps of the same workload -----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import s2d2_oracle as O  # test infrastructure, used for the reported CPU baseline only
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        ses.reset_blocks(lens, last)
        torch.cuda.synchronize()
        k_cpu, v_cpu = ses.kv.k.cpu(), ses.kv.v.cpu()
        tb = ses.kv.page_table.cpu().numpy()
        ps = wl.page_size
        t0 = time.perf_counter()
        tokens = 0
        n_seq, n_steps = 1, 0  # bounded sample: one sequence, consecutive steps until about 10 s have been spent (at most 4)
        for n in range(n_seq):
            S = int(lens[n])
            pages = torch.as_tensor(tb[n, :(S + ps - 1) // ps].astype(np.int64))
            ck = [k_cpu[l][pages].permute(0, 2, 1, 3).reshape(-1, cfg.n_kv_heads, cfg.head_dim)[:S] for l in range(cfg.n_layers)]
            cv = [v_cpu[l][pages].permute(0, 3, 1, 2).reshape(-1, cfg.n_kv_heads, cfg.head_dim)[:S] for l in range(cfg.n_layers)]
            st = O.SeqState(S, S, np.full(B, cfg.mask_id, dtype=np.int64))
            if args.right_shifted:
                st = O.shifted_prefill_state(S, last[n], B, cfg.mask_id)
                ck, cv = [x[:S - 1] for x in ck], [x[:S - 1] for x in cv]
            while True:
                _, _, a = O.step(cfg, weights, st, ck, cv, prm.tau, args.seed, n_steps, n)
                tokens += a.n_commit
                n_steps += 1
                if time.perf_counter() - t0 >= 10.0 or n_steps >= 4:
                    break
        dt = time.perf_counter() - t0
        cpu = {"value": round(tokens / dt * (N / n_seq), 4), "unit": "accepted tokens/s", "cores": int(cores),
               "kind": "oracle", "sample": f"{n_seq} sequence(s) x {n_steps} consecutive draft+verify+accept+append step(s) of the "
               f"same workload (fp64 numpy, {dt:.1f}s)"}
        log(f"[bench] oracle: {n_steps} step(s) in {dt:.1f}s, {tokens} tokens")

    out = {
        "metric": "accepted tokens/s per draft+verify step", "value": round(value, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(elapsed * 1e3 / K, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "launch": "host calls" if args.no_graph else "hip graph of one step, replayed",
        "config": {"workload": f"config {args.config}: {cfg.name} {cfg.n_layers}L d{cfg.d_model} V{cfg.vocab}, batch {N}, "
                               f"prefix {int(lens.min())}-{int(lens.max())}, block {B}, tau {prm.tau}, {K} consecutive steps"
                               + (", right-shifted model" if args.right_shifted else ""),
                   "tokens_committed": committed, "drafts_accepted": accepted},
        "roofline": roofline, "cpu_baseline": cpu, "phases": phases,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
