#!/usr/bin/env python3
"""Benchmark of the module-replica hot path on ONE MI355X.

A step = one replicated forward (split -> k replica forwards on their streams -> join) of the
Llama-2-7B-shaped decoder layer in a decode step: batch 32, 1024 cached positions per sequence
(BASELINE configs[1]), bf16, seeded synthetic tensors resident in HBM before timing starts.
`value` is tokens/s at k = 1; k = 2 and k = 4 (same total batch) and the replica-clone rate are
reported beside it.  The `roofline` object prices the dominant kernel (decode attention) against
HBM; `cpu_baseline` is the CPU oracle timed on this machine's host cores.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
METRIC = "decoder-layer tokens/s (7B shape, k=1/2/4 replicas); module replicate GB/s"

# HBM bytes per launch of the decode-attention kernel on configs[1], from two `rocprofv3 --pmc`
# runs (FETCH_SIZE, WRITE_SIZE) scaled by the same counters on the clone kernel of known size;
# see profiles/decoder_layer_decode_C2_k1_pmc_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {"attn_decode@C2": 540769864}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replicas", type=str, default="1,2,4")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (replicas are HIP streams of one MI355X, no "
              "collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    from paper_2507_18006_amd import binding as B
    if not os.path.exists(B.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    from tests import gpu_util as U

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU fallback)"
    cfg = workloads.CONFIGS["C2"]
    K, W = args.steps, args.warmup
    ks = [int(v) for v in args.replicas.split(",")]

    w = workloads.make_weights(cfg, 0)
    inp = workloads.make_inputs(cfg, 0)
    m = U.make_module(cfg, w)
    db = U.DeviceBatch(m, cfg, inp)
    torch.cuda.synchronize()

    n_tok = cfg.n_seqs
    arena = m.arena_bytes
    kv_bytes = int((inp.lens.astype(np.int64) + 1).sum()) * cfg.n_kv_heads * cfg.head_dim * 2 * 2
    act_bytes = n_tok * (2 * cfg.hidden + 2 * cfg.n_kv_heads * cfg.head_dim) * 2   # x in, y out, new K/V out

    def timed(k, stages=()):
        m.replicate(k)
        m.profile(stages)
        for _ in range(W):
            m.forward_split(db.batch)
        torch.cuda.synchronize()
        for j in range(k):
            m.profile_read(j, reset=True)
        t0 = time.perf_counter()
        for _ in range(K):
            m.forward_split(db.batch)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = [m.profile_read(j, reset=True) for j in range(k)]
        m.profile([])
        return dt / K, prof

    per_k = {}
    # k = 1: the timed region also brackets the dominant kernel with HIP events on its stream
    t1, prof1 = timed(1, ("attn",))
    attn_ms, attn_n = prof1[0]["attn"]
    attn_avg_s = attn_ms / attn_n * 1e-3
    per_k[1] = t1
    for k in ks:
        if k != 1:
            per_k[k], _ = timed(k)

    # per-kernel breakdown at k = 1 (separate pass: bracketing every launch perturbs the step)
    _, prof_all = timed(1, None)
    breakdown_us = {s: round(ms / n * 1e3, 2) for s, (ms, n) in prof_all[0].items()}

    # replica clone: this layer's arena, and a 70B-layer-sized buffer (configs[3]: 1,711.3 MB)
    m.replicate(1)
    spare = torch.empty(arena, dtype=torch.uint8, device=U.DEV)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_clone(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps * 1e-3

    t_clone = time_clone(lambda: m.copy_into(0, spare))
    big_bytes = 2 * (2 * 8192 * 8192 + 2 * 8192 * 1024 + 3 * 8192 * 28672)
    src_big = torch.empty(big_bytes, dtype=torch.uint8, device=U.DEV).random_(0, 255)
    dst_big = torch.empty_like(src_big)
    t_clone_big = time_clone(lambda: B.cache_copy(dst_big, src_big))
    assert torch.equal(dst_big[:: 4097], src_big[:: 4097])
    del src_big, dst_big, spare

    # check the timed configuration once against the oracle (sampled sequences keep it short)
    y = db.out()
    sel = slice(0, 4)
    ref = U.oracle_forward(cfg, 0, w, inp, seqs=sel)
    parity = U.rel_err(y[sel], ref)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        reps, t_cpu = 0, 0.0
        while reps < 8 and t_cpu < 12.0:
            t0 = time.perf_counter()
            U.oracle_forward(cfg, 0, w, inp)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cpu = {"value": round(n_tok / (t_cpu / reps), 2), "unit": "tokens/s", "cores": oracle.omp_threads(),
               "kind": "oracle",
               "sample": f"full configs[1] decode step (32 sequences x 1024 cached), mean of {reps} passes, fp64 arithmetic"}

    m.destroy()
    out = {
        "metric": METRIC,
        "value": round(n_tok / per_k[1], 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(per_k[1] * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-2-7B-shaped decoder layer, decode step, batch 32, KV length 1024, "
                               "k=1 replica (k=2,4 in `replicas`)",
                   "hidden": cfg.hidden, "heads": cfg.n_q_heads, "head_dim": cfg.head_dim,
                   "intermediate": cfg.intermediate, "batch": cfg.n_seqs, "kv_len": int(inp.lens[0])},
        "replicas": {str(k): {"tokens_per_s": round(n_tok / t, 1), "ms_per_step": round(t * 1e3, 4),
                              "algorithmic_bytes": k * arena + kv_bytes + act_bytes,
                              "hbm_frac": round((k * arena + kv_bytes + act_bytes) / t / 1e9 / HBM_PEAK_GBPS, 4)}
                     for k, t in per_k.items()},
        "clone": {"payload_GBps": round(arena / t_clone / 1e9, 1), "bytes": arena,
                  "hbm_frac": round(2 * arena / t_clone / 1e9 / HBM_PEAK_GBPS, 4),
                  "layer70b_payload_GBps": round(big_bytes / t_clone_big / 1e9, 1), "layer70b_bytes": big_bytes,
                  "layer70b_hbm_frac": round(2 * big_bytes / t_clone_big / 1e9 / HBM_PEAK_GBPS, 4),
                  "note": "payload = bytes cloned / time; HBM traffic is 2 x payload (read + write)"},
        "kernel_us_k1": breakdown_us,
        "parity_rel_err_vs_oracle": float(f"{parity:.3e}"),
        "roofline": {"kernel": "attn_decode_kernel<1,16>", "bound": "hbm",
                     "achieved": round(kv_bytes / attn_avg_s / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(kv_bytes / attn_avg_s / 1e9 / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES["attn_decode@C2"],
                     "algorithmic_bytes_per_launch": kv_bytes, "avg_launch_us": round(attn_avg_s * 1e6, 2),
                     "launches_timed": attn_n},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
