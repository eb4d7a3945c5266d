#!/usr/bin/env python3
"""Benchmark of the verification pass (ee_verify) on one MI355X.

A "step" is one whole verify pass: embedding, all layers, the exit heads with
their accept/publish steps, the final head with accept and KV commit.  The
default workload is the Llama2-7B-shaped model, gamma = 4, exits after layers 8
and 16, prompt of 512 tokens, consecutive rounds with KV rollback; drafts are
the greedy continuation with each position replaced by a random id with
p = 0.3.  Weights, prompt and drafts are seeded synthetic data already resident
in HBM when the timed region starts.

Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import eegen  # noqa: E402

HBM_PEAK_GBS = 8000.0

WORKLOADS = {
    # name: (model config, prompt, gamma, exits, p_corrupt, max_rows)
    "llama7b_g4_ctx512": (eegen.LLAMA7B, 512, 4, (8, 16), 0.3),
    "llama7b_g8_ctx2048": (eegen.LLAMA7B, 2048, 8, (8, 16, 24), 0.5),
    "llama13b_g5_ctx1024": (eegen.LLAMA13B, 1024, 5, (20,), 0.3),
    "tiny_g4_ctx64": (eegen.TINY, 64, 4, (2,), 0.3),
}


def algorithmic_bytes(cfg, n_exits, P, M, B=1):
    """One read of every weight byte each time it is applied, one read of the live
    KV cache, one write of the new KV rows, one read of the embedding rows."""
    L, d, F, V = cfg.n_layers, cfg.d_model, cfg.d_ffn, cfg.vocab
    weights = 2 * (L * (4 * d * d + 3 * d * F + 2 * d) + (n_exits + 1) * (V * d + d))
    kv_read = B * (2 * (P + M) * d * 2 * L)
    kv_write = B * (M * d * 2 * 2 * L)
    return weights + kv_read + kv_write + B * M * d * 2


def launch_bytes(cfg, code, P, M, B=1):
    """Algorithmic bytes of one launch, by launch code (same accounting as above)."""
    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    return {
        "qkv": 2 * (3 * d * d + d) + B * M * d * 2 * 2,
        "o": 2 * d * d,
        "gu": 2 * (2 * d * F + d),
        "dn": 2 * d * F,
        "head": 2 * (V * d + d),
        "att": B * 2 * (P + M) * d * 2,
        "embed": B * M * d * 2,
    }.get(code, 0)


def per_launch_roofline(ee, model, cfg, prompt, first, drafts_per_round, ex, M, flags, passes):
    """Event pairs around every launch of `passes` further verify passes of the same
    trajectory (a second session, so that the timed region above stays unperturbed).
    Returns per-launch-kind mean duration and achieved bandwidth."""
    sess = model.session(len(prompt) + (passes + 2) * M + 16, max_gamma=M - 1, flags=flags | ee.TIME_LAUNCHES)
    sess.ee_prefill(prompt)
    acc = {}
    for r in range(passes):
        P = sess.ee_kv_len()
        sess.verify_sync(drafts_per_round[r], ex)
        if r == 0:
            continue  # first pass after prefill: cold instruction caches
        for code, ms in sess.ee_launch_times():
            name = ee.LAUNCH_NAMES[code]
            a = acc.setdefault(name, [0, 0.0, 0.0])
            a[0] += 1
            a[1] += ms
            a[2] += launch_bytes(cfg, name, P, M)
    sess.free()
    return {k: {"launches_per_pass": v[0] / (passes - 1), "avg_launch_us": v[1] / v[0] * 1e3,
                "algorithmic_bytes_per_launch": v[2] / v[0],
                "achieved_GBps": (v[2] / (v[1] * 1e-3) / 1e9) if v[2] else None} for k, v in acc.items()}


def model_file(cfg, name, seed, workdir):
    path = os.path.join(workdir, f"ee_{name}_seed{seed}.bin")
    _, total = eegen.tensor_table(cfg)
    if not (os.path.exists(path) and os.path.getsize(path) == total):
        t = time.time()
        eegen.write_model(path, cfg, seed, gains="ones", std=0.02)
        print(f"[bench] wrote {path} ({total / 1e9:.2f} GB) in {time.time() - t:.1f}s", file=sys.stderr, flush=True)
    return path


def pick_workdir():
    for d in (os.environ.get("EE_MODEL_DIR"), "/dev/shm", os.environ.get("TMPDIR"), "/tmp"):
        if d and os.path.isdir(d) and os.access(d, os.W_OK):
            return d
    return "."


def gpu_greedy(sess, gamma):
    """The session's own greedy continuation after `pending` (gamma tokens), by
    single-draft passes rolled back afterwards.  Untimed helper of the driver."""
    kv0, pend0 = sess.ee_kv_len(), sess.ee_pending()
    out = []
    for j in range(gamma):
        r = sess.verify_sync([0])
        t = int(r.final_tokens[0])
        sess.ee_kv_truncate(kv0 + j + 1)
        sess.ee_set_pending(t)
        out.append(t)
    sess.ee_kv_truncate(kv0)
    sess.ee_set_pending(pend0)
    return out


def cpu_baseline(path, cfg, gamma, exits, seed, passes=64, ctx=64):
    """The oracle as it stands, timed on the host cores on a bounded sample."""
    from oracle import oracle as eo
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    m = eo.Model(path)
    s = m.session(ctx + (passes + 1) * (gamma + 1) + 8)
    s.prefill(eegen.prompt_tokens(seed + 1, ctx, cfg.vocab))
    times = []
    t_all = time.perf_counter()
    for i in range(passes):
        drafts = eegen.prompt_tokens(seed + 2, gamma, cfg.vocab, session=i)
        t = time.perf_counter()
        s.verify(drafts, list(exits))
        times.append(time.perf_counter() - t)
        if time.perf_counter() - t_all > 25.0:  # bounded: about 10-30 s of CPU work
            break
    m.close()
    med = statistics.median(times)
    return {"value": 1.0 / med, "unit": "verify passes/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(times)} verify passes (gamma={gamma}, exits={list(exits)}) of the same model at context {ctx} "
                      f"instead of the workload's prompt (weights are >97% of the bytes); median {med:.2f} s/pass"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama7b_g4_ctx512", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=20250521)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chain-launches", action="store_true",
                    help="run consecutive GEMM stages in one persistent launch with grid barriers")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import paper_2505_21594_amd as ee

    cfg, n_prompt, gamma, exits, p_corrupt = WORKLOADS[args.workload]
    M = gamma + 1
    K, W = args.steps, args.warmup
    path = model_file(cfg, args.workload.split("_")[0], args.seed, pick_workdir())

    t = time.time()
    model = ee.Model(path, device=0, max_rows=M)
    print(f"[bench] model on GPU in {time.time() - t:.1f}s, {model.n_workgroups} workgroups", file=sys.stderr, flush=True)
    rounds = W + K
    max_ctx = n_prompt + rounds * M + 2 * M + 16
    flags = ee.CHAIN_LAUNCHES if args.chain_launches else 0
    sess = model.session(max_ctx, max_gamma=max(gamma, 1), flags=flags)
    prompt = eegen.prompt_tokens(args.seed, n_prompt, cfg.vocab)
    t = time.time()
    first = sess.ee_prefill(prompt)
    print(f"[bench] prefill of {n_prompt} tokens in {time.time() - t:.2f}s", file=sys.stderr, flush=True)

    # Untimed rehearsal: walk the whole trajectory once to build every round's drafts
    # (greedy continuation, corrupted), then roll the session back to the prompt.
    drafts_per_round = []
    for r in range(rounds):
        g = gpu_greedy(sess, gamma)
        d = eegen.corrupt_drafts(g, p_corrupt, cfg.vocab, args.seed, r)
        drafts_per_round.append(d)
        sess.verify_sync(d, exits)
    sess.ee_kv_truncate(n_prompt)
    sess.ee_set_pending(first)

    ex = list(exits)
    for r in range(W):
        sess.verify_sync(drafts_per_round[r], ex)

    ee.ee_device_synchronize(0)
    dev_ms, exit_ms, accepted, ctx_at = [], [], [], []
    t0 = time.perf_counter()
    for r in range(W, rounds):
        ctx_at.append(sess.ee_kv_len())
        sess.ee_verify(drafts_per_round[r], ex)
        sess.ee_wait_final()
        accepted.append(sess.final_result().accept_len)
        dev_ms.append(sess.ee_pass_time_ms(len(ex)))
        exit_ms.append([sess.ee_pass_time_ms(e) for e in range(len(ex))])
    ee.ee_device_synchronize(0)
    wall = time.perf_counter() - t0

    kinds = per_launch_roofline(ee, model, cfg, prompt, first, drafts_per_round, ex, M, flags, min(rounds, 9))
    gemm = [k for k in ("qkv", "o", "gu", "dn", "head", "chain") if k in kinds]
    g_n = sum(kinds[k]["launches_per_pass"] for k in gemm)
    g_ms = sum(kinds[k]["launches_per_pass"] * kinds[k]["avg_launch_us"] for k in gemm) * 1e-3
    g_bytes = sum(kinds[k]["launches_per_pass"] * kinds[k]["algorithmic_bytes_per_launch"] for k in gemm)
    if "chain" in kinds:  # chained launches: every GEMM byte of the pass
        g_bytes = sum(algorithmic_bytes(cfg, len(ex), P, M) - launch_bytes(cfg, "att", P, M) * cfg.n_layers
                      - launch_bytes(cfg, "embed", P, M) for P in ctx_at) / len(ctx_at)

    mean_dev_ms = sum(dev_ms) / len(dev_ms)
    bytes_per_pass = [algorithmic_bytes(cfg, len(ex), P, M) for P in ctx_at]
    mean_bytes = sum(bytes_per_pass) / len(bytes_per_pass)
    pass_gbps = mean_bytes / (mean_dev_ms * 1e-3) / 1e9
    achieved = g_bytes / (g_ms * 1e-3) / 1e9
    committed = sum(a + 1 for a in accepted)
    out = {
        "metric": "verify passes/s (Llama2-7B-shape, gamma=4, ctx 512)" if args.workload == "llama7b_g4_ctx512"
        else f"verify passes/s ({args.workload})",
        "value": K / wall,
        "unit": "passes/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "gamma": gamma, "exit_layers": ex, "prompt": n_prompt,
                   "batch": 1, "context_first": ctx_at[0], "context_last": ctx_at[-1],
                   "launch_mode": "chain" if args.chain_launches else "stage"},
        "device_ms_per_pass": {"mean": mean_dev_ms, "median": statistics.median(dev_ms),
                               "p10": float(np.percentile(dev_ms, 10)), "p90": float(np.percentile(dev_ms, 90))},
        "verified_tokens_per_s": committed / wall,
        "mean_accept_len": sum(accepted) / len(accepted),
        "exit_lead_ms": [mean_dev_ms - sum(e[i] for e in exit_ms) / len(exit_ms) for i in range(len(ex))],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "ee_gemm_chain_kernel<1>" if M <= 16 else "ee_gemm_chain_kernel",
                     "launches_per_pass": g_n, "algorithmic_bytes_per_launch": g_bytes / g_n,
                     "avg_launch_us": g_ms / g_n * 1e3,
                     "how": "HIP events on the session stream right before and after every launch, "
                            "passes of the same trajectory in a second session after the timed region",
                     "by_launch_kind": kinds,
                     "whole_pass": {"algorithmic_bytes": mean_bytes, "device_ms": mean_dev_ms,
                                    "achieved": pass_gbps, "frac": pass_gbps / HBM_PEAK_GBS}},
    }
    sess.free()
    model.free()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path, cfg, gamma, exits, args.seed)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
