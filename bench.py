#!/usr/bin/env python3
"""Benchmark of the verification pass (ee_verify) on one MI355X.

A "step" is one whole verify pass: embedding, all layers, the exit heads with
their accept/publish steps, the final head with accept and KV commit.  The
default workload is the Llama2-7B-shaped model, gamma = 4, exits after layers 8
and 16, prompt of 512 tokens, consecutive rounds with KV rollback; drafts are
the greedy continuation with each position replaced by a random id with
p = 0.3.  Weights, prompt and drafts are seeded synthetic data already resident
in HBM when the timed region starts.

Prints ONE JSON line: metric, value, unit, steps, ms_per_step, config, device_ms_per_pass,
verified_tokens_per_s, exit_lead_ms, roofline (dominant kernel against the HBM peak, with the
measured HBM traffic per launch) and cpu_baseline (the CPU oracle timed on the host cores).
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

_L7 = eegen.LLAMA7B
# the regime the paper runs: an exit head after every layer but the last, each with its adapters
LLAMA7B_31 = eegen.ModelConfig(_L7.n_layers, _L7.d_model, _L7.n_heads, _L7.head_dim, _L7.d_ffn, _L7.vocab,
                               tuple(range(1, _L7.n_layers)), n_adapters=3, adapter_width=128)

WORKLOADS = {
    # name: (model config, model file tag, prompt tokens, gamma, exits, corruption p (None: per session in
    #        [0.1, 0.6]), sessions, embedding-prefix rows, exit heads per launch of the LM head)
    "llama7b_g4_ctx512": (eegen.LLAMA7B, "llama7b", 512, 4, (8, 16), 0.3, 1, 0, 1),
    "llama7b_g8_ctx2048": (eegen.LLAMA7B, "llama7b", 2048, 8, (8, 16, 24), 0.5, 1, 0, 1),
    "llama13b_g5_ctx1024": (eegen.LLAMA13B, "llama13b", 1024, 5, (20,), 0.3, 1, 0, 1),
    "llama7b_b8_vlm": (eegen.LLAMA7B, "llama7b", 64, 4, (16,), None, 8, 576, 1),
    "llama7b_g15_ctx512": (eegen.LLAMA7B, "llama7b", 512, 15, (8, 16), 0.3, 1, 0, 1),     # 16 rows: one full row tile
    "llama7b_g4_ctx512_31exits": (LLAMA7B_31, "llama7b_31exits", 512, 4, LLAMA7B_31.exit_layers, 0.3, 1, 0, 1),
    "llama7b_g4_ctx512_31exits_groups8": (LLAMA7B_31, "llama7b_31exits", 512, 4, LLAMA7B_31.exit_layers, 0.3, 1, 0, 8),
    "tiny_g4_ctx64": (eegen.TINY, "tiny", 64, 4, (2,), 0.3, 1, 0, 1),
}


def algorithmic_bytes(cfg, n_exits, P, M, B=1):
    """One read of every weight byte each time it is applied, one read of the live
    KV cache, one write of the new KV rows, one read of the embedding rows."""
    L, d, F, V = cfg.n_layers, cfg.d_model, cfg.d_ffn, cfg.vocab
    A = cfg.n_adapters * cfg.adapter_width
    weights = 2 * (L * (4 * d * d + 3 * d * F + 2 * d) + (n_exits + 1) * (V * d + d) + n_exits * (2 * A * d + A + d))
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
        "adapter_down": 2 * (cfg.n_adapters * cfg.adapter_width) * (d + 1),
        "adapter_up": 2 * (cfg.n_adapters * cfg.adapter_width + 1) * d,
        "att": B * 2 * (P + M) * d * 2,
        "embed": B * M * d * 2,
    }.get(code, 0)


def per_launch_roofline(ee, run, passes):
    """Event pairs around every launch of `passes` further verify passes of the same
    trajectory (a second set of sessions, so that the timed region stays unperturbed).
    Returns per-launch-kind mean duration and achieved bandwidth."""
    sessions = run.make_sessions(extra_flags=ee.TIME_LAUNCHES, rounds=passes)
    acc = {}
    for r in range(passes):
        P = sum(s.ee_kv_len() for s in sessions) / len(sessions)
        run.verify(sessions, r)
        if r == 0:
            continue  # first pass after prefill: cold instruction caches
        for code, ms in sessions[0].ee_launch_times():
            name = ee.LAUNCH_NAMES[code]
            a = acc.setdefault(name, [0, 0.0, 0.0])
            a[0] += 1
            a[1] += ms
            a[2] += launch_bytes(run.cfg, name, P, run.M, run.B)
    for s in sessions:
        s.free()
    return {k: {"launches_per_pass": v[0] / (passes - 1), "avg_launch_us": v[1] / v[0] * 1e3,
                "algorithmic_bytes_per_launch": v[2] / v[0],
                "achieved_GBps": (v[2] / (v[1] * 1e-3) / 1e9) if v[2] else None} for k, v in acc.items()}


class Run:
    """One workload: the model, its sessions' prompts and every round's drafts."""

    def __init__(self, ee, model, cfg, seed, n_prompt, gamma, exits, p, B, n_emb, flags, head_batch=1):
        self.ee, self.model, self.cfg, self.seed, self.head_batch = ee, model, cfg, seed, head_batch
        self.n_prompt, self.gamma, self.M, self.exits, self.B, self.n_emb, self.flags = n_prompt, gamma, gamma + 1, list(exits), B, n_emb, flags
        self.p = [p if p is not None else eegen.session_corruption_p(seed, b) for b in range(B)]
        self.prompts = [eegen.prompt_tokens(seed, n_prompt, cfg.vocab, session=b) for b in range(B)]
        self.embs = [eegen.embedding_prefix(seed, n_emb, cfg.d_model, session=b) if n_emb else None for b in range(B)]
        self.drafts = []  # [round][session]

    def make_sessions(self, extra_flags=0, rounds=0):
        max_ctx = self.n_emb + self.n_prompt + (rounds + 2) * self.M + 16
        out = []
        for b in range(self.B):
            s = self.model.session(max_ctx, max_gamma=self.gamma, flags=self.flags | extra_flags)
            s.first = s.ee_prefill(self.prompts[b], emb=self.embs[b])
            if self.head_batch > 1:
                s.ee_session_option(self.ee.OPT_HEAD_BATCH, self.head_batch)
            s.base = self.n_emb + self.n_prompt
            out.append(s)
        return out

    def verify(self, sessions, r, wait=True):
        if self.B == 1:
            sessions[0].ee_verify(self.drafts[r][0], self.exits)
        else:
            self.ee.ee_verify_batch(sessions, self.drafts[r], self.exits)
        if wait:
            sessions[0].ee_wait_final()
            for s in sessions[1:]:
                s.ee_wait_final()

    def rehearse(self, sessions, rounds):
        """Untimed: walk the trajectory once to build every round's drafts (each session's greedy
        continuation, corrupted), then roll the sessions back to their prompts."""
        for r in range(rounds):
            row = []
            for b, s in enumerate(sessions):
                g = gpu_greedy(s, self.gamma)
                row.append(eegen.corrupt_drafts(g, self.p[b], self.cfg.vocab, self.seed, r, session=b))
            self.drafts.append(row)
            self.verify(sessions, r)
        for s in sessions:
            s.ee_kv_truncate(s.base)
            s.ee_set_pending(s.first)


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy kernel's reading), or None."""
    d = os.path.join(ROOT, "profiles")
    try:
        for f in sorted(os.listdir(d)):
            if f.startswith("hbm_traffic"):
                for line in open(os.path.join(d, f)):
                    t = line.split()
                    if len(t) == 4 and t[0] == "traffic" and t[1] == kernel and t[2] == workload:
                        return float(t[3])
    except OSError:
        pass
    return None


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


def cpu_baseline(path, run, first_round, budget_s=25.0, prefill_rows_max=1100):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload: the
    same model file, the same prompt (session 0) and the drafts of the timed rounds."""
    from oracle import oracle as eo
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    cfg, gamma, exits = run.cfg, run.gamma, run.exits
    m = eo.Model(path)
    n_rows = run.n_emb + run.n_prompt
    prompt, emb, note = run.prompts[0], run.embs[0], "the workload's own prompt"
    # the oracle's prefill runs at about 50 rows/s per 7e9 parameters: bound it to about 20 s
    n_params = cfg.n_layers * (4 * cfg.d_model ** 2 + 3 * cfg.d_model * cfg.d_ffn) + 2 * cfg.vocab * cfg.d_model
    rows_cap = max(64, int(prefill_rows_max * 6.7e9 / n_params))
    if n_rows > rows_cap:   # keep the tail of the prompt (text rows only)
        emb = None
        prompt = prompt[-min(rows_cap, len(prompt)):]
        note = f"the last {len(prompt)} rows of the workload's {n_rows}-row prompt"
    rounds = len(run.drafts) - first_round
    s = m.session((0 if emb is None else run.n_emb) + len(prompt) + (rounds + 1) * (gamma + 1) + 8)
    t0 = time.perf_counter()
    s.prefill(prompt, emb=emb)
    t_prefill = time.perf_counter() - t0
    times = []
    t_all = time.perf_counter()
    for r in range(first_round, len(run.drafts)):
        t = time.perf_counter()
        s.verify(run.drafts[r][0], list(exits))
        times.append(time.perf_counter() - t)
        if time.perf_counter() - t_all > budget_s and len(times) >= 5:  # bounded: about 10-30 s of CPU work
            break
    m.close()
    med = statistics.median(times)
    return {"value": 1.0 / med, "unit": "verify passes/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(times)} consecutive verify passes of one session (gamma={gamma}, {len(exits)} exits) after the oracle's own "
                      f"prefill of {note} ({t_prefill:.1f} s, untimed), fed the drafts of the timed rounds; median {med:.3f} s/pass"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama7b_g4_ctx512", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=20250521)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 20 plain copies of 1 GiB (reference reading for the HBM traffic counters)")
    args = ap.parse_args()
    if args.copy_calibration:
        import paper_2505_21594_amd as ee
        ee.ee_debug_copy(0, 1 << 30, 20)
        print(json.dumps({"copy_calibration": {"kernel": "ee_copy_kernel", "bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 20}}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import paper_2505_21594_amd as ee

    cfg, tag, n_prompt, gamma, exits, p_corrupt, B, n_emb, head_batch = WORKLOADS[args.workload]
    M = gamma + 1
    K, W = args.steps, args.warmup
    path = model_file(cfg, tag, args.seed, pick_workdir())

    t = time.time()
    model = ee.Model(path, device=0, max_rows=max(B * M, min(48, head_batch * B * M)))
    print(f"[bench] model on GPU in {time.time() - t:.1f}s, {model.n_workgroups} workgroups", file=sys.stderr, flush=True)
    rounds = W + K
    flags = 0
    run = Run(ee, model, cfg, args.seed, n_prompt, gamma, exits, p_corrupt, B, n_emb, flags, head_batch)
    t = time.time()
    sessions = run.make_sessions(rounds=rounds)
    print(f"[bench] prefill of {B} x {n_emb + n_prompt} rows in {time.time() - t:.2f}s", file=sys.stderr, flush=True)
    run.rehearse(sessions, rounds)
    ex = run.exits
    for r in range(W):
        run.verify(sessions, r)

    ee.ee_device_synchronize(0)
    lead = sessions[0]
    dev_ms, exit_ms, accepted, ctx_at = [], [], [], []
    t0 = time.perf_counter()
    for r in range(W, rounds):
        ctx_at.append(sum(s.ee_kv_len() for s in sessions) / B)
        run.verify(sessions, r)
        accepted.append(sum(s.final_result().accept_len for s in sessions))
        dev_ms.append(lead.ee_pass_time_ms(len(ex)))
        exit_ms.append([lead.ee_pass_time_ms(e) for e in range(len(ex))])
    ee.ee_device_synchronize(0)
    wall = time.perf_counter() - t0

    # the host holding the first exit's result while the pass is still running (8 further passes of the trajectory)
    host_lead = []
    if ex and B == 1:
        extra = run.make_sessions(rounds=rounds)
        for r in range(min(rounds, 8)):
            extra[0].ee_verify(run.drafts[r][0], ex)
            extra[0].ee_wait_exit(0)
            t_exit = time.perf_counter()
            early = not extra[0].ee_query_final()
            extra[0].ee_wait_final()
            if early:
                host_lead.append((time.perf_counter() - t_exit) * 1e3)
        for sx in extra:
            sx.free()

    kinds = per_launch_roofline(ee, run, min(rounds, 9))
    gemm = [k for k in ("qkv", "o", "gu", "dn", "head", "adapter_down", "adapter_up") if k in kinds]
    g_n = sum(kinds[k]["launches_per_pass"] for k in gemm)
    g_ms = sum(kinds[k]["launches_per_pass"] * kinds[k]["avg_launch_us"] for k in gemm) * 1e-3
    g_bytes = sum(kinds[k]["launches_per_pass"] * kinds[k]["algorithmic_bytes_per_launch"] for k in gemm)

    mean_dev_ms = sum(dev_ms) / len(dev_ms)
    bytes_per_pass = [algorithmic_bytes(cfg, len(ex), P, M, B) for P in ctx_at]
    mean_bytes = sum(bytes_per_pass) / len(bytes_per_pass)
    pass_gbps = mean_bytes / (mean_dev_ms * 1e-3) / 1e9
    achieved = g_bytes / (g_ms * 1e-3) / 1e9
    committed = sum(a + B for a in accepted)
    kernel_name = "ee_gemm_kernel<%d>" % ((B * M + 15) // 16)
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
                   "batch": B, "embedding_prefix_rows": n_emb, "context_first": ctx_at[0], "context_last": ctx_at[-1],
                   "exit_heads_per_lm_head_launch": head_batch, "adapters": [cfg.n_adapters, cfg.adapter_width],
                   "launch_mode": "stage"},
        "device_ms_per_pass": {"mean": mean_dev_ms, "median": statistics.median(dev_ms),
                               "p10": float(np.percentile(dev_ms, 10)), "p90": float(np.percentile(dev_ms, 90))},
        "verified_tokens_per_s": committed / wall,
        "mean_accept_len": sum(accepted) / len(accepted) / B,
        "exit_lead_ms": [mean_dev_ms - sum(e[i] for e in exit_ms) / len(exit_ms) for i in range(len(ex))],
        "exit0_lead_seen_by_host_ms": {"median": statistics.median(host_lead), "passes_with_exit_before_final": len(host_lead)} if host_lead else None,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(kernel_name, args.workload),
                     "traffic_source": "committed rocprofv3 --pmc summary profiles/hbm_traffic.md (FETCH_SIZE + WRITE_SIZE, "
                                       "scaled by a plain copy kernel's reading); not measured in this run",
                     "kernel": kernel_name,
                     "launches_per_pass": g_n, "algorithmic_bytes_per_launch": g_bytes / g_n,
                     "avg_launch_us": g_ms / g_n * 1e3,
                     "how": "HIP events on the session stream right before and after every launch, "
                            "passes of the same trajectory in a second session after the timed region",
                     "by_launch_kind": kinds,
                     "whole_pass": {"algorithmic_bytes": mean_bytes, "device_ms": mean_dev_ms,
                                    "achieved": pass_gbps, "frac": pass_gbps / HBM_PEAK_GBS}},
    }
    for sx in sessions:
        sx.free()
    model.free()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path, run, W)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
