"""GPU parity at the benchmark's full size: Llama2-7B-shaped model, prompt 512,
gamma 4, exits after layers 8 and 16, in the launch configuration bench.py
times.  The oracle runs the same passes on the host cores (weights stay bf16 in
RAM, arithmetic fp32); every logit of every head of every row is compared."""
import os

import numpy as np
import pytest

import eegen
import paper_2505_21594_amd as ee
from oracle import oracle as eo
from tests.parity import check_pass, gpu_logits

pytestmark = pytest.mark.gpu


def _workdir():
    for d in (os.environ.get("EE_MODEL_DIR"), "/dev/shm", "/tmp"):
        if d and os.path.isdir(d) and os.access(d, os.W_OK):
            return d
    return "."


@pytest.fixture(scope="module")
def llama7b_path():
    path = os.path.join(_workdir(), "ee_llama7b_seed20250521.bin")   # same file bench.py uses
    _, total = eegen.tensor_table(eegen.LLAMA7B)
    if not (os.path.exists(path) and os.path.getsize(path) == total):
        eegen.write_model(path, eegen.LLAMA7B, 20250521, gains="ones", std=0.02)
    return path


@pytest.mark.timeout(900)
def test_llama7b_gamma4_ctx512_rounds(llama7b_path):
    cfg = eegen.LLAMA7B
    gamma, exits, rounds = 4, [8, 16], 3
    g = ee.Model(llama7b_path, max_rows=gamma + 1)
    o = eo.Model(llama7b_path)
    prompt = eegen.prompt_tokens(20250521, 512, cfg.vocab)
    gs = g.session(640, max_gamma=gamma, flags=ee.KEEP_LOGITS)
    os_ = o.session(640)
    first_o = os_.prefill(prompt)
    first_g = gs.ee_prefill(prompt)
    if first_g != first_o:
        gs.ee_set_pending(first_o)
    hist = list(prompt) + [first_o]
    worst, exempt_rounds = 0.0, 0
    for r in range(rounds):
        kv0, pend0 = os_.kv_len, os_.pending
        greedy = []
        for _ in range(gamma):             # the oracle's own greedy continuation
            t = int(os_.verify([0], commit=False).final_tokens[0])
            kv = os_.kv_len
            os_.verify([t], commit=True)
            os_.kv_truncate(kv + 1)
            os_.set_pending(t)
            greedy.append(t)
        os_.kv_truncate(kv0)
        os_.set_pending(pend0)
        drafts = eegen.corrupt_drafts(greedy, 0.3, cfg.vocab, 20250521, r)
        ro = os_.verify(drafts, exits, commit=True, want_logits=True)
        hist += [int(t) for t in drafts[:ro.accept_len]] + [int(ro.next_token)]
        gs.ee_verify(drafts, exits)
        gs.ee_wait_exit(0)
        gs.ee_wait_exit(1)
        gs.ee_wait_final()
        rg = gs.final_result()
        exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, f"7B round {r}")
        worst = max(worst, err)
        if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
            assert exempt
            exempt_rounds += 1
            gs.ee_prefill(hist, flags=ee.HOLD_LAST)
        assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
        t_e0, t_e1, t_f = gs.ee_pass_time_ms(0), gs.ee_pass_time_ms(1), gs.ee_pass_time_ms(2)
        assert 0 < t_e0 < t_e1 < t_f          # exit results were published mid-pass
    print(f"7B: worst logits max-abs-err {worst:.4g}, exempt rounds {exempt_rounds}")
    gs.free()
    g.free()


def _greedy(os_, gamma):
    """The oracle session's own greedy continuation after `pending` (session left unchanged)."""
    kv0, pend0 = os_.kv_len, os_.pending
    out = []
    for _ in range(gamma):
        t = int(os_.verify([0], commit=False).final_tokens[0])
        kv = os_.kv_len
        os_.verify([t], commit=True)
        os_.kv_truncate(kv + 1)
        os_.set_pending(t)
        out.append(t)
    os_.kv_truncate(kv0)
    os_.set_pending(pend0)
    return out


@pytest.mark.timeout(900)
def test_llama7b_gamma8_ctx2048_three_exits(llama7b_path):
    """Long context (attention walks several pages per wave, K-blocked GEMM inputs for 9 rows),
    exits after layers 8, 16 and 24, drafts corrupted with p = 0.5."""
    cfg = eegen.LLAMA7B
    gamma, exits = 8, [8, 16, 24]
    g = ee.Model(llama7b_path, max_rows=gamma + 1)
    o = eo.Model(llama7b_path)
    prompt = eegen.prompt_tokens(20250522, 2048, cfg.vocab)
    gs = g.session(2048 + 64, max_gamma=gamma, flags=ee.KEEP_LOGITS)
    os_ = o.session(2048 + 64)
    first_o = os_.prefill(prompt)
    if gs.ee_prefill(prompt) != first_o:
        gs.ee_set_pending(first_o)
    drafts = eegen.corrupt_drafts(_greedy(os_, gamma), 0.5, cfg.vocab, 20250522, 0)
    ro = os_.verify(drafts, exits, commit=True, want_logits=True)
    rg = gs.verify_sync(drafts, exits)
    exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, "7B ctx 2048")
    print(f"7B ctx 2048 gamma 8: logits max-abs-err {err:.4g}, accept_len {ro.accept_len}")
    if not exempt:
        assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
    gs.free()
    g.free()


@pytest.mark.timeout(900)
def test_llama7b_eight_sessions_with_embedding_prefix(llama7b_path):
    """Eight sessions in one pass, each with 576 embedding rows (image-patch stand-ins) and 64
    text ids, gamma 4, exit after layer 16, per-session corruption probability."""
    cfg = eegen.LLAMA7B
    gamma, exits, B, n_emb, n_txt, seed = 4, [16], 8, 576, 64, 20250523
    g = ee.Model(llama7b_path, max_rows=B * (gamma + 1))
    o = eo.Model(llama7b_path)
    gss, oss, drafts = [], [], []
    for b in range(B):
        emb = eegen.embedding_prefix(seed, n_emb, cfg.d_model, session=b)
        txt = eegen.prompt_tokens(seed, n_txt, cfg.vocab, session=b)
        gs = g.session(n_emb + n_txt + 32, max_gamma=gamma)
        os_ = o.session(n_emb + n_txt + 32)
        first_o = os_.prefill(txt, emb=emb)
        if gs.ee_prefill(txt, emb=emb) != first_o:
            gs.ee_set_pending(first_o)
        p = eegen.session_corruption_p(seed, b)
        drafts.append(eegen.corrupt_drafts(_greedy(os_, gamma), p, cfg.vocab, seed, 0, session=b))
        gss.append(gs)
        oss.append(os_)
    ee.ee_verify_batch(gss, drafts, exits)
    for gs in gss:
        gs.ee_wait_final()
    accepts = []
    for b in range(B):
        ro = oss[b].verify(drafts[b], exits, commit=True, want_logits=True)
        rg = gss[b].final_result()
        exempt, _ = check_pass(ro, rg, None, drafts[b], f"batch session {b}")
        if not exempt:
            assert gss[b].ee_kv_len() == oss[b].kv_len and gss[b].ee_pending() == oss[b].pending
        accepts.append(int(ro.accept_len))
    print("eight sessions: accept lengths", accepts)
    for gs in gss:
        gs.free()
    g.free()


@pytest.mark.timeout(900)
def test_llama13b_gamma5_ctx1024():
    """Llama2-13B shape (40 layers, d = 5120, 40 heads, F = 13824), exit after layer 20."""
    cfg = eegen.LLAMA13B
    path = os.path.join(_workdir(), "ee_llama13b_seed20250521.bin")
    _, total = eegen.tensor_table(cfg)
    if not (os.path.exists(path) and os.path.getsize(path) == total):
        eegen.write_model(path, cfg, 20250521, gains="ones", std=0.02)
    try:
        gamma, exits = 5, [20]
        g = ee.Model(path, max_rows=gamma + 1)
        o = eo.Model(path)
        prompt = eegen.prompt_tokens(20250524, 1024, cfg.vocab)
        gs = g.session(1024 + 64, max_gamma=gamma, flags=ee.KEEP_LOGITS)
        os_ = o.session(1024 + 64)
        first_o = os_.prefill(prompt)
        if gs.ee_prefill(prompt) != first_o:
            gs.ee_set_pending(first_o)
        drafts = eegen.corrupt_drafts(_greedy(os_, gamma), 0.3, cfg.vocab, 20250524, 0)
        ro = os_.verify(drafts, exits, commit=True, want_logits=True)
        rg = gs.verify_sync(drafts, exits)
        exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, "13B")
        print(f"13B: logits max-abs-err {err:.4g}, accept_len {ro.accept_len}")
        gs.free()
        g.free()
        o.close()
    finally:
        if os.path.exists(path):
            os.remove(path)   # 26 GB of /dev/shm
