"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
Llama2-7B- and 13B-shaped models, the four full-size workloads (prompt 512 / gamma 4 / exits
8, 16 for 64 rounds; prompt 2048 / gamma 8 / exits 8, 16, 24 / p = 0.5; 13B / prompt 1024 /
gamma 5; eight sessions with embedding prefixes).  The oracle runs the same passes on the host
cores (weights stay bf16 in RAM, arithmetic fp32); every logit of every head of every row is
compared, every round commits and rolls back, and a GPU session that legitimately leaves the
oracle's trajectory at a low-margin row is put back on it."""
import os
import sys
import time

import numpy as np
import pytest

import eegen
import paper_2505_21594_amd as ee
from oracle import oracle as eo
from tests.parity import check_first_token, check_pass, gpu_logits, oracle_greedy, oracle_prefill, sampled_chain

pytestmark = pytest.mark.gpu


def _workdir():
    for d in (os.environ.get("EE_MODEL_DIR"), "/dev/shm", "/tmp"):
        if d and os.path.isdir(d) and os.access(d, os.W_OK):
            return d
    return "."


def _model_file(cfg, tag):
    path = os.path.join(_workdir(), f"ee_{tag}_seed20250521.bin")   # same files bench.py uses
    _, total = eegen.tensor_table(cfg)
    if not (os.path.exists(path) and os.path.getsize(path) == total):
        eegen.write_model(path, cfg, 20250521, gains="ones", std=0.02)
    return path


@pytest.fixture(scope="module")
def llama7b_path():
    return _model_file(eegen.LLAMA7B, "llama7b")


def _say(capsys, msg):
    """Progress line past pytest's capture: a long test must not look hung."""
    with capsys.disabled():
        print(msg, file=sys.stderr, flush=True)


def _rounds(capsys, what, g, o, cfg, prompt, gamma, exits, p, rounds, seed, host_lead=False):
    """`rounds` consecutive verify rounds with commit and rollback on one session, drafts = the
    oracle's greedy continuation corrupted with probability p."""
    max_ctx = len(prompt) + rounds * (gamma + 1) + 16
    gs = g.session(max_ctx, max_gamma=gamma, flags=ee.KEEP_LOGITS)
    os_ = o.session(max_ctx)
    t0 = time.time()
    first_o, margin = oracle_prefill(os_, prompt)
    first_g = gs.ee_prefill(prompt)
    check_first_token(gs, first_g, first_o, margin, what)
    _say(capsys, f"[{what}] prefill of {len(prompt)} rows on both sides in {time.time() - t0:.1f}s, first token margin {margin:.3g}")
    hist = list(prompt) + [first_o]
    worst, exempt_rounds, accepted, leads = 0.0, 0, [], []
    for r in range(rounds):
        drafts = eegen.corrupt_drafts(oracle_greedy(os_, gamma), p, cfg.vocab, seed, r)
        ro = os_.verify(drafts, exits, commit=True, want_logits=True)
        hist += [int(t) for t in drafts[:ro.accept_len]] + [int(ro.next_token)]
        gs.ee_verify(drafts, exits)
        if host_lead and exits:
            # the host holds the first exit's result while the pass is still running
            gs.ee_wait_exit(0)
            t_exit = time.perf_counter()
            assert gs.ee_query_exit(0), "exit 0 waited for but not published"
            assert not gs.ee_query_final(), "the final result was already there when exit 0 was observed"
            toks, delta = gs.exit_result(0)
            assert 0 <= delta <= gamma
        for e in range(len(exits)):
            gs.ee_wait_exit(e)
        gs.ee_wait_final()
        if host_lead and exits:
            leads.append(time.perf_counter() - t_exit)
        rg = gs.final_result()
        exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, f"{what} round {r}")
        worst = max(worst, err)
        accepted.append(int(ro.accept_len))
        if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
            assert exempt
            exempt_rounds += 1
            gs.ee_prefill(hist, flags=ee.HOLD_LAST)
        assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
        times = [gs.ee_pass_time_ms(e) for e in range(len(exits) + 1)]
        assert all(0 < a < b for a, b in zip(times, times[1:]))   # exit results were published mid-pass, in order
        if r % 8 == 7 or r == rounds - 1:
            _say(capsys, f"[{what}] round {r + 1}/{rounds}: worst logits max-abs-err {worst:.3g}, exempt rounds {exempt_rounds}, "
                         f"mean accept {np.mean(accepted):.2f}, context {os_.kv_len}, {time.time() - t0:.0f}s")
    if leads:
        _say(capsys, f"[{what}] host held exit 0's result {1e3 * float(np.median(leads)):.2f} ms (median) before the final result")
    gs.free()
    return worst, exempt_rounds


@pytest.mark.timeout(600)
def test_llama7b_gamma4_ctx512_64_rounds(llama7b_path, capsys):
    cfg = eegen.LLAMA7B
    g = ee.Model(llama7b_path, max_rows=5)
    o = eo.Model(llama7b_path)
    prompt = eegen.prompt_tokens(20250521, 512, cfg.vocab)
    try:
        worst, _ = _rounds(capsys, "7B g4 ctx512", g, o, cfg, prompt, 4, [8, 16], 0.3, 64, 20250521, host_lead=True)
        assert worst <= 3e-2
    finally:
        g.free()
        o.close()


@pytest.mark.timeout(600)
def test_llama7b_gamma8_ctx2048_three_exits(llama7b_path, capsys):
    """Long context (attention walks several pages per wave, K-blocked GEMM inputs for 9 rows),
    exits after layers 8, 16 and 24, drafts corrupted with p = 0.5: frequent early rejection,
    so most rounds roll the cache back."""
    cfg = eegen.LLAMA7B
    g = ee.Model(llama7b_path, max_rows=9)
    o = eo.Model(llama7b_path)
    prompt = eegen.prompt_tokens(20250522, 2048, cfg.vocab)
    try:
        _rounds(capsys, "7B g8 ctx2048", g, o, cfg, prompt, 8, [8, 16, 24], 0.5, 8, 20250522)
    finally:
        g.free()
        o.close()


@pytest.mark.timeout(600)
def test_llama7b_eight_sessions_with_embedding_prefix(llama7b_path, capsys):
    """Eight sessions in one pass (40 rows, one stream of the weights), each with 576 embedding
    rows (image-patch stand-ins) and 64 text ids, gamma 4, exit after layer 16, per-session
    corruption probability: ragged accept lengths, per-session rollback, 8 rounds, every
    session's logits compared."""
    cfg = eegen.LLAMA7B
    gamma, exits, B, n_emb, n_txt, seed, rounds = 4, [16], 8, 576, 64, 20250523, 8
    g = ee.Model(llama7b_path, max_rows=B * (gamma + 1))
    o = eo.Model(llama7b_path)
    gss, oss, ps, hists, embs = [], [], [], [], []
    t0 = time.time()
    try:
        for b in range(B):
            emb = eegen.embedding_prefix(seed, n_emb, cfg.d_model, session=b)
            txt = eegen.prompt_tokens(seed, n_txt, cfg.vocab, session=b)
            max_ctx = n_emb + n_txt + rounds * (gamma + 1) + 16
            gs = g.session(max_ctx, max_gamma=gamma, flags=ee.KEEP_LOGITS if b == 0 else 0)
            os_ = o.session(max_ctx)
            first_o, margin = oracle_prefill(os_, txt, emb=emb)
            check_first_token(gs, gs.ee_prefill(txt, emb=emb), first_o, margin, f"batch session {b}")
            ps.append(eegen.session_corruption_p(seed, b))
            gss.append(gs)
            oss.append(os_)
            embs.append(emb)
            hists.append(list(txt) + [first_o])
            _say(capsys, f"[7B b8] session {b} prefilled, {time.time() - t0:.0f}s")
        worst, exempt_rounds = 0.0, 0
        for r in range(rounds):
            drafts = [eegen.corrupt_drafts(oracle_greedy(oss[b], gamma), ps[b], cfg.vocab, seed, r, session=b) for b in range(B)]
            ee.ee_verify_batch(gss, drafts, exits)
            for gs in gss:
                gs.ee_wait_final()
            accepts = []
            for b in range(B):
                ro = oss[b].verify(drafts[b], exits, commit=True, want_logits=True)
                hists[b] += [int(t) for t in drafts[b][:ro.accept_len]] + [int(ro.next_token)]
                rg = gss[b].final_result()
                exempt, err = check_pass(ro, rg, gpu_logits(gss[b], len(exits)), drafts[b], f"batch round {r} session {b}")
                worst = max(worst, err)
                accepts.append(int(ro.accept_len))
                if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
                    assert exempt
                    exempt_rounds += 1
                    gss[b].ee_prefill(hists[b], flags=ee.HOLD_LAST, emb=embs[b])
                assert gss[b].ee_kv_len() == oss[b].kv_len and gss[b].ee_pending() == oss[b].pending
            _say(capsys, f"[7B b8] round {r + 1}/{rounds}: accept lengths {accepts}, worst logits err {worst:.3g}, "
                         f"exempt {exempt_rounds}, {time.time() - t0:.0f}s")
        assert len({gs.ee_kv_len() for gs in gss}) > 1        # the sessions' contexts have drifted apart
    finally:
        for gs in gss:
            gs.free()
        g.free()
        o.close()


@pytest.mark.timeout(600)
def test_llama13b_gamma5_ctx1024(capsys):
    """Llama2-13B shape (40 layers, d = 5120, 40 heads, F = 13824), exit after layer 20."""
    cfg = eegen.LLAMA13B
    path = _model_file(cfg, "llama13b")
    try:
        g = ee.Model(path, max_rows=6)
        o = eo.Model(path)
        prompt = eegen.prompt_tokens(20250524, 1024, cfg.vocab)
        try:
            _rounds(capsys, "13B g5 ctx1024", g, o, cfg, prompt, 5, [20], 0.3, 8, 20250524)
        finally:
            g.free()
        try:
            _batch_13b(capsys, path, o, cfg)
        finally:
            o.close()
    finally:
        if os.path.exists(path):
            os.remove(path)   # 26 GB of /dev/shm


def _batch_13b(capsys, path, o, cfg):
    """Four sessions of six rows in one pass on the 13B shape (24 rows: two row tiles; output and
    down projection with K split over workgroups, 320 units over 64 groups of four), short prompts,
    three rounds with commit, every session's logits compared."""
    gamma, exits, B, seed, rounds = 5, [20], 4, 20250525, 3
    g = ee.Model(path, max_rows=B * (gamma + 1))
    gss, oss = [], []
    t0 = time.time()
    try:
        for b in range(B):
            txt = eegen.prompt_tokens(seed, 24 + 5 * b, cfg.vocab, session=b)
            gs = g.session(128, max_gamma=gamma, flags=ee.KEEP_LOGITS if b == 0 else 0)
            os_ = o.session(128)
            first_o, margin = oracle_prefill(os_, txt)
            check_first_token(gs, gs.ee_prefill(txt), first_o, margin, f"13B batch session {b}")
            gss.append(gs)
            oss.append(os_)
        worst = 0.0
        for r in range(rounds):
            drafts = [eegen.corrupt_drafts(oracle_greedy(oss[b], gamma), 0.3, cfg.vocab, seed, r, session=b) for b in range(B)]
            ee.ee_verify_batch(gss, drafts, exits)
            for gs in gss:
                gs.ee_wait_final()
            for b in range(B):
                ro = oss[b].verify(drafts[b], exits, commit=True, want_logits=True)
                rg = gss[b].final_result()
                exempt, err = check_pass(ro, rg, gpu_logits(gss[b], len(exits)), drafts[b], f"13B batch round {r} session {b}")
                worst = max(worst, err)
                if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
                    assert exempt
                    gss[b].ee_kv_truncate(oss[b].kv_len)
                    gss[b].ee_set_pending(oss[b].pending)
                assert gss[b].ee_kv_len() == oss[b].kv_len and gss[b].ee_pending() == oss[b].pending
            _say(capsys, f"[13B b4] round {r + 1}/{rounds}: worst logits err {worst:.3g}, {time.time() - t0:.0f}s")
    finally:
        for gs in gss:
            gs.free()
        g.free()


@pytest.mark.timeout(600)
def test_llama7b_31_exits_with_adapters(capsys):
    """The regime the paper runs: an exit head after every layer but the last (31 on the 7B
    shape), each with its adapters (three bottlenecks of width 128), the LM head streamed once
    for groups of eight exits (40 rows)."""
    base = eegen.LLAMA7B
    cfg = eegen.ModelConfig(base.n_layers, base.d_model, base.n_heads, base.head_dim, base.d_ffn, base.vocab,
                            tuple(range(1, base.n_layers)), n_adapters=3, adapter_width=128)
    path = _model_file(cfg, "llama7b_31exits")
    try:
        g = ee.Model(path, max_rows=40)
        o = eo.Model(path)
        exits = list(cfg.exit_layers)
        prompt = eegen.prompt_tokens(20250525, 128, cfg.vocab)
        gs = g.session(256, max_gamma=4, flags=ee.KEEP_LOGITS)
        os_ = o.session(256)
        try:
            first_o, margin = oracle_prefill(os_, prompt)
            check_first_token(gs, gs.ee_prefill(prompt), first_o, margin, "31 exits")
            gs.ee_session_option(ee.OPT_HEAD_BATCH, 8)
            worst = 0.0
            for r in range(3):
                drafts = eegen.corrupt_drafts(oracle_greedy(os_, 4), 0.3, cfg.vocab, 20250525, r)
                ro = os_.verify(drafts, exits, commit=True, want_logits=True)
                rg = gs.verify_sync(drafts, exits)
                exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, f"31 exits round {r}")
                worst = max(worst, err)
                if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
                    assert exempt
                    gs.ee_kv_truncate(os_.kv_len)
                    gs.ee_set_pending(os_.pending)
                assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
                _say(capsys, f"[7B 31 exits] round {r}: worst logits err {worst:.3g}, exit accept lengths {list(ro.exit_accept_len)}, "
                             f"final {ro.accept_len}, pass {gs.ee_pass_time_ms(len(exits)):.2f} ms")
        finally:
            gs.free()
            g.free()
            o.close()
    finally:
        if os.path.exists(path):
            os.remove(path)


@pytest.mark.timeout(600)
def test_llama7b_probabilistic_verification(llama7b_path, capsys):
    """Probabilistic verification at full size: 8 rounds, gamma 4, exits 8 and 16, temperature 0.2
    (the random-weight model's logits have a standard deviation of about 1.3 over 32000 tokens; at
    this temperature its distributions are as peaked as a trained model's, so keep tests and draws
    are decided away from their thresholds and the comparison with the oracle binds)."""
    cfg = eegen.LLAMA7B
    g = ee.Model(llama7b_path, max_rows=5)
    o = eo.Model(llama7b_path)
    prompt = eegen.prompt_tokens(20250522, 128, cfg.vocab)
    rounds, gamma = 8, 4
    try:
        exempt_rounds, bound, kept, more = sampled_chain(g, o, prompt, gamma, [8, 16], rounds, 0.2, 20250522, "7B sampled",
                                                        say=lambda m: _say(capsys, m))
        _say(capsys, f"[7B sampled] decisions bound {bound} of {rounds * 3 * (gamma + 2)}, exempt rounds {exempt_rounds}, drafts kept {kept}")
        assert bound >= 0.7 * rounds * 3 * (gamma + 2)
    finally:
        g.free()
        o.close()
