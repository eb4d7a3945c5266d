"""GPU parity: libeeverify (through its C ABI) against the CPU oracle on the
same seeded inputs.  Everything here needs a real MI355X."""
import numpy as np
import pytest

import eegen
import paper_2505_21594_amd as ee
from oracle import oracle as eo
from tests.parity import check_first_token, check_pass, check_sampled_pass, gpu_logits, oracle_greedy, oracle_prefill, sampled_chain

pytestmark = pytest.mark.gpu

TINY_EXITS = [2]
# several tiles along N and K, ragged K (F = 1072 -> 33.5 k-tiles), two K-blocks, hd = 128
MID = eegen.ModelConfig(n_layers=3, d_model=1280, n_heads=10, head_dim=128, d_ffn=1072, vocab=3000,
                        exit_layers=(1, 2))


@pytest.fixture(scope="module")
def tiny_path(model_dir):
    p = f"{model_dir}/gpu_tiny.bin"
    eegen.write_model(p, eegen.TINY, 2024, gains="uniform")
    return p


@pytest.fixture(scope="module")
def tiny_pair(tiny_path):
    g = ee.Model(tiny_path)
    o = eo.Model(tiny_path)
    yield g, o
    g.free()


@pytest.fixture(scope="module")
def mid_pair(model_dir):
    p = f"{model_dir}/gpu_mid.bin"
    eegen.write_model(p, MID, 77, gains="uniform", std=0.03)
    g = ee.Model(p)
    o = eo.Model(p)
    yield g, o
    g.free()


def test_mfma_lane_layout():
    ee.ee_debug_mfma_layout(0)


def test_reciprocal_division_is_exact():
    """The kernels' x / d by reciprocal and multiply, over the whole range the loader admits
    (every x up to 2.5 million), for every divisor up to 4096 and the sizes that occur as divisors
    (rows * 4, workgroups, model and head widths, vocabulary)."""
    divisors = list(range(1, 4097)) + [5120, 11008, 13824, 32000, 65536, 140000, 1 << 20, 2499999, 2500000, 2500001, 1 << 30]
    assert ee.ee_debug_div_small(divisors) == 0


def _one_round(g, o, prompt, drafts, exits, flags=0, what="", options=()):
    gs = g.session(len(prompt) + 64, max_gamma=15, flags=ee.KEEP_LOGITS | flags)
    os_ = o.session(len(prompt) + 64)
    try:
        for opt, val in options:
            gs.ee_session_option(opt, val)
        first_o, margin = oracle_prefill(os_, prompt)
        first_g = gs.ee_prefill(prompt)
        same = check_first_token(gs, first_g, first_o, margin, what)
        assert gs.ee_kv_len() == os_.kv_len == len(prompt)
        ro = os_.verify(drafts, exits, commit=True, want_logits=True)
        rg = gs.verify_sync(drafts, exits)
        exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, what)
        return exempt, err, same
    finally:
        gs.free()


@pytest.mark.parametrize("seed", range(6))
def test_tiny_single_round(tiny_pair, seed):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(seed, 64, o.vocab)
    s = o.session(96)
    s.prefill(prompt)
    drafts = eegen.corrupt_drafts(oracle_greedy(s, 4), 0.3, o.vocab, seed, 0)
    _one_round(g, o, prompt, drafts, TINY_EXITS, what=f"tiny seed {seed}")


@pytest.mark.parametrize("n_prompt,gamma", [(1, 1), (2, 4), (15, 8), (16, 15), (17, 3), (33, 5), (100, 4)])
def test_tiny_ragged_shapes(tiny_pair, n_prompt, gamma):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(100 + n_prompt, n_prompt, o.vocab)
    drafts = eegen.prompt_tokens(200 + gamma, gamma, o.vocab)
    _one_round(g, o, prompt, drafts, TINY_EXITS, what=f"tiny P={n_prompt} gamma={gamma}")


def test_tiny_runs_bit_identical(tiny_pair):
    """Every reduction has a fixed order: two runs (fresh sessions) give bit-identical logits."""
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(7, 40, o.vocab)
    drafts = eegen.prompt_tokens(8, 4, o.vocab)
    outs = []
    for _ in range(3):
        gs = g.session(128, max_gamma=8, flags=ee.KEEP_LOGITS)
        gs.ee_prefill(prompt)
        r = gs.verify_sync(drafts, TINY_EXITS)
        outs.append((r, gpu_logits(gs, 1)))
        gs.free()
    for r, lg in outs[1:]:
        assert r.accept_len == outs[0][0].accept_len and r.next_token == outs[0][0].next_token
        for a, b in zip(lg, outs[0][1]):
            assert np.array_equal(a, b)


def _chain(g, o, prompt, gamma, exits, rounds, p_corrupt, seed, max_ctx, what):
    gs = g.session(max_ctx, max_gamma=gamma, flags=ee.KEEP_LOGITS)
    os_ = o.session(max_ctx)
    exempt_rounds, max_err = 0, 0.0
    try:
        first_o, margin = oracle_prefill(os_, prompt)
        first_g = gs.ee_prefill(prompt)
        check_first_token(gs, first_g, first_o, margin, what)
        hist = list(prompt) + [first_o]      # every committed token; the last one is pending
        for r_i in range(rounds):
            drafts = eegen.corrupt_drafts(oracle_greedy(os_, gamma), p_corrupt, o.vocab, seed, r_i)
            ro = os_.verify(drafts, exits, commit=True, want_logits=True)
            hist += [int(t) for t in drafts[:ro.accept_len]] + [int(ro.next_token)]
            gs.ee_verify(drafts, exits)
            for e in range(len(exits)):
                gs.ee_wait_exit(e)
            gs.ee_wait_final()
            rg = gs.final_result()
            exempt, err = check_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, f"{what} round {r_i}")
            max_err = max(max_err, err)
            if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
                # only possible at an exempt row: put the GPU session on the oracle's trajectory
                assert exempt
                exempt_rounds += 1
                gs.ee_prefill(hist, flags=ee.HOLD_LAST)
            assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
    finally:
        gs.free()
    return exempt_rounds, max_err


def test_tiny_chain_with_rollback(tiny_pair):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(3, 64, o.vocab)
    _chain(g, o, prompt, 4, TINY_EXITS, rounds=12, p_corrupt=0.3, seed=5, max_ctx=64 + 12 * 5 + 8, what="tiny chain")


def test_mid_model_chain(mid_pair):
    g, o = mid_pair
    prompt = eegen.prompt_tokens(9, 70, o.vocab)
    _chain(g, o, prompt, 5, [1, 2], rounds=5, p_corrupt=0.4, seed=6, max_ctx=160, what="mid chain")


def test_mid_model_gamma8_no_exits(mid_pair):
    g, o = mid_pair
    prompt = eegen.prompt_tokens(19, 130, o.vocab)
    _chain(g, o, prompt, 8, [], rounds=3, p_corrupt=0.5, seed=7, max_ctx=200, what="mid gamma 8")


def test_truncate_and_refeed(tiny_pair):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(41, 30, o.vocab)
    gs = g.session(96, max_gamma=4, flags=ee.KEEP_LOGITS)
    gs.ee_prefill(prompt)
    kv, pend = gs.ee_kv_len(), gs.ee_pending()
    d1 = eegen.prompt_tokens(42, 4, o.vocab)
    r1 = gs.verify_sync(d1, TINY_EXITS)
    l1 = gpu_logits(gs, 1)
    gs.verify_sync(eegen.prompt_tokens(43, 4, o.vocab), TINY_EXITS)
    gs.ee_kv_truncate(kv)
    gs.ee_set_pending(pend)
    r2 = gs.verify_sync(d1, TINY_EXITS)
    l2 = gpu_logits(gs, 1)
    assert r1.accept_len == r2.accept_len and list(r1.final_tokens) == list(r2.final_tokens)
    for a, b in zip(l1, l2):
        assert np.array_equal(a, b)
    gs.free()


def test_hold_last_and_embedding_prefix(tiny_pair):
    g, o = tiny_pair
    emb = eegen.embedding_prefix(81, 37, o.d_model)
    toks = eegen.prompt_tokens(82, 9, o.vocab)
    drafts = eegen.prompt_tokens(83, 4, o.vocab)
    for flags_o, flags_g in ((0, 0), (eo.HOLD_LAST, ee.HOLD_LAST)):
        gs = g.session(96, max_gamma=4, flags=ee.KEEP_LOGITS)
        os_ = o.session(96)
        fg = gs.ee_prefill(toks, flags=flags_g, emb=emb)
        if flags_g == 0:
            fo, margin = oracle_prefill(os_, toks, emb=emb)
            check_first_token(gs, fg, fo, margin, "embedding prefix")
        else:
            os_.prefill(toks, flags=flags_o, emb=emb)
        assert gs.ee_kv_len() == os_.kv_len
        ro = os_.verify(drafts, TINY_EXITS, want_logits=True)
        rg = gs.verify_sync(drafts, TINY_EXITS)
        check_pass(ro, rg, gpu_logits(gs, 1), drafts, "embedding prefix")
        gs.free()


def test_no_autocommit(tiny_pair):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(51, 20, o.vocab)
    gs = g.session(64, max_gamma=4, flags=ee.NO_AUTOCOMMIT)
    gs.ee_prefill(prompt)
    kv, pend = gs.ee_kv_len(), gs.ee_pending()
    r = gs.verify_sync(eegen.prompt_tokens(52, 4, o.vocab), TINY_EXITS)
    assert gs.ee_kv_len() == kv and gs.ee_pending() == pend
    r2 = gs.verify_sync(eegen.prompt_tokens(52, 4, o.vocab), TINY_EXITS)
    assert list(r.final_tokens) == list(r2.final_tokens)
    gs.free()


def test_error_paths(tiny_pair):
    g, o = tiny_pair
    gs = g.session(16, max_gamma=8)
    with pytest.raises(ee.EEError) as e:
        gs.ee_verify([1, 2], TINY_EXITS)
    assert e.value.code == ee.EE_ESTATE
    gs.ee_prefill(eegen.prompt_tokens(1, 8, o.vocab))
    for bad in ([0], [4], [3], [2, 2], [5]):
        with pytest.raises(ee.EEError) as e:
            gs.ee_verify([1, 2], bad)
        assert e.value.code == ee.EE_EINVAL
    with pytest.raises(ee.EEError) as e:
        gs.ee_verify([o.vocab], TINY_EXITS)
    assert e.value.code == ee.EE_EINVAL
    with pytest.raises(ee.EEError) as e:
        gs.ee_verify([], TINY_EXITS)
    assert e.value.code == ee.EE_EINVAL
    with pytest.raises(ee.EEError) as e:
        gs.ee_verify([1] * 9, TINY_EXITS)
    assert e.value.code == ee.EE_EINVAL          # beyond max_gamma
    with pytest.raises(ee.EEError) as e:
        gs.ee_verify([1] * 8, TINY_EXITS)
    assert e.value.code == ee.EE_ECAPACITY       # 8 + 9 rows > max_ctx 16
    with pytest.raises(ee.EEError) as e:
        gs.ee_kv_truncate(9)
    assert e.value.code == ee.EE_EINVAL
    with pytest.raises(ee.EEError) as e:
        gs.ee_wait_final()
    assert e.value.code == ee.EE_ESTATE
    with pytest.raises(ee.EEError) as e:
        gs.ee_prefill(list(range(40)))
    assert e.value.code == ee.EE_ECAPACITY
    # the session still works after the rejected calls
    gs.ee_prefill(eegen.prompt_tokens(1, 8, o.vocab))
    gs.verify_sync([1, 2, 3], TINY_EXITS)
    gs.free()


def test_batched_sessions_match_single(model_dir):
    """Eight sessions in one pass (multi-client serving) = each session alone."""
    p = f"{model_dir}/gpu_tiny_b.bin"
    eegen.write_model(p, eegen.TINY, 31, gains="uniform")
    g = ee.Model(p, max_rows=40)
    o = eo.Model(p)
    B, gamma = 8, 4
    sess, osess, drafts = [], [], []
    for b in range(B):
        emb = eegen.embedding_prefix(300, 20 + 3 * b, o.d_model, session=b)
        toks = eegen.prompt_tokens(301, 5 + b, o.vocab, session=b)
        gs = g.session(128, max_gamma=gamma, flags=ee.KEEP_LOGITS if b == 0 else 0)
        os_ = o.session(128)
        fo, margin = oracle_prefill(os_, toks, emb=emb)
        check_first_token(gs, gs.ee_prefill(toks, emb=emb), fo, margin, f"batch session {b}")
        sess.append(gs)
        osess.append(os_)
    for rnd in range(3):
        drafts = []
        for b in range(B):
            probe = osess[b].verify([0] * gamma, commit=False)
            d = np.array([probe.final_tokens[0]] + [0] * (gamma - 1), dtype=np.int32)
            drafts.append(eegen.corrupt_drafts(d, 0.3, o.vocab, 302 + rnd, rnd, session=b))
        ee.ee_verify_batch(sess, drafts, TINY_EXITS)
        for b in range(B):
            sess[b].ee_wait_exit(0)
            sess[b].ee_wait_final()
            ro = osess[b].verify(drafts[b], TINY_EXITS, want_logits=True)
            rg = sess[b].final_result()
            check_pass(ro, rg, gpu_logits(sess[b], 1), drafts[b], f"batch round {rnd} session {b}")
            assert rg.accept_len == ro.accept_len and rg.next_token == ro.next_token, \
                "low-margin divergence in the batch test: pick another seed"
            assert sess[b].ee_kv_len() == osess[b].kv_len
    for s in sess:
        s.free()
    g.free()


def test_exit_results_visible_before_final(mid_pair):
    """Exit tokens are published while the pass is still running: the exit
    event's GPU timestamp precedes the final one."""
    g, o = mid_pair
    prompt = eegen.prompt_tokens(61, 50, o.vocab)
    gs = g.session(128, max_gamma=4)
    gs.ee_prefill(prompt)
    gs.ee_verify(eegen.prompt_tokens(62, 4, o.vocab), [1, 2])
    gs.ee_wait_exit(0)
    assert gs.ee_query_exit(0)                       # EE_OK: published
    toks, delta = gs.exit_result(0)
    assert 0 <= delta <= 4 and all(0 <= t < o.vocab for t in toks)
    gs.ee_wait_final()
    assert gs.ee_query_final() and gs.ee_query_exit(1)
    t0, t1, tf = gs.ee_pass_time_ms(0), gs.ee_pass_time_ms(1), gs.ee_pass_time_ms(2)
    assert 0 < t0 < t1 < tf
    gs.free()


@pytest.mark.parametrize("splits,prompt_len", [(1, 300), (2, 500), (3, 200)])
def test_attention_several_pages_per_wave(mid_pair, splits, prompt_len):
    """Few attention splits on a longer context: a wave then walks several KV pages per item
    (normally the split count is chosen so that a wave gets about one)."""
    g, o = mid_pair
    prompt = eegen.prompt_tokens(900 + splits, prompt_len, o.vocab)
    drafts = eegen.prompt_tokens(901 + splits, 7, o.vocab)
    exempt, err, _ = _one_round(g, o, prompt, drafts, [1, 2], what=f"splits={splits} P={prompt_len}",
                                options=[(ee.OPT_ATT_SPLITS, splits)])
    assert err <= 3e-2


def test_gamma_extremes_and_page_boundary(tiny_pair):
    """gamma = 1 and gamma = 15 (the most rows of one attention item), prompts that end right
    before, on and after a page boundary."""
    g, o = tiny_pair
    for P in (15, 16, 17, 31, 32):
        for gamma in (1, 15):
            prompt = eegen.prompt_tokens(700 + P, P, o.vocab)
            drafts = eegen.prompt_tokens(701 + P + gamma, gamma, o.vocab)
            _one_round(g, o, prompt, drafts, TINY_EXITS, what=f"P={P} gamma={gamma}")


def test_scattered_pages_use_the_page_table(tiny_pair, mid_pair):
    """A fresh session's pages are consecutive and the kernels then skip the table lookup;
    with the pages handed out in descending order the lookup path runs."""
    for (g, o), exits in ((tiny_pair, TINY_EXITS), (mid_pair, [1, 2])):
        prompt = eegen.prompt_tokens(1200, 75, o.vocab)
        drafts = eegen.prompt_tokens(1201, 6, o.vocab)
        _one_round(g, o, prompt, drafts, exits, what="scattered pages", options=[(ee.OPT_SCATTER_PAGES, 1)])


def test_empty_cache_and_exit_after_every_layer(model_dir):
    """Degenerate cases: the first round of the paper's client (prompt of one token held back,
    nothing cached: attention sees only the pass's own rows) and an exit after every layer."""
    cfg = eegen.ModelConfig(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                            exit_layers=(1, 2, 3))
    p = f"{model_dir}/gpu_tiny_all_exits.bin"
    eegen.write_model(p, cfg, 31, gains="uniform")
    g, o = ee.Model(p), eo.Model(p)
    try:
        for n_prompt in (1, 2):
            prompt = eegen.prompt_tokens(40 + n_prompt, n_prompt, cfg.vocab)
            drafts = eegen.prompt_tokens(50 + n_prompt, 4, cfg.vocab)
            gs = g.session(64, max_gamma=8, flags=ee.KEEP_LOGITS)
            os_ = o.session(64)
            os_.prefill(prompt, flags=eo.HOLD_LAST)
            gs.ee_prefill(prompt, flags=ee.HOLD_LAST)
            assert gs.ee_kv_len() == os_.kv_len == n_prompt - 1
            for rnd in range(3):
                ro = os_.verify(drafts, [1, 2, 3], commit=True, want_logits=True)
                rg = gs.verify_sync(drafts, [1, 2, 3])
                exempt, _ = check_pass(ro, rg, gpu_logits(gs, 3), drafts, f"prompt {n_prompt} round {rnd}")
                if exempt and (rg.accept_len != ro.accept_len or rg.next_token != ro.next_token):
                    gs.ee_kv_truncate(os_.kv_len)
                    gs.ee_set_pending(os_.pending)
                assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
            gs.free()
    finally:
        g.free()


@pytest.mark.parametrize("B,gamma,max_rows", [(5, 2, 15), (7, 1, 14), (3, 7, 24), (6, 4, 30), (3, 15, 48), (16, 2, 48)])
def test_batch_shapes(model_dir, B, gamma, max_rows):
    """Batches of one, two and three 16-row tiles with ragged last tiles (15, 14, 24, 30, 48
    rows); also: more rows than the model was loaded for is refused."""
    p = f"{model_dir}/gpu_tiny_groups.bin"
    eegen.write_model(p, eegen.TINY, 77, gains="uniform")
    g = ee.Model(p, max_rows=max_rows)
    o = eo.Model(p)
    sess, osess = [], []
    try:
        for b in range(B):
            toks = eegen.prompt_tokens(400, 9 + 2 * b, o.vocab, session=b)
            gs = g.session(96, max_gamma=gamma)
            os_ = o.session(96)
            fo, margin = oracle_prefill(os_, toks)
            check_first_token(gs, gs.ee_prefill(toks), fo, margin, f"B={B} session {b}")
            sess.append(gs)
            osess.append(os_)
        for rnd in range(2):
            drafts = [eegen.prompt_tokens(401 + rnd, gamma, o.vocab, session=b) for b in range(B)]
            ee.ee_verify_batch(sess, drafts, TINY_EXITS)
            for b in range(B):
                sess[b].ee_wait_final()
                ro = osess[b].verify(drafts[b], TINY_EXITS, want_logits=True)
                rg = sess[b].final_result()
                exempt, _ = check_pass(ro, rg, None, drafts[b], f"B={B} gamma={gamma} round {rnd} session {b}")
                if exempt and (rg.accept_len != ro.accept_len or rg.next_token != ro.next_token):
                    sess[b].ee_kv_truncate(osess[b].kv_len)
                    sess[b].ee_set_pending(osess[b].pending)
                assert sess[b].ee_kv_len() == osess[b].kv_len and sess[b].ee_pending() == osess[b].pending
        if B * (gamma + 1) == max_rows and B < ee.EE_MAX_BATCH:
            extra = g.session(96, max_gamma=gamma)
            extra.ee_prefill(eegen.prompt_tokens(402, 8, o.vocab))
            with pytest.raises(ee.EEError) as e:
                ee.ee_verify_batch(sess + [extra], [d for d in drafts] + [drafts[0]], TINY_EXITS)
            assert e.value.code == ee.EE_EINVAL
            extra.free()
    finally:
        for s in sess:
            s.free()
        g.free()


@pytest.mark.parametrize("ksl,B,gamma", [(2, 6, 4), (1, 3, 15), (3, 6, 4), (2, 16, 2)])
def test_k_split_over_workgroups(model_dir, ksl, B, gamma):
    """Launches of more than 16 rows with K split over groups of 2, 4 and 8 workgroups, forced for
    every GEMM kind (QKV, O, gate/up, down, adapters, LM head: each epilogue runs on the partial
    tiles of the splits), two and three row tiles, a prefill chunk of more than 16 rows included;
    twice the same pass gives bit-identical results (the sums do not depend on which workgroup
    arrives last)."""
    cfg = eegen.ModelConfig(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=640, vocab=1024,
                            exit_layers=(1, 3), n_adapters=2, adapter_width=64)
    p = f"{model_dir}/gpu_ksplit.bin"
    eegen.write_model(p, cfg, 91, gains="uniform", std=0.05)
    ee.ee_tune_k_split(127, ksl)
    try:
        g = ee.Model(p, max_rows=48)
    finally:
        ee.ee_tune_k_split(0b1010, 2)   # back to the default: output and down projection, four splits
    o = eo.Model(p)
    exits = [1, 3]
    sess, osess = [], []
    try:
        for b in range(B):
            toks = eegen.prompt_tokens(410, 19 + 3 * b, o.vocab, session=b)
            gs = g.session(128, max_gamma=gamma, flags=ee.KEEP_LOGITS if b == 0 else 0)
            os_ = o.session(128)
            fo, margin = oracle_prefill(os_, toks)
            check_first_token(gs, gs.ee_prefill(toks), fo, margin, f"k split session {b}")
            sess.append(gs)
            osess.append(os_)
        for rnd in range(2):
            drafts = [eegen.prompt_tokens(411 + rnd, gamma, o.vocab, session=b) for b in range(B)]
            again = None
            if rnd == 0:     # the same pass twice, without committing the first time
                lens = [s_.ee_kv_len() for s_ in sess]
                pend = [s_.ee_pending() for s_ in sess]
                ee.ee_verify_batch(sess, drafts, exits)
                for s_ in sess:
                    s_.ee_wait_final()
                again = [sess[b].final_result() for b in range(B)]
                for b in range(B):
                    sess[b].ee_kv_truncate(lens[b])
                    sess[b].ee_set_pending(pend[b])
            ee.ee_verify_batch(sess, drafts, exits)
            for b in range(B):
                sess[b].ee_wait_final()
                ro = osess[b].verify(drafts[b], exits, want_logits=True)
                rg = sess[b].final_result()
                if again is not None:
                    assert np.array_equal(rg.final_tokens, again[b].final_tokens) and np.array_equal(rg.exit_tokens, again[b].exit_tokens)
                    assert np.array_equal(rg.exit_conf.view(np.uint32), again[b].exit_conf.view(np.uint32))
                exempt, _ = check_pass(ro, rg, None, drafts[b], f"k split {1 << ksl} B={B} round {rnd} session {b}")
                if exempt and (rg.accept_len != ro.accept_len or rg.next_token != ro.next_token):
                    sess[b].ee_kv_truncate(osess[b].kv_len)
                    sess[b].ee_set_pending(osess[b].pending)
                assert sess[b].ee_kv_len() == osess[b].kv_len and sess[b].ee_pending() == osess[b].pending
    finally:
        for s_ in sess:
            s_.free()
        g.free()


def _with_duplicated_rows(src_path, dst_path, groups):
    """Copy of a model file in which, for every (source id, [ids]) in groups, the LM-head rows
    `ids` are overwritten with the row of the source id: their logits tie exactly."""
    import shutil
    shutil.copyfile(src_path, dst_path)
    cfg = eegen.read_header(dst_path)
    off, shape = eegen.tensor_table(cfg)[0]["w_lm"]
    mm = np.memmap(dst_path, dtype=np.uint16, mode="r+", offset=off, shape=shape)
    for src, ids in groups:
        for i in ids:
            mm[i] = mm[src]
    mm.flush()
    del mm


@pytest.mark.parametrize("which", ["tiny", "mid"])
def test_argmax_ties_go_to_the_lowest_id(model_dir, tiny_path, which):
    """The lowest token id wins an exact tie (reading of the paper's argmax; the oracle has the
    same rule).  The winning LM-head row of one pass row is copied to a lower id in another
    workgroup's n-tile, to its neighbour in the same n-tile and to a higher id in a third
    n-tile, for the final head and for an exit head: the lanes of a wave, the waves' candidates
    and the workgroups' candidates all see equal values with different ids."""
    if which == "tiny":
        cfg, src, exits = eegen.TINY, tiny_path, TINY_EXITS
    else:
        cfg, exits = MID, [1, 2]
        src = f"{model_dir}/gpu_mid_tie_src.bin"
        eegen.write_model(src, MID, 77, gains="uniform", std=0.03)
    o0 = eo.Model(src)
    prompt = eegen.prompt_tokens(1500, 37, cfg.vocab)
    drafts = eegen.prompt_tokens(1501, 5, cfg.vocab)
    s0 = o0.session(96)
    s0.prefill(prompt)
    r0 = s0.verify(drafts, exits, commit=False, want_logits=True)
    margins = eo.top2_margin(r0.logits)
    row = int(np.argmax(margins[-1]))                     # the most decisive row of the final head
    groups, used = [], set()
    for head_tokens in (r0.final_tokens, r0.exit_tokens[0]):
        t = int(head_tokens[row])
        if t in used:
            continue
        ids = [i for i in (t - 16 * 3 - 1, t ^ 1, t + 16 * 5 + 2) if 0 <= i < cfg.vocab and i not in used and i != t]
        groups.append((t, ids))
        used.update(ids + [t])
    dst = f"{model_dir}/gpu_{which}_tie.bin"
    _with_duplicated_rows(src, dst, groups)
    g, o = ee.Model(dst), eo.Model(dst)
    try:
        gs = g.session(96, max_gamma=8, flags=ee.KEEP_LOGITS)
        os_ = o.session(96)
        fo, margin = oracle_prefill(os_, prompt)
        check_first_token(gs, gs.ee_prefill(prompt), fo, margin, "tie")
        ro = os_.verify(drafts, exits, commit=False, want_logits=True)
        rg = gs.verify_sync(drafts, exits)
        lg = gpu_logits(gs, len(exits))
        check_pass(ro, rg, lg, drafts, f"{which} tie")
        n_ties = 0
        for e in range(len(exits) + 1):
            ot = ro.final_tokens if e == len(exits) else ro.exit_tokens[e]
            gt = rg.final_tokens if e == len(exits) else rg.exit_tokens[e]
            for t, ids in groups:
                if int(ot[row]) == min([t] + ids):        # the tie is at the top of this head's row
                    n_ties += 1
                    assert ro.logits[e][row][t] == ro.logits[e][row][ids[0]]
                    assert int(gt[row]) == min([t] + ids), f"head {e}: GPU picked {gt[row]}, lowest tied id is {min([t] + ids)}"
                    vals = {float(lg[e][row][i]) for i in [t] + ids}
                    assert len(vals) == 1, f"head {e}: tied rows give different GPU logits {vals}"
        assert n_ties >= 1
        gs.free()
    finally:
        g.free()


def test_sender_queue_order_and_pop(model_dir):
    """Exit results leave the server in the order of their confidence score (Algorithm 2):
    ee_exit_order against the oracle's ordering of its own confidences, and the invariants of
    the live queue (ee_exit_pop): every exit at most once, only published ones, its score is the
    one of the published result, EE_DONE at the end."""
    from oracle import latency as lo
    cfg = eegen.ModelConfig(n_layers=6, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                            exit_layers=(1, 2, 3, 4, 5))
    p = f"{model_dir}/gpu_tiny_five_exits.bin"
    eegen.write_model(p, cfg, 55, gains="uniform", std=0.08)   # wider logits: confidences well apart
    g, o = ee.Model(p), eo.Model(p)
    exits = [1, 2, 3, 4, 5]
    try:
        gs = g.session(96, max_gamma=4)
        os_ = o.session(96)
        prompt = eegen.prompt_tokens(56, 20, cfg.vocab)
        fo, margin = oracle_prefill(os_, prompt)
        check_first_token(gs, gs.ee_prefill(prompt), fo, margin, "queue")
        for rnd in range(4):
            drafts = eegen.corrupt_drafts(oracle_greedy(os_, 4), 0.3, cfg.vocab, 57, rnd)
            ro = os_.verify(drafts, exits, commit=True, want_logits=True)
            gs.ee_verify(drafts, exits)
            popped = []
            while True:
                rc, e, sc = gs.ee_exit_pop(wait=True)
                if rc == ee.EE_DONE:
                    break
                assert rc == ee.EE_OK and e not in popped and gs.ee_query_exit(e)
                toks, delta = gs.exit_result(e)
                assert sc == float(gs.exit_conf(e)[: delta + 1].max())
                popped.append(e)
            assert gs.ee_exit_pop(wait=False)[0] == ee.EE_DONE
            gs.ee_wait_final()
            rg = gs.final_result()
            exempt, _ = check_pass(ro, rg, None, drafts, f"queue round {rnd}")
            order_g, scores_g = gs.ee_exit_order()
            order_o, scores_o = lo.sender_order(ro.exit_conf, ro.exit_accept_len)
            assert sorted(order_g) == list(range(len(exits)))
            assert scores_g == sorted(scores_g, reverse=True)
            if not exempt:
                np.testing.assert_allclose(scores_g, scores_o, rtol=1e-3)
                gaps = np.diff(sorted(scores_o))
                if gaps.size == 0 or gaps.min() > 1e-3 * max(scores_o):   # an order a rounding error cannot change
                    assert order_g == order_o
            if rg.accept_len != ro.accept_len or rg.next_token != ro.next_token:
                gs.ee_kv_truncate(os_.kv_len)
                gs.ee_set_pending(os_.pending)
        gs.free()
    finally:
        g.free()


AD_TINY = eegen.ModelConfig(n_layers=6, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                            exit_layers=(1, 2, 3, 4, 5), n_adapters=3, adapter_width=16)
AD_MID = eegen.ModelConfig(n_layers=3, d_model=1280, n_heads=10, head_dim=128, d_ffn=1072, vocab=3000,
                           exit_layers=(1, 2), n_adapters=3, adapter_width=128)


@pytest.mark.parametrize("which", ["tiny", "mid"])
def test_adapter_exit_heads(model_dir, which):
    """Exit heads with adapters (three bottlenecks in parallel on the layer's output, then
    RMSNorm and the shared LM head): every head's logits and tokens against the oracle, several
    rounds with commit; an exit after every layer but the last."""
    cfg = AD_TINY if which == "tiny" else AD_MID
    p = f"{model_dir}/gpu_ad_{which}.bin"
    eegen.write_model(p, cfg, 61, gains="uniform", std=0.05 if which == "tiny" else 0.03)
    g, o = ee.Model(p), eo.Model(p)
    assert g.config.n_adapters == 3 and g.config.adapter_width == cfg.adapter_width
    exits = list(cfg.exit_layers)
    try:
        prompt = eegen.prompt_tokens(62, 45, cfg.vocab)
        _chain(g, o, prompt, 4, exits, rounds=4, p_corrupt=0.3, seed=63, max_ctx=128, what=f"adapters {which}")
        _chain(g, o, prompt[:7], 7, exits[1:], rounds=2, p_corrupt=0.5, seed=64, max_ctx=64, what=f"adapters {which} gamma 7")
    finally:
        g.free()


@pytest.mark.parametrize("adapters", [False, True])
def test_exit_heads_in_groups_match_one_by_one(model_dir, adapters):
    """EE_OPT_HEAD_BATCH: the LM head streamed once for k consecutive exits gives bit-identical
    logits and results to one launch per exit; the results of a group are published together
    (after its last exit), never later than the final result."""
    cfg = AD_TINY if adapters else eegen.ModelConfig(6, 256, 4, 64, 688, 1024, (1, 2, 3, 4, 5))
    p = f"{model_dir}/gpu_groups_{int(adapters)}.bin"
    eegen.write_model(p, cfg, 65, gains="uniform", std=0.05)
    g, o = ee.Model(p, max_rows=48), eo.Model(p)
    exits = [1, 2, 3, 4, 5]
    prompt = eegen.prompt_tokens(66, 30, cfg.vocab)
    drafts = eegen.prompt_tokens(67, 4, cfg.vocab)
    try:
        os_ = o.session(64)
        fo, margin = oracle_prefill(os_, prompt)
        ro = os_.verify(drafts, exits, commit=False, want_logits=True)
        ref = None
        for k in (1, 2, 3, 5, 9):
            gs = g.session(64, max_gamma=4, flags=ee.KEEP_LOGITS)
            check_first_token(gs, gs.ee_prefill(prompt), fo, margin, "groups")
            gs.ee_session_option(ee.OPT_HEAD_BATCH, k)
            gs.ee_verify(drafts, exits)
            gs.ee_wait_exit(0)
            gs.ee_wait_final()
            rg, lg = gs.final_result(), gpu_logits(gs, len(exits))
            check_pass(ro, rg, lg, drafts, f"head batch {k}")
            times = [gs.ee_pass_time_ms(e) for e in range(len(exits) + 1)]
            assert all(a <= b for a, b in zip(times, times[1:])) and times[-2] < times[-1]
            if k >= 2:
                assert times[1] - times[0] < 0.03    # exits 0 and 1 share a group: published together (one launch of the head)
            if ref is None:
                ref = (rg, lg)
            else:
                assert np.array_equal(rg.exit_tokens, ref[0].exit_tokens) and np.array_equal(rg.final_tokens, ref[0].final_tokens)
                assert np.array_equal(rg.exit_accept_len, ref[0].exit_accept_len)
                assert np.array_equal(rg.exit_conf.view(np.uint32), ref[0].exit_conf.view(np.uint32))
                for a, b in zip(lg, ref[1]):
                    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
            gs.free()
    finally:
        g.free()


@pytest.mark.parametrize("temperature", [1.0, 0.1, 0.05])
def test_sampled_verification_tiny(tiny_pair, temperature):
    g, o = tiny_pair
    prompt = eegen.prompt_tokens(41, 48, o.vocab)
    rounds, gamma = 24, 4
    exempt_rounds, bound, kept, more = sampled_chain(g, o, prompt, gamma, TINY_EXITS, rounds, temperature, seed=21, what=f"sampled tiny T={temperature}")
    print(f"sampled tiny T={temperature}: bound {bound} of {rounds * 2 * (gamma + 2)}, exempt rounds {exempt_rounds}, drafts kept {kept}, "
          f"rounds that keep more than exact match {more}")
    # the comparison must bind almost everywhere: 2 heads x (gamma + 1 draws + 1 accept length) per round
    assert bound >= 0.8 * rounds * 2 * (gamma + 2), (bound, exempt_rounds)


def test_sampled_verification_mid(mid_pair):
    g, o = mid_pair
    prompt = eegen.prompt_tokens(43, 90, o.vocab)
    rounds, gamma = 6, 7
    exempt_rounds, bound, kept, more = sampled_chain(g, o, prompt, gamma, [1, 2], rounds, 0.2, seed=22, what="sampled mid")
    print(f"sampled mid: bound {bound} of {rounds * 3 * (gamma + 2)}, exempt rounds {exempt_rounds}, drafts kept {kept}, more than exact match {more}")
    assert bound >= 0.8 * rounds * 3 * (gamma + 2), (bound, exempt_rounds)


@pytest.mark.parametrize("B,gamma,max_rows", [(3, 4, 16), (5, 4, 25), (4, 7, 32)])
def test_sampled_verification_batch(model_dir, B, gamma, max_rows):
    """Probabilistic verification for several sessions in one pass (one, two row tiles): each
    session with its own draft distributions, uniform numbers and temperature; every session's
    heads against the oracle's sampler, several rounds with commit."""
    p = f"{model_dir}/gpu_tiny_sampled_batch.bin"
    eegen.write_model(p, eegen.TINY, 77, gains="uniform")
    g = ee.Model(p, max_rows=max_rows)
    o = eo.Model(p)
    temps = [1.0, 0.3, 0.1, 0.7, 0.05][:B]
    sess, osess, hists = [], [], []
    try:
        for b in range(B):
            toks = eegen.prompt_tokens(430, 21 + 4 * b, o.vocab, session=b)
            gs = g.session(128, max_gamma=gamma, flags=ee.KEEP_LOGITS | ee.SAMPLING)
            os_ = o.session(128)
            fo, margin = oracle_prefill(os_, toks)
            check_first_token(gs, gs.ee_prefill(toks), fo, margin, f"sampled batch session {b}")
            sess.append(gs)
            osess.append(os_)
            hists.append(list(toks) + [fo])
        bound, total = 0, 0
        for rnd in range(4):
            gen = [eegen.draft_distributions(oracle_greedy(osess[b], gamma), o.vocab, 431, rnd, session=b) for b in range(B)]
            probs, drafts, u, v = ([x[i] for x in gen] for i in range(4))
            ros = [osess[b].verify(drafts[b], TINY_EXITS, commit=False, want_logits=True) for b in range(B)]
            ee.ee_verify_sampled_batch(sess, drafts, probs, u, v, temps, TINY_EXITS)
            for b in range(B):
                sess[b].ee_wait_final()
                rg = sess[b].final_result()
                exempt, err, n_bound, fin = check_sampled_pass(ros[b], rg, gpu_logits(sess[b], len(TINY_EXITS)), drafts[b], probs[b], u[b], v[b],
                                                             temps[b], f"sampled batch B={B} round {rnd} session {b}")
                bound += n_bound
                total += (len(TINY_EXITS) + 1) * (gamma + 2)
                osess[b].commit_rows(fin.accept_len, fin.next_token)
                hists[b] += [int(t) for t in drafts[b][:fin.accept_len]] + [int(fin.next_token)]
                if rg.accept_len != fin.accept_len or rg.next_token != fin.next_token:
                    assert exempt
                    sess[b].ee_prefill(hists[b], flags=ee.HOLD_LAST)
                assert sess[b].ee_kv_len() == osess[b].kv_len and sess[b].ee_pending() == osess[b].pending
        assert bound >= 0.75 * total, (bound, total)
        # a session without EE_SAMPLING in the batch is refused
        plain = g.session(64, max_gamma=gamma)
        plain.ee_prefill(eegen.prompt_tokens(432, 8, o.vocab))
        if (B + 1) * (gamma + 1) <= max_rows:
            with pytest.raises(ee.EEError) as ei:
                ee.ee_verify_sampled_batch(sess + [plain], drafts + [drafts[0]], probs + [probs[0]], u + [u[0]], v + [v[0]], temps + [1.0], TINY_EXITS)
            assert ei.value.code == ee.EE_ESTATE
        plain.free()
    finally:
        for s_ in sess:
            s_.free()
        g.free()


def test_sampled_verification_special_cases(tiny_pair):
    """One-hot draft distributions at a low temperature reproduce the exact-match pass; the draft
    model's own distribution equal to the target's keeps every draft; argument checks."""
    g, o = tiny_pair
    V = o.vocab
    prompt = eegen.prompt_tokens(44, 40, V)
    gs = g.session(128, max_gamma=4, flags=ee.KEEP_LOGITS | ee.SAMPLING | ee.NO_AUTOCOMMIT)
    os_ = o.session(128)
    try:
        first_o, margin = oracle_prefill(os_, prompt)
        check_first_token(gs, gs.ee_prefill(prompt), first_o, margin)
        greedy = oracle_greedy(os_, 4)
        drafts = [greedy[0], greedy[1], (greedy[2] + 5) % V, greedy[3]]
        ro = os_.verify(drafts, TINY_EXITS, commit=False, want_logits=True)
        exact = gs.verify_sync(drafts, TINY_EXITS)
        onehot = np.zeros((4, V), dtype=np.float32)
        onehot[np.arange(4), drafts] = 1.0
        gs.ee_verify_sampled(drafts, onehot, [0.5] * 4, [0.5] * 5, 1e-3, TINY_EXITS)
        gs.ee_wait_final()
        rs = gs.final_result()
        if eo.top2_margin(ro.logits).min() >= 1e-2:
            assert rs.accept_len == exact.accept_len == ro.accept_len
            assert rs.next_token == exact.next_token
            assert rs.exit_accept_len[0] == exact.exit_accept_len[0]
            assert rs.exit_tokens[0][rs.exit_accept_len[0]] == exact.exit_tokens[0][exact.exit_accept_len[0]]
        # p = q (the oracle's own target distribution for these drafts): every draft is kept
        d2 = [int(t) for t in greedy]
        ro2 = os_.verify(d2, [], commit=False, want_logits=True)
        q2 = np.stack([np.exp(ro2.logits[-1][i] - ro2.logits[-1][i].max()) for i in range(4)])
        q2 = (q2 / q2.sum(axis=1, keepdims=True)).astype(np.float32)
        gs.ee_verify_sampled(d2, q2, [0.9] * 4, [0.3] * 5, 1.0, [])
        gs.ee_wait_final()
        # u = 0.9 < 1 = q/p up to the logit error: kept unless q(x) deviates by 10 %
        assert gs.final_result().accept_len == 4
        # argument checks
        for bad in (dict(u=[1.0, 0, 0, 0]), dict(v=[0, 0, 0, 0, -0.1]), dict(temperature=0.0)):
            kw = dict(u=[0.5] * 4, v=[0.5] * 5, temperature=1.0)
            kw.update(bad)
            with pytest.raises(ee.EEError) as ei:
                gs.ee_verify_sampled(d2, q2, kw["u"], kw["v"], kw["temperature"], [])
            assert ei.value.code == ee.EE_EINVAL
        plain = g.session(64, max_gamma=4)
        plain.ee_prefill(prompt[:8])
        with pytest.raises(ee.EEError) as ei:
            plain.ee_verify_sampled(d2, q2, [0.5] * 4, [0.5] * 5, 1.0, [])
        assert ei.value.code == ee.EE_ESTATE
        plain.free()
    finally:
        gs.free()
