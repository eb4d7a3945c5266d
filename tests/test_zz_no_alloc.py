"""ee_verify_static (the entry point for callers that cannot allocate GPU memory) against
ee_verify, through the C ABI: same kernels, scratch in the library's static device array
instead of the session's buffers.  Results must be bit-identical."""
import numpy as np
import pytest

import eegen
import paper_2505_21594_amd as ee

pytestmark = pytest.mark.gpu

MID = eegen.ModelConfig(n_layers=3, d_model=1280, n_heads=10, head_dim=128, d_ffn=1072, vocab=3000,
                        exit_layers=(1, 2))


def _same(a, b, what):
    assert a.accept_len == b.accept_len and a.next_token == b.next_token, what
    assert np.array_equal(a.final_tokens, b.final_tokens), what
    assert np.array_equal(a.exit_tokens, b.exit_tokens) and np.array_equal(a.exit_accept_len, b.exit_accept_len), what
    assert np.array_equal(a.final_conf.view(np.uint32), b.final_conf.view(np.uint32)), what
    assert np.array_equal(a.exit_conf.view(np.uint32), b.exit_conf.view(np.uint32)), what


def test_static_scratch_matches_session_scratch(model_dir):
    path = f"{model_dir}/noalloc_mid.bin"
    eegen.write_model(path, MID, 91, gains="uniform", std=0.03)
    g = ee.Model(path)
    exits = [1, 2]
    prompt = eegen.prompt_tokens(92, 150, MID.vocab)
    a = g.session(256, max_gamma=8, flags=ee.KEEP_LOGITS)    # ee_verify, its own scratch
    b = g.session(256, max_gamma=8, flags=ee.KEEP_LOGITS)    # ee_verify_static
    try:
        assert a.ee_prefill(prompt) == b.ee_prefill(prompt)
        # two calls in a row, the second with a smaller input; the array keeps the first call's contents
        for call, gamma in enumerate((8, 3)):
            drafts = eegen.prompt_tokens(93 + call, gamma, MID.vocab)
            if call == 0:
                drafts[0] = a.ee_pending()      # (any ids would do; makes the passes differ in what they accept)
            a.ee_verify(drafts, exits)
            a.ee_wait_final()
            b.ee_verify_static(drafts, exits)
            b.ee_wait_exit(0)
            b.ee_wait_final()
            ra, rb = a.final_result(), b.final_result()
            _same(ra, rb, f"call {call} gamma {gamma}")
            for e in range(len(exits) + 1):
                la, lb = a.ee_debug_logits(e), b.ee_debug_logits(e)
                assert np.array_equal(la.view(np.uint32), lb.view(np.uint32)), f"call {call} head {e}: logits differ"
            assert a.ee_kv_len() == b.ee_kv_len() and a.ee_pending() == b.ee_pending()
        # the ordinary entry point still works on a session that has used the static one, and the other way round
        drafts = eegen.prompt_tokens(97, 5, MID.vocab)
        b.ee_verify(drafts, exits)
        b.ee_wait_final()
        a.ee_verify_static(drafts, exits)
        a.ee_wait_final()
        _same(a.final_result(), b.final_result(), "entry points swapped")
    finally:
        a.free()
        b.free()
        g.free()


def test_static_scratch_rejects_what_does_not_fit(model_dir):
    """Sizes beyond the array's 8 MiB are refused with EE_ECAPACITY before anything is enqueued:
    a model whose FFN width makes the gate/up output of 16 rows alone larger than the array."""
    wide = eegen.ModelConfig(n_layers=1, d_model=256, n_heads=4, head_dim=64, d_ffn=140000, vocab=1024)
    path = f"{model_dir}/noalloc_wide.bin"
    eegen.write_model(path, wide, 5)
    g = ee.Model(path)
    s = g.session(64, max_gamma=15)
    try:
        s.ee_prefill(eegen.prompt_tokens(6, 9, wide.vocab))
        kv, pend = s.ee_kv_len(), s.ee_pending()
        with pytest.raises(ee.EEError) as e:
            s.ee_verify_static(eegen.prompt_tokens(7, 15, wide.vocab), [])
        assert e.value.code == ee.EE_ECAPACITY and "static scratch" in str(e.value)
        assert s.ee_kv_len() == kv and s.ee_pending() == pend
        r = s.verify_sync(eegen.prompt_tokens(7, 15, wide.vocab), [])       # the session is unharmed
        assert 0 <= r.accept_len <= 15
        # a single row of the same model fits
        s.ee_verify_static(eegen.prompt_tokens(8, 1, wide.vocab), [])
        s.ee_wait_final()
    finally:
        s.free()
        g.free()
