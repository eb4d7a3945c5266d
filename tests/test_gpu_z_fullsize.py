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
