"""Shared helpers of the GPU parity tests: the bar GPU results are held to.

Bar (from the benchmark spec): accept_len, exit and final tokens bit-exact,
except at rows where the oracle's top-2 logit margin is below 1e-2; logits
within max-abs-error 3e-2.
"""
import numpy as np

import eegen

from oracle import oracle as eo
from oracle import sampling as osamp

LOGIT_TOL = 3e-2
MARGIN = 1e-2


def check_pass(o: eo.VerifyResult, g_final, g_logits, drafts, what=""):
    """o: oracle result with logits [E+1][M][V]; g_final: binding.VerifyOutput;
    g_logits: list of [M][V] arrays (exit heads in order, final last) or None.
    Returns (exempt, max_abs_err): exempt is True when a low-margin row made the
    token comparison non-binding somewhere."""
    E = o.exit_tokens.shape[0]
    margins = eo.top2_margin(o.logits)            # [E+1][M]
    exempt = False
    max_err = 0.0
    if g_logits is not None:
        for e in range(E + 1):
            err = float(np.abs(g_logits[e].astype(np.float64) - o.logits[e]).max())
            max_err = max(max_err, err)
            assert err <= LOGIT_TOL, f"{what}: head {e} logits max-abs-err {err:.4g} > {LOGIT_TOL}"
    heads = [(o.exit_tokens[e], g_final.exit_tokens[e], o.exit_accept_len[e], g_final.exit_accept_len[e])
             for e in range(E)]
    heads.append((o.final_tokens, g_final.final_tokens, o.accept_len, g_final.accept_len))
    for e, (ot, gt, od, gd) in enumerate(heads):
        firm = margins[e] >= MARGIN
        for i in range(len(ot)):
            if firm[i]:
                assert ot[i] == gt[i], f"{what}: head {e} row {i}: token {gt[i]} != oracle {ot[i]} (margin {margins[e][i]:.3g})"
            else:
                exempt = True
        # accept length binds when every row it depends on (0..delta_oracle) is firm
        if firm[: od + 1].all():
            assert od == gd, f"{what}: head {e}: accept_len {gd} != oracle {od}"
        # whatever the margins, the GPU's accept length must follow from its own tokens
        k = 0
        while k < len(drafts) and drafts[k] == gt[k]:
            k += 1
        assert gd == k, f"{what}: head {e}: accept_len {gd} inconsistent with its tokens (first mismatch {k})"
    # Confidence score (paper Eq. 4).  ln(conf) = z_max - logsumexp(z) moves by at most twice the
    # largest logit error: 2 * LOGIT_TOL is the ceiling the logit bar implies.  With the logits
    # compared above the bound is twice the error actually seen in this pass, plus the fp32
    # rounding of the score itself (sum of V exponentials, one division).
    conf_tol = 2 * LOGIT_TOL if g_logits is None else 2 * max_err + 1e-5
    for e in range(E + 1):
        oc = o.exit_conf[e] if e < E else o.final_conf
        gc = g_final.exit_conf[e] if e < E else g_final.final_conf
        rel = float(np.abs(np.log(gc.astype(np.float64)) - np.log(oc)).max())
        assert rel <= conf_tol, f"{what}: head {e}: confidence differs by a factor exp({rel:.3g}) > exp({conf_tol:.3g})"
        assert np.all(gc > 0) and np.all(gc <= 1.0 + 1e-6)
    if firm[: o.accept_len + 1].all():
        assert g_final.next_token == o.next_token, f"{what}: next_token {g_final.next_token} != {o.next_token}"
    assert g_final.next_token == g_final.final_tokens[g_final.accept_len]
    return exempt, max_err


def gpu_logits(sess, n_exits):
    return [sess.ee_debug_logits(e) for e in range(n_exits + 1)]


def oracle_prefill(os_, tokens, emb=None):
    """Prefills the oracle session so that it ends like a plain prefill (kv_len = all rows,
    pending = the first generated token) and returns (first_token, top-2 margin of the logits
    it was taken from).  The last prompt token is held back and fed through one verify row, which
    is the only way to see the logits behind the first token."""
    os_.prefill(tokens, flags=eo.HOLD_LAST, emb=emb)
    probe = os_.verify([0], commit=False, want_logits=True)
    first = int(probe.final_tokens[0])
    margin = float(eo.top2_margin(probe.logits[-1][0]))
    r = os_.verify([(first + 1) % os_.model.vocab], commit=True)   # a draft that is rejected: commits row 0 only
    assert r.accept_len == 0 and int(r.next_token) == first
    return first, margin


def check_first_token(gs, first_g, first_o, margin, what=""):
    """ee_prefill's first token is an argmax like any other: it must equal the oracle's unless
    the oracle's own margin is below the bar (then the GPU session is put on the oracle's token)."""
    if margin >= MARGIN:
        assert first_g == first_o, f"{what}: ee_prefill first_token {first_g} != oracle {first_o} (margin {margin:.3g})"
    elif first_g != first_o:
        gs.ee_set_pending(first_o)
    return first_g == first_o


def oracle_greedy(os_, gamma):
    """The oracle session's own greedy continuation after `pending` (gamma tokens), token by
    token: each step is a one-draft pass whose draft is rejected, so it commits exactly the
    pending token and makes the model's next token pending.  The session is left unchanged."""
    kv0, pend0 = os_.kv_len, os_.pending
    V = os_.model.vocab
    out = []
    for _ in range(gamma):
        t = int(os_.verify([0], commit=False).final_tokens[0])
        r = os_.verify([(t + 1) % V], commit=True)
        assert r.accept_len == 0
        out.append(t)
    os_.kv_truncate(kv0)
    os_.set_pending(pend0)
    return out


def check_sampled_pass(o: eo.VerifyResult, g_final, g_logits, drafts, probs, u, v, temperature, what=""):
    """Probabilistic verification: the GPU's keep decisions, emitted tokens and accept lengths of
    every head against the oracle's sampler run on the oracle's own logits with the same draft
    distributions and uniform numbers.

    Where floating point decides an integer both sides can only agree when the decision is not
    within rounding of its threshold.  The GPU's logits differ from the oracle's by at most
    err (measured in this pass, <= LOGIT_TOL), so every target probability differs by a factor
    within exp(+-2 err / T); its own arithmetic (fp32 exponentials, 40-bit fixed-point sums) adds
    about 2e-5 relative.  With eps = expm1(2 err / T) + 2e-5:
      * a keep test u p(x) < q(x) binds when |u p(x) - q(x)| > eps q(x) + 1e-6 u p(x);
      * a draw binds when v * (sum of weights) is farther than 2 eps from both ends of the drawn
        token's interval of the cumulative sum (every cumulative sum and the total move by at most
        eps, since the weights are q or the positive part of q - p and sum q = 1).
    A head's accept length binds when the keep tests of rows 0..min(delta, gamma-1) bind, its
    emitted token when the draw of row delta binds as well.  Returns (exempt, max_err, n_bound)."""
    E = o.exit_tokens.shape[0]
    gamma = len(drafts)
    max_err = 0.0
    for e in range(E + 1):
        err = float(np.abs(g_logits[e].astype(np.float64) - o.logits[e]).max())
        max_err = max(max_err, err)
        assert err <= LOGIT_TOL, f"{what}: head {e} logits max-abs-err {err:.4g} > {LOGIT_TOL}"
    eps = float(np.expm1(2.0 * max_err / temperature)) + 2e-5
    exempt, n_bound = False, 0
    oracle_final = None
    for e in range(E + 1):
        r = osamp.speculative_verify(o.logits[e], drafts, probs, u, v, temperature)
        gt = g_final.exit_tokens[e] if e < E else g_final.final_tokens
        gd = int(g_final.exit_accept_len[e] if e < E else g_final.accept_len)
        up = np.array([float(u[i]) * float(probs[i][drafts[i]]) for i in range(gamma)])
        keep_firm = r.keep_gap > eps * r.q_draft + 1e-6 * up
        draw_firm = r.cdf_gap > 2.0 * eps
        for i in range(gamma + 1):
            if draw_firm[i]:
                assert gt[i] == r.tokens[i], f"{what}: head {e} row {i}: emitted token {gt[i]} != oracle {r.tokens[i]} (gap {r.cdf_gap[i]:.3g}, eps {eps:.3g})"
                n_bound += 1
            else:
                exempt = True
        if keep_firm[: min(r.accept_len, gamma - 1) + 1].all():
            assert gd == r.accept_len, f"{what}: head {e}: accept_len {gd} != oracle {r.accept_len} (kept {r.kept}, gaps {r.keep_gap})"
            n_bound += 1
        else:
            exempt = True
        assert 0 <= gd <= gamma and all(0 <= int(t) < o.logits.shape[-1] for t in gt)
        if e == E:
            oracle_final = r
            assert g_final.next_token == g_final.final_tokens[g_final.accept_len]
    # confidences are those of the exact-match pass (Eq. 4 on the logits as they are)
    conf_tol = 2 * max_err + 1e-5
    for e in range(E + 1):
        oc = o.exit_conf[e] if e < E else o.final_conf
        gc = g_final.exit_conf[e] if e < E else g_final.final_conf
        rel = float(np.abs(np.log(gc.astype(np.float64)) - np.log(oc)).max())
        assert rel <= conf_tol, f"{what}: head {e}: confidence differs by a factor exp({rel:.3g})"
    return exempt, max_err, n_bound, oracle_final


def sampled_chain(g, o, prompt, gamma, exits, rounds, temperature, seed, what, say=None):
    """Rounds of probabilistic verification on one session pair; the oracle's trajectory leads."""
    max_ctx = len(prompt) + rounds * (gamma + 1) + 8
    gs = g.session(max_ctx, max_gamma=gamma, flags=1 | 4)   # EE_KEEP_LOGITS | EE_SAMPLING
    os_ = o.session(max_ctx)
    exempt_rounds, bound, kept_total, more_than_greedy = 0, 0, 0, 0
    try:
        first_o, margin = oracle_prefill(os_, prompt)
        first_g = gs.ee_prefill(prompt)
        check_first_token(gs, first_g, first_o, margin, what)
        hist = list(prompt) + [first_o]
        for r_i in range(rounds):
            probs, drafts, u, v = eegen.draft_distributions(oracle_greedy(os_, gamma), o.vocab, seed, r_i)
            ro = os_.verify(drafts, exits, commit=False, want_logits=True)
            gs.ee_verify_sampled(drafts, probs, u, v, temperature, exits)
            for e in range(len(exits)):
                gs.ee_wait_exit(e)
            gs.ee_wait_final()
            rg = gs.final_result()
            exempt, err, n_bound, fin = check_sampled_pass(ro, rg, gpu_logits(gs, len(exits)), drafts, probs, u, v, temperature,
                                                         f"{what} round {r_i}")
            bound += n_bound
            kept_total += fin.accept_len
            more_than_greedy += int(fin.accept_len > ro.accept_len)
            os_.commit_rows(fin.accept_len, fin.next_token)
            hist += [int(t) for t in drafts[:fin.accept_len]] + [int(fin.next_token)]
            if rg.accept_len != fin.accept_len or rg.next_token != fin.next_token:
                assert exempt   # only where a decision was within rounding of its threshold
                exempt_rounds += 1
                gs.ee_prefill(hist, flags=1)   # EE_HOLD_LAST
            assert gs.ee_kv_len() == os_.kv_len and gs.ee_pending() == os_.pending
            if say:
                say(f"[{what}] round {r_i + 1}/{rounds}: logits max-abs-err {err:.3g}, bound so far {bound}, drafts kept {fin.accept_len}")
    finally:
        gs.free()
    return exempt_rounds, bound, kept_total, more_than_greedy
