"""Shared helpers of the GPU parity tests: the bar GPU results are held to.

Bar (from the benchmark spec): accept_len, exit and final tokens bit-exact,
except at rows where the oracle's top-2 logit margin is below 1e-2; logits
within max-abs-error 3e-2.
"""
import numpy as np

from oracle import oracle as eo

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
