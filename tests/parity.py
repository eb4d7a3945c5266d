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
    # largest logit error, so the logit tolerance bounds the relative error of the score.
    for e in range(E + 1):
        oc = o.exit_conf[e] if e < E else o.final_conf
        gc = g_final.exit_conf[e] if e < E else g_final.final_conf
        rel = float(np.abs(np.log(gc.astype(np.float64)) - np.log(oc)).max())
        assert rel <= 2 * LOGIT_TOL, f"{what}: head {e}: confidence differs by a factor exp({rel:.3g})"
        assert np.all(gc > 0) and np.all(gc <= 1.0 + 1e-6)
    if firm[: o.accept_len + 1].all():
        assert g_final.next_token == o.next_token, f"{what}: next_token {g_final.next_token} != {o.next_token}"
    assert g_final.next_token == g_final.final_tokens[g_final.accept_len]
    return exempt, max_err


def gpu_logits(sess, n_exits):
    return [sess.ee_debug_logits(e) for e in range(n_exits + 1)]
