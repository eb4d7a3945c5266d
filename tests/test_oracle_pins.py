"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself's cached path -- brute-force decoding without a cache,
closed forms, PyTorch-CPU library routines in float64, and invariants.

The paper prints no numeric example of the verification pass (its figure of the
method shows two draft tokens without values), so there are no paper-printed
values to store for this path.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import eegen
from eegen import bf16_to_f32
from oracle import oracle as eo

EXITS = [2]


def _mk(model_dir, name, cfg=eegen.TINY, seed=1234, **kw):
    path = f"{model_dir}/{name}.bin"
    eegen.write_model(path, cfg, seed, **kw)
    return path


@pytest.fixture(scope="module")
def tiny_path(model_dir):
    return _mk(model_dir, "tiny_u", gains="uniform")


@pytest.fixture(scope="module")
def tiny(tiny_path):
    return eo.Model(tiny_path)


@pytest.fixture(scope="module")
def tiny_wide_path(model_dir):
    # larger weight scale: attention and position matter much more, greedy text varies
    return _mk(model_dir, "tiny_wide", gains="uniform", std=0.08, seed=99)


@pytest.fixture(scope="module")
def tiny_wide(tiny_wide_path):
    return eo.Model(tiny_wide_path)


def first_mismatch(drafts, greedy):
    k = 0
    while k < len(drafts) and drafts[k] == greedy[k]:
        k += 1
    return k


# ---------------------------------------------------------------- accept rule / AR (P1-P3)

@pytest.mark.parametrize("which", ["tiny", "tiny_wide"])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_verify_matches_bruteforce_ar(which, seed, request):
    m = request.getfixturevalue(which)
    gamma = 4
    prompt = eegen.prompt_tokens(seed, 24, m.vocab)
    g = m.ar_decode(prompt, gamma + 2)              # g[0] is the first generated token
    s = m.session(128)
    assert s.prefill(prompt) == g[0]
    drafts = eegen.corrupt_drafts(g[1:1 + gamma], 0.3, m.vocab, seed, 0)
    r = s.verify(drafts, EXITS, commit=False)
    k = first_mismatch(drafts, g[1:1 + gamma])
    assert r.accept_len == k
    assert r.next_token == g[1 + k]
    # accepted drafts followed by the generated token = the first k+1 greedy tokens
    assert list(drafts[:k]) + [r.next_token] == list(g[1:k + 2])
    # every row up to the first wrong draft predicts the greedy token
    assert list(r.final_tokens[:k + 1]) == list(g[1:k + 2])


def test_all_correct_and_all_wrong(tiny_wide):
    m, gamma = tiny_wide, 5
    prompt = eegen.prompt_tokens(11, 17, m.vocab)
    g = m.ar_decode(prompt, gamma + 2)
    s = m.session(64)
    s.prefill(prompt)
    r = s.verify(g[1:1 + gamma], commit=False)
    assert r.accept_len == gamma and r.next_token == g[1 + gamma]
    wrong = g[1:1 + gamma].copy()
    wrong[0] = (wrong[0] + 1) % m.vocab
    r = s.verify(wrong, commit=False)
    assert r.accept_len == 0 and r.next_token == g[1]


@pytest.mark.parametrize("mode", ["corrupt", "random", "exact"])
def test_chain_equals_ar(tiny_wide, mode):
    """Committed tokens over many rounds = greedy continuation, for any drafts."""
    m, gamma, rounds = tiny_wide, 4, 10
    prompt = eegen.prompt_tokens(5, 12, m.vocab)
    n_ar = rounds * (gamma + 1) + gamma + 1
    g = m.ar_decode(prompt, n_ar)
    s = m.session(len(prompt) + n_ar + gamma + 2)
    committed = [s.prefill(prompt)]
    rng = np.random.default_rng(3)
    for r_i in range(rounds):
        nxt = g[len(committed):len(committed) + gamma]
        if mode == "corrupt":
            drafts = eegen.corrupt_drafts(nxt, 0.3, m.vocab, 17, r_i)
        elif mode == "random":
            drafts = rng.integers(0, m.vocab, gamma).astype(np.int32)
        else:
            drafts = nxt
        kv_before = s.kv_len
        r = s.verify(drafts, EXITS)
        assert s.kv_len == kv_before + r.accept_len + 1
        assert s.pending == r.next_token
        committed += list(drafts[:r.accept_len]) + [r.next_token]
    assert committed == list(g[:len(committed)])
    assert s.kv_len == len(prompt) + len(committed) - 1


def test_accept_rule_invariant_random(tiny):
    """accept_len is the first index where draft != argmax of the previous row."""
    m = tiny
    rng = np.random.default_rng(0)
    prompt = eegen.prompt_tokens(2, 9, m.vocab)
    s = m.session(64)
    s.prefill(prompt)
    for gamma in (1, 2, 4, 8):
        for _ in range(4):
            drafts = rng.integers(0, m.vocab, gamma).astype(np.int32)
            # force partial agreement sometimes
            probe = s.verify(drafts, EXITS, commit=False)
            drafts[0] = probe.final_tokens[0]
            r = s.verify(drafts, EXITS, commit=False)
            k = first_mismatch(drafts, r.final_tokens)
            assert r.accept_len == k and r.next_token == r.final_tokens[k]
            ke = first_mismatch(drafts, r.exit_tokens[0])
            assert r.exit_accept_len[0] == ke


# ---------------------------------------------------------------- rows vs from-scratch (P4, P5)

def test_rows_equal_from_scratch_logits(tiny_wide):
    m, gamma = tiny_wide, 4
    prompt = eegen.prompt_tokens(8, 37, m.vocab)     # 3 prefill chunks
    s = m.session(64)
    first = s.prefill(prompt)
    drafts = eegen.prompt_tokens(9, gamma, m.vocab)
    r = s.verify(drafts, EXITS, commit=False, want_logits=True)
    seq = list(prompt) + [first] + list(drafts)
    full_final = m.full_logits(seq, 0)
    full_exit = m.full_logits(seq, 2)
    P = len(prompt)
    assert np.abs(full_final[P - 1].argmax() - first) == 0
    np.testing.assert_allclose(r.logits[1], full_final[P:], atol=2e-5, rtol=0)
    np.testing.assert_allclose(r.logits[0], full_exit[P:], atol=2e-5, rtol=0)


def test_prefill_equals_single_steps(tiny_wide):
    """Chunked prefill = feeding one row at a time: start from a one-token
    hold-last prefill, then a committed single-draft verify per prompt token,
    rolled back so that exactly the pending row stays cached."""
    m = tiny_wide
    prompt = eegen.prompt_tokens(21, 19, m.vocab)
    a = m.session(64)
    a.prefill(prompt, flags=eo.HOLD_LAST)
    b = m.session(64)
    b.prefill(prompt[:1], flags=eo.HOLD_LAST)
    for t in prompt[1:]:
        kv = b.kv_len
        b.verify([int(t)], commit=True)      # advances by accept_len+1 >= 1 rows
        b.kv_truncate(kv + 1)                # keep only the row of the old pending token
        b.set_pending(int(t))
    assert a.kv_len == b.kv_len == len(prompt) - 1
    drafts = eegen.prompt_tokens(22, 3, m.vocab)
    ra = a.verify(drafts, EXITS, commit=False, want_logits=True)
    rb = b.verify(drafts, EXITS, commit=False, want_logits=True)
    np.testing.assert_allclose(ra.logits, rb.logits, atol=2e-5, rtol=0)


# ---------------------------------------------------------------- rollback (P6, P7)

def test_rollback_equals_recompute(tiny_wide):
    m, gamma = tiny_wide, 4
    prompt = eegen.prompt_tokens(31, 15, m.vocab)
    s = m.session(96)
    committed = [s.prefill(prompt)]
    rng = np.random.default_rng(5)
    for r_i in range(4):
        drafts = rng.integers(0, m.vocab, gamma).astype(np.int32)  # mostly rejected at once
        if r_i % 2:
            drafts[:2] = s.verify(drafts, commit=False).final_tokens[:1].tolist() + [drafts[1]]
        r = s.verify(drafts, EXITS)
        committed += list(drafts[:r.accept_len]) + [r.next_token]
    # fresh session that never saw the rejected rows
    f = m.session(96)
    f.prefill(list(prompt) + committed, flags=eo.HOLD_LAST)
    assert f.kv_len == s.kv_len and f.pending == s.pending
    drafts = rng.integers(0, m.vocab, gamma).astype(np.int32)
    a = s.verify(drafts, EXITS, commit=False, want_logits=True)
    b = f.verify(drafts, EXITS, commit=False, want_logits=True)
    np.testing.assert_allclose(a.logits, b.logits, atol=2e-5, rtol=0)


def test_truncate_and_refeed_is_identical(tiny_wide):
    m = tiny_wide
    prompt = eegen.prompt_tokens(41, 20, m.vocab)
    s = m.session(64)
    s.prefill(prompt)
    pend, kv = s.pending, s.kv_len
    d1 = eegen.prompt_tokens(42, 4, m.vocab)
    r1 = s.verify(d1, EXITS, commit=True, want_logits=True)
    # overwrite the tail with other rows, then roll back and feed the same rows again
    s.verify(eegen.prompt_tokens(43, 4, m.vocab), EXITS, commit=True)
    s.kv_truncate(kv)
    s.set_pending(pend)
    r2 = s.verify(d1, EXITS, commit=False, want_logits=True)
    assert np.array_equal(r1.logits, r2.logits)
    with pytest.raises(eo.OracleError):
        s.kv_truncate(s.kv_len + 1)


# ---------------------------------------------------------------- exit head (P8)

def test_exit_equals_truncated_model(model_dir, tiny_path, tiny):
    """Exit head after layer e = final head of the same model cut to e layers
    with g_final := g_exit[e] (per-layer weights are seeded by name, so the cut
    model regenerates identical layers)."""
    cfg = eegen.TINY
    cut = eegen.ModelConfig(2, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, ())
    cut_path = _mk(model_dir, "tiny_cut2", cfg=cut, gains="uniform")
    full_t = eegen.open_tensors(tiny_path)
    cut_t = eegen.open_tensors(cut_path, mode="r+")
    assert np.array_equal(full_t["l2.wd"], cut_t["l2.wd"])
    cut_t["g_final"][:] = full_t["g_exit2"]
    cut_t["g_final"].base.flush() if hasattr(cut_t["g_final"].base, "flush") else None
    del cut_t
    mc = eo.Model(cut_path)
    prompt = eegen.prompt_tokens(51, 13, cfg.vocab)
    drafts = eegen.prompt_tokens(52, 4, cfg.vocab)
    a = tiny.session(32)
    a.prefill(prompt, flags=eo.HOLD_LAST)
    b = mc.session(32)
    b.prefill(prompt, flags=eo.HOLD_LAST)
    ra = a.verify(drafts, EXITS, commit=False, want_logits=True)
    rb = b.verify(drafts, (), commit=False, want_logits=True)
    assert np.array_equal(ra.logits[0], rb.logits[0])
    assert list(ra.exit_tokens[0]) == list(rb.final_tokens)
    assert ra.exit_accept_len[0] == rb.accept_len


# ---------------------------------------------------------------- closed forms (P10)

def _rms(x, g, eps):
    return x / np.sqrt((x * x).mean(-1, keepdims=True) + eps) * g


def test_closed_form_zero_output_projections(model_dir):
    """Wo = Wd = 0 => h^(L) = Emb[row] => logits = rmsnorm(Emb[row]) . W_lm^T."""
    path = _mk(model_dir, "tiny_zero", gains="uniform", zero=("wo", "wd"))
    m = eo.Model(path)
    t = eegen.open_tensors(path)
    emb, wlm = bf16_to_f32(t["emb"]).astype(np.float64), bf16_to_f32(t["w_lm"]).astype(np.float64)
    gf, ge = bf16_to_f32(t["g_final"]).astype(np.float64), bf16_to_f32(t["g_exit2"]).astype(np.float64)
    prompt = eegen.prompt_tokens(61, 6, m.vocab)
    drafts = eegen.prompt_tokens(62, 4, m.vocab)
    s = m.session(32)
    s.prefill(prompt, flags=eo.HOLD_LAST)
    r = s.verify(drafts, EXITS, commit=False, want_logits=True)
    rows = [int(prompt[-1])] + list(drafts)
    eps = float(m.rms_eps)
    np.testing.assert_allclose(r.logits[1], _rms(emb[rows], gf, eps) @ wlm.T, atol=1e-5, rtol=0)
    np.testing.assert_allclose(r.logits[0], _rms(emb[rows], ge, eps) @ wlm.T, atol=1e-5, rtol=0)
    assert list(r.final_tokens) == list((_rms(emb[rows], gf, eps) @ wlm.T).argmax(-1))


def test_confidence_score_against_library_softmax(tiny_wide):
    """Eq. 4: every row's score equals max(softmax(z)) computed by the library routine
    from the logits the same pass returned, for the exit head and the final head."""
    import torch
    m = tiny_wide
    s = m.session(64)
    s.prefill(eegen.prompt_tokens(81, 17, m.vocab))
    r = s.verify(eegen.prompt_tokens(82, 4, m.vocab), EXITS, commit=False, want_logits=True)
    ref = torch.softmax(torch.from_numpy(r.logits), dim=-1).max(dim=-1).values.numpy()   # [E+1][M]
    np.testing.assert_allclose(r.exit_conf[0], ref[0], rtol=2e-5, atol=0)
    np.testing.assert_allclose(r.final_conf, ref[1], rtol=2e-5, atol=0)
    # and it is the probability of the token the head reports
    p = torch.softmax(torch.from_numpy(r.logits[1]), dim=-1).numpy()
    np.testing.assert_allclose(r.final_conf, p[np.arange(p.shape[0]), r.final_tokens], rtol=2e-5, atol=0)


def test_confidence_score_closed_forms(model_dir):
    """All-zero LM head => uniform distribution => score 1/V for every row and head;
    a duplicated best row of W_lm => two equal largest logits => score <= 1/2."""
    path = _mk(model_dir, "tiny_zero_lm", gains="uniform", zero=("w_lm",))
    m = eo.Model(path)
    s = m.session(32)
    s.prefill(eegen.prompt_tokens(83, 6, m.vocab))
    r = s.verify(eegen.prompt_tokens(84, 4, m.vocab), EXITS, commit=False)
    np.testing.assert_allclose(r.final_conf, 1.0 / m.vocab, rtol=1e-6)
    np.testing.assert_allclose(r.exit_conf[0], 1.0 / m.vocab, rtol=1e-6)
    assert list(r.final_tokens) == [0] * 5   # all logits equal: lowest id


def test_rope_properties(tiny_wide_path, tiny_wide):
    """Position 0 is the identity; rotation keeps each pair's norm; layer-1
    q_i . k_j of a constant-token sequence depends on i-j only."""
    m = tiny_wide
    t = eegen.open_tensors(tiny_wide_path)
    tok = 77
    s = m.session(32)
    s.prefill([tok], flags=eo.HOLD_LAST)           # kv_len 0, rows start at position 0
    r = s.verify([tok] * 7, commit=False, want_trace=True)
    tr = r.trace
    d, H, hd = m.d_model, m.n_heads, m.head_dim
    x = _rms(tr["h"][0], bf16_to_f32(t["l1.g_attn"]).astype(np.float64), float(m.rms_eps))
    q_raw = x @ bf16_to_f32(t["l1.wq"]).astype(np.float64).T
    k_raw = x @ bf16_to_f32(t["l1.wk"]).astype(np.float64).T
    q, k = tr["q"][0], tr["k"][0]
    np.testing.assert_allclose(q[0], q_raw[0], atol=1e-5)          # pos 0: identity
    np.testing.assert_allclose(k[0], k_raw[0], atol=1e-5)
    qh = q.reshape(-1, H, hd)
    qr = q_raw.reshape(-1, H, hd)
    half = hd // 2
    np.testing.assert_allclose(qh[..., :half] ** 2 + qh[..., half:] ** 2,
                               qr[..., :half] ** 2 + qr[..., half:] ** 2, atol=1e-5)
    assert np.abs(q[3] - q_raw[3]).max() > 1e-2                      # it does rotate
    kh = k.reshape(-1, H, hd)
    sc = np.einsum("ihe,jhe->hij", qh, kh)
    for i, j in [(3, 1), (5, 3), (2, 0), (7, 5)]:
        np.testing.assert_allclose(sc[:, i, j], sc[:, 2, 0], atol=1e-4)
    for i, j in [(4, 1), (6, 3), (7, 4)]:
        np.testing.assert_allclose(sc[:, i, j], sc[:, 3, 0], atol=1e-4)
    assert np.abs(sc[:, 3, 0] - sc[:, 2, 0]).max() > 1e-3


# ---------------------------------------------------------------- library routines (P11)

def _torch_reference(path, emb_rows, tokens, upto_layer, gain_name):
    """Llama block composed from PyTorch-CPU library routines in float64:
    F.embedding, F.rms_norm, F.linear, F.scaled_dot_product_attention, F.silu;
    rotary embedding as a complex multiplication."""
    cfg = eegen.read_header(path)
    t = {k: torch.from_numpy(bf16_to_f32(np.asarray(v)).astype(np.float64))
         for k, v in eegen.open_tensors(path).items()}
    H, hd, eps = cfg.n_heads, cfg.head_dim, float(np.float32(cfg.rms_eps))
    h = F.embedding(torch.as_tensor(np.asarray(tokens), dtype=torch.long), t["emb"])
    if emb_rows is not None:
        h = torch.cat([torch.from_numpy(bf16_to_f32(emb_rows).astype(np.float64)), h], 0)
    T = h.shape[0]
    inv = torch.tensor(float(cfg.rope_base), dtype=torch.float64) ** (
        -torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                    # e^{i pos theta}

    def rope(x):                                                    # x: [T, H, hd]
        z = torch.complex(x[..., :hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    hs = [h]
    for l in range(1, upto_layer + 1):
        x = F.rms_norm(h, (cfg.d_model,), t[f"l{l}.g_attn"], eps)
        q = rope(F.linear(x, t[f"l{l}.wq"]).view(T, H, hd)).transpose(0, 1)
        k = rope(F.linear(x, t[f"l{l}.wk"]).view(T, H, hd)).transpose(0, 1)
        v = F.linear(x, t[f"l{l}.wv"]).view(T, H, hd).transpose(0, 1)
        a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + F.linear(a.transpose(0, 1).reshape(T, -1), t[f"l{l}.wo"])
        x = F.rms_norm(h, (cfg.d_model,), t[f"l{l}.g_ffn"], eps)
        h = h + F.linear(F.silu(F.linear(x, t[f"l{l}.wg"])) * F.linear(x, t[f"l{l}.wu"]), t[f"l{l}.wd"])
        hs.append(h)
    z = F.linear(F.rms_norm(h, (cfg.d_model,), t[gain_name], eps), t["w_lm"])
    return z.numpy(), [x.numpy() for x in hs]


@pytest.mark.parametrize("real,tol", [("f32", 3e-5), ("f64", 1e-9)])
def test_against_torch_library_block(tiny_wide_path, real, tol):
    m = eo.Model(tiny_wide_path, real)
    prompt = eegen.prompt_tokens(71, 21, m.vocab)
    drafts = eegen.prompt_tokens(72, 4, m.vocab)
    s = m.session(64)
    s.prefill(prompt, flags=eo.HOLD_LAST)
    r = s.verify(drafts, EXITS, commit=False, want_logits=True, want_trace=True)
    seq = list(prompt) + list(drafts)
    P = len(prompt) - 1
    z_final, hs = _torch_reference(tiny_wide_path, None, seq, m.n_layers, "g_final")
    z_exit, _ = _torch_reference(tiny_wide_path, None, seq, 2, "g_exit2")
    np.testing.assert_allclose(r.logits[1], z_final[P:], atol=tol, rtol=0)
    np.testing.assert_allclose(r.logits[0], z_exit[P:], atol=tol, rtol=0)
    for l in range(m.n_layers + 1):
        np.testing.assert_allclose(r.trace["h"][l], hs[l][P:], atol=tol, rtol=0)
    # the brute-force path too
    np.testing.assert_allclose(m.full_logits(seq, 0), z_final, atol=tol, rtol=0)
    np.testing.assert_allclose(m.full_logits(seq, 2), z_exit, atol=tol, rtol=0)


def test_embedding_prefix_against_torch(tiny_wide_path, tiny_wide):
    m = tiny_wide
    emb = eegen.embedding_prefix(81, 18, m.d_model)
    toks = eegen.prompt_tokens(82, 7, m.vocab)
    drafts = eegen.prompt_tokens(83, 4, m.vocab)
    s = m.session(64)
    s.prefill(toks, flags=eo.HOLD_LAST, emb=emb)
    assert s.kv_len == 18 + 7 - 1
    r = s.verify(drafts, EXITS, commit=False, want_logits=True)
    z, _ = _torch_reference(tiny_wide_path, emb, list(toks) + list(drafts), m.n_layers, "g_final")
    np.testing.assert_allclose(r.logits[1], z[18 + 6:], atol=2e-4, rtol=0)
    # and the default prefill's first token
    s2 = m.session(64)
    first = s2.prefill(toks, emb=emb)
    z2, _ = _torch_reference(tiny_wide_path, emb, list(toks), m.n_layers, "g_final")
    assert first == int(z2[-1].argmax())


def test_f32_and_f64_builds_agree(tiny_path):
    a, b = eo.Model(tiny_path, "f32"), eo.Model(tiny_path, "f64")
    prompt = eegen.prompt_tokens(91, 64, a.vocab)
    sa, sb = a.session(96), b.session(96)
    assert sa.prefill(prompt) == sb.prefill(prompt)
    drafts = eegen.prompt_tokens(92, 4, a.vocab)
    ra = sa.verify(drafts, EXITS, want_logits=True)
    rb = sb.verify(drafts, EXITS, want_logits=True)
    assert np.abs(ra.logits - rb.logits).max() < 5e-6


# ---------------------------------------------------------------- argmax ties (P12)

def test_argmax_tie_goes_to_lowest_index(model_dir, tiny_path):
    import shutil
    path = f"{model_dir}/tiny_tie.bin"
    shutil.copy(tiny_path, path)
    m = eo.Model(path)
    prompt = eegen.prompt_tokens(101, 10, m.vocab)
    drafts = eegen.prompt_tokens(102, 3, m.vocab)
    s = m.session(32)
    s.prefill(prompt, flags=eo.HOLD_LAST)
    base = s.verify(drafts, EXITS, commit=False, want_logits=True)
    a = int(base.final_tokens[0])
    lo, hi = (a - 5) % m.vocab, (a + 5) % m.vocab
    lo, hi = min(lo, hi), max(lo, hi)
    m.close()
    t = eegen.open_tensors(path, mode="r+")
    t["w_lm"][hi if hi != a else lo] = t["w_lm"][a]     # duplicate the winning row elsewhere
    other = hi if hi != a else lo
    del t
    m2 = eo.Model(path)
    s2 = m2.session(32)
    s2.prefill(prompt, flags=eo.HOLD_LAST)
    r = s2.verify(drafts, EXITS, commit=False, want_logits=True)
    assert r.logits[1][0, a] == r.logits[1][0, other]
    assert eo.top2_margin(r.logits[1][0]) == 0.0
    assert r.final_tokens[0] == min(a, other)


# ---------------------------------------------------------------- errors

def test_error_paths(tiny):
    m = tiny
    s = m.session(16)
    with pytest.raises(eo.OracleError) as e:
        s.verify([1, 2], EXITS)
    assert e.value.code == eo.EO_ESTATE
    s.prefill(eegen.prompt_tokens(1, 8, m.vocab))
    for bad_exits in ([0], [4], [3], [2, 2], [5]):
        with pytest.raises(eo.OracleError) as e:
            s.verify([1, 2], bad_exits)
        assert e.value.code == eo.EO_EINVAL
    with pytest.raises(eo.OracleError) as e:
        s.verify([m.vocab], EXITS)
    assert e.value.code == eo.EO_EINVAL
    with pytest.raises(eo.OracleError) as e:
        s.verify([1] * 8, EXITS)
    assert e.value.code == eo.EO_ECAPACITY
    with pytest.raises(eo.OracleError):
        eo.Model("/nonexistent/file")


# ---------------------------------------------------------------- exit heads with adapters

AD_CFG = eegen.ModelConfig(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024,
                           exit_layers=(1, 2, 3), n_adapters=3, adapter_width=16)


def test_adapter_parameter_counts_match_the_papers_table():
    """The fine-tuning table's trainable-parameter counts fix the adapters' shape: three
    bias-carrying bottlenecks of width 128 after each of the 32 / 40 layers (values in
    tests/golden/adapter_parameter_counts.txt)."""
    import os
    gold = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "adapter_parameter_counts.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            gold[t[0]] = int(t[1])
    for base, key in ((eegen.LLAMA7B, "llama2_7b"), (eegen.LLAMA13B, "vicuna_13b")):
        cfg = eegen.ModelConfig(base.n_layers, base.d_model, base.n_heads, base.head_dim, base.d_ffn, base.vocab,
                                tuple(range(1, base.n_layers)), n_adapters=3, adapter_width=128)
        assert eegen.adapter_parameters(cfg, base.n_layers) == gold[key]
        # and the file the generator writes holds exactly these tensors per exit head
        table, _ = eegen.tensor_table(cfg)
        per_exit = sum(int(np.prod(shape)) for name, (_, shape) in table.items() if name in ("ad_down1", "ad_bdown1", "ad_up1", "ad_bup1"))
        assert per_exit * base.n_layers == gold[key]


def test_adapter_with_zero_output_is_the_plain_exit_head(model_dir):
    """W_up = 0 and b_up = 0 make every adapter add nothing: the exit head is then RMSNorm +
    LM head on the layer's output, i.e. the logits of the same model without adapters."""
    plain = eegen.ModelConfig(AD_CFG.n_layers, AD_CFG.d_model, AD_CFG.n_heads, AD_CFG.head_dim, AD_CFG.d_ffn, AD_CFG.vocab,
                              AD_CFG.exit_layers)
    pa = _mk(model_dir, "ad_zero_up", cfg=AD_CFG, gains="uniform", zero=("ad_up*", "ad_bup*"))
    pp = _mk(model_dir, "ad_plain", cfg=plain, gains="uniform")
    ma, mp = eo.Model(pa), eo.Model(pp)
    prompt, drafts = eegen.prompt_tokens(71, 9, plain.vocab), eegen.prompt_tokens(72, 4, plain.vocab)
    out = []
    for m in (ma, mp):
        s = m.session(32)
        s.prefill(prompt)
        out.append(s.verify(drafts, [1, 2, 3], commit=False, want_logits=True))
    assert np.array_equal(out[0].logits, out[1].logits)
    assert np.array_equal(out[0].exit_tokens, out[1].exit_tokens)


@pytest.mark.parametrize("real,tol", [("f64", 1e-9), ("f32", 2e-4)])
def test_adapter_exit_head_against_numpy(model_dir, real, tol):
    """a = h + sum_j (W_up,j silu(W_down,j h + b_down,j) + b_up,j), z = W_lm RMSNorm(a; g_exit), restated
    in float64 numpy on the layer outputs the oracle reports; the final head stays without adapter."""
    path = _mk(model_dir, "ad_full", cfg=AD_CFG, gains="uniform", std=0.05)
    m = eo.Model(path, real=real)
    t = eegen.open_tensors(path)
    f = lambda name: bf16_to_f32(t[name]).astype(np.float64)
    prompt, drafts = eegen.prompt_tokens(73, 11, AD_CFG.vocab), eegen.prompt_tokens(74, 5, AD_CFG.vocab)
    s = m.session(32)
    s.prefill(prompt)
    r = s.verify(drafts, [1, 3], commit=False, want_logits=True, want_trace=True)
    eps = float(m.rms_eps)
    for idx, e in enumerate((1, 3)):
        h = r.trace["h"][e]                                    # output of layer e, [M][d]
        pre = h @ f(f"ad_down{e}").T + f(f"ad_bdown{e}")
        act = pre / (1.0 + np.exp(-pre))
        a = h + act @ f(f"ad_up{e}").T + f(f"ad_bup{e}").sum(0)
        z = _rms(a, f(f"g_exit{e}"), eps) @ f("w_lm").T
        np.testing.assert_allclose(r.logits[idx], z, atol=tol, rtol=0)
        # the adapter really changes the logits (the pin would be blind otherwise)
        assert np.abs(z - _rms(h, f(f"g_exit{e}"), eps) @ f("w_lm").T).max() > 1e-2
    zf = _rms(r.trace["h"][AD_CFG.n_layers], f("g_final"), eps) @ f("w_lm").T
    np.testing.assert_allclose(r.logits[2], zf, atol=tol, rtol=0)
    # brute force without a cache goes through the same head
    full = m.full_logits(list(prompt) + [s.pending] + list(drafts), exit_layer=3)
    np.testing.assert_allclose(full[-6:], r.logits[1], atol=max(tol, 1e-5), rtol=0)
