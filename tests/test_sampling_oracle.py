"""Pins of the probabilistic-verification oracle (oracle/sampling.py) against what the scheme and
the mathematics fix, and planted mistakes that each must trip at least one pin.

What pins it (none of these re-types the oracle's formulas):
  * the theorem the scheme rests on: a draft drawn from p, kept or replaced by the rule, is
    distributed exactly as q = softmax(z / T) (q from scipy's softmax) -- checked by integrating
    the oracle's decisions over dense midpoint grids of u and v, for every draft token;
  * the share of drafts kept is sum_k min(p_k, q_k);
  * p = q keeps everything; a draft the target gives no mass is never kept and the replacement
    then follows q itself;
  * as T -> 0 with one-hot draft distributions the rule becomes the greedy accept rule: the
    C oracle's own verify result on a tiny model;
  * inversion of a cumulative sum on a hand-made example, zero-weight tokens never drawn.
"""
import importlib.util
import os
import sys

import numpy as np
import pytest
import scipy.special

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
SRC = os.path.join(ROOT, "oracle", "sampling.py")


def load(path=SRC, name="sampling_under_test"):
    spec = importlib.util.spec_from_file_location(name, path)
    mod = importlib.util.module_from_spec(spec)
    sys.modules[name] = mod   # dataclasses look the module up while the class is being built
    spec.loader.exec_module(mod)
    return mod


def grid(n):
    return (np.arange(n) + 0.5) / n


def case(seed, V, T, scale=1.5):
    rng = np.random.default_rng(seed)
    z = rng.normal(size=V) * scale
    p = rng.dirichlet(np.ones(V) * 0.7)
    q = scipy.special.softmax(z / T)
    return z, p, q


# ---- pins (each takes the module under test)

def pin_output_distribution(sp):
    """P(emitted = k) = sum_d p_d [kept(d) 1{k = d} + (1 - kept(d)) resid_k] must equal q_k."""
    G = 4000
    for seed, V, T in ((1, 6, 1.0), (2, 9, 0.6), (3, 5, 2.0)):
        z, p, q = case(seed, V, T)
        out = np.zeros(V)
        for d in range(V):
            r_keep = np.mean([sp.speculative_verify(np.stack([z, z]), [d], p[None], [u], [0.5, 0.5], T).kept[0] for u in grid(G)])
            hist = np.zeros(V)
            for v in grid(G):
                hist[sp.speculative_verify(np.stack([z, z]), [d], p[None], [0.999999], [v, 0.5], T).tokens[0]] += 1.0 / G
            out[d] += p[d] * r_keep
            out += p[d] * (1.0 - r_keep) * hist
        assert np.abs(out - q).max() < 3e-3, (seed, out, q)


def pin_keep_rate(sp):
    G = 4000
    z, p, q = case(7, 8, 0.8)
    rate = sum(p[d] * np.mean([sp.speculative_verify(np.stack([z, z]), [d], p[None], [u], [0.1, 0.1], 0.8).kept[0] for u in grid(G)])
               for d in range(8))
    assert abs(rate - np.minimum(p, q).sum()) < 2e-3


def pin_equal_distributions_keep_everything(sp):
    rng = np.random.default_rng(11)
    V, gamma, T = 7, 3, 0.9
    z = rng.normal(size=(gamma + 1, V))
    q = scipy.special.softmax(z / T, axis=-1)
    for trial in range(50):
        drafts = rng.integers(0, V, gamma)
        u = rng.random(gamma)
        v = rng.random(gamma + 1)
        r = sp.speculative_verify(z, drafts, q[:gamma], u, v, T)
        assert r.accept_len == gamma
    # the token after gamma kept drafts follows q_gamma
    hist = np.zeros(V)
    G = 4000
    for v_last in grid(G):
        r = sp.speculative_verify(z, [0, 1, 2], q[:gamma], [0.3] * gamma, [0.5] * gamma + [v_last], T)
        assert r.next_token == r.tokens[gamma]
        hist[r.next_token] += 1.0 / G
    assert np.abs(hist - q[gamma]).max() < 2e-3


def pin_draft_without_target_mass(sp):
    V, T = 6, 1.0
    z = np.array([2.0, -800.0, 1.0, 0.5, 0.0, -1.0])   # token 1 has no mass under q
    q = scipy.special.softmax(z / T)
    p = np.zeros(V)
    p[1] = 1.0                                         # the draft model is certain of token 1
    hist = np.zeros(V)
    G = 4000
    for v in grid(G):
        r = sp.speculative_verify(np.stack([z, z]), [1], p[None], [1e-9], [v, 0.5], T)
        assert not r.kept[0] and r.accept_len == 0 and r.next_token == r.tokens[0]
        hist[r.next_token] += 1.0 / G
    assert hist[1] == 0.0
    assert np.abs(hist - q).max() < 2e-3               # q - p is positive everywhere but at the draft


def pin_stops_at_first_rejection(sp):
    rng = np.random.default_rng(5)
    V, gamma = 5, 4
    z = rng.normal(size=(gamma + 1, V))
    p = rng.dirichlet(np.ones(V), size=gamma)
    q = scipy.special.softmax(z, axis=-1)
    drafts = [int(np.argmax(q[i] / p[i])) for i in range(gamma)]   # q >= p there: kept for every u
    for i in range(gamma):
        assert q[i][drafts[i]] >= p[i][drafts[i]]
    for j in range(gamma):
        d = list(drafts)
        d[j] = int(np.argmin(q[j] / p[j]))                        # q < p there
        ratio = q[j][d[j]] / p[j][d[j]]
        assert ratio < 1.0
        r = sp.speculative_verify(z, d, p, [min(0.999, ratio + 1e-3)] * gamma, [0.4] * (gamma + 1), 1.0)
        assert r.accept_len == j and r.next_token == r.tokens[j]
        r = sp.speculative_verify(z, d, p, [max(0.0, ratio - 1e-3)] * gamma, [0.4] * (gamma + 1), 1.0)
        assert r.accept_len == gamma


def pin_inverse_cdf_by_hand(sp):
    w = np.array([0.0, 0.2, 0.0, 0.5, 0.3])
    assert sp.inverse_cdf(w, 0.0)[0] == 1
    assert sp.inverse_cdf(w, 0.19)[0] == 1
    assert sp.inverse_cdf(w, 0.2)[0] == 3      # the cumulative weight must exceed the target
    assert sp.inverse_cdf(w, 0.69)[0] == 3
    assert sp.inverse_cdf(w, 0.71)[0] == 4
    assert sp.inverse_cdf(w, 0.999999)[0] == 4
    assert sp.inverse_cdf(w * 10.0, 0.19)[0] == 1  # the scale of the weights does not matter
    k, gap = sp.inverse_cdf(w, 0.45)
    assert k == 3 and abs(gap - 0.25) < 1e-12


def pin_low_temperature_is_greedy(sp):
    """One-hot draft distributions and T -> 0: kept iff the draft is the argmax, the replacement is
    the argmax -- the greedy rule of the C oracle on the same logits."""
    import eegen
    from oracle import oracle as eo
    path = "/dev/shm/ee_sampling_pin_tiny.bin"
    eegen.write_model(path, eegen.TINY, seed=3)
    om = eo.Model(path, real="f64")
    V = eegen.TINY.vocab
    prompt = eegen.prompt_tokens(5, 24, V)
    s = om.session(128)
    s.prefill(prompt)
    greedy = om.ar_decode(prompt, 6)
    for corrupt in (None, 0, 2, 3):
        drafts = [int(t) for t in greedy[1:5]]
        if corrupt is not None:
            drafts[corrupt] = (drafts[corrupt] + 17) % V
        res = s.verify(drafts, exit_layers=[2], commit=False, want_logits=True)
        onehot = np.zeros((4, V))
        onehot[np.arange(4), drafts] = 1.0
        for head, (dlt, toks) in enumerate(((res.exit_accept_len[0], res.exit_tokens[0]), (res.accept_len, res.final_tokens))):
            r = sp.speculative_verify(res.logits[head], drafts, onehot, [0.5] * 4, [0.5] * 5, 1e-4)
            assert r.accept_len == dlt
            assert r.next_token == toks[dlt]
    s.close()
    om.close()
    os.unlink(path)


PINS = [pin_inverse_cdf_by_hand, pin_stops_at_first_rejection, pin_draft_without_target_mass, pin_equal_distributions_keep_everything,
        pin_keep_rate, pin_low_temperature_is_greedy, pin_output_distribution]


@pytest.mark.parametrize("pin", PINS, ids=[p.__name__ for p in PINS])
def test_pin(pin):
    pin(load())


def test_commit_of_a_sampled_pass_matches_brute_force():
    """Several sampled rounds through the oracle session (verify without commit, decision by the
    sampler, eo_commit_rows): the next pass's logits must equal those of the cache-free brute
    force over the whole committed sequence -- also when more drafts are kept than greedy would."""
    import eegen
    from oracle import oracle as eo
    sp = load()
    path = "/dev/shm/ee_sampling_commit_tiny.bin"
    eegen.write_model(path, eegen.TINY, seed=4)
    om = eo.Model(path, real="f64")
    V = eegen.TINY.vocab
    prompt = [int(t) for t in eegen.prompt_tokens(9, 20, V)]
    s = om.session(128)
    first = s.prefill(prompt)
    seq = prompt + [first]
    rng = np.random.default_rng(1)
    more_than_greedy = 0
    for rnd in range(6):
        drafts = [int(t) for t in rng.integers(0, V, 3)]
        p = rng.dirichlet(np.ones(V) * 0.05, size=3)
        res = s.verify(drafts, commit=False, want_logits=True)
        r = sp.speculative_verify(res.logits[0], drafts, p, rng.random(3) * 0.05, rng.random(4), 1.0)   # small u: drafts are mostly kept
        more_than_greedy += int(r.accept_len > res.accept_len)
        s.commit_rows(r.accept_len, r.next_token)
        seq += drafts[:r.accept_len] + [r.next_token]
        assert s.kv_len == len(seq) - 1 and s.pending == seq[-1]
    assert more_than_greedy > 0
    res = s.verify([1, 2, 3], commit=False, want_logits=True)
    brute = om.full_logits(seq + [1, 2, 3])
    assert np.abs(res.logits[0] - brute[len(seq) - 1:]).max() < 1e-9
    s.close()
    om.close()
    os.unlink(path)


# ---- planted mistakes (in a copy of the oracle's source, on the CPU)

MUTATIONS = {
    "residual_sign": ("return np.maximum(q - np.asarray(p, dtype=np.float64), 0.0)", "return np.maximum(np.asarray(p, dtype=np.float64) - q, 0.0)"),
    "residual_not_clipped": ("return np.maximum(q - np.asarray(p, dtype=np.float64), 0.0)", "return np.abs(q - np.asarray(p, dtype=np.float64))"),
    "replacement_from_q": ("w = residual_weights(q, p)\n", "w = q\n"),
    "keep_test_inverted_ratio": ("kept[i] = float(u[i]) * p[x] < q[x]", "kept[i] = float(u[i]) * q[x] < p[x]"),
    "keep_test_ignores_u": ("kept[i] = float(u[i]) * p[x] < q[x]", "kept[i] = p[x] <= q[x]"),
    "temperature_dropped": ("z = np.asarray(z, dtype=np.float64) / float(temperature)", "z = np.asarray(z, dtype=np.float64)"),
    "temperature_inverted": ("z = np.asarray(z, dtype=np.float64) / float(temperature)", "z = np.asarray(z, dtype=np.float64) * float(temperature)"),
    "cdf_not_strict": ('side="right"', 'side="left"'),
    "cdf_unscaled_target": ("target = float(v) * c[-1]", "target = float(v)"),
    "does_not_stop": ("while delta < gamma and kept[delta]:\n        delta += 1", "delta = int(kept.sum())"),
    "next_token_wrong_row": ("int(tokens[delta]))", "int(tokens[gamma]))"),
    "last_row_uses_residual": ("        else:\n            w = q\n        tokens[i]", "        else:\n            w = residual_weights(q, draft_probs[gamma - 1])\n        tokens[i]"),
    "wrong_rows_draft_distribution": ("p = np.asarray(draft_probs[i], dtype=np.float64)", "p = np.asarray(draft_probs[0], dtype=np.float64)"),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation {name}: source text not found exactly once"
    path = tmp_path / "sampling_mutant.py"
    path.write_text(text.replace(old, new))
    mod = load(str(path), "sampling_mutant_" + name)
    caught = []
    for pin in PINS:
        try:
            pin(mod)
        except AssertionError:
            caught.append(pin.__name__)
        except Exception as exc:  # a mutant may also crash a pin: that counts
            caught.append(pin.__name__ + ":" + type(exc).__name__)
        if caught:
            break
    assert caught, f"no pin notices the planted mistake {name}"
