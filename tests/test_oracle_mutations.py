"""Each plausible mistake, planted in a copy of the oracle's source (on the
CPU, in a temporary folder), must make at least one pin in
tests/test_oracle_pins.py fail; the untouched copy must pass."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ee_oracle.c")

MUTATIONS = {
    "control": None,
    "rope_sign": ("p[i] = a * c - b * s;", "p[i] = a * c + b * s;"),
    "rope_frequency": ("-2.0 * (double)i / (double)hd", "-1.0 * (double)i / (double)hd"),
    "rope_not_applied_to_k": ("rope_row(k + (size_t)i * d, H, hd, P + i, (double)m->c.rope_base);", ";"),
    "score_scale": ("const real scale = (real)(1.0 / sqrt((double)hd));\n    size_t Md",
                    "const real scale = (real)(1.0 / (double)hd);\n    size_t Md"),
    "causal_excludes_self": ("int n_pos = P + i + 1;", "int n_pos = P + i > 0 ? P + i : 1;"),
    "attn_residual_dropped": ("linear(w->wo, d, d, att, M, o);\n        for (size_t i = 0; i < Md; ++i)\n            h[i] += o[i];",
                              "linear(w->wo, d, d, att, M, o);\n        for (size_t i = 0; i < Md; ++i)\n            h[i] = o[i];"),
    "swiglu_operands_swapped": ("gate[i] = silu(gate[i]) * up[i];\n        linear(w->wd, d, F, gate, M, o);",
                                "gate[i] = silu(up[i]) * gate[i];\n        linear(w->wd, d, F, gate, M, o);"),
    "q_k_weights_swapped": ("linear(w->wq, d, d, x, M, q);\n        linear(w->wk, d, d, x, M, k);\n        linear(w->wv, d, d, x, M, v);\n        #pragma",
                            None),  # filled below (needs exact text)
    "rms_mean_dropped": ("ss / (real)d + eps", "ss + eps"),
    "norm_gain_dropped": ("out[(size_t)m * d + k] = xr[k] * inv * bf16_val(g[k]);", "out[(size_t)m * d + k] = xr[k] * inv;"),
    "argmax_highest_index": ("if (z[i] > z[best]) best = i;\n    return best;", "if (z[i] >= z[best]) best = i;\n    return best;"),
    "accept_off_by_one": ("while (d < gamma && drafts[d] == a[d])", "while (d < gamma && drafts[d] == a[d + 1])"),
    "next_token_wrong_row": ("if (next) *next = a[d];", "if (next) *next = a[0];"),
    "commit_off_by_one": ("s->kv_len = P + out->accept_len + 1;", "s->kv_len = P + out->accept_len;"),
    "exit_uses_final_gain": ("hr.gain[e] = exit_gain(m, exit_layers[e]);", "hr.gain[e] = m->g_final;"),
    "exit_one_layer_late": ("if (hr->layer[e] != l) continue;", "if (hr->layer[e] != l - 1 && !(hr->layer[e] == L && l == L)) continue;"),
    "kv_written_one_row_off": ("memcpy(vc + (size_t)(P + i) * d, v + (size_t)i * d", "memcpy(vc + (size_t)(P + (i > 0 ? i - 1 : 0)) * d, v + (size_t)i * d"),
    "v_not_cached_value": ("out[e] += sc[t] * vt[e];", "out[e] += sc[t] * vt[(e + 1) % hd];"),
    "softmax_no_normalise": ("for (int i = 0; i < n; ++i)\n        s[i] /= sum;", "(void)sum;"),
    "down_proj_transposed_shape": ("linear(w->wd, d, F, gate, M, o);\n        for (size_t i = 0; i < Md; ++i)\n            h[i] += o[i];\n        if (tr",
                                   None),
    "embedding_row_stride": ("h[(size_t)i * d + kx] = bf16_val(m->emb[(size_t)tok[i] * d + kx]);",
                             "h[(size_t)i * d + kx] = bf16_val(m->emb[(size_t)tok[i] + (size_t)kx * m->c.vocab]);"),
    "confidence_not_normalised": ("real p = (real)exp((double)(z[i] - mx)) / sum;", "real p = (real)exp((double)(z[i] - mx));"),
    "confidence_of_wrong_head": ("double *conf = e < n_exits ? out->exit_conf[e] : out->final_conf;",
                                 None),
}
MUTATIONS["adapter_residual_dropped"] = ("a[(size_t)i * d + c] = h[(size_t)i * d + c] + a[(size_t)i * d + c] + b;",
                                        "a[(size_t)i * d + c] = a[(size_t)i * d + c] + b;")
MUTATIONS["adapter_down_bias_dropped"] = ("silu(t[(size_t)i * A + r] + bf16_val(m->ad_bdown[slot][r]))", "silu(t[(size_t)i * A + r])")
MUTATIONS["adapter_only_first_up_bias"] = ("for (int j = 0; j < m->n_ad; ++j)\n                b +=", "for (int j = 0; j < 1; ++j)\n                b +=")
MUTATIONS["adapter_no_activation"] = ("t[(size_t)i * A + r] = silu(t[(size_t)i * A + r] + bf16_val(m->ad_bdown[slot][r]));",
                                     "t[(size_t)i * A + r] = t[(size_t)i * A + r] + bf16_val(m->ad_bdown[slot][r]);")
MUTATIONS["adapter_on_final_head"] = ("const int slot = l < L ? exit_slot(m, l) : -1;", "const int slot = l < L ? exit_slot(m, l) : 0;")
MUTATIONS["adapter_of_wrong_exit"] = ("adapter_rows(m, slot, h, M, o);\n                rmsnorm(o, hr->gain[e]", "adapter_rows(m, 0, h, M, o);\n                rmsnorm(o, hr->gain[e]")
MUTATIONS["q_k_weights_swapped"] = ("linear(w->wq, d, d, x, M, q);\n        linear(w->wk, d, d, x, M, k);",
                                    "linear(w->wk, d, d, x, M, q);\n        linear(w->wq, d, d, x, M, k);")
MUTATIONS["confidence_of_wrong_head"] = ("conf[i] = max_softmax(hr.logits[e] + (size_t)i * V, V);",
                                         "conf[i] = max_softmax(hr.logits[n_exits] + (size_t)i * V, V);")
MUTATIONS["down_proj_transposed_shape"] = ("y[(size_t)m * N + n] = dot_w(W + (size_t)n * K, x + (size_t)m * K, K);",
                                           "y[(size_t)m * N + n] = dot_w(W + (size_t)n * K, x + (size_t)m * K, K - 1);")


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    src = open(SRC).read()
    mut = MUTATIONS[name]
    if mut is not None:
        old, new = mut
        assert src.count(old) >= 1, f"mutation anchor for {name} not found"
        # mutate the first (cached-path) occurrence only
        src = src.replace(old, new, 1)
    c = tmp_path / "ee_oracle.c"
    c.write_text(src)
    for out, extra in (("liboracle32.so", []), ("liboracle64.so", ["-DEO_REAL=double"])):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ftree-vectorize", "-shared", "-fPIC",
                               f"-I{os.path.join(ROOT, 'oracle')}", *extra, "-o", str(tmp_path / out),
                               str(c), "-lm"])
    env = dict(os.environ, EE_ORACLE_LIBDIR=str(tmp_path))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    if mut is None:
        assert r.returncode == 0, r.stdout[-2000:]
    else:
        assert r.returncode != 0, f"planted mistake '{name}' passed every pin"
