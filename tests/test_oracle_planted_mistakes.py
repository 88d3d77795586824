"""The pins must notice a plausible mistake anywhere in the oracle.  Each case plants ONE mistake in a
copy of the oracle's source (a dropped term, a wrong sign or index, a transposed operand, an off-by-one,
a swapped comparison), builds that copy, and runs the pin suite against it in a child process: at least
one pin has to fail.  Everything here runs on the CPU; the real oracle is never touched."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "mrp_oracle.c")

# (name, text in the oracle, what the mistake turns it into)
MISTAKES = [
    ("argmax keeps the last of equal maxima", "if (r[v] > m) { m = r[v]; am = v; }", "if (r[v] >= m) { m = r[v]; am = v; }"),
    ("confidence is not the top-1 probability", "conf[i] = 1.0 / s;", "conf[i] = 1.0 / (s + 1.0);"),
    ("log-sum-exp drops the maximum", "lse[i] = m + log(s);", "lse[i] = log(s);"),
    ("concatenation order [e ; h]", "for (int j = 0; j < d; ++j) x[j] = hrun[(size_t)i * d + j];\n            for (int j = 0; j < d; ++j) x[d + j] = bf16_bits_to_double(e[j]);",
     "for (int j = 0; j < d; ++j) x[d + j] = hrun[(size_t)i * d + j];\n            for (int j = 0; j < d; ++j) x[j] = bf16_bits_to_double(e[j]);"),
    ("SiLU with the wrong sign in the sigmoid", "s[j] = a * (1.0 / (1.0 + exp(-a)));", "s[j] = a * (1.0 / (1.0 + exp(a)));"),
    ("W2 read transposed", "const uint16_t *w = W2 + (size_t)j * d;\n                double acc = 0.0;\n                for (int k = 0; k < d; ++k) acc += bf16_bits_to_double(w[k]) * s[k];",
     "double acc = 0.0;\n                for (int k = 0; k < d; ++k) acc += bf16_bits_to_double(W2[(size_t)k * d + j]) * s[k];"),
    ("RMSNorm without the mean", "const double inv = 1.0 / sqrt(ss / d + c->rms_eps);", "const double inv = 1.0 / sqrt(ss + c->rms_eps);"),
    ("RMSNorm without epsilon", "const double inv = 1.0 / sqrt(ss / d + c->rms_eps);", "const double inv = 1.0 / sqrt(ss / d);"),
    ("gain dropped", "const double yd = u[j] * inv * bf16_bits_to_double(gamma[j]);", "const double yd = u[j] * inv;"),
    ("hidden carry dropped", "if (c->carry_hidden) hrun[(size_t)i * d + j] += u[j];", "if (c->carry_hidden) hrun[(size_t)i * d + j] += 0.0;"),
    ("logit update overwrites instead of adding", "z[(size_t)i * V + v] += acc;", "z[(size_t)i * V + v] = acc;"),
    ("LM head indexed by the wrong row", "const double *yi = y + (size_t)i * d;", "const double *yi = y + (size_t)(i ? i - 1 : 0) * d;"),
    ("tie between positions goes to the higher one", "    return a < b;\n}\n\nint orc_max_accept_cap", "    return a > b;\n}\n\nint orc_max_accept_cap"),
    ("threshold compared with >=", "if (cf[cand[a]] > c->tau) sel[ns++] = cand[a];", "if (cf[cand[a]] >= c->tau) sel[ns++] = cand[a];"),
    ("cap floor(0.7 n) without its lower bound", "    if (m < 5) m = 5;\n", "    if (m < 1) m = 1;\n"),
    ("forced minimum off by one", "ns = c->r_min < nc ? c->r_min : nc;", "ns = c->r_min + 1 < nc ? c->r_min + 1 : nc;"),
    ("draft is the last selected, not the most confident", "const int top = sel[0];", "const int top = sel[ns - 1];"),
    ("remask reaches the current state's reveals", "if (ra < 0 || ra > state - 1) continue;", "if (ra < 0 || ra > state) continue;"),
    ("remask ignores the protected position", "if (protect_pos && protect_pos[b] == p) continue;", "if (protect_pos && protect_pos[b] == -7) continue;"),
    ("remask compared with <=", "if (conf[i] < tau_remask) { masked[i] = 1;", "if (conf[i] <= tau_remask) { masked[i] = 1;"),
    ("commit counts revealed rows as masked", "if (masked[i]) ++n;", "if (masked[i] || revealed_at[i] == -2) ++n;"),
    ("accept length counts matches after a reject", "else { open = 0; correction_tok[b] = vj; }\n            }\n        }\n        accept_len[b] = alen;\n    }\n}\n\n/* Joint",
     "else { correction_tok[b] = vj; }\n            }\n        }\n        accept_len[b] = alen;\n    }\n}\n\n/* Joint"),
    ("joint verification reads candidate j + 1", "const float *r = verify + (((size_t)b * (K + 1) + j) * L + pos) * V;",
     "const float *r = verify + (((size_t)b * (K + 1) + j + 1) * L + pos) * V;"),
    ("candidate k holds drafts 0..k", "for (int j = 0; j < k; ++j) {\n                const int pos = draft_pos[(size_t)b * K + j];",
     "for (int j = 0; j <= k && j < K; ++j) {\n                const int pos = draft_pos[(size_t)b * K + j];"),
    ("KL with teacher and student swapped", "kl += exp(lp[v]) * (lp[v] - lq[v]);", "kl += exp(lq[v]) * (lq[v] - lp[v]);"),
    ("KL gradient with the wrong sign", "scale * (exp(lq[v]) - exp(lp[v]));", "scale * (exp(lp[v]) - exp(lq[v]));"),
    ("RMS without the 1/N", "(u >= t) ? sqrt(acc / (double)N) : 0.0;", "(u >= t) ? sqrt(acc) : 0.0;"),
    ("bf16 rounding truncates", "double q = nearbyint(m * 256.0);", "double q = trunc(m * 256.0);"),
    ("bf16 keeps 9 significant bits", "double q = nearbyint(m * 256.0);    /* default mode: ties to even */\n    return ldexp(q / 256.0, e);",
     "double q = nearbyint(m * 512.0);\n    return ldexp(q / 512.0, e);"),
    ("rotary angle with the wrong sign", "x[j] = a * cs - b * sn;\n        x[j + half] = b * cs + a * sn;", "x[j] = a * cs + b * sn;\n        x[j + half] = b * cs - a * sn;"),
    ("rotary frequencies over hd / 2", "const double ang = pos * pow(theta, -2.0 * (double)j / (double)hd);", "const double ang = pos * pow(theta, -(double)j / (double)hd);"),
    ("query heads mapped to the wrong kv head", "const int g = h / rep;", "const int g = h % nkv;"),
    ("attention scores not scaled", "sc[tt] = acc / sqrt((double)hd);", "sc[tt] = acc;"),
    ("block positions rotated without the prefix offset", "for (int h = 0; h < nh; ++h) orc_rope(r + h * hd, hd, (double)(P + i), t->rope_theta);",
     "for (int h = 0; h < nh; ++h) orc_rope(r + h * hd, hd, (double)i, t->rope_theta);"),
    ("attention sees one prefix position too few", "for (int tt = 0; tt < T; ++tt) {\n                double acc = 0.0;", "for (int tt = (P > 0); tt < T; ++tt) {\n                double acc = 0.0;"),
    ("values read from the key block", "const double *v = qkv + (size_t)(tt - P) * (qd + 2 * kvd) + qd + kvd + g * hd;", "const double *v = qkv + (size_t)(tt - P) * (qd + 2 * kvd) + qd + g * hd;"),
    ("attention residual dropped", "A[(size_t)i * d + j] = U[(size_t)i * d + j] + tmp[j];", "A[(size_t)i * d + j] = tmp[j];"),
    ("gate and up swapped", "act[j] = tmp[j] / (1.0 + exp(-tmp[j])) * tmp[ff + j];", "act[j] = tmp[ff + j] / (1.0 + exp(-tmp[ff + j])) * tmp[j];"),
    ("MLP residual dropped", "U[(size_t)i * d + j] = a[j] + n[j];", "U[(size_t)i * d + j] = n[j];"),
    ("second norm uses the first gain", "rmsnorm_gain(a, g2, d, eps, n);", "rmsnorm_gain(a, g1, d, eps, n);"),
    ("only the first layer runs", "for (int l = 0; l < t->D; ++l)\n            orc_tlayer(", "for (int l = 0; l < 1; ++l)\n            orc_tlayer("),
    ("state index of head k off by one", "const int state = c->state_offset + k;", "const int state = c->state_offset + k - 1;"),
    ("remask runs before the reveal", "        if (c->head_reveal) {\n            orc_reveal(c, state,", "        if (0) {\n            orc_reveal(c, state,"),
    ("recorded token taken from state 0", "if (revealed_at[i] == state) x_tok[i] = tok[(size_t)k * M + i];", "if (revealed_at[i] == state) x_tok[i] = tok[i];"),
    ("heads all use the first head's weights", "orc_head_mlp(c, W1[k - 1], W2[k - 1], gamma[k - 1], E, cond_tok, hrun, NULL, y);", "orc_head_mlp(c, W1[0], W2[0], gamma[0], E, cond_tok, hrun, NULL, y);"),
    ("token probability without the log-sum-exp", "exp(z[(size_t)i * V + t] - lse[i]) : 0.0;", "exp(z[(size_t)i * V + t]) : 0.0;"),
    ("conditioning token not updated by a reveal", "        cond_tok[b] = tok[(size_t)b * L + top];\n", "        (void)cond_tok;\n"),
    ("reference line includes state 0", "for (int t = (r == 0 ? 1 : 0); t + r < S; ++t)", "for (int t = 0; t + r < S; ++t)"),
]


def _build(tmp, tag, text):
    c = os.path.join(tmp, f"{tag}.c")
    with open(c, "w") as f:
        f.write(text)
    so = os.path.join(tmp, f"lib{tag}.so")
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-fPIC", "-shared", c, "-o", so, "-lm"])
    return so


def _run_pins(lib):
    env = dict(os.environ, MRP_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=900)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Builds every mutant and runs the pin suite against each, a few at a time (one child process per mutant)."""
    from concurrent.futures import ThreadPoolExecutor
    tmp = str(tmp_path_factory.mktemp("mutants"))
    src = open(SRC).read()
    for name, old, new in MISTAKES:
        assert src.count(old) == 1, f"the text to replace must occur exactly once in the oracle ({name}): {old!r}"
    jobs = {"unchanged": src}
    jobs.update({str(i): src.replace(old, new) for i, (_, old, new) in enumerate(MISTAKES)})

    def one(item):
        tag, text = item
        return tag, _run_pins(_build(tmp, "m" + tag, text))

    with ThreadPoolExecutor(max_workers=4) as ex:
        return dict(ex.map(one, jobs.items()))


@pytest.mark.parametrize("idx", range(len(MISTAKES)), ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(outcomes, idx):
    r = outcomes[str(idx)]
    assert r.returncode != 0 and " failed" in r.stdout, f"no pin noticed: {MISTAKES[idx][0]}\n{r.stdout[-800:]}"


def test_the_unchanged_copy_passes(outcomes):
    """The same machinery on an unchanged copy: every pin passes (so a failure above is the mistake's)."""
    r = outcomes["unchanged"]
    assert r.returncode == 0, r.stdout[-800:]
