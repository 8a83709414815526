"""CPU hygiene of the oracle, the root of every parity claim.

1. Its source, built with AddressSanitizer and UndefinedBehaviorSanitizer, walks every function
   over ragged shapes without a report (tests/sanitize_oracle.c).
2. Mutation check: single planted mistakes in a copy of the source (a wrong sign, a dropped term,
   a transposed index, a broken tie-break ...) must each fail the pins of tests/test_oracle_pins.py;
   the unmutated copy passes them.  A pin suite that lets a mutant through would not bite.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as obuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")


def test_oracle_source_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = obuild.build_sanitized(os.path.join(ROOT, "tests", "sanitize_oracle.c"), str(tmp_path / "sanitize_oracle"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    assert r.returncode == 0, r.stderr[-3000:]
    assert "sanitized oracle walk: ok" in r.stdout


# (what the mutation is, the exact source text it replaces, the replacement)
MUTANTS = [
    ("tie-break prefers the higher index", "logits[e] > logits[best]) best = e;", "logits[e] >= logits[best]) best = e;"),
    ("gates not renormalised", "gate[j] = probs[idx[j]] / sel;", "gate[j] = probs[idx[j]];"),
    ("softmax without the maximum subtracted", "probs[e] = exp(logits[e] - mx);", "probs[e] = exp(logits[e]);"),
    ("router bias dropped", "if (rb) acc += (double)rb[e];", ""),
    ("SiLU sign", "return z / (1.0 + exp(-z));", "return z / (1.0 + exp(z));"),
    ("SiLU on the up branch", "g[f] = silu(g[f]) * u[f];", "g[f] = g[f] * silu(u[f]);"),
    ("unstable sort (descending pairs)", "for (int p = 0; p < P; ++p) {\n        int32_t s = next[topk_idx[p]]++;",
     "for (int p = P - 1; p >= 0; --p) {\n        int32_t s = next[topk_idx[p]]++;"),
    ("shared base indexed per expert", "size_t eb = (L->flags & FLAG_SHARED_BASE) ? 0 : (size_t)e;", "size_t eb = (size_t)e;"),
    ("low-rank term overwrites the base term", "n_out, L->r, tmp_r, L->dtype, out, have);", "n_out, L->r, tmp_r, L->dtype, out, 0);"),
    ("down projection uses the up factors' rank input", "expert_matvec(L, e, L->w_down, L->rd, L->ld, L->d, L->F, g, out, tr);",
     "expert_matvec(L, e, L->w_down, L->rd, L->ld, L->d, L->F, u, out, tr);"),
    ("combine takes the gate of slot 0", "acc += topk_gate[(size_t)t * k + j] * y_perm[s * d + i];",
     "acc += topk_gate[(size_t)t * k] * y_perm[s * d + i];"),
    ("residual dropped from the layer", "for (int i = 0; i < d; ++i) yt[i] += xv[i];", ""),
    ("experts mixed without their gates", "yt[i] += gate[j] * out[i];", "yt[i] += out[i] / k;"),
    ("H_norm denominator", "(double)(H / 2) / ((double)B * K * (T - 1))", "(double)(H / 2) / ((double)B * K * T)"),
    ("Eq. 5 without the floor", "(double)(H / 2) / ((double)B * K * (T - 1))", "((double)H / 2.0) / ((double)B * K * (T - 1))"),
    ("L_norm denominator", "double Ln = L / ((double)B * T);", "double Ln = L / ((double)B * (T - 1));"),
    ("replacements look at the first slot only", "for (int j = 0; j < K; ++j) {\n                    a0 |=", "for (int j = 0; j < 1; ++j) {\n                    a0 |="),
    ("offload loads count the whole set", "uint64_t in = cur & ~prev;", "uint64_t in = cur;"),
    ("Delta Uniform pools the layers", "for (int e = 0; e < E; ++e) cnt[e] = 0;\n        for (int t = 0; t < T; ++t)",
     "if (l == 0) for (int e = 0; e < E; ++e) cnt[e] = 0;\n        for (int t = 0; t < T; ++t)"),
    ("Delta Uniform against 1/K", "- 1.0 / (double)E;", "- 1.0 / (double)K;"),
    ("Delta Uniform sums squares", "delta += dev < 0 ? -dev : dev;", "delta += dev * dev;"),
    ("stack applies the layers in reverse", "oracle_layer L = layers[l];", "oracle_layer L = layers[n_layers - 1 - l];"),
]


def _pins_pass(lib_path):
    env = dict(os.environ, MOE_ORACLE_LIB=lib_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    return r.returncode == 0, r.stdout[-800:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    text = open(SRC).read()
    jobs = [("control: the unmutated source", text)]
    for what, old, new in MUTANTS:
        assert text.count(old) == 1, f"mutation site for {what!r} not found exactly once"
        jobs.append((what, text.replace(old, new)))

    def run(job):
        i, (what, src_text) = job
        c = tmp_path / f"mutant_{i}.c"
        c.write_text(src_text)
        lib = obuild.build(src=str(c), out=str(tmp_path / f"mutant_{i}.so"))
        return what, _pins_pass(lib)

    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(run, enumerate(jobs)))
    what, (ok, tail) = results[0]
    assert ok, f"the unmutated copy must pass its pins:\n{tail}"
    survivors = [what for what, (ok, _) in results[1:] if ok]
    assert not survivors, f"planted mistakes that no pin caught: {survivors}"
