"""Mutation check of the oracle's pins (test infrastructure, CPU only).

Each entry below plants one plausible mistake -- a dropped term, a wrong sign or index, a transposed layout --
in a temporary copy of asyncspade_oracle.c, rebuilds that copy and runs the CPU test-suite against it.  A pin
set that is worth its name fails on every planted mistake; `python -m oracle.mutation_check` prints which test
caught which one.  Nothing here touches the GPU path or the library's own copy of the oracle.

Entries marked equivalent change the text but not the function (the reason is given); they must NOT be caught.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)

# (what is planted, text in the oracle source, its replacement[, why the mutant is equivalent])
MUTANTS = [
 ("ridge: eps dropped from the Gram diagonal", "G[i * k + j] = s + (i == j ? eps : 0.0);", "G[i * k + j] = s;"),
 ("ridge: rhs uses R_j.R_0 instead of R_i.T", "for (int d = 0; d < D; ++d) s += R[i * D + d] * T[d];\n    b[i] = s;", "for (int d = 0; d < D; ++d) s += R[i * D + d] * R[d];\n    b[i] = s;"),
 ("predict: window read oldest-first (no reversal)", "R[(i - 1) * D + d] = bf16_to_f64(win[(size_t)(W - i) * D + d]);\n    /* shifted", "R[(i - 1) * D + d] = bf16_to_f64(win[(size_t)(i - 1) * D + d]);\n    /* shifted"),
 ("predict: no shift (weights applied to the predecessors)", "for (int i = 0; i < k; ++i) c += w[i] * S[i * D + d];\n        acc[d] += c;\n      }\n    }\n    for (int d = 0; d < D; ++d) q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)W);\n    free(R); free(S); free(T); free(om); free(w); free(acc);\n  }\n  return fail ? -1 : 0;\n}\n\n/*\n * Predictor with a single", "for (int i = 0; i < k; ++i) c += w[i] * R[i * D + d];\n        acc[d] += c;\n      }\n    }\n    for (int d = 0; d < D; ++d) q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)W);\n    free(R); free(S); free(T); free(om); free(w); free(acc);\n  }\n  return fail ? -1 : 0;\n}\n\n/*\n * Predictor with a single"),
 ("predict: softmax sign flipped", "{ w[i] = exp(beta * om[i] - mx); z += w[i]; }\n      for (int i = 0; i < k; ++i) w[i] /= z;\n      if (weights_out) {\n        double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;\n        for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;\n      }\n      /* candidate", "{ w[i] = exp(-(beta * om[i] - mx)); z += w[i]; }\n      for (int i = 0; i < k; ++i) w[i] /= z;\n      if (weights_out) {\n        double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;\n        for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;\n      }\n      /* candidate"),
 ("predict: no softmax (raw omega as weights)", "for (int i = 0; i < k; ++i) w[i] /= z;\n      if (weights_out) {\n        double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;\n        for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;\n      }\n      /* candidate", "for (int i = 0; i < k; ++i) w[i] = om[i];\n      if (weights_out) {\n        double* wo = weights_out + ((size_t)bh * W + (k - 1)) * W;\n        for (int i = 0; i < W; ++i) wo[i] = i < k ? w[i] : 0.0;\n      }\n      /* candidate"),
 ("predict: mean divides by W+1", "q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)W);\n    free(R); free(S); free(T); free(om); free(w); free(acc);\n  }\n  return fail ? -1 : 0;\n}\n\n/*\n * Predictor with a single", "q_hat[(size_t)bh * D + d] = (float)(acc[d] / (double)(W + 1));\n    free(R); free(S); free(T); free(om); free(w); free(acc);\n  }\n  return fail ? -1 : 0;\n}\n\n/*\n * Predictor with a single"),
 ("predict: only the largest window (no mean over k)", "    for (int k = 1; k <= W; ++k) {\n      if (aso_ridge_weights(k, D, R, T, eps, om) != 0) {", "    for (int k = W; k <= W; ++k) {\n      if (aso_ridge_weights(k, D, R, T, eps, om) != 0) {"),
 ("single-solve: solves per window size instead of once", "    if (aso_ridge_weights(W, D, R, T, eps, om) != 0) {", "    if (aso_ridge_weights(W > 1 ? W - 1 : W, D, R, T, eps, om) != 0) {"),
 ("score: min instead of max over the group", "else if (s > best) best = s;", "else if (s < best) best = s;"),
 ("score: query head index ignores the group offset", "const float* q = q_hat + ((size_t)b * Hq + (size_t)j * G + g) * D;\n          double s = 0.0;\n          for (int d = 0; d < D; ++d) s += (double)q[d] * bf16_to_f64(kr[d]);\n          if (g == 0)", "const float* q = q_hat + ((size_t)b * Hq + (size_t)g * Hkv + j) * D;\n          double s = 0.0;\n          for (int d = 0; d < D; ++d) s += (double)q[d] * bf16_to_f64(kr[d]);\n          if (g == 0)"),
 ("paging: slot and page swapped", "int slot = n % P;\n  return pool + ((page * Hkv + j) * P + slot) * (int64_t)D;", "int slot = n % P;\n  return pool + ((page * P + slot) * Hkv + j) * (int64_t)D;"),
 ("score: -0 not canonicalised", "f = f + 0.0f;                     /* -0 -> +0 */", "/* nothing */",
  "the fp64 sum starts at +0.0, and +0 + -0 = +0: the oracle cannot produce -0, the line only documents the convention"),
 ("topk: ties to the highest index", "return (a->n > b->n) - (a->n < b->n);", "return (a->n < b->n) - (a->n > b->n);"),
 ("topk: ascending scores", "if (a->s > b->s) return -1;\n    if (a->s < b->s) return 1;", "if (a->s > b->s) return 1;\n    if (a->s < b->s) return -1;"),
 ("topk: output not sorted by index", "qsort(out, keep, sizeof(int32_t), int_cmp);", ""),
 ("topk: keeps C even when N < C", "int keep = N < C ? N : C;\n      for (int i = 0; i < keep; ++i) out[i] = c[i].n;", "int keep = C; for (int i = N; i < C; ++i) { }\n      for (int i = 0; i < (N < C ? N : C); ++i) out[i] = c[i].n;"),
 ("attn: scale dropped", "logit[i] = s * sm_scale;", "logit[i] = s;"),
 ("attn: V rows from the K pool", "token_ptr(v_pool, block_table, max_pages, Hkv, P, D, b, j, toks[i]);\n        for (int d = 0; d < D; ++d) acc[d] += p", "token_ptr(k_pool, block_table, max_pages, Hkv, P, D, b, j, toks[i]);\n        for (int d = 0; d < D; ++d) acc[d] += p"),
 ("attn: unnormalised output", "o[d] = f64_to_bf16(acc[d] / z);", "o[d] = f64_to_bf16(acc[d]);"),
 ("attn: lse without the max", "lse[(size_t)b * Hq + h] = (float)(m + log(z));", "lse[(size_t)b * Hq + h] = (float)(log(z));"),
 ("attn: tail starts one token late", "for (int n = tail0; n < N; ++n) toks[cnt + (n - tail0)] = n;", "for (int n = tail0; n < N; ++n) toks[cnt + (n - tail0)] = n + 1 < N ? n + 1 : n;"),
 ("attn: kv head of query head h = h % Hkv", "int j = h / G;\n      int N = ctx_lens[b];\n      int cnt", "int j = h % Hkv;\n      int N = ctx_lens[b];\n      int cnt"),
 ("softmax-sum: scale dropped", "logit[(size_t)g * N + n] = scale * s;\n          if (scale * s > m) m = scale * s;", "logit[(size_t)g * N + n] = s;\n          if (s > m) m = s;"),
 ("softmax-sum: normaliser shared across heads", "for (int g = 0; g < G; ++g) s += exp(logit[(size_t)g * N + n] - lse[g]);", "for (int g = 0; g < G; ++g) s += exp(logit[(size_t)g * N + n] - lse[0]);"),
 ("overlap: denominator is the smaller set", "int den = na > nb ? na : nb;", "int den = na < nb ? na : nb;"),
 ("append: length not bumped", "ctx_lens[b] = n + 1;", "ctx_lens[b] = n;"),
 ("push: newest entry not replaced by the current query", "for (int d = 0; d < D; ++d) win[(size_t)(W - 1) * D + d] = cur[d];", ""),
 ("gather: rows in page-major order of the source", "int64_t off = ((((int64_t)b * Cp + i / P) * Hkv + j) * P + i % P) * (int64_t)D;", "int64_t off = ((((int64_t)b * Cp + i / P) * Hkv + j) * P + (P - 1 - i % P)) * (int64_t)D;"),
 ("bf16 rounding: truncation instead of nearest-even", "double q = nearbyint(ldexp(fabs(d), -lsb));", "double q = floor(ldexp(fabs(d), -lsb));"),
]


def _run_one(entry, extra_ignores=()):
    name, old, new = entry[:3]
    src = open(os.path.join(_HERE, "asyncspade_oracle.c")).read()
    if src.count(old) < 1:
        return name, None, "pattern not found in the oracle source"
    tmp = tempfile.mkdtemp(prefix="oracle_mutant_")
    try:
        shutil.copytree(_HERE, os.path.join(tmp, "oracle"), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
        shutil.copytree(os.path.join(_ROOT, "tests"), os.path.join(tmp, "tests"),
                        ignore=shutil.ignore_patterns("__pycache__"))
        for d in ("paper_2510_07486_amd", "include"):          # read-only: input generators, header
            os.symlink(os.path.join(_ROOT, d), os.path.join(tmp, d))
        with open(os.path.join(tmp, "oracle", "asyncspade_oracle.c"), "w") as f:
            f.write(src.replace(old, new, 1))
        cmd = [sys.executable, "-m", "pytest", "tests", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
               "--ignore", "tests/test_abi_host.py", "--ignore", "tests/test_oracle_mutation_check.py"]
        for ig in extra_ignores:
            cmd += ["--ignore", ig]
        env = dict(os.environ, OMP_NUM_THREADS="2")
        r = subprocess.run(cmd, cwd=tmp, capture_output=True, text=True, timeout=900, env=env)
        first = [ln for ln in r.stdout.splitlines() if ln.startswith(("FAILED", "ERROR"))]
        return name, r.returncode != 0, (first[0] if first else r.stdout.strip().splitlines()[-1])
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def run(jobs: int = 4, only=()):
    """Returns [(name, caught, first failing test or summary line, equivalent)] for every mutant."""
    todo = [m for m in MUTANTS if not only or any(o in m[0] for o in only)]
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        out = list(ex.map(_run_one, todo))
    return [(n, c, msg, len(m) > 3) for (n, c, msg), m in zip(out, todo)]


if __name__ == "__main__":
    res = run(only=sys.argv[1:])
    for name, caught, msg, equiv in res:
        tag = "caught " if caught else ("equiv. " if equiv else "MISSED ")
        print(tag, name, "|", msg[:120])
    print(sum(1 for _, c, _, _ in res if c), "of", len(res), "caught;",
          sum(1 for _, c, _, e in res if not c and not e), "missed")
