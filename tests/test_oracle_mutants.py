"""Do the oracle's pins notice a mistake?  Each case below plants ONE plausible mistake in a copy of the oracle's
C source (a swapped operand, a dropped term, a wrong index, a reversed tie-break ...), builds it, and runs the
oracle pin tests against that build in a child process: the pins must fail.  Everything here runs on the CPU."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")

# (name, source file, text to replace, replacement, pin files that must catch it)
MUTANTS = [
    ("ratio inverted", "pe_oracle.c", "return sqrt(sv) / sqrt(sk);", "return sqrt(sk) / sqrt(sv);", "scores"),
    ("norms not rooted", "pe_oracle.c", "return sqrt(sv) / sqrt(sk);", "return sv / sk;", "scores"),
    ("last coordinate of K dropped", "pe_oracle.c",
     "for (int d = 0; d < D; ++d) sk += (double)k_row[d] * (double)k_row[d];",
     "for (int d = 0; d + 1 < D; ++d) sk += (double)k_row[d] * (double)k_row[d];", "scores"),
    ("zero V norm not special", "pe_oracle.c", "if (sv == 0.0) return 0.0;", "", "scores"),
    ("page sum not divided by B", "pe_oracle.c", "out[j] = (float)(sum / (double)B);", "out[j] = (float)sum;", "scores"),
    ("page found without the table", "pe_oracle.c", "const int64_t page = (int64_t)bt[j] * B * D;",
     "const int64_t page = (int64_t)j * B * D;", "scores"),
    ("partial page scored", "pe_oracle.c", "const int nfull = seq_lens[s] / B;",
     "const int nfull = (seq_lens[s] + B - 1) / B;", "scores"),
    ("prefill tie-break reversed", "pe_oracle.c", "return (x->idx > y->idx) - (x->idx < y->idx);\n}\n\nstatic int cmp_i32",
     "return (x->idx < y->idx) - (x->idx > y->idx);\n}\n\nstatic int cmp_i32", "prune"),
    ("prefill keeps the lowest scores", "pe_oracle.c", "kept[i] = tok[E + i].idx;", "kept[i] = tok[i].idx;", "prune"),
    ("prefill survivors not put back in order", "pe_oracle.c",
     "qsort(kept, (size_t)keep, sizeof(int32_t), cmp_i32);", "", "prune"),
    ("prefill slot off by one", "pe_oracle.c", "const int64_t dst = ((int64_t)bt[i / B] * B + (i % B)) * (int64_t)D;\n      memcpy(k_pool + dst, k_in + src",
     "const int64_t dst = ((int64_t)bt[i / B] * B + ((i + 1) % B)) * (int64_t)D;\n      memcpy(k_pool + dst, k_in + src", "prune"),
    ("prefill V taken from K", "pe_oracle.c", "memcpy(v_pool + dst, v_in + src, sizeof(float) * (size_t)D);\n    }\n    if (kept_idx_out) {",
     "memcpy(v_pool + dst, k_in + src, sizeof(float) * (size_t)D);\n    }\n    if (kept_idx_out) {", "prune"),
    ("evict ties to the highest index", "pe_oracle.c", "if (sc[j] < sc[best]) best = j;", "if (sc[j] <= sc[best]) best = j;", "evict"),
    ("evict the highest score", "pe_oracle.c", "if (sc[j] < sc[best]) best = j;", "if (sc[j] > sc[best]) best = j;", "evict"),
    ("evict without the budget gate", "pe_oracle.c",
     "const int trigger = (len > 0) && (len % B == 0) && (len >= C);\n    for (int h = 0; h < Hk; ++h) {\n      const int row = s * Hk + h;\n      if (!trigger) {\n        evicted_logical_out[row] = -1;\n        freed_phys_out[row] = -1;\n        continue;\n      }\n      const int n = len / B;\n      const float* sc",
     "const int trigger = (len > 0) && (len % B == 0);\n    for (int h = 0; h < Hk; ++h) {\n      const int row = s * Hk + h;\n      if (!trigger) {\n        evicted_logical_out[row] = -1;\n        freed_phys_out[row] = -1;\n        continue;\n      }\n      const int n = len / B;\n      const float* sc", "evict"),
    ("evict shift starts one late", "pe_oracle.c",
     "freed_phys_out[row] = bt[best];\n      for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];\n      bt[n - 1] = -1;\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants",
     "freed_phys_out[row] = bt[best];\n      for (int j = best + 1; j + 1 < n; ++j) bt[j] = bt[j + 1];\n      bt[n - 1] = -1;\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants", "evict"),
    ("evict drops one token instead of a page", "pe_oracle.c",
     "if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants",
     "if (trigger) seq_lens[s] = len - 1;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants", "evict"),
    ("variant: protection off by one", "pe_oracle.c", "lo = protect_first < n - 1 ? protect_first : n - 1;",
     "lo = protect_first + 1 < n - 1 ? protect_first + 1 : n - 1;", "evict_ex"),
    ("variant: shared score is head 0 only", "pe_oracle.c",
     "for (int g = 0; g < Hk; ++g) sum += (double)scores[((int64_t)s * Hk + g) * max_blocks + j];",
     "for (int g = 0; g < 1; ++g) sum += (double)scores[((int64_t)s * Hk + g) * max_blocks + j] * Hk;", "evict_ex"),
    ("append: freed page not consumed", "pe_oracle.c", "page = freed_phys[row];\n          freed_phys[row] = -1;",
     "page = freed_phys[row];", "loop"),
    ("append: slot off by one", "pe_oracle.c",
     "const int64_t dst = ((int64_t)bt[len / B] * B + (len % B)) * (int64_t)D;",
     "const int64_t dst = ((int64_t)bt[len / B] * B + ((len + 1) % B)) * (int64_t)D;", "loop"),
    ("attention: scale dropped", "pe_oracle.c", "logit[t] = scale * dot;", "logit[t] = dot;", "attention"),
    ("attention: wrong KV head for a query head", "pe_oracle.c", "const int s = sh / Hq, hq = sh % Hq, g = hq / G;\n    const int len = seq_lens[s];\n    const float* qv = q + (int64_t)sh * D;\n    const int32_t* bt = block_table + ((int64_t)s * Hk + g) * max_blocks;",
     "const int s = sh / Hq, hq = sh % Hq, g = hq % Hk;\n    const int len = seq_lens[s];\n    const float* qv = q + (int64_t)sh * D;\n    const int32_t* bt = block_table + ((int64_t)s * Hk + g) * max_blocks;", "attention"),
    ("attention: values read from the key pool", "pe_oracle.c",
     "const float* vr = v_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;",
     "const float* vr = k_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;", "attention"),
    ("attention: not normalised", "pe_oracle.c", "for (int d = 0; d < D; ++d) o[d] /= denom;\n    if (weights_sum_out) weights_sum_out[sh] = wsum;\n    free(logit);",
     "if (weights_sum_out) weights_sum_out[sh] = wsum;\n    free(logit);", "attention"),
    ("attention: slot within the page ignored", "pe_oracle.c",
     "const float* kr = k_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;",
     "const float* kr = k_pool + ((int64_t)bt[t / B] * B) * (int64_t)D;", "attention"),
    ("shared: head mean not divided", "pe_oracle_shared.c", "return (float)(sum / (double)Hk);", "return (float)sum;", "shared"),
    ("shared: head stride forgotten", "pe_oracle_shared.c", "return ((p * B + i) * Hk + h) * (int64_t)D;",
     "return ((p * B + i) * Hk) * (int64_t)D;", "shared"),
    ("shared: tokens chosen by head 0", "pe_oracle_shared.c", "tok[i].score = head_mean(tmp, Hk);", "tok[i].score = tmp[0];", "shared"),
    ("shared: eviction ties to the highest index", "pe_oracle_shared.c", "if (j == lo || sc < best_score) {",
     "if (j == lo || sc <= best_score) {", "shared"),
    ("shared: append forgets the other heads", "pe_oracle_shared.c",
     "for (int h = 0; h < Hk; ++h) {\n      const int64_t dst = sh_off(bt[len / B], len % B, h, B, Hk, D);",
     "for (int h = 0; h < 1; ++h) {\n      const int64_t dst = sh_off(bt[len / B], len % B, h, B, Hk, D);", "shared"),
    ("block score reads K in place of V", "pe_oracle.c",
     "sum += oracle_token_ratio(k_pool + page + (int64_t)i * D, v_pool + page + (int64_t)i * D, D);",
     "sum += oracle_token_ratio(k_pool + page + (int64_t)i * D, k_pool + page + (int64_t)i * D, D);", "scores"),
    ("token ratios stored token-major", "pe_oracle.c", "ratio_out[(int64_t)h * total_tokens + t] =",
     "ratio_out[(int64_t)t * Hk + h] =", "scores"),
    ("prefill evicts one token too few", "pe_oracle.c", "const int keep = L < C ? L : C;\n    const int E = L - keep; /* max(0, L - C) */",
     "const int keep = L < C ? L : C;\n    const int E = L > C ? L - C - 1 : 0;", "prune"),
    ("prefill reports the prompt length", "pe_oracle.c", "if (h == 0) seq_lens_out[s] = keep;", "if (h == 0) seq_lens_out[s] = L;", "prune"),
    ("evict reports the logical index as the freed page", "pe_oracle.c",
     "evicted_logical_out[row] = best;\n      freed_phys_out[row] = bt[best];\n      for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];\n      bt[n - 1] = -1;\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants",
     "evicted_logical_out[row] = best;\n      freed_phys_out[row] = best;\n      for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];\n      bt[n - 1] = -1;\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants", "evict"),
    ("evict leaves the tail entry", "pe_oracle.c",
     "for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];\n      bt[n - 1] = -1;\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants",
     "for (int j = best; j + 1 < n; ++j) bt[j] = bt[j + 1];\n    }\n    if (trigger) seq_lens[s] = len - B;\n  }\n  return ORACLE_OK;\n}\n\n/* Variants", "evict"),
    ("variant: last pages not protected", "pe_oracle.c", "hi = n - protect_last > lo + 1 ? n - protect_last : lo + 1;",
     "hi = n > lo + 1 ? n : lo + 1;", "evict_ex"),
    ("variant: oldest policy takes the newest candidate", "pe_oracle.c", "int best = lo;\n      if (policy == 0) {",
     "int best = hi - 1;\n      if (policy == 0) {", "evict_ex"),
    ("append: spare cursor not advanced", "pe_oracle.c", "spare_used[row] += 1;", "", "loop"),
    ("attention: newest token left out", "pe_oracle.c", "double m = -INFINITY;\n    for (int t = 0; t < len; ++t) {\n      const float* kr = k_pool + ((int64_t)bt[t / B] * B + (t % B)) * (int64_t)D;",
     "double m = -INFINITY;\n    for (int t = 0; t < len; ++t) {\n      const float* kr = k_pool + ((int64_t)bt[(t > 0 ? t - 1 : 0) / B] * B + ((t > 0 ? t - 1 : 0) % B)) * (int64_t)D;", "attention"),
    ("shared: queries all read head 0", "pe_oracle_shared.c", "const float* kr = k_pool + sh_off(bt[t / B], t % B, g, B, Hk, D);",
     "const float* kr = k_pool + sh_off(bt[t / B], t % B, 0, B, Hk, D);", "shared"),
    ("shared: prune copies head 0 into every head", "pe_oracle_shared.c", "const int64_t src = ((t0 + kept[i]) * Hk + h) * (int64_t)D;",
     "const int64_t src = ((t0 + kept[i]) * Hk) * (int64_t)D;", "shared"),
    ("shared: page score from the first slot only", "pe_oracle_shared.c", "for (int i = 0; i < B; ++i)\n            sum += oracle_token_ratio(k_pool + sh_off(p, i, h, B, Hk, D)",
     "for (int i = 0; i < B; ++i)\n            sum += oracle_token_ratio(k_pool + sh_off(p, 0, h, B, Hk, D)", "shared"),
]


def _kill(case, tmp):
    name, fname, old, new, pins = case
    srcs = {}
    for f in ("pe_oracle.c", "pe_oracle_shared.c"):
        srcs[f] = open(os.path.join(ORACLE, f)).read()
    assert srcs[fname].count(old) == 1, "mutant %r: the text to replace must occur exactly once" % name
    srcs[fname] = srcs[fname].replace(old, new)
    tag = "".join(c if c.isalnum() else "_" for c in name)
    paths = []
    for f, text in srcs.items():
        path = os.path.join(tmp, tag + "_" + f)
        open(path, "w").write(text)
        paths.append(path)
    lib = os.path.join(tmp, tag + ".so")
    subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-w", "-o", lib] + paths +
                   ["-lm"], check=True)
    env = dict(os.environ, PE_ORACLE_LIB=lib, PE_ORACLE_MUTANT_RUN="1", OMP_NUM_THREADS="2")
    target = os.path.join(ROOT, "tests", "test_oracle_%s.py" % pins)
    r = subprocess.run([sys.executable, "-m", "pytest", target, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return name, r.returncode, r.stdout[-400:]


@pytest.mark.skipif("PE_ORACLE_LIB" in os.environ, reason="already running against a planted mistake")
def test_every_planted_mistake_is_caught(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda c: _kill(c, str(tmp_path)), MUTANTS))
    survivors = [(n, out) for n, rc, out in results if rc == 0]
    assert not survivors, "pins did not notice: %s" % [n for n, _ in survivors]
    crashed = [(n, rc) for n, rc, _ in results if rc not in (0, 1)]
    assert not crashed, "pin run did not end in an ordinary test failure: %s" % crashed
