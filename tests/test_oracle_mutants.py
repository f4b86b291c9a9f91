"""Do the pins hold the oracle?  Each case below plants one plausible mistake (a dropped term, a wrong
sign or index, a swapped order, a flipped tie rule) in a copy of oracle/br_oracle.c, builds it, and runs the
oracle's pin tests against that build: at least one of them has to fail.  The unmodified copy has to pass.
Everything here runs on the CPU.

Not planted, because it changes nothing: dropping the clip of the margins at zero (the envelope is a maximum
over the same loads, so no margin is negative)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "br_oracle.c")
PIN_FILES = ["tests/test_oracle_scores.py", "tests/test_oracle_round.py", "tests/test_oracle_bypass.py",
             "tests/test_oracle_survival.py", "tests/test_oracle_baselines.py"]

MUTANTS = [
    # eq. (br0-Fscore)
    ("br0 slope", "return delta - G * over;", "return delta - (G - 1) * over;"),
    ("br0 sign of the overflow", "int64_t over = delta - m;\n  if (over < 0) over = 0;\n  return delta",
     "int64_t over = m - delta;\n  if (over < 0) over = 0;\n  return delta"),
    # eq. (brh-Fscore)
    ("brh last offset dropped", "for (h = 0; h <= S->H; ++h) {\n    int64_t over", "for (h = 0; h < S->H; ++h) {\n    int64_t over"),
    ("brh discount dropped", "pen = fmaf(S->d[h], (float)over, pen);", "pen = pen + (float)over;"),
    ("brh discount sum starts late", "for (h = 0; h <= P->H; ++h) D = D + S->d[h];", "for (h = 1; h <= P->H; ++h) D = D + S->d[h];"),
    ("brh gamma ignored", "S->d[h] = S->d[h - 1] * P->gamma;", "S->d[h] = S->d[h - 1];"),
    ("brh alpha and beta swapped", "return S->aD * (float)delta - S->beta * pen;", "return S->beta * (float)delta - S->aD * pen;"),
    # in-window contribution
    ("survival sum shifted by one", "c = c + S;\n      S = S * (1.0f - p[j - 1]);", "S = S * (1.0f - p[j - 1]);\n      c = c + S;"),
    ("gate inverted", "pfin = 1.0f - S;\n    if (gate_pfin > 0.0f && pfin < gate_pfin) c = Hf;",
     "pfin = 1.0f - S;\n    if (gate_pfin > 0.0f && pfin > gate_pfin) c = Hf;"),
    ("pair: regressor term unweighted", "c = (1.0f - pfin) * Hf + pfin * mu;", "c = (1.0f - pfin) * Hf + mu;"),
    ("pair: gate inverted", "c = (1.0f - pfin) * Hf + pfin * mu;\n    if (gate_pfin > 0.0f && pfin < gate_pfin) c = Hf;",
     "c = (1.0f - pfin) * Hf + pfin * mu;\n    if (gate_pfin > 0.0f && pfin > gate_pfin) c = Hf;"),
    ("floor dropped", "  if (c < 1.0f) c = 1.0f;\n  if (c > Hf) c = Hf;\n  return c;\n}\n\n/* floats kept", "  if (c > Hf) c = Hf;\n  return c;\n}\n\n/* floats kept"),
    # projection, envelope, margins
    ("projection cut one offset early", "if ((float)h <= c) R->Lh[g][h] += kv + h;", "if ((float)h < c) R->Lh[g][h] += kv + h;"),
    ("projection without growth", "R->Lh[g][h] += kv + h;", "R->Lh[g][h] += kv;"),
    ("envelope takes the minimum", "if (R->Lh[g][h] > M) M = R->Lh[g][h];", "if (R->Lh[g][h] < M) M = R->Lh[g][h];"),
    ("horizon minimum is a maximum", "if (h == 0 || v < mn) mn = v;", "if (h == 0 || v > mn) mn = v;"),
    # Stage 2 subsets
    ("subset size unbounded", "if (popcount32(mask) > kmax) continue;", ""),
    ("subset ties to the highest mask", "if (best == 0 || f > bs) {\n      best = (int32_t)mask;", "if (best == 0 || f >= bs) {\n      best = (int32_t)mask;"),
    ("reachable sums: a request used twice", "    for (j = kmax; j >= 1; --j)\n      for (sum = top; sum >= s; --sum) {", "    for (j = 1; j <= kmax; ++j)\n      for (sum = s; sum <= top; ++sum) {"),
    ("reachable sums: ties to the highest mask", "(f == bs && mask < (int64_t)(uint32_t)best)", "(f == bs && mask > (int64_t)(uint32_t)best)"),
    ("reachable sums: a later subset replaces the entry", "if (from >= 0 && tab[j * (top + 1) + sum] < 0) tab", "if (from >= 0) tab"),
    ("reachable sums: table one row short", "    int64_t mask = tab[kmax * (top + 1) + sum];", "    int64_t mask = tab[(kmax - 1) * (top + 1) + sum];"),
    ("reachable sums: watermark ignored", "    if (mask < 0) continue;\n    if (P->token_watermark > 0 && L_g + sum > P->token_watermark) continue;", "    if (mask < 0) continue;"),
    # the round
    ("waiting set ascending", "if (x->s != y->s) return x->s > y->s ? -1 : 1;", "if (x->s != y->s) return x->s < y->s ? -1 : 1;"),
    ("stage 1 prefers the heaviest", "(R.cap[g] == R.cap[bw] && R.L[g] < R.L[bw])) bw = g;", "(R.cap[g] == R.cap[bw] && R.L[g] > R.L[bw])) bw = g;"),
    ("stage 2 prefers the smallest margin", "R.minm[g] > R.minm[bw])) bw = g;", "R.minm[g] < R.minm[bw])) bw = g;"),
    ("guard only below zero", "if (mask == 0 || f <= 0.0) {", "if (mask == 0 || f < 0.0) {"),
    ("stage 1 threshold off by one", "while (T.S_tot > P->S_greedy && T.n_alive > 0) {", "while (T.S_tot >= P->S_greedy && T.n_alive > 0) {"),
    ("admitted load only at offset 0", "  R->L[g] += delta;\n  for (h = 0; h <= R->P->H; ++h) {", "  R->L[g] += delta;\n  for (h = 0; h <= 0; ++h) {"),
    ("envelope not raised after an admission", "    if (R->Lh[g][h] > R->Mh[h]) R->Mh[h] = R->Lh[g][h];\n", ""),
    ("single-request ties to the last", "    if (best < 0 || f > bf) {\n      best = pos;", "    if (best < 0 || f >= bf) {\n      best = pos;"),
    ("imbalance", "return (int64_t)G * M - sum;", "return (int64_t)(G - 1) * M - sum;"),
    # snapshot reductions
    ("snapshot best worker ties to the highest index", "if (bg < 0 || f > bgf) {", "if (bg < 0 || f >= bgf) {"),
    ("snapshot best request: shorter request on equal scores", "(f == bi_f[g] && io->qs[i] > bi_s[g])", "(f == bi_f[g] && io->qs[i] < bi_s[g])"),
    ("snapshot best request: later arrival on equal scores and lengths", "if (cur < 0 || f > bi_f[g] ||", "if (cur < 0 || f >= bi_f[g] ||"),
    # decode step
    ("leaves one step late", "if (rem <= 0) { /* finished", "if (rem < 0) { /* finished"),
    ("kv does not grow", "io->kv[base + k] = kv + 1;", "io->kv[base + k] = kv;"),
    # empirical-survival estimator and refresh rules
    ("remainder not taken from the age", "- cnt * age;", "- cnt * 0;"),
    ("p_fin over the whole history", "p = (float)cnt / (float)surv;", "p = (float)cnt / (float)P->hist_n;"),
    ("window one short", "hi = hist_rank(P, age + P->H);", "hi = hist_rank(P, age + P->H - 1);"),
    ("no decrement between refreshes", "c = c - 1.0f;\n            if (c < 1.0f) {", "if (c < 1.0f) {"),
    ("refresh one token late", "if ((int64_t)since >= P->refresh) {", "if ((int64_t)since > P->refresh) {"),
    # comparison policies
    ("generator: wrong shift", "z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;", "z = (z ^ (z >> 28)) * 0x94D049BB133111EBULL;"),
    ("generator: counter starts at zero", "uint64_t z = key + (c + 1) * 0x9E3779B97F4A7C15ULL;", "uint64_t z = key + c * 0x9E3779B97F4A7C15ULL;"),
    ("round robin: cursor stays on the chosen worker", "pol_state[0] = (pick + 1) % G;", "pol_state[0] = pick % G;"),
    ("jsq takes the fullest", "(pick < 0 || io->n[g] < io->n[pick])) pick = g;", "(pick < 0 || io->n[g] > io->n[pick])) pick = g;"),
    ("jsq ties to the highest index", "(pick < 0 || io->n[g] < io->n[pick])) pick = g;", "(pick < 0 || io->n[g] <= io->n[pick])) pick = g;"),
    ("p2c keeps the fuller", "if (io->n[b] < io->n[a]) pick = b;", "if (io->n[b] > io->n[a]) pick = b;"),
    ("p2c second pick may repeat the first", "(E - 1)) >> 32), a);", "(E - 1)) >> 32), -1);"),
    ("p2c uses the same half twice", "uint32_t lo = (uint32_t)z, hi = (uint32_t)(z >> 32);", "uint32_t lo = (uint32_t)z, hi = (uint32_t)z;"),
    ("policies ignore the slot limit", "    if (E == 0) break; /* every worker is full: the rest keeps waiting */\n", ""),
    ("random pick ignores full workers' absence", "int a = kth_eligible(P, io, (int)(((uint64_t)lo * (uint64_t)E) >> 32), -1);", "int a = (int)(((uint64_t)lo * (uint64_t)G) >> 32);"),
    # pool bypass
    ("bypass ignores the slot limit", "      if (io->n[g] >= P->B) continue;\n", ""),
    ("bypass scores against the stale load", "      io->L[best] += s;\n", ""),
]


def _build(tmp, name, text):
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-I", os.path.join(ROOT, "oracle"),
                           "-o", so, c, "-lm"])
    return so


def _pins_pass(so):
    env = dict(os.environ, BR_ORACLE_LIB=so)
    # the stored c1 round was written by the oracle itself: it guards against drift, it is no independent pin
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                        "-k", "not stored_round"] + PIN_FILES,
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    return r.returncode == 0, r.stdout.decode()[-800:]


def test_every_planted_mistake_is_noticed(tmp_path):
    src = open(SRC).read()
    ok, tail = _pins_pass(_build(str(tmp_path), "control", src))
    assert ok, "the unmodified oracle must pass its pins:\n" + tail
    jobs = []
    for k, (name, old, new) in enumerate(MUTANTS):
        assert src.count(old) == 1, f"mutant '{name}': pattern must occur exactly once ({src.count(old)})"
        jobs.append((name, _build(str(tmp_path), f"m{k}", src.replace(old, new))))
    with ThreadPoolExecutor(max_workers=4) as ex:
        res = list(ex.map(lambda j: (j[0], _pins_pass(j[1])[0]), jobs))
    survivors = [name for name, passed in res if passed]
    assert not survivors, f"pins did not notice: {survivors}"
