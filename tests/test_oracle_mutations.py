"""Do the pins notice a mistake in the oracle?  Each case plants one plausible mistake (a wrong sign, an
off-by-one, a dropped term, swapped operands, a reversed order) in a copy of the oracle's C source, builds
it, and runs the pin tests against that build in a child process: they must fail.  Everything here happens
on the CPU; the HIP library is not involved.

A case names the pin files that are expected to catch it, so a pin that silently stops covering a part of
the oracle shows up here.  Patterns must occur exactly once in the source: a change to the oracle that
touches one of these lines has to update its case."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PLAN_SRC = os.path.join(ROOT, "oracle", "msched_oracle.c")
ANA_SRC = os.path.join(ROOT, "oracle", "analyzer_oracle.c")

BELADY = ["tests/test_oracle_belady.py"]
EXPAND = ["tests/test_oracle_expander.py"]
MIGRATE = ["tests/test_oracle_migrate.py"]
EARLY = ["tests/test_oracle_early_start.py"]
PRIORITY = ["tests/test_priority_policy.py"]
ABLATE = ["tests/test_ablations.py"]
ANALYZER = ["tests/test_oracle_analyzer.py"]

# (name, source, text to find, replacement, pin files that must fail)
PLAN_MUTANTS = [
    ("next use is the last toucher, not the first", PLAN_SRC,
     "if (g < nu[pages.v[i]]) nu[pages.v[i]] = g;", "nu[pages.v[i]] = g;", BELADY),
    ("victims: nearest next use first", PLAN_SRC,
     "if (x->nu != y->nu) return x->nu > y->nu ? -1 : 1;", "if (x->nu != y->nu) return x->nu < y->nu ? -1 : 1;", BELADY),
    ("fetch list in reverse order of use", PLAN_SRC,
     "if (x->nu != y->nu) return x->nu < y->nu ? -1 : 1;", "if (x->nu != y->nu) return x->nu > y->nu ? -1 : 1;", EARLY),
    ("evicts a victim for every fetch, free frames or not", PLAN_SRC,
     "size_t n_evict = n_fetch > n_free ? n_fetch - n_free : 0;", "size_t n_evict = n_fetch < n_cand ? n_fetch : n_cand;", BELADY),
    ("a byte range ends one byte late", PLAN_SRC,
     "if (__builtin_add_overflow(a, len - 1, &last)) return E_OVERFLOW;",
     "if (__builtin_add_overflow(a, len, &last)) return E_OVERFLOW;", EXPAND),
    ("a byte range starts at the next page boundary (aligned inward)", PLAN_SRC,
     "uint64_t p0 = a >> o->page_shift,", "uint64_t p0 = (a + (((uint64_t)1 << o->page_shift) - 1)) >> o->page_shift,", EXPAND),
    ("the coefficient is dropped from the formula", PLAN_SRC,
     "uint64_t v = q->coeff[f];", "uint64_t v = 1; (void)q->coeff[f];", EXPAND),
    ("strided rule: chunks follow each other at the chunk size, not the stride", PLAN_SRC,
     "if (__builtin_mul_overflow(j, stride, &off)) return E_OVERFLOW;",
     "if (__builtin_mul_overflow(j, size, &off)) return E_OVERFLOW;", EXPAND),
    ("a command belongs to the timeslice in which it ends", PLAN_SRC,
     "elapsed < tl_slice[e]) {", "(elapsed == 0 || elapsed + t->cmds[pos[tl_task[e]]].latency <= tl_slice[e])) {", PRIORITY),
    ("the cut leaves one frame unused", PLAN_SRC,
     "if (distinct <= o->F) break;", "if (distinct < o->F) break;", BELADY),
    ("the second timeline entry is fetched as well", PLAN_SRC,
     "if (e == 0) g_end0 = G;", "if (e <= 1) g_end0 = G;", BELADY),
    ("resident wanted pages are fetched again", PLAN_SRC,
     "if (wanted && !resident) {", "if (wanted) {", BELADY),
    ("unwanted pages are not candidates unless some command uses them later", PLAN_SRC,
     "if (!wanted && resident) {", "if (!wanted && resident && nu[p] != NONE32) {", BELADY),
    ("victims' frames handed out in reverse", PLAN_SRC,
     "o->evict_frames.v[i - used_free]);", "o->evict_frames.v[n_evict - 1 - (i - used_free)]);", EARLY),
    ("free frames handed out highest first", PLAN_SRC,
     "i < used_free ? free_frames.v[i] :", "i < used_free ? free_frames.v[n_free - 1 - i] :", BELADY + MIGRATE),
    ("an eviction does not copy the page back", PLAN_SRC,
     "if (o->pool) memcpy(o->host + slot_of(o, p) * P, o->pool + (size_t)f * P, P);", "(void)f;", MIGRATE),
    ("a fetch maps the page but leaves the frame's old bytes", PLAN_SRC,
     "        if (o->pool) memcpy(o->pool + (size_t)f * P, o->host + slot_of(o, p) * P, P);\n        o->page_table[p] = f;\n        o->frame_owner[f] = p;\n    }\n    o->plan_pending = 0;",
     "        o->page_table[p] = f;\n        o->frame_owner[f] = p;\n    }\n    o->plan_pending = 0;", MIGRATE),
    ("a victim stays mapped", PLAN_SRC,
     "        o->page_table[p] = NONE32;\n        o->frame_owner[f] = NONE32;\n        if (o->pool) memcpy(o->host + slot_of(o, p)",
     "        o->frame_owner[f] = NONE32;\n        if (o->pool) memcpy(o->host + slot_of(o, p)", MIGRATE),
    ("readiness: a command waits only for pages of earlier commands", PLAN_SRC,
     "if (o->nu[o->fetch_pages.v[i]] <= g) n++;", "if (o->nu[o->fetch_pages.v[i]] < g) n++;", EARLY),
    ("prefix migration brings the target in before its victim has left", PLAN_SRC,
     "if (i >= o->n_free_used) {", "if (i > o->n_free_used) {", EARLY),
    ("a fault evicts the page needed soonest", PLAN_SRC,
     "if (victim == NONE32 || o->nu[q] > o->nu[victim]) victim = (uint32_t)q;",
     "if (victim == NONE32 || o->nu[q] < o->nu[victim]) victim = (uint32_t)q;", ABLATE),
    ("a fault may evict a page the running command uses", PLAN_SRC,
     "if (o->page_table[q] == NONE32 || in_use[q]) continue;", "if (o->page_table[q] == NONE32) continue;", ABLATE),
    ("LRU holds one page fewer than its capacity", PLAN_SRC,
     "if (resident == capacity) {", "if (resident + 1 >= capacity) {", BELADY),
    ("LRU evicts the most recently used page", PLAN_SRC,
     "uint32_t v = head;\n                    head = next[v];\n                    if (head != NONE32) prev[head] = NONE32; else tail = NONE32;",
     "uint32_t v = tail;\n                    tail = prev[v];\n                    if (tail != NONE32) next[tail] = NONE32; else head = NONE32;", BELADY),
]

ANA_MUTANTS = [
    ("the constant candidate is tried last, so a product can win over it", ANA_SRC,
     "    if (fits(k, val, use, S, 0, c_out)) { *nS_out = 0; return 1; }\n    for (int x = 0; x < nc; x++) {\n        S[0] = cand[x];\n        if (fits(k, val, use, S, 1, c_out)) { *nS_out = 1; S_out[0] = S[0]; return 1; }\n    }",
     "    for (int x = 0; x < nc; x++) {\n        S[0] = cand[x];\n        if (fits(k, val, use, S, 1, c_out)) { *nS_out = 1; S_out[0] = S[0]; return 1; }\n    }\n    if (fits(k, val, use, S, 0, c_out)) { *nS_out = 0; return 1; }", ANALYZER),
    ("proportionality is checked on the first invocation only", ANA_SRC,
     "if (__builtin_mul_overflow(c, prod, &want) || want != val[i]) return 0;",
     "if (__builtin_mul_overflow(c, prod, &want)) return 0;", ANALYZER),
    ("a base pointer need only start a region in one invocation", ANA_SRC,
     "for (int i = 0; i < n_inv && ok; i++) ok = find_start(&k, i, args[(size_t)i * MAX_ARGS + a]) >= 0;",
     "ok = 0; for (int i = 0; i < n_inv && !ok; i++) ok = find_start(&k, i, args[(size_t)i * MAX_ARGS + a]) >= 0;", ANALYZER),
    ("pairs of arguments are never tried", ANA_SRC,
     "if (fits(k, val, use, S, 2, c_out)) {", "if (0 && fits(k, val, use, S, 2, c_out)) {", ANALYZER),
    ("a strided run does not stop at an irregular gap", ANA_SRC,
     "if (count[i] == 1) stride[i] = gap; else if (gap != stride[i]) break;",
     "if (count[i] == 1) stride[i] = gap;", ANALYZER),
    ("a strided run runs over another buffer's base pointer", ANA_SRC,
     "if (other_base) break;", "(void)other_base;", ANALYZER),
    ("aliases of a base produce a second rule", ANA_SRC,
     "if (alias) continue;", "(void)alias;", ANALYZER),
    ("the stride is taken from the gap between chunks, end to start", ANA_SRC,
     "uint64_t gap = row[m].start - row[m - 1].start;", "uint64_t gap = row[m].start - (row[m - 1].start + row[m - 1].len);", ANALYZER),
    ("covered regions are not marked, everything counts as unexplained", ANA_SRC,
     "for (uint64_t j = 0; j < count[i]; j++) covered[(size_t)i * max_iv + m0 + j] = 1;",
     "(void)m0;", ANALYZER),
]

MUTANTS = PLAN_MUTANTS + ANA_MUTANTS


def _build_mutant(tmp_path, src, find, repl):
    text = open(src).read()
    assert text.count(find) == 1, f"the text to change must occur exactly once in {os.path.basename(src)}: {find!r}"
    c = tmp_path / "mutant.c"
    c.write_text(text.replace(find, repl))
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-w", "-shared", "-fPIC", "-o", str(so), str(c)])
    return str(so)


def _run_pins(files, env_extra):
    env = dict(os.environ, **env_extra)
    try:
        return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                               "--timeout", "60", *files],
                              cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    except subprocess.TimeoutExpired as e:       # a schedule that never ends under the mistake is a failed pin too
        return subprocess.CompletedProcess(e.cmd, 124, stdout="timed out")


@pytest.mark.parametrize("name,src,find,repl,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_its_pins(tmp_path, name, src, find, repl, pins):
    so = _build_mutant(tmp_path, src, find, repl)
    var = "MSCHED_ORACLE_LIB" if src == PLAN_SRC else "MSCHED_ANALYZER_ORACLE_LIB"
    r = _run_pins(pins, {var: so})
    assert r.returncode != 0, f"the pins in {pins} passed although the oracle was built with: {name}\n{r.stdout[-2000:]}"
    assert r.returncode != 5, "no test was collected"


def test_the_unchanged_oracle_passes_through_the_same_route(tmp_path):
    """The route itself (a library named by the environment, pins in a child process) does not fail pins."""
    so = _build_mutant(tmp_path, PLAN_SRC, "uint64_t v = q->coeff[f];", "uint64_t v = q->coeff[f] * 1;")
    r = _run_pins(BELADY + EXPAND + MIGRATE, {"MSCHED_ORACLE_LIB": so})
    assert r.returncode == 0, r.stdout[-2000:]
