"""Are the oracle's pins strong enough?  Each case plants ONE plausible mistake in a copy of the oracle's C
source (a wrong sign, a misplaced epsilon, an off-by-one mask, a swapped operand, a dropped term ...), builds
the copy with the oracle's own compiler line and runs the pin suites against it in a fresh interpreter: at
least one pin must fail.  The mistakes live on the CPU, in the copy only; nothing here touches the GPU path."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rs_oracle.c")

# (name, exact text in rs_oracle.c, what a mistaken author might have written, pin files that must notice)
MUTANTS = [
    ("rope: sign of the sine term", "v[i] = a * c - b * s;", "v[i] = a * c + b * s;", ["test_oracle_pins.py"]),
    ("rope: angle uses hd/2 instead of hd", "-2.0 * (double)i / (double)hd", "-2.0 * (double)i / (double)half", ["test_oracle_pins.py"]),
    ("rmsnorm: epsilon outside the square root", "1.0f / sqrtf(ss / (float)d + eps)", "1.0f / (sqrtf(ss / (float)d) + eps)", ["test_oracle_pins.py"]),
    ("rmsnorm: sum instead of mean", "sqrtf(ss / (float)d + eps)", "sqrtf(ss + eps)", ["test_oracle_pins.py"]),
    ("attention: scale 1/hd", "float scale = 1.0f / sqrtf((float)hd);", "float scale = 1.0f / (float)hd;", ["test_oracle_pins.py"]),
    ("attention: the own position masked out", "int64_t n_keys = r - start + 1; /* keys j <= own position */",
     "int64_t n_keys = r - start > 0 ? r - start : 1;", ["test_oracle_pins.py"]),
    ("attention: weights not normalised", "float w = scratch[j] / den;", "float w = scratch[j];", ["test_oracle_pins.py"]),
    ("swiglu: gate and up exchanged", "out[i] = silu(g[i]) * u[i];", "out[i] = silu(u[i]) * g[i];", ["test_oracle_pins.py"]),
    ("silu: sign of the exponent", "return z / (1.0f + expf(-z));", "return z / (1.0f + expf(z));", ["test_oracle_pins.py"]),
    ("first residual dropped", "x1[i] = x_rows[i] + x1[i];", "x1[i] = x1[i];", ["test_oracle_pins.py"]),
    ("second residual takes x instead of x1", "y_rows[i] = x1[i] + y_rows[i];", "y_rows[i] = x_rows[i] + y_rows[i];", ["test_oracle_pins.py"]),
    ("second norm uses the first gain", "orc_rmsnorm(x1, L->g2, n, d, L->eps, h2);", "orc_rmsnorm(x1, L->g1, n, d, L->eps, h2);", ["test_oracle_pins.py"]),
    ("cache write: slot and block index exchanged", "int64_t bi = pos / block, slot = pos % block;",
     "int64_t bi = pos % block, slot = pos / block;", ["test_oracle_pins.py"]),
    ("cache write: V stored from K", "memcpy(Vc + off, v, sizeof(float) * Hkv * hd);", "memcpy(Vc + off, k, sizeof(float) * Hkv * hd);", ["test_oracle_pins.py"]),
    ("decode: the new token does not attend to itself", "nk[i] = ctx_lens[i] + 1;", "nk[i] = ctx_lens[i] > 0 ? ctx_lens[i] : 1;", ["test_oracle_pins.py"]),
    ("decode: keys rotated at position + 1", "orc_rope(qkv + qd, ctx_lens, B, Hkv, hd, L->rope_base, nqkv);",
     "{ int32_t *p1 = (int32_t *)malloc(sizeof(int32_t) * B); for (int64_t i = 0; i < B; ++i) p1[i] = ctx_lens[i] + 1; "
     "orc_rope(qkv + qd, p1, B, Hkv, hd, L->rope_base, nqkv); free(p1); }", ["test_oracle_pins.py"]),
    ("prefill attention: query heads interleaved over kv heads instead of grouped", "int64_t hk = hq / G;\n            for (int64_t j = 0; j < n_keys; ++j) {",
     "int64_t hk = hq % Hkv;\n            for (int64_t j = 0; j < n_keys; ++j) {", ["test_oracle_pins.py"]),
    ("decode attention: query heads interleaved over kv heads instead of grouped",
     "int64_t hk = hq / G;\n            int bad = 0;\n            for (int64_t j = 0; j < n; ++j) {\n                int64_t blk = tables[i * max_blk + j / block];",
     "int64_t hk = hq % Hkv;\n            int bad = 0;\n            for (int64_t j = 0; j < n; ++j) {\n                int64_t blk = tables[i * max_blk + j / block];", ["test_oracle_pins.py"]),
    ("decode attention: block table of the neighbouring request", "int64_t blk = tables[i * max_blk + j / block];",
     "int64_t blk = tables[(i > 0 ? i - 1 : 0) * max_blk + j / block];", ["test_oracle_pins.py"]),
    ("chunk rows: cached keys read from the wrong slot", "int64_t off = ((blk * block + j % block) * Hkv + hk) * hd;\n                kp[j] = Kc + off;",
     "int64_t off = ((blk * block + (j + 1) % block) * Hkv + hk) * hd;\n                kp[j] = Kc + off;", ["test_oracle_pins.py"]),
    ("chunk rows: a row does not see its own position", "int64_t n = (int64_t)pos_of_row[r] + 1;\n        const int32_t *tab = tables + (int64_t)req_of_row[r] * max_blk;\n        if (n <= 0 || (n + block - 1) / block > max_blk) { err = 1; continue; }\n        const float **kp = (const float **)malloc(sizeof(float *) * n * 2);",
     "int64_t n = (int64_t)pos_of_row[r] > 0 ? (int64_t)pos_of_row[r] : 1;\n        const int32_t *tab = tables + (int64_t)req_of_row[r] * max_blk;\n        if (n <= 0 || (n + block - 1) / block > max_blk) { err = 1; continue; }\n        const float **kp = (const float **)malloc(sizeof(float *) * n * 2);", ["test_oracle_pins.py"]),
]


def _occurrences(text, pat):
    return len(re.findall(re.escape(pat), text))


@pytest.mark.parametrize("name,good,bad,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, good, bad, pins):
    text = open(SRC).read()
    good, bad = good.replace("\\n", "\n"), bad.replace("\\n", "\n")
    assert _occurrences(text, good) >= 1, f"{name}: the oracle no longer contains the text this case edits"
    mutated = text.replace(good, bad, 1)
    c = tmp_path / "rs_oracle_mutant.c"
    so = tmp_path / "librs_oracle_mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c), "-lm"])
    env = dict(os.environ, RS_ORACLE_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", "-m", "not gpu"]
                       + [os.path.join(ROOT, "tests", f) for f in pins], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0, f"{name}: every pin still passes with this mistake planted\n{r.stdout[-800:]}"
    assert "failed" in r.stdout or "error" in r.stdout.lower(), r.stdout[-400:]


# ---- the oracles written in Python: the same exercise on a copy of the package
PY_MUTANTS = [
    # allocator (section 4.5.1: the block count of a prompt follows from its length)
    ("allocator: floor instead of ceiling", "kv_alloc.py", "need = (n_tokens_total + self.block - 1) // self.block",
     "need = n_tokens_total // self.block", "test_oracle_manager_alloc.py"),
    ("allocator: released blocks return in table order", "kv_alloc.py", "for b in reversed(self.owned.pop(req_id)):",
     "for b in self.owned.pop(req_id):", "test_oracle_manager_alloc.py"),
    ("allocator: a failed allocation takes what there is", "kv_alloc.py", "        if extra > len(self.free):\n            raise NoBlocks()",
     "        if extra > len(self.free):\n            self.owned[req_id] = have + [self.free.pop() for _ in range(len(self.free))]\n            raise NoBlocks()",
     "test_oracle_manager_alloc.py"),
    # manager (section 4.5.3)
    ("manager: buckets round down", "manager.py", "        if value <= e:\n            return i", "        if value < e:\n            return max(i - 1, 0)",
     "test_oracle_manager_alloc.py"),
    ("manager: largest instead of smallest decode share that meets the objective", "manager.py",
     "    for s, cus in enumerate(prof.decode_cus):\n        if row[s] <= slo_us:",
     "    for s, cus in reversed(list(enumerate(prof.decode_cus))):\n        if row[s] <= slo_us:", "test_oracle_manager_alloc.py"),
    ("manager: over-allocation never taken", "manager.py", "    if prof.lat_over_us[b][c] <= slo_us:", "    if False and prof.lat_over_us[b][c] <= slo_us:",
     "test_oracle_manager_alloc.py"),
    ("manager: decode keeps its share when no prefill is pending", "manager.py", "    if not prefill_pending:\n        return 0, TOTAL_CUS",
     "    if False:\n        return 0, TOTAL_CUS", "test_oracle_manager_alloc.py"),
    # request life cycle (sections 4.4, 4.5.1, 4.5.2)
    ("life cycle: the decode batch takes one request too many", "lifecycle.py", "if r.state == PREFILL_DONE and len(self.running) < self.max_batch:",
     "if r.state == PREFILL_DONE and len(self.running) <= self.max_batch:", "test_host_lifecycle.py"),
    ("life cycle: the first arrival is preempted, not the last", "lifecycle.py", "for rid in reversed(self.arrival)", "for rid in self.arrival",
     "test_host_lifecycle.py"),
    ("life cycle: recomputation forgets the generated tokens", "lifecycle.py", "v.state, v.n_prefill, v.ctx = WAITING, v.prompt_len + len(v.out), 0",
     "v.state, v.n_prefill, v.ctx = WAITING, v.prompt_len, 0", "test_host_lifecycle.py"),
    ("life cycle: a finished request keeps its blocks", "lifecycle.py", "        if r.id in self.alloc.owned:\n            self.alloc.release(r.id)",
     "        pass", "test_host_lifecycle.py"),
    ("life cycle: the end-of-sequence token does not end a request", "lifecycle.py", "if tok == self.eos or len(r.out) >= r.max_new:",
     "if len(r.out) >= r.max_new:", "test_host_lifecycle.py"),
    ("hybrid batching: a part that does not end its prompt is not rounded to whole blocks", "lifecycle.py",
     "            if n < rest:\n                n -= n % 16", "            if False:\n                n -= n % 16", "test_host_lifecycle.py"),
    ("hybrid batching: the first token of a prompt is seen in the step that takes its last part", "lifecycle.py",
     "                self.hyb_finishing.append(rid)             # its first token is seen at the next step",
     "                r.state, r.ctx = PREFILL_DONE, r.n_prefill; self._sample(r)", "test_host_lifecycle.py"),
    # token boundary
    ("greedy: the highest index among the maxima", "lm.py", "            if logits[r, j] > best:", "            if logits[r, j] >= best:",
     "test_oracle_lm_pins.py"),
    ("lm head: no final norm", "lm.py", "    h = rmsnorm(np.ascontiguousarray(x, dtype=np.float32), widen(g_final_bf16), eps)",
     "    h = np.ascontiguousarray(x, dtype=np.float32)", "test_oracle_lm_pins.py"),
    ("generation: the fed-back token sits one position early", "lm.py", "[n + len(out) - 1]", "[n + len(out) - 2]", "test_oracle_lm_pins.py"),
    # mixture of experts
    ("moe: the second expert is the smallest logit", "moe.py", "if e != a and (b < 0 or lg[i, e] > lg[i, b]):",
     "if e != a and (b < 0 or lg[i, e] < lg[i, b]):", "test_oracle_moe_pins.py"),
    ("moe: routing weights exchanged", "moe.py", "out[i] = wt[i, 0] * per[int(sel[i, 0])][i] + wt[i, 1] * per[int(sel[i, 1])][i]",
     "out[i] = wt[i, 1] * per[int(sel[i, 0])][i] + wt[i, 0] * per[int(sel[i, 1])][i]", "test_oracle_moe_pins.py"),
    ("moe: weights not normalised over the two", "moe.py", "wt[i, 1] = eb / (np.float32(1.0) + eb)", "wt[i, 1] = eb", "test_oracle_moe_pins.py"),
]


@pytest.mark.parametrize("name,module,good,bad,pins", PY_MUTANTS, ids=[m[0] for m in PY_MUTANTS])
def test_a_mistake_planted_in_a_python_oracle_fails_a_pin(tmp_path, name, module, good, bad, pins):
    import shutil
    good, bad = good.replace("\\n", "\n"), bad.replace("\\n", "\n")
    # a copy of the repository's layout: the oracle package copied (and edited), everything else linked
    shutil.copytree(os.path.join(ROOT, "oracle"), tmp_path / "oracle", ignore=shutil.ignore_patterns("__pycache__"))
    for entry in ("tests", "rs_synth", "paper_2601_11822_amd"):
        os.symlink(os.path.join(ROOT, entry), tmp_path / entry)
    f = tmp_path / "oracle" / module
    text = f.read_text()
    assert _occurrences(text, good) >= 1, f"{name}: {module} no longer contains the text this case edits"
    f.write_text(text.replace(good, bad, 1))
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1")
    env.pop("RS_ORACLE_LIB", None)
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", "-m", "not gpu", "-k", "oracle",
                        os.path.join("tests", pins)], cwd=tmp_path, env=env, capture_output=True, text=True)
    assert r.returncode != 0, f"{name}: every pin still passes with this mistake planted\n{r.stdout[-800:]}"
    assert "failed" in r.stdout, r.stdout[-600:] + r.stderr[-300:]
