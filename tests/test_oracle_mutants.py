"""Do the oracle's pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's source (on the
CPU, in a temporary directory), builds it, and runs the pins of the other test files against the mutant: at
least one of them has to fail.  A mutant that every pin accepts means a hole in the pins, not in the oracle."""
import importlib.util
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "mc_oracle.c")
PIN_MODULES = ["test_oracle_attn", "test_oracle_pack", "test_oracle_append", "test_oracle_merge", "test_oracle_prefix"]

# (name, exact text in mc_oracle.c, replacement)
MUTANTS = [
    ("scores not scaled", "    acc *= scale;\n", "    acc *= 1.0;\n"),
    ("row does not see its own position", "  int64_t hi = (int64_t)P + i + 1;", "  int64_t hi = (int64_t)P + i;"),
    ("row sees one position too many", "  int64_t hi = (int64_t)P + i + 1;", "  int64_t hi = (int64_t)P + i + 2;"),
    ("query heads dealt round-robin over KV heads", "  const int g = h / G;", "  const int g = h % Hkv;"),
    ("no shift by the row maximum", "    s[j - lo] = exp(s[j - lo] - m);", "    s[j - lo] = exp(s[j - lo]);"),
    ("values read from the K pool", "o[d] += p * widen(v_pool, dtype, vb + d);", "o[d] += p * widen(k_pool, dtype, vb + d);"),
    ("lse without the maximum", "  *lse = m + log(Z);", "  *lse = log(Z);"),
    ("slot index off by one inside a page", "  return ((page * Hkv + g) * S + (j % S)) * (int64_t)D;",
     "  return ((page * Hkv + g) * S + ((j + 1) % S)) * (int64_t)D;"),
    ("pool indexed [N, S, Hkv, D]", "  return ((page * Hkv + g) * S + (j % S)) * (int64_t)D;",
     "  return ((page * S + (j % S)) * Hkv + g) * (int64_t)D;"),
    ("pack takes V from the K pool", "    memcpy(v_out + i * page_bytes, v_pool + (int64_t)page_ids[i] * page_bytes, (size_t)page_bytes);",
     "    memcpy(v_out + i * page_bytes, k_pool + (int64_t)page_ids[i] * page_bytes, (size_t)page_bytes);"),
    ("unpack writes page i instead of page ids[i]", "    memcpy(k_pool + (int64_t)page_ids[i] * page_bytes, k_in + i * page_bytes, (size_t)page_bytes);",
     "    memcpy(k_pool + (int64_t)i * page_bytes, k_in + i * page_bytes, (size_t)page_bytes);"),
    ("append starts one slot late", "      const int64_t pos = (int64_t)prefix_lens[r] + i;", "      const int64_t pos = (int64_t)prefix_lens[r] + i + 1;"),
    ("append ignores the KV head in the destination", "        const int64_t dst = ((page * Hkv + g) * S + pos % S) * row_bytes;",
     "        const int64_t dst = ((page * Hkv + 0) * S + pos % S) * row_bytes;"),
    ("merge weights not normalised", "      const double w = exp((double)lse_parts[(int64_t)s * rows + t] - m) / Z;",
     "      const double w = exp((double)lse_parts[(int64_t)s * rows + t] - m);"),
    ("merged lse forgets the shift", "    lse[t] = m + log(Z);", "    lse[t] = log(Z);"),
    ("block keys not chained", "                                  : mix64(digest ^ (((prev << 23) | (prev >> 41)) * 0x9E3779B97F4A7C15ull));",
     "                                  : mix64(digest ^ 0x243F6A8885A308D3ull);"),
    ("block digest ignores token positions", "        sum += mix64((uint64_t)(uint32_t)t[b * block_tokens + j] + ((uint64_t)j << 32));",
     "        sum += mix64((uint64_t)(uint32_t)t[b * block_tokens + j]);"),
    ("wrong multiplier in the mixing function", "  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;", "  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B7ull;"),
    ("partial last block dropped", "    const int64_t blocks = (len + block_tokens - 1) / block_tokens;", "    const int64_t blocks = len / block_tokens;"),
    ("prefix match goes on after a miss", "        if (!found) break;\n        ++len;", "        if (!found) continue;\n        ++len;"),
    ("best instance: last one wins ties", "      if (len > best_len[r]) {", "      if (len >= best_len[r]) {"),
]


def load_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutant '{name}': its target text occurs {text.count(old)} times in mc_oracle.c"
    src = tmp_path / "mc_oracle.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmc_oracle_mutant.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(src), "-lm"],
                   check=True)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{abs(hash(name))}", os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC, mod._LIB, mod._lib = str(src), str(lib), None
    return mod


def pin_calls():
    """Every pin of the other oracle test files as (label, function, keyword arguments), parametrisations expanded."""
    if HERE not in sys.path:
        sys.path.insert(0, HERE)
    calls = []
    for m in PIN_MODULES:
        mod = importlib.import_module(m)
        for fname in sorted(n for n in dir(mod) if n.startswith("test_")):
            fn = getattr(mod, fname)
            combos = [{}]
            for mark in getattr(fn, "pytestmark", []):
                if mark.name != "parametrize":
                    continue
                names = [a.strip() for a in mark.args[0].split(",")]
                new = []
                for base in combos:
                    for val in mark.args[1]:
                        vals = val if len(names) > 1 else (val,)
                        new.append({**base, **dict(zip(names, vals))})
                combos = new
            for kw in combos:
                calls.append((f"{m}.{fname}{kw if kw else ''}", fn, kw))
    return calls


def run_pins_against(index: int, workdir: str) -> int:
    """Child process body: 3 = some pin rejected mutant `index`, 0 = every pin accepted it."""
    import pathlib
    name, old, new = MUTANTS[index]
    mutant = load_mutant(pathlib.Path(workdir), name, old, new)
    for label, fn, kw in pin_calls():
        try:
            fn(mutant, **kw)
        except Exception:           # an assertion, or the mutant failing outright: either way it is caught
            print(f"caught by {label}", flush=True)
            return 3
    return 0


@pytest.mark.parametrize("index", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_some_pin_rejects_the_mutant(tmp_path, index):
    # in a process of its own: a mutant may read or write out of bounds and take the interpreter down with it
    # (that, too, is a mistake being noticed)
    code = f"import sys; sys.path.insert(0, {HERE!r}); sys.path.insert(0, {ROOT!r}); import test_oracle_mutants as t; " \
           f"sys.exit(t.run_pins_against({index}, {str(tmp_path)!r}))"
    res = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=600)
    assert res.returncode != 0, f"no pin noticed the mistake '{MUTANTS[index][0]}'"
    assert res.returncode in (3, -6, -11, 134, 139), f"harness trouble, not a verdict: {res.returncode}\n{res.stderr[-2000:]}"


def test_the_unmodified_oracle_passes_every_pin_through_this_harness(oracle):
    for label, fn, kw in pin_calls():
        fn(oracle, **kw)
