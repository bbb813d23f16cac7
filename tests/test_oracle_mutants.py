"""Do the pins notice a mistake in the oracle?  (CPU only.)

Each case plants one plausible mistake in a copy of the oracle's source (a wrong comparison,
a dropped term, a wrong index, a swapped operand), builds it, and runs the oracle's pin
tests against that copy in a fresh process.  The pins must fail.  The unmodified source,
run the same way, must pass (otherwise a failure would prove nothing)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "fdy_oracle.cpp")

# (name, text in the oracle, replacement, pin files that must catch it)
MUTANTS = [
    ("scan: closed interval", "if (i >= 0 && (w - table[i].base) < table[i].size) {",
     "if (i >= 0 && (w - table[i].base) <= table[i].size) {", ["test_oracle_scan.py"]),
    ("scan: word equal to a base missed", "std::upper_bound(bases.begin(), bases.end(), w)",
     "std::lower_bound(bases.begin(), bases.end(), w)", ["test_oracle_scan.py"]),
    ("scan: offset from the wrong end", "relocs[K] = Reloc{(uint32_t)j, (uint32_t)i, w - table[i].base};",
     "relocs[K] = Reloc{(uint32_t)j, (uint32_t)i, table[i].base + table[i].size - w};", ["test_oracle_scan.py"]),
    ("stride-4 scan: halves swapped", "value[q] = (uint64_t)units[q] | ((uint64_t)units[q + 1] << 32);",
     "value[q] = (uint64_t)units[q + 1] | ((uint64_t)units[q] << 32);", ["test_oracle_scan.py"]),
    ("stride-4 scan: pairs instead of every position", "for (uint64_t q = 0; q + 1 < n_units; ++q) value[q]",
     "for (uint64_t q = 0; q + 1 < n_units; q += 2) value[q]", ["test_oracle_scan.py"]),
    ("segment: boundary word counted", "(uint64_t)relocs[c].word < word_off[s]) ++c;",
     "(uint64_t)relocs[c].word <= word_off[s]) ++c;", ["test_oracle_scan.py"]),
    ("validate: touching ranges refused", "t[i - 1].base + t[i - 1].size <= t[i].base;",
     "t[i - 1].base + t[i - 1].size < t[i].base;", ["test_oracle_scan.py"]),
    ("mix: wrong shift", "x ^= x >> 27; x *= 0x94d049bb133111ebull;", "x ^= x >> 28; x *= 0x94d049bb133111ebull;",
     ["test_oracle_fingerprint.py"]),
    ("node hash: a block dimension dropped", "a = mix(a ^ ((uint64_t)n.block[1] | ((uint64_t)n.block[2] << 32)));",
     "a = mix(a ^ ((uint64_t)n.block[2] << 32));", ["test_oracle_fingerprint.py"]),
    ("fold: order-insensitive", "H = H * kP + node_hash(nodes[node_off[g] + n], mask);",
     "H = H + kP * node_hash(nodes[node_off[g] + n], mask);", ["test_oracle_fingerprint.py"]),
    ("fold: no length salt", "uint64_t H = mix(N);", "uint64_t H = 0;", ["test_oracle_fingerprint.py"]),
    ("grouping: ids not in order of first appearance", "template_id[g] = T++;", "template_id[g] = G - 1 - T++;",
     ["test_oracle_fingerprint.py"]),
    ("rebase: offset subtracted", "a->new_base[(uint64_t)m * a->A + r.region] + r.offset;",
     "a->new_base[(uint64_t)m * a->A + r.region] - r.offset;", ["test_oracle_materialize.py"]),
    ("rebase: base map ignored", "out[r.word - w0] = a->new_base[(uint64_t)m * a->A + r.region] + r.offset;",
     "out[r.word - w0] = a->new_base[r.region] + r.offset;", ["test_oracle_materialize.py"]),
    ("override: wrong half", "std::memcpy(reinterpret_cast<unsigned char*>(out) + a->ovr[k].byte_off, &v, 4);",
     "std::memcpy(reinterpret_cast<unsigned char*>(out) + (a->ovr[k].byte_off ^ 4), &v, 4);",
     ["test_oracle_materialize.py"]),
    ("patch: template ignored", "const uint64_t row = (uint64_t)t * a->R + a->map_rank[m];\n        for (uint64_t k = a->patch_off[row]; k < a->patch_off[row + 1]; ++k)\n          out[",
     "const uint64_t row = a->map_rank[m];\n        for (uint64_t k = a->patch_off[row]; k < a->patch_off[row + 1]; ++k)\n          out[",
     ["test_oracle_materialize.py"]),
    ("dims: grid override lands on the block", "d[(uint64_t)a->govr[k].node * 6 + c] = a->govr[k].grid[c];",
     "d[(uint64_t)a->govr[k].node * 6 + 3 + c] = a->govr[k].grid[c];", ["test_oracle_materialize.py"]),
    ("derive: the template's value stored", "ovr[K].value = va;", "ovr[K].value = vb;", ["test_oracle_derive.py"]),
    ("derive: only low halves compared", "for (uint64_t off = 0; off < nw * 8; off += 4) {",
     "for (uint64_t off = 0; off < nw * 8; off += 8) {", ["test_oracle_derive.py"]),
]


def run_pins(lib, files):
    env = dict(os.environ, FDY_ORACLE_LIB=lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [
        os.path.join(ROOT, "tests", f) for f in files]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True).returncode


def build(src_text, out_dir, name):
    cpp = os.path.join(out_dir, name + ".cpp")
    lib = os.path.join(out_dir, name + ".so")
    with open(cpp, "w") as f:
        f.write(src_text)
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", cpp, "-o", lib])
    return lib


def test_unmodified_copy_passes(tmp_path):
    lib = build(open(SRC).read(), str(tmp_path), "plain")
    files = sorted({f for m in MUTANTS for f in m[3]})
    assert run_pins(lib, files) == 0


@pytest.mark.parametrize("case", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, case):
    name, old, new, files = MUTANTS[case]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutant '{name}': its anchor must occur exactly once in the oracle"
    lib = build(src.replace(old, new), str(tmp_path), f"mutant{case}")
    assert run_pins(lib, files) != 0, f"no pin noticed: {name}"
