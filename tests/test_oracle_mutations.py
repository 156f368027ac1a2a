"""The pins must notice a broken oracle.

Each case plants one plausible mistake in a copy of oracle/zen_ref.c (on the CPU, never in the GPU
path), builds it, and runs a compact battery of the same pins the other oracle tests use: published
hash vectors, the library hash, brute force on tiny inputs, the paper's worked hash-bitmap example,
the dense-sum aggregate.  Every mutant has to fail the battery; the unmodified source has to pass.
"""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "zen_ref.c")).read()

MUTANTS = [
    ("hash: wrong first constant", "k *= 0xcc9e2d51u;", "k *= 0xcc9e2d53u;"),
    ("hash: rotation 15 -> 16", "k = rotl32(k, 15);", "k = rotl32(k, 16);"),
    ("hash: key length not mixed in", "h ^= 4u; /* key length in bytes */", ""),
    ("hash: h*5 -> h*3", "h = h * 5u + 0xe6546b64u;", "h = h * 3u + 0xe6546b64u;"),
    ("hash: finaliser shift dropped", "h ^= h >> 13;\n    h *= 0xc2b2ae35u;", "h *= 0xc2b2ae35u;"),
    ("owner: seed ignored", "return zen_ref_hash(idx, seed) % n;", "return zen_ref_hash(idx, 0) % n;"),
    ("nonzero: sign bit counted (-0 becomes non-zero)", "if ((bits & 0x7fffffffu) != 0) { nz = 1; break; }",
     "if (bits != 0) { nz = 1; break; }"),
    ("nonzero: only the first column looked at", "for (uint32_t c = 0; c < row_dim; ++c) {\n            uint32_t bits;",
     "for (uint32_t c = 0; c < 1; ++c) {\n            uint32_t bits;"),
    ("partition: offsets shifted by one", "offsets[p + 1] = (uint32_t)pos;", "offsets[p + 1] = (uint32_t)pos + (p + 1 < n);"),
    ("partition: wrong partition order", "for (uint32_t p = 0; p < n; ++p) {\n        for (uint64_t k = 0; k < nnz; ++k)\n            if (owner_of_I[k] == p)",
     "for (uint32_t p = 0; p < n; ++p) {\n        for (uint64_t k = 0; k < nnz; ++k)\n            if (owner_of_I[k] == n - 1 - p)"),
    ("gather: row k instead of row indices[k]", "grad + (uint64_t)indices[k] * row_dim,", "grad + (uint64_t)k * row_dim,"),
    ("bitmap layout: no padding to a word", "word_off[p + 1] = word_off[p] + (dom_count[p] + 31) / 32;",
     "word_off[p + 1] = word_off[p] + dom_count[p] / 32 + 1;"),
    ("bitmap encode: MSB-first", "bitmap[word_off[p] + (j >> 5)] |= 1u << (j & 31);",
     "bitmap[word_off[p] + (j >> 5)] |= 0x80000000u >> (j & 31);"),
    ("bitmap encode: position counted over all rows", "if (nz[r]) bitmap[word_off[p] + (j >> 5)] |= 1u << (j & 31);\n            ++j;",
     "if (nz[r]) bitmap[word_off[p] + (r >> 5)] |= 1u << (r & 31);\n            ++j;"),
    ("bitmap decode: wrong bit", "if ((bitmap_p[j >> 5] >> (j & 31)) & 1u) indices[count++] = (uint32_t)r;",
     "if ((bitmap_p[j >> 5] >> ((j + 1) & 31)) & 1u) indices[count++] = (uint32_t)r;"),
    ("aggregate: last occurrence wins", "sum[o + c] += (double)row[c];", "sum[o + c] = (double)row[c];"),
    ("aggregate: sign lost", "sum[o + c] += (double)row[c];", "sum[o + c] += fabs((double)row[c]);"),
    ("aggregate: transposed value index", "const float *row = val[w] + k * (uint64_t)row_dim;",
     "const float *row = val[w] + (counts[w] - 1 - k) * (uint64_t)row_dim;"),
    ("aggregate: zero sums dropped from the count", "for (uint64_t r = 0; r < n_rows; ++r) if (occ[r]) ++U;",
     "for (uint64_t r = 0; r < n_rows; ++r) if (occ[r] > 1) ++U;"),
    ("member mask: index shifted by one", "member[idx[k]] = 1;", "member[idx[k] ? idx[k] - 1 : 0] = 1;"),
    ("densify: row k placed at row k", "memcpy(dense + (uint64_t)r * row_dim, val[w] + k * (uint64_t)row_dim,",
     "memcpy(dense + (uint64_t)k * row_dim, val[w] + k * (uint64_t)row_dim,"),
    ("densify: value row taken from the index", "memcpy(dense + (uint64_t)r * row_dim, val[w] + k * (uint64_t)row_dim,",
     "memcpy(dense + (uint64_t)r * row_dim, val[w] + (counts[w] - 1 - k) * (uint64_t)row_dim,"),
    ("pull apply: every partition reads partition 0's words", "zen_ref_bitmap_decode(owner, n_rows, p, bitmap + word_off[p], idx);",
     "zen_ref_bitmap_decode(owner, n_rows, p, bitmap + word_off[0], idx);"),
    ("pull apply: value of the next set bit", "val[p] + (uint64_t)i * row_dim, (size_t)row_dim * 4);",
     "val[p] + (uint64_t)(i + 1 < k ? i + 1 : i) * row_dim, (size_t)row_dim * 4);"),
    ("pull apply: count not checked", "if ((uint64_t)k != counts[p]) { free(idx); return ZEN_REF_ERR_INVALID; }", ""),
    ("hash memory: serial counter starts at 0", "for (uint32_t p = 0; p < n; ++p) c[p] = r1;", "for (uint32_t p = 0; p < n; ++p) c[p] = 0;"),
    ("hash memory: occupied cell overwritten", "if (x[p * cells + q] == 0xffffffffu) { x[p * cells + q] = I[t]; placed = 1; }",
     "{ x[p * cells + q] = I[t]; placed = 1; }"),
    ("hash memory: only the first hash function tried", "for (uint32_t i = 0; i < k && !placed; ++i) {\n            const uint64_t q = slot[i][t];",
     "for (uint32_t i = 0; i < 1 && !placed; ++i) {\n            const uint64_t q = slot[i][t];"),
    ("hash memory: partition ignored", "const uint32_t p = part[t];\n        if (p >= n) { free(c); return ZEN_REF_ERR_INVALID; }\n        int placed = 0;",
     "const uint32_t p = 0;\n        int placed = 0;"),
    ("hash memory: overflow not reported", "return worst > r2 ? ZEN_REF_ERR_CAPACITY : ZEN_REF_OK;", "return ZEN_REF_OK;"),
    ("hash slots: seed ignored", "(uint32_t)(zen_ref_hash(I[t], seed_i) % r1);", "(uint32_t)(zen_ref_hash(I[t], 0) % r1);"),
    ("extract: a cell skipped", "for (uint64_t q = 0; q < cells; ++q)\n            if (x[p * cells + q] != 0xffffffffu)",
     "for (uint64_t q = 1; q < cells; ++q)\n            if (x[p * cells + q] != 0xffffffffu)"),
    ("overlap: divided by the larger set", "return (double)both / (double)(n1 < n2 ? n1 : n2);",
     "return (double)both / (double)(n1 > n2 ? n1 : n2);"),
    ("union sizes: repeats counted again", "if (!seen[idx[w][k]]) { seen[idx[w][k]] = 1; ++u; }", "{ seen[idx[w][k]] = 1; ++u; }"),
    ("skewness: last partition taken as full", "const uint64_t rows = (lo + size <= n_rows ? size : n_rows - lo);",
     "const uint64_t rows = size;"),
    ("skewness: not divided by the density", "return worst / ((double)nnz / (double)n_rows);", "return worst;"),
    ("time BP: the Pull term forgotten", "(gamma_n + 1.0) * 2.0 * M * d_G / b;", "(1.0) * 2.0 * M * d_G / b;"),
    ("time BP: factor (n-1)/n missing", "return (double)(n - 1) / (double)n * (gamma_n + 1.0)", "return (gamma_n + 1.0)"),
    ("time HC: one stage too many", "while ((1u << stages) < n) ++stages;", "while ((1u << stages) <= n) ++stages;"),
    ("top-k: ascending instead of descending", "return x < y ? 1 : (x > y ? -1 : 0);", "return x > y ? 1 : (x < y ? -1 : 0);"),
    ("top-k: sign bit compared", "mag[t] = bits & 0x7fffffffu;", "mag[t] = bits;"),
    ("top-k: sample offset ignored", "memcpy(&bits, g + first + t * stride, 4);", "memcpy(&bits, g + t * stride, 4);"),
    ("threshold: strictly greater", "if ((bits & 0x7fffffffu) >= thr) { out[i] = g[i]; ++kept; }", "if ((bits & 0x7fffffffu) > thr) { out[i] = g[i]; ++kept; }"),
    ("threshold: zeros kept at threshold 0", "const uint32_t thr = threshold ? threshold : 1u;", "const uint32_t thr = threshold;"),
    ("format bytes: hash bitmap charged per server", "out[3] = 4.0 * (double)nnz + (double)G / 8.0;", "out[3] = 4.0 * (double)nnz + (double)n * (double)G / 8.0;"),
    ("format bytes: block id forgotten", "(4.0 * (double)block + 4.0);", "(4.0 * (double)block);"),
    ("nonzero blocks: every index counted", "if (!hit[b]) { hit[b] = 1; ++c; }", "{ hit[b] = 1; ++c; }"),
    ("imbalance: factor n missing", "return (double)n * (double)mx / (double)total;", "return (double)mx / (double)total;"),
]


def _build(source, tmpdir, name):
    c = os.path.join(tmpdir, name + ".c")
    so = os.path.join(tmpdir, name + ".so")
    open(c, "w").write(source)
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-shared", "-fPIC", "-o", so, c, "-lm"])
    return so


def run_battery(so_path):
    """Runs tests/pins_battery.py on a build of the oracle in a child process (a broken oracle may
    corrupt memory); returns True iff every pin held."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "pins_battery.py"), so_path],
                       capture_output=True, text=True, timeout=120)
    return r.returncode == 0 and "battery ok" in r.stdout


def test_unmodified_oracle_passes_the_battery():
    with tempfile.TemporaryDirectory() as d:
        assert run_battery(_build(SRC, d, "clean"))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_mutant_fails_a_pin(name, old, new):
    assert SRC.count(old) >= 1, "mutation site not found: " + name
    with tempfile.TemporaryDirectory() as d:
        assert not run_battery(_build(SRC.replace(old, new, 1), d, "mutant")), "mutant survived every pin: " + name
