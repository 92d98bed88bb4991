"""How sharp the oracle's pins are: each case plants ONE plausible mistake in a copy of the
oracle's source (a dropped square, a wrong sign, a shifted block boundary, a reversed
tie-break, a copy in the wrong direction, truncation instead of rounding, ...), builds it,
and runs the pin tests against that build.  Every mutant must be caught.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "scar_oracle.c")

MUTANTS = [
    ("dropped square", "    s += d * d;", "    s += d;"),
    ("sum instead of difference", "double d = load_real(x_type(dtype), x, j) - load_real(c_type(dtype), c, j);",
     "double d = load_real(x_type(dtype), x, j) + load_real(c_type(dtype), c, j);"),
    ("float accumulator", "  double s = 0.0;\n  for (uint64_t j = lo; j < hi; ++j) {\n    double d = load_real",
     "  float s = 0.0;\n  for (uint64_t j = lo; j < hi; ++j) {\n    double d = load_real"),
    ("signed instead of absolute difference", "    s += d < 0 ? -d : d;", "    s += d;"),
    ("32-bit difference", "int64_t d = (int64_t)x[j] - (int64_t)c[j];", "int64_t d = (int32_t)(x[j] - c[j]);"),
    ("block starts one element late", "  *lo = b * (uint64_t)block_len;", "  *lo = b * (uint64_t)block_len + 1;"),
    ("tail block reads a full length", "  if (*hi > n_elems) *hi = n_elems;", "  if (*hi > n_elems + block_len) *hi = n_elems;"),
    ("bfloat16 taken as the low half", "uint32_t bits = (uint32_t)((const uint16_t *)p)[j] << 16;",
     "uint32_t bits = (uint32_t)((const uint16_t *)p)[j];"),
    ("smallest scores selected", "    if (a->f > b->f) return -1;\n    if (a->f < b->f) return 1;",
     "    if (a->f > b->f) return 1;\n    if (a->f < b->f) return -1;"),
    ("ties to the higher index (real)", "  return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);\n}\n\nstatic int cmp_int_desc",
     "  return a->idx < b->idx ? 1 : (a->idx > b->idx ? -1 : 0);\n}\n\nstatic int cmp_int_desc"),
    ("smallest integer scores selected", "  if (a->i > b->i) return -1;\n  if (a->i < b->i) return 1;",
     "  if (a->i > b->i) return 1;\n  if (a->i < b->i) return -1;"),
    ("NaN ranked lowest", "  if (an != bn) return an ? -1 : 1;", "  if (an != bn) return an ? 1 : -1;"),
    ("selection not sorted by index", "  qsort(out_idx, k, sizeof(uint32_t), cmp_u32_asc);\n  free(all);", "  free(all);"),
    ("one block too few selected", "  for (uint32_t i = 0; i < k; ++i) out_idx[i] = all[i].idx;",
     "  for (uint32_t i = 0; i < k; ++i) out_idx[i] = all[i + (k < n_blocks)].idx;"),
    ("commit copies the checkpoint into x", "      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo) * es);\n    }\n    if (staging)",
     "      memcpy((char *)x + lo * es, (const char *)c + lo * es, (hi - lo) * es);\n    }\n    if (staging)"),
    ("commit truncates instead of rounding", "  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;", "  (void)rest;"),
    ("commit rounds ties away from zero", "(rest == 0x8000u && (keep & 1u))", "(rest == 0x8000u)"),
    ("staging rows laid out by block number", "(char *)staging + (uint64_t)i * block_len * es", "(char *)staging + (uint64_t)idx[i] % n_idx * block_len * es"),
    ("recovery overwrites the checkpoint", "      memcpy((char *)x + lo * es, (const char *)c + lo * es, (hi - lo) * es);\n    }\n  }\n  return ORACLE_OK;\n}\n\n/* The lost set",
     "      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo) * es);\n    }\n  }\n  return ORACLE_OK;\n}\n\n/* The lost set"),
    ("norm measured after the overwrite", "int rc = oracle_perturbation_norm(dtype, x, c, n_elems, block_len, lost, n_lost, norm_out);\n      if (rc) return rc;",
     "int rc = oracle_perturbation_norm(dtype, c, c, n_elems, block_len, lost, n_lost, norm_out);\n      if (rc) return rc;"),
    ("norm without the square root", "    out->norm = sqrt(fs);\n  }\n  return ORACLE_OK;\n}\n\n/* Partial recovery", "    out->norm = fs;\n  }\n  return ORACLE_OK;\n}\n\n/* Partial recovery"),
    ("integer norm as root of squares", "    out->isum = is;\n    out->sum = (double)is;\n    out->norm = (double)is;", "    out->isum = is;\n    out->sum = (double)is;\n    out->norm = sqrt((double)is);"),
    ("norm over all blocks ignores the list", "    block_range(idx ? idx[i] : (uint64_t)i, n_elems, block_len, &lo, &hi);", "    block_range((uint64_t)i, n_elems, block_len, &lo, &hi);"),
    ("duplicates accepted", "    if (idx[i] >= n_blocks || seen[idx[i]]) {", "    if (idx[i] >= n_blocks) {"),
    ("mask inverted", "    if (mask[b]) out_idx[m++] = b;", "    if (!mask[b]) out_idx[m++] = b;"),
    ("round-robin ignores the cursor", "out_idx[i] = (uint32_t)((cursor + i) % n_blocks);", "out_idx[i] = (uint32_t)(i % n_blocks);"),
    ("Philox with nine rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
    ("Philox key not advanced", "      k0 += W0;\n      k1 += W1;", "      k0 += W0;"),
    ("random draw ignores the checkpoint number", "const uint32_t ctr[4] = {b, 0u, (uint32_t)draw, (uint32_t)(draw >> 32)};", "const uint32_t ctr[4] = {b, 0u, 0u, 0u};"),
    ("unequal blocks: score of the next block", "block_sqdist(dtype, x, c, offsets[b], offsets[b + 1]);\n  }\n  return ORACLE_OK;",
     "block_sqdist(dtype, x, c, offsets[b + 1], b + 2 <= n_blocks ? offsets[b + 2 <= n_blocks ? b + 2 : b + 1] : offsets[b + 1]);\n  }\n  return ORACLE_OK;"),
    ("listed scores stored by list position", "      ((double *)scores)[idx[i]] = block_sqdist(dtype, x, c, lo, hi);",
     "      ((double *)scores)[i] = block_sqdist(dtype, x, c, lo, hi);"),
    ("listed integer scores of the block before", "      ((int64_t *)scores)[idx[i]] = block_l1((const int32_t *)x, (const int32_t *)c, lo, hi);",
     "      ((int64_t *)scores)[idx[i]] = block_l1((const int32_t *)x, (const int32_t *)c, lo - (lo ? 1 : 0), hi);"),
    ("total variation without the half", "  return 0.5 * s;", "  return s;"),
    ("total variation of squares", "s += fabs(load_real(dtype, x, j) - load_real(dtype, c, j));",
     "s += (load_real(dtype, x, j) - load_real(dtype, c, j)) * (load_real(dtype, x, j) - load_real(dtype, c, j));"),
    ("total variation signed", "s += fabs(load_real(dtype, x, j) - load_real(dtype, c, j));",
     "s += load_real(dtype, x, j) - load_real(dtype, c, j);"),
    ("document length ignored in the score", "    scores[b] = (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, lo, hi);",
     "    scores[b] = block_tv(dtype, x, c, lo, hi);"),
    ("document length of the list position", "    total += (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, lo, hi);",
     "    total += (weights ? (double)weights[i] : 1.0) * block_tv(dtype, x, c, lo, hi);"),
    ("scaled norm as a root", "block_tv(dtype, x, c, lo, hi);\n  }\n  out->sum = out->norm = total;",
     "block_tv(dtype, x, c, lo, hi);\n  }\n  out->sum = total; out->norm = sqrt(total);"),
    ("unequal blocks: scaled norm as a root", "offsets[b + 1]);\n  }\n  out->sum = out->norm = total;",
     "offsets[b + 1]);\n  }\n  out->sum = total; out->norm = sqrt(total);"),
    ("unequal blocks: staging offsets include the block itself", "      staging_offsets[i] = packed;\n", "      staging_offsets[i] = packed + (hi - lo);\n"),
    ("unequal blocks: staging packed by block position", "memcpy((char *)staging + packed * es, (const char *)c + lo * es, (hi - lo) * es);",
     "memcpy((char *)staging + lo * es, (const char *)c + lo * es, (hi - lo) * es);"),
    ("unequal blocks: bfloat16 checkpoint truncated on commit", "for (uint64_t j = lo; j < hi; ++j) ((uint16_t *)c)[j] = round_to_bf16(((const float *)x)[j]);\n    } else if (hi > lo) {",
     "for (uint64_t j = lo; j < hi; ++j) ((uint16_t *)c)[j] = (uint16_t)(((const uint32_t *)x)[j] >> 16);\n    } else if (hi > lo) {"),
    ("unequal blocks: rows read from the block's own offset", "memcpy((char *)x + lo * es, (const char *)rows + row_offsets[i] * es, len * es);",
     "memcpy((char *)x + lo * es, (const char *)rows + lo * es, len * es);"),
    ("unequal blocks: norm of the rows after the overwrite", "double d = load_real(c_type(dtype), rows, r0 + t) - load_real(x_type(dtype), x, lo + t);",
     "double d = load_real(c_type(dtype), rows, r0 + t) - load_real(c_type(dtype), rows, r0 + t);"),
    ("unequal rows: document length ignored in the scaled score",
     "    scores[b] = (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, offsets[b], offsets[b + 1]);",
     "    scores[b] = block_tv(dtype, x, c, offsets[b], offsets[b + 1]);"),
    ("unequal rows: scaled norm weighs by list position",
     "    total += (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, offsets[b], offsets[b + 1]);",
     "    total += (weights ? (double)weights[i] : 1.0) * block_tv(dtype, x, c, offsets[b], offsets[b + 1]);"),
    ("unequal blocks: commit one element short", "    } else if (hi > lo) {\n      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo) * es);\n    }\n    if (staging_offsets) {",
     "    } else if (hi > lo) {\n      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo - 1) * es);\n    }\n    if (staging_offsets) {"),
]


def run_pins(lib_path):
    env = dict(os.environ, SCAR_ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def build(source_text, out_dir, name):
    src = os.path.join(out_dir, name + ".c")
    lib = os.path.join(out_dir, name + ".so")
    with open(src, "w") as fh:
        fh.write(source_text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", lib, src, "-lm"], check=True)
    return lib


def test_the_unmutated_copy_passes(tmp_path):
    r = run_pins(build(open(SRC).read(), str(tmp_path), "clean"))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_is_caught(what, old, new, tmp_path):
    text = open(SRC).read()
    assert text.count(old) == 1, "the oracle's source no longer holds the line to mutate: %r" % old
    r = run_pins(build(text.replace(old, new), str(tmp_path), "mutant"))
    assert r.returncode != 0, "no pin noticed: " + what
