/*
 * CPU oracle for the five steps of SCAR's checkpoint path.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain, slow statement of what each step
 * computes, used only to check the GPU library (tests, the smoke check and the
 * benchmark's CPU-baseline leg).  It shares no code, header or table with the GPU
 * library and the GPU library never calls it.
 *
 * Notation follows the paper: x = live parameters, c (the paper's z) = running
 * checkpoint, both cut into n_blocks blocks of block_len elements (the last block
 * may be short); a block is one "parameter" of Section 4.3 / 5.1 (a matrix row, a
 * shard).  K = blocks chosen for a checkpoint, S = blocks lost in a failure.
 *
 * Arithmetic: floating data are widened to double and everything is accumulated in
 * double; integer tables are widened to int64 and results are exact.
 *
 * Every loop is over whole blocks in index order; the only threading is an OpenMP
 * "parallel for" over independent blocks (thread count set by
 * oracle_set_num_threads, default 1).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ORACLE_F32_BF16C: x is float32 and the checkpoint c is kept in bfloat16 (a reduced-
 * precision checkpoint, Example 2.1): saving rounds to nearest even, restoring widens. */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_I32 = 2, ORACLE_F32_BF16C = 3 };
enum { ORACLE_OK = 0, ORACLE_ERR_ARG = -1, ORACLE_ERR_INDEX = -2, ORACLE_ERR_NOMEM = -3 };

typedef struct {
  double sum;   /* float data: sum of squared differences; integer: (double)isum */
  double norm;  /* float data: sqrt(sum) (Euclidean norm); integer: (double)isum */
  int64_t isum; /* integer data: sum of absolute differences; float data: 0      */
} oracle_norm;

static int g_threads = 1;

void oracle_set_num_threads(int n) { g_threads = n > 0 ? n : 1; }

int oracle_get_num_threads(void) {
#ifdef _OPENMP
  return g_threads;
#else
  return 1;
#endif
}

/* Element types of x and of c for a store type. */
static int x_type(int dtype) { return dtype == ORACLE_F32_BF16C ? ORACLE_F32 : dtype; }
static int c_type(int dtype) { return dtype == ORACLE_F32_BF16C ? ORACLE_BF16 : dtype; }
static size_t elem_size(int type) { return type == ORACLE_BF16 ? 2 : 4; }

static int dtype_ok(int dtype) {
  return dtype == ORACLE_F32 || dtype == ORACLE_BF16 || dtype == ORACLE_I32 ||
         dtype == ORACLE_F32_BF16C;
}

/* float32 -> bfloat16, round to nearest, ties to even (IEEE 754 roundTiesToEven on the
 * 8-bit significand); NaN stays NaN (quiet), overflow rounds to infinity. */
static uint16_t round_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t keep = u >> 16, rest = u & 0xffffu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  return (uint16_t)keep;
}

static uint64_t count_blocks(uint64_t n_elems, uint32_t block_len) {
  return (n_elems + block_len - 1) / block_len;
}

/* Element j of a float-typed store, widened exactly to double.  bfloat16 is the
 * upper half of an IEEE binary32, so its value is that of the float whose bit
 * pattern is the 16 stored bits followed by 16 zero bits. */
static double load_real(int dtype, const void *p, uint64_t j) {
  if (dtype == ORACLE_F32) return (double)((const float *)p)[j];
  uint32_t bits = (uint32_t)((const uint16_t *)p)[j] << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* [lo, hi) element range of block b. */
static void block_range(uint64_t b, uint64_t n_elems, uint32_t block_len, uint64_t *lo,
                        uint64_t *hi) {
  *lo = b * (uint64_t)block_len;
  *hi = *lo + block_len;
  if (*hi > n_elems) *hi = n_elems;
}

/* Squared Euclidean distance between block b of x and of c (Appendix A.3 uses the
 * Euclidean norm; squaring keeps the order of distances). */
static double block_sqdist(int dtype, const void *x, const void *c, uint64_t lo, uint64_t hi) {
  double s = 0.0;
  for (uint64_t j = lo; j < hi; ++j) {
    double d = load_real(x_type(dtype), x, j) - load_real(c_type(dtype), c, j);
    s += d * d;
  }
  return s;
}

/* L1 distance between block b of two integer count tables.  For a row of topic
 * counts whose total N is unchanged this is 2 * N * TV(x/N, c/N): twice the
 * document-length-scaled total variation of Appendix C. */
static int64_t block_l1(const int32_t *x, const int32_t *c, uint64_t lo, uint64_t hi) {
  int64_t s = 0;
  for (uint64_t j = lo; j < hi; ++j) {
    int64_t d = (int64_t)x[j] - (int64_t)c[j];
    s += d < 0 ? -d : d;
  }
  return s;
}

/* Index lists must be in range and without repeats (a repeat would count a block
 * twice in the norm). */
static int check_indices(const uint32_t *idx, uint32_t n_idx, uint64_t n_blocks) {
  if (n_idx == 0) return ORACLE_OK;
  if (!idx) return ORACLE_ERR_ARG;
  uint8_t *seen = (uint8_t *)calloc(n_blocks ? n_blocks : 1, 1);
  if (!seen) return ORACLE_ERR_NOMEM;
  int rc = ORACLE_OK;
  for (uint32_t i = 0; i < n_idx; ++i) {
    if (idx[i] >= n_blocks || seen[idx[i]]) {
      rc = ORACLE_ERR_INDEX;
      break;
    }
    seen[idx[i]] = 1;
  }
  free(seen);
  return rc;
}

/* Checkpoint step 1 (Section 4.3): distance of every block from its value in the
 * running checkpoint.  scores: double[n_blocks] for float data (squared L2),
 * int64_t[n_blocks] for integer tables (L1). */
int oracle_block_scores(int dtype, const void *x, const void *c, uint64_t n_elems,
                        uint32_t block_len, void *scores) {
  if (!dtype_ok(dtype) || block_len == 0) return ORACLE_ERR_ARG;
  if (n_elems == 0) return ORACLE_OK;
  if (!x || !c || !scores) return ORACLE_ERR_ARG;
  int64_t n_blocks = (int64_t)count_blocks(n_elems, block_len);
#pragma omp parallel for schedule(static) num_threads(g_threads)
  for (int64_t b = 0; b < n_blocks; ++b) {
    uint64_t lo, hi;
    block_range((uint64_t)b, n_elems, block_len, &lo, &hi);
    if (dtype == ORACLE_I32)
      ((int64_t *)scores)[b] = block_l1((const int32_t *)x, (const int32_t *)c, lo, hi);
    else
      ((double *)scores)[b] = block_sqdist(dtype, x, c, lo, hi);
  }
  return ORACLE_OK;
}

/* The same distances for the listed blocks only: scores[b] is recomputed for b in idx and
 * every other entry is left alone (a trainer that knows which rows an iteration touched
 * need not look at the rest; the values are those of oracle_block_scores). */
int oracle_block_scores_rows(int dtype, const void *x, const void *c, uint64_t n_elems,
                             uint32_t block_len, const uint32_t *idx, uint32_t n_idx, void *scores) {
  if (!dtype_ok(dtype) || block_len == 0) return ORACLE_ERR_ARG;
  if (n_idx == 0) return ORACLE_OK;
  if (!x || !c || !scores) return ORACLE_ERR_ARG;
  int rc = check_indices(idx, n_idx, count_blocks(n_elems, block_len));
  if (rc) return rc;
  for (uint32_t i = 0; i < n_idx; ++i) {
    uint64_t lo, hi;
    block_range(idx[i], n_elems, block_len, &lo, &hi);
    if (dtype == ORACLE_I32)
      ((int64_t *)scores)[idx[i]] = block_l1((const int32_t *)x, (const int32_t *)c, lo, hi);
    else
      ((double *)scores)[idx[i]] = block_sqdist(dtype, x, c, lo, hi);
  }
  return ORACLE_OK;
}

/* ---- checkpoint step 3: the k blocks with the largest distances -------------- */

typedef struct {
  double f;
  int64_t i;
  uint32_t idx;
} keyed;

/* Larger score first; NaN counts as larger than every number; equal scores go to
 * the lower block index. */
static int cmp_real_desc(const void *pa, const void *pb) {
  const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
  int an = isnan(a->f), bn = isnan(b->f);
  if (an != bn) return an ? -1 : 1;
  if (!an) {
    if (a->f > b->f) return -1;
    if (a->f < b->f) return 1;
  }
  return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);
}

static int cmp_int_desc(const void *pa, const void *pb) {
  const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
  if (a->i > b->i) return -1;
  if (a->i < b->i) return 1;
  return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0);
}

static int cmp_u32_asc(const void *pa, const void *pb) {
  uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
  return a < b ? -1 : (a > b ? 1 : 0);
}

/* scores: double[n_blocks] (scores_are_int == 0) or int64_t[n_blocks].
 * out_idx: k block indices, ascending. */
int oracle_select_topk(int scores_are_int, const void *scores, uint32_t n_blocks, uint32_t k,
                       uint32_t *out_idx) {
  if (k > n_blocks) return ORACLE_ERR_ARG;
  if (k == 0) return ORACLE_OK;
  if (!scores || !out_idx) return ORACLE_ERR_ARG;
  keyed *all = (keyed *)malloc((size_t)n_blocks * sizeof(keyed));
  if (!all) return ORACLE_ERR_NOMEM;
  for (uint32_t b = 0; b < n_blocks; ++b) {
    all[b].idx = b;
    all[b].f = scores_are_int ? 0.0 : ((const double *)scores)[b];
    all[b].i = scores_are_int ? ((const int64_t *)scores)[b] : 0;
  }
  qsort(all, n_blocks, sizeof(keyed), scores_are_int ? cmp_int_desc : cmp_real_desc);
  for (uint32_t i = 0; i < k; ++i) out_idx[i] = all[i].idx;
  qsort(out_idx, k, sizeof(uint32_t), cmp_u32_asc);
  free(all);
  return ORACLE_OK;
}

/* Test helper: the largest total score any k-subset of n (n <= 24) blocks can have,
 * found by trying every subset.  result: double (real scores) or int64_t. */
int oracle_brute_force_topk(int scores_are_int, const void *scores, uint32_t n, uint32_t k,
                            void *result) {
  if (n > 24 || k > n || !scores || !result) return ORACLE_ERR_ARG;
  double best_f = -INFINITY;
  int64_t best_i = INT64_MIN;
  for (uint32_t mask = 0; mask < (1u << n); ++mask) {
    if ((uint32_t)__builtin_popcount(mask) != k) continue;
    double sf = 0.0;
    int64_t si = 0;
    for (uint32_t b = 0; b < n; ++b)
      if (mask >> b & 1u) {
        if (scores_are_int)
          si += ((const int64_t *)scores)[b];
        else
          sf += ((const double *)scores)[b];
      }
    if (sf > best_f) best_f = sf;
    if (si > best_i) best_i = si;
  }
  if (scores_are_int)
    *(int64_t *)result = best_i;
  else
    *(double *)result = best_f;
  return ORACLE_OK;
}

/* Checkpoint step 4, the in-memory part: c_b <- x_b for b in K.  If staging is not
 * NULL, row i of staging (block_len elements per row) also receives block idx[i]
 * (the rows that would go to persistent storage). */
int oracle_checkpoint_commit(int dtype, const void *x, void *c, uint64_t n_elems,
                             uint32_t block_len, const uint32_t *idx, uint32_t n_idx,
                             void *staging) {
  if (!dtype_ok(dtype) || block_len == 0) return ORACLE_ERR_ARG;
  if (n_idx == 0) return ORACLE_OK;
  if (!x || !c) return ORACLE_ERR_ARG;
  int rc = check_indices(idx, n_idx, count_blocks(n_elems, block_len));
  if (rc) return rc;
  size_t es = elem_size(c_type(dtype));
#pragma omp parallel for schedule(static) num_threads(g_threads)
  for (int64_t i = 0; i < (int64_t)n_idx; ++i) {
    uint64_t lo, hi;
    block_range(idx[i], n_elems, block_len, &lo, &hi);
    if (dtype == ORACLE_F32_BF16C) { /* what is saved is x rounded to the checkpoint's precision */
      for (uint64_t j = lo; j < hi; ++j) ((uint16_t *)c)[j] = round_to_bf16(((const float *)x)[j]);
    } else {
      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo) * es);
    }
    if (staging) /* the saved rows, in the checkpoint's element type */
      memcpy((char *)staging + (uint64_t)i * block_len * es, (const char *)c + lo * es,
             (hi - lo) * es);
  }
  return ORACLE_OK;
}

/* Size of the perturbation a recovery of the blocks in idx causes (Appendix A.3):
 * ||c_S - x_S||.  idx == NULL means every block (full recovery, ||c - x||).
 * Float data: Euclidean.  Integer tables: sum of the per-block L1 distances (a
 * positive combination of per-row norms, Appendix C). */
int oracle_perturbation_norm(int dtype, const void *x, const void *c, uint64_t n_elems,
                             uint32_t block_len, const uint32_t *idx, uint32_t n_idx,
                             oracle_norm *out) {
  if (!dtype_ok(dtype) || block_len == 0 || !out) return ORACLE_ERR_ARG;
  uint64_t n_blocks = count_blocks(n_elems, block_len);
  int64_t m = idx ? (int64_t)n_idx : (int64_t)n_blocks;
  out->sum = 0.0;
  out->norm = 0.0;
  out->isum = 0;
  if (m == 0) return ORACLE_OK;
  if (!x || !c) return ORACLE_ERR_ARG;
  if (idx) {
    int rc = check_indices(idx, n_idx, n_blocks);
    if (rc) return rc;
  }
  double *fpart = (double *)calloc((size_t)m, sizeof(double));
  int64_t *ipart = (int64_t *)calloc((size_t)m, sizeof(int64_t));
  if (!fpart || !ipart) {
    free(fpart);
    free(ipart);
    return ORACLE_ERR_NOMEM;
  }
#pragma omp parallel for schedule(static) num_threads(g_threads)
  for (int64_t i = 0; i < m; ++i) {
    uint64_t lo, hi;
    block_range(idx ? idx[i] : (uint64_t)i, n_elems, block_len, &lo, &hi);
    if (dtype == ORACLE_I32)
      ipart[i] = block_l1((const int32_t *)c, (const int32_t *)x, lo, hi);
    else
      fpart[i] = block_sqdist(dtype, x, c, lo, hi);
  }
  double fs = 0.0;
  int64_t is = 0;
  for (int64_t i = 0; i < m; ++i) {
    fs += fpart[i];
    is += ipart[i];
  }
  free(fpart);
  free(ipart);
  if (dtype == ORACLE_I32) {
    out->isum = is;
    out->sum = (double)is;
    out->norm = (double)is;
  } else {
    out->sum = fs;
    out->norm = sqrt(fs);
  }
  return ORACLE_OK;
}

/* Partial recovery (Section 4.1): x_b <- c_b for the lost blocks b in S and nothing
 * else.  If norm_out is not NULL it receives the perturbation ||c_S - x_S|| measured
 * on x as it was before the overwrite. */
int oracle_partial_recover(int dtype, void *x, const void *c, uint64_t n_elems,
                           uint32_t block_len, const uint32_t *lost, uint32_t n_lost,
                           oracle_norm *norm_out) {
  if (!dtype_ok(dtype) || block_len == 0) return ORACLE_ERR_ARG;
  if (norm_out) {
    if (n_lost == 0) {
      norm_out->sum = norm_out->norm = 0.0;
      norm_out->isum = 0;
    } else {
      int rc = oracle_perturbation_norm(dtype, x, c, n_elems, block_len, lost, n_lost, norm_out);
      if (rc) return rc;
    }
  }
  if (n_lost == 0) return ORACLE_OK;
  if (!x || !c) return ORACLE_ERR_ARG;
  int rc = check_indices(lost, n_lost, count_blocks(n_elems, block_len));
  if (rc) return rc;
  size_t es = elem_size(x_type(dtype));
#pragma omp parallel for schedule(static) num_threads(g_threads)
  for (int64_t i = 0; i < (int64_t)n_lost; ++i) {
    uint64_t lo, hi;
    block_range(lost[i], n_elems, block_len, &lo, &hi);
    if (dtype == ORACLE_F32_BF16C) {
      for (uint64_t j = lo; j < hi; ++j) ((float *)x)[j] = (float)load_real(ORACLE_BF16, c, j);
    } else {
      memcpy((char *)x + lo * es, (const char *)c + lo * es, (hi - lo) * es);
    }
  }
  return ORACLE_OK;
}

/* The lost set as an index list: ascending indices b with mask[b] != 0. */
int oracle_mask_to_indices(const uint8_t *mask, uint32_t n_blocks, uint32_t *out_idx,
                           uint32_t *out_count) {
  if (!out_count || (n_blocks && (!mask || !out_idx))) return ORACLE_ERR_ARG;
  uint32_t m = 0;
  for (uint32_t b = 0; b < n_blocks; ++b)
    if (mask[b]) out_idx[m++] = b;
  *out_count = m;
  return ORACLE_OK;
}

/* ---- the comparison strategies of Section 5.4: which blocks a checkpoint saves -------- */

/* "round": blocks are saved in a round-robin manner.  A checkpoint that starts at
 * `cursor` saves the k blocks cursor, cursor+1, ... (mod n_blocks); the caller advances
 * the cursor by k per checkpoint.  out_idx ascending. */
int oracle_select_round(uint32_t n_blocks, uint32_t k, uint64_t cursor, uint32_t *out_idx) {
  if (k > n_blocks) return ORACLE_ERR_ARG;
  if (k == 0) return ORACLE_OK;
  if (!out_idx) return ORACLE_ERR_ARG;
  for (uint32_t i = 0; i < k; ++i) out_idx[i] = (uint32_t)((cursor + i) % n_blocks);
  qsort(out_idx, k, sizeof(uint32_t), cmp_u32_asc);
  return ORACLE_OK;
}

/* Philox4x32-10, the counter-based generator of Salmon, Moraes, Dror and Shaw
 * ("Parallel random numbers: as easy as 1, 2, 3", SC'11): ten rounds of
 *   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * with the key advanced by the Weyl constants (W0, W1) before every round but the first. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += W0;
      k1 += W1;
    }
    uint64_t p0 = M0 * c0, p1 = M1 * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0, c1 = n1, c2 = n2, c3 = n3;
  }
  out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

/* "random": blocks are saved uniformly at random.  Block b draws the 32-bit number
 * Philox4x32-10(counter = (b, 0, draw_lo, draw_hi), key = (seed_lo, seed_hi))[0]; the k
 * blocks with the largest numbers are saved (equal numbers: lower index first), which is
 * a uniformly random k-subset up to ties between 32-bit draws.  `draw` numbers the
 * checkpoint so that every checkpoint gets fresh numbers. */
int oracle_select_random(uint32_t n_blocks, uint32_t k, uint64_t seed, uint64_t draw,
                         uint32_t *out_idx) {
  if (k > n_blocks) return ORACLE_ERR_ARG;
  if (k == 0) return ORACLE_OK;
  if (!out_idx) return ORACLE_ERR_ARG;
  int64_t *num = (int64_t *)malloc((size_t)n_blocks * sizeof(int64_t));
  if (!num) return ORACLE_ERR_NOMEM;
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (uint32_t b = 0; b < n_blocks; ++b) {
    const uint32_t ctr[4] = {b, 0u, (uint32_t)draw, (uint32_t)(draw >> 32)};
    uint32_t r[4];
    oracle_philox4x32_10(ctr, key, r);
    num[b] = (int64_t)r[0];
  }
  int rc = oracle_select_topk(1, num, n_blocks, k, out_idx);
  free(num);
  return rc;
}

/* ---- blocks of unequal length (Section 5.1: "by-layer" partitioning, where every weight
 * or bias tensor of the network is one parameter) --------------------------------------
 * offsets has n_blocks + 1 non-decreasing entries, offsets[0] = 0; block b is the element
 * range [offsets[b], offsets[b+1]) and may be empty.  Everything else is as above. */

static int offsets_ok(const uint64_t *offsets, uint32_t n_blocks) {
  if (!offsets || offsets[0] != 0) return 0;
  for (uint32_t b = 0; b < n_blocks; ++b)
    if (offsets[b + 1] < offsets[b]) return 0;
  return 1;
}

int oracle_var_block_scores(int dtype, const void *x, const void *c, const uint64_t *offsets,
                            uint32_t n_blocks, void *scores) {
  if (!dtype_ok(dtype) || !offsets_ok(offsets, n_blocks)) return ORACLE_ERR_ARG;
  if (n_blocks == 0) return ORACLE_OK;
  if (!scores || (offsets[n_blocks] && (!x || !c))) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
  for (int64_t b = 0; b < (int64_t)n_blocks; ++b) {
    if (dtype == ORACLE_I32)
      ((int64_t *)scores)[b] =
          block_l1((const int32_t *)x, (const int32_t *)c, offsets[b], offsets[b + 1]);
    else
      ((double *)scores)[b] = block_sqdist(dtype, x, c, offsets[b], offsets[b + 1]);
  }
  return ORACLE_OK;
}

/* Checkpoint step 4 of Section 4.3 for blocks of unequal length (Section 5.1, by-layer):
 * c_b <- x_b for the listed blocks.  If staging is given, the listed blocks are also packed
 * into it one after the other in the order of the list - the bytes that go to persistent
 * storage - and staging_offsets[i] receives the element offset of block idx[i] within staging
 * (the lengths of the blocks listed before it, added up), staging_offsets[n_idx] the total. */
int oracle_var_checkpoint_commit(int dtype, const void *x, void *c, const uint64_t *offsets,
                                 uint32_t n_blocks, const uint32_t *idx, uint32_t n_idx,
                                 void *staging, uint64_t *staging_offsets) {
  if (!dtype_ok(dtype) || !offsets_ok(offsets, n_blocks)) return ORACLE_ERR_ARG;
  if (staging && !staging_offsets) return ORACLE_ERR_ARG;
  if (staging_offsets) staging_offsets[0] = 0;
  if (n_idx == 0) return ORACLE_OK;
  int rc = check_indices(idx, n_idx, n_blocks);
  if (rc) return rc;
  size_t es = elem_size(c_type(dtype));
  uint64_t packed = 0; /* elements already in staging */
  for (uint32_t i = 0; i < n_idx; ++i) {
    uint64_t lo = offsets[idx[i]], hi = offsets[idx[i] + 1];
    if (dtype == ORACLE_F32_BF16C) { /* what is saved is x rounded to the checkpoint's precision */
      for (uint64_t j = lo; j < hi; ++j) ((uint16_t *)c)[j] = round_to_bf16(((const float *)x)[j]);
    } else if (hi > lo) {
      memcpy((char *)c + lo * es, (const char *)x + lo * es, (hi - lo) * es);
    }
    if (staging_offsets) {
      staging_offsets[i] = packed;
      /* the saved rows, in the checkpoint's element type */
      if (staging && hi > lo) memcpy((char *)staging + packed * es, (const char *)c + lo * es, (hi - lo) * es);
      packed += hi - lo;
      staging_offsets[i + 1] = packed;
    }
  }
  return ORACLE_OK;
}

/* idx == NULL: every block. */
int oracle_var_perturbation_norm(int dtype, const void *x, const void *c, const uint64_t *offsets,
                                 uint32_t n_blocks, const uint32_t *idx, uint32_t n_idx,
                                 oracle_norm *out) {
  if (!dtype_ok(dtype) || !offsets_ok(offsets, n_blocks) || !out) return ORACLE_ERR_ARG;
  out->sum = out->norm = 0.0;
  out->isum = 0;
  uint32_t m = idx ? n_idx : n_blocks;
  if (idx) {
    int rc = check_indices(idx, n_idx, n_blocks);
    if (rc) return rc;
  }
  double fs = 0.0;
  int64_t is = 0;
  for (uint32_t i = 0; i < m; ++i) {
    uint32_t b = idx ? idx[i] : i;
    if (dtype == ORACLE_I32)
      is += block_l1((const int32_t *)c, (const int32_t *)x, offsets[b], offsets[b + 1]);
    else
      fs += block_sqdist(dtype, x, c, offsets[b], offsets[b + 1]);
  }
  if (dtype == ORACLE_I32) {
    out->isum = is;
    out->sum = out->norm = (double)is;
  } else {
    out->sum = fs;
    out->norm = sqrt(fs);
  }
  return ORACLE_OK;
}

int oracle_var_partial_recover(int dtype, void *x, const void *c, const uint64_t *offsets,
                               uint32_t n_blocks, const uint32_t *lost, uint32_t n_lost,
                               oracle_norm *norm_out) {
  if (!dtype_ok(dtype) || !offsets_ok(offsets, n_blocks)) return ORACLE_ERR_ARG;
  oracle_norm zero = {0.0, 0.0, 0};
  if (n_lost == 0) {
    if (norm_out) *norm_out = zero;
    return ORACLE_OK;
  }
  if (norm_out) {
    int rc = oracle_var_perturbation_norm(dtype, x, c, offsets, n_blocks, lost, n_lost, norm_out);
    if (rc) return rc;
  } else {
    int rc = check_indices(lost, n_lost, n_blocks);
    if (rc) return rc;
  }
  size_t es = elem_size(x_type(dtype));
  for (uint32_t i = 0; i < n_lost; ++i) {
    uint64_t lo = offsets[lost[i]], hi = offsets[lost[i] + 1];
    if (dtype == ORACLE_F32_BF16C) {
      for (uint64_t j = lo; j < hi; ++j) ((float *)x)[j] = (float)load_real(ORACLE_BF16, c, j);
    } else if (hi > lo) {
      memcpy((char *)x + lo * es, (const char *)c + lo * es, (hi - lo) * es);
    }
  }
  return ORACLE_OK;
}

/* Recovery from storage for blocks of unequal length (Section 4.3, recovery step 2): the
 * checkpoint values of the lost blocks come as packed rows - block lost[i] at element
 * row_offsets[i] of rows, as oracle_var_checkpoint_commit packs them - instead of from c.
 * norm_out, if given, receives || rows - x_S || measured before x is overwritten. */
int oracle_var_partial_recover_rows(int dtype, void *x, const void *rows, const uint64_t *row_offsets,
                                    const uint64_t *offsets, uint32_t n_blocks, const uint32_t *lost,
                                    uint32_t n_lost, oracle_norm *norm_out) {
  if (!dtype_ok(dtype) || !offsets_ok(offsets, n_blocks)) return ORACLE_ERR_ARG;
  oracle_norm zero = {0.0, 0.0, 0};
  if (norm_out) *norm_out = zero;
  if (n_lost == 0) return ORACLE_OK;
  if (!row_offsets || !rows || !x) return ORACLE_ERR_ARG;
  int rc = check_indices(lost, n_lost, n_blocks);
  if (rc) return rc;
  size_t es = elem_size(dtype);
  if (norm_out) {
    double fs = 0.0;
    int64_t is = 0;
    for (uint32_t i = 0; i < n_lost; ++i) {
      uint64_t lo = offsets[lost[i]], len = offsets[lost[i] + 1] - lo, r0 = row_offsets[i];
      for (uint64_t t = 0; t < len; ++t) {
        if (dtype == ORACLE_I32) {
          int64_t d = (int64_t)((const int32_t *)rows)[r0 + t] - (int64_t)((const int32_t *)x)[lo + t];
          is += d < 0 ? -d : d;
        } else {
          double d = load_real(c_type(dtype), rows, r0 + t) - load_real(x_type(dtype), x, lo + t);
          fs += d * d;
        }
      }
    }
    if (dtype == ORACLE_I32) {
      norm_out->isum = is;
      norm_out->sum = norm_out->norm = (double)is;
    } else {
      norm_out->sum = fs;
      norm_out->norm = sqrt(fs);
    }
  }
  for (uint32_t i = 0; i < n_lost; ++i) {
    uint64_t lo = offsets[lost[i]], len = offsets[lost[i] + 1] - lo;
    if (dtype == ORACLE_F32_BF16C) {
      for (uint64_t t = 0; t < len; ++t) ((float *)x)[lo + t] = (float)load_real(ORACLE_BF16, rows, row_offsets[i] + t);
    } else if (len) {
      memcpy((char *)x + lo * es, (const char *)rows + row_offsets[i] * es, len * es);
    }
  }
  return ORACLE_OK;
}

/* ---- document-length-scaled total variation (Section 5.1 "LDA", Appendix C) ----------
 * When the rows of a float store are distributions (a document's topic proportions), the
 * distance of row b is w_b * TV(x_b, c_b) with TV(p, q) = 1/2 * sum_j |p_j - q_j| and w_b
 * the length of document b; the size of a whole perturbation is the sum of the rows'
 * distances (a positive linear combination of total-variation norms).  weights == NULL
 * means w_b = 1 (plain total variation).  Only float stores (ORACLE_F32, ORACLE_BF16). */

static int tv_dtype_ok(int dtype) { return dtype == ORACLE_F32 || dtype == ORACLE_BF16; }

static double block_tv(int dtype, const void *x, const void *c, uint64_t lo, uint64_t hi) {
  double s = 0.0;
  for (uint64_t j = lo; j < hi; ++j) s += fabs(load_real(dtype, x, j) - load_real(dtype, c, j));
  return 0.5 * s;
}

int oracle_tv_block_scores(int dtype, const void *x, const void *c, uint64_t n_elems,
                           uint32_t block_len, const float *weights, double *scores) {
  if (!tv_dtype_ok(dtype) || block_len == 0) return ORACLE_ERR_ARG;
  if (n_elems == 0) return ORACLE_OK;
  if (!x || !c || !scores) return ORACLE_ERR_ARG;
  int64_t n_blocks = (int64_t)count_blocks(n_elems, block_len);
#pragma omp parallel for schedule(static) num_threads(g_threads)
  for (int64_t b = 0; b < n_blocks; ++b) {
    uint64_t lo, hi;
    block_range((uint64_t)b, n_elems, block_len, &lo, &hi);
    scores[b] = (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, lo, hi);
  }
  return ORACLE_OK;
}

/* sum = norm = sum over the listed blocks (all blocks if idx == NULL) of w_b * TV_b. */
int oracle_tv_perturbation_norm(int dtype, const void *x, const void *c, uint64_t n_elems,
                                uint32_t block_len, const float *weights, const uint32_t *idx,
                                uint32_t n_idx, oracle_norm *out) {
  if (!tv_dtype_ok(dtype) || block_len == 0 || !out) return ORACLE_ERR_ARG;
  uint64_t n_blocks = count_blocks(n_elems, block_len);
  int64_t m = idx ? (int64_t)n_idx : (int64_t)n_blocks;
  out->sum = out->norm = 0.0;
  out->isum = 0;
  if (m == 0) return ORACLE_OK;
  if (!x || !c) return ORACLE_ERR_ARG;
  if (idx) {
    int rc = check_indices(idx, n_idx, n_blocks);
    if (rc) return rc;
  }
  double total = 0.0;
  for (int64_t i = 0; i < m; ++i) {
    uint64_t b = idx ? idx[i] : (uint64_t)i, lo, hi;
    block_range(b, n_elems, block_len, &lo, &hi);
    total += (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, lo, hi);
  }
  out->sum = out->norm = total;
  return ORACLE_OK;
}

/* Partial recovery whose perturbation is measured in the scaled total variation. */
int oracle_tv_partial_recover(int dtype, void *x, const void *c, uint64_t n_elems,
                              uint32_t block_len, const float *weights, const uint32_t *lost,
                              uint32_t n_lost, oracle_norm *norm_out) {
  if (!tv_dtype_ok(dtype)) return ORACLE_ERR_ARG;
  if (norm_out) {
    if (n_lost == 0) {
      norm_out->sum = norm_out->norm = 0.0;
      norm_out->isum = 0;
    } else {
      int rc = oracle_tv_perturbation_norm(dtype, x, c, n_elems, block_len, weights, lost, n_lost,
                                           norm_out);
      if (rc) return rc;
    }
  }
  return oracle_partial_recover(dtype, x, c, n_elems, block_len, lost, n_lost, NULL);
}

/* The same three in the scaled total variation for blocks of unequal length (rows that are
 * distributions over vocabularies or topic sets of different sizes; Section 5.1, Appendix C):
 * block b is [offsets[b], offsets[b+1]), its distance w_b * 1/2 * sum |x - c|. */
int oracle_var_tv_block_scores(int dtype, const void *x, const void *c, const uint64_t *offsets,
                               uint32_t n_blocks, const float *weights, double *scores) {
  if (!tv_dtype_ok(dtype) || !offsets_ok(offsets, n_blocks)) return ORACLE_ERR_ARG;
  if (n_blocks == 0) return ORACLE_OK;
  if (!scores || (offsets[n_blocks] && (!x || !c))) return ORACLE_ERR_ARG;
  for (uint32_t b = 0; b < n_blocks; ++b)
    scores[b] = (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, offsets[b], offsets[b + 1]);
  return ORACLE_OK;
}

int oracle_var_tv_perturbation_norm(int dtype, const void *x, const void *c, const uint64_t *offsets,
                                    uint32_t n_blocks, const float *weights, const uint32_t *idx,
                                    uint32_t n_idx, oracle_norm *out) {
  if (!tv_dtype_ok(dtype) || !offsets_ok(offsets, n_blocks) || !out) return ORACLE_ERR_ARG;
  out->sum = out->norm = 0.0;
  out->isum = 0;
  uint32_t m = idx ? n_idx : n_blocks;
  if (idx) {
    int rc = check_indices(idx, n_idx, n_blocks);
    if (rc) return rc;
  }
  double total = 0.0;
  for (uint32_t i = 0; i < m; ++i) {
    uint32_t b = idx ? idx[i] : i;
    total += (weights ? (double)weights[b] : 1.0) * block_tv(dtype, x, c, offsets[b], offsets[b + 1]);
  }
  out->sum = out->norm = total;
  return ORACLE_OK;
}

int oracle_var_tv_partial_recover(int dtype, void *x, const void *c, const uint64_t *offsets,
                                  uint32_t n_blocks, const float *weights, const uint32_t *lost,
                                  uint32_t n_lost, oracle_norm *norm_out) {
  if (!tv_dtype_ok(dtype)) return ORACLE_ERR_ARG;
  if (norm_out) {
    oracle_norm zero = {0.0, 0.0, 0};
    *norm_out = zero;
    if (n_lost) {
      int rc = oracle_var_tv_perturbation_norm(dtype, x, c, offsets, n_blocks, weights, lost, n_lost, norm_out);
      if (rc) return rc;
    }
  }
  return oracle_var_partial_recover(dtype, x, c, offsets, n_blocks, lost, n_lost, NULL);
}

