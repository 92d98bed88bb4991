/*
 * scar.h - C ABI of the checkpoint hot path of SCAR (Self-Correcting Algorithm
 * Recovery; "Fault Tolerance in Iterative-Convergent Machine Learning", Sections 4.1-4.3)
 * for one AMD MI355X (gfx950).
 *
 * Vocabulary (the paper's):
 *   x   live model parameters;
 *   c   the running checkpoint (the paper's z): the in-memory cache of what was last
 *       saved for every parameter, a mix of ages (Section 4.2, Section 4.3);
 *   block   one "parameter" in the sense of the checkpoint protocol: the unit that is
 *       scored, saved and lost as a whole - a matrix row, a factor row, a row of a count
 *       table, a shard of a tensor (Section 5.1).  x and c are cut identically into
 *       n_blocks = ceil(n_elems / block_len) blocks of block_len consecutive elements;
 *       the last block may be short;
 *   K   the blocks chosen for a partial checkpoint;  S  the blocks lost in a failure.
 *
 * One checkpoint-and-recovery cycle is
 *   scar_block_scores -> scar_select_topk -> scar_checkpoint_commit      (Section 4.3,
 *                                                     checkpoint steps 1, 3 and 4)
 *   scar_partial_recover (with the norm)  /  scar_perturbation_norm      (Section 4.1,
 *                                                     Appendix A.3)
 *
 * Conventions for every call
 *   - Every data pointer (x, c, scores, idx, out_idx, staging, norm_out, mask, workspace)
 *     is DEVICE memory owned by the caller.  The library allocates nothing and keeps no
 *     state between calls, with two exceptions that are fixed arrays inside its code object
 *     (one copy per GPU, nothing to free): the scratch of scar_select_topk_static and the
 *     piece sums of scar_block_scores on a few very long blocks; calls that use the same one
 *     must not overlap on one GPU.  scar_layout and scalar arguments are host values.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call
 *     validates its arguments on the host, enqueues its kernels on `stream` and returns;
 *     it never synchronises.  Results are in device memory once the stream reaches them.
 *   - Return value: SCAR_OK (0) or a negative scar_status.  SCAR_ERR_INVALID_ARG,
 *     SCAR_ERR_WORKSPACE and SCAR_ERR_UNSUPPORTED are found on the host before anything is
 *     enqueued.  SCAR_ERR_DEVICE is the status HIP returned for one of this call's own
 *     launches (the thread's HIP error state is neither read nor cleared, so an error left by
 *     the caller's earlier work is not reported here); launches of the call that came before
 *     the failed one have been enqueued, none after it.  Nothing throws or aborts.
 *   - x and c must not overlap.  x, c and staging must be aligned to the element size;
 *     scores / out_idx / idx to their element type; workspace to 256 bytes.  When x and c
 *     are 16-byte aligned and block_len * element size is a multiple of 16 the kernels
 *     use 16-byte accesses throughout (fastest).  Otherwise every row is walked as a few
 *     leading elements, a 16-byte body and a tail, which needs x and c at the same offset
 *     within their 16-byte lines; if they are not, rows are walked element by element
 *     (SCAR_F32_BF16C: 16 bytes of x against 8 bytes of c; the two addresses, counted in
 *     elements, must agree modulo 4).  Copies and integer results are identical in every
 *     case, float sums up to the order of the additions.
 *   - Index lists (idx, lost_idx) hold block numbers < n_blocks without repeats, in any
 *     order (ascending is fastest).  This is not checked on the host (the lists live in
 *     device memory); on the device an entry >= n_blocks is skipped, and a repeated
 *     entry is counted twice by the norm.
 *   - Calls that share a workspace must be ordered (same stream, or by events).
 *   - n_elems == 0, k == 0, n_idx == 0 and n_lost == 0 are valid and do nothing
 *     (norm_out, if given, is still written: all zero).
 */
#ifndef SCAR_H_
#define SCAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of x and c. */
typedef enum {
  SCAR_F32 = 0,  /* IEEE binary32 */
  SCAR_BF16 = 1, /* bfloat16 (upper 16 bits of a binary32), 2 bytes per element */
  SCAR_I32 = 2,  /* signed 32-bit counts (e.g. topic-count tables) */
  SCAR_F32_BF16C = 3 /* reduced-precision checkpoint (Example 2.1): x is binary32, c is
                        bfloat16.  Scores and norms use c widened exactly; a commit stores x
                        rounded to nearest even (so a freshly saved block keeps a rounding
                        distance of at most 2^-8 |x| per element); recovery widens c into x.
                        staging rows are bfloat16. */
} scar_dtype;

/* Element type of a score array. */
typedef enum {
  SCAR_SCORE_F32 = 0, /* float[n_blocks]: squared Euclidean distances (F32 / BF16 stores) */
  SCAR_SCORE_I64 = 1  /* int64_t[n_blocks]: L1 distances (I32 stores) */
} scar_score_type;

typedef enum {
  SCAR_OK = 0,
  SCAR_ERR_INVALID_ARG = -1, /* NULL where data is required, block_len == 0, bad enum,
                                k > n_blocks, n_blocks > SCAR_MAX_BLOCKS, misaligned pointer */
  SCAR_ERR_WORKSPACE = -2,   /* workspace NULL, misaligned or smaller than scar_workspace_bytes */
  SCAR_ERR_DEVICE = -3,      /* HIP reported an error when a kernel was enqueued */
  /* -4 is SCAR_ERR_IO of scar_store.h */
  SCAR_ERR_UNSUPPORTED = -5  /* every argument is valid, but this combination of store type
                                and call is not built (the total-variation calls on
                                SCAR_I32 or SCAR_F32_BF16C stores) */
} scar_status;

#define SCAR_MAX_BLOCKS 0x7fffffffu

/* How x and c are cut into blocks. */
typedef struct {
  int32_t dtype;      /* scar_dtype */
  uint32_t block_len; /* elements per block, >= 1 */
  uint64_t n_elems;   /* total elements in x (and in c); n_blocks <= SCAR_MAX_BLOCKS */
} scar_layout;

/* Size of a perturbation.  Float stores: sum = sum of (c_j - x_j)^2 over the blocks
 * asked for, norm = sqrt(sum) (the Euclidean norm of Appendix A.3), isum = 0.
 * I32 stores: isum = sum of |c_j - x_j| (exact), sum = norm = (double)isum. */
typedef struct {
  double sum;
  double norm;
  int64_t isum;
} scar_norm;

/* Number of blocks of a layout; 0 if the layout is invalid. */
uint64_t scar_n_blocks(const scar_layout* layout);

/* Bytes of device scratch that any call on a store of up to n_blocks blocks needs.
 * Host-only arithmetic; never fails (returns 0 for n_blocks > SCAR_MAX_BLOCKS). */
size_t scar_workspace_bytes(uint64_t n_blocks);

/* Checkpoint step 1 (Section 4.3): the distance of every block of x from its value in
 * the running checkpoint c.
 *   F32 / BF16: scores = float[n_blocks], s_b = sum_j (x_j - c_j)^2 over block b
 *               (the square of the Euclidean distance used in Appendix A; the order of
 *               blocks is the same with or without the square root); bfloat16 values are
 *               widened exactly and accumulated in float32/float64.
 *   I32:        scores = int64_t[n_blocks], s_b = sum_j |x_j - c_j|, exact (for a row of
 *               topic counts this is twice the document-length-scaled total variation of
 *               Appendix C).
 * Reads x and c once; writes scores.  Stores of at most 16,384 blocks of 64 KiB or more (a
 * tensor cut into a few large shards) are scored in pieces by many workgroups per block; the
 * pieces' sums wait in a fixed 2 MiB array inside the library (this call takes no workspace),
 * so two calls of that kind must not overlap on one GPU.  The copy calls below hand long rows
 * out in 4 KiB pieces. */
int scar_block_scores(const scar_layout* layout, const void* x, const void* c, void* scores,
                      void* stream);

/* The same scores for the listed blocks only: scores[b] is recomputed for every b in idx
 * (device memory, entries >= n_blocks are skipped) and all other entries of scores are left
 * as they are.  For trainers that know which rows an iteration touched (sparse updates, as in
 * matrix factorisation or LDA): between two checkpoints only those rows can have moved, so
 * rescoring them - and setting the score of a block to 0 when it is saved, which scoring it
 * after the commit does - keeps `scores` equal to what the full scan would give, at a
 * fraction of the traffic: the values are bit for bit those of scar_block_scores on the same
 * data, for every store type.  (An economy on top of the paper's protocol, which looks at
 * every parameter at every checkpoint.) */
int scar_block_scores_rows(const scar_layout* layout, const void* x, const void* c,
                           const uint32_t* idx, uint32_t n_idx, void* scores, void* stream);

/* Checkpoint step 3 (Section 4.3): the k blocks with the largest scores, i.e. those that
 * moved farthest from their last saved value - the priority rule of Section 4.2.  The order
 * is total: larger score first, equal scores to the lower
 * block index; NaN ranks above every number and -0 equals +0.  out_idx receives the k
 * chosen block indices in ascending order.  scores is not modified.
 *   score_type: SCAR_SCORE_F32 (float scores) or SCAR_SCORE_I64 (int64_t scores). */
int scar_select_topk(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                     uint32_t* out_idx, void* workspace, size_t workspace_bytes, void* stream);

/* scar_select_topk for 64-bit integer scores with a known upper bound.  A caller that scores
 * an int32 store knows one without looking at the data: an L1 distance over block_len
 * elements is at most block_len * (2^32 - 1).  The selection looks at the keys one 11-bit
 * digit at a time, most significant first; the digits above the bound are the same in every
 * key, and each pass not needed to find that out is a kernel launch saved (bound < 2^44:
 * four passes instead of six; < 2^33: three; < 2^22: two).
 *   score_max: every score is taken into [0, score_max]: a negative score counts as 0, a
 *              larger one as score_max (so a wrong bound costs order among the offenders, no
 *              more).  score_max >= 2^55 needs all six passes.  SCAR_SCORE_F32 scores
 *              ignore the bound: exactly scar_select_topk. */
int scar_select_topk_bounded(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                             uint64_t score_max, uint32_t* out_idx, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Testing aid.  The ordered write of scar_select_topk, scar_select_random and
 * scar_mask_to_indices is a chained scan: a workgroup waits for the counts of the tiles before
 * its own for at most `polls` polls (about a microsecond each; default 65,536) and then counts
 * those tiles itself, which always ends.  0 forces that path.  Process-wide, host-side; not
 * to be changed while calls are being made on other threads. */
void scar_set_lookback_spin_limit(uint32_t polls);

/* Testing aid.  The ordered write gives every workgroup one tile of 2,048 keys up to 2,048
 * tiles and a span of consecutive tiles beyond (longer key arrays), whose first 32 tiles are
 * placed from classes kept while counting and whose further tiles are read again.  A smaller
 * number of workgroups makes short key arrays take those paths: `groups` in [1, 2048]; 0 or a
 * larger value restores the default.  Results never depend on it.  Process-wide, host-side;
 * not to be changed while calls are being made on other threads. */
void scar_set_compaction_groups(uint32_t groups);

/* scar_select_topk for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result (index for index) as scar_select_topk, but the scratch is a fixed
 * array inside the library's code object - about 641 KiB on every GPU the library runs on,
 * held until the process ends - so the call allocates nothing, directly or indirectly.
 *   n_blocks > SCAR_STATIC_MAX_BLOCKS: SCAR_ERR_WORKSPACE, nothing enqueued.
 *   The first call on a device looks up the array's address on that device (one runtime
 *   query, no allocation; make it before a capture starts); it returns SCAR_ERR_DEVICE if
 *   that fails.
 *   All calls on one GPU share the one array, and it keeps the last call's contents; every
 *   call clears what it needs with a kernel of its own.  Calls that overlap on one GPU (two
 *   streams, two threads) race on it: order them, or use scar_select_topk with a workspace
 *   each. */
#define SCAR_STATIC_MAX_BLOCKS (1u << 24)
int scar_select_topk_static(int32_t score_type, const void* scores, uint32_t n_blocks, uint32_t k,
                            uint32_t* out_idx, void* stream);

/* Checkpoint step 4, the part on the critical path (Section 4.3): update the in-memory
 * checkpoint, c_b <- x_b for the n_idx blocks in idx.  If staging is not NULL, row i of
 * staging (block_len elements per row, packed) also receives block idx[i]: the bytes a
 * background writer would send to persistent storage.  x is not modified; blocks of c
 * outside idx are not touched. */
int scar_checkpoint_commit(const scar_layout* layout, const void* x, void* c,
                           const uint32_t* idx, uint32_t n_idx, void* staging, void* stream);

/* Partial recovery (Section 4.1): x_b <- c_b for the n_lost lost blocks only; every
 * other block of x keeps its value and c is not modified.  If norm_out is not NULL it
 * receives, from the same pass, the size of the perturbation this recovery causes,
 * ||c_S - x_S|| measured on x as it was before being overwritten (Appendix A.3).
 * workspace may be NULL when norm_out is NULL. */
int scar_partial_recover(const scar_layout* layout, void* x, const void* c,
                         const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Size of the perturbation a recovery of the blocks in idx would cause, ||c_S - x_S||
 * (Appendix A.3; the quantity the iteration-cost bound of Theorem 3.1 grows with),
 * without changing anything.  idx == NULL means every block: ||c - x||, the
 * perturbation of a traditional full recovery (n_idx is then ignored). */
int scar_perturbation_norm(const scar_layout* layout, const void* x, const void* c,
                           const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Convenience for callers that hold the lost set as a mask (one byte per block,
 * non-zero = lost; Section 4.1's random partitions): out_idx receives the ascending
 * indices of the non-zero bytes (room for n_blocks entries), *out_count how many. */
int scar_mask_to_indices(const uint8_t* mask, uint32_t n_blocks, uint32_t* out_idx,
                         uint32_t* out_count, void* workspace, size_t workspace_bytes,
                         void* stream);

/* A debugging aid for the one precondition on index lists that no call checks: counts
 * (DEVICE, two uint32) receives how many entries of idx are >= n_blocks (the calls skip
 * those) and how many repeat an earlier entry (the norm would count such a block twice).
 * workspace: scar_check_workspace_bytes(n_blocks) bytes of device scratch (a bit per block),
 * 256-byte aligned.  Enqueues two small kernels; the list is not modified. */
size_t scar_check_workspace_bytes(uint64_t n_blocks);
int scar_check_indices(const uint32_t* idx, uint32_t n_idx, uint32_t n_blocks, uint32_t* counts,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The comparison strategies of Section 5.4 for choosing K; their output feeds
 * scar_checkpoint_commit exactly like scar_select_topk's.
 *
 * "round": blocks are saved in a round-robin manner.  out_idx receives the k blocks
 * cursor, cursor+1, ... (taken modulo n_blocks) in ascending order; the caller advances
 * cursor by k per checkpoint. */
int scar_select_round(uint32_t n_blocks, uint32_t k, uint64_t cursor, uint32_t* out_idx,
                      void* stream);

/* "random": blocks are saved uniformly at random.  Block b draws the 32-bit number
 * Philox4x32-10(counter = (b, 0, draw_lo, draw_hi), key = (seed_lo, seed_hi))[0]
 * (Salmon et al., SC'11); the k blocks with the largest numbers are chosen, equal numbers
 * to the lower index - a uniformly random k-subset up to ties between 32-bit draws.
 * `draw` numbers the checkpoint, so each checkpoint of a run uses fresh numbers.
 * out_idx ascending.  Same (seed, draw, n_blocks, k) => same result on every run. */
int scar_select_random(uint32_t n_blocks, uint32_t k, uint64_t seed, uint64_t draw,
                       uint32_t* out_idx, void* workspace, size_t workspace_bytes, void* stream);

/* ---- Blocks of unequal length ---------------------------------------------------------
 * Section 5.1's "by-layer" partitioning makes every weight or bias tensor of a network one
 * parameter, so blocks differ in size by orders of magnitude.  Block b is the element
 * range [offsets[b], offsets[b+1]); empty blocks are allowed (score 0).
 * The calls below mirror the five above (scar_select_topk, _round and _random work on
 * any score array and serve both layouts).  Every store type is served, SCAR_F32_BF16C
 * included (staging rows and packed rows are then bfloat16, like c).
 * All of them need a workspace of scar_var_workspace_bytes(n_blocks) bytes. */
typedef struct {
  int32_t dtype;           /* scar_dtype */
  uint32_t n_blocks;       /* <= SCAR_MAX_BLOCKS */
  uint64_t n_elems;        /* total elements of x (and c); must equal offsets[n_blocks] */
  const uint64_t* offsets; /* DEVICE memory: n_blocks + 1 non-decreasing element offsets,
                              offsets[0] = 0.  Not checked on the host; kernels never read or
                              write outside [0, n_elems) whatever the offsets hold. */
} scar_var_layout;

size_t scar_var_workspace_bytes(uint64_t n_blocks);

/* As scar_block_scores: scores = float[n_blocks] or int64_t[n_blocks]. */
int scar_var_block_scores(const scar_var_layout* layout, const void* x, const void* c, void* scores,
                          void* workspace, size_t workspace_bytes, void* stream);

/* As scar_checkpoint_commit (without staging). */
int scar_var_checkpoint_commit(const scar_var_layout* layout, const void* x, void* c,
                               const uint32_t* idx, uint32_t n_idx, void* workspace,
                               size_t workspace_bytes, void* stream);

/* As scar_checkpoint_commit with staging rows (Section 4.3, checkpoint step 4): the listed
 * blocks are also packed into `staging` one after the other in the order of the list - the
 * bytes a background writer sends to persistent storage - and staging_offsets (DEVICE,
 * n_idx + 1 entries) receives where: block idx[i] starts at element staging_offsets[i] of
 * staging, staging_offsets[n_idx] is the total (the lengths of the listed blocks added up; an
 * empty block takes no room).  staging must have room for that total; its elements have c's
 * type.  The offsets are computed on the device; nothing comes back to the host. */
int scar_var_checkpoint_commit_staged(const scar_var_layout* layout, const void* x, void* c,
                                      const uint32_t* idx, uint32_t n_idx, void* staging,
                                      uint64_t* staging_offsets, void* workspace,
                                      size_t workspace_bytes, void* stream);

/* As scar_partial_recover; the workspace is always required. */
int scar_var_partial_recover(const scar_var_layout* layout, void* x, const void* c,
                             const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/* scar_var_partial_recover with the lost blocks' checkpoint values taken from packed rows
 * (Section 4.3, recovery step 2: re-loaded from storage) instead of from the in-memory
 * checkpoint: block lost_idx[i] is read from element row_offsets[i] of rows (DEVICE arrays;
 * the layout scar_var_checkpoint_commit_staged writes and scar_var_store_load returns), and
 * norm_out, if given, receives || rows - x_S || measured before the overwrite. */
int scar_var_partial_recover_rows(const scar_var_layout* layout, void* x, const void* rows,
                                  const uint64_t* row_offsets, const uint32_t* lost_idx,
                                  uint32_t n_lost, scar_norm* norm_out, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* As scar_perturbation_norm (idx == NULL: every block). */
int scar_var_perturbation_norm(const scar_var_layout* layout, const void* x, const void* c,
                               const uint32_t* idx, uint32_t n_idx, scar_norm* norm_out,
                               void* workspace, size_t workspace_bytes, void* stream);

/* ---- document-length-scaled total variation (Section 5.1 "LDA", Appendix C) -----------
 * When the rows of a float store are distributions (a document's topic proportions), the
 * paper measures distances in total variation, each row scaled by the length of its
 * document: distance of block b = w_b * 1/2 * sum_j |x_j - c_j|, and the size of a
 * perturbation is the sum of its rows' distances (a positive combination of total-variation
 * norms), not a root of squares.  The three calls below are scar_block_scores,
 * scar_partial_recover and scar_perturbation_norm in that norm; selection and commit do not
 * depend on the norm and are shared.
 *   layout->dtype: SCAR_F32 or SCAR_BF16 (other store types: SCAR_ERR_UNSUPPORTED).
 *   weights: float[n_blocks] in DEVICE memory (document lengths, > 0 by the caller's care),
 *            or NULL for w_b = 1 (plain total variation).
 *   scores:  float[n_blocks].
 *   norm_out: sum = norm = the scaled total variation over the listed blocks, isum = 0.
 * A table of integer topic counts needs none of this: with SCAR_I32 the plain calls score the
 * L1 distance of the counts, which is exactly twice this norm when row totals are unchanged. */
int scar_tv_block_scores(const scar_layout* layout, const void* x, const void* c,
                         const float* weights, float* scores, void* stream);

int scar_tv_partial_recover(const scar_layout* layout, void* x, const void* c, const float* weights,
                            const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                            void* workspace, size_t workspace_bytes, void* stream);

int scar_tv_perturbation_norm(const scar_layout* layout, const void* x, const void* c,
                              const float* weights, const uint32_t* idx, uint32_t n_idx,
                              scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                              void* stream);

/* The same three for blocks of unequal length (rows that are distributions over sets of
 * different sizes): scar_var_block_scores, scar_var_partial_recover and
 * scar_var_perturbation_norm in the scaled total variation.  weights: float[n_blocks] in DEVICE
 * memory or NULL.  SCAR_F32 and SCAR_BF16 stores (others: SCAR_ERR_UNSUPPORTED); the workspace is
 * that of the scar_var_* calls. */
int scar_var_tv_block_scores(const scar_var_layout* layout, const void* x, const void* c,
                             const float* weights, float* scores, void* workspace,
                             size_t workspace_bytes, void* stream);

int scar_var_tv_partial_recover(const scar_var_layout* layout, void* x, const void* c,
                                const float* weights, const uint32_t* lost_idx, uint32_t n_lost,
                                scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                void* stream);

int scar_var_tv_perturbation_norm(const scar_var_layout* layout, const void* x, const void* c,
                                  const float* weights, const uint32_t* idx, uint32_t n_idx,
                                  scar_norm* norm_out, void* workspace, size_t workspace_bytes,
                                  void* stream);

/* Static, never NULL. */
const char* scar_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SCAR_H_ */
