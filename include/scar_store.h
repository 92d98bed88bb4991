/*
 * scar_store.h - the persistent-storage leg of SCAR's checkpoint protocol (Section 4.3,
 * checkpoint step 4 and recovery step 2): the blocks chosen for a partial checkpoint go to
 * the in-memory checkpoint first and from there, in the background and off the critical
 * path, to persistent storage; after a failure the lost blocks are read back from the
 * running checkpoint that storage holds.
 *
 * A store file holds the running checkpoint of one parameter store with fixed-length
 * blocks: a 4,096-byte header, then block b at byte 4096 + b * row_bytes, where row_bytes =
 * block_len * (element size of the checkpoint c: 4 for SCAR_F32 / SCAR_I32, 2 for SCAR_BF16
 * and SCAR_F32_BF16C).  Blocks are overwritten in place, so the file is always a mix of ages
 * like the in-memory checkpoint (Section 4.2).  Header (little endian): bytes 0-7 the ASCII
 * magic "SCARSTO1", then int32 dtype, uint32 block_len, uint64 n_elems, uint32 row_bytes.
 *
 * The object owns two pinned host buffers (each max_rows rows plus max_rows indices), two
 * HIP events and one writer thread; these are allocated when it is created, never in
 * scar_store_save_async / scar_store_load.  Functions of one scar_store must not be called
 * concurrently from several host threads.
 */
#ifndef SCAR_STORE_H_
#define SCAR_STORE_H_

#include "scar.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct scar_store scar_store;

#define SCAR_ERR_IO (-4) /* the file could not be created, opened, read or written */

/* Creates (or truncates) `path` for a store of `layout`, all blocks zero, and opens it.
 * max_rows: the largest number of rows one save or load will carry.  The running checkpoint
 * starts as x(0) (Section 4.2): save all blocks once before relying on the file. */
int scar_store_create(const char* path, const scar_layout* layout, uint32_t max_rows,
                      scar_store** out);

/* Opens an existing store file of fixed-length blocks; *layout_out receives its layout. */
int scar_store_open(const char* path, uint32_t max_rows, scar_layout* layout_out, scar_store** out);

/* Background save of one partial checkpoint.  staging (DEVICE): the packed rows written by
 * scar_checkpoint_commit's staging output, row i = block idx[i]; idx (DEVICE): the n_idx
 * block numbers.  The call enqueues two device-to-host copies on `stream` into a pinned
 * buffer and returns; the writer thread waits for the copies and then writes every row at
 * its block's place in the file.  staging and idx may be reused once `stream` has passed the
 * copies.  If both pinned buffers are still being written the call blocks until one is free.
 * n_idx > max_rows is SCAR_ERR_INVALID_ARG. */
int scar_store_save_async(scar_store* store, const void* staging, const uint32_t* idx, uint32_t n_idx,
                          void* stream);

/* Blocks until every save handed in so far is in the file (written and flushed with fsync);
 * returns SCAR_ERR_IO if any of them failed since the last call. */
int scar_store_wait(scar_store* store);

/* Recovery from storage: reads the blocks idx_host[0..n_idx) (HOST array) from the file and
 * copies them to rows (DEVICE, packed: row i = block idx_host[i], block_len elements per
 * row) on `stream`; returns after the copy has completed.  Pending saves are waited for
 * first.  Feed rows to scar_partial_recover_rows. */
int scar_store_load(scar_store* store, const uint32_t* idx_host, uint32_t n_idx, void* rows,
                    void* stream);

/* ---- stores whose blocks differ in length (Section 5.1, by-layer partitioning) -------------
 * The same object and the same writer thread for a scar_var_layout store.  File: a 4,096-byte
 * header (ASCII magic "SCARSTV1", int32 dtype, uint32 n_blocks, uint64 n_elems, uint64
 * data_offset), the n_blocks + 1 uint64 element offsets at byte 4,096, then block b at byte
 * data_offset + offsets[b] * element size (data_offset = the next multiple of 4,096 after the
 * offsets).  scar_store_wait and scar_store_close serve both kinds of store; the calls above
 * refuse a store of this kind and the calls below one of the other (SCAR_ERR_INVALID_ARG).
 *
 * offsets_host: HOST array, n_blocks + 1 non-decreasing element offsets, offsets[0] = 0.
 * max_rows: most blocks per save or load; max_elems: most elements per save or load (the
 * size of the two pinned buffers).  Every store type; elements in the file have c's type. */
int scar_var_store_create(const char* path, int32_t dtype, uint32_t n_blocks,
                          const uint64_t* offsets_host, uint32_t max_rows, uint64_t max_elems,
                          scar_store** out);

/* Background save of the rows scar_var_checkpoint_commit_staged packed: staging (DEVICE) holds
 * the blocks idx[0..n_idx) (DEVICE) one after the other.  Which blocks were chosen, and so how
 * many elements that is, is known only on the device: the caller says how many elements to
 * transfer - staging_elems, at least the listed blocks' total, the capacity of the staging
 * buffer will always do - and the writer thread, which knows the offsets, finds the rows in
 * them.  Fewer elements than the list needs make the save fail (reported by scar_store_wait). */
int scar_var_store_save_async(scar_store* store, const void* staging, uint64_t staging_elems,
                              const uint32_t* idx, uint32_t n_idx, void* stream);

/* Recovery from storage: reads the blocks idx_host[0..n_idx) (HOST) from the file into rows
 * (DEVICE, packed in list order) and writes where each one starts to row_offsets (DEVICE,
 * n_idx + 1 element offsets; the last is the total); returns after the copies have completed.
 * Feed both to scar_var_partial_recover_rows. */
int scar_var_store_load(scar_store* store, const uint32_t* idx_host, uint32_t n_idx, void* rows,
                        uint64_t* row_offsets, void* stream);

/* Waits for pending saves, stops the writer thread, closes the file, frees everything. */
int scar_store_close(scar_store* store);

/* scar_partial_recover with the lost blocks' checkpoint values taken from packed rows (row
 * i = block lost_idx[i], e.g. as loaded by scar_store_load) instead of from the in-memory
 * checkpoint: x_b <- rows[i], and norm_out, if given, receives ||rows - x_S|| measured
 * before the overwrite.  For SCAR_F32_BF16C the rows are bfloat16. */
int scar_partial_recover_rows(const scar_layout* layout, void* x, const void* rows,
                              const uint32_t* lost_idx, uint32_t n_lost, scar_norm* norm_out,
                              void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SCAR_STORE_H_ */
