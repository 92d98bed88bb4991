/*
 * scar_ceilings.h - three plain bandwidth kernels, the measured ceilings that the kernels of
 * the checkpoint path (scar.h) are compared with.  They compute nothing of the method: each
 * has the memory access shape of one step of Section 4.3's cycle with the index lists,
 * block boundaries and arithmetic taken away, written with the same access style (16-byte
 * non-temporal accesses, each XCD walking a contiguous eighth of the range) and launched in
 * the shape that was measured fastest for it.
 *
 *   scar_ceiling_read2         reads a and b                  - the shape of scar_block_scores
 *   scar_ceiling_copy          reads a, writes b              - the shape of scar_checkpoint_commit
 *   scar_ceiling_read2_write1  reads a and b, then b <- a     - the shape of scar_partial_recover
 *                                                               with the fused norm
 *
 * a, b: DEVICE memory, 16-byte aligned, `bytes` bytes each (a multiple of 16), not overlapping.
 * sink: DEVICE memory, 8 bytes; it is written only if the data happen to add up to one
 * particular value, so that the reads cannot be optimised away.  stream: hipStream_t as void*.
 * Returns 0, or -1 for a bad argument, -3 if HIP reported an error when the kernel was enqueued.
 * Nothing is allocated or synchronised.
 */
#ifndef SCAR_CEILINGS_H_
#define SCAR_CEILINGS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int scar_ceiling_read2(const void* a, const void* b, uint64_t bytes, void* sink, void* stream);
int scar_ceiling_copy(const void* a, void* b, uint64_t bytes, void* stream);
int scar_ceiling_read2_write1(const void* a, void* b, uint64_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SCAR_CEILINGS_H_ */
