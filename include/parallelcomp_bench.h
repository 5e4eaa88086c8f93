/*
 * parallelcomp_bench.h - measurement aids of the ParallelComp library (not part of the method's
 * boundary: nothing here computes a step of the path).  Used by the benchmark only.
 */
#ifndef PARALLELCOMP_BENCH_H
#define PARALLELCOMP_BENCH_H

#include <stddef.h>
#include <stdint.h>
#include "parallelcomp.h"   /* pc_status */

#ifdef __cplusplus
extern "C" {
#endif

/* ---- per-kernel timing (measurement aid; off by default) ------------------------------------
 * While enabled, every kernel the library launches is bracketed by a pair of HIP events recorded
 * on the stream of the call.  pc_profile_begin resets the record list (at most 4096 records are
 * kept, later launches are not recorded); pc_profile_end stops recording; pc_profile_get waits
 * for record i and returns its kernel id (pc_kernel_id) and elapsed milliseconds.
 * Not thread-safe; meant for one benchmarking thread. */
typedef enum pc_kernel_id {
  PC_KERNEL_ROPE_TABLE = 0, PC_KERNEL_KV_PREPASS = 1, PC_KERNEL_FLASH = 2, PC_KERNEL_SCORES_P1 = 3,
  PC_KERNEL_SCORES_P2 = 4, PC_KERNEL_CHUNK_SCORE = 5, PC_KERNEL_SELECT_CHUNKS = 6,
  PC_KERNEL_SELECT_TOKENS = 7, PC_KERNEL_GATHER = 8, PC_KERNEL_ROPE_Q = 9, PC_KERNEL_DECODE = 10,
  PC_KERNEL_MERGE = 11, PC_KERNEL_SELF_INFO = 12, PC_KERNEL_KV_APPEND = 13,
  PC_KERNEL_SCORES_LSE = 14, PC_KERNEL_KV_QUANTIZE = 15, PC_KERNEL_DECODE_FP8 = 16,
  PC_KERNEL_PREPASS_SCORES = 17,   /* scores pass 1 fused with the K/V pre-pass */
  PC_KERNEL_CHUNK_QUEUE = 18, PC_KERNEL_FP8_TO_ROWS = 19,
  PC_KERNEL_COUNT = 20
} pc_kernel_id;
int         pc_profile_begin(void);
int         pc_profile_begin_kernel(int kernel_id);   /* as pc_profile_begin, but only the launches of one
                                                        kernel are bracketed (two event records per kernel
                                                        cost about 7 us of stream time each) */
int         pc_profile_end(void);
int         pc_profile_count(void);
int         pc_profile_get(int i, int* kernel_id, float* ms);
const char* pc_kernel_name(int kernel_id);

/* ---- matrix-pipe ceiling (measurement aid) ---------------------------------------------------
 * Enqueues a kernel built around independent 32x32x16 bf16 MFMAs: n_cus workgroups of 8
 * wavefronts (two per SIMD), iters x 8 MFMAs each.  mode 0: nothing but MFMAs on constant
 * operands; mode 1: the same on random operands (more bits toggle, the power-limited clock falls);
 * mode 2: random operands plus, per MFMA, one 16-byte-per-lane LDS read feeding the A operand and
 * one softmax element on the vector ALU (exponential, add, multiply), the instruction mix of a
 * flash-attention loop at 32 queries per wavefront.  scratch (device, >= n_cus * 512 * 4 bytes)
 * receives one float per lane so the work cannot be optimised away.  *flops (host) receives the
 * MFMA floating-point operations the launch performs; the caller times the launch on its stream
 * and divides.  Returns PC_ERR_NULL / PC_ERR_SHAPE (mode outside 0..2, n_cus outside 1..4096,
 * iters outside 1..2^22) / PC_ERR_WORKSPACE / PC_ERR_HIP. */
int pc_mfma_ceiling(int mode, int n_cus, int iters, float* scratch, size_t scratch_bytes,
                    double* flops, void* stream);

/* ---- copy ceiling (measurement aid) -----------------------------------------------------------
 * Enqueues a bare copy of `bytes` bytes (device pointers, 16-byte aligned, bytes a multiple of
 * 16) with 16-byte loads and stores, four in flight per thread: mode 0 ordinary, mode 1 with the
 * non-temporal hint on both sides.  The caller times it: what a read-and-write stream sustains on
 * this machine.  PC_ERR_NULL / PC_ERR_SHAPE / PC_ERR_HIP. */
int pc_copy_ceiling(int mode, const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PARALLELCOMP_BENCH_H */
