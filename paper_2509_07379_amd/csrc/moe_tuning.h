/*
 * Internal test and tuning hook of the MoE-layer library: not part of the public interface
 * (include/moe_offload.h), exported so that the parity tests can force every kernel variant onto
 * the same inputs.  Settings belong to one context; a new context starts with every choice made
 * by shape.
 *
 *   mode 0 / 1 / 2  GEMM kernel of the gate/up GEMM / the down GEMM / (unused): 0 = by shape,
 *                   1 = 128 x 128 tiles, 6 = 256 x 256 tiles of the single-phase kernel,
 *                   12 = the persistent ping-pong kernel
 *   mode 3          K slices of the down GEMM: 0 = heuristic, else at most the heuristic's number
 *   mode 4          weight rows per wave of the per-token mat-vec kernels: 0 = by shape, 1, 2, 4
 *   mode 5          0: a one-token decode call with every expert resident waits for the gate's
 *                   result on the host like any other call; non-zero (default): it is enqueued at
 *                   once and the mat-vec launches take the k experts from the gate's id list
 *   mode 6          (not in use)
 *   mode 7          1: a one-token all-resident decode call runs the down mat-vec and the weighted
 *                   sum as two launches instead of one (the same bits either way)
 *   mode 8          tokens per expert from which a mat-vec launch may use the matrix-core kernel:
 *                   0 = default, 1 = wherever the shapes allow it, a large value = never
 *   mode 9          largest group a decode call still gives to the mat-vec launches (0 = default)
 *   mode 10         K slices (waves) per block of the matrix-core mat-vec (0 = by shape, 1..8)
 *   mode 11         how the persistent down GEMM of a prefill call cuts groups into row tiles and deals
 *                   them out: 0 = by shape (fewer than 16 experts: 1, else 2), 1 = row tiles of equal
 *                   height in a fixed order per block, 2 = full tiles plus a remainder, taken from the
 *                   per-XCD queues of the plan the grouping kernel writes, 3 = equal heights from queues
 *   mode 12         the same for the gate/up GEMM: 0 = by shape, 1 = equal heights in a fixed order,
 *                   2 = full tiles plus a remainder from queues
 */
#ifndef MOE_TUNING_H
#define MOE_TUNING_H

#include "../../include/moe_offload.h"

#ifdef __cplusplus
extern "C" {
#endif
int moe_tune(moe_ctx *ctx, int mode, int variant);

/* The nth_hip_call-th HIP runtime call that the library's host code makes on this thread from now
 * on is skipped and reported as failed (0 cancels).  Host side only: nothing wrong reaches the GPU.
 * Used to check what a layer call or a prefetch that fails midway leaves behind. */
int moe_inject_failure(int nth_hip_call);

/* Parity hook: the two work plans (gate/up GEMM, down GEMM) the last prefill call on T tokens left in
 * dev_workspace, as 2 x (3 + 9 + 65 + 128) int32: n_items, s_full, s_rem, xcd_begin[9], item_begin[65],
 * queue[128] (the queue counters as the launches left them).  Blocks until `stream` has drained. */
int moe_debug_plans(moe_ctx *ctx, const void *dev_workspace, int T, int32_t *host_out, void *stream);

/* Which GEMM kernel the launcher would pick (1, 6, 12, or 100 for the kernel that pads a ragged K)
 * for GemmMode `mode` on an A of a_rows x lda (gathered through a permutation or used in place),
 * B rows of ldb elements with the second B matrix b1_minus_b0 bytes behind the first, N output
 * columns, K, at most max_rows rows in n_groups groups.  Pure host arithmetic. */
int moe_debug_gemm_choice(int mode, int gathered, long long a_rows, int lda, int N, int ldb, int K,
                          long long b1_minus_b0, int max_rows, int n_groups);
#ifdef __cplusplus
}
#endif
#endif
