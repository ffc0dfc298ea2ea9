/*
 * computron_test.h — entry points for tests and tuning runs of the MI355X model-swapping library.
 *
 * Nothing here is needed to serve models (computron.h is the product's boundary): these calls read
 * back device copies, replay the host-only policies (replacement, scheduling, prediction) without a
 * device so that CPU tests can compare them with their oracles, and force single mechanisms of the
 * product kernels on or off.  None of them keeps process-wide state.
 */
#ifndef COMPUTRON_TEST_H
#define COMPUTRON_TEST_H

#include "computron.h"

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default)

/* Reads the device copy of tensor `index` of a resident model into dst (host,
 * at least that tensor's nbytes); waits for the model's load first.  Tests. */
int ctn_debug_read_param(ctn_ctx* ctx, ctn_model m, int32_t index, void* dst_host, uint64_t cap);

/* Host only, no device needed: replays a sequence of uses (trace, host array
 * of n model indices below n_models) through the same replacement policy the
 * context uses (Section 3 demand paging with Section 4's LRU, byte budget)
 * and writes one event per use to out (host, n entries). */
int ctn_residency_replay(uint64_t budget_bytes, const uint64_t* sizes, int32_t n_models,
                         const int32_t* trace, uint64_t n, ctn_event* out);

/* The same for block residency: model i has n_blocks[i] blocks whose parameter
 * bytes follow each other in block_bytes (host, sum of n_blocks entries).
 * out receives one event per use (victims: models that lost blocks, least
 * recently used first), blocks_out up to cap block-level records (*n_blocks_out
 * = number produced; CTN_E_INVAL when cap is too small). */
int ctn_block_residency_replay(uint64_t budget_bytes, const int32_t* n_blocks, const uint64_t* block_bytes,
                               int32_t n_models, const int32_t* trace, uint64_t n, ctn_event* out,
                               ctn_block_event* blocks_out, uint64_t cap, uint64_t* n_blocks_out);


/* Host only: the prediction after each of n dispatches (host arrays; -1 = none). */
int ctn_predictor_replay(int32_t n_models, int32_t min_count, int32_t min_share_percent,
                         const int32_t* dispatches, uint64_t n, int32_t* predictions);
/* Host only, simulated clock: replays a trace (arrival times ascending, host
 * arrays of n entries) through the same queues, batch selection and
 * replacement policy; a batch of b requests takes t_base + b * t_per_request
 * (+ t_miss when its model was not resident) and the next one is dispatched
 * when it has finished.  batches (cap entries) and requests (n entries) are
 * host arrays. */
int ctn_engine_replay(int32_t n_models, int32_t max_batch, uint64_t budget_bytes, const uint64_t* sizes,
                      const double* arrival, const int32_t* model_of, uint64_t n, double t_base,
                      double t_per_request, double t_miss, ctn_batch_record* batches, uint64_t cap,
                      uint64_t* n_batches, uint64_t* requests);
/* The same for the two-lane engine (ctn_engine_dispatch's rule on a simulated
 * clock: each lane runs one batch at a time, a miss occupies lane 1 for
 * t_base + b * t_per_request + t_miss); batches[i].reserved holds the lane. */
int ctn_engine_replay_async(int32_t n_models, int32_t max_batch, uint64_t budget_bytes, const uint64_t* sizes,
                            const double* arrival, const int32_t* model_of, uint64_t n, double t_base,
                            double t_per_request, double t_miss, ctn_batch_record* batches, uint64_t cap,
                            uint64_t* n_batches, uint64_t* requests);


/* Test and tuning hook of one context: forces tile configuration cfg on every product of that context's
 * ctn_infer; -1 restores the library's choice.  Other contexts and the ctn_op_* entry points are not affected.
 *   0        128x128x64 tiles, filled straight from global memory into LDS when K is a multiple of 64
 *   1..8, 11..13  the other register-staged tile shapes
 *   9, 10    the streaming kernels for M <= 64 (ignored for larger M)
 *   14, 15   split-K over 64x64 / 32x128 tiles where a workspace is given
 *   16       the row-contiguous streaming kernel for M <= 16 (ignored for larger M)
 *   17       128x128x64 tiles always staged through registers
 * Switches that force no tile (all default on; 100..107 change no result):
 *   100 / 101  direct global -> LDS fills off / on
 *   102 / 103  the register-staged tiles' second stage of loads in flight off / on (where K is a multiple
 *              of the tile's K step)
 *   104 / 105  off / on: a K-sliced row-parallel product inside ctn_infer leaves the sum of its slices to the
 *              LayerNorm that follows
 *   106 / 107  off / on: the second pass of a K-sliced product reads four columns per thread with every
 *              slice in flight
 *   108 / 109  off / on: where the last round of 128x128 tiles would fill at most half of the chip, its columns
 *              are computed in K slices by a second launch (a workspace is needed; the order of the fp32
 *              additions in those columns differs from the one-launch product, nothing else)
 * CTN_E_INVAL for any other value. */
int ctn_debug_gemm_tile(ctn_ctx* ctx, int32_t cfg);
/* ctn_op_gemm_ws under an explicit list of the switches above (hooks: host array of n_hooks values, applied
 * in order to a fresh set of defaults that lives for this call only).  CTN_E_INVAL for an unknown value. */
int ctn_test_op_gemm(const void* A_f16, const void* W_f16, const void* bias_f16, void* out, int32_t M, int32_t N,
                     int32_t K, int32_t epilogue, void* workspace, uint64_t workspace_bytes, const int32_t* hooks,
                     int32_t n_hooks, void* stream);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif
