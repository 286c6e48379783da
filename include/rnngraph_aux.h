/*
 * rnngraph_aux -- measurement and inspection aids of librnngraph.so.  Not part of the forward /
 * BPTT boundary (rnngraph.h): benchmarks and tests use these to time kernel classes, to see which
 * build of the recurrent-step kernel served a recurrent node, and to read the control words.
 */
#ifndef RNNGRAPH_AUX_H
#define RNNGRAPH_AUX_H

#include "rnngraph.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Which build of the persistent recurrent-step kernel (Section 3.1, sequential part) ran the step
 * loop of the recurrent node that contains `node` at its last launch in the given direction
 * (backward = 0 / 1); RNN_BUILD_NONE if the node is in no recurrent node or nothing ran yet.
 * RNN_BUILD_CHAIN is or-ed in when stacked recurrent nodes shared one launch (RNN_BUILD_HELPERS too if
 * that launch had helper members). */
enum {
    RNN_BUILD_NONE = 0,
    RNN_BUILD_WAVE = 1,         /* run-time specialised, weights in registers (few streams) */
    RNN_BUILD_MATRIX = 2,       /* run-time specialised, matrix cores, weights in LDS (many streams) */
    RNN_BUILD_MATRIX_2D = 3,    /* the same with the two-dimensional split of wide layers */
    RNN_BUILD_LDS = 4,          /* run-time specialised, weights in LDS, several phases per step */
    RNN_BUILD_INTERPRETED = 5,  /* ahead-of-time build that interprets the step programs */
    RNN_BUILD_PER_FRAME = 6,    /* no persistent kernel: launches per frame */
    RNN_BUILD_STREAMING = 7,    /* run-time specialised, weights streamed from memory every step
                                   (layers too wide to keep on chip) */
    RNN_BUILD_CHAIN = 16,
    RNN_BUILD_HELPERS = 32      /* or-ed in with RNN_BUILD_CHAIN: the launch had helper members, which took the
                                   products of the connections between the stacked nodes (backward, many streams) */
};
int rnn_step_build(const rnn_graph* g, int32_t node, int32_t backward, int32_t* build);

/* Synchronises the device and copies the first `bytes` (at most 1024) of the workspace's
 * control-word area to HOST memory: E_total (double) at byte 0, the kernels' error flag (uint32)
 * at byte 16, and, if the step kernels were built with RNNG_STEP_TRACE=1 in the environment, 64
 * cycle stamps (uint64) at byte 80. */
int rnn_debug_read_control(rnn_graph* g, void* out, int32_t bytes);

/* Kernel-class timing for benchmarks: HIP events are recorded on the call's stream around the
 * launches of every class whose bit is set in class_mask (0 switches timing off; it is off by
 * default and costs nothing then).  rnn_profile_read waits for the recorded events, stores the
 * summed duration in milliseconds and the number of kernel launches of that class since the
 * last read (HOST pointers, either may be NULL) and resets both. */
enum {
    RNN_PROF_STEP_FWD = 0,   /* recurrent-node forward step kernels (Section 3.1 sequential part) */
    RNN_PROF_STEP_BWD = 1,   /* recurrent-node backward step kernels */
    RNN_PROF_GEMM_FWD = 2,   /* batched forward edge products */
    RNN_PROF_GEMM_BWD = 3,   /* batched backward edge products */
    RNN_PROF_GEMM_GRAD = 4,  /* weight-gradient GEMMs */
    RNN_PROF_OTHER = 5,      /* element-wise programs over all frames, softmax, reductions, fills */
    RNN_PROF_CLASSES = 6
};
int rnn_profile_enable(rnn_graph* g, int32_t class_mask);
int rnn_profile_read(rnn_graph* g, int32_t cls, double* ms, int64_t* launches);

/* What the plan that ran last worked on, for benchmarks.  flops[0..4]: multiply-adds x 2 of one
 * window of T frames x N streams in the batched forward products, the batched backward products,
 * the weight-gradient products, the forward step loops and the backward step loops.
 * step_bytes[0..1]: weight bytes (full matrices and diagonal vectors, 4 bytes each) that the
 * forward / backward step loops touch per time step.  Connections between stacked recurrent nodes
 * that shared a step launch were stepped, not batched: they count under the step loops.
 * HOST int64 arrays. */
int rnn_plan_work(const rnn_graph* g, int32_t T, int32_t N, int64_t* flops, int64_t* step_bytes);

#ifdef __cplusplus
}
#endif
#endif /* RNNGRAPH_AUX_H */
