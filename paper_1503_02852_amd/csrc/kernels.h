// Launch wrappers of the HIP kernels (implemented in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "program.h"

namespace rnng {

// ---------------------------------------------------------------------------------------
// Grouped fp32 MFMA GEMM:  C[M][N] (+)= sum over pairs  A_p(M x K_p) * B_p(K_p x N)
// ---------------------------------------------------------------------------------------
constexpr int GEMM_MAX_PAIRS = 4;
constexpr int GEMM_MAX_PROBLEMS = 8;

struct GemmPair {
    const float* A;   // K-contiguous modes: element (m, k) at A[(m + a_row_off) * lda + k], zero if the
                      // shifted row falls outside [0, a_rows);  M-contiguous mode: element (m, k) at A[k * lda + m]
    const float* B;   // K-contiguous mode: element (k, n) at B[n * ldb + k];  N-contiguous: B[k * ldb + n]
    int K, lda, ldb, a_row_off, a_rows;
};
struct GemmProblem {
    float* C; int ldc, M, N, n_pairs;
    GemmPair pairs[GEMM_MAX_PAIRS];
};
struct GemmGroup {
    GemmProblem p[GEMM_MAX_PROBLEMS];
    int n_problems;
    int split_k;      // >1: K is split over blockIdx.z and results are added atomically (C must be pre-zeroed)
    int accumulate;   // 1: C += result instead of C = result (ignored when split_k > 1)
    int group_m;      // set by launch_gemm_group: tile order (see the kernel); 0: row by row, no XCD ranges
};
enum GemmMode {
    GEMM_NT = 0,   // A K-contiguous, B K-contiguous      (forward:  Y_dst = Y_src W^T)
    GEMM_NN = 1,   // A K-contiguous, B N-contiguous      (backward: dY_src = dS_dst W)
    GEMM_TN = 2    // A M-contiguous, B N-contiguous      (gradient: G = dS_dst^T Y_src)
};
hipError_t launch_gemm_group(GemmMode mode, const GemmGroup& g, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Element-wise node programs, step matrix-vector products, softmax, reductions
// ---------------------------------------------------------------------------------------
// Runs a node program for frames [t0, t1) and all streams.
hipError_t launch_node_program(const PlanView& pv, int prog_off, int max_dim, const float* weights,
                               int T, int N, int t0, int t1, hipStream_t stream);
// Matrix-vector task list for frame t (per-step launch).
hipError_t launch_step_matvec(const PlanView& pv, int mv_off, int n_tasks, int max_out, const float* weights,
                              int T, int N, int t, hipStream_t stream);
// In-place row softmax over `rows` rows of width dim.
hipError_t launch_softmax_rows(float* y, int64_t rows, int dim, hipStream_t stream);
// ds = y - onehot(target) (0 where target < 0); *loss += sum of -ln y[target].
// A target not below dim leaves its frame out and sets *flag to 3.
hipError_t launch_softmax_ce_delta(const float* y, const int32_t* targets, float* ds, double* loss, unsigned* flag,
                                   int64_t rows, int dim, hipStream_t stream);
// Squared-error output layer: ds = (y - d) f'(s) element by element (0 where d is NaN), f' from y
// for act = linear / sigmoid / tanh / rectifier; *loss += 1/2 sum (d - y)^2.
hipError_t launch_squared_error_delta(const float* y, const float* d, float* ds, double* loss, int64_t n, int act,
                                      hipStream_t stream);
// Column-sum tasks (diagonal-weight and bias gradients), atomically added into grads.
// The sums run over frames [t0, T); factors may reach back to frames before t0.
hipError_t launch_colsum(const PlanView& pv, int tasks_off, int n_tasks, int max_dim, const float* weights, float* grads,
                         int T, int N, int t0, bool one_writer, hipStream_t stream);
// Zeroes the first `rows` rows of every buffer whose flag is 1 (the history frames in front of a fresh window).
hipError_t launch_zero_history(float* const* buf_ptr, const int32_t* buf_dim, const int32_t* buf_flags, int n_bufs, int64_t rows,
                               hipStream_t stream);
hipError_t launch_fill(float* p, int64_t n, float v, hipStream_t stream);
hipError_t launch_copy(float* dst, const float* src, int64_t n, hipStream_t stream);
// dst[c][r] = src[r][c] for a row-major rows x cols matrix.
hipError_t launch_transpose(float* dst, const float* src, int rows, int cols, hipStream_t stream);
// n 32-bit words from HOST memory to DEVICE memory, carried as kernel arguments (the words are read
// when the call is made; no staging buffer, no allocation).
hipError_t launch_upload_words(uint32_t* d_dst, const uint32_t* h_src, int64_t n, hipStream_t stream);
// Writes the hardware XCD id of workgroup b (256 threads each) to out[b], b < n_blocks.
hipError_t launch_xcc_probe(unsigned* out, int n_blocks, hipStream_t stream);
// One-hot sources given as class indices [total_rows]: C[f][j] (+)= W[j][idx[f - shift_rows]] for rows
// [row0, row0 + rows), and the matching weight gradient G[j][idx[f - shift_rows]] += ds[f][j].
hipError_t launch_onehot_gather(float* C, const float* W, const int* idx, int n_dst, int n_src, int64_t row0, int64_t rows,
                                int64_t shift_rows, int64_t total_rows, bool accumulate, hipStream_t stream);
// ordered: the rows are added one after another in increasing order (one writer per element: the
// sums are the same bits from run to run), else with float atomics from many workgroups.
hipError_t launch_onehot_scatter(float* G, const float* ds, const int* idx, int n_dst, int n_src, int64_t shift_rows, int64_t total_rows,
                                 bool ordered, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Persistent recurrent-step kernel (all T steps of one recurrent node and direction)
// ---------------------------------------------------------------------------------------
struct StepLaunchPlan {
    bool ok; int G, NB, xcd_stride; size_t lds_bytes;
    int threads = 256;      // per workgroup (run-time specialised variants only)
};
// Chooses the number of workgroups for a component's step descriptor; ok = false if the
// component does not fit the kernel's limits (then the caller steps with per-frame launches).
int step_nb_for(int N);   // streams per pass of the step kernel for N streams (0: not supported)
bool plan_step_launch(const int32_t* words, int desc_off, int N, int force_G, StepLaunchPlan& out);
hipError_t launch_recurrent_steps(const PlanView& pv, const StepLaunchPlan& lp, int desc_off, const float* weights,
                                  unsigned* ctrl, int T, int N, bool backward, int spin_limit, int t_begin, int t_end,
                                  hipStream_t stream);
// Fills n floats with the "not yet written" bit pattern the step kernel's consumers wait on.
hipError_t launch_fill_sentinel(float* p, int64_t n, hipStream_t stream);
// The same for up to FILL_MAX_RANGES ranges with one launch (a step launch's exchanged tensors).
constexpr int FILL_MAX_RANGES = 16;
struct FillRanges { float* p[FILL_MAX_RANGES]; long long n[FILL_MAX_RANGES]; int count; };
hipError_t launch_fill_sentinel_ranges(const FillRanges& r, hipStream_t stream);

}  // namespace rnng
