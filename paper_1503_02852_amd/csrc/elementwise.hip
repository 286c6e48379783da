// Element-wise kernels: node programs over many frames (additive / multiplicative layers,
// activation functions and their derivatives: paper Section 2.1 and the delta / epsilon
// equations of Section 2.2), row softmax with the cross-entropy output delta (Section 2.2),
// column sums for diagonal-weight and bias gradients, and fills.
#include "interp.h"
#include "kernels.h"

namespace rnng {
namespace {

// One thread per (frame, stream, unit); the accumulator entries of the program (if any) are
// read from their one-frame buffers.
__global__ __launch_bounds__(256)
void node_program_kernel(PlanView pv, int prog_off, int max_dim,
                                                           const float* __restrict__ weights,
                                                           int T, int N, int t0, long long total) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long row = idx / max_dim;
    const UnitMap um{0, 1, (int)(idx - row * max_dim)};
    const int t = t0 + (int)(row / N), n = (int)(row % N);
    const ProgramView pg(pv.words + prog_off);
    float s[MAX_SLOTS];
    auto acc = [&](int buf, int dim, int nn, int i, int) { return pv.buf_ptr[buf][(size_t)nn * dim + i]; };
    load_gathers(s, pg, pv, um, T, N, t, n, acc, true);
    load_invariants(s, pg, weights, um);
    run_ops(s, pg);
    run_stores(s, pg, pv, um, N, t, n, [](float* p, float v) { *p = v; });
}

// One wavefront per output unit u of a task; all streams n in a loop.
__global__ __launch_bounds__(256) void step_matvec_kernel(PlanView pv, int mv_off, const float* __restrict__ weights,
                                                          int T, int N, int t) {
    const int32_t* w = pv.words + mv_off + 1;
    for (int task = 0; task < (int)blockIdx.y; ++task) w += MV_HEADER_WORDS + w[MV_NEDGES] * MVE_WORDS;
    const int n_out = w[MV_NOUT], n_edges = w[MV_NEDGES];
    const int lane = threadIdx.x & 63;
    const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (u >= n_out) return;
    float* acc = pv.buf_ptr[w[MV_ACC_BUF]];
    for (int n = 0; n < N; ++n) {
        float s = 0.0f;
        for (int e = 0; e < n_edges; ++e) {
            const int32_t* ed = w + MV_HEADER_WORDS + e * MVE_WORDS;
            const int frame = t + ed[MVE_FRAME_OFF];
            if (frame < 0 || frame >= T) continue;
            const int K = ed[MVE_KLEN];
            const float* W = weights + ed[MVE_W_OFF];
            const float* x = pv.buf_ptr[ed[MVE_SRC_BUF]] + ((size_t)frame * N + n) * K;
            if (ed[MVE_TRANSPOSED]) { for (int k = lane; k < K; k += 64) s += W[(size_t)k * n_out + u] * x[k]; }
            else { for (int k = lane; k < K; k += 64) s += W[(size_t)u * K + k] * x[k]; }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) acc[(size_t)n * n_out + u] = s;
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// One wavefront per row, in place.
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* __restrict__ y, long long rows, int dim) {
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int lane = threadIdx.x & 63;
    float* p = y + row * dim;
    float m = -INFINITY;
    for (int i = lane; i < dim; i += 64) m = fmaxf(m, p[i]);
    m = wave_max(m);
    float s = 0.0f;
    for (int i = lane; i < dim; i += 64) s += __expf(p[i] - m);
    s = wave_sum(s);
    const float inv = 1.0f / s;
    for (int i = lane; i < dim; i += 64) p[i] = __expf(p[i] - m) * inv;
}

__global__ __launch_bounds__(256) void softmax_ce_delta_kernel(const float* __restrict__ y, const int32_t* __restrict__ targets,
                                                               float* __restrict__ ds, double* loss, unsigned* flag, long long rows, int dim) {
    __shared__ float wl[4];
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float l = 0.0f;
    if (row < rows) {
        int tg = targets[row];
        if (tg >= dim) { if (lane == 0) atomicMax(flag, 3u); tg = -1; }      // not a class of this layer: the frame is left out
        const float* p = y + row * dim;
        float* d = ds + row * dim;
        for (int i = lane; i < dim; i += 64) d[i] = tg >= 0 ? p[i] - (i == tg ? 1.0f : 0.0f) : 0.0f;
        if (tg >= 0 && lane == 0) l = -__logf(p[tg]);
    }
    if (lane == 0) wl[wave] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double s = (double)wl[0] + (double)wl[1] + (double)wl[2] + (double)wl[3];
        if (s != 0.0) atomicAdd(loss, s);
    }
}

// Squared error E = 1/2 sum_j (d_j - y_j)^2 on an output layer y = f(s) (Section 2.2: the output delta
// follows the error criterion and the layer's activation): dE/ds = (y - d) f'(s).
__global__ __launch_bounds__(256) void squared_error_delta_kernel(const float* __restrict__ y, const float* __restrict__ d,
                                                                  float* __restrict__ ds, double* loss, long long n, int act) {
    __shared__ float wl[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float l = 0.0f;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += 256LL * gridDim.x) {
        const float yi = y[i], di = d[i];
        const float err = di != di ? 0.0f : yi - di;      // a NaN target element carries no error
        const float fp = act == 1 ? yi * (1.0f - yi) : act == 2 ? 1.0f - yi * yi : act == 4 ? (yi > 0.0f ? 1.0f : 0.0f) : 1.0f;
        ds[i] = err * fp;
        l += 0.5f * err * err;
    }
    l = wave_sum(l);
    if (lane == 0) wl[wave] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double s = (double)wl[0] + (double)wl[1] + (double)wl[2] + (double)wl[3];
        if (s != 0.0) atomicAdd(loss, s);
    }
}

// grid: (ceil(dim / 64), n_tasks, row splits); block (64, 4).
__global__ __launch_bounds__(256) void colsum_kernel(PlanView pv, int tasks_off, const float* __restrict__ weights,
                                                     float* __restrict__ grads, int T, int N, int t0) {
    __shared__ float part[4][64];
    const int32_t* w = pv.words + tasks_off;
    for (int task = 0; task < (int)blockIdx.y; ++task) w += CS_HEADER_WORDS + w[CS_NFACTORS] * CF_WORDS;
    const int dim = w[CS_DIM], nf = w[CS_NFACTORS];
    const int i = blockIdx.x * 64 + threadIdx.x;
    const long long rows = (long long)T * N;
    float s = 0.0f;
    if (i < dim) {
        for (long long r = (long long)t0 * N + (long long)blockIdx.z * 4 + threadIdx.y; r < rows; r += 4LL * gridDim.z) {
            const int t = (int)(r / N), n = (int)(r % N);
            float prod = 1.0f;
            auto value = [&](int j) {
                const int32_t* f = w + CS_HEADER_WORDS + j * CF_WORDS;
                const int frame = t + f[CF_FRAME_OFF];
                float v = 0.0f;
                if (frame >= 0 && frame < T) v = pv.buf_ptr[f[CF_BUF]][((size_t)frame * N + n) * dim + i];
                if (f[CF_W_OFF] >= 0) v *= weights[f[CF_W_OFF] + i];
                return v;
            };
            for (int j = 0; j < nf; ++j) {
                const int cmp = w[CS_HEADER_WORDS + j * CF_WORDS + CF_CMP];
                if (cmp != 0 && j + 1 < nf) {      // [this >= next] or [this > next]: a maximum node's routing
                    const float a = value(j), b = value(j + 1);
                    prod *= (cmp == 1 ? a >= b : a > b) ? 1.0f : 0.0f;
                    ++j;
                } else {
                    prod *= value(j);
                }
            }
            s += prod;
        }
    }
    part[threadIdx.y][threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.y == 0 && i < dim) {
        const float tot = part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x];
        unsafeAtomicAdd(&grads[w[CS_OUT_OFF] + i], tot);
    }
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, long long n, float v) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += 256LL * gridDim.x) p[i] = v;
}

}  // namespace

hipError_t launch_node_program(const PlanView& pv, int prog_off, int max_dim, const float* weights,
                               int T, int N, int t0, int t1, hipStream_t stream) {
    const long long total = (long long)(t1 - t0) * N * max_dim;
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(node_program_kernel, dim3(blocks), dim3(256), 0, stream, pv, prog_off, max_dim, weights, T, N, t0, total);
    return hipGetLastError();
}

hipError_t launch_step_matvec(const PlanView& pv, int mv_off, int n_tasks, int max_out, const float* weights,
                              int T, int N, int t, hipStream_t stream) {
    if (n_tasks <= 0 || max_out <= 0) return hipSuccess;
    hipLaunchKernelGGL(step_matvec_kernel, dim3((max_out + 3) / 4, n_tasks), dim3(256), 0, stream, pv, mv_off, weights, T, N, t);
    return hipGetLastError();
}

hipError_t launch_softmax_rows(float* y, int64_t rows, int dim, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(softmax_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, y, (long long)rows, dim);
    return hipGetLastError();
}

hipError_t launch_softmax_ce_delta(const float* y, const int32_t* targets, float* ds, double* loss, unsigned* flag,
                                   int64_t rows, int dim, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(softmax_ce_delta_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, y, targets, ds, loss, flag,
                       (long long)rows, dim);
    return hipGetLastError();
}

hipError_t launch_squared_error_delta(const float* y, const float* d, float* ds, double* loss, int64_t n, int act,
                                      hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(squared_error_delta_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, y, d, ds, loss, (long long)n, act);
    return hipGetLastError();
}

hipError_t launch_colsum(const PlanView& pv, int tasks_off, int n_tasks, int max_dim, const float* weights, float* grads,
                         int T, int N, int t0, bool one_writer, hipStream_t stream) {
    if (n_tasks <= 0 || max_dim <= 0) return hipSuccess;
    const long long rows = (long long)(T - t0) * N;
    int splits = (int)((rows + 63) / 64);
    if (splits > 128) splits = 128;
    if (splits < 1 || one_writer) splits = 1;      // one workgroup per (task, 64 units): a fixed order of additions
    hipLaunchKernelGGL(colsum_kernel, dim3((max_dim + 63) / 64, n_tasks, splits), dim3(64, 4), 0, stream, pv, tasks_off,
                       weights, grads, T, N, t0);
    return hipGetLastError();
}

namespace {
__global__ __launch_bounds__(256) void copy_kernel(float* __restrict__ dst, const float* __restrict__ src, long long n) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += 256LL * gridDim.x) dst[i] = src[i];
}
constexpr int UPLOAD_CHUNK_WORDS = 960;      // 3840 bytes of kernel arguments
struct UploadChunk { uint32_t w[UPLOAD_CHUNK_WORDS]; };
__global__ __launch_bounds__(256) void upload_words_kernel(uint32_t* __restrict__ dst, UploadChunk c, int n) {
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.w[i];
}
}  // namespace

namespace {
__global__ __launch_bounds__(256) void transpose_kernel(float* __restrict__ dst, const float* __restrict__ src, int rows, int cols) {
    __shared__ float tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}
}  // namespace

hipError_t launch_transpose(float* dst, const float* src, int rows, int cols, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(transpose_kernel, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(256), 0, stream, dst, src, rows, cols);
    return hipGetLastError();
}

hipError_t launch_copy(float* dst, const float* src, int64_t n, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dst, src, (long long)n);
    return hipGetLastError();
}

hipError_t launch_upload_words(uint32_t* d_dst, const uint32_t* h_src, int64_t n, hipStream_t stream) {
    for (int64_t off = 0; off < n; off += UPLOAD_CHUNK_WORDS) {
        UploadChunk c;
        const int m = (int)std::min<int64_t>(UPLOAD_CHUNK_WORDS, n - off);
        for (int i = 0; i < m; ++i) c.w[i] = h_src[off + i];
        hipLaunchKernelGGL(upload_words_kernel, dim3(1), dim3(256), 0, stream, d_dst + off, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

namespace {
// One workgroup per buffer: the first `rows` rows of a flagged buffer become zero.
__global__ __launch_bounds__(256) void zero_history_kernel(float* const* __restrict__ buf_ptr, const int32_t* __restrict__ buf_dim,
                                                           const int32_t* __restrict__ buf_flags, long long rows) {
    const int b = blockIdx.x;
    if (buf_flags[b] != 1) return;
    float* p = buf_ptr[b];
    const long long n = rows * buf_dim[b];
    for (long long i = threadIdx.x; i < n; i += 256) p[i] = 0.0f;
}
}  // namespace

hipError_t launch_zero_history(float* const* buf_ptr, const int32_t* buf_dim, const int32_t* buf_flags, int n_bufs, int64_t rows,
                               hipStream_t stream) {
    if (n_bufs <= 0 || rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(zero_history_kernel, dim3((unsigned)n_bufs), dim3(256), 0, stream, buf_ptr, buf_dim, buf_flags, (long long)rows);
    return hipGetLastError();
}

hipError_t launch_fill(float* p, int64_t n, float v, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, (long long)n, v);
    return hipGetLastError();
}


namespace {
// One-hot source (Section 4's word-input layer): C[f][j] (+)= W[j][idx[f - shift]] for rows f of
// frames [row0, row0 + rows); an index of -1 (or a frame before the window) contributes nothing.
__global__ __launch_bounds__(256) void onehot_gather_kernel(float* __restrict__ C, const float* __restrict__ W, const int* __restrict__ idx,
                                                            int n_dst, int n_src, long long row0, long long rows, long long shift_rows,
                                                            long long total_rows, int accumulate) {
    for (long long r = blockIdx.x; r < rows; r += gridDim.x) {
        const long long f = row0 + r, fs = f - shift_rows;
        const int c = (fs >= 0 && fs < total_rows) ? idx[fs] : -1;
        for (int j = threadIdx.x; j < n_dst; j += 256) {
            const float v = (c >= 0 && c < n_src) ? W[(size_t)j * n_src + c] : 0.0f;
            float* dst = C + f * n_dst + j;
            *dst = accumulate ? *dst + v : v;
        }
    }
}
// G[j][idx[f - shift]] += ds[f][j] over all rows f >= shift.
__global__ __launch_bounds__(256) void onehot_scatter_kernel(float* __restrict__ G, const float* __restrict__ ds, const int* __restrict__ idx,
                                                             int n_dst, int n_src, long long shift_rows, long long total_rows) {
    for (long long f = shift_rows + blockIdx.x; f < total_rows; f += gridDim.x) {
        const int c = idx[f - shift_rows];
        if (c < 0 || c >= n_src) continue;
        for (int j = threadIdx.x; j < n_dst; j += 256) unsafeAtomicAdd(&G[(size_t)j * n_src + c], ds[f * n_dst + j]);
    }
}
}  // namespace

hipError_t launch_onehot_gather(float* C, const float* W, const int* idx, int n_dst, int n_src, int64_t row0, int64_t rows,
                                int64_t shift_rows, int64_t total_rows, bool accumulate, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>(rows, 8192);
    hipLaunchKernelGGL(onehot_gather_kernel, dim3(grid), dim3(256), 0, stream, C, W, idx, n_dst, n_src, (long long)row0, (long long)rows,
                       (long long)shift_rows, (long long)total_rows, accumulate ? 1 : 0);
    return hipGetLastError();
}

namespace {
// The same sum with one writer per element: thread j walks the rows in order.
__global__ __launch_bounds__(256) void onehot_scatter_ordered_kernel(float* __restrict__ G, const float* __restrict__ ds, const int* __restrict__ idx,
                                                                     int n_dst, int n_src, long long shift_rows, long long total_rows) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n_dst) return;
    for (long long f = shift_rows; f < total_rows; ++f) {
        const int c = idx[f - shift_rows];
        if (c >= 0 && c < n_src) G[(size_t)j * n_src + c] += ds[f * n_dst + j];
    }
}
}  // namespace

hipError_t launch_onehot_scatter(float* G, const float* ds, const int* idx, int n_dst, int n_src, int64_t shift_rows, int64_t total_rows,
                                 bool ordered, hipStream_t stream) {
    if (total_rows - shift_rows <= 0) return hipSuccess;
    if (ordered) {
        hipLaunchKernelGGL(onehot_scatter_ordered_kernel, dim3((n_dst + 255) / 256), dim3(256), 0, stream, G, ds, idx, n_dst, n_src,
                           (long long)shift_rows, (long long)total_rows);
        return hipGetLastError();
    }
    const int grid = (int)std::min<int64_t>(total_rows - shift_rows, 8192);
    hipLaunchKernelGGL(onehot_scatter_kernel, dim3(grid), dim3(256), 0, stream, G, ds, idx, n_dst, n_src, (long long)shift_rows, (long long)total_rows);
    return hipGetLastError();
}

}  // namespace rnng
