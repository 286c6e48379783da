// Grouped fp32 GEMM on the CDNA matrix cores (v_mfma_f32_32x32x2_f32) for the batched part of
// the intra-stream schedule (paper Section 3.1: everything outside the recurrent nodes is
// computed for all frames of the window at once) and for the weight gradients (Section 2.2,
// last equation: a sum over all frames of outer products, i.e. one GEMM whose contraction
// runs over frames).
//
// Block tile 128 x 128, K chunk 16, 256 threads = 4 wavefronts in a 2 x 2 arrangement, each
// wavefront owning a 64 x 64 sub-tile as 2 x 2 MFMA 32x32 accumulators.  Operand tiles are
// staged through LDS in k-major order ([k][m], row stride 132 floats) so that the MFMA operand
// fetch of a wavefront is a conflict-free ds_read_b32 for both operand orientations; global
// loads for chunk c+1 are in flight while chunk c is multiplied.
#include <cstdlib>

#include "kernels.h"

namespace rnng {
namespace {

constexpr int BM = 128, BN = 128, BK = 16, NTHREADS = 256;
constexpr int STRIDE = 132;   // floats per k-row in LDS

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---- K-contiguous source: element (r, k) at base[(r + row_off) * ld + k] --------------------
__device__ __forceinline__ void load_kc(float (&r)[8], const float* __restrict__ base, int ld, int row0, int row_limit,
                                        int row_off, int src_rows, int k0, int k_limit, bool vec_ok, int tid) {
    const int k = k0 + 4 * (tid & 3);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = row0 + (tid >> 2) + 64 * j;
        const int srow = row + row_off;
        const bool ok = row < row_limit && srow >= 0 && srow < src_rows;
        const float* p = base + (size_t)(ok ? srow : 0) * ld + k;
        if (ok && vec_ok && k + 3 < k_limit) {
            floatx4 v = *reinterpret_cast<const floatx4*>(p);
            r[4 * j + 0] = v.x; r[4 * j + 1] = v.y; r[4 * j + 2] = v.z; r[4 * j + 3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) r[4 * j + e] = (ok && k + e < k_limit) ? p[e] : 0.0f;
        }
    }
}
// A thread holds four consecutive k of one row; k rows lie 132 floats apart, so the four threads
// that share a row index group would hit two banks twice if all stored their element e at once.
// Instruction i stores element (e0 + i) % 4 with e0 = 0, 2, 2, 0 for tid % 4 = 0 .. 3: the 32 lanes
// of a half-wavefront then fall into four disjoint windows of eight banks.
__device__ __forceinline__ void store_kc(float* __restrict__ lds, const float (&r)[8], int tid) {
    const int a = tid & 3, e0 = (a == 1 || a == 2) ? 2 : 0;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = (e0 + i) & 3;
            const float v = e == 0 ? r[4 * j] : e == 1 ? r[4 * j + 1] : e == 2 ? r[4 * j + 2] : r[4 * j + 3];
            lds[(4 * a + e) * STRIDE + (tid >> 2) + 64 * j] = v;
        }
}

// ---- M/N-contiguous source: element (k, c) at base[k * ld + c] ------------------------------
__device__ __forceinline__ void load_mc(float (&r)[8], const float* __restrict__ base, int ld, int c0, int c_limit,
                                        int k0, int k_limit, bool vec_ok, int tid) {
    const int c = c0 + 4 * (tid & 31);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = k0 + (tid >> 5) + 8 * j;
        const bool ok = k < k_limit;
        const float* p = base + (size_t)(ok ? k : 0) * ld + c;
        if (ok && vec_ok && c + 3 < c_limit) {
            floatx4 v = *reinterpret_cast<const floatx4*>(p);
            r[4 * j + 0] = v.x; r[4 * j + 1] = v.y; r[4 * j + 2] = v.z; r[4 * j + 3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) r[4 * j + e] = (ok && c + e < c_limit) ? p[e] : 0.0f;
        }
    }
}
__device__ __forceinline__ void store_mc(float* __restrict__ lds, const float (&r)[8], int tid) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        floatx4 v = {r[4 * j + 0], r[4 * j + 1], r[4 * j + 2], r[4 * j + 3]};
        *reinterpret_cast<floatx4*>(&lds[((tid >> 5) + 8 * j) * STRIDE + 4 * (tid & 31)]) = v;
    }
}

__device__ __forceinline__ bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(const GemmGroup g) {
    __shared__ __attribute__((aligned(16))) float sA[BK * STRIDE];
    __shared__ __attribute__((aligned(16))) float sB[BK * STRIDE];

    const int pi = blockIdx.z / g.split_k;
    const int split = blockIdx.z - pi * g.split_k;
    const GemmProblem& P = g.p[pi];
    const int tiles_m = (P.M + BM - 1) / BM, tiles_n = (P.N + BN - 1) / BN;
    const int n_tiles = tiles_m * tiles_n;
    if ((int)blockIdx.x >= n_tiles) return;
    // Which tile a workgroup takes.  Workgroups go to the eight XCDs in turn and each XCD has an
    // L2 of its own, so workgroup b takes tile start(b % 8) + b / 8: every XCD works on one
    // consecutive range of tiles.  Inside the range the tiles run down groups of g.group_m row
    // blocks before they move to the next column block, so that the workgroups that are resident
    // together on an XCD share both A panels and B panels in its L2.
    int tile = blockIdx.x;
    const int GM = g.group_m;
    if (GM > 0) {
        const int q = n_tiles / 8, r = n_tiles - 8 * q, x = tile & 7;
        tile = x * q + (x < r ? x : r) + (tile >> 3);
    }
    int tm, tn;
    if (GM > 1) {
        const int per_group = GM * tiles_n, group = tile / per_group, first_m = group * GM;
        const int gsz = tiles_m - first_m < GM ? tiles_m - first_m : GM;
        const int in_group = tile - group * per_group;
        tn = in_group / gsz; tm = first_m + in_group - tn * gsz;
    } else {
        tm = tile / tiles_n; tn = tile - tm * tiles_n;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    for (int p = 0; p < P.n_pairs; ++p) {
        const GemmPair pr = P.pairs[p];
        const int nk = (pr.K + BK - 1) / BK;
        const int c_begin = (int)((long long)nk * split / g.split_k);
        const int c_end = (int)((long long)nk * (split + 1) / g.split_k);
        if (c_begin >= c_end) continue;
        const bool a_vec = (pr.lda & 3) == 0 && aligned16(pr.A);
        const bool b_vec = (pr.ldb & 3) == 0 && aligned16(pr.B);
        float ra[8], rb[8];
        auto fetch = [&](int c) {
            const int k0 = c * BK;
            if (A_KC) load_kc(ra, pr.A, pr.lda, m0, P.M, pr.a_row_off, pr.a_rows, k0, pr.K, a_vec, tid);
            else load_mc(ra, pr.A, pr.lda, m0, P.M, k0, pr.K, a_vec, tid);
            if (B_KC) load_kc(rb, pr.B, pr.ldb, n0, P.N, 0, P.N, k0, pr.K, b_vec, tid);
            else load_mc(rb, pr.B, pr.ldb, n0, P.N, k0, pr.K, b_vec, tid);
        };
        fetch(c_begin);
        for (int c = c_begin; c < c_end; ++c) {
            __syncthreads();
            if (A_KC) store_kc(sA, ra, tid); else store_mc(sA, ra, tid);
            if (B_KC) store_kc(sB, rb, tid); else store_mc(sB, rb, tid);
            __syncthreads();
            if (c + 1 < c_end) fetch(c + 1);
#pragma unroll
            for (int kk = 0; kk < BK / 2; ++kk) {
                const int krow = (2 * kk + (lane >> 5)) * STRIDE + (lane & 31);
                const float a0 = sA[krow + wm * 64], a1 = sA[krow + wm * 64 + 32];
                const float b0 = sB[krow + wn * 64], b1 = sB[krow + wn * 64 + 32];
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            }
        }
    }

    // 32x32 accumulator layout: register e of lane l holds row 8*(e/4) + 4*(l/32) + e%4, column l%32.
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = n0 + wn * 64 + b * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * 64 + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < P.M && col < P.N) {
                    float* dst = P.C + (size_t)row * P.ldc + col;
                    if (g.split_k > 1) unsafeAtomicAdd(dst, acc[a][b][e]);
                    else if (g.accumulate) *dst += acc[a][b][e];
                    else *dst = acc[a][b][e];
                }
            }
        }
}

}  // namespace

hipError_t launch_gemm_group(GemmMode mode, const GemmGroup& g, hipStream_t stream) {
    if (g.n_problems <= 0) return hipSuccess;
    int max_tiles = 0;
    for (int i = 0; i < g.n_problems; ++i) {
        const int t = ((g.p[i].M + BM - 1) / BM) * ((g.p[i].N + BN - 1) / BN);
        max_tiles = t > max_tiles ? t : max_tiles;
    }
    if (max_tiles == 0) return hipSuccess;
    dim3 grid(max_tiles, 1, g.n_problems * g.split_k), block(NTHREADS);
    static const int group_m = [] { const char* env = std::getenv("RNNG_GEMM_GROUP_M"); return env ? std::atoi(env) : 8; }();
    GemmGroup gg = g;
    gg.group_m = group_m < 0 ? 0 : group_m;
    switch (mode) {
        case GEMM_NT: hipLaunchKernelGGL((gemm_kernel<true, true>), grid, block, 0, stream, gg); break;
        case GEMM_NN: hipLaunchKernelGGL((gemm_kernel<true, false>), grid, block, 0, stream, gg); break;
        case GEMM_TN: hipLaunchKernelGGL((gemm_kernel<false, false>), grid, block, 0, stream, gg); break;
    }
    return hipGetLastError();
}

}  // namespace rnng
