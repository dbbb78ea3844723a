// Combination stage of the backward pass on the active rows only (Alg. 1, backward loop):
//     W' = Y^T (x) X'      (F_in x F_out, a sum over vertices)
//     Y' = X' (x) W^T      (one row per vertex)
// Theorem 1 makes every row of X' outside N^k zero, so both products run over the ascending id
// list of N^k only: the rows are gathered (and, for Y', scattered) by vertex id, everything
// else is a dense contraction and runs on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32).
//
// Both kernels are 64 x 64 output tiles per workgroup, four wavefronts in a 2 x 2 arrangement
// with one 32 x 32 accumulator block each, and a contraction step of 32 staged through LDS.
//
// Operand layout of the 32x32x2 instruction: lane l supplies A[l % 32][l / 32] and
// B[l / 32][l % 32]; element j of its accumulator is C[8 (j / 4) + 4 (l / 32) + j % 4][l % 32].

#include <algorithm>

#include "epp_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int kTile = 64;   // output tile edge
constexpr int kStep = 32;   // contraction step
constexpr int kMaxWidth = 4096;

// Y'[id, n] = sum_k X'[id, k] W[n, k] for the ids of one 64-row tile and 64 columns n.
__global__ __launch_bounds__(kBlock) void k_input_gradient(const int32_t* __restrict__ ids, int64_t n_rows,
                                                           const float* __restrict__ G, int Fo,
                                                           const float* __restrict__ W, int Fi,
                                                           float* __restrict__ Yg) {
    __shared__ float As[kTile][kStep + 1];   // X' rows of the tile, [row][k]
    __shared__ float Bs[kStep][kTile + 1];   // W^T, [k][n]
    __shared__ int64_t sid[kTile];           // vertex of each tile row, -1 past the end
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w & 1, wn = w >> 1;
    const int64_t row0 = (int64_t)blockIdx.x * kTile;
    const int n0 = blockIdx.y * kTile;
    if (t < kTile) {
        const int64_t r = row0 + t;
        sid[t] = r < n_rows ? (ids ? (int64_t)ids[r] : r) : -1;
    }
    __syncthreads();
    floatx16 acc = {};
    for (int k0 = 0; k0 < Fo; k0 += kStep) {
#pragma unroll
        for (int i = 0; i < (kTile * kStep) / kBlock; ++i) {
            const int e = t + kBlock * i;
            const int r = e / kStep, k = e % kStep;
            const int64_t id = sid[r];
            As[r][k] = (id >= 0 && k0 + k < Fo) ? G[id * Fo + k0 + k] : 0.0f;
            const int n = n0 + r;  // the same split serves the 64 x 32 block of W
            Bs[k][r] = (n < Fi && k0 + k < Fo) ? W[(int64_t)n * Fo + k0 + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kStep; kk += 2) {
            const float a = As[32 * wm + (lane & 31)][kk + (lane >> 5)];
            const float b = Bs[kk + (lane >> 5)][32 * wn + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    const int n = n0 + 32 * wn + (lane & 31);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int i = 8 * (j / 4) + 4 * (lane >> 5) + (j % 4);
        const int64_t id = sid[32 * wm + i];
        if (id >= 0 && n < Fi) Yg[id * Fi + n] = acc[j];
    }
}

// partial[chunk][m][n] = sum over the chunk's rows of Y[id, m] X'[id, n], one 64 x 64 tile.
__global__ __launch_bounds__(kBlock) void k_weight_gradient(const int32_t* __restrict__ ids, int64_t n_rows,
                                                            int64_t rows_per_chunk, const float* __restrict__ Y,
                                                            int Fi, const float* __restrict__ G, int Fo,
                                                            float* __restrict__ partial) {
    __shared__ float As[kStep][kTile];   // Y rows, [row][m]
    __shared__ float Bs[kStep][kTile];   // X' rows, [row][n]
    __shared__ int64_t sid[kStep];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w & 1, wn = w >> 1;
    const int m0 = blockIdx.y * kTile, n0 = blockIdx.z * kTile;
    const int64_t first = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t last = std::min<int64_t>(first + rows_per_chunk, n_rows);
    floatx16 acc = {};
    for (int64_t r0 = first; r0 < last; r0 += kStep) {
        if (t < kStep) {
            const int64_t r = r0 + t;
            sid[t] = r < last ? (ids ? (int64_t)ids[r] : r) : -1;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < (kStep * kTile) / kBlock; ++i) {
            const int e = t + kBlock * i;
            const int k = e / kTile, c = e % kTile;
            const int64_t id = sid[k];
            As[k][c] = (id >= 0 && m0 + c < Fi) ? Y[id * Fi + m0 + c] : 0.0f;
            Bs[k][c] = (id >= 0 && n0 + c < Fo) ? G[id * Fo + n0 + c] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < kStep; kk += 2) {
            const float a = As[kk + (lane >> 5)][32 * wm + (lane & 31)];
            const float b = Bs[kk + (lane >> 5)][32 * wn + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }
    const int n = n0 + 32 * wn + (lane & 31);
    float* __restrict__ mine = partial + (int64_t)blockIdx.x * Fi * Fo;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int m = m0 + 32 * wm + 8 * (j / 4) + 4 * (lane >> 5) + (j % 4);
        if (m < Fi && n < Fo) mine[(int64_t)m * Fo + n] = acc[j];
    }
}

// W'[e] = sum over chunks, in chunk order, accumulated in double.
__global__ __launch_bounds__(kBlock) void k_weight_gradient_reduce(const float* __restrict__ partial, int64_t n_chunks,
                                                                   int64_t total, float* __restrict__ Wg) {
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= total) return;
    double s = 0.0;
    for (int64_t c = 0; c < n_chunks; ++c) s += (double)partial[c * total + e];
    Wg[e] = (float)s;
}

int check_widths(int Fi, int Fo) {
    if (Fi < 1 || Fo < 1 || Fi > kMaxWidth || Fo > kMaxWidth) {
        epp_set_error("widths F_in=%d F_out=%d outside [1, %d]", Fi, Fo, kMaxWidth);
        return EPP_ERR_INVALID_ARG;
    }
    return EPP_OK;
}

// Row set of the products: N^k, or every vertex for k = -1.
int row_set(epp_paths* p, int k, hipStream_t s, const int32_t** ids, int64_t* count) {
    if (k == -1) {
        *ids = nullptr;
        *count = p->n;
        return EPP_OK;
    }
    return epp_active_ids(p, k, s, ids, count);
}

// Rows per partial sum: enough chunks to fill the chip a few times over, whole steps each.
void chunking(int64_t n_rows, int Fi, int Fo, int64_t* rows_per_chunk, int64_t* n_chunks) {
    const int64_t tiles = (int64_t)((Fi + kTile - 1) / kTile) * ((Fo + kTile - 1) / kTile);
    const int64_t want = std::max<int64_t>(1, 2048 / tiles);
    int64_t per = (n_rows + want - 1) / want;
    per = std::max<int64_t>(kStep, (per + kStep - 1) / kStep * kStep);
    *rows_per_chunk = per;
    *n_chunks = (n_rows + per - 1) / per;
}

}  // namespace

extern "C" int64_t epp_weight_gradient_workspace(const epp_paths_t* paths, int k, int F_in, int F_out) {
    if (!paths) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    if (check_widths(F_in, F_out) != EPP_OK) return EPP_ERR_INVALID_ARG;
    int64_t per, chunks;
    chunking(k < 0 ? paths->n : paths->set_size[k], F_in, F_out, &per, &chunks);
    return std::max<int64_t>(chunks, 1) * F_in * F_out * (int64_t)sizeof(float);
}

extern "C" int epp_weight_gradient(epp_paths_t* paths, int k, const float* Y, int F_in, const float* grad_X, int F_out,
                                   float* grad_W, void* workspace, int64_t workspace_bytes, epp_stream_t stream) {
    if (!paths || !Y || !grad_X || !grad_W || !workspace) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(check_widths(F_in, F_out));
    const int64_t need = epp_weight_gradient_workspace(paths, k, F_in, F_out);
    if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15)) {
        epp_set_error("workspace of %lld bytes (need %lld, 16-byte aligned)", (long long)workspace_bytes, (long long)need);
        return EPP_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    const int32_t* ids = nullptr;
    int64_t n_rows = 0;
    EPP_TRY(row_set(paths, k, s, &ids, &n_rows));
    int64_t per, chunks;
    chunking(n_rows, F_in, F_out, &per, &chunks);
    if (chunks > 0) {
        const dim3 grid((unsigned)chunks, (unsigned)((F_in + kTile - 1) / kTile), (unsigned)((F_out + kTile - 1) / kTile));
        hipLaunchKernelGGL(k_weight_gradient, grid, dim3(kBlock), 0, s, ids, n_rows, per, Y, F_in, grad_X, F_out,
                           static_cast<float*>(workspace));
    }
    const int64_t total = (int64_t)F_in * F_out;
    hipLaunchKernelGGL(k_weight_gradient_reduce, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       static_cast<const float*>(workspace), chunks, total, grad_W);
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}

extern "C" int epp_input_gradient(epp_paths_t* paths, int k, const float* grad_X, int F_out, const float* W, int F_in,
                                  float* grad_Y, epp_stream_t stream) {
    if (!paths || !grad_X || !W || !grad_Y) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(check_widths(F_in, F_out));
    hipStream_t s = (hipStream_t)stream;
    const int32_t* ids = nullptr;
    int64_t n_rows = 0;
    EPP_TRY(row_set(paths, k, s, &ids, &n_rows));
    if (n_rows == 0) return EPP_OK;
    const dim3 grid((unsigned)((n_rows + kTile - 1) / kTile), (unsigned)((F_in + kTile - 1) / kTile));
    hipLaunchKernelGGL(k_input_gradient, grid, dim3(kBlock), 0, s, ids, n_rows, grad_X, F_out, W, F_in, grad_Y);
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}
