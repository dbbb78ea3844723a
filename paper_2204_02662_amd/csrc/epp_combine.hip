// Combination stage of the backward pass on the active rows only (Alg. 1, backward loop):
//     W' = Y^T (x) X'      (F_in x F_out, a sum over vertices)
//     Y' = X' (x) W^T      (one row per vertex)
// Theorem 1 makes every row of X' outside N^k zero, so both products run over the ascending id
// list of N^k only: the rows are gathered (and, for Y', scattered) by vertex id, everything
// else is a dense contraction and runs on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32).
//
// Both kernels give a workgroup of four wavefronts, arranged WM x WN, an output tile of
// 32 WM BM x 32 WN BN, every wavefront BM x BN accumulator blocks of 32 x 32, and step through
// the contraction 32 at a time: the operand tiles of the next step are fetched into registers
// while the matrix cores work on the current ones in LDS.  The arrangement follows the matrix:
// 2 x 2 wavefronts with up to 2 x 2 blocks each for wide outputs, 4 x 1 (a 128 x 32 tile) when
// one side has at most 32 columns, as the weight matrices of a GCN with 16 hidden units or a
// few classes do.
//
// Operand layout of the 32x32x2 instruction: lane l supplies A[l % 32][l / 32] and
// B[l / 32][l % 32]; element j of its accumulator is C[8 (j / 4) + 4 (l / 32) + j % 4][l % 32].

#include <algorithm>

#include "epp_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int kStep = 32;   // contraction step
constexpr int kMaxWidth = 4096;
constexpr int kMinChunkRows = 256;
constexpr int64_t kNoChunkLimit = (int64_t)1 << 40;

typedef float float4v __attribute__((ext_vector_type(4)));

// Four consecutive floats of a row; VEC: one 16-byte access (the caller has checked that widths
// are multiples of four and bases 16-byte aligned), else element by element up to `valid`.
template <bool VEC>
__device__ __forceinline__ float4v load4(const float* __restrict__ p, int valid) {
    if constexpr (VEC) {
        return valid > 0 ? *reinterpret_cast<const float4v*>(p) : float4v{0.f, 0.f, 0.f, 0.f};
    } else {
        float4v v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < valid) v[i] = p[i];
        return v;
    }
}

// Thread mapping of all tile loads: eight threads per row, four consecutive floats each, so a
// row segment of 32 floats is one 128-byte access and a thread needs one vertex id per row.

// Y'[id, n] = sum_k X'[id, k] W[n, k] for the ids of one tile of 32 WM BM rows and 32 WN BN columns n.
template <int WM, int WN, int BM, int BN, bool VEC>
__global__ __launch_bounds__(kBlock) void k_input_gradient(const int32_t* __restrict__ ids, int64_t n_rows,
                                                           const float* __restrict__ G, int Fo,
                                                           const float* __restrict__ W, int Fi,
                                                           float* __restrict__ Yg) {
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int TM = 32 * WM * BM, TN = 32 * WN * BN;
    constexpr int NA = TM / 32, NB = TN / 32;  // rows per thread and step
    __shared__ float As[TM][kStep + 1];   // X' rows of the tile, [row][k]
    __shared__ float Bs[kStep][TN + 1];   // W^T, [k][n]
    __shared__ int64_t sid[TM];           // vertex of each tile row, -1 past the end
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w % WM, wn = w / WM;
    const int64_t row0 = (int64_t)blockIdx.x * TM;
    const int n0 = blockIdx.y * TN;
    for (int r = t; r < TM; r += kBlock) {
        const int64_t row = row0 + r;
        sid[r] = row < n_rows ? (ids ? (int64_t)ids[row] : row) : -1;
    }
    __syncthreads();
    const int tr = t >> 3, k = 4 * (t & 7);
    int64_t oa[NA], ob[NB];  // element offset of this thread's piece at k0 = 0; -1: no such row
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int64_t id = sid[tr + 32 * i];
        oa[i] = id >= 0 ? id * Fo + k : -1;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int n = n0 + tr + 32 * i;
        ob[i] = n < Fi ? (int64_t)n * Fo + k : -1;
    }
    float4v ra[NA], rb[NB];
    auto fetch = [&](int k0) {
        const int valid = Fo - (k0 + k);
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = load4<VEC>(G + (oa[i] >= 0 ? oa[i] + k0 : 0), oa[i] >= 0 ? valid : 0);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = load4<VEC>(W + (ob[i] >= 0 ? ob[i] + k0 : 0), ob[i] >= 0 ? valid : 0);
    };
    floatx16 acc[BM][BN] = {};
    fetch(0);
    for (int k0 = 0; k0 < Fo; k0 += kStep) {
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) As[tr + 32 * i][k + c] = ra[i][c];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) Bs[k + c][tr + 32 * i] = rb[i][c];
        __syncthreads();
        if (k0 + kStep < Fo) fetch(k0 + kStep);
#pragma unroll
        for (int kk = 0; kk < kStep; kk += 2) {
            float a[BM], b[BN];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) a[bm] = As[32 * (BM * wm + bm) + (lane & 31)][kk + (lane >> 5)];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) b[bn] = Bs[kk + (lane >> 5)][32 * (BN * wn + bn) + (lane & 31)];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bm], b[bn], acc[bm][bn], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            const int n = n0 + 32 * (BN * wn + bn) + (lane & 31);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int i = 8 * (j / 4) + 4 * (lane >> 5) + (j % 4);
                const int64_t id = sid[32 * (BM * wm + bm) + i];
                if (id >= 0 && n < Fi) Yg[id * Fi + n] = acc[bm][bn][j];
            }
        }
}

// partial[chunk][m][n] = sum over the chunk's rows of Y[id, m] X'[id, n], one tile of 32 WM BM x 32 WN BN.
// The vertex id of a row is fetched one step before the row itself, so that the row loads of a
// step never wait for an id.
template <int WM, int WN, int BM, int BN, bool VEC>
__global__ __launch_bounds__(kBlock) void k_weight_gradient(const int32_t* __restrict__ ids, int64_t n_rows,
                                                            int64_t rows_per_chunk, const float* __restrict__ Y,
                                                            int Fi, const float* __restrict__ G, int Fo,
                                                            float* __restrict__ partial) {
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int TM = 32 * WM * BM, TN = 32 * WN * BN;
    constexpr int NA = TM / 32, NB = TN / 32;  // 4-float pieces per thread and step
    __shared__ __attribute__((aligned(16))) float As[kStep][TM];   // Y rows, [row][m]
    __shared__ __attribute__((aligned(16))) float Bs[kStep][TN];   // X' rows, [row][n]
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int wm = w % WM, wn = w / WM;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.z * TN;
    const int64_t first = (int64_t)blockIdx.x * rows_per_chunk;
    const int64_t last = std::min<int64_t>(first + rows_per_chunk, n_rows);
    const int tr = t >> 3, c4 = 4 * (t & 7);
    auto vertex = [&](int64_t r) -> int64_t { return r < last ? (ids ? (int64_t)ids[r] : r) : -1; };
    float4v ra[NA], rb[NB];
    auto fetch = [&](int64_t id) {
        const float* y = Y + (id >= 0 ? id * Fi + m0 + c4 : 0);
        const float* g = G + (id >= 0 ? id * Fo + n0 + c4 : 0);
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = load4<VEC>(y + 32 * i, id >= 0 ? Fi - (m0 + c4 + 32 * i) : 0);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = load4<VEC>(g + 32 * i, id >= 0 ? Fo - (n0 + c4 + 32 * i) : 0);
    };
    floatx16 acc[BM][BN] = {};
    int64_t id_next = -1;
    if (first < last) {
        fetch(vertex(first + tr));
        id_next = vertex(first + kStep + tr);
    }
    for (int64_t r0 = first; r0 < last; r0 += kStep) {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<float4v*>(&As[tr][c4 + 32 * i]) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<float4v*>(&Bs[tr][c4 + 32 * i]) = rb[i];
        __syncthreads();
        if (r0 + kStep < last) {
            fetch(id_next);
            id_next = vertex(r0 + 2 * kStep + tr);
        }
#pragma unroll
        for (int kk = 0; kk < kStep; kk += 2) {
            float a[BM], b[BN];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) a[bm] = As[kk + (lane >> 5)][32 * (BM * wm + bm) + (lane & 31)];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) b[bn] = Bs[kk + (lane >> 5)][32 * (BN * wn + bn) + (lane & 31)];
#pragma unroll
            for (int bm = 0; bm < BM; ++bm)
#pragma unroll
                for (int bn = 0; bn < BN; ++bn)
                    acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bm], b[bn], acc[bm][bn], 0, 0, 0);
        }
        __syncthreads();
    }
    float* __restrict__ mine = partial + (int64_t)blockIdx.x * Fi * Fo;
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
        for (int bn = 0; bn < BN; ++bn) {
            const int n = n0 + 32 * (BN * wn + bn) + (lane & 31);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int m = m0 + 32 * (BM * wm + bm) + 8 * (j / 4) + 4 * (lane >> 5) + (j % 4);
                if (m < Fi && n < Fo) mine[(int64_t)m * Fo + n] = acc[bm][bn][j];
            }
        }
}

// W'[e] = sum over chunks: 16 threads per element take every 16th chunk each, accumulate in
// double, and are added in lane order (the result does not depend on timing).
__global__ __launch_bounds__(kBlock) void k_weight_gradient_reduce(const float* __restrict__ partial, int64_t n_chunks,
                                                                   int64_t total, float* __restrict__ Wg) {
    __shared__ double part[16][17];
    const int el = threadIdx.x & 15, cl = threadIdx.x >> 4;
    const int64_t e = (int64_t)blockIdx.x * 16 + el;
    double s = 0.0;
    if (e < total)
        for (int64_t c = cl; c < n_chunks; c += 16) s += (double)partial[c * total + e];
    part[cl][el] = s;
    __syncthreads();
    if (cl == 0 && e < total) {
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += part[i][el];
        Wg[e] = (float)sum;
    }
}

// 16-byte row accesses need widths that are multiples of four and aligned bases.
bool aligned4(int Fa, int Fb, const void* a, const void* b) {
    return Fa % 4 == 0 && Fb % 4 == 0 && ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0;
}

// Output tile of a launch, by the extents of the two tiled dimensions (m is always "long" for the
// input gradient, whose rows are the active vertices).
enum TileShape { T128x128, T128x64, T64x128, T64x64, T128x32, T32x128 };
TileShape tile_shape(int m, int n) {
    if (n <= 32 && m > 32) return T128x32;
    if (m <= 32 && n > 32) return T32x128;
    if (m > 64) return n > 64 ? T128x128 : T128x64;
    return n > 64 ? T64x128 : T64x64;
}
void tile_dims(TileShape t, int* tm, int* tn) {
    static const int dims[6][2] = {{128, 128}, {128, 64}, {64, 128}, {64, 64}, {128, 32}, {32, 128}};
    *tm = dims[t][0];
    *tn = dims[t][1];
}

int check_widths(int Fi, int Fo) {
    if (Fi < 1 || Fo < 1 || Fi > kMaxWidth || Fo > kMaxWidth) {
        epp_set_error("widths F_in=%d F_out=%d outside [1, %d]", Fi, Fo, kMaxWidth);
        return EPP_ERR_INVALID_ARG;
    }
    return EPP_OK;
}

// Row set of the products: N^k, or every vertex for k = -1.
int row_set(const epp_paths* p, int k, const int32_t** ids, int64_t* count) {
    if (k == -1) {
        *ids = nullptr;
        *count = p->n;
        return EPP_OK;
    }
    return epp_active_ids(p, k, ids, count);
}

// Rows per partial sum: enough chunks to fill the chip a few times over (at most `max_chunks`
// of them), whole steps each.
void chunking(int64_t n_rows, int Fi, int Fo, int64_t max_chunks, int64_t* rows_per_chunk, int64_t* n_chunks) {
    int tm, tn;
    tile_dims(tile_shape(Fi, Fo), &tm, &tn);
    const int64_t tiles = (int64_t)((Fi + tm - 1) / tm) * ((Fo + tn - 1) / tn);
    const int64_t want = std::min(std::max<int64_t>(1, 2048 / tiles), std::max<int64_t>(max_chunks, 1));
    int64_t per = std::max<int64_t>((n_rows + want - 1) / want, kMinChunkRows);
    per = (per + kStep - 1) / kStep * kStep;
    *rows_per_chunk = per;
    *n_chunks = (n_rows + per - 1) / per;
}

}  // namespace

extern "C" int64_t epp_weight_gradient_workspace(const epp_paths_t* paths, int k, int F_in, int F_out) {
    if (!paths) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    if (check_widths(F_in, F_out) != EPP_OK) return EPP_ERR_INVALID_ARG;
    int64_t per, chunks;
    chunking(k < 0 ? paths->n : paths->set_size[k], F_in, F_out, kNoChunkLimit, &per, &chunks);
    return std::max<int64_t>(chunks, 1) * F_in * F_out * (int64_t)sizeof(float);
}

namespace {

// Both weight-gradient entry points: partial sums of at most `max_chunks` blocks of rows go to
// `part` (max_chunks * F_in * F_out floats at least), a second kernel adds them in a fixed order.
int weight_gradient(const epp_paths* paths, int k, const float* Y, int F_in, const float* grad_X, int F_out,
                    float* grad_W, float* part, int64_t max_chunks, hipStream_t s) {
    const int32_t* ids = nullptr;
    int64_t n_rows = 0;
    EPP_TRY(row_set(paths, k, &ids, &n_rows));
    int64_t per, chunks;
    chunking(n_rows, F_in, F_out, max_chunks, &per, &chunks);
    if (chunks > 0) {
        const TileShape shape = tile_shape(F_in, F_out);
        int tm, tn;
        tile_dims(shape, &tm, &tn);
        const dim3 grid((unsigned)chunks, (unsigned)((F_in + tm - 1) / tm), (unsigned)((F_out + tn - 1) / tn));
        const bool vec = aligned4(F_in, F_out, Y, grad_X);
#define EPP_LAUNCH_WG(WM, WN, BM, BN)                                                                            \
    do {                                                                                                         \
        if (vec)                                                                                                 \
            hipLaunchKernelGGL((k_weight_gradient<WM, WN, BM, BN, true>), grid, dim3(kBlock), 0, s, ids, n_rows, \
                               per, Y, F_in, grad_X, F_out, part);                                               \
        else                                                                                                     \
            hipLaunchKernelGGL((k_weight_gradient<WM, WN, BM, BN, false>), grid, dim3(kBlock), 0, s, ids, n_rows, \
                               per, Y, F_in, grad_X, F_out, part);                                               \
    } while (0)
        switch (shape) {
            case T128x128: EPP_LAUNCH_WG(2, 2, 2, 2); break;
            case T128x64: EPP_LAUNCH_WG(2, 2, 2, 1); break;
            case T64x128: EPP_LAUNCH_WG(2, 2, 1, 2); break;
            case T64x64: EPP_LAUNCH_WG(2, 2, 1, 1); break;
            case T128x32: EPP_LAUNCH_WG(4, 1, 1, 1); break;
            case T32x128: EPP_LAUNCH_WG(1, 4, 1, 1); break;
        }
#undef EPP_LAUNCH_WG
    }
    const int64_t total = (int64_t)F_in * F_out;
    hipLaunchKernelGGL(k_weight_gradient_reduce, dim3((unsigned)((total + 15) / 16)), dim3(kBlock), 0, s,
                       static_cast<const float*>(part), chunks, total, grad_W);
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}

}  // namespace

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
    return weight_gradient(paths, k, Y, F_in, grad_X, F_out, grad_W, static_cast<float*>(workspace), kNoChunkLimit,
                           (hipStream_t)stream);
}

// ---- the entry point that allocates nothing --------------------------------------------------
// Partial sums of epp_weight_gradient_static: a file-scope device array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code the array's name is only a handle for the symbol lookup; the device address of the current
// GPU's copy comes from hipGetSymbolAddress, once per device, and is what the kernels receive.
constexpr size_t kStaticScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};  // per device; written once (the same value by any thread that races)
}  // namespace

int epp_static_scratch(float** ptr) {
    int dev = -1;
    EPP_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { epp_set_error("device index %d not supported", dev); return EPP_ERR_INVALID_ARG; }
    float* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        void* addr = nullptr;
        EPP_HIP_TRY(hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)));
        if (!addr) { epp_set_error("the static scratch array has no device address"); return EPP_ERR_HIP; }
        p = static_cast<float*>(addr);
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *ptr = p;
    return EPP_OK;
}

extern "C" int epp_weight_gradient_static(epp_paths_t* paths, int k, const float* Y, int F_in, const float* grad_X,
                                          int F_out, float* grad_W, epp_stream_t stream) {
    if (!paths || !Y || !grad_X || !grad_W) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(check_widths(F_in, F_out));
    const int64_t block_bytes = (int64_t)F_in * F_out * (int64_t)sizeof(float);
    if (block_bytes > (int64_t)kStaticScratchBytes) {
        epp_set_error("F_in * F_out = %lld exceeds the %lld elements the static scratch array holds; use "
                      "epp_weight_gradient with a workspace", (long long)F_in * F_out,
                      (long long)(kStaticScratchBytes / sizeof(float)));
        return EPP_ERR_TOO_LARGE;
    }
    float* part = nullptr;
    EPP_TRY(epp_static_scratch(&part));
    // as many blocks of rows as fit the array; every block is written in full before the second
    // kernel reads it, so nothing left over from an earlier call is ever read
    return weight_gradient(paths, k, Y, F_in, grad_X, F_out, grad_W, part, (int64_t)kStaticScratchBytes / block_bytes,
                           (hipStream_t)stream);
}

extern "C" int epp_input_gradient(epp_paths_t* paths, int k, const float* grad_X, int F_out, const float* W, int F_in,
                                  float* grad_Y, epp_stream_t stream) {
    if (!paths || !grad_X || !W || !grad_Y) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < -1 || k > paths->L) { epp_set_error("k=%d outside [-1, %d]", k, paths->L); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(check_widths(F_in, F_out));
    hipStream_t s = (hipStream_t)stream;
    const int32_t* ids = nullptr;
    int64_t n_rows = 0;
    EPP_TRY(row_set(paths, k, &ids, &n_rows));
    if (n_rows == 0) return EPP_OK;
    // rows are the long dimension: 128 of them per tile
    const TileShape shape = tile_shape(1 << 20, F_in);
    int tm, tn;
    tile_dims(shape, &tm, &tn);
    const dim3 grid((unsigned)((n_rows + tm - 1) / tm), (unsigned)((F_in + tn - 1) / tn));
    const bool vec = aligned4(F_out, F_out, grad_X, W);  // both operands are read along F_out
#define EPP_LAUNCH_IG(WM, WN, BM, BN)                                                                              \
    do {                                                                                                           \
        if (vec)                                                                                                   \
            hipLaunchKernelGGL((k_input_gradient<WM, WN, BM, BN, true>), grid, dim3(kBlock), 0, s, ids, n_rows,    \
                               grad_X, F_out, W, F_in, grad_Y);                                                    \
        else                                                                                                       \
            hipLaunchKernelGGL((k_input_gradient<WM, WN, BM, BN, false>), grid, dim3(kBlock), 0, s, ids, n_rows,   \
                               grad_X, F_out, W, F_in, grad_Y);                                                    \
    } while (0)
    switch (shape) {
        case T128x128: EPP_LAUNCH_IG(2, 2, 2, 2); break;
        case T128x64: EPP_LAUNCH_IG(2, 2, 2, 1); break;
        default: EPP_LAUNCH_IG(4, 1, 1, 1); break;  // T128x32
    }
#undef EPP_LAUNCH_IG
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}
