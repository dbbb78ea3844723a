// Gather-reduce SpMM of backward aggregation (Alg. 1 / Alg. 2 aggregation loops) for
// gfx950, and the neighbour-group schedule it runs on (Sec. 2.2, Sec. 5).
//
// Work decomposition (wave64):
//   * a source row of F floats is read by T lanes, VEC floats each (T*VEC >= F when it fits);
//   * a group (<= gs consecutive entries of one destination row) is processed by E "slots"
//     of T lanes; slot k takes entries k, k+E, k+2E, ...; partial sums meet through
//     cross-lane shuffles;
//   * a wavefront therefore carries 64/(T*E) groups at once.  Groups are binned by length
//     class, and E is chosen per class, so the groups of one wavefront have similar lengths.
//   * rows longer than gs are cut into several groups, whose partial sums are added to the
//     (pre-zeroed) output row with hardware fp32 atomics; all other rows use plain stores.

#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "epp_internal.h"

namespace {

constexpr int kBlock = 256;

struct ClassTab {
    int n_used;
    int n_waves;
    int wave_begin[EPP_NCLASS + 1];  // first wavefront of the k-th used class
    int group_begin[EPP_NCLASS];     // first group of that class in the group arrays
    int group_count[EPP_NCLASS];
    int log2E[EPP_NCLASS];           // slots per group
};

__device__ __forceinline__ int length_class(int len) { return len <= 1 ? 0 : 32 - __clz(len - 1); }

// ---------------------------------------------------------------- schedule construction
// counts[c] = groups of class c; counts[32] = rows cut into more than one group.
__global__ __launch_bounds__(kBlock) void k_sched_count(const int32_t* __restrict__ rowptr, int64_t n_rows, int gs,
                                                        unsigned long long* __restrict__ counts) {
    __shared__ int h[EPP_NCLASS + 1];
    if (threadIdx.x <= EPP_NCLASS) h[threadIdx.x] = 0;
    __syncthreads();
    int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r < n_rows) {
        int len = rowptr[r + 1] - rowptr[r];
        if (len <= gs) {
            atomicAdd(&h[length_class(len)], 1);
        } else {
            int q = len / gs, rem = len - q * gs;
            atomicAdd(&h[length_class(gs)], q);
            if (rem) atomicAdd(&h[length_class(rem)], 1);
            atomicAdd(&h[EPP_NCLASS], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x <= EPP_NCLASS && h[threadIdx.x])
        atomicAdd(&counts[threadIdx.x], (unsigned long long)h[threadIdx.x]);
}

// cursor[c] starts at the first slot of class c (cursor[32] at 0 for the split-row list).
__global__ __launch_bounds__(kBlock) void k_sched_fill(const int32_t* __restrict__ rowptr,
                                                       const int32_t* __restrict__ row_ids, int64_t n_rows, int gs,
                                                       unsigned int* __restrict__ cursor, int32_t* __restrict__ g_start,
                                                       int32_t* __restrict__ g_len, int32_t* __restrict__ g_dst,
                                                       int32_t* __restrict__ split_dst) {
    __shared__ int h[EPP_NCLASS + 1];
    __shared__ unsigned int base[EPP_NCLASS + 1];
    if (threadIdx.x <= EPP_NCLASS) h[threadIdx.x] = 0;
    __syncthreads();
    int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int start = 0, len = 0, q = 0, rem = 0, cq = 0, cr = 0, rank_q = 0, rank_r = 0, rank_s = 0;
    bool split = false, have = r < n_rows;
    if (have) {
        start = rowptr[r];
        len = rowptr[r + 1] - start;
        if (len <= gs) {
            rem = len;
            cr = length_class(len);
            rank_r = atomicAdd(&h[cr], 1);
        } else {
            split = true;
            q = len / gs;
            rem = len - q * gs;
            cq = length_class(gs);
            rank_q = atomicAdd(&h[cq], q);
            if (rem) { cr = length_class(rem); rank_r = atomicAdd(&h[cr], 1); }
            rank_s = atomicAdd(&h[EPP_NCLASS], 1);
        }
    }
    __syncthreads();
    if (threadIdx.x <= EPP_NCLASS && h[threadIdx.x])
        base[threadIdx.x] = atomicAdd(&cursor[threadIdx.x], (unsigned int)h[threadIdx.x]);
    __syncthreads();
    if (!have) return;
    const int32_t dst = row_ids ? row_ids[r] : (int32_t)r;
    const int flag = split ? (int)0x80000000u : 0;
    for (int i = 0; i < q; ++i) {
        unsigned int g = base[cq] + rank_q + i;
        g_start[g] = start + i * gs;
        g_len[g] = gs | flag;
        g_dst[g] = dst;
    }
    if (!split || rem) {
        unsigned int g = base[cr] + rank_r;
        g_start[g] = start + q * gs;
        g_len[g] = rem | flag;
        g_dst[g] = dst;
    }
    if (split) split_dst[base[EPP_NCLASS] + rank_s] = dst;
}

// ------------------------------------------------------------------------- aggregation
__global__ __launch_bounds__(kBlock) void k_zero_rows(const int32_t* __restrict__ rows, int64_t n_rows, int F,
                                                      float* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_rows * F) return;
    int64_t r = i / F;
    int f = (int)(i - r * F);
    out[(size_t)rows[r] * F + f] = 0.0f;
}

template <int VEC> struct Vec;
template <> struct Vec<1> { float v[1]; };
template <> struct alignas(8) Vec<2> { float v[2]; };
template <> struct alignas(16) Vec<4> { float v[4]; };

// VEC floats per lane, T lanes per source row, U gathers in flight per lane.
template <int VEC, int LOG2T, int U>
__global__ __launch_bounds__(kBlock) void k_aggregate(const int2* __restrict__ cv, const int32_t* __restrict__ g_start,
                                                      const int32_t* __restrict__ g_len,
                                                      const int32_t* __restrict__ g_dst, const float* __restrict__ in,
                                                      float* __restrict__ out, int F, ClassTab tab) {
    constexpr int T = 1 << LOG2T;
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (wave >= tab.n_waves) return;
    int k = 0;
    while (k + 1 < tab.n_used && wave >= tab.wave_begin[k + 1]) ++k;
    const int log2E = tab.log2E[k];
    const int E = 1 << log2E;
    const int log2W = LOG2T + log2E;
    const int sub = lane >> log2W;                // which group of this wavefront
    const int slot = (lane >> LOG2T) & (E - 1);   // which slot of the group
    const int t = lane & (T - 1);                 // which fragment of the row
    const int gi = ((wave - tab.wave_begin[k]) << (6 - log2W)) + sub;
    int start = 0, len = 0, dst = 0;
    bool split = false;
    const bool has = gi < tab.group_count[k];
    if (has) {
        const int g = tab.group_begin[k] + gi;
        start = g_start[g];
        const int lf = g_len[g];
        len = lf & 0x7FFFFFFF;
        split = lf < 0;
        dst = g_dst[g];
    }
    const int2* __restrict__ my = cv + start;
    for (int f0 = 0; f0 < F; f0 += T * VEC) {
        const int f = f0 + t * VEC;
        const bool fok = f < F;
        const float* __restrict__ src = in + f;
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        if (fok) {
            for (int j = slot; j < len; j += U << log2E) {
                int2 e[U];
                Vec<VEC> x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int jj = j + (u << log2E);
                    e[u] = jj < len ? my[jj] : make_int2(-1, 0);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (e[u].x >= 0) {
                        x[u] = *reinterpret_cast<const Vec<VEC>*>(src + (size_t)e[u].x * (size_t)F);
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) x[u].v[i] = 0.0f;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float w = __int_as_float(e[u].y);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, x[u].v[i], acc[i]);
                }
            }
        }
        // partial sums of the E slots meet in every slot
        for (int s = T; s < (T << log2E); s <<= 1) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], s, 64);
        }
        if (has && slot == 0 && fok) {
            float* __restrict__ o = out + (size_t)dst * (size_t)F + f;
            if (split) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) unsafeAtomicAdd(o + i, acc[i]);
            } else {
                Vec<VEC> r;
#pragma unroll
                for (int i = 0; i < VEC; ++i) r.v[i] = acc[i];
                *reinterpret_cast<Vec<VEC>*>(o) = r;
            }
        }
    }
}

int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : dflt;
}

int ceil_log2(int x) {
    int l = 0;
    while ((1 << l) < x) ++l;
    return l;
}

// Lanes per source row and floats per lane for width F.
void row_shape(int F, int* vec, int* log2T) {
    int v = (F % 4 == 0) ? 4 : (F % 2 == 0 ? 2 : 1);
    int frags = (F + v - 1) / v;
    int lt = std::min(ceil_log2(frags), 6);
    *vec = v;
    *log2T = lt;
}

template <int VEC, int LOG2T>
void launch_one(unsigned blocks, hipStream_t s, const epp_path* p, const Schedule* sc, const float* in, float* out, int F,
                const ClassTab& tab) {
    hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, 8>), dim3(blocks), dim3(kBlock), 0, s, p->cv.as<int2>(),
                       sc->g_start.as<int32_t>(), sc->g_len.as<int32_t>(), sc->g_dst.as<int32_t>(), in, out, F, tab);
}

template <int VEC>
void launch_vec(int log2T, unsigned blocks, hipStream_t s, const epp_path* p, const Schedule* sc, const float* in,
                float* out, int F, const ClassTab& tab) {
    switch (log2T) {
        case 0: launch_one<VEC, 0>(blocks, s, p, sc, in, out, F, tab); break;
        case 1: launch_one<VEC, 1>(blocks, s, p, sc, in, out, F, tab); break;
        case 2: launch_one<VEC, 2>(blocks, s, p, sc, in, out, F, tab); break;
        case 3: launch_one<VEC, 3>(blocks, s, p, sc, in, out, F, tab); break;
        case 4: launch_one<VEC, 4>(blocks, s, p, sc, in, out, F, tab); break;
        case 5: launch_one<VEC, 5>(blocks, s, p, sc, in, out, F, tab); break;
        default: launch_one<VEC, 6>(blocks, s, p, sc, in, out, F, tab); break;
    }
}

}  // namespace

// Upper bound on entries per group for width F.  A group is worked on by at most 64/T
// slots; the bound keeps every slot to a few dozen gathers so that long rows spread over
// many wavefronts, while staying large enough that the atomic write-back of a split row
// (F atomics per group) is a small fraction of the F * gs floats the group gathers.
int epp_default_group_size(const epp_path* p, int F) {
    int vec, log2T;
    row_shape(F, &vec, &log2T);
    const int slots = 64 >> log2T;
    const int iters = env_int("EPP_TUNE_GROUP_ITERS", 64);
    int64_t gs = (int64_t)slots * iters;
    gs = std::max<int64_t>(gs, 64);
    (void)p;
    return (int)std::min<int64_t>(gs, 1 << 20);
}

int epp_build_schedule(epp_path* p, int gs, hipStream_t s, Schedule** out) {
    Schedule* sc = new Schedule();
    struct Guard { Schedule* s; ~Guard() { delete s; } } guard{sc};
    sc->gs = gs;
    DevBuf counts;
    EPP_TRY(counts.alloc((EPP_NCLASS + 1) * sizeof(unsigned long long)));
    EPP_HIP_TRY(hipMemsetAsync(counts.p, 0, counts.bytes, s));
    const unsigned blocks = (unsigned)((p->n_rows + kBlock - 1) / kBlock);
    unsigned long long host[EPP_NCLASS + 1] = {};
    if (blocks) {
        hipLaunchKernelGGL(k_sched_count, dim3(blocks), dim3(kBlock), 0, s, p->rowptr.as<int32_t>(), p->n_rows, gs,
                           counts.as<unsigned long long>());
        EPP_HIP_TRY(hipGetLastError());
        EPP_HIP_TRY(hipMemcpyAsync(host, counts.p, sizeof(host), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
    }
    // longest classes first: the long groups start early and the short ones fill the tail
    int64_t total = 0;
    unsigned int cursor[EPP_NCLASS + 1] = {};
    for (int c = EPP_NCLASS - 1; c >= 0; --c) {
        sc->class_count[c] = (int64_t)host[c];
        sc->class_begin[c] = total;
        cursor[c] = (unsigned int)total;
        total += (int64_t)host[c];
    }
    if (total >= 0x7FFFFFFFll) { epp_set_error("too many groups"); return EPP_ERR_TOO_LARGE; }
    sc->n_groups = total;
    sc->n_split_rows = (int64_t)host[EPP_NCLASS];
    EPP_TRY(sc->g_start.alloc((size_t)total * 4));
    EPP_TRY(sc->g_len.alloc((size_t)total * 4));
    EPP_TRY(sc->g_dst.alloc((size_t)total * 4));
    EPP_TRY(sc->split_dst.alloc((size_t)sc->n_split_rows * 4));
    if (blocks) {
        DevBuf cur;
        EPP_TRY(cur.alloc(sizeof(cursor)));
        EPP_HIP_TRY(hipMemcpyAsync(cur.p, cursor, sizeof(cursor), hipMemcpyHostToDevice, s));
        hipLaunchKernelGGL(k_sched_fill, dim3(blocks), dim3(kBlock), 0, s, p->rowptr.as<int32_t>(),
                           p->all_rows ? nullptr : p->row_ids.as<int32_t>(), p->n_rows, gs, cur.as<unsigned int>(),
                           sc->g_start.as<int32_t>(), sc->g_len.as<int32_t>(), sc->g_dst.as<int32_t>(),
                           sc->split_dst.as<int32_t>());
        EPP_HIP_TRY(hipGetLastError());
        EPP_HIP_TRY(hipStreamSynchronize(s));
    }
    guard.s = nullptr;
    p->scheds.push_back(sc);
    *out = sc;
    return EPP_OK;
}

int epp_launch_aggregate(epp_path* p, Schedule* sc, int lanes_hint, const float* in, float* out, int F,
                         hipStream_t s) {
    if (sc->n_groups == 0) return EPP_OK;
    int vec, log2T;
    row_shape(F, &vec, &log2T);
    if (vec > 1 && ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & (uintptr_t)(vec * 4 - 1))) {
        vec = 1;  // base pointers not aligned for vector access
        log2T = std::min(ceil_log2(F), 6);
    }
    const int max_log2E = std::min(6 - log2T, lanes_hint > 0 ? std::max(ceil_log2(lanes_hint) - log2T, 0) : 6);
    const int slot_iters = std::max(env_int("EPP_TUNE_SLOT_ITERS", 8), 1);

    ClassTab tab;
    std::memset(&tab, 0, sizeof(tab));
    int64_t waves = 0;
    for (int c = EPP_NCLASS - 1; c >= 0; --c) {
        if (sc->class_count[c] == 0) continue;
        // class c holds lengths up to 2^c: widen until a slot has about slot_iters entries
        int want = c - ceil_log2(slot_iters);
        int log2E = std::min(std::max(want, 0), max_log2E);
        int groups_per_wave = 64 >> (log2T + log2E);
        int k = tab.n_used++;
        tab.wave_begin[k] = (int)waves;
        tab.group_begin[k] = (int)sc->class_begin[c];
        tab.group_count[k] = (int)sc->class_count[c];
        tab.log2E[k] = log2E;
        waves += (sc->class_count[c] + groups_per_wave - 1) / groups_per_wave;
    }
    if (waves >= 0x7FFFFFFFll) { epp_set_error("too many wavefronts"); return EPP_ERR_TOO_LARGE; }
    tab.wave_begin[tab.n_used] = (int)waves;
    tab.n_waves = (int)waves;

    if (sc->n_split_rows > 0) {
        const int64_t total = sc->n_split_rows * F;
        hipLaunchKernelGGL(k_zero_rows, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                           sc->split_dst.as<int32_t>(), sc->n_split_rows, F, out);
    }
    const unsigned blocks = (unsigned)((waves + (kBlock / 64) - 1) / (kBlock / 64));
    switch (vec) {
        case 4: launch_vec<4>(log2T, blocks, s, p, sc, in, out, F, tab); break;
        case 2: launch_vec<2>(log2T, blocks, s, p, sc, in, out, F, tab); break;
        default: launch_vec<1>(log2T, blocks, s, p, sc, in, out, F, tab); break;
    }
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}
