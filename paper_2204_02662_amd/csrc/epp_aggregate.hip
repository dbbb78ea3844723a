// Gather-reduce SpMM of backward aggregation (Alg. 1 / Alg. 2 aggregation loops) for
// gfx950, and the neighbour-group schedule it runs on (Sec. 2.2, Sec. 5).
//
// Neighbour grouping, re-derived for 64-lane wavefronts.  The path's entry array (the
// concatenated filtered neighbour lists, rows in ascending order) is cut into groups of gs
// consecutive entries.  A group is the scheduling unit, as in Sec. 2.2, but it is a slice
// of the *edge array*, not of one row: a long row is cut into several groups, and many
// short rows share one group.  Every group costs the same number of gathers, so
// wavefronts stay busy equally long whatever the degree distribution looks like.
//
// Execution (wave64):
//   * a source row of F floats is read by T lanes, VEC floats each (T*VEC >= F if it fits);
//     such a set of T lanes is a "slot" and owns one group: a wavefront carries 64/T groups;
//   * the slot streams its group's (column, weight) pairs U at a time, issues the U row
//     gathers back to back, and prefetches the next U pairs while they are in flight;
//   * the last entry of every row carries a flag (sign bit of the column id).  When a slot
//     meets it, the accumulated row is written to the output if the whole row lies inside the
//     group; the part of a row cut by a group boundary goes to one of the group's two
//     partial-row slots instead, and a small second kernel adds the pieces of every cut row in
//     group order.  No floating-point atomics: results are bit-reproducible;
//   * no cross-lane reduction is needed: lanes split the feature dimension, never a row's
//     neighbours, so the only cross-group combination is that sum of partial rows.

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>

#include "epp_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowEnd = kEntRowEnd, kCold = kEntCold, kOuterOnly = kEntOuterOnly, kColMask = kEntCol;

typedef int int2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
template <int VEC> struct VecT;
template <> struct VecT<1> { typedef float type; };
template <> struct VecT<2> { typedef float2v type; };
template <> struct VecT<4> { typedef float4v type; };
template <int VEC, class V> __device__ __forceinline__ float lane_get(const V& x, int i) {
    if constexpr (VEC == 1) return x; else return x[i];
}

// ---------------------------------------------------------------- schedule construction
// One thread per group: the row that holds the group's first entry (search in the row
// pointer; streamed rows are non-empty, so the pointer is strictly increasing).  Bit 31
// marks a group that starts inside a row.  A row cut by group boundaries is appended to
// cut_rows once, by the first boundary inside it.
__global__ __launch_bounds__(kBlock) void k_sched_groups(const int32_t* __restrict__ rowptr, int64_t n_rows, int gs,
                                                         int64_t n_groups, int32_t* __restrict__ group_row,
                                                         int32_t* __restrict__ cut_rows,
                                                         unsigned int* __restrict__ n_cut) {
    int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (g >= n_groups) return;
    const int64_t first = g * gs;
    int64_t lo = 0, hi = n_rows - 1;  // largest r with rowptr[r] <= first
    while (lo < hi) {
        int64_t mid = (lo + hi + 1) >> 1;
        if (rowptr[mid] <= first) lo = mid; else hi = mid - 1;
    }
    const int64_t start = rowptr[lo];
    const bool inside = start < first;
    group_row[g] = (int32_t)lo | (inside ? kRowEnd : 0);
    if (inside && start >= first - gs) cut_rows[atomicAdd(n_cut, 1u)] = (int32_t)lo;
}

// ------------------------------------------------------------------------- aggregation
// Zero the given rows (all-active graph: the vertices whose lists are empty).
__global__ __launch_bounds__(kBlock) void k_zero_rows(const int32_t* __restrict__ rows, int64_t n_rows,
                                                      const int32_t* __restrict__ row_ids, int F,
                                                      const unsigned int* __restrict__ only_bits,
                                                      float* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_rows * F) return;
    int64_t r = i / F;
    int f = (int)(i - r * F);
    int32_t v = rows[r];
    if (row_ids) v = row_ids[v];
    if (only_bits && !((only_bits[v >> 5] >> (v & 31)) & 1u)) return;
    out[(size_t)v * F + f] = 0.0f;
}

struct AggArgs {
    const int2v* cv;           // (column | row-end flag, weight bits) per entry
    const int32_t* group_row;  // per group: first row (bit 31: starts inside that row)
    const int32_t* row_ids;    // streamed row -> vertex; NULL: identity
    int64_t n_rows;            // streamed rows
    const float* in;
    float* out;
    int64_t nnz;
    int64_t n_groups;
    int F;
    int gs;
    int log2ns;                // feature slices spread over the XCDs (1 << log2ns of them)
    int has_cold;              // some entries carry the cold flag (host-side kernel choice)
    float* pieces;             // partial rows of the groups, [n_groups][2][F]
    // if-else selective scheduling only: membership bitmaps of the layer's rows and sources
    const unsigned int* row_bits;
    const unsigned int* src_bits;
    // source-partitioned layout only (part != 0): the entry array consists of 8 sections of entries
    // whose sources belong to one partition of the most referenced sources each, followed by the
    // section of all other entries; the groups of section x < 8 run on XCD x only.
    int part;                  // 0: off; 1: on
    int hot_rounds;            // rounds of 8 workgroups (one per XCD) that cover the longest hot section
    int total_rounds;          // hot_rounds + rounds of the last section
    int sec_g[10];             // first group of sections 0..8, then n_groups
    int n;                     // a row target t >= n is row t - n of the partial rows of the cut rows
                               // (float[slots][F]); INT_MAX without the partitioned layout
    uintptr_t part_delta;      // address of that array minus address of row n of `out`
    // launch for the inner path that shares these arrays only: 256 zero bytes, gathered in place of
    // the source row of an entry that is not the inner path's
    const float* zero;
};

template <int VEC>
__device__ __forceinline__ void write_row(float* __restrict__ o, const float (&acc)[VEC]) {
    typename VecT<VEC>::type r;
    if constexpr (VEC == 1) {
        r = acc[0];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) r[i] = acc[i];
    }
    __builtin_nontemporal_store(r, reinterpret_cast<typename VecT<VEC>::type*>(o));
}

// out[vertex(r), :] = sum of the partial rows of cut row r, in group order: the row starts in
// group g0 (whose end-of-group slot holds its head), runs through whole groups (end-of-group
// slots) and ends in group g1 (whose start-of-group slot holds its tail).  Fp lanes (a power of
// two >= min(F, 64)) work on one row, eight independent loads at a time; the additions stay in
// group order, so the result does not depend on the launch shape.
__global__ __launch_bounds__(kBlock) void k_combine_cut_rows(const int32_t* __restrict__ cut_rows, int64_t n_cut,
                                                             const int32_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ row_ids, int gs, int F,
                                                             int log2Fp, const float* __restrict__ pieces,
                                                             const unsigned int* __restrict__ only_bits,
                                                             float* __restrict__ out, int n,
                                                             float* __restrict__ vpart) {
    const int Fp = 1 << log2Fp;
    const int64_t k = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> log2Fp;
    if (k >= n_cut) return;
    const int32_t r = cut_rows[k];
    int32_t v = row_ids ? row_ids[r] : r;
    if (vpart && v >= n) {  // partitioned layout: the row is one section's share of a vertex's list
        out = vpart;
        v -= n;
    } else if (only_bits && !((only_bits[v >> 5] >> (v & 31)) & 1u)) {
        return;  // not a row of this launch (if-else baseline; inner path on shared arrays)
    }
    const int64_t g0 = rowptr[r] / gs, g1 = ((int64_t)rowptr[r + 1] - 1) / gs;
    for (int f = threadIdx.x & (Fp - 1); f < F; f += Fp) {
        float sum = 0.0f;
        int64_t g = g0;
        for (; g + 8 <= g1; g += 8) {
            float x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = pieces[((g + i) * 2 + 1) * F + f];
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += x[i];
        }
        for (; g < g1; ++g) sum += pieces[(g * 2 + 1) * F + f];
        sum += pieces[(g1 * 2) * F + f];
        out[(size_t)v * F + f] = sum;
    }
}

// Partitioned layout: out[vertex(m), :] = sum of the partial rows of split row m (one per section in
// which it has entries), in section order.  Fp lanes per row.
__global__ __launch_bounds__(kBlock) void k_combine_sections(const int32_t* __restrict__ mvert,
                                                             const int32_t* __restrict__ mptr, int64_t n_split, int F,
                                                             int log2Fp, const float* __restrict__ vpart,
                                                             const unsigned int* __restrict__ only_bits,
                                                             float* __restrict__ out) {
    const int Fp = 1 << log2Fp;
    const int64_t m = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> log2Fp;
    if (m >= n_split) return;
    const int32_t v = mvert[m];
    if (only_bits && !((only_bits[v >> 5] >> (v & 31)) & 1u)) return;  // not a row of the inner path
    const int s0 = mptr[m], s1 = mptr[m + 1];
    for (int f = threadIdx.x & (Fp - 1); f < F; f += Fp) {
        float x[9];
#pragma unroll
        for (int i = 0; i < 9; ++i) x[i] = s0 + i < s1 ? vpart[(size_t)(s0 + i) * F + f] : 0.0f;
        float sum = x[0];
#pragma unroll
        for (int i = 1; i < 9; ++i) sum += x[i];
        out[(size_t)v * F + f] = sum;
    }
}

// VEC floats per lane, T = 2^LOG2T lanes per source row, U gathers in flight per lane.
//
// The (column, weight) pairs of a group are staged through LDS: the T lanes of a slot load
// 4T consecutive pairs with four coalesced 8-byte loads, so every 128-byte line of the edge
// array is fetched once and fully used even when T is small and the 64/T groups of the
// wavefront lie far apart; each lane then reads the pair it needs as an LDS broadcast.
// The next 4T pairs are fetched into registers while the current ones are consumed.  The
// staging area is private to the wavefront (LDS operations of one wavefront execute in
// order), so no workgroup barrier is involved.
//
// The membership tests of the if-else variant cost a few registers, enough to lose a
// wavefront per SIMD; its register budget is capped to the occupancy of the plain kernel
// (five wavefronts per SIMD, four where the hot/cold branch of 8- and 16-byte lanes needs more).
//
// PART: the source-partitioned layout (block-to-group mapping by XCD, targets in the array of
// partial rows).  A variant of its own, so that the plain kernels keep their register budget (the
// few registers the extra addressing needs cost the 4-byte-lane kernel a wavefront per SIMD).
//
// INNER: the launch serves the inner path that shares these entry arrays.  An entry that is not
// the inner path's (kOuterOnly) is parked with weight zero and gathers from a block of zeros
// instead of its source row (which the inner layer must not read), so the gathers stay
// unconditional; a row left without any entry of the inner path is not written, unless its target
// is a partial row, which the adding kernels always read.
template <int VEC, int LOG2T, int U_, bool IFELSE, bool COLD, bool PART, bool INNER>
__global__ __launch_bounds__(kBlock, IFELSE ? ((COLD && VEC != 1) ? 4 : 5) : ((INNER && VEC == 1 && !PART) ? 5 : 4)) void k_aggregate(AggArgs a) {
    static_assert(!(IFELSE && PART), "the if-else baseline walks the graph as it is given");
    static_assert(!(IFELSE && INNER), "the if-else baseline has its own tests");
    constexpr int T = 1 << LOG2T;
    constexpr int S = 4 * T;              // pairs staged per slot
    constexpr int U = U_ < S ? U_ : S;    // S is a multiple of U
    typedef typename VecT<VEC>::type vec_t;
    typedef __attribute__((address_space(1))) const vec_t* gvec_ptr;  // global memory, stated for the loads
    __shared__ int2v stage_all[kBlock / 64][64 * 4];
    __shared__ int32_t ids_all[kBlock / 64][64];
    int2v* __restrict__ stage = stage_all[threadIdx.x >> 6] + (((threadIdx.x & 63) >> LOG2T) * S);
    // vertex ids of the slot's next T rows, streamed through LDS like the pairs (rows are
    // consumed in order, so one coalesced load serves T row ends)
    int32_t* __restrict__ ids = ids_all[threadIdx.x >> 6] + (((threadIdx.x & 63) >> LOG2T) * T);

    // XCD-aware mapping.  Workgroups are dealt round-robin to the 8 XCDs (each with its own
    // L2).  With ns > 1 feature slices, XCD x works on slice x % ns of every row only, so its
    // L2 holds ns times as many distinct source rows; the 8/ns XCDs of a slice share the
    // groups.  (A different dispatch order would cost locality, never correctness.)
    const int ns = 1 << a.log2ns;
    const int xcd = blockIdx.x & 7;
    const int slice = xcd & (ns - 1);
    int64_t g, g_end = a.n_groups;
    if constexpr (PART) {
        // Source-partitioned layout.  The first hot_rounds rounds of 8 workgroups are "hot":
        // the workgroup on XCD x takes the next groups of section x, so that L2 x only ever
        // holds the source rows of partition x.  The rounds after them share the last section.
        // (Interleaving the two kinds of rounds, so that gathers served by L2 and gathers served
        // from beyond it are in flight together, measured slower: 13.9 against 13.6 ms.)
        const int i = blockIdx.x >> 3;
        if (i < a.hot_rounds) {
            g = a.sec_g[xcd] + (int64_t)i * (kBlock >> LOG2T) + (threadIdx.x >> LOG2T);
            g_end = a.sec_g[xcd + 1];
        } else {
            g = a.sec_g[8] + ((int64_t)(i - a.hot_rounds) * 8 + xcd) * (kBlock >> LOG2T) + (threadIdx.x >> LOG2T);
        }
    } else {
        const int64_t qb = ((int64_t)(blockIdx.x >> 3) << (3 - a.log2ns)) + (xcd >> a.log2ns);
        g = qb * (kBlock >> LOG2T) + (threadIdx.x >> LOG2T);
    }
    const unsigned gi = (unsigned)g;  // n_groups < 2^31
    const bool has = g < g_end;  // slots past the end idle through the loop (no early exit: LDS order)
    const int t = threadIdx.x & (T - 1);
    const int64_t j0 = has ? g * a.gs : 0;
    const int len = has ? (int)(std::min<int64_t>(j0 + a.gs, a.nnz) - j0) : 0;
    const int2v* __restrict__ my = a.cv + j0;
    const int gr = has ? a.group_row[g] : 0;

    for (int f0 = 0; f0 < a.F; f0 += (T * VEC) << a.log2ns) {
        const int f = f0 + (slice * T + t) * VEC;
        const bool fok = f < a.F;
        const float* __restrict__ src = a.in + (fok ? f : 0);
        // first 4T pairs of the group: issued before anything that depends on the group table,
        // so that the two load chains (pairs -> gathers, group row -> vertex id) overlap
        // (pairs past the end of the group are clamped loads; they are neutralised only when they
        // are parked in LDS, so that nothing waits on a load right after issuing it)
        int2v pre[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            pre[i] = len > 0 ? __builtin_nontemporal_load(my + std::min(i * T + t, len - 1)) : int2v{0, 0};
        int r = gr & 0x7FFFFFFF;
        bool shared = gr < 0;  // the current row is shared with the previous group
        const int64_t r_last = a.n_rows - 1;
        int id_base = r;        // ids[] holds the vertices of rows id_base .. id_base + T - 1
        int32_t id_pre = 0;     // lane's share of the following T rows, already in flight
        int32_t v = r;
        if (a.row_ids) {
            const int32_t mine = has ? a.row_ids[std::min<int64_t>((int64_t)r + t, r_last)] : 0;
            id_pre = has ? a.row_ids[std::min<int64_t>((int64_t)r + T + t, r_last)] : 0;
            __builtin_amdgcn_wave_barrier();
            ids[t] = mine;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            v = ids[0];
        }
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        bool open = false;  // acc holds entries of a row whose end has not been met
        bool any = false;   // INNER: the current row has an entry of the inner path (in this group)
        for (int base = 0; base < len; base += S) {
            if constexpr (IFELSE) {
                // "is this neighbour active" test of selective scheduling, done for the 4T pairs
                // of a stage at once; inactive neighbours keep their flags but lose their column
                // (no valid id has all 30 bits set), so that the gather below skips them
                bool act[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int c = pre[i].x & kColMask;
                    act[i] = (a.src_bits[c >> 5] >> (c & 31)) & 1u;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (!act[i]) { pre[i].x |= kColMask; pre[i].y = 0; }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (INNER) {
                    if (base + i * T + t >= len) pre[i] = int2v{kOuterOnly, 0};
                    else if (pre[i].x & kOuterOnly) { pre[i].x &= ~kCold; pre[i].y = 0; }
                } else {
                    if (base + i * T + t >= len) { pre[i].x &= kColMask; pre[i].y = 0; }  // no row end, weight 0
                }
                stage[i * T + t] = pre[i];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (base + S < len) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    pre[i] = __builtin_nontemporal_load(my + std::min(base + S + i * T + t, len - 1));
            }
            const int n_here = std::min(S, len - base);
            for (int b = 0; b < n_here; b += U) {
                // U independent row reads back to back, then U multiply-adds
                int2v e[U];
                vec_t x[U];
#pragma unroll
                for (int u = 0; u < U; ++u) e[u] = stage[b + u];
                // (lanes past the last feature read feature 0 and never write: the loads stay
                // unconditional, so that nothing but their own results is ever waited on)
                bool act[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    act[u] = true;
                    if constexpr (IFELSE) act[u] = (e[u].x & kColMask) != kColMask;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (act[u]) {
                        const int c = e[u].x & kColMask;
                        gvec_ptr p = (gvec_ptr)(src + (size_t)c * (size_t)a.F);
                        if constexpr (INNER) p = (e[u].x & kOuterOnly) ? (gvec_ptr)a.zero : p;
                        if (COLD && (e[u].x & kCold)) {
                            // rarely referenced source: streamed, so that it does not evict hot rows from
                            // L2 and the memory-side cache.  (The address is laundered, and the branch
                            // ends in an empty statement the other one lacks, so that the two loads stay
                            // two instructions, each with its own cache policy.)
                            asm volatile("" : "+v"(p));
                            x[u] = __builtin_nontemporal_load(p);
                            asm volatile("");
                        } else {
                            x[u] = *p;
                        }
                        // the address stays live past both loads: a result register that overlapped it
                        // would make the second load wait for the first
                        if constexpr (COLD) asm volatile("" ::"v"(p));
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float w = __int_as_float(e[u].y);
                    if (act[u]) {  // (a skipped neighbour has no x[u]: nothing is zero-filled between loads)
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, lane_get<VEC>(x[u], i), acc[i]);
                    }
                    const int j = base + b + u;
                    if (j < len) open = true;
                    if constexpr (INNER) any |= !(e[u].x & kOuterOnly);
                    if (e[u].x < 0) {  // last entry of row r
                        bool wr = fok;
                        if constexpr (IFELSE) wr = fok && ((a.row_bits[v >> 5] >> (v & 31)) & 1u);
                        if constexpr (INNER) wr = fok && (any || (PART && v >= a.n));
                        // a row that began in an earlier group: its tail goes to the group's first slot
                        if (shared) {
                            // (the slot's address is formed here, from a value the compiler cannot
                            // trace, so that it is not kept in registers across the whole loop)
                            unsigned gl = gi;
                            asm volatile("" : "+v"(gl));
                            if (fok) write_row<VEC>(a.pieces + (size_t)(2 * gl) * (size_t)a.F + f, acc);
                        } else if (wr) {
                            // (a target >= n is one section's share of a cut row: it goes to the array of
                            // partial rows, addressed relative to `out` so that the store stays one instruction)
                            uintptr_t base = reinterpret_cast<uintptr_t>(a.out);
                            if constexpr (PART) base += v >= a.n ? a.part_delta : 0;
                            write_row<VEC>(reinterpret_cast<float*>(base) + ((size_t)v * (size_t)a.F + f), acc);
                        }
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
                        shared = false;
                        open = false;
                        any = false;
                        ++r;
                        if (!a.row_ids) {
                            v = r;
                        } else {
                            if (r - id_base == T) {  // the T staged ids are used up: switch to the next T
                                id_base = r;
                                __builtin_amdgcn_wave_barrier();
                                ids[t] = id_pre;
                                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                                __builtin_amdgcn_wave_barrier();
                                id_pre = a.row_ids[std::min<int64_t>((int64_t)r + T + t, r_last)];
                            }
                            v = ids[r - id_base];
                        }
                    }
                }
            }
        }
        // the group ends inside a row: that row continues in the next group
        if (open && fok) {
            unsigned gl = gi;
            asm volatile("" : "+v"(gl));
            write_row<VEC>(a.pieces + (size_t)(2 * gl + 1) * (size_t)a.F + f, acc);
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

// Lanes per source row and floats per lane for width F.  (16-byte accesses at 4-byte
// alignment for widths that are not a multiple of four were tried and measured no faster:
// F = 41: 1.34 vs 1.45 ms, F = 47: 0.51 vs 0.48 ms; the plain per-float form is kept.)
void row_shape(int F, bool aligned16, int* vec, int* log2T) {
    int v = (F % 4 == 0) ? 4 : (F % 2 == 0 ? 2 : 1);
    if (!aligned16) v = 1;
    int frags = (F + v - 1) / v;
    *vec = v;
    *log2T = std::min(ceil_log2(frags), 6);
}

template <int VEC, int LOG2T, int U, bool INNER>
void launch_plain(dim3 grid, dim3 block, hipStream_t s, const AggArgs& a) {
    if (a.part) {
        if (a.has_cold) hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, false, true, true, INNER>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, false, false, true, INNER>), grid, block, 0, s, a);
    } else {
        if (a.has_cold) hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, false, true, false, INNER>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, false, false, false, INNER>), grid, block, 0, s, a);
    }
}

template <int VEC, int LOG2T, int U>
void launch_one(hipStream_t s, const AggArgs& a) {
    const int64_t per_block = kBlock >> LOG2T;
    const int64_t blocks_per_slice = (a.n_groups + per_block - 1) / per_block;
    const int64_t xcds_per_slice = 8 >> a.log2ns;
    const int64_t q = a.part ? a.total_rounds : (blocks_per_slice + xcds_per_slice - 1) / xcds_per_slice;
    const dim3 grid((unsigned)(q * 8)), block(kBlock);
    if (a.row_bits) {
        if (a.has_cold) hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, true, true, false, false>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_aggregate<VEC, LOG2T, U, true, false, false, false>), grid, block, 0, s, a);
    } else if (a.zero) {
        launch_plain<VEC, LOG2T, U, true>(grid, block, s, a);
    } else {
        launch_plain<VEC, LOG2T, U, false>(grid, block, s, a);
    }
}

template <int VEC, int U>
void launch_vec(int log2T, hipStream_t s, const AggArgs& a) {
    switch (log2T) {
        case 0: launch_one<VEC, 0, U>(s, a); break;
        case 1: launch_one<VEC, 1, U>(s, a); break;
        case 2: launch_one<VEC, 2, U>(s, a); break;
        case 3: launch_one<VEC, 3, U>(s, a); break;
        case 4: launch_one<VEC, 4, U>(s, a); break;
        case 5: launch_one<VEC, 5, U>(s, a); break;
        default: launch_one<VEC, 6, U>(s, a); break;
    }
}

// ---- hot / cold sources -----------------------------------------------------------------
// Reference counts of the sources from a sample of the entries: every `stride`-th 64-entry
// segment is counted (ranking the often referenced sources does not need exact counts, and a
// full count means one atomic per entry, tens of thousands of them on the same hub address).
__global__ __launch_bounds__(kBlock) void k_count_sources(const int2v* __restrict__ cv, int64_t nnz, int64_t stride,
                                                          int* __restrict__ cnt) {
    const int64_t seg = ((int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)) * stride;
    const int64_t e = seg * 64 + (threadIdx.x & 63);
    if (e < nnz) atomicAdd(&cnt[cv[e].x & kColMask], 1);
}

// Quarter-octave bins of the reference count k >= 1: bin = k for k < 4, else
// 4 * floor(log2 k) + (next two bits of k); bin_floor(bin) is the smallest k of a bin.
constexpr int kCountBins = 128;
__host__ __device__ inline int count_bin(int k) {
    if (k < 4) return k;
    int e = 31 - __builtin_clz((unsigned)k);
    return 4 * e + ((k >> (e - 2)) & 3);
}
inline int bin_floor(int bin) {
    if (bin < 8) return bin;  // bins 4..7 do not occur (k = 4..7 map to bins 8..11)
    if (bin >= 124) return 0x7FFFFFFF;
    int e = bin >> 2, sub = bin & 3;
    return (4 + sub) << (e - 2);
}

__global__ __launch_bounds__(kBlock) void k_count_hist(const int* __restrict__ cnt, int64_t n,
                                                       unsigned long long* __restrict__ hist) {
    __shared__ int h[kCountBins];
    if (threadIdx.x < kCountBins) h[threadIdx.x] = 0;
    __syncthreads();
    // grid-stride, whole wavefronts per iteration (the ballots below need all 64 lanes)
    const int64_t span = (int64_t)gridDim.x * kBlock;
    for (int64_t base = (int64_t)blockIdx.x * kBlock + (threadIdx.x & ~63); base < n; base += span) {
        const int64_t v = base + (threadIdx.x & 63);
        const int k = v < n ? cnt[v] : 0;
        const int bin = k > 0 ? count_bin(k) : -1;
        // lanes with the same bin add once together (most lanes share a handful of small bins)
        unsigned long long todo = __ballot(bin >= 0);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int b = __shfl(bin, leader, 64);
            const unsigned long long same = __ballot(bin == b);
            if ((threadIdx.x & 63) == leader) atomicAdd(&h[b], __popcll(same));
            todo &= ~same;
        }
    }
    __syncthreads();
    if (threadIdx.x < kCountBins && h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], (unsigned long long)h[threadIdx.x]);
}

// One bit per vertex: referenced at least `thr` times in the sample.
__global__ __launch_bounds__(kBlock) void k_hot_bitmap(const int* __restrict__ cnt, int64_t n, int thr,
                                                       unsigned long long* __restrict__ bits) {
    int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const unsigned long long b = __ballot(v < n && cnt[v] >= thr);
    if ((threadIdx.x & 63) == 0 && (v >> 6) < ((n + 63) >> 6)) bits[v >> 6] = b;
}

// Set or clear the cold flag of every entry (hot == NULL: clear all).  Two entries per lane:
// 16-byte accesses, and the two bitmap lookups of a lane are in flight together.
typedef int int4v __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kBlock) void k_mark_cold(int2v* __restrict__ cv, int64_t nnz,
                                                      const unsigned int* __restrict__ hot) {
    const int64_t e = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 2;
    if (e >= nnz) return;
    if (e + 1 < nnz) {
        int4v x = *reinterpret_cast<const int4v*>(cv + e);  // the entry array is 16-byte aligned, e is even
        const int c0 = x.x & kColMask, c1 = x.z & kColMask;
        x.x &= ~kCold;
        x.z &= ~kCold;
        if (hot) {
            const unsigned int w0 = hot[c0 >> 5], w1 = hot[c1 >> 5];
            if (!((w0 >> (c0 & 31)) & 1u)) x.x |= kCold;
            if (!((w1 >> (c1 & 31)) & 1u)) x.z |= kCold;
        }
        *reinterpret_cast<int4v*>(cv + e) = x;
    } else {
        int2v x = cv[e];
        x.x &= ~kCold;
        const int c = x.x & kColMask;
        if (hot && !((hot[c >> 5] >> (c & 31)) & 1u)) x.x |= kCold;
        cv[e] = x;
    }
}

}  // namespace

// Structure-aware group size (Sec. 5) re-derived for 64-lane wavefronts.
//
// On this machine a group is a fixed-cost unit (gs gathers of one row fragment each), so
// load balance no longer depends on the degree distribution; what the group size trades is
// (a) the per-group cost and the partial rows of the rows cut by group boundaries (written by the
// groups, added by a second kernel), which fall as gs grows, against (b) having enough groups in flight, which
// matters for small paths.  As in Sec. 5 the size is predicted by a linear regression on
// structural features, learned from a generated corpus: 72 R-MAT and Chung-Lu graphs (2^12 to
// 2^21 vertices, average degree 4 to 64, 1 % and 10 % training vertices), two paths each,
// widths 16 / 64 / 128, every sample labelled with the best group size of an exhaustive
// power-of-two sweep on an MI355X (432 samples; `python -m paper_2204_02662_amd.studies gsfit
// --log2n 12,13,15,17,19,21` repeats the fit).  Model, in octaves:
//     log2 gs = 0.3557 log2(entries) + 0.1744 log2(entries per row) + 0.5099 log2(F) - 3.8123
// rounded to a power of two and clamped to [8, 4096].  Leave-one-graph-out, the predicted size
// costs 5 % over the best on average (39 % at worst); on the five benchmark configurations
// at most 4 % (most layers 0 %).
int epp_default_group_size(const epp_path* p, int F) {
    int forced = env_int("EPP_TUNE_GS", 0);
    if (forced > 0) return forced;
    if (p->nnz <= 0) return 8;
    const double entries = (double)p->nnz;
    const double per_row = entries / (double)std::max<int64_t>(p->n_stream_rows, 1);
    const double x = 0.3557363781872999 * std::log2(entries) + 0.1743635851953411 * std::log2(per_row) +
                     0.509920634920635 * std::log2((double)F) - 3.8123401416789617;
    const int e = (int)std::lround(std::min(std::max(x, 3.0), 12.0));
    return 1 << e;
}

int epp_build_schedule_over(const epp_path* p, const int32_t* rowptr, int64_t n_rows, int64_t nnz, int gs,
                            hipStream_t s, Schedule** out) {
    Schedule* sc = new Schedule();
    struct Guard { Schedule* s; ~Guard() { delete s; } } guard{sc};
    sc->gs = gs;
    const int64_t n_groups = (nnz + gs - 1) / gs;
    if (n_groups >= 0x7FFFFFFFll) { epp_set_error("too many groups"); return EPP_ERR_TOO_LARGE; }
    sc->n_groups = n_groups;
    const epp_alloc_t* al = epp_alloc_of(p);
    EPP_TRY(sc->group_row.alloc((size_t)n_groups * 4, al));
    EPP_TRY(sc->cut_rows.alloc((size_t)n_groups * 4, al));
    if (n_groups > 0) {
        DevBuf cnt;
        EPP_TRY(cnt.alloc(sizeof(unsigned int), al));
        EPP_HIP_TRY(hipMemsetAsync(cnt.p, 0, sizeof(unsigned int), s));
        hipLaunchKernelGGL(k_sched_groups, dim3((unsigned)((n_groups + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                           rowptr, n_rows, gs, n_groups, sc->group_row.as<int32_t>(),
                           sc->cut_rows.as<int32_t>(), cnt.as<unsigned int>());
        EPP_HIP_TRY(hipGetLastError());
        unsigned int h = 0;
        EPP_HIP_TRY(hipMemcpyAsync(&h, cnt.p, sizeof(h), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        sc->n_split_rows = h;
    }
    guard.s = nullptr;
    *out = sc;
    return EPP_OK;
}

int epp_build_schedule(epp_path* p, int gs, hipStream_t s, Schedule** out) {
    Schedule* sc = nullptr;
    EPP_TRY(epp_build_schedule_over(p, p->rowptr.as<int32_t>(), p->n_stream_rows, p->nnz, gs, s, &sc));
    p->scheds.push_back(sc);
    *out = sc;
    return EPP_OK;
}

int epp_launch_aggregate(epp_path* p, Schedule* sc, int log2_slices, const float* in, float* out, int F, hipStream_t s,
                         const unsigned int* row_bits, const unsigned int* src_bits, const Partition* part,
                         const unsigned int* inner_rows) {
    if (inner_rows && (row_bits || !p->has_inner || !p->zero_block.p)) {
        epp_set_error("the path's entries are not marked for an inner path");
        return EPP_ERR_INVALID_ARG;
    }
    int vec, log2T;
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    row_shape(F, aligned16, &vec, &log2T);
    // feature slices over the XCDs: each slice keeps whole 128-byte lines of a row
    int log2ns = part ? 0 : std::min(std::max(log2_slices, 0), 3);
    while (log2ns > 0 && ((log2T - log2ns) < 0 || ((vec * 4) << (log2T - log2ns)) < 128)) --log2ns;
    log2T -= log2ns;
    if (part) sc = part->sched;  // groups over the partitioned entry array
    const int32_t* row_ids = part ? part->tgt.as<int32_t>() : (p->row_ids.p ? p->row_ids.as<int32_t>() : nullptr);
    const int32_t* rowptr = part ? part->vptr.as<int32_t>() : p->rowptr.as<int32_t>();
    float* pieces = sc->pieces_for(F);
    if (sc->n_split_rows > 0 && !pieces) { epp_set_error("no partial-row buffer for F=%d", F); return EPP_ERR_INVALID_ARG; }
    if (p->n_empty_rows > 0 && !row_bits) {  // all-active graph: vertices without any entry become zero
        const int64_t total = p->n_empty_rows * F;
        hipLaunchKernelGGL(k_zero_rows, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                           p->empty_rows.as<int32_t>(), p->n_empty_rows, (const int32_t*)nullptr, F,
                           (const unsigned int*)nullptr, out);
    }
    if (sc->n_groups > 0) {
        AggArgs a;
        a.cv = reinterpret_cast<const int2v*>(part ? part->cv2.p : p->cv.p);
        a.group_row = sc->group_row.as<int32_t>();
        a.row_ids = row_ids;
        a.n_rows = part ? part->n_vrows : p->n_stream_rows;
        a.in = in;
        a.out = out;
        a.nnz = p->nnz;
        a.n_groups = sc->n_groups;
        a.F = F;
        a.gs = sc->gs;
        a.log2ns = log2ns;
        a.has_cold = p->cold_thr > 0 && (int64_t)F * 4 >= 256;  // narrow rows ignore the marks (bit 30 is masked)
        a.pieces = pieces;
        a.row_bits = row_bits;
        a.src_bits = src_bits;
        a.part = 0;
        a.hot_rounds = a.total_rounds = 0;
        for (int x = 0; x < 10; ++x) a.sec_g[x] = 0;
        a.n = 0x7FFFFFFF;
        a.part_delta = 0;
        a.zero = inner_rows ? p->zero_block.as<float>() : nullptr;
        if (part) {
            const int per_block = kBlock >> log2T;
            int hot = 0;
            for (int x = 0; x < 8; ++x) hot = std::max(hot, (part->sec_g[x + 1] - part->sec_g[x] + per_block - 1) / per_block);
            const int64_t rest_blocks = ((int64_t)part->sec_g[9] - part->sec_g[8] + per_block - 1) / per_block;
            a.part = 1;
            a.hot_rounds = hot;
            a.total_rounds = hot + (int)((rest_blocks + 7) / 8);
            for (int x = 0; x < 10; ++x) a.sec_g[x] = part->sec_g[x];
            a.n = (int)p->n;
            a.part_delta = reinterpret_cast<uintptr_t>(part->vpart) - reinterpret_cast<uintptr_t>(out) -
                           (uintptr_t)p->n * (uintptr_t)F * sizeof(float);
        }
        // gathers in flight per lane: 8 x 16 bytes, or 16 narrower ones
        if (vec == 4) launch_vec<4, 8>(log2T, s, a);
        else if (vec == 2) launch_vec<2, 16>(log2T, s, a);
        else launch_vec<1, 16>(log2T, s, a);
    }
    if (sc->n_split_rows > 0) {
        const int log2Fp = std::min(ceil_log2(F), 6);
        const int64_t total = sc->n_split_rows << log2Fp;
        hipLaunchKernelGGL(k_combine_cut_rows, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                           sc->cut_rows.as<int32_t>(), sc->n_split_rows, rowptr, row_ids, sc->gs, F,
                           log2Fp, pieces, row_bits ? row_bits : inner_rows, out, (int)p->n,
                           part ? part->vpart : (float*)nullptr);
    }
    if (part && part->n_split > 0) {
        const int log2Fp = std::min(ceil_log2(F), 6);
        const int64_t total = part->n_split << log2Fp;
        hipLaunchKernelGGL(k_combine_sections, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                           part->mvert.as<int32_t>(), part->mptr.as<int32_t>(), part->n_split, F, log2Fp,
                           part->vpart, inner_rows, out);
    }
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}

// Cache-locality choices of one (path, width), made from how often the path references each
// source.
//
// Hot / cold sources.  The gathered rows of a big path do not fit the caches (4 MB L2 per
// XCD, 256 MB memory-side cache); with plain loads the rarely referenced rows keep evicting
// the often referenced ones.  The most referenced sources, as many as fit the budget, stay
// "hot"; all entries of the others get the cold flag and are gathered with streaming loads.
//
// Source partition (epp_partition.hip).  The entries that reference the sources the eight L2s can
// hold together are moved into one section per XCD; built where the counts say it pays.
//
// XCD feature slicing (only without the source partition).  Two slices double the number of
// distinct rows an L2 can hold at the price of reading the index stream twice and of touching
// twice as many rows per gather instruction.  It pays when the hottest sources carry much of the
// traffic: it is switched on when rows are at least 512 bytes and the sources that fit with
// slicing, but not without, receive at least 6 % of all references (measured: R-MAT
// configuration, 8 % -> 16.5 to 15.3 ms; Chung-Lu configuration, 4 % -> 4.3 to 4.6 ms, left off).
int epp_tune_locality(epp_path* p, int F, int gs, hipStream_t s, int* log2_slices, Partition** part) {
    const int64_t budget_mb = env_int("EPP_TUNE_HOT_MB", 96);
    const int64_t rows_budget = budget_mb * (1ll << 20) / ((int64_t)F * 4);
    const int forced_slices = env_int("EPP_TUNE_LOG2_SLICES", -1);
    *log2_slices = forced_slices >= 0 ? forced_slices : 0;
    *part = nullptr;
    // (measured useful for rows of 256 bytes and more; at F = 47 the extra branch costs 3 %)
    const int part_mode = env_int("EPP_TUNE_PART", 1);
    if (p->nnz == 0 || ((int64_t)F * 4 < 256 && part_mode != 2)) return EPP_OK;
    const int64_t part_rows = forced_slices >= 0 ? 0 : epp_partition_hot_rows(F);  // a forced slicing is a measurement
    const bool want_cold = budget_mb > 0 && p->n_src > rows_budget && (int64_t)F * 4 >= 256;
    // (in the automatic mode only where the source rows do not fit the eight L2s together; forced,
    // for tests and measurements, at any width and size: on a graph whose narrow source rows all fit,
    // it lifts the L2 hit rate from 62-76 % to 93 % and the time stays the same, because such
    // launches are bound by the rate at which a CU's address unit and L1 take gather requests)
    const bool want_part = part_rows > 0 && (part_mode == 2 || (part_mode == 1 && p->n_src > part_rows));
    if (!want_cold && !want_part) return EPP_OK;

    // sampled reference counts, their histogram, and two bitmaps, in one allocation
    DevArena arena;
    DevBuf cnt, hist, hot, part_hot;
    const size_t hot_bytes = (size_t)((p->n + 63) / 64) * 8;
    EPP_TRY(arena.reserve(DevArena::rounded((size_t)p->n * 4) + DevArena::rounded(kCountBins * sizeof(unsigned long long)) +
                          2 * DevArena::rounded(hot_bytes), epp_alloc_of(p)));
    arena.take(&cnt, (size_t)p->n * 4);
    arena.take(&hist, kCountBins * sizeof(unsigned long long));
    arena.take(&hot, hot_bytes);
    arena.take(&part_hot, hot_bytes);
    EPP_HIP_TRY(hipMemsetAsync(cnt.p, 0, cnt.bytes, s));
    EPP_HIP_TRY(hipMemsetAsync(hist.p, 0, hist.bytes, s));
    // at most ~16 M sampled entries
    const int64_t n_seg = (p->nnz + 63) / 64;
    const int64_t stride = std::max<int64_t>(1, n_seg / (1 << 18));
    const int64_t n_sampled_seg = (n_seg + stride - 1) / stride;
    hipLaunchKernelGGL(k_count_sources, dim3((unsigned)((n_sampled_seg + (kBlock / 64) - 1) / (kBlock / 64))),
                       dim3(kBlock), 0, s, reinterpret_cast<const int2v*>(p->cv.p), p->nnz, stride, cnt.as<int>());
    hipLaunchKernelGGL(k_count_hist, dim3((unsigned)std::min<int64_t>((p->n + kBlock - 1) / kBlock, 2048)), dim3(kBlock), 0, s,
                       cnt.as<int>(), p->n, hist.as<unsigned long long>());
    EPP_HIP_TRY(hipGetLastError());
    unsigned long long h[kCountBins];
    EPP_HIP_TRY(hipMemcpyAsync(h, hist.p, sizeof(h), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    // smallest reference count of the sources kept when whole bins, most referenced first, are
    // taken while they fit `budget` rows (sources the sample never met are never kept)
    auto threshold_for = [&](int64_t budget) {
        int64_t kept = 0;
        int c = kCountBins - 1;
        for (; c >= 1; --c) {
            if (kept + (int64_t)h[c] > budget) break;
            kept += (int64_t)h[c];
        }
        return c < 1 ? 1 : bin_floor(c + 1 == 4 ? 8 : c + 1);  // bins 1..c are left out
    };

    // One set of marks per path, shared by all its widths: it is the one chosen for the largest
    // prepared width that marks at all (a smaller budget in rows; narrower widths then stream a
    // few rows they could have kept).  The marks therefore depend on which widths have been
    // prepared, never on the order of the calls.
    int new_thr = 0;  // > 0: the marks have to be set anew with this threshold
    if (want_cold && F > p->cold_F) {
        p->cold_F = F;
        const int thr = threshold_for(rows_budget);
        if (thr != p->cold_thr) {
            new_thr = thr;
            hipLaunchKernelGGL(k_hot_bitmap, dim3((unsigned)((p->n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                               cnt.as<int>(), p->n, thr, hot.as<unsigned long long>());
            EPP_HIP_TRY(hipGetLastError());
        }
    }

    if (want_part) {
        const int thr = threshold_for(part_rows);
        if (thr < 0x7FFFFFFF) {
            hipLaunchKernelGGL(k_hot_bitmap, dim3((unsigned)((p->n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                               cnt.as<int>(), p->n, thr, part_hot.as<unsigned long long>());
            EPP_HIP_TRY(hipGetLastError());
            // (new marks are set by the copy itself, from the bitmap)
            EPP_TRY(epp_build_partition(p, F, gs, part_hot.as<unsigned int>(), new_thr > 0 ? hot.as<unsigned int>() : nullptr,
                                        s, part));
        }
    }

    if (new_thr > 0) {
        // The canonical array needs the new marks only if something will still read it: not when it
        // is given back right after this width is prepared (a rebuilt one takes the marks of the copy).
        if (!(*part && epp_canonical_unused(p, F))) {
            hipLaunchKernelGGL(k_mark_cold, dim3((unsigned)((p->nnz + 2 * kBlock - 1) / (2 * kBlock))), dim3(kBlock), 0, s,
                               reinterpret_cast<int2v*>(p->cv.p), p->nnz, hot.as<unsigned int>());
            EPP_HIP_TRY(hipGetLastError());
        }
        EPP_HIP_TRY(hipStreamSynchronize(s));
        p->cold_thr = new_thr;
    }

    // (chosen whether or not the width has a partitioned layout: the if-else baseline never uses that layout)
    if (forced_slices < 0 && (int64_t)F * 4 >= 512) {
        // share of the references that goes to the sources ranked (rows one L2 holds) ..
        // (twice that), estimated from the bins (a bin's sources count as its lower bound)
        const int64_t l2_rows = (4ll << 20) / ((int64_t)F * 4);
        double refs_between = 0.0;
        int64_t rank = 0;
        for (int b = kCountBins - 1; b >= 1; --b) {
            const int64_t lo = std::max(rank, l2_rows), hi = std::min<int64_t>(rank + (int64_t)h[b], 2 * l2_rows);
            if (hi > lo) refs_between += (double)(hi - lo) * (double)bin_floor(b);
            rank += (int64_t)h[b];
        }
        if (refs_between >= 0.06 * (double)p->nnz / (double)stride) *log2_slices = 1;
    }
    EPP_HIP_TRY(hipStreamSynchronize(s));
    return EPP_OK;
}
