// Execution path preparing on the GPU (Sec. 4): frontier expansion from the training set
// (Theorem 1's sets N^k), stable extraction of the filtered neighbour lists, row
// renumbering and prefix-sum compaction into compact CSR.  Hand-written for gfx950, wave64.
//
// One level k -> k+1 is two streaming passes over the edge array and two over the rows:
//   edge_mask     keep[j] = (col[j] in N^k) as one 64-bit ballot per 64 edges + tile counts
//   scan          exclusive scan of the tile counts (one readback: nnz of the path)
//   edge_extract  stable compaction of (col, val) through the ballots; also stores the
//                 running count at every 64-edge boundary
//   row_flags     filtered row pointer of every vertex from those counts; a vertex is in
//                 N^{k+1} iff its filtered list is non-empty -> next bitmap
//   bitmap_count / scan / bitmap_compact   ascending ids of N^{k+1} + compact row pointer
// All kept entries belong to rows of N^{k+1} by definition, so compacting the edge array
// alone yields the path's entries in canonical order.

#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "epp_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kSegsPerTile = 32;  // 32 ballots of 64 edges = 2048 edges per workgroup
constexpr int kWordsPerTile = 256;

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ unsigned long long low_mask(int lane) { return (1ull << lane) - 1ull; }

// Inclusive scan across the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan over the 256 threads of a workgroup; *total receives the block sum.
__device__ __forceinline__ int block_exclusive_scan(int x, int* total) {
    __shared__ int wave_sum[4];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    int incl = wave_inclusive_scan(x);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) base += wave_sum[w];
        all += wave_sum[w];
    }
    __syncthreads();
    *total = all;
    return base + incl - x;
}

// N^0 = V_t as a bitmap; ids outside [0, n) raise the error flag instead of being written.
__global__ __launch_bounds__(kBlock) void k_mark_training(const int32_t* __restrict__ ids, int64_t n_ids, int64_t n,
                                                          unsigned int* __restrict__ bitmap32,
                                                          int* __restrict__ err) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_ids) return;
    int32_t v = ids[i];
    if (v < 0 || v >= n) { atomicOr(err, 1); return; }
    atomicOr(&bitmap32[v >> 5], 1u << (v & 31));
}

// keep-mask of every 64-edge segment and kept entries per tile.
//
// `prev` is the keep-mask of the previous level, or NULL.  If N^{k-1} is a
// subset of N^k (*not_subset == 0; always the case when every vertex has a self-loop), an entry
// kept at the previous level has its column in N^{k-1}, hence in N^k, and is kept again: only
// the other entries are loaded and looked up.  Once the sets are close to saturation this
// turns a pass bound by the rate of random bitmap lookups into a scan of the previous mask.
//
// Columns are range-checked where they are loaded (every entry at the first level): an id outside
// [0, n) raises bit 1 of *err and is treated as not kept, so it is never used as an index.
__global__ __launch_bounds__(kBlock) void k_edge_mask(const int32_t* __restrict__ col, int64_t nnz, int64_t n_seg,
                                                      int64_t n, const unsigned int* __restrict__ bitmap32,
                                                      const unsigned long long* __restrict__ prev,
                                                      const int* __restrict__ not_subset,
                                                      unsigned long long* __restrict__ mask,
                                                      int* __restrict__ tile_count, int* __restrict__ err) {
    __shared__ int wave_cnt[4];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    int cnt = 0;
    // a wavefront owns 8 consecutive segments; all column loads, then all bitmap lookups, are
    // issued back to back so that the two dependent memory latencies are paid once per tile
    constexpr int kPerWave = kSegsPerTile / 4;
    const int64_t seg0 = (int64_t)blockIdx.x * kSegsPerTile + wave * kPerWave;
    const bool use_prev = prev && *not_subset == 0;
    bool known[kPerWave];
    int32_t c[kPerWave];
    unsigned int w[kPerWave];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const unsigned long long pm = (use_prev && seg0 + i < n_seg) ? prev[seg0 + i] : 0ull;
        known[i] = (pm >> lane) & 1ull;
    }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const int64_t e = (seg0 + i) * 64 + lane;
        c[i] = (e < nnz && !known[i]) ? col[e] : -1;
    }
    bool bad = false;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const int64_t e = (seg0 + i) * 64 + lane;
        if (e < nnz && !known[i] && (c[i] < 0 || c[i] >= n)) { bad = true; c[i] = -1; }
    }
    if (bad) atomicOr(err, 2);
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) w[i] = c[i] >= 0 ? bitmap32[c[i] >> 5] : 0u;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const bool keep = known[i] || (c[i] >= 0 && ((w[i] >> (c[i] & 31)) & 1u));
        const unsigned long long m = __ballot(keep);
        if (lane == 0 && seg0 + i < n_seg) mask[seg0 + i] = m;
        cnt += __popcll(m);
    }
    if (lane == 0) wave_cnt[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) tile_count[blockIdx.x] = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
}

// Exclusive scan of `n` counts (per-tile numbers of kept entries or set bits).  A workgroup of
// 1024 threads, kScanPerThread consecutive counts each, scans a chunk of kScanChunk counts;
// k_scan_counts walks all chunks in one workgroup (short arrays), the three-kernel form scans
// the chunks in parallel, then the chunk sums, then adds the chunk offsets.
constexpr int kScanPerThread = 8;
constexpr int kScanChunk = 1024 * kScanPerThread;

// Scans in[base .. base + kScanChunk) into out, starting from `carry`; returns the chunk's sum
// to every thread.  Called by all 1024 threads of the workgroup.
__device__ __forceinline__ int scan_chunk(const int* __restrict__ in, int* __restrict__ out, int64_t n, int64_t base,
                                          int carry) {
    __shared__ int wave_sum[16];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int64_t i0 = base + (int64_t)threadIdx.x * kScanPerThread;
    int x[kScanPerThread];
    int mine = 0;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        x[j] = i0 + j < n ? in[i0 + j] : 0;
        mine += x[j];
    }
    const int incl = wave_inclusive_scan(mine);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int off = carry, all = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) off += wave_sum[w];
        all += wave_sum[w];
    }
    __syncthreads();  // wave_sum is reused by the next call
    off += incl - mine;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        if (i0 + j < n) out[i0 + j] = off;
        off += x[j];
    }
    return all;
}

__global__ __launch_bounds__(1024) void k_scan_counts(const int* __restrict__ in, int* __restrict__ out, int64_t n,
                                                      long long* __restrict__ total) {
    int carry = 0;
    for (int64_t base = 0; base < n; base += kScanChunk) carry += scan_chunk(in, out, n, base, carry);
    if (threadIdx.x == 0) *total = carry;
}

__global__ __launch_bounds__(1024) void k_scan_chunks(const int* __restrict__ in, int* __restrict__ out, int64_t n,
                                                      int* __restrict__ chunk_sum) {
    const int all = scan_chunk(in, out, n, (int64_t)blockIdx.x * kScanChunk, 0);
    if (threadIdx.x == 0) chunk_sum[blockIdx.x] = all;
}

__global__ __launch_bounds__(1024) void k_scan_add_offsets(int* __restrict__ out, int64_t n,
                                                           const int* __restrict__ chunk_base) {
    const int off = chunk_base[blockIdx.x];
    const int64_t i0 = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanPerThread;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j)
        if (i0 + j < n) out[i0 + j] += off;
}

// seg_base[s] = number of kept entries before segment s: the tile's offset plus the kept
// entries of the tile's earlier segments.  One wavefront per tile.
__global__ __launch_bounds__(64) void k_seg_base(const unsigned long long* __restrict__ mask, int64_t n_seg,
                                                 const int* __restrict__ tile_base, int* __restrict__ seg_base) {
    const int lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kSegsPerTile + lane;
    const int c = (lane < kSegsPerTile && seg < n_seg) ? __popcll(mask[seg]) : 0;
    const int incl = wave_inclusive_scan(c);
    if (lane < kSegsPerTile && seg < n_seg) seg_base[seg] = tile_base[blockIdx.x] + incl - c;
}

// Stable compaction of the kept entries into interleaved (col, val) pairs: a kept entry of
// segment s goes to seg_base[s] + (kept entries before it in the segment).  With `inner` (the
// keep-mask of the level before, a subset of `mask`) the entries that level did not keep get
// the kEntOuterOnly mark: the path of the level before will run on this array.
__global__ __launch_bounds__(kBlock) void k_edge_extract(const int32_t* __restrict__ col, const float* __restrict__ val,
                                                         int64_t n_seg, const unsigned long long* __restrict__ mask,
                                                         const unsigned long long* __restrict__ inner,
                                                         const int* __restrict__ seg_base, int2* __restrict__ cv) {
    const int wave = threadIdx.x >> 6, lane = lane_id();
    constexpr int kPerWave = kSegsPerTile / 4;
    unsigned long long m[kPerWave], fr[kPerWave];
    int sb[kPerWave];
    int2 x[kPerWave];
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const int64_t seg = (int64_t)blockIdx.x * kSegsPerTile + wave * kPerWave + i;
        m[i] = seg < n_seg ? mask[seg] : 0ull;
        fr[i] = (inner && seg < n_seg) ? (m[i] & ~inner[seg]) : 0ull;
        sb[i] = seg < n_seg ? seg_base[seg] : 0;
    }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        const int64_t e = ((int64_t)blockIdx.x * kSegsPerTile + wave * kPerWave + i) * 64 + lane;
        if ((m[i] >> lane) & 1ull)
            x[i] = make_int2(col[e] | (((fr[i] >> lane) & 1ull) ? kEntOuterOnly : 0), __float_as_int(val[e]));
    }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
        if ((m[i] >> lane) & 1ull) cv[sb[i] + __popcll(m[i] & low_mask(lane))] = x[i];
    }
}

// Filtered row pointer of every vertex and membership of N^{k+1}.  A row pointer that does not
// rise from 0 to nnz raises bit 0 of *err; the offending row is treated as empty, so no index
// outside the mask arrays is formed.
__global__ __launch_bounds__(kBlock) void k_row_flags(const int32_t* __restrict__ rowptr, int64_t n, int64_t nnz,
                                                      const unsigned long long* __restrict__ mask,
                                                      const int* __restrict__ seg_base,
                                                      const long long* __restrict__ total_p,
                                                      int* __restrict__ newptr,
                                                      unsigned long long* __restrict__ bitmap_next,
                                                      int* __restrict__ err) {
    int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    bool flag = false;
    if (v < n) {
        const int total = (int)*total_p;  // kept entries of the level (the host has not read it yet)
        int64_t p0 = rowptr[v], p1 = rowptr[v + 1];
        if (p0 < 0 || p1 < p0 || p1 > nnz || (v == 0 && p0 != 0) || (v == n - 1 && p1 != nnz)) {
            atomicOr(err, 1);
            p0 = p1 = nnz;
        }
        int a = p0 >= nnz ? total : seg_base[p0 >> 6] + __popcll(mask[p0 >> 6] & low_mask((int)(p0 & 63)));
        int b = p1 >= nnz ? total : seg_base[p1 >> 6] + __popcll(mask[p1 >> 6] & low_mask((int)(p1 & 63)));
        newptr[v] = a;
        if (v == n - 1) newptr[n] = b;
        flag = b > a;
    }
    unsigned long long bal = __ballot(flag);
    if (lane_id() == 0 && (v >> 6) < ((n + 63) >> 6)) bitmap_next[v >> 6] = bal;
}

__global__ __launch_bounds__(kBlock) void k_bitmap_count(const unsigned long long* __restrict__ bitmap, int64_t n_words,
                                                         int* __restrict__ tile_count) {
    int64_t w = (int64_t)blockIdx.x * kWordsPerTile + threadIdx.x;
    int c = w < n_words ? __popcll(bitmap[w]) : 0;
    int total;
    (void)block_exclusive_scan(c, &total);
    if (threadIdx.x == 0) tile_count[blockIdx.x] = total;
}

// Ascending ids of the set bits; optionally the compact row pointer gathered from newptr.
__global__ __launch_bounds__(kBlock) void k_bitmap_compact(const unsigned long long* __restrict__ bitmap,
                                                           int64_t n_words, const int* __restrict__ tile_base,
                                                           const int* __restrict__ newptr, int32_t* __restrict__ ids,
                                                           int32_t* __restrict__ ptr_out, int64_t n_set,
                                                           int total_nnz) {
    __shared__ int wbase[kWordsPerTile];
    int64_t w = (int64_t)blockIdx.x * kWordsPerTile + threadIdx.x;
    int c = w < n_words ? __popcll(bitmap[w]) : 0;
    int total;
    wbase[threadIdx.x] = block_exclusive_scan(c, &total);
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int tb = tile_base[blockIdx.x];
    for (int i = wave; i < kWordsPerTile; i += 4) {
        int64_t ww = (int64_t)blockIdx.x * kWordsPerTile + i;
        if (ww >= n_words) break;
        unsigned long long m = bitmap[ww];
        if ((m >> lane) & 1ull) {
            int r = tb + wbase[i] + __popcll(m & low_mask(lane));
            int32_t v = (int32_t)(ww * 64 + lane);
            ids[r] = v;
            if (ptr_out) ptr_out[r] = newptr[v];
        }
    }
    if (ptr_out && blockIdx.x == 0 && threadIdx.x == 0) ptr_out[n_set] = total_nnz;
}

__device__ __forceinline__ int length_class(int len) { return len <= 1 ? 0 : 32 - __clz(len - 1); }

// Row-length histogram by class and the maximal length.  Grid-stride; a wavefront adds one
// count per distinct class among its 64 rows (ballots), a workgroup 33 global atomics in all.
__global__ __launch_bounds__(kBlock) void k_len_hist(const int32_t* __restrict__ rowptr, int64_t n_rows,
                                                     unsigned long long* __restrict__ hist, int* __restrict__ max_len) {
    __shared__ int h[EPP_NCLASS];
    __shared__ int mx;
    if (threadIdx.x < EPP_NCLASS) h[threadIdx.x] = 0;
    if (threadIdx.x == 0) mx = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    int my_max = 0;
    const int64_t span = (int64_t)gridDim.x * kBlock;
    // whole wavefronts enter every iteration, so the ballots below see all 64 lanes
    for (int64_t base = (int64_t)blockIdx.x * kBlock + (threadIdx.x & ~63); base < n_rows; base += span) {
        const int64_t r = base + lane;
        int cls = -1;
        if (r < n_rows) {
            const int len = rowptr[r + 1] - rowptr[r];
            my_max = max(my_max, len);
            cls = length_class(len);
        }
        unsigned long long todo = __ballot(cls >= 0);
        while (todo) {
            const int c = __shfl(cls, __ffsll((long long)todo) - 1);
            const unsigned long long same = __ballot(cls == c);
            if (lane == __ffsll((long long)same) - 1) atomicAdd(&h[c], __popcll(same));
            todo &= ~same;
        }
    }
    if (my_max) atomicMax(&mx, my_max);
    __syncthreads();
    if (threadIdx.x < EPP_NCLASS && h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], (unsigned long long)h[threadIdx.x]);
    if (threadIdx.x == 0 && mx) atomicMax(max_len, mx);
}

// Interleave a plain CSR's (col, val) into pairs (all-active graph).
// A column outside [0, n) raises bit 1 of *err (if given) and is stored as 0.
__global__ __launch_bounds__(kBlock) void k_interleave(const int32_t* __restrict__ col, const float* __restrict__ val,
                                                       int64_t nnz, int64_t n, int2* __restrict__ cv,
                                                       int* __restrict__ err) {
    int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= nnz) return;
    int32_t c = col[e];
    if (c < 0 || c >= n) {
        if (err) atomicOr(err, 2);
        c = 0;
    }
    cv[e] = make_int2(c, __float_as_int(val[e]));
}

// Row pointer of a whole graph: must rise from 0 to nnz (bit 0 of *err otherwise).
__global__ __launch_bounds__(kBlock) void k_check_rowptr(const int32_t* __restrict__ rowptr, int64_t n, int64_t nnz,
                                                         int* __restrict__ err) {
    int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n) return;
    const int64_t p0 = rowptr[v], p1 = rowptr[v + 1];
    if (p0 < 0 || p1 < p0 || p1 > nnz || (v == 0 && p0 != 0) || (v == n - 1 && p1 != nnz)) atomicOr(err, 1);
}

__global__ __launch_bounds__(kBlock) void k_deinterleave(const int2* __restrict__ cv, int64_t nnz, int32_t* __restrict__ col,
                                                         float* __restrict__ val) {
    int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e < nnz) {
        int2 x = cv[e];
        if (col) col[e] = x.x & kEntCol;  // (the high bits are flags)
        if (val) val[e] = __int_as_float(x.y);
    }
}

// Entries of an inner path that shares the arrays of `outer` (canonical form, for export): row r of
// the inner path is the row of the same vertex in the outer path without the entries that carry
// the kEntOuterOnly mark, in the same order.  One wavefront per inner row.
__global__ __launch_bounds__(kBlock) void k_export_inner(const int32_t* __restrict__ row_ids,
                                                         const int32_t* __restrict__ rowptr, int64_t n_rows,
                                                         const int32_t* __restrict__ o_row_ids,
                                                         const int32_t* __restrict__ o_rowptr, int64_t o_rows,
                                                         const int2* __restrict__ o_cv, int32_t* __restrict__ col,
                                                         float* __restrict__ val) {
    const int64_t r = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    const int lane = lane_id();
    const int32_t v = row_ids[r];
    int64_t lo = 0, hi = o_rows - 1;  // the outer row of vertex v (it exists: the inner rows are outer rows)
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (o_row_ids[mid] < v) lo = mid + 1; else hi = mid;
    }
    int dst = rowptr[r];
    const int dst_end = rowptr[r + 1];
    for (int j0 = o_rowptr[lo]; j0 < o_rowptr[lo + 1]; j0 += 64) {
        const int j = j0 + lane;
        const bool in_row = j < o_rowptr[lo + 1];
        const int2 x = in_row ? o_cv[j] : make_int2(kEntOuterOnly, 0);
        const bool keep = !(x.x & kEntOuterOnly);
        const unsigned long long m = __ballot(keep);
        const int at = dst + __popcll(m & low_mask(lane));
        if (keep && at < dst_end) {  // (the bound only guards against arrays that do not belong together)
            if (col) col[at] = x.x & kEntCol;
            if (val) val[at] = __int_as_float(x.y);
        }
        dst += __popcll(m);
    }
}

__global__ __launch_bounds__(kBlock) void k_iota(int32_t* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = (int32_t)i;
}

// Flag the last entry of every (non-empty) row in bit 31 of its column id.
__global__ __launch_bounds__(kBlock) void k_mark_row_ends(const int32_t* __restrict__ rowptr, int64_t n_rows,
                                                          int2* __restrict__ cv) {
    int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= n_rows) return;
    int32_t end = rowptr[r + 1];
    if (end > rowptr[r]) cv[end - 1].x |= (int)0x80000000u;
}

// Bitmap of the vertices with a non-empty (invert = 0) or empty (invert = 1) list.
__global__ __launch_bounds__(kBlock) void k_nonempty_bitmap(const int32_t* __restrict__ rowptr, int64_t n, int invert,
                                                            unsigned long long* __restrict__ bitmap) {
    int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    bool flag = false;
    if (v < n) flag = (rowptr[v + 1] > rowptr[v]) != (invert != 0);
    unsigned long long bal = __ballot(flag);
    if (lane_id() == 0 && (v >> 6) < ((n + 63) >> 6)) bitmap[v >> 6] = bal;
}

// flag |= 1 if the two bitmaps differ anywhere.
__global__ __launch_bounds__(kBlock) void k_bitmap_differs(const unsigned long long* __restrict__ a,
                                                           const unsigned long long* __restrict__ b, int64_t n_words,
                                                           int* __restrict__ flag) {
    int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (w < n_words && a[w] != b[w]) atomicOr(flag, 1);
}

// flag |= 1 if some member of set a is not in set b.
__global__ __launch_bounds__(kBlock) void k_bitmap_not_subset(const unsigned long long* __restrict__ a,
                                                              const unsigned long long* __restrict__ b, int64_t n_words,
                                                              int* __restrict__ flag) {
    int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (w < n_words && (a[w] & ~b[w]) != 0ull) atomicOr(flag, 1);
}

inline unsigned grid_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

// out = exclusive scan of in[0 .. n), *total = sum.  `tmp` holds 2 * ceil(n / kScanChunk) ints.
inline size_t scan_tmp_bytes(int64_t n) { return (size_t)(2 * ((n + kScanChunk - 1) / kScanChunk) + 2) * sizeof(int); }
void scan_counts(const int* in, int* out, int64_t n, long long* total, int* tmp, hipStream_t s) {
    const int64_t chunks = (n + kScanChunk - 1) / kScanChunk;
    if (chunks <= 2) {
        hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, s, in, out, n, total);
        return;
    }
    int* chunk_sum = tmp;
    int* chunk_base = tmp + chunks;
    hipLaunchKernelGGL(k_scan_chunks, dim3((unsigned)chunks), dim3(1024), 0, s, in, out, n, chunk_sum);
    hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, s, (const int*)chunk_sum, chunk_base, chunks, total);
    hipLaunchKernelGGL(k_scan_add_offsets, dim3((unsigned)chunks), dim3(1024), 0, s, out, n, (const int*)chunk_base);
}

// Pinned host staging for the few scalars read back per level.
struct HostScalars {
    long long* p = nullptr;
    int init(size_t count = 64) {
        if (hipHostMalloc((void**)&p, count * sizeof(long long), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            epp_set_error("pinned host allocation failed");
            return EPP_ERR_ALLOC;
        }
        return EPP_OK;
    }
    ~HostScalars() { if (p) (void)hipHostFree(p); }
};

int validate_csr(const epp_csr_t* g) {
    if (!g) { epp_set_error("graph is NULL"); return EPP_ERR_INVALID_ARG; }
    if (g->n < 0 || g->nnz < 0) { epp_set_error("negative graph size"); return EPP_ERR_INVALID_ARG; }
    if (g->n >= kMaxVertices || g->nnz >= 0x7FFFFFFFll) {
        epp_set_error("graph too large: n=%lld (limit 2^29-1) nnz=%lld (limit 2^31-1)", (long long)g->n,
                      (long long)g->nnz);
        return EPP_ERR_TOO_LARGE;
    }
    if (!g->rowptr || (g->nnz > 0 && (!g->col || !g->val))) {
        epp_set_error("graph arrays are NULL");
        return EPP_ERR_INVALID_ARG;
    }
    return EPP_OK;
}

// Ascending ids of a bitmap (and optionally the compact row pointer).  Returns the count.
int compact_bitmap(const DevBuf& bitmap, int64_t n, const int* newptr, int total_nnz, DevBuf* ids, DevBuf* ptr_out,
                   int64_t* count, DevBuf& tile_cnt, DevBuf& tile_base, DevBuf& dev_total, HostScalars& hs,
                   const epp_alloc_t* al, hipStream_t s) {
    const int64_t n_words = (n + 63) / 64;
    const unsigned tiles = grid_for(n_words, kWordsPerTile);
    long long R = 0;
    if (tiles) {
        hipLaunchKernelGGL(k_bitmap_count, dim3(tiles), dim3(kBlock), 0, s, bitmap.as<unsigned long long>(), n_words,
                           tile_cnt.as<int>());
        hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, s, tile_cnt.as<int>(), tile_base.as<int>(),
                           (int64_t)tiles, dev_total.as<long long>());
        EPP_HIP_TRY(hipMemcpyAsync(hs.p, dev_total.p, sizeof(long long), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        R = hs.p[0];
    }
    *count = R;
    if (!ids) return EPP_OK;
    EPP_TRY(ids->alloc((size_t)R * sizeof(int32_t), al));
    if (ptr_out) EPP_TRY(ptr_out->alloc((size_t)(R + 1) * sizeof(int32_t), al));
    if (tiles) {
        hipLaunchKernelGGL(k_bitmap_compact, dim3(tiles), dim3(kBlock), 0, s, bitmap.as<unsigned long long>(), n_words,
                           tile_base.as<int>(), newptr, ids->as<int32_t>(),
                           ptr_out ? ptr_out->as<int32_t>() : nullptr, (int64_t)R, total_nnz);
    } else if (ptr_out) {
        EPP_HIP_TRY(hipMemsetAsync(ptr_out->p, 0, sizeof(int32_t), s));
    }
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}

// Checks of imported path arrays: bit 0 structure (ids not ascending, pointer decreasing, empty
// row, wrong end points), bit 1 an id outside [0, n).  Also sets the bitmap of the row set.
__global__ __launch_bounds__(kBlock) void k_check_rows(const int32_t* __restrict__ row_ids,
                                                       const int32_t* __restrict__ rowptr, int64_t n_rows, int64_t nnz,
                                                       int64_t n, unsigned int* __restrict__ bitmap32,
                                                       int* __restrict__ err) {
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r == 0 && (rowptr[0] != 0 || rowptr[n_rows] != nnz)) atomicOr(err, 1);
    if (r >= n_rows) return;
    const int32_t v = row_ids[r];
    if (v < 0 || v >= n) { atomicOr(err, 2); return; }
    if (r > 0 && row_ids[r - 1] >= v) atomicOr(err, 1);
    if (rowptr[r + 1] <= rowptr[r]) atomicOr(err, 1);
    atomicOr(&bitmap32[v >> 5], 1u << (v & 31));
}

__global__ __launch_bounds__(kBlock) void k_check_cols(const int32_t* __restrict__ col, int64_t nnz, int64_t n,
                                                       int* __restrict__ err) {
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e < nnz && (col[e] < 0 || col[e] >= n)) atomicOr(err, 2);
}

// Message and code for the error bits raised by the input checks (bit 0 row pointer, bit 1 ids).
long long env_share_pct() {
    const char* e = std::getenv("EPP_TUNE_SHARE_PCT");
    return (e && *e) ? std::atoll(e) : 95;
}

int input_error(int bits, int64_t n) {
    if (bits & 2) { epp_set_error("a column id lies outside [0, %lld)", (long long)n); return EPP_ERR_OUT_OF_RANGE_ID; }
    epp_set_error("the row pointer does not rise from 0 to nnz");
    return EPP_ERR_INVALID_ARG;
}

}  // namespace

size_t epp_scan_tmp_bytes(int64_t n) { return scan_tmp_bytes(n); }
void epp_scan_exclusive(const int* in, int* out, int64_t n, long long* total, int* tmp, hipStream_t s) {
    scan_counts(in, out, n, total, tmp, s);
}

void epp_path_set_stats(epp_path* p, const unsigned long long* host) {
    for (int c = 0; c < EPP_NCLASS; ++c) p->len_hist[c] = (int64_t)host[c];
    int mx;
    std::memcpy(&mx, &host[EPP_NCLASS], sizeof(int));
    p->max_len = mx;
}

int epp_path_finish(epp_path* p, hipStream_t s, void* stats_scratch, unsigned long long* host_later,
                    bool mark_row_ends) {
    DevBuf stats;
    if (stats_scratch) stats.view(stats_scratch, (EPP_NCLASS + 1) * sizeof(unsigned long long));
    else EPP_TRY(stats.alloc((EPP_NCLASS + 1) * sizeof(unsigned long long), epp_alloc_of(p)));
    EPP_HIP_TRY(hipMemsetAsync(stats.p, 0, stats.bytes, s));
    if (p->n_rows > 0) {
        // canonical rows: the all-active graph counts its empty rows too
        const int32_t* ptr = p->all_rows ? p->full_rowptr.as<int32_t>() : p->rowptr.as<int32_t>();
        hipLaunchKernelGGL(k_len_hist, dim3(std::min(grid_for(p->n_rows, kBlock), 2048u)), dim3(kBlock), 0, s, ptr,
                           p->n_rows, stats.as<unsigned long long>(),
                           reinterpret_cast<int*>(stats.as<unsigned long long>() + EPP_NCLASS));
        EPP_HIP_TRY(hipGetLastError());
    }
    if (host_later) {
        // pinned destination: the caller reads it (epp_path_set_stats) after its own synchronisation
        EPP_HIP_TRY(hipMemcpyAsync(host_later, stats.p, (EPP_NCLASS + 1) * sizeof(unsigned long long),
                                   hipMemcpyDeviceToHost, s));
    } else {
        unsigned long long host[EPP_NCLASS + 1];
        EPP_HIP_TRY(hipMemcpyAsync(host, stats.p, sizeof(host), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        epp_path_set_stats(p, host);
    }
    if (mark_row_ends && p->n_stream_rows > 0) {
        hipLaunchKernelGGL(k_mark_row_ends, dim3(grid_for(p->n_stream_rows, kBlock)), dim3(kBlock), 0, s,
                           p->rowptr.as<int32_t>(), p->n_stream_rows, p->cv.as<int2>());
        EPP_HIP_TRY(hipGetLastError());
    }
    return EPP_OK;  // the callers synchronise once, before they return the handle
}

extern "C" int epp_prepare(const epp_csr_t* g, const int32_t* train_ids, int64_t n_train, int L,
                           const epp_alloc_t* alloc, epp_stream_t stream, epp_paths_t** out) {
    if (!out) { epp_set_error("out is NULL"); return EPP_ERR_INVALID_ARG; }
    *out = nullptr;
    EPP_TRY(validate_csr(g));
    if (L < 1) { epp_set_error("L must be >= 1 (got %d)", L); return EPP_ERR_INVALID_ARG; }
    if (n_train < 0 || (n_train > 0 && !train_ids)) { epp_set_error("bad training set"); return EPP_ERR_INVALID_ARG; }
    hipStream_t s = (hipStream_t)stream;
    {   // set-up of this GPU's static scratch array (used by epp_weight_gradient_static)
        float* unused = nullptr;
        EPP_TRY(epp_static_scratch(&unused));
    }
    // small graphs: one launch builds everything (EPP_TUNE_SMALL_PREPARE=0 forces the general construction)
    if (epp_prepare_small_fits(g, n_train, L)) {
        const char* e = std::getenv("EPP_TUNE_SMALL_PREPARE");
        if (!(e && e[0] == '0')) return epp_prepare_small(g, train_ids, n_train, L, alloc, s, out);
    }
    const int64_t n = g->n, nnz = g->nnz;
    const int64_t n_words = (n + 63) / 64;
    const int64_t n_seg = (nnz + 63) / 64;
    const unsigned edge_tiles = grid_for(n_seg, kSegsPerTile);
    const unsigned word_tiles = grid_for(n_words, kWordsPerTile);

    // pinned words read back from the device: [0] kept entries, [1] |N^{k+1}| (also the scratch of
    // compact_bitmap), then EPP_NCLASS + 1 statistics words per level
    constexpr int kStatWords = EPP_NCLASS + 1;
    HostScalars hs;
    EPP_TRY(hs.init(8 + (size_t)L * kStatWords));
    epp_paths* P = new epp_paths();
    struct Guard { epp_paths* p; ~Guard() { delete p; } } guard{P};
    P->L = L;
    P->n = n;
    if (alloc && alloc->alloc && alloc->free) P->alloc = *alloc;
    const epp_alloc_t* al = epp_alloc_of(P);
    P->bitmaps.resize(L + 1);
    P->set_size.assign(L + 1, 0);
    P->path.assign(L, nullptr);
    for (int k = 0; k <= L; ++k) {
        EPP_TRY(P->bitmaps[k].alloc((size_t)n_words * 8, al));
        EPP_HIP_TRY(hipMemsetAsync(P->bitmaps[k].p, 0, P->bitmaps[k].bytes, s));
    }

    // all temporaries of the construction come from one allocation
    // (keep-mask and segment offsets twice: the entries of a level are extracted once the next
    // level has shown whether the two paths share them, so two levels' masks are alive at a time)
    DevBuf mask[2], seg_base[2], tile_cnt, tile_base, scan_tmp, newptr, dev_total, err, stats;
    const size_t max_tiles = std::max<size_t>(std::max(edge_tiles, word_tiles), 1);
    const size_t stats_bytes = kStatWords * sizeof(unsigned long long);
    DevArena arena;
    EPP_TRY(arena.reserve(2 * DevArena::rounded((size_t)n_seg * 8) + 2 * DevArena::rounded((size_t)n_seg * 4) +
                          2 * DevArena::rounded(max_tiles * 4) + DevArena::rounded(scan_tmp_bytes(edge_tiles)) +
                          DevArena::rounded((size_t)(n + 1) * 4) +
                          2 * DevArena::rounded(32) + DevArena::rounded(stats_bytes), al));
    for (int i = 0; i < 2; ++i) {
        arena.take(&mask[i], (size_t)n_seg * 8);
        arena.take(&seg_base[i], (size_t)n_seg * 4);
    }
    arena.take(&tile_cnt, max_tiles * 4);
    arena.take(&tile_base, max_tiles * 4);
    arena.take(&scan_tmp, scan_tmp_bytes(edge_tiles));
    arena.take(&newptr, (size_t)(n + 1) * 4);
    // [0] kept entries, [1] rows of the level, [2] input error bits, [3] "N^{k-1} is not inside N^k"
    arena.take(&dev_total, 4 * sizeof(long long));
    arena.take(&err, sizeof(int));
    arena.take(&stats, stats_bytes);
    EPP_HIP_TRY(hipMemsetAsync(err.p, 0, sizeof(int), s));
    EPP_HIP_TRY(hipMemsetAsync(newptr.p, 0, newptr.bytes, s));

    // N^0 = V_t (Property 1)
    if (n_train > 0) {
        hipLaunchKernelGGL(k_mark_training, dim3(grid_for(n_train, kBlock)), dim3(kBlock), 0, s, train_ids, n_train, n,
                           P->bitmaps[0].as<unsigned int>(), err.as<int>());
        EPP_HIP_TRY(hipGetLastError());
        int herr = 0;
        EPP_HIP_TRY(hipMemcpyAsync(&herr, err.p, sizeof(int), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        if (herr) {
            epp_set_error("training id outside [0, %lld)", (long long)n);
            return EPP_ERR_OUT_OF_RANGE_ID;
        }
    }
    // ascending ids of N^0 (the other sets are the row ids of the paths)
    EPP_TRY(compact_bitmap(P->bitmaps[0], n, nullptr, 0, &P->set0_ids, nullptr, &P->set_size[0], tile_cnt, tile_base,
                           dev_total, hs, al, s));

    // One level: everything that only needs the two counts (kept entries, rows) on the device is
    // enqueued first, the host waits once for both, allocates the level's arrays, and enqueues
    // the passes that fill them.  The row-length statistics come back through pinned memory and
    // are read after the last level.
    //
    // Shared entries: the path of a level runs on the arrays of the next level's path if nearly
    // all of that path's entries are its own too (the extra entries are skipped one by one at
    // run time, so the inner layer pays for them; EPP_TUNE_SHARE_PCT, default 95, 0: never).
    // A level's entries are therefore extracted only when the next level's count is known: not
    // at all if it shares them, and the outer path's extraction marks the entries that are not
    // the inner path's.  Every other level at most: a path whose marks serve an inner path
    // keeps its own arrays.
    std::vector<epp_path*> built;  // in level order, for the statistics
    struct { epp_path* p = nullptr; int slot = 0; } pending;  // path whose entries are not extracted yet
    auto extract = [&](epp_path* q, int slot, const unsigned long long* inner_mask) -> int {
        // the entries in an allocation of their own (it can be given back once every prepared width
        // runs on a reconstructed copy)
        EPP_TRY(q->cv.alloc((size_t)q->nnz * sizeof(int2), al));
        if (edge_tiles) {
            hipLaunchKernelGGL(k_edge_extract, dim3(edge_tiles), dim3(kBlock), 0, s, g->col, g->val, n_seg,
                               mask[slot].as<unsigned long long>(), inner_mask, seg_base[slot].as<int>(), q->cv.as<int2>());
        }
        if (q->n_stream_rows > 0) {
            hipLaunchKernelGGL(k_mark_row_ends, dim3(grid_for(q->n_stream_rows, kBlock)), dim3(kBlock), 0, s,
                               q->rowptr.as<int32_t>(), q->n_stream_rows, q->cv.as<int2>());
        }
        EPP_HIP_TRY(hipGetLastError());
        return EPP_OK;
    };
    const long long share_pct = env_share_pct();
    for (int k = 0; k < L; ++k) {
        const int l = L - 1 - k;  // rows N^{k+1} = N^{L-l}, sources N^k = N^{L-l-1}
        const int slot = k & 1;
        epp_path* p = new epp_path();
        P->path[l] = p;
        built.push_back(p);
        p->n = n;
        p->alloc = P->alloc;
        p->pool = &P->pool;
        p->n_src = P->set_size[k];
        long long* d_total = dev_total.as<long long>();
        int* d_err = reinterpret_cast<int*>(d_total + 2);
        int* d_not_subset = reinterpret_cast<int*>(d_total + 3);
        EPP_HIP_TRY(hipMemsetAsync(d_total, 0, 4 * sizeof(long long), s));
        if (edge_tiles) {
            // from the second level on the mask of the level before is reused where N^{k-1} lies in N^k
            if (k > 0) {
                hipLaunchKernelGGL(k_bitmap_not_subset, dim3(grid_for(n_words, kBlock)), dim3(kBlock), 0, s,
                                   P->bitmaps[k - 1].as<unsigned long long>(), P->bitmaps[k].as<unsigned long long>(),
                                   n_words, d_not_subset);
            }
            hipLaunchKernelGGL(k_edge_mask, dim3(edge_tiles), dim3(kBlock), 0, s, g->col, nnz, n_seg, n,
                               P->bitmaps[k].as<unsigned int>(),
                               k > 0 ? mask[slot ^ 1].as<unsigned long long>() : (const unsigned long long*)nullptr,
                               (const int*)d_not_subset, mask[slot].as<unsigned long long>(), tile_cnt.as<int>(), d_err);
            scan_counts(tile_cnt.as<int>(), tile_base.as<int>(), (int64_t)edge_tiles, d_total, scan_tmp.as<int>(), s);
            hipLaunchKernelGGL(k_seg_base, dim3(edge_tiles), dim3(64), 0, s, mask[slot].as<unsigned long long>(), n_seg,
                               tile_base.as<int>(), seg_base[slot].as<int>());
            EPP_HIP_TRY(hipGetLastError());
        }
        if (n > 0) {
            hipLaunchKernelGGL(k_row_flags, dim3(grid_for(n, kBlock)), dim3(kBlock), 0, s, g->rowptr, n, nnz,
                               mask[slot].as<unsigned long long>(), seg_base[slot].as<int>(), (const long long*)d_total,
                               newptr.as<int>(), P->bitmaps[k + 1].as<unsigned long long>(), d_err);
            // rows of the level: set bits of the new bitmap, counted per tile of words and scanned
            // (the edge-tile offsets are no longer needed: seg_base holds them)
            hipLaunchKernelGGL(k_bitmap_count, dim3(word_tiles), dim3(kBlock), 0, s,
                               P->bitmaps[k + 1].as<unsigned long long>(), n_words, tile_cnt.as<int>());
            hipLaunchKernelGGL(k_scan_counts, dim3(1), dim3(1024), 0, s, tile_cnt.as<int>(), tile_base.as<int>(),
                               (int64_t)word_tiles, d_total + 1);
            EPP_HIP_TRY(hipGetLastError());
        }
        EPP_HIP_TRY(hipMemcpyAsync(hs.p, d_total, 4 * sizeof(long long), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        if (hs.p[2] != 0) return input_error((int)hs.p[2], n);
        if (n == 0 && nnz > 0) return input_error(2, n);
        const long long kept = hs.p[0], R = hs.p[1];
        const bool nested = (int)hs.p[3] == 0;
        p->nnz = kept;
        p->n_rows = R;
        p->n_stream_rows = R;  // every row of a path has at least one entry
        P->set_size[k + 1] = R;
        // row ids | row pointer in one allocation, each 256-byte aligned
        const size_t ids_bytes = (size_t)R * 4, ptr_bytes = (size_t)(R + 1) * 4;
        EPP_TRY(p->store.alloc(DevArena::rounded(ids_bytes) + DevArena::rounded(ptr_bytes), al));
        char* base = p->store.as<char>();
        p->row_ids.view(base, ids_bytes);
        p->rowptr.view(base + DevArena::rounded(ids_bytes), ptr_bytes);
        if (n > 0) {
            hipLaunchKernelGGL(k_bitmap_compact, dim3(word_tiles), dim3(kBlock), 0, s,
                               P->bitmaps[k + 1].as<unsigned long long>(), n_words, tile_base.as<int>(), newptr.as<int>(),
                               p->row_ids.as<int32_t>(), p->rowptr.as<int32_t>(), (int64_t)R, (int)kept);
        } else {
            EPP_HIP_TRY(hipMemsetAsync(p->rowptr.p, 0, sizeof(int32_t), s));
        }
        EPP_HIP_TRY(hipGetLastError());
        EPP_TRY(epp_path_finish(p, s, stats.p, reinterpret_cast<unsigned long long*>(hs.p) + 8 + (size_t)k * kStatWords,
                                /*mark_row_ends=*/false));
        epp_path* q = pending.p;  // the path of the level before, if its entries still wait
        if (q && nested && share_pct > 0 && q->nnz > 0 && q->nnz * 100 >= kept * share_pct) {
            EPP_TRY(p->zero_block.alloc(256, al));
            EPP_HIP_TRY(hipMemsetAsync(p->zero_block.p, 0, 256, s));
            p->has_inner = true;
            q->outer = p;
            q->inner_rows = P->bitmaps[k].as<unsigned int>();  // its rows are N^k
            EPP_TRY(extract(p, slot, mask[slot ^ 1].as<unsigned long long>()));
            pending.p = nullptr;
        } else {
            if (q) EPP_TRY(extract(q, pending.slot, nullptr));
            pending.p = p;
            pending.slot = slot;
        }
        // Fixed point: N^{k+1} == N^k means every further set is the same set, so every deeper
        // layer (rows and sources both equal to it) has exactly this path; share it.
        if (k + 1 < L && P->set_size[k + 1] == P->set_size[k]) {
            int differs = 0;
            EPP_HIP_TRY(hipMemsetAsync(err.p, 0, sizeof(int), s));
            if (n_words > 0) {
                hipLaunchKernelGGL(k_bitmap_differs, dim3(grid_for(n_words, kBlock)), dim3(kBlock), 0, s,
                                   P->bitmaps[k].as<unsigned long long>(), P->bitmaps[k + 1].as<unsigned long long>(),
                                   n_words, err.as<int>());
                EPP_HIP_TRY(hipGetLastError());
            }
            EPP_HIP_TRY(hipMemcpyAsync(&differs, err.p, sizeof(int), hipMemcpyDeviceToHost, s));
            EPP_HIP_TRY(hipStreamSynchronize(s));
            if (!differs) {
                for (int j = k + 1; j < L; ++j) {
                    EPP_HIP_TRY(hipMemcpyAsync(P->bitmaps[j + 1].p, P->bitmaps[k + 1].p, P->bitmaps[k + 1].bytes,
                                               hipMemcpyDeviceToDevice, s));
                    P->set_size[j + 1] = P->set_size[k + 1];
                    P->path[L - 1 - j] = p;
                }
                break;
            }
        }
    }
    if (pending.p) EPP_TRY(extract(pending.p, pending.slot, nullptr));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    for (size_t k = 0; k < built.size(); ++k)
        epp_path_set_stats(built[k], reinterpret_cast<const unsigned long long*>(hs.p) + 8 + k * kStatWords);
    guard.p = nullptr;
    *out = P;
    return EPP_OK;
}

extern "C" int epp_prepare_full(const epp_csr_t* g, const epp_alloc_t* alloc, epp_stream_t stream,
                                epp_path_t** out) {
    if (!out) { epp_set_error("out is NULL"); return EPP_ERR_INVALID_ARG; }
    *out = nullptr;
    EPP_TRY(validate_csr(g));
    hipStream_t s = (hipStream_t)stream;
    epp_path* p = new epp_path();
    struct Guard { epp_path* p; ~Guard() { delete p; } } guard{p};
    p->n = g->n;
    p->n_rows = g->n;
    p->nnz = g->nnz;
    p->n_src = g->n;
    p->all_rows = true;
    if (alloc && alloc->alloc && alloc->free) p->alloc = *alloc;
    const epp_alloc_t* al = epp_alloc_of(p);
    EPP_TRY(p->full_rowptr.alloc((size_t)(g->n + 1) * 4, al));
    EPP_TRY(p->cv.alloc((size_t)g->nnz * sizeof(int2), al));
    {   // streamed form: the vertices with non-empty lists, ascending, with a compact row pointer
        HostScalars hs;
        EPP_TRY(hs.init());
        DevBuf bitmap, tile_cnt, tile_base, dev_total, err;
        const int64_t n_words = (g->n + 63) / 64;
        const size_t tiles = std::max<size_t>(grid_for(n_words, kWordsPerTile), 1);
        DevArena arena;
        EPP_TRY(arena.reserve(DevArena::rounded((size_t)n_words * 8) + 2 * DevArena::rounded(tiles * 4) +
                              2 * DevArena::rounded(16), al));
        arena.take(&bitmap, (size_t)n_words * 8);
        arena.take(&tile_cnt, tiles * 4);
        arena.take(&tile_base, tiles * 4);
        arena.take(&dev_total, sizeof(long long));
        arena.take(&err, sizeof(int));
        // the caller's arrays are checked before anything is indexed with them
        EPP_HIP_TRY(hipMemsetAsync(err.p, 0, sizeof(int), s));
        if (g->n > 0)
            hipLaunchKernelGGL(k_check_rowptr, dim3(grid_for(g->n, kBlock)), dim3(kBlock), 0, s, g->rowptr, g->n, g->nnz,
                               err.as<int>());
        if (g->nnz > 0)
            hipLaunchKernelGGL(k_interleave, dim3(grid_for(g->nnz, kBlock)), dim3(kBlock), 0, s, g->col, g->val, g->nnz,
                               g->n, p->cv.as<int2>(), err.as<int>());
        EPP_HIP_TRY(hipGetLastError());
        EPP_HIP_TRY(hipMemcpyAsync(hs.p, err.p, sizeof(int), hipMemcpyDeviceToHost, s));
        EPP_HIP_TRY(hipStreamSynchronize(s));
        int herr;
        std::memcpy(&herr, hs.p, sizeof(int));
        if (g->n == 0 && g->nnz > 0) herr |= 2;
        if (herr) return input_error(herr, g->n);
        EPP_HIP_TRY(hipMemcpyAsync(p->full_rowptr.p, g->rowptr, (size_t)(g->n + 1) * 4, hipMemcpyDeviceToDevice, s));
        if (g->n > 0) {
            hipLaunchKernelGGL(k_nonempty_bitmap, dim3(grid_for(g->n, kBlock)), dim3(kBlock), 0, s, g->rowptr, g->n, 0,
                               bitmap.as<unsigned long long>());
            EPP_HIP_TRY(hipGetLastError());
        }
        EPP_TRY(compact_bitmap(bitmap, g->n, g->rowptr, (int)g->nnz, &p->row_ids, &p->rowptr, &p->n_stream_rows,
                               tile_cnt, tile_base, dev_total, hs, al, s));
        p->n_empty_rows = g->n - p->n_stream_rows;
        if (p->n_empty_rows == 0) {
            EPP_HIP_TRY(hipStreamSynchronize(s));
            p->row_ids.release();  // identity
        } else {
            hipLaunchKernelGGL(k_nonempty_bitmap, dim3(grid_for(g->n, kBlock)), dim3(kBlock), 0, s, g->rowptr, g->n, 1,
                               bitmap.as<unsigned long long>());
            EPP_HIP_TRY(hipGetLastError());
            int64_t cnt = 0;
            EPP_TRY(compact_bitmap(bitmap, g->n, nullptr, 0, &p->empty_rows, nullptr, &cnt, tile_cnt, tile_base,
                                   dev_total, hs, al, s));
            EPP_HIP_TRY(hipStreamSynchronize(s));
        }
    }
    EPP_TRY(epp_path_finish(p, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    guard.p = nullptr;
    *out = p;
    return EPP_OK;
}

extern "C" int epp_paths_import(int64_t n, int L, const int32_t* train_ids, int64_t n_train,
                                const epp_path_arrays_t* layers, const epp_alloc_t* alloc, epp_stream_t stream,
                                epp_paths_t** out) {
    if (!out) { epp_set_error("out is NULL"); return EPP_ERR_INVALID_ARG; }
    *out = nullptr;
    if (L < 1 || !layers) { epp_set_error("L must be >= 1 and layers non-NULL"); return EPP_ERR_INVALID_ARG; }
    if (n < 0 || n_train < 0 || (n_train > 0 && !train_ids)) { epp_set_error("bad sizes"); return EPP_ERR_INVALID_ARG; }
    if (n >= kMaxVertices) { epp_set_error("graph too large: n=%lld (limit 2^29-1)", (long long)n); return EPP_ERR_TOO_LARGE; }
    for (int l = 0; l < L; ++l) {
        const epp_path_arrays_t& a = layers[l];
        if (a.n_rows < 0 || a.n_rows > n || a.nnz < 0 || !a.rowptr || (a.n_rows > 0 && !a.row_ids) ||
            (a.nnz > 0 && (!a.col || !a.val)) || (a.n_rows == 0 && a.nnz != 0)) {
            epp_set_error("layer %d: inconsistent sizes or NULL arrays", l);
            return EPP_ERR_INVALID_ARG;
        }
        if (a.nnz >= 0x7FFFFFFFll) { epp_set_error("layer %d: nnz=%lld (limit 2^31-1)", l, (long long)a.nnz); return EPP_ERR_TOO_LARGE; }
    }
    hipStream_t s = (hipStream_t)stream;
    {   // set-up of this GPU's static scratch array (used by epp_weight_gradient_static)
        float* unused = nullptr;
        EPP_TRY(epp_static_scratch(&unused));
    }
    const int64_t n_words = (n + 63) / 64;
    HostScalars hs;
    EPP_TRY(hs.init());
    epp_paths* P = new epp_paths();
    struct Guard { epp_paths* p; ~Guard() { delete p; } } guard{P};
    P->L = L;
    P->n = n;
    if (alloc && alloc->alloc && alloc->free) P->alloc = *alloc;
    const epp_alloc_t* al = epp_alloc_of(P);
    P->bitmaps.resize(L + 1);
    P->set_size.assign(L + 1, 0);
    P->path.assign(L, nullptr);
    for (int k = 0; k <= L; ++k) {
        EPP_TRY(P->bitmaps[k].alloc((size_t)n_words * 8, al));
        EPP_HIP_TRY(hipMemsetAsync(P->bitmaps[k].p, 0, P->bitmaps[k].bytes, s));
    }
    DevBuf tile_cnt, tile_base, dev_total, err;
    const size_t tiles = std::max<size_t>(grid_for(n_words, kWordsPerTile), 1);
    EPP_TRY(tile_cnt.alloc(tiles * 4, al));
    EPP_TRY(tile_base.alloc(tiles * 4, al));
    EPP_TRY(dev_total.alloc(sizeof(long long), al));
    EPP_TRY(err.alloc(2 * sizeof(int), al));  // [0]: path arrays, [1]: training ids
    EPP_HIP_TRY(hipMemsetAsync(err.p, 0, 2 * sizeof(int), s));
    if (n_train > 0)
        hipLaunchKernelGGL(k_mark_training, dim3(grid_for(n_train, kBlock)), dim3(kBlock), 0, s, train_ids, n_train, n,
                           P->bitmaps[0].as<unsigned int>(), err.as<int>() + 1);
    for (int l = 0; l < L; ++l) {
        const epp_path_arrays_t& a = layers[l];
        hipLaunchKernelGGL(k_check_rows, dim3(std::max(grid_for(a.n_rows, kBlock), 1u)), dim3(kBlock), 0, s, a.row_ids,
                           a.rowptr, a.n_rows, a.nnz, n, P->bitmaps[L - l].as<unsigned int>(), err.as<int>());
        if (a.nnz > 0)
            hipLaunchKernelGGL(k_check_cols, dim3(grid_for(a.nnz, kBlock)), dim3(kBlock), 0, s, a.col, a.nnz, n,
                               err.as<int>());
    }
    EPP_HIP_TRY(hipGetLastError());
    int herr2[2] = {0, 0};
    EPP_HIP_TRY(hipMemcpyAsync(herr2, err.p, sizeof(herr2), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    const int herr = herr2[0] | (herr2[1] ? 2 : 0);
    if (herr & 2) { epp_set_error("an id lies outside [0, %lld)", (long long)n); return EPP_ERR_OUT_OF_RANGE_ID; }
    if (herr & 1) { epp_set_error("path arrays are not in canonical form"); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(compact_bitmap(P->bitmaps[0], n, nullptr, 0, &P->set0_ids, nullptr, &P->set_size[0], tile_cnt, tile_base,
                           dev_total, hs, al, s));
    for (int l = L - 1; l >= 0; --l) {
        const epp_path_arrays_t& a = layers[l];
        const int k = L - l - 1;
        epp_path* p = new epp_path();
        P->path[l] = p;
        p->n = n;
        p->alloc = P->alloc;
        p->pool = &P->pool;
        p->n_rows = p->n_stream_rows = a.n_rows;
        p->nnz = a.nnz;
        p->n_src = P->set_size[k];
        P->set_size[k + 1] = a.n_rows;
        EPP_TRY(p->row_ids.alloc((size_t)a.n_rows * 4, al));
        EPP_TRY(p->rowptr.alloc((size_t)(a.n_rows + 1) * 4, al));
        EPP_TRY(p->cv.alloc((size_t)a.nnz * sizeof(int2), al));
        if (a.n_rows > 0)
            EPP_HIP_TRY(hipMemcpyAsync(p->row_ids.p, a.row_ids, (size_t)a.n_rows * 4, hipMemcpyDeviceToDevice, s));
        EPP_HIP_TRY(hipMemcpyAsync(p->rowptr.p, a.rowptr, (size_t)(a.n_rows + 1) * 4, hipMemcpyDeviceToDevice, s));
        if (a.nnz > 0) {
            hipLaunchKernelGGL(k_interleave, dim3(grid_for(a.nnz, kBlock)), dim3(kBlock), 0, s, a.col, a.val, a.nnz, n,
                               p->cv.as<int2>(), (int*)nullptr);
            EPP_HIP_TRY(hipGetLastError());
        }
        EPP_TRY(epp_path_finish(p, s));
    }
    EPP_HIP_TRY(hipStreamSynchronize(s));
    guard.p = nullptr;
    *out = P;
    return EPP_OK;
}

extern "C" int epp_num_layers(const epp_paths_t* p) {
    if (!p) { epp_set_error("paths is NULL"); return EPP_ERR_INVALID_ARG; }
    return p->L;
}

extern "C" epp_path_t* epp_get_path(epp_paths_t* p, int l) {
    if (!p || l < 0 || l >= p->L) { epp_set_error("no such layer"); return nullptr; }
    return p->path[l];
}

extern "C" int epp_path_export(const epp_path_t* p, int32_t* row_ids, int32_t* rowptr, int32_t* col, float* val,
                               epp_stream_t stream) {
    if (!p) { epp_set_error("path is NULL"); return EPP_ERR_INVALID_ARG; }
    hipStream_t s = (hipStream_t)stream;
    if (row_ids && p->n_rows > 0) {
        if (p->all_rows) {
            hipLaunchKernelGGL(k_iota, dim3(grid_for(p->n_rows, kBlock)), dim3(kBlock), 0, s, row_ids, p->n_rows);
        } else {
            EPP_HIP_TRY(hipMemcpyAsync(row_ids, p->row_ids.p, (size_t)p->n_rows * 4, hipMemcpyDeviceToDevice, s));
        }
    }
    if (rowptr) {
        const void* ptr = p->all_rows ? p->full_rowptr.p : p->rowptr.p;
        EPP_HIP_TRY(hipMemcpyAsync(rowptr, ptr, (size_t)(p->n_rows + 1) * 4, hipMemcpyDeviceToDevice, s));
    }
    if ((col || val) && p->nnz > 0) {
        if (p->outer) {  // the entries live in the outer path's array
            epp_path* o = p->outer;
            EPP_TRY(epp_ensure_canonical(o, s));
            hipLaunchKernelGGL(k_export_inner, dim3(grid_for(p->n_rows, kBlock / 64)), dim3(kBlock), 0, s,
                               p->row_ids.as<int32_t>(), p->rowptr.as<int32_t>(), p->n_rows, o->row_ids.as<int32_t>(),
                               o->rowptr.as<int32_t>(), o->n_stream_rows, o->cv.as<int2>(), col, val);
        } else {
            EPP_TRY(epp_ensure_canonical(const_cast<epp_path*>(p), s));
            hipLaunchKernelGGL(k_deinterleave, dim3(grid_for(p->nnz, kBlock)), dim3(kBlock), 0, s, p->cv.as<int2>(),
                               p->nnz, col, val);
        }
    }
    EPP_HIP_TRY(hipGetLastError());
    EPP_HIP_TRY(hipStreamSynchronize(s));
    // (an entry array that was rebuilt for this call only is given back again)
    epp_release_canonical_if_unused(p->outer ? p->outer : const_cast<epp_path*>(p));
    return EPP_OK;
}

extern "C" int epp_active_set_export(const epp_paths_t* p, int k, int32_t* ids, int64_t* count, epp_stream_t stream) {
    if (!p || !count) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (k < 0 || k > p->L) { epp_set_error("k=%d outside [0, %d]", k, p->L); return EPP_ERR_INVALID_ARG; }
    hipStream_t s = (hipStream_t)stream;
    if (!ids) { *count = p->set_size[k]; return EPP_OK; }
    if (*count < p->set_size[k]) {
        epp_set_error("ids buffer holds %lld entries, need %lld", (long long)*count, (long long)p->set_size[k]);
        return EPP_ERR_INVALID_ARG;
    }
    HostScalars hs;
    EPP_TRY(hs.init());
    DevBuf tile_cnt, tile_base, dev_total, tmp;
    const size_t tiles = std::max<size_t>(grid_for((p->n + 63) / 64, kWordsPerTile), 1);
    const epp_alloc_t* al = epp_alloc_of(p);
    EPP_TRY(tile_cnt.alloc(tiles * 4, al));
    EPP_TRY(tile_base.alloc(tiles * 4, al));
    EPP_TRY(dev_total.alloc(sizeof(long long), al));
    int64_t c = 0;
    EPP_TRY(compact_bitmap(p->bitmaps[k], p->n, nullptr, 0, &tmp, nullptr, &c, tile_cnt, tile_base, dev_total, hs, al, s));
    if (c > 0) EPP_HIP_TRY(hipMemcpyAsync(ids, tmp.p, (size_t)c * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    *count = c;
    return EPP_OK;
}

int epp_active_ids(const epp_paths* p, int k, const int32_t** ids, int64_t* count) {
    if (k < 0 || k > p->L) { epp_set_error("k=%d outside [0, %d]", k, p->L); return EPP_ERR_INVALID_ARG; }
    *count = p->set_size[k];
    // N^k, k >= 1, is the row set of SG_{L-k}; N^0 was compacted when the handle was made
    *ids = k > 0 ? p->path[p->L - k]->row_ids.as<int32_t>() : p->set0_ids.as<int32_t>();
    return EPP_OK;
}

extern "C" void epp_destroy_paths(epp_paths_t* p) { delete p; }
extern "C" void epp_destroy_path(epp_path_t* p) { delete p; }
