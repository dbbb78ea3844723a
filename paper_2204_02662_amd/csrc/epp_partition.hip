// Source-partitioned layout of an execution path: the path's entry array "reconstructed" for a
// GPU whose eight XCDs have private L2 caches (Sec. 6 names this step of pre-processing:
// the execution paths are reconstructed for the kernel that will run them; Sec. 2.2's neighbour
// groups are then cut from the reconstructed array).
//
// Why.  A gathered source row that misses the 4 MB L2 of its XCD costs four times the time of
// one that hits, and with plain row-major processing all eight L2s end up holding the same few
// thousand most referenced rows.  Here the most referenced sources ("hot": as many as the eight L2s
// can hold together) are dealt to eight partitions by a hash of their id, and the entries of
// the long rows that reference them are moved into eight sections of the entry array, one per
// partition; section x is processed by the workgroups that run on XCD x only, so the eight L2s
// hold eight different sets of rows.  All other entries (short rows, rarely referenced sources)
// form a ninth section that all XCDs share.
//
// A row with entries in several sections becomes one "virtual row" per section.  Each writes a
// partial row; k_combine_sections adds a vertex's partial rows in section order (no atomics:
// results stay bit-reproducible).  Only rows of at least `min_len` entries are cut, so that the
// partial rows (at most nine per cut row) stay a small fraction of the gathered rows.
//
// Layout of the reconstructed entry array: sections 0..7 hold the hot shares of the cut rows (rows
// ascending, a row's entries in their order), section 8 holds first the remaining entries of the cut
// rows (same order), then all rows that are not cut, whole and in ascending order.
//
// Construction (all on the GPU, deterministic, stable).  The cut rows are split into tiles of 1024
// consecutive entries, one wavefront per tile, so that a row of a quarter of a million entries
// is no slower than four hundred short ones:
//   flag + scans           the rows to cut (m = 0 .. M-1) and their tiles
//   k_part_count           entries per (section, tile); their scan is every tile's place in every
//                          section, because the sections list the tiles in the same order
//   k_part_keys + 2 scans  keys (section, row) in layout order -> virtual-row index and first entry
//   k_part_vrows           row pointer and target of every virtual row
//   k_part_scatter_*       entries to their places, row-end flag on the last entry of each virtual row

#include <algorithm>
#include <cstdlib>

#include "epp_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowEnd = kEntRowEnd, kCold = kEntCold, kOuterOnly = kEntOuterOnly, kColMask = kEntCol;
constexpr int kHot = 8;        // hot sections = XCDs
constexpr int kSec = kHot + 1;
constexpr int kTile = 1024;    // entries of a cut row handled by one wavefront

typedef int int2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ unsigned long long low_mask(int lane) { return (1ull << lane) - 1ull; }
// partition of a hot source: a multiplicative hash, so that any numbering of the vertices spreads
__device__ __forceinline__ int part_of(int c) { return (int)(((unsigned)c * 0x9E3779B1u) >> 29); }
__device__ __forceinline__ int section_of(int c, const unsigned int* __restrict__ hot) {
    return ((hot[c >> 5] >> (c & 31)) & 1u) ? part_of(c) : kHot;
}

__global__ __launch_bounds__(kBlock) void k_part_flag_rows(const int32_t* __restrict__ rowptr, int64_t R, int min_len,
                                                           int* __restrict__ flag) {
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r < R) flag[r] = (rowptr[r + 1] - rowptr[r]) >= min_len ? 1 : 0;
}

// srow[m] = r and m_of_row[r] = m for the rows to cut (m = exclusive scan of the flags), -1 otherwise
__global__ __launch_bounds__(kBlock) void k_part_list_rows(const int* __restrict__ flag, const int* __restrict__ midx,
                                                           int64_t R, int32_t* __restrict__ srow,
                                                           int32_t* __restrict__ m_of_row) {
    const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= R) return;
    if (flag[r]) {
        srow[midx[r]] = (int32_t)r;
        m_of_row[r] = midx[r];
    } else {
        m_of_row[r] = -1;
    }
}

// Tiles of the cut rows: tile_row[t] = m for the tiles of row m (tile_first = scan of the tile counts).
__global__ __launch_bounds__(kBlock) void k_part_tiles_per_row(const int32_t* __restrict__ rowptr,
                                                               const int32_t* __restrict__ srow, int64_t M,
                                                               int* __restrict__ ntiles, int* __restrict__ nbytes) {
    const int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (m >= M) return;
    const int32_t r = srow[m];
    const int len = rowptr[r + 1] - rowptr[r];
    ntiles[m] = (len + kTile - 1) / kTile;
    nbytes[m] = (len + 1) / 2;  // one 4-bit section id per entry, the row starts on a byte
}

__global__ __launch_bounds__(kBlock) void k_part_tile_rows(const int* __restrict__ tile_first, const int* __restrict__ ntiles,
                                                           int64_t M, int32_t* __restrict__ tile_row) {
    // one wavefront per row: its tiles are numbered consecutively
    const int64_t m = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (m >= M) return;
    const int first = tile_first[m], cnt = ntiles[m];
    for (int i = lane_id(); i < cnt; i += 64) tile_row[first + i] = (int32_t)m;
}

// One wavefront per tile: its entries per section, stored section-major (tcnt[x * T + t]).
__global__ __launch_bounds__(kBlock) void k_part_count(const int2v* __restrict__ cv, const int32_t* __restrict__ rowptr,
                                                       const int32_t* __restrict__ srow,
                                                       const int32_t* __restrict__ tile_row,
                                                       const int* __restrict__ tile_first, int64_t T,
                                                       const unsigned int* __restrict__ hot, int* __restrict__ tcnt) {
    const int64_t t = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = lane_id();
    const int32_t m = tile_row[t], r = srow[m];
    const int p0 = rowptr[r] + (int)(t - tile_first[m]) * kTile, p1 = min(p0 + kTile, rowptr[r + 1]);
    // all entries of the tile first, then all bitmap lookups: the two dependent latencies are paid once
    int col[kTile / 64];
    int sec[kTile / 64];
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) {
        const int j = p0 + i * 64 + lane;
        col[i] = j < p1 ? (cv[j].x & kColMask) : -1;
    }
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) sec[i] = col[i] >= 0 ? section_of(col[i], hot) : -1;
    int c[kSec];
#pragma unroll
    for (int x = 0; x < kSec; ++x) c[x] = 0;
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) {
#pragma unroll
        for (int x = 0; x < kSec; ++x) c[x] += __popcll(__ballot(sec[i] == x));
    }
    if (lane < kSec) {
        int mine = 0;
#pragma unroll
        for (int x = 0; x < kSec; ++x) mine = lane == x ? c[x] : mine;
        tcnt[lane * T + t] = mine;
    }
}

// Keys in layout order: key x * M + m (x <= 8) is section x's share of cut row m (its length is the
// distance between the places of the row's first tile and the next row's first tile in that
// section); key 9 * M + r is row r if it is not cut.  Length and non-empty flag of each; for the
// cut rows also the number of sections they have entries in.
__global__ __launch_bounds__(kBlock) void k_part_keys(const int32_t* __restrict__ rowptr, int64_t R, int64_t M, int64_t T,
                                                      const int32_t* __restrict__ m_of_row,
                                                      const int* __restrict__ tile_first, const int* __restrict__ toff,
                                                      int cut_entries, int* __restrict__ klen, int* __restrict__ kflag) {
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= kSec * M + R) return;
    int len;
    if (k < kSec * M) {
        const int64_t x = k / M, m = k - x * M;
        const int begin = toff[x * T + tile_first[m]];
        const int end = m + 1 < M ? toff[x * T + tile_first[m + 1]] : (x + 1 < kSec ? toff[(x + 1) * T] : cut_entries);
        len = end - begin;
    } else {
        const int64_t r = k - kSec * M;
        len = m_of_row[r] >= 0 ? 0 : rowptr[r + 1] - rowptr[r];
    }
    klen[k] = len;
    kflag[k] = len > 0 ? 1 : 0;
}

__global__ __launch_bounds__(kBlock) void k_part_pieces(const int* __restrict__ kflag, int64_t M, int* __restrict__ npieces,
                                                        unsigned long long* __restrict__ hot_entries,
                                                        const int* __restrict__ klen) {
    const int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    int pieces = 0, hot = 0;
    if (m < M) {
        for (int x = 0; x < kSec; ++x) {
            pieces += kflag[x * M + m];
            if (x < kHot) hot += klen[x * M + m];
        }
        npieces[m] = pieces;
    }
    // one addition per wavefront (all 64 lanes take part in the exchange)
    for (int d = 32; d > 0; d >>= 1) hot += __shfl_down(hot, d, 64);
    if (lane_id() == 0 && hot) atomicAdd(hot_entries, (unsigned long long)hot);
}

// Row pointer and target of every virtual row; vertex of every cut row; first entry of every section.
__global__ __launch_bounds__(kBlock) void k_part_vrows(int64_t R, int64_t M, int64_t T, const int32_t* __restrict__ srow,
                                                       const int32_t* __restrict__ row_ids,
                                                       const int* __restrict__ kflag, const int* __restrict__ voff,
                                                       const int* __restrict__ vidx, const int* __restrict__ toff,
                                                       const int* __restrict__ mptr, int n, int64_t n_vrows, int nnz,
                                                       int32_t* __restrict__ vptr, int32_t* __restrict__ tgt,
                                                       int32_t* __restrict__ mvert, int* __restrict__ sec_start) {
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k == 0) vptr[n_vrows] = nnz;
    if (k < kSec) sec_start[k] = toff[k * T];
    if (k < M) {
        const int32_t r = srow[k];
        mvert[k] = row_ids ? row_ids[r] : r;
    }
    if (k >= kSec * M + R || !kflag[k]) return;
    int t;
    if (k < kSec * M) {  // a cut row: partial row number = the row's first slot + sections before this one
        const int x = (int)(k / M);
        const int64_t m = k - (int64_t)x * M;
        int rank = 0;
        for (int y = 0; y < x; ++y) rank += kflag[y * M + m];
        t = n + mptr[m] + rank;
    } else {
        const int32_t r = (int32_t)(k - kSec * M);
        t = row_ids ? row_ids[r] : r;
    }
    const int j = vidx[k];
    vptr[j] = voff[k];
    tgt[j] = t;
}

// One wavefront per tile: every entry to its section, in the row's order; the last entry of the
// row's share of a section carries the row-end flag; the streamed-source mark survives only in the
// last section (the hot sections are gathered with plain loads throughout).  With `unstreamed` (one
// bit per source that stays unmarked) the marks are set here instead of being copied: the caller
// then need not mark the canonical array first, a pass over all entries of its own.
__global__ __launch_bounds__(kBlock) void k_part_scatter_cut(const int2v* __restrict__ cv,
                                                             const int32_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ srow,
                                                             const int32_t* __restrict__ tile_row,
                                                             const int* __restrict__ tile_first, int64_t M, int64_t T,
                                                             const unsigned int* __restrict__ hot,
                                                             const unsigned int* __restrict__ unstreamed,
                                                             const int* __restrict__ toff, const int* __restrict__ voff,
                                                             const int* __restrict__ klen, int2v* __restrict__ cv2,
                                                             const int* __restrict__ sec_off,
                                                             unsigned char* __restrict__ sec4) {
    const int64_t t = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = lane_id();
    const int32_t m = tile_row[t], r = srow[m];
    const int p0 = rowptr[r] + (int)(t - tile_first[m]) * kTile, p1 = min(p0 + kTile, rowptr[r + 1]);
    int next[kSec], end[kSec];
    {
        int b = 0, e = 0;
        if (lane < kSec) {
            b = toff[lane * T + t];
            e = voff[lane * M + m] + klen[lane * M + m];  // one past the row's share of the section
        }
#pragma unroll
        for (int x = 0; x < kSec; ++x) {
            next[x] = __shfl(b, x, 64);
            end[x] = __shfl(e, x, 64);
        }
    }
    int2v ent[kTile / 64];
    int sec[kTile / 64];
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) {
        const int j = p0 + i * 64 + lane;
        ent[i] = j < p1 ? cv[j] : int2v{-1, 0};
    }
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) sec[i] = ent[i].x != -1 ? section_of(ent[i].x & kColMask, hot) : -1;
#pragma unroll
    for (int i = 0; i < kTile / 64; ++i) {
        int dest = 0;
        bool last = false;
#pragma unroll
        for (int x = 0; x < kSec; ++x) {
            const unsigned long long mask = __ballot(sec[i] == x);
            if (sec[i] == x) {
                dest = next[x] + __popcll(mask & low_mask(lane));
                last = dest + 1 == end[x];
            }
            next[x] += __popcll(mask);
        }
        if (sec[i] >= 0) {
            int2v e = ent[i];
            int cold = e.x & kCold;
            if (unstreamed && sec[i] == kHot) {
                const int c = e.x & kColMask;
                cold = ((unstreamed[c >> 5] >> (c & 31)) & 1u) ? 0 : kCold;
            }
            e.x = (e.x & (kColMask | kOuterOnly)) | (sec[i] == kHot ? cold : 0) | (last ? kRowEnd : 0);
            cv2[dest] = e;
        }
        // the section ids, two to a byte (an even lane writes its own and its neighbour's): they are
        // what puts the entries back into the row's order later
        const int mine = sec[i] & 15;  // (-1 beyond the row's end -> 15, never read)
        const int both = mine | (__shfl_down(mine, 1, 64) << 4);
        const int j = (int)(t - tile_first[m]) * kTile + i * 64 + lane;  // entry index within the row
        if ((lane & 1) == 0 && p0 + i * 64 + lane < p1) sec4[sec_off[m] + (j >> 1)] = (unsigned char)both;
    }
}

// The reverse: the entries of the cut rows back in their rows' order (canonical entry array), from
// the recorded section ids; flags as the canonical array carries them (row end on the row's last
// entry; the streamed-source mark survives in the last section only, and hot sources never carry it).
__global__ __launch_bounds__(kBlock) void k_part_gather_cut(const int2v* __restrict__ cv2,
                                                            const int32_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ srow,
                                                            const int32_t* __restrict__ tile_row,
                                                            const int* __restrict__ tile_first, int64_t T,
                                                            const int* __restrict__ toff, const int* __restrict__ sec_off,
                                                            const unsigned char* __restrict__ sec4,
                                                            int2v* __restrict__ cv) {
    const int64_t t = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = lane_id();
    const int32_t m = tile_row[t], r = srow[m];
    const int p0 = rowptr[r] + (int)(t - tile_first[m]) * kTile, row_end = rowptr[r + 1], p1 = min(p0 + kTile, row_end);
    int next[kSec];
    {
        const int b = lane < kSec ? toff[lane * T + t] : 0;
#pragma unroll
        for (int x = 0; x < kSec; ++x) next[x] = __shfl(b, x, 64);
    }
    const unsigned char* __restrict__ ids = sec4 + sec_off[m] + ((int)(t - tile_first[m]) * kTile >> 1);
#pragma unroll 4
    for (int i = 0; i < kTile / 64; ++i) {
        const int j = p0 + i * 64 + lane;
        int sec = -1;
        if (j < p1) sec = (ids[(i * 64 + lane) >> 1] >> ((lane & 1) * 4)) & 15;
        int src = 0;
#pragma unroll
        for (int x = 0; x < kSec; ++x) {
            const unsigned long long mask = __ballot(sec == x);
            if (sec == x) src = next[x] + __popcll(mask & low_mask(lane));
            next[x] += __popcll(mask);
        }
        if (sec >= 0) {
            int2v e = cv2[src];
            e.x = (e.x & ~kRowEnd) | (j == row_end - 1 ? kRowEnd : 0);
            cv[j] = e;
        }
    }
}

// (Eight lanes per row: a row's entries are consecutive on both sides, so the lanes of a row move
// 64 contiguous bytes per step.)
constexpr int kRowLanes = 8;

__global__ __launch_bounds__(kBlock) void k_part_gather_whole(const int2v* __restrict__ cv2,
                                                              const int32_t* __restrict__ rowptr, int64_t R,
                                                              const int* __restrict__ whole_off, int2v* __restrict__ cv) {
    const int64_t r = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kRowLanes;
    if (r >= R || whole_off[r] < 0) return;
    const int p0 = rowptr[r], p1 = rowptr[r + 1];
    const int2v* __restrict__ src = cv2 + whole_off[r];
    for (int j = p0 + (threadIdx.x & (kRowLanes - 1)); j < p1; j += kRowLanes) cv[j] = src[j - p0];
}

// Rows that are not cut: copied to their place at the end of the last section, flags included; with
// `unstreamed` the streamed-source marks are set from that bitmap instead (see k_part_scatter_cut).
__global__ __launch_bounds__(kBlock) void k_part_scatter_whole(const int2v* __restrict__ cv,
                                                               const int32_t* __restrict__ rowptr, int64_t R, int64_t M,
                                                               const int32_t* __restrict__ m_of_row,
                                                               const int* __restrict__ voff,
                                                               const unsigned int* __restrict__ unstreamed,
                                                               int2v* __restrict__ cv2, int* __restrict__ whole_off) {
    const int64_t r = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kRowLanes;
    if (r >= R) return;
    const int sub = threadIdx.x & (kRowLanes - 1);
    if (m_of_row[r] >= 0) {
        if (sub == 0) whole_off[r] = -1;
        return;
    }
    const int p0 = rowptr[r], p1 = rowptr[r + 1];
    const int at = voff[kSec * M + r];
    if (sub == 0) whole_off[r] = at;
    int2v* __restrict__ d = cv2 + at;
    for (int j = p0 + sub; j < p1; j += kRowLanes) {
        int2v e = cv[j];
        if (unstreamed) {
            const int c = e.x & kColMask;
            e.x = (e.x & ~kCold) | (((unstreamed[c >> 5] >> (c & 31)) & 1u) ? 0 : kCold);
        }
        d[j - p0] = e;
    }
}

inline unsigned grid_for(int64_t n, int per_block) { return (unsigned)std::max<int64_t>((n + per_block - 1) / per_block, 1); }

int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : dflt;
}

}  // namespace

int epp_partition_hot_rows(int F) {
    // what the eight L2s hold together when each keeps 3.5 of its 4 MB for source rows
    const int64_t kb_per_xcd = env_int("EPP_TUNE_PART_KB", 3584);
    return (int)std::min<int64_t>(kHot * kb_per_xcd * 1024 / ((int64_t)F * 4), 1 << 30);
}

int epp_build_partition(epp_path* p, int F, int gs, const unsigned int* hot_bitmap, const unsigned int* unstreamed,
                        hipStream_t s, Partition** out) {
    *out = nullptr;
    const int mode = env_int("EPP_TUNE_PART", 1);  // 0: never, 1: where it pays, 2: always (tests)
    if (mode == 0 || p->nnz == 0 || p->n_stream_rows == 0) return EPP_OK;
    const int min_len = std::max(env_int("EPP_TUNE_PART_MINLEN", 96), 1);
    const int64_t R = p->n_stream_rows, nnz = p->nnz;
    const epp_alloc_t* al = epp_alloc_of(p);
    const int32_t* rowptr = p->rowptr.as<int32_t>();
    const int2v* cv = reinterpret_cast<const int2v*>(p->cv.p);

    // ---- which rows to cut
    DevArena a1;
    DevBuf flag, midx, scan_tmp, totals, m_of_row;
    EPP_TRY(a1.reserve(3 * DevArena::rounded((size_t)R * 4) + DevArena::rounded(epp_scan_tmp_bytes(R)) +
                       DevArena::rounded(64), al));
    a1.take(&flag, (size_t)R * 4);
    a1.take(&midx, (size_t)R * 4);
    a1.take(&m_of_row, (size_t)R * 4);
    a1.take(&scan_tmp, epp_scan_tmp_bytes(R));
    // [0] cut rows, [1] tiles, [2] entries of cut rows, [3] hot entries, [4] partial rows, [5] all entries,
    // [6] virtual rows, [7] bytes of the recorded section ids
    a1.take(&totals, 8 * sizeof(long long));
    EPP_HIP_TRY(hipMemsetAsync(totals.p, 0, totals.bytes, s));
    long long* d_tot = totals.as<long long>();
    long long h_tot[8] = {};
    hipLaunchKernelGGL(k_part_flag_rows, dim3(grid_for(R, kBlock)), dim3(kBlock), 0, s, rowptr, R, min_len, flag.as<int>());
    epp_scan_exclusive(flag.as<int>(), midx.as<int>(), R, d_tot, scan_tmp.as<int>(), s);
    EPP_HIP_TRY(hipGetLastError());
    EPP_HIP_TRY(hipMemcpyAsync(h_tot, d_tot, sizeof(long long), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    const int64_t M = h_tot[0];
    if (M == 0) return EPP_OK;  // no long rows: nothing to move

    // ---- tiles of the cut rows
    DevArena a2;
    DevBuf srow, ntiles, tile_first, npieces, mptr_tmp, nbytes, sec_off;
    EPP_TRY(a2.reserve(7 * DevArena::rounded((size_t)(M + 1) * 4), al));
    a2.take(&srow, (size_t)M * 4);
    a2.take(&ntiles, (size_t)M * 4);
    a2.take(&tile_first, (size_t)M * 4);
    a2.take(&npieces, (size_t)M * 4);
    a2.take(&mptr_tmp, (size_t)(M + 1) * 4);
    a2.take(&nbytes, (size_t)M * 4);
    a2.take(&sec_off, (size_t)M * 4);
    hipLaunchKernelGGL(k_part_list_rows, dim3(grid_for(R, kBlock)), dim3(kBlock), 0, s, flag.as<int>(), midx.as<int>(), R,
                       srow.as<int32_t>(), m_of_row.as<int32_t>());
    hipLaunchKernelGGL(k_part_tiles_per_row, dim3(grid_for(M, kBlock)), dim3(kBlock), 0, s, rowptr, srow.as<int32_t>(), M,
                       ntiles.as<int>(), nbytes.as<int>());
    epp_scan_exclusive(ntiles.as<int>(), tile_first.as<int>(), M, d_tot + 1, scan_tmp.as<int>(), s);
    epp_scan_exclusive(nbytes.as<int>(), sec_off.as<int>(), M, d_tot + 7, scan_tmp.as<int>(), s);
    EPP_HIP_TRY(hipGetLastError());
    EPP_HIP_TRY(hipMemcpyAsync(h_tot + 1, d_tot + 1, sizeof(long long), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipMemcpyAsync(h_tot + 7, d_tot + 7, sizeof(long long), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    const int64_t T = h_tot[1], sec_bytes = h_tot[7];

    // ---- entries per (section, tile), their places, the keys; is it worth it?
    const int64_t K = kSec * M + R;
    DevArena a3;
    DevBuf tile_row, tcnt, toff, klen, kflag, voff, vidx, scan_tmp2, sec_start;
    EPP_TRY(a3.reserve(DevArena::rounded((size_t)T * 4) + 2 * DevArena::rounded((size_t)kSec * T * 4) +
                       4 * DevArena::rounded((size_t)K * 4) + DevArena::rounded(epp_scan_tmp_bytes(std::max(K, kSec * T))) +
                       DevArena::rounded(64), al));
    a3.take(&tile_row, (size_t)T * 4);
    a3.take(&tcnt, (size_t)kSec * T * 4);
    a3.take(&toff, (size_t)kSec * T * 4);
    a3.take(&klen, (size_t)K * 4);
    a3.take(&kflag, (size_t)K * 4);
    a3.take(&voff, (size_t)K * 4);
    a3.take(&vidx, (size_t)K * 4);
    a3.take(&scan_tmp2, epp_scan_tmp_bytes(std::max(K, kSec * T)));
    a3.take(&sec_start, kSec * sizeof(int));
    hipLaunchKernelGGL(k_part_tile_rows, dim3(grid_for(M, kBlock / 64)), dim3(kBlock), 0, s, tile_first.as<int>(),
                       ntiles.as<int>(), M, tile_row.as<int32_t>());
    hipLaunchKernelGGL(k_part_count, dim3(grid_for(T, kBlock / 64)), dim3(kBlock), 0, s, cv, rowptr, srow.as<int32_t>(),
                       tile_row.as<int32_t>(), tile_first.as<int>(), T, hot_bitmap, tcnt.as<int>());
    epp_scan_exclusive(tcnt.as<int>(), toff.as<int>(), kSec * T, d_tot + 2, scan_tmp2.as<int>(), s);
    EPP_HIP_TRY(hipGetLastError());
    EPP_HIP_TRY(hipMemcpyAsync(h_tot + 2, d_tot + 2, sizeof(long long), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));  // (the key lengths need the number of entries in cut rows)
    const int64_t cut_entries = h_tot[2];
    hipLaunchKernelGGL(k_part_keys, dim3(grid_for(K, kBlock)), dim3(kBlock), 0, s, rowptr, R, M, T, m_of_row.as<int32_t>(),
                       tile_first.as<int>(), toff.as<int>(), (int)cut_entries, klen.as<int>(), kflag.as<int>());
    hipLaunchKernelGGL(k_part_pieces, dim3(grid_for(M, kBlock)), dim3(kBlock), 0, s, kflag.as<int>(), M, npieces.as<int>(),
                       reinterpret_cast<unsigned long long*>(d_tot + 3), klen.as<int>());
    epp_scan_exclusive(npieces.as<int>(), mptr_tmp.as<int>(), M, d_tot + 4, scan_tmp.as<int>(), s);
    epp_scan_exclusive(klen.as<int>(), voff.as<int>(), K, d_tot + 5, scan_tmp2.as<int>(), s);
    epp_scan_exclusive(kflag.as<int>(), vidx.as<int>(), K, d_tot + 6, scan_tmp2.as<int>(), s);
    EPP_HIP_TRY(hipGetLastError());
    EPP_HIP_TRY(hipMemcpyAsync(h_tot + 3, d_tot + 3, 4 * sizeof(long long), hipMemcpyDeviceToHost, s));
    EPP_HIP_TRY(hipStreamSynchronize(s));
    const int64_t hot_entries = h_tot[3], n_slots = h_tot[4], n_vrows = h_tot[6];
    if (h_tot[5] != nnz) { epp_set_error("partition: %lld entries placed, the path has %lld", h_tot[5], (long long)nnz); return EPP_ERR_HIP; }
    // A gather served by L2 costs a quarter of one served from beyond it; a partial row is written
    // once and read once.  Measured on an MI355X at 512-byte rows: a path with 42 % of its entries in
    // hot sections and 1.3 % as many partial rows as entries runs 14 % faster, one with 13 % / 0.9 %
    // gains 2 %, one with 28 % / 7 % loses 14 %.  The layout is built when the modelled saving,
    // 0.75 hot - 2.5 partial rows (in gathers), exceeds a fifth of the entries.
    const double score = (0.75 * (double)hot_entries - 2.5 * (double)n_slots) / (double)nnz;
    if (mode == 1 && score < 0.20) return EPP_OK;
    if (p->n + n_slots >= 0x7FFFFFFFll) return EPP_OK;  // targets are 31-bit

    Partition* q = new Partition();
    struct Guard { Partition* q; ~Guard() { delete q; } } guard{q};
    q->n_vrows = n_vrows;
    q->n_split = M;
    q->n_slots = n_slots;
    q->hot_entries = hot_entries;
    EPP_TRY(q->cv2.alloc((size_t)nnz * 8, al));
    EPP_TRY(q->vptr.alloc((size_t)(n_vrows + 1) * 4, al));
    EPP_TRY(q->tgt.alloc((size_t)n_vrows * 4, al));
    EPP_TRY(q->mvert.alloc((size_t)M * 4, al));
    EPP_TRY(q->mptr.alloc((size_t)(M + 1) * 4, al));
    // kept for putting the entries back into canonical order
    q->n_tiles = T;
    EPP_TRY(q->srow.alloc((size_t)M * 4, al));
    EPP_TRY(q->tile_first.alloc((size_t)M * 4, al));
    EPP_TRY(q->sec_off.alloc((size_t)M * 4, al));
    EPP_TRY(q->tile_row.alloc((size_t)T * 4, al));
    EPP_TRY(q->toff.alloc((size_t)kSec * T * 4, al));
    EPP_TRY(q->sec4.alloc((size_t)sec_bytes, al));
    EPP_TRY(q->whole_off.alloc((size_t)R * 4, al));
    EPP_HIP_TRY(hipMemcpyAsync(q->srow.p, srow.p, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipMemcpyAsync(q->tile_first.p, tile_first.p, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipMemcpyAsync(q->sec_off.p, sec_off.p, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipMemcpyAsync(q->tile_row.p, tile_row.p, (size_t)T * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipMemcpyAsync(q->toff.p, toff.p, (size_t)kSec * T * 4, hipMemcpyDeviceToDevice, s));
    {   // the partial rows live in the scratch the handle's paths share
        void* scratch = nullptr;
        EPP_TRY(p->pool->get((size_t)n_slots * (size_t)F * 4, al, &scratch));
        if (!p->pool->accounted_by) p->pool->accounted_by = p;
        q->vpart = static_cast<float*>(scratch);
    }
    // the scan left mptr[0 .. M-1]; its last element is the total
    EPP_HIP_TRY(hipMemcpyAsync(q->mptr.p, mptr_tmp.p, (size_t)M * 4, hipMemcpyDeviceToDevice, s));
    EPP_HIP_TRY(hipMemcpyAsync(q->mptr.as<int32_t>() + M, d_tot + 4, 4, hipMemcpyDeviceToDevice, s));  // (little endian)
    const int32_t* row_ids = p->row_ids.p ? p->row_ids.as<int32_t>() : nullptr;
    hipLaunchKernelGGL(k_part_vrows, dim3(grid_for(K, kBlock)), dim3(kBlock), 0, s, R, M, T, srow.as<int32_t>(), row_ids,
                       kflag.as<int>(), voff.as<int>(), vidx.as<int>(), toff.as<int>(), q->mptr.as<int32_t>(), (int)p->n,
                       n_vrows, (int)nnz, q->vptr.as<int32_t>(), q->tgt.as<int32_t>(), q->mvert.as<int32_t>(),
                       sec_start.as<int>());
    hipLaunchKernelGGL(k_part_scatter_cut, dim3(grid_for(T, kBlock / 64)), dim3(kBlock), 0, s, cv, rowptr,
                       srow.as<int32_t>(), tile_row.as<int32_t>(), tile_first.as<int>(), M, T, hot_bitmap, unstreamed,
                       toff.as<int>(),
                       voff.as<int>(), klen.as<int>(), reinterpret_cast<int2v*>(q->cv2.p), sec_off.as<int>(),
                       q->sec4.as<unsigned char>());
    hipLaunchKernelGGL(k_part_scatter_whole, dim3(grid_for(R * kRowLanes, kBlock)), dim3(kBlock), 0, s, cv, rowptr, R, M,
                       m_of_row.as<int32_t>(), voff.as<int>(), unstreamed, reinterpret_cast<int2v*>(q->cv2.p),
                       q->whole_off.as<int>());
    EPP_HIP_TRY(hipGetLastError());
    int h_sec[kSec];
    EPP_HIP_TRY(hipMemcpyAsync(h_sec, sec_start.p, sizeof(h_sec), hipMemcpyDeviceToHost, s));
    EPP_TRY(epp_build_schedule_over(p, q->vptr.as<int32_t>(), n_vrows, nnz, gs, s, &q->sched));  // synchronises
    EPP_TRY(q->sched->ensure_pieces(F, al));
    q->sec_g[0] = 0;
    for (int x = 1; x < kSec; ++x) q->sec_g[x] = (int)(((int64_t)h_sec[x] + gs - 1) / gs);
    q->sec_g[kSec] = (int)q->sched->n_groups;
    guard.q = nullptr;
    *out = q;
    return EPP_OK;
}

// The canonical entry array of a path is only read when a width is prepared, by launches of a width
// without a reconstructed copy, and by epp_path_export.  While every prepared width of a path
// (other than the all-active graph, which also serves the if-else baseline) runs on its reconstructed
// copy, the canonical array is given back to the allocator; it is rebuilt from a copy, bit for bit,
// the next time one of those needs it.
bool epp_canonical_unused(const epp_path* p, int F_with_copy) {
    const char* e = std::getenv("EPP_TUNE_KEEP_CANONICAL");
    if (e && e[0] == '1') return false;
    if (p->all_rows || !p->cv.p || !p->cv.owned) return false;
    bool any = F_with_copy > 0;
    for (const auto& w : p->widths) {
        if (w.F == F_with_copy) continue;
        if (w.sched && !w.part) return false;  // a width that launches on the canonical array
        any |= (w.part != nullptr);
    }
    return any;
}

void epp_release_canonical_if_unused(epp_path* p) {
    if (epp_canonical_unused(p, 0)) p->cv.release();
}

int epp_ensure_canonical(epp_path* p, hipStream_t s) {
    if (p->cv.p || p->nnz == 0) return EPP_OK;
    const Partition* q = nullptr;
    for (const auto& w : p->widths)
        if (w.part) q = w.part;
    if (!q) { epp_set_error("the path has no entry array"); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(p->cv.alloc((size_t)p->nnz * 8, epp_alloc_of(p)));
    const int2v* cv2 = reinterpret_cast<const int2v*>(q->cv2.p);
    int2v* cv = reinterpret_cast<int2v*>(p->cv.p);
    hipLaunchKernelGGL(k_part_gather_cut, dim3(grid_for(q->n_tiles, kBlock / 64)), dim3(kBlock), 0, s, cv2,
                       p->rowptr.as<int32_t>(), q->srow.as<int32_t>(), q->tile_row.as<int32_t>(), q->tile_first.as<int>(),
                       q->n_tiles, q->toff.as<int>(), q->sec_off.as<int>(), q->sec4.as<unsigned char>(), cv);
    hipLaunchKernelGGL(k_part_gather_whole, dim3(grid_for(p->n_stream_rows * kRowLanes, kBlock)), dim3(kBlock), 0, s, cv2,
                       p->rowptr.as<int32_t>(), p->n_stream_rows, q->whole_off.as<int>(), cv);
    EPP_HIP_TRY(hipGetLastError());
    return EPP_OK;
}
