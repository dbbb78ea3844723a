// Internal declarations shared by the translation units of libepp (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "epp.h"

#define EPP_NCLASS 32

// An entry of a path is the pair (column word, weight bits).  The column word holds the source's
// vertex id in its low 29 bits and three flags:
constexpr int kEntRowEnd = (int)0x80000000u;  // last entry of its row
constexpr int kEntCold = 0x40000000;           // rarely referenced source: gathered with streaming loads
constexpr int kEntOuterOnly = 0x20000000;      // not an entry of the inner path that shares this array (below)
constexpr int kEntCol = 0x1FFFFFFF;
constexpr long long kMaxVertices = 0x20000000ll;  // vertex ids must leave the flag bits free

void epp_set_error(const char* fmt, ...);

#define EPP_HIP_TRY(expr)                                                                           \
    do {                                                                                            \
        hipError_t epp_e_ = (expr);                                                                 \
        if (epp_e_ != hipSuccess) {                                                                 \
            epp_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(epp_e_), __FILE__,      \
                          __LINE__);                                                                \
            return EPP_ERR_HIP;                                                                     \
        }                                                                                           \
    } while (0)

#define EPP_TRY(expr)                  \
    do {                               \
        int epp_rc_ = (expr);          \
        if (epp_rc_ != EPP_OK) return epp_rc_; \
    } while (0)

// Device allocation that frees itself; `bytes` is kept for the footprint report.  The memory
// comes from the caller's allocator (epp_alloc_t, the handle keeps a copy) or, without one, from
// hipMalloc.  A buffer can also be a view of part of another allocation (temporaries carved from
// one arena: every hipMalloc / hipFree pair costs about 0.15 ms, hipFree waits for the device).
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    bool owned = true;
    epp_alloc_t via = {nullptr, nullptr, nullptr};  // allocator that owns p (alloc == NULL: hipMalloc)
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    DevBuf(DevBuf&& o) noexcept : p(o.p), bytes(o.bytes), owned(o.owned), via(o.via) { o.p = nullptr; o.bytes = 0; }
    DevBuf& operator=(DevBuf&& o) noexcept {
        if (this != &o) { release(); p = o.p; bytes = o.bytes; owned = o.owned; via = o.via; o.p = nullptr; o.bytes = 0; }
        return *this;
    }
    ~DevBuf() { release(); }
    int alloc(size_t n, const epp_alloc_t* a) {
        release();
        if (n == 0) n = 4;  // keep a valid pointer for empty arrays
        if (a && a->alloc && a->free) {
            p = a->alloc(n, a->ctx);
            if (!p || (reinterpret_cast<uintptr_t>(p) & 255)) {
                if (p) a->free(p, a->ctx);
                p = nullptr;
                epp_set_error("the caller's allocator gave no 256-byte aligned block of %zu bytes", n);
                return EPP_ERR_ALLOC;
            }
            via = *a;
        } else {
            if (hipMalloc(&p, n) != hipSuccess) {
                (void)hipGetLastError();
                p = nullptr;
                epp_set_error("device allocation of %zu bytes failed", n);
                return EPP_ERR_ALLOC;
            }
            via = {nullptr, nullptr, nullptr};
        }
        bytes = n;
        owned = true;
        return EPP_OK;
    }
    void view(void* ptr, size_t n) {  // memory owned by someone who outlives this view
        release();
        p = ptr;
        bytes = n;
        owned = false;
    }
    void release() {
        if (p && owned) {
            if (via.alloc) via.free(p, via.ctx);
            else (void)hipFree(p);
        }
        p = nullptr;
        bytes = 0;
        owned = true;
    }
    template <class T> T* as() const { return static_cast<T*>(p); }
};

// Bump allocator over one device allocation (256-byte aligned pieces).
struct DevArena {
    DevBuf store;
    size_t used = 0;
    static size_t rounded(size_t n) { return (std::max<size_t>(n, 4) + 255) & ~(size_t)255; }
    int reserve(size_t total, const epp_alloc_t* a) { used = 0; return store.alloc(total, a); }
    void take(DevBuf* b, size_t n) {
        b->view(static_cast<char*>(store.p) + used, n);
        used += rounded(n);
    }
};

// Group table of one path for one group size gs (neighbour grouping, Sec. 2.2): the path's
// entry array is cut into groups of gs consecutive entries; group g covers entries
// [g * gs, min((g + 1) * gs, nnz)).
struct Schedule {
    int gs = 0;
    int64_t n_groups = 0;
    int64_t n_split_rows = 0;  // rows cut by a group boundary (summed from the groups' partial rows)
    DevBuf group_row;          // int32[n_groups] row holding the group's first entry; bit 31: starts inside it
    DevBuf cut_rows;           // int32[n_split_rows] (path-row indices)
    // Partial rows of the groups, per width F: float[n_groups][2][F].  Slot 0 of a group holds the
    // sum of the tail of a row that began in an earlier group, slot 1 the sum of the row still
    // open at the group's end.  Written by every launch before it is read; sized at schedule time
    // so that a launch never allocates.
    struct Pieces { int F; DevBuf buf; };
    std::vector<Pieces*> pieces;
    ~Schedule() { for (Pieces* q : pieces) delete q; }
    float* pieces_for(int F) const {
        for (const Pieces* q : pieces)
            if (q->F == F) return q->buf.as<float>();
        return nullptr;
    }
    int ensure_pieces(int F, const epp_alloc_t* a) {
        if (pieces_for(F) || n_split_rows == 0) return EPP_OK;
        Pieces* q = new Pieces();
        q->F = F;
        if (q->buf.alloc((size_t)n_groups * 2 * (size_t)F * sizeof(float), a) != EPP_OK) { delete q; return EPP_ERR_ALLOC; }
        pieces.push_back(q);
        return EPP_OK;
    }
    void drop_pieces(int F) {  // (hipFree waits for the device; a caller's allocator must be stream-ordered)
        for (size_t i = 0; i < pieces.size(); ++i)
            if (pieces[i]->F == F) { delete pieces[i]; pieces.erase(pieces.begin() + i); return; }
    }
    size_t bytes() const {
        size_t b = group_row.bytes + cut_rows.bytes;
        for (const Pieces* q : pieces) b += q->buf.bytes;
        return b;
    }
};

// Scratch memory of a launch that the paths of one handle share: a handle is used by one call at
// a time, so two of its paths never need their scratch at once.  Buffers only ever get added (a
// captured HIP graph may hold the address of an older one); a request is served by the smallest
// buffer that is large enough, else by a new one, sized an eighth above the request at most so
// that paths of nearly equal size end up on one buffer.
struct ScratchPool {
    std::vector<DevBuf*> bufs;
    const void* accounted_by = nullptr;  // the path whose footprint report includes the pool
    ~ScratchPool() { for (DevBuf* b : bufs) delete b; }
    int get(size_t bytes, const epp_alloc_t* al, void** out) {
        DevBuf* best = nullptr;
        for (DevBuf* b : bufs)
            if (b->bytes >= bytes && (!best || b->bytes < best->bytes)) best = b;
        if (!best) {
            size_t step = 256;
            while (step * 16 <= bytes) step *= 2;  // an eighth of the leading power of two
            best = new DevBuf();
            if (best->alloc((bytes + step - 1) / step * step, al) != EPP_OK) { delete best; return EPP_ERR_ALLOC; }
            bufs.push_back(best);
        }
        *out = best->p;
        return EPP_OK;
    }
    size_t bytes() const {
        size_t b = 0;
        for (const DevBuf* x : bufs) b += x->bytes;
        return b;
    }
};

// Source-partitioned layout of a path for one width ("reconstructed" execution path, Sec. 6's
// pre-processing step, re-derived for a GPU of 8 XCDs with private L2s).  The entries of the long
// rows whose source is among the most referenced ones are moved into 8 sections by partition of the
// source; section x is processed by XCD x only, whose L2 then holds only the source rows of
// partition x.  All other entries form the last section.  A row that has entries in several
// sections becomes one virtual row per section; each writes a partial row to `vpart`, and a last
// kernel adds a vertex's partial rows in section order.
struct Partition {
    DevBuf cv2;        // int2[nnz] entries, section after section, canonical order inside a section
    DevBuf vptr;       // int32[n_vrows + 1] entry range of every virtual row
    DevBuf tgt;        // int32[n_vrows] vertex id (< n) or n + slot in vpart
    int64_t n_vrows = 0;
    DevBuf mvert;      // int32[n_split] vertex of every row that is cut into sections
    DevBuf mptr;       // int32[n_split + 1] its slots in vpart
    int64_t n_split = 0, n_slots = 0;
    float* vpart = nullptr;  // float[n_slots][F], in the handle's scratch pool
    // what is needed to put the entries back into canonical order (the path may give its canonical
    // entry array back while every prepared width runs on a reconstructed copy)
    DevBuf srow, tile_first, tile_row;  // cut rows, their first tile, the row of every tile
    DevBuf toff;       // int32[9 * n_tiles] place of every tile in every section
    DevBuf sec4;       // section of every entry of the cut rows, 4 bits each, rows byte-aligned
    DevBuf sec_off;    // int32[n_split] first byte of a cut row in sec4
    DevBuf whole_off;  // int32[rows] place of a row that is not cut (-1: cut)
    int64_t n_tiles = 0;
    int sec_g[10] = {};    // first group of every section, then n_groups
    int64_t hot_entries = 0;  // entries in the eight hot sections
    Schedule* sched = nullptr;  // groups over (vptr, cv2)
    ~Partition() { delete sched; }
    size_t bytes() const {
        return cv2.bytes + vptr.bytes + tgt.bytes + mvert.bytes + mptr.bytes + srow.bytes + tile_first.bytes +
               tile_row.bytes + toff.bytes + sec4.bytes + sec_off.bytes + whole_off.bytes + (sched ? sched->bytes() : 0);
    }
};

struct epp_path {
    int64_t n = 0;       // vertices of the input graph
    int64_t n_rows = 0;  // R: rows of the path in canonical form (all-active graph: n)
    int64_t nnz = 0;
    int64_t n_src = 0;
    int64_t max_len = 0;
    int64_t len_hist[EPP_NCLASS] = {};
    bool all_rows = false;       // all-active graph (handle from epp_prepare_full)
    // Streamed form: only rows with at least one entry, in ascending vertex order.
    int64_t n_stream_rows = 0;
    DevBuf store;                // one allocation behind row_ids, rowptr and cv where they are views of it
    DevBuf row_ids;              // int32[n_stream_rows] vertex of each streamed row; unset: identity
    DevBuf rowptr;               // int32[n_stream_rows + 1]
    DevBuf cv;                   // int2[nnz]: (column word, weight bits)
    // Shared entries (Sec. 4: consecutive execution paths of a model overlap almost entirely once the
    // active sets approach saturation).  With N^{k-1} inside N^k, every entry of the path one level
    // further in is an entry of this one, in the same order.  Such an inner path can do without entry
    // arrays of its own: it keeps its row ids and row pointer (canonical form, export, combination
    // stage) and runs on this path's arrays, group tables and reconstructed copies, skipping the
    // entries that carry kEntOuterOnly and the rows left without any entry.
    epp_path* outer = nullptr;            // set on the inner path: the path whose entries it shares
    const unsigned int* inner_rows = nullptr;  // set on the inner path: bitmap of its rows (owned by the handle)
    bool has_inner = false;               // set on the outer path: kEntOuterOnly marks are in place
    DevBuf zero_block;                    // outer path: 256 zero bytes, what a skipped entry gathers
    int cold_thr = 0;            // entries whose source is referenced fewer times than this carry the cold flag
    int cold_F = 0;              // width the cold flags were chosen for (the largest prepared width that marks)
    epp_alloc_t alloc = {nullptr, nullptr, nullptr};  // the caller's allocator (alloc == NULL: hipMalloc)
    ScratchPool own_pool;        // launch scratch of a path that belongs to no epp_paths handle
    ScratchPool* pool = &own_pool;  // the handle's pool for the paths of an epp_paths handle
    // all-active graph only
    DevBuf full_rowptr;          // int32[n + 1] as given (for export)
    int64_t n_empty_rows = 0;
    DevBuf empty_rows;           // int32[n_empty_rows] vertices with empty lists
    std::vector<Schedule*> scheds;
    // per-width choices
    // sched == NULL: the width has not been prepared (epp_path_prepare_width); slices: XCD feature slicing
    // part: source-partitioned layout of this width, if it pays (owned by the path)
    struct WidthCfg { int F; int forced_gs; Schedule* sched; int log2_slices; Partition* part; };
    std::vector<WidthCfg> widths;
    int last_F = 0;
    ~epp_path() {
        for (Schedule* s : scheds) delete s;
        for (auto& w : widths) delete w.part;
    }
};

struct epp_paths {
    int L = 0;
    int64_t n = 0;
    std::vector<DevBuf> bitmaps;    // L+1 bitmaps of N^k, uint64 words
    std::vector<int64_t> set_size;  // |N^k|
    std::vector<epp_path*> path;    // index l; once the sets stop growing, deeper layers share one object
    DevBuf set0_ids;                // ascending ids of N^0 (the other sets are path rows)
    DevBuf small_store;             // small graphs: the one allocation that all arrays above are views of
    ScratchPool pool;               // launch scratch shared by the paths
    epp_alloc_t alloc = {nullptr, nullptr, nullptr};
    ~epp_paths() {
        for (size_t i = 0; i < path.size(); ++i) {
            bool seen = false;
            for (size_t j = 0; j < i; ++j) seen |= (path[j] == path[i]);
            if (!seen) delete path[i];
        }
    }
};

// prepare.hip
// histogram + max length of a built path; `stats_scratch`: (EPP_NCLASS + 1) * 8 device bytes, or NULL
// `host_later` (pinned host memory, EPP_NCLASS + 1 words): the statistics are copied there
// without waiting; the caller hands them to epp_path_set_stats after it has synchronised
// mark_row_ends = false: the entry array is not there yet (the caller marks the row ends itself)
int epp_path_finish(epp_path* p, hipStream_t s, void* stats_scratch = nullptr, unsigned long long* host_later = nullptr,
                    bool mark_row_ends = true);
void epp_path_set_stats(epp_path* p, const unsigned long long* host);
// ascending vertex ids of N^k (device, owned by `p`); allocates nothing, never waits
int epp_active_ids(const epp_paths* p, int k, const int32_t** ids, int64_t* count);

// prepare_small.hip: the whole construction in one launch, for graphs of at most 65,536 vertices and 131,072 entries
bool epp_prepare_small_fits(const epp_csr_t* g, int64_t n_train, int L);
int epp_prepare_small(const epp_csr_t* g, const int32_t* train_ids, int64_t n_train, int L, const epp_alloc_t* alloc,
                      hipStream_t s, epp_paths_t** out);

// combine.hip
// device address of the static scratch array on the current GPU (symbol lookup once per device;
// no allocation).  Handles are created with the GPU current, so they resolve it up front.
int epp_static_scratch(float** ptr);

// aggregate.hip
int epp_build_schedule(epp_path* p, int gs, hipStream_t s, Schedule** out);
// inner_rows != NULL: the launch serves the inner path that shares p's entries (bitmap of its rows)
int epp_launch_aggregate(epp_path* p, Schedule* sc, int log2_slices, const float* in, float* out, int F, hipStream_t s,
                         const unsigned int* row_bits = nullptr, const unsigned int* src_bits = nullptr,
                         const Partition* part = nullptr, const unsigned int* inner_rows = nullptr);
// group table over any (row pointer, entry count); not registered with the path
int epp_build_schedule_over(const epp_path* p, const int32_t* rowptr, int64_t n_rows, int64_t nnz, int gs, hipStream_t s,
                            Schedule** out);
int epp_default_group_size(const epp_path* p, int F);
int epp_tune_locality(epp_path* p, int F, int gs, hipStream_t s, int* log2_slices, Partition** part);

// partition.hip
int epp_partition_hot_rows(int F);  // source rows of width F the eight L2s hold together
// source-partitioned layout of `p` for width F and group size gs, or *out = NULL where it does not pay
// `unstreamed` (or NULL): bitmap of the sources whose entries stay unmarked in the last section; the
// copy then sets the streamed-source marks itself, whatever the canonical array carries
int epp_build_partition(epp_path* p, int F, int gs, const unsigned int* hot_bitmap, const unsigned int* unstreamed,
                        hipStream_t s, Partition** out);

// partition.hip: canonical entry array of `p` rebuilt from a reconstructed copy, if it was given back
int epp_ensure_canonical(epp_path* p, hipStream_t s);
// gives the canonical entry array back if every prepared width runs on a reconstructed copy
void epp_release_canonical_if_unused(epp_path* p);
// would it be given back if width F_with_copy (0: none) had a reconstructed copy and were prepared?
bool epp_canonical_unused(const epp_path* p, int F_with_copy);

// prepare.hip: exclusive scan of n ints (*total, device, receives the sum); tmp: epp_scan_tmp_bytes(n)
size_t epp_scan_tmp_bytes(int64_t n);
void epp_scan_exclusive(const int* in, int* out, int64_t n, long long* total, int* tmp, hipStream_t s);
inline const epp_alloc_t* epp_alloc_of(const epp_path* p) { return p->alloc.alloc ? &p->alloc : nullptr; }
inline const epp_alloc_t* epp_alloc_of(const epp_paths* p) { return p->alloc.alloc ? &p->alloc : nullptr; }
