// Internal declarations shared by the translation units of libepp (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

#include "epp.h"

#define EPP_NCLASS 32

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

// Device allocation that frees itself; `bytes` is kept for the footprint report.
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    DevBuf() = default;
    DevBuf(const DevBuf&) = delete;
    DevBuf& operator=(const DevBuf&) = delete;
    DevBuf(DevBuf&& o) noexcept : p(o.p), bytes(o.bytes) { o.p = nullptr; o.bytes = 0; }
    DevBuf& operator=(DevBuf&& o) noexcept {
        if (this != &o) { release(); p = o.p; bytes = o.bytes; o.p = nullptr; o.bytes = 0; }
        return *this;
    }
    ~DevBuf() { release(); }
    int alloc(size_t n) {
        release();
        if (n == 0) n = 4;  // keep a valid pointer for empty arrays
        if (hipMalloc(&p, n) != hipSuccess) {
            (void)hipGetLastError();
            p = nullptr;
            epp_set_error("device allocation of %zu bytes failed", n);
            return EPP_ERR_ALLOC;
        }
        bytes = n;
        return EPP_OK;
    }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
        bytes = 0;
    }
    template <class T> T* as() const { return static_cast<T*>(p); }
};

// Group table of one path for one group size gs (neighbour grouping, Sec. 2.2): every row
// is cut into consecutive groups of at most gs entries.  Groups are binned by length class
// (class c holds lengths in (2^(c-1), 2^c], class 0 lengths 0 and 1) so that a wavefront
// only ever works on groups of similar length.
struct Schedule {
    int gs = 0;
    int64_t n_groups = 0;
    int64_t n_split_rows = 0;
    int64_t class_count[EPP_NCLASS] = {};  // groups per class
    int64_t class_begin[EPP_NCLASS] = {};  // first group of the class in the arrays below
    DevBuf g_start;    // int32[n_groups]  first entry of the group in cv
    DevBuf g_len;      // int32[n_groups]  entries; bit 31 set: row is split -> atomic write-back
    DevBuf g_dst;      // int32[n_groups]  destination vertex
    DevBuf split_dst;  // int32[n_split_rows]  vertices whose rows must be zeroed before atomics
    size_t bytes() const { return g_start.bytes + g_len.bytes + g_dst.bytes + split_dst.bytes; }
};

struct epp_path {
    int64_t n = 0;       // vertices of the input graph
    int64_t n_rows = 0;  // R
    int64_t nnz = 0;
    int64_t n_src = 0;
    int64_t max_len = 0;
    int64_t len_hist[EPP_NCLASS] = {};
    bool all_rows = false;  // all-active graph: row r is vertex r, row_ids unused
    DevBuf row_ids;         // int32[R] ascending vertex ids
    DevBuf rowptr;          // int32[R+1]
    DevBuf cv;              // int2[nnz]: (column id, weight bits) interleaved
    std::vector<Schedule*> scheds;
    // per-width choices
    struct WidthCfg { int F; int forced_gs; int lanes_hint; Schedule* sched; };
    std::vector<WidthCfg> widths;
    int last_F = 0;
    ~epp_path() { for (Schedule* s : scheds) delete s; }
};

struct epp_paths {
    int L = 0;
    int64_t n = 0;
    std::vector<DevBuf> bitmaps;    // L+1 bitmaps of N^k, uint64 words
    std::vector<int64_t> set_size;  // |N^k|
    std::vector<epp_path*> path;    // index l
    ~epp_paths() { for (epp_path* p : path) delete p; }
};

// prepare.hip
int epp_path_finish(epp_path* p, hipStream_t s);  // histogram + max length of a built path

// aggregate.hip
int epp_build_schedule(epp_path* p, int gs, hipStream_t s, Schedule** out);
int epp_launch_aggregate(epp_path* p, Schedule* sc, int lanes_hint, const float* in, float* out, int F,
                         hipStream_t s);
int epp_default_group_size(const epp_path* p, int F);
