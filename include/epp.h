/* libepp -- partially-active backward aggregation for GCN training on one MI355X (gfx950).
 *
 * C ABI.  Every pointer marked "device" is GPU global memory owned by the caller unless
 * stated otherwise; "host" pointers are ordinary CPU memory.  All calls are made with the
 * target GPU current.  Functions returning int give 0 on success or a negative EPP_ERR_*
 * code; epp_last_error() then holds a human-readable message for the calling thread.  No
 * function aborts or throws across this boundary.  A handle (epp_paths_t / epp_path_t) must
 * not be used by two calls at the same time (calls on one stream, one after the other, are fine).
 *
 * Environment variables read when a schedule is built (measurement knobs; defaults in brackets):
 *   EPP_TUNE_GS           group size for every (path, F) that has none forced            [selector]
 *   EPP_TUNE_HOT_MB       budget of the hot source rows, 0 switches hot/cold marking off [96]
 *   EPP_TUNE_LOG2_SLICES  log2 of the XCD feature slices, 0..3                           [chosen per path]
 *   EPP_TUNE_SMALL_PREPARE  0: graphs of at most 65,536 vertices and 131,072 entries are prepared by the general
 *                         construction instead of the single-launch one                     [1]
 *   EPP_TUNE_PART         source-partitioned layout: 0 never, 1 where it pays, 2 always  [1]
 *   EPP_TUNE_PART_KB      L2 kilobytes per XCD given to the most referenced source rows  [3584]
 *   EPP_TUNE_PART_MINLEN  shortest row that is cut into per-XCD sections                 [96]
 *   EPP_TUNE_SHARE_PCT    a path runs on the arrays of the next outer path (no entry arrays of its own) if it
 *                         holds at least this percentage of that path's entries; 0: never     [95]
 *   EPP_TUNE_KEEP_CANONICAL  1: a path keeps its canonical entry array beside the source-partitioned
 *                         copy (otherwise it is given back and rebuilt when export or a new width needs it) [0]
 * None of them changes a result beyond the order of floating-point additions.
 *
 * Notation (paper, Table 1 / Sec. 3 / Sec. 4): V_t training set; N^k the k-neighbour set
 * of V_t (vertices reached from V_t by exactly k edges, N^0 = V_t); L layers; SG_l the
 * execution path of layer l with destination vertices N^{L-l} and, for each, the
 * neighbour list filtered by N^{L-l-1}.
 */
#ifndef EPP_H
#define EPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EPP_OK 0
#define EPP_ERR_INVALID_ARG (-1)     /* NULL pointer, L < 1, F < 1, negative size ...       */
#define EPP_ERR_OUT_OF_RANGE_ID (-2) /* a training id outside [0, n)                        */
#define EPP_ERR_TOO_LARGE (-3)       /* n >= 2^29 or nnz >= 2^31                            */
#define EPP_ERR_ALLOC (-4)           /* device or host allocation failed                    */
#define EPP_ERR_HIP (-5)             /* a HIP runtime call failed (message has the detail)  */

typedef void* epp_stream_t; /* a hipStream_t (spelled void* so that this header needs no HIP header);
                               NULL = the default stream */

/* Device-memory allocator of the caller (for instance PyTorch's caching allocator), so that the
 * framework that owns the GPU's memory also owns every byte the library holds: the handle keeps a
 * copy of the struct and takes every device buffer from it, the long-lived ones (path arrays,
 * bitmaps of N^k, group tables, partial rows) and the temporaries of a call, and gives each back
 * through `free` (at the latest when the handle is destroyed).
 *   alloc   returns device memory of at least `bytes` bytes, 256-byte aligned, usable at once on the
 *           stream of the call that asks for it; NULL = failure (the call returns EPP_ERR_ALLOC)
 *   free    takes back a block from `alloc`.  It may be called while work that uses the block is
 *           still queued on the stream of the library call that is freeing it: the allocator must
 *           be stream-ordered on that stream (PyTorch's is, for the stream a block was allocated
 *           on) or wait itself.  epp_destroy_paths / epp_destroy_path take no stream: finish the
 *           work on a handle before destroying it.
 *   ctx     passed through to both.
 * A NULL epp_alloc_t pointer (or alloc == NULL) selects hipMalloc / hipFree. */
typedef struct {
    void* (*alloc)(size_t bytes, void* ctx);
    void (*free)(void* p, void* ctx);
    void* ctx;
} epp_alloc_t;

/* Input graph: pull-mode CSR of the BACKWARD operator M (Alg. 1, backward aggregation
 * loop: X'_v += e_vu * Y'_u for u in N(v)).  Row v lists the sources u with weight e_vu.
 * Columns must be unique within a row (ascending order is what the synthetic inputs use;
 * the library only relies on the order being the caller's canonical one and preserves it).
 * Self-loops are not added: whatever is stored is the operator. */
typedef struct {
    int64_t n;             /* number of vertices, < 2^29                        */
    int64_t nnz;           /* number of stored entries, < 2^31                  */
    const int32_t* rowptr; /* device, n + 1 entries, rowptr[0] = 0              */
    const int32_t* col;    /* device, nnz entries, each in [0, n)               */
    const float* val;      /* device, nnz entries                               */
} epp_csr_t;

typedef struct epp_paths epp_paths_t; /* all L execution paths + the sets N^0..N^L    */
typedef struct epp_path epp_path_t;   /* one execution path (or the all-active graph) */

typedef struct {
    int64_t n;            /* vertices of the input graph (rows of the gradient matrices)    */
    int64_t n_rows;       /* |N^{L-l}|: destination rows of this path                       */
    int64_t nnz;          /* entries kept                                                   */
    int64_t n_src;        /* |N^{L-l-1}|: size of the source set                            */
    int64_t max_len;      /* longest filtered neighbour list                                */
    int64_t len_hist[32]; /* rows per length class c: len <= 1 -> 0, else ceil(log2(len))   */
    int64_t bytes;        /* device bytes held by the path (canonical arrays + schedules,
                             the per-group partial rows of every width used included)     */
    /* schedule most recently used / built (0 if none yet) */
    int32_t sched_F;        /* gradient width it was built for                              */
    int32_t group_size;     /* gs: entries per group (Sec. 2.2, Sec. 5)                     */
    int64_t n_groups;       /* ceil(nnz / gs)                                               */
    int64_t n_split_rows;   /* rows cut by a group boundary (summed from per-group pieces)  */
    /* source-partitioned layout of that width (all 0 if it is not in use): the entries of long rows
       whose source is among the most referenced ones are kept in one section per XCD */
    int64_t part_rows;          /* rows cut into per-section shares                          */
    int64_t part_hot_entries;   /* entries in the eight XCD sections                         */
    int64_t part_partial_rows;  /* partial rows of F floats written and added up per launch  */
    /* 1: the path keeps no entry arrays of its own and runs on those of the next outer path (path
       l - 1), skipping that path's extra entries (Sec. 4: the paths of consecutive layers overlap
       almost entirely once the active sets saturate).  The schedule fields above then describe the
       outer path's tables; `bytes` counts only what this path holds itself. */
    int32_t shares_entries;
} epp_path_info_t;

/* Execution path preparing (Sec. 4): computes N^k for k = 0..L (Theorem 1) by backward
 * frontier expansion from train_ids, and for every layer l the sub-graph SG_l in compact
 * CSR (rows ascending by vertex id, entries in input order, original column ids).
 *   g          host struct with device arrays (read only during the call)
 *   train_ids  device, n_train entries; duplicates allowed (set semantics)
 *   L          number of layers, >= 1
 *   alloc      the caller's device allocator, or NULL (see epp_alloc_t)
 *   stream     work is enqueued here; the call synchronises the stream before returning
 *   out        receives a handle owned by the library; release with epp_destroy_paths
 * Where the active sets are nested (always with self-loops) and the path of layer l holds nearly
 * all entries of the path of layer l - 1, it is stored as a view of that path: see
 * epp_path_info_t.shares_entries.  The exported canonical form is the same either way.
 * n_train = 0 is valid (all paths empty).  Any training id or column id outside [0, n):
 * EPP_ERR_OUT_OF_RANGE_ID; a row pointer that does not rise from 0 to nnz: EPP_ERR_INVALID_ARG
 * (both are checked on the GPU as part of the first pass; neither can make a kernel fault). */
int epp_prepare(const epp_csr_t* g, const int32_t* train_ids, int64_t n_train, int L, const epp_alloc_t* alloc,
                epp_stream_t stream, epp_paths_t** out);

/* The all-active baseline (Alg. 1, backward aggregation over every vertex of the input
 * graph) wrapped as a "path" whose rows are all n vertices, so that the same kernels run
 * it.  Copies what it needs; g may be freed afterwards.  The arrays are checked as in epp_prepare. */
int epp_prepare_full(const epp_csr_t* g, const epp_alloc_t* alloc, epp_stream_t stream, epp_path_t** out);

int epp_num_layers(const epp_paths_t* p);
/* Path of layer l in [0, L) as numbered in Alg. 2 (layer L-1 runs first in an epoch).
 * Borrowed pointer, valid until epp_destroy_paths.  NULL if l is out of range.  (The handle is
 * not const: preparing a width and aggregating over the path change its schedules.) */
epp_path_t* epp_get_path(epp_paths_t* p, int l);

int epp_path_info(const epp_path_t* p, epp_path_info_t* info /* host */);

/* Canonical form of a path into caller buffers (device): row_ids[n_rows], rowptr[n_rows+1],
 * col[nnz], val[nnz]; any of the four may be NULL to skip it.  Synchronises the stream. */
int epp_path_export(const epp_path_t* p, int32_t* row_ids, int32_t* rowptr, int32_t* col, float* val,
                    epp_stream_t stream);

/* N^k (k in [0, L]) as ascending vertex ids.  ids (device, may be NULL to query the size
 * only) must hold *count entries; count (host) receives |N^k|.  Synchronises the stream. */
int epp_active_set_export(const epp_paths_t* p, int k, int32_t* ids, int64_t* count, epp_stream_t stream);

/* Structure-aware group size (Sec. 5, re-derived for 64-lane wavefronts): the number gs of
 * consecutive entries of the path's edge array that form one group (the scheduling unit of
 * Sec. 2.2), as this library picks it for gradient width F.  As in Sec. 5 it is a linear regression
 * on structural features of the sub-graph, fitted on a generated corpus: log2 gs is linear in
 * log2(entries), log2(entries per row) and log2(F), rounded to a power of two in [8, 4096].  The
 * row-length histogram that epp_path_info reports is informational: features taken from it (share
 * of the entries in long rows, entry-weighted mean length, longest row) were fitted too and do not
 * lower the leave-one-graph-out loss.  Pure function of (path, F); returns gs >= 1 or a negative error. */
int epp_select_group_size(const epp_path_t* p, int F);

/* The paper's linear-regression group size (Sec. 5, the regression equation and its four
 * coefficients), provided for comparison only: gs = b0 + b1*#vertices + b2*#edges + b3*avgdeg
 * rounded to the nearest positive integer.  Applied to a (sub-)graph with `vertices` vertices
 * and `undirected_edges` edges, avgdeg = undirected_edges / vertices as in Table 3.  The
 * coefficients were fitted on the paper's GPUs and graphs; far outside that domain the value
 * clamps to 1.  Pure host function. */
int epp_paper_linreg_group_size(int64_t vertices, int64_t undirected_edges);

/* One-off preparation of a path for gradient width F: builds the group table for the group size
 * in force (the selector's, or the one forced by epp_path_set_group_size), allocates the
 * partial rows of the groups (2 * n_groups * F floats, only if some row is cut by a group
 * boundary) and chooses the cache-locality marks of the entries.  Allocates through the handle's
 * allocator and synchronises `stream`; must not be called under stream capture.  Calling it again
 * for a prepared width does nothing.  The aggregate entry points below require it: they never
 * allocate and never wait. */
int epp_path_prepare_width(epp_path_t* p, int F, epp_stream_t stream);

/* Force the group size used for width F (sweeps, ablations); gs <= 0 restores the selector.
 * Rebuilds the group table: group g holds entries [g*gs, (g+1)*gs) of the edge array, so a
 * row longer than gs is always cut and short rows share a group.  Prepares the width as
 * epp_path_prepare_width does (allocates, synchronises).  The partial rows of the previous
 * table are freed: a HIP graph captured with the old table must not be replayed any more.
 * Two paths that share their entries (epp_path_info_t.shares_entries) share their group tables:
 * the size set through either holds for both. */
int epp_path_set_group_size(epp_path_t* p, int F, int gs, epp_stream_t stream);

/* Partially-active backward aggregation of one layer (Alg. 2, aggregation loop):
 *     grad_out[v, :] = sum over entries (u, e_vu) of row v in SG_l of  e_vu * grad_in[u, :]
 * for every destination vertex v of the path.
 *   grad_in, grad_out   device, row-major n x F fp32 (leading dimension F), not aliased
 *   rows of grad_out outside the path are NOT touched (zero them once; the active sets never
 *   change across epochs); rows of grad_in outside the source set are never read.
 * A row whose list is cut by group boundaries is summed from per-group partial rows kept in the
 * handle, in group order and without floating-point atomics: equal inputs give bit-identical
 * results.  The call only enqueues kernels on `stream`: no allocation, no host wait, so it may be
 * captured in a HIP graph.  The width must have been prepared with epp_path_prepare_width
 * (EPP_ERR_INVALID_ARG otherwise). */
int epp_backward_aggregate(epp_path_t* p, const float* grad_in, float* grad_out, int F, epp_stream_t stream);

/* All-active backward aggregation (Alg. 1) over a handle from epp_prepare_full: writes
 * every one of the n rows of grad_out (rows with empty lists become zero).  Enqueues only; the
 * width must have been prepared on `full`. */
int epp_full_aggregate(epp_path_t* full, const float* grad_in, float* grad_out, int F, epp_stream_t stream);

/* If-else selective scheduling (Sec. 4, the first straightforward alternative; comparison
 * baseline of Fig. 6): the all-active kernel on the whole input graph with an "is this vertex
 * active" test on every row (is v in N^{L-l}?) and every neighbour (is u in N^{L-l-1}?), using
 * the membership bitmaps kept in `paths`.  Same result and output contract as
 * epp_backward_aggregate(epp_get_path(paths, l), ...): rows of N^{L-l} are overwritten, all
 * other rows untouched, inactive source rows are never read.  The whole edge array of the
 * graph is still traversed.  Enqueues only; the width must have been prepared on `full`. */
int epp_ifelse_aggregate(epp_path_t* full, const epp_paths_t* paths, int l, const float* grad_in, float* grad_out,
                         int F, epp_stream_t stream);

/* Execution paths prepared earlier and saved by the caller (the paper's pre-processing scenario,
 * Sec. 6: paths are built once per (G, V_t, L) and reused by later training runs).  `layers[l]`
 * holds SG_l in the canonical form that epp_path_export writes; all arrays are device memory and
 * are copied.  The arrays are checked on the GPU before use (row ids ascending and in range, row
 * pointer non-decreasing from 0 to nnz with no empty row, columns in range): a violation gives
 * EPP_ERR_INVALID_ARG or EPP_ERR_OUT_OF_RANGE_ID, never a fault.  That the arrays really are the
 * paths of some graph is the caller's responsibility.  N^0 comes from train_ids as in epp_prepare,
 * N^k (k >= 1) from the row ids of SG_{L-k}.  Synchronises `stream` before returning. */
typedef struct {
    int64_t n_rows;         /* |N^{L-l}|                              */
    int64_t nnz;            /* entries, < 2^31                        */
    const int32_t* row_ids; /* device, n_rows, ascending              */
    const int32_t* rowptr;  /* device, n_rows + 1                     */
    const int32_t* col;     /* device, nnz                            */
    const float* val;       /* device, nnz                            */
} epp_path_arrays_t;
int epp_paths_import(int64_t n, int L, const int32_t* train_ids, int64_t n_train, const epp_path_arrays_t* layers,
                     const epp_alloc_t* alloc, epp_stream_t stream, epp_paths_t** out);

/* Combination stage of the backward pass restricted to the active rows (Alg. 1, backward
 * loop: W'(l) = Y(l)^T (x) X'(l+1) and Y'(l) = X'(l+1) (x) W(l)^T; by Theorem 1 the rows of
 * X'(l+1) outside N^k, k = L-l-1, are zero and add nothing to either product).  Both run on
 * the matrix cores in fp32.
 *   k        which active set holds the non-zero rows of grad_X: 0..L, or -1 for all n rows
 *            (the unrestricted products)
 *   Y        device, n x F_in   forward aggregation result of the layer
 *   grad_X   device, n x F_out  rows outside N^k are never read
 *   W        device, F_in x F_out row-major
 *   grad_W   device, F_in x F_out, overwritten (all zeros when N^k is empty)
 *   grad_Y   device, n x F_in: rows of N^k are overwritten, all others are not touched (they are
 *            the rows that epp_backward_aggregate never reads)
 *   workspace  device scratch of at least epp_weight_gradient_workspace(...) bytes, 16-byte
 *            aligned, owned by the caller; holds partial sums over blocks of rows that a second
 *            kernel adds in a fixed order (results do not depend on timing)
 * 1 <= F_in, F_out <= 4096.  Asynchronous on `stream`: both calls only enqueue kernels (no
 * allocation, no host wait).  Matrices must not alias. */
int64_t epp_weight_gradient_workspace(const epp_paths_t* paths, int k, int F_in, int F_out); /* bytes, < 0: error */
int epp_weight_gradient(epp_paths_t* paths, int k, const float* Y, int F_in, const float* grad_X, int F_out,
                        float* grad_W, void* workspace, int64_t workspace_bytes, epp_stream_t stream);
int epp_input_gradient(epp_paths_t* paths, int k, const float* grad_X, int F_out, const float* W, int F_in,
                       float* grad_Y, epp_stream_t stream);

/* epp_weight_gradient for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and result as epp_weight_gradient (to the same tolerance: the partial sums may be cut
 * at other rows), minus the workspace: the partial sums live in a 32 MiB device array that is part
 * of the library's code object (every GPU the library runs on holds its own copy until the process
 * ends).  The call allocates nothing, on the device or through any library, and only enqueues
 * kernels on `stream`.
 *   limit   F_in * F_out <= 8,388,608 (one block of partial sums must fit the array); beyond it
 *           EPP_ERR_TOO_LARGE, and epp_weight_gradient with a workspace is the way.  Wide matrices
 *           get fewer blocks of rows (32 MiB / (4 F_in F_out)), hence less parallelism.
 *   sharing every call on one GPU uses that GPU's one array: calls that can overlap in time on one
 *           GPU (different streams, different host threads) race on it and must be serialised by
 *           the caller.  Nothing in the array has to be zero; a call writes every word it later reads. */
int epp_weight_gradient_static(epp_paths_t* paths, int k, const float* Y, int F_in, const float* grad_X, int F_out,
                               float* grad_W, epp_stream_t stream);

void epp_destroy_paths(epp_paths_t* p);
void epp_destroy_path(epp_path_t* p); /* only for handles from epp_prepare_full */

const char* epp_last_error(void); /* thread-local, never NULL */

#ifdef __cplusplus
}
#endif
#endif /* EPP_H */
