// C-ABI entry points that tie paths, schedules and kernels together.

#include <cstdarg>
#include <cstring>

#include "epp_internal.h"

namespace {

thread_local char g_err[512] = "";

epp_path::WidthCfg* width_cfg(epp_path* p, int F) {
    for (auto& w : p->widths)
        if (w.F == F) return &w;
    p->widths.push_back(epp_path::WidthCfg{F, 0, nullptr, 0, nullptr});
    return &p->widths.back();
}

Schedule* find_schedule(epp_path* p, int gs) {
    for (Schedule* s : p->scheds)
        if (s->gs == gs) return s;
    return nullptr;
}

// The path whose entry arrays, group tables and per-width choices `p` runs on: itself, or the
// next outer path where the two share their entries.
epp_path* entries_of(epp_path* p) { return p->outer ? p->outer : p; }
const epp_path* entries_of(const epp_path* p) { return p->outer ? p->outer : p; }

// One-off work of a (path, width): group table, partial rows, locality marks.  Allocates and
// waits; the aggregate entry points only look the result up.
int prepare_width(epp_path* self, int F, hipStream_t s, epp_path::WidthCfg** out) {
    epp_path* p = entries_of(self);
    self->last_F = F;
    epp_path::WidthCfg* w = width_cfg(p, F);
    if (!w->sched) {
        EPP_TRY(epp_ensure_canonical(p, s));  // (given back while all widths ran on reconstructed copies)
        const int gs = w->forced_gs > 0 ? w->forced_gs : epp_default_group_size(p, F);
        Schedule* sc = find_schedule(p, gs);
        if (!sc) EPP_TRY(epp_build_schedule(p, gs, s, &sc));
        delete w->part;
        w->part = nullptr;
        EPP_TRY(epp_tune_locality(p, F, gs, s, &w->log2_slices, &w->part));
        // partial rows of the plain group table: not needed where every launch uses the partitioned
        // layout (the all-active handle also serves the if-else baseline, which never does)
        if (!w->part || p->all_rows) EPP_TRY(sc->ensure_pieces(F, epp_alloc_of(p)));
        w->sched = sc;
        EPP_HIP_TRY(hipStreamSynchronize(s));
        epp_release_canonical_if_unused(p);
    }
    p->last_F = F;
    if (out) *out = w;
    return EPP_OK;
}

int check_width(int F) {
    if (F < 1) { epp_set_error("F must be >= 1 (got %d)", F); return EPP_ERR_INVALID_ARG; }
    return EPP_OK;
}

int aggregate(epp_path* self, const float* in, float* out, int F, hipStream_t s, const unsigned int* row_bits = nullptr,
              const unsigned int* src_bits = nullptr) {
    if (!self || !in || !out) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    epp_path* p = entries_of(self);
    EPP_TRY(check_width(F));
    if ((int64_t)p->n * F >= (1ll << 40)) { epp_set_error("gradient matrix too large"); return EPP_ERR_TOO_LARGE; }
    if (in == out) { epp_set_error("grad_in and grad_out must not alias"); return EPP_ERR_INVALID_ARG; }
    const epp_path::WidthCfg* w = nullptr;
    for (const auto& x : p->widths)
        if (x.F == F && x.sched) w = &x;
    if (!w) {
        epp_set_error("width F=%d has not been prepared on this path: call epp_path_prepare_width first", F);
        return EPP_ERR_INVALID_ARG;
    }
    self->last_F = F;
    // (the if-else baseline walks the whole graph in its given order: no partitioned layout)
    return epp_launch_aggregate(p, w->sched, w->log2_slices, in, out, F, s, row_bits, src_bits,
                                row_bits ? nullptr : w->part, self->outer ? self->inner_rows : nullptr);
}

}  // namespace

void epp_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* epp_last_error(void) { return g_err; }

extern "C" int epp_path_info(const epp_path_t* p, epp_path_info_t* info) {
    if (!p || !info) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    std::memset(info, 0, sizeof(*info));
    info->n = p->n;
    info->n_rows = p->n_rows;
    info->nnz = p->nnz;
    info->n_src = p->n_src;
    info->max_len = p->max_len;
    for (int c = 0; c < EPP_NCLASS; ++c) info->len_hist[c] = p->len_hist[c];
    size_t bytes = p->row_ids.bytes + p->rowptr.bytes + p->cv.bytes + p->full_rowptr.bytes + p->empty_rows.bytes;
    bytes += p->zero_block.bytes;
    for (const Schedule* s : p->scheds) bytes += s->bytes();
    for (const auto& w : p->widths)
        if (w.part) bytes += w.part->bytes();
    if (p->pool->accounted_by == p) bytes += p->pool->bytes();  // shared by the handle's paths: reported once
    info->bytes = (int64_t)bytes;
    info->shares_entries = p->outer ? 1 : 0;
    // (a path that runs on the next outer path's arrays reports that path's tables as what it uses;
    // their bytes are part of the outer path's footprint)
    for (const auto& w : entries_of(p)->widths) {
        if (w.F == p->last_F && w.sched) {
            const Schedule* used = w.part ? w.part->sched : w.sched;
            info->sched_F = w.F;
            info->group_size = used->gs;
            info->n_groups = used->n_groups;
            info->n_split_rows = used->n_split_rows;
            if (w.part) {
                info->part_rows = w.part->n_split;
                info->part_hot_entries = w.part->hot_entries;
                info->part_partial_rows = w.part->n_slots;
            }
        }
    }
    return EPP_OK;
}

extern "C" int epp_select_group_size(const epp_path_t* p, int F) {
    if (!p) { epp_set_error("path is NULL"); return EPP_ERR_INVALID_ARG; }
    if (F < 1) { epp_set_error("F must be >= 1"); return EPP_ERR_INVALID_ARG; }
    return epp_default_group_size(entries_of(p), F);  // (groups are cut from the array the path runs on)
}

extern "C" int epp_paper_linreg_group_size(int64_t vertices, int64_t undirected_edges) {
    if (vertices < 1 || undirected_edges < 0) { epp_set_error("bad graph size"); return EPP_ERR_INVALID_ARG; }
    // Sec. 5: least-squares coefficients of the regression equation
    const double b0 = 0.65538, b1 = 1.67431e-5, b2 = -2.24342e-6, b3 = 0.63641;
    const double v = (double)vertices, e = (double)undirected_edges;
    const double x = b0 + b1 * v + b2 * e + b3 * (e / v);
    if (!(x >= 1.0)) return 1;
    if (x > 1e9) return 1000000000;
    return (int)(x + 0.5);
}

extern "C" int epp_path_set_group_size(epp_path_t* self, int F, int gs, epp_stream_t stream) {
    if (!self) { epp_set_error("path is NULL"); return EPP_ERR_INVALID_ARG; }
    if (F < 1) { epp_set_error("F must be >= 1"); return EPP_ERR_INVALID_ARG; }
    epp_path* p = entries_of(self);
    EPP_TRY(epp_ensure_canonical(p, (hipStream_t)stream));  // before the copy it would be rebuilt from goes
    EPP_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    epp_path::WidthCfg* w = width_cfg(p, F);
    w->forced_gs = gs > 0 ? gs : 0;
    if (w->sched) w->sched->drop_pieces(F);  // a table shared with other widths keeps theirs
    w->sched = nullptr;
    delete w->part;
    w->part = nullptr;
    // drop cached tables that no width refers to any more
    for (size_t i = 0; i < p->scheds.size();) {
        bool used = false;
        for (const auto& x : p->widths) used |= (x.sched == p->scheds[i]);
        if (!used) { delete p->scheds[i]; p->scheds.erase(p->scheds.begin() + i); } else ++i;
    }
    return prepare_width(self, F, (hipStream_t)stream, nullptr);
}

extern "C" int epp_path_prepare_width(epp_path_t* p, int F, epp_stream_t stream) {
    if (!p) { epp_set_error("path is NULL"); return EPP_ERR_INVALID_ARG; }
    EPP_TRY(check_width(F));
    if ((int64_t)p->n * F >= (1ll << 40)) { epp_set_error("gradient matrix too large"); return EPP_ERR_TOO_LARGE; }
    return prepare_width(p, F, (hipStream_t)stream, nullptr);
}

extern "C" int epp_backward_aggregate(epp_path_t* p, const float* grad_in, float* grad_out, int F,
                                      epp_stream_t stream) {
    return aggregate(p, grad_in, grad_out, F, (hipStream_t)stream);
}

extern "C" int epp_full_aggregate(epp_path_t* full, const float* grad_in, float* grad_out, int F,
                                  epp_stream_t stream) {
    if (full && !full->all_rows) {
        epp_set_error("epp_full_aggregate needs a handle from epp_prepare_full");
        return EPP_ERR_INVALID_ARG;
    }
    return aggregate(full, grad_in, grad_out, F, (hipStream_t)stream);
}

extern "C" int epp_ifelse_aggregate(epp_path_t* full, const epp_paths_t* paths, int l, const float* grad_in,
                                    float* grad_out, int F, epp_stream_t stream) {
    if (!full || !paths) { epp_set_error("NULL argument"); return EPP_ERR_INVALID_ARG; }
    if (!full->all_rows) { epp_set_error("epp_ifelse_aggregate needs a handle from epp_prepare_full"); return EPP_ERR_INVALID_ARG; }
    if (l < 0 || l >= paths->L) { epp_set_error("no such layer"); return EPP_ERR_INVALID_ARG; }
    if (full->n != paths->n) { epp_set_error("handles belong to different graphs"); return EPP_ERR_INVALID_ARG; }
    const int k = paths->L - 1 - l;  // rows N^{k+1}, sources N^k
    return aggregate(full, grad_in, grad_out, F, (hipStream_t)stream, paths->bitmaps[k + 1].as<unsigned int>(),
                     paths->bitmaps[k].as<unsigned int>());
}
