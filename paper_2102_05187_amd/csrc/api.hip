// C ABI of the library: tensor construction from per-level pos/crd/vals, structure validation,
// schedule building, and dispatch of the five contractions to the HIP kernels.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "kernels.hpp"
#include "stream_kernels.hpp"
#include "tensor.hpp"

using comet::DevRef;
using comet::Format;

#define HIP_TRY(expr)                                              \
    do {                                                           \
        hipError_t e_ = (expr);                                    \
        if (e_ != hipSuccess) { (void)hipGetLastError(); return COMET_ERR_DEVICE; } \
    } while (0)

namespace {

Format classify(int order, const int32_t *lv) {
    if (order == 2) {
        if (lv[0] == COMET_D && lv[1] == COMET_CU) return Format::CSR;
        if (lv[0] == COMET_CU && lv[1] == COMET_CU) return Format::DCSR;
        if (lv[0] == COMET_CN && lv[1] == COMET_S) return Format::COO2;
    } else if (order == 3) {
        if (lv[0] == COMET_CN && lv[1] == COMET_S && lv[2] == COMET_S) return Format::COO3;
        if (lv[0] == COMET_CU && lv[1] == COMET_CU && lv[2] == COMET_CU) return Format::CSF3;
        if (lv[0] == COMET_CU && lv[1] == COMET_CU && lv[2] == COMET_D) return Format::CSF3_DENSE_LEAF;
        if (lv[0] == COMET_CN && lv[1] == COMET_S && lv[2] == COMET_D) return Format::COO3_DENSE_LEAF;
    }
    return Format::OTHER;
}

// number of positions of level l given the number of positions of its parent
int64_t level_positions(const comet_tensor &t, int l, int64_t parent_positions) {
    switch (t.levels[l]) {
    case COMET_D:  return parent_positions * t.dims[l];
    case COMET_CU: return t.crd_len[l];
    case COMET_CN: return t.crd_len[l];
    case COMET_S:  return parent_positions;
    }
    return -1;
}

comet_status read_i32(const int32_t *dev, int n, int32_t *host, hipStream_t st) {
    HIP_TRY(hipMemcpyAsync(host, dev, sizeof(int32_t) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return COMET_OK;
}

// The segments a sweep leaves to the tiled kernel, as a matrix handle of their own over the plan's copy of them
// (row r of the copy writes result row lc.rows[r]; `nrows_total` only bounds those row numbers).
static comet_status make_light_handle(comet_tensor &t, const comet::LightCopy &lc, int64_t nrows_total, int64_t ncols,
                                      hipStream_t st) {
    const int64_t dims2[2] = {nrows_total, ncols};
    const comet_level_t lv[2] = {COMET_CU, COMET_CU};
    const int32_t *pp[2] = {(const int32_t *)lc.root->ptr, (const int32_t *)lc.pos->ptr};
    const int32_t *cc[2] = {(const int32_t *)lc.rows->ptr, (const int32_t *)lc.crd->ptr};
    const int64_t pl[2] = {2, lc.nrows + 1}, cl[2] = {lc.nrows, lc.nnz};
    comet_tensor *lh = nullptr;
    comet_status ls = comet_tensor_create(&lh, 2, dims2, lv, pp, pl, cc, cl, (const double *)lc.vals->ptr, lc.nnz, COMET_LEAN, st);
    if (ls != COMET_OK) return ls;
    t.light.reset(lh);
    return COMET_OK;
}

// Builds the tile tables of the nonzero-tiled kernels for the formats that have them.
comet_status build_schedule(comet_tensor &t, hipStream_t st) {
    comet::Schedule &sc = t.sched;
    const int tile = comet::kTile;
    int leaf = -1;
    if (t.fmt == Format::CSR || t.fmt == Format::DCSR) leaf = 1;
    else if (t.fmt == Format::CSF3) leaf = 2;
    if (leaf >= 0) {
        sc.nnz = t.crd_len[leaf];
        sc.nseg = t.pos_len[leaf] - 1;
        sc.ntiles = (sc.nnz + tile - 1) / tile;
        sc.seg_begin = comet::dev_alloc(sizeof(int32_t) * (sc.ntiles + 1));
        if (!sc.seg_begin) return COMET_ERR_ALLOC;
        HIP_TRY(comet::build_seg_begin(t.pos_i(leaf), sc.nseg, sc.nnz, tile, sc.ntiles,
                                       (int32_t *)sc.seg_begin->ptr, st));
        if (t.fmt == Format::CSF3) {
            sc.slice_begin = comet::dev_alloc(sizeof(int32_t) * (sc.ntiles + 1));
            if (!sc.slice_begin) return COMET_ERR_ALLOC;
            HIP_TRY(comet::build_parent_begin(t.pos_i(1), t.pos_len[1] - 1, (const int32_t *)sc.seg_begin->ptr,
                                              sc.ntiles, (int32_t *)sc.slice_begin->ptr, st));
        }
        DevRef mx = comet::dev_alloc(sizeof(int32_t));
        if (!mx) return COMET_ERR_ALLOC;
        HIP_TRY(hipMemsetAsync(mx->ptr, 0, sizeof(int32_t), st));
        HIP_TRY(comet::max_segment_length(t.pos_i(leaf), sc.nseg, (int32_t *)mx->ptr, st));
        int32_t h = 0;
        comet_status rs = read_i32((const int32_t *)mx->ptr, 1, &h, st);
        if (rs != COMET_OK) return rs;
        sc.max_seg_len = h;
        sc.nchunks = (sc.nnz + comet::kChunk - 1) / comet::kChunk;
        sc.chunk_seg_begin = comet::dev_alloc(sizeof(int32_t) * (sc.nchunks + 1));
        if (!sc.chunk_seg_begin) return COMET_ERR_ALLOC;
        HIP_TRY(comet::build_seg_begin(t.pos_i(leaf), sc.nseg, sc.nnz, comet::kChunk, sc.nchunks,
                                       (int32_t *)sc.chunk_seg_begin->ptr, st));
        HIP_TRY(hipMemsetAsync(mx->ptr, 0, sizeof(int32_t), st));
        HIP_TRY(comet::count_empty_segments(t.pos_i(leaf), sc.nseg, (int32_t *)mx->ptr, st));
        rs = read_i32((const int32_t *)mx->ptr, 1, &h, st);
        if (rs != COMET_OK) return rs;
        sc.empty_segments = h;
        if (t.levels[0] == COMET_CU) {
            HIP_TRY(hipMemsetAsync(mx->ptr, 0, sizeof(int32_t), st));
            HIP_TRY(comet::max_coordinate_gap(t.crd_i(0), t.crd_len[0], t.dims[0], (int32_t *)mx->ptr, st));
            rs = read_i32((const int32_t *)mx->ptr, 1, &h, st);
            if (rs != COMET_OK) return rs;
            sc.max_root_gap = h;
        }
        if ((t.fmt == Format::CSR || t.fmt == Format::DCSR) && !t.lean) {
            // the plans are optional: without the memory for one, the tiled kernel takes everything
            hipError_t pe = comet::heavy_plan_build(t.pos_i(1), sc.nseg, t.crd_i(1), t.vals_d(), sc.nnz, t.dims[1],
                                                    t.fmt == Format::DCSR ? t.crd_i(0) : nullptr, sc.heavy, st);
            if (pe == hipErrorOutOfMemory) { (void)hipGetLastError(); sc.heavy = comet::HeavyPlan(); pe = hipSuccess; }
            HIP_TRY(pe);
            if (sc.heavy.nunits > 0 && sc.heavy.light.nrows > 0 &&
                make_light_handle(t, sc.heavy.light, t.dims[0], t.dims[1], st) != COMET_OK)
                sc.heavy = comet::HeavyPlan();          // no sweep then: the tiled kernel takes every row
        }
        if (t.fmt == Format::CSF3 && !t.lean) {
            hipError_t pe = comet::fiber_plan_build(t.pos_i(2), sc.nseg, t.crd_i(2), t.vals_d(), sc.nnz, t.dims[2], sc.fibers, st);
            if (pe == hipErrorOutOfMemory) { (void)hipGetLastError(); sc.fibers = comet::FiberPlan(); pe = hipSuccess; }
            HIP_TRY(pe);
            if (sc.fibers.nheavy > 0 && make_light_handle(t, sc.fibers.light, sc.nseg, t.dims[2], st) != COMET_OK)
                sc.fibers = comet::FiberPlan();         // no sweep then: the tiled kernel takes every fiber
        }
        if (t.fmt == Format::CSF3) {
            HIP_TRY(hipMemsetAsync(mx->ptr, 0, sizeof(int32_t), st));
            HIP_TRY(comet::max_parent_span(t.pos_i(1), t.pos_len[1] - 1, t.pos_i(2), (int32_t *)mx->ptr, st));
            rs = read_i32((const int32_t *)mx->ptr, 1, &h, st);
            if (rs != COMET_OK) return rs;
            sc.max_parent_len = h;
        }
    } else if (t.fmt == Format::COO3) {
        sc.nnz = t.nvals;
        sc.ntiles = (sc.nnz + tile - 1) / tile;
        sc.run_base = comet::dev_alloc(sizeof(int32_t) * (sc.ntiles + 1));
        if (!sc.run_base) return COMET_ERR_ALLOC;
        HIP_TRY(comet::build_run_base(t.crd_i(0), t.crd_i(1), sc.nnz, tile, sc.ntiles,
                                      (int32_t *)sc.run_base->ptr, st));
        int32_t h = 0;
        comet_status rs = read_i32((const int32_t *)sc.run_base->ptr + sc.ntiles, 1, &h, st);
        if (rs != COMET_OK) return rs;
        sc.nruns = h;
        sc.nseg = h;
        sc.nchunks = (sc.nnz + comet::kChunk - 1) / comet::kChunk;
        sc.chunk_run_base = comet::dev_alloc(sizeof(int32_t) * (sc.nchunks + 1));
        if (!sc.chunk_run_base) return COMET_ERR_ALLOC;
        HIP_TRY(comet::build_run_base(t.crd_i(0), t.crd_i(1), sc.nnz, comet::kChunk, sc.nchunks,
                                      (int32_t *)sc.chunk_run_base->ptr, st));
    }
    HIP_TRY(hipStreamSynchronize(st));
    return COMET_OK;
}

comet_status validate_on_device(const comet_tensor &t, hipStream_t st) {
    DevRef err = comet::dev_alloc(sizeof(int32_t));
    if (!err) return COMET_ERR_ALLOC;
    int32_t *e = (int32_t *)err->ptr;
    HIP_TRY(hipMemsetAsync(e, 0, sizeof(int32_t), st));
    for (int l = 0; l < t.order; ++l) {
        if (t.levels[l] == COMET_CU) {
            HIP_TRY(comet::check_pos(t.pos_i(l), t.pos_len[l], t.crd_len[l], e, st));
            HIP_TRY(comet::check_crd_range(t.crd_i(l), t.crd_len[l], t.dims[l], e, st));
        } else if (t.levels[l] == COMET_CN || t.levels[l] == COMET_S) {
            HIP_TRY(comet::check_crd_range(t.crd_i(l), t.crd_len[l], t.dims[l], e, st));
        }
    }
    int32_t h = 0;
    comet_status rs = read_i32(e, 1, &h, st);
    if (rs != COMET_OK) return rs;
    if (h) return COMET_ERR_BAD_FORMAT;       // order checks below index through pos, so stop here
    for (int l = 0; l < t.order; ++l)
        if (t.levels[l] == COMET_CU)
            HIP_TRY(comet::check_cu_sorted(t.pos_i(l), t.pos_len[l] - 1, t.crd_i(l), t.crd_len[l], e, st));
    if (t.levels[0] == COMET_CN)
        HIP_TRY(comet::check_coo_sorted(t.order, t.crd_i(0), t.crd_i(1), t.order > 2 ? t.crd_i(2) : nullptr,
                                        t.nvals, e, st));
    rs = read_i32(e, 1, &h, st);
    if (rs != COMET_OK) return rs;
    return h ? COMET_ERR_BAD_FORMAT : COMET_OK;
}

// Grow-only: a buffer that is too small is retired (kept alive until the handle is destroyed), never freed
// inside an operation -- earlier work, or a captured graph, may still hold its address.
comet_status ensure_scratch(const comet_tensor *t, size_t bytes) {
    if (t->scratch && t->scratch_bytes >= bytes) return COMET_OK;
    comet::DevRef fresh = comet::dev_alloc(bytes);
    if (!fresh) return COMET_ERR_ALLOC;
    if (t->scratch) t->retired_scratch.push_back(t->scratch);
    t->scratch = fresh;
    t->scratch_bytes = bytes;
    return COMET_OK;
}

// Remember the stream an operation was enqueued on, so that destroy can wait for it.
void note_stream(const comet_tensor *t, hipStream_t st) {
    if (!st) { t->used_null_stream = true; return; }
    for (int q = 0; q < t->n_used_streams && q < 4; ++q)
        if (t->used_streams[q] == (void *)st) return;
    if (t->n_used_streams < 4) t->used_streams[t->n_used_streams] = (void *)st;
    t->n_used_streams += 1;
}

constexpr int64_t kShortSegment = 256;
constexpr int64_t kSmallProblemNnz = int64_t(4) << 20;

// Clearing only the rows between the stored root coordinates beats clearing the whole dense result when
// most rows are stored -- but one thread clears one gap, so a long gap (say, an empty lower half) must
// not be left to it.
bool gaps_are_short(const comet_tensor *t, int64_t R) {
    const int64_t nstored = t->crd_len[0];
    return nstored * 2 >= t->dims[0] && t->sched.max_root_gap >= 0 && t->sched.max_root_gap * R <= 4096;
}

// The tiled kernels read crd / vals with 16-byte vector loads, so the arrays must be 16-byte aligned
// (device allocations are; sub-views handed in by a caller may not be).
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The rank-R tiled kernel addresses operand rows with 32-bit offsets counted in doubles: the operand must
// hold fewer than 2^32 values (32 GiB).  The MTTKRP kernel forms 64-bit addresses and passes dense_rows = 0.
// Small rank-1 problems whose segments are all short go to the group-per-segment kernel when the
// choice is left open: one launch with no tile tables or fix-up pass, which is what matters while the
// whole product takes a few microseconds (measured: 2 us against 12 us at 4096 rows x 10 nonzeros,
// level with the tiled kernel from about 4M nonzeros on, far behind it once one segment is long).
// `serial` = the most nonzeros one thread of the simple kernel would walk alone (longest leaf segment, or
// for MTTKRP the most nonzeros under one slice); 0 = unknown.
bool use_tiled(const comet_tensor *t, int64_t R, const void *dense, const void *result, int64_t dense_rows,
               int64_t serial) {
    if (t->variant == 1) return false;
    if (!comet::stream_supports_rank(R)) return false;
    if (t->variant == 0 && R == 1 && serial > 0 && serial <= kShortSegment && t->sched.nnz <= kSmallProblemNnz)
        return false;
    // The same for rank R: a thread per (segment, column) walks its short segment alone (4 against 17 us at
    // 4096 rows x 10 nonzeros, R = 32; level with the tiled kernel at about 10M multiply-adds).
    if (t->variant == 0 && R > 1 && serial > 0 && serial <= 64 && t->sched.nnz * R <= (int64_t(8) << 20))
        return false;
    // Far more (empty) segments than nonzeros -- a hypersparse matrix kept in CSR: a tile would spend its
    // time clearing the rows of the empty segments it covers; one thread or lane group per row does that evenly.
    if (t->variant == 0 && t->sched.empty_segments > 16 * t->sched.nnz + 4096) return false;
    if (R > 1 && dense_rows * R >= (int64_t(1) << 32) - 4096) return false;
    const int leaf = t->order - 1;
    if (!aligned16(t->crd_i(leaf)) || !aligned16(t->vals_d()) || !aligned16(dense) || !aligned16(result)) return false;
    return true;
}

// A fresh result handle for TTV / TTM on `X`, or the caller's handle if it fits.
comet_status result_handle(const comet_tensor *X, int kind, int64_t R, comet_tensor **Y, bool *fresh) {
    *fresh = false;
    if (*Y) {
        comet_tensor *y = *Y;
        if (y->result_of != X || y->result_kind != kind || y->result_R != R) return COMET_ERR_INVALID_ARG;
        return COMET_OK;
    }
    comet_tensor *y = new (std::nothrow) comet_tensor();
    if (!y) return COMET_ERR_ALLOC;
    y->result_of = X; y->result_kind = kind; y->result_R = R;
    *Y = y;
    *fresh = true;
    return COMET_OK;
}

}  // namespace

extern "C" {

const char *comet_status_string(comet_status s) {
    switch (s) {
    case COMET_OK: return "ok";
    case COMET_ERR_INVALID_ARG: return "invalid argument";
    case COMET_ERR_BAD_FORMAT: return "arrays do not form a valid tensor of the stated level formats";
    case COMET_ERR_SHAPE: return "operand shape mismatch";
    case COMET_ERR_UNSUPPORTED: return "unsupported level tuple, mode or rank";
    case COMET_ERR_ALLOC: return "allocation failed";
    case COMET_ERR_DEVICE: return "HIP call failed";
    }
    return "unknown status";
}

comet_status comet_tensor_create(comet_tensor **out, int order, const int64_t *dims, const comet_level_t *levels,
                                 const int32_t *const *pos, const int64_t *pos_len,
                                 const int32_t *const *crd, const int64_t *crd_len,
                                 const double *vals, int64_t nvals, unsigned flags, void *stream) {
    if (!out) return COMET_ERR_INVALID_ARG;
    *out = nullptr;
    if (!dims || !levels || !pos || !pos_len || !crd || !crd_len) return COMET_ERR_INVALID_ARG;
    if (order < 1 || order > COMET_MAX_ORDER) return COMET_ERR_UNSUPPORTED;
    if (nvals < 0 || nvals >= (int64_t(1) << 31)) return COMET_ERR_INVALID_ARG;
    if (nvals > 0 && !vals) return COMET_ERR_INVALID_ARG;
    if (flags & ~(COMET_COPY | COMET_VALIDATE | COMET_LEAN)) return COMET_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;

    comet_tensor *t = new (std::nothrow) comet_tensor();
    if (!t) return COMET_ERR_ALLOC;
    std::unique_ptr<comet_tensor> guard(t);
    t->order = order;
    t->nvals = nvals;
    t->lean = (flags & COMET_LEAN) != 0;
    for (int l = 0; l < order; ++l) {
        if (dims[l] < 0 || dims[l] >= (int64_t(1) << 31)) return COMET_ERR_INVALID_ARG;
        if ((int)levels[l] < 0 || (int)levels[l] > 3) return COMET_ERR_INVALID_ARG;
        if (pos_len[l] < 0 || crd_len[l] < 0) return COMET_ERR_INVALID_ARG;
        if (pos_len[l] >= (int64_t(1) << 31) || crd_len[l] >= (int64_t(1) << 31)) return COMET_ERR_INVALID_ARG;
        if ((pos_len[l] > 0 && !pos[l]) || (crd_len[l] > 0 && !crd[l])) return COMET_ERR_INVALID_ARG;
        t->dims[l] = dims[l];
        t->levels[l] = (int32_t)levels[l];
        t->pos_len[l] = pos_len[l];
        t->crd_len[l] = crd_len[l];
    }
    t->fmt = classify(order, t->levels);
    if (t->fmt == Format::OTHER) return COMET_ERR_UNSUPPORTED;

    // -- cheap structural checks: array lengths per level, contents of the short pos arrays ------
    int64_t parent = 1;
    for (int l = 0; l < order; ++l) {
        int32_t h[2] = {0, 0};
        switch (t->levels[l]) {
        case COMET_D:
            if (pos_len[l] != 1 || crd_len[l] != 0) return COMET_ERR_BAD_FORMAT;
            { comet_status rs = read_i32(pos[l], 1, h, st); if (rs != COMET_OK) return rs; }
            if ((int64_t)h[0] != dims[l]) return COMET_ERR_BAD_FORMAT;
            break;
        case COMET_CU:
            if (pos_len[l] != parent + 1) return COMET_ERR_BAD_FORMAT;
            if (l == 0) {
                comet_status rs = read_i32(pos[l], 2, h, st); if (rs != COMET_OK) return rs;
                if (h[0] != 0 || (int64_t)h[1] != crd_len[l]) return COMET_ERR_BAD_FORMAT;
            }
            break;
        case COMET_CN:
            if (l != 0 || pos_len[l] != 2) return COMET_ERR_BAD_FORMAT;
            { comet_status rs = read_i32(pos[l], 2, h, st); if (rs != COMET_OK) return rs; }
            if (h[0] != 0 || (int64_t)h[1] != crd_len[l]) return COMET_ERR_BAD_FORMAT;
            break;
        case COMET_S:
            if (l == 0 || pos_len[l] != 0 || crd_len[l] != parent) return COMET_ERR_BAD_FORMAT;
            break;
        }
        parent = level_positions(*t, l, parent);
        if (parent < 0 || parent >= (int64_t(1) << 31)) return COMET_ERR_BAD_FORMAT;
    }
    if (parent != nvals) return COMET_ERR_BAD_FORMAT;

    // -- take (borrow or copy) the arrays -------------------------------------------------------
    auto take = [&](const void *p, size_t bytes, DevRef &dst) -> comet_status {
        if (!p || bytes == 0) { dst = (flags & COMET_COPY) ? comet::dev_alloc(16) : comet::borrow(p, 0); return dst ? COMET_OK : COMET_ERR_ALLOC; }
        if (flags & COMET_COPY) {
            dst = comet::dev_alloc(bytes);
            if (!dst) return COMET_ERR_ALLOC;
            HIP_TRY(hipMemcpyAsync(dst->ptr, p, bytes, hipMemcpyDeviceToDevice, st));
        } else {
            dst = comet::borrow(p, bytes);
        }
        return COMET_OK;
    };
    for (int l = 0; l < order; ++l) {
        comet_status rs;
        if (pos_len[l] > 0) { rs = take(pos[l], sizeof(int32_t) * pos_len[l], t->pos[l]); if (rs != COMET_OK) return rs; }
        if (crd_len[l] > 0 || t->levels[l] != COMET_D) {
            rs = take(crd[l], sizeof(int32_t) * crd_len[l], t->crd[l]); if (rs != COMET_OK) return rs;
        }
    }
    { comet_status rs = take(vals, sizeof(double) * nvals, t->vals); if (rs != COMET_OK) return rs; }

    // The tile tables index through pos, so pos arrays are always checked; the rest on request.
    if (flags & COMET_VALIDATE) {
        comet_status rs = validate_on_device(*t, st);
        if (rs != COMET_OK) return rs;
    } else {
        DevRef err = comet::dev_alloc(sizeof(int32_t));
        if (!err) return COMET_ERR_ALLOC;
        HIP_TRY(hipMemsetAsync(err->ptr, 0, sizeof(int32_t), st));
        for (int l = 0; l < order; ++l)
            if (t->levels[l] == COMET_CU)
                HIP_TRY(comet::check_pos(t->pos_i(l), t->pos_len[l], t->crd_len[l], (int32_t *)err->ptr, st));
        int32_t h = 0;
        comet_status rs = read_i32((const int32_t *)err->ptr, 1, &h, st);
        if (rs != COMET_OK) return rs;
        if (h) return COMET_ERR_BAD_FORMAT;
    }
    comet_status rs = build_schedule(*t, st);
    if (rs != COMET_OK) return rs;
    *out = guard.release();
    return COMET_OK;
}

// Work that uses the handle's arrays may still be in flight: wait for the streams its operations were
// enqueued on (the whole device only if there were more of them than the handle remembers, or the null stream).
comet_status comet_tensor_destroy(comet_tensor *t) {
    if (!t) return COMET_OK;
    if (t->used_null_stream || t->n_used_streams > 4) {
        (void)hipDeviceSynchronize();
    } else {
        for (int q = 0; q < t->n_used_streams; ++q)
            if (hipStreamSynchronize((hipStream_t)t->used_streams[q]) != hipSuccess) { (void)hipGetLastError(); (void)hipDeviceSynchronize(); break; }
    }
    delete t;
    return COMET_OK;
}

static comet_status ensure_shadow(const comet_tensor *X, hipStream_t st);

// Scratch that operations of rank <= R may ask for on this handle.
static size_t scratch_need(const comet_tensor *t, int64_t R) {
    size_t need = 0;
    if (t->sched.nchunks > 0) need = comet::stream_scratch_bytes(t->sched.nchunks, 1);
    if (t->sched.ntiles > 0 && comet::stream_supports_rank(R)) {
        size_t b = comet::stream_scratch_bytes(t->sched.ntiles, R);
        if (t->sched.heavy.nunits > 0) b += comet::heavy_partial_bytes(t->sched.heavy, R > 64 ? 64 : R);
        if (t->sched.fibers.nheavy > 0) b += comet::fiber_partial_bytes(t->sched.fibers, R >= 32 ? 32 : 16);
        if (b > need) need = b;
    }
    return need;
}

comet_status comet_tensor_reserve(comet_tensor *t, int64_t R, void *stream) {
    if (!t || R < 1 || R > 1024) return COMET_ERR_INVALID_ARG;
    const int64_t Rt = R > 128 ? 128 : R;     // ranks above 128 run on kernels that need no scratch
    const comet_tensor *target = t;
    if (t->fmt == Format::COO2 || t->fmt == Format::COO3) {
        comet_status rs = ensure_shadow(t, (hipStream_t)stream);
        if (rs != COMET_OK) return rs;
        target = t->shadow.get();
        if (t->fmt == Format::COO3) {               // TTV runs on the coordinate list itself
            const size_t own = scratch_need(t, 1);
            if (own) { rs = ensure_scratch(t, own); if (rs != COMET_OK) return rs; }
        }
    }
    if (target->light) {                        // the short fibers of a tensor with a heavy-fiber plan run on their own handle
        const size_t own = scratch_need(target->light.get(), Rt);
        if (own) { comet_status rs = ensure_scratch(target->light.get(), own); if (rs != COMET_OK) return rs; }
    }
    const size_t need = scratch_need(target, Rt);
    return need ? ensure_scratch(target, need) : COMET_OK;
}

comet_status comet_tensor_info(const comet_tensor *t, comet_tensor_info_t *info) {
    if (!t || !info) return COMET_ERR_INVALID_ARG;
    std::memset(info, 0, sizeof(*info));
    info->order = t->order;
    for (int l = 0; l < t->order; ++l) {
        info->dims[l] = t->dims[l];
        info->levels[l] = t->levels[l];
        info->mode_of_level[l] = t->mode_of_level[l];
        info->pos[l] = t->pos_len[l] ? t->pos_i(l) : nullptr;
        info->pos_len[l] = t->pos_len[l];
        info->crd[l] = t->crd_len[l] ? t->crd_i(l) : nullptr;
        info->crd_len[l] = t->crd_len[l];
    }
    info->vals = t->nvals ? t->vals_d() : nullptr;
    info->nvals = t->nvals;
    info->heavy_rows = t->sched.heavy.nunits > 0 ? t->sched.heavy.nheavy : t->sched.fibers.nheavy;
    info->heavy_nnz = t->sched.heavy.nunits > 0 ? t->sched.heavy.heavy_nnz : t->sched.fibers.heavy_nnz;
    info->heavy_stream_bytes = t->sched.heavy.nunits > 0
                                   ? t->sched.heavy.stream_items * 16 + (int64_t)t->sched.heavy.light.bytes()
                                   : (int64_t)t->sched.fibers.light.bytes();
    return COMET_OK;
}

comet_status comet_tensor_set_variant(comet_tensor *t, int variant) {
    if (!t || variant < 0 || variant > 3) return COMET_ERR_INVALID_ARG;
    t->variant = variant;
    return COMET_OK;
}

// ---- re-storing with another mode order ----------------------------------------------------------
static int bit_width(int64_t dim) {
    int b = 1;
    while (b < 63 && (int64_t(1) << b) < dim) ++b;
    return b;
}

enum class Target { ALL_CU, CSR, COO };

static comet_status restore(const comet_tensor *X, const int32_t *mode_order, Target target, comet_tensor **out,
                            hipStream_t st) {
    const int order = X->order;
    comet::CoordSource src;
    switch (X->fmt) {
    case Format::CSR:  src.kind = comet::CoordSource::kCsr; break;
    case Format::DCSR: src.kind = comet::CoordSource::kDcsr; break;
    case Format::COO2: case Format::COO3: src.kind = comet::CoordSource::kCoo; break;
    case Format::CSF3: src.kind = comet::CoordSource::kCsf3; break;
    default: return COMET_ERR_UNSUPPORTED;
    }
    src.order = order;
    src.nnz = X->nvals;
    for (int l = 0; l < order; ++l) {
        src.pos[l] = X->pos_i(l); src.npos[l] = (int32_t)X->pos_len[l]; src.crd[l] = X->crd_i(l);
    }
    comet::KeyLayout lay;
    bool used[COMET_MAX_ORDER] = {false, false, false, false};
    int bits[3] = {0, 0, 0}, total_bits = 0;
    for (int l = 0; l < order; ++l) {
        int s = -1;
        for (int q = 0; q < order; ++q) if (X->mode_of_level[q] == mode_order[l]) s = q;
        if (s < 0 || used[s]) return COMET_ERR_INVALID_ARG;     // not a permutation of the modes
        used[s] = true;
        lay.src_level[l] = s;
        bits[l] = bit_width(X->dims[s]);
        total_bits += bits[l];
    }
    // Up to 64 bits the whole coordinate is one sort key; beyond that (three large modes) the root level's
    // coordinate is kept apart and the sort takes two stable passes.
    const bool wide = total_bits > 64;
    for (int l = order - 1, sh = 0; l >= 0; --l) {
        lay.shift[l] = sh;
        lay.mask[l] = bits[l] >= 64 ? ~uint64_t(0) : (uint64_t(1) << bits[l]) - 1;
        sh += bits[l];
    }

    comet_tensor *t = new (std::nothrow) comet_tensor();
    if (!t) return COMET_ERR_ALLOC;
    std::unique_ptr<comet_tensor> guard(t);
    t->order = order;
    t->nvals = X->nvals;
    for (int l = 0; l < order; ++l) {
        t->dims[l] = X->dims[lay.src_level[l]];
        t->levels[l] = COMET_CU;
        t->mode_of_level[l] = mode_order[l];
    }
    t->fmt = classify(order, t->levels);

    const int64_t n = X->nvals;
    int64_t nmid = 0, nroot = 0;        // order 3: #(root,middle) prefixes and #root coordinates; order 2: nroot only
    DevRef keys, rootc, flags, before;
    const uint32_t *rootp = nullptr;    // sorted root coordinates when the key is wide
    if (n > 0) {
        DevRef raw = comet::dev_alloc(sizeof(uint64_t) * n);
        keys = comet::dev_alloc(sizeof(uint64_t) * n);
        t->vals = comet::dev_alloc(sizeof(double) * n);
        flags = comet::dev_alloc(sizeof(uint64_t) * n);
        before = comet::dev_alloc(sizeof(uint64_t) * n);
        DevRef err = comet::dev_alloc(sizeof(int32_t));
        if (!raw || !keys || !t->vals || !flags || !before || !err) return COMET_ERR_ALLOC;
        DevRef temp;
        if (!wide) {
            HIP_TRY(comet::reorder_pack_keys(src, lay, (uint64_t *)raw->ptr, nullptr, st));
            size_t tb = 0;
            HIP_TRY(comet::reorder_sort_pairs(nullptr, &tb, (const uint64_t *)raw->ptr, (uint64_t *)keys->ptr, X->vals_d(),
                                              (double *)t->vals->ptr, n, total_bits, st));
            temp = comet::dev_alloc(tb);
            if (!temp) return COMET_ERR_ALLOC;
            HIP_TRY(comet::reorder_sort_pairs(temp->ptr, &tb, (const uint64_t *)raw->ptr, (uint64_t *)keys->ptr, X->vals_d(),
                                              (double *)t->vals->ptr, n, total_bits, st));
        } else {
            // pass 1: order by (middle, last) carrying the nonzero's number; pass 2: stable order by root
            DevRef root_raw = comet::dev_alloc(sizeof(uint32_t) * n), root_1 = comet::dev_alloc(sizeof(uint32_t) * n);
            DevRef idx_a = comet::dev_alloc(sizeof(uint32_t) * n), idx_b = comet::dev_alloc(sizeof(uint32_t) * n);
            rootc = comet::dev_alloc(sizeof(uint32_t) * n);
            if (!root_raw || !root_1 || !idx_a || !idx_b || !rootc) return COMET_ERR_ALLOC;
            uint64_t *lo_raw = (uint64_t *)raw->ptr, *lo_tmp = (uint64_t *)keys->ptr;
            HIP_TRY(comet::reorder_pack_keys(src, lay, lo_raw, (uint32_t *)root_raw->ptr, st));
            HIP_TRY(comet::reorder_iota((uint32_t *)idx_a->ptr, n, st));
            size_t tb1 = 0, tb2 = 0;
            HIP_TRY(comet::reorder_sort_lo(nullptr, &tb1, lo_raw, lo_tmp, (const uint32_t *)idx_a->ptr, (uint32_t *)idx_b->ptr, n,
                                           bits[1] + bits[2], st));
            HIP_TRY(comet::reorder_sort_hi(nullptr, &tb2, (const uint32_t *)root_1->ptr, (uint32_t *)rootc->ptr,
                                           (const uint32_t *)idx_b->ptr, (uint32_t *)idx_a->ptr, n, bits[0], st));
            temp = comet::dev_alloc(tb1 > tb2 ? tb1 : tb2);
            if (!temp) return COMET_ERR_ALLOC;
            HIP_TRY(comet::reorder_sort_lo(temp->ptr, &tb1, lo_raw, lo_tmp, (const uint32_t *)idx_a->ptr, (uint32_t *)idx_b->ptr, n,
                                           bits[1] + bits[2], st));
            HIP_TRY(comet::reorder_gather_u32((const uint32_t *)root_raw->ptr, (const uint32_t *)idx_b->ptr,
                                              (uint32_t *)root_1->ptr, n, st));
            HIP_TRY(comet::reorder_sort_hi(temp->ptr, &tb2, (const uint32_t *)root_1->ptr, (uint32_t *)rootc->ptr,
                                           (const uint32_t *)idx_b->ptr, (uint32_t *)idx_a->ptr, n, bits[0], st));
            // idx_a = final order; bring the (middle, last) keys and the values into it
            HIP_TRY(comet::reorder_gather_pairs(lo_raw, X->vals_d(), (const uint32_t *)idx_a->ptr, lo_tmp,
                                                (double *)t->vals->ptr, n, st));
            HIP_TRY(hipStreamSynchronize(st));  // the index and root scratch arrays go out of scope here
            rootp = (const uint32_t *)rootc->ptr;
        }
        HIP_TRY(hipMemsetAsync(err->ptr, 0, sizeof(int32_t), st));
        HIP_TRY(comet::reorder_mark_heads((const uint64_t *)keys->ptr, rootp, n, lay, order, (uint64_t *)flags->ptr,
                                          (int32_t *)err->ptr, st));
        size_t sb = 0;
        HIP_TRY(comet::reorder_scan_flags(nullptr, &sb, (const uint64_t *)flags->ptr, (uint64_t *)before->ptr, n, st));
        HIP_TRY(hipStreamSynchronize(st));      // the sort is done with `temp` before it is replaced
        temp = comet::dev_alloc(sb);
        if (!temp) return COMET_ERR_ALLOC;
        HIP_TRY(comet::reorder_scan_flags(temp->ptr, &sb, (const uint64_t *)flags->ptr, (uint64_t *)before->ptr, n, st));
        uint64_t last[2] = {0, 0};
        int32_t dup = 0;
        HIP_TRY(hipMemcpyAsync(&last[0], (const uint64_t *)before->ptr + (n - 1), sizeof(uint64_t), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(&last[1], (const uint64_t *)flags->ptr + (n - 1), sizeof(uint64_t), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(&dup, err->ptr, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (dup) return COMET_ERR_BAD_FORMAT;   // one coordinate stored more than once
        const uint64_t tot = last[0] + last[1];
        if (order == 3) { nmid = (int64_t)(tot & 0xffffffffu); nroot = (int64_t)(tot >> 32); }
        else nroot = (int64_t)(tot & 0xffffffffu);
    } else {
        t->vals = comet::dev_alloc(16);
        if (!t->vals) return COMET_ERR_ALLOC;
    }

    // -- the new levels ---------------------------------------------------------------------------
    comet::CuLevels lv;
    if (target == Target::COO) {
        t->levels[0] = COMET_CN;
        for (int l = 1; l < order; ++l) t->levels[l] = COMET_S;
        t->pos_len[0] = 2;
        t->pos[0] = comet::dev_alloc(2 * sizeof(int32_t));
        if (!t->pos[0]) return COMET_ERR_ALLOC;
        for (int l = 0; l < order; ++l) {
            t->crd_len[l] = n;
            t->crd[l] = comet::dev_alloc(sizeof(int32_t) * n);
            if (!t->crd[l]) return COMET_ERR_ALLOC;
            lv.crd[l] = (int32_t *)t->crd[l]->ptr;
        }
        int32_t h[2] = {0, (int32_t)n};
        HIP_TRY(hipMemcpyAsync(t->pos[0]->ptr, h, sizeof h, hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (n > 0) HIP_TRY(comet::reorder_unpack_keys((const uint64_t *)keys->ptr, rootp, n, lay, order, lv, st));
    } else {
        const int64_t count[3] = {nroot, order == 3 ? nmid : n, n};   // positions per level (order 2 uses [0], [1])
        for (int l = 0; l < order; ++l) {
            const int64_t parents = l == 0 ? 1 : count[l - 1];
            t->pos_len[l] = parents + 1;
            t->crd_len[l] = count[l];
            t->pos[l] = comet::dev_alloc(sizeof(int32_t) * t->pos_len[l]);
            t->crd[l] = comet::dev_alloc(sizeof(int32_t) * t->crd_len[l]);
            if (!t->pos[l] || !t->crd[l]) return COMET_ERR_ALLOC;
            lv.pos[l] = (int32_t *)t->pos[l]->ptr;
            lv.crd[l] = (int32_t *)t->crd[l]->ptr;
        }
        {
            int32_t h[2] = {0, (int32_t)nroot};
            HIP_TRY(hipMemcpyAsync(lv.pos[0], h, sizeof h, hipMemcpyHostToDevice, st));
            HIP_TRY(hipStreamSynchronize(st));
        }
        if (n > 0) {
            HIP_TRY(comet::reorder_cut_levels((const uint64_t *)keys->ptr, rootp, (const uint64_t *)flags->ptr,
                                              (const uint64_t *)before->ptr, n, lay, order, lv, st));
        } else {
            for (int l = 1; l < order; ++l) HIP_TRY(hipMemsetAsync(lv.pos[l], 0, sizeof(int32_t), st));
        }
        if (target == Target::CSR) {
            // dense root: one pos entry per row of the matrix instead of one per stored row
            const int64_t dim0 = t->dims[0];
            DevRef dense = comet::dev_alloc(sizeof(int32_t) * (dim0 + 1));
            DevRef size0 = comet::dev_alloc(sizeof(int32_t));
            if (!dense || !size0) return COMET_ERR_ALLOC;
            HIP_TRY(comet::reorder_dense_pos(lv.crd[0], nroot, lv.pos[1], dim0, n, (int32_t *)dense->ptr, st));
            int32_t h = (int32_t)dim0;
            HIP_TRY(hipMemcpyAsync(size0->ptr, &h, sizeof h, hipMemcpyHostToDevice, st));
            HIP_TRY(hipStreamSynchronize(st));
            t->levels[0] = COMET_D;
            t->pos[0] = size0; t->pos_len[0] = 1;
            t->crd[0].reset(); t->crd_len[0] = 0;
            t->pos[1] = dense; t->pos_len[1] = dim0 + 1;
        }
    }
    t->fmt = classify(order, t->levels);
    t->lean = X->lean;                          // a lean handle's re-stored forms are lean too
    comet_status rs = build_schedule(*t, st);   // synchronises: the temporaries above may go
    if (rs != COMET_OK) return rs;
    *out = guard.release();
    return COMET_OK;
}

comet_status comet_tensor_reorder(const comet_tensor *X, const int32_t *mode_order, comet_tensor **out,
                                  void *stream) {
    if (!out) return COMET_ERR_INVALID_ARG;
    *out = nullptr;
    if (!X || !mode_order) return COMET_ERR_INVALID_ARG;
    return restore(X, mode_order, Target::ALL_CU, out, (hipStream_t)stream);
}

comet_status comet_tensor_convert(const comet_tensor *X, const int32_t *mode_order, const comet_level_t *levels,
                                  comet_tensor **out, void *stream) {
    if (!out) return COMET_ERR_INVALID_ARG;
    *out = nullptr;
    if (!X || !mode_order || !levels) return COMET_ERR_INVALID_ARG;
    int32_t lv[COMET_MAX_ORDER] = {0, 0, 0, 0};
    if (X->order < 2 || X->order > 3) return COMET_ERR_UNSUPPORTED;
    for (int l = 0; l < X->order; ++l) lv[l] = (int32_t)levels[l];
    Target target;
    switch (classify(X->order, lv)) {
    case Format::DCSR: case Format::CSF3: target = Target::ALL_CU; break;
    case Format::CSR: target = Target::CSR; break;
    case Format::COO2: case Format::COO3: target = Target::COO; break;
    default: return COMET_ERR_UNSUPPORTED;
    }
    return restore(X, mode_order, target, out, (hipStream_t)stream);
}

// The compressed copy of a sorted coordinate list (same level order), built on first use.
static comet_status ensure_shadow(const comet_tensor *X, hipStream_t st) {
    if (X->shadow) return COMET_OK;
    comet_tensor *s = nullptr;
    comet_status rs = restore(X, X->mode_of_level, Target::ALL_CU, &s, st);
    if (rs != COMET_OK) return rs;
    s->variant = X->variant;
    X->shadow.reset(s);
    return COMET_OK;
}

// ---- SpMV / SpMM: the last level is compressed; rows come from a dense or compressed root -------
// ext_scratch != nullptr: the caller supplies the carry scratch (ext_bytes of it) and nothing may be allocated.
// ep: what the kernels do with a finished element (off: out = A * Dn; on: out = alpha * A * Dn + beta * out).
static comet_status matrix_product(const comet_tensor *A, const double *Dn, int64_t R, double *out, hipStream_t st,
                                   void *ext_scratch = nullptr, size_t ext_bytes = 0,
                                   comet::Epilogue ep = comet::Epilogue()) {
    if (!A || !Dn || !out) return COMET_ERR_INVALID_ARG;
    note_stream(A, st);
    if (A->fmt == Format::COO2) {
        if (ext_scratch) return COMET_ERR_UNSUPPORTED;      // the compressed copy would have to be allocated
        // a coordinate list [CN,S]: rows come from its compressed ([CU,CU]) copy, built on the first call
        comet_status rs = ensure_shadow(A, st);
        if (rs != COMET_OK) return rs;
        A->shadow->variant = A->variant;
        A = A->shadow.get();
    }
    if (A->fmt != Format::CSR && A->fmt != Format::DCSR) return COMET_ERR_UNSUPPORTED;
    if (R < 1 || R > 1024) return COMET_ERR_UNSUPPORTED;
    const int64_t nseg = A->pos_len[1] - 1, nnz = A->nvals;
    const bool tiled = nnz > 0 && use_tiled(A, R, Dn, out, A->dims[1], A->sched.max_seg_len);
    const size_t carry = tiled ? comet::stream_scratch_bytes(R == 1 ? A->sched.nchunks : A->sched.ntiles, R) : 0;
    // The heavy-row sweep pays when the dense operand is much larger than the L2 caches (else its rows are
    // cache hits anyway) and the long rows hold a good share of the nonzeros (decided when the plan was built).
    const bool heavy = tiled && !ext_scratch && A->variant != 3 && A->sched.heavy.nunits > 0 &&
                       A->dims[1] * R * 8 >= (int64_t(16) << 20) && R <= 64 && comet::heavy_supports(A->sched.heavy, R);
    const size_t need = carry + (heavy ? comet::heavy_partial_bytes(A->sched.heavy, R) : 0);
    if (ext_scratch && need > ext_bytes) return COMET_ERR_UNSUPPORTED;       // before anything is enqueued
    const int32_t *rowmap = nullptr;
    if (A->fmt == Format::DCSR) {
        // Rows absent from the root level hold no nonzeros and must come out as zeros.  Every stored row is
        // written by the kernels below (also one without nonzeros), so when most rows are stored only
        // the gaps between them are cleared; otherwise, or when there is nothing to run, the whole result.
        rowmap = A->crd_i(0);
        const int64_t nstored = A->crd_len[0];
        if (nnz > 0 && gaps_are_short(A, R)) {
            HIP_TRY(comet::zero_unstored_rows(rowmap, nstored, A->dims[0], R, out, st, ep.on ? ep.beta : 0.0));
        } else {
            // every element is cleared (scaled by beta) here, so the kernels add to what they find
            HIP_TRY(comet::scale_f64(out, A->dims[0] * R, ep.on ? ep.beta : 0.0, st));
            if (ep.on && ep.beta != 0.0) ep.beta = 1.0;
        }
    }
    if (nnz == 0) {
        if (A->fmt == Format::CSR) HIP_TRY(comet::scale_f64(out, A->dims[0] * R, ep.on ? ep.beta : 0.0, st));
        return COMET_OK;
    }
    if (tiled) {
        void *scr = ext_scratch;
        if (!ext_scratch) {
            comet_status rs = ensure_scratch(A, need);
            if (rs != COMET_OK) return rs;
            scr = A->scratch->ptr;
        }
        if (heavy) {
            // the long rows from the sweep, all other rows from the tiled kernel run on the plan's copy of them
            // (whose rows carry their result rows, DCSR's included)
            const comet_tensor *Lh = A->light.get();
            if (Lh && Lh->sched.ntiles > 0) {
                comet_status rs = ensure_scratch(Lh, comet::stream_scratch_bytes(Lh->sched.ntiles, R));
                if (rs != COMET_OK) return rs;
                HIP_TRY(comet::stream_segreduce(Lh->sched, Lh->pos_i(1), Lh->crd_i(1), Lh->vals_d(), Lh->crd_i(0), Dn,
                                                A->dims[1], R, out, Lh->scratch->ptr, false, st, ep));
            }
            HIP_TRY(comet::heavy_spmm(A->sched.heavy, rowmap, Dn, R, out, (char *)scr + carry, st, ep));
            return COMET_OK;
        }
        HIP_TRY(comet::stream_segreduce(A->sched, A->pos_i(1), A->crd_i(1), A->vals_d(), rowmap, Dn, A->dims[1], R, out,
                                        scr, A->variant == 3, st, ep));
        return COMET_OK;
    }
    HIP_TRY(comet::simple_segreduce(A->pos_i(1), A->crd_i(1), A->vals_d(), nseg, nnz, rowmap, Dn, R, out, st, ep));
    return COMET_OK;
}

// alpha == 0: the product is not formed at all (the operands may hold anything), the result is beta * out.
static comet::Epilogue make_epilogue(double alpha, double beta) {
    comet::Epilogue ep;
    ep.alpha = alpha; ep.beta = beta; ep.on = 1;
    return ep;
}

comet_status comet_spmv(const comet_tensor *A, const double *x, double *y, void *stream) {
    return matrix_product(A, x, 1, y, (hipStream_t)stream);
}

comet_status comet_spmm(const comet_tensor *A, const double *B, int64_t R, double *C, void *stream) {
    return matrix_product(A, B, R, C, (hipStream_t)stream);
}

comet_status comet_spmv_axpby(const comet_tensor *A, double alpha, const double *x, double beta, double *y, void *stream) {
    if (!A || !y) return COMET_ERR_INVALID_ARG;
    if (alpha == 0.0) {
        if (A->order != 2) return COMET_ERR_UNSUPPORTED;
        note_stream(A, (hipStream_t)stream);
        HIP_TRY(comet::scale_f64(y, A->dims[0], beta, (hipStream_t)stream));
        return COMET_OK;
    }
    return matrix_product(A, x, 1, y, (hipStream_t)stream, nullptr, 0, make_epilogue(alpha, beta));
}

comet_status comet_spmm_axpby(const comet_tensor *A, double alpha, const double *B, int64_t R, double beta, double *C,
                              void *stream) {
    if (!A || !C) return COMET_ERR_INVALID_ARG;
    if (alpha == 0.0) {
        if (A->order != 2 || R < 1 || R > 1024) return COMET_ERR_UNSUPPORTED;
        note_stream(A, (hipStream_t)stream);
        HIP_TRY(comet::scale_f64(C, A->dims[0] * R, beta, (hipStream_t)stream));
        return COMET_OK;
    }
    return matrix_product(A, B, R, C, (hipStream_t)stream, nullptr, 0, make_epilogue(alpha, beta));
}

// ---- SpMV for callers that cannot allocate --------------------------------------------------------
// The carry scratch of the tiled kernels lives in this array instead of in memory owned by the handle.
// Every GPU the library runs on holds its own copy at its own address: host code must go through the
// address that hipGetSymbolAddress returns for the current device, never through the array's name.
static __device__ __align__(256) unsigned char g_static_scratch[COMET_STATIC_SCRATCH_BYTES];

static void *static_scratch_of_current_device(hipError_t *err) {
    static std::mutex mu;
    static void *ptrs[64] = {};
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= 64) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
        if (*err != hipSuccess) return nullptr;
        ptrs[dev] = p;
    }
    return ptrs[dev];
}

comet_status comet_spmv_static(const comet_tensor *A, const double *x, double *y, void *stream) {
    if (!A || !x || !y) return COMET_ERR_INVALID_ARG;
    if (A->fmt != Format::CSR && A->fmt != Format::DCSR) return COMET_ERR_UNSUPPORTED;
    hipError_t e = hipSuccess;
    void *scr = static_scratch_of_current_device(&e);
    if (!scr) { (void)hipGetLastError(); return COMET_ERR_DEVICE; }
    return matrix_product(A, x, 1, y, (hipStream_t)stream, scr, (size_t)COMET_STATIC_SCRATCH_BYTES);
}

// ---- TTV / TTM along the mode stored in the last level ------------------------------------------
static comet_status leaf_contract(const comet_tensor *X, int mode, const double *Dn, int64_t R, int kind,
                                  comet_tensor **Y, hipStream_t st) {
    if (!X || !Dn || !Y) return COMET_ERR_INVALID_ARG;
    note_stream(X, st);
    if (X->order != 3) return COMET_ERR_UNSUPPORTED;
    if (R < 1 || R > 1024) return COMET_ERR_UNSUPPORTED;
    const bool csf = X->fmt == Format::CSF3, coo = X->fmt == Format::COO3;
    if (!csf && !coo) return COMET_ERR_UNSUPPORTED;
    if (mode < 0 || mode >= 3) return COMET_ERR_INVALID_ARG;
    if (mode != X->mode_of_level[2]) return COMET_ERR_UNSUPPORTED;   // re-store with comet_tensor_reorder first
    bool fresh = false;
    comet_status rs = result_handle(X, kind, R, Y, &fresh);
    if (rs != COMET_OK) return rs;
    comet_tensor *y = *Y;
    std::unique_ptr<comet_tensor> guard(fresh ? y : nullptr);
    if (fresh) *Y = nullptr;
    // TTM on a coordinate list runs on its compressed copy; the result lists the distinct (i,j) like TTV's
    const comet_tensor *S = nullptr;
    if (coo && kind == 2) {
        rs = ensure_shadow(X, st);
        if (rs != COMET_OK) return rs;
        S = X->shadow.get();
        X->shadow->variant = X->variant;                          // the kernel family chosen for X applies to its copy
    }
    const int64_t nout = csf ? X->crd_len[1] : (S ? S->crd_len[1] : X->sched.nruns);    // stored (i,j) pairs
    if (fresh) {
        y->order = kind == 1 ? 2 : 3;
        y->dims[0] = X->dims[0]; y->dims[1] = X->dims[1];
        for (int l = 0; l < 3; ++l) y->mode_of_level[l] = X->mode_of_level[l];
        if (csf) {
            y->levels[0] = COMET_CU; y->levels[1] = COMET_CU;
            for (int l = 0; l < 2; ++l) {
                y->pos[l] = X->pos[l]; y->crd[l] = X->crd[l];
                y->pos_len[l] = X->pos_len[l]; y->crd_len[l] = X->crd_len[l];
            }
        } else {
            y->levels[0] = COMET_CN; y->levels[1] = COMET_S;
            y->pos[0] = comet::dev_alloc(2 * sizeof(int32_t));
            y->crd[0] = comet::dev_alloc(sizeof(int32_t) * nout);
            y->crd[1] = S ? S->crd[1] : comet::dev_alloc(sizeof(int32_t) * nout);   // the copy's fiber coordinates as they are
            if (!y->pos[0] || !y->crd[0] || !y->crd[1]) return COMET_ERR_ALLOC;
            if (S) HIP_TRY(comet::expand_parent_coords(S->pos_i(1), S->crd_len[0], S->crd_i(0), nout, (int32_t *)y->crd[0]->ptr, st));
            int32_t h[2] = {0, (int32_t)nout};
            HIP_TRY(hipMemcpyAsync(y->pos[0]->ptr, h, sizeof h, hipMemcpyHostToDevice, st));
            HIP_TRY(hipStreamSynchronize(st));
            y->pos_len[0] = 2; y->crd_len[0] = nout; y->crd_len[1] = nout;
        }
        if (kind == 2) {
            y->dims[2] = R; y->levels[2] = COMET_D;
            y->pos[2] = comet::dev_alloc(sizeof(int32_t));
            if (!y->pos[2]) return COMET_ERR_ALLOC;
            int32_t h = (int32_t)R;
            HIP_TRY(hipMemcpyAsync(y->pos[2]->ptr, &h, sizeof h, hipMemcpyHostToDevice, st));
            HIP_TRY(hipStreamSynchronize(st));
            y->pos_len[2] = 1;
        }
        // positions of a dense last level are never stored in an int32 array, so only the values of a
        // level that some pos array indexes are limited to 2^31; the TTM result may be larger
        y->nvals = nout * R;
        y->vals = comet::dev_alloc(sizeof(double) * y->nvals);
        if (!y->vals) return COMET_ERR_ALLOC;
        y->fmt = classify(y->order, y->levels);
    }
    double *yv = (double *)y->vals->ptr;
    if (X->nvals > 0) {
        if (csf || S) {
            const comet_tensor *C = csf ? X : S;                 // the compressed storage the kernels walk
            if (use_tiled(C, R, Dn, yv, C->dims[2], C->sched.max_seg_len)) {
                // long fibers over a small last mode: their rows come from the heavy-fiber sweep (operand rows in
                // LDS), all other fibers from the tiled kernel run on the compacted copy of them
                const comet_tensor *Lh = C->light.get();
                const bool sweep = kind == 2 && C->variant != 3 && Lh && comet::fiber_supports(C->sched.fibers, R) &&
                                   Lh->sched.ntiles > 0 && aligned16(Lh->crd_i(1)) && aligned16(Lh->vals_d());
                if (sweep) {
                    rs = ensure_scratch(Lh, comet::stream_scratch_bytes(Lh->sched.ntiles, R));
                    if (rs != COMET_OK) return rs;
                    rs = ensure_scratch(C, comet::fiber_partial_bytes(C->sched.fibers, R));
                    if (rs != COMET_OK) return rs;
                    HIP_TRY(comet::stream_segreduce(Lh->sched, Lh->pos_i(1), Lh->crd_i(1), Lh->vals_d(), Lh->crd_i(0), Dn,
                                                    C->dims[2], R, yv, Lh->scratch->ptr, false, st));
                    HIP_TRY(comet::fiber_ttm(C->sched.fibers, C->crd_i(2), C->vals_d(), Dn, C->dims[2], R, yv,
                                             C->scratch->ptr, st));
                } else {
                    rs = ensure_scratch(C, comet::stream_scratch_bytes(R == 1 ? C->sched.nchunks : C->sched.ntiles, R));
                    if (rs != COMET_OK) return rs;
                    HIP_TRY(comet::stream_segreduce(C->sched, C->pos_i(2), C->crd_i(2), C->vals_d(), nullptr, Dn, C->dims[2], R,
                                                    yv, C->scratch->ptr, C->variant == 3, st));
                }
            } else {
                HIP_TRY(comet::simple_segreduce(C->pos_i(2), C->crd_i(2), C->vals_d(), C->pos_len[2] - 1, C->nvals,
                                                nullptr, Dn, R, yv, st));
            }
        } else {
            if (use_tiled(X, 1, Dn, yv, 0, 0) && comet::stream_supports_coo()) {
                rs = ensure_scratch(X, comet::stream_scratch_bytes(X->sched.nchunks, 1));
                if (rs != COMET_OK) return rs;
                HIP_TRY(comet::stream_ttv_coo(X->sched, X->crd_i(0), X->crd_i(1), X->crd_i(2), X->vals_d(), Dn, X->dims[2],
                                              (int32_t *)y->crd[0]->ptr, (int32_t *)y->crd[1]->ptr, yv,
                                              X->scratch->ptr, X->variant == 3, st));
            } else {
                HIP_TRY(comet::simple_ttv_coo(X->crd_i(0), X->crd_i(1), X->crd_i(2), X->vals_d(), X->nvals, comet::kTile,
                                              X->sched.ntiles, (const int32_t *)X->sched.run_base->ptr, Dn,
                                              (int32_t *)y->crd[0]->ptr, (int32_t *)y->crd[1]->ptr, yv, st));
            }
        }
    } else if (y->nvals > 0) {
        HIP_TRY(comet::fill_zero_f64(yv, y->nvals, st));   // stored fibers that hold no nonzero
    }
    if (fresh) *Y = guard.release();
    return COMET_OK;
}

comet_status comet_ttv(const comet_tensor *X, int mode, const double *v, comet_tensor **Y, void *stream) {
    return leaf_contract(X, mode, v, 1, 1, Y, (hipStream_t)stream);
}

comet_status comet_ttm(const comet_tensor *X, int mode, const double *U, int64_t R, comet_tensor **Y, void *stream) {
    return leaf_contract(X, mode, U, R, 2, Y, (hipStream_t)stream);
}

static comet_status mttkrp_impl(const comet_tensor *X, int mode, const double *const *factors, int64_t R, double *M,
                                void *stream, comet::Epilogue ep) {
    if (!X || !factors || !M) return COMET_ERR_INVALID_ARG;
    note_stream(X, (hipStream_t)stream);
    if (X->fmt == Format::COO3) {
        // a sorted coordinate list: the slice / fiber structure comes from its compressed copy
        comet_status rs = ensure_shadow(X, (hipStream_t)stream);
        if (rs != COMET_OK) return rs;
        X->shadow->variant = X->variant;
        X = X->shadow.get();
    }
    if (X->fmt != Format::CSF3) return COMET_ERR_UNSUPPORTED;
    if (mode < 0 || mode >= 3) return COMET_ERR_INVALID_ARG;
    if (mode != X->mode_of_level[0]) return COMET_ERR_UNSUPPORTED;   // re-store with comet_tensor_reorder first
    if (R < 1 || R > 1024) return COMET_ERR_UNSUPPORTED;
    // B belongs to the mode of the middle level, C to the mode of the last level
    const double *B = factors[X->mode_of_level[1]], *C = factors[X->mode_of_level[2]];
    if (!B || !C) return COMET_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int64_t nslice = X->pos_len[1] - 1;
    const bool tiled = X->nvals > 0 &&
                       use_tiled(X, R, B, M, 0, X->sched.max_parent_len) && aligned16(C) &&
                       comet::stream_mttkrp_supports_rank(R);
    // Rows of M whose index is not stored at the root level receive no contribution.  The tiled kernel
    // writes every stored slice's row itself (a slice without nonzeros is cleared in its slice pass), so
    // when most rows are stored only the gaps between them are cleared; otherwise all of M is.
    if (tiled && gaps_are_short(X, R)) {
        HIP_TRY(comet::zero_unstored_rows(X->crd_i(0), nslice, X->dims[0], R, M, st, ep.on ? ep.beta : 0.0));
    } else {
        // every element is cleared (scaled by beta) here, so the kernels add to what they find
        HIP_TRY(comet::scale_f64(M, X->dims[0] * R, ep.on ? ep.beta : 0.0, st));
        if (ep.on && ep.beta != 0.0) ep.beta = 1.0;
    }
    if (X->nvals == 0) return COMET_OK;
    if (tiled) {
        comet_status rs = ensure_scratch(X, comet::stream_scratch_bytes(X->sched.ntiles, R));
        if (rs != COMET_OK) return rs;
        HIP_TRY(comet::stream_mttkrp(X->sched, X->pos_i(1), X->crd_i(0), nslice, X->pos_i(2), X->crd_i(1),
                                     X->crd_i(2), X->vals_d(), B, C, R, M, X->scratch->ptr, st, ep));
        return COMET_OK;
    }
    HIP_TRY(comet::simple_mttkrp(X->pos_i(1), X->crd_i(0), X->pos_len[1] - 1, X->pos_i(2), X->crd_i(1), X->crd_i(2),
                                 X->vals_d(), B, C, R, M, st, ep));
    return COMET_OK;
}

comet_status comet_mttkrp(const comet_tensor *X, int mode, const double *const *factors, int64_t R, double *M,
                          void *stream) {
    return mttkrp_impl(X, mode, factors, R, M, stream, comet::Epilogue());
}

comet_status comet_mttkrp_axpby(const comet_tensor *X, int mode, double alpha, const double *const *factors, int64_t R,
                                double beta, double *M, void *stream) {
    if (!X || !M) return COMET_ERR_INVALID_ARG;
    if (alpha == 0.0) {
        if (X->order != 3 || mode != X->mode_of_level[0] || R < 1 || R > 1024) return COMET_ERR_UNSUPPORTED;
        note_stream(X, (hipStream_t)stream);
        HIP_TRY(comet::scale_f64(M, X->dims[0] * R, beta, (hipStream_t)stream));
        return COMET_OK;
    }
    return mttkrp_impl(X, mode, factors, R, M, stream, make_epilogue(alpha, beta));
}

}  // extern "C"
