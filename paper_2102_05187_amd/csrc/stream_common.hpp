// Shared device helpers of the nonzero-tiled streaming kernels (included by kernels_rank1.hip,
// kernels_rankR.hip and kernels_mttkrp.hip; everything here has internal linkage).
// Nonzero-tiled streaming kernels for gfx950 (wave64).
//
// Work is cut by nonzeros, not by rows: tile t owns leaf positions [t*kTile, (t+1)*kTile), whatever
// segments (rows / fibers / slices) they belong to, so a power-law head segment is spread over many
// workgroups -- load imbalance across rows is what the paper names as the main source of slowdown
// (Section 8.3).  The per-level access rule is the compressed-unique one of Table "Generated code to
// access nonzeros coordinates" (segment s owns positions pos[s]..pos[s+1]-1, coordinate crd[p], value
// vals[p]); sorted coordinate lists use the compressed-nonunique / singleton rule (one coordinate per
// position, a segment = a run of equal leading coordinates).
//
// Segment ends are marked in LDS (a map ts[i] = id of the segment whose LAST nonzero is tile item i,
// else -1; or a bit mask when ids can be counted).  A unit of work (lane or lane group, wavefront,
// tile) summarises its item range as
//     has_tail    a segment ends inside the range
//     first       sum of the items up to and including the first segment end   (+ its segment id)
//     open        sum of the items after the last segment end (all items if there is none)
// and two adjacent summaries combine associatively; a segment that closes at the boundary of two
// units is final once the left unit contains a segment end.  Tile summaries go to a carry buffer
// and small follow-up kernels finish the segments cut by tile boundaries in a fixed order, so the
// results do not depend on scheduling (no atomics).
//
// Kernels:  k_stream_rank1_ldsvec  rank 1, dense vector staged in LDS, one wavefront per 1024-item chunk
//           k_stream_rank1[_coo]   rank 1, vector gathered through L1, tail-id map per 4096-item tile
//           k_stream_rankR         rank R, lane groups walk item runs, per-item records in LDS
//           k_stream_mttkrp        rank R, two nested segment levels (fibers inside slices)
//           k_fixup_level / k_stream_fixup   carry resolution
#pragma once

#include "kernels.hpp"
#include "stream_kernels.hpp"

namespace comet {

// Finishes every segment that a tile boundary cut (defined in kernels_rank1.hip).
hipError_t run_fixup(void *scratch, int64_t ntiles, int R, const int32_t *rowmap, double *out, int64_t max_chain,
                     hipStream_t st, Epilogue ep = Epilogue());
// Rank-R part of stream_segreduce (defined in kernels_rankR.hip).
hipError_t stream_segreduce_rankR(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                                  const int32_t *rowmap, const double *Dn, int R, double *out, void *scratch,
                                  hipStream_t st, Epilogue ep = Epilogue());

namespace {

// Carry-buffer layout inside the per-tensor scratch.  Level 0 holds one summary per tile: first[R],
// open[R] (fp64), has_tail and first_id (int32).  Level l+1 holds one summary per group of
// kFixGroup consecutive level-l summaries (same layout), so that a segment cut over thousands of
// tiles is finished in a few short passes instead of one long serial walk.
constexpr int kFixGroup = 64;
struct CarryView {
    double  *first, *open;
    int32_t *has_tail, *first_id;
};
__host__ __device__ inline size_t carry_level_bytes(int64_t n, int64_t R) {
    size_t b = (size_t)n * (size_t)R * 2 * sizeof(double) + (size_t)n * 2 * sizeof(int32_t);
    return (b + 255) & ~(size_t)255;
}
__host__ __device__ inline CarryView carry_view(void *scratch, int64_t n, int64_t R) {
    CarryView c;
    c.first = (double *)scratch;
    c.open = c.first + n * R;
    c.has_tail = (int32_t *)(c.open + n * R);
    c.first_id = c.has_tail + n;
    return c;
}

// ---- phase A/B for compressed levels: fill the tail map from pos, zero-fill empty segments -------
// Segments [seg_begin[t], seg_begin[t+1]) end inside tile t (the segment that contains the first
// item of the next tile ends later), so each of them owns exactly one map entry.
// rows_in_map: the entry of a segment end is the segment's result row rowmap[s] instead of s (looked up here by
// all threads at once, so that the walk has no dependent load at a segment end); ids are opaque to the fix-up.
__device__ __forceinline__ void build_tail_map_from_pos(int32_t *ts, const int32_t *__restrict__ pos,
                                                        const int32_t *__restrict__ rowmap, int64_t tb, int32_t s0,
                                                        int32_t s1, double *__restrict__ out, int R,
                                                        bool rows_in_map = false, const Epilogue ep = Epilogue()) {
    for (int i = threadIdx.x * 4; i < kTile; i += blockDim.x * 4)
        *reinterpret_cast<int4 *>(ts + i) = make_int4(-1, -1, -1, -1);
    __syncthreads();
    for (int32_t s = s0 + threadIdx.x; s < s1; s += blockDim.x) {
        int32_t b = pos[s], e = pos[s + 1];
        if (e > b) {
            ts[(int64_t)e - 1 - tb] = rows_in_map ? rowmap[s] : s;
        } else {
            int64_t row = rowmap ? (int64_t)rowmap[s] : (int64_t)s;
            for (int r = 0; r < R; ++r) out[row * R + r] = ep_empty(ep, out + row * R + r);
        }
    }
    __syncthreads();
}

// Cross-lane broadcast inside a lane group (quad_perm inside a quad, plus one row_shr:4 / row_shl:4 with a
// bank mask to cross the two quads of an 8-lane group); used where LDS bandwidth or space is better
// spent on operand rows than on per-item records.
template <int L, int BP>
__device__ __forceinline__ int grp_bcast_i(int v) {
    static_assert(L == 4 || L == 8, "lane groups of 4 or 8");
    // quad_perm broadcast; every lane is written, and bound_ctrl with full masks tells the compiler so
    // (no move of the unused old value in front of it)
    const int x1 = __builtin_amdgcn_update_dpp(0, v, (BP % 4) * 0x55, 0xf, 0xf, true);
    if constexpr (L == 4) return x1;
    else if constexpr (BP < 4) return __builtin_amdgcn_update_dpp(x1, x1, 0x114, 0xf, 0xa, false);   // row_shr:4 into the odd quads
    else return __builtin_amdgcn_update_dpp(x1, x1, 0x104, 0xf, 0x5, false);                          // row_shl:4 into the even quads
}
template <int L, int BP>
__device__ __forceinline__ double grp_bcast_d(double v) {
    return __hiloint2double(grp_bcast_i<L, BP>(__double2hiint(v)), grp_bcast_i<L, BP>(__double2loint(v)));
}

// ---- rank-R walk: a group of L lanes (4 or 8) walks a run of consecutive items --------------------
// The 256 threads of a tile form 256/L lane groups ("walkers"); walker g owns the 16*L consecutive
// items [tb + 16*L*g, +16*L).  Every 4*L items (a super-block) each lane loads four consecutive
// (crd, val) pairs with 16-byte loads, looks up their tail ids, turns crd into the offset of
// the operand row, and writes one small record per item into the walker's private LDS area.  The
// group then takes the items one at a time: every lane reads the current item's record with a
// broadcast LDS read (no cross-lane VALU work), adds its own 16-byte slot, and gathers its share of
// the operand row Dn[crd, :] -- contiguous 16-byte pieces (WIDE, R a multiple of 2L: lane j takes
// ranks 2L*q+2j, 2L*q+2j+1) or 8-byte pieces (lane j takes ranks L*q+j) -- so a load instruction
// reads each gathered row as one contiguous run of 16*L bytes.  Gathers run G steps ahead of the
// FMAs (double-buffered in registers).  Row offsets are 32-bit counts of doubles, so an operand must hold fewer than 2^32 values.
template <int L, int NI>
struct RecLayout {                                     // per-walker record area, in 4-byte words
    static constexpr int SB = 4 * L;                   // items per super-block
    static constexpr int kVal = NI * SB;               // values start after the integer records
    static constexpr int kStride = NI * SB + 2 * SB + 4;   // + 16 bytes so that walkers start on different banks
};

// This lane's share of a dense row: V values.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_load_row(const double *__restrict__ Dn, int64_t row, int R, int j, double *d) {
    const double *rowp = Dn + row * R;
    if constexpr (WIDE) {
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            const double2 x = *reinterpret_cast<const double2 *>(rowp + 2 * L * q + 2 * j);
            d[2 * q] = x.x; d[2 * q + 1] = x.y;
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) { int r = L * q + j; d[q] = r < R ? rowp[r] : 0.0; }
    }
}
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_store_row(double *__restrict__ out, int64_t row, int R, int j, const double *v,
                                              const Epilogue ep = Epilogue()) {
    double *p = out + row * R;
    if constexpr (WIDE) {
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            double *d = p + 2 * L * q + 2 * j;
            *reinterpret_cast<double2 *>(d) = make_double2(ep_apply(ep, v[2 * q], d), ep_apply(ep, v[2 * q + 1], d + 1));
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) { int r = L * q + j; if (r < R) p[r] = ep_apply(ep, v[q], p + r); }
    }
}

// The same for a result row that this kernel does not read again: non-temporal stores.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_store_row_stream(double *__restrict__ out, int64_t row, int R, int j, const double *v,
                                                     const Epilogue ep = Epilogue()) {
    double *p = out + row * R;
    if constexpr (WIDE) {
        typedef double v2d __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            double *d = p + 2 * L * q + 2 * j;
            v2d x; x.x = ep_apply(ep, v[2 * q], d); x.y = ep_apply(ep, v[2 * q + 1], d + 1);
            __builtin_nontemporal_store(x, reinterpret_cast<v2d *>(d));
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) { int r = L * q + j; if (r < R) __builtin_nontemporal_store(ep_apply(ep, v[q], p + r), p + r); }
    }
}

// compile-time loop: f(IntC<B>{}), ..., f(IntC<E-1>{})
template <int N> struct IntC { static constexpr int value = N; };
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (B < E) { f(IntC<B>{}); static_for<B + 1, E>(f); }
}

// Four consecutive items of one lane: the streamed part of a 4*L-item super-block.
struct LaneItems {
    int    cr[4];
    double va[4];
};
__device__ __forceinline__ void lane_load_items(LaneItems &it, const int32_t *__restrict__ crd,
                                                const double *__restrict__ vals, int64_t i0, int64_t nnz) {
    if (i0 + 3 < nnz) {
        // streamed once: non-temporal, so the caches keep the operand rows rather than the nonzeros
        typedef int v4i __attribute__((ext_vector_type(4)));
        typedef double v2d __attribute__((ext_vector_type(2)));
        const v4i c4 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(crd + i0));
        const v2d a01 = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(vals + i0));
        const v2d a23 = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(vals + i0 + 2));
        it.cr[0] = c4.x; it.cr[1] = c4.y; it.cr[2] = c4.z; it.cr[3] = c4.w;
        it.va[0] = a01.x; it.va[1] = a01.y; it.va[2] = a23.x; it.va[3] = a23.y;
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) { bool in = i0 + s < nnz; it.cr[s] = in ? crd[i0 + s] : 0; it.va[s] = in ? vals[i0 + s] : 0.0; }
    }
}

template <int V> struct RowBuf { double d[V]; int tail; double a; int boff, mrow; };

// Steps per pipeline group: the gathers of group g+1 are in flight while group g is consumed.
template <int V> struct StepGroup { static constexpr int value = V <= 4 ? 4 : (V <= 8 ? 2 : 1); };

template <int V>
struct WalkState {
    double acc[V];
    double first[V];
    int ht, first_id;
};

// This lane's share of the dense row that starts `off` doubles into Dn (off already includes the
// lane's own slot).  Offsets are 32-bit counts of doubles, so an operand may hold up to 2^32 values
// (32 GiB); the sum with the q-th piece is formed in 64 bits.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_load_row_off(const double *__restrict__ Dn, unsigned off, int R, int j, double *d) {
    const double *base = Dn + (size_t)off;
    if constexpr (WIDE) {
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            const double2 x = *reinterpret_cast<const double2 *>(base + 2 * L * q);
            d[2 * q] = x.x; d[2 * q + 1] = x.y;
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) d[q] = L * q + j < R ? base[L * q] : 0.0;
    }
}
template <int L, bool WIDE>
__device__ __forceinline__ unsigned lane_slot_doubles(int j) { return WIDE ? 2u * j : (unsigned)j; }

// Close the first segment end of every walker of the tile and publish the tile summary.
// wopen[(g*L + j)*V + q] holds walker g's open sum, wht[g] its has_tail flag (both already written
// and separated from this call by a barrier).  `first_row` is the output row of the walker's first
// segment end; `open` its trailing sum.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void finish_tile_walkers(const double *wopen, const int *wht, int g, int j, int ht,
                                                    const double *first, int64_t first_row, int32_t first_id,
                                                    const double *open, double *__restrict__ out, int R,
                                                    CarryView cb, int64_t t, const Epilogue ep = Epilogue()) {
    constexpr int NW = 256 / L;
    const bool last = g == NW - 1;
    if (!(ht || last)) return;
    double sum[V];
#pragma unroll
    for (int q = 0; q < V; ++q) sum[q] = 0.0;
    int found = 0;
    for (int g2 = g - 1; g2 >= 0; --g2) {
        const double *wo = wopen + (g2 * L + j) * V;
#pragma unroll
        for (int q = 0; q < V; ++q) sum[q] += wo[q];
        if (wht[g2]) { found = 1; break; }
    }
    if (ht) {
        double value[V];
#pragma unroll
        for (int q = 0; q < V; ++q) value[q] = sum[q] + first[q];
        if (found) {
            grp_store_row<L, V, WIDE>(out, first_row, R, j, value, ep);
        } else {                                              // first segment end of the whole tile
            grp_store_row<L, V, WIDE>(cb.first, t, R, j, value);
            if (j == 0) cb.first_id[t] = first_id;
        }
    }
    if (last) {
        double topen[V];
#pragma unroll
        for (int q = 0; q < V; ++q) topen[q] = ht ? open[q] : open[q] + sum[q];
        grp_store_row<L, V, WIDE>(cb.open, t, R, j, topen);
        if (j == 0) cb.has_tail[t] = ht | found;
    }
}

}  // namespace

// Lane-group width of the rank-R kernels: 8 lanes, quads for ranks up to 8.
inline int lanes_per_item(int64_t R) { return R <= 8 ? 4 : 8; }

// Calls F<L, V, WIDE>(args...) for the specialisation that covers rank R.
#define COMET_DISPATCH_RANK(F, R, ...)                                                     \
    [&]() -> hipError_t {                                                                  \
        const int r_ = (int)(R);                                                           \
        if (lanes_per_item(r_) == 4) {                                                     \
            if (r_ == 8)  return F<4, 2, true>(__VA_ARGS__);                               \
            if (r_ <= 4)  return F<4, 1, false>(__VA_ARGS__);                              \
            return F<4, 2, false>(__VA_ARGS__);                                            \
        }                                                                                  \
        if (r_ == 16)  return F<8, 2, true>(__VA_ARGS__);                                  \
        if (r_ == 32)  return F<8, 4, true>(__VA_ARGS__);                                  \
        if (r_ == 48)  return F<8, 6, true>(__VA_ARGS__);                                  \
        if (r_ == 64)  return F<8, 8, true>(__VA_ARGS__);                                  \
        if (r_ == 96)  return F<8, 12, true>(__VA_ARGS__);                                 \
        if (r_ == 128) return F<8, 16, true>(__VA_ARGS__);                                 \
        if (r_ <= 16)  return F<8, 2, false>(__VA_ARGS__);                                 \
        if (r_ <= 32)  return F<8, 4, false>(__VA_ARGS__);                                 \
        if (r_ <= 64)  return F<8, 8, false>(__VA_ARGS__);                                 \
        return F<8, 16, false>(__VA_ARGS__);                                               \
    }()

}  // namespace comet
