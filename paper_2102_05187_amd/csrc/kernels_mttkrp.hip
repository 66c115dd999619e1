// MTTKRP kernel of the nonzero-tiled family: the rank-R walk over two nested segment levels.
#include "stream_common.hpp"

namespace comet {

namespace {

// ---- MTTKRP: the same walk, two nested segment levels ---------------------------------------------
// Inner level: fibers (segments of pos3); the per-fiber sum of vals * C[crd3, :] is scaled by the row
// B[crd2[fiber], :] when the fiber ends and folded into the slice accumulator.  Scaling is linear,
// so a fiber cut by a walker or tile boundary is folded piecewise (each piece times the same B row);
// only the slice level needs carries.  Outer level: slices (segments of pos2); a slice end writes
// row crd1[slice] of M.  Two LDS maps, both keyed by tile item: ts = the fiber's coordinate crd2[fiber]
// (its row of B) at a fiber's last nonzero, tm = output row at a slice's last nonzero (-1 elsewhere).  Both
// are looked up while the maps are built, with coalesced loads, so that the walk has no dependent index load.
template <int L, int V, bool WIDE>
__global__ void __launch_bounds__(256) k_stream_mttkrp(const int32_t *__restrict__ pos2, const int32_t *__restrict__ crd1,
                                                       const int32_t *__restrict__ pos3, const int32_t *__restrict__ crd2,
                                                       const int32_t *__restrict__ crd3, const double *__restrict__ vals,
                                                       const int32_t *__restrict__ seg_begin,
                                                       const int32_t *__restrict__ slice_begin,
                                                       const double *__restrict__ Bm, const double *__restrict__ Cm,
                                                       double *__restrict__ M, int64_t nnz, int64_t nfib, int64_t ntiles,
                                                       int R, void *scratch, Epilogue ep) {
    constexpr int NW = 256 / L, WI = kTile / NW, SB = 4 * L;
    constexpr int kMapInts = 2 * kTile;
    constexpr int kOpenInts = 256 * V * 2;
    constexpr int kLdsInts = kMapInts > kOpenInts ? kMapInts : kOpenInts;
    __shared__ __attribute__((aligned(16))) int32_t lds[kLdsInts];
    __shared__ int wht[NW], wfirst_j[NW];
    int32_t *ts = lds, *tm = lds + kTile;
    double *wopen = reinterpret_cast<double *>(lds);              // reused once the maps are dead
    const int64_t t = blockIdx.x;
    const int64_t tb = t * (int64_t)kTile, te = tb + kTile;
    const int g = threadIdx.x / L, j = threadIdx.x % L;
    const int64_t gb = tb + (int64_t)g * WI;
    LaneItems cur;
    lane_load_items(cur, crd3, vals, gb + 4 * j, nnz);            // in flight while the maps are built

    for (int i = threadIdx.x * 4; i < 2 * kTile; i += blockDim.x * 4)
        *reinterpret_cast<int4 *>(lds + i) = make_int4(-1, -1, -1, -1);
    __syncthreads();
    for (int32_t f = seg_begin[t] + threadIdx.x; f < seg_begin[t + 1]; f += blockDim.x) {
        int32_t b = pos3[f], e = pos3[f + 1];
        if (e > b) ts[(int64_t)e - 1 - tb] = crd2[f];
    }
    for (int32_t sl = slice_begin[t] + threadIdx.x; sl < slice_begin[t + 1]; sl += blockDim.x) {
        int32_t fb = pos2[sl], fe = pos2[sl + 1];
        int64_t il = -1;                                          // last nonzero of the slice
        for (int32_t f = fe - 1; f >= fb; --f) {
            int32_t b = pos3[f], e = pos3[f + 1];
            if (e > b) { il = (int64_t)e - 1; break; }
        }
        if (il >= tb && il < te) tm[il - tb] = crd1[sl];
        if (il < 0) {                                             // a stored slice without any nonzero: its row is zero
            double *row = M + (int64_t)crd1[sl] * R;
            for (int r = 0; r < R; ++r) row[r] = ep_empty(ep, row + r);
        }
    }
    __syncthreads();

    double facc[V], sacc[V], first[V];
#pragma unroll
    for (int q = 0; q < V; ++q) { facc[q] = 0.0; sacc[q] = 0.0; first[q] = 0.0; }
    int ht = 0, first_row = -1, first_j = -1, last_is_tail = 1;

    // narrow rows: two steps per pipeline group instead of four keeps the kernel under 128 registers
    // (four wavefronts per SIMD instead of three), which is worth more here than the deeper gather queue
    constexpr int G = V <= 2 ? 2 : StepGroup<V>::value, NG = SB / G;
    for (int sb = 0; sb < WI / SB; ++sb) {
        const int64_t i0 = gb + SB * sb + 4 * j;
        LaneItems nxt;
        if (sb + 1 < WI / SB) lane_load_items(nxt, crd3, vals, i0 + SB, nnz);
        int tl[4], tr[4];
        {
            const int4 t4 = *reinterpret_cast<const int4 *>(ts + (i0 - tb));
            const int4 m4 = *reinterpret_cast<const int4 *>(tm + (i0 - tb));
            tl[0] = t4.x; tl[1] = t4.y; tl[2] = t4.z; tl[3] = t4.w;
            tr[0] = m4.x; tr[1] = m4.y; tr[2] = m4.z; tr[3] = m4.w;
        }
        const bool any_item = gb + SB * sb < nnz;
        RowBuf<V> cbuf[2][G], bbuf[2][G];
        auto issue = [&](auto gc, RowBuf<V> *cb_, RowBuf<V> *bb_) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;
                constexpr int s_ = decltype(sc)::value;
                const int c = grp_bcast_i<L, k / 4>(cur.cr[k % 4]);
                grp_load_row<L, V, WIDE>(Cm, c, R, j, cb_[s_].d);
                const int tf = grp_bcast_i<L, k / 4>(tl[k % 4]);
                // The B row is needed where a fiber ends.  Narrow rows: loaded at every item (row 0, a cache hit,
                // where no fiber ends), so that the number of loads in flight is fixed and the gathers of the next
                // group really overlap these FMAs (a load under a branch makes the wait for the rows of this group
                // cover part of the next group's loads): 1.74 -> 1.61 ms at rank 16.  Wide rows pay more for the
                // extra load instructions than they gain (5.18 -> 5.32 ms at rank 64) and keep the branch.
                if constexpr (V <= 2) grp_load_row<L, V, WIDE>(Bm, tf >= 0 ? tf : 0, R, j, bb_[s_].d);
                else if (tf >= 0) grp_load_row<L, V, WIDE>(Bm, tf, R, j, bb_[s_].d);
            });
        };
        auto consume = [&](auto gc, const RowBuf<V> *cb_, const RowBuf<V> *bb_) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;
                constexpr int s_ = decltype(sc)::value;
                const double a = grp_bcast_d<L, k / 4>(cur.va[k % 4]);
                const int tf = grp_bcast_i<L, k / 4>(tl[k % 4]);
                const int tmr = grp_bcast_i<L, k / 4>(tr[k % 4]);
#pragma unroll
                for (int q = 0; q < V; ++q) facc[q] = fma(a, cb_[s_].d[q], facc[q]);
                if (any_item) last_is_tail = tf >= 0;
                if (tf >= 0) {
                    if (first_j < 0) first_j = tf;
#pragma unroll
                    for (int q = 0; q < V; ++q) { sacc[q] = fma(bb_[s_].d[q], facc[q], sacc[q]); facc[q] = 0.0; }
                    if (tmr >= 0) {
                        if (!ht) {
#pragma unroll
                            for (int q = 0; q < V; ++q) first[q] = sacc[q];
                            first_row = tmr; ht = 1;
                        } else {
                            grp_store_row_stream<L, V, WIDE>(M, tmr, R, j, sacc, ep);
                        }
#pragma unroll
                        for (int q = 0; q < V; ++q) sacc[q] = 0.0;
                    }
                }
            });
        };
        issue(IntC<0>{}, cbuf[0], bbuf[0]);
        static_for<0, NG>([&](auto gc) {
            constexpr int gi = decltype(gc)::value;
            if constexpr (gi + 1 < NG) issue(IntC<gi + 1>{}, cbuf[(gi + 1) & 1], bbuf[(gi + 1) & 1]);
            consume(gc, cbuf[gi & 1], bbuf[gi & 1]);
        });
        if (sb + 1 < WI / SB) cur = nxt;
    }

    // A fiber left open at the end of this walker's range ends at the next fiber end of the tile, or,
    // if there is none, it is the fiber that contains the first nonzero of the next tile.
    if (j == 0) wfirst_j[g] = first_j;
    __syncthreads();                                              // also: every walk is done, the maps are dead
    if (!last_is_tail) {
        int jrow = -1;
        for (int g2 = g + 1; g2 < NW; ++g2) { const int j2 = wfirst_j[g2]; if (j2 >= 0) { jrow = j2; break; } }
        if (jrow < 0 && (int64_t)seg_begin[t + 1] < nfib) jrow = crd2[seg_begin[t + 1]];
        if (jrow >= 0) {
            double bw[V];
            grp_load_row<L, V, WIDE>(Bm, jrow, R, j, bw);
#pragma unroll
            for (int q = 0; q < V; ++q) sacc[q] = fma(bw[q], facc[q], sacc[q]);
        }
    }
    {
        double *wo = wopen + (g * L + j) * V;
#pragma unroll
        for (int q = 0; q < V; ++q) wo[q] = sacc[q];
        if (j == 0) wht[g] = ht;
    }
    __syncthreads();
    finish_tile_walkers<L, V, WIDE>(wopen, wht, g, j, ht, first, first_row, first_row, sacc, M, R,
                                    carry_view(scratch, ntiles, R), t, ep);
}

template <int L, int V, bool WIDE>
hipError_t launch_mttkrp(const Schedule &sc, const int32_t *pos2, const int32_t *crd1, const int32_t *pos3,
                         const int32_t *crd2, const int32_t *crd3, const double *vals, const double *B, const double *C,
                         int R, double *M, void *scratch, hipStream_t st, Epilogue ep) {
    hipLaunchKernelGGL((k_stream_mttkrp<L, V, WIDE>), dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos2, crd1, pos3, crd2,
                       crd3, vals, (const int32_t *)sc.seg_begin->ptr, (const int32_t *)sc.slice_begin->ptr, B, C, M,
                       sc.nnz, sc.nseg, sc.ntiles, R, scratch, ep);
    return hipGetLastError();
}

}  // namespace

hipError_t stream_mttkrp(const Schedule &sc, const int32_t *pos2, const int32_t *crd1, int64_t nslice,
                         const int32_t *pos3, const int32_t *crd2, const int32_t *crd3, const double *vals,
                         const double *B, const double *C, int64_t R, double *M, void *scratch, hipStream_t st,
                         Epilogue ep) {
    (void)nslice;
    if (sc.ntiles <= 0) return hipSuccess;
    if (!stream_mttkrp_supports_rank(R) || !sc.slice_begin) return hipErrorNotSupported;
    const int r = (int)R;
    hipError_t e = COMET_DISPATCH_RANK(launch_mttkrp, R, sc, pos2, crd1, pos3, crd2, crd3, vals, B, C, r, M, scratch, st, ep);
    if (e != hipSuccess) return e;
    return run_fixup(scratch, sc.ntiles, r, nullptr, M, sc.max_parent_len > 0 ? sc.max_parent_len / kTile + 2 : 0, st, ep);
}

}  // namespace comet
