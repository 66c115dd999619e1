// Rank-R kernel of the nonzero-tiled family (SpMM, TTM): lane groups walk runs of consecutive nonzeros.
#include "stream_common.hpp"

namespace comet {

namespace {

// ROWMAP: segment s writes result row rowmap[s]; the tail map then holds rows, and so do the ids this kernel
// publishes in its carries (the fix-up takes them as rows).
template <int L, int V, bool WIDE, bool ROWMAP>
__global__ void __launch_bounds__(256) k_stream_rankR(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                      const double *__restrict__ vals,
                                                      const int32_t *__restrict__ seg_begin,
                                                      const int32_t *__restrict__ rowmap, const double *__restrict__ Dn,
                                                      double *__restrict__ out, int64_t nnz, int64_t ntiles, int R,
                                                      void *scratch, Epilogue ep) {
    constexpr int NW = 256 / L;                // walkers per tile
    constexpr int WI = kTile / NW;             // items per walker
    using RL = RecLayout<L, 2>;                // record = {row offset in doubles, tail id} + value
    constexpr int SB = RL::SB;
    __shared__ __attribute__((aligned(16))) int32_t ts[kTile];
    __shared__ __attribute__((aligned(16))) int32_t rec_all[NW * RL::kStride];
    __shared__ __attribute__((aligned(16))) double wopen[256 * V];       // [walker][lane j][V]
    __shared__ int wht[NW];
    const int64_t t = blockIdx.x;
    const int64_t tb = t * (int64_t)kTile;
    const int g = threadIdx.x / L, j = threadIdx.x % L;
    const int64_t gb = tb + (int64_t)g * WI;                      // first item of this walker
    LaneItems cur;
    lane_load_items(cur, crd, vals, gb + 4 * j, nnz);             // in flight while the map is built
    build_tail_map_from_pos(ts, pos, rowmap, tb, seg_begin[t], seg_begin[t + 1], out, R, ROWMAP, ep);

    WalkState<V> st;
#pragma unroll
    for (int q = 0; q < V; ++q) { st.acc[q] = 0.0; st.first[q] = 0.0; }
    st.ht = 0; st.first_id = -1;
    int32_t *rec = rec_all + g * RL::kStride;
    const unsigned R8 = 8u * (unsigned)R;
    const unsigned slot = lane_slot_doubles<L, WIDE>(j), Ru = (unsigned)R;
    char *outb = reinterpret_cast<char *>(out);

    constexpr int G = StepGroup<V>::value, NG = SB / G;
    for (int sb = 0; sb < WI / SB; ++sb) {
        const int64_t i0 = gb + SB * sb + 4 * j;                  // this lane's four items
        LaneItems nxt;
        if (sb + 1 < WI / SB) lane_load_items(nxt, crd, vals, i0 + SB, nnz);
        {
            const int4 t4 = *reinterpret_cast<const int4 *>(ts + (i0 - tb));
            *reinterpret_cast<int4 *>(rec + 8 * j) =
                make_int4((int)((unsigned)cur.cr[0] * Ru), t4.x, (int)((unsigned)cur.cr[1] * Ru), t4.y);
            *reinterpret_cast<int4 *>(rec + 8 * j + 4) =
                make_int4((int)((unsigned)cur.cr[2] * Ru), t4.z, (int)((unsigned)cur.cr[3] * Ru), t4.w);
            *reinterpret_cast<double2 *>(rec + RL::kVal + 8 * j) = make_double2(cur.va[0], cur.va[1]);
            *reinterpret_cast<double2 *>(rec + RL::kVal + 8 * j + 4) = make_double2(cur.va[2], cur.va[3]);
        }
        __builtin_amdgcn_wave_barrier();                          // records are read by the other lanes of the group
        RowBuf<V> buf[2][G];
        auto issue = [&](auto gc, RowBuf<V> *bb) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;      // step inside the super-block
                RowBuf<V> &b = bb[decltype(sc)::value];
                const int2 ct = *reinterpret_cast<const int2 *>(rec + 2 * k);
                b.a = *reinterpret_cast<const double *>(rec + RL::kVal + 2 * k);
                b.tail = ct.y;
                grp_load_row_off<L, V, WIDE>(Dn, (unsigned)ct.x + slot, R, j, b.d);
            });
        };
        auto consume = [&](auto gc, const RowBuf<V> *bb) {
            static_for<0, G>([&](auto sc) {
                const RowBuf<V> &b = bb[decltype(sc)::value];
#pragma unroll
                for (int q = 0; q < V; ++q) st.acc[q] = fma(b.a, b.d[q], st.acc[q]);
                if (b.tail >= 0) {                                // the item ends segment `tail` (same for the group)
                    if (!st.ht) {
#pragma unroll
                        for (int q = 0; q < V; ++q) st.first[q] = st.acc[q];
                        st.first_id = b.tail;
                        st.ht = 1;
                    } else {
                        const unsigned row = (unsigned)b.tail;
                        grp_store_row_stream<L, V, WIDE>(reinterpret_cast<double *>(outb + (size_t)row * R8), 0, R, j, st.acc, ep);
                    }
#pragma unroll
                    for (int q = 0; q < V; ++q) st.acc[q] = 0.0;
                }
            });
        };
        issue(IntC<0>{}, buf[0]);
        static_for<0, NG>([&](auto gc) {
            constexpr int gi = decltype(gc)::value;
            if constexpr (gi + 1 < NG) issue(IntC<gi + 1>{}, buf[(gi + 1) & 1]);
            consume(gc, buf[gi & 1]);
        });
        __builtin_amdgcn_wave_barrier();                          // all reads of this super-block's records are done
        if (sb + 1 < WI / SB) cur = nxt;
    }

    {
        double *wo = wopen + (g * L + j) * V;
#pragma unroll
        for (int q = 0; q < V; ++q) wo[q] = st.acc[q];
        if (j == 0) wht[g] = st.ht;
    }
    __syncthreads();
    const int64_t first_row = st.ht ? (int64_t)st.first_id : 0;
    finish_tile_walkers<L, V, WIDE>(wopen, wht, g, j, st.ht, st.first, first_row, st.first_id, st.acc, out, R,
                                    carry_view(scratch, ntiles, R), t, ep);
}

template <int L, int V, bool WIDE, bool ROWMAP>
void launch_rankR_one(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals, const int32_t *rowmap,
                      const double *Dn, int R, double *out, void *scratch, hipStream_t st, Epilogue ep) {
    hipLaunchKernelGGL((k_stream_rankR<L, V, WIDE, ROWMAP>), dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals,
                       (const int32_t *)sc.seg_begin->ptr, rowmap, Dn, out, sc.nnz, sc.ntiles, R, scratch, ep);
}

template <int L, int V, bool WIDE>
hipError_t launch_rankR(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                        const int32_t *rowmap, const double *Dn, int R, double *out, void *scratch, hipStream_t st,
                        Epilogue ep) {
    if (rowmap) launch_rankR_one<L, V, WIDE, true>(sc, pos, crd, vals, rowmap, Dn, R, out, scratch, st, ep);
    else launch_rankR_one<L, V, WIDE, false>(sc, pos, crd, vals, rowmap, Dn, R, out, scratch, st, ep);
    return hipGetLastError();
}

}  // namespace

hipError_t stream_segreduce_rankR(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                                  const int32_t *rowmap, const double *Dn, int R, double *out, void *scratch,
                                  hipStream_t st, Epilogue ep) {
    return COMET_DISPATCH_RANK(launch_rankR, R, sc, pos, crd, vals, rowmap, Dn, R, out, scratch, st, ep);
}

}  // namespace comet
