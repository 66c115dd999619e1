// Rank-1 kernels of the nonzero-tiled family (SpMV, TTV on CSF and on sorted coordinate lists), the
// carry fix-up kernels shared by all of them, and the host entry points of the family.
#include <atomic>

#include "stream_common.hpp"

namespace comet {

namespace {


constexpr int kWaves = 4;                    // wavefronts per workgroup
constexpr int kWaveItems = kTile / kWaves;   // 1024 consecutive items per wavefront

// ---- DPP helpers (gfx9 controls: row_shr:n = 0x110+n, wave_shr:1 = 0x138, row_bcast:15 = 0x142,
//      row_bcast:31 = 0x143, quad_perm = 8-bit selector) ------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_d(double old, double v) {
    int lo = __builtin_amdgcn_update_dpp(__double2loint(old), __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    int hi = __builtin_amdgcn_update_dpp(__double2hiint(old), __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}
// Same with every row and bank enabled and zero fill for lanes that have no source (bound_ctrl): the
// result does not depend on a previous register value, so no identity has to be materialised first.
template <int CTRL>
__device__ __forceinline__ int dpp0_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp0_d(double v) {
    int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
    int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double readlane_d(double v, int lane) {
    int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Inclusive segmented scan over the 64 lanes.  Element = (f, v); combine(left, right) =
// (left.f | right.f, right.f ? right.v : left.v + right.v): a flagged element cuts the running sum.
__device__ __forceinline__ void segscan_inclusive(int &f, double &v) {
#define COMET_SCAN_STEP0(CTRL)                            \
    {                                                     \
        int nf = dpp0_i<CTRL>(f);                         \
        double nv = dpp0_d<CTRL>(v);                      \
        v = f ? v : nv + v;                               \
        f |= nf;                                          \
    }
#define COMET_SCAN_STEP(CTRL, RM)                         \
    {                                                     \
        int nf = dpp_i<CTRL, RM>(0, f);                   \
        double nv = dpp_d<CTRL, RM>(0.0, v);              \
        v = f ? v : nv + v;                               \
        f |= nf;                                          \
    }
    COMET_SCAN_STEP0(0x111)       // row_shr:1
    COMET_SCAN_STEP0(0x112)       // row_shr:2
    COMET_SCAN_STEP0(0x114)       // row_shr:4
    COMET_SCAN_STEP0(0x118)       // row_shr:8
    COMET_SCAN_STEP(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
    COMET_SCAN_STEP(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef COMET_SCAN_STEP0
#undef COMET_SCAN_STEP
}

// ---- rank-1 walk ---------------------------------------------------------------------------------
// A wavefront owns 1024 consecutive items = 8 blocks of 128; in a block lane l holds items 2l, 2l+1
// (one 8-byte crd load and one 16-byte vals load per lane, consecutive lanes on consecutive bytes).
// The loads of four blocks are issued together, and the first four before the tail map is built, so
// the HBM latency overlaps the map construction and the scans of the preceding blocks.
struct Rank1Half {
    int2    c[4];
    double2 a[4];
};

__device__ __forceinline__ void rank1_load_half(Rank1Half &h, const int32_t *__restrict__ crd,
                                                const double *__restrict__ vals, int64_t base, int lane, int64_t nnz) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t i0 = base + b * 128 + 2 * lane;
        if (i0 + 1 < nnz) {
            // streamed once: non-temporal, so the lines do not displace the gathered operand in L1/L2
            const long long cc = __builtin_nontemporal_load(reinterpret_cast<const long long *>(crd + i0));
            h.c[b].x = (int)(cc & 0xffffffffll); h.c[b].y = (int)(cc >> 32);
            h.a[b].x = __builtin_nontemporal_load(vals + i0);
            h.a[b].y = __builtin_nontemporal_load(vals + i0 + 1);
        } else {
            h.c[b].x = i0 < nnz ? crd[i0] : 0;   h.c[b].y = 0;
            h.a[b].x = i0 < nnz ? vals[i0] : 0.0; h.a[b].y = 0.0;
        }
    }
}

struct Rank1Carry {
    int    cf;     // a segment end was seen in the blocks done so far
    double cv;     // sum of the items after the last segment end
};

template <bool ROWMAP>
__device__ __forceinline__ void rank1_process_half(const Rank1Half &h, const double2 *xv, const int2 *tt,
                                                   int64_t base, int64_t nnz, int lane, int w,
                                                   const int32_t *__restrict__ rowmap, double *__restrict__ out,
                                                   Rank1Carry &cy, double *wsum_first, int *wsum_first_id,
                                                   const Epilogue ep = Epilogue()) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t i0 = base + b * 128 + 2 * lane;
        const int2 t = tt[b];                                // segment ids of the items that end a segment, else -1
        const double p0 = i0 < nnz ? h.a[b].x * xv[b].x : 0.0;
        const double p1 = i0 + 1 < nnz ? h.a[b].y * xv[b].y : 0.0;
        const int f = (t.x >= 0) | (t.y >= 0);
        const double first = t.x >= 0 ? p0 : p0 + p1;
        const int first_id = t.x >= 0 ? t.x : t.y;
        const double open = t.y >= 0 ? 0.0 : (t.x >= 0 ? p1 : p0 + p1);
        if (t.x >= 0 && t.y >= 0) {                          // item i0+1 is a whole segment by itself
            const int64_t row = ROWMAP ? (int64_t)rowmap[t.y] : (int64_t)t.y;
            out[row] = ep_apply(ep, p1, out + row);
        }
        int sf = f;
        double sv = open;
        segscan_inclusive(sf, sv);
        // exclusive value for this lane = carry (+) inclusive value of the previous lane
        const int pf = dpp0_i<0x138>(sf);                    // wave_shr:1, lane 0 gets the identity (0, 0.0)
        const double pv = dpp0_d<0x138>(sv);
        const int ef = cy.cf | pf;
        const double ev = pf ? pv : cy.cv + pv;
        if (f) {
            const double value = ev + first;
            if (ef) {
                const int64_t row = ROWMAP ? (int64_t)rowmap[first_id] : (int64_t)first_id;
                out[row] = ep_apply(ep, value, out + row);
            } else {                                         // the first segment end of this wavefront's range
                wsum_first[w] = value;
                wsum_first_id[w] = first_id;
            }
        }
        const int tf = __builtin_amdgcn_readlane(sf, 63);
        const double tv = readlane_d(sv, 63);
        cy.cv = tf ? tv : cy.cv + tv;
        cy.cf |= tf;
    }
}

__device__ __forceinline__ void rank1_gather(const Rank1Half &h, const double *__restrict__ x, double2 *xv) {
#pragma unroll
    for (int b = 0; b < 4; ++b) { xv[b].x = x[h.c[b].x]; xv[b].y = x[h.c[b].y]; }
}

// Second part of the walk (after the map is complete); h0 holds the already issued first half.
template <bool ROWMAP>
__device__ __forceinline__ void walk_rank1(Rank1Half &h0, const int32_t *ts, const int32_t *__restrict__ crd,
                                           const double *__restrict__ vals, const double *__restrict__ x,
                                           const int32_t *__restrict__ rowmap, double *__restrict__ out, int64_t tb,
                                           int64_t nnz, int *wsum_ht, double *wsum_open, double *wsum_first,
                                           int *wsum_first_id, const Epilogue ep = Epilogue()) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t wb = tb + (int64_t)w * kWaveItems;
    Rank1Carry cy{0, 0.0};
    double2 xv[4];
    rank1_gather(h0, x, xv);
    Rank1Half h1;
    rank1_load_half(h1, crd, vals, wb + 512, lane, nnz);
    int2 tt[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) tt[b] = *reinterpret_cast<const int2 *>(ts + (wb - tb) + b * 128 + 2 * lane);
    rank1_process_half<ROWMAP>(h0, xv, tt, wb, nnz, lane, w, rowmap, out, cy, wsum_first, wsum_first_id, ep);
    rank1_gather(h1, x, xv);
#pragma unroll
    for (int b = 0; b < 4; ++b) tt[b] = *reinterpret_cast<const int2 *>(ts + (wb - tb) + 512 + b * 128 + 2 * lane);
    rank1_process_half<ROWMAP>(h1, xv, tt, wb + 512, nnz, lane, w, rowmap, out, cy, wsum_first, wsum_first_id, ep);
    if (lane == 0) { wsum_ht[w] = cy.cf; wsum_open[w] = cy.cv; }
}

// Combine the wavefront summaries of one tile in order and publish the tile summary.
template <bool ROWMAP>
__device__ __forceinline__ void finish_tile_rank1(const int *wsum_ht, const double *wsum_open, const double *wsum_first,
                                                  const int *wsum_first_id, const int32_t *__restrict__ rowmap,
                                                  double *__restrict__ out, CarryView cb, int64_t t,
                                                  const Epilogue ep = Epilogue()) {
    if (threadIdx.x != 0) return;
    int rf = 0, fid = -1;
    double rv = 0.0, tfirst = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        if (wsum_ht[w]) {
            const double value = rv + wsum_first[w];
            if (rf) {
                const int64_t row = ROWMAP ? (int64_t)rowmap[wsum_first_id[w]] : (int64_t)wsum_first_id[w];
                out[row] = ep_apply(ep, value, out + row);
            } else {
                tfirst = value; fid = wsum_first_id[w]; rf = 1;
            }
            rv = wsum_open[w];
        } else {
            rv += wsum_open[w];
        }
    }
    cb.has_tail[t] = rf;
    cb.first_id[t] = fid;
    cb.first[t] = tfirst;
    cb.open[t] = rv;
}

template <bool ROWMAP>
__global__ void __launch_bounds__(256) k_stream_rank1(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                      const double *__restrict__ vals,
                                                      const int32_t *__restrict__ seg_begin,
                                                      const int32_t *__restrict__ rowmap, const double *__restrict__ x,
                                                      double *__restrict__ out, int64_t nnz, int64_t ntiles,
                                                      void *scratch, Epilogue ep) {
    __shared__ __attribute__((aligned(16))) int32_t ts[kTile];
    __shared__ int wsum_ht[kWaves], wsum_first_id[kWaves];
    __shared__ double wsum_open[kWaves], wsum_first[kWaves];
    const int64_t t = blockIdx.x;
    const int64_t tb = t * (int64_t)kTile;
    Rank1Half h0;
    rank1_load_half(h0, crd, vals, tb + (int64_t)(threadIdx.x >> 6) * kWaveItems, threadIdx.x & 63, nnz);
    build_tail_map_from_pos(ts, pos, rowmap, tb, seg_begin[t], seg_begin[t + 1], out, 1, false, ep);
    walk_rank1<ROWMAP>(h0, ts, crd, vals, x, rowmap, out, tb, nnz, wsum_ht, wsum_open, wsum_first, wsum_first_id, ep);
    __syncthreads();
    finish_tile_rank1<ROWMAP>(wsum_ht, wsum_open, wsum_first, wsum_first_id, rowmap, out, carry_view(scratch, ntiles, 1), t, ep);
}

// ---- rank-1 kernel with the dense vector staged in LDS ----------------------------------------------
// When x (SpMV) / v (TTV) fits in the 160 KB of LDS next to a few hundred bytes of bookkeeping, one
// workgroup of 16 wavefronts per CU copies it in once and every gather x[crd] becomes an LDS read: the
// L1 / texture-address path, which handles only about one scattered 8-byte gather per clock per CU,
// is then left to the streaming loads.  Each wavefront works alone on 1024-item chunks (no workgroup
// barrier after the staging): it marks the segment ends of its chunk in a private 1024-bit mask,
// gets the segment id of an end as (first segment of the chunk) + (ends before it) -- valid because
// this kernel is only used when the level has no empty segment -- and writes the chunk summary
// straight to the carry buffer (one entry per chunk).
// COO = true: the input is a sorted coordinate list [CN,S,S]; segment ends come from neighbour
// comparisons of (c0, c1) instead of pos, the id of a run is (runs started before the chunk) + (runs
// started earlier in the chunk), and the result's coordinate arrays y0 / y1 are written here too.
template <bool ROWMAP, bool COO>
__global__ void __launch_bounds__(1024) k_stream_rank1_ldsvec(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                              const double *__restrict__ vals,
                                                              const int32_t *__restrict__ chunk_begin,
                                                              const int32_t *__restrict__ rowmap,
                                                              const double *__restrict__ x, int64_t ncols,
                                                              double *__restrict__ out, int64_t nnz, int64_t nchunks,
                                                              void *scratch, const int32_t *__restrict__ c0,
                                                              const int32_t *__restrict__ c1, int32_t *__restrict__ y0,
                                                              int32_t *__restrict__ y1, Epilogue ep) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int64_t xpad = (ncols + 1) & ~(int64_t)1;
    double *xs = reinterpret_cast<double *>(lds_raw);
    unsigned *bits_all = reinterpret_cast<unsigned *>(lds_raw + xpad * 8);            // [16][32]
    double *wfirst_all = reinterpret_cast<double *>(lds_raw + xpad * 8 + 16 * 128);   // [16]
    int *wfirst_id_all = reinterpret_cast<int *>(lds_raw + xpad * 8 + 16 * 128 + 16 * 8);   // [16]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned *bits = bits_all + w * 32;
    const int64_t stride = (int64_t)gridDim.x * 16;
    int64_t c = (int64_t)blockIdx.x * 16 + w;
    Rank1Half h0;
    if (c < nchunks) rank1_load_half(h0, crd, vals, c * kChunk, lane, nnz);          // in flight during the staging
    for (int64_t i = (int64_t)threadIdx.x * 2; i + 1 < ncols; i += 2048)
        *reinterpret_cast<double2 *>(xs + i) = *reinterpret_cast<const double2 *>(x + i);
    if ((ncols & 1) && threadIdx.x == 0) xs[ncols - 1] = x[ncols - 1];
    __syncthreads();
    CarryView cb = carry_view(scratch, nchunks, 1);
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (; c < nchunks; c += stride) {
        const int64_t cbeg = c * kChunk;
        int base_id;
        if constexpr (COO) {
            constexpr int kRows = kChunk / 64, kBatch = 4;
            // run starts of a row of 64 items (hm), and the same with items past the end counted as starts (hx);
            // the mask of run ENDS of row r-1 is written as soon as row r is known, so only one row is kept
            unsigned long long hx_prev = 0ull;
            bool first_is_head = false;
            const int runs_before = chunk_begin[c];
            // the coordinate loads of a batch of rows are issued together; the predecessor of an item comes from
            // the neighbouring lane (wave_shr:1), of lane 0 from the previous row (or the item before the chunk)
            const int64_t inext = cbeg + kChunk;
            int before0 = -2, before1 = -2, after0 = -1, after1 = -1;
            if (cbeg > 0) { before0 = c0[cbeg - 1]; before1 = c1[cbeg - 1]; }
            if (inext < nnz) { after0 = c0[inext]; after1 = c1[inext]; }
            int running = runs_before;
            // item e ends a run when item e+1 starts one or lies past the end of the list
            auto write_ends = [&](int r, unsigned long long hx_r, unsigned long long nextbit) {
                const int64_t left = nnz - (cbeg + 64 * r);          // items of this row that exist
                const unsigned long long exist = left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
                const unsigned long long tmask = ((hx_r >> 1) | (nextbit << 63)) & exist;
                if (lane == 0) *reinterpret_cast<unsigned long long *>(bits + 2 * r) = tmask;
            };
#pragma unroll
            for (int rb = 0; rb < kRows; rb += kBatch) {          // batches of rows keep the register count down
                int a0[kBatch], a1[kBatch];
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    const int64_t i = cbeg + 64 * (rb + q) + lane;
                    a0[q] = i < nnz ? __builtin_nontemporal_load(c0 + i) : -1;
                    a1[q] = i < nnz ? __builtin_nontemporal_load(c1 + i) : -1;
                }
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    const int r = rb + q;
                    const int64_t i = cbeg + 64 * r + lane;
                    const int p0 = dpp_i<0x138, 0xf>(before0, a0[q]);
                    const int p1 = dpp_i<0x138, 0xf>(before1, a1[q]);
                    const bool differs = a0[q] != p0 || a1[q] != p1;
                    const unsigned long long hm = __ballot(differs && i < nnz);
                    const unsigned long long hx = __ballot(differs);
                    before0 = __builtin_amdgcn_readlane(a0[q], 63);
                    before1 = __builtin_amdgcn_readlane(a1[q], 63);
                    if ((hm >> lane) & 1ull) {
                        const int id = running + __popcll(hm & lt_mask);
                        y0[id] = a0[q]; y1[id] = a1[q];
                    }
                    running += __popcll(hm);
                    if (r == 0) first_is_head = (hm & 1ull) != 0ull;
                    else write_ends(r - 1, hx_prev, hx & 1ull);
                    hx_prev = hx;
                }
            }
            write_ends(kRows - 1, hx_prev, (after0 != before0 || after1 != before1) ? 1ull : 0ull);
            base_id = runs_before - (first_is_head ? 0 : 1);          // the run that holds the chunk's first item
        } else {
            if (lane < 32) bits[lane] = 0u;
            __builtin_amdgcn_wave_barrier();
            const int32_t s0 = chunk_begin[c], s1 = chunk_begin[c + 1];
            for (int32_t sgm = s0 + lane; sgm < s1; sgm += 64) {
                const int64_t idx = (int64_t)pos[sgm + 1] - 1 - cbeg;                  // in [0, 1024): the segment ends here
                atomicOr(&bits[idx >> 5], 1u << (idx & 31));
            }
            base_id = s0;
        }
        __builtin_amdgcn_wave_barrier();
        Rank1Carry cy{0, 0.0};
        auto tails_of_half = [&](int half, int2 *tt) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const unsigned word = bits[(half * 4 + b) * 4 + (lane >> 4)];
                const int sh = (2 * lane) & 31;
                const bool t0 = (word >> sh) & 1u, t1 = (word >> (sh + 1)) & 1u;
                const unsigned long long b0 = __ballot(t0), b1 = __ballot(t1);
                const int id0 = base_id + __popcll(b0 & lt_mask) + __popcll(b1 & lt_mask);
                tt[b].x = t0 ? id0 : -1;
                tt[b].y = t1 ? id0 + (t0 ? 1 : 0) : -1;
                base_id += __popcll(b0) + __popcll(b1);
            }
        };
        auto gather = [&](const Rank1Half &h, double2 *xv) {
#pragma unroll
            for (int b = 0; b < 4; ++b) { xv[b].x = xs[h.c[b].x]; xv[b].y = xs[h.c[b].y]; }
        };
        double2 xv[4];
        int2 tt[4];
        Rank1Half h1;
        rank1_load_half(h1, crd, vals, cbeg + 512, lane, nnz);
        gather(h0, xv);
        tails_of_half(0, tt);
        rank1_process_half<ROWMAP>(h0, xv, tt, cbeg, nnz, lane, w, rowmap, out, cy, wfirst_all, wfirst_id_all, ep);
        if (c + stride < nchunks) rank1_load_half(h0, crd, vals, (c + stride) * kChunk, lane, nnz);   // next chunk
        gather(h1, xv);
        tails_of_half(1, tt);
        rank1_process_half<ROWMAP>(h1, xv, tt, cbeg + 512, nnz, lane, w, rowmap, out, cy, wfirst_all, wfirst_id_all, ep);
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) {
            cb.has_tail[c] = cy.cf;
            cb.open[c] = cy.cv;
            cb.first[c] = cy.cf ? wfirst_all[w] : 0.0;
            cb.first_id[c] = cy.cf ? wfirst_id_all[w] : -1;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- rank-1 kernel for sorted coordinate lists [CN,S,S] -------------------------------------------
// A segment is a run of equal (c0, c1).  The root level keeps every coordinate and the lower levels
// are singletons (one coordinate per position), so run ends are found by comparing neighbours.  The
// result's own coordinate arrays are written here too: run number n (run_base[t] + runs started
// earlier in the tile) gets y0[n], y1[n] from the run's first nonzero.
__global__ void __launch_bounds__(256) k_stream_rank1_coo(const int32_t *__restrict__ c0, const int32_t *__restrict__ c1,
                                                          const int32_t *__restrict__ c2, const double *__restrict__ vals,
                                                          const int32_t *__restrict__ run_base,
                                                          const double *__restrict__ v, int32_t *__restrict__ y0,
                                                          int32_t *__restrict__ y1, double *__restrict__ yv, int64_t nnz,
                                                          int64_t ntiles, void *scratch) {
    __shared__ __attribute__((aligned(16))) int32_t ts[kTile];
    __shared__ int wsum_ht[kWaves], wsum_first_id[kWaves], wcount[kWaves];
    __shared__ double wsum_open[kWaves], wsum_first[kWaves];
    const int64_t t = blockIdx.x;
    const int64_t tb = t * (int64_t)kTile;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t wb = tb + (int64_t)w * kWaveItems;
    Rank1Half h0;
    rank1_load_half(h0, c2, vals, wb, lane, nnz);
    constexpr int kRows = kWaveItems / 64;
    unsigned long long hm[kRows];
    int count = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t i = wb + 64 * r + lane;
        bool head = false;
        if (i < nnz) head = i == 0 || c0[i] != c0[i - 1] || c1[i] != c1[i - 1];
        hm[r] = __ballot(head);
        count += __popcll(hm[r]);
    }
    // does the item right after this wavefront's range start a run (or lie past the end)?
    const int64_t inext = wb + kWaveItems;
    const bool next_head = inext >= nnz || c0[inext] != c0[inext - 1] || c1[inext] != c1[inext - 1];
    if (lane == 0) wcount[w] = count;
    __syncthreads();
    int running = run_base[t];
    for (int u = 0; u < w; ++u) running += wcount[u];
    const unsigned long long le_mask = (2ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t i = wb + 64 * r + lane;
        const int id = running + __popcll(hm[r] & le_mask) - 1;
        const bool head = (hm[r] >> lane) & 1ull;
        bool tail;
        if (lane < 63) tail = (hm[r] >> (lane + 1)) & 1ull;
        else tail = r + 1 < kRows ? (hm[r + 1] & 1ull) != 0 : next_head;
        if (i + 1 >= nnz) tail = true;
        if (head) { y0[id] = c0[i]; y1[id] = c1[i]; }
        ts[i - tb] = (i < nnz && tail) ? id : -1;
        running += __popcll(hm[r]);
    }
    __syncthreads();
    walk_rank1<false>(h0, ts, c2, vals, v, nullptr, yv, tb, nnz, wsum_ht, wsum_open, wsum_first, wsum_first_id);
    __syncthreads();
    finish_tile_rank1<false>(wsum_ht, wsum_open, wsum_first, wsum_first_id, nullptr, yv, carry_view(scratch, ntiles, 1), t);
}

// ---- fix-up: finish the first segment end of every tile -------------------------------------------
// value = first[t] + open[t-1] + open[t-2] + ... up to and including the nearest tile that contains
// a segment end.  One thread per (tile, r).
__global__ void __launch_bounds__(256) k_stream_fixup(void *scratch, int64_t ntiles, int R,
                                                      const int32_t *__restrict__ rowmap, double *__restrict__ out,
                                                      Epilogue ep) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= ntiles * R) return;
    const int64_t t = g / R;
    const int r = (int)(g - t * R);
    CarryView cb = carry_view(scratch, ntiles, R);
    if (!cb.has_tail[t]) return;
    double v = cb.first[t * R + r];
    for (int64_t u = t - 1; u >= 0; --u) {
        v += cb.open[u * R + r];
        if (cb.has_tail[u]) break;
    }
    const int32_t id = cb.first_id[t];
    const int64_t row = rowmap ? (int64_t)rowmap[id] : (int64_t)id;
    out[row * R + r] = ep_apply(ep, v, out + row * R + r);
}


// One pass of the hierarchical fix-up: thread (g, r) folds the kFixGroup summaries of group g in
// order.  A segment end whose carry chain starts inside the group is final and is written to out;
// the group's own summary (first segment end, trailing open sum) goes one level up.
__global__ void __launch_bounds__(256) k_fixup_level(const double *__restrict__ lo_first, const double *__restrict__ lo_open,
                                                     const int32_t *__restrict__ lo_ht, const int32_t *__restrict__ lo_id,
                                                     int64_t n_lo, double *__restrict__ up_first,
                                                     double *__restrict__ up_open, int32_t *__restrict__ up_ht,
                                                     int32_t *__restrict__ up_id, int64_t n_up, int R,
                                                     const int32_t *__restrict__ rowmap, double *__restrict__ out,
                                                     Epilogue ep) {
    const int64_t gidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gidx >= n_up * R) return;
    const int64_t g = gidx / R;
    const int r = (int)(gidx - g * R);
    const int64_t u0 = g * kFixGroup;
    const int64_t u1 = u0 + kFixGroup < n_lo ? u0 + kFixGroup : n_lo;
    int rf = 0, gid = -1;
    double rv = 0.0, gfirst = 0.0;
    for (int64_t ub = u0; ub < u1; ub += 16) {
        // 16 summaries at a time: all loads are independent of the fold, so they are issued together
        int ht[16], id[16];
        double op[16], fi[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t u = ub + i;
            const bool in = u < u1;
            ht[i] = in ? lo_ht[u] : 0;
            id[i] = in ? lo_id[u] : -1;
            op[i] = in ? lo_open[u * R + r] : 0.0;
            fi[i] = in ? lo_first[u * R + r] : 0.0;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (ht[i]) {
                const double value = rv + fi[i];
                if (rf) {
                    const int64_t row = rowmap ? (int64_t)rowmap[id[i]] : (int64_t)id[i];
                    out[row * R + r] = ep_apply(ep, value, out + row * R + r);
                } else {
                    gfirst = value; gid = id[i]; rf = 1;
                }
                rv = op[i];
            } else {
                rv += op[i];
            }
        }
    }
    up_first[g * R + r] = gfirst;
    up_open[g * R + r] = rv;
    if (r == 0) { up_ht[g] = rf; up_id[g] = gid; }
}


}  // namespace

// Finish every segment that a tile boundary cut: fold the tile summaries level by level, then
// walk the few top-level summaries serially.  `max_chain` bounds the number of consecutive tiles
// one segment can span (0 = unknown); short chains go straight to the serial walk.
hipError_t run_fixup(void *scratch, int64_t ntiles, int R, const int32_t *rowmap, double *out, int64_t max_chain,
                     hipStream_t st, Epilogue ep) {
    char *base = (char *)scratch;
    int64_t n = ntiles;
    const bool direct = max_chain > 0 && max_chain <= 24;
    while (!direct && n > kFixGroup) {
        const int64_t n_up = (n + kFixGroup - 1) / kFixGroup;
        CarryView lo = carry_view(base, n, R);
        char *up_base = base + carry_level_bytes(n, R);
        CarryView up = carry_view(up_base, n_up, R);
        const int64_t threads = n_up * R;
        hipLaunchKernelGGL(k_fixup_level, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, lo.first, lo.open,
                           lo.has_tail, lo.first_id, n, up.first, up.open, up.has_tail, up.first_id, n_up, R, rowmap, out, ep);
        base = up_base;
        n = n_up;
    }
    const int64_t threads = n * R;
    hipLaunchKernelGGL(k_stream_fixup, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (void *)base, n, R,
                       rowmap, out, ep);
    return hipGetLastError();
}


// Allows a kernel to use up to the whole 160 KB of LDS as dynamic shared memory; done once per kernel
// (it is not a stream operation, but calling it once keeps it out of captured regions after the first call).
template <auto Kernel>
static hipError_t allow_full_lds() {
    static hipError_t status = hipFuncSetAttribute((const void *)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return status;
}

int current_device_cu_count() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 256; }
    if (dev >= 0 && dev < 64 && cached[dev].load() > 0) return cached[dev].load();
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) { (void)hipGetLastError(); n = 256; }
    if (dev >= 0 && dev < 64) cached[dev].store(n);
    return n;
}

bool stream_supports_rank(int64_t R) { return R >= 1 && R <= 128; }
bool stream_mttkrp_supports_rank(int64_t R) { return R >= 1 && R <= 128; }
bool stream_supports_coo() { return true; }

size_t stream_scratch_bytes(int64_t ntiles, int64_t R) {
    int64_t n = ntiles < 1 ? 1 : ntiles;
    size_t total = 0;
    for (;;) {
        total += carry_level_bytes(n, R);
        if (n <= kFixGroup) break;
        n = (n + kFixGroup - 1) / kFixGroup;
    }
    return total + 256;
}

hipError_t stream_segreduce(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                            const int32_t *rowmap, const double *Dn, int64_t dense_rows, int64_t R, double *out,
                            void *scratch, bool plain, hipStream_t st, Epilogue ep) {
    if (sc.ntiles <= 0) return hipSuccess;
    if (!stream_supports_rank(R)) return hipErrorNotSupported;
    const int32_t *sb = (const int32_t *)sc.seg_begin->ptr;
    hipError_t e = hipSuccess;
    if (R == 1) {
        const size_t lds_bytes = (size_t)((dense_rows + 1) & ~(int64_t)1) * 8 + 16 * 128 + 16 * 8 + 16 * 4;
        if (sc.empty_segments == 0 && sc.chunk_seg_begin && sc.nchunks >= 16 && lds_bytes <= 160 * 1024 && !plain) {
            // the dense vector fits in LDS and every segment holds a nonzero: wavefront-per-chunk kernel
            const int ncu = current_device_cu_count();
            const int64_t want = (sc.nchunks + 15) / 16;
            const unsigned grid = (unsigned)(want < ncu ? want : ncu);
            const int32_t *csb = (const int32_t *)sc.chunk_seg_begin->ptr;
            if (rowmap) {
                e = allow_full_lds<k_stream_rank1_ldsvec<true, false>>();
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((k_stream_rank1_ldsvec<true, false>), dim3(grid), dim3(1024), lds_bytes, st, pos, crd, vals,
                                   csb, rowmap, Dn, dense_rows, out, sc.nnz, sc.nchunks, scratch, (const int32_t *)nullptr,
                                   (const int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr, ep);
            } else {
                e = allow_full_lds<k_stream_rank1_ldsvec<false, false>>();
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((k_stream_rank1_ldsvec<false, false>), dim3(grid), dim3(1024), lds_bytes, st, pos, crd, vals,
                                   csb, rowmap, Dn, dense_rows, out, sc.nnz, sc.nchunks, scratch, (const int32_t *)nullptr,
                                   (const int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr, ep);
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            return run_fixup(scratch, sc.nchunks, 1, rowmap, out, sc.max_seg_len / kChunk + 2, st, ep);
        }
        if (rowmap)
            hipLaunchKernelGGL(k_stream_rank1<true>, dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals, sb,
                               rowmap, Dn, out, sc.nnz, sc.ntiles, scratch, ep);
        else
            hipLaunchKernelGGL(k_stream_rank1<false>, dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals, sb,
                               rowmap, Dn, out, sc.nnz, sc.ntiles, scratch, ep);
        e = hipGetLastError();
    } else {
        e = stream_segreduce_rankR(sc, pos, crd, vals, rowmap, Dn, (int)R, out, scratch, st, ep);
    }
    if (e != hipSuccess) return e;
    // the rank-R kernel publishes result rows as ids, the rank-1 kernel segment numbers
    return run_fixup(scratch, sc.ntiles, (int)R, R == 1 ? rowmap : nullptr, out, sc.max_seg_len / kTile + 2, st, ep);
}

hipError_t stream_ttv_coo(const Schedule &sc, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                          const double *vals, const double *v, int64_t dense_rows, int32_t *y0, int32_t *y1, double *yv,
                          void *scratch, bool plain, hipStream_t st) {
    if (sc.ntiles <= 0) return hipSuccess;
    // a run of equal (c0, c1) holds at most one nonzero per coordinate of the last mode
    const int64_t max_run = dense_rows;
    const size_t lds_bytes = (size_t)((dense_rows + 1) & ~(int64_t)1) * 8 + 16 * 128 + 16 * 8 + 16 * 4;
    if (sc.chunk_run_base && sc.nchunks >= 16 && lds_bytes <= 160 * 1024 && !plain) {
        const int ncu = current_device_cu_count();
        const int64_t want = (sc.nchunks + 15) / 16;
        const unsigned grid = (unsigned)(want < ncu ? want : ncu);
        hipError_t e = allow_full_lds<k_stream_rank1_ldsvec<false, true>>();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_stream_rank1_ldsvec<false, true>), dim3(grid), dim3(1024), lds_bytes, st,
                           (const int32_t *)nullptr, c2, vals, (const int32_t *)sc.chunk_run_base->ptr,
                           (const int32_t *)nullptr, v, dense_rows, yv, sc.nnz, sc.nchunks, scratch, c0, c1, y0, y1, Epilogue());
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        return run_fixup(scratch, sc.nchunks, 1, nullptr, yv, max_run / kChunk + 2, st);
    }
    hipLaunchKernelGGL(k_stream_rank1_coo, dim3((unsigned)sc.ntiles), dim3(256), 0, st, c0, c1, c2, vals,
                       (const int32_t *)sc.run_base->ptr, v, y0, y1, yv, sc.nnz, sc.ntiles, scratch);
    return run_fixup(scratch, sc.ntiles, 1, nullptr, yv, max_run / kTile + 2, st);
}

}  // namespace comet
