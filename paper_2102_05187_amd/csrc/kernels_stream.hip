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
#include <cstdlib>

#include "stream_kernels.hpp"

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
__device__ __forceinline__ void build_tail_map_from_pos(int32_t *ts, const int32_t *__restrict__ pos,
                                                        const int32_t *__restrict__ rowmap, int64_t tb, int32_t s0,
                                                        int32_t s1, double *__restrict__ out, int R) {
    for (int i = threadIdx.x * 4; i < kTile; i += blockDim.x * 4)
        *reinterpret_cast<int4 *>(ts + i) = make_int4(-1, -1, -1, -1);
    __syncthreads();
    for (int32_t s = s0 + threadIdx.x; s < s1; s += blockDim.x) {
        int32_t b = pos[s], e = pos[s + 1];
        if (e > b) {
            ts[(int64_t)e - 1 - tb] = s;
        } else {
            int64_t row = rowmap ? (int64_t)rowmap[s] : (int64_t)s;
            for (int r = 0; r < R; ++r) out[row * R + r] = 0.0;
        }
    }
    __syncthreads();
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
                                                   Rank1Carry &cy, double *wsum_first, int *wsum_first_id) {
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
            out[row] = p1;
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
                out[row] = value;
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
                                           int *wsum_first_id) {
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
    rank1_process_half<ROWMAP>(h0, xv, tt, wb, nnz, lane, w, rowmap, out, cy, wsum_first, wsum_first_id);
    rank1_gather(h1, x, xv);
#pragma unroll
    for (int b = 0; b < 4; ++b) tt[b] = *reinterpret_cast<const int2 *>(ts + (wb - tb) + 512 + b * 128 + 2 * lane);
    rank1_process_half<ROWMAP>(h1, xv, tt, wb + 512, nnz, lane, w, rowmap, out, cy, wsum_first, wsum_first_id);
    if (lane == 0) { wsum_ht[w] = cy.cf; wsum_open[w] = cy.cv; }
}

// Combine the wavefront summaries of one tile in order and publish the tile summary.
template <bool ROWMAP>
__device__ __forceinline__ void finish_tile_rank1(const int *wsum_ht, const double *wsum_open, const double *wsum_first,
                                                  const int *wsum_first_id, const int32_t *__restrict__ rowmap,
                                                  double *__restrict__ out, CarryView cb, int64_t t) {
    if (threadIdx.x != 0) return;
    int rf = 0, fid = -1;
    double rv = 0.0, tfirst = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        if (wsum_ht[w]) {
            const double value = rv + wsum_first[w];
            if (rf) {
                const int64_t row = ROWMAP ? (int64_t)rowmap[wsum_first_id[w]] : (int64_t)wsum_first_id[w];
                out[row] = value;
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
                                                      void *scratch) {
    __shared__ __attribute__((aligned(16))) int32_t ts[kTile];
    __shared__ int wsum_ht[kWaves], wsum_first_id[kWaves];
    __shared__ double wsum_open[kWaves], wsum_first[kWaves];
    const int64_t t = blockIdx.x;
    const int64_t tb = t * (int64_t)kTile;
    Rank1Half h0;
    rank1_load_half(h0, crd, vals, tb + (int64_t)(threadIdx.x >> 6) * kWaveItems, threadIdx.x & 63, nnz);
    build_tail_map_from_pos(ts, pos, rowmap, tb, seg_begin[t], seg_begin[t + 1], out, 1);
    walk_rank1<ROWMAP>(h0, ts, crd, vals, x, rowmap, out, tb, nnz, wsum_ht, wsum_open, wsum_first, wsum_first_id);
    __syncthreads();
    finish_tile_rank1<ROWMAP>(wsum_ht, wsum_open, wsum_first, wsum_first_id, rowmap, out, carry_view(scratch, ntiles, 1), t);
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
                                                              int32_t *__restrict__ y1) {
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
            unsigned long long hm[kRows], hx[kRows];     // run starts; the same with items past the end counted as starts
            const int runs_before = chunk_begin[c];
            // all coordinate loads of the chunk are issued together; the predecessor of an item comes from the
            // neighbouring lane (wave_shr:1), of lane 0 from the previous row (or the item before the chunk)
            const int64_t inext = cbeg + kChunk;
            int before0 = -2, before1 = -2, after0 = -1, after1 = -1;
            if (cbeg > 0) { before0 = c0[cbeg - 1]; before1 = c1[cbeg - 1]; }
            if (inext < nnz) { after0 = c0[inext]; after1 = c1[inext]; }
            int running = runs_before;
#pragma unroll
            for (int rb = 0; rb < kRows; rb += kBatch) {          // batches of rows keep the register count down
                int a0[kBatch], a1[kBatch];
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    const int64_t i = cbeg + 64 * (rb + q) + lane;
                    a0[q] = i < nnz ? c0[i] : -1;
                    a1[q] = i < nnz ? c1[i] : -1;
                }
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    const int r = rb + q;
                    const int64_t i = cbeg + 64 * r + lane;
                    const int p0 = dpp_i<0x138, 0xf>(before0, a0[q]);
                    const int p1 = dpp_i<0x138, 0xf>(before1, a1[q]);
                    const bool differs = a0[q] != p0 || a1[q] != p1;
                    hm[r] = __ballot(differs && i < nnz);
                    hx[r] = __ballot(differs);
                    before0 = __builtin_amdgcn_readlane(a0[q], 63);
                    before1 = __builtin_amdgcn_readlane(a1[q], 63);
                    if ((hm[r] >> lane) & 1ull) {
                        const int id = running + __popcll(hm[r] & lt_mask);
                        y0[id] = a0[q]; y1[id] = a1[q];
                    }
                    running += __popcll(hm[r]);
                }
            }
            const bool next_head = after0 != before0 || after1 != before1;
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
            // item e ends a run when item e+1 starts one or lies past the end of the list
                const unsigned long long nextbit = r + 1 < kRows ? (hx[r + 1] & 1ull) : (next_head ? 1ull : 0ull);
                const int64_t left = nnz - (cbeg + 64 * r);          // items of this row that exist
                const unsigned long long exist = left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
                const unsigned long long tmask = ((hx[r] >> 1) | (nextbit << 63)) & exist;
                if (lane == 0) *reinterpret_cast<unsigned long long *>(bits + 2 * r) = tmask;
            }
            base_id = runs_before - ((hm[0] & 1ull) ? 0 : 1);        // the run that holds the chunk's first item
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
        rank1_process_half<ROWMAP>(h0, xv, tt, cbeg, nnz, lane, w, rowmap, out, cy, wfirst_all, wfirst_id_all);
        if (c + stride < nchunks) rank1_load_half(h0, crd, vals, (c + stride) * kChunk, lane, nnz);   // next chunk
        gather(h1, xv);
        tails_of_half(1, tt);
        rank1_process_half<ROWMAP>(h1, xv, tt, cbeg + 512, nnz, lane, w, rowmap, out, cy, wfirst_all, wfirst_id_all);
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
                                                      const int32_t *__restrict__ rowmap, double *__restrict__ out) {
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
    out[row * R + r] = v;
}


// ---- rank-R walk: a group of L lanes (4 or 8) walks a run of consecutive items --------------------
// The 256 threads of a tile form 256/L lane groups ("walkers"); walker g owns the 16*L consecutive
// items [tb + 16*L*g, +16*L).  Every 4*L items (a super-block) each lane loads four consecutive
// (crd, val) pairs with 16-byte loads, looks up their tail ids, turns crd into the byte offset of
// the operand row, and writes one small record per item into the walker's private LDS area.  The
// group then takes the items one at a time: every lane reads the current item's record with a
// broadcast LDS read (no cross-lane VALU work), adds its own 16-byte slot, and gathers its share of
// the operand row Dn[crd, :] -- contiguous 16-byte pieces (WIDE, R a multiple of 2L: lane j takes
// ranks 2L*q+2j, 2L*q+2j+1) or 8-byte pieces (lane j takes ranks L*q+j) -- so a load instruction
// reads each gathered row as one contiguous run of 16*L bytes.  Gathers run G steps ahead of the
// FMAs (double-buffered in registers).  Row offsets are 32-bit, so an operand must be < 4 GiB.
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
__device__ __forceinline__ void grp_store_row(double *__restrict__ out, int64_t row, int R, int j, const double *v) {
    double *p = out + row * R;
    if constexpr (WIDE) {
#pragma unroll
        for (int q = 0; q < V / 2; ++q) *reinterpret_cast<double2 *>(p + 2 * L * q + 2 * j) = make_double2(v[2 * q], v[2 * q + 1]);
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) { int r = L * q + j; if (r < R) p[r] = v[q]; }
    }
}

// The same for a result row that this kernel does not read again: non-temporal stores.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_store_row_stream(double *__restrict__ out, int64_t row, int R, int j, const double *v) {
    double *p = out + row * R;
    if constexpr (WIDE) {
        typedef double v2d __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            v2d x; x.x = v[2 * q]; x.y = v[2 * q + 1];
            __builtin_nontemporal_store(x, reinterpret_cast<v2d *>(p + 2 * L * q + 2 * j));
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) { int r = L * q + j; if (r < R) __builtin_nontemporal_store(v[q], p + r); }
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

// This lane's share of the dense row that starts `off` bytes into Dn (off already includes the
// lane's own slot).
template <int L, int V, bool WIDE>
__device__ __forceinline__ void grp_load_row_off(const double *__restrict__ Dn, unsigned off, int R, int j, double *d) {
    const char *base = reinterpret_cast<const char *>(Dn);
    if constexpr (WIDE) {
#pragma unroll
        for (int q = 0; q < V / 2; ++q) {
            const double2 x = *reinterpret_cast<const double2 *>(base + (size_t)(off + (unsigned)(16 * L * q)));
            d[2 * q] = x.x; d[2 * q + 1] = x.y;
        }
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) {
            d[q] = L * q + j < R ? *reinterpret_cast<const double *>(base + (size_t)(off + (unsigned)(8 * L * q))) : 0.0;
        }
    }
}
template <int L, bool WIDE>
__device__ __forceinline__ unsigned lane_slot_bytes(int j) { return WIDE ? 16u * j : 8u * j; }

// Close the first segment end of every walker of the tile and publish the tile summary.
// wopen[(g*L + j)*V + q] holds walker g's open sum, wht[g] its has_tail flag (both already written
// and separated from this call by a barrier).  `first_row` is the output row of the walker's first
// segment end; `open` its trailing sum.
template <int L, int V, bool WIDE>
__device__ __forceinline__ void finish_tile_walkers(const double *wopen, const int *wht, int g, int j, int ht,
                                                    const double *first, int64_t first_row, int32_t first_id,
                                                    const double *open, double *__restrict__ out, int R,
                                                    CarryView cb, int64_t t) {
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
            grp_store_row<L, V, WIDE>(out, first_row, R, j, value);
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

template <int L, int V, bool WIDE, bool ROWMAP>
__global__ void __launch_bounds__(256) k_stream_rankR(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                      const double *__restrict__ vals,
                                                      const int32_t *__restrict__ seg_begin,
                                                      const int32_t *__restrict__ rowmap, const double *__restrict__ Dn,
                                                      double *__restrict__ out, int64_t nnz, int64_t ntiles, int R,
                                                      void *scratch) {
    constexpr int NW = 256 / L;                // walkers per tile
    constexpr int WI = kTile / NW;             // items per walker
    using RL = RecLayout<L, 2>;                // record = {row byte offset, tail id} + value
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
    build_tail_map_from_pos(ts, pos, rowmap, tb, seg_begin[t], seg_begin[t + 1], out, R);

    WalkState<V> st;
#pragma unroll
    for (int q = 0; q < V; ++q) { st.acc[q] = 0.0; st.first[q] = 0.0; }
    st.ht = 0; st.first_id = -1;
    int32_t *rec = rec_all + g * RL::kStride;
    const unsigned R8 = 8u * (unsigned)R;
    const unsigned slot = lane_slot_bytes<L, WIDE>(j);
    char *outb = reinterpret_cast<char *>(out);

    constexpr int G = StepGroup<V>::value, NG = SB / G;
    for (int sb = 0; sb < WI / SB; ++sb) {
        const int64_t i0 = gb + SB * sb + 4 * j;                  // this lane's four items
        LaneItems nxt;
        if (sb + 1 < WI / SB) lane_load_items(nxt, crd, vals, i0 + SB, nnz);
        {
            const int4 t4 = *reinterpret_cast<const int4 *>(ts + (i0 - tb));
            *reinterpret_cast<int4 *>(rec + 8 * j) =
                make_int4((int)((unsigned)cur.cr[0] * R8), t4.x, (int)((unsigned)cur.cr[1] * R8), t4.y);
            *reinterpret_cast<int4 *>(rec + 8 * j + 4) =
                make_int4((int)((unsigned)cur.cr[2] * R8), t4.z, (int)((unsigned)cur.cr[3] * R8), t4.w);
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
                        const unsigned row = ROWMAP ? (unsigned)rowmap[b.tail] : (unsigned)b.tail;
                        grp_store_row_stream<L, V, WIDE>(reinterpret_cast<double *>(outb + (size_t)row * R8), 0, R, j, st.acc);
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
    const int64_t first_row = st.ht ? (ROWMAP ? (int64_t)rowmap[st.first_id] : (int64_t)st.first_id) : 0;
    finish_tile_walkers<L, V, WIDE>(wopen, wht, g, j, st.ht, st.first, first_row, st.first_id, st.acc, out, R,
                                    carry_view(scratch, ntiles, R), t);
}

template <int L, int V, bool WIDE>
hipError_t launch_rankR(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                        const int32_t *rowmap, const double *Dn, int R, double *out, void *scratch, hipStream_t st) {
    if (rowmap)
        hipLaunchKernelGGL((k_stream_rankR<L, V, WIDE, true>), dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals,
                           (const int32_t *)sc.seg_begin->ptr, rowmap, Dn, out, sc.nnz, sc.ntiles, R, scratch);
    else
        hipLaunchKernelGGL((k_stream_rankR<L, V, WIDE, false>), dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals,
                           (const int32_t *)sc.seg_begin->ptr, rowmap, Dn, out, sc.nnz, sc.ntiles, R, scratch);
    return hipGetLastError();
}

// Cross-lane broadcast inside a lane group (quad_perm inside a quad, plus one row_shr:4 / row_shl:4 with a
// bank mask to cross the two quads of an 8-lane group); used by the MTTKRP walk, whose LDS budget goes
// to its two tail maps.
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

// ---- MTTKRP: the same walk, two nested segment levels ---------------------------------------------
// Inner level: fibers (segments of pos3); the per-fiber sum of vals * C[crd3, :] is scaled by the row
// B[crd2[fiber], :] when the fiber ends and folded into the slice accumulator.  Scaling is linear,
// so a fiber cut by a walker or tile boundary is folded piecewise (each piece times the same B row);
// only the slice level needs carries.  Outer level: slices (segments of pos2); a slice end writes
// row crd1[slice] of M.  Two LDS maps, both keyed by tile item: ts = fiber id at a fiber's last
// nonzero, tm = output row at a slice's last nonzero (-1 elsewhere).
template <int L, int V, bool WIDE>
__global__ void __launch_bounds__(256) k_stream_mttkrp(const int32_t *__restrict__ pos2, const int32_t *__restrict__ crd1,
                                                       const int32_t *__restrict__ pos3, const int32_t *__restrict__ crd2,
                                                       const int32_t *__restrict__ crd3, const double *__restrict__ vals,
                                                       const int32_t *__restrict__ seg_begin,
                                                       const int32_t *__restrict__ slice_begin,
                                                       const double *__restrict__ Bm, const double *__restrict__ Cm,
                                                       double *__restrict__ M, int64_t nnz, int64_t nfib, int64_t ntiles,
                                                       int R, void *scratch) {
    constexpr int NW = 256 / L, WI = kTile / NW, SB = 4 * L;
    constexpr int kMapInts = 2 * kTile;
    constexpr int kOpenInts = 256 * V * 2;
    constexpr int kLdsInts = kMapInts > kOpenInts ? kMapInts : kOpenInts;
    __shared__ __attribute__((aligned(16))) int32_t lds[kLdsInts];
    __shared__ int wht[NW], wfirst_fid[NW];
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
        if (e > b) ts[(int64_t)e - 1 - tb] = f;
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
            for (int r = 0; r < R; ++r) row[r] = 0.0;
        }
    }
    __syncthreads();

    double facc[V], sacc[V], first[V];
#pragma unroll
    for (int q = 0; q < V; ++q) { facc[q] = 0.0; sacc[q] = 0.0; first[q] = 0.0; }
    int ht = 0, first_row = -1, first_fid = -1, last_is_tail = 1;

    constexpr int G = StepGroup<V>::value, NG = SB / G;
    for (int sb = 0; sb < WI / SB; ++sb) {
        const int64_t i0 = gb + SB * sb + 4 * j;
        LaneItems nxt;
        if (sb + 1 < WI / SB) lane_load_items(nxt, crd3, vals, i0 + SB, nnz);
        int tl[4], tr[4], jb[4];
        {
            const int4 t4 = *reinterpret_cast<const int4 *>(ts + (i0 - tb));
            const int4 m4 = *reinterpret_cast<const int4 *>(tm + (i0 - tb));
            tl[0] = t4.x; tl[1] = t4.y; tl[2] = t4.z; tl[3] = t4.w;
            tr[0] = m4.x; tr[1] = m4.y; tr[2] = m4.z; tr[3] = m4.w;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) jb[s] = tl[s] >= 0 ? crd2[tl[s]] : 0;      // B row of a fiber that ends here
        const bool any_item = gb + SB * sb < nnz;
        RowBuf<V> cbuf[2][G], bbuf[2][G];
        auto issue = [&](auto gc, RowBuf<V> *cb_, RowBuf<V> *bb_) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;
                constexpr int s_ = decltype(sc)::value;
                const int c = grp_bcast_i<L, k / 4>(cur.cr[k % 4]);
                grp_load_row<L, V, WIDE>(Cm, c, R, j, cb_[s_].d);
                const int tf = grp_bcast_i<L, k / 4>(tl[k % 4]);
                if (tf >= 0) {                                    // the fiber ends here: its B row is needed too
                    const int jrow = grp_bcast_i<L, k / 4>(jb[k % 4]);
                    grp_load_row<L, V, WIDE>(Bm, jrow, R, j, bb_[s_].d);
                }
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
                    if (first_fid < 0) first_fid = tf;
#pragma unroll
                    for (int q = 0; q < V; ++q) { sacc[q] = fma(bb_[s_].d[q], facc[q], sacc[q]); facc[q] = 0.0; }
                    if (tmr >= 0) {
                        if (!ht) {
#pragma unroll
                            for (int q = 0; q < V; ++q) first[q] = sacc[q];
                            first_row = tmr; ht = 1;
                        } else {
                            grp_store_row<L, V, WIDE>(M, tmr, R, j, sacc);
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
    if (j == 0) wfirst_fid[g] = first_fid;
    __syncthreads();                                              // also: every walk is done, the maps are dead
    if (!last_is_tail) {
        int64_t fid = seg_begin[t + 1];
        for (int g2 = g + 1; g2 < NW; ++g2) { int f2 = wfirst_fid[g2]; if (f2 >= 0) { fid = f2; break; } }
        if (fid < nfib) {
            double bw[V];
            grp_load_row<L, V, WIDE>(Bm, crd2[fid], R, j, bw);
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
                                    carry_view(scratch, ntiles, R), t);
}

template <int L, int V, bool WIDE>
hipError_t launch_mttkrp(const Schedule &sc, const int32_t *pos2, const int32_t *crd1, const int32_t *pos3,
                         const int32_t *crd2, const int32_t *crd3, const double *vals, const double *B, const double *C,
                         int R, double *M, void *scratch, hipStream_t st) {
    hipLaunchKernelGGL((k_stream_mttkrp<L, V, WIDE>), dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos2, crd1, pos3, crd2,
                       crd3, vals, (const int32_t *)sc.seg_begin->ptr, (const int32_t *)sc.slice_begin->ptr, B, C, M,
                       sc.nnz, sc.nseg, sc.ntiles, R, scratch);
    return hipGetLastError();
}

// One pass of the hierarchical fix-up: thread (g, r) folds the kFixGroup summaries of group g in
// order.  A segment end whose carry chain starts inside the group is final and is written to out;
// the group's own summary (first segment end, trailing open sum) goes one level up.
__global__ void __launch_bounds__(256) k_fixup_level(const double *__restrict__ lo_first, const double *__restrict__ lo_open,
                                                     const int32_t *__restrict__ lo_ht, const int32_t *__restrict__ lo_id,
                                                     int64_t n_lo, double *__restrict__ up_first,
                                                     double *__restrict__ up_open, int32_t *__restrict__ up_ht,
                                                     int32_t *__restrict__ up_id, int64_t n_up, int R,
                                                     const int32_t *__restrict__ rowmap, double *__restrict__ out) {
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
                    out[row * R + r] = value;
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

// Finish every segment that a tile boundary cut: fold the tile summaries level by level, then
// walk the few top-level summaries serially.  `max_chain` bounds the number of consecutive tiles
// one segment can span (0 = unknown); short chains go straight to the serial walk.
hipError_t run_fixup(void *scratch, int64_t ntiles, int R, const int32_t *rowmap, double *out, int64_t max_chain,
                     hipStream_t st) {
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
                           lo.has_tail, lo.first_id, n, up.first, up.open, up.has_tail, up.first_id, n_up, R, rowmap, out);
        base = up_base;
        n = n_up;
    }
    const int64_t threads = n * R;
    hipLaunchKernelGGL(k_stream_fixup, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (void *)base, n, R,
                       rowmap, out);
    return hipGetLastError();
}

}  // namespace

// Allows a kernel to use up to the whole 160 KB of LDS as dynamic shared memory; done once per kernel
// (it is not a stream operation, but calling it once keeps it out of captured regions after the first call).
template <auto Kernel>
static hipError_t allow_full_lds() {
    static hipError_t status = hipFuncSetAttribute((const void *)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return status;
}

// Lane-group width of the rank-R kernels: 8 by default; COMET_LANES=4 selects the quad mapping
// (for measurements).  Ranks up to 8 always use quads.
static int lanes_per_item(int64_t R) {
    static int forced = [] { const char *e = getenv("COMET_LANES"); return e ? atoi(e) : 0; }();
    if (R <= 8) return 4;
    if (forced == 4 && R <= 64) return 4;
    return 8;
}

// COMET_NO_LDS_VECTOR=1 keeps rank-1 operations on the L1-gather kernel (for measurements).
static bool no_lds_vector() {
    static int v = [] { const char *e = getenv("COMET_NO_LDS_VECTOR"); return e ? atoi(e) : 0; }();
    return v != 0;
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

// Calls F<L, V, WIDE>(args...) for the specialisation that covers rank R.
#define COMET_DISPATCH_RANK(F, R, ...)                                                     \
    [&]() -> hipError_t {                                                                  \
        const int r_ = (int)(R);                                                           \
        if (lanes_per_item(r_) == 4) {                                                     \
            if (r_ == 8)  return F<4, 2, true>(__VA_ARGS__);                               \
            if (r_ == 16) return F<4, 4, true>(__VA_ARGS__);                               \
            if (r_ == 32) return F<4, 8, true>(__VA_ARGS__);                               \
            if (r_ == 64) return F<4, 16, true>(__VA_ARGS__);                              \
            if (r_ <= 4)  return F<4, 1, false>(__VA_ARGS__);                              \
            if (r_ <= 8)  return F<4, 2, false>(__VA_ARGS__);                              \
            if (r_ <= 16) return F<4, 4, false>(__VA_ARGS__);                              \
            if (r_ <= 32) return F<4, 8, false>(__VA_ARGS__);                              \
            return F<4, 16, false>(__VA_ARGS__);                                           \
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

hipError_t stream_segreduce(const Schedule &sc, const int32_t *pos, const int32_t *crd, const double *vals,
                            const int32_t *rowmap, const double *Dn, int64_t dense_rows, int64_t R, double *out,
                            void *scratch, hipStream_t st) {
    if (sc.ntiles <= 0) return hipSuccess;
    if (!stream_supports_rank(R)) return hipErrorNotSupported;
    const int32_t *sb = (const int32_t *)sc.seg_begin->ptr;
    hipError_t e = hipSuccess;
    if (R == 1) {
        const size_t lds_bytes = (size_t)((dense_rows + 1) & ~(int64_t)1) * 8 + 16 * 128 + 16 * 8 + 16 * 4;
        if (sc.empty_segments == 0 && sc.chunk_seg_begin && sc.nchunks >= 16 && lds_bytes <= 160 * 1024 && !no_lds_vector()) {
            // the dense vector fits in LDS and every segment holds a nonzero: wavefront-per-chunk kernel
            static int ncu = [] { hipDeviceProp_t p; return hipGetDeviceProperties(&p, 0) == hipSuccess ? p.multiProcessorCount : 256; }();
            const int64_t want = (sc.nchunks + 15) / 16;
            const unsigned grid = (unsigned)(want < ncu ? want : ncu);
            const int32_t *csb = (const int32_t *)sc.chunk_seg_begin->ptr;
            if (rowmap) {
                e = allow_full_lds<k_stream_rank1_ldsvec<true, false>>();
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((k_stream_rank1_ldsvec<true, false>), dim3(grid), dim3(1024), lds_bytes, st, pos, crd, vals,
                                   csb, rowmap, Dn, dense_rows, out, sc.nnz, sc.nchunks, scratch, (const int32_t *)nullptr,
                                   (const int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr);
            } else {
                e = allow_full_lds<k_stream_rank1_ldsvec<false, false>>();
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL((k_stream_rank1_ldsvec<false, false>), dim3(grid), dim3(1024), lds_bytes, st, pos, crd, vals,
                                   csb, rowmap, Dn, dense_rows, out, sc.nnz, sc.nchunks, scratch, (const int32_t *)nullptr,
                                   (const int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr);
            }
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            return run_fixup(scratch, sc.nchunks, 1, rowmap, out, sc.max_seg_len / kChunk + 2, st);
        }
        if (rowmap)
            hipLaunchKernelGGL(k_stream_rank1<true>, dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals, sb,
                               rowmap, Dn, out, sc.nnz, sc.ntiles, scratch);
        else
            hipLaunchKernelGGL(k_stream_rank1<false>, dim3((unsigned)sc.ntiles), dim3(256), 0, st, pos, crd, vals, sb,
                               rowmap, Dn, out, sc.nnz, sc.ntiles, scratch);
        e = hipGetLastError();
    } else {
        e = COMET_DISPATCH_RANK(launch_rankR, R, sc, pos, crd, vals, rowmap, Dn, (int)R, out, scratch, st);
    }
    if (e != hipSuccess) return e;
    return run_fixup(scratch, sc.ntiles, (int)R, rowmap, out, sc.max_seg_len / kTile + 2, st);
}

hipError_t stream_ttv_coo(const Schedule &sc, const int32_t *c0, const int32_t *c1, const int32_t *c2,
                          const double *vals, const double *v, int64_t dense_rows, int32_t *y0, int32_t *y1, double *yv,
                          void *scratch, hipStream_t st) {
    if (sc.ntiles <= 0) return hipSuccess;
    // a run of equal (c0, c1) holds at most one nonzero per coordinate of the last mode
    const int64_t max_run = dense_rows;
    const size_t lds_bytes = (size_t)((dense_rows + 1) & ~(int64_t)1) * 8 + 16 * 128 + 16 * 8 + 16 * 4;
    if (sc.chunk_run_base && sc.nchunks >= 16 && lds_bytes <= 160 * 1024 && !no_lds_vector()) {
        static int ncu = [] { hipDeviceProp_t p; return hipGetDeviceProperties(&p, 0) == hipSuccess ? p.multiProcessorCount : 256; }();
        const int64_t want = (sc.nchunks + 15) / 16;
        const unsigned grid = (unsigned)(want < ncu ? want : ncu);
        hipError_t e = allow_full_lds<k_stream_rank1_ldsvec<false, true>>();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_stream_rank1_ldsvec<false, true>), dim3(grid), dim3(1024), lds_bytes, st,
                           (const int32_t *)nullptr, c2, vals, (const int32_t *)sc.chunk_run_base->ptr,
                           (const int32_t *)nullptr, v, dense_rows, yv, sc.nnz, sc.nchunks, scratch, c0, c1, y0, y1);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        return run_fixup(scratch, sc.nchunks, 1, nullptr, yv, max_run / kChunk + 2, st);
    }
    hipLaunchKernelGGL(k_stream_rank1_coo, dim3((unsigned)sc.ntiles), dim3(256), 0, st, c0, c1, c2, vals,
                       (const int32_t *)sc.run_base->ptr, v, y0, y1, yv, sc.nnz, sc.ntiles, scratch);
    return run_fixup(scratch, sc.ntiles, 1, nullptr, yv, max_run / kTile + 2, st);
}

hipError_t stream_mttkrp(const Schedule &sc, const int32_t *pos2, const int32_t *crd1, int64_t nslice,
                         const int32_t *pos3, const int32_t *crd2, const int32_t *crd3, const double *vals,
                         const double *B, const double *C, int64_t R, double *M, void *scratch, hipStream_t st) {
    (void)nslice;
    if (sc.ntiles <= 0) return hipSuccess;
    if (!stream_mttkrp_supports_rank(R) || !sc.slice_begin) return hipErrorNotSupported;
    const int r = (int)R;
    hipError_t e = COMET_DISPATCH_RANK(launch_mttkrp, R, sc, pos2, crd1, pos3, crd2, crd3, vals, B, C, r, M, scratch, st);
    if (e != hipSuccess) return e;
    return run_fixup(scratch, sc.ntiles, r, nullptr, M, sc.max_parent_len > 0 ? sc.max_parent_len / kTile + 2 : 0, st);
}

}  // namespace comet
