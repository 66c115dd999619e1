// The two sweeps that take the long segments of a power-law tensor out of the nonzero-tiled kernels' hands,
// and the compacted copy of all other segments that those kernels then walk:
//   - the heavy-row sweep of SpMM (this comment; kernels k_heavy_sweep, k_heavy_reduce),
//   - the heavy-fiber sweep of TTM (second half of the file; k_fiber_sweep, k_fiber_reduce),
//   - light_copy_build (the copy; see LightCopy in tensor.hpp).
//
// Heavy-row sweep of SpMM: the long rows of a power-law matrix, processed so that the rows of the dense
// operand they gather are shared through the L2 caches instead of being fetched from memory once per nonzero.
//
// With uniformly scattered columns every gather of a row of B (R * 8 bytes) misses the caches when the rows
// of A are walked one after the other: B is far larger than any cache.  But the few long rows hold most of
// the nonzeros (the paper's load-imbalance discussion, Section 8.3, is about exactly these rows), and all of
// them touch the same columns.  So the columns are cut into windows of kWindow (a window's rows of B fit
// the 4 MB L2 of one XCD several times over), the windows are dealt to the eight XCDs in contiguous ranges,
// and on each XCD all heavy rows are walked window by window at the same pace: a row of B is fetched from
// memory once per sweep and then hit in L2 by every other heavy row with a nonzero in that column.
// Workgroups are placed on the XCDs round-robin, so workgroup b sweeps the window range of XCD b mod 8 (were
// the placement different only the cache reuse would suffer).
//
// A heavy row is cut into units of comparable length (a unit takes the q-th of nsplit equal pieces of the
// row's nonzeros inside every window); every lane group (8 lanes) owns a few units, dealt longest first and
// back and forth so that all groups carry about the same number of nonzeros, and keeps their running sums
// in LDS.  What a group has to do is then a fixed sequence: window by window, unit by unit, nonzero by
// nonzero.  That sequence is laid out once, when the tensor is created, as a stream per wavefront: the 8
// groups of a wavefront advance in lockstep, so every window is padded for each group to the longest of the
// 8 (padding items are skipped without a gather), and a wavefront reads its stream with fully coalesced
// 16-byte loads, 32 positions x 8 groups at a time.  At run time a group is a plain walker over its stream --
// rows of B gathered a few positions ahead of the multiply-adds, a sum flushed into LDS where a unit's piece
// ends -- and the 16 wavefronts of a compute unit meet at a barrier where a window ends (no data is
// exchanged there; it only keeps them on the same rows of B).  Each (unit, XCD) pair yields one partial row;
// a second kernel adds the partial rows of a heavy row in a fixed order (no atomics anywhere: results are
// reproducible run to run).
#include <algorithm>
#include <atomic>
#include <vector>

#include "stream_common.hpp"

namespace comet {

namespace {

constexpr int kXcd = 8;              // XCDs of the device = number of column ranges
constexpr int kWindow = 4096;        // columns per window
constexpr int kHeavyLen = 128;       // a row with at least this many nonzeros is heavy
constexpr int kUnitLen = 4096;       // target nonzeros per unit
constexpr int kHeavyThreads = 1024;  // one workgroup fills a compute unit: 16 wavefronts, 128 lane groups of 8 lanes
constexpr int kHeavyGroups = kHeavyThreads / 8;
constexpr int kSlots = 32;           // workgroups per column range (= compute units of an XCD)
constexpr int kWaves = kSlots * (kHeavyThreads / 64);      // wavefronts per column range
constexpr int kGroupSlots = kSlots * kHeavyGroups;         // lane groups per column range
constexpr int kMaxUnitsPerGroup = 4;
constexpr int kBlock = 32;           // stream positions per lane group in one super-block (4 per lane)
constexpr int kSync = 4;             // windows between two points where the groups of a wavefront (and the wavefronts of a
                                     // compute unit) line up again: padding and barriers cost less, and within such an
                                     // interval the groups stay within a window or two of each other anyway
constexpr int32_t kNoFlush = -1, kSkip = -2;               // stream item codes (>= 0: flush into that unit slot)

__global__ void __launch_bounds__(256) k_count_heavy(const int32_t *__restrict__ pos, int64_t nseg, int32_t min_len,
                                                     unsigned long long *__restrict__ count_and_nnz) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int len = 0;
    if (s < nseg) len = pos[s + 1] - pos[s];
    const bool heavy = len >= min_len;
    const unsigned long long b = __ballot(heavy);
    long long sum = heavy ? len : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if ((threadIdx.x & 63) == 0 && b) {
        atomicAdd(&count_and_nnz[0], (unsigned long long)__popcll(b));
        atomicAdd(&count_and_nnz[1], (unsigned long long)sum);
    }
}

// list[k] = (segment, length) of the heavy segments, in no particular order (the host sorts them)
__global__ void __launch_bounds__(256) k_collect_heavy(const int32_t *__restrict__ pos, int64_t nseg, int32_t min_len,
                                                       unsigned long long *__restrict__ cursor, int2 *__restrict__ list,
                                                       int64_t cap) {
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= nseg) return;
    const int len = pos[s + 1] - pos[s];
    if (len < min_len) return;
    const unsigned long long k = atomicAdd(cursor, 1ull);
    if ((int64_t)k < cap) list[k] = make_int2((int)s, len);
}

// wstart[h][w] = first position of heavy row h whose column is >= w * window (w = nwin: the row's end)
__global__ void __launch_bounds__(256) k_build_wstart(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                      const int32_t *__restrict__ hseg, int64_t nheavy, int nwin,
                                                      int window, int32_t *__restrict__ wstart) {
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per = nwin + 1;
    if (g >= nheavy * per) return;
    const int64_t h = g / per;
    const int w = (int)(g - h * per);
    const int s = hseg[h];
    int lo = pos[s], hi = pos[s + 1];
    if (w < nwin) {
        const long long target = (long long)w * window;
        while (lo < hi) {                                  // first position with crd >= target
            const int mid = lo + ((hi - lo) >> 1);
            if ((long long)crd[mid] < target) lo = mid + 1; else hi = mid;
        }
    } else {
        lo = hi;
    }
    wstart[g] = lo;
}

// flags[f] = (length << 32) | 1 for a light segment, 0 for a heavy one: one exclusive scan then gives every light
// segment its row number (low half) and the position of its first nonzero in the copy (high half)
__global__ void __launch_bounds__(256) k_light_flags(const int32_t *__restrict__ pos, int64_t nseg, int32_t min_len,
                                                     uint64_t *__restrict__ flags) {
    const int64_t f = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= nseg) return;
    const int len = pos[f + 1] - pos[f];
    flags[f] = len < min_len ? (((uint64_t)(uint32_t)len << 32) | 1u) : 0u;
}

// 8 lanes copy the nonzeros of one light segment; its result row is rowmap[segment] if there is a map
__global__ void __launch_bounds__(256) k_light_copy(const int32_t *__restrict__ pos, const int32_t *__restrict__ crd,
                                                    const double *__restrict__ vals, int64_t nseg, int32_t min_len,
                                                    const uint64_t *__restrict__ before,
                                                    const int32_t *__restrict__ rowmap, int32_t *__restrict__ lrows,
                                                    int32_t *__restrict__ lpos, int32_t *__restrict__ lcrd,
                                                    double *__restrict__ lvals) {
    const int64_t f = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 3;
    const int j = threadIdx.x & 7;
    if (f >= nseg) return;
    const int b = pos[f], len = pos[f + 1] - b;
    if (len >= min_len) return;
    const uint64_t w = before[f];
    const int64_t r = (int64_t)(w & 0xffffffffu), p0 = (int64_t)(w >> 32);
    if (j == 0) { lrows[r] = rowmap ? rowmap[f] : (int32_t)f; lpos[r] = (int32_t)p0; }
    for (int i = j; i < len; i += 8) { lcrd[p0 + i] = crd[b + i]; lvals[p0 + i] = vals[b + i]; }
}


// Copies the segments of fewer than min_len nonzeros out (see LightCopy); nlight / light_nnz are their counts.
hipError_t light_copy_build(const int32_t *pos, int64_t nseg, const int32_t *crd, const double *vals, int32_t min_len,
                            const int32_t *rowmap, int64_t nlight, int64_t light_nnz, LightCopy &lc, hipStream_t st) {
    lc = LightCopy();
    DevRef flags = dev_alloc(sizeof(uint64_t) * nseg), before = dev_alloc(sizeof(uint64_t) * nseg);
    lc.root = dev_alloc(2 * sizeof(int32_t));
    lc.rows = dev_alloc(sizeof(int32_t) * nlight);
    lc.pos = dev_alloc(sizeof(int32_t) * (nlight + 1));
    lc.crd = dev_alloc(sizeof(int32_t) * light_nnz);
    lc.vals = dev_alloc(sizeof(double) * light_nnz);
    if (!flags || !before || !lc.root || !lc.rows || !lc.pos || !lc.crd || !lc.vals) { lc = LightCopy(); return hipErrorOutOfMemory; }
    const unsigned grid = (unsigned)((nseg + 255) / 256);
    hipLaunchKernelGGL(k_light_flags, dim3(grid), dim3(256), 0, st, pos, nseg, min_len, (uint64_t *)flags->ptr);
    size_t temp_bytes = 0;
    hipError_t e = reorder_scan_flags(nullptr, &temp_bytes, (const uint64_t *)flags->ptr, (uint64_t *)before->ptr, nseg, st);
    if (e != hipSuccess) { lc = LightCopy(); return e; }
    DevRef temp = dev_alloc(temp_bytes ? temp_bytes : 16);
    if (!temp) { lc = LightCopy(); return hipErrorOutOfMemory; }
    e = reorder_scan_flags(temp->ptr, &temp_bytes, (const uint64_t *)flags->ptr, (uint64_t *)before->ptr, nseg, st);
    if (e != hipSuccess) { lc = LightCopy(); return e; }
    hipLaunchKernelGGL(k_light_copy, dim3((unsigned)((nseg * 8 + 255) / 256)), dim3(256), 0, st, pos, crd, vals, nseg, min_len,
                       (const uint64_t *)before->ptr, rowmap, (int32_t *)lc.rows->ptr, (int32_t *)lc.pos->ptr,
                       (int32_t *)lc.crd->ptr, (double *)lc.vals->ptr);
    const int32_t root[2] = {0, (int32_t)nlight}, last = (int32_t)light_nnz;
    e = hipMemcpyAsync(lc.root->ptr, root, sizeof root, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync((int32_t *)lc.pos->ptr + nlight, &last, sizeof last, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);                     // host values and temporaries go out of scope
    if (e != hipSuccess) { lc = LightCopy(); return e; }
    lc.nrows = nlight; lc.nnz = light_nnz;
    return hipGetLastError();
}

// ---- laying out the streams (once per tensor) ------------------------------------------------------------
// Unit of lane-group slot gs (0 .. kGroupSlots-1) in round k: units come longest first and are dealt back and forth.
__device__ __host__ inline int unit_of_slot(int gs, int k) { return k * kGroupSlots + ((k & 1) ? kGroupSlots - 1 - gs : gs); }
// Lane-group slot of group gl (0..7) of wavefront wv (0 .. kWaves-1): consecutive slots go to different workgroups.
__device__ __host__ inline int slot_of_group(int wv, int gl) {
    const int wg = wv / (kHeavyThreads / 64), g = (wv % (kHeavyThreads / 64)) * 8 + gl;
    return g * kSlots + wg;
}
// Positions [lo, hi) of unit u's piece inside window w (absolute window number).
__device__ inline void piece_of(const int4 *__restrict__ units, const int32_t *__restrict__ wstart, int nwin, int u, int w,
                                int *lo, int *hi) {
    const int4 un = units[u];
    const int64_t row = (int64_t)un.x * (nwin + 1);
    const int a = wstart[row + w], e = wstart[row + w + 1];
    const int n = e - a;                                              // at most kWindow
    *lo = a + n * un.y / un.z;
    *hi = a + n * (un.y + 1) / un.z;
}

// wmax[(x * kWaves + wv) * nsx + i] = positions wavefront wv of range x needs for its i-th interval of kSync
// windows: the most nonzeros any of its 8 groups has there
__global__ void __launch_bounds__(256) k_window_lengths(const int4 *__restrict__ units, int nunits, int nu,
                                                        const int32_t *__restrict__ wstart, int nwin, int nwx, int nsx,
                                                        int32_t *__restrict__ wmax) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)kXcd * kWaves * nsx) return;
    const int iv = (int)(t % nsx), wv = (int)((t / nsx) % kWaves), x = (int)(t / ((int64_t)nsx * kWaves));
    int m = 0;
    for (int gl = 0; gl < 8; ++gl) {
        const int gs = slot_of_group(wv, gl);
        int total = 0;
        for (int w = iv * kSync; w < (iv + 1) * kSync && w < nwx; ++w) {
            const int wabs = x * nwx + w;
            if (wabs >= nwin) break;
            for (int k = 0; k < nu; ++k) {
                const int u = unit_of_slot(gs, k);
                if (u >= nunits) continue;
                int lo, hi;
                piece_of(units, wstart, nwin, u, wabs, &lo, &hi);
                total += hi - lo;
            }
        }
        m = total > m ? total : m;
    }
    wmax[t] = m;
}

// wend[(x * kWaves + wv) * (nsx + 1) + i] = first position of interval i (last entry: all positions);
// nblocks[x * kWaves + wv] = super-blocks of kBlock positions the wavefront's stream takes
__global__ void __launch_bounds__(256) k_window_ends(const int32_t *__restrict__ wmax, int nwx, int32_t *__restrict__ wend,
                                                     int32_t *__restrict__ nblocks) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= kXcd * kWaves) return;
    int p = 0;
    for (int w = 0; w < nwx; ++w) { wend[(int64_t)t * (nwx + 1) + w] = p; p += wmax[(int64_t)t * nwx + w]; }
    wend[(int64_t)t * (nwx + 1) + nwx] = p;
    nblocks[t] = (p + kBlock - 1) / kBlock;
}

// One thread per (range, wavefront, interval, group): writes that group's positions of that interval -- window by
// window, unit by unit -- and pads them to the interval's length.
__global__ void __launch_bounds__(256) k_fill_streams(const int32_t *__restrict__ crd, const double *__restrict__ vals,
                                                      const int4 *__restrict__ units, int nunits, int nu,
                                                      const int32_t *__restrict__ wstart, int nwin, int nwx, int nsx,
                                                      const int32_t *__restrict__ wend, const int32_t *__restrict__ block_start,
                                                      int32_t *__restrict__ scrd, int32_t *__restrict__ scode,
                                                      double *__restrict__ sval) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)kXcd * kWaves * nsx * 8) return;
    const int gl = (int)(t % 8), iv = (int)((t / 8) % nsx), wv = (int)((t / (8 * (int64_t)nsx)) % kWaves),
              x = (int)(t / (8 * (int64_t)nsx * kWaves));
    const int wave = x * kWaves + wv;
    const int32_t *we = wend + (int64_t)wave * (nsx + 1);
    const int64_t base = (int64_t)block_start[wave] * (8 * kBlock) + gl * kBlock;
    auto put = [&](int p, int c, int code, double v) {
        const int64_t i = base + (int64_t)(p / kBlock) * (8 * kBlock) + (p % kBlock);
        scrd[i] = c; scode[i] = code; sval[i] = v;
    };
    int p = we[iv];
    const int gs = slot_of_group(wv, gl);
    for (int w = iv * kSync; w < (iv + 1) * kSync && w < nwx; ++w) {
        const int wabs = x * nwx + w;
        if (wabs >= nwin) break;
        for (int k = 0; k < nu; ++k) {
            const int u = unit_of_slot(gs, k);
            if (u >= nunits) continue;
            int lo, hi;
            piece_of(units, wstart, nwin, u, wabs, &lo, &hi);
            for (int i = lo; i < hi; ++i, ++p) put(p, crd[i], i + 1 == hi ? k : kNoFlush, vals[i]);
        }
    }
    int pend = we[iv + 1];
    if (iv == nsx - 1) pend = (block_start[wave + 1] - block_start[wave]) * kBlock;   // and the padding behind the last interval
    for (; p < pend; ++p) put(p, 0, kSkip, 0.0);
}

// ---- the sweep -------------------------------------------------------------------------------------------
// Lane j of a group holds ranks 16 q + 2 j, 16 q + 2 j + 1 of a row (q < V / 2): one load instruction reads a
// whole 128-byte line of a gathered row per lane group.  In a super-block lane j holds stream positions
// 4 j .. 4 j + 3 of its group and hands them to the group one at a time with DPP broadcasts.
template <int V>
__global__ void __launch_bounds__(kHeavyThreads) k_heavy_sweep(const int32_t *__restrict__ scrd, const int32_t *__restrict__ scode,
                                                               const double *__restrict__ sval,
                                                               const int32_t *__restrict__ block_start,
                                                               const int32_t *__restrict__ wend, int nsx, int nu,
                                                               const int4 *__restrict__ units, int nunits,
                                                               const double *__restrict__ Dn, int R,
                                                               double *__restrict__ partial) {
    constexpr int L = 8, G = V <= 4 ? 4 : 2, NG = kBlock / G;     // G rows gathered ahead of the multiply-adds
    extern __shared__ __attribute__((aligned(16))) double accs[];              // [nu][groups][R]
    const int x = blockIdx.x % kXcd, wg = blockIdx.x / kXcd;
    const int g = threadIdx.x >> 3, j = threadIdx.x & 7, gl = g & 7;
    const int wave = x * kWaves + wg * (kHeavyThreads / 64) + (threadIdx.x >> 6);
    for (int k = 0; k < nu; ++k) {
        double *ac = accs + (size_t)(k * kHeavyGroups + g) * R;
#pragma unroll
        for (int q = 0; q < V / 2; ++q) *reinterpret_cast<double2 *>(ac + 2 * L * q + 2 * j) = make_double2(0.0, 0.0);
    }
    __builtin_amdgcn_wave_barrier();           // a group's sums are written and read by its own lanes only

    const int nsb = block_start[wave + 1] - block_start[wave];
    const int64_t base = (int64_t)block_start[wave] * (8 * kBlock) + gl * kBlock + 4 * j;
    const int32_t *we = wend + (int64_t)wave * (nsx + 1);
    int w = 0;                                 // intervals (of kSync windows) finished so far
    int next_end = we[1];                      // position at which interval w ends
    typedef int v4i __attribute__((ext_vector_type(4)));
    typedef double v2d __attribute__((ext_vector_type(2)));
    struct Items { int cr[4], cd[4]; double va[4]; };
    auto load_items = [&](Items &it, int sb) {
        const int64_t i = base + (int64_t)sb * (8 * kBlock);
        const v4i c4 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(scrd + i));
        const v4i d4 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(scode + i));
        const v2d a01 = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(sval + i));
        const v2d a23 = __builtin_nontemporal_load(reinterpret_cast<const v2d *>(sval + i + 2));
        it.cr[0] = c4.x; it.cr[1] = c4.y; it.cr[2] = c4.z; it.cr[3] = c4.w;
        it.cd[0] = d4.x; it.cd[1] = d4.y; it.cd[2] = d4.z; it.cd[3] = d4.w;
        it.va[0] = a01.x; it.va[1] = a01.y; it.va[2] = a23.x; it.va[3] = a23.y;
    };
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
    Items cur;
    if (nsb > 0) load_items(cur, 0);
    for (int sb = 0; sb < nsb; ++sb) {
        Items nxt;
        if (sb + 1 < nsb) load_items(nxt, sb + 1);
        const int p0 = sb * kBlock;
        struct Row { double d[V]; };
        Row buf[2][G];
        auto issue = [&](auto gc, Row *bb) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;
                const int c = grp_bcast_i<L, k / 4>(cur.cr[k % 4]);
                const int code = grp_bcast_i<L, k / 4>(cur.cd[k % 4]);
                if (code != kSkip) {
                    grp_load_row<L, V, true>(Dn, c, R, j, bb[decltype(sc)::value].d);
                } else {
#pragma unroll
                    for (int v = 0; v < V; ++v) bb[decltype(sc)::value].d[v] = 0.0;
                }
            });
        };
        auto consume = [&](auto gc, const Row *bb) {
            static_for<0, G>([&](auto sc) {
                constexpr int k = decltype(gc)::value * G + decltype(sc)::value;
                // intervals that end before this position: all wavefronts of the compute unit finish an
                // interval before any of them starts the next (wavefront-uniform condition)
                while (p0 + k == next_end && w < nsx) {
                    __builtin_amdgcn_s_barrier();
                    ++w;
                    next_end = w < nsx ? we[w + 1] : -1;
                }
                const double a = grp_bcast_d<L, k / 4>(cur.va[k % 4]);
                const int code = grp_bcast_i<L, k / 4>(cur.cd[k % 4]);
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] = fma(a, bb[decltype(sc)::value].d[v], acc[v]);
                if (code >= 0) {                                   // the unit's piece ends here: add it to the unit's sum
                    double *ac = accs + (size_t)(code * kHeavyGroups + g) * R;
#pragma unroll
                    for (int q = 0; q < V / 2; ++q) {
                        double2 *pp = reinterpret_cast<double2 *>(ac + 2 * L * q + 2 * j);
                        const double2 o = *pp;
                        *pp = make_double2(o.x + acc[2 * q], o.y + acc[2 * q + 1]);
                        acc[2 * q] = 0.0; acc[2 * q + 1] = 0.0;
                    }
                }
            });
        };
        issue(IntC<0>{}, buf[0]);
        static_for<0, NG>([&](auto gc) {
            constexpr int gi = decltype(gc)::value;
            if constexpr (gi + 1 < NG) issue(IntC<gi + 1>{}, buf[(gi + 1) & 1]);
            consume(gc, buf[gi & 1]);
        });
        if (sb + 1 < nsb) cur = nxt;
    }
    while (w < nsx) { __builtin_amdgcn_s_barrier(); ++w; }         // every wavefront meets every barrier
    const int gs = g * kSlots + wg;
    for (int k = 0; k < nu; ++k) {
        const int u = unit_of_slot(gs, k);
        if (u >= nunits) continue;
        const double *ac = accs + (size_t)(k * kHeavyGroups + g) * R;
        double *pr = partial + ((int64_t)x * nunits + units[u].w) * R;
#pragma unroll
        for (int q = 0; q < V / 2; ++q)
            *reinterpret_cast<double2 *>(pr + 2 * L * q + 2 * j) = *reinterpret_cast<const double2 *>(ac + 2 * L * q + 2 * j);
    }
}

// out[row(h), r] = sum over the units of heavy row h, and over the column ranges, of the partial rows
__global__ void __launch_bounds__(256) k_heavy_reduce(const double *__restrict__ partial, const int32_t *__restrict__ unit_begin,
                                                      const int32_t *__restrict__ hseg, const int32_t *__restrict__ rowmap,
                                                      int64_t nheavy, int nunits, int R, double *__restrict__ out,
                                                      Epilogue ep) {
    const int64_t gidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gidx >= nheavy * R) return;
    const int64_t h = gidx / R;
    const int r = (int)(gidx - h * R);
    double s = 0.0;
    for (int u = unit_begin[h]; u < unit_begin[h + 1]; ++u)
        for (int x = 0; x < kXcd; ++x) s += partial[((int64_t)x * nunits + u) * R + r];
    const int seg = hseg[h];
    const int64_t row = rowmap ? (int64_t)rowmap[seg] : (int64_t)seg;
    out[row * R + r] = ep_apply(ep, s, out + row * R + r);
}

size_t heavy_lds_bytes(int nu, int R) { return (size_t)nu * kHeavyGroups * (size_t)R * sizeof(double); }

template <int V>
hipError_t launch_sweep(const HeavyPlan &plan, const double *Dn, int R, double *partial, hipStream_t st) {
    static hipError_t attr = hipFuncSetAttribute((const void *)k_heavy_sweep<V>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    const int nwx = (plan.nwin + kXcd - 1) / kXcd, nsx = (nwx + kSync - 1) / kSync;
    hipLaunchKernelGGL((k_heavy_sweep<V>), dim3(kXcd * kSlots), dim3(kHeavyThreads), heavy_lds_bytes(plan.nu, R), st,
                       (const int32_t *)plan.scrd->ptr, (const int32_t *)plan.scode->ptr, (const double *)plan.sval->ptr,
                       (const int32_t *)plan.block_start->ptr, (const int32_t *)plan.wend->ptr, nsx, plan.nu,
                       (const int4 *)plan.units->ptr, (int)plan.nunits, Dn, R, partial);
    return hipGetLastError();
}

}  // namespace

bool heavy_supports(const HeavyPlan &plan, int64_t R) {
    if (plan.nunits <= 0) return false;
    if (R != 16 && R != 32 && R != 48 && R != 64) return false;
    return heavy_lds_bytes(plan.nu, (int)R) <= 150 * 1024;          // the units' sums must fit next to nothing else in LDS
}

size_t heavy_partial_bytes(const HeavyPlan &plan, int64_t R) {
    return ((size_t)kXcd * (size_t)plan.nunits * (size_t)R * sizeof(double) + 255) & ~(size_t)255;
}

hipError_t heavy_plan_build(const int32_t *pos, int64_t nseg, const int32_t *crd, const double *vals, int64_t nnz,
                            int64_t ncols, const int32_t *rowmap, HeavyPlan &plan, hipStream_t st) {
    plan = HeavyPlan();
    // worth it only when the dense operand is far larger than the caches and there is real work
    if (nnz < (int64_t(1) << 20) || ncols < (int64_t(1) << 16) || nseg < 1) return hipSuccess;
    DevRef counters = dev_alloc(3 * sizeof(unsigned long long));
    if (!counters) return hipErrorOutOfMemory;
    unsigned long long *cn = (unsigned long long *)counters->ptr;
    hipError_t e = hipMemsetAsync(cn, 0, 3 * sizeof(unsigned long long), st);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((nseg + 255) / 256);
    hipLaunchKernelGGL(k_count_heavy, dim3(grid), dim3(256), 0, st, pos, nseg, (int32_t)kHeavyLen, cn);
    unsigned long long h[2] = {0, 0};
    e = hipMemcpyAsync(h, cn, sizeof h, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return e;
    const int64_t nheavy = (int64_t)h[0], heavy_nnz = (int64_t)h[1];
    const int64_t nwin = (ncols + kWindow - 1) / kWindow;
    const int nwx = (int)((nwin + kXcd - 1) / kXcd), nsx = (nwx + kSync - 1) / kSync;
    if (nheavy < 1 || heavy_nnz * 8 < nnz) return hipSuccess;              // the long rows hold under an eighth
    if (nheavy * (nwin + 1) > (int64_t(1) << 27)) return hipSuccess;      // window table beyond 512 MB: not worth it
    DevRef list = dev_alloc(sizeof(int2) * nheavy);
    if (!list) return hipErrorOutOfMemory;
    hipLaunchKernelGGL(k_collect_heavy, dim3(grid), dim3(256), 0, st, pos, nseg, (int32_t)kHeavyLen, cn + 2,
                       (int2 *)list->ptr, nheavy);
    std::vector<int2> rows((size_t)nheavy);
    e = hipMemcpyAsync(rows.data(), list->ptr, sizeof(int2) * nheavy, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return e;
    // longest rows first, ties by segment: the order (and with it every sum) does not depend on how the
    // collection kernel happened to be scheduled
    std::sort(rows.begin(), rows.end(), [](const int2 &a, const int2 &b) { return a.y != b.y ? a.y > b.y : a.x < b.x; });
    std::vector<int32_t> hseg((size_t)nheavy), ubeg((size_t)nheavy + 1);
    struct UnitRec { int h, q, nsplit, id, len; };
    std::vector<UnitRec> recs;
    recs.reserve((size_t)(heavy_nnz / kUnitLen + nheavy));
    for (int64_t k = 0; k < nheavy; ++k) {
        hseg[(size_t)k] = rows[(size_t)k].x;
        ubeg[(size_t)k] = (int32_t)recs.size();
        int nsplit = (rows[(size_t)k].y + kUnitLen - 1) / kUnitLen;
        if (nsplit > kWindow) nsplit = kWindow;
        for (int qq = 0; qq < nsplit; ++qq)
            recs.push_back({(int)k, qq, nsplit, (int)recs.size(), rows[(size_t)k].y / nsplit});
    }
    ubeg[(size_t)nheavy] = (int32_t)recs.size();
    const int64_t nunits = (int64_t)recs.size();
    const int nu = (int)((nunits + kGroupSlots - 1) / kGroupSlots);
    if (nu > kMaxUnitsPerGroup) return hipSuccess;                         // more units than one sweep can hold
    // the kernel takes the units longest first (ties in row order): units of equal rank in two rounds of the
    // dealing then have about the same length.  The partial row of a unit keeps its row-major number (.w).
    std::stable_sort(recs.begin(), recs.end(), [](const UnitRec &a, const UnitRec &b) { return a.len > b.len; });
    std::vector<int4> units(recs.size());
    for (size_t k = 0; k < recs.size(); ++k) units[k] = make_int4(recs[k].h, recs[k].q, recs[k].nsplit, recs[k].id);

    const int nwaves = kXcd * kWaves;
    plan.units = dev_alloc(sizeof(int4) * units.size());
    plan.unit_begin = dev_alloc(sizeof(int32_t) * ubeg.size());
    plan.hseg = dev_alloc(sizeof(int32_t) * hseg.size());
    plan.wend = dev_alloc(sizeof(int32_t) * (size_t)nwaves * (nsx + 1));
    plan.block_start = dev_alloc(sizeof(int32_t) * (nwaves + 1));
    DevRef wstart = dev_alloc(sizeof(int32_t) * (size_t)(nheavy * (nwin + 1)));
    DevRef wmax = dev_alloc(sizeof(int32_t) * (size_t)nwaves * nsx);
    DevRef nblocks = dev_alloc(sizeof(int32_t) * nwaves);
    if (!plan.units || !plan.unit_begin || !plan.hseg || !plan.wend || !plan.block_start || !wstart || !wmax || !nblocks) {
        plan = HeavyPlan();
        return hipErrorOutOfMemory;
    }
    e = hipMemcpyAsync(plan.units->ptr, units.data(), sizeof(int4) * units.size(), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(plan.unit_begin->ptr, ubeg.data(), sizeof(int32_t) * ubeg.size(), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(plan.hseg->ptr, hseg.data(), sizeof(int32_t) * hseg.size(), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    const int64_t cells = nheavy * (nwin + 1);
    hipLaunchKernelGGL(k_build_wstart, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st, pos, crd,
                       (const int32_t *)plan.hseg->ptr, nheavy, (int)nwin, (int)kWindow, (int32_t *)wstart->ptr);
    const int64_t nlen = (int64_t)nwaves * nsx;
    hipLaunchKernelGGL(k_window_lengths, dim3((unsigned)((nlen + 255) / 256)), dim3(256), 0, st, (const int4 *)plan.units->ptr,
                       (int)nunits, nu, (const int32_t *)wstart->ptr, (int)nwin, nwx, nsx, (int32_t *)wmax->ptr);
    hipLaunchKernelGGL(k_window_ends, dim3((unsigned)((nwaves + 255) / 256)), dim3(256), 0, st, (const int32_t *)wmax->ptr, nsx,
                       (int32_t *)plan.wend->ptr, (int32_t *)nblocks->ptr);
    std::vector<int32_t> nb((size_t)nwaves), bs((size_t)nwaves + 1);
    e = hipMemcpyAsync(nb.data(), nblocks->ptr, sizeof(int32_t) * nwaves, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    int64_t total_blocks = 0;
    for (int k = 0; k < nwaves; ++k) { bs[(size_t)k] = (int32_t)total_blocks; total_blocks += nb[(size_t)k]; }
    bs[(size_t)nwaves] = (int32_t)total_blocks;
    const int64_t npos = total_blocks * 8 * kBlock;                       // stream items, padding included
    int64_t longest = 0;
    for (int k = 0; k < nwaves; ++k) longest = std::max<int64_t>(longest, nb[(size_t)k]);
    // The sweep lasts as long as its longest wavefront stream.  With the columns of every unit spread evenly over
    // the column ranges, the stream of a lane group holds an eighth of the nonzeros of the group's units (plus
    // padding).  Columns clustered in a few windows (a banded or relabelled matrix) put whole units into one
    // stream and leave the other wavefronts idle; the nonzero-tiled kernel, which is insensitive to that, then
    // does the whole matrix.
    int64_t even_share = 0;
    for (int gs = 0; gs < kGroupSlots; ++gs) {
        int64_t sum = 0;
        for (int k = 0; k < nu; ++k) {
            const int u = unit_of_slot(gs, k);
            if (u < (int)nunits) sum += recs[(size_t)u].len;
        }
        even_share = std::max(even_share, sum / kXcd);
    }
    if (total_blocks >= (int64_t(1) << 31) / (8 * kBlock) || npos > 8 * heavy_nnz + (int64_t(1) << 24) ||
        longest * kBlock > 3 * even_share + 16 * kBlock) {
        plan = HeavyPlan();
        return hipSuccess;
    }
    plan.scrd = dev_alloc(sizeof(int32_t) * (size_t)npos);
    plan.scode = dev_alloc(sizeof(int32_t) * (size_t)npos);
    plan.sval = dev_alloc(sizeof(double) * (size_t)npos);
    if (!plan.scrd || !plan.scode || !plan.sval) { plan = HeavyPlan(); return hipErrorOutOfMemory; }
    e = hipMemcpyAsync(plan.block_start->ptr, bs.data(), sizeof(int32_t) * bs.size(), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    const int64_t nfill = (int64_t)nwaves * nsx * 8;
    hipLaunchKernelGGL(k_fill_streams, dim3((unsigned)((nfill + 255) / 256)), dim3(256), 0, st, crd, vals,
                       (const int4 *)plan.units->ptr, (int)nunits, nu, (const int32_t *)wstart->ptr, (int)nwin, nwx, nsx,
                       (const int32_t *)plan.wend->ptr, (const int32_t *)plan.block_start->ptr, (int32_t *)plan.scrd->ptr,
                       (int32_t *)plan.scode->ptr, (double *)plan.sval->ptr);
    e = hipStreamSynchronize(st);                                          // the host vectors and the temporaries go out of scope
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    // all other rows, copied out as a matrix (a matrix made of long rows only needs none)
    if (nseg - nheavy > 0 && nnz - heavy_nnz > 0) {
        e = light_copy_build(pos, nseg, crd, vals, (int32_t)kHeavyLen, rowmap, nseg - nheavy, nnz - heavy_nnz, plan.light, st);
        if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    } else if (nseg - nheavy > 0) {
        plan = HeavyPlan();                                                // empty rows only: leave it to the tiled kernel
        return hipSuccess;
    }
    plan.nheavy = nheavy; plan.nunits = nunits; plan.heavy_nnz = heavy_nnz; plan.nu = nu;
    plan.min_len = kHeavyLen; plan.window = kWindow; plan.nwin = (int32_t)nwin; plan.stream_items = npos;
    return hipGetLastError();
}

hipError_t heavy_spmm(const HeavyPlan &plan, const int32_t *rowmap, const double *Dn, int64_t R, double *out, void *partial,
                      hipStream_t st, Epilogue ep) {
    if (plan.nunits <= 0) return hipSuccess;
    if (!heavy_supports(plan, R)) return hipErrorNotSupported;
    hipError_t e;
    double *pp = (double *)partial;
    switch ((int)R) {
    case 16: e = launch_sweep<2>(plan, Dn, 16, pp, st); break;
    case 32: e = launch_sweep<4>(plan, Dn, 32, pp, st); break;
    case 48: e = launch_sweep<6>(plan, Dn, 48, pp, st); break;
    default: e = launch_sweep<8>(plan, Dn, 64, pp, st); break;
    }
    if (e != hipSuccess) return e;
    const int64_t threads = plan.nheavy * R;
    hipLaunchKernelGGL(k_heavy_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (const double *)pp,
                       (const int32_t *)plan.unit_begin->ptr, (const int32_t *)plan.hseg->ptr, rowmap, plan.nheavy,
                       (int)plan.nunits, (int)R, out, ep);
    return hipGetLastError();
}


// ======================================================================================================
// Heavy-fiber sweep of TTM.
//
// y[f, :] = sum_p vals[p] * U[crd[p], :] over the nonzeros of fiber f (Section 8.2, SpTTM).  When the
// contracted mode is small (a few thousand coordinates) U is cut into windows of rows that fill LDS (128 KB:
// 1024 rows of 16 doubles or 512 rows of 32), every compute unit keeps ONE window for the whole kernel, and the
// long fibers are handled piecewise: the nonzeros of a fiber are sorted by coordinate, so those inside window w
// are the consecutive positions wstart[h][w] .. wstart[h][w+1].  A lane group of 8 takes such pieces one after
// the other (pieces of window w are dealt back and forth over the lane groups of the compute units that hold
// w, longest fibers first), gathers the operand rows from LDS -- 16 bytes per lane, a whole 128-byte row per
// group and instruction, at LDS rather than L1 / texture-address cost -- and writes one partial row per
// (fiber, window); a second kernel adds the windows of a fiber in a fixed order.  The remaining fibers stay with
// the nonzero-tiled kernel, which skips the heavy ones.
namespace {

constexpr int kFiberLen = 256;         // a fiber with at least this many nonzeros is heavy
constexpr int kFiberLdsBytes = 128 * 1024;
constexpr int kFiberMaxWindows = 16;
constexpr int kFiberThreads = 1024;

template <int L, int V>                // L lanes per group, V doubles per lane; rank = L * V
__global__ void __launch_bounds__(kFiberThreads) k_fiber_sweep(const int32_t *__restrict__ crd, const double *__restrict__ vals,
                                                               const int32_t *__restrict__ wstart, int nheavy, int nwin,
                                                               int window, const double *__restrict__ U, int ncols,
                                                               double *__restrict__ partial) {
    extern __shared__ __attribute__((aligned(16))) double2 urows[];          // [window][R / 2]
    constexpr int R = L * V, R2 = R / 2, kGroups = kFiberThreads / L;
    const int w = (int)(blockIdx.x % (unsigned)nwin), cw = (int)(blockIdx.x / (unsigned)nwin);
    const int ncw = ((int)gridDim.x - w + nwin - 1) / nwin;                  // workgroups that hold window w
    const int k0 = w * window, k1 = k0 + window < ncols ? k0 + window : ncols;
    {
        const int n2 = (k1 - k0) * R2;
        const double2 *src = reinterpret_cast<const double2 *>(U + (size_t)k0 * R);
        for (int i = threadIdx.x; i < n2; i += kFiberThreads) urows[i] = src[i];
    }
    __syncthreads();
    const int g = threadIdx.x / L, j = threadIdx.x % L;
    const int Gw = ncw * kGroups, mine = cw * kGroups + g;
    const int per = nwin + 1;
    auto piece_of = [&](int t) { return t * Gw + ((t & 1) ? Gw - 1 - mine : mine); };
    const int rounds = (nheavy + Gw - 1) / Gw;
    // bounds of the first piece
    int h = piece_of(0), p0 = 0, p1 = 0;
    if (rounds > 0 && h < nheavy) { p0 = wstart[(size_t)h * per + w]; p1 = wstart[(size_t)h * per + w + 1]; }
    for (int t = 0; t < rounds; ++t) {
        // bounds of the next piece: in flight during this one
        const int hn = piece_of(t + 1);
        int p0n = 0, p1n = 0;
        if (t + 1 < rounds && hn < nheavy) { p0n = wstart[(size_t)hn * per + w]; p1n = wstart[(size_t)hn * per + w + 1]; }
        double acc[V];
#pragma unroll
        for (int q = 0; q < V; ++q) acc[q] = 0.0;
        int c_cur = 0;
        double a_cur = 0.0;
        if (p0 + j < p1) { c_cur = crd[p0 + j]; a_cur = vals[p0 + j]; }
        int p = p0;
        auto block = [&](auto checked) {                                   // L items: one per lane, taken one by one
            int c_nxt = 0;
            double a_nxt = 0.0;
            if (p + L + j < p1) { c_nxt = crd[p + L + j]; a_nxt = vals[p + L + j]; }
            const int rowoff = (c_cur - k0) * R2;                          // of this lane's item, in 16-byte pieces
            static_for<0, L>([&](auto sc) {
                constexpr int s_ = decltype(sc)::value;
                if (!decltype(checked)::value || p + s_ < p1) {             // the same for the whole group
                    const int o = grp_bcast_i<L, s_>(rowoff) + j;
                    const double a = grp_bcast_d<L, s_>(a_cur);
#pragma unroll
                    for (int q = 0; q < V / 2; ++q) {
                        const double2 d = urows[o + L * q];
                        acc[2 * q] = fma(a, d.x, acc[2 * q]);
                        acc[2 * q + 1] = fma(a, d.y, acc[2 * q + 1]);
                    }
                }
            });
            c_cur = c_nxt; a_cur = a_nxt;
            p += L;
        };
        while (p + L <= p1) block(IntC<0>{});
        if (p < p1) block(IntC<1>{});
        if (h < nheavy) {
            double2 *dst = reinterpret_cast<double2 *>(partial + ((size_t)h * nwin + w) * R) + j;
#pragma unroll
            for (int q = 0; q < V / 2; ++q) dst[L * q] = make_double2(acc[2 * q], acc[2 * q + 1]);
        }
        h = hn; p0 = p0n; p1 = p1n;
    }
}

// out[fiber(h), r] = sum over the windows of the partial rows of heavy fiber h, in window order
__global__ void __launch_bounds__(256) k_fiber_reduce(const double *__restrict__ partial, const int32_t *__restrict__ hseg,
                                                      int64_t nheavy, int nwin, int R, double *__restrict__ out) {
    const int64_t gidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gidx >= nheavy * R) return;
    const int64_t h = gidx / R;
    const int r = (int)(gidx - h * R);
    double s = 0.0;
    for (int w = 0; w < nwin; ++w) s += partial[((size_t)h * nwin + w) * R + r];
    out[(int64_t)hseg[h] * R + r] = s;
}

int fiber_plan_index(int64_t R) { return R == 16 ? 0 : (R == 32 ? 1 : -1); }

}  // namespace

bool fiber_supports(const FiberPlan &plan, int64_t R) {
    const int k = fiber_plan_index(R);
    return plan.nheavy > 0 && k >= 0 && plan.nwin[k] > 0;
}

size_t fiber_partial_bytes(const FiberPlan &plan, int64_t R) {
    const int k = fiber_plan_index(R);
    if (plan.nheavy <= 0 || k < 0) return 0;
    return ((size_t)plan.nheavy * (size_t)plan.nwin[k] * (size_t)R * sizeof(double) + 255) & ~(size_t)255;
}

hipError_t fiber_plan_build(const int32_t *pos, int64_t nseg, const int32_t *crd, const double *vals, int64_t nnz,
                            int64_t ncols, FiberPlan &plan, hipStream_t st) {
    plan = FiberPlan();
    const int window[2] = {kFiberLdsBytes / (16 * 8), kFiberLdsBytes / (32 * 8)};
    if (nnz < (int64_t(1) << 20) || nseg < 1 || ncols < 1 || ncols > (int64_t)window[1] * kFiberMaxWindows) return hipSuccess;
    DevRef counters = dev_alloc(3 * sizeof(unsigned long long));
    if (!counters) return hipErrorOutOfMemory;
    unsigned long long *cn = (unsigned long long *)counters->ptr;
    hipError_t e = hipMemsetAsync(cn, 0, 3 * sizeof(unsigned long long), st);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((nseg + 255) / 256);
    hipLaunchKernelGGL(k_count_heavy, dim3(grid), dim3(256), 0, st, pos, nseg, (int32_t)kFiberLen, cn);
    unsigned long long hc[2] = {0, 0};
    e = hipMemcpyAsync(hc, cn, sizeof hc, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return e;
    const int64_t nheavy = (int64_t)hc[0], heavy_nnz = (int64_t)hc[1];
    if (nheavy < 1 || heavy_nnz * 4 < nnz || nheavy > (int64_t(1) << 24)) return hipSuccess;   // the long fibers hold under a quarter
    DevRef list = dev_alloc(sizeof(int2) * nheavy);
    if (!list) return hipErrorOutOfMemory;
    hipLaunchKernelGGL(k_collect_heavy, dim3(grid), dim3(256), 0, st, pos, nseg, (int32_t)kFiberLen, cn + 2,
                       (int2 *)list->ptr, nheavy);
    std::vector<int2> fib((size_t)nheavy);
    e = hipMemcpyAsync(fib.data(), list->ptr, sizeof(int2) * nheavy, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return e;
    // longest first, ties by fiber: the dealing (and with it nothing but the schedule) does not depend on how the
    // collection kernel happened to run
    std::sort(fib.begin(), fib.end(), [](const int2 &a, const int2 &b) { return a.y != b.y ? a.y > b.y : a.x < b.x; });
    std::vector<int32_t> hseg((size_t)nheavy);
    for (int64_t k = 0; k < nheavy; ++k) hseg[(size_t)k] = fib[(size_t)k].x;
    plan.hseg = dev_alloc(sizeof(int32_t) * nheavy);
    if (!plan.hseg) { plan = FiberPlan(); return hipErrorOutOfMemory; }
    e = hipMemcpyAsync(plan.hseg->ptr, hseg.data(), sizeof(int32_t) * nheavy, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { plan = FiberPlan(); return e; }
    for (int k = 0; k < 2; ++k) {
        const int64_t nwin = (ncols + window[k] - 1) / window[k];
        if (nwin > kFiberMaxWindows) continue;
        const int64_t cells = nheavy * (nwin + 1);
        plan.wstart[k] = dev_alloc(sizeof(int32_t) * (size_t)cells);
        if (!plan.wstart[k]) { plan = FiberPlan(); return hipErrorOutOfMemory; }
        hipLaunchKernelGGL(k_build_wstart, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st, pos, crd,
                           (const int32_t *)plan.hseg->ptr, nheavy, (int)nwin, window[k], (int32_t *)plan.wstart[k]->ptr);
        plan.window[k] = window[k];
        plan.nwin[k] = (int32_t)nwin;
    }
    e = hipStreamSynchronize(st);                                          // the host vector goes out of scope
    if (e != hipSuccess) { plan = FiberPlan(); return e; }
    if (plan.nwin[0] == 0 && plan.nwin[1] == 0) { plan = FiberPlan(); return hipSuccess; }
    // all other fibers, copied out as a matrix
    const int64_t nlight = nseg - nheavy, light_nnz = nnz - heavy_nnz;
    if (nlight < 1 || light_nnz < 1) { plan = FiberPlan(); return hipSuccess; }
    e = light_copy_build(pos, nseg, crd, vals, (int32_t)kFiberLen, nullptr, nlight, light_nnz, plan.light, st);
    if (e != hipSuccess) { plan = FiberPlan(); return e; }
    plan.nheavy = nheavy; plan.heavy_nnz = heavy_nnz; plan.min_len = kFiberLen;
    return hipGetLastError();
}

hipError_t fiber_ttm(const FiberPlan &plan, const int32_t *crd, const double *vals, const double *Dn, int64_t ncols,
                     int64_t R, double *out, void *partial, hipStream_t st) {
    if (!fiber_supports(plan, R)) return hipErrorNotSupported;
    const int k = fiber_plan_index(R);
    const int ncu = current_device_cu_count();
    const unsigned grid = (unsigned)(ncu < plan.nwin[k] ? plan.nwin[k] : ncu);      // every window needs a workgroup
    const size_t lds = (size_t)plan.window[k] * (size_t)R * sizeof(double);
    double *pp = (double *)partial;
    hipError_t e;
    if (R == 16) {
        static hipError_t attr = hipFuncSetAttribute((const void *)k_fiber_sweep<8, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if ((e = attr) != hipSuccess) return e;
        hipLaunchKernelGGL((k_fiber_sweep<8, 2>), dim3(grid), dim3(kFiberThreads), lds, st, crd, vals, (const int32_t *)plan.wstart[k]->ptr,
                           (int)plan.nheavy, (int)plan.nwin[k], (int)plan.window[k], Dn, (int)ncols, pp);
    } else {
        static hipError_t attr = hipFuncSetAttribute((const void *)k_fiber_sweep<8, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if ((e = attr) != hipSuccess) return e;
        hipLaunchKernelGGL((k_fiber_sweep<8, 4>), dim3(grid), dim3(kFiberThreads), lds, st, crd, vals, (const int32_t *)plan.wstart[k]->ptr,
                           (int)plan.nheavy, (int)plan.nwin[k], (int)plan.window[k], Dn, (int)ncols, pp);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t threads = plan.nheavy * R;
    hipLaunchKernelGGL(k_fiber_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (const double *)pp,
                       (const int32_t *)plan.hseg->ptr, plan.nheavy, (int)plan.nwin[k], (int)R, out);
    return hipGetLastError();
}

}  // namespace comet
