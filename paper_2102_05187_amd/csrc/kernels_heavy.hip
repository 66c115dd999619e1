// Heavy-row sweep of SpMM: the long rows of a power-law matrix, processed so that the rows of the dense
// operand they gather are shared through the L2 caches instead of being fetched from memory once per nonzero.
//
// With uniformly scattered columns every gather of a row of B (R * 8 bytes) misses the caches when the rows
// of A are walked one after the other: B is far larger than any cache.  But the few long rows hold most of
// the nonzeros (the paper's load-imbalance discussion, Section 8.3, is about exactly these rows), and all of
// them touch the same columns.  So the columns are cut into windows of kWindow (a window's rows of B fit
// the 4 MB L2 of one XCD several times over), the windows are dealt to the eight XCDs in contiguous ranges,
// and on each XCD every heavy row is walked window by window by lane groups that all advance at the same
// pace: a row of B is fetched from memory once per sweep and then hit in L2 by every other heavy row that
// has a nonzero in that column.  Workgroups are placed on the XCDs round-robin, so workgroup b sweeps the
// window range of XCD b mod 8; were the placement different only the cache reuse would suffer.
//
// A heavy row is cut into units of comparable length (a unit takes the q-th of nsplit equal pieces of the
// row's nonzeros inside every window), every lane group owns up to RPG units and keeps their sums in
// registers for the whole sweep, and units are dealt to the lane groups longest rows first, so all groups
// carry about the same number of nonzeros per window, and the grid fills every compute unit with the same
// number of workgroups, so that none runs ahead for having a compute unit more to itself -- that, not a
// barrier, is what keeps the sweeps in step.  (A window clock in memory that every wavefront counts into and
// waits on was tried: same-address atomics across the device cost more than the drift they remove.)
// Each (unit, XCD) pair yields one partial row; a second kernel adds the partial rows of a heavy row in a
// fixed order (no atomics: results are reproducible run to run).
#include <algorithm>
#include <atomic>
#include <vector>

#include "stream_common.hpp"

namespace comet {

namespace {

constexpr int kXcd = 8;              // XCDs of the device = number of column ranges
constexpr int kWindow = 4096;        // columns per window
constexpr int kHeavyLen = 256;       // a row with at least this many nonzeros is heavy
constexpr int kUnitLen = 2048;       // target nonzeros per unit
constexpr int kHeavyThreads = 1024;  // 128 lane groups of 8 lanes per workgroup: one workgroup fills a compute unit
constexpr int kHeavyGroups = kHeavyThreads / 8;

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

// ---- the sweep -------------------------------------------------------------------------------------------
// Lane group = 8 lanes; lane j holds ranks 16 q + 2 j, 16 q + 2 j + 1 of a row (q < V / 2), so one load
// instruction reads a whole 128-byte line of a gathered row per lane group.  A lane group owns `nu` units
// (their running sums sit in LDS, R doubles each) and walks them window by window: the work of a group is
// the flat sequence of pieces t = (window, unit).  Three pieces are in flight at a time -- the window bounds
// of piece t + 2 and the nonzeros of piece t + 1 are being fetched while the rows of B for piece t are
// gathered (all of a piece's rows at once, up to 8) -- so that the chain bounds -> nonzeros -> rows is not
// walked one memory latency at a time.
struct UnitMeta { int woff, qn, uid; };      // window-table row offset, (piece << 16 | pieces of the row), partial row

template <int V>
__global__ void __launch_bounds__(kHeavyThreads) k_spmm_heavy(const int32_t *__restrict__ crd, const double *__restrict__ vals,
                                                              const int4 *__restrict__ units, int nunits, int nu,
                                                              const int32_t *__restrict__ wstart, int nwin, int nwx,
                                                              const double *__restrict__ Dn, int R,
                                                              double *__restrict__ partial) {
    constexpr int L = 8;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    double *accs = reinterpret_cast<double *>(lds_raw);                          // [nu][groups][R]
    int *meta = reinterpret_cast<int *>(lds_raw + (size_t)nu * kHeavyGroups * R * sizeof(double));   // [nu][groups][3]
    const int x = blockIdx.x % kXcd, slot = blockIdx.x / kXcd, nslots = gridDim.x / kXcd;
    const int g = threadIdx.x >> 3, j = threadIdx.x & 7;
    // group slot: consecutive units (the table comes longest unit first) go to different workgroups, back and
    // forth from one round to the next, so that every group -- and every workgroup -- gets about the same number
    // of nonzeros per window and all of them need about the same time for it
    const int gslot = g * nslots + slot, ngslots = nslots * kHeavyGroups;
    const int w0 = x * nwx, w1 = (w0 + nwx < nwin) ? w0 + nwx : nwin;
    const int per = nwin + 1;
    for (int k = 0; k < nu; ++k) {
        const int u = k * ngslots + ((k & 1) ? ngslots - 1 - gslot : gslot);
        const int4 un = u < nunits ? units[u] : make_int4(0, 0, 1, -1);
        if (j == 0) {
            int *m = meta + (k * kHeavyGroups + g) * 3;
            m[0] = un.x * per; m[1] = (un.y << 16) | un.z; m[2] = u < nunits ? un.w : -1;
        }
        double *ac = accs + (size_t)(k * kHeavyGroups + g) * R;
#pragma unroll
        for (int q = 0; q < V / 2; ++q) *reinterpret_cast<double2 *>(ac + 2 * L * q + 2 * j) = make_double2(0.0, 0.0);
    }
    __builtin_amdgcn_wave_barrier();      // meta and sums of a group are written and read by the group's own lanes only

    const int T = (w1 - w0) * nu;         // pieces of this group: t = (w - w0) * nu + k
    // piece t + 2: bounds;  piece t + 1: first L nonzeros;  piece t: being processed
    int ba = 0, be = 0, bq = 1;           // bounds (and split code) of the piece two ahead
    int nc = 0, nlo = 0, nhi = 0;         // the piece one ahead
    double na = 0.0;
    auto fetch_bounds = [&](int t) {      // t < T
        const int k = t % nu, w = w0 + t / nu;
        const int *m = meta + (k * kHeavyGroups + g) * 3;
        const bool have = m[2] >= 0;
        ba = have ? wstart[m[0] + w] : 0;
        be = have ? wstart[m[0] + w + 1] : 0;
        bq = m[1];
    };
    auto fetch_items = [&]() {            // from the bounds in (ba, be, bq)
        const int n = be - ba;                                                  // at most kWindow
        const int qq = bq >> 16, ns = bq & 0xffff;
        nlo = ba + n * qq / ns;
        nhi = ba + n * (qq + 1) / ns;
        const int i = nlo + j;
        const bool in = i < nhi;
        nc = in ? __builtin_nontemporal_load(crd + i) : 0;
        na = in ? __builtin_nontemporal_load(vals + i) : 0.0;                   // 0 past the end
    };
    if (T > 0) { fetch_bounds(0); fetch_items(); }
    if (T > 1) fetch_bounds(1);
    for (int t = 0; t < T; ++t) {
        int c = nc;
        double a0 = na;
        const int lo = nlo, hi = nhi;
        if (t + 1 < T) fetch_items();
        if (t + 2 < T) fetch_bounds(t + 2);
        if (lo < hi) {
            double *ac = accs + (size_t)((t % nu) * kHeavyGroups + g) * R;
            double acc[V];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = 0.0;
            for (int base = lo; base < hi; base += L) {
                if (base != lo) {                                              // a piece of more than L nonzeros: the rest on demand
                    const int i = base + j;
                    const bool in = i < hi;
                    c = in ? __builtin_nontemporal_load(crd + i) : 0;
                    a0 = in ? __builtin_nontemporal_load(vals + i) : 0.0;
                }
                const int cnt = hi - base;                                     // items of this batch (more than L: then L)
                double row[L][V];
                static_for<0, L>([&](auto bp) {
                    constexpr int BP = decltype(bp)::value;
                    const int cb = grp_bcast_i<L, BP>(c);
                    if (BP < cnt) {
                        grp_load_row<L, V, true>(Dn, cb, R, j, row[BP]);
                    } else {
#pragma unroll
                        for (int v = 0; v < V; ++v) row[BP][v] = 0.0;
                    }
                });
                static_for<0, L>([&](auto bp) {
                    constexpr int BP = decltype(bp)::value;
                    const double av = grp_bcast_d<L, BP>(a0);                  // 0 for the lanes past the end
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = fma(av, row[BP][v], acc[v]);
                });
            }
#pragma unroll
            for (int q = 0; q < V / 2; ++q) {
                double2 *p = reinterpret_cast<double2 *>(ac + 2 * L * q + 2 * j);
                const double2 o = *p;
                *p = make_double2(o.x + acc[2 * q], o.y + acc[2 * q + 1]);
            }
        }
        // all wavefronts of the compute unit finish a window before any starts the next (no data is exchanged:
        // this only keeps them on the same rows of B)
        if ((t + 1) % nu == 0) __builtin_amdgcn_s_barrier();
    }
    for (int k = 0; k < nu; ++k) {
        const int uid = meta[(k * kHeavyGroups + g) * 3 + 2];
        if (uid < 0) continue;
        const double *ac = accs + (size_t)(k * kHeavyGroups + g) * R;
        double *pr = partial + ((int64_t)x * nunits + uid) * R;
#pragma unroll
        for (int q = 0; q < V / 2; ++q)
            *reinterpret_cast<double2 *>(pr + 2 * L * q + 2 * j) = *reinterpret_cast<const double2 *>(ac + 2 * L * q + 2 * j);
    }
}

// out[row(h), r] = sum over the units of heavy row h, and over the column ranges, of the partial rows
__global__ void __launch_bounds__(256) k_heavy_reduce(const double *__restrict__ partial, const int32_t *__restrict__ unit_begin,
                                                      const int32_t *__restrict__ hseg, const int32_t *__restrict__ rowmap,
                                                      int64_t nheavy, int nunits, int R, double *__restrict__ out) {
    const int64_t gidx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gidx >= nheavy * R) return;
    const int64_t h = gidx / R;
    const int r = (int)(gidx - h * R);
    double s = 0.0;
    for (int u = unit_begin[h]; u < unit_begin[h + 1]; ++u)
        for (int x = 0; x < kXcd; ++x) s += partial[((int64_t)x * nunits + u) * R + r];
    const int seg = hseg[h];
    const int64_t row = rowmap ? (int64_t)rowmap[seg] : (int64_t)seg;
    out[row * R + r] = s;
}

size_t heavy_lds_bytes(int nu, int R) { return (size_t)nu * kHeavyGroups * ((size_t)R * sizeof(double) + 3 * sizeof(int)); }

constexpr int kMaxUnitsPerGroup = 6;

// Units per lane group (nu) and workgroups per column range (nslots): the smallest nu for which all units are
// resident at once, every compute unit filled with the same number of workgroups -- a workgroup that had a
// compute unit more to itself would run ahead of the others and the sweeps would fall out of step.
// False when one sweep cannot hold all units.
template <int V>
bool heavy_shape(const HeavyPlan &plan, int R, int *nu_out, int *nslots_out) {
    static std::atomic<int> per_cu_of[kMaxUnitsPerGroup + 1];          // occupancy by nu, cached (0 = not asked yet)
    static hipError_t attr = hipFuncSetAttribute((const void *)k_spmm_heavy<V>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) { (void)hipGetLastError(); return false; }
    const int cus_per_xcd = current_device_cu_count() / kXcd > 0 ? current_device_cu_count() / kXcd : 1;
    for (int nu = 1; nu <= kMaxUnitsPerGroup; ++nu) {
        int per_cu = per_cu_of[nu].load();
        if (per_cu == 0) {
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)k_spmm_heavy<V>, kHeavyThreads,
                                                             heavy_lds_bytes(nu, R)) != hipSuccess || per_cu < 1) {
                (void)hipGetLastError();
                per_cu = -1;
            }
            per_cu_of[nu].store(per_cu);
        }
        if (per_cu < 1) return false;
        if ((int64_t)per_cu * cus_per_xcd * kHeavyGroups * nu >= plan.nunits) {
            int64_t want = (plan.nunits + (int64_t)nu * kHeavyGroups - 1) / ((int64_t)nu * kHeavyGroups);
            want = (want + cus_per_xcd - 1) / cus_per_xcd * cus_per_xcd;
            *nu_out = nu;
            *nslots_out = (int)want;
            return true;
        }
    }
    return false;
}

template <int V>
hipError_t launch_heavy_v(const HeavyPlan &plan, const int32_t *crd, const double *vals, const double *Dn, int R,
                          double *partial, hipStream_t st) {
    int nu = 0, nslots = 0;
    if (!heavy_shape<V>(plan, R, &nu, &nslots)) return hipErrorNotSupported;
    const int nwx = (plan.nwin + kXcd - 1) / kXcd;
    hipLaunchKernelGGL((k_spmm_heavy<V>), dim3((unsigned)(nslots * kXcd)), dim3(kHeavyThreads), heavy_lds_bytes(nu, R), st, crd,
                       vals, (const int4 *)plan.units->ptr, (int)plan.nunits, nu, (const int32_t *)plan.wstart->ptr,
                       (int)plan.nwin, nwx, Dn, R, partial);
    return hipGetLastError();
}

}  // namespace

bool heavy_supports(const HeavyPlan &plan, int64_t R) {
    int nu = 0, nslots = 0;
    if (plan.nunits <= 0) return false;
    switch ((int)R) {
    case 16: return R == 16 && heavy_shape<2>(plan, 16, &nu, &nslots);
    case 32: return heavy_shape<4>(plan, 32, &nu, &nslots);
    case 48: return heavy_shape<6>(plan, 48, &nu, &nslots);
    case 64: return heavy_shape<8>(plan, 64, &nu, &nslots);
    }
    return false;
}

size_t heavy_partial_bytes(const HeavyPlan &plan, int64_t R) {
    return ((size_t)kXcd * (size_t)plan.nunits * (size_t)R * sizeof(double) + 255) & ~(size_t)255;
}

hipError_t heavy_plan_build(const int32_t *pos, int64_t nseg, const int32_t *crd, int64_t nnz, int64_t ncols,
                            HeavyPlan &plan, hipStream_t st) {
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
        if (nsplit > 0x7fff) nsplit = 0x7fff;                              // (piece, pieces) travel in 16 bits each
        for (int qq = 0; qq < nsplit; ++qq)
            recs.push_back({(int)k, qq, nsplit, (int)recs.size(), rows[(size_t)k].y / nsplit});
    }
    ubeg[(size_t)nheavy] = (int32_t)recs.size();
    // the kernel takes the units longest first (ties in row order): units of equal rank in two rounds of the
    // dealing then have about the same length.  The partial row of a unit keeps its row-major number (.w).
    std::stable_sort(recs.begin(), recs.end(), [](const UnitRec &a, const UnitRec &b) { return a.len > b.len; });
    std::vector<int4> units(recs.size());
    for (size_t k = 0; k < recs.size(); ++k) units[k] = make_int4(recs[k].h, recs[k].q, recs[k].nsplit, recs[k].id);
    if (units.size() >= (size_t(1) << 28)) return hipSuccess;
    plan.units = dev_alloc(sizeof(int4) * units.size());
    plan.unit_begin = dev_alloc(sizeof(int32_t) * ubeg.size());
    plan.hseg = dev_alloc(sizeof(int32_t) * hseg.size());
    plan.wstart = dev_alloc(sizeof(int32_t) * (size_t)(nheavy * (nwin + 1)));
    if (!plan.units || !plan.unit_begin || !plan.hseg || !plan.wstart) { plan = HeavyPlan(); return hipErrorOutOfMemory; }
    e = hipMemcpyAsync(plan.units->ptr, units.data(), sizeof(int4) * units.size(), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(plan.unit_begin->ptr, ubeg.data(), sizeof(int32_t) * ubeg.size(), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(plan.hseg->ptr, hseg.data(), sizeof(int32_t) * hseg.size(), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    const int64_t cells = nheavy * (nwin + 1);
    hipLaunchKernelGGL(k_build_wstart, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st, pos, crd,
                       (const int32_t *)plan.hseg->ptr, nheavy, (int)nwin, (int)kWindow, (int32_t *)plan.wstart->ptr);
    e = hipStreamSynchronize(st);                                          // the host vectors go out of scope
    if (e != hipSuccess) { plan = HeavyPlan(); return e; }
    plan.nheavy = nheavy; plan.nunits = (int64_t)units.size(); plan.heavy_nnz = heavy_nnz;
    plan.min_len = kHeavyLen; plan.window = kWindow; plan.nwin = (int32_t)nwin;
    return hipGetLastError();
}

hipError_t heavy_spmm(const HeavyPlan &plan, const int32_t *crd, const double *vals, const int32_t *rowmap,
                      const double *Dn, int64_t R, double *out, void *partial, hipStream_t st) {
    if (plan.nunits <= 0) return hipSuccess;
    if (!heavy_supports(plan, R)) return hipErrorNotSupported;
    hipError_t e;
    double *pp = (double *)partial;
    switch ((int)R) {
    case 16: e = launch_heavy_v<2>(plan, crd, vals, Dn, 16, pp, st); break;
    case 32: e = launch_heavy_v<4>(plan, crd, vals, Dn, 32, pp, st); break;
    case 48: e = launch_heavy_v<6>(plan, crd, vals, Dn, 48, pp, st); break;
    default: e = launch_heavy_v<8>(plan, crd, vals, Dn, 64, pp, st); break;
    }
    if (e != hipSuccess) return e;
    const int64_t threads = plan.nheavy * R;
    hipLaunchKernelGGL(k_heavy_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (const double *)pp,
                       (const int32_t *)plan.unit_begin->ptr, (const int32_t *)plan.hseg->ptr, rowmap, plan.nheavy,
                       (int)plan.nunits, (int)R, out);
    return hipGetLastError();
}

}  // namespace comet
