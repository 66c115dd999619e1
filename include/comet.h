/*
 * comet.h -- C ABI of the MI355X (gfx950) sparse x dense contraction library.
 *
 * The library evaluates the mixed sparse/dense contractions of the COMET paper
 * (arXiv 2102.05187) -- SpMV, SpMM, SpTTV, SpTTM (Section 8.2, "Sparse Tensor
 * Operations") and MTTKRP (named in Section 8.3) -- on tensors held in the paper's
 * per-dimension level storage (Section 4, "Tensor Storage Format").
 *
 * General conventions
 *   - Every array pointer is a DEVICE pointer unless a parameter says "host".
 *   - Index arrays (pos, crd) are int32, values are fp64 (Section 6.1, "Sparse Tensor
 *     Data Type"); coordinates, positions and modes are 0-based.
 *   - Dense operands and dense results are contiguous and row-major, last index fastest
 *     (Section 6.2 Step II: the dense index update vIdx = vIdx*SIZE + arg).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Operations
 *     enqueue work on it and return without synchronising; comet_tensor_create and
 *     comet_tensor_destroy synchronise with the stream they are given.
 *   - Every call returns a comet_status; nothing aborts or throws.  Device faults caused
 *     by arrays that violate the format (and were not validated) are not detected.
 *   - A tensor handle owns per-tensor scratch memory: at most one operation per handle may
 *     be in flight at a time (operations on one stream are ordered and therefore safe).  The
 *     scratch is allocated by comet_tensor_reserve, or else by the first operation that needs more
 *     than the handle holds (a device allocation, so that call cannot be captured into a HIP
 *     graph); calls that fit into what is there allocate nothing, clear what they reuse with
 *     kernels, and can be captured.  Scratch only grows and is never freed before the handle is
 *     destroyed, so an address that earlier work or a captured graph uses stays valid.
 */
#ifndef COMET_H
#define COMET_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COMET_MAX_ORDER 4

/* Storage attribute of one level (Section 4):
 *   D   dense:               pos = {size}, no crd; every coordinate 0..size-1 is visited and the
 *                            child position is parent*size + coordinate.
 *   CU  compressed-unique:   crd holds each distinct coordinate once per parent; the children
 *                            of parent position m are positions pos[m] .. pos[m+1]-1.  At the
 *                            root m = 0, so pos = {0, n}.
 *   CN  compressed-nonunique: crd holds the coordinate of every nonzero (duplicates kept);
 *                            pos = {0, n} (start and extent of crd).  Root level only.
 *   S   singleton:           no pos; crd[m] is the coordinate that belongs to parent position m.
 * Level l stores mode l of the tensor.                                                        */
typedef enum { COMET_D = 0, COMET_CU = 1, COMET_CN = 2, COMET_S = 3 } comet_level_t;

typedef enum {
    COMET_OK = 0,
    COMET_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad flag                      */
    COMET_ERR_BAD_FORMAT  = 2,   /* arrays do not form a valid tensor of the stated levels     */
    COMET_ERR_SHAPE       = 3,   /* operand sizes do not match the tensor                      */
    COMET_ERR_UNSUPPORTED = 4,   /* level tuple / mode / rank outside what the kernels cover   */
    COMET_ERR_ALLOC       = 5,   /* device or host allocation failed                           */
    COMET_ERR_DEVICE      = 6    /* a HIP call failed                                          */
} comet_status;

/* comet_tensor_create flags */
#define COMET_BORROW   0u   /* default: the caller keeps pos/crd/vals alive and unchanged until destroy */
#define COMET_COPY     1u   /* the library copies pos/crd/vals into memory it owns              */
#define COMET_VALIDATE 2u   /* run the device-side structure check (see below)                  */
#define COMET_LEAN     4u   /* keep no copies of parts of the tensor: the heavy-row sweep of    */
                            /* comet_spmm and the heavy-fiber sweep of comet_ttm are not planned */
                            /* (same results from the nonzero-tiled kernels alone, less memory) */

typedef struct comet_tensor comet_tensor;   /* opaque, library-owned */

/* Read-only description of a handle (host struct filled by comet_tensor_info). */
typedef struct {
    int32_t        order;
    int64_t        dims[COMET_MAX_ORDER];
    int32_t        levels[COMET_MAX_ORDER];   /* comet_level_t                                  */
    const int32_t *pos[COMET_MAX_ORDER];      /* device pointers (NULL where the level has none) */
    int64_t        pos_len[COMET_MAX_ORDER];
    const int32_t *crd[COMET_MAX_ORDER];
    int64_t        crd_len[COMET_MAX_ORDER];
    const double  *vals;                      /* device pointer                                 */
    int64_t        nvals;
    int32_t        mode_of_level[COMET_MAX_ORDER];  /* tensor mode stored at each level: 0,1,2,..
                                                 * unless comet_tensor_reorder chose another order;
                                                 * dims / levels / pos / crd above are per LEVEL    */
    int64_t        heavy_rows;                /* schedule: rows that comet_spmm hands to its heavy-row sweep  */
                                              /* (order 3: fibers that comet_ttm hands to its heavy-fiber sweep) */
    int64_t        heavy_nnz;                 /* ... and the nonzeros they hold (both 0: no sweep planned)   */
    int64_t        heavy_stream_bytes;        /* device memory of the sweep's re-ordered copy of those rows   */
                                              /* plus the compacted copy of all other rows (order 3: of the   */
                                              /* compacted copy of all other fibers)                          */
} comet_tensor_info_t;

/*
 * Build a tensor handle from per-level pos/crd arrays and a value array -- the construction
 * `sptensor_construct(A1pos, A1crd, A2pos, A2crd, AVal)` of Section 6.1, generalised to
 * `order` levels.
 *
 *   out      host; receives the handle.
 *   order    number of modes = number of levels (2 or 3 for the operations below).
 *   dims     host, [order]; logical size of each mode (each < 2^31).
 *   levels   host, [order]; storage attribute of each level.
 *   pos      host array of [order] device pointers; pos_len host, [order].  NULL / 0 for S.
 *            Expected lengths: D 1; root CU or CN 2; non-root CU (#parent positions)+1.
 *   crd      host array of [order] device pointers; crd_len host, [order].  NULL / 0 for D.
 *   vals     device, [nvals]; one value per position of the last level.  nvals < 2^31.
 *   flags    COMET_BORROW | COMET_COPY, optionally | COMET_VALIDATE, optionally | COMET_LEAN.
 *
 * Cheap consistency checks (lengths, root pos contents, D size == dims) always run.  With
 * COMET_VALIDATE a device pass also checks: pos starts at 0, is non-decreasing and ends at
 * crd_len; every coordinate lies in [0, dim); coordinates are strictly increasing inside each CU
 * segment; a CN/S coordinate list is lexicographically sorted without duplicates.  Failures give
 * COMET_ERR_BAD_FORMAT and no handle.  Explicit zeros in vals are legal stored entries.
 *
 * The arrays must not change while the handle lives: besides the tile tables below, a handle may keep
 * copies of parts of the tensor, values included (the plans of the two sweeps, see COMET_LEAN and
 * heavy_stream_bytes; the compressed copy of a coordinate list), and these would not follow.  Values that
 * change call for a new handle.
 *
 * The call also builds the per-tensor schedule (nonzero-balanced tile tables used by the
 * kernels; load imbalance is what Section 8.3 identifies as the main source of slowdown), which
 * is why it synchronises.  Accepted tuples: [D,CU] (CSR), [CU,CU] (DCSR), [CN,S] and [CN,S,S]
 * (COO), [CU,CU,CU] (CSF); results of TTV/TTM may additionally be [CU,CU,D] or [CN,S,D].
 */
comet_status comet_tensor_create(comet_tensor **out, int order,
                                 const int64_t *dims, const comet_level_t *levels,
                                 const int32_t *const *pos, const int64_t *pos_len,
                                 const int32_t *const *crd, const int64_t *crd_len,
                                 const double *vals, int64_t nvals,
                                 unsigned flags, void *stream);

/* Release a handle and everything the library allocated for it (borrowed arrays are left
 * alone).  Level arrays that a TTV/TTM result shares with its input stay valid until the last
 * handle that uses them is destroyed.  Waits for the streams the handle's operations were enqueued
 * on (for the whole device if they were more than four, or the null stream).  NULL is accepted. */
comet_status comet_tensor_destroy(comet_tensor *t);

/* Allocate now everything that operations of rank <= R on this handle would otherwise allocate on
 * their first call: the carry / partial-sum scratch of the kernels and, for a coordinate list
 * ([CN,S], [CN,S,S]), the compressed copy that SpMV / SpMM / TTM / MTTKRP work through (one device
 * sort; synchronises with `stream`).  Afterwards those operations allocate nothing, except the
 * result handle of comet_ttv / comet_ttm when *Y is NULL.  R = 1 covers SpMV and TTV.
 * Errors: COMET_ERR_INVALID_ARG (null handle, R outside 1..1024), COMET_ERR_ALLOC. */
comet_status comet_tensor_reserve(comet_tensor *t, int64_t R, void *stream);

/* Fill *info (host) with the handle's description; pointers inside are device pointers that
 * stay valid until the handle is destroyed. */
comet_status comet_tensor_info(const comet_tensor *t, comet_tensor_info_t *info);

/*
 * Store X again with its modes in another level order, every level compressed-unique
 * ([CU,CU] for order 2, [CU,CU,CU] for order 3).  Section 4 ties each level to one mode and the
 * operations below contract (TTV, TTM) the mode of the LAST level or produce (MTTKRP) the mode of
 * the FIRST level, so this call is how the other modes are reached -- e.g. the first-mode TTV / TTM
 * that Section 8.2 writes out need the order {1, 2, 0}.  It also converts: an (even unsorted)
 * coordinate list [CN,S(,S)] or a CSR / DCSR matrix comes back as sorted CSF / DCSR, and the order
 * {1, 0} transposes a matrix.
 *
 *   X           handle of format [D,CU], [CU,CU], [CN,S], [CN,S,S] or [CU,CU,CU]; for a coordinate
 *               list the nonzeros may come in any order (create it without COMET_VALIDATE).
 *   mode_order  host, [order]; a permutation of X's modes: level l of the result stores mode
 *               mode_order[l] of the tensor (modes are numbered as in the tensor X was first
 *               created from, also when X itself is a reordered handle).
 *   out         host; receives a new handle that owns all its arrays (nothing is shared with X) and
 *               reports the order in comet_tensor_info_t::mode_of_level.  Its dims are per level.
 *
 * Work: one key/value radix sort of the nonzeros on the device plus a few streaming passes (two
 * sorts when the bit widths of the three mode sizes add up to more than 64, as for tensors whose
 * modes all run into the millions); temporary device memory of about 40 to 60 bytes per nonzero.
 * Synchronises with `stream`.
 * Errors: COMET_ERR_INVALID_ARG if mode_order is not a permutation; COMET_ERR_UNSUPPORTED if the
 * format is not listed above;
 * COMET_ERR_BAD_FORMAT if two nonzeros have the same coordinates (coordinates out of range are not
 * detected here: use COMET_VALIDATE at creation for sorted input).
 */
comet_status comet_tensor_reorder(const comet_tensor *X, const int32_t *mode_order, comet_tensor **out,
                                  void *stream);

/*
 * The same with a choice of the result's level formats: the conversion that the paper's runtime
 * function space_read() performs after reading a coordinate list (Section 5), on the device.
 *   levels   host, [order]; one of [CU,CU], [D,CU] (CSR), [CN,S] for order 2 and [CU,CU,CU],
 *            [CN,S,S] for order 3; a coordinate-list result is sorted and duplicate-free.
 * Other arguments, work and errors as for comet_tensor_reorder (which is this call with every
 * level CU); other level tuples give COMET_ERR_UNSUPPORTED.
 */
comet_status comet_tensor_convert(const comet_tensor *X, const int32_t *mode_order, const comet_level_t *levels,
                                  comet_tensor **out, void *stream);

/* SpMV, y = A x :  y_i = sum_j a_ij x_j   (Section 8.2, SpMV).
 *   A   order-2 handle, [D,CU] or [CU,CU]; a coordinate list [CN,S] is accepted too and works
 *       through a compressed copy built inside the handle on the first call (see comet_ttm).
 *   x   device, [dims[1]].          y   device, [dims[0]]; every entry is overwritten
 *                                       (rows without stored nonzeros become 0). */
comet_status comet_spmv(const comet_tensor *A, const double *x, double *y, void *stream);

/* SpMV for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same result as comet_spmv (the same kernels run), but the
 * kernels' carry scratch is a static device array of COMET_STATIC_SCRATCH_BYTES inside the library
 * (one copy per GPU, held until the process ends) instead of memory owned by the handle, and the call
 * makes no hipMalloc / hipFree or other allocating call.
 *   A   order-2 handle, [D,CU] or [CU,CU]; a coordinate list gives COMET_ERR_UNSUPPORTED (its compressed
 *       copy would have to be allocated).
 *   The kernels need about 24.4 bytes of scratch per 1024 nonzeros, so the array covers matrices of up
 *   to about 88 M nonzeros; a larger one gives COMET_ERR_UNSUPPORTED and nothing is enqueued.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *   streams, different threads) race -- serialise them.  Nothing in the array has to be cleared between
 *   calls (every entry that is read was written by the same call).  The first call on each device looks
 *   up the array's address, which is not a stream operation: make one call before starting a capture. */
#define COMET_STATIC_SCRATCH_BYTES (2u << 20)
comet_status comet_spmv_static(const comet_tensor *A, const double *x, double *y, void *stream);

/* SpMM, C = A B :  c_ir = sum_j a_ij b_jr   (Section 8.2, SpMM; the paper's example program).
 *   A   order-2 handle, [D,CU], [CU,CU] or (through a compressed copy) [CN,S].
 *   B   device, [dims[1] x R] row-major.   C   device, [dims[0] x R] row-major, overwritten.
 *   R   number of dense columns, 1 <= R <= 1024. */
comet_status comet_spmm(const comet_tensor *A, const double *B, int64_t R, double *C, void *stream);

/* SpTTV, Y = X x_mode v :  y_ij = sum_k x_ijk v_k   (Section 8.2, SpTTV).
 *   X     order-3 handle, [CU,CU,CU] or sorted [CN,S,S].
 *   mode  contracted mode (0, 1 or 2, numbered as in the original tensor); it must be the mode
 *         stored in the last level -- 2 unless the handle comes from comet_tensor_reorder -- else
 *         COMET_ERR_UNSUPPORTED.  Section 8.2's first-mode product y_jk = sum_i x_ijk v_i is
 *         comet_ttv(reorder(X, {1,2,0}), 0, v).
 *   v     device, [size of the contracted mode].
 *   Y     host; *Y must be NULL or a handle returned earlier by this call for the same X.
 *         On return *Y is an order-2 sparse result with the uncontracted levels of X:
 *         [CU,CU] whose pos/crd are X's level-0/1 arrays (shared, not copied) for CSF input,
 *         [CN,S] listing the distinct (i,j) in order for COO input.  One value per stored
 *         (i,j), kept even when the sum is exactly 0.  Release with comet_tensor_destroy. */
comet_status comet_ttv(const comet_tensor *X, int mode, const double *v, comet_tensor **Y, void *stream);

/* SpTTM, Y = X x_mode U :  y_ijr = sum_k x_ijk u_kr   (Section 8.2, SpTTM; R takes the place
 * of the contracted mode).
 *   X     order-3 handle, [CU,CU,CU] or sorted [CN,S,S].   mode  as for comet_ttv (the mode of the
 *         last level).  For a coordinate list the first call builds a compressed copy of X inside the
 *         handle (one device sort, about 16 more bytes per nonzero, kept until X is destroyed) and
 *         synchronises; the result is then [CN,S,D]: the distinct (i,j) as for comet_ttv, R values each.
 *         A [CU,CU,CU] tensor whose last mode has at most a few thousand coordinates and whose fibers of 256
 *         or more nonzeros hold a quarter of the nonzeros or more also keeps, from comet_tensor_create on, a
 *         compacted copy of all its other fibers (12 bytes per nonzero of them; see heavy_stream_bytes of
 *         comet_tensor_info): for R = 16 and 32 the long fibers are then computed with the rows of U in LDS.
 *   U     device, [size of the contracted mode x R] row-major, 1 <= R <= 1024.
 *   Y     as for comet_ttv; the result is [CU,CU,D] with dims (I, J, R): levels 0/1 shared
 *         with X, a dense last level of size R, vals of [#fibers x R] row-major (#fibers x R
 *         may exceed 2^31: no int32 array indexes the positions of a dense last level). */
comet_status comet_ttm(const comet_tensor *X, int mode, const double *U, int64_t R,
                       comet_tensor **Y, void *stream);

/* MTTKRP, M = X_(mode) (C (.) B) :  m_ir = sum_jk x_ijk b_jr c_kr.  The paper names the operation
 * (Section 8.3) without defining it; this is the usual definition with the output indexed by
 * the mode stored in the root level.
 *   X        order-3 handle, [CU,CU,CU] or sorted [CN,S,S] (which works through a compressed copy
 *            built on the first call, as described at comet_ttm).
 *   mode     output mode (numbered as in the original tensor); must be the mode stored in the root
 *            level -- 0 unless the handle comes from comet_tensor_reorder, e.g. {1,0,2} for mode 1
 *            -- else COMET_ERR_UNSUPPORTED.
 *   factors  host array of 3 device pointers indexed by MODE: factors[m] is the [size of mode m x R]
 *            row-major factor of mode m; factors[mode] is ignored.
 *   M        device, [size of mode `mode` x R] row-major, overwritten (rows without a stored
 *            slice = 0). */
comet_status comet_mttkrp(const comet_tensor *X, int mode, const double *const *factors,
                          int64_t R, double *M, void *stream);

/* Scaled and accumulating forms of the three products with a dense result (Section 6.2 Step III: the
 * generated code accumulates into the output, "C[...] += A[...] * B[...]"; alpha and beta are the usual
 * generalisation):
 *     y = alpha A x + beta y        C = alpha A B + beta C        M = alpha X_(mode) (C (.) B) + beta M
 * Arguments as for comet_spmv / comet_spmm / comet_mttkrp; the result array is read and written in place.
 * beta == 0: the old contents of the result are not read (they may be NaN); alpha == 0: the product is not
 * formed and the operands are not read.  beta == 1 accumulates.  The scaling is fused into the kernels'
 * stores (each result element is read and written once); rows that receive no contribution (empty rows,
 * rows absent from a compressed root level) become beta times their old value. */
comet_status comet_spmv_axpby(const comet_tensor *A, double alpha, const double *x, double beta, double *y, void *stream);
comet_status comet_spmm_axpby(const comet_tensor *A, double alpha, const double *B, int64_t R, double beta, double *C,
                              void *stream);
comet_status comet_mttkrp_axpby(const comet_tensor *X, int mode, double alpha, const double *const *factors, int64_t R,
                                double beta, double *M, void *stream);

/* Human-readable name of a status (static string). */
const char *comet_status_string(comet_status s);

/* Choose the kernel family used by later operations on this handle: 0 = automatic,
 * 1 = the simple one-lane-group-per-segment kernels, 2 = the nonzero-tiled streaming kernels with
 * all their specialisations, 3 = the nonzero-tiled kernels in their plain per-tile form only (no
 * operand staging in LDS, no heavy-row sweep): the baseline the specialisations are measured against.
 * For testing and measurement; results are the same up to summation order. */
comet_status comet_tensor_set_variant(comet_tensor *t, int variant);

/* Calibration of the device's memory system, for the benchmark (no tensor involved): the two access
 * patterns the operations are made of, timed by the caller.
 *   comet_calibrate_read    streams n doubles (n >= 2, data 16-byte aligned) once through the device.
 *   comet_calibrate_gather  lets lane groups of 8 gather `gathers` (rounded up to a multiple of 262144) whole
 *                           rows of R doubles (R = 16, 32 or 64) at pseudo-random row numbers from a
 *                           [nrows x R] row-major table (nrows < 2^29): L2-resident, cache-exceeding or
 *                           memory-resident according to the table's size.
 *   sink                    device, 1 double; never written for finite data (it keeps the loads alive). */
comet_status comet_calibrate_read(const double *data, int64_t n, double *sink, void *stream);
comet_status comet_calibrate_gather(const double *table, int64_t nrows, int64_t R, int64_t gathers, double *sink,
                                    void *stream);

#ifdef __cplusplus
}
#endif
#endif /* COMET_H */
