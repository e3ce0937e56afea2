/* ssam.h -- C ABI of the MI355X (gfx950) software-systolic structured-grid library.
 *
 * The library evaluates regular structured-grid kernels
 *        out[p] = sum_k  w_k * in[p + offset_k]
 * -- dense 2D filters (paper Sec. 2.1, evaluated as in Listing 1), 2D and 3D stencils
 * (Sec. 2.2) and their Jacobi iteration -- with the paper's execution model (Sec. 3.3,
 * Sec. 4): a register cache per lane, partial sums passed between the lanes of a
 * wavefront, overlapped blocking; re-designed for 64-lane CDNA4 wavefronts.
 *
 * Conventions common to every entry point
 *   - Grids are dense, row-major, x fastest:  index = (z*H + y)*W + x.  No pitch.
 *   - `d_*` arguments are DEVICE pointers owned by the caller; the library neither frees
 *     nor retains them.  They must hold W*H(*D) elements of the type named by `dtype`.
 *   - `h_*` arguments are HOST pointers, read synchronously during the call (they may be
 *     freed or changed as soon as the call returns), in the type named by `dtype`.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and the call returns without synchronising.  Launches on one stream are
 *     ordered; the caller synchronises before reading results.
 *   - The return value is the only error channel (an ssam_status).  All argument checks
 *     happen before any GPU call, so a bad call never touches the device.
 *   - Boundary rule: a read outside the grid gives 0 (SSAM_BOUNDARY_ZERO) or the value of
 *     the nearest grid point, every coordinate clamped on its own (SSAM_BOUNDARY_CLAMP).
 *     The paper does not state a rule; these are the two its comparison libraries use.
 *   - Results are deterministic run to run (the filter and stencil kernels use no atomics; the
 *     one-pass scan hands out work through an atomic counter but combines partial sums in a fixed
 *     order); the order of additions differs from a sequential sum, so results agree with a
 *     reference to rounding, not bitwise.
 *   - Thread safety: calls may be made from several host threads on different streams.
 *   - The compute entry points only enqueue kernels: no allocation, no memset, no synchronisation.
 *     They may therefore be recorded by stream capture into a HIP graph and replayed (the host
 *     arrays are read at capture time; make one ordinary call first so that one-time occupancy
 *     queries are not part of the capture).
 */
#ifndef SSAM_H_
#define SSAM_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SSAM_OK = 0,
    SSAM_ERR_NULL = 1,   /* a required pointer is NULL                                    */
    SSAM_ERR_DIM = 2,    /* W, H or D not positive or above SSAM_MAX_EXTENT, the grid exceeds
                            2^31-1 elements, or its tile plan exceeds what one launch holds
                            (3D grids of extreme aspect ratio, e.g. 1 x 2^30 x 2);
                            scan / probes: count out of range, misaligned pointer,
                            scratch or workspace too small                                */
    SSAM_ERR_SHAPE = 3,  /* filter / radius not positive, anchor outside the filter, or
                            larger than SSAM_MAX_FILTER / SSAM_MAX_RADIUS; steps < 0      */
    SSAM_ERR_ENUM = 4,   /* unknown dtype or boundary value                               */
    SSAM_ERR_ALIAS = 5,  /* input and output buffers overlap                              */
    SSAM_ERR_HIP = 6     /* a HIP runtime call failed (no device, launch failure)         */
} ssam_status;

typedef enum { SSAM_F32 = 0, SSAM_F64 = 1 } ssam_dtype;
typedef enum { SSAM_BOUNDARY_ZERO = 0, SSAM_BOUNDARY_CLAMP = 1 } ssam_boundary;

#define SSAM_MAX_FILTER 32   /* largest filter width or height accepted by ssam_conv2d   */
#define SSAM_MAX_RADIUS 8    /* largest stencil radius per axis                          */
#define SSAM_MAX_EXTENT (1 << 30)   /* largest W, H or D (and W*H*D at most 2^31-1)      */
#define SSAM_MAX_FILTER3D 17 /* largest extent of an ssam_conv3d filter along any axis   */

/* 2D filter (paper Sec. 2.1; Listing 1 evaluates it without flipping the filter):
 *     out[y][x] = sum_{n<N} sum_{m<M}  h_filter[n*M + m] * IN(x + m - ax, y + n - ay)
 * M is the filter width (x extent), N its height (y extent), as in the paper.  (ax, ay) is
 * the filter element placed on the output point; pass -1 for the default M/2, N/2 (integer
 * division).  The canonical flipped convolution of Sec. 2.1 is obtained by passing the
 * filter reversed in both axes.  d_in and d_out must not overlap. */
int ssam_conv2d(const void *d_in, void *d_out, int W, int H,
                const void *h_filter, int M, int N, int ax, int ay,
                int boundary, int dtype, void *hip_stream);

/* One sweep of a 2D stencil (paper Sec. 2.2, Listing 2):
 *     out[y][x] = sum_{|dy|<=ry} sum_{|dx|<=rx}  h_coef[(dy+ry)*(2rx+1) + (dx+rx)] * IN(x+dx, y+dy)
 * h_coef is the dense (2ry+1) x (2rx+1) coefficient box; an exactly-zero entry means that
 * offset is not part of the stencil (star shapes are boxes with zeros).  In the paper's
 * five-point naming: West = (dx,dy)=(-1,0), North = (0,-1), South = (0,+1), East = (+1,0). */
int ssam_stencil2d(const void *d_in, void *d_out, int W, int H,
                   const void *h_coef, int rx, int ry,
                   int boundary, int dtype, void *hip_stream);

/* One sweep of a 3D stencil (paper Sec. 2.2 last paragraph, Sec. 4.9):
 *     out[z][y][x] = sum  h_coef[((dz+rz)*(2ry+1) + (dy+ry))*(2rx+1) + (dx+rx)] * IN(x+dx, y+dy, z+dz)
 * with the same zero-means-no-tap rule; Above = dz -1, Below = dz +1.
 * Shapes with a compiled instance (or that fit zero-padded inside one: stars up to radius 4, boxes
 * up to radius 3) run on the register-cache kernels; any other, up to SSAM_MAX_RADIUS per axis, runs
 * on a direct one-point-per-thread kernel (correct, not fast) whose taps travel in the launch
 * arguments, in as many launches on hip_stream as the tap count needs. */
int ssam_stencil3d(const void *d_in, void *d_out, int W, int H, int D,
                   const void *h_coef, int rx, int ry, int rz,
                   int boundary, int dtype, void *hip_stream);

/* 3D filter: the 2D filter of Sec. 2.1 with a third index, the mapping the paper names as its next
 * (Sec. 6, opening paragraph; Sec. 8), evaluated without a flip like the 2D one:
 *     out[z][y][x] = sum_{k<K} sum_{n<N} sum_{m<M}  h_filter[(k*N + n)*M + m] * IN(x + m - ax, y + n - ay, z + k - az)
 * M, N, K are the filter's extents along x, y, z, each 1 .. SSAM_MAX_FILTER3D, even sizes included;
 * (ax, ay, az) is the filter element placed on the output point, -1 for the default M/2, N/2, K/2.
 * Every element of the filter is a tap (a zero multiplies, it is not skipped).  Filters that fit a cube
 * of radius 1, 2 or 3 around their anchor run on the register-cache kernels (3x3x3, 5x5x5, 7x7x7 as
 * they are, anything else zero-padded inside the smallest such cube); larger ones run on the direct
 * one-point-per-thread kernel (correct, not fast).  d_in and d_out must not overlap. */
int ssam_conv3d(const void *d_in, void *d_out, int W, int H, int D,
                const void *h_filter, int M, int N, int K, int ax, int ay, int az,
                int boundary, int dtype, void *hip_stream);

/* `steps` Jacobi sweeps (paper Sec. 2.2: s_{i+1} computed from s_i) with two buffers, each
 * launch reading one and writing the other; every grid point is updated each sweep, the
 * boundary rule supplying reads outside the grid.  D == 1 with rz == 0 is the 2D case.
 * A launch performs one sweep, or -- where the shape has a compiled multi-sweep instance (2D,
 * either boundary rule: up to 8 sweeps; 3D radius 1 and 2: two, under the clamp rule the
 * 7-point star only) -- several sweeps with the intermediate fields held in registers (temporal
 * blocking, which Sec. 6.4 says the model permits); the result is the same field to rounding
 * either way.
 * *d_result (host location, may be NULL) receives the buffer that holds the field after
 * `steps` sweeps: d_a when the number of LAUNCHES is even (steps == 0 does nothing), d_b when
 * it is odd -- read it rather than infer it from `steps`.  Both buffers are overwritten when
 * more than one launch runs.  No host synchronisation happens between sweeps. */
int ssam_stencil_iterate(void *d_a, void *d_b, int W, int H, int D,
                         const void *h_coef, int rx, int ry, int rz,
                         int boundary, int dtype, int steps,
                         void *hip_stream, void **d_result);

/* Human-readable name of an ssam_status value (static storage; never NULL). */
const char *ssam_status_string(int status);

/* Planning query, host only (nothing is launched, no pointer is dereferenced except h_coef):
 * writes a NUL-terminated description of the kernel instance and tile geometry the
 * dispatcher would use -- e.g. "float_M3N3_b2_v4p8 V=4 P=8 halo_lanes=1+1 valid_lanes=61
 * strips_x=34 ..." -- into buf (at most buflen bytes).  kind 0 = ssam_conv2d with (a, b) =
 * (M, N) and the default anchor; kind 1 = ssam_stencil2d with (a, b) = (rx, ry); kind 2 =
 * ssam_stencil3d with (a, b, c) = (rx, ry, rz); kind 3 = the launch ssam_stencil_iterate uses
 * on a 2D grid with (a, b) = (rx, ry) while c sweeps remain (c <= 0: many); an instance named
 * "..._fusedS" performs S sweeps; kind 4 = the same for a 3D grid with (a, b, c) = (rx, ry, rz)
 * while two or more sweeps remain; kind 5 = ssam_conv3d with (a, b, c) = (M, N, K) and the default
 * anchor.  The tile plan follows the paper's overlapped
 * blocking (Sec. 4.5, Sec. 4.7) re-derived for 64 lanes of V columns each. */
int ssam_describe(int kind, int W, int H, int D, const void *h_coef, int a, int b, int c,
                  int boundary, int dtype, char *buf, int buflen);

/* Inclusive scan of a 1D array, b_i = a_0 + a_1 + ... + a_i for 0 <= i < n (Sec. 3.6: partial
 * sums shifted between the lanes of a wave, every lane holding several consecutive elements in
 * registers).  d_in, d_out: device, n contiguous elements of dtype, aligned to the element
 * size (16-byte alignment of both selects the vector-access kernels); d_out may be the same
 * pointer as d_in (in place), any other overlap gives SSAM_ERR_ALIAS.  d_work: device
 * workspace of at least ssam_scan_workspace_bytes(n, dtype) bytes, 8-byte aligned, not
 * overlapping the arrays, owned by the caller, contents irrelevant on entry, free for reuse once
 * the call's work on hip_stream has finished (two calls in flight must not share one); it may be
 * NULL when that size is 0 (short arrays).  The call enqueues its launches on hip_stream and
 * returns without waiting and without allocating; no memset is enqueued, so it can be captured.
 * Schedules, chosen by size:
 *   - one workgroup, one launch (up to 128 KiB; no workspace);
 *   - three launches (below 128 MiB, and always in place beyond 128 KiB): the array is cut into contiguous
 *     segments, one per wave; segment sums, their exclusive prefixes, the scan of every segment
 *     (2 reads + 1 write per element);
 *   - one pass (from 128 MiB, out of place, up to 2^30 fp32 / 2^29 fp64 elements): every wave
 *     keeps a segment in registers, publishes its sum in the workspace and combines the sums of
 *     the waves before it, always in the same order (1 read + 1 write per element, results
 *     reproducible run to run).  Waves take segments from a ticket counter, so they only wait
 *     for waves already running, and every wait is bounded: if a wave runs out of polls (a
 *     device shared with other work) it raises a flag, 8-byte word 16 of the workspace, and a
 *     one-workgroup kernel enqueued behind the pass (it returns at once otherwise) redoes the
 *     array, slowly (about 30 ms per GiB).
 * Totals that cross a 64-lane step are carried in fp64 for both element types, so the result is
 * within a few roundings of the element type of the exact prefix, relative to the sum of
 * magnitudes.  A non-finite partial sum makes the later results non-finite (an infinity may read
 * as NaN).  n == 0 is a no-op.  Errors: SSAM_ERR_ENUM (dtype), SSAM_ERR_DIM (n < 0 or above
 * 2^40, misaligned pointer, workspace too small), SSAM_ERR_NULL, SSAM_ERR_ALIAS, SSAM_ERR_HIP. */
int ssam_scan(const void *d_in, void *d_out, long long n, int dtype,
              void *d_work, size_t work_bytes, void *hip_stream);

/* Host only: bytes of workspace ssam_scan needs for n elements of dtype under the current
 * tuning, whichever schedule the pointers then select (at most about 2.1 MiB; 0 when one segment
 * suffices or the arguments are invalid). */
size_t ssam_scan_workspace_bytes(long long n, int dtype);

/* ssam_scan for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * ssam_scan on the same arguments (same kernels, same schedules), with the workspace taken from an
 * array the library holds in device memory (about 2.1 MiB on every GPU it runs on, until the
 * process ends) instead of a d_work argument.  The call allocates nothing and frees nothing; its
 * first call on a device looks the array's address up once.  What must start at zero is cleared by
 * a kernel on hip_stream, so earlier calls leave nothing behind.  All calls on one GPU share the
 * one array: two calls whose work overlaps in time on the same GPU (different streams, or several
 * host threads) race -- serialise them, or give ssam_scan workspaces of their own.
 * n above SSAM_SCAN_STATIC_MAX_ELEMENTS gives SSAM_ERR_DIM (use ssam_scan); the other errors are
 * ssam_scan's. */
#define SSAM_SCAN_STATIC_MAX_ELEMENTS (1LL << 32)
int ssam_scan_static(const void *d_in, void *d_out, long long n, int dtype, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SSAM_H_ */
