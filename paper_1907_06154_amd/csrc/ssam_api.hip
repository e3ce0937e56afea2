// C ABI of the library: argument validation, shape classification, dispatch to the compiled
// register-cache instances, the direct fallback kernel for every other shape, Jacobi
// ping-pong, tuning overrides.  All validation happens before the first HIP call.
#include <atomic>
#include <cstdint>
#include <cstring>
#include <string>

#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {

std::vector<Instance2D>& registry2d()
{
    static std::vector<Instance2D> r;
    return r;
}
std::vector<Instance3D>& registry3d()
{
    static std::vector<Instance3D> r;
    return r;
}

namespace {

constexpr int kMaxFusedSweeps = 8;
constexpr long long kFuseTwoMinPoints = 1LL << 22;
std::atomic<int> g_rows_per_wave{-1}, g_valid_lanes{-1}, g_planes_per_wave{-1}, g_xcd_remap{-1},
    g_force_generic{-1}, g_variant{-1}, g_march_axis{-1}, g_fuse_sweeps{-1}, g_embed_waste{-1};

Tuning current_tuning()
{
    Tuning t;
    t.rows_per_wave = g_rows_per_wave.load();
    t.valid_lanes = g_valid_lanes.load();
    t.planes_per_wave = g_planes_per_wave.load();
    t.xcd_remap = g_xcd_remap.load();
    t.force_generic = g_force_generic.load();
    t.variant = g_variant.load();
    t.march_axis = g_march_axis.load();
    t.fuse_sweeps = g_fuse_sweeps.load();
    t.embed_waste = g_embed_waste.load();
    return t;
}

// ---- direct fallback kernel -------------------------------------------------------------
// One output point per thread, taps read straight from global memory (cached).  It keeps the
// ABI total: any filter or stencil shape without a compiled register-cache instance runs
// here.  The taps travel in the kernel-argument block as a list of (coefficient, offset) pairs --
// for a stencil only the non-zero ones, so a star of any radius is a short list.  A list too long
// for one argument block is evaluated by several launches on the same stream, the first writing
// the partial sum of its part, every later one adding its own part to what the output holds
// (each thread only ever touches its own output element).
constexpr int kGenericBytes = 3584;

template <typename T>
struct GenericArgs {
    static constexpr int kCap = kGenericBytes / (sizeof(T) + sizeof(int));
    const T* in;
    T* out;
    int W, H, D;
    int boundary;
    int ntaps;         // taps in this launch
    int accumulate;    // 1: add to the value the output already holds
    long long nblocks; // blocks of 64 x 4 points in the grid
    T w[kCap];
    int off[kCap];     // dx, dy, dz as signed bytes 0, 1, 2
};

template <typename T>
__device__ __forceinline__ T fetch(const GenericArgs<T>& a, int x, int y, int z)
{
    if (a.boundary == kClamp) {
        x = min(max(x, 0), a.W - 1);
        y = min(max(y, 0), a.H - 1);
        z = min(max(z, 0), a.D - 1);
    } else if (x < 0 || x >= a.W || y < 0 || y >= a.H || z < 0 || z >= a.D) {
        return T(0);
    }
    return a.in[((size_t)z * a.H + y) * a.W + x];
}

template <typename T>
__global__ __launch_bounds__(256) void generic_kernel(const GenericArgs<T> a)
{
    // blocks of 64 x 4 points, numbered x fastest; the launched blocks stride over them (a tall
    // or deep grid has more of them than one launch dimension takes)
    const long long nbx = (a.W + 63) / 64, nby = (a.H + 3) / 4;
    for (long long b = blockIdx.x; b < a.nblocks; b += gridDim.x) {
        const int x = (int)(b % nbx) * 64 + (threadIdx.x & 63);
        const int y = (int)((b / nbx) % nby) * 4 + (threadIdx.x >> 6);
        const int z = (int)(b / nbx / nby);
        if (x >= a.W || y >= a.H) continue;
        T* o = a.out + ((size_t)z * a.H + y) * a.W + x;
        T sum = a.accumulate ? *o : T(0);
        for (int t = 0; t < a.ntaps; ++t) {
            const int off = a.off[t];
            sum = fma_t(a.w[t], fetch(a, x + (int)(signed char)(off & 0xff), y + (int)(signed char)((off >> 8) & 0xff),
                                      z + (int)(signed char)((off >> 16) & 0xff)), sum);
        }
        *o = sum;
    }
}

// Largest number of simultaneously non-zero offset components among the taps (0..3).
template <typename T>
int tap_budget(const T* c, int M, int N, int K, int ax, int ay, int az)
{
    int b = 0;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            for (int m = 0; m < M; ++m)
                if (c[(k * N + n) * M + m] != T(0)) {
                    const int u = (k != az) + (n != ay) + (m != ax);
                    if (u > b) b = u;
                }
    return b;
}

template <typename T>
hipError_t launch_generic(const T* in, T* out, int W, int H, int D, const T* c, int M, int N, int K, int ax,
                          int ay, int az, int boundary, bool skip_zero, hipStream_t stream)
{
    GenericArgs<T> a;
    a.in = in;
    a.out = out;
    a.W = W; a.H = H; a.D = D;
    a.boundary = boundary;
    a.nblocks = (long long)ceil_div(W, 64) * ceil_div(H, 4) * D;
    const unsigned grid = (unsigned)(a.nblocks < (1LL << 20) ? a.nblocks : (1LL << 20));
    a.ntaps = 0;
    a.accumulate = 0;
    auto flush = [&]() {
        hipLaunchKernelGGL(generic_kernel<T>, dim3(grid), dim3(256), 0, stream, a);
        a.ntaps = 0;
        a.accumulate = 1;
        return hipGetLastError();
    };
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            for (int m = 0; m < M; ++m) {
                const T v = c[((size_t)k * N + n) * M + m];
                if (skip_zero && v == T(0)) continue;
                a.w[a.ntaps] = v;
                a.off[a.ntaps] = ((m - ax) & 0xff) | (((n - ay) & 0xff) << 8) | (((k - az) & 0xff) << 16);
                if (++a.ntaps == GenericArgs<T>::kCap)
                    if (hipError_t e = flush()) return e;
            }
    if (a.ntaps > 0 || !a.accumulate)      // the last part; a stencil without any tap still writes zeros
        if (hipError_t e = flush()) return e;
    return hipSuccess;
}

// ---- plain copy (measurement aid) ---------------------------------------------------------
// 16 bytes per lane, grid-stride: a reference rate for 1-read-1-write kernels (tile-shaped
// access with streaming stores exceeds it), and the known-size reference the hardware traffic
// counters are scaled by.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) out[i] = in[i];
}

// ---- validation helpers ------------------------------------------------------------------
int check_enums(int boundary, int dtype)
{
    if (boundary != SSAM_BOUNDARY_ZERO && boundary != SSAM_BOUNDARY_CLAMP) return SSAM_ERR_ENUM;
    if (dtype != SSAM_F32 && dtype != SSAM_F64) return SSAM_ERR_ENUM;
    return SSAM_OK;
}

int check_dims(int W, int H, int D)
{
    if (W <= 0 || H <= 0 || D <= 0) return SSAM_ERR_DIM;
    if (W > SSAM_MAX_EXTENT || H > SSAM_MAX_EXTENT || D > SSAM_MAX_EXTENT) return SSAM_ERR_DIM;
    if ((long long)W * H * D > 2147483647LL) return SSAM_ERR_DIM;
    return SSAM_OK;
}

bool overlap(const void* a, const void* b, size_t bytes)
{
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + bytes && pb < pa + bytes;
}

size_t elem(int dtype) { return dtype == SSAM_F32 ? 4 : 8; }

// A launcher reports a tile plan that no launch can hold (more blocks than a grid dimension takes:
// grids of extreme aspect ratio) as hipErrorInvalidConfiguration, before it launches anything.
int status_of(hipError_t e)
{
    return e == hipSuccess ? SSAM_OK : e == hipErrorInvalidConfiguration ? SSAM_ERR_DIM : SSAM_ERR_HIP;
}

// ---- dispatch ---------------------------------------------------------------------------
template <typename T>
const Instance2D* pick2d(const Problem2D& p, bool stencil_semantics, int want_variant, int sweeps = 1,
                         bool any_depth = false)
{
    const T* w = static_cast<const T*>(p.w);
    int budget = 2;
    if (stencil_semantics) {
        budget = tap_budget<T>(w, p.M, p.N, 1, p.ax, p.ay, 0);
        if (budget == 0) budget = 1;
    }
    const Instance2D* best = nullptr;
    for (const Instance2D& i : registry2d()) {
        if (i.dtype != p.dtype || i.M != p.M || i.N != p.N || i.AX != p.ax) continue;
        if (i.budget < budget) continue;
        if (i.budget == 1 && p.ay != p.N / 2) continue;   // star instances assume the centre row
        if (i.variant != want_variant) continue;
        if (any_depth ? i.sweeps < 2 : i.sweeps != sweeps) continue;
        if (!best || i.budget < best->budget) best = &i;
    }
    return best;
}

int run2d(const Problem2D& p, bool stencil_semantics, Geometry* geo, bool dry, std::string* name)
{
    const Tuning tu = current_tuning();
    const Instance2D* inst = nullptr;
    if (tu.force_generic <= 0)
    {
        const int v = tu.variant > 0 ? tu.variant : 0;
        inst = p.dtype == SSAM_F32 ? pick2d<float>(p, stencil_semantics, v) : pick2d<double>(p, stencil_semantics, v);
        if (!inst && v != 0)   // no such alternative for this shape: use the default instance
            inst = p.dtype == SSAM_F32 ? pick2d<float>(p, stencil_semantics, 0) : pick2d<double>(p, stencil_semantics, 0);
    }
    if (inst) {
        if (name) *name = inst->name;
        return status_of(inst->launch(p, tu, geo, dry));
    }
    // No instance of this exact shape (a non-square filter, an anchor off the centre, unequal
    // radii): embed it in the smallest compiled square box whose centre anchor leaves enough room
    // on every side.  The added zero weights cost arithmetic, but even a 1x20 filter inside the 20x20
    // box measured faster than the direct kernel, so there is no limit unless "embed_waste" sets one.
    if (tu.force_generic <= 0) {
        const int need_lo = p.ax > p.ay ? p.ax : p.ay;
        const int hi_x = p.M - 1 - p.ax, hi_y = p.N - 1 - p.ay;
        const int need_hi = hi_x > hi_y ? hi_x : hi_y;
        const Instance2D* box = nullptr;
        for (const Instance2D& i : registry2d()) {
            if (i.dtype != p.dtype || i.M != i.N || i.budget != 2 || i.variant != 0 || i.sweeps != 1) continue;
            if (i.AX != i.M / 2 || i.M / 2 < need_lo || i.M - 1 - i.M / 2 < need_hi) continue;
            if (!box || i.M < box->M) box = &i;
        }
        if (box && (tu.embed_waste < 0 || box->M * box->N <= tu.embed_waste * p.M * p.N)) {
            const int K = box->M, c = K / 2;
            const size_t es = elem(p.dtype);
            std::vector<char> padded((size_t)K * K * es, 0);
            const char* src = static_cast<const char*>(p.w);
            for (int n = 0; n < p.N; ++n)
                memcpy(&padded[((size_t)(n + c - p.ay) * K + (c - p.ax)) * es], src + (size_t)n * p.M * es,
                       (size_t)p.M * es);
            Problem2D q = p;
            q.M = q.N = K;
            q.ax = q.ay = c;
            q.w = padded.data();
            if (name) *name = std::string(box->name) + "+embedded";
            return status_of(box->launch(q, tu, geo, dry));   // weights are copied into the launch arguments
        }
    }
    if (name) *name = "generic_direct";
    if (geo) {
        *geo = Geometry();
        geo->blocks = ceil_div(p.W, 64) * ceil_div(p.H, 4);
    }
    if (dry) return SSAM_OK;
    hipError_t e = p.dtype == SSAM_F32
                       ? launch_generic<float>((const float*)p.in, (float*)p.out, p.W, p.H, 1, (const float*)p.w, p.M,
                                               p.N, 1, p.ax, p.ay, 0, p.boundary, stencil_semantics, p.stream)
                       : launch_generic<double>((const double*)p.in, (double*)p.out, p.W, p.H, 1, (const double*)p.w,
                                                p.M, p.N, 1, p.ax, p.ay, 0, p.boundary, stencil_semantics, p.stream);
    return status_of(e);
}

template <typename T>
const Instance3D* pick3d(const Problem3D& p, int want_variant, int sweeps = 1)
{
    const T* c = static_cast<const T*>(p.c);
    int budget = p.dense ? 3 : tap_budget<T>(c, 2 * p.rx + 1, 2 * p.ry + 1, 2 * p.rz + 1, p.rx, p.ry, p.rz);
    if (budget == 0) budget = 1;
    // an instance is compiled for (reach along x, along the strip axis, along the march axis)
    const int strip_r = p.march_y ? p.rz : p.ry, march_r = p.march_y ? p.ry : p.rz;
    const Instance3D* best = nullptr;
    for (const Instance3D& i : registry3d()) {
        if (i.dtype != p.dtype || i.rx != p.rx || i.ry != strip_r || i.rz != march_r || i.budget < budget) continue;
        if (i.variant != want_variant || i.sweeps != sweeps) continue;
        if (!best || i.budget < best->budget) best = &i;
    }
    return best;
}

// Several sweeps in one launch, where the shape has a fused instance (zero padding; 3D only when
// marching along z): the deepest compiled one that does not exceed `max_sweeps` (the sweeps still
// to do) nor the "fuse_sweeps" cap.  Returns the number of sweeps the launch performs, 0 when the
// caller should run a single sweep instead.
int run_fused(const Problem3D& p, int max_sweeps, Geometry* geo, bool dry, std::string* name, int* rc)
{
    const Tuning tu = current_tuning();
    if (tu.fuse_sweeps == 0 || tu.fuse_sweeps == 1 || tu.force_generic > 0) return 0;
    if (tu.fuse_sweeps > 1 && tu.fuse_sweeps < max_sweeps) max_sweeps = tu.fuse_sweeps;
    if (max_sweeps > kMaxFusedSweeps) max_sweeps = kMaxFusedSweeps;
    const int v = tu.variant > 0 ? tu.variant : 0;
    const bool flat = p.D == 1 && p.rz == 0;
    if (!flat && tu.march_axis == 1) return 0;   // 3D: z march only
    // Two sweeps per launch pay only on grids large enough to be bandwidth-bound (measured: from about
    // 4M points); on smaller ones the fatter, fewer tiles lose more than the saved launch gains.  Three
    // sweeps and more per launch were faster at every size tried (256^2 upwards).
    const bool small = (long long)p.W * p.H * p.D < kFuseTwoMinPoints && tu.fuse_sweeps < 0;
    Problem2D q{p.in, p.out, p.W, p.H, p.c, 2 * p.rx + 1, 2 * p.ry + 1, p.rx, p.ry, p.boundary, p.dtype, p.stream};
    // the tightest tap shape any multi-sweep instance offers for this stencil: a deeper instance of a
    // wider shape (a box standing in for a star) is not taken over a shallower one of the exact shape
    int shape_budget = 0;
    if (flat) {
        const Instance2D* tight = p.dtype == SSAM_F32 ? pick2d<float>(q, true, 0, 0, true) : pick2d<double>(q, true, 0, 0, true);
        if (!tight) return 0;
        shape_budget = tight->budget;
    }
    for (int sweeps = max_sweeps; sweeps >= 2; --sweeps) {
        if (sweeps == 2 && small) break;
        hipError_t e;
        if (flat) {
            const Instance2D* inst = p.dtype == SSAM_F32 ? pick2d<float>(q, true, v, sweeps) : pick2d<double>(q, true, v, sweeps);
            if ((!inst || inst->budget != shape_budget) && v != 0)
                inst = p.dtype == SSAM_F32 ? pick2d<float>(q, true, 0, sweeps) : pick2d<double>(q, true, 0, sweeps);
            if (!inst || inst->budget != shape_budget) continue;
            if (name) *name = inst->name;
            e = inst->launch(q, tu, geo, dry);
        } else {
            const Instance3D* inst = p.dtype == SSAM_F32 ? pick3d<float>(p, v, sweeps) : pick3d<double>(p, v, sweeps);
            if (!inst && v != 0) inst = p.dtype == SSAM_F32 ? pick3d<float>(p, 0, sweeps) : pick3d<double>(p, 0, sweeps);
            if (!inst || (p.boundary == SSAM_BOUNDARY_CLAMP && !inst->fuses_clamp)) continue;
            if (name) *name = inst->name;
            e = inst->launch(p, tu, geo, dry);
        }
        *rc = status_of(e);
        return sweeps;
    }
    return 0;
}

int run3d(const Problem3D& p_in, Geometry* geo, bool dry, std::string* name)
{
    const Tuning tu = current_tuning();
    Problem3D p = p_in;
    p.march_y = tu.march_axis == 1;
    if (p.D == 1 && p.rz == 0) {   // a 2D problem through the 3D door
        Problem2D q{p.in, p.out, p.W, p.H, p.c, 2 * p.rx + 1, 2 * p.ry + 1, p.rx, p.ry, p.boundary, p.dtype, p.stream};
        return run2d(q, true, geo, dry, name);
    }
    // Taps a compiled shape evaluates: what a launch costs in arithmetic.
    auto taps = [](const Instance3D& i) {
        const long n = 2 * i.rx + 1;
        return i.budget == 1 ? 6L * i.rx + 1 : i.budget == 2 ? n * n * n - 8L * i.rx * i.rx * i.rx : n * n * n;
    };
    const Instance3D* inst = nullptr;   // an instance of exactly these radii
    const Instance3D* cube = nullptr;   // the cheapest compiled shape of equal radii that covers the box, zero-padded
    if (tu.force_generic <= 0) {
        const int v = tu.variant > 0 ? tu.variant : 0;
        inst = p.dtype == SSAM_F32 ? pick3d<float>(p, v) : pick3d<double>(p, v);
        if (!inst && v != 0) inst = p.dtype == SSAM_F32 ? pick3d<float>(p, 0) : pick3d<double>(p, 0);
        if (tu.embed_waste != 0) {
            const int budget = p.dense ? 3 : p.dtype == SSAM_F32
                                   ? tap_budget<float>((const float*)p.c, 2 * p.rx + 1, 2 * p.ry + 1, 2 * p.rz + 1, p.rx, p.ry, p.rz)
                                   : tap_budget<double>((const double*)p.c, 2 * p.rx + 1, 2 * p.ry + 1, 2 * p.rz + 1, p.rx, p.ry, p.rz);
            const int need = p.rx > p.ry ? (p.rx > p.rz ? p.rx : p.rz) : (p.ry > p.rz ? p.ry : p.rz);
            for (const Instance3D& i : registry3d()) {
                if (i.dtype != p.dtype || i.rx != i.ry || i.ry != i.rz || i.rx < need || i.budget < budget) continue;
                if (i.variant != 0 || i.sweeps != 1) continue;
                if (!cube || taps(i) < taps(*cube)) cube = &i;
            }
        }
    }
    // The exact instance unless a padded one evaluates fewer taps (a radius-3 star has no instance of
    // its own: the radius-4 star, 25 taps, beats the radius-3 box, 343); whichever is tried first, a
    // launcher that does not take this grid (hipErrorNotSupported) leaves the turn to the other.
    const bool cube_first = cube && cube != inst && (!inst || taps(*cube) < taps(*inst));
    for (int attempt = 0; attempt < 2; ++attempt) {
        const bool use_cube = (attempt == 0) == cube_first;
        if (!use_cube && inst) {
            if (name) *name = inst->name;
            const hipError_t e = inst->launch(p, tu, geo, dry);
            if (e != hipErrorNotSupported) return status_of(e);
        }
        if (use_cube && cube && cube != inst) {
            const int R = cube->rx, K = 2 * R + 1;
            const int M = 2 * p.rx + 1, N = 2 * p.ry + 1, L = 2 * p.rz + 1;
            const size_t es = elem(p.dtype);
            std::vector<char> padded((size_t)K * K * K * es, 0);
            const char* src = static_cast<const char*>(p.c);
            for (int k = 0; k < L; ++k)
                for (int n = 0; n < N; ++n)
                    memcpy(&padded[((((size_t)(k + R - p.rz) * K) + (n + R - p.ry)) * K + (R - p.rx)) * es],
                           src + ((size_t)k * N + n) * M * es, (size_t)M * es);
            Problem3D q = p;
            q.rx = q.ry = q.rz = R;
            q.c = padded.data();
            if (name) *name = std::string(cube->name) + "+embedded";
            const hipError_t e = cube->launch(q, tu, geo, dry);   // the coefficients are copied into the launch arguments
            if (e != hipErrorNotSupported) return status_of(e);
        }
    }
    if (name) *name = "generic_direct";
    if (geo) {
        *geo = Geometry();
        geo->blocks = ceil_div(p.W, 64) * ceil_div(p.H, 4) * p.D;
    }
    const int M = 2 * p.rx + 1, N = 2 * p.ry + 1, K = 2 * p.rz + 1;
    if (dry) return SSAM_OK;
    hipError_t e = p.dtype == SSAM_F32
                       ? launch_generic<float>((const float*)p.in, (float*)p.out, p.W, p.H, p.D, (const float*)p.c, M,
                                               N, K, p.rx, p.ry, p.rz, p.boundary, !p.dense, p.stream)
                       : launch_generic<double>((const double*)p.in, (double*)p.out, p.W, p.H, p.D,
                                                (const double*)p.c, M, N, K, p.rx, p.ry, p.rz, p.boundary, !p.dense,
                                                p.stream);
    return status_of(e);
}

// 3D filter of extents (M, N, K) anchored at (ax, ay, az).  A cube of odd extent anchored at its
// centre is the dense coefficient box of a stencil and runs on the compiled box instances (radius 1, 2, 3);
// any other filter that fits such a cube around its anchor runs zero-padded inside the smallest one
// (as 2D filters without an instance of their own do); the rest runs on the direct kernel, which
// takes extents and anchor as they are.
int run_conv3d(const void* in, void* out, int W, int H, int D, const void* f, int M, int N, int K, int ax, int ay,
               int az, int boundary, int dtype, hipStream_t stream, Geometry* geo, bool dry, std::string* name)
{
    const Tuning tu = current_tuning();
    const int lo = ax > ay ? (ax > az ? ax : az) : (ay > az ? ay : az);
    const int hx = M - 1 - ax, hy = N - 1 - ay, hz = K - 1 - az;
    const int hi = hx > hy ? (hx > hz ? hx : hz) : (hy > hz ? hy : hz);
    const int R = lo > hi ? lo : hi;
    const size_t es = elem(dtype);
    // zero padding costs arithmetic: a cube with more than 8 times the filter's taps (or the "embed_waste"
    // override) is left to the direct kernel
    const long waste = tu.embed_waste > 0 ? tu.embed_waste : 8;
    if (R >= 1 && R <= 3 && tu.force_generic <= 0 && tu.embed_waste != 0 &&
        (long)(2 * R + 1) * (2 * R + 1) * (2 * R + 1) <= waste * M * N * K) {
        const int S = 2 * R + 1;
        std::vector<char> cube((size_t)S * S * S * es, 0);
        const char* src = static_cast<const char*>(f);
        for (int k = 0; k < K; ++k)
            for (int n = 0; n < N; ++n)
                memcpy(&cube[((((size_t)(k - az + R) * S) + (n - ay + R)) * S + (R - ax)) * es],
                       src + ((size_t)k * N + n) * M * es, (size_t)M * es);
        Problem3D p{in, out, W, H, D, cube.data(), R, R, R, boundary, dtype, stream};
        p.dense = true;
        std::string inner;
        const int rc = run3d(p, geo, dry, &inner);
        if (inner != "generic_direct") {     // a compiled instance took it (the coefficients are copied into the launch arguments)
            if (name) *name = (M == S && N == S && K == S) ? inner : inner + "+embedded";
            return rc;
        }
    }
    if (name) *name = "generic_direct";
    if (geo) {
        *geo = Geometry();
        geo->blocks = ceil_div(W, 64) * ceil_div(H, 4) * D;
    }
    if (dry) return SSAM_OK;
    const hipError_t e = dtype == SSAM_F32
                             ? launch_generic<float>((const float*)in, (float*)out, W, H, D, (const float*)f, M, N, K, ax, ay,
                                                     az, boundary, false, stream)
                             : launch_generic<double>((const double*)in, (double*)out, W, H, D, (const double*)f, M, N, K,
                                                      ax, ay, az, boundary, false, stream);
    return status_of(e);
}

// Everything but the grid pointers (the planning query has none).
int check_conv3d(int W, int H, int D, const void* f, int M, int N, int K, int* ax, int* ay, int* az, int boundary,
                 int dtype)
{
    if (!f) return SSAM_ERR_NULL;
    if (int e = check_enums(boundary, dtype)) return e;
    if (int e = check_dims(W, H, D)) return e;
    if (M <= 0 || N <= 0 || K <= 0 || M > SSAM_MAX_FILTER3D || N > SSAM_MAX_FILTER3D || K > SSAM_MAX_FILTER3D)
        return SSAM_ERR_SHAPE;
    if (*ax == -1) *ax = M / 2;
    if (*ay == -1) *ay = N / 2;
    if (*az == -1) *az = K / 2;
    if (*ax < 0 || *ax >= M || *ay < 0 || *ay >= N || *az < 0 || *az >= K) return SSAM_ERR_SHAPE;
    return SSAM_OK;
}

int validate_conv(const void* in, const void* out, int W, int H, const void* f, int M, int N, int* ax, int* ay,
                  int boundary, int dtype)
{
    if (!in || !out || !f) return SSAM_ERR_NULL;
    if (int e = check_enums(boundary, dtype)) return e;
    if (int e = check_dims(W, H, 1)) return e;
    if (M <= 0 || N <= 0 || M > SSAM_MAX_FILTER || N > SSAM_MAX_FILTER) return SSAM_ERR_SHAPE;
    if (*ax == -1) *ax = M / 2;
    if (*ay == -1) *ay = N / 2;
    if (*ax < 0 || *ax >= M || *ay < 0 || *ay >= N) return SSAM_ERR_SHAPE;
    if (overlap(in, out, (size_t)W * H * elem(dtype))) return SSAM_ERR_ALIAS;
    return SSAM_OK;
}

int validate_stencil(const void* in, const void* out, int W, int H, int D, const void* c, int rx, int ry, int rz,
                     int boundary, int dtype)
{
    if (!in || !out || !c) return SSAM_ERR_NULL;
    if (int e = check_enums(boundary, dtype)) return e;
    if (int e = check_dims(W, H, D)) return e;
    if (rx < 0 || ry < 0 || rz < 0 || rx > SSAM_MAX_RADIUS || ry > SSAM_MAX_RADIUS || rz > SSAM_MAX_RADIUS)
        return SSAM_ERR_SHAPE;
    if (overlap(in, out, (size_t)W * H * D * elem(dtype))) return SSAM_ERR_ALIAS;
    return SSAM_OK;
}

int describe(int rc, const std::string& name, const Geometry& g, char* buf, int buflen)
{
    if (buf && buflen > 0) {
        snprintf(buf, (size_t)buflen,
                 "%s V=%d P=%d halo_lanes=%d+%d valid_lanes=%d strips_x=%d tiles_y=%d tiles_z=%d rows_per_wave=%d "
                 "planes_per_wave=%d tiles=%ld blocks=%d xcd_remap=%d",
                 name.c_str(), g.V, g.P, g.halo_left, g.halo_right, g.valid_lanes, g.strips_x, g.tiles_y, g.tiles_z,
                 g.rows_per_wave, g.planes_per_wave, g.tiles, g.blocks, g.xcd_remap);
    }
    return rc;
}

}  // namespace
}  // namespace ssam

using namespace ssam;

extern "C" {

int ssam_conv2d(const void* d_in, void* d_out, int W, int H, const void* h_filter, int M, int N, int ax, int ay,
                int boundary, int dtype, void* hip_stream)
{
    if (int e = validate_conv(d_in, d_out, W, H, h_filter, M, N, &ax, &ay, boundary, dtype)) return e;
    Problem2D p{d_in, d_out, W, H, h_filter, M, N, ax, ay, boundary, dtype, (hipStream_t)hip_stream};
    return run2d(p, false, nullptr, false, nullptr);
}

int ssam_stencil2d(const void* d_in, void* d_out, int W, int H, const void* h_coef, int rx, int ry, int boundary,
                   int dtype, void* hip_stream)
{
    if (int e = validate_stencil(d_in, d_out, W, H, 1, h_coef, rx, ry, 0, boundary, dtype)) return e;
    Problem2D p{d_in, d_out, W, H, h_coef, 2 * rx + 1, 2 * ry + 1, rx, ry, boundary, dtype, (hipStream_t)hip_stream};
    return run2d(p, true, nullptr, false, nullptr);
}

int ssam_stencil3d(const void* d_in, void* d_out, int W, int H, int D, const void* h_coef, int rx, int ry, int rz,
                   int boundary, int dtype, void* hip_stream)
{
    if (int e = validate_stencil(d_in, d_out, W, H, D, h_coef, rx, ry, rz, boundary, dtype)) return e;
    Problem3D p{d_in, d_out, W, H, D, h_coef, rx, ry, rz, boundary, dtype, (hipStream_t)hip_stream};
    return run3d(p, nullptr, false, nullptr);
}

int ssam_conv3d(const void* d_in, void* d_out, int W, int H, int D, const void* h_filter, int M, int N, int K, int ax,
                int ay, int az, int boundary, int dtype, void* hip_stream)
{
    if (!d_in || !d_out) return SSAM_ERR_NULL;
    if (int e = check_conv3d(W, H, D, h_filter, M, N, K, &ax, &ay, &az, boundary, dtype)) return e;
    if (overlap(d_in, d_out, (size_t)W * H * D * elem(dtype))) return SSAM_ERR_ALIAS;
    return run_conv3d(d_in, d_out, W, H, D, h_filter, M, N, K, ax, ay, az, boundary, dtype, (hipStream_t)hip_stream,
                      nullptr, false, nullptr);
}

int ssam_stencil_iterate(void* d_a, void* d_b, int W, int H, int D, const void* h_coef, int rx, int ry, int rz,
                         int boundary, int dtype, int steps, void* hip_stream, void** d_result)
{
    if (int e = validate_stencil(d_a, d_b, W, H, D, h_coef, rx, ry, rz, boundary, dtype)) return e;
    if (steps < 0) return SSAM_ERR_SHAPE;
    void* src = d_a;
    void* dst = d_b;
    for (int t = 0; t < steps;) {
        Problem3D p{src, dst, W, H, D, h_coef, rx, ry, rz, boundary, dtype, (hipStream_t)hip_stream};
        int rc = SSAM_OK;
        if (const int fused = run_fused(p, steps - t, nullptr, false, nullptr, &rc)) {
            if (rc) return rc;
            t += fused;
        } else {
            if (int e = run3d(p, nullptr, false, nullptr)) return e;
            t += 1;
        }
        void* tmp = src;
        src = dst;
        dst = tmp;
    }
    if (d_result) *d_result = src;
    return SSAM_OK;
}

int ssam_probe_copy(const void* d_in, void* d_out, size_t nbytes, void* hip_stream)
{
    if (!d_in || !d_out) return SSAM_ERR_NULL;
    if (nbytes == 0 || nbytes % 16 != 0 || ((uintptr_t)d_in % 16) || ((uintptr_t)d_out % 16)) return SSAM_ERR_DIM;
    if (overlap(d_in, d_out, nbytes)) return SSAM_ERR_ALIAS;
    const size_t n16 = nbytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       static_cast<const uint4*>(d_in), static_cast<uint4*>(d_out), n16);
    return hipGetLastError() == hipSuccess ? SSAM_OK : SSAM_ERR_HIP;
}

const char* ssam_status_string(int status)
{
    switch (status) {
        case SSAM_OK: return "ok";
        case SSAM_ERR_NULL: return "null pointer argument";
        case SSAM_ERR_DIM: return "size out of range (grid dimension, element count), misaligned pointer or workspace too small";
        case SSAM_ERR_SHAPE: return "filter, radius, anchor or step count out of range";
        case SSAM_ERR_ENUM: return "unknown dtype, boundary or tuning name";
        case SSAM_ERR_ALIAS: return "input and output buffers overlap";
        case SSAM_ERR_HIP: return "HIP runtime call failed";
        default: return "unknown status";
    }
}

int ssam_set_tuning(const char* name, int value)
{
    if (!name) return SSAM_ERR_NULL;
    if (!strcmp(name, "rows_per_wave")) g_rows_per_wave = value;
    else if (!strcmp(name, "valid_lanes")) g_valid_lanes = value;
    else if (!strcmp(name, "planes_per_wave")) g_planes_per_wave = value;
    else if (!strcmp(name, "xcd_remap")) g_xcd_remap = value;
    else if (!strcmp(name, "force_generic")) g_force_generic = value;
    else if (!strcmp(name, "variant")) g_variant = value;
    else if (!strcmp(name, "march_axis")) g_march_axis = value;
    else if (!strcmp(name, "fuse_sweeps")) g_fuse_sweeps = value;
    else if (!strcmp(name, "embed_waste")) g_embed_waste = value;
    else if (!strcmp(name, "scan_segments")) g_scan_segments = value;
    else if (!strcmp(name, "scan_order")) g_scan_order = value;
    else if (!strcmp(name, "scan_chained")) g_scan_chained = value;
    else if (!strcmp(name, "scan_spin_limit")) g_scan_spin_limit = value;
    else if (!strcmp(name, "scan_one_group")) g_scan_one_group = value;
    else return SSAM_ERR_ENUM;
    return SSAM_OK;
}

int ssam_describe(int kind, int W, int H, int D, const void* h_coef, int a, int b, int c, int boundary, int dtype,
                  char* buf, int buflen)
{
    void* out = nullptr;   // describe plans only: no pointer is dereferenced, no kernel runs
    std::string name;
    Geometry g;
    if (kind == 0) {
        int ax = -1, ay = -1;
        if (!h_coef) return SSAM_ERR_NULL;
        if (int e = check_enums(boundary, dtype)) return e;
        if (int e = check_dims(W, H, 1)) return e;
        if (a <= 0 || b <= 0 || a > SSAM_MAX_FILTER || b > SSAM_MAX_FILTER) return SSAM_ERR_SHAPE;
        ax = a / 2;
        ay = b / 2;
        Problem2D p{nullptr, out, W, H, h_coef, a, b, ax, ay, boundary, dtype, nullptr};
        return describe(run2d(p, false, &g, true, &name), name, g, buf, buflen);
    }
    if (kind == 1 || kind == 2) {
        if (!h_coef) return SSAM_ERR_NULL;
        if (int e = check_enums(boundary, dtype)) return e;
        if (kind == 1) { D = 1; c = 0; }
        if (int e = check_dims(W, H, D)) return e;
        if (a < 0 || b < 0 || c < 0 || a > SSAM_MAX_RADIUS || b > SSAM_MAX_RADIUS || c > SSAM_MAX_RADIUS)
            return SSAM_ERR_SHAPE;
        Problem3D p{nullptr, out, W, H, D, h_coef, a, b, c, boundary, dtype, nullptr};
        return describe(run3d(p, &g, true, &name), name, g, buf, buflen);
    }
    if (kind == 3) {   // the launch ssam_stencil_iterate uses while c (or more) 2D sweeps remain
        if (!h_coef) return SSAM_ERR_NULL;
        if (int e = check_enums(boundary, dtype)) return e;
        if (int e = check_dims(W, H, 1)) return e;
        if (a < 0 || b < 0 || a > SSAM_MAX_RADIUS || b > SSAM_MAX_RADIUS) return SSAM_ERR_SHAPE;
        Problem3D p{nullptr, out, W, H, 1, h_coef, a, b, 0, boundary, dtype, nullptr};
        int rc = SSAM_OK;
        if (run_fused(p, c > 0 ? c : kMaxFusedSweeps, &g, true, &name, &rc)) return describe(rc, name, g, buf, buflen);
        return describe(run3d(p, &g, true, &name), name, g, buf, buflen);
    }
    if (kind == 4) {   // the launch ssam_stencil_iterate uses on a 3D grid while two or more sweeps remain
        if (!h_coef) return SSAM_ERR_NULL;
        if (int e = check_enums(boundary, dtype)) return e;
        if (int e = check_dims(W, H, D)) return e;
        if (a < 0 || b < 0 || c < 0 || a > SSAM_MAX_RADIUS || b > SSAM_MAX_RADIUS || c > SSAM_MAX_RADIUS)
            return SSAM_ERR_SHAPE;
        Problem3D p{nullptr, out, W, H, D, h_coef, a, b, c, boundary, dtype, nullptr};
        int rc = SSAM_OK;
        if (run_fused(p, kMaxFusedSweeps, &g, true, &name, &rc)) return describe(rc, name, g, buf, buflen);
        return describe(run3d(p, &g, true, &name), name, g, buf, buflen);
    }
    if (kind == 5) {   // ssam_conv3d with (a, b, c) = (M, N, K) and the default anchor
        int ax = -1, ay = -1, az = -1;
        if (int e = check_conv3d(W, H, D, h_coef, a, b, c, &ax, &ay, &az, boundary, dtype)) return e;
        return describe(run_conv3d(nullptr, nullptr, W, H, D, h_coef, a, b, c, ax, ay, az, boundary, dtype, nullptr, &g,
                                   true, &name), name, g, buf, buflen);
    }
    return SSAM_ERR_ENUM;
}

}  // extern "C"
