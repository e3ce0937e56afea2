// 3D stencil kernel: lanes span x (V columns each), the register cache holds a strip of
// P + 2*RY rows of the current input plane, and the wave marches along z.
//
// The paper couples z-neighbours through shared memory between the warps of a block
// (Sec. 4.9).  Here the z direction is the "vertical" direction of the software systolic
// array (Fig. 1d: registers of one thread, direct access): every loaded plane contributes
// to the 2*RZ+1 output planes in flight, whose partial sums stay in the same lane's
// registers, so no LDS and no barrier is needed.  Within a plane, each dz-slice of the
// stencil is a 2D filter evaluated by the same converging partial-sum chains as in 2D.
#pragma once
#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {

template <typename T, int NW>
struct Args3D {
    const T* in;
    T* out;
    int W, H, D;
    int boundary;
    int strips_x, tiles_y;
    long tiles;
    int valid_lanes;
    int planes_per_wave;
    int blocks;
    int xcd_remap;
    int aligned;
    long stride_row, stride_plane;   // element strides of the strip axis and of the march axis
    T w[NW];
};

// One step of the z march: input plane `r` (z = zin) is added into the in-flight output
// planes.  acc[k] holds output plane zin - RZ + k, which takes the stencil slice dz = RZ - k
// of this input plane.  Each plane's sums are read from slot k+1 and written to slot k, so
// the planes move one slot towards completion per step at no cost in instructions; the
// newest plane (slot 2*RZ) starts from zero, and after the step slot 0 is complete.
template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int K>
struct PlaneStep {
    static __device__ __forceinline__ void run(const T (&r)[P + 2 * RY][V], ConstPtr<T> w,
                                               T (&acc)[2 * RZ + 1][P][V])
    {
        constexpr int NZ = 2 * RZ + 1;
        typedef SliceMask<RX, RY, RZ, BUDGET, RZ - K> Mask;
        if constexpr (K == NZ - 1) {
            systolic_rows<T, V, P, Mask, false>(RowBlock<T, V, P + 2 * RY>{r}, w, acc[K], acc[K]);
        } else {
            systolic_rows<T, V, P, Mask, true>(RowBlock<T, V, P + 2 * RY>{r}, w, acc[K + 1], acc[K]);
            PlaneStep<T, V, P, RX, RY, RZ, BUDGET, K + 1>::run(r, w, acc);
        }
    }
};

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH>
__global__ __launch_bounds__(kBlock) void ssam3d_kernel(
    const Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW> a)
{
    constexpr int NZ = 2 * RZ + 1;
    constexpr int C = P + 2 * RY;
    constexpr int HL = (RX + V - 1) / V;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
    // Tiles are numbered strip-fastest, so the waves of a block read neighbouring pieces of the
    // same rows at the same time (measured slightly faster than stacking a block's waves in y).
    const long tile = (long)lb * kWavesPerBlock + wave;
    if (tile >= a.tiles) return;
    const int strip = (int)(tile % a.strips_x);
    const int ytile = (int)((tile / a.strips_x) % a.tiles_y);
    const int ztile = (int)(tile / ((long)a.strips_x * a.tiles_y));

    const int W = a.W, H = a.H, D = a.D;
    const int xo0 = strip * a.valid_lanes * V;
    const int xw0 = xo0 - HL * V;
    const int xc = xw0 + lane * V;
    const int y0 = ytile * P;
    const int z0 = ztile * a.planes_per_wave;
    const int z1 = min(z0 + a.planes_per_wave, D);
    const bool vec_ok = a.aligned && (W % V) == 0;
    // lanes past the right halo hold nothing any stored output depends on: they re-read the last
    // needed lane's columns (same cache line, no extra traffic, no divergence)
    const int used_lanes = min(a.valid_lanes + 2 * HL, kWave);
    const int xl = xw0 + min(lane, used_lanes - 1) * V;
    const bool clamp = a.boundary == kClamp;
    const T* __restrict__ in = a.in;
    typedef Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));
    // strides of the two outer axes in elements: the rows of a lane's strip are `rowst` apart, the
    // planes the wave marches over `plane` apart (W and W*H when marching z; swapped when the host
    // asks for a march along y, where a.H and a.D are then the extents of z and y)
    const size_t rowst = (size_t)a.stride_row, plane = (size_t)a.stride_plane;
    const bool lane_stores = lane >= HL && lane < HL + a.valid_lanes && xc < W;
    const unsigned left_mask = xc < 0 ? ~0u : 0u, right_mask = xc >= W ? ~0u : 0u;
    const unsigned left_pick = clamp ? left_mask : 0u, right_pick = clamp ? right_mask : 0u;
    const unsigned keep_cols = clamp ? ~0u : ~(left_mask | right_mask);
    const unsigned keep_rows = clamp ? ~0u : 0u;
    const int nt = (z1 - z0) + 2 * RZ;    // input planes z0-RZ .. z1-1+RZ

    // "Interior" tiles touch nothing outside the grid and use aligned vectors: no checks at all.
    // All other tiles take the general path: wave-uniform row/plane logic and per-lane selects
    // for the columns (still vector loads when rows are V-aligned), element loads otherwise.
    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && y0 - RY >= 0 &&
                          y0 + P - 1 + RY < H && z0 - RZ >= 0 && z1 - 1 + RZ < D;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        auto load_plane = [&](int z, T (&dst)[C][V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                const T* pz = in + (size_t)z * plane + (size_t)(y0 - RY) * rowst + xl;
#pragma unroll
                for (int k = 0; k < C; ++k) load_vec<T, V, (NT & kStreamLoads) != 0>(pz + (size_t)k * rowst, dst[k]);
            } else {
                const bool plane_in = z >= 0 && z < D;
                const T* pz = in + (size_t)min(max(z, 0), D - 1) * plane;
                const int xv = min(max(xl, 0), W - V);
#pragma unroll
                for (int k = 0; k < C; ++k) {
                    const int y = y0 - RY + k;
                    const bool row_in = plane_in && y >= 0 && y < H;     // wave-uniform
                    const T* rowp = pz + (size_t)min(max(y, 0), H - 1) * rowst;
                    if constexpr (VEC) {
                        // W and xc are multiples of V: a lane's V columns are all in or all out
                        load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + xv, dst[k]);
                        const T first = dst[k][0], last = dst[k][V - 1];
                        const unsigned keep = keep_cols & (row_in ? ~0u : keep_rows);
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            dst[k][i] = keep_if(pick(pick(dst[k][i], first, left_pick), last, right_pick), keep);
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i) {
                            const int x = xc + i;
                            const T v = rowp[min(max(x, 0), W - 1)];
                            dst[k][i] = (clamp || (row_in && x >= 0 && x < W)) ? v : T(0);
                        }
                    }
                }
            }
        };

        T acc[NZ][P][V];
#pragma unroll
        for (int s = 0; s < NZ; ++s)
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int j = 0; j < V; ++j) acc[s][p][j] = T(0);

        // Two plane buffers alternate: the next plane is requested before the current one is
        // used, so its latency hides behind the arithmetic.  The march is unrolled by two so the
        // buffer in use is known at compile time.
        T buf[PREFETCH ? 2 : 1][C][V];
        if constexpr (PREFETCH) load_plane(z0 - RZ, buf[0]);

        for (int tb = 0; tb < nt; tb += 2) {
            static_for<2>([&](auto uc) __attribute__((always_inline)) {
                constexpr int cur = PREFETCH ? decltype(uc)::value : 0;
                const int t = tb + decltype(uc)::value;
                if (t < nt) {
                    const int zin = z0 - RZ + t;
                    if constexpr (PREFETCH) {
                        if (t + 1 < nt) load_plane(zin + 1, buf[cur ^ 1]);
                    } else {
                        load_plane(zin, buf[0]);   // no second buffer: other waves hide the latency
                    }
                    PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(buf[cur], wts, acc);

                    // output plane zin - RZ has now received its last contribution
                    const int zo = zin - RZ;
                    if (zo >= z0 && lane_stores) {
                        T* po = a.out + (size_t)zo * plane + (size_t)y0 * rowst + xc;
#pragma unroll
                        for (int p = 0; p < P; ++p) {
                            T* rowp = po + (size_t)p * rowst;
                            if constexpr (!EDGE) {
                                store_vec<T, V, (NT & kStreamStores) != 0>(rowp, acc[0][p]);
                            } else if (y0 + p < H) {
                                if constexpr (VEC) {
                                    store_vec<T, V, (NT & kStreamStores) != 0>(rowp, acc[0][p]);
                                } else {
#pragma unroll
                                    for (int i = 0; i < V; ++i)
                                        if (xc + i < W) rowp[i] = acc[0][p][i];
                                }
                            }
                        }
                    }
                }
            });
        }
    };

    // the mode is wave-uniform and fixed for the whole march, so no load sits behind a branch
    if (interior) march(std::integral_constant<int, 0>{});
    else if (vec_ok) march(std::integral_constant<int, 1>{});
    else march(std::integral_constant<int, 2>{});
}

// Fills the kernel-argument block: pointers, sizes, tile plan and the packed coefficients.
template <typename T, int V, int RX, int RY, int RZ, int BUDGET>
void fill_args3d(const Problem3D& pr, const Geometry& g, Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW>* a)
{
    typedef SliceMask<RX, RY, RZ, BUDGET, 0> Mask0;
    constexpr int NX = 2 * RX + 1, NY = 2 * RY + 1, NZ = 2 * RZ + 1;
    a->in = static_cast<const T*>(pr.in);
    a->out = static_cast<T*>(pr.out);
    // march along z: strip axis y.  march along y (pr.march_y): strip axis z; the kernel then sees
    // extents and coefficients with y and z exchanged, and the real strides.
    const bool my = pr.march_y;
    a->W = pr.W;
    a->H = my ? pr.D : pr.H;
    a->D = my ? pr.H : pr.D;
    a->stride_row = my ? (long)pr.W * pr.H : (long)pr.W;
    a->stride_plane = my ? (long)pr.W : (long)pr.W * pr.H;
    a->boundary = pr.boundary;
    a->strips_x = g.strips_x;
    a->tiles_y = g.tiles_y;
    a->tiles = g.tiles;
    a->valid_lanes = g.valid_lanes;
    a->planes_per_wave = g.planes_per_wave;
    a->blocks = g.blocks;
    a->xcd_remap = g.xcd_remap;
    a->aligned = pointers_aligned(pr.in, pr.out, V * sizeof(T)) ? 1 : 0;
    const T* c = static_cast<const T*>(pr.c);   // host, dense [2rz+1][2ry+1][2rx+1] in real axes
    for (int i = 0; i < Mask0::kNW; ++i) a->w[i] = T(0);
    for (int k = 0; k < NZ; ++k)          // k: offset along the march axis, n: along the strip axis
        for (int n = 0; n < NY; ++n)
            for (int m = 0; m < NX; ++m) {
                const int used = (k != RZ) + (n != RY) + (m != RX);
                if (used > BUDGET) continue;
                int idx;
                if (BUDGET == 1) idx = k != RZ ? k : (n != RY ? NZ + n : (m != RX ? NZ + NY + m : RZ));
                else idx = (k * NX + m) * NY + n;
                a->w[idx] = my ? c[(n * NZ + k) * NX + m] : c[(k * NY + n) * NX + m];
            }
}

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH>
hipError_t launch3d(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    typedef SliceMask<RX, RY, RZ, BUDGET, 0> Mask0;
    constexpr int HL = (RX + V - 1) / V;
    Geometry g;
    plan_strips(pr.W, V, HL, HL, tu.valid_lanes, &g);
    g.P = P;
    g.rows_per_wave = P;
    const int LH = pr.march_y ? pr.D : pr.H, LD = pr.march_y ? pr.H : pr.D;   // strip / march extents
    g.tiles_y = ceil_div(LH, P);
    // z-chunk per wave: short chunks (more waves, shorter tails) measured 3-5 % faster for radius 1
    // on 512^3 in spite of the 2*RZ planes every chunk re-reads; small grids get shorter ones still
    int planes = tu.planes_per_wave;
    if (planes <= 0) {
        static const int slots = wave_slots(reinterpret_cast<const void*>(&ssam3d_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH>));
        planes = balanced_planes(LD, (long)g.strips_x * g.tiles_y, slots, RZ == 1 ? 16 : 64, 4 * RZ);
    }
    if (planes > LD) planes = LD;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(LD, planes);
    plan_blocks(&g, tu.xcd_remap);
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args3D<T, Mask0::kNW> a;
    fill_args3d<T, V, RX, RY, RZ, BUDGET>(pr, g, &a);
    hipLaunchKernelGGL((ssam3d_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH>), dim3(g.blocks), dim3(kBlock), 0,
                       pr.stream, a);
    return hipGetLastError();
}

#define SSAM_INSTANCE_3D_V(T, DT, V, P, RX, RY, RZ, BUDGET, PREFETCH, NT, VARIANT)                    \
    static ::ssam::Register3D SSAM_CAT(reg3d_, __COUNTER__)(::ssam::Instance3D{                      \
        #T "_r" #RX #RY #RZ "_b" #BUDGET "_v" #V "p" #P "f" #PREFETCH "nt" #NT, DT, RX, RY, RZ,       \
        BUDGET, VARIANT, &::ssam::launch3d<T, V, P, RX, RY, RZ, BUDGET, NT, (PREFETCH) != 0>})
#define SSAM_INSTANCE_3D(T, DT, V, P, RX, RY, RZ, BUDGET) SSAM_INSTANCE_3D_V(T, DT, V, P, RX, RY, RZ, BUDGET, 1, 2, 0)

}  // namespace ssam
