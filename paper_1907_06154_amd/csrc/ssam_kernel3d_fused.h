// Two Jacobi sweeps of a 3D stencil in one pass over the grid (temporal blocking in the
// register cache; Sec. 6.4 says the model permits it and gives no algorithm -- this one is
// ours, the 3D counterpart of ssam2d_fused_kernel).
//
// The z march of ssam3d_kernel runs at two levels inside the wave.  Level 1 is the first sweep
// on a strip widened by RY rows on each side: every loaded input plane (P + 4*RY rows) is added
// into 2*RZ+1 in-flight first-sweep planes of P + 2*RY rows.  The first-sweep plane that completes
// is not stored: it is the "input plane" of level 2, the ordinary march over P rows, whose
// completed plane is stored.  HBM sees one read and one write per two sweeps.  Overlap: ceil(2*RX/V)
// halo lanes per side, 2*RY halo rows per side of the strip, 4*RZ extra planes per z-chunk.
//
// Zero padding only: first-sweep values at positions outside the grid are forced to 0 by a
// plane mask, row masks (both wave-uniform) and a per-lane column mask before level 2 reads them.
#pragma once
#include "ssam_kernel3d.h"

namespace ssam {

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH>
__global__ __launch_bounds__(kBlock) void ssam3d_fused_kernel(
    const Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW> a)
{
    constexpr int NZ = 2 * RZ + 1;
    constexpr int P1 = P + 2 * RY;      // rows of a first-sweep plane
    constexpr int C0 = P1 + 2 * RY;     // rows of an input plane
    constexpr int HL = (2 * RX + V - 1) / V;   // two sweeps leave 2*RX incomplete columns at each end of the wave

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
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
    const int used_lanes = min(a.valid_lanes + 2 * HL, kWave);
    const int xl = xw0 + min(lane, used_lanes - 1) * V;
    const T* __restrict__ in = a.in;
    typedef Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));
    const size_t rowst = (size_t)a.stride_row, plane = (size_t)a.stride_plane;
    const bool lane_stores = lane >= HL && lane < HL + a.valid_lanes && xc < W;
    const int nt = (z1 - z0) + 4 * RZ;    // input planes z0-2RZ .. z1-1+2RZ

    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && y0 - 2 * RY >= 0 &&
                          y0 + P - 1 + 2 * RY < H && z0 - 2 * RZ >= 0 && z1 - 1 + 2 * RZ < D;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        unsigned col_keep[V];   // all-ones where the lane's column lies inside the grid
#pragma unroll
        for (int i = 0; i < V; ++i) col_keep[i] = (xc + i >= 0 && xc + i < W) ? ~0u : 0u;

        auto load_plane = [&](int z, T (&dst)[C0][V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                const T* pz = in + (size_t)z * plane + (size_t)(y0 - 2 * RY) * rowst + xl;
#pragma unroll
                for (int k = 0; k < C0; ++k) load_vec<T, V, (NT & kStreamLoads) != 0>(pz + (size_t)k * rowst, dst[k]);
            } else {
                const bool plane_in = z >= 0 && z < D;
                const T* pz = in + (size_t)min(max(z, 0), D - 1) * plane;
                const int xv = min(max(xl, 0), W - V);
#pragma unroll
                for (int k = 0; k < C0; ++k) {
                    const int y = y0 - 2 * RY + k;
                    const unsigned row_keep = (plane_in && y >= 0 && y < H) ? ~0u : 0u;   // wave-uniform
                    const T* rowp = pz + (size_t)min(max(y, 0), H - 1) * rowst;
                    if constexpr (VEC) {
                        load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + xv, dst[k]);
#pragma unroll
                        for (int i = 0; i < V; ++i) dst[k][i] = keep_if(dst[k][i], col_keep[0] & row_keep);
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            dst[k][i] = keep_if(rowp[min(max(xc + i, 0), W - 1)], col_keep[i] & row_keep);
                    }
                }
            }
        };

        T acc1[NZ][P1][V];   // first-sweep planes in flight
        T acc2[NZ][P][V];    // output planes in flight
#pragma unroll
        for (int s = 0; s < NZ; ++s) {
#pragma unroll
            for (int p = 0; p < P1; ++p)
#pragma unroll
                for (int j = 0; j < V; ++j) acc1[s][p][j] = T(0);
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int j = 0; j < V; ++j) acc2[s][p][j] = T(0);
        }

        T buf[PREFETCH ? 2 : 1][C0][V];
        if constexpr (PREFETCH) load_plane(z0 - 2 * RZ, buf[0]);

        for (int tb = 0; tb < nt; tb += 2) {
            static_for<2>([&](auto uc) __attribute__((always_inline)) {
                constexpr int cur = PREFETCH ? decltype(uc)::value : 0;
                const int t = tb + decltype(uc)::value;
                if (t < nt) {
                    const int zin = z0 - 2 * RZ + t;
                    if constexpr (PREFETCH) {
                        if (t + 1 < nt) load_plane(zin + 1, buf[cur ^ 1]);
                    } else {
                        load_plane(zin, buf[0]);
                    }
                    // level 1: first-sweep plane zin - RZ receives its last contribution
                    PlaneStep<T, V, P1, RX, RY, RZ, BUDGET, 0>::run(buf[cur], wts, acc1);
                    if constexpr (EDGE) {
                        const int zm = zin - RZ;
                        const bool plane_in = zm >= 0 && zm < D;
#pragma unroll
                        for (int k = 0; k < P1; ++k) {
                            const int y = y0 - RY + k;
                            const unsigned row_keep = (plane_in && y >= 0 && y < H) ? ~0u : 0u;
#pragma unroll
                            for (int i = 0; i < V; ++i) acc1[0][k][i] = keep_if(acc1[0][k][i], col_keep[VEC ? 0 : i] & row_keep);
                        }
                    }
                    // level 2: that plane is the input of the second sweep; output plane zin - 2RZ completes
                    PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(acc1[0], wts, acc2);

                    const int zo = zin - 2 * RZ;
                    if (zo >= z0 && lane_stores) {
                        T* po = a.out + (size_t)zo * plane + (size_t)y0 * rowst + xc;
#pragma unroll
                        for (int p = 0; p < P; ++p) {
                            T* rowp = po + (size_t)p * rowst;
                            if constexpr (!EDGE) {
                                store_vec<T, V, (NT & kStreamStores) != 0>(rowp, acc2[0][p]);
                            } else if (y0 + p < H) {
                                if constexpr (VEC) {
                                    store_vec<T, V, (NT & kStreamStores) != 0>(rowp, acc2[0][p]);
                                } else {
#pragma unroll
                                    for (int i = 0; i < V; ++i)
                                        if (xc + i < W) rowp[i] = acc2[0][p][i];
                                }
                            }
                        }
                    }
                }
            });
        }
    };

    if (interior) march(std::integral_constant<int, 0>{});
    else if (vec_ok) march(std::integral_constant<int, 1>{});
    else march(std::integral_constant<int, 2>{});
}

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH>
hipError_t launch3d_fused(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    typedef SliceMask<RX, RY, RZ, BUDGET, 0> Mask0;
    constexpr int HL = (2 * RX + V - 1) / V;
    if (pr.boundary != SSAM_BOUNDARY_ZERO || pr.march_y) return hipErrorInvalidValue;
    Geometry g;
    plan_strips(pr.W, V, HL, HL, tu.valid_lanes, &g);
    g.P = P;
    g.rows_per_wave = P;
    g.tiles_y = ceil_div(pr.H, P);
    int planes = tu.planes_per_wave;
    if (planes <= 0) {
        static const int slots = wave_slots(reinterpret_cast<const void*>(&ssam3d_fused_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH>));
        planes = balanced_planes(pr.D, (long)g.strips_x * g.tiles_y, slots, 64, 8 * RZ);
    }
    if (planes > pr.D) planes = pr.D;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(pr.D, planes);
    plan_blocks(&g, tu.xcd_remap);
    if (geo) *geo = g;
    if (dry_run) return hipSuccess;

    Args3D<T, Mask0::kNW> a;
    fill_args3d<T, V, RX, RY, RZ, BUDGET>(pr, g, &a);
    hipLaunchKernelGGL((ssam3d_fused_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH>), dim3(g.blocks), dim3(kBlock),
                       0, pr.stream, a);
    return hipGetLastError();
}

#define SSAM_INSTANCE_3D_FUSED(T, DT, V, P, RX, RY, RZ, BUDGET, PREFETCH, NT, VARIANT)                       \
    static ::ssam::Register3D SSAM_CAT(reg3df_, __COUNTER__)(::ssam::Instance3D{                             \
        #T "_r" #RX #RY #RZ "_b" #BUDGET "_v" #V "p" #P "f" #PREFETCH "nt" #NT "_fused2", DT, RX, RY, RZ,     \
        BUDGET, VARIANT, &::ssam::launch3d_fused<T, V, P, RX, RY, RZ, BUDGET, NT, (PREFETCH) != 0>, 2})

}  // namespace ssam
