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
// Boundary rule between the sweeps (edge tiles only).  Zero padding: first-sweep values at positions
// outside the grid are forced to 0 by a plane mask, row masks (both wave-uniform) and a per-lane
// column mask before level 2 reads them.  Clamp (a kernel instantiation of its own, so that its extra
// registers do not weigh on the other): columns outside the grid take the first sweep's value at
// column 0 / W-1 by v_readlane, rows outside take row 0 / H-1 of the same plane; a first-sweep plane
// above the grid would have to equal plane 0, which completes later, so such planes are not fed to
// level 2 at all -- plane 0 is fed RZ+1 times when it completes (the in-flight planes only rotate,
// they do not know z), and plane D-1 likewise at the bottom, each extra feed completing and storing
// one more output plane.
#pragma once
#include "ssam_kernel3d.h"

namespace ssam {

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH, bool CLAMP>
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
    // input planes z0-2RZ .. z1-1+2RZ; under the clamp rule the chunk that ends at the grid's bottom
    // stops RZ planes earlier (first-sweep planes below the grid are copies of plane D-1)
    const int nt = (z1 - z0) + ((CLAMP && z1 == D) ? 3 : 4) * RZ;

    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && y0 - 2 * RY >= 0 &&
                          y0 + P - 1 + 2 * RY < H && z0 - 2 * RZ >= 0 && z1 - 1 + 2 * RZ < D;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        unsigned col_keep[V], col_left[V], col_right[V];   // all-ones where the column lies inside / left of / right of the grid
#pragma unroll
        for (int i = 0; i < V; ++i) {
            col_left[i] = xc + i < 0 ? ~0u : 0u;
            col_right[i] = xc + i >= W ? ~0u : 0u;
            col_keep[i] = ~(col_left[i] | col_right[i]);
        }
        // clamp rule: the lanes (wave-uniform) that own grid columns 0 and W-1, when they are in this wave
        const int lane_first = __builtin_amdgcn_readfirstlane(min(max(-xw0, 0) / V, kWave - 1));
        const int last_off = max(W - 1 - xw0, 0);
        const int lane_last = __builtin_amdgcn_readfirstlane(min(last_off / V, kWave - 1));
        const int elem_last = __builtin_amdgcn_readfirstlane(last_off % V);

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
                        if constexpr (CLAMP) {   // rows and planes were clamped in the address
                            const T first = dst[k][0], last = dst[k][V - 1];
#pragma unroll
                            for (int i = 0; i < V; ++i)
                                dst[k][i] = pick(pick(dst[k][i], first, col_left[0]), last, col_right[0]);
                        } else {
#pragma unroll
                            for (int i = 0; i < V; ++i) dst[k][i] = keep_if(dst[k][i], col_keep[0] & row_keep);
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            dst[k][i] = keep_if(rowp[min(max(xc + i, 0), W - 1)], CLAMP ? ~0u : (col_keep[i] & row_keep));
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
                    const int zm = zin - RZ;
                    auto store_plane = [&](int zo) __attribute__((always_inline)) {
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
                    };
                    if constexpr (EDGE && !CLAMP) {
                        const bool plane_in = zm >= 0 && zm < D;
#pragma unroll
                        for (int k = 0; k < P1; ++k) {
                            const int y = y0 - RY + k;
                            const unsigned row_keep = (plane_in && y >= 0 && y < H) ? ~0u : 0u;
#pragma unroll
                            for (int i = 0; i < V; ++i) acc1[0][k][i] = keep_if(acc1[0][k][i], col_keep[VEC ? 0 : i] & row_keep);
                        }
                    }
                    if constexpr (EDGE && CLAMP) {
                        // columns outside the grid take the plane's own value at column 0 / W-1
#pragma unroll
                        for (int k = 0; k < P1; ++k) {
                            const T bl = read_lane(acc1[0][k][0], lane_first);
                            T pickd = acc1[0][k][0];
#pragma unroll
                            for (int i = 1; i < V; ++i) pickd = pick(pickd, acc1[0][k][i], elem_last == i ? ~0u : 0u);
                            const T br = read_lane(pickd, lane_last);
#pragma unroll
                            for (int i = 0; i < V; ++i)
                                acc1[0][k][i] = pick(pick(acc1[0][k][i], bl, col_left[VEC ? 0 : i]), br, col_right[VEC ? 0 : i]);
                        }
                        // rows outside the grid take the plane's row 0 / H-1 (both are in the strip
                        // whenever a row outside it feeds a row inside)
                        if (y0 - RY < 0 || y0 + P - 1 + RY >= H) {
                            T r0[V], rl[V];
#pragma unroll
                            for (int i = 0; i < V; ++i) r0[i] = rl[i] = T(0);
#pragma unroll
                            for (int k = 0; k < P1; ++k) {
                                const int y = y0 - RY + k;
                                const unsigned m0 = y == 0 ? ~0u : 0u, ml = y == H - 1 ? ~0u : 0u;
#pragma unroll
                                for (int i = 0; i < V; ++i) {
                                    r0[i] = pick(r0[i], acc1[0][k][i], m0);
                                    rl[i] = pick(rl[i], acc1[0][k][i], ml);
                                }
                            }
#pragma unroll
                            for (int k = 0; k < P1; ++k) {
                                const int y = y0 - RY + k;
                                const unsigned lo = y < 0 ? ~0u : 0u, hi = y >= H ? ~0u : 0u;
#pragma unroll
                                for (int i = 0; i < V; ++i) acc1[0][k][i] = pick(pick(acc1[0][k][i], r0[i], lo), rl[i], hi);
                            }
                        }
                    }
                    // level 2: that plane is the input of the second sweep; output plane zin - 2RZ completes
                    if constexpr (!CLAMP) {
                        PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(acc1[0], wts, acc2);
                        store_plane(zin - 2 * RZ);
                    } else if (zm >= 0 && zm < D) {
                        if (zm == 0) {   // stands in for the planes above the grid as well
#pragma unroll
                            for (int j = 0; j < RZ; ++j) PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(acc1[0], wts, acc2);
                        }
                        PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(acc1[0], wts, acc2);
                        store_plane(zm - RZ);
                        if (zm == D - 1) {   // ... and for the planes below it: each feed completes one more output plane
#pragma unroll
                            for (int j = 1; j <= RZ; ++j) {
                                PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(acc1[0], wts, acc2);
                                if (zm - RZ + j < z1) store_plane(zm - RZ + j);
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

template <int RX, int RY, int RZ, int BUDGET>
constexpr bool kFusedClamp3D = BUDGET == 1 && RX == 1 && RY == 1 && RZ == 1;

template <typename T, int V, int P, int RX, int RY, int RZ, int BUDGET, int NT, bool PREFETCH>
hipError_t launch3d_fused(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    typedef SliceMask<RX, RY, RZ, BUDGET, 0> Mask0;
    constexpr int HL = (2 * RX + V - 1) / V;
    if (pr.march_y) return hipErrorInvalidValue;
    Geometry g;
    plan_strips(pr.W, V, HL, HL, tu.valid_lanes, &g);
    g.P = P;
    g.rows_per_wave = P;
    g.tiles_y = ceil_div(pr.H, P);
    int planes = tu.planes_per_wave;
    if (planes <= 0) {
        static const int slots = wave_slots(reinterpret_cast<const void*>(&ssam3d_fused_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH, false>));
        planes = balanced_planes(pr.D, (long)g.strips_x * g.tiles_y, slots, 64, 8 * RZ);
    }
    if (planes > pr.D) planes = pr.D;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(pr.D, planes);
    plan_blocks(&g, tu.xcd_remap);
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args3D<T, Mask0::kNW> a;
    fill_args3d<T, V, RX, RY, RZ, BUDGET>(pr, g, &a);
    // The clamp version needs more registers; it is compiled where it still beat single sweeps: the
    // radius-1 stars (7-point fp64 324 -> 484, fp32 642 -> 842 GStencil/s on 512^3; the 19- and
    // 27-point shapes spill and lose).
    if (pr.boundary == SSAM_BOUNDARY_CLAMP) {
        if constexpr (kFusedClamp3D<RX, RY, RZ, BUDGET>)
            hipLaunchKernelGGL((ssam3d_fused_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH, true>), dim3(g.blocks),
                               dim3(kBlock), 0, pr.stream, a);
        else
            return hipErrorInvalidValue;
    } else
        hipLaunchKernelGGL((ssam3d_fused_kernel<T, V, P, RX, RY, RZ, BUDGET, NT, PREFETCH, false>), dim3(g.blocks),
                           dim3(kBlock), 0, pr.stream, a);
    return hipGetLastError();
}

#define SSAM_INSTANCE_3D_FUSED(T, DT, V, P, RX, RY, RZ, BUDGET, PREFETCH, NT, VARIANT)                       \
    static ::ssam::Register3D SSAM_CAT(reg3df_, __COUNTER__)(::ssam::Instance3D{                             \
        #T "_r" #RX #RY #RZ "_b" #BUDGET "_v" #V "p" #P "f" #PREFETCH "nt" #NT "_fused2", DT, RX, RY, RZ,     \
        BUDGET, VARIANT, &::ssam::launch3d_fused<T, V, P, RX, RY, RZ, BUDGET, NT, (PREFETCH) != 0>, 2,        \
        ::ssam::kFusedClamp3D<RX, RY, RZ, BUDGET>})

}  // namespace ssam
