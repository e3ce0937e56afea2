// Several Jacobi sweeps of a 2D stencil in one pass over the grid (temporal blocking in the
// register cache; Sec. 6.4 states that the register cache and the lane shifts do not stand in
// the way of temporal blocking but gives no algorithm for it -- this one is our own).
//
// The march of ssam2d_kernel is run S times, back to back, inside the wave: the P rows sweep k
// produces for a group never leave the registers -- they join the 2R rows of sweep k kept from
// the previous group and form the window of sweep k+1.  HBM sees one read and one write per S
// sweeps.  The price is a wider overlap between tiles: every sweep invalidates R more columns at
// each end of the wave, so the wave stores 64 - 2*ceil(S*R/V) lanes, and each tile spends
// ceil(2(S-1)R/P) extra groups at its top producing the intermediate rows its first outputs need.
//
// Boundary rule between sweeps (edge tiles only; interior tiles touch nothing outside the grid):
// an intermediate value at a position outside the grid must read as 0 under zero padding, which a
// mask does, and as the value of the nearest grid point under the clamp rule.  For columns that is
// the value held by the lane that owns column 0 (or W-1), broadcast with v_readlane to the lanes
// outside the grid.  For rows it is row 0 (or H-1) of the same sweep: rows above the grid are
// produced before row 0 exists, so they are patched when they are consumed -- every window that
// holds rows outside the grid and feeds a row inside it also holds row 0 (or H-1).
#pragma once
#include "ssam_kernel2d.h"

namespace ssam {

template <typename T, int V, int P, class Mask, int S, int NT>
__global__ __launch_bounds__(kBlock) void ssam2d_fused_kernel(const Args2D<T, Mask::kNW> a)
{
    constexpr int N = Mask::kN;
    constexpr int R = Mask::kAY;          // rows above the centre
    constexpr int KEEP = N - 1;
    static_assert(S >= 2 && N == 2 * R + 1 && Mask::kLeft == Mask::kRight, "fused sweeps need a centred stencil");
    // after S sweeps the S*RX outermost columns of the wave are incomplete (validity is per
    // column, not per lane: a lane's inner columns find their neighbours in the same lane)
    constexpr int HL = (S * Mask::kLeft + V - 1) / V, HR = HL;
    constexpr int WARM = (2 * (S - 1) * R + P - 1) / P;   // groups run before the first output group

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
    const long tile = (long)lb * kWavesPerBlock + wave;
    if (tile >= a.tiles) return;
    const int strip = (int)(tile % a.strips_x);
    const int ytile = (int)(tile / a.strips_x);

    const int W = a.W, H = a.H;
    const int xo0 = strip * a.valid_lanes * V;
    const int xw0 = xo0 - HL * V;
    const int xc = xw0 + lane * V;
    const int y0 = ytile * a.rows_per_wave;
    const int y1 = min(y0 + a.rows_per_wave, H);
    const int ys = y0 - WARM * P;                    // base of the first (warm-up) group
    const bool vec_ok = a.aligned && (W % V) == 0;
    const int used_lanes = min(HL + a.valid_lanes + HR, kWave);
    const int xl = xw0 + min(lane, used_lanes - 1) * V;
    const T* __restrict__ in = a.in;
    typedef Args2D<T, Mask::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));
    const bool lane_stores = lane >= HL && lane < HL + a.valid_lanes && xc < W;
    const bool clamp = a.boundary == kClamp;

    // The group with base y loads input rows y + S*R .. y + S*R + P-1; sweep k (0-based) turns
    // them into its rows y + (S-1-k)*R .. + P-1, and the last sweep's rows y .. y+P-1 are stored
    // from y0 on.  Sweep k's rows are complete from row ys + (S-1+k)*R on (its kept rows start
    // as zeros), which the warm-up groups put at or above y0 for the last sweep.
    const int nchunks = (y1 - y0 + P - 1) / P;
    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && (y1 - y0) % P == 0 &&
                          ys + (S - 2) * R >= 0 && y0 + (nchunks - 1) * P + S * R + P - 1 < H;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        // 0 interior; edge tiles: 1 vectors / 2 by element with zero padding, 3 / 4 the same with the clamp rule
        constexpr int MODE = decltype(mode_tag)::value;
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2 && MODE != 4;
        constexpr bool CLAMP = MODE >= 3;

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

        auto load_row = [&](int y, T (&dst)[V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                load_vec<T, V, (NT & kStreamLoads) != 0>(in + (size_t)y * W + xl, dst);
            } else {
                const unsigned row_keep = (y >= 0 && y < H) ? ~0u : 0u;   // wave-uniform
                const T* rowp = in + (size_t)min(max(y, 0), H - 1) * W;
                if constexpr (VEC) {
                    load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + min(max(xl, 0), W - V), dst);
                    if constexpr (CLAMP) {
                        // columns outside the grid take the edge column, which is the first (last)
                        // element of the vector such a lane loaded; rows were clamped in the address
                        const T first = dst[0], last = dst[V - 1];
#pragma unroll
                        for (int i = 0; i < V; ++i) dst[i] = pick(pick(dst[i], first, col_left[0]), last, col_right[0]);
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i) dst[i] = keep_if(dst[i], col_keep[0] & row_keep);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i)
                        dst[i] = keep_if(rowp[min(max(xc + i, 0), W - 1)], CLAMP ? ~0u : (col_keep[i] & row_keep));
                }
            }
        };

        auto store_rows = [&](int y, const T (&acc)[P][V]) __attribute__((always_inline)) {
            if (lane_stores) {
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    T* rowp = a.out + (size_t)(y + p) * W;
                    if constexpr (!EDGE) {
                        store_vec<T, V, (NT & kStreamStores) != 0>(rowp + xc, acc[p]);
                    } else if (y + p < y1) {
                        if constexpr (VEC) {
                            store_vec<T, V, (NT & kStreamStores) != 0>(rowp + xc, acc[p]);
                        } else {
#pragma unroll
                            for (int i = 0; i < V; ++i)
                                if (xc + i < W) rowp[xc + i] = acc[p][i];
                        }
                    }
                }
            }
        };

        // rows P .. P+KEEP-1 of a window open the next one
        auto carry = [&](T (&kept)[KEEP][V], const T (&fresh)[P][V]) __attribute__((always_inline)) {
#pragma unroll
            for (int k = 0; k < KEEP; ++k)
#pragma unroll
                for (int i = 0; i < V; ++i)
                    kept[k][i] = (k + P < KEEP) ? kept[(k + P < KEEP) ? k + P : 0][i]
                                                : fresh[(k + P >= KEEP) ? k + P - KEEP : 0][i];
        };

        T kept[S][KEEP][V];   // kept[0]: input rows; kept[k]: rows of sweep k-1
        T fresh[2][P][V];
#pragma unroll
        for (int k = 0; k < KEEP; ++k) {
            load_row(ys + (S - 2) * R + k, kept[0][k]);
#pragma unroll
            for (int s = 1; s < S; ++s)
#pragma unroll
                for (int i = 0; i < V; ++i) kept[s][k][i] = T(0);
        }
#pragma unroll
        for (int k = 0; k < P; ++k) load_row(ys + S * R + k, fresh[0][k]);

        for (int yb = ys; yb < y1; yb += 2 * P) {
            static_for<2>([&](auto half) __attribute__((always_inline)) {
                constexpr int cur = decltype(half)::value;
                const int y = yb + cur * P;
                if (y < y1) {
                    if (y + P < y1) {
#pragma unroll
                        for (int k = 0; k < P; ++k) load_row(y + P + S * R + k, fresh[cur ^ 1][k]);
                    }

                    T mid[S - 1][P][V];   // rows of the sweeps before the last, this group
                    static_for<S - 1>([&](auto kk) __attribute__((always_inline)) {
                        constexpr int k = decltype(kk)::value;
                        if constexpr (k == 0)
                            systolic_rows<T, V, P, Mask, false>(RowPair<T, V, KEEP, P>{kept[0], fresh[cur]}, wts, mid[0], mid[0]);
                        else
                            systolic_rows<T, V, P, Mask, false>(RowPair<T, V, KEEP, P>{kept[k], mid[k > 0 ? k - 1 : 0]}, wts, mid[k], mid[k]);
                        if constexpr (EDGE) {
                            if constexpr (!CLAMP) {
#pragma unroll
                                for (int p = 0; p < P; ++p) {
                                    const int yr = y + (S - 1 - k) * R + p;
                                    const unsigned row_keep = (yr >= 0 && yr < H) ? ~0u : 0u;
#pragma unroll
                                    for (int i = 0; i < V; ++i)
                                        mid[k][p][i] = keep_if(mid[k][p][i], col_keep[VEC ? 0 : i] & row_keep);
                                }
                            } else {
                                // columns outside the grid take this sweep's value at column 0 / W-1
#pragma unroll
                                for (int p = 0; p < P; ++p) {
                                    const T bl = read_lane(mid[k][p][0], lane_first);
                                    T pickd = mid[k][p][0];
#pragma unroll
                                    for (int i = 1; i < V; ++i) pickd = pick(pickd, mid[k][p][i], elem_last == i ? ~0u : 0u);
                                    const T br = read_lane(pickd, lane_last);
#pragma unroll
                                    for (int i = 0; i < V; ++i)
                                        mid[k][p][i] = pick(pick(mid[k][p][i], bl, col_left[VEC ? 0 : i]), br, col_right[VEC ? 0 : i]);
                                }
                                // rows outside the grid, in the window the next sweep is about to read
                                // (kept[k+1] then mid[k]), take row 0 / H-1 of this sweep
                                const int wb = y + (S - 1 - k) * R - KEEP;   // grid row of the window's first row
                                if (wb < 0 || wb + KEEP + P - 1 >= H) {
                                    T r0[V], rl[V];
#pragma unroll
                                    for (int i = 0; i < V; ++i) r0[i] = rl[i] = T(0);
#pragma unroll
                                    for (int q = 0; q < KEEP + P; ++q) {
                                        const unsigned m0 = wb + q == 0 ? ~0u : 0u, ml = wb + q == H - 1 ? ~0u : 0u;
#pragma unroll
                                        for (int i = 0; i < V; ++i) {
                                            const T v = q < KEEP ? kept[k + 1][q < KEEP ? q : 0][i] : mid[k][q >= KEEP ? q - KEEP : 0][i];
                                            r0[i] = pick(r0[i], v, m0);
                                            rl[i] = pick(rl[i], v, ml);
                                        }
                                    }
#pragma unroll
                                    for (int q = 0; q < KEEP + P; ++q) {
                                        const unsigned lo = wb + q < 0 ? ~0u : 0u, hi = wb + q >= H ? ~0u : 0u;
#pragma unroll
                                        for (int i = 0; i < V; ++i) {
                                            if (q < KEEP) {
                                                T& v = kept[k + 1][q < KEEP ? q : 0][i];
                                                v = pick(pick(v, r0[i], lo), rl[i], hi);
                                            } else {
                                                T& v = mid[k][q >= KEEP ? q - KEEP : 0][i];
                                                v = pick(pick(v, r0[i], lo), rl[i], hi);
                                            }
                                        }
                                    }
                                }
                            }
                        }
                    });
                    if (y >= y0) {
                        T acc[P][V];
                        systolic_rows<T, V, P, Mask, false>(RowPair<T, V, KEEP, P>{kept[S - 1], mid[S - 2]}, wts, acc, acc);
                        store_rows(y, acc);
                    }
                    carry(kept[0], fresh[cur]);
                    static_for<S - 1>([&](auto kk) __attribute__((always_inline)) {
                        carry(kept[decltype(kk)::value + 1], mid[decltype(kk)::value]);
                    });
                }
            });
        }
    };

    if (interior) march(std::integral_constant<int, 0>{});
    else if (!clamp && vec_ok) march(std::integral_constant<int, 1>{});
    else if (!clamp) march(std::integral_constant<int, 2>{});
    else if (vec_ok) march(std::integral_constant<int, 3>{});
    else march(std::integral_constant<int, 4>{});
}

template <typename T, int V, int P, class Mask, int S, int NT>
hipError_t launch2d_fused(const Problem2D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int M = Mask::kM, N = Mask::kN;
    constexpr int HL = (S * Mask::kLeft + V - 1) / V;
    static_assert(64 - 2 * HL >= 8, "stencil too wide for this many sweeps in one wave");
    Geometry g;
    plan_strips(pr.W, V, HL, HL, tu.valid_lanes, &g, true);
    g.P = P;
    // The deep instances are arithmetic-bound: every wave takes about the same time, so the tile
    // count should fill the machine's wave slots a whole number of times; tiles at least 8 groups
    // tall keep the warm-up groups at each tile's top a small part of the work.
    int rows;
    if (tu.rows_per_wave > 0) {
        rows = tu.rows_per_wave;
    } else {
        static const int slots = wave_slots(reinterpret_cast<const void*>(&ssam2d_fused_kernel<T, V, P, Mask, S, NT>));
        rows = balanced_rows(pr.H, P, g.strips_x, slots, 8 * P);
    }
    rows = ceil_div(rows, P) * P;
    if (rows > ceil_div(pr.H, P) * P) rows = ceil_div(pr.H, P) * P;
    g.rows_per_wave = rows;
    g.tiles_y = ceil_div(pr.H, rows);
    plan_blocks(&g, tu.xcd_remap);
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args2D<T, Mask::kNW> a;
    a.in = static_cast<const T*>(pr.in);
    a.out = static_cast<T*>(pr.out);
    a.W = pr.W;
    a.H = pr.H;
    a.ay = pr.ay;
    a.boundary = pr.boundary;
    a.strips_x = g.strips_x;
    a.tiles = g.tiles;
    a.valid_lanes = g.valid_lanes;
    a.rows_per_wave = g.rows_per_wave;
    a.blocks = g.blocks;
    a.xcd_remap = g.xcd_remap;
    a.aligned = pointers_aligned(pr.in, pr.out, V * sizeof(T)) ? 1 : 0;
    const T* w = static_cast<const T*>(pr.w);
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m)
            if (Mask::tap(n, m)) a.w[Mask::widx(n, m)] = w[n * M + m];
    hipLaunchKernelGGL((ssam2d_fused_kernel<T, V, P, Mask, S, NT>), dim3(g.blocks), dim3(kBlock), 0, pr.stream, a);
    return hipGetLastError();
}

// Registers the S-sweep kernel for the centred (2R+1)x(2R+1) stencil of the given budget.
#define SSAM_INSTANCE_2D_FUSED(T, DT, V, P, R, BUDGET, S, NT, VARIANT)                                          \
    static ::ssam::Register2D SSAM_CAT(reg2df_, __COUNTER__)(::ssam::Instance2D{                                 \
        #T "_R" #R "_b" #BUDGET "_v" #V "p" #P "nt" #NT "_fused" #S, DT, 2 * (R) + 1, 2 * (R) + 1, R, BUDGET,    \
        VARIANT,                                                                                                 \
        &::ssam::launch2d_fused<T, V, P, ::ssam::TapMask<2 * (R) + 1, 2 * (R) + 1, R, R, BUDGET>, S, NT>, S})

}  // namespace ssam
