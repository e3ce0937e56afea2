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
// Zero padding only: an intermediate value at a position outside the grid must read as 0 for
// the next sweep, which a mask does; under the clamp rule it would be the value of another
// row or lane, so the dispatcher keeps clamp on the one-sweep kernel.
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

    // The group with base y loads input rows y + S*R .. y + S*R + P-1; sweep k (0-based) turns
    // them into its rows y + (S-1-k)*R .. + P-1, and the last sweep's rows y .. y+P-1 are stored
    // from y0 on.  Sweep k's rows are complete from row ys + (S-1+k)*R on (its kept rows start
    // as zeros), which the warm-up groups put at or above y0 for the last sweep.
    const int nchunks = (y1 - y0 + P - 1) / P;
    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && (y1 - y0) % P == 0 &&
                          ys + (S - 2) * R >= 0 && y0 + (nchunks - 1) * P + S * R + P - 1 < H;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        unsigned col_keep[V];   // all-ones where the lane's column lies inside the grid
#pragma unroll
        for (int i = 0; i < V; ++i) col_keep[i] = (xc + i >= 0 && xc + i < W) ? ~0u : 0u;

        auto load_row = [&](int y, T (&dst)[V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                load_vec<T, V, (NT & kStreamLoads) != 0>(in + (size_t)y * W + xl, dst);
            } else {
                const unsigned row_keep = (y >= 0 && y < H) ? ~0u : 0u;   // wave-uniform
                const T* rowp = in + (size_t)min(max(y, 0), H - 1) * W;
                if constexpr (VEC) {
                    load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + min(max(xl, 0), W - V), dst);
#pragma unroll
                    for (int i = 0; i < V; ++i) dst[i] = keep_if(dst[i], col_keep[0] & row_keep);
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i) dst[i] = keep_if(rowp[min(max(xc + i, 0), W - 1)], col_keep[i] & row_keep);
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
#pragma unroll
                            for (int p = 0; p < P; ++p) {
                                const int yr = y + (S - 1 - k) * R + p;
                                const unsigned row_keep = (yr >= 0 && yr < H) ? ~0u : 0u;
#pragma unroll
                                for (int i = 0; i < V; ++i) mid[k][p][i] = keep_if(mid[k][p][i], col_keep[VEC ? 0 : i] & row_keep);
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
    else if (vec_ok) march(std::integral_constant<int, 1>{});
    else march(std::integral_constant<int, 2>{});
}

template <typename T, int V, int P, class Mask, int S, int NT>
hipError_t launch2d_fused(const Problem2D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int M = Mask::kM, N = Mask::kN;
    constexpr int HL = (S * Mask::kLeft + V - 1) / V;
    static_assert(64 - 2 * HL >= 8, "stencil too wide for this many sweeps in one wave");
    if (pr.boundary != SSAM_BOUNDARY_ZERO) return hipErrorInvalidValue;
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
