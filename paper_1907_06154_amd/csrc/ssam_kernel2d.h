// 2D filter / stencil kernel: register cache + systolic partial sums, one wave per tile.
//
// Tile of one wave (overlapped blocking, paper Sec. 4.5): 64 lanes x V columns wide, of
// which `valid_lanes` lanes store; `rows_per_wave` output rows tall.  The wave marches down
// its rows P at a time (the sliding window of Sec. 4.2, extended to a march: after each
// group of P window positions the last N-1 cached rows are kept and P new rows are loaded,
// so the vertical halo is read once per tile rather than once per P rows).
// Waves are independent (Sec. 4.5): the vector-unit engine uses no LDS and no barrier; the
// matrix-core engine builds its filter table in LDS once per workgroup (one barrier, before the
// march) and shares nothing else.
#pragma once
#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {

template <typename T, int NW>
struct Args2D {
    const T* in;
    T* out;
    int W, H;
    int ay;             // filter row that sits on the output row
    int boundary;
    int strips_x;
    long tiles;
    int valid_lanes;
    int rows_per_wave;  // multiple of P
    int blocks;         // launched blocks
    int xcd_remap;
    int aligned;
    int nt_loads, nt_stores;   // streaming cache policy for grid loads / stores        // both base pointers are aligned to V elements
    T w[NW];            // packed per Mask::widx, read through scalar loads (wave-uniform broadcast, Sec. 4.6)
};

// ENGINE 0: products on the vector unit (any type, any P).  ENGINE 1: products on the matrix cores
// (fp32, P = 4; see systolic_rows_mfma), with the filter laid out for them in LDS.
template <typename T, int V, int P, class Mask, bool PREFETCH, int NT, int ENGINE = 0>
__global__ __launch_bounds__(kBlock) void ssam2d_kernel(const Args2D<T, Mask::kNW> a)
{
    constexpr int N = Mask::kN;
    constexpr int HL = (Mask::kLeft + V - 1) / V;
    constexpr int HR = (Mask::kRight + V - 1) / V;
    static_assert(ENGINE == 0 || (sizeof(T) == 4 && P == 4), "the matrix-core engine is fp32, four window positions");

    typedef Args2D<T, Mask::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));
    __shared__ __attribute__((aligned(16))) float mfma_tab[ENGINE == 1 ? MfmaWeights<Mask>::kWords : 4];
    if constexpr (ENGINE == 1) {
        fill_mfma_weights<Mask>(wts, mfma_tab);      // before any wave leaves: every thread helps and waits
        __syncthreads();
    }

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
    const long tile = (long)lb * kWavesPerBlock + wave;
    if (tile >= a.tiles) return;
    const int strip = (int)(tile % a.strips_x);
    const int ytile = (int)(tile / a.strips_x);

    const int W = a.W, H = a.H;
    const int xo0 = strip * a.valid_lanes * V;   // first output column of the wave
    const int xw0 = xo0 - HL * V;                // first cached column of the wave
    const int xc = xw0 + lane * V;               // first column cached by this lane
    const int y0 = ytile * a.rows_per_wave;
    const int y1 = min(y0 + a.rows_per_wave, H);
    const bool vec_ok = a.aligned && (W % V) == 0;   // row starts stay V-aligned
    // lanes past the right halo hold nothing any stored output depends on: they re-read the last
    // needed lane's columns (same cache line, no extra traffic, no divergence)
    const int used_lanes = min(HL + a.valid_lanes + HR, kWave);
    const int xl = xw0 + min(lane, used_lanes - 1) * V;   // first column this lane loads
    const bool clamp = a.boundary == kClamp;
    const T* __restrict__ in = a.in;
    const bool lane_stores = lane >= HL && lane < HL + a.valid_lanes && xc < W;
    // per-lane column masks for the general path (a lane's V columns are all inside or all outside
    // the grid when rows are V-aligned)
    const unsigned left_mask = xc < 0 ? ~0u : 0u, right_mask = xc >= W ? ~0u : 0u;
    const unsigned left_pick = clamp ? left_mask : 0u, right_pick = clamp ? right_mask : 0u;
    const unsigned keep_cols = clamp ? ~0u : ~(left_mask | right_mask);
    const unsigned keep_rows = clamp ? ~0u : 0u;   // mask applied to a row outside the grid

    // A tile is "interior" when every row and column it touches lies inside the grid and can be
    // accessed as aligned vectors: then loads and stores need no check at all.  Every other
    // tile takes the general path, which applies the boundary rule (wave-uniform row logic,
    // per-lane selects for columns) and also serves grids whose rows are not V-aligned.
    const int nchunks = (y1 - y0 + P - 1) / P;
    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && (y1 - y0) % P == 0 &&
                          y0 - a.ay >= 0 && y0 + nchunks * P - 1 - a.ay + N - 1 < H;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        auto load_row = [&](int y, T (&dst)[V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                load_vec<T, V, (NT & kStreamLoads) != 0>(in + (size_t)y * W + xl, dst);
            } else {
                const bool row_in = y >= 0 && y < H;          // wave-uniform
                const int yy = min(max(y, 0), H - 1);
                const T* rowp = in + (size_t)yy * W;
                if constexpr (VEC) {
                    // x: W and xc are multiples of V, so a lane's V columns are all in or all out
                    const int xv = min(max(xl, 0), W - V);
                    load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + xv, dst);
                    // one branch-free sequence serves both rules: clamp replaces out-of-grid
                    // columns by the edge column, zero padding blanks them (and whole rows)
                    const T first = dst[0], last = dst[V - 1];
                    const unsigned keep = keep_cols & (row_in ? ~0u : keep_rows);
#pragma unroll
                    for (int i = 0; i < V; ++i)
                        dst[i] = keep_if(pick(pick(dst[i], first, left_pick), last, right_pick), keep);
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i) {
                        const int x = xc + i;
                        const T v = rowp[min(max(x, 0), W - 1)];
                        dst[i] = (clamp || (row_in && x >= 0 && x < W)) ? v : T(0);
                    }
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

        // The window of a group of P output rows is the N-1 rows kept from the previous group
        // (`keep`) followed by P newly loaded rows.  PREFETCH: two buffers of new rows alternate
        // and the next group's rows are requested before the current group is evaluated, so
        // their latency hides behind the arithmetic inside the wave; the march is unrolled by
        // two so the buffer in use is known at compile time and no row is copied except the
        // N-1 kept ones.  Without PREFETCH rows are loaded just before use and other waves
        // hide the latency.
        constexpr int KEEP = N - 1;
        T keep[KEEP > 0 ? KEEP : 1][V];
        T fresh[PREFETCH ? 2 : 1][P][V];
#pragma unroll
        for (int k = 0; k < KEEP; ++k) load_row(y0 - a.ay + k, keep[k]);
        if constexpr (PREFETCH) {
#pragma unroll
            for (int k = 0; k < P; ++k) load_row(y0 - a.ay + KEEP + k, fresh[0][k]);
        }

        for (int yb = y0; yb < y1; yb += 2 * P) {
            static_for<2>([&](auto half) __attribute__((always_inline)) {
                constexpr int cur = PREFETCH ? decltype(half)::value : 0;
                const int y = yb + decltype(half)::value * P;
                if (y < y1) {
                    if constexpr (PREFETCH) {
                        if (y + P < y1) {
#pragma unroll
                            for (int k = 0; k < P; ++k) load_row(y + P - a.ay + KEEP + k, fresh[cur ^ 1][k]);
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < P; ++k) load_row(y - a.ay + KEEP + k, fresh[0][k]);
                    }

                    T acc[P][V];
                    if constexpr (ENGINE == 1)
                        systolic_rows_mfma<V, Mask>(RowPair<T, V, KEEP, P>{keep, fresh[cur]}, mfma_tab + (lane & 3) * MfmaWeights<Mask>::kPitch, acc);
                    else
                        systolic_rows<T, V, P, Mask, false>(RowPair<T, V, KEEP, P>{keep, fresh[cur]}, wts, acc, acc);
                    store_rows(y, acc);

                    // rows P .. P+KEEP-1 of this window open the next one
#pragma unroll
                    for (int k = 0; k < KEEP; ++k)
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            keep[k][i] = (k + P < KEEP) ? keep[(k + P < KEEP) ? k + P : 0][i]
                                                        : fresh[cur][(k + P >= KEEP) ? k + P - KEEP : 0][i];
                }
            });
        }
    };

    // the mode is wave-uniform and fixed for the whole march, so no load sits behind a branch
    if (interior) march(std::integral_constant<int, 0>{});
    else if (vec_ok) march(std::integral_constant<int, 1>{});
    else march(std::integral_constant<int, 2>{});
}

template <typename T, int V, int P, class Mask, bool PREFETCH, int NT, int ENGINE = 0>
hipError_t launch2d(const Problem2D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int M = Mask::kM, N = Mask::kN;
    constexpr int HL = (Mask::kLeft + V - 1) / V, HR = (Mask::kRight + V - 1) / V;
    Geometry g;
    // Filters of 7x7 and more are limited by instruction issue: they use every lane they can and balance the
    // tile count; bandwidth-bound ones keep strips line-aligned and tiles short.  (Measured on 8192^2 fp32 with
    // the input cold in the memory-side cache: 6x6 124 -> 104 us, 11x3 123 -> 102, 3x11 120 -> 110 when planned
    // as bandwidth-bound, and no slower on an input resident in that cache; 7x7 the same either way; 8x8 and up
    // 3-4 % slower.)
    constexpr bool kArith = Mask::kNW >= 40;
    plan_strips(pr.W, V, HL, HR, tu.valid_lanes, &g, !kArith);
    g.P = P;
    int rows;
    if (tu.rows_per_wave > 0) {
        rows = tu.rows_per_wave;
    } else if (kArith) {
        // arithmetic-heavy filters: every wave takes about the same time, so the tile count should
        // fill the machine's wave slots a whole number of times (a partly filled last round costs
        // a full one).  Measured on 8192^2, 20x20: 57 -> 73 GStencil/s.
        static const int slots = wave_slots(reinterpret_cast<const void*>(&ssam2d_kernel<T, V, P, Mask, PREFETCH, NT, ENGINE>));
        rows = balanced_rows(pr.H, P, g.strips_x, slots, 3 * (N - 1), sizeof(T) == 8);
    } else {
        // bandwidth-bound: the shortest tiles measured best -- one or two groups per wave, about twice the
        // N-1 rows a tile re-reads at its top (8192^2: 3x3 fp32 839 -> 918 GStencil/s from 32 to 8 rows,
        // 5x5 760 -> 858, fp64 17-point star 343 -> 370 from 64 to 16); many short waves sweep the grid
        // in step and finish together, which matters more than the re-read rows, which hit in L2
        rows = 2 * (N - 1) > P ? 2 * (N - 1) : P;
    }
    while ((long)g.strips_x * ceil_div(pr.H, rows) > 4 * kMaxBlocks) rows *= 2;   // very tall grids: fewer, taller tiles
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
    const T* w = static_cast<const T*>(pr.w);   // host, dense [N][M]
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m)
            if (Mask::tap(n, m)) a.w[Mask::widx(n, m)] = w[n * M + m];
    hipLaunchKernelGGL((ssam2d_kernel<T, V, P, Mask, PREFETCH, NT, ENGINE>), dim3(g.blocks), dim3(kBlock), 0, pr.stream, a);
    return hipGetLastError();
}

// Registers ssam2d_kernel<T, V, P, TapMask<M, N, AX, N/2, BUDGET>, PREFETCH, NT> under the
// dispatcher.  NT: bit 0 = streaming loads, bit 1 = streaming stores.  VARIANT 0 is the
// instance used by default; others are alternatives selectable for tuning.
#define SSAM_INSTANCE_2D_V(T, DT, V, P, M, N, AX, BUDGET, PREFETCH, NT, VARIANT)                     \
    static ::ssam::Register2D SSAM_CAT(reg2d_, __COUNTER__)(::ssam::Instance2D{                      \
        #T "_M" #M "N" #N "_b" #BUDGET "_v" #V "p" #P "f" #PREFETCH "nt" #NT, DT, M, N, AX, BUDGET,   \
        VARIANT,                                                                                      \
        &::ssam::launch2d<T, V, P, ::ssam::TapMask<M, N, AX, (N) / 2, BUDGET>, (PREFETCH) != 0, NT>})
#define SSAM_INSTANCE_2D(T, DT, V, P, M, N, AX, BUDGET) SSAM_INSTANCE_2D_V(T, DT, V, P, M, N, AX, BUDGET, 1, 2, 0)
// The same with the products on the matrix cores (fp32, P = 4); the name ends in "mx".
#define SSAM_INSTANCE_2D_MFMA(V, M, N, AX, BUDGET, PREFETCH, NT, VARIANT)                                 \
    static ::ssam::Register2D SSAM_CAT(reg2d_, __COUNTER__)(::ssam::Instance2D{                      \
        "float_M" #M "N" #N "_b" #BUDGET "_v" #V "p4f" #PREFETCH "nt" #NT "mx", SSAM_F32, M, N, AX, BUDGET, \
        VARIANT,                                                                                      \
        &::ssam::launch2d<float, V, 4, ::ssam::TapMask<M, N, AX, (N) / 2, BUDGET>, (PREFETCH) != 0, NT, 1>})

}  // namespace ssam
