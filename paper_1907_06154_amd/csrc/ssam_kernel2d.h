// 2D filter / stencil kernel: register cache + systolic partial sums, one wave per tile.
//
// Tile of one wave (overlapped blocking, paper Sec. 4.5): 64 lanes x V columns wide, of
// which `valid_lanes` lanes store; `rows_per_wave` output rows tall.  The wave marches down
// its rows P at a time (the sliding window of Sec. 4.2, extended to a march: after each
// group of P window positions the last N-1 cached rows are kept and P new rows are loaded,
// so the vertical halo is read once per tile rather than once per P rows).
// No LDS and no barrier: waves are independent (Sec. 4.5).
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

template <typename T, int V, int P, class Mask, bool PREFETCH, int NT>
__global__ __launch_bounds__(kBlock) void ssam2d_kernel(const Args2D<T, Mask::kNW> a)
{
    constexpr int N = Mask::kN;
    constexpr int HL = (Mask::kLeft + V - 1) / V;
    constexpr int C = N + P - 1;   // cached rows per lane (paper Eq. 3)

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
    const bool fast_x = vec_ok && xw0 >= 0 && xw0 + kWave * V <= W;   // wave-uniform
    const bool clamp = a.boundary == kClamp;
    const T* __restrict__ in = a.in;
    typedef Args2D<T, Mask::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));

    auto load_row = [&](int y, T (&dst)[V]) __attribute__((always_inline)) {
        if (clamp) {
            y = min(max(y, 0), H - 1);
        } else if (y < 0 || y >= H) {
#pragma unroll
            for (int i = 0; i < V; ++i) dst[i] = T(0);
            return;
        }
        const T* rowp = in + (size_t)y * W;
        if (fast_x) {
            load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + xc, dst);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const int x = xc + i;
                if (clamp) dst[i] = rowp[min(max(x, 0), W - 1)];
                else dst[i] = (x >= 0 && x < W) ? rowp[x] : T(0);
            }
        }
    };

    // PREFETCH: the next P rows are requested into a second buffer before the current ones
    // are used (latency hidden inside the wave, at the price of P*V more registers);
    // otherwise rows are loaded straight into the cache and other waves hide the latency.
    T r[C][V];
    T nxt[PREFETCH ? P : 1][V];
#pragma unroll
    for (int k = 0; k < N - 1; ++k) load_row(y0 - a.ay + k, r[k]);
    if constexpr (PREFETCH) {
#pragma unroll
        for (int k = 0; k < P; ++k) load_row(y0 - a.ay + N - 1 + k, nxt[k]);
    }

    const bool lane_stores = lane >= HL && lane < HL + a.valid_lanes && xc < W;

    for (int y = y0; y < y1; y += P) {
        if constexpr (PREFETCH) {
#pragma unroll
            for (int k = 0; k < P; ++k)
#pragma unroll
                for (int i = 0; i < V; ++i) r[N - 1 + k][i] = nxt[k][i];
            if (y + P < y1) {
#pragma unroll
                for (int k = 0; k < P; ++k) load_row(y + P - a.ay + N - 1 + k, nxt[k]);
            }
        } else {
#pragma unroll
            for (int k = 0; k < P; ++k) load_row(y - a.ay + N - 1 + k, r[N - 1 + k]);
        }

        T acc[P][V];
        systolic_rows<T, V, P, Mask, false, C>(r, wts, acc, acc);

        if (lane_stores) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (y + p < y1) {
                    T* rowp = a.out + (size_t)(y + p) * W;
                    if (vec_ok) {
                        store_vec<T, V, (NT & kStreamStores) != 0>(rowp + xc, acc[p]);
                    } else {
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            if (xc + i < W) rowp[xc + i] = acc[p][i];
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < N - 1; ++k)
#pragma unroll
            for (int i = 0; i < V; ++i) r[k][i] = r[k + P][i];
    }
}

template <typename T, int V, int P, class Mask, bool PREFETCH, int NT>
hipError_t launch2d(const Problem2D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int M = Mask::kM, N = Mask::kN;
    constexpr int HL = (Mask::kLeft + V - 1) / V, HR = (Mask::kRight + V - 1) / V;
    Geometry g;
    plan_strips(pr.W, V, HL, HR, tu.valid_lanes, &g);
    g.P = P;
    int rows = tu.rows_per_wave > 0 ? tu.rows_per_wave : (N <= 5 ? 32 : (N <= 11 ? 64 : 128));
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
    const T* w = static_cast<const T*>(pr.w);   // host, dense [N][M]
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m)
            if (Mask::tap(n, m)) a.w[Mask::widx(n, m)] = w[n * M + m];
    hipLaunchKernelGGL((ssam2d_kernel<T, V, P, Mask, PREFETCH, NT>), dim3(g.blocks), dim3(kBlock), 0, pr.stream, a);
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

}  // namespace ssam
