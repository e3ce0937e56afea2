// Two sweeps of the 7-point 3D star (radius 1, zero padding) in one launch, block-cooperative: the
// temporal blocking of ssam_kernel3d_fused.h on the plane ring of ssam_kernel3d_star.h.
//
// The block stages every input plane once (its NW*P output rows plus two rows and two columns on every
// side) straight into a ring of LDS buffers, two plane-steps ahead, exactly as the single-sweep kernel
// does.  Each wave then runs both sweeps in its own registers and shares nothing but the staged input:
//   level 1  the first sweep on the wave's P rows widened by one row above and below and one COLUMN on
//            either side of every lane's V columns: (P + 2) x (V + 2) points per lane, the output planes
//            in flight along z as usual.  The widening rows are recomputed by the neighbouring wave and
//            the widening columns by the neighbouring lane; that redundancy (3x the first sweep at P = 4, V = 2 and
//            at P = 2, V = 4) is arithmetic the 7-point star has to spare -- one sweep keeps 12 % of the
//            vector issue slots busy -- and in exchange no first-sweep value ever crosses a lane or a wave,
//            all 64 lanes store, and nothing but the grid itself goes through memory;
//   level 2  the second sweep on the P x V points the lane owns, fed by the first-sweep plane that has just
//            completed (masked to zero where it lies outside the grid: zero padding of the second sweep).
// A launch reads the grid once and writes it once for two sweeps.
// Requirements (the launcher falls back to the one-wave-per-tile two-sweep kernel otherwise): zero padding,
// march along z, W a multiple of V, 16-byte aligned base pointers, planes below 4 GiB.
#pragma once
#include "ssam_kernel3d_fused.h"
#include "ssam_kernel3d_star.h"

namespace ssam {

template <typename T, int P, int NW, int NBUF, int NT>
__global__ __launch_bounds__(NW* kWave) __attribute__((amdgpu_waves_per_eu(2))) void ssam3d_star2_kernel(
    const Args3D<T, SliceMask<1, 1, 1, 1, 0>::kNW> a)
{
    static_assert(NBUF == 3 || NBUF == 4, "a ring of three or four staged planes");
    constexpr int PF = NBUF - 1;               // planes requested ahead
    constexpr int V = Piece16<T>::V;
    typedef typename Piece16<T>::type vec_t;
    constexpr int HR = 2;                      // input rows / columns / planes needed beyond the outputs, per side
    constexpr int C = P + 2 * HR;              // input rows one wave evaluates from
    constexpr int L1R = P + 2, L1C = V + 2;    // first-sweep points per lane: rows y0-1 .. y0+P, columns xc-1 .. xc+V
    constexpr int NTHR = NW * kWave;
    typedef PlaneFetch<T, NW * P + 2 * HR, 1, NTHR> Fetch;   // NW*P + 4 rows per plane; one halo piece per side holds the two columns
    constexpr int RS = Fetch::RS, NCH = Fetch::NCH, SLOTS = Fetch::SLOTS;
    constexpr bool NT_STORE = (NT & kStreamStores) != 0;
    static_assert(V >= 2, "the two halo columns of a side come from one 16-byte piece");
    static_assert((PF - 1) * NCH + PF * P <= 30, "request count beyond what the wait encodes");

    __shared__ vec_t stage[NBUF][SLOTS];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
    if (lb >= a.tiles) return;                 // block-uniform: no wave is left waiting at a barrier
    const int strip = lb % a.strips_x;
    const int yblock = (lb / a.strips_x) % a.tiles_y;
    const int ztile = lb / (a.strips_x * a.tiles_y);

    const int W = a.W, H = a.H, D = a.D;
    const int x0 = strip * (kWave * V);
    const int xc = x0 + lane * V;              // first column this lane owns
    const int yb0 = yblock * (NW * P);
    const int y0 = yb0 + wave * P;             // first output row of this wave
    const int z0 = ztile * a.planes_per_wave;
    const int z1 = min(z0 + a.planes_per_wave, D);
    const T* __restrict__ in = a.in;
    typedef Args3D<T, SliceMask<1, 1, 1, 1, 0>::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));   // z line (0..2, centre at 1), y line (3..5), x line (6..8)
    const size_t rowst = (size_t)a.stride_row, plane = (size_t)a.stride_plane;
    const int nt = (z1 - z0) + 2 * HR;         // input planes z0-2 .. z1+1

    const bool inside_xy = x0 - V >= 0 && x0 + (kWave + 1) * V <= W && yb0 - HR >= 0 && yb0 + NW * P + HR <= H;

    Fetch fetch;
    fetch.plan(tid, x0, yb0 - HR, W, H, rowst);

    // where the first sweep's points of this lane lie inside the grid (outside, the second sweep sees zero)
    unsigned colmask[L1C], rowmask[L1R];
#pragma unroll
    for (int c = 0; c < L1C; ++c) colmask[c] = (xc + c - 1 >= 0 && xc + c - 1 < W) ? ~0u : 0u;
#pragma unroll
    for (int r = 0; r < L1R; ++r) rowmask[r] = (y0 + r - 1 >= 0 && y0 + r - 1 < H) ? ~0u : 0u;

    // planes in flight: slot 1 = the plane the current input plane is the centre of, slot 2 = the one below it
    // (slot 0, the plane that completes, is produced and consumed within a step)
    T acc1[3][L1R][L1C], acc2[3][P][V];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
#pragma unroll
        for (int r = 0; r < L1R; ++r)
#pragma unroll
            for (int c = 0; c < L1C; ++c) acc1[s][r][c] = T(0);
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int j = 0; j < V; ++j) acc2[s][p][j] = T(0);
    }

    const bool lane_stores = xc < W;
    const int own = (wave * P) * RS + 1 + lane;      // this lane's piece of the wave's first staged row
    const int edge_l = (wave * P) * RS;              // the row's left halo piece
    const int edge_r = (wave * P) * RS + 1 + kWave;  // the row's right halo piece
    const T wzm = wts[0], wzc = wts[1], wzp = wts[2], wym = wts[3], wyp = wts[5], wxm = wts[6], wxp = wts[8];

    // one step of the march: the staged plane `st` is input plane zin
    auto step = [&](const vec_t* st, int zin) __attribute__((always_inline)) {
        // ---- level 1: input plane zin into the first-sweep planes zin-1 (completes), zin, zin+1 ----
        T sum[L1R][L1C];
#pragma unroll
        for (int r = 0; r < L1R; ++r)
#pragma unroll
            for (int c = 0; c < L1C; ++c) sum[r][c] = acc1[2][r][c];     // what plane zin has received from plane zin-1
#pragma unroll
        for (int k = 0; k < C; ++k) {          // input row y0 - 2 + k
            T xs[V + 4];                       // columns xc-2 .. xc+V+1
            const vec_t v = st[own + k * RS];
            const vec_t el = st[edge_l + k * RS], er = st[edge_r + k * RS];   // same address in every lane: a broadcast
#pragma unroll
            for (int j = 0; j < V; ++j) xs[2 + j] = v[j];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                xs[j] = shift_in_up((T)v[V - 2 + j], (T)el[V - 2 + j]);       // the last two columns of the lane below
                xs[V + 2 + j] = shift_in_down((T)v[j], (T)er[j]);             // the first two of the lane above
            }
            const int rc = k - 1;              // first-sweep row this input row is the centre row of
            if (rc >= 0 && rc < L1R) {
#pragma unroll
                for (int c = 0; c < L1C; ++c) {
                    const T x = xs[c + 1];
                    acc1[0][rc][c] = fma_into(x, wzp, acc1[1][rc][c]);
                    acc1[2][rc][c] = x * wzm;
                    sum[rc][c] = fma_t(x, wzc, sum[rc][c]);
                    sum[rc][c] = fma_t(xs[c], wxm, sum[rc][c]);
                    sum[rc][c] = fma_t(xs[c + 2], wxp, sum[rc][c]);
                }
            }
            if (k < L1R) {                     // the row above first-sweep row k
#pragma unroll
                for (int c = 0; c < L1C; ++c) sum[k][c] = fma_t(xs[c + 1], wym, sum[k][c]);
            }
            if (k - 2 >= 0) {                  // the row below first-sweep row k - 2
#pragma unroll
                for (int c = 0; c < L1C; ++c) sum[k - 2][c] = fma_t(xs[c + 1], wyp, sum[k - 2][c]);
            }
        }
#pragma unroll
        for (int r = 0; r < L1R; ++r)
#pragma unroll
            for (int c = 0; c < L1C; ++c) acc1[1][r][c] = sum[r][c];

        // ---- the first-sweep plane zin-1 is complete: zero outside the grid, then level 2 --------------
        const int zl = zin - 1;
        const unsigned planemask = (zl >= 0 && zl < D) ? ~0u : 0u;
        T u[L1R][L1C];
#pragma unroll
        for (int r = 0; r < L1R; ++r)
#pragma unroll
            for (int c = 0; c < L1C; ++c) u[r][c] = keep_if(acc1[0][r][c], rowmask[r] & colmask[c] & planemask);
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const T x = u[p + 1][j + 1];
                acc2[0][p][j] = fma_into(x, wzp, acc2[1][p][j]);
                T s2 = fma_into(x, wzc, acc2[2][p][j]);
                acc2[2][p][j] = x * wzm;
                s2 = fma_t(u[p + 1][j], wxm, s2);
                s2 = fma_t(u[p + 1][j + 2], wxp, s2);
                s2 = fma_t(u[p][j + 1], wym, s2);
                s2 = fma_t(u[p + 2][j + 1], wyp, s2);
                acc2[1][p][j] = s2;
            }

        // output plane zin - 2 has now received its last contribution
        const int zo = zin - 2;
        if (zo >= z0 && lane_stores) {
            T* po = a.out + (size_t)zo * plane + (size_t)y0 * rowst + xc;
#pragma unroll
            for (int p = 0; p < P; ++p)
                if (y0 + p < H) store_vec<T, V, NT_STORE>(po + (size_t)p * rowst, acc2[0][p]);
        }
    };

    // ---- planes straight into LDS, PF steps ahead (see ssam3d_star_kernel) ---------------------------
    auto request = [&](int z, int b) __attribute__((always_inline)) { fetch.request(in, plane, z, D, false, inside_xy, stage[b], wave); };
    // a wave that stores all P rows issues P stores per step once output planes complete (step 2*HR on)
    const bool full_rows = y0 + P <= H;
#pragma unroll
    for (int k = 0; k < PF; ++k)
        if (k < nt) request(z0 - HR + k, k);
    int b = 0;
    for (int t = 0; t < nt; ++t) {
        // away from both ends of the chunk the count is one of two constants (as in ssam3d_star_kernel)
        constexpr int kSteadyLoads = (PF - 1) * NCH, kSteadyAll = kSteadyLoads + PF * P;
        if (t >= 2 * HR + PF && t + PF <= nt) {
            if (full_rows) wait_and_sync_n<(kSteadyAll & ~1)>();
            else wait_and_sync_n<(kSteadyLoads & ~1)>();
        } else {
            wait_and_sync(younger_requests<PF, NCH, P>(t, nt, full_rows, 2 * HR));
        }
        if (t + PF < nt) request(z0 - HR + t + PF, b + PF >= NBUF ? b + PF - NBUF : b + PF);
        asm volatile("" ::: "memory");   // the step's stores stay behind its requests: the count above relies on it
        step(stage[b], z0 - HR + t);
        b = b + 1 == NBUF ? 0 : b + 1;
    }
}

// FALLBACK: the launcher of the two-sweep instance that takes what this kernel does not (the clamp rule, rows
// that are not a multiple of 16 bytes, unaligned base pointers, planes beyond 4 GiB).
template <typename T, int P, int NW, int NBUF, int NT, Launch3DFn FALLBACK>
hipError_t launch3d_star2(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int V = Piece16<T>::V;
    if (pr.march_y) return hipErrorInvalidValue;
    const size_t slice = (size_t)pr.H * pr.W * sizeof(T);
    if (pr.boundary != SSAM_BOUNDARY_ZERO || pr.W % V != 0 || slice > 0xffffffffull ||
        (!dry_run && !pointers_aligned(pr.in, pr.out, 16)))
        return FALLBACK(pr, tu, geo, dry_run);
    Geometry g;
    g.V = V;
    g.P = P;
    g.halo_left = g.halo_right = 0;
    g.valid_lanes = kWave;
    g.strips_x = ceil_div(pr.W, kWave * V);
    g.rows_per_wave = P;
    g.tiles_y = ceil_div(pr.H, NW * P);
    int planes = tu.planes_per_wave;
    if (planes <= 0) {
        // the longest z-chunks that still give every compute unit its share of blocks (each re-reads four planes)
        int blocks_per_cu = 0, dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &blocks_per_cu, reinterpret_cast<const void*>(&ssam3d_star2_kernel<T, P, NW, NBUF, NT>), NW * kWave, 0) !=
                hipSuccess ||
            blocks_per_cu <= 0) {
            (void)hipGetLastError();
            cus = 256;
            blocks_per_cu = 1;
        }
        planes = balanced_planes(pr.D, (long)g.strips_x * g.tiles_y, cus * blocks_per_cu, pr.D, 8);
        planes = staggered_planes(planes, pr.D, slice);
    }
    if (planes > pr.D) planes = pr.D;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(pr.D, planes);
    g.tiles = (long)g.strips_x * g.tiles_y * g.tiles_z;   // block tiles
    g.xcd_remap = tu.xcd_remap < 0 ? 1 : (tu.xcd_remap ? 1 : 0);
    g.blocks = g.tiles > kMaxBlocks ? -1 : (g.xcd_remap ? ceil_div((int)g.tiles, kXcds) * kXcds : (int)g.tiles);
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args3D<T, SliceMask<1, 1, 1, 1, 0>::kNW> a;
    fill_args3d<T, V, 1, 1, 1, 1>(pr, g, &a);
    hipLaunchKernelGGL((ssam3d_star2_kernel<T, P, NW, NBUF, NT>), dim3(g.blocks), dim3(NW * kWave), 0, pr.stream, a);
    return hipGetLastError();
}

// Two sweeps per launch; the clamp rule goes to FALLBACK, which has it.
#define SSAM_INSTANCE_3D_STAR2(T, DT, P, NW, NBUF, NT, FALLBACK, VARIANT)                                    \
    static ::ssam::Register3D SSAM_CAT(reg3ds2_, __COUNTER__)(::ssam::Instance3D{                           \
        #T "_r111_b1_p" #P "w" #NW "star_ring" #NBUF "nt" #NT "_fused2", DT, 1, 1, 1, 1, VARIANT,            \
        &::ssam::launch3d_star2<T, P, NW, NBUF, NT, FALLBACK>, 2, true})

}  // namespace ssam
