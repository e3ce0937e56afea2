// 3D stencil kernel, block-cooperative variant: the waves of a block are stacked in y on the
// same x-strip and z range and share each input plane through LDS.
//
// Why: in the one-wave-per-tile kernel every wave fetches its own P + 2*RY rows of each plane,
// so neighbouring waves request the halo rows twice (3x the needed requests at RY = 4, P = 4).
// The march is bound by the latency of those requests, not by arithmetic or HBM bandwidth.
// Here the block fetches its NW*P + 2*RY rows once (each wave a share), stages them in LDS,
// and every wave reads its own window back from LDS.  LDS carries input rows between waves
// only -- the one place where waves need each other's data (the paper's Sec. 4.9 also couples
// the warps of a block through shared memory, there for the z direction).  Partial sums still
// move between lanes by DPP, and z is still the in-register direction (see ssam_kernel3d.h).
//
// Per step: request plane t+1 from global memory into a few staging registers; read this
// wave's window of plane t from LDS; evaluate; write the staged rows into the other LDS
// buffer; one barrier.  Boundary fix-ups are applied by the fetching wave, so LDS always holds
// boundary-corrected rows and the evaluation has no edge logic.
#pragma once
#include "ssam_kernel3d.h"

namespace ssam {

template <typename T, int V, int P, int NW, int RX, int RY, int RZ, int BUDGET, int NT>
__global__ __launch_bounds__(NW* kWave) void ssam3d_lds_kernel(
    const Args3D<T, SliceMask<RX, RY, RZ, BUDGET, 0>::kNW> a)
{
    constexpr int NZ = 2 * RZ + 1;
    constexpr int C = P + 2 * RY;            // rows one wave evaluates from
    constexpr int CB = NW * P + 2 * RY;      // rows the block stages per plane
    constexpr int RPW = (CB + NW - 1) / NW;  // rows each wave fetches per plane
    constexpr int ROWS = RPW * NW;           // staged rows incl. padding (>= CB)
    constexpr int HL = (RX + V - 1) / V;
    typedef typename VecOf<T, V>::type vec_t;

    __shared__ vec_t stage[2][ROWS][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lb = logical_block(blockIdx.x, a.blocks, a.xcd_remap);
    // block tile: strip fastest, then y block, then z chunk.  No wave may leave before the last
    // barrier, so blocks past the end are excluded as a whole (uniform for the block).
    if (lb >= a.tiles) return;
    const int strip = lb % a.strips_x;
    const int yblock = (lb / a.strips_x) % a.tiles_y;
    const int ztile = lb / (a.strips_x * a.tiles_y);

    const int W = a.W, H = a.H, D = a.D;
    const int xo0 = strip * a.valid_lanes * V;
    const int xw0 = xo0 - HL * V;
    const int xc = xw0 + lane * V;
    const int yb0 = yblock * (NW * P);       // first output row of the block
    const int y0 = yb0 + wave * P;           // first output row of this wave
    const int z0 = ztile * a.planes_per_wave;
    const int z1 = min(z0 + a.planes_per_wave, D);
    const bool vec_ok = a.aligned && (W % V) == 0;
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
    const int nt = (z1 - z0) + 2 * RZ;       // input planes z0-RZ .. z1-1+RZ

    const bool interior = vec_ok && xw0 >= 0 && xw0 + used_lanes * V <= W && yb0 - RY >= 0 &&
                          yb0 + ROWS - 1 - RY < H && z0 - RZ >= 0 && z1 - 1 + RZ < D;

    auto march = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;   // 0 interior, 1 general with vectors, 2 general by element
        constexpr bool EDGE = MODE != 0;
        constexpr bool VEC = MODE != 2;

        // this wave's share of plane z: staged rows wave, wave+NW, ... (row index within the block)
        auto fetch = [&](int z, T (&g)[RPW][V]) __attribute__((always_inline)) {
            if constexpr (!EDGE) {
                const T* pz = in + (size_t)z * plane + (size_t)(yb0 - RY + wave) * rowst + xl;
#pragma unroll
                for (int i = 0; i < RPW; ++i)
                    load_vec<T, V, (NT & kStreamLoads) != 0>(pz + (size_t)(i * NW) * rowst, g[i]);
            } else {
                const bool plane_in = z >= 0 && z < D;
                const T* pz = in + (size_t)min(max(z, 0), D - 1) * plane;
                const int xv = min(max(xl, 0), W - V);
#pragma unroll
                for (int i = 0; i < RPW; ++i) {
                    const int y = yb0 - RY + wave + i * NW;
                    const bool row_in = plane_in && y >= 0 && y < H;     // wave-uniform
                    const T* rowp = pz + (size_t)min(max(y, 0), H - 1) * rowst;
                    if constexpr (VEC) {
                        load_vec<T, V, (NT & kStreamLoads) != 0>(rowp + xv, g[i]);
                        const T first = g[i][0], last = g[i][V - 1];
                        const unsigned keep = keep_cols & (row_in ? ~0u : keep_rows);
#pragma unroll
                        for (int e = 0; e < V; ++e)
                            g[i][e] = keep_if(pick(pick(g[i][e], first, left_pick), last, right_pick), keep);
                    } else {
#pragma unroll
                        for (int e = 0; e < V; ++e) {
                            const int x = xc + e;
                            const T v = rowp[min(max(x, 0), W - 1)];
                            g[i][e] = (clamp || (row_in && x >= 0 && x < W)) ? v : T(0);
                        }
                    }
                }
            }
        };
        auto stash = [&](int b, const T (&g)[RPW][V]) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < RPW; ++i) {
                vec_t v;
                if constexpr (V == 1) v = g[i][0];
                else {
#pragma unroll
                    for (int e = 0; e < V; ++e) v[e] = g[i][e];
                }
                stage[b][wave + i * NW][lane] = v;
            }
        };
        auto grab = [&](int b, T (&r)[C][V]) __attribute__((always_inline)) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const vec_t v = stage[b][wave * P + k][lane];
                if constexpr (V == 1) r[k][0] = v;
                else {
#pragma unroll
                    for (int e = 0; e < V; ++e) r[k][e] = v[e];
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

        T g[RPW][V];
        fetch(z0 - RZ, g);
        stash(0, g);
        __syncthreads();

        for (int tb = 0; tb < nt; tb += 2) {
            static_for<2>([&](auto uc) __attribute__((always_inline)) {
                constexpr int cur = decltype(uc)::value;
                const int t = tb + cur;
                if (t < nt) {                                   // uniform for the whole block
                    const int zin = z0 - RZ + t;
                    // request the next plane (the step after the last re-reads an in-grid plane)
                    fetch(EDGE ? zin + 1 : min(zin + 1, D - 1), g);
                    T r[C][V];
                    grab(cur, r);
                    PlaneStep<T, V, P, RX, RY, RZ, BUDGET, 0>::run(r, wts, acc);

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
                                    for (int e = 0; e < V; ++e)
                                        if (xc + e < W) rowp[e] = acc[0][p][e];
                                }
                            }
                        }
                    }
                    stash(cur ^ 1, g);
                    __syncthreads();
                }
            });
        }
    };

    if (interior) march(std::integral_constant<int, 0>{});
    else if (vec_ok) march(std::integral_constant<int, 1>{});
    else march(std::integral_constant<int, 2>{});
}

template <typename T, int V, int P, int NW, int RX, int RY, int RZ, int BUDGET, int NT>
hipError_t launch3d_lds(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    typedef SliceMask<RX, RY, RZ, BUDGET, 0> Mask0;
    constexpr int HL = (RX + V - 1) / V;
    Geometry g;
    plan_strips(pr.W, V, HL, HL, tu.valid_lanes, &g);
    g.P = P;
    g.rows_per_wave = P;
    const int LH = pr.march_y ? pr.D : pr.H, LD = pr.march_y ? pr.H : pr.D;   // strip / march extents
    g.tiles_y = ceil_div(LH, NW * P);            // blocks of NW waves along the strip axis
    int planes = tu.planes_per_wave;
    if (planes <= 0) {   // 64 planes per block where the grid fills the machine with that, fewer on small grids
        int blocks_per_cu = 0, dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &blocks_per_cu, reinterpret_cast<const void*>(&ssam3d_lds_kernel<T, V, P, NW, RX, RY, RZ, BUDGET, NT>),
                NW * kWave, 0) != hipSuccess || blocks_per_cu <= 0) {
            (void)hipGetLastError();
            cus = 256;
            blocks_per_cu = 2;
        }
        planes = balanced_planes(LD, (long)g.strips_x * g.tiles_y, cus * blocks_per_cu, 64, 4 * RZ);
    }
    if (planes > LD) planes = LD;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(LD, planes);
    g.tiles = (long)g.strips_x * g.tiles_y * g.tiles_z;   // block tiles
    g.xcd_remap = tu.xcd_remap < 0 ? 1 : (tu.xcd_remap ? 1 : 0);
    g.blocks = g.xcd_remap ? ceil_div((int)g.tiles, kXcds) * kXcds : (int)g.tiles;
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args3D<T, Mask0::kNW> a;
    fill_args3d<T, V, RX, RY, RZ, BUDGET>(pr, g, &a);
    hipLaunchKernelGGL((ssam3d_lds_kernel<T, V, P, NW, RX, RY, RZ, BUDGET, NT>), dim3(g.blocks), dim3(NW * kWave),
                       0, pr.stream, a);
    return hipGetLastError();
}

#define SSAM_INSTANCE_3D_LDS(T, DT, V, P, NW, RX, RY, RZ, BUDGET, NT, VARIANT)                       \
    static ::ssam::Register3D SSAM_CAT(reg3dl_, __COUNTER__)(::ssam::Instance3D{                     \
        #T "_r" #RX #RY #RZ "_b" #BUDGET "_v" #V "p" #P "w" #NW "lds_nt" #NT, DT, RX, RY, RZ, BUDGET, \
        VARIANT, &::ssam::launch3d_lds<T, V, P, NW, RX, RY, RZ, BUDGET, NT>})

}  // namespace ssam
