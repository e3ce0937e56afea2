// Host-side types shared by the dispatcher (ssam_api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/ssam.h"
#include "../../include/ssam_tuning.h"

#define SSAM_CAT_(a, b) a##b
#define SSAM_CAT(a, b) SSAM_CAT_(a, b)

namespace ssam {

// Launch parameters a caller may override through ssam_set_tuning (negative = built-in).
// Scan overrides (ssam_set_tuning "scan_segments", "scan_order", "scan_chained", "scan_spin_limit",
// "scan_one_group");
// defined beside the scan kernels.
extern std::atomic<int> g_scan_segments, g_scan_order, g_scan_chained, g_scan_spin_limit, g_scan_one_group;

struct Tuning {
    int rows_per_wave = -1;    // 2D: output rows one wave marches over
    int valid_lanes = -1;      // lanes of a wave that store results (the rest are halo)
    int planes_per_wave = -1;  // 3D: output planes one wave marches over
    int xcd_remap = -1;        // 1: consecutive logical blocks share an XCD
    int force_generic = -1;    // 1: skip the compiled instances, use the direct kernel
    int variant = -1;          // pick an alternative compiled instance of the same shape
    int march_axis = -1;       // 3D: 0 march along z (strip along y), 1 march along y (strip along z)
    int embed_waste = -1;      // largest box-to-filter tap ratio for embedding an odd shape in a compiled box (0: never)
    int fuse_sweeps = -1;      // iteration: 0 = one sweep per launch, otherwise two where a fused instance exists
};

struct Problem2D {
    const void* in;
    void* out;
    int W, H;
    const void* w;  // host, [N][M]
    int M, N, ax, ay;
    int boundary, dtype;
    hipStream_t stream;
};

struct Problem3D {
    const void* in;
    void* out;
    int W, H, D;
    const void* c;  // host, [2rz+1][2ry+1][2rx+1]
    int rx, ry, rz;
    int boundary, dtype;
    hipStream_t stream;
    bool march_y = false;  // march along y with the register strip along z (instances see ry, rz exchanged)
    bool dense = false;    // filter semantics: every element of the box is a tap, zeros included
};

// Tile geometry of one launch (all host arithmetic; also reported by ssam_describe).
struct Geometry {
    int V = 0, P = 0;          // columns per lane, window positions per chunk
    int halo_left = 0, halo_right = 0;  // halo lanes on each side of a wave
    int valid_lanes = 0;       // lanes that store
    int strips_x = 0;          // tiles along x, each valid_lanes*V columns wide
    int tiles_y = 0;           // tiles along y
    int tiles_z = 1;           // tiles along z (3D)
    int rows_per_wave = 0;     // 2D: rows per tile; 3D: P
    int planes_per_wave = 0;   // 3D
    long tiles = 0;            // waves with work
    int blocks = 0;            // launched blocks (padded to a multiple of 8 when remapped)
    int xcd_remap = 0;
};

typedef hipError_t (*Launch2DFn)(const Problem2D&, const Tuning&, Geometry*, bool dry_run);
typedef hipError_t (*Launch3DFn)(const Problem3D&, const Tuning&, Geometry*, bool dry_run);

struct Instance2D {
    const char* name;
    int dtype, M, N, AX, budget;  // budget 2 = dense box, 1 = star
    int variant;                  // 0 = default instance for the shape
    Launch2DFn launch;
    int sweeps = 1;               // Jacobi sweeps one launch performs (2: the fused kernel, zero padding only)
};

struct Instance3D {
    const char* name;
    int dtype, rx, ry, rz, budget;  // budget = max number of non-zero offset components (1 star, 2, 3 box)
    int variant;
    Launch3DFn launch;
    int sweeps = 1;                 // Jacobi sweeps one launch performs (2: the fused kernel, z march only)
    bool fuses_clamp = false;       // the fused kernel also exists for the clamp rule (where it measured faster)
};

std::vector<Instance2D>& registry2d();
std::vector<Instance3D>& registry3d();

struct Register2D {
    explicit Register2D(const Instance2D& i) { registry2d().push_back(i); }
};
struct Register3D {
    explicit Register3D(const Instance3D& i) { registry3d().push_back(i); }
};

// a, b > 0; the sum is formed in 64 bits so that extents near 2^31 do not wrap
inline int ceil_div(int a, int b) { return (int)(((long long)a + b - 1) / b); }

inline bool pointers_aligned(const void* a, const void* b, size_t bytes)
{
    return ((uintptr_t)a % bytes) == 0 && ((uintptr_t)b % bytes) == 0;
}

// Overlapped blocking along x (paper Sec. 4.5 / 4.7 re-derived for 64 lanes of V columns):
// a wave caches 64*V columns and stores valid_lanes*V of them.  The strip width is kept a
// multiple of 8 lanes = 128 bytes where possible, so that strips start on cache-line
// boundaries and no line is written by two waves (measured: +7 % on 8192^2); among such
// widths the smallest that still covers W with the same number of strips is taken, so the
// last strip is not mostly empty.
inline void plan_strips(int W, int V, int halo_left, int halo_right, int valid_override, Geometry* g,
                        bool line_aligned = true)
{
    const int vmax = 64 - halo_left - halo_right;
    int valid;
    if (valid_override > 0) {
        valid = valid_override < vmax ? valid_override : vmax;
    } else {
        const int vline = (line_aligned && vmax >= 8) ? vmax / 8 * 8 : vmax;   // widest (line-aligned) strip
        const int strips = ceil_div(W, vline * V);
        valid = ceil_div(ceil_div(W, strips), V);             // balanced
        if (line_aligned && vmax >= 8) valid = ceil_div(valid, 8) * 8;
        if (valid > vline) valid = vline;
    }
    g->V = V;
    g->halo_left = halo_left;
    g->halo_right = halo_right;
    g->valid_lanes = valid;
    g->strips_x = ceil_div(W, valid * V);
}

// Waves of `kernel` (launched as blocks of 4 waves) the whole device can hold at once.  Falls
// back to a typical figure when no device is present (planning queries on a CPU-only host).
inline int wave_slots(const void* kernel)
{
    int blocks_per_cu = 0, dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks_per_cu, kernel, 256, 0) != hipSuccess ||
        blocks_per_cu <= 0) {
        (void)hipGetLastError();
        return 256 * 3 * 4;
    }
    return cus * blocks_per_cu * 4;
}

// Rows per tile (a multiple of P, at least min_rows) such that strips * ceil(H / rows) tiles fill
// `slots` wave slots k times as exactly as possible, k = 1 .. 4.  Among fills within 2 % of each other
// the tallest tiles win (they amortise the rows re-read at tile tops); with prefer_short the shortest win
// unless they are more than 5 % less full (measured better for the fp64 boxes in spite of the re-read rows:
// 8192^2 81-point 265 -> 258 us, 121-point 363 -> 351).  A grid too
// small to fill the slots even once gets the shortest tiles allowed (most waves).
inline int balanced_rows(int H, int P, int strips, int slots, int min_rows, bool prefer_short = false)
{
    const int shortest = ceil_div(min_rows < P ? P : min_rows, P) * P;
    auto fill = [&](int rows) {
        const long tiles = (long)strips * ceil_div(H, rows);
        const long rounds = (tiles + slots - 1) / slots;
        return (double)tiles / ((double)rounds * slots);
    };
    int best_rows = shortest;
    double best_eff = fill(shortest);
    bool first = true;
    for (int i = 1; i <= 4; ++i) {
        const int k = prefer_short ? 5 - i : i;
        const int ytiles = slots * k / strips;
        if (ytiles < 1) continue;
        int rows = ceil_div(ceil_div(H, ytiles), P) * P;
        if (rows < shortest) rows = shortest;
        const double eff = fill(rows);
        const bool preferred = prefer_short ? (first || rows < best_rows) : rows > best_rows;
        const double margin = prefer_short ? 0.05 : 0.02;
        if (eff > best_eff + margin || (preferred && eff > best_eff - margin)) {
            best_eff = eff;
            best_rows = rows;
        }
        first = false;
    }
    return best_rows;
}

// Planes per z-chunk of the 3D march: `preferred` where the grid is large enough to fill the wave
// slots with it, otherwise fewer (never under `fewest`), so that a small grid still spreads over
// the machine; every chunk re-reads its leading planes, which is why large grids keep `preferred`.
inline int balanced_planes(int D, long tiles_xy, int slots, int preferred, int fewest)
{
    int planes = preferred < D ? preferred : D;
    while (planes > fewest && tiles_xy * ceil_div(D, planes) < slots) planes = (planes + 1) / 2;
    if (planes < fewest) planes = fewest < D ? fewest : D;
    return planes;
}

// A launch dimension holds fewer than 2^32 threads: with blocks of at most 1024 threads that is 2^22
// blocks, whatever the kernel.  Launchers return hipErrorInvalidConfiguration for a plan beyond it.
constexpr long kMaxBlocks = (1L << 22) - 8;
inline bool launchable(const Geometry& g) { return g.blocks > 0 && g.blocks <= kMaxBlocks && g.tiles <= 4 * kMaxBlocks; }

inline void plan_blocks(Geometry* g, int remap_override)
{
    g->tiles = (long)g->strips_x * g->tiles_y * g->tiles_z;
    if (g->tiles > 4 * kMaxBlocks) {   // not launchable: leave a block count that says so
        g->xcd_remap = 0;
        g->blocks = -1;
        return;
    }
    int blocks = (int)((g->tiles + 3) / 4);
    g->xcd_remap = remap_override < 0 ? 1 : (remap_override ? 1 : 0);
    if (g->xcd_remap) blocks = ceil_div(blocks, 8) * 8;
    g->blocks = blocks;
}

}  // namespace ssam
