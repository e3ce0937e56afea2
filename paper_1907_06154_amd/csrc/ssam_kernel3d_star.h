// 3D star stencil of radius R, block-cooperative: the NW waves of a block are stacked in y on one
// x-strip, share every input plane through LDS, and march along z with the output planes in
// flight held in registers (z is the in-register direction, see ssam_kernel3d.h).
//
// What differs from ssam_kernel3d_lds.h, and why (measured on 512^3, radius 4, where that kernel
// ran at 0.45 / 0.53 of the HBM peak with half its wave-cycles waiting):
//   - No halo lanes.  A wave's 64 lanes own 64*V adjacent columns and store all of them.  The
//     columns a wave needs beyond its own come from the staged plane in LDS, which holds the
//     strip plus R columns on either side: lane 0 (lane 63) reads them, and the lane-to-lane
//     shift takes them in as the value of the lane that does not exist -- a DPP whole-wave shift
//     leaves the destination of a lane without a source untouched, so the shift writes into the
//     register that already holds the halo columns.  No instruction is added for it, and a 512-
//     column row is two (fp32) or four (fp64) full waves instead of five with 56 storing lanes.
//   - The in-plane x taps multiply neighbouring INPUT columns, shifted in once per centre row
//     (ceil(R/V) shifts of V values per side), instead of shifting partial sums per tap group:
//     a star has x taps in the centre row of each window only.
//   - The fetch is decoupled from the lane layout: the block's threads split the staged tile
//     (NW*P + 2R rows of 64 + 2*ceil(R/V) 16-byte pieces) evenly, so every row is read as one
//     contiguous run and the rows shared by the waves of a block are fetched once.
//   - Planes travel from global memory straight into LDS (global_load_lds_dwordx4: every lane
//     names its own 16 source bytes, the wave's 64 pieces land side by side in LDS), NBUF - 1
//     plane-steps ahead of their use in a ring of NBUF buffers.  No register is spent on data in
//     flight, so two plane-steps of arithmetic cover the memory latency where the register-staged
//     kernel had less than one.  The block synchronises once per step: every wave waits until its
//     own loads of the plane about to be used have landed (they complete in order, so a count of
//     the younger requests that may stay outstanding is enough), then one barrier.
//   - Boundary rule in the fetch.  Zero padding: a piece outside the grid is loaded from 16 zero
//     bytes the library keeps in device memory (so every lane issues every load and the request
//     counts are the same in all waves).  Clamp: row and plane indices are clamped in the fetch (a
//     replicated row or plane is a plain load); columns left or right of the grid take the edge
//     column of their row, which no plain load delivers, so blocks at the left or right edge of the
//     grid replace those pieces when they READ the staged plane: one more broadcast read of the
//     row's edge piece, only in those blocks.
// Requirements (the launcher falls back to ssam3d_lds_kernel otherwise): W a multiple of V and
// both base pointers 16-byte aligned.
#pragma once
#include "ssam_kernel3d_lds.h"

namespace ssam {

template <typename T>
struct Piece16 {
    static constexpr int V = 16 / (int)sizeof(T);
    typedef typename VecOf<T, V>::type type;
};

// old where the lane has no source, else the value of the lane below / above (see the file header)
__device__ __forceinline__ int shift_in_up(int v, int edge) { return __builtin_amdgcn_update_dpp(edge, v, 0x138, 0xf, 0xf, false); }
__device__ __forceinline__ int shift_in_down(int v, int edge) { return __builtin_amdgcn_update_dpp(edge, v, 0x130, 0xf, 0xf, false); }
__device__ __forceinline__ float shift_in_up(float v, float edge)
{
    return __builtin_bit_cast(float, shift_in_up(__builtin_bit_cast(int, v), __builtin_bit_cast(int, edge)));
}
__device__ __forceinline__ float shift_in_down(float v, float edge)
{
    return __builtin_bit_cast(float, shift_in_down(__builtin_bit_cast(int, v), __builtin_bit_cast(int, edge)));
}
__device__ __forceinline__ double shift_in_up(double v, double edge)
{
    Halves a = __builtin_bit_cast(Halves, v), e = __builtin_bit_cast(Halves, edge);
    a.lo = shift_in_up(a.lo, e.lo);
    a.hi = shift_in_up(a.hi, e.hi);
    return __builtin_bit_cast(double, a);
}
__device__ __forceinline__ double shift_in_down(double v, double edge)
{
    Halves a = __builtin_bit_cast(Halves, v), e = __builtin_bit_cast(Halves, edge);
    a.lo = shift_in_down(a.lo, e.lo);
    a.hi = shift_in_down(a.hi, e.hi);
    return __builtin_bit_cast(double, a);
}

// Waits until at most n of this wave's vector-memory requests are outstanding and every LDS
// access of the wave is done, then joins the block's barrier.  One statement, so that nothing is
// scheduled in between, and a compiler-level memory barrier.  (The fence of __syncthreads would
// wait for ALL outstanding loads into LDS, which is exactly what the ring of buffers avoids.)
template <int N>
__device__ __forceinline__ void wait_and_sync_n()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}
__device__ __forceinline__ void wait_and_sync(int n)   // n block-uniform, 0 .. 31; rounded down to a multiple of 2
{
    switch (n >> 1) {
#define SSAM_WS(k) case k: wait_and_sync_n<2 * k>(); break;
        SSAM_WS(0) SSAM_WS(1) SSAM_WS(2) SSAM_WS(3) SSAM_WS(4) SSAM_WS(5) SSAM_WS(6) SSAM_WS(7)
        SSAM_WS(8) SSAM_WS(9) SSAM_WS(10) SSAM_WS(11) SSAM_WS(12) SSAM_WS(13) SSAM_WS(14)
#undef SSAM_WS
        default: wait_and_sync_n<30>(); break;
    }
}

// Every lane of the wave loads its own 16 bytes at `src`; the 64 pieces land side by side in LDS
// from `lds_base` (wave-uniform) on, in lane order.  Completion is counted by vmcnt.
__device__ __forceinline__ void load16_to_lds(const void* src, void* lds_base)
{
    __builtin_amdgcn_global_load_lds(src, lds_base, 16, 0, 0);
}

// Sixteen zero bytes: what a piece outside the grid is loaded from under zero padding.
static __device__ __align__(16) const unsigned kZeroPiece[4] = {0u, 0u, 0u, 0u};

// What one thread of a block fetches of every staged plane.  The staged tile is ROWS rows of RS = 64 + 2*HC
// 16-byte pieces (HC halo pieces on either side of the strip's 64), split evenly over the block's NTHR threads:
// piece f = i*NTHR + tid of the tile is row f / RS, piece f % RS of that row, so a wave's 64 loads of one
// round are 64 consecutive pieces.  The pieces are the same for every plane: offsets are computed once.
template <typename T, int ROWS, int HC, int NTHR>
struct PlaneFetch {
    static constexpr int V = 16 / (int)sizeof(T);
    static constexpr int RS = kWave + 2 * HC;
    static constexpr int TOTAL = ROWS * RS;
    static constexpr int NCH = (TOTAL + NTHR - 1) / NTHR;   // pieces one thread fetches per plane
    static constexpr int SLOTS = NCH * NTHR;                // LDS pieces per buffer (the last few are padding)
    unsigned off[NCH];   // byte offset of the piece inside a plane, row and column clamped into the grid (32 bits:
                         // the launcher sends larger planes to another kernel)
    unsigned inb;        // bit i: piece i exists and lies inside the grid in x and y

    // x0: first column of the strip; y_first: grid row of the tile's first row
    __device__ __forceinline__ void plan(int tid, int x0, int y_first, int W, int H, size_t rowst)
    {
        inb = 0;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int f = i * NTHR + tid;
            const int row = f / RS, c = f - row * RS;
            const int y = y_first + row, x = x0 + (c - HC) * V;
            const int yy = min(max(y, 0), H - 1), xx = min(max(x, 0), W - V);
            off[i] = (unsigned)(((size_t)yy * rowst + xx) * sizeof(T));
            inb |= (f < TOTAL && y >= 0 && y < H && x >= 0 && x < W) ? 1u << i : 0u;
        }
    }

    // Requests plane z of `in` into `buf` (SLOTS pieces of LDS), straight from global memory.  Zero padding:
    // pieces and planes outside the grid come from kZeroPiece, so every lane issues every load and the request
    // counts agree in all waves.  Clamp: every offset is already clamped into the grid, and so is z.
    // inside_xy (block-uniform): every piece of the tile lies inside the grid in x and y.
    template <class Vec>
    __device__ __forceinline__ void request(const T* in, size_t plane, int z, int D, bool clamp, bool inside_xy, Vec* buf,
                                            int wave) const
    {
        const char* zero_src = reinterpret_cast<const char*>(kZeroPiece);
        const bool plane_in = clamp || (z >= 0 && z < D);                     // block-uniform
        const char* pz = plane_in ? reinterpret_cast<const char*>(in + (size_t)min(max(z, 0), D - 1) * plane) : zero_src;
        const unsigned keep = plane_in ? ~0u : 0u;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const char* src = pz + (off[i] & keep);
            if (!clamp && (!inside_xy || (i + 1) * NTHR > TOTAL)) src = (inb >> i) & 1u ? src : zero_src;
            load16_to_lds(src, &buf[i * NTHR + wave * kWave]);
        }
    }
};

// Requests of a wave that are younger than the loads of the plane used at step t, which were issued at the
// start of step t - PF: the stores of steps t-PF .. t-1 (P per step from step `first_store` on, for a wave
// that stores all its rows) and the loads of planes t+1 .. t+PF-1 (NCH each).  Requests complete in order, so
// waiting until at most this many are outstanding means plane t has landed.
template <int PF, int NCH, int P>
__device__ __forceinline__ int younger_requests(int t, int nt, bool full_rows, int first_store)
{
    int younger = 0;
#pragma unroll
    for (int k = 1; k <= PF; ++k) {
        if (k < PF && t + k < nt) younger += NCH;
        if (full_rows && t - k >= first_store) younger += P;
    }
    return younger;
}

template <typename T, int P, int NW, int R, int BUDGET, int NBUF, int NT>
__global__ __launch_bounds__(NW* kWave) __attribute__((amdgpu_waves_per_eu(2))) void ssam3d_star_kernel(
    const Args3D<T, SliceMask<R, R, R, BUDGET, 0>::kNW> a)
{
    static_assert(NBUF == 3 || NBUF == 4, "a ring of three or four staged planes");
    constexpr int PF = NBUF - 1;               // planes requested ahead
    constexpr int V = Piece16<T>::V;
    typedef typename Piece16<T>::type vec_t;
    constexpr int NZ = 2 * R + 1;
    constexpr int HC = (R + V - 1) / V;        // halo pieces on each side of a staged row
    constexpr int C = P + 2 * R;               // rows one wave evaluates from
    constexpr int NTHR = NW * kWave;
    typedef PlaneFetch<T, NW * P + 2 * R, HC, NTHR> Fetch;   // the block stages NW*P + 2R rows per plane
    constexpr int RS = Fetch::RS, NCH = Fetch::NCH, SLOTS = Fetch::SLOTS;
    constexpr bool NT_STORE = (NT & kStreamStores) != 0;
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
    const int x0 = strip * (kWave * V);        // first column of the strip
    const int xc = x0 + lane * V;              // first column this lane owns
    const int yb0 = yblock * (NW * P);         // first output row of the block
    const int y0 = yb0 + wave * P;             // first output row of this wave
    const int z0 = ztile * a.planes_per_wave;
    const int z1 = min(z0 + a.planes_per_wave, D);
    const bool clamp = a.boundary == kClamp;
    const T* __restrict__ in = a.in;
    typedef Args3D<T, SliceMask<R, R, R, BUDGET, 0>::kNW> Args;
    const ConstPtr<T> wts = kernarg_member<T>(offsetof(Args, w));   // star: z line (centre at R), y line, x line; else dense [dz][dx][dy]
    const size_t rowst = (size_t)a.stride_row, plane = (size_t)a.stride_plane;
    const int nt = (z1 - z0) + 2 * R;          // input planes z0-R .. z1-1+R

    // block-uniform: every staged piece lies inside the grid in x and y
    const bool inside_xy = x0 - HC * V >= 0 && x0 + (kWave + HC) * V <= W && yb0 - R >= 0 && yb0 + NW * P + R <= H;

    Fetch fetch;
    fetch.plan(tid, x0, yb0 - R, W, H, rowst);

    T acc[NZ][P][V];
#pragma unroll
    for (int s = 0; s < NZ; ++s)
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int j = 0; j < V; ++j) acc[s][p][j] = T(0);

    const bool lane_stores = xc < W;
    const int own = (wave * P) * RS + HC + lane;     // this lane's piece of the wave's first staged row
    const int edge_l = (wave * P) * RS;              // the row's first piece; HC pieces of left halo
    const int edge_r = (wave * P) * RS + HC + kWave; // HC pieces of right halo

    // Clamp rule at the left / right edge of the grid (block-uniform): the halo pieces, and the pieces of lanes
    // beyond the last column, are the row's edge column repeated.
    const bool clamp_l = clamp && x0 == 0;                  // the left halo pieces lie outside the grid
    const bool clamp_r = clamp && x0 + kWave * V > W;       // so do the pieces of the lanes from column W on
    // right halo pieces 1 .. right_in lie inside the grid, the others outside
    const int right_in = clamp ? min(max((W - x0 - kWave * V) / V, 0), HC) : HC;
    const int last_piece = (wave * P) * RS + HC + (W - x0) / V - 1;   // the piece that ends in column W-1 (when one of the above is outside)
    const bool beyond = xc >= W;
    // row `k` of the wave's window in staged plane `st`: the lane's own piece, and halo piece h (1 = nearest).
    // EX (compile time): the block lies at the left or right edge of the grid under the clamp rule; every other
    // block reads the staged pieces as they are and pays nothing for the rule.
    // The selections below are by value (address and element selects), never by a branch: a branch per piece would
    // cut the unrolled step into short basic blocks (7x7x7 box, fp32, 512^3, every block at an edge: 1.83 ms with
    // branches, 1.61 ms without, against 1.52 ms under zero padding).
    const bool beyond_r = clamp_r && beyond;
    // the lane whose piece ends in column W-1 (meaningful when clamp_r)
    const int last_lane = __builtin_amdgcn_readfirstlane(min(max((W - x0) / V - 1, 0), kWave - 1));
    // Each selection is a read (possibly from a selected address) and a fix of the value read, so that a step can
    // request all its pieces first and fix them afterwards.
    auto read_own = [&](const vec_t* st, int k) __attribute__((always_inline)) { return st[own + k * RS]; };
    auto fix_own = [&](auto ex, vec_t v) __attribute__((always_inline)) {
        if constexpr (decltype(ex)::value) {
            // lanes beyond the grid repeat column W-1, which the lane last_lane has just read: a lane broadcast,
            // no second LDS read
            const T e = read_lane((T)v[V - 1], last_lane);
#pragma unroll
            for (int j = 0; j < V; ++j) v[j] = beyond_r ? e : v[j];
        }
        return v;
    };
    auto read_left = [&](auto ex, const vec_t* st, int k, int h) __attribute__((always_inline)) {
        // under the rule the row's first column repeated: its piece is the first after the halo.  Without it the
        // halo piece itself (the same address in every lane: a broadcast)
        if constexpr (decltype(ex)::value) return st[edge_l + k * RS + (clamp_l ? HC : HC - h)];
        else return st[edge_l + k * RS + (HC - h)];
    };
    auto fix_left = [&](auto ex, vec_t v) __attribute__((always_inline)) {
        if constexpr (decltype(ex)::value) {
#pragma unroll
            for (int j = 1; j < V; ++j) v[j] = clamp_l ? v[0] : v[j];
        }
        return v;
    };
    auto read_right = [&](auto ex, const vec_t* st, int k, int h) __attribute__((always_inline)) {
        if constexpr (decltype(ex)::value) return st[(h > right_in ? last_piece : edge_r + (h - 1)) + k * RS];
        else return st[edge_r + k * RS + (h - 1)];
    };
    auto fix_right = [&](auto ex, vec_t v, int h) __attribute__((always_inline)) {
        if constexpr (decltype(ex)::value) {
            const bool outside = h > right_in;       // block-uniform
#pragma unroll
            for (int j = 0; j < V - 1; ++j) v[j] = outside ? v[V - 1] : v[j];
        }
        return v;
    };
    auto own_piece = [&](auto ex, const vec_t* st, int k) __attribute__((always_inline)) { return fix_own(ex, read_own(st, k)); };
    auto left_piece = [&](auto ex, const vec_t* st, int k, int h) __attribute__((always_inline)) {
        return fix_left(ex, read_left(ex, st, k, h));
    };
    auto right_piece = [&](auto ex, const vec_t* st, int k, int h) __attribute__((always_inline)) {
        return fix_right(ex, read_right(ex, st, k, h), h);
    };

    // one step of the march: the staged plane `st` is input plane zin
    auto step = [&](auto ex, const vec_t* st, int zin) __attribute__((always_inline)) {
        if constexpr (BUDGET == 1) {
            T sum[P][V];       // in-plane sums, seeded with the plane above's partial sums
            // every piece the step reads is requested before anything is computed from it: one wait for all of them
            vec_t rowv[C], hl[P][HC], hr[P][HC];
#pragma unroll
            for (int k = 0; k < C; ++k) rowv[k] = read_own(st, k);
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int h = 1; h <= HC; ++h) {
                    hl[p][h - 1] = read_left(ex, st, p + R, h);
                    hr[p][h - 1] = read_right(ex, st, p + R, h);
                }
            if constexpr (decltype(ex)::value) {
                __builtin_amdgcn_sched_barrier(0);
                // one block-uniform branch per step: this kernel has few instructions per step to hide the fixes
                // behind (radius 4, 512^3: 15 % when every edge block made them, needed or not)
                if (clamp_r) {
#pragma unroll
                    for (int k = 0; k < C; ++k) rowv[k] = fix_own(ex, rowv[k]);
                }
            }
            // -- per window: z taps and the centre tap (in-flight plane s takes dz = R - s from this
            //    input plane), then the x taps: neighbouring columns of the centre row, shifted in
            //    from the lanes beside (the columns beyond the wave's own come in as the edge lanes'
            //    "old" values)
#pragma unroll
            for (int p = 0; p < P; ++p) {
                T xs[(2 * HC + 1) * V];     // columns -HC*V .. (HC+1)*V - 1 relative to the lane's first
                const vec_t v = rowv[p + R];
#pragma unroll
                for (int j = 0; j < V; ++j) xs[HC * V + j] = v[j];
                const T* cen = &xs[HC * V];
#pragma unroll
                for (int s = 0; s < R; ++s)
#pragma unroll
                    for (int j = 0; j < V; ++j) acc[s][p][j] = fma_into(cen[j], wts[2 * R - s], acc[s + 1][p][j]);
#pragma unroll
                for (int j = 0; j < V; ++j) sum[p][j] = fma_into(cen[j], wts[R], acc[R + 1][p][j]);
#pragma unroll
                for (int s = R + 1; s < NZ - 1; ++s)
#pragma unroll
                    for (int j = 0; j < V; ++j) acc[s][p][j] = fma_into(cen[j], wts[2 * R - s], acc[s + 1][p][j]);
#pragma unroll
                for (int j = 0; j < V; ++j) acc[NZ - 1][p][j] = cen[j] * wts[0];
#pragma unroll
                for (int h = 1; h <= HC; ++h) {
                    const vec_t el = fix_left(ex, hl[p][h - 1]);
                    const vec_t er = fix_right(ex, hr[p][h - 1], h);
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        xs[(HC - h) * V + j] = shift_in_up(xs[(HC - h + 1) * V + j], (T)el[j]);
                        xs[(HC + h) * V + j] = shift_in_down(xs[(HC + h - 1) * V + j], (T)er[j]);
                    }
                }
#pragma unroll
                for (int dx = -R; dx <= R; ++dx) {
                    if (dx == 0) continue;
                    const T wx = wts[2 * NZ + dx + R];
#pragma unroll
                    for (int j = 0; j < V; ++j) sum[p][j] = fma_t(xs[HC * V + j + dx], wx, sum[p][j]);
                }
            }
            // -- y taps: every staged row of the wave's window
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const vec_t v = rowv[k];
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const int dy = k - R - p;
                    if (dy != 0 && dy >= -R && dy <= R) {
                        const T wy = wts[NZ + dy + R];
#pragma unroll
                        for (int j = 0; j < V; ++j) sum[p][j] = fma_t((T)v[j], wy, sum[p][j]);
                    }
                }
            }
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int j = 0; j < V; ++j) acc[R][p][j] = sum[p][j];
        } else {
            // Any tap shape (BUDGET 2: faces and edges, 3: the dense box): row by row, every staged row
            // of the window extended by the neighbouring columns it needs, shifted in from the lanes
            // beside; row k holds the taps dy = k - R - p of window p, for every in-flight plane s
            // (dz = R - s).  The first product a sum receives starts it from the partial sum of the
            // plane above (slot s + 1), so the planes advance one slot per step as in the star.
            T nacc[NZ][P][V];
            bool have[NZ][P];
#pragma unroll
            for (int s = 0; s < NZ; ++s)
#pragma unroll
                for (int p = 0; p < P; ++p) have[s][p] = false;
#pragma unroll
            for (int k = 0; k < C; ++k) {
                T xs[(2 * HC + 1) * V];
                const vec_t v = own_piece(ex, st, k);
#pragma unroll
                for (int j = 0; j < V; ++j) xs[HC * V + j] = v[j];
#pragma unroll
                for (int h = 1; h <= HC; ++h) {
                    const vec_t el = left_piece(ex, st, k, h);
                    const vec_t er = right_piece(ex, st, k, h);
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        xs[(HC - h) * V + j] = shift_in_up(xs[(HC - h + 1) * V + j], (T)el[j]);
                        xs[(HC + h) * V + j] = shift_in_down(xs[(HC + h - 1) * V + j], (T)er[j]);
                    }
                }
                static_for<NZ>([&](auto sc) __attribute__((always_inline)) {
                    constexpr int sl = decltype(sc)::value;
                    typedef SliceMask<R, R, R, BUDGET, R - sl> Mask;
#pragma unroll
                    for (int p = 0; p < P; ++p) {
                        const int n = k - p;                 // dy + R
                        if (n < 0 || n > 2 * R) continue;
#pragma unroll
                        for (int m = 0; m < 2 * R + 1; ++m) {
                            if (!Mask::tap(n, m)) continue;
                            const T w = wts[Mask::widx(n, m)];
#pragma unroll
                            for (int j = 0; j < V; ++j) {
                                const T x = xs[HC * V + j + m - R];
                                if (have[sl][p]) nacc[sl][p][j] = fma_t(x, w, nacc[sl][p][j]);
                                else if (sl < NZ - 1) nacc[sl][p][j] = fma_into(x, w, acc[sl < NZ - 1 ? sl + 1 : sl][p][j]);
                                else nacc[sl][p][j] = x * w;
                            }
                            have[sl][p] = true;
                        }
                    }
                });
            }
#pragma unroll
            for (int s = 0; s < NZ; ++s)
#pragma unroll
                for (int p = 0; p < P; ++p)
#pragma unroll
                    for (int j = 0; j < V; ++j)
                        acc[s][p][j] = have[s][p] ? nacc[s][p][j] : (s < NZ - 1 ? acc[s < NZ - 1 ? s + 1 : s][p][j] : T(0));
        }

        // output plane zin - R has now received its last contribution
        const int zo = zin - R;
        if (zo >= z0 && lane_stores) {
            T* po = a.out + (size_t)zo * plane + (size_t)y0 * rowst + xc;
#pragma unroll
            for (int p = 0; p < P; ++p)
                if (y0 + p < H) store_vec<T, V, NT_STORE>(po + (size_t)p * rowst, acc[0][p]);
        }
    };

    // ---- planes straight into LDS, PF steps ahead --------------------------------------------
    auto request = [&](int z, int b) __attribute__((always_inline)) { fetch.request(in, plane, z, D, clamp, inside_xy, stage[b], wave); };
    // a wave that stores all P rows issues P stores per step once output planes complete (step 2R on)
    const bool full_rows = y0 + P <= H;
#pragma unroll
    for (int k = 0; k < PF; ++k)
        if (k < nt) request(z0 - R + k, k);
    auto march = [&](auto ex) __attribute__((always_inline)) {
        int b = 0;
        for (int t = 0; t < nt; ++t) {
            // Away from both ends of the chunk the count is one of two constants; naming them spares every step the
            // chain of compares and branches that picks the wait's immediate.
            constexpr int kSteadyLoads = (PF - 1) * NCH, kSteadyAll = kSteadyLoads + PF * P;
            if (t >= 2 * R + PF && t + PF <= nt) {
                if (full_rows) wait_and_sync_n<(kSteadyAll & ~1)>();
                else wait_and_sync_n<(kSteadyLoads & ~1)>();
            } else {
                wait_and_sync(younger_requests<PF, NCH, P>(t, nt, full_rows, 2 * R));
            }
            // buffer (t + PF) % NBUF held plane t - 1, which every wave has finished reading
            if (t + PF < nt) request(z0 - R + t + PF, b + PF >= NBUF ? b + PF - NBUF : b + PF);
            asm volatile("" ::: "memory");   // the step's stores stay behind its requests: the count above relies on it
            step(ex, stage[b], z0 - R + t);
            b = b + 1 == NBUF ? 0 : b + 1;
        }
    };
    if (clamp_l || clamp_r || right_in < HC) march(std::true_type{});   // block-uniform
    else march(std::false_type{});
}

// All blocks of these kernels march through their z-chunks in step, so at any moment the device reads one plane and
// writes one plane per chunk.  When the chunks start a multiple of 128 MiB apart, those planes fall on the same
// DRAM banks in every chunk, and for many distances between the input and the output buffer the reads then collide
// with the writes (512^3 fp64: 360 us at the good distances, 395-415 us in bands that cover half of all
// distances; mean over distances 385 us).  Chunks four planes longer (the last one shorter) spread them: mean
// 370 us, worst 395.  (fp32 grids of this size, with chunks 64 MiB apart, show no such effect.)
inline int staggered_planes(int planes, int depth, size_t plane_bytes)
{
    if (planes >= depth || (planes * plane_bytes) % (128u << 20) != 0) return planes;
    const int longer = planes + 4;
    return ceil_div(depth, longer) == ceil_div(depth, planes) ? longer : planes;
}

// Fallback of a shape that has no other compiled instance: the dispatcher then takes the direct kernel.
inline hipError_t launch3d_unavailable(const Problem3D&, const Tuning&, Geometry*, bool) { return hipErrorNotSupported; }

// FALLBACK: the launcher of the instance that takes what this kernel does not (rows that are not a
// multiple of 16 bytes, unaligned base pointers, planes beyond 4 GiB).
template <typename T, int P, int NW, int R, int BUDGET, int NBUF, int NT, Launch3DFn FALLBACK>
hipError_t launch3d_star(const Problem3D& pr, const Tuning& tu, Geometry* geo, bool dry_run)
{
    constexpr int V = Piece16<T>::V;
    const size_t slice = (size_t)(pr.march_y ? pr.D : pr.H) * (pr.march_y ? (size_t)pr.W * pr.H : (size_t)pr.W) * sizeof(T);
    if (pr.W % V != 0 || slice > 0xffffffffull || (!dry_run && !pointers_aligned(pr.in, pr.out, 16)))
        return FALLBACK(pr, tu, geo, dry_run);
    Geometry g;
    g.V = V;
    g.P = P;
    g.halo_left = g.halo_right = 0;
    g.valid_lanes = kWave;
    g.strips_x = ceil_div(pr.W, kWave * V);
    g.rows_per_wave = P;
    const int LH = pr.march_y ? pr.D : pr.H, LD = pr.march_y ? pr.H : pr.D;   // strip / march extents
    g.tiles_y = ceil_div(LH, NW * P);
    int planes = tu.planes_per_wave;
    if (planes <= 0) {
        // The longest z-chunks that still give every compute unit its share of blocks: each chunk
        // re-reads 2R planes, and one round of equally long blocks finishes together (512^3, radius 4:
        // fp32 202 -> 195 us from 64 to 128 planes, fp64 406 -> 364 us from 64 to 256).
        int blocks_per_cu = 0, dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &blocks_per_cu, reinterpret_cast<const void*>(&ssam3d_star_kernel<T, P, NW, R, BUDGET, NBUF, NT>), NW * kWave,
                0) != hipSuccess || blocks_per_cu <= 0) {
            (void)hipGetLastError();
            cus = 256;
            blocks_per_cu = 1;
        }
        planes = balanced_planes(LD, (long)g.strips_x * g.tiles_y, cus * blocks_per_cu, LD, 4 * R);
        if (!pr.march_y) planes = staggered_planes(planes, LD, slice);
    }
    if (planes > LD) planes = LD;
    g.planes_per_wave = planes;
    g.tiles_z = ceil_div(LD, planes);
    g.tiles = (long)g.strips_x * g.tiles_y * g.tiles_z;   // block tiles
    g.xcd_remap = tu.xcd_remap < 0 ? 1 : (tu.xcd_remap ? 1 : 0);
    g.blocks = g.tiles > kMaxBlocks ? -1 : (g.xcd_remap ? ceil_div((int)g.tiles, kXcds) * kXcds : (int)g.tiles);
    if (geo) *geo = g;
    if (!launchable(g)) return hipErrorInvalidConfiguration;
    if (dry_run) return hipSuccess;

    Args3D<T, SliceMask<R, R, R, BUDGET, 0>::kNW> a;
    fill_args3d<T, V, R, R, R, BUDGET>(pr, g, &a);
    hipLaunchKernelGGL((ssam3d_star_kernel<T, P, NW, R, BUDGET, NBUF, NT>), dim3(g.blocks), dim3(NW * kWave), 0, pr.stream, a);
    return hipGetLastError();
}

// FALLBACK is written as the launcher's template-id, e.g. (::ssam::launch3d_lds<float, 2, 4, 4, 4, 4, 4, 1, 2>).
#define SSAM_INSTANCE_3D_RING(T, DT, P, NW, R, BUDGET, NBUF, NT, FALLBACK, VARIANT)                     \
    static ::ssam::Register3D SSAM_CAT(reg3ds_, __COUNTER__)(::ssam::Instance3D{                       \
        #T "_r" #R #R #R "_b" #BUDGET "_p" #P "w" #NW "star_ring" #NBUF "nt" #NT, DT, R, R, R, BUDGET,  \
        VARIANT, &::ssam::launch3d_star<T, P, NW, R, BUDGET, NBUF, NT, FALLBACK>})
#define SSAM_INSTANCE_3D_STAR(T, DT, P, NW, R, NBUF, NT, FALLBACK, VARIANT)                             \
    SSAM_INSTANCE_3D_RING(T, DT, P, NW, R, 1, NBUF, NT, FALLBACK, VARIANT)

}  // namespace ssam
