// Device-side building blocks shared by the 2D and 3D kernels (gfx950, wave64).
//
// The paper's execution model (Sec. 3.3): (i) a register cache per lane, (ii) partial sums
// handed to the neighbouring lane, (iii) all lanes accumulating in parallel.  On CDNA4 the
// hand-over is a DPP whole-wave shift by one lane (no LDS traffic, no bpermute), and one
// lane owns V adjacent columns, loaded as one 16-byte vector, so that one shift moves the
// partial sums of V outputs and only ceil(reach/V) shifts are needed per filter side
// (Sec. 5.4: keep horizontal transfers few).
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <type_traits>
#include <utility>

namespace ssam {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kXcds = 8;

enum : int { kZero = 0, kClamp = 1 };

// ---- whole-wave shift by one lane ------------------------------------------------------
// shift_up:   lane L receives the value lane L-1 held (lane 0 receives 0).
// shift_down: lane L receives the value lane L+1 held (lane 63 receives 0).
// DPP control 0x138 = wave_shr:1, 0x130 = wave_shl:1 (GFX9 encoding).  bound_ctrl makes the
// lane without a source read 0, so no "old" value has to be materialised first.
#if defined(SSAM_SHIFT_BPERMUTE)
// Comparison build only: the same shift through the LDS crossbar (what a recompiled
// __shfl_up / __shfl_down does).  The values read by lanes 0 / 63 are never used.
__device__ __forceinline__ int dpp_up(int v) { return __builtin_amdgcn_ds_bpermute(((int)(threadIdx.x & 63) - 1) << 2, v); }
__device__ __forceinline__ int dpp_down(int v) { return __builtin_amdgcn_ds_bpermute(((int)(threadIdx.x & 63) + 1) << 2, v); }
#else
__device__ __forceinline__ int dpp_up(int v) { return __builtin_amdgcn_mov_dpp(v, 0x138, 0xf, 0xf, true); }
__device__ __forceinline__ int dpp_down(int v) { return __builtin_amdgcn_mov_dpp(v, 0x130, 0xf, 0xf, true); }
#endif

__device__ __forceinline__ float shift_up(float v) { return __builtin_bit_cast(float, dpp_up(__builtin_bit_cast(int, v))); }
__device__ __forceinline__ float shift_down(float v) { return __builtin_bit_cast(float, dpp_down(__builtin_bit_cast(int, v))); }

struct Halves { int lo, hi; };
__device__ __forceinline__ double shift_up(double v)
{
    Halves h = __builtin_bit_cast(Halves, v);
    h.lo = dpp_up(h.lo);
    h.hi = dpp_up(h.hi);
    return __builtin_bit_cast(double, h);
}
__device__ __forceinline__ double shift_down(double v)
{
    Halves h = __builtin_bit_cast(Halves, v);
    h.lo = dpp_down(h.lo);
    h.hi = dpp_down(h.hi);
    return __builtin_bit_cast(double, h);
}

__device__ __forceinline__ float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }

// x * c + addend written as a three-address FMA (c wave-uniform, in scalar registers).  The
// compiler prefers the two-address form, which overwrites the addend's register; when the
// result has to live in a *different* register than the addend (the in-flight planes of the 3D
// march advance one slot per step) that costs a move per value, which this form avoids.
__device__ __forceinline__ float fma_into(float x, float c, float addend)
{
    float d;
    asm("v_fma_f32 %0, %1, %2, %3" : "=v"(d) : "s"(c), "v"(x), "v"(addend));
    return d;
}
__device__ __forceinline__ double fma_into(double x, double c, double addend)
{
    double d;
    asm("v_fma_f64 %0, %1, %2, %3" : "=v"(d) : "s"(c), "v"(x), "v"(addend));
    return d;
}

// ---- coefficients -------------------------------------------------------------------------
// Coefficients live in the kernel-argument block and are read through a constant-address-space
// pointer with wave-uniform indices, i.e. by scalar loads into SGPRs: one fetch serves all 64
// lanes and the multiply-add takes the SGPR as an operand.  This is the CDNA counterpart of
// the paper's conflict-free broadcast read from shared memory (Sec. 4.6).
template <typename T>
using ConstPtr = const T __attribute__((address_space(4)))*;

// Pointer to a member of the kernel's (single, by-value) argument struct at byte offset `off`.
template <typename T>
__device__ __forceinline__ ConstPtr<T> kernarg_member(size_t off)
{
    typedef const char __attribute__((address_space(4)))* Bytes;
    return (ConstPtr<T>)((Bytes)__builtin_amdgcn_kernarg_segment_ptr() + off);
}

// ---- V-wide vector access --------------------------------------------------------------
template <typename T, int V> struct VecOf;
template <> struct VecOf<float, 4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<float, 2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<float, 1> { typedef float type; };
template <> struct VecOf<double, 2> { typedef double type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<double, 1> { typedef double type; };

// STREAM selects the non-temporal (streaming) cache policy at compile time: the grid is far
// larger than the caches and every output is written once and never read back by the same
// sweep.  (A run-time choice between the two forms is folded into the plain one by the
// compiler, which drops the hint.)
constexpr int kStreamLoads = 1, kStreamStores = 2;

template <typename T, int V, bool STREAM>
__device__ __forceinline__ void load_vec(const T* __restrict__ p, T (&dst)[V])
{
    typedef typename VecOf<T, V>::type vec_t;
    const vec_t* vp = reinterpret_cast<const vec_t*>(p);
    vec_t v;
    if constexpr (STREAM) v = __builtin_nontemporal_load(vp);
    else v = *vp;
    if constexpr (V == 1) {
        dst[0] = v;
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) dst[i] = v[i];
    }
}

template <typename T, int V, bool STREAM>
__device__ __forceinline__ void store_vec(T* __restrict__ p, const T (&src)[V])
{
    typedef typename VecOf<T, V>::type vec_t;
    vec_t v;
    if constexpr (V == 1) {
        v = src[0];
    } else {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = src[i];
    }
    if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<vec_t*>(p));
    else *reinterpret_cast<vec_t*>(p) = v;
}

// ---- branch-free boundary fix-ups --------------------------------------------------------
// keep_if(v, m): v where the 32-bit mask m is all ones, +0 where it is zero.
// pick(a, b, m): b where m is all ones, a where it is zero (v_bfi_b32).
// Written on the bit patterns so the compiler cannot turn them into divergent branches
// around the loads they follow (which would serialise the loads of a tile's rows).
__device__ __forceinline__ float keep_if(float v, unsigned m) { return __builtin_bit_cast(float, __builtin_bit_cast(unsigned, v) & m); }
__device__ __forceinline__ double keep_if(double v, unsigned m)
{
    Halves h = __builtin_bit_cast(Halves, v);
    h.lo &= (int)m;
    h.hi &= (int)m;
    return __builtin_bit_cast(double, h);
}
__device__ __forceinline__ unsigned pick_bits(unsigned a, unsigned b, unsigned m) { return (b & m) | (a & ~m); }
__device__ __forceinline__ float pick(float a, float b, unsigned m)
{
    return __builtin_bit_cast(float, pick_bits(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), m));
}
__device__ __forceinline__ double pick(double a, double b, unsigned m)
{
    Halves x = __builtin_bit_cast(Halves, a), y = __builtin_bit_cast(Halves, b);
    x.lo = (int)pick_bits((unsigned)x.lo, (unsigned)y.lo, m);
    x.hi = (int)pick_bits((unsigned)x.hi, (unsigned)y.hi, m);
    return __builtin_bit_cast(double, x);
}

// Value of lane `l` (wave-uniform) broadcast to the whole wave.
__device__ __forceinline__ float read_lane(float v, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ double read_lane(double v, int l)
{
    Halves h = __builtin_bit_cast(Halves, v);
    h.lo = __builtin_amdgcn_readlane(h.lo, l);
    h.hi = __builtin_amdgcn_readlane(h.hi, l);
    return __builtin_bit_cast(double, h);
}

// ---- tap masks ------------------------------------------------------------------------
// Coefficients are run-time data; only the *shape* is compiled in, as in the paper's
// one-instance-per-(M,N) template.  A mask describes one filter slice of width M (x) and
// height N (y) anchored at (AX, AY): which (n, m) are taps, how far they reach sideways,
// and where each tap's coefficient sits in the packed array the kernel receives.
//
// BUDGET is how many offset components may be non-zero at once: for a 2D slice 2 = dense
// box, 1 = star (taps on the axes only), 0 = the anchor alone.
template <int M, int N, int AX, int AY, int BUDGET>
struct TapMask {
    static constexpr int kM = M, kN = N, kAX = AX, kAY = AY;
    static __host__ __device__ constexpr bool tap(int n, int m) { return (n != AY ? 1 : 0) + (m != AX ? 1 : 0) <= BUDGET; }
    static constexpr int kLeft = BUDGET >= 1 ? AX : 0;            // farthest tap left of the anchor
    static constexpr int kRight = BUDGET >= 1 ? M - 1 - AX : 0;   // farthest tap right of the anchor
    // packed coefficients: a box is stored column by column ([m][n]) so that the N values one
    // filter column needs are adjacent and arrive in one wide scalar load; a star stores its N
    // column values, then its M row values
    static constexpr int kNW = BUDGET >= 2 ? M * N : (BUDGET == 1 ? M + N : 1);
    static __host__ __device__ constexpr int widx(int n, int m)
    {
        return BUDGET >= 2 ? m * N + n : (BUDGET == 1 ? (n != AY ? n : N + m) : 0);
    }
};

// Slice dz of a 3D stencil of radii (RX, RY, RZ); BUDGET = 1 star, 2 faces+edges, 3 dense box.
template <int RX, int RY, int RZ, int BUDGET, int DZ>
struct SliceMask {
    static constexpr int kM = 2 * RX + 1, kN = 2 * RY + 1, kAX = RX, kAY = RY;
    static constexpr int kUsed = DZ != 0 ? 1 : 0;
    static __host__ __device__ constexpr bool tap(int n, int m) { return kUsed + (n != RY ? 1 : 0) + (m != RX ? 1 : 0) <= BUDGET; }
    static constexpr int kLeft = BUDGET - kUsed >= 1 ? RX : 0;
    static constexpr int kRight = kLeft;
    // packed coefficients: dense [dz][dx][dy] (columns adjacent, as in 2D) unless star, which stores
    // the z line, the y line, the x line
    static constexpr int kNW = BUDGET == 1 ? (2 * RZ + 1) + (2 * RY + 1) + (2 * RX + 1)
                                           : (2 * RZ + 1) * (2 * RY + 1) * (2 * RX + 1);
    static __host__ __device__ constexpr int widx(int n, int m)
    {
        return BUDGET == 1 ? (DZ != 0 ? DZ + RZ
                                      : (n != RY ? (2 * RZ + 1) + n : (m != RX ? (2 * RZ + 1) + (2 * RY + 1) + m : RZ)))
                           : ((DZ + RZ) * kM + m) * kN + n;
    }
};

// Calls f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}) in order.
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// ---- the systolic row evaluation --------------------------------------------------------
// A wave-uniform zero the compiler cannot see through.  Added to a coefficient index it pins
// the scalar load of that coefficient to the place where it is used: without it the
// compiler hoists every coefficient of a large filter out of the row loop and spills the
// scalar registers it needs for them.
__device__ __forceinline__ int opaque_zero()
{
    int z;
    asm volatile("s_mov_b32 %0, 0" : "=s"(z));
    return z;
}

// Views of the register cache handed to the row evaluation.  Row and column indices are
// compile-time constants after unrolling, so at(k, i) names one register.
template <typename T, int V, int ROWS>
struct RowBlock {               // one array of ROWS cached rows
    static constexpr int kRows = ROWS;
    const T (&r)[ROWS][V];
    __device__ __forceinline__ T at(int k, int i) const { return r[k][i]; }
};
template <typename T, int V, int HEAD, int TAIL>
struct RowPair {                // HEAD rows kept from the previous window, then TAIL new rows
    static constexpr int kRows = HEAD + TAIL;
    const T (&head)[HEAD > 0 ? HEAD : 1][V];
    const T (&tail)[TAIL][V];
    __device__ __forceinline__ T at(int k, int i) const { return k < HEAD ? head[k < HEAD ? k : 0][i] : tail[k >= HEAD ? k - HEAD : 0][i]; }
};

// Products of one filter column, for all P window positions: the lane's own column i = j + COL
// multiplies filter column AX + DX and accumulates into the partial sum of output column j.
// (Sec. 4.3: an N-term inner product between a register vector and a filter column.)
// set[j] says whether the sums of output column j hold a value yet: the first product is a plain
// multiplication, so no sum is ever zero-initialised.  All indices are compile-time constants
// after unrolling, and so are the flags.
template <typename T, int V, int P, class Mask, int DX, int COL, bool PIN, bool SKIP_ANCHOR, class Rows>
__device__ __forceinline__ void column_products(const Rows& r, ConstPtr<T> w, T (&s)[P][V], bool (&set)[V])
{
    constexpr int N = Mask::kN, AX = Mask::kAX;
    const int z = PIN ? opaque_zero() : 0;
#pragma unroll
    for (int n = 0; n < N; ++n) {
        if (Mask::tap(n, AX + DX) && !(SKIP_ANCHOR && DX == 0 && n == Mask::kAY)) {
            const T wv = w[Mask::widx(n, AX + DX) + z];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const int i = j + COL;
                if (i >= 0 && i < V) {
                    if (set[j]) {
#pragma unroll
                        for (int p = 0; p < P; ++p) s[p][j] = fma_t(r.at(p + n, i), wv, s[p][j]);
                    } else {
#pragma unroll
                        for (int p = 0; p < P; ++p) s[p][j] = r.at(p + n, i) * wv;
                        set[j] = true;
                    }
                }
            }
        }
    }
}

// For P window positions p (the sliding window of Sec. 4.2) computes
//     out[p][j] = (ACCUMULATE ? in[p][j] : 0) + sum over taps (n, m) of
//                 w[widx(n, m)] * column(x_j + m - AX)[p + n]
// where lane L's register cache r.at(k, i) holds row k of its own column L*V + i, and x_j is
// the lane's own column j: the result lands in the lane that owns the output column, so
// loads and stores are both V-aligned.  `in` and `out` may be different arrays (the 3D march
// uses that to rotate its in-flight planes for free) or the same one.
//
// Dependency graph (the paper's D): two chains of partial sums converge on the owning lane.
// Taps left of the anchor are accumulated by the lanes to the left and travel up-lane
// (towards higher lane ids); taps right of the anchor travel down-lane.  At distance d from
// the owner a lane adds the products of its own columns that fall inside the filter
// footprint, then hands the V partial sums on (Sec. 4.4).  After ceil(kLeft/V) +
// ceil(kRight/V) shifts the owner adds the columns it holds itself.  A sum that has received no
// product yet is not shifted, and the first product of every sum is a plain multiplication: with V
// columns per lane only the outputs near the lane's edge depend on the neighbouring lane when the
// filter is narrow (Sec. 5.4: fewer horizontal transfers), so for a radius-1 stencil each chain
// carries one of the V sums and the two chains never meet.  Lanes nearer than
// ceil(kLeft/V) to the low end of the wave, or ceil(kRight/V) to the high end, end with
// incomplete sums: they are the overlapped-blocking halo (Sec. 4.5).
template <typename T, int V, int P, class Mask, bool ACCUMULATE, class Rows>
__device__ __forceinline__ void systolic_rows(const Rows& r, ConstPtr<T> w,
                                              const T (&in)[P][V], T (&out)[P][V])
{
    constexpr int N = Mask::kN;
    static_assert(Rows::kRows >= N + P - 1, "register cache too small for the sliding window");
    constexpr int DL = (Mask::kLeft + V - 1) / V;
    constexpr int DR = (Mask::kRight + V - 1) / V;
    constexpr bool PIN = Mask::kNW > 64;   // small coefficient sets stay resident in scalar registers

    T sum[P][V];
    bool have[V];   // per output column: does `sum` hold a value yet (folds to constants)
#pragma unroll
    for (int j = 0; j < V; ++j) have[j] = ACCUMULATE;
    if constexpr (ACCUMULATE) {
        // the anchor tap (every mask has it) seeds the sums from `in` with a three-address FMA
        const T wa = w[Mask::widx(Mask::kAY, Mask::kAX)];
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int j = 0; j < V; ++j) sum[p][j] = fma_into(r.at(p + Mask::kAY, j), wa, in[p][j]);
    }

    // chain arriving from the left (lower lane ids)
    if constexpr (DL > 0) {
        T s[P][V];
        bool got[V];
#pragma unroll
        for (int j = 0; j < V; ++j) got[j] = false;
        static_for<DL>([&](auto dc) __attribute__((always_inline)) {
            constexpr int d = DL - decltype(dc)::value;            // DL, DL-1, ..., 1
            // columns of this lane relative to an output column d lanes up: dx = i - j - d*V
            static_for<2 * V - 1>([&](auto cc) __attribute__((always_inline)) {
                constexpr int dx = decltype(cc)::value - (V - 1) - d * V;
                if constexpr (dx >= -Mask::kLeft && dx <= -1)
                    column_products<T, V, P, Mask, dx, dx + d * V, PIN, false, Rows>(r, w, s, got);
            });
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (got[j]) {
#pragma unroll
                    for (int p = 0; p < P; ++p) s[p][j] = shift_up(s[p][j]);
                }
        });
#pragma unroll
        for (int j = 0; j < V; ++j)
            if (got[j]) {
#pragma unroll
                for (int p = 0; p < P; ++p) sum[p][j] = have[j] ? sum[p][j] + s[p][j] : s[p][j];
                have[j] = true;
            }
    }
    // chain arriving from the right (higher lane ids)
    if constexpr (DR > 0) {
        T s[P][V];
        bool got[V];
#pragma unroll
        for (int j = 0; j < V; ++j) got[j] = false;
        static_for<DR>([&](auto dc) __attribute__((always_inline)) {
            constexpr int d = DR - decltype(dc)::value;
            static_for<2 * V - 1>([&](auto cc) __attribute__((always_inline)) {
                constexpr int dx = decltype(cc)::value - (V - 1) + d * V;
                if constexpr (dx >= 1 && dx <= Mask::kRight)
                    column_products<T, V, P, Mask, dx, dx - d * V, PIN, false, Rows>(r, w, s, got);
            });
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (got[j]) {
#pragma unroll
                    for (int p = 0; p < P; ++p) s[p][j] = shift_down(s[p][j]);
                }
        });
#pragma unroll
        for (int j = 0; j < V; ++j)
            if (got[j]) {
#pragma unroll
                for (int p = 0; p < P; ++p) sum[p][j] = have[j] ? sum[p][j] + s[p][j] : s[p][j];
                have[j] = true;
            }
    }
    // the owner's own columns: dx = i - j
    static_for<2 * V - 1>([&](auto cc) __attribute__((always_inline)) {
        constexpr int dx = decltype(cc)::value - (V - 1);
        if constexpr (dx >= -Mask::kLeft && dx <= Mask::kRight)
            column_products<T, V, P, Mask, dx, dx, PIN, ACCUMULATE, Rows>(r, w, sum, have);
    });
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int j = 0; j < V; ++j) out[p][j] = have[j] ? sum[p][j] : T(0);
}

// ---- the same evaluation on the matrix cores -------------------------------------------
// v_mfma_f32_4x4x1 (16 blocks of 4 lanes, K = 1) computes, in lane l and for i = 0..3,
//     d[i] = a(lane 4*(l/4) + i) * b(lane l) + c[i]
// i.e. every lane multiplies ITS OWN b by the four a values of its group of four lanes.  With
// b = the lane's cached row k of one of its columns, a = the filter-column value that row k
// contributes to window position i with (w[k - i][m], the same pattern in every group of four),
// and c/d = the four window sums of one output column, one instruction performs the four
// multiply-adds that row k owes to the P = 4 window positions -- the products of Sec. 4.3 at twice
// the rate of the vector unit (32 instead of 16 multiply-adds per SIMD and cycle, full fp32), while the
// vector unit is left with the lane shifts.  N + 3 instructions replace 4 N fused multiply-adds
// per filter column and output column; rows k that meet no tap of the column are skipped.
//
// The a operands come from a table in LDS, laid out for this: tab[(m * 4 + q) * CP + k] = w[k - q][m], 0
// outside the filter, CP = N + 3 rounded up to a multiple of four; each lane reads the entries q = lane % 4
// of four consecutive window rows k with one 16-byte read (four addresses per read, broadcast, no
// conflict).  The caller fills the table once per workgroup (fill_mfma_weights).
typedef float v4f __attribute__((ext_vector_type(4)));

template <class Mask>
struct MfmaWeights {
    static constexpr int kRows = Mask::kN + 3;              // rows of the window of four positions
    static constexpr int kPitch = (kRows + 3) / 4 * 4;      // words per (filter column, q): whole 16-byte pieces
    static constexpr int kWords = Mask::kM * 4 * kPitch;
};

// Workgroup-cooperative; the caller synchronises afterwards.
template <class Mask>
__device__ __forceinline__ void fill_mfma_weights(ConstPtr<float> w, float* tab)
{
    constexpr int N = Mask::kN, CP = MfmaWeights<Mask>::kPitch;
    for (int e = threadIdx.x; e < MfmaWeights<Mask>::kWords; e += blockDim.x) {
        const int k = e % CP, q = (e / CP) & 3, m = e / (4 * CP);
        const int n = k - q;
        tab[e] = (n >= 0 && n < N && Mask::tap(n, m)) ? w[Mask::widx(n, m)] : 0.0f;
    }
}

template <class Mask>
__host__ __device__ constexpr bool window_row_meets_column(int k, int m)
{
    for (int q = 0; q < 4; ++q)
        if (k - q >= 0 && k - q < Mask::kN && Mask::tap(k - q, m)) return true;
    return false;
}

// The order of work of one group of four window positions, as a compile-time list of jobs, one per filter
// column a lane meets at one lane-column distance COL from the output column (such a column feeds V - |COL|
// of the V sums).  The list follows the two converging chains of systolic_rows: the columns a lane meets d
// lanes left of the output lane, d = DL .. 1, each distance followed by a shift; the same from the right;
// then the owner's own columns.
struct MfmaJob {
    int m, col;          // filter column (0 .. M-1) and lane-column distance COL
    int chain;           // 0: sums arriving from the left, 1: from the right, 2: the output lane itself
    bool shift, merge;   // after the job: shift the chain's sums one lane on / add them to the lane's own
};

template <int V, class Mask>
struct MfmaPlan {
    static constexpr int kMaxJobs = 2 * Mask::kM;
    struct List {
        MfmaJob job[kMaxJobs];
        int n;
    };
    // the filter columns dx = COL + base, lo <= dx <= hi, a lane meets at one distance from the output lane
    static constexpr void add_group(List& l, int base, int lo, int hi, int chain)
    {
        for (int col = -(V - 1); col <= V - 1; ++col) {
            const int dx = col + base;
            if (dx >= lo && dx <= hi) l.job[l.n++] = MfmaJob{Mask::kAX + dx, col, chain, false, false};
        }
    }
    static constexpr List make()
    {
        List l{};
        constexpr int DL = (Mask::kLeft + V - 1) / V, DR = (Mask::kRight + V - 1) / V;
        for (int d = DL; d >= 1; --d) {
            add_group(l, -d * V, -Mask::kLeft, -1, 0);
            l.job[l.n - 1].shift = true;
        }
        if (DL > 0) l.job[l.n - 1].merge = true;
        for (int d = DR; d >= 1; --d) {
            add_group(l, d * V, 1, Mask::kRight, 1);
            l.job[l.n - 1].shift = true;
        }
        if (DR > 0) l.job[l.n - 1].merge = true;
        add_group(l, 0, -Mask::kLeft, Mask::kRight, 2);
        return l;
    }
    static constexpr List list = make();
};

// systolic_rows for fp32, P = 4, no incoming sums, with the products on the matrix cores: the same two
// converging chains and the same shifts.  tab_lane = table + (lane % 4) * pitch.  The a operands of a job
// are requested from LDS while the MFMAs of the job before it run (two sets of operand registers that
// alternate): waiting for them at every filter column otherwise costs 2-6 % of the launch.  Scheduling
// barriers keep that order: without them the compiler either requests the whole table ahead and spills, or
// puts every read next to its use and waits for each; the opaque zero in the table address keeps the reads
// of a job from being hoisted further.  (Evaluating the columns COL and COL + V, which feed complementary
// sums, interleaved -- so that no MFMA follows one it depends on -- measured the same as this order.)
template <int V, class Mask, class Rows>
__device__ __forceinline__ void systolic_rows_mfma(const Rows& r, const float* tab_lane, float (&out)[4][V])
{
    static_assert(Rows::kRows >= Mask::kN + 3, "register cache too small for the sliding window");
    typedef MfmaPlan<V, Mask> Plan;
    constexpr int C = MfmaWeights<Mask>::kRows, CP = MfmaWeights<Mask>::kPitch;
    constexpr int T = Plan::list.n;
    v4f sum[V], sl[V], sr[V];
    bool have[V], gl[V], gr[V];
#pragma unroll
    for (int j = 0; j < V; ++j) have[j] = gl[j] = gr[j] = false;
    float a[2][CP];
    typedef __attribute__((address_space(3))) const float lds_float;
    lds_float* col = (lds_float*)tab_lane;         // the table lives in LDS

    auto request = [&](auto tt) __attribute__((always_inline)) {
        constexpr int t = decltype(tt)::value;
        constexpr MfmaJob jb = Plan::list.job[t];
        // the table pointer passes through an empty asm statement: the compiler cannot see through it, so the reads
        // of this job stay here, and no instruction is spent (the same register carries on to the next job)
        asm volatile("" : "+v"(col));
#pragma unroll
        for (int k = 0; k < CP; k += 4) {
            const v4f piece = *reinterpret_cast<__attribute__((address_space(3))) const v4f*>(col + jb.m * 4 * CP + k);
#pragma unroll
            for (int e = 0; e < 4; ++e) a[t & 1][k + e] = piece[e];
        }
    };
    auto products = [&](auto tt, v4f (&s)[V], bool (&set)[V]) __attribute__((always_inline)) {
        constexpr int t = decltype(tt)::value;
        constexpr MfmaJob jb = Plan::list.job[t];
#pragma unroll
        for (int k = 0; k < C; ++k) {
            if (window_row_meets_column<Mask>(k, jb.m)) {
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    const int i = j + jb.col;
                    if (i >= 0 && i < V) {
                        const v4f c = set[j] ? s[j] : v4f{0.0f, 0.0f, 0.0f, 0.0f};
                        s[j] = __builtin_amdgcn_mfma_f32_4x4x1f32(a[t & 1][k], r.at(k, i), c, 0, 0, 0);
                        set[j] = true;
                    }
                }
            }
        }
    };

    request(std::integral_constant<int, 0>{});
    static_for<T>([&](auto tt) __attribute__((always_inline)) {
        constexpr int t = decltype(tt)::value;
        constexpr MfmaJob jb = Plan::list.job[t];
        if constexpr (t + 1 < T) request(std::integral_constant<int, t + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (jb.chain == 0) products(tt, sl, gl);
        else if constexpr (jb.chain == 1) products(tt, sr, gr);
        else products(tt, sum, have);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (jb.shift) {
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (jb.chain == 0 ? gl[j] : gr[j]) {
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        if constexpr (jb.chain == 0) sl[j][p] = shift_up(sl[j][p]);
                        else sr[j][p] = shift_down(sr[j][p]);
                    }
                }
        }
        if constexpr (jb.merge) {
#pragma unroll
            for (int j = 0; j < V; ++j)
                if (jb.chain == 0 ? gl[j] : gr[j]) {
                    const v4f s = jb.chain == 0 ? sl[j] : sr[j];
                    sum[j] = have[j] ? sum[j] + s : s;
                    have[j] = true;
                }
        }
    });
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int j = 0; j < V; ++j) out[p][j] = have[j] ? sum[j][p] : 0.0f;
}

// Map the hardware block id to a logical one so that consecutive logical blocks (which
// share halo rows and cache lines) run on the same XCD and hence behind the same L2:
// hardware deals block b to XCD b % 8.  nblocks_padded is a multiple of 8.
__device__ __forceinline__ int logical_block(int b, int nblocks_padded, int remap)
{
    if (!remap) return b;
    const int per = nblocks_padded / kXcds;
    return (b % kXcds) * per + b / kXcds;
}

}  // namespace ssam
