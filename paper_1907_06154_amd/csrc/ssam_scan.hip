// Inclusive scan b_i = a_0 + ... + a_i (Sec. 3.6) mapped onto the register cache: every lane
// holds V consecutive elements, partial sums move between lanes with DPP shifts (a Kogge-Stone
// network inside each row of 16 lanes, two row broadcasts across the rows), and a wave walks its
// contiguous segment of the array with the running total carried in a register.  No LDS and no
// barrier is used by the streaming kernels.
//
// The array is cut into at most kMaxSegments contiguous segments, one per wave, and three
// launches run on the caller's stream:
//   1. scan_reduce   -- every wave sums its segment                 (reads n elements)
//   2. scan_offsets  -- one workgroup turns the segment sums into exclusive prefixes
//   3. scan_segments -- every wave scans its segment, starting from its prefix
//                                                                   (reads n, writes n elements)
// No launch waits for another wave, so there is nothing to spin on.  Segment sums, prefixes and
// the running total are kept in fp64 for both element types; sums inside one wave-round
// (64 V elements) are formed in the element type.
#include <atomic>
#include <cstdint>

#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {

std::atomic<int> g_scan_segments{-1}, g_scan_order{-1};

namespace {

constexpr int kScanMaxSegments = 32768;  // upper limit of waves per launch = doubles in the workspace
constexpr int kScanRounds = 4;           // wave-rounds in flight per wave (loads issued together)
constexpr int kOffsetsThreads = 1024;    // the one workgroup of launch 2

// DPP controls (GFX9 encoding): 0x110 + n = row_shr:n, 0x142 = row_bcast:15, 0x143 = row_bcast:31.
// "old" is 0: a lane without a source (bound_ctrl) or outside the row mask contributes 0.
template <int CTRL, int ROWS, bool BOUND>
__device__ __forceinline__ int dpp_or_zero(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROWS, 0xf, BOUND);
}
template <int CTRL, int ROWS, bool BOUND>
__device__ __forceinline__ float from_lane(float v)
{
    return __builtin_bit_cast(float, dpp_or_zero<CTRL, ROWS, BOUND>(__builtin_bit_cast(int, v)));
}
template <int CTRL, int ROWS, bool BOUND>
__device__ __forceinline__ double from_lane(double v)
{
    Halves h = __builtin_bit_cast(Halves, v);
    h.lo = dpp_or_zero<CTRL, ROWS, BOUND>(h.lo);
    h.hi = dpp_or_zero<CTRL, ROWS, BOUND>(h.hi);
    return __builtin_bit_cast(double, h);
}

// Inclusive scan over the 64 lanes of a wave: four Kogge-Stone steps inside each row of 16
// lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
template <class T>
__device__ __forceinline__ T wave_inclusive_scan(T x)
{
    x += from_lane<0x111, 0xf, true>(x);
    x += from_lane<0x112, 0xf, true>(x);
    x += from_lane<0x114, 0xf, true>(x);
    x += from_lane<0x118, 0xf, true>(x);
    x += from_lane<0x142, 0xa, false>(x);
    x += from_lane<0x143, 0xc, false>(x);
    return x;
}

template <class T> struct ScanVec;
template <> struct ScanVec<float> { using type = float4; static constexpr int V = 4; };
template <> struct ScanVec<double> { using type = double2; static constexpr int V = 2; };

// Elements [i, i + V) of a, zeros past n.  ALIGNED: the base pointer is 16-byte aligned, so a
// vector that lies wholly inside the array is one 16-byte access.
template <class T, bool ALIGNED>
__device__ __forceinline__ void load_elems(const T* __restrict__ a, long long i, long long n, T (&v)[ScanVec<T>::V])
{
    constexpr int V = ScanVec<T>::V;
    if (ALIGNED && i + V <= n) {
        const typename ScanVec<T>::type q = *reinterpret_cast<const typename ScanVec<T>::type*>(a + i);
        if constexpr (V == 4) { v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w; }
        else { v[0] = q.x; v[1] = q.y; }
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = (i + j < n) ? a[i + j] : T(0);
    }
}

template <class T, bool ALIGNED>
__device__ __forceinline__ void store_elems(T* __restrict__ b, long long i, long long n, const T (&v)[ScanVec<T>::V])
{
    constexpr int V = ScanVec<T>::V;
    if (ALIGNED && i + V <= n) {
        typename ScanVec<T>::type q;
        if constexpr (V == 4) { q.x = v[0]; q.y = v[1]; q.z = v[2]; q.w = v[3]; }
        else { q.x = v[0]; q.y = v[1]; }
        *reinterpret_cast<typename ScanVec<T>::type*>(b + i) = q;
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j)
            if (i + j < n) b[i + j] = v[j];
    }
}

struct ScanPlan {
    long long n;         // elements
    long long rounds;    // wave-rounds in the array: ceil(n / (64 V))
    long long per_seg;   // wave-rounds per segment (a multiple of kScanRounds)
    int segments;        // ceil(rounds / per_seg), at most kScanMaxSegments
    int reverse;         // launch 3 takes the segments last to first
};

// Launch 1: sums[s] = sum of segment s.
template <class T, bool ALIGNED>
__global__ __launch_bounds__(kBlock) void scan_reduce(const T* __restrict__ a, double* __restrict__ sums, ScanPlan pl)
{
    constexpr int V = ScanVec<T>::V;
    const int lane = threadIdx.x & (kWave - 1);
    const long long s = (long long)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (s >= pl.segments) return;
    const long long r0 = s * pl.per_seg;
    const long long r1 = r0 + pl.per_seg < pl.rounds ? r0 + pl.per_seg : pl.rounds;
    double acc = 0.0;
    for (long long r = r0; r < r1; r += kScanRounds) {
        T v[kScanRounds][V];
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
            if (r + k < r1) load_elems<T, ALIGNED>(a, ((r + k) * kWave + lane) * V, pl.n, v[k]);
            else
#pragma unroll
                for (int j = 0; j < V; ++j) v[k][j] = T(0);
        }
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
            T t = v[k][0];
#pragma unroll
            for (int j = 1; j < V; ++j) t += v[k][j];
            acc += (double)t;
        }
    }
    acc = wave_inclusive_scan(acc);
    if (lane == kWave - 1) sums[s] = acc;
}

// Launch 2: sums[s] <- sums[0] + ... + sums[s-1], in place, by one workgroup.
__global__ __launch_bounds__(kOffsetsThreads) void scan_offsets(double* __restrict__ sums, int segments)
{
    __shared__ double wave_total[kOffsetsThreads / kWave];
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t >> 6;
    const int each = (segments + kOffsetsThreads - 1) / kOffsetsThreads;
    const int i0 = t * each;
    double mine = 0.0;
    for (int i = i0; i < i0 + each && i < segments; ++i) mine += sums[i];
    const double incl = wave_inclusive_scan(mine);
    if (lane == kWave - 1) wave_total[w] = incl;
    __syncthreads();
    double run = shift_up(incl);   // total of the lanes below (0 in lane 0)
    for (int k = 0; k < w; ++k) run += wave_total[k];
    for (int i = i0; i < i0 + each && i < segments; ++i) {
        const double x = sums[i];
        sums[i] = run;
        run += x;
    }
}

// Launch 3: the scan proper.  offsets == nullptr: a single segment that starts from 0.
template <class T, bool ALIGNED>
__global__ __launch_bounds__(kBlock) void scan_segments(const T* a, T* b, const double* __restrict__ offsets, ScanPlan pl)
{
    constexpr int V = ScanVec<T>::V;
    const int lane = threadIdx.x & (kWave - 1);
    long long s = (long long)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (s >= pl.segments) return;
    if (pl.reverse) s = pl.segments - 1 - s;
    const long long r0 = s * pl.per_seg;
    const long long r1 = r0 + pl.per_seg < pl.rounds ? r0 + pl.per_seg : pl.rounds;
    double carry = offsets ? offsets[s] : 0.0;
    for (long long r = r0; r < r1; r += kScanRounds) {
        T v[kScanRounds][V];
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
            if (r + k < r1) load_elems<T, ALIGNED>(a, ((r + k) * kWave + lane) * V, pl.n, v[k]);
            else
#pragma unroll
                for (int j = 0; j < V; ++j) v[k][j] = T(0);
        }
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
            if (r + k < r1) {
#pragma unroll
                for (int j = 1; j < V; ++j) v[k][j] += v[k][j - 1];      // prefixes of the lane's own elements
                const T incl = wave_inclusive_scan(v[k][V - 1]);          // ... of the lane totals
                const T before = shift_up(incl);                           // total of the lanes below
                T o[V];
#pragma unroll
                for (int j = 0; j < V; ++j) o[j] = (T)(carry + (double)(before + v[k][j]));
                store_elems<T, ALIGNED>(b, ((r + k) * kWave + lane) * V, pl.n, o);
                carry += (double)read_lane(incl, kWave - 1);
            }
        }
    }
}

ScanPlan plan_scan(long long n, int dtype)
{
    const int V = dtype == SSAM_F32 ? 4 : 2;
    ScanPlan pl{};
    pl.n = n;
    pl.rounds = (n + (long long)kWave * V - 1) / ((long long)kWave * V);
    int cap = g_scan_segments.load();
    if (cap < 1 || cap > kScanMaxSegments) cap = kScanMaxSegments;
    long long per = (pl.rounds + cap - 1) / cap;
    per = (per + kScanRounds - 1) / kScanRounds * kScanRounds;
    if (per < kScanRounds) per = kScanRounds;
    pl.per_seg = per;
    pl.segments = (int)((pl.rounds + per - 1) / per);
    pl.reverse = g_scan_order.load() == 0 ? 0 : 1;
    return pl;
}

template <class T, bool ALIGNED>
int launch_scan(const void* d_in, void* d_out, void* d_work, const ScanPlan& pl, hipStream_t st)
{
    const unsigned blocks = (unsigned)((pl.segments + kWavesPerBlock - 1) / kWavesPerBlock);
    double* sums = static_cast<double*>(d_work);
    if (pl.segments > 1) {
        hipLaunchKernelGGL((scan_reduce<T, ALIGNED>), dim3(blocks), dim3(kBlock), 0, st,
                           static_cast<const T*>(d_in), sums, pl);
        hipLaunchKernelGGL(scan_offsets, dim3(1), dim3(kOffsetsThreads), 0, st, sums, pl.segments);
    }
    hipLaunchKernelGGL((scan_segments<T, ALIGNED>), dim3(blocks), dim3(kBlock), 0, st,
                       static_cast<const T*>(d_in), static_cast<T*>(d_out),
                       pl.segments > 1 ? sums : nullptr, pl);
    return hipGetLastError() == hipSuccess ? SSAM_OK : SSAM_ERR_HIP;
}

}  // namespace
}  // namespace ssam

extern "C" {

size_t ssam_scan_workspace_bytes(long long n, int dtype)
{
    if (n <= 0 || (dtype != SSAM_F32 && dtype != SSAM_F64)) return 0;
    const ssam::ScanPlan pl = ssam::plan_scan(n, dtype);
    return pl.segments > 1 ? (size_t)pl.segments * sizeof(double) : 0;
}

int ssam_scan(const void* d_in, void* d_out, long long n, int dtype, void* d_work, size_t work_bytes, void* hip_stream)
{
    using namespace ssam;
    if (dtype != SSAM_F32 && dtype != SSAM_F64) return SSAM_ERR_ENUM;
    if (n < 0 || n > (1LL << 40)) return SSAM_ERR_DIM;
    if (n == 0) return SSAM_OK;
    if (!d_in || !d_out) return SSAM_ERR_NULL;
    const size_t esz = dtype == SSAM_F32 ? 4 : 8;
    const uintptr_t pa = (uintptr_t)d_in, pb = (uintptr_t)d_out;
    if (pa % esz || pb % esz) return SSAM_ERR_DIM;
    const size_t bytes = (size_t)n * esz;
    if (pa != pb && pa < pb + bytes && pb < pa + bytes) return SSAM_ERR_ALIAS;   // in place is fine, a partial overlap is not
    const ScanPlan pl = plan_scan(n, dtype);
    const size_t need = pl.segments > 1 ? (size_t)pl.segments * sizeof(double) : 0;
    if (need) {
        if (!d_work) return SSAM_ERR_NULL;
        const uintptr_t pw = (uintptr_t)d_work;
        if (work_bytes < need || pw % sizeof(double)) return SSAM_ERR_DIM;
        if ((pw < pa + bytes && pa < pw + need) || (pw < pb + bytes && pb < pw + need)) return SSAM_ERR_ALIAS;
    }
    const bool aligned = pa % 16 == 0 && pb % 16 == 0;
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == SSAM_F32)
        return aligned ? launch_scan<float, true>(d_in, d_out, d_work, pl, st) : launch_scan<float, false>(d_in, d_out, d_work, pl, st);
    return aligned ? launch_scan<double, true>(d_in, d_out, d_work, pl, st) : launch_scan<double, false>(d_in, d_out, d_work, pl, st);
}

}  // extern "C"
