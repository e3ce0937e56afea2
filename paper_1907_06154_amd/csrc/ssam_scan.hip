// Inclusive scan b_i = a_0 + ... + a_i (Sec. 3.6) mapped onto the register cache: every lane
// holds V consecutive elements, partial sums move between lanes with DPP shifts (a Kogge-Stone
// network inside each row of 16 lanes, two row broadcasts across the rows), and a wave walks its
// contiguous segment of the array with the running total carried in a register.  No LDS and no
// barrier is used by the streaming kernels.
//
// Two schedules share the wave-level code.
//
// Three launches (any size, also in place).  The array is cut into at most kScanMaxSegments (4096)
// contiguous segments, one per wave:
//   1. scan_reduce   -- every wave sums its segment                 (reads n elements)
//   2. scan_offsets  -- one workgroup turns the segment sums into exclusive prefixes
//   3. scan_segments -- every wave scans its segment, starting from its prefix
//                                                                   (reads n, writes n elements)
// No launch waits for another wave.
//
// One pass (large arrays, out of place): every wave keeps a segment of 32 wave-rounds (32 KiB)
// in registers, publishes the segment's sum, obtains the sum of everything before it from what
// earlier waves published, and writes its outputs: n elements read, n written.  Segments are
// handed out through a ticket counter, so a wave only ever waits for waves that are already
// running.  Every wait is bounded: a wave that gives up raises a flag and writes nothing, and a
// one-workgroup kernel enqueued behind the pass (it returns at once unless the flag is up) then
// redoes the whole array.  What is published, with fan = 64 (one item per lane of the reader):
//   A[s]   sum of segment s                          by wave s, right after its loads
//   G[g]   sum of the 64 segments of group g         by the last wave of the group, once it has
//                                                    the A's of its group (and nothing else)
//   SP[q]  sum of everything up to the end of the q-th run of 64 groups
//                                                    by the last wave of the run
// Wave s of group g adds, always in the same order: the A's of the earlier segments of its group;
// the sum of the previous group, formed from that group's A's exactly as its publisher forms it
// (the published G[g-1] would arrive one publication later); the G's of the groups before that in
// the run; and the SP before the run.  Only the A's of the last 64 + i segments are recent when a
// wave asks for them; the first group of a run takes the G's of the whole previous run and the SP
// before that instead of the SP published a moment ago.  The chain SP[0] -> SP[1] -> ... has at
// most 64 links; nothing else that is published waits for another publication.  An item is one
// 64-bit word: the fp64 sum with its lowest mantissa bit set, which doubles as the valid mark
// (the workspace is cleared before the pass), written and read with relaxed device-scope atomics.
// Publisher and readers all use the marked value, so every wave sees the same sums whatever the
// timing, and results are reproducible run to run.  (A non-finite sum stays non-finite, but the
// mark turns an infinity into a NaN.)
//
// Segment sums, prefixes and the running total are kept in fp64 for both element types; sums
// inside one wave-round (64 V elements) are formed in the element type.
#include <atomic>
#include <cstdint>

#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {

std::atomic<int> g_scan_segments{-1}, g_scan_order{-1}, g_scan_chained{-1}, g_scan_spin_limit{-1}, g_scan_one_group{-1};

namespace {

constexpr int kScanMaxSegments = 4096;   // upper limit of waves per launch = doubles in the workspace
constexpr int kScanRounds = 4;           // wave-rounds in flight per wave (loads issued together)
constexpr long long kOneGroupBytes = 128 << 10;  // arrays up to this size: one workgroup, one launch (8 instead of 12.5 us)
constexpr int kOffsetsThreads = 1024;    // the one workgroup of launch 2 ...
constexpr int kOffsetsEach = kScanMaxSegments / kOffsetsThreads;   // ... and the sums one of its threads owns

// One-pass schedule.
// Wave-rounds a wave holds in registers: with 16-byte accesses 32 KiB per segment for fp32 and
// 26 KiB for fp64 (the most that fits 256 registers, two waves per SIMD -- fewer, longer segments
// measured faster than more waves), 16 KiB with element-wise accesses.  The workspace is sized for
// the shortest segments.
constexpr int kChainRoundsF64 = 26;
constexpr int kChainRoundsUnaligned = 16;
constexpr int chain_rounds(int dtype, bool aligned)
{
    return !aligned ? kChainRoundsUnaligned : dtype == SSAM_F32 ? 32 : kChainRoundsF64;
}
constexpr int kChainFan = 64;                                      // items summed per level = lanes
constexpr long long kChainMaxSegments = 64LL * 64 * 64;            // three levels
constexpr long long kChainMinBytes = 128LL << 20;                  // shorter arrays take the three launches (as fast or faster there)
constexpr int kChainSpinLimit = 1 << 16;                           // polls before a wave gives up
using Word = unsigned long long;
// Workspace of the one-pass schedule, in 8-byte words: ticket counter, flag, SP, G, A.  The ticket counter (one atomic per workgroup) and
// every SP item (read by all 4096 waves of the following run) have a 128-byte line to themselves:
// sharing one line made the runs that watch it several times slower.
constexpr long long kWsTicket = 0, kWsGaveUp = 16, kWsSP = 32, kWsSPStride = 16,
                    kWsG = kWsSP + kWsSPStride * kChainFan, kWsA = kWsG + kChainFan * kChainFan;

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

// 16 bytes per lane.
template <class T> struct ScanVec { static constexpr int V = 16 / sizeof(T); };

// Elements [i, i + V) of a, zeros past n.  ALIGNED: the base pointer is 16-byte aligned, so a
// vector that lies wholly inside the array is one 16-byte access.  STREAM: non-temporal access --
// the one-pass schedule, whose arrays are far larger than the caches, gains 6 % from it; the three
// launches keep plain accesses, their second read of a mid-sized array comes from the caches.
template <class T, bool ALIGNED, bool STREAM = false>
__device__ __forceinline__ void load_elems(const T* __restrict__ a, long long i, long long n, T (&v)[ScanVec<T>::V])
{
    constexpr int V = ScanVec<T>::V;
    if (ALIGNED && i + V <= n) {
        load_vec<T, V, STREAM>(a + i, v);
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = (i + j < n) ? a[i + j] : T(0);
    }
}

template <class T, bool ALIGNED, bool STREAM = false>
__device__ __forceinline__ void store_elems(T* __restrict__ b, long long i, long long n, const T (&v)[ScanVec<T>::V])
{
    constexpr int V = ScanVec<T>::V;
    if (ALIGNED && i + V <= n) {
        store_vec<T, V, STREAM>(b + i, v);
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

// Launch 2: sums[s] <- sums[0] + ... + sums[s-1], in place, by one workgroup.  A thread owns up to
// kOffsetsEach consecutive sums and fetches them all before it adds any.
__global__ __launch_bounds__(kOffsetsThreads) void scan_offsets(double* __restrict__ sums, int segments)
{
    __shared__ double wave_total[kOffsetsThreads / kWave];
    const int t = threadIdx.x, lane = t & (kWave - 1), w = t >> 6;
    const int each = (segments + kOffsetsThreads - 1) / kOffsetsThreads;
    const int i0 = t * each;
    double x[kOffsetsEach];
#pragma unroll
    for (int k = 0; k < kOffsetsEach; ++k) x[k] = (k < each && i0 + k < segments) ? sums[i0 + k] : 0.0;
    double mine = 0.0;
#pragma unroll
    for (int k = 0; k < kOffsetsEach; ++k) mine += x[k];
    const double incl = wave_inclusive_scan(mine);
    if (lane == kWave - 1) wave_total[w] = incl;
    __syncthreads();
    double run = shift_up(incl);   // total of the lanes below (0 in lane 0)
    for (int k = 0; k < w; ++k) run += wave_total[k];
#pragma unroll
    for (int k = 0; k < kOffsetsEach; ++k) {
        if (k < each && i0 + k < segments) sums[i0 + k] = run;
        run += x[k];
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

// ---- one pass ---------------------------------------------------------------------------

struct ChainPlan {
    long long n;
    int segments;     // ceil(n / (rounds per segment * 64 * V))
    int spin_limit;   // polls a waiting wave makes before it gives up
};

__global__ __launch_bounds__(kBlock) void scan_clear(Word* ws, long long words)
{
    for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < words; i += (long long)gridDim.x * kBlock) ws[i] = 0;
}

// A published sum: the value with the lowest mantissa bit set.
__device__ __forceinline__ double marked(double v)
{
    return __builtin_bit_cast(double, __builtin_bit_cast(Word, v) | 1ull);
}
__device__ __forceinline__ void publish(Word* item, double marked_value)
{
    __hip_atomic_store(item, __builtin_bit_cast(Word, marked_value), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool poll(const Word* item, Word& w)
{
    w = __hip_atomic_load(item, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return (w & 1ull) != 0;
}
__device__ __forceinline__ double item_value(Word w) { return __builtin_bit_cast(double, w); }

// Sum over the lanes, the same association every time.
__device__ __forceinline__ double wave_total_of(double x)
{
    return read_lane(wave_inclusive_scan(x), kWave - 1);
}

// The sum of a group as its publisher forms it: the first 63 segment sums through the lane
// network, plus the last one, marked.
__device__ __forceinline__ double group_sum(double first63, double last)
{
    return marked(first63 + last);
}

template <class T, bool ALIGNED>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2))) void scan_chained(const T* __restrict__ a, T* __restrict__ b, Word* ws, ChainPlan pl)
{
    constexpr int V = ScanVec<T>::V;
    constexpr int kChainRounds = chain_rounds(sizeof(T) == 4 ? SSAM_F32 : SSAM_F64, ALIGNED);
    __shared__ unsigned ticket;
    if (threadIdx.x == 0)
        ticket = __hip_atomic_fetch_add(reinterpret_cast<unsigned*>(ws + kWsTicket), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const long long s = (long long)ticket * kWavesPerBlock + (threadIdx.x >> 6);   // every lower-numbered segment has a running wave
    if (s >= pl.segments) return;

    T v[kChainRounds][V];
    const long long e0 = (s * kChainRounds * kWave + lane) * V;
#pragma unroll
    for (int k = 0; k < kChainRounds; ++k) load_elems<T, ALIGNED, true>(a, e0 + (long long)k * kWave * V, pl.n, v[k]);

    // the segment's sum, published before anything is waited for
    double mine = 0.0;
#pragma unroll
    for (int k = 0; k < kChainRounds; ++k) {
        T t = v[k][0];
#pragma unroll
        for (int j = 1; j < V; ++j) t += v[k][j];
        mine += (double)t;
    }
    const double own = marked(wave_total_of(mine));
    Word* const A = ws + kWsA;
    Word* const G = ws + kWsG;
    Word* const SP = ws + kWsSP;
    if (lane == 0) publish(A + s, own);

    // The scan inside the segment, while the sums of the earlier waves arrive: afterwards v holds
    // every element's prefix within its wave-round, and lane k the sum of the rounds before round k.
    double round_total = 0.0;
#pragma unroll
    for (int k = 0; k < kChainRounds; ++k) {
#pragma unroll
        for (int j = 1; j < V; ++j) v[k][j] += v[k][j - 1];
        const T incl = wave_inclusive_scan(v[k][V - 1]);
        const T before = shift_up(incl);
#pragma unroll
        for (int j = 0; j < V; ++j) v[k][j] += before;
        const double t = (double)read_lane(incl, kWave - 1);
        if (lane == k) round_total = t;
    }
    const double round_start = shift_up(wave_inclusive_scan(round_total));

    // What lies before the segment, one item per lane and kind:
    //   mine_[l] = A[64 g + l], l < i         the earlier segments of the group
    //   prev[l]  = A[64 (g - 1) + l]          the previous group, every segment of it
    //   grp[l]   = G[gbase + l], l < gcount   the groups before that: of this run, or (first group of
    //                                         a run) of the previous run without its last group
    //   run      = SP[qprev]                  everything before those groups' run
    const long long g = s / kChainFan, q = g / kChainFan;
    const int i = (int)(s % kChainFan), gi = (int)(g % kChainFan);
    const long long gbase = (gi >= 1 ? q : q - 1) * kChainFan, qprev = gi >= 1 ? q - 1 : q - 2;
    const int gcount = gi >= 1 ? gi - 1 : (q >= 1 ? kChainFan - 1 : 0);
    const bool need_mine = lane < i, need_prev = g > 0, need_grp = lane < gcount, need_run = lane == 0 && qprev >= 0;
    bool ok_mine = !need_mine, ok_prev = !need_prev, ok_grp = !need_grp, ok_run = !need_run;
    Word w_mine = 0, w_prev = 0, w_grp = 0, w_run = 0;
    bool latest_in = s == 0;      // A[s - 1], the item published last, is in: until then one lane polls
    bool group_out = i != kChainFan - 1;
    double sum_mine = 0.0;
    int polls = 0;
    for (;;) {
        if (!group_out && !__any(!ok_mine)) {
            // last wave of a group: the group's sum goes out as soon as its segment sums are in
            sum_mine = wave_total_of(need_mine ? item_value(w_mine) : 0.0);
            if (lane == 0) publish(G + g, group_sum(sum_mine, own));
            group_out = true;
        }
        if (!__any(!(ok_mine && ok_prev && ok_grp && ok_run))) break;
        if (polls++ >= pl.spin_limit) {      // give up: the kernel behind this pass redoes the array
            if (lane == 0) __hip_atomic_store(ws + kWsGaveUp, (Word)1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (!latest_in) {
            Word w = 0;
            if (lane == 0) poll(A + s - 1, w);
            latest_in = __any((int)(w & 1ull));
        }
        if (latest_in) {
            if (!ok_mine) ok_mine = poll(A + g * kChainFan + lane, w_mine);
            if (!ok_prev) ok_prev = poll(A + (g - 1) * kChainFan + lane, w_prev);
            if (!ok_grp) ok_grp = poll(G + gbase + lane, w_grp);
            if (!ok_run) ok_run = poll(SP + kWsSPStride * qprev, w_run);
            if (!__any(!(ok_mine && ok_prev && ok_grp && ok_run))) continue;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    if (i != kChainFan - 1) sum_mine = wave_total_of(need_mine ? item_value(w_mine) : 0.0);
    const double prev_group = g > 0 ? group_sum(wave_total_of(lane < kChainFan - 1 ? item_value(w_prev) : 0.0),
                                                read_lane(item_value(w_prev), kChainFan - 1))
                                    : 0.0;
    const double sum_grp = wave_total_of(need_grp ? item_value(w_grp) : 0.0);
    const double before_group = (read_lane(need_run ? item_value(w_run) : 0.0, 0) + sum_grp) + prev_group;
    if (i == kChainFan - 1 && gi == kChainFan - 1 && lane == 0)
        publish(SP + kWsSPStride * q, marked(before_group + group_sum(sum_mine, own)));

    // only the start value is missing now: add it, round once, store
    const double start = before_group + sum_mine;
#pragma unroll
    for (int k = 0; k < kChainRounds; ++k) {
        const double c = start + read_lane(round_start, k);
        T o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = (T)(c + (double)v[k][j]);
        store_elems<T, ALIGNED, true>(b, e0 + (long long)k * kWave * V, pl.n, o);
    }
}

// The whole scan by ONE workgroup: 16 waves, each a contiguous piece of kScanRounds wave-rounds per
// step, piece sums exchanged through LDS, one barrier per step; in place is fine.  Two uses:
//  - short arrays (gave_up == nullptr): one launch instead of three, which is all that counts there;
//  - the fallback of the one-pass schedule, enqueued behind every pass: it returns at once unless
//    the word at gave_up is set.  It is slow (about 30 ms per GiB) and only runs after a wave has
//    already waited for 2^16 polls.
template <class T, bool ALIGNED>
__global__ __launch_bounds__(kOffsetsThreads) void scan_one_group(const T* a, T* b, long long n, const Word* gave_up)
{
    if (gave_up && __hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) return;
    constexpr int V = ScanVec<T>::V;
    constexpr int NWAVES = kOffsetsThreads / kWave;
    __shared__ double piece_total[2][NWAVES];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    const long long per_wave = (long long)kScanRounds * kWave * V, per_step = per_wave * NWAVES;
    double carry = 0.0;
    int buf = 0;
    for (long long base = 0; base < n; base += per_step, buf ^= 1) {
        T v[kScanRounds][V];
        const long long e0 = base + w * per_wave + (long long)lane * V;
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) load_elems<T, ALIGNED>(a, e0 + (long long)k * kWave * V, n, v[k]);
        double round_total = 0.0;
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
#pragma unroll
            for (int j = 1; j < V; ++j) v[k][j] += v[k][j - 1];
            const T incl = wave_inclusive_scan(v[k][V - 1]);
            const T before = shift_up(incl);
#pragma unroll
            for (int j = 0; j < V; ++j) v[k][j] += before;
            const double t = (double)read_lane(incl, kWave - 1);
            if (lane == k) round_total = t;
        }
        const double rounds_incl = wave_inclusive_scan(round_total);
        const double round_start = shift_up(rounds_incl);
        if (lane == kWave - 1) piece_total[buf][w] = rounds_incl;
        __syncthreads();       // the other buffer is written next step, after every wave has passed this barrier
        double start = carry, step_total = 0.0;
        for (int u = 0; u < NWAVES; ++u) {
            const double t = piece_total[buf][u];
            if (u < w) start += t;
            step_total += t;
        }
#pragma unroll
        for (int k = 0; k < kScanRounds; ++k) {
            const double c = start + read_lane(round_start, k);
            T o[V];
#pragma unroll
            for (int j = 0; j < V; ++j) o[j] = (T)(c + (double)v[k][j]);
            store_elems<T, ALIGNED>(b, e0 + (long long)k * kWave * V, n, o);
        }
        carry += step_total;
    }
}

// ---- host side ---------------------------------------------------------------------------

ScanPlan plan_scan(long long n, int dtype, int cap)
{
    const int V = dtype == SSAM_F32 ? 4 : 2;
    ScanPlan pl{};
    pl.n = n;
    pl.rounds = (n + (long long)kWave * V - 1) / ((long long)kWave * V);
    long long per = (pl.rounds + cap - 1) / cap;
    per = (per + kScanRounds - 1) / kScanRounds * kScanRounds;
    if (per < kScanRounds) per = kScanRounds;
    pl.per_seg = per;
    pl.segments = (int)((pl.rounds + per - 1) / per);
    pl.reverse = g_scan_order.load() == 0 ? 0 : 1;
    return pl;
}

int segment_cap()
{
    const int cap = g_scan_segments.load();
    return cap < 1 || cap > kScanMaxSegments ? kScanMaxSegments : cap;
}

// Segments of the one-pass schedule with `rounds` wave-rounds each, or 0 if an array of this size
// does not take it (the pointers can still rule it out: in place always takes the three launches).
// Whether it does is decided on the shorter segments, whatever the alignment.
long long chained_segments(long long n, int dtype, int rounds)
{
    const int V = dtype == SSAM_F32 ? 4 : 2;
    const long long per_short = (long long)kChainRoundsUnaligned * kWave * V, per = (long long)rounds * kWave * V;
    const int mode = g_scan_chained.load();
    if (mode == 0 || (n + per_short - 1) / per_short > kChainMaxSegments) return 0;
    if (mode < 0 && n * (dtype == SSAM_F32 ? 4 : 8) < kChainMinBytes) return 0;
    return (n + per - 1) / per;
}

// Arrays up to this many elements are scanned by one workgroup in one launch (no workspace).
long long one_group_limit(int dtype)
{
    const int v = g_scan_one_group.load();
    return v < 0 ? kOneGroupBytes / (dtype == SSAM_F32 ? 4 : 8) : v;
}

size_t three_launch_bytes(long long n, int dtype)
{
    if (n <= one_group_limit(dtype)) return 0;
    const ScanPlan pl = plan_scan(n, dtype, segment_cap());
    return pl.segments > 1 ? (size_t)pl.segments * sizeof(double) : 0;
}

size_t chained_bytes(long long segs)
{
    return segs ? (size_t)(kWsA + segs) * sizeof(Word) : 0;
}

template <class T, bool ALIGNED>
void launch_three(const void* d_in, void* d_out, double* sums, const ScanPlan& pl, hipStream_t st)
{
    const unsigned blocks = (unsigned)((pl.segments + kWavesPerBlock - 1) / kWavesPerBlock);
    if (pl.segments > 1) {
        hipLaunchKernelGGL((scan_reduce<T, ALIGNED>), dim3(blocks), dim3(kBlock), 0, st,
                           static_cast<const T*>(d_in), sums, pl);
        hipLaunchKernelGGL(scan_offsets, dim3(1), dim3(kOffsetsThreads), 0, st, sums, pl.segments);
    }
    hipLaunchKernelGGL((scan_segments<T, ALIGNED>), dim3(blocks), dim3(kBlock), 0, st,
                       static_cast<const T*>(d_in), static_cast<T*>(d_out),
                       pl.segments > 1 ? sums : nullptr, pl);
}

template <class T, bool ALIGNED>
int launch_scan(const void* d_in, void* d_out, void* d_work, long long n, int dtype, long long chain_segs, hipStream_t st)
{
    if (!chain_segs && n <= one_group_limit(dtype)) {
        hipLaunchKernelGGL((scan_one_group<T, ALIGNED>), dim3(1), dim3(kOffsetsThreads), 0, st,
                           static_cast<const T*>(d_in), static_cast<T*>(d_out), n, static_cast<const Word*>(nullptr));
        return hipGetLastError() == hipSuccess ? SSAM_OK : SSAM_ERR_HIP;
    }
    if (!chain_segs) {
        launch_three<T, ALIGNED>(d_in, d_out, static_cast<double*>(d_work), plan_scan(n, dtype, segment_cap()), st);
        return hipGetLastError() == hipSuccess ? SSAM_OK : SSAM_ERR_HIP;
    }
    Word* ws = static_cast<Word*>(d_work);
    const long long words = kWsA + chain_segs;
    const long long fill_blocks = (words + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(scan_clear, dim3((unsigned)(fill_blocks < 512 ? fill_blocks : 512)), dim3(kBlock), 0, st, ws, words);
    ChainPlan cp{};
    cp.n = n;
    cp.segments = (int)chain_segs;
    const int limit = g_scan_spin_limit.load();
    cp.spin_limit = limit < 0 ? kChainSpinLimit : limit > (1 << 20) ? (1 << 20) : limit;
    const unsigned blocks = (unsigned)((chain_segs + kWavesPerBlock - 1) / kWavesPerBlock);
    hipLaunchKernelGGL((scan_chained<T, ALIGNED>), dim3(blocks), dim3(kBlock), 0, st,
                       static_cast<const T*>(d_in), static_cast<T*>(d_out), ws, cp);
    hipLaunchKernelGGL((scan_one_group<T, ALIGNED>), dim3(1), dim3(kOffsetsThreads), 0, st,
                       static_cast<const T*>(d_in), static_cast<T*>(d_out), n, ws + kWsGaveUp);
    return hipGetLastError() == hipSuccess ? SSAM_OK : SSAM_ERR_HIP;
}

// ---- workspace held by the library (ssam_scan_static) ----------------------------------------
// Sized for the largest workspace any schedule asks for: the one-pass layout with the most
// segments it accepts.  Every GPU the library runs on holds its own copy until the process ends.
constexpr long long kStaticWords = kWsA + kChainMaxSegments;
static __device__ __align__(256) Word scratch[kStaticWords];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_of_device[kMaxDevices];

// Device address of `scratch` on the current device (the array's name is only a host-side handle:
// each GPU has its copy at an address of its own, looked up once per device).
int static_scratch(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSAM_ERR_HIP;
    void* p = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SSAM_ERR_HIP;
        }
        g_scratch_of_device[dev].store(p, std::memory_order_release);   // every thread finds the same address
    }
    *out = p;
    return SSAM_OK;
}

}  // namespace
}  // namespace ssam

extern "C" {

int ssam_scan_static(const void* d_in, void* d_out, long long n, int dtype, void* hip_stream)
{
    using namespace ssam;
    if (dtype != SSAM_F32 && dtype != SSAM_F64) return SSAM_ERR_ENUM;
    if (n < 0 || n > SSAM_SCAN_STATIC_MAX_ELEMENTS) return SSAM_ERR_DIM;
    if (n == 0) return SSAM_OK;
    if (!d_in || !d_out) return SSAM_ERR_NULL;
    if (ssam_scan_workspace_bytes(n, dtype) > sizeof(Word) * (size_t)kStaticWords) return SSAM_ERR_DIM;
    void* ws = nullptr;
    if (int e = static_scratch(&ws)) return e;
    // ssam_scan clears what its kernels expect to start at zero (the one-pass schedule's counter,
    // flag and published sums) with a kernel of its own on the same stream, so the contents the
    // previous call left behind do not matter.
    return ssam_scan(d_in, d_out, n, dtype, ws, sizeof(Word) * (size_t)kStaticWords, hip_stream);
}

size_t ssam_scan_workspace_bytes(long long n, int dtype)
{
    if (n <= 0 || n > (1LL << 40) || (dtype != SSAM_F32 && dtype != SSAM_F64)) return 0;
    const size_t three = ssam::three_launch_bytes(n, dtype), one = ssam::chained_bytes(ssam::chained_segments(n, dtype, ssam::kChainRoundsUnaligned));
    return three > one ? three : one;
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
    const bool aligned = pa % 16 == 0 && pb % 16 == 0;
    const long long chain_segs = pa == pb ? 0 : chained_segments(n, dtype, chain_rounds(dtype, aligned));
    const size_t need = chain_segs ? chained_bytes(chained_segments(n, dtype, kChainRoundsUnaligned)) : three_launch_bytes(n, dtype);
    if (need) {
        if (!d_work) return SSAM_ERR_NULL;
        const uintptr_t pw = (uintptr_t)d_work;
        if (work_bytes < need || pw % sizeof(double)) return SSAM_ERR_DIM;
        if ((pw < pa + bytes && pa < pw + need) || (pw < pb + bytes && pb < pw + need)) return SSAM_ERR_ALIAS;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == SSAM_F32)
        return aligned ? launch_scan<float, true>(d_in, d_out, d_work, n, dtype, chain_segs, st)
                       : launch_scan<float, false>(d_in, d_out, d_work, n, dtype, chain_segs, st);
    return aligned ? launch_scan<double, true>(d_in, d_out, d_work, n, dtype, chain_segs, st)
                   : launch_scan<double, false>(d_in, d_out, d_work, n, dtype, chain_segs, st);
}

}  // extern "C"
