// Micro-benchmarks behind the gfx950 latency table (the counterpart of the paper's Table 2,
// Sec. 5.1): cycles per operation of the primitives the kernels are built from -- multiply-add,
// the lane shifts (DPP) and their alternatives through the LDS crossbar, an LDS read, a cached
// global load -- measured as chains of dependent operations inside one wave, optionally with
// several independent chains per wave and several waves per SIMD to expose issue throughput.
#include "ssam_device.h"
#include "ssam_host.h"

namespace ssam {
namespace {

constexpr int kProbeUnroll = 32;
constexpr int kLdsWords = 4096;        // 16 KiB table for the LDS read chain
constexpr int kChaseNearWords = 4096;  // 16 KiB: stays in the vector L1
constexpr int kChaseFarWords = 262144; // 1 MiB: misses the 32 KiB L1, stays in L2

struct ProbeArgs {
    long long* out;      // per wave w < 16: [w] shader clock at start, [16+w] at end, [32+w] / [48+w] the same
                         // on the constant-rate wall clock; [64] sink
    const int* chase;    // successor table for the global-load chains
    int iters;           // chain length = iters * kProbeUnroll operations
    int chase_mask;
    float fa, fb;
    double da, db;
};

struct ProbeState {
    float f;
    double d;
    int i;
};

template <int OP>
__device__ __forceinline__ void probe_step(ProbeState& s, const ProbeArgs& a, const int* lds, int perm_addr)
{
    if constexpr (OP == SSAM_PROBE_FMA_F32) s.f = __builtin_fmaf(s.f, a.fa, a.fb);
    else if constexpr (OP == SSAM_PROBE_FMA_F64) s.d = __builtin_fma(s.d, a.da, a.db);
    else if constexpr (OP == SSAM_PROBE_ADD_F32) s.f = s.f + a.fb;
    else if constexpr (OP == SSAM_PROBE_DPP_WAVE_SHR) s.i = __builtin_amdgcn_mov_dpp(s.i, 0x138, 0xf, 0xf, true);
    else if constexpr (OP == SSAM_PROBE_DPP_ROW_SHR) s.i = __builtin_amdgcn_mov_dpp(s.i, 0x111, 0xf, 0xf, true);
    else if constexpr (OP == SSAM_PROBE_DS_SWIZZLE) s.i = __builtin_amdgcn_ds_swizzle(s.i, 0x041f);   // lane ^ 1
    else if constexpr (OP == SSAM_PROBE_DS_BPERMUTE) s.i = __builtin_amdgcn_ds_bpermute(perm_addr, s.i);
    else if constexpr (OP == SSAM_PROBE_LDS_READ) s.i = lds[s.i];
    else if constexpr (OP == SSAM_PROBE_LOAD_L1 || OP == SSAM_PROBE_LOAD_L2) s.i = a.chase[s.i];
    else if constexpr (OP == SSAM_PROBE_SHIFT_F64) s.d = shift_up(s.d);
}

template <int OP, int ILP>
__global__ __launch_bounds__(1024) void probe_kernel(const ProbeArgs a)
{
    __shared__ int lds[kLdsWords];
    for (int k = threadIdx.x; k < kLdsWords; k += blockDim.x) lds[k] = (k + 64) & (kLdsWords - 1);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int perm_addr = ((lane + 63) & 63) << 2;   // read from the lane below
    ProbeState s[ILP];
#pragma unroll
    for (int k = 0; k < ILP; ++k) {
        s[k].f = a.fa * (float)(lane + k);
        s[k].d = a.da * (double)(lane + k);
        // index chains: each lane walks its own word of consecutive 64-word groups (no bank or
        // line conflicts); independent chains start 64*k words apart
        s[k].i = (lane + 64 * k) & ((OP == SSAM_PROBE_LOAD_L1 || OP == SSAM_PROBE_LOAD_L2) ? a.chase_mask : kLdsWords - 1);
    }

    auto run = [&](int iters) __attribute__((always_inline)) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
                for (int k = 0; k < ILP; ++k) probe_step<OP>(s[k], a, lds, perm_addr);
        }
    };
    auto pin = [&]() __attribute__((always_inline)) {   // the states exist in registers at this point
#pragma unroll
        for (int k = 0; k < ILP; ++k) asm volatile("" : "+v"(s[k].f), "+v"(s[k].d), "+v"(s[k].i));
    };

    // one pass to warm the instruction cache (and, for the load chains, the data caches)
    run(OP == SSAM_PROBE_LOAD_L2 ? (a.chase_mask + 1) / 1024 / kProbeUnroll + 1 : 2);
    pin();
    const long long c0 = clock64();
    const long long r0 = wall_clock64();
    pin();
    run(a.iters);
    pin();
    const long long c1 = clock64();
    const long long r1 = wall_clock64();

    long long sink = 0;
#pragma unroll
    for (int k = 0; k < ILP; ++k) sink += (long long)s[k].f + (long long)s[k].d + s[k].i;
    if (lane == 0) {   // every wave reports: the oldest wave is served first and alone would look uncontended
        const int w = threadIdx.x >> 6;
        a.out[w] = c0;
        a.out[16 + w] = c1;
        a.out[32 + w] = r0;
        a.out[48 + w] = r1;
    }
    if (sink == 0x7fffffffffffffffLL) a.out[64] = sink;   // keeps the chains alive
}

// successor table: word k points 64*stride_groups words ahead, so that a wave (64 consecutive
// words) moves as a unit and consecutive steps touch different cache lines
__global__ void probe_chase_init(int* chase, int words, int step)
{
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < words; k += gridDim.x * blockDim.x)
        chase[k] = (k + step) & (words - 1);
}

template <int OP>
hipError_t probe_launch(int ilp, int waves, const ProbeArgs& a, hipStream_t stream)
{
    const dim3 block(64 * waves);
    switch (ilp) {
        case 1: hipLaunchKernelGGL((probe_kernel<OP, 1>), dim3(1), block, 0, stream, a); break;
        case 2: hipLaunchKernelGGL((probe_kernel<OP, 2>), dim3(1), block, 0, stream, a); break;
        case 4: hipLaunchKernelGGL((probe_kernel<OP, 4>), dim3(1), block, 0, stream, a); break;
        case 8: hipLaunchKernelGGL((probe_kernel<OP, 8>), dim3(1), block, 0, stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace
}  // namespace ssam

using namespace ssam;

extern "C" int ssam_probe_latency(int op, int ilp, int waves, int chain, void* d_scratch, size_t scratch_bytes,
                                  double* h_result, void* hip_stream)
{
    if (!d_scratch || !h_result) return SSAM_ERR_NULL;
    if (op < 0 || op >= SSAM_PROBE_OPS) return SSAM_ERR_ENUM;
    if (ilp != 1 && ilp != 2 && ilp != 4 && ilp != 8) return SSAM_ERR_SHAPE;
    if (waves < 1 || waves > 16 || chain < kProbeUnroll || chain > (1 << 24)) return SSAM_ERR_SHAPE;
    if (scratch_bytes < SSAM_PROBE_SCRATCH_BYTES || ((uintptr_t)d_scratch % 256) != 0) return SSAM_ERR_DIM;
    hipStream_t stream = (hipStream_t)hip_stream;

    ProbeArgs a;
    a.out = static_cast<long long*>(d_scratch);
    int* chase = reinterpret_cast<int*>(static_cast<char*>(d_scratch) + 1024);
    a.chase = chase;
    a.iters = chain / kProbeUnroll;
    a.chase_mask = (op == SSAM_PROBE_LOAD_L2 ? kChaseFarWords : kChaseNearWords) - 1;
    a.fa = 0.999f;
    a.fb = 1e-3f;
    a.da = 0.999;
    a.db = 1e-3;
    if (op == SSAM_PROBE_LOAD_L1 || op == SSAM_PROBE_LOAD_L2) {
        // near table: 64 words per step (every step a new 256-byte group, 16 KiB in all); far
        // table: 1024 words per step (4 KiB apart, 1 MiB in all)
        const int words = a.chase_mask + 1;
        hipLaunchKernelGGL(probe_chase_init, dim3(64), dim3(256), 0, stream, chase, words,
                           op == SSAM_PROBE_LOAD_L2 ? 1024 : 64);
        if (hipGetLastError() != hipSuccess) return SSAM_ERR_HIP;
    }
    hipError_t e;
    switch (op) {
        case SSAM_PROBE_FMA_F32: e = probe_launch<SSAM_PROBE_FMA_F32>(ilp, waves, a, stream); break;
        case SSAM_PROBE_FMA_F64: e = probe_launch<SSAM_PROBE_FMA_F64>(ilp, waves, a, stream); break;
        case SSAM_PROBE_ADD_F32: e = probe_launch<SSAM_PROBE_ADD_F32>(ilp, waves, a, stream); break;
        case SSAM_PROBE_DPP_WAVE_SHR: e = probe_launch<SSAM_PROBE_DPP_WAVE_SHR>(ilp, waves, a, stream); break;
        case SSAM_PROBE_DPP_ROW_SHR: e = probe_launch<SSAM_PROBE_DPP_ROW_SHR>(ilp, waves, a, stream); break;
        case SSAM_PROBE_DS_SWIZZLE: e = probe_launch<SSAM_PROBE_DS_SWIZZLE>(ilp, waves, a, stream); break;
        case SSAM_PROBE_DS_BPERMUTE: e = probe_launch<SSAM_PROBE_DS_BPERMUTE>(ilp, waves, a, stream); break;
        case SSAM_PROBE_LDS_READ: e = probe_launch<SSAM_PROBE_LDS_READ>(ilp, waves, a, stream); break;
        case SSAM_PROBE_LOAD_L1: e = probe_launch<SSAM_PROBE_LOAD_L1>(ilp, waves, a, stream); break;
        case SSAM_PROBE_LOAD_L2: e = probe_launch<SSAM_PROBE_LOAD_L2>(ilp, waves, a, stream); break;
        default: e = probe_launch<SSAM_PROBE_SHIFT_F64>(ilp, waves, a, stream); break;
    }
    if (e != hipSuccess) return SSAM_ERR_HIP;
    long long host[64];
    if (hipMemcpyAsync(host, a.out, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess) return SSAM_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return SSAM_ERR_HIP;
    // the block's span: first wave to start until last wave to finish
    long long c0 = host[0], c1 = host[16], r0 = host[32], r1 = host[48];
    for (int w = 1; w < waves; ++w) {
        if (host[w] < c0) c0 = host[w];
        if (host[16 + w] > c1) c1 = host[16 + w];
        if (host[32 + w] < r0) r0 = host[32 + w];
        if (host[48 + w] > r1) r1 = host[48 + w];
    }
    const double ops = (double)a.iters * kProbeUnroll;
    h_result[0] = (double)(c1 - c0) / ops;        // shader-clock ticks per operation of one chain
    int dev = 0, khz = 0;   // rate of the constant wall clock; 100 MHz where the runtime does not say
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
        (void)hipGetLastError();
        khz = 100000;
    }
    h_result[1] = (double)(r1 - r0) * (1e6 / khz) / ops;   // nanoseconds per operation
    return SSAM_OK;
}
