/* ssam_tuning.h -- experiment and measurement aids of the library; NOT part of its stable interface.
 *
 * Nothing here is needed for correct use of the entry points in ssam.h.  ssam_set_tuning changes
 * launch parameters for the WHOLE PROCESS (every thread's later calls), which is what benchmark
 * sweeps and the tests of alternative kernels want and what a production caller does not; some of its
 * knobs exist only so that tests can force rare paths from the host (the direct kernel, the scan's
 * give-up-and-redo path).  The probes are the kernels the measurements in profiles/ are scaled by.
 */
#ifndef SSAM_TUNING_H_
#define SSAM_TUNING_H_

#include "ssam.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning override for experiments and benchmarks (not needed for correct use): sets a named
 * integer launch parameter for subsequent calls, process-wide.  Names: "rows_per_wave",
 * "valid_lanes", "planes_per_wave", "xcd_remap", "force_generic", "variant" (an alternative
 * compiled instance of the same shape, where one exists; e.g. 5 = the vector-unit instance of a dense
 * fp32 filter whose default instance evaluates its products on the matrix cores), "march_axis" (3D: 0 = march along z,
 * 1 = march along y), "fuse_sweeps" (ssam_stencil_iterate: 0 or 1 = always one sweep per launch, n >= 2 = at most n),
 * "embed_waste" (a 2D filter shape without a compiled instance runs inside the smallest compiled
 * square box that holds it, zero-padded; a value n >= 0 allows that only while the box has at most
 * n times its taps, 0 = never: such shapes then use the direct one-point-per-thread kernel),
 * "scan_segments" (ssam_scan, three-launch schedule: upper limit of segments, 1 .. 4096),
 * "scan_order" (0 = its last launch takes the segments first to last), "scan_chained" (0 = never
 * the one-pass schedule, 1 = for every out-of-place array it can hold; built-in: from 128 MiB),
 * "scan_spin_limit" (polls a waiting wave of the one-pass schedule makes before it gives up, at
 * most 2^20; 0 makes every wave that would wait give up at once -- a test of the redo path),
 * "scan_one_group" (largest element count scanned by one workgroup in one launch; 0 = never);
 * ssam_scan_workspace_bytes follows these.
 * value < 0 restores the built-in choice.  Returns SSAM_OK or SSAM_ERR_ENUM for an unknown name. */
int ssam_set_tuning(const char *name, int value);

/* Measurement aid: copies nbytes (a multiple of 16; both pointers 16-byte aligned, not
 * overlapping) from d_in to d_out with a plain grid-stride 16-bytes-per-lane kernel on hip_stream.
 * It is a reference rate for one-read-one-write kernels (not a ceiling: kernels whose waves move
 * long contiguous runs with streaming accesses, like the one-pass scan, exceed it) and the
 * known-size reference that hardware traffic counters are scaled by. */
int ssam_probe_copy(const void *d_in, void *d_out, size_t nbytes, void *hip_stream);

/* Measurement aid: cycles per operation of the primitives the kernels are built from -- the
 * gfx950 counterpart of the latency table of the paper's performance model (Sec. 5.1, Table 2;
 * the shuffle, multiply-add and shared-memory read of Eq. (4)-(5)).  One block of `waves` waves
 * (1..16; more than 4 put several waves on one SIMD) runs, in every wave, `ilp` (1, 2, 4 or 8)
 * independent chains of `chain` dependent operations each (32..2^24, rounded down to a multiple
 * of 32) and every wave reads the shader clock and the constant-rate wall clock before and after; the
 * time reported is the span from the first wave's start to the last wave's end.
 * ilp = 1, waves = 1 gives the latency of one dependent operation; larger values approach the
 * issue rate.  d_scratch: device memory, 256-byte aligned, at least SSAM_PROBE_SCRATCH_BYTES,
 * overwritten.  h_result (host, 2 doubles): [0] shader-clock ticks per operation of one chain,
 * [1] nanoseconds per operation.  Unlike the other entry points this one synchronises
 * hip_stream before it returns.  Errors: SSAM_ERR_NULL, SSAM_ERR_ENUM (op), SSAM_ERR_SHAPE (ilp,
 * waves, chain), SSAM_ERR_DIM (scratch too small or misaligned), SSAM_ERR_HIP. */
typedef enum {
    SSAM_PROBE_FMA_F32 = 0,       /* v_fma_f32, dependent through the multiplicand            */
    SSAM_PROBE_FMA_F64 = 1,       /* v_fma_f64                                                */
    SSAM_PROBE_ADD_F32 = 2,       /* v_add_f32                                                */
    SSAM_PROBE_DPP_WAVE_SHR = 3,  /* v_mov_b32 with DPP wave_shr:1 -- the shift the kernels use */
    SSAM_PROBE_DPP_ROW_SHR = 4,   /* v_mov_b32 with DPP row_shr:1 (within rows of 16 lanes)    */
    SSAM_PROBE_DS_SWIZZLE = 5,    /* ds_swizzle_b32, lane ^ 1                                  */
    SSAM_PROBE_DS_BPERMUTE = 6,   /* ds_bpermute_b32 from the lane below (a recompiled __shfl_up) */
    SSAM_PROBE_LDS_READ = 7,      /* ds_read_b32, address from the previous read, no conflicts */
    SSAM_PROBE_LOAD_L1 = 8,       /* global_load_dword, address from the previous load, 16 KiB footprint */
    SSAM_PROBE_LOAD_L2 = 9,       /* the same with a 1 MiB footprint, 4 KiB between steps      */
    SSAM_PROBE_SHIFT_F64 = 10,    /* the 64-bit lane shift of the fp64 kernels (two DPP moves)  */
    SSAM_PROBE_OPS = 11
} ssam_probe_op;
#define SSAM_PROBE_SCRATCH_BYTES (2u << 20)
int ssam_probe_latency(int op, int ilp, int waves, int chain, void *d_scratch, size_t scratch_bytes,
                       double *h_result, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SSAM_TUNING_H_ */
