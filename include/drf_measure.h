/*
 * drf_measure.h -- test and measurement hooks of libdrf.
 *
 * These calls are not part of the method's interface (include/drf.h): they expose
 * intermediate state for parity tests and single kernels / per-launch timings for roofline
 * reports.  Same conventions as drf.h: DEVICE pointers belong to the caller, work is enqueued
 * on the given HIP stream, every call returns a drf_status.
 */
#ifndef DRF_MEASURE_H
#define DRF_MEASURE_H

#include "drf.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Introspection for parity tests: run only the first n_blocks blocks (0 = embedding
 * only) and write the fp32 residual stream, DEVICE [slots][T][D], to resid_out.
 */
drf_status drf_eps_trace(drf_denoiser* den, const float* x, const int32_t* t, const void* cond,
                         int slots, int n_blocks, float* resid_out, void* hip_stream);

/*
 * Timing with HIP events on the handle's stream, for roofline reports.
 *   on = 1: every launch of a kernel family is bracketed by two events (this adds a few
 *           microseconds per launch; leave it off when timing whole calls);
 *   on = 2: only each batched predictor pass of drf_sample as a whole is bracketed (all the
 *           kernels of one forward pass; two events per pass, so the pass runs undisturbed);
 *   on = 0: off.
 * drf_profile_read synchronises the device and returns, for family `which` (DRF_PROF_*), the
 * number of bracketed intervals, their summed duration in milliseconds and their summed
 * algorithmic work (flops for GEMM, attention and whole passes, bytes otherwise), then clears
 * that family's counters.  DRF_PROF_PASS_FULL are the passes that evaluate the drafts of a full
 * block (n groups of slots), DRF_PROF_PASS_OTHER all other passes of the call (stand-alone
 * evaluations, cut-short last blocks); their work is slots x the flops of one slot evaluation
 * (2 M N K of every Linear of the blocks and 4 T^2 D per attention, unpadded head width).
 */
enum { DRF_PROF_GEMM = 0, DRF_PROF_ATTN = 1, DRF_PROF_ELEMWISE = 2, DRF_PROF_UPDATE = 3, DRF_PROF_PASS_FULL = 4,
       DRF_PROF_PASS_OTHER = 5, DRF_PROF_FAMILIES = 6 };
drf_status drf_profile_enable(drf_denoiser* den, int on);
drf_status drf_profile_read(drf_denoiser* den, int which, long long* launches, double* ms, double* work);

/*
 * Measurement hook: one launch of the library's bf16 GEMM on caller buffers,
 * out[M][N] (bf16) = A[M][K] (bf16) . W[N][K]^T (bf16) + bias[N] (fp32), all DEVICE.
 * variant 0 = the tile shape the forward pass would pick, > 0 forces one (for sweeps); 10 = the 128 x 128 tile with K
 * split across workgroups where the library's rule allows it (few tiles, at least 18 64-wide k-tiles).
 * K % 64 == 0 and N % 4 == 0 are required.
 */
drf_status drf_probe_gemm_bf16(const void* A, const void* W, int M, int N, int K, void* out_bf16, const float* bias,
                               int variant, void* hip_stream);

/*
 * Measurement hook: one launch of the bf16 self-attention kernel.  qkv: DEVICE bf16
 * [slots * tokens][3 * heads * head_dim] (q | k | v), out: DEVICE bf16 [slots * tokens][heads * head_dim].
 */
drf_status drf_probe_attn_bf16(const void* qkv, void* out, int slots, int tokens, int heads, int head_dim,
                               void* hip_stream);

/*
 * Introspection for the graph-replay tests: how many drf_sample launch sequences the handle holds as
 * instantiated graphs, how many captures failed (those argument sets launch kernel by kernel), and how
 * many calls were served by a graph launch since the handle was created.
 */
drf_status drf_graph_stats(drf_denoiser* den, int* captured, int* failed, long long* replays);

/*
 * Measurement hook: ONE launch of the fused update kernel in the shape drf_sample gives it after a
 * draft pass: guidance combine of the pass's noise fields (g = 2: eps = eps_null + w (eps_cond -
 * eps_null); g = 1: none), the chain of n_chain standard updates s_from -> s_from - 1 -> ... starting
 * from x_base with noise fields 0 .. n_chain - 1, and n_draft skip transitions from the chain's end
 * state (index s_from - n_chain, paired with the last chain field, or field 0 when n_chain == 0) to
 * the next n_draft indices.  Samplers without variance only.
 *   x_base DEVICE fp32 [field]; eps DEVICE fp32 [max(n_chain, 1)][g][field];
 *   x_out DEVICE fp32 [field] or NULL (the chain's end state); draft_out DEVICE fp32 [n_draft][field].
 * Algorithmic bytes: 4 field (1 + g max(n_chain, 1) + (x_out ? 1 : 0) + n_draft).
 */
drf_status drf_probe_update_fused(const drf_sched_config* sched, int s_from, int n_chain, int n_draft, int g, float w,
                                  size_t field, const float* x_base, const float* eps, float* x_out, float* draft_out,
                                  void* hip_stream);

/*
 * Calibration kernels for the roofline denominators, timed with HIP events on `hip_stream`
 * (synchronous: the call returns after `iters` launches have finished).
 *   drf_calibrate_mfma_bf16: `iters` launches of a loop of dependent-free 16x16x32 bf16 MFMAs
 *     (the instruction of the GEMM kernel, 8 waves per CU, operands in registers, no memory
 *     traffic): random_operands != 0 fills the operand registers from a hash, 0 uses constants.
 *     *tflops receives 2 * 16 * 16 * 32 flops per MFMA over the mean launch time.
 *   drf_calibrate_copy: `iters` launches of a plain 16-byte-per-lane copy kernel of `bytes`
 *     bytes from src to dst (DEVICE, 16-byte aligned, bytes % 16 == 0); *gbps receives
 *     2 * bytes (read + written) over the mean launch time.
 */
drf_status drf_calibrate_mfma_bf16(int random_operands, int iters, double* tflops, void* hip_stream);
drf_status drf_calibrate_copy(const void* src, void* dst, size_t bytes, int iters, double* gbps, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DRF_MEASURE_H */
