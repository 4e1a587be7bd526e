/*
 * mrl_diag.h - measurement aids of the MI355X GRPO scoring library.
 *
 * Not part of the product boundary (include/mrl.h): a training or serving loop needs none of
 * this.  The benchmark uses these calls to time the kernel classes of a step with HIP events
 * on the launch stream (the figures behind its roofline object) and to measure what the matrix
 * cores of the box sustain with no memory traffic.  Same conventions as mrl.h: mrl_status
 * return codes, device pointers owned by the caller, nothing allocated on the device.
 */
#ifndef MRL_DIAG_H
#define MRL_DIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------
 * Per-kernel-class timing for benchmarks.  When enabled, every kernel launch
 * of the entry points of mrl.h is bracketed by HIP events on the launch stream.
 * mrl_profile_collect synchronises the device, adds up the elapsed time and
 * launch count per class since the last collect, and resets the log.
 * Arrays are HOST memory of MRL_PROF_NCLASS entries.
 * ---------------------------------------------------------------------- */
enum {
  MRL_PROF_PREP = 0,      /* mask scan, compaction, sequence weights, zero fill */
  MRL_PROF_ADV = 1,       /* group advantages */
  MRL_PROF_GEMM_FWD = 2,  /* logits tile GEMM with fused log-sum-exp */
  MRL_PROF_ROW_EPI = 3,   /* partial merge, ratio / clip / KL, loss partials */
  MRL_PROF_CONVERT = 4,   /* operand preparation: row gather, transposes (fp32 path: logits -> dz) */
  MRL_PROF_GEMM_DH = 5,   /* dH = dz W */
  MRL_PROF_GEMM_DW = 6,   /* dW += dz^T H */
  MRL_PROF_FINAL = 7,     /* final reductions */
  MRL_PROF_NCLASS = 8
};
int mrl_profile_enable(int on);
int mrl_profile_collect(double* ms_per_class /*host*/, int64_t* launches_per_class /*host*/);

/* ------------------------------------------------------------------------
 * Diagnostic: sustained rate of the matrix cores on the MFMA instruction the
 * GEMM kernels use (bf16 16x16x32, fp32 accumulate), registers only, no memory
 * traffic.  random_operands = 0: constant operands (clock-limited peak);
 * 1: random sign / mantissa operands, which is what activations and weights
 * look like - the device lowers its clock under the higher switching power, so
 * this is the ceiling of any bf16 GEMM on real data.  Benchmarks print both
 * next to the published peak (Sec. 3 defines the contraction this bounds).
 * Synchronous: runs on the null stream for about `seconds` (0 < seconds <= 5)
 * and waits.  scratch: device memory, at least 1024 bytes per compute unit
 * (512 KiB is enough for any device); out_tflops: host.  Errors: MRL_ERR_NULL,
 * MRL_ERR_CONFIG (seconds), MRL_ERR_WORKSPACE (scratch too small), MRL_ERR_DEVICE.
 * ---------------------------------------------------------------------- */
int mrl_probe_mfma_rate(int32_t random_operands, double seconds, void* scratch /*dev*/,
                        size_t scratch_bytes, double* out_tflops /*host*/);

/* ------------------------------------------------------------------------
 * The launch plan of the dW GEMM for an LM head of V rows and d columns (host
 * code only, no GPU call): which rows of 256 x 256 tiles are cut into slices of
 * the contraction at the end of the launch, into how many, and how many of the
 * resulting work items each of the 8 XCDs takes.  For tests of the host logic
 * and for reading profiles.  out12 (host): [0] first tile row of the tail,
 * [1] tile rows in the tail, [2] slices per tile (0: the tiles stay whole),
 * [3 + x], x = 0..8: items before XCD x (so [11] is the item count).
 * Errors: MRL_ERR_NULL, MRL_ERR_SHAPE (V or d not positive).
 * ---------------------------------------------------------------------- */
int mrl_diag_dw_tail_plan(int32_t V, int32_t d, int32_t* out12 /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* MRL_DIAG_H */
