// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace mrl {

// Column padding of the per-chunk logit / dz buffers: the vocabulary is padded
// to a multiple of the GEMM tile so that inner kernels never see a ragged K.
constexpr int kTile = 256;
inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// A kernel that asks for more than 64 KB of dynamic LDS needs its limit raised first; the
// attribute belongs to the (kernel, device) pair, so it is set once on every device used.
struct LdsLimit {
  std::atomic<bool> done[64] = {};
  void ensure(const void* kernel, int bytes) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && done[dev].load(std::memory_order_acquire)) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (tracked) done[dev].store(true, std::memory_order_release);
  }
};

// Number of sum-exp partials each token row receives from the forward kernel: the bf16
// kernel emits two per 256-wide vocabulary tile (one per wave row), the fp32 path a single
// (max, sum-exp) pair per row.
inline int fwd_partials_bf16(int V) { return 2 * (int)((V + kTile - 1) / kTile); }

// bf16 path: exponentials are taken relative to a per-row offset that is known before the forward
// launch, c2[n] = z_t[n] * log2(e) + kStashMargin2 (log2 domain, z_t = the row's target logit):
//   e[n, v] = 2^(min(z[n, v] * log2(e) - c2[n], kStashClamp2)),   S[n] = sum_v e[n, v].
// One offset for the whole row is what lets the forward kernel write e itself (as bf16) for the
// backward pass: softmax = e / S, so dz = g (onehot - e / S) = (-g / S) (e - S onehot) is the
// stored row, patched at the target column, times a per-row scalar that the dH epilogue applies
// to its output rows and that the dW launch finds folded into its copy of the hidden rows.
// Relative to the target logit nothing of weight can underflow (e >= p * 2^-margin) and the
// largest entry is exp(-logp_target) * 2^-margin.  With margin 60 and clamp 100 every quantity
// stays a normal bf16 / fp32 number for log-probs of the target down to about -97; below that
// the row saturates (finite, inexact) and is counted.
constexpr float kStashMargin2 = 60.f;
constexpr float kStashClamp2 = 100.f;
constexpr float kSaturatedLogp = -97.f;

// ---- bf16 MFMA GEMM family: C[m][n] = sum_k A[m][k] * B[n][k] ---------------
// n_scored: device pointer to the number of compacted rows; chunk_start/chunk_rows
// select the rows this launch covers (valid rows = clamp(n_scored - chunk_start, 0, chunk_rows)).

// Forward: A = W [V, k_len] (row stride ldw), B = Hc [chunk_rows, k_len] (row stride ldh): the
// launch's token rows, gathered and contiguous; k_len = d rounded up to 128, the columns beyond d
// zero in both operands; zt[chunk_start + n] is the row's target logit.  Writes per-row partials part_sum[(2*tile_m + wave_m) * part_stride + n]
// = sum of e[n, v] over the partial's 128 vocabulary rows (e as defined above), when part_ez != nullptr
// also sum e * z (for the entropy), and, when estash != nullptr, e itself as bf16 into
// estash[n * lde + v] (n = row within this launch; columns V .. round_up(V, 256) get zeros).
void launch_gemm_fwd_bf16(const void* W, int64_t ldw, const void* Hc, int64_t ldh, int k_len, const float* zt,
                          const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                          int V, int d, float* part_sum, float* part_ez,
                          int64_t part_stride, void* estash, int64_t lde, hipStream_t stream);

// dH: A = E [chunk_rows, Vp] (the patched bf16 stash), B = Wt [d, Vp]; row m, multiplied by
// row_scale[chunk_start + m], goes to dH[row_index[chunk_start + m], :] as bf16 (dh_f32 = 0) or
// float (dh_f32 = 1).
void launch_gemm_dh_bf16(const void* E, int64_t lde, const void* Wt, int64_t ldwt,
                         const int32_t* row_index, const float* row_scale, const int64_t* n_scored,
                         int64_t chunk_start, int chunk_rows, int Vp, int d, void* dH, int dh_f32,
                         hipStream_t stream);

// dW: A = E^T read in place from E [chunk_rows, Vp] (rows >= valid rows rounded up to 128 and
// columns >= V must be zero), B = Ht [d, chunk_rows] (the pass's hidden rows, each already
// multiplied by its row scale); dW[v, :] = (or +=) sum over the chunk's valid rows.
// overwrite = 1 stores, 0 adds into the existing values.
// tail_part: scratch of gemm_dw_tail_bytes() bytes for the K-split tail tiles (nullptr: the
// ragged last rows of tiles run as whole tiles).
size_t gemm_dw_tail_bytes();
void launch_gemm_dw_bf16(const void* P, int64_t ldp, const void* Ht, int64_t ldht,
                         const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                         int V, int d, float* dW, int overwrite, float* tail_part, hipStream_t stream);

// ---- fp32 plain GEMM (sanity path): C[m][n] = sum_k A[m][k] * B[n][k] --------
// a_rows / c_rows: optional row maps (index arrays already offset to the chunk);
// m_valid is computed on the device from n_scored when m_dynamic != 0, and
// k_valid likewise when k_dynamic != 0.
struct GemmF32Args {
  const float* A; int64_t lda; const int32_t* a_rows;
  const float* B; int64_t ldb;
  float* C; int64_t ldc; const int32_t* c_rows;
  int M, N, K;
  const int64_t* n_scored; int64_t chunk_start; int chunk_rows;
  int m_dynamic, k_dynamic;
  int accumulate;
};
void launch_gemm_f32(const GemmF32Args& a, hipStream_t stream);

// ---- auxiliary kernels ------------------------------------------------------
struct PrepOut {
  int32_t* row_index;   // [N] compacted scored slots, in slot order; tail filled with 0
  int64_t* n_scored;    // [1]
  int64_t* n_bad;       // [1] masked-in slots with a target outside [0, V)
  int32_t* block_counts; // scratch: per 1024-slot block a scored count and a bad-target count (int32),
                         // followed, 8-byte aligned, by the blocks' exclusive offsets (int64)
};
void launch_prep(const uint8_t* mask, const int32_t* targets, int64_t N, int V, const PrepOut& o,
                 hipStream_t stream);

// Per-sequence scored length (valid targets only) and loss weights.
// seq_coef[b] = 1 / (P K_g L_b) for GRPO rows, lambda / (S_aux L_b) for SGT rows
// (sign and lambda folded so that g = seq_coef * (...)), 0 for empty rows.
void launch_seq_weights(const uint8_t* mask, const int32_t* targets, const int32_t* group_id,
                        const uint8_t* seq_kind, int64_t B, int T, int G, int V, int loss_agg,
                        int32_t* seq_len, float* seq_coef, int32_t* group_count /*[G] scratch*/,
                        int64_t* n_bad_groups /*[1]: sequences whose group id is outside [0, G)*/,
                        hipStream_t stream);

// Response-level log-ratio (App. I.1): seq_expo[b] = sum over the scored tokens of sequence b of
// (logp - behav_logp), divided by the number of scored tokens when level == 2.  Fixed-order
// reduction, one workgroup per sequence.
void launch_seq_log_ratio(const uint8_t* mask, const int32_t* targets, const float* logp,
                          const float* behav_logp, int64_t B, int T, int V, int level, float* seq_expo,
                          hipStream_t stream);

// Zero out_logp (and out_lse, dH rows) of unscored slots.
void launch_zero_unscored(const uint8_t* mask, const int32_t* targets, int64_t N, int V, int d,
                          float* out_logp, float* out_lse, void* dH, int dh_elem_bytes,
                          hipStream_t stream);

// Target logit z_t[i] = <H[row_index[i]], W[target]> for compacted rows (fp32 accumulate).
void launch_target_logit(const void* H, const void* W, const int32_t* targets,
                         const int32_t* row_index, const int64_t* n_scored, int64_t N_max,
                         int d, int is_bf16, float* zt, hipStream_t stream);

// fp32 path: (max, sum-exp[, sum exp * z]) of each row of Z [rows, V] -> one partial per row.
void launch_row_lse_f32(const float* Z, int64_t ldz, const int64_t* n_scored, int64_t chunk_start,
                        int chunk_rows, int V, float* part_max, float* part_sum, float* part_ez,
                        hipStream_t stream);

struct RowEpiArgs {
  // part_max == nullptr: part_sum holds the bf16 kernel's offset sums (see kStashMargin2);
  // else (fp32 path) one (max, sum exp(z - max)) pair per row
  const float* part_max; const float* part_sum; int n_partials; int chunk_rows;
  const float* part_ez; float* out_entropy;   // both nullptr unless the entropy is asked for (per slot)
  const float* zt;            // [N] compacted
  const int32_t* row_index; const int64_t* n_scored; int64_t chunk_start;
  // loss inputs (all nullptr for the log-prob-only entry point)
  const float* behav_logp; const float* ref_logp; const float* seq_adv;
  const float* seq_coef; const uint8_t* seq_kind; int T;
  // response-level ratio (App. I.1): exponent per sequence, lengths, level 1 (sum) or 2 (mean); null = token ratio
  const float* seq_expo; const int32_t* seq_len; int ratio_level;
  float eps_lo, eps_hi, beta, lambda;
  float* out_logp; float* out_lse;  // per slot
  float* lse_c; float* g_c;         // per compacted row (nullptr to skip)
  // bf16 backward: row_scale[ci] = -g / S, and the stash row's target column becomes e - S
  float* row_scale; uint16_t* estash; int64_t lde; const int32_t* targets;
  double* loss_partials;            // [n_blocks_total][8], block index = chunk block offset + blockIdx
  int64_t partial_block_offset;
};
int row_epilogue_blocks(int chunk_rows);
void launch_row_epilogue(const RowEpiArgs& a, hipStream_t stream);

// fp32 path, dz conversion: reads the chunk's float logits, writes P[i][v] = g_i (1[v = y_i] -
// exp(z - lse_i)) in place and its transpose Pt[v][i].
void launch_convert_f32(float* ZP, int64_t ldz, float* Pt, int64_t ldpt, const float* lse_c,
                        const float* g_c, const int32_t* targets, const int32_t* row_index,
                        const int64_t* n_scored, int64_t chunk_start, int chunk_rows, int V,
                        hipStream_t stream);

// bf16 path: zeroes the stash rows from the pass's valid count up to its multiple of 128 (the dW
// contraction runs over pairs of 64-row panels; the forward kernel writes valid rows only).
void launch_zero_stash_tail(void* estash, int64_t lde, const int64_t* n_scored, int64_t chunk_start,
                            int chunk_rows, int Vp, hipStream_t stream);

// bf16 path: Out[r][0:dp] = In[rows[r]][0:d], zero in [d, dp) (rows == nullptr: identity), for
// r < valid rows of the chunk (n_scored != nullptr) or r < n_rows_static.  16-byte vectors: d, dp,
// both row strides multiples of 8 elements.
void launch_gather_rows_b16(const void* in, int64_t ld_in, const int32_t* rows, void* out, int64_t ld_out,
                            int64_t n_rows_static, const int64_t* n_scored, int64_t chunk_start,
                            int chunk_rows, int d, int dp, hipStream_t stream);

// Out[c][r] = scale[r] * In[rows[r]][c] (rows == nullptr: identity; scale == nullptr: 1, 2-byte
// elements only) for r < n_rows_valid, zero beyond, r in [0, out_cols_pad), c in [0, n_cols).
// Used for Wt (static) and Ht (gathered, dynamic, scaled).
void launch_transpose(const void* in, int64_t ld_in, const int32_t* rows, const float* scale, void* out, int64_t ld_out,
                      int64_t n_rows_static, const int64_t* n_scored, int64_t chunk_start,
                      int chunk_rows, int n_cols, int64_t out_cols_pad, int elem_bytes,
                      hipStream_t stream);

// Group-relative advantages (Sec. 3) with pooled / own statistics and SGT gate flags.
void launch_group_advantages(const float* rewards, const int32_t* group_id, const uint8_t* in_stats,
                             const uint8_t* scored, const uint8_t* is_own, const float* baseline_shift,
                             int64_t B, int G, int mode, float eps_norm, int ddof, float mix_alpha, float neg_thresh,
                             float pos_thresh, float* out_adv, float* out_mean, float* out_std,
                             uint8_t* out_flags, hipStream_t stream);

// rows_enqueued: number of compacted rows covered by the enqueued passes; scored rows beyond
// it (a wrong scored_rows_hint) get NaN log-probs and are counted in the stats.
void launch_finalize(const double* loss_partials, int64_t n_blocks, const int64_t* n_scored,
                     const int64_t* n_bad, float beta, float lambda, int64_t rows_enqueued,
                     const int32_t* row_index, float* out_logp, void* out_stats, hipStream_t stream);

// MRL_OK when the current device is a gfx950, else MRL_ERR_UNSUPPORTED_ARCH / MRL_ERR_DEVICE.
int require_gfx950();

// ---- profiling ---------------------------------------------------------------
void prof_begin(int cls, hipStream_t stream);
void prof_end(int cls, hipStream_t stream);

}  // namespace mrl
