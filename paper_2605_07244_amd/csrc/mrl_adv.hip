// Group-relative advantages (Sec. 3), pool-wide (Sec. 5.1) and pooled-baseline
// (App. I.1) variants, and the SGT gate flags (Sec. 5.3 / App. B).
//
// One wavefront per group scans all B entries (B is a few thousand: the whole
// input is a few KB and stays in L2), so group members need not be contiguous
// and every sum has a fixed order: lane-strided partial sums in fp64, then a
// fixed butterfly.  Mean and variance are taken in two passes so that binary
// rewards give exact zeros for all-equal groups.
#include "mrl_internal.h"

namespace mrl {
namespace {

__device__ inline double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ inline int wave_sum_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

struct AdvArgs {
  const float* rewards; const int32_t* group_id;
  const uint8_t* in_stats; const uint8_t* scored; const uint8_t* is_own; const float* baseline_shift;
  int64_t B; int G; int mode; float eps_norm; int ddof; float mix_alpha;
  float neg_thresh, pos_thresh;
  float* out_adv; float* out_mean; float* out_std; uint8_t* out_flags;
};

__global__ __launch_bounds__(256) void k_group_adv(AdvArgs a) {
  const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= a.G) return;
  const int lane = threadIdx.x & 63;
  // pass 1: counts, sums, gate predicates
  double sum_p = 0.0, sum_o = 0.0;
  int cnt_p = 0, cnt_o = 0, n_own = 0, own_not_fail = 0, peer_succ = 0;
  for (int64_t b = lane; b < a.B; b += 64) {
    if (a.group_id[b] != g) continue;
    const float r = a.rewards[b];
    const bool st = a.in_stats == nullptr || a.in_stats[b] != 0;
    const bool own = a.is_own == nullptr || a.is_own[b] != 0;
    if (st) { sum_p += (double)r; cnt_p++; if (own) { sum_o += (double)r; cnt_o++; } }
    if (own) { n_own++; own_not_fail += !(r < a.neg_thresh); }
    else peer_succ += (r > a.pos_thresh);
  }
  sum_p = wave_sum(sum_p); sum_o = wave_sum(sum_o);
  cnt_p = wave_sum_i(cnt_p); cnt_o = wave_sum_i(cnt_o);
  n_own = wave_sum_i(n_own); own_not_fail = wave_sum_i(own_not_fail); peer_succ = wave_sum_i(peer_succ);
  const double mu_p = cnt_p > 0 ? sum_p / cnt_p : 0.0;
  const double mu_o = cnt_o > 0 ? sum_o / cnt_o : 0.0;
  // pass 2: squared deviations
  double sq_p = 0.0, sq_o = 0.0;
  for (int64_t b = lane; b < a.B; b += 64) {
    if (a.group_id[b] != g) continue;
    const bool st = a.in_stats == nullptr || a.in_stats[b] != 0;
    if (!st) continue;
    const bool own = a.is_own == nullptr || a.is_own[b] != 0;
    const double r = (double)a.rewards[b];
    sq_p += (r - mu_p) * (r - mu_p);
    if (own) sq_o += (r - mu_o) * (r - mu_o);
  }
  sq_p = wave_sum(sq_p); sq_o = wave_sum(sq_o);
  const double sd_p = cnt_p - a.ddof > 0 ? sqrt(sq_p / (cnt_p - a.ddof)) : 0.0;
  const double sd_o = cnt_o - a.ddof > 0 ? sqrt(sq_o / (cnt_o - a.ddof)) : 0.0;
  // pass 3: advantages
  const bool zn = a.mode == 1;
  const double eps = (double)a.eps_norm, alpha = (double)a.mix_alpha;
  // perturbed-baseline control (App. C.4): the shift moves the baseline, not the std
  const double shift = a.baseline_shift != nullptr ? (double)a.baseline_shift[g] : 0.0;
  const double bl_p = mu_p + shift, bl_o = mu_o + shift;
  for (int64_t b = lane; b < a.B; b += 64) {
    if (a.group_id[b] != g) continue;
    const bool sc = a.scored == nullptr || a.scored[b] != 0;
    double adv = 0.0;
    if (sc) {
      const double r = (double)a.rewards[b];
      const double ap = cnt_p > 0 ? (zn ? (r - bl_p) / (sd_p + eps) : r - bl_p) : 0.0;
      if (a.mix_alpha == 1.0f) {
        adv = ap;
      } else {
        const double ao = cnt_o > 0 ? (zn ? (r - bl_o) / (sd_o + eps) : r - bl_o) : 0.0;
        adv = (1.0 - alpha) * ao + alpha * ap;
      }
    }
    a.out_adv[b] = (float)adv;
  }
  if (lane == 0) {
    if (a.out_mean) a.out_mean[g] = (float)mu_p;
    if (a.out_std) a.out_std[g] = (float)sd_p;
    if (a.out_flags) {
      const bool all_fail = n_own > 0 && own_not_fail == 0;
      const bool ps = peer_succ > 0;
      a.out_flags[g] = (uint8_t)((all_fail ? 1u : 0u) | (ps ? 2u : 0u) | ((all_fail && ps) ? 4u : 0u));
    }
  }
}

// entries whose group id is outside [0, G) are owned by no wavefront: clear them first
__global__ __launch_bounds__(256) void k_adv_clear_orphans(const int32_t* group_id, int64_t B, int G,
                                                           float* out_adv) {
  const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b < B && (group_id[b] < 0 || group_id[b] >= G)) out_adv[b] = 0.f;
}

// batch normalisation (App. A): divide the group-centred advantages of scored,
// in-range entries by their std over the batch (+ eps); single block, fixed order.
__global__ __launch_bounds__(1024) void k_adv_batch_scale(const int32_t* group_id, const uint8_t* scored,
                                                         int64_t B, int G, float eps_norm, int ddof,
                                                         float* adv) {
  __shared__ double sh[1024];
  __shared__ long long shc[1024];
  __shared__ double mean_s, sd_s;
  double s = 0.0; long long c = 0;
  for (int64_t b = threadIdx.x; b < B; b += 1024) {
    const bool sc = (scored == nullptr || scored[b] != 0) && group_id[b] >= 0 && group_id[b] < G;
    if (sc) { s += (double)adv[b]; c++; }
  }
  sh[threadIdx.x] = s; shc[threadIdx.x] = c;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) { sh[threadIdx.x] += sh[threadIdx.x + off]; shc[threadIdx.x] += shc[threadIdx.x + off]; }
    __syncthreads();
  }
  const long long cnt = shc[0];
  if (threadIdx.x == 0) mean_s = cnt > 0 ? sh[0] / (double)cnt : 0.0;
  __syncthreads();
  const double mu = mean_s;
  double q = 0.0;
  for (int64_t b = threadIdx.x; b < B; b += 1024) {
    const bool sc = (scored == nullptr || scored[b] != 0) && group_id[b] >= 0 && group_id[b] < G;
    if (sc) { const double dlt = (double)adv[b] - mu; q += dlt * dlt; }
  }
  __syncthreads();
  sh[threadIdx.x] = q;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) sd_s = cnt - ddof > 0 ? sqrt(sh[0] / (double)(cnt - ddof)) : 0.0;
  __syncthreads();
  const double denom = sd_s + (double)eps_norm;
  for (int64_t b = threadIdx.x; b < B; b += 1024) {
    const bool sc = (scored == nullptr || scored[b] != 0) && group_id[b] >= 0 && group_id[b] < G;
    if (sc) adv[b] = (float)((double)adv[b] / denom);
  }
}

}  // namespace

void launch_group_advantages(const float* rewards, const int32_t* group_id, const uint8_t* in_stats,
                             const uint8_t* scored, const uint8_t* is_own, const float* baseline_shift,
                             int64_t B, int G, int mode, float eps_norm, int ddof, float mix_alpha, float neg_thresh,
                             float pos_thresh, float* out_adv, float* out_mean, float* out_std,
                             uint8_t* out_flags, hipStream_t stream) {
  AdvArgs a = {rewards, group_id, in_stats, scored, is_own, baseline_shift, B, G, mode, eps_norm, ddof, mix_alpha,
               neg_thresh, pos_thresh, out_adv, out_mean, out_std, out_flags};
  hipLaunchKernelGGL(k_adv_clear_orphans, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, stream, group_id, B,
                     G, out_adv);
  hipLaunchKernelGGL(k_group_adv, dim3((G + 3) / 4), dim3(256), 0, stream, a);
  if (mode == 2)
    hipLaunchKernelGGL(k_adv_batch_scale, dim3(1), dim3(1024), 0, stream, group_id, scored, B, G, eps_norm,
                       ddof, out_adv);
}

}  // namespace mrl
