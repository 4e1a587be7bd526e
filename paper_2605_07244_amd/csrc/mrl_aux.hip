// Memory-bound kernels of the scoring path: mask compaction, sequence weights,
// target logits, partial-merge + token-loss epilogue (Eq. 1 / Eq. 2 terms), operand
// transposes, the fp32 path's logits -> dz conversion, final reductions.
#include "mrl_internal.h"

namespace mrl {
namespace {

__device__ inline bool slot_valid(const uint8_t* mask, const int32_t* targets, int64_t n, int V) {
  const bool m = mask == nullptr || mask[n] != 0;
  const int32_t y = targets[n];
  return m && y >= 0 && y < V;
}

__device__ inline int valid_rows(const int64_t* n_scored, int64_t chunk_start, int chunk_rows) {
  const int64_t r = *n_scored - chunk_start;
  return r < 0 ? 0 : (r > chunk_rows ? chunk_rows : (int)r);
}

// ----------------------------------------------------------------------------
// Compaction of scored slots (order preserving): count, scan, fill.
// ----------------------------------------------------------------------------
constexpr int PREP_PER_THREAD = 4;
constexpr int PREP_BLOCK = 256;
constexpr int PREP_PER_BLOCK = PREP_PER_THREAD * PREP_BLOCK;

__device__ inline int block_exclusive_scan(int val, int* total) {
  // 256 threads; returns the exclusive prefix of val, *total = block sum.
  __shared__ int wave_sums[4];
  __shared__ int wave_off[5];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = val;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int w = 0; w < 4; ++w) { wave_off[w] = run; run += wave_sums[w]; }
    wave_off[4] = run;
  }
  __syncthreads();
  *total = wave_off[4];
  const int res = wave_off[wave] + incl - val;
  __syncthreads();
  return res;
}

__global__ __launch_bounds__(PREP_BLOCK) void k_prep_count(const uint8_t* mask, const int32_t* targets,
                                                          int64_t N, int V, int32_t* block_counts,
                                                          int64_t nblocks) {
  const int64_t base = (int64_t)blockIdx.x * PREP_PER_BLOCK + threadIdx.x * PREP_PER_THREAD;
  int cnt = 0, bad = 0;
#pragma unroll
  for (int k = 0; k < PREP_PER_THREAD; ++k) {
    const int64_t n = base + k;
    if (n < N) {
      const bool m = mask == nullptr || mask[n] != 0;
      const int32_t y = targets[n];
      const bool ok = y >= 0 && y < V;
      cnt += (m && ok);
      bad += (m && !ok);
    }
  }
  int tot_c, tot_b;
  block_exclusive_scan(cnt, &tot_c);
  block_exclusive_scan(bad, &tot_b);
  if (threadIdx.x == 0) {
    block_counts[blockIdx.x] = tot_c;
    block_counts[nblocks + blockIdx.x] = tot_b;
  }
}

__global__ __launch_bounds__(1024) void k_prep_scan(int32_t* block_counts, int64_t nblocks,
                                                   int64_t* block_offsets, int64_t* n_scored,
                                                   int64_t* n_bad) {
  // single block: exclusive scan of block_counts[0..nblocks) into block_offsets (int64)
  __shared__ int64_t sh[1024];
  __shared__ int64_t carry, bad_total;
  if (threadIdx.x == 0) { carry = 0; bad_total = 0; }
  __syncthreads();
  for (int64_t base = 0; base < nblocks; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const int64_t v = i < nblocks ? block_counts[i] : 0;
    const int64_t b = i < nblocks ? block_counts[nblocks + i] : 0;
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const int64_t t = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
      __syncthreads();
      sh[threadIdx.x] += t;
      __syncthreads();
    }
    if (i < nblocks) block_offsets[i] = carry + sh[threadIdx.x] - v;
    __syncthreads();
    const int64_t chunk_total = sh[1023];
    // reuse sh for the bad-target sum
    __syncthreads();
    sh[threadIdx.x] = b;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
      if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
      __syncthreads();
    }
    if (threadIdx.x == 0) { carry += chunk_total; bad_total += sh[0]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { *n_scored = carry; *n_bad = bad_total; }
}

__global__ __launch_bounds__(PREP_BLOCK) void k_prep_fill(const uint8_t* mask, const int32_t* targets,
                                                         int64_t N, int V, const int64_t* block_offsets,
                                                         const int64_t* n_scored, int32_t* row_index) {
  const int64_t base = (int64_t)blockIdx.x * PREP_PER_BLOCK + threadIdx.x * PREP_PER_THREAD;
  bool ok[PREP_PER_THREAD];
  int cnt = 0;
#pragma unroll
  for (int k = 0; k < PREP_PER_THREAD; ++k) {
    const int64_t n = base + k;
    ok[k] = n < N && slot_valid(mask, targets, n, V);
    cnt += ok[k];
  }
  int total;
  const int excl = block_exclusive_scan(cnt, &total);
  int64_t pos = block_offsets[blockIdx.x] + excl;
  const int64_t ns = *n_scored;
#pragma unroll
  for (int k = 0; k < PREP_PER_THREAD; ++k) {
    const int64_t n = base + k;
    if (ok[k]) row_index[pos++] = (int32_t)n;
    if (n < N && n >= ns) row_index[n] = 0;   // tail entries: a harmless valid slot
  }
}

// ----------------------------------------------------------------------------
// Sequence lengths and the aggregation weights of Eq. (1) / Eq. (2).
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_seq_len(const uint8_t* mask, const int32_t* targets, int T,
                                                 int V, int32_t* seq_len) {
  const int64_t b = blockIdx.x;
  int cnt = 0;
  for (int t = threadIdx.x; t < T; t += 256) cnt += slot_valid(mask, targets, b * T + t, V);
  int total;
  block_exclusive_scan(cnt, &total);
  if (threadIdx.x == 0) seq_len[b] = total;
}

__global__ __launch_bounds__(1024) void k_seq_coef(const int32_t* seq_len, const int32_t* group_id,
                                                  const uint8_t* seq_kind, int64_t B, int G,
                                                  int loss_agg, int32_t* group_count, float* seq_coef,
                                                  int64_t* n_bad_groups) {
  __shared__ long long sh_a[1024];
  __shared__ long long sh_b[1024];
  __shared__ long long tot_aux, tot_tok, tot_groups;
  for (int g = threadIdx.x; g < G; g += 1024) group_count[g] = 0;
  __threadfence();
  __syncthreads();
  long long aux = 0, tok = 0;
  for (int64_t b = threadIdx.x; b < B; b += 1024) {
    const int kind = seq_kind ? seq_kind[b] : 0;
    const int L = seq_len[b];
    const int g = group_id[b];
    if (kind == 0) {
      if (g >= 0 && g < G) { atomicAdd(&group_count[g], 1); tok += L; }
    } else {
      aux += (L > 0);
    }
  }
  sh_a[threadIdx.x] = aux; sh_b[threadIdx.x] = tok;
  __threadfence();
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) { sh_a[threadIdx.x] += sh_a[threadIdx.x + off]; sh_b[threadIdx.x] += sh_b[threadIdx.x + off]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { tot_aux = sh_a[0]; tot_tok = sh_b[0]; }
  __syncthreads();
  long long ng = 0;
  for (int g = threadIdx.x; g < G; g += 1024) ng += (group_count[g] > 0);
  sh_a[threadIdx.x] = ng;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh_a[threadIdx.x] += sh_a[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) tot_groups = sh_a[0];
  __syncthreads();
  // sequences whose group id is out of range (they get weight 0 below)
  long long nbad = 0;
  for (int64_t b = threadIdx.x; b < B; b += 1024) nbad += (group_id[b] < 0 || group_id[b] >= G);
  sh_b[threadIdx.x] = nbad;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh_b[threadIdx.x] += sh_b[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *n_bad_groups = sh_b[0];
  const double P = (double)tot_groups, S = (double)tot_aux, NT = (double)tot_tok;
  for (int64_t b = threadIdx.x; b < B; b += 1024) {
    const int kind = seq_kind ? seq_kind[b] : 0;
    const int L = seq_len[b];
    const int g = group_id[b];
    double c = 0.0;
    if (L > 0) {
      if (kind == 0) {
        if (g >= 0 && g < G) c = loss_agg == 1 ? 1.0 / NT : 1.0 / (P * (double)group_count[g] * (double)L);
      } else {
        c = 1.0 / (S * (double)L);
      }
    }
    seq_coef[b] = (float)c;
  }
}

// ----------------------------------------------------------------------------
// Response-level log-ratio: one workgroup per sequence, fp64 partial sums, fixed order.
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_seq_log_ratio(const uint8_t* mask, const int32_t* targets,
                                                       const float* logp, const float* behav, int T, int V,
                                                       int level, float* seq_expo) {
  __shared__ double sh[256];
  __shared__ int shn[256];
  const int64_t b = blockIdx.x;
  double acc = 0.0;
  int cnt = 0;
  for (int t = threadIdx.x; t < T; t += 256) {
    const int64_t n = b * T + t;
    if (slot_valid(mask, targets, n, V)) { acc += (double)logp[n] - (double)behav[n]; ++cnt; }
  }
  sh[threadIdx.x] = acc;
  shn[threadIdx.x] = cnt;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) { sh[threadIdx.x] += sh[threadIdx.x + off]; shn[threadIdx.x] += shn[threadIdx.x + off]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) seq_expo[b] = (float)(level == 2 ? (shn[0] > 0 ? sh[0] / shn[0] : 0.0) : sh[0]);
}

// ----------------------------------------------------------------------------
// Zero the outputs of unscored slots.
// ----------------------------------------------------------------------------
constexpr int ZERO_SLOTS_PER_BLOCK = 16;
__global__ __launch_bounds__(256) void k_zero_unscored(const uint8_t* mask, const int32_t* targets,
                                                       int64_t N, int V, int64_t row_bytes,
                                                       float* out_logp, float* out_lse,
                                                       unsigned char* dH) {
  const int64_t first = (int64_t)blockIdx.x * ZERO_SLOTS_PER_BLOCK;
  for (int s = 0; s < ZERO_SLOTS_PER_BLOCK; ++s) {
    const int64_t n = first + s;
    if (n >= N) return;
    if (slot_valid(mask, targets, n, V)) continue;
    if (threadIdx.x == 0) {
      if (out_logp) out_logp[n] = 0.f;
      if (out_lse) out_lse[n] = 0.f;
    }
    if (dH) {
      unsigned char* row = dH + n * row_bytes;
      if ((row_bytes & 15) == 0) {
        uint4 z = make_uint4(0, 0, 0, 0);
        for (int64_t o = threadIdx.x * 16; o < row_bytes; o += 256 * 16) *reinterpret_cast<uint4*>(row + o) = z;
      } else {
        for (int64_t o = threadIdx.x * 4; o < row_bytes; o += 256 * 4) *reinterpret_cast<uint32_t*>(row + o) = 0u;
      }
    }
  }
}

// ----------------------------------------------------------------------------
// Target logit z_t[i] = <H[slot_i], W[y_i]>, one wavefront per compacted row.
// ----------------------------------------------------------------------------
__device__ inline float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <bool BF16>
__global__ __launch_bounds__(256) void k_target_logit(const void* H, const void* W, const int32_t* targets,
                                                      const int32_t* row_index, const int64_t* n_scored,
                                                      int d, float* zt) {
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= *n_scored) return;
  const int lane = threadIdx.x & 63;
  const int64_t slot = row_index[i];
  const int64_t y = targets[slot];
  float acc = 0.f;
  if (BF16) {
    const uint4* h = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(H) + slot * d);
    const uint4* w = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(W) + y * d);
    for (int c = lane; c < d / 8; c += 64) {
      const uint4 a = h[c], b = w[c];
      const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc = fmaf(bf16_bits_to_float(av[q] & 0xffffu), bf16_bits_to_float(bv[q] & 0xffffu), acc);
        acc = fmaf(bf16_bits_to_float(av[q] >> 16), bf16_bits_to_float(bv[q] >> 16), acc);
      }
    }
  } else {
    const float* h = static_cast<const float*>(H) + slot * d;
    const float* w = static_cast<const float*>(W) + y * d;
    for (int c = lane; c < d; c += 64) acc = fmaf(h[c], w[c], acc);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) zt[i] = acc;
}

// ----------------------------------------------------------------------------
// fp32 path: one (max, sum-exp) partial per row of the materialised chunk logits.
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_row_lse_f32(const float* Z, int64_t ldz, const int64_t* n_scored,
                                                     int64_t chunk_start, int chunk_rows, int V,
                                                     float* part_max, float* part_sum, float* part_ez) {
  const int i = blockIdx.x;
  if (i >= valid_rows(n_scored, chunk_start, chunk_rows)) return;
  __shared__ float sh[256];
  const float* z = Z + (int64_t)i * ldz;
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  sh[threadIdx.x] = mx;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] = fmaxf(sh[threadIdx.x], sh[threadIdx.x + off]);
    __syncthreads();
  }
  mx = sh[0];
  __syncthreads();
  float s = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) s += expf(z[v] - mx);
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) { part_max[i] = mx; part_sum[i] = sh[0]; }
  if (part_ez == nullptr) return;
  __syncthreads();
  float t = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) t += expf(z[v] - mx) * z[v];
  sh[threadIdx.x] = t;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) part_ez[i] = sh[0];
}

// ----------------------------------------------------------------------------
// Row epilogue: merge partials -> lse, log-prob; Eq. (1) token terms; loss partials; for the
// bf16 backward the row scale -g / S and the patch of the stash's target column.
// Block = 64 rows x 4 partial lanes.
// ----------------------------------------------------------------------------
constexpr int EPI_ROWS = 64;
constexpr int EPI_NQ = 10;   // doubles per block in loss_partials
// loss_partials layout per block: 0 pg, 1 kl, 2 sgt, 3 sum_ratio, 4 max_ratio, 5 sum_k3,
// 6 n_clipped, 7 n_zero_grad, 8 n_grpo_tokens, 9 n_saturated_rows

__global__ __launch_bounds__(256) void k_row_epilogue(RowEpiArgs a) {
  __shared__ float sh_m[4][EPI_ROWS];
  __shared__ float sh_s[4][EPI_ROWS];
  __shared__ double sh_q[EPI_ROWS];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int nvalid = valid_rows(a.n_scored, a.chunk_start, a.chunk_rows);
  const int i = blockIdx.x * EPI_ROWS + tx;           // row within the chunk
  const bool live = i < nvalid;
  const bool offset_sums = a.part_max == nullptr;     // bf16 kernel: sums of 2^(z log2e - c2)

  float mx = 0.f;
  if (!offset_sums) {
    mx = -INFINITY;
    if (live)
      for (int p = ty; p < a.n_partials; p += 4) mx = fmaxf(mx, a.part_max[(int64_t)p * a.chunk_rows + i]);
    sh_m[ty][tx] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(sh_m[0][tx], sh_m[1][tx]), fmaxf(sh_m[2][tx], sh_m[3][tx]));
    __syncthreads();
  }
  float s = 0.f, t = 0.f;
  if (live)
    for (int p = ty; p < a.n_partials; p += 4) {
      const float ps = a.part_sum[(int64_t)p * a.chunk_rows + i];
      float sc = 1.f;
      if (!offset_sums) {
        const float pm = a.part_max[(int64_t)p * a.chunk_rows + i];
        sc = pm == -INFINITY ? 0.f : expf(pm - mx);
      }
      s += ps * sc;
      if (a.part_ez != nullptr) t += a.part_ez[(int64_t)p * a.chunk_rows + i] * sc;
    }
  sh_s[ty][tx] = s;
  sh_m[ty][tx] = t;
  __syncthreads();

  double q[EPI_NQ];
#pragma unroll
  for (int k = 0; k < EPI_NQ; ++k) q[k] = 0.0;
  if (ty == 0 && live) {
    constexpr float LOG2E = 1.4426950408889634f;
    constexpr double LN2 = 0.6931471805599453;
    s = (sh_s[0][tx] + sh_s[1][tx]) + (sh_s[2][tx] + sh_s[3][tx]);
    const int64_t ci = a.chunk_start + i;
    const float zt = a.zt[ci];
    // offset sums: lse = (c2 + log2 S) ln 2 with the very c2 the forward kernel subtracted
    const double lse_d = offset_sums ? ((double)fmaf(zt, LOG2E, kStashMargin2) + log2((double)s)) * LN2
                                     : (double)mx + log((double)s);
    const float lse = (float)lse_d;
    const float logp = (float)((double)zt - lse_d);
    const int64_t slot = a.row_index[ci];
    a.out_logp[slot] = logp;
    if (a.out_lse) a.out_lse[slot] = lse;
    if (a.lse_c) a.lse_c[ci] = lse;
    if (a.part_ez != nullptr) {
      // entropy H = lse - (sum_v e z) / (sum_v e)
      const float tsum = (sh_m[0][tx] + sh_m[1][tx]) + (sh_m[2][tx] + sh_m[3][tx]);
      a.out_entropy[slot] = (float)(lse_d - (double)tsum / (double)s);
    }
    // A target log-prob below the range the bf16 backward operands represent (only possible for a
    // token the learner deems impossible): the row is counted and dropped from the loss and the
    // gradients (weight 0), as a row with an invalid target would be.
    const bool saturated = offset_sums && logp < kSaturatedLogp;
    if (saturated) {
      q[9] = 1.0;
      if (a.g_c) a.g_c[ci] = 0.f;
      if (a.row_scale) a.row_scale[ci] = 0.f;
    }
    if (a.seq_coef != nullptr && !saturated) {
      const int64_t b = slot / a.T;
      const float c = a.seq_coef[b];
      const int kind = a.seq_kind ? a.seq_kind[b] : 0;
      float g;
      if (kind == 0) {
        const float A = a.seq_adv[b];
        // token ratio of Eq. (1), or the response's ratio (App. I.1) whose derivative with
        // respect to each token's log-prob is rho (summed form) or rho / L_b (mean form)
        const float w = a.seq_expo ? expf(a.seq_expo[b]) : expf(logp - a.behav_logp[slot]);
        const float s1 = w * A;
        const float wc = fminf(fmaxf(w, 1.f - a.eps_lo), 1.f + a.eps_hi);
        const float s2 = wc * A;
        const float J = fminf(s1, s2);
        float dJ = s1 <= s2 ? s1 : 0.f;
        if (a.seq_expo && a.ratio_level == 1) dJ *= (float)a.seq_len[b];
        float k3 = 0.f, dk3 = 0.f;
        if (a.ref_logp != nullptr) {
          const float rho = a.ref_logp[slot] - logp;
          const float em1 = expm1f(rho);
          k3 = em1 - rho;
          dk3 = -em1;
        }
        g = c * (-dJ + a.beta * dk3);
        q[0] = -(double)c * (double)J;
        q[1] = (double)c * (double)k3;
        q[3] = (double)w;
        q[4] = (double)w;
        q[5] = (double)k3;
        q[6] = (w < 1.f - a.eps_lo || w > 1.f + a.eps_hi) ? 1.0 : 0.0;
        q[7] = s2 < s1 ? 1.0 : 0.0;
        q[8] = 1.0;
      } else {
        g = -a.lambda * c;
        q[2] = -(double)c * (double)logp;
      }
      if (a.g_c) a.g_c[ci] = g;
      if (a.row_scale) {
        // dz = g (onehot - e / S) = (-g / S) (e - S onehot): the scale, and the one entry of the
        // stash row that differs from e
        a.row_scale[ci] = -g / s;
        uint16_t* cell = a.estash + (int64_t)i * a.lde + a.targets[slot];
        const float e_y = __uint_as_float((uint32_t)*cell << 16);
        const __bf16 patched = (__bf16)(e_y - s);
        uint16_t bits;
        __builtin_memcpy(&bits, &patched, 2);
        *cell = bits;
      }
    }
  }
  if (a.loss_partials == nullptr) return;
  // fixed-order block reduction of the 64 row threads (ty == 0)
  double* out = a.loss_partials + (a.partial_block_offset + blockIdx.x) * EPI_NQ;
  for (int k = 0; k < EPI_NQ; ++k) {
    __syncthreads();
    if (ty == 0) sh_q[tx] = q[k];
    __syncthreads();
    if (threadIdx.x == 0) {
      double acc = 0.0;
      if (k == 4) { for (int r = 0; r < EPI_ROWS; ++r) acc = sh_q[r] > acc ? sh_q[r] : acc; }
      else { for (int r = 0; r < EPI_ROWS; ++r) acc += sh_q[r]; }
      out[k] = acc;
    }
  }
}

__global__ __launch_bounds__(256) void k_finalize(const double* parts, int64_t n_blocks,
                                                  const int64_t* n_scored, const int64_t* n_bad,
                                                  float beta, float lambda, int64_t rows_enqueued,
                                                  const int32_t* row_index, float* out_logp,
                                                  double* out_d, int64_t* out_i) {
  __shared__ double sh[256];
  // rows the enqueued passes did not cover (only when the caller's hint was too small)
  for (int64_t i = rows_enqueued + threadIdx.x; i < *n_scored; i += 256)
    out_logp[row_index[i]] = __builtin_nanf("");
  __shared__ double tot[EPI_NQ];
  for (int k = 0; k < EPI_NQ; ++k) {
    double acc = 0.0;
    for (int64_t b = threadIdx.x; b < n_blocks; b += 256) {
      const double v = parts[b * EPI_NQ + k];
      acc = k == 4 ? (v > acc ? v : acc) : acc + v;
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (threadIdx.x < off) {
        const double o = sh[threadIdx.x + off];
        sh[threadIdx.x] = k == 4 ? (o > sh[threadIdx.x] ? o : sh[threadIdx.x]) : sh[threadIdx.x] + o;
      }
      __syncthreads();
    }
    if (threadIdx.x == 0) tot[k] = sh[0];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double ng = tot[8];
    out_d[0] = tot[0] + (double)beta * tot[1] + (double)lambda * tot[2];
    out_d[1] = tot[0];
    out_d[2] = tot[1];
    out_d[3] = tot[2];
    out_d[4] = ng > 0 ? tot[3] / ng : 0.0;
    out_d[5] = tot[4];
    out_d[6] = ng > 0 ? tot[5] / ng : 0.0;
    out_i[0] = *n_scored;
    out_i[1] = (int64_t)(tot[6] + 0.5);
    out_i[2] = (int64_t)(tot[7] + 0.5);
    out_i[3] = *n_bad;
    out_i[4] = *n_scored > rows_enqueued ? *n_scored - rows_enqueued : 0;
    out_i[5] = (int64_t)(tot[9] + 0.5);
  }
}

// ----------------------------------------------------------------------------
// bf16 path: rows of the stash from the pass's valid count up to its multiple of 128 are cleared
// (the dW contraction runs over pairs of 64-row panels and must not meet stale bits there).
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_zero_stash_tail(uint16_t* E, int64_t lde, const int64_t* n_scored,
                                                         int64_t chunk_start, int chunk_rows, int Vp) {
  const int nvalid = valid_rows(n_scored, chunk_start, chunk_rows);
  const int nzero = (nvalid + 127) / 128 * 128 < chunk_rows ? (nvalid + 127) / 128 * 128 : chunk_rows;
  const int i = nvalid + blockIdx.y;
  if (i >= nzero) return;
  const int v = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (v < Vp) *reinterpret_cast<uint4*>(E + (int64_t)i * lde + v) = make_uint4(0, 0, 0, 0);
}

// ----------------------------------------------------------------------------
// dz conversion of the fp32 path (proof of Prop. 4: grad log pi(a_i) = e_i - pi).
// ----------------------------------------------------------------------------
// fp32 path: scalar, bounds-checked.
__global__ __launch_bounds__(256) void k_convert_f32(float* ZP, int64_t ldz, float* Pt, int64_t ldpt,
                                                     const float* lse_c, const float* g_c,
                                                     const int32_t* targets, const int32_t* row_index,
                                                     const int64_t* n_scored, int64_t chunk_start,
                                                     int chunk_rows, int V) {
  const int nvalid = valid_rows(n_scored, chunk_start, chunk_rows);
  const int i = blockIdx.y;
  if (i >= nvalid) return;
  const int64_t ci = chunk_start + i;
  const float lse = lse_c[ci], g = g_c[ci];
  const int y = targets[row_index[ci]];
  for (int v = blockIdx.x * 256 + threadIdx.x; v < V; v += gridDim.x * 256) {
    const float p = expf(ZP[(int64_t)i * ldz + v] - lse);
    const float val = g * ((v == y ? 1.f : 0.f) - p);
    ZP[(int64_t)i * ldz + v] = val;
    Pt[(int64_t)v * ldpt + i] = val;
  }
}

// ----------------------------------------------------------------------------
// Row gather with zero padding: Out[r][0:dp] = In[rows[r]][0:d] | 0.  Makes the forward launch's
// token-row operand contiguous (no index lookups in the kernel) and its K extent a multiple of
// the kernel's 128-wide panel pairs; the same routine pads W when d is not such a multiple.
// ----------------------------------------------------------------------------
constexpr int GATHER_ROWS = 4;
__global__ __launch_bounds__(256) void k_gather_rows_b16(const uint16_t* in, int64_t ld_in, const int32_t* rows,
                                                         uint16_t* out, int64_t ld_out, int64_t n_rows_static,
                                                         const int64_t* n_scored, int64_t chunk_start,
                                                         int chunk_rows, int d, int dp) {
  int64_t nrows = n_rows_static;
  if (n_scored != nullptr) nrows = valid_rows(n_scored, chunk_start, chunk_rows);
#pragma unroll
  for (int k = 0; k < GATHER_ROWS; ++k) {
    const int64_t r = (int64_t)blockIdx.x * GATHER_ROWS + k;
    if (r >= nrows) return;
    const int64_t src = rows ? (int64_t)rows[r] : r;
    for (int c = threadIdx.x * 8; c < dp; c += 256 * 8) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (c < d) v = *reinterpret_cast<const uint4*>(in + src * ld_in + c);
      *reinterpret_cast<uint4*>(out + r * ld_out + c) = v;
    }
  }
}

// ----------------------------------------------------------------------------
// Transposes.  Out[c][r] = In[rows[r]][c].
// ----------------------------------------------------------------------------
// 2-byte elements, vectorised: tile 64 rows x 64 cols; requires n_cols % 64 == 0,
// 16-byte aligned rows on both sides and out_cols_pad % 64 == 0.
__global__ __launch_bounds__(256) void k_transpose_b16(const uint16_t* in, int64_t ld_in, const int32_t* rows,
                                                       const float* scale /*per row, or nullptr*/,
                                                       uint16_t* out, int64_t ld_out, int64_t n_rows_static,
                                                       const int64_t* n_scored, int64_t chunk_start,
                                                       int chunk_rows) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64 * 72];
  int64_t nrows = n_rows_static;
  if (n_scored != nullptr) nrows = valid_rows(n_scored, chunk_start, chunk_rows);
  const int64_t r0 = (int64_t)blockIdx.y * 64;
  const int c0 = blockIdx.x * 64;
  // gathered rows: zero fill up to the multiple of 128 the dW contraction runs over, nothing beyond
  if (n_scored != nullptr && r0 >= (nrows + 127) / 128 * 128) return;
  const int tc = threadIdx.x & 7, tr = threadIdx.x >> 3;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int rr = tr + 32 * k;
    const int64_t r = r0 + rr;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < nrows) {
      const int64_t src_row = rows ? (int64_t)rows[r] : r;
      v = *reinterpret_cast<const uint4*>(in + src_row * ld_in + c0 + tc * 8);
      if (scale != nullptr) {
        // bf16 elements times the row's scale, rounded back to bf16 (nearest even)
        const float sc = scale[r];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const __bf16 lo = (__bf16)(sc * bf16_bits_to_float(w[q] & 0xffffu));
          const __bf16 hi = (__bf16)(sc * bf16_bits_to_float(w[q] >> 16));
          uint16_t ul, uh;
          __builtin_memcpy(&ul, &lo, 2);
          __builtin_memcpy(&uh, &hi, 2);
          w[q] = (uint32_t)ul | ((uint32_t)uh << 16);
        }
        v = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
    *reinterpret_cast<uint4*>(&tile[rr * 72 + tc * 8]) = v;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int cc = tr + 32 * k;
    uint32_t ow[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t lo = tile[(tc * 8 + q * 2) * 72 + cc];
      const uint32_t hi = tile[(tc * 8 + q * 2 + 1) * 72 + cc];
      ow[q] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4*>(out + (int64_t)(c0 + cc) * ld_out + r0 + tc * 8) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  }
}

// 4-byte elements, scalar, bounds-checked: tile 32 x 32.
__global__ __launch_bounds__(256) void k_transpose_b32(const uint32_t* in, int64_t ld_in, const int32_t* rows,
                                                       uint32_t* out, int64_t ld_out, int64_t n_rows_static,
                                                       const int64_t* n_scored, int64_t chunk_start,
                                                       int chunk_rows, int n_cols, int64_t out_cols_pad) {
  __shared__ uint32_t tile[32][33];
  int64_t nrows = n_rows_static;
  if (n_scored != nullptr) nrows = valid_rows(n_scored, chunk_start, chunk_rows);
  const int64_t r0 = (int64_t)blockIdx.y * 32;
  const int c0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int k = ty; k < 32; k += 8) {
    const int64_t r = r0 + k;
    const int c = c0 + tx;
    uint32_t v = 0;
    if (r < nrows && c < n_cols) {
      const int64_t src_row = rows ? (int64_t)rows[r] : r;
      v = in[src_row * ld_in + c];
    }
    tile[k][tx] = v;
  }
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int c = c0 + k;
    const int64_t r = r0 + tx;
    if (c < n_cols && r < out_cols_pad) out[(int64_t)c * ld_out + r] = tile[tx][k];
  }
}

}  // namespace

// ------------------------------------------------------------------ launchers
void launch_prep(const uint8_t* mask, const int32_t* targets, int64_t N, int V, const PrepOut& o,
                 hipStream_t stream) {
  const int64_t nblocks = (N + PREP_PER_BLOCK - 1) / PREP_PER_BLOCK;
  // block_counts: [2 * nblocks] int32 counts followed (8-byte aligned) by [nblocks] int64 offsets
  int64_t* block_offsets = reinterpret_cast<int64_t*>(o.block_counts + round_up(2 * nblocks, 2));
  hipLaunchKernelGGL(k_prep_count, dim3((unsigned)nblocks), dim3(PREP_BLOCK), 0, stream, mask, targets, N, V,
                     o.block_counts, nblocks);
  hipLaunchKernelGGL(k_prep_scan, dim3(1), dim3(1024), 0, stream, o.block_counts, nblocks, block_offsets,
                     o.n_scored, o.n_bad);
  hipLaunchKernelGGL(k_prep_fill, dim3((unsigned)nblocks), dim3(PREP_BLOCK), 0, stream, mask, targets, N, V,
                     block_offsets, o.n_scored, o.row_index);
}

void launch_seq_weights(const uint8_t* mask, const int32_t* targets, const int32_t* group_id,
                        const uint8_t* seq_kind, int64_t B, int T, int G, int V, int loss_agg,
                        int32_t* seq_len, float* seq_coef, int32_t* group_count, int64_t* n_bad_groups,
                        hipStream_t stream) {
  hipLaunchKernelGGL(k_seq_len, dim3((unsigned)B), dim3(256), 0, stream, mask, targets, T, V, seq_len);
  hipLaunchKernelGGL(k_seq_coef, dim3(1), dim3(1024), 0, stream, seq_len, group_id, seq_kind, B, G, loss_agg,
                     group_count, seq_coef, n_bad_groups);
}

void launch_seq_log_ratio(const uint8_t* mask, const int32_t* targets, const float* logp,
                          const float* behav_logp, int64_t B, int T, int V, int level, float* seq_expo,
                          hipStream_t stream) {
  hipLaunchKernelGGL(k_seq_log_ratio, dim3((unsigned)B), dim3(256), 0, stream, mask, targets, logp, behav_logp,
                     T, V, level, seq_expo);
}

void launch_zero_unscored(const uint8_t* mask, const int32_t* targets, int64_t N, int V, int d,
                          float* out_logp, float* out_lse, void* dH, int dh_elem_bytes,
                          hipStream_t stream) {
  const int64_t blocks = (N + ZERO_SLOTS_PER_BLOCK - 1) / ZERO_SLOTS_PER_BLOCK;
  hipLaunchKernelGGL(k_zero_unscored, dim3((unsigned)blocks), dim3(256), 0, stream, mask, targets, N, V,
                     (int64_t)d * dh_elem_bytes, out_logp, out_lse, static_cast<unsigned char*>(dH));
}

void launch_target_logit(const void* H, const void* W, const int32_t* targets,
                         const int32_t* row_index, const int64_t* n_scored, int64_t N_max,
                         int d, int is_bf16, float* zt, hipStream_t stream) {
  const int64_t blocks = (N_max + 3) / 4;
  if (is_bf16)
    hipLaunchKernelGGL(k_target_logit<true>, dim3((unsigned)blocks), dim3(256), 0, stream, H, W, targets,
                       row_index, n_scored, d, zt);
  else
    hipLaunchKernelGGL(k_target_logit<false>, dim3((unsigned)blocks), dim3(256), 0, stream, H, W, targets,
                       row_index, n_scored, d, zt);
}

void launch_row_lse_f32(const float* Z, int64_t ldz, const int64_t* n_scored, int64_t chunk_start,
                        int chunk_rows, int V, float* part_max, float* part_sum, float* part_ez,
                        hipStream_t stream) {
  hipLaunchKernelGGL(k_row_lse_f32, dim3(chunk_rows), dim3(256), 0, stream, Z, ldz, n_scored, chunk_start,
                     chunk_rows, V, part_max, part_sum, part_ez);
}

int row_epilogue_blocks(int chunk_rows) { return (chunk_rows + EPI_ROWS - 1) / EPI_ROWS; }

void launch_row_epilogue(const RowEpiArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(k_row_epilogue, dim3(row_epilogue_blocks(a.chunk_rows)), dim3(256), 0, stream, a);
}

void launch_convert_f32(float* ZP, int64_t ldz, float* Pt, int64_t ldpt, const float* lse_c,
                        const float* g_c, const int32_t* targets, const int32_t* row_index,
                        const int64_t* n_scored, int64_t chunk_start, int chunk_rows, int V,
                        hipStream_t stream) {
  int gx = (V + 255) / 256; gx = gx > 64 ? 64 : gx;
  dim3 grid(gx, chunk_rows);
  hipLaunchKernelGGL(k_convert_f32, grid, dim3(256), 0, stream, ZP, ldz, Pt, ldpt, lse_c, g_c, targets,
                     row_index, n_scored, chunk_start, chunk_rows, V);
}

void launch_zero_stash_tail(void* estash, int64_t lde, const int64_t* n_scored, int64_t chunk_start,
                            int chunk_rows, int Vp, hipStream_t stream) {
  dim3 grid((Vp / 8 + 255) / 256, 127);
  hipLaunchKernelGGL(k_zero_stash_tail, grid, dim3(256), 0, stream, static_cast<uint16_t*>(estash), lde,
                     n_scored, chunk_start, chunk_rows, Vp);
}

void launch_gather_rows_b16(const void* in, int64_t ld_in, const int32_t* rows, void* out, int64_t ld_out,
                            int64_t n_rows_static, const int64_t* n_scored, int64_t chunk_start,
                            int chunk_rows, int d, int dp, hipStream_t stream) {
  const int64_t max_rows = n_scored != nullptr ? chunk_rows : n_rows_static;
  if (max_rows <= 0) return;
  hipLaunchKernelGGL(k_gather_rows_b16, dim3((unsigned)((max_rows + GATHER_ROWS - 1) / GATHER_ROWS)), dim3(256), 0,
                     stream, static_cast<const uint16_t*>(in), ld_in, rows, static_cast<uint16_t*>(out), ld_out,
                     n_rows_static, n_scored, chunk_start, chunk_rows, d, dp);
}

void launch_transpose(const void* in, int64_t ld_in, const int32_t* rows, const float* scale, void* out, int64_t ld_out,
                      int64_t n_rows_static, const int64_t* n_scored, int64_t chunk_start,
                      int chunk_rows, int n_cols, int64_t out_cols_pad, int elem_bytes,
                      hipStream_t stream) {
  if (elem_bytes == 2) {
    dim3 grid(n_cols / 64, (unsigned)(out_cols_pad / 64));
    hipLaunchKernelGGL(k_transpose_b16, grid, dim3(256), 0, stream, static_cast<const uint16_t*>(in), ld_in,
                       rows, scale, static_cast<uint16_t*>(out), ld_out, n_rows_static, n_scored, chunk_start,
                       chunk_rows);
  } else {
    dim3 grid((n_cols + 31) / 32, (unsigned)((out_cols_pad + 31) / 32));
    hipLaunchKernelGGL(k_transpose_b32, grid, dim3(256), 0, stream, static_cast<const uint32_t*>(in), ld_in,
                       rows, static_cast<uint32_t*>(out), ld_out, n_rows_static, n_scored, chunk_start,
                       chunk_rows, n_cols, out_cols_pad);
  }
}

void launch_finalize(const double* loss_partials, int64_t n_blocks, const int64_t* n_scored,
                     const int64_t* n_bad, float beta, float lambda, int64_t rows_enqueued,
                     const int32_t* row_index, float* out_logp, void* out_stats, hipStream_t stream) {
  double* out_d = static_cast<double*>(out_stats);
  int64_t* out_i = reinterpret_cast<int64_t*>(out_d + 7);
  hipLaunchKernelGGL(k_finalize, dim3(1), dim3(256), 0, stream, loss_partials, n_blocks, n_scored, n_bad,
                     beta, lambda, rows_enqueued, row_index, out_logp, out_d, out_i);
}

}  // namespace mrl
