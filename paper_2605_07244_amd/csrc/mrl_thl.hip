// THL word-level trace alignment on integer word maps (Sec. 4.3; App. D, Alg. 2):
// the source model's log-probs are summed per textual word and each word total is
// spread evenly over the target tokens of that word.  One workgroup per sequence;
// per-word sums and counts live in LDS.  The sums are accumulated as 64-bit fixed
// point (2^-32 units) with integer LDS atomics, so the result does not depend on
// the order in which tokens arrive: runs are bit-reproducible.
#include "../../include/mrl.h"
#include "mrl_internal.h"

namespace mrl {
namespace {

constexpr int THL_THREADS = 256;
constexpr int THL_MAX_WORDS = 8192;                 // 8 B sum + 4 B count per word: 96 KB of LDS
constexpr double THL_SCALE = 4294967296.0;          // 2^32

// Index of this thread's position among the set mask bits of the row, counted from the
// row start: `base` (bits before this 256-position chunk) + bits before the thread in the
// chunk.  Returns the chunk's bit count through `chunk_total`.  All threads must call it.
__device__ inline int rank_in_chunk(bool bit, int base, int* wave_counts, int& chunk_total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long ball = __ballot(bit);
  const int before = __popcll(ball & ((1ull << lane) - 1ull));
  __syncthreads();                                   // wave_counts of the previous chunk are consumed
  if (lane == 0) wave_counts[wave] = __popcll(ball);
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < THL_THREADS / 64; ++w) {
    const int c = wave_counts[w];
    off += w < wave ? c : 0;
    tot += c;
  }
  chunk_total = tot;
  return base + off + before;
}

__global__ __launch_bounds__(THL_THREADS) void k_thl_word_align(
    const float* src_logp, const uint8_t* src_mask, const int32_t* src_map, const int32_t* src_map_len,
    const uint8_t* tgt_mask, const int32_t* tgt_map, const int32_t* tgt_map_len, int S_src, int S_tgt,
    int max_words, float ignore_value, float* out, unsigned long long* bad_words) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  long long* wsum = reinterpret_cast<long long*>(smem);                       // [max_words]
  int* wcnt = reinterpret_cast<int*>(smem + (size_t)max_words * 8);           // [max_words]
  __shared__ int wave_counts[THL_THREADS / 64];
  __shared__ int any_word;
  __shared__ int n_bad;

  const int64_t i = blockIdx.x;
  const float* lp = src_logp + i * S_src;
  const uint8_t* sm = src_mask + i * S_src;
  const int32_t* smap = src_map + i * S_src;
  const uint8_t* tm = tgt_mask + i * S_tgt;
  const int32_t* tmap = tgt_map + i * S_tgt;
  float* o = out + i * S_tgt;
  const int slen = src_map_len[i], tlen = tgt_map_len[i];

  for (int w = threadIdx.x; w < max_words; w += THL_THREADS) { wsum[w] = 0; wcnt[w] = 0; }
  if (threadIdx.x == 0) { any_word = 0; n_bad = 0; }
  __syncthreads();

  // aggregation pass: Z_w = sum of the source log-probs of the response tokens mapped to w
  int base = 0, my_bad = 0;
  for (int j0 = 0; j0 < S_src; j0 += THL_THREADS) {
    const int j = j0 + threadIdx.x;
    const bool bit = j < S_src && sm[j] == 1;
    int tot;
    const int p = rank_in_chunk(bit, base, wave_counts, tot);
    base += tot;
    if (bit && p < slen) {
      const int wid = smap[p];
      if (wid >= 0 && wid < max_words) {
        const long long q = __double2ll_rn((double)lp[j] * THL_SCALE);
        atomicAdd(reinterpret_cast<unsigned long long*>(&wsum[wid]), (unsigned long long)q);
        any_word = 1;
      } else if (wid != -1) {
        ++my_bad;
      }
    }
  }
  __syncthreads();
  const bool active = any_word != 0;   // a sequence whose source side carries no word stays inactive

  // count pass: C_w = number of target response tokens mapped to w
  if (active) {
    base = 0;
    for (int j0 = 0; j0 < S_tgt; j0 += THL_THREADS) {
      const int j = j0 + threadIdx.x;
      const bool bit = j < S_tgt && tm[j] == 1;
      int tot;
      const int p = rank_in_chunk(bit, base, wave_counts, tot);
      base += tot;
      if (bit && p < tlen) {
        const int wid = tmap[p];
        if (wid >= 0 && wid < max_words) atomicAdd(&wcnt[wid], 1);
        else if (wid != -1) ++my_bad;
      }
    }
    __syncthreads();
  }

  // redistribution pass: each target token of word w receives Z_w / C_w
  base = 0;
  for (int j0 = 0; j0 < S_tgt; j0 += THL_THREADS) {
    const int j = j0 + threadIdx.x;
    const bool bit = active && j < S_tgt && tm[j] == 1;
    int tot;
    const int p = rank_in_chunk(bit, base, wave_counts, tot);
    base += tot;
    if (j < S_tgt) {
      float v = ignore_value;
      if (bit && p < tlen) {
        const int wid = tmap[p];
        if (wid >= 0 && wid < max_words) v = (float)(((double)wsum[wid] / THL_SCALE) / (double)wcnt[wid]);
      }
      o[j] = v;
    }
  }
  if (bad_words != nullptr) {
    if (my_bad) atomicAdd(&n_bad, my_bad);
    __syncthreads();
    if (threadIdx.x == 0 && n_bad) atomicAdd(bad_words, (unsigned long long)n_bad);
  }
}

__global__ void k_zero_u64(unsigned long long* p) { *p = 0; }

}  // namespace
}  // namespace mrl

extern "C" int mrl_thl_word_align(const float* src_logp, const uint8_t* src_mask,
                                  const int32_t* src_word_map, const int32_t* src_map_len,
                                  const uint8_t* tgt_mask, const int32_t* tgt_word_map,
                                  const int32_t* tgt_map_len, int64_t B, int32_t S_src, int32_t S_tgt,
                                  int32_t max_words, float ignore_value, float* out,
                                  int64_t* out_bad_words, void* stream) {
  using namespace mrl;
  if (B < 0 || S_src <= 0 || S_tgt <= 0 || B > ((int64_t)1 << 31) - 1) return MRL_ERR_SHAPE;
  if (max_words <= 0 || max_words > THL_MAX_WORDS) return MRL_ERR_SHAPE;
  if (B == 0) return MRL_OK;
  if (!src_logp || !src_mask || !src_word_map || !src_map_len || !tgt_mask || !tgt_word_map ||
      !tgt_map_len || !out)
    return MRL_ERR_NULL;
  const int rc = require_gfx950();
  if (rc != MRL_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t lds = (size_t)max_words * 12;
  static LdsLimit lds_limit;
  lds_limit.ensure(reinterpret_cast<const void*>(&k_thl_word_align), THL_MAX_WORDS * 12);
  if (out_bad_words) hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, s, reinterpret_cast<unsigned long long*>(out_bad_words));
  hipLaunchKernelGGL(k_thl_word_align, dim3((unsigned)B), dim3(THL_THREADS), lds, s, src_logp, src_mask,
                     src_word_map, src_map_len, tgt_mask, tgt_word_map, tgt_map_len, S_src, S_tgt, max_words,
                     ignore_value, out, reinterpret_cast<unsigned long long*>(out_bad_words));
  return hipGetLastError() == hipSuccess ? MRL_OK : MRL_ERR_DEVICE;
}
