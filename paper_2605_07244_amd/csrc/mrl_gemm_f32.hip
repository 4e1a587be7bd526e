// Plain fp32 GEMM C[m][n] = sum_k A[m][k] * B[n][k] for the small-shape sanity
// path (dtype MRL_F32).  64 x 64 tile, 16-wide K panels through LDS, 4 x 4
// outputs per thread, every access bounds-checked; not tuned.
#include "mrl_internal.h"

namespace mrl {
namespace {

constexpr int FT = 64, FK = 16;

__global__ __launch_bounds__(256) void k_gemm_f32(GemmF32Args a) {
  __shared__ float As[FK][FT + 1];
  __shared__ float Bs[FK][FT + 1];
  int M = a.M, K = a.K;
  if (a.m_dynamic || a.k_dynamic) {
    int64_t r = *a.n_scored - a.chunk_start;
    const int nv = r < 0 ? 0 : (r > a.chunk_rows ? a.chunk_rows : (int)r);
    if (a.m_dynamic) M = nv;
    if (a.k_dynamic) K = nv;
  }
  const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
  if (m0 >= M) return;
  if (a.k_dynamic && K == 0 && a.accumulate) return;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  const int lrow = threadIdx.x >> 2;         // 0..63
  const int lk = (threadIdx.x & 3) * 4;      // 0,4,8,12
  const int am = m0 + lrow, bn = n0 + lrow;
  const int64_t arow = am < M ? (a.a_rows ? (int64_t)a.a_rows[am] : (int64_t)am) : -1;
  for (int k0 = 0; k0 < K; k0 += FK) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = k0 + lk + q;
      As[lk + q][lrow] = (arow >= 0 && k < K) ? a.A[arow * a.lda + k] : 0.f;
      Bs[lk + q][lrow] = (bn < a.N && k < K) ? a.B[(int64_t)bn * a.ldb + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FK; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[k][ty * 4 + i]; bv[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    const int64_t crow = a.c_rows ? (int64_t)a.c_rows[m] : (int64_t)m;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= a.N) continue;
      float* dst = a.C + crow * a.ldc + n;
      if (a.accumulate) *dst += acc[i][j]; else *dst = acc[i][j];
    }
  }
}

}  // namespace

void launch_gemm_f32(const GemmF32Args& a, hipStream_t stream) {
  dim3 grid((a.N + FT - 1) / FT, (a.M + FT - 1) / FT);
  hipLaunchKernelGGL(k_gemm_f32, grid, dim3(256), 0, stream, a);
}

}  // namespace mrl
