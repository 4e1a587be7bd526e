// bf16 MFMA tile GEMM for gfx950 with three fused epilogues.
//
// One kernel body computes C[m][n] = sum_k A[m][k] * B[n][k] for a 256 x 256
// tile per workgroup (both operands K-contiguous, "NT" form).  Four wave64
// wavefronts form a 2 x 2 grid, each owning a 128 x 128 sub-tile as 4 x 4
// MFMA 32x32x16 accumulators (256 accumulator registers per lane).  Operand
// panels of 64 K-elements are staged through LDS, double-buffered, in rows of
// 128 bytes whose 16-byte chunks are XOR-swizzled with the row number so that
// the 128-bit fragment reads of the MFMA operands are bank-conflict free.
//
// The three uses on the scoring path (Sec. 3: log pi(y_t | ...) needs the
// softmax over the whole vocabulary of the LM-head logits):
//   FWD: A = W (vocabulary rows), B = H (token rows, gathered).  The MFMA result
//        layout keeps 16 rows x 1 column per lane, so putting the vocabulary on
//        the M side makes the max / sum-exp reduction over the vocabulary an
//        in-register reduction with a single cross-lane step.
//   DH : A = dz rows (tokens), B = W^T;  rows are scattered to the padded slots.
//   DW : A = dz^T (vocabulary rows), B = H^T; fp32 read-modify-write of dW.
#include "mrl_internal.h"

namespace mrl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 256;
constexpr int TILE_BYTES = BM * BK * 2;            // one operand panel: 32 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + B
constexpr int LDS_BYTES = 2 * STAGE_BYTES;         // double buffered: 128 KB

enum { MODE_FWD = 0, MODE_DH = 1, MODE_DW = 2 };

struct Params {
  const uint16_t* A; int64_t lda; int M;
  const uint16_t* B; int64_t ldb; int N;
  int K;
  const int32_t* row_index;   // already offset to the chunk start
  const int64_t* n_scored; int64_t chunk_start; int chunk_rows;
  // FWD
  float* part_max; float* part_sum; uint16_t* zstash; int64_t ldz; int V;
  // DH
  void* dH; int dh_f32; int d;
  // DW
  float* dW; int overwrite;
};

// Workgroup -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs,
// each with its own L2; 32 consecutive workgroups of one XCD form a 4 x 8
// super-tile so that they share operand panels in that L2, and super-tiles are
// numbered N-fastest so that the XCDs walk the same A rows at the same time.
constexpr int SUP_M = 4, SUP_N = 8, NXCD = 8;
__host__ __device__ inline int num_blocks(int Mt, int Nt) {
  int s = ((Mt + SUP_M - 1) / SUP_M) * ((Nt + SUP_N - 1) / SUP_N);
  return (s + NXCD - 1) / NXCD * NXCD * (SUP_M * SUP_N);
}
__device__ inline bool tile_coords(int bid, int Mt, int Nt, int& tm, int& tn) {
  const int sNt = (Nt + SUP_N - 1) / SUP_N, sMt = (Mt + SUP_M - 1) / SUP_M;
  const int xcd = bid % NXCD, local = bid / NXCD;
  const int q = local / (SUP_M * SUP_N), within = local % (SUP_M * SUP_N);
  const int s = q * NXCD + xcd;
  if (s >= sMt * sNt) return false;
  tm = (s / sNt) * SUP_M + within % SUP_M;
  tn = (s % sNt) * SUP_N + within / SUP_M;
  return tm < Mt && tn < Nt;
}

__device__ inline float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

template <int MODE>
__global__ __launch_bounds__(NTHREADS) void gemm_nt_bf16(Params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // valid rows of this chunk (device-side, no host sync)
  int64_t nv64 = *p.n_scored - p.chunk_start;
  const int nvalid = nv64 < 0 ? 0 : (nv64 > p.chunk_rows ? p.chunk_rows : (int)nv64);

  int M = p.M, N = p.N, K = p.K;
  if (MODE == MODE_FWD) N = nvalid;
  if (MODE == MODE_DH) M = nvalid;
  if (MODE == MODE_DW) { int kv = (nvalid + BK - 1) / BK * BK; K = kv < K ? kv : K; }
  if (MODE == MODE_FWD && nvalid == 0) return;
  if (MODE == MODE_DH && nvalid == 0) return;
  if (MODE == MODE_DW && nvalid == 0 && !p.overwrite) return;

  const int Mt = (p.M + BM - 1) / BM, Nt = (p.N + BN - 1) / BN;
  int tm, tn;
  if (!tile_coords(blockIdx.x, Mt, Nt, tm, tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;
  if (m0 >= M || n0 >= N) return;

  // ---- global -> LDS staging: 8 threads cover one 128-byte row, 32 rows per pass
  const int lc = tid & 7;        // 16-byte chunk within the row
  const int lr = tid >> 3;       // 0..31
  const uint16_t* a_ptr[8];
  const uint16_t* b_ptr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int ra = m0 + lr + 32 * i; ra = ra < M ? ra : M - 1;
    int rb = n0 + lr + 32 * i; rb = rb < N ? rb : N - 1;
    int64_t rowa = ra, rowb = rb;
    if (MODE == MODE_FWD) rowb = p.row_index[rb];
    a_ptr[i] = p.A + rowa * p.lda + lc * 8;
    b_ptr[i] = p.B + rowb * p.ldb + lc * 8;
  }
  // swizzled LDS write offset of (row lr + 32 i, chunk lc): (row & 7) == (lr & 7)
  const int st_off = lr * 128 + ((lc ^ (lr & 7)) << 4);

  // ---- fragment read offsets: lane -> row (lane & 31), k-half (lane >> 5)
  const int frow = lane & 31, fhalf = lane >> 5;
  int a_off[4], b_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int chunk = ((kk << 1) | fhalf) ^ (frow & 7);
    a_off[kk] = (wm * 128 + frow) * 128 + (chunk << 4);
    b_off[kk] = TILE_BYTES + (wn * 128 + frow) * 128 + (chunk << 4);
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra[8], rb[8];
  const int nk = K / BK;
  if (nk > 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      ra[i] = *reinterpret_cast<const u32x4*>(a_ptr[i]);
      rb[i] = *reinterpret_cast<const u32x4*>(b_ptr[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4*>(smem + st_off + i * 4096) = ra[i];
      *reinterpret_cast<u32x4*>(smem + TILE_BYTES + st_off + i * 4096) = rb[i];
    }
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = (kt & 1) * STAGE_BYTES;
    const int nxt = STAGE_BYTES - cur;
    const bool more = kt + 1 < nk;
    if (more) {
      const int koff = (kt + 1) * BK;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        ra[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + koff);
        rb[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + koff);
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 af[4], bfr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        af[i] = *reinterpret_cast<const bf16x8*>(smem + cur + a_off[kk] + i * 4096);
        bfr[i] = *reinterpret_cast<const bf16x8*>(smem + cur + b_off[kk] + i * 4096);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        *reinterpret_cast<u32x4*>(smem + nxt + st_off + i * 4096) = ra[i];
        *reinterpret_cast<u32x4*>(smem + nxt + TILE_BYTES + st_off + i * 4096) = rb[i];
      }
    }
    __syncthreads();
  }

  // ---- epilogues.  Accumulator element (i, j, e) of this lane is
  //   row m = m0 + wm*128 + i*32 + 8*(e/4) + 4*(lane>>5) + (e&3)
  //   col n = n0 + wn*128 + j*32 + (lane & 31)
  const int mrow_base = m0 + wm * 128 + 4 * fhalf;
  const int ncol_base = n0 + wn * 128 + frow;

  if (MODE == MODE_FWD) {
    // rows = vocabulary ids, cols = token rows of the chunk
    constexpr float LOG2E = 1.4426950408889634f;
    const bool full = (m0 + BM <= p.V);
    const int pidx = tm * 2 + wm;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = ncol_base + j * 32;
      float mx = -INFINITY;
      if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) mx = fmaxf(mx, acc[i][j][e]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = mrow_base + i * 32 + 8 * (e >> 2) + (e & 3);
            mx = v < p.V ? fmaxf(mx, acc[i][j][e]) : mx;
          }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mneg = (mx == -INFINITY) ? 0.f : -mx * LOG2E;
      float s = 0.f;
      if (full) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) s += exp2_fast(fmaf(acc[i][j][e], LOG2E, mneg));
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = mrow_base + i * 32 + 8 * (e >> 2) + (e & 3);
            const float t = exp2_fast(fmaf(acc[i][j][e], LOG2E, mneg));
            s += v < p.V ? t : 0.f;
          }
      }
      s += __shfl_xor(s, 32);
      if (fhalf == 0 && n < N) {
        p.part_max[(int64_t)pidx * p.chunk_rows + n] = mx;
        p.part_sum[(int64_t)pidx * p.chunk_rows + n] = s;
      }
      if (p.zstash != nullptr && n < N) {
        uint16_t* zrow = p.zstash + (int64_t)n * p.ldz;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f16x4 h;
#pragma unroll
            for (int r = 0; r < 4; ++r)
              h[r] = (_Float16)__builtin_amdgcn_fmed3f(acc[i][j][q * 4 + r], -65504.f, 65504.f);
            const int v = mrow_base + i * 32 + 8 * q;
            *reinterpret_cast<f16x4*>(zrow + v) = h;
          }
      }
    }
  } else if (MODE == MODE_DH) {
    // rows = token rows of the chunk (scattered to their slots), cols = hidden index
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = mrow_base + i * 32 + 8 * (e >> 2) + (e & 3);
        if (m < M) {
          const int64_t slot = p.row_index[m];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int n = ncol_base + j * 32;
            if (n < p.d) {
              if (p.dh_f32) {
                reinterpret_cast<float*>(p.dH)[slot * p.d + n] = acc[i][j][e];
              } else {
                reinterpret_cast<__bf16*>(p.dH)[slot * p.d + n] = (__bf16)acc[i][j][e];
              }
            }
          }
        }
      }
  } else {
    // rows = vocabulary ids, cols = hidden index; fp32 accumulate into dW
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int v = mrow_base + i * 32 + 8 * (e >> 2) + (e & 3);
        if (v < p.V) {
          float* row = p.dW + (int64_t)v * p.d;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int n = ncol_base + j * 32;
            if (n < p.d) {
              if (p.overwrite) row[n] = acc[i][j][e];
              else row[n] += acc[i][j][e];
            }
          }
        }
      }
  }
}

template <int MODE>
void launch(const Params& p, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_bf16<MODE>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    attr_set = true;
  }
  const int Mt = (p.M + BM - 1) / BM, Nt = (p.N + BN - 1) / BN;
  const int blocks = num_blocks(Mt, Nt);
  hipLaunchKernelGGL(gemm_nt_bf16<MODE>, dim3(blocks), dim3(NTHREADS), LDS_BYTES, stream, p);
}

}  // namespace

void launch_gemm_fwd_bf16(const void* W, const void* H, const int32_t* row_index,
                          const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                          int V, int d, float* part_max, float* part_sum,
                          void* zstash, int64_t ldz, hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(W); p.lda = d; p.M = V;
  p.B = static_cast<const uint16_t*>(H); p.ldb = d; p.N = chunk_rows;
  p.K = d;
  p.row_index = row_index + chunk_start;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.part_max = part_max; p.part_sum = part_sum;
  p.zstash = static_cast<uint16_t*>(zstash); p.ldz = ldz; p.V = V; p.d = d;
  launch<MODE_FWD>(p, stream);
}

void launch_gemm_dh_bf16(const void* P, int64_t ldp, const void* Wt, int64_t ldwt,
                         const int32_t* row_index, const int64_t* n_scored, int64_t chunk_start,
                         int chunk_rows, int Vp, int d, void* dH, int dh_f32, hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(P); p.lda = ldp; p.M = chunk_rows;
  p.B = static_cast<const uint16_t*>(Wt); p.ldb = ldwt; p.N = d;
  p.K = Vp;
  p.row_index = row_index + chunk_start;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.dH = dH; p.dh_f32 = dh_f32; p.d = d; p.V = Vp;
  launch<MODE_DH>(p, stream);
}

void launch_gemm_dw_bf16(const void* Pt, int64_t ldpt, const void* Ht, int64_t ldht,
                         const int64_t* n_scored, int64_t chunk_start, int chunk_rows,
                         int V, int d, float* dW, int overwrite, hipStream_t stream) {
  Params p = {};
  p.A = static_cast<const uint16_t*>(Pt); p.lda = ldpt; p.M = (int)round_up(V, kTile);
  p.B = static_cast<const uint16_t*>(Ht); p.ldb = ldht; p.N = d;
  p.K = chunk_rows;
  p.n_scored = n_scored; p.chunk_start = chunk_start; p.chunk_rows = chunk_rows;
  p.dW = dW; p.overwrite = overwrite; p.V = V; p.d = d;
  launch<MODE_DW>(p, stream);
}

}  // namespace mrl
