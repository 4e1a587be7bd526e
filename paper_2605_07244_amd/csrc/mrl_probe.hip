// MFMA-only rate probe: what the matrix cores of this device sustain on the
// instruction the GEMM kernel uses (v_mfma_f32_16x16x32_bf16, 8 x 8 register
// tile per wave, one wave per SIMD), with no memory traffic at all.  With
// constant operands the result is the clock-limited peak; with random-mantissa
// operands (what real activations and weights look like) the chip lowers its
// clock to stay inside its power limit, and the result is the ceiling any
// bf16 GEMM can reach on such data.  Benchmarks report both beside the
// published peak.
#include "../../include/mrl.h"
#include "../../include/mrl_diag.h"
#include "mrl_internal.h"

namespace mrl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

// bf16 bit patterns: random sign and mantissa, exponent in a band of 8 binades (|x| in [2^-11, 2^-3))
__device__ inline bf16x8 operand(unsigned& x, bool random) {
  u16x8 u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    x = x * 1664525u + 1013904223u;
    u[e] = random ? (unsigned short)(((x >> 9) & 0x807f) | (0x3a00 + ((x >> 3) & 0x380))) : (unsigned short)0x3c00;
  }
  return __builtin_bit_cast(bf16x8, u);
}

__global__ __launch_bounds__(256) void k_mfma_rate(float* out, int iters, int random) {
  bf16x8 a[8], b[8];
  unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = operand(x, random != 0); b[i] = operand(x, random != 0); }
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace
}  // namespace mrl

extern "C" int mrl_probe_mfma_rate(int32_t random_operands, double seconds, void* scratch,
                                   size_t scratch_bytes, double* out_tflops) {
  using namespace mrl;
  if (scratch == nullptr || out_tflops == nullptr) return MRL_ERR_NULL;
  if (!(seconds > 0.0) || seconds > 5.0) return MRL_ERR_CONFIG;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return MRL_ERR_DEVICE;
  }
  const int blocks = prop.multiProcessorCount;              // one workgroup of 4 waves per CU
  if (scratch_bytes < (size_t)blocks * 256 * sizeof(float)) return MRL_ERR_WORKSPACE;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { (void)hipGetLastError(); return MRL_ERR_DEVICE; }
  const double flop_per_iter = (double)blocks * 4 * 64 * 2.0 * 16 * 16 * 32;
  // calibrate on a short run, then time one launch of about the requested length
  int iters = 2000;
  double tflops = 0.0;
  int rc = MRL_OK;
  for (int pass = 0; pass < 2 && rc == MRL_OK; ++pass) {
    (void)hipEventRecord(e0, nullptr);
    hipLaunchKernelGGL(k_mfma_rate, dim3(blocks), dim3(256), 0, nullptr, static_cast<float*>(scratch), iters, random_operands);
    (void)hipEventRecord(e1, nullptr);
    if (hipEventSynchronize(e1) != hipSuccess) { (void)hipGetLastError(); rc = MRL_ERR_DEVICE; break; }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (!(ms > 0.f)) { rc = MRL_ERR_DEVICE; break; }
    tflops = flop_per_iter * iters / (ms * 1e-3) / 1e12;
    double next = iters * (seconds * 1e3 / ms);
    iters = next > 4e7 ? 40000000 : (next < 2000 ? 2000 : (int)next);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *out_tflops = tflops;
  return rc;
}
