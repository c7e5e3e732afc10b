// Measurement helper, not part of the method: the rate this device sustains on a loop of nothing but
// v_mfma_f32_32x32x16_bf16 (the instruction the attention and projection kernels run on), with operands that
// are either constant or random.  The benchmark reports the attention kernel against this rate as well as
// against the nominal peak, because the sustained clock under matrix load depends on the operand data.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparse_attn.h"
#include "sparse_attn_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;

constexpr int kChains = 4;   // independent accumulator chains per wave

__global__ void __launch_bounds__(256) mfma_loop(float* out, unsigned long long* clocks, int iters, int random_operands) {
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  const int l = threadIdx.x;
  bf16x8 a[kChains], b[kChains];
  unsigned rng = 0x9E3779B9u * (blockIdx.x * 256 + l + 1);
  for (int r = 0; r < kChains; ++r) {
    u16x8 av, bv;
    for (int s = 0; s < 8; ++s) {
      // random sign and mantissa with a fixed exponent (|a| in [1, 2), |b| in [1/8, 1/4)), or the constants 1 and 1/8
      rng = rng * 1664525u + 1013904223u;
      av[s] = random_operands ? (unsigned short)(((rng >> 16) & 0x807f) | 0x3f80) : 0x3f80;
      rng = rng * 1664525u + 1013904223u;
      bv[s] = random_operands ? (unsigned short)(((rng >> 16) & 0x807f) | 0x3e00) : 0x3e00;
    }
    a[r] = __builtin_bit_cast(bf16x8, av);
    b[r] = __builtin_bit_cast(bf16x8, bv);
  }
  f32x16 c[kChains];
  for (int r = 0; r < kChains; ++r)
    for (int e = 0; e < 16; ++e) c[r][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < kChains; ++r) c[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r], b[r], c[r], 0, 0, 0);
  }
  float s = 0.f;
  for (int r = 0; r < kChains; ++r)
    for (int e = 0; e < 16; ++e) s += c[r][e];
  out[blockIdx.x * 256 + l] = s;
  if (l == 0) {
    clocks[2 * blockIdx.x] = clock64() - c0;
    clocks[2 * blockIdx.x + 1] = wall_clock64() - w0;
  }
}

#define PROBE_TRY(expr)                                                                                       \
  do {                                                                                                        \
    hipError_t e_ = (expr);                                                                                   \
    if (e_ != hipSuccess) {                                                                                   \
      if (out) (void)hipFree(out);                                                                            \
      if (clk) (void)hipFree(clk);                                                                            \
      return sa_fail(SPARSE_ATTN_ERR_HIP, "probe: %s failed: %s", #expr, hipGetErrorString(e_));              \
    }                                                                                                         \
  } while (0)

}  // namespace

extern "C" int sparse_attn_probe_mfma(int random_operands, int launches, double* tflops, double* shader_mhz) {
  if (launches < 1 || launches > 64 || !tflops)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "probe: launches must be 1..64 and tflops must not be NULL");
  float* out = nullptr;
  unsigned long long* clk = nullptr;
  int dev = 0, cus = 0;
  PROBE_TRY(hipGetDevice(&dev));
  PROBE_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int blocks = 2 * cus;             // 8 waves per CU, two per SIMD
  const int iters = 100000;               // about 10 ms per launch
  PROBE_TRY(hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)));
  PROBE_TRY(hipMalloc(&clk, (size_t)blocks * 2 * sizeof(unsigned long long)));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  float ms = 0.f;
  for (int rep = 0; rep < launches; ++rep) {   // the last launch is the one reported: clocks have settled by then
    PROBE_TRY(hipEventRecord(e0, nullptr));
    hipLaunchKernelGGL(mfma_loop, dim3(blocks), dim3(256), 0, nullptr, out, clk, iters, random_operands ? 1 : 0);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipEventRecord(e1, nullptr));
    PROBE_TRY(hipEventSynchronize(e1));
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  }
  unsigned long long h[2] = {0, 1};
  PROBE_TRY(hipMemcpy(h, clk, sizeof h, hipMemcpyDeviceToHost));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(out);
  (void)hipFree(clk);
  const double flop = (double)blocks * 4 /* waves */ * (double)iters * kChains * 2.0 * 32 * 32 * 16;
  *tflops = flop / ((double)ms * 1e-3) / 1e12;
  if (shader_mhz) *shader_mhz = (double)h[0] / (double)h[1] * 100.0;   // wall_clock64 counts at 100 MHz
  return 0;
}
