// Bench-side measurement helper -- NOT part of the product library and not part of the method.
//
// The rate this device sustains on a loop of nothing but v_mfma_f32_32x32x16_bf16 (the instruction the attention
// and projection kernels run on), two waves per SIMD, with operands that are either constant or random, and the
// shader clock it runs at meanwhile.  bench.py reports the attention kernel against this rate next to the nominal
// peak: the clock a power-limited chip sustains under matrix load depends on the operand data.
// Built by __graft_entry__.build() into bench_mfma_probe.so beside bench.py; loaded by bench.py only.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace

// Runs `launches` (1..64) launches of about 10 ms each on the null stream of the current device and reports the
// last one (the clock has settled by then): tflops (host, required) and shader_mhz (host, may be NULL).
// Returns 0, -1 for bad arguments, or the positive hipError_t of the call that failed.
extern "C" int bench_mfma_probe(int random_operands, int launches, double* tflops, double* shader_mhz) {
  if (launches < 1 || launches > 64 || !tflops) return -1;
  float* out = nullptr;
  unsigned long long* clk = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t err = hipSuccess;
  int dev = 0, cus = 0;
  float ms = 0.f;
  unsigned long long h[2] = {0, 1};
  int blocks = 0;
  const int iters = 100000;
#define PROBE_TRY(expr) do { err = (expr); if (err != hipSuccess) goto done; } while (0)
  PROBE_TRY(hipGetDevice(&dev));
  PROBE_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  blocks = 2 * cus;   // 8 waves per CU, two per SIMD
  PROBE_TRY(hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)));
  PROBE_TRY(hipMalloc(&clk, (size_t)blocks * 2 * sizeof(unsigned long long)));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  for (int rep = 0; rep < launches; ++rep) {
    PROBE_TRY(hipEventRecord(e0, nullptr));
    hipLaunchKernelGGL(mfma_loop, dim3(blocks), dim3(256), 0, nullptr, out, clk, iters, random_operands ? 1 : 0);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipEventRecord(e1, nullptr));
    PROBE_TRY(hipEventSynchronize(e1));
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
  }
  PROBE_TRY(hipMemcpy(h, clk, sizeof h, hipMemcpyDeviceToHost));
  *tflops = (double)blocks * 4 /* waves */ * (double)iters * kChains * 2.0 * 32 * 32 * 16 / ((double)ms * 1e-3) / 1e12;
  if (shader_mhz) *shader_mhz = (double)h[0] / (double)h[1] * 100.0;   // wall_clock64 counts at 100 MHz
#undef PROBE_TRY
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (out) (void)hipFree(out);
  if (clk) (void)hipFree(clk);
  return (int)err;
}
