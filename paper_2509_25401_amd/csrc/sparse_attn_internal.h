// Shared between the translation units of the library (not part of the public ABI).
#ifndef SPARSE_ATTN_INTERNAL_H
#define SPARSE_ATTN_INTERNAL_H

#include <hip/hip_runtime.h>

// Records a printf-style message for sparse_attn_last_error() on the calling thread and returns `code`.
int sa_fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// The library's scratch buffer of the current device and `stream`, grown (with a stream synchronisation) to at
// least `need` bytes.  Every entry point that needs scratch memory shares it: work on one stream runs in
// order, and no entry point keeps anything in it between calls.
int sa_get_scratch(size_t need, hipStream_t stream, void** out);

// Direct-to-LDS load: every lane fetches 16 bytes from gbase (wave-uniform) + lane_off, the wave's
// 1 KiB lands at consecutive LDS addresses starting at the wave-uniform `lds_addr`.  Written as
// inline assembly so that the compiler does not serialise later LDS reads of the OTHER buffer
// behind these loads (it cannot tell the two buffers apart); the kernels wait for them themselves
// (s_waitcnt vmcnt(0) + barrier) before the buffer is read.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void sa_load_to_lds_16B(const char* gbase, unsigned lane_off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(lane_off), "s"(gbase)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// A wave-uniform pointer that the compiler may have left in vector registers, moved to scalar registers.
__device__ __forceinline__ const char* sa_uniform_ptr(const char* ptr) {
  const unsigned long long v = (unsigned long long)ptr;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const char*)(((unsigned long long)hi << 32) | lo);
}

// s_waitcnt vmcnt(0) only: expcnt and lgkmcnt fields left at their maxima
__device__ __forceinline__ void sa_wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// s_waitcnt vmcnt(N): at most the N newest vector-memory requests of the wave are still outstanding (loads
// return in order).  The six-bit count is split over bits 3:0 and 15:14 of the immediate.
template <int N>
__device__ __forceinline__ void sa_wait_vmem_but() {
  static_assert(N >= 0 && N < 64, "vmcnt is a six-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// ---------------------------------------------------------------------------------------
// Operand staging of the two projection kernels (query and output projection).
//
// Both compute a transposed product C^T[n][token] = sum_k W[n][k] X[token][k] with
// v_mfma_f32_32x32x16_bf16 (A = weight rows, B = token rows, both k-contiguous) and stream the
// operands through two LDS buffers, kStepK reduction channels per stage.  A stage holds W_ROWS
// weight rows and X_ROWS token rows of kRowB bytes; LDS layout: W stage 0, W stage 1, X stage 0,
// X stage 1.  The 16-byte chunks of a row are permuted by row_swizzle so that the operand reads of a
// wave spread over all banks; a direct-to-LDS load writes consecutive LDS, so the permutation is
// applied to the global address each lane fetches.  Every wave owns a 64 x 64 corner of the
// tile: [2 blocks of 32 output channels][2 blocks of 32 tokens] accumulators.
// ---------------------------------------------------------------------------------------
namespace sa_gemm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kStepK = 64;          // reduction channels per LDS stage
constexpr int kRowB = kStepK * 2;   // bytes per tile row in LDS

// 16-byte chunk permutation of a 128-byte tile row (two rows share a 256-byte bank line)
__device__ __forceinline__ int row_swizzle(int row) { return (row >> 1) & 7; }

template <int W_ROWS, int X_ROWS, int NWAVES>
struct Stages {
  static constexpr int W_TILEB = W_ROWS * kRowB;            // bytes of one weight stage
  static constexpr int X_TILEB = X_ROWS * kRowB;            // bytes of one token stage
  static constexpr int W_LOAD = W_TILEB / 1024 / NWAVES;    // direct-to-LDS wave instructions per stage and wave
  static constexpr int X_LOAD = X_TILEB / 1024 / NWAVES;
  static constexpr int kLdsBytes = 2 * (W_TILEB + X_TILEB);
  static_assert((W_TILEB / 1024) % NWAVES == 0 && (X_TILEB / 1024) % NWAVES == 0, "stage loads must split evenly over the waves");

  unsigned w_goff[W_LOAD], x_goff[X_LOAD];   // per-lane global offsets of this wave's stage loads (8 rows per instruction)
  int w_off[kStepK / 16], x_off[kStepK / 16];   // per-lane LDS offsets of the operand reads, k-step ks
  unsigned lds_base;
  int wave;

  // wn / wm: this wave's 64-channel / 64-token corner; w_pitch / x_pitch: bytes between rows of the operands in
  // memory; token rows from x_rows_valid on do not exist (short last block): their loads re-read the last row that
  // does, and the caller never stores their results.
  __device__ __forceinline__ void init(unsigned lds_base_, int wave_, int lane, int wn, int wm, size_t w_pitch,
                                       size_t x_pitch, int x_rows_valid) {
    lds_base = lds_base_;
    wave = wave_;
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int u = 0; u < W_LOAD; ++u) {
      const int r = (wave + u * NWAVES) * 8 + lane / 8;
      w_goff[u] = (unsigned)(r * w_pitch + (((lane % 8) ^ row_swizzle(r)) * 16));
    }
#pragma unroll
    for (int u = 0; u < X_LOAD; ++u) {
      const int r = (wave + u * NWAVES) * 8 + lane / 8;
      x_goff[u] = (unsigned)(min(r, x_rows_valid - 1) * x_pitch + (((lane % 8) ^ row_swizzle(r)) * 16));
    }
#pragma unroll
    for (int ks = 0; ks < kStepK / 16; ++ks) {
      const int o = l32 * kRowB + (((2 * ks + half) ^ row_swizzle(l32)) * 16);
      w_off[ks] = wn * 64 * kRowB + o;
      x_off[ks] = 2 * W_TILEB + wm * 64 * kRowB + o;
    }
  }

  // Requests one stage: w_src / x_src point at the first row's channels of this stage (wave-uniform).
  template <int STAGE>
  __device__ __forceinline__ void issue(const char* w_src, const char* x_src) const {
#pragma unroll
    for (int u = 0; u < W_LOAD; ++u)
      sa_load_to_lds_16B(w_src, w_goff[u], lds_base + (unsigned)(STAGE * W_TILEB + (wave + u * NWAVES) * 1024));
#pragma unroll
    for (int u = 0; u < X_LOAD; ++u)
      sa_load_to_lds_16B(x_src, x_goff[u], lds_base + (unsigned)(2 * W_TILEB + STAGE * X_TILEB + (wave + u * NWAVES) * 1024));
  }

  // The 16 MFMAs of one stage on this wave's corner.  The stage is a compile-time constant, so every LDS address
  // is a lane register plus an immediate; all 16 operand reads are issued before the first MFMA, which then only
  // waits for its own two operands.
  template <int STAGE>
  __device__ __forceinline__ void mfma(const char* smem, f32x16 (&acc)[2][2]) const {
    bf16x8 wa[kStepK / 16][2], xb[kStepK / 16][2];
#pragma unroll
    for (int ks = 0; ks < kStepK / 16; ++ks) {
#pragma unroll
      for (int a = 0; a < 2; ++a) wa[ks][a] = *(const bf16x8*)(smem + STAGE * W_TILEB + a * 32 * kRowB + w_off[ks]);
#pragma unroll
      for (int c = 0; c < 2; ++c) xb[ks][c] = *(const bf16x8*)(smem + STAGE * X_TILEB + c * 32 * kRowB + x_off[ks]);
    }
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int ks = 0; ks < kStepK / 16; ++ks)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
          acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[ks][a], xb[ks][c], acc[a][c], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  }
};

}  // namespace sa_gemm

#endif
