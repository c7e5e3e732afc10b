// Sparse query projection (GEMM-Q of the paper, Section 3.5, Observation 2 / Equation 2) for gfx950.
//
// Q[b,h,i-th block,:] = X[b, i-th block, :] . W_h^T (+ bias_h) for every (b,h,i) whose cache flag
// is clear; a workgroup whose tile is flagged returns at once (its attention output is reused from
// the cache, so its queries are never read).  One workgroup per (query block, head) output tile, the
// same granularity as the flags, written straight into the [B,H,L,D] layout the attention kernel
// reads.  The product is computed transposed, C^T[d][token] = sum_k W[d][k] X[token][k], with
// v_mfma_f32_32x32x16_bf16: both operands are "k contiguous" rows (A = weight rows, B = token
// rows), so both come out of LDS with plain 16-byte reads, and a lane ends up holding 4 consecutive
// d of one token, which stores as 8 bytes.  X and W tiles stream to LDS with direct-to-LDS loads,
// 64 channels per stage, double buffered.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "sparse_attn.h"
#include "sparse_attn_internal.h"

namespace {

using sa_gemm::f32x16;
using sa_gemm::kRowB;
using sa_gemm::kStepK;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define LDS_PTR(T) T __attribute__((address_space(3)))*

struct GemmQParams {
  const char* X;       // bf16 [B, L, C]
  const char* W;       // bf16 [H*D, C]
  const uint16_t* bias;  // bf16 [H*D] or nullptr
  const uint8_t* flags;  // [B, H, Tq] or nullptr
  char* Q;             // bf16 [B, H, L, D]
  int H, L, C, Tq;
  // fused epilogue (NORM_ROPE instantiations only)
  const uint16_t* norm_w;   // bf16 [D] or nullptr (= ones)
  const float* rope_cos;    // fp32 [L, D/2] or nullptr (= no rotation)
  const float* rope_sin;
  float eps;
};

template <int BQ, int D, bool NORM_ROPE>
__global__ void __launch_bounds__((BQ / 64) * (D / 64) * 64, 2) gemm_q_kernel(const GemmQParams p) {
  constexpr int WM = BQ / 64;              // waves along tokens
  constexpr int WN = D / 64;               // waves along head channels
  constexpr int NWAVES = WM * WN;
  using Stage = sa_gemm::Stages<D, BQ, NWAVES>;   // weight rows = the head's D channels, token rows = the query block
  constexpr int TS = D / 2 + 2;            // padded row of the cos / sin tiles in LDS (floats)

  // tile of this workgroup: head fastest, so the 8 XCDs (workgroup n runs on XCD n mod 8) each keep
  // the weights of a fixed set of heads in their L2
  const int t = blockIdx.x;
  const int h = t % p.H;
  const int i = (t / p.H) % p.Tq;
  const int b = t / (p.H * p.Tq);
  if (p.flags && p.flags[((size_t)b * p.H + h) * p.Tq + i]) return;   // spatial-axis symbol says: cached

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // layout: W stage 0, W stage 1, X stage 0, X stage 1
  const unsigned lds_base = (unsigned)(uintptr_t)(LDS_PTR(char))smem;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int l32 = lane & 31, half = lane >> 5;

  const size_t row_pitch = (size_t)p.C * 2;
  const char* gW = p.W + (size_t)h * D * row_pitch;
  const char* gX = p.X + ((size_t)b * p.L + (size_t)i * BQ) * row_pitch;
  // the last token block may be short: loads of missing rows re-read the last row that exists, their results
  // are never stored
  const int rows_valid = min(BQ, p.L - i * BQ);

  Stage st;
  st.init(lds_base, wave, lane, wn, wm, row_pitch, row_pitch, rows_valid);
  auto issue = [&](int kstep, auto stage_c) {
    st.template issue<decltype(stage_c)::value>(gW + (size_t)kstep * kRowB, gX + (size_t)kstep * kRowB);
  };

  f32x16 acc[2][2];   // [d block][token block] of this wave's 64x64 corner
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

  auto compute = [&](auto stage_c) { st.template mfma<decltype(stage_c)::value>(smem, acc); };

  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  const int nk = p.C / kStepK;
  issue(0, S0{});
  int k = 0;
  for (; k + 1 < nk; k += 2) {   // two stages per trip, one per LDS buffer
    sa_wait_vmem();   // this wave's part of the stage has landed
    __syncthreads();
    issue(k + 1, S1{});
    compute(S0{});
    sa_wait_vmem();
    __syncthreads();
    if (k + 2 < nk) issue(k + 2, S0{});
    compute(S1{});
  }
  if (k < nk) {                  // odd number of stages: the last one sits in buffer 0
    sa_wait_vmem();
    __syncthreads();
    compute(S0{});
  }

  // epilogue: lane holds token l32 (+32*c) and, per accumulator quad q4, head channels
  // 32*a + 8*q4 + 4*half + 0..3 of this wave's corner
  float inv_rms[2] = {1.f, 1.f};
  if constexpr (NORM_ROPE) {
    // Equation 2: token-wise RMS normalisation over the head's D channels, then the rotation.  The bias
    // goes into the accumulators first; a token's sum of squares is spread over this lane's 32 values,
    // the lane 32 further on, and (D = 128) the wave that holds the other 64 channels.
    if (p.bias) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float bv = __builtin_bit_cast(float, (unsigned)p.bias[h * D + wn * 64 + 32 * a + 8 * q4 + 4 * half + e] << 16);
            acc[a][0][4 * q4 + e] += bv;
            acc[a][1][4 * q4 + e] += bv;
          }
    }
    // The tile's cos / sin rows (one contiguous block of the tables) come through LDS: read straight
    // from memory in the accumulator layout, every lane would fetch 8 bytes from its own 256-byte row,
    // 64 dependent round trips per lane.  The operand stages are dead by now; rows are padded by two
    // floats so that 32 lanes reading 8 bytes of 32 rows hit 64 different banks.
    __syncthreads();                           // every wave is done reading the operand stages
    float* tab = (float*)smem;                 // cos [BQ][TS], then sin [BQ][TS], then the sums [WN][BQ]
    if (p.rope_cos) {
      constexpr int NV = BQ * (D / 2) / 4;     // 16-byte pieces per table
      const float4* gc = (const float4*)(p.rope_cos + (size_t)i * BQ * (D / 2));
      const float4* gs = (const float4*)(p.rope_sin + (size_t)i * BQ * (D / 2));
      for (int e = tid; e < NV; e += NWAVES * 64) {
        const bool there = (4 * e) / (D / 2) < rows_valid;          // the tables have L rows
        const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 vc = there ? gc[e] : zero, vs = there ? gs[e] : zero;
        const int o = (4 * e) / (D / 2) * TS + (4 * e) % (D / 2);
        *(float2*)(tab + o) = make_float2(vc.x, vc.y);
        *(float2*)(tab + o + 2) = make_float2(vc.z, vc.w);
        *(float2*)(tab + BQ * TS + o) = make_float2(vs.x, vs.y);
        *(float2*)(tab + BQ * TS + o + 2) = make_float2(vs.z, vs.w);
      }
    }
    float ss[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      float v = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) v = fmaf(acc[a][c][e], acc[a][c][e], v);
      ss[c] = v + __shfl_xor(v, 32);
    }
    float* part = tab + 2 * BQ * TS;           // [WN][BQ]
    if (WN == 2 && half == 0) {
      part[wn * BQ + wm * 64 + l32] = ss[0];
      part[wn * BQ + wm * 64 + 32 + l32] = ss[1];
    }
    __syncthreads();                           // tables and partial sums are in place
    if constexpr (WN == 2) {
      ss[0] = part[wm * 64 + l32] + part[BQ + wm * 64 + l32];
      ss[1] = part[wm * 64 + 32 + l32] + part[BQ + wm * 64 + 32 + l32];
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) inv_rms[c] = 1.0f / sqrtf(ss[c] * (1.0f / D) + p.eps);
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d0 = wn * 64 + 32 * a + 8 * q4 + 4 * half;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      float gain[4] = {1.f, 1.f, 1.f, 1.f};
      if constexpr (NORM_ROPE) {
        if (p.norm_w) {
#pragma unroll
          for (int e = 0; e < 4; ++e) gain[e] = __builtin_bit_cast(float, (unsigned)p.norm_w[d0 + e] << 16);
        }
      } else if (p.bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          bv[e] = __builtin_bit_cast(float, (unsigned)p.bias[h * D + d0 + e] << 16);
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = acc[a][c][4 * q4 + e] + bv[e];
        if constexpr (NORM_ROPE) {
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = y[e] * inv_rms[c] * gain[e];
          if (p.rope_cos) {
            // channels d0..d0+3 are the pairs d0/2 and d0/2 + 1 of this token
            const float* tab = (const float*)smem;
            const int at = (wm * 64 + 32 * c + l32) * TS + d0 / 2;
            const float2 cs = *(const float2*)(tab + at);
            const float2 sn = *(const float2*)(tab + BQ * TS + at);
            const float y0 = y[0] * cs.x - y[1] * sn.x, y1 = y[0] * sn.x + y[1] * cs.x;
            const float y2 = y[2] * cs.y - y[3] * sn.y, y3 = y[2] * sn.y + y[3] * cs.y;
            y[0] = y0; y[1] = y1; y[2] = y2; y[3] = y3;
          }
        }
        // the finished values go back into the accumulator registers; they leave through LDS below
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[a][c][4 * q4 + e] = y[e];
      }
    }
  // Output side.  A lane holds 4 channels of one token: written from here a store would be 8 bytes per lane, 256
  // bytes apart.  The tile goes through LDS instead (rows of D bf16, 16-byte chunks XOR-permuted by the token so that
  // the 32 tokens of a write hit different banks) and leaves as whole rows, 16 bytes per lane, with non-temporal
  // stores: the projection writes its result once and must not push the weights and token rows out of L2 with it.
  constexpr int ROWB_OUT = D * 2;            // bytes per token row of the tile
  constexpr int CH = ROWB_OUT / 16;          // 16-byte chunks per row
  __syncthreads();                           // every wave is done with the operand stages / the tables
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int d0 = wn * 64 + 32 * a + 8 * q4 + 4 * half;
        const int token = wm * 64 + 32 * c + l32;
        bf16x2 lo, hi;
        lo[0] = (__bf16)acc[a][c][4 * q4 + 0];
        lo[1] = (__bf16)acc[a][c][4 * q4 + 1];
        hi[0] = (__bf16)acc[a][c][4 * q4 + 2];
        hi[1] = (__bf16)acc[a][c][4 * q4 + 3];
        u32x2 pk;
        pk[0] = __builtin_bit_cast(unsigned, lo);
        pk[1] = __builtin_bit_cast(unsigned, hi);
        *(u32x2*)(smem + token * ROWB_OUT + (((d0 / 8) ^ (token & (CH - 1))) * 16) + (d0 % 8) * 2) = pk;
      }
  __syncthreads();
  constexpr int NT = NWAVES * 64;
  char* const out0 = p.Q + (((size_t)b * p.H + h) * p.L + (size_t)i * BQ) * (size_t)ROWB_OUT;
#pragma unroll
  for (int it = 0; it < BQ * CH / NT; ++it) {
    const int token = it * (NT / CH) + tid / CH, ch = tid % CH;
    const u32x4 v = *(const u32x4*)(smem + token * ROWB_OUT + ((ch ^ (token & (CH - 1))) * 16));
    if (token < rows_valid) __builtin_nontemporal_store(v, (u32x4*)(out0 + (size_t)token * ROWB_OUT + ch * 16));
  }
}

template <int BQ, int D, bool NORM_ROPE>
int launch(const GemmQParams& p, int tiles, hipStream_t stream) {
  constexpr size_t stage_lds = sa_gemm::Stages<D, BQ, (BQ / 64) * (D / 64)>::kLdsBytes;
  constexpr size_t epi_lds = NORM_ROPE ? (size_t)(2 * BQ * (D / 2 + 2) + 2 * BQ) * 4 : 0;   // cos, sin tiles + row sums
  constexpr size_t lds = stage_lds > epi_lds ? stage_lds : epi_lds;
  constexpr int threads = (BQ / 64) * (D / 64) * 64;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute((const void*)gemm_q_kernel<BQ, D, NORM_ROPE>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)lds);
  });
  if (attr_err != hipSuccess)
    return sa_fail(SPARSE_ATTN_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr_err));
  hipLaunchKernelGGL((gemm_q_kernel<BQ, D, NORM_ROPE>), dim3(tiles), dim3(threads), lds, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "gemm_q launch failed: %s", hipGetErrorString(e));
  return 0;
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

int gemm_q_run(const void* X, const void* W, const void* bias, const uint8_t* cache_flags, void* Q, int B, int L, int C,
               int H, int D, int block_q, hipStream_t stream, bool norm_rope, const void* norm_weight, float eps,
               const float* rope_cos, const float* rope_sin) {
  if (B <= 0 || L <= 0 || C <= 0 || H <= 0 || D <= 0 || block_q <= 0)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: sizes must be positive (B=%d L=%d C=%d H=%d D=%d block_q=%d)", B,
                   L, C, H, D, block_q);
  if ((D != 64 && D != 128) || (block_q != 64 && block_q != 128))
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_q: D and block_q must be 64 or 128 (got %d, %d)", D, block_q);
  if (C % kStepK) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_q: C=%d must be a multiple of %d", C, kStepK);
  if ((long long)128 * C * 2 >= (1LL << 31)) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_q: C=%d too large", C);
  const int tq = (L + block_q - 1) / block_q;      // a short last block counts as a block
  const long long tiles = (long long)B * H * tq;
  if (tiles > 0x3fffffffLL) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_q: too many tiles (%lld)", tiles);
  if (!X || !W || !Q) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: X, W and Q must not be NULL");
  if (((uintptr_t)X | (uintptr_t)W | (uintptr_t)Q) & 15)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: X, W and Q must be 16-byte aligned");
  const size_t xb = (size_t)B * L * C * 2, wb = (size_t)H * D * C * 2, qb = (size_t)B * H * L * D * 2;
  if (ranges_overlap(Q, qb, X, xb) || ranges_overlap(Q, qb, W, wb))
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: Q must not overlap X or W");
  if (norm_rope) {
    if (!(eps >= 0.f) || eps - eps != 0.f) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: eps must be finite and >= 0");
    if ((rope_cos == nullptr) != (rope_sin == nullptr))
      return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: rope_cos and rope_sin must be given together");
    if (((uintptr_t)rope_cos | (uintptr_t)rope_sin) & 7)
      return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: rope_cos and rope_sin must be 8-byte aligned");
    if ((uintptr_t)norm_weight & 1) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_q: norm_weight must be 2-byte aligned");
  }

  GemmQParams p;
  p.X = (const char*)X;
  p.W = (const char*)W;
  p.bias = (const uint16_t*)bias;
  p.flags = cache_flags;
  p.Q = (char*)Q;
  p.H = H;
  p.L = L;
  p.C = C;
  p.Tq = tq;
  p.norm_w = (const uint16_t*)norm_weight;
  p.rope_cos = rope_cos;
  p.rope_sin = rope_sin;
  p.eps = eps;
  if (norm_rope) {
    if (block_q == 128 && D == 128) return launch<128, 128, true>(p, (int)tiles, stream);
    if (block_q == 128 && D == 64) return launch<128, 64, true>(p, (int)tiles, stream);
    if (block_q == 64 && D == 128) return launch<64, 128, true>(p, (int)tiles, stream);
    return launch<64, 64, true>(p, (int)tiles, stream);
  }
  if (block_q == 128 && D == 128) return launch<128, 128, false>(p, (int)tiles, stream);
  if (block_q == 128 && D == 64) return launch<128, 64, false>(p, (int)tiles, stream);
  if (block_q == 64 && D == 128) return launch<64, 128, false>(p, (int)tiles, stream);
  return launch<64, 64, false>(p, (int)tiles, stream);
}

}  // namespace

extern "C" {

int sparse_gemm_q_stream(const void* X, const void* W, const void* bias, const uint8_t* cache_flags, void* Q, int B,
                         int L, int C, int H, int D, int block_q, void* hip_stream) {
  return gemm_q_run(X, W, bias, cache_flags, Q, B, L, C, H, D, block_q, (hipStream_t)hip_stream, false, nullptr, 0.f,
                    nullptr, nullptr);
}

int sparse_gemm_q(const void* X, const void* W, const void* bias, const uint8_t* cache_flags, void* Q, int B, int L,
                  int C, int H, int D, int block_q) {
  return sparse_gemm_q_stream(X, W, bias, cache_flags, Q, B, L, C, H, D, block_q, nullptr);
}

int sparse_gemm_q_norm_rope(const void* X, const void* W, const void* bias, const void* norm_weight, float eps,
                            const float* rope_cos, const float* rope_sin, const uint8_t* cache_flags, void* Q, int B,
                            int L, int C, int H, int D, int block_q, void* hip_stream) {
  return gemm_q_run(X, W, bias, cache_flags, Q, B, L, C, H, D, block_q, (hipStream_t)hip_stream, true, norm_weight, eps,
                    rope_cos, rope_sin);
}

}  // extern "C"
