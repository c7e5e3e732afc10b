// Sparse output projection (GEMM-O of the paper, Section 3.5, Observation 3 / Equations 3-4) for gfx950.
//
// Out[b, token, n] = addend[b, token, n] + bias[n] + sum over SELECTED heads h of O[b,h,token,:] . W[n, h*D:(h+1)*D]
// where, for the token block i the token lies in, head h is selected when its cache flag equals
// `select`.  The paper's two stages are two calls: stage 1 at an Update step (select = flag set,
// no addend) produces the cached bias B_c, the part of the projection that comes from heads whose
// attention output is reused; stage 2 at every step (select = flag clear, addend = B_c) adds the
// heads that were really computed.  The skipping is along the REDUCTION axis: the K loop of a tile
// walks a bitmap of that token block's selected heads (built with one wave ballot, walked with
// scalar find-first-set) and never loads the O or W columns of the others.
//
// The addend may also be given as the stored terms of the cached bias and their weights: the kernel then forms
// OP_reuse(B_c) = sum_d coef[d] * terms[d] itself while it fetches them (fp32, term order, rounded to bf16 exactly
// as the stand-alone element-wise kernel rounds it), so a Dispatch step needs no separate pass that writes the
// forecast bias and reads it back.  A token block none of whose heads is selected only streams: addend + bias.
//
// One workgroup per (token block, 128 output channels) tile; transposed MFMA product as in the
// query projection (A = weight rows, B = token rows, both k-contiguous in LDS), direct-to-LDS
// loads, 64 reduction channels per stage, double buffered.
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
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define LDS_PTR(T) T __attribute__((address_space(3)))*

constexpr int kBN = 128;                   // output channels per workgroup
constexpr int kMaxTerms = 4;               // stored feature + up to three derivatives

struct GemmOParams {
  const char* O;         // bf16 [B, H, L, D]
  const char* W;         // bf16 [C_out, H*D]
  const uint16_t* bias;  // bf16 [C_out] or nullptr
  const uint8_t* flags;  // [B, H, Tq] or nullptr
  const char* addend;    // bf16 [B, L, C_out] or nullptr; with n_terms > 0: the first term
  char* Out;             // bf16 [B, L, C_out]
  int H, L, Tq, C_out, select;
  // OP_reuse of the cached bias fused into the addend: addend = sum_d coef[d] * term[d], term[0] = `addend`
  const char* term[kMaxTerms - 1];
  float coef[kMaxTerms];
  int n_terms;           // 0: `addend` is taken as it is
};

__device__ __forceinline__ float bf16_bits_to_float(unsigned bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}

template <int BQ, int D>
__global__ void __launch_bounds__((BQ / 64) * 2 * 64, 2) gemm_o_kernel(const GemmOParams p) {
  constexpr int WM = BQ / 64;              // waves along tokens
  constexpr int WN = kBN / 64;             // waves along output channels
  constexpr int NWAVES = WM * WN;
  constexpr int PARTS = D / kStepK;        // stages per head
  using Stage = sa_gemm::Stages<kBN, BQ, NWAVES>;   // weight rows = the tile's output channels, token rows = the block

  // column tile fastest: the 8 XCDs (workgroup n runs on XCD n mod 8) each keep the weight rows of a
  // fixed set of column tiles in their L2 while the token blocks stream past
  const int ncol = p.C_out / kBN;
  const int t = blockIdx.x;
  const int col = t % ncol;
  const int i = (t / ncol) % p.Tq;
  const int b = t / (ncol * p.Tq);

  extern __shared__ __attribute__((aligned(1024))) char smem[];   // W stage 0, W stage 1, O stage 0, O stage 1
  const unsigned lds_base = (unsigned)(uintptr_t)(LDS_PTR(char))smem;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int l32 = lane & 31, half = lane >> 5;

  // reduction-axis symbol of this token block: one bit per head, set = visit
  unsigned long long heads;
  {
    bool mine = false;
    if (lane < p.H) {
      const int flag = p.flags ? (p.flags[((size_t)b * p.H + lane) * p.Tq + i] != 0) : 0;
      mine = flag == p.select;
    }
    heads = __builtin_amdgcn_ballot_w64(mine);
  }

  const size_t w_pitch = (size_t)p.H * D * 2;
  const char* gW = p.W + (size_t)col * kBN * w_pitch;
  const char* gO = p.O + ((size_t)b * p.H * p.L + (size_t)i * BQ) * (size_t)(D * 2);   // head 0; head h adds h*L*D*2

  // the last token block may be short: loads of missing rows re-read the last row that exists, their results
  // are never stored
  const int rows_valid = min(BQ, p.L - i * BQ);
  Stage st;
  st.init(lds_base, wave, lane, wn, wm, w_pitch, (size_t)(D * 2), rows_valid);
  auto issue = [&](int h, int part, auto stage_c) {
    st.template issue<decltype(stage_c)::value>(gW + ((size_t)h * D + (size_t)part * kStepK) * 2,
                                                gO + (size_t)h * p.L * (D * 2) + (size_t)part * kRowB);
  };

  f32x16 acc[2][2];   // [output-channel block][token block] of this wave's 64x64 corner
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][c][e] = 0.f;

  auto compute = [&](auto stage_c) { st.template mfma<decltype(stage_c)::value>(smem, acc); };

  // Output side.  The result tile leaves through LDS so that a lane writes 16 contiguous bytes of a
  // token's row (and reads the addend the same way): thread -> (token, group of 8 output channels).
  constexpr int NT = NWAVES * 64;
  constexpr int OUT_ITERS = BQ * 16 / NT;
  const int out_g = tid % 16;              // 8-channel group inside the 128-channel tile
  const size_t out_row0 = (size_t)b * p.L + (size_t)i * BQ;
  auto out_offset = [&](int it) -> size_t {
    const int token = it * (NT / 16) + tid / 16;
    return ((out_row0 + token) * p.C_out + col * kBN + out_g * 8) * 2;
  };
  u32x4 add_bits[OUT_ITERS];
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (p.bias) {
#pragma unroll
    for (int e = 0; e < 8; ++e) bv[e] = bf16_bits_to_float(p.bias[col * kBN + out_g * 8 + e]);
  }
  // accumulated channels v[0..7] of one token + bias + addend -> 16 bytes of bf16
  auto finish = [&](int it, float (&v)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += bv[e];
    if (p.addend) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] += bf16_bits_to_float(add_bits[it][e] & 0xffffu);
        v[2 * e + 1] += bf16_bits_to_float(add_bits[it][e] >> 16);
      }
    }
    u32x4 pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bf16x2 pr;
      pr[0] = (__bf16)v[2 * e];
      pr[1] = (__bf16)v[2 * e + 1];
      pk[e] = __builtin_bit_cast(unsigned, pr);
    }
    // streamed once: non-temporal, so that it does not push the weight rows out of the XCD's L2
    if (it * (NT / 16) + tid / 16 < rows_valid) __builtin_nontemporal_store(pk, (u32x4*)(p.Out + out_offset(it)));
  };
  // The addend (cached bias) is requested right after the first stage of the reduction loop: the stage's data comes
  // from L2 and is needed first, the addend comes from HBM and is needed last, and loads return in order.
  auto fetch_addend = [&]() {
    if (p.addend) {
#pragma unroll
      for (int it = 0; it < OUT_ITERS; ++it)
        if (it * (NT / 16) + tid / 16 < rows_valid)
          add_bits[it] = __builtin_nontemporal_load((const u32x4*)(p.addend + out_offset(it)));
      if (p.n_terms > 0) {
        // OP_reuse(B_c): fp32 sum of the scaled terms in term order, one rounding to bf16 (what the element-wise
        // kernel computes), kept packed like a plain addend
#pragma unroll
        for (int it = 0; it < OUT_ITERS; ++it) {
          if (it * (NT / 16) + tid / 16 >= rows_valid) continue;
          float v[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[2 * e] = p.coef[0] * bf16_bits_to_float(add_bits[it][e] & 0xffffu);
            v[2 * e + 1] = p.coef[0] * bf16_bits_to_float(add_bits[it][e] >> 16);
          }
          for (int d = 1; d < p.n_terms; ++d) {
            const u32x4 tb = __builtin_nontemporal_load((const u32x4*)(p.term[d - 1] + out_offset(it)));
            const float cd = p.coef[d];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              v[2 * e] = fmaf(cd, bf16_bits_to_float(tb[e] & 0xffffu), v[2 * e]);
              v[2 * e + 1] = fmaf(cd, bf16_bits_to_float(tb[e] >> 16), v[2 * e + 1]);
            }
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            bf16x2 pr;
            pr[0] = (__bf16)v[2 * e];
            pr[1] = (__bf16)v[2 * e + 1];
            add_bits[it][e] = __builtin_bit_cast(unsigned, pr);
          }
        }
      }
    }
  };
  if (heads == 0ull) {
    // no head of this token block is selected: the tile is addend + bias, straight from registers
    fetch_addend();
#pragma unroll
    for (int it = 0; it < OUT_ITERS; ++it) {
      float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      finish(it, v);
    }
    return;
  }

  // scalar walk over the selected heads, PARTS stages per head
  int h = heads ? __builtin_ctzll(heads) : -1;
  int part = 0;
  auto advance = [&](int& nh, int& npart) {
    nh = h;
    npart = part + 1;
    if (npart == PARTS) {
      npart = 0;
      heads &= heads - 1ull;
      nh = heads ? __builtin_ctzll(heads) : -1;
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  bool first = true;
  auto step = [&](auto cur, auto other) {
    int nh, npart;
    advance(nh, npart);
    // stage 0 has landed; the addend's OUT_ITERS requests, issued after it, may still be out.  Only where every
    // wave has issued all of them: in a short last block a wave skips those of rows that do not exist.
    if (first && p.addend && p.n_terms == 0 && rows_valid == BQ)
      sa_wait_vmem_but<OUT_ITERS>();
    else
      sa_wait_vmem();
    first = false;
    __syncthreads();   // this stage has landed for every wave; the other buffer is free
    if (nh >= 0) issue(nh, npart, other);
    compute(cur);
    h = nh;
    part = npart;
  };
  issue(h, 0, S0{});
  fetch_addend();
  while (h >= 0) {
    step(S0{}, S1{});
    if (h < 0) break;
    step(S1{}, S0{});
  }

  // epilogue, part 1: the accumulators (lane = token l32 + 32*c, registers = output channels
  // 32*a + 8*q4 + 4*half + 0..3 of this wave's corner) go to LDS as fp32 rows of 512 bytes, 16-byte
  // chunks XOR-permuted by the token so that the 32 tokens of a store hit different banks
  __syncthreads();   // every wave is done reading the stage buffers
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int token = wm * 64 + 32 * c + l32;
        const int chunk = wn * 16 + 8 * a + 2 * q4 + half;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[a][c][4 * q4 + e];
        *(f32x4*)(smem + token * 512 + ((chunk ^ (token & 31)) * 16)) = v;
      }
  __syncthreads();
  // part 2: row-contiguous read back, + bias + addend, round to bf16, 16-byte stores
#pragma unroll
  for (int it = 0; it < OUT_ITERS; ++it) {
    const int token = it * (NT / 16) + tid / 16;
    const f32x4 v0 = *(const f32x4*)(smem + token * 512 + (((2 * out_g) ^ (token & 31)) * 16));
    const f32x4 v1 = *(const f32x4*)(smem + token * 512 + (((2 * out_g + 1) ^ (token & 31)) * 16));
    float v[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = v0[e];
      v[4 + e] = v1[e];
    }
    finish(it, v);
  }
}

template <int BQ, int D>
int launch(const GemmOParams& p, int tiles, hipStream_t stream) {
  constexpr size_t lds = sa_gemm::Stages<kBN, BQ, (BQ / 64) * (kBN / 64)>::kLdsBytes;
  constexpr int threads = (BQ / 64) * 2 * 64;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute((const void*)gemm_o_kernel<BQ, D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr_err != hipSuccess)
    return sa_fail(SPARSE_ATTN_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr_err));
  hipLaunchKernelGGL((gemm_o_kernel<BQ, D>), dim3(tiles), dim3(threads), lds, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "gemm_o launch failed: %s", hipGetErrorString(e));
  return 0;
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

}  // namespace

namespace {

int gemm_o_run(const void* O, const void* W, const void* bias, const uint8_t* cache_flags, int select_cached,
               const void* addend, const void* const* terms, const float* coef, int n_terms, void* Out, int B, int H,
               int L, int D, int C_out, int block_q, hipStream_t stream) {
  if (B <= 0 || H <= 0 || L <= 0 || D <= 0 || C_out <= 0 || block_q <= 0)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: sizes must be positive (B=%d H=%d L=%d D=%d C_out=%d block_q=%d)",
                   B, H, L, D, C_out, block_q);
  if (select_cached != 0 && select_cached != 1)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: select_cached must be 0 or 1 (got %d)", select_cached);
  if ((D != 64 && D != 128) || (block_q != 64 && block_q != 128))
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: D and block_q must be 64 or 128 (got %d, %d)", D, block_q);
  if (H > 64) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: at most 64 heads (got %d)", H);
  if (C_out % kBN)
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: C_out=%d must be a multiple of %d", C_out, kBN);
  if ((long long)kBN * H * D * 2 >= (1LL << 31)) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: H*D too large");
  const int tq = (L + block_q - 1) / block_q;      // a short last block counts as a block
  const long long tiles = (long long)B * tq * (C_out / kBN);
  if (tiles > 0x3fffffffLL) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: too many tiles (%lld)", tiles);
  if (!O || !W || !Out) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: O, W and Out must not be NULL");
  if (((uintptr_t)O | (uintptr_t)W | (uintptr_t)Out | (uintptr_t)addend) & 15)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: O, W, addend and Out must be 16-byte aligned");
  const size_t ob = (size_t)B * H * L * D * 2, wb = (size_t)C_out * H * D * 2, outb = (size_t)B * L * C_out * 2;
  if (ranges_overlap(Out, outb, O, ob) || ranges_overlap(Out, outb, W, wb))
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: Out must not overlap O or W");
  if (addend && addend != Out && ranges_overlap(Out, outb, addend, outb))
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: addend must be Out itself or must not overlap Out");

  GemmOParams p;
  p.O = (const char*)O;
  p.W = (const char*)W;
  p.bias = (const uint16_t*)bias;
  p.flags = cache_flags;
  p.addend = (const char*)addend;
  p.Out = (char*)Out;
  p.H = H;
  p.L = L;
  p.Tq = tq;
  p.C_out = C_out;
  p.select = select_cached;
  p.n_terms = 0;
  for (int d = 0; d < kMaxTerms; ++d) p.coef[d] = 0.f;
  for (int d = 0; d + 1 < kMaxTerms; ++d) p.term[d] = nullptr;
  if (terms) {
    if (n_terms < 1 || n_terms > kMaxTerms)
      return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "gemm_o: n_terms=%d must be between 1 and %d", n_terms, kMaxTerms);
    if (!coef) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: coef must not be NULL");
    for (int d = 0; d < n_terms; ++d) {
      if (!terms[d]) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: terms[%d] must not be NULL", d);
      if ((uintptr_t)terms[d] & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: terms[%d] must be 16-byte aligned", d);
      if (terms[d] != Out && ranges_overlap(Out, outb, terms[d], outb))
        return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: terms[%d] must be Out itself or must not overlap Out", d);
      if (!(coef[d] == coef[d]) || coef[d] - coef[d] != 0.f)
        return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: coef[%d] must be finite", d);
    }
    p.addend = (const char*)terms[0];
    if (!(n_terms == 1 && coef[0] == 1.0f)) {      // one term with weight 1 is the plain addend
      p.n_terms = n_terms;
      for (int d = 0; d < n_terms; ++d) p.coef[d] = coef[d];
      for (int d = 1; d < n_terms; ++d) p.term[d - 1] = (const char*)terms[d];
    }
  }
  if (block_q == 128 && D == 128) return launch<128, 128>(p, (int)tiles, stream);
  if (block_q == 128 && D == 64) return launch<128, 64>(p, (int)tiles, stream);
  if (block_q == 64 && D == 128) return launch<64, 128>(p, (int)tiles, stream);
  return launch<64, 64>(p, (int)tiles, stream);
}

}  // namespace

extern "C" {

int sparse_gemm_o_stream(const void* O, const void* W, const void* bias, const uint8_t* cache_flags,
                         int select_cached, const void* addend, void* Out, int B, int H, int L, int D, int C_out,
                         int block_q, void* hip_stream) {
  return gemm_o_run(O, W, bias, cache_flags, select_cached, addend, nullptr, nullptr, 0, Out, B, H, L, D, C_out, block_q,
                    (hipStream_t)hip_stream);
}

int sparse_gemm_o(const void* O, const void* W, const void* bias, const uint8_t* cache_flags, int select_cached,
                  const void* addend, void* Out, int B, int H, int L, int D, int C_out, int block_q) {
  return sparse_gemm_o_stream(O, W, bias, cache_flags, select_cached, addend, Out, B, H, L, D, C_out, block_q, nullptr);
}

int sparse_gemm_o_reuse(const void* O, const void* W, const void* bias, const uint8_t* cache_flags,
                        const void* const* terms, const float* coef, int n_terms, void* Out, int B, int H, int L, int D,
                        int C_out, int block_q, void* hip_stream) {
  if (!terms) return sa_fail(SPARSE_ATTN_ERR_INVALID, "gemm_o: terms must not be NULL");
  return gemm_o_run(O, W, bias, cache_flags, 0, nullptr, terms, coef, n_terms, Out, B, H, L, D, C_out, block_q,
                    (hipStream_t)hip_stream);
}

}  // extern "C"
