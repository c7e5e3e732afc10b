// Sparse-symbol generation of an Update step (Section 3.3 "Logical Masks Generation", Equation 1, and
// the tau_kv / S_q rules of the settings table in the appendix) for gfx950.
//
// Three kernels, all plain fp32 vector arithmetic:
//   pool_blocks   mean of the n*b_q query rows / n*b_k key rows of every pooled block (granularity n): the only
//                 pass over Q and K, HBM-bound (reads both tensors once, 16 bytes per lane, row-contiguous)
//   map_rows      one workgroup per 8 rows of the compressed attention map of one head: scores of the
//                 pooled queries against all pooled keys (scale 1/sqrt(d)), row softmax, then for
//                 every row the block-skipping rule -- a key block is skipped iff the sum of all row
//                 entries that come at or before it in ascending order (ties by index) stays <= tau_kv
//                 -- packed most-significant-bit first into the kv_mask row.  The text rows and text
//                 columns of the map (all that the caching rule needs) go to scratch memory.
//   select_blocks one workgroup per head: contribution C_u = sum over text rows of their weight on
//                 vision key block u (carried over to the vision query blocks by token overlap when
//                 n*b_q != n*b_k), guidance G_v = sum over text columns of the softmax, along the vision
//                 axis, of the vision rows' weights on that column; Equation 1 caches v iff its
//                 ascending cumulative sums of C and of G both stay <= tau_c times the totals; text
//                 blocks are never cached; if the share of blocks left to compute drops below S_q,
//                 every block of the head is cached.
// Neither rule needs a sort.  Equation 1 (once per head): entry v adds up every entry that is smaller, or equal with
// a smaller-or-same index.  The skipping rule (once per map row): the skipped set is "everything up to a threshold
// value", found by bisection on the bits of that value.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "sparse_attn.h"
#include "sparse_attn_internal.h"

namespace {

constexpr int kMapRows = 8;          // map rows per workgroup (two per wave)
constexpr int kChunk = 32;           // pooled key rows staged in LDS per step
constexpr int kMaxBlocks = 2048;     // blocks per sequence the LDS arrays are sized for

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Sum over the 64 lanes, the same bits in every lane, without going through LDS: exchanges inside a row of 16
// lanes are DPP operands of the add, the two exchanges between rows are the gfx950 lane-swap instructions.
// Every step adds a value and its mirror partner's, so both partners compute the same sum.
__device__ __forceinline__ float wave_sum_dpp(float v) {
  auto dpp = [](float x, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xf, 0xf, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]: lane ^ 1
  v += dpp(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]: lane ^ 2
  v += dpp(v, std::integral_constant<int, 0x141>{});   // row_half_mirror: the other quad of each 8 lanes
  v += dpp(v, std::integral_constant<int, 0x140>{});   // row_mirror: the other 8 lanes of each row
  {
    const unsigned bits = __float_as_uint(v);
    const auto sw = __builtin_amdgcn_permlane16_swap(bits, bits, false, false);   // rows 0<->1, 2<->3
    v = __uint_as_float((unsigned)sw[0]) + __uint_as_float((unsigned)sw[1]);
  }
  {
    const unsigned bits = __float_as_uint(v);
    const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);   // lanes 0-31 <-> 32-63
    v = __uint_as_float((unsigned)sw[0]) + __uint_as_float((unsigned)sw[1]);
  }
  return v;
}

// Block-wide reductions for 256 threads; `red` is 4 floats of LDS.  Every thread gets the result.
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// Pooled queries [BH][Tq][D], then pooled keys [BH][Tk][D]: mean over the pooled block's rows.  Grid
// (BH * max(Tq, Tk), 2), y = 0 for Q (pool_q rows per block), 1 for K (pool_k rows per block).
template <int D>
__global__ void __launch_bounds__(256) pool_blocks(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                                                   float* __restrict__ pooled, int pool_q, int pool_k, int Tq, int Tk,
                                                   int L, long long n_q_blocks) {
  constexpr int TPR = D / 8;          // threads per row, 8 bf16 = 16 bytes each
  constexpr int RPP = 256 / TPR;      // rows per pass
  __shared__ float part[RPP][D];
  const int Tmax = max(Tq, Tk);
  const int T = blockIdx.y ? Tk : Tq, pool = blockIdx.y ? pool_k : pool_q;
  // pooled block t of head bh; the last block of a head may be short: the mean is over the rows that exist
  const int bh = blockIdx.x / Tmax, t = blockIdx.x - bh * Tmax;
  if (t >= T) return;
  const int rows = min(pool, L - t * pool);
  const uint16_t* src = (blockIdx.y ? K : Q) + ((size_t)bh * L + (size_t)t * pool) * D;
  const int c = threadIdx.x % TPR, r0 = threadIdx.x / TPR;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = r0; r < rows; r += RPP) {
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    const u32x4 v = __builtin_nontemporal_load((const u32x4*)(src + (size_t)r * D + c * 8));   // read once
    const unsigned w[4] = {v[0], v[1], v[2], v[3]};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] += __uint_as_float(w[e] << 16);
      acc[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[r0][c * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
    for (int r = 0; r < RPP; ++r) s += part[r][threadIdx.x];
    const size_t slot = (blockIdx.y ? (size_t)n_q_blocks : 0) + (size_t)bh * T + t;
    pooled[slot * D + threadIdx.x] = s / (float)rows;
  }
}

// The skipping rule without a sort.  "Skip block j iff the ascending cumulative sum at j is <= tau" selects a prefix
// of the ascending order, i.e. all entries up to some value theta (plus, among entries equal to the next value,
// the first few in index order).  S(x) = sum of the entries <= x is a non-decreasing step function of x (also as
// computed here in fp32: a fixed summation structure is monotone in every term), so the largest float theta with
// S(theta) <= tau is found by fixing its bits from the top: 30 wave-wide conditional sums per row instead of one
// per entry.  Entries lie in (0, 1], so bit 29 is the highest that can be set.  Two rows (pa, pb) are searched
// together so that their reductions overlap.  s_* returns S(theta_*).
__device__ __forceinline__ void find_thresholds2(const float* pa, const float* pb, int T, int lane, float tau,
                                                 float& theta_a, float& theta_b, float& s_a, float& s_b) {
  unsigned lo_a = 0u, lo_b = 0u;
  float sa = 0.f, sb = 0.f;
  for (int bit = 29; bit >= 0; --bit) {
    const float ca = __uint_as_float(lo_a | (1u << bit)), cb = __uint_as_float(lo_b | (1u << bit));
    float xa = 0.f, xb = 0.f;
    for (int k = lane; k < T; k += 64) {
      const float a = pa[k], b = pb[k];
      xa += a <= ca ? a : 0.f;
      xb += b <= cb ? b : 0.f;
    }
    xa = wave_sum_dpp(xa);   // the same sum in every lane
    xb = wave_sum_dpp(xb);
    if (xa <= tau) {
      lo_a |= 1u << bit;
      sa = xa;
    }
    if (xb <= tau) {
      lo_b |= 1u << bit;
      sb = xb;
    }
  }
  theta_a = __uint_as_float(lo_a);
  theta_b = __uint_as_float(lo_b);
  s_a = sa;
  s_b = sb;
}

// Entries equal to the smallest value above theta come next in the ascending order, in index order: how many of
// them still fit under tau when added one by one to S(theta).  (With distinct values: none, by the choice of theta.)
__device__ __forceinline__ void next_value_ties(const float* pr, int T, int lane, float theta, float s_theta, float tau,
                                                float& next, int& n_skip) {
  float nx = INFINITY;
  for (int k = lane; k < T; k += 64) {
    const float a = pr[k];
    nx = fminf(nx, a > theta ? a : INFINITY);
  }
  for (int o = 32; o > 0; o >>= 1) nx = fminf(nx, __shfl_xor(nx, o));
  int m = 0;
  for (int k0 = 0; k0 < T; k0 += 64) m += __popcll(__ballot(k0 + lane < T && pr[min(k0 + lane, T - 1)] == nx));
  int n = 0;
  float run = s_theta;
  while (n < m) {
    run += nx;
    if (!(run <= tau)) break;
    ++n;
  }
  next = nx;
  n_skip = n;
}

// Dynamic LDS: pooled query rows [kMapRows][D], one stage of pooled key rows [kChunk][D + 4] (padded so
// that 16 lanes reading 16 bytes of 16 different rows hit 64 different banks), map rows [kMapRows][T_pad].
template <int D>
__global__ void __launch_bounds__(256) map_rows(const float* __restrict__ pooled, long long n_q_blocks, int Tq, int T, int T_pad,
                                                int n_tq, int n_t, int row_bytes, float scale, float tau_kv,
                                                uint8_t* __restrict__ kv_mask, float* __restrict__ text_rows,
                                                float* __restrict__ text_cols) {
  extern __shared__ float lds[];
  constexpr int KS = D + 4;
  float* q = lds;
  float* kst = q + kMapRows * D;
  float* p = kst + kChunk * KS;
  const int tid = threadIdx.x;
  // T = pooled key blocks (columns of the map), n_t of them text; Tq = pooled query blocks (rows), n_tq of them text
  const int groups = (Tq + kMapRows - 1) / kMapRows;
  const int bh = blockIdx.x / groups, i0 = (blockIdx.x % groups) * kMapRows;
  const float* qt = pooled + (size_t)bh * Tq * D;
  const float* kt = pooled + ((size_t)n_q_blocks + (size_t)bh * T) * D;
  for (int e = tid; e < kMapRows * D; e += 256) {
    const int r = e / D, i = min(i0 + r, Tq - 1);
    q[e] = qt[(size_t)i * D + e % D];
  }
  for (int e = tid; e < kMapRows * (T_pad - T); e += 256) p[(e / (T_pad - T)) * T_pad + T + e % (T_pad - T)] = INFINITY;

  // scores: keys come through LDS kChunk at a time (coalesced 16-byte reads of the pooled keys); thread
  // (key tid % kChunk, row tid / kChunk) then takes one dot product
  static_assert(256 / kChunk == kMapRows, "one thread per (staged key, row)");
  const int jj = tid % kChunk, r = tid / kChunk;
  constexpr int NPF = kChunk * (D / 4) / 256;          // 16-byte pieces of a key stage per thread
  float4 pre[NPF];                                     // the next stage, in flight while this one is used
  auto fetch = [&](int j0) {
    const int nk = min(kChunk, T - j0);
#pragma unroll
    for (int u = 0; u < NPF; ++u) {
      const int e = tid + u * 256;
      pre[u] = e < nk * (D / 4) ? *(const float4*)&kt[(size_t)j0 * D + 4 * e] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  fetch(0);
  for (int j0 = 0; j0 < T; j0 += kChunk) {
    __syncthreads();                                   // the previous stage has been consumed
    const int nk = min(kChunk, T - j0);
#pragma unroll
    for (int u = 0; u < NPF; ++u) {
      const int e = tid + u * 256;
      *(float4*)&kst[(e / (D / 4)) * KS + 4 * (e % (D / 4))] = pre[u];
    }
    __syncthreads();
    if (j0 + kChunk < T) fetch(j0 + kChunk);
    if (jj < nk) {
      const float4* kr = (const float4*)(kst + jj * KS);
      const float4* qr = (const float4*)(q + r * D);
      float s0 = 0.f, s1 = 0.f;                         // two partial sums: even and odd 16-byte groups
#pragma unroll 8
      for (int c = 0; c < D / 4; c += 2) {
        const float4 k0 = kr[c], a0 = qr[c], k1 = kr[c + 1], a1 = qr[c + 1];
        s0 += k0.x * a0.x + k0.y * a0.y + k0.z * a0.z + k0.w * a0.w;
        s1 += k1.x * a1.x + k1.y * a1.y + k1.z * a1.z + k1.w * a1.w;
      }
      p[r * T_pad + j0 + jj] = (s0 + s1) * scale;
    }
  }
  __syncthreads();

  // each wave owns two rows from here on; all waves run the same loops (bounds depend on T only)
  const int w = tid / 64, lane = tid % 64;
  for (int rr = 0; rr < 2; ++rr) {
    const int i = i0 + 2 * w + rr;
    float* pr = p + (2 * w + rr) * T_pad;
    float m = -INFINITY;
    for (int j = lane; j < T; j += 64) m = fmaxf(m, pr[j]);
    m = wave_max(m);
    float sum = 0.f;
    for (int j = lane; j < T; j += 64) {
      const float e = expf(pr[j] - m);
      pr[j] = e;
      sum += e;
    }
    sum = wave_sum(sum);
    for (int j = lane; j < T; j += 64) {
      const float v = pr[j] / sum;
      pr[j] = v;
      if (i < n_tq) text_rows[((size_t)bh * n_tq + i) * T + j] = v;       // i < n_tq < Tq
      if (j < n_t && i < Tq) text_cols[((size_t)bh * Tq + i) * n_t + j] = v;
    }
  }
  __syncthreads();

  const float* pa = p + (2 * w) * T_pad;
  const float* pb = pa + T_pad;
  const int ia = i0 + 2 * w, ib = ia + 1;
  float theta_a, theta_b, s_a, s_b, next_a, next_b;
  int nskip_a, nskip_b;
  find_thresholds2(pa, pb, T, lane, tau_kv, theta_a, theta_b, s_a, s_b);
  next_value_ties(pa, T, lane, theta_a, s_a, tau_kv, next_a, nskip_a);
  next_value_ties(pb, T, lane, theta_b, s_b, tau_kv, next_b, nskip_b);
  const unsigned long long below = (1ull << lane) - 1ull;
  int seen_a = 0, seen_b = 0;                                 // entries equal to next_* at smaller indices
  for (int j0 = 0; j0 < T; j0 += 64) {
    const int j = j0 + lane;
    const bool in = j < T;
    const float a = in ? pa[j] : INFINITY, b = in ? pb[j] : INFINITY;
    const unsigned long long tie_a = __ballot(a == next_a), tie_b = __ballot(b == next_b);
    const bool skip_a = a <= theta_a || (a == next_a && seen_a + __popcll(tie_a & below) < nskip_a);
    const bool skip_b = b <= theta_b || (b == next_b && seen_b + __popcll(tie_b & below) < nskip_b);
    seen_a += __popcll(tie_a);
    seen_b += __popcll(tie_b);
    const unsigned long long kept_a = __ballot(in && !skip_a), kept_b = __ballot(in && !skip_b);   // bit l = block j0 + l
    // lanes 0-7 write the bytes of row a, lanes 8-15 those of row b; first block of a byte = bit 7
    const int byte = j0 / 8 + (lane & 7);
    const int i = lane < 8 ? ia : ib;
    if (lane < 16 && i < Tq && byte < row_bytes) {
      const unsigned long long kept = lane < 8 ? kept_a : kept_b;
      const unsigned bits = (unsigned)(kept >> (8 * (lane & 7))) & 0xffu;
      kv_mask[((size_t)bh * Tq + i) * row_bytes + byte] = (uint8_t)(__brev(bits) >> 24);
    }
  }
}

// Tq / Tk pooled query / key blocks, n_tq / n_tk of them text; pool_q / pool_k tokens per pooled block.
__global__ void __launch_bounds__(256) select_blocks(const float* __restrict__ text_rows,
                                                     const float* __restrict__ text_cols, int Tq, int Tk, int n_tq,
                                                     int n_tk, int pool_q, int pool_k, int L, float tau_c, float s_q,
                                                     uint8_t* __restrict__ cache_flags) {
  __shared__ float C[kMaxBlocks], G[kMaxBlocks], Ck[kMaxBlocks];
  __shared__ float red[4];
  const int bh = blockIdx.x, Tv = Tq - n_tq, Tu = Tk - n_tk, tid = threadIdx.x;
  const float* tr = text_rows + (size_t)bh * n_tq * Tk;
  const float* tc = text_cols + (size_t)bh * Tq * n_tk;
  // contribution of every vision key block: what the text rows put on it
  for (int u = tid; u < Tu; u += 256) {
    float c = 0.f;
    for (int j = 0; j < n_tq; ++j) c += tr[(size_t)j * Tk + n_tk + u];
    Ck[u] = c;
  }
  __syncthreads();
  for (int v = tid; v < Tv; v += 256) {
    float c;
    if (pool_q == pool_k) {
      c = Ck[v];
    } else {
      // carried over to the query axis: every key block's contribution spread evenly over its tokens
      c = 0.f;
      const int q0 = (n_tq + v) * pool_q, q1 = min(q0 + pool_q, L);
      const int u_lo = max(q0 / pool_k - n_tk, 0), u_hi = min((q1 - 1) / pool_k - n_tk, Tu - 1);
      for (int u = u_lo; u <= u_hi; ++u) {
        const int k0 = (n_tk + u) * pool_k, k1 = min(k0 + pool_k, L);
        const int common = min(k1, q1) - max(k0, q0);
        if (common > 0) c += Ck[u] * (float)common / (float)(k1 - k0);
      }
    }
    C[v] = c;
    G[v] = 0.f;
  }
  for (int j = 0; j < n_tk; ++j) {
    float m = -INFINITY;
    for (int v = tid; v < Tv; v += 256) m = fmaxf(m, tc[(size_t)(n_tq + v) * n_tk + j]);
    m = block_max(m, red);
    float s = 0.f;
    for (int v = tid; v < Tv; v += 256) s += expf(tc[(size_t)(n_tq + v) * n_tk + j] - m);
    s = block_sum(s, red);
    for (int v = tid; v < Tv; v += 256) G[v] += expf(tc[(size_t)(n_tq + v) * n_tk + j] - m) / s;   // v belongs to one thread
  }
  __syncthreads();
  // totals in index order: what the ascending sum of the largest entry adds up to as well
  float tot_c = 0.f, tot_g = 0.f;
  for (int u = 0; u < Tv; ++u) {
    tot_c += C[u];
    tot_g += G[u];
  }
  int n_cached = 0;
  unsigned mine = 0;                               // decisions of this thread's blocks, bit n = block tid + 256 n
  for (int v = tid, n = 0; v < Tv; v += 256, ++n) {
    const float cv = C[v], gv = G[v];
    float cs_c = 0.f, cs_g = 0.f;
    for (int u = 0; u < Tv; ++u) {
      const float cu = C[u], gu = G[u];
      cs_c += ((cu < cv) | ((cu == cv) & (u <= v))) ? cu : 0.f;      // bitwise on purpose: no branches
      cs_g += ((gu < gv) | ((gu == gv) & (u <= v))) ? gu : 0.f;
    }
    const bool cached = cs_c <= tau_c * tot_c && cs_g <= tau_c * tot_g;
    mine |= (cached ? 1u : 0u) << n;
    n_cached += cached ? 1 : 0;
  }
  const float total_cached = block_sum((float)n_cached, red);    // exact: counts stay far below 2^24
  const bool degrade = ((float)Tq - total_cached) / (float)Tq < s_q;
  uint8_t* out = cache_flags + (size_t)bh * Tq;
  for (int b = tid; b < n_tq; b += 256) out[b] = degrade ? 1 : 0;
  for (int v = tid, n = 0; v < Tv; v += 256, ++n) out[n_tq + v] = (degrade || ((mine >> n) & 1u)) ? 1 : 0;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

#define HIP_TRY(expr)                                                                                \
  do {                                                                                               \
    hipError_t e_ = (expr);                                                                          \
    if (e_ != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

extern "C" {

int sparse_symbols_update_granular(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H,
                                   int L, int D, int block_q, int block_k, int granularity, int text_tokens, float tau_c,
                                   float tau_kv, float s_q, void* hip_stream) {
  if (B <= 0 || H <= 0 || L <= 0 || D <= 0 || block_q <= 0 || block_k <= 0)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: sizes must be positive (B=%d H=%d L=%d D=%d block_q=%d block_k=%d)", B, H,
                   L, D, block_q, block_k);
  if ((D != 64 && D != 128) || (block_q != 64 && block_q != 128) || (block_k != 64 && block_k != 128))
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "symbols: D, block_q and block_k must be 64 or 128 (got %d, %d, %d)", D,
                   block_q, block_k);
  if (granularity < 1 || granularity > 64)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: granularity=%d must be between 1 and 64", granularity);
  if (text_tokens <= 0 || text_tokens >= L)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: text_tokens=%d must leave text and vision tokens (L=%d)", text_tokens, L);
  // pooled blocks of n * b tokens; a short last block counts as a block, and a pooled block that holds any text
  // token counts as text (the ceiling of Section 3.3)
  const int pool_q = granularity * block_q, pool_k = granularity * block_k;
  const int Tq = (L + pool_q - 1) / pool_q, Tk = (L + pool_k - 1) / pool_k;
  const int n_tq = (text_tokens + pool_q - 1) / pool_q, n_tk = (text_tokens + pool_k - 1) / pool_k;
  if (n_tq >= Tq || n_tk >= Tk)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: no vision block is left (%d of %d query blocks and %d of %d key blocks are text)",
                   n_tq, Tq, n_tk, Tk);
  if (Tq > kMaxBlocks || Tk > kMaxBlocks)
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "symbols: %d x %d pooled blocks exceed %d", Tq, Tk, kMaxBlocks);
  if (!(tau_c >= 0.f && tau_c <= 1.f) || !(tau_kv >= 0.f && tau_kv <= 1.f) || !(s_q >= 0.f && s_q <= 1.f))
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: tau_c, tau_kv and s_q must lie in [0, 1] (got %g, %g, %g)",
                   (double)tau_c, (double)tau_kv, (double)s_q);
  const long long BH = (long long)B * H;
  const long long n_q_blocks = BH * Tq, n_k_blocks = BH * Tk;
  if (BH * (Tq > Tk ? Tq : Tk) > 0x3fffffffLL)
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "symbols: too many blocks (%lld)", BH * (Tq > Tk ? Tq : Tk));
  if (!Q || !K || !cache_flags || !kv_mask)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: Q, K, cache_flags and kv_mask must not be NULL");
  if (((uintptr_t)Q | (uintptr_t)K) & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "symbols: Q and K must be 16-byte aligned");

  hipStream_t stream = (hipStream_t)hip_stream;
  const size_t pooled_b = align256((size_t)(n_q_blocks + n_k_blocks) * D * 4);
  const size_t rows_b = align256((size_t)BH * n_tq * Tk * 4);
  const size_t cols_b = align256((size_t)BH * Tq * n_tk * 4);
  void* ws = nullptr;
  if (int rc = sa_get_scratch(pooled_b + rows_b + cols_b, stream, &ws)) return rc;
  float* pooled = (float*)ws;
  float* text_rows = (float*)((char*)ws + pooled_b);
  float* text_cols = (float*)((char*)ws + pooled_b + rows_b);

  const int row_bytes = (Tk + 7) / 8;
  const float scale = (float)(1.0 / sqrt((double)D));
  const int groups = (Tq + kMapRows - 1) / kMapRows;
  const int T_pad = (Tk + 3) & ~3;
  const size_t map_lds = ((size_t)kMapRows * D + (size_t)kChunk * (D + 4) + (size_t)kMapRows * T_pad) * 4;
  static std::once_flag attr_once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [] {
    constexpr int kMaxLds = (kMapRows * 128 + kChunk * 132 + kMapRows * kMaxBlocks) * 4;
    attr_err = hipFuncSetAttribute((const void*)map_rows<128>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
    if (attr_err == hipSuccess)
      attr_err = hipFuncSetAttribute((const void*)map_rows<64>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  });
  if (attr_err != hipSuccess)
    return sa_fail(SPARSE_ATTN_ERR_HIP, "hipFuncSetAttribute(map_rows) failed: %s", hipGetErrorString(attr_err));
  const unsigned pool_grid = (unsigned)(BH * (Tq > Tk ? Tq : Tk));
  if (D == 128) {
    hipLaunchKernelGGL(pool_blocks<128>, dim3(pool_grid, 2), dim3(256), 0, stream, (const uint16_t*)Q,
                       (const uint16_t*)K, pooled, pool_q, pool_k, Tq, Tk, L, n_q_blocks);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(map_rows<128>, dim3((unsigned)(BH * groups)), dim3(256), map_lds, stream, pooled, n_q_blocks, Tq, Tk,
                       T_pad, n_tq, n_tk, row_bytes, scale, tau_kv, kv_mask, text_rows, text_cols);
  } else {
    hipLaunchKernelGGL(pool_blocks<64>, dim3(pool_grid, 2), dim3(256), 0, stream, (const uint16_t*)Q,
                       (const uint16_t*)K, pooled, pool_q, pool_k, Tq, Tk, L, n_q_blocks);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(map_rows<64>, dim3((unsigned)(BH * groups)), dim3(256), map_lds, stream, pooled, n_q_blocks, Tq, Tk,
                       T_pad, n_tq, n_tk, row_bytes, scale, tau_kv, kv_mask, text_rows, text_cols);
  }
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(select_blocks, dim3((unsigned)BH), dim3(256), 0, stream, text_rows, text_cols, Tq, Tk, n_tq, n_tk,
                     pool_q, pool_k, L, tau_c, s_q, cache_flags);
  HIP_TRY(hipGetLastError());
  return 0;
}

int sparse_symbols_update_stream(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H,
                                 int L, int D, int block, int text_tokens, float tau_c, float tau_kv, float s_q,
                                 void* hip_stream) {
  return sparse_symbols_update_granular(Q, K, cache_flags, kv_mask, B, H, L, D, block, block, 1, text_tokens, tau_c, tau_kv,
                                        s_q, hip_stream);
}

int sparse_symbols_update(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H, int L,
                          int D, int block, int text_tokens, float tau_c, float tau_kv, float s_q) {
  return sparse_symbols_update_stream(Q, K, cache_flags, kv_mask, B, H, L, D, block, text_tokens, tau_c, tau_kv, s_q,
                                      nullptr);
}

}  // extern "C"
