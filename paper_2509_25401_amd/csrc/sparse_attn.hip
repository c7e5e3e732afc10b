// FlashOmni attention (Algorithm 1 of the paper) for AMD MI355X / gfx950.
//
// Three kernels per call, all on the caller's stream:
//   plan_rows   decodes the packed symbols of Section 3.3 once per (b,h,i) row into aligned
//               32-bit words (bit j of the row = key block j, padding cleared), counts the
//               kept key blocks of every non-cached row and notes the first of them;
//   plan_order  sorts the rows into one work queue per XCD (a head's rows all go to one XCD, so
//               its K/V stream through one L2): rows that are a large part of a workgroup's
//               share first (longest first), the others head by head and heaviest first inside a
//               head (55 kept-count buckets), cached rows (plain copies) last;
//   attn        a persistent grid of two workgroups per CU pulls items from its XCD's queue and
//               steals from the others when that is drained.  A compute item is one query block:
//               Q lives in registers as stored (the 1/sqrt(D) scale is applied to the fp32 score),
//               the reduction-axis symbol is walked with scalar find-first-set on the decoded words, and only kept
//               K/V tiles are streamed to LDS with direct-to-LDS loads, double buffered in 64-key
//               sub-tiles.  S^T = K Q^T and O^T = V^T P^T run on v_mfma_f32_32x32x16_bf16, so
//               each lane owns one query row: the row maximum needs a single half-wave exchange,
//               the row sum none until the end, and the exponentiated S^T accumulators are the
//               B operand of the O^T product without any data movement.  The reference of the
//               exponent is the C operand of the first S^T MFMA; it is checked after the fact
//               (the sum of a block's weights shows whether a score left the allowed range)
//               and moves only then, so the steady state takes no row maximum at all.  The
//               vector instructions of the softmax sit between matrix instructions that do not
//               depend on them (weights of one 32-key block under the scores of the next and
//               under the O^T product of the previous), where they issue in the shadow of the
//               wave's own MFMAs.  The finished block leaves through LDS as whole rows.  The ticket
//               of the next item is drawn a few key blocks before the current one ends, and its
//               work-list entry names the first kept key block, so that tile is requested before
//               the row's symbol words are touched.  A copy item moves one cached block
//               O_cache -> O.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <map>
#include <mutex>
#include <new>
#include <type_traits>
#include <utility>

#include "sparse_attn.h"
#include "sparse_attn_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define LDS_PTR(T) T __attribute__((address_space(3)))*
#define GLOBAL_PTR(T) T __attribute__((address_space(1)))*

constexpr int kKeys = 64;             // keys per LDS sub-tile
constexpr int kLongBuckets = 8;       // kept-count buckets of the long rows of a queue (longest first, across heads)
constexpr int kFineBuckets = 55;      // ... of its other rows (head by head); with the bucket of cached rows: 64,
constexpr int kCachedBucket = kLongBuckets + kFineBuckets;   // one lane each in the ranking pass
constexpr int kWgsPerXcd = 64;        // workgroups of the persistent grid per XCD (32 CUs x 2) the ordering plans for
constexpr int kXcds = 8;               // accelerator dies (XCDs) of the MI355X, each with its own L2
constexpr int kMaxHeadGroups = 24;    // head groups per (XCD, bucket) in the ordering histogram (48 KiB of LDS)
constexpr int kMaxTq = 16384;
constexpr unsigned kCopyFlag = 0x80000000u;
// Queue counters: every queue head sits in a 128-byte line of its own (all workgroups of an XCD bump the same
// head once per item; eight heads in one line would make every workgroup of the chip contend for that line),
// the queue ends, which the attention kernel only reads, in a line that is never written while it runs.
constexpr int kHeadStride = 32;                   // words between two queue heads
constexpr int kEndOffset = 8 * kHeadStride;       // first queue end
constexpr int kQueueWords = kEndOffset + 64;      // 1280 bytes
constexpr int kHwRegXccId = (3 << 11) | 20;   // s_getreg operand: 4 bits at offset 0 of hardware register 20 (XCC_ID)
constexpr int kOrderThreads = 1024;
constexpr int kMaxTerms = 4;            // stored feature + up to three derivatives
constexpr int kMfmaPrio = 1;            // wave priority while it feeds the matrix pipe
constexpr float kSumLimit = 256.0f;     // a lane's 16 weights of one 32-key block may add up to this before the reference moves

struct AttnParams {
  const char* Q;
  const char* K;
  const char* V;
  const char* O_cache;
  char* O;
  const uint32_t* words;   // [N][nw32] decoded symbol words
  const uint32_t* order;   // [N][2] work list: {row | kCopyFlag, sort key of the row (see plan_rows)}
  uint32_t* queues;        // kXcds queue heads at [q * kHeadStride], kXcds queue ends at [kEndOffset + q]
  int N;                   // B*H*Tq
  int Tq;
  int Tkv;
  int L;
  int nw32;
  int do_copy;             // 0: cached blocks are already in place
  float scale_log2;        // log2(e) / sqrt(D)
  // OP_reuse as a Taylor forecast: cached block = sum_d coef[d] * term[d]; term[0] is O_cache.
  // n_terms == 0 selects the plain bit-exact copy.
  const char* term[kMaxTerms - 1];
  float coef[kMaxTerms];
  int n_terms;
};

// ---------------------------------------------------------------------------------------
// Symbol pre-pass
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) plan_rows(const uint8_t* __restrict__ cache_flags,
                                                 const uint8_t* __restrict__ kv_mask, int N, int Tq, int Tkv,
                                                 int gran, int sym_Tq, int sym_row_bytes, int nw32,
                                                 uint32_t* __restrict__ words, int32_t* __restrict__ keys) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= N) return;
  // one symbol covers gran x gran tiles: tile (i, j) reads flag i / gran and mask bit (i / gran, j / gran)
  const int bh = row / Tq;
  const size_t sym_row = (size_t)bh * sym_Tq + (row - bh * Tq) / gran;
  const bool cached = cache_flags != nullptr && cache_flags[sym_row] != 0;
  int count = 0, first_kept = -1;
  const uint8_t* src = kv_mask ? kv_mask + sym_row * sym_row_bytes : nullptr;
  for (int w = 0; w < nw32; ++w) {
    uint32_t word = 0;
    if (!cached) {
      if (!src) {
        word = 0xffffffffu;
      } else if (gran == 1) {
        for (int b = 0; b < 4; ++b) {
          const int byte = 4 * w + b;
          if (byte < sym_row_bytes) word |= (__brev((uint32_t)src[byte]) >> 24) << (8 * b);
        }
      } else {
        for (int t = 0; t < 32 && 32 * w + t < Tkv; ++t) {
          const int js = (32 * w + t) / gran;
          word |= (uint32_t)((src[js >> 3] >> (7 - (js & 7))) & 1) << t;
        }
      }
      const int valid = Tkv - 32 * w;   // >= 1 by construction of nw32
      if (valid < 32) word &= (1u << valid) - 1u;
    }
    words[(size_t)row * nw32 + w] = word;
    count += __popc(word);
    if (first_kept < 0 && word != 0u) first_kept = 32 * w + __ffs(word) - 1;
  }
  // key of a computed row: kept blocks in the low 16 bits (0 .. 32768), first kept block above them
  keys[row] = cached ? -1 : (count | (max(first_kept, 0) << 16));
}

// Copies the initial queue heads and ends of a stored plan into the live ones its next run consumes.
__global__ void reset_queues(const uint32_t* __restrict__ init, uint32_t* __restrict__ live) {
  const int t = threadIdx.x;
  if (t < kXcds) {
    live[t * kHeadStride] = init[t * kHeadStride];
    live[kEndOffset + t] = init[kEndOffset + t];
  }
}

// Work list order: one queue per XCD (head bh belongs to XCD bh % kXcds), in three parts.
//   long rows    rows with more kept blocks than `limit` = a third of what one workgroup gets to do in total
//                (kept blocks of the queue / (3 * kWgsPerXcd)): longest first across heads (kLongBuckets buckets,
//                heads adjacent inside a bucket), so that none of them starts late.  Uniform masks have none; with
//                few rows per workgroup (short sequences) every row is long.
//   other rows   head by head, inside a head the heaviest first (kFineBuckets buckets), inside a bucket in sequence
//                order.  All workgroups of an XCD then stream the K/V of the same head at the same time, and because
//                rows that run at the same time have (almost) the same number of kept blocks they also stay at
//                about the same key position while they sweep it: a tile one of them has fetched is still in that
//                XCD's L2 when the others ask for it.  What counts for the balance is the end of the queue, and
//                there the light rows of the last head come last.
//   cached rows  (plain copies) of all heads at the very end.
// Bucket of a row: 0 .. kLongBuckets-1 long (heaviest = 0), then kFineBuckets buckets, then kCachedBucket.
// `lightest` = the smallest kept count among the queue's computed rows: the fine buckets span lightest .. limit, so
// that masks whose rows differ by a few blocks only are still sorted block by block.
__device__ inline int order_major(int key, int Tkv, int limit, int lightest) {
  if (key < 0) return kCachedBucket;
  const int count = key & 0xffff;   // < 2^16, bucket counts < 2^6: the products fit in 32 bits
  if (count > limit)
    return (kLongBuckets - 1) - (int)((unsigned)(count - limit - 1) * kLongBuckets / (unsigned)(Tkv - limit));
  return kLongBuckets + (kFineBuckets - 1) -
         (int)((unsigned)(count - lightest) * kFineBuckets / (unsigned)(limit - lightest + 1));
}
__device__ inline int order_bin(int key, int row, int Tq, int Tkv, int shift, int groups, const int* limit,
                                const int* lightest) {
  const int bh = row / Tq;
  const int xcd = bh % kXcds;
  const int group = (bh / kXcds) >> shift, major = order_major(key, Tkv, limit[xcd], lightest[xcd]);
  int inner;
  if (major < kLongBuckets)
    inner = major * groups + group;
  else if (major < kCachedBucket)
    inner = kLongBuckets * groups + group * kFineBuckets + (major - kLongBuckets);
  else
    inner = kCachedBucket * groups + group;
  return xcd * (kCachedBucket + 1) * groups + inner;
}

__global__ void __launch_bounds__(kOrderThreads) plan_order(const int32_t* __restrict__ keys, int N, int Tq,
                                                            int Tkv, int shift, int groups,
                                                            uint32_t* __restrict__ order,
                                                            uint32_t* __restrict__ queues) {
  __shared__ uint32_t bins[kXcds * (kCachedBucket + 1) * kMaxHeadGroups];
  __shared__ uint32_t partial[kOrderThreads];
  __shared__ unsigned long long queue_kept[kXcds];   // kept key blocks of all rows of a queue
  __shared__ int limit[kXcds];                       // kept blocks from which a row of the queue counts as long
  __shared__ uint32_t heaviest[kXcds], lightest_u[kXcds];   // largest / smallest kept count of its computed rows
  __shared__ int lightest[kXcds];
  __shared__ uint32_t seen_rows[kOrderThreads / 64][64];
  const int tid = threadIdx.x;
  const int per_xcd = (kCachedBucket + 1) * groups;
  const int nbins = kXcds * per_xcd;
  for (int b = tid; b < nbins; b += kOrderThreads) bins[b] = 0;
  if (tid < kXcds) {
    queue_kept[tid] = 0ull;
    heaviest[tid] = 0u;
    lightest_u[tid] = 0xffffu;
  }
  __syncthreads();
  {
    // one wave per head: sum, maximum and minimum of the kept counts of its rows (a head has at most 2^14 rows of at
    // most 2^16 - 1 kept blocks: the sum fits in 32 bits), one atomic each per head
    const int wave = tid >> 6, lane = tid & 63;
    for (int bh = wave; bh < N / Tq; bh += kOrderThreads / 64) {
      uint32_t sum = 0, hi = 0, lo = 0xffffu;
      for (int i = lane; i < Tq; i += 64) {
        const int key = keys[bh * Tq + i];
        if (key >= 0) {
          const uint32_t count = (uint32_t)(key & 0xffff);
          sum += count;
          hi = max(hi, count);
          lo = min(lo, count);
        }
      }
      for (int off = 32; off > 0; off >>= 1) {
        sum += __shfl_xor(sum, off);
        hi = max(hi, __shfl_xor(hi, off));
        lo = min(lo, __shfl_xor(lo, off));
      }
      if (lane == 0) {
        atomicAdd(&queue_kept[bh % kXcds], (unsigned long long)sum);
        atomicMax(&heaviest[bh % kXcds], hi);
        atomicMin(&lightest_u[bh % kXcds], lo);
      }
    }
  }
  __syncthreads();
  if (tid < kXcds) {
    // long = more than a third of a workgroup's share; where no row is that long the fine buckets end at the
    // heaviest row instead
    const int share = (int)min(queue_kept[tid] / (3ull * kWgsPerXcd), (unsigned long long)Tkv);
    limit[tid] = (int)heaviest[tid] <= share ? (int)heaviest[tid] : share;
    lightest[tid] = min((int)lightest_u[tid], limit[tid]);
  }
  __syncthreads();
  for (int r = tid; r < N; r += kOrderThreads) atomicAdd(&bins[order_bin(keys[r], r, Tq, Tkv, shift, groups, limit, lightest)], 1u);
  __syncthreads();
  // exclusive scan of bins: contiguous chunk per thread, then a scan over the chunk sums
  const int chunk = (nbins + kOrderThreads - 1) / kOrderThreads;
  const int lo = min(nbins, tid * chunk), hi = min(nbins, lo + chunk);
  uint32_t sum = 0;
  for (int b = lo; b < hi; ++b) sum += bins[b];
  partial[tid] = sum;
  __syncthreads();
  for (int off = 1; off < kOrderThreads; off <<= 1) {
    uint32_t add = tid >= off ? partial[tid - off] : 0u;
    __syncthreads();
    partial[tid] += add;
    __syncthreads();
  }
  uint32_t run = partial[tid] - sum;
  for (int b = lo; b < hi; ++b) {
    const uint32_t c = bins[b];
    bins[b] = run;
    run += c;
  }
  __syncthreads();
  if (tid < kXcds) {
    const uint32_t begin = bins[tid * per_xcd];
    queues[tid * kHeadStride] = begin;                      // queue head
    if (tid > 0) queues[kEndOffset + tid - 1] = begin;      // previous queue's end
    if (tid == kXcds - 1) queues[kEndOffset + kXcds - 1] = (uint32_t)N;
  }
  __syncthreads();
  // Inside a bin the rows keep their order in the sequence: neighbouring query blocks, which with windowed symbols
  // keep nearly the same key blocks, are then worked on at the same time and find each other's tiles in L2.  A bin
  // holds rows of one head as long as there are no more than kMaxHeadGroups heads per queue: a wave then walks a
  // head 64 query blocks at a time, keeps the number of rows seen so far in every bucket, and a row's place is the
  // start of its bin + that count + the rows of its bucket at lower lanes (ballots).  With more heads several of them
  // share a bin and the rows take their places in arrival order.
  if (shift == 0) {
    const int wave = tid >> 6, lane = tid & 63;
    const int heads = N / Tq;
    volatile uint32_t* seen = seen_rows[wave];   // rows of the current head met so far, per bucket
    for (int bh = wave; bh < heads; bh += kOrderThreads / 64) {
      seen[lane] = 0u;
      for (int i0 = 0; i0 < Tq; i0 += 64) {
        const int i = i0 + lane;
        const bool valid = i < Tq;
        const int r = bh * Tq + min(i, Tq - 1);
        const int key = keys[r];
        const int major = valid ? order_major(key, Tkv, limit[bh % kXcds], lightest[bh % kXcds]) : 0;
        // the lanes whose row falls into the same bucket as this lane's: one ballot per bit of the bucket number
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
          const unsigned long long set = __ballot((major >> b) & 1);
          same &= ((major >> b) & 1) ? set : ~set;
        }
        if (valid) {
          // LDS accesses of a wave execute in program order: every lane reads its bucket's count before the first
          // lane of each bucket moves it on
          const uint32_t before = seen[major];
          const uint32_t rank = before + (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
          if ((same & ((1ull << lane) - 1ull)) == 0ull) seen[major] = before + (uint32_t)__popcll(same);
          const uint32_t pos = bins[order_bin(key, r, Tq, Tkv, shift, groups, limit, lightest)] + rank;
          order[2 * pos] = (uint32_t)r | (key < 0 ? kCopyFlag : 0u);
          order[2 * pos + 1] = (uint32_t)key;
        }
      }
    }
    return;
  }
  for (int r = tid; r < N; r += kOrderThreads) {
    const int key = keys[r];
    const uint32_t pos = atomicAdd(&bins[order_bin(key, r, Tq, Tkv, shift, groups, limit, lightest)], 1u);
    order[2 * pos] = (uint32_t)r | (key < 0 ? kCopyFlag : 0u);
    order[2 * pos + 1] = (uint32_t)key;
  }
}

// One atomic increment per wave, issued by lane 0 only and left in flight: returns a register whose lane 0
// will hold the counter's previous value.  Written as assembly around an exec-mask switch, not as
// `if (lane == 0) atomicAdd(...)`: a value that stays live across loop iterations inside a lane-dependent
// branch makes the compiler treat the whole scheduling state of the kernel as lane-dependent.
__device__ __forceinline__ unsigned sa_lane0_atomic_inc(uint32_t* counter) {
  unsigned old;
  unsigned long long saved;
  asm volatile(
      "s_mov_b64 %1, exec\n\ts_mov_b64 exec, 1\n\tglobal_atomic_add %0, %2, %3, %4 sc0\n\ts_mov_b64 exec, %1"
      : "=&v"(old), "=&s"(saved)
      : "v"(0u), "v"(1u), "s"(counter)
      : "memory");
  return old;
}
// Waits for this wave's outstanding memory operations and returns lane 0 of `v` as a wave-uniform value.
__device__ __forceinline__ unsigned sa_lane0_value(unsigned v) {
  unsigned r;
  asm volatile("s_waitcnt vmcnt(0)\n\tv_readfirstlane_b32 %0, %1" : "=s"(r) : "v"(v) : "memory");
  return r;
}
// A work-list entry (two words) read with one scalar load instead of a vector load and a lane broadcast.  Load and
// wait are one statement on purpose: the compiler does not know that the result arrives late and may copy the
// registers in between.
__device__ __forceinline__ unsigned long long sa_scalar_load_b64(const uint32_t* ptr) {
  unsigned long long v;
  asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(ptr) : "memory");
  return v;
}

// ---------------------------------------------------------------------------------------
// LDS layouts.  A sub-tile is kKeys rows of D bf16, row major, with the 16-byte chunks of a
// row permuted by an XOR that depends on the row, so that (a) the 32 rows x 16 B that one
// S^T operand read touches and (b) the 8 rows x 64 B that one transposed V read touches fall
// into distinct banks.  A direct-to-LDS load writes 1 KiB of consecutive LDS per wave
// instruction, so the permutation is applied to the global address each lane fetches.
// ---------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int k_swizzle(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int v_swizzle(int row) {
  return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1);
}

// RAGGED: the sequence length is not a multiple of the blocks (Definition 1 counts ceil(L / b) of them).
// The last query block then has fewer rows and the last key block fewer keys: loads of missing rows
// re-read the last row that exists, scores of missing keys are set to -inf before the softmax, stores of
// missing query rows are dropped, and a 64-key sub-tile that lies entirely past the end is not visited.
// The aligned instantiation contains none of this.
template <int D, int BQ, int BK, bool RAGGED>
__global__ void __launch_bounds__(BQ * 2, 2) attn_kernel(const AttnParams p) {
  constexpr int NWAVES = BQ / 32;
  constexpr int NT = NWAVES * 64;
  constexpr int SUB = BK / kKeys;          // LDS sub-tiles per symbol bit
  constexpr int CH = D / 8;                // 16-byte chunks per row
  constexpr int ROWB = D * 2;              // bytes per row
  constexpr int TILEB = kKeys * ROWB;      // bytes per K or V sub-tile
  constexpr int NINST = TILEB / 1024;      // direct-to-LDS wave instructions per sub-tile
  constexpr int NLOAD = NINST / NWAVES;    // of which this wave issues
  constexpr int ROWS_PER_INST = 1024 / ROWB;
  constexpr int KS = D / 16;               // k-steps of the S^T product
  constexpr int DB = D / 32;               // 32-row blocks of O^T
  constexpr int NQK = 2 * KS;              // MFMAs of S^T per sub-tile
  constexpr int NPV = 4 * DB;              // MFMAs of O^T per sub-tile
  constexpr int kPre = 4;                  // operand reads run this many MFMAs ahead
  static_assert(NINST % NWAVES == 0, "sub-tile loads must split evenly over the waves");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* const ldsK = smem;                 // two K sub-tiles, then two V sub-tiles
  char* const ldsV = smem + 2 * TILEB;
  LDS_PTR(volatile int) const s_item = (LDS_PTR(volatile int))(smem + 4 * TILEB);
  const unsigned lds_base = (unsigned)(uintptr_t)(LDS_PTR(char))smem;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;    // query row inside the wave's 32-row slab / key row of an operand read
  const int half = lane >> 5;   // which 8 of the 16 k-slots of an MFMA this lane feeds
  const int i16 = lane & 15;
  const int g4 = lane >> 4;
  const float score_scale = p.scale_log2;

  // Per-lane offsets, the same for every item.
  // Global byte offsets inside a sub-tile (swizzle applied to the source).  The swizzles repeat every 16 rows, so
  // the offsets of load t and load t + TP differ by a constant that goes into the (scalar) base address.
  constexpr int TP = NWAVES * ROWS_PER_INST >= 16 ? 1 : 16 / (NWAVES * ROWS_PER_INST);
  constexpr int TSTEP = TP * NWAVES * ROWS_PER_INST * ROWB;
  static_assert(NLOAD % TP == 0, "loads of a wave must be whole swizzle periods");
  unsigned k_goff[TP], v_goff[TP];
#pragma unroll
  for (int t = 0; t < TP; ++t) {
    const int r = (wave + t * NWAVES) * ROWS_PER_INST + lane / CH;
    const int pch = lane % CH;
    k_goff[t] = (unsigned)(r * ROWB + ((pch ^ k_swizzle<D>(r)) * 16));
    v_goff[t] = (unsigned)(r * ROWB + ((pch ^ v_swizzle<D>(r)) * 16));
  }
  int k_off[KS];     // S^T operand (K rows): LDS byte offset of k-step ks inside this lane's key row
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = l32 * ROWB + (((2 * ks + half) ^ k_swizzle<D>(l32)) * 16);
  int v_off[DB];     // O^T operand (V transposed): LDS byte offset of d-block db for this lane
  {
    const int r = 4 * (g4 >> 1) + (i16 >> 2);   // key row inside an 8-row group; rows +8, +16, ... share the swizzle
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int ch = 4 * db + 2 * (g4 & 1) + ((i16 & 3) >> 1);
      v_off[db] = r * ROWB + ((ch ^ v_swizzle<D>(r)) * 16) + 8 * (i16 & 1);
    }
  }

  // This workgroup's home queue is the one of the XCD it runs on (hardware register XCC_ID).
  const int my_q = (int)(__builtin_amdgcn_s_getreg(kHwRegXccId) & 15u) % kXcds;
  uint32_t* const q_head = p.queues;
  const uint32_t* const q_end = p.queues + kEndOffset;

  // Work acquisition.  The ticket of the next item is one atomic on the home queue, issued by wave 0 and left in
  // flight; it is drawn a few kept blocks before the current item ends (earlier would let an idle workgroup find
  // the queue empty while this one still sits on an item it has not started), so at the end of the item it has
  // long arrived.  The item number reaches the other waves through one of two LDS slots, used in turn: a wave
  // reads slot s of item i before it arrives at the barrier of item i + 1, and the slot is not written again
  // before that barrier has been passed, so one barrier per item is enough.  The barrier waits for LDS traffic
  // only; __syncthreads() would also make every wave wait for the acknowledgement of its stores of the previous
  // item.  The work-list entry then comes through the scalar cache and carries the row's kept-block count and
  // first kept block, so the first K/V sub-tile is requested before the row's symbol words have been looked at.
  constexpr int kDrawTiles = 6;        // kept blocks an item still has to visit when the next ticket is drawn
  bool drawn = false;
  unsigned ticket = 0;                 // wave 0: lane 0 holds the ticket of the home queue, possibly still in flight
  auto draw_issue = [&]() {
    if (wave == 0) ticket = sa_lane0_atomic_inc(q_head + my_q * kHeadStride);   // a drained queue just keeps counting
    drawn = true;
  };
  for (int parity = 0;; parity ^= 1) {
    if (!drawn) draw_issue();
    drawn = false;
    if (wave == 0) {
      // resolve the ticket; when the home queue is drained, steal from the other XCDs' queues
      const uint32_t t = sa_lane0_value(ticket);
      int item = t < q_end[my_q] ? (int)t : -1;
      for (int k = 1; k < kXcds && item < 0; ++k) {
        const int q = (my_q + k) % kXcds;
        const uint32_t end = q_end[q];
        const uint32_t got = sa_lane0_value(sa_lane0_atomic_inc(q_head + q * kHeadStride));
        if (got < end) item = (int)got;
      }
      s_item[parity] = item;           // every lane writes the same value
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int n = __builtin_amdgcn_readfirstlane(s_item[parity]);
    if (n < 0) break;
    const unsigned long long entry64 = sa_scalar_load_b64(p.order + 2 * (size_t)n);
    const uint32_t entry = (uint32_t)entry64;
    const uint32_t key = (uint32_t)(entry64 >> 32);
    const int row = (int)(entry & ~kCopyFlag);
    const int bh = row / p.Tq;
    const int iq = row - bh * p.Tq;
    const size_t head_off = (size_t)bh * p.L * ROWB;
    const size_t blk_off = head_off + (size_t)iq * BQ * ROWB;

    if (entry & kCopyFlag) {
      // cache-then-reuse: O_i <- cached O_i, bit exact
      int NV = BQ * ROWB / 16;
      if constexpr (RAGGED) NV = min(BQ, p.L - iq * BQ) * (ROWB / 16);
      if (p.n_terms > 0) {
        // forecast: fp32 sum of the scaled terms in order, rounded once to bf16
        const bf16x8* t0 = (const bf16x8*)(p.O_cache + blk_off);
        bf16x8* dst = (bf16x8*)(p.O + blk_off);
        for (int t = tid; t < NV; t += NT) {
          const bf16x8 a = t0[t];
          float acc[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = p.coef[0] * (float)a[e];
          for (int d = 1; d < p.n_terms; ++d) {
            const bf16x8 b = ((const bf16x8*)(p.term[d - 1] + blk_off))[t];
            const float c = p.coef[d];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(c, (float)b[e], acc[e]);
          }
          bf16x8 r;
#pragma unroll
          for (int e = 0; e < 8; ++e) r[e] = (__bf16)acc[e];
          dst[t] = r;
        }
      } else if (p.do_copy) {
        const u32x4* src = (const u32x4*)(p.O_cache + blk_off);
        u32x4* dst = (u32x4*)(p.O + blk_off);
#pragma unroll 4
        for (int t = tid; t < NV; t += NT) dst[t] = src[t];
      }
      continue;
    }

    // ---- compute-on-demand ----
    const char* Kh = p.K + head_off;
    const char* Vh = p.V + head_off;
    const uint32_t* wp = p.words + (size_t)row * p.nw32;

    // Q fragment: B operand of S^T = K Q^T; lane holds query row l32, d = 16*ks + 8*half .. +7, exactly as stored:
    // the products accumulate in fp32 and the scale log2(e)/sqrt(D) is applied to the fp32 score on its way into
    // the exponential (scaling the fragment instead would save that multiply but round the queries a second time).
    // (It is loaded further down, behind the first K/V sub-tile's loads, so that the two latencies overlap.)
    bf16x8 qf[KS];

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    // Reference of the scores (raw q.k units, before the scale) of this lane's query row, kept NEGATED in all 16
    // registers of an accumulator: it is the C operand of the first MFMA of every S^T block, so
    // the MFMA delivers score - reference and the softmax needs no subtraction per score either.
    // The reference is not the running maximum: it is raised (to the row maximum seen so far) only
    // when the weights of a sub-tile show that a score left the allowed range above it; the final
    // division by the row sum cancels it exactly.
    f32x16 neg_ref;
#pragma unroll
    for (int e = 0; e < 16; ++e) neg_ref[e] = 0.f;
    bool first = true;
    float l_run = 0.f;   // per-lane partial row sum (this lane's half of the keys)

    // Scalar walk over the set bits of the decoded symbol row.  The row's words sit one per lane in a vector
    // register (one coalesced load per item, 64 words at a time), so moving on to the next word is a lane read,
    // not a memory access.
    int tiles_left = (int)(key & 0xffffu);          // kept blocks not yet visited, the current one included
    int w_idx = (int)(key >> 21);                    // word of the first kept block
    auto load_words = [&](int w0) -> uint32_t { return w0 + lane < p.nw32 ? wp[w0 + lane] : 0u; };
    uint32_t w_lanes = load_words(w_idx & ~63);
    uint32_t w_bits = 0;
    auto next_block = [&]() -> int {
      while (w_bits == 0u) {
        ++w_idx;
        if (w_idx >= p.nw32) return -1;
        if ((w_idx & 63) == 0) w_lanes = load_words(w_idx);
        w_bits = (uint32_t)__builtin_amdgcn_readlane((int)w_lanes, w_idx & 63);
      }
      const int b = __builtin_ctz(w_bits);
      w_bits &= w_bits - 1u;
      return 32 * w_idx + b;
    };

    // loads lo .. hi-1 of this wave's NLOAD for sub-tile (j, sub)
    auto issue_loads = [&](int j, int sub, auto buf_c, int lo, int hi) {
      constexpr int buf = decltype(buf_c)::value;
      const size_t tile_off = ((size_t)j * BK + (size_t)sub * kKeys) * ROWB;
      const char* gK = Kh + tile_off;
      const char* gV = Vh + tile_off;
      if constexpr (RAGGED) {
        const int valid = p.L - (j * BK + sub * kKeys);     // >= 1: sub-tiles past the end are never requested
        if (valid < kKeys) {
#pragma unroll
          for (int t = lo; t < hi; ++t) {
            const int r = (wave + t * NWAVES) * ROWS_PER_INST + lane / CH;
            const int pch = lane % CH;
            const int src_row = min(r, valid - 1);            // LDS row r receives the last row that exists
            const unsigned dst = (unsigned)(buf * TILEB + (wave + t * NWAVES) * 1024);
            sa_load_to_lds_16B(gK, (unsigned)(src_row * ROWB + ((pch ^ k_swizzle<D>(r)) * 16)), lds_base + dst);
            sa_load_to_lds_16B(gV, (unsigned)(src_row * ROWB + ((pch ^ v_swizzle<D>(r)) * 16)), lds_base + 2 * TILEB + dst);
          }
          return;
        }
      }
#pragma unroll
      for (int t = lo; t < hi; ++t) {
        const unsigned dst = (unsigned)(buf * TILEB + (wave + t * NWAVES) * 1024);
        sa_load_to_lds_16B(gK + (t / TP) * TSTEP, k_goff[t % TP], lds_base + dst);
        sa_load_to_lds_16B(gV + (t / TP) * TSTEP, v_goff[t % TP], lds_base + 2 * TILEB + dst);
      }
    };

    // valid: keys of this sub-tile that exist (RAGGED only); (nj, nsub): the sub-tile to fetch into the other
    // buffer meanwhile, nj < 0 if there is none
    auto compute = [&](auto buf_c, auto other_c, int valid, int nj, int nsub) {
      // the buffer index is a compile-time constant, so every LDS address below is a per-lane
      // register that never changes plus an immediate offset
      constexpr int buf = decltype(buf_c)::value;
      const char* kb = ldsK + buf * TILEB;
      const char* vb = ldsV + buf * TILEB;
      auto k_read = [&](int t) -> bf16x8 {   // operand t = (kb2, ks)
        return *(const bf16x8*)(kb + (t / KS) * 32 * ROWB + k_off[t % KS]);
      };
      auto v_read = [&](int t) -> bf16x8 {   // operand t = ((kb2, ksp), db): keys 16*(t/DB) .. +15, d-block t%DB
        const char* base = vb + (t / DB) * 16 * ROWB + v_off[t % DB];
        const s16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(base));
        const s16x4 t2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(base + 8 * ROWB));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(t1, t2, 0, 1, 2, 3, 4, 5, 6, 7));
      };

      // The sub-tile's 64 keys are two blocks of 32 (one 32x32 S^T accumulator each).  Within this wave the
      // instruction stream is ordered so that the vector work of the softmax sits BETWEEN matrix instructions
      // that do not depend on it -- a wave's VALU instructions issue while its own earlier MFMA is still in the
      // matrix pipe, but only if they come right behind it in program order:
      //   S0:  scores of block 0                      (KS MFMAs)
      //   S1:  scores of block 1      || weights of block 0   (KS MFMAs, 32 vector instructions spread over them)
      //   PV0: O^T += V^T P^T, block 0 || weights of block 1
      //   PV1: O^T += V^T P^T, block 1
      // Weights are rounded to bf16 for the O^T product and the row sum adds up the same rounded values.
      // k-slot s of lane-half h of the O^T MFMA maps to key 32*kb2 + 16*ksp + 8*(s/4) + 4*h + s%4, which is
      // exactly the key order of the S^T accumulator registers 8*ksp .. 8*ksp+7.
      // The exponent's reference is checked after the fact, block by block: the weights are formed against
      // the current reference straight away, and only if their sum shows that one of them left the allowed
      // range is the block's row maximum taken, the reference moved and the block's weights formed again.
      constexpr int CPS = 8 / KS;     // weight chunks (two scores each) per MFMA slot of a group
      f32x16 s[2];
      bf16x8 pb[4];
      bf16x2 ones;
      ones[0] = (__bf16)1.0f;
      ones[1] = (__bf16)1.0f;
      auto chunk = [&](int kb2, int c, float& dl) {
        const int g = 2 * kb2 + c / 4, e = 2 * (c % 4);
        bf16x2 pr;
        pr[0] = (__bf16)__builtin_amdgcn_exp2f(s[kb2][8 * (g & 1) + e] * score_scale);
        pr[1] = (__bf16)__builtin_amdgcn_exp2f(s[kb2][8 * (g & 1) + e + 1] * score_scale);
        pb[g][e] = pr[0];
        pb[g][e + 1] = pr[1];
        dl = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, dl, false);
      };
      auto mask_block = [&](int kb2) {
        // accumulator register e of block kb2 is key 32*kb2 + 8*(e/4) + 4*half + e%4 of the sub-tile
        const int lim = valid - 4 * half;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb2][e] = (32 * kb2 + 8 * (e / 4) + e % 4 >= lim) ? -INFINITY : s[kb2][e];
      };
      // Moves the reference to the row maximum of block kb2 (upwards only, except on the very first block of an
      // item, which sets it).  `other_too`: block 1's scores were formed against the old reference as well.
      auto move_reference = [&](int kb2, bool other_too) {
        float mx = s[kb2][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s[kb2][e]);
        {
          // this lane sees 16 of the 32 scores of its query row in this block; the other half sits in lane ^ 32
          const unsigned bits = __builtin_bit_cast(unsigned, mx);
          const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
          mx = fmaxf(__builtin_bit_cast(float, (unsigned)sw[0]), __builtin_bit_cast(float, (unsigned)sw[1]));
        }
        const float d = first ? mx : fmaxf(mx, 0.f);
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb2][e] -= d;
        if (other_too) {
#pragma unroll
          for (int e = 0; e < 16; ++e) s[1][e] -= d;
        }
        if (!first) {
          const float alpha = __builtin_amdgcn_exp2f(-d * score_scale);
          l_run *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
        }
        const float nr = neg_ref[0] - d;
#pragma unroll
        for (int e = 0; e < 16; ++e) neg_ref[e] = nr;
        first = false;
      };

      bf16x8 ka[NQK];
#pragma unroll
      for (int t = 0; t < kPre; ++t) ka[t] = k_read(t);
      __builtin_amdgcn_s_setprio(kMfmaPrio);
      // ---- S0
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        if (t + kPre < NQK) ka[t + kPre] = k_read(t + kPre);
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[t], qf[t], t == 0 ? neg_ref : s[0], 0, 0, 0);
        // the next sub-tile's loads go out here, a few behind each matrix instruction, instead of in one
        // burst in front of the first one
        if (nj >= 0) issue_loads(nj, nsub, other_c, t * NLOAD / KS, (t + 1) * NLOAD / KS);
      }
      if constexpr (RAGGED) {
        if (valid < kKeys) mask_block(0);
      }
      if (first) move_reference(0, false);     // the first block of an item sets the reference; block 1 is not formed yet
      // first operands of the O^T product: on their way while the scores of block 1 are formed
      bf16x8 va[NPV];
#pragma unroll
      for (int t = 0; t < kPre; ++t) va[t] = v_read(t);
      // ---- S1 || weights of block 0
      float dl0 = 0.f;
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        if (KS + t + kPre < NQK) ka[KS + t + kPre] = k_read(KS + t + kPre);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[KS + t], qf[t], t == 0 ? neg_ref : s[1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cc = 0; cc < CPS; ++cc) chunk(0, t * CPS + cc, dl0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (RAGGED) {
        if (valid < kKeys) mask_block(1);
      }
      // !(sum <= limit) also catches an overflowed (infinite or NaN) sum
      if (__builtin_amdgcn_ballot_w64(!(dl0 <= kSumLimit)) != 0) {
        move_reference(0, true);
        dl0 = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) chunk(0, c, dl0);
      }
      l_run += dl0;
      // ---- PV0 || weights of block 1
      float dl1 = 0.f;
#pragma unroll
      for (int t = 0; t < NPV / 2; ++t) {
        if (t + kPre < NPV) va[t + kPre] = v_read(t + kPre);
        o[t % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[t], pb[t / DB], o[t % DB], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cc = 0; cc < CPS; ++cc) chunk(1, t * CPS + cc, dl1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (__builtin_amdgcn_ballot_w64(!(dl1 <= kSumLimit)) != 0) {
        move_reference(1, false);
        dl1 = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) chunk(1, c, dl1);
      }
      l_run += dl1;
      // ---- PV1
#pragma unroll
      for (int t = NPV / 2; t < NPV; ++t) {
        if (t + kPre < NPV) va[t + kPre] = v_read(t + kPre);
        o[t % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[t], pb[t / DB], o[t % DB], 0, 0, 0);
      }
      __builtin_amdgcn_s_setprio(0);
    };

    // Two sub-tiles per trip, one per LDS buffer: while sub-tile u is computed from one buffer
    // the loads of sub-tile u+1 are in flight into the other.
    using Buf0 = std::integral_constant<int, 0>;
    using Buf1 = std::integral_constant<int, 1>;
    int j = tiles_left > 0 ? (int)(key >> 16) : -1;
    int sub = 0;
    if (j >= 0) issue_loads(j, 0, Buf0{}, 0, NLOAD);
    {
      int qr = wave * 32 + l32;
      if constexpr (RAGGED) qr = min(qr, p.L - 1 - iq * BQ);
      const char* qrow = p.Q + blk_off + (size_t)qr * ROWB + half * 16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 q = *(const bf16x8*)(qrow + ks * 32);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[ks][e] = q[e];
      }
    }
    // the walk continues behind the first kept block
    if (j >= 0) w_bits = (uint32_t)__builtin_amdgcn_readlane((int)w_lanes, w_idx & 63) & ~((2u << (j & 31)) - 1u);
    if (tiles_left <= kDrawTiles) draw_issue();
    auto step = [&](auto cur, auto other) {
      int nj = j, nsub = sub + 1;
      if constexpr (RAGGED) {
        if (nsub < SUB && j * BK + nsub * kKeys >= p.L) nsub = SUB;   // the rest of the last block does not exist
      }
      if (nsub == SUB) {
        nsub = 0;
        nj = next_block();
        if (--tiles_left == kDrawTiles) draw_issue();
      }
      sa_wait_vmem();
      __syncthreads();   // this sub-tile has landed for every wave; the other buffer is free
      compute(cur, other, RAGGED ? p.L - (j * BK + sub * kKeys) : kKeys, nj, nsub);
      j = nj;
      sub = nsub;
    };
    int last = 0;     // buffer of the last sub-tile
    while (j >= 0) {
      step(Buf0{}, Buf1{});
      last = 0;
      if (j < 0) break;
      step(Buf1{}, Buf0{});
      last = 1;
    }

    // O_i = diag(l)^-1 O_acc; both lane halves hold partial sums of the same row.  A lane owns one query row, so
    // stored straight from the accumulators every store instruction would touch 32 rows with 16 bytes each; the
    // block goes through LDS instead and leaves as whole rows, 16 bytes per lane.  The staging area is the buffer
    // that the last sub-tile did NOT use: nothing was fetched into it meanwhile and every wave has finished
    // reading it (it passed the barrier of the last sub-tile after that); each wave stages its own 32 rows, so
    // no barrier is needed here, and the barrier at the top of the next item comes before anything is fetched
    // into that buffer again.
    {
      const unsigned bits = __builtin_bit_cast(unsigned, l_run);
      const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
      const float l_tot = __builtin_bit_cast(float, (unsigned)sw[0]) + __builtin_bit_cast(float, (unsigned)sw[1]);
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      char* const stage = (wave < 2 ? ldsK : ldsV) + (last ^ 1) * TILEB + (wave & 1) * 32 * ROWB;
      // (the lane number passes through an empty asm statement: otherwise the two dozen lane-dependent offsets
      // below are computed once, in front of the item loop, and occupy registers for the whole kernel)
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int srow = ln & 31;
      char* const wr = stage + srow * ROWB + (ln >> 5) * 8;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          // accumulator registers 4*q4 .. 4*q4+3 hold d = 32*db + 8*q4 + 4*half + 0..3
          bf16x2 lo, hi;
          lo[0] = (__bf16)(o[db][4 * q4 + 0] * inv);
          lo[1] = (__bf16)(o[db][4 * q4 + 1] * inv);
          hi[0] = (__bf16)(o[db][4 * q4 + 2] * inv);
          hi[1] = (__bf16)(o[db][4 * q4 + 3] * inv);
          u32x2 pk;
          pk[0] = __builtin_bit_cast(unsigned, lo);
          pk[1] = __builtin_bit_cast(unsigned, hi);
          // 16-byte chunks of a row permuted by the row, so that the 32 rows of one write fall into distinct banks
          *(u32x2*)(wr + (((4 * db + q4) ^ (srow & (CH - 1))) * 16)) = pk;
        }
      constexpr int RPI = 1024 / ROWB;       // rows per store instruction
      char* const obase = p.O + blk_off + (size_t)(wave * 32) * ROWB;
      const int rows_here = RAGGED ? p.L - (iq * BQ + wave * 32) : 32;   // rows of this wave's slab that exist
#pragma unroll
      for (int t = 0; t < 32 / RPI; ++t) {
        const int r = t * RPI + ln / CH, ch = ln % CH;
        const u32x4 v = *(const u32x4*)(stage + r * ROWB + ((ch ^ (r & (CH - 1))) * 16));
        if (!RAGGED || r < rows_here) *(u32x4*)(obase + r * ROWB + ch * 16) = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------
thread_local char g_err[512] = "";

}  // namespace

int sa_fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

namespace {

#define fail sa_fail

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(SPARSE_ATTN_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

struct Shape {
  int B, H, L, D, bq, bk, Tq, Tkv, N, row_bytes, nw32;
};

int check_shape(int B, int H, int L, int D, int bq, int bk, bool need_d, Shape* s) {
  if (B <= 0 || H <= 0 || L <= 0 || bq <= 0 || bk <= 0 || (need_d && D <= 0))
    return fail(SPARSE_ATTN_ERR_INVALID, "sizes must be positive (B=%d H=%d L=%d D=%d block_q=%d block_k=%d)", B, H,
                L, D, bq, bk);
  if ((bq != 64 && bq != 128) || (bk != 64 && bk != 128))
    return fail(SPARSE_ATTN_ERR_UNSUPPORTED, "block_q and block_k must be 64 or 128 (got %d, %d)", bq, bk);
  if (need_d && D != 64 && D != 128) return fail(SPARSE_ATTN_ERR_UNSUPPORTED, "D must be 64 or 128 (got %d)", D);
  const int tq = (L + bq - 1) / bq;      // a short last block counts as a block
  const long long n = (long long)B * H * tq;
  if (tq > kMaxTq) return fail(SPARSE_ATTN_ERR_UNSUPPORTED, "Tq=%d exceeds %d", tq, kMaxTq);
  if (n > 0x3fffffffLL) return fail(SPARSE_ATTN_ERR_UNSUPPORTED, "too many query blocks (%lld)", n);
  s->B = B; s->H = H; s->L = L; s->D = D; s->bq = bq; s->bk = bk;
  s->Tq = tq;
  s->Tkv = (L + bk - 1) / bk;
  s->N = (int)n;
  s->row_bytes = (s->Tkv + 7) / 8;
  s->nw32 = (s->Tkv + 31) / 32;
  return 0;
}

// scratch layout: [queue heads and ends (kQueueBytes)] [order N x 2 u32] [keys N i32] [words N*nw32 u32]
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr size_t kQueueBytes = (size_t)kQueueWords * 4;
size_t workspace_bytes(const Shape& s) {
  return kQueueBytes + align256((size_t)s.N * 8) + align256((size_t)s.N * 4) + align256((size_t)s.N * s.nw32 * 4);
}

struct Scratch {
  void* ptr = nullptr;
  size_t bytes = 0;
};
std::mutex g_mu;
std::map<std::pair<int, void*>, Scratch> g_scratch;

}  // namespace

// Scratch of the entry point that allocates nothing: every GPU the library runs on holds its own copy of this
// array for the life of the process.  In host code the name is only a handle for hipGetSymbolAddress; kernels
// and copies use the per-device address that call returns.
constexpr size_t kStaticScratchBytes = SPARSE_ATTN_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {};

// Address of `scratch` on the current device, looked up once per device.
int static_scratch_ptr(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "device index %d is out of range", dev);
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_static_scratch[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return sa_fail(SPARSE_ATTN_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    g_static_scratch[dev] = ptr;
  }
  *out = g_static_scratch[dev];
  return 0;
}

}  // namespace

int sa_get_scratch(size_t need, hipStream_t stream, void** out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(g_mu);
  Scratch& sc = g_scratch[std::make_pair(dev, (void*)stream)];
  if (sc.bytes < need) {
    if (sc.ptr) {
      HIP_TRY(hipStreamSynchronize(stream));
      HIP_TRY(hipFree(sc.ptr));
      sc.ptr = nullptr;
      sc.bytes = 0;
    }
    const size_t want = need + need / 2;
    HIP_TRY(hipMalloc(&sc.ptr, want));
    sc.bytes = want;
  }
  *out = sc.ptr;
  return 0;
}

namespace {

// Optional per-call event recording (sparse_attn_profile_begin/end): three events per call,
// recorded on the call's stream without any synchronisation.
struct Profile {
  bool on = false;
  int capacity = 0;
  int calls = 0;
  hipEvent_t* ev = nullptr;   // 3 per call: start, after the pre-pass, end
};
Profile g_prof;

bool overlaps(const void* a, const void* b, size_t bytes) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + bytes && y < x + bytes;
}

template <int D, int BQ, int BK, bool RAGGED>
int launch_attn_variant(const AttnParams& p, int grid, hipStream_t stream) {
  constexpr size_t lds = 4 * (size_t)kKeys * D * 2 + 16;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute((const void*)attn_kernel<D, BQ, BK, RAGGED>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)lds);
  });
  if (attr_err != hipSuccess)
    return fail(SPARSE_ATTN_ERR_HIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr_err));
  hipLaunchKernelGGL((attn_kernel<D, BQ, BK, RAGGED>), dim3(grid), dim3(BQ * 2), lds, stream, p);
  HIP_TRY(hipGetLastError());
  return 0;
}

template <int D, int BQ, int BK>
int launch_attn(const AttnParams& p, int grid, hipStream_t stream) {
  if (p.L % BQ || p.L % BK) return launch_attn_variant<D, BQ, BK, true>(p, grid, stream);
  return launch_attn_variant<D, BQ, BK, false>(p, grid, stream);
}

struct PlanBuffers {
  uint32_t* queues;   // live queue heads and ends (kQueueWords)
  uint32_t* order;    // [N][2]
  int32_t* keys;      // [N]
  uint32_t* words;    // [N][nw32]
};

PlanBuffers carve(char* base, const Shape& s) {
  PlanBuffers b;
  b.queues = (uint32_t*)base;
  b.order = (uint32_t*)(base + kQueueBytes);
  b.keys = (int32_t*)(base + kQueueBytes + align256((size_t)s.N * 8));
  b.words = (uint32_t*)(base + kQueueBytes + align256((size_t)s.N * 8) + align256((size_t)s.N * 4));
  return b;
}

}  // namespace

// A stored pre-pass: decoded symbol words and the ordered work list of one set of symbols.
struct sparse_attn_plan {
  Shape s;
  int gran;
  int dev;
  void* mem;               // [initial queue heads and ends (kQueueBytes)] [workspace as carved above]
  uint32_t* queues_init;
  PlanBuffers bufs;
};

namespace {

// Enqueues the symbol pre-pass: decode + count per row, then the ordered work list; the queue heads and
// ends go to `queues_out`.
int launch_plan(const uint8_t* cache_flags, const uint8_t* kv_mask, const Shape& s, int gran, const PlanBuffers& pb,
                uint32_t* queues_out, hipStream_t stream) {
  const int BH = s.B * s.H;
  const int heads_per_xcd = (BH + kXcds - 1) / kXcds;
  int shift = 0;
  while (((heads_per_xcd - 1) >> shift) + 1 > kMaxHeadGroups) ++shift;
  const int groups = ((heads_per_xcd - 1) >> shift) + 1;
  const int sym_Tq = (s.Tq + gran - 1) / gran;
  const int sym_row_bytes = ((s.Tkv + gran - 1) / gran + 7) / 8;
  hipLaunchKernelGGL(plan_rows, dim3((s.N + 255) / 256), dim3(256), 0, stream, cache_flags, kv_mask, s.N, s.Tq, s.Tkv,
                     gran, sym_Tq, sym_row_bytes, s.nw32, pb.words, pb.keys);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(plan_order, dim3(1), dim3(kOrderThreads), 0, stream, pb.keys, s.N, s.Tq, s.Tkv, shift, groups,
                     pb.order, queues_out);
  HIP_TRY(hipGetLastError());
  return 0;
}

struct Forecast {
  const void* const* terms;   // host array of n device pointers
  const float* coef;          // host array of n weights
  int n;
};

int run(const void* Q, const void* K, const void* V, const uint8_t* cache_flags, const uint8_t* kv_mask,
        const void* O_cache, void* O, int B, int H, int L, int D, int bq, int bk, hipStream_t stream, float* plan_ms,
        float* attn_ms, bool timed, const Forecast* fc = nullptr, const sparse_attn_plan* plan = nullptr,
        bool static_scratch = false, void* user_ws = nullptr, size_t user_ws_bytes = 0, bool use_user_ws = false) {
  Shape s;
  if (int rc = check_shape(B, H, L, D, bq, bk, true, &s)) return rc;
  if (!Q || !K || !V || !O) return fail(SPARSE_ATTN_ERR_INVALID, "Q, K, V and O must not be NULL");
  const size_t tensor_bytes = (size_t)B * H * L * D * 2;
  if (overlaps(O, Q, tensor_bytes) || overlaps(O, K, tensor_bytes) || overlaps(O, V, tensor_bytes))
    return fail(SPARSE_ATTN_ERR_INVALID, "O must not overlap Q, K or V");
  if (O_cache && O_cache != O && overlaps(O, O_cache, tensor_bytes))
    return fail(SPARSE_ATTN_ERR_INVALID, "O_cache must be O itself or must not overlap O");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O | (uintptr_t)O_cache) & 15)
    return fail(SPARSE_ATTN_ERR_INVALID, "tensor base pointers must be 16-byte aligned");
  if (fc) {
    if (fc->n < 1 || fc->n > kMaxTerms)
      return fail(SPARSE_ATTN_ERR_UNSUPPORTED, "n_terms=%d must be between 1 and %d", fc->n, kMaxTerms);
    if (!fc->terms || !fc->coef) return fail(SPARSE_ATTN_ERR_INVALID, "O_terms and coef must not be NULL");
    for (int d = 0; d < fc->n; ++d) {
      if (!fc->terms[d]) return fail(SPARSE_ATTN_ERR_INVALID, "O_terms[%d] must not be NULL", d);
      if ((uintptr_t)fc->terms[d] & 15) return fail(SPARSE_ATTN_ERR_INVALID, "O_terms[%d] must be 16-byte aligned", d);
      if (overlaps(O, fc->terms[d], tensor_bytes)) return fail(SPARSE_ATTN_ERR_INVALID, "O_terms[%d] must not overlap O", d);
      if (!(fc->coef[d] == fc->coef[d]) || fc->coef[d] - fc->coef[d] != 0.f)
        return fail(SPARSE_ATTN_ERR_INVALID, "coef[%d] must be finite", d);
    }
  }

  if (use_user_ws) {
    const size_t need = workspace_bytes(s);
    if (!user_ws) return fail(SPARSE_ATTN_ERR_INVALID, "workspace must not be NULL");
    if ((uintptr_t)user_ws & 255) return fail(SPARSE_ATTN_ERR_INVALID, "workspace must be 256-byte aligned");
    if (user_ws_bytes < need)
      return fail(SPARSE_ATTN_ERR_INVALID, "workspace holds %zu bytes, this shape needs %zu (sparse_attn_workspace_bytes)",
                  user_ws_bytes, need);
  }
  if (static_scratch && workspace_bytes(s) > kStaticScratchBytes)
    return fail(SPARSE_ATTN_ERR_UNSUPPORTED,
                "this shape needs %zu bytes of scratch, the no-allocation entry point holds %zu "
                "(B*H*Tq*(ceil(Tkv/32)+3)*4 bytes must fit)", workspace_bytes(s), kStaticScratchBytes);

  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (plan && dev != plan->dev) return fail(SPARSE_ATTN_ERR_INVALID, "the plan was created on device %d, current device is %d", plan->dev, dev);

  PlanBuffers pb;
  if (plan) {
    pb = plan->bufs;
  } else if (use_user_ws) {
    pb = carve((char*)user_ws, s);
  } else if (static_scratch) {
    void* ws = nullptr;
    if (int rc = static_scratch_ptr(&ws)) return rc;
    pb = carve((char*)ws, s);
  } else {
    void* ws = nullptr;
    if (int rc = sa_get_scratch(workspace_bytes(s), stream, &ws)) return rc;
    pb = carve((char*)ws, s);
  }

  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));

  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  bool record = timed;
  if (timed) {
    for (auto& e : ev) HIP_TRY(hipEventCreate(&e));
  } else {
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_prof.on && g_prof.calls < g_prof.capacity) {
      for (int t = 0; t < 3; ++t) ev[t] = g_prof.ev[3 * g_prof.calls + t];
      ++g_prof.calls;
      record = true;
    }
  }
  if (record) HIP_TRY(hipEventRecord(ev[0], stream));

  if (plan) {
    hipLaunchKernelGGL(reset_queues, dim3(1), dim3(64), 0, stream, plan->queues_init, pb.queues);
    HIP_TRY(hipGetLastError());
  } else {
    if (int rc = launch_plan(cache_flags, kv_mask, s, 1, pb, pb.queues, stream)) return rc;
  }
  if (record) HIP_TRY(hipEventRecord(ev[1], stream));

  uint32_t* const queues = pb.queues;
  uint32_t* const order = pb.order;
  uint32_t* const words = pb.words;
  AttnParams p;
  p.Q = (const char*)Q;
  p.K = (const char*)K;
  p.V = (const char*)V;
  p.O_cache = (const char*)O_cache;
  p.O = (char*)O;
  p.words = words;
  p.order = order;
  p.queues = queues;
  p.N = s.N;
  p.Tq = s.Tq;
  p.Tkv = s.Tkv;
  p.L = L;
  p.nw32 = s.nw32;
  p.do_copy = (O_cache != nullptr && O_cache != O) ? 1 : 0;
  for (int d = 0; d < kMaxTerms; ++d) p.coef[d] = 0.f;
  for (int d = 0; d + 1 < kMaxTerms; ++d) p.term[d] = nullptr;
  p.n_terms = 0;
  if (fc) {
    p.O_cache = (const char*)fc->terms[0];
    if (fc->n == 1 && fc->coef[0] == 1.0f) {
      p.do_copy = 1;                       // order 0 with weight 1 is the plain copy
    } else {
      p.n_terms = fc->n;
      for (int d = 0; d < fc->n; ++d) p.coef[d] = fc->coef[d];
      for (int d = 1; d < fc->n; ++d) p.term[d - 1] = (const char*)fc->terms[d];
    }
  }
  p.scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  // persistent grid: two workgroups per CU (64 KiB of LDS each), fewer if there are fewer items
  const int grid = s.N < 2 * cus ? s.N : 2 * cus;

  int rc = 0;
  if (D == 128 && bq == 128 && bk == 128) rc = launch_attn<128, 128, 128>(p, grid, stream);
  else if (D == 128 && bq == 128 && bk == 64) rc = launch_attn<128, 128, 64>(p, grid, stream);
  else if (D == 128 && bq == 64 && bk == 128) rc = launch_attn<128, 64, 128>(p, grid, stream);
  else if (D == 128 && bq == 64 && bk == 64) rc = launch_attn<128, 64, 64>(p, grid, stream);
  else if (D == 64 && bq == 128 && bk == 128) rc = launch_attn<64, 128, 128>(p, grid, stream);
  else if (D == 64 && bq == 128 && bk == 64) rc = launch_attn<64, 128, 64>(p, grid, stream);
  else if (D == 64 && bq == 64 && bk == 128) rc = launch_attn<64, 64, 128>(p, grid, stream);
  else rc = launch_attn<64, 64, 64>(p, grid, stream);
  if (rc) return rc;

  if (record) HIP_TRY(hipEventRecord(ev[2], stream));
  if (timed) {
    HIP_TRY(hipEventSynchronize(ev[2]));
    float a = 0.f, b = 0.f;
    HIP_TRY(hipEventElapsedTime(&a, ev[0], ev[1]));
    HIP_TRY(hipEventElapsedTime(&b, ev[1], ev[2]));
    if (plan_ms) *plan_ms = a;
    if (attn_ms) *attn_ms = b;
    for (auto& e : ev) HIP_TRY(hipEventDestroy(e));
  }
  return 0;
}

}  // namespace

extern "C" {

int sparse_attn_fwd(const void* Q, const void* K, const void* V, const uint8_t* cache_flags, const uint8_t* kv_mask,
                    const void* O_cache, void* O, int B, int H, int L, int D, int block_q, int block_k) {
  return run(Q, K, V, cache_flags, kv_mask, O_cache, O, B, H, L, D, block_q, block_k, nullptr, nullptr, nullptr,
             false);
}

int sparse_attn_fwd_stream(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                           const uint8_t* kv_mask, const void* O_cache, void* O, int B, int H, int L, int D,
                           int block_q, int block_k, void* hip_stream) {
  return run(Q, K, V, cache_flags, kv_mask, O_cache, O, B, H, L, D, block_q, block_k, (hipStream_t)hip_stream,
             nullptr, nullptr, false);
}

int sparse_attn_fwd_timed(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                          const uint8_t* kv_mask, const void* O_cache, void* O, int B, int H, int L, int D,
                          int block_q, int block_k, void* hip_stream, float* plan_ms, float* attn_ms) {
  return run(Q, K, V, cache_flags, kv_mask, O_cache, O, B, H, L, D, block_q, block_k, (hipStream_t)hip_stream,
             plan_ms, attn_ms, true);
}

int sparse_attn_fwd_noalloc(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                            const uint8_t* kv_mask, const void* O_cache, void* O, int B, int H, int L, int D,
                            int block_q, int block_k, void* hip_stream) {
  return run(Q, K, V, cache_flags, kv_mask, O_cache, O, B, H, L, D, block_q, block_k, (hipStream_t)hip_stream,
             nullptr, nullptr, false, nullptr, nullptr, true);
}

int sparse_attn_fwd_forecast(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                             const uint8_t* kv_mask, const void* const* O_terms, const float* coef, int n_terms, void* O,
                             int B, int H, int L, int D, int block_q, int block_k, void* hip_stream) {
  const Forecast fc = {O_terms, coef, n_terms};
  return run(Q, K, V, cache_flags, kv_mask, nullptr, O, B, H, L, D, block_q, block_k, (hipStream_t)hip_stream, nullptr,
             nullptr, false, &fc);
}

int sparse_attn_plan_create(const uint8_t* cache_flags, const uint8_t* kv_mask, int B, int H, int L, int block_q,
                            int block_k, int granularity, void* hip_stream, sparse_attn_plan** plan_out) {
  if (!plan_out) return fail(SPARSE_ATTN_ERR_INVALID, "plan_out must not be NULL");
  *plan_out = nullptr;
  Shape s;
  if (int rc = check_shape(B, H, L, 0, block_q, block_k, false, &s)) return rc;
  if (granularity < 1 || granularity > 64)
    return fail(SPARSE_ATTN_ERR_INVALID, "granularity=%d must be between 1 and 64", granularity);
  sparse_attn_plan* pl = new (std::nothrow) sparse_attn_plan();
  if (!pl) return fail(SPARSE_ATTN_ERR_HIP, "out of host memory");
  pl->s = s;
  pl->gran = granularity;
  pl->mem = nullptr;
  hipError_t e = hipGetDevice(&pl->dev);
  if (e == hipSuccess) e = hipMalloc(&pl->mem, kQueueBytes + workspace_bytes(s));
  if (e != hipSuccess) {
    delete pl;
    return fail(SPARSE_ATTN_ERR_HIP, "plan allocation failed: %s", hipGetErrorString(e));
  }
  pl->queues_init = (uint32_t*)pl->mem;
  pl->bufs = carve((char*)pl->mem + kQueueBytes, s);
  if (int rc = launch_plan(cache_flags, kv_mask, s, granularity, pl->bufs, pl->queues_init, (hipStream_t)hip_stream)) {
    (void)hipFree(pl->mem);
    delete pl;
    return rc;
  }
  *plan_out = pl;
  return 0;
}

int sparse_attn_plan_run(sparse_attn_plan* plan, const void* Q, const void* K, const void* V, const void* O_cache,
                         void* O, int D, void* hip_stream) {
  if (!plan) return fail(SPARSE_ATTN_ERR_INVALID, "plan must not be NULL");
  const Shape& s = plan->s;
  return run(Q, K, V, nullptr, nullptr, O_cache, O, s.B, s.H, s.L, D, s.bq, s.bk, (hipStream_t)hip_stream, nullptr,
             nullptr, false, nullptr, plan);
}

int sparse_attn_plan_run_forecast(sparse_attn_plan* plan, const void* Q, const void* K, const void* V,
                                  const void* const* O_terms, const float* coef, int n_terms, void* O, int D,
                                  void* hip_stream) {
  if (!plan) return fail(SPARSE_ATTN_ERR_INVALID, "plan must not be NULL");
  const Shape& s = plan->s;
  const Forecast fc = {O_terms, coef, n_terms};
  return run(Q, K, V, nullptr, nullptr, nullptr, O, s.B, s.H, s.L, D, s.bq, s.bk, (hipStream_t)hip_stream, nullptr,
             nullptr, false, &fc, plan);
}

int sparse_attn_plan_destroy(sparse_attn_plan* plan) {
  if (!plan) return 0;
  const hipError_t e = hipFree(plan->mem);     // waits for work that still uses the buffer
  delete plan;
  if (e != hipSuccess) return fail(SPARSE_ATTN_ERR_HIP, "hipFree failed: %s", hipGetErrorString(e));
  return 0;
}

int sparse_attn_fwd_workspace(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                              const uint8_t* kv_mask, const void* O_cache, void* O, int B, int H, int L, int D,
                              int block_q, int block_k, void* workspace, size_t workspace_size, void* hip_stream) {
  return run(Q, K, V, cache_flags, kv_mask, O_cache, O, B, H, L, D, block_q, block_k, (hipStream_t)hip_stream, nullptr,
             nullptr, false, nullptr, nullptr, false, workspace, workspace_size, true);
}

int sparse_attn_release_scratch(void* hip_stream) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_scratch.find(std::make_pair(dev, hip_stream));
    if (it == g_scratch.end()) return 0;
    ptr = it->second.ptr;
    g_scratch.erase(it);
  }
  if (ptr) {
    HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));    // work that still uses the buffer
    HIP_TRY(hipFree(ptr));
  }
  return 0;
}

size_t sparse_attn_workspace_bytes(int B, int H, int L, int block_q, int block_k) {
  Shape s;
  if (check_shape(B, H, L, 0, block_q, block_k, false, &s)) return 0;
  return workspace_bytes(s);
}

int sparse_attn_count_kept(const uint8_t* cache_flags, const uint8_t* kv_mask, int B, int H, int L, int block_q,
                           int block_k, unsigned long long* kept_pairs, unsigned long long* total_pairs) {
  Shape s;
  if (int rc = check_shape(B, H, L, 0, block_q, block_k, false, &s)) return rc;
  if (!kept_pairs) return fail(SPARSE_ATTN_ERR_INVALID, "kept_pairs must not be NULL");
  unsigned long long kept = 0;
  for (int row = 0; row < s.N; ++row) {
    if (cache_flags && cache_flags[row]) continue;
    if (!kv_mask) {
      kept += (unsigned long long)s.Tkv;
      continue;
    }
    const uint8_t* r = kv_mask + (size_t)row * s.row_bytes;
    for (int byte = 0; byte < s.row_bytes; ++byte) {
      unsigned v = r[byte];
      const int valid = s.Tkv - 8 * byte;
      if (valid < 8) v &= (0xffu << (8 - valid)) & 0xffu;
      kept += (unsigned long long)__builtin_popcount(v);
    }
  }
  *kept_pairs = kept;
  if (total_pairs) *total_pairs = (unsigned long long)s.N * (unsigned long long)s.Tkv;
  return 0;
}

int sparse_attn_pack_mask(const uint8_t* logical, long long rows, int Tkv, uint8_t* packed) {
  if (!logical || !packed || rows < 0 || Tkv <= 0)
    return fail(SPARSE_ATTN_ERR_INVALID, "pack_mask: bad arguments (rows=%lld Tkv=%d)", rows, Tkv);
  const int row_bytes = (Tkv + 7) / 8;
  for (long long r = 0; r < rows; ++r) {
    const uint8_t* src = logical + (size_t)r * Tkv;
    uint8_t* dst = packed + (size_t)r * row_bytes;
    for (int byte = 0; byte < row_bytes; ++byte) {
      unsigned v = 0;
      for (int t = 0; t < 8; ++t) {
        const int j = 8 * byte + t;
        if (j < Tkv && src[j]) v |= 0x80u >> t;
      }
      dst[byte] = (uint8_t)v;
    }
  }
  return 0;
}

int sparse_attn_profile_begin(int max_calls) {
  if (max_calls <= 0 || max_calls > (1 << 20)) return fail(SPARSE_ATTN_ERR_INVALID, "profile_begin: bad max_calls %d", max_calls);
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_prof.on) return fail(SPARSE_ATTN_ERR_INVALID, "profile_begin: a profile is already open");
  g_prof.ev = new hipEvent_t[3 * (size_t)max_calls];
  for (int t = 0; t < 3 * max_calls; ++t) {
    hipError_t e = hipEventCreate(&g_prof.ev[t]);
    if (e != hipSuccess) {
      for (int u = 0; u < t; ++u) (void)hipEventDestroy(g_prof.ev[u]);
      delete[] g_prof.ev;
      g_prof.ev = nullptr;
      return fail(SPARSE_ATTN_ERR_HIP, "hipEventCreate failed: %s", hipGetErrorString(e));
    }
  }
  g_prof.capacity = max_calls;
  g_prof.calls = 0;
  g_prof.on = true;
  return 0;
}

int sparse_attn_profile_end(int* calls, double* plan_ms_total, double* attn_ms_total) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_prof.on) return fail(SPARSE_ATTN_ERR_INVALID, "profile_end: no profile is open");
  int rc = 0;
  double plan = 0.0, attn = 0.0;
  for (int c = 0; c < g_prof.calls && rc == 0; ++c) {
    hipError_t e = hipEventSynchronize(g_prof.ev[3 * c + 2]);
    float a = 0.f, b = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&a, g_prof.ev[3 * c], g_prof.ev[3 * c + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&b, g_prof.ev[3 * c + 1], g_prof.ev[3 * c + 2]);
    if (e != hipSuccess) rc = fail(SPARSE_ATTN_ERR_HIP, "profile_end: %s", hipGetErrorString(e));
    plan += a;
    attn += b;
  }
  for (int t = 0; t < 3 * g_prof.capacity; ++t) (void)hipEventDestroy(g_prof.ev[t]);
  delete[] g_prof.ev;
  if (calls) *calls = g_prof.calls;
  if (plan_ms_total) *plan_ms_total = plan;
  if (attn_ms_total) *attn_ms_total = attn;
  g_prof = Profile();
  return rc;
}


const char* sparse_attn_last_error(void) { return g_err; }

int sparse_attn_version(void) { return 100; }

}  // extern "C"
