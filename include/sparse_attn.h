/*
 * sparse_attn.h -- C ABI of the MI355X (gfx950) FlashOmni attention library.
 *
 * The operation is the paper's Algorithm 1 ("FlashOmni Attention"): a FlashAttention-style
 * fused QK^T -> online softmax -> PV pass over bf16 Q/K/V that is steered by two block
 * level sparse symbols (Definitions 1 and 2, Section 3.3):
 *   - a per (batch, head, query block) cache flag, the spatial-axis symbol S_c: a flagged
 *     block is not computed, its output is reused from a cached output tensor
 *     ("cache-then-reuse"; OP_reuse is the identity, a bit-exact copy, in sparse_attn_fwd
 *     and a Taylor-series forecast in sparse_attn_fwd_forecast);
 *   - a bit-packed per (batch, head, query block, key block) mask, the reduction-axis symbol
 *     S_s: a pair whose bit is 0 is skipped, its K/V tile is never loaded, and the softmax
 *     normalises over the kept key blocks only ("compute-on-demand").
 *
 * Conventions shared by every entry point
 *   - Tensors Q, K, V, O_cache, O: bf16, shape [B, H, L, D], D fastest, fully contiguous,
 *     16-byte aligned base.  Tq = ceil(L / block_q), Tkv = ceil(L / block_k).
 *   - cache_flags: uint8 [B, H, Tq]; non-zero = reuse the block from O_cache.  Note the
 *     polarity: the paper's logical mask M_c holds 0 for cached blocks, this flag holds 1.
 *     NULL = no block is cached.
 *   - kv_mask: uint8 [B, H, Tq, ceil(Tkv / 8)]; logical entry j of a row lives in byte j / 8
 *     at bit 7 - j % 8 (most significant bit first, as the worked example of Section 3.3
 *     [1,1,1,0] -> 0b11100000 = 224 fixes); 1 = compute the pair.  Every (b, h, i) row starts
 *     on a byte boundary; bits past Tkv are ignored; rows of cached blocks are ignored.
 *     NULL = every pair is kept (dense attention).
 *   - A computed block whose mask row is empty is written as +0.0.
 *   - Scores are scaled by 1 / sqrt(D) (Section 3.1).  Products run on bf16 MFMA with fp32
 *     accumulation, the softmax weights are rounded to bf16 before the PV product, the result
 *     is rounded to bf16 (nearest even).
 *   - Supported shapes: D in {64, 128}; block_q, block_k in {64, 128}; any L >= 1 with
 *     Tq = ceil(L / block_q) <= 16384 and Tkv = ceil(L / block_k) (Definition 1): the last query
 *     block and the last key block may be short; nothing past row L - 1 of a head is read or
 *     written.  The projections and the symbol generation below accept any L as well.
 *   - "device" pointers are HIP device memory owned by the caller; the library never frees
 *     or keeps them.  "host" pointers are ordinary host memory.
 *   - Return value: 0 on success, a negative SPARSE_ATTN_ERR_* code otherwise; a message for
 *     the last failure on the calling thread is available from sparse_attn_last_error().
 *     Argument validation happens before any HIP call, and nothing is written on failure.
 *   - There is no CPU fallback: without a usable HIP device the compute entry points fail
 *     with SPARSE_ATTN_ERR_HIP.
 */
#ifndef SPARSE_ATTN_H
#define SPARSE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPARSE_ATTN_OK 0
#define SPARSE_ATTN_ERR_INVALID (-1)     /* NULL pointer, non-positive size, a size that does not fit the others, O aliases an input */
#define SPARSE_ATTN_ERR_UNSUPPORTED (-2) /* D or block size outside the supported set, Tq too large */
#define SPARSE_ATTN_ERR_HIP (-3)         /* a HIP runtime call failed; see sparse_attn_last_error() */

/*
 * Algorithm 1 on the HIP null stream.
 *   Q, K, V      device, bf16 [B,H,L,D], read only
 *   cache_flags  device, uint8 [B,H,Tq] or NULL
 *   kv_mask      device, uint8 [B,H,Tq,ceil(Tkv/8)] or NULL
 *   O_cache      device, bf16 [B,H,L,D]; NULL or equal to O means the cached blocks of O are
 *                already in place (the early-continue of Algorithm 1's cache branch) and are
 *                not touched
 *   O            device, bf16 [B,H,L,D], written (computed blocks always; cached blocks only
 *                when O_cache is a different tensor).  Must not overlap Q, K or V.
 * The call is asynchronous with respect to the host.  It uses a per (device, stream) scratch
 * buffer that the library allocates on first use and grows when needed (hipMalloc); calls that
 * overlap in time on one stream object are not supported.
 */
int sparse_attn_fwd(const void* Q, const void* K, const void* V,
                    const uint8_t* cache_flags, const uint8_t* kv_mask,
                    const void* O_cache, void* O,
                    int B, int H, int L, int D, int block_q, int block_k);

/* Same, enqueued on the caller's stream (a hipStream_t passed as void*; NULL = null stream). */
int sparse_attn_fwd_stream(const void* Q, const void* K, const void* V,
                           const uint8_t* cache_flags, const uint8_t* kv_mask,
                           const void* O_cache, void* O,
                           int B, int H, int L, int D, int block_q, int block_k,
                           void* hip_stream);

/*
 * sparse_attn_fwd_stream for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same output bits; the symbol
 * pre-pass (queue counters, work list, kept counts, decoded symbol words) lives in a fixed array of
 * SPARSE_ATTN_NOALLOC_SCRATCH_BYTES bytes inside the library's device image instead of an allocated buffer.
 * The call allocates and frees nothing, on the host side of HIP or on the device.
 *   - A shape is accepted iff sparse_attn_workspace_bytes(B, H, L, block_q, block_k) fits in the array
 *     (about 4 * B*H*Tq * (ceil(Tkv/32) + 3) bytes: 0.3 MiB at B=1, H=24, L=33024 with 128 x 128 blocks);
 *     anything larger returns SPARSE_ATTN_ERR_UNSUPPORTED with a message that names both sizes.
 *   - Every GPU the library runs on holds its own copy of the array until the process ends.  All calls on a
 *     GPU share it, whatever their stream: two calls that overlap in time on one GPU race and give wrong
 *     results.  Calls on one stream, or otherwise ordered, are fine; the array keeps the previous call's
 *     contents and every word a call reads is written by that call's own pre-pass first.
 */
#define SPARSE_ATTN_NOALLOC_SCRATCH_BYTES ((size_t)2 << 20)
int sparse_attn_fwd_noalloc(const void* Q, const void* K, const void* V,
                            const uint8_t* cache_flags, const uint8_t* kv_mask,
                            const void* O_cache, void* O,
                            int B, int H, int L, int D, int block_q, int block_k,
                            void* hip_stream);

/*
 * Measurement variant: same work as sparse_attn_fwd_stream, bracketed by HIP events on the
 * given stream, synchronised before returning.  plan_ms (host, may be NULL) receives the
 * duration of the symbol pre-pass (decode, count and ordering of work items), attn_ms (host,
 * may be NULL) the duration of the attention kernel itself, both in milliseconds.
 */
int sparse_attn_fwd_timed(const void* Q, const void* K, const void* V,
                          const uint8_t* cache_flags, const uint8_t* kv_mask,
                          const void* O_cache, void* O,
                          int B, int H, int L, int D, int block_q, int block_k,
                          void* hip_stream, float* plan_ms, float* attn_ms);

/*
 * Sparse query projection (GEMM-Q, Section 3.5, Observation 2 / Equation 2): the step right before
 * the attention call.  For every (b, h, i) whose cache flag is clear
 *     Q[b, h, i*block_q : (i+1)*block_q, :] = X[b, i*block_q : (i+1)*block_q, :] . W_h^T (+ bias_h)
 * and a flagged block of Q is left untouched (its attention output is reused from the cache, so its
 * queries are never read).  The per-token RMSNorm and RoPE of Equation 2 are not part of this call.
 *   X            device, bf16 [B, L, C], C fastest
 *   W            device, bf16 [H*D, C]: one row per output feature (the layout a Linear layer
 *                stores), head h owns rows h*D .. (h+1)*D-1
 *   bias         device, bf16 [H*D], or NULL
 *   cache_flags  device, uint8 [B, H, ceil(L/block_q)], same meaning as in sparse_attn_fwd, or NULL
 *   Q            device, bf16 [B, H, L, D], written for the computed blocks (fp32 accumulation,
 *                rounded to nearest even); must not overlap X or W
 * Supported: D and block_q in {64, 128}, C a multiple of 64; any L >= 1 (the last token block may be short,
 * flags are [B, H, ceil(L / block_q)]).
 * Errors as for sparse_attn_fwd.  Allocates nothing.
 */
int sparse_gemm_q(const void* X, const void* W, const void* bias, const uint8_t* cache_flags, void* Q,
                  int B, int L, int C, int H, int D, int block_q);
int sparse_gemm_q_stream(const void* X, const void* W, const void* bias, const uint8_t* cache_flags, void* Q,
                         int B, int L, int C, int H, int D, int block_q, void* hip_stream);

/*
 * Reusable plan (Section 3.2: symbols are refreshed at an Update step and then drive the following Dispatch
 * steps unchanged; Section 3.3: one symbol may cover n x n tiles).  sparse_attn_plan_create runs the
 * symbol pre-pass once -- decode of S_c and S_s, kept-pair counts, the ordered work list -- and keeps its
 * result on the device; sparse_attn_plan_run is sparse_attn_fwd_stream without that pre-pass.
 *   cache_flags  device, uint8 [B, H, ceil(Tq / granularity)] or NULL
 *   kv_mask      device, uint8 [B, H, ceil(Tq / granularity), ceil(ceil(Tkv / granularity) / 8)] or NULL, bit
 *                order as for sparse_attn_fwd: tile (i, j) is computed iff bit (i / granularity, j / granularity)
 *                is set, the decoding functions F and J of Section 3.4 with n = granularity
 *   granularity  1..64; block_q x block_k stays the tile the kernel works on
 * create allocates the plan's device buffer (hipMalloc) and enqueues the pre-pass on hip_stream; the symbol
 * arrays may be changed or freed once that work has run.  The plan belongs to the device that was current at
 * create.  run allocates nothing; it must be ordered after create (same stream, or synchronise), and two
 * runs of one plan must not overlap in time (a run resets and consumes the plan's queue counters, which is why
 * the plan is not const).  destroy waits for the device
 * and frees.  Errors as for sparse_attn_fwd; on failure *plan is NULL.
 */
typedef struct sparse_attn_plan sparse_attn_plan;
int sparse_attn_plan_create(const uint8_t* cache_flags, const uint8_t* kv_mask, int B, int H, int L, int block_q,
                            int block_k, int granularity, void* hip_stream, sparse_attn_plan** plan);
int sparse_attn_plan_run(sparse_attn_plan* plan, const void* Q, const void* K, const void* V, const void* O_cache,
                         void* O, int D, void* hip_stream);
int sparse_attn_plan_destroy(sparse_attn_plan* plan);
/*
 * sparse_attn_plan_run with the Taylor-series OP_reuse of sparse_attn_fwd_forecast in its cache branch (Section
 * 3.2's Dispatch step with forecast features: stored symbols, stored pre-pass, cached blocks forecast from their
 * terms).  O_terms, coef, n_terms as for sparse_attn_fwd_forecast; everything else as for sparse_attn_plan_run.
 */
int sparse_attn_plan_run_forecast(sparse_attn_plan* plan, const void* Q, const void* K, const void* V,
                                  const void* const* O_terms, const float* coef, int n_terms, void* O, int D,
                                  void* hip_stream);

/*
 * GEMM-Q with the two token-wise operations of Equation 2 fused into its epilogue:
 *     Q[b,h,token,:] = OP_RoPE(OP_RMSNorm(X[b,token,:] . W_h^T + bias_h))
 * for every (b,h,i) whose flag is clear (flagged tiles return at once, as in sparse_gemm_q).
 *   OP_RMSNorm  y / sqrt(mean over the head's D channels of y^2 + eps) * norm_weight
 *   OP_RoPE     adjacent channel pairs (2m, 2m+1) of token l are rotated by the angle whose cosine and sine are
 *               rope_cos[l, m] and rope_sin[l, m]:  (y0, y1) -> (y0 cos - y1 sin, y0 sin + y1 cos)
 * fp32 throughout after the bf16 MFMA products, one rounding to bf16 at the end.
 *   norm_weight  device, bf16 [D] (shared by all heads), or NULL for ones
 *   eps          finite, >= 0
 *   rope_cos, rope_sin  device, fp32 [L, D/2], 8-byte aligned (shared by batches and heads), or both NULL
 *                for no rotation
 * Everything else as for sparse_gemm_q_stream.  Allocates nothing.
 */
int sparse_gemm_q_norm_rope(const void* X, const void* W, const void* bias, const void* norm_weight, float eps,
                            const float* rope_cos, const float* rope_sin, const uint8_t* cache_flags, void* Q,
                            int B, int L, int C, int H, int D, int block_q, void* hip_stream);

/*
 * Sparse output projection (GEMM-O, Section 3.5, Observation 3 / Equations 3-4): the step right after
 * the attention call.  For every token block i and every output channel n
 *     Out[b, token, n] = addend[b, token, n] + bias[n]
 *                        + sum over heads h with (cache_flags[b,h,i] != 0) == select_cached of
 *                          O[b, h, token, :] . W[n, h*D : (h+1)*D]
 * The paper's two stages are two calls.  Stage 1, at an Update step: select_cached = 1, addend = NULL,
 * bias = NULL; the result is the cached bias B_c, the part of the projection that comes from the heads
 * whose attention output will be reused.  Stage 2, at every step: select_cached = 0, addend = B_c;
 * heads whose flag is set are skipped along the reduction axis (their O and W columns are never
 * loaded).  With cache_flags NULL no head counts as cached.
 *   O            device, bf16 [B, H, L, D] (the attention output)
 *   W            device, bf16 [C_out, H*D]: one row per output feature (Linear layer layout)
 *   bias         device, bf16 [C_out], or NULL
 *   cache_flags  device, uint8 [B, H, ceil(L/block_q)] or NULL
 *   addend       device, bf16 [B, L, C_out], NULL, or Out itself (accumulate in place)
 *   Out          device, bf16 [B, L, C_out], written everywhere (fp32 accumulation, rounded to
 *                nearest even); must not overlap O or W
 * Supported: D and block_q in {64, 128}, H <= 64, C_out a multiple of 128; any L >= 1 (the last token block may
 * be short, flags are [B, H, ceil(L / block_q)]).
 * Errors as for sparse_attn_fwd.  Allocates nothing.
 */
int sparse_gemm_o(const void* O, const void* W, const void* bias, const uint8_t* cache_flags, int select_cached,
                  const void* addend, void* Out, int B, int H, int L, int D, int C_out, int block_q);
int sparse_gemm_o_stream(const void* O, const void* W, const void* bias, const uint8_t* cache_flags,
                         int select_cached, const void* addend, void* Out, int B, int H, int L, int D, int C_out,
                         int block_q, void* hip_stream);
/*
 * Stage 2 of GEMM-O at a Dispatch step with the output "initialised by OP_reuse(B_c)" (Section 3.5) in one call:
 *     Out = OP_reuse(B_c terms) + bias + sum over the heads whose flag is clear of O^h . W^h
 * with OP_reuse(terms) = sum_d coef[d] * terms[d] as defined for sparse_op_reuse below (fp32 sum in term order,
 * rounded to bf16 once, then used as the addend): the result is bit-identical to sparse_op_reuse into a buffer
 * followed by sparse_gemm_o(..., select_cached = 0, addend = that buffer), without writing the forecast bias to
 * memory and reading it back.
 *   terms    HOST array of n_terms (1..4) DEVICE pointers, each bf16 [B, L, C_out], 16-byte aligned; a term may be
 *            Out itself (in place), otherwise it must not overlap Out
 *   coef     HOST array of n_terms finite weights (sparse_taylor_coefficients)
 * Everything else as for sparse_gemm_o_stream.  Allocates nothing.
 */
int sparse_gemm_o_reuse(const void* O, const void* W, const void* bias, const uint8_t* cache_flags,
                        const void* const* terms, const float* coef, int n_terms, void* Out, int B, int H, int L, int D,
                        int C_out, int block_q, void* hip_stream);

/*
 * OP_reuse as a Taylor-series forecast (Section 3.3: cached blocks are forecast from stored features and their
 * derivatives; Section 3.4: the cache-then-reuse branch is an element-wise sum of products fused into the
 * attention kernel, or a separate element-wise kernel; Section 3.5: the same operation transforms the cached
 * bias B_c).  The operation is
 *     OP_reuse(terms) = sum over d = 0..n_terms-1 of coef[d] * terms[d]
 * with terms[0] the stored feature, terms[d] its d-th derivative per step and coef[d] = k^d / d! for a forecast
 * k steps after the features were stored (sparse_taylor_coefficients writes these weights; estimating the
 * derivatives is the caller's business).  bf16 terms, fp32 sum in term order, one rounding to bf16 (nearest
 * even).  n_terms is 1..4; n_terms = 1 with coef[0] = 1 is the bit-exact copy of sparse_attn_fwd.
 *
 * sparse_attn_fwd_forecast: Algorithm 1 with this OP_reuse in its cache branch.  All arguments as for
 * sparse_attn_fwd_stream, except
 *   O_terms  HOST array of n_terms DEVICE pointers, each bf16 [B,H,L,D], 16-byte aligned, none overlapping O
 *   coef     HOST array of n_terms finite weights
 * Only the blocks whose flag is set are read from the terms.
 *
 * sparse_op_reuse: the element-wise kernel on flat arrays of n_elems bf16 values (a positive multiple of 8).
 *   terms    HOST array of n_terms DEVICE pointers, 16-byte aligned; a term may be `out` itself (in place)
 *   out      DEVICE, 16-byte aligned, written everywhere
 * Typical use: Out = OP_reuse(B_c terms), then sparse_gemm_o(..., addend = Out, Out) adds the computed heads.
 *
 * Errors as for sparse_attn_fwd.  Neither call allocates beyond what sparse_attn_fwd does.
 */
int sparse_attn_fwd_forecast(const void* Q, const void* K, const void* V, const uint8_t* cache_flags,
                             const uint8_t* kv_mask, const void* const* O_terms, const float* coef, int n_terms, void* O,
                             int B, int H, int L, int D, int block_q, int block_k, void* hip_stream);
int sparse_op_reuse(const void* const* terms, const float* coef, int n_terms, void* out, unsigned long long n_elems,
                    void* hip_stream);
/* coef[d] = steps^d / d! for d = 0..order (host arrays; coef holds order + 1 floats). */
void sparse_taylor_coefficients(int order, float steps, float* coef);

/*
 * Refresh of the stored terms at an Update step.  Section 3.3 names what the forecast uses (the stored
 * feature and its derivatives) but not how they are obtained; the derivatives are estimated the way the forecasting method it cites
 * does, by backward finite differences over the Update interval:
 *     new[0] = fresh,   new[d] = (new[d-1] - old[d-1]) / interval  for 1 <= d <= n_valid,   new[d] = 0 beyond
 * with n_valid the number of terms that were valid before this call (0 at the first refresh; the caller then
 * raises it by one per refresh up to n_terms).  Differences are taken in fp32 between the stored bf16 values and
 * rounded once per term.
 *   fresh   device, bf16, n_elems values (the freshly computed feature, e.g. the attention output O or B_c)
 *   terms   HOST array of n_terms (1..4) DEVICE pointers, each n_elems bf16 values, updated in place; they must
 *           not overlap each other or fresh; all 16-byte aligned; n_elems a positive multiple of 8
 * Errors as for sparse_attn_fwd.  Allocates nothing.
 */
int sparse_taylor_update(const void* fresh, void* const* terms, int n_terms, int n_valid, float interval,
                         unsigned long long n_elems, void* hip_stream);

/*
 * Sparse-symbol generation of an Update step (Section 3.3 "Logical Masks Generation", Equation 1; the
 * tau_kv and S_q rules of the settings table in the appendix).  From the step's Q and K it writes the
 * two symbol arrays that the attention calls, sparse_gemm_q and sparse_gemm_o read at the following steps.
 * Per (batch, head), with symbol granularity n: pooled query blocks of n * block_q tokens, T_q = ceil(L / (n block_q))
 * of them, and pooled key blocks of n * block_k tokens, T_k = ceil(L / (n block_k)) (a short last block is pooled
 * over the tokens that exist); the first ceil(text_tokens / (n block_q)) query blocks and ceil(text_tokens /
 * (n block_k)) key blocks are text (a pooled block that holds any text token is a text block):
 *   1. q~, k~ = per-block means of the query / key rows; P~ = row softmax of q~ k~^T / sqrt(D), [T_q, T_k]
 *   2. C_u = sum over text rows of P~[row, vision key block u], carried over to the vision query blocks by token
 *      overlap when n block_q != n block_k (C_v = sum_u C_u * |v and u| / |u|); G_v = sum over text columns j of
 *      softmax over v of P~[vision query block v, j]
 *   3. vision query block v is cached iff the ascending cumulative sums (ties by index) of C and of G at v are
 *      both <= tau_c times the totals; text blocks are never cached; if afterwards the share of the
 *      head's blocks that still need computation is below s_q, all T_q blocks are cached
 *   4. in row i of P~ key block j is skipped iff the ascending cumulative sum at j is <= tau_kv
 * All arithmetic is fp32; a decision whose deciding sum lies within rounding of its threshold may
 * differ from an exact evaluation.
 *   Q, K         device, bf16 [B, H, L, D], 16-byte aligned (read once each)
 *   cache_flags  device, uint8 [B, H, T_q], written: 1 = cached
 *   kv_mask      device, uint8 [B, H, T_q, ceil(T_k / 8)], written: bit = 1 keeps the pair, first block in
 *                bit 7 of byte 0, padding bits 0
 *   text_tokens  number of leading text tokens, 0 < text_tokens < L, with at least one vision block left on both axes
 *   tau_c, tau_kv, s_q  in [0, 1]
 * The arrays are exactly what sparse_attn_plan_create(..., block_q, block_k, granularity) reads; with granularity 1
 * they are what sparse_attn_fwd reads.  sparse_symbols_update / _stream are the case block_q = block_k = block,
 * granularity 1.
 * Supported: D, block_q, block_k in {64, 128}, granularity 1..64, T_q and T_k <= 2048.
 * Uses the library's per-stream scratch buffer (grown with hipMalloc on first use).  Errors as for
 * sparse_attn_fwd.
 */
int sparse_symbols_update(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H, int L,
                          int D, int block, int text_tokens, float tau_c, float tau_kv, float s_q);
int sparse_symbols_update_stream(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H,
                                 int L, int D, int block, int text_tokens, float tau_c, float tau_kv, float s_q,
                                 void* hip_stream);
int sparse_symbols_update_granular(const void* Q, const void* K, uint8_t* cache_flags, uint8_t* kv_mask, int B, int H,
                                   int L, int D, int block_q, int block_k, int granularity, int text_tokens,
                                   float tau_c, float tau_kv, float s_q, void* hip_stream);

/*
 * Live kernel timing for benchmarks.  Between sparse_attn_profile_begin(max_calls) and
 * sparse_attn_profile_end(), each of the first max_calls calls of sparse_attn_fwd /
 * sparse_attn_fwd_stream records three HIP events on its own stream (start, after the symbol
 * pre-pass, end) and does not synchronise.  sparse_attn_profile_end() waits for the recorded
 * calls and returns their number and the summed durations in milliseconds of the pre-pass and
 * of the attention kernel (host pointers, each may be NULL).  One profile at a time per process.
 */
int sparse_attn_profile_begin(int max_calls);
int sparse_attn_profile_end(int* calls, double* plan_ms_total, double* attn_ms_total);

/*
 * Scratch memory of the one-shot calls.  sparse_attn_fwd, sparse_attn_fwd_stream, sparse_attn_fwd_timed,
 * sparse_attn_fwd_forecast and sparse_symbols_update* keep one device buffer per (device, stream) inside the
 * library: allocated on the first call on that stream (hipMalloc), grown when a later call needs more (stream
 * synchronisation + hipFree + hipMalloc), shared by all of these calls on the stream, never shrunk.  Consequences:
 * such a call can be captured into a HIP graph only after a call of at least the same size has run on that stream,
 * and a graph captured from it becomes invalid if the buffer grows afterwards; the plan calls, sparse_attn_fwd_noalloc
 * and sparse_attn_fwd_workspace have no such restriction.  sparse_attn_release_scratch waits for the stream and frees
 * its buffer (call it before destroying a stream: the library cannot see that a stream handle has died, and a
 * recycled handle would inherit the old buffer, which is harmless but keeps memory).
 *
 * sparse_attn_workspace_bytes: bytes of scratch one attention call of this shape uses (0 for invalid shapes).
 * sparse_attn_fwd_workspace: sparse_attn_fwd_stream with that scratch supplied by the caller -- `workspace` is
 * device memory, 256-byte aligned, of at least sparse_attn_workspace_bytes(...) bytes, used only while the call's
 * work runs; the call allocates nothing.  Two calls that overlap in time must not share a workspace.
 */
size_t sparse_attn_workspace_bytes(int B, int H, int L, int block_q, int block_k);
int sparse_attn_fwd_workspace(const void* Q, const void* K, const void* V,
                              const uint8_t* cache_flags, const uint8_t* kv_mask,
                              const void* O_cache, void* O,
                              int B, int H, int L, int D, int block_q, int block_k,
                              void* workspace, size_t workspace_size, void* hip_stream);
int sparse_attn_release_scratch(void* hip_stream);

/*
 * Pair accounting of Section 4.1 (Sparsity = skip / total over (Q_i K_j^T, P_ij V_j) pairs).
 * cache_flags and kv_mask are HOST copies (either may be NULL, meaning as above).
 * kept_pairs (host) receives the number of pairs that are computed, i.e. set mask bits of
 * non-cached rows; total_pairs (host, may be NULL) receives B*H*Tq*Tkv.  Pure host code.
 */
int sparse_attn_count_kept(const uint8_t* cache_flags, const uint8_t* kv_mask,
                           int B, int H, int L, int block_q, int block_k,
                           unsigned long long* kept_pairs, unsigned long long* total_pairs);

/*
 * Symbol compression of Section 3.3 for the kv_mask argument.  logical (host): rows x Tkv
 * bytes, each 0 or non-zero; packed (host): rows x ceil(Tkv/8) bytes, written.  Pure host code.
 */
int sparse_attn_pack_mask(const uint8_t* logical, long long rows, int Tkv, uint8_t* packed);

/* Message for the last non-zero return on the calling thread ("" if none). Never NULL. */
const char* sparse_attn_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int sparse_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_ATTN_H */
