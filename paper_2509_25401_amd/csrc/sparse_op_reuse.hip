// OP_reuse as a stand-alone element-wise kernel (Section 3.4: "an elementwise kernel can be invoked to
// perform simple value-reuse computations"; Section 3.5: the cached bias B_c is transformed by OP_reuse
// before GEMM-O adds the computed heads to it):  out = sum over d of coef[d] * terms[d], the Taylor
// polynomial of a stored feature and its stored derivatives.  bf16 in, fp32 sum in term order, one
// rounding to bf16.  HBM-bound: (n_terms + 1) * 2 bytes per element; 16 bytes per lane and access.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sparse_attn.h"
#include "sparse_attn_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

constexpr int kMaxTerms = 4;

struct ReuseParams {
  const bf16x8* term[kMaxTerms];
  float coef[kMaxTerms];
  bf16x8* out;
  size_t n_vec;            // 16-byte vectors
};

template <int N>
__global__ void __launch_bounds__(256) op_reuse_kernel(const ReuseParams p) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < p.n_vec; t += stride) {
    bf16x8 v[N];
#pragma unroll
    for (int d = 0; d < N; ++d) v[d] = __builtin_nontemporal_load(p.term[d] + t);   // streamed once
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float acc = p.coef[0] * (float)v[0][e];
#pragma unroll
      for (int d = 1; d < N; ++d) acc = fmaf(p.coef[d], (float)v[d][e], acc);
      r[e] = (__bf16)acc;
    }
    __builtin_nontemporal_store(r, p.out + t);
  }
}

// Refresh of the stored terms at an Update step: new[0] = fresh, new[d] = (new[d-1] - old[d-1]) / interval for
// d <= n_valid, zero beyond; differences between the stored (bf16-rounded) values, fp32, one rounding per term.
struct UpdateParams {
  const bf16x8* fresh;
  bf16x8* term[kMaxTerms];
  size_t n_vec;
  float interval;
  int n_valid;
};

template <int N>
__global__ void __launch_bounds__(256) taylor_update_kernel(const UpdateParams p) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < p.n_vec; t += stride) {
    bf16x8 old_lower = p.term[0][t];          // old term d-1
    bf16x8 new_lower = p.fresh[t];            // new term d-1 as it is stored
    p.term[0][t] = new_lower;
#pragma unroll
    for (int d = 1; d < N; ++d) {
      const bf16x8 old_this = p.term[d][t];
      bf16x8 r;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        r[e] = d <= p.n_valid ? (__bf16)(((float)new_lower[e] - (float)old_lower[e]) / p.interval) : (__bf16)0.0f;
      p.term[d][t] = r;
      old_lower = old_this;
      new_lower = r;
    }
  }
}

}  // namespace

extern "C" {

int sparse_taylor_update(const void* fresh, void* const* terms, int n_terms, int n_valid, float interval,
                         unsigned long long n_elems, void* hip_stream) {
  if (n_terms < 1 || n_terms > kMaxTerms)
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "taylor_update: n_terms=%d must be between 1 and %d", n_terms, kMaxTerms);
  if (n_valid < 0 || n_valid > n_terms)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: n_valid=%d must be between 0 and n_terms=%d", n_valid, n_terms);
  if (!(interval > 0.f) || interval - interval != 0.f)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: interval must be finite and > 0");
  if (!fresh || !terms) return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: fresh and terms must not be NULL");
  if (n_elems == 0 || n_elems % 8)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: n_elems=%llu must be a positive multiple of 8", n_elems);
  if ((uintptr_t)fresh & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: fresh must be 16-byte aligned");
  const size_t bytes = (size_t)n_elems * 2;
  UpdateParams p;
  for (int d = 0; d < kMaxTerms; ++d) p.term[d] = nullptr;
  for (int d = 0; d < n_terms; ++d) {
    void* t = terms[d];
    if (!t) return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: terms[%d] must not be NULL", d);
    if ((uintptr_t)t & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: terms[%d] must be 16-byte aligned", d);
    const uintptr_t a = (uintptr_t)t, f = (uintptr_t)fresh;
    if (a < f + bytes && f < a + bytes) return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: terms[%d] overlaps fresh", d);
    for (int e = 0; e < d; ++e) {
      const uintptr_t b = (uintptr_t)terms[e];
      if (a < b + bytes && b < a + bytes)
        return sa_fail(SPARSE_ATTN_ERR_INVALID, "taylor_update: terms[%d] overlaps terms[%d]", d, e);
    }
    p.term[d] = (bf16x8*)t;
  }
  p.fresh = (const bf16x8*)fresh;
  p.n_vec = (size_t)(n_elems / 8);
  p.interval = interval;
  p.n_valid = n_valid;
  const size_t want = (p.n_vec + 255) / 256;
  const unsigned grid = (unsigned)(want < 8192 ? want : 8192);
  hipStream_t stream = (hipStream_t)hip_stream;
  switch (n_terms) {
    case 1: hipLaunchKernelGGL(taylor_update_kernel<1>, dim3(grid), dim3(256), 0, stream, p); break;
    case 2: hipLaunchKernelGGL(taylor_update_kernel<2>, dim3(grid), dim3(256), 0, stream, p); break;
    case 3: hipLaunchKernelGGL(taylor_update_kernel<3>, dim3(grid), dim3(256), 0, stream, p); break;
    default: hipLaunchKernelGGL(taylor_update_kernel<4>, dim3(grid), dim3(256), 0, stream, p); break;
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "taylor_update: launch failed: %s", hipGetErrorString(e));
  return 0;
}

int sparse_op_reuse(const void* const* terms, const float* coef, int n_terms, void* out, unsigned long long n_elems,
                    void* hip_stream) {
  if (n_terms < 1 || n_terms > kMaxTerms)
    return sa_fail(SPARSE_ATTN_ERR_UNSUPPORTED, "op_reuse: n_terms=%d must be between 1 and %d", n_terms, kMaxTerms);
  if (!terms || !coef || !out) return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: terms, coef and out must not be NULL");
  if (n_elems == 0 || n_elems % 8)
    return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: n_elems=%llu must be a positive multiple of 8", n_elems);
  if ((uintptr_t)out & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: out must be 16-byte aligned");
  const size_t bytes = (size_t)n_elems * 2;
  ReuseParams p;
  for (int d = 0; d < kMaxTerms; ++d) {
    p.term[d] = nullptr;
    p.coef[d] = 0.f;
  }
  for (int d = 0; d < n_terms; ++d) {
    const void* t = terms[d];
    if (!t) return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: terms[%d] must not be NULL", d);
    if ((uintptr_t)t & 15) return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: terms[%d] must be 16-byte aligned", d);
    const uintptr_t a = (uintptr_t)t, b = (uintptr_t)out;
    if (a != b && a < b + bytes && b < a + bytes)
      return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: terms[%d] must be out itself or must not overlap it", d);
    if (!(coef[d] == coef[d]) || coef[d] - coef[d] != 0.f)
      return sa_fail(SPARSE_ATTN_ERR_INVALID, "op_reuse: coef[%d] must be finite", d);
    p.term[d] = (const bf16x8*)t;
    p.coef[d] = coef[d];
  }
  p.out = (bf16x8*)out;
  p.n_vec = (size_t)(n_elems / 8);
  // enough workgroups for every CU to keep several loads in flight; a grid-stride loop covers the rest
  const size_t want = (p.n_vec + 255) / 256;
  const unsigned grid = (unsigned)(want < 8192 ? want : 8192);
  hipStream_t stream = (hipStream_t)hip_stream;
  switch (n_terms) {
    case 1: hipLaunchKernelGGL(op_reuse_kernel<1>, dim3(grid), dim3(256), 0, stream, p); break;
    case 2: hipLaunchKernelGGL(op_reuse_kernel<2>, dim3(grid), dim3(256), 0, stream, p); break;
    case 3: hipLaunchKernelGGL(op_reuse_kernel<3>, dim3(grid), dim3(256), 0, stream, p); break;
    default: hipLaunchKernelGGL(op_reuse_kernel<4>, dim3(grid), dim3(256), 0, stream, p); break;
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return sa_fail(SPARSE_ATTN_ERR_HIP, "op_reuse: launch failed: %s", hipGetErrorString(e));
  return 0;
}

void sparse_taylor_coefficients(int order, float steps, float* coef) {
  // k^d / d!, the weights of the Taylor polynomial `steps` away from the expansion point
  double c = 1.0;
  for (int d = 0; d <= order; ++d) {
    coef[d] = (float)c;
    c = c * (double)steps / (double)(d + 1);
  }
}

}  // extern "C"
