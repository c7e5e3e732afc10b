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

#endif
