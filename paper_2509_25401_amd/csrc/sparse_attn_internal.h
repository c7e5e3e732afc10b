// Shared between the translation units of the library (not part of the public ABI).
#ifndef SPARSE_ATTN_INTERNAL_H
#define SPARSE_ATTN_INTERNAL_H

// Records a printf-style message for sparse_attn_last_error() on the calling thread and returns `code`.
int sa_fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#endif
