// Shared host-side declarations of the restoration library (internal).
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>

#include "cacheflow.h"

namespace cf {

// Thread-local message for cf_last_error().
void set_error(const char* fmt, ...);
int fail(int status, const char* fmt, ...);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_bytes(int dtype) { return dtype == CF_F32 ? 4 : 2; }
inline size_t page_bytes(int n_kv_heads, int head_dim, int dtype) {
    return (size_t)2 * n_kv_heads * CF_PAGE_TOKENS * head_dim * elem_bytes(dtype);
}

}  // namespace cf

// Host page-table object behind the opaque cf_cache handle.
struct cf_cache {
    void* pool = nullptr;
    size_t pool_bytes = 0;
    int n_layers = 0, n_kv_heads = 0, head_dim = 0, dtype = 0;
    int n_pages = 0, n_free = 0;
    size_t page_bytes = 0;
    struct Impl;
    Impl* impl = nullptr;
    // internal lookups used by the executor
    bool has(uint64_t req_id) const;
    const int32_t* table_of(uint64_t req_id, int* n_pages_out) const;  // may be null if empty
};
