// Paged KV-cache bookkeeping: lowest-numbered-free-page-first allocator and
// per-request page tables (the paged cache the method restores into, Sec. 4.1).
#include <algorithm>
#include <unordered_map>
#include <vector>

#include "cf_common.h"

struct cf_cache::Impl {
    // bit i of word w set <=> page 64*w+i is free
    std::vector<uint64_t> free_bits;
    std::unordered_map<uint64_t, std::vector<int32_t>> tables;
    int first_maybe_free = 0;  // no free page has a word index below this
};

bool cf_cache::has(uint64_t req_id) const { return impl->tables.count(req_id) != 0; }

const int32_t* cf_cache::table_of(uint64_t req_id, int* n_pages_out) const {
    auto it = impl->tables.find(req_id);
    if (n_pages_out) *n_pages_out = 0;
    if (it == impl->tables.end()) return nullptr;
    if (n_pages_out) *n_pages_out = (int)it->second.size();
    return it->second.data();
}

extern "C" int cf_cache_create(void* pool, size_t pool_bytes, int32_t n_layers, int32_t n_kv_heads,
                               int32_t head_dim, int32_t dtype, cf_cache** out) {
    if (!out || n_layers <= 0 || n_kv_heads <= 0 || head_dim <= 0 ||
        (dtype != CF_F32 && dtype != CF_BF16))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_cache_create: bad shape or null out");
    size_t pb = cf::page_bytes(n_kv_heads, head_dim, dtype);
    size_t n_pages = pool_bytes / ((size_t)n_layers * pb);
    if (n_pages > (size_t)INT32_MAX / CF_PAGE_TOKENS)
        return cf::fail(CF_ERR_INVALID_ARG, "cf_cache_create: pool has too many pages");
    cf_cache* c = new cf_cache;
    c->pool = pool;
    c->pool_bytes = pool_bytes;
    c->n_layers = n_layers;
    c->n_kv_heads = n_kv_heads;
    c->head_dim = head_dim;
    c->dtype = dtype;
    c->page_bytes = pb;
    c->n_pages = c->n_free = (int)n_pages;
    c->impl = new cf_cache::Impl;
    c->impl->free_bits.assign((n_pages + 63) / 64, 0);
    for (size_t p = 0; p < n_pages; ++p) c->impl->free_bits[p >> 6] |= 1ull << (p & 63);
    *out = c;
    return CF_OK;
}

extern "C" void cf_cache_destroy(cf_cache* cache) {
    if (!cache) return;
    delete cache->impl;
    delete cache;
}

extern "C" int cf_cache_n_pages(const cf_cache* cache) { return cache ? cache->n_pages : 0; }
extern "C" int cf_cache_n_free(const cf_cache* cache) { return cache ? cache->n_free : 0; }
extern "C" size_t cf_cache_page_bytes(const cf_cache* cache) { return cache ? cache->page_bytes : 0; }

extern "C" int cf_cache_alloc(cf_cache* cache, uint64_t req_id, int32_t n_tokens) {
    if (!cache || n_tokens < 0) return cf::fail(CF_ERR_INVALID_ARG, "cf_cache_alloc: bad argument");
    auto& im = *cache->impl;
    if (im.tables.count(req_id))
        return cf::fail(CF_ERR_UNKNOWN_REQUEST, "cf_cache_alloc: request %llu already has pages",
                        (unsigned long long)req_id);
    int need = (int)cf::ceil_div(n_tokens, CF_PAGE_TOKENS);
    if (need > cache->n_free)
        return cf::fail(CF_ERR_OUT_OF_PAGES, "cf_cache_alloc: need %d pages, %d free", need,
                        cache->n_free);
    std::vector<int32_t> got;
    got.reserve(need);
    // need <= n_free, so the scan ends before the bitmap does
    for (size_t w = im.first_maybe_free; (int)got.size() < need; ++w) {
        uint64_t bits = im.free_bits[w];
        while (bits && (int)got.size() < need) {
            int b = __builtin_ctzll(bits);
            bits &= bits - 1;
            got.push_back((int32_t)(w * 64 + b));
        }
        im.free_bits[w] = bits;
    }
    while (im.first_maybe_free < (int)im.free_bits.size() &&
           im.free_bits[im.first_maybe_free] == 0)
        ++im.first_maybe_free;
    cache->n_free -= need;
    im.tables.emplace(req_id, std::move(got));
    return CF_OK;
}

extern "C" int cf_cache_free(cf_cache* cache, uint64_t req_id) {
    if (!cache) return cf::fail(CF_ERR_INVALID_ARG, "cf_cache_free: null cache");
    auto& im = *cache->impl;
    auto it = im.tables.find(req_id);
    if (it == im.tables.end())
        return cf::fail(CF_ERR_UNKNOWN_REQUEST, "cf_cache_free: request %llu has no pages",
                        (unsigned long long)req_id);
    for (int32_t p : it->second) {
        im.free_bits[p >> 6] |= 1ull << (p & 63);
        im.first_maybe_free = std::min(im.first_maybe_free, p >> 6);
    }
    cache->n_free += (int)it->second.size();
    im.tables.erase(it);
    return CF_OK;
}

extern "C" int cf_cache_page_table(const cf_cache* cache, uint64_t req_id, int32_t* out,
                                   int32_t cap, int32_t* n_pages) {
    if (!cache || !n_pages || cap < 0 || (cap > 0 && !out))
        return cf::fail(CF_ERR_INVALID_ARG, "cf_cache_page_table: bad argument");
    int n = 0;
    const int32_t* t = cache->table_of(req_id, &n);
    if (!cache->has(req_id))
        return cf::fail(CF_ERR_UNKNOWN_REQUEST, "cf_cache_page_table: request %llu has no pages",
                        (unsigned long long)req_id);
    *n_pages = n;
    for (int i = 0; i < n && i < cap; ++i) out[i] = t[i];
    return CF_OK;
}

extern "C" size_t cf_host_kv_bytes(int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                                   int32_t dtype, int32_t n_ctx) {
    if (n_layers <= 0 || n_kv_heads <= 0 || head_dim <= 0 || n_ctx < 0) return 0;
    return (size_t)n_layers * (size_t)cf::ceil_div(n_ctx, CF_PAGE_TOKENS) *
           cf::page_bytes(n_kv_heads, head_dim, dtype);
}
