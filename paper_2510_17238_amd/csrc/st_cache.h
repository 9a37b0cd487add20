// Kernel-side view of one paged KV cache (internal).
#pragma once
#include "st_internal.h"

namespace st {

struct CacheView {
    uint16_t* k_pool;            // [n_pages][Hkv][D/8][16][8] bf16 bits
    uint16_t* v_pool;            // [n_pages][Hkv][D][16]
    const int32_t* page_table;   // [batch][max_pages]
    int32_t* appended_len;       // [batch]
    int32_t max_pages;
    int32_t n_pages;
    int32_t n_kv_heads;
    // 8-bit caches: the pools hold bytes ([n_pages][Hkv][D/16][16][16] and [n_pages][Hkv][D][16]) and every
    // (page, head, slot) has an fp32 power-of-two scale for its key row and one for its value row
    float* k_scale;
    float* v_scale;
};

st_status check_cache(const st_kv_cache& c, const char* who, const char* which, bool allow_fp8 = false);
CacheView cache_view(const st_kv_cache& c);
// One token per sequence into a (checked, bf16) cache at index len_after[b] - 1; the length becomes len_after[b].
st_status append_token_at(const st_kv_cache& c, const void* k_new, const void* v_new, const int32_t* len_after, int batch,
                          bool rotate, double theta_base, hipStream_t s);

}  // namespace st
