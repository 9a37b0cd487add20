// Paged append to the source / reasoning KV cache (Sec. 3.3 "Parallel KV caches";
// Alg. 1: arriving input sentences go to the source cache, decoded tokens to the
// reasoning cache).
//
// Pure data movement, HBM-bound.  One workgroup handles the slots of ONE page of ONE
// KV head that the append touches, and rewrites the rows from token-major
// [token][head][d] into the pool layouts the decode kernel reads with contiguous
// 16-byte loads:
//   K: [page][head][d / 8][slot][8]      V: [page][head][d][slot]
// The new length is written by a second, tiny kernel so that every workgroup of the
// first one sees the old length (a single new token per sequence takes one launch: see
// kv_append_token_kernel).
//
// ROPE = true is the fused form: k_new holds UNROTATED keys and each key is rotated on its way
// into the pool by its position id, which is its index in this cache (Sec. 3.2 numbers the tokens
// of a stream from 0, independently of the other stream, so a stored key never has to be rotated
// again).  One full read + write of K by a separate rotation kernel disappears.
#include <math.h>

#include "st_cache.h"

namespace st {

struct alignas(16) Piece {
    uint16_t v[8];
};

template <int D, bool ROPE>
__global__ __launch_bounds__(256) void kv_append_kernel(CacheView cache, const uint16_t* __restrict__ k_new,
                                                        const uint16_t* __restrict__ v_new,
                                                        const int32_t* __restrict__ n_new, int max_new,
                                                        int pages_per_seq_touched, RopeFreq freq) {
    constexpr int KCH = D / 8;
    __shared__ uint16_t s_v[kPage][D + 2];
    const int pi = blockIdx.x % pages_per_seq_touched;
    const int h = (blockIdx.x / pages_per_seq_touched) % cache.n_kv_heads;
    const int b = blockIdx.x / (pages_per_seq_touched * cache.n_kv_heads);
    const int capacity = cache.max_pages * kPage;
    const int start = min(max(cache.appended_len[b], 0), capacity);
    int n = n_new ? min(max(n_new[b], 0), max_new) : max_new;
    n = min(n, capacity - start);                       // tokens past the page table are dropped
    const int page = start / kPage + pi;
    const int lo = max(start, page * kPage), hi = min(start + n, (page + 1) * kPage);
    if (lo >= hi) return;
    const int id = cache.page_table[int64_t(b) * cache.max_pages + page];
    if (id < 0 || id >= cache.n_pages) return;          // never write outside the pool
    const int slot_lo = lo - page * kPage, cnt = hi - lo;
    const int64_t row0 = int64_t(b) * max_new + (lo - start);        // first source row in k_new / v_new
    const int64_t row_stride = int64_t(cache.n_kv_heads) * D;
    const int tid = threadIdx.x;

    if (ROPE) {
        // K: a thread takes the two 16-byte pieces d = 8 c .. + 7 and D/2 + 8 c .. + 7 of one token --
        // the two halves of eight rotation pairs
        for (int w = tid; w < (KCH / 2) * kPage; w += 256) {
            const int c8 = w / kPage, s = w % kPage;
            if (s >= cnt) continue;
            const uint16_t* src = k_new + (row0 + s) * row_stride + h * D + c8 * 8;
            const Piece lo_in = *reinterpret_cast<const Piece*>(src), hi_in = *reinterpret_cast<const Piece*>(src + D / 2);
            Piece lo_out, hi_out;
            const int pos = lo + s;                              // index in this cache == position id
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float cs, sn;
                rope_cos_sin(pos, freq.f[c8 * 8 + e], &cs, &sn);
                const float a = bf16_bits_to_f32(lo_in.v[e]), b2 = bf16_bits_to_f32(hi_in.v[e]);
                lo_out.v[e] = f32_to_bf16_bits(a * cs - b2 * sn);
                hi_out.v[e] = f32_to_bf16_bits(b2 * cs + a * sn);
            }
            uint16_t* dst = cache.k_pool + ((int64_t(id) * cache.n_kv_heads + h) * KCH + c8) * (kPage * 8) + (slot_lo + s) * 8;
            *reinterpret_cast<Piece*>(dst) = lo_out;
            *reinterpret_cast<Piece*>(dst + (KCH / 2) * (kPage * 8)) = hi_out;
        }
    } else
    // K: 16-byte pieces, consecutive threads -> consecutive slots of one d-chunk
    for (int w = tid; w < KCH * kPage; w += 256) {
        const int c8 = w / kPage, s = w % kPage;
        if (s < cnt) {
            const u32x4 val = *reinterpret_cast<const u32x4*>(k_new + (row0 + s) * row_stride + h * D + c8 * 8);
            uint16_t* dst = cache.k_pool + ((int64_t(id) * cache.n_kv_heads + h) * KCH + c8) * (kPage * 8) + (slot_lo + s) * 8;
            *reinterpret_cast<u32x4*>(dst) = val;
        }
    }
    // V: transpose through LDS
    for (int w = tid; w < kPage * D; w += 256) {
        const int s = w / D, d = w % D;
        if (s < cnt) s_v[s][d] = v_new[(row0 + s) * row_stride + h * D + d];
    }
    __syncthreads();
    uint16_t* vdst = cache.v_pool + (int64_t(id) * cache.n_kv_heads + h) * (D * kPage);
    if (cnt == kPage) {
        // whole page: every d row is 32 contiguous bytes
        for (int w = tid; w < D * 2; w += 256) {
            const int d = w >> 1, half = w & 1;
            u32x4 val;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                val[e] = uint32_t(s_v[half * 8 + 2 * e][d]) | (uint32_t(s_v[half * 8 + 2 * e + 1][d]) << 16);
            *reinterpret_cast<u32x4*>(vdst + d * kPage + half * 8) = val;
        }
    } else {
        for (int w = tid; w < D * kPage; w += 256) {
            const int d = w / kPage, s = w % kPage;
            if (s < cnt) vdst[d * kPage + slot_lo + s] = s_v[s][d];
        }
    }
}

// One new token per sequence (the decoding step): one workgroup per sequence, no staging, and -- nobody else reads
// this sequence's length -- the workgroup writes the new length itself, which saves the second launch per layer and
// token.  Threads split the token's Hkv x D / 8 pieces of K (rotated on the way in if ROPE) and of V.
template <int D, bool ROPE>
__global__ __launch_bounds__(256) void kv_append_token_kernel(CacheView cache, const uint16_t* __restrict__ k_new,
                                                              const uint16_t* __restrict__ v_new,
                                                              const int32_t* __restrict__ n_new,
                                                              const int32_t* __restrict__ len_after, RopeFreq freq) {
    constexpr int KCH = D / 8;
    const int b = blockIdx.x;
    const int capacity = cache.max_pages * kPage;
    // the token's index: the cache's own length, or -- len_after given -- the caller's length INCLUDING the token
    // minus one (a length of 0 there: nothing to store for this sequence)
    const int given = len_after ? min(max(len_after[b], 0), capacity) : 0;
    const int start = len_after ? max(given - 1, 0) : min(max(cache.appended_len[b], 0), capacity);
    int n = len_after ? (given > 0 ? 1 : 0) : (n_new ? min(max(n_new[b], 0), 1) : 1);
    n = min(n, capacity - start);
    __syncthreads();                                     // every thread has read the old length
    if (n == 0) return;
    const int id = cache.page_table[int64_t(b) * cache.max_pages + start / kPage];
    if (id >= 0 && id < cache.n_pages) {                 // never write outside the pool
        const int slot = start % kPage;
        const int pieces = cache.n_kv_heads * KCH;
        const uint16_t* krow = k_new + int64_t(b) * cache.n_kv_heads * D;
        const uint16_t* vrow = v_new + int64_t(b) * cache.n_kv_heads * D;
        for (int w = threadIdx.x; w < pieces; w += 256) {
            const int h = w / KCH, c8 = w % KCH;
            uint16_t* kdst = cache.k_pool + ((int64_t(id) * cache.n_kv_heads + h) * KCH + c8) * (kPage * 8) + slot * 8;
            if (ROPE) {
                // piece c8 < KCH / 2 and its partner c8 + KCH / 2: the two halves of eight rotation pairs
                if (c8 < KCH / 2) {
                    const Piece lo_in = *reinterpret_cast<const Piece*>(krow + h * D + c8 * 8);
                    const Piece hi_in = *reinterpret_cast<const Piece*>(krow + h * D + c8 * 8 + D / 2);
                    Piece lo_out, hi_out;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float cs, sn;
                        rope_cos_sin(start, freq.f[c8 * 8 + e], &cs, &sn);      // index in this cache == position id
                        const float a = bf16_bits_to_f32(lo_in.v[e]), b2 = bf16_bits_to_f32(hi_in.v[e]);
                        lo_out.v[e] = f32_to_bf16_bits(a * cs - b2 * sn);
                        hi_out.v[e] = f32_to_bf16_bits(b2 * cs + a * sn);
                    }
                    *reinterpret_cast<Piece*>(kdst) = lo_out;
                    *reinterpret_cast<Piece*>(kdst + (KCH / 2) * (kPage * 8)) = hi_out;
                }
            } else {
                *reinterpret_cast<Piece*>(kdst) = *reinterpret_cast<const Piece*>(krow + h * D + c8 * 8);
            }
            // V: the piece's 8 values go to 8 rows d of the page, slot `slot` each
            const Piece vin = *reinterpret_cast<const Piece*>(vrow + h * D + c8 * 8);
            uint16_t* vdst = cache.v_pool + (int64_t(id) * cache.n_kv_heads + h) * (D * kPage) + (c8 * 8) * kPage + slot;
#pragma unroll
            for (int e = 0; e < 8; ++e) vdst[e * kPage] = vin.v[e];
        }
    }
    if (threadIdx.x == 0) cache.appended_len[b] = start + n;
}

// 8-bit store: every key row and every value row (one token, one KV head) is divided by its own power of
// two 2^k -- k the smallest integer, not below kScaleExpMin, with max|row| 2^-k <= 448 -- and rounded to
// E4M3 (nearest, ties to even); 2^k goes to the scale arrays.  Same work split as above: one workgroup per
// (page touched, KV head, sequence); the 16 x D tile of each tensor passes through LDS.
constexpr int kScaleExpMin = -100;

__device__ __forceinline__ int row_scale_exponent(float amax) {
    if (!(amax > 0.f)) return 0;
    int ex;
    const float m = frexpf(amax, &ex);                  // amax = m 2^ex, m in [0.5, 1);  448 = 0.875 * 2^9
    return max(m <= 0.875f ? ex - 9 : ex - 8, kScaleExpMin);
}

template <int D>
__global__ __launch_bounds__(256) void kv_append_fp8_kernel(CacheView cache, const uint16_t* __restrict__ k_new,
                                                            const uint16_t* __restrict__ v_new,
                                                            const int32_t* __restrict__ n_new, int max_new,
                                                            int pages_per_seq_touched) {
    constexpr int C16 = D / 16, C8 = D / 8;
    __shared__ float s_x[2][kPage][D + 1];              // [0] keys, [1] values of the page's new tokens
    __shared__ int s_exp[2][kPage];
    const int pi = blockIdx.x % pages_per_seq_touched;
    const int h = (blockIdx.x / pages_per_seq_touched) % cache.n_kv_heads;
    const int b = blockIdx.x / (pages_per_seq_touched * cache.n_kv_heads);
    const int capacity = cache.max_pages * kPage;
    const int start = min(max(cache.appended_len[b], 0), capacity);
    int n = n_new ? min(max(n_new[b], 0), max_new) : max_new;
    n = min(n, capacity - start);
    const int page = start / kPage + pi;
    const int lo = max(start, page * kPage), hi = min(start + n, (page + 1) * kPage);
    if (lo >= hi) return;
    const int id = cache.page_table[int64_t(b) * cache.max_pages + page];
    if (id < 0 || id >= cache.n_pages) return;
    const int slot_lo = lo - page * kPage, cnt = hi - lo;
    const int64_t row0 = int64_t(b) * max_new + (lo - start);
    const int64_t row_stride = int64_t(cache.n_kv_heads) * D;
    const int tid = threadIdx.x;

    for (int w = tid; w < 2 * kPage * C8; w += 256) {
        const int which = w / (kPage * C8), s = (w / C8) % kPage, c = w % C8;
        if (s >= cnt) continue;
        const Piece in = *reinterpret_cast<const Piece*>((which ? v_new : k_new) + (row0 + s) * row_stride + h * D + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s_x[which][s][c * 8 + e] = bf16_bits_to_f32(in.v[e]);
    }
    __syncthreads();
    // 8 threads per row: largest magnitude, exponent, scale
    {
        const int row = tid >> 3, part = tid & 7;       // 32 rows: 16 key rows, then 16 value rows
        const int which = row >> 4, s = row & 15;
        float amax = 0.f;
        if (s < cnt)
            for (int d = part; d < D; d += 8) amax = fmaxf(amax, fabsf(s_x[which][s][d]));
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
        if (part == 0 && s < cnt) {
            const int k = row_scale_exponent(amax);
            s_exp[which][s] = k;
            (which ? cache.v_scale : cache.k_scale)[(int64_t(id) * cache.n_kv_heads + h) * kPage + slot_lo + s] = ldexpf(1.f, k);
        }
    }
    __syncthreads();
    uint8_t* kdst = reinterpret_cast<uint8_t*>(cache.k_pool) + (int64_t(id) * cache.n_kv_heads + h) * (C16 * kPage * 16);
    uint8_t* vdst = reinterpret_cast<uint8_t*>(cache.v_pool) + (int64_t(id) * cache.n_kv_heads + h) * (D * kPage);
    // K: 8 codes (8 bytes) per thread: d = 8 c .. 8 c + 7 of one token -> chunk c / 2, byte 8 (c % 2)
    for (int w = tid; w < kPage * C8; w += 256) {
        const int c = w / kPage, s = w % kPage;
        if (s >= cnt) continue;
        const int k = s_exp[0][s];
        uint32_t lo32 = 0, hi32 = 0;
        const float* x = &s_x[0][s][c * 8];
        lo32 = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[0], -k), ldexpf(x[1], -k), lo32, false);
        lo32 = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[2], -k), ldexpf(x[3], -k), lo32, true);
        hi32 = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[4], -k), ldexpf(x[5], -k), hi32, false);
        hi32 = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(x[6], -k), ldexpf(x[7], -k), hi32, true);
        *reinterpret_cast<u32x2*>(kdst + ((c >> 1) * kPage + slot_lo + s) * 16 + 8 * (c & 1)) = u32x2{lo32, hi32};
    }
    // V: one byte per (d, slot)
    for (int w = tid; w < D * kPage; w += 256) {
        const int d = w / kPage, s = w % kPage;
        if (s >= cnt) continue;
        const uint32_t code = __builtin_amdgcn_cvt_pk_fp8_f32(ldexpf(s_x[1][s][d], -s_exp[1][s]), 0.f, 0u, false);
        vdst[d * kPage + slot_lo + s] = uint8_t(code & 0xffu);
    }
}

__global__ void kv_append_bump_kernel(int32_t* __restrict__ appended_len, const int32_t* __restrict__ n_new,
                                      int max_new, int batch, int capacity) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int start = min(max(appended_len[b], 0), capacity);
    int n = n_new ? min(max(n_new[b], 0), max_new) : max_new;
    n = min(n, capacity - start);
    appended_len[b] = start + n;
}

st_status check_cache(const st_kv_cache& c, const char* who, const char* which, bool allow_fp8) {
    if (!c.k_pool || !c.v_pool || !c.page_table) return fail(ST_ERR_INVALID_ARG, "%s: %s cache has a null pointer", who, which);
    if (!aligned16(c.k_pool) || !aligned16(c.v_pool)) return fail(ST_ERR_INVALID_ARG, "%s: %s pools must be 16-byte aligned", who, which);
    if (c.page_size != kPage) return fail(ST_ERR_UNSUPPORTED, "%s: page_size %d (must be %d)", who, c.page_size, kPage);
    if (c.dtype == ST_FP8_E4M3) {
        if (!allow_fp8) return fail(ST_ERR_UNSUPPORTED, "%s: 8-bit caches are not supported by this call", who);
        if (!c.k_scale || !c.v_scale) return fail(ST_ERR_INVALID_ARG, "%s: %s cache is ST_FP8_E4M3 but has no scale arrays", who, which);
        if (!aligned16(c.k_scale) || !aligned16(c.v_scale)) return fail(ST_ERR_INVALID_ARG, "%s: %s scale arrays must be 16-byte aligned", who, which);
    } else if (c.dtype != ST_BF16) {
        return fail(ST_ERR_UNSUPPORTED, "%s: cache dtype %d (ST_BF16 or ST_FP8_E4M3)", who, c.dtype);
    }
    if (c.head_dim != 64 && c.head_dim != 128) return fail(ST_ERR_UNSUPPORTED, "%s: head_dim %d (64 or 128)", who, c.head_dim);
    if (c.n_kv_heads <= 0 || c.max_pages_per_seq <= 0 || c.n_pages <= 0) return fail(ST_ERR_INVALID_ARG, "%s: %s cache has non-positive sizes", who, which);
    return ST_OK;
}

CacheView cache_view(const st_kv_cache& c) {
    CacheView v;
    v.k_pool = static_cast<uint16_t*>(c.k_pool);
    v.v_pool = static_cast<uint16_t*>(c.v_pool);
    v.page_table = c.page_table;
    v.appended_len = c.appended_len;
    v.max_pages = c.max_pages_per_seq;
    v.n_pages = c.n_pages;
    v.n_kv_heads = c.n_kv_heads;
    v.k_scale = c.dtype == ST_FP8_E4M3 ? c.k_scale : nullptr;
    v.v_scale = c.dtype == ST_FP8_E4M3 ? c.v_scale : nullptr;
    return v;
}

st_status append_token_at(const st_kv_cache& c, const void* k_new, const void* v_new, const int32_t* len_after, int batch,
                          bool rotate, double theta_base, hipStream_t s) {
    const CacheView cv = cache_view(c);
    const RopeFreq freq = rotate ? make_rope_freq(theta_base, c.head_dim) : RopeFreq{};
    auto token = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)batch), dim3(256), 0, s, cv, (const uint16_t*)k_new, (const uint16_t*)v_new,
                           (const int32_t*)nullptr, len_after, freq);
    };
    if (c.head_dim == 64) {
        if (rotate) token(kv_append_token_kernel<64, true>); else token(kv_append_token_kernel<64, false>);
    } else {
        if (rotate) token(kv_append_token_kernel<128, true>); else token(kv_append_token_kernel<128, false>);
    }
    ST_LAUNCH_CHECK("kv_append_token_kernel");
    return ST_OK;
}

}  // namespace st

using namespace st;

static st_status kv_append_impl(const char* who, const st_dual_cache* caches, st_stream_kind which, const void* k_new,
                                const void* v_new, const int32_t* n_new, int32_t max_new, int32_t batch,
                                int32_t host_len_upper_bound, bool rotate, double theta_base, void* hip_stream) {
    if (!caches || !k_new || !v_new) return fail(ST_ERR_INVALID_ARG, "%s: null pointer", who);
    if (which != ST_SOURCE && which != ST_REASONING) return fail(ST_ERR_INVALID_ARG, "%s: which = %d", who, int(which));
    const st_kv_cache& c = which == ST_SOURCE ? caches->source : caches->reasoning;
    st_status r = check_cache(c, who, which == ST_SOURCE ? "source" : "reasoning", !rotate);
    if (r != ST_OK) return r;
    const bool fp8 = c.dtype == ST_FP8_E4M3;
    if (!c.appended_len) return fail(ST_ERR_INVALID_ARG, "%s: appended_len is null", who);
    if (!aligned16(k_new) || !aligned16(v_new)) return fail(ST_ERR_INVALID_ARG, "%s: k_new / v_new must be 16-byte aligned", who);
    if (batch <= 0 || max_new < 0) return fail(ST_ERR_INVALID_ARG, "%s: bad sizes", who);
    const int64_t capacity = int64_t(c.max_pages_per_seq) * kPage;
    if (host_len_upper_bound < 0 || host_len_upper_bound > capacity)
        return fail(ST_ERR_CAPACITY, "%s: length bound %d exceeds the page table (%lld tokens per sequence)", who,
                    host_len_upper_bound, (long long)capacity);
    if (rotate && !(theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "%s: theta_base must be positive", who);
    if (max_new == 0) return ST_OK;
    const int touched = (max_new + kPage - 1) / kPage + 1;
    const int64_t blocks = int64_t(batch) * c.n_kv_heads * touched;
    if (blocks > 0x7fffffff) return fail(ST_ERR_SHAPE, "%s: grid too large", who);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const CacheView cv = cache_view(c);
    const RopeFreq freq = rotate ? make_rope_freq(theta_base, c.head_dim) : RopeFreq{};
    if (max_new == 1 && !fp8) {
        // the decoding step: one launch, the workgroup of a sequence writes its new length itself
        auto token = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, dim3((unsigned)batch), dim3(256), 0, s, cv, (const uint16_t*)k_new, (const uint16_t*)v_new, n_new,
                               (const int32_t*)nullptr, freq);
        };
        if (c.head_dim == 64) {
            if (rotate) token(kv_append_token_kernel<64, true>); else token(kv_append_token_kernel<64, false>);
        } else {
            if (rotate) token(kv_append_token_kernel<128, true>); else token(kv_append_token_kernel<128, false>);
        }
        ST_LAUNCH_CHECK("kv_append_token_kernel");
        return ST_OK;
    }
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(256), 0, s, cv, (const uint16_t*)k_new, (const uint16_t*)v_new,
                           n_new, max_new, touched, freq);
    };
    if (fp8) {
        if (c.head_dim == 64)
            hipLaunchKernelGGL((kv_append_fp8_kernel<64>), dim3((unsigned)blocks), dim3(256), 0, s, cv, (const uint16_t*)k_new,
                               (const uint16_t*)v_new, n_new, max_new, touched);
        else
            hipLaunchKernelGGL((kv_append_fp8_kernel<128>), dim3((unsigned)blocks), dim3(256), 0, s, cv, (const uint16_t*)k_new,
                               (const uint16_t*)v_new, n_new, max_new, touched);
    } else if (c.head_dim == 64) {
        if (rotate) launch(kv_append_kernel<64, true>); else launch(kv_append_kernel<64, false>);
    } else {
        if (rotate) launch(kv_append_kernel<128, true>); else launch(kv_append_kernel<128, false>);
    }
    ST_LAUNCH_CHECK("kv_append_kernel");
    hipLaunchKernelGGL(kv_append_bump_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, c.appended_len, n_new, max_new,
                       batch, int(capacity));
    ST_LAUNCH_CHECK("kv_append_bump_kernel");
    return ST_OK;
}

extern "C" st_status st_kv_append(const st_dual_cache* caches, st_stream_kind which, const void* k_new,
                                  const void* v_new, const int32_t* n_new, int32_t max_new, int32_t batch,
                                  int32_t host_len_upper_bound, void* hip_stream) {
    return kv_append_impl("st_kv_append", caches, which, k_new, v_new, n_new, max_new, batch, host_len_upper_bound, false, 0.0,
                          hip_stream);
}

extern "C" st_status st_kv_append_rope(const st_dual_cache* caches, st_stream_kind which, const void* k_new,
                                       const void* v_new, const int32_t* n_new, int32_t max_new, int32_t batch,
                                       int32_t host_len_upper_bound, double theta_base, void* hip_stream) {
    return kv_append_impl("st_kv_append_rope", caches, which, k_new, v_new, n_new, max_new, batch, host_len_upper_bound, true,
                          theta_base, hip_stream);
}
