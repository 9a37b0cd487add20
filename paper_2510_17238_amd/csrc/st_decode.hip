// Dual-cache decode (Sec. 3.3 "Parallel KV caches"; Alg. 1: merge the visible source
// slice with the reasoning cache, then decode).
//
// Nothing is merged in memory.  The two caches are cut into work units of 128 to 1,024 tokens
// (decode_unit_tokens; 512 for the 32-row kernel); one WAVE takes one (sequence, KV head, unit),
// streams that unit's K and V pages from HBM exactly once for all query heads of the group, and
// emits an un-normalised partial (o, m, l).  A second kernel merges all partials of BOTH caches per (sequence, query
// row, head) by log-sum-exp -- identical to a softmax over the concatenated cache.
//
// HBM-bound: 4 * D bytes per cached token and KV head, 2 * G * D useful flops for it.
// The arithmetic rides on the matrix cores only to keep the vector ALUs out of the
// way: S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, where the 32
// columns are the (up to 32) query rows q_len * G.  The pool layouts make every operand
// a contiguous 16-byte load straight from global memory into MFMA registers:
//   K [page][head][d/8][slot][8] : lane (m, hg) reads slot m of d-chunk 2 j + hg
//   V [page][head][d][slot]      : lane (n, hg) reads slots 8 hg .. 8 hg + 7 of row d
#include <type_traits>

#include "st_cache.h"
#include <mutex>

#include "st_tiles.h"

namespace st {

constexpr int kChunk = 512;                 // tokens per work unit
constexpr int kSmallDecodeTokens = 1024;    // both caches together: below this one wave per (sequence, KV head) finishes the rows itself
constexpr int kChunkMin = 128;              // ... of the one-token decode step of a few sequences
constexpr int kChunkLong = 1024;            // ... of the one-token decode step when there is plenty of work (64 pages: one id per lane)

// 16 bytes of a pool that this launch reads once and never again, taken in whole 128-byte lines per instruction: the
// load carries the non-temporal hint.  Value loads always do (measured on the decode step of 28 layers: 3 to 4 %
// faster).  Key loads do in launches of up to about 2 GB (STREAM_KEYS; 1 to 2.5 % faster on 0.7 GB per launch,
// 2 to 4 % slower on 3.8 GB per launch, A/B on one box each time).
template <typename T>
__device__ __forceinline__ u32x4 stream_load(const T* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
template <bool STREAM, typename T>
__device__ __forceinline__ u32x4 key_load(const T* p) {
    if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return *reinterpret_cast<const u32x4*>(p);
}

struct DecodeArgs {
    CacheView src, rsn;
    const int32_t* src_len;
    const int32_t* rsn_len;
    const uint16_t* q;
    float* part_o;     // [B][Hkv][nc][rows][D]
    float* part_ml;    // [B][Hkv][nc][rows][2]
    int batch, q_len, n_q_heads, n_kv_heads, group, rows;
    int ncs, ncr;      // chunk slots per (sequence, head) for the two caches
    int chunk;         // tokens per work unit (kChunk; kChunkMin .. kChunkLong for the one-wave decode kernels)
    float scale_log2;
    // source-chunk prefill only: ragged query counts and 32-row blocks
    const int32_t* n_new;   // [B] query tokens per sequence, or null for max_new everywhere
    int max_new;            // token stride of q / out
    int row_blocks;         // ceil(max_new * group / 32)
    // fused query rotation: q holds unrotated queries; row t is the token at index len - q_len + t of its own
    // stream (reasoning for a decode step, source for a source chunk), which is its position id
    int rope;
    RopeFreq freq;
    // one decoding step in one call (bf16, q_len = 1, <= 16 rows): the token k_new / v_new [batch][Hkv][D] is the one at
    // index rsn_len[b] - 1 of the reasoning stream and is NOT in the cache yet -- the launch stores it, attends over
    // the cached tokens before it, and takes the token itself from registers as one more partial state
    int append;
    const uint16_t* k_new;
    const uint16_t* v_new;
    // wave timeline (st_profile_wave_trace): (start, end) wall-clock pairs per workgroup, or null
    unsigned long long* trace;
    int trace_cap;
};

// Stamps the workgroup's start and end into the timeline buffer, whichever way the kernel is left.
struct WaveStamp {
    unsigned long long* slot;
    unsigned long long t0;
    __device__ __forceinline__ WaveStamp(const DecodeArgs& a) : slot(nullptr), t0(0) {
        if (a.trace && int(blockIdx.x) < a.trace_cap) {
            slot = a.trace + 2 * size_t(blockIdx.x);
            t0 = wall_clock64();
        }
    }
    __device__ __forceinline__ ~WaveStamp() {
        if (slot && threadIdx.x == 0) {
            slot[0] = t0;
            slot[1] = wall_clock64();
        }
    }
};

// Fused query rotation (Sec. 3.2, stream-local position ids): fragments j and j + KS/2 of a lane hold the
// two halves of eight rotation pairs, head dims STRIDE j + off + e and D/2 + the same.
template <int KS, int STRIDE>
__device__ __forceinline__ void rotate_query(bf16x8 (&qf)[KS], int off, int pos, const RopeFreq& fr) {
#pragma unroll
    for (int j = 0; j < KS / 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float cs, sn;
            rope_cos_sin(pos, fr.f[STRIDE * j + off + e], &cs, &sn);
            const float x = float(qf[j][e]), y = float(qf[j + KS / 2][e]);
            qf[j][e] = (__bf16)(x * cs - y * sn);
            qf[j + KS / 2][e] = (__bf16)(y * cs + x * sn);
        }
}

// The decode step with 17 .. 32 query rows q_len * G per sequence and KV head, both caches: four waves per
// workgroup, each with a unit of its own.
template <int D>
__global__ __launch_bounds__(256) void decode_split_kernel(DecodeArgs a) {
    constexpr int KS = D / 16, DB = D / 32, KCH = D / 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nc = a.ncs + a.ncr;
    int64_t unit = int64_t(blockIdx.x) * 4 + wave;
    const int c = int(unit % nc);
    unit /= nc;
    const int h = int(unit % a.n_kv_heads);
    const int b = int(unit / a.n_kv_heads);
    if (b >= a.batch) return;
    const bool is_src = c < a.ncs;
    const CacheView& cv = is_src ? a.src : a.rsn;
    const int cc = is_src ? c : c - a.ncs;
    const int len = min(max(is_src ? a.src_len[b] : a.rsn_len[b], 0), cv.max_pages * kPage);
    const int tok0 = cc * kChunk;
    if (tok0 >= len) return;

    const int n = lane & 31, hg = lane >> 5;
    const int q_len = a.q_len;
    const int r = n;                                // query row of this (sequence, KV head): token r / G, head r % G
    const int t_row = r / a.group;
    const bool valid_row = r < q_len * a.group;
    const int hq = h * a.group + r % a.group;
    const int tok_end = min(len, tok0 + kChunk);
    // visible reasoning tokens of query row t: [0, len - q_len + t]; the source slice is seen whole
    const int limit = !valid_row ? 0 : (is_src ? len : max(len - q_len + t_row + 1, 0));

    bf16x8 qf[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) {
        u32x4 z = {0u, 0u, 0u, 0u};
        if (valid_row)
            z = *reinterpret_cast<const u32x4*>(a.q + ((int64_t(b) * a.q_len + t_row) * a.n_q_heads + hq) * D + 16 * j + 8 * hg);
        qf[j] = __builtin_bit_cast(bf16x8, z);
    }
    if (a.rope) {
        // the row's position id: its index in the reasoning stream
        const int len_own = min(max(a.rsn_len[b], 0), a.rsn.max_pages * kPage);
        rotate_query<KS, 16>(qf, 8 * hg, max(len_own - q_len + t_row, 0), a.freq);
    }
    f32x16 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int32_t* table = cv.page_table + int64_t(b) * cv.max_pages;
    const int64_t head_k = int64_t(h) * KCH * (kPage * 8);
    const int64_t page_k = int64_t(cv.n_kv_heads) * KCH * (kPage * 8);
    const int64_t head_v = int64_t(h) * D * kPage;
    const int64_t page_v = int64_t(cv.n_kv_heads) * D * kPage;
    const int k_slot = swap23(n & 15);

    for (int tok = tok0; tok < tok_end; tok += 32) {
        // ---- K operand: lane (m = n, hg) -> page tok/16 + m/16, slot swap23(m % 16) ----
        const int pg_k = tok / kPage + (n >> 4);
        int id_k = -1;
        if (pg_k * kPage < tok_end) id_k = table[pg_k];
        const bool ok_k = id_k >= 0 && id_k < cv.n_pages;
        f32x16 s_acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) s_acc[i] = 0.f;
        {
            const uint16_t* kp = cv.k_pool + int64_t(ok_k ? id_k : 0) * page_k + head_k + k_slot * 8;
            bf16x8 ak[KS];
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                u32x4 z = {0u, 0u, 0u, 0u};
                if (ok_k) z = *reinterpret_cast<const u32x4*>(kp + (2 * j + hg) * (kPage * 8));
                ak[j] = __builtin_bit_cast(bf16x8, z);
            }
#pragma unroll
            for (int j = 0; j < KS; ++j) s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[j], qf[j], s_acc, 0, 0, 0);
        }
        // ---- V operand: page t, lane (d = 32 db + n, hg) -> slots 8 hg .. 8 hg + 7 ----
        bf16x8 av[2][DB];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int pg_v = tok / kPage + t;
            int id_v = -1;
            if (pg_v * kPage < tok_end) id_v = table[pg_v];
            const bool ok_v = id_v >= 0 && id_v < cv.n_pages;
            const uint16_t* vp = cv.v_pool + int64_t(ok_v ? id_v : 0) * page_v + head_v + n * kPage + 8 * hg;
            const int first = tok + 16 * t + 8 * hg;     // token held in element 0
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                u32x4 z = {0u, 0u, 0u, 0u};
                if (ok_v) z = *reinterpret_cast<const u32x4*>(vp + db * 32 * kPage);
                if (first + 8 > len) {
                    // slots past the visible length may hold anything: select them away
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t keep_lo = first + 2 * e < len ? 0x0000ffffu : 0u;
                        const uint32_t keep_hi = first + 2 * e + 1 < len ? 0xffff0000u : 0u;
                        z[e] &= keep_lo | keep_hi;
                    }
                }
                av[t][db] = __builtin_bit_cast(bf16x8, z);
            }
        }
        // ---- mask + online softmax; register i <-> token tok + 16 (i/8) + 8 hg + i%8 ----
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int kv = tok + 16 * (i >> 3) + 8 * hg + (i & 7);
            s_acc[i] = kv < limit ? s_acc[i] : -INFINITY;
            mx = fmaxf(mx, s_acc[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * a.scale_log2);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pb[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[i], a.scale_log2, -m_use));
            psum += p;
            pb[i >> 3][i & 7] = (__bf16)p;
        }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
#pragma unroll
            for (int t = 0; t < 2; ++t)
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[t][db], pb[t], o_acc[db], 0, 0, 0);
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!valid_row) return;
    const int64_t slot = ((int64_t(b) * a.n_kv_heads + h) * nc + c) * a.rows + n;
    float* po = a.part_o + slot * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = o_acc[db][4 * q4 + e];
            *reinterpret_cast<f32x4*>(po + 32 * db + 8 * q4 + 4 * hg) = o4;
        }
    if (hg == 0) {
        a.part_ml[slot * 2] = m_run;
        a.part_ml[slot * 2 + 1] = l_tot;
    }
}

// Variant for q_len * G <= 16 query rows (the one-token decode step): the same scheme on
// v_mfma_f32_16x16x32_bf16, ONE WAVE PER WORKGROUP.  With a single wave everything that selects
// the work unit is uniform (scalar registers, scalar branches), a finished unit frees its slot
// at once, and at <= 128 VGPRs sixteen such waves share a CU, each with 16 KB of loads in flight.
//
// A wave takes 32 tokens (two pages) per step with two first-product MFMAs X and Y whose 16 key
// rows are chosen so that afterwards quarter-wave g4 (lanes 16 g4 .. 16 g4 + 15) holds, for its
// query column, the 8 CONSECUTIVE slots 8 (g4 % 2) .. + 7 of page g4 / 2: X gives slots +0..3,
// Y gives slots +4..7.  Those 8 probabilities are exactly one B operand of the second product,
// whose A operand (V^T) is then one contiguous 16-byte load.  All loads are unconditional (page
// ids are clamped into the pool); what lies beyond the visible length is removed afterwards by
// index: scores by select, V by bit mask.
// One unit (tokens [tok0, tok_end) of one cache) folded into the running state of a query column: the step loop of the
// one-wave kernels.  State in base-2 exponent units: m_ref is the column's reference exponent (the same in its four
// lanes); it starts at 0 with has_ref = false and is moved, out of line, only when a step brings an exponent more
// than kLazyRise above it (or the first finite score): the common step then needs no exchange between lanes and no
// rescale of the accumulator -- probabilities are bounded by 2^kLazyRise instead of 1, which fp32 and bf16 do not
// mind, and whoever finishes the row divides by l anyway.
template <int D, bool PREFETCH = false, bool STREAM_KEYS = false>
__device__ __forceinline__ void scan_unit16(const CacheView& cv, int b, int h, int lane, int tok0, int tok_end, int len, int limit,
                                            int limit_min, float scale_log2, const bf16x8 (&qf)[D / 32], f32x4 (&o_acc)[D / 16],
                                            float& m_ref, float& l_run, bool& has_ref) {
    constexpr int KS = D / 32, DB = D / 16, KCH = D / 8;
    constexpr float kLazyRise = 8.f;
    const int n = lane & 15, g4 = lane >> 4;
    const int n_steps = (tok_end - tok0 + 31) / 32;
    bf16x2 ones2;
    ones2[0] = (__bf16)1.f;
    ones2[1] = (__bf16)1.f;
    // the page ids of the whole unit, one per lane, fetched once: no dependent scalar load per step
    const int last_page = (tok_end - 1) / kPage - tok0 / kPage;      // last page of the chunk that holds visible tokens
    int my_page = cv.page_table[int64_t(b) * cv.max_pages + tok0 / kPage + min(lane, last_page)];
    my_page = min(max(my_page, 0), cv.n_pages - 1);
    const int64_t page_k = int64_t(cv.n_kv_heads) * KCH * (kPage * 8);
    const int64_t page_v = int64_t(cv.n_kv_heads) * D * kPage;
    // K: lane (m = n, g4) reads d-chunk 4 j + g4 of key row m; row m lives in page m / 8, slot m % 8 for X and
    // + 8 for Y -- the 64 lanes of one load instruction take whole 128-byte lines (eight slots of a d-chunk), none
    // shared with another instruction
    const bool k_second_page = (n >> 3) != 0;
    const uint16_t* k_lane = cv.k_pool + int64_t(h) * KCH * (kPage * 8) + g4 * (kPage * 8) + (n & 7) * 8;
    // V: lane (m = n, g4) reads slots 8 (g4 % 2) .. + 7 of row d = 16 db + m in page g4 / 2
    const bool v_second_page = (g4 >> 1) != 0;
    const uint16_t* v_lane = cv.v_pool + int64_t(h) * D * kPage + n * kPage + 8 * (g4 & 1);

    // value of the three other lanes of a query column folded in (lanes n, n + 16, n + 32, n + 48):
    // v_permlane16_swap / v_permlane32_swap exchange 16- / 32-lane rows between their two operands; with
    // both operands set to x, every lane finds x of lane ^ 16 (^ 32) in one of the two results
    auto column_max = [&](float x) {
        float a1 = x, b1 = x;
        asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a1), "+v"(b1));
        float a2 = fmaxf(a1, b1), b2 = a2;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a2), "+v"(b2));
        return fmaxf(a2, b2);
    };

    // one step = 32 tokens (two pages): 8 key loads and 8 value loads of 16 bytes per lane
    auto load = [&](int s, u32x4 (&kx)[KS], u32x4 (&ky)[KS], u32x4 (&vv)[DB]) {
        // page ids of this step (uniform); pages past the visible length fall back to the last visible one
        const int id0 = __builtin_amdgcn_readlane(my_page, min(2 * s, last_page));
        const int id1 = __builtin_amdgcn_readlane(my_page, min(2 * s + 1, last_page));
        const uint16_t* kp = k_lane + int64_t(k_second_page ? id1 : id0) * page_k;
        const uint16_t* vp = v_lane + int64_t(v_second_page ? id1 : id0) * page_v;
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            kx[j] = key_load<STREAM_KEYS>(kp + 4 * j * (kPage * 8));
            ky[j] = key_load<STREAM_KEYS>(kp + 4 * j * (kPage * 8) + 8 * 8);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) vv[db] = stream_load(vp + db * 16 * kPage);
    };
    auto compute = [&](int s, const u32x4 (&kx)[KS], const u32x4 (&ky)[KS], u32x4 (&vv)[DB]) {
        const int first = tok0 + 32 * s + 8 * g4;       // token of this lane's first VALUE slot
        // scores of this lane: X rows 4 g4 .. + 3 and the Y rows eight slots further on
        const int first_k = tok0 + 32 * s + 16 * (g4 >> 1) + 4 * (g4 & 1);
        f32x4 sx = {0.f, 0.f, 0.f, 0.f}, sy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kx[j]), qf[j], sx, 0, 0, 0);
            sy = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ky[j]), qf[j], sy, 0, 0, 0);
        }
        float t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = fmaf(e < 4 ? sx[e] : sy[e - 4], scale_log2, -m_ref);
        if (tok0 + 32 * s + 32 > limit_min) {           // uniform: a step that reaches some row's limit
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = first_k + (e & 3) + 8 * (e >> 2) < limit ? t[e] : -INFINITY;
        }
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, t[e]);
        if (__any(mx > kLazyRise || (!has_ref && mx > -INFINITY))) {
            // out of line: move the reference of the rows that need it, rescale what they have accumulated
            const float rise = column_max(mx);
            const bool move = has_ref ? rise > 0.f : rise > -INFINITY;
            const float shift = move ? rise : 0.f;
            const float alpha = has_ref ? __builtin_amdgcn_exp2f(-shift) : 1.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] -= shift;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 4; ++i) o_acc[db][i] *= alpha;
            m_ref += shift;
            has_ref = has_ref || move;
        }
        u32x4 pw;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            bf16x2 p2;
            p2[0] = (__bf16)__builtin_amdgcn_exp2f(t[e]);
            p2[1] = (__bf16)__builtin_amdgcn_exp2f(t[e + 1]);
            l_run = __builtin_amdgcn_fdot2_f32_bf16(p2, ones2, l_run, false);
            pw[e / 2] = __builtin_bit_cast(uint32_t, p2);
        }
        // The value operand of lane group g4 holds slots 8 (g4 % 2) .. + 7 of page g4 / 2, in order; the weights
        // of those slots sit half in this lane (X for even, Y for odd groups) and half in the lane of group g4 ^ 1:
        // one exchange of 16-lane rows per register pair (odd rows of the X words against even rows of the Y words)
        // leaves every lane with the eight weights of its value slots, in slot order.
#pragma unroll
        for (int r = 0; r < 2; ++r)
            asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(pw[r]), "+v"(pw[2 + r]));
        const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
        if (tok0 + 32 * s + 32 > len) {                 // uniform: only the step that holds the end of the cache
            u32x4 keep;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                keep[e] = (first + 2 * e < len ? 0x0000ffffu : 0u) | (first + 2 * e + 1 < len ? 0xffff0000u : 0u);
#pragma unroll
            for (int db = 0; db < DB; ++db) vv[db] &= keep;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
            o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv[db]), pb, o_acc[db], 0, 0, 0);
    };
    if (PREFETCH) {
        // The loads of step s + 1 are issued before step s is computed (two register sets, used in turn): a wave
        // has up to two steps' worth of bytes in flight, and a load's latency is covered by the step before it.
        u32x4 kxa[KS], kya[KS], vva[DB], kxb[KS], kyb[KS], vvb[DB];
        if (n_steps > 0) load(0, kxa, kya, vva);
        for (int s = 0; s < n_steps; s += 2) {
            if (s + 1 < n_steps) load(s + 1, kxb, kyb, vvb);
            __builtin_amdgcn_sched_barrier(0);
            compute(s, kxa, kya, vva);
            if (s + 1 < n_steps) {
                if (s + 2 < n_steps) load(s + 2, kxa, kya, vva);
                __builtin_amdgcn_sched_barrier(0);
                compute(s + 1, kxb, kyb, vvb);
            }
        }
    } else {
        for (int s = 0; s < n_steps; ++s) {
            u32x4 kx[KS], ky[KS], vv[DB];
            load(s, kx, ky, vv);
            compute(s, kx, ky, vv);
        }
    }
}

template <int D, bool STREAM_KEYS>
__global__ __launch_bounds__(64, 2) void decode_split16_kernel(DecodeArgs a) {
    constexpr int KS = D / 32, DB = D / 16, KCH = D / 8;
    const WaveStamp stamp(a);
    const int lane = threadIdx.x;
    const int nc = a.ncs + a.ncr + a.append;             // (append: one more slot per sequence and head, the new token's)
    const int c = int(blockIdx.x % unsigned(nc));
    const unsigned bh = blockIdx.x / unsigned(nc);
    const int h = int(bh % unsigned(a.n_kv_heads));
    const int b = int(bh / unsigned(a.n_kv_heads));
    const bool is_src = c < a.ncs;
    const bool is_tok = c == a.ncs + a.ncr;
    const CacheView& cv = is_src ? a.src : a.rsn;
    const int cc = is_src ? c : c - a.ncs;
    const int len_all = min(max(is_src ? a.src_len[b] : a.rsn_len[b], 0), cv.max_pages * kPage);
    const int len = (a.append && !is_src && len_all > 0) ? len_all - 1 : len_all;     // cached tokens to walk
    const int tok0 = is_tok ? 0 : cc * a.chunk;
    if (is_tok ? len_all == 0 : tok0 >= len) return;
    const int tok_end = min(len, tok0 + a.chunk);

    const int n = lane & 15, g4 = lane >> 4;
    const bool valid_row = n < a.rows;
    const int nr = min(n, a.rows - 1);                  // rows past the end repeat the last one (never stored)
    const int t_row = nr / a.group;
    const int hq = h * a.group + nr % a.group;
    const int limit = is_src ? len : max(len - a.q_len + t_row + 1, 0);
    const int limit_min = is_src ? len : max(len - a.q_len + 1, 0);     // the smallest limit of any row (row 0's)
    bf16x8 qf[KS];
    {
        const uint16_t* qp = a.q + ((int64_t(b) * a.q_len + t_row) * a.n_q_heads + hq) * D + 8 * g4;
#pragma unroll
        for (int j = 0; j < KS; ++j) qf[j] = *reinterpret_cast<const bf16x8*>(qp + 32 * j);
    }
    if (a.rope) {
        const int len_r = min(max(a.rsn_len[b], 0), a.rsn.max_pages * kPage);
        rotate_query<KS, 32>(qf, 8 * g4, max(len_r - a.q_len + t_row, 0), a.freq);
    }
    f32x4 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_ref = 0.f, l_run = 0.f;
    bool has_ref = false;
    if (is_tok) {
        // the new token: key fragments in the query's layout (piece 4 j + g4 of the row), rotated by the token's index
        const int idx = len_all - 1;
        bf16x8 kf[KS];
        const uint16_t* kp = a.k_new + (int64_t(b) * a.n_kv_heads + h) * D + 8 * g4;
#pragma unroll
        for (int j = 0; j < KS; ++j) kf[j] = *reinterpret_cast<const bf16x8*>(kp + 32 * j);
        if (a.rope) rotate_query<KS, 32>(kf, 8 * g4, idx, a.freq);
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < KS; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(float(qf[j][e]), float(kf[j][e]), dot);
        dot += __shfl_xor(dot, 16);
        dot += __shfl_xor(dot, 32);
        m_ref = dot * a.scale_log2;
        has_ref = true;
        l_run = g4 == 0 ? 1.f : 0.f;                                  // (summed over the four lanes of a row below)
        const uint16_t* vp = a.v_new + (int64_t(b) * a.n_kv_heads + h) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) o_acc[db][i] = bf16_bits_to_f32(vp[16 * db + 4 * g4 + i]);
        // into the cache: this head's key and value at index idx; the workgroup of head 0 writes the new length
        const int id = a.rsn.page_table[int64_t(b) * a.rsn.max_pages + idx / kPage];
        const int slot_in_page = idx % kPage;
        if (id >= 0 && id < a.rsn.n_pages) {                          // never write outside the pool
            if (n == 0) {
                uint16_t* kdst = a.rsn.k_pool + (int64_t(id) * a.n_kv_heads + h) * KCH * (kPage * 8) + slot_in_page * 8;
#pragma unroll
                for (int j = 0; j < KS; ++j) *reinterpret_cast<bf16x8*>(kdst + (4 * j + g4) * (kPage * 8)) = kf[j];
            }
            uint16_t* vdst = a.rsn.v_pool + (int64_t(id) * a.n_kv_heads + h) * (D * kPage) + slot_in_page;
            for (int d0 = lane; d0 < D; d0 += 64) vdst[d0 * kPage] = vp[d0];
        }
        if (h == 0 && lane == 0) a.rsn.appended_len[b] = len_all;
    } else {
        scan_unit16<D, true, STREAM_KEYS>(cv, b, h, lane, tok0, tok_end, len, min(limit, len), min(limit_min, len), a.scale_log2, qf, o_acc, m_ref, l_run,
                                                has_ref);
    }

    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (!valid_row) return;
    const int64_t slot = ((int64_t(b) * a.n_kv_heads + h) * nc + c) * a.rows + n;
    float* po = a.part_o + slot * D;
    // lane (n, g4), block db, register i  <->  d = 16 db + 4 g4 + i
#pragma unroll
    for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db + 4 * g4) = o_acc[db];
    if (g4 == 0) {
        a.part_ml[slot * 2] = has_ref ? m_ref : -INFINITY;
        a.part_ml[slot * 2 + 1] = l_tot;
    }
}

// Short caches (the streaming session of one listener: a hundred source tokens, a few hundred reasoning tokens): one
// workgroup per (sequence, KV head) does everything -- no partial results in memory, no merge kernel, one launch per
// layer and token instead of two.  Such a step is bound by the chain of memory round trips a wave makes walking its
// tokens, so the tokens of BOTH caches are dealt out in short units to the waves of the workgroup (wave w folds
// units w, w + W, ... into one running state), and the waves' states meet in LDS, where all threads merge them
// (log-sum-exp, fixed order) and write the finished rows.
constexpr int kSmallWaves = 8, kSmallUnit = 64;

// Rotation of a fragment set (layout of rotate_query<KS, 32>) by cos / sin values parked in LDS: entry i belongs
// to head dims i and D/2 + i.
template <int KS>
__device__ __forceinline__ void rotate_fragments(bf16x8 (&f)[KS], int off, const float* cs, const float* sn) {
#pragma unroll
    for (int j = 0; j < KS / 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float c = cs[32 * j + off + e], s_ = sn[32 * j + off + e];
            const float x = float(f[j][e]), y = float(f[j + KS / 2][e]);
            f[j][e] = (__bf16)(x * c - y * s_);
            f[j + KS / 2][e] = (__bf16)(y * c + x * s_);
        }
}

// APPEND (one new token per sequence, q_len = 1): k_new / v_new [batch][Hkv][D] is the token at index
// rsn_len[b] - 1 of the reasoning stream.  The workgroup of (sequence, KV head) stores its head's key (rotated by
// that index if a.rope) and value in the reasoning cache, folds the token in from registers -- score in fp32 from
// the bf16 operands, as the matrix instruction would -- and walks the cache only up to the token before it; the
// workgroup of head 0 writes the new length.  Nobody in this launch reads what it writes.
template <int D, bool APPEND>
__global__ __launch_bounds__(64 * kSmallWaves) void decode_small16_kernel(DecodeArgs a, uint16_t* __restrict__ out, float* __restrict__ lse,
                                                                          const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new) {
    constexpr int KS = D / 32, DB = D / 16, KCH = D / 8;
    constexpr int W = kSmallWaves, UNIT = kSmallUnit;
    constexpr int WP = APPEND ? W + 1 : W;            // states to merge: the waves' and the new token's
    extern __shared__ __align__(16) unsigned char smem_raw[];
    // [WP][rows][D] partial outputs, [WP][rows] reference exponents, [WP][rows] sums, [D/2] cos, [D/2] sin
    float* sm_o = reinterpret_cast<float*>(smem_raw);
    float* sm_m = sm_o + WP * a.rows * D;
    float* sm_l = sm_m + WP * a.rows;
    float* sm_cs = sm_l + WP * a.rows;
    float* sm_sn = sm_cs + D / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = int(blockIdx.x % unsigned(a.n_kv_heads));
    const int b = int(blockIdx.x / unsigned(a.n_kv_heads));
    const int n = lane & 15, g4 = lane >> 4;
    const bool valid_row = n < a.rows;
    const int nr = min(n, a.rows - 1);
    const int t_row = nr / a.group;
    const int hq = h * a.group + nr % a.group;
    const int len_s = min(max(a.src_len[b], 0), a.src.max_pages * kPage);
    const int len_all = min(max(a.rsn_len[b], 0), a.rsn.max_pages * kPage);
    const bool add = APPEND && len_all > 0;          // (rsn_len 0: an idle sequence, nothing to store)
    const int len_r = add ? len_all - 1 : len_all;   // cached reasoning tokens to walk
    const int units_s = (len_s + UNIT - 1) / UNIT, units = units_s + (len_r + UNIT - 1) / UNIT;

    if (a.rope) {
        // q_len rows at consecutive positions: the workgroup evaluates the D/2 (cos, sin) pairs of the LAST row's
        // position once; other rows (q_len > 1 only) rotate by their own position the slow way
        if (threadIdx.x < D / 2) rope_cos_sin(max(len_all - 1, 0), a.freq.f[threadIdx.x], &sm_cs[threadIdx.x], &sm_sn[threadIdx.x]);
        __syncthreads();
    }
    f32x4 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_ref = 0.f, l_run = 0.f;
    bool has_ref = false;
    if (wave < units || (APPEND && wave == W - 1)) {      // (uniform per wave)
        bf16x8 qf[KS];
        {
            const uint16_t* qp = a.q + ((int64_t(b) * a.q_len + t_row) * a.n_q_heads + hq) * D + 8 * g4;
#pragma unroll
            for (int j = 0; j < KS; ++j) qf[j] = *reinterpret_cast<const bf16x8*>(qp + 32 * j);
        }
        if (a.rope) {
            if (a.q_len == 1) rotate_fragments<KS>(qf, 8 * g4, sm_cs, sm_sn);
            else rotate_query<KS, 32>(qf, 8 * g4, max(len_all - a.q_len + t_row, 0), a.freq);
        }
        if (APPEND && wave == W - 1 && add) {
            // the new token: key fragments in the query's layout (piece 4 j + g4 of the row), the same for every row
            bf16x8 kf[KS];
            const uint16_t* kp = k_new + (int64_t(b) * a.n_kv_heads + h) * D + 8 * g4;
#pragma unroll
            for (int j = 0; j < KS; ++j) kf[j] = *reinterpret_cast<const bf16x8*>(kp + 32 * j);
            if (a.rope) rotate_fragments<KS>(kf, 8 * g4, sm_cs, sm_sn);
            float dot = 0.f;
#pragma unroll
            for (int j = 0; j < KS; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(float(qf[j][e]), float(kf[j][e]), dot);
            dot += __shfl_xor(dot, 16);
            dot += __shfl_xor(dot, 32);
            if (valid_row && g4 == 0) {
                sm_m[W * a.rows + n] = dot * a.scale_log2;
                sm_l[W * a.rows + n] = 1.f;
            }
            // into the cache: page of index len_all - 1, this head
            const int idx = len_all - 1;
            const int id = a.rsn.page_table[int64_t(b) * a.rsn.max_pages + idx / kPage];
            const int slot = idx % kPage;
            const uint16_t* vp = v_new + (int64_t(b) * a.n_kv_heads + h) * D;
            if (id >= 0 && id < a.rsn.n_pages) {             // never write outside the pool
                if (n == 0) {
                    uint16_t* kdst = a.rsn.k_pool + (int64_t(id) * a.n_kv_heads + h) * KCH * (kPage * 8) + slot * 8;
#pragma unroll
                    for (int j = 0; j < KS; ++j) *reinterpret_cast<bf16x8*>(kdst + (4 * j + g4) * (kPage * 8)) = kf[j];
                }
                uint16_t* vdst = a.rsn.v_pool + (int64_t(id) * a.n_kv_heads + h) * (D * kPage) + slot;
                for (int d0 = lane; d0 < D; d0 += 64) vdst[d0 * kPage] = vp[d0];
            }
            // the token's value row is its partial output, the same for every row
            for (int e = lane; e < a.rows * D; e += 64) sm_o[W * a.rows * D + e] = bf16_bits_to_f32(vp[e % D]);
            if (h == 0 && lane == 0) a.rsn.appended_len[b] = len_all;
        }
        // the source slice is seen whole; reasoning token j by rows t with j <= len_all - q_len + t
        const int limit = min(max(len_all - a.q_len + t_row + 1, 0), len_r), limit_min = min(max(len_all - a.q_len + 1, 0), len_r);
        for (int u = wave; u < units; u += W) {
            if (u < units_s) {
                const int tok0 = u * UNIT;
                scan_unit16<D>(a.src, b, h, lane, tok0, min(len_s, tok0 + UNIT), len_s, len_s, len_s, a.scale_log2, qf, o_acc, m_ref, l_run, has_ref);
            } else {
                const int tok0 = (u - units_s) * UNIT;
                scan_unit16<D>(a.rsn, b, h, lane, tok0, min(len_r, tok0 + UNIT), len_r, limit, limit_min, a.scale_log2, qf, o_acc, m_ref, l_run, has_ref);
            }
        }
    }
    if (APPEND && !add && wave == W - 1 && lane < a.rows) sm_m[W * a.rows + lane] = -INFINITY;
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (valid_row) {
        // lane (n, g4), block db, register i  <->  d = 16 db + 4 g4 + i
        float* po = sm_o + (wave * a.rows + n) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db + 4 * g4) = o_acc[db];
        if (g4 == 0) {
            sm_m[wave * a.rows + n] = has_ref ? m_ref : -INFINITY;
            sm_l[wave * a.rows + n] = l_tot;
        }
    }
    __syncthreads();
    // merge: thread -> (row, 4 head dims); rows * D / 4 of the threads have work
    const int e0 = int(threadIdx.x) * 4;
    for (int e = e0; e < a.rows * D; e += 64 * W * 4) {
        const int row = e / D, d0 = e % D;
        float m_all = -INFINITY;
#pragma unroll
        for (int w = 0; w < WP; ++w) m_all = fmaxf(m_all, sm_m[w * a.rows + row]);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
        if (m_all != -INFINITY) {
#pragma unroll
            for (int w = 0; w < WP; ++w) {
                const float mw = sm_m[w * a.rows + row];
                if (mw == -INFINITY) continue;                        // a state that holds nothing for this row
                const float wt = __builtin_amdgcn_exp2f(mw - m_all);
                den = fmaf(wt, sm_l[w * a.rows + row], den);
                const f32x4 o = *reinterpret_cast<const f32x4*>(sm_o + (w * a.rows + row) * D + d0);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fmaf(wt, o[i], acc[i]);
            }
        }
        const float inv = den > 0.f ? 1.f / den : 0.f;               // a row that sees nothing: out = 0, lse = -inf
        const int t = row / a.group, hq_row = h * a.group + row % a.group;
        bf16x4 o4;
#pragma unroll
        for (int i = 0; i < 4; ++i) o4[i] = (__bf16)(acc[i] * inv);
        *reinterpret_cast<bf16x4*>(out + ((int64_t(b) * a.q_len + t) * a.n_q_heads + hq_row) * D + d0) = o4;
        if (lse && d0 == 0)
            lse[(int64_t(b) * a.q_len + t) * a.n_q_heads + hq_row] = den > 0.f ? (m_all + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
    }
}

// The one-wave kernel over 8-bit caches (E4M3 codes, one power-of-two fp32 scale per key row and per value
// row): half the bytes per token.  Codes become bf16 in registers (exact: 3 mantissa bits) and feed the same
// two bf16 products; the key scale multiplies the score (folded into the softmax scale factor), the value
// scale multiplies the probability before the second product -- both exact, the scales being powers of two.
// Pool layouts [page][head][D/16][slot][16] and [page][head][D][slot] bytes keep the loads contiguous:
//   K: lane (m, g4) reads the 16 bytes d = 64 jj + 16 g4 .. + 15 of key row m: two k-steps' worth (the query
//      fragments use the same assignment of head dims to k-steps)
//   V: lane (m, g4) reads the 16 bytes (all slots) of row d = 16 db + m in page g4: two k-steps' worth
//   scales: the 16 + 16 floats of page g4.
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16(uint32_t lo, uint32_t hi) {
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.f, false), b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.f, false), d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.f, true);
    bf16x8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

template <int D>
__global__ __launch_bounds__(64, 3) void decode_split16_fp8_kernel(DecodeArgs a) {
    constexpr int KS = D / 32, KP = D / 64, DB = D / 16, C16 = D / 16;
    const int lane = threadIdx.x;
    const int nc = a.ncs + a.ncr;
    const int c = int(blockIdx.x % unsigned(nc));
    const unsigned bh = blockIdx.x / unsigned(nc);
    const int h = int(bh % unsigned(a.n_kv_heads));
    const int b = int(bh / unsigned(a.n_kv_heads));
    const bool is_src = c < a.ncs;
    const CacheView& cv = is_src ? a.src : a.rsn;
    const int cc = is_src ? c : c - a.ncs;
    const int len = min(max(is_src ? a.src_len[b] : a.rsn_len[b], 0), cv.max_pages * kPage);
    const int tok0 = cc * a.chunk;
    if (tok0 >= len) return;
    const int tok_end = min(len, tok0 + a.chunk);
    // With half the bytes per token, a wave takes 64 tokens (four pages) per step to keep as many bytes in flight
    // as the bf16 kernel does with 32.
    const int n_steps = (tok_end - tok0 + 63) / 64;

    const int n = lane & 15, g4 = lane >> 4;
    const bool valid_row = n < a.rows;
    const int nr = min(n, a.rows - 1);
    const int t_row = nr / a.group;
    const int hq = h * a.group + nr % a.group;
    const int limit = is_src ? len : max(len - a.q_len + t_row + 1, 0);
    const int limit_min = is_src ? len : max(len - a.q_len + 1, 0);
    bf16x2 ones2;
    ones2[0] = (__bf16)1.f;
    ones2[1] = (__bf16)1.f;

    // query fragments: k-step j = 2 jj + u holds head dims 64 jj + 16 g4 + 8 u + e
    bf16x8 qf[KS];
    {
        const uint16_t* qp = a.q + ((int64_t(b) * a.q_len + t_row) * a.n_q_heads + hq) * D;
        const int len_r = min(max(a.rsn_len[b], 0), a.rsn.max_pages * kPage);
        const int pos = max(len_r - a.q_len + t_row, 0);
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            const int d0 = 64 * (j >> 1) + 16 * g4 + 8 * (j & 1);
            qf[j] = *reinterpret_cast<const bf16x8*>(qp + d0);
            if (a.rope) {
                // rotation pair of head dim d: (d, d + D/2); both halves come straight from memory
                const bool upper = d0 >= D / 2;
                const bf16x8 other = *reinterpret_cast<const bf16x8*>(qp + (upper ? d0 - D / 2 : d0 + D / 2));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float cs, sn;
                    rope_cos_sin(pos, a.freq.f[(upper ? d0 - D / 2 : d0) + e], &cs, &sn);
                    const float x = float(qf[j][e]), y = float(other[e]);
                    qf[j][e] = (__bf16)(upper ? x * cs + y * sn : x * cs - y * sn);
                }
            }
        }
    }
    f32x4 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) o_acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr float kLazyRise = 8.f;
    float m_ref = 0.f, l_run = 0.f;
    bool has_ref = false;

    const int last_page = (tok_end - 1) / kPage - tok0 / kPage;
    int my_page = cv.page_table[int64_t(b) * cv.max_pages + tok0 / kPage + min(lane, last_page)];
    my_page = min(max(my_page, 0), cv.n_pages - 1);
    const int64_t page_k = int64_t(cv.n_kv_heads) * C16 * (kPage * 16);      // bytes
    const int64_t page_v = int64_t(cv.n_kv_heads) * D * kPage;
    const int64_t page_s = int64_t(cv.n_kv_heads) * kPage;                   // floats
    // K: four 16-key sets per step; in set s, key row m = 4 gq + i is slot 4 s + i of page gq, so that afterwards
    //    lane group g4 holds all 16 slots of page g4 (set s, register i -> slot 4 s + i).  Lane (m = n, g4) reads
    //    the 16 bytes d = 64 jj + 16 g4 .. + 15 of its row.
    const int k_page_sel = n >> 2;
    const uint8_t* k_lane = reinterpret_cast<const uint8_t*>(cv.k_pool) + int64_t(h) * C16 * (kPage * 16) + g4 * (kPage * 16) + (n & 3) * 16;
    // V: lane (m = n, g4) reads the whole 16-slot row d = 16 db + m of page g4: slots 0..7 feed the first, 8..15 the
    //    second matrix instruction of the block
    const uint8_t* v_lane = reinterpret_cast<const uint8_t*>(cv.v_pool) + int64_t(h) * D * kPage + n * kPage;
    const int s_lane = h * kPage;

    auto column_max = [&](float x) {
        float a1 = x, b1 = x;
        asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a1), "+v"(b1));
        float a2 = fmaxf(a1, b1), b2 = a2;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a2), "+v"(b2));
        return fmaxf(a2, b2);
    };

    for (int s = 0; s < n_steps; ++s) {
        int id[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) id[u] = __builtin_amdgcn_readlane(my_page, min(4 * s + u, last_page));
        const int id_k = k_page_sel == 0 ? id[0] : k_page_sel == 1 ? id[1] : k_page_sel == 2 ? id[2] : id[3];
        const int id_g = g4 == 0 ? id[0] : g4 == 1 ? id[1] : g4 == 2 ? id[2] : id[3];
        const uint8_t* kp = k_lane + int64_t(id_k) * page_k;
        const uint8_t* vp = v_lane + int64_t(id_g) * page_v;
        const int64_t sp = int64_t(id_g) * page_s + s_lane;
        u32x4 k8[4][KP], v8[DB];
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int jj = 0; jj < KP; ++jj) k8[st][jj] = *reinterpret_cast<const u32x4*>(kp + 4 * jj * (kPage * 16) + 4 * st * 16);
#pragma unroll
        for (int db = 0; db < DB; ++db) v8[db] = stream_load(vp + db * 16 * kPage);
        f32x4 ks[4], vs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ks[u] = *reinterpret_cast<const f32x4*>(cv.k_scale + sp + 4 * u);
            vs[u] = *reinterpret_cast<const f32x4*>(cv.v_scale + sp + 4 * u);
        }

        const int first = tok0 + 64 * s + 16 * g4;      // token of this lane's slot 0
        f32x4 sc[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            sc[st] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const int jj = j >> 1, u = j & 1;
                sc[st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(k8[st][jj][2 * u], k8[st][jj][2 * u + 1]), qf[j], sc[st], 0, 0, 0);
            }
        }
        const bool reaches_limit = tok0 + 64 * s + 64 > limit_min;      // uniform
        float t[16], vsc[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {                  // slot e = 4 set + register
            t[e] = fmaf(sc[e >> 2][e & 3], ks[e >> 2][e & 3] * a.scale_log2, -m_ref);
            vsc[e] = vs[e >> 2][e & 3];
        }
        if (reaches_limit) {
            // slots past the visible length hold anything (scales included): remove them by index
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                t[e] = first + e < limit ? t[e] : -INFINITY;
                vsc[e] = first + e < len ? vsc[e] : 0.f;
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, t[e]);
        if (__any(mx > kLazyRise || (!has_ref && mx > -INFINITY))) {
            const float rise = column_max(mx);
            const bool move = has_ref ? rise > 0.f : rise > -INFINITY;
            const float shift = move ? rise : 0.f;
            const float alpha = has_ref ? __builtin_amdgcn_exp2f(-shift) : 1.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) t[e] -= shift;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 4; ++i) o_acc[db][i] *= alpha;
            m_ref += shift;
            has_ref = has_ref || move;
        }
        bf16x8 pb[2];
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(t[e]), p1 = __builtin_amdgcn_exp2f(t[e + 1]);
            bf16x2 p2;
            p2[0] = (__bf16)p0;
            p2[1] = (__bf16)p1;
            l_run = __builtin_amdgcn_fdot2_f32_bf16(p2, ones2, l_run, false);
            pb[e >> 3][e & 7] = (__bf16)(p0 * vsc[e]);
            pb[e >> 3][(e & 7) + 1] = (__bf16)(p1 * vsc[e + 1]);
        }
        u32x4 keep[2];
        keep[0] = keep[1] = u32x4{0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
        if (tok0 + 64 * s + 64 > len) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    keep[hf][e] = (first + 8 * hf + 2 * e < len ? 0x0000ffffu : 0u) | (first + 8 * hf + 2 * e + 1 < len ? 0xffff0000u : 0u);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const u32x4 vb = __builtin_bit_cast(u32x4, e4m3x8_to_bf16(v8[db][2 * hf], v8[db][2 * hf + 1])) & keep[hf];
                o_acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vb), pb[hf], o_acc[db], 0, 0, 0);
            }
    }

    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (!valid_row) return;
    const int64_t slot = ((int64_t(b) * a.n_kv_heads + h) * nc + c) * a.rows + n;
    float* po = a.part_o + slot * D;
#pragma unroll
    for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db + 4 * g4) = o_acc[db];
    if (g4 == 0) {
        a.part_ml[slot * 2] = has_ref ? m_ref : -INFINITY;
        a.part_ml[slot * 2 + 1] = l_tot;
    }
}

// One wave (one workgroup) per (sequence, query row, query head): log-sum-exp merge of the
// partials of both caches, in a fixed order (run-to-run identical results).  The partial rows are
// fetched 32 at a time with independent loads -- one memory round trip per batch instead of one
// per partial -- and folded with a running maximum across batches.
template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(DecodeArgs a, uint16_t* __restrict__ out,
                                                            float* __restrict__ lse) {
    constexpr int PER = D / 64;
    constexpr int BATCH = 32;
    const int lane = threadIdx.x;
    const int hq = int(blockIdx.x % unsigned(a.n_q_heads));
    const int t = int((blockIdx.x / unsigned(a.n_q_heads)) % unsigned(a.q_len));
    const int b = int(blockIdx.x / unsigned(a.n_q_heads * a.q_len));
    const int h = hq / a.group, n = t * a.group + hq % a.group;
    const int nc = a.ncs + a.ncr + a.append;
    const int len_s = min(max(a.src_len[b], 0), a.src.max_pages * kPage);
    const int len_all = min(max(a.rsn_len[b], 0), a.rsn.max_pages * kPage);
    const int n_tok = (a.append && len_all > 0) ? 1 : 0;            // the new token's own partial (slot ncs + ncr)
    const int len_r = len_all - n_tok;                               // what the split kernel walked
    const int n_s = min((len_s + a.chunk - 1) / a.chunk, a.ncs), n_r = min((len_r + a.chunk - 1) / a.chunk, a.ncr);
    const int n_tot = n_s + n_r + n_tok;
    const int64_t base = (int64_t(b) * a.n_kv_heads + h) * nc;
    // partial i of the row -> slot: source units, reasoning units, then the token
    auto slot_of = [&](int i) { return i < n_s ? i : i < n_s + n_r ? a.ncs + (i - n_s) : a.ncs + a.ncr; };

    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;
    float den = 0.f, m_run = -INFINITY;
    for (int i0 = 0; i0 < n_tot; i0 += BATCH) {
        const int cnt = min(BATCH, n_tot - i0);
        // lane u < cnt owns (m, l) of partial i0 + u
        float m_mine = -INFINITY, l_mine = 0.f;
        if (lane < cnt) {
            const int i = i0 + lane;
            const int c = slot_of(i);
            const f32x2 ml = *reinterpret_cast<const f32x2*>(a.part_ml + ((base + c) * a.rows + n) * 2);
            m_mine = ml[0];
            l_mine = ml[1];
        }
        float rows[BATCH][PER];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int i = i0 + min(u, cnt - 1);          // rows past the end repeat the last one, with weight 0
            const int c = slot_of(i);
            const float* po = a.part_o + ((base + c) * a.rows + n) * D + lane * PER;
#pragma unroll
            for (int e = 0; e < PER; ++e) rows[u][e] = po[e];
        }
        float bm = m_mine;
        for (int o = 32; o > 0; o >>= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
        const float m_new = fmaxf(m_run, bm);
        if (m_new == -INFINITY) continue;                // nothing visible in this batch or before
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        const float w_mine = __builtin_amdgcn_exp2f(m_mine - m_new);     // 0 for lanes >= cnt
        float wl = w_mine * l_mine;
        for (int o = 32; o > 0; o >>= 1) wl += __shfl_xor(wl, o);
        den = den * alpha + wl;
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const float w = __shfl(w_mine, u);
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[e] = fmaf(w, rows[u][e], acc[e]);
        }
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    uint16_t* op = out + ((int64_t(b) * a.q_len + t) * a.n_q_heads + hq) * D + lane * PER;
#pragma unroll
    for (int e = 0; e < PER; ++e) op[e] = f32_to_bf16_bits(acc[e] * inv);
    if (lse && lane == 0)
        lse[(int64_t(b) * a.q_len + t) * a.n_q_heads + hq] = den > 0.f ? (m_run + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
}

// Source-chunk prefill (Alg. 1, prefill loop) with the cache pages SHARED through LDS: one workgroup per
// (sequence, KV head, group of 128 query rows, work unit of the source cache: chunk_units), wave w = the w-th block of
// 32 (token, head) rows.  Per step the four waves copy four pages (64 tokens) of K and of V -- 4 KB each at
// D = 128, verbatim, with asynchronous global -> LDS copies, one step ahead -- and every wave takes its matrix
// operands from there, so a page is fetched from L2 once per workgroup and not once per row block.  The pool
// layout of K is conflict-free as it is (16 slots x 16 bytes contiguous per 8-dim chunk); the 32-byte rows of V
// are not, so the copy swaps the two halves of every second group of 8 rows (by choosing what each lane fetches).
// Softmax as in the prefill kernel (prescaled queries, reference parked in the last score block, no running maximum);
// partial results [B][Hkv][row block][unit][32 rows],
// merged by chunk_combine_kernel.
// Work units of one sequence's source cache: as few as keep a unit within `target` tokens, all of the same length
// (a multiple of 64 tokens) -- equal units finish together, a long one beside a short remainder does not.
struct ChunkUnits {
    int len;      // tokens of the cache
    int size;     // tokens per unit
    int count;    // units
};
__device__ __forceinline__ ChunkUnits chunk_units(int len, int target) {
    ChunkUnits u;
    u.len = len;
    u.count = max((len + target - 1) / target, 1);
    u.size = ((len + u.count - 1) / u.count + 63) & ~63;
    return u;
}
constexpr int kChunkRankMax = 256;

template <int D, int STAGES, int TOK>
struct ChunkSmem {
    uint16_t k[STAGES][TOK * D];
    uint16_t v[STAGES][TOK * D];
};

// TOK tokens (TOK / 16 pages) per step, STAGES buffers of one step each, copies STAGES - 1 steps ahead.
template <int D, int STAGES, int TOK>
__global__ __launch_bounds__(256, 2) void chunk_split_lds_kernel(DecodeArgs a) {
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int PAGE = D * kPage;                   // elements of one page of one head, K or V
    constexpr int NL = PAGE * 2 / 1024;               // 1 KB copies per page
    constexpr int PG = TOK / kPage;                   // pages per step
    constexpr int SBN = TOK / 32;                     // 32-key blocks per step
    constexpr int PER_WAVE = 2 * PG / 4;              // page copies (K or V) per wave and step
    static_assert(TOK == 32 || TOK == 64, "32 or 64 tokens per step");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    ChunkSmem<D, STAGES, TOK>& sm = *reinterpret_cast<ChunkSmem<D, STAGES, TOK>*>(smem_raw);

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rb_groups = (a.row_blocks + 3) / 4;
    const CacheView& cv = a.src;
    // Which unit: the workgroups of a launch are handed out in index order and a unit keeps its compute unit for as
    // long as it has tokens, so the LONGEST units go first -- workgroup index / (heads x row groups) is a rank in the
    // order of decreasing unit length over all (sequence, unit) pairs (ties by index), worked out by every
    // workgroup from the lengths themselves (one entry per thread and pass; kChunkRankMax entries at most, beyond
    // that the units go in index order).
    __shared__ __align__(16) int s_unit_len[kChunkRankMax];
    __shared__ int s_pick;
    const int per_rank = a.n_kv_heads * rb_groups;
    const int rank = int(blockIdx.x / unsigned(per_rank));
    const int hr = int(blockIdx.x % unsigned(per_rank));
    const int h = hr / rb_groups, rbg = hr % rb_groups;
    const int n_entries = a.batch * a.ncs;
    int entry = rank;
    if (n_entries <= kChunkRankMax) {
        const int padded = (n_entries + 3) & ~3;     // (entries past the end: -1, behind every real one)
        for (int e = threadIdx.x; e < padded; e += 256) {
            int tokens = -1;
            if (e < n_entries) {
                const int bb = e / a.ncs, cc = e % a.ncs;
                const ChunkUnits u = chunk_units(min(max(a.src_len[bb], 0), cv.max_pages * kPage), a.chunk);
                tokens = max(min(u.len - cc * u.size, u.size), 0);
            }
            s_unit_len[e] = tokens;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < n_entries; e += 256) {
            const int mine = s_unit_len[e];
            int before = 0;
            for (int o = 0; o < padded; o += 4) {
                const int4 other = *reinterpret_cast<const int4*>(&s_unit_len[o]);
                before += (other.x > mine || (other.x == mine && o < e)) ? 1 : 0;
                before += (other.y > mine || (other.y == mine && o + 1 < e)) ? 1 : 0;
                before += (other.z > mine || (other.z == mine && o + 2 < e)) ? 1 : 0;
                before += (other.w > mine || (other.w == mine && o + 3 < e)) ? 1 : 0;
            }
            if (before == rank) s_pick = e;          // exactly one entry has this rank
        }
        __syncthreads();
        entry = s_pick;
    }
    const int b = __builtin_amdgcn_readfirstlane(entry / a.ncs), c = __builtin_amdgcn_readfirstlane(entry % a.ncs);
    const int len = min(max(a.src_len[b], 0), cv.max_pages * kPage);
    const ChunkUnits units_b = chunk_units(len, a.chunk);
    const int tok0 = c * units_b.size;
    if (tok0 >= len) return;
    const int q_len = min(min(max(a.n_new ? a.n_new[b] : a.max_new, 0), a.max_new), len);
    const int n_rows = q_len * a.group;
    if (rbg * 128 >= n_rows) return;
    // the group's last row sees the most: a chunk past its limit holds nothing for any of its blocks
    const int group_last_t = min(q_len - 1, (rbg * 128 + 127) / a.group);
    if (tok0 >= len - q_len + group_last_t + 1) return;
    const int tok_end = min(len, tok0 + units_b.size);
    const int n_steps = (tok_end - tok0 + TOK - 1) / TOK;

    const int n = lane & 31, hg = lane >> 5;
    const int rb = rbg * 4 + wave;
    const int r = rb * 32 + n;
    const bool valid_row = r < n_rows;
    const int t_row = min(r, n_rows - 1) / a.group;
    const int hq = h * a.group + min(r, n_rows - 1) % a.group;
    // this wave's block: anything to do in this chunk?  (uniform; the wave still copies and meets the barriers)
    const int block_last_t = min(q_len - 1, (rb * 32 + 31) / a.group);
    const bool wave_works = rb * 32 < n_rows && tok0 < len - q_len + block_last_t + 1;
    const int limit = valid_row ? len - q_len + t_row + 1 : 0;                   // row sees tokens [0, limit)
    const int block_first_t = min(q_len - 1, (rb * 32) / a.group);
    const int limit_min = len - q_len + block_first_t + 1;                       // smallest limit of the block's valid rows

    bf16x8 qf[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j)
        qf[j] = *reinterpret_cast<const bf16x8*>(a.q + ((int64_t(b) * a.max_new + t_row) * a.n_q_heads + hq) * D + 16 * j + 8 * hg);
    if (a.rope) rotate_query<KS, 16>(qf, 8 * hg, max(len - q_len + t_row, 0), a.freq);
    // queries times scale * log2(e), rounded to bf16 again: K q' is the exponent of the softmax weight
#pragma unroll
    for (int j = 0; j < KS; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[j][e] = (__bf16)(float(qf[j][e]) * a.scale_log2);

    // Copies.  A step is PG pages of K and PG pages of V; the four waves share them out, PER_WAVE page copies each:
    // copy number x = wave * PER_WAVE + u is page x % PG of K (x < PG) or of V.
    const int32_t* table = cv.page_table + int64_t(b) * cv.max_pages;
    const int last_page = (tok_end - 1) / kPage;                                 // last page that holds visible tokens
    const int64_t page_stride = int64_t(cv.n_kv_heads) * PAGE;
    const uint16_t* k_src = cv.k_pool + int64_t(h) * PAGE;                       // (+ 16 bytes per lane)
    // V rows are 32 bytes: read as they lie, lanes d and d + 8 of a 16-lane group would meet in the same banks.  A copy
    // places lane l's 16 bytes at position l, but WHICH 16 bytes a lane fetches is free: position 2 d + x holds the
    // half x ^ bit 3 of d of row d, and the readers below undo that.
    const int v_perm = (lane & ~1) | ((lane & 1) ^ ((lane >> 4) & 1));           // chunk fetched by this lane (same for every 1 KB piece: 32 rows)
    const uint16_t* v_src = cv.v_pool + int64_t(h) * PAGE;                       // (+ 16 bytes per fetched chunk)
    const uint32_t k_lane_off = uint32_t(lane) * 16u, v_lane_off = uint32_t(v_perm) * 16u;
    const uint32_t lds_k = uint32_t(uintptr_t(&sm.k[0][0])), lds_v = uint32_t(uintptr_t(&sm.v[0][0]));
    // the page ids of the whole unit, fetched once (up to 256 pages: four per lane): a load per step would make
    // every step wait for a round trip to memory, and for all copies in flight with it
    int my_pages[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int id = table[min(tok0 / kPage + 64 * u + lane, last_page)];
        my_pages[u] = min(max(id, 0), cv.n_pages - 1);
    }
    auto issue = [&](int s, int stage) {
        s = min(s, n_steps - 1);                                                 // past the last step: the same pages again, never used
#pragma unroll
        for (int w = 0; w < PER_WAVE; ++w) {
            const int x = wave * PER_WAVE + w;                                   // (uniform)
            const bool is_v = x >= PG;
            const int pg = is_v ? x - PG : x;
            const int pl = min(PG * s + pg, last_page - tok0 / kPage);          // pages past the end: the last one again (masked)
            const int quarter = pl >> 6;
            const int held = quarter == 0 ? my_pages[0] : quarter == 1 ? my_pages[1] : quarter == 2 ? my_pages[2] : my_pages[3];
            const int id = __builtin_amdgcn_readlane(held, pl & 63);
            const uint16_t* src = (is_v ? v_src : k_src) + int64_t(id) * page_stride;
            const uint32_t dst = (is_v ? lds_v : lds_k) + uint32_t(stage) * (TOK * D * 2) + uint32_t(pg) * (PAGE * 2);
            async_copy_rows_nt<NL>(src, is_v ? v_lane_off : k_lane_off, dst);        // read once: 2 % faster with the hint
        }
    };
    // The chunk streams from HBM (about 125 flop per byte: below the ridge of this machine), so the bytes in flight
    // matter: copies run STAGES - 1 steps ahead.  Every iteration issues exactly one step's copies (clamped at the
    // end), which keeps the count the waits rely on.
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(s, s);

    f32x16 o_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
    constexpr float kRise = 16777216.f;               // 2^24
    float m_ref = 0.f, l_run = 0.f;
    bool has_ref = false;
    // operand addresses inside a stage (elements): K lane (m = n, hg): page n / 16 of the 32-key block, slot
    // swap23(n % 16), chunk 2 j + hg; V lane (m = n, hg): row 32 db + n, slots 8 hg .. + 7 of page t (halves swapped
    // for every second group of 8 rows, see above)
    const int k_off = (n >> 4) * PAGE + swap23(n & 15) * 8 + hg * (kPage * 8);
    const int v_off = n * kPage + 8 * (hg ^ ((n >> 3) & 1));
    // Score blocks of a step.  Between steps the LAST one holds -m_ref of this lane's row in all sixteen registers:
    // the first matrix instruction of every block takes it as its accumulator input (the last block in place, after
    // the others have read it), so the scores come out relative to the reference without a subtraction.
    f32x16 s_acc[SBN];
#pragma unroll
    for (int i = 0; i < 16; ++i) s_acc[SBN - 1][i] = 0.f;

    int stage = 0;
    for (int s = 0; s < n_steps; ++s) {
        wait_vmcnt<(STAGES - 2) * PER_WAVE * NL>();   // step s has landed (the STAGES - 2 younger ones may still fly) ...
        __syncthreads();                              // ... for every wave; and everybody is done with step s - 1,
        issue(s + STAGES - 1, stage == 0 ? STAGES - 1 : stage - 1);              // whose buffer the next copies take
        const uint16_t* kb = &sm.k[stage][0];
        const uint16_t* vb = &sm.v[stage][0];
        stage = stage == STAGES - 1 ? 0 : stage + 1;
        const int tok = tok0 + TOK * s;
        if (!wave_works || tok >= len - q_len + block_last_t + 1) continue;      // (uniform) nothing for this block here
        // operands leave LDS ahead of the matrix instructions that take them: all key fragments now, all value
        // fragments before the exponentials (scheduling barriers keep the compiler from moving them back)
        bf16x8 fk[SBN * KS];
#pragma unroll
        for (int f = 0; f < SBN * KS; ++f)
            fk[f] = *reinterpret_cast<const bf16x8*>(kb + 2 * (f % SBN) * PAGE + k_off + 2 * (f / SBN) * (kPage * 8));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < SBN * KS; ++f)
            s_acc[f % SBN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[f], qf[f / SBN], f < SBN ? s_acc[SBN - 1] : s_acc[f % SBN], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        u32x4 fv[PG * DB];
#pragma unroll
        for (int f = 0; f < PG * DB; ++f)
            fv[f] = *reinterpret_cast<const u32x4*>(vb + (f / DB) * PAGE + 32 * (f % DB) * kPage + v_off);
        __builtin_amdgcn_sched_barrier(0);
        // block sb, register i  <->  token tok + 32 sb + 16 (i/8) + 8 hg + i%8.  The scores leave the matrix pipe as
        // exponents relative to the row's reference (queries prescaled, -m_ref where the accumulators start).
        const bool masked = tok + TOK > limit_min || !valid_row;                 // (uniform up to the row validity)
        if (masked) {
#pragma unroll
            for (int sb = 0; sb < SBN; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    s_acc[sb][i] = tok + 32 * sb + 16 * (i >> 3) + 8 * hg + (i & 7) < limit ? s_acc[sb][i] : -INFINITY;
        }
        bf16x8 pb[PG];
        float psum;
        auto weights = [&]() {
            psum = 0.f;
#pragma unroll
            for (int sb = 0; sb < SBN; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(s_acc[sb][i]);
                    psum += p;
                    pb[2 * sb + (i >> 3)][i & 7] = (__bf16)p;
                }
        };
        // No running maximum: the reference only moves when a row has none yet, or when a step's weights say that
        // the scores have risen far above it (their sum beyond 2^24, overflow included).
        bool slow = __any(!has_ref && limit > tok);
        if (!slow) {
            weights();
            slow = __any(!(psum <= kRise));
        }
        if (slow) {
            // out of line: move the reference of the rows that need it (a row lives in lanes n and n + 32)
            float mx = -INFINITY;
#pragma unroll
            for (int sb = 0; sb < SBN; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s_acc[sb][i]);
            const float rise = fmaxf(mx, __shfl_xor(mx, 32));
            const bool move = has_ref ? rise > 0.f : rise > -INFINITY;
            const float shift = move ? rise : 0.f;
            const float alpha = has_ref ? __builtin_amdgcn_exp2f(-shift) : 1.f;
#pragma unroll
            for (int sb = 0; sb < SBN; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s_acc[sb][i] -= shift;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
            m_ref += shift;
            has_ref = has_ref || move;
            weights();
        }
        // the last score block is where the next step's accumulators start: -m_ref again
#pragma unroll
        for (int i = 0; i < 16; ++i) s_acc[SBN - 1][i] = -m_ref;
        l_run += psum;
        if (tok + TOK > len) {                                                   // (uniform) the step that holds the end of the cache
            // slots past the visible length may hold anything (0 x NaN): remove them by bit mask
#pragma unroll
            for (int t4 = 0; t4 < PG; ++t4) {
                u32x4 keep;
                const int first = tok + 16 * t4 + 8 * hg;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    keep[e] = (first + 2 * e < len ? 0x0000ffffu : 0u) | (first + 2 * e + 1 < len ? 0xffff0000u : 0u);
#pragma unroll
                for (int db = 0; db < DB; ++db) fv[t4 * DB + db] &= keep;
            }
        }
#pragma unroll
        for (int t4 = 0; t4 < PG; ++t4)
#pragma unroll
            for (int db = 0; db < DB; ++db)
                o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fv[t4 * DB + db]), pb[t4], o_acc[db], 0, 0, 0);
    }
    wait_vmcnt<0>();
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!valid_row || !wave_works) return;
    const int64_t slot = (((int64_t(b) * a.n_kv_heads + h) * a.row_blocks + rb) * a.ncs + c) * 32 + n;
    float* po = a.part_o + slot * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = o_acc[db][4 * q4 + e];
            *reinterpret_cast<f32x4*>(po + 32 * db + 8 * q4 + 4 * hg) = o4;
        }
    if (hg == 0) {
        a.part_ml[slot * 2] = has_ref ? m_ref : -INFINITY;
        a.part_ml[slot * 2 + 1] = l_tot;
    }
}

// Merge for the source-chunk prefill: one wave per (sequence, query token, query head).
template <int D>
__global__ __launch_bounds__(64) void chunk_combine_kernel(DecodeArgs a, uint16_t* __restrict__ out,
                                                           float* __restrict__ lse) {
    constexpr int PER = D / 64;
    constexpr int BATCH = 8;                         // partial rows fetched per round trip (units are long: few partials per row)
    const int lane = threadIdx.x;
    const int hq = int(blockIdx.x % unsigned(a.n_q_heads));
    const int t = int((blockIdx.x / unsigned(a.n_q_heads)) % unsigned(a.max_new));
    const int b = int(blockIdx.x / unsigned(a.n_q_heads * a.max_new));
    const int len = min(max(a.src_len[b], 0), a.src.max_pages * kPage);
    const int q_len = min(min(max(a.n_new ? a.n_new[b] : a.max_new, 0), a.max_new), len);
    if (t >= q_len) return;                          // rows past n_new[b] are left untouched
    const int h = hq / a.group;
    const int r = t * a.group + hq % a.group, rb = r / 32, n = r % 32;
    const int last_t = min(q_len - 1, (rb * 32 + 31) / a.group);
    const int unit_size = chunk_units(len, a.chunk).size;
    const int n_tot = min((len - q_len + last_t + 1 + unit_size - 1) / unit_size, a.ncs);   // units the split kernel wrote for this block
    const int64_t base = ((int64_t(b) * a.n_kv_heads + h) * a.row_blocks + rb) * a.ncs;

    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;
    float den = 0.f, m_run = -INFINITY;
    for (int i0 = 0; i0 < n_tot; i0 += BATCH) {
        const int cnt = min(BATCH, n_tot - i0);
        float m_mine = -INFINITY, l_mine = 0.f;
        if (lane < cnt) {
            const f32x2 ml = *reinterpret_cast<const f32x2*>(a.part_ml + ((base + i0 + lane) * 32 + n) * 2);
            m_mine = ml[0];
            l_mine = ml[1];
        }
        float rows[BATCH][PER];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const float* po = a.part_o + ((base + i0 + min(u, cnt - 1)) * 32 + n) * D + lane * PER;
#pragma unroll
            for (int e = 0; e < PER; ++e) rows[u][e] = po[e];
        }
        float bm = m_mine;
        for (int o = 32; o > 0; o >>= 1) bm = fmaxf(bm, __shfl_xor(bm, o));
        const float m_new = fmaxf(m_run, bm);
        if (m_new == -INFINITY) continue;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        const float w_mine = __builtin_amdgcn_exp2f(m_mine - m_new);
        float wl = w_mine * l_mine;
        for (int o = 32; o > 0; o >>= 1) wl += __shfl_xor(wl, o);
        den = den * alpha + wl;
#pragma unroll
        for (int e = 0; e < PER; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const float w = __shfl(w_mine, u);
#pragma unroll
            for (int e = 0; e < PER; ++e) acc[e] = fmaf(w, rows[u][e], acc[e]);
        }
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    uint16_t* op = out + ((int64_t(b) * a.max_new + t) * a.n_q_heads + hq) * D + lane * PER;
#pragma unroll
    for (int e = 0; e < PER; ++e) op[e] = f32_to_bf16_bits(acc[e] * inv);
    if (lse && lane == 0)
        lse[(int64_t(b) * a.max_new + t) * a.n_q_heads + hq] = den > 0.f ? (m_run + __builtin_amdgcn_logf(den)) * kLn2 : -INFINITY;
}

static inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
static inline int chunks_of(int len) { return (len + kChunk - 1) / kChunk; }

// Partial results of a decode step cut into `unit`-token work units.
static inline size_t decode_partial_bytes(int unit, int64_t batch, int hkv, int rows, int d, int max_src, int max_rsn) {
    const size_t nc = size_t((max_src + unit - 1) / unit) + size_t((max_rsn + unit - 1) / unit) + 1;   // + the appended token's slot
    const size_t slots = size_t(batch) * hkv * nc * rows;
    return align256(slots * d * sizeof(float)) + align256(slots * 2 * sizeof(float)) + 256;
}
// Tokens per work unit of the one-wave decode kernels (<= 16 query rows): a wave walks its unit serially, one
// memory round trip per 32 tokens, so the unit is as long as still leaves enough units -- 1024 tokens when that
// gives four thousand (fewest partial results; measured best on 64 streams of 36 layers), else 512 if that gives a
// thousand (measured best on configs[2]: 32 streams), down to 128 for a few sequences, where the step is bound by
// that serial walk and not by bandwidth.
static inline int decode_unit_tokens(int64_t batch, int hkv, int rows, int max_src, int max_rsn, int pinned, bool fp8 = false) {
    if (rows > 16) return kChunk;
    if (pinned) return pinned;               // the caller's choice (st_dual_lens::unit_tokens)
    auto units = [&](int unit) { return batch * hkv * ((max_src + unit - 1) / unit + (max_rsn + unit - 1) / unit); };
    // (counted with the length BOUNDS: about half are real; the 8-bit kernel, which walks 64 tokens per step and
    // keeps four waves per SIMD, is best with the long unit from a thousand on)
    if (units(kChunkLong) >= (fp8 ? 1024 : 4096)) return kChunkLong;
    int unit = kChunk;
    while (unit > kChunkMin && units(unit) < 1024) unit /= 2;
    return unit;
}

}  // namespace st

using namespace st;

static inline bool valid_unit(int tokens) { return tokens == 0 || tokens == 128 || tokens == 256 || tokens == 512 || tokens == 1024; }

extern "C" size_t st_decode_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                            int32_t q_len, int32_t max_src_len, int32_t max_rsn_len, int32_t unit_tokens) {
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || q_len <= 0 || head_dim <= 0 || max_src_len < 0 || max_rsn_len < 0 ||
        !valid_unit(unit_tokens))
        return 0;
    const int rows = q_len * (n_q_heads / n_kv_heads);
    // enough for 512-token units whatever the bounds of a later call, and for the unit this very call would use
    const size_t base = decode_partial_bytes(kChunk, batch, n_kv_heads, rows, head_dim, max_src_len, max_rsn_len);
    const int unit = decode_unit_tokens(batch, n_kv_heads, rows, max_src_len, max_rsn_len, unit_tokens);
    const size_t own = decode_partial_bytes(unit, batch, n_kv_heads, rows, head_dim, max_src_len, max_rsn_len);
    return base > own ? base : own;
}

// ---- the decode step for callers that cannot allocate: partial results in a device array of the library ----
// One copy of `scratch` exists on every GPU the library's code object is loaded on, at an address of its own; in host
// code the array's NAME is only a stand-in for it, so its device address is looked up once per device
// (hipGetSymbolAddress, with that device current) and only that pointer is ever handed to kernels.
constexpr size_t kStaticScratchBytes = size_t(64) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

// Device address of `scratch` on the CURRENT device (looked up at the first call on that device).
static st_status static_scratch(void** ptr) {
    int dev = -1;
    ST_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual_static: device index %d (0 .. %d)", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        ST_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return fail(ST_ERR_RUNTIME, "st_attn_decode_dual_static: bad address of the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return ST_OK;
}

static st_status decode_dual_impl(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                  const st_dual_lens* lens, int32_t batch, int32_t n_q_heads, float scale, bool rotate,
                                  double theta_base, void* workspace, size_t workspace_bytes, void* hip_stream,
                                  const void* k_new = nullptr, const void* v_new = nullptr, bool append = false, bool no_alloc = false) {
    if (!out || !q || !caches || !lens) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: null pointer");
    if (append) {
        if (!k_new || !v_new) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_append: null pointer");
        if (!aligned16(k_new) || !aligned16(v_new)) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_append: k_new / v_new must be 16-byte aligned");
        if (lens->q_len != 1) return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual_append: one token per step (q_len %d)", lens->q_len);
        if (caches->source.dtype != ST_BF16 || caches->reasoning.dtype != ST_BF16)
            return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual_append: bf16 caches only");
        if (!caches->reasoning.appended_len) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_append: appended_len is null");
    }
    if (!lens->src_visible_len || !lens->rsn_len) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: null length vector");
    if (!aligned16(out) || !aligned16(q)) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: q / out must be 16-byte aligned");
    st_status r = check_cache(caches->source, "st_attn_decode_dual", "source", true);
    if (r != ST_OK) return r;
    r = check_cache(caches->reasoning, "st_attn_decode_dual", "reasoning", true);
    if (r != ST_OK) return r;
    const st_kv_cache& cs = caches->source;
    const st_kv_cache& cr = caches->reasoning;
    if (cs.n_kv_heads != cr.n_kv_heads || cs.head_dim != cr.head_dim)
        return fail(ST_ERR_SHAPE, "st_attn_decode_dual: the two caches differ in head geometry");
    if (cs.dtype != cr.dtype) return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual: the two caches differ in dtype");
    const bool fp8 = cs.dtype == ST_FP8_E4M3;
    const int hkv = cs.n_kv_heads, d = cs.head_dim;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % hkv != 0)
        return fail(ST_ERR_SHAPE, "st_attn_decode_dual: n_q_heads %d must be a positive multiple of n_kv_heads %d", n_q_heads, hkv);
    const int group = n_q_heads / hkv;
    if (lens->q_len <= 0 || lens->q_len * group > 32)
        return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual: q_len %d x group %d must be in 1..32", lens->q_len, group);
    if (fp8 && lens->q_len * group > 16)
        return fail(ST_ERR_UNSUPPORTED, "st_attn_decode_dual: 8-bit caches take q_len %d x group %d up to 16", lens->q_len, group);
    if (lens->max_src_len < 0 || lens->max_rsn_len < 0) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: negative length bound");
    if (!valid_unit(lens->unit_tokens)) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: unit_tokens %d (0, 128, 256, 512 or 1024)", lens->unit_tokens);
    if (int64_t(lens->max_src_len) > int64_t(cs.max_pages_per_seq) * kPage || int64_t(lens->max_rsn_len) > int64_t(cr.max_pages_per_seq) * kPage)
        return fail(ST_ERR_CAPACITY, "st_attn_decode_dual: length bound exceeds the page table");
    const size_t need = decode_partial_bytes(kChunk, batch, hkv, lens->q_len * group, d, lens->max_src_len, lens->max_rsn_len);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual: workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < need) return fail(ST_ERR_CAPACITY, "st_attn_decode_dual: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    if (scale <= 0.f) scale = 1.f / sqrtf(float(d));

    DecodeArgs a;
    a.src = cache_view(cs);
    a.rsn = cache_view(cr);
    a.src_len = lens->src_visible_len;
    a.rsn_len = lens->rsn_len;
    a.q = static_cast<const uint16_t*>(q);
    a.batch = batch;
    a.q_len = lens->q_len;
    a.n_q_heads = n_q_heads;
    a.n_kv_heads = hkv;
    a.group = group;
    a.rows = lens->q_len * group;
    // Work unit: see decode_unit_tokens; a workspace sized for other length bounds may only hold longer units.
    a.chunk = decode_unit_tokens(batch, hkv, a.rows, lens->max_src_len, lens->max_rsn_len, lens->unit_tokens, fp8);
    while (a.chunk < kChunk && decode_partial_bytes(a.chunk, batch, hkv, a.rows, d, lens->max_src_len, lens->max_rsn_len) > workspace_bytes)
        a.chunk *= 2;
    a.ncs = (lens->max_src_len + a.chunk - 1) / a.chunk;
    a.ncr = (lens->max_rsn_len + a.chunk - 1) / a.chunk;
    a.scale_log2 = scale * kLog2e;
    a.n_new = nullptr;
    a.max_new = lens->q_len;
    a.row_blocks = 1;
    a.rope = rotate ? 1 : 0;
    a.freq = rotate ? make_rope_freq(theta_base, d) : RopeFreq{};
    // long caches: the one-wave split kernel stores the token itself (one more slot per sequence and head); the
    // 32-row kernel does not, the token then goes in with a launch of its own
    const bool fuse_token = append && !fp8 && a.rows <= 16;
    a.append = fuse_token ? 1 : 0;
    a.k_new = static_cast<const uint16_t*>(k_new);
    a.v_new = static_cast<const uint16_t*>(v_new);
    {
        const WaveTrace wt = no_alloc ? WaveTrace{nullptr, 0} : prof_wave_trace();
        a.trace = wt.buf;
        a.trace_cap = wt.capacity;
    }
    const size_t slots = size_t(batch) * hkv * size_t(a.ncs + a.ncr + a.append) * a.rows;
    a.part_o = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + align256(slots * d * sizeof(float)));

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // Short caches: one wave per (sequence, KV head) does everything (no partials, no merge launch) -- when the
    // serial walk of both caches is short and there are too few sequences for the split to pay anyway.
    if (!fp8 && a.rows <= 16 && lens->max_src_len + lens->max_rsn_len <= kSmallDecodeTokens && int64_t(batch) * hkv <= 0x7fffffff) {
        const size_t smem = (size_t(kSmallWaves + (append ? 1 : 0)) * a.rows * (d + 2) + d) * sizeof(float);
        auto launch = [&](auto kernel) -> st_status {
            if (smem > 64 * 1024)                       // beyond the default limit (16 rows of 128 dims only)
                ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
            hipLaunchKernelGGL(kernel, dim3((unsigned)(batch * hkv)), dim3(64 * kSmallWaves), smem, s, a, static_cast<uint16_t*>(out), lse,
                               static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new));
            return ST_OK;
        };
        const st_status lr = d == 64 ? (append ? launch(decode_small16_kernel<64, true>) : launch(decode_small16_kernel<64, false>))
                                     : (append ? launch(decode_small16_kernel<128, true>) : launch(decode_small16_kernel<128, false>));
        if (lr != ST_OK) return lr;
        ST_LAUNCH_CHECK("decode_small16_kernel");
        return ST_OK;
    }
    if (append && !fuse_token) {
        // the token goes in with a launch of its own, then the step below reads it like any other
        const st_status ar = append_token_at(cr, k_new, v_new, lens->rsn_len, batch, rotate, theta_base, s);
        if (ar != ST_OK) return ar;
    }
    const int64_t units = int64_t(batch) * hkv * (a.ncs + a.ncr + a.append);
    const int64_t out_units = int64_t(batch) * a.q_len * n_q_heads;
    if (units / 4 + 1 > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_decode_dual: grid too large");
    if (units > 0) {
        const dim3 grid((unsigned)((units + 3) / 4)), block(256);
        if (a.rows <= 16) {
            if (units > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_decode_dual: grid too large");
            if (!no_alloc) prof_begin(kProfDecodeSplit, s);      // (the timing hooks create events)
            for (int rep = 0, n_rep = no_alloc ? 1 : prof_repeat(); rep < n_rep; ++rep)
            if (fp8) {
                if (d == 64) hipLaunchKernelGGL((decode_split16_fp8_kernel<64>), dim3((unsigned)units), dim3(64), 0, s, a);
                else hipLaunchKernelGGL((decode_split16_fp8_kernel<128>), dim3((unsigned)units), dim3(64), 0, s, a);
            } else {
                // (bytes of the launch from the length bounds: about half are real)
                const double bound_bytes = double(batch) * hkv * (double(lens->max_src_len) + lens->max_rsn_len) * 4.0 * d;
                const bool stream_keys = bound_bytes <= 4.0e9;
                if (d == 64) {
                    if (stream_keys) hipLaunchKernelGGL((decode_split16_kernel<64, true>), dim3((unsigned)units), dim3(64), 0, s, a);
                    else hipLaunchKernelGGL((decode_split16_kernel<64, false>), dim3((unsigned)units), dim3(64), 0, s, a);
                } else {
                    if (stream_keys) hipLaunchKernelGGL((decode_split16_kernel<128, true>), dim3((unsigned)units), dim3(64), 0, s, a);
                    else hipLaunchKernelGGL((decode_split16_kernel<128, false>), dim3((unsigned)units), dim3(64), 0, s, a);
                }
            }
            if (!no_alloc) prof_end(kProfDecodeSplit, s);
        } else {
            if (d == 64) hipLaunchKernelGGL((decode_split_kernel<64>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((decode_split_kernel<128>), grid, block, 0, s, a);
        }
        ST_LAUNCH_CHECK("decode_split_kernel");
    }
    if (out_units > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_decode_dual: grid too large");
    if (d == 64)
        hipLaunchKernelGGL((decode_combine_kernel<64>), dim3((unsigned)out_units), dim3(64), 0, s, a,
                           static_cast<uint16_t*>(out), lse);
    else
        hipLaunchKernelGGL((decode_combine_kernel<128>), dim3((unsigned)out_units), dim3(64), 0, s, a,
                           static_cast<uint16_t*>(out), lse);
    ST_LAUNCH_CHECK("decode_combine_kernel");
    return ST_OK;
}

extern "C" st_status st_attn_decode_dual(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                         const st_dual_lens* lens, int32_t batch, int32_t n_q_heads, float scale,
                                         void* workspace, size_t workspace_bytes, void* hip_stream) {
    return decode_dual_impl(out, lse, q, caches, lens, batch, n_q_heads, scale, false, 0.0, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t st_decode_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" st_status st_attn_decode_dual_static(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                                const st_dual_lens* lens, int32_t batch, int32_t n_q_heads, float scale,
                                                void* hip_stream) {
    if (!caches || !lens) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_static: null pointer");
    const int hkv = caches->source.n_kv_heads, d = caches->source.head_dim;
    if (batch <= 0 || n_q_heads <= 0 || hkv <= 0 || d <= 0 || n_q_heads % hkv != 0 || lens->q_len <= 0 || lens->max_src_len < 0 || lens->max_rsn_len < 0)
        return fail(ST_ERR_SHAPE, "st_attn_decode_dual_static: bad sizes");
    // what st_attn_decode_dual asks of a workspace for these bounds (partials of 512-token units) must fit the array
    const size_t need = decode_partial_bytes(kChunk, batch, hkv, lens->q_len * (n_q_heads / hkv), d, lens->max_src_len, lens->max_rsn_len);
    if (need > kStaticScratchBytes)
        return fail(ST_ERR_CAPACITY, "st_attn_decode_dual_static: the step needs %zu bytes of partial results, the library's array holds %zu; use st_attn_decode_dual with a workspace", need, kStaticScratchBytes);
    void* ws = nullptr;
    const st_status r = static_scratch(&ws);
    if (r != ST_OK) return r;
    // Nothing in the array has to start at zero: the split kernel writes every partial the merge kernel reads in the
    // same call (both walk the same units of the same lengths), so what an earlier call left is never looked at.
    return decode_dual_impl(out, lse, q, caches, lens, batch, n_q_heads, scale, false, 0.0, ws, kStaticScratchBytes, hip_stream,
                            nullptr, nullptr, false, /*no_alloc=*/true);
}

extern "C" st_status st_attn_decode_dual_rope(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                              const st_dual_lens* lens, int32_t batch, int32_t n_q_heads, float scale,
                                              double theta_base, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!(theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_rope: theta_base must be positive");
    return decode_dual_impl(out, lse, q, caches, lens, batch, n_q_heads, scale, true, theta_base, workspace, workspace_bytes,
                            hip_stream);
}

extern "C" st_status st_attn_decode_dual_append(void* out, float* lse, const void* q, const void* k_new, const void* v_new,
                                                const st_dual_cache* caches, const st_dual_lens* lens, int32_t batch,
                                                int32_t n_q_heads, float scale, double theta_base, void* workspace,
                                                size_t workspace_bytes, void* hip_stream) {
    if (theta_base < 0.0 || theta_base != theta_base) return fail(ST_ERR_INVALID_ARG, "st_attn_decode_dual_append: theta_base must be positive, or 0 for rotated inputs");
    return decode_dual_impl(out, lse, q, caches, lens, batch, n_q_heads, scale, theta_base > 0.0, theta_base, workspace, workspace_bytes,
                            hip_stream, k_new, v_new, true);
}

extern "C" size_t st_source_chunk_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                                  int32_t max_new, int32_t max_src_len) {
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || max_new <= 0 || max_src_len < 0) return 0;
    const size_t rb = (size_t(max_new) * (n_q_heads / n_kv_heads) + 31) / 32;
    const size_t slots = size_t(batch) * n_kv_heads * rb * size_t(chunks_of(max_src_len)) * 32;
    return align256(slots * head_dim * sizeof(float)) + align256(slots * 2 * sizeof(float)) + 256;
}

static st_status source_chunk_impl(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                   const int32_t* src_len, const int32_t* n_new, int32_t max_new,
                                   int32_t max_src_len, int32_t batch, int32_t n_q_heads, float scale, bool rotate,
                                   double theta_base, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out || !q || !caches || !src_len) return fail(ST_ERR_INVALID_ARG, "st_attn_source_chunk: null pointer");
    if (!aligned16(out) || !aligned16(q)) return fail(ST_ERR_INVALID_ARG, "st_attn_source_chunk: q / out must be 16-byte aligned");
    st_status r = check_cache(caches->source, "st_attn_source_chunk", "source");
    if (r != ST_OK) return r;
    const st_kv_cache& cs = caches->source;
    const int hkv = cs.n_kv_heads, d = cs.head_dim;
    if (batch <= 0 || n_q_heads <= 0 || n_q_heads % hkv != 0)
        return fail(ST_ERR_SHAPE, "st_attn_source_chunk: n_q_heads %d must be a positive multiple of n_kv_heads %d", n_q_heads, hkv);
    if (max_new <= 0 || max_src_len < 0) return fail(ST_ERR_INVALID_ARG, "st_attn_source_chunk: bad sizes");
    if (int64_t(max_src_len) > int64_t(cs.max_pages_per_seq) * kPage)
        return fail(ST_ERR_CAPACITY, "st_attn_source_chunk: length bound exceeds the page table");
    const size_t need = st_source_chunk_workspace_bytes(batch, n_q_heads, hkv, d, max_new, max_src_len);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ST_ERR_INVALID_ARG, "st_attn_source_chunk: workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < need) return fail(ST_ERR_CAPACITY, "st_attn_source_chunk: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    if (scale <= 0.f) scale = 1.f / sqrtf(float(d));

    DecodeArgs a;
    a.src = cache_view(cs);
    a.rsn = a.src;                       // unused: there are no reasoning chunk slots
    a.src_len = src_len;
    a.rsn_len = src_len;
    a.q = static_cast<const uint16_t*>(q);
    a.batch = batch;
    a.q_len = max_new;
    a.n_q_heads = n_q_heads;
    a.n_kv_heads = hkv;
    a.group = n_q_heads / hkv;
    a.rows = 32;
    // Work unit: 512 tokens of the cache; longer ones when that still leaves a thousand workgroups or more --
    // a unit's partial result (128 rows x D floats) is written and merged once per unit.  (The workspace is
    // sized for the smallest unit.)
    a.chunk = kChunk;
    {
        const int64_t groups = int64_t(batch) * hkv * ((int64_t(max_new) * (n_q_heads / hkv) + 127) / 128);
        for (int unit = 8 * kChunk; unit > kChunk; unit /= 2)
            if (groups * ((max_src_len + unit - 1) / unit) >= 1024) {
                a.chunk = unit;
                break;
            }
    }
    a.ncs = (max_src_len + a.chunk - 1) / a.chunk;
    a.ncr = 0;
    a.append = 0;
    a.k_new = a.v_new = nullptr;
    a.trace = nullptr;
    a.trace_cap = 0;
    a.scale_log2 = scale * kLog2e;
    a.n_new = n_new;
    a.max_new = max_new;
    a.row_blocks = (max_new * a.group + 31) / 32;
    a.rope = rotate ? 1 : 0;
    a.freq = rotate ? make_rope_freq(theta_base, d) : RopeFreq{};
    const size_t slots = size_t(batch) * hkv * a.row_blocks * size_t(a.ncs) * 32;
    a.part_o = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + align256(slots * d * sizeof(float)));

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t units = int64_t(batch) * hkv * a.row_blocks * a.ncs;
    const int64_t out_units = int64_t(batch) * max_new * n_q_heads;
    if (units / 4 + 1 > 0x7fffffff || out_units > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_source_chunk: grid too large");
    if (units > 0) {
        const int64_t wgs = int64_t(batch) * hkv * ((a.row_blocks + 3) / 4) * a.ncs;
        auto launch = [&](auto dtag) -> st_status {
            constexpr int HD = decltype(dtag)::value;
            constexpr int STAGES = 2, TOK = 64;      // (measured: three to five stages of 32 tokens, or four of 64 with one workgroup per compute unit, are no faster)
            const size_t smem = sizeof(ChunkSmem<HD, STAGES, TOK>);
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&chunk_split_lds_kernel<HD, STAGES, TOK>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
            prof_begin(kProfSourceChunk, s);
            for (int rep = 0; rep < prof_repeat(); ++rep)
                hipLaunchKernelGGL((chunk_split_lds_kernel<HD, STAGES, TOK>), dim3((unsigned)wgs), dim3(256), smem, s, a);
            prof_end(kProfSourceChunk, s);
            return ST_OK;
        };
        const st_status lr = d == 64 ? launch(std::integral_constant<int, 64>{}) : launch(std::integral_constant<int, 128>{});
        if (lr != ST_OK) return lr;
        ST_LAUNCH_CHECK("chunk_split_lds_kernel");
    }
    if (d == 64) hipLaunchKernelGGL((chunk_combine_kernel<64>), dim3((unsigned)out_units), dim3(64), 0, s, a, static_cast<uint16_t*>(out), lse);
    else hipLaunchKernelGGL((chunk_combine_kernel<128>), dim3((unsigned)out_units), dim3(64), 0, s, a, static_cast<uint16_t*>(out), lse);
    ST_LAUNCH_CHECK("chunk_combine_kernel");
    return ST_OK;
}

extern "C" st_status st_attn_source_chunk(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                          const int32_t* src_len, const int32_t* n_new, int32_t max_new,
                                          int32_t max_src_len, int32_t batch, int32_t n_q_heads, float scale,
                                          void* workspace, size_t workspace_bytes, void* hip_stream) {
    return source_chunk_impl(out, lse, q, caches, src_len, n_new, max_new, max_src_len, batch, n_q_heads, scale, false, 0.0,
                             workspace, workspace_bytes, hip_stream);
}

extern "C" st_status st_attn_source_chunk_rope(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                               const int32_t* src_len, const int32_t* n_new, int32_t max_new,
                                               int32_t max_src_len, int32_t batch, int32_t n_q_heads, float scale,
                                               double theta_base, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!(theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "st_attn_source_chunk_rope: theta_base must be positive");
    return source_chunk_impl(out, lse, q, caches, src_len, n_new, max_new, max_src_len, batch, n_q_heads, scale, true, theta_base,
                             workspace, workspace_bytes, hip_stream);
}
