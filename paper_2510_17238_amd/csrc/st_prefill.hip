// Streaming-mask prefill attention (Sec. 3.2, "Streaming Attention Mask Matrix", Eq. 2).
//
// The dense additive mask of Eq. 2 never exists here.  Work is cut into query tiles
// of one stream of one sequence (st::WorkItem), and each item walks two runs of key
// tiles in stream-compact coordinates:
//   block A -- causal over the row's own stream (source x source, or reasoning x
//              reasoning),
//   block B -- for reasoning rows, the prefix of the source stream they may see.
// Inside a run, tiles [0, full) need no mask, tiles [full, total) compare the column
// index with a per-row limit, tiles past `total` are never read.
//
// Kernels:
//   tile_pack_kernel   bf16, O(N) bytes: gathers the K rows and the TRANSPOSED V rows of every
//                         64-row key tile (stream-compact order) into contiguous 16 KB blocks, so
//                         that the attention kernel streams tiles with plain linear loads and needs
//                         no per-row token lookup and no transpose in its inner loop.
//   prefill_attn_kernel<D, NH, ROPE>
//                         bf16, 4 waves x 32 query rows x NH query heads (1 or 2) of one KV head; K and V^T
//                         tiles copied asynchronously into swizzled LDS buffers; QK^T and PV on
//                         v_mfma_f32_32x32x16_bf16, fp32 softmax state.  Both products are computed
//                         TRANSPOSED (S^T = K Q^T, O^T = V^T P^T): a lane then owns one query row, so a
//                         row sum is an in-register reduction plus one exchange with lane^32, and the S^T
//                         accumulators are already laid out as the B operand of the second product.  The
//                         loop is software-pipelined by hand (see the kernel).
//   rope_table_kernel, tile_pack_rope_kernel
//                         the fused rotation of st_attn_prefill_rope: (cos, sin) of every token once, keys rotated
//                         on their way into the key tiles; the attention kernel's ROPE form rotates its query rows.
//   prefill_simple_kernel any dtype, one thread per query row, plain fp32 arithmetic.  It is
//                         the fp32 path (tolerance 1e-4) and walks the same work items.
#include <type_traits>

#include "st_tiles.h"

namespace st {

struct ItemGeom {
    int S;           // source tokens
    int n_stream;    // tokens of the row's own stream
    int a_base;      // compact row of column 0 of block A
    int b_base;      // compact row of column 0 of block B (the source stream)
};

__device__ __forceinline__ ItemGeom item_geom(const PlanView&, const WorkItem& it) {
    return ItemGeom{it.n_src, it.n_stream, it.a_base, it.b_base};
}

// --------------------------------------------------------------------------
// Plain kernel: one thread per query row.
// --------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float load_f32(const T* p);
template <>
__device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_f32<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void store_f32(T* p, float x);
template <>
__device__ __forceinline__ void store_f32<float>(float* p, float x) { *p = x; }
template <>
__device__ __forceinline__ void store_f32<uint16_t>(uint16_t* p, float x) { *p = f32_to_bf16_bits(x); }

template <typename T, int D>
__global__ __launch_bounds__(kTileM) void prefill_simple_kernel(T* __restrict__ out, float* __restrict__ lse,
                                                               const T* __restrict__ q, const T* __restrict__ k,
                                                               const T* __restrict__ v, PlanView pv, int n_q_heads,
                                                               int n_kv_heads, float scale) {
    constexpr int CH = 16;  // keys per softmax update
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float (*s_q)[D + 1] = reinterpret_cast<float (*)[D + 1]>(smem_raw);
    const int rank = blockIdx.x / n_q_heads;
    const int hq = blockIdx.x % n_q_heads;
    const int hk = hq / (n_q_heads / n_kv_heads);
    const WorkItem it = pv.sorted[rank];
    if (it.n_rows == 0) return;
    const ItemGeom g = item_geom(pv, it);
    const int r = threadIdx.x;
    const bool active = r < it.n_rows;
    const int my_row = it.row0 + min(r, it.n_rows - 1);        // relative to the row's stream
    const int tok_q = pv.perm[g.a_base + my_row];
    for (int d = 0; d < D; ++d) s_q[r][d] = load_f32(q + (int64_t(tok_q) * n_q_heads + hq) * D + d);
    const int my_vis = pv.vis[g.a_base + my_row];

    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int n_tiles = it.a_total + it.b_total;
    for (int ti = 0; ti < n_tiles; ++ti) {
        const bool in_a = ti < it.a_total;
        const int kt = in_a ? ti : ti - it.a_total;
        const bool partial = kt >= (in_a ? it.a_full : it.b_full);
        const int base = in_a ? g.a_base : g.b_base;
        const int n_cols = in_a ? g.n_stream : g.S;
        const int limit = in_a ? my_row + 1 : my_vis;          // columns < limit are visible
        const int c_end = min((kt + 1) * kTileN, n_cols);
        for (int c0 = kt * kTileN; c0 < c_end; c0 += CH) {
            float s[CH];
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int col = c0 + u;
                s[u] = -INFINITY;
                if (col < c_end) {
                    const int tok_k = pv.perm[base + col];
                    const T* kp = k + (int64_t(tok_k) * n_kv_heads + hk) * D;
                    float acc = 0.f;
                    for (int d = 0; d < D; ++d) acc = fmaf(s_q[r][d], load_f32(kp + d), acc);
                    if (!partial || col < limit) s[u] = acc * scale;
                }
                mx = fmaxf(mx, s[u]);
            }
            if (mx == -INFINITY) continue;
            const float m_new = fmaxf(m_run, mx);
            const float alpha = expf(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int d = 0; d < D; ++d) o[d] *= alpha;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int col = c0 + u;
                if (col < c_end && s[u] != -INFINITY) {
                    const float p = expf(s[u] - m_new);
                    l_run += p;
                    const int tok_k = pv.perm[base + col];
                    const T* vp = v + (int64_t(tok_k) * n_kv_heads + hk) * D;
#pragma unroll
                    for (int d = 0; d < D; ++d) o[d] = fmaf(p, load_f32(vp + d), o[d]);
                }
            }
            m_run = m_new;
        }
    }
    if (!active) return;
    const float inv = 1.f / l_run;
    T* op = out + (int64_t(tok_q) * n_q_heads + hq) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) store_f32(op + d, o[d] * inv);
    if (lse) lse[int64_t(tok_q) * n_q_heads + hq] = m_run + logf(l_run);
}

// --------------------------------------------------------------------------
// MFMA kernel (bf16): NH = 1 or 2 query heads of one KV head per workgroup.
// --------------------------------------------------------------------------
// Every wave owns 32 query rows of a work item for NH query heads that share a KV head.
//   NH = 2  A K (or V^T) operand fragment read from LDS feeds two MFMAs and one tile copied into LDS
//           serves twice the arithmetic: LDS read traffic and L2 -> LDS copy traffic per flop are both
//           halved.  The price is registers (two output accumulators, two score blocks, two Q operands:
//           about 440 per lane, the output accumulators in accumulation registers), so one wave per SIMD;
//           three K and three V^T buffers (96 KB), copies two tiles ahead.
//   NH = 1  fits the ordinary vector registers twice per SIMD: two workgroups per CU, two buffers each
//           (64 KB), copies one tile ahead.
// Either way a wave cannot count on other waves to fill the matrix pipe while it does its softmax, so
// the loop is software-pipelined by hand, in the exact instruction order wanted:
//   phase X of tile t:  scores of tile t+1   beside  exp2 / bf16 P / row sum of tile t
//   phase Y of tile t:  O^T += V^T P^T        beside  the moves of tile t+1's scores out of the accumulation registers
// with ONE barrier per key tile.  There is no running maximum of a row (see the list at the kernel): the reference
// exponent m_ref is the row maximum of the first tile and only moves when a tile's weights sum beyond 2^kRiseLog2,
// an out-of-line block.
// Fused rotation (Sec. 3.2), step 1: the (cos, sin) pairs of every packed row -- `tab` [packed tile][64 rows][D/2]
// float2, row r of a stream's tile t at (tile t) * 64 + r -- evaluated ONCE per token (not once per head): the key
// pack below and the attention kernel's query load both rotate with them.  The angle position * theta^(-2i/D) is
// reduced in fp64, cos / sin are fp32 (rope_cos_sin).  One workgroup per packed tile.
template <int D>
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ tab, const int32_t* __restrict__ positions, PlanView pv,
                                                         RopeFreq freq) {
    constexpr int HALF = D / 2;
    const int tile = blockIdx.x;
    const int b = find_seq(pv.pack_base, pv.batch, tile);
    const int lt = tile - pv.pack_base[b];
    const int t0 = pv.cu[b], S = pv.n_src[b], R = pv.cu[b + 1] - t0 - S;
    const int ts = (S + kTileN - 1) / kTileN, tr = (R + kTileN - 1) / kTileN;
    if (lt >= ts + tr) return;                      // spare tile of this sequence: never read
    const bool src = lt < ts;
    const int kt = src ? lt : lt - ts;
    const int base = t0 + (src ? 0 : S) + kt * kTileN;
    const int valid = min(kTileN, (src ? S : R) - kt * kTileN);
    for (int w = threadIdx.x; w < valid * HALF; w += 256) {
        const int row = w / HALF, i = w % HALF;
        float cs, sn;
        rope_cos_sin(positions[pv.perm[base + row]], freq.f[i], &cs, &sn);
        tab[(size_t(tile) * kTileN + row) * HALF + i] = float2{cs, sn};
    }
}

// Step 2: tile_pack_kernel for UNROTATED keys -- every key row is rotated with its table row on its way into the row
// tile.  A thread owns two rows x one pair of 8-dim pieces (dims 8 cp .. + 7 and D/2 + the same).
template <int D>
__global__ __launch_bounds__(256) void tile_pack_rope_kernel(uint16_t* __restrict__ kc, uint16_t* __restrict__ vc,
                                                            const float2* __restrict__ tab, const uint16_t* __restrict__ k,
                                                            const uint16_t* __restrict__ v, PlanView pv, int n_kv_heads) {
    constexpr int KCH = D / 8, CP = KCH / 2;
    constexpr int PER_THREAD = kTileN * CP / 256;
    const int tile = blockIdx.x / n_kv_heads;
    const int h = blockIdx.x % n_kv_heads;
    const int b = find_seq(pv.pack_base, pv.batch, tile);
    const int lt = tile - pv.pack_base[b];
    const int t0 = pv.cu[b], S = pv.n_src[b], R = pv.cu[b + 1] - t0 - S;
    const int ts = (S + kTileN - 1) / kTileN, tr = (R + kTileN - 1) / kTileN;
    if (lt >= ts + tr) return;                      // spare tile of this sequence: never read
    const bool src = lt < ts;
    const int kt = src ? lt : lt - ts;
    const int base = t0 + (src ? 0 : S) + kt * kTileN;
    const int valid = min(kTileN, (src ? S : R) - kt * kTileN);
    const int tid = threadIdx.x;
    const uint32_t row_stride = uint32_t(n_kv_heads) * D;
    uint16_t* kdst = kc + (size_t(h) * pv.pack_tiles + tile) * (kTileN * D);
    uint16_t* vdst = vc + (size_t(h) * pv.pack_tiles + tile) * (kTileN * D);
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const int c = tid + 256 * u;
        const int row = c / CP, cp = c % CP;
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
        if (row < valid) {
            const uint16_t* kr = k + (uint32_t(pv.perm[base + row]) * row_stride + uint32_t(h) * D + cp * 8);
            const u32x4 lo_in = *reinterpret_cast<const u32x4*>(kr), hi_in = *reinterpret_cast<const u32x4*>(kr + D / 2);
            const f32x4* trow = reinterpret_cast<const f32x4*>(tab + (size_t(tile) * kTileN + row) * (D / 2) + cp * 8);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const f32x4 t = trow[w];                                  // (cos, sin) of pairs 2 w and 2 w + 1
                uint32_t out_lo = 0, out_hi = 0;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const float cs = t[2 * half], sn = t[2 * half + 1];
                    const float x = bf16_bits_to_f32(uint16_t(lo_in[w] >> (16 * half))), y = bf16_bits_to_f32(uint16_t(hi_in[w] >> (16 * half)));
                    out_lo |= uint32_t(f32_to_bf16_bits(x * cs - y * sn)) << (16 * half);
                    out_hi |= uint32_t(f32_to_bf16_bits(y * cs + x * sn)) << (16 * half);
                }
                lo[w] = out_lo;
                hi[w] = out_hi;
            }
        }
        const int lr = swap23(row);                                    // row position in the tile
        *reinterpret_cast<u32x4*>(kdst + lr * D + (cp ^ swizzle_key<2 * D>(lr)) * 8) = lo;
        *reinterpret_cast<u32x4*>(kdst + lr * D + ((cp + CP) ^ swizzle_key<2 * D>(lr)) * 8) = hi;
    }
    // V: as in tile_pack_kernel -- 8 keys x 8 d per thread (16-byte loads), transposed in registers to 8 d x 8 keys
    const int kvb = tid & 7, dq = tid >> 3;
    if (dq < D / 8) {
        u32x4 vreg[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int row = kvb * 8 + r;
            vreg[r] = u32x4{0u, 0u, 0u, 0u};
            if (row < valid) vreg[r] = *reinterpret_cast<const u32x4*>(v + (uint32_t(pv.perm[base + row]) * row_stride + uint32_t(h) * D + dq * 8));
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            u32x4 even, odd;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                const uint32_t a = vreg[2 * pr][w], bb = vreg[2 * pr + 1][w];
                even[pr] = __builtin_amdgcn_perm(bb, a, 0x05040100u);   // low halves
                odd[pr] = __builtin_amdgcn_perm(bb, a, 0x07060302u);    // high halves
            }
            const int d0 = dq * 8 + 2 * w;
            *reinterpret_cast<u32x4*>(vdst + d0 * kTileN + (kvb ^ swizzle_key<2 * kTileN>(d0)) * 8) = even;
            *reinterpret_cast<u32x4*>(vdst + (d0 + 1) * kTileN + (kvb ^ swizzle_key<2 * kTileN>(d0 + 1)) * 8) = odd;
        }
    }
}

template <int D, int STAGES>
struct PipeSmem {
    uint16_t k[STAGES][kTileN * D];
    uint16_t vt[STAGES][D * kTileN];
};
// --------------------------------------------------------------------------
// The attention kernel (bf16): NH = 1 or 2 query heads of one KV head per workgroup.
// Every wave owns 32 query rows of a work item for NH query heads that share a KV head.
//   NH = 2  A K (or V^T) operand fragment read from LDS feeds two matrix instructions and one tile copied into
//           LDS serves twice the arithmetic: LDS read traffic and L2 -> LDS copy traffic per flop are both halved.
//           The price is registers (two output accumulators, two score blocks, two Q operands: about 430 per lane,
//           the accumulators in accumulation registers), so one wave per SIMD; three K and three V^T buffers
//           (96 KB), K copied two tiles ahead.
//   NH = 1  fits the ordinary vector registers twice per SIMD: two workgroups per CU, two buffers each (64 KB),
//           copies one tile ahead.
// Either way a wave cannot count on other waves to fill the matrix pipe while it does its softmax, so the loop
// is software-pipelined by hand, in the exact instruction order wanted:
//   phase X of tile t:  scores of tile t+1   beside  exp2 / bf16 P / row sum of tile t
//   phase Y of tile t:  O^T += V^T P^T        beside  the exponents of tile t+1 leaving the accumulation registers
// with ONE barrier per key tile, and the vector work per matrix instruction cut to what one wave can issue beside
// its own matrix instructions: it issues at most one instruction every few cycles; beside a
// v_mfma_f32_32x32x16_bf16 (32 cycles of the matrix pipe) about 3.5 plain vector instructions are free, every
// further one costs about 5 cycles, a ds_read_b128 about 4 and a v_dot2_f32_bf16 about 18 -- it shares the matrix
// pipe (measured on this chip, one wave per SIMD).
//   * The queries are multiplied by scale * log2(e) once, when they are loaded (and rounded to bf16 again), and
//     the first matrix instruction of a score block starts from -m_ref instead of 0: a score leaves the matrix
//     pipe as the base-2 exponent of its probability relative to the row's reference exponent m_ref -- no
//     multiply-add per element.  Between two tiles the -m_ref values are parked in the last score block.
//   * No running maximum.  m_ref is the row maximum of the FIRST tile (every row sees column 0 of its own stream,
//     so it is finite); bf16 and fp32 have the same exponent range, so probabilities may grow far beyond 1 without
//     any loss.  Only when a tile's row sum exceeds 2^kRiseLog2 (or is not finite) -- seen right after the
//     probabilities of that tile were formed, before they are used -- the reference is moved, out of line: the
//     tile's probabilities are formed again, the sum and the output accumulator are rescaled.
//   * The first operand fragments of a phase are read from LDS in the slots of the phase before that need no
//     fragment of their own any more (with three buffers the K tile is known to have landed one tile early), and
//     the copies of the next tiles are issued behind the first matrix instructions instead of in front of them.
//   * The last tile of an item has no scores behind it: it is peeled out of the loop, whose body has no branch
//     around its matrix instructions.
// What was tried on top and did not pay: the first product's matrix instructions placed by hand with their results
// in ordinary vector registers (no move out of the accumulation registers, a third of the vector instructions
// gone): as fast, not faster -- the vector instructions co-execute less often with matrix instructions that use the
// same register file (SQ_VALU_MFMA_COEXEC_CYCLES fell by a quarter); longer LDS rings (tiles requested three or four
// tiles ahead): no change, the copies are not waited for.  Removing the tile copies altogether (wrong results, same
// instruction stream otherwise) makes the kernel 15 % faster through the CLOCK, not through cycles: the chip is
// power-limited under this kernel and the L2 -> LDS traffic is part of the bill; what can be saved of it is saved
// by the order of the work items (see st_plan.hip).
// --------------------------------------------------------------------------
constexpr float kRiseLog2 = 24.f;

template <int D, int NH, bool ROPE>
__global__ __launch_bounds__(256, NH == 2 ? 1 : 2) void prefill_attn_kernel(uint16_t* __restrict__ out, float* __restrict__ lse,
                                                                   const uint16_t* __restrict__ q,
                                                                   const uint16_t* __restrict__ kc,
                                                                   const uint16_t* __restrict__ vc, PlanView pv,
                                                                   int n_q_heads, int n_kv_heads, float scale_log2,
                                                                   const float2* __restrict__ rope_tab) {
    constexpr int KS = D / 16, DB = D / 32, SB = kTileN / 32;
    constexpr int TILE = kTileN * D;
    constexpr int STAGES = NH == 2 ? 3 : 2;
    constexpr bool EARLY_K = STAGES == 3;          // K(t + 2) has landed when tile t starts: its first fragments may be read a phase early
    constexpr int PER = 16 / KS;                   // score elements of vector work per matrix instruction (both phases)
    constexpr int kPF = 3;                         // operand fragments read ahead
    extern __shared__ __align__(16) unsigned char smem_raw[];
    PipeSmem<D, STAGES>& sm = *reinterpret_cast<PipeSmem<D, STAGES>*>(smem_raw);

    const int n_sets = n_q_heads / NH;
    const int rank = blockIdx.x / n_sets;
    const int hh0 = blockIdx.x % n_sets;
    const int group = n_q_heads / n_kv_heads;
    const int hk = hh0 % n_kv_heads;                // consecutive workgroups -> consecutive KV heads
    const int hq0 = hk * group + NH * (hh0 / n_kv_heads);
    const WorkItem it = pv.sorted[rank];
    if (it.n_rows == 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hg = lane >> 5;
    const int n_tiles = it.a_total + it.b_total;

    constexpr int NL = TILE * 2 / 1024 / 4;         // 1 KB copies per wave per tile
    // a copy instruction takes the tile's address from scalar registers and one 32-bit byte offset per lane
    const uint16_t* kc_head = kc + size_t(hk) * pv.pack_tiles * TILE;
    const uint16_t* vc_head = vc + size_t(hk) * pv.pack_tiles * TILE;
    const uint32_t lane_off = uint32_t(wave) * (NL * 1024) + uint32_t(lane) * 16;
    auto tile_of = [&](int ti) {
        ti = min(ti, n_tiles - 1);                   // past the end: fetch the last tile again (never used)
        return ti < it.a_total ? it.tile_a0 + ti : it.tile_b0 + (ti - it.a_total);
    };
    const uint32_t lds_k0 = uint32_t(uintptr_t(&sm.k[0][0])) + uint32_t(wave) * (NL * 1024);
    const uint32_t lds_v0 = uint32_t(uintptr_t(&sm.vt[0][0])) + uint32_t(wave) * (NL * 1024);
    auto issue_k = [&](int ti, int stage) { async_copy_rows<NL>(kc_head + size_t(tile_of(ti)) * TILE, lane_off, lds_k0 + stage * (TILE * 2)); };
    auto issue_v = [&](int ti, int stage) { async_copy_rows<NL>(vc_head + size_t(tile_of(ti)) * TILE, lane_off, lds_v0 + stage * (TILE * 2)); };
    // copy order (tile x lives in buffer x % STAGES):
    //   three buffers: K0 V0 K1 K2 V1 | K3 V2 | K4 V3 | ...   K two tiles ahead, V^T one
    //   two buffers:   K0 V0 K1       | V1 K2 | V2 K3 | ...   one tile ahead
    issue_k(0, 0);
    issue_v(0, 0);
    issue_k(1, 1);
    if (STAGES == 3) {
        issue_k(2, 2);
        issue_v(1, 1);
    }

    const int row_in_tile = wave * 32 + n;
    const bool active = row_in_tile < it.n_rows;
    const int my_row = it.row0 + min(row_in_tile, it.n_rows - 1);
    const int tok_q = pv.perm[it.a_base + my_row];
    const int my_vis = pv.vis[it.a_base + my_row];

    bf16x8 qf[NH][KS];
    {
        const uint16_t* qp = q + (int64_t(tok_q) * n_q_heads + hq0) * D + 8 * hg;
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int j = 0; j < KS; ++j) qf[h][j] = *reinterpret_cast<const bf16x8*>(qp + h * D + 16 * j);
    }
    if (ROPE) {
        const float2* trow = rope_tab + (size_t(it.tile_a0) * kTileN + my_row) * (D / 2) + 8 * hg;
#pragma unroll
        for (int j = 0; j < KS / 2; ++j) {
            f32x4 cs4[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) cs4[w] = *reinterpret_cast<const f32x4*>(trow + 16 * j + 2 * w);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float cs = cs4[e / 2][2 * (e % 2)], sn = cs4[e / 2][2 * (e % 2) + 1];
#pragma unroll
                for (int h = 0; h < NH; ++h) {
                    const float x = float(qf[h][j][e]), y = float(qf[h][j + KS / 2][e]);
                    qf[h][j][e] = (__bf16)(x * cs - y * sn);
                    qf[h][j + KS / 2][e] = (__bf16)(y * cs + x * sn);
                }
            }
        }
    }
    // scores in base-2 exponent units straight out of the matrix pipe
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int j = 0; j < KS; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[h][j][e] = (__bf16)(float(qf[h][j][e]) * scale_log2);

    f32x16 o_acc[NH][DB];
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o_acc[h][db][i] = 0.f;
    // Softmax state of a row, per head, in base-2 exponent units: m_ref is the reference exponent, l_run the sum of
    // the probabilities 2^(s - m_ref) so far (this lane's half of the row).
    float l_run[NH], m_ref[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        l_run[h] = 0.f;
        m_ref[h] = 0.f;
    }

    int koff[KS], voff[4];
    {
        const int xk = swizzle_key<2 * D>(n) ^ hg, xv = swizzle_key<2 * kTileN>(n) ^ hg;
#pragma unroll
        for (int j = 0; j < KS; ++j) koff[j] = n * D + ((2 * j) ^ xk) * 8;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) voff[qd] = n * kTileN + ((2 * qd) ^ xv) * 8;
    }
    {
        int t0 = my_vis, t1 = tok_q;
        asm volatile("" : "+v"(t0), "+v"(t1));
    }
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int j = 0; j < KS; ++j) {
            u32x4 t = __builtin_bit_cast(u32x4, qf[h][j]);
            asm volatile("" : "+v"(t));
            qf[h][j] = __builtin_bit_cast(bf16x8, t);
        }

    // K fragment f of a tile: key block f % SB, k-step f / SB; V^T fragment f: d block f % DB, 16-key step f / DB
    auto ld_k = [&](const uint16_t* kb, int f) { return *reinterpret_cast<const bf16x8*>(kb + 32 * (f % SB) * D + koff[f / SB]); };
    auto ld_v = [&](const uint16_t* vb, int f) { return *reinterpret_cast<const bf16x8*>(vb + 32 * (f % DB) * kTileN + voff[f / DB]); };

    struct TileInfo { bool partial; int limit; int c0; };
    auto tile_info = [&](int ti) {
        const bool in_a = ti < it.a_total;
        const int kt = in_a ? ti : ti - it.a_total;
        const bool partial = kt >= (in_a ? it.a_full : it.b_full) || (kt + 1) * kTileN > (in_a ? it.n_stream : it.n_src);
        return TileInfo{partial, in_a ? my_row + 1 : my_vis, kt * kTileN + 8 * hg};
    };
    auto max_with_partner = [&](float x) {
        float a = x, b = x;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
        return fmaxf(a, b);
    };
    auto rescale_acc = [&](int h, float alpha) {
        if constexpr (NH == 2) {
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float x = o_acc[h][db][i], tmp;
                    asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                                 : "+a"(x), "=&v"(tmp) : "v"(alpha));
                    o_acc[h][db][i] = x;
                }
            asm volatile("s_nop 7" ::: "memory");
        } else {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o_acc[h][db][i] *= alpha;
        }
    };
    // the columns of a partial tile that a row may not see: exponent -inf, probability 0
    // lane (n, hg), block sb, register i  <->  key column kt*64 + 32 sb + 16 (i/8) + 8 hg + i%8
    auto mask_tile = [&](f32x16 (&sv)[NH][SB], const TileInfo& ti) {
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int col = ti.c0 + 32 * sb + 16 * (i >> 3) + (i & 7);
                    sv[h][sb][i] = col < ti.limit ? sv[h][sb][i] : -INFINITY;
                }
    };
    // row maximum (both lanes of the row) of a tile's exponents
    auto row_max = [&](const f32x16 (&blk)[SB]) {
        float mx = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, blk[sb][i]);
        return max_with_partner(mx);
    };

    // ---- prologue: tile 0 gives every row its reference exponent ----
    // sv: the exponents of the tile whose probabilities are formed next (vector registers); s_next: the score blocks
    // the matrix pipe is filling.  Between two tiles the LAST block of s_next holds -m_ref in all its 16 registers:
    // the first matrix instruction of every score block starts from it (the last block in place), so a score leaves
    // the pipe as s - m_ref.
    f32x16 sv[NH][SB], s_next[NH][SB];
    wait_vmcnt<(STAGES == 3 ? 4 : 2) * NL>();            // K0 has landed
    __syncthreads();
    {
        const uint16_t* kb = &sm.k[0][0];
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < SB * KS; ++f) {
            const bf16x8 a = ld_k(kb, f);
#pragma unroll
            for (int h = 0; h < NH; ++h)
                sv[h][f % SB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[h][f / SB], f / SB == 0 ? zero16 : sv[h][f % SB], 0, 0, 0);
        }
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float x = sv[h][sb][i];
                    asm volatile("" : "+v"(x));                   // in vector registers from here on
                    sv[h][sb][i] = x;
                }
        const TileInfo t0 = tile_info(0);
        if (t0.partial) mask_tile(sv, t0);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            m_ref[h] = row_max(sv[h]);                            // finite: column 0 is visible to every row
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) sv[h][sb][i] -= m_ref[h];
#pragma unroll
            for (int i = 0; i < 16; ++i) s_next[h][SB - 1][i] = -m_ref[h];
        }
    }

    bf16x8 pb[NH][SB][2];                                // probabilities of the current tile, as the second product's operand
    float psum[NH];
    // slot m of NH SB KS: PER elements of the probabilities of the tile in sv, in the order (head, block, register)
    // (the two-head form sums the probabilities as the second product will see them, rounded to bf16, two per
    // instruction: one vector instruction less per pair, +0.8 % there; the one-head form measured 1 % slower with it
    // and keeps its fp32 adds)
    bf16x2 ones2;
    ones2[0] = (__bf16)1.f;
    ones2[1] = (__bf16)1.f;
    static_assert(PER % 2 == 0, "probabilities are formed in pairs");
    auto exp_slot = [&](int m) {
#pragma unroll
        for (int u = 0; u < PER; u += 2) {
            const int e = m * PER + u;
            const int hh = e / (SB * 16), sb2 = (e / 16) % SB, i = e % 16;
            const float pr0 = __builtin_amdgcn_exp2f(sv[hh][sb2][i]), pr1 = __builtin_amdgcn_exp2f(sv[hh][sb2][i + 1]);
            bf16x2 p2;
            p2[0] = (__bf16)pr0;
            p2[1] = (__bf16)pr1;
            if constexpr (NH == 2) psum[hh] = __builtin_amdgcn_fdot2_f32_bf16(p2, ones2, psum[hh], false);
            else psum[hh] += pr0 + pr1;
            pb[hh][sb2][i >> 3][i & 7] = p2[0];
            pb[hh][sb2][i >> 3][(i & 7) + 1] = p2[1];
        }
    };
    // A row sum beyond 2^kRiseLog2 (or not finite) means the tile's exponents outgrew the reference: move it to the
    // tile's row maximum, form the tile's probabilities again, rescale what has been accumulated.  Scores already in
    // flight relative to the old reference still have `late` to lose when they arrive.
    float late[NH];
    auto check_rise = [&]() {
        bool trig = false;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            asm volatile("" : "+v"(psum[h]));
            late[h] = 0.f;
            trig = trig || !(psum[h] <= __builtin_exp2f(kRiseLog2));
        }
        const bool any = __any(trig);
        if (any) {
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float rise = row_max(sv[h]);
                const float shift = rise > 0.f ? rise : 0.f;           // (-inf: the row sees nothing in this tile)
                const float alpha = __builtin_amdgcn_exp2f(-shift);
                late[h] = shift;
                psum[h] = 0.f;
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float pr = __builtin_amdgcn_exp2f(sv[h][sb][i] - shift);
                        psum[h] += pr;
                        pb[h][sb][i >> 3][i & 7] = (__bf16)pr;
                    }
                l_run[h] *= alpha;
                rescale_acc(h, alpha);
                m_ref[h] += shift;
            }
        }
#pragma unroll
        for (int h = 0; h < NH; ++h) l_run[h] += psum[h];
        return any;
    };

    int stage = 0;                                       // buffer of tile ti
    bf16x8 kpre[kPF], vpre[kPF];                         // first fragments of a phase, read during the phase before
    // every tile but the last: the loop body has no branch around its matrix instructions
    for (int ti = 0; ti + 1 < n_tiles; ++ti) {
        // three buffers: K(ti+2) and V^T(ti) have landed (V^T(ti+1) is in flight behind them); two: K(ti+1), V^T(ti);
        // everybody is done with K(ti) and V^T(ti-1), whose buffers the next copies go to
        wait_vmcnt<(STAGES == 3 ? 1 : 0) * NL>();
        __syncthreads();
        const int stage1 = stage == STAGES - 1 ? 0 : stage + 1;
        const int stage2 = stage1 == STAGES - 1 ? 0 : stage1 + 1;
        const uint16_t* copy_k = kc_head + size_t(tile_of(ti + (STAGES == 3 ? 3 : 2))) * TILE;
        const uint16_t* copy_v = vc_head + size_t(tile_of(ti + (STAGES == 3 ? 2 : 1))) * TILE;
        const uint32_t copy_k_lds = lds_k0 + stage * (TILE * 2);
        const uint32_t copy_v_lds = lds_v0 + (STAGES == 3 ? (stage == 0 ? 2 : stage - 1) : stage1) * (TILE * 2);
        const uint16_t* kb = &sm.k[0][0] + stage1 * TILE;
        const uint16_t* vb = &sm.vt[0][0] + stage * TILE;
        const uint16_t* kb2 = &sm.k[0][0] + stage2 * TILE;        // K(ti+2): the tile of the next round's phase X
        if (!EARLY_K || ti == 0) {
#pragma unroll
            for (int f = 0; f < kPF; ++f) kpre[f] = ld_k(kb, f);
        }

        // ---- phase X: scores of tile ti+1  |  probabilities of tile ti ----
#pragma unroll
        for (int h = 0; h < NH; ++h) psum[h] = 0.f;
        {
            constexpr int NF = SB * KS;
            bf16x8 a[NF];
#pragma unroll
            for (int f = 0; f < kPF; ++f) a[f] = kpre[f];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                if (f + kPF < NF) a[f + kPF] = ld_k(kb, f + kPF);
                else vpre[f + kPF - NF] = ld_v(vb, f + kPF - NF);     // the first V^T fragments of phase Y
                const int sb = f % SB, j = f / SB;
#pragma unroll
                for (int h = 0; h < NH; ++h) {
                    // k-step 0 starts from -m_ref, parked in the last block (which starts in place)
                    s_next[h][sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], qf[h][j], j == 0 ? s_next[h][SB - 1] : s_next[h][sb], 0, 0, 0);
                    // the copies of this round go out behind the first matrix instructions
                    if (f * NH + h == 0) {
                        if (STAGES == 3) async_copy_rows<NL>(copy_k, lane_off, copy_k_lds);
                        else async_copy_rows<NL>(copy_v, lane_off, copy_v_lds);
                    }
                    if (f * NH + h == 1) {
                        if (STAGES == 3) async_copy_rows<NL>(copy_v, lane_off, copy_v_lds);
                        else async_copy_rows<NL>(copy_k, lane_off, copy_k_lds);
                    }
                    exp_slot(f * NH + h);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        const bool moved = check_rise();

        // ---- phase Y: O^T += V^T P^T of tile ti  |  the exponents of tile ti+1 leave the accumulation registers ----
        // slot m of NH DB SB 2: PER fresh exponents, in the order (block, head, register); the last block is left
        // holding -m_ref for the next round
        float neg[NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) neg[h] = -m_ref[h];
        auto move_slot = [&](int m) {
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int e = m * PER + u;
                const int sb2 = e / (NH * 16), hh = (e / 16) % NH, i = e % 16;
                // ONE move out of the accumulation registers, HERE (a plain copy would be sunk to its use, into
                // the crowded phase X); the producing matrix instruction retired at least three of them ago
                float x;
                if constexpr (NH == 2) {
                    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(s_next[hh][sb2][i]));
                } else {
                    x = s_next[hh][sb2][i];
                    asm volatile("" : "+v"(x));
                }
                sv[hh][sb2][i] = x;
                if (sb2 == SB - 1) {
                    if constexpr (NH == 2) {
                        float t;
                        asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(t) : "v"(neg[hh]));
                        s_next[hh][sb2][i] = t;
                    } else {
                        s_next[hh][sb2][i] = neg[hh];
                    }
                }
            }
        };
        {
            constexpr int NF = DB * SB * 2;
            bf16x8 a[NF];
#pragma unroll
            for (int f = 0; f < kPF; ++f) a[f] = vpre[f];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                if (f + kPF < NF) a[f + kPF] = ld_v(vb, f + kPF);
                else if (EARLY_K) kpre[f + kPF - NF] = ld_k(kb2, f + kPF - NF);   // the first K fragments of the next round
                const int db = f % DB, st = f / DB;              // keys 16 st .. 16 st + 15
#pragma unroll
                for (int h = 0; h < NH; ++h) {
                    o_acc[h][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], pb[h][st >> 1][st & 1], o_acc[h][db], 0, 0, 0);
                    move_slot(f * NH + h);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (moved) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sv[h][sb][i] -= late[h];
        }
        const TileInfo fresh = tile_info(ti + 1);
        if (fresh.partial) mask_tile(sv, fresh);
        stage = stage1;
    }
    // ---- the last tile: its probabilities and the second product, no scores behind it ----
    {
        wait_vmcnt<0>();                                 // (also: no copy into LDS may outlive the workgroup)
        __syncthreads();
        const uint16_t* vb = &sm.vt[0][0] + stage * TILE;
        constexpr int NF = DB * SB * 2;
        bf16x8 a[NF];
#pragma unroll
        for (int f = 0; f < kPF; ++f) a[f] = ld_v(vb, f);
#pragma unroll
        for (int h = 0; h < NH; ++h) psum[h] = 0.f;
#pragma unroll
        for (int m = 0; m < NH * SB * KS; ++m) exp_slot(m);
        check_rise();
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (f + kPF < NF) a[f + kPF] = ld_v(vb, f + kPF);
            const int db = f % DB, st = f / DB;
#pragma unroll
            for (int h = 0; h < NH; ++h)
                o_acc[h][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], pb[h][st >> 1][st & 1], o_acc[h][db], 0, 0, 0);
        }
    }

#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const float l_tot = l_run[h] + __shfl_xor(l_run[h], 32);   // wave-wide exchange: inactive rows take part
        if (!active) continue;
        const float inv = 1.f / l_tot;
        uint16_t* op = out + (int64_t(tok_q) * n_q_heads + hq0 + h) * D;
        // lane (n, hg), block db, register i  <->  d = 32 db + 8 (i/4) + 4 hg + i%4
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 o4;
#pragma unroll
                for (int c = 0; c < 4; ++c) o4[c] = (__bf16)(o_acc[h][db][4 * q4 + c] * inv);
                *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * q4 + 4 * hg) = o4;
            }
        if (lse && hg == 0) lse[int64_t(tok_q) * n_q_heads + hq0 + h] = (m_ref[h] + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
}


}  // namespace st

using namespace st;

// packed K and V^T tiles, then the (cos, sin) table of the fused rotation (one float2 per packed row and pair)
static size_t prefill_tile_bytes(const st_plan* plan, int n_kv_heads, int head_dim) {
    return 2 * size_t(n_kv_heads) * size_t(plan->pack_tiles) * kTileN * size_t(head_dim) * sizeof(uint16_t);
}
static size_t prefill_ws_bytes(const st_plan* plan, int n_kv_heads, int head_dim, st_dtype dt) {
    if (dt != ST_BF16) return 0;                     // the fp32 path reads q / k / v in place
    return prefill_tile_bytes(plan, n_kv_heads, head_dim) + size_t(plan->pack_tiles) * kTileN * size_t(head_dim / 2) * sizeof(float2);
}

extern "C" size_t st_prefill_workspace_bytes(const st_plan* plan, int32_t n_kv_heads, int32_t head_dim, st_dtype dt) {
    if (!plan || n_kv_heads <= 0 || head_dim <= 0) return 0;
    return prefill_ws_bytes(plan, n_kv_heads, head_dim, dt);
}

// positions == nullptr: rotated q / k (st_attn_prefill); otherwise unrotated, rotated here (st_attn_prefill_rope)
static st_status prefill_impl(void* out, float* lse, const void* q, const void* k, const void* v, const int32_t* positions,
                              double theta_base, const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                              float scale, st_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out || !q || !k || !v || !plan) return fail(ST_ERR_INVALID_ARG, "st_attn_prefill: null pointer");
    if (!aligned16(out) || !aligned16(q) || !aligned16(k) || !aligned16(v))
        return fail(ST_ERR_INVALID_ARG, "st_attn_prefill: tensors must be 16-byte aligned");
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0)
        return fail(ST_ERR_SHAPE, "st_attn_prefill: n_q_heads %d must be a positive multiple of n_kv_heads %d", n_q_heads, n_kv_heads);
    if (head_dim != 64 && head_dim != 128) return fail(ST_ERR_UNSUPPORTED, "st_attn_prefill: head_dim %d (64 or 128)", head_dim);
    if (dt != ST_F32 && dt != ST_BF16) return fail(ST_ERR_UNSUPPORTED, "st_attn_prefill: dtype %d", int(dt));
    if (plan->n_tokens == 0) return ST_OK;
    if (plan->n_tokens * int64_t(n_q_heads) * head_dim >= (int64_t(1) << 31))
        return fail(ST_ERR_SHAPE, "st_attn_prefill: n_tokens * n_q_heads * head_dim must stay below 2^31 elements");
    const size_t need = prefill_ws_bytes(plan, n_kv_heads, head_dim, dt);
    if (need > 0) {
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
            return fail(ST_ERR_INVALID_ARG, "st_attn_prefill: workspace must be non-null and 256-byte aligned");
        if (workspace_bytes < need)
            return fail(ST_ERR_CAPACITY, "st_attn_prefill: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    }
    if (scale <= 0.f) scale = 1.f / sqrtf(float(head_dim));
    const int64_t blocks = int64_t(plan->m_max) * n_q_heads;
    const int64_t pack_blocks = int64_t(plan->pack_tiles) * n_kv_heads;
    if (blocks > 0x7fffffff || pack_blocks > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_prefill: grid too large");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ST_HIP(plan->wait_built(s));
    const PlanView pv = plan->view();
    if (dt == ST_F32) {
        const size_t smem = sizeof(float) * kTileM * (head_dim + 1);
        if (head_dim == 64) {
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_simple_kernel<float, 64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
            hipLaunchKernelGGL((prefill_simple_kernel<float, 64>), dim3((unsigned)blocks), dim3(kTileM), smem, s, (float*)out, lse,
                               (const float*)q, (const float*)k, (const float*)v, pv, n_q_heads, n_kv_heads, scale);
        } else {
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_simple_kernel<float, 128>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
            hipLaunchKernelGGL((prefill_simple_kernel<float, 128>), dim3((unsigned)blocks), dim3(kTileM), smem, s, (float*)out, lse,
                               (const float*)q, (const float*)k, (const float*)v, pv, n_q_heads, n_kv_heads, scale);
        }
        ST_LAUNCH_CHECK("prefill_simple_kernel");
        return ST_OK;
    }
    const size_t tile_bytes = prefill_tile_bytes(plan, n_kv_heads, head_dim);
    uint16_t* kc = static_cast<uint16_t*>(workspace);
    uint16_t* vc = kc + tile_bytes / (2 * sizeof(uint16_t));
    float2* tab = reinterpret_cast<float2*>(static_cast<char*>(workspace) + tile_bytes);
    const bool rope = positions != nullptr;
    const RopeFreq freq = rope ? make_rope_freq(theta_base, head_dim) : RopeFreq{};
    const float scale_log2 = scale * kLog2e;
    // Two query heads per workgroup when heads come in pairs over a KV head and the sequences are long (an item then
    // walks a hundred key tiles and more, and the halved LDS / L2 traffic per flop pays); short sequences finish
    // sooner with twice as many, lighter workgroups, two per compute unit.
    const int heads_wanted = plan->heads_per_workgroup;
    const bool can_pair = (n_q_heads / n_kv_heads) % 2 == 0;
    const bool pair = can_pair && (heads_wanted == 2 || (heads_wanted == 0 && plan->n_tokens / plan->batch >= 8192));
    auto launch = [&](auto dtag) -> st_status {
        constexpr int HD = decltype(dtag)::value;
        prof_begin(kProfTilePack, s);
        for (int rep = 0; rep < prof_repeat(); ++rep)
        if (rope) {
            hipLaunchKernelGGL((rope_table_kernel<HD>), dim3((unsigned)plan->pack_tiles), dim3(256), 0, s, tab, positions, pv, freq);
            hipLaunchKernelGGL((tile_pack_rope_kernel<HD>), dim3((unsigned)pack_blocks), dim3(256), 0, s, kc, vc, (const float2*)tab,
                               (const uint16_t*)k, (const uint16_t*)v, pv, n_kv_heads);
        } else
            hipLaunchKernelGGL((tile_pack_kernel<HD>), dim3((unsigned)pack_blocks), dim3(256), 0, s, kc, vc, (const uint16_t*)k,
                               (const uint16_t*)v, pv, n_kv_heads);
        prof_end(kProfTilePack, s);
        auto run = [&](auto nh_tag, auto rope_tag) -> st_status {
            constexpr int NH = decltype(nh_tag)::value;
            constexpr bool ROPE = decltype(rope_tag)::value;
            const size_t smem = sizeof(PipeSmem<HD, NH == 2 ? 3 : 2>);
            auto* kern = &prefill_attn_kernel<HD, NH, ROPE>;
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
            prof_begin(kProfPrefillAttn, s);
            for (int rep = 0; rep < prof_repeat(); ++rep)
                hipLaunchKernelGGL(kern, dim3((unsigned)(blocks / NH)), dim3(256), smem, s, (uint16_t*)out,
                                   lse, (const uint16_t*)q, kc, vc, pv, n_q_heads, n_kv_heads, scale_log2, (const float2*)tab);
            prof_end(kProfPrefillAttn, s);
            return ST_OK;
        };
        using One = std::integral_constant<int, 1>;
        using Two = std::integral_constant<int, 2>;
        return rope ? (pair ? run(Two{}, std::true_type{}) : run(One{}, std::true_type{}))
                    : (pair ? run(Two{}, std::false_type{}) : run(One{}, std::false_type{}));
    };
    const st_status lr = head_dim == 64 ? launch(std::integral_constant<int, 64>{}) : launch(std::integral_constant<int, 128>{});
    if (lr != ST_OK) return lr;
    ST_LAUNCH_CHECK("tile_pack_kernel / prefill_attn_kernel");
    return ST_OK;
}

extern "C" st_status st_attn_prefill(void* out, float* lse, const void* q, const void* k, const void* v,
                                     const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     float scale, st_dtype dt, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
    return prefill_impl(out, lse, q, k, v, nullptr, 0.0, plan, n_q_heads, n_kv_heads, head_dim, scale, dt, workspace, workspace_bytes,
                        hip_stream);
}

extern "C" st_status st_attn_prefill_rope(void* out, float* lse, const void* q, const void* k, const void* v,
                                          const int32_t* positions, double theta_base, const st_plan* plan, int32_t n_q_heads,
                                          int32_t n_kv_heads, int32_t head_dim, float scale, st_dtype dt, void* workspace,
                                          size_t workspace_bytes, void* hip_stream) {
    if (!positions) return fail(ST_ERR_INVALID_ARG, "st_attn_prefill_rope: positions is null");
    if (!(theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "st_attn_prefill_rope: theta_base must be positive");
    if (dt != ST_BF16) return fail(ST_ERR_UNSUPPORTED, "st_attn_prefill_rope: bf16 only (dtype %d); rotate fp32 inputs with st_rope_apply", int(dt));
    return prefill_impl(out, lse, q, k, v, positions, theta_base, plan, n_q_heads, n_kv_heads, head_dim, scale, dt, workspace,
                        workspace_bytes, hip_stream);
}

extern "C" st_status st_attn_prefill_ids(void* out, float* lse, const void* q, const void* k, const void* v,
                                         const int32_t* segment_ids, const int32_t* stream_ids,
                                         const int32_t* positions, const int32_t* cu_seqlens_host, int32_t batch,
                                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float scale,
                                         st_dtype dt, void* hip_stream) {
    st_plan* plan = nullptr;
    st_status r = st_plan_create(&plan, segment_ids, stream_ids, positions, cu_seqlens_host, batch, nullptr, 0, 1, hip_stream);
    if (r != ST_OK) return r;
    void* ws = nullptr;
    const size_t ws_bytes = (n_kv_heads > 0 && head_dim > 0) ? prefill_ws_bytes(plan, n_kv_heads, head_dim, dt) : 0;
    if (ws_bytes > 0) {
        hipError_t e = hipMalloc(&ws, ws_bytes);
        if (e != hipSuccess) {
            st_plan_destroy(plan);
            return fail(ST_ERR_RUNTIME, "st_attn_prefill_ids: hipMalloc(%zu) failed: %s", ws_bytes, hipGetErrorString(e));
        }
    }
    r = st_attn_prefill(out, lse, q, k, v, plan, n_q_heads, n_kv_heads, head_dim, scale, dt, ws, ws_bytes, hip_stream);
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream));
    if (ws) (void)hipFree(ws);
    st_plan_destroy(plan);
    if (r == ST_OK && e != hipSuccess) return fail(ST_ERR_RUNTIME, "st_attn_prefill_ids: %s", hipGetErrorString(e));
    return r;
}
