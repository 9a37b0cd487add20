// Backward of the streaming-mask prefill attention (streaming-constrained training, Sec. 3.2: the mask
// of Eq. 2 is part of the forward pass of supervised fine-tuning, so only visible pairs carry gradient).
//
// With P = softmax over the visible keys (recomputed from the forward's log-sum-exp), delta_i = dO_i . O_i:
//     dV_j = sum_i P_ij dO_i      dP_ij = dO_i . V_j      dS_ij = P_ij (dP_ij - delta_i)
//     dQ_i = scale sum_j dS_ij K_j                       dK_j = scale sum_i dS_ij Q_i
// This is the plain path: one thread per row, fp32 arithmetic, no matrix cores -- correct for both
// dtypes and every structure the forward accepts, and the baseline a tiled MFMA version has to beat.
// The same segment tables drive it: query rows walk the forward's work items (tiles past `total` are
// never read); key rows find the queries that see them from the same tables read the other way round --
// a source key c is seen by source rows >= c and by the reasoning rows whose visible-source count exceeds
// c (a suffix of the reasoning stream, found by bisection), a reasoning key by reasoning rows >= c.
//   bwd_dq_kernel    thread = query row of one query head: delta, dQ
//   bwd_dkv_kernel   thread = key row of one KV head, all query heads of its group: dV (pass 0) or dK (pass 1)
#include <math.h>

#include <type_traits>

#include "st_tiles.h"

namespace st {

template <typename T>
__device__ __forceinline__ float ldf(const T* p);
template <>
__device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ldf<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }
template <typename T>
__device__ __forceinline__ void stf(T* p, float x);
template <>
__device__ __forceinline__ void stf<float>(float* p, float x) { *p = x; }
template <>
__device__ __forceinline__ void stf<uint16_t>(uint16_t* p, float x) { *p = f32_to_bf16_bits(x); }

template <typename T, int D>
__global__ __launch_bounds__(kTileM) void bwd_dq_kernel(T* __restrict__ dq, float* __restrict__ delta_out,
                                                       const T* __restrict__ d_out, const T* __restrict__ q,
                                                       const T* __restrict__ k, const T* __restrict__ v,
                                                       const T* __restrict__ out, const float* __restrict__ lse,
                                                       PlanView pv, int n_q_heads, int n_kv_heads, float scale) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float (*s_q)[D + 1] = reinterpret_cast<float (*)[D + 1]>(smem_raw);
    float (*s_do)[D + 1] = s_q + kTileM;
    const int rank = blockIdx.x / n_q_heads;
    const int hq = blockIdx.x % n_q_heads;
    const int hk = hq / (n_q_heads / n_kv_heads);
    const WorkItem it = pv.sorted[rank];
    if (it.n_rows == 0) return;
    const int r = threadIdx.x;
    const bool active = r < it.n_rows;
    const int my_row = it.row0 + min(r, it.n_rows - 1);
    const int tok_q = pv.perm[it.a_base + my_row];
    const int my_vis = pv.vis[it.a_base + my_row];
    const int64_t qoff = (int64_t(tok_q) * n_q_heads + hq) * D;
    float delta = 0.f;
    for (int d = 0; d < D; ++d) {
        s_q[r][d] = ldf(q + qoff + d);
        s_do[r][d] = ldf(d_out + qoff + d);
        delta = fmaf(s_do[r][d], ldf(out + qoff + d), delta);
    }
    const float my_lse = lse[int64_t(tok_q) * n_q_heads + hq];
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;

    const int n_tiles = it.a_total + it.b_total;
    for (int ti = 0; ti < n_tiles; ++ti) {
        const bool in_a = ti < it.a_total;
        const int kt = in_a ? ti : ti - it.a_total;
        const int base = in_a ? it.a_base : it.b_base;
        const int n_cols = in_a ? it.n_stream : it.n_src;
        const int limit = in_a ? my_row + 1 : my_vis;          // columns < limit are visible
        const int c_end = min(min((kt + 1) * kTileN, n_cols), limit);
        for (int col = kt * kTileN; col < c_end; ++col) {
            const int tok_k = pv.perm[base + col];
            const T* kp = k + (int64_t(tok_k) * n_kv_heads + hk) * D;
            const T* vp = v + (int64_t(tok_k) * n_kv_heads + hk) * D;
            float s = 0.f, dp = 0.f;
            for (int d = 0; d < D; ++d) {
                s = fmaf(s_q[r][d], ldf(kp + d), s);
                dp = fmaf(s_do[r][d], ldf(vp + d), dp);
            }
            const float p = expf(s * scale - my_lse);
            const float ds = p * (dp - delta) * scale;
#pragma unroll
            for (int d = 0; d < D; ++d) acc[d] = fmaf(ds, ldf(kp + d), acc[d]);
        }
    }
    if (!active) return;
#pragma unroll
    for (int d = 0; d < D; ++d) stf(dq + qoff + d, acc[d]);
    delta_out[int64_t(tok_q) * n_q_heads + hq] = delta;
}

// first reasoning row (compact, relative to the reasoning stream) whose visible-source count exceeds c
__device__ __forceinline__ int first_row_seeing(const int32_t* vis_rsn, int n_rsn, int c) {
    int lo = 0, hi = n_rsn;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (vis_rsn[mid] > c) hi = mid; else lo = mid + 1;
    }
    return lo;
}

template <typename T, int D, int PASS>
__global__ __launch_bounds__(kTileM) void bwd_dkv_kernel(T* __restrict__ dkv, const float* __restrict__ delta,
                                                        const T* __restrict__ d_out, const T* __restrict__ q,
                                                        const T* __restrict__ k, const T* __restrict__ v,
                                                        const float* __restrict__ lse, PlanView pv, int n_q_heads,
                                                        int n_kv_heads, float scale) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float (*s_k)[D + 1] = reinterpret_cast<float (*)[D + 1]>(smem_raw);
    float (*s_v)[D + 1] = s_k + kTileM;
    const int rank = blockIdx.x / n_kv_heads;
    const int hk = blockIdx.x % n_kv_heads;
    const int group = n_q_heads / n_kv_heads;
    const WorkItem it = pv.sorted[rank];                       // 128 rows of one stream, read as KEYS here
    if (it.n_rows == 0) return;
    const int r = threadIdx.x;
    if (r >= it.n_rows) return;                                // (no barrier below)
    const int c = it.row0 + r;                                 // key index in its stream
    const int tok_k = pv.perm[it.a_base + c];
    const int64_t koff = (int64_t(tok_k) * n_kv_heads + hk) * D;
    for (int d = 0; d < D; ++d) {
        s_k[r][d] = ldf(k + koff + d);
        s_v[r][d] = ldf(v + koff + d);
    }
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;

    // the query rows that see this key, as up to two runs of compact rows
    const int S = it.n_src;
    const int seq_base = it.b_base;                            // compact row of the sequence's first source token
    const int n_rsn = (it.kind == ST_SOURCE) ? (pv.cu[it.seq + 1] - pv.cu[it.seq] - S) : it.n_stream;
    int run_lo[2], run_hi[2];
    if (it.kind == ST_SOURCE) {
        run_lo[0] = seq_base + c;                              // source rows >= c
        run_hi[0] = seq_base + S;
        run_lo[1] = seq_base + S + first_row_seeing(pv.vis + seq_base + S, n_rsn, c);
        run_hi[1] = seq_base + S + n_rsn;
    } else {
        run_lo[0] = it.a_base + c;                             // reasoning rows >= c
        run_hi[0] = it.a_base + n_rsn;
        run_lo[1] = run_hi[1] = 0;
    }
    for (int run = 0; run < 2; ++run)
        for (int row = run_lo[run]; row < run_hi[run]; ++row) {
            const int tok_q = pv.perm[row];
            for (int g = 0; g < group; ++g) {
                const int hq = hk * group + g;
                const int64_t qoff = (int64_t(tok_q) * n_q_heads + hq) * D;
                float s = 0.f, dp = 0.f;
                for (int d = 0; d < D; ++d) {
                    s = fmaf(ldf(q + qoff + d), s_k[r][d], s);
                    if (PASS == 1) dp = fmaf(ldf(d_out + qoff + d), s_v[r][d], dp);
                }
                const float p = expf(s * scale - lse[int64_t(tok_q) * n_q_heads + hq]);
                if (PASS == 0) {
#pragma unroll
                    for (int d = 0; d < D; ++d) acc[d] = fmaf(p, ldf(d_out + qoff + d), acc[d]);
                } else {
                    const float ds = p * (dp - delta[int64_t(tok_q) * n_q_heads + hq]) * scale;
#pragma unroll
                    for (int d = 0; d < D; ++d) acc[d] = fmaf(ds, ldf(q + qoff + d), acc[d]);
                }
            }
        }
#pragma unroll
    for (int d = 0; d < D; ++d) stf(dkv + koff + d, acc[d]);
}


// --------------------------------------------------------------------------
// MFMA path (bf16).
// --------------------------------------------------------------------------
// dQ: the forward's loop over the key tiles of a query tile (same work items, same transposed products, a lane
// owns one query row), with three products per key tile:
//   S^T  = K  Q^T     (K row tile from LDS, Q^T in registers)        -> P^T = exp2(S^T scale - lse)
//   dP^T = V  dO^T    (V row tile from LDS, dO^T in registers)       -> dS^T = P^T (dP^T - delta)
//   dQ^T += K^T dS^T  (K^T read out of the same K row tile with transposing LDS reads; dS^T from the accumulators,
//                      rounded to bf16)
// The kernel fits 256 registers, so TWO workgroups share a CU (two waves per SIMD fill each other's gaps between
// matrix and vector work); the K and V row tiles are double-buffered and copied one tile ahead (64 KB of LDS per
// workgroup), one barrier per key tile.
template <int D>
struct BwdDqSmem {
    uint16_t k[2][kTileN * D];        // K rows
    uint16_t v[2][kTileN * D];        // V rows
};

template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dq_mfma_kernel(uint16_t* __restrict__ dq, const uint16_t* __restrict__ d_out,
                                                             const uint16_t* __restrict__ q, const uint16_t* __restrict__ krows,
                                                             const uint16_t* __restrict__ vrows,
                                                             const float* __restrict__ lse, const float* __restrict__ delta,
                                                             PlanView pv, int n_q_heads, int n_kv_heads, float scale) {
    constexpr int KS = D / 16, DB = D / 32, SB = kTileN / 32;
    constexpr int TILE = kTileN * D;
    constexpr int NL = TILE * 2 / 1024 / 4;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    BwdDqSmem<D>& sm = *reinterpret_cast<BwdDqSmem<D>*>(smem_raw);

    const int rank = blockIdx.x / n_q_heads;
    const int hh = blockIdx.x % n_q_heads;
    const int group = n_q_heads / n_kv_heads;
    const int hk = hh % n_kv_heads;
    const int hq = hk * group + hh / n_kv_heads;
    const WorkItem it = pv.sorted[rank];
    if (it.n_rows == 0) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hg = lane >> 5;
    const int n_tiles = it.a_total + it.b_total;

    const size_t head_off = size_t(hk) * pv.pack_tiles * TILE + size_t(__builtin_amdgcn_readfirstlane(wave) * NL) * 512;   // (+ 16 bytes per lane)
    const uint32_t lane_off = uint32_t(lane) * 16u;
    auto tile_of = [&](int ti) {
        ti = min(ti, n_tiles - 1);
        return ti < it.a_total ? it.tile_a0 + ti : it.tile_b0 + (ti - it.a_total);
    };
    const uint32_t wave_off = uint32_t(__builtin_amdgcn_readfirstlane(wave)) * (NL * 1024);
    const uint32_t lds_k = uint32_t(uintptr_t(&sm.k[0][0])) + wave_off, lds_v = uint32_t(uintptr_t(&sm.v[0][0])) + wave_off;
    auto issue_rows = [&](int ti, int buf) {
        const size_t off = head_off + size_t(tile_of(ti)) * TILE;
        async_copy_rows<NL>(krows + off, lane_off, lds_k + buf * (TILE * 2));
        async_copy_rows<NL>(vrows + off, lane_off, lds_v + buf * (TILE * 2));
    };
    issue_rows(0, 0);

    const int row_in_tile = wave * 32 + n;
    const bool active = row_in_tile < it.n_rows;
    const int my_row = it.row0 + min(row_in_tile, it.n_rows - 1);
    const int tok_q = pv.perm[it.a_base + my_row];
    const int my_vis = pv.vis[it.a_base + my_row];
    const int64_t rowhead = int64_t(tok_q) * n_q_heads + hq;
    const float lse2 = lse[rowhead] * kLog2e, my_delta = delta[rowhead];
    const float scale_log2 = scale * kLog2e;

    bf16x8 qf[KS], dof[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) {
        qf[j] = *reinterpret_cast<const bf16x8*>(q + rowhead * D + 8 * hg + 16 * j);
        dof[j] = *reinterpret_cast<const bf16x8*>(d_out + rowhead * D + 8 * hg + 16 * j);
    }
    // queries times scale * log2(e), rounded to bf16 again (as in the forward kernel): K q' is a score in exponent units
#pragma unroll
    for (int j = 0; j < KS; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[j][e] = (__bf16)(float(qf[j][e]) * scale_log2);
    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

    int koff[KS];
    {
        const int xk = swizzle_key<2 * D>(n) ^ hg;
#pragma unroll
        for (int j = 0; j < KS; ++j) koff[j] = n * D + ((2 * j) ^ xk) * 8;
    }
    const TrOffsets<D> tr(lane);
    // Score and dP blocks of a tile.  A lane owns one query row, so what has to be taken off every score (the row's
    // log-sum-exp) and off every dP (the row's delta) is one number per lane: between tiles the LAST block of each
    // kind holds it, negated, in all sixteen registers, and the first matrix instruction of every block takes that as
    // its accumulator input (the last block in place, after the others have read it).
    f32x16 s_acc[SB], dp_acc[SB];
    const float neg_lse2 = -lse2, neg_delta = -my_delta;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        asm volatile("v_mov_b32 %0, %1" : "=v"(s_acc[SB - 1][i]) : "v"(neg_lse2));
        asm volatile("v_mov_b32 %0, %1" : "=v"(dp_acc[SB - 1][i]) : "v"(neg_delta));
    }

    for (int ti = 0; ti < n_tiles; ++ti) {
        const int buf = ti & 1;
        wait_vmcnt<0>();                 // the row tiles of ti have landed; everybody is done with tile ti - 1
        __syncthreads();
        issue_rows(ti + 1, buf ^ 1);     // (past the end: the last tile again, never used)

        const bool in_a = ti < it.a_total;
        const int kt = in_a ? ti : ti - it.a_total;
        const bool partial = kt >= (in_a ? it.a_full : it.b_full) || (kt + 1) * kTileN > (in_a ? it.n_stream : it.n_src);
        const int limit = in_a ? my_row + 1 : my_vis;

        // operands leave LDS a group of matrix instructions ahead of their use (one wave per SIMD: nobody else hides
        // that latency); scheduling barriers keep the order
        const uint16_t* kb = &sm.k[buf][0];
        const uint16_t* vb = &sm.v[buf][0];
        constexpr int G = 4, NG1 = SB * KS / G, NG2 = DB * SB * 2 / (2 * G);
        bf16x8 fk[2][G], fv[2][G];
        auto load1 = [&](int g, int slot) {
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int f = g * G + u, sb = f % SB, j = f / SB;
                fk[slot][u] = *reinterpret_cast<const bf16x8*>(kb + 32 * sb * D + koff[j]);
                fv[slot][u] = *reinterpret_cast<const bf16x8*>(vb + 32 * sb * D + koff[j]);
            }
        };
        auto load2 = [&](int g, int slot) {                 // 2 G fragments of K^T (transposing reads of the K rows): fk then fv of the slot
#pragma unroll
            for (int u = 0; u < 2 * G; ++u) {
                const int f = g * 2 * G + u;
                (u < G ? fk[slot][u] : fv[slot][u - G]) = tr.fragment(kb, f / DB, f % DB);
            }
        };
        load1(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NG1; ++g) {
            if (g + 1 < NG1) load1(g + 1, (g + 1) & 1);
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int f = g * G + u, sb = f % SB, j = f / SB;
                s_acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[g & 1][u], qf[j], j == 0 ? s_acc[SB - 1] : s_acc[sb], 0, 0, 0);
                dp_acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[g & 1][u], dof[j], j == 0 ? dp_acc[SB - 1] : dp_acc[sb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // lane (n, hg), block sb, register i  <->  key column kt*64 + 32 sb + 16 (i/8) + 8 hg + i%8
        bf16x8 dsb[SB][2];
        if (partial) {                   // (uniform) only the tiles on the edge of what the rows may see
            const int c0 = kt * kTileN + 8 * hg;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int col = c0 + 32 * sb + 16 * (i >> 3) + (i & 7);
                    s_acc[sb][i] = col < limit ? s_acc[sb][i] : -INFINITY;
                }
        }
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(s_acc[sb][i]);
                dsb[sb][i >> 3][i & 7] = (__bf16)(p * dp_acc[sb][i]);
            }
        // (written as instructions: left to the compiler, the two constant blocks become thirty-two more live registers)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            asm volatile("v_mov_b32 %0, %1" : "=v"(s_acc[SB - 1][i]) : "v"(neg_lse2));
            asm volatile("v_mov_b32 %0, %1" : "=v"(dp_acc[SB - 1][i]) : "v"(neg_delta));
        }
        load2(0, NG1 & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NG2; ++g) {
            const int slot = (NG1 + g) & 1;
            if (g + 1 < NG2) load2(g + 1, slot ^ 1);
#pragma unroll
            for (int u = 0; u < 2 * G; ++u) {
                const int f = g * 2 * G + u, db = f % DB, st = f / DB;
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u < G ? fk[slot][u] : fv[slot][u - G], dsb[st >> 1][st & 1], acc[db], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vmcnt<0>();
    if (!active) return;
    uint16_t* op = dq + rowhead * D;
    // lane (n, hg), block db, register i  <->  d = 32 db + 8 (i/4) + 4 hg + i%4
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 o4;
#pragma unroll
            for (int c = 0; c < 4; ++c) o4[c] = (__bf16)(acc[db][4 * q4 + c] * scale);
            *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * q4 + 4 * hg) = o4;
        }
}


// Row statistics of the backward in tile order: for every 64-row tile of a stream and every query head one
// 1 KB block of 256 floats -- [0, 64) MINUS lse in base-2 units (-inf for rows past the end of the stream: their
// probabilities become 0), [64, 128) MINUS delta, [128, 192) the visible-source count of the row (as int bits) --
// so that the key-side kernel fetches them with ONE asynchronous copy per tile.  delta is also written in
// token order for the query-side kernel.
template <int D>
__global__ __launch_bounds__(256) void bwd_rowstats_kernel(float* __restrict__ stats, float* __restrict__ delta_tok,
                                                          const uint16_t* __restrict__ d_out, const uint16_t* __restrict__ out,
                                                          const float* __restrict__ lse, PlanView pv, int n_q_heads) {
    constexpr int PER = D / 4;                                   // elements per thread: 4 threads share a row
    const int tile = blockIdx.x / n_q_heads;
    const int h = blockIdx.x % n_q_heads;
    const int b = find_seq(pv.pack_base, pv.batch, tile);
    const int lt = tile - pv.pack_base[b];
    const int t0 = pv.cu[b], S = pv.n_src[b], R = pv.cu[b + 1] - t0 - S;
    const int ts = (S + kTileN - 1) / kTileN, tr = (R + kTileN - 1) / kTileN;
    if (lt >= ts + tr) return;
    const bool src = lt < ts;
    const int kt = src ? lt : lt - ts;
    const int base = t0 + (src ? 0 : S) + kt * kTileN;
    const int valid = min(kTileN, (src ? S : R) - kt * kTileN);
    const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
    float l2 = INFINITY, dl = 0.f;
    int vs = 0;
    int64_t rh = 0;
    if (r < valid) {
        const int tok = pv.perm[base + r];
        rh = int64_t(tok) * n_q_heads + h;
        const uint16_t* a = d_out + rh * D + part * PER;
        const uint16_t* o = out + rh * D + part * PER;
#pragma unroll
        for (int c = 0; c < PER / 8; ++c) {
            const bf16x8 x = *reinterpret_cast<const bf16x8*>(a + 8 * c), y = *reinterpret_cast<const bf16x8*>(o + 8 * c);
#pragma unroll
            for (int e = 0; e < 8; ++e) dl = fmaf(float(x[e]), float(y[e]), dl);
        }
    }
    dl += __shfl_xor(dl, 1);
    dl += __shfl_xor(dl, 2);
    if (part != 0) return;
    if (r < valid) {
        l2 = lse[rh] * kLog2e;
        vs = pv.vis[base + r];
        delta_tok[rh] = dl;
    }
    float* blk = stats + (size_t(h) * pv.pack_tiles + tile) * 256;
    blk[r] = -l2;                                                // (negated: where the key-side kernel's accumulators start)
    blk[64 + r] = -dl;
    blk[128 + r] = __int_as_float(vs);
    blk[192 + r] = 0.f;
}

// dK, dV: one workgroup per (128 keys of one stream of one sequence, KV head) -- the forward's work items read
// as KEYS -- 4 waves x 32 keys, a lane owns one key.  It loops over the 64-row query tiles that can see its keys
// (own stream: tiles from the one holding its first key on; for source keys also the reasoning tiles from the
// first row whose visible-source count exceeds its first key on), for every query head of its group:
//   S   = Q  K^T    (Q row tile from LDS, K^T in registers)      -> P  = exp2(S scale - lse_row)
//   dP  = dO V^T    (dO row tile from LDS, V^T in registers)     -> dS = P (dP - delta_row)
//   dV^T += dO^T P  (dO^T out of the dO row tile with transposing LDS reads, P from the accumulators, rounded to bf16)
//   dK^T += Q^T dS  (Q^T out of the Q row tile likewise, dS from the accumulators)
// Rows run along the accumulator registers here, so lse / delta / visible count of the rows come from the
// tile's 1 KB statistics block in LDS.  Two buffers per tile kind (66 KB), one barrier per query tile.
// acc += A B with the accumulator in ACCUMULATION registers, whatever form the compiler gives the file's other matrix
// instructions: the key-side kernel's two output accumulators (128 registers) live there for the whole kernel, the
// score and dP blocks in vector registers where the exponentials read them -- no copies between the two files.
__device__ __forceinline__ void mfma_into_agprs(f32x16& acc, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int D>
struct BwdDkvSmem {
    uint16_t qr[2][kTileN * D];       // Q rows
    uint16_t dor[2][kTileN * D];      // dO rows
    float stats[2][256];
};

template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_mfma_kernel(uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                                              const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                              const uint16_t* __restrict__ qrows, const uint16_t* __restrict__ dorows,
                                                              const float* __restrict__ stats, PlanView pv, int n_q_heads,
                                                              int n_kv_heads, float scale) {
    constexpr int KS = D / 16, DB = D / 32, SB = kTileN / 32;
    constexpr int TILE = kTileN * D;
    constexpr int NL = TILE * 2 / 1024 / 4;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    BwdDkvSmem<D>& sm = *reinterpret_cast<BwdDkvSmem<D>*>(smem_raw);

    // The table is sorted by the FORWARD's cost (late rows first); a key's cost runs the other way (early keys
    // are seen by the most rows), so walk the table backwards: longest first again, unused slots at once.
    const int rank = pv.m_max - 1 - int(blockIdx.x / n_kv_heads);
    const int hk = blockIdx.x % n_kv_heads;
    const int group = n_q_heads / n_kv_heads;
    const WorkItem it = pv.sorted[rank];
    if (it.n_rows == 0) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hg = lane >> 5;
    const bool key_is_src = it.kind == ST_SOURCE;
    const int S = it.n_src;
    const int n_rsn = key_is_src ? (pv.cu[it.seq + 1] - pv.cu[it.seq] - S) : it.n_stream;

    // query tiles that can see keys >= row0: run A over the own stream, run B (source keys) over the reasoning stream
    const int a_first = it.row0 / kTileN, a_end = (it.n_stream + kTileN - 1) / kTileN;
    int b_first = 0, b_end = 0;
    if (key_is_src) {
        // first reasoning row whose visible count exceeds row0 (counts do not decrease along the stream), searched by
        // the whole wave: every lane tests the end of one 64th of the range, so the range shrinks 64-fold per memory
        // round trip (three for a few thousand rows, where a bisection takes a dozen)
        int lo = 0, hi = n_rsn;                                 // the answer lies in [lo, hi]; hi == n_rsn: no such row
        const int32_t* vr = pv.vis + it.b_base + S;
        while (lo < hi) {
            const int span = hi - lo, step = (span + 63) >> 6;
            const int last = min(span - 1, lane * step + step - 1);             // end of this lane's piece
            const unsigned long long seen = __ballot(vr[lo + last] > it.row0);  // (monotone along the lanes)
            if (seen == 0ull) {
                lo = hi;
            } else {
                const int first = __ffsll((long long)seen) - 1;
                hi = lo + min(span - 1, first * step + step - 1);               // this row exceeds row0 ...
                lo = lo + first * step;                                         // ... and none before this piece does
            }
            lo = __builtin_amdgcn_readfirstlane(lo);
            hi = __builtin_amdgcn_readfirstlane(hi);
        }
        b_first = lo / kTileN;
        b_end = (n_rsn + kTileN - 1) / kTileN;
        if (lo >= n_rsn) b_first = b_end;
    }
    const int n_a = a_end - a_first, n_b = b_end - b_first;
    const int n_iter = (n_a + n_b) * group;
    const int tile_own0 = it.tile_a0;                           // packed tile of row 0 of the own stream
    const int tile_rsn0 = it.tile_b0 + (S + kTileN - 1) / kTileN;   // ... of the reasoning stream (source keys)

    const int key_in_tile = wave * 32 + n;
    const int wave_last_key = it.row0 + min(__builtin_amdgcn_readfirstlane(wave) * 32 + 31, it.n_rows - 1);
    const bool active = key_in_tile < it.n_rows;
    const int my_key = it.row0 + min(key_in_tile, it.n_rows - 1);
    const int tok_k = pv.perm[it.a_base + my_key];
    const int64_t keyhead = int64_t(tok_k) * n_kv_heads + hk;
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) {
        kf[j] = *reinterpret_cast<const bf16x8*>(k + keyhead * D + 8 * hg + 16 * j);
        vf[j] = *reinterpret_cast<const bf16x8*>(v + keyhead * D + 8 * hg + 16 * j);
    }
    // keys times scale * log2(e), rounded to bf16 again: Q k' is a score in exponent units (dK takes Q, not K)
#pragma unroll
    for (int j = 0; j < KS; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) kf[j][e] = (__bf16)(float(kf[j][e]) * (scale * kLog2e));
#pragma unroll
    for (int j = 0; j < KS; ++j) {                              // landed before the loop (it counts its own copies)
        u32x4 t = __builtin_bit_cast(u32x4, kf[j]), u = __builtin_bit_cast(u32x4, vf[j]);
        asm volatile("" : "+v"(t), "+v"(u));
        kf[j] = __builtin_bit_cast(bf16x8, t);
        vf[j] = __builtin_bit_cast(bf16x8, u);
    }

    // iteration -> (query tile, head): heads fastest, so that a tile's row statistics change slowest; tiles from the LAST one
    // down (reasoning tiles, then the own stream's) -- every key block of a sequence then starts at the same query tile, and
    // the blocks that start together read the same tiles at about the same time (a quarter less traffic into L2)
    struct Iter { int tile; int hq; int row0; bool rs; };
    auto iter_at = [&](int t, int g) {                          // (tile count t of the walk, head g of the group)
        Iter r;
        r.hq = hk * group + g;
        if (t < n_a) {
            r.tile = tile_own0 + a_first + t;
            r.row0 = (a_first + t) * kTileN;
            r.rs = false;
        } else {
            r.tile = tile_rsn0 + b_first + (t - n_a);
            r.row0 = (b_first + (t - n_a)) * kTileN;
            r.rs = true;
        }
        return r;
    };
    const uint32_t wave_off = uint32_t(__builtin_amdgcn_readfirstlane(wave)) * (NL * 1024);
    const uint32_t lds_qr = uint32_t(uintptr_t(&sm.qr[0][0])) + wave_off, lds_dor = uint32_t(uintptr_t(&sm.dor[0][0])) + wave_off,
                   lds_st = uint32_t(uintptr_t(&sm.stats[0][0]));
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // the copies of one iteration go out in two pieces (one tensor each; the statistics with the first), so that the loop
    // can issue them from the shadows of its first matrix instructions
    const uint32_t lane_off = uint32_t(lane) * 16u;
    auto issue_piece = [&](const Iter& r, int buf, int piece) {
        const size_t off = (size_t(r.hq) * pv.pack_tiles + r.tile) * TILE + size_t(wave_u * NL) * 512;      // (+ 16 bytes per lane)
        if (piece == 0) {
            if (wave_u == 0) async_copy16(stats + (size_t(r.hq) * pv.pack_tiles + r.tile) * 256 + lane * 4, lds_st + buf * 1024);
            async_copy_rows<NL>(qrows + off, lane_off, lds_qr + buf * (TILE * 2));
        } else {
            async_copy_rows<NL>(dorows + off, lane_off, lds_dor + buf * (TILE * 2));
        }
    };
    if (n_iter > 0) {
        const Iter r0 = iter_at(n_a + n_b - 1, 0);
#pragma unroll
        for (int piece = 0; piece < 2; ++piece) issue_piece(r0, 0, piece);
    }

    f32x16 dk_acc[DB], dv_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            dk_acc[db][i] = 0.f;
            dv_acc[db][i] = 0.f;
        }
    int koff[KS];
    {
        const int xk = swizzle_key<2 * D>(n) ^ hg;
#pragma unroll
        for (int j = 0; j < KS; ++j) koff[j] = n * D + ((2 * j) ^ xk) * 8;
    }
    const TrOffsets<D> tr(lane);

    int t_next = n_a + n_b - 1, g_next = 0;
    Iter nxt = iter_at(t_next, g_next);
    for (int x = 0; x < n_iter; ++x) {
        const int buf = x & 1;
        wait_vmcnt<0>();                 // the tiles of iteration x have landed; everybody is done with x - 1
        __syncthreads();
        const bool more = x + 1 < n_iter;
        const Iter cur = nxt;
        if (more) {                      // (no division in the loop: the walk is stepped)
            if (++g_next == group) {
                g_next = 0;
                --t_next;
            }
            nxt = iter_at(t_next, g_next);
        }

        // Operands come out of LDS a group of matrix instructions ahead of their use (one wave per SIMD: nobody else
        // hides that latency): groups of 4 fragments per tensor, the next group requested before the current one is
        // multiplied; scheduling barriers keep that order.  The tile's two 32-row halves are staggered so that the
        // vector work of one half runs beside matrix work of the other:
        //     matrix pipe:  S, dP of half 0 | S, dP of half 1     | dV, dK of half 0    | dV, dK of half 1
        //     vector ALU :                  | P, dS of half 0     | P, dS of half 1     |
        // (two scores' worth of vector work behind every second matrix instruction; tiles on the edge of what the
        // rows may see form P and dS with their masks between the blocks instead).
        static_assert(SB == 2 && (DB == 4 || DB == 2) && KS == 2 * DB, "the stagger below is written for 64-row tiles of 64 or 128 dims");
        f32x16 s_acc[SB], dp_acc[SB];
        const uint16_t* qb = &sm.qr[buf][0];
        const uint16_t* ob = &sm.dor[buf][0];
        constexpr int G = DB;                                // fragments per tensor and group; eight score pairs per half go beside 2 G pairs of matrix instructions
        constexpr int PIECES = 4 / G;
        bf16x8 fq[2][G], fo[2][G];
        auto load1 = [&](int rb, int g, int slot) {          // Q and dO rows of half rb, k-steps G g .. G g + G - 1
#pragma unroll
            for (int u = 0; u < G; ++u) {
                fq[slot][u] = *reinterpret_cast<const bf16x8*>(qb + 32 * rb * D + koff[G * g + u]);
                fo[slot][u] = *reinterpret_cast<const bf16x8*>(ob + 32 * rb * D + koff[G * g + u]);
            }
        };
        auto load2 = [&](int stp, int slot) {                // dO^T and Q^T of rows 16 stp .. 16 stp + 15, all d blocks
#pragma unroll
            for (int u = 0; u < G; ++u) {
                fo[slot][u] = tr.fragment(ob, stp, u);
                fq[slot][u] = tr.fragment(qb, stp, u);
            }
        };
        // lane (n, hg), block rb, register i  <->  query row cur.row0 + 32 rb + 16 (i/8) + 8 hg + i%8, key my_key.
        // The accumulators start at minus the rows' log-sum-exp (scores) and minus their delta (dP), straight from the
        // tile's statistics block: what comes out is the exponent of P and dP - delta.
        const float* st = &sm.stats[buf][0];
#pragma unroll
        for (int rb = 0; rb < SB; ++rb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int r0 = 32 * rb + 16 * (q4 >> 1) + 8 * hg + 4 * (q4 & 1);
                const f32x4 a = *reinterpret_cast<const f32x4*>(st + r0);
                const f32x4 b2 = *reinterpret_cast<const f32x4*>(st + 64 + r0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s_acc[rb][4 * q4 + e] = a[e];
                    dp_acc[rb][4 * q4 + e] = b2[e];
                }
            }
        // every row of the tile sees every key of this wave?  (rows are ordered, visible counts do not decrease)
        const int first_vis = __builtin_amdgcn_readfirstlane(__float_as_int(st[128]));
        const bool all_seen = cur.rs ? first_vis > wave_last_key : cur.row0 >= wave_last_key;
        bf16x8 pb[SB][2], dsb[SB][2];
        // P and dS of two neighbouring registers of half rb (no mask)
        auto soft2 = [&](int rb, int i) {
            const float p0 = __builtin_amdgcn_exp2f(s_acc[rb][i]), p1 = __builtin_amdgcn_exp2f(s_acc[rb][i + 1]);
            pb[rb][i >> 3][i & 7] = (__bf16)p0;
            pb[rb][i >> 3][(i & 7) + 1] = (__bf16)p1;
            dsb[rb][i >> 3][i & 7] = (__bf16)(p0 * dp_acc[rb][i]);
            dsb[rb][i >> 3][(i & 7) + 1] = (__bf16)(p1 * dp_acc[rb][i + 1]);
        };
        // ... of a whole half, with the rows' masks
        auto soft_masked = [&](int rb) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int r0 = 32 * rb + 16 * half + 8 * hg;           // first of the 8 consecutive rows of these registers
                int vs[8];
#pragma unroll
                for (int q4 = 0; q4 < 2; ++q4) {
                    const f32x4 c2 = *reinterpret_cast<const f32x4*>(st + 128 + r0 + 4 * q4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) vs[4 * q4 + e] = __float_as_int(c2[e]);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int i = 8 * half + e;
                    const int row = cur.row0 + r0 + e;
                    const bool seen = cur.rs ? vs[e] > my_key : row >= my_key;
                    float p = __builtin_amdgcn_exp2f(s_acc[rb][i]);
                    p = seen ? p : 0.f;
                    pb[rb][half][e] = (__bf16)p;
                    dsb[rb][half][e] = (__bf16)(p * dp_acc[rb][i]);
                }
            }
        };
        // S, dP of half rb: 16 matrix instructions in two groups; `next` requests the fragments that follow the block;
        // SOFT >= 0: P and dS of that (other) half beside them
        auto scores = [&](auto soft_tag, int rb, int slot0, auto next) {
            constexpr int SOFT = decltype(soft_tag)::value;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int slot = slot0 ^ g;
                if (g == 0) load1(rb, 1, slot ^ 1);
                else next(slot ^ 1);
#pragma unroll
                for (int u = 0; u < G; ++u) {
                    s_acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[slot][u], kf[G * g + u], s_acc[rb], 0, 0, 0);
                    if (SOFT == -2 && u == 0) {              // the first block of an iteration: the next iteration's copies
                        __builtin_amdgcn_sched_barrier(0);
                        if (more) issue_piece(nxt, buf ^ 1, g);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (SOFT >= 0) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (all_seen) {                      // (uniform; only the vector work is conditional: a branch
                                                             //  around matrix instructions makes the compiler copy their accumulators)
#pragma unroll
                            for (int k = 0; k < PIECES; ++k) soft2(SOFT, 2 * ((G * g + u) * PIECES + k));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    dp_acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[slot][u], vf[G * g + u], dp_acc[rb], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // dV, dK of half rb: 16 matrix instructions in two groups (rows 16 stp .. + 15 each)
        auto grads = [&](auto soft_tag, int rb, int slot0, auto next) {
            constexpr int SOFT = decltype(soft_tag)::value;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int slot = slot0 ^ g;
                if (g == 0) load2(2 * rb + 1, slot ^ 1);
                else next(slot ^ 1);
#pragma unroll
                for (int u = 0; u < G; ++u) {
                    mfma_into_agprs(dv_acc[u], fo[slot][u], pb[rb][g]);
                    if (SOFT >= 0) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (all_seen) {                      // (uniform; only the vector work is conditional: a branch
                                                             //  around matrix instructions makes the compiler copy their accumulators)
#pragma unroll
                            for (int k = 0; k < PIECES; ++k) soft2(SOFT, 2 * ((G * g + u) * PIECES + k));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    mfma_into_agprs(dk_acc[u], fq[slot][u], dsb[rb][g]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using None = std::integral_constant<int, -1>;
        using Copies = std::integral_constant<int, -2>;
        using Half0 = std::integral_constant<int, 0>;
        using Half1 = std::integral_constant<int, 1>;
        load1(0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        scores(Copies{}, 0, 0, [&](int slot) { load1(1, 0, slot); });
        scores(Half0{}, 1, 0, [&](int slot) { load2(0, slot); });
        if (!all_seen) {
            soft_masked(0);
            soft_masked(1);
        }
        __builtin_amdgcn_sched_barrier(0);
        grads(Half1{}, 0, 0, [&](int slot) { load2(2, slot); });
        grads(None{}, 1, 0, [&](int) {});
    }
    wait_vmcnt<0>();
    // (the matrix instructions above are written as text: the compiler does not know that their results need some
    // cycles before an ordinary instruction may read them)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    if (!active) return;
    uint16_t* pk = dk + keyhead * D;
    uint16_t* pvv = dv + keyhead * D;
    // lane (n, hg), block db, register i  <->  d = 32 db + 8 (i/4) + 4 hg + i%4
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 a4, b4;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                a4[c] = (__bf16)(dk_acc[db][4 * q4 + c] * scale);
                b4[c] = (__bf16)dv_acc[db][4 * q4 + c];
            }
            *reinterpret_cast<bf16x4*>(pk + 32 * db + 8 * q4 + 4 * hg) = a4;
            *reinterpret_cast<bf16x4*>(pvv + 32 * db + 8 * q4 + 4 * hg) = b4;
        }
}

}  // namespace st

using namespace st;

namespace {
inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }
// workspace of the bf16 path: delta (token order) | row statistics | K rows | V rows | Q rows | dO rows
struct BwdLayout {
    size_t delta, stats, krows, vrows, qrows, dorows, total;
};
BwdLayout bwd_layout(const st_plan* plan, int n_q_heads, int n_kv_heads, int head_dim, st_dtype dt) {
    BwdLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += up256(bytes); return at; };
    L.delta = take(size_t(plan->n_tokens) * size_t(n_q_heads) * sizeof(float));
    if (dt == ST_BF16) {
        const size_t tile = size_t(kTileN) * head_dim * sizeof(uint16_t);
        const size_t kvt = size_t(n_kv_heads) * plan->pack_tiles * tile, qt = size_t(n_q_heads) * plan->pack_tiles * tile;
        L.stats = take(size_t(n_q_heads) * plan->pack_tiles * 256 * sizeof(float));
        L.krows = take(kvt);
        L.vrows = take(kvt);
        L.qrows = take(qt);
        L.dorows = take(qt);
    }
    L.total = off + 256;
    return L;
}
}  // namespace

extern "C" size_t st_prefill_bwd_workspace_bytes(const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                                 st_dtype dt) {
    if (!plan || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0) return 0;
    return bwd_layout(plan, n_q_heads, n_kv_heads, head_dim, dt).total;
}

extern "C" st_status st_attn_prefill_bwd(void* dq, void* dk, void* dv, const void* d_out, const void* q, const void* k,
                                         const void* v, const void* out, const float* lse, const st_plan* plan,
                                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float scale, st_dtype dt,
                                         void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dq || !dk || !dv || !d_out || !q || !k || !v || !out || !lse || !plan)
        return fail(ST_ERR_INVALID_ARG, "st_attn_prefill_bwd: null pointer");
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0)
        return fail(ST_ERR_SHAPE, "st_attn_prefill_bwd: n_q_heads %d must be a positive multiple of n_kv_heads %d", n_q_heads, n_kv_heads);
    if (head_dim != 64 && head_dim != 128) return fail(ST_ERR_UNSUPPORTED, "st_attn_prefill_bwd: head_dim %d (64 or 128)", head_dim);
    if (dt != ST_F32 && dt != ST_BF16) return fail(ST_ERR_UNSUPPORTED, "st_attn_prefill_bwd: dtype %d", int(dt));
    if (plan->n_tokens == 0) return ST_OK;
    if (plan->n_tokens * int64_t(n_q_heads) * head_dim >= (int64_t(1) << 31))
        return fail(ST_ERR_SHAPE, "st_attn_prefill_bwd: n_tokens * n_q_heads * head_dim must stay below 2^31 elements");
    const BwdLayout L = bwd_layout(plan, n_q_heads, n_kv_heads, head_dim, dt);
    const size_t need = L.total;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ST_ERR_INVALID_ARG, "st_attn_prefill_bwd: workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < need) return fail(ST_ERR_CAPACITY, "st_attn_prefill_bwd: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    if (scale <= 0.f) scale = 1.f / sqrtf(float(head_dim));
    const int64_t qblocks = int64_t(plan->m_max) * n_q_heads, kblocks = int64_t(plan->m_max) * n_kv_heads;
    if (qblocks > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_prefill_bwd: grid too large");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ST_HIP(plan->wait_built(s));
    const PlanView pv = plan->view();
    float* delta = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + L.delta);
    auto run = [&](auto ttag, auto dtag) -> st_status {
        using T = decltype(ttag);
        constexpr int HD = decltype(dtag)::value;
        const size_t smem = 2 * sizeof(float) * kTileM * (HD + 1);
        ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dq_kernel<T, HD>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
        ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dkv_kernel<T, HD, 0>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
        ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dkv_kernel<T, HD, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem)));
        hipLaunchKernelGGL((bwd_dq_kernel<T, HD>), dim3((unsigned)qblocks), dim3(kTileM), smem, s, (T*)dq, delta, (const T*)d_out, (const T*)q,
                           (const T*)k, (const T*)v, (const T*)out, lse, pv, n_q_heads, n_kv_heads, scale);
        hipLaunchKernelGGL((bwd_dkv_kernel<T, HD, 0>), dim3((unsigned)kblocks), dim3(kTileM), smem, s, (T*)dv, delta, (const T*)d_out,
                           (const T*)q, (const T*)k, (const T*)v, lse, pv, n_q_heads, n_kv_heads, scale);
        hipLaunchKernelGGL((bwd_dkv_kernel<T, HD, 1>), dim3((unsigned)kblocks), dim3(kTileM), smem, s, (T*)dk, delta, (const T*)d_out,
                           (const T*)q, (const T*)k, (const T*)v, lse, pv, n_q_heads, n_kv_heads, scale);
        return ST_OK;
    };
    // bf16: every operand gathered once into 64-row row tiles, then two MFMA kernels
    auto run_mfma = [&](auto dtag) -> st_status {
        constexpr int HD = decltype(dtag)::value;
        unsigned char* w = static_cast<unsigned char*>(workspace);
        auto at = [&](size_t o) { return reinterpret_cast<uint16_t*>(w + o); };
        float* stats = reinterpret_cast<float*>(w + L.stats);
        const unsigned kv_tiles = unsigned(plan->pack_tiles) * n_kv_heads, q_tiles = unsigned(plan->pack_tiles) * n_q_heads;
        hipLaunchKernelGGL((tile_pack_kernel<HD>), dim3(kv_tiles), dim3(256), 0, s, at(L.krows), (uint16_t*)nullptr, (const uint16_t*)k,
                           (const uint16_t*)k, pv, n_kv_heads);
        hipLaunchKernelGGL((tile_pack_kernel<HD>), dim3(kv_tiles), dim3(256), 0, s, at(L.vrows), (uint16_t*)nullptr, (const uint16_t*)v,
                           (const uint16_t*)v, pv, n_kv_heads);
        hipLaunchKernelGGL((tile_pack_kernel<HD>), dim3(q_tiles), dim3(256), 0, s, at(L.qrows), (uint16_t*)nullptr, (const uint16_t*)q,
                           (const uint16_t*)q, pv, n_q_heads);
        hipLaunchKernelGGL((tile_pack_kernel<HD>), dim3(q_tiles), dim3(256), 0, s, at(L.dorows), (uint16_t*)nullptr, (const uint16_t*)d_out,
                           (const uint16_t*)d_out, pv, n_q_heads);
        hipLaunchKernelGGL((bwd_rowstats_kernel<HD>), dim3(q_tiles), dim3(256), 0, s, stats, delta, (const uint16_t*)d_out,
                           (const uint16_t*)out, lse, pv, n_q_heads);
        const size_t smem_q = sizeof(BwdDqSmem<HD>), smem_k = sizeof(BwdDkvSmem<HD>);
        ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dq_mfma_kernel<HD>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem_q)));
        ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_dkv_mfma_kernel<HD>), hipFuncAttributeMaxDynamicSharedMemorySize, int(smem_k)));
        prof_begin(kProfBwdDq, s);
        for (int rep = 0; rep < prof_repeat(); ++rep)
        hipLaunchKernelGGL((bwd_dq_mfma_kernel<HD>), dim3((unsigned)qblocks), dim3(256), smem_q, s, (uint16_t*)dq, (const uint16_t*)d_out,
                           (const uint16_t*)q, at(L.krows), at(L.vrows), lse, delta, pv, n_q_heads, n_kv_heads, scale);
        prof_end(kProfBwdDq, s);
        prof_begin(kProfBwdDkv, s);
        for (int rep = 0; rep < prof_repeat(); ++rep)
        hipLaunchKernelGGL((bwd_dkv_mfma_kernel<HD>), dim3((unsigned)kblocks), dim3(256), smem_k, s, (uint16_t*)dk, (uint16_t*)dv,
                           (const uint16_t*)k, (const uint16_t*)v, at(L.qrows), at(L.dorows), stats, pv,
                           n_q_heads, n_kv_heads, scale);
        prof_end(kProfBwdDkv, s);
        return ST_OK;
    };
    st_status r;
    if (dt == ST_F32) r = head_dim == 64 ? run(float{}, std::integral_constant<int, 64>{}) : run(float{}, std::integral_constant<int, 128>{});
    else r = head_dim == 64 ? run_mfma(std::integral_constant<int, 64>{}) : run_mfma(std::integral_constant<int, 128>{});
    if (r != ST_OK) return r;
    ST_LAUNCH_CHECK("st_attn_prefill_bwd kernels");
    return ST_OK;
}
