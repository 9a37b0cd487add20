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

#include "st_plan.h"

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

}  // namespace st

using namespace st;

extern "C" size_t st_prefill_bwd_workspace_bytes(const st_plan* plan, int32_t n_q_heads) {
    if (!plan || n_q_heads <= 0) return 0;
    return ((size_t(plan->n_tokens) * size_t(n_q_heads) * sizeof(float) + 255) & ~size_t(255)) + 256;
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
    const size_t need = st_prefill_bwd_workspace_bytes(plan, n_q_heads);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ST_ERR_INVALID_ARG, "st_attn_prefill_bwd: workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < need) return fail(ST_ERR_CAPACITY, "st_attn_prefill_bwd: workspace has %zu bytes, needs %zu", workspace_bytes, need);
    if (scale <= 0.f) scale = 1.f / sqrtf(float(head_dim));
    const int64_t qblocks = int64_t(plan->m_max) * n_q_heads, kblocks = int64_t(plan->m_max) * n_kv_heads;
    if (qblocks > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_attn_prefill_bwd: grid too large");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const PlanView pv = plan->view();
    float* delta = static_cast<float*>(workspace);
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
    st_status r;
    if (dt == ST_F32) r = head_dim == 64 ? run(float{}, std::integral_constant<int, 64>{}) : run(float{}, std::integral_constant<int, 128>{});
    else r = head_dim == 64 ? run(uint16_t{}, std::integral_constant<int, 64>{}) : run(uint16_t{}, std::integral_constant<int, 128>{});
    if (r != ST_OK) return r;
    ST_LAUNCH_CHECK("bwd_dq_kernel / bwd_dkv_kernel");
    return ST_OK;
}
