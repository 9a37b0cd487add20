// Segment-table builder: turns per-token (stream, segment, position) ids into the
// tables that replace the dense additive mask of Eq. 2 (Sec. 3.2; Appendix E.1).
//
// Attention is indifferent to the order of keys, and the streaming mask is a pure
// function of the ids, so everything is expressed in "grouped stream-compact
// order": per sequence, the source tokens by position, then the reasoning tokens
// by position -- the paper's own training layout.  There the mask is two causal
// triangles (source x source, reasoning x reasoning) plus a staircase rectangle
// (reasoning rows x a prefix of the source stream), and a reasoning row needs just
// one number: how many source tokens it sees.
//
// All tables are built by three small integer kernels (init, per-sequence scan, work items), O(N)
// work, no host round trip.
#include <new>

#include "st_plan.h"

namespace st {

static inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

static int32_t m_max_bound(int32_t batch, int64_t n_tokens) { return int32_t(n_tokens / kTileM) + 2 * batch; }

struct WsLayout {
    size_t cu, slot_base, pack_base, n_src, n_rsn, pairs, flag, perm, seg_c, vis, cost, items, sorted, total;
};

static WsLayout ws_layout(int32_t batch, int64_t n_tokens) {
    WsLayout L;
    const size_t m = size_t(m_max_bound(batch, n_tokens));
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    L.cu = take(sizeof(int32_t) * (batch + 1));
    L.slot_base = take(sizeof(int32_t) * (batch + 1));
    L.pack_base = take(sizeof(int32_t) * (batch + 1));
    L.n_src = take(sizeof(int32_t) * batch);
    L.n_rsn = take(sizeof(int32_t) * batch);
    L.pairs = take(sizeof(unsigned long long) * batch);
    L.flag = take(sizeof(int32_t));
    L.perm = take(sizeof(int32_t) * n_tokens);
    L.seg_c = take(sizeof(int32_t) * n_tokens);
    L.vis = take(sizeof(int32_t) * n_tokens);
    L.cost = take(sizeof(int32_t) * m);
    L.items = take(sizeof(WorkItem) * m);
    L.sorted = take(sizeof(WorkItem) * m);
    L.total = off;
    return L;
}

constexpr int kPlanThreads = 1024;
constexpr int kSegLds = 8192;            // source tokens of a sequence whose segment ids are searched in LDS
constexpr int kSortedMax = 4096;          // work items up to which one workgroup builds and orders them
constexpr int kTablesMaxBatch = 64;      // up to this batch the three host tables travel as kernel arguments

struct HostTables {                      // cu_seqlens | item slot bases | packed tile bases, batch + 1 entries each
    int32_t v[3 * (kTablesMaxBatch + 1)];
};

// ---- fill kernel that clears the validation flag (a kernel, so that the build can be recorded into a HIP graph) ----
__global__ void plan_clear_kernel(int32_t* flag) {
    if (threadIdx.x == 0) *flag = 0;
}

__device__ __forceinline__ int block_sum(int v, int* s_wave) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if (lane == 0) s_wave[wave] = v;
    __syncthreads();
    int tot = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) tot += s_wave[w];
    return tot;
}

// ---- kernel 1: one workgroup per sequence ------------------------------------------------------
// (1) rank every token inside its stream -> perm / seg_c in grouped compact order, stream sizes;
// (2) per compact row the number of visible source tokens (binary search over the source segment
//     ids), the visible-pair count of the sequence, and the optional ordering checks.
__global__ __launch_bounds__(kPlanThreads) void plan_sequence_kernel(const int32_t* __restrict__ stream_ids,
                                                                     const int32_t* __restrict__ segment_ids,
                                                                     const int32_t* __restrict__ positions,
                                                                     const int32_t* __restrict__ cu,
                                                                     int32_t* __restrict__ n_src, int32_t* __restrict__ n_rsn,
                                                                     int32_t* __restrict__ perm, int32_t* __restrict__ seg_c,
                                                                     int32_t* __restrict__ vis,
                                                                     unsigned long long* __restrict__ pairs,
                                                                     int32_t* __restrict__ flag, int validate, HostTables tables,
                                                                     int batch, int32_t* __restrict__ cu_out,
                                                                     int32_t* __restrict__ slot_base_out,
                                                                     int32_t* __restrict__ pack_base_out) {
    __shared__ int s_wave[kPlanThreads / 64];
    __shared__ unsigned long long s_pairs[kPlanThreads / 64];
    __shared__ int s_seg[kSegLds];            // segment ids of the source stream: the bisection below stays in LDS
    const int b = blockIdx.x;
    // batch > 0: the host tables travel as a kernel argument (no separate launch to publish them): this kernel reads
    // its offsets from there, and workgroup 0 writes the device copies that every later kernel uses.  batch = 0: the
    // tables were copied to `cu` beforehand.
    const int t0 = batch > 0 ? tables.v[b] : cu[b], t1 = batch > 0 ? tables.v[b + 1] : cu[b + 1];
    if (batch > 0 && b == 0)
        for (int i = threadIdx.x; i <= batch; i += kPlanThreads) {
            cu_out[i] = tables.v[i];
            slot_base_out[i] = tables.v[(batch + 1) + i];
            pack_base_out[i] = tables.v[2 * (batch + 1) + i];
        }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // The ids of the first kPre chunks (8,192 tokens) are fetched once, up front, and serve both passes below, so
    // that the iterations of the rank pass do not each wait for memory.
    constexpr int kPre = 8;
    int pre_stream[kPre], pre_seg[kPre];
#pragma unroll
    for (int j = 0; j < kPre; ++j) {
        const int t = t0 + j * kPlanThreads + threadIdx.x;
        pre_stream[j] = t < t1 ? stream_ids[t] : -1;
        pre_seg[j] = t < t1 ? segment_ids[t] : 0;
    }

    // pass 1: number of source tokens
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < kPre; ++j) {
        const int t = t0 + j * kPlanThreads + threadIdx.x;
        if (t < t1) {
            if (pre_stream[j] != ST_SOURCE && pre_stream[j] != ST_REASONING) atomicOr(flag, 1);
            cnt += (pre_stream[j] == ST_SOURCE);
        }
    }
    for (int t = t0 + kPre * kPlanThreads + threadIdx.x; t < t1; t += kPlanThreads) {
        const int s = stream_ids[t];
        if (s != ST_SOURCE && s != ST_REASONING) atomicOr(flag, 1);
        cnt += (s == ST_SOURCE);
    }
    const int S = block_sum(cnt, s_wave);
    if (threadIdx.x == 0) {
        n_src[b] = S;
        n_rsn[b] = (t1 - t0) - S;
    }
    __syncthreads();

    // pass 2: running rank of source tokens; reasoning rank = index - source rank.  One barrier per chunk: the wave
    // counts go to two buffers used in turn, and every thread keeps the running total itself.
    __shared__ int s_cnt[2][kPlanThreads / 64];
    int total_before = 0;                                    // sources in the chunks already done (same in every thread)
    auto rank_chunk = [&](int parity, int t, int sid, int seg) {
        const bool in = t < t1;
        const bool is_src = in && sid == ST_SOURCE;
        const unsigned long long mask = __ballot(is_src);
        const int before_in_wave = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[parity][wave] = __popcll(mask);
        __syncthreads();
        int before = total_before, all = 0;
        for (int w = 0; w < kPlanThreads / 64; ++w) {
            const int c = s_cnt[parity][w];
            before += w < wave ? c : 0;
            all += c;
        }
        const int src_rank = before + before_in_wave;          // sources strictly before t
        if (in) {
            const int r = is_src ? src_rank : S + ((t - t0) - src_rank);
            perm[t0 + r] = t;
            seg_c[t0 + r] = seg;
        }
        total_before += all;
    };
#pragma unroll
    for (int j = 0; j < kPre; ++j) {
        if (t0 + j * kPlanThreads < t1)                        // (uniform)
            rank_chunk(j & 1, t0 + j * kPlanThreads + threadIdx.x, pre_stream[j], pre_seg[j]);
    }
    for (int base = t0 + kPre * kPlanThreads, j = kPre; base < t1; base += kPlanThreads, ++j) {
        const int t = base + threadIdx.x;
        rank_chunk(j & 1, t, t < t1 ? stream_ids[t] : -1, t < t1 ? segment_ids[t] : 0);
    }
    __threadfence_block();      // perm / seg_c of this sequence are read back below by other threads
    __syncthreads();

    // pass 3: visible source count per compact row, pair count, validation
    const int n = t1 - t0;
    const bool seg_in_lds = S <= kSegLds;      // (a dozen dependent loads per row otherwise go to global memory)
    if (seg_in_lds) {
        for (int i = threadIdx.x; i < S; i += kPlanThreads) s_seg[i] = seg_c[t0 + i];
        __syncthreads();
    }
    unsigned long long mine = 0ull;
    for (int r = threadIdx.x; r < n; r += kPlanThreads) {
        const int c = t0 + r;
        int v;
        if (r < S) {
            v = r + 1;
            mine += (unsigned long long)(r + 1);
        } else {
            const int g = seg_c[c];
            int lo = 0, hi = S;  // first source index whose segment id is > g
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if ((seg_in_lds ? s_seg[mid] : seg_c[t0 + mid]) <= g) lo = mid + 1; else hi = mid;
            }
            v = lo;
            mine += (unsigned long long)v + (unsigned long long)(r - S + 1);
        }
        vis[c] = v;
        if (validate) {
            // neighbours inside one stream: positions strictly increase, segment ids do not decrease
            const bool has_next = (r + 1 < n) && ((r < S) == (r + 1 < S));
            if (has_next) {
                const int p0 = positions[perm[c]], p1 = positions[perm[c + 1]];
                if (!(p0 < p1) || seg_c[c] > seg_c[c + 1]) atomicOr(flag, 2);
            }
            if (positions[perm[c]] < 0 || seg_c[c] < 0) atomicOr(flag, 4);
        }
    }
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
    if (lane == 0) s_pairs[wave] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long tot = 0ull;
        for (int w = 0; w < kPlanThreads / 64; ++w) tot += s_pairs[w];
        pairs[b] = tot;
    }
}

// ---- work items ---------------------------------------------------------------------------------
__device__ __forceinline__ int full_tiles(int limit, int n_cols) {
    // key tiles whose in-range columns are all < limit
    return n_cols <= limit ? (n_cols + kTileN - 1) / kTileN : limit / kTileN;
}

__device__ __forceinline__ WorkItem make_item(int slot, const int32_t* cu, const int32_t* slot_base,
                                              const int32_t* pack_base, int batch, const int32_t* n_src,
                                              const int32_t* n_rsn, const int32_t* vis, int* cost) {
    WorkItem it = {};
    *cost = 0;
    if (slot >= slot_base[batch]) return it;
    const int b = find_seq(slot_base, batch, slot);
    const int local = slot - slot_base[b];
    const int S = n_src[b], R = n_rsn[b];
    const int ts = (S + kTileM - 1) / kTileM, tr = (R + kTileM - 1) / kTileM;
    if (local >= ts + tr) return it;
    const bool src = local < ts;
    const int n_stream = src ? S : R;
    it.seq = b;
    it.kind = src ? ST_SOURCE : ST_REASONING;
    it.row0 = (src ? local : local - ts) * kTileM;
    it.n_rows = min(kTileM, n_stream - it.row0);
    const int last = it.row0 + it.n_rows - 1;
    it.a_total = last / kTileN + 1;
    it.a_full = full_tiles(it.row0 + 1, n_stream);
    it.a_base = cu[b] + (src ? 0 : S);
    it.b_base = cu[b];
    it.n_stream = n_stream;
    it.n_src = S;
    it.tile_b0 = pack_base[b];
    it.tile_a0 = pack_base[b] + (src ? 0 : (S + kTileN - 1) / kTileN);
    if (!src) {
        const int vmin = vis[it.a_base + it.row0], vmax = vis[it.a_base + last];
        it.b_total = (vmax + kTileN - 1) / kTileN;
        it.b_full = full_tiles(vmin, S);
    }
    *cost = it.a_total + it.b_total;
    return it;
}

// ---- kernel 2 (small plans): one workgroup builds every work item and writes them longest first
// (stable rank by counting; unused slots have cost 0 and come last) -----------------------------
__global__ __launch_bounds__(kPlanThreads) void plan_items_sorted_kernel(const int32_t* __restrict__ cu,
                                                                         const int32_t* __restrict__ slot_base,
                                                                         const int32_t* __restrict__ pack_base, int batch,
                                                                         int m_max, const int32_t* __restrict__ n_src,
                                                                         const int32_t* __restrict__ n_rsn,
                                                                         const int32_t* __restrict__ vis,
                                                                         WorkItem* __restrict__ items, int32_t* __restrict__ cost,
                                                                         WorkItem* __restrict__ sorted, int seq_major) {
    __shared__ int s_cost[kSortedMax];
    for (int slot = threadIdx.x; slot < m_max; slot += kPlanThreads) {
        int c;
        const WorkItem it = make_item(slot, cu, slot_base, pack_base, batch, n_src, n_rsn, vis, &c);
        items[slot] = it;
        if (seq_major && c > 0) c = ((batch - 1 - it.seq) << 20) + min(c, (1 << 20) - 1);
        cost[slot] = c;
        s_cost[slot] = c;
    }
    __threadfence_block();
    __syncthreads();
    for (int i = threadIdx.x; i < m_max; i += kPlanThreads) {
        const int ci = s_cost[i];
        int rank = 0;
        for (int j = 0; j < m_max; ++j) {
            const int cj = s_cost[j];
            rank += (cj > ci) || (cj == ci && j < i);
        }
        sorted[rank] = items[i];
    }
}

// ---- kernels 2a / 2b (large plans): the same in two grid-wide steps ---------------------------------
__global__ __launch_bounds__(256) void plan_items_kernel(const int32_t* __restrict__ cu,
                                                         const int32_t* __restrict__ slot_base,
                                                         const int32_t* __restrict__ pack_base, int batch, int m_max,
                                                         const int32_t* __restrict__ n_src,
                                                         const int32_t* __restrict__ n_rsn,
                                                         const int32_t* __restrict__ vis,
                                                         WorkItem* __restrict__ items, int32_t* __restrict__ cost, int seq_major) {
    const int slot = blockIdx.x * 256 + threadIdx.x;
    if (slot >= m_max) return;
    int c;
    const WorkItem it = make_item(slot, cu, slot_base, pack_base, batch, n_src, n_rsn, vis, &c);
    items[slot] = it;
    // sort key: the cost, or -- sequence by sequence, longest first inside each -- the sequence in the high bits
    cost[slot] = (seq_major && c > 0) ? ((batch - 1 - it.seq) << 20) + min(c, (1 << 20) - 1) : c;
}

__global__ __launch_bounds__(256) void plan_order_kernel(const int32_t* __restrict__ cost, int m_max,
                                                         const WorkItem* __restrict__ items,
                                                         WorkItem* __restrict__ sorted) {
    __shared__ int s_cost[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int ci = i < m_max ? cost[i] : 0;
    int rank = 0;
    for (int base = 0; base < m_max; base += 256) {
        const int j = base + threadIdx.x;
        s_cost[threadIdx.x] = j < m_max ? cost[j] : -1;
        __syncthreads();
        const int n = min(256, m_max - base);
        for (int k = 0; k < n; ++k) {
            const int cj = s_cost[k];
            rank += (cj > ci) || (cj == ci && base + k < i);
        }
        __syncthreads();
    }
    if (i < m_max) sorted[rank] = items[i];
}

}  // namespace st

using namespace st;

extern "C" size_t st_plan_workspace_bytes(int32_t batch, int64_t n_tokens) {
    if (batch <= 0 || n_tokens < 0) return 0;
    return ws_layout(batch, n_tokens).total;
}

extern "C" st_status st_plan_create(st_plan** plan_out, const int32_t* segment_ids, const int32_t* stream_ids,
                                    const int32_t* positions, const int32_t* cu_seqlens_host, int32_t batch,
                                    void* workspace, size_t workspace_bytes, int32_t validate, void* hip_stream) {
    if (!plan_out) return fail(ST_ERR_INVALID_ARG, "st_plan_create: plan is null");
    *plan_out = nullptr;
    if (!segment_ids || !stream_ids || !positions || !cu_seqlens_host)
        return fail(ST_ERR_INVALID_ARG, "st_plan_create: null pointer");
    if (batch <= 0) return fail(ST_ERR_INVALID_ARG, "st_plan_create: batch must be positive");
    if (cu_seqlens_host[0] != 0) return fail(ST_ERR_LAYOUT, "st_plan_create: cu_seqlens[0] must be 0");
    for (int b = 0; b < batch; ++b)
        if (cu_seqlens_host[b + 1] < cu_seqlens_host[b])
            return fail(ST_ERR_LAYOUT, "st_plan_create: cu_seqlens must be non-decreasing (entry %d)", b + 1);
    const int64_t n_tokens = cu_seqlens_host[batch];
    const WsLayout L = ws_layout(batch, n_tokens);
    if (workspace) {
        if (reinterpret_cast<uintptr_t>(workspace) & 255u)
            return fail(ST_ERR_INVALID_ARG, "st_plan_create: workspace must be 256-byte aligned");
        if (workspace_bytes < L.total)
            return fail(ST_ERR_CAPACITY, "st_plan_create: workspace has %zu bytes, needs %zu", workspace_bytes, L.total);
    }
    st_plan* p = new (std::nothrow) st_plan();
    if (!p) return fail(ST_ERR_RUNTIME, "st_plan_create: out of host memory");
    p->batch = batch;
    p->n_tokens = n_tokens;
    p->stream = static_cast<hipStream_t>(hip_stream);
    p->cu_host.assign(cu_seqlens_host, cu_seqlens_host + batch + 1);
    p->slot_base_host.resize(batch + 1);
    p->slot_base_host[0] = 0;
    for (int b = 0; b < batch; ++b) {
        const int n = p->cu_host[b + 1] - p->cu_host[b];
        p->slot_base_host[b + 1] = p->slot_base_host[b] + (n + kTileM - 1) / kTileM + 1;
    }
    p->m_max = p->slot_base_host[batch];   // <= m_max_bound(batch, n_tokens)
    // key tiles of the packed K / V^T buffers: ceil(S / 64) + ceil(R / 64) <= ceil(N / 64) + 1 per sequence
    p->pack_base_host.resize(batch + 1);
    p->pack_base_host[0] = 0;
    for (int b = 0; b < batch; ++b) {
        const int n = p->cu_host[b + 1] - p->cu_host[b];
        p->pack_base_host[b + 1] = p->pack_base_host[b] + (n + kTileN - 1) / kTileN + 1;
    }
    p->pack_tiles = p->pack_base_host[batch];
    if (workspace) {
        p->ws = workspace;
    } else {
        hipError_t e = hipMalloc(&p->ws, L.total);
        if (e != hipSuccess) {
            delete p;
            return fail(ST_ERR_RUNTIME, "st_plan_create: hipMalloc(%zu) failed: %s", L.total, hipGetErrorString(e));
        }
        p->owns_ws = true;
    }
    char* w = static_cast<char*>(p->ws);
    p->cu = reinterpret_cast<int32_t*>(w + L.cu);
    p->slot_base = reinterpret_cast<int32_t*>(w + L.slot_base);
    p->pack_base = reinterpret_cast<int32_t*>(w + L.pack_base);
    p->n_src = reinterpret_cast<int32_t*>(w + L.n_src);
    p->n_rsn = reinterpret_cast<int32_t*>(w + L.n_rsn);
    p->pairs = reinterpret_cast<unsigned long long*>(w + L.pairs);
    p->flag = reinterpret_cast<int32_t*>(w + L.flag);
    p->perm = reinterpret_cast<int32_t*>(w + L.perm);
    p->seg_c = reinterpret_cast<int32_t*>(w + L.seg_c);
    p->vis = reinterpret_cast<int32_t*>(w + L.vis);
    p->cost = reinterpret_cast<int32_t*>(w + L.cost);
    p->items = reinterpret_cast<WorkItem*>(w + L.items);
    p->sorted = reinterpret_cast<WorkItem*>(w + L.sorted);

    hipStream_t s = p->stream;
    auto bail = [&](hipError_t e, const char* what) {
        st_status r = fail(ST_ERR_RUNTIME, "st_plan_create: %s failed: %s", what, hipGetErrorString(e));
        st_plan_destroy(p);
        return r;
    };
    hipError_t e;
    HostTables t = {};
    const bool by_value = batch <= kTablesMaxBatch;
    if (by_value) {
        for (int i = 0; i <= batch; ++i) {
            t.v[i] = p->cu_host[i];
            t.v[(batch + 1) + i] = p->slot_base_host[i];
            t.v[2 * (batch + 1) + i] = p->pack_base_host[i];
        }
        // (the validation flag is only read back when validation is asked for: cleared then, by a fill kernel, so
        // that the build can be recorded into a HIP graph)
        if (validate) hipLaunchKernelGGL(plan_clear_kernel, dim3(1), dim3(64), 0, s, p->flag);
    } else {
        // the host vectors live as long as the plan, so the asynchronous copies may read them later
        if ((e = hipMemcpyAsync(p->cu, p->cu_host.data(), sizeof(int32_t) * (batch + 1), hipMemcpyHostToDevice, s)) != hipSuccess)
            return bail(e, "copy of cu_seqlens");
        if ((e = hipMemcpyAsync(p->slot_base, p->slot_base_host.data(), sizeof(int32_t) * (batch + 1), hipMemcpyHostToDevice, s)) != hipSuccess)
            return bail(e, "copy of slot table");
        if ((e = hipMemcpyAsync(p->pack_base, p->pack_base_host.data(), sizeof(int32_t) * (batch + 1), hipMemcpyHostToDevice, s)) != hipSuccess)
            return bail(e, "copy of pack table");
        hipLaunchKernelGGL(plan_clear_kernel, dim3(1), dim3(64), 0, s, p->flag);
    }
    hipLaunchKernelGGL(plan_sequence_kernel, dim3(batch), dim3(kPlanThreads), 0, s, stream_ids, segment_ids, positions, p->cu,
                       p->n_src, p->n_rsn, p->perm, p->seg_c, p->vis, p->pairs, p->flag, validate ? 1 : 0, t, by_value ? batch : 0, p->cu,
                       p->slot_base, p->pack_base);
    // Order of the work items.  Small batches: longest first over the whole batch (best balance at the end of the
    // launch).  From 32K tokens on: sequence by sequence, longest first inside a sequence -- the workgroups running at
    // any time then stream the key / value tiles of ONE sequence, which stay in the caches (on 8 x 16K tokens the
    // attention kernel's HBM fetch falls from 18 GB to 3.5 GB per launch and it runs 7 to 9 % faster; four sequences
    // of 4K tokens lose 2 to 6 % to the worse balance, hence the threshold).
    const bool seq_major = n_tokens >= 32768 && batch > 1 && batch < 2048;
    if (p->m_max <= kSortedMax) {
        hipLaunchKernelGGL(plan_items_sorted_kernel, dim3(1), dim3(kPlanThreads), 0, s, p->cu, p->slot_base, p->pack_base, batch,
                           p->m_max, p->n_src, p->n_rsn, p->vis, p->items, p->cost, p->sorted, seq_major ? 1 : 0);
    } else {
        const int mb = (p->m_max + 255) / 256;
        hipLaunchKernelGGL(plan_items_kernel, dim3(mb), dim3(256), 0, s, p->cu, p->slot_base, p->pack_base, batch, p->m_max,
                           p->n_src, p->n_rsn, p->vis, p->items, p->cost, seq_major ? 1 : 0);
        hipLaunchKernelGGL(plan_order_kernel, dim3(mb), dim3(256), 0, s, p->cost, p->m_max, p->items, p->sorted);
    }
    if ((e = hipGetLastError()) != hipSuccess) return bail(e, "launch of plan kernels");
    // calls that use the plan on another stream wait for this point
    if ((e = hipEventCreateWithFlags(&p->built, hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreateWithFlags");
    if ((e = hipEventRecord(p->built, s)) != hipSuccess) return bail(e, "hipEventRecord");
    if (validate) {
        int32_t flag = 0;
        if ((e = hipMemcpyAsync(&flag, p->flag, sizeof(flag), hipMemcpyDeviceToHost, s)) != hipSuccess)
            return bail(e, "copy of validation flag");
        if ((e = hipStreamSynchronize(s)) != hipSuccess) return bail(e, "hipStreamSynchronize");
        if (flag) {
            st_plan_destroy(p);
            return fail(ST_ERR_LAYOUT,
                        "st_plan_create: malformed token metadata (%s%s%s)", (flag & 1) ? "stream id outside {0,1}; " : "",
                        (flag & 2) ? "positions not strictly increasing or segment ids decreasing inside a stream; " : "",
                        (flag & 4) ? "negative id" : "");
        }
    }
    *plan_out = p;
    return ST_OK;
}

extern "C" void st_plan_destroy(st_plan* plan) {
    if (!plan) return;
    if (plan->owns_ws && plan->ws) (void)hipFree(plan->ws);
    if (plan->built) (void)hipEventDestroy(plan->built);
    delete plan;
}

extern "C" st_status st_plan_heads_per_workgroup(st_plan* plan, int32_t heads) {
    if (!plan) return fail(ST_ERR_INVALID_ARG, "st_plan_heads_per_workgroup: null plan");
    if (heads < 0 || heads > 2) return fail(ST_ERR_INVALID_ARG, "st_plan_heads_per_workgroup: %d (0 = by problem size, 1 or 2)", heads);
    plan->heads_per_workgroup = heads;
    return ST_OK;
}

extern "C" st_status st_plan_tile_shape(const st_plan* plan, int32_t* tile_m, int32_t* tile_n) {
    if (!plan || !tile_m || !tile_n) return fail(ST_ERR_INVALID_ARG, "st_plan_tile_shape: null pointer");
    *tile_m = kTileM;
    *tile_n = kTileN;
    return ST_OK;
}

static st_status fetch(const st_plan* plan, void* dst, const void* src, size_t bytes) {
    if (bytes == 0) return ST_OK;
    ST_HIP(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, plan->stream));
    ST_HIP(hipStreamSynchronize(plan->stream));
    return ST_OK;
}

extern "C" st_status st_plan_stream_counts(const st_plan* plan, int32_t* n_src_host, int32_t* n_rsn_host) {
    if (!plan || !n_src_host || !n_rsn_host) return fail(ST_ERR_INVALID_ARG, "st_plan_stream_counts: null pointer");
    st_status r = fetch(plan, n_src_host, plan->n_src, sizeof(int32_t) * plan->batch);
    if (r != ST_OK) return r;
    return fetch(plan, n_rsn_host, plan->n_rsn, sizeof(int32_t) * plan->batch);
}

extern "C" st_status st_plan_compact_index(const st_plan* plan, int32_t* index_host) {
    if (!plan || !index_host) return fail(ST_ERR_INVALID_ARG, "st_plan_compact_index: null pointer");
    return fetch(plan, index_host, plan->perm, sizeof(int32_t) * plan->n_tokens);
}

extern "C" st_status st_plan_visible_source(const st_plan* plan, int32_t* vis_host) {
    if (!plan || !vis_host) return fail(ST_ERR_INVALID_ARG, "st_plan_visible_source: null pointer");
    return fetch(plan, vis_host, plan->vis, sizeof(int32_t) * plan->n_tokens);
}

extern "C" st_status st_plan_visible_pairs(const st_plan* plan, uint64_t* pairs_host) {
    if (!plan || !pairs_host) return fail(ST_ERR_INVALID_ARG, "st_plan_visible_pairs: null pointer");
    return fetch(plan, pairs_host, plan->pairs, sizeof(uint64_t) * plan->batch);
}

extern "C" st_status st_plan_tile_classes(const st_plan* plan, int32_t seq, int32_t block, uint8_t* classes_host,
                                          int32_t* n_q_tiles, int32_t* n_k_tiles) {
    if (!plan || !n_q_tiles || !n_k_tiles) return fail(ST_ERR_INVALID_ARG, "st_plan_tile_classes: null pointer");
    if (seq < 0 || seq >= plan->batch) return fail(ST_ERR_INVALID_ARG, "st_plan_tile_classes: seq %d out of range", seq);
    if (block != ST_BLOCK_SS && block != ST_BLOCK_RS && block != ST_BLOCK_RR)
        return fail(ST_ERR_INVALID_ARG, "st_plan_tile_classes: block %d", block);
    int32_t S = 0, R = 0;
    st_status r = fetch(plan, &S, plan->n_src + seq, sizeof(int32_t));
    if (r != ST_OK) return r;
    r = fetch(plan, &R, plan->n_rsn + seq, sizeof(int32_t));
    if (r != ST_OK) return r;
    const int ts = (S + kTileM - 1) / kTileM, tr = (R + kTileM - 1) / kTileM;
    const int tq = block == ST_BLOCK_SS ? ts : tr;
    const int tk = ((block == ST_BLOCK_RR ? R : S) + kTileN - 1) / kTileN;
    *n_q_tiles = tq;
    *n_k_tiles = tk;
    if (!classes_host || tq == 0) return ST_OK;
    std::vector<WorkItem> items(tq);
    const int first = plan->slot_base_host[seq] + (block == ST_BLOCK_SS ? 0 : ts);
    r = fetch(plan, items.data(), plan->items + first, sizeof(WorkItem) * tq);
    if (r != ST_OK) return r;
    for (int a = 0; a < tq; ++a) {
        const int full = block == ST_BLOCK_RS ? items[a].b_full : items[a].a_full;
        const int total = block == ST_BLOCK_RS ? items[a].b_total : items[a].a_total;
        for (int c = 0; c < tk; ++c)
            classes_host[size_t(a) * tk + c] = c < full ? ST_TILE_FULL : (c < total ? ST_TILE_PARTIAL : ST_TILE_SKIP);
    }
    return ST_OK;
}
