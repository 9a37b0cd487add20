// Device-resident segment tables of one packed batch (internal view of st_plan).
#pragma once
#include <vector>

#include "st_internal.h"

namespace st {

// One query tile of one stream of one sequence, in stream-compact coordinates.
// Block A is the causal block over the row's own stream (SS for source rows, RR
// for reasoning rows); block B is the rectangular source prefix of reasoning rows
// (RS) and is empty for source rows.  Key tiles [0, full) of a block need no mask,
// [full, total) are compared element-wise, the rest is never visited.
struct WorkItem {
    int32_t seq;
    int32_t kind;     // ST_SOURCE / ST_REASONING
    int32_t row0;     // first row, relative to the start of the row's stream
    int32_t n_rows;   // 0 marks an unused slot
    int32_t a_full, a_total;
    int32_t b_full, b_total;
    // everything else a kernel needs about the item's sequence, so that one 64-byte load suffices
    int32_t a_base;   // compact row of column 0 of block A (start of the row's own stream)
    int32_t b_base;   // compact row of column 0 of block B (start of the source stream)
    int32_t n_stream; // tokens of the row's own stream
    int32_t n_src;    // source tokens of the sequence
    int32_t tile_a0;  // packed key tile of column 0 of block A
    int32_t tile_b0;  // packed key tile of column 0 of block B
    int32_t pad0, pad1;
};
static_assert(sizeof(WorkItem) == 64, "WorkItem is one 64-byte record");

struct PlanView {  // what kernels need
    const int32_t* cu;       // [B+1] token offsets
    const int32_t* n_src;    // [B]
    const int32_t* perm;     // [N] compact row -> token index
    const int32_t* vis;      // [N] visible source count per compact row
    const WorkItem* sorted;  // [m_max] work items, longest first (unused slots last)
    int32_t m_max;
    // Packed K / V^T buffers (bf16 path): sequence b owns key tiles [pack_base[b], pack_base[b+1]) of
    // kTileN rows each: first ceil(S / kTileN) source tiles, then the reasoning tiles.
    const int32_t* pack_base;  // [B+1]
    int32_t pack_tiles;        // = pack_base[B]
    int32_t batch;
};

// largest b in [0, batch) with table[b] <= c, for a non-decreasing table of batch + 1 offsets
__device__ __forceinline__ int find_seq(const int32_t* table, int batch, int c) {
    int lo = 0, hi = batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (table[mid] <= c) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace st

struct st_plan {
    int32_t batch = 0;
    int64_t n_tokens = 0;
    int32_t m_max = 0;
    int32_t heads_per_workgroup = 0;   // bf16 attention kernel: 0 = chosen by problem size, 1, 2 (st_plan_heads_per_workgroup)
    std::vector<int32_t> cu_host, slot_base_host, pack_base_host;
    int32_t pack_tiles = 0;
    void* ws = nullptr;
    bool owns_ws = false;
    hipStream_t stream = nullptr;
    hipEvent_t built = nullptr;        // recorded on `stream` behind the kernels that build the tables
    int32_t *cu = nullptr, *slot_base = nullptr, *pack_base = nullptr, *n_src = nullptr, *n_rsn = nullptr;
    int32_t *perm = nullptr, *seg_c = nullptr, *vis = nullptr, *cost = nullptr, *flag = nullptr;
    unsigned long long* pairs = nullptr;
    st::WorkItem* items = nullptr;    // slot order (sequence by sequence)
    st::WorkItem* sorted = nullptr;   // longest first

    // Orders `s` behind the build of the tables (nothing to do on the stream that built them).
    hipError_t wait_built(hipStream_t s) const { return (s == stream || !built) ? hipSuccess : hipStreamWaitEvent(s, built, 0); }

    st::PlanView view() const { return st::PlanView{cu, n_src, perm, vis, sorted, m_max, pack_base, pack_tiles, batch}; }
};
