// Packed 64-row operand tiles and their way into LDS, shared by the forward and the backward attention kernels.
//
// tile_pack_kernel gathers, for every 64-row tile of a stream (stream-compact order) and every head, the rows of
// one tensor as a "row tile" ([64 rows][D], rows parked in the order the first-type MFMA wants, 16-byte chunks
// XOR-swizzled) and the rows of a second tensor as a "transposed tile" ([D][64 rows], swizzled), 16 KB each at
// D = 128, contiguous -- so that a kernel streams tiles with plain linear copies and needs no per-row token lookup
// and no transpose in its inner loop.  Either destination may be null (that half is skipped).  The forward packs
// (K rows, V^T); the backward packs row tiles only (K, V, Q, dO) and takes its transposed operands out of them with
// transposing LDS reads (TrOffsets below).
#pragma once
#include "st_plan.h"

namespace st {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// One wave-wide asynchronous copy global -> LDS: lane l's 16 bytes at `g` land at LDS byte offset
// lds_off + 16 l (lds_off must be wave-uniform).  Completion is counted by vmcnt like any load.
__device__ __forceinline__ void async_copy16(const void* g, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_off) : "memory", "m0");
}
// the same with the non-temporal hint: for bytes that are read once
__device__ __forceinline__ void async_copy16_nt(const void* g, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_off) : "memory", "m0");
}
// the same with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit byte offset per lane
__device__ __forceinline__ void async_copy16_s(const void* base, uint32_t lane_off, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
}
// NL wave-wide 16-byte copies global -> LDS, 1 KB apart on both sides: the instruction's immediate offset moves
// the global address and the LDS address alike, so the LDS base goes into m0 once.
template <int NL>
__device__ __forceinline__ void async_copy_rows(const void* base, uint32_t lane_off, uint32_t lds_off) {
    static_assert(NL == 2 || NL == 4, "tile sizes of head_dim 64 and 128");
    if constexpr (NL == 4)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024\n\t"
                     "global_load_lds_dwordx4 %0, %1 offset:2048\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072"
                     ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024"
                     ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
}

// NL such copies 1 KB apart on both sides, read-once bytes: the instruction's immediate offset moves the global and
// the LDS address alike, so the LDS base goes into m0 once
template <int NL>
__device__ __forceinline__ void async_copy_rows_nt(const void* base, uint32_t lane_off, uint32_t lds_off) {
    static_assert(NL == 2 || NL == 4, "pages of head_dim 64 and 128");
    if constexpr (NL == 4)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024 nt\n\t"
                     "global_load_lds_dwordx4 %0, %1 offset:2048 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072 nt"
                     ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024 nt"
                     ::"v"(lane_off), "s"(base), "s"(lds_off) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS tiles of the MFMA kernel: no padding; inside every row the 16-byte chunks are stored at
// position chunk ^ key(row).  The LDS has 64 four-byte banks, so a 16-byte operand read serves 16
// lanes (16 consecutive rows) per cycle, and the key must send those 16 rows to 16 different
// 16-byte columns of the 256-byte bank line: for 256-byte rows the key is row % 16 with its two
// 2-bit halves exchanged -- any one-to-one key serves the 16-byte reads, and this one also sends
// four CONSECUTIVE rows to four different 64-byte quarters of the bank line, which is what the
// transposing reads below (four rows x 64 bytes per pass) need; (row / 2) % 8 for 128-byte rows
// (two rows per bank line).  The packed global tiles already have this arrangement, so a tile
// travels global -> LDS as a plain linear copy.
template <int ROW_BYTES>
__device__ __forceinline__ int swizzle_key(int row) {
    return ROW_BYTES == 256 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((row >> 1) & 7);
}

// A transposed operand fragment straight out of a ROW tile ([64 rows][D], rows parked in swap23 order, chunks
// swizzled as above): ds_read_b64_tr_b16 gives lane l of a 16-lane group, as its element j, the (l % 4)-th 16-bit
// value of the 8 bytes that lane 4 j + l / 4 of the group points at.  With lane i of a group pointing at row
// i / 4, columns 4 (i % 4) .. + 3 of a 4-row x 16-column block, every lane receives one COLUMN of the block: two
// such reads (rows 0-3 and 4-7 of an 8-row group) are the eight k-values of an A operand whose M index runs
// along the tile's columns.  TrOffsets holds a lane's element offsets inside a 16-row step for the two reads
// and every 32-column block; the step's first row (a multiple of 16) is added as a constant.
template <int D>
struct TrOffsets {
    int off[2][D / 32];
    __device__ __forceinline__ explicit TrOffsets(int lane) {
        const int l16 = lane & 15, mg = (lane >> 4) & 1, hg = lane >> 5;
        const int j = l16 >> 2, cm = 2 * mg + ((l16 & 3) >> 1);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            // logical row 8 hg + 4 t + j of the step sits at position 8 t + 4 hg + j (bits 2 and 3 swapped)
            const int lr = 8 * t + 4 * hg + j;
#pragma unroll
            for (int u = 0; u < D / 32; ++u) off[t][u] = lr * D + ((4 * u + cm) ^ swizzle_key<2 * D>(lr)) * 8 + 4 * (l16 & 1);
        }
    }
    // columns 32 u .. 32 u + 31 (M index = lane % 32), rows 16 step .. + 15 (k index 8 (lane / 32) .. + 7) of `tile`
    __device__ __forceinline__ bf16x8 fragment(const uint16_t* tile, int step, int u) const {
        typedef __bf16 lds_bf16x4 __attribute__((ext_vector_type(4), address_space(3)));
        const uint16_t* p = tile + step * 16 * D;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + off[0][u]));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + off[1][u]));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

// swap bits 2 and 3: the row order in which K is parked in LDS, so that after the
// first MFMA each half-wave holds 8 CONSECUTIVE keys per 16-key step
__device__ __forceinline__ int swap23(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

template <int D>
__global__ __launch_bounds__(256) void tile_pack_kernel(uint16_t* __restrict__ kc, uint16_t* __restrict__ vc,
                                                           const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v, PlanView pv,
                                                           int n_kv_heads) {
    constexpr int KCH = D / 8;
    constexpr int K_PER_THREAD = kTileN * KCH / 256;
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
    // K rows, parked in the row order the first MFMA wants (bits 2 and 3 of the row swapped) and with
    // the chunk swizzle of the LDS tile; rows past the end of the stream are zero (they are masked,
    // but must be finite)
    if (kc != nullptr)
#pragma unroll
    for (int u = 0; u < K_PER_THREAD; ++u) {
        const int c = tid + 256 * u;
        const int row = c / KCH, ch = c % KCH;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (row < valid) val = *reinterpret_cast<const u32x4*>(k + (uint32_t(pv.perm[base + row]) * row_stride + uint32_t(h) * D + ch * 8));
        const int lr = swap23(row);                                    // row position in the tile
        *reinterpret_cast<u32x4*>(kdst + lr * D + (ch ^ swizzle_key<2 * D>(lr)) * 8) = val;
    }
    // V: 8 keys x 8 d per thread (16-byte loads), transposed in registers to 8 d x 8 keys (16-byte stores)
    const int kvb = tid & 7, dq = tid >> 3;
    if (vc != nullptr && dq < D / 8) {
        u32x4 vreg[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int row = kvb * 8 + r;
            vreg[r] = u32x4{0u, 0u, 0u, 0u};
            if (row < valid) vreg[r] = *reinterpret_cast<const u32x4*>(v + (uint32_t(pv.perm[base + row]) * row_stride + uint32_t(h) * D + dq * 8));
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {                 // word w of every row holds d = 2 w and 2 w + 1
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


}  // namespace st
