/*
 * st.h -- C ABI of the streaming-constrained attention library (MI355X / gfx950).
 *
 * The library computes the attention operator of StreamingThinker ("think while
 * reading"): a decoder attends over an INPUT ("source") stream and a REASONING
 * stream such that a reasoning step never sees input sentences that arrive after
 * it (paper Eq. 1, Eq. 2), with position ids counted separately per stream
 * (Sec. 3.2, "Streaming Position Encoding"), and at inference reads two KV
 * caches -- one per stream -- jointly while the source cache keeps growing
 * (Sec. 3.3, "Parallel KV caches"; Appendix E.2, Alg. 1).
 *
 * Conventions common to every call
 *   - Pointers are DEVICE pointers unless the comment says "host".
 *   - Every device buffer is owned by the caller.  The library owns only st_plan
 *     objects and a thread-local error string.
 *   - Calls only ENQUEUE work on `hip_stream` (a hipStream_t passed as void*; NULL
 *     is the default stream) and return without waiting, unless stated otherwise.
 *   - Argument errors are found on the host before anything is launched; the
 *     return value says which kind, st_last_error() gives the text.  Nothing
 *     aborts or throws across this boundary.
 *   - Tensors are dense row-major with the listed dimension order, 16-byte aligned.
 *   - Grouped-query attention: query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - Softmax scale: scale <= 0 selects 1 / sqrt(head_dim).
 *   - head_dim is 64 or 128.
 */
#ifndef ST_H
#define ST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum st_status {
    ST_OK = 0,
    ST_ERR_INVALID_ARG = 1,  /* null / misaligned pointer, negative size */
    ST_ERR_SHAPE = 2,        /* head counts / dims that do not fit together */
    ST_ERR_LAYOUT = 3,       /* malformed token metadata (found by validation) */
    ST_ERR_CAPACITY = 4,     /* append past the page table, workspace too small */
    ST_ERR_UNSUPPORTED = 5,  /* dtype / head_dim / page size the kernels do not cover */
    ST_ERR_RUNTIME = 6       /* a HIP call failed; text in st_last_error() */
} st_status;

/* ST_FP8_E4M3 (OCP FP8 E4M3: bias 7, largest value 448, no infinities) names a STORAGE format of the
 * KV caches only; activations are ST_BF16 or ST_F32. */
typedef enum st_dtype { ST_F32 = 0, ST_BF16 = 1, ST_FP8_E4M3 = 2 } st_dtype;

/* The two streams of the method; also the value set of stream_ids[]. */
typedef enum st_stream_kind { ST_SOURCE = 0, ST_REASONING = 1 } st_stream_kind;

/* Tile classes reported by st_plan_tile_classes. */
enum { ST_TILE_SKIP = 0, ST_TILE_FULL = 1, ST_TILE_PARTIAL = 2 };

/* Blocks of the mask in grouped stream-compact coordinates. */
enum { ST_BLOCK_SS = 0, ST_BLOCK_RS = 1, ST_BLOCK_RR = 2 };

/* Text of the last error on the calling thread; never NULL. */
const char* st_last_error(void);

/* Library version (major * 100 + minor). */
int32_t st_version(void);

/* Optional kernel timing for benchmarks, a property of the CALLING THREAD (like the error text):
 * while the thread has it enabled, its calls bracket these kernels with HIP events on the launch
 * stream -- st_attn_prefill(_rope) the tile packing (ST_PROF_TILE_PACK: the packing kernel, with
 * fused rotation also the table kernel) and the attention kernel (ST_PROF_PREFILL_ATTN),
 * st_attn_decode_dual(_rope, _append) the split kernel (ST_PROF_DECODE_SPLIT), the bf16
 * st_attn_prefill_bwd its two attention kernels (ST_PROF_BWD_DQ, ST_PROF_BWD_DKV),
 * st_attn_source_chunk(_rope) its attention kernel (ST_PROF_SOURCE_CHUNK).  st_profile_read WAITS
 * for the launches the thread recorded, returns their mean duration in milliseconds and their
 * number in host variables, and forgets them.  (Creating events allocates: not under graph capture.)
 * A pair of events around ONE launch also measures the dispatch of that launch and the completion of
 * the second event, several microseconds that are no part of the kernel: st_profile_repeat(n),
 * 1 <= n <= 64, makes the thread's calls, while timing is enabled, launch each timed kernel n times
 * back to back between its two events (every timed kernel writes the same results again), and the
 * reading is the mean over those launches, as a kernel trace reports it.  n = 1 is the default. */
enum { ST_PROF_PREFILL_ATTN = 0, ST_PROF_DECODE_SPLIT = 1, ST_PROF_BWD_DQ = 2, ST_PROF_BWD_DKV = 3,
       ST_PROF_TILE_PACK = 4, ST_PROF_SOURCE_CHUNK = 5 };
void st_profile_enable(int32_t on);
st_status st_profile_repeat(int32_t launches);
/* Wave timeline of the decode split kernel (<= 16 query rows per sequence and KV head, bf16 caches), for the calling
 * thread's calls while timing is enabled: workgroup i of a launch (one wave: one work unit of one cache of one
 * sequence and KV head, in the order sequence, head, unit; units past a cache's length end at once) writes the
 * 100 MHz wall clock at its start and at its end to device_buffer[2 i], device_buffer[2 i + 1] (uint64; device
 * memory of the caller, 16-byte aligned, n_pairs pairs; workgroups beyond n_pairs write nothing).  Every launch
 * overwrites the buffer; a null buffer switches the timeline off.  The results of the call are not affected. */
st_status st_profile_wave_trace(void* device_buffer, int32_t n_pairs);
st_status st_profile_read(int32_t which, double* mean_ms, int32_t* count);

/* ------------------------------------------------------------------------
 * st_rope_apply -- rotary position encoding with caller-supplied (stream-local)
 * position ids.  Sec. 3.2 "Streaming Position Encoding": input tokens and
 * reasoning tokens are numbered independently, both from 0, so that a reasoning
 * token and its input token at the same index have relative rotation R(0).
 *
 *   x, out    : [n_tokens, n_heads, head_dim], dtype dt; out may equal x (in place)
 *   positions : int32 [n_tokens], >= 0
 *   Pairing is (i, i + head_dim/2); angle = position * theta_base^(-2 i / head_dim),
 *   evaluated in fp64 and applied in fp32; bf16 results are rounded to nearest even.
 * ---------------------------------------------------------------------- */
st_status st_rope_apply(void* out, const void* x, const int32_t* positions,
                        int64_t n_tokens, int32_t n_heads, int32_t head_dim,
                        double theta_base, st_dtype dt, void* hip_stream);

/* The queries and the keys of the same tokens in ONE launch: q [n_tokens, n_q_heads, head_dim] and
 * k [n_tokens, n_kv_heads, head_dim] are rotated with the same cos / sin values, evaluated once --
 * the same bits as two st_rope_apply calls.  q_out / k_out may equal q / k. */
st_status st_rope_apply_qk(void* q_out, const void* q, int32_t n_q_heads, void* k_out, const void* k,
                           int32_t n_kv_heads, const int32_t* positions, int64_t n_tokens,
                           int32_t head_dim, double theta_base, st_dtype dt, void* hip_stream);

/* ------------------------------------------------------------------------
 * st_plan -- segment tables of one packed batch, replacing the dense additive
 * mask of Eq. 2.  The mask depends only on the training / prefill instance
 * (Appendix E.1), so one plan serves every layer and head.
 *
 * Visibility rule encoded (Eq. 1; Eq. 2; Alg. 1's N_EOS == N_EOT + 1):
 *   a SOURCE token sees source tokens at positions <= its own;
 *   a REASONING token sees reasoning tokens at positions <= its own, and source
 *   tokens whose segment id is <= its own segment id.
 *
 * Inputs (device int32 [n_tokens], n_tokens = cu_seqlens[batch]):
 *   segment_ids : sentence / reasoning-unit index of each token, >= 0
 *   stream_ids  : ST_SOURCE or ST_REASONING
 *   positions   : stream-local position id
 *   Within one sequence the tokens of each stream must appear in memory in
 *   strictly increasing position order with non-decreasing segment ids; the two
 *   streams may be interleaved or grouped in any way.
 * cu_seqlens : HOST int32 [batch + 1], cu_seqlens[0] = 0, non-decreasing.
 *
 * The plan holds, per sequence, in "grouped stream-compact order" (all source
 * tokens by position, then all reasoning tokens by position):
 *   the token index of every compact row, the number of source tokens each
 *   reasoning row may see, the per-tile SKIP / FULL / PARTIAL extents of the three
 *   mask blocks SS, RS, RR, a longest-first work list, and the visible-pair count.
 * All of it is built by device kernels on hip_stream; st_plan_create itself does
 * not wait for them.  Calls that take the plan on ANOTHER stream are ordered behind
 * the build by the library (an event recorded here, waited for there).
 *
 * workspace: device memory of at least st_plan_workspace_bytes(batch, n_tokens)
 * bytes, 256-byte aligned, which must outlive the plan; or NULL, in which case the
 * plan allocates its own (hipMalloc) and frees it in st_plan_destroy.
 * validate != 0: additionally checks the ordering rules above on the device and
 * WAITS for the result; returns ST_ERR_LAYOUT (and no plan) if they are violated.
 * ---------------------------------------------------------------------- */
typedef struct st_plan st_plan;

size_t st_plan_workspace_bytes(int32_t batch, int64_t n_tokens);

st_status st_plan_create(st_plan** plan,
                         const int32_t* segment_ids, const int32_t* stream_ids,
                         const int32_t* positions, const int32_t* cu_seqlens_host,
                         int32_t batch, void* workspace, size_t workspace_bytes,
                         int32_t validate, void* hip_stream);

/* Frees the plan (and its own workspace, if it allocated one).  The caller must
 * make sure no kernel that uses the plan is still running.  NULL is ignored.
 * A plan that owns its workspace frees device memory here: not while a stream of
 * the process is being captured into a graph (that would invalidate the capture). */
void st_plan_destroy(st_plan* plan);

/* How many query heads of one KV head a workgroup of the bf16 attention kernel serves when
 * st_attn_prefill / st_attn_prefill_rope run with this plan (the backward is not affected):
 * 0 (default) chooses by problem size -- two for sequences of 8K tokens and more on average, else
 * one --, 1 keeps one head per workgroup, 2 serves two wherever n_q_heads / n_kv_heads is even
 * (otherwise one).  Results agree within rounding.  A property of the plan object: set it before
 * the calls that use the plan; other values give ST_ERR_INVALID_ARG. */
st_status st_plan_heads_per_workgroup(st_plan* plan, int32_t heads);

/* Query tile size (rows of a query tile, columns of a key tile). */
st_status st_plan_tile_shape(const st_plan* plan, int32_t* tile_m, int32_t* tile_n);

/* The getters below copy plan tables to HOST buffers and wait for the plan's
 * stream first.  They exist for inspection and bit-exact checks. */

/* n_src[b], n_rsn[b]: tokens per stream; host int32 [batch] each. */
st_status st_plan_stream_counts(const st_plan* plan, int32_t* n_src_host, int32_t* n_rsn_host);
/* compact_index[cu_seqlens[b] + r] = token index (into the packed batch) of compact
 * row r of sequence b: rows [0, n_src) are the source stream, the rest reasoning.
 * host int32 [n_tokens]. */
st_status st_plan_compact_index(const st_plan* plan, int32_t* index_host);
/* visible_source[cu_seqlens[b] + r]: for a reasoning row, the number of source
 * tokens it sees (a prefix of the compact source stream); for a source row r,
 * r + 1.  host int32 [n_tokens]. */
st_status st_plan_visible_source(const st_plan* plan, int32_t* vis_host);
/* visible (query, key) pairs per sequence; host uint64 [batch]. */
st_status st_plan_visible_pairs(const st_plan* plan, uint64_t* pairs_host);
/* Class map of one block (ST_BLOCK_*) of sequence seq, row-major
 * [n_q_tiles][n_k_tiles] uint8 of ST_TILE_*.  Call with classes_host == NULL to
 * get the two counts, then with a buffer of n_q_tiles * n_k_tiles bytes.  The map
 * is expanded from the same per-tile extents the attention kernel loops over. */
st_status st_plan_tile_classes(const st_plan* plan, int32_t seq, int32_t block,
                               uint8_t* classes_host, int32_t* n_q_tiles, int32_t* n_k_tiles);

/* ------------------------------------------------------------------------
 * st_attn_prefill -- streaming-mask attention over a packed batch (prefill /
 * training forward shape).  Sec. 3.2 "Streaming Attention Mask Matrix", Eq. 2:
 * softmax(scale * q k^T + M_streaming) v, with M_streaming given by the plan.
 *
 *   q, out : [n_tokens, n_q_heads, head_dim]      (dtype dt; already rotated)
 *   k, v   : [n_tokens, n_kv_heads, head_dim]
 *   lse    : fp32 [n_tokens, n_q_heads] natural-log softmax denominator, or NULL
 * Key tiles that the plan marks SKIP are never read.  bf16: MFMA products with
 * fp32 accumulation and fp32 softmax state; the queries carry the softmax scale
 * (q * scale * log2(e), rounded to bf16 once more: a perturbation of q of at most
 * half a bf16 unit in the last place, the size of its own quantisation), the
 * probabilities are rounded to bf16 before the second product.  f32: plain fp32
 * arithmetic.
 *
 * workspace (bf16 only): at least st_prefill_workspace_bytes(...) bytes, 256-byte
 * aligned; holds K and V^T regrouped into contiguous key tiles for the duration of
 * the call (about the size of k plus v), and room for the rotation table of
 * st_attn_prefill_rope (head_dim * 4 bytes per token).  Not needed for f32 (may be NULL).
 * ---------------------------------------------------------------------- */
size_t st_prefill_workspace_bytes(const st_plan* plan, int32_t n_kv_heads, int32_t head_dim, st_dtype dt);

st_status st_attn_prefill(void* out, float* lse, const void* q, const void* k, const void* v,
                          const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, float scale, st_dtype dt,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* st_attn_prefill with the rotation of Sec. 3.2 fused in: q and k are UNROTATED and are rotated by
 * positions[token] (device int32 [n_tokens], the stream-local position ids the plan was built
 * from) with base theta_base, as st_rope_apply would -- k on its way into the key tiles, q as the
 * attention kernel loads it -- so neither tensor makes the extra trip through memory.  The angle
 * is reduced in fp64, cos / sin are fp32 (st_rope_apply evaluates them in fp64): a rotated
 * element may differ from st_rope_apply's in its last bf16 bit.  bf16 only (ST_ERR_UNSUPPORTED
 * for f32: rotate with st_rope_apply); theta_base <= 0 or positions == NULL give
 * ST_ERR_INVALID_ARG.  Everything else as for st_attn_prefill, same workspace. */
st_status st_attn_prefill_rope(void* out, float* lse, const void* q, const void* k, const void* v,
                               const int32_t* positions, double theta_base, const st_plan* plan,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float scale,
                               st_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same, taking the token metadata directly: builds a plan, runs the attention,
 * WAITS for it and frees the plan (and a workspace it allocates itself).  For one-off
 * calls; a caller with several layers should create the plan once. */
st_status st_attn_prefill_ids(void* out, float* lse, const void* q, const void* k, const void* v,
                              const int32_t* segment_ids, const int32_t* stream_ids,
                              const int32_t* positions, const int32_t* cu_seqlens_host,
                              int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t head_dim, float scale, st_dtype dt, void* hip_stream);

/* ------------------------------------------------------------------------
 * st_attn_prefill_bwd -- gradients of st_attn_prefill (streaming-constrained training,
 * Sec. 3.2: the mask of Eq. 2 is applied in the forward pass of fine-tuning, so only visible
 * pairs carry gradient).
 *
 *   d_out        : [N, n_q_heads,  head_dim]   dL / d out
 *   q, out       : [N, n_q_heads,  head_dim]   the forward's input and output
 *   k, v         : [N, n_kv_heads, head_dim]
 *   lse          : fp32 [N, n_q_heads]         the forward's log-sum-exp (natural log)
 *   dq           : [N, n_q_heads,  head_dim]   (written)
 *   dk, dv       : [N, n_kv_heads, head_dim]   (written; summed over the query heads of a KV group)
 * all of dtype dt, same plan as the forward.  Deterministic (no atomics).
 * ST_BF16: products on the matrix cores (bf16 operands -- P and dS are rounded to bf16 before the
 * second products, as the forward rounds P -- fp32 accumulation); every operand is first gathered
 * into 64-row tiles in the workspace, which therefore holds about 1.1x the bytes of q, k, v, d_out.
 * ST_F32: a plain one-thread-per-row path in fp32, not tuned.
 * workspace: at least st_prefill_bwd_workspace_bytes(plan, n_q_heads, n_kv_heads, head_dim, dt)
 * bytes, 256-byte aligned.  Errors as for st_attn_prefill.
 * ---------------------------------------------------------------------- */
size_t st_prefill_bwd_workspace_bytes(const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads,
                                      int32_t head_dim, st_dtype dt);

st_status st_attn_prefill_bwd(void* dq, void* dk, void* dv, const void* d_out, const void* q,
                              const void* k, const void* v, const void* out, const float* lse,
                              const st_plan* plan, int32_t n_q_heads, int32_t n_kv_heads,
                              int32_t head_dim, float scale, st_dtype dt,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------
 * Paged KV caches.  Sec. 3.3: a source cache for input tokens and a separate
 * cache for reasoning tokens.  Logical position p of sequence b lives in page
 * page_table[b * max_pages_per_seq + p / 16], slot p % 16.  bf16 only.
 *
 * Pool layouts (fixed; chosen so that the decode kernel's matrix-core operands are
 * contiguous 16-byte loads), with c = d / 8, e = d % 8:
 *   k_pool : [n_pages][n_kv_heads][head_dim / 8][16 slots][8]   element (page,h,c,slot,e)
 *   v_pool : [n_pages][n_kv_heads][head_dim][16 slots]          element (page,h,d,slot)
 * appended_len[b] is advanced only by st_kv_append.
 *
 * 8-bit caches (dtype = ST_FP8_E4M3; a storage variant, not in the paper): every row -- one token
 * of one KV head, keys and values separately -- is stored as E4M3 codes of the row divided by a
 * power of two 2^k, k the smallest integer (not below -100) for which the row's largest magnitude
 * is at most 448, and 2^k is kept as an fp32 number beside it (k = 0 for an all-zero row).  The
 * division is exact, the rounding is to nearest, ties to even.  Layouts, 1 byte per element:
 *   k_pool  : [n_pages][n_kv_heads][head_dim / 16][16 slots][16]
 *   v_pool  : [n_pages][n_kv_heads][head_dim][16 slots]
 *   k_scale, v_scale : fp32 [n_pages][n_kv_heads][16 slots]
 * st_kv_append (bf16 rows in, quantised on the way) and st_attn_decode_dual(_rope) with
 * q_len * (n_q_heads / n_kv_heads) <= 16 accept them; every other call that takes a cache gives
 * ST_ERR_UNSUPPORTED.  Both caches of a pair must have the same dtype.
 * ---------------------------------------------------------------------- */
typedef struct st_kv_cache {
    void* k_pool;
    void* v_pool;
    const int32_t* page_table; /* device int32 [batch][max_pages_per_seq] */
    int32_t* appended_len;     /* device int32 [batch] */
    int32_t max_pages_per_seq;
    int32_t n_pages;           /* pages in the pools (page ids must be < n_pages) */
    int32_t page_size;         /* must be 16 */
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;             /* st_dtype of the pools: ST_BF16 or ST_FP8_E4M3 */
    float* k_scale;            /* ST_FP8_E4M3 only (NULL otherwise): row scales, see above */
    float* v_scale;
} st_kv_cache;

typedef struct st_dual_cache {
    st_kv_cache source;
    st_kv_cache reasoning;
} st_dual_cache;

/* ------------------------------------------------------------------------
 * st_kv_append -- append tokens to the source or the reasoning cache.
 * Sec. 3.3 / Alg. 1: arriving input sentences are stored in the source cache in
 * arrival order; decoded reasoning tokens are stored in the reasoning cache.
 *
 *   k_new, v_new : bf16 [batch, max_new, n_kv_heads, head_dim] (already rotated)
 *   n_new        : device int32 [batch], tokens to take from each row of k_new
 *                  (0 .. max_new), or NULL for max_new everywhere
 *   host_len_upper_bound : the caller's bound on max_b(appended_len[b] + n_new[b]);
 *                  more than max_pages_per_seq * 16 gives ST_ERR_CAPACITY without
 *                  touching the device.  Tokens that would still fall outside the
 *                  page table on the device are dropped, never written.
 * Page-table entries for the pages written must be valid before the call.
 * Writes only slots [appended_len, appended_len + n_new) and then advances
 * appended_len; it may run on another stream concurrently with
 * st_attn_decode_dual as long as the decode's src_visible_len does not reach into
 * the range being written.
 * ---------------------------------------------------------------------- */
st_status st_kv_append(const st_dual_cache* caches, st_stream_kind which,
                       const void* k_new, const void* v_new, const int32_t* n_new,
                       int32_t max_new, int32_t batch, int32_t host_len_upper_bound,
                       void* hip_stream);

/* ------------------------------------------------------------------------
 * st_kv_append_rope -- st_kv_append with the rotation fused in.
 * Sec. 3.2 "Streaming Position Encoding": the tokens of each stream are numbered
 * from 0 independently of the other stream, so the position id of a token is its
 * index in its own cache and a key, once rotated and stored, is never rotated
 * again.  k_new holds UNROTATED keys; key i of sequence b is rotated by position
 * appended_len[b] + i with base theta_base (same pairing (i, i + D/2) and angle as
 * st_rope_apply; the angle is reduced in fp64, cos / sin are fp32) and stored;
 * v_new is stored as it is.  All other arguments, limits and errors as for
 * st_kv_append; theta_base <= 0 gives ST_ERR_INVALID_ARG.
 * ---------------------------------------------------------------------- */
st_status st_kv_append_rope(const st_dual_cache* caches, st_stream_kind which,
                            const void* k_new, const void* v_new, const int32_t* n_new,
                            int32_t max_new, int32_t batch, int32_t host_len_upper_bound,
                            double theta_base, void* hip_stream);

/* ------------------------------------------------------------------------
 * st_attn_decode_dual -- one decode step over both caches.  Alg. 1: the slice of
 * the source cache that keeps N_EOS == N_EOT + 1 and the reasoning cache are read
 * as one merged cache.  Here nothing is copied: partial softmaxes over chunks of
 * either cache are merged by log-sum-exp, which equals attention over the
 * concatenation.
 *
 *   q, out : bf16 [batch, q_len, n_q_heads, head_dim]
 *   lse    : fp32 [batch, q_len, n_q_heads] or NULL
 *   src_visible_len[b] : source tokens visible to this step (the caller's snapshot,
 *                        NOT the cache's appended_len; 0 allowed)
 *   rsn_len[b]         : reasoning tokens including the q_len tokens being decoded
 *                        (they are appended first); row t of q_len sees reasoning
 *                        tokens [0, rsn_len - q_len + t]
 *   q_len * (n_q_heads / n_kv_heads) must be <= 32.
 *   max_src_len / max_rsn_len : host upper bounds on the two length vectors (grid size).
 * A row that sees nothing (both lengths 0) gets out = 0, lse = -inf.  Cache slots
 * outside the visible ranges are never used, whatever bit patterns they hold.
 * workspace: at least st_decode_workspace_bytes(...) bytes, 256-byte aligned.
 * ---------------------------------------------------------------------- */
typedef struct st_dual_lens {
    const int32_t* src_visible_len; /* device int32 [batch] */
    const int32_t* rsn_len;         /* device int32 [batch] */
    int32_t q_len;
    int32_t max_src_len;
    int32_t max_rsn_len;
    int32_t unit_tokens;            /* tokens per work unit of the step, see below; 0 = chosen by launch size */
} st_dual_lens;

/* Work units.  A step with q_len * (n_q_heads / n_kv_heads) <= 16 cuts each cache into units of
 * lens->unit_tokens tokens, one wave each: 0 chooses by launch size -- 1024 for large batches down
 * to 128 for a few sequences, whose step is bound by a wave's serial walk over its unit --, 128,
 * 256, 512 or 1024 pins it (tests, tuning); other values give ST_ERR_INVALID_ARG.  Results agree
 * within rounding.  st_decode_workspace_bytes takes the same value and answers for it (and always
 * provides for 512-token units).  A workspace sized for other length bounds or another unit is
 * accepted as long as it holds 512-token units; the call then uses the smallest unit not below the
 * wanted one that the workspace has room for.  0 bytes are returned for arguments that make no sense. */
size_t st_decode_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                 int32_t head_dim, int32_t q_len,
                                 int32_t max_src_len, int32_t max_rsn_len, int32_t unit_tokens);

st_status st_attn_decode_dual(void* out, float* lse, const void* q,
                              const st_dual_cache* caches, const st_dual_lens* lens,
                              int32_t batch, int32_t n_q_heads, float scale,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* st_attn_decode_dual for callers that cannot allocate device memory or hand over a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * partial results live in a device array that is part of the library's code object
 * (st_decode_static_scratch_bytes() bytes -- 64 MiB -- on every GPU the library is used on, held
 * until the process ends); the call itself allocates nothing and frees nothing.  Same arguments,
 * kernels and results as st_attn_decode_dual.  A step whose partial results (for 512-token work
 * units: what st_attn_decode_dual demands of its workspace) do not fit the array gives
 * ST_ERR_CAPACITY and launches nothing.  All calls on one GPU share that GPU's array: two such
 * calls that overlap in time on one GPU (different streams or threads) race; calls on one stream
 * are ordered.  Nothing in the array needs clearing between calls. */
size_t st_decode_static_scratch_bytes(void);

st_status st_attn_decode_dual_static(void* out, float* lse, const void* q,
                                     const st_dual_cache* caches, const st_dual_lens* lens,
                                     int32_t batch, int32_t n_q_heads, float scale, void* hip_stream);

/* st_attn_decode_dual with the query rotation fused in (Sec. 3.2): q holds UNROTATED
 * queries; row t of sequence b is the reasoning token at index rsn_len[b] - q_len + t of
 * its stream (already appended, Alg. 1), and is rotated by that position id with base
 * theta_base before it is used.  Everything else as for st_attn_decode_dual;
 * theta_base <= 0 gives ST_ERR_INVALID_ARG. */
st_status st_attn_decode_dual_rope(void* out, float* lse, const void* q,
                                   const st_dual_cache* caches, const st_dual_lens* lens,
                                   int32_t batch, int32_t n_q_heads, float scale, double theta_base,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* One decoding step in one call (Alg. 1, decoding loop: the new token's key and value are stored
 * in the reasoning cache, then the token attends over both caches): the same result as
 *   st_kv_append[_rope](caches, ST_REASONING, k_new, v_new, NULL, 1, ...) followed by
 *   st_attn_decode_dual[_rope](out, lse, q, caches, lens, ...)
 * for q_len = 1, within rounding.  lens->rsn_len[b] is the length of sequence b's reasoning stream
 * INCLUDING the new token, as for st_attn_decode_dual: the token is stored at index
 * rsn_len[b] - 1 and reasoning.appended_len[b] becomes rsn_len[b] (the caller's lengths are
 * authoritative here; with rsn_len[b] = 0 nothing is stored for sequence b and its length stays).
 *   q            : [batch, 1, n_q_heads, head_dim] bf16 device
 *   k_new, v_new : [batch, 1, n_kv_heads, head_dim] bf16 device, 16-byte aligned
 *   theta_base   : > 0: q and k_new are UNROTATED and are rotated by the token's position id
 *                  rsn_len[b] - 1 (Sec. 3.2); 0: both are already rotated
 * When both caches are short (max_src_len + max_rsn_len <= 1024) the step is ONE kernel launch:
 * the workgroup that attends for a KV head also stores that head's key and value, and takes the
 * new token from registers.  Longer caches take two launches (the split kernel stores the token
 * through one more work unit per sequence and KV head and merges it as one more partial state;
 * with more than 16 query heads per KV head the token goes in with a launch of its own).
 * lens->q_len other than 1 and 8-bit caches give ST_ERR_UNSUPPORTED.  Everything else (workspace,
 * bounds, errors) as for st_attn_decode_dual. */
st_status st_attn_decode_dual_append(void* out, float* lse, const void* q, const void* k_new,
                                     const void* v_new, const st_dual_cache* caches,
                                     const st_dual_lens* lens, int32_t batch, int32_t n_q_heads,
                                     float scale, double theta_base, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------
 * st_attn_source_chunk -- attention of an arriving source chunk over the paged source
 * cache.  Alg. 1, prefill loop; Sec. 3.3 "Parallel KV caches": every arriving input sentence is
 * run through the model in arrival order and its keys / values go to the source cache; its
 * tokens attend causally to the source stream only, never to reasoning.
 *
 * Call order: st_kv_append(ST_SOURCE, chunk) first, then this call with
 *   src_len[b]  : device int32 [batch], source tokens in the cache INCLUDING the chunk
 *   n_new[b]    : device int32 [batch], tokens of the chunk (0 .. max_new), or NULL for max_new
 *   q, out      : bf16 [batch, max_new, n_q_heads, head_dim]; row t < n_new[b] sees source
 *                 positions [0, src_len[b] - n_new[b] + t]; rows t >= n_new[b] are not written
 *   lse         : fp32 [batch, max_new, n_q_heads] or NULL
 *   max_src_len : host upper bound on src_len
 * The reasoning cache of `caches` is not touched.  The same machinery as the decode step
 * (split over 512-token chunks of the cache, log-sum-exp merge) with the queries cut into
 * blocks of 32 (token, head) rows.
 * workspace: at least st_source_chunk_workspace_bytes(...) bytes, 256-byte aligned.
 * ---------------------------------------------------------------------- */
size_t st_source_chunk_workspace_bytes(int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                       int32_t head_dim, int32_t max_new, int32_t max_src_len);

st_status st_attn_source_chunk(void* out, float* lse, const void* q, const st_dual_cache* caches,
                               const int32_t* src_len, const int32_t* n_new, int32_t max_new,
                               int32_t max_src_len, int32_t batch, int32_t n_q_heads, float scale,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* st_attn_source_chunk with the query rotation fused in (Sec. 3.2): q holds UNROTATED
 * queries; row t of sequence b is the source token at index src_len[b] - n_new[b] + t of the
 * source stream and is rotated by that position id with base theta_base.  Together with
 * st_kv_append_rope the prefill loop of Alg. 1 then needs no separate rotation pass.
 * theta_base <= 0 gives ST_ERR_INVALID_ARG; everything else as for st_attn_source_chunk. */
st_status st_attn_source_chunk_rope(void* out, float* lse, const void* q, const st_dual_cache* caches,
                                    const int32_t* src_len, const int32_t* n_new, int32_t max_new,
                                    int32_t max_src_len, int32_t batch, int32_t n_q_heads, float scale,
                                    double theta_base, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------
 * Alg. 1 ("Streaming thinking with parallel KV caches") as a host scheduler.
 *
 * st_stream_run drives the attention path of n_layers layers through one streaming session
 * of a batch of identical streams: input sentence k has src_tokens[k] tokens and becomes
 * available arrival_s[k] seconds after the start; reasoning unit k has rsn_tokens[k] tokens
 * (Alg. 1 takes the source and target length lists as input).  Schedules:
 *   ST_SCHED_STREAMING  Alg. 1: a prefill loop (host thread + prefill_stream) appends every
 *                       sentence as soon as it has arrived and lets it attend over the source
 *                       cache; a decoding loop (host thread + decode_stream) starts unit t when
 *                       unit t-1 has ended and sentence t is prefilled (N_EOS >= N_EOT + 1): it
 *                       waits for the prefill if necessary, and selects the slice of the source
 *                       cache ending with sentence t if later sentences are already cached.
 *   ST_SCHED_SERIAL     one worker alternates: prefill sentence k, decode unit k.  Same results
 *                       as ST_SCHED_STREAMING, bit for bit.
 *   ST_SCHED_BATCH      the batch paradigm: wait for the last sentence, prefill everything,
 *                       then decode every unit with the WHOLE input visible.
 * The keys and queries are given unrotated and are rotated inside the kernels by their index in
 * their stream (st_kv_append_rope, st_attn_source_chunk_rope, st_attn_decode_dual_append).
 * Every layer is fed the same activations (projections and MLP need weights and are outside this
 * path); outputs are those of the last layer.  All caches must be empty at the start.
 *
 * Tensor layouts (device, bf16), with S_k = src_tokens[k], step g = decoded token number g overall:
 *   src_q, src_out : concatenation over k of [batch, S_k, n_q_heads,  head_dim]
 *   src_k, src_v   : concatenation over k of [batch, S_k, n_kv_heads, head_dim]
 *   rsn_q, rsn_out : [total steps][batch, n_q_heads,  head_dim]
 *   rsn_k, rsn_v   : [total steps][batch, n_kv_heads, head_dim]
 * Workspaces: prefill_workspace >= st_source_chunk_workspace_bytes(batch, n_q_heads, n_kv_heads,
 * head_dim, max_k S_k, sum_k S_k), decode_workspace >= st_decode_workspace_bytes(batch, ..., 1,
 * sum_k S_k, total steps); the two are used concurrently and must not overlap.
 * The call BLOCKS until the session has run; it creates host threads and a few device words of
 * its own.  report: host arrays of n_sentences entries each, seconds since the start (GPU event
 * times): prefill_done_s, first_token_s, unit_done_s; waited[t] = the decoding loop found sentence
 * t not yet prefilled, sliced[t] = it found sentence t+1 already prefilled; total_s = wall time.
 * ---------------------------------------------------------------------- */
enum { ST_SCHED_STREAMING = 0, ST_SCHED_SERIAL = 1, ST_SCHED_BATCH = 2 };

typedef struct st_stream_job {
    int32_t n_layers;
    int32_t batch;
    int32_t n_q_heads;
    int32_t n_sentences;
    const st_dual_cache* caches;   /* host array [n_layers] */
    const int32_t* src_tokens;     /* host [n_sentences] */
    const int32_t* rsn_tokens;     /* host [n_sentences] */
    const double* arrival_s;       /* host [n_sentences], non-decreasing, or NULL (everything present at the start) */
    const void* src_q;
    const void* src_k;
    const void* src_v;
    void* src_out;
    const void* rsn_q;
    const void* rsn_k;
    const void* rsn_v;
    void* rsn_out;
    float scale;                   /* <= 0: 1 / sqrt(head_dim) */
    double theta_base;
    void* prefill_workspace;
    size_t prefill_workspace_bytes;
    void* decode_workspace;
    size_t decode_workspace_bytes;
    void* prefill_stream;          /* hipStream_t */
    void* decode_stream;           /* hipStream_t, different from prefill_stream for ST_SCHED_STREAMING */
    int32_t decode_graph;          /* != 0: one decoded token (all layers) is recorded into a HIP graph once and
                                      replayed per token (small batches are bound by launch gaps otherwise); the
                                      session falls back to plain launches if the recording fails.  Results agree
                                      with decode_graph = 0 within rounding (the work is cut into units for the
                                      longest reasoning cache of the session instead of the current one). */
} st_stream_job;

typedef struct st_stream_report {
    double* prefill_done_s;
    double* first_token_s;
    double* unit_done_s;
    int32_t* waited;
    int32_t* sliced;
    double total_s;
} st_stream_report;

st_status st_stream_run(const st_stream_job* job, int32_t mode, st_stream_report* report);

/* The control logic of the three schedules as a pure host model (no GPU): event times for given
 * stage durations -- sentence k takes prefill_s[k] to prefill, every decoded token decode_s -- with
 * the two loops of ST_SCHED_STREAMING on resources of their own.  Output arrays (n_sentences
 * entries each) may be NULL.  unit_start_s[t] = max(end of unit t-1, prefill of sentence t). */
st_status st_stream_timeline(int32_t mode, int32_t n_sentences, const double* arrival_s,
                             const double* prefill_s, const int32_t* n_decode, double decode_s,
                             double* prefill_done_s, double* unit_start_s, double* first_token_s,
                             double* unit_done_s, int32_t* waited, int32_t* sliced);

#ifdef __cplusplus
}
#endif
#endif /* ST_H */
