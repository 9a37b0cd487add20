// Alg. 1 ("Streaming thinking with parallel KV caches") as a host scheduler over the attention path.
//
// Two loops run side by side, each on a HIP stream and a host thread of its own:
//   prefill loop  -- when input sentence k has arrived, its keys / values are appended to the source
//                    cache of every layer (rotated on the way in) and its tokens attend causally over
//                    that cache (st_kv_append_rope + st_attn_source_chunk_rope); an event marks the
//                    sentence as prefilled (N_EOS = k + 1);
//   decoding loop -- reasoning unit t starts when unit t - 1 has ended and sentence t is prefilled
//                    (N_EOS >= N_EOT + 1).  If the prefill is not there yet the loop waits for its event;
//                    if later sentences are already cached it selects the slice of the source cache that
//                    ends with sentence t (src_visible_len).  Each token is appended to the reasoning
//                    cache and attends over both caches (st_attn_decode_dual_append: one launch per layer while the caches are short).
// The paper's merge / split of the caches around every sentence does not exist here: the two caches are
// attended in place.  Projections, MLP and sampling need weights and are outside this path, so the
// activations are given (one set, reused by every layer) and the number of tokens of every reasoning unit
// is an input, as it is in Alg. 1 (source and target length lists).
//
// A decoded token is one or two small launches per layer, a chain of dependent kernels for the host to feed.  With
// job.decode_graph set, one token (all layers) is recorded ONCE into a HIP graph and replayed for every token:
// the token's activations reach fixed staging buffers through a kernel that reads the step number from a device
// word (bumped at the end of the graph), so a replay needs no host-side update at all; the grid is sized for the
// longest reasoning cache of the session (units past the current length exit at once).
//
// st_stream_timeline is the same control logic as a pure host model: event times for given stage durations.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "st_cache.h"

namespace st {
namespace {

using Clock = std::chrono::steady_clock;

struct Shared {
    std::mutex mu;
    std::condition_variable cv;
    int enqueued = 0;                 // sentences whose prefill has been enqueued (their event is recorded)
    std::atomic<bool> abort{false};
    st_status status = ST_OK;
    std::string message;

    void fail_with(st_status s, const char* msg) {
        std::lock_guard<std::mutex> lock(mu);
        if (status == ST_OK) {
            status = s;
            message = msg;
        }
        abort.store(true);
        cv.notify_all();
    }
};

struct Events {
    hipEvent_t start = nullptr;
    std::vector<hipEvent_t> prefilled, first_token, unit_done;
    ~Events() {
        if (start) (void)hipEventDestroy(start);
        for (auto* v : {&prefilled, &first_token, &unit_done})
            for (hipEvent_t e : *v)
                if (e) (void)hipEventDestroy(e);
    }
};

struct Layout {
    std::vector<int64_t> src_row0;    // first token row of sentence k in the sentence-major source tensors
    std::vector<int64_t> step0;       // first decoding step of unit t
    int64_t total_src = 0, total_steps = 0;
    int max_src = 0;
};

#define SCHED_CALL(sh, call)                                   \
    do {                                                       \
        st_status s_ = (call);                                 \
        if (s_ != ST_OK) {                                     \
            (sh).fail_with(s_, st_last_error());               \
            return;                                            \
        }                                                      \
    } while (0)
#define SCHED_HIP(sh, call)                                                        \
    do {                                                                           \
        hipError_t e_ = (call);                                                    \
        if (e_ != hipSuccess) {                                                    \
            (sh).fail_with(ST_ERR_RUNTIME, hipGetErrorString(e_));                 \
            return;                                                                \
        }                                                                          \
    } while (0)

// ---- staging kernels of the graph-replayed decode step ----
// copy the activations of step *step from the step-major tensors into the staging buffers (16-byte pieces)
__global__ void stage_in_kernel(u32x4* __restrict__ qs, u32x4* __restrict__ ks, u32x4* __restrict__ vs, const u32x4* __restrict__ q,
                                const u32x4* __restrict__ k, const u32x4* __restrict__ v, const int32_t* __restrict__ step,
                                int32_t* __restrict__ rsn_len, int batch, int q_pieces, int kv_pieces) {
    const int64_t g = *step;
    // token g is the (g + 1)-th of every sequence's reasoning stream
    if (blockIdx.x == 0)
        for (int b = threadIdx.x; b < batch; b += blockDim.x) rsn_len[b] = int32_t(g + 1);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < q_pieces + 2 * kv_pieces; i += gridDim.x * blockDim.x) {
        if (i < q_pieces) qs[i] = q[g * q_pieces + i];
        else if (i < q_pieces + kv_pieces) ks[i - q_pieces] = k[g * kv_pieces + (i - q_pieces)];
        else vs[i - q_pieces - kv_pieces] = v[g * kv_pieces + (i - q_pieces - kv_pieces)];
    }
}
__global__ void stage_out_kernel(u32x4* __restrict__ out, const u32x4* __restrict__ os, const int32_t* __restrict__ step, int q_pieces) {
    const int64_t g = *step;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < q_pieces; i += gridDim.x * blockDim.x) out[g * q_pieces + i] = os[i];
}
__global__ void step_bump_kernel(int32_t* step) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *step += 1;
}
__global__ void copy_i32_kernel(int32_t* __restrict__ dst, const int32_t* __restrict__ src, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = src[i];
}

struct Staging {                      // device memory of the graph-replayed decode step
    int32_t* step = nullptr;          // [1] number of the token the next replay decodes
    int32_t* vis = nullptr;           // [batch] visible source length of the current unit
    int32_t* len = nullptr;           // [batch] reasoning length including the token being decoded
    uint16_t *q = nullptr, *k = nullptr, *v = nullptr, *out = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    ~Staging() {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
    }
};

struct Runner {
    const st_stream_job& job;
    const Layout& lay;
    Events& ev;
    Shared& sh;
    const int32_t* vis_dev;           // [n_sentences][batch] visible source length of unit t
    const int32_t* len_dev;           // [total_steps][batch] reasoning length including token g: g + 1
    int device;
    Clock::time_point t0;
    int hkv, d;
    hipStream_t ps, ds;
    Staging* stg = nullptr;           // null: eager launches for every token

    const char* at(const void* base, int64_t rows, int heads) const {
        return static_cast<const char*>(base) + rows * job.batch * heads * d * 2;
    }
    char* at(void* base, int64_t rows, int heads) const {
        return static_cast<char*>(base) + rows * job.batch * heads * d * 2;
    }

    void sleep_until_arrival(int k) const {
        if (!job.arrival_s) return;
        const auto when = t0 + std::chrono::duration_cast<Clock::duration>(std::chrono::duration<double>(job.arrival_s[k]));
        while (!sh.abort.load() && Clock::now() < when) {
            const auto left = when - Clock::now();
            std::this_thread::sleep_for(std::min<Clock::duration>(left, std::chrono::milliseconds(2)));
        }
    }

    // prefill of sentence k on stream s, every layer
    void prefill_sentence(int k, hipStream_t s) {
        const int n = job.src_tokens[k];
        if (n > 0) {
            const int64_t r0 = lay.src_row0[k];
            const int bound = int(r0 + n);                      // source tokens per sequence after this sentence
            for (int l = 0; l < job.n_layers; ++l) {
                SCHED_CALL(sh, st_kv_append_rope(&job.caches[l], ST_SOURCE, at(job.src_k, r0, hkv), at(job.src_v, r0, hkv), nullptr, n,
                                                 job.batch, bound, job.theta_base, s));
                SCHED_CALL(sh, st_attn_source_chunk_rope(at(job.src_out, r0, job.n_q_heads), nullptr, at(job.src_q, r0, job.n_q_heads), &job.caches[l],
                                                         job.caches[l].source.appended_len, nullptr, n, bound, job.batch,
                                                         job.n_q_heads, job.scale, job.theta_base, job.prefill_workspace,
                                                         job.prefill_workspace_bytes, s));
            }
        }
        SCHED_HIP(sh, hipEventRecord(ev.prefilled[k], s));
    }

    // one token, every layer, from and to the staging buffers: recorded into a graph on stream s
    st_status enqueue_staged_token(hipStream_t s) {
        const int q_pieces = job.batch * job.n_q_heads * d / 8, kv_pieces = job.batch * hkv * d / 8;
        const int blocks = std::min(64, (q_pieces + 2 * kv_pieces + 255) / 256);
        hipLaunchKernelGGL(stage_in_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<u32x4*>(stg->q), reinterpret_cast<u32x4*>(stg->k),
                           reinterpret_cast<u32x4*>(stg->v), static_cast<const u32x4*>(job.rsn_q), static_cast<const u32x4*>(job.rsn_k),
                           static_cast<const u32x4*>(job.rsn_v), stg->step, stg->len, job.batch, q_pieces, kv_pieces);
        st_dual_lens lens = {};
        lens.src_visible_len = stg->vis;
        lens.rsn_len = stg->len;
        lens.q_len = 1;
        lens.max_src_len = int(lay.total_src);
        lens.max_rsn_len = int(lay.total_steps);
        for (int l = 0; l < job.n_layers; ++l) {
            const st_status r = st_attn_decode_dual_append(stg->out, nullptr, stg->q, stg->k, stg->v, &job.caches[l], &lens, job.batch,
                                                           job.n_q_heads, job.scale, job.theta_base, job.decode_workspace,
                                                           job.decode_workspace_bytes, s);
            if (r != ST_OK) return r;
        }
        hipLaunchKernelGGL(stage_out_kernel, dim3(std::min(64, (q_pieces + 255) / 256)), dim3(256), 0, s, static_cast<u32x4*>(job.rsn_out),
                           reinterpret_cast<const u32x4*>(stg->out), stg->step, q_pieces);
        hipLaunchKernelGGL(step_bump_kernel, dim3(1), dim3(64), 0, s, stg->step);
        if (hipGetLastError() != hipSuccess) return fail(ST_ERR_RUNTIME, "st_stream_run: launch of a staging kernel failed");
        return ST_OK;
    }

    // Record one token into a graph (nothing runs).  On any failure the session falls back to eager launches.
    void record_token_graph(hipStream_t s) {
        if (!stg || lay.total_steps == 0) return;
        bool ok = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) == hipSuccess;
        if (ok) {
            const st_status r = enqueue_staged_token(s);
            hipGraph_t g = nullptr;
            const hipError_t e = hipStreamEndCapture(s, &g);
            stg->graph = g;
            ok = r == ST_OK && e == hipSuccess && g != nullptr;
        }
        if (ok) ok = hipGraphInstantiate(&stg->exec, stg->graph, nullptr, nullptr, 0) == hipSuccess;
        if (!ok) {
            (void)hipGetLastError();
            stg = nullptr;
        }
    }

    // decoding of unit t on stream s, every layer; vis_unit: which unit's slice of the source cache is visible
    void decode_unit(int t, int vis_unit, hipStream_t s) {
        const int n = job.rsn_tokens[t];
        if (stg) {
            // the unit's slice of the source cache, then one replay per token (they find their step number on the device)
            hipLaunchKernelGGL(copy_i32_kernel, dim3(1), dim3(256), 0, s, stg->vis, vis_dev + int64_t(vis_unit) * job.batch, job.batch);
            for (int j = 0; j < n; ++j) {
                SCHED_HIP(sh, hipGraphLaunch(stg->exec, s));
                if (j == 0) SCHED_HIP(sh, hipEventRecord(ev.first_token[t], s));
            }
            if (n == 0) SCHED_HIP(sh, hipEventRecord(ev.first_token[t], s));
            SCHED_HIP(sh, hipEventRecord(ev.unit_done[t], s));
            return;
        }
        for (int j = 0; j < n; ++j) {
            const int64_t g = lay.step0[t] + j;
            st_dual_lens lens = {};
            lens.src_visible_len = vis_dev + int64_t(vis_unit) * job.batch;
            lens.rsn_len = len_dev + g * job.batch;
            lens.q_len = 1;
            lens.max_src_len = int(lay.total_src);
            lens.max_rsn_len = int(g + 1);
            for (int l = 0; l < job.n_layers; ++l)
                SCHED_CALL(sh, st_attn_decode_dual_append(at(job.rsn_out, g, job.n_q_heads), nullptr, at(job.rsn_q, g, job.n_q_heads),
                                                          at(job.rsn_k, g, hkv), at(job.rsn_v, g, hkv), &job.caches[l], &lens, job.batch,
                                                          job.n_q_heads, job.scale, job.theta_base, job.decode_workspace,
                                                          job.decode_workspace_bytes, s));
            if (j == 0) SCHED_HIP(sh, hipEventRecord(ev.first_token[t], s));
        }
        if (n == 0) SCHED_HIP(sh, hipEventRecord(ev.first_token[t], s));
        SCHED_HIP(sh, hipEventRecord(ev.unit_done[t], s));
    }

    void prefill_loop() {
        if (hipSetDevice(device) != hipSuccess) return sh.fail_with(ST_ERR_RUNTIME, "hipSetDevice failed in the prefill loop");
        for (int k = 0; k < job.n_sentences && !sh.abort.load(); ++k) {
            sleep_until_arrival(k);
            prefill_sentence(k, ps);
            if (sh.abort.load()) return;
            {
                std::lock_guard<std::mutex> lock(sh.mu);
                sh.enqueued = k + 1;
            }
            sh.cv.notify_all();
        }
    }

    bool prefilled_now(int k) {
        {
            std::lock_guard<std::mutex> lock(sh.mu);
            if (sh.enqueued <= k) return false;
        }
        return hipEventQuery(ev.prefilled[k]) == hipSuccess;
    }

    void decode_loop(int32_t* waited, int32_t* sliced) {
        if (hipSetDevice(device) != hipSuccess) return sh.fail_with(ST_ERR_RUNTIME, "hipSetDevice failed in the decoding loop");
        record_token_graph(ds);
        for (int t = 0; t < job.n_sentences && !sh.abort.load(); ++t) {
            if (t > 0) SCHED_HIP(sh, hipEventSynchronize(ev.unit_done[t - 1]));     // the unit ended (its last token is out)
            const bool here = prefilled_now(t);
            waited[t] = here ? 0 : 1;                                                // N_EOS < N_EOT + 1: wait for the prefill
            sliced[t] = (t + 1 < job.n_sentences && prefilled_now(t + 1)) ? 1 : 0;   // N_EOS > N_EOT + 1: select a slice
            {
                std::unique_lock<std::mutex> lock(sh.mu);
                sh.cv.wait(lock, [&] { return sh.enqueued > t || sh.abort.load(); });
            }
            if (sh.abort.load()) return;
            SCHED_HIP(sh, hipStreamWaitEvent(ds, ev.prefilled[t], 0));
            decode_unit(t, t, ds);
        }
    }

    // one worker: prefill sentence k, decode unit k, next sentence
    void serial_loop(int32_t* waited, int32_t* sliced) {
        record_token_graph(ds);
        for (int k = 0; k < job.n_sentences && !sh.abort.load(); ++k) {
            sleep_until_arrival(k);
            waited[k] = (k == 0 || hipEventQuery(ev.unit_done[k - 1]) == hipSuccess) ? 1 : 0;   // the worker was idle when it arrived
            sliced[k] = 0;
            if (k > 0) SCHED_HIP(sh, hipStreamWaitEvent(ps, ev.unit_done[k - 1], 0));
            prefill_sentence(k, ps);
            if (sh.abort.load()) return;
            SCHED_HIP(sh, hipStreamWaitEvent(ds, ev.prefilled[k], 0));
            decode_unit(k, k, ds);
        }
    }

    // read everything, prefill everything, then decode with the whole input visible
    void batch_loop(int32_t* waited, int32_t* sliced) {
        record_token_graph(ds);
        if (job.n_sentences > 0) sleep_until_arrival(job.n_sentences - 1);
        for (int k = 0; k < job.n_sentences && !sh.abort.load(); ++k) prefill_sentence(k, ps);
        if (sh.abort.load() || job.n_sentences == 0) return;
        SCHED_HIP(sh, hipStreamWaitEvent(ds, ev.prefilled[job.n_sentences - 1], 0));
        for (int t = 0; t < job.n_sentences && !sh.abort.load(); ++t) {
            waited[t] = t == 0 ? 1 : 0;
            sliced[t] = 0;
            decode_unit(t, job.n_sentences - 1, ds);
        }
    }
};

}  // namespace
}  // namespace st

using namespace st;

extern "C" st_status st_stream_timeline(int32_t mode, int32_t n_sentences, const double* arrival_s, const double* prefill_s,
                                        const int32_t* n_decode, double decode_s, double* prefill_done_s, double* unit_start_s,
                                        double* first_token_s, double* unit_done_s, int32_t* waited, int32_t* sliced) {
    if (n_sentences < 0 || (n_sentences > 0 && (!arrival_s || !prefill_s || !n_decode)))
        return fail(ST_ERR_INVALID_ARG, "st_stream_timeline: null input");
    if (mode != ST_SCHED_STREAMING && mode != ST_SCHED_SERIAL && mode != ST_SCHED_BATCH)
        return fail(ST_ERR_INVALID_ARG, "st_stream_timeline: mode = %d", int(mode));
    if (!(decode_s >= 0.0)) return fail(ST_ERR_INVALID_ARG, "st_stream_timeline: negative decode time");
    for (int k = 0; k < n_sentences; ++k) {
        if (!(prefill_s[k] >= 0.0) || n_decode[k] < 0 || !(arrival_s[k] >= 0.0) || (k > 0 && arrival_s[k] < arrival_s[k - 1]))
            return fail(ST_ERR_INVALID_ARG, "st_stream_timeline: sentence %d: times must be non-negative, arrivals non-decreasing", k);
    }
    const int K = n_sentences;
    std::vector<double> pf(K), start(K), first(K), done(K);
    std::vector<int32_t> w(K), sl(K);
    if (mode == ST_SCHED_STREAMING) {
        double t_free = 0.0;
        for (int k = 0; k < K; ++k) pf[k] = t_free = std::max(arrival_s[k], t_free) + prefill_s[k];
        double ready = 0.0;
        for (int t = 0; t < K; ++t) {
            w[t] = pf[t] > ready;
            start[t] = std::max(ready, pf[t]);
            sl[t] = t + 1 < K && pf[t + 1] <= start[t];
            first[t] = n_decode[t] > 0 ? start[t] + decode_s : start[t];
            done[t] = ready = start[t] + n_decode[t] * decode_s;
        }
    } else if (mode == ST_SCHED_SERIAL) {
        double t_free = 0.0;
        for (int k = 0; k < K; ++k) {
            w[k] = arrival_s[k] > t_free;
            sl[k] = 0;
            pf[k] = start[k] = std::max(arrival_s[k], t_free) + prefill_s[k];
            first[k] = n_decode[k] > 0 ? start[k] + decode_s : start[k];
            done[k] = t_free = start[k] + n_decode[k] * decode_s;
        }
    } else {
        double t_free = K ? arrival_s[K - 1] : 0.0;
        for (int k = 0; k < K; ++k) pf[k] = t_free += prefill_s[k];
        for (int t = 0; t < K; ++t) {
            w[t] = t == 0;
            sl[t] = 0;
            start[t] = t_free;
            first[t] = n_decode[t] > 0 ? t_free + decode_s : t_free;
            done[t] = t_free += n_decode[t] * decode_s;
        }
    }
    for (int k = 0; k < K; ++k) {
        if (prefill_done_s) prefill_done_s[k] = pf[k];
        if (unit_start_s) unit_start_s[k] = start[k];
        if (first_token_s) first_token_s[k] = first[k];
        if (unit_done_s) unit_done_s[k] = done[k];
        if (waited) waited[k] = w[k];
        if (sliced) sliced[k] = sl[k];
    }
    return ST_OK;
}

extern "C" st_status st_stream_run(const st_stream_job* job_in, int32_t mode, st_stream_report* report) {
    if (!job_in || !report) return fail(ST_ERR_INVALID_ARG, "st_stream_run: null pointer");
    st_stream_job job = *job_in;
    if (mode != ST_SCHED_STREAMING && mode != ST_SCHED_SERIAL && mode != ST_SCHED_BATCH)
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: mode = %d", int(mode));
    if (job.n_layers <= 0 || job.batch <= 0 || job.n_q_heads <= 0 || job.n_sentences < 0)
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: bad sizes");
    if (!job.caches || (job.n_sentences > 0 && (!job.src_tokens || !job.rsn_tokens)))
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: null caches or length lists");
    if (!(job.theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "st_stream_run: theta_base must be positive");
    if (!report->prefill_done_s || !report->first_token_s || !report->unit_done_s || !report->waited || !report->sliced)
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: the report's arrays must be provided");
    Layout lay;
    lay.src_row0.resize(job.n_sentences);
    lay.step0.resize(job.n_sentences);
    for (int k = 0; k < job.n_sentences; ++k) {
        if (job.src_tokens[k] < 0 || job.rsn_tokens[k] < 0) return fail(ST_ERR_INVALID_ARG, "st_stream_run: negative length in sentence %d", k);
        if (job.arrival_s && (!(job.arrival_s[k] >= 0.0) || (k > 0 && job.arrival_s[k] < job.arrival_s[k - 1])))
            return fail(ST_ERR_INVALID_ARG, "st_stream_run: arrival times must be non-negative and non-decreasing");
        lay.src_row0[k] = lay.total_src;
        lay.step0[k] = lay.total_steps;
        lay.total_src += job.src_tokens[k];
        lay.total_steps += job.rsn_tokens[k];
        lay.max_src = std::max(lay.max_src, job.src_tokens[k]);
    }
    if (lay.total_src > 0 && (!job.src_q || !job.src_k || !job.src_v || !job.src_out))
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: null source activations or output");
    if (lay.total_steps > 0 && (!job.rsn_q || !job.rsn_k || !job.rsn_v || !job.rsn_out))
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: null reasoning activations or output");
    const st_kv_cache& c0 = job.caches[0].source;
    for (int l = 0; l < job.n_layers; ++l) {
        st_status r = check_cache(job.caches[l].source, "st_stream_run", "source");
        if (r == ST_OK) r = check_cache(job.caches[l].reasoning, "st_stream_run", "reasoning");
        if (r != ST_OK) return r;
        const st_kv_cache &s = job.caches[l].source, &g = job.caches[l].reasoning;
        if (s.n_kv_heads != c0.n_kv_heads || g.n_kv_heads != c0.n_kv_heads || s.head_dim != c0.head_dim || g.head_dim != c0.head_dim)
            return fail(ST_ERR_SHAPE, "st_stream_run: layer %d: all caches must share n_kv_heads and head_dim", l);
        if (!s.appended_len || !g.appended_len) return fail(ST_ERR_INVALID_ARG, "st_stream_run: layer %d: appended_len is null", l);
        if (lay.total_src > int64_t(s.max_pages_per_seq) * kPage || lay.total_steps > int64_t(g.max_pages_per_seq) * kPage)
            return fail(ST_ERR_CAPACITY, "st_stream_run: layer %d: the page tables hold fewer tokens than the job appends", l);
    }
    if (job.n_q_heads % c0.n_kv_heads != 0) return fail(ST_ERR_SHAPE, "st_stream_run: n_q_heads must be a multiple of n_kv_heads");
    int device = 0;
    ST_HIP(hipGetDevice(&device));
    hipStream_t ps = static_cast<hipStream_t>(job.prefill_stream), ds = static_cast<hipStream_t>(job.decode_stream);
    if (mode == ST_SCHED_STREAMING && ps == ds)
        return fail(ST_ERR_INVALID_ARG, "st_stream_run: the streaming schedule needs two different streams");

    // every cache must start empty: the position ids and the visible slices below count from 0
    ST_HIP(hipStreamSynchronize(ps));
    ST_HIP(hipStreamSynchronize(ds));
    std::vector<int32_t> host_len(job.batch);
    for (int l = 0; l < job.n_layers; ++l)
        for (const st_kv_cache* c : {&job.caches[l].source, &job.caches[l].reasoning}) {
            ST_HIP(hipMemcpy(host_len.data(), c->appended_len, sizeof(int32_t) * job.batch, hipMemcpyDeviceToHost));
            for (int b = 0; b < job.batch; ++b)
                if (host_len[b] != 0) return fail(ST_ERR_INVALID_ARG, "st_stream_run: layer %d: caches must be empty at the start", l);
        }

    // visible source length of unit t: the input up to and including sentence t
    std::vector<int32_t> vis_host(size_t(std::max(job.n_sentences, 1)) * job.batch);
    for (int t = 0; t < job.n_sentences; ++t)
        for (int b = 0; b < job.batch; ++b) vis_host[size_t(t) * job.batch + b] = int32_t(lay.src_row0[t] + job.src_tokens[t]);
    // reasoning length of every sequence while token g is decoded (the token included)
    std::vector<int32_t> len_host(size_t(std::max<int64_t>(lay.total_steps, 1)) * job.batch);
    for (int64_t g = 0; g < lay.total_steps; ++g)
        for (int b = 0; b < job.batch; ++b) len_host[size_t(g) * job.batch + b] = int32_t(g + 1);
    // one device block: the visibility table, the length table, then (graph-replayed decode) the step word, the current
    // unit's slice, the current lengths and the staging buffers of one token
    const size_t vis_bytes = (vis_host.size() * sizeof(int32_t) + 255) & ~size_t(255);
    const size_t len_bytes = (len_host.size() * sizeof(int32_t) + 255) & ~size_t(255);
    const size_t q_bytes = (size_t(job.batch) * job.n_q_heads * c0.head_dim * 2 + 255) & ~size_t(255);
    const size_t kv_bytes = (size_t(job.batch) * c0.n_kv_heads * c0.head_dim * 2 + 255) & ~size_t(255);
    const size_t vis1_bytes = (size_t(job.batch) * sizeof(int32_t) + 255) & ~size_t(255);
    const bool use_graph = job.decode_graph != 0 && lay.total_steps > 0;
    unsigned char* block = nullptr;
    ST_HIP(hipMalloc(&block, vis_bytes + len_bytes + (use_graph ? 256 + 2 * vis1_bytes + 2 * q_bytes + 2 * kv_bytes : 0)));
    struct Free { void* p; ~Free() { (void)hipFree(p); } } free_block{block};
    int32_t* vis_dev = reinterpret_cast<int32_t*>(block);
    ST_HIP(hipMemcpy(vis_dev, vis_host.data(), vis_host.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    int32_t* len_dev = reinterpret_cast<int32_t*>(block + vis_bytes);
    ST_HIP(hipMemcpy(len_dev, len_host.data(), len_host.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    Staging staging;
    if (use_graph) {
        unsigned char* p = block + vis_bytes + len_bytes;
        staging.step = reinterpret_cast<int32_t*>(p); p += 256;
        staging.vis = reinterpret_cast<int32_t*>(p); p += vis1_bytes;
        staging.len = reinterpret_cast<int32_t*>(p); p += vis1_bytes;
        staging.q = reinterpret_cast<uint16_t*>(p); p += q_bytes;
        staging.out = reinterpret_cast<uint16_t*>(p); p += q_bytes;
        staging.k = reinterpret_cast<uint16_t*>(p); p += kv_bytes;
        staging.v = reinterpret_cast<uint16_t*>(p);
        ST_HIP(hipMemset(staging.step, 0, 256));
    }

    Events ev;
    ST_HIP(hipEventCreate(&ev.start));
    for (auto* v : {&ev.prefilled, &ev.first_token, &ev.unit_done}) {
        v->assign(job.n_sentences, nullptr);
        for (auto& e : *v) ST_HIP(hipEventCreate(&e));
    }
    Shared sh;
    Runner run{job, lay, ev, sh, vis_dev, len_dev, device, Clock::now(), c0.n_kv_heads, c0.head_dim, ps, ds, use_graph ? &staging : nullptr};
    for (int k = 0; k < job.n_sentences; ++k) report->waited[k] = report->sliced[k] = 0;

    ST_HIP(hipEventRecord(ev.start, ps));
    ST_HIP(hipStreamWaitEvent(ds, ev.start, 0));
    run.t0 = Clock::now();
    if (mode == ST_SCHED_STREAMING) {
        std::thread a([&] { run.prefill_loop(); });
        std::thread b([&] { run.decode_loop(report->waited, report->sliced); });
        a.join();
        b.join();
    } else if (mode == ST_SCHED_SERIAL) {
        run.serial_loop(report->waited, report->sliced);
    } else {
        run.batch_loop(report->waited, report->sliced);
    }
    const hipError_t e1 = hipStreamSynchronize(ps), e2 = hipStreamSynchronize(ds);
    const double wall = std::chrono::duration<double>(Clock::now() - run.t0).count();
    if (sh.status != ST_OK) return fail(sh.status, "st_stream_run: %s", sh.message.c_str());
    if (e1 != hipSuccess || e2 != hipSuccess) return fail(ST_ERR_RUNTIME, "st_stream_run: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2));
    auto since_start = [&](hipEvent_t e, double* out) -> hipError_t {
        float ms = 0.f;
        const hipError_t r = hipEventElapsedTime(&ms, ev.start, e);
        *out = double(ms) * 1e-3;
        return r;
    };
    for (int k = 0; k < job.n_sentences; ++k) {
        ST_HIP(since_start(ev.prefilled[k], &report->prefill_done_s[k]));
        ST_HIP(since_start(ev.first_token[k], &report->first_token_s[k]));
        ST_HIP(since_start(ev.unit_done[k], &report->unit_done_s[k]));
    }
    report->total_s = wall;
    return ST_OK;
}
