// RoPE with caller-supplied stream-local positions (Sec. 3.2, "Streaming Position Encoding").
//
// HBM-bound: every element is read once and written once.  One workgroup takes a
// few tokens: first the D/2 (cos, sin) pairs of each token are evaluated once in
// fp64 (the angle position * theta^(-2i/D) reaches 1e4 rad at long contexts, where
// an fp32 product is off by 1e-3 rad) and parked in LDS as fp32; then all heads of
// those tokens are rotated with 16-byte loads and stores.
#include <math.h>

#include "st_internal.h"

namespace st {

RopeFreq make_rope_freq(double theta_base, int head_dim) {
    RopeFreq freq;
    for (int i = 0; i < 64; ++i) freq.f[i] = i < head_dim / 2 ? pow(theta_base, -2.0 * double(i) / double(head_dim)) : 0.0;
    return freq;
}

template <typename T>
struct Vec16;  // 16 bytes of T
template <>
struct Vec16<float> {
    static constexpr int n = 4;
    float v[4];
    __device__ float get(int i) const { return v[i]; }
    __device__ void set(int i, float x) { v[i] = x; }
};
template <>
struct Vec16<uint16_t> {
    static constexpr int n = 8;
    uint16_t v[8];
    __device__ float get(int i) const { return bf16_bits_to_f32(v[i]); }
    __device__ void set(int i, float x) { v[i] = f32_to_bf16_bits(x); }
};

// (x2 / out2 with n_heads2 heads: a second tensor over the same tokens -- the keys beside the queries -- rotated in
// the same launch with the same cos / sin values; n_heads2 = 0 for a single tensor)
template <typename T, int D>
__global__ __launch_bounds__(256) void rope_kernel(T* out, const T* x, T* out2, const T* x2,
                                                   const int32_t* __restrict__ positions,
                                                   int64_t n_tokens, int n_heads, int n_heads2, RopeFreq freq) {
    constexpr int HALF = D / 2;
    constexpr int TOK = 256 / HALF;          // tokens per workgroup
    constexpr int VN = Vec16<T>::n;          // elements per 16-byte vector
    constexpr int CH = HALF / VN;            // vectors per half head
    __shared__ float s_cos[TOK][HALF];
    __shared__ float s_sin[TOK][HALF];

    const int64_t tok0 = int64_t(blockIdx.x) * TOK;
    {
        const int t = threadIdx.x / HALF, i = threadIdx.x % HALF;
        const int64_t tok = tok0 + t;
        double sn = 0.0, cs = 1.0;
        if (tok < n_tokens) sincos(double(positions[tok]) * freq.f[i], &sn, &cs);
        s_cos[t][i] = float(cs);
        s_sin[t][i] = float(sn);
    }
    __syncthreads();

    const int per_tok = (n_heads + n_heads2) * CH;
    const int total = TOK * per_tok;
    for (int w = threadIdx.x; w < total; w += 256) {
        const int t = w / per_tok;
        const int r = w % per_tok;
        const int hh = r / CH, c = r % CH;
        const int64_t tok = tok0 + t;
        if (tok >= n_tokens) continue;
        const bool second = hh >= n_heads;
        const T* src = second ? x2 : x;
        T* dst = second ? out2 : out;
        const int64_t base = (tok * (second ? n_heads2 : n_heads) + (second ? hh - n_heads : hh)) * D + c * VN;
        const Vec16<T> lo = *reinterpret_cast<const Vec16<T>*>(src + base);
        const Vec16<T> hi = *reinterpret_cast<const Vec16<T>*>(src + base + HALF);
        Vec16<T> ylo, yhi;
#pragma unroll
        for (int e = 0; e < VN; ++e) {
            const float cs = s_cos[t][c * VN + e], sn = s_sin[t][c * VN + e];
            const float a = lo.get(e), b = hi.get(e);
            ylo.set(e, a * cs - b * sn);
            yhi.set(e, b * cs + a * sn);
        }
        *reinterpret_cast<Vec16<T>*>(dst + base) = ylo;
        *reinterpret_cast<Vec16<T>*>(dst + base + HALF) = yhi;
    }
}

template <typename T, int D>
static st_status launch_rope(void* out, const void* x, void* out2, const void* x2, const int32_t* positions, int64_t n_tokens,
                             int n_heads, int n_heads2, const RopeFreq& freq, hipStream_t stream) {
    constexpr int TOK = 256 / (D / 2);
    const int64_t blocks = (n_tokens + TOK - 1) / TOK;
    if (blocks > 0x7fffffff) return fail(ST_ERR_SHAPE, "st_rope_apply: too many tokens");
    hipLaunchKernelGGL((rope_kernel<T, D>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<T*>(out), static_cast<const T*>(x), static_cast<T*>(out2), static_cast<const T*>(x2), positions,
                       n_tokens, n_heads, n_heads2, freq);
    ST_LAUNCH_CHECK("rope_kernel");
    return ST_OK;
}

}  // namespace st

static st_status rope_impl(const char* who, void* out, const void* x, int32_t n_heads, void* out2, const void* x2, int32_t n_heads2,
                           const int32_t* positions, int64_t n_tokens, int32_t head_dim, double theta_base, st_dtype dt,
                           void* hip_stream) {
    using namespace st;
    if (!out || !x || !positions || (n_heads2 > 0 && (!out2 || !x2))) return fail(ST_ERR_INVALID_ARG, "%s: null pointer", who);
    if (!aligned16(out) || !aligned16(x) || !aligned16(out2) || !aligned16(x2))
        return fail(ST_ERR_INVALID_ARG, "%s: tensors must be 16-byte aligned", who);
    if (n_tokens < 0 || n_heads <= 0 || n_heads2 < 0) return fail(ST_ERR_INVALID_ARG, "%s: bad sizes", who);
    if (head_dim != 64 && head_dim != 128) return fail(ST_ERR_UNSUPPORTED, "%s: head_dim %d (64 or 128)", who, head_dim);
    if (!(theta_base > 0.0)) return fail(ST_ERR_INVALID_ARG, "%s: theta_base must be positive", who);
    if (dt != ST_F32 && dt != ST_BF16) return fail(ST_ERR_UNSUPPORTED, "%s: dtype %d", who, int(dt));
    if (n_tokens == 0) return ST_OK;
    const RopeFreq freq = make_rope_freq(theta_base, head_dim);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dt == ST_F32) {
        return head_dim == 64 ? launch_rope<float, 64>(out, x, out2, x2, positions, n_tokens, n_heads, n_heads2, freq, stream)
                              : launch_rope<float, 128>(out, x, out2, x2, positions, n_tokens, n_heads, n_heads2, freq, stream);
    }
    return head_dim == 64 ? launch_rope<uint16_t, 64>(out, x, out2, x2, positions, n_tokens, n_heads, n_heads2, freq, stream)
                          : launch_rope<uint16_t, 128>(out, x, out2, x2, positions, n_tokens, n_heads, n_heads2, freq, stream);
}

extern "C" st_status st_rope_apply(void* out, const void* x, const int32_t* positions,
                                   int64_t n_tokens, int32_t n_heads, int32_t head_dim,
                                   double theta_base, st_dtype dt, void* hip_stream) {
    return rope_impl("st_rope_apply", out, x, n_heads, nullptr, nullptr, 0, positions, n_tokens, head_dim, theta_base, dt, hip_stream);
}

extern "C" st_status st_rope_apply_qk(void* q_out, const void* q, int32_t n_q_heads, void* k_out, const void* k, int32_t n_kv_heads,
                                      const int32_t* positions, int64_t n_tokens, int32_t head_dim, double theta_base,
                                      st_dtype dt, void* hip_stream) {
    if (n_kv_heads <= 0) return st::fail(ST_ERR_INVALID_ARG, "st_rope_apply_qk: bad sizes");
    return rope_impl("st_rope_apply_qk", q_out, q, n_q_heads, k_out, k, n_kv_heads, positions, n_tokens, head_dim, theta_base, dt,
                     hip_stream);
}
