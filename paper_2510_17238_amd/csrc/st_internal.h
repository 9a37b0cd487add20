// Internal helpers shared by the translation units of libst (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "st.h"

namespace st {

// thread-local error text behind st_last_error()
void set_error(const char* fmt, ...);
const char* get_error();

inline st_status fail(st_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    set_error("%s", buf);
    return code;
}

#define ST_HIP(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return st::fail(ST_ERR_RUNTIME, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define ST_LAUNCH_CHECK(name)                                                             \
    do {                                                                                  \
        hipError_t e_ = hipGetLastError();                                                \
        if (e_ != hipSuccess)                                                             \
            return st::fail(ST_ERR_RUNTIME, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

// Optional kernel timing (st_profile_enable, per calling thread): HIP events recorded on the launch stream right
// before and after one kernel, read back by st_profile_read.  A pair of events around a single launch adds several
// microseconds of its own (the launch's dispatch after the first event, the second event's completion), so a timed
// kernel is launched prof_repeat() times back to back between its two events (1 unless timing is on; all timed
// kernels write the same results again) and the reading is divided by that.
enum { kProfPrefillAttn = 0, kProfDecodeSplit = 1, kProfBwdDq = 2, kProfBwdDkv = 3, kProfTilePack = 4, kProfSourceChunk = 5, kProfCount = 6 };
bool prof_enabled();
int prof_repeat();
void prof_begin(int which, hipStream_t stream);
void prof_end(int which, hipStream_t stream);
// Wave timeline (st_profile_wave_trace, per calling thread; only while timing is on): a device buffer of
// (start, end) pairs of the 100 MHz wall clock, one per workgroup of the decode split kernel's launch.
struct WaveTrace {
    unsigned long long* buf;
    int capacity;        // pairs
};
WaveTrace prof_wave_trace();

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device-side vector types -------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kPage = 16;           // tokens per cache page
constexpr int kTileM = 128;         // query rows per prefill work item
constexpr int kTileN = 64;          // key columns per prefill tile

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// round-to-nearest-even fp32 -> bf16 bits (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

// ---- RoPE frequencies (Sec. 3.2), shared by the rotation kernel and the fused forms ----
struct RopeFreq {
    double f[64];  // theta^(-2 i / D), i < D/2 <= 64
};
RopeFreq make_rope_freq(double theta_base, int head_dim);

// cos / sin of position * f for the fused kernels: the angle (up to 1e5 rad at long contexts, where an
// fp32 product would be off by 1e-3 rad) is reduced to [-pi, pi] in fp64, the functions themselves are fp32
__device__ __forceinline__ void rope_cos_sin(int pos, double f, float* c, float* s) {
    const double rev = double(pos) * f * 0.15915494309189535;     // angle / 2 pi
    const double r = rev - rint(rev);
    sincosf(float(r * 6.283185307179586), s, c);
}

}  // namespace st
