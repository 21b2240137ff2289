// Shared device helpers of libzo2: storage formats, error plumbing.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/zo2.h"

namespace zo2 {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;
struct fp8_e4m3_t { uint8_t v; };
struct fp8_e5m2_t { uint8_t v; };

// ---------------------------------------------------------------- error plumbing (op level)
void set_op_error(const char* fmt, ...);
#define ZO2_OP_CHECK(cond, status, ...)        \
    do {                                       \
        if (!(cond)) {                         \
            zo2::set_op_error(__VA_ARGS__);    \
            return status;                     \
        }                                      \
    } while (0)
#define ZO2_HIP_LAUNCH_CHECK()                                               \
    do {                                                                     \
        hipError_t e__ = hipGetLastError();                                  \
        if (e__ != hipSuccess) {                                             \
            zo2::set_op_error("HIP launch failed: %s", hipGetErrorString(e__)); \
            return ZO2_EHIP;                                                 \
        }                                                                    \
    } while (0)

// ---------------------------------------------------------------- scalar conversions
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// Round-to-nearest-even fp32 -> 8-bit float with EB exponent / MB mantissa bits, saturating
// at the largest finite code MAXC.  NaN -> NANC.
template <int EB, int MB, int BIAS, uint32_t MAXC, uint32_t NANC>
__device__ __forceinline__ uint32_t encode_fp8(float x) {
    const uint32_t u = f2u(x);
    const uint32_t sign = (u >> 31) << 7;
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return sign | NANC;
    // largest finite value of the format as fp32 bits
    const uint32_t max_bits = ((MAXC >> MB) + (127 - BIAS)) << 23 | ((MAXC & ((1u << MB) - 1)) << (23 - MB));
    if (a >= max_bits) return sign | MAXC;
    const uint32_t min_normal_bits = (uint32_t)(1 + 127 - BIAS) << 23;
    uint32_t code;
    if (a < min_normal_bits) {
        // subnormal target: multiples of 2^(1-BIAS-MB); rintf rounds to nearest even
        const float q = u2f(a) * u2f((uint32_t)(127 + BIAS - 1 + MB) << 23);
        code = (uint32_t)__builtin_rintf(q);
    } else {
        a += ((a >> (23 - MB)) & 1u) + ((1u << (22 - MB)) - 1u);
        code = (a >> (23 - MB)) - ((uint32_t)(127 - BIAS) << MB);
        code = code > MAXC ? MAXC : code;
    }
    return sign | code;
}

template <int EB, int MB, int BIAS, bool IEEE>
__device__ __forceinline__ float decode_fp8(uint32_t c) {
    const uint32_t sign = (c & 0x80u) << 24;
    const uint32_t em = c & 0x7fu;
    const uint32_t E = em >> MB, M = em & ((1u << MB) - 1);
    float v;
    if (E == 0) {
        v = (float)M * u2f((uint32_t)(127 + 1 - BIAS - MB) << 23);
    } else if (IEEE && E == (1u << EB) - 1) {
        v = M ? u2f(0x7fc00000u) : u2f(0x7f800000u);
    } else if (!IEEE && em == 0x7fu) {
        v = u2f(0x7fc00000u);
    } else {
        v = u2f(((E + 127 - BIAS) << 23) | (M << (23 - MB)));
    }
    return u2f(f2u(v) | sign);
}

// ---------------------------------------------------------------- typed load / store of one element
template <typename T> struct Fmt;
template <> struct Fmt<float> {
    static constexpr int kBytes = 4;
    static __device__ __forceinline__ float load(float v) { return v; }
    static __device__ __forceinline__ float store(float v) { return v; }
};
template <> struct Fmt<bf16_t> {
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ float load(bf16_t v) { return (float)v; }
    static __device__ __forceinline__ bf16_t store(float v) { return (bf16_t)v; }
};
template <> struct Fmt<f16_t> {
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ float load(f16_t v) { return (float)v; }
    static __device__ __forceinline__ f16_t store(float v) { return (f16_t)v; }
};
template <> struct Fmt<fp8_e4m3_t> {
    static constexpr int kBytes = 1;
    // gfx950 converts the OCP 8-bit formats in hardware (round to nearest even, subnormals included): one instruction per
    // direction instead of about twenty.  What the instruction does beyond the largest finite magnitude is not relied on:
    // the value is clamped to it first (the format saturates here), and NaN keeps this library's code for it.
    static __device__ __forceinline__ float load(fp8_e4m3_t v) { return __builtin_amdgcn_cvt_f32_fp8((int)v.v, 0); }
    static __device__ __forceinline__ fp8_e4m3_t store(float v) {
        const int c = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(v, -448.0f, 448.0f), 0.0f, 0, false) & 0xff;
        return fp8_e4m3_t{(uint8_t)(v != v ? (((f2u(v) >> 31) << 7) | 0x7fu) : (uint32_t)c)};
    }
};
template <> struct Fmt<fp8_e5m2_t> {
    static constexpr int kBytes = 1;
    static __device__ __forceinline__ float load(fp8_e5m2_t v) { return __builtin_amdgcn_cvt_f32_bf8((int)v.v, 0); }
    static __device__ __forceinline__ fp8_e5m2_t store(float v) {
        const int c = __builtin_amdgcn_cvt_pk_bf8_f32(__builtin_amdgcn_fmed3f(v, -57344.0f, 57344.0f), 0.0f, 0, false) & 0xff;
        return fp8_e5m2_t{(uint8_t)(v != v ? (((f2u(v) >> 31) << 7) | 0x7eu) : (uint32_t)c)};
    }
};

// ---------------------------------------------------------------- stochastic rounding to a storage format
// Bit pattern of a stored element as an integer and back; kSign is the sign bit, kMaxMag the largest finite
// magnitude pattern.  In all these formats the magnitude patterns are ordered like the magnitudes.
template <typename T> struct FmtBits;
template <> struct FmtBits<bf16_t> {
    static constexpr uint32_t kSign = 0x8000u, kMaxMag = 0x7f7fu;
    static __device__ __forceinline__ uint32_t get(bf16_t v) { return __builtin_bit_cast(uint16_t, v); }
    static __device__ __forceinline__ bf16_t make(uint32_t b) { return __builtin_bit_cast(bf16_t, (uint16_t)b); }
};
template <> struct FmtBits<f16_t> {
    static constexpr uint32_t kSign = 0x8000u, kMaxMag = 0x7bffu;
    static __device__ __forceinline__ uint32_t get(f16_t v) { return __builtin_bit_cast(uint16_t, v); }
    static __device__ __forceinline__ f16_t make(uint32_t b) { return __builtin_bit_cast(f16_t, (uint16_t)b); }
};
template <> struct FmtBits<fp8_e4m3_t> {
    static constexpr uint32_t kSign = 0x80u, kMaxMag = 0x7eu;
    static __device__ __forceinline__ uint32_t get(fp8_e4m3_t v) { return v.v; }
    static __device__ __forceinline__ fp8_e4m3_t make(uint32_t b) { return fp8_e4m3_t{(uint8_t)b}; }
};
template <> struct FmtBits<fp8_e5m2_t> {
    static constexpr uint32_t kSign = 0x80u, kMaxMag = 0x7bu;
    static __device__ __forceinline__ uint32_t get(fp8_e5m2_t v) { return v.v; }
    static __device__ __forceinline__ fp8_e5m2_t make(uint32_t b) { return fp8_e5m2_t{(uint8_t)b}; }
};

// x goes to one of its two neighbours lo <= |x| <= hi in format T (sign kept): to hi iff
// r16 < 65536 (|x| - lo) / (hi - lo), r16 uniform in [0, 65536).  hi - lo is a power of two and |x| - lo is
// exact in float32, so the comparison is exact.  Beyond the largest finite value: that value.  NaN: NaN.
template <typename T>
__device__ __forceinline__ T store_stochastic(float x, uint32_t r16) {
    const T n = Fmt<T>::store(x);                                   // nearest: never more than one step from lo
    const uint32_t nb = FmtBits<T>::get(n);
    const uint32_t sign = nb & FmtBits<T>::kSign, mag = nb & (FmtBits<T>::kSign - 1u);
    const float ax = __builtin_fabsf(x);
    if (!(ax == ax)) return n;
    uint32_t lo = mag;
    if (mag > FmtBits<T>::kMaxMag) lo = FmtBits<T>::kMaxMag;         // rounded to infinity: saturate instead
    else if (__builtin_fabsf(Fmt<T>::load(n)) > ax) lo = mag - 1u;  // nearest rounded away from zero
    if (lo >= FmtBits<T>::kMaxMag) return FmtBits<T>::make(sign | FmtBits<T>::kMaxMag);
    const float vlo = Fmt<T>::load(FmtBits<T>::make(lo)), vhi = Fmt<T>::load(FmtBits<T>::make(lo + 1u));
    const float frac = (ax - vlo) / (vhi - vlo);
    return FmtBits<T>::make(sign | (lo + ((float)r16 < frac * 65536.0f ? 1u : 0u)));
}
template <>
__device__ __forceinline__ float store_stochastic<float>(float x, uint32_t) { return x; }
// bfloat16 keeps the upper half of the float32 pattern, so the dropped half is 65536 times the fraction itself:
// "r16 < fraction" is a carry out of (dropped half + 65535 - r16).
template <>
__device__ __forceinline__ bf16_t store_stochastic<bf16_t>(float x, uint32_t r16) {
    const uint32_t u = f2u(x), a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return Fmt<bf16_t>::store(x);
    uint32_t m = (a + (0xffffu - r16)) & 0xffff0000u;
    m = m > 0x7f7f0000u ? 0x7f7f0000u : m;
    return FmtBits<bf16_t>::make(((u >> 31) << 15) | (m >> 16));
}

// A group of N elements moved with one (or two) wide memory operations.
// One-time, per-device set-up (a kernel's LDS reservation, the compute-unit count) keeps its flags in arrays indexed by
// the current device: a process may hold contexts on several GPUs.
static constexpr int kMaxDevices = 64;
inline int current_device() {
    int d = 0;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) d = 0;
    return d;
}
inline int device_cu_count() {          // compute units of the current device (256 if the query fails)
    static int n[kMaxDevices] = {0};
    const int dev = current_device();
    if (n[dev] == 0) {
        int v = 0;
        n[dev] = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
    }
    return n[dev];
}

template <typename T, int N>
struct alignas(sizeof(T) * N) Vec {
    T v[N];
};

template <typename T, int N>
__device__ __forceinline__ Vec<T, N> load_vec(const T* p) {
    return *reinterpret_cast<const Vec<T, N>*>(p);
}
template <typename T, int N>
__device__ __forceinline__ void store_vec(T* p, const Vec<T, N>& v) {
    *reinterpret_cast<Vec<T, N>*>(p) = v;
}

// The same with the streaming ("non-temporal") cache policy: for data this kernel touches once and nobody reads soon.
typedef uint32_t stream_u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t stream_u32x4_t __attribute__((ext_vector_type(4)));
template <typename T, int N>
__device__ __forceinline__ Vec<T, N> load_vec_stream(const T* p) {
    static_assert(sizeof(T) * N == 16 || sizeof(T) * N == 8 || sizeof(T) * N == 32, "vector of 8, 16 or 32 bytes");
    Vec<T, N> v;
    if constexpr (sizeof(T) * N == 8) {
        const stream_u32x2_t r = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x2_t*>(p));
        __builtin_memcpy(&v, &r, 8);
    } else {
        constexpr int Q = sizeof(T) * N / 16;
        stream_u32x4_t r[Q];
#pragma unroll
        for (int i = 0; i < Q; ++i) r[i] = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4_t*>(p) + i);
        __builtin_memcpy(&v, r, sizeof(v));
    }
    return v;
}
template <typename T, int N>
__device__ __forceinline__ void store_vec_stream(T* p, const Vec<T, N>& v) {
    static_assert(sizeof(T) * N == 16 || sizeof(T) * N == 8 || sizeof(T) * N == 32, "vector of 8, 16 or 32 bytes");
    if constexpr (sizeof(T) * N == 8) {
        stream_u32x2_t r;
        __builtin_memcpy(&r, &v, 8);
        __builtin_nontemporal_store(r, reinterpret_cast<stream_u32x2_t*>(p));
    } else {
        constexpr int Q = sizeof(T) * N / 16;
        stream_u32x4_t r[Q];
        __builtin_memcpy(r, &v, sizeof(v));
#pragma unroll
        for (int i = 0; i < Q; ++i) __builtin_nontemporal_store(r[i], reinterpret_cast<stream_u32x4_t*>(p) + i);
    }
}
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// dispatch a zo2_dtype to a type tag
#define ZO2_DISPATCH_WIRE(dt, T, ...)                                             \
    switch (dt) {                                                                 \
        case ZO2_F32: { typedef float T; __VA_ARGS__; break; }                    \
        case ZO2_BF16: { typedef zo2::bf16_t T; __VA_ARGS__; break; }             \
        case ZO2_F16: { typedef zo2::f16_t T; __VA_ARGS__; break; }               \
        case ZO2_FP8_E4M3: { typedef zo2::fp8_e4m3_t T; __VA_ARGS__; break; }     \
        case ZO2_FP8_E5M2: { typedef zo2::fp8_e5m2_t T; __VA_ARGS__; break; }     \
        default: zo2::set_op_error("unknown dtype %d", (int)(dt)); return ZO2_EINVAL; \
    }
#define ZO2_DISPATCH_COMPUTE(dt, T, ...)                                          \
    switch (dt) {                                                                 \
        case ZO2_F32: { typedef float T; __VA_ARGS__; break; }                    \
        case ZO2_BF16: { typedef zo2::bf16_t T; __VA_ARGS__; break; }             \
        case ZO2_F16: { typedef zo2::f16_t T; __VA_ARGS__; break; }               \
        default: zo2::set_op_error("dtype %d is not a compute dtype", (int)(dt)); return ZO2_EINVAL; \
    }

// Eight consecutive elements of an 8-bit format at once: the hardware conversions read a chosen byte of a 32-bit word and
// write two results into a chosen half of one, so a group of eight needs no byte extraction or assembly at all.
template <typename W> struct Fp8Pack;
template <> struct Fp8Pack<fp8_e4m3_t> {
    static constexpr float kMax = 448.0f;
    template <int B> static __device__ __forceinline__ float dec(uint32_t w) { return __builtin_amdgcn_cvt_f32_fp8((int)w, B); }
    template <bool HI> static __device__ __forceinline__ uint32_t enc2(float a, float b, uint32_t old) { return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, HI); }
};
template <> struct Fp8Pack<fp8_e5m2_t> {
    static constexpr float kMax = 57344.0f;
    template <int B> static __device__ __forceinline__ float dec(uint32_t w) { return __builtin_amdgcn_cvt_f32_bf8((int)w, B); }
    template <bool HI> static __device__ __forceinline__ uint32_t enc2(float a, float b, uint32_t old) { return (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, HI); }
};
template <typename W>
__device__ __forceinline__ void fp8_decode8(const Vec<W, 8>& v, float out[8]) {
    uint32_t w[2];
    __builtin_memcpy(w, &v, 8);
    out[0] = Fp8Pack<W>::template dec<0>(w[0]); out[1] = Fp8Pack<W>::template dec<1>(w[0]);
    out[2] = Fp8Pack<W>::template dec<2>(w[0]); out[3] = Fp8Pack<W>::template dec<3>(w[0]);
    out[4] = Fp8Pack<W>::template dec<0>(w[1]); out[5] = Fp8Pack<W>::template dec<1>(w[1]);
    out[6] = Fp8Pack<W>::template dec<2>(w[1]); out[7] = Fp8Pack<W>::template dec<3>(w[1]);
}
// round to nearest even, saturating; a group that contains a NaN (never the case for finite parameters) goes element by
// element through Fmt<W>::store, which keeps this library's NaN code
template <typename W>
__device__ __forceinline__ void fp8_encode8(const float in[8], Vec<W, 8>& v) {
    const float s = ((in[0] + in[1]) + (in[2] + in[3])) + ((in[4] + in[5]) + (in[6] + in[7]));
    if (s != s) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v.v[j] = Fmt<W>::store(in[j]);
        return;
    }
    constexpr float m = Fp8Pack<W>::kMax;
    float c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = __builtin_amdgcn_fmed3f(in[j], -m, m);
    uint32_t w[2];
    w[0] = Fp8Pack<W>::template enc2<false>(c[0], c[1], 0u);
    w[0] = Fp8Pack<W>::template enc2<true>(c[2], c[3], w[0]);
    w[1] = Fp8Pack<W>::template enc2<false>(c[4], c[5], 0u);
    w[1] = Fp8Pack<W>::template enc2<true>(c[6], c[7], w[1]);
    __builtin_memcpy(&v, w, 8);
}

}  // namespace zo2
