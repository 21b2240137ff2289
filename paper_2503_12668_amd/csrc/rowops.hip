// Row-wise and elementwise kernels around the GEMMs: random-stream test hooks, format
// conversion (Sec. 5.5 pack / unpack), LayerNorm, embedding gather with on-the-fly
// update + perturb, cross-entropy, and the scalar epilogue that forms g (Eq. 2).
#include "rowops.h"
#include "philox.h"

namespace zo2 {

// ------------------------------------------------------------------ wave / block reductions
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
// all threads of a 256-thread block receive the sum
template <typename T>
__device__ __forceinline__ T block_sum(T v, T* sh) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[w] = v;
    __syncthreads();
    T r = sh[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r += sh[i];
    return r;
}
__device__ __forceinline__ float block_max(float v, float* sh) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[w] = v;
    __syncthreads();
    float r = sh[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, sh[i]);
    return r;
}

// ------------------------------------------------------------------ random-stream hooks
__global__ void philox_words_kernel(PhiloxKeys k, uint32_t tensor_id, uint64_t e0, uint64_t n, uint32_t* out) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t e = e0 + i, q = e >> 2;
    uint32_t w[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, 0u, k, w);
    const uint32_t r = (uint32_t)(e & 3);
    out[i] = r == 0 ? w[0] : r == 1 ? w[1] : r == 2 ? w[2] : w[3];
}

__global__ void gaussian_kernel(PhiloxKeys k, uint32_t tensor_id, uint64_t e0, uint64_t n, float* out) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint64_t e = e0 + i;
    float z[4];
    gaussian4(k, tensor_id, e & ~(uint64_t)3, z);
    const uint32_t r = (uint32_t)(e & 3);
    out[i] = r == 0 ? z[0] : r == 1 ? z[1] : r == 2 ? z[2] : z[3];
}

zo2_status philox_words(uint64_t seed, uint32_t tid, uint64_t e0, uint64_t n, uint32_t* out, hipStream_t st) {
    if (n == 0) return ZO2_OK;
    ZO2_OP_CHECK(out != nullptr, ZO2_EINVAL, "philox_words: out is NULL");
    ZO2_OP_CHECK(n < (1ull << 39), ZO2_EINVAL, "philox_words: n too large");
    hipLaunchKernelGGL(philox_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, philox_keys(seed), tid, e0, n, out);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}
zo2_status gaussian(uint64_t seed, uint32_t tid, uint64_t e0, uint64_t n, float* out, hipStream_t st) {
    if (n == 0) return ZO2_OK;
    ZO2_OP_CHECK(out != nullptr, ZO2_EINVAL, "gaussian: out is NULL");
    ZO2_OP_CHECK(n < (1ull << 39), ZO2_EINVAL, "gaussian: n too large");
    hipLaunchKernelGGL(gaussian_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, philox_keys(seed), tid, e0, n, out);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ pack / unpack
template <typename S, typename D>
__global__ __launch_bounds__(256) void convert_kernel(const S* __restrict__ src, D* __restrict__ dst, uint64_t n,
                                                      float mul, int vec_ok) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (vec_ok) {
        const uint64_t groups = n / 8;
        for (uint64_t gi = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; gi < groups; gi += stride) {
            const Vec<S, 8> s = load_vec<S, 8>(src + gi * 8);
            Vec<D, 8> d;
#pragma unroll
            for (int j = 0; j < 8; ++j) d.v[j] = Fmt<D>::store(Fmt<S>::load(s.v[j]) * mul);
            store_vec<D, 8>(dst + gi * 8, d);
        }
        for (uint64_t i = groups * 8 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
            dst[i] = Fmt<D>::store(Fmt<S>::load(src[i]) * mul);
    } else {
        for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
            dst[i] = Fmt<D>::store(Fmt<S>::load(src[i]) * mul);
    }
}

zo2_status convert(const void* src, int sdt, float sscale, void* dst, int ddt, float dscale, uint64_t n, hipStream_t st) {
    if (n == 0) return ZO2_OK;
    ZO2_OP_CHECK(src && dst, ZO2_EINVAL, "convert: NULL buffer");
    ZO2_OP_CHECK(sscale > 0.f && dscale > 0.f, ZO2_EINVAL, "convert: scales must be positive");
    const float mul = dscale / sscale;
    const uint64_t want = (n / 8 + 255) / 256 + 1;
    const unsigned grid = (unsigned)(want > 65536 ? 65536 : want);
    ZO2_DISPATCH_WIRE(sdt, S, {
        ZO2_DISPATCH_WIRE(ddt, D, {
            const int vec_ok = ((uintptr_t)src % (sizeof(S) * 8) == 0) && ((uintptr_t)dst % (sizeof(D) * 8) == 0);
            hipLaunchKernelGGL((convert_kernel<S, D>), dim3(grid), dim3(256), 0, st, (const S*)src, (D*)dst, n, mul, vec_ok);
        });
    });
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ LayerNorm
// One 256-thread workgroup per row.  Rows of up to 12288 elements are read once and held in
// registers for the mean, the centred variance and the output; longer rows are re-read from cache.
template <typename C, bool CACHED>
__global__ __launch_bounds__(256) void layernorm_kernel(const float* __restrict__ x, const C* __restrict__ w, const C* __restrict__ b,
                                                        const C* __restrict__ w2, const C* __restrict__ b2, C* __restrict__ y,
                                                        int rows_first, int d, float eps) {
    constexpr int kMaxVec = 12;                     // float4 per lane held in registers
    __shared__ float sh[4];
    const int r = blockIdx.x;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)r * d);
    const C* ww = r < rows_first ? w : w2;
    const C* bb = r < rows_first ? b : b2;
    const int nv = d >> 2;
    float4 v[kMaxVec];
    float s = 0.f;
    if (CACHED) {
#pragma unroll
        for (int k = 0; k < kMaxVec; ++k) {
            const int i = threadIdx.x + 256 * k;
            v[k] = i < nv ? xr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < kMaxVec; ++k) s += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    } else {
        for (int i = threadIdx.x; i < nv; i += 256) {
            const float4 t = xr[i];
            s += (t.x + t.y) + (t.z + t.w);
        }
    }
    const float mean = block_sum(s, sh) / (float)d;
    float q = 0.f;
    if (CACHED) {
#pragma unroll
        for (int k = 0; k < kMaxVec; ++k) {
            if (threadIdx.x + 256 * k < nv) {
                const float a0 = v[k].x - mean, a1 = v[k].y - mean, a2 = v[k].z - mean, a3 = v[k].w - mean;
                q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
            }
        }
    } else {
        for (int i = threadIdx.x; i < nv; i += 256) {
            const float4 t = xr[i];
            const float a0 = t.x - mean, a1 = t.y - mean, a2 = t.z - mean, a3 = t.w - mean;
            q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    }
    const float var = block_sum(q, sh) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    C* yr = y + (size_t)r * d;
    auto emit = [&](int i, const float4& t) {
        const Vec<C, 4> wv = load_vec<C, 4>(ww + 4 * i), bv = load_vec<C, 4>(bb + 4 * i);
        Vec<C, 4> o;
        o.v[0] = Fmt<C>::store((t.x - mean) * rstd * Fmt<C>::load(wv.v[0]) + Fmt<C>::load(bv.v[0]));
        o.v[1] = Fmt<C>::store((t.y - mean) * rstd * Fmt<C>::load(wv.v[1]) + Fmt<C>::load(bv.v[1]));
        o.v[2] = Fmt<C>::store((t.z - mean) * rstd * Fmt<C>::load(wv.v[2]) + Fmt<C>::load(bv.v[2]));
        o.v[3] = Fmt<C>::store((t.w - mean) * rstd * Fmt<C>::load(wv.v[3]) + Fmt<C>::load(bv.v[3]));
        store_vec<C, 4>(yr + 4 * i, o);
    };
    if (CACHED) {
#pragma unroll
        for (int k = 0; k < kMaxVec; ++k) {
            const int i = threadIdx.x + 256 * k;
            if (i < nv) emit(i, v[k]);
        }
    } else {
        for (int i = threadIdx.x; i < nv; i += 256) emit(i, xr[i]);
    }
}

// One wavefront per row (rows of up to 4 * 64 * KV elements): the row lives in the wave's registers and
// both reductions are cross-lane only, so the four waves of a workgroup never wait for each other.
template <typename C, int KV>
__global__ __launch_bounds__(256) void layernorm_wave_kernel(const float* __restrict__ x, const C* __restrict__ w, const C* __restrict__ b,
                                                             const C* __restrict__ w2, const C* __restrict__ b2, C* __restrict__ y,
                                                             int rows, int rows_first, int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)r * d);
    const C* ww = r < rows_first ? w : w2;
    const C* bb = r < rows_first ? b : b2;
    const int nv = d >> 2;
    float4 v[KV];
#pragma unroll
    for (int k = 0; k < KV; ++k) {
        const int i = lane + 64 * k;
        v[k] = i < nv ? xr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < KV; ++k) s += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < KV; ++k) {
        if (lane + 64 * k < nv) {
            const float a0 = v[k].x - mean, a1 = v[k].y - mean, a2 = v[k].z - mean, a3 = v[k].w - mean;
            q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    }
    const float var = wave_sum(q) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    C* yr = y + (size_t)r * d;
#pragma unroll
    for (int k = 0; k < KV; ++k) {
        const int i = lane + 64 * k;
        if (i < nv) {
            const Vec<C, 4> wv = load_vec<C, 4>(ww + 4 * i), bv = load_vec<C, 4>(bb + 4 * i);
            Vec<C, 4> o;
            o.v[0] = Fmt<C>::store((v[k].x - mean) * rstd * Fmt<C>::load(wv.v[0]) + Fmt<C>::load(bv.v[0]));
            o.v[1] = Fmt<C>::store((v[k].y - mean) * rstd * Fmt<C>::load(wv.v[1]) + Fmt<C>::load(bv.v[1]));
            o.v[2] = Fmt<C>::store((v[k].z - mean) * rstd * Fmt<C>::load(wv.v[2]) + Fmt<C>::load(bv.v[2]));
            o.v[3] = Fmt<C>::store((v[k].w - mean) * rstd * Fmt<C>::load(wv.v[3]) + Fmt<C>::load(bv.v[3]));
            store_vec<C, 4>(yr + 4 * i, o);
        }
    }
}

// The same with 8 consecutive elements per lane and piece (two adjacent 16-byte loads, one 16-byte store of 16-bit
// results): for rows whose length is a multiple of 8.  WAVES rows per workgroup.
template <typename C, int KP, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void layernorm_wave8_kernel(const float* __restrict__ x, const C* __restrict__ w, const C* __restrict__ b,
                                                                     const C* __restrict__ w2, const C* __restrict__ b2, C* __restrict__ y,
                                                                     int rows, int rows_first, int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (r >= rows) return;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)r * d);
    const C* ww = r < rows_first ? w : w2;
    const C* bb = r < rows_first ? b : b2;
    const int n8 = d >> 3;
    float4 v[KP][2];
#pragma unroll
    for (int k = 0; k < KP; ++k) {
        const int i = lane + 64 * k;
        if (i < n8) { v[k][0] = xr[2 * i]; v[k][1] = xr[2 * i + 1]; }
        else v[k][0] = v[k][1] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < KP; ++k)
#pragma unroll
        for (int h = 0; h < 2; ++h) s += (v[k][h].x + v[k][h].y) + (v[k][h].z + v[k][h].w);
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < KP; ++k) {
        if (lane + 64 * k < n8) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float a0 = v[k][h].x - mean, a1 = v[k][h].y - mean, a2 = v[k][h].z - mean, a3 = v[k][h].w - mean;
                q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
            }
        }
    }
    const float var = wave_sum(q) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    C* yr = y + (size_t)r * d;
#pragma unroll
    for (int k = 0; k < KP; ++k) {
        const int i = lane + 64 * k;
        if (i < n8) {
            const Vec<C, 8> wv = load_vec<C, 8>(ww + 8 * i), bv = load_vec<C, 8>(bb + 8 * i);
            Vec<C, 8> o;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                o.v[4 * h + 0] = Fmt<C>::store((v[k][h].x - mean) * rstd * Fmt<C>::load(wv.v[4 * h + 0]) + Fmt<C>::load(bv.v[4 * h + 0]));
                o.v[4 * h + 1] = Fmt<C>::store((v[k][h].y - mean) * rstd * Fmt<C>::load(wv.v[4 * h + 1]) + Fmt<C>::load(bv.v[4 * h + 1]));
                o.v[4 * h + 2] = Fmt<C>::store((v[k][h].z - mean) * rstd * Fmt<C>::load(wv.v[4 * h + 2]) + Fmt<C>::load(bv.v[4 * h + 2]));
                o.v[4 * h + 3] = Fmt<C>::store((v[k][h].w - mean) * rstd * Fmt<C>::load(wv.v[4 * h + 3]) + Fmt<C>::load(bv.v[4 * h + 3]));
            }
            store_vec<C, 8>(yr + 8 * i, o);
        }
    }
}

static constexpr int kLnWaves = 1;      // rows per workgroup of the kernel above (1, 2, 4, 8 measured inside the step: within 2 %, 1 ahead)

zo2_status layernorm(int dtype, const float* x, const void* w, const void* b, const void* w2, const void* b2, void* y,
                     int rows, int rows_first, int d, float eps, hipStream_t st) {
    if (rows == 0) return ZO2_OK;
    ZO2_OP_CHECK(rows > 0 && d > 0 && d % 4 == 0, ZO2_EINVAL, "layernorm: rows %d, d %d (d must be a multiple of 4)", rows, d);
    ZO2_OP_CHECK(x && w && b && y, ZO2_EINVAL, "layernorm: NULL buffer");
    ZO2_OP_CHECK(rows_first >= rows || (w2 && b2), ZO2_EINVAL, "layernorm: second gain / bias missing");
    {   // rows are moved in groups of 4 elements
        const uintptr_t ca = 4 * (uintptr_t)zo2_dtype_size(dtype);
        ZO2_OP_CHECK(ca != 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)y % ca) == 0 && ((uintptr_t)w % ca) == 0 && ((uintptr_t)b % ca) == 0 &&
                     ((uintptr_t)w2 % ca) == 0 && ((uintptr_t)b2 % ca) == 0, ZO2_EINVAL, "layernorm: unknown dtype, or buffers not aligned to 4 elements");
    }
#define ZO2_LN8(KP)                                                                                                                       \
    hipLaunchKernelGGL((layernorm_wave8_kernel<C, KP, kLnWaves>), dim3((rows + kLnWaves - 1) / kLnWaves), dim3(64 * kLnWaves), 0, st, x, \
                       (const C*)w, (const C*)b, (const C*)w2, (const C*)b2, (C*)y, rows, rows_first, d, eps)
    ZO2_DISPATCH_COMPUTE(dtype, C, {
        const bool by8 = sizeof(C) == 2 && d % 8 == 0 && ((uintptr_t)y % 16) == 0 && ((uintptr_t)w % 16) == 0 && ((uintptr_t)b % 16) == 0 &&
                         ((uintptr_t)w2 % 16) == 0 && ((uintptr_t)b2 % 16) == 0;
        // pieces of 512 elements per row: instances for rows of up to 2048 and 5120 elements; longer rows take too many
        // registers for one wavefront (measured at 8192 rows: 5120 46 us against 55 with the kernels below, 7168 76
        // against 69, 12288 145 against 115) and stay with the workgroup-per-row kernel
        if (by8 && d <= 4 * 512) ZO2_LN8(4);
        else if (by8 && d <= 10 * 512) ZO2_LN8(10);
        else if (d <= 8 * 64 * 4)
            hipLaunchKernelGGL((layernorm_wave_kernel<C, 8>), dim3((rows + 3) / 4), dim3(256), 0, st, x, (const C*)w, (const C*)b,
                               (const C*)w2, (const C*)b2, (C*)y, rows, rows_first, d, eps);
        else if (d <= 20 * 64 * 4)
            hipLaunchKernelGGL((layernorm_wave_kernel<C, 20>), dim3((rows + 3) / 4), dim3(256), 0, st, x, (const C*)w, (const C*)b,
                               (const C*)w2, (const C*)b2, (C*)y, rows, rows_first, d, eps);
        else if (d <= 12 * 256 * 4)
            hipLaunchKernelGGL((layernorm_kernel<C, true>), dim3(rows), dim3(256), 0, st, x, (const C*)w, (const C*)b,
                               (const C*)w2, (const C*)b2, (C*)y, rows_first, d, eps);
        else
            hipLaunchKernelGGL((layernorm_kernel<C, false>), dim3(rows), dim3(256), 0, st, x, (const C*)w, (const C*)b,
                               (const C*)w2, (const C*)b2, (C*)y, rows_first, d, eps);
    });
#undef ZO2_LN8
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ embedding gather (Alg. 2, DualForward(Embedding))
// h+[t] = W+tok[id_t] + W+pos[t + off], h-[t] likewise, with the pending update and the
// perturbation evaluated only for the rows the batch touches.  The tables themselves are
// brought up to date by K1 afterwards; both evaluate the same per-element expression.
template <typename W, typename C, bool UPDATE>
__global__ __launch_bounds__(256) void embed_kernel(EmbedArgs a) {
    const int dv = a.d >> 2;
    const int64_t gi = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gi >= (int64_t)a.T * dv) return;
    const int t = (int)(gi / dv), j = (int)(gi % dv) * 4;
    const int id = a.tokens[t];
    const int pos = t % a.seq + a.pos_offset;
    const float c = UPDATE ? *a.c_ptr : 0.f;
    constexpr bool kScaled = (Fmt<W>::kBytes == 1);
    float hp[4] = {0.f, 0.f, 0.f, 0.f}, hm[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const W* table = reinterpret_cast<const W*>(which == 0 ? a.tok_emb : a.pos_emb);
        const uint64_t e = (uint64_t)(which == 0 ? id : pos) * a.d + j;
        const float scale = which == 0 ? a.scale_tok : a.scale_pos, inv_scale = 1.0f / scale;
        const Vec<W, 4> tv = load_vec<W, 4>(table + e);
        float th[4], z[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            th[i] = Fmt<W>::load(tv.v[i]);
            if (kScaled) th[i] *= inv_scale;
        }
        if (UPDATE) {
            gaussian4(a.k_prev, (uint32_t)which, e, z);
            uint32_t rw[4] = {0u, 0u, 0u, 0u};
            const bool sr = Fmt<W>::kBytes < 4 && a.stochastic != 0;
            if (sr) rounding_words(a.k_prev, (uint32_t)which, e >> 3, rw);
            // this group of 4 is the lower or the upper half of its Philox call: rounding words 0, 1 or 2, 3
            const uint32_t r2[2] = {(e & 4) ? rw[2] : rw[0], (e & 4) ? rw[3] : rw[1]};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float u = __builtin_fmaf(-c, z[i], th[i]);
                const float us = kScaled ? u * scale : u;
                const uint32_t r16 = (r2[i >> 1] >> (16 * (i & 1))) & 0xffffu;
                th[i] = Fmt<W>::load(sr ? store_stochastic<W>(us, r16) : Fmt<W>::store(us));
                if (kScaled) th[i] *= inv_scale;
            }
        }
        if (a.single) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hp[i] += Fmt<C>::load(Fmt<C>::store(th[i]));
            continue;
        }
        gaussian4(a.k_cur, (uint32_t)which, e, z);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hp[i] += Fmt<C>::load(Fmt<C>::store(__builtin_fmaf(a.eps, z[i], th[i])));
            hm[i] += Fmt<C>::load(Fmt<C>::store(__builtin_fmaf(-a.eps, z[i], th[i])));
        }
    }
    float* op = a.h + (size_t)t * a.d + j;
    *reinterpret_cast<float4*>(op) = make_float4(hp[0], hp[1], hp[2], hp[3]);
    if (a.single) return;
    float* om = a.h + ((size_t)a.T + t) * a.d + j;
    *reinterpret_cast<float4*>(om) = make_float4(hm[0], hm[1], hm[2], hm[3]);
}

zo2_status embed_gather(const EmbedArgs& a, int wire_dtype, int compute_dtype, bool update, hipStream_t st) {
    if (a.T == 0) return ZO2_OK;
    ZO2_OP_CHECK(a.d % 4 == 0, ZO2_EINVAL, "embed: d %d not a multiple of 4", a.d);
    const int64_t n = (int64_t)a.T * (a.d / 4);
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    ZO2_DISPATCH_WIRE(wire_dtype, W, {
        ZO2_DISPATCH_COMPUTE(compute_dtype, C, {
            if (update) hipLaunchKernelGGL((embed_kernel<W, C, true>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((embed_kernel<W, C, false>), grid, block, 0, st, a);
        });
    });
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ cross-entropy per row
__global__ __launch_bounds__(256) void ce_rows_kernel(const float* __restrict__ logits, int64_t ld, const int32_t* __restrict__ labels,
                                                      int row0, int label_period, int vocab, float* __restrict__ row_loss) {
    __shared__ float shf[4];
    __shared__ double shd[4];
    // logits row blockIdx.x is row (row0 + blockIdx.x) of the stacked [+ rows; - rows] batch
    const int r = row0 + blockIdx.x;
    const int lab = labels[r % label_period];
    if (lab < 0) {                       // ignored position (uniform per workgroup)
        if (threadIdx.x == 0) row_loss[r] = 0.f;
        return;
    }
    const float* lr = logits + (size_t)blockIdx.x * ld;
    // one pass: running maximum m and sum s of exp(x - m) per lane, rescaled when m grows
    float m = -INFINITY, s = 0.f;
    const bool vec = ((ld & 3) == 0) && (((uintptr_t)logits & 15) == 0);
    const int nv = vec ? (vocab >> 2) : 0;
    for (int i = threadIdx.x; i < nv; i += 256) {
        const float4 x = reinterpret_cast<const float4*>(lr)[i];
        const float mx = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
        if (mx > m) { s *= expf(m - mx); m = mx; }
        s += (expf(x.x - m) + expf(x.y - m)) + (expf(x.z - m) + expf(x.w - m));
    }
    for (int i = nv * 4 + threadIdx.x; i < vocab; i += 256) {
        const float x = lr[i];
        if (x > m) { s *= expf(m - x); m = x; }
        s += expf(x - m);
    }
    const float mall = block_max(m, shf);
    const double tot = block_sum((double)(m == -INFINITY ? 0.f : s * expf(m - mall)), shd);
    if (threadIdx.x == 0) row_loss[r] = (float)(log(tot) + (double)mall - (double)lr[lab]);
}

zo2_status cross_entropy_rows(const float* logits, int64_t ld, const int32_t* labels, int rows, int row0, int label_period,
                              int vocab, float* row_loss, hipStream_t st) {
    if (rows == 0) return ZO2_OK;
    ZO2_OP_CHECK(logits && labels && row_loss, ZO2_EINVAL, "cross_entropy: NULL buffer");
    ZO2_OP_CHECK(vocab > 0 && ld >= vocab && label_period > 0 && row0 >= 0, ZO2_EINVAL, "cross_entropy: bad shape");
    hipLaunchKernelGGL(ce_rows_kernel, dim3(rows), dim3(256), 0, st, logits, ld, labels, row0, label_period, vocab, row_loss);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ combine the LM-head kernel's cross-entropy partials
// Row r has n_parts pairs (m_i, s_i), span-major ([i * part_ld + r]), with s_i = sum over a 64-column span of
// exp(y - m_i); then logsumexp = M + log(sum_i s_i exp(m_i - M)), M = max_i m_i.
__global__ __launch_bounds__(256) void ce_combine_kernel(const float* __restrict__ part_max, const float* __restrict__ part_sum,
                                                         const float* __restrict__ label_logit, const int32_t* __restrict__ labels,
                                                         int rows, int n_parts, int64_t part_ld, int row0, int label_period,
                                                         float* __restrict__ row_loss) {
    // 32 rows per block; 8 groups of lanes split the spans, so every load is 32 consecutive floats.
    // Two sweeps (max, then sum) keep the loads independent of each other.
    constexpr int kRows = 32, kGroups = 8;
    __shared__ float sh_m[kGroups][kRows];
    __shared__ double sh_s[kGroups][kRows];
    const int lr = threadIdx.x & (kRows - 1), grp = threadIdx.x / kRows;
    const int r = blockIdx.x * kRows + lr;
    const int rc = r < rows ? r : rows - 1;
    const float* pm = part_max + rc;
    const float* ps = part_sum + rc;
    float m = -INFINITY;
#pragma unroll 4
    for (int i = grp; i < n_parts; i += kGroups) m = fmaxf(m, pm[(size_t)i * part_ld]);
    double s = 0.0;
    if (m != -INFINITY) {
#pragma unroll 4
        for (int i = grp; i < n_parts; i += kGroups) {
            const float mi = pm[(size_t)i * part_ld];
            s += (double)(ps[(size_t)i * part_ld] * expf(mi - m));     // a span past the last column has sum 0 and exp(-inf) = 0
        }
    }
    sh_m[grp][lr] = m;
    sh_s[grp][lr] = s;
    __syncthreads();
    if (grp != 0 || r >= rows) return;
    const int lab = labels[(row0 + r) % label_period];
    if (lab < 0) {
        row_loss[row0 + r] = 0.f;
        return;
    }
    float mm = -INFINITY;
#pragma unroll
    for (int k = 0; k < kGroups; ++k) mm = fmaxf(mm, sh_m[k][lr]);
    double ss = 0.0;
#pragma unroll
    for (int k = 0; k < kGroups; ++k)
        if (sh_m[k][lr] != -INFINITY) ss += sh_s[k][lr] * (double)expf(sh_m[k][lr] - mm);
    row_loss[row0 + r] = (float)(log(ss) + (double)mm - (double)label_logit[r]);
}

zo2_status ce_combine(const float* part_max, const float* part_sum, const float* label_logit, const int32_t* labels, int rows,
                      int n_parts, int64_t part_ld, int row0, int label_period, float* row_loss, hipStream_t st) {
    if (rows == 0) return ZO2_OK;
    ZO2_OP_CHECK(part_max && part_sum && label_logit && labels && row_loss && n_parts > 0 && label_period > 0 && part_ld >= rows,
                 ZO2_EINVAL, "ce_combine: bad argument");
    hipLaunchKernelGGL(ce_combine_kernel, dim3((rows + 31) / 32), dim3(256), 0, st, part_max, part_sum, label_logit, labels, rows, n_parts,
                       part_ld, row0, label_period, row_loss);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// ------------------------------------------------------------------ scalar epilogue (Eq. 2)
// l+ = mean of row_loss[0..T) over non-ignored labels, l- of row_loss[T..2T);
// g = (l+ - l-) / (2 eps); the pending step c = lr * g stays in device memory.
__global__ __launch_bounds__(256) void loss_epilogue_kernel(const float* __restrict__ row_loss, const int32_t* __restrict__ labels,
                                                            int T, float eps, float lr, int ns, float* __restrict__ result,
                                                            float* __restrict__ c_pending) {
    __shared__ double shd[4];
    double sp = 0.0, sm = 0.0, cnt = 0.0;
    for (int i = threadIdx.x; i < T; i += 256) {
        if (labels[i] >= 0) {
            sp += (double)row_loss[i];
            if (ns == 2) sm += (double)row_loss[T + i];
            cnt += 1.0;
        }
    }
    sp = block_sum(sp, shd);
    sm = block_sum(sm, shd);
    cnt = block_sum(cnt, shd);
    if (threadIdx.x == 0) {
        const float lp = (float)(sp / cnt), lm = ns == 2 ? (float)(sm / cnt) : lp;
        const float g = ns == 2 ? (lp - lm) / (2.0f * eps) : 0.f;
        result[0] = lp;
        result[1] = lm;
        result[2] = g;
        result[3] = (float)cnt;
        if (ns == 2) *c_pending = lr * g;
    }
}

zo2_status loss_epilogue(const float* row_loss, const int32_t* labels, int T, float eps, float lr, int ns, float* result,
                         float* c_pending, hipStream_t st) {
    hipLaunchKernelGGL(loss_epilogue_kernel, dim3(1), dim3(256), 0, st, row_loss, labels, T, eps, lr, ns, result, c_pending);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

}  // namespace zo2
