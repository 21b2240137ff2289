// Causal multi-head self-attention of the decoder block (Alg. 2 "forward"), flash style:
// keys / values are visited in tiles staged through LDS, the softmax is accumulated online,
// and the S x S score matrix is never written to memory.
//
// Vector-ALU kernel with float32 arithmetic throughout (used by the float32 mode, whose
// losses must track a float64 reference to 1e-5, and as the general fallback): one
// wavefront per 64 queries of one (sequence, head); a lane owns one query row.
#include "attention.h"

namespace zo2 {

template <typename T, int DH>
__global__ __launch_bounds__(64) void attention_valu_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                                            T* __restrict__ out, int seq, int64_t ld) {
    constexpr int KT = 16;                     // keys per tile
    __shared__ float Ks[KT][DH];
    __shared__ float Vs[KT][DH];
    const int lane = threadIdx.x;
    const int q0 = blockIdx.x * 64, head = blockIdx.y, sq = blockIdx.z;
    const size_t base = (size_t)sq * seq * ld + (size_t)head * DH;
    const int i = q0 + lane;                   // this lane's query position
    const bool live = i < seq;
    float qr[DH], o[DH];
#pragma unroll
    for (int d = 0; d < DH; d += 8) {
        Vec<T, 8> t;
        if (live) t = load_vec<T, 8>(q + base + (size_t)i * ld + d);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qr[d + e] = live ? Fmt<T>::load(t.v[e]) : 0.f;
            o[d + e] = 0.f;
        }
    }
    float m = -INFINITY, l = 0.f;
    const int jend = min(seq, q0 + 64);
    for (int j0 = 0; j0 < jend; j0 += KT) {
        __syncthreads();
        // stage KT keys and values: KT * DH / 8 chunks of 8 elements over 64 lanes
        for (int c = lane; c < KT * DH / 8; c += 64) {
            const int jj = c / (DH / 8), d = (c % (DH / 8)) * 8;
            const int j = j0 + jj;
            if (j < seq) {
                const Vec<T, 8> kk = load_vec<T, 8>(k + base + (size_t)j * ld + d);
                const Vec<T, 8> vv = load_vec<T, 8>(v + base + (size_t)j * ld + d);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    Ks[jj][d + e] = Fmt<T>::load(kk.v[e]);
                    Vs[jj][d + e] = Fmt<T>::load(vv.v[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) { Ks[jj][d + e] = 0.f; Vs[jj][d + e] = 0.f; }
            }
        }
        __syncthreads();
        float s[KT];
        float tmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < KT; ++jj) {
            float acc = 0.f;
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(&Ks[jj][d]);
                acc = __builtin_fmaf(qr[d], kv.x, acc);
                acc = __builtin_fmaf(qr[d + 1], kv.y, acc);
                acc = __builtin_fmaf(qr[d + 2], kv.z, acc);
                acc = __builtin_fmaf(qr[d + 3], kv.w, acc);
            }
            const bool ok = live && (j0 + jj <= i);
            s[jj] = ok ? acc : -INFINITY;
            tmax = fmaxf(tmax, s[jj]);
        }
        if (tmax == -INFINITY) continue;       // nothing visible for this lane in the tile (uniform barriers: none inside)
        const float mn = fmaxf(m, tmax);
        const float resc = expf(m - mn);       // exp(-inf) = 0 on the first visible tile
        l *= resc;
#pragma unroll
        for (int d = 0; d < DH; ++d) o[d] *= resc;
#pragma unroll
        for (int jj = 0; jj < KT; ++jj) {
            const float pj = expf(s[jj] - mn);  // 0 for masked keys
            l += pj;
#pragma unroll
            for (int d = 0; d < DH; d += 4) {
                const float4 vv = *reinterpret_cast<const float4*>(&Vs[jj][d]);
                o[d] = __builtin_fmaf(pj, vv.x, o[d]);
                o[d + 1] = __builtin_fmaf(pj, vv.y, o[d + 1]);
                o[d + 2] = __builtin_fmaf(pj, vv.z, o[d + 2]);
                o[d + 3] = __builtin_fmaf(pj, vv.w, o[d + 3]);
            }
        }
        m = mn;
    }
    if (live) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int d = 0; d < DH; d += 8) {
            Vec<T, 8> t;
#pragma unroll
            for (int e = 0; e < 8; ++e) t.v[e] = Fmt<T>::store(o[d + e] * inv);
            store_vec<T, 8>(out + base + (size_t)i * ld + d, t);
        }
    }
}

template <typename T>
static zo2_status launch_valu(const T* q, const T* k, const T* v, T* out, int n_seq, int seq, int n_heads, int d_head,
                              int64_t ld, hipStream_t st) {
    const dim3 grid((seq + 63) / 64, n_heads, n_seq), block(64);
    switch (d_head) {
#define ZO2_ATT_CASE(D) \
    case D: hipLaunchKernelGGL((attention_valu_kernel<T, D>), grid, block, 0, st, q, k, v, out, seq, ld); break;
        ZO2_ATT_CASE(8) ZO2_ATT_CASE(16) ZO2_ATT_CASE(32) ZO2_ATT_CASE(64) ZO2_ATT_CASE(128)
#undef ZO2_ATT_CASE
        default:
            set_op_error("attention: d_head %d not supported (8, 16, 32, 64, 128)", d_head);
            return ZO2_EINVAL;
    }
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

zo2_status attention_launch(int dtype, const void* q, const void* k, const void* v, void* out,
                            int n_seq, int seq, int n_heads, int d_head, int64_t ld, hipStream_t st) {
    if (n_seq == 0 || seq == 0) return ZO2_OK;
    ZO2_OP_CHECK(n_seq > 0 && seq > 0 && n_heads > 0 && d_head > 0, ZO2_EINVAL, "attention: bad shape");
    ZO2_OP_CHECK(q && k && v && out, ZO2_EINVAL, "attention: NULL buffer");
    ZO2_OP_CHECK(ld >= (int64_t)n_heads * d_head && ld % 8 == 0, ZO2_EINVAL, "attention: bad leading dimension");
    ZO2_OP_CHECK(n_seq <= 65535 && n_heads <= 65535, ZO2_EINVAL, "attention: grid too large");
    ZO2_DISPATCH_COMPUTE(dtype, T, {
        return launch_valu<T>((const T*)q, (const T*)k, (const T*)v, (T*)out, n_seq, seq, n_heads, d_head, ld, st);
    });
    return ZO2_OK;
}

}  // namespace zo2
