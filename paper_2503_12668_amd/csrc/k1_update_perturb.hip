// K1: fused regenerate + deferred update + perturb (Alg. 2 DualForward, Sec. 5.4).
//
// The paper sweeps a module's parameters four times per iteration (update, +eps, -2eps,
// +eps), drawing a fresh Gaussian vector each time.  Here one sweep reads theta once,
// regenerates z_prev (last iteration's direction) and z (this iteration's) from their
// counters, writes theta' = theta - c z_prev back in the transfer format, and writes the
// two perturbed copies W+ = theta' + eps z, W- = theta' - eps z in the compute format.
// theta itself is never perturbed, so "restore" costs nothing and is exact.
//
// HBM-streaming kernel: each lane moves groups of 8 consecutive elements with 128-bit
// accesses (bf16/fp16; two for fp32, one 64-bit for the 8-bit formats), a workgroup owns
// a contiguous chunk of one tensor, the grid covers up to 16 tensors of a bucket.
#include "k1.h"
#include "philox.h"

namespace zo2 {

static constexpr int kThreads = 256;
static constexpr int kPerLane = 8;
static constexpr int kIters = 4;
static constexpr int kChunk = kThreads * kPerLane * kIters;   // 8192 elements per workgroup

template <typename W, typename C, bool UPDATE, bool PERTURB>
__global__ __launch_bounds__(kThreads) void k1_kernel(const K1Args a) {
    // which tensor does this workgroup work on (wave-uniform search)
    int s = 0;
#pragma unroll 1
    for (int i = 1; i < a.nseg; ++i)
        if (blockIdx.x >= a.seg[i].first_chunk) s = i;
    const K1Seg sg = a.seg[s];
    const uint64_t chunk0 = (uint64_t)(blockIdx.x - sg.first_chunk) * kChunk;
    W* __restrict__ theta = reinterpret_cast<W*>(a.theta) + sg.off;
    C* __restrict__ wp = PERTURB ? reinterpret_cast<C*>(a.w_plus) + (sg.off - a.w_off0) : nullptr;
    C* __restrict__ wm = PERTURB ? reinterpret_cast<C*>(a.w_minus) + (sg.off - a.w_off0) : nullptr;
    const float c = UPDATE ? (a.c_ptr ? *a.c_ptr : a.c_imm) : 0.f;
    const float eps = a.eps;
    const float scale = sg.scale, inv_scale = 1.0f / sg.scale;
    constexpr bool kScaled = (Fmt<W>::kBytes == 1);

#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const uint64_t i0 = chunk0 + (uint64_t)it * (kThreads * kPerLane) + (uint64_t)threadIdx.x * kPerLane;
        if (i0 >= sg.n) break;
        const int valid = (sg.n - i0 >= (uint64_t)kPerLane) ? kPerLane : (int)(sg.n - i0);
        Vec<W, kPerLane> tv;
        if (valid == kPerLane) {
            tv = load_vec<W, kPerLane>(theta + i0);
        } else {
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) tv.v[j] = (j < valid) ? theta[i0 + j] : Fmt<W>::store(0.f);
        }
        float th[kPerLane];
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            th[j] = Fmt<W>::load(tv.v[j]);
            if (kScaled) th[j] *= inv_scale;
        }
        const uint64_t q = (sg.e0 + i0) >> 2;
        if (UPDATE) {
            float zp[kPerLane];
            gaussian4(a.k_prev, sg.tensor_id, q, zp);
            gaussian4(a.k_prev, sg.tensor_id, q + 1, zp + 4);
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const float t = __builtin_fmaf(-c, zp[j], th[j]);
                tv.v[j] = Fmt<W>::store(kScaled ? t * scale : t);
                th[j] = Fmt<W>::load(tv.v[j]);
                if (kScaled) th[j] *= inv_scale;
            }
            if (valid == kPerLane) {
                store_vec<W, kPerLane>(theta + i0, tv);
            } else {
#pragma unroll
                for (int j = 0; j < kPerLane; ++j)
                    if (j < valid) theta[i0 + j] = tv.v[j];
            }
        }
        if (PERTURB) {
            float z[kPerLane];
            gaussian4(a.k_cur, sg.tensor_id, q, z);
            gaussian4(a.k_cur, sg.tensor_id, q + 1, z + 4);
            Vec<C, kPerLane> p, m;
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                p.v[j] = Fmt<C>::store(__builtin_fmaf(eps, z[j], th[j]));
                m.v[j] = Fmt<C>::store(__builtin_fmaf(-eps, z[j], th[j]));
            }
            if (valid == kPerLane) {
                store_vec<C, kPerLane>(wp + i0, p);
                store_vec<C, kPerLane>(wm + i0, m);
            } else {
#pragma unroll
                for (int j = 0; j < kPerLane; ++j)
                    if (j < valid) { wp[i0 + j] = p.v[j]; wm[i0 + j] = m.v[j]; }
            }
        }
    }
}

template <typename W, typename C>
static zo2_status launch_wc(const K1Args& a, bool update, bool perturb, hipStream_t st) {
    const dim3 grid(a.total_chunks), block(kThreads);
    if (update && perturb) hipLaunchKernelGGL((k1_kernel<W, C, true, true>), grid, block, 0, st, a);
    else if (update) hipLaunchKernelGGL((k1_kernel<W, C, true, false>), grid, block, 0, st, a);
    else if (perturb) hipLaunchKernelGGL((k1_kernel<W, C, false, true>), grid, block, 0, st, a);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

uint32_t k1_chunks(uint64_t n) { return (uint32_t)((n + kChunk - 1) / kChunk); }

zo2_status k1_launch(K1Args& a, int wire_dtype, int compute_dtype, bool update, bool perturb, hipStream_t st) {
    ZO2_OP_CHECK(a.nseg >= 1 && a.nseg <= K1Args::kMaxSeg, ZO2_EINVAL, "k1: %d segments", a.nseg);
    uint32_t chunks = 0;
    for (int i = 0; i < a.nseg; ++i) {
        ZO2_OP_CHECK((a.seg[i].e0 & 7) == 0 && (a.seg[i].off & 7) == 0, ZO2_EINVAL,
                     "k1: segment %d not aligned to 8 elements", i);
        ZO2_OP_CHECK(a.seg[i].scale > 0.f, ZO2_EINVAL, "k1: segment %d has scale %g", i, (double)a.seg[i].scale);
        a.seg[i].first_chunk = chunks;
        const uint64_t nc = (a.seg[i].n + kChunk - 1) / kChunk;
        ZO2_OP_CHECK(chunks + nc < 0x7fffffffull, ZO2_EINVAL, "k1: too many chunks");
        chunks += (uint32_t)nc;
    }
    a.total_chunks = chunks;
    if (chunks == 0 || (!update && !perturb)) return ZO2_OK;
    ZO2_OP_CHECK(a.theta != nullptr, ZO2_EINVAL, "k1: theta is NULL");
    ZO2_OP_CHECK(!perturb || (a.w_plus && a.w_minus), ZO2_EINVAL, "k1: W+/W- missing");
    ZO2_DISPATCH_WIRE(wire_dtype, W, {
        ZO2_DISPATCH_COMPUTE(compute_dtype, C, { return launch_wc<W, C>(a, update, perturb, st); });
    });
    return ZO2_OK;
}

}  // namespace zo2
