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
#include <math.h>

#include "k1.h"
#include "philox.h"

namespace zo2 {

static constexpr int kThreads = 256;
static constexpr int kPerLane = 8;
// one group per lane and workgroup: measured inside the step, workgroups of 2048 elements sweep a block at 6.4 TB/s,
// of 8192 (four groups per lane, all loads up front) at 5.9 - many small workgroups keep the streams of consecutive
// addresses denser than few large ones
static constexpr int kIters = 1;
static constexpr int kChunk = kThreads * kPerLane * kIters;   // 2048 elements per workgroup

// The arithmetic of one group of 8 consecutive elements (one Philox call q per random stream): tv holds
// theta on entry and theta' on return.
template <typename W, typename C, bool UPDATE, bool PERTURB, bool SR, bool DRAW>
__device__ __forceinline__ void k1_group(const K1Args& a, uint32_t tensor_id, uint64_t q, float c, float eps, float scale,
                                         float inv_scale, Vec<W, kPerLane>& tv, Vec<C, kPerLane>& p, Vec<C, kPerLane>& m) {
    constexpr bool kScaled = (Fmt<W>::kBytes == 1);
    float th[kPerLane];
    if constexpr (kScaled) {        // 8-bit storage: the group's eight bytes are converted by the packed hardware instructions
        fp8_decode8<W>(tv, th);
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) th[j] *= inv_scale;
    } else {
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) th[j] = Fmt<W>::load(tv.v[j]);
    }
    if (UPDATE) {
        float zp[kPerLane];
        gaussian8(a.k_prev, tensor_id, q, zp);
        uint32_t rw[4] = {0u, 0u, 0u, 0u};
        constexpr bool sr = SR && Fmt<W>::kBytes < 4;
        if (sr) rounding_words(a.k_prev, tensor_id, q, rw);
        if constexpr (kScaled && !sr) {
            float ts[kPerLane];
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) ts[j] = __builtin_fmaf(-c, zp[j], th[j]) * scale;
            fp8_encode8<W>(ts, tv);
            fp8_decode8<W>(tv, th);
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) th[j] *= inv_scale;
        } else {
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const float t = __builtin_fmaf(-c, zp[j], th[j]);
                const float ts = kScaled ? t * scale : t;
                tv.v[j] = sr ? store_stochastic<W>(ts, rounding_bits_of(rw, j)) : Fmt<W>::store(ts);
                th[j] = Fmt<W>::load(tv.v[j]);
                if (kScaled) th[j] *= inv_scale;
            }
        }
    }
    if constexpr (PERTURB && DRAW) {
        float z[kPerLane];
        gaussian8(a.k_cur, tensor_id, q, z);
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) {
            p.v[j] = Fmt<C>::store(__builtin_fmaf(eps, z[j], th[j]));
            m.v[j] = Fmt<C>::store(__builtin_fmaf(-eps, z[j], th[j]));
        }
    } else if constexpr (PERTURB) {
        // eps = 0 (the single forward of an evaluation): W+ = theta' in the compute format, nothing to draw.  A kernel
        // instance of its own, chosen on the host: as a branch on eps inside one instance the two paths' 16-bit results
        // were merged through scratch memory.
#pragma unroll
        for (int j = 0; j < kPerLane; ++j) p.v[j] = m.v[j] = Fmt<C>::store(th[j]);
    }
}

template <typename W, typename C, bool UPDATE, bool PERTURB, bool SR, bool DRAW>
__global__ __launch_bounds__(kThreads) void k1_kernel(const K1Args a) {
    // which tensor does this workgroup work on: first_chunk[] ascends (0xffffffff past the last segment),
    // so the segment index is the number of entries at or below this workgroup's index
    // Workgroups are dispatched in index order; chunks are taken in the opposite order, so that the sweep ends with
    // the first tensors of the list: the projections that run right after the sweep (q, k, v of a block) then find
    // their perturbed copies still in the memory-side cache, which a whole block's copies exceed.
    const uint32_t chunk = a.reverse ? a.total_chunks - 1u - blockIdx.x : blockIdx.x;
    int s = 0;
#pragma unroll
    for (int i = 1; i < K1Args::kMaxSeg; ++i) s += (chunk >= a.first_chunk[i]) ? 1 : 0;
    const K1Seg sg = a.seg[s];
    const uint64_t chunk0 = (uint64_t)(chunk - a.first_chunk[s]) * kChunk;
    W* __restrict__ theta = reinterpret_cast<W*>(a.theta) + sg.off;
    const int64_t wofs = a.packed_w ? sg.woff : sg.off - a.w_off0;
    C* __restrict__ wp = PERTURB ? reinterpret_cast<C*>(a.w_plus) + wofs : nullptr;
    const bool has_m = PERTURB && a.w_minus != nullptr;            // a single forward needs W+ only
    C* __restrict__ wm = has_m ? reinterpret_cast<C*>(a.w_minus) + wofs : nullptr;
    const float c = UPDATE ? (a.c_ptr ? *a.c_ptr : a.c_imm) : 0.f;
    const float eps = a.eps;
    const float scale = sg.scale, inv_scale = 1.0f / sg.scale;
    constexpr int kStride = kThreads * kPerLane;

    if (chunk0 + kChunk <= sg.n) {
        // whole chunk inside the tensor (all but the last workgroup of a segment): every load is in
        // flight before the first group is computed, and nothing is masked
        const uint64_t i0 = chunk0 + (uint64_t)threadIdx.x * kPerLane;
        Vec<W, kPerLane> tv[kIters];
#pragma unroll
        // (theta is read once per step: loaded with the streaming policy it leaves the caches to the perturbed copies,
        // which the projections read next - the sweep itself runs 5 % faster and the projections 1 %)
        for (int it = 0; it < kIters; ++it) tv[it] = load_vec_stream<W, kPerLane>(theta + i0 + (uint64_t)it * kStride);
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const uint64_t i = i0 + (uint64_t)it * kStride;
            Vec<C, kPerLane> p, m;
            k1_group<W, C, UPDATE, PERTURB, SR, DRAW>(a, sg.tensor_id, (sg.e0 + i) >> 3, c, eps, scale, inv_scale, tv[it], p, m);
            // (theta' is not read again before the next step when the perturbed copies are written here: streamed past the
            // caches it leaves them to the copies; in an update-only sweep the projections read theta' next, so it stays)
            if (UPDATE && PERTURB) store_vec_stream<W, kPerLane>(theta + i, tv[it]);
            else if (UPDATE) store_vec<W, kPerLane>(theta + i, tv[it]);
            if (PERTURB) {
                store_vec<C, kPerLane>(wp + i, p);
                if (has_m) store_vec<C, kPerLane>(wm + i, m);
            }
        }
        return;
    }
    // last chunk of a segment: ragged end, element-wise masking
#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
        const uint64_t i0 = chunk0 + (uint64_t)it * kStride + (uint64_t)threadIdx.x * kPerLane;
        if (i0 >= sg.n) break;
        const int valid = (sg.n - i0 >= (uint64_t)kPerLane) ? kPerLane : (int)(sg.n - i0);
        Vec<W, kPerLane> tv;
        if (valid == kPerLane) {
            tv = load_vec<W, kPerLane>(theta + i0);
        } else {
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) tv.v[j] = (j < valid) ? theta[i0 + j] : Fmt<W>::store(0.f);
        }
        Vec<C, kPerLane> p, m;
        k1_group<W, C, UPDATE, PERTURB, SR, DRAW>(a, sg.tensor_id, (sg.e0 + i0) >> 3, c, eps, scale, inv_scale, tv, p, m);
        if (valid == kPerLane) {
            if (UPDATE && PERTURB) store_vec_stream<W, kPerLane>(theta + i0, tv);
            else if (UPDATE) store_vec<W, kPerLane>(theta + i0, tv);
            if (PERTURB) {
                store_vec<C, kPerLane>(wp + i0, p);
                if (has_m) store_vec<C, kPerLane>(wm + i0, m);
            }
        } else {
#pragma unroll
            for (int j = 0; j < kPerLane; ++j)
                if (j < valid) {
                    if (UPDATE) theta[i0 + j] = tv.v[j];
                    if (PERTURB) { wp[i0 + j] = p.v[j]; if (has_m) wm[i0 + j] = m.v[j]; }
                }
        }
    }
}

template <typename W, typename C>
static zo2_status launch_wc(const K1Args& a, bool update, bool perturb, hipStream_t st) {
    const dim3 grid(a.total_chunks), block(kThreads);
    const bool sr = update && a.stochastic != 0 && sizeof(W) < 4;      // stochastic rounding only concerns a low-bit theta'
    const bool draw = a.eps != 0.f;
#define ZO2_K1_LAUNCH(U, P, S, D) hipLaunchKernelGGL((k1_kernel<W, C, U, P, S, D>), grid, block, 0, st, a)
    if (update && perturb && sr) { if (draw) ZO2_K1_LAUNCH(true, true, true, true); else ZO2_K1_LAUNCH(true, true, true, false); }
    else if (update && perturb) { if (draw) ZO2_K1_LAUNCH(true, true, false, true); else ZO2_K1_LAUNCH(true, true, false, false); }
    else if (update && sr) ZO2_K1_LAUNCH(true, false, true, false);
    else if (update) ZO2_K1_LAUNCH(true, false, false, false);
    else if (perturb) { if (draw) ZO2_K1_LAUNCH(false, true, false, true); else ZO2_K1_LAUNCH(false, true, false, false); }
#undef ZO2_K1_LAUNCH
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
        int ex = 0;
        ZO2_OP_CHECK(a.seg[i].scale > 0.f && isfinite(a.seg[i].scale) && frexpf(a.seg[i].scale, &ex) == 0.5f, ZO2_EINVAL,
                     "k1: segment %d has scale %g (must be a power of two)", i, (double)a.seg[i].scale);
        a.first_chunk[i] = chunks;
        const uint64_t nc = (a.seg[i].n + kChunk - 1) / kChunk;
        ZO2_OP_CHECK(chunks + nc < 0x7fffffffull, ZO2_EINVAL, "k1: too many chunks");
        chunks += (uint32_t)nc;
    }
    for (int i = a.nseg; i < K1Args::kMaxSeg; ++i) a.first_chunk[i] = 0xffffffffu;
    a.total_chunks = chunks;
    if (chunks == 0 || (!update && !perturb)) return ZO2_OK;
    ZO2_OP_CHECK(a.theta != nullptr, ZO2_EINVAL, "k1: theta is NULL");
    ZO2_OP_CHECK(!perturb || a.w_plus, ZO2_EINVAL, "k1: W+ missing");
    ZO2_DISPATCH_WIRE(wire_dtype, W, {
        ZO2_DISPATCH_COMPUTE(compute_dtype, C, { return launch_wc<W, C>(a, update, perturb, st); });
    });
    return ZO2_OK;
}

}  // namespace zo2
