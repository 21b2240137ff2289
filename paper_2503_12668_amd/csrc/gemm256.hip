// Large-tile MFMA GEMM for the big projections: 256 x 256 x 64 block tile, four wavefronts
// (2 x 2), each owning 128 x 128 = 4 x 4 MFMA tiles of 32 x 32 with float32 accumulators in
// the accumulation registers.  One workgroup per compute unit.
//
// Data path: global memory -> LDS with the direct-to-LDS loads of gfx950 (16 bytes per
// lane, no staging through vector registers), two LDS stages of 64 KB, 128-bit LDS reads
// into MFMA operand registers.  The tile is stored as rows of 8 chunks of 16 bytes with the
// chunk index XOR-swizzled by (row & 7); because a direct-to-LDS load writes lane i's 16 bytes
// at LDS offset 16 i, the swizzle is applied on the global side: lane i fetches the chunk that
// belongs at position i.
//
// Requires K % 64 == 0; M and N are arbitrary (rows are clamped on load, masked on store).
#include <type_traits>

#include "gemm.h"

namespace zo2 {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

template <typename T> struct Mfma32;
template <> struct Mfma32<bf16_t> {
    static __device__ __forceinline__ f32x16_t run(uint4 a, uint4 b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma32<f16_t> {
    static __device__ __forceinline__ f32x16_t run(uint4 a, uint4 b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

#ifndef ZO2_GEMM_SWZ_SHIFT
#define ZO2_GEMM_SWZ_SHIFT 0
#endif
static constexpr int kBM = 256, kBN = 256, kBK = 64;
static constexpr int kStageBytes = (kBM + kBN) * kBK * 2;      // 65536
static constexpr int kLdsBytes = 4 * 34816;                    // two 64 KB stages; the epilogue needs 4 x 34816

// direct-to-LDS load of 16 bytes per lane: lane i's data lands at lds_base + 16 i
__device__ __forceinline__ void load_to_lds(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory");
}

// swizzle of the 16-byte chunk index inside a 128-byte tile row
__device__ __forceinline__ int swz(int row) { return (row >> ZO2_GEMM_SWZ_SHIFT) & 7; }

template <typename T, typename OutT>
__global__ __launch_bounds__(256, 1) void gemm_mfma256_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const GemmProblem p = a.p[blockIdx.z];
    const int tiles_n = (a.N + kBN - 1) / kBN;
    const int tiles_m = (a.M + kBM - 1) / kBM;
    // XCD-aware order: consecutive workgroup ids go to different XCDs (8 of them, each with its
    // own L2), so give each XCD a contiguous run of tiles, and walk tiles in groups of 8 rows
    // of the tile grid so that concurrently running workgroups share operand panels.
    const int ntiles = tiles_m * tiles_n;
    int vid = blockIdx.x;
    if (ntiles % 8 == 0) vid = (vid & 7) * (ntiles >> 3) + (vid >> 3);
    constexpr int GM = 8;
    const int group = vid / (GM * tiles_n);
    const int gm0 = group * GM;
    const int gsz = min(GM, tiles_m - gm0);
    const int tm = gm0 + (vid % (GM * tiles_n)) % gsz;
    const int tn = (vid % (GM * tiles_n)) / gsz;
    const int m0 = tm * kBM, n0 = tn * kBN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1, r = lane & 31, kh = lane >> 5;
    const T* __restrict__ X = reinterpret_cast<const T*>(p.X);
    const T* __restrict__ W = reinterpret_cast<const T*>(p.W);

    // loader plan: per stage each wavefront brings 64 rows of A and 64 rows of B, 8 rows per
    // instruction; lane -> (row lane/8, position lane%8) and the chunk that belongs there
    const int lrow = lane >> 3;
    const T* pa[8];
    const T* pb[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int row = wave * 64 + t * 8 + lrow;
        const int lkc = (lane & 7) ^ swz(row);
        pa[t] = X + (size_t)min(m0 + row, a.M - 1) * a.ldx + lkc * 8;
        pb[t] = W + (size_t)min(n0 + row, a.N - 1) * a.ldw + lkc * 8;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;   // LDS byte address
    const uint32_t ld_a = lds0 + wave * 8192, ld_b = lds0 + 32768 + wave * 8192;

    // fragment read plan: row (w*128 + i*32 + r), chunk (2 ks + kh) ^ swz(row); swz(row) = swz(r)
    const uint32_t fr_a = (wm * 128 + r) * 128, fr_b = 32768 + (wn * 128 + r) * 128;
    uint32_t koff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = (uint32_t)(((ks * 2 + kh) ^ swz(r)) * 16);

    // acc[i][j]: X rows (m) i-th 32-block, W rows (n) j-th 32-block.  The W fragment is the
    // MFMA "A" operand, so a lane ends up with one m (= r) and runs of 4 consecutive n.
    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 fa[2][4], fb[2][4];
    // One "group" = the four MFMAs of X row-block i at k-step buffer `buf`, preceded by the two
    // LDS reads that fetch row-block i of both operands for the next k-step into buffer `nbuf`,
    // and optionally two direct-to-LDS loads of the tile after next.  A scheduling barrier after
    // every group keeps memory instructions spread evenly under the MFMAs instead of bunched.
    auto mgroup = [&](int i, int buf, int nbuf, bool do_read, const char* sa, const char* sb, bool do_dma, int dma_stage, int dma_k0, int dma_t) {
        if (do_dma) {
            const uint32_t so = dma_stage * kStageBytes;
            load_to_lds(pa[dma_t] + dma_k0, ld_a + so + dma_t * 1024);
            load_to_lds(pb[dma_t] + dma_k0, ld_b + so + dma_t * 1024);
        }
#ifndef ZO2_GEMM_EXP_NOREAD
        if (do_read) {
            fa[nbuf][i] = *reinterpret_cast<const uint4*>(sa + i * 4096);
            fb[nbuf][i] = *reinterpret_cast<const uint4*>(sb + i * 4096);
        }
#endif
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = Mfma32<T>::run(fb[buf][j], fa[buf][i], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int nk = a.K / kBK;
    // prologue: tile 0 into stage 0, its first fragments into buffer 0
    {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            load_to_lds(pa[t], ld_a + t * 1024);
            load_to_lds(pb[t], ld_b + t * 1024);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        const char* sa = smem + fr_a + koff[0];
        const char* sb = smem + fr_b + koff[0];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[0][i] = *reinterpret_cast<const uint4*>(sa + i * 4096);
            fb[0][i] = *reinterpret_cast<const uint4*>(sb + i * 4096);
        }
    }
    // `more`: another tile follows (its loads are issued under k-steps 0 and 1, its first
    // fragments are read under k-step 3); compile-time so that no group carries a branch
    auto tile_iter = [&](int kt, auto more_c) {
        constexpr bool more = decltype(more_c)::value;
#ifdef ZO2_GEMM_EXP_NODMA
        constexpr bool dma = false;
#else
        constexpr bool dma = more;
#endif
        const int cur = kt & 1;
        const char* base_a = smem + cur * kStageBytes + fr_a;
        const char* base_b = smem + cur * kStageBytes + fr_b;
#pragma unroll
        for (int i = 0; i < 4; ++i) mgroup(i, 0, 1, true, base_a + koff[1], base_b + koff[1], dma, cur ^ 1, (kt + 1) * kBK, i);
#pragma unroll
        for (int i = 0; i < 4; ++i) mgroup(i, 1, 0, true, base_a + koff[2], base_b + koff[2], dma, cur ^ 1, (kt + 1) * kBK, 4 + i);
#pragma unroll
        for (int i = 0; i < 4; ++i) mgroup(i, 0, 1, true, base_a + koff[3], base_b + koff[3], false, 0, 0, 0);
        // one barrier per tile: publishes tile kt+1 (every wavefront waited for its own loads) and
        // retires stage cur (every wavefront has its last fragments in registers)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        const char* next_a = smem + (cur ^ 1) * kStageBytes + fr_a + koff[0];
        const char* next_b = smem + (cur ^ 1) * kStageBytes + fr_b + koff[0];
#pragma unroll
        for (int i = 0; i < 4; ++i) mgroup(i, 1, 0, more, next_a, next_b, false, 0, 0, 0);
    };
    for (int kt = 0; kt + 1 < nk; ++kt) tile_iter(kt, std::true_type{});
    tile_iter(nk - 1, std::false_type{});

    // ---- epilogue.  For tile (i, j) a lane holds row m = r and columns 8 q + 4 kh + (0..3).
    // Writing that straight to memory would touch 32 different cache lines per store with 8-16
    // bytes each; instead every wavefront parks its 128 x 128 sub-tile in its own LDS region
    // (all main-loop reads are behind the last barrier) and streams it out as 16-byte pieces of
    // whole rows, so a store covers complete cache lines.
    const T* __restrict__ bias = reinterpret_cast<const T*>(p.bias);
    OutT* __restrict__ Y = reinterpret_cast<OutT*>(p.Y);
    constexpr int EPC = 16 / (int)sizeof(OutT);                 // elements per 16-byte piece
    constexpr int ROWB = 128 * (int)sizeof(OutT) + 16;         // padded row of the wave's sub-tile
    constexpr int PASS_I = (sizeof(OutT) == 2) ? 4 : 2;        // 32-row blocks per pass (region = 34816 B)
    constexpr int CPR = 128 / EPC;                             // pieces per row
    constexpr int RPI = 64 / CPR;                              // rows per store instruction
    const bool fast = (a.N % EPC == 0) && (a.ldy % EPC == 0) && (((uintptr_t)p.Y & 15) == 0) &&
                      (p.residual == nullptr || (sizeof(OutT) == 4 && ((uintptr_t)p.residual & 15) == 0));
    if (fast) {
        char* reg = smem + wave * 34816;
#pragma unroll
        for (int pass = 0; pass < 4 / PASS_I; ++pass) {
            if (pass) __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ii = 0; ii < PASS_I; ++ii) {
                const int i = pass * PASS_I + ii;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int col = j * 32 + 8 * q + 4 * kh;
                        const int n = n0 + wn * 128 + col;
                        float bv[4] = {0.f, 0.f, 0.f, 0.f};
                        if (bias && n < a.N) {
                            const Vec<T, 4> b4 = load_vec<T, 4>(bias + n);
#pragma unroll
                            for (int e = 0; e < 4; ++e) bv[e] = Fmt<T>::load(b4.v[e]);
                        }
                        Vec<OutT, 4> ov;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float t = (acc[i][j][4 * q + e] + bv[e]) * p.out_scale;
                            if (a.relu) t = fmaxf(t, 0.f);
                            ov.v[e] = Fmt<OutT>::store(t);
                        }
                        store_vec<OutT, 4>(reinterpret_cast<OutT*>(reg + (ii * 32 + r) * ROWB) + col, ov);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
            const int rr = lane / CPR, ch = lane % CPR;
            const int n = n0 + wn * 128 + ch * EPC;
#pragma unroll 4
            for (int rl = 0; rl < PASS_I * 32; rl += RPI) {
                const int m = m0 + wm * 128 + pass * PASS_I * 32 + rl + rr;
                uint4 v = *reinterpret_cast<const uint4*>(reg + (rl + rr) * ROWB + ch * 16);
                if (m < a.M && n < a.N) {
                    const size_t o = (size_t)m * a.ldy + n;
                    if (sizeof(OutT) == 4 && p.residual) {
                        const float4 rv = *reinterpret_cast<const float4*>(p.residual + o);
                        float4 f = __builtin_bit_cast(float4, v);
                        f.x += rv.x; f.y += rv.y; f.z += rv.z; f.w += rv.w;
                        v = __builtin_bit_cast(uint4, f);
                    }
                    *reinterpret_cast<uint4*>(Y + o) = v;
                }
            }
        }
        return;
    }
    // general path (odd N or leading dimension, or a residual with a 16-bit output)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + wm * 128 + i * 32 + r;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * 128 + j * 32 + 8 * q + 4 * kh;
                const size_t o = (size_t)m * a.ldy + n;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (n + e >= a.N) continue;
                    float t = (acc[i][j][4 * q + e] + (bias ? Fmt<T>::load(bias[n + e]) : 0.f)) * p.out_scale;
                    if (a.relu) t = fmaxf(t, 0.f);
                    if (p.residual) t += p.residual[o + e];
                    Y[o + e] = Fmt<OutT>::store(t);
                }
            }
        }
    }
}

template <typename T, typename OutT>
static zo2_status launch256_t(const GemmArgs& a, hipStream_t st) {
    static bool attr_set = false;
    auto kern = gemm_mfma256_kernel<T, OutT>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) {
            set_op_error("gemm: cannot reserve %d bytes of LDS: %s", kLdsBytes, hipGetErrorString(e));
            return ZO2_EHIP;
        }
        attr_set = true;
    }
    const unsigned tiles = (unsigned)(((a.M + kBM - 1) / kBM) * ((a.N + kBN - 1) / kBN));
    hipLaunchKernelGGL(kern, dim3(tiles, 1, a.nprob), dim3(256), kLdsBytes, st, a);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

zo2_status gemm_launch_256(const GemmArgs& a, int dtype, hipStream_t st) {
    if (dtype == ZO2_BF16) return a.out_f32 ? launch256_t<bf16_t, float>(a, st) : launch256_t<bf16_t, bf16_t>(a, st);
    if (dtype == ZO2_F16) return a.out_f32 ? launch256_t<f16_t, float>(a, st) : launch256_t<f16_t, f16_t>(a, st);
    set_op_error("gemm256: dtype %d unsupported", dtype);
    return ZO2_EINVAL;
}

}  // namespace zo2
