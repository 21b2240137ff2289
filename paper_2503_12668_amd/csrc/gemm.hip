// Projection GEMMs of the dual forward (Alg. 2 "forward"): Y = act((X W^T + b) s) + R.
//
// Both operands are K-contiguous (activations [M, K], weights [N, K]), which is exactly
// the per-lane operand shape of the CDNA MFMA instructions: lane l of a wavefront supplies
// 8 consecutive k of row l % 32.  So tiles go global -> LDS -> registers as 16-byte chunks
// with no transposition; an XOR swizzle of the chunk index keeps the 128-bit LDS accesses
// conflict free.  bf16 / fp16 inputs use v_mfma_f32_32x32x16 (float32 accumulate); the
// float32 mode uses v_mfma_f32_32x32x2_f32 (gemm_f32_mfma_kernel).
//
// The +/- streams (and q, k, v) are independent problems of one shape: they share a launch
// through grid.z so that even the narrow projections fill 256 compute units.
#include <math.h>
#include <string.h>

#include "gemm.h"

namespace zo2 {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
// (native vector types for everything staged in registers: arrays of HIP's struct-based float4 / uint4 are not always
// taken apart into registers by the compiler and then live in scratch memory)
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));

template <typename T> struct Mfma;
template <> struct Mfma<bf16_t> {
    static __device__ __forceinline__ f32x16_t run(v4u_t a, v4u_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<f16_t> {
    static __device__ __forceinline__ f32x16_t run(v4u_t a, v4u_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------------------
// MFMA kernel.  Block tile BM x BN x 64, four wavefronts in a 2 x 2 grid, each owning a
// (BM/2) x (BN/2) tile made of 32 x 32 MFMA tiles.  LDS holds two stages of 16-byte chunks:
// chunk (row, kc) of a tile lives at index row * 8 + (kc ^ (row & 7)).
// ---------------------------------------------------------------------------------------
template <typename T, int BM, int BN, typename OutT>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(const GemmArgs a) {
    constexpr int BK = 64, KC = BK / 8;            // 8 chunks of 8 elements per row
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int CA = BM * KC / 256, CB = BN * KC / 256;   // chunks each thread stages per tile
    __shared__ v4u_t lds[2][(BM + BN) * KC];

    const GemmProblem p = a.p[blockIdx.z];
    const int tiles_n = (a.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tiles_n) * BM, n0 = (blockIdx.x % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, r = lane & 31, kh = lane >> 5;
    const T* __restrict__ X = reinterpret_cast<const T*>(p.X);
    const T* __restrict__ W = reinterpret_cast<const T*>(p.W);

    // per-thread staging plan
    const T* ga[CA];
    const T* gb[CB];
    int la[CA], lb[CB], kca[CA], kcb[CB];
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        const int m = min(m0 + row, a.M - 1);
        ga[i] = X + (size_t)m * a.ldx + kc * 8;
        la[i] = row * KC + (kc ^ (row & 7));
        kca[i] = kc * 8;
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        const int n = min(n0 + row, a.N - 1);
        gb[i] = W + (size_t)n * a.ldw + kc * 8;
        lb[i] = BM * KC + row * KC + (kc ^ (row & 7));
        kcb[i] = kc * 8;
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    v4u_t ra[CA], rb[CB];
    const v4u_t zero4 = v4u_t{0u, 0u, 0u, 0u};
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int i = 0; i < CA; ++i) ra[i] = (k0 + kca[i] < a.K) ? *reinterpret_cast<const v4u_t*>(ga[i] + k0) : zero4;
#pragma unroll
        for (int i = 0; i < CB; ++i) rb[i] = (k0 + kcb[i] < a.K) ? *reinterpret_cast<const v4u_t*>(gb[i] + k0) : zero4;
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) lds[buf][la[i]] = ra[i];
#pragma unroll
        for (int i = 0; i < CB; ++i) lds[buf][lb[i]] = rb[i];
    };

    const int nk = (a.K + BK - 1) / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_tile((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kc = ks * 2 + kh;
            v4u_t fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WM + i * 32 + r;
                fa[i] = lds[cur][row * KC + (kc ^ (row & 7))];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * WN + j * 32 + r;
                fb[j] = lds[cur][BM * KC + row * KC + (kc ^ (row & 7))];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::run(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < nk) store_tile(cur ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds column n = r of each 32 x 32 tile and rows 8 (v/4) + 4 kh + v%4
    const T* __restrict__ bias = reinterpret_cast<const T*>(p.bias);
    OutT* __restrict__ Y = reinterpret_cast<OutT*>(p.Y);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + r;
        if (n >= a.N) continue;
        const float bv = bias ? Fmt<T>::load(bias[n]) : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * kh + (v & 3);
                if (m >= a.M) continue;
                float y = (acc[i][j][v] + bv) * p.out_scale;
                if (a.relu) y = fmaxf(y, 0.f);
                const size_t o = (size_t)m * a.ldy + n;
                if (p.residual) y += p.residual[o];
                Y[o] = Fmt<OutT>::store(y);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// float32 kernel on the matrix cores: v_mfma_f32_32x32x2_f32 (true float32 products, float32 accumulate).
// Block tile 128 x 128 x 32, four wavefronts in a 2 x 2 grid, each owning 64 x 64 = 2 x 2 MFMA tiles; two
// workgroups per compute unit.  LDS layout as in the 16-bit kernel: rows of 8 chunks of 16 bytes (4 floats), chunk
// index XOR-swizzled by (row & 7).
//
// The instruction contracts two k per issue: lanes 0..31 supply k = 0, lanes 32..63 k = 1 of a row.  A dot product does
// not care in which order its k are visited, as long as both operands visit them in the same order; so a lane of half
// h reads one chunk - the four consecutive k = 8 g + 4 h .. + 3 of its row - with a single 128-bit LDS read, and issue t
// of group g contracts k = 8 g + t (lower half) with k = 8 g + 4 + t (upper half).  One LDS read per operand tile feeds
// four MFMAs.  The weight tile is the instruction's first operand, which leaves a lane with one output row m and runs
// of four consecutive columns n: 16-byte stores.
// ---------------------------------------------------------------------------------------
template <bool KTAIL>      // KTAIL: K is not a multiple of 32, the last slab is zero-filled past the end of the rows
__global__ __launch_bounds__(256, 2) void gemm_f32_mfma_kernel(const GemmArgs a) {
    constexpr int BM = 128, BN = 128, BK = 32, KC = BK / 4;       // 8 chunks of 4 floats per row
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int CA = BM * KC / 256, CB = BN * KC / 256;         // chunks each thread stages per tile
    __shared__ v4f_t lds[2][(BM + BN) * KC];

    const GemmProblem p = a.p[blockIdx.z];
    const int tiles_n = (a.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tiles_n) * BM, n0 = (blockIdx.x % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, r = lane & 31, kh = lane >> 5;
    const float* __restrict__ X = reinterpret_cast<const float*>(p.X);
    const float* __restrict__ W = reinterpret_cast<const float*>(p.W);

    const float* ga[CA];
    const float* gb[CB];
    int la[CA], lb[CB], kca[CA], kcb[CB];
#pragma unroll
    for (int i = 0; i < CA; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        ga[i] = X + (size_t)min(m0 + row, a.M - 1) * a.ldx + kc * 4;
        la[i] = row * KC + (kc ^ (row & 7));
        kca[i] = kc * 4;
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        gb[i] = W + (size_t)min(n0 + row, a.N - 1) * a.ldw + kc * 4;
        lb[i] = BM * KC + row * KC + (kc ^ (row & 7));
        kcb[i] = kc * 4;
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    v4f_t ra[CA], rb[CB];
    const v4f_t zero4 = v4f_t{0.f, 0.f, 0.f, 0.f};
    auto load_tile = [&](int k0) {        // K is a multiple of 4: a chunk is inside the row or entirely past its end
#pragma unroll
        for (int i = 0; i < CA; ++i) ra[i] = (!KTAIL || k0 + kca[i] < a.K) ? *reinterpret_cast<const v4f_t*>(ga[i] + k0) : zero4;
#pragma unroll
        for (int i = 0; i < CB; ++i) rb[i] = (!KTAIL || k0 + kcb[i] < a.K) ? *reinterpret_cast<const v4f_t*>(gb[i] + k0) : zero4;
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) lds[buf][la[i]] = ra[i];
#pragma unroll
        for (int i = 0; i < CB; ++i) lds[buf][lb[i]] = rb[i];
    };

    const int nk = (a.K + BK - 1) / BK;
    load_tile(0);
    store_tile(0);
    if (nk > 1) load_tile(BK);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
#pragma unroll
        for (int g = 0; g < BK / 8; ++g) {
            // the other buffer is free for the whole slab (its last readers passed the barrier that ended the previous
            // one): the next slab is parked there half-way through, not at the end, where every wavefront would arrive
            // at the barrier behind a burst of LDS stores; the registers it leaves are reloaded at once with the slab
            // after it, which then has a whole slab's time (4096 cycles of MFMA) to arrive
            if (g == BK / 16 && kt + 1 < nk) {
                store_tile(cur ^ 1);
                if (kt + 2 < nk) load_tile((kt + 2) * BK);
            }
            const int kc = 2 * g + kh;
            v4f_t fx[TM], fw[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WM + i * 32 + r;
                fx[i] = lds[cur][row * KC + (kc ^ (row & 7))];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * WN + j * 32 + r;
                fw[j] = lds[cur][BM * KC + row * KC + (kc ^ (row & 7))];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[j].x, fx[i].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[j].y, fx[i].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[j].z, fx[i].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[j].w, fx[i].w, acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // epilogue: in MFMA tile (i, j) a lane holds output row m = r (the second operand's row) and the columns
    // n = 8 (v / 4) + 4 kh + v % 4 (the first operand's rows): four runs of four consecutive columns
    const float* __restrict__ bias = reinterpret_cast<const float*>(p.bias);
    float* __restrict__ Y = reinterpret_cast<float*>(p.Y);
    const bool vec_ok = (a.N % 4 == 0) && (a.ldy % 4 == 0) && (((uintptr_t)Y & 15) == 0) &&
                        (!p.residual || ((uintptr_t)p.residual & 15) == 0) && (!bias || ((uintptr_t)bias & 15) == 0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WM + i * 32 + r;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + j * 32 + 8 * q + 4 * kh;
                if (n >= a.N) continue;
                const size_t o = (size_t)m * a.ldy + n;
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * q + e];
                if (vec_ok) {                      // N % 4 == 0: the run of four is inside the row or entirely past its end
                    const v4f_t b4 = bias ? *reinterpret_cast<const v4f_t*>(bias + n) : zero4;
                    const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        y[e] = (y[e] + bb[e]) * p.out_scale;
                        if (a.relu) y[e] = fmaxf(y[e], 0.f);
                    }
                    if (p.residual) {
                        const v4f_t r4 = *reinterpret_cast<const v4f_t*>(p.residual + o);
                        y[0] += r4.x; y[1] += r4.y; y[2] += r4.z; y[3] += r4.w;
                    }
                    *reinterpret_cast<v4f_t*>(Y + o) = v4f_t{y[0], y[1], y[2], y[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (n + e >= a.N) continue;
                        float v = (y[e] + (bias ? bias[n + e] : 0.f)) * p.out_scale;
                        if (a.relu) v = fmaxf(v, 0.f);
                        if (p.residual) v += p.residual[o + e];
                        Y[o + e] = v;
                    }
                }
            }
        }
    }
}

template <typename T>
static zo2_status launch_mfma(const GemmArgs& a, hipStream_t st) {
    constexpr int BM = 128, BN = 128;
    const unsigned tiles = (unsigned)(((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN));
    const dim3 grid(tiles, 1, a.nprob), block(256);
    if (a.out_f32) hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, float>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, T>), grid, block, 0, st, a);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

zo2_status gemm_launch(const GemmArgs& a, int dtype, hipStream_t st) {
    ZO2_OP_CHECK(a.M >= 0 && a.N >= 0 && a.K > 0, ZO2_EINVAL, "gemm: bad shape %d x %d x %d", a.M, a.N, a.K);
    if (a.M == 0 || a.N == 0 || a.nprob == 0) return ZO2_OK;
    ZO2_OP_CHECK(a.K % 8 == 0, ZO2_EINVAL, "gemm: K = %d is not a multiple of 8", a.K);
    ZO2_OP_CHECK(a.ldx >= a.K && a.ldw >= a.K && a.ldy >= a.N, ZO2_EINVAL, "gemm: leading dimension too small");
    ZO2_OP_CHECK(a.ldx % 8 == 0 && a.ldw % 8 == 0, ZO2_EINVAL, "gemm: ldx / ldw must be multiples of 8");
    ZO2_OP_CHECK(a.nprob >= 1 && a.nprob <= GemmArgs::kMaxProblems, ZO2_EINVAL, "gemm: %d problems", a.nprob);
    for (int i = 0; i < a.nprob; ++i) {
        ZO2_OP_CHECK(a.p[i].X && a.p[i].W && (a.p[i].Y || a.ce_mode), ZO2_EINVAL, "gemm: NULL operand in problem %d", i);
        ZO2_OP_CHECK(((uintptr_t)a.p[i].X & 15) == 0 && ((uintptr_t)a.p[i].W & 15) == 0, ZO2_EINVAL,
                     "gemm: operands must be 16-byte aligned");
    }
    // cross-entropy mode has no output matrix (Y may be NULL): only the 256 x 256 kernel implements it, so every
    // other path must be refused before anything is launched
    ZO2_OP_CHECK(!a.ce_mode || (dtype != ZO2_F32 && gemm256_applicable(a, dtype)), ZO2_EINVAL,
                 "gemm: cross-entropy mode needs the 256 x 256 kernel (16-bit inputs, K %% 128 == 0, M, N >= 256, N %% 4 == 0)");
    if (dtype == ZO2_F32) {
        ZO2_OP_CHECK(a.out_f32, ZO2_EINVAL, "gemm: the float32 kernel writes float32 output");
        const unsigned tiles = (unsigned)(((a.M + 127) / 128) * ((a.N + 127) / 128));
        if (a.K % 32 == 0) hipLaunchKernelGGL(gemm_f32_mfma_kernel<false>, dim3(tiles, 1, a.nprob), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(gemm_f32_mfma_kernel<true>, dim3(tiles, 1, a.nprob), dim3(256), 0, st, a);
        ZO2_HIP_LAUNCH_CHECK();
        return ZO2_OK;
    }
    if (gemm256_applicable(a, dtype)) return gemm_launch_256(a, dtype, st);
    if (dtype == ZO2_BF16) return launch_mfma<bf16_t>(a, st);
    if (dtype == ZO2_F16) return launch_mfma<f16_t>(a, st);
    set_op_error("gemm: dtype %d is not a compute dtype", dtype);
    return ZO2_EINVAL;
}


// ---------------------------------------------------------------------------------------- split-k
// With few rows per stream a projection has a handful of tiles for 256 compute units (attention output and FC2 of a
// d_model 2048 block at 512 tokens per stream: 64 tiles of 128 rows).  The k range is then cut into 2 or 4 pieces that
// run as problems of their own - the kernels take a list of problems of one shape - and a small second kernel sums a
// problem's pieces in piece order and finishes the values.
template <typename T, typename OutT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs a, const float* __restrict__ part, int splits) {
    const int n4 = a.N >> 2;
    const size_t gi = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gi >= (size_t)a.M * n4) return;
    const GemmProblem p = a.p[blockIdx.y];
    const int m = (int)(gi / n4), n = (int)(gi % n4) * 4;
    const size_t plane = (size_t)a.M * a.N;
    const float* src = part + (size_t)blockIdx.y * splits * plane + (size_t)m * a.N + n;
    v4f_t t[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (k < splits) t[k] = *reinterpret_cast<const v4f_t*>(src + (size_t)k * plane);
    v4f_t sum = t[0];
#pragma unroll
    for (int k = 1; k < 4; ++k)
        if (k < splits) sum += t[k];
    const T* bias = reinterpret_cast<const T*>(p.bias);
    OutT* Y = reinterpret_cast<OutT*>(p.Y);
    const size_t o = (size_t)m * a.ldy + n;
    Vec<OutT, 4> out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float y = (sum[e] + (bias ? Fmt<T>::load(bias[n + e]) : 0.f)) * p.out_scale;
        if (a.relu) y = fmaxf(y, 0.f);
        if (p.residual) y += p.residual[o + e];
        out.v[e] = Fmt<OutT>::store(y);
    }
    store_vec<OutT, 4>(Y + o, out);
}

// Pieces per problem: a small cost model of the large kernel.  A launch of t tiles runs in ceil(t / CUs) rounds; a tile
// costs its k range plus a fixed part (prologue and epilogue, about 256 k), a 128-row tile two thirds of a 256-row one;
// split pieces add the write and the re-read of their float32 partial sums.  One k of a 256 x 256 tile is 26.75 ns at the
// rate the kernel reaches (1.25 PFLOP/s over 256 compute units), the partial sums move at about 4 TB/s.  A split, and a
// further doubling, must win 8 % to be taken (measured launches agree with the model to a few percent).  Splits are
// taken where tiles are few (128 - 1024 tokens per stream at d_model 2048) and where the tile count sits badly on the
// rounds with a long k (FC2 of the OPT-13B shape at 2048 tokens: 320 tiles, 1.25 rounds).
int gemm_pick_splits(int M, int N, int K, int nprob, int dtype) {
    if (!(dtype == ZO2_BF16 || dtype == ZO2_F16) || M <= 0 || N <= 0 || N % 4 != 0 || nprob <= 0) return 1;
    const double cu = (double)device_cu_count();
    const double tn = (double)((N + 255) / 256);
    auto launch_ns = [&](int s) {
        const double kk = (double)K / s + 256.0;
        const double t256 = nprob * s * (double)((M + 255) / 256) * tn, t128 = nprob * s * (double)((M + 127) / 128) * tn;
        double ns = ceil(t128 / cu) * kk * (2.0 / 3.0);
        if (M >= 256) ns = fmin(ns, ceil(t256 / cu) * kk);
        ns *= 26.75;
        if (s > 1) ns += (double)nprob * s * (double)M * (double)N * 8.0 / 4.0e3;      // bytes / (4e12 B/s) in ns
        return ns;
    };
    int best = 1;
    double best_ns = launch_ns(1);
    for (int s = 2; s <= 4; s *= 2) {
        if (K % (s * 128) != 0 || K / s < 512 || nprob * s > GemmArgs::kMaxProblems) break;
        const double ns = launch_ns(s);
        if (ns < 0.92 * best_ns) { best = s; best_ns = ns; }
    }
    return best;
}

size_t gemm_splitk_workspace_bytes(int M, int N, int nprob, int splits) {
    return splits > 1 ? (size_t)nprob * splits * (size_t)M * N * sizeof(float) : 0;
}

template <typename T>
static void launch_splitk_reduce(const GemmArgs& a, const float* part, int splits, hipStream_t st) {
    const size_t work = (size_t)a.M * (a.N / 4);
    const dim3 grid((unsigned)((work + 255) / 256), a.nprob), block(256);
    if (a.out_f32) hipLaunchKernelGGL((splitk_reduce_kernel<T, float>), grid, block, 0, st, a, part, splits);
    else hipLaunchKernelGGL((splitk_reduce_kernel<T, T>), grid, block, 0, st, a, part, splits);
}

zo2_status gemm_launch_splitk(const GemmArgs& a, int dtype, int splits, void* workspace, size_t workspace_bytes, hipStream_t st) {
    if (splits <= 1) return gemm_launch(a, dtype, st);
    ZO2_OP_CHECK(dtype == ZO2_BF16 || dtype == ZO2_F16, ZO2_EINVAL, "gemm split-k: 16-bit compute formats only");
    ZO2_OP_CHECK(!a.ce_mode, ZO2_EINVAL, "gemm split-k: not with the cross-entropy epilogue");
    ZO2_OP_CHECK(splits == 2 || splits == 4, ZO2_EINVAL, "gemm split-k: %d pieces (2 or 4)", splits);
    ZO2_OP_CHECK(a.M > 0 && a.N > 0 && a.N % 4 == 0 && a.ldy % 4 == 0 && a.K % (splits * 8) == 0, ZO2_EINVAL,
                 "gemm split-k: bad shape %d x %d x %d for %d pieces", a.M, a.N, a.K, splits);
    ZO2_OP_CHECK(a.nprob >= 1 && a.nprob * splits <= GemmArgs::kMaxProblems, ZO2_EINVAL, "gemm split-k: %d problems x %d pieces", a.nprob, splits);
    const size_t need = gemm_splitk_workspace_bytes(a.M, a.N, a.nprob, splits);
    ZO2_OP_CHECK(workspace && ((uintptr_t)workspace & 15) == 0 && workspace_bytes >= need, ZO2_EINVAL,
                 "gemm split-k: workspace of %zu bytes needed (16-byte aligned)", need);
    const size_t osz = a.out_f32 ? 4 : 2;
    for (int i = 0; i < a.nprob; ++i) {
        ZO2_OP_CHECK(a.p[i].X && a.p[i].W && a.p[i].Y, ZO2_EINVAL, "gemm split-k: NULL operand in problem %d", i);
        ZO2_OP_CHECK(((uintptr_t)a.p[i].Y & (4 * osz - 1)) == 0 && ((uintptr_t)a.p[i].residual & 15) == 0 && ((uintptr_t)a.p[i].bias & 7) == 0,
                     ZO2_EINVAL, "gemm split-k: output, residual and bias must be aligned to 4 elements");
        ZO2_OP_CHECK(!a.p[i].residual || a.out_f32, ZO2_EINVAL, "gemm split-k: a residual needs float32 output");
    }
    float* part = reinterpret_cast<float*>(workspace);
    const size_t plane = (size_t)a.M * a.N, esz = 2;
    const int kp = a.K / splits;
    GemmArgs e;
    memset(&e, 0, sizeof(e));
    e.M = a.M; e.N = a.N; e.K = kp; e.ldx = a.ldx; e.ldw = a.ldw; e.ldy = a.N; e.relu = 0; e.out_f32 = 1; e.nprob = a.nprob * splits;
    for (int i = 0; i < a.nprob; ++i)
        for (int k = 0; k < splits; ++k) {
            GemmProblem& q = e.p[i * splits + k];
            q.X = reinterpret_cast<const char*>(a.p[i].X) + (size_t)k * kp * esz;
            q.W = reinterpret_cast<const char*>(a.p[i].W) + (size_t)k * kp * esz;
            q.Y = part + ((size_t)i * splits + k) * plane;
            q.out_scale = 1.0f;
        }
    zo2_status s = gemm_launch(e, dtype, st);
    if (s != ZO2_OK) return s;
    if (dtype == ZO2_BF16) launch_splitk_reduce<bf16_t>(a, part, splits, st);
    else launch_splitk_reduce<f16_t>(a, part, splits, st);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

}  // namespace zo2
