// Projections of the dual forward when a step has few tokens (at most 256 per stream).
//
// With so few rows the projections are bound by reading the weights, not by the matrix cores, and the large-tile
// kernel has a handful of tiles for 256 compute units.  This kernel turns the layout around: a workgroup owns 128 output
// features and a slice of k, streams the stored weights theta through once for BOTH perturbation streams, and forms
// W+ = theta + eps z, W- = theta - eps z in its loader, chunk by chunk in registers (z regenerated from the counters,
// Alg. 2 "perturb"; the same arithmetic and rounding as the sweep kernel, so the same bits) - the two perturbed copies
// of a block are never written to memory nor read back.  The k range is cut into slices so that a launch has a few hundred
// workgroups; the slices' float32 partial sums go to a workspace and a second kernel adds them in slice order
// (deterministic, unlike atomics) and applies bias, scale, ReLU and residual.
#include "gemm_skinny.h"

namespace zo2 {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

template <typename T> struct SkMfma;
template <> struct SkMfma<bf16_t> {
    static __device__ __forceinline__ f32x16_t run(v4u_t a, v4u_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct SkMfma<f16_t> {
    static __device__ __forceinline__ f32x16_t run(v4u_t a, v4u_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    }
};

// Eight consecutive stored elements (one 16-byte chunk starting at element index e, a multiple of 8) -> the same chunk
// of W+ and of W-: one Philox call, four Box-Muller pairs, one fused multiply-add and one rounding per element and sign.
template <typename T>
__device__ __forceinline__ void perturb_chunk(const PhiloxKeys& key, uint32_t tensor_id, uint64_t e, float eps, v4u_t th, v4u_t& wp, v4u_t& wm) {
    Vec<T, 8> t8, p8, m8;
    __builtin_memcpy(&t8, &th, 16);
    float z[8];
    gaussian8(key, tensor_id, e >> 3, z);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = Fmt<T>::load(t8.v[j]);
        p8.v[j] = Fmt<T>::store(__builtin_fmaf(eps, z[j], t));
        m8.v[j] = Fmt<T>::store(__builtin_fmaf(-eps, z[j], t));
    }
    __builtin_memcpy(&wp, &p8, 16);
    __builtin_memcpy(&wm, &m8, 16);
}

static constexpr int kSkBN = 128, kSkBK = 64, kSkKC = 8;      // weight rows per workgroup, k per slab, 16-byte chunks per slab row

// MT: 32-row MFMA tiles per stream (the workgroup covers 32 MT rows of each stream, every wavefront all of them).
//
// A wavefront owns 32 of the workgroup's 128 output features.  The MFMA's weight operand wants, in lane (r, kh), the 8
// consecutive k of feature r starting at 16 ks + 8 kh: exactly one 16-byte chunk of the stored weight and one call of
// the generator, so a lane loads its chunk of theta, perturbs it in registers and feeds both MFMAs from there - the
// weights never pass through LDS and no wavefront waits for another's generation.  Only the activations are shared:
// their slab (2 streams x 32 MT rows x 64 k) is staged in LDS, double-buffered, one barrier per slab.
template <typename T, int MT>
__global__ __launch_bounds__(256, (MT <= 4 ? 2 : 1)) void skinny_dual_kernel(const SkinnyArgs a) {
    constexpr int MP = 32 * MT, CX = MT;                      // rows per stream; X chunks each thread stages per stream and slab
    extern __shared__ __attribute__((aligned(16))) char smem[];
    v4u_t* Xs = reinterpret_cast<v4u_t*>(smem);               // [2 buffers][2 streams][MP rows][8 chunks], chunk index XOR-swizzled

    const SkinnyProblem p = a.p[blockIdx.z];
    const int n0 = blockIdx.x * kSkBN;
    const int k_begin = blockIdx.y * a.k_per_split, k_end = min(a.K, k_begin + a.k_per_split);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, kh = lane >> 5;
    const T* __restrict__ Xp = reinterpret_cast<const T*>(p.Xp);
    const T* __restrict__ Xm = reinterpret_cast<const T*>(p.Xm);
    const T* __restrict__ Th = reinterpret_cast<const T*>(p.theta);

    // staging plan of the activations: chunk c = tid + 256 i of a stream's slab is (row c >> 3, position c & 7); rows past
    // M re-read row M - 1.  Position kc of row m sits at chunk kc ^ ((m >> 1) & 7): sixteen lanes that read one position
    // of sixteen consecutive rows, and eight that write one row, each touch every bank once.
    uint32_t xoff[CX];
    int xl[CX];
#pragma unroll
    for (int i = 0; i < CX; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        xoff[i] = (uint32_t)((size_t)min(row, a.M - 1) * a.ldx + kc * 8);
        xl[i] = row * kSkKC + (kc ^ ((row >> 1) & 7));
    }
    // this lane's weight row (features past N re-read row N - 1; their sums are dropped) and, in elements from the
    // tensor's start, where its first chunk begins: the random stream's counter and the load address in one
    const int n = n0 + wave * 32 + r;
    const uint64_t we = (uint64_t)min(n, a.N - 1) * (uint64_t)a.K + (uint64_t)(kh * 8);

    f32x16_t acc[2][MT];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][i][v] = 0.f;

    v4u_t xr[2][CX], tr[4], tn[4];
    auto load_x = [&](int k0) {
#pragma unroll
        for (int i = 0; i < CX; ++i) {
            xr[0][i] = *reinterpret_cast<const v4u_t*>(Xp + xoff[i] + k0);
            xr[1][i] = *reinterpret_cast<const v4u_t*>(Xm + xoff[i] + k0);
        }
    };
    auto store_x = [&](int buf) {
        v4u_t* Xb = Xs + buf * (2 * MP * kSkKC);
#pragma unroll
        for (int i = 0; i < CX; ++i) {
            Xb[xl[i]] = xr[0][i];
            Xb[MP * kSkKC + xl[i]] = xr[1][i];
        }
    };

    load_x(k_begin);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) tr[ks] = *reinterpret_cast<const v4u_t*>(Th + we + k_begin + 16 * ks);
    store_x(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += kSkBK, buf ^= 1) {
        const bool more = k0 + kSkBK < k_end;
        if (more) {
            load_x(k0 + kSkBK);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) tn[ks] = *reinterpret_cast<const v4u_t*>(Th + we + k0 + kSkBK + 16 * ks);
        }
        const v4u_t* Xb = Xs + buf * (2 * MP * kSkKC);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            v4u_t wp, wm;
            perturb_chunk<T>(a.key, p.tensor_id, we + (uint64_t)(k0 + 16 * ks), a.eps, tr[ks], wp, wm);
            const int kc = ks * 2 + kh;
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const int row = i * 32 + r, at = row * kSkKC + (kc ^ ((row >> 1) & 7));
                acc[0][i] = SkMfma<T>::run(Xb[at], wp, acc[0][i]);
                acc[1][i] = SkMfma<T>::run(Xb[MP * kSkKC + at], wm, acc[1][i]);
            }
        }
        if (more) {
            store_x(buf ^ 1);              // last read before the barrier that ended the previous slab
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) tr[ks] = tn[ks];
        }
        __syncthreads();
    }

    // partial sums of this k slice: lane holds column n of each 32 x 32 tile and rows 8 (v / 4) + 4 kh + v % 4
    if (n >= a.N) return;
    const size_t plane = (size_t)a.M * a.N;
    float* __restrict__ part = a.partial + ((size_t)blockIdx.z * a.splits + blockIdx.y) * 2 * plane;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = i * 32 + 8 * (v >> 2) + 4 * kh + (v & 3);
                if (m < a.M) part[s * plane + (size_t)m * a.N + n] = acc[s][i][v];
            }
}

// Sum of the k slices in slice order, then bias, scale, ReLU, residual; four consecutive columns per thread.
template <typename T, typename OutT>
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const SkinnyArgs a) {
    const int n4 = a.N >> 2;
    const size_t per_stream = (size_t)a.M * n4;
    const size_t gi = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gi >= 2 * per_stream) return;
    const SkinnyProblem p = a.p[blockIdx.y];
    const int s = (int)(gi / per_stream);
    const size_t rem = gi - (size_t)s * per_stream;
    const int m = (int)(rem / n4), n = (int)(rem % n4) * 4;
    const size_t plane = (size_t)a.M * a.N;
    const float* part = a.partial + (size_t)blockIdx.y * a.splits * 2 * plane + (size_t)s * plane + (size_t)m * a.N + n;
    // slice order; the loads of sixteen slices are in flight together (one after the other, a thread would wait out the
    // memory latency once per slice, and so few threads run here that nothing else would hide it)
    v4f_t sum = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < a.splits; k0 += 16) {
        v4f_t t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (k0 + j < a.splits) t[j] = *reinterpret_cast<const v4f_t*>(part + (size_t)(k0 + j) * 2 * plane);
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (k0 + j < a.splits) sum += t[j];
    }
    const T* bias = reinterpret_cast<const T*>(s ? p.bias_m : p.bias_p);
    const float* res = s ? p.res_m : p.res_p;
    OutT* Y = reinterpret_cast<OutT*>(s ? p.Ym : p.Yp);
    const size_t o = (size_t)m * a.ldy + n;
    Vec<OutT, 4> out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float y = (sum[e] + (bias ? Fmt<T>::load(bias[n + e]) : 0.f)) * p.out_scale;
        if (a.relu) y = fmaxf(y, 0.f);
        if (res) y += res[o + e];
        out.v[e] = Fmt<OutT>::store(y);
    }
    store_vec<OutT, 4>(Y + o, out);
}

template <typename T>
__global__ __launch_bounds__(256) void perturbed_rows_kernel(const T* theta, uint64_t e0, uint64_t chunks, uint32_t tensor_id, PhiloxKeys key,
                                                             float eps, T* w_plus, T* w_minus) {
    const uint64_t c = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= chunks) return;
    v4u_t wp, wm;
    perturb_chunk<T>(key, tensor_id, e0 + 8 * c, eps, *reinterpret_cast<const v4u_t*>(theta + 8 * c), wp, wm);
    *reinterpret_cast<v4u_t*>(w_plus + 8 * c) = wp;
    *reinterpret_cast<v4u_t*>(w_minus + 8 * c) = wm;
}

bool skinny_applicable(int M, int N, int K, int dtype) {
    return (dtype == ZO2_BF16 || dtype == ZO2_F16) && M >= 1 && M <= 256 && N >= 1 && N % 4 == 0 && K >= 64 && K % 64 == 0;
}

// How many pieces the k range is cut into: enough workgroups to occupy the chip (about two per compute unit for up to
// 32 rows, one above - measured on d_model 2048 shapes), but never more float32 partial sums than four times the bytes
// of the weights themselves (a piece writes 2 M x 128 sums for the 128 x k_per_split weights it reads).
static void pick_splits(int M, int N, int K, int nprob, int& splits, int& k_per_split) {
    const int n_tiles = (N + kSkBN - 1) / kSkBN, slabs = K / kSkBK;
    int want = (M <= 32 ? 512 : 256) / (n_tiles * nprob);
    const int cap = K / M > 1 ? K / M : 1;
    want = want > cap ? cap : want;
    want = want < 1 ? 1 : (want > slabs ? slabs : want);
    const int slabs_per = (slabs + want - 1) / want;
    k_per_split = slabs_per * kSkBK;
    splits = (slabs + slabs_per - 1) / slabs_per;
}

size_t skinny_workspace_bytes(int M, int N, int K, int nprob) {
    if (M <= 0 || N <= 0 || K < kSkBK || nprob <= 0) return 0;
    int splits, kps;
    pick_splits(M, N, K, nprob, splits, kps);
    return (size_t)nprob * splits * 2 * (size_t)M * N * sizeof(float);
}

template <typename T, int MT>
static zo2_status skinny_launch_mt(const SkinnyArgs& a, hipStream_t st) {
    const dim3 grid((a.N + kSkBN - 1) / kSkBN, a.splits, a.nprob), block(256);
    constexpr int lds = 2 * 2 * 32 * MT * kSkKC * 16;
    static bool reserved_on[kMaxDevices] = {false};
    bool& reserved = reserved_on[current_device()];
    auto kern = skinny_dual_kernel<T, MT>;
    if (!reserved) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) {
            set_op_error("skinny gemm: cannot reserve %d bytes of LDS", lds);
            return ZO2_EHIP;
        }
        reserved = true;
    }
    hipLaunchKernelGGL(kern, grid, block, lds, st, a);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

template <typename T>
static zo2_status skinny_launch_t(const SkinnyArgs& a, hipStream_t st) {
    const dim3 block(256);
    zo2_status s = a.M <= 32 ? skinny_launch_mt<T, 1>(a, st) : a.M <= 64 ? skinny_launch_mt<T, 2>(a, st)
                 : a.M <= 128 ? skinny_launch_mt<T, 4>(a, st) : skinny_launch_mt<T, 8>(a, st);
    if (s != ZO2_OK) return s;
    const size_t work = 2 * (size_t)a.M * (a.N / 4);
    const dim3 rgrid((unsigned)((work + 255) / 256), a.nprob);
    if (a.out_f32) hipLaunchKernelGGL((skinny_reduce_kernel<T, float>), rgrid, block, 0, st, a);
    else hipLaunchKernelGGL((skinny_reduce_kernel<T, T>), rgrid, block, 0, st, a);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

zo2_status skinny_launch(SkinnyArgs& a, int dtype, void* workspace, size_t workspace_bytes, hipStream_t st) {
    ZO2_OP_CHECK(skinny_applicable(a.M, a.N, a.K, dtype), ZO2_EINVAL,
                 "skinny gemm: needs 16-bit dtype, 1 <= M <= 256, N %% 4 == 0, K %% 64 == 0 (got %d x %d x %d)", a.M, a.N, a.K);
    ZO2_OP_CHECK(a.nprob >= 1 && a.nprob <= SkinnyArgs::kMaxProblems, ZO2_EINVAL, "skinny gemm: %d problems", a.nprob);
    ZO2_OP_CHECK(a.ldx >= a.K && a.ldx % 8 == 0 && a.ldy >= a.N && a.ldy % 4 == 0, ZO2_EINVAL, "skinny gemm: bad leading dimension");
    ZO2_OP_CHECK((size_t)a.M * (size_t)a.ldx < 0xffffffffull, ZO2_EINVAL, "skinny gemm: activation panel too large");
    const size_t osz = a.out_f32 ? 4 : 2;
    for (int i = 0; i < a.nprob; ++i) {
        const SkinnyProblem& p = a.p[i];
        ZO2_OP_CHECK(p.Xp && p.Xm && p.theta && p.Yp && p.Ym, ZO2_EINVAL, "skinny gemm: NULL operand in problem %d", i);
        ZO2_OP_CHECK((((uintptr_t)p.Xp | (uintptr_t)p.Xm | (uintptr_t)p.theta) & 15) == 0, ZO2_EINVAL, "skinny gemm: operands must be 16-byte aligned");
        ZO2_OP_CHECK((((uintptr_t)p.Yp | (uintptr_t)p.Ym) & (4 * osz - 1)) == 0, ZO2_EINVAL, "skinny gemm: outputs must be aligned to 4 elements");
        ZO2_OP_CHECK((p.bias_p == nullptr) == (p.bias_m == nullptr) && (p.res_p == nullptr) == (p.res_m == nullptr), ZO2_EINVAL,
                     "skinny gemm: bias / residual must be given for both streams or neither");
        ZO2_OP_CHECK(!p.res_p || a.out_f32, ZO2_EINVAL, "skinny gemm: a residual needs float32 output");
    }
    pick_splits(a.M, a.N, a.K, a.nprob, a.splits, a.k_per_split);
    const size_t need = (size_t)a.nprob * a.splits * 2 * (size_t)a.M * a.N * sizeof(float);
    ZO2_OP_CHECK(workspace && ((uintptr_t)workspace & 15) == 0 && workspace_bytes >= need, ZO2_EINVAL,
                 "skinny gemm: workspace of %zu bytes needed (16-byte aligned)", need);
    a.partial = reinterpret_cast<float*>(workspace);
    if (dtype == ZO2_BF16) return skinny_launch_t<bf16_t>(a, st);
    return skinny_launch_t<f16_t>(a, st);
}

zo2_status skinny_perturbed_rows(int dtype, const void* theta, int64_t K, int64_t n0, int64_t rows, uint32_t tensor_id, uint64_t seed,
                                 float eps, void* w_plus, void* w_minus, hipStream_t st) {
    ZO2_OP_CHECK(dtype == ZO2_BF16 || dtype == ZO2_F16, ZO2_EINVAL, "perturbed_rows: dtype must be BF16 or F16");
    ZO2_OP_CHECK(theta && w_plus && w_minus && K > 0 && K % 8 == 0 && n0 >= 0 && rows >= 0, ZO2_EINVAL, "perturbed_rows: bad argument");
    ZO2_OP_CHECK((((uintptr_t)theta | (uintptr_t)w_plus | (uintptr_t)w_minus) & 15) == 0, ZO2_EINVAL, "perturbed_rows: pointers must be 16-byte aligned");
    const uint64_t chunks = (uint64_t)rows * (uint64_t)K / 8;
    if (chunks == 0) return ZO2_OK;
    const PhiloxKeys key = philox_keys(seed);
    const dim3 grid((unsigned)((chunks + 255) / 256)), block(256);
    if (dtype == ZO2_BF16)
        hipLaunchKernelGGL(perturbed_rows_kernel<bf16_t>, grid, block, 0, st, reinterpret_cast<const bf16_t*>(theta), (uint64_t)n0 * (uint64_t)K, chunks,
                           tensor_id, key, eps, reinterpret_cast<bf16_t*>(w_plus), reinterpret_cast<bf16_t*>(w_minus));
    else
        hipLaunchKernelGGL(perturbed_rows_kernel<f16_t>, grid, block, 0, st, reinterpret_cast<const f16_t*>(theta), (uint64_t)n0 * (uint64_t)K, chunks,
                           tensor_id, key, eps, reinterpret_cast<f16_t*>(w_plus), reinterpret_cast<f16_t*>(w_minus));
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

}  // namespace zo2
