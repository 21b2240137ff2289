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

// ---------------------------------------------------------------------------------------
// MFMA kernel (bf16 / fp16, d_head 64, 80 or 128).  One wavefront owns 32 queries and walks the
// keys in tiles of 32 staged through LDS.
//
//   S^T = K Q^T   (32 keys x 32 queries)   A operand: K rows, B operand: Q rows
//   O^T += V^T P^T (d_head x 32 queries)   A operand: V^T rows, read out of the key-major V
//                                           tile with the transposing LDS read,
//                                           B operand: P^T taken directly from the S^T
//                                           accumulator registers.
// In the 32x32 accumulator layout a lane holds one query column and 16 key rows
// rho = 8 (v/4) + 4 kh + v%4.  As a B operand of the second product a lane must supply 8
// consecutive contraction slots 8 kh .. 8 kh + 7 per 16-slot step.  Both fit together if
// accumulator row rho carries key pi(rho), pi swapping the bits "kh" and "v/4 & 1" inside each
// 16-block: then registers v = 8 s .. 8 s + 7 are keys 16 s + 8 kh .. + 7, the same run of keys
// a lane holds of its V^T row.  pi is applied for free when choosing which K row a lane loads.
// ---------------------------------------------------------------------------------------
typedef __bf16 att_bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 att_f16x8 __attribute__((ext_vector_type(8)));
typedef float att_f32x16 __attribute__((ext_vector_type(16)));
typedef short att_i16x4 __attribute__((ext_vector_type(4)));

template <typename T> struct AttMfma;
template <> struct AttMfma<bf16_t> {
    static __device__ __forceinline__ att_f32x16 run(uint4 a, uint4 b, att_f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(att_bf16x8, a), __builtin_bit_cast(att_bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct AttMfma<f16_t> {
    static __device__ __forceinline__ att_f32x16 run(uint4 a, uint4 b, att_f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(att_f16x8, a), __builtin_bit_cast(att_f16x8, b), c, 0, 0, 0);
    }
};

// direct-to-LDS load of 16 bytes per lane (lane i lands at lds_base + 16 i)
__device__ __forceinline__ void att_load_to_lds(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory");
}

// One workgroup = 128 queries of one (sequence, head); wavefront w owns queries 32 w .. 32 w + 31.
// Key tiles of 32 keys are brought into LDS once per workgroup (direct-to-LDS loads, two buffers,
// one barrier per tile) and shared by the four wavefronts; a wavefront skips the tiles past its
// diagonal.  K and V tiles: 32 rows of d_head elements, 16-byte chunks XOR-swizzled by (row & 7).
// The transposing 8-byte LDS read works on groups of 16 lanes: lane 4 j + g of a group supplies the
// address of 4 consecutive elements, and lane 4 g + c receives element c of lanes g, 4 + g, 8 + g, 12 + g.
// Pointing lane 4 j + g at V[key0 + j][m0 + 4 g ..] therefore hands lane i the keys key0 .. key0 + 3 of
// column m0 + i: four consecutive contraction slots of its V^T row.
template <typename T, int DH>
__global__ __launch_bounds__(256, 2) void attention_mfma_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                                                 T* __restrict__ out, int seq, int64_t ld, int n_heads, int n_pairs) {
    constexpr int KS = DH / 16;          // contraction steps of the first product
    constexpr int DT = (DH + 31) / 32;   // 32-row tiles of O^T (rows past DH are computed on padding and dropped)
    constexpr int DHP = DH <= 64 ? 64 : 128;   // LDS row pitch in elements: a power of two, so that the swizzle stays inside the row
    constexpr int KCH = DHP / 8;         // 16-byte chunk positions per LDS row
    constexpr int GCH = DH / 8;          // 16-byte chunks per row in memory
    constexpr int KTILE = 32 * DHP * 2, BUF = 2 * KTILE;                  // K tile, then V tile
    constexpr int KINSTR = KTILE / 1024 / 4;                              // direct-to-LDS loads per wavefront per tile and operand
    constexpr int NBUF = 4;                                               // ring of K / V tiles: loads run NBUF - 1 tiles ahead of the MFMAs
    __shared__ __attribute__((aligned(1024))) char lds[NBUF * BUF];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, kh = lane >> 5;
    // Workgroup id -> (block of 128 queries, head, sequence).  The query blocks of one (sequence, head) read the same
    // keys and values; consecutive workgroup ids go to different XCDs, each with its own L2, so those blocks get ids that
    // are congruent mod 8 and adjacent in their XCD's order.  Late query blocks (more keys under the causal mask) first.
    const int nqb = (seq + 127) >> 7;
    const int slot = blockIdx.x >> 3;
    const int qb = nqb - 1 - slot % nqb;
    const int pair = (slot / nqb) * 8 + (int)(blockIdx.x & 7);
    if (pair >= n_pairs) return;                             // padding of the last group of 8 (whole workgroup)
    const int head = pair % n_heads, sq = pair / n_heads;
    const int q0 = qb * 128 + wave * 32;
    const bool active = q0 < seq;                            // inactive wavefronts still load and synchronise
    const size_t base = (size_t)sq * seq * ld + (size_t)head * DH;
    const int qi = q0 + r;                                   // this lane's query
    const int qrow = min(qi, seq - 1);
    // key carried by accumulator row rho: swap bits 2 (kh of rho) and 3 inside each 16-block
    const int pr = (r & 0x13) | ((r & 4) << 1) | ((r & 8) >> 1);

    uint4 qf[KS];
#pragma unroll
    for (int c = 0; c < KS; ++c) qf[c] = *reinterpret_cast<const uint4*>(q + base + (size_t)qrow * ld + c * 16 + kh * 8);

    att_f32x16 o[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[d][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    constexpr float kLog2e = 1.4426950408889634f;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int wg_last_q = min(qb * 128 + 127, seq - 1);
    const int wg_last_tile = wg_last_q >> 5;
    const int my_last_tile = q0 >> 5;
    // transposing read: lane = 16 g16 + a; the group covers columns 16 (g16 & 1) .. + 15 and keys 8 (g16 >> 1) + 4 h + (a >> 2)
    const int g16 = lane >> 4, a16 = lane & 15;

    auto issue_tile = [&](int tile, int buf) {
        const int j0 = tile * 32;
#pragma unroll
        for (int x = 0; x < KINSTR; ++x) {                   // K rows: 1024 / (2 DH) rows per instruction
            const int inst = wave * KINSTR + x;
            const int row = inst * (512 / DHP) + lane / KCH;
            int chunk = (lane % KCH) ^ (row & 7);
            if (GCH < KCH && chunk >= GCH) chunk &= 7;       // padding positions of a row repeat a real chunk (finite, never used in a kept result)
            const size_t g = base + (size_t)min(j0 + row, seq - 1) * ld + chunk * 8;   // rows past the end repeat the last one (masked keys)
            att_load_to_lds(k + g, lds0 + buf * BUF + inst * 1024);
            att_load_to_lds(v + g, lds0 + buf * BUF + KTILE + inst * 1024);
        }
    };
    auto process_tile = [&](int tile, int buf) {
        const int j0 = tile * 32;
        const char* kb = lds + buf * BUF;
        const char* vb = kb + KTILE;
        uint4 kf[KS], vf[DT][2];
#pragma unroll
        for (int c = 0; c < KS; ++c) kf[c] = *reinterpret_cast<const uint4*>(kb + pr * (DHP * 2) + (((2 * c + kh) ^ (pr & 7)) * 16));
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                att_i16x4 half[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int key = 16 * s2 + 8 * (g16 >> 1) + 4 * h + (a16 >> 2);
                    const int chunk = 4 * d + 2 * (g16 & 1) + ((a16 & 3) >> 1);
                    const char* src = vb + key * (DHP * 2) + ((chunk ^ (key & 7)) * 16) + 8 * (a16 & 1);
                    half[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) att_i16x4*)src);
                }
                vf[d][s2] = make_uint4(__builtin_bit_cast(uint2, half[0]).x, __builtin_bit_cast(uint2, half[0]).y,
                                       __builtin_bit_cast(uint2, half[1]).x, __builtin_bit_cast(uint2, half[1]).y);
            }
        // ---- S^T = K Q^T
        att_f32x16 st;
#pragma unroll
        for (int v = 0; v < 16; ++v) st[v] = 0.f;
#pragma unroll
        for (int c = 0; c < KS; ++c) st = AttMfma<T>::run(kf[c], qf[c], st);
        // ---- mask (only the diagonal tile has hidden keys; the branch is wave-uniform) and online softmax
        if (tile == my_last_tile) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                // accumulator row rho = 8 (v/4) + 4 kh + v%4 carries key j0 + pi(rho) = j0 + 16 (v/8) + 8 kh + v%8
                const int key = j0 + 16 * (v >> 3) + 8 * kh + (v & 7);
                if (key > qi) st[v] = -INFINITY;
            }
        }
        float tmax = st[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, st[v]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);              // finite: key j0 <= q0 <= qi is always visible in tile 0
        const float m2 = m_new * kLog2e;
        float psum = 0.f;
        float p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[v], kLog2e, -m2));      // exp(st - m_new)
            psum += p[v];
        }
        // the running maximum of a query rarely moves after its first tiles: the accumulators are rescaled only when it
        // moved for some query of this wavefront
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
            const float resc = __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e);
            l_run *= resc;
#pragma unroll
            for (int d = 0; d < DT; ++d)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[d][v] *= resc;
            m_run = m_new;
        }
        l_run += psum;
        // ---- O^T += V^T P^T
        uint4 pf[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            Vec<T, 8> pv;
#pragma unroll
            for (int e = 0; e < 8; ++e) pv.v[e] = Fmt<T>::store(p[8 * s2 + e]);
            pf[s2] = __builtin_bit_cast(uint4, pv);
        }
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) o[d] = AttMfma<T>::run(vf[d][s2], pf[s2], o[d]);
    };

    // A tile is 8 - 16 KB and its MFMAs take a few hundred cycles, far less than a trip to memory: with one tile in
    // flight every iteration waited out the full latency.  NBUF - 1 tiles are kept in flight instead; direct-to-LDS loads
    // complete in issue order, so "all but the loads of the `ahead` younger tiles" is an exact wait for this tile.
#pragma unroll
    for (int t = 0; t < NBUF - 1; ++t)
        if (t <= wg_last_tile) issue_tile(t, t);
    // (the Q fragments were requested before the tiles; consuming them here puts the compiler's wait for them in front
    // of the loop instead of inside it, where it would also wait for every tile in flight)
#pragma unroll
    for (int c = 0; c < KS; ++c) asm volatile("" : : "v"(qf[c].x), "v"(qf[c].y), "v"(qf[c].z), "v"(qf[c].w));
    for (int tile = 0; tile <= wg_last_tile; ++tile) {
        const int ahead = min(NBUF - 2, wg_last_tile - tile);        // younger tiles already issued
        // own loads of this tile landed; own reads of the buffer that is refilled below are done
        if (ahead >= 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(2 * 2 * KINSTR) : "memory");
        else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(2 * KINSTR) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        if (tile + NBUF - 1 <= wg_last_tile) issue_tile(tile + NBUF - 1, (tile + NBUF - 1) % NBUF);   // into the buffer of tile - 1
        if (active && tile <= my_last_tile) process_tile(tile, tile % NBUF);
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (active && qi < seq) {
        T* op = out + base + (size_t)qi * ld;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (d * 32 + 8 * g >= DH) continue;          // rows of the last O^T tile that lie past d_head
                Vec<T, 4> ov;
#pragma unroll
                for (int e = 0; e < 4; ++e) ov.v[e] = Fmt<T>::store(o[d][4 * g + e] * inv);
                store_vec<T, 4>(op + d * 32 + 8 * g + 4 * kh, ov);
            }
    }
}

template <typename T>
static zo2_status launch_mfma_att(const T* q, const T* k, const T* v, T* out, int n_seq, int seq, int n_heads, int d_head,
                                  int64_t ld, hipStream_t st) {
    const int n_pairs = n_heads * n_seq, nqb = (seq + 127) / 128;
    const dim3 grid((unsigned)(8 * nqb) * (unsigned)((n_pairs + 7) / 8)), block(256);
    if (d_head == 64) hipLaunchKernelGGL((attention_mfma_kernel<T, 64>), grid, block, 0, st, q, k, v, out, seq, ld, n_heads, n_pairs);
    else if (d_head == 80) hipLaunchKernelGGL((attention_mfma_kernel<T, 80>), grid, block, 0, st, q, k, v, out, seq, ld, n_heads, n_pairs);
    else hipLaunchKernelGGL((attention_mfma_kernel<T, 128>), grid, block, 0, st, q, k, v, out, seq, ld, n_heads, n_pairs);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

template <typename T>
static zo2_status launch_valu(const T* q, const T* k, const T* v, T* out, int n_seq, int seq, int n_heads, int d_head,
                              int64_t ld, hipStream_t st) {
    const dim3 grid((seq + 63) / 64, n_heads, n_seq), block(64);
    switch (d_head) {
#define ZO2_ATT_CASE(D) \
    case D: hipLaunchKernelGGL((attention_valu_kernel<T, D>), grid, block, 0, st, q, k, v, out, seq, ld); break;
        ZO2_ATT_CASE(8) ZO2_ATT_CASE(16) ZO2_ATT_CASE(32) ZO2_ATT_CASE(64) ZO2_ATT_CASE(80) ZO2_ATT_CASE(128)
#undef ZO2_ATT_CASE
        default:
            set_op_error("attention: d_head %d not supported (8, 16, 32, 64, 80, 128)", d_head);
            return ZO2_EINVAL;
    }
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

zo2_status attention_launch(int dtype, const void* q, const void* k, const void* v, void* out, int n_seq, int seq, int n_heads,
                            int d_head, int64_t ld, int vector_kernel, hipStream_t st) {
    if (n_seq == 0 || seq == 0) return ZO2_OK;
    ZO2_OP_CHECK(n_seq > 0 && seq > 0 && n_heads > 0 && d_head > 0, ZO2_EINVAL, "attention: bad shape");
    ZO2_OP_CHECK(q && k && v && out, ZO2_EINVAL, "attention: NULL buffer");
    ZO2_OP_CHECK(ld >= (int64_t)n_heads * d_head && ld % 8 == 0, ZO2_EINVAL, "attention: bad leading dimension");
    ZO2_OP_CHECK(n_seq <= 65535 && n_heads <= 65535 && (int64_t)n_seq * n_heads * ((seq + 127) / 128 + 1) < (int64_t)1 << 30, ZO2_EINVAL,
                 "attention: grid too large");
    {   // every kernel moves groups of 8 elements
        const uintptr_t align = 8 * (uintptr_t)zo2_dtype_size(dtype);
        ZO2_OP_CHECK(align != 0 && ((uintptr_t)q % align) == 0 && ((uintptr_t)k % align) == 0 && ((uintptr_t)v % align) == 0 &&
                     ((uintptr_t)out % align) == 0, ZO2_EINVAL, "attention: unknown dtype, or operands not aligned to 8 elements");
    }
    if (!vector_kernel && dtype != ZO2_F32 && (d_head == 64 || d_head == 80 || d_head == 128)) {
        if (dtype == ZO2_BF16)
            return launch_mfma_att<bf16_t>((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)out, n_seq, seq, n_heads, d_head, ld, st);
        return launch_mfma_att<f16_t>((const f16_t*)q, (const f16_t*)k, (const f16_t*)v, (f16_t*)out, n_seq, seq, n_heads, d_head, ld, st);
    }
    ZO2_DISPATCH_COMPUTE(dtype, T, {
        return launch_valu<T>((const T*)q, (const T*)k, (const T*)v, (T*)out, n_seq, seq, n_heads, d_head, ld, st);
    });
    return ZO2_OK;
}

}  // namespace zo2
