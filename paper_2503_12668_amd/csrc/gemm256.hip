// Large-tile MFMA GEMM for the big projections: 256 x 256 x 64 block tile, one workgroup per compute unit,
// v_mfma_f32_16x16x32 with float32 accumulators in the accumulation registers.  Three instances:
//   256-row tiles, eight wavefronts (2 x 4, two per SIMD), each owning 128 x 64 = 8 x 4 MFMA tiles.  While one
//     wavefront of a SIMD issues LDS reads, loads or waits, the other one's MFMAs keep the matrix pipeline busy.
//   256-row tiles, four wavefronts (2 x 2) of 128 x 128: the deeper prefetch below; taken for long k (pick_waves).
//   128-row tiles: four wavefronts (2 x 2) of 64 x 128, for launches that 256-row tiles would spread badly over
//     the compute units.
// (Under this kernel's full load - MFMA, LDS reads, 64 KB per k-slab streaming from L2 - the chip sustains a
// higher clock with the 16 x 16 x 32 shape than with 32 x 32 x 16, although the latter is faster in an MFMA-only loop.)
//
// Data path.  The tile is stored in LDS as rows of 8 chunks of 16 bytes with the chunk index XOR-swizzled by
// (row & 7), two stages of one k-slab each, read with 128-bit LDS reads into MFMA operand registers.  Slabs arrive by
// the direct-to-LDS loads of gfx950 (16 bytes per lane, no staging through vector registers); because such a load
// writes lane i's 16 bytes at LDS offset 16 i, the swizzle is applied on the global side: lane i fetches the chunk
// that belongs at position i.  The first slab of a tile is loaded under the previous tile's epilogue.
//   Eight wavefronts: slab kt + 2 is loaded straight into the stage that the barrier in the middle of slab kt
//     retires, one load per group of four MFMAs (the register budget of two wavefronts per SIMD, 128 + 128, has
//     no room for a slab in flight in registers).
//   Four wavefronts: three k-slabs deep.  Two slabs live in the LDS stages; the third is on its way in vector
//     registers (buffer loads issued two k-steps before the registers are stored to the stage that has just been
//     retired), so that a load has two full k-steps to come back.
//
// Requires K % 128 == 0 (an even number of k-slabs), N % 4 == 0, ldy % 4 == 0 and 16-byte aligned Y / residual (gemm256_applicable);
// M and N are otherwise arbitrary (rows are clamped on load, masked on store).
#include <type_traits>

#include "gemm.h"

namespace zo2 {

// Measurement build (-DZO2_GEMM_STAMPS): one workgroup records the shader clock around the phases of its tiles and sums
// the cycles it spends in the waits in the middle of the slabs (GemmArgs::stamps).  The timer reads are scalar memory
// operations and wait for the wavefront's LDS traffic, so that build runs a few percent slower; the library proper
// compiles all of it away.
#ifdef ZO2_GEMM_STAMPS
#define ZO2_STAMP() do { if (tlog && blockIdx.x == kStampWorkgroup && threadIdx.x == 0 && tcount < 56) tlog[tcount++] = __builtin_amdgcn_s_memtime(); } while (0)
#define ZO2_TIMED(sum, ...) do { const unsigned long long t0_ = __builtin_amdgcn_s_memtime(); __VA_ARGS__; sum += __builtin_amdgcn_s_memtime() - t0_; } while (0)
#else
#define ZO2_STAMP() do { } while (0)
#define ZO2_TIMED(sum, ...) do { __VA_ARGS__; } while (0)
#endif

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// D[16 x 16] += A[16 x 32] B[32 x 16]: lane l supplies row (l & 15), k = 8 (l >> 4) .. + 7 of both operands and
// receives D[4 (l >> 4) + e][l & 15], e = 0..3.  Written as inline assembly with the accumulator tied to an
// accumulation-register tuple ("+a"): left to the register allocator, some of the 64 accumulator tuples end up in
// ordinary vector registers and are copied back and forth on every k-slab.  The compiler does not see an MFMA
// here, so the kernel itself keeps the required distance between the last MFMA and the first read of a result.
template <typename T> struct Mfma16;
template <> struct Mfma16<bf16_t> {
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x4_t& c) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(__builtin_bit_cast(u32x4_t, a)), "v"(__builtin_bit_cast(u32x4_t, b)));
    }
};
// c = 0: one MFMA on zero operands with a literal-zero addend clears a tuple in a quarter of the issue time of four
// register writes (the compiler's own zero-initialisation wrote every accumulation register twice)
__device__ __forceinline__ u32x4_t mfma16_zero_operand() {
    // made where it is used, through a statement the compiler cannot move: as a loop-invariant constant it was hoisted out
    // of the tile loop and, with every register taken in the k loop, spilled to scratch and reloaded per tile
    uint32_t z0 = 0u;
    asm volatile("" : "+v"(z0));
    u32x4_t z = {z0, z0, z0, z0};
    asm volatile("s_nop 4" : "+v"(z));      // wait states between the moves that write z and the first MFMA that reads it
    return z;
}
__device__ __forceinline__ void mfma16_clear(f32x4_t& c, const u32x4_t& z) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %1, 0" : "=a"(c) : "v"(z));
}
template <> struct Mfma16<f16_t> {
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, f32x4_t& c) {
        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(__builtin_bit_cast(u32x4_t, a)), "v"(__builtin_bit_cast(u32x4_t, b)));
    }
};

// Tile: (32 MI) x 256 x 64 with MI = 8 (256 rows; the main shape) or MI = 4 (128 rows: twice as many tiles for
// launches whose 256-row tiles would leave compute units idle or a last round of tiles mostly empty).
static constexpr int kBN = 256, kBK = 64;
static constexpr int kEpiRegion = 24576;                       // per-wave output staging above stage 0
template <int MI> struct Tile256 {
    static constexpr int BM = 32 * MI;
    static constexpr int kStageBytes = (BM + kBN) * kBK * 2;           // 65536 / 49152
    static constexpr int kLdsBytes = kStageBytes + 4 * kEpiRegion;     // 163840 (all 160 KB of a compute unit) / 147456
};

// direct-to-LDS load of 16 bytes per lane: lane i's data lands at lds_base + 16 i
// source address = wave-uniform base (SGPR pair) + per-lane 32-bit byte offset
__device__ __forceinline__ const void* uniform_ptr(const void* p) {   // pin a wave-uniform pointer into scalar registers
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const void*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void load_to_lds(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_base), "v"(voff), "s"(sbase) : "memory");
}

// The same load split into its pieces, for the main loop: the MFMA issued between the write of m0 and the load takes the
// place of the wait state they need.
__device__ __forceinline__ void m0_set(uint32_t lds_base) { asm volatile("s_mov_b32 m0, %0" : : "s"(lds_base) : "memory"); }
// `lanes` (wave-uniform: all ones or zero) is the execution mask of the load: zero turns it into a no-op without a
// branch, so that the compiler sees straight-line code and keeps one register assignment for the accumulators over the
// whole k loop (see Mfma16).  The k loop runs with all 64 lanes active, which is what the mask is restored to.
// (`lanes`: all ones or zero, wave-uniform; both halves of the execution mask are set from it.  It is pinned into a scalar
// register here: left to the register allocator, a mask that lives across the k loop can end up in a vector register when
// scalar registers run short, which this instruction cannot take.)
__device__ __forceinline__ void load_to_lds_masked(const void* sbase, uint32_t voff, uint32_t lds_base, uint32_t lanes) {
    asm volatile("s_mov_b32 m0, %0\n\ts_mov_b32 exec_lo, %3\n\ts_mov_b32 exec_hi, %3\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, -1"
                 : : "s"(lds_base), "v"(voff), "s"(sbase), "s"(__builtin_amdgcn_readfirstlane(lanes)) : "memory");
}
__device__ __forceinline__ void load_to_lds_at_m0_masked(const void* sbase, uint32_t voff, uint64_t lanes) {
    asm volatile("s_mov_b64 exec, %2\n\tglobal_load_lds_dwordx4 %0, %1\n\ts_mov_b64 exec, -1" : : "v"(voff), "s"(sbase), "s"(lanes) : "memory");
}

// Buffer load of 16 bytes per lane: resource (wave-uniform, base = first row of the tile's operand panel) + per-lane 32-bit
// byte offset + wave-uniform byte offset.  An ordinary load as far as the compiler is concerned: it keeps track of the
// registers in flight and places the waits itself.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t panel_rsrc(const void* base, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(bytes > 0x7fffffffull ? 0x7fffffffull : bytes), 0x00020000);
}
__device__ __forceinline__ u32x4_t panel_load(__amdgpu_buffer_rsrc_t rs, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, (int)soff, 0);
}

// The lane index, derived anew from the execution mask (all 64 lanes active) through an operand the compiler cannot
// see through: values computed from it cannot be hoisted out of the loop that contains the call.
__device__ __forceinline__ int fresh_lane_id() {
    uint32_t ones = 0xffffffffu;
    asm volatile("" : "+s"(ones));
    return (int)__builtin_amdgcn_mbcnt_hi(ones, __builtin_amdgcn_mbcnt_lo(ones, 0u));
}

// swizzle of the 16-byte chunk index inside a 128-byte tile row
__device__ __forceinline__ int swz(int row) { return row & 7; }

// Where virtual tile id `vid` (0 .. ntiles * nprob - 1) lives: problem, tile row, tile column.
// Tiles of one problem are walked in groups of 8 rows of the tile grid (column-major inside a
// group) so that workgroups running at the same time share operand panels in L2.
struct TileCoord { int prob, m0, n0; };
template <int BM>
__device__ __forceinline__ TileCoord tile_coord(int vid, int ntiles, int tiles_m, int tiles_n) {
    constexpr int GM = 8;
    TileCoord c;
    c.prob = vid / ntiles;
    const int local = vid - c.prob * ntiles;
    const int group = local / (GM * tiles_n);
    const int gm0 = group * GM;
    const int gsz = min(GM, tiles_m - gm0);
    const int in_group = local - group * GM * tiles_n;
    c.m0 = (gm0 + in_group % gsz) * BM;
    c.n0 = (in_group / gsz) * kBN;
    return c;
}

// Persistent kernel: gridDim.x workgroups (one per compute unit) walk the tile list with stride
// gridDim.x.  Consecutive workgroup ids sit on different XCDs (8 of them, each with its own L2),
// so within a round of gridDim.x tiles XCD x takes a contiguous run of tile ids.
template <typename T, typename OutT, int MI, int NW>
__global__ __launch_bounds__(NW * 64, 1) void gemm_mfma256_kernel(const GemmArgs a, int total_tiles) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int kBM = Tile256<MI>::BM, kStageBytes = Tile256<MI>::kStageBytes;
    constexpr int WPG = 8 / MI;                 // W row-blocks handled per group of eight MFMAs: 1 or 2
    static_assert(NW == 4 || (NW == 8 && MI == 8), "eight wavefronts: 256-row tiles only");
    constexpr int WAVES_N = NW / 2;             // wavefronts side by side along the columns: 2 or 4
    constexpr int NJ = 16 / WAVES_N;            // 16-column MFMA tiles per wavefront: 8 or 4
    constexpr int XA = 4 * MI / NW;             // 8-row X loads per wavefront per slab
    constexpr int WB = 32 / NW;                 // 8-row W loads per wavefront per slab
    constexpr int kEpi = 4 * kEpiRegion / NW;   // output staging per wavefront
    const int tiles_n = (a.N + kBN - 1) / kBN;
    const int tiles_m = (a.M + kBM - 1) / kBM;
    const int ntiles = tiles_m * tiles_n;
    const int G = gridDim.x;
    const int slot = (G % 8 == 0) ? (int)((blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;

    const int tid = threadIdx.x, lane_id = tid & 63, lane = lane_id;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N, r = lane & 15, kg = lane >> 4;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;   // LDS byte address
    // a stage holds the X rows (128 bytes each), then the W rows; a wavefront loads a quarter of each
    const uint32_t ld_a = lds0 + wave * (XA * 1024), ld_b = lds0 + kBM * 128 + wave * (WB * 1024);
    // fragment read plan: row (w*16 MI + i*16 + r) of X, (w*128 + j*16 + r) of W, chunk (4 ks + kg) ^ swz(row); swz(row) = swz(r); two k-steps of 32 per slab
    const uint32_t fr_a = (wm * (16 * MI) + r) * 128, fr_b = kBM * 128 + (wn * (16 * NJ) + r) * 128;
    uint32_t koff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) koff[ks] = (uint32_t)(((ks * 4 + kg) ^ swz(r)) * 16);
    // where this lane's X / W fragments of k-step ks sit in stage st: fixed for the whole kernel, so that the
    // k-slab loop (unrolled by two, one copy per stage) contains no address arithmetic at all
    const char* frag_x[2][2];
    const char* frag_w[2][2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            frag_x[st][ks] = smem + st * kStageBytes + fr_a + koff[ks];
            frag_w[st][ks] = smem + st * kStageBytes + fr_b + koff[ks];
        }
    const int nk = a.K / kBK;

    // loader plan: per stage each wavefront brings 8 MI rows of X and 64 rows of W, 8 rows per
    // instruction; lane -> (row lane/8, position lane%8) and the chunk that belongs there
    // (rows past the end of the matrix are clamped to its last row; their products are never stored)
    uint32_t pa[XA], pb[WB];            // per-lane byte offsets from the tile's first row
    const T* base_x;                    // wave-uniform: first row of the tile in X / W
    const T* base_w;
    __amdgpu_buffer_rsrc_t rs_x, rs_w;  // the same two panels as buffer resources, for the register-staged loads
    // where this lane's 16 bytes of load t go in a stage: the layout the direct-to-LDS loads produce (lane i at 16 i)
    char* wr_a[2];
    char* wr_b[2];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        wr_a[st] = smem + st * kStageBytes + wave * (XA * 1024) + lane * 16;
        wr_b[st] = smem + st * kStageBytes + kBM * 128 + wave * (WB * 1024) + lane * 16;
    }
    auto plan_loads = [&](const TileCoord& tc) {
        const GemmProblem& pp = a.p[tc.prob];
        // (a freshly derived lane index: this arithmetic is redone per tile instead of being kept in registers, or
        // spilled, across the k loop)
        const int lane = fresh_lane_id();
        const int lrow = lane >> 3;
        base_x = reinterpret_cast<const T*>(uniform_ptr(reinterpret_cast<const T*>(pp.X) + (size_t)tc.m0 * a.ldx));
        base_w = reinterpret_cast<const T*>(uniform_ptr(reinterpret_cast<const T*>(pp.W) + (size_t)tc.n0 * a.ldw));
        const int mrem = a.M - 1 - tc.m0, nrem = a.N - 1 - tc.n0;
        rs_x = panel_rsrc(base_x, ((size_t)mrem * a.ldx + a.K) * sizeof(T));        // up to the end of the matrix's last row
        rs_w = panel_rsrc(base_w, ((size_t)nrem * a.ldw + a.K) * sizeof(T));
        const int lkc = (lane & 7) ^ swz(lrow);             // rows of one instruction differ in their low three bits only
#pragma unroll
        for (int t = 0; t < XA; ++t) pa[t] = (uint32_t)((size_t)min(wave * (8 * XA) + t * 8 + lrow, mrem) * a.ldx + lkc * 8) * (uint32_t)sizeof(T);
#pragma unroll
        for (int t = 0; t < WB; ++t) pb[t] = (uint32_t)((size_t)min(wave * (8 * WB) + t * 8 + lrow, nrem) * a.ldw + lkc * 8) * (uint32_t)sizeof(T);
    };
    auto issue_slab = [&](int stage, int k0) {          // one k-slab of the planned tile, all at once
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t < XA) load_to_lds(base_x + k0, pa[t], ld_a + stage * kStageBytes + t * 1024);
            if (t < WB) load_to_lds(base_w + k0, pb[t], ld_b + stage * kStageBytes + t * 1024);
        }
    };
    auto issue_slab0 = [&]() { issue_slab(0, 0); };     // k-slab 0 into stage 0

#ifdef ZO2_GEMM_STAMPS
    unsigned long long* tlog = a.stamps;
    int tcount = 0;
    unsigned long long wait_vm = 0, wait_bar = 0;
#endif
    int vid = slot;
    if (vid >= total_tiles) return;
    TileCoord tc = tile_coord<kBM>(vid, ntiles, tiles_m, tiles_n);
    plan_loads(tc);
    issue_slab0();
    issue_slab(1, kBK);                  // before the first tile both stages are free: its second slab travels with the first
    bool slab1_in_flight = true;

    for (;;) {
        ZO2_STAMP();
        // acc[i][j]: X rows (m) i-th 16-block, W rows (n) j-th 16-block.  The W fragment is the
        // MFMA "A" operand, so a lane ends up with one m (= r) and a run of 4 consecutive n (4 kg ..).
        f32x4_t acc[MI][NJ];
        const u32x4_t zero_operand = mfma16_zero_operand();
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                mfma16_clear(acc[i][j], zero_operand);

        uint4 fa[MI], fb[2][NJ];     // X fragments: one set, each refilled as soon as its group is done; W fragments: two sets
        constexpr bool kStaged = NW == 4;
        u32x4_t sx[kStaged ? XA : 1], sw[kStaged ? WB : 1];      // the slab in flight: this lane's 16 bytes of each of the wavefront's MI + 8 loads
        // One "group" = the NJ MFMAs of X row-block i at k-step buffer `buf`, with the LDS reads that fetch
        // row-block i of X (and the group's share of W) for the next k-step into buffer `nbuf`, and the group's share of
        // the traffic that brings a later k-slab in, dealt out between them.  Every instruction takes an issue slot
        // of its wavefront and only about three fit under one 16-cycle MFMA: scheduling barriers pin one piece of
        // memory work behind each MFMA.
        // stage_out, four wavefronts: the group moves its share of the register-staged slab on: row-block i of X and WPG
        // row-blocks of W are stored to stage `st` (retired by the barrier just passed) and their registers are reloaded
        // with the same pieces of the slab at byte offset `soff` of the panels.
        // stage_out, eight wavefronts: the group issues one of the wavefront's eight direct-to-LDS loads of the slab at k
        // offset `soff` (elements) into stage `st`; `lanes` is all ones, or zero where that slab does not exist.
        auto mgroup = [&](int i, int buf, int nbuf, const char* sa, const char* sb, bool stage_out, int st, uint32_t soff, uint32_t lanes = 0) {
          if constexpr (NW == 8) {
            // four MFMAs per group; group i issues load i of the incoming slab (W rows in groups 0 - 3, X rows in
            // groups 4 - 7: inside a step the weights come from HBM and the activations from the caches, so the weights
            // get the longer flight), even groups read a W fragment of the next k-step, every group reads its own X fragment
            // at its end
            Mfma16<T>::run(fb[buf][0], fa[i], acc[i][0]);
            __builtin_amdgcn_sched_barrier(0);
            if (stage_out) {
                if (i >= 4) load_to_lds_masked(base_x + soff, pa[i & 3], ld_a + st * kStageBytes + (i & 3) * 1024, lanes);
                else load_to_lds_masked(base_w + soff, pb[i & 3], ld_b + st * kStageBytes + (i & 3) * 1024, lanes);
            }
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][1], fa[i], acc[i][1]);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][2], fa[i], acc[i][2]);
            __builtin_amdgcn_sched_barrier(0);
            if ((i & 1) == 0) fb[nbuf][(i >> 1) & 3] = *reinterpret_cast<const uint4*>(sb + ((i >> 1) & 3) * 2048);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][3], fa[i], acc[i][3]);
            __builtin_amdgcn_sched_barrier(0);
            fa[i] = *reinterpret_cast<const uint4*>(sa + i * 2048);
            __builtin_amdgcn_sched_barrier(0);
          } else {
            Mfma16<T>::run(fb[buf][0], fa[i], acc[i][0]);
            __builtin_amdgcn_sched_barrier(0);
            if (stage_out) *reinterpret_cast<u32x4_t*>(wr_a[st] + i * 1024) = sx[i];
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][1], fa[i], acc[i][1]);
            __builtin_amdgcn_sched_barrier(0);
            if (stage_out) sx[i] = panel_load(rs_x, pa[i], soff);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][2], fa[i], acc[i][2]);
            __builtin_amdgcn_sched_barrier(0);
            if (stage_out) *reinterpret_cast<u32x4_t*>(wr_b[st] + (i * WPG) * 1024) = sw[i * WPG];
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][3], fa[i], acc[i][3]);
            __builtin_amdgcn_sched_barrier(0);
            if (stage_out) sw[i * WPG] = panel_load(rs_w, pb[i * WPG], soff);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][4], fa[i], acc[i][4]);
            __builtin_amdgcn_sched_barrier(0);
            fb[nbuf][i * WPG] = *reinterpret_cast<const uint4*>(sb + (i * WPG) * 2048);
            if (WPG == 2 && stage_out) *reinterpret_cast<u32x4_t*>(wr_b[st] + (i * WPG + 1) * 1024) = sw[i * WPG + WPG - 1];
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][5], fa[i], acc[i][5]);
            __builtin_amdgcn_sched_barrier(0);
            if (WPG == 2 && stage_out) sw[i * WPG + WPG - 1] = panel_load(rs_w, pb[i * WPG + WPG - 1], soff);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][6], fa[i], acc[i][6]);
            __builtin_amdgcn_sched_barrier(0);
            if (WPG == 2) fb[nbuf][i * WPG + WPG - 1] = *reinterpret_cast<const uint4*>(sb + (i * WPG + WPG - 1) * 2048);
            __builtin_amdgcn_sched_barrier(0);
            Mfma16<T>::run(fb[buf][7], fa[i], acc[i][7]);
            __builtin_amdgcn_sched_barrier(0);
            fa[i] = *reinterpret_cast<const uint4*>(sa + i * 2048);      // this group's X fragment is free now
            __builtin_amdgcn_sched_barrier(0);
          }
        };

        // k-slab 0 of this tile is in flight into stage 0 (issued before the loop or under the
        // previous tile's epilogue): wait, publish, read the first fragments
        // (as a builtin, not an assembly statement: the compiler's own wait-count bookkeeping must learn that no
        // load of the previous tile's epilogue is outstanding any more, or it protects the first register the k loop
        // overwrites with a vmcnt(0) of its own - which there also waits for the loads issued one k-step earlier)
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0), other counters untouched
        asm volatile("" ::: "memory");
        __syncthreads();
        {
            const char* sa = frag_x[0][0];
            const char* sb = frag_w[0][0];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i < MI) fa[i] = *reinterpret_cast<const uint4*>(sa + i * 2048);
                if (i < NJ) fb[0][i] = *reinterpret_cast<const uint4*>(sb + i * 2048);
            }
        }
        // A slab is two k-steps of 32.  Under k-step 0 the fragments of k-step 1 are read; then one barrier
        // (publishes slab kt+1: every wavefront waited for its own loads or stores to it; retires stage cur: every wavefront
        // has its last fragments in registers); under k-step 1 the first fragments of slab kt+1 are read and the retired
        // stage is refilled.  Eight wavefronts: with the direct-to-LDS loads of slab kt+2, which have until the barrier of
        // the next slab to land (masked off where that slab does not exist: a load landing after the k loop would hit
        // the epilogue's staging or the next tile's first slab).  Four wavefronts: the registers
        // holding slab kt+2 - loaded during k-step 1 of the previous slab - are stored to the retired stage and reloaded
        // with slab kt+3.  Every slab runs the same instructions: where slab kt+3 does not exist the loads fetch the
        // panel's last slab again, and where slab kt+2 does not exist that is also what gets stored (nobody reads it);
        // the fragment reads of a slab kt+1 that does not exist fetch bytes nobody uses.  A separate copy of the loop
        // body for the last slabs would invite the compiler to give the accumulators another register assignment there
        // and to move them between MFMAs that it does not know to be MFMAs.
        // Four wavefronts: the wait in the middle of a slab leaves the MI + 8 register loads in flight; what it does wait
        // for, besides this wavefront's LDS traffic, is older: in a tile's first slab, the direct-to-LDS loads of slab 1.
        const uint32_t last_slab = (uint32_t)(a.K - kBK) * (uint32_t)sizeof(T);
        auto slab_iter = [&](int kt, auto stage_c) {
            constexpr int cur = decltype(stage_c)::value;          // kt & 1
            if constexpr (!kStaged) {
                const uint32_t lanes = __builtin_amdgcn_readfirstlane(kt + 2 < nk ? 0xffffffffu : 0u);
                const uint32_t k2 = (uint32_t)((kt + 2 < nk ? kt + 2 : kt) * kBK);
#pragma unroll
                for (int i = 0; i < MI; ++i) mgroup(i, 0, 1, frag_x[cur][1], frag_w[cur][1], false, 0, 0u);
                ZO2_TIMED(wait_vm, asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"));
                ZO2_TIMED(wait_bar, __syncthreads());
#pragma unroll
                for (int i = 0; i < MI; ++i) mgroup(i, 1, 0, frag_x[cur ^ 1][0], frag_w[cur ^ 1][0], true, cur, k2, lanes);
                return;
            }
            const uint32_t soff = min((uint32_t)((kt + 3) * kBK) * (uint32_t)sizeof(T), last_slab);
#pragma unroll
            for (int i = 0; i < MI; ++i) mgroup(i, 0, 1, frag_x[cur][1], frag_w[cur][1], false, 0, 0u);
            ZO2_TIMED(wait_vm, {
                if constexpr (XA + WB == 16) asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
                else if constexpr (XA + WB == 12) asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
            });
            ZO2_TIMED(wait_bar, __syncthreads());
#pragma unroll
            for (int i = 0; i < MI; ++i) mgroup(i, 1, 0, frag_x[cur ^ 1][0], frag_w[cur ^ 1][0], true, cur, soff);
        };
        ZO2_STAMP();
        // slab 1 of a later tile: stage 1 held the previous tile's epilogue staging and is free once the barrier above is passed
        if (!slab1_in_flight) issue_slab(1, kBK);
        slab1_in_flight = false;
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kStaged) {   // slab 2 (or, if the tile has only two, slab 1 again) starts its trip through the registers
            const uint32_t soff = min((uint32_t)(2 * kBK) * (uint32_t)sizeof(T), last_slab);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (t < XA) sx[t] = panel_load(rs_x, pa[t], soff);
                if (t < WB) sw[t] = panel_load(rs_w, pb[t], soff);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // nk is even (K % 128 == 0): slabs alternate between the two stages, two per trip
        using St0 = std::integral_constant<int, 0>;
        using St1 = std::integral_constant<int, 1>;
        for (int kt = 0; kt < nk; kt += 2) {
            slab_iter(kt, St0{});
            slab_iter(kt + 1, St1{});
        }
        // the last k-step stored a slab nobody reads into stage 1, which the epilogue's output staging overlaps: every
        // wavefront's stores must have landed before any wavefront starts its epilogue
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
        // the last MFMAs' results must have left the pipeline before the epilogue reads them (see Mfma16)
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        ZO2_STAMP();

        // Both stages are free now (all fragment reads are behind the last barrier).  Start the
        // next tile's k-slab 0 into stage 0 so that its latency hides under this tile's epilogue,
        // which stages its output in the LDS above stage 0.
        const GemmProblem p = a.p[tc.prob];
        const int m0 = tc.m0, n0 = tc.n0;
        const int next_vid = vid + G;
        const bool have_next = next_vid < total_tiles;
        if (have_next) {
            tc = tile_coord<kBM>(next_vid, ntiles, tiles_m, tiles_n);
            plan_loads(tc);
            issue_slab0();
        }
        vid = next_vid;

        // ---- epilogue.  For MFMA tile (i, j) a lane holds row m = 16 i + r and columns 16 j + 4 kg + (0..3).
        // Writing that straight to memory would touch 32 different cache lines per store with 8-16
        // bytes each; instead every wavefront parks its sub-tile, 32 rows at a time and still in
        // float32, in its own LDS region and reads it back so that a lane owns 4 consecutive
        // columns of a row: bias, scale, ReLU and residual are applied there (the bias is loaded
        // once per lane) and a store covers complete cache lines.
        const T* __restrict__ bias = reinterpret_cast<const T*>(p.bias);
        OutT* __restrict__ Y = reinterpret_cast<OutT*>(p.Y);
        // the epilogue's many per-lane offsets derive from the lane index; recomputing them per tile (see plan_loads)
        // keeps them out of the k loop's register budget
        const int lane = fresh_lane_id();
        const int r = lane & 15, kg = lane >> 4;
        if constexpr (sizeof(OutT) == 2) {
            // 16-bit output without residual (QKV, FC1): finish the values in registers (the 8 bias
            // vectors a lane needs are fetched together up front), park them in LDS as 16-bit values,
            // two 32-row passes in flight (double-buffered region), and store 16 bytes per lane.
            constexpr int ROWH = NJ * 32 + 16;                     // padded 16-bit row of the wave's sub-tile
            constexpr int PIECES = 2 * NJ, RPI = 64 / PIECES, U16 = 32 / RPI;     // 16-byte pieces per row, rows per store instruction, stores per pass
            char* reg = smem + kStageBytes + wave * kEpi;
            const float lower = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(a.relu ? 0u : 0xff800000u));   // 0 or -inf, in a scalar register
            const float sc = p.out_scale;
            float bvv[NJ][4];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int n = n0 + wn * (16 * NJ) + j * 16 + 4 * kg;
                Vec<T, 4> b4;
#pragma unroll
                for (int e = 0; e < 4; ++e) b4.v[e] = Fmt<T>::store(0.f);
                if (bias && n < a.N) b4 = load_vec<T, 4>(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bvv[j][e] = Fmt<T>::load(b4.v[e]) * sc;      // (acc + b) s = acc s + b s: one FMA per value
            }
            const int rr = lane / PIECES, ch = lane % PIECES;      // RPI rows x PIECES pieces of 8 elements per store
            const int n = n0 + wn * (16 * NJ) + ch * 8;
            const bool n_ok = n < a.N;                             // N % 8 == 0 is required for this path
            const bool interior = (m0 + kBM <= a.M) && (n0 + kBN <= a.N);
#pragma unroll
            for (int i = 0; i < MI / 2; ++i) {
                char* buf = reg + (i & 1) * (32 * ROWH);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)                 // pass i = X row-blocks 2 i and 2 i + 1
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        Vec<OutT, 4> ov;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            ov.v[e] = Fmt<OutT>::store(fmaxf(__builtin_fmaf(acc[2 * i + mb][j][e], sc, bvv[j][e]), lower));
                        store_vec<OutT, 4>(reinterpret_cast<OutT*>(buf + (mb * 16 + r) * ROWH) + j * 16 + 4 * kg, ov);
                    }
                __builtin_amdgcn_wave_barrier();
                uint4 v8[U16];
#pragma unroll
                for (int u = 0; u < U16; ++u) v8[u] = *reinterpret_cast<const uint4*>(buf + (RPI * u + rr) * ROWH + ch * 16);
                const int mf = m0 + wm * (16 * MI) + i * 32 + rr;
                OutT* yp = Y + (size_t)mf * a.ldy + n;
                if (interior) {
#pragma unroll
                    for (int u = 0; u < U16; ++u) *reinterpret_cast<uint4*>(yp + (size_t)(RPI * u) * a.ldy) = v8[u];
                } else {
#pragma unroll
                    for (int u = 0; u < U16; ++u)
                        if (n_ok && mf + RPI * u < a.M) *reinterpret_cast<uint4*>(yp + (size_t)(RPI * u) * a.ldy) = v8[u];
                }
            }
        } else {
        constexpr int ROWB = NJ * 64 + 16;                         // padded float32 row of the wave's sub-tile
        constexpr int CH32 = 4 * NJ, RPI32 = 64 / CH32, U32 = 32 / RPI32;     // float4 pieces per row, rows per store instruction, stores per pass
        {
            char* reg = smem + kStageBytes + wave * kEpi;
            const int rr = lane / CH32, ch = lane % CH32;
            const int n = n0 + wn * (16 * NJ) + ch * 4;
            const bool n_ok = n < a.N;
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (bias && n_ok) {
                const Vec<T, 4> b4 = load_vec<T, 4>(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[e] = Fmt<T>::load(b4.v[e]) * p.out_scale;      // (acc + b) s = acc s + b s
            }
            const float lower = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(a.relu ? 0u : 0xff800000u));   // 0 or -inf, in a scalar register
            const float sc = p.out_scale;
            // interior tiles (the common case) run without any masking; the residual branch is
            // taken once per tile, not per store
            const bool interior = (m0 + kBM <= a.M) && (n0 + kBN <= a.N);
            const size_t row_step = RPI32 * (size_t)a.ldy;
            auto run_passes = [&](auto masked_c, auto res_c) {
                constexpr bool MASKED = decltype(masked_c)::value, RES = decltype(res_c)::value;
#pragma unroll
                for (int i = 0; i < MI / 2; ++i) {
                    if (i) __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)             // pass i = X row-blocks 2 i and 2 i + 1
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const f32x4_t t4 = acc[2 * i + mb][j];
                            *reinterpret_cast<float4*>(reg + (mb * 16 + r) * ROWB + (j * 16 + 4 * kg) * 4) = make_float4(t4[0], t4[1], t4[2], t4[3]);
                        }
                    __builtin_amdgcn_wave_barrier();
                    const int mf = m0 + wm * (16 * MI) + i * 32 + rr;                 // row of u = 0; u adds RPI32 rows
                    const size_t off0 = (size_t)(MASKED ? min(mf, a.M - 1) : mf) * a.ldy + (MASKED && !n_ok ? 0 : n);
                    float4 v4[U32], rv[U32];
#pragma unroll
                    for (int u = 0; u < U32; ++u) v4[u] = *reinterpret_cast<const float4*>(reg + (RPI32 * u + rr) * ROWB + ch * 16);
                    if (RES) {
#pragma unroll
                        for (int u = 0; u < U32; ++u) {
                            // masked rows re-read a valid row (their sums are never stored)
                            const size_t o = MASKED ? (mf + RPI32 * u < a.M ? off0 + u * row_step : off0) : off0 + u * row_step;
                            rv[u] = *reinterpret_cast<const float4*>(p.residual + o);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U32; ++u) {
                        float y0 = fmaxf(__builtin_fmaf(v4[u].x, sc, bv[0]), lower), y1 = fmaxf(__builtin_fmaf(v4[u].y, sc, bv[1]), lower);
                        float y2 = fmaxf(__builtin_fmaf(v4[u].z, sc, bv[2]), lower), y3 = fmaxf(__builtin_fmaf(v4[u].w, sc, bv[3]), lower);
                        if (RES) { y0 += rv[u].x; y1 += rv[u].y; y2 += rv[u].z; y3 += rv[u].w; }
                        {
                            Vec<OutT, 4> ov;
                            ov.v[0] = Fmt<OutT>::store(y0); ov.v[1] = Fmt<OutT>::store(y1);
                            ov.v[2] = Fmt<OutT>::store(y2); ov.v[3] = Fmt<OutT>::store(y3);
                            if (!MASKED || (n_ok && mf + RPI32 * u < a.M)) store_vec<OutT, 4>(Y + off0 + u * row_step, ov);
                        }
                    }
                }
            };
            // Cross-entropy mode (LM head): instead of storing logits, a lane owns one row of the pass and a
            // 64-column span of it, and reduces that span to max and sum(exp(y - max)) in registers: no
            // cross-lane traffic, and the partials of 32 consecutive rows leave as one 128-byte store.
            auto run_ce = [&](auto masked_c) {
                constexpr bool MASKED = decltype(masked_c)::value;
                constexpr float kL2e = 1.4426950408889634f;
                constexpr int SPANC = 8 * NJ, NV = SPANC / 4;         // columns a lane reduces (64 or 32), as float4
                const int crow = lane & 31, chalf = lane >> 5;
                const int ncol0 = n0 + wn * (16 * NJ) + chalf * SPANC;
                // partials are kept per 64-column span: with 32 columns per lane the two halves of the wavefront are merged below
                const size_t span = (size_t)(NW == 4 ? 4 * (n0 / kBN) + 2 * wn + chalf : 4 * (n0 / kBN) + wn) * (size_t)a.part_ld;
#pragma unroll
                for (int i = 0; i < MI / 2; ++i) {
                    if (i) __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)             // pass i = X row-blocks 2 i and 2 i + 1
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const f32x4_t t4 = acc[2 * i + mb][j];
                            *reinterpret_cast<float4*>(reg + (mb * 16 + r) * ROWB + (j * 16 + 4 * kg) * 4) = make_float4(t4[0], t4[1], t4[2], t4[3]);
                        }
                    __builtin_amdgcn_wave_barrier();
                    const int row = m0 + wm * (16 * MI) + i * 32 + crow;
                    const bool row_ok = !MASKED || row < a.M;
                    const char* rp = reg + crow * ROWB + chalf * (SPANC * 4);
                    const int lab = p.labels[MASKED ? min(row, a.M - 1) : row];
                    float4 v4[NV];
#pragma unroll
                    for (int t = 0; t < NV; ++t) v4[t] = *reinterpret_cast<const float4*>(rp + t * 16);
                    const int dl = lab - ncol0;
                    if (row_ok && dl >= 0 && dl < SPANC) p.label_logit[row] = *reinterpret_cast<const float*>(rp + dl * 4) * sc;
                    float mx = -INFINITY;
#pragma unroll
                    for (int t = 0; t < NV; ++t) {
                        v4[t].x *= sc; v4[t].y *= sc; v4[t].z *= sc; v4[t].w *= sc;
                        if (MASKED && ncol0 + 4 * t >= a.N) v4[t] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);   // N % 4 == 0
                        mx = fmaxf(mx, fmaxf(fmaxf(v4[t].x, v4[t].y), fmaxf(v4[t].z, v4[t].w)));
                    }
                    const float mb = mx == -INFINITY ? 0.f : mx;        // a fully masked span sums to 0
                    float s0 = 0.f, s1 = 0.f;
#pragma unroll
                    for (int t = 0; t < NV; ++t) {
                        s0 += __builtin_amdgcn_exp2f((v4[t].x - mb) * kL2e) + __builtin_amdgcn_exp2f((v4[t].y - mb) * kL2e);
                        s1 += __builtin_amdgcn_exp2f((v4[t].z - mb) * kL2e) + __builtin_amdgcn_exp2f((v4[t].w - mb) * kL2e);
                    }
                    float ssum = s0 + s1;
                    if constexpr (NW == 8) {
                        // lanes l and l + 32 hold the two 32-column halves of one row's span
                        const float mxo = __shfl_xor(mx, 32), so = __shfl_xor(ssum, 32);
                        const float mbo = mxo == -INFINITY ? 0.f : mxo;
                        const float mall = fmaxf(mx, mxo), mab = mall == -INFINITY ? 0.f : mall;
                        ssum = ssum * __builtin_amdgcn_exp2f((mb - mab) * kL2e) + so * __builtin_amdgcn_exp2f((mbo - mab) * kL2e);
                        mx = mall;
                    }
                    if (row_ok && (NW == 4 || chalf == 0)) {
                        p.part_max[span + row] = mx;
                        p.part_sum[span + row] = ssum;
                    }
                }
            };
            if (a.ce_mode) {
                if (interior) run_ce(std::false_type{});
                else run_ce(std::true_type{});
            } else if (interior) {
                if (p.residual) run_passes(std::false_type{}, std::true_type{});
                else run_passes(std::false_type{}, std::false_type{});
            } else {
                if (p.residual) run_passes(std::true_type{}, std::true_type{});
                else run_passes(std::true_type{}, std::false_type{});
            }
        }
        }
        ZO2_STAMP();
#ifdef ZO2_GEMM_STAMPS
        if (tlog && blockIdx.x == kStampWorkgroup && threadIdx.x == 0) { tlog[60] = wait_vm; tlog[61] = wait_bar; tlog[62] = (unsigned long long)(tcount / 4); }
#endif
        if (!have_next) break;
        // the epilogue's LDS reads must be done in every wavefront before stage 1 is loaded again;
        // the barrier at the top of the loop (after the wait for slab 0) provides that
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
}

template <typename T, typename OutT, int MI, int NW>
static zo2_status launch256_t(const GemmArgs& a, hipStream_t st) {
    static bool attr_set_on[kMaxDevices] = {false};
    bool& attr_set = attr_set_on[current_device()];
    constexpr int BM = Tile256<MI>::BM, lds = Tile256<MI>::kLdsBytes;
    auto kern = gemm_mfma256_kernel<T, OutT, MI, NW>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) {
            set_op_error("gemm: cannot reserve %d bytes of LDS: %s", lds, hipGetErrorString(e));
            return ZO2_EHIP;
        }
        attr_set = true;
    }
    const int total = ((a.M + BM - 1) / BM) * ((a.N + kBN - 1) / kBN) * a.nprob;
    const int grid = total < device_cu_count() ? total : device_cu_count();
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), lds, st, a, total);
    ZO2_HIP_LAUNCH_CHECK();
    return ZO2_OK;
}

// Rows per tile for a launch.  Workgroups are persistent, one per compute unit, and take whole tiles: with 256-row tiles
// a launch of 128 tiles keeps half of 256 compute units busy, one of 640 tiles leaves the third round half empty.
// A 128-row tile does half the work at a lower rate (same W panel per slab, half the X panel, half the MFMAs per
// fragment read): measured 0.78 - 0.9 of the 256-row rate for K <= 4096 and 0.67 - 0.78 beyond on launches that fill the
// chip either way.  It is chosen when the better filling of the rounds outweighs that.
static int g_forced_tile_rows = 0;      // 0: per launch; 128 / 256: every launch (tests and measurements, see gemm256_force_tile_rows)
void gemm256_force_tile_rows(int rows) { g_forced_tile_rows = rows; }
static int pick_tile_rows(const GemmArgs& a) {
    if (g_forced_tile_rows == 128 || g_forced_tile_rows == 256) return g_forced_tile_rows;
    if (a.M <= 128) return 128;
    const long cu = device_cu_count();
    const long tn = (a.N + kBN - 1) / kBN;
    auto filling = [&](long rows) {        // useful tile rows over the tile rows the rounds have room for
        const long t = ((a.M + rows - 1) / rows) * tn * a.nprob, rounds = (t + cu - 1) / cu;
        return (double)a.M * tn * a.nprob / (double)(rounds * cu * rows);
    };
    const double small_tile_rate = a.K > 4096 ? 0.72 : 0.78;
    return filling(128) * small_tile_rate > filling(256) ? 128 : 256;
}

// Wavefronts per workgroup for a launch of 256-row tiles.  Eight wavefronts keep the matrix pipeline busier (two per
// SIMD) but can only prefetch one k-slab ahead; four wavefronts hold a further slab in registers.  Measured inside the
// benchmark step, same box: eight are 3 - 4 % faster at K = 2048 (QKV, FC1, LM head), four are 4 % faster at K = 8192
// (FC2), where a panel's rows lie 16 KB apart and a slab takes longer to arrive from HBM.
static int g_forced_waves = 0;          // 0: per launch; 4 / 8: every launch of 256-row tiles (tests and measurements)
void gemm256_force_waves(int waves) { g_forced_waves = waves; }
// With at most 2048 rows per problem a launch leans on reading its weights, and four are ahead again or level (whole
// steps at 1024 - 2048 tokens per stream, OPT-1.3B / 6.7B / 13B shapes: 0 - 1.5 %).
static constexpr int kLongK = 6144, kFewRows = 2048;
static int pick_waves(const GemmArgs& a) {
    if (g_forced_waves == 4 || g_forced_waves == 8) return g_forced_waves;
    return (a.K >= kLongK || a.M <= kFewRows) ? 4 : 8;
}

bool gemm256_applicable(const GemmArgs& a, int dtype) {
    if (!(dtype == ZO2_BF16 || dtype == ZO2_F16)) return false;
    // any number of rows: rows past M are clamped on load and masked on store, and a launch of fewer than 256 rows takes
    // the 128-row tile (few rows make a launch bound by reading W, which this kernel's loader does far better than the
    // small-shape kernel)
    if (a.K % 128 != 0 || a.M < 1 || a.N < 256 || a.N % 4 != 0 || a.ldy % 4 != 0) return false;
    if (!a.out_f32 && (a.N % 8 != 0 || a.ldy % 8 != 0)) return false;
    if (a.ce_mode && !a.out_f32) return false;
    const size_t tsz = 2;
    for (int i = 0; i < a.nprob; ++i) {
        if (a.ce_mode) {
            if (!a.p[i].labels || !a.p[i].part_max || !a.p[i].part_sum || !a.p[i].label_logit || a.p[i].residual || a.p[i].bias ||
                a.relu || a.part_ld < a.M)
                return false;
            continue;
        }
        if (((uintptr_t)a.p[i].Y & 15) != 0) return false;
        if (a.p[i].residual && (((uintptr_t)a.p[i].residual & 15) != 0 || !a.out_f32)) return false;
        if (a.p[i].bias && ((uintptr_t)a.p[i].bias & (4 * tsz - 1)) != 0) return false;
    }
    return true;
}

zo2_status gemm_launch_256(const GemmArgs& a, int dtype, hipStream_t st) {
    if (!gemm256_applicable(a, dtype)) {
        set_op_error("gemm256: shape or alignment not supported by the 256 x 256 kernel");
        return ZO2_EINVAL;
    }
    const bool small = pick_tile_rows(a) == 128;
    const bool eight = !small && pick_waves(a) == 8;
    if (dtype == ZO2_BF16) {
        if (small) return a.out_f32 ? launch256_t<bf16_t, float, 4, 4>(a, st) : launch256_t<bf16_t, bf16_t, 4, 4>(a, st);
        if (eight) return a.out_f32 ? launch256_t<bf16_t, float, 8, 8>(a, st) : launch256_t<bf16_t, bf16_t, 8, 8>(a, st);
        return a.out_f32 ? launch256_t<bf16_t, float, 8, 4>(a, st) : launch256_t<bf16_t, bf16_t, 8, 4>(a, st);
    }
    if (dtype == ZO2_F16) {
        if (small) return a.out_f32 ? launch256_t<f16_t, float, 4, 4>(a, st) : launch256_t<f16_t, f16_t, 4, 4>(a, st);
        if (eight) return a.out_f32 ? launch256_t<f16_t, float, 8, 8>(a, st) : launch256_t<f16_t, f16_t, 8, 8>(a, st);
        return a.out_f32 ? launch256_t<f16_t, float, 8, 4>(a, st) : launch256_t<f16_t, f16_t, 8, 4>(a, st);
    }
    set_op_error("gemm256: dtype %d unsupported", dtype);
    return ZO2_EINVAL;
}

}  // namespace zo2
