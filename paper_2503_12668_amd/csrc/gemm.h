// Launch interface of the projection GEMMs (QKV, attention output, FFN, LM head).
#pragma once
#include "common.h"

namespace zo2 {

struct GemmProblem {
    const void* X;          // [M, ldx] activations (compute dtype)
    const void* W;          // [N, ldw] weights, row n = output feature n
    const void* bias;       // [N] or nullptr
    const float* residual;  // [M, ldy] float32 or nullptr
    void* Y;                // [M, ldy] compute dtype or float32
    float out_scale;        // multiplies (acc + bias); 1/sqrt(d_head) for the query projection
    int32_t pad_;
    // cross-entropy mode (GemmArgs::ce_mode): nothing is stored to Y; per row and per 64-column span the
    // kernel writes max and sum(exp(y - max)), and the logit of the row's label.  The partial arrays are
    // span-major: span s of row m sits at [s * part_ld + m], s < 4 * ceil(N / 256).  No bias, relu, residual.
    const int32_t* labels;  // [M] device, -100 = ignored (partials are still written)
    float* part_max;        // [4 * ceil(N / 256), part_ld]
    float* part_sum;        // [4 * ceil(N / 256), part_ld]
    float* label_logit;     // [M]
};

struct GemmArgs {
    static constexpr int kMaxProblems = 12;      // q/k/v x two streams x two k pieces
    int32_t M, N, K;
    int64_t ldx, ldw, ldy;
    int64_t part_ld;        // cross-entropy mode: elements between consecutive spans of the partial arrays (>= M)
    int32_t relu;
    int32_t out_f32;        // Y is float32 instead of the compute dtype
    int32_t ce_mode;        // 1: LM-head + cross-entropy partials instead of an output matrix (256 x 256 kernel only)
    int32_t nprob;          // problems of identical shape, one per grid.z (the +/- streams, q/k/v)
    // Cycle stamps of one workgroup, for the measurement build of the 256 x 256 kernel only (-DZO2_GEMM_STAMPS: build.py
    // --gemm-stamps); NULL otherwise.  64 device words: s_memtime at the start of each tile, after the wait for its first
    // slab, after its k loop and after its epilogue (4 per tile, up to 14 tiles), then [60] cycles spent in the waits for
    // loads and [61] at the barriers in the middle of the slabs, [62] the number of tiles.
    unsigned long long* stamps;
    GemmProblem p[kMaxProblems];
};
static constexpr int kStampWorkgroup = 37;      // the workgroup that writes them

// Y = act((X W^T + bias) * out_scale) + residual for every problem; float32 accumulation.
zo2_status gemm_launch(const GemmArgs& a, int dtype, hipStream_t st);
// the 256 x 256 x 64 kernel (bf16 / fp16, K % 128 == 0); gemm_launch picks it for large problems
zo2_status gemm_launch_256(const GemmArgs& a, int dtype, hipStream_t st);
// Split-k for launches that leave most compute units idle (few rows per stream): each problem is cut into `splits` pieces
// of K / splits along k, the pieces run as problems of their own into float32 partial sums
// ([nprob][splits][M][N] in `workspace`), and a second kernel adds a problem's pieces in order (deterministic) and applies
// bias, scale, ReLU and residual.  gemm_pick_splits: 1 (do not split), 2 or 4 for a launch of `nprob` problems.
int gemm_pick_splits(int M, int N, int K, int nprob, int dtype);
size_t gemm_splitk_workspace_bytes(int M, int N, int nprob, int splits);
zo2_status gemm_launch_splitk(const GemmArgs& a, int dtype, int splits, void* workspace, size_t workspace_bytes, hipStream_t st);
// 0 (default): the 256 x 256 kernel picks 256- or 128-row tiles per launch; 128 / 256: every launch uses that height
void gemm256_force_tile_rows(int rows);
void gemm256_force_waves(int waves);      // 0: chosen per launch; 4 or 8: every launch of 256-row tiles
bool gemm256_applicable(const GemmArgs& a, int dtype);

}  // namespace zo2
