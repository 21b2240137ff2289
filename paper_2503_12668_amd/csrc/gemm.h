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
};

struct GemmArgs {
    static constexpr int kMaxProblems = 6;
    int32_t M, N, K;
    int64_t ldx, ldw, ldy;
    int32_t relu;
    int32_t out_f32;        // Y is float32 instead of the compute dtype
    int32_t nprob;          // problems of identical shape, one per grid.z (the +/- streams, q/k/v)
    GemmProblem p[kMaxProblems];
};

// Y = act((X W^T + bias) * out_scale) + residual for every problem; float32 accumulation.
zo2_status gemm_launch(const GemmArgs& a, int dtype, hipStream_t st);
// the 256 x 256 x 64 kernel (bf16 / fp16, K % 64 == 0); gemm_launch picks it for large problems
zo2_status gemm_launch_256(const GemmArgs& a, int dtype, hipStream_t st);
bool gemm256_applicable(const GemmArgs& a, int dtype);

}  // namespace zo2
