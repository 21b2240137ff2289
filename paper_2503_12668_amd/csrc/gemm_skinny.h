// Launch interface of the projection for few tokens per step: both perturbation streams in one pass over the weights,
// with the perturbation generated in the weight-tile loader.
#pragma once
#include "common.h"
#include "philox.h"

namespace zo2 {

struct SkinnyProblem {
    const void* Xp;         // [M, ldx] activations of the "+" stream (compute dtype)
    const void* Xm;         // [M, ldx] activations of the "-" stream
    const void* theta;      // [N, K] the weight as stored (dense, row n = output feature n; its update already applied)
    const void* bias_p;     // [N] perturbed bias of the "+" stream (compute dtype) or nullptr
    const void* bias_m;
    const float* res_p;     // [M, ldy] float32 residual or nullptr
    const float* res_m;
    void* Yp;               // [M, ldy] compute dtype or float32
    void* Ym;
    float out_scale;        // multiplies (acc + bias)
    uint32_t tensor_id;     // random stream of theta
};

struct SkinnyArgs {
    static constexpr int kMaxProblems = 3;
    int32_t M, N, K;        // M <= 256 rows per stream; K % 64 == 0; N % 4 == 0
    int64_t ldx, ldy;
    int32_t relu, out_f32, nprob;
    int32_t splits, k_per_split;     // filled in by skinny_launch: the k range is cut into `splits` pieces of k_per_split
    float eps;
    PhiloxKeys key;         // of the step seed
    float* partial;         // filled in by skinny_launch: [nprob][splits][2][M][N] float32 partial sums
    SkinnyProblem p[kMaxProblems];
};

// Y+- = act((X+- (theta +- eps z)^T + bias+-) * out_scale) + residual+- for every problem; the weights are read once
// and W+ = store(fma(+eps, z, theta)), W- = store(fma(-eps, z, theta)) exist only tile by tile in LDS.
zo2_status skinny_launch(SkinnyArgs& a, int dtype, void* workspace, size_t workspace_bytes, hipStream_t st);
size_t skinny_workspace_bytes(int M, int N, int K, int nprob);
bool skinny_applicable(int M, int N, int K, int dtype);
// W+ and W- of rows [n0, n0 + rows) of a dense [N, K] tensor, through the loader's own code path (a test hook)
zo2_status skinny_perturbed_rows(int dtype, const void* theta, int64_t K, int64_t n0, int64_t rows, uint32_t tensor_id, uint64_t seed,
                                 float eps, void* w_plus, void* w_minus, hipStream_t st);

}  // namespace zo2
