// Launch interface of causal self-attention.
#pragma once
#include "common.h"

namespace zo2 {

// q, k, v, out: [n_seq * seq, ld] of `dtype`; head h occupies columns h*d_head..; q pre-scaled.
// bf16 / fp16 with d_head 64, 80 or 128 run on the matrix cores unless vector_kernel != 0; everything else
// (and float32) runs on the float32 vector-ALU kernel.
zo2_status attention_launch(int dtype, const void* q, const void* k, const void* v, void* out, int n_seq, int seq, int n_heads,
                            int d_head, int64_t ld, int vector_kernel, hipStream_t st);

}  // namespace zo2
