// Launch interface of causal self-attention.
#pragma once
#include "common.h"

namespace zo2 {

// q, k, v, out: [n_seq * seq, ld] of `dtype`; head h occupies columns h*d_head..; q pre-scaled.
zo2_status attention_launch(int dtype, const void* q, const void* k, const void* v, void* out,
                            int n_seq, int seq, int n_heads, int d_head, int64_t ld, hipStream_t st);

}  // namespace zo2
