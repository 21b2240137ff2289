// Launch interface of causal self-attention.
#pragma once
#include "common.h"

namespace zo2 {

// q, k, v, out: [n_seq * seq, ld] of `dtype`; head h occupies columns h*d_head..; q pre-scaled.
// workspace: device scratch for the transposed values used by the MFMA path (bf16 / fp16 with
// d_head 64 or 128); attention_workspace_bytes gives its size (0 = the path does not apply).
// Without a large enough workspace the vector-ALU kernel runs instead.
zo2_status attention_launch(int dtype, const void* q, const void* k, const void* v, void* out, void* workspace, size_t workspace_bytes,
                            int n_seq, int seq, int n_heads, int d_head, int64_t ld, hipStream_t st);
size_t attention_workspace_bytes(int dtype, int n_seq, int seq, int n_heads, int d_head);

}  // namespace zo2
