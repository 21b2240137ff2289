// Launch interface of the fused update + perturb kernel (K1).
#pragma once
#include "common.h"
#include "philox.h"

namespace zo2 {

struct K1Seg {
    int64_t off;          // element offset of the segment inside the theta buffer
    uint64_t e0;          // index, inside its tensor, of the segment's first element (multiple of 8)
    uint64_t n;           // elements
    uint32_t tensor_id;   // selects the random stream
    float scale;          // wire scale of the tensor (8-bit formats), else 1
    int64_t woff;         // with K1Args::packed_w: element offset of the segment inside w_plus / w_minus
};

struct K1Args {
    static constexpr int kMaxSeg = 16;
    void* theta;          // wire dtype; rewritten in place when an update is pending
    void* w_plus;         // compute dtype, addressed as w_plus[off - w_off0 + i]
    void* w_minus;        // may be nullptr: only W+ is written (single forward)
    int64_t w_off0;       // element offset (in theta's numbering) that maps to w_plus[0]
    int32_t nseg;
    uint32_t total_chunks;
    float c_imm;          // eta_prev * g_prev, used when c_ptr == nullptr
    int32_t stochastic;   // 1: theta' is stored with stochastic rounding (low-bit wire formats), 0: to nearest
    int32_t reverse;      // 1: the grid walks the chunks from the last to the first
    int32_t packed_w;     // 1: a segment's copies start at w_plus[seg.woff] (segments packed densely) instead of w_plus[off - w_off0]
    int32_t pad_;
    float eps;
    const float* c_ptr;   // device scalar holding eta_prev * g_prev (stays on the GPU between steps)
    PhiloxKeys k_prev, k_cur;
    uint32_t first_chunk[kMaxSeg];   // filled in by k1_launch: first workgroup of each segment (0xffffffff past nseg)
    K1Seg seg[kMaxSeg];
};

// Enqueue K1 over the segments.  update: apply theta' = theta - c z_prev; perturb: write W+, W-.
zo2_status k1_launch(K1Args& a, int wire_dtype, int compute_dtype, bool update, bool perturb, hipStream_t st);
uint32_t k1_chunks(uint64_t n);

}  // namespace zo2
