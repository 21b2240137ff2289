// Launch interfaces of the row-wise / elementwise kernels.
#pragma once
#include "common.h"
#include "philox.h"

namespace zo2 {

zo2_status philox_words(uint64_t seed, uint32_t tid, uint64_t e0, uint64_t n, uint32_t* out, hipStream_t st);
zo2_status gaussian(uint64_t seed, uint32_t tid, uint64_t e0, uint64_t n, float* out, hipStream_t st);
zo2_status convert(const void* src, int sdt, float sscale, void* dst, int ddt, float dscale, uint64_t n, hipStream_t st);
zo2_status layernorm(int dtype, const float* x, const void* w, const void* b, const void* w2, const void* b2, void* y,
                     int rows, int rows_first, int d, float eps, hipStream_t st);

struct EmbedArgs {
    const void* tok_emb;     // wire dtype [vocab, d] (not yet updated this step)
    const void* pos_emb;     // wire dtype [max_pos + pos_offset, d]
    const int32_t* tokens;   // device int32 [T]
    float* h;                // out: float32 [2 T, d]; rows 0..T-1 the "+" stream, T..2T-1 the "-" stream
    int32_t T, seq, d, pos_offset;
    float eps, scale_tok, scale_pos;
    int32_t single;          // 1: only the "+" rows are produced (single forward; eps is 0 then)
    int32_t stochastic;      // 1: the pending update is stored with stochastic rounding, as K1 will do for the table
    const float* c_ptr;      // device scalar eta_prev * g_prev
    PhiloxKeys k_prev, k_cur;
};
zo2_status embed_gather(const EmbedArgs& a, int wire_dtype, int compute_dtype, bool update, hipStream_t st);

// rows of logits -> row_loss[row0 + r]; the label of stacked row i is labels[i % label_period]
zo2_status cross_entropy_rows(const float* logits, int64_t ld, const int32_t* labels, int rows, int row0, int label_period,
                              int vocab, float* row_loss, hipStream_t st);
// span-major (max, sum exp) partials written by the LM-head kernel's cross-entropy mode -> row_loss[row0 + r]
zo2_status ce_combine(const float* part_max, const float* part_sum, const float* label_logit, const int32_t* labels, int rows,
                      int n_parts, int64_t part_ld, int row0, int label_period, float* row_loss, hipStream_t st);
// result[0..3] = l+, l-, g, number of counted labels; *c_pending = lr * g.  ns = 1 (single forward): only rows 0..T-1
// exist, result = (l, l, 0, count) and c_pending is left alone
zo2_status loss_epilogue(const float* row_loss, const int32_t* labels, int T, float eps, float lr, int ns, float* result,
                         float* c_pending, hipStream_t st);

}  // namespace zo2
