/*
 * zo2.h -- C ABI of libzo2: the zeroth-order (MeZO / SPSA) fine-tuning step of ZO2
 * over an OPT-shaped decoder on one AMD MI355X (gfx950).
 *
 * Two layers of entry points:
 *
 *   1. the training context: zo2_init / zo2_set_resident_budget / zo2_step / zo2_step_extra / zo2_step_multi / zo2_flush / zo2_eval /
 *      zo2_get_pending / zo2_set_pending / zo2_sync_to_host / zo2_get_plan / zo2_get_scratch_plan / zo2_destroy.  One call of zo2_step is one iteration of the paper's
 *      Alg. 2: for every module (embedding, decoder blocks, LM head) apply the update left
 *      pending by the previous iteration, perturb by +eps z and -eps z, run both forwards,
 *      and form the projected gradient g (Eq. 2).  Blocks that do not fit the HBM budget
 *      live in host memory and are streamed (Alg. 3, Sec. 5.2-5.5).
 *
 *   2. zo2_op_*: the individual HIP kernels on caller-supplied device buffers, so that
 *      each can be checked and timed alone at full problem shapes.
 *
 * Conventions for every function:
 *   - plain C, no exceptions, no hidden global state (the two measurement switches zo2_op_set_gemm_tile_rows and
 *     zo2_op_set_gemm_wavefronts are process-wide and say so); every call returns a zo2_status
 *     (0 = success) and, on failure, leaves a message retrievable with zo2_last_error
 *     (context calls) or zo2_op_last_error (op calls, thread local);
 *   - "host" pointers are ordinary or pinned host memory; "device" pointers are HBM of the
 *     current HIP device; `stream` arguments are hipStream_t passed as void* (NULL = the
 *     default stream).  Op calls only enqueue work on that stream; they never synchronise;
 *   - matrices are row-major; a linear layer's weight is [out_features, in_features];
 *   - nothing here allocates device memory: the caller hands in an arena (context) or the
 *     buffers themselves (ops);
 *   - zo2_step / zo2_step_extra / zo2_eval emit named ranges ("zo2_step", "block 7", "lm_head + loss") through the
 *     profiler's marker library when it can be loaded (rocprofv3 --marker-trace), bracketing the enqueue of each phase.
 */
#ifndef ZO2_H
#define ZO2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zo2_ctx zo2_ctx;

typedef enum {
    ZO2_OK = 0,
    ZO2_EINVAL = 1,     /* bad argument, shape or token / label id                      */
    ZO2_ENOMEM = 2,     /* host allocation failed or the arena is too small             */
    ZO2_EBUDGET = 3,    /* the HBM budget cannot hold embeddings + 3 block slots + work */
    ZO2_EHIP = 4,       /* a HIP runtime call failed                                    */
    ZO2_ESTATE = 5,     /* the context is unusable after an earlier ZO2_EHIP            */
    ZO2_ENONFINITE = 6  /* a loss came out NaN or infinite: outputs are still written, that
                           iteration's update is dropped, the context stays usable      */
} zo2_status;

/* Storage formats.  F32/BF16/F16 may be compute formats; all five may be transfer
 * ("wire") formats, i.e. the format parameters are held in on the host and in the
 * upload slots (Sec. 5.5: bf16/fp16 halve, 8-bit floats quarter the fp32 volume).
 * The 8-bit formats are the OCP E4M3 (no infinity, max 448) and E5M2 encodings,
 * converted with round-to-nearest-even and saturation. */
typedef enum { ZO2_F32 = 0, ZO2_BF16 = 1, ZO2_F16 = 2, ZO2_FP8_E4M3 = 3, ZO2_FP8_E5M2 = 4 } zo2_dtype;

typedef struct {
    int32_t n_layers, d_model, n_heads, d_ffn, vocab;
    int32_t max_pos;        /* longest sequence; the position table has max_pos + pos_offset rows */
    int32_t pos_offset;     /* row used for position t is t + pos_offset (2 for OPT)               */
    int32_t tied_lm_head;   /* 1: the LM head is the token embedding (one tensor, one z)           */
    int32_t wire_dtype;     /* zo2_dtype of the parameters in host memory and in the slots         */
    int32_t compute_dtype;  /* zo2_dtype of W+ / W- and of the GEMM inputs: F32, BF16 or F16       */
    float ln_eps;           /* LayerNorm epsilon (1e-5)                                            */
} zo2_config;

/* Parameter tensors are numbered for the random stream in module order (Alg. 2):
 *   0 tok_emb [vocab, d]; 1 pos_emb [max_pos + pos_offset, d];
 *   2 + 16 l + k for block l, k = 0..15 over
 *     ln1.w ln1.b q.w q.b k.w k.b v.w v.b o.w o.b ln2.w ln2.b fc1.w fc1.b fc2.w fc2.b;
 *   2 + 16 L, 3 + 16 L: final_ln.w, final_ln.b;  4 + 16 L: lm_head.w (only if untied).
 * z of element e of tensor p at step seed s is a pure function of (s, p, e): Philox4x32-10
 * with key (lo32 s, hi32 s) and counter (lo32 q, hi32 q, p, 0), q = e >> 3; output word
 * (e >> 1) & 3 feeds the Box-Muller pair of elements (e & ~1, e | 1): its high 16 bits give
 * the radius, its low 16 bits the angle (cosine for the even element, sine for the odd one).
 * This replaces the saved / restored generator states of Alg. 2 (Sec. 5.1). */
#define ZO2_BLOCK_TENSORS 16

/* A block's 16 tensors are packed into one contiguous "bucket" (Sec. 5.3): tensor k starts
 * at element offset offs[k], a multiple of 256 elements; offs[16] is the padded element
 * count of the bucket.  The same element offsets hold for every dtype.  Returns ZO2_EINVAL
 * if d_model or d_ffn is not a positive multiple of 8 or n_heads does not divide d_model. */
zo2_status zo2_block_tensor_offsets(const zo2_config* cfg, int64_t offs[ZO2_BLOCK_TENSORS + 1]);
size_t zo2_dtype_size(int32_t dtype);   /* bytes per element; 0 for an unknown dtype */

typedef struct {
    void* tok_emb;            /* host, [vocab, d], wire dtype                                     */
    void* pos_emb;            /* host, [max_pos + pos_offset, d]                                   */
    void* final_ln_w;         /* host, [d]                                                         */
    void* final_ln_b;         /* host, [d]                                                         */
    void* lm_head;            /* host, [vocab, d]; must be NULL when tied_lm_head = 1              */
    void** block_bucket;      /* host array of n_layers host pointers, one bucket each; pinned
                                 memory is needed for the streamed mode to overlap copies          */
    const float* tensor_scale;/* host, one float per tensor id, or NULL (= all 1).  Stored value =
                                 round(theta * scale); used by the 8-bit wire formats (Sec. 5.5), must
                                 be NULL or all 1 otherwise.  Every scale must be a power of two, so
                                 that scaling and un-scaling are exact (ZO2_EINVAL otherwise).     */
} zo2_host_weights;

typedef struct {
    void* arena;              /* device memory the library may use, 256-byte aligned              */
    size_t arena_bytes;
    void* stream_compute;     /* hipStream_t; kernels                                             */
    void* stream_upload;      /* hipStream_t; host -> device block copies                         */
    void* stream_offload;     /* hipStream_t; device -> host block copies                         */
    void* stream_k1;          /* hipStream_t or NULL.  When given (and the budget has room for a
                                 second W+/W- scratch set) the fused update + perturb pass of block
                                 l+1 runs on it concurrently with the forwards of block l          */
} zo2_device;

/* Create a context.  The host weight buffers are borrowed until zo2_destroy and are the
 * master copy of every streamed block: they are overwritten in place as training proceeds
 * (Sec. 4.2).  Embeddings, final LayerNorm and LM head are copied into the arena and stay
 * there (Sec. 5.2); zo2_sync_to_host writes them back.  The arena and the three streams
 * are borrowed too.  The initial budget is the whole arena.  Not thread safe. */
zo2_status zo2_init(zo2_ctx** out, const zo2_config* cfg, const zo2_host_weights* w, const zo2_device* dev);

/* Limit the arena bytes the library may touch (embeddings + block slots + W+/W- scratch +
 * activations).  If every block fits, all blocks are kept resident and no copies are issued
 * per step; otherwise blocks are streamed through a ring of >= 3 equal slots.  Takes effect
 * at the next step (the plan also depends on that step's batch x seq).  Fails with
 * ZO2_EBUDGET at that step if even 3 slots do not fit. */
zo2_status zo2_set_resident_budget(zo2_ctx* ctx, size_t hbm_bytes);

/* One ZO-SGD iteration (Alg. 2) on a batch.  tokens, labels: host int32 [batch, seq];
 * labels[b, t] is the target of position t (the caller shifts), -100 = ignored.
 * lr given here belongs to this iteration's g (eta_j): it is applied, with this seed's z,
 * when each module is next visited (Sec. 5.4) or by zo2_flush.  Blocks until the three
 * results are on the host:  *loss_plus = L(theta + eps z), *loss_minus = L(theta - eps z),
 * *g = (l+ - l-) / (2 eps). */
zo2_status zo2_step(zo2_ctx* ctx, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                    uint64_t seed, float eps, float lr, float* loss_plus, float* loss_minus, float* g);

/* One more direction of the current round: the q-direction form of the randomized gradient estimate (Sec. 3:
 * the framework carries over to other ZO estimators; this one averages Eq. 2 over q directions z_0 .. z_q-1
 * drawn at the same parameters).  A round is zo2_step(seed_0, lr_0) followed by q - 1 calls of
 * zo2_step_extra(seed_i, lr_i) on the same batch (lr_i = eta / q for the plain average).  The call perturbs
 * the parameters as zo2_step left them -- none of the round's own updates is visible to it -- runs the same
 * dual forward, and defers its update eta_i g_i z_i with the others; nothing is applied, and streamed blocks
 * are uploaded but not written back.  The next zo2_step, zo2_eval or zo2_flush applies the round's updates to
 * each module in the order i = 0 .. q - 1 (the first q - 1 as update-only sweeps while the module is on the
 * device, the last one fused with the next perturbation as usual).  At most 16 directions per round
 * (ZO2_ESTATE beyond, and without a zo2_step before).  Arguments, outputs and ZO2_ENONFINITE as for zo2_step;
 * a non-finite direction is dropped from the round. */
zo2_status zo2_step_extra(zo2_ctx* ctx, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                          uint64_t seed, float eps, float lr, float* loss_plus, float* loss_minus, float* g);

/* A whole round of n_dirs directions in one pass over the model (the same estimator as zo2_step + zo2_step_extra,
 * Sec. 3): every module - embedding, each block, head - runs the dual forwards of all directions before the pass moves
 * on, so a streamed block is uploaded once per round instead of once per direction; where the host link bounds the step
 * (Sec. 5.2: compute waits for uploads) further directions cost little until compute catches up with the link.
 * seeds: host array of n_dirs seeds; lr: the step size of each direction (eta / n_dirs for the plain average);
 * results: host array of 3 n_dirs floats, (l+, l-, g) per direction.  Losses, g and the state left behind (deferred
 * updates, parameters) equal those of zo2_step(seeds[0]) followed by zo2_step_extra(seeds[1 ..]) bit for bit.  Needs one
 * more residual stream (2 tokens x d_model floats) of arena per further direction; the plan is redone when n_dirs
 * exceeds what it holds.  1 <= n_dirs <= 16 (ZO2_EINVAL beyond); ZO2_ENONFINITE if any direction's loss is not finite:
 * then the whole round is dropped (results still filled in). */
zo2_status zo2_step_multi(zo2_ctx* ctx, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                          int32_t n_dirs, const uint64_t* seeds, float eps, float lr, float* results);

/* Apply the pending update to every parameter now (Alg. 2 leaves the last g unapplied). */
zo2_status zo2_flush(zo2_ctx* ctx);

/* Loss of the current parameters on a batch with a single, unperturbed forward pass over the same
 * block walk as zo2_step (the evaluation regime of the paper's Limitation section: one forward per
 * block, so a streamed block's copy time is hidden by half the compute).  A pending update is applied
 * to each module on the way, exactly as zo2_step would (Sec. 5.4), so *loss = L(theta_up_to_date)
 * and nothing is pending afterwards; training continued after the call gives the same results as
 * without it.  Streamed blocks are written back only if an update was pending.  tokens, labels as
 * for zo2_step.  *loss is written on ZO2_OK (it may be non-finite). */
zo2_status zo2_eval(zo2_ctx* ctx, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq, float* loss);

/* The deferred update as data (Sec. 5.4): *has_pending, and if set the seed whose z it uses and
 * *step = eta * g.  With the parameters in the host buffers (zo2_sync_to_host) this is the complete
 * training state: a context created from those buffers and given the same triple with
 * zo2_set_pending continues bit-identically.  zo2_set_pending replaces whatever was pending. */
zo2_status zo2_get_pending(zo2_ctx* ctx, int32_t* has_pending, uint64_t* seed, float* step);
zo2_status zo2_set_pending(zo2_ctx* ctx, int32_t has_pending, uint64_t seed, float step);

/* The same for a round of several directions (zo2_step_extra): how many updates are deferred, update i
 * (0 <= i < count, in the order of application), and appending one to those already deferred.
 * zo2_get_pending answers ZO2_ESTATE while more than one is deferred. */
zo2_status zo2_pending_count(zo2_ctx* ctx, int32_t* count);
zo2_status zo2_get_pending_at(zo2_ctx* ctx, int32_t i, uint64_t* seed, float* step);
zo2_status zo2_add_pending(zo2_ctx* ctx, uint64_t seed, float step);

/* Copy device-resident parameters (embeddings, final LayerNorm, LM head, and the blocks when
 * all are resident) back into the caller's host buffers.  Does not flush. */
zo2_status zo2_sync_to_host(zo2_ctx* ctx);

/* Facts about the plan used by the last step: how many block slots exist, whether blocks are
 * resident, how many arena bytes are in use.  Any pointer may be NULL. */
zo2_status zo2_get_plan(const zo2_ctx* ctx, int32_t* n_slots, int32_t* resident, size_t* bytes_used);

/* How the W+ / W- scratch of the last plan is organised (Sec. 5.3's reusable block space, applied to the perturbed
 * copies).  The forward of a block needs its tensors in four groups, {ln1, q, k, v} {o} {ln2, fc1} {fc2}, one after
 * the other.  *sweeps_per_block = 1: the scratch holds a whole block and one update + perturb sweep per block fills
 * it; 2: it holds the larger half ({ln1 .. o} or {ln2 .. fc2}) and is refilled before the FFN; 4: it holds the
 * largest group and is refilled before every projection.  More sweeps need less memory (the two whole-block copies
 * of the OPT-175B shape alone would take 7 GB) and hand each copy to its projection while it is still in the
 * memory-side cache.  *scratch_elems = elements of one copy; *scratch_sets = 1, or 2 when zo2_device.stream_k1 is in
 * use.  Any pointer may be NULL.  Results do not depend on the organisation. */
zo2_status zo2_get_scratch_plan(const zo2_ctx* ctx, int32_t* sweeps_per_block, int64_t* scratch_elems, int32_t* scratch_sets);

/* sweeps = 1, 2 or 4: use exactly that organisation (ZO2_EBUDGET at the next step if 3 block slots do not fit next to
 * it); 0 (default): the planner starts from its preferred organisation and moves to smaller scratch sets until 3
 * block slots fit.  Takes effect at the next step.  ZO2_EINVAL for any other value. */
zo2_status zo2_set_scratch_plan(zo2_ctx* ctx, int32_t sweeps);

/* Where the perturbation of a block's six weight matrices is generated.  By default (mode 0) a step of at most 64
 * tokens per stream - where the projections are bound by reading the weights - lets the projections read the stored
 * weights and form W+ / W- in their loader (zo2_op_gemm_perturbed), the sweep kernel then only applies the pending
 * update and perturbs the block's one-dimensional tensors; larger steps write the perturbed copies with the sweep kernel,
 * because a weight tile would otherwise be regenerated once per 256-row tile of activations.  mode 1: in the loader
 * whenever the shapes allow (16-bit storage equal to the compute format, d_model and d_ffn multiples of 64, at most
 * 256 tokens per stream); mode -1: never.  The two paths give the same W+- bit for bit; their projections add the
 * same products in a different order (results agree to float32 rounding, each path is deterministic by itself).
 * Evaluation passes (zo2_eval) always take the sweep-kernel path.  Takes effect at the next step. */
zo2_status zo2_set_loader_fusion(zo2_ctx* ctx, int32_t mode);
/* *active = 1 if the last plan lets the projections perturb in their loader. */
zo2_status zo2_get_loader_fusion(const zo2_ctx* ctx, int32_t* active);
/* How often streamed blocks travel back to the host (Sec. 5.2 offloads a block after every update; this is an option on
 * top of it).  A block's update is a function of (seed, eta g) alone (Sec. 5.1, 5.4), so a block whose host copy lacks a
 * few updates can take them - in order, with the same roundings - the next time it is uploaded, and skip the trip back:
 * with an interval of k updates the offload stream carries a block every k-th step only, the other steps move half the
 * bytes over the host link.  Losses, g and (after zo2_flush / zo2_sync_to_host) parameters are bit-identical to an
 * interval of 1.  While updates are lacking the caller's block buffers are NOT current: zo2_flush, zo2_sync_to_host,
 * a new memory plan and zo2_destroy bring them up to date first.  1 (default) .. 16.  No effect on resident blocks. */
zo2_status zo2_set_writeback_interval(zo2_ctx* ctx, int32_t updates);
/* *interval: the setting; *lacking: updates the host copies of streamed blocks lack at the moment. */
zo2_status zo2_get_writeback_state(const zo2_ctx* ctx, int32_t* interval, int32_t* lacking);
/* Split-k of the block projections (Alg. 2 "forward"; a launch-shape decision, not part of the method).  mode 0 (default):
 * a projection whose tiles would fill the compute units badly - few tokens per stream, or a tile count just above a
 * multiple of the compute units with a long k - is cut into 2 or 4 pieces along k that run side by side into float32 partial sums, added in piece order by a second kernel (deterministic;
 * results differ from the unsplit launch by float32 rounding order only).  mode -1: never.  Takes effect at the next step. */
zo2_status zo2_set_split_k(zo2_ctx* ctx, int32_t mode);

/* Per-stream busy time of the last step in milliseconds (compute, upload, offload) and the
 * bytes copied each way; for host-link rate reporting.  Any pointer may be NULL. */
zo2_status zo2_get_step_stats(const zo2_ctx* ctx, float* ms_compute, float* ms_upload, float* ms_offload,
                              uint64_t* bytes_up, uint64_t* bytes_down);

/* Per-kernel-class timing of zo2_step, for roofline reporting.  With a class's bit set, every
 * launch of that class on the compute stream is bracketed by a pair of HIP events;
 * zo2_get_kernel_times returns, for the last step, the summed elapsed milliseconds and the
 * number of launches per class.  Off (mask 0) by default. */
#define ZO2_KERNEL_CLASSES 6
enum { ZO2_KC_K1 = 0,     /* fused update + perturb                        */
       ZO2_KC_GEMM = 1,   /* QKV / output / FFN / LM-head projections      */
       ZO2_KC_ATTN = 2,   /* causal attention                              */
       ZO2_KC_LN = 3,     /* LayerNorm                                     */
       ZO2_KC_EMBED = 4,  /* embedding gather                              */
       ZO2_KC_CE = 5 };   /* cross-entropy rows + scalar epilogue          */
zo2_status zo2_set_profiling(zo2_ctx* ctx, uint32_t class_mask);
zo2_status zo2_get_kernel_times(const zo2_ctx* ctx, float ms[ZO2_KERNEL_CLASSES], int32_t launches[ZO2_KERNEL_CLASSES]);

/* Test aid for the block scheduler (Alg. 3): before every block's work on stream `which`
 * (0 compute, 1 upload, 2 offload) an idle kernel of the given duration (<= 100 ms) is enqueued.  With the
 * dependency rules of Sec. 5.2 in place no choice of delays can change any result. */
zo2_status zo2_debug_set_stream_delay(zo2_ctx* ctx, int32_t which, uint32_t microseconds);

/* Second test aid for the same rules: with enabled != 0 every slot is filled with 0xFF bytes (a NaN pattern in each of
 * the five formats) on the upload stream right before a block is copied into it.  A kernel that read a slot before its
 * upload had landed ("computing on a half-uploaded block", Sec. 5.2) would turn the losses into NaN; with the
 * dependencies in place nothing changes. */
zo2_status zo2_debug_set_slot_poison(zo2_ctx* ctx, int32_t enabled);

/* Rounding of the updated parameters into a low-bit wire format (Sec. 5.5 leaves it open; default 0 = to
 * nearest, ties to even, which is what a plain cast does).  With stochastic != 0, theta' = theta - eta g z is
 * stored as one of its two neighbours in the format, the one further from zero with probability
 * (|x| - lo) / (hi - lo): realised as r16 < 65536 (|x| - lo) / (hi - lo) with 16 bits r16 per element from the
 * same Philox4x32-10 stream as z_prev but with the last counter word set to 1 (call e >> 3, low / high half of
 * output word (e >> 1) & 3 for even / odd e).  Values beyond the largest finite value saturate.  A master copy
 * in bf16 / fp16 / fp8 then follows updates far below its spacing in expectation; with rounding to nearest
 * such updates are lost.  No effect on a float32 wire.  Takes effect at the next update. */
zo2_status zo2_set_wire_rounding(zo2_ctx* ctx, int32_t stochastic);

/* Ablation switch for the dynamic scheduler (Sec. 5.2; the paper's reverse ablation, Table 4, "no
 * scheduler overlap"): with enabled = 0 a streamed block's upload, compute and offload run strictly
 * one after the other (the host waits in between), and the next block's upload starts only then.
 * Results do not change.  Default: enabled; ignored while zo2_device.stream_k1 is in use.  The table's "no efficient update" column needs no
 * switch: call zo2_flush after every zo2_step (each block then travels twice per iteration). */
zo2_status zo2_set_stream_overlap(zo2_ctx* ctx, int32_t enabled);

const char* zo2_last_error(const zo2_ctx* ctx);
void zo2_destroy(zo2_ctx* ctx);

/* ------------------------------------------------------------------------------------
 * Kernel-level entry points.  All pointers are device pointers unless named host_*.
 * ------------------------------------------------------------------------------------ */

const char* zo2_op_last_error(void);

/* Words e0 .. e0+n-1 of the random stream of tensor `tensor_id` at `seed`: word j is output
 * j & 3 of Philox call j >> 2; elements 2j and 2j+1 are drawn from it (test hook for the
 * bit-exactness of the stream).  out: device uint32[n]. */
zo2_status zo2_op_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t e0, uint64_t n, uint32_t* out, void* stream);

/* z of elements e0 .. e0+n-1 of the tensor as float32.  out: device float[n]. */
zo2_status zo2_op_gaussian(uint64_t seed, uint32_t tensor_id, uint64_t e0, uint64_t n, float* out, void* stream);

/* Fused regenerate + update + perturb (Alg. 2 DualForward lines "update", "perturb";
 * Sec. 5.4) over a window of one tensor:
 *   theta'  = store_wire( fma(-c, z_prev, theta) )        (skipped when has_pending = 0)
 *   w_plus  = store_compute( fma(+eps, z, theta') ),  w_minus = store_compute( fma(-eps, z, theta') )
 * theta: n elements of wire dtype, element i being element e0 + i of the tensor; e0 and
 * every pointer must be aligned to 8 elements.  theta is rewritten in place; w_plus /
 * w_minus (compute dtype, n elements) may both be NULL for an update-only pass, or w_minus
 * alone for a pass that writes only w_plus; with eps = 0 no z is drawn and w_plus = theta'.
 * scale: the tensor's wire scale (1 unless an 8-bit format uses one; a power of two).  stochastic_rounding != 0 stores theta'
 * as zo2_set_wire_rounding describes. */
zo2_status zo2_op_update_perturb(void* theta, int32_t wire_dtype, void* w_plus, void* w_minus, int32_t compute_dtype,
                                 uint32_t tensor_id, uint64_t e0, uint64_t n,
                                 int32_t has_pending, uint64_t seed_prev, float c,
                                 uint64_t seed, float eps, float scale, int32_t stochastic_rounding, void* stream);

/* The same over one whole block bucket (Sec. 5.3) in a single launch, as the step issues it per decoder block:
 * bucket holds the 16 tensors of block `layer` at the offsets of zo2_block_tensor_offsets(cfg) in cfg->wire_dtype
 * and is rewritten in place; w_plus / w_minus: buffers of the same element count in cfg->compute_dtype (same
 * offsets; NULL as above); tensor k draws from random stream 2 + 16 layer + k.  host_scales: 16 floats in host
 * memory (powers of two) or NULL for all 1.  The padding between tensors is neither read nor written. */
zo2_status zo2_op_update_perturb_block(const zo2_config* cfg, int32_t layer, void* bucket, void* w_plus, void* w_minus,
                                       int32_t has_pending, uint64_t seed_prev, float c, uint64_t seed, float eps,
                                       const float* host_scales, int32_t stochastic_rounding, void* stream);

/* Low-bit pack / unpack (Sec. 5.5): convert n elements between two storage formats,
 * dst = store_dst(load_src(src) / scale_src * scale_dst). */
zo2_status zo2_op_convert(const void* src, int32_t src_dtype, float src_scale,
                          void* dst, int32_t dst_dtype, float dst_scale, uint64_t n, void* stream);

/* Y[M, N] = act( (X[M, K] . W[N, K]^T + bias[N]) * out_scale ) + residual[M, N].
 * X, W, bias: `dtype` (F32, BF16 or F16), leading dimensions ldx, ldw in elements;
 * residual: float32 [M, ldy] or NULL; Y: out_dtype (F32 or `dtype`) with leading dimension ldy;
 * relu: apply max(.,0) before the residual.  Accumulation is float32.  K must be a multiple of 8. */
zo2_status zo2_op_gemm(int32_t dtype, int32_t M, int32_t N, int32_t K,
                       const void* X, int64_t ldx, const void* W, int64_t ldw, const void* bias,
                       const float* residual, void* Y, int32_t out_dtype, int64_t ldy,
                       float out_scale, int32_t relu, void* stream);

/* zo2_op_gemm with the k range cut into `splits` (2 or 4) pieces: the pieces run as one launch into float32 partial sums
 * in `workspace` (device, 16-byte aligned, zo2_op_gemm_split_k_workspace_bytes(M, N, splits) bytes, overwritten), a second
 * kernel adds them in piece order and applies bias, scale, ReLU and residual.  16-bit dtypes; N % 4 == 0, ldy % 4 == 0,
 * K % (8 splits) == 0.  zo2_op_gemm_split_k_pieces: the number of pieces (1, 2 or 4) zo2_step would use for a launch of `nprob`
 * problems of this shape.  ZO2_EINVAL on anything else. */
zo2_status zo2_op_gemm_split_k(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                               const void* bias, const float* residual, void* Y, int32_t out_dtype, int64_t ldy, float out_scale,
                               int32_t relu, int32_t splits, void* workspace, size_t workspace_bytes, void* stream);
size_t zo2_op_gemm_split_k_workspace_bytes(int32_t M, int32_t N, int32_t splits);
int32_t zo2_op_gemm_split_k_pieces(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t nprob);
/* The same projection for both perturbation streams at once, with the perturbation generated in the weight loader
 * (Alg. 2 "perturb" folded into the forward; for steps of few tokens, where the projections are bound by reading the
 * weights): Y+- [M, N] = act( (X+- [M, K] . (theta +- eps z)^T + bias+-) * out_scale ) + residual+-, where theta [N, K]
 * is the stored weight (dense, leading dimension K, in `dtype` = BF16 or F16, its pending update already applied) and
 * z its random direction at `seed` (tensor_id selects the stream).  W+ = store(fma(+eps, z, theta)) and
 * W- = store(fma(-eps, z, theta)) are formed tile by tile on chip - bit for bit what zo2_op_update_perturb writes - and
 * theta is read once for both streams.  M <= 256, K % 64 == 0, N % 4 == 0, operands 16-byte aligned; bias+-: already
 * perturbed [N] vectors of `dtype` or both NULL; residual+-: float32 [M, ldy] or both NULL (needs F32 output).  The k
 * range is cut into slices whose float32 partial sums live in `workspace` (device, 16-byte aligned, at least
 * zo2_op_gemm_perturbed_workspace_bytes(M, N, K) bytes) and are added in slice order: results are deterministic. */
zo2_status zo2_op_gemm_perturbed(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X_plus, const void* X_minus, int64_t ldx,
                                 const void* theta, uint32_t tensor_id, uint64_t seed, float eps,
                                 const void* bias_plus, const void* bias_minus, const float* residual_plus, const float* residual_minus,
                                 void* Y_plus, void* Y_minus, int32_t out_dtype, int64_t ldy, float out_scale, int32_t relu,
                                 void* workspace, size_t workspace_bytes, void* stream);
size_t zo2_op_gemm_perturbed_workspace_bytes(int32_t M, int32_t N, int32_t K);

/* W+ and W- of rows n0 .. n0 + rows - 1 of a dense [N, K] tensor through the code path of that loader (test hook:
 * the bits must equal those of zo2_op_update_perturb without an update).  theta points at row n0. */
zo2_status zo2_op_perturbed_rows(int32_t dtype, const void* theta, int64_t K, int64_t n0, int64_t rows, uint32_t tensor_id,
                                 uint64_t seed, float eps, void* w_plus, void* w_minus, void* stream);

/* The large-tile GEMM kernel works on 256- or 128-row tiles and picks the height per launch (whichever fills the
 * rounds of tiles over the compute units better).  rows = 128 or 256 forces one height for every later launch of the
 * process, step calls included; 0 restores the choice per launch.  For tests and measurements: results are the same
 * bit for bit either way (the order in which a dot product is accumulated does not depend on the tile height).
 * Returns ZO2_EINVAL for any other value. */
zo2_status zo2_op_set_gemm_tile_rows(int32_t rows);

/* Measurement aid, available in the instrumented build only (`build.py --gemm-stamps` -> libzo2_stamps.so; the ordinary
 * library returns ZO2_ESTATE): zo2_op_gemm without bias on the large-tile kernel (K % 128 == 0, N >= 256; ZO2_EINVAL
 * otherwise), during which workgroup 37 records the shader clock around the phases of its tiles.  stamps: 64 device
 * words: per tile (up to 14) the clock at its start, after the wait for its first k-slab, after its k loop and after
 * its epilogue; [60] cycles spent waiting for loads and [61] at the barriers in the middle of the k-slabs (the last
 * launch's tiles), [62] the number of tiles.  The timer reads slow the kernel down by a few percent. */
zo2_status zo2_op_gemm_phases(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                              const float* residual, void* Y, int32_t out_dtype, int64_t ldy, uint64_t* stamps, void* stream);

/* Launches of 256-row tiles run with eight wavefronts per workgroup (two per SIMD, one k-slab of prefetch) or with
 * four (a further slab in flight in registers), chosen per launch by the length of k and the number of rows.  waves = 4 or 8 forces one form
 * for every later launch of the process, step calls included; 0 restores the choice per launch.  For tests and
 * measurements: results are the same bit for bit either way.  Returns ZO2_EINVAL for any other value. */
zo2_status zo2_op_set_gemm_wavefronts(int32_t waves);

/* Causal multi-head self-attention.  q, k, v, out: [n_seq * seq, ld] of `dtype`, head h in
 * columns h*d_head .. (h+1)*d_head-1; q already carries the 1/sqrt(d_head) factor.
 * out[i] = softmax_{j <= i}(q_i . k_j) v_j within each sequence.  d_head in {8,16,32,64,80,128}.
 * bf16 / fp16 with d_head 64, 80 or 128 run on the matrix cores (operands 16-byte aligned) unless
 * vector_kernel != 0; everything else, and F32, runs on a float32 vector kernel. */
zo2_status zo2_op_attention(int32_t dtype, const void* q, const void* k, const void* v, void* out,
                            int32_t n_seq, int32_t seq, int32_t n_heads, int32_t d_head, int64_t ld,
                            int32_t vector_kernel, void* stream);

/* y[r, :] = (x[r, :] - mean) / sqrt(var + eps) * w + b, biased variance; x float32 [rows, d],
 * w, b, y of `dtype`.  Rows >= rows_first use w2 / b2 (the "-" stream's perturbed gain and
 * bias); pass rows_first = rows to use w / b only. */
zo2_status zo2_op_layernorm(int32_t dtype, const float* x, const void* w, const void* b, const void* w2, const void* b2,
                            void* y, int32_t rows, int32_t rows_first, int32_t d, float eps, void* stream);

/* Row-wise cross-entropy of float32 logits [rows, ld] against labels (device int32, -100 =
 * ignored): row_loss[r] = logsumexp(logits[r, :vocab]) - logits[r, label], or 0 if ignored. */
zo2_status zo2_op_cross_entropy_rows(const float* logits, int64_t ld, const int32_t* labels, int32_t rows, int32_t vocab,
                                     float* row_loss, void* stream);

/* LM head and cross-entropy in one pass, without materialising the logits (Alg. 2
 * "DualForward(LM head)"; the step uses this for 16-bit compute formats): for X [M, ldx] and
 * W [N, ldw] (row n = vocabulary entry n) of `dtype` (BF16 or F16),
 *   row_loss[r] = logsumexp_n(X[r, :] . W[n, :]) - X[r, :] . W[labels[r], :],   0 if labels[r] = -100.
 * The GEMM epilogue reduces every 64-column span of a row to (max, sum exp) in float32; a second
 * kernel merges the spans.  Needs M, N >= 256, K % 128 == 0, N % 4 == 0, 16-byte aligned operands
 * (ZO2_EINVAL otherwise) and a 256-byte aligned device workspace of at least
 * zo2_op_lm_head_ce_workspace_bytes(M, N) bytes.  labels: device int32 [M]; row_loss: device float [M]. */
zo2_status zo2_op_lm_head_ce(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx,
                             const void* W, int64_t ldw, const int32_t* labels, float* row_loss,
                             void* workspace, size_t workspace_bytes, void* stream);
size_t zo2_op_lm_head_ce_workspace_bytes(int32_t M, int32_t N);

/* zo2_op_lm_head_ce for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc) and therefore have no workspace to pass: same arguments without the
 * workspace, same kernels, same results bit for bit.  The (max, sum exp) partials go to a buffer of
 * ZO2_STATIC_SCRATCH_BYTES built into the library (one copy per GPU, held until the process ends); the call
 * allocates nothing and frees nothing.  Shapes whose partials need more - (8 ceil(N / 256) + 1) * M * 4 bytes, e.g.
 * beyond 2659 rows at N = 50272 - are refused with ZO2_EINVAL; use zo2_op_lm_head_ce for those.  All calls on one
 * GPU share that GPU's buffer: calls that overlap in time on one GPU (different streams or threads) race and must
 * be serialised by the caller; calls on one stream are ordered by the stream.  The buffer keeps the previous
 * call's contents; nothing in it needs clearing, every value read is written earlier in the same call. */
#define ZO2_STATIC_SCRATCH_BYTES (16u << 20)
zo2_status zo2_op_lm_head_ce_static(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx,
                                    const void* W, int64_t ldw, const int32_t* labels, float* row_loss, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZO2_H */
