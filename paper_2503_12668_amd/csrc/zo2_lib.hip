// libzo2: the training context (Alg. 2 + Alg. 3) and the C ABI.
//
// One zo2_step enqueues, without any host-side wait inside the block loop:
//   embedding gather (with on-the-fly update + perturb)  ->  for each decoder block
//   { [upload] -> K1 (update + perturb) -> dual forward -> [offload] }  ->  final LayerNorm
//   -> K1 on the LM-head weights -> LM head + cross-entropy -> g.
// Upload, compute and offload run on three HIP streams tied together by events only
// (Sec. 5.2); blocks cycle through a ring of equal slots carved out of the caller's arena
// (Sec. 5.3); each block crosses the host link once per direction per step because the
// update of iteration j-1 is applied when the block is visited in iteration j (Sec. 5.4).
#include <dlfcn.h>
#include <math.h>
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "attention.h"
#include "common.h"
#include "gemm.h"
#include "gemm_skinny.h"
#include "k1.h"
#include "rowops.h"

namespace zo2 {

static thread_local char g_op_error[512] = "";
void set_op_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_op_error, sizeof(g_op_error), fmt, ap);
    va_end(ap);
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Named ranges for profiler timelines (rocprofv3 --marker-trace): the tool's marker library is looked up at run time,
// once; without it the ranges cost one branch.  A range brackets the host-side enqueue of a phase of the step.
struct TraceRange {
    typedef int (*push_fn)(const char*);
    typedef int (*pop_fn)();
    static void lookup(push_fn& push, pop_fn& pop) {
        static push_fn p_push = nullptr;
        static pop_fn p_pop = nullptr;
        static std::once_flag once;
        std::call_once(once, [] {
            void* h = dlopen("librocprofiler-sdk-roctx.so.1", RTLD_NOW | RTLD_GLOBAL);     // what rocprofv3 listens to
            if (!h) h = dlopen("librocprofiler-sdk-roctx.so", RTLD_NOW | RTLD_GLOBAL);
            if (!h) h = dlopen("libroctx64.so.4", RTLD_NOW | RTLD_GLOBAL);                 // the older tools' library
            if (!h) h = dlopen("libroctx64.so", RTLD_NOW | RTLD_GLOBAL);
            if (!h) return;
            p_push = (push_fn)dlsym(h, "roctxRangePushA");
            p_pop = (pop_fn)dlsym(h, "roctxRangePop");
            if (!p_push || !p_pop) p_push = nullptr, p_pop = nullptr;
        });
        push = p_push;
        pop = p_pop;
    }
    pop_fn pop_;
    explicit TraceRange(const char* fmt, int arg = 0) : pop_(nullptr) {
        push_fn push;
        lookup(push, pop_);
        if (!push) { pop_ = nullptr; return; }
        char name[64];
        snprintf(name, sizeof(name), fmt, arg);
        push(name);
    }
    ~TraceRange() { if (pop_) pop_(); }
};
static constexpr int64_t kTensorAlign = 256;   // elements
static constexpr int kDefaultSweeps = 1;       // update + perturb sweeps per block when the budget leaves the choice
static constexpr int kFuseMaxTokens = 64;      // up to this many tokens per stream the projections perturb in their weight loader (measured, OPT-1.3B shape: steps 1.06 - 1.23x faster up to 64 tokens, 0.96x at 80, 0.93x at 128)

static bool config_ok(const zo2_config* c, char* why, size_t n) {
#define BAD(...) do { snprintf(why, n, __VA_ARGS__); return false; } while (0)
    if (!c) BAD("config is NULL");
    if (c->n_layers < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->d_ffn <= 0 || c->vocab <= 0 || c->max_pos <= 0 || c->pos_offset < 0)
        BAD("non-positive model dimension");
    if (c->d_model % 8 || c->d_ffn % 8) BAD("d_model (%d) and d_ffn (%d) must be multiples of 8", c->d_model, c->d_ffn);
    if (c->d_model % c->n_heads) BAD("n_heads %d does not divide d_model %d", c->n_heads, c->d_model);
    const int dh = c->d_model / c->n_heads;
    if (!(dh == 8 || dh == 16 || dh == 32 || dh == 64 || dh == 80 || dh == 128)) BAD("head dimension %d not in {8,16,32,64,80,128}", dh);
    if (zo2_dtype_size(c->wire_dtype) == 0) BAD("unknown wire dtype %d", c->wire_dtype);
    if (!(c->compute_dtype == ZO2_F32 || c->compute_dtype == ZO2_BF16 || c->compute_dtype == ZO2_F16))
        BAD("compute dtype %d is not F32, BF16 or F16", c->compute_dtype);
    if (!(c->ln_eps > 0.f)) BAD("ln_eps must be positive");
    return true;
#undef BAD
}

static void block_tensor_elems(const zo2_config* c, int64_t n[ZO2_BLOCK_TENSORS]) {
    const int64_t d = c->d_model, f = c->d_ffn;
    const int64_t v[ZO2_BLOCK_TENSORS] = {d, d, d * d, d, d * d, d, d * d, d, d * d, d, d, d, f * d, f, d * f, d};
    for (int i = 0; i < ZO2_BLOCK_TENSORS; ++i) n[i] = v[i];
}

}  // namespace zo2

using namespace zo2;

// =========================================================================================
// context
// =========================================================================================
struct zo2_ctx {
    zo2_config cfg;
    zo2_device dev;
    std::vector<void*> host_bucket;
    void *h_tok, *h_pos, *h_flnw, *h_flnb, *h_lm;
    std::vector<float> scales;          // per tensor id
    char err[512];
    bool dead;
    size_t budget;

    // layout
    int64_t offs[ZO2_BLOCK_TENSORS + 1];
    int64_t tn[ZO2_BLOCK_TENSORS];
    size_t wsz, csz;                    // bytes per element: wire, compute
    size_t bucket_bytes;
    int64_t tok_elems, pos_elems, fln_off_b, fln_elems;   // final LN mini bucket: w at 0, b at fln_off_b
    int n_tensors;

    // persistent device region
    char *d_tok, *d_pos, *d_fln, *d_lm;
    float* d_state;                     // [4..7] result of a pass, [16 + k] coefficient eta g of deferred update k
    size_t persistent_bytes;

    // plan (depends on budget and batch x seq)
    bool planned, need_plan;
    int plan_T, plan_seq;
    bool resident;
    int sweeps;                         // update + perturb sweeps per block: 1 (whole-block scratch), 2 (per half) or 4 (per tensor group)
    int pb[5];                          // sweep p, issued at point p of the block's forward, covers tensors pb[p] .. pb[p + 1] - 1 (may be empty)
    int scratch_plan_forced;            // 0: the planner chooses; 1 / 2 / 4: that many sweeps per block
    int loader_fusion;                  // 0: for few tokens per step (kFuseMaxTokens); 1: whenever the shapes allow; -1: never
    int split_k;                        // 0: projections that leave most compute units idle are split along k; -1: never
    bool fuse;                          // this plan: the projections of a block perturb in their weight loader (step passes only)
    char* sk_ws;                        // their workspace (float32 partial sums of the k slices)
    size_t sk_ws_bytes;
    int n_slots;
    char* slots;
    char *wp, *wm;                      // W+ / W- scratch in use (compute dtype)
    char *wps[2], *wms[2];              // the scratch sets; two when K1 of block l+1 may overlap the forwards of block l
    bool overlap_k1;
    hipStream_t sk;                     // optional fourth stream for that overlap
    hipEvent_t ev_k1done[2], ev_fwd_done[2], ev_embed;
    int64_t scratch_elems;
    char *fln_wp, *fln_wm;
    float* h;
    char *x, *qb, *kb, *vb, *ctxb, *mid;
    float* logits;
    int logit_rows;                     // rows per sign per chunk
    bool fused_ce;                      // LM head writes cross-entropy partials instead of logits
    bool stochastic;                     // theta' is stored with stochastic rounding (low-bit wire formats)
    bool serial_streams;                 // ablation: upload, compute and offload of a block run one after the other
    int ns;                              // perturbation streams of the pass in progress: 2 (step) or 1 (evaluation)
    float *ce_pmax, *ce_psum, *ce_lab;  // [4 ceil(V/256), 2T] x 2 and [2T]
    int ce_parts;
    float* row_loss;
    int32_t *d_tokens, *d_labels;
    size_t bytes_used;
    bool blocks_on_device;

    // deferred updates (Sec. 5.4): none, one (the paper's case), or the directions of one round of the q-direction
    // estimator (zo2_step_extra), in the order in which they are applied.  Coefficient k sits at d_state[16 + k].
    static constexpr int kMaxPending = 16;
    int n_pend;
    uint64_t pend_seed[kMaxPending];
    bool apply_now;                      // the pass in progress applies them (false: a further direction at unchanged parameters)
    // Several directions in one pass (zo2_step_multi): every direction keeps its own residual stream; inside a module the
    // first direction applies the deferred updates, the later ones find the parameters final.
    float* hs[kMaxPending];              // residual streams of the directions (hs[0] is the only one of an ordinary pass)
    int plan_dirs, want_dirs;            // residual streams the plan holds / asked for
    bool dir_later;                      // the direction in progress is not the first of its pass
    // Streamed blocks with a write-back interval above one: updates already applied wherever parameters stay on the device
    // (embeddings, head) that the host copies of the blocks still lack.  Every upload of a block replays them, in order,
    // before anything else; coefficient k sits at d_state[32 + k].  Empty whenever the blocks are resident.
    static constexpr int kMaxStale = 32;
    int wb_interval;                     // a block is written back once its host copy would lack this many updates (1: after every update, as in Alg. 2)
    int n_stale;
    uint64_t stale_seed[kMaxStale];
    bool pass_writes_back;               // decided at the start of a pass

    // streams / events
    hipStream_t sc, su, so;
    std::vector<hipEvent_t> ev_up, ev_k1, ev_free, ev_read;
    std::vector<char> ev_free_valid, ev_read_valid;    // ev_read: the forwards that read the slot itself (loader fusion) are done
    hipEvent_t ev_step0, ev_c1, ev_u0, ev_u1, ev_o0, ev_o1;
    bool stat_u, stat_o;
    uint64_t bytes_up, bytes_down;
    float ms_c, ms_u, ms_o;

    uint32_t debug_delay_us[3];         // test aid: idle time inserted before each block's work on compute / upload / offload
    bool debug_poison;                  // test aid: a slot is filled with 0xFF bytes (NaN in every format) before each upload into it

    // optional per-kernel-class timing with events on the compute stream
    uint32_t prof_mask;
    std::vector<hipEvent_t> prof_ev;    // pairs (begin, end)
    std::vector<int> prof_cls;
    size_t prof_used;
    float prof_ms[ZO2_KERNEL_CLASSES];
    int32_t prof_launches[ZO2_KERNEL_CLASSES];

    // pinned staging
    int32_t* h_ids;                     // tokens then labels
    int h_ids_cap;
    float* h_result;
};

static zo2_status fail(zo2_ctx* c, zo2_status s, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, sizeof(c->err), fmt, ap);
    va_end(ap);
    if (s == ZO2_EHIP) c->dead = true;
    return s;
}
#define HIPCHK(c, call)                                                                        \
    do {                                                                                       \
        hipError_t e__ = (call);                                                               \
        if (e__ != hipSuccess) return fail(c, ZO2_EHIP, "%s failed: %s", #call, hipGetErrorString(e__)); \
    } while (0)
#define OPCHK(c, call)                                                       \
    do {                                                                     \
        zo2_status s__ = (call);                                             \
        if (s__ != ZO2_OK) return fail(c, s__, "%s", zo2_op_last_error());   \
    } while (0)

// Bracket one launch with a pair of events when its class is being profiled.
struct ProfScope {
    zo2_ctx* c;
    int cls;
    bool on;
    hipStream_t st;
    ProfScope(zo2_ctx* c_, int cls_, hipStream_t st_ = nullptr) : c(c_), cls(cls_), on((c_->prof_mask >> cls_) & 1u), st(st_ ? st_ : c_->sc) {
        if (!on) return;
        if (c->prof_used + 2 > c->prof_ev.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
            c->prof_ev.push_back(a);
            c->prof_ev.push_back(b);
        }
        (void)hipEventRecord(c->prof_ev[c->prof_used], st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(c->prof_ev[c->prof_used + 1], st);
        c->prof_cls.push_back(cls);
        c->prof_used += 2;
    }
};
static void prof_reset(zo2_ctx* c) {
    c->prof_used = 0;
    c->prof_cls.clear();
    for (int i = 0; i < ZO2_KERNEL_CLASSES; ++i) { c->prof_ms[i] = 0.f; c->prof_launches[i] = 0; }
}
static void prof_collect(zo2_ctx* c) {   // after the compute stream has been synchronised
    for (size_t i = 0; i < c->prof_cls.size(); ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]) == hipSuccess) {
            c->prof_ms[c->prof_cls[i]] += ms;
            c->prof_launches[c->prof_cls[i]] += 1;
        }
    }
}
#define OPKS(c, cls, stream, call)                                           \
    do {                                                                     \
        zo2_status s__;                                                      \
        {                                                                    \
            ProfScope ps__(c, cls, stream);                                  \
            s__ = (call);                                                    \
        }                                                                    \
        if (s__ != ZO2_OK) return fail(c, s__, "%s", zo2_op_last_error());   \
    } while (0)
#define OPK(c, cls, call)                                                    \
    do {                                                                     \
        zo2_status s__;                                                      \
        {                                                                    \
            ProfScope ps__(c, cls);                                          \
            s__ = (call);                                                    \
        }                                                                    \
        if (s__ != ZO2_OK) return fail(c, s__, "%s", zo2_op_last_error());   \
    } while (0)

// Test aid for the scheduler: a kernel that idles for a bounded time on one stream, so that a test can make
// any of the three streams arbitrarily slow; with correct event dependencies the results cannot change.
__global__ void delay_kernel(unsigned long long ticks_100mhz) {
    const unsigned long long t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks_100mhz) { __builtin_amdgcn_s_sleep(32); }
}
__global__ void poison_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0xffffffffu;
}
static zo2_status debug_delay(zo2_ctx* c, int which, hipStream_t st) {
    const uint32_t us = c->debug_delay_us[which];
    if (us == 0) return ZO2_OK;
    hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(1), 0, st, (unsigned long long)us * 100ull);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, ZO2_EHIP, "delay kernel: %s", hipGetErrorString(e));
    return ZO2_OK;
}

static inline uint32_t block_tid(int l, int k) { return (uint32_t)(2 + 16 * l + k); }
static inline uint32_t fln_tid(const zo2_ctx* c) { return (uint32_t)(2 + 16 * c->cfg.n_layers); }
static inline uint32_t lm_tid(const zo2_ctx* c) { return (uint32_t)(4 + 16 * c->cfg.n_layers); }

extern "C" size_t zo2_dtype_size(int32_t dt) {
    switch (dt) {
        case ZO2_F32: return 4;
        case ZO2_BF16: case ZO2_F16: return 2;
        case ZO2_FP8_E4M3: case ZO2_FP8_E5M2: return 1;
        default: return 0;
    }
}

extern "C" zo2_status zo2_block_tensor_offsets(const zo2_config* cfg, int64_t offs[ZO2_BLOCK_TENSORS + 1]) {
    char why[256];
    if (!offs || !config_ok(cfg, why, sizeof(why))) {
        set_op_error("%s", offs ? why : "offs is NULL");
        return ZO2_EINVAL;
    }
    int64_t n[ZO2_BLOCK_TENSORS];
    block_tensor_elems(cfg, n);
    int64_t o = 0;
    for (int i = 0; i < ZO2_BLOCK_TENSORS; ++i) {
        offs[i] = o;
        o += (n[i] + kTensorAlign - 1) / kTensorAlign * kTensorAlign;
    }
    offs[ZO2_BLOCK_TENSORS] = o;
    return ZO2_OK;
}

extern "C" const char* zo2_op_last_error(void) { return g_op_error; }
extern "C" const char* zo2_last_error(const zo2_ctx* c) { return c ? c->err : "context is NULL"; }

// ---------------------------------------------------------------------------------- init
extern "C" zo2_status zo2_init(zo2_ctx** out, const zo2_config* cfg, const zo2_host_weights* w, const zo2_device* dev) {
    if (!out) return ZO2_EINVAL;
    *out = nullptr;
    char why[256];
    if (!config_ok(cfg, why, sizeof(why))) { set_op_error("%s", why); return ZO2_EINVAL; }
    if (!w || !dev || !w->tok_emb || !w->pos_emb || !w->final_ln_w || !w->final_ln_b || (cfg->n_layers > 0 && !w->block_bucket)) {
        set_op_error("zo2_init: NULL weight or device argument");
        return ZO2_EINVAL;
    }
    if ((cfg->tied_lm_head != 0) != (w->lm_head == nullptr)) {
        set_op_error("zo2_init: lm_head must be NULL exactly when tied_lm_head = 1");
        return ZO2_EINVAL;
    }
    if (!dev->arena || ((uintptr_t)dev->arena & 255) || dev->arena_bytes == 0) {
        set_op_error("zo2_init: arena must be non-NULL and 256-byte aligned");
        return ZO2_EINVAL;
    }
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->block_bucket[l]) { set_op_error("zo2_init: block_bucket[%d] is NULL", l); return ZO2_EINVAL; }

    zo2_ctx* c = new (std::nothrow) zo2_ctx();
    if (c) c->ns = 2;
    if (!c) { set_op_error("zo2_init: out of host memory"); return ZO2_ENOMEM; }
    c->cfg = *cfg;
    c->dev = *dev;
    c->err[0] = 0;
    c->dead = false;
    c->budget = dev->arena_bytes;
    c->host_bucket.assign(w->block_bucket, w->block_bucket + cfg->n_layers);
    c->h_tok = w->tok_emb; c->h_pos = w->pos_emb; c->h_flnw = w->final_ln_w; c->h_flnb = w->final_ln_b; c->h_lm = w->lm_head;
    c->n_tensors = 4 + 16 * cfg->n_layers + (cfg->tied_lm_head ? 0 : 1);
    c->scales.assign(c->n_tensors, 1.0f);
    const bool wire8 = zo2_dtype_size(cfg->wire_dtype) == 1;
    if (w->tensor_scale) {
        for (int i = 0; i < c->n_tensors; ++i) {
            const float s = w->tensor_scale[i];
            int ex = 0;
            if (!(s > 0.f) || !isfinite(s) || frexpf(s, &ex) != 0.5f || (!wire8 && s != 1.0f)) {
                set_op_error("zo2_init: tensor_scale[%d] = %g is invalid for this wire dtype (a power of two; 1 unless the format has 8 bits)", i, (double)s);
                delete c;
                return ZO2_EINVAL;
            }
            c->scales[i] = s;
        }
    }
    zo2_block_tensor_offsets(cfg, c->offs);
    block_tensor_elems(cfg, c->tn);
    c->wsz = zo2_dtype_size(cfg->wire_dtype);
    c->csz = zo2_dtype_size(cfg->compute_dtype);
    c->bucket_bytes = (size_t)c->offs[ZO2_BLOCK_TENSORS] * c->wsz;
    c->tok_elems = (int64_t)cfg->vocab * cfg->d_model;
    c->pos_elems = (int64_t)(cfg->max_pos + cfg->pos_offset) * cfg->d_model;
    c->fln_off_b = align_up(cfg->d_model, kTensorAlign);
    c->fln_elems = 2 * c->fln_off_b;
    c->sc = as_stream(dev->stream_compute);
    c->su = as_stream(dev->stream_upload);
    c->so = as_stream(dev->stream_offload);
    c->sk = as_stream(dev->stream_k1);
    c->overlap_k1 = false;
    c->planned = false;
    c->need_plan = false;
    c->blocks_on_device = false;
    c->n_pend = 0;
    c->apply_now = true;
    c->wb_interval = 1;
    c->n_stale = 0;
    c->pass_writes_back = true;
    c->h_ids = nullptr;
    c->h_ids_cap = 0;
    c->h_result = nullptr;
    c->plan_dirs = 0; c->want_dirs = 1; c->dir_later = false;
    for (float*& hp : c->hs) hp = nullptr;
    c->bytes_up = c->bytes_down = 0;
    c->ms_c = c->ms_u = c->ms_o = 0.f;
    c->bytes_used = 0;
    c->debug_delay_us[0] = c->debug_delay_us[1] = c->debug_delay_us[2] = 0;
    c->prof_mask = 0;
    prof_reset(c);
    c->n_slots = 0;
    c->resident = false;
    c->sweeps = 1;
    c->scratch_plan_forced = 0;
    c->loader_fusion = 0;
    c->split_k = 0;
    c->fuse = false;
    c->scratch_elems = 0;
    *out = c;   // from here on errors are reported through the context

    // persistent region: embeddings, final LayerNorm, LM head, state
    char* base = (char*)dev->arena;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base + off; off = align_up(off + bytes, 256); return p; };
    c->d_tok = take((size_t)c->tok_elems * c->wsz);
    c->d_pos = take((size_t)c->pos_elems * c->wsz);
    c->d_fln = take((size_t)c->fln_elems * c->wsz);
    c->d_lm = cfg->tied_lm_head ? nullptr : take((size_t)c->tok_elems * c->wsz);
    c->d_state = (float*)take(64 * sizeof(float));
    c->persistent_bytes = off;
    if (off > dev->arena_bytes) return fail(c, ZO2_ENOMEM, "arena of %zu bytes cannot hold the %zu bytes of embeddings", dev->arena_bytes, off);

    HIPCHK(c, hipMemcpy(c->d_tok, w->tok_emb, (size_t)c->tok_elems * c->wsz, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->d_pos, w->pos_emb, (size_t)c->pos_elems * c->wsz, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemset(c->d_fln, 0, (size_t)c->fln_elems * c->wsz));
    HIPCHK(c, hipMemcpy(c->d_fln, w->final_ln_w, (size_t)cfg->d_model * c->wsz, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(c->d_fln + (size_t)c->fln_off_b * c->wsz, w->final_ln_b, (size_t)cfg->d_model * c->wsz, hipMemcpyHostToDevice));
    if (c->d_lm) HIPCHK(c, hipMemcpy(c->d_lm, w->lm_head, (size_t)c->tok_elems * c->wsz, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemset(c->d_state, 0, 64 * sizeof(float)));
    HIPCHK(c, hipHostMalloc((void**)&c->h_result, (16 + 4 * zo2_ctx::kMaxPending) * sizeof(float), hipHostMallocDefault));
    hipEvent_t* evs[] = {&c->ev_step0, &c->ev_c1, &c->ev_u0, &c->ev_u1, &c->ev_o0, &c->ev_o1};
    for (hipEvent_t* e : evs) HIPCHK(c, hipEventCreate(e));
    hipEvent_t* evs2[] = {&c->ev_k1done[0], &c->ev_k1done[1], &c->ev_fwd_done[0], &c->ev_fwd_done[1], &c->ev_embed};
    for (hipEvent_t* e : evs2) HIPCHK(c, hipEventCreateWithFlags(e, hipEventDisableTiming));
    return ZO2_OK;
}

static zo2_status writeback_pass(zo2_ctx* c);

extern "C" void zo2_destroy(zo2_ctx* c) {
    if (!c) return;
    if (!c->dead) (void)writeback_pass(c);       // the caller's block buffers are left current (best effort: no status to report)
    hipStreamSynchronize(c->sc);
    hipStreamSynchronize(c->su);
    hipStreamSynchronize(c->so);
    if (c->sk) hipStreamSynchronize(c->sk);
    for (auto e : c->ev_up) hipEventDestroy(e);
    for (auto e : c->ev_k1) hipEventDestroy(e);
    for (auto e : c->ev_free) hipEventDestroy(e);
    for (auto e : c->ev_read) hipEventDestroy(e);
    for (auto e : c->prof_ev) hipEventDestroy(e);
    hipEvent_t evs[] = {c->ev_step0, c->ev_c1, c->ev_u0, c->ev_u1, c->ev_o0, c->ev_o1, c->ev_k1done[0], c->ev_k1done[1], c->ev_fwd_done[0], c->ev_fwd_done[1], c->ev_embed};
    if (c->h_result) for (hipEvent_t e : evs) hipEventDestroy(e);
    if (c->h_ids) hipHostFree(c->h_ids);
    if (c->h_result) hipHostFree(c->h_result);
    delete c;
}

extern "C" zo2_status zo2_set_resident_budget(zo2_ctx* c, size_t hbm_bytes) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (hbm_bytes == 0) return fail(c, ZO2_EINVAL, "budget must be positive");
    c->budget = hbm_bytes < c->dev.arena_bytes ? hbm_bytes : c->dev.arena_bytes;
    c->need_plan = true;   // re-plan at the next step
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- sync to host
static zo2_status sync_blocks_to_host(zo2_ctx* c) {
    if (c->resident && c->blocks_on_device) {
        HIPCHK(c, hipStreamSynchronize(c->sc));
        for (int l = 0; l < c->cfg.n_layers; ++l)
            HIPCHK(c, hipMemcpy(c->host_bucket[l], c->slots + (size_t)l * c->bucket_bytes, c->bucket_bytes, hipMemcpyDeviceToHost));
    }
    return ZO2_OK;
}

extern "C" zo2_status zo2_sync_to_host(zo2_ctx* c) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    { zo2_status s = writeback_pass(c); if (s != ZO2_OK) return s; }
    HIPCHK(c, hipStreamSynchronize(c->sc));
    HIPCHK(c, hipStreamSynchronize(c->so));
    const size_t d = c->cfg.d_model;
    HIPCHK(c, hipMemcpy(c->h_tok, c->d_tok, (size_t)c->tok_elems * c->wsz, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(c->h_pos, c->d_pos, (size_t)c->pos_elems * c->wsz, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(c->h_flnw, c->d_fln, d * c->wsz, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(c->h_flnb, c->d_fln + (size_t)c->fln_off_b * c->wsz, d * c->wsz, hipMemcpyDeviceToHost));
    if (c->d_lm) HIPCHK(c, hipMemcpy(c->h_lm, c->d_lm, (size_t)c->tok_elems * c->wsz, hipMemcpyDeviceToHost));
    return sync_blocks_to_host(c);
}

// ---------------------------------------------------------------------------------- planning
// The W+ / W- scratch holds the perturbed copies of the tensors one sweep of K1 writes.  The forward of a block needs
// them at four points: {ln1, q, k, v} before the QKV projection, {o} before the output projection, {ln2, fc1} before the
// first FFN projection, {fc2} before the second.  Three organisations: one sweep over the whole block at point 0; two
// sweeps (attention half at point 0, FFN half at point 2); four sweeps (one per group).  Fewer tensors per sweep = a
// smaller scratch, and the copies are consumed right after they are written, while they still sit in the memory-side
// cache; more sweeps = more, shorter launches.
static const int kSweepBounds[3][5] = {{0, 16, 16, 16, 16}, {0, 10, 10, 16, 16}, {0, 8, 10, 14, 16}};
static inline const int* sweep_bounds(int sweeps) { return kSweepBounds[sweeps == 1 ? 0 : sweeps == 2 ? 1 : 2]; }

static zo2_status plan(zo2_ctx* c, int T, int batch, int seq) {
    const zo2_config& g = c->cfg;
    // a new layout starts from current host copies of the blocks (it may make them resident)
    { zo2_status s = writeback_pass(c); if (s != ZO2_OK) return s; }
    const size_t d = g.d_model, f = g.d_ffn, V = g.vocab;
    const size_t budget = c->budget;
    const size_t rows2 = 2 * (size_t)T;
    // logits chunk (float32 mode and shapes the fused LM-head + cross-entropy kernel does not take): up to 1/8 of the
    // budget, at least 128 rows per sign
    const bool fused_ce = (g.compute_dtype != ZO2_F32) && T >= 256 && V >= 256 && (d % 128 == 0) && (V % 4 == 0);
    const size_t ce_parts = 4 * ((V + 255) / 256);
    size_t lrows = budget / 8 / (V * 4) / 2;
    lrows = lrows / 128 * 128;
    if (lrows < 128) lrows = 128;
    if (lrows > (size_t)T) lrows = T;
    // few tokens per step: the block projections read the stored weights and perturb in their loader (16-bit storage
    // that is also the compute format, no wire scale)
    const bool fuse_shapes = g.wire_dtype == g.compute_dtype && g.compute_dtype != ZO2_F32 && T <= 256 && d % 64 == 0 && f % 64 == 0 &&
                             (size_t)T * f * 2 < 0xffffffffull;
    const bool fuse = fuse_shapes && c->loader_fusion >= 0 && (c->loader_fusion == 1 || T <= kFuseMaxTokens) && !c->sk;
    size_t sk_ws_bytes = 0;
    if (fuse) {
        sk_ws_bytes = std::max(std::max(skinny_workspace_bytes(T, (int)d, (int)d, 3), skinny_workspace_bytes(T, (int)d, (int)d, 1)),
                               std::max(skinny_workspace_bytes(T, (int)f, (int)d, 1), skinny_workspace_bytes(T, (int)d, (int)f, 1)));
    }
    if (c->split_k >= 0 && g.compute_dtype != ZO2_F32) {      // split-k partial sums of the block projections (steps and single forwards)
        for (int ns_ = 1; ns_ <= 2; ++ns_) {
            const int shapes[4][3] = {{(int)d, (int)d, 3 * ns_}, {(int)d, (int)d, ns_}, {(int)f, (int)d, ns_}, {(int)d, (int)f, ns_}};      // N, K, problems
            for (const auto& sh : shapes)
                sk_ws_bytes = std::max(sk_ws_bytes, gemm_splitk_workspace_bytes(T, sh[0], sh[2], gemm_pick_splits(T, sh[0], sh[1], sh[2], g.compute_dtype)));
        }
    }
    size_t act = 0;
    auto sz = [&](size_t bytes) { size_t o = act; act = align_up(act + bytes, 256); return o; };
    const int n_dirs = std::max(1, c->want_dirs);
    const size_t h_bytes = align_up(rows2 * d * 4, 256);
    const size_t o_h = sz(h_bytes * n_dirs), o_x = sz(rows2 * d * c->csz), o_q = sz(rows2 * d * c->csz), o_k = sz(rows2 * d * c->csz),
                 o_v = sz(rows2 * d * c->csz), o_ctx = sz(rows2 * d * c->csz), o_mid = sz(rows2 * f * c->csz),
                 o_logits = sz(fused_ce ? 0 : 2 * lrows * V * 4), o_rl = sz(rows2 * 4),
                 o_cpm = sz(fused_ce ? rows2 * ce_parts * 4 : 0), o_cps = sz(fused_ce ? rows2 * ce_parts * 4 : 0), o_cl = sz(fused_ce ? rows2 * 4 : 0), o_tok = sz((size_t)T * 4), o_lab = sz((size_t)T * 4),
                 o_fwp = sz((size_t)c->fln_elems * c->csz), o_fwm = sz((size_t)c->fln_elems * c->csz), o_skws = sz(sk_ws_bytes);
    const size_t act_bytes = act;

    const int64_t head_elems = (int64_t)align_up(c->tok_elems, kTensorAlign);
    auto scratch_for = [&](int sweeps) {
        const int* pb = sweep_bounds(sweeps);
        int64_t m = 0;
        for (int p = 0; p < 4; ++p) m = std::max(m, c->offs[pb[p + 1]] - c->offs[pb[p]]);
        return std::max(m, head_elems);
    };
    bool resident = false, two_sets = false;
    int sweeps = 1;
    int64_t scratch = 0;
    long slots = 0;
    // preference: two whole-block scratch sets (K1 of the next block overlaps this block's forwards) when a stream for
    // it was given, then the default organisation, then ever smaller scratch sets until 3 block slots fit
    const int forced = c->scratch_plan_forced;
    const int first = forced ? forced : kDefaultSweeps;
    for (int attempt = (c->sk && !forced ? 0 : 1); attempt < 4; ++attempt) {
        two_sets = attempt == 0;
        sweeps = attempt == 0 ? 1 : attempt == 1 ? first : attempt == 2 ? std::max(first, 2) : 4;
        scratch = scratch_for(sweeps);
        const size_t fixed = c->persistent_bytes + act_bytes + (two_sets ? 4 : 2) * align_up((size_t)scratch * c->csz, 256);
        slots = fixed > budget ? -1 : (long)((budget - fixed) / align_up(c->bucket_bytes, 256));
        if (slots >= g.n_layers || slots >= 3 || forced) break;      // a forced organisation is not traded for a smaller one
    }
    if (g.n_layers > 0 && slots < g.n_layers && slots < 3)
        return fail(c, ZO2_EBUDGET, "budget of %zu bytes cannot hold embeddings + 3 block slots + scratch + activations for %d tokens", budget, T);
    resident = slots >= g.n_layers;
    const int n_slots = resident ? g.n_layers : (int)slots;

    // moving between resident and streamed (or resizing the ring) needs the host copy current
    if (c->planned && c->resident && c->blocks_on_device && !resident) {
        zo2_status s = sync_blocks_to_host(c);
        if (s != ZO2_OK) return s;
        c->blocks_on_device = false;
    }
    HIPCHK(c, hipStreamSynchronize(c->sc));
    HIPCHK(c, hipStreamSynchronize(c->su));
    HIPCHK(c, hipStreamSynchronize(c->so));
    if (c->sk) HIPCHK(c, hipStreamSynchronize(c->sk));

    char* base = (char*)c->dev.arena;
    size_t off = c->persistent_bytes;
    c->slots = base + off;
    off += (size_t)n_slots * align_up(c->bucket_bytes, 256);
    for (int k = 0; k < (two_sets ? 2 : 1); ++k) {
        c->wps[k] = base + off; off += align_up((size_t)scratch * c->csz, 256);
        c->wms[k] = base + off; off += align_up((size_t)scratch * c->csz, 256);
    }
    if (!two_sets) { c->wps[1] = c->wps[0]; c->wms[1] = c->wms[0]; }
    c->wp = c->wps[0]; c->wm = c->wms[0];
    c->overlap_k1 = two_sets;
    char* a0 = base + off;
    for (int j = 0; j < zo2_ctx::kMaxPending; ++j) c->hs[j] = j < n_dirs ? (float*)(a0 + o_h + (size_t)j * h_bytes) : nullptr;
    c->plan_dirs = n_dirs;
    c->h = c->hs[0]; c->x = a0 + o_x; c->qb = a0 + o_q; c->kb = a0 + o_k; c->vb = a0 + o_v; c->ctxb = a0 + o_ctx;
    c->mid = a0 + o_mid; c->logits = (float*)(a0 + o_logits); c->row_loss = (float*)(a0 + o_rl);
    c->d_tokens = (int32_t*)(a0 + o_tok); c->d_labels = (int32_t*)(a0 + o_lab);
    c->fln_wp = a0 + o_fwp; c->fln_wm = a0 + o_fwm;
    c->fuse = fuse; c->sk_ws = a0 + o_skws; c->sk_ws_bytes = sk_ws_bytes;
    c->fused_ce = fused_ce; c->ce_parts = (int)ce_parts;
    c->ce_pmax = (float*)(a0 + o_cpm); c->ce_psum = (float*)(a0 + o_cps); c->ce_lab = (float*)(a0 + o_cl);
    off += act_bytes;
    c->bytes_used = off;
    c->logit_rows = (int)lrows;
    c->scratch_elems = scratch;
    c->sweeps = sweeps;
    for (int p = 0; p < 5; ++p) c->pb[p] = sweep_bounds(sweeps)[p];
    if (c->bucket_bytes % 256) return fail(c, ZO2_EINVAL, "internal: bucket size not aligned");

    // events per slot
    while ((int)c->ev_up.size() < n_slots) {
        hipEvent_t e1, e2, e3, e4;
        HIPCHK(c, hipEventCreateWithFlags(&e1, hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&e2, hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&e3, hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&e4, hipEventDisableTiming));
        c->ev_up.push_back(e1); c->ev_k1.push_back(e2); c->ev_free.push_back(e3); c->ev_read.push_back(e4);
    }
    c->ev_free_valid.assign(c->ev_up.size(), 0);
    c->ev_read_valid.assign(c->ev_up.size(), 0);

    if (resident && !(c->planned && c->resident && c->blocks_on_device && c->n_slots == n_slots)) {
        for (int l = 0; l < g.n_layers; ++l)
            HIPCHK(c, hipMemcpy(c->slots + (size_t)l * c->bucket_bytes, c->host_bucket[l], c->bucket_bytes, hipMemcpyHostToDevice));
        c->blocks_on_device = true;
    }
    if (!resident) c->blocks_on_device = false;
    c->resident = resident;
    c->n_slots = n_slots;
    c->plan_T = T;
    c->plan_seq = seq;
    c->planned = true;
    c->need_plan = false;

    if (c->h_ids_cap < 2 * T) {
        if (c->h_ids) hipHostFree(c->h_ids);
        c->h_ids = nullptr;
        HIPCHK(c, hipHostMalloc((void**)&c->h_ids, (size_t)2 * T * sizeof(int32_t), hipHostMallocDefault));
        c->h_ids_cap = 2 * T;
    }
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_plan(const zo2_ctx* c, int32_t* n_slots, int32_t* resident, size_t* bytes_used) {
    if (!c) return ZO2_EINVAL;
    if (n_slots) *n_slots = c->n_slots;
    if (resident) *resident = c->resident ? 1 : 0;
    if (bytes_used) *bytes_used = c->planned ? c->bytes_used : c->persistent_bytes;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_scratch_plan(const zo2_ctx* c, int32_t* sweeps_per_block, int64_t* scratch_elems, int32_t* scratch_sets) {
    if (!c) return ZO2_EINVAL;
    if (sweeps_per_block) *sweeps_per_block = c->planned ? c->sweeps : 0;
    if (scratch_elems) *scratch_elems = c->planned ? c->scratch_elems : 0;
    if (scratch_sets) *scratch_sets = c->planned ? (c->overlap_k1 ? 2 : 1) : 0;
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_scratch_plan(zo2_ctx* c, int32_t mode) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (mode != 0 && mode != 1 && mode != 2 && mode != 4) return fail(c, ZO2_EINVAL, "zo2_set_scratch_plan: %d sweeps per block (0, 1, 2 or 4)", mode);
    c->scratch_plan_forced = mode;
    c->need_plan = true;   // re-plan at the next step
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_loader_fusion(zo2_ctx* c, int32_t mode) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (mode < -1 || mode > 1) return fail(c, ZO2_EINVAL, "zo2_set_loader_fusion: mode %d (-1, 0 or 1)", mode);
    c->loader_fusion = mode;
    c->need_plan = true;   // re-plan at the next step
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_split_k(zo2_ctx* c, int32_t mode) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (mode < -1 || mode > 0) return fail(c, ZO2_EINVAL, "zo2_set_split_k: mode %d (-1 or 0)", mode);
    c->split_k = mode;
    c->need_plan = true;   // re-plan at the next step
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_writeback_interval(zo2_ctx* c, int32_t updates) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (updates < 1 || updates > zo2_ctx::kMaxStale - zo2_ctx::kMaxPending)
        return fail(c, ZO2_EINVAL, "zo2_set_writeback_interval: %d (1 .. %d)", updates, zo2_ctx::kMaxStale - zo2_ctx::kMaxPending);
    c->wb_interval = updates;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_writeback_state(const zo2_ctx* c, int32_t* interval, int32_t* lacking) {
    if (!c || !interval || !lacking) return ZO2_EINVAL;
    *interval = c->wb_interval;
    *lacking = c->n_stale;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_loader_fusion(const zo2_ctx* c, int32_t* active) {
    if (!c || !active) return ZO2_EINVAL;
    *active = (c->planned && c->fuse) ? 1 : 0;
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_profiling(zo2_ctx* c, uint32_t class_mask) {
    if (!c) return ZO2_EINVAL;
    c->prof_mask = class_mask & ((1u << ZO2_KERNEL_CLASSES) - 1);
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_kernel_times(const zo2_ctx* c, float ms[ZO2_KERNEL_CLASSES], int32_t launches[ZO2_KERNEL_CLASSES]) {
    if (!c) return ZO2_EINVAL;
    for (int i = 0; i < ZO2_KERNEL_CLASSES; ++i) {
        if (ms) ms[i] = c->prof_ms[i];
        if (launches) launches[i] = c->prof_launches[i];
    }
    return ZO2_OK;
}

extern "C" zo2_status zo2_debug_set_slot_poison(zo2_ctx* c, int32_t enabled) {
    if (!c) return ZO2_EINVAL;
    c->debug_poison = enabled != 0;
    return ZO2_OK;
}

extern "C" zo2_status zo2_debug_set_stream_delay(zo2_ctx* c, int32_t which, uint32_t microseconds) {
    if (!c || which < 0 || which > 2 || microseconds > 100000u) return ZO2_EINVAL;
    c->debug_delay_us[which] = microseconds;
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_wire_rounding(zo2_ctx* c, int32_t stochastic) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    c->stochastic = stochastic != 0;
    return ZO2_OK;
}

extern "C" zo2_status zo2_set_stream_overlap(zo2_ctx* c, int32_t enabled) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    c->serial_streams = enabled == 0;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_step_stats(const zo2_ctx* c, float* ms_c, float* ms_u, float* ms_o, uint64_t* up, uint64_t* down) {
    if (!c) return ZO2_EINVAL;
    if (ms_c) *ms_c = c->ms_c;
    if (ms_u) *ms_u = c->ms_u;
    if (ms_o) *ms_o = c->ms_o;
    if (up) *up = c->bytes_up;
    if (down) *down = c->bytes_down;
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- K1 helpers
static inline float* coef_slot(const zo2_ctx* c, int k) { return c->d_state + 16 + k; }
// does the fused sweep (update + perturb) of the pass in progress carry an update?  It carries the last deferred one;
// the earlier ones of a round of several directions are applied by update-only sweeps in front of it.
static inline bool fused_update(const zo2_ctx* c) { return c->apply_now && c->n_pend > 0; }

// pend: index of the deferred update this sweep applies; -1 = the last one (the fused sweep's)
static void k1_common(const zo2_ctx* c, K1Args& a, uint64_t seed, float eps, int pend = -1) {
    memset(&a, 0, sizeof(a));
    const int k = pend >= 0 ? pend : (c->n_pend > 0 ? c->n_pend - 1 : 0);
    a.c_ptr = coef_slot(c, k);
    a.c_imm = 0.f;
    a.stochastic = c->stochastic ? 1 : 0;
    a.eps = eps;
    a.k_prev = philox_keys(c->n_pend > 0 ? c->pend_seed[k] : 0);
    a.k_cur = philox_keys(seed);
}

// one whole tensor held contiguously at `theta`
static zo2_status k1_tensor(zo2_ctx* c, void* theta, int64_t n, uint32_t tid, bool perturb, void* wp, void* wm,
                            uint64_t seed, float eps, hipStream_t st = nullptr, int pend = -1) {
    if (!st) st = c->sc;
    K1Args a;
    k1_common(c, a, seed, eps, pend);
    a.theta = theta; a.w_plus = wp; a.w_minus = c->ns == 2 ? wm : nullptr; a.w_off0 = 0; a.nseg = 1;
    a.seg[0].off = 0; a.seg[0].e0 = 0; a.seg[0].n = (uint64_t)n; a.seg[0].tensor_id = tid; a.seg[0].scale = c->scales[tid];
    OPKS(c, ZO2_KC_K1, st, k1_launch(a, c->cfg.wire_dtype, c->cfg.compute_dtype, pend >= 0 || fused_update(c), perturb, st));
    return ZO2_OK;
}

// tensors [t0, t1) of block l whose bucket sits at `bucket`; W+- go to the scratch, tensor t0 at its start
static zo2_status k1_block(zo2_ctx* c, int l, char* bucket, int t0, int t1, bool perturb, uint64_t seed, float eps,
                           hipStream_t st = nullptr, int pend = -1) {
    if (!st) st = c->sc;
    K1Args a;
    k1_common(c, a, seed, eps, pend);
    a.theta = bucket; a.w_plus = c->wp; a.w_minus = c->ns == 2 ? c->wm : nullptr; a.w_off0 = c->offs[t0]; a.nseg = t1 - t0;
    a.reverse = perturb ? 1 : 0;      // end with the tensors the next projection reads (see k1_kernel)
    for (int k = t0; k < t1; ++k) {
        K1Seg& s = a.seg[k - t0];
        s.off = c->offs[k]; s.e0 = 0; s.n = (uint64_t)c->tn[k]; s.tensor_id = block_tid(l, k); s.scale = c->scales[s.tensor_id];
    }
    OPKS(c, ZO2_KC_K1, st, k1_launch(a, c->cfg.wire_dtype, c->cfg.compute_dtype, pend >= 0 || fused_update(c), perturb, st));
    return ZO2_OK;
}

// update-only sweep over block l with an explicit coefficient (device scalar) and seed: replays an update the block's
// host copy lacks
static inline float* stale_slot(const zo2_ctx* c, int k) { return c->d_state + 32 + k; }
static zo2_status k1_block_replay(zo2_ctx* c, int l, char* bucket, const float* coef, uint64_t seed_prev, hipStream_t st) {
    if (!st) st = c->sc;
    K1Args a;
    k1_common(c, a, 0, 0.f, -1);
    a.c_ptr = coef;
    a.k_prev = philox_keys(seed_prev);
    a.theta = bucket; a.w_plus = nullptr; a.w_minus = nullptr; a.w_off0 = 0; a.nseg = ZO2_BLOCK_TENSORS;
    for (int k = 0; k < ZO2_BLOCK_TENSORS; ++k) {
        K1Seg& s = a.seg[k];
        s.off = c->offs[k]; s.e0 = 0; s.n = (uint64_t)c->tn[k]; s.tensor_id = block_tid(l, k); s.scale = c->scales[s.tensor_id];
    }
    OPKS(c, ZO2_KC_K1, st, k1_launch(a, c->cfg.wire_dtype, c->cfg.compute_dtype, true, false, st));
    return ZO2_OK;
}
static zo2_status stale_updates_block(zo2_ctx* c, int l, char* bucket, hipStream_t st = nullptr) {
    if (c->resident) return ZO2_OK;
    for (int k = 0; k < c->n_stale; ++k) {
        zo2_status s = k1_block_replay(c, l, bucket, stale_slot(c, k), c->stale_seed[k], st);
        if (s != ZO2_OK) return s;
    }
    return ZO2_OK;
}

// the final LayerNorm's two vectors
static zo2_status k1_final_ln(zo2_ctx* c, bool perturb, uint64_t seed, float eps, int pend = -1) {
    K1Args a;
    k1_common(c, a, seed, eps, pend);
    a.theta = c->d_fln; a.w_off0 = 0; a.nseg = 2;
    if (perturb) { a.w_plus = c->fln_wp; a.w_minus = c->ns == 2 ? c->fln_wm : nullptr; }
    for (int k = 0; k < 2; ++k) {
        a.seg[k].off = k * c->fln_off_b; a.seg[k].e0 = 0; a.seg[k].n = (uint64_t)c->cfg.d_model;
        a.seg[k].tensor_id = fln_tid(c) + k; a.seg[k].scale = c->scales[fln_tid(c) + k];
    }
    OPK(c, ZO2_KC_K1, k1_launch(a, c->cfg.wire_dtype, c->cfg.compute_dtype, pend >= 0 || fused_update(c), perturb, c->sc));
    return ZO2_OK;
}

// Deferred updates 0 .. n_pend - 2 of a module, in order, as update-only sweeps: after a round of several directions
// they precede the fused sweep, which applies the last one together with the new perturbation.
static zo2_status earlier_updates_tensor(zo2_ctx* c, void* theta, int64_t n, uint32_t tid, hipStream_t st = nullptr) {
    if (!c->apply_now) return ZO2_OK;
    for (int k = 0; k + 1 < c->n_pend; ++k) {
        zo2_status s = k1_tensor(c, theta, n, tid, false, nullptr, nullptr, 0, 0.f, st, k);
        if (s != ZO2_OK) return s;
    }
    return ZO2_OK;
}
static zo2_status earlier_updates_block(zo2_ctx* c, int l, char* bucket, hipStream_t st = nullptr) {
    if (c->dir_later) return ZO2_OK;          // the first direction of the pass has brought the block up to date
    { zo2_status s = stale_updates_block(c, l, bucket, st); if (s != ZO2_OK) return s; }      // what the host copy lacks comes first, whatever the pass
    if (!c->apply_now) return ZO2_OK;
    for (int k = 0; k + 1 < c->n_pend; ++k) {
        zo2_status s = k1_block(c, l, bucket, 0, ZO2_BLOCK_TENSORS, false, 0, 0.f, st, k);
        if (s != ZO2_OK) return s;
    }
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- block forward
// A block projection: split along k when the launch would leave most compute units idle (few rows per stream)
static zo2_status block_gemm(zo2_ctx* c, const GemmArgs& ga) {
    const int dt = c->cfg.compute_dtype;
    const int splits = c->split_k >= 0 ? gemm_pick_splits(ga.M, ga.N, ga.K, ga.nprob, dt) : 1;
    if (splits > 1 && gemm_splitk_workspace_bytes(ga.M, ga.N, ga.nprob, splits) <= c->sk_ws_bytes)
        return gemm_launch_splitk(ga, dt, splits, c->sk_ws, c->sk_ws_bytes, c->sc);
    return gemm_launch(ga, dt, c->sc);
}

struct PhaseView {       // where tensor k's perturbed copies are inside the scratch
    const zo2_ctx* c;
    int64_t off0;
    const char* P(int k) const { return c->wp + (size_t)(c->offs[k] - off0) * c->csz; }
    const char* M(int k) const { return c->wm + (size_t)(c->offs[k] - off0) * c->csz; }
};

static zo2_status block_forward(zo2_ctx* c, int l, char* bucket, int batch, int seq, uint64_t seed, float eps, hipEvent_t k1_done,
                                bool k1_enqueued = false) {
    const zo2_config& g = c->cfg;
    const int T = batch * seq, d = g.d_model, f = g.d_ffn, dh = d / g.n_heads;
    const int dt = g.compute_dtype;
    const size_t cs = c->csz;
    const size_t half_d = (size_t)T * d * cs, half_f = (size_t)T * f * cs;
    const bool f32 = dt == ZO2_F32;
    const int ns = c->ns;                 // 2: both perturbation streams (rows 0..T-1 and T..2T-1); 1: a single forward
    auto phase = [&](int p) -> zo2_status {
        if (k1_enqueued || c->pb[p + 1] == c->pb[p]) return ZO2_OK;
        zo2_status s = k1_block(c, l, bucket, c->pb[p], c->pb[p + 1], true, seed, eps);
        // the block's parameters are final after its last sweep: the offload may start (streamed mode)
        if (s == ZO2_OK && c->pb[p + 1] == ZO2_BLOCK_TENSORS && k1_done) HIPCHK(c, hipEventRecord(k1_done, c->sc));
        return s;
    };
    // the scratch holds the tensors of the last sweep issued at or before point p, the first of them at its start
    auto view = [&](int p) {
        int q = p;
        while (c->pb[q + 1] == c->pb[q]) --q;       // sweep 0 is never empty
        return PhaseView{c, c->offs[c->pb[q]]};
    };
    GemmArgs ga;

    // ---- attention half: h += O(Attn(LN1(h)))
    if (!k1_enqueued) { zo2_status s = earlier_updates_block(c, l, bucket); if (s != ZO2_OK) return s; }
    { zo2_status s = phase(0); if (s != ZO2_OK) return s; }
    PhaseView w = view(0);
    OPK(c, ZO2_KC_LN, layernorm(dt, c->h, w.P(0), w.P(1), w.M(0), w.M(1), c->x, ns * T, T, d, g.ln_eps, c->sc));
    memset(&ga, 0, sizeof(ga));
    ga.M = T; ga.N = d; ga.K = d; ga.ldx = d; ga.ldw = d; ga.ldy = d; ga.relu = 0; ga.out_f32 = f32; ga.nprob = 3 * ns;
    char* outs[3] = {c->qb, c->kb, c->vb};
    for (int s = 0; s < ns; ++s)
        for (int t = 0; t < 3; ++t) {
            GemmProblem& p = ga.p[s * 3 + t];
            p.X = c->x + s * half_d;
            p.W = s ? w.M(2 + 2 * t) : w.P(2 + 2 * t);
            p.bias = s ? w.M(3 + 2 * t) : w.P(3 + 2 * t);
            p.residual = nullptr;
            p.Y = outs[t] + s * half_d;
            p.out_scale = t == 0 ? 1.0f / sqrtf((float)dh) : 1.0f;
        }
    OPK(c, ZO2_KC_GEMM, block_gemm(c, ga));
    OPK(c, ZO2_KC_ATTN, attention_launch(dt, c->qb, c->kb, c->vb, c->ctxb, ns * batch, seq, g.n_heads, dh, d, 0, c->sc));
    { zo2_status s = phase(1); if (s != ZO2_OK) return s; }
    w = view(1);
    memset(&ga, 0, sizeof(ga));
    ga.M = T; ga.N = d; ga.K = d; ga.ldx = d; ga.ldw = d; ga.ldy = d; ga.relu = 0; ga.out_f32 = 1; ga.nprob = ns;
    for (int s = 0; s < ns; ++s) {
        GemmProblem& p = ga.p[s];
        p.X = c->ctxb + s * half_d; p.W = s ? w.M(8) : w.P(8); p.bias = s ? w.M(9) : w.P(9);
        p.residual = c->h + (size_t)s * T * d; p.Y = c->h + (size_t)s * T * d; p.out_scale = 1.0f;
    }
    OPK(c, ZO2_KC_GEMM, block_gemm(c, ga));

    // ---- FFN half: h += FC2(ReLU(FC1(LN2(h))))
    { zo2_status s = phase(2); if (s != ZO2_OK) return s; }
    w = view(2);
    OPK(c, ZO2_KC_LN, layernorm(dt, c->h, w.P(10), w.P(11), w.M(10), w.M(11), c->x, ns * T, T, d, g.ln_eps, c->sc));
    memset(&ga, 0, sizeof(ga));
    ga.M = T; ga.N = f; ga.K = d; ga.ldx = d; ga.ldw = d; ga.ldy = f; ga.relu = 1; ga.out_f32 = f32; ga.nprob = ns;
    for (int s = 0; s < ns; ++s) {
        GemmProblem& p = ga.p[s];
        p.X = c->x + s * half_d; p.W = s ? w.M(12) : w.P(12); p.bias = s ? w.M(13) : w.P(13);
        p.residual = nullptr; p.Y = c->mid + s * half_f; p.out_scale = 1.0f;
    }
    OPK(c, ZO2_KC_GEMM, block_gemm(c, ga));
    { zo2_status s = phase(3); if (s != ZO2_OK) return s; }
    w = view(3);
    memset(&ga, 0, sizeof(ga));
    ga.M = T; ga.N = d; ga.K = f; ga.ldx = f; ga.ldw = f; ga.ldy = d; ga.relu = 0; ga.out_f32 = 1; ga.nprob = ns;
    for (int s = 0; s < ns; ++s) {
        GemmProblem& p = ga.p[s];
        p.X = c->mid + s * half_f; p.W = s ? w.M(14) : w.P(14); p.bias = s ? w.M(15) : w.P(15);
        p.residual = c->h + (size_t)s * T * d; p.Y = c->h + (size_t)s * T * d; p.out_scale = 1.0f;
    }
    OPK(c, ZO2_KC_GEMM, block_gemm(c, ga));
    return ZO2_OK;
}

// The same block for a step of few tokens: K1 only applies the pending update (theta' is final after it) and perturbs
// the block's ten one-dimensional tensors into a densely packed scratch; the six projections read theta' itself and
// perturb in their weight loader, both streams per pass over the weights (gemm_skinny.hip).
static const int kVecTensors[10] = {0, 1, 3, 5, 7, 9, 10, 11, 13, 15};      // ln1.w ln1.b q.b k.b v.b o.b ln2.w ln2.b fc1.b fc2.b

static zo2_status block_forward_fused(zo2_ctx* c, int l, char* bucket, int batch, int seq, uint64_t seed, float eps, hipEvent_t k1_done) {
    const zo2_config& g = c->cfg;
    const int T = batch * seq, d = g.d_model, f = g.d_ffn, dh = d / g.n_heads;
    const int dt = g.compute_dtype;
    const size_t cs = c->csz;
    const size_t half_d = (size_t)T * d * cs, half_f = (size_t)T * f * cs;
    { zo2_status s = earlier_updates_block(c, l, bucket); if (s != ZO2_OK) return s; }
    { zo2_status s = k1_block(c, l, bucket, 0, ZO2_BLOCK_TENSORS, false, seed, eps); if (s != ZO2_OK) return s; }     // the update alone
    if (k1_done) HIPCHK(c, hipEventRecord(k1_done, c->sc));      // the block's parameters are final: the offload may start
    int64_t voff[ZO2_BLOCK_TENSORS] = {0};
    {
        K1Args a;
        k1_common(c, a, seed, eps);
        a.theta = bucket; a.w_plus = c->wp; a.w_minus = c->wm; a.packed_w = 1; a.nseg = 10;
        int64_t o = 0;
        for (int i = 0; i < 10; ++i) {
            const int k = kVecTensors[i];
            K1Seg& sg = a.seg[i];
            sg.off = c->offs[k]; sg.e0 = 0; sg.n = (uint64_t)c->tn[k]; sg.tensor_id = block_tid(l, k); sg.scale = 1.0f; sg.woff = o;
            voff[k] = o;
            o += (c->tn[k] + kTensorAlign - 1) / kTensorAlign * kTensorAlign;
        }
        OPK(c, ZO2_KC_K1, k1_launch(a, g.wire_dtype, g.compute_dtype, false, true, c->sc));
    }
    auto VP = [&](int k) { return (const void*)(c->wp + (size_t)voff[k] * cs); };
    auto VM = [&](int k) { return (const void*)(c->wm + (size_t)voff[k] * cs); };
    auto TH = [&](int k) { return (const void*)(bucket + (size_t)c->offs[k] * cs); };
    SkinnyArgs sa;
    auto common = [&](int N, int K, int ldx, int ldy, int relu, int out_f32, int nprob) {
        memset(&sa, 0, sizeof(sa));
        sa.M = T; sa.N = N; sa.K = K; sa.ldx = ldx; sa.ldy = ldy; sa.relu = relu; sa.out_f32 = out_f32; sa.nprob = nprob; sa.eps = eps;
        sa.key = philox_keys(seed);
    };

    // ---- attention half: h += O(Attn(LN1(h)))
    OPK(c, ZO2_KC_LN, layernorm(dt, c->h, VP(0), VP(1), VM(0), VM(1), c->x, 2 * T, T, d, g.ln_eps, c->sc));
    common(d, d, d, d, 0, 0, 3);
    char* outs[3] = {c->qb, c->kb, c->vb};
    for (int t = 0; t < 3; ++t) {
        SkinnyProblem& p = sa.p[t];
        p.Xp = c->x; p.Xm = c->x + half_d; p.theta = TH(2 + 2 * t); p.bias_p = VP(3 + 2 * t); p.bias_m = VM(3 + 2 * t);
        p.Yp = outs[t]; p.Ym = outs[t] + half_d; p.out_scale = t == 0 ? 1.0f / sqrtf((float)dh) : 1.0f; p.tensor_id = block_tid(l, 2 + 2 * t);
    }
    OPK(c, ZO2_KC_GEMM, skinny_launch(sa, dt, c->sk_ws, c->sk_ws_bytes, c->sc));
    OPK(c, ZO2_KC_ATTN, attention_launch(dt, c->qb, c->kb, c->vb, c->ctxb, 2 * batch, seq, g.n_heads, dh, d, 0, c->sc));
    common(d, d, d, d, 0, 1, 1);
    {
        SkinnyProblem& p = sa.p[0];
        p.Xp = c->ctxb; p.Xm = c->ctxb + half_d; p.theta = TH(8); p.bias_p = VP(9); p.bias_m = VM(9);
        p.res_p = c->h; p.res_m = c->h + (size_t)T * d; p.Yp = c->h; p.Ym = c->h + (size_t)T * d; p.out_scale = 1.0f; p.tensor_id = block_tid(l, 8);
    }
    OPK(c, ZO2_KC_GEMM, skinny_launch(sa, dt, c->sk_ws, c->sk_ws_bytes, c->sc));

    // ---- FFN half: h += FC2(ReLU(FC1(LN2(h))))
    OPK(c, ZO2_KC_LN, layernorm(dt, c->h, VP(10), VP(11), VM(10), VM(11), c->x, 2 * T, T, d, g.ln_eps, c->sc));
    common(f, d, d, f, 1, 0, 1);
    {
        SkinnyProblem& p = sa.p[0];
        p.Xp = c->x; p.Xm = c->x + half_d; p.theta = TH(12); p.bias_p = VP(13); p.bias_m = VM(13);
        p.Yp = c->mid; p.Ym = c->mid + half_f; p.out_scale = 1.0f; p.tensor_id = block_tid(l, 12);
    }
    OPK(c, ZO2_KC_GEMM, skinny_launch(sa, dt, c->sk_ws, c->sk_ws_bytes, c->sc));
    common(d, f, f, d, 0, 1, 1);
    {
        SkinnyProblem& p = sa.p[0];
        p.Xp = c->mid; p.Xm = c->mid + half_f; p.theta = TH(14); p.bias_p = VP(15); p.bias_m = VM(15);
        p.res_p = c->h; p.res_m = c->h + (size_t)T * d; p.Yp = c->h; p.Ym = c->h + (size_t)T * d; p.out_scale = 1.0f; p.tensor_id = block_tid(l, 14);
    }
    OPK(c, ZO2_KC_GEMM, skinny_launch(sa, dt, c->sk_ws, c->sk_ws_bytes, c->sc));
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- streaming (Alg. 3)
// U(W_i): runs on the upload stream once the slot's previous occupant has left it.
static zo2_status enqueue_upload(zo2_ctx* c, int l) {
    const int s = l % c->n_slots;
    if (c->ev_free_valid[s]) HIPCHK(c, hipStreamWaitEvent(c->su, c->ev_free[s], 0));
    // with the perturbation in the projections' loader the forwards read the slot itself: its next occupant also waits for them
    if (c->ev_read_valid[s]) HIPCHK(c, hipStreamWaitEvent(c->su, c->ev_read[s], 0));
    if (!c->stat_u) { HIPCHK(c, hipEventRecord(c->ev_u0, c->su)); c->stat_u = true; }
    { zo2_status ds = debug_delay(c, 1, c->su); if (ds != ZO2_OK) return ds; }
    if (c->debug_poison) {      // whoever reads the slot before the copy below has landed computes NaN
        hipLaunchKernelGGL(poison_kernel, dim3(1024), dim3(256), 0, c->su, (uint32_t*)(c->slots + (size_t)s * c->bucket_bytes), c->bucket_bytes / 4);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(c, ZO2_EHIP, "poison kernel: %s", hipGetErrorString(e));
    }
    HIPCHK(c, hipMemcpyAsync(c->slots + (size_t)s * c->bucket_bytes, c->host_bucket[l], c->bucket_bytes, hipMemcpyHostToDevice, c->su));
    HIPCHK(c, hipEventRecord(c->ev_up[s], c->su));
    c->bytes_up += c->bucket_bytes;
    return ZO2_OK;
}

// O(W_i): the updated block goes back as soon as its K1 pass is done (the forwards read
// only the scratch copies, never the slot); without a pending update nothing changed.
static zo2_status enqueue_offload(zo2_ctx* c, int l, bool changed) {
    const int s = l % c->n_slots;
    if (changed) {
        HIPCHK(c, hipStreamWaitEvent(c->so, c->ev_k1[s], 0));
        if (!c->stat_o) { HIPCHK(c, hipEventRecord(c->ev_o0, c->so)); c->stat_o = true; }
        { zo2_status ds = debug_delay(c, 2, c->so); if (ds != ZO2_OK) return ds; }
        HIPCHK(c, hipMemcpyAsync(c->host_bucket[l], c->slots + (size_t)s * c->bucket_bytes, c->bucket_bytes, hipMemcpyDeviceToHost, c->so));
        HIPCHK(c, hipEventRecord(c->ev_free[s], c->so));
        c->bytes_down += c->bucket_bytes;
    } else {
        HIPCHK(c, hipStreamWaitEvent(c->so, c->ev_k1[s], 0));
        HIPCHK(c, hipEventRecord(c->ev_free[s], c->so));
    }
    c->ev_free_valid[s] = 1;
    return ZO2_OK;
}

// Brings the host copies of streamed blocks up to date: every block travels once, takes the updates its host copy lacks
// and goes back.  Nothing to do when the blocks are resident or nothing is lacking.
static zo2_status writeback_pass(zo2_ctx* c) {
    if (!c->planned || c->resident || c->n_stale == 0) return ZO2_OK;
    const zo2_config& g = c->cfg;
    TraceRange range("zo2 write-back");
    c->stat_u = c->stat_o = true;   // no span statistics
    int next_upload = 0;
    for (; next_upload < c->n_slots && next_upload < g.n_layers; ++next_upload) {
        zo2_status s = enqueue_upload(c, next_upload);
        if (s != ZO2_OK) return s;
    }
    for (int l = 0; l < g.n_layers; ++l) {
        const int sl = l % c->n_slots;
        HIPCHK(c, hipStreamWaitEvent(c->sc, c->ev_up[sl], 0));
        { zo2_status s = stale_updates_block(c, l, c->slots + (size_t)sl * c->bucket_bytes); if (s != ZO2_OK) return s; }
        HIPCHK(c, hipEventRecord(c->ev_k1[sl], c->sc));
        c->ev_read_valid[sl] = 0;
        zo2_status s = enqueue_offload(c, l, true);
        if (s != ZO2_OK) return s;
        if (next_upload < g.n_layers) {
            s = enqueue_upload(c, next_upload++);
            if (s != ZO2_OK) return s;
        }
    }
    HIPCHK(c, hipStreamSynchronize(c->sc));
    HIPCHK(c, hipStreamSynchronize(c->su));
    HIPCHK(c, hipStreamSynchronize(c->so));
    c->n_stale = 0;
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- one pass over the model
// ns = 2: Alg. 2's iteration (update, perturb both ways, dual forward, g).  ns = 1: the same walk with a
// single unperturbed forward (evaluation): the pending update is still applied on the way, W+ = theta'.
// extra: a further direction of the current round (ns = 2): nothing deferred is applied, the parameters stay as
// they are, and the pass's own (seed, eta g) joins the deferred updates instead of replacing them.
// One pass over the model.  seeds[0 .. ndirs - 1]: the directions evaluated in this pass (ndirs > 1: zo2_step_multi; every
// module - embedding, each block while it sits in its slot, head - runs the dual forward of all directions before the
// pass moves on, so a streamed block travels once for all of them).  Results of direction j: pass_result(c, j).
static inline float* pass_result(const zo2_ctx* c, int j) { return j == 0 ? c->h_result : c->h_result + 16 + 4 * (j - 1); }
static zo2_status model_pass(zo2_ctx* c, const char* who, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                             const uint64_t* seeds, int ndirs, float eps, float lr, int ns, bool extra = false) {
    const uint64_t seed = seeds[0];
    const zo2_config& g = c->cfg;
    if (batch <= 0 || seq <= 0 || seq > g.max_pos) return fail(c, ZO2_EINVAL, "%s: batch %d, seq %d (max_pos %d)", who, batch, seq, g.max_pos);
    if ((int64_t)batch * seq > (1 << 24)) return fail(c, ZO2_EINVAL, "%s: too many tokens", who);
    c->ns = ns;
    const int T = batch * seq;
    for (int i = 0; i < T; ++i) {
        if (tokens[i] < 0 || tokens[i] >= g.vocab) return fail(c, ZO2_EINVAL, "%s: token %d at %d outside [0, %d)", who, tokens[i], i, g.vocab);
        if (labels[i] != -100 && (labels[i] < 0 || labels[i] >= g.vocab)) return fail(c, ZO2_EINVAL, "%s: label %d at %d invalid", who, labels[i], i);
    }
    c->want_dirs = std::max(c->want_dirs, ndirs);
    if (!c->planned || c->need_plan || c->plan_T != T || c->plan_seq != seq || c->plan_dirs < ndirs) {
        zo2_status s = plan(c, T, batch, seq);
        if (s != ZO2_OK) return s;
    }
    const int d = g.d_model, dt = g.compute_dtype;
    c->apply_now = !extra;
    c->dir_later = false;
    // direction j of the pass: its residual stream; only the first direction of a pass applies deferred updates
    auto set_dir = [&](int j) {
        c->h = c->hs[j];
        c->dir_later = j > 0;
        c->apply_now = j == 0 ? !extra : false;
    };
    const bool upd = fused_update(c);
    // streamed blocks: does this pass write them back?  Their host copies lack n_stale updates already; this pass adds the
    // deferred ones it applies.  (The list of lacking updates must keep room for a whole round of the next pass.)
    const int lack = c->resident ? 0 : c->n_stale + (upd ? c->n_pend : 0);
    c->pass_writes_back = c->resident || lack >= c->wb_interval || lack > zo2_ctx::kMaxStale - zo2_ctx::kMaxPending;
    const bool changed = upd || (!c->resident && c->n_stale > 0);
    c->bytes_up = c->bytes_down = 0;
    c->stat_u = c->stat_o = false;
    prof_reset(c);

    memcpy(c->h_ids, tokens, (size_t)T * 4);
    memcpy(c->h_ids + T, labels, (size_t)T * 4);
    HIPCHK(c, hipEventRecord(c->ev_step0, c->sc));
    HIPCHK(c, hipMemcpyAsync(c->d_tokens, c->h_ids, (size_t)T * 4, hipMemcpyHostToDevice, c->sc));
    HIPCHK(c, hipMemcpyAsync(c->d_labels, c->h_ids + T, (size_t)T * 4, hipMemcpyHostToDevice, c->sc));

    // U(W_1..): prefetch as many blocks as there are slots; overlaps the embedding
    int next_upload = 0;
    const bool serial = c->serial_streams && !c->overlap_k1;   // the ablation is defined for the three-stream schedule
    if (!c->resident && !serial)
        for (; next_upload < c->n_slots && next_upload < g.n_layers; ++next_upload) {
            zo2_status s = enqueue_upload(c, next_upload);
            if (s != ZO2_OK) return s;
        }

    TraceRange step_range(ns == 2 ? (extra ? "zo2_step_extra" : "zo2_step") : "zo2_eval");
    // DualForward(Embedding)
    {   // earlier directions of the last round: the tables first, the gather then sees them
        zo2_status s = earlier_updates_tensor(c, c->d_tok, c->tok_elems, 0);
        if (s == ZO2_OK) s = earlier_updates_tensor(c, c->d_pos, c->pos_elems, 1);
        if (s != ZO2_OK) return s;
    }
    EmbedArgs ea;
    memset(&ea, 0, sizeof(ea));
    ea.tok_emb = c->d_tok; ea.pos_emb = c->d_pos; ea.tokens = c->d_tokens; ea.h = c->h;
    ea.T = T; ea.seq = seq; ea.d = d; ea.pos_offset = g.pos_offset; ea.eps = eps; ea.single = ns == 1; ea.stochastic = c->stochastic ? 1 : 0;
    ea.scale_tok = c->scales[0]; ea.scale_pos = c->scales[1]; ea.c_ptr = coef_slot(c, c->n_pend > 0 ? c->n_pend - 1 : 0);
    ea.k_prev = philox_keys(c->n_pend > 0 ? c->pend_seed[c->n_pend - 1] : 0); ea.k_cur = philox_keys(seed);
    for (int j = 0; j < ndirs; ++j) {      // every direction gathers before the tables are updated in place below
        ea.h = c->hs[j];
        ea.k_cur = philox_keys(seeds[j]);
        OPK(c, ZO2_KC_EMBED, embed_gather(ea, g.wire_dtype, dt, upd, c->sc));
    }
    if (upd) {
        { zo2_status s = k1_tensor(c, c->d_pos, c->pos_elems, 1, false, nullptr, nullptr, seed, eps); if (s != ZO2_OK) return s; }
        if (!g.tied_lm_head) { zo2_status s = k1_tensor(c, c->d_tok, c->tok_elems, 0, false, nullptr, nullptr, seed, eps); if (s != ZO2_OK) return s; }
    }

    // DualForward(W_1 .. W_N).  With a fourth stream and two scratch sets, K1 of block l runs on that
    // stream as soon as the forwards of block l-2 have released its scratch set, i.e. under the
    // forwards of block l-1 (K1 is bound by the vector ALU and HBM, the forwards by the matrix cores).
    if (c->overlap_k1) HIPCHK(c, hipEventRecord(c->ev_embed, c->sc));
    for (int l = 0; l < g.n_layers; ++l) {
        TraceRange block_range("block %d", l);
        const int sl = c->resident ? l : l % c->n_slots;
        char* bucket = c->slots + (size_t)sl * c->bucket_bytes;
        const int sb = l & 1;
        c->wp = c->wps[sb];
        c->wm = c->wms[sb];
        if (c->overlap_k1) {
            if (l >= 2) HIPCHK(c, hipStreamWaitEvent(c->sk, c->ev_fwd_done[sb], 0));
            if (!c->resident) HIPCHK(c, hipStreamWaitEvent(c->sk, c->ev_up[sl], 0));  // C(W_i) after U(W_i)
            { zo2_status s = earlier_updates_block(c, l, bucket, c->sk); if (s != ZO2_OK) return s; }
            { zo2_status s = k1_block(c, l, bucket, 0, ZO2_BLOCK_TENSORS, true, seed, eps, c->sk); if (s != ZO2_OK) return s; }
            HIPCHK(c, hipEventRecord(c->ev_k1done[sb], c->sk));
            if (!c->resident) HIPCHK(c, hipEventRecord(c->ev_k1[sl], c->sk));
            HIPCHK(c, hipStreamWaitEvent(c->sc, c->ev_k1done[sb], 0));
            zo2_status s = block_forward(c, l, bucket, batch, seq, seed, eps, nullptr, true);
            if (s != ZO2_OK) return s;
            HIPCHK(c, hipEventRecord(c->ev_fwd_done[sb], c->sc));
        } else {
            if (!c->resident && serial) {      // ablation of Sec. 5.2: nothing overlaps, U(W_i) starts when O(W_{i-1}) is done
                zo2_status us = enqueue_upload(c, next_upload++);
                if (us != ZO2_OK) return us;
                HIPCHK(c, hipStreamSynchronize(c->su));
            }
            if (!c->resident) HIPCHK(c, hipStreamWaitEvent(c->sc, c->ev_up[sl], 0));  // C(W_i) after U(W_i)
            { zo2_status ds = debug_delay(c, 0, c->sc); if (ds != ZO2_OK) return ds; }
            const bool fused_block = c->fuse && ns == 2;
            for (int j = 0; j < ndirs; ++j) {
                set_dir(j);
                // the slot is read by every direction's sweep: it is released (offload, next occupant) after the last one
                hipEvent_t k1_done = (c->resident || j + 1 < ndirs) ? nullptr : c->ev_k1[sl];
                zo2_status s = fused_block ? block_forward_fused(c, l, bucket, batch, seq, seeds[j], eps, k1_done)
                                           : block_forward(c, l, bucket, batch, seq, seeds[j], eps, k1_done);
                if (s != ZO2_OK) { set_dir(0); return s; }
            }
            set_dir(0);
            if (!c->resident) {
                if (fused_block) HIPCHK(c, hipEventRecord(c->ev_read[sl], c->sc));
                c->ev_read_valid[sl] = fused_block ? 1 : 0;
            }
        }
        if (!c->resident && serial) {
            HIPCHK(c, hipStreamSynchronize(c->sc));
            zo2_status s = enqueue_offload(c, l, changed && c->pass_writes_back);
            if (s != ZO2_OK) return s;
            HIPCHK(c, hipStreamSynchronize(c->so));
        } else if (!c->resident) {
            zo2_status s = enqueue_offload(c, l, changed && c->pass_writes_back);                             // O(W_i) after its update
            if (s != ZO2_OK) return s;
            if (next_upload < g.n_layers) {                                        // U(W_{i+n}) into the slot O(W_i) frees
                s = enqueue_upload(c, next_upload++);
                if (s != ZO2_OK) return s;
            }
        }
    }

    // DualForward(LM head): final LayerNorm, (tied) vocabulary matrix, loss
    TraceRange head_range("lm_head + loss");
    for (int j = 0; j < ndirs; ++j) {
        const uint64_t seed = seeds[j];
        set_dir(j);
        if (c->apply_now)
            for (int k = 0; k + 1 < c->n_pend; ++k) { zo2_status s = k1_final_ln(c, false, 0, 0.f, k); if (s != ZO2_OK) return s; }
        { zo2_status s = k1_final_ln(c, true, seed, eps); if (s != ZO2_OK) return s; }
        const size_t boff = (size_t)c->fln_off_b * c->csz;
        OPK(c, ZO2_KC_LN, layernorm(dt, c->h, c->fln_wp, c->fln_wp + boff, c->fln_wm, c->fln_wm + boff, c->x, ns * T, T, d, g.ln_eps, c->sc));
        {
            const int sb = g.n_layers & 1;
            c->wp = c->wps[sb];
            c->wm = c->wms[sb];
            hipStream_t st = c->sc;
            if (c->overlap_k1) {      // the vocabulary matrix is swept under the last block's forwards
                st = c->sk;
                HIPCHK(c, hipStreamWaitEvent(c->sk, c->ev_embed, 0));                  // the gather read the table before its update
                if (g.n_layers >= 2) HIPCHK(c, hipStreamWaitEvent(c->sk, c->ev_fwd_done[sb], 0));
            }
            if (!g.tied_lm_head) { zo2_status es = earlier_updates_tensor(c, c->d_lm, c->tok_elems, lm_tid(c), st); if (es != ZO2_OK) return es; }
            zo2_status s = g.tied_lm_head ? k1_tensor(c, c->d_tok, c->tok_elems, 0, true, c->wp, c->wm, seed, eps, st)
                                          : k1_tensor(c, c->d_lm, c->tok_elems, lm_tid(c), true, c->wp, c->wm, seed, eps, st);
            if (s != ZO2_OK) return s;
            if (c->overlap_k1) {
                HIPCHK(c, hipEventRecord(c->ev_k1done[sb], c->sk));
                HIPCHK(c, hipStreamWaitEvent(c->sc, c->ev_k1done[sb], 0));
            }
        }
        if (c->fused_ce) {
            // logits are never written: the GEMM epilogue reduces each 64-column span to (max, sum exp) and picks the label's logit
            GemmArgs ga;
            memset(&ga, 0, sizeof(ga));
            ga.M = T; ga.N = g.vocab; ga.K = d; ga.ldx = d; ga.ldw = d; ga.ldy = g.vocab; ga.relu = 0; ga.out_f32 = 1; ga.nprob = ns; ga.ce_mode = 1; ga.part_ld = 2 * (int64_t)T;
            for (int s = 0; s < ns; ++s) {
                GemmProblem& p = ga.p[s];
                p.X = c->x + (size_t)s * T * d * c->csz; p.W = s ? c->wm : c->wp; p.bias = nullptr; p.residual = nullptr; p.Y = nullptr;
                p.out_scale = 1.0f; p.labels = c->d_labels;
                p.part_max = c->ce_pmax + (size_t)s * T; p.part_sum = c->ce_psum + (size_t)s * T;
                p.label_logit = c->ce_lab + (size_t)s * T;
            }
            OPK(c, ZO2_KC_GEMM, gemm_launch(ga, dt, c->sc));
            OPK(c, ZO2_KC_CE, ce_combine(c->ce_pmax, c->ce_psum, c->ce_lab, c->d_labels, ns * T, c->ce_parts, 2 * (int64_t)T, 0, T, c->row_loss, c->sc));
        } else {
            const int R = c->logit_rows;
            for (int r0 = 0; r0 < T; r0 += R) {
                const int rows = std::min(R, T - r0);
                GemmArgs ga;
                memset(&ga, 0, sizeof(ga));
                ga.M = rows; ga.N = g.vocab; ga.K = d; ga.ldx = d; ga.ldw = d; ga.ldy = g.vocab; ga.relu = 0; ga.out_f32 = 1; ga.nprob = ns;
                for (int s = 0; s < ns; ++s) {
                    GemmProblem& p = ga.p[s];
                    p.X = c->x + ((size_t)s * T + r0) * d * c->csz; p.W = s ? c->wm : c->wp; p.bias = nullptr; p.residual = nullptr;
                    p.Y = c->logits + (size_t)s * R * g.vocab; p.out_scale = 1.0f;
                }
                OPK(c, ZO2_KC_GEMM, gemm_launch(ga, dt, c->sc));
                for (int s = 0; s < ns; ++s)
                    OPK(c, ZO2_KC_CE, cross_entropy_rows(c->logits + (size_t)s * R * g.vocab, g.vocab, c->d_labels, rows, s * T + r0, T, g.vocab, c->row_loss, c->sc));
            }
        }
        // eta g of this pass: deferred update 0 of a new round (every older one has been applied on the way), or one more of
        // the current round
        if (j == 0 && !c->resident && upd && !c->pass_writes_back)      // the coefficients of the updates the blocks' host copies now lack, before slot 0 is rewritten
            HIPCHK(c, hipMemcpyAsync(stale_slot(c, c->n_stale), coef_slot(c, 0), (size_t)c->n_pend * sizeof(float), hipMemcpyDeviceToDevice, c->sc));
        OPK(c, ZO2_KC_CE, loss_epilogue(c->row_loss, c->d_labels, T, eps, lr, ns, c->d_state + 4, coef_slot(c, extra ? c->n_pend : j), c->sc));
        HIPCHK(c, hipMemcpyAsync(pass_result(c, j), c->d_state + 4, 4 * sizeof(float), hipMemcpyDeviceToHost, c->sc));
    }
    set_dir(0);
    HIPCHK(c, hipEventRecord(c->ev_c1, c->sc));
    if (c->stat_u) HIPCHK(c, hipEventRecord(c->ev_u1, c->su));
    if (c->stat_o) HIPCHK(c, hipEventRecord(c->ev_o1, c->so));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    if (c->overlap_k1) HIPCHK(c, hipStreamSynchronize(c->sk));
    if (!c->resident) {
        HIPCHK(c, hipStreamSynchronize(c->su));
        HIPCHK(c, hipStreamSynchronize(c->so));
    }
    prof_collect(c);
    // statistics only: a failed query leaves the figure at zero
    c->ms_c = c->ms_u = c->ms_o = 0.f;
    (void)hipEventElapsedTime(&c->ms_c, c->ev_step0, c->ev_c1);
    if (c->stat_u) (void)hipEventElapsedTime(&c->ms_u, c->ev_u0, c->ev_u1);
    if (c->stat_o) (void)hipEventElapsedTime(&c->ms_o, c->ev_o0, c->ev_o1);

    c->apply_now = true;
    c->dir_later = false;
    if (!c->resident) {
        if (c->pass_writes_back) {
            if (changed) c->n_stale = 0;          // the host copies are current again
        } else if (upd) {
            for (int k = 0; k < c->n_pend; ++k) c->stale_seed[c->n_stale++] = c->pend_seed[k];
        }
    }
    if (ns == 1) {
        c->n_pend = 0;            // the pending updates have been applied to every module on the way
        return ZO2_OK;
    }
    if (ndirs > 1) {          // a new round of ndirs directions; a non-finite loss in any of them drops the whole round
        for (int j = 0; j < ndirs; ++j) {
            const float* r = pass_result(c, j);
            if (!(isfinite(r[0]) && isfinite(r[1]) && isfinite(r[2]))) {
                c->n_pend = 0;
                return fail(c, ZO2_ENONFINITE, "%s: non-finite loss in direction %d (l+ %g, l- %g)", who, j, (double)r[0], (double)r[1]);
            }
        }
        c->n_pend = ndirs;
        for (int j = 0; j < ndirs; ++j) c->pend_seed[j] = seeds[j];
        return ZO2_OK;
    }
    const bool finite = isfinite(c->h_result[0]) && isfinite(c->h_result[1]) && isfinite(c->h_result[2]);
    if (extra) {
        if (finite) c->pend_seed[c->n_pend++] = seed;
    } else {
        c->n_pend = finite ? 1 : 0;
        c->pend_seed[0] = seed;
    }
    // a non-finite g must never reach the parameters: this direction's update is dropped
    if (!finite) return fail(c, ZO2_ENONFINITE, "%s: non-finite loss (l+ %g, l- %g)", who, (double)c->h_result[0], (double)c->h_result[1]);
    return ZO2_OK;
}

// ---------------------------------------------------------------------------------- step
extern "C" zo2_status zo2_step(zo2_ctx* c, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                               uint64_t seed, float eps, float lr, float* loss_plus, float* loss_minus, float* gout) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!tokens || !labels || !loss_plus || !loss_minus || !gout) return fail(c, ZO2_EINVAL, "zo2_step: NULL argument");
    if (!(eps != 0.f) || !isfinite(eps) || !isfinite(lr)) return fail(c, ZO2_EINVAL, "zo2_step: eps must be non-zero and finite, lr finite");
    const zo2_status s = model_pass(c, "zo2_step", tokens, labels, batch, seq, &seed, 1, eps, lr, 2);
    if (s == ZO2_OK || s == ZO2_ENONFINITE) {
        *loss_plus = c->h_result[0];
        *loss_minus = c->h_result[1];
        *gout = c->h_result[2];
    }
    return s;
}

// A further direction of the current round (q-direction form of the estimator): same parameters, same arithmetic,
// nothing applied; its update joins the deferred ones.
extern "C" zo2_status zo2_step_extra(zo2_ctx* c, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                                     uint64_t seed, float eps, float lr, float* loss_plus, float* loss_minus, float* gout) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!tokens || !labels || !loss_plus || !loss_minus || !gout) return fail(c, ZO2_EINVAL, "zo2_step_extra: NULL argument");
    if (!(eps != 0.f) || !isfinite(eps) || !isfinite(lr)) return fail(c, ZO2_EINVAL, "zo2_step_extra: eps must be non-zero and finite, lr finite");
    if (c->n_pend < 1) return fail(c, ZO2_ESTATE, "zo2_step_extra: no round in progress (call zo2_step first)");
    if (c->n_pend >= zo2_ctx::kMaxPending) return fail(c, ZO2_ESTATE, "zo2_step_extra: at most %d directions per round", zo2_ctx::kMaxPending);
    const zo2_status s = model_pass(c, "zo2_step_extra", tokens, labels, batch, seq, &seed, 1, eps, lr, 2, true);
    if (s == ZO2_OK || s == ZO2_ENONFINITE) {
        *loss_plus = c->h_result[0];
        *loss_minus = c->h_result[1];
        *gout = c->h_result[2];
    }
    return s;
}

// A whole round of n_dirs directions in one pass: the results and the state it leaves equal those of zo2_step(seeds[0])
// followed by zo2_step_extra(seeds[1]) ... bit for bit, but every module is visited once - a streamed block is uploaded
// once and runs the dual forwards of all directions while it sits in its slot.
extern "C" zo2_status zo2_step_multi(zo2_ctx* c, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq,
                                     int32_t n_dirs, const uint64_t* seeds, float eps, float lr, float* results) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!tokens || !labels || !seeds || !results) return fail(c, ZO2_EINVAL, "zo2_step_multi: NULL argument");
    if (n_dirs < 1 || n_dirs > zo2_ctx::kMaxPending) return fail(c, ZO2_EINVAL, "zo2_step_multi: %d directions (1 .. %d)", n_dirs, zo2_ctx::kMaxPending);
    if (!(eps != 0.f) || !isfinite(eps) || !isfinite(lr)) return fail(c, ZO2_EINVAL, "zo2_step_multi: eps must be non-zero and finite, lr finite");
    if (c->overlap_k1 && n_dirs > 1) return fail(c, ZO2_ESTATE, "zo2_step_multi: not available with the sweep kernel on a stream of its own");
    const zo2_status s = model_pass(c, "zo2_step_multi", tokens, labels, batch, seq, seeds, n_dirs, eps, lr, 2);
    if (s == ZO2_OK || s == ZO2_ENONFINITE)
        for (int j = 0; j < n_dirs; ++j) {
            const float* r = pass_result(c, j);
            results[3 * j] = r[0]; results[3 * j + 1] = r[1]; results[3 * j + 2] = r[2];
        }
    return s;
}

// ---------------------------------------------------------------------------------- evaluation (single forward)
extern "C" zo2_status zo2_eval(zo2_ctx* c, const int32_t* tokens, const int32_t* labels, int32_t batch, int32_t seq, float* loss) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!tokens || !labels || !loss) return fail(c, ZO2_EINVAL, "zo2_eval: NULL argument");
    const uint64_t no_seed = 0;
    const zo2_status s = model_pass(c, "zo2_eval", tokens, labels, batch, seq, &no_seed, 1, 0.f, 0.f, 1);
    if (s == ZO2_OK) *loss = c->h_result[0];
    return s;
}

// ---------------------------------------------------------------------------------- the deferred update as data
// What Sec. 5.4 carries from one iteration to the next: (seed, c = eta * g).  Together with the parameters
// (zo2_sync_to_host) this is the whole training state, so it is what a checkpoint has to hold.
extern "C" zo2_status zo2_pending_count(zo2_ctx* c, int32_t* n) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!n) return fail(c, ZO2_EINVAL, "zo2_pending_count: NULL argument");
    *n = c->n_pend;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_pending_at(zo2_ctx* c, int32_t i, uint64_t* seed, float* step) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!seed || !step) return fail(c, ZO2_EINVAL, "zo2_get_pending_at: NULL argument");
    if (i < 0 || i >= c->n_pend) return fail(c, ZO2_EINVAL, "zo2_get_pending_at: index %d of %d", i, c->n_pend);
    HIPCHK(c, hipMemcpyAsync(c->h_result + 8, coef_slot(c, i), sizeof(float), hipMemcpyDeviceToHost, c->sc));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    *seed = c->pend_seed[i];
    *step = c->h_result[8];
    return ZO2_OK;
}

extern "C" zo2_status zo2_add_pending(zo2_ctx* c, uint64_t seed, float step) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!isfinite(step)) return fail(c, ZO2_EINVAL, "zo2_add_pending: step must be finite");
    if (c->n_pend >= zo2_ctx::kMaxPending) return fail(c, ZO2_ESTATE, "zo2_add_pending: at most %d deferred updates", zo2_ctx::kMaxPending);
    c->h_result[8] = step;
    HIPCHK(c, hipMemcpyAsync(coef_slot(c, c->n_pend), c->h_result + 8, sizeof(float), hipMemcpyHostToDevice, c->sc));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    c->pend_seed[c->n_pend++] = seed;
    return ZO2_OK;
}

extern "C" zo2_status zo2_get_pending(zo2_ctx* c, int32_t* has_pending, uint64_t* seed, float* step) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (!has_pending || !seed || !step) return fail(c, ZO2_EINVAL, "zo2_get_pending: NULL argument");
    if (c->n_pend > 1) return fail(c, ZO2_ESTATE, "zo2_get_pending: %d updates are deferred; read them with zo2_get_pending_at", c->n_pend);
    *has_pending = c->n_pend;
    *seed = 0;
    *step = 0.f;
    return c->n_pend ? zo2_get_pending_at(c, 0, seed, step) : ZO2_OK;
}

extern "C" zo2_status zo2_set_pending(zo2_ctx* c, int32_t has_pending, uint64_t seed, float step) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (has_pending && !isfinite(step)) return fail(c, ZO2_EINVAL, "zo2_set_pending: step must be finite");
    c->n_pend = 0;
    return has_pending ? zo2_add_pending(c, seed, step) : ZO2_OK;
}

// ---------------------------------------------------------------------------------- flush
extern "C" zo2_status zo2_flush(zo2_ctx* c) {
    if (!c) return ZO2_EINVAL;
    if (c->dead) return ZO2_ESTATE;
    if (c->n_pend == 0) return writeback_pass(c);
    const zo2_config& g = c->cfg;
    if (!c->planned) return fail(c, ZO2_EINVAL, "zo2_flush: nothing to flush");
    c->apply_now = true;
    const int np = c->n_pend;       // every module takes all deferred updates, in order, while it is on the device
    for (int k = 0; k < np; ++k) { zo2_status s = k1_tensor(c, c->d_tok, c->tok_elems, 0, false, nullptr, nullptr, 0, 0.f, nullptr, k); if (s != ZO2_OK) return s; }
    for (int k = 0; k < np; ++k) { zo2_status s = k1_tensor(c, c->d_pos, c->pos_elems, 1, false, nullptr, nullptr, 0, 0.f, nullptr, k); if (s != ZO2_OK) return s; }
    c->bytes_up = c->bytes_down = 0;
    c->stat_u = c->stat_o = true;   // no span statistics for a flush
    int next_upload = 0;
    if (!c->resident)
        for (; next_upload < c->n_slots && next_upload < g.n_layers; ++next_upload) {
            zo2_status s = enqueue_upload(c, next_upload);
            if (s != ZO2_OK) return s;
        }
    for (int l = 0; l < g.n_layers; ++l) {
        if (c->resident) {
            for (int k = 0; k < np; ++k) {
                zo2_status s = k1_block(c, l, c->slots + (size_t)l * c->bucket_bytes, 0, ZO2_BLOCK_TENSORS, false, 0, 0.f, nullptr, k);
                if (s != ZO2_OK) return s;
            }
        } else {
            const int sl = l % c->n_slots;
            HIPCHK(c, hipStreamWaitEvent(c->sc, c->ev_up[sl], 0));
            { zo2_status s = stale_updates_block(c, l, c->slots + (size_t)sl * c->bucket_bytes); if (s != ZO2_OK) return s; }
            for (int k = 0; k < np; ++k) {
                zo2_status s = k1_block(c, l, c->slots + (size_t)sl * c->bucket_bytes, 0, ZO2_BLOCK_TENSORS, false, 0, 0.f, nullptr, k);
                if (s != ZO2_OK) return s;
            }
            HIPCHK(c, hipEventRecord(c->ev_k1[sl], c->sc));
            zo2_status s = enqueue_offload(c, l, true);
            if (s != ZO2_OK) return s;
            if (next_upload < g.n_layers) {
                s = enqueue_upload(c, next_upload++);
                if (s != ZO2_OK) return s;
            }
        }
    }
    for (int k = 0; k < np; ++k) { zo2_status s = k1_final_ln(c, false, 0, 0.f, k); if (s != ZO2_OK) return s; }
    if (c->d_lm)
        for (int k = 0; k < np; ++k) { zo2_status s = k1_tensor(c, c->d_lm, c->tok_elems, lm_tid(c), false, nullptr, nullptr, 0, 0.f, nullptr, k); if (s != ZO2_OK) return s; }
    HIPCHK(c, hipStreamSynchronize(c->sc));
    HIPCHK(c, hipStreamSynchronize(c->su));
    HIPCHK(c, hipStreamSynchronize(c->so));
    c->n_pend = 0;
    c->n_stale = 0;
    return ZO2_OK;
}

// =========================================================================================
// kernel-level entry points
// =========================================================================================
extern "C" zo2_status zo2_op_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t e0, uint64_t n, uint32_t* out, void* stream) {
    return philox_words(seed, tensor_id, e0, n, out, as_stream(stream));
}
extern "C" zo2_status zo2_op_gaussian(uint64_t seed, uint32_t tensor_id, uint64_t e0, uint64_t n, float* out, void* stream) {
    return gaussian(seed, tensor_id, e0, n, out, as_stream(stream));
}

extern "C" zo2_status zo2_op_update_perturb(void* theta, int32_t wire_dtype, void* w_plus, void* w_minus, int32_t compute_dtype,
                                            uint32_t tensor_id, uint64_t e0, uint64_t n, int32_t has_pending, uint64_t seed_prev,
                                            float cval, uint64_t seed, float eps, float scale, int32_t stochastic, void* stream) {
    if (n == 0) return ZO2_OK;
    const size_t ws = zo2_dtype_size(wire_dtype), cs = zo2_dtype_size(compute_dtype);
    ZO2_OP_CHECK(ws != 0 && cs != 0, ZO2_EINVAL, "update_perturb: unknown dtype");
    ZO2_OP_CHECK(w_plus != nullptr || w_minus == nullptr, ZO2_EINVAL, "update_perturb: W- without W+");
    ZO2_OP_CHECK(((uintptr_t)theta % (8 * ws)) == 0 && ((uintptr_t)w_plus % (8 * cs)) == 0 && ((uintptr_t)w_minus % (8 * cs)) == 0,
                 ZO2_EINVAL, "update_perturb: pointers must be aligned to 8 elements");
    K1Args a;
    memset(&a, 0, sizeof(a));
    a.theta = theta; a.w_plus = w_plus; a.w_minus = w_minus; a.w_off0 = 0; a.nseg = 1;
    a.c_imm = cval; a.c_ptr = nullptr; a.eps = eps; a.stochastic = stochastic != 0;
    a.k_prev = philox_keys(seed_prev); a.k_cur = philox_keys(seed);
    a.seg[0].off = 0; a.seg[0].e0 = e0; a.seg[0].n = n; a.seg[0].tensor_id = tensor_id; a.seg[0].scale = scale;
    return k1_launch(a, wire_dtype, compute_dtype, has_pending != 0, w_plus != nullptr, as_stream(stream));
}

// One block bucket, all 16 tensors in one grid: the launch the context issues per decoder block.
extern "C" zo2_status zo2_op_update_perturb_block(const zo2_config* cfg, int32_t layer, void* bucket, void* w_plus, void* w_minus,
                                                  int32_t has_pending, uint64_t seed_prev, float cval, uint64_t seed, float eps,
                                                  const float* host_scales, int32_t stochastic, void* stream) {
    char why[256];
    ZO2_OP_CHECK(config_ok(cfg, why, sizeof(why)), ZO2_EINVAL, "update_perturb_block: %s", why);
    ZO2_OP_CHECK(layer >= 0 && bucket != nullptr, ZO2_EINVAL, "update_perturb_block: bad layer or NULL bucket");
    ZO2_OP_CHECK(w_plus != nullptr || w_minus == nullptr, ZO2_EINVAL, "update_perturb_block: W- without W+");
    const size_t ws = zo2_dtype_size(cfg->wire_dtype), cs = zo2_dtype_size(cfg->compute_dtype);
    ZO2_OP_CHECK(((uintptr_t)bucket % (8 * ws)) == 0 && ((uintptr_t)w_plus % (8 * cs)) == 0 && ((uintptr_t)w_minus % (8 * cs)) == 0,
                 ZO2_EINVAL, "update_perturb_block: pointers must be aligned to 8 elements");
    int64_t offs[ZO2_BLOCK_TENSORS + 1], tn[ZO2_BLOCK_TENSORS];
    zo2_block_tensor_offsets(cfg, offs);
    block_tensor_elems(cfg, tn);
    K1Args a;
    memset(&a, 0, sizeof(a));
    a.theta = bucket; a.w_plus = w_plus; a.w_minus = w_minus; a.w_off0 = 0; a.nseg = ZO2_BLOCK_TENSORS;
    a.c_imm = cval; a.c_ptr = nullptr; a.eps = eps; a.stochastic = stochastic != 0;
    a.k_prev = philox_keys(seed_prev); a.k_cur = philox_keys(seed);
    for (int k = 0; k < ZO2_BLOCK_TENSORS; ++k) {
        K1Seg& sg = a.seg[k];
        sg.off = offs[k]; sg.e0 = 0; sg.n = (uint64_t)tn[k]; sg.tensor_id = block_tid(layer, k); sg.scale = host_scales ? host_scales[k] : 1.0f;
    }
    return k1_launch(a, cfg->wire_dtype, cfg->compute_dtype, has_pending != 0, w_plus != nullptr, as_stream(stream));
}

extern "C" zo2_status zo2_op_convert(const void* src, int32_t sdt, float sscale, void* dst, int32_t ddt, float dscale, uint64_t n, void* stream) {
    return convert(src, sdt, sscale, dst, ddt, dscale, n, as_stream(stream));
}

extern "C" zo2_status zo2_op_gemm(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                                  const void* bias, const float* residual, void* Y, int32_t out_dtype, int64_t ldy, float out_scale,
                                  int32_t relu, void* stream) {
    ZO2_OP_CHECK(out_dtype == ZO2_F32 || out_dtype == dtype, ZO2_EINVAL, "gemm: output dtype must be F32 or the input dtype");
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M; a.N = N; a.K = K; a.ldx = ldx; a.ldw = ldw; a.ldy = ldy; a.relu = relu; a.out_f32 = out_dtype == ZO2_F32; a.nprob = 1;
    a.p[0].X = X; a.p[0].W = W; a.p[0].bias = bias; a.p[0].residual = residual; a.p[0].Y = Y; a.p[0].out_scale = out_scale;
    return gemm_launch(a, dtype, as_stream(stream));
}

// zo2_op_gemm on the 256 x 256 kernel with one workgroup's cycle stamps (measurement build only)
extern "C" zo2_status zo2_op_gemm_phases(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                                         const float* residual, void* Y, int32_t out_dtype, int64_t ldy, uint64_t* stamps, void* stream) {
#ifdef ZO2_GEMM_STAMPS
    ZO2_OP_CHECK(stamps != nullptr, ZO2_EINVAL, "gemm_phases: stamps is NULL");
    ZO2_OP_CHECK(out_dtype == ZO2_F32 || out_dtype == dtype, ZO2_EINVAL, "gemm_phases: output dtype must be F32 or the input dtype");
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M; a.N = N; a.K = K; a.ldx = ldx; a.ldw = ldw; a.ldy = ldy; a.out_f32 = out_dtype == ZO2_F32; a.nprob = 1;
    a.p[0].X = X; a.p[0].W = W; a.p[0].residual = residual; a.p[0].Y = Y; a.p[0].out_scale = 1.0f;
    a.stamps = reinterpret_cast<unsigned long long*>(stamps);
    return gemm_launch_256(a, dtype, as_stream(stream));
#else
    (void)dtype; (void)M; (void)N; (void)K; (void)X; (void)ldx; (void)W; (void)ldw; (void)residual; (void)Y; (void)out_dtype; (void)ldy; (void)stamps; (void)stream;
    set_op_error("zo2_op_gemm_phases: this library was built without cycle stamps (build.py --gemm-stamps builds libzo2_stamps.so)");
    return ZO2_ESTATE;
#endif
}

extern "C" size_t zo2_op_gemm_split_k_workspace_bytes(int32_t M, int32_t N, int32_t splits) { return gemm_splitk_workspace_bytes(M, N, 1, splits); }

extern "C" int32_t zo2_op_gemm_split_k_pieces(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t nprob) { return gemm_pick_splits(M, N, K, nprob, dtype); }

extern "C" zo2_status zo2_op_gemm_split_k(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                                          const void* bias, const float* residual, void* Y, int32_t out_dtype, int64_t ldy, float out_scale,
                                          int32_t relu, int32_t splits, void* workspace, size_t workspace_bytes, void* stream) {
    if (M == 0 || N == 0) return ZO2_OK;
    ZO2_OP_CHECK(out_dtype == ZO2_F32 || out_dtype == dtype, ZO2_EINVAL, "gemm: output dtype must be F32 or the input dtype");
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M; a.N = N; a.K = K; a.ldx = ldx; a.ldw = ldw; a.ldy = ldy; a.relu = relu; a.out_f32 = out_dtype == ZO2_F32; a.nprob = 1;
    a.p[0].X = X; a.p[0].W = W; a.p[0].bias = bias; a.p[0].residual = residual; a.p[0].Y = Y; a.p[0].out_scale = out_scale;
    return gemm_launch_splitk(a, dtype, splits, workspace, workspace_bytes, as_stream(stream));
}

extern "C" size_t zo2_op_gemm_perturbed_workspace_bytes(int32_t M, int32_t N, int32_t K) { return skinny_workspace_bytes(M, N, K, 1); }

extern "C" zo2_status zo2_op_gemm_perturbed(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X_plus, const void* X_minus, int64_t ldx,
                                            const void* theta, uint32_t tensor_id, uint64_t seed, float eps, const void* bias_plus,
                                            const void* bias_minus, const float* residual_plus, const float* residual_minus, void* Y_plus,
                                            void* Y_minus, int32_t out_dtype, int64_t ldy, float out_scale, int32_t relu, void* workspace,
                                            size_t workspace_bytes, void* stream) {
    if (M == 0 || N == 0) return ZO2_OK;
    ZO2_OP_CHECK(out_dtype == ZO2_F32 || out_dtype == dtype, ZO2_EINVAL, "gemm_perturbed: output dtype must be F32 or the input dtype");
    SkinnyArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M; a.N = N; a.K = K; a.ldx = ldx; a.ldy = ldy; a.relu = relu; a.out_f32 = out_dtype == ZO2_F32; a.nprob = 1; a.eps = eps;
    a.key = philox_keys(seed);
    SkinnyProblem& p = a.p[0];
    p.Xp = X_plus; p.Xm = X_minus; p.theta = theta; p.bias_p = bias_plus; p.bias_m = bias_minus; p.res_p = residual_plus; p.res_m = residual_minus;
    p.Yp = Y_plus; p.Ym = Y_minus; p.out_scale = out_scale; p.tensor_id = tensor_id;
    return skinny_launch(a, dtype, workspace, workspace_bytes, as_stream(stream));
}

extern "C" zo2_status zo2_op_perturbed_rows(int32_t dtype, const void* theta, int64_t K, int64_t n0, int64_t rows, uint32_t tensor_id,
                                            uint64_t seed, float eps, void* w_plus, void* w_minus, void* stream) {
    return skinny_perturbed_rows(dtype, theta, K, n0, rows, tensor_id, seed, eps, w_plus, w_minus, as_stream(stream));
}

extern "C" zo2_status zo2_op_attention(int32_t dtype, const void* q, const void* k, const void* v, void* out, int32_t n_seq,
                                       int32_t seq, int32_t n_heads, int32_t d_head, int64_t ld, int32_t vector_kernel, void* stream) {
    return attention_launch(dtype, q, k, v, out, n_seq, seq, n_heads, d_head, ld, vector_kernel, as_stream(stream));
}

extern "C" zo2_status zo2_op_set_gemm_tile_rows(int32_t rows) {
    ZO2_OP_CHECK(rows == 0 || rows == 128 || rows == 256, ZO2_EINVAL, "zo2_op_set_gemm_tile_rows: %d (0, 128 or 256)", rows);
    gemm256_force_tile_rows(rows);
    return ZO2_OK;
}

extern "C" zo2_status zo2_op_set_gemm_wavefronts(int32_t waves) {
    ZO2_OP_CHECK(waves == 0 || waves == 4 || waves == 8, ZO2_EINVAL, "zo2_op_set_gemm_wavefronts: %d (0, 4 or 8)", waves);
    gemm256_force_waves(waves);
    return ZO2_OK;
}

extern "C" zo2_status zo2_op_layernorm(int32_t dtype, const float* x, const void* w, const void* b, const void* w2, const void* b2, void* y,
                                       int32_t rows, int32_t rows_first, int32_t d, float eps, void* stream) {
    return layernorm(dtype, x, w, b, w2, b2, y, rows, rows_first, d, eps, as_stream(stream));
}

extern "C" zo2_status zo2_op_cross_entropy_rows(const float* logits, int64_t ld, const int32_t* labels, int32_t rows, int32_t vocab,
                                                float* row_loss, void* stream) {
    return cross_entropy_rows(logits, ld, labels, rows, 0, rows > 0 ? rows : 1, vocab, row_loss, as_stream(stream));
}

extern "C" size_t zo2_op_lm_head_ce_workspace_bytes(int32_t M, int32_t N) {
    if (M <= 0 || N <= 0) return 0;
    const size_t parts = 4 * (((size_t)N + 255) / 256);
    return (2 * parts + 1) * (size_t)M * sizeof(float);
}

static zo2_status lm_head_ce_on(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                                const int32_t* labels, float* row_loss, void* workspace, hipStream_t st) {
    const int parts = 4 * ((N + 255) / 256);
    float* pmax = (float*)workspace;
    float* psum = pmax + (size_t)parts * M;
    float* lab = psum + (size_t)parts * M;
    GemmArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.M = M; ga.N = N; ga.K = K; ga.ldx = ldx; ga.ldw = ldw; ga.ldy = N; ga.out_f32 = 1; ga.nprob = 1; ga.ce_mode = 1; ga.part_ld = M;
    ga.p[0].X = X; ga.p[0].W = W; ga.p[0].out_scale = 1.0f; ga.p[0].labels = labels;
    ga.p[0].part_max = pmax; ga.p[0].part_sum = psum; ga.p[0].label_logit = lab;
    const zo2_status s = gemm_launch(ga, dtype, st);
    if (s != ZO2_OK) return s;
    return ce_combine(pmax, psum, lab, labels, M, parts, M, 0, M, row_loss, st);
}

extern "C" zo2_status zo2_op_lm_head_ce(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W,
                                        int64_t ldw, const int32_t* labels, float* row_loss, void* workspace, size_t workspace_bytes,
                                        void* stream) {
    if (M == 0) return ZO2_OK;
    ZO2_OP_CHECK(X && W && labels && row_loss && workspace, ZO2_EINVAL, "lm_head_ce: NULL argument");
    ZO2_OP_CHECK(dtype == ZO2_BF16 || dtype == ZO2_F16, ZO2_EINVAL, "lm_head_ce: dtype must be BF16 or F16");
    ZO2_OP_CHECK(M >= 256 && N >= 256 && K > 0 && K % 128 == 0 && N % 4 == 0, ZO2_EINVAL,
                 "lm_head_ce: needs M, N >= 256, K %% 128 == 0, N %% 4 == 0 (got %d x %d x %d)", M, N, K);
    ZO2_OP_CHECK(((uintptr_t)workspace & 255) == 0 && workspace_bytes >= zo2_op_lm_head_ce_workspace_bytes(M, N) && M > 0 && N > 0,
                 ZO2_EINVAL, "lm_head_ce: workspace too small or not 256-byte aligned");
    return lm_head_ce_on(dtype, M, N, K, X, ldx, W, ldw, labels, row_loss, workspace, as_stream(stream));
}

// ---------------------------------------------------------------------------------- LM head + cross-entropy without a workspace
// For callers that cannot allocate device memory: the partials live in a fixed array inside the library's
// code object.  Every GPU the library runs on holds its own copy of the array at its own address; in host
// code the array's name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[ZO2_STATIC_SCRATCH_BYTES];

static constexpr int kMaxStaticDevices = 64;
static void* g_static_scratch[kMaxStaticDevices];      // per device: where `scratch` lives there (NULL: not asked yet)
static std::mutex g_static_scratch_lock;

// The address of `scratch` on the current device, looked up once per device.
static zo2_status static_scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_op_error("lm_head_ce_static: hipGetDevice failed: %s", hipGetErrorString(e)); return ZO2_EHIP; }
    ZO2_OP_CHECK(dev >= 0 && dev < kMaxStaticDevices, ZO2_EINVAL, "lm_head_ce_static: device index %d beyond %d", dev, kMaxStaticDevices);
    std::lock_guard<std::mutex> guard(g_static_scratch_lock);
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_op_error("lm_head_ce_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return ZO2_EHIP;
        }
        g_static_scratch[dev] = p;
    }
    *out = g_static_scratch[dev];
    return ZO2_OK;
}

extern "C" zo2_status zo2_op_lm_head_ce_static(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W,
                                               int64_t ldw, const int32_t* labels, float* row_loss, void* stream) {
    if (M == 0) return ZO2_OK;
    ZO2_OP_CHECK(X && W && labels && row_loss, ZO2_EINVAL, "lm_head_ce_static: NULL argument");
    ZO2_OP_CHECK(dtype == ZO2_BF16 || dtype == ZO2_F16, ZO2_EINVAL, "lm_head_ce_static: dtype must be BF16 or F16");
    ZO2_OP_CHECK(M >= 256 && N >= 256 && K > 0 && K % 128 == 0 && N % 4 == 0, ZO2_EINVAL,
                 "lm_head_ce_static: needs M, N >= 256, K %% 128 == 0, N %% 4 == 0 (got %d x %d x %d)", M, N, K);
    const size_t need = zo2_op_lm_head_ce_workspace_bytes(M, N);
    ZO2_OP_CHECK(need <= (size_t)ZO2_STATIC_SCRATCH_BYTES, ZO2_EINVAL,
                 "lm_head_ce_static: %d rows x %d columns need %zu bytes of partials, the built-in buffer holds %zu; "
                 "use zo2_op_lm_head_ce with a workspace", M, N, need, (size_t)ZO2_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    const zo2_status s = static_scratch_address(&ws);
    if (s != ZO2_OK) return s;
    // every partial and label logit the second kernel reads is written by the first in the same call: nothing in the
    // buffer has to start at zero, and what an earlier (larger) call left behind is never read
    return lm_head_ce_on(dtype, M, N, K, X, ldx, W, ldw, labels, row_loss, ws, as_stream(stream));
}
