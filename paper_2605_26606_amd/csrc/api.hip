// Context, paged KV bookkeeping and the C ABI entry points (include/pc.h).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "kv_book.h"
#include "pc_internal.h"

// Scratch of pc_decode_step_static, the decode step that allocates nothing: one fixed array per GPU in the
// library's code object (every GPU the library is loaded on holds its own copy until the process ends).
// In host code this name is only a handle for hipGetSymbolAddress: the address kernels get is looked up once
// per device (static_scratch_base) and that pointer is what is passed on.
static constexpr size_t PC_STATIC_SCRATCH_BYTES = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[PC_STATIC_SCRATCH_BYTES];

namespace pc {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// Pinned host staging for the small control arrays that go to the device (block-table rows, row
// metadata, sequence lists).  An asynchronous copy reads its host source when the stream reaches it, so
// the source must stay untouched until then: every upload is copied into a fresh piece of a pinned ring
// first, and a piece is reused only after an event recorded behind its copies has completed.
struct Staging {
    static constexpr int N_FENCE = 16;
    char *base = nullptr;
    size_t cap = 0, head = 0, open_begin = 0;
    struct Fence {
        size_t begin = 0, end = 0;
        hipEvent_t ev = nullptr;
        bool pending = false;
    } fences[N_FENCE];
    int next_fence = 0;

    pc_status init(size_t bytes) {
        cap = (bytes + 4095) / 4096 * 4096;
        PC_HIP(hipHostMalloc((void **)&base, cap, hipHostMallocDefault));
        for (Fence &f : fences) PC_HIP(hipEventCreateWithFlags(&f.ev, hipEventDisableTiming));
        return PC_OK;
    }
    void destroy() {
        for (Fence &f : fences)
            if (f.ev) (void)hipEventDestroy(f.ev);
        if (base) (void)hipHostFree(base);
        base = nullptr;
    }
    // closes the pieces handed out since the last mark: they are free again once `st` has passed this point
    pc_status mark(hipStream_t st) {
        if (head == open_begin) return PC_OK;
        Fence &f = fences[next_fence];
        next_fence = (next_fence + 1) % N_FENCE;
        if (f.pending) PC_HIP(hipEventSynchronize(f.ev));
        f.begin = open_begin;
        f.end = head;
        PC_HIP(hipEventRecord(f.ev, st));
        f.pending = true;
        open_begin = head;
        return PC_OK;
    }
    // dst (device) <- src (host, n bytes) on stream st, through the ring
    pc_status push(void *dst, const void *src, size_t n, hipStream_t st) {
        if (n == 0) return PC_OK;
        const size_t need = (n + 63) / 64 * 64;
        if (need > cap / 2) PC_FAIL(PC_ERR_OOM, "staging: one upload of %zu bytes exceeds the ring", n);
        if (head + need > cap) {   // wrap: everything handed out so far has been enqueued on st
            pc_status rc = mark(st);
            if (rc != PC_OK) return rc;
            head = open_begin = 0;
        }
        for (Fence &f : fences)
            if (f.pending && f.begin < head + need && head < f.end) {
                PC_HIP(hipEventSynchronize(f.ev));
                f.pending = false;
            }
        memcpy(base + head, src, n);
        PC_HIP(hipMemcpyAsync(dst, base + head, n, hipMemcpyHostToDevice, st));
        head += need;
        return PC_OK;
    }
};

}  // namespace pc

using namespace pc;

struct pc_ctx {
    pc_model_config m;
    pc_cache_config c;
    int device = 0;
    int kd = KD_F32;      // kernel dtype of activations, KV cache and weight copies
    void *lm_head_copy = nullptr;   // half copy of lm_head (KD_F16)
    size_t esz = 2;
    // weights (library-owned fused copies, except embed / lm_head / final_norm)
    const void *tok_embed = nullptr, *lm_head = nullptr;
    const float *final_norm = nullptr;
    std::vector<void *> wqkv, wo, wgu, wdown;
    std::vector<float *> attn_norm, ffn_norm;
    // KV cache
    void *pool = nullptr;
    int64_t n_blocks = 0;
    int max_blocks_per_slot = 0;
    int32_t *d_block_table = nullptr, *d_slot_len = nullptr;
    KvBook book;   // slots, block lists, reference counts, free lists, host mirrors of the device tables
    float *rope_cos = nullptr, *rope_sin = nullptr;
    // activations
    float *h = nullptr, *qkv = nullptr, *attn_scratch = nullptr;
    float *score_logits = nullptr;    // pc_score: logits of score_rows rows at a time (allocated on first use)
    int score_rows = 0;
    void *a = nullptr, *q = nullptr, *attn = nullptr, *act = nullptr;
    void *h_act = nullptr;          // activation-type copy of the residual rows (fused decode path)
    float *ssq = nullptr;           // [d_model / 32][rows] partial sums of squares of the residual rows
    // 16-bit models: the library's weight copies are laid out for the fused decode kernels
    bool qkv_perm = false;          // q and k head rows in the order of qkv_packed_dim
    int fuse_decode = 1;            // PC_OPT_FUSE_DECODE
    int32_t *d_meta = nullptr;   // row_slot | row_pos | cu_rows | prompt_slot | last_rows | copy pairs
    int32_t *d_dec_slot = nullptr;
    float *slices = nullptr;       // split-K slices of the decode projections
    size_t slice_cap = 0;
    // the scratch the layer kernels use right now: the context's own buffers, or the static device array
    // of the entry point that allocates nothing
    float *cur_slices = nullptr, *cur_attn_scratch = nullptr;
    size_t cur_slice_cap = 0;
    unsigned char *static_scratch = nullptr;   // this device's copy of the static scratch array
    uint32_t *d_sat = nullptr;     // stores clamped to the half range (KD_F16)
    Staging stage;
    std::vector<int32_t> dec_seq;     // sequence list currently resident in d_dec_slot
    int dec_group = 1;                // consecutive entries of dec_seq that share a prompt
    std::vector<int32_t> stamp;
    int32_t stamp_gen = 0;
    // options
    int use_graph = 1, force_simt = 0;
    // captured decode step
    hipGraphExec_t exec = nullptr;
    struct {
        const void *tokens = nullptr, *logits = nullptr;
        hipStream_t stream = nullptr;
        int n = -1;
        uint64_t list_version = 0;
    } gkey;
    uint64_t list_version = 1;
    // event timing of one kernel class on selected eager steps
    int time_class = -1;
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    std::vector<hipEvent_t> ev_empty;   // back-to-back pairs with nothing between: the cost of the bracket itself
    size_t ev_empty_used = 0;

    KvGeom geom() const {
        KvGeom g;
        g.pool = pool;
        g.layer_stride = n_blocks * (int64_t)m.n_kv_heads * 2 * c.block_size * m.head_dim;
        g.block_size = c.block_size;
        g.n_kv_heads = m.n_kv_heads;
        g.head_dim = m.head_dim;
        g.max_blocks_per_slot = max_blocks_per_slot;
        g.block_table = d_block_table;
        return g;
    }
    int impl() const { return (kd != KD_F32 && !force_simt) ? 1 : 0; }
    bool mfma_attention() const { return impl() == 1 && m.head_dim == 128 && (m.n_q_heads / m.n_kv_heads) <= 16; }
};

namespace {

template <typename T> pc_status dev_alloc(T **p, size_t n_elems) {
    *p = nullptr;
    if (n_elems == 0) n_elems = 1;
    PC_HIP(hipMalloc((void **)p, n_elems * sizeof(T)));
    return PC_OK;
}

void free_all(pc_ctx *ctx) {
    if (ctx->exec) (void)hipGraphExecDestroy(ctx->exec);
    for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->ev_empty) (void)hipEventDestroy(e);
    auto fr = [](const void *p) { if (p) (void)hipFree(const_cast<void *>(p)); };
    for (auto p : ctx->wqkv) fr(p);
    for (auto p : ctx->wo) fr(p);
    for (auto p : ctx->wgu) fr(p);
    for (auto p : ctx->wdown) fr(p);
    for (auto p : ctx->attn_norm) fr(p);
    for (auto p : ctx->ffn_norm) fr(p);
    fr(ctx->pool); fr(ctx->d_block_table); fr(ctx->d_slot_len); fr(ctx->rope_cos); fr(ctx->rope_sin);
    fr(ctx->h); fr(ctx->qkv); fr(ctx->attn_scratch); fr(ctx->score_logits); fr(ctx->a); fr(ctx->q); fr(ctx->attn); fr(ctx->act);
    fr(ctx->d_meta); fr(ctx->d_dec_slot); fr(ctx->slices); fr(ctx->lm_head_copy); fr(ctx->d_sat);
    fr(ctx->h_act); fr(ctx->ssq);
    ctx->stage.destroy();
}

// uploads rows [s0, s1] of the host block table and slot lengths
pc_status upload_slots(pc_ctx *ctx, int s0, int s1, hipStream_t st) {
    if (s1 < s0) return PC_OK;
    const size_t w = ctx->max_blocks_per_slot;
    // in pieces: a single upload may not exceed half of the staging ring
    const int per = std::max<int>(1, (int)(ctx->stage.cap / 4 / (w * sizeof(int32_t))));
    for (int a = s0; a <= s1; a += per) {
        const int b = std::min(s1, a + per - 1);
        pc_status rc = ctx->stage.push(ctx->d_block_table + (size_t)a * w, ctx->book.h_table.data() + (size_t)a * w,
                                       (size_t)(b - a + 1) * w * sizeof(int32_t), st);
        if (rc != PC_OK) return rc;
    }
    return ctx->stage.push(ctx->d_slot_len + s0, ctx->book.h_len.data() + s0, (size_t)(s1 - s0 + 1) * sizeof(int32_t), st);
}

void release_slot(pc_ctx *ctx, int slot) { ctx->book.release(slot); }

// Brackets a launch with an event pair when its class is being timed.
struct Timed {
    pc_ctx *ctx;
    hipStream_t st;
    bool on;
    Timed(pc_ctx *c, int cls, hipStream_t s) : ctx(c), st(s), on(c->time_class == cls) {
        if (on) record();
    }
    ~Timed() {
        if (on) record();
    }
    void record() {
        if (ctx->ev_used == ctx->ev_pool.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) {
                on = false;
                return;
            }
            ctx->ev_pool.push_back(e);
        }
        (void)hipEventRecord(ctx->ev_pool[ctx->ev_used++], st);
    }
};

// One transformer layer stack over `rows` rows already embedded in ctx->h.
// prefill: cu_rows/prompt_slot describe the prompts (matrix-core attention); row_pos given.
// decode:  row_pos == nullptr, positions come from the device slot lengths.
// Returns the number of split-K slices of the last down projection still to be added to ctx->h
// (1: none pending); the caller's next launch_rmsnorm folds them in.
int enqueue_layers(pc_ctx *ctx, int rows, const int32_t *row_slot, const int32_t *row_pos, const int32_t *cu_rows,
                   const int32_t *prompt_slot, int n_prompts, int max_len, hipStream_t st) {
    const pc_model_config &m = ctx->m;
    const int dt = ctx->kd, impl = ctx->impl();
    const int qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
    const KvGeom kv = ctx->geom();
    const int n_splits = attention_decode_splits(rows, m.n_kv_heads, ctx->c.max_ctx);
    uint32_t *sat = ctx->d_sat;
    int pending = 1;
    // Decode batches of a 16-bit model on the matrix-core path: six launches per layer instead of eight.  The q/k/v
    // projection rotates q and k and appends k and v itself; the output projection updates the residual stream and
    // leaves the new rows times the next RMSNorm's gain plus that norm's row statistics, and the gate/up epilogue
    // applies the norm's scale.
    // (the fused projections own whole-K 64 x 32 tiles and re-read the activation rows once per 32 output columns:
    // that pays up to a few million weights per projection -- the 1.5B shape -- and loses to the K-sliced kernels
    // beyond, measured at the 8B shape)
    const bool fused = !row_pos && ctx->fuse_decode && impl == 1 && ctx->mfma_attention() && ctx->qkv_perm &&
                       skinny_ok(rows, qd + 2 * kvd, m.d_model, m.head_dim) &&
                       skinny_ok(rows, m.d_model, qd, m.head_dim) &&
                       (int64_t)(qd + 2 * kvd) * m.d_model <= ((int64_t)8 << 20) &&
                       (2 * m.d_ff) % 64 == 0;   // the gate/up epilogue with the norm scale exists on the matrix-core kernel only
    for (int l = 0; l < m.n_layers; ++l) {
        launch_rmsnorm(dt, ctx->h, nullptr, ctx->attn_norm[l], rows, m.d_model, m.rms_eps, ctx->a, ctx->cur_slices, pending,
                       sat, st);
        if (fused) {
            {
                Timed t(ctx, PC_KERNEL_GEMM_QKV, st);
                launch_skinny_qkv(dt, ctx->a, ctx->wqkv[l], rows, m.d_model, row_slot, ctx->d_slot_len, ctx->rope_cos,
                                  ctx->rope_sin, m.n_q_heads, kv, l, ctx->q, sat, st);
            }
            {
                Timed t(ctx, PC_KERNEL_ATTN_DECODE, st);
                launch_attention_decode_mfma(dt, ctx->q, row_slot, ctx->d_slot_len, rows, m.n_q_heads, kv, l, n_splits,
                                             ctx->dec_group, ctx->cur_attn_scratch, ctx->attn, sat, st);
            }
            launch_attention_decode_merge(dt, row_slot, ctx->d_slot_len, rows, m.n_q_heads, m.n_kv_heads, n_splits,
                                          ctx->cur_attn_scratch, ctx->attn, sat, st);
            {
                Timed t(ctx, PC_KERNEL_GEMM_WO, st);
                launch_skinny_o(dt, ctx->attn, ctx->wo[l], rows, m.d_model, qd, ctx->h, ctx->ffn_norm[l], ctx->h_act, ctx->ssq,
                                sat, st);
            }
            {
                Timed t(ctx, PC_KERNEL_GEMM_GATE_UP, st);
                const GemmRowScale rsc{ctx->ssq, m.d_model / 32, m.d_model, m.rms_eps};
                launch_gemm(dt, impl, ctx->h_act, ctx->wgu[l], ctx->act, rows, 2 * m.d_ff, m.d_model, EPI_SWIGLU_RS, nullptr,
                            0, sat, st, &rsc);
            }
            {
                Timed t(ctx, PC_KERNEL_GEMM_DOWN, st);
                pending = launch_gemm(dt, impl, ctx->act, ctx->wdown[l], ctx->h, rows, m.d_model, m.d_ff, EPI_RESID_F32,
                                      ctx->cur_slices, ctx->cur_slice_cap, sat, st);
            }
            continue;
        }
        int s_qkv;
        {
            Timed t(ctx, PC_KERNEL_GEMM_QKV, st);
            s_qkv = launch_gemm(dt, impl, ctx->a, ctx->wqkv[l], ctx->qkv, rows, qd + 2 * kvd, m.d_model, EPI_STORE_F32,
                                ctx->cur_slices, ctx->cur_slice_cap, sat, st);
        }
        launch_rope_append(dt, s_qkv > 1 ? ctx->cur_slices : ctx->qkv, s_qkv, row_slot, row_pos, ctx->d_slot_len,
                           ctx->rope_cos, ctx->rope_sin, rows, m.n_q_heads, kv, l, ctx->q, sat, ctx->qkv_perm ? 1 : 0, st);
        if (ctx->mfma_attention()) {
            if (row_pos)
                launch_attention_prefill_mfma(dt, ctx->q, cu_rows, prompt_slot, n_prompts, max_len, m.n_q_heads, kv, l,
                                              ctx->attn, sat, st);
            else {
                {
                    Timed t(ctx, PC_KERNEL_ATTN_DECODE, st);
                    launch_attention_decode_mfma(dt, ctx->q, row_slot, ctx->d_slot_len, rows, m.n_q_heads, kv, l, n_splits,
                                                 ctx->dec_group, ctx->cur_attn_scratch, ctx->attn, sat, st);
                }
                launch_attention_decode_merge(dt, row_slot, ctx->d_slot_len, rows, m.n_q_heads, m.n_kv_heads, n_splits,
                                              ctx->cur_attn_scratch, ctx->attn, sat, st);
            }
        } else {
            launch_attention_simt(dt, ctx->q, row_slot, row_pos, ctx->d_slot_len, rows, m.n_q_heads, kv, l, ctx->attn,
                                  sat, st);
        }
        int s_wo;
        {
            Timed t(ctx, PC_KERNEL_GEMM_WO, st);
            s_wo = launch_gemm(dt, impl, ctx->attn, ctx->wo[l], ctx->h, rows, m.d_model, qd, EPI_RESID_F32, ctx->cur_slices,
                               ctx->cur_slice_cap, sat, st);
        }
        launch_rmsnorm(dt, ctx->h, nullptr, ctx->ffn_norm[l], rows, m.d_model, m.rms_eps, ctx->a, ctx->cur_slices, s_wo, sat,
                       st);
        {
            Timed t(ctx, PC_KERNEL_GEMM_GATE_UP, st);
            launch_gemm(dt, impl, ctx->a, ctx->wgu[l], ctx->act, rows, 2 * m.d_ff, m.d_model, EPI_SWIGLU, nullptr, 0, sat,
                        st);
        }
        {
            Timed t(ctx, PC_KERNEL_GEMM_DOWN, st);
            pending = launch_gemm(dt, impl, ctx->act, ctx->wdown[l], ctx->h, rows, m.d_model, m.d_ff, EPI_RESID_F32,
                                  ctx->cur_slices, ctx->cur_slice_cap, sat, st);
        }
    }
    return pending;
}

void enqueue_decode(pc_ctx *ctx, const int32_t *tokens_in, int n, float *logits, hipStream_t st) {
    const pc_model_config &m = ctx->m;
    launch_embed(ctx->kd, ctx->tok_embed, tokens_in, n, m.d_model, m.vocab, ctx->h, st);
    const int pending = enqueue_layers(ctx, n, ctx->d_dec_slot, nullptr, nullptr, nullptr, 0, 0, st);
    launch_rmsnorm(ctx->kd, ctx->h, nullptr, ctx->final_norm, n, m.d_model, m.rms_eps, ctx->a, ctx->cur_slices, pending,
                   ctx->d_sat, st);
    {
        Timed t(ctx, PC_KERNEL_GEMM_LM_HEAD, st);
        launch_gemm(ctx->kd, ctx->impl(), ctx->a, ctx->lm_head, logits, n, m.vocab, m.d_model, EPI_STORE_F32, nullptr, 0,
                    ctx->d_sat, st);
    }
    launch_advance_len(ctx->d_slot_len, ctx->d_dec_slot, n, st);
}

// Device address of the static scratch array on `device` (which must be current): looked up once per device.
pc_status static_scratch_base(int device, unsigned char **out) {
    static std::mutex mu;
    static unsigned char *base[64] = {nullptr};
    if (device < 0 || device >= 64) PC_FAIL(PC_ERR_UNSUPPORTED, "device index %d outside 0..63", device);
    std::lock_guard<std::mutex> lock(mu);
    if (!base[device]) {
        void *p = nullptr;
        PC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) PC_FAIL(PC_ERR_HIP, "hipGetSymbolAddress returned no address for the static scratch array");
        base[device] = (unsigned char *)p;
    }
    *out = base[device];
    return PC_OK;
}

pc_status check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) PC_FAIL(PC_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return PC_OK;
}

}  // namespace

extern "C" {

const char *pc_last_error(void) { return g_err; }

pc_status pc_create(const pc_model_config *model, const pc_weights *w, const pc_cache_config *cache, pc_ctx **out) {
    if (!model || !w || !cache || !out) PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: null argument");
    *out = nullptr;
    const pc_model_config &m = *model;
    if (m.n_layers <= 0 || m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.head_dim <= 0 || m.d_ff <= 0 ||
        m.vocab <= 0 || !(m.rms_eps >= 0.f) || !(m.rope_theta > 0.f))
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: non-positive model dimension");
    if (m.dtype != PC_DTYPE_F32 && m.dtype != PC_DTYPE_BF16) PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: unknown dtype");
    if (m.act_dtype < PC_ACT_DEFAULT || m.act_dtype > PC_ACT_F16) PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: unknown act_dtype");
    if (m.n_q_heads % m.n_kv_heads) PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: n_q_heads not a multiple of n_kv_heads");
    if (m.head_dim % 2 || m.head_dim > 256) PC_FAIL(PC_ERR_UNSUPPORTED, "pc_create: head_dim must be even and <= 256");
    if (m.d_ff % 32) PC_FAIL(PC_ERR_UNSUPPORTED, "pc_create: d_ff must be a multiple of 32");
    if (cache->block_size <= 0 || cache->block_size % 32 || cache->block_size > 256)
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: block_size must be a multiple of 32, at most 256");
    if (cache->max_slots <= 0 || cache->max_ctx <= 0 || cache->max_batch_rows <= 0 || cache->kv_pool_bytes <= 0)
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: non-positive cache dimension");
    if (!w->tok_embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
        !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: null weight pointer");
    for (int l = 0; l < m.n_layers; ++l)
        if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] ||
            !w->w_up[l] || !w->w_down[l])
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_create: null weight pointer in layer %d", l);

    pc_ctx *ctx = new (std::nothrow) pc_ctx();
    if (!ctx) PC_FAIL(PC_ERR_OOM, "pc_create: host allocation failed");
    ctx->m = m;
    ctx->c = *cache;
    ctx->esz = (m.dtype == PC_DTYPE_F32) ? 4 : 2;
    ctx->kd = (m.dtype == PC_DTYPE_F32) ? KD_F32 : (m.act_dtype == PC_ACT_BF16 ? KD_BF16 : KD_F16);
    ctx->qkv_perm = ctx->kd != KD_F32 && m.head_dim == 128;
    pc_status rc = PC_OK;
#define TRY(expr)                 \
    do {                          \
        rc = (expr);              \
        if (rc != PC_OK) {        \
            free_all(ctx);        \
            delete ctx;           \
            return rc;            \
        }                         \
    } while (0)
#define TRY_HIP(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            set_error("%s failed: %s", #expr, hipGetErrorString(e_));                        \
            free_all(ctx);                                                                   \
            delete ctx;                                                                      \
            return PC_ERR_HIP;                                                               \
        }                                                                                    \
    } while (0)
    TRY_HIP(hipGetDevice(&ctx->device));
    TRY(static_scratch_base(ctx->device, &ctx->static_scratch));
    gemm_init();
    skinny_init();
    const size_t esz = ctx->esz;
    const int qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim;
    hipStream_t st = nullptr;

    // ---- fused weight copies
    ctx->tok_embed = w->tok_embed;
    ctx->lm_head = w->lm_head;
    ctx->final_norm = (const float *)w->final_norm;
    for (int l = 0; l < m.n_layers; ++l) {
        void *p;
        float *g;
        TRY(dev_alloc((char **)&p, (size_t)(qd + 2 * kvd) * m.d_model * esz));
        ctx->wqkv.push_back(p);
        launch_pack_rows(ctx->kd, w->wq[l], p, qd, m.d_model, 0, ctx->qkv_perm ? m.head_dim : 0, st);
        launch_pack_rows(ctx->kd, w->wk[l], p, kvd, m.d_model, qd, ctx->qkv_perm ? m.head_dim : 0, st);
        launch_pack_rows(ctx->kd, w->wv[l], p, kvd, m.d_model, qd + kvd, 0, st);
        TRY(dev_alloc((char **)&p, (size_t)m.d_model * qd * esz));
        ctx->wo.push_back(p);
        launch_pack_rows(ctx->kd, w->wo[l], p, m.d_model, qd, 0, 0, st);
        TRY(dev_alloc((char **)&p, (size_t)2 * m.d_ff * m.d_model * esz));
        ctx->wgu.push_back(p);
        launch_pack_gate_up(ctx->kd, w->w_gate[l], w->w_up[l], p, m.d_ff, m.d_model, st);
        TRY(dev_alloc((char **)&p, (size_t)m.d_model * m.d_ff * esz));
        ctx->wdown.push_back(p);
        launch_pack_rows(ctx->kd, w->w_down[l], p, m.d_model, m.d_ff, 0, 0, st);
        TRY(dev_alloc(&g, (size_t)m.d_model));
        ctx->attn_norm.push_back(g);
        TRY_HIP(hipMemcpyAsync(g, w->attn_norm[l], (size_t)m.d_model * 4, hipMemcpyDeviceToDevice, st));
        TRY(dev_alloc(&g, (size_t)m.d_model));
        ctx->ffn_norm.push_back(g);
        TRY_HIP(hipMemcpyAsync(g, w->ffn_norm[l], (size_t)m.d_model * 4, hipMemcpyDeviceToDevice, st));
    }

    if (ctx->kd == KD_F16) {   // the output projection is read through a half copy
        TRY(dev_alloc((char **)&ctx->lm_head_copy, (size_t)m.vocab * m.d_model * esz));
        launch_pack_rows(ctx->kd, w->lm_head, ctx->lm_head_copy, m.vocab, m.d_model, 0, 0, st);
        ctx->lm_head = ctx->lm_head_copy;
    }

    // ---- KV pool
    const int bs = cache->block_size;
    const int64_t block_bytes_all_layers = (int64_t)m.n_layers * m.n_kv_heads * 2 * bs * m.head_dim * (int64_t)esz;
    ctx->n_blocks = cache->kv_pool_bytes / block_bytes_all_layers;
    if (ctx->n_blocks <= 0 || ctx->n_blocks > 0x7fffffff) {
        set_error("pc_create: kv_pool_bytes holds %lld blocks of %lld bytes", (long long)ctx->n_blocks,
                  (long long)block_bytes_all_layers);
        free_all(ctx);
        delete ctx;
        return PC_ERR_INVALID_ARG;
    }
    TRY_HIP(hipMalloc(&ctx->pool, (size_t)(ctx->n_blocks * block_bytes_all_layers)));
    // stale cache entries are multiplied by zero probabilities: they must be finite
    TRY_HIP(hipMemsetAsync(ctx->pool, 0, (size_t)(ctx->n_blocks * block_bytes_all_layers), st));
    ctx->max_blocks_per_slot = (cache->max_ctx + bs - 1) / bs;
    TRY(dev_alloc(&ctx->d_block_table, (size_t)cache->max_slots * ctx->max_blocks_per_slot));
    TRY(dev_alloc(&ctx->d_slot_len, (size_t)cache->max_slots));
    TRY_HIP(hipMemsetAsync(ctx->d_block_table, 0, (size_t)cache->max_slots * ctx->max_blocks_per_slot * 4, st));
    TRY_HIP(hipMemsetAsync(ctx->d_slot_len, 0, (size_t)cache->max_slots * 4, st));
    ctx->book.init(bs, cache->max_slots, cache->max_ctx, ctx->n_blocks);
    ctx->stamp.assign(cache->max_slots, 0);

    // ---- rotary tables, angles in double
    {
        const int half = m.head_dim / 2;
        std::vector<float> cs((size_t)cache->max_ctx * half), sn((size_t)cache->max_ctx * half);
        for (int i = 0; i < half; ++i) {
            const double inv = pow((double)m.rope_theta, -2.0 * i / (double)m.head_dim);
            for (int p = 0; p < cache->max_ctx; ++p) {
                const double ang = (double)p * inv;
                cs[(size_t)p * half + i] = (float)cos(ang);
                sn[(size_t)p * half + i] = (float)sin(ang);
            }
        }
        TRY(dev_alloc(&ctx->rope_cos, cs.size()));
        TRY(dev_alloc(&ctx->rope_sin, sn.size()));
        TRY_HIP(hipMemcpy(ctx->rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice));
        TRY_HIP(hipMemcpy(ctx->rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice));
    }

    // ---- activations
    const size_t R = (size_t)cache->max_batch_rows;
    TRY(dev_alloc(&ctx->h, R * m.d_model));
    TRY(dev_alloc(&ctx->qkv, R * (qd + 2 * kvd)));
    TRY(dev_alloc((char **)&ctx->a, R * std::max(m.d_model, qd) * esz));
    TRY(dev_alloc((char **)&ctx->q, R * qd * esz));
    TRY(dev_alloc((char **)&ctx->attn, R * qd * esz));
    TRY(dev_alloc((char **)&ctx->act, R * m.d_ff * esz));
    if (ctx->kd != KD_F32) {
        const size_t Rd = std::min<size_t>(R, 512);   // the fused decode path takes at most 512 rows
        TRY(dev_alloc((char **)&ctx->h_act, Rd * m.d_model * esz));
        TRY(dev_alloc(&ctx->ssq, Rd * (size_t)((m.d_model + 31) / 32)));
    }
    TRY(dev_alloc(&ctx->attn_scratch,
                  attention_decode_scratch_floats(std::min<int>((int)R, cache->max_slots), m.n_q_heads, m.head_dim)));
    ctx->slice_cap = (size_t)8 << 20;   // 32 MB
    TRY(dev_alloc(&ctx->slices, ctx->slice_cap));
    ctx->cur_slices = ctx->slices;
    ctx->cur_slice_cap = ctx->slice_cap;
    ctx->cur_attn_scratch = ctx->attn_scratch;
    TRY(dev_alloc(&ctx->d_sat, 1));
    TRY_HIP(hipMemsetAsync(ctx->d_sat, 0, sizeof(uint32_t), st));
    // staging ring: four times the largest set of control arrays one call uploads
    TRY(ctx->stage.init(4 * ((2 * R + 8 * (size_t)cache->max_slots + 64) * sizeof(int32_t) +
                             (size_t)cache->max_slots * (ctx->max_blocks_per_slot + 1) * sizeof(int32_t))));
    ctx->dec_seq.reserve((size_t)cache->max_slots);
    TRY(dev_alloc(&ctx->d_meta, 2 * R + 3 * (size_t)cache->max_slots + 2 * (size_t)cache->max_slots + 16));
    TRY(dev_alloc(&ctx->d_dec_slot, (size_t)cache->max_slots));
    TRY_HIP(hipDeviceSynchronize());
    TRY(check_launch());
#undef TRY
#undef TRY_HIP
    *out = ctx;
    return PC_OK;
}

pc_status pc_destroy(pc_ctx *ctx) {
    if (!ctx) return PC_OK;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    delete ctx;
    return PC_OK;
}

pc_status pc_set_option(pc_ctx *ctx, int32_t option, int32_t value) {
    if (!ctx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_set_option: null context");
    switch (option) {
        case PC_OPT_USE_GRAPH: ctx->use_graph = value ? 1 : 0; break;
        case PC_OPT_FORCE_SIMT: ctx->force_simt = value ? 1 : 0; break;
        case PC_OPT_FUSE_DECODE: ctx->fuse_decode = value ? 1 : 0; break;
        case PC_OPT_TIME_NEXT_STEP:
            if (value < -1 || value > PC_KERNEL_GEMM_LM_HEAD) PC_FAIL(PC_ERR_INVALID_ARG, "pc_set_option: unknown kernel class");
            ctx->time_class = value;
            return PC_OK;   // a captured step stays valid
        default: PC_FAIL(PC_ERR_INVALID_ARG, "pc_set_option: unknown option %d", option);
    }
    ctx->gkey.n = -1;   // any captured step is stale
    return PC_OK;
}

pc_status pc_timing_read(pc_ctx *ctx, double *total_ms, int64_t *launches, double *empty_ms, int64_t *empty_pairs,
                         int32_t reset) {
    if (!ctx || !total_ms || !launches) PC_FAIL(PC_ERR_INVALID_ARG, "pc_timing_read: null argument");
    double tot = 0.0, etot = 0.0;
    int64_t cnt = 0, ecnt = 0;
    for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
        PC_HIP(hipEventSynchronize(ctx->ev_pool[i + 1]));
        float ms = 0.f;
        PC_HIP(hipEventElapsedTime(&ms, ctx->ev_pool[i], ctx->ev_pool[i + 1]));
        tot += (double)ms;
        ++cnt;
    }
    for (size_t i = 0; i + 1 < ctx->ev_empty_used; i += 2) {
        PC_HIP(hipEventSynchronize(ctx->ev_empty[i + 1]));
        float ms = 0.f;
        PC_HIP(hipEventElapsedTime(&ms, ctx->ev_empty[i], ctx->ev_empty[i + 1]));
        etot += (double)ms;
        ++ecnt;
    }
    *total_ms = tot;
    *launches = cnt;
    if (empty_ms) *empty_ms = etot;
    if (empty_pairs) *empty_pairs = ecnt;
    if (reset) ctx->ev_used = ctx->ev_empty_used = 0;
    return PC_OK;
}

pc_status pc_saturation_count(pc_ctx *ctx, int64_t *count, int32_t reset) {
    if (!ctx || !count) PC_FAIL(PC_ERR_INVALID_ARG, "pc_saturation_count: null argument");
    uint32_t v = 0;
    PC_HIP(hipDeviceSynchronize());
    PC_HIP(hipMemcpy(&v, ctx->d_sat, sizeof(v), hipMemcpyDeviceToHost));
    if (reset) PC_HIP(hipMemset(ctx->d_sat, 0, sizeof(v)));
    *count = (int64_t)v;
    return PC_OK;
}

pc_status pc_kv_blocks(const pc_ctx *ctx, int64_t *free_blocks, int64_t *total_blocks) {
    if (!ctx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_kv_blocks: null context");
    if (free_blocks) *free_blocks = (int64_t)ctx->book.free_blocks.size();
    if (total_blocks) *total_blocks = ctx->n_blocks;
    return PC_OK;
}

// What a scoring pass wants from the forward of the given sequences instead of the last rows' logits.
struct ScoreRequest {
    const int32_t *prompt_len;   // host [P]
    float temperature;
    float *out;                  // device, packed
};

// The forward of P packed sequences from position 0 (shared by pc_prefill_shared and pc_score): allocates a
// prompt slot and KV blocks per sequence, runs the layers in chunks of whole sequences, and then either
// writes the last row's logits of every sequence (last_logits) or the log-probabilities of the completion
// tokens (score).
static pc_status forward_chunks(pc_ctx *ctx, const int32_t *prompt_tokens, const int32_t *cu_lens, int32_t P,
                                const int32_t *handle_out, float *last_logits, const ScoreRequest *score, int smin,
                                int smax, hipStream_t st);

static pc_status forward_sequences(pc_ctx *ctx, const int32_t *prompt_tokens, const int32_t *cu_lens, int32_t P,
                                   int32_t *handle_out, float *last_logits, const ScoreRequest *score,
                                   hipStream_t st) {
    const int bs = ctx->c.block_size;
    if (cu_lens[0] != 0) PC_FAIL(PC_ERR_INVALID_ARG, "forward: cu_lens[0] must be 0");
    int64_t need_blocks = 0;
    for (int p = 0; p < P; ++p) {
        const int len = cu_lens[p + 1] - cu_lens[p];
        if (len <= 0) PC_FAIL(PC_ERR_INVALID_ARG, "forward: prompt %d is empty", p);
        if (len > ctx->c.max_ctx) PC_FAIL(PC_ERR_INVALID_ARG, "forward: prompt %d longer than max_ctx", p);
        if (len > ctx->c.max_batch_rows)
            PC_FAIL(PC_ERR_INVALID_ARG, "forward: prompt %d longer than max_batch_rows", p);
        need_blocks += (len + bs - 1) / bs;
    }
    if ((size_t)P > ctx->book.free_slots.size()) PC_FAIL(PC_ERR_OOM, "forward: out of slots");
    if ((size_t)need_blocks > ctx->book.free_blocks.size())
        PC_FAIL(PC_ERR_OOM, "forward: needs %lld KV blocks, %zu free", (long long)need_blocks,
                ctx->book.free_blocks.size());
    // ---- allocate
    int smin = ctx->c.max_slots, smax = -1;
    for (int p = 0; p < P; ++p) {
        const int len = cu_lens[p + 1] - cu_lens[p];
        const int slot = ctx->book.take_prompt(len);
        handle_out[p] = slot;
        smin = std::min(smin, slot);
        smax = std::max(smax, slot);
    }
    pc_status rc = forward_chunks(ctx, prompt_tokens, cu_lens, P, handle_out, last_logits, score, smin, smax, st);
    const pc_status rc_mark = ctx->stage.mark(st);
    if (rc == PC_OK) rc = rc_mark;
    if (rc != PC_OK) {   // a HIP call failed on the way: the slots and blocks taken above go back
        for (int p = 0; p < P; ++p) release_slot(ctx, handle_out[p]);
        ctx->dec_seq.clear();
        ctx->list_version++;
    }
    return rc;
}

static pc_status forward_chunks(pc_ctx *ctx, const int32_t *prompt_tokens, const int32_t *cu_lens, int32_t P,
                                const int32_t *handle_out, float *last_logits, const ScoreRequest *score, int smin,
                                int smax, hipStream_t st) {
    const pc_model_config &m = ctx->m;
    pc_status rc = upload_slots(ctx, smin, smax, st);
    if (rc != PC_OK) return rc;
    // ---- chunks of whole prompts, at most max_batch_rows rows each
    const size_t R = (size_t)ctx->c.max_batch_rows, S = (size_t)ctx->c.max_slots;
    int32_t *d_row_slot = ctx->d_meta, *d_row_pos = ctx->d_meta + R, *d_cu = ctx->d_meta + 2 * R,
            *d_pslot = d_cu + S + 1, *d_last = d_pslot + S;
    std::vector<int32_t> row_slot, row_pos, cu, pslot, last;
    size_t score_done = 0;   // completion tokens scored so far (offset into the packed output)
    int p0 = 0;
    while (p0 < P) {
        int p1 = p0, rows = 0, max_len = 0;
        while (p1 < P && rows + (cu_lens[p1 + 1] - cu_lens[p1]) <= (int)R) {
            rows += cu_lens[p1 + 1] - cu_lens[p1];
            ++p1;
        }
        row_slot.clear(); row_pos.clear(); cu.clear(); pslot.clear(); last.clear();
        cu.push_back(0);
        for (int p = p0; p < p1; ++p) {
            const int len = cu_lens[p + 1] - cu_lens[p];
            max_len = std::max(max_len, len);
            for (int i = 0; i < len; ++i) {
                row_slot.push_back(handle_out[p]);
                row_pos.push_back(i);
            }
            cu.push_back(cu.back() + len);
            pslot.push_back(handle_out[p]);
            last.push_back(cu.back() - 1);
        }
        const int np = p1 - p0;
        if ((rc = ctx->stage.push(d_row_slot, row_slot.data(), (size_t)rows * 4, st)) != PC_OK) return rc;
        if ((rc = ctx->stage.push(d_row_pos, row_pos.data(), (size_t)rows * 4, st)) != PC_OK) return rc;
        if ((rc = ctx->stage.push(d_cu, cu.data(), (size_t)(np + 1) * 4, st)) != PC_OK) return rc;
        if ((rc = ctx->stage.push(d_pslot, pslot.data(), (size_t)np * 4, st)) != PC_OK) return rc;
        if ((rc = ctx->stage.push(d_last, last.data(), (size_t)np * 4, st)) != PC_OK) return rc;
        launch_embed(ctx->kd, ctx->tok_embed, prompt_tokens + cu_lens[p0], rows, m.d_model, m.vocab, ctx->h, st);
        const int pending = enqueue_layers(ctx, rows, d_row_slot, d_row_pos, d_cu, d_pslot, np, max_len, st);
        if (pending > 1)   // small chunk whose last projection was split: fold the slices into h first
            launch_rmsnorm(ctx->kd, ctx->h, nullptr, ctx->final_norm, rows, m.d_model, m.rms_eps, ctx->a, ctx->cur_slices,
                           pending, ctx->d_sat, st);
        if (!score) {
            launch_rmsnorm(ctx->kd, ctx->h, d_last, ctx->final_norm, np, m.d_model, m.rms_eps, ctx->a, nullptr, 1,
                           ctx->d_sat, st);
            launch_gemm(ctx->kd, ctx->impl(), ctx->a, ctx->lm_head, last_logits + (size_t)p0 * m.vocab, np, m.vocab,
                        m.d_model, EPI_STORE_F32, nullptr, 0, ctx->d_sat, st);
        } else {
            // rows whose NEXT token belongs to a completion: positions prompt_len-1 .. len-2 of every sequence
            std::vector<int32_t> local, global;
            for (int p = p0; p < p1; ++p) {
                const int len = cu_lens[p + 1] - cu_lens[p];
                for (int i = score->prompt_len[p] - 1; i + 1 < len; ++i) {
                    local.push_back(cu[p - p0] + i);
                    global.push_back(cu_lens[p] + i);
                }
            }
            const int n_sc = (int)local.size();
            if (n_sc > 0) {
                // the row metadata is free again once the layers are enqueued (stream order)
                if ((rc = ctx->stage.push(d_row_slot, local.data(), (size_t)n_sc * 4, st)) != PC_OK) return rc;
                if ((rc = ctx->stage.push(d_row_pos, global.data(), (size_t)n_sc * 4, st)) != PC_OK) return rc;
                for (int off = 0; off < n_sc; off += ctx->score_rows) {
                    const int sr = std::min(ctx->score_rows, n_sc - off);
                    launch_rmsnorm(ctx->kd, ctx->h, d_row_slot + off, ctx->final_norm, sr, m.d_model, m.rms_eps, ctx->a,
                                   nullptr, 1, ctx->d_sat, st);
                    launch_gemm(ctx->kd, ctx->impl(), ctx->a, ctx->lm_head, ctx->score_logits, sr, m.vocab, m.d_model,
                                EPI_STORE_F32, nullptr, 0, ctx->d_sat, st);
                    launch_logprob(ctx->score_logits, sr, m.vocab, score->temperature, prompt_tokens, d_row_pos + off,
                                   score->out + score_done + off, st);
                }
                score_done += n_sc;
            }
        }
        rc = check_launch();
        if (rc != PC_OK) return rc;
        // the device-side metadata buffers are reused by the next chunk (stream order keeps that safe); the host
        // side of every copy above sits in the pinned ring until the stream has passed it
        p0 = p1;
    }
    return PC_OK;
}

pc_status pc_prefill_shared(pc_ctx *ctx, const int32_t *prompt_tokens, const int32_t *cu_lens, int32_t P,
                            int32_t *handle_out, float *last_logits, void *stream) {
    if (!ctx || !cu_lens || !handle_out) PC_FAIL(PC_ERR_INVALID_ARG, "pc_prefill_shared: null argument");
    if (P < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_prefill_shared: negative prompt count");
    if (P == 0) return PC_OK;
    if (!prompt_tokens || !last_logits) PC_FAIL(PC_ERR_INVALID_ARG, "pc_prefill_shared: null argument");
    return forward_sequences(ctx, prompt_tokens, cu_lens, P, handle_out, last_logits, nullptr, (hipStream_t)stream);
}

pc_status pc_score(pc_ctx *ctx, const int32_t *tokens, const int32_t *cu_lens, const int32_t *prompt_len, int32_t S,
                   float temperature, float *logprob_out, void *stream) {
    if (!ctx || !cu_lens || !prompt_len) PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: null argument");
    if (S < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: negative sequence count");
    if (S == 0) return PC_OK;
    if (!tokens || !logprob_out) PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: null argument");
    if (!(temperature > 0.f)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: temperature must be positive");
    if (cu_lens[0] != 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: cu_lens[0] must be 0");
    for (int i = 0; i < S; ++i) {
        const int len = cu_lens[i + 1] - cu_lens[i];
        if (prompt_len[i] < 1 || prompt_len[i] > len)
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_score: prompt_len[%d] = %d outside 1 .. %d", i, prompt_len[i], len);
    }
    if (!ctx->score_logits) {   // first use: room for the logits of up to 1024 rows at a time
        const int rows = std::min(ctx->c.max_batch_rows, 1024);
        pc_status rc = dev_alloc(&ctx->score_logits, (size_t)rows * ctx->m.vocab);
        if (rc != PC_OK) return rc;
        ctx->score_rows = rows;
    }
    std::vector<int32_t> handles((size_t)S, -1);
    ScoreRequest req{prompt_len, temperature, logprob_out};
    const pc_status rc = forward_sequences(ctx, tokens, cu_lens, S, handles.data(), nullptr, &req, (hipStream_t)stream);
    // the sequences were only passing through: their slots and blocks go back (work already enqueued keeps its
    // place in the stream ahead of whoever reuses them)
    for (int32_t h : handles)
        if (h >= 0 && ctx->book.slots[h].used) release_slot(ctx, h);
    ctx->dec_seq.clear();
    ctx->list_version++;
    return rc;
}

pc_status pc_slots(const pc_ctx *ctx, int64_t *free_slots, int64_t *total_slots) {
    if (!ctx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_slots: null context");
    if (free_slots) *free_slots = (int64_t)ctx->book.free_slots.size();
    if (total_slots) *total_slots = (int64_t)ctx->c.max_slots;
    return PC_OK;
}

pc_status pc_fork_need(const pc_ctx *ctx, const int32_t *prompt_handle, int32_t n, int32_t max_new_tokens,
                       int64_t *blocks_out) {
    if (!ctx || n < 0 || max_new_tokens < 0 || (n > 0 && (!prompt_handle || !blocks_out)))
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork_need: null argument or negative count");
    const int bs = ctx->c.block_size;
    for (int i = 0; i < n; ++i) {
        const int h = prompt_handle[i];
        if (h < 0 || h >= ctx->c.max_slots || !ctx->book.slots[h].used || !ctx->book.slots[h].is_prompt)
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork_need: entry %d is not a live prompt handle", i);
        const int len = ctx->book.slots[h].len;
        blocks_out[i] = (len + max_new_tokens + bs - 1) / bs - len / bs;
    }
    return PC_OK;
}

pc_status pc_fork(pc_ctx *ctx, const int32_t *prompt_handle, int32_t n, int32_t max_new_tokens, int32_t *seq_out,
                  void *stream) {
    if (!ctx || (n > 0 && (!prompt_handle || !seq_out))) PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork: null argument");
    if (n < 0 || max_new_tokens < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork: negative count");
    if (n == 0) return PC_OK;
    hipStream_t st = (hipStream_t)stream;
    const int bs = ctx->c.block_size;
    int64_t need_blocks = 0;
    for (int i = 0; i < n; ++i) {
        const int h = prompt_handle[i];
        if (h < 0 || h >= ctx->c.max_slots || !ctx->book.slots[h].used || !ctx->book.slots[h].is_prompt)
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork: entry %d is not a live prompt handle", i);
        const int len = ctx->book.slots[h].len;
        if (len + max_new_tokens > ctx->c.max_ctx)
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork: prompt length %d + %d new tokens exceeds max_ctx %d", len,
                    max_new_tokens, ctx->c.max_ctx);
        need_blocks += (len + max_new_tokens + bs - 1) / bs - len / bs;
    }
    if ((size_t)n > ctx->book.free_slots.size()) PC_FAIL(PC_ERR_OOM, "pc_fork: out of slots");
    if ((size_t)need_blocks > ctx->book.free_blocks.size())
        PC_FAIL(PC_ERR_OOM, "pc_fork: needs %lld KV blocks, %zu free", (long long)need_blocks, ctx->book.free_blocks.size());
    if ((size_t)n > (size_t)ctx->c.max_slots) PC_FAIL(PC_ERR_INVALID_ARG, "pc_fork: too many sequences");
    std::vector<int32_t> pairs;
    int smin = ctx->c.max_slots, smax = -1;
    for (int i = 0; i < n; ++i) {
        const int slot = ctx->book.take_fork(prompt_handle[i], max_new_tokens, pairs);
        seq_out[i] = slot;
        smin = std::min(smin, slot);
        smax = std::max(smax, slot);
    }
    pc_status rc = upload_slots(ctx, smin, smax, st);
    if (rc == PC_OK && !pairs.empty()) {
        int32_t *d_pairs = ctx->d_meta + 2 * (size_t)ctx->c.max_batch_rows + 3 * (size_t)ctx->c.max_slots + 8;
        rc = ctx->stage.push(d_pairs, pairs.data(), pairs.size() * 4, st);
        if (rc == PC_OK) {
            launch_copy_block(ctx->kd, ctx->geom(), ctx->m.n_layers, d_pairs, (int)pairs.size() / 2, st);
            rc = check_launch();
        }
    }
    const pc_status rc_mark = ctx->stage.mark(st);
    if (rc == PC_OK) rc = rc_mark;
    if (rc != PC_OK) {   // a HIP call failed on the way: nothing of this call is kept
        for (int i = 0; i < n; ++i) release_slot(ctx, seq_out[i]);
        ctx->dec_seq.clear();
        ctx->list_version++;
    }
    return rc;
}

pc_status pc_release(pc_ctx *ctx, const int32_t *ids, int32_t n, int32_t kind) {
    if (!ctx || (n > 0 && !ids)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_release: null argument");
    if (kind != 0 && kind != 1) PC_FAIL(PC_ERR_INVALID_ARG, "pc_release: kind must be 0 (sequence) or 1 (prompt)");
    for (int i = 0; i < n; ++i) {
        const int s = ids[i];
        if (s < 0 || s >= ctx->c.max_slots || !ctx->book.slots[s].used || ctx->book.slots[s].is_prompt != (kind == 1))
            PC_FAIL(PC_ERR_INVALID_ARG, "pc_release: entry %d is not a live %s", i, kind ? "prompt" : "sequence");
        for (int j = 0; j < i; ++j)
            if (ids[j] == s) PC_FAIL(PC_ERR_INVALID_ARG, "pc_release: entry %d repeats", i);
    }
    for (int i = 0; i < n; ++i) release_slot(ctx, ids[i]);
    ctx->dec_seq.clear();
    ctx->list_version++;
    return PC_OK;
}

// Argument checks of a decode step and the upload of its sequence list (shared by the two entry points).
static pc_status prepare_decode(pc_ctx *ctx, const int32_t *seq, const int32_t *tokens_in, int32_t n, float *logits,
                                hipStream_t st, const char *who) {
    if (!seq || !tokens_in || !logits) PC_FAIL(PC_ERR_INVALID_ARG, "%s: null argument", who);
    if (n > ctx->c.max_batch_rows) PC_FAIL(PC_ERR_INVALID_ARG, "%s: n exceeds max_batch_rows", who);
    const int32_t gen = ++ctx->stamp_gen;
    for (int i = 0; i < n; ++i) {
        const int s = seq[i];
        if (s < 0 || s >= ctx->c.max_slots || !ctx->book.slots[s].used || ctx->book.slots[s].is_prompt)
            PC_FAIL(PC_ERR_INVALID_ARG, "%s: entry %d is not a live sequence", who, i);
        if (ctx->stamp[s] == gen) PC_FAIL(PC_ERR_INVALID_ARG, "%s: sequence %d repeats", who, s);
        ctx->stamp[s] = gen;
        if (ctx->book.slots[s].len >= ctx->book.slots[s].limit)
            PC_FAIL(PC_ERR_INVALID_ARG, "%s: sequence %d already holds its %d tokens (prompt + reserved new tokens)", who,
                    s, ctx->book.slots[s].limit);
    }
    if ((int)ctx->dec_seq.size() != n || memcmp(ctx->dec_seq.data(), seq, (size_t)n * 4) != 0) {
        ctx->dec_seq.assign(seq, seq + n);   // within the capacity reserved at creation
        ctx->list_version++;
        // rollouts of one prompt that sit next to each other in the list share their prefix blocks
        int g = 1;
        while (g < n && ctx->book.slots[seq[g]].prompt == ctx->book.slots[seq[0]].prompt) ++g;
        bool uniform = (n % g == 0);
        for (int i = 0; uniform && i < n; i += g)
            for (int k = 1; k < g; ++k)
                if (ctx->book.slots[seq[i + k]].prompt != ctx->book.slots[seq[i]].prompt) uniform = false;
        ctx->dec_group = uniform ? g : 1;
        pc_status rc = ctx->stage.push(ctx->d_dec_slot, ctx->dec_seq.data(), (size_t)n * 4, st);
        if (rc == PC_OK) rc = ctx->stage.mark(st);
        if (rc != PC_OK) {
            ctx->dec_seq.clear();
            return rc;
        }
    }
    return PC_OK;
}

static void advance_host_lengths(pc_ctx *ctx, const int32_t *seq, int32_t n) {
    for (int i = 0; i < n; ++i) ctx->book.advance(seq[i]);
}

pc_status pc_decode_step(pc_ctx *ctx, const int32_t *seq, const int32_t *tokens_in, int32_t n, float *logits,
                         void *stream) {
    if (!ctx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_decode_step: null context");
    if (n < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_decode_step: negative count");
    if (n == 0) return PC_OK;
    hipStream_t st = (hipStream_t)stream;
    {
        const pc_status rc = prepare_decode(ctx, seq, tokens_in, n, logits, st, "pc_decode_step");
        if (rc != PC_OK) return rc;
    }
    if (ctx->use_graph && st != nullptr && ctx->time_class < 0) {   // the default stream cannot be captured
        const bool hit = ctx->exec && ctx->gkey.n == n && ctx->gkey.tokens == tokens_in && ctx->gkey.logits == logits &&
                         ctx->gkey.stream == st &&
                         ctx->gkey.list_version == ctx->list_version;
        if (!hit) {
            if (ctx->exec) {
                (void)hipGraphExecDestroy(ctx->exec);
                ctx->exec = nullptr;
            }
            hipGraph_t graph = nullptr;
            ctx->gkey.n = -1;   // no captured step until this one is instantiated
            PC_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
            enqueue_decode(ctx, tokens_in, n, logits, st);
            hipError_t e = hipStreamEndCapture(st, &graph);
            if (e != hipSuccess || !graph) {
                (void)hipGetLastError();
                PC_FAIL(PC_ERR_HIP, "pc_decode_step: stream capture failed: %s", hipGetErrorString(e));
            }
            e = hipGraphInstantiate(&ctx->exec, graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            if (e != hipSuccess) {
                ctx->exec = nullptr;
                PC_FAIL(PC_ERR_HIP, "pc_decode_step: graph instantiate failed: %s", hipGetErrorString(e));
            }
            ctx->gkey.n = n;
            ctx->gkey.tokens = tokens_in;
            ctx->gkey.logits = logits;
            ctx->gkey.stream = st;
            ctx->gkey.list_version = ctx->list_version;
        }
        PC_HIP(hipGraphLaunch(ctx->exec, st));
    } else {
        if (ctx->time_class >= 0) {   // calibrate: an event pair around nothing
            for (int k = 0; k < 2; ++k) {
                if (ctx->ev_empty_used == ctx->ev_empty.size()) {
                    hipEvent_t e;
                    if (hipEventCreate(&e) != hipSuccess) break;
                    ctx->ev_empty.push_back(e);
                }
                (void)hipEventRecord(ctx->ev_empty[ctx->ev_empty_used++], st);
            }
        }
        enqueue_decode(ctx, tokens_in, n, logits, st);
        ctx->time_class = -1;   // timing covers one step
        pc_status rc = check_launch();
        if (rc != PC_OK) return rc;
    }
    advance_host_lengths(ctx, seq, n);
    return PC_OK;
}

pc_status pc_decode_step_static(pc_ctx *ctx, const int32_t *seq, const int32_t *tokens_in, int32_t n, float *logits,
                                void *stream) {
    if (!ctx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_decode_step_static: null context");
    if (n < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_decode_step_static: negative count");
    if (n == 0) return PC_OK;
    hipStream_t st = (hipStream_t)stream;
    // what the step's kernels may use of the static array: the K slices of the split projections (at most 8
    // slices of n rows of the widest split output) and the partial results of the split attention
    const pc_model_config &m = ctx->m;
    const size_t width = (size_t)std::max(m.n_q_heads * m.head_dim + 2 * m.n_kv_heads * m.head_dim, m.d_model);
    const size_t slice_floats = (size_t)8 * (size_t)n * width;
    const size_t attn_floats = attention_decode_scratch_floats(n, m.n_q_heads, m.head_dim);
    const size_t slice_bytes = (slice_floats * sizeof(float) + 255) / 256 * 256;
    const size_t need = slice_bytes + attn_floats * sizeof(float);
    if (need > PC_STATIC_SCRATCH_BYTES)
        PC_FAIL(PC_ERR_INVALID_ARG,
                "pc_decode_step_static: %d sequences of this model need %zu bytes of scratch, the static array holds %zu "
                "(use pc_decode_step)", n, need, PC_STATIC_SCRATCH_BYTES);
    {
        const pc_status rc = prepare_decode(ctx, seq, tokens_in, n, logits, st, "pc_decode_step_static");
        if (rc != PC_OK) return rc;
    }
    // same kernels, same launch shapes and the same K-slice decisions as pc_decode_step (cur_slice_cap keeps the
    // context's value; the slices actually written never exceed slice_floats), only the scratch is the static array
    const int saved_time_class = ctx->time_class;
    ctx->time_class = -1;   // per-launch event timing creates events: not here
    ctx->cur_slices = (float *)ctx->static_scratch;
    ctx->cur_attn_scratch = (float *)(ctx->static_scratch + slice_bytes);
    enqueue_decode(ctx, tokens_in, n, logits, st);
    ctx->cur_slices = ctx->slices;
    ctx->cur_attn_scratch = ctx->attn_scratch;
    ctx->time_class = saved_time_class;
    const pc_status rc = check_launch();
    if (rc != PC_OK) return rc;
    advance_host_lengths(ctx, seq, n);
    return PC_OK;
}

pc_status pc_sample(const float *logits, const int32_t *logit_row, int32_t n, int32_t vocab, float temperature,
                    float top_p, uint64_t seed, const uint64_t *seq_uid, const int32_t *step, int32_t step_base,
                    int32_t eos_id, float eos_logit_bias, int32_t *tokens_out, float *logprob_out, uint8_t *finished,
                    int32_t *hist_tokens, float *hist_logprob, const int32_t *hist_index, void *stream) {
    if (n < 0 || vocab <= 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: bad count");
    if (n == 0) return PC_OK;
    if (!logits || !seq_uid || !tokens_out) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: null argument");
    if (!(temperature > 0.f)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: temperature must be positive");
    if (!(top_p > 0.f && top_p <= 1.f)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: top_p must lie in (0, 1]");
    if (eos_id >= vocab) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: eos_id outside the vocabulary");
    if (finished && eos_id < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: finished flags need an eos_id");
    if (hist_index && !hist_tokens && !hist_logprob)
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_sample: hist_index without a history destination");
    launch_sample(logits, logit_row, n, vocab, temperature, top_p, seed, seq_uid, step, step_base, eos_id, eos_logit_bias,
                  tokens_out, logprob_out, finished, hist_tokens, hist_logprob, hist_index, (hipStream_t)stream);
    return check_launch();
}

pc_status pc_group_stats(const float *rewards, const int32_t *group_off, int32_t P, int32_t *n_pos, int32_t *n_tot,
                         float *mean, float *var, void *stream) {
    if (P < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_group_stats: negative group count");
    if (P == 0) return PC_OK;
    if (!rewards || !group_off) PC_FAIL(PC_ERR_INVALID_ARG, "pc_group_stats: null argument");
    launch_group_stats(rewards, group_off, P, n_pos, n_tot, mean, var, (hipStream_t)stream);
    return check_launch();
}

pc_status pc_select_commit(const float *p_hat, int32_t P, float p_lower, float p_upper, float p_solve, int32_t b_t,
                           uint8_t *cls, uint8_t *evict, int32_t *commit_idx, int32_t *surplus_idx, int32_t *counts,
                           void *stream) {
    if (P < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit: negative prompt count");
    if (!counts || (P > 0 && (!p_hat || !commit_idx))) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit: null argument");
    if (!(p_lower <= p_upper)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit: p_lower > p_upper");
    if (b_t > 0 && !surplus_idx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit: a cap needs surplus_idx");
    launch_select_commit(p_hat, P, p_lower, p_upper, p_solve, b_t, cls, evict, commit_idx, surplus_idx, counts,
                         (hipStream_t)stream);
    return check_launch();
}

pc_status pc_select_commit_var(const float *mean, const float *var, int32_t P, float var_hard, float var_easy,
                               float mean_pivot, float mean_solve, int32_t b_t, uint8_t *cls, uint8_t *evict,
                               int32_t *commit_idx, int32_t *surplus_idx, int32_t *counts, void *stream) {
    if (P < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit_var: negative prompt count");
    if (!counts || (P > 0 && (!mean || !var || !commit_idx))) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit_var: null argument");
    if (!(var_hard >= 0.f) || !(var_easy >= 0.f))
        PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit_var: a variance threshold is negative or not a number");
    if (b_t > 0 && !surplus_idx) PC_FAIL(PC_ERR_INVALID_ARG, "pc_select_commit_var: a cap needs surplus_idx");
    launch_select_commit_var(mean, var, P, var_hard, var_easy, mean_pivot, mean_solve, b_t, cls, evict, commit_idx,
                             surplus_idx, counts, (hipStream_t)stream);
    return check_launch();
}

pc_status pc_advantages(const float *rewards, const int32_t *group_off, int32_t P, float eps, float *adv, float *mu,
                        float *sigma, void *stream) {
    if (P < 0) PC_FAIL(PC_ERR_INVALID_ARG, "pc_advantages: negative group count");
    if (P == 0) return PC_OK;
    if (!rewards || !group_off || !adv) PC_FAIL(PC_ERR_INVALID_ARG, "pc_advantages: null argument");
    if (!(eps >= 0.f)) PC_FAIL(PC_ERR_INVALID_ARG, "pc_advantages: negative eps");
    launch_advantages(rewards, group_off, P, eps, adv, mu, sigma, (hipStream_t)stream);
    return check_launch();
}

}  // extern "C"
