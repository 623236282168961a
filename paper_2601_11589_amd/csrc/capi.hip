// C ABI of liblaps: context, workspace carving, the layer / stack driver, captured short-bucket
// graphs, per-kernel event timing.  Every device step is a kernel from gemm.hip, elementwise.hip or
// attention.hip; this file only sequences launches on the caller's stream.
#include <climits>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "laps_internal.h"

// ----------------------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

void laps_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
extern "C" const char* laps_last_error(void) { return g_err; }
extern "C" const char* laps_version(void) { return "laps-gfx950 0.1"; }

// ----------------------------------------------------------------------------- static scratch
// Workspace of laps_prefill_stack_static, for callers that may not allocate.  The array lives in this code
// object's device image: every GPU the library is loaded on holds its own copy at its own address for the life
// of the process.  In host code the array's name is only a handle for hipGetSymbolAddress; the address the
// kernels are given is the one resolved below, per device, with that device current.
#define LAPS_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
static __device__ __align__(256) unsigned char scratch[LAPS_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];   // resolved address per device ordinal, nullptr = not yet
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the CURRENT device (which must be `device`).  Resolved once per device.
static int resolve_static_scratch(int device, unsigned char** out) {
    if (device < 0 || device >= kMaxDevices) {
        laps_set_error("static scratch: device ordinal %d out of range", device);
        return LAPS_EINVAL;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            laps_set_error("static scratch: hipGetSymbolAddress failed on device %d: %s", device, hipGetErrorString(e));
            return LAPS_EHIP;
        }
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return LAPS_OK;
}

// ----------------------------------------------------------------------------- context
struct laps_ctx {
    laps_model_cfg cfg;
    int device;
    int max_pos;
    int pool_pages;  // page ids must be below this (INT_MAX: unknown, not checked)
    float2* rope;  // [max_pos][hd/2] (cos, sin)
    unsigned char* static_ws;  // this device's copy of the static scratch array (resolved at creation)
    // timing
    bool prof_on;
    std::vector<hipEvent_t> ev;  // pairs (start, stop)
    std::vector<int> ev_class;
    size_t ev_used;
};

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
    size_t tok_pos, tok_slot, new_len, tile_start, item_seq, r, q, attn, act, x_mid, partial, total;
};

static size_t partial_bytes_for(const laps_model_cfg& c, int m) {
    const int qd = c.n_q_heads * c.head_dim, qkv = qd + 2 * c.n_kv_heads * c.head_dim;
    size_t b = laps_gemm_partial_bytes(m, qkv, c.hidden);
    size_t t = laps_gemm_partial_bytes(m, c.hidden, qd);
    b = t > b ? t : b;
    t = laps_gemm_partial_bytes(m, 2 * c.intermediate, c.hidden);
    b = t > b ? t : b;
    t = laps_gemm_partial_bytes(m, c.hidden, c.intermediate);
    return t > b ? t : b;
}

// max_pages: width of the page tables the workspace will serve (default: any width)
static WsLayout ws_layout(const laps_model_cfg& c, int max_tokens, int max_seqs, int max_pages = 1 << 24) {
    WsLayout w;
    const size_t M = (size_t)max_tokens;
    const int qd = c.n_q_heads * c.head_dim;
    size_t o = 0;
    w.tok_pos = o;    o += align256(M * 4);
    w.tok_slot = o;   o += align256(M * 4);
    w.new_len = o;    o += align256((size_t)max_seqs * 4);
    w.tile_start = o; o += align256((size_t)(max_seqs + 1) * 4);
    w.item_seq = o;   o += align256(laps_attn_item_table_bytes(max_tokens, max_seqs, c.n_q_heads / c.n_kv_heads));
    w.r = o;          o += align256(M * c.hidden * 2);
    w.q = o;          o += align256(M * qd * 2);
    w.attn = o;       o += align256(M * qd * 2);
    w.act = o;        o += align256(M * c.intermediate * 2);
    w.x_mid = o;      o += align256(M * c.hidden * 4);
    // split-K partial sums: the split factor depends on the number of row tiles, and the byte count
    // grows with m inside one row-tile count, so the maximum over m <= max_tokens is reached at a
    // row-tile boundary (or at max_tokens, or at the largest skinny m = 128).
    size_t pb = partial_bytes_for(c, max_tokens);
    if (max_tokens > 128) {
        const size_t t = partial_bytes_for(c, 128);
        pb = t > pb ? t : pb;
    }
    for (int m = 256; m < max_tokens; m += 256) {
        const size_t t = partial_bytes_for(c, m);
        pb = t > pb ? t : pb;
    }
    {   // the same region holds the attention's key-split partial results (the two uses never overlap in time)
        const size_t t = laps_attn_partial_bytes(c.head_dim, max_pages);
        pb = t > pb ? t : pb;
    }
    w.partial = o;    o += align256(pb);
    w.total = o;
    return w;
}

static int check_cfg(const laps_model_cfg* c) {
    if (!c) return 0;
    const int qd = c->n_q_heads * c->head_dim, qkv = qd + 2 * c->n_kv_heads * c->head_dim;
    if (c->head_dim != 64 && c->head_dim != 128) return 0;
    if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return 0;
    if (c->hidden < 128 || c->hidden % 128 || qd % 64 || c->intermediate < 64 || c->intermediate % 64) return 0;
    if (qkv % 128 || (2 * c->intermediate) % 128) return 0;
    if (c->hidden > 8192) return 0;
    if (c->page_size != LAPS_PAGE || c->n_layers < 1) return 0;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps > 0.f)) return 0;
    return 1;
}

extern "C" int laps_ctx_create(const laps_model_cfg* cfg, int32_t max_positions, laps_ctx** out) {
    if (!out || !check_cfg(cfg) || max_positions < 1) {
        laps_set_error("ctx_create: unsupported model shape or max_positions < 1");
        return LAPS_EINVAL;
    }
    laps_ctx* c = new (std::nothrow) laps_ctx();
    if (!c) {
        laps_set_error("ctx_create: out of host memory");
        return LAPS_ENOMEM;
    }
    c->cfg = *cfg;
    c->max_pos = max_positions;
    c->pool_pages = INT_MAX;
    c->rope = nullptr;
    c->static_ws = nullptr;
    c->prof_on = false;
    c->ev_used = 0;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipMalloc(&c->rope, (size_t)max_positions * (cfg->head_dim / 2) * sizeof(float2));
    if (e != hipSuccess) {
        laps_set_error("ctx_create: %s", hipGetErrorString(e));
        delete c;
        return e == hipErrorOutOfMemory ? LAPS_ENOMEM : LAPS_EHIP;
    }
    int rc = resolve_static_scratch(c->device, &c->static_ws);   // the context's device is current here
    if (rc == LAPS_OK) rc = laps_launch_rope_table(c->rope, max_positions, cfg->head_dim, cfg->rope_theta, nullptr);
    if (rc == LAPS_OK && hipDeviceSynchronize() != hipSuccess) {
        laps_set_error("ctx_create: rope table kernel failed");
        rc = LAPS_EHIP;
    }
    if (rc != LAPS_OK) {
        (void)hipFree(c->rope);
        delete c;
        return rc;
    }
    *out = c;
    return LAPS_OK;
}

extern "C" void laps_ctx_destroy(laps_ctx* c) {
    if (!c) return;
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    if (c->rope) (void)hipFree(c->rope);
    delete c;
}

extern "C" size_t laps_workspace_bytes_for(const laps_model_cfg* cfg, int32_t max_tokens, int32_t max_seqs) {
    if (!check_cfg(cfg) || max_tokens < 1 || max_seqs < 1) return 0;
    return ws_layout(*cfg, max_tokens, max_seqs).total;
}

extern "C" int laps_ctx_set_pool_pages(laps_ctx* c, int32_t n_pages) {
    if (!c || n_pages < 0) {
        laps_set_error("ctx_set_pool_pages: NULL context or negative page count");
        return LAPS_EINVAL;
    }
    c->pool_pages = n_pages == 0 ? INT_MAX : n_pages;
    return LAPS_OK;
}

extern "C" size_t laps_workspace_bytes(const laps_ctx* c, int32_t max_tokens, int32_t max_seqs) {
    if (!c || max_tokens < 1 || max_seqs < 1) return 0;
    return ws_layout(c->cfg, max_tokens, max_seqs).total;
}

// ----------------------------------------------------------------------------- timing
struct ProfScope {
    laps_ctx* c;
    hipStream_t s;
    bool on;
    ProfScope(laps_ctx* ctx, hipStream_t st, int cls, bool capturing) : c(ctx), s(st), on(ctx->prof_on && !capturing) {
        if (!on) return;
        if (c->ev_used + 2 > c->ev.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
                on = false;
                return;
            }
            c->ev.push_back(a);
            c->ev.push_back(b);
        }
        c->ev_class.resize(c->ev.size() / 2);
        c->ev_class[c->ev_used / 2] = cls;
        (void)hipEventRecord(c->ev[c->ev_used], s);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(c->ev[c->ev_used + 1], s);
        c->ev_used += 2;
    }
};

extern "C" int laps_prof_enable(laps_ctx* c, int32_t on) {
    if (!c) return LAPS_EINVAL;
    c->prof_on = on != 0;
    c->ev_used = 0;
    return LAPS_OK;
}

extern "C" int laps_prof_read(laps_ctx* c, double* ms_out, int64_t* count_out) {
    if (!c || !ms_out || !count_out) return LAPS_EINVAL;
    for (int i = 0; i < LAPS_K_COUNT; ++i) {
        ms_out[i] = 0.0;
        count_out[i] = 0;
    }
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        LAPS_HIP(hipEventSynchronize(c->ev[i + 1]));
        float ms = 0.f;
        LAPS_HIP(hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]));
        const int cls = c->ev_class[i / 2];
        ms_out[cls] += ms;
        count_out[cls] += 1;
    }
    c->ev_used = 0;
    return LAPS_OK;
}

// ----------------------------------------------------------------------------- layer driver
struct BatchDesc {
    int n_seq, n_tokens;
    const int *row_start, *seq_len, *prefix_len, *page_table;
    int max_pages;
};

#define LAPS_TRY(x)                 \
    do {                            \
        int rc_ = (x);              \
        if (rc_ != LAPS_OK) return rc_; \
    } while (0)

// One projection.  `want` is the epilogue the caller would like fused; the plan falls back to raw
// K-slice partial sums when it splits K.  Returns the plan so the caller knows which case ran.
static int run_gemm(laps_ctx* c, int cls, bool capturing, const bf16_t* a, const bf16_t* w, int m, int n, int k,
                    int want, float* partial, float* out_f32, const float* resid, bf16_t* out_bf16, const int* row_live,
                    GemmPlan* plan, hipStream_t s) {
    const GemmPlan p = laps_gemm_plan(m, n, k, 0, want);
    *plan = p;
    ProfScope ps(c, s, cls, capturing);
    if (p.epi == EPI_PARTIAL) return laps_gemm_launch(p, a, w, m, n, k, partial, nullptr, nullptr, row_live, s);
    return laps_gemm_launch(p, a, w, m, n, k, out_f32, resid, out_bf16, row_live, s);
}

// Runs layers [0, n_layers) of `w`.  Token metadata (prep) is computed once.  r0_staged: the first layer's normed
// rows, with token metadata and the attention's work-item table already in the workspace (a captured graph:
// laps_graph_stage prepared them, so that a replay starts with the first projection).
static int run_layers(laps_ctx* c, const laps_layer_weights* w, int n_layers, const BatchDesc& b, void* const* k_pools,
                      void* const* v_pools, const float* x_in, float* x_out, unsigned char* ws, bool capturing,
                      hipStream_t s, const bf16_t* r0_staged = nullptr) {
    const laps_model_cfg& cf = c->cfg;
    const int M = b.n_tokens, d = cf.hidden, hd = cf.head_dim;
    const int qd = cf.n_q_heads * hd, qkv = qd + 2 * cf.n_kv_heads * hd, I = cf.intermediate;
    const WsLayout L = ws_layout(cf, M, b.n_seq);
    int* tok_pos = reinterpret_cast<int*>(ws + L.tok_pos);
    int* tok_slot = reinterpret_cast<int*>(ws + L.tok_slot);
    int* new_len = reinterpret_cast<int*>(ws + L.new_len);
    int* tile_start = reinterpret_cast<int*>(ws + L.tile_start);
    int* item_seq = reinterpret_cast<int*>(ws + L.item_seq);
    bf16_t* r = reinterpret_cast<bf16_t*>(ws + L.r);
    bf16_t* q = reinterpret_cast<bf16_t*>(ws + L.q);
    bf16_t* attn = reinterpret_cast<bf16_t*>(ws + L.attn);
    bf16_t* act = reinterpret_cast<bf16_t*>(ws + L.act);
    float* x_mid = reinterpret_cast<float*>(ws + L.x_mid);
    float* partial = reinterpret_cast<float*>(ws + L.partial);

    if (r0_staged == nullptr) {
        {
            ProfScope ps(c, s, LAPS_K_PREP, capturing);
            LAPS_TRY(laps_launch_prep(M, b.n_seq, b.row_start, b.seq_len, b.prefix_len, b.page_table, b.max_pages,
                                      c->pool_pages, new_len, tok_pos, tok_slot, s));
        }
        {
            ProfScope ps(c, s, LAPS_K_PREP, capturing);
            LAPS_TRY(laps_launch_attn_sched(new_len, b.n_seq, M, b.max_pages, tile_start, item_seq, cf.n_q_heads, cf.n_kv_heads, s));
        }
        {
            ProfScope ps(c, s, LAPS_K_RMSNORM, capturing);
            LAPS_TRY(laps_launch_rmsnorm(x_in, static_cast<const bf16_t*>(w[0].ln1_w), r, M, d, cf.rms_eps, tok_pos, s));
        }
    }
    for (int l = 0; l < n_layers; ++l) {
        const laps_layer_weights& lw = w[l];
        const float* resid = (l == 0) ? x_in : x_out;
        bf16_t* kp = static_cast<bf16_t*>(k_pools[l]);
        bf16_t* vp = static_cast<bf16_t*>(v_pools[l]);
        GemmPlan gp;
        // q, k, v: GEMM -> K-slice sums -> bias + RoPE + KV append
        const bf16_t* r_in = (l == 0 && r0_staged != nullptr) ? r0_staged : r;
        LAPS_TRY(run_gemm(c, LAPS_K_GEMM_QKV, capturing, r_in, static_cast<const bf16_t*>(lw.w_qkv), M, qkv, d, EPI_PARTIAL,
                          partial, nullptr, nullptr, nullptr, tok_pos, &gp, s));
        {
            ProfScope ps(c, s, LAPS_K_EPI_QKV, capturing);
            LAPS_TRY(laps_launch_epi_qkv(partial, gp.split, cf.has_qkv_bias ? static_cast<const bf16_t*>(lw.b_qkv) : nullptr,
                                         tok_pos, tok_slot, c->rope, c->max_pos, q, kp, vp, M, cf.n_q_heads,
                                         cf.n_kv_heads, hd, s));
        }
        {
            ProfScope ps(c, s, LAPS_K_ATTN, capturing);
            LAPS_TRY(laps_launch_attention(q, attn, kp, vp, b.row_start, new_len, b.prefix_len, b.page_table, b.max_pages,
                                           b.n_seq, M, tile_start, item_seq, partial, cf.n_q_heads, cf.n_kv_heads, hd,
                                           c->pool_pages, s));
        }
        // x_mid = resid + attn W_o^T ; r = rmsnorm(x_mid; ln2)
        LAPS_TRY(run_gemm(c, LAPS_K_GEMM_O, capturing, attn, static_cast<const bf16_t*>(lw.w_o), M, d, qd, EPI_RESID,
                          partial, x_mid, resid, nullptr, tok_pos, &gp, s));
        if (gp.epi == EPI_RESID) {
            ProfScope ps(c, s, LAPS_K_RMSNORM, capturing);
            LAPS_TRY(laps_launch_rmsnorm(x_mid, static_cast<const bf16_t*>(lw.ln2_w), r, M, d, cf.rms_eps, tok_pos, s));
        } else {
            ProfScope ps(c, s, LAPS_K_EPI_RESID, capturing);
            LAPS_TRY(laps_launch_epi_resid(partial, gp.split, resid, x_mid, static_cast<const bf16_t*>(lw.ln2_w), r, M, d,
                                           cf.rms_eps, tok_pos, s));
        }
        // act = silu(r W_g^T) * (r W_u^T)
        LAPS_TRY(run_gemm(c, LAPS_K_GEMM_GATEUP, capturing, r, static_cast<const bf16_t*>(lw.w_gate_up), M, 2 * I, d,
                          EPI_SWIGLU, partial, nullptr, nullptr, act, tok_pos, &gp, s));
        if (gp.epi != EPI_SWIGLU) {
            ProfScope ps(c, s, LAPS_K_EPI_SWIGLU, capturing);
            LAPS_TRY(laps_launch_epi_swiglu(partial, gp.split, act, M, I, tok_pos, s));
        }
        // x_out = x_mid + act W_d^T ; r = rmsnorm(x_out; next layer's ln1)
        const bf16_t* next_ln = (l + 1 < n_layers) ? static_cast<const bf16_t*>(w[l + 1].ln1_w) : nullptr;
        LAPS_TRY(run_gemm(c, LAPS_K_GEMM_DOWN, capturing, act, static_cast<const bf16_t*>(lw.w_down), M, d, I, EPI_RESID,
                          partial, x_out, x_mid, nullptr, tok_pos, &gp, s));
        if (gp.epi == EPI_RESID) {
            if (next_ln) {
                ProfScope ps(c, s, LAPS_K_RMSNORM, capturing);
                LAPS_TRY(laps_launch_rmsnorm(x_out, next_ln, r, M, d, cf.rms_eps, tok_pos, s));
            }
        } else {
            ProfScope ps(c, s, LAPS_K_EPI_RESID, capturing);
            LAPS_TRY(laps_launch_epi_resid(partial, gp.split, x_mid, x_out, next_ln, r, M, d, cf.rms_eps, tok_pos, s));
        }
    }
    return LAPS_OK;
}

static int check_batch_args(laps_ctx* c, const laps_layer_weights* w, int n_layers, int n_seq, int n_tokens,
                            const void* cu, const void* prefix, const void* pt, int max_pages, const void* x_in,
                            const void* x_out, const void* ws, size_t ws_bytes) {
    if (!c || !w || !cu || !prefix || !pt || !x_in || !x_out || !ws || n_seq < 1 || n_tokens < 1 || max_pages < 1) {
        laps_set_error("prefill: NULL pointer or non-positive size");
        return LAPS_EINVAL;
    }
    for (int l = 0; l < n_layers; ++l)
        if (!w[l].ln1_w || !w[l].w_qkv || !w[l].w_o || !w[l].ln2_w || !w[l].w_gate_up || !w[l].w_down ||
            (c->cfg.has_qkv_bias && !w[l].b_qkv)) {
            laps_set_error("prefill: layer %d has a NULL weight pointer", l);
            return LAPS_EINVAL;
        }
    if (((uintptr_t)ws & 255) != 0) {
        laps_set_error("prefill: workspace must be 256-byte aligned");
        return LAPS_EINVAL;
    }
    const size_t need = ws_layout(c->cfg, n_tokens, n_seq).total;
    if (ws_bytes < need) {
        laps_set_error("prefill: workspace too small (%zu < %zu bytes)", ws_bytes, need);
        return LAPS_ENOMEM;
    }
    return LAPS_OK;
}

extern "C" int laps_prefill_layer(laps_ctx* c, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                                  const int32_t* cu, const int32_t* seq_len, const int32_t* prefix_len,
                                  const int32_t* page_table, int32_t max_pages, void* k_pool, void* v_pool,
                                  const float* x_in, float* x_out, void* ws, size_t ws_bytes, void* stream) {
    LAPS_TRY(check_batch_args(c, w, 1, n_seq, n_tokens, cu, prefix_len, page_table, max_pages, x_in, x_out, ws, ws_bytes));
    if (!k_pool || !v_pool) {
        laps_set_error("prefill_layer: NULL KV pool");
        return LAPS_EINVAL;
    }
    const BatchDesc b{n_seq, n_tokens, cu, seq_len, prefix_len, page_table, max_pages};
    void* kp[1] = {k_pool};
    void* vp[1] = {v_pool};
    return run_layers(c, w, 1, b, kp, vp, x_in, x_out, static_cast<unsigned char*>(ws), false,
                      static_cast<hipStream_t>(stream));
}

// no_events: never create or record timing events, whatever laps_prof_enable said (the entry point that must
// not allocate: hipEventCreate and the event list's growth are allocations)
static int prefill_stack_impl(laps_ctx* c, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                              const int32_t* cu, const int32_t* seq_len, const int32_t* prefix_len,
                              const int32_t* page_table, int32_t max_pages, void* const* k_pools,
                              void* const* v_pools, const float* x_in, float* x_out, void* ws, size_t ws_bytes,
                              void* stream, bool no_events) {
    if (!c) {
        laps_set_error("prefill_stack: NULL context");
        return LAPS_EINVAL;
    }
    LAPS_TRY(check_batch_args(c, w, c->cfg.n_layers, n_seq, n_tokens, cu, prefix_len, page_table, max_pages, x_in, x_out,
                              ws, ws_bytes));
    if (!k_pools || !v_pools) {
        laps_set_error("prefill_stack: NULL KV pool array");
        return LAPS_EINVAL;
    }
    for (int l = 0; l < c->cfg.n_layers; ++l)
        if (!k_pools[l] || !v_pools[l]) {
            laps_set_error("prefill_stack: layer %d has a NULL KV pool", l);
            return LAPS_EINVAL;
        }
    const BatchDesc b{n_seq, n_tokens, cu, seq_len, prefix_len, page_table, max_pages};
    return run_layers(c, w, c->cfg.n_layers, b, k_pools, v_pools, x_in, x_out, static_cast<unsigned char*>(ws), no_events,
                      static_cast<hipStream_t>(stream));
}

extern "C" int laps_prefill_stack(laps_ctx* c, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                                  const int32_t* cu, const int32_t* seq_len, const int32_t* prefix_len,
                                  const int32_t* page_table, int32_t max_pages, void* const* k_pools,
                                  void* const* v_pools, const float* x_in, float* x_out, void* ws, size_t ws_bytes,
                                  void* stream) {
    return prefill_stack_impl(c, w, n_seq, n_tokens, cu, seq_len, prefix_len, page_table, max_pages, k_pools, v_pools,
                              x_in, x_out, ws, ws_bytes, stream, false);
}

extern "C" size_t laps_static_scratch_bytes(void) { return LAPS_STATIC_SCRATCH_BYTES; }

// laps_prefill_stack with the library's static device array as workspace: no allocation of any kind here or
// below (the launches take the address resolved at context creation as a kernel argument).
extern "C" int laps_prefill_stack_static(laps_ctx* c, const laps_layer_weights* w, int32_t n_seq, int32_t n_tokens,
                                         const int32_t* cu, const int32_t* seq_len, const int32_t* prefix_len,
                                         const int32_t* page_table, int32_t max_pages, void* const* k_pools,
                                         void* const* v_pools, const float* x_in, float* x_out, void* stream) {
    if (!c || !c->static_ws) {
        laps_set_error("prefill_stack_static: NULL context or static scratch not resolved");
        return LAPS_EINVAL;
    }
    if (n_seq < 1 || n_tokens < 1) {
        laps_set_error("prefill_stack_static: non-positive size");
        return LAPS_EINVAL;
    }
    const size_t need = ws_layout(c->cfg, n_tokens, n_seq).total;
    if (need > LAPS_STATIC_SCRATCH_BYTES) {
        laps_set_error("prefill_stack_static: %d tokens x %d sequences need %zu bytes of workspace, the static scratch "
                       "holds %zu; use laps_prefill_stack with a caller-owned workspace", n_tokens, n_seq, need,
                       (size_t)LAPS_STATIC_SCRATCH_BYTES);
        return LAPS_EINVAL;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != c->device) {
        laps_set_error("prefill_stack_static: the context's device %d must be current (current: %d)", c->device, dev);
        return LAPS_EINVAL;
    }
    return prefill_stack_impl(c, w, n_seq, n_tokens, cu, seq_len, prefix_len, page_table, max_pages, k_pools, v_pools,
                              x_in, x_out, c->static_ws, LAPS_STATIC_SCRATCH_BYTES, stream, true);
}

// ----------------------------------------------------------------------------- helpers
extern "C" int laps_pack_gate_up(laps_ctx* c, const void* wg, const void* wu, void* dst, void* stream) {
    if (!c || !wg || !wu || !dst) {
        laps_set_error("pack_gate_up: NULL argument");
        return LAPS_EINVAL;
    }
    if (c->cfg.intermediate % 32 || c->cfg.hidden % 8) {
        laps_set_error("pack_gate_up: intermediate must be a multiple of 32");
        return LAPS_EINVAL;
    }
    return laps_launch_pack_gate_up(static_cast<const bf16_t*>(wg), static_cast<const bf16_t*>(wu),
                                    static_cast<bf16_t*>(dst), c->cfg.intermediate, c->cfg.hidden,
                                    static_cast<hipStream_t>(stream));
}

static int kv_move(bool scatter, laps_ctx* c, int n_seq, int n_tokens, const int* cu, const int* start_pos,
                   const int* pt, int max_pages, void* k_tok, void* v_tok, void* k_pool, void* v_pool, void* stream) {
    if (!c || n_seq < 1 || n_tokens < 0 || !cu || !start_pos || !pt || max_pages < 1 || !k_pool || !v_pool ||
        (n_tokens > 0 && (!k_tok || !v_tok))) {
        laps_set_error("kv move: NULL pointer or bad size");
        return LAPS_EINVAL;
    }
    return laps_launch_kv_move(scatter, n_seq, n_tokens, cu, start_pos, pt, max_pages, static_cast<bf16_t*>(k_tok),
                               static_cast<bf16_t*>(v_tok), static_cast<bf16_t*>(k_pool), static_cast<bf16_t*>(v_pool),
                               c->cfg.n_kv_heads, c->cfg.head_dim, c->pool_pages, static_cast<hipStream_t>(stream));
}

extern "C" int laps_kv_scatter(laps_ctx* c, int32_t n_seq, int32_t n_tokens, const int32_t* cu, const int32_t* start_pos,
                               const int32_t* pt, int32_t max_pages, const void* k_src, const void* v_src, void* k_pool,
                               void* v_pool, void* stream) {
    return kv_move(true, c, n_seq, n_tokens, cu, start_pos, pt, max_pages, const_cast<void*>(k_src),
                   const_cast<void*>(v_src), k_pool, v_pool, stream);
}

extern "C" int laps_kv_gather(laps_ctx* c, int32_t n_seq, int32_t n_tokens, const int32_t* cu, const int32_t* start_pos,
                              const int32_t* pt, int32_t max_pages, const void* k_pool, const void* v_pool, void* k_dst,
                              void* v_dst, void* stream) {
    return kv_move(false, c, n_seq, n_tokens, cu, start_pos, pt, max_pages, k_dst, v_dst, const_cast<void*>(k_pool),
                   const_cast<void*>(v_pool), stream);
}

extern "C" size_t laps_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t split_k) {
    if (m < 1 || n < 64 || n % 64 || k < 64 || k % 64 || split_k < 0) return 0;
    const GemmPlan p = laps_gemm_plan(m, n, k, split_k, EPI_PARTIAL);
    return p.split == 1 ? 0 : (size_t)p.split * m * n * sizeof(float);
}

extern "C" int laps_gemm_bf16(laps_ctx* c, const void* a, const void* w, float* out, int32_t m, int32_t n, int32_t k,
                              int32_t split_k, void* ws, size_t ws_bytes, void* stream) {
    if (!c || !a || !w || !out || m < 1 || split_k < 0) {
        laps_set_error("gemm: NULL pointer or bad size");
        return LAPS_EINVAL;
    }
    if (n < 64 || n % 64 || k < 64 || k % 64) {
        laps_set_error("gemm: need n %% 64 == 0 and k %% 64 == 0 (n=%d k=%d)", n, k);
        return LAPS_EINVAL;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const GemmPlan p = laps_gemm_plan(m, n, k, split_k, EPI_PARTIAL);
    if (p.split == 1)
        return laps_gemm_launch(p, static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(w), m, n, k, out, nullptr, nullptr, nullptr, s);
    const size_t need = (size_t)p.split * m * n * sizeof(float);
    if (!ws || ws_bytes < need || ((uintptr_t)ws & 255)) {
        laps_set_error("gemm: split-K needs %zu bytes of 256-byte aligned workspace", need);
        return LAPS_ENOMEM;
    }
    LAPS_TRY(laps_gemm_launch(p, static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(w), m, n, k, static_cast<float*>(ws),
                              nullptr, nullptr, nullptr, s));
    // sum the slices: view [m, n] as rows of `cols` columns, cols | n and cols <= 8192
    int cols = n;
    while (cols > 8192) {
        if (cols % 2) {
            laps_set_error("gemm: cannot fold n=%d for the slice reducer", n);
            return LAPS_EINVAL;
        }
        cols /= 2;
    }
    const int rows = (int)(((size_t)m * n) / cols);
    return laps_launch_epi_resid(static_cast<const float*>(ws), p.split, nullptr, out, nullptr, nullptr, rows, cols, 1.f, nullptr, s);
}

// One projection with the epilogue the layer driver asks for, launched exactly as the driver launches it: fused
// into the GEMM when K is a single slice, else K-slice partial sums followed by the row kernel that adds them.
extern "C" int laps_gemm_epilogue_bf16(laps_ctx* c, const void* a, const void* w, int32_t m, int32_t n, int32_t k,
                                       int32_t epilogue, const float* resid, float* out_f32, void* out_bf16, void* ws,
                                       size_t ws_bytes, void* stream) {
    if (!c || !a || !w || m < 1 || n < 64 || n % 64 || k < 64 || k % 64) {
        laps_set_error("gemm_epilogue: NULL pointer or unsupported shape (m=%d n=%d k=%d)", m, n, k);
        return LAPS_EINVAL;
    }
    if ((epilogue == EPI_RESID && (!resid || !out_f32)) || (epilogue == EPI_SWIGLU && (!out_bf16 || n % 64)) ||
        (epilogue != EPI_RESID && epilogue != EPI_SWIGLU)) {
        laps_set_error("gemm_epilogue: epilogue %d needs its operands (1: resid, out_f32; 2: out_bf16)", epilogue);
        return LAPS_EINVAL;
    }
    if (epilogue == EPI_RESID && n > 8192) {
        laps_set_error("gemm_epilogue: the residual row kernel handles rows of at most 8192 columns (n=%d)", n);
        return LAPS_EINVAL;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const GemmPlan p = laps_gemm_plan(m, n, k, 0, epilogue);
    if (p.epi == epilogue)
        return laps_gemm_launch(p, static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(w), m, n, k, out_f32, resid,
                                static_cast<bf16_t*>(out_bf16), nullptr, s);
    const size_t need = (size_t)p.split * m * n * sizeof(float);
    if (!ws || ws_bytes < need || ((uintptr_t)ws & 255)) {
        laps_set_error("gemm_epilogue: this shape splits K and needs %zu bytes of 256-byte aligned workspace", need);
        return LAPS_ENOMEM;
    }
    LAPS_TRY(laps_gemm_launch(p, static_cast<const bf16_t*>(a), static_cast<const bf16_t*>(w), m, n, k,
                              static_cast<float*>(ws), nullptr, nullptr, nullptr, s));
    if (epilogue == EPI_RESID)
        return laps_launch_epi_resid(static_cast<const float*>(ws), p.split, resid, out_f32, nullptr, nullptr, m, n, 1.f,
                                     nullptr, s);
    return laps_launch_epi_swiglu(static_cast<const float*>(ws), p.split, static_cast<bf16_t*>(out_bf16), m, n / 2, nullptr, s);
}

extern "C" int laps_attention(laps_ctx* c, int32_t n_seq, int32_t n_tokens, const int32_t* cu, const int32_t* seq_len,
                              const int32_t* prefix_len, const int32_t* pt, int32_t max_pages, const void* k_pool,
                              const void* v_pool, const void* q, void* out, void* ws, size_t ws_bytes, void* stream) {
    if (!c || n_seq < 1 || n_tokens < 1 || !cu || !prefix_len || !pt || max_pages < 1 || !k_pool || !v_pool || !q ||
        !out || !ws || ((uintptr_t)ws & 255)) {
        laps_set_error("attention: NULL pointer or bad size");
        return LAPS_EINVAL;
    }
    const WsLayout L = ws_layout(c->cfg, n_tokens, n_seq);
    if (ws_bytes < L.total) {
        laps_set_error("attention: workspace too small (%zu < %zu bytes)", ws_bytes, L.total);
        return LAPS_ENOMEM;
    }
    unsigned char* w8 = static_cast<unsigned char*>(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int* new_len = reinterpret_cast<int*>(w8 + L.new_len);
    LAPS_TRY(laps_launch_prep(n_tokens, n_seq, cu, seq_len, prefix_len, pt, max_pages, c->pool_pages, new_len,
                              reinterpret_cast<int*>(w8 + L.tok_pos), reinterpret_cast<int*>(w8 + L.tok_slot), s));
    LAPS_TRY(laps_launch_attn_sched(new_len, n_seq, n_tokens, max_pages, reinterpret_cast<int*>(w8 + L.tile_start),
                                    reinterpret_cast<int*>(w8 + L.item_seq), c->cfg.n_q_heads, c->cfg.n_kv_heads, s));
    return laps_launch_attention(static_cast<const bf16_t*>(q), static_cast<bf16_t*>(out),
                                 static_cast<const bf16_t*>(k_pool), static_cast<const bf16_t*>(v_pool), cu, new_len,
                                 prefix_len, pt, max_pages, n_seq, n_tokens, reinterpret_cast<int*>(w8 + L.tile_start),
                                 reinterpret_cast<int*>(w8 + L.item_seq), reinterpret_cast<float*>(w8 + L.partial), c->cfg.n_q_heads, c->cfg.n_kv_heads,
                                 c->cfg.head_dim, c->pool_pages, s);
}

// ----------------------------------------------------------------------------- launch plans (host only)
extern "C" int laps_gemm_plan_info(int32_t m, int32_t n, int32_t k, int32_t split_k, int32_t epilogue, int32_t* out) {
    if (!out || m < 1 || n < 64 || n % 64 || k < 64 || k % 64 || split_k < 0 || epilogue < 0 || epilogue > 2) {
        laps_set_error("gemm_plan_info: NULL output or unsupported shape (m=%d n=%d k=%d)", m, n, k);
        return LAPS_EINVAL;
    }
    const GemmPlan p = laps_gemm_plan(m, n, k, split_k, epilogue);
    int bm = 0, bn = 0;
    laps_gemm_tile_dims(p.cfg, &bm, &bn);
    if (bm == 0 || n % bn != 0) {
        laps_set_error("gemm_plan_info: no tile shape divides n=%d", n);
        return LAPS_EINVAL;
    }
    out[0] = bm;
    out[1] = bn;
    out[2] = p.split;
    out[3] = p.k_per_split;
    out[4] = p.epi;
    out[5] = p.ws;
    out[6] = ((m + bm - 1) / bm) * (n / bn) * p.split;
    return LAPS_OK;
}

extern "C" int laps_attn_plan_info(int32_t n_seq, int32_t n_tokens, int32_t n_q_heads, int32_t n_kv_heads,
                                   int32_t head_dim, int32_t max_pages, int64_t* out) {
    if (!out || n_seq < 1 || n_tokens < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads ||
        (head_dim != 64 && head_dim != 128) || max_pages < 1) {
        laps_set_error("attn_plan_info: NULL output or unsupported shape");
        return LAPS_EINVAL;
    }
    int rows = 0, items = 0, split = 0, min_tiles = 0;
    laps_attn_plan(n_seq, n_tokens, n_q_heads / n_kv_heads, n_kv_heads, max_pages, &rows, &items, &split, &min_tiles);
    out[0] = rows;
    out[1] = items;
    out[2] = split;
    out[3] = min_tiles;
    out[4] = (int64_t)laps_attn_item_table_bytes(n_tokens, n_seq, n_q_heads / n_kv_heads);
    out[5] = (int64_t)laps_attn_partial_bytes(head_dim, max_pages);
    return LAPS_OK;
}

// ----------------------------------------------------------------------------- captured buckets
struct laps_graph {
    laps_ctx* ctx;
    int len_bucket, depth, max_pages, n_layers;
    unsigned char* block;  // one device allocation holding everything below
    size_t block_bytes;
    float *x_in, *x_out;
    int *row_start, *seq_len, *prefix_len, *page_table;
    bf16_t* r0;               // first layer's normed rows, written when a batch is staged
    const bf16_t* ln1_first;  // the first layer's RMSNorm gain
    unsigned char* ws;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

// The two staging launches of a graph (see StageArgs): everything a replay needs besides the layers themselves.
static int graph_stage_launch(laps_graph* g, int n_real, const int* seq_len, const int* prefix_len, const int* page_table,
                              const float* x_rows, int n_rows, hipStream_t s) {
    const laps_model_cfg& cf = g->ctx->cfg;
    const int M = g->depth * g->len_bucket;
    const WsLayout L = ws_layout(cf, M, g->depth);
    StageArgs a;
    a.seq_len = seq_len;
    a.prefix_len = prefix_len;
    a.page_table = page_table;
    a.x_rows = x_rows;
    a.n_real = n_real;
    a.n_rows = n_rows;
    a.depth = g->depth;
    a.len_bucket = g->len_bucket;
    a.max_pages = g->max_pages;
    a.n_pool_pages = g->ctx->pool_pages;
    a.group = cf.n_q_heads / cf.n_kv_heads;
    int n_split = 0, min_tiles = 0;
    laps_attn_plan(g->depth, M, a.group, cf.n_kv_heads, g->max_pages, &a.rows_per_wg, &a.max_items, &n_split, &min_tiles);
    a.seq_len_out = g->seq_len;
    a.prefix_out = g->prefix_len;
    a.row_start_out = g->row_start;
    a.page_table_out = g->page_table;
    a.new_len_out = reinterpret_cast<int*>(g->ws + L.new_len);
    a.tok_pos = reinterpret_cast<int*>(g->ws + L.tok_pos);
    a.tok_slot = reinterpret_cast<int*>(g->ws + L.tok_slot);
    a.tile_start = reinterpret_cast<int*>(g->ws + L.tile_start);
    a.item_seq = reinterpret_cast<int*>(g->ws + L.item_seq);
    a.x_in = g->x_in;
    a.ln_w = g->ln1_first;
    a.r0 = g->r0;
    a.d = cf.hidden;
    a.eps = cf.rms_eps;
    return laps_launch_stage(a, s);
}

extern "C" int laps_graph_capture(laps_ctx* c, const laps_layer_weights* w, int32_t len_bucket, int32_t depth,
                                  int32_t max_pages, void* const* k_pools, void* const* v_pools, void* stream,
                                  laps_graph** out) {
    if (!c || !w || !out || len_bucket < 1 || depth < 1 || max_pages < 1 || !k_pools || !v_pools) {
        laps_set_error("graph_capture: NULL pointer or non-positive size");
        return LAPS_EINVAL;
    }
    const int nl = c->cfg.n_layers;
    for (int l = 0; l < nl; ++l)
        if (!k_pools[l] || !v_pools[l] || !w[l].ln1_w || !w[l].w_qkv || !w[l].w_o || !w[l].ln2_w || !w[l].w_gate_up ||
            !w[l].w_down) {
            laps_set_error("graph_capture: layer %d has a NULL pointer", l);
            return LAPS_EINVAL;
        }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (s == nullptr) {
        laps_set_error("graph_capture: the null stream cannot be captured; pass a created stream");
        return LAPS_EINVAL;
    }
    laps_graph* g = new (std::nothrow) laps_graph();
    if (!g) {
        laps_set_error("graph_capture: out of host memory");
        return LAPS_ENOMEM;
    }
    memset(g, 0, sizeof(*g));
    g->ctx = c;
    g->len_bucket = len_bucket;
    g->depth = depth;
    g->max_pages = max_pages;
    g->n_layers = nl;
    const size_t M = (size_t)len_bucket * depth, d = c->cfg.hidden;
    const size_t ws_bytes = ws_layout(c->cfg, (int)M, depth, max_pages).total;
    size_t o = 0;
    const size_t o_xin = o;  o += align256(M * d * 4);
    const size_t o_xout = o; o += align256(M * d * 4);
    const size_t o_rs = o;   o += align256((size_t)(depth + 1) * 4);
    const size_t o_sl = o;   o += align256((size_t)depth * 4);
    const size_t o_pl = o;   o += align256((size_t)depth * 4);
    const size_t o_pt = o;   o += align256((size_t)depth * max_pages * 4);
    const size_t o_r0 = o;   o += align256(M * d * 2);
    const size_t o_ws = o;   o += ws_bytes;
    g->block_bytes = o;
    auto fail = [&](int rc) {
        if (g->exec) (void)hipGraphExecDestroy(g->exec);
        if (g->graph) (void)hipGraphDestroy(g->graph);
        if (g->block) (void)hipFree(g->block);
        delete g;
        return rc;
    };
    hipError_t e = hipMalloc(&g->block, g->block_bytes);
    if (e != hipSuccess) {
        laps_set_error("graph_capture: hipMalloc(%zu) failed: %s", g->block_bytes, hipGetErrorString(e));
        g->block = nullptr;
        return fail(e == hipErrorOutOfMemory ? LAPS_ENOMEM : LAPS_EHIP);
    }
    g->x_in = reinterpret_cast<float*>(g->block + o_xin);
    g->x_out = reinterpret_cast<float*>(g->block + o_xout);
    g->row_start = reinterpret_cast<int*>(g->block + o_rs);
    g->seq_len = reinterpret_cast<int*>(g->block + o_sl);
    g->prefix_len = reinterpret_cast<int*>(g->block + o_pl);
    g->page_table = reinterpret_cast<int*>(g->block + o_pt);
    g->r0 = reinterpret_cast<bf16_t*>(g->block + o_r0);
    g->ln1_first = static_cast<const bf16_t*>(w[0].ln1_w);
    g->ws = g->block + o_ws;
    // all slots empty (every row offset 0, every length 0), inputs zero; done before capture, so a plain
    // memset is fine here
    if ((e = hipMemsetAsync(g->block, 0, o_ws, s)) != hipSuccess || (e = hipStreamSynchronize(s)) != hipSuccess) {
        laps_set_error("graph_capture: staging init failed: %s", hipGetErrorString(e));
        return fail(LAPS_EHIP);
    }
    const BatchDesc b{depth, (int)M, g->row_start, g->seq_len, g->prefix_len, g->page_table, max_pages};
    // every slot empty: token metadata and work-item table of an empty batch, as the captured kernels expect to find them
    int rc = graph_stage_launch(g, 0, nullptr, nullptr, nullptr, nullptr, 0, s);
    // warm-up pass: loads code objects and sets kernel attributes outside the capture
    if (rc == LAPS_OK) rc = run_layers(c, w, nl, b, k_pools, v_pools, g->x_in, g->x_out, g->ws, true, s, g->r0);
    if (rc == LAPS_OK && (e = hipStreamSynchronize(s)) != hipSuccess) {
        laps_set_error("graph_capture: warm-up failed: %s", hipGetErrorString(e));
        rc = LAPS_EHIP;
    }
    if (rc != LAPS_OK) return fail(rc);
    if ((e = hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed)) != hipSuccess) {
        laps_set_error("graph_capture: hipStreamBeginCapture failed: %s", hipGetErrorString(e));
        return fail(LAPS_EHIP);
    }
    rc = run_layers(c, w, nl, b, k_pools, v_pools, g->x_in, g->x_out, g->ws, true, s, g->r0);
    e = hipStreamEndCapture(s, &g->graph);
    if (rc != LAPS_OK) return fail(rc);
    if (e != hipSuccess || !g->graph) {
        laps_set_error("graph_capture: hipStreamEndCapture failed: %s", hipGetErrorString(e));
        return fail(LAPS_EHIP);
    }
    if ((e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0)) != hipSuccess) {
        laps_set_error("graph_capture: hipGraphInstantiate failed: %s", hipGetErrorString(e));
        g->exec = nullptr;
        return fail(LAPS_EHIP);
    }
    *out = g;
    return LAPS_OK;
}

extern "C" int laps_graph_stage(laps_graph* g, int32_t n_real, const int32_t* seq_len, const int32_t* prefix_len,
                                const int32_t* page_table, const float* x_rows, int32_t n_rows, void* stream) {
    if (!g || n_real < 0 || n_real > g->depth || (n_real > 0 && (!seq_len || !prefix_len || !page_table))) {
        laps_set_error("graph_stage: bad slot count or NULL pointer");
        return LAPS_EINVAL;
    }
    if (n_rows < 0 || n_rows > g->depth * g->len_bucket || (n_rows > 0 && !x_rows)) {
        laps_set_error("graph_stage: %d input rows do not fit the graph's %d rows", n_rows, g->depth * g->len_bucket);
        return LAPS_EINVAL;
    }
    return graph_stage_launch(g, n_real, seq_len, prefix_len, page_table, x_rows, n_rows, static_cast<hipStream_t>(stream));
}

extern "C" int laps_graph_replay(laps_graph* g, void* stream) {
    if (!g || !g->exec) {
        laps_set_error("graph_replay: NULL graph");
        return LAPS_EINVAL;
    }
    LAPS_HIP(hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)));
    return LAPS_OK;
}

extern "C" const float* laps_graph_output(const laps_graph* g) { return g ? g->x_out : nullptr; }
extern "C" float* laps_graph_input(laps_graph* g) { return g ? g->x_in : nullptr; }
extern "C" int laps_graph_read_output(const laps_graph* g, int32_t n_rows, float* dst, void* stream) {
    if (!g || !dst || n_rows < 0 || n_rows > g->depth * g->len_bucket) {
        laps_set_error("graph_read_output: NULL pointer or row count out of range");
        return LAPS_EINVAL;
    }
    if (n_rows == 0) return LAPS_OK;
    LAPS_HIP(hipMemcpyAsync(dst, g->x_out, (size_t)n_rows * g->ctx->cfg.hidden * 4, hipMemcpyDeviceToDevice,
                            static_cast<hipStream_t>(stream)));
    return LAPS_OK;
}
extern "C" size_t laps_graph_device_bytes(const laps_graph* g) { return g ? g->block_bytes : 0; }

extern "C" void laps_graph_destroy(laps_graph* g) {
    if (!g) return;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    if (g->block) (void)hipFree(g->block);
    delete g;
}
