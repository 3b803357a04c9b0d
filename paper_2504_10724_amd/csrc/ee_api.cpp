// ee_api.cpp -- the C ABI of libee: argument checks, handle bookkeeping and the
// sequencing of one early-exit decode step.  All arithmetic is in the kernels.
#include "ee_internal.h"

#include <cmath>
#include <cstring>
#include <new>

static thread_local std::string g_last_error;

void ee_set_error(const std::string& msg) { g_last_error = msg; }
int ee_fail(int code, const std::string& msg) {
    g_last_error = msg;
    return code;
}

static hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// ------------------------------------------------------------------ kernel timing
unsigned g_ee_timing_mask = 0;
namespace {
struct TimingPair { int kind; hipEvent_t a, b; bool closed; };
std::vector<TimingPair> g_pairs;
std::vector<hipEvent_t> g_free_events;
int   g_launches[EE_K_COUNT];
float g_total_ms[EE_K_COUNT];

hipEvent_t take_event() {
    if (!g_free_events.empty()) { hipEvent_t e = g_free_events.back(); g_free_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

void drain_pairs() {
    for (TimingPair& p : g_pairs) {
        if (p.closed && p.a && p.b && hipEventSynchronize(p.b) == hipSuccess) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) { g_total_ms[p.kind] += ms; g_launches[p.kind] += 1; }
        }
        if (p.a) g_free_events.push_back(p.a);
        if (p.b) g_free_events.push_back(p.b);
    }
    g_pairs.clear();
}
}  // namespace

void ee_timing_mark(int kind, hipStream_t s, bool begin) {
    if (kind < 0 || kind >= EE_K_COUNT) return;
    if (begin) {
        TimingPair p{kind, take_event(), take_event(), false};
        if (p.a) (void)hipEventRecord(p.a, s);
        g_pairs.push_back(p);
    } else {
        for (size_t i = g_pairs.size(); i-- > 0;) {
            if (g_pairs[i].kind == kind && !g_pairs[i].closed) {
                if (g_pairs[i].b) (void)hipEventRecord(g_pairs[i].b, s);
                g_pairs[i].closed = true;
                break;
            }
        }
    }
}

extern "C" {

const char* ee_last_error(void) { return g_last_error.c_str(); }

int ee_device_count(void) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess) return ee_fail(EE_ERR_HIP, std::string("hipGetDeviceCount: ") + hipGetErrorString(e));
    return n;
}

int ee_timing_enable(int class_mask) {
    g_ee_timing_mask = (unsigned)class_mask & ((1u << EE_K_COUNT) - 1u);
    return EE_OK;
}

int ee_timing_reset(void) {
    drain_pairs();
    for (int k = 0; k < EE_K_COUNT; ++k) { g_launches[k] = 0; g_total_ms[k] = 0.f; }
    return EE_OK;
}

int ee_timing_read(int kernel_class, int* launches, float* total_ms) {
    if (kernel_class < 0 || kernel_class >= EE_K_COUNT || !launches || !total_ms)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_timing_read: bad argument");
    drain_pairs();
    *launches = g_launches[kernel_class];
    *total_ms = g_total_ms[kernel_class];
    return EE_OK;
}

// ------------------------------------------------------------------ weights
size_t ee_packed_bytes(int n_out, int n_in) {
    if (n_out <= 0 || n_in <= 0) return 0;
    return (size_t)n_out * (size_t)n_in * 2;
}

int ee_pack_weight(const void* dev_src, int n_out, int n_in, void* dev_dst, int row_offset, int row_stride,
                   int dst_rows, void* stream) {
    if (!dev_src || !dev_dst) return ee_fail(EE_ERR_INVALID_ARG, "ee_pack_weight: null pointer");
    if (n_out <= 0 || n_in <= 0 || n_in % 16 != 0 || dst_rows <= 0 || dst_rows % 32 != 0)
        return ee_fail(EE_ERR_SHAPE, "ee_pack_weight: n_in must be a multiple of 16 and dst_rows of 32");
    if (row_offset < 0 || row_stride < 1 || (int64_t)row_offset + (int64_t)(n_out - 1) * row_stride >= dst_rows)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_pack_weight: row placement outside the destination");
    return launch_pack_weight(dev_src, n_out, n_in, dev_dst, row_offset, row_stride, dst_rows, as_stream(stream));
}

// ------------------------------------------------------------------ model
static int check_config(const ee_model_config* c) {
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 ||
        c->vocab < 1 || c->max_pos < 1)
        return ee_fail(EE_ERR_SHAPE, "ee_model_create: non-positive dimension");
    if (c->n_q_heads % c->n_kv_heads != 0 || c->n_q_heads / c->n_kv_heads > 16)
        return ee_fail(EE_ERR_SHAPE, "ee_model_create: H_q must be a multiple of H_kv with ratio <= 16");
    if (c->head_dim < 2 || c->head_dim % 2 != 0) return ee_fail(EE_ERR_SHAPE, "ee_model_create: head_dim must be even");
    if (c->dtype != EE_F32 && c->dtype != EE_BF16) return ee_fail(EE_ERR_DTYPE, "ee_model_create: unknown dtype");
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 1.f))
        return ee_fail(EE_ERR_INVALID_ARG, "ee_model_create: rms_eps must be >= 0 and rope_theta > 1");
    if (c->n_exits < 1 || c->n_exits > EE_MAX_EXITS) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_create: n_exits out of range");
    for (int e = 0; e < c->n_exits; ++e) {
        if (c->exit_layers[e] < 1 || c->exit_layers[e] > c->n_layers ||
            (e > 0 && c->exit_layers[e] <= c->exit_layers[e - 1]))
            return ee_fail(EE_ERR_INVALID_ARG, "ee_model_create: exit_layers must be ascending layers of the model");
    }
    if (c->dtype == EE_BF16) {
        int qd = c->n_q_heads * c->head_dim, qkv = (c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
        if (c->head_dim != 128) return ee_fail(EE_ERR_SHAPE, "ee_model_create: bf16 models need head_dim 128");
        if (c->d_model % 64 || c->d_ffn % 64 || qd % 64 || qkv % 32 || c->vocab % 32)
            return ee_fail(EE_ERR_SHAPE, "ee_model_create: bf16 models need d, F, H_q*hd multiples of 64 and "
                                         "(H_q+2H_kv)*hd, V multiples of 32");
    } else {
        if (c->head_dim > 256) return ee_fail(EE_ERR_SHAPE, "ee_model_create: fp32 models need head_dim <= 256");
        if (c->max_pos > 8192) return ee_fail(EE_ERR_SHAPE, "ee_model_create: fp32 models need max_pos <= 8192");
    }
    return EE_OK;
}

int ee_model_create(const ee_model_config* cfg, ee_model** out) {
    if (!cfg || !out) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_create: null pointer");
    int rc = check_config(cfg);
    if (rc != EE_OK) return rc;
    ee_model* m = new (std::nothrow) ee_model();
    if (!m) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_create: out of host memory");
    m->cfg = *cfg;
    m->layers.resize(cfg->n_layers);
    m->resident.assign(cfg->n_layers, 0);
    hipError_t e = hipGetDevice(&m->device);
    if (e == hipSuccess)
        e = hipMalloc((void**)&m->d_rope, (size_t)cfg->max_pos * (cfg->head_dim / 2) * 2 * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&m->d_wqkv_tab, sizeof(void*) * cfg->n_layers);
    if (e == hipSuccess) e = hipMalloc((void**)&m->d_gattn_tab, sizeof(void*) * cfg->n_layers);
    if (e == hipSuccess) e = hipMemset(m->d_wqkv_tab, 0, sizeof(void*) * cfg->n_layers);
    if (e == hipSuccess) e = hipMemset(m->d_gattn_tab, 0, sizeof(void*) * cfg->n_layers);
    if (e != hipSuccess) {
        if (m->d_rope) (void)hipFree(m->d_rope);
        if (m->d_wqkv_tab) (void)hipFree(m->d_wqkv_tab);
        if (m->d_gattn_tab) (void)hipFree(m->d_gattn_tab);
        delete m;
        return ee_fail(EE_ERR_HIP, std::string("ee_model_create: ") + hipGetErrorString(e));
    }
    rc = launch_rope_table(m->d_rope, cfg->max_pos, cfg->head_dim, (double)cfg->rope_theta, nullptr);
    if (rc == EE_OK && hipStreamSynchronize(nullptr) != hipSuccess) rc = ee_fail(EE_ERR_HIP, "ee_model_create: rotary table kernel failed");
    if (rc != EE_OK) {
        (void)hipFree(m->d_rope);
        (void)hipFree(m->d_wqkv_tab);
        (void)hipFree(m->d_gattn_tab);
        delete m;
        return rc;
    }
    *out = m;
    return EE_OK;
}

int ee_model_destroy(ee_model* m) {
    if (!m) return EE_OK;
    if (m->d_rope) (void)hipFree(m->d_rope);
    if (m->d_wqkv_tab) (void)hipFree(m->d_wqkv_tab);
    if (m->d_gattn_tab) (void)hipFree(m->d_gattn_tab);
    delete m;
    return EE_OK;
}

int ee_model_set_layer(ee_model* m, int layer, const ee_layer_weights* w) {
    if (!m || !w) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer: null pointer");
    if (layer < 1 || layer > m->cfg.n_layers) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer: layer out of range");
    if (!w->g_attn || !w->w_qkv || !w->w_o || !w->g_ffn || !w->w_gate_up || !w->w_down)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer: null weight pointer");
    // the per-layer device tables the multi-layer launches index
    hipError_t e = hipMemcpy(m->d_wqkv_tab + (layer - 1), &w->w_qkv, sizeof(void*), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->d_gattn_tab + (layer - 1), &w->g_attn, sizeof(void*), hipMemcpyHostToDevice);
    if (e != hipSuccess) return ee_fail(EE_ERR_HIP, std::string("ee_model_set_layer: ") + hipGetErrorString(e));
    m->layers[layer - 1] = *w;
    m->resident[layer - 1] = 1;
    return EE_OK;
}

int ee_model_set_layer_on(ee_model* m, int layer, const ee_layer_weights* w, void* stream) {
    if (!m || !w) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer_on: null pointer");
    if (layer < 1 || layer > m->cfg.n_layers) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer_on: layer out of range");
    if (!w->g_attn || !w->w_qkv || !w->w_o || !w->g_ffn || !w->w_gate_up || !w->w_down)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_layer_on: null weight pointer");
    int rc = launch_set_layer_ptrs(m, layer, w->w_qkv, (const float*)w->g_attn, as_stream(stream));
    if (rc != EE_OK) return rc;
    m->layers[layer - 1] = *w;
    m->resident[layer - 1] = 1;
    return EE_OK;
}

int ee_model_set_exit(ee_model* m, int exit_idx, const float* gain, const void* w) {
    if (!m || !gain || !w) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_exit: null pointer");
    if (exit_idx < 0 || exit_idx >= m->cfg.n_exits) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_exit: exit index out of range");
    m->exits[exit_idx].gain = gain;
    m->exits[exit_idx].w = w;
    m->exits[exit_idx].set = true;
    return EE_OK;
}

int ee_model_set_embed(ee_model* m, const void* emb) {
    if (!m || !emb) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_set_embed: null pointer");
    m->emb = emb;
    return EE_OK;
}

int ee_model_resident_depth(const ee_model* m) {
    if (!m) return ee_fail(EE_ERR_INVALID_ARG, "ee_model_resident_depth: null model");
    int R = 0;
    while (R < m->cfg.n_layers && m->resident[R]) ++R;
    for (int l = R; l < m->cfg.n_layers; ++l)
        if (m->resident[l]) return ee_fail(EE_ERR_INVALID_ARG, "resident layers are not a prefix 1..R");
    return R;
}

// ------------------------------------------------------------------ key/value pool
static size_t elem_size(const ee_model* m) { return m->cfg.dtype == EE_BF16 ? 2 : 4; }

static int check_capacity(const ee_model* m, const int32_t* cap, int B, int64_t* total) {
    if (!m || !cap || B < 1) return ee_fail(EE_ERR_INVALID_ARG, "key/value pool: null pointer or empty batch");
    int64_t T = 0;
    for (int b = 0; b < B; ++b) {
        if (cap[b] < 1 || cap[b] > m->cfg.max_pos)
            return ee_fail(EE_ERR_CAPACITY, "key/value pool: row capacity must be in 1..max_pos");
        if (m->cfg.dtype == EE_BF16 && cap[b] % 32 != 0)
            return ee_fail(EE_ERR_SHAPE, "key/value pool: bf16 row capacity must be a multiple of 32");
        T += cap[b];
    }
    *total = T;
    return EE_OK;
}

size_t ee_kv_pool_bytes(const ee_model* m, int n_resident_layers, const int32_t* host_capacity, int B) {
    int64_t T = 0;
    if (n_resident_layers < 1 || check_capacity(m, host_capacity, B, &T) != EE_OK) return 0;
    return (size_t)n_resident_layers * (size_t)T * 2 * m->cfg.n_kv_heads * m->cfg.head_dim * elem_size(m);
}

int ee_kv_bind(const ee_model* m, void* dev_pool, size_t pool_bytes, int n_resident_layers,
               const int32_t* host_capacity, int B, ee_kv** out) {
    if (!m || !dev_pool || !out) return ee_fail(EE_ERR_INVALID_ARG, "ee_kv_bind: null pointer");
    if (n_resident_layers < 1 || n_resident_layers > m->cfg.n_layers)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_kv_bind: layer count out of range");
    int64_t T = 0;
    int rc = check_capacity(m, host_capacity, B, &T);
    if (rc != EE_OK) return rc;
    size_t need = ee_kv_pool_bytes(m, n_resident_layers, host_capacity, B);
    if (pool_bytes < need) return ee_fail(EE_ERR_CAPACITY, "ee_kv_bind: pool smaller than ee_kv_pool_bytes");
    if ((uintptr_t)dev_pool % 256 != 0) return ee_fail(EE_ERR_INVALID_ARG, "ee_kv_bind: pool must be 256-byte aligned");
    ee_kv* kv = new (std::nothrow) ee_kv();
    if (!kv) return ee_fail(EE_ERR_INVALID_ARG, "ee_kv_bind: out of host memory");
    kv->pool = (char*)dev_pool;
    kv->bytes = pool_bytes;
    kv->n_layers = n_resident_layers;
    kv->B = B;
    kv->T = T;
    kv->h_cap.assign(host_capacity, host_capacity + B);
    kv->h_off.resize(B);
    int64_t acc = 0;
    for (int b = 0; b < B; ++b) { kv->h_off[b] = acc; acc += host_capacity[b]; }
    hipError_t e = hipMalloc((void**)&kv->d_cap, sizeof(int32_t) * B);
    if (e == hipSuccess) e = hipMalloc((void**)&kv->d_off, sizeof(int64_t) * B);
    if (e == hipSuccess) e = hipMemcpy(kv->d_cap, kv->h_cap.data(), sizeof(int32_t) * B, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(kv->d_off, kv->h_off.data(), sizeof(int64_t) * B, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        ee_kv_destroy(kv);
        return ee_fail(EE_ERR_HIP, std::string("ee_kv_bind: ") + hipGetErrorString(e));
    }
    *out = kv;
    return EE_OK;
}

int ee_kv_destroy(ee_kv* kv) {
    if (!kv) return EE_OK;
    if (kv->d_cap) (void)hipFree(kv->d_cap);
    if (kv->d_off) (void)hipFree(kv->d_off);
    delete kv;
    return EE_OK;
}

static int check_context_args(const ee_model* m, const ee_kv* kv, int layer, int row, int pos0, int n_pos,
                              const void* k, const void* v) {
    if (!m || !kv || !k || !v) return ee_fail(EE_ERR_INVALID_ARG, "key/value context copy: null pointer");
    if (layer < 1 || layer > kv->n_layers) return ee_fail(EE_ERR_CAPACITY, "key/value context copy: layer not in the pool");
    if (row < 0 || row >= kv->B) return ee_fail(EE_ERR_CAPACITY, "key/value context copy: row out of range");
    if (pos0 < 0 || n_pos < 0 || (int64_t)pos0 + n_pos > kv->h_cap[row])
        return ee_fail(EE_ERR_CAPACITY, "key/value context copy: positions exceed the row capacity");
    return EE_OK;
}

int ee_kv_write_context(const ee_model* m, ee_kv* kv, int layer, int row, int pos0, int n_pos,
                        const void* dev_k, const void* dev_v, void* stream) {
    int rc = check_context_args(m, kv, layer, row, pos0, n_pos, dev_k, dev_v);
    if (rc != EE_OK) return rc;
    return launch_kv_copy_context(m, kv, layer, row, pos0, n_pos, const_cast<void*>(dev_k),
                                  const_cast<void*>(dev_v), true, as_stream(stream));
}

int ee_kv_read_context(const ee_model* m, const ee_kv* kv, int layer, int row, int pos0, int n_pos,
                       void* dev_k, void* dev_v, void* stream) {
    int rc = check_context_args(m, kv, layer, row, pos0, n_pos, dev_k, dev_v);
    if (rc != EE_OK) return rc;
    return launch_kv_copy_context(m, kv, layer, row, pos0, n_pos, dev_k, dev_v, false, as_stream(stream));
}

// ------------------------------------------------------------------ batch
static void lay_state(const ee_model* m, int B, ee_batch_layout* L, size_t* total) {
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L->h = take((size_t)B * m->cfg.d_model * 4);
    L->tok_in = take((size_t)B * 4);
    L->pos = take((size_t)B * 4);
    L->row_scale = take((size_t)B * 4);
    L->active_idx = take((size_t)B * 4);
    L->n_active = take(4);
    L->exited_idx = take((size_t)B * 4);
    L->n_exited = take(4);
    L->head_conf = take((size_t)B * 4);
    L->head_tok = take((size_t)B * 4);
    L->head_exit = take((size_t)B);
    L->head_breach = take((size_t)B);
    L->out_tok = take((size_t)B * 4);
    L->out_layer = take((size_t)B * 4);
    L->out_conf = take((size_t)B * 4);
    L->out_breach = take((size_t)B);
    L->exit_counts = take(EE_MAX_EXITS * 4);
    L->breach_count = take(4);
    L->status = take(4);
    *total = o;
}

static void lay_workspace(const ee_model* m, int B, WsLayout* W) {
    const ee_model_config& c = m->cfg;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    size_t Mpad = align_up((size_t)B, 32);
    size_t qd = (size_t)c.n_q_heads * c.head_dim, qkv = qd + 2 * (size_t)c.n_kv_heads * c.head_dim;
    size_t kvn = 2 * (size_t)c.n_kv_heads * c.head_dim;
    if (c.dtype == EE_BF16) {
        size_t n_part = (size_t)c.vocab / 32;
        W->x = take(Mpad * c.d_model * 2);
        W->qkv = take(Mpad * qkv * 4);
        W->q_hi = take(Mpad * qd * 2);
        W->q_lo = take(Mpad * qd * 2);
        W->ao = take(Mpad * qd * 2);
        W->act = take(Mpad * c.d_ffn * 2);
        W->part_max = take(Mpad * n_part * 4);
        W->part_sum = take(Mpad * n_part * 4);
        W->part_arg = take(Mpad * n_part * 4);
        W->logits = take(0);
        size_t fill_layers = c.n_layers > 1 ? (size_t)c.n_layers - 1 : 1;   // all skipped layers in one launch
        W->fill_x = take(fill_layers * Mpad * c.d_model * 2);
        W->fill_kv = take(fill_layers * Mpad * kvn * 4);
        W->gemm_part_bytes = Mpad * ((size_t)384 << 10);   // K-slice planes: 96 MiB at 256 rows
        W->gemm_part = take(W->gemm_part_bytes);
        size_t pairs = Mpad * (size_t)c.n_kv_heads;   // position shares only when there are few pairs
        W->attn_part_bytes = pairs < 512 + 32 * (size_t)c.n_kv_heads ? pairs * 16 * 16 * 130 * 4 : 0;
        W->attn_part = take(W->attn_part_bytes);
        W->attn_order = take(Mpad * 4);
        W->kv_seq = take(Mpad * 4);
        W->gone_idx = take(Mpad * 4);
        W->n_gone = take(4);
    } else {
        size_t wide = (size_t)c.vocab > 2 * (size_t)c.d_ffn ? (size_t)c.vocab : 2 * (size_t)c.d_ffn;
        W->x = take(Mpad * c.d_model * 4);
        W->qkv = take(Mpad * qkv * 4);
        W->q_hi = take(0);
        W->q_lo = take(0);
        W->ao = take(Mpad * qd * 4);
        W->act = take(Mpad * c.d_ffn * 4);
        W->part_max = take(Mpad * 4);
        W->part_sum = take(Mpad * 4);
        W->part_arg = take(Mpad * 4);
        W->logits = take(Mpad * wide * 4);
        W->fill_x = take(Mpad * c.d_model * 4);
        W->fill_kv = take(Mpad * kvn * 4);
        W->gemm_part_bytes = 0; W->gemm_part = take(0);
        W->attn_part_bytes = 0; W->attn_part = take(0);
        W->attn_order = take(0);
        W->kv_seq = take(Mpad * 4);
        W->gone_idx = take(Mpad * 4);
        W->n_gone = take(4);
    }
    W->total = o;
}

size_t ee_batch_state_bytes(const ee_model* m, int B) {
    if (!m || B < 1) return 0;
    ee_batch_layout L;
    size_t t = 0;
    lay_state(m, B, &L, &t);
    return t;
}

size_t ee_workspace_bytes(const ee_model* m, int B) {
    if (!m || B < 1) return 0;
    WsLayout W;
    lay_workspace(m, B, &W);
    return W.total;
}

int ee_batch_get_layout(const ee_model* m, int B, ee_batch_layout* out) {
    if (!m || !out || B < 1) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_get_layout: bad argument");
    size_t t = 0;
    lay_state(m, B, out, &t);
    return EE_OK;
}

int ee_batch_bind(const ee_model* m, int B, void* dev_state, size_t state_bytes, void* dev_workspace,
                  size_t workspace_bytes, ee_batch** out) {
    if (!m || !dev_state || !dev_workspace || !out) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_bind: null pointer");
    if (B < 1 || B > 65535) return ee_fail(EE_ERR_CAPACITY, "ee_batch_bind: batch must be in 1..65535");
    if ((uintptr_t)dev_state % 256 != 0 || (uintptr_t)dev_workspace % 256 != 0)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_bind: buffers must be 256-byte aligned");
    if (state_bytes < ee_batch_state_bytes(m, B) || workspace_bytes < ee_workspace_bytes(m, B))
        return ee_fail(EE_ERR_CAPACITY, "ee_batch_bind: state or workspace buffer too small");
    ee_batch* b = new (std::nothrow) ee_batch();
    if (!b) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_bind: out of host memory");
    b->m = m;
    b->B = B;
    b->Mpad = (int)align_up((size_t)B, 32);
    b->state = (char*)dev_state;
    b->ws = (char*)dev_workspace;
    size_t t = 0;
    lay_state(m, B, &b->L, &t);
    lay_workspace(m, B, &b->W);
    *out = b;
    return EE_OK;
}

int ee_batch_destroy(ee_batch* b) {
    delete b;
    return EE_OK;
}

int ee_batch_reset(ee_batch* b, const int32_t* dev_tok_in, const int32_t* dev_pos, const float* dev_row_scale,
                   void* stream) {
    if (!b || !dev_tok_in || !dev_pos) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_reset: null pointer");
    return launch_reset(b, dev_tok_in, dev_pos, dev_row_scale, as_stream(stream));
}

int ee_batch_set_row_scale(ee_batch* b, const float* dev_row_scale, void* stream) {
    if (!b || !dev_row_scale) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_set_row_scale: null pointer");
    return launch_set_scale(b, dev_row_scale, as_stream(stream));
}

int ee_batch_begin_step(const ee_model* m, ee_batch* b, void* stream) {
    if (!m || !b || b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_begin_step: batch not bound to this model");
    if (!m->emb) return ee_fail(EE_ERR_INVALID_ARG, "ee_batch_begin_step: embedding not set");
    return launch_begin_step(m, b, as_stream(stream));
}

// ------------------------------------------------------------------ hot path
static int check_pair(const char* who, const ee_model* m, const ee_kv* kv, const ee_batch* b) {
    if (!m || !b || (kv == nullptr)) return ee_fail(EE_ERR_INVALID_ARG, std::string(who) + ": null handle");
    if (b->m != m) return ee_fail(EE_ERR_INVALID_ARG, std::string(who) + ": batch not bound to this model");
    if (kv->B != b->B) return ee_fail(EE_ERR_CAPACITY, std::string(who) + ": cache and batch have different row counts");
    return EE_OK;
}

int ee_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, void* stream) {
    int rc = check_pair("ee_layer_forward", m, kv, b);
    if (rc != EE_OK) return rc;
    if (layer < 1 || layer > m->cfg.n_layers) return ee_fail(EE_ERR_INVALID_ARG, "ee_layer_forward: layer out of range");
    if (!m->resident[layer - 1]) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, "ee_layer_forward: layer is not resident");
    if (layer > kv->n_layers) return ee_fail(EE_ERR_CAPACITY, "ee_layer_forward: cache holds fewer layers");
    return m->cfg.dtype == EE_BF16 ? bf16_layer_forward(m, layer, kv, b, as_stream(stream))
                                   : f32_layer_forward(m, layer, kv, b, as_stream(stream));
}

int ee_exit_head(const ee_model* m, int exit_idx, float threshold, int force_exit, ee_batch* b,
                 float* dev_dbg_logits, void* stream) {
    if (!m || !b || b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head: batch not bound to this model");
    if (exit_idx < 0 || exit_idx >= m->cfg.n_exits) return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head: exit index out of range");
    if (!m->exits[exit_idx].set) return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, "ee_exit_head: exit head not set");
    if (std::isnan(threshold)) return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head: threshold is NaN");
    return m->cfg.dtype == EE_BF16
               ? bf16_exit_head(m, exit_idx, threshold, force_exit ? 1 : 0, b, dev_dbg_logits, as_stream(stream))
               : f32_exit_head(m, exit_idx, threshold, force_exit ? 1 : 0, b, dev_dbg_logits, as_stream(stream));
}

int ee_compact_active(ee_batch* b, int exit_idx, int exit_layer, void* stream) {
    if (!b) return ee_fail(EE_ERR_INVALID_ARG, "ee_compact_active: null batch");
    if (exit_idx < 0 || exit_idx >= EE_MAX_EXITS) return ee_fail(EE_ERR_INVALID_ARG, "ee_compact_active: exit index out of range");
    return launch_compact(b, exit_idx, exit_layer, as_stream(stream));
}

int ee_fill_skipped_kv(const ee_model* m, int from_layer_excl, int to_layer_incl, ee_kv* kv, ee_batch* b,
                       void* stream) {
    int rc = check_pair("ee_fill_skipped_kv", m, kv, b);
    if (rc != EE_OK) return rc;
    if (from_layer_excl < 0 || to_layer_incl > m->cfg.n_layers)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_fill_skipped_kv: layer range out of the model");
    for (int l = from_layer_excl + 1; l <= to_layer_incl; ++l)
        if (!m->resident[l - 1]) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, "ee_fill_skipped_kv: layer is not resident");
    if (to_layer_incl > kv->n_layers) return ee_fail(EE_ERR_CAPACITY, "ee_fill_skipped_kv: cache holds fewer layers");
    if (from_layer_excl >= to_layer_incl) return EE_OK;
    return m->cfg.dtype == EE_BF16 ? bf16_fill_kv(m, from_layer_excl, to_layer_incl, kv, b, as_stream(stream))
                                   : f32_fill_kv(m, from_layer_excl, to_layer_incl, kv, b, as_stream(stream));
}

int ee_prefill(const ee_model* m, ee_kv* kv, ee_batch* b, const int32_t* dev_tok, const int32_t* dev_pos,
               const int32_t* dev_seq, int n, void* stream) {
    if (!m || !kv || !b) return ee_fail(EE_ERR_INVALID_ARG, "ee_prefill: null handle");
    if (b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_prefill: batch not bound to this model");
    if (n < 0 || n > b->B) return ee_fail(EE_ERR_CAPACITY, "ee_prefill: more entries than the batch has rows");
    if (n == 0) return EE_OK;
    if (!dev_tok || !dev_pos || !dev_seq) return ee_fail(EE_ERR_INVALID_ARG, "ee_prefill: null array");
    int R = ee_model_resident_depth(m);
    if (R < 0) return R;
    if (R == 0) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, "ee_prefill: no layer is resident");
    if (kv->n_layers < R) return ee_fail(EE_ERR_CAPACITY, "ee_prefill: cache was bound for fewer layers than are resident");
    if (!m->emb) return ee_fail(EE_ERR_INVALID_ARG, "ee_prefill: embedding not set");
    const ee_model_config& c = m->cfg;
    hipStream_t s = as_stream(stream);
    int rc = launch_prefill_begin(m, kv, b, dev_tok, dev_pos, dev_seq, n, s);
    b->kv_seq = b->wsp<int32_t>(b->W.kv_seq);      // the layers address the cache through the entry's row
    bool x_ready = false;
    for (int l = 1; l <= R && rc == EE_OK; ++l) {
        if (c.dtype == EE_BF16) {
            const float* tail_gain = l < R ? (const float*)m->layers[l].g_attn : nullptr;
            bool x_done = false;
            rc = bf16_layer_forward(m, l, kv, b, s, x_ready, tail_gain, &x_done);
            x_ready = x_done;
        } else {
            rc = f32_layer_forward(m, l, kv, b, s);
        }
    }
    b->kv_seq = nullptr;
    return rc;
}

size_t ee_hstore_bytes(const ee_model* m, const ee_kv* kv) {
    if (!m || !kv) return 0;
    return (size_t)kv->T * (size_t)m->cfg.d_model * sizeof(float);
}

int ee_hstore_put_step(const ee_model* m, const ee_kv* kv, const ee_batch* b, float* dev_store, void* stream) {
    int rc = check_pair("ee_hstore_put_step", m, kv, b);
    if (rc != EE_OK) return rc;
    if (!dev_store) return ee_fail(EE_ERR_INVALID_ARG, "ee_hstore_put_step: null store");
    return launch_hstore_put(m, kv, b, b->B, false, dev_store, as_stream(stream));
}

int ee_hstore_put_prefill(const ee_model* m, const ee_kv* kv, const ee_batch* b, int n, float* dev_store, void* stream) {
    if (!m || !kv || !b || !dev_store) return ee_fail(EE_ERR_INVALID_ARG, "ee_hstore_put_prefill: null pointer");
    if (b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_hstore_put_prefill: batch not bound to this model");
    if (n < 0 || n > b->B) return ee_fail(EE_ERR_CAPACITY, "ee_hstore_put_prefill: more entries than the batch has rows");
    if (n == 0) return EE_OK;
    return launch_hstore_put(m, kv, b, n, true, dev_store, as_stream(stream));
}

int ee_backfill_kv(const ee_model* m, int from_layer_excl, int to_layer_incl, ee_kv* kv, ee_batch* b,
                   const float* dev_store, const int32_t* dev_pos, const int32_t* dev_seq, int n, void* stream) {
    if (!m || !kv || !b) return ee_fail(EE_ERR_INVALID_ARG, "ee_backfill_kv: null handle");
    if (b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_backfill_kv: batch not bound to this model");
    if (n < 0 || n > b->B) return ee_fail(EE_ERR_CAPACITY, "ee_backfill_kv: more entries than the batch has rows");
    if (from_layer_excl < 0 || to_layer_incl > m->cfg.n_layers)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_backfill_kv: layer range out of the model");
    for (int l = from_layer_excl + 1; l <= to_layer_incl; ++l)
        if (!m->resident[l - 1]) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, "ee_backfill_kv: layer is not resident");
    if (to_layer_incl > kv->n_layers) return ee_fail(EE_ERR_CAPACITY, "ee_backfill_kv: cache holds fewer layers");
    if (from_layer_excl >= to_layer_incl || n == 0) return EE_OK;
    if (!dev_store || !dev_pos || !dev_seq) return ee_fail(EE_ERR_INVALID_ARG, "ee_backfill_kv: null array");
    hipStream_t s = as_stream(stream);
    int rc = launch_backfill_begin(m, kv, b, dev_store, dev_pos, dev_seq, n, s);
    if (rc != EE_OK) return rc;
    b->kv_seq = b->wsp<int32_t>(b->W.kv_seq);
    rc = m->cfg.dtype == EE_BF16 ? bf16_fill_kv(m, from_layer_excl, to_layer_incl, kv, b, s)
                                 : f32_fill_kv(m, from_layer_excl, to_layer_incl, kv, b, s);
    b->kv_seq = nullptr;
    return rc;
}

// ------------------------------------------------------------------ self-speculative decoding
// layers first .. last on the batch's active rows, the way the decode step chains them: the kernel that
// finishes a layer leaves the normalised operand of what comes next (next layer, or the head `then_gain`)
static int run_layers(const ee_model* m, int first, int last, ee_kv* kv, ee_batch* b, const float* then_gain,
                      hipStream_t s, bool* x_ready_out) {
    int rc = EE_OK;
    bool x_ready = false;
    for (int l = first; l <= last && rc == EE_OK; ++l) {
        if (m->cfg.dtype == EE_BF16) {
            const float* tail_gain = l < last ? (const float*)m->layers[l].g_attn : then_gain;
            bool x_done = false;
            rc = bf16_layer_forward(m, l, kv, b, s, x_ready, tail_gain, &x_done);
            x_ready = x_done;
        } else {
            rc = f32_layer_forward(m, l, kv, b, s);
        }
    }
    *x_ready_out = x_ready;
    return rc;
}

static int head_on(const ee_model* m, int e, ee_batch* b, hipStream_t s, bool x_ready) {
    // greedy token of head e for every active row: threshold 0 is always met, so no row is a breach
    return m->cfg.dtype == EE_BF16 ? bf16_exit_head(m, e, 0.0f, 1, b, nullptr, s, x_ready)
                                   : f32_exit_head(m, e, 0.0f, 1, b, nullptr, s);
}

static int check_speculation(const char* who, const ee_model* m, const ee_kv* kv, int draft_exit, int* Le, int* R,
                             int* last_exit) {
    const ee_model_config& c = m->cfg;
    *R = ee_model_resident_depth(m);
    if (*R < 0) return *R;
    if (*R == 0) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, std::string(who) + ": no layer is resident");
    if (draft_exit < 0 || draft_exit >= c.n_exits) return ee_fail(EE_ERR_INVALID_ARG, std::string(who) + ": exit index out of range");
    *Le = c.exit_layers[draft_exit];
    *last_exit = -1;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] == *R) *last_exit = e;
    if (*last_exit < 0 || !m->exits[*last_exit].set)
        return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, std::string(who) + ": the deepest resident layer carries no exit head");
    if (*Le >= *R) return ee_fail(EE_ERR_INVALID_ARG, std::string(who) + ": the draft exit must lie below the deepest resident layer");
    if (!m->exits[draft_exit].set) return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, std::string(who) + ": the draft exit head was never set");
    if (kv->n_layers < *R) return ee_fail(EE_ERR_CAPACITY, std::string(who) + ": cache was bound for fewer layers than are resident");
    if (!m->emb) return ee_fail(EE_ERR_INVALID_ARG, std::string(who) + ": embedding not set");
    return EE_OK;
}

int ee_draft_step(const ee_model* m, ee_kv* kv, ee_batch* b, int draft_exit, int32_t* dev_draft_out, void* stream) {
    int rc = check_pair("ee_draft_step", m, kv, b);
    if (rc != EE_OK) return rc;
    int Le, R, last_exit;
    rc = check_speculation("ee_draft_step", m, kv, draft_exit, &Le, &R, &last_exit);
    if (rc != EE_OK) return rc;
    hipStream_t s = as_stream(stream);
    rc = ee_batch_begin_step(m, b, stream);
    bool x_ready = false;
    if (rc == EE_OK) rc = run_layers(m, 1, Le, kv, b, (const float*)m->exits[draft_exit].gain, s, &x_ready);
    if (rc == EE_OK) rc = head_on(m, draft_exit, b, s, x_ready);
    if (rc == EE_OK) rc = ee_compact_active(b, draft_exit, Le, stream);          // every row leaves: out_tok = its draft
    if (rc == EE_OK) rc = launch_end_step(b, s);
    if (rc == EE_OK && dev_draft_out)
        EE_HIP_CHECK(hipMemcpyAsync(dev_draft_out, b->st<int32_t>(b->L.out_tok), sizeof(int32_t) * b->B,
                                    hipMemcpyDeviceToDevice, s));
    return rc;
}

int ee_verify_drafts(const ee_model* m, ee_kv* kv, ee_batch* b, ee_batch* vb, int draft_exit, int k,
                     const float* dev_store, const int32_t* dev_drafts, int32_t* dev_n_emit, int32_t* dev_emit,
                     void* stream) {
    int rc = check_pair("ee_verify_drafts", m, kv, b);
    if (rc != EE_OK) return rc;
    if (!vb || vb->m != m || vb == b) return ee_fail(EE_ERR_INVALID_ARG, "ee_verify_drafts: the entries batch must be another batch of this model");
    if (!dev_store || !dev_drafts || !dev_n_emit || !dev_emit) return ee_fail(EE_ERR_INVALID_ARG, "ee_verify_drafts: null array");
    if (k < 1) return ee_fail(EE_ERR_INVALID_ARG, "ee_verify_drafts: at least one draft per row");
    if ((int64_t)b->B * k > vb->B) return ee_fail(EE_ERR_CAPACITY, "ee_verify_drafts: the entries batch has fewer than B * k rows");
    int Le, R, last_exit;
    rc = check_speculation("ee_verify_drafts", m, kv, draft_exit, &Le, &R, &last_exit);
    if (rc != EE_OK) return rc;
    hipStream_t s = as_stream(stream);
    rc = launch_verify_begin(m, kv, b, vb, k, dev_store, s);
    vb->kv_seq = vb->wsp<int32_t>(vb->W.kv_seq);   // the layers address the cache through the entry's row
    bool x_ready = false;
    if (rc == EE_OK) rc = run_layers(m, Le + 1, R, kv, vb, (const float*)m->exits[last_exit].gain, s, &x_ready);
    vb->kv_seq = nullptr;
    if (rc == EE_OK) rc = head_on(m, last_exit, vb, s, x_ready);
    if (rc == EE_OK) rc = launch_accept_drafts(b, vb, k, dev_drafts, dev_n_emit, dev_emit, s);
    return rc;
}

size_t ee_cbc_state_bytes(int window) {
    if (window < 1 || window > EE_CBC_MAX_WINDOW) return 0;
    return align_up(sizeof(ee_cbc_state) + (size_t)window, 8);
}

int ee_cbc_init(void* dev_state, int window, int cbc_max, void* stream) {
    if (!dev_state) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_init: null state");
    if (window < 1 || window > EE_CBC_MAX_WINDOW) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_init: window out of range");
    if (cbc_max < 0) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_init: negative cbc_max");
    return launch_cbc_init(dev_state, window, cbc_max, as_stream(stream));
}

int ee_cbc_push(void* dev_state, const uint8_t* dev_flags, int n, void* stream) {
    if (!dev_state || (!dev_flags && n > 0)) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_push: null pointer");
    if (n < 0) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_push: negative token count");
    if (n == 0) return EE_OK;
    return launch_cbc_push(dev_state, dev_flags, n, as_stream(stream));
}

int ee_cbc_push_step(void* dev_state, const ee_batch* b, void* stream) {
    if (!dev_state || !b) return ee_fail(EE_ERR_INVALID_ARG, "ee_cbc_push_step: null pointer");
    return launch_cbc_push(dev_state, b->st<uint8_t>(b->L.out_breach), b->B, as_stream(stream));
}

int ee_pht_init(void* dev_row, void* stream) {
    if (!dev_row) return ee_fail(EE_ERR_INVALID_ARG, "ee_pht_init: null row");
    return launch_pht_init(dev_row, as_stream(stream));
}

int ee_pht_push_step(void* dev_row, const ee_model* m, const ee_batch* b, void* stream) {
    if (!dev_row || !m || !b) return ee_fail(EE_ERR_INVALID_ARG, "ee_pht_push_step: null pointer");
    if (b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_pht_push_step: batch not bound to this model");
    return launch_pht_push(dev_row, m, b, as_stream(stream));
}

// what every form of the decode step checks first; *R_out = deepest resident layer, *n_res_out = resident exits
static int check_step(const char* who, const ee_model* m, const ee_kv* kv, const ee_batch* b, const float* host_thresholds,
                      int n_thresholds, int* R_out, int* n_res_out) {
    const std::string w(who);
    int rc = check_pair(who, m, kv, b);
    if (rc != EE_OK) return rc;
    if (!host_thresholds) return ee_fail(EE_ERR_INVALID_ARG, w + ": null thresholds");
    int R = ee_model_resident_depth(m);
    if (R < 0) return R;
    if (R == 0) return ee_fail(EE_ERR_LAYER_NOT_RESIDENT, w + ": no layer is resident");
    const ee_model_config& c = m->cfg;
    int n_res = 0;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] <= R) ++n_res;
    if (n_res == 0 || c.exit_layers[n_res - 1] != R)
        return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, w + ": the deepest resident layer carries no exit head");
    for (int e = 0; e < n_res; ++e)
        if (!m->exits[e].set) return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, w + ": a resident exit head was never set");
    if (n_thresholds != n_res) return ee_fail(EE_ERR_INVALID_ARG, w + ": one threshold per resident exit is required");
    for (int e = 0; e < n_res; ++e)
        if (std::isnan(host_thresholds[e])) return ee_fail(EE_ERR_INVALID_ARG, w + ": threshold is NaN");
    if (kv->n_layers < R) return ee_fail(EE_ERR_CAPACITY, w + ": cache was bound for fewer layers than are resident");
    if (!m->emb) return ee_fail(EE_ERR_INVALID_ARG, w + ": embedding not set");
    *R_out = R;
    *n_res_out = n_res;
    return EE_OK;
}

// Segment e of a step: the layers after exit e - 1 up to exit layer e (segment 0 starts with the embedding), the
// exit head there, the compaction, and the K/V of the layers up to the next exit for the rows that have left.
static int step_segment(const ee_model* m, ee_kv* kv, ee_batch* b, const float* host_thresholds, int e, int R, void* s) {
    const ee_model_config& c = m->cfg;
    int rc = e == 0 ? ee_batch_begin_step(m, b, s) : EE_OK;
    const int first = e == 0 ? 1 : c.exit_layers[e - 1] + 1, last = c.exit_layers[e];
    // bf16: the kernel that finishes a layer can leave the normalised operand of whatever comes
    // next (the exit head, or the next layer when no compaction lies between): one launch less
    bool x_ready = false;
    for (int l = first; l <= last && rc == EE_OK; ++l) {
        if (c.dtype == EE_BF16) {
            const float* tail_gain = l == last ? (const float*)m->exits[e].gain : (const float*)m->layers[l].g_attn;
            bool x_done = false;
            rc = bf16_layer_forward(m, l, kv, b, as_stream(s), x_ready, tail_gain, &x_done);
            x_ready = x_done;
        } else {
            rc = ee_layer_forward(m, l, kv, b, s);
        }
    }
    if (rc != EE_OK) return rc;
    if (c.dtype == EE_BF16)
        rc = bf16_exit_head(m, e, host_thresholds[e], last == R ? 1 : 0, b, nullptr, as_stream(s), x_ready);
    else
        rc = ee_exit_head(m, e, host_thresholds[e], last == R, b, nullptr, s);
    if (rc == EE_OK) rc = ee_compact_active(b, e, last, s);    // renumbers the list entries
    if (rc != EE_OK || last == R) return rc;
    if (c.dtype == EE_BF16) {
        // Sec. 2.2 asks for the skipped layers' K/V of every row that left; when they are computed
        // within the step is free, since nothing reads them before the next step.  Filling only up
        // to the next exit layer, for all rows that have left so far in this step, reads W_k, W_v of
        // every layer once per step instead of once per earlier exit.
        rc = bf16_fill_kv(m, last, c.exit_layers[e + 1], kv, b, as_stream(s), b->wsp<int32_t>(b->W.gone_idx),
                          b->wsp<int32_t>(b->W.n_gone));
    } else {
        rc = ee_fill_skipped_kv(m, last, R, kv, b, s);
    }
    return rc;
}

int ee_decode_step(const ee_model* m, ee_kv* kv, ee_batch* b, const float* host_thresholds, int n_thresholds,
                   void* stream) {
    int R = 0, n_res = 0;
    int rc = check_step("ee_decode_step", m, kv, b, host_thresholds, n_thresholds, &R, &n_res);
    for (int e = 0; e < n_res && rc == EE_OK; ++e) rc = step_segment(m, kv, b, host_thresholds, e, R, stream);
    if (rc == EE_OK) rc = launch_end_step(b, as_stream(stream));
    return rc;
}

int ee_decode_segment(const ee_model* m, ee_kv* kv, ee_batch* b, const float* host_thresholds, int n_thresholds,
                      int segment, void* stream) {
    int R = 0, n_res = 0;
    int rc = check_step("ee_decode_segment", m, kv, b, host_thresholds, n_thresholds, &R, &n_res);
    if (rc != EE_OK) return rc;
    if (segment < 0 || segment >= n_res) return ee_fail(EE_ERR_INVALID_ARG, "ee_decode_segment: no such segment");
    return step_segment(m, kv, b, host_thresholds, segment, R, stream);
}

int ee_decode_finish(const ee_model* m, ee_kv* kv, ee_batch* b, int last_segment, void* stream) {
    int rc = check_pair("ee_decode_finish", m, kv, b);
    if (rc != EE_OK) return rc;
    int R = ee_model_resident_depth(m);
    if (R <= 0) return R < 0 ? R : ee_fail(EE_ERR_LAYER_NOT_RESIDENT, "ee_decode_finish: no layer is resident");
    const ee_model_config& c = m->cfg;
    int n_res = 0;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] <= R) ++n_res;
    if (last_segment < 0 || last_segment >= n_res) return ee_fail(EE_ERR_INVALID_ARG, "ee_decode_finish: no such segment");
    if (kv->n_layers < R) return ee_fail(EE_ERR_CAPACITY, "ee_decode_finish: cache was bound for fewer layers than are resident");
    // the segments that were not run would have filled the K/V of their layers for the rows that have left
    // (all of them, if the caller stops here rightly); an fp32 segment fills through layer R itself
    if (c.dtype == EE_BF16 && last_segment + 1 < n_res && c.exit_layers[last_segment + 1] < R)
        rc = bf16_fill_kv(m, c.exit_layers[last_segment + 1], R, kv, b, as_stream(stream), b->wsp<int32_t>(b->W.gone_idx),
                          b->wsp<int32_t>(b->W.n_gone));
    if (rc == EE_OK) rc = launch_end_step(b, as_stream(stream));
    return rc;
}

}  // extern "C"
