// ee_oracle.cpp -- CPU oracle for the batched early-exit decode step.
//
// TEST INFRASTRUCTURE ONLY (see ee_oracle.h).  Row-at-a-time, no blocking, no
// fusion: each function is the definition of the operation written out, so it
// can be checked against the paper (HELIOS, arXiv 2504.10724) and the Llama
// decoder definitions by eye.  Sums are accumulated in fp64 and rounded once.
#include "ee_oracle.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace {

struct Layer {
    const float* g_attn = nullptr;
    const void*  W_qkv  = nullptr;
    const void*  W_o    = nullptr;
    const float* g_ffn  = nullptr;
    const void*  W_gate = nullptr;
    const void*  W_up   = nullptr;
    const void*  W_down = nullptr;
    bool resident = false;
};

struct Exit {
    const float* g = nullptr;
    const void*  W = nullptr;
    bool set = false;
};

inline float bf16_bits_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// round-to-nearest-even to the 8-bit-mantissa bfloat16 grid, result as fp32
inline float round_to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return f;  // inf / nan unchanged
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    std::memcpy(&f, &u, 4);
    return f;
}

inline float weight_at(const void* W, int dtype, size_t idx) {
    if (dtype == ORC_BF16) return bf16_bits_to_f32(((const uint16_t*)W)[idx]);
    return ((const float*)W)[idx];
}

}  // namespace

struct orc_model {
    orc_config cfg;
    std::vector<Layer> layers;  // index 0 = layer 1
    std::vector<Exit>  exits;
    const void*  emb = nullptr;
    double rope_theta = 0.0;  // 0 = not set
    int max_pos = 0;
};

extern "C" {

int orc_model_create(const orc_config* cfg, orc_model** out) {
    if (!cfg || !out) return ORC_ERR_ARG;
    if (cfg->n_layers < 1 || cfg->d_model < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 ||
        cfg->n_q_heads % cfg->n_kv_heads != 0 || cfg->head_dim < 2 || cfg->head_dim % 2 != 0 ||
        cfg->d_ffn < 1 || cfg->vocab < 1 || cfg->n_exits < 1 || cfg->n_exits > 16)
        return ORC_ERR_ARG;
    if (cfg->dtype != ORC_F32 && cfg->dtype != ORC_BF16) return ORC_ERR_ARG;
    for (int e = 0; e < cfg->n_exits; ++e) {
        if (cfg->exit_layers[e] < 1 || cfg->exit_layers[e] > cfg->n_layers) return ORC_ERR_ARG;
        if (e > 0 && cfg->exit_layers[e] <= cfg->exit_layers[e - 1]) return ORC_ERR_ARG;
    }
    orc_model* m = new orc_model();
    m->cfg = *cfg;
    m->layers.resize(cfg->n_layers);
    m->exits.resize(cfg->n_exits);
    *out = m;
    return ORC_OK;
}

void orc_model_destroy(orc_model* m) { delete m; }

int orc_model_set_layer(orc_model* m, int layer, const float* g_attn, const void* W_qkv,
                        const void* W_o, const float* g_ffn, const void* W_gate,
                        const void* W_up, const void* W_down) {
    if (!m || layer < 1 || layer > m->cfg.n_layers) return ORC_ERR_ARG;
    if (!g_attn || !W_qkv || !W_o || !g_ffn || !W_gate || !W_up || !W_down) return ORC_ERR_ARG;
    Layer& L = m->layers[layer - 1];
    L.g_attn = g_attn; L.W_qkv = W_qkv; L.W_o = W_o;
    L.g_ffn = g_ffn;   L.W_gate = W_gate; L.W_up = W_up; L.W_down = W_down;
    L.resident = true;
    return ORC_OK;
}

int orc_model_set_exit(orc_model* m, int exit_idx, const float* g_exit, const void* W_exit) {
    if (!m || exit_idx < 0 || exit_idx >= m->cfg.n_exits || !g_exit || !W_exit) return ORC_ERR_ARG;
    m->exits[exit_idx].g = g_exit;
    m->exits[exit_idx].W = W_exit;
    m->exits[exit_idx].set = true;
    return ORC_OK;
}

int orc_model_set_embed(orc_model* m, const void* emb) {
    if (!m || !emb) return ORC_ERR_ARG;
    m->emb = emb;
    return ORC_OK;
}

int orc_model_set_rope(orc_model* m, double theta, int max_pos) {
    if (!m || !(theta > 1.0) || max_pos < 1) return ORC_ERR_ARG;
    m->rope_theta = theta;
    m->max_pos = max_pos;
    return ORC_OK;
}

int orc_model_resident_depth(const orc_model* m) {
    if (!m) return -1;
    int R = 0;
    while (R < m->cfg.n_layers && m->layers[R].resident) ++R;
    for (int l = R; l < m->cfg.n_layers; ++l)
        if (m->layers[l].resident) return -1;  // resident set is not a prefix
    return R;
}

// ------------------------------------------------------------------ primitives

void orc_round_bf16(float* x, size_t n) {
    for (size_t i = 0; i < n; ++i) x[i] = round_to_bf16(x[i]);
}

// RMSNorm: out_i = h_i / sqrt(mean(h^2) + eps) * g_i
void orc_rmsnorm(const float* h, const float* g, int d, float eps, int round_bf16, float* out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += (double)h[i] * (double)h[i];
    float ms  = (float)(ss / (double)d);
    float inv = 1.0f / std::sqrt(ms + eps);
    for (int i = 0; i < d; ++i) {
        float v = (h[i] * inv) * g[i];
        out[i] = round_bf16 ? round_to_bf16(v) : v;
    }
}

// out_j = sum_k x_k W[j][k]
void orc_matvec(const float* x, const void* W, int dtype, int N, int K, float* out) {
    if (dtype == ORC_BF16) {
        const uint16_t* Wb = (const uint16_t*)W;
#pragma omp parallel for schedule(static)
        for (int j = 0; j < N; ++j) {
            const uint16_t* w = Wb + (size_t)j * (size_t)K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += (double)x[k] * (double)bf16_bits_to_f32(w[k]);
            out[j] = (float)acc;
        }
    } else {
        const float* Wf = (const float*)W;
#pragma omp parallel for schedule(static)
        for (int j = 0; j < N; ++j) {
            const float* w = Wf + (size_t)j * (size_t)K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += (double)x[k] * (double)w[k];
            out[j] = (float)acc;
        }
    }
}

// Rotary embedding, half-split pairing: element i pairs with i + hd/2 and the
// pair is rotated by the angle pos * theta^(-2i/hd).  The angle and its cosine
// and sine are evaluated in fp64 and rounded to fp32; the rotation is fp32.
void orc_rope(float* v, int hd, int pos, double theta) {
    int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        double angle = (double)pos * std::pow(theta, -2.0 * (double)i / (double)hd);
        float c = (float)std::cos(angle), s = (float)std::sin(angle);
        float a = v[i], b = v[i + half];
        v[i]        = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

// softmax(q.K^T / sqrt(hd)) . V for one query head
void orc_attention_head(const float* q, const float* K, const float* V, int n_pos, int hd, float* out) {
    std::vector<float> a(n_pos);
    float inv_sqrt = 1.0f / std::sqrt((float)hd);
    float mx = -INFINITY;
    for (int t = 0; t < n_pos; ++t) {
        double acc = 0.0;
        for (int i = 0; i < hd; ++i) acc += (double)q[i] * (double)K[(size_t)t * hd + i];
        a[t] = (float)acc * inv_sqrt;
        if (a[t] > mx) mx = a[t];
    }
    std::vector<double> p(n_pos);
    double denom = 0.0;
    for (int t = 0; t < n_pos; ++t) {
        p[t] = std::exp((double)a[t] - (double)mx);
        denom += p[t];
    }
    for (int i = 0; i < hd; ++i) {
        double acc = 0.0;
        for (int t = 0; t < n_pos; ++t) acc += p[t] * (double)V[(size_t)t * hd + i];
        out[i] = (float)(acc / denom);
    }
}

float orc_silu(float t) { return (float)((double)t / (1.0 + std::exp(-(double)t))); }

// confidence = largest softmax probability = 1 / sum_j exp(z_j - max z);
// token = lowest index attaining the maximum
void orc_softmax_conf(const float* z, int V, float* conf, int32_t* tok) {
    float mx = z[0];
    int32_t arg = 0;
    for (int j = 1; j < V; ++j)
        if (z[j] > mx) { mx = z[j]; arg = j; }
    double S = 0.0;
    for (int j = 0; j < V; ++j) S += std::exp((double)z[j] - (double)mx);
    *conf = (float)(1.0 / S);
    *tok = arg;
}

void orc_compact(const uint8_t* exit_mask, const int32_t* active, int n, int32_t* out_active,
                 int32_t* out_n, int32_t* out_exited, int32_t* out_m) {
    int keep = 0, gone = 0;
    for (int i = 0; i < n; ++i) {
        if (exit_mask[i]) out_exited[gone++] = active[i];
        else              out_active[keep++] = active[i];
    }
    *out_n = keep;
    *out_m = gone;
}

// ------------------------------------------------------------- calls of the path

int orc_embed(const orc_model* m, int32_t tok, float* h_row) {
    if (!m || !m->emb || tok < 0 || tok >= m->cfg.vocab) return ORC_ERR_ARG;
    int d = m->cfg.d_model;
    for (int i = 0; i < d; ++i) h_row[i] = weight_at(m->emb, m->cfg.dtype, (size_t)tok * d + i);
    return ORC_OK;
}

static inline float* kv_at(float* base, const orc_model* m, const orc_kv* kv, int layer, int b,
                           int kvh, int pos) {
    const orc_config& c = m->cfg;
    size_t idx = ((((size_t)(layer - 1) * kv->B + b) * c.n_kv_heads + kvh) * kv->cap + pos) * c.head_dim;
    return base + idx;
}

// K and V of one row for one layer from a (pre-attention-norm) hidden state:
// x = RMSNorm(h; g_attn); k = RoPE(x W_k, pos); v = x W_v; both stored at pos.
static void project_and_store_kv(const orc_model* m, int layer, orc_kv* kv, int b, int pos,
                                 const float* x /* normalised, already rounded */) {
    const orc_config& c = m->cfg;
    const Layer& L = m->layers[layer - 1];
    bool bf = c.dtype == ORC_BF16;
    int hd = c.head_dim, d = c.d_model;
    size_t k_row0 = (size_t)c.n_q_heads * hd;             // first key row of W_qkv
    size_t v_row0 = k_row0 + (size_t)c.n_kv_heads * hd;   // first value row
    std::vector<float> kk(hd), vv(hd);
    for (int g = 0; g < c.n_kv_heads; ++g) {
        const char* Wb = (const char*)L.W_qkv;
        size_t esz = bf ? 2 : 4;
        orc_matvec(x, Wb + (k_row0 + (size_t)g * hd) * d * esz, c.dtype, hd, d, kk.data());
        orc_matvec(x, Wb + (v_row0 + (size_t)g * hd) * d * esz, c.dtype, hd, d, vv.data());
        orc_rope(kk.data(), hd, pos, m->rope_theta);
        if (bf) { orc_round_bf16(kk.data(), hd); orc_round_bf16(vv.data(), hd); }
        std::memcpy(kv_at(kv->K, m, kv, layer, b, g, pos), kk.data(), sizeof(float) * hd);
        std::memcpy(kv_at(kv->V, m, kv, layer, b, g, pos), vv.data(), sizeof(float) * hd);
    }
}

static int layer_forward_row(const orc_model* m, int layer, orc_kv* kv, int b, int pos, float* h) {
    const orc_config& c = m->cfg;
    const Layer& L = m->layers[layer - 1];
    bool bf = c.dtype == ORC_BF16;
    int d = c.d_model, hd = c.head_dim, Hq = c.n_q_heads, Hkv = c.n_kv_heads, F = c.d_ffn;
    if (pos < 0 || pos >= kv->cap || pos >= m->max_pos) return ORC_ERR_ARG;

    // attention half: h += Attn(RMSNorm(h)) W_o
    std::vector<float> x(d);
    orc_rmsnorm(h, L.g_attn, d, c.rms_eps, bf, x.data());
    project_and_store_kv(m, layer, kv, b, pos, x.data());
    std::vector<float> q((size_t)Hq * hd), o((size_t)Hq * hd);
    orc_matvec(x.data(), L.W_qkv, c.dtype, Hq * hd, d, q.data());
    int group = Hq / Hkv;
    for (int i = 0; i < Hq; ++i) {
        orc_rope(&q[(size_t)i * hd], hd, pos, m->rope_theta);
        int g = i / group;  // query head i reads key/value head floor(i / (Hq/Hkv))
        orc_attention_head(&q[(size_t)i * hd], kv_at(kv->K, m, kv, layer, b, g, 0),
                           kv_at(kv->V, m, kv, layer, b, g, 0), pos + 1, hd, &o[(size_t)i * hd]);
    }
    if (bf) orc_round_bf16(o.data(), o.size());
    std::vector<float> r(d);
    orc_matvec(o.data(), L.W_o, c.dtype, d, Hq * hd, r.data());
    for (int i = 0; i < d; ++i) h[i] += r[i];

    // feed-forward half: h += (silu(y W_g) * (y W_u)) W_d
    std::vector<float> y(d), gate(F), up(F), act(F);
    orc_rmsnorm(h, L.g_ffn, d, c.rms_eps, bf, y.data());
    orc_matvec(y.data(), L.W_gate, c.dtype, F, d, gate.data());
    orc_matvec(y.data(), L.W_up, c.dtype, F, d, up.data());
    for (int j = 0; j < F; ++j) act[j] = orc_silu(gate[j]) * up[j];
    if (bf) orc_round_bf16(act.data(), F);
    orc_matvec(act.data(), L.W_down, c.dtype, d, F, r.data());
    for (int i = 0; i < d; ++i) h[i] += r[i];
    return ORC_OK;
}

int orc_layer_forward(const orc_model* m, int layer, orc_kv* kv, const uint8_t* active,
                      const int32_t* pos, float* h) {
    if (!m || !kv || !active || !pos || !h || m->rope_theta == 0.0) return ORC_ERR_ARG;
    if (layer < 1 || layer > m->cfg.n_layers) return ORC_ERR_ARG;
    if (!m->layers[layer - 1].resident) return ORC_ERR_NOT_RESIDENT;
    for (int b = 0; b < kv->B; ++b) {
        if (!active[b]) continue;
        int rc = layer_forward_row(m, layer, kv, b, pos[b], h + (size_t)b * m->cfg.d_model);
        if (rc != ORC_OK) return rc;
    }
    return ORC_OK;
}

int orc_exit_head(const orc_model* m, int exit_idx, const float* h_row, float scale,
                  float* logits, float* conf, int32_t* tok) {
    if (!m || exit_idx < 0 || exit_idx >= m->cfg.n_exits || !h_row || !conf || !tok) return ORC_ERR_ARG;
    const Exit& E = m->exits[exit_idx];
    if (!E.set) return ORC_ERR_NOT_RESIDENT;
    const orc_config& c = m->cfg;
    std::vector<float> x(c.d_model), z(c.vocab);
    orc_rmsnorm(h_row, E.g, c.d_model, c.rms_eps, c.dtype == ORC_BF16, x.data());
    orc_matvec(x.data(), E.W, c.dtype, c.vocab, c.d_model, z.data());
    for (int j = 0; j < c.vocab; ++j) z[j] = z[j] * scale;
    orc_softmax_conf(z.data(), c.vocab, conf, tok);
    if (logits) std::memcpy(logits, z.data(), sizeof(float) * c.vocab);
    return ORC_OK;
}

int orc_fill_skipped_kv(const orc_model* m, int from_excl, int to_incl, orc_kv* kv, int b,
                        int32_t pos_b, const float* h_row) {
    if (!m || !kv || !h_row || m->rope_theta == 0.0) return ORC_ERR_ARG;
    if (from_excl < 0 || to_incl > m->cfg.n_layers || b < 0 || b >= kv->B) return ORC_ERR_ARG;
    if (pos_b < 0 || pos_b >= kv->cap || pos_b >= m->max_pos) return ORC_ERR_ARG;
    const orc_config& c = m->cfg;
    std::vector<float> x(c.d_model);
    // a skipped layer leaves the hidden state as it was, so each deeper layer
    // sees the exit hidden state as its input
    for (int l = from_excl + 1; l <= to_incl; ++l) {
        if (!m->layers[l - 1].resident) return ORC_ERR_NOT_RESIDENT;
        orc_rmsnorm(h_row, m->layers[l - 1].g_attn, c.d_model, c.rms_eps, c.dtype == ORC_BF16, x.data());
        project_and_store_kv(m, l, kv, b, pos_b, x.data());
    }
    return ORC_OK;
}

int orc_decode_step(const orc_model* m, orc_kv* kv, const int32_t* tok_in, int32_t* pos,
                    const float* scale, const float* thresholds, int n_thresholds,
                    int32_t* out_tok, int32_t* out_layer, float* out_conf, uint8_t* out_breach,
                    int32_t* counts, int64_t* layers_run, float* h_out, float* conf_trace) {
    if (!m || !kv || !tok_in || !pos || !thresholds || !out_tok || !out_layer || !out_conf || !out_breach)
        return ORC_ERR_ARG;
    const orc_config& c = m->cfg;
    int R = orc_model_resident_depth(m);
    if (R < 1) return ORC_ERR_ARG;
    // resident exits = exits at layers <= R; the deepest resident layer must be one
    int n_res_exits = 0;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] <= R) ++n_res_exits;
    if (n_res_exits == 0 || c.exit_layers[n_res_exits - 1] != R) return ORC_ERR_NOT_RESIDENT;
    if (n_thresholds != n_res_exits) return ORC_ERR_ARG;
    for (int e = 0; e < n_thresholds; ++e)
        if (thresholds[e] != thresholds[e]) return ORC_ERR_ARG;  // NaN

    int B = kv->B, d = c.d_model;
    std::vector<float> h((size_t)B * d);
    std::vector<uint8_t> active(B, 1);
    for (int b = 0; b < B; ++b) {
        int rc = orc_embed(m, tok_in[b], &h[(size_t)b * d]);
        if (rc != ORC_OK) return rc;
    }
    int n_active = B;
    int next_exit = 0;
    for (int l = 1; l <= R && n_active > 0; ++l) {
        int rc = orc_layer_forward(m, l, kv, active.data(), pos, h.data());
        if (rc != ORC_OK) return rc;
        if (layers_run) *layers_run += n_active;
        if (c.exit_layers[next_exit] != l) continue;
        int e = next_exit++;
        float th = thresholds[e];
        for (int b = 0; b < B; ++b) {
            if (!active[b]) continue;
            float conf; int32_t tok;
            float s = scale ? scale[b] : 1.0f;
            rc = orc_exit_head(m, e, &h[(size_t)b * d], s, nullptr, &conf, &tok);
            if (rc != ORC_OK) return rc;
            if (conf_trace) conf_trace[(size_t)b * c.n_exits + e] = conf;
            bool met = conf >= th;           // "meets" the threshold
            bool last = (l == R);            // nothing deeper is loaded
            if (!(met || last)) continue;
            out_tok[b] = tok;
            out_layer[b] = l;
            out_conf[b] = conf;
            out_breach[b] = (last && !met) ? 1 : 0;
            if (counts) counts[e] += 1;
            rc = orc_fill_skipped_kv(m, l, R, kv, b, pos[b], &h[(size_t)b * d]);
            if (rc != ORC_OK) return rc;
            active[b] = 0;
            --n_active;
        }
    }
    if (h_out) std::memcpy(h_out, h.data(), sizeof(float) * h.size());
    for (int b = 0; b < B; ++b) pos[b] += 1;
    return ORC_OK;
}

int orc_vanilla_step(const orc_model* m, orc_kv* kv, const int32_t* tok_in, int32_t* pos,
                     const float* scale, int32_t* out_tok, float* out_conf, float* h_out) {
    if (!m || !kv || !tok_in || !pos || !out_tok || !out_conf) return ORC_ERR_ARG;
    const orc_config& c = m->cfg;
    int R = orc_model_resident_depth(m);
    if (R < 1) return ORC_ERR_ARG;
    int head = -1;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] == R) head = e;
    if (head < 0) return ORC_ERR_NOT_RESIDENT;
    int d = c.d_model;
    std::vector<float> h(d);
    for (int b = 0; b < kv->B; ++b) {
        int rc = orc_embed(m, tok_in[b], h.data());
        if (rc != ORC_OK) return rc;
        for (int l = 1; l <= R; ++l) {
            rc = layer_forward_row(m, l, kv, b, pos[b], h.data());
            if (rc != ORC_OK) return rc;
        }
        rc = orc_exit_head(m, head, h.data(), scale ? scale[b] : 1.0f, nullptr, &out_conf[b], &out_tok[b]);
        if (rc != ORC_OK) return rc;
        if (h_out) std::memcpy(h_out + (size_t)b * d, h.data(), sizeof(float) * d);
        pos[b] += 1;
    }
    return ORC_OK;
}

int orc_prefill(const orc_model* m, orc_kv* kv, int b, const int32_t* tok, int n, int32_t pos0,
                float* h_out) {
    if (!m || !kv || !tok || n < 0 || b < 0 || b >= kv->B || pos0 < 0) return ORC_ERR_ARG;
    if (m->rope_theta == 0.0) return ORC_ERR_ARG;
    int R = orc_model_resident_depth(m);
    if (R < 1) return ORC_ERR_ARG;
    if ((int64_t)pos0 + n > kv->cap || (int64_t)pos0 + n > m->max_pos) return ORC_ERR_ARG;
    int d = m->cfg.d_model;
    std::vector<float> H((size_t)n * d);
    for (int t = 0; t < n; ++t) {
        int rc = orc_embed(m, tok[t], &H[(size_t)t * d]);
        if (rc != ORC_OK) return rc;
    }
    // all positions through layer l before any enters layer l + 1; within the layer in
    // rising position order, so the cache holds exactly positions 0 .. pos0+t when
    // position pos0+t attends: that is the causal mask
    for (int l = 1; l <= R; ++l)
        for (int t = 0; t < n; ++t) {
            int rc = layer_forward_row(m, l, kv, b, pos0 + t, &H[(size_t)t * d]);
            if (rc != ORC_OK) return rc;
        }
    if (h_out) std::memcpy(h_out, H.data(), sizeof(float) * H.size());
    return ORC_OK;
}

int orc_accept_drafts(const int32_t* drafts, const int32_t* verified, int k, int32_t* emitted) {
    int a = 0;
    while (a < k && drafts[a] == verified[a]) ++a;
    int n = a + 1 < k ? a + 1 : k;
    for (int j = 0; j < n; ++j) emitted[j] = verified[j];
    return n;
}

// (largest - second largest) / largest magnitude of z[0..V)
static float relative_margin(const float* z, int V) {
    float top = -INFINITY, second = -INFINITY, mag = 0.f;
    for (int j = 0; j < V; ++j) {
        if (z[j] > top) { second = top; top = z[j]; }
        else if (z[j] > second) second = z[j];
        if (std::fabs(z[j]) > mag) mag = std::fabs(z[j]);
    }
    return mag > 0.f ? (top - second) / mag : 0.f;
}

int orc_selfspec_round(const orc_model* m, orc_kv* kv, int b, int32_t tok_in, int32_t* pos, int draft_exit,
                       int k, int32_t* drafts, int32_t* verified, int32_t* n_emitted, int32_t* emitted,
                       float* draft_margin, float* verify_margin) {
    if (!m || !kv || !pos || !drafts || !verified || !n_emitted || !emitted) return ORC_ERR_ARG;
    if (b < 0 || b >= kv->B || k < 1 || m->rope_theta == 0.0) return ORC_ERR_ARG;
    const orc_config& c = m->cfg;
    int R = orc_model_resident_depth(m);
    if (R < 1 || draft_exit < 0 || draft_exit >= c.n_exits) return ORC_ERR_ARG;
    int Le = c.exit_layers[draft_exit];
    int head = -1;
    for (int e = 0; e < c.n_exits; ++e)
        if (c.exit_layers[e] == R) head = e;
    if (head < 0 || Le >= R) return ORC_ERR_NOT_RESIDENT;
    int p0 = *pos, d = c.d_model;
    if ((int64_t)p0 + k > kv->cap || (int64_t)p0 + k > m->max_pos) return ORC_ERR_ARG;
    std::vector<float> S((size_t)k * d);      // state of each drafted position after layer L_e
    std::vector<float> z(c.vocab);
    float conf;
    // 1. draft
    int32_t tok = tok_in;
    for (int j = 0; j < k; ++j) {
        float* h = &S[(size_t)j * d];
        int rc = orc_embed(m, tok, h);
        if (rc != ORC_OK) return rc;
        for (int l = 1; l <= Le; ++l) {
            rc = layer_forward_row(m, l, kv, b, p0 + j, h);
            if (rc != ORC_OK) return rc;
        }
        rc = orc_exit_head(m, draft_exit, h, 1.0f, z.data(), &conf, &drafts[j]);
        if (rc != ORC_OK) return rc;
        if (draft_margin) draft_margin[j] = relative_margin(z.data(), c.vocab);
        tok = drafts[j];
    }
    // 2. verify
    for (int l = Le + 1; l <= R; ++l)
        for (int j = 0; j < k; ++j) {
            int rc = layer_forward_row(m, l, kv, b, p0 + j, &S[(size_t)j * d]);
            if (rc != ORC_OK) return rc;
        }
    for (int j = 0; j < k; ++j) {
        int rc = orc_exit_head(m, head, &S[(size_t)j * d], 1.0f, z.data(), &conf, &verified[j]);
        if (rc != ORC_OK) return rc;
        if (verify_margin) verify_margin[j] = relative_margin(z.data(), c.vocab);
    }
    // 3. accept
    *n_emitted = orc_accept_drafts(drafts, verified, k, emitted);
    *pos = p0 + *n_emitted;
    return ORC_OK;
}

}  // extern "C"
