// ee_kernels_f32.hip -- the decode step for EE_F32 models: plain fp32 kernels
// for any (small) shape.  Nothing is rounded on this path.  These kernels are
// simple LDS-tiled VALU code; the bandwidth- and MFMA-bound work of the large
// bf16 models lives in ee_kernels_bf16.hip.
#include "ee_device.h"

#include <float.h>

// ------------------------------------------------------------------ RMSNorm
// one block per list entry i: out[i] = h[idx[i]] / sqrt(mean(h^2) + eps) * gain
__global__ void __launch_bounds__(256)
k_f32_rmsnorm(const float* __restrict__ h, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_ptr,
              int B, const float* __restrict__ gain, float eps, int d, float* __restrict__ out) {
    __shared__ float red[4];
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    const float* hr = h + (int64_t)idx[i] * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) ss += hr[c] * hr[c];
    ss = block_sum<256>(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) out[(int64_t)i * d + c] = (hr[c] * inv) * gain[c];
}

// ------------------------------------------------------------------ GEMM
// out[i][j] = sum_k X[i][k] * W[j][k] for list entries i < n; 16x16 tile per block
enum { F32_EPI_STORE = 0, F32_EPI_RESID = 1, F32_EPI_SCALE = 2 };

template <int EPI>
__global__ void __launch_bounds__(256)
k_f32_gemm(const float* __restrict__ X, int ldx, const float* __restrict__ W, int N, int K,
           const int32_t* __restrict__ n_ptr, int B, float* __restrict__ out, int ldo,
           const int32_t* __restrict__ idx, const float* __restrict__ row_scale) {
    __shared__ float xs[16][17];
    __shared__ float ws[16][17];
    int n = min(*n_ptr, B);
    int row0 = blockIdx.y * 16;
    if (row0 >= n) return;
    int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    int row = row0 + ty, col = blockIdx.x * 16 + tx;
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        int kx = k0 + tx;
        xs[ty][tx] = (row < n && kx < K) ? X[(int64_t)row * ldx + kx] : 0.f;
        int wrow = blockIdx.x * 16 + ty;
        ws[ty][tx] = (wrow < N && kx < K) ? W[(int64_t)wrow * K + kx] : 0.f;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) acc += xs[ty][k] * ws[tx][k];
        __syncthreads();
    }
    if (row >= n || col >= N) return;
    if (EPI == F32_EPI_STORE) {
        out[(int64_t)row * ldo + col] = acc;
    } else if (EPI == F32_EPI_RESID) {
        out[(int64_t)idx[row] * ldo + col] += acc;
    } else {
        out[(int64_t)row * ldo + col] = acc * row_scale[idx[row]];
    }
}

// ------------------------------------------------------------------ RoPE + cache append
// buf[i] holds [q (n_q*hd, may be empty) | k (Hkv*hd) | v (Hkv*hd)] of list entry i.
// Rotates q in place and k on its way into the cache, at the row's position.
__global__ void __launch_bounds__(256)
k_f32_rope_append(float* __restrict__ buf, int ld, int n_q, const int32_t* __restrict__ idx,
                  const int32_t* __restrict__ n_ptr, int B, const int32_t* __restrict__ pos,
                  const float* __restrict__ rope, int max_pos, KvView kv, int32_t* __restrict__ status) {
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    int b = idx[i];
    int p = pos[b];
    int hd = kv.head_dim, half = hd >> 1, Hkv = kv.n_kv_heads;
    const int sq = kv_row(kv, b);
    int cap = kv.cap[sq];
    bool ok = p >= 0 && p < cap && p < max_pos;
    if (!ok) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        return;
    }
    float* r = buf + (int64_t)i * ld;
    const float* cs = rope + (int64_t)p * half * 2;
    for (int t = threadIdx.x; t < n_q * half; t += 256) {
        int hh = t / half, j = t % half;
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = r[hh * hd + j], bb = r[hh * hd + j + half];
        r[hh * hd + j] = a * c - bb * s;
        r[hh * hd + j + half] = bb * c + a * s;
    }
    float* kin = r + n_q * hd;
    float* vin = kin + Hkv * hd;
    for (int t = threadIdx.x; t < Hkv * half; t += 256) {
        int g = t / half, j = t % half;
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = kin[g * hd + j], bb = kin[g * hd + j + half];
        float* base = reinterpret_cast<float*>(kv.pool) + kv_block(kv, sq, g, cap);
        base[(int64_t)p * hd + j] = a * c - bb * s;
        base[(int64_t)p * hd + j + half] = bb * c + a * s;
    }
    for (int t = threadIdx.x; t < Hkv * hd; t += 256) {
        int g = t / hd, j = t % hd;
        float* base = reinterpret_cast<float*>(kv.pool) + kv_block(kv, sq, g, cap);
        base[(int64_t)cap * hd + (int64_t)p * hd + j] = vin[g * hd + j];
    }
}

// ------------------------------------------------------------------ attention
// one block per (query head, list entry): softmax(q.K^T / sqrt(hd)) V over positions 0..pos
__global__ void __launch_bounds__(256)
k_f32_attn(const float* __restrict__ qkv, int ld, int Hq, const int32_t* __restrict__ idx,
           const int32_t* __restrict__ n_ptr, int B, const int32_t* __restrict__ pos, KvView kv,
           float* __restrict__ out /* [i][Hq*hd] */) {
    extern __shared__ float sm[];   // q[hd] | scores[n_pos]
    __shared__ float red[4];
    int hq = blockIdx.x, i = blockIdx.y;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    int b = idx[i];
    int hd = kv.head_dim;
    const int sq = kv_row(kv, b);
    int cap = kv.cap[sq];
    int n_pos = min(pos[b] + 1, cap);
    int g = hq / (Hq / kv.n_kv_heads);
    const float* Kb = reinterpret_cast<const float*>(kv.pool) + kv_block(kv, sq, g, cap);
    const float* Vb = Kb + (int64_t)cap * hd;
    float* q = sm;
    float* sc = sm + hd;
    for (int t = threadIdx.x; t < hd; t += 256) q[t] = qkv[(int64_t)i * ld + hq * hd + t];
    __syncthreads();
    float inv_sqrt = 1.0f / sqrtf((float)hd);
    float mx = -FLT_MAX;
    for (int t = threadIdx.x; t < n_pos; t += 256) {
        float a = 0.f;
        for (int j = 0; j < hd; ++j) a += q[j] * Kb[(int64_t)t * hd + j];
        a *= inv_sqrt;
        sc[t] = a;
        mx = fmaxf(mx, a);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.f;
    for (int t = threadIdx.x; t < n_pos; t += 256) {
        float p = expf(sc[t] - mx);
        sc[t] = p;
        sum += p;
    }
    sum = block_sum<256>(sum, red);   // also makes sc[] visible to all threads
    for (int j = threadIdx.x; j < hd; j += 256) {
        float acc = 0.f;
        for (int t = 0; t < n_pos; ++t) acc += sc[t] * Vb[(int64_t)t * hd + j];
        out[(int64_t)i * (Hq * hd) + hq * hd + j] = acc / sum;
    }
}

// ------------------------------------------------------------------ SwiGLU
__global__ void k_f32_swiglu(const float* __restrict__ gu, int F, const int32_t* __restrict__ n_ptr, int B,
                             float* __restrict__ act) {
    int n = min(*n_ptr, B);
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)n * F) return;
    int i = (int)(t / F), j = (int)(t % F);
    float gt = gu[(int64_t)i * 2 * F + j], up = gu[(int64_t)i * 2 * F + F + j];
    act[t] = (gt / (1.0f + expf(-gt))) * up;
}

// ------------------------------------------------------------------ logits -> row statistics
__global__ void __launch_bounds__(256)
k_f32_row_stats(const float* __restrict__ logits, int V, const int32_t* __restrict__ n_ptr, int B,
                float* __restrict__ part_max, float* __restrict__ part_sum, int32_t* __restrict__ part_arg) {
    __shared__ Stat sw[4];
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    Stat st{-FLT_MAX, 0.f, 0x7fffffff};
    for (int j = threadIdx.x; j < V; j += 256) st = stat_merge(st, Stat{logits[(int64_t)i * V + j], 1.0f, j});
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Stat y{__shfl_xor(st.m, o, 64), __shfl_xor(st.s, o, 64), __shfl_xor(st.a, o, 64)};
        st = stat_merge(st, y);
    }
    if ((threadIdx.x & 63) == 0) sw[threadIdx.x >> 6] = st;
    __syncthreads();
    if (threadIdx.x == 0) {
        Stat r = sw[0];
        for (int w = 1; w < 4; ++w) r = stat_merge(r, sw[w]);
        part_max[i] = r.m; part_sum[i] = r.s; part_arg[i] = r.a;
    }
}

// ------------------------------------------------------------------ host side
static KvView make_view(const ee_model* m, const ee_kv* kv, int layer, const ee_batch* b) {
    return KvView{kv->pool, kv->d_cap, kv->d_off, kv->T, m->cfg.n_kv_heads, m->cfg.head_dim, layer - 1, b->kv_seq};
}

template <int EPI>
static void gemm(const float* X, int ldx, const float* W, int N, int K, const int32_t* n_ptr, int B,
                 float* out, int ldo, const int32_t* idx, const float* scale, hipStream_t s) {
    dim3 grid((N + 15) / 16, (B + 15) / 16);
    hipLaunchKernelGGL((k_f32_gemm<EPI>), grid, dim3(256), 0, s, X, ldx, W, N, K, n_ptr, B, out, ldo, idx, scale);
}

int f32_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_layer_weights& w = m->layers[layer - 1];
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, hd = c.head_dim, qd = c.n_q_heads * hd, F = c.d_ffn;
    int qkv_n = (c.n_q_heads + 2 * c.n_kv_heads) * hd;
    const int32_t* idx = b->st<int32_t>(L.active_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_active);
    float* h = b->st<float>(L.h);
    float* x = b->wsp<float>(b->W.x);
    float* qkv = b->wsp<float>(b->W.qkv);
    float* ao = b->wsp<float>(b->W.ao);
    float* act = b->wsp<float>(b->W.act);
    float* gu = b->wsp<float>(b->W.logits);   // [B][2F] fits: checked when the workspace is laid out
    KvView view = make_view(m, kv, layer, b);

    hipLaunchKernelGGL(k_f32_rmsnorm, dim3(B), dim3(256), 0, s, h, idx, n_ptr, B, w.g_attn, c.rms_eps, d, x);
    gemm<F32_EPI_STORE>(x, d, (const float*)w.w_qkv, qkv_n, d, n_ptr, B, qkv, qkv_n, idx, nullptr, s);
    hipLaunchKernelGGL(k_f32_rope_append, dim3(B), dim3(256), 0, s, qkv, qkv_n, c.n_q_heads, idx, n_ptr, B,
                       b->st<int32_t>(L.pos), m->d_rope, c.max_pos, view, b->st<int32_t>(L.status));
    size_t smem = (size_t)(hd + c.max_pos) * sizeof(float);
    hipLaunchKernelGGL(k_f32_attn, dim3(c.n_q_heads, B), dim3(256), smem, s, qkv, qkv_n, c.n_q_heads, idx, n_ptr,
                       B, b->st<int32_t>(L.pos), view, ao);
    gemm<F32_EPI_RESID>(ao, qd, (const float*)w.w_o, d, qd, n_ptr, B, h, d, idx, nullptr, s);
    hipLaunchKernelGGL(k_f32_rmsnorm, dim3(B), dim3(256), 0, s, h, idx, n_ptr, B, w.g_ffn, c.rms_eps, d, x);
    gemm<F32_EPI_STORE>(x, d, (const float*)w.w_gate_up, 2 * F, d, n_ptr, B, gu, 2 * F, idx, nullptr, s);
    int64_t tot = (int64_t)B * F;
    hipLaunchKernelGGL(k_f32_swiglu, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, gu, F, n_ptr, B, act);
    gemm<F32_EPI_RESID>(act, F, (const float*)w.w_down, d, F, n_ptr, B, h, d, idx, nullptr, s);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

int f32_exit_head(const ee_model* m, int e, float th, int force, ee_batch* b, float* dbg, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, V = c.vocab;
    const int32_t* idx = b->st<int32_t>(L.active_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_active);
    float* x = b->wsp<float>(b->W.x);
    float* logits = dbg ? dbg : b->wsp<float>(b->W.logits);
    hipLaunchKernelGGL(k_f32_rmsnorm, dim3(B), dim3(256), 0, s, b->st<float>(L.h), idx, n_ptr, B,
                       m->exits[e].gain, c.rms_eps, d, x);
    gemm<F32_EPI_SCALE>(x, d, (const float*)m->exits[e].w, V, d, n_ptr, B, logits, V, idx,
                        b->st<float>(L.row_scale), s);
    hipLaunchKernelGGL(k_f32_row_stats, dim3(B), dim3(256), 0, s, logits, V, n_ptr, B,
                       b->wsp<float>(b->W.part_max), b->wsp<float>(b->W.part_sum), b->wsp<int32_t>(b->W.part_arg));
    EE_LAUNCH_CHECK();
    return launch_exit_decide(b, 1, th, force, s);
}

int f32_fill_kv(const ee_model* m, int from_excl, int to_incl, ee_kv* kv, ee_batch* b, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, hd = c.head_dim;
    int kv_n = 2 * c.n_kv_heads * hd;
    const int32_t* idx = b->st<int32_t>(L.exited_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_exited);
    float* x = b->wsp<float>(b->W.fill_x);
    float* kvb = b->wsp<float>(b->W.fill_kv);
    for (int l = from_excl + 1; l <= to_incl; ++l) {
        const ee_layer_weights& w = m->layers[l - 1];
        hipLaunchKernelGGL(k_f32_rmsnorm, dim3(B), dim3(256), 0, s, b->st<float>(L.h), idx, n_ptr, B, w.g_attn,
                           c.rms_eps, d, x);
        const float* Wkv = (const float*)w.w_qkv + (int64_t)c.n_q_heads * hd * d;
        gemm<F32_EPI_STORE>(x, d, Wkv, kv_n, d, n_ptr, B, kvb, kv_n, idx, nullptr, s);
        hipLaunchKernelGGL(k_f32_rope_append, dim3(B), dim3(256), 0, s, kvb, kv_n, 0, idx, n_ptr, B,
                           b->st<int32_t>(L.pos), m->d_rope, c.max_pos, make_view(m, kv, l, b),
                           b->st<int32_t>(L.status));
    }
    EE_LAUNCH_CHECK();
    return EE_OK;
}
