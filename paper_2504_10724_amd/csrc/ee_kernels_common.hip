// ee_kernels_common.hip -- kernels of the early-exit decode step that do not
// depend on the weight format: step begin/end, exit decision, order-preserving
// compaction, weight repacking, key/value pool import/export, rotary table.
#include "ee_device.h"

#include <float.h>

// ------------------------------------------------------------------ rotary table
// table[pos][i] = (cos, sin)(pos * theta^(-2i/hd)), evaluated in fp64, stored fp32
__global__ void k_rope_table(float* __restrict__ table, int max_pos, int half, int hd, double theta) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)max_pos * half) return;
    int pos = (int)(idx / half), i = (int)(idx % half);
    double angle = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
    table[2 * idx]     = (float)cos(angle);
    table[2 * idx + 1] = (float)sin(angle);
}

int launch_rope_table(float* d_table, int max_pos, int hd, double theta, hipStream_t s) {
    int64_t n = (int64_t)max_pos * (hd / 2);
    hipLaunchKernelGGL(k_rope_table, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d_table, max_pos,
                       hd / 2, hd, theta);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ step begin / end
// One block per row: every row becomes active again and its residual stream is
// the embedding of its input token.
__global__ void __launch_bounds__(256)
k_begin_step(const int32_t* __restrict__ tok_in, const void* __restrict__ emb, int is_bf16, int d, int V,
             float* __restrict__ h, int32_t* __restrict__ active_idx, int32_t* __restrict__ n_active,
             int32_t* __restrict__ n_exited, int32_t* __restrict__ out_layer, int32_t* __restrict__ status, int B) {
    int b = blockIdx.x;
    int tok = tok_in[b];
    if (tok < 0 || tok >= V) {
        if (threadIdx.x == 0) atomicOr(status, 2);
        tok = 0;
    }
    if (threadIdx.x == 0) {
        active_idx[b] = b;
        out_layer[b] = 0;
        if (b == 0) { *n_active = B; *n_exited = 0; }
    }
    float* hr = h + (int64_t)b * d;
    if (is_bf16) {
        const bf16_t* e = (const bf16_t*)emb + (int64_t)tok * d;
        for (int i = threadIdx.x; i < d; i += blockDim.x) hr[i] = bf16_to_f32(e[i]);
    } else {
        const float* e = (const float*)emb + (int64_t)tok * d;
        for (int i = threadIdx.x; i < d; i += blockDim.x) hr[i] = e[i];
    }
}

int launch_begin_step(const ee_model* m, ee_batch* b, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    TimedScope t(EE_K_EMBED, s);
    hipLaunchKernelGGL(k_begin_step, dim3(b->B), dim3(256), 0, s, b->st<int32_t>(L.tok_in), m->emb,
                       m->cfg.dtype == EE_BF16 ? 1 : 0, m->cfg.d_model, m->cfg.vocab, b->st<float>(L.h),
                       b->st<int32_t>(L.active_idx), b->st<int32_t>(L.n_active), b->st<int32_t>(L.n_exited),
                       b->st<int32_t>(L.out_layer), b->st<int32_t>(L.status), b->B);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// Context pass: entry i < n is token tok[i] at position pos[i] of cache row seq[i].  It becomes
// batch row i: active, its residual stream the token's embedding.  An entry whose cache row
// does not exist gets position -1, which the append kernel refuses (status bit 1), and cache
// row 0, so that every later address stays inside the pool.
__global__ void __launch_bounds__(256)
k_prefill_begin(const int32_t* __restrict__ tok, const int32_t* __restrict__ pos, const int32_t* __restrict__ seq,
                int n, int n_seq, const void* __restrict__ emb, int is_bf16, int d, int V, float* __restrict__ h,
                int32_t* __restrict__ s_tok, int32_t* __restrict__ s_pos, int32_t* __restrict__ kv_seq,
                int32_t* __restrict__ active_idx, int32_t* __restrict__ n_active, int32_t* __restrict__ n_exited,
                int32_t* __restrict__ status) {
    int i = blockIdx.x;
    if (i >= n) return;
    int t = tok[i], p = pos[i], sq = seq[i];
    if (t < 0 || t >= V) {
        if (threadIdx.x == 0) atomicOr(status, 2);
        t = 0;
    }
    if (sq < 0 || sq >= n_seq) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        sq = 0;
        p = -1;
    }
    if (threadIdx.x == 0) {
        s_tok[i] = t;
        s_pos[i] = p;
        kv_seq[i] = sq;
        active_idx[i] = i;
        if (i == 0) { *n_active = n; *n_exited = 0; }
    }
    float* hr = h + (int64_t)i * d;
    if (is_bf16) {
        const bf16_t* e = (const bf16_t*)emb + (int64_t)t * d;
        for (int j = threadIdx.x; j < d; j += blockDim.x) hr[j] = bf16_to_f32(e[j]);
    } else {
        const float* e = (const float*)emb + (int64_t)t * d;
        for (int j = threadIdx.x; j < d; j += blockDim.x) hr[j] = e[j];
    }
}

int launch_prefill_begin(const ee_model* m, const ee_kv* kv, ee_batch* b, const int32_t* tok, const int32_t* pos,
                         const int32_t* seq, int n, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    TimedScope t(EE_K_EMBED, s);
    hipLaunchKernelGGL(k_prefill_begin, dim3(n), dim3(256), 0, s, tok, pos, seq, n, kv->B, m->emb,
                       m->cfg.dtype == EE_BF16 ? 1 : 0, m->cfg.d_model, m->cfg.vocab, b->st<float>(L.h),
                       b->st<int32_t>(L.tok_in), b->st<int32_t>(L.pos), b->wsp<int32_t>(b->W.kv_seq),
                       b->st<int32_t>(L.active_idx), b->st<int32_t>(L.n_active), b->st<int32_t>(L.n_exited),
                       b->st<int32_t>(L.status));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ loading more layers while serving
__global__ void k_set_layer_ptrs(const void** wqkv_tab, const float** gattn_tab, int at, const void* w_qkv,
                                 const float* g_attn) {
    if (threadIdx.x == 0) { wqkv_tab[at] = w_qkv; gattn_tab[at] = g_attn; }
}

int launch_set_layer_ptrs(ee_model* m, int layer, const void* w_qkv, const float* g_attn, hipStream_t s) {
    hipLaunchKernelGGL(k_set_layer_ptrs, dim3(1), dim3(64), 0, s, m->d_wqkv_tab, m->d_gattn_tab, layer - 1, w_qkv, g_attn);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// store[(positions of cache rows before r) + p][:] = h[i][:].  After a decode step (seq == null):
// batch row i is cache row i and p = pos[i] + delta with delta = -1; after a context pass: entry i
// is cache row seq[i] at p = pos[i].
__global__ void __launch_bounds__(256)
k_hstore_put(const float* __restrict__ h, int d, int n, const int32_t* __restrict__ pos, int delta,
             const int32_t* __restrict__ seq, int n_seq, const int64_t* __restrict__ off,
             const int32_t* __restrict__ cap, float* __restrict__ store, int32_t* __restrict__ status) {
    int i = blockIdx.x;
    if (i >= n) return;
    int sq = seq ? seq[i] : i;
    int p = pos[i] + delta;
    if (sq < 0 || sq >= n_seq || p < 0 || p >= cap[sq]) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        return;
    }
    const float4* src = reinterpret_cast<const float4*>(h + (int64_t)i * d);
    float4* dst = reinterpret_cast<float4*>(store + (off[sq] + p) * (int64_t)d);
    for (int j = threadIdx.x; j < d / 4; j += 256) dst[j] = src[j];
}

int launch_hstore_put(const ee_model* m, const ee_kv* kv, const ee_batch* b, int n, bool entries, float* store,
                      hipStream_t s) {
    const ee_batch_layout& L = b->L;
    hipLaunchKernelGGL(k_hstore_put, dim3(n), dim3(256), 0, s, b->st<float>(L.h), m->cfg.d_model, n,
                       b->st<int32_t>(L.pos), entries ? 0 : -1, entries ? b->wsp<int32_t>(b->W.kv_seq) : (const int32_t*)nullptr,
                       kv->B, kv->d_off, kv->d_cap, store, b->st<int32_t>(L.status));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// Entry i < n = position pos[i] of cache row seq[i]: it becomes batch row i of the list of rows that
// left (the list the skipped-layer fill works on), with its stored state as h.  An entry that names
// no cache row or a position outside the capacity gets position -1 (refused by the append kernel,
// status bit 1) and cache row 0, so that every later address stays inside the pool and the store.
__global__ void __launch_bounds__(256)
k_backfill_begin(const float* __restrict__ store, int d, int n, const int32_t* __restrict__ pos,
                 const int32_t* __restrict__ seq, int n_seq, const int64_t* __restrict__ off,
                 const int32_t* __restrict__ cap, float* __restrict__ h, int32_t* __restrict__ s_pos,
                 int32_t* __restrict__ kv_seq, int32_t* __restrict__ exited_idx, int32_t* __restrict__ n_exited,
                 int32_t* __restrict__ status) {
    int i = blockIdx.x;
    if (i >= n) return;
    int sq = seq[i], p = pos[i];
    bool ok = sq >= 0 && sq < n_seq && p >= 0 && p < cap[sq];
    if (!ok) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        sq = 0;
        p = -1;
    }
    if (threadIdx.x == 0) {
        s_pos[i] = p;
        kv_seq[i] = sq;
        exited_idx[i] = i;
        if (i == 0) *n_exited = n;
    }
    float4* dst = reinterpret_cast<float4*>(h + (int64_t)i * d);
    if (ok) {
        const float4* src = reinterpret_cast<const float4*>(store + (off[sq] + p) * (int64_t)d);
        for (int j = threadIdx.x; j < d / 4; j += 256) dst[j] = src[j];
    } else {
        for (int j = threadIdx.x; j < d / 4; j += 256) dst[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

int launch_backfill_begin(const ee_model* m, const ee_kv* kv, ee_batch* b, const float* store, const int32_t* pos,
                          const int32_t* seq, int n, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    hipLaunchKernelGGL(k_backfill_begin, dim3(n), dim3(256), 0, s, store, m->cfg.d_model, n, pos, seq, kv->B, kv->d_off,
                       kv->d_cap, b->st<float>(L.h), b->st<int32_t>(L.pos), b->wsp<int32_t>(b->W.kv_seq),
                       b->st<int32_t>(L.exited_idx), b->st<int32_t>(L.n_exited), b->st<int32_t>(L.status));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ self-speculative decoding
// Verification pass: entry i = r * k + j (row r < n_rows, draft position j < k) becomes row i of the
// entries batch: cache row r, position pos[r] - k + j (pos[r] = the decode batch's position after its
// k draft steps), residual stream = the state kept for that position after the draft layers.  An entry
// whose position lies outside its cache row gets position -1 (refused by the append kernel, status bit 1).
__global__ void __launch_bounds__(256)
k_verify_begin(const float* __restrict__ store, int d, int n_rows, int k, const int32_t* __restrict__ pos,
               const int64_t* __restrict__ off, const int32_t* __restrict__ cap, float* __restrict__ h,
               int32_t* __restrict__ e_pos, int32_t* __restrict__ kv_seq, int32_t* __restrict__ active_idx,
               int32_t* __restrict__ n_active, int32_t* __restrict__ n_exited, float* __restrict__ row_scale,
               int32_t* __restrict__ status) {
    const int i = blockIdx.x;
    if (i >= n_rows * k) return;
    const int r = i / k, j = i % k;
    int p = pos[r] - k + j;
    const bool ok = p >= 0 && p < cap[r];
    if (!ok) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        p = -1;
    }
    if (threadIdx.x == 0) {
        e_pos[i] = p;
        kv_seq[i] = r;
        active_idx[i] = i;
        row_scale[i] = 1.0f;
        if (i == 0) { *n_active = n_rows * k; *n_exited = 0; }
    }
    float4* dst = reinterpret_cast<float4*>(h + (int64_t)i * d);
    if (ok) {
        const float4* src = reinterpret_cast<const float4*>(store + (off[r] + p) * (int64_t)d);
        for (int c = threadIdx.x; c < d / 4; c += 256) dst[c] = src[c];
    } else {
        for (int c = threadIdx.x; c < d / 4; c += 256) dst[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

int launch_verify_begin(const ee_model* m, const ee_kv* kv, const ee_batch* b, ee_batch* vb, int k, const float* store,
                        hipStream_t s) {
    const ee_batch_layout& L = vb->L;
    hipLaunchKernelGGL(k_verify_begin, dim3(b->B * k), dim3(256), 0, s, store, m->cfg.d_model, b->B, k,
                       b->st<int32_t>(b->L.pos), kv->d_off, kv->d_cap, vb->st<float>(L.h), vb->st<int32_t>(L.pos),
                       vb->wsp<int32_t>(vb->W.kv_seq), vb->st<int32_t>(L.active_idx), vb->st<int32_t>(L.n_active),
                       vb->st<int32_t>(L.n_exited), vb->st<float>(L.row_scale), vb->st<int32_t>(L.status));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// Acceptance, one thread per row: drafts d_j = drafts[j * n_rows + r] against the full-depth tokens
// v_j = head_tok[r * k + j] of the same positions; with a = number of leading positions where they
// agree, the row emits n = min(a + 1, k) tokens v_0 .. v_{n-1}, its position becomes its position
// before the drafts + n and its next input token v_{n-1}.
__global__ void k_accept_drafts(const int32_t* __restrict__ drafts, const int32_t* __restrict__ head_tok, int k,
                                int n_rows, int32_t* __restrict__ pos, int32_t* __restrict__ tok_in,
                                int32_t* __restrict__ out_tok, int32_t* __restrict__ n_emit,
                                int32_t* __restrict__ emit) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    int a = 0;
    while (a < k && drafts[(int64_t)a * n_rows + r] == head_tok[(int64_t)r * k + a]) ++a;
    const int n = a + 1 < k ? a + 1 : k;
    for (int j = 0; j < k; ++j) emit[(int64_t)r * k + j] = j < n ? head_tok[(int64_t)r * k + j] : -1;
    const int last = head_tok[(int64_t)r * k + n - 1];
    n_emit[r] = n;
    pos[r] = pos[r] - k + n;
    tok_in[r] = last;
    out_tok[r] = last;
}

int launch_accept_drafts(ee_batch* b, const ee_batch* vb, int k, const int32_t* drafts, int32_t* n_emit, int32_t* emit,
                         hipStream_t s) {
    hipLaunchKernelGGL(k_accept_drafts, dim3((b->B + 255) / 256), dim3(256), 0, s, drafts, vb->st<int32_t>(vb->L.head_tok),
                       k, b->B, b->st<int32_t>(b->L.pos), b->st<int32_t>(b->L.tok_in), b->st<int32_t>(b->L.out_tok),
                       n_emit, emit);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// every row advances one position, whatever layer it left at, and the token it
// emitted is the input of the next step
__global__ void k_end_step(int32_t* __restrict__ pos, int32_t* __restrict__ tok_in,
                           const int32_t* __restrict__ out_tok, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    pos[b] += 1;
    tok_in[b] = out_tok[b];
}

int launch_end_step(ee_batch* b, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    hipLaunchKernelGGL(k_end_step, dim3((b->B + 255) / 256), dim3(256), 0, s, b->st<int32_t>(L.pos),
                       b->st<int32_t>(L.tok_in), b->st<int32_t>(L.out_tok), b->B);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

__global__ void k_reset(const int32_t* __restrict__ tok, const int32_t* __restrict__ pos,
                        const float* __restrict__ scale, int B, int32_t* s_tok, int32_t* s_pos, float* s_scale,
                        int32_t* active_idx, int32_t* n_active, int32_t* n_exited, int32_t* out_tok,
                        int32_t* out_layer, float* out_conf, uint8_t* out_breach, int32_t* exit_counts,
                        int32_t* breach_count, int32_t* status) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) {
        s_tok[b] = tok[b];
        s_pos[b] = pos[b];
        s_scale[b] = scale ? scale[b] : 1.0f;
        active_idx[b] = b;
        out_tok[b] = -1;
        out_layer[b] = 0;
        out_conf[b] = 0.f;
        out_breach[b] = 0;
    }
    if (b < EE_MAX_EXITS) exit_counts[b] = 0;
    if (b == 0) { *n_active = B; *n_exited = 0; *breach_count = 0; *status = 0; }
}

int launch_reset(ee_batch* b, const int32_t* tok, const int32_t* pos, const float* scale, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    int n = b->B > EE_MAX_EXITS ? b->B : EE_MAX_EXITS;
    hipLaunchKernelGGL(k_reset, dim3((n + 255) / 256), dim3(256), 0, s, tok, pos, scale, b->B,
                       b->st<int32_t>(L.tok_in), b->st<int32_t>(L.pos), b->st<float>(L.row_scale),
                       b->st<int32_t>(L.active_idx), b->st<int32_t>(L.n_active), b->st<int32_t>(L.n_exited),
                       b->st<int32_t>(L.out_tok), b->st<int32_t>(L.out_layer), b->st<float>(L.out_conf),
                       b->st<uint8_t>(L.out_breach), b->st<int32_t>(L.exit_counts),
                       b->st<int32_t>(L.breach_count), b->st<int32_t>(L.status));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

__global__ void k_set_scale(const float* __restrict__ scale, float* __restrict__ s_scale, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) s_scale[b] = scale[b];
}

int launch_set_scale(ee_batch* b, const float* scale, hipStream_t s) {
    hipLaunchKernelGGL(k_set_scale, dim3((b->B + 255) / 256), dim3(256), 0, s, scale,
                       b->st<float>(b->L.row_scale), b->B);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ compaction
// Order-preserving split of the active list by head_exit.  One workgroup; each
// wave turns its 64 flags into a ballot mask, a lane's rank among the kept (or
// leaving) rows of its wave is the population count of the mask below the
// lane, and the wave totals are combined through LDS.  Lists longer than the
// workgroup are processed in consecutive chunks with running offsets.
#define COMPACT_THREADS 512
__global__ void __launch_bounds__(COMPACT_THREADS)
k_compact(int32_t* __restrict__ active_idx, int32_t* __restrict__ n_active, int32_t* __restrict__ exited_idx,
          int32_t* __restrict__ n_exited, const float* __restrict__ head_conf,
          const int32_t* __restrict__ head_tok, const uint8_t* __restrict__ head_exit,
          const uint8_t* __restrict__ head_breach, int32_t* __restrict__ out_tok,
          int32_t* __restrict__ out_layer, float* __restrict__ out_conf, uint8_t* __restrict__ out_breach,
          int32_t* __restrict__ exit_counts, int32_t* __restrict__ breach_count, int exit_idx, int exit_layer,
          int B, int32_t* __restrict__ gone_idx, int32_t* __restrict__ n_gone) {
    __shared__ int s_keep[COMPACT_THREADS / 64];
    __shared__ int s_gone[COMPACT_THREADS / 64];
    __shared__ int s_brch[COMPACT_THREADS / 64];
    int n = *n_active;
    if (n > B) n = B;
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int keep_base = 0, gone_base = 0, breaches = 0;
    // gone_idx collects the leavers of all exits of a step (the first exit starts it again); the
    // bounds hold whatever order the compactions are called in
    const int all_base = exit_idx == 0 ? 0 : max(0, min(*n_gone, B));
    for (int base = 0; base < n; base += COMPACT_THREADS) {
        int i = base + threadIdx.x;
        bool valid = i < n;
        int row = valid ? active_idx[i] : 0;
        bool leaves = valid && head_exit[i] != 0;
        bool stays = valid && !leaves;
        bool br = leaves && head_breach[i] != 0;
        unsigned long long mk = __ballot(stays), mg = __ballot(leaves), mb = __ballot(br);
        unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        int rk = __popcll(mk & below), rg = __popcll(mg & below);
        if (lane == 0) { s_keep[w] = __popcll(mk); s_gone[w] = __popcll(mg); s_brch[w] = __popcll(mb); }
        __syncthreads();   // all reads of active_idx[base ..] are done, wave totals visible
        int ko = keep_base, go = gone_base, tk = 0, tg = 0, tb = 0;
        for (int j = 0; j < COMPACT_THREADS / 64; ++j) {
            if (j < w) { ko += s_keep[j]; go += s_gone[j]; }
            tk += s_keep[j]; tg += s_gone[j]; tb += s_brch[j];
        }
        if (stays) active_idx[ko + rk] = row;          // ko + rk <= i: never overtakes a later read
        if (leaves) {
            exited_idx[go + rg] = row;
            if (all_base + go + rg < B) gone_idx[all_base + go + rg] = row;
            out_tok[row] = head_tok[i];
            out_layer[row] = exit_layer;
            out_conf[row] = head_conf[i];
            out_breach[row] = br ? 1 : 0;
        }
        keep_base += tk; gone_base += tg; breaches += tb;
        __syncthreads();   // wave totals are consumed before the next chunk overwrites them
    }
    if (threadIdx.x == 0) {
        *n_active = keep_base;
        *n_exited = gone_base;
        *n_gone = min(all_base + gone_base, B);
        exit_counts[exit_idx] += gone_base;
        *breach_count += breaches;
    }
}

int launch_compact(ee_batch* b, int exit_idx, int exit_layer, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    TimedScope t(EE_K_COMPACT, s);
    hipLaunchKernelGGL(k_compact, dim3(1), dim3(COMPACT_THREADS), 0, s, b->st<int32_t>(L.active_idx),
                       b->st<int32_t>(L.n_active), b->st<int32_t>(L.exited_idx), b->st<int32_t>(L.n_exited),
                       b->st<float>(L.head_conf), b->st<int32_t>(L.head_tok), b->st<uint8_t>(L.head_exit),
                       b->st<uint8_t>(L.head_breach), b->st<int32_t>(L.out_tok), b->st<int32_t>(L.out_layer),
                       b->st<float>(L.out_conf), b->st<uint8_t>(L.out_breach), b->st<int32_t>(L.exit_counts),
                       b->st<int32_t>(L.breach_count), exit_idx, exit_layer, b->B, b->wsp<int32_t>(b->W.gone_idx),
                       b->wsp<int32_t>(b->W.n_gone));
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ confidence-breach counter
// One wave.  The ring of breach bits and the incoming flags are staged in LDS; lane 0 then takes
// the tokens one by one, exactly as the rule is stated (the work is a few hundred tokens per
// decode step: the sequential loop costs microseconds once per step).
__global__ void k_cbc_init(ee_cbc_state* st, int window, int cbc_max) {
    uint8_t* ring = reinterpret_cast<uint8_t*>(st + 1);
    for (int j = threadIdx.x; j < window; j += blockDim.x) ring[j] = 0;
    for (int j = threadIdx.x; j < EE_CBC_LOG; j += blockDim.x) st->trigger_at[j] = 0;
    if (threadIdx.x == 0) {
        st->window = window; st->cbc_max = cbc_max;
        st->head = 0; st->filled = 0; st->count = 0; st->n_triggers = 0; st->tokens_seen = 0;
    }
}

#define CBC_CHUNK 1024
__global__ void __launch_bounds__(64)
k_cbc_push(ee_cbc_state* st, const uint8_t* __restrict__ flags, int n) {
    __shared__ uint8_t s_ring[EE_CBC_MAX_WINDOW];
    __shared__ uint8_t s_flag[CBC_CHUNK];
    uint8_t* ring = reinterpret_cast<uint8_t*>(st + 1);
    const int window = min(max(st->window, 1), EE_CBC_MAX_WINDOW);
    const int cbc_max = st->cbc_max;
    for (int j = threadIdx.x; j < window; j += 64) s_ring[j] = ring[j];
    int head = st->head, filled = st->filled, count = st->count, n_trig = st->n_triggers;
    int64_t seen = st->tokens_seen;
    for (int base = 0; base < n; base += CBC_CHUNK) {
        const int m = min(CBC_CHUNK, n - base);
        __syncthreads();                                  // the previous chunk has been consumed
        for (int j = threadIdx.x; j < m; j += 64) s_flag[j] = flags[base + j] ? 1 : 0;
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int j = 0; j < m; ++j) {
                const int f = s_flag[j];
                ++seen;
                if (filled == window) count -= s_ring[head];   // the oldest token leaves the window
                else ++filled;
                s_ring[head] = (uint8_t)f;
                count += f;
                head = head + 1 == window ? 0 : head + 1;
                if (count > cbc_max) {                         // re-assessment: the window starts empty
                    if (n_trig < EE_CBC_LOG) st->trigger_at[n_trig] = seen;
                    ++n_trig;
                    head = 0; filled = 0; count = 0;
                }
            }
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < window; j += 64) ring[j] = s_ring[j];
    if (threadIdx.x == 0) {
        st->head = head; st->filled = filled; st->count = count; st->n_triggers = n_trig; st->tokens_seen = seen;
    }
}

int launch_cbc_init(void* st, int window, int cbc_max, hipStream_t s) {
    hipLaunchKernelGGL(k_cbc_init, dim3(1), dim3(256), 0, s, (ee_cbc_state*)st, window, cbc_max);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

int launch_cbc_push(void* st, const uint8_t* flags, int n, hipStream_t s) {
    TimedScope t(EE_K_CBC, s);
    hipLaunchKernelGGL(k_cbc_push, dim3(1), dim3(64), 0, s, (ee_cbc_state*)st, flags, n);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ Performance History Table row
__global__ void k_pht_init(ee_pht_row* row) {
    if (threadIdx.x == 0) { row->tokens = 0; row->breaches = 0; row->nll = 0.0; }
    if (threadIdx.x < EE_MAX_EXITS) row->exits[threadIdx.x] = 0;
}

struct ExitLayers { int32_t n; int32_t layer[EE_MAX_EXITS]; };

// One workgroup.  Thread t takes rows t, t + 256, ...; the -ln p partial sums are added in a
// fixed tree order in fp64, so the result does not depend on scheduling.
__global__ void __launch_bounds__(256)
k_pht_push(ee_pht_row* row, const int32_t* __restrict__ out_layer, const float* __restrict__ out_conf,
           const uint8_t* __restrict__ out_breach, int B, ExitLayers ex) {
    __shared__ int s_cnt[EE_MAX_EXITS + 2];
    __shared__ double s_sum[256];
    if (threadIdx.x < EE_MAX_EXITS + 2) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    double acc = 0.0;
    for (int b = threadIdx.x; b < B; b += 256) {
        const int l = out_layer[b];
        int e = -1;
        for (int j = 0; j < ex.n; ++j)
            if (ex.layer[j] == l) e = j;
        if (e < 0) continue;
        atomicAdd(&s_cnt[e], 1);
        atomicAdd(&s_cnt[EE_MAX_EXITS], 1);
        if (out_breach[b]) atomicAdd(&s_cnt[EE_MAX_EXITS + 1], 1);
        acc += -log((double)out_conf[b]);
    }
    s_sum[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) s_sum[threadIdx.x] += s_sum[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x < EE_MAX_EXITS) row->exits[threadIdx.x] += s_cnt[threadIdx.x];
    if (threadIdx.x == 0) {
        row->tokens += s_cnt[EE_MAX_EXITS];
        row->breaches += s_cnt[EE_MAX_EXITS + 1];
        row->nll += s_sum[0];
    }
}

int launch_pht_init(void* row, hipStream_t s) {
    hipLaunchKernelGGL(k_pht_init, dim3(1), dim3(64), 0, s, (ee_pht_row*)row);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

int launch_pht_push(void* row, const ee_model* m, const ee_batch* b, hipStream_t s) {
    ExitLayers ex;
    ex.n = m->cfg.n_exits;
    for (int e = 0; e < EE_MAX_EXITS; ++e) ex.layer[e] = e < ex.n ? m->cfg.exit_layers[e] : -1;
    const ee_batch_layout& L = b->L;
    TimedScope t(EE_K_PHT, s);
    hipLaunchKernelGGL(k_pht_push, dim3(1), dim3(256), 0, s, (ee_pht_row*)row, b->st<int32_t>(L.out_layer),
                       b->st<float>(L.out_conf), b->st<uint8_t>(L.out_breach), b->B, ex);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ weight repacking
// one thread per 8-value chunk of the source matrix: source row i, columns 8 co .. 8 co + 7 go to
// destination row R = row_off + i * row_stride, i.e. to lane R % 32 + 32 (co % 2) of tile (R / 32, co / 2)
__global__ void k_pack_weight(const bf16_t* __restrict__ src, int n_out, int n_in, bf16_t* __restrict__ dst,
                              int row_off, int row_stride, int dst_rows) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int n8 = n_in >> 3;
    if (c >= (int64_t)n_out * n8) return;
    const int i = (int)(c / n8), co = (int)(c % n8);
    const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)i * n_in + (int64_t)co * 8);
    const int64_t R = (int64_t)row_off + (int64_t)i * row_stride;
    const int64_t slot = (int64_t)(co >> 1) * (dst_rows >> 5) + (R >> 5);
    *reinterpret_cast<uint4*>(dst + (slot * 64 + (R & 31) + 32 * (co & 1)) * 8) = v;
}

int launch_pack_weight(const void* src, int n_out, int n_in, void* dst, int row_off, int row_stride,
                       int dst_rows, hipStream_t s) {
    int64_t total = (int64_t)n_out * (n_in / 8);
    hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const bf16_t*)src, n_out, n_in, (bf16_t*)dst, row_off, row_stride, dst_rows);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ pool import / export
// plain [H_kv][n_pos][hd] context <-> pool layout of one (layer, row)
template <typename T, bool BF16_LAYOUT>
__global__ void k_kv_copy(KvView kv, int row, int pos0, int n_pos, T* __restrict__ k, T* __restrict__ v,
                          int to_pool) {
    int hd = kv.head_dim;
    int64_t total = (int64_t)kv.n_kv_heads * n_pos * hd;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int i = (int)(idx % hd);
    int p = (int)((idx / hd) % n_pos);
    int g = (int)(idx / ((int64_t)hd * n_pos));
    int cap = kv.cap[row];
    if (pos0 + p >= cap) return;
    T* base = reinterpret_cast<T*>(kv.pool) + kv_block(kv, row, g, cap);
    T* kp = base + (BF16_LAYOUT ? k_bf16_offset(pos0 + p, i, hd) : ((int64_t)(pos0 + p) * hd + i));
    T* vp = base + (BF16_LAYOUT ? v_bf16_offset(pos0 + p, i, hd)
                                : ((int64_t)cap * hd + (int64_t)(pos0 + p) * hd + i));
    if (to_pool) { *kp = k[idx]; *vp = v[idx]; }
    else         { k[idx] = *kp; v[idx] = *vp; }
}

int launch_kv_copy_context(const ee_model* m, const ee_kv* kv, int layer, int row, int pos0, int n_pos,
                           void* k, void* v, bool to_pool, hipStream_t s) {
    KvView view{kv->pool, kv->d_cap, kv->d_off, kv->T, m->cfg.n_kv_heads, m->cfg.head_dim, layer - 1, nullptr};
    int64_t total = (int64_t)m->cfg.n_kv_heads * n_pos * m->cfg.head_dim;
    if (total == 0) return EE_OK;
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (m->cfg.dtype == EE_BF16)
        hipLaunchKernelGGL((k_kv_copy<bf16_t, true>), grid, block, 0, s, view, row, pos0, n_pos, (bf16_t*)k,
                           (bf16_t*)v, to_pool ? 1 : 0);
    else
        hipLaunchKernelGGL((k_kv_copy<float, false>), grid, block, 0, s, view, row, pos0, n_pos, (float*)k,
                           (float*)v, to_pool ? 1 : 0);
    EE_LAUNCH_CHECK();
    return EE_OK;
}

// ------------------------------------------------------------------ exit decision
// Each active row has n_part partial softmax statistics over disjoint column
// ranges of the (scaled) logits: the range's maximum, the sum of exp(z - max)
// over the range, and the lowest column attaining the maximum.  This kernel
// merges them, in a fixed order, into the row's confidence (largest softmax
// probability = 1 / sum_j exp(z_j - max)) and token, and takes the exit decision:
// a row leaves when its confidence meets the threshold, or when nothing deeper
// is resident; leaving below the threshold is a breach.
__global__ void __launch_bounds__(256)
k_exit_decide(const float* __restrict__ part_max, const float* __restrict__ part_sum,
              const int32_t* __restrict__ part_arg, int n_part, const int32_t* __restrict__ n_active, int B,
              float threshold, int force_exit, float* __restrict__ head_conf, int32_t* __restrict__ head_tok,
              uint8_t* __restrict__ head_exit, uint8_t* __restrict__ head_breach) {
    __shared__ Stat sw[4];
    int i = blockIdx.x;
    int n = *n_active;
    if (n > B) n = B;
    if (i >= n) return;
    Stat st{-FLT_MAX, 0.f, 0x7fffffff};
    int64_t base = (int64_t)i * n_part;
    for (int t = threadIdx.x; t < n_part; t += 256) {
        Stat p{part_max[base + t], part_sum[base + t], part_arg[base + t]};
        st = stat_merge(st, p);
    }
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
        float conf = 1.0f / r.s;
        bool met = conf >= threshold;
        head_conf[i] = conf;
        head_tok[i] = r.a;
        head_exit[i] = (met || force_exit) ? 1 : 0;
        head_breach[i] = (force_exit && !met) ? 1 : 0;
    }
}

int launch_exit_decide(ee_batch* b, int n_part, float th, int force, hipStream_t s) {
    const ee_batch_layout& L = b->L;
    TimedScope t(EE_K_EXIT_DECIDE, s);
    hipLaunchKernelGGL(k_exit_decide, dim3(b->B), dim3(256), 0, s, b->wsp<float>(b->W.part_max),
                       b->wsp<float>(b->W.part_sum), b->wsp<int32_t>(b->W.part_arg), n_part,
                       b->st<int32_t>(L.n_active), b->B, th, force, b->st<float>(L.head_conf),
                       b->st<int32_t>(L.head_tok), b->st<uint8_t>(L.head_exit), b->st<uint8_t>(L.head_breach));
    EE_LAUNCH_CHECK();
    return EE_OK;
}
