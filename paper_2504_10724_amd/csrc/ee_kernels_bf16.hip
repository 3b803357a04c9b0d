// ee_kernels_bf16.hip -- the decode step for EE_BF16 models on gfx950.
//
// Data layout
//   * Weight matrices are streamed from HBM exactly once per call, in the tile
//     order ee_pack_weight produces: a 32(out) x 16(in) tile is 1 KiB and is the
//     B operand of one v_mfma_f32_32x32x16_bf16 as it sits in memory (lane l
//     holds output row l%32, inputs 8*(l/32)..+7), so a wave loads it with one
//     fully coalesced 16-byte-per-lane read and no LDS transpose.
//   * Activations that feed a matrix product (normalised rows, attention
//     output, SwiGLU product) are written by their producers in the same tile
//     order (32 rows x 16 columns per tile), i.e. as ready-made A operands.
//   * Everything indexed by "i" is in compacted order (i-th active row);
//     the residual stream, the cache, positions and outputs are indexed by row id.
#include "ee_device.h"

#include <float.h>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// ------------------------------------------------------------------ RMSNorm -> A tiles
// one block per list entry i; out is the [Mpad][d] activation matrix in tile order
__global__ void __launch_bounds__(256)
k_bf16_rmsnorm(const float* __restrict__ h, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_ptr,
               int B, const float* __restrict__ gain, float eps, int d, uint4* __restrict__ out) {
    __shared__ float red[4];
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    const float4* hr = reinterpret_cast<const float4*>(h + (int64_t)idx[i] * d);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    int n8 = d >> 3;
    float ss = 0.f;
    for (int c = threadIdx.x; c < n8; c += 256) {
        float4 a = hr[2 * c], b = hr[2 * c + 1];
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
    }
    ss = block_sum<256>(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)d + eps);
    int KB = d >> 4;
    for (int c = threadIdx.x; c < n8; c += 256) {
        float4 a = hr[2 * c], b = hr[2 * c + 1];
        float4 ga = g4[2 * c], gb = g4[2 * c + 1];
        uint4 o;
        o.x = pack2((a.x * inv) * ga.x, (a.y * inv) * ga.y);
        o.y = pack2((a.z * inv) * ga.z, (a.w * inv) * ga.w);
        o.z = pack2((b.x * inv) * gb.x, (b.y * inv) * gb.y);
        o.w = pack2((b.z * inv) * gb.z, (b.w * inv) * gb.w);
        out[afrag_chunk(i, c * 8, KB)] = o;
    }
}

// ------------------------------------------------------------------ weight-streaming MFMA GEMM
// out[i][j] = sum_k X[i][k] W[j][k] for the first n rows of X (n read on the device).
// A workgroup has WK x WN waves.  Wave (wk, wn) owns NS consecutive 32-column
// tile-rows of W, all MS 32-row tiles of X, and the wk-th slice of the K range;
// the WK partial sums of a tile are added in a fixed order through LDS.
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_EXIT = 3 };

struct EpiArgs {
    float*         out;       // STORE: [i][ldo]; RESID: residual stream [row id][ldo]
    int            ldo;
    const int32_t* idx;       // row id of list entry i
    const float*   row_scale; // EXIT: per row id
    float*         part_max;  // EXIT: [i][n_part]
    float*         part_sum;
    int32_t*       part_arg;
    int            n_part;
    float*         dbg_logits;// EXIT, nullable: [i][ldo]
    bf16_t*        act;       // SWIGLU: [Mpad][F] in tile order
    int            KB_act;    // F / 16
};

template <int MS, int NS, int WK, int WN, int EPI>
__global__ void __launch_bounds__(64 * WK * WN)
k_bf16_gemm(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int KB, int NB_total,
            const int32_t* __restrict__ n_ptr, int B, EpiArgs ep) {
    constexpr int IPW = 16 / WK;   // accumulator registers each wave finishes after the reduction
    __shared__ float red[(WK > 1) ? (WK * WN * NS * 16 * 64) : 1];
    const int n = min(*n_ptr, B);
    const int row_base = blockIdx.y * (32 * MS);
    if (row_base >= n) return;
    const int mbs = min(MS, (n - row_base + 31) >> 5);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wk = wave % WK, wn = wave / WK;
    const int nb0 = (blockIdx.x * WN + wn) * NS;
    const int kb_lo = (int)(((int64_t)KB * wk) / WK), kb_hi = (int)(((int64_t)KB * (wk + 1)) / WK);
    const uint4* xw = Xp + ((int64_t)blockIdx.y * MS * KB) * 64 + lane;
    const uint4* ww = Wp + ((int64_t)nb0 * KB) * 64 + lane;
    const bool has_cols = nb0 + NS <= NB_total;   // uniform per wave

    floatx16 acc[MS][NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < NS; ++ns)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][ns][r] = 0.f;

    if (has_cols) {
        int kb = kb_lo;
        for (; kb + 4 <= kb_hi; kb += 4) {
            uint4 bw[4][NS];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int ns = 0; ns < NS; ++ns) bw[u][ns] = ww[((int64_t)ns * KB + kb + u) * 64];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    if (ms < mbs) {
                        uint4 a = xw[((int64_t)ms * KB + kb + u) * 64];
#pragma unroll
                        for (int ns = 0; ns < NS; ++ns)
                            acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(bw[u][ns]),
                                                                                   acc[ms][ns], 0, 0, 0);
                    }
                }
            }
        }
        for (; kb < kb_hi; ++kb) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
                if (ms < mbs) {
                    uint4 a = xw[((int64_t)ms * KB + kb) * 64];
#pragma unroll
                    for (int ns = 0; ns < NS; ++ns) {
                        uint4 bwv = ww[((int64_t)ns * KB + kb) * 64];
                        acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(bwv),
                                                                               acc[ms][ns], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- reduction over the K slices and epilogue, one 32-row tile at a time
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) {
        if (ms >= mbs) break;              // uniform over the workgroup
        float v[NS][IPW];
        if (WK > 1) {
#pragma unroll
            for (int ns = 0; ns < NS; ++ns)
#pragma unroll
                for (int r = 0; r < 16; ++r) red[((wave * NS + ns) * 16 + r) * 64 + lane] = acc[ms][ns][r];
            __syncthreads();
#pragma unroll
            for (int ns = 0; ns < NS; ++ns)
#pragma unroll
                for (int ii = 0; ii < IPW; ++ii) {
                    float s = 0.f;
#pragma unroll
                    for (int k2 = 0; k2 < WK; ++k2)
                        s += red[(((wn * WK + k2) * NS + ns) * 16 + (wk * IPW + ii)) * 64 + lane];
                    v[ns][ii] = s;
                }
            __syncthreads();
        } else {
#pragma unroll
            for (int ns = 0; ns < NS; ++ns)
#pragma unroll
                for (int ii = 0; ii < IPW; ++ii) v[ns][ii] = acc[ms][ns][ii];
        }
        if (!has_cols) continue;
#pragma unroll
        for (int ii = 0; ii < IPW; ++ii) {
            const int r = wk * IPW + ii;   // accumulator register index 0..15
            const int row = row_base + 32 * ms + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            const bool live = row < n;
            const int cl = lane & 31;
            if (EPI == EPI_STORE) {
                if (live) {
#pragma unroll
                    for (int ns = 0; ns < NS; ++ns)
                        ep.out[(int64_t)row * ep.ldo + 32 * (nb0 + ns) + cl] = v[ns][ii];
                }
            } else if (EPI == EPI_RESID) {
                if (live) {
                    float* hr = ep.out + (int64_t)ep.idx[row] * ep.ldo;
#pragma unroll
                    for (int ns = 0; ns < NS; ++ns) hr[32 * (nb0 + ns) + cl] += v[ns][ii];
                }
            } else if (EPI == EPI_SWIGLU) {
                // tile-rows 2j / 2j+1 of the packed matrix are gate / up of columns 32j..32j+31
                if (live) {
                    float gt = v[0][ii], up = v[NS - 1][ii];
                    float a = (gt / (1.0f + expf(-gt))) * up;
                    int col = 32 * (nb0 >> 1) + cl;
                    ep.act[afrag_chunk(row, col & ~7, ep.KB_act) * 8 + (col & 7)] = f32_to_bf16(a);
                }
            } else {   // EPI_EXIT
                int col = 32 * nb0 + cl;
                float z = live ? v[0][ii] * ep.row_scale[ep.idx[row]] : 0.f;
                if (live && ep.dbg_logits) ep.dbg_logits[(int64_t)row * ep.ldo + col] = z;
                Stat st{z, 1.0f, col};
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) {
                    Stat y{__shfl_xor(st.m, o, 64), __shfl_xor(st.s, o, 64), __shfl_xor(st.a, o, 64)};
                    st = stat_merge(st, y);
                }
                if (live && cl == 0) {
                    int64_t at = (int64_t)row * ep.n_part + nb0;
                    ep.part_max[at] = st.m; ep.part_sum[at] = st.s; ep.part_arg[at] = st.a;
                }
            }
        }
    }
}

// ------------------------------------------------------------------ RoPE + cache append
// buf[i] = [q (n_q heads, may be 0) | k (Hkv heads) | v (Hkv heads)], fp32, hd = 128.
// Queries are rotated and written as a bf16 pair (hi, lo) with hi + lo = q to 16
// mantissa bits, so that the attention kernel can feed them to the bf16 matrix
// cores without giving up fp32-grade scores.  Keys are rotated, rounded and
// appended; values are rounded and appended in the grouped layout.
__global__ void __launch_bounds__(256)
k_bf16_rope_append(const float* __restrict__ buf, int ld, int n_q, const int32_t* __restrict__ idx,
                   const int32_t* __restrict__ n_ptr, int B, const int32_t* __restrict__ pos,
                   const float* __restrict__ rope, int max_pos, KvView kv, bf16_t* __restrict__ q_hi,
                   bf16_t* __restrict__ q_lo, int32_t* __restrict__ status) {
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    int b = idx[i];
    int p = pos[b];
    const int hd = 128, half = 64;
    int Hkv = kv.n_kv_heads;
    int cap = kv.cap[b];
    if (p < 0 || p >= cap || p >= max_pos) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        return;
    }
    const float* r = buf + (int64_t)i * ld;
    const float* cs = rope + (int64_t)p * half * 2;
    for (int t = threadIdx.x; t < n_q * half; t += 256) {
        int hh = t >> 6, j = t & 63;
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = r[hh * hd + j], bb = r[hh * hd + j + half];
        float x0 = a * c - bb * s, x1 = bb * c + a * s;
        bf16_t h0 = f32_to_bf16(x0), h1 = f32_to_bf16(x1);
        int64_t o = ((int64_t)i * n_q + hh) * hd + j;
        q_hi[o] = h0; q_hi[o + half] = h1;
        q_lo[o] = f32_to_bf16(x0 - bf16_to_f32(h0));
        q_lo[o + half] = f32_to_bf16(x1 - bf16_to_f32(h1));
    }
    const float* kin = r + n_q * hd;
    const float* vin = kin + Hkv * hd;
    for (int t = threadIdx.x; t < Hkv * half; t += 256) {
        int g = t >> 6, j = t & 63;
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = kin[g * hd + j], bb = kin[g * hd + j + half];
        bf16_t* base = reinterpret_cast<bf16_t*>(kv.pool) + kv_block(kv, b, g, cap);
        base[(int64_t)p * hd + j] = f32_to_bf16(a * c - bb * s);
        base[(int64_t)p * hd + j + half] = f32_to_bf16(bb * c + a * s);
    }
    for (int t = threadIdx.x; t < Hkv * hd; t += 256) {
        int g = t >> 7, j = t & 127;
        bf16_t* base = reinterpret_cast<bf16_t*>(kv.pool) + kv_block(kv, b, g, cap);
        base[(int64_t)cap * hd + v_bf16_offset(p, j, hd)] = f32_to_bf16(vin[g * hd + j]);
    }
}

// ------------------------------------------------------------------ decode attention
// One workgroup per (kv head g, list entry i); its 4 waves take the 32-position
// groups of the row's cache round-robin and are merged at the end.  Per group:
//   S^T[pos][head] = K[pos][:] . q[head][:]   two 16x16x32 MFMAs per 32 features
//   online softmax over positions (fp32, per head)
//   O^T[feat][head] += V^T[feat][pos] P^T[pos][head]
// The G = H_q/H_kv query heads that share the kv head are the N dimension of
// the MFMAs, so each cached element is read from HBM once and used G times.
// The result registers of the score MFMAs are, lane for lane, the P operand
// of the value MFMAs (the grouped V layout is chosen to make that so).
// q and P enter as bf16 (hi, lo) pairs: two MFMAs each, fp32-grade products.
__global__ void __launch_bounds__(256)
k_bf16_attn(const bf16_t* __restrict__ q_hi, const bf16_t* __restrict__ q_lo, int Hq,
            const int32_t* __restrict__ idx, const int32_t* __restrict__ n_ptr, int B,
            const int32_t* __restrict__ pos, KvView kv, uint4* __restrict__ ao, int KB_ao) {
    __shared__ float sm_m[4][16];
    __shared__ float sm_l[4][16];
    __shared__ float sm_o[4][16][128];
    const int g = blockIdx.x, i = blockIdx.y;
    const int n = min(*n_ptr, B);
    if (i >= n) return;
    const int b = idx[i];
    const int cap = kv.cap[b];
    const int n_pos = max(1, min(pos[b] + 1, cap));
    const int G = Hq / kv.n_kv_heads;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n16 = lane & 15, gq = lane >> 4;
    const bf16_t* Kb = reinterpret_cast<const bf16_t*>(kv.pool) + kv_block(kv, b, g, cap);
    const bf16_t* Vb = Kb + (int64_t)cap * 128;

    bf16x8 qh[4], ql[4];
    {
        uint4 z = make_uint4(0, 0, 0, 0);
        const int64_t qo = ((int64_t)i * Hq + (int64_t)g * G + n16) * 128 + 8 * gq;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            qh[c] = as_bf16x8(n16 < G ? *reinterpret_cast<const uint4*>(q_hi + qo + 32 * c) : z);
            ql[c] = as_bf16x8(n16 < G ? *reinterpret_cast<const uint4*>(q_lo + qo + 32 * c) : z);
        }
    }
    const float inv_sqrt = 1.0f / sqrtf(128.0f);
    const float NEG = -1.0e30f;
    float m_run = NEG, l_run = 0.f;
    floatx4 O[8];
#pragma unroll
    for (int hb = 0; hb < 8; ++hb) O[hb] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_groups = (n_pos + 31) >> 5;
    for (int t = w; t < n_groups; t += 4) {
        const int p0 = t << 5;
        floatx4 S0 = {0.f, 0.f, 0.f, 0.f}, S1 = {0.f, 0.f, 0.f, 0.f};
        const bf16_t* k0 = Kb + (int64_t)(p0 + n16) * 128 + 8 * gq;
        const bf16_t* k1 = k0 + 16 * 128;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bf16x8 a0 = as_bf16x8(*reinterpret_cast<const uint4*>(k0 + 32 * c));
            bf16x8 a1 = as_bf16x8(*reinterpret_cast<const uint4*>(k1 + 32 * c));
            S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qh[c], S0, 0, 0, 0);
            S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, ql[c], S0, 0, 0, 0);
            S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qh[c], S1, 0, 0, 0);
            S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, ql[c], S1, 0, 0, 0);
        }
        // S0[r]: position p0 + 4 gq + r ; S1[r]: position p0 + 16 + 4 gq + r ; head n16
        float s[8];
        float mx = NEG;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s[r]     = (p0 + 4 * gq + r < n_pos) ? S0[r] * inv_sqrt : NEG;
            s[4 + r] = (p0 + 16 + 4 * gq + r < n_pos) ? S1[r] * inv_sqrt : NEG;
            mx = fmaxf(mx, fmaxf(s[r], s[4 + r]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __expf(m_run - m_new);
        float pv[8], lsum = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) { pv[r] = __expf(s[r] - m_new); lsum += pv[r]; }
        l_run = l_run * alpha + lsum;
        m_run = m_new;
        uint4 ph, pl;
        {
            bf16_t hi[8], lo[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                hi[r] = f32_to_bf16(pv[r]);
                lo[r] = f32_to_bf16(pv[r] - bf16_to_f32(hi[r]));
            }
            ph = make_uint4(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16),
                            hi[4] | ((uint32_t)hi[5] << 16), hi[6] | ((uint32_t)hi[7] << 16));
            pl = make_uint4(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16),
                            lo[4] | ((uint32_t)lo[5] << 16), lo[6] | ((uint32_t)lo[7] << 16));
        }
        const bool partial = p0 + 32 > n_pos;
        const bf16_t* vg = Vb + ((int64_t)(t * 4 + gq) * 128 + n16) * 8;
#pragma unroll
        for (int hb = 0; hb < 8; ++hb) {
            uint4 vv = *reinterpret_cast<const uint4*>(vg + (int64_t)hb * 16 * 8);
            if (partial) {
                // element j of the chunk is position p0 + 4 gq + j (j < 4) or p0 + 16 + 4 gq + j - 4
                uint32_t* vw = reinterpret_cast<uint32_t*>(&vv);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    int pj = p0 + ((j < 4) ? (4 * gq + j) : (16 + 4 * gq + j - 4));
                    if (pj >= n_pos) vw[j >> 1] &= (j & 1) ? 0x0000ffffu : 0xffff0000u;
                }
            }
            O[hb] = O[hb] * alpha;
            O[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), as_bf16x8(ph), O[hb], 0, 0, 0);
            O[hb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), as_bf16x8(pl), O[hb], 0, 0, 0);
        }
    }
    // O[hb][r]: feature 16 hb + 4 gq + r of head n16 (unnormalised), this wave's positions
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (gq == 0) { sm_m[w][n16] = m_run; sm_l[w][n16] = l_run; }
#pragma unroll
    for (int hb = 0; hb < 8; ++hb)
#pragma unroll
        for (int r = 0; r < 4; ++r) sm_o[w][n16][16 * hb + 4 * gq + r] = O[hb][r];
    __syncthreads();
    {
        const int head = threadIdx.x >> 4, c0 = (threadIdx.x & 15) * 8;
        if (head < G) {
            float M = fmaxf(fmaxf(sm_m[0][head], sm_m[1][head]), fmaxf(sm_m[2][head], sm_m[3][head]));
            float wgt[4], Lsum = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) { wgt[k] = __expf(sm_m[k][head] - M); Lsum += sm_l[k][head] * wgt[k]; }
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k) acc += sm_o[k][head][c0 + j] * wgt[k];
                o[j] = acc / Lsum;
            }
            uint4 pk = make_uint4(pack2(o[0], o[1]), pack2(o[2], o[3]), pack2(o[4], o[5]), pack2(o[6], o[7]));
            int col = (g * G + head) * 128 + c0;
            ao[afrag_chunk(i, col, KB_ao)] = pk;
        }
    }
}

// ------------------------------------------------------------------ host side
static KvView make_view(const ee_model* m, const ee_kv* kv, int layer) {
    return KvView{kv->pool, kv->d_cap, kv->d_off, kv->T, m->cfg.n_kv_heads, m->cfg.head_dim, layer - 1};
}

template <int MS, int NS, int WK, int WN, int EPI>
static void gemm_launch(const void* X, const void* W, int K, int NB_total, const int32_t* n_ptr, int B,
                        int row_groups, const EpiArgs& ep, hipStream_t s) {
    dim3 grid((NB_total + WN * NS - 1) / (WN * NS), row_groups);
    hipLaunchKernelGGL((k_bf16_gemm<MS, NS, WK, WN, EPI>), grid, dim3(64 * WK * WN), 0, s, (const uint4*)X,
                       (const uint4*)W, K / 16, NB_total, n_ptr, B, ep);
}

// picks the tile configuration from the row capacity of the batch
template <int NS, int EPI>
static void gemm(const void* X, const void* W, int N, int K, const int32_t* n_ptr, int B, const EpiArgs& ep,
                 hipStream_t s) {
    int NB = N / 32;
    int Mpad = (B + 31) / 32 * 32;
    if (Mpad <= 32)       gemm_launch<1, NS, 8, 1, EPI>(X, W, K, NB, n_ptr, B, 1, ep, s);
    else if (Mpad <= 64)  gemm_launch<2, NS, 8, 1, EPI>(X, W, K, NB, n_ptr, B, 1, ep, s);
    else if (Mpad <= 128) gemm_launch<4, NS, 2, 2, EPI>(X, W, K, NB, n_ptr, B, 1, ep, s);
    else                  gemm_launch<8, NS, 1, 4, EPI>(X, W, K, NB, n_ptr, B, (Mpad + 255) / 256, ep, s);
}

int bf16_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_layer_weights& w = m->layers[layer - 1];
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, hd = c.head_dim, qd = c.n_q_heads * hd, F = c.d_ffn;
    int qkv_n = (c.n_q_heads + 2 * c.n_kv_heads) * hd;
    const int32_t* idx = b->st<int32_t>(L.active_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_active);
    float* h = b->st<float>(L.h);
    uint4* x = b->wsp<uint4>(b->W.x);
    float* qkv = b->wsp<float>(b->W.qkv);
    uint4* ao = b->wsp<uint4>(b->W.ao);
    bf16_t* act = b->wsp<bf16_t>(b->W.act);
    KvView view = make_view(m, kv, layer);

    {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(256), 0, s, h, idx, n_ptr, B, w.g_attn, c.rms_eps, d, x);
    }
    EpiArgs e1{};
    e1.out = qkv; e1.ldo = qkv_n; e1.idx = idx;
    {
        TimedScope t(EE_K_GEMM_QKV, s);
        gemm<1, EPI_STORE>(x, w.w_qkv, qkv_n, d, n_ptr, B, e1, s);
    }
    {
        TimedScope t(EE_K_ROPE_APPEND, s);
        hipLaunchKernelGGL(k_bf16_rope_append, dim3(B), dim3(256), 0, s, qkv, qkv_n, c.n_q_heads, idx, n_ptr, B,
                           b->st<int32_t>(L.pos), m->d_rope, c.max_pos, view, b->wsp<bf16_t>(b->W.q_hi),
                           b->wsp<bf16_t>(b->W.q_lo), b->st<int32_t>(L.status));
    }
    {
        TimedScope t(EE_K_ATTENTION, s);
        hipLaunchKernelGGL(k_bf16_attn, dim3(c.n_kv_heads, B), dim3(256), 0, s, b->wsp<bf16_t>(b->W.q_hi),
                           b->wsp<bf16_t>(b->W.q_lo), c.n_q_heads, idx, n_ptr, B, b->st<int32_t>(L.pos), view, ao,
                           qd / 16);
    }
    EpiArgs e2{};
    e2.out = h; e2.ldo = d; e2.idx = idx;
    {
        TimedScope t(EE_K_GEMM_O, s);
        gemm<1, EPI_RESID>(ao, w.w_o, d, qd, n_ptr, B, e2, s);
    }
    {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(256), 0, s, h, idx, n_ptr, B, w.g_ffn, c.rms_eps, d, x);
    }
    EpiArgs e3{};
    e3.act = act; e3.KB_act = F / 16; e3.idx = idx;
    {
        TimedScope t(EE_K_GEMM_GATE_UP, s);
        gemm<2, EPI_SWIGLU>(x, w.w_gate_up, 2 * F, d, n_ptr, B, e3, s);
    }
    {
        TimedScope t(EE_K_GEMM_DOWN, s);
        gemm<1, EPI_RESID>(act, w.w_down, d, F, n_ptr, B, e2, s);
    }
    EE_LAUNCH_CHECK();
    return EE_OK;
}

int bf16_exit_head(const ee_model* m, int e, float th, int force, ee_batch* b, float* dbg, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, V = c.vocab;
    const int32_t* idx = b->st<int32_t>(L.active_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_active);
    uint4* x = b->wsp<uint4>(b->W.x);
    {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(256), 0, s, b->st<float>(L.h), idx, n_ptr, B,
                           m->exits[e].gain, c.rms_eps, d, x);
    }
    EpiArgs ep{};
    ep.idx = idx; ep.row_scale = b->st<float>(L.row_scale);
    ep.part_max = b->wsp<float>(b->W.part_max); ep.part_sum = b->wsp<float>(b->W.part_sum);
    ep.part_arg = b->wsp<int32_t>(b->W.part_arg); ep.n_part = V / 32;
    ep.dbg_logits = dbg; ep.ldo = V;
    {
        TimedScope t(EE_K_EXIT_GEMM, s);
        gemm<1, EPI_EXIT>(x, m->exits[e].w, V, d, n_ptr, B, ep, s);
    }
    EE_LAUNCH_CHECK();
    return launch_exit_decide(b, V / 32, th, force, s);
}

int bf16_fill_kv(const ee_model* m, int from_excl, int to_incl, ee_kv* kv, ee_batch* b, hipStream_t s) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, hd = c.head_dim;
    int kv_n = 2 * c.n_kv_heads * hd;
    const int32_t* idx = b->st<int32_t>(L.exited_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_exited);
    uint4* x = b->wsp<uint4>(b->W.fill_x);
    float* kvb = b->wsp<float>(b->W.fill_kv);
    TimedScope t(EE_K_FILL_KV, s);
    for (int l = from_excl + 1; l <= to_incl; ++l) {
        const ee_layer_weights& w = m->layers[l - 1];
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(256), 0, s, b->st<float>(L.h), idx, n_ptr, B, w.g_attn,
                           c.rms_eps, d, x);
        // key and value rows are the last 2*H_kv*hd rows of W_qkv: tile-rows H_q*hd/32 onwards
        const char* Wkv = (const char*)w.w_qkv + (size_t)(c.n_q_heads * hd / 32) * (d / 16) * 1024;
        EpiArgs ep{};
        ep.out = kvb; ep.ldo = kv_n; ep.idx = idx;
        gemm<1, EPI_STORE>(x, Wkv, kv_n, d, n_ptr, B, ep, s);
        hipLaunchKernelGGL(k_bf16_rope_append, dim3(B), dim3(256), 0, s, kvb, kv_n, 0, idx, n_ptr, B,
                           b->st<int32_t>(L.pos), m->d_rope, c.max_pos, make_view(m, kv, l), (bf16_t*)nullptr,
                           (bf16_t*)nullptr, b->st<int32_t>(L.status));
    }
    EE_LAUNCH_CHECK();
    return EE_OK;
}
