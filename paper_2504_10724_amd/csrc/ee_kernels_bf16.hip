// ee_kernels_bf16.hip -- the decode step for EE_BF16 models on gfx950.
//
// Data layout
//   * Weight matrices are streamed from HBM exactly once per call, in the tile
//     order ee_pack_weight produces: a 32(out) x 16(in) tile is 1 KiB and is the
//     B operand of one v_mfma_f32_32x32x16_bf16 as it sits in memory (lane l
//     holds output row l%32, inputs 8*(l/32)..+7), so a wave loads it with one
//     fully coalesced 16-byte-per-lane read and no LDS transpose.  Tiles are
//     ordered K-slice-major (tile (r, c) at slot c * R + r): the workgroups of a
//     launch walk K more or less together, so what they fetch at any moment is
//     one contiguous window of the matrix, spread evenly over the HBM channels,
//     instead of addresses a power of two apart.
//   * Activations that feed a matrix product (normalised rows, attention
//     output, SwiGLU product) are written by their producers in the same tile
//     order (32 rows x 16 columns per tile), i.e. as ready-made A operands.
//   * Everything indexed by "i" is in compacted order (i-th active row);
//     the residual stream, the cache, positions and outputs are indexed by row id.
#include "ee_device.h"

#include <float.h>
#include <algorithm>
#include <type_traits>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Several layers in one launch (blockIdx.z = layer - first layer): used to produce the keys and
// values of all skipped layers at once.  Null tables / zero strides mean a single-layer launch.
struct ZBatch {
    const void* const*  w_tab;     // per layer: packed W_qkv           (device table, index layer - 1)
    const float* const* g_tab;     // per layer: attention-norm gain
    int     z0;                    // table index of blockIdx.z == 0
    int64_t x_stride;              // uint4 units between the layers' activation matrices
    int64_t out_stride;            // floats between the layers' output matrices
};

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// ------------------------------------------------------------------ RMSNorm -> A tiles
// The NORM_THREADS threads of a block normalise one row (hr: d floats) and write it as list entry
// i of the [Mpad][d] activation matrix in tile order.  Every thread reads only the 8-float chunks
// c = threadIdx.x + NORM_THREADS j, so a caller may have written those same chunks just before.
// (1024 threads: one chunk each at d = 8192; the kernels here are latency bound, and every
// user of this routine takes the same thread count so that all give the same bits.)
#define NORM_THREADS 1024
__device__ __forceinline__ void rmsnorm_row(const float* hr_, const float* gain, float eps, int d, uint4* out, int i,
                                            float* red /* NORM_THREADS / 64 floats */) {
    const float4* hr = reinterpret_cast<const float4*>(hr_);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    int n8 = d >> 3;
    float ss = 0.f;
    for (int c = threadIdx.x; c < n8; c += NORM_THREADS) {
        float4 a = hr[2 * c], b = hr[2 * c + 1];
        ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
    }
    ss = block_sum<NORM_THREADS>(ss, red);
    float inv = 1.0f / sqrtf(ss / (float)d + eps);
    int KB = d >> 4;
    for (int c = threadIdx.x; c < n8; c += NORM_THREADS) {
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

// one block per list entry i; out is the [Mpad][d] activation matrix in tile order
__global__ void __launch_bounds__(NORM_THREADS)
k_bf16_rmsnorm(const float* __restrict__ h, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_ptr,
               int B, const float* __restrict__ gain, float eps, int d, uint4* __restrict__ out, ZBatch zb) {
    __shared__ float red[NORM_THREADS / 64];
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    if (zb.g_tab) gain = zb.g_tab[zb.z0 + blockIdx.z];
    out += (int64_t)blockIdx.z * zb.x_stride;
    rmsnorm_row(h + (int64_t)idx[i] * d, gain, eps, d, out, i, red);
}

// ------------------------------------------------------------------ weight-streaming MFMA GEMM
// out[i][j] = sum_k X[i][k] W[j][k] for the first n rows of X (n read on the device).
// A workgroup has WK x WN waves.  Wave (wk, wn) owns NS consecutive 32-column
// tile-rows of W, all MS 32-row tiles of X, and the wk-th slice of the K range;
// the WK partial sums of a tile are added in a fixed order through LDS.
// 16 bytes that this launch reads once (weights, cached keys and values): a non-temporal load.
// Measured: streams of such loads run 10-13 % faster than ordinary ones, which hold a line of
// the vector cache while they are in flight.
__device__ __forceinline__ uint4 load_nt(const uint4* p) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}

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
k_bf16_gemm(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int KB, int NB_total, int NBs, int nb_off,
            const int32_t* __restrict__ n_ptr, int B, EpiArgs ep, ZBatch zb) {
    constexpr int IPW = 16 / WK;   // accumulator registers each wave finishes after the reduction
    constexpr int GD = 4;          // K tiles per load group
    __shared__ float red[(WK > 1) ? (WK * WN * NS * 16 * 64) : 1];
    const int n = min(*n_ptr, B);
    const int row_base = blockIdx.y * (32 * MS);
    if (row_base >= n) return;
    if (zb.w_tab) Wp = reinterpret_cast<const uint4*>(zb.w_tab[zb.z0 + blockIdx.z]);
    Xp += (int64_t)blockIdx.z * zb.x_stride;
    ep.out += (int64_t)blockIdx.z * zb.out_stride;
    const int mbs = min(MS, (n - row_base + 31) >> 5);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wk = wave % WK, wn = wave / WK;
    const int nb0 = (blockIdx.x * WN + wn) * NS;
    const int kb_lo = (int)(((int64_t)KB * wk) / WK), kb_hi = (int)(((int64_t)KB * (wk + 1)) / WK);
    const uint4* xw = Xp + ((int64_t)blockIdx.y * MS * KB) * 64 + lane;
    const uint4* ww = Wp + (int64_t)(nb_off + nb0) * 64 + lane;   // tile (r, c) sits at slot c * NBs + r
    const bool has_cols = nb0 + NS <= NB_total;   // uniform per wave

    floatx16 acc[MS][NS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int ns = 0; ns < NS; ++ns)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ms][ns][r] = 0.f;

    if (has_cols) {
        // groups of GD K tiles, the next group's W and X tiles in flight while the current one is
        // multiplied (dead row tiles re-read a live one, so the loads need no branch); groups twice
        // as deep change nothing: with one row tile per wave half of what a CU requests is X
        struct Group { uint4 w[GD][NS]; uint4 x[GD][MS]; };
        auto load_group = [&](int kb) -> Group {
            Group g;
#pragma unroll
            for (int u = 0; u < GD; ++u) {
#pragma unroll
                for (int ns = 0; ns < NS; ++ns) g.w[u][ns] = load_nt(ww + ((int64_t)(kb + u) * NBs + ns) * 64);
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) g.x[u][ms] = xw[((int64_t)min(ms, mbs - 1) * KB + kb + u) * 64];
            }
            return g;
        };
        auto mul_group = [&](const Group& g) {
#pragma unroll
            for (int u = 0; u < GD; ++u)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms) {
                    if (ms < mbs) {
#pragma unroll
                        for (int ns = 0; ns < NS; ++ns)
                            acc[ms][ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(g.x[u][ms]), as_bf16x8(g.w[u][ns]),
                                                                                   acc[ms][ns], 0, 0, 0);
                    }
                }
        };
        int kb = kb_lo;
        const int n_groups = (kb_hi - kb_lo) / GD;
        if (n_groups > 0) {
            Group cur = load_group(kb);
            for (int gi = 1; gi < n_groups; ++gi) {
                Group nxt = load_group(kb + GD);
                mul_group(cur);
                cur = nxt;
                kb += GD;
            }
            mul_group(cur);
            kb += GD;
        }
        for (; kb < kb_hi; ++kb) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
                if (ms < mbs) {
                    uint4 a = xw[((int64_t)ms * KB + kb) * 64];
#pragma unroll
                    for (int ns = 0; ns < NS; ++ns) {
                        uint4 bwv = ww[((int64_t)kb * NBs + ns) * 64];
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
                // rows 2j / 2j+1 of the gate/up matrix are gate / up of output j: neighbouring lanes
                // (same batch row) hold them, the even lane writes the product
#pragma unroll
                for (int ns = 0; ns < NS; ++ns) {
                    const float mine = v[ns][ii], other = __shfl_xor(mine, 1, 64);
                    const float gt = (cl & 1) ? other : mine, up = (cl & 1) ? mine : other;
                    const float a = (gt / (1.0f + expf(-gt))) * up;
                    const int col = 16 * (nb0 + ns) + (cl >> 1);
                    if (live && !(cl & 1)) ep.act[afrag_chunk(row, col & ~7, ep.KB_act) * 8 + (col & 7)] = f32_to_bf16(a);
                }
            } else {   // EPI_EXIT
                int col = 32 * nb0 + cl;
                float z = live ? v[0][ii] * ep.row_scale[ep.idx[row]] : 0.f;
                if (live && ep.dbg_logits) ep.dbg_logits[(int64_t)row * ep.ldo + col] = z;
                float mx = z;
                int arg = col;
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) {
                    float m2 = __shfl_xor(mx, o, 64);
                    int a2 = __shfl_xor(arg, o, 64);
                    if (m2 > mx || (m2 == mx && a2 < arg)) { mx = m2; arg = a2; }
                }
                float se = expf(z - mx);
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
                if (live && cl == 0) {
                    int64_t at = (int64_t)row * ep.n_part + nb0;
                    ep.part_max[at] = mx; ep.part_sum[at] = se; ep.part_arg[at] = arg;
                }
            }
        }
    }
}

// ------------------------------------------------------------------ large-batch MFMA GEMM
// 256-row tiles (up to 256 rows per row group), 128 or 256 columns wide, one K slice per
// workgroup, operands fed by LDS-DMA loads (k_bf16_gemm_dma8, k_bf16_gemm_dma2 below).  When K
// is sliced, every slice writes an fp32 partial tile into its own plane and a later kernel adds
// the planes in slice order, so the result does not depend on timing and needs no atomics.
#define BIG_THREADS 256
struct Half { uint4 v[4]; };   // A operands of one K half: 4 row tiles

// One 32x32x16 step of a result tile.  A and B operands have the same register layout, so handing
// them over in the other order gives the transposed tile at no cost: a lane then holds 16 columns of
// ONE batch row (of the tile-row's 32 columns, those at 8 q + 4 (lane / 32) + s, q, s = 0..3, in
// register 4 q + s; lane ^ 32 holds the others).  The exit head wants that: the row statistics
// (maximum, its column, sum of exponentials) need one exchange between the two half-waves instead of
// a 32-lane butterfly per accumulator register (measured: 83 of 230 us of the exit-head product).
// So does the SwiGLU epilogue: gate row j and up row j of the gate/up matrix are neighbouring
// columns, i.e. two registers of one lane.
template <int EPI>
__device__ __forceinline__ floatx16 tile_mfma(const uint4& x, const uint4& w, const floatx16& acc) {
    if constexpr (EPI == EPI_EXIT || EPI == EPI_SWIGLU)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(w), as_bf16x8(x), acc, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(x), as_bf16x8(w), acc, 0, 0, 0);
}

// v: the 32x32 result of tile-row nb (columns 32 nb ..) for rows row0 .. row0+31; every lane of the wave calls it
template <int EPI>
__device__ __forceinline__ void epilogue_one(const EpiArgs& ep, const floatx16& v, int row0, int n, int nb, int lane) {
    const int cl = lane & 31;
    if constexpr (EPI == EPI_EXIT) {
        // transposed tile: this lane holds batch row row0 + cl
        const int row = row0 + cl;
        const bool live = row < n;
        const float sc = live ? ep.row_scale[ep.idx[row]] : 0.f;
        const int col0 = 32 * nb + 4 * (lane >> 5);
        float z[16];
        float mx = -FLT_MAX;
        int arg = col0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int col = col0 + 8 * (r >> 2) + (r & 3);        // rising with r: > keeps the lowest column
            z[r] = v[r] * sc;
            if (live && ep.dbg_logits) ep.dbg_logits[(int64_t)row * ep.ldo + col] = z[r];
            if (z[r] > mx) { mx = z[r]; arg = col; }
        }
        const float m2 = __shfl_xor(mx, 32, 64);
        const int a2 = __shfl_xor(arg, 32, 64);
        if (m2 > mx || (m2 == mx && a2 < arg)) { mx = m2; arg = a2; }
        float se = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) se += expf(z[r] - mx);
        se += __shfl_xor(se, 32, 64);
        if (live && lane < 32) {
            const int64_t at = (int64_t)row * ep.n_part + nb;
            ep.part_max[at] = mx; ep.part_sum[at] = se; ep.part_arg[at] = arg;
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // transposed tile of the gate/up matrix (row 2j gate, row 2j+1 up of output j): registers
        // 4q, 4q+1 are gate and up of output 4q + 2h (h = lane / 32) of the tile-row's 16 outputs,
        // registers 4q+2, 4q+3 those of output 4q + 2h + 1.  The half-waves swap two packed pairs so
        // that lane < 32 writes outputs 0..7 and lane >= 32 outputs 8..15 of its batch row as one
        // 16-byte chunk of the next product's operand tiles.
        const int row = row0 + cl, h = lane >> 5;
        uint32_t d[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float g0 = v[4 * q], u0 = v[4 * q + 1], g1 = v[4 * q + 2], u1 = v[4 * q + 3];
            d[q] = pack2((g0 / (1.0f + expf(-g0))) * u0, (g1 / (1.0f + expf(-g1))) * u1);
        }
        const uint32_t r0 = __shfl_xor(h ? d[0] : d[2], 32, 64), r1 = __shfl_xor(h ? d[1] : d[3], 32, 64);
        const uint4 o = h ? make_uint4(r0, d[2], r1, d[3]) : make_uint4(d[0], r0, d[1], r1);
        if (row < n) reinterpret_cast<uint4*>(ep.act)[afrag_chunk(row, 16 * nb + 8 * h, ep.KB_act)] = o;
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = row0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (row >= n) continue;
            if constexpr (EPI == EPI_STORE) ep.out[(int64_t)row * ep.ldo + 32 * nb + cl] = v[r];
            else ep.out[(int64_t)ep.idx[row] * ep.ldo + 32 * nb + cl] += v[r];      // EPI_RESID
        }
    }
}

template <int EPI>
__device__ __forceinline__ void epilogue_tile(const EpiArgs& ep, const floatx16& v0, const floatx16& v1, int row0,
                                              int n, int nb, int lane) {
    epilogue_one<EPI>(ep, v0, row0, n, nb, lane);
    epilogue_one<EPI>(ep, v1, row0, n, nb + 1, lane);
}

// ------------------------------------------------------------------ tile GEMMs fed by LDS-DMA loads
// No operand passes through registers on its way in: the waves of a workgroup send the X and W
// tiles of a 32-wide K stage straight from global memory into LDS (global_load_lds_dwordx4: 64
// lanes x 16 B per instruction, lane l lands at byte 16 l of the slot), and all MFMA operands are
// read from LDS.  A load that returns into registers holds up the matrix pipe of its SIMD while
// it writes back (measured: streaming time and MFMA time add up, even across waves); a load
// into LDS does not, so here the weight stream runs under the MFMAs.  The loads of a stage are
// issued one behind each MFMA group (a burst would queue up in the vector-memory path and hold the
// wave).  The compiler does not see these loads, so it adds no wait of its own; the waits are
// written out.  Loads past the end of the K slice re-read its last stage.
// Which (row group, column tile x K slice) a workgroup takes.  One row group: blockIdx.x is the
// unit.  Several row groups (context pass; the grid is then one-dimensional with gridDim.x =
// 8 ceil(units / 8) x row groups): workgroups are handed to the 8 XCDs round-robin, each XCD has
// its own L2, and the row groups of a unit read the same weight tiles, so they get block numbers
// 8 apart: same XCD, started one after the other, and the tiles come from HBM once, not once
// per row group.  unit = -1: a block past the last unit.
__device__ __forceinline__ void tile_of_block(int units, int& rg, int& unit) {
    if (gridDim.y == 1 && (int)gridDim.x > units) {
        const int u8 = (units + 7) / 8 * 8, R = gridDim.x / u8;
        const int x = blockIdx.x & 7, q = blockIdx.x >> 3;
        rg = q % R;
        unit = (q / R) * 8 + x;
        if (unit >= units) unit = -1;
    } else {
        rg = blockIdx.y;
        unit = blockIdx.x;
    }
}

// tile and lds_byte are the same in all lanes; going through readfirstlane makes that explicit, so
// that both end up in scalar registers whatever the optimiser did to the address arithmetic
// NT: the tile is read once per launch (weights): a non-temporal load, which does not hold a line of
// the vector cache while it is in flight; activations, which every workgroup re-reads, stay cacheable
template <bool NT = false>
__device__ __forceinline__ void dma_tile(const uint4* tile, unsigned lane_bytes, unsigned lds_byte) {
    const uint64_t a = reinterpret_cast<uint64_t>(tile);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    const uint64_t base = ((uint64_t)hi << 32) | lo;
    const uint32_t slot = __builtin_amdgcn_readfirstlane(lds_byte);
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(slot), "v"(lane_bytes), "s"(base)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(slot), "v"(lane_bytes), "s"(base)
                     : "memory");
}

// ------------------------------------------------------------------ 128-column tile fed by LDS-DMA loads
// 256 rows x 128 columns per workgroup, waves 2 x 2: wave (wm, wn) owns rows 128 wm .. +127
// and columns 64 wn .. +63 (4 x 2 MFMA tiles, 128 accumulator registers).  LDS: 6 stage buffers x 24 slots: X tile (row tile m, K half kk)
// at 2 m + kk, W tile (column tile nb of the 4, K half kk) at 16 + 2 nb + kk.  A wave sends up to 4 X
// tiles (those of its live row tiles: against re-reading a live tile in place of a dead one, the
// exit head takes 7-10 % less up to 64 rows and QKV 3-5 %) and 2 W tiles per stage and reads the 8 + 4 it needs.  For products with few columns
// (QKV, O projection, exit head) it gives twice as many workgroups per K slice as the 256-column tile.
// Its stages are short (16 MFMAs per wave), so a stage is requested five stages ahead, not three:
// measured against three it takes 5 % off the QKV product at 256 rows and 14 % at 64.
struct BHalf { uint4 v[2]; };

template <int EPI>
__global__ void __launch_bounds__(BIG_THREADS, 1)
k_bf16_gemm_dma2(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int KB, int NBs, int nb_off,
                 int n_tiles, int splits, const int32_t* __restrict__ n_ptr, int B, float* __restrict__ partial,
                 int64_t part_plane, int part_ld, EpiArgs ep, ZBatch zb) {
    __shared__ uint4 lds[6][24][64];          // six stage buffers: a stage is requested five stages ahead
    const int n = min(*n_ptr, B);
    int rg, unit;
    tile_of_block(n_tiles * splits, rg, unit);
    if (unit < 0) return;
    const int row_base = rg * 256;
    if (row_base >= n) return;
    if (zb.w_tab) Wp = reinterpret_cast<const uint4*>(zb.w_tab[zb.z0 + blockIdx.z]);
    Xp += (int64_t)blockIdx.z * zb.x_stride;
    ep.out += (int64_t)blockIdx.z * zb.out_stride;
    const int mbs = min(8, (n - row_base + 31) >> 5);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int cnt = max(0, min(4, mbs - 4 * wm));            // live 32-row tiles of this wave
    const int tile = unit / splits, sp = unit % splits;
    const int nbw = (tile * 2 + wn) * 2;                     // first of this wave's two tile-rows of W
    const int KS4 = KB >> 3;
    const int ks_lo = 4 * (int)(((int64_t)KS4 * sp) / splits), ks_hi = 4 * (int)(((int64_t)KS4 * (sp + 1)) / splits);
    const int T = ks_hi - ks_lo;                             // stages of this slice: a positive multiple of 4
    const uint4* xg = Xp + ((int64_t)rg * 8 * KB) * 64;
    const uint4* wg = Wp + (int64_t)(nb_off + tile * 4) * 64;   // the tile's four tile-rows of W
    const unsigned lane_bytes = (unsigned)lane * 16u;
    const unsigned lds0 = (unsigned)(size_t)&lds[0][0][0];

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // j-th load of a stage: j = 0..3 X tiles (row tile 2 wave + j/2, K half j%2; sent only if that
    // row tile is live); j = 4, 5 the W slots 2 wave + (j - 4) of the stage's eight (column tile
    // q/2, K half q%2).  A tile's address is the stage's base pointer (scalar, computed once per
    // stage) plus a lane offset that is the same in every stage, so a load costs few instructions.
    unsigned voff[6];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = min(2 * wave + (j >> 1), mbs - 1);
        voff[j] = lane_bytes + ((unsigned)(m * KB + (j & 1)) << 10);
    }
#pragma unroll
    for (int j = 4; j < 6; ++j) {
        const int q = 2 * wave + (j - 4), nb = q >> 1, kk = q & 1;
        voff[j] = lane_bytes + ((unsigned)(kk * NBs + nb) << 10);
    }
    auto x_base = [&](int t) { return xg + (int64_t)(2 * (ks_lo + min(t, T - 1))) * 64; };
    auto w_base = [&](int t) { return wg + (int64_t)(2 * (ks_lo + min(t, T - 1))) * NBs * 64; };
    auto issue = [&](const uint4* xs, const uint4* ws, int buf, int j) {
        if (j < 4) dma_tile(xs, voff[j], lds0 + (unsigned)((buf * 24 + (2 * wave + (j >> 1)) * 2 + (j & 1)) << 10));
        else dma_tile<true>(ws, voff[j], lds0 + (unsigned)((buf * 24 + 16 + 2 * wave + (j - 4)) << 10));
    };
    Half a0, a1;
    BHalf b0, b1;
    auto rd_a = [&](Half& o, int buf, int kk, int i) { o.v[i] = (&lds[0][0][lane] + buf * (24 * 64))[((4 * wm + i) * 2 + kk) * 64]; };
    auto rd_b = [&](BHalf& o, int buf, int kk) {
        const uint4* p = &lds[0][0][lane] + buf * (24 * 64);
        o.v[0] = p[(16 + (2 * wn) * 2 + kk) * 64];
        o.v[1] = p[(16 + (2 * wn + 1) * 2 + kk) * 64];
    };
    auto mf_all = [&](const Half& a, const BHalf& bw, int i) {
        acc[i][0] = tile_mfma<EPI>(a.v[i], bw.v[0], acc[i][0]);
        acc[i][1] = tile_mfma<EPI>(a.v[i], bw.v[1], acc[i][1]);
    };
    auto mf_some = [&](const Half& a, const BHalf& bw, int i) {
        if (i < cnt) mf_all(a, bw, i);
    };
#define SB __builtin_amdgcn_sched_barrier(0);
// three stages of this wave's loads (VM of them) may stay in flight: everything up to stage t+2 has landed
#define STAGE_END(VM) asm volatile("s_waitcnt vmcnt(" #VM ") lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // bc / bn / bi: buffers of the current stage, the next one and the one being requested (stage + 5);
    // six buffers and an unroll of four do not divide, so the indices are counted at run time.
    // XL: how many of this wave's two row tiles are live and fetched
#define DMA2_STAGE(MF, XL, VM, U)                                                             \
    { const uint4* xs_ = x_base(t0 + (U) + 5); const uint4* ws_ = w_base(t0 + (U) + 5);       \
    MF(a0, b0, 0); SB if (XL >= 1) issue(xs_, ws_, bi, 0); rd_a(a1, bc, 1, 0); rd_a(a1, bc, 1, 1); rd_b(b1, bc, 1); SB \
    MF(a0, b0, 1); SB if (XL >= 1) issue(xs_, ws_, bi, 1); rd_a(a1, bc, 1, 2); rd_a(a1, bc, 1, 3); SB \
    MF(a0, b0, 2); SB if (XL >= 2) issue(xs_, ws_, bi, 2); SB                                 \
    MF(a0, b0, 3); SB if (XL >= 2) issue(xs_, ws_, bi, 3); SB                                 \
    MF(a1, b1, 0); SB issue(xs_, ws_, bi, 4); rd_a(a0, bn, 0, 0); rd_a(a0, bn, 0, 1); rd_b(b0, bn, 0); SB \
    MF(a1, b1, 1); SB issue(xs_, ws_, bi, 5); rd_a(a0, bn, 0, 2); rd_a(a0, bn, 0, 3); SB      \
    MF(a1, b1, 2); SB                                                                         \
    MF(a1, b1, 3); SB                                                                         \
    STAGE_END(VM) }                                                                           \
    bc = bn; bn = bn == 5 ? 0 : bn + 1; bi = bi == 5 ? 0 : bi + 1;
#define DMA2_LOOP(MF, XL, VM) \
    for (int t0 = 0; t0 < T; t0 += 4) { DMA2_STAGE(MF, XL, VM, 0) DMA2_STAGE(MF, XL, VM, 1) DMA2_STAGE(MF, XL, VM, 2) DMA2_STAGE(MF, XL, VM, 3) }

    // only live row tiles are fetched; the count of loads a wave may leave in flight is per wave
    // and follows from how many X tiles it sends
    const int xl = max(0, min(2, mbs - 2 * wave));
#pragma unroll
    for (int st = 0; st < 5; ++st)
#pragma unroll
        for (int j = 0; j < 6; ++j)
            if (j >= 4 || (j >> 1) < xl) issue(x_base(st), w_base(st), st, j);
    int bc = 0, bn = 1, bi = 5;
    if (xl == 2) { STAGE_END(18) } else if (xl == 1) { STAGE_END(12) } else { STAGE_END(6) }   // stages 0 and 1 have landed
    a1 = Half{};
    b1 = BHalf{};
    rd_a(a0, 0, 0, 0); rd_a(a0, 0, 0, 1); rd_a(a0, 0, 0, 2); rd_a(a0, 0, 0, 3);
    rd_b(b0, 0, 0);
    // a wave that does not send both of its X tiles has fewer than 4 live row tiles
    if (xl == 0) { DMA2_LOOP(mf_some, 0, 6) }
    else if (xl == 1) { DMA2_LOOP(mf_some, 1, 12) }
    else if (cnt == 4) { DMA2_LOOP(mf_all, 2, 18) }
    else { DMA2_LOOP(mf_some, 2, 18) }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef DMA2_LOOP
#undef DMA2_STAGE
#undef STAGE_END
#undef SB
#define EPI_ROW(E, ARGS, I) \
    if (4 * wm + (I) < mbs) epilogue_tile<E>(ARGS, acc[I][0], acc[I][1], row_base + 32 * (4 * wm + (I)), n, nbw, lane);
    if (splits > 1) {
        EpiArgs pe = ep;
        pe.out = partial + (int64_t)sp * part_plane;
        pe.ldo = part_ld;
        EPI_ROW(EPI_STORE, pe, 0) EPI_ROW(EPI_STORE, pe, 1) EPI_ROW(EPI_STORE, pe, 2) EPI_ROW(EPI_STORE, pe, 3)
        return;
    }
    EPI_ROW(EPI, ep, 0) EPI_ROW(EPI, ep, 1) EPI_ROW(EPI, ep, 2) EPI_ROW(EPI, ep, 3)
#undef EPI_ROW
}

// ------------------------------------------------------------------ 256-column tile, two waves per SIMD
// 256 rows x 256 columns per workgroup, eight waves (2 x 4): wave (wm, wn) owns rows
// 128 wm .. +127 and columns 64 wn .. +63 (4 x 2 MFMA tiles, 128 accumulator registers), so two waves
// share a SIMD and one computes while the other waits at a barrier or for LDS (an MFMA-only
// kernel issues 10 % more per SIMD with two waves than with one; against four waves that own
// 8 x 2 tiles each, gate/up is 4-6 % faster at 160 to 512 rows and the same at 64).  Used for the
// products with many columns (gate/up with the SwiGLU epilogue, down, the K/V of skipped layers).  LDS: 5 stage buffers x 32 slots
// (X tile (row tile m, K half kk) at 2 m + kk, W tile (column tile nb of 8, K half kk) at
// 16 + 2 nb + kk) = all 160 KiB.  A wave sends 2 X and 2 W tiles per stage, four stages ahead, and
// may leave two stages in flight at the barrier: a load has two to three stages to land.
template <int EPI>
__global__ void __launch_bounds__(512, 2)
k_bf16_gemm_dma8(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int KB, int NBs, int nb_off,
                 int n_tiles, int splits, const int32_t* __restrict__ n_ptr, int B, float* __restrict__ partial,
                 int64_t part_plane, int part_ld, EpiArgs ep, ZBatch zb) {
    __shared__ uint4 lds[5][32][64];
    const int n = min(*n_ptr, B);
    int rg, unit;
    tile_of_block(n_tiles * splits, rg, unit);
    if (unit < 0) return;
    const int row_base = rg * 256;
    if (row_base >= n) return;
    if (zb.w_tab) Wp = reinterpret_cast<const uint4*>(zb.w_tab[zb.z0 + blockIdx.z]);
    Xp += (int64_t)blockIdx.z * zb.x_stride;
    ep.out += (int64_t)blockIdx.z * zb.out_stride;
    const int mbs = min(8, (n - row_base + 31) >> 5);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int cnt = max(0, min(4, mbs - 4 * wm));            // live 32-row tiles of this wave
    const int tile = unit / splits, sp = unit % splits;
    const int nbw = (tile * 4 + wn) * 2;                     // first of this wave's two tile-rows of W
    const int KS4 = KB >> 3;
    const int ks_lo = 4 * (int)(((int64_t)KS4 * sp) / splits), ks_hi = 4 * (int)(((int64_t)KS4 * (sp + 1)) / splits);
    const int T = ks_hi - ks_lo;                             // stages of this slice: a positive multiple of 4
    const uint4* xg = Xp + ((int64_t)rg * 8 * KB) * 64;
    const uint4* wg = Wp + (int64_t)(nb_off + tile * 8) * 64;   // the tile's eight tile-rows of W
    const unsigned lane_bytes = (unsigned)lane * 16u;
    const unsigned lds0 = (unsigned)(size_t)&lds[0][0][0];

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // j-th load of a stage: j = 0, 1 the X tile of row tile `wave`, K half j (sent only if that row
    // tile is live); j = 2, 3 the W tile of column tile `wave`, K half j - 2.  Address = the stage's base pointer (scalar, once per stage) plus a lane
    // offset that is the same in every stage.
    unsigned voff[4];
#pragma unroll
    for (int j = 0; j < 2; ++j) voff[j] = lane_bytes + ((unsigned)(min(wave, mbs - 1) * KB + j) << 10);
#pragma unroll
    for (int j = 2; j < 4; ++j) voff[j] = lane_bytes + ((unsigned)((j - 2) * NBs + wave) << 10);
    auto x_base = [&](int t) { return xg + (int64_t)(2 * (ks_lo + min(t, T - 1))) * 64; };
    auto w_base = [&](int t) { return wg + (int64_t)(2 * (ks_lo + min(t, T - 1))) * NBs * 64; };
    auto issue = [&](const uint4* xs, const uint4* ws, int buf, int j) {
        if (j < 2) dma_tile(xs, voff[j], lds0 + (unsigned)((buf * 32 + wave * 2 + j) << 10));
        else dma_tile<true>(ws, voff[j], lds0 + (unsigned)((buf * 32 + 16 + wave * 2 + (j - 2)) << 10));
    };
    Half a0, a1;
    BHalf b0, b1;
    auto rd_a = [&](Half& o, int buf, int kk, int i) { o.v[i] = (&lds[0][0][lane] + buf * (32 * 64))[((4 * wm + i) * 2 + kk) * 64]; };
    auto rd_b = [&](BHalf& o, int buf, int kk) {
        const uint4* p = &lds[0][0][lane] + buf * (32 * 64);
        o.v[0] = p[(16 + (2 * wn) * 2 + kk) * 64];
        o.v[1] = p[(16 + (2 * wn + 1) * 2 + kk) * 64];
    };
    auto mf_all = [&](const Half& a, const BHalf& bw, int i) {
        acc[i][0] = tile_mfma<EPI>(a.v[i], bw.v[0], acc[i][0]);
        acc[i][1] = tile_mfma<EPI>(a.v[i], bw.v[1], acc[i][1]);
    };
    auto mf_some = [&](const Half& a, const BHalf& bw, int i) {
        if (i < cnt) mf_all(a, bw, i);
    };
#define SB __builtin_amdgcn_sched_barrier(0);
// two stages of this wave's loads (VM of them) may stay in flight: everything up to stage t+2 has landed
#define STAGE_END(VM) asm volatile("s_waitcnt vmcnt(" #VM ") lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // bc / bn / bi: buffers of the current stage, the next one and the one being requested (stage + 4)
#define DMA8_STAGE(MF, XL, VM, U)                                                             \
    { const uint4* xs_ = x_base(t0 + (U) + 4); const uint4* ws_ = w_base(t0 + (U) + 4);       \
    MF(a0, b0, 0); SB if (XL) issue(xs_, ws_, bi, 0); rd_a(a1, bc, 1, 0); rd_a(a1, bc, 1, 1); rd_b(b1, bc, 1); SB \
    MF(a0, b0, 1); SB if (XL) issue(xs_, ws_, bi, 1); rd_a(a1, bc, 1, 2); rd_a(a1, bc, 1, 3); SB \
    MF(a0, b0, 2); SB                                                                         \
    MF(a0, b0, 3); SB                                                                         \
    MF(a1, b1, 0); SB issue(xs_, ws_, bi, 2); rd_a(a0, bn, 0, 0); rd_a(a0, bn, 0, 1); rd_b(b0, bn, 0); SB \
    MF(a1, b1, 1); SB issue(xs_, ws_, bi, 3); rd_a(a0, bn, 0, 2); rd_a(a0, bn, 0, 3); SB      \
    MF(a1, b1, 2); SB                                                                         \
    MF(a1, b1, 3); SB                                                                         \
    STAGE_END(VM) }                                                                           \
    bc = bn; bn = bn == 4 ? 0 : bn + 1; bi = bi == 4 ? 0 : bi + 1;
#define DMA8_LOOP(MF, XL, VM) \
    for (int t0 = 0; t0 < T; t0 += 4) { DMA8_STAGE(MF, XL, VM, 0) DMA8_STAGE(MF, XL, VM, 1) DMA8_STAGE(MF, XL, VM, 2) DMA8_STAGE(MF, XL, VM, 3) }

    // only live row tiles are fetched: wave w sends the X tiles of row tile w if there is one, and
    // the count of loads it may leave in flight follows (the counter is per wave)
    const bool sends_x = wave < mbs;
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j >= 2 || sends_x) issue(x_base(st), w_base(st), st, j);
    int bc = 0, bn = 1, bi = 4;
    if (sends_x) { STAGE_END(8) } else { STAGE_END(4) }   // stages 0 and 1 have landed
    a1 = Half{};
    b1 = BHalf{};
    rd_a(a0, 0, 0, 0); rd_a(a0, 0, 0, 1); rd_a(a0, 0, 0, 2); rd_a(a0, 0, 0, 3);
    rd_b(b0, 0, 0);
    if (!sends_x) { DMA8_LOOP(mf_some, false, 4) }         // such a wave has fewer than 4 live tiles
    else if (cnt == 4) { DMA8_LOOP(mf_all, true, 8) }
    else { DMA8_LOOP(mf_some, true, 8) }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef DMA8_LOOP
#undef DMA8_STAGE
#undef STAGE_END
#undef SB
#define EPI_ROW(E, ARGS, I) \
    if (4 * wm + (I) < mbs) epilogue_tile<E>(ARGS, acc[I][0], acc[I][1], row_base + 32 * (4 * wm + (I)), n, nbw, lane);
    if (splits > 1) {
        EpiArgs pe = ep;
        pe.out = partial + (int64_t)sp * part_plane;
        pe.ldo = part_ld;
        EPI_ROW(EPI_STORE, pe, 0) EPI_ROW(EPI_STORE, pe, 1) EPI_ROW(EPI_STORE, pe, 2) EPI_ROW(EPI_STORE, pe, 3)
        return;
    }
    EPI_ROW(EPI, ep, 0) EPI_ROW(EPI, ep, 1) EPI_ROW(EPI, ep, 2) EPI_ROW(EPI, ep, 3)
#undef EPI_ROW
}

// ------------------------------------------------------------------ tile of 192 columns
// k_bf16_gemm_cols<EPI, NT>: 256 rows x 32 NT columns per workgroup (NT = 5 .. 7; 6 is used), for products whose
// column tiles fill the 256 CUs badly at 128 or 256 columns (gate/up of the 34B shape has 1376
// tile-rows: 344 workgroups of 4 take two rounds, 172 of 8 leave a third of the CUs idle, 230 of 6 run
// in one round).  Same operand path, staging and waits as k_bf16_gemm_dma8, same wave layout: wave
// (wm, wn) = (w / 4, w % 4) owns row tiles 4 wm .. 4 wm + 3, and the NT column tiles are dealt out
// over wn (the four SIMDs) as evenly as they go, one or two each, so that whatever the number of
// live row tiles every SIMD with the same number of column tiles carries the same MFMA work.  LDS: 5
// stage buffers of 32 slots, X tile (row tile m, K half kk) at 2 m + kk, W tile (column tile nb, K half
// kk) at 16 + 2 nb + kk; wave w sends the X tiles of row tile w (if live) and the W tiles of column
// tile w (if w < NT), four stages ahead.  The last workgroup of a product whose tile-rows are no
// multiple of NT re-reads its last tile-row in place of the missing ones and drops their results.
struct ColsCtx {
    uint4*       lds;        // [5][32][64]
    const uint4* xg;
    const uint4* wg;
    int KB, NBs, ks_lo, T, mbs, nt_live, wave, lane, row_base, n, nb0;
};

template <int EPI, int NT, int NC>
__device__ __forceinline__ void cols_wave(const ColsCtx& c, const int c0, const EpiArgs& ep) {
    const int wave = c.wave, lane = c.lane, wm = wave >> 2;
    const int cnt = max(0, min(4, c.mbs - 4 * wm));           // live row tiles among 4 wm .. 4 wm + 3
    const unsigned lane_bytes = (unsigned)lane * 16u;
    const unsigned lds0 = (unsigned)(size_t)c.lds;
    const bool sends_x = wave < c.mbs, sends_w = wave < NT;

    floatx16 acc[4][NC];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NC; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // j-th load of a stage: j = 0, 1 the X tile of row tile `wave`, K half j; j = 2, 3 the W tile of
    // column tile `wave`, K half j - 2.  Address = the stage's base pointer (scalar, once per stage)
    // plus a lane offset that is the same in every stage.
    unsigned voff[4];
#pragma unroll
    for (int j = 0; j < 2; ++j) voff[j] = lane_bytes + ((unsigned)(min(wave, c.mbs - 1) * c.KB + j) << 10);
#pragma unroll
    for (int j = 2; j < 4; ++j) voff[j] = lane_bytes + ((unsigned)((j - 2) * c.NBs + min(wave, c.nt_live - 1)) << 10);
    auto x_base = [&](int t) { return c.xg + (int64_t)(2 * (c.ks_lo + min(t, c.T - 1))) * 64; };
    auto w_base = [&](int t) { return c.wg + (int64_t)(2 * (c.ks_lo + min(t, c.T - 1))) * c.NBs * 64; };
    auto issue = [&](const uint4* xs, const uint4* ws, int buf, int j) {
        if (j < 2) dma_tile(xs, voff[j], lds0 + (unsigned)((buf * 32 + wave * 2 + j) << 10));
        else dma_tile<true>(ws, voff[j], lds0 + (unsigned)((buf * 32 + 16 + wave * 2 + (j - 2)) << 10));
    };
    uint4 a[2][4], b[2][NC];                                  // [K half][row tile], [K half][column tile]
    auto slot = [&](int buf, int s_) { return (c.lds + lane + buf * (32 * 64))[s_ * 64]; };
    auto rd_a = [&](int buf, int kk, int i) { a[kk][i] = slot(buf, (4 * wm + i) * 2 + kk); };
    auto rd_b = [&](int buf, int kk, int j) { b[kk][j] = slot(buf, 16 + (c0 + j) * 2 + kk); };

    int bc = 0, bn = 1, bi = 4;   // buffers of the current stage, the next one and the one being requested (stage + 4)
    // One stage: the MFMAs of K half 0 while K half 1 is read from LDS and the X tiles of stage + 4 are
    // requested, then those of K half 1 while K half 0 of the next stage is read and the W tiles are
    // requested; the loads are issued one behind an MFMA group each.  Two stages of this wave's loads
    // may stay in flight at the barrier: everything up to stage + 2 has landed.
    auto stage = [&](auto xl_, auto wl_, auto all_, int t_req) {
        constexpr bool XL = decltype(xl_)::value, WL = decltype(wl_)::value, ALL = decltype(all_)::value;
        const uint4* xs = x_base(t_req);
        const uint4* ws = w_base(t_req);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int rb = kk == 0 ? bc : bn;                 // buffer the other K half is read from
            const int ok = 1 - kk;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (ALL || g < cnt) {
#pragma unroll
                    for (int j = 0; j < NC; ++j) acc[g][j] = tile_mfma<EPI>(a[kk][g], b[kk][j], acc[g][j]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (g == 0) {
                    if (kk == 0 ? XL : WL) issue(xs, ws, bi, 2 * kk);
                    rd_a(rb, ok, 0); rd_a(rb, ok, 1); rd_b(rb, ok, 0);
                    if (NC > 1) rd_b(rb, ok, 1);
                } else if (g == 1) {
                    if (kk == 0 ? XL : WL) issue(xs, ws, bi, 2 * kk + 1);
                    rd_a(rb, ok, 2); rd_a(rb, ok, 3);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * (2 * (XL ? 1 : 0) + 2 * (WL ? 1 : 0))) : "memory");
        bc = bn; bn = bn == 4 ? 0 : bn + 1; bi = bi == 4 ? 0 : bi + 1;
    };
    auto slice = [&](auto xl_, auto wl_, auto all_) {
        constexpr bool XL = decltype(xl_)::value, WL = decltype(wl_)::value;
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < 2 ? XL : WL) issue(x_base(st), w_base(st), st, j);
        // stages 0 and 1 have landed
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * (2 * (XL ? 1 : 0) + 2 * (WL ? 1 : 0))) : "memory");
#pragma unroll
        for (int i = 0; i < 4; ++i) { rd_a(0, 0, i); a[1][i] = a[0][i]; }
#pragma unroll
        for (int j = 0; j < NC; ++j) { rd_b(0, 0, j); b[1][j] = b[0][j]; }
        for (int t0 = 0; t0 < c.T; t0 += 4) {
            stage(xl_, wl_, all_, t0 + 4); stage(xl_, wl_, all_, t0 + 5); stage(xl_, wl_, all_, t0 + 6); stage(xl_, wl_, all_, t0 + 7);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    using Yes = std::true_type;
    using No = std::false_type;
    // the count of loads a wave may leave in flight is per wave and follows from what it sends, so each
    // combination runs its own copy of the loop; a wave whose four row tiles are live (the common case)
    // runs a copy without the live-tile test
    const bool all = cnt == 4;
    if (sends_x && sends_w) { if (all) slice(Yes{}, Yes{}, Yes{}); else slice(Yes{}, Yes{}, No{}); }
    else if (sends_x)       { if (all) slice(Yes{}, No{}, Yes{});  else slice(Yes{}, No{}, No{}); }
    else if (sends_w)       { slice(No{}, Yes{}, No{}); }
    else                    { slice(No{}, No{}, No{}); }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i >= cnt) continue;
#pragma unroll
        for (int j = 0; j < NC; ++j)
            if (c0 + j < c.nt_live)
                epilogue_one<EPI>(ep, acc[i][j], c.row_base + 32 * (4 * wm + i), c.n, c.nb0 + c0 + j, lane);
    }
}

template <int EPI, int NT>
__global__ void __launch_bounds__(512, 2)
k_bf16_gemm_cols(const uint4* __restrict__ Xp, const uint4* __restrict__ Wp, int KB, int NBs, int nb_off, int NB_total,
                 int n_tiles, const int32_t* __restrict__ n_ptr, int B, EpiArgs ep) {
    static_assert(NT >= 5 && NT <= 7, "column tiles per workgroup");
    __shared__ uint4 lds[5][32][64];
    const int n = min(*n_ptr, B);
    int rg, tile;
    tile_of_block(n_tiles, rg, tile);
    if (tile < 0) return;
    const int row_base = rg * 256;
    if (row_base >= n) return;
    ColsCtx c;
    c.lds = &lds[0][0][0];
    c.KB = KB; c.NBs = NBs;
    c.ks_lo = 0;
    c.T = KB >> 1;                                            // stages: a positive multiple of 4 (K is a multiple of 128)
    c.mbs = min(8, (n - row_base + 31) >> 5);
    c.nt_live = min(NT, NB_total - tile * NT);
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.lane = threadIdx.x & 63;
    c.row_base = row_base; c.n = n; c.nb0 = tile * NT;
    c.xg = Xp + ((int64_t)rg * 8 * KB) * 64;
    c.wg = Wp + (int64_t)(nb_off + tile * NT) * 64;            // the tile's NT tile-rows of W
    // column tiles of SIMD wn: two for wn < NT - 4, one for the others, in rising order
    const int wn = c.wave & 3;
    if (wn < NT - 4) cols_wave<EPI, NT, 2>(c, 2 * wn, ep);
    else cols_wave<EPI, NT, 1>(c, 2 * (NT - 4) + (wn - (NT - 4)), ep);
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
                   bf16_t* __restrict__ q_lo, int32_t* __restrict__ status, int64_t z_stride,
                   int32_t* __restrict__ order, int splits, int64_t plane) {
    int i = blockIdx.x;
    int n = min(*n_ptr, B);
    if (i >= n) return;
    buf += (int64_t)blockIdx.z * z_stride;     // several layers in one launch: blockIdx.z = layer offset
    kv.layer0 += blockIdx.z;
    int b = idx[i];
    int p = pos[b];
    if (order != nullptr && blockIdx.y == 0 && threadIdx.x < 64) {
        // launch order of the attention workgroups: list entries by falling context length (ties by
        // entry), so that the longest rows start first and the last wave of workgroups is short.
        // rank of this entry = how many entries come before it; the ranks form a permutation.
        int before = 0;
        for (int j = threadIdx.x; j < n; j += 64) {
            int pj = pos[idx[j]];
            before += (pj > p || (pj == p && j < i)) ? 1 : 0;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o, 64);
        if (threadIdx.x == 0) order[before] = i;
    }
    const int hd = 128, half = 64;
    int Hkv = kv.n_kv_heads;
    const int sq = kv_row(kv, b);
    int cap = kv.cap[sq];
    if (p < 0 || p >= cap || p >= max_pos) {
        if (threadIdx.x == 0) atomicOr(status, 1);
        return;
    }
    // buf holds `splits` K-slice planes of the product (plane floats apart): their sum in slice
    // order is the value; splits = 1 is a finished matrix
    const float* r0 = buf + (int64_t)i * ld;
    // four consecutive values at once (x is a multiple of 4: 16-byte loads from every plane)
    auto rd4 = [&](int x) -> float4 {
        float4 v = *reinterpret_cast<const float4*>(r0 + x);
        for (int q = 1; q < splits; ++q) {
            const float4 u = *reinterpret_cast<const float4*>(r0 + x + (int64_t)q * plane);
            v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
        }
        return v;
    };
    auto pack4 = [](float a, float b, float c, float d) -> uint2 {
        return make_uint2(f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16), f32_to_bf16(c) | ((uint32_t)f32_to_bf16(d) << 16));
    };
    const float* cs = rope + (int64_t)p * half * 2;
    // The work of a row, in items of four rotation pairs (q, k) or four values (v), is dealt out over
    // the threads of the gridDim.y blocks that share the row: items [0, nq4) rotate queries, the next
    // nk4 rotate and append keys, the last nv4 append values.
    const int nq4 = n_q * (half / 4), nk4 = Hkv * (half / 4), nv4 = Hkv * (hd / 4);
    const int kin = n_q * hd;
    const int vin = kin + Hkv * hd;
    for (int t = blockIdx.y * 256 + threadIdx.x; t < nq4 + nk4 + nv4; t += 256 * gridDim.y) {
        if (t < nq4 + nk4) {
            const bool is_q = t < nq4;
            const int u = is_q ? t : t - nq4;
            const int hh = u >> 4, j0 = (u & 15) * 4;                 // head, first of the four pairs
            const int x = (is_q ? 0 : kin) + hh * hd + j0;
            const float4 a = rd4(x), bb = rd4(x + half);
            const float4 cs0 = *reinterpret_cast<const float4*>(cs + 2 * j0);       // c0 s0 c1 s1
            const float4 cs1 = *reinterpret_cast<const float4*>(cs + 2 * j0 + 4);   // c2 s2 c3 s3
            const float x0[4] = {a.x * cs0.x - bb.x * cs0.y, a.y * cs0.z - bb.y * cs0.w,
                                 a.z * cs1.x - bb.z * cs1.y, a.w * cs1.z - bb.w * cs1.w};
            const float x1[4] = {bb.x * cs0.x + a.x * cs0.y, bb.y * cs0.z + a.y * cs0.w,
                                 bb.z * cs1.x + a.z * cs1.y, bb.w * cs1.z + a.w * cs1.w};
            if (is_q) {
                const int64_t o = ((int64_t)i * n_q + hh) * hd + j0;
                const uint2 h0 = pack4(x0[0], x0[1], x0[2], x0[3]), h1 = pack4(x1[0], x1[1], x1[2], x1[3]);
                *reinterpret_cast<uint2*>(q_hi + o) = h0;
                *reinterpret_cast<uint2*>(q_hi + o + half) = h1;
                float l0[4], l1[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    l0[k] = x0[k] - bf16_to_f32(f32_to_bf16(x0[k]));
                    l1[k] = x1[k] - bf16_to_f32(f32_to_bf16(x1[k]));
                }
                *reinterpret_cast<uint2*>(q_lo + o) = pack4(l0[0], l0[1], l0[2], l0[3]);
                *reinterpret_cast<uint2*>(q_lo + o + half) = pack4(l1[0], l1[1], l1[2], l1[3]);
            } else {
                // four consecutive features of a key sit side by side in the cache (same octet)
                bf16_t* base = reinterpret_cast<bf16_t*>(kv.pool) + kv_block(kv, sq, hh, cap);
                *reinterpret_cast<uint2*>(base + k_bf16_offset(p, j0, hd)) = pack4(x0[0], x0[1], x0[2], x0[3]);
                *reinterpret_cast<uint2*>(base + k_bf16_offset(p, j0 + half, hd)) = pack4(x1[0], x1[1], x1[2], x1[3]);
            }
        } else {
            const int u = t - nq4 - nk4;
            const int g = u >> 5, j0 = (u & 31) * 4;
            const float4 v = rd4(vin + g * hd + j0);
            bf16_t* base = reinterpret_cast<bf16_t*>(kv.pool) + kv_block(kv, sq, g, cap);
            base[v_bf16_offset(p, j0, hd)] = f32_to_bf16(v.x);
            base[v_bf16_offset(p, j0 + 1, hd)] = f32_to_bf16(v.y);
            base[v_bf16_offset(p, j0 + 2, hd)] = f32_to_bf16(v.z);
            base[v_bf16_offset(p, j0 + 3, hd)] = f32_to_bf16(v.w);
        }
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
template <bool PAIR>
__global__ void __launch_bounds__(256, PAIR ? 3 : 2)
k_bf16_attn(const bf16_t* __restrict__ q_hi, const bf16_t* __restrict__ q_lo, int Hq,
            const int32_t* __restrict__ idx, const int32_t* __restrict__ n_ptr, int B,
            const int32_t* __restrict__ pos, KvView kv, uint4* __restrict__ ao, int KB_ao, int n_splits,
            float* __restrict__ part, const int32_t* __restrict__ order) {
    __shared__ float sm_m[4][16];
    __shared__ float sm_l[4][16];
    __shared__ float sm_o[4][16][128];
    const int g = blockIdx.x;
    const int n = min(*n_ptr, B);
    const int G = Hq / kv.n_kv_heads;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n16 = lane & 15, gq = lane >> 4;
    // PAIR (context pass and other passes over list entries, 2 G <= 16): the workgroup serves the E = 16 / G
    // list entries E y .. E y + E - 1.  Consecutive entries that read the same cache row (a context passed
    // in rising position order) share its K/V stream: entry j of such a run has its G heads in the MFMA
    // columns G j .. G j + G - 1, each column masked at its own entry's position.  With one query head per
    // kv head 16 entries share a stream, with eight heads two.  A change of cache row inside the E entries
    // starts another run, served after the first.
    int first, cnt = 1;
    if (PAIR) {
        const int E = 16 / G;
        first = E * (int)blockIdx.y;
        if (first >= n) return;
        cnt = min(E, n - first);
    } else {
        if ((int)blockIdx.y >= n) return;
        first = order[blockIdx.y];            // longest contexts first
    }
    for (int r0 = 0; r0 < cnt;) {
    const int sq = kv_row(kv, idx[first + r0]);
    int r1 = r0 + 1;
    if (PAIR) while (r1 < cnt && kv_row(kv, idx[first + r1]) == sq) ++r1;
    const int n_col = (r1 - r0) * G;                       // live MFMA columns
    const int cap = kv.cap[sq];
    int n_pos = 1;                                         // positions read: the longest of the run
    for (int j = r0; j < r1; ++j) n_pos = max(n_pos, min(pos[idx[first + j]] + 1, cap));
    const int my_ent = n16 < n_col ? n16 / G : 0;          // this lane's column: entry, head, positions
    const int my_e = first + r0 + my_ent;
    const int my_head = n16 - my_ent * G;
    const int my_np = n16 < n_col ? max(1, min(pos[idx[my_e]] + 1, cap)) : 0;
    const bf16_t* Kb = reinterpret_cast<const bf16_t*>(kv.pool) + kv_block(kv, sq, g, cap);

    bf16x8 qh[4], ql[4];
    {
        uint4 z = make_uint4(0, 0, 0, 0);
        const int64_t qo = ((int64_t)my_e * Hq + (int64_t)g * G + my_head) * 128 + 8 * gq;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            qh[c] = as_bf16x8(n16 < n_col ? *reinterpret_cast<const uint4*>(q_hi + qo + 32 * c) : z);
            ql[c] = as_bf16x8(n16 < n_col ? *reinterpret_cast<const uint4*>(q_lo + qo + 32 * c) : z);
        }
    }
    const float inv_sqrt = 1.0f / sqrtf(128.0f);
    const float NEG = -1.0e30f;
    float m_run = NEG, l_run = 0.f;
    floatx4 O[8];
#pragma unroll
    for (int hb = 0; hb < 8; ++hb) O[hb] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_groups = (n_pos + 31) >> 5;
    // with n_splits > 1 this workgroup covers the blockIdx.z-th share of the position groups
    const int g_lo = (int)(((int64_t)n_groups * blockIdx.z) / n_splits);
    const int g_hi = (int)(((int64_t)n_groups * (blockIdx.z + 1)) / n_splits);
    // K and V tiles of one 32-position group as this lane holds them for the MFMAs
    struct KVTiles { uint4 k[2][4]; uint4 v[8]; };
    auto load_kv = [&](int t) -> KVTiles {
        KVTiles x;
        // K: two blocks of 16 positions; slice c of a block is 1 KiB, lane l takes bytes 16 l ..
        const bf16_t* k0 = Kb + (int64_t)t * 8192 + lane * 8;      // the group's 16 KiB: K blocks, then V
        const bf16_t* k1 = k0 + 2048;
        const bf16_t* vg = k0 + 4096;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            x.k[0][c] = load_nt(reinterpret_cast<const uint4*>(k0 + 512 * c));
            x.k[1][c] = load_nt(reinterpret_cast<const uint4*>(k1 + 512 * c));
        }
#pragma unroll
        for (int hb = 0; hb < 8; ++hb) x.v[hb] = load_nt(reinterpret_cast<const uint4*>(vg + hb * 512));
        return x;
    };
    // Decode: a wave asks for its next group before it works on the current one (two workgroups per
    // CU then; against three workgroups that load and compute in turn: -2..4 % from 64 to 192 rows,
    // equal at 256).  Context pass with two entries per workgroup: three workgroups, no prefetch
    // (0.8 % faster there).
    KVTiles nxt;
    if constexpr (!PAIR) nxt = load_kv(min(g_lo + w, max(g_hi - 1, 0)));   // a group this workgroup's row has
    for (int t = g_lo + w; t < g_hi; t += 4) {
        const int p0 = t << 5;
        KVTiles cur;
        if constexpr (PAIR) {
            cur = load_kv(t);
        } else {
            cur = nxt;
            if (t + 4 < g_hi) nxt = load_kv(t + 4);
        }
        floatx4 S0 = {0.f, 0.f, 0.f, 0.f}, S1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            bf16x8 a0 = as_bf16x8(cur.k[0][c]);
            bf16x8 a1 = as_bf16x8(cur.k[1][c]);
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
            s[r]     = (p0 + 4 * gq + r < my_np) ? S0[r] * inv_sqrt : NEG;
            s[4 + r] = (p0 + 16 + 4 * gq + r < my_np) ? S1[r] * inv_sqrt : NEG;
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
#pragma unroll
        for (int hb = 0; hb < 8; ++hb) {
            uint4 vv = cur.v[hb];
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
        const int head = threadIdx.x >> 4, c0 = (threadIdx.x & 15) * 8;     // head = MFMA column
        if (head < n_col) {
            const int i = first + r0 + head / G;
            const int hq = head % G;
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
                o[j] = acc;
            }
            if (n_splits == 1) {
                uint4 pk = make_uint4(pack2(o[0] / Lsum, o[1] / Lsum), pack2(o[2] / Lsum, o[3] / Lsum),
                                      pack2(o[4] / Lsum, o[5] / Lsum), pack2(o[6] / Lsum, o[7] / Lsum));
                int col = (g * G + hq) * 128 + c0;
                ao[afrag_chunk(i, col, KB_ao)] = pk;
            } else {
                // unnormalised share: [i][kv head][split][head][130] = 128 features, max, sum
                float* p = part + ((((int64_t)i * kv.n_kv_heads + g) * n_splits + blockIdx.z) * 16 + hq) * 130;
#pragma unroll
                for (int j = 0; j < 8; ++j) p[c0 + j] = o[j];
                if (c0 == 0) { p[128] = M; p[129] = Lsum; }
            }
        }
    }
    r0 = r1;
    if (r0 < cnt) __syncthreads();         // the merge has read the shared arrays before the next run writes them
    }
}

// merges the position shares of k_bf16_attn in share order: one workgroup per (kv head, list entry)
__global__ void __launch_bounds__(256)
k_bf16_attn_merge(const float* __restrict__ part, int Hq, int Hkv, int n_splits, const int32_t* __restrict__ n_ptr,
                  int B, uint4* __restrict__ ao, int KB_ao) {
    const int g = blockIdx.x, i = blockIdx.y;
    const int n = min(*n_ptr, B);
    if (i >= n) return;
    const int G = Hq / Hkv;
    const int head = threadIdx.x >> 4, c0 = (threadIdx.x & 15) * 8;
    if (head >= G) return;
    const float* base = part + (((int64_t)i * Hkv + g) * n_splits * 16 + head) * 130;
    float M = -1.0e30f;
    for (int q = 0; q < n_splits; ++q) M = fmaxf(M, base[(int64_t)q * 16 * 130 + 128]);
    float L = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int q = 0; q < n_splits; ++q) {
        const float* p = base + (int64_t)q * 16 * 130;
        float wq = __expf(p[128] - M);
        L += p[129] * wq;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] += p[c0 + j] * wq;
    }
    uint4 pk = make_uint4(pack2(o[0] / L, o[1] / L), pack2(o[2] / L, o[3] / L), pack2(o[4] / L, o[5] / L),
                          pack2(o[6] / L, o[7] / L));
    ao[afrag_chunk(i, (g * G + head) * 128 + c0, KB_ao)] = pk;
}

// ------------------------------------------------------------------ host side
static KvView make_view(const ee_model* m, const ee_kv* kv, int layer, const ee_batch* b) {
    return KvView{kv->pool, kv->d_cap, kv->d_off, kv->T, m->cfg.n_kv_heads, m->cfg.head_dim, layer - 1, b->kv_seq};
}

template <int MS, int NS, int WK, int WN, int EPI>
static void gemm_launch(const void* X, const void* W, int K, int NB_total, int NBs, int nb_off, const int32_t* n_ptr,
                        int B, int row_groups, const EpiArgs& ep, hipStream_t s, const ZBatch& zb, int nz) {
    dim3 grid((NB_total + WN * NS - 1) / (WN * NS), row_groups, nz);
    hipLaunchKernelGGL((k_bf16_gemm<MS, NS, WK, WN, EPI>), grid, dim3(64 * WK * WN), 0, s, (const uint4*)X,
                       (const uint4*)W, K / 16, NB_total, NBs, nb_off, n_ptr, B, ep, zb);
}

// picks the tile configuration from the row capacity of the batch
template <int NS, int EPI>
static void gemm(const void* X, const void* W, int N, int K, int NBs, int nb_off, const int32_t* n_ptr, int B,
                 const EpiArgs& ep, hipStream_t s, const ZBatch& zb = ZBatch{}, int nz = 1) {
    int NB = N / 32;
    int Mpad = (B + 31) / 32 * 32;
    if (Mpad <= 32)       gemm_launch<1, NS, 8, 1, EPI>(X, W, K, NB, NBs, nb_off, n_ptr, B, 1, ep, s, zb, nz);
    else if (Mpad <= 64)  gemm_launch<2, NS, 8, 1, EPI>(X, W, K, NB, NBs, nb_off, n_ptr, B, 1, ep, s, zb, nz);
    else if (Mpad <= 128) gemm_launch<4, NS, 2, 2, EPI>(X, W, K, NB, NBs, nb_off, n_ptr, B, 1, ep, s, zb, nz);
    else                  gemm_launch<8, NS, 1, 4, EPI>(X, W, K, NB, NBs, nb_off, n_ptr, B, (Mpad + 255) / 256, ep, s, zb, nz);
}

// Adds the K-slice planes in slice order and applies the epilogue: plain store, or
// residual update h[row id] += sum.  One thread per 4 consecutive columns.
template <int EPI>
__global__ void __launch_bounds__(256)
k_splitk_finish(const float* __restrict__ partial, int64_t plane, int ld, int splits, int N,
                const int32_t* __restrict__ n_ptr, int B, EpiArgs ep) {
    const int n = min(*n_ptr, B);
    const int row = blockIdx.y;
    if (row >= n) return;
    const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (col >= N) return;
    const float* p = partial + (int64_t)row * ld + col;
    float4 sum = *reinterpret_cast<const float4*>(p);
    for (int q = 1; q < splits; ++q) {
        float4 v = *reinterpret_cast<const float4*>(p + (int64_t)q * plane);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    if (EPI == EPI_STORE) {
        *reinterpret_cast<float4*>(ep.out + (int64_t)row * ep.ldo + col) = sum;
    } else {
        float4* h = reinterpret_cast<float4*>(ep.out + (int64_t)ep.idx[row] * ep.ldo + col);
        float4 o = *h;
        o.x += sum.x; o.y += sum.y; o.z += sum.z; o.w += sum.w;
        *h = o;
    }
}

// Residual finish of a K-sliced product, one block per list entry: h[row id] += sum of the
// slice planes (in slice order, as k_splitk_finish does), and, if a gain is given, the RMSNorm
// of the updated row straight into the operand matrix of the next product.
__global__ void __launch_bounds__(NORM_THREADS)
k_splitk_resid_norm(const float* __restrict__ partial, int64_t plane, int ld, int splits, int N,
                    const int32_t* __restrict__ n_ptr, int B, float* h, int ldh, const int32_t* __restrict__ idx,
                    const float* gain, float eps, uint4* xout) {
    __shared__ float red[NORM_THREADS / 64];
    const int n = min(*n_ptr, B);
    const int i = blockIdx.x;
    if (i >= n) return;
    float* hrow = h + (int64_t)idx[i] * ldh;
    const float* prow = partial + (int64_t)i * ld;
    if ((N >> 3) <= NORM_THREADS) {
        // at most one 8-float chunk per thread (d <= 8192): the updated chunk stays in registers for
        // the norm instead of being read back twice; same arithmetic, same bits as the general path
        const int c = threadIdx.x;
        const bool has = c < (N >> 3);
        float4 o0 = make_float4(0.f, 0.f, 0.f, 0.f), o1 = o0;
        if (has) {
            const float* p = prow + c * 8;
            float4 s0 = *reinterpret_cast<const float4*>(p), s1 = *reinterpret_cast<const float4*>(p + 4);
#pragma unroll 4
            for (int q = 1; q < splits; ++q) {
                const float4 v0 = *reinterpret_cast<const float4*>(p + (int64_t)q * plane);
                const float4 v1 = *reinterpret_cast<const float4*>(p + (int64_t)q * plane + 4);
                s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
                s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
            }
            float4* hp = reinterpret_cast<float4*>(hrow + c * 8);
            o0 = hp[0]; o1 = hp[1];
            o0.x += s0.x; o0.y += s0.y; o0.z += s0.z; o0.w += s0.w;
            o1.x += s1.x; o1.y += s1.y; o1.z += s1.z; o1.w += s1.w;
            hp[0] = o0; hp[1] = o1;
        }
        if (gain == nullptr) return;
        float ss = 0.f;
        if (has) ss += o0.x * o0.x + o0.y * o0.y + o0.z * o0.z + o0.w * o0.w + o1.x * o1.x + o1.y * o1.y + o1.z * o1.z + o1.w * o1.w;
        ss = block_sum<NORM_THREADS>(ss, red);
        const float inv = 1.0f / sqrtf(ss / (float)N + eps);
        if (has) {
            const float4* g4 = reinterpret_cast<const float4*>(gain);
            const float4 ga = g4[2 * c], gb = g4[2 * c + 1];
            uint4 o;
            o.x = pack2((o0.x * inv) * ga.x, (o0.y * inv) * ga.y);
            o.y = pack2((o0.z * inv) * ga.z, (o0.w * inv) * ga.w);
            o.z = pack2((o1.x * inv) * gb.x, (o1.y * inv) * gb.y);
            o.w = pack2((o1.z * inv) * gb.z, (o1.w * inv) * gb.w);
            xout[afrag_chunk(i, c * 8, N >> 4)] = o;
        }
        return;
    }
    for (int c = threadIdx.x; c < (N >> 3); c += NORM_THREADS) {
        const float* p = prow + c * 8;
        float4 s0 = *reinterpret_cast<const float4*>(p), s1 = *reinterpret_cast<const float4*>(p + 4);
#pragma unroll 4
        for (int q = 1; q < splits; ++q) {
            const float4 v0 = *reinterpret_cast<const float4*>(p + (int64_t)q * plane);
            const float4 v1 = *reinterpret_cast<const float4*>(p + (int64_t)q * plane + 4);
            s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
            s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
        }
        float4* hp = reinterpret_cast<float4*>(hrow + c * 8);
        float4 o0 = hp[0], o1 = hp[1];
        o0.x += s0.x; o0.y += s0.y; o0.z += s0.z; o0.w += s0.w;
        o1.x += s1.x; o1.y += s1.y; o1.z += s1.z; o1.w += s1.w;
        hp[0] = o0; hp[1] = o1;
    }
    if (gain != nullptr) rmsnorm_row(hrow, gain, eps, N, xout, i, red);   // reads back this thread's own chunks
}

// what the caller wants done with the K-slice planes of a product
struct SliceTail {
    const float* norm_gain = nullptr;   // RESID: also normalise the updated rows with this gain ...
    float        eps = 0.f;
    uint4*       norm_out = nullptr;    // ... into this operand matrix
    bool*        norm_done = nullptr;   // set when that happened
    bool         defer_store = false;   // STORE: leave the planes to the caller ...
    int*         splits_out = nullptr;  // ... who gets their number (1 = the result is in out already)
};

// the 256-row tile kernels, 128 or 256 columns wide, K sliced so that about one workgroup per CU
// runs; returns false where the weight-streaming kernel is the better choice
template <int EPI>
static bool gemm_tiled(const ee_batch* b, const void* X, const void* W, int N, int K, int NBs, int nb_off,
                     const int32_t* n_ptr, int B, const EpiArgs& ep, hipStream_t s, const ZBatch& zb = ZBatch{},
                     int nz = 1, const SliceTail& tail = SliceTail{}) {
    if (N % 128 != 0 || K % 128 != 0) return false;
    // One product at a time: the tile kernels at every batch size (at 1 to 32 rows, measured on the
    // 70B shapes against the weight-streaming kernel plus the normalisation launch that the finish of
    // a sliced product saves: QKV 36 against 46 us, O 34 against 37, down 84 against 87, exit head 94
    // against 95-100, and 99 against 149 at 64 rows).  Several layers in one launch (K/V of skipped
    // layers): from 65 rows up.
    if (nz > 1 && B < 65) return false;
    int row_groups = (B + 255) / 256;
    int Mpad = (B + 31) / 32 * 32;
    int KS = K / 32;
    // the 256-column tile loads each activation tile once per 256 columns instead of once per 128;
    // worth it when it still gives every CU a workgroup, or when K is long enough that a deeper K
    // slicing costs little
    // (long K: with more than 128 rows the 256-column tile's halved activation traffic outweighs its
    // doubled K-slice planes; up to 128 rows the 128-column tile is 2-8 % faster on the down projection)
    bool wide = (N % 256 == 0) && ((N / 256) * row_groups * nz >= 200 || (EPI == EPI_RESID && K >= 2 * N && Mpad > 128));
    // K slices of a narrow product when the launch is left to itself: about one workgroup per CU
    auto slices_for = [&](int tiles) {
        int sp = (256 + tiles / 2) / tiles;
        // rounding up may push the launch past one round of 256 workgroups (96 column tiles x 3 slices):
        // one slice fewer then runs in a single round with longer slices and one plane less
        while (sp > 1 && tiles * sp > 256 && tiles * (sp - 1) >= 176) --sp;
        return sp;
    };
    auto fit_slices = [&](int sp) {
        while (sp > 1 && KS / sp < 16) --sp;               // every slice keeps at least 16 K steps (> 4)
        while (sp > 1 && (size_t)sp * Mpad * N * sizeof(float) > b->W.gemm_part_bytes) --sp;
        return sp;
    };
    const bool sliceable = (EPI == EPI_STORE || EPI == EPI_RESID) && nz == 1;
    int splits = 0;                                        // 0: not decided yet
    if (!wide && N % 256 == 0 && row_groups >= 2 && nz == 1) {
        // several row groups (context pass, batches above 256): the products are bound by the MFMAs and by
        // what a CU can pull from L2, and the 256-column tile moves a quarter less per MFMA issued
        const int ww = (N / 256) * row_groups, wn = (N / 128) * row_groups;
        auto fill = [](int wgs) { return (float)wgs / (float)((wgs + 255) / 256 * 256); };
        if (sliceable && ww <= 256) {
            // a product that may be K-sliced: the 256-column tile with as many slices (at most 4) as keep
            // it inside one round of workgroups, against the 128-column tile with the slices it would get
            // below; ties go to the 256-column tile unless it needs 4 planes for it.  (70B shape, context
            // pass, per launch with the kernel that adds the planes: QKV at 512 entries 134 -> 104 us, at
            // 1024 entries 219 -> 198 us; O projection at 768 entries 158 -> 124 us, at 1024 168 -> 148 us.)
            const int s_w = fit_slices(std::min(4, 256 / ww));
            const int s_n = fit_slices(wn < 200 ? slices_for(wn) : 1);
            const float f_w = fill(ww * s_w), f_n = fill(wn * s_n);
            wide = f_w > f_n || (f_w == f_n && s_w < 4);
            splits = wide ? s_w : s_n;
        } else {
            wide = fill(ww) >= fill(wn);
        }
    }
    if constexpr (EPI == EPI_SWIGLU) if (row_groups == 1 && nz == 1) {
        // one row group (decode; with several the product is MFMA bound and the rule above stands).
        // Tile width for the widest product: 256, 192 or 128 columns, whichever makes the column tiles cost
        // the fewest rounds of 256 workgroups times the tile's width (what a round costs a CU in operand
        // traffic); ties go to the wider tile, which re-reads the activations less often.  (224 columns
        // were measured too, for the 70B shape's 1792 tile-rows = 256 x 7: within 2 % of 256 columns.)
        const int NB = N / 32;
        int nt = 4, best = 1 << 30;
        for (int t = 8; t >= 4; t -= 2) {
            if (t == 8 && N % 256 != 0) continue;
            const int wgs = (NB + t - 1) / t * row_groups * nz, cost = (wgs + 255) / 256 * t;
            if (cost < best) { best = cost; nt = t; }
        }
        if (nt == 6) {
            const int n_tiles = (NB + 5) / 6;
            dim3 grid(n_tiles, 1, 1);
            hipLaunchKernelGGL((k_bf16_gemm_cols<EPI, 6>), grid, dim3(512), 0, s, (const uint4*)X, (const uint4*)W, K / 16,
                               NBs, nb_off, NB, n_tiles, n_ptr, B, ep);
            if (tail.splits_out) *tail.splits_out = 1;
            return true;
        }
        wide = nt == 8;
    }
    int n_tiles = wide ? N / 256 : N / 128;
    if (splits == 0) splits = sliceable && n_tiles * row_groups < 200 ? fit_slices(slices_for(n_tiles * row_groups)) : 1;
    dim3 grid(n_tiles * splits, row_groups, nz);
    if (row_groups > 1) grid = dim3((n_tiles * splits + 7) / 8 * 8 * row_groups, 1, nz);   // see tile_of_block
    if (wide)
        hipLaunchKernelGGL((k_bf16_gemm_dma8<EPI>), grid, dim3(512), 0, s, (const uint4*)X, (const uint4*)W,
                           K / 16, NBs, nb_off, n_tiles, splits, n_ptr, B, b->wsp<float>(b->W.gemm_part),
                           (int64_t)Mpad * N, N, ep, zb);
    else
        hipLaunchKernelGGL((k_bf16_gemm_dma2<EPI>), grid, dim3(BIG_THREADS), 0, s, (const uint4*)X, (const uint4*)W,
                           K / 16, NBs, nb_off, n_tiles, splits, n_ptr, B, b->wsp<float>(b->W.gemm_part),
                           (int64_t)Mpad * N, N, ep, zb);
    if (tail.splits_out) *tail.splits_out = splits;
    if (splits > 1) {
        if (EPI == EPI_RESID) {
            hipLaunchKernelGGL(k_splitk_resid_norm, dim3(B), dim3(NORM_THREADS), 0, s, b->wsp<float>(b->W.gemm_part),
                               (int64_t)Mpad * N, N, splits, N, n_ptr, B, ep.out, ep.ldo, ep.idx, tail.norm_gain,
                               tail.eps, tail.norm_out);
            if (tail.norm_gain && tail.norm_done) *tail.norm_done = true;
        } else if (!tail.defer_store) {
            hipLaunchKernelGGL((k_splitk_finish<EPI_STORE>), dim3((N / 4 + 255) / 256, B), dim3(256), 0, s,
                               b->wsp<float>(b->W.gemm_part), (int64_t)Mpad * N, N, splits, N, n_ptr, B, ep);
        }
    }
    return true;
}

// x_ready: the operand matrix already holds RMSNorm(h; attention gain of this layer).
// tail_gain (with x_done): if the last product of the layer is finished from K-slice planes, that
// kernel also leaves RMSNorm(h; tail_gain) in the operand matrix and sets *x_done.
int bf16_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, hipStream_t s, bool x_ready,
                       const float* tail_gain, bool* x_done) {
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
    KvView view = make_view(m, kv, layer, b);

    if (!x_ready) {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(NORM_THREADS), 0, s, h, idx, n_ptr, B, w.g_attn, c.rms_eps, d, x, ZBatch{});
    }
    EpiArgs e1{};
    e1.out = qkv; e1.ldo = qkv_n; e1.idx = idx;
    int qkv_splits = 1;
    {
        TimedScope t(EE_K_GEMM_QKV, s);
        SliceTail st;                  // K-slice planes of q|k|v are added up by the RoPE kernel
        st.defer_store = true; st.splits_out = &qkv_splits;
        if (!gemm_tiled<EPI_STORE>(b, x, w.w_qkv, qkv_n, d, qkv_n / 32, 0, n_ptr, B, e1, s, ZBatch{}, 1, st))
            gemm<1, EPI_STORE>(x, w.w_qkv, qkv_n, d, qkv_n / 32, 0, n_ptr, B, e1, s);
    }
    {
        TimedScope t(EE_K_ROPE_APPEND, s);
        const float* src = qkv_splits > 1 ? b->wsp<float>(b->W.gemm_part) : qkv;
        hipLaunchKernelGGL(k_bf16_rope_append, dim3(B, 4), dim3(256), 0, s, src, qkv_n, c.n_q_heads, idx, n_ptr, B,
                           b->st<int32_t>(L.pos), m->d_rope, c.max_pos, view, b->wsp<bf16_t>(b->W.q_hi),
                           b->wsp<bf16_t>(b->W.q_lo), b->st<int32_t>(L.status), (int64_t)0,
                           b->wsp<int32_t>(b->W.attn_order), qkv_splits, (int64_t)b->Mpad * qkv_n);
    }
    {
        TimedScope t(EE_K_ATTENTION, s);
        // few (row, kv head) pairs: also split the positions, so that the chip has workgroups to run
        int pairs = c.n_kv_heads * B;
        int n_splits = pairs >= 512 ? 1 : (1024 + pairs - 1) / pairs;
        if (n_splits > 16) n_splits = 16;
        while (n_splits > 1 && (size_t)b->Mpad * c.n_kv_heads * n_splits * 16 * 130 * 4 > b->W.attn_part_bytes) --n_splits;
        // context pass: 16 / G entries per workgroup, which share the K/V stream where they sit in the same cache row
        const int G = c.n_q_heads / c.n_kv_heads;
        const bool pair = b->kv_seq != nullptr && n_splits == 1 && 2 * G <= 16;
        if (pair)
            hipLaunchKernelGGL(k_bf16_attn<true>, dim3(c.n_kv_heads, (B + 16 / G - 1) / (16 / G), 1), dim3(256), 0, s, b->wsp<bf16_t>(b->W.q_hi),
                               b->wsp<bf16_t>(b->W.q_lo), c.n_q_heads, idx, n_ptr, B, b->st<int32_t>(L.pos), view, ao,
                               qd / 16, 1, b->wsp<float>(b->W.attn_part), b->wsp<int32_t>(b->W.attn_order));
        else
            hipLaunchKernelGGL(k_bf16_attn<false>, dim3(c.n_kv_heads, B, n_splits), dim3(256), 0, s, b->wsp<bf16_t>(b->W.q_hi),
                               b->wsp<bf16_t>(b->W.q_lo), c.n_q_heads, idx, n_ptr, B, b->st<int32_t>(L.pos), view, ao,
                               qd / 16, n_splits, b->wsp<float>(b->W.attn_part), b->wsp<int32_t>(b->W.attn_order));
        if (n_splits > 1)
            hipLaunchKernelGGL(k_bf16_attn_merge, dim3(c.n_kv_heads, B), dim3(256), 0, s, b->wsp<float>(b->W.attn_part),
                               c.n_q_heads, c.n_kv_heads, n_splits, n_ptr, B, ao, qd / 16);
    }
    EpiArgs e2{};
    e2.out = h; e2.ldo = d; e2.idx = idx;
    bool ffn_x_done = false;
    {
        TimedScope t(EE_K_GEMM_O, s);
        SliceTail st;                  // the finish of a sliced product also normalises for the FFN
        st.norm_gain = w.g_ffn; st.eps = c.rms_eps; st.norm_out = x; st.norm_done = &ffn_x_done;
        if (!gemm_tiled<EPI_RESID>(b, ao, w.w_o, d, qd, d / 32, 0, n_ptr, B, e2, s, ZBatch{}, 1, st))
            gemm<1, EPI_RESID>(ao, w.w_o, d, qd, d / 32, 0, n_ptr, B, e2, s);
    }
    if (!ffn_x_done) {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(NORM_THREADS), 0, s, h, idx, n_ptr, B, w.g_ffn, c.rms_eps, d, x, ZBatch{});
    }
    EpiArgs e3{};
    e3.act = act; e3.KB_act = F / 16; e3.idx = idx;
    {
        TimedScope t(EE_K_GEMM_GATE_UP, s);
        if (!gemm_tiled<EPI_SWIGLU>(b, x, w.w_gate_up, 2 * F, d, 2 * F / 32, 0, n_ptr, B, e3, s))
            gemm<2, EPI_SWIGLU>(x, w.w_gate_up, 2 * F, d, 2 * F / 32, 0, n_ptr, B, e3, s);
    }
    {
        TimedScope t(EE_K_GEMM_DOWN, s);
        SliceTail st;
        st.norm_gain = tail_gain; st.eps = c.rms_eps; st.norm_out = x; st.norm_done = x_done;
        if (!gemm_tiled<EPI_RESID>(b, act, w.w_down, d, F, d / 32, 0, n_ptr, B, e2, s, ZBatch{}, 1, st))
            gemm<1, EPI_RESID>(act, w.w_down, d, F, d / 32, 0, n_ptr, B, e2, s);
    }
    EE_LAUNCH_CHECK();
    return EE_OK;
}

int bf16_exit_head(const ee_model* m, int e, float th, int force, ee_batch* b, float* dbg, hipStream_t s,
                   bool x_ready) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, V = c.vocab;
    const int32_t* idx = b->st<int32_t>(L.active_idx);
    const int32_t* n_ptr = b->st<int32_t>(L.n_active);
    uint4* x = b->wsp<uint4>(b->W.x);
    if (!x_ready) {
        TimedScope t(EE_K_NORM, s);
        hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B), dim3(NORM_THREADS), 0, s, b->st<float>(L.h), idx, n_ptr, B,
                           m->exits[e].gain, c.rms_eps, d, x, ZBatch{});
    }
    EpiArgs ep{};
    ep.idx = idx; ep.row_scale = b->st<float>(L.row_scale);
    ep.part_max = b->wsp<float>(b->W.part_max); ep.part_sum = b->wsp<float>(b->W.part_sum);
    ep.part_arg = b->wsp<int32_t>(b->W.part_arg); ep.n_part = V / 32;
    ep.dbg_logits = dbg; ep.ldo = V;
    {
        TimedScope t(EE_K_EXIT_GEMM, s);
        if (!gemm_tiled<EPI_EXIT>(b, x, m->exits[e].w, V, d, V / 32, 0, n_ptr, B, ep, s))
            gemm<1, EPI_EXIT>(x, m->exits[e].w, V, d, V / 32, 0, n_ptr, B, ep, s);
    }
    EE_LAUNCH_CHECK();
    return launch_exit_decide(b, V / 32, th, force, s);
}

int bf16_fill_kv(const ee_model* m, int from_excl, int to_incl, ee_kv* kv, ee_batch* b, hipStream_t s,
                 const int32_t* idx, const int32_t* n_ptr) {
    const ee_model_config& c = m->cfg;
    const ee_batch_layout& L = b->L;
    int B = b->B, d = c.d_model, hd = c.head_dim;
    int kv_n = 2 * c.n_kv_heads * hd;
    int nl = to_incl - from_excl;                       // layers to fill: from_excl + 1 .. to_incl
    if (idx == nullptr) { idx = b->st<int32_t>(L.exited_idx); n_ptr = b->st<int32_t>(L.n_exited); }
    uint4* x = b->wsp<uint4>(b->W.fill_x);              // [layer][Mpad][d] normalised exit rows, tile order
    float* kvb = b->wsp<float>(b->W.fill_kv);           // [layer][Mpad][2 H_kv hd]
    TimedScope t(EE_K_FILL_KV, s);
    // all layers of the range in three launches (blockIdx.z = layer): the layers differ only in
    // their norm gain and their W_k / W_v
    ZBatch zb{};
    zb.w_tab = m->d_wqkv_tab; zb.g_tab = m->d_gattn_tab; zb.z0 = from_excl;
    zb.x_stride = (int64_t)b->Mpad * d / 8; zb.out_stride = (int64_t)b->Mpad * kv_n;
    hipLaunchKernelGGL(k_bf16_rmsnorm, dim3(B, 1, nl), dim3(NORM_THREADS), 0, s, b->st<float>(L.h), idx, n_ptr, B,
                       (const float*)nullptr, c.rms_eps, d, x, zb);
    // key and value rows are the last 2*H_kv*hd rows of W_qkv: tile-rows H_q*hd/32 onwards
    EpiArgs ep{};
    ep.out = kvb; ep.ldo = kv_n; ep.idx = idx;
    int NBs = (c.n_q_heads + 2 * c.n_kv_heads) * hd / 32, nb_off = c.n_q_heads * hd / 32;
    if (!gemm_tiled<EPI_STORE>(b, x, nullptr, kv_n, d, NBs, nb_off, n_ptr, B, ep, s, zb, nl))
        gemm<1, EPI_STORE>(x, nullptr, kv_n, d, NBs, nb_off, n_ptr, B, ep, s, zb, nl);
    hipLaunchKernelGGL(k_bf16_rope_append, dim3(B, 1, nl), dim3(256), 0, s, kvb, kv_n, 0, idx, n_ptr, B,
                       b->st<int32_t>(L.pos), m->d_rope, c.max_pos, make_view(m, kv, from_excl + 1, b),
                       (bf16_t*)nullptr, (bf16_t*)nullptr, b->st<int32_t>(L.status), zb.out_stride,
                       (int32_t*)nullptr, 1, (int64_t)0);
    EE_LAUNCH_CHECK();
    return EE_OK;
}
