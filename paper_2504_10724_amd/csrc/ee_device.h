// ee_device.h -- small device-side helpers shared by the kernels of libee.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ee_internal.h"

typedef uint16_t bf16_t;   // storage: upper 16 bits of the fp32 pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}

// round to nearest even; inf/nan pass through
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (bf16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// element offset (in elements of the model dtype) of the (layer, row, kv-head) block
// cache row that batch row b reads and appends to
__device__ __forceinline__ int kv_row(const KvView& kv, int b) { return kv.seq ? kv.seq[b] : b; }

__device__ __forceinline__ int64_t kv_block(const KvView& kv, int b, int g, int cap_b) {
    return ((int64_t)kv.layer0 * kv.T + kv.off[b]) * (2LL * kv.n_kv_heads * kv.head_dim) +
           (int64_t)g * 2LL * cap_b * kv.head_dim;
}

// bf16 layout of a (layer, cache row, kv head) block (hd = 128): groups of 32 positions, each
// group 16 KiB = [K of the group, 8 KiB][V of the group, 8 KiB], so that a workgroup of the
// attention kernel walks ONE contiguous stream.  Offsets are relative to the block's start.
// K part of a group: two blocks of 16 positions; inside a block the four 32-feature slices follow
// each other, each stored as [feature octet (4)][position (16)][8 features]: lane l of a wave reads
// the 16 bytes at l * 16 of a slice and holds exactly its part of the score-MFMA operand
__device__ __forceinline__ int64_t k_bf16_offset(int p, int i, int hd) {
    int q = p >> 5, r = p & 31;
    return (int64_t)q * (64 * hd) + ((((r >> 4) * 4 + (i >> 5)) * 4 + ((i >> 3) & 3)) * 16 + (r & 15)) * 8 + (i & 7);
}

// V part of a group: the 16-feature slices follow each other, each stored as
// [position quad (4)][feature (16)][8 positions: r, r+1, r+2, r+3, r+16, .. r+19 of the quad]:
// lane l of a wave reads the 16 bytes at l * 16 of a slice and holds its part of the PV-MFMA operand
__device__ __forceinline__ int64_t v_bf16_offset(int p, int i, int hd) {
    int q = p >> 5, r = p & 31;
    return (int64_t)q * (64 * hd) + 32 * hd + ((((i >> 4) * 4 + ((r & 15) >> 2)) * 16 + (i & 15)) * 8 + ((r >> 4) << 2) + (r & 3));
}

// index (in 8-element chunks) of the chunk holding row `row`, columns [c, c+8) (c % 8 == 0)
// of an activation matrix with K columns stored in 32x16 tile order
__device__ __forceinline__ int64_t afrag_chunk(int row, int c, int KB /* K/16 */) {
    int mb = row >> 5, kb = c >> 4;
    int lane = (row & 31) + (((c & 15) >> 3) << 5);
    return ((int64_t)mb * KB + kb) * 64 + lane;
}

template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float* smem /* THREADS/64 floats */) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) smem[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < THREADS / 64; ++i) t += smem[i];
    __syncthreads();
    return t;
}

// Partial softmax statistics of a range of logits: maximum, sum of exp(z - max),
// lowest index attaining the maximum.  Merging is associative up to rounding.
struct Stat { float m; float s; int a; };

__device__ __forceinline__ Stat stat_merge(Stat x, Stat y) {
    Stat r;
    r.m = fmaxf(x.m, y.m);
    r.s = x.s * expf(x.m - r.m) + y.s * expf(y.m - r.m);
    r.a = (x.m > y.m) ? x.a : ((y.m > x.m) ? y.a : min(x.a, y.a));
    return r;
}
