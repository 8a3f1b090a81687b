// Shared device-side types and small helpers for the gfx950 decode kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

constexpr int WAVE = 64;

// ---- deterministic stream-K bookkeeping (see qgemm.hip) ------------------------
// A [K][N] projection is cut into units = (tile of `tile_cols` columns, 128-k
// chunk), ordered tile-major; workgroup g of G takes the contiguous unit range
// [g*U/G, (g+1)*U/G), U = T*C.  Inside a tile the chunks are also grouped into
// scale blocks (chunks [0, c_split) in blocks of blk0, chunks [c_split, C) in
// blocks of blk1) over which the exact int32 sums run on; at the end of a block
// they are folded into fp32 tile accumulators.  The part of a tile that lies in one
// workgroup's range produces one fp32 partial of the tile, stored in slot = index
// of that workgroup among those that share the tile, and consumers add the slots of
// a tile in index order: results do not depend on timing.
struct SkqPlan {
    int tile_cols, C, T, G;
    int c_split, blk0, blk1;
    int align;        // workgroup ranges start at multiples of this many units
    int rows;         // rows of one partial slot: the batch rounded up to whole row groups
    int max_slots;    // most slots in any tile
    const int* nseg;  // device table (skq_table_kernel): slots per tile, then one record per workgroup
};
// First unit of workgroup g's range (g = G: one past the last unit).
__host__ __device__ inline long long skq_begin(int g, long long U, int G, int align) {
    if (g >= G) return U;
    return (long long)g * U / G / align * align;
}
// Workgroup that owns unit u:
__host__ __device__ inline int skq_owner(long long u, long long U, int G, int align) {
    int g = (int)(((u + 1) * G - 1) / U);  // owner for unaligned ranges; aligned starts are never later
    if (g + 1 < G && skq_begin(g + 1, U, G, align) <= u) g++;
    return g;
}
// Workgroup ranges that start at a chunk position in (0, c] of tile t, c <= C - 1:
// the slot of the range that holds chunk c.
__host__ __device__ inline int skq_segments_upto(int t, int c, const SkqPlan& pl) {
    if (c <= 0) return 0;
    int n = 0;
    const long long U = (long long)pl.T * pl.C, base = (long long)t * pl.C;
    for (int g = skq_owner(base, U, pl.G, pl.align) + 1; g < pl.G; g++) {
        const long long pos = skq_begin(g, U, pl.G, pl.align) - base;
        if (pos > c) break;
        if (pos > 0) n++;
    }
    return n;
}
// slots of tile t
__host__ __device__ inline int skq_segments(int t, const SkqPlan& pl) {
    return skq_segments_upto(t, pl.C - 1, pl) + 1;
}

// Device table of a plan, in ints: [0, T) slots per tile; from skq_wg_offset(T), four
// per workgroup g: first unit, one past the last unit, slot of its range in its first
// tile, first tile.
__host__ __device__ inline int skq_wg_offset(int T) { return (T + 3) & ~3; }
__host__ __device__ inline size_t skq_table_ints(int T, int G) { return (size_t)skq_wg_offset(T) + 4 * (size_t)G; }

// Cache policy of buffer stores whose data the NEXT kernel reads (partial sums,
// split-KV partials): sc0 sc1 = written through to memory as it is produced.  Left
// as ordinary write-back data it sits dirty in the XCD's L2 until the kernel ends,
// and the end-of-kernel write-back of tens of megabytes is then paid as idle time
// (62B-shaped input projection: 138 -> 124 us).
#define PD_WRITE_THROUGH 17
// the same policy for an ordinary store of up to 8 bytes (a relaxed system-scope
// atomic store is a plain store with sc0 sc1)
template <typename T>
__device__ __forceinline__ void store_through(T* p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// round-to-nearest-even fp32 -> bf16 bit pattern (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 p = {lo, hi};
    bf16x2 q = __builtin_convertvector(p, bf16x2);
    return __builtin_bit_cast(uint32_t, q);
}
__device__ __forceinline__ uint16_t to_bf16(float v) {
    return (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
}
__device__ __forceinline__ float from_bf16(uint16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 16-byte streaming load that is read once (weights, KV): non-temporal hint
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains
// every outstanding global load (vmcnt(0)), which would serialise a weight
// prefetch with each step of a streaming loop; here only the LDS counter is waited on.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Column map of the fused input projection: packed column -> canonical column.
// q|k|v keep their place; gate and up are interleaved in 32-column groups
// (gate group m, then up group m) so one workgroup sees both halves of a
// SwiGLU pair.  mode 0 = identity.
__device__ __forceinline__ int packed_col_map(int pn, int mode, int n_qkv, int F) {
    if (mode == 0 || pn < n_qkv) return pn;
    int r = pn - n_qkv, pair = r >> 6, within = r & 63;
    return within < 32 ? n_qkv + pair * 32 + within : n_qkv + F + pair * 32 + (within - 32);
}

// ---- block fixed-point activations ------------------------------------------
// The operands of the two projections are stored as ND (2 or 3) int8 digit
// planes with one power-of-two scale per (row, 128-element chunk); producers
// give all chunks of a larger "scale block" the same scale so that the consumer
// can keep its exact int32 sums running across the block:
//     value ~= scale * sum_p 256^(ND-1-p) * d_p,   d_0 in [-127,127], others in [-128,127]
// i.e. 8*ND - 1 bits + sign relative to the chunk maximum (ND = 3: fp32-grade),
// which the int8 MFMA multiplies with the int8 weights exactly (int32 sums).
// Row layout (bytes): chunk j of a row at j*128*ND: plane p at +128*p (plane 0 is
// the most significant digit); row pitch = ND*K.
// Scales are stored transposed, scale_t[chunk][256 rows], so that the four rows
// a lane needs are contiguous.
constexpr int QCHUNK = 128;
constexpr int QSCALE_ROWS = 256;

// Power-of-two scale for a block whose largest magnitude is mx: the smallest
// 2^e with mx / 2^e <= 127 * 256^(nd-1).
__device__ __forceinline__ float qscale_from_max(float mx, int nd) {
    const int top_bits = 8 * (nd - 1);                  // weight of the top digit = 2^top_bits
    const float nmax = (float)(127 << top_bits);        // 32512 or 8323072
    float s = 1.0f;
    if (mx >= 1e-30f && mx < 1e30f) {
        const int fl = (int)((__float_as_uint(mx) >> 23) & 0xff) - 127;  // floor(log2 mx)
        s = __uint_as_float((uint32_t)(fl - (top_bits + 6) + 127) << 23);  // nmax < 2^(top_bits+7)
        if (mx > nmax * s) s *= 2.0f;
    }
    return s;
}

// Lane `lane` of a wavefront writes the digits of elements 2*lane and 2*lane+1 of
// one 128-element chunk (row_chunk points at the chunk's plane 0).
__device__ __forceinline__ void quantize_pair_store(float v0, float v1, float inv_scale, int nd,
                                                    int lane, unsigned char* __restrict__ row_chunk) {
    const int lim = 127 << (8 * (nd - 1));
    int n0 = (int)rintf(v0 * inv_scale), n1 = (int)rintf(v1 * inv_scale);
    n0 = n0 > lim ? lim : (n0 < -lim ? -lim : n0);  // only NaN/inf inputs get here
    n1 = n1 > lim ? lim : (n1 < -lim ? -lim : n1);
    // digits from the least significant up: floor division keeps every lower digit in [-128,127]
    for (int p = nd - 1; p >= 0; p--) {
        int d0, d1;
        if (p > 0) {
            const int h0 = (n0 + 128) >> 8, h1 = (n1 + 128) >> 8;
            d0 = n0 - (h0 << 8);
            d1 = n1 - (h1 << 8);
            n0 = h0;
            n1 = h1;
        } else {
            d0 = n0;
            d1 = n1;
        }
        // (written through, see PD_WRITE_THROUGH: the next kernel's projection reads these)
        store_through(reinterpret_cast<uint16_t*>(row_chunk + p * QCHUNK) + lane,
                      (uint16_t)((d0 & 0xff) | ((d1 & 0xff) << 8)));
    }
}

// One wavefront quantises one chunk with its own scale (lane holds elements
// 2*lane and 2*lane+1).
__device__ __forceinline__ void quantize_chunk_wave(float v0, float v1, int lane, int nd,
                                                    unsigned char* __restrict__ row_chunk,
                                                    float* __restrict__ scale_slot) {
    const float s = qscale_from_max(wave_max(fmaxf(fabsf(v0), fabsf(v1))), nd);
    quantize_pair_store(v0, v1, 1.0f / s, nd, lane, row_chunk);
    if (lane == 0) *scale_slot = s;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Sum over a 256-thread block; every thread gets the result.  `red` = 4 floats of LDS.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();  // protects `red` against the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// Max over a 256-thread block; every thread gets the result.  `red` = 4 floats of LDS.
__device__ __forceinline__ float block_max_256(float v, float* red) {
    v = wave_max(v);
    __syncthreads();  // protects `red` against the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

}  // namespace pd
