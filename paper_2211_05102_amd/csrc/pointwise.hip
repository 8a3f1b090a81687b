// The small kernels between the two projections of the parallel block (paper
// Section 3.4: one LayerNorm per layer feeds both branches, attention and FFN
// outputs are summed by the fused output projection and added to the residual).
//   prep       : per-step rotation table cos/sin(positions[b] * base^(-2i/dh)), position check
//   ln_first   : bf16 input -> fp32 residual stream, then LayerNorm of layer 0
//   epi_in     : sum K-split partials of the input projection, apply the per-channel
//                scale (Section 3.6), rotate q and k, append k/v to the cache,
//                SwiGLU gate (Section 3.5 names the base-2 Swish)
//   residual   : sum partials of the output projection, scale, add the residual; slice
//                statistics of the updated rows
//   ln_slices  : LayerNorm of the updated residual for the next layer
// Operands of the projections (LayerNorm output, SwiGLU output) leave these
// kernels in block fixed point (common.h), one wavefront per 128-element chunk.
#include "common.h"
#include "kernels.h"

namespace pd {

__global__ __launch_bounds__(128) void prep_kernel(const int32_t* __restrict__ positions, int L_ctx,
                                                   int dh, double rope_base, float* __restrict__ cs,
                                                   int32_t* __restrict__ flag,
                                                   const int32_t* __restrict__ seq, int cache_rows) {
    const int b = blockIdx.x, i = threadIdx.x;
    const int P = positions[b];
    const int sb = seq ? seq[b] : b;  // cache row of this token row
    const bool bad = P < 0 || P >= L_ctx || sb < 0 || sb >= cache_rows;
    // one flag word per row, rewritten every step (256 words; rows >= B cleared by block 0)
    if (i == 0) flag[b] = bad ? 1 : 0;
    if (b == 0)
        for (int r = (int)gridDim.x + i; r < 256; r += 128) flag[r] = 0;
    if (i < dh / 2) {
        // angle in fp64: at position ~8000 an fp32 product is off by ~5e-4 rad
        double theta = pow(rope_base, -2.0 * (double)i / (double)dh);
        double phi = (bad ? 0.0 : (double)P) * theta;
        double sn, cn;
        sincos(phi, &sn, &cn);
        cs[((size_t)b * (dh / 2) + i) * 2 + 0] = (float)cn;
        cs[((size_t)b * (dh / 2) + i) * 2 + 1] = (float)sn;
    }
}

// h = gamma * (x - mean) / sqrt(var + eps), population variance, two passes over
// the row; h is written in block fixed point with ONE scale for the whole row
// (a LayerNorm output has no outlying chunk).  `sum` is this thread's share of
// sum(x) over the elements tid, tid + 256, ...
__device__ __forceinline__ void layernorm_row(const float* __restrict__ xrow,
                                              const float* __restrict__ gamma, int d, float eps,
                                              float sum, int b, int nd,
                                              unsigned char* __restrict__ hq,
                                              float* __restrict__ hs, float* red) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float mean = block_sum_256(sum, red) / (float)d;
    float sq = 0.f;
    for (int c = tid; c < d; c += 256) {
        float t = xrow[c] - mean;
        sq += t * t;
    }
    const float var = block_sum_256(sq, red) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    float mx = 0.f;
    for (int c = tid; c < d; c += 256) mx = fmaxf(mx, fabsf(gamma[c] * (xrow[c] - mean) * rstd));
    const float s = qscale_from_max(block_max_256(mx, red), nd);
    const float inv = 1.0f / s;
    for (int j = wave; j < (d >> 7); j += 4) {
        const int c = j * QCHUNK + 2 * lane;
        const f32x2 xv = *reinterpret_cast<const f32x2*>(xrow + c);
        const f32x2 gv = *reinterpret_cast<const f32x2*>(gamma + c);
        quantize_pair_store(gv.x * (xv.x - mean) * rstd, gv.y * (xv.y - mean) * rstd, inv, nd, lane,
                            hq + ((size_t)b * d + (size_t)j * QCHUNK) * nd);
        if (lane == 0) hs[(size_t)j * QSCALE_ROWS + b] = s;
    }
}

__global__ __launch_bounds__(256) void ln_first_kernel(const uint16_t* __restrict__ x_in,
                                                       const float* __restrict__ gamma, int d,
                                                       float eps, float* __restrict__ xres,
                                                       unsigned char* __restrict__ hq,
                                                       float* __restrict__ hs, int nd) {
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    float* xrow = xres + (size_t)b * d;
    float sum = 0.f;
    for (int c = tid; c < d; c += 256) {
        float v = from_bf16(x_in[(size_t)b * d + c]);
        xrow[c] = v;
        sum += v;
    }
    __syncthreads();  // the row is re-read with a different thread mapping below
    layernorm_row(xrow, gamma, d, eps, sum, b, nd, hq, hs, red);
}

// sum over the partial slots of the tile that holds packed column `col` (fixed order)
__device__ __forceinline__ float sum_partials(const float* __restrict__ part, const SkqPlan& pl,
                                              size_t stride, size_t off, int col) {
    const int ns = pl.nseg[col / pl.tile_cols];
    float acc = 0.f;
    for (int s = 0; s < ns; s++) acc += part[(size_t)s * stride + off];
    return acc;
}

// Section A (blockIdx.x < n_blocks_a): one item per thread over H*dh/2 q pairs |
// G*dh/2 k pairs | G*dh v elements (G K/V heads: 1 = multiquery, H = multihead; K/V head j
// of row b is pseudo-sequence b*G + j of the cache).  Section B: one workgroup per scale block of the
// SwiGLU output (blk_a chunks of 128, at most 64): wave w takes chunks w, w + 16, ...
// (one each for blocks of up to 16 chunks, so all of a block's loads are in flight
// together), the block maximum fixes one power-of-two scale, and the digits go into
// the operand of the output projection (chunks H*dh/128 ... of the row).
// `part` is in packed column order: q|k|v in place, then 64-column groups of
// (32 gate, 32 up).  Cache element offsets follow the library block layouts.
// (Several rows per workgroup, to have more loads in flight per lane, was measured
// slower: 18.3 against 14.4 us at 64 rows of the 62B shape.)
constexpr int EPI_THREADS = 1024;
__global__ __launch_bounds__(EPI_THREADS) void epi_in_kernel(
    const float* __restrict__ part, SkqPlan pl, const float* __restrict__ scale,
    const float* __restrict__ cs, const int32_t* __restrict__ positions,
    const int32_t* __restrict__ seq, int cache_rows, int B, int H, int G, int dh, int F,
    int L_ctx, int n_blocks_a, float* __restrict__ q, uint16_t* __restrict__ kc,
    uint16_t* __restrict__ vc, unsigned char* __restrict__ actq, float* __restrict__ acts,
    int blk_a, int nd) {
    __shared__ float red[EPI_THREADS / 64];
    const int b = blockIdx.y;
    const int half = dh >> 1;
    const int n_q = H * half, n_k = G * half, n_v = G * dh;
    const int n_qkv = H * dh + 2 * G * dh;
    const int N = n_qkv + 2 * F;
    const int k_out = H * dh + F;
    const size_t stride = (size_t)pl.rows * N, rowoff = (size_t)b * N;

    if ((int)blockIdx.x >= n_blocks_a) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int c_lo = ((int)blockIdx.x - n_blocks_a) * blk_a;
        const int c_hi = c_lo + blk_a < (F >> 7) ? c_lo + blk_a : (F >> 7);
        float a0[4], a1[4], mx = 0.f;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int j = c_lo + wave + 16 * k;  // chunk of the FFN activation
            a0[k] = a1[k] = 0.f;
            if (j < c_hi) {
                const int f = j * QCHUNK + 2 * lane;  // f and f + 1 share a 32-group
                const int pcol = n_qkv + (f >> 5) * 64 + (f & 31);
                const int ns = pl.nseg[pcol / pl.tile_cols];
                const float* p = part + rowoff + pcol;
                f32x2 gv = *reinterpret_cast<const f32x2*>(p);
                f32x2 uv = *reinterpret_cast<const f32x2*>(p + 32);
                for (int s = 1; s < ns; s++) {  // fixed order
                    gv += *reinterpret_cast<const f32x2*>(p + (size_t)s * stride);
                    uv += *reinterpret_cast<const f32x2*>(p + (size_t)s * stride + 32);
                }
                const float g0 = gv.x * scale[pcol], g1 = gv.y * scale[pcol + 1];
                const float u0 = uv.x * scale[pcol + 32], u1 = uv.y * scale[pcol + 33];
                // swish(g) = g / (1 + e^-g) = g / (1 + 2^(-g log2 e))
                a0[k] = g0 / (1.0f + __builtin_amdgcn_exp2f(-g0 * 1.4426950408889634f)) * u0;
                a1[k] = g1 / (1.0f + __builtin_amdgcn_exp2f(-g1 * 1.4426950408889634f)) * u1;
                mx = fmaxf(mx, fmaxf(fabsf(a0[k]), fabsf(a1[k])));
            }
        }
        mx = wave_max(mx);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < EPI_THREADS / 64; w++) mx = fmaxf(mx, red[w]);
        const float s = qscale_from_max(mx, nd);
        const float inv = 1.0f / s;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int j = c_lo + wave + 16 * k;
            if (j < c_hi) {
                const int chunk = (H * dh >> 7) + j;
                quantize_pair_store(a0[k], a1[k], inv, nd, lane,
                                    actq + ((size_t)b * k_out + (size_t)chunk * QCHUNK) * nd);
                if (lane == 0) acts[(size_t)chunk * QSCALE_ROWS + b] = s;
            }
        }
        return;
    }

    const int item = blockIdx.x * EPI_THREADS + threadIdx.x;
    const int P = positions[b];
    const int sb = seq ? seq[b] : b;  // cache row this token row appends to
    const bool ok = P >= 0 && P < L_ctx && sb >= 0 && sb < cache_rows;
    if (item < n_q + n_k) {
        // rotation pair (i, i + dh/2) of a q head or of k
        const bool is_k = item >= n_q;
        const int pi = is_k ? item - n_q : item;
        const int head = pi / half, i = pi % half;  // query head, or K/V head
        const int col = (is_k ? H * dh : 0) + head * dh + i;
        float lo = scale[col] * sum_partials(part, pl, stride, rowoff + col, col);
        float hi = scale[col + half] * sum_partials(part, pl, stride, rowoff + col + half, col + half);
        const float cn = cs[((size_t)b * half + i) * 2], sn = cs[((size_t)b * half + i) * 2 + 1];
        const float rlo = lo * cn - hi * sn, rhi = hi * cn + lo * sn;
        if (!is_k) {
            float* qrow = q + ((size_t)b * H + head) * dh;
            qrow[i] = rlo;
            qrow[i + half] = rhi;
        } else if (ok) {
            const size_t blk = (((size_t)sb * G + head) * (L_ctx >> 5) + (P >> 5)) * 32 * dh;
            const int tt = P & 31;
            int c = i;
            kc[blk + (((size_t)(c >> 4) * 2 + ((c & 15) >> 3)) * 32 + tt) * 8 + (c & 7)] = to_bf16(rlo);
            c = i + half;
            kc[blk + (((size_t)(c >> 4) * 2 + ((c & 15) >> 3)) * 32 + tt) * 8 + (c & 7)] = to_bf16(rhi);
        }
    } else if (item < n_q + n_k + n_v) {
        const int cv = item - n_q - n_k;
        const int head = cv / dh, c = cv - head * dh;
        const int col = H * dh + G * dh + cv;
        float v = scale[col] * sum_partials(part, pl, stride, rowoff + col, col);
        if (ok) {
            const size_t blk = (((size_t)sb * G + head) * (L_ctx >> 5) + (P >> 5)) * 32 * dh;
            const int tt = P & 31;
            vc[blk + ((((size_t)(c >> 5) * 2 + (tt >> 4)) * 2 + ((tt & 7) >> 2)) * 32 + (c & 31)) * 8 +
               4 * ((tt & 15) >> 3) + (tt & 3)] = to_bf16(v);
        }
    }
}

// x' = [x +] scale * sum over slots of part   (elementwise; slots summed in index order).
// If `stats` is given, every workgroup also leaves (mean, M2, max |x - mean|) of its
// 1024-column slice of the updated row for the LayerNorm kernel that follows.
__global__ __launch_bounds__(256) void residual_kernel(const float* __restrict__ part, SkqPlan pl,
                                                       const float* __restrict__ scale,
                                                       float* __restrict__ xres, int B, int d,
                                                       int add_residual,
                                                       uint16_t* __restrict__ x_out_bf16,
                                                       float* __restrict__ y_out_f32,
                                                       float* __restrict__ stats) {
    __shared__ float red[4];
    const int tid = threadIdx.x, b = blockIdx.y, c = (blockIdx.x * 256 + tid) * 4;
    const bool in = c < d;
    const size_t stride = (size_t)pl.rows * d, off = (size_t)b * d + c;
    f32x4 xn = {0.f, 0.f, 0.f, 0.f};
    if (in) {
        const int ns = pl.nseg[c / pl.tile_cols];  // 4 columns share a tile
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < ns; s++) acc += *reinterpret_cast<const f32x4*>(part + (size_t)s * stride + off);
        const f32x4 sc = *reinterpret_cast<const f32x4*>(scale + c);
        xn = sc * acc;
        if (add_residual) xn += *reinterpret_cast<const f32x4*>(xres + off);
        *reinterpret_cast<f32x4*>(xres + off) = xn;
        if (y_out_f32) *reinterpret_cast<f32x4*>(y_out_f32 + off) = xn;
        if (x_out_bf16) {
            uint2 o = {pack_bf16x2(xn.x, xn.y), pack_bf16x2(xn.z, xn.w)};
            *reinterpret_cast<uint2*>(x_out_bf16 + off) = o;
        }
    }
    if (!stats) return;
    const int n_here = d - (int)blockIdx.x * 1024 < 1024 ? d - (int)blockIdx.x * 1024 : 1024;
    const float mean_s = block_sum_256(in ? (xn.x + xn.y) + (xn.z + xn.w) : 0.f, red) / (float)n_here;
    const f32x4 dv = xn - mean_s;
    const float m2_s = block_sum_256(in ? (dv.x * dv.x + dv.y * dv.y) + (dv.z * dv.z + dv.w * dv.w) : 0.f, red);
    const float dev_s = block_max_256(
        in ? fmaxf(fmaxf(fabsf(dv.x), fabsf(dv.y)), fmaxf(fabsf(dv.z), fabsf(dv.w))) : 0.f, red);
    if (tid == 0) {
        float* st = stats + ((size_t)b * gridDim.x + blockIdx.x) * 4;
        st[0] = mean_s;
        st[1] = m2_s;
        st[2] = dev_s;
    }
}

// LayerNorm of the updated residual row for the next layer, one workgroup per
// 1024-column slice.  Every workgroup merges the slice statistics of its row in
// index order (pairwise update of count, mean, M2), so all of them get the same
// mean and variance bit for bit.  The row's single power-of-two scale comes from a
// bound instead of the exact maximum, so that no second pass over the row is
// needed:  |h| <= max|gamma| * max_s(maxdev_s + |mean_s - mean|) / sigma; the bound
// costs at most a bit or two of the 23 that three digit planes carry.
__global__ __launch_bounds__(256) void ln_slices_kernel(const float* __restrict__ xres,
                                                        const float* __restrict__ gamma,
                                                        const float* __restrict__ gamma_absmax,
                                                        const float* __restrict__ stats, int d,
                                                        float eps, unsigned char* __restrict__ hq,
                                                        float* __restrict__ hs, int nd) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y, nsl = gridDim.x;
    float n_tot = 0.f, mean = 0.f, m2 = 0.f;
    for (int sl = 0; sl < nsl; sl++) {
        const float n_i = (float)(d - sl * 1024 < 1024 ? d - sl * 1024 : 1024);
        const float* st = stats + ((size_t)b * nsl + sl) * 4;
        const float delta = st[0] - mean, n_new = n_tot + n_i;
        mean += delta * (n_i / n_new);
        m2 += st[1] + delta * delta * (n_tot * n_i / n_new);
        n_tot = n_new;
    }
    float dev = 0.f;
    for (int sl = 0; sl < nsl; sl++) {
        const float* st = stats + ((size_t)b * nsl + sl) * 4;
        dev = fmaxf(dev, st[2] + fabsf(st[0] - mean));
    }
    const float rstd = 1.0f / sqrtf(m2 / (float)d + eps);
    const float s = qscale_from_max(gamma_absmax[0] * dev * rstd * 1.0001f, nd);
    const float inv = 1.0f / s;
    const float* xrow = xres + (size_t)b * d;
    const int j_end = (blockIdx.x * 8 + 8) < (d >> 7) ? (blockIdx.x * 8 + 8) : (d >> 7);
    for (int j = blockIdx.x * 8 + wave; j < j_end; j += 4) {
        const int cc = j * QCHUNK + 2 * lane;
        const f32x2 xv = *reinterpret_cast<const f32x2*>(xrow + cc);
        const f32x2 gv = *reinterpret_cast<const f32x2*>(gamma + cc);
        quantize_pair_store(gv.x * (xv.x - mean) * rstd, gv.y * (xv.y - mean) * rstd, inv, nd, lane,
                            hq + ((size_t)b * d + (size_t)j * QCHUNK) * nd);
        if (lane == 0) hs[(size_t)j * QSCALE_ROWS + b] = s;
    }
}

// ---- residual add and the next layer's LayerNorm in one kernel ------------------
// One workgroup of 1024 threads per batch row, for rows of at most 16384 columns: the
// updated row stays in registers between the residual add and the LayerNorm, mean and
// variance are the exact two-pass ones and the row's power-of-two scale comes from the
// exact maximum.  Sums over the 16 waves go through LDS in wave order (fixed order).
constexpr int RL_THREADS = 1024;
constexpr int RL_MAXQ = 4;  // f32x4 groups per thread: rows of up to 1024 * 4 * 4 columns (more would spill)

__device__ __forceinline__ float block_sum_1024(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();  // protects `red` against the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < RL_THREADS / 64; w++) t += red[w];
    return t;
}
__device__ __forceinline__ float block_max_1024(float v, float* red) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int w = 1; w < RL_THREADS / 64; w++) t = fmaxf(t, red[w]);
    return t;
}

// digits of four consecutive elements c .. c + 3 of a row (c % 4 == 0) into the chunk
// that holds them; plane p of chunk j sits at j * 128 * nd + 128 * p (see common.h)
__device__ __forceinline__ void quantize_quad_store(const f32x4 v, float inv_scale, int nd, int c,
                                                    unsigned char* __restrict__ row) {
    const int lim = 127 << (8 * (nd - 1));
    int n[4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
        n[k] = (int)rintf(v[k] * inv_scale);
        n[k] = n[k] > lim ? lim : (n[k] < -lim ? -lim : n[k]);
    }
    unsigned char* chunk = row + (size_t)(c >> 7) * QCHUNK * nd + (c & 127);
    for (int p = nd - 1; p >= 0; p--) {
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            int d;
            if (p > 0) {
                const int h = (n[k] + 128) >> 8;  // floor division keeps every lower digit in [-128, 127]
                d = n[k] - (h << 8);
                n[k] = h;
            } else {
                d = n[k];
            }
            word |= (uint32_t)(d & 0xff) << (8 * k);
        }
        store_through(reinterpret_cast<uint32_t*>(chunk + p * QCHUNK), word);
    }
}

template <int NQ>  // f32x4 groups per thread
__global__ __launch_bounds__(RL_THREADS) void residual_ln_kernel(
    const float* __restrict__ part, SkqPlan pl, const float* __restrict__ scale,
    float* __restrict__ xres, int d, int add_residual, const float* __restrict__ gamma, float eps,
    unsigned char* __restrict__ hq, float* __restrict__ hs, int nd) {
    __shared__ float red[RL_THREADS / 64];
    const int tid = threadIdx.x, b = blockIdx.x;
    const size_t stride = (size_t)pl.rows * d, rowoff = (size_t)b * d;
    f32x4 xn[NQ];
    float sum = 0.f;
    // Slot sums of this thread's NQ column groups.  The slots of a group are added in index
    // order; the loads of all groups go out together, eight in flight per thread per round trip
    // (a slot index past a group's last one re-reads its last slot and is not added).
    constexpr int BATCH = 8 / NQ;
    int ns[NQ], ns_max = 0;
#pragma unroll
    for (int i = 0; i < NQ; i++) {
        const int c = (i * RL_THREADS + tid) * 4;
        ns[i] = c < d ? pl.nseg[c / pl.tile_cols] : 0;  // 4 columns share a tile
        ns_max = ns[i] > ns_max ? ns[i] : ns_max;
        xn[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    for (int s0 = 0; s0 < ns_max; s0 += BATCH) {
        f32x4 pv[NQ][BATCH];
#pragma unroll
        for (int i = 0; i < NQ; i++) {
            const int c = (i * RL_THREADS + tid) * 4;
#pragma unroll
            for (int k = 0; k < BATCH; k++) {
                int sk = s0 + k < ns[i] ? s0 + k : ns[i] - 1;
                sk = sk < 0 ? 0 : sk;
                pv[i][k] = c < d ? *reinterpret_cast<const f32x4*>(part + (size_t)sk * stride + rowoff + c)
                                 : (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int i = 0; i < NQ; i++)
#pragma unroll
            for (int k = 0; k < BATCH; k++)
                if (s0 + k < ns[i]) xn[i] += pv[i][k];
    }
#pragma unroll
    for (int i = 0; i < NQ; i++) {
        const int c = (i * RL_THREADS + tid) * 4;
        if (c < d) {
            f32x4 v = *reinterpret_cast<const f32x4*>(scale + c) * xn[i];
            if (add_residual) v += *reinterpret_cast<const f32x4*>(xres + rowoff + c);
            *reinterpret_cast<f32x4*>(xres + rowoff + c) = v;
            xn[i] = v;
            sum += (v.x + v.y) + (v.z + v.w);
        }
    }
    const float mean = block_sum_1024(sum, red) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NQ; i++) {
        const int c = (i * RL_THREADS + tid) * 4;
        if (c < d) {
            xn[i] -= mean;
            sq += (xn[i].x * xn[i].x + xn[i].y * xn[i].y) + (xn[i].z * xn[i].z + xn[i].w * xn[i].w);
        }
    }
    const float rstd = 1.0f / sqrtf(block_sum_1024(sq, red) / (float)d + eps);
    float mx = 0.f;
#pragma unroll
    for (int i = 0; i < NQ; i++) {
        const int c = (i * RL_THREADS + tid) * 4;
        if (c < d) xn[i] = *reinterpret_cast<const f32x4*>(gamma + c) * xn[i] * rstd;  // (zero beyond the row)
        mx = fmaxf(mx, fmaxf(fmaxf(fabsf(xn[i].x), fabsf(xn[i].y)), fmaxf(fabsf(xn[i].z), fabsf(xn[i].w))));
    }
    const float s = qscale_from_max(block_max_1024(mx, red), nd);
    const float inv = 1.0f / s;
    unsigned char* hrow = hq + rowoff * nd;
#pragma unroll
    for (int i = 0; i < NQ; i++) {
        const int c = (i * RL_THREADS + tid) * 4;
        if (c < d) {
            quantize_quad_store(xn[i], inv, nd, c, hrow);
            if ((c & 127) == 0) hs[(size_t)(c >> 7) * QSCALE_ROWS + b] = s;
        }
    }
}

// max |v[i]| of an fp32 vector (pack time: the LayerNorm gain of a layer)
__global__ __launch_bounds__(256) void vec_absmax_kernel(const float* __restrict__ v, int n,
                                                         float* __restrict__ out) {
    __shared__ float red[4];
    float mx = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) mx = fmaxf(mx, fabsf(v[i]));
    mx = block_max_256(mx, red);
    if (threadIdx.x == 0) out[0] = mx;
}

hipError_t launch_prep(const int32_t* positions, int B, int L_ctx, int dh, float rope_base,
                       float* cs, int32_t* flag, const int32_t* seq, int cache_rows, hipStream_t stream) {
    prep_kernel<<<dim3(B), dim3(128), 0, stream>>>(positions, L_ctx, dh, (double)rope_base, cs, flag, seq,
                                                   cache_rows);
    return hipGetLastError();
}

hipError_t launch_ln_first(const uint16_t* x_in, const float* gamma, int B, int d, float eps,
                           float* xres, void* hq, float* hs, int nd, hipStream_t stream) {
    ln_first_kernel<<<dim3(B), dim3(256), 0, stream>>>(x_in, gamma, d, eps, xres,
                                                       reinterpret_cast<unsigned char*>(hq), hs, nd);
    return hipGetLastError();
}

hipError_t launch_epi_in(const float* part, SkqPlan pl, const float* scale, const float* cs,
                         const int32_t* positions, const int32_t* seq, int cache_rows, int B, int H, int G,
                         int dh, int F, int L_ctx,
                         float* q, void* kc_layer, void* vc_layer, void* actq, float* acts,
                         int blk_a, int nd, hipStream_t stream) {
    if (blk_a < 1 || blk_a > 64) return hipErrorInvalidValue;
    const int items = H * dh / 2 + G * dh / 2 + G * dh;
    const int n_blocks_a = (items + EPI_THREADS - 1) / EPI_THREADS;
    const int n_blocks_b = (F / 128 + blk_a - 1) / blk_a;
    epi_in_kernel<<<dim3(n_blocks_a + n_blocks_b, B), dim3(EPI_THREADS), 0, stream>>>(
        part, pl, scale, cs, positions, seq, cache_rows, B, H, G, dh, F, L_ctx, n_blocks_a, q,
        reinterpret_cast<uint16_t*>(kc_layer), reinterpret_cast<uint16_t*>(vc_layer),
        reinterpret_cast<unsigned char*>(actq), acts, blk_a, nd);
    return hipGetLastError();
}

hipError_t launch_residual(const float* part, SkqPlan pl, const float* scale, float* xres, int B,
                           int d, int add_residual, uint16_t* x_out_bf16, float* y_out_f32,
                           float* stats, hipStream_t stream) {
    residual_kernel<<<dim3((d / 4 + 255) / 256, B), dim3(256), 0, stream>>>(
        part, pl, scale, xres, B, d, add_residual, x_out_bf16, y_out_f32, stats);
    return hipGetLastError();
}

hipError_t launch_ln_slices(const float* xres, const float* gamma, const float* gamma_absmax,
                            const float* stats, int B, int d, float eps, void* hq, float* hs,
                            int nd, hipStream_t stream) {
    ln_slices_kernel<<<dim3((d + 1023) / 1024, B), dim3(256), 0, stream>>>(
        xres, gamma, gamma_absmax, stats, d, eps, reinterpret_cast<unsigned char*>(hq), hs, nd);
    return hipGetLastError();
}

hipError_t launch_residual_ln(const float* part, SkqPlan pl, const float* scale, float* xres, int B,
                              int d, int add_residual, const float* gamma, float eps, void* hq, float* hs,
                              int nd, hipStream_t stream) {
    if (d > RL_THREADS * 4 * RL_MAXQ) return hipErrorInvalidValue;
    const int nq = (d + RL_THREADS * 4 - 1) / (RL_THREADS * 4);
    unsigned char* q = reinterpret_cast<unsigned char*>(hq);
#define PD_RL(NQ) residual_ln_kernel<NQ><<<dim3(B), dim3(RL_THREADS), 0, stream>>>(part, pl, scale, xres, d, add_residual, gamma, eps, q, hs, nd)
    if (nq <= 1) PD_RL(1);
    else if (nq <= 2) PD_RL(2);
    else PD_RL(4);
#undef PD_RL
    return hipGetLastError();
}

hipError_t launch_vec_absmax(const float* v, int n, float* out, hipStream_t stream) {
    vec_absmax_kernel<<<dim3(1), dim3(256), 0, stream>>>(v, n, out);
    return hipGetLastError();
}

}  // namespace pd
