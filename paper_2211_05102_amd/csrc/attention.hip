// Multiquery decode attention for gfx950 (paper Section 3.3: n_heads query
// heads, ONE shared K/V head; during generation one query token per sequence
// meets a cache of many tokens, so the time goes to loading the cache once).
//
// Per sequence b with T = positions[b] + 1 live slots:
//     s[h][t] = q[h] . K[t] / sqrt(dh),  p = softmax_t(s),  o[h] = sum_t p[h][t] V[t]
// K and V are read from HBM exactly once for all heads: the heads sit on one
// dimension of a 32x32 MFMA tile, a 32-token block of the cache on the other.
//
//   S^T[t][h] = sum_c K[t][c] q[h][c]     A = K block (M = token), B = q^T (N = head)
//   O^T[c][h] = sum_t V[t][c] P^T[t][h]   A = V^T block (M = channel), B = P^T
// The accumulator layout of the first product (lane = head, registers = tokens
// 8i + 4g + j) is, element for element, the B-operand layout of the second once
// the token order inside a 16-token MFMA step is permuted the same way on the
// V side; the V cache is stored in exactly that order, the K cache in A-operand
// order, so both stream from HBM as 1 KiB-per-wavefront contiguous loads with
// no LDS staging or transposition:
//   K block (32 tokens): uint4 index (j*64 + lane)       = K[t = lane%32][16j + 8(lane/32) + 0..7]
//   V block: uint4 index ((db*2 + kk)*64 + lane), element e
//            = V[t = 16kk + 8(e/4) + 4(lane/32) + e%4][c = 32db + lane%32]
// Split-KV: workgroup (split, b) takes `bps` consecutive 32-token blocks, its 4
// waves take them round-robin with a running (max, sum, acc) each (base-2
// exponentials, Section 3.5), merge through LDS, and write one fp32 partial; a
// second kernel combines the partials of a sequence in fixed order.
#include "common.h"
#include "kernels.h"

namespace pd {

template <int DH>
__global__ __launch_bounds__(256) void mqa_attend_kernel(
    const uint16_t* __restrict__ q, const uint4* __restrict__ kc, const uint4* __restrict__ vc,
    const int32_t* __restrict__ positions, int H, int L_ctx, int bps, int nsplit,
    float* __restrict__ opart, float* __restrict__ ml, float scale_log2e) {
    constexpr int KJ = DH / 16;  // MFMA steps of the q.K product
    constexpr int DB = DH / 32;  // 32-channel blocks of the output
    constexpr int BLK_U4 = 4 * DH;  // uint4 per 32-token block (K and V alike)
    __shared__ float ml_s[4][64][2];
    __shared__ float obuf[DB * 16][64];

    const int b = blockIdx.y, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int P = positions[b];
    if (P < 0 || P >= L_ctx) return;  // reported by the prep kernel; nothing is read or written
    const int nblk = (P >> 5) + 1;
    const int blk0 = split * bps;
    const int blk1 = blk0 + bps < nblk ? blk0 + bps : nblk;
    if (blk0 >= blk1) return;
    const int nblk_cap = L_ctx >> 5;

    // q operand (B matrix): lane (head l32, g) holds q[h][16j + 8g .. +8) for every j
    const int hq = l32 < H ? l32 : H - 1;  // padded heads duplicate the last one; never stored
    uint4 qop[KJ];
#pragma unroll
    for (int j = 0; j < KJ; j++)
        qop[j] = *reinterpret_cast<const uint4*>(q + ((size_t)b * H + hq) * DH + 16 * j + 8 * g);

    const uint4* kbase = kc + (size_t)b * nblk_cap * BLK_U4 + lane;
    const uint4* vbase = vc + (size_t)b * nblk_cap * BLK_U4 + lane;

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 O[DB];
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) O[db][r] = 0.f;

    for (int blk = blk0 + wave; blk < blk1; blk += 4) {
        uint4 kreg[KJ], vreg[DB][2];
        const uint4* kp = kbase + (size_t)blk * BLK_U4;
        const uint4* vp = vbase + (size_t)blk * BLK_U4;
#pragma unroll
        for (int j = 0; j < KJ; j++) kreg[j] = ld_stream(kp + j * 64);
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int kk = 0; kk < 2; kk++) vreg[db][kk] = ld_stream(vp + (db * 2 + kk) * 64);

        f32x16 S;
#pragma unroll
        for (int r = 0; r < 16; r++) S[r] = 0.f;
#pragma unroll
        for (int j = 0; j < KJ; j++)
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[j]),
                                                        __builtin_bit_cast(bf16x8, qop[j]), S, 0, 0, 0);
        const bool tail = (blk == nblk - 1) && ((P & 31) != 31);
#pragma unroll
        for (int r = 0; r < 16; r++) S[r] *= scale_log2e;
        if (tail) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                int t = blk * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t > P) S[r] = -INFINITY;
            }
            // slots past P may hold anything (even NaN); p is exactly 0 there, so zero V too
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int kk = 0; kk < 2; kk++) {
                    uint32_t w[4] = {vreg[db][kk].x, vreg[db][kk].y, vreg[db][kk].z, vreg[db][kk].w};
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        int t = blk * 32 + 16 * kk + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (t > P) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                    }
                    vreg[db][kk] = make_uint4(w[0], w[1], w[2], w[3]);
                }
        }
        float mloc = S[0];
#pragma unroll
        for (int r = 1; r < 16; r++) mloc = fmaxf(mloc, S[r]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));  // the other 16 tokens of this head
        const float m_new = fmaxf(m_run, mloc);        // finite: every block has a live token
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            S[r] = __builtin_amdgcn_exp2f(S[r] - m_new);
            psum += S[r];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int r = 0; r < 16; r++) O[db][r] *= alpha;
        }
        bf16x8 pop[2];
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
            uint4 pk = {pack_bf16x2(S[8 * kk + 0], S[8 * kk + 1]), pack_bf16x2(S[8 * kk + 2], S[8 * kk + 3]),
                        pack_bf16x2(S[8 * kk + 4], S[8 * kk + 5]), pack_bf16x2(S[8 * kk + 6], S[8 * kk + 7])};
            pop[kk] = __builtin_bit_cast(bf16x8, pk);
        }
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int kk = 0; kk < 2; kk++)
                O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vreg[db][kk]),
                                                                pop[kk], O[db], 0, 0, 0);
    }

    // ---- merge the 4 waves (a wave without blocks has m = -inf, l = 0, O = 0)
    float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    ml_s[wave][lane][0] = m_run;
    ml_s[wave][lane][1] = l_tot;
    __syncthreads();
    float m_all = fmaxf(fmaxf(ml_s[0][lane][0], ml_s[1][lane][0]),
                        fmaxf(ml_s[2][lane][0], ml_s[3][lane][0]));  // finite: wave 0 had a block
    const float f_own = __builtin_amdgcn_exp2f(m_run - m_all);
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) O[db][r] *= f_own;
    for (int w = 1; w < 4; w++) {
        if (wave == w) {
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int r = 0; r < 16; r++) obuf[db * 16 + r][lane] = O[db][r];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int r = 0; r < 16; r++) O[db][r] += obuf[db * 16 + r][lane];
        }
        __syncthreads();
    }
    if (wave == 0 && l32 < H) {
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < 4; w++)
            l_all += ml_s[w][lane][1] * __builtin_amdgcn_exp2f(ml_s[w][lane][0] - m_all);
        const size_t row = ((size_t)b * nsplit + split) * H + l32;
        if (g == 0) {
            ml[row * 2 + 0] = m_all;
            ml[row * 2 + 1] = l_all;
        }
        float* orow = opart + row * DH;
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                f32x4 v = {O[db][4 * i + 0], O[db][4 * i + 1], O[db][4 * i + 2], O[db][4 * i + 3]};
                *reinterpret_cast<f32x4*>(orow + db * 32 + 8 * i + 4 * g) = v;
            }
    }
}

// o[b][h*dh + c] = sum_s w_s O_s[c] / sum_s w_s l_s,  w_s = 2^(m_s - max m), splits in index order
__global__ __launch_bounds__(256) void mqa_combine_kernel(const float* __restrict__ opart,
                                                          const float* __restrict__ ml,
                                                          const int32_t* __restrict__ positions,
                                                          int H, int dh, int L_ctx, int bps, int nsplit,
                                                          uint16_t* __restrict__ o, int o_stride) {
    const int b = blockIdx.y;
    const int P = positions[b];
    if (P < 0 || P >= L_ctx) return;
    const int live = ((P >> 5) + bps) / bps;  // ceil(nblk / bps), nblk = P/32 + 1
    const int idx = blockIdx.x * 256 + threadIdx.x;  // over H*dh
    if (idx >= H * dh) return;
    const int h = idx / dh, c = idx - h * dh;
    const size_t row0 = (size_t)b * nsplit * H + h;
    float m_all = -INFINITY;
    for (int s = 0; s < live; s++) m_all = fmaxf(m_all, ml[(row0 + (size_t)s * H) * 2]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < live; s++) {
        size_t row = row0 + (size_t)s * H;
        float w = __builtin_amdgcn_exp2f(ml[row * 2] - m_all);
        den += w * ml[row * 2 + 1];
        num += w * opart[row * dh + c];
    }
    o[(size_t)b * o_stride + idx] = to_bf16(num / den);
}

// canonical [B][L_ctx][dh]  <->  library block layout, one element per thread
__global__ __launch_bounds__(256) void kv_convert_kernel(const uint16_t* __restrict__ src,
                                                         uint16_t* __restrict__ dst, int B, int L_ctx,
                                                         int dh, int is_v, int to_library) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)B * L_ctx * dh;
    if (idx >= total) return;
    int c = (int)(idx % dh);
    size_t r = idx / dh;
    int t = (int)(r % L_ctx);
    int b = (int)(r / L_ctx);
    size_t blk = (size_t)b * (L_ctx >> 5) + (t >> 5);
    int tt = t & 31;
    size_t off;
    if (!is_v)
        off = (((size_t)(c >> 4) * 2 + ((c & 15) >> 3)) * 32 + tt) * 8 + (c & 7);
    else
        off = ((((size_t)(c >> 5) * 2 + (tt >> 4)) * 2 + ((tt & 7) >> 2)) * 32 + (c & 31)) * 8 +
              4 * ((tt & 15) >> 3) + (tt & 3);
    size_t lib = blk * 32 * dh + off;
    if (to_library) dst[lib] = src[idx];
    else dst[idx] = src[lib];
}

hipError_t launch_mqa_attend(const uint16_t* q, const void* kc_layer, const void* vc_layer,
                             const int32_t* positions, int B, int H, int dh, int L_ctx, int bps,
                             float* opart, float* ml, uint16_t* o, int o_stride,
                             hipStream_t stream) {
    const int nblk_cap = L_ctx / 32;
    const int nsplit = (nblk_cap + bps - 1) / bps;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
    dim3 grid(nsplit, B), block(256);
    const uint4* k4 = reinterpret_cast<const uint4*>(kc_layer);
    const uint4* v4 = reinterpret_cast<const uint4*>(vc_layer);
    if (dh == 256)
        mqa_attend_kernel<256><<<grid, block, 0, stream>>>(q, k4, v4, positions, H, L_ctx, bps, nsplit,
                                                           opart, ml, scale_log2e);
    else if (dh == 128)
        mqa_attend_kernel<128><<<grid, block, 0, stream>>>(q, k4, v4, positions, H, L_ctx, bps, nsplit,
                                                           opart, ml, scale_log2e);
    else if (dh == 64)
        mqa_attend_kernel<64><<<grid, block, 0, stream>>>(q, k4, v4, positions, H, L_ctx, bps, nsplit,
                                                          opart, ml, scale_log2e);
    else
        return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    mqa_combine_kernel<<<dim3((H * dh + 255) / 256, B), block, 0, stream>>>(
        opart, ml, positions, H, dh, L_ctx, bps, nsplit, o, o_stride);
    return hipGetLastError();
}

hipError_t launch_kv_convert(const void* src, void* dst, int B, int L_ctx, int dh, int is_v,
                             int to_library, hipStream_t stream) {
    size_t total = (size_t)B * L_ctx * dh;
    kv_convert_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        reinterpret_cast<const uint16_t*>(src), reinterpret_cast<uint16_t*>(dst), B, L_ctx, dh, is_v,
        to_library);
    return hipGetLastError();
}

}  // namespace pd
