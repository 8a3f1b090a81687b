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
// K and V are bf16 data and enter the MFMAs exactly.  The two operands this
// kernel creates itself, q (pre-multiplied by log2(e)/sqrt(dh)) and the softmax
// weights P, are each split into a bf16 head and a bf16 remainder (hi + lo, 16
// significant bits) and cost two MFMAs per step: the matrix pipe has an order of
// magnitude of slack in this HBM-bound kernel, and a single bf16 rounding of q
// and P would be the largest error of the whole step.
// Split-KV: workgroup (split, b) takes `bps` consecutive 32-token blocks, its 4
// waves take them round-robin with a running (max, sum, acc) each (base-2
// exponentials, Section 3.5), merge through LDS, and write one fp32 partial; the
// second kernel combines the partials of a sequence in fixed order.
#include "common.h"
#include "kernels.h"

namespace pd {

// o[b][h*dh + c] = sum_s w_s O_s[c] / sum_s w_s l_s,  w_s = 2^(m_s - max m), splits in index order.
// One workgroup per scale block of the row (blk_o chunks of 128 elements, at most
// 16), one wavefront per chunk (blockDim = 64 * blk_o), two adjacent channels per
// lane: every load of the row's partials is in flight at once, so the kernel is one
// round trip to memory however many chunks the block has.  The result goes out as
// fp32 (`o`) and/or in block fixed point as the first H*dh/128 chunks of the output
// projection's operand (`actq`, `acts`).
// MAXS: upper bound of the live splits (0: run-time loop, for long contexts cut into
// many small splits).
__device__ __forceinline__ float combine_block_max(float v, float* red, int waves) {
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = red[0];
    for (int w = 1; w < waves; w++) t = fmaxf(t, red[w]);
    return t;
}

template <int MAXS>
__global__ __launch_bounds__(1024) void mqa_combine_kernel(
    const float* __restrict__ opart, const float* __restrict__ ml,
    const int32_t* __restrict__ positions, int H, int G, int dh, int L_ctx, int bps, int nsplit,
    float* __restrict__ o, unsigned char* __restrict__ actq, float* __restrict__ acts,
    int k_out, int blk_o, int nd) {
    __shared__ float red[16];
    const int b = blockIdx.y;
    const int P = positions[b];
    if (P < 0 || P >= L_ctx) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * blk_o + wave;  // this wave's chunk
    const bool in_row = j < (H * dh >> 7);
    const int live = ((P >> 5) + bps) / bps;  // ceil(nblk / bps), nblk = P/32 + 1
    float o0 = 0.f, o1 = 0.f;
    if (in_row) {
        const int idx = j * QCHUNK + 2 * lane;  // idx and idx + 1 lie in the same head
        const int h = idx / dh, c = idx - h * dh;
        // K/V head h / per of row b is pseudo-sequence b*G + h/per; it holds `per` query heads
        const int per = H / G;
        const size_t row0 = ((size_t)b * G + h / per) * nsplit * per + h % per;
        float n0 = 0.f, n1 = 0.f, den = 0.f;
        if constexpr (MAXS > 0) {
            f32x2 mlv[MAXS], ov[MAXS];
#pragma unroll
            for (int s = 0; s < MAXS; s++) {
                const size_t row = row0 + (size_t)(s < live ? s : live - 1) * per;
                mlv[s] = *reinterpret_cast<const f32x2*>(ml + row * 2);
                ov[s] = *reinterpret_cast<const f32x2*>(opart + row * dh + c);
            }
            float m_all = -INFINITY;
#pragma unroll
            for (int s = 0; s < MAXS; s++)
                if (s < live) m_all = fmaxf(m_all, mlv[s].x);
#pragma unroll
            for (int s = 0; s < MAXS; s++)
                if (s < live) {
                    const float w = __builtin_amdgcn_exp2f(mlv[s].x - m_all);
                    den += w * mlv[s].y;
                    n0 += w * ov[s].x;
                    n1 += w * ov[s].y;
                }
        } else {
            float m_all = -INFINITY;
            for (int s = 0; s < live; s++) m_all = fmaxf(m_all, ml[(row0 + (size_t)s * per) * 2]);
            for (int s = 0; s < live; s++) {
                const size_t row = row0 + (size_t)s * per;
                const float w = __builtin_amdgcn_exp2f(ml[row * 2] - m_all);
                den += w * ml[row * 2 + 1];
                const f32x2 ov = *reinterpret_cast<const f32x2*>(opart + row * dh + c);
                n0 += w * ov.x;
                n1 += w * ov.y;
            }
        }
        o0 = n0 / den;
        o1 = n1 / den;
        if (o) {
            const f32x2 out = {o0, o1};
            *reinterpret_cast<f32x2*>(o + (size_t)b * H * dh + idx) = out;
        }
    }
    if (!actq) return;
    const float s = qscale_from_max(combine_block_max(fmaxf(fabsf(o0), fabsf(o1)), red, blockDim.x >> 6), nd);
    if (in_row) {
        quantize_pair_store(o0, o1, 1.0f / s, nd, lane, actq + ((size_t)b * k_out + (size_t)j * QCHUNK) * nd);
        if (lane == 0) acts[(size_t)j * QSCALE_ROWS + b] = s;
    }
}

template <int DH>
__global__ __launch_bounds__(256) void mqa_attend_kernel(
    const float* __restrict__ q, const uint4* __restrict__ kc, const uint4* __restrict__ vc,
    const int32_t* __restrict__ positions, const int32_t* __restrict__ seq, int cache_rows, int H, int G,
    int L_ctx, int bps, int nsplit, float* __restrict__ opart, float* __restrict__ ml, float scale_log2e) {
    constexpr int KJ = DH / 16;  // MFMA steps of the q.K product
    constexpr int DB = DH / 32;  // 32-channel blocks of the output
    constexpr int BLK_U4 = 4 * DH;  // uint4 per 32-token block (K and V alike)
    __shared__ float ml_s[4][64][2];
    // q operands [plane][j][lane] during the block loop, then the merge buffer [DB][3][4][64] of f32x4
    constexpr int SMEM_U4 = 2 * KJ * 64 > DB * 3 * 4 * 64 ? 2 * KJ * 64 : DB * 3 * 4 * 64;
    __shared__ uint4 smem[SMEM_U4];

    const int b = blockIdx.y, split = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    // (uniform by construction; saying so keeps the buffer offsets derived from it scalar --
    // otherwise every load below is wrapped in a loop over the "distinct" values)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;
    // b is a pseudo-sequence: K/V head b % G of token row b / G, with H query heads; the
    // row's keys and values live in cache row seq[b / G] (the row itself without a map)
    const int P = positions[b / G];
    const int sb = seq ? seq[b / G] : b / G;
    if (P < 0 || P >= L_ctx || sb < 0 || sb >= cache_rows) return;  // reported by the prep kernel; nothing is read or written
    const size_t cache_seq = (size_t)sb * G + b % G;
    const int nblk = (P >> 5) + 1;
    const int blk0 = split * bps;
    const int blk1 = blk0 + bps < nblk ? blk0 + bps : nblk;
    if (blk0 >= blk1) return;
    const int nblk_cap = L_ctx >> 5;

    // K and V of this sequence as buffers that end where this workgroup's share
    // ends: the software pipeline below always asks for the next block, and a read
    // past the end returns zeros without touching memory.
    const __amdgpu_buffer_rsrc_t k_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(kc + cache_seq * nblk_cap * BLK_U4), 0, blk1 * BLK_U4 * 16, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(vc + cache_seq * nblk_cap * BLK_U4), 0, blk1 * BLK_U4 * 16, 0x00020000);
    const uint32_t lane16 = lane * 16;

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 O[DB];
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) O[db][r] = 0.f;

    // Two rings of KJ 1-KiB pieces per wave, always full: the K pieces of a block are
    // consumed in order and each slot is refilled at once with the same piece of this
    // wave's next block; likewise the V pieces.  A whole block ahead (32 KiB per wave,
    // 128 KiB per compute unit) stays in flight.  Non-temporal: every byte is used once.
    // q of this row first (vector-memory operations complete in order: the wait for these
    // few loads must not include the K and V blocks requested after them)
    constexpr int QIT = (KJ * 64 + 255) / 256;
    f32x4 qa0[QIT], qa1[QIT];
#pragma unroll
    for (int it = 0; it < QIT; it++) {
        int slot = it * 256 + tid;
        slot = slot < KJ * 64 ? slot : KJ * 64 - 1;
        const int j = slot >> 6, ln = slot & 63;
        const int hh = (ln & 31) < H ? (ln & 31) : H - 1;
        const float* src = q + ((size_t)b * H + hh) * DH + 16 * j + 8 * (ln >> 5);
        qa0[it] = *reinterpret_cast<const f32x4*>(src);
        qa1[it] = *reinterpret_cast<const f32x4*>(src + 4);
    }
    __builtin_amdgcn_sched_barrier(0);
    u32x4 ring[KJ];
    const int first = blk0 + wave;
#pragma unroll
    for (int j = 0; j < KJ; j++)
        ring[j] = __builtin_amdgcn_raw_buffer_load_b128(k_rs, lane16, (first * BLK_U4 + j * 64) * 16, 2);

    // (staged while the first K and V blocks are on their way from HBM)
    // q operand (B matrix): slot (j, lane = (head, g)) holds q[h][16j + 8g .. +8) * log2(e)/sqrt(dh),
    // split into bf16 hi (plane 0) and lo (plane 1).  Padded heads duplicate the last one.
#pragma unroll
    for (int it = 0; it < QIT; it++) {
        const int slot = it * 256 + tid;
        const f32x4 a0 = qa0[it] * scale_log2e, a1 = qa1[it] * scale_log2e;
        const uint4 hi = {pack_bf16x2(a0.x, a0.y), pack_bf16x2(a0.z, a0.w), pack_bf16x2(a1.x, a1.y),
                          pack_bf16x2(a1.z, a1.w)};
        const uint4 lo = {pack_bf16x2(a0.x - bf16_lo(hi.x), a0.y - bf16_hi(hi.x)),
                          pack_bf16x2(a0.z - bf16_lo(hi.y), a0.w - bf16_hi(hi.y)),
                          pack_bf16x2(a1.x - bf16_lo(hi.z), a1.y - bf16_hi(hi.z)),
                          pack_bf16x2(a1.z - bf16_lo(hi.w), a1.w - bf16_hi(hi.w))};
        if (slot < KJ * 64) {
            smem[slot] = hi;
            smem[KJ * 64 + slot] = lo;
        }
    }
    __syncthreads();

    for (int blk = first; blk < blk1; blk += 4) {
        const int blk_off = blk * BLK_U4 * 16, next_off = (blk + 4) * BLK_U4 * 16;
        f32x16 S;
#pragma unroll
        for (int r = 0; r < 16; r++) S[r] = 0.f;
#pragma unroll
        for (int j = 0; j < KJ; j++) {
            const bf16x8 kop = __builtin_bit_cast(bf16x8, ring[j]);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                kop, __builtin_bit_cast(bf16x8, smem[j * 64 + lane]), S, 0, 0, 0);
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                kop, __builtin_bit_cast(bf16x8, smem[(KJ + j) * 64 + lane]), S, 0, 0, 0);
            ring[j] = __builtin_amdgcn_raw_buffer_load_b128(v_rs, lane16, blk_off + j * 1024, 2);
        }
        const bool tail = (blk == nblk - 1) && ((P & 31) != 31);
        if (tail) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                int t = blk * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t > P) S[r] = -INFINITY;
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
            // The output accumulators stay in AGPRs for the whole loop (that is what leaves
            // room for the second ring in the vector registers); this rare rescale reads
            // each value out, scales it and writes it back explicitly.  The trailing no-ops
            // cover the wait states between an AGPR write and the MFMA that reads it.
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    float t_;
                    asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                                 : "+a"(O[db][r]), "=&v"(t_)
                                 : "v"(alpha));
                }
            asm volatile("s_nop 4");
        }
        bf16x8 pop[2][2];  // [kk][hi, lo]
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float p0 = S[8 * kk + 2 * e], p1 = S[8 * kk + 2 * e + 1];
                hi[e] = pack_bf16x2(p0, p1);
                lo[e] = pack_bf16x2(p0 - bf16_lo(hi[e]), p1 - bf16_hi(hi[e]));
            }
            pop[kk][0] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
            pop[kk][1] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
        }
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int kk = 0; kk < 2; kk++) {
                u32x4 vr = ring[db * 2 + kk];
                if (tail) {
                    // slots past P may hold anything (even NaN); p is exactly 0 there, so zero V too
                    uint32_t w[4] = {vr.x, vr.y, vr.z, vr.w};
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        int t = blk * 32 + 16 * kk + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (t > P) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                    }
                    vr.x = w[0]; vr.y = w[1]; vr.z = w[2]; vr.w = w[3];
                }
                const bf16x8 vop = __builtin_bit_cast(bf16x8, vr);
                O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[kk][0], O[db], 0, 0, 0);
                O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[kk][1], O[db], 0, 0, 0);
                ring[db * 2 + kk] =
                    __builtin_amdgcn_raw_buffer_load_b128(k_rs, lane16, next_off + (db * 2 + kk) * 1024, 2);
            }
    }
    __syncthreads();  // every wave is done with the q operands: smem becomes the merge buffer

    // ---- merge the 4 waves (a wave without blocks has m = -inf, l = 0, O = 0).  Output
    // block db belongs to wave db % 4: every wave leaves its scaled sums of the blocks it
    // does not own in LDS (one exchange, all waves at once), the owner adds the three
    // contributions to its own in wave order and stores its share of the partial.
    float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    ml_s[wave][lane][0] = m_run;
    ml_s[wave][lane][1] = l_tot;
    __syncthreads();
    float m_all = fmaxf(fmaxf(ml_s[0][lane][0], ml_s[1][lane][0]),
                        fmaxf(ml_s[2][lane][0], ml_s[3][lane][0]));  // finite: wave 0 had a block
    const float f_own = __builtin_amdgcn_exp2f(m_run - m_all);
    f32x4 (*mbuf)[3][4][64] = reinterpret_cast<f32x4 (*)[3][4][64]>(smem);  // [db][source][i][lane]
#pragma unroll
    for (int db = 0; db < DB; db++) {
#pragma unroll
        for (int r = 0; r < 16; r++) O[db][r] *= f_own;
        const int src = (wave - (db & 3) - 1) & 3;  // 0..2 for the three waves that do not own db
        if ((db & 3) != wave) {
#pragma unroll
            for (int i = 0; i < 4; i++)
                mbuf[db][src][i][lane] = (f32x4){O[db][4 * i], O[db][4 * i + 1], O[db][4 * i + 2], O[db][4 * i + 3]};
        }
    }
    __syncthreads();
    const size_t row = ((size_t)b * nsplit + split) * H + l32;
    if (wave == 0 && l32 < H && g == 0) {
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < 4; w++)
            l_all += ml_s[w][lane][1] * __builtin_amdgcn_exp2f(ml_s[w][lane][0] - m_all);
        ml[row * 2 + 0] = m_all;
        ml[row * 2 + 1] = l_all;
    }
    float* orow = opart + row * DH;
#pragma unroll
    for (int db = 0; db < DB; db++) {
        if ((db & 3) != wave) continue;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            f32x4 v = {O[db][4 * i + 0], O[db][4 * i + 1], O[db][4 * i + 2], O[db][4 * i + 3]};
            // contributions in wave order (fixed summation order): sources (wave+1, wave+2, wave+3) % 4
            f32x4 c[3];
#pragma unroll
            for (int k = 0; k < 3; k++) c[k] = mbuf[db][k][i][lane];
            // source index k is wave (owner + 1 + k) % 4; add own and the others by ascending wave
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; w++) {
                const int k = (w - wave - 1) & 3;
                sum += (w == wave) ? v : c[k < 3 ? k : 0];
            }
            if (l32 < H) *reinterpret_cast<f32x4*>(orow + db * 32 + 8 * i + 4 * g) = sum;
        }
    }
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

// G K/V heads per row (1 = multiquery, H = multihead): the attend kernel runs on B*G
// pseudo-sequences of H/G query heads each; q [B][H][dh] and o [B][H*dh] need no reordering.
hipError_t launch_mqa_attend(const float* q, const void* kc_layer, const void* vc_layer,
                             const int32_t* positions, const int32_t* seq, int cache_rows, int B, int H,
                             int G, int dh, int L_ctx, int bps,
                             float* opart, float* ml, float* o, void* actq, float* acts,
                             int k_out, int blk_o, int nd, hipStream_t stream) {
    if (blk_o < 1 || blk_o > 16) return hipErrorInvalidValue;
    if (G < 1 || H % G || H / G > 32 || (long long)B * G > 65535) return hipErrorInvalidValue;
    const int per = H / G;
    const int nblk_cap = L_ctx / 32;
    const int nsplit = (nblk_cap + bps - 1) / bps;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
    dim3 grid(nsplit, B * G), block(256);
    const uint4* k4 = reinterpret_cast<const uint4*>(kc_layer);
    const uint4* v4 = reinterpret_cast<const uint4*>(vc_layer);
    if (dh == 256)
        mqa_attend_kernel<256><<<grid, block, 0, stream>>>(q, k4, v4, positions, seq, cache_rows, per, G, L_ctx, bps, nsplit,
                                                           opart, ml, scale_log2e);
    else if (dh == 128)
        mqa_attend_kernel<128><<<grid, block, 0, stream>>>(q, k4, v4, positions, seq, cache_rows, per, G, L_ctx, bps, nsplit,
                                                           opart, ml, scale_log2e);
    else if (dh == 64)
        mqa_attend_kernel<64><<<grid, block, 0, stream>>>(q, k4, v4, positions, seq, cache_rows, per, G, L_ctx, bps, nsplit,
                                                          opart, ml, scale_log2e);
    else
        return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 cgrid((H * dh / 128 + blk_o - 1) / blk_o, B), cblock(64 * blk_o);  // one wave per chunk
    unsigned char* aq = reinterpret_cast<unsigned char*>(actq);
#define PD_COMB(K) K<<<cgrid, cblock, 0, stream>>>(opart, ml, positions, H, G, dh, L_ctx, bps, nsplit, o, aq, acts, k_out, blk_o, nd)
    if (nsplit <= 4) PD_COMB(mqa_combine_kernel<4>);
    else if (nsplit <= 8) PD_COMB(mqa_combine_kernel<8>);
    else if (nsplit <= 16) PD_COMB(mqa_combine_kernel<16>);
    else PD_COMB(mqa_combine_kernel<0>);
#undef PD_COMB
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
