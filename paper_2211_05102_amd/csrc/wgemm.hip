// bf16-weight skinny GEMM for gfx950: the two fused projections of the parallel block
// (paper Section 3.4) with the weights kept in bf16, the format the int8 weights of
// Section 3.6 are measured against in Section 4.4.
//
//   part[slot][b][n] = sum_{k in a K-range} a[b][k] * w[k][n]        (fp32)
//
// Same contract as the int8 product in qgemm.hip -- the same block fixed-point
// activations in, the same deterministic stream-K plan, the same partial-sum slots
// out -- so every consumer (epilogues, residual, LayerNorm) is shared; the per-channel
// scale vector of such a layer is all ones.
//
// Arithmetic.  A chunk's activations (ND int8 digit planes and a power-of-two scale)
// are rebuilt as the fp32 value they stand for, which is then split exactly into ND
// bf16 planes, hi + mid (+ lo): each plane takes the 8 leading bits of what the
// planes before it left.  v_mfma_f32_32x32x16_bf16 multiplies every plane with the
// raw bf16 weights into ONE fp32 accumulator: products are exact, sums are rounded
// by the matrix pipe in fp32.  (The int8 product keeps exact int32 sums; this one
// cannot, the weights carry their own exponents.)
//
// Data movement.  2 bytes per weight, 2*B flops per weight: HBM-bound by a wide
// margin (64 rows: 3 planes * 2 MFMAs of 32 cycles per KiB of weights and wave).
// Weights are pre-tiled so that a wavefront's 16-byte-per-lane load is 1 KiB
// contiguous and already a B operand:
//   packed[(st*(K/16) + kb)*64 + lane] holds W[kb*16 + (lane/32)*8 + 0..7][st*32 + lane%32].
// 8 wavefronts per workgroup, two 32-column subtiles each (512-column tiles), two per SIMD;
// each keeps one unit (16 KiB) of its weight stream in flight in registers.  The digit
// planes go global -> registers -> (conversion) -> one of two LDS stages shared by the
// 8 waves.
#include "common.h"
#include "kernels.h"

namespace pd {

constexpr int WNT = 512;

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Eight elements of one row: digits (8 bytes per plane, plane 0 most significant) and
// the chunk's scale -> ND bf16 planes of 8 elements each.
template <int ND>
__device__ __forceinline__ void digits_to_bf16_planes(const u32x2 (&dg)[ND], float s, u32x4 (&out)[ND]) {
#pragma unroll
    for (int j = 0; j < 4; j++) {  // elements 2j, 2j+1
        float v[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int e = 2 * j + h;
            int n = 0;
#pragma unroll
            for (int p = 0; p < ND; p++) {
                const uint32_t word = e < 4 ? dg[p].x : dg[p].y;
                const int d = (int)(word << (24 - 8 * (e & 3))) >> 24;  // signed byte e
                n = n * 256 + d;
            }
            v[h] = (float)n * s;  // exact: |n| < 2^23, s a power of two
        }
#pragma unroll
        for (int p = 0; p < ND; p++) {
            const uint32_t w = pack_bf16x2(v[0], v[1]);  // nearest bf16 of what is left
            out[p][j] = w;
            v[0] -= bf16_lo(w);  // exact
            v[1] -= bf16_hi(w);
        }
    }
}

// BM: 32-row batch blocks; ND: digit planes in = bf16 planes fed to the matrix pipe.
// grid = (G workgroups, row groups of 32*BM rows).  Each wavefront owns NS = 2 adjacent
// 32-column subtiles of a 512-column tile (an operand read from LDS feeds two MFMAs) and
// keeps one unit of its weight stream (16 KiB) in registers as a rolling buffer: a 1 KiB
// piece is requested again, for the next unit, as soon as its last MFMA has been issued.
template <int BM, int ND, int WAUX>
__global__ __launch_bounds__(WNT) void wgemm_bf16_kernel(const uint4* __restrict__ wp,
                                                          const unsigned char* __restrict__ qa,
                                                          const float* __restrict__ scale_t,
                                                          float* __restrict__ part, int B, int K, int N,
                                                          SkqPlan pl) {
    constexpr int KC = QCHUNK;                 // k-extent of one unit = one LDS stage
    constexpr int NS = 2;                      // 32-column subtiles per wave
    constexpr int ROWS = BM * 32;
    constexpr int PITCH = ND * KC * 2 + 16;    // bytes per row: ND bf16 planes; +16 spreads rows over banks
    constexpr int PPR = KC / 8;                // 8-element pieces per row
    constexpr int NPIECE = ROWS * PPR;
    constexpr int APT = NPIECE / WNT;          // pieces per thread per stage
    constexpr int KB = KC / 16;                // 16-k blocks (1 KiB per wave and subtile each) per unit
    constexpr int TSUB = (WNT / 64) * NS;      // 32-column subtiles per tile
    constexpr int STAGE = ROWS * PITCH;
    static_assert(TSUB * 32 == PD_WGEMM_TILE_COLS, "the plan's tiles are this kernel's tiles");
    static_assert(NPIECE % WNT == 0 && APT >= 1, "pieces divide over the threads");
    static_assert(2 * STAGE <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;
    const int n_sub = N >> 5;
    const int C = pl.C;
    const int* rec = pl.nseg + skq_wg_offset(pl.T) + 4 * (int)blockIdx.x;
    const int u0 = __builtin_amdgcn_readfirstlane(rec[0]);
    const int u1 = __builtin_amdgcn_readfirstlane(rec[1]);
    if (u0 >= u1) return;
    int slot = __builtin_amdgcn_readfirstlane(rec[2]);
    int t_cur = __builtin_amdgcn_readfirstlane(rec[3]);
    int c_cur = u0 - t_cur * C;
    const int row0 = blockIdx.y * ROWS;

    // every global access is a buffer access: scalar descriptor + scalar offset that moves
    // with the unit + a per-lane offset that never changes; reads past the end give zero
    const uint32_t lane16 = lane * 16;
    const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(reinterpret_cast<const unsigned char*>(wp)), 0,
        (int)((uint32_t)n_sub * (uint32_t)K * 64u), 0x00020000);
    const __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(qa), 0, B * K * ND, 0x00020000);
    const __amdgpu_buffer_rsrc_t s_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(scale_t), 0, C * QSCALE_ROWS * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t p_rs = __builtin_amdgcn_make_buffer_rsrc(
        part, 0, (int)((uint32_t)pl.max_slots * (uint32_t)pl.rows * (uint32_t)N * 4u), 0x00020000);

    // (tile, chunk) of the next weight unit to fetch and chunk of the next activation stage to
    // load; both saturate at the last unit of the range (fetching it again is an L2 hit)
    int u_w = u0, t_w = t_cur, c_w = c_cur, u_a = u0, c_a = c_cur;
    uint32_t wo[NS];  // byte offsets of the unit's two 8 KiB pieces in the packed matrix
    auto w_next = [&]() {
#pragma unroll
        for (int i = 0; i < NS; i++) {
            int st = t_w * TSUB + wave * NS + i;
            st = st < n_sub ? st : n_sub - 1;  // ragged last tile: result dropped at the store
            wo[i] = (uint32_t)st * (uint32_t)(K * 64) + (uint32_t)c_w * (uint32_t)(KC * 64);
        }
        if (u_w < u1 - 1) {
            u_w++;
            if (++c_w == C) { c_w = 0; t_w++; }
        }
    };
    auto a_next = [&]() {
        const int c = c_a;
        if (u_a < u1 - 1) {
            u_a++;
            if (++c_a == C) c_a = 0;
        }
        return c;
    };
    // pieces of an activation stage this thread converts; rows >= B repeat row B - 1
    uint32_t aoff[APT], aslot[APT], soff[APT];
#pragma unroll
    for (int it = 0; it < APT; it++) {
        const int p_ = it * WNT + tid;
        aslot[it] = (p_ / PPR) * PITCH + (p_ % PPR) * 16;
        int rg = row0 + p_ / PPR;
        rg = rg < B ? rg : B - 1;
        aoff[it] = (uint32_t)rg * (uint32_t)(K * ND) + (p_ % PPR) * 8;
        soff[it] = rg * 4;
    }

    u32x4 ring[NS][KB];
    u32x2 areg[APT][ND];
    float sreg[APT];
    f32x16 acc[BM][NS];
#pragma unroll
    for (int bm = 0; bm < BM; bm++)
#pragma unroll
        for (int i = 0; i < NS; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[bm][i][r] = 0.f;

    // digits and scales of the next activation chunk -> registers
#define W_ALOAD()                                                                        \
    {                                                                                    \
        const int c_ = a_next();                                                         \
        _Pragma("unroll") for (int it = 0; it < APT; it++) {                             \
            _Pragma("unroll") for (int p = 0; p < ND; p++)                               \
                areg[it][p] = __builtin_amdgcn_raw_buffer_load_b64(a_rs, aoff[it] + p * KC, c_ * (ND * KC), 0); \
            sreg[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(s_rs, soff[it], c_ * (QSCALE_ROWS * 4), 0)); \
        }                                                                                \
    }
    // registers -> bf16 planes -> LDS stage
#define W_ASTORE(buf)                                                                    \
    {                                                                                    \
        _Pragma("unroll") for (int it = 0; it < APT; it++) {                             \
            u32x4 pl_[ND];                                                               \
            digits_to_bf16_planes<ND>(areg[it], sreg[it], pl_);                          \
            _Pragma("unroll") for (int p = 0; p < ND; p++)                               \
                *reinterpret_cast<u32x4*>(&lds[buf][aslot[it] + p * (KC * 2)]) = pl_[p]; \
        }                                                                                \
    }

    // fill: the first unit's weights, its activation stage, the digits of the second unit
    W_ALOAD()
    w_next();
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int i = 0; i < NS; i++)
            ring[i][kb] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, lane16 + kb * 1024, wo[i], WAUX);
    W_ASTORE(0)
    W_ALOAD()
    // Everything requested so far is waited for here, once: the compiler derives the wait at
    // the head of the unit loop from all paths that reach it, and merged with this path it
    // would otherwise drain the weight buffer on every turn.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    lds_barrier();

    int cur = 0;
    for (int u = u0; u < u1; u++) {
        // One unit: stage `cur` against the weight buffer.  First the next unit's stage is
        // written and the digits of the unit after that are requested.
        W_ASTORE(cur ^ 1)
        W_ALOAD()
        w_next();  // wo[]: where the next unit's pieces are
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < KB; kb++) {
            const bf16x8 b0 = __builtin_bit_cast(bf16x8, ring[0][kb]);
            const bf16x8 b1 = __builtin_bit_cast(bf16x8, ring[1][kb]);
#pragma unroll
            for (int p = 0; p < ND; p++) {
#pragma unroll
                for (int bm = 0; bm < BM; bm++) {
                    const bf16x8 a_ = *reinterpret_cast<const bf16x8*>(
                        &lds[cur][(bm * 32 + l32) * PITCH + p * (KC * 2) + kb * 32 + g * 16]);
                    acc[bm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b0, acc[bm][0], 0, 0, 0);
                    acc[bm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b1, acc[bm][1], 0, 0, 0);
                }
            }
            ring[0][kb] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, lane16 + kb * 1024, wo[0], WAUX);
            ring[1][kb] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, lane16 + kb * 1024, wo[1], WAUX);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();
        cur ^= 1;
        // The part of a tile inside this range is done: store its fp32 sums as this range's
        // partial of the tile.  D layout of the 32x32 MFMA: register r of lane (l32, g) is row
        // 8*(r/4) + 4*g + r%4, column l32.
        if (++c_cur == C || u + 1 == u1) {
            const uint32_t rowb = (uint32_t)N * 4u;
#pragma unroll
            for (int i = 0; i < NS; i++) {
                const int st = t_cur * TSUB + wave * NS + i;
#pragma unroll
                for (int bm = 0; bm < BM; bm++)
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        const uint32_t row = (uint32_t)(slot * pl.rows + row0 + bm * 32 + 8 * (r >> 2) + 4 * g + (r & 3));
                        const float f_ = acc[bm][i][r];  // (a bit cast of a vector element lvalue reads element 0)
                        if (st < n_sub)
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, f_), p_rs,
                                                                  row * rowb + (uint32_t)(st * 128 + l32 * 4), 0,
                                                                  PD_WRITE_THROUGH);
                        acc[bm][i][r] = 0.f;
                    }
            }
            if (c_cur == C) { c_cur = 0; t_cur++; slot = 0; }
        }
    }
#undef W_ALOAD
#undef W_ASTORE
}

// canonical bf16 [K][N] -> the packed operand order above, columns through the same
// map as the int8 matrices (interleaved gate/up for the input projection)
__global__ __launch_bounds__(256) void pack_matrix_bf16_kernel(const uint16_t* __restrict__ w,
                                                               uint4* __restrict__ dst, int K, int N,
                                                               int mode, int n_qkv, int F) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)(N >> 5) * (K >> 4) * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    size_t t = idx >> 6;
    int kb = (int)(t % (size_t)(K >> 4));
    int st = (int)(t / (size_t)(K >> 4));
    int n = packed_col_map(st * 32 + (lane & 31), mode, n_qkv, F);
    int k0 = kb * 16 + (lane >> 5) * 8;
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; j++) {
        uint32_t h = w[(size_t)(k0 + j) * N + n];
        o[j >> 1] |= h << (16 * (j & 1));
    }
    dst[idx] = make_uint4(o[0], o[1], o[2], o[3]);
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float* __restrict__ dst, int n, float v) {
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = v;
}

hipError_t launch_wgemm_bf16(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                             int K, int N, SkqPlan pl, int nd, hipStream_t stream) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    if (pl.tile_cols != PD_WGEMM_TILE_COLS) return hipErrorInvalidValue;  // the plan's tiles are this kernel's tiles
    dim3 grid(pl.G, (B + 32 * bm - 1) / (32 * bm)), block(WNT);
    const uint4* w4 = reinterpret_cast<const uint4*>(wp);
    const unsigned char* q = reinterpret_cast<const unsigned char*>(qa);
    if (nd != 2 && nd != 3) return hipErrorInvalidValue;
    // buffer descriptors address 32 bits
    if ((long long)B * K * nd >= (1ll << 31) || (long long)K * N * 2 >= (1ll << 32)) return hipErrorInvalidValue;
    if ((long long)pl.T * pl.C >= (1ll << 31)) return hipErrorInvalidValue;
    if ((long long)pl.max_slots * pl.rows * N * 4 >= (1ll << 32)) return hipErrorInvalidValue;
#define PD_LAUNCH(BMv, WAUXv)                                                                          \
    do {                                                                                               \
        if (nd == 3)                                                                                   \
            wgemm_bf16_kernel<BMv, 3, WAUXv><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, pl); \
        else                                                                                           \
            wgemm_bf16_kernel<BMv, 2, WAUXv><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, pl); \
    } while (0)
    if (bm == 1) PD_LAUNCH(1, 2);
    else if (grid.y > 1) PD_LAUNCH(2, 0);  // several row groups read the weights: leave them cacheable
    else PD_LAUNCH(2, 2);
#undef PD_LAUNCH
    return hipGetLastError();
}

hipError_t launch_pack_matrix_bf16(const uint16_t* w, void* dst, int K, int N, int mode, int n_qkv, int F,
                                   hipStream_t stream) {
    size_t total = (size_t)(N / 32) * (K / 16) * 64;
    pack_matrix_bf16_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        w, reinterpret_cast<uint4*>(dst), K, N, mode, n_qkv, F);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float* dst, int n, float v, hipStream_t stream) {
    fill_f32_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(dst, n, v);
    return hipGetLastError();
}

}  // namespace pd
