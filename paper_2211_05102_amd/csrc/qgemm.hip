// int8-weight skinny GEMM for gfx950 (paper Section 3.6: weights stored int8
// with one scale per output channel; Section 3.4: the fused input and output
// projections of the parallel block are the two instances of this product).
//
//   part[slot][b][n] = sum_{k in a K-range} a[b][k] * q8[k][n]        (fp32, unscaled)
//
// The per-channel weight scale s[n] is applied once per output by the consumer
// of the partial sums, which is exact because it does not depend on k.
//
// Arithmetic.  Activations arrive in block fixed point (common.h): ND int8 digit
// planes and a power-of-two scale per (row, 128-k chunk).  Every digit plane goes
// through v_mfma_i32_32x32x32_i8 against the raw int8 weights -- no weight
// conversion, exact int32 sums, one int32 accumulator per plane -- and every
// `fold_chunks` chunks (over which the producer keeps the scale constant) the
// planes are folded into the fp32 accumulator:
//     acc += scale[b] * (65536 * float(top) + 256 * float(mid) + float(low)).
// ND = 3 gives 23-bit activations (bf16 rounding of the LayerNorm and SwiGLU
// outputs would otherwise dominate the error of a deep stack) for 1.5x the MFMA
// time of a single bf16 pass.
//
// Data movement (HBM-bound: 1 byte per weight, 2*B flops per byte).
//   - weights are pre-tiled by pd_pack_* so that a wavefront's 16-byte-per-lane
//     load is 1 KiB contiguous and is already an MFMA B operand:
//     packed[(st*(K/32) + kb)*64 + lane] holds W[kb*32 + (lane/32)*16 + 0..15][st*32 + lane%32];
//     each wave keeps PF units of its weight stream in flight in registers;
//   - activations (and their scales) are shared by the 4 waves through LDS.
// A = activations (M = batch row), B = weights (N = output channel).
//
// Work split (deterministic stream-K).  The matrix is cut into units = (tile of
// 128*NS columns, 128-k chunk), ordered tile-major; workgroup g of G takes the
// contiguous range [g*U/G, (g+1)*U/G).  All workgroups stream the same number of
// bytes (+-1 unit), whatever the matrix shape.  A tile covered by several
// workgroups gets one partial per workgroup, in slot (g - first g of the tile);
// consumers add the slots in index order, so results do not depend on timing.
#include "common.h"
#include "kernels.h"

namespace pd {

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains
// every outstanding global load (vmcnt(0)), which would serialise the weight
// prefetch with each unit; here only the LDS counter is waited on.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// BM: 32-row batch blocks held in accumulators; NS: 32-column subtiles per wave;
// R: weight units per wave held in a register ring (R - 1 in flight while one is
// consumed).  grid = (G workgroups, row groups of 32*BM rows).
//
// Weights go HBM -> registers with non-temporal 16-byte loads (each is 1 KiB
// contiguous per wave and already a B operand); the loop body is unrolled R
// times so every ring slot is a fixed register range and the compiler's own
// vmcnt bookkeeping keeps exactly R - 1 units in flight.  Every step issues the
// same loads unconditionally (past the end of the range the last unit is
// fetched again, an L2 hit) so that no control-flow join weakens those waits.
// Activations of the next unit travel L2 -> registers -> LDS behind the MFMAs
// of the current one and are shared by the 4 waves.
constexpr int NT = 512;  // threads per GEMM workgroup (8 waves, two per SIMD)

template <int BM, int NS, int ND, int R>
__global__ __launch_bounds__(NT) void qgemm_kernel(const uint4* __restrict__ wp,
                                                    const unsigned char* __restrict__ qa,
                                                    const float* __restrict__ scale_t,
                                                    float* __restrict__ part, int B, int K, int N,
                                                    int c_split, int blk0, int blk1) {
    constexpr int KC = QCHUNK;                  // k-extent of one unit = one LDS stage
    constexpr int ROWS = BM * 32;
    constexpr int PITCH = ND * KC + 16;         // bytes; +16 spreads rows over LDS banks
    constexpr int PPR = ND * KC / 16;           // 16-byte pieces per row per stage
    constexpr int APT = (ROWS * PPR + NT - 1) / NT;  // pieces per thread per stage (tail repeats the last piece)
    constexpr int KB = KC / 32;                 // 32-k blocks per unit
    constexpr int TSUB = (NT / 64) * NS;        // 32-column subtiles per tile
    constexpr int STAGE = ROWS * PITCH + ROWS * 4;  // digits + one scale per row
    static_assert(R == 2 || R == 4 || R == 6, "ring depth (even: the activation register stages alternate)");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][STAGE];
    // fp32 tile accumulator, one private column per thread: it is touched only when
    // a scale block or a tile ends, so it lives in LDS and leaves the registers to
    // the int32 accumulators and the weight ring
    __shared__ float accl[NS * BM * 16][NT];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int n_sub = N >> 5;
    const int kblocks = K >> 5;
    const int C = K >> 7;                                   // chunks per tile
    const int T = (n_sub + TSUB - 1) / TSUB;                // tiles
    const long long U = (long long)T * C;
    const int G = gridDim.x;
    const long long u0 = (long long)blockIdx.x * U / G, u1 = ((long long)blockIdx.x + 1) * U / G;
    if (u0 >= u1) return;
    const int row0 = blockIdx.y * ROWS;

    // byte offsets (within one chunk column of the activation matrix) of the pieces
    // this thread moves; rows >= B repeat row B-1 (their results are never stored)
    uint32_t aoff[APT], aslot[APT];
#pragma unroll
    for (int it = 0; it < APT; it++) {
        int p_ = it * NT + tid;
        p_ = p_ < ROWS * PPR ? p_ : ROWS * PPR - 1;
        aslot[it] = (p_ / PPR) * PITCH + (p_ % PPR) * 16;
        int rg = row0 + p_ / PPR;
        rg = rg < B ? rg : B - 1;
        aoff[it] = (uint32_t)rg * (uint32_t)(K * ND) + (p_ % PPR) * 16;
    }
    int srow = row0 + tid;
    srow = srow < B ? srow : B - 1;

    i32x16 iacc[ND][NS][BM];
#pragma unroll
    for (int i = 0; i < NS; i++)
#pragma unroll
        for (int bm = 0; bm < BM; bm++) {
#pragma unroll
            for (int r = 0; r < 16; r++) accl[(i * BM + bm) * 16 + r][tid] = 0.f;
#pragma unroll
            for (int p = 0; p < ND; p++)
#pragma unroll
                for (int r = 0; r < 16; r++) iacc[p][i][bm][r] = 0;
        }

    uint4 wreg[R][NS][KB];
    const uint4* wsrc[NS];
    u32x4 areg[2][APT];
    float sreg[2] = {0.f, 0.f};

    // (tile, chunk) of the unit being computed; of the next weight unit to fetch
    // (saturates at the last unit of the range); chunk of the next activation stage
    int t_cur = (int)(u0 / C), c_cur = (int)(u0 % C);
    int t_w = t_cur, c_w = c_cur, c_a = c_cur;
    long long u = u0, u_w = u0, u_a = u0;

    // end of the scale block that holds chunk c: chunks [0, c_split) come in blocks
    // of blk0, chunks [c_split, C) in blocks of blk1
    auto block_end = [&](int c) {
        int e;
        if (c < c_split) {
            e = (c / blk0 + 1) * blk0;
            e = e < c_split ? e : c_split;
        } else {
            e = c_split + ((c - c_split) / blk1 + 1) * blk1;
            e = e < C ? e : C;
        }
        return e;
    };
    int seg_end = block_end(c_cur);

    // weight unit (t_w, c_w) -> ring slot s, one 32-k block at a time
#define PD_W_PTRS()                                                                      \
    _Pragma("unroll") for (int i = 0; i < NS; i++) {                                     \
        int st_ = t_w * TSUB + wave * NS + i;                                            \
        st_ = st_ < n_sub ? st_ : n_sub - 1; /* ragged last tile: result dropped */      \
        wsrc[i] = wp + ((size_t)st_ * kblocks + (size_t)c_w * KB) * 64 + lane;           \
    }
#define PD_W_LOAD(s, kb)                                                                 \
    _Pragma("unroll") for (int i = 0; i < NS; i++) wreg[s][i][kb] = ld_stream(wsrc[i] + (kb) * 64);
#define PD_W_NEXT()                                                                      \
    if (u_w + 1 < u1) {                                                                  \
        u_w++;                                                                           \
        if (++c_w == C) { c_w = 0; t_w++; }                                              \
    }
#define PD_FETCH_W(s)                                                                    \
    {                                                                                    \
        PD_W_PTRS()                                                                      \
        _Pragma("unroll") for (int kb = 0; kb < KB; kb++) { PD_W_LOAD(s, kb) }           \
        PD_W_NEXT()                                                                      \
    }
    // activations of the unit two steps ahead -> register stage `as`; vector-memory
    // operations retire in order, so a load that is waited on must be older than
    // everything that is meant to stay in flight: these loads are consumed one step
    // after they are issued, with R - 1 weight units still outstanding behind them
#define PD_LOAD_A(as)                                                                    \
    {                                                                                    \
        if (u_a + 1 < u1) {                                                              \
            u_a++;                                                                       \
            if (++c_a == C) c_a = 0;                                                     \
        }                                                                                \
        const unsigned char* base_ = qa + (size_t)c_a * (ND * KC);                       \
        _Pragma("unroll") for (int it = 0; it < APT; it++)                               \
            areg[as][it] = *reinterpret_cast<const u32x4*>(base_ + aoff[it]);            \
        if (tid < ROWS) sreg[as] = scale_t[(size_t)c_a * QSCALE_ROWS + srow];            \
    }
#define PD_STORE_A(buf, as)                                                              \
    {                                                                                    \
        _Pragma("unroll") for (int it = 0; it < APT; it++)                               \
            *reinterpret_cast<u32x4*>(&lds[buf][aslot[it]]) = areg[as][it];              \
        if (tid < ROWS) *reinterpret_cast<float*>(&lds[buf][ROWS * PITCH + tid * 4]) = sreg[as]; \
    }
    // One unit of MFMAs.  Group gi = (kb, plane p): BM operand reads from LDS feed
    // NS*BM MFMAs; the reads run two groups ahead of the MFMAs, and scheduling
    // barriers keep that order (left alone, the scheduler hoists every read of the
    // unit and runs out of registers).  As soon as the last plane of a 32-k block
    // is issued, the ring registers of that block are refilled from the next unit.
    // Plane 0 of a row chunk is the most significant digit.
#define PD_A_READ(buf, gi, slot)                                                         \
    _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                                    \
        aop[slot][bm] = *reinterpret_cast<const i32x4*>(                                 \
            &lds[buf][(bm * 32 + l32) * PITCH + ((gi) % ND) * KC + ((gi) / ND) * 32 + g * 16]);
#define PD_MFMA(buf, s)                                                                  \
    {                                                                                    \
        i32x4 aop[3][BM];                                                                \
        PD_W_PTRS()                                                                      \
        PD_A_READ(buf, 0, 0)                                                             \
        PD_A_READ(buf, 1, 1)                                                             \
        _Pragma("unroll") for (int gi = 0; gi < KB * ND; gi++) {                         \
            if (gi + 2 < KB * ND) { PD_A_READ(buf, gi + 2, (gi + 2) % 3) }               \
            _Pragma("unroll") for (int i = 0; i < NS; i++)                               \
                _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                        \
                    iacc[gi % ND][i][bm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(        \
                        aop[gi % 3][bm], __builtin_bit_cast(i32x4, wreg[s][i][gi / ND]), \
                        iacc[gi % ND][i][bm], 0, 0, 0);                                  \
            if (gi % ND == ND - 1) { PD_W_LOAD(s, gi / ND) }                             \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
        PD_W_NEXT()                                                                      \
    }
    // acc += scale * sum_p 256^(ND-1-p) * float(iacc[p]); iacc = 0.  int32 bound per
    // plane and scale block: 128 * 127 * 128 * chunks < 2^31 for blocks of up to 1023
    // chunks.  Lane (l32, g) holds rows 8q + 4g + 0..3 of each 32-row block.
#define PD_FOLD(buf)                                                                     \
    _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                                  \
        f32x4 sc[4];                                                                     \
        _Pragma("unroll") for (int q = 0; q < 4; q++)                                    \
            sc[q] = *reinterpret_cast<const f32x4*>(                                     \
                &lds[buf][ROWS * PITCH + (bm * 32 + 8 * q + 4 * g) * 4]);                \
        _Pragma("unroll") for (int i = 0; i < NS; i++) {                                 \
            _Pragma("unroll") for (int r = 0; r < 16; r++) {                             \
                float v_ = (float)iacc[0][i][bm][r];                                     \
                _Pragma("unroll") for (int p = 1; p < ND; p++)                           \
                    v_ = v_ * 256.0f + (float)iacc[p][i][bm][r];                         \
                accl[(i * BM + bm) * 16 + r][tid] += sc[r >> 2][r & 3] * v_;             \
                _Pragma("unroll") for (int p = 0; p < ND; p++) iacc[p][i][bm][r] = 0;    \
            }                                                                            \
            __builtin_amdgcn_sched_barrier(0); /* one tile at a time: bounded live set */ \
        }                                                                                \
    }
    // D layout of the 32x32 MFMA: register r of lane (l32, g) is row 8*(r/4) + 4*g + r%4, column l32
#define PD_STORE_TILE()                                                                  \
    {                                                                                    \
        const int slot_ = (int)blockIdx.x - skq_owner((long long)t_cur * C, U, G);       \
        _Pragma("unroll") for (int i = 0; i < NS; i++) {                                 \
            const int st_ = t_cur * TSUB + wave * NS + i;                                \
            if (st_ < n_sub) {                                                           \
                const int n_ = st_ * 32 + l32;                                           \
                _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                      \
                    _Pragma("unroll") for (int r = 0; r < 16; r++) {                     \
                        const int b_ = row0 + bm * 32 + 8 * (r >> 2) + 4 * g + (r & 3);  \
                        if (b_ < B)                                                      \
                            part[((size_t)slot_ * B + b_) * N + n_] = accl[(i * BM + bm) * 16 + r][tid]; \
                    }                                                                    \
                    __builtin_amdgcn_sched_barrier(0);                                   \
                }                                                                        \
            }                                                                            \
            _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                            \
                _Pragma("unroll") for (int r = 0; r < 16; r++)                           \
                    accl[(i * BM + bm) * 16 + r][tid] = 0.f;                             \
        }                                                                                \
    }
    // One unit: fetch the next activation stage into registers, multiply the current
    // one, refill the ring slot just consumed, close a scale block / tile if this
    // unit ended one (the scales are read before the barrier: afterwards another
    // wave may already overwrite this stage), publish the next stage.
#define PD_STEP(s)                                                                       \
    {                                                                                    \
        PD_LOAD_A((s) % 2)                                                               \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PD_MFMA(cur, s)                                                                  \
        c_cur++;                                                                         \
        u++;                                                                             \
        if (c_cur == seg_end || u == u1) {                                               \
            PD_FOLD(cur)                                                                 \
            if (c_cur == C || u == u1) {                                                 \
                PD_STORE_TILE()                                                          \
                if (c_cur == C) { c_cur = 0; t_cur++; }                                  \
            }                                                                            \
            seg_end = block_end(c_cur);                                                  \
        }                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PD_STORE_A(cur ^ 1, ((s) + 1) % 2)                                               \
        lds_barrier();                                                                   \
        cur ^= 1;                                                                        \
    }

    // prologue: activations of the first unit straight into stage 0, those of the
    // second into register stage 1 (where step 0 expects them), R weight units in flight
    {
        const unsigned char* base_ = qa + (size_t)c_a * (ND * KC);
#pragma unroll
        for (int it = 0; it < APT; it++) areg[0][it] = *reinterpret_cast<const u32x4*>(base_ + aoff[it]);
        if (tid < ROWS) sreg[0] = scale_t[(size_t)c_a * QSCALE_ROWS + srow];
    }
    PD_STORE_A(0, 0)
    PD_LOAD_A(1)
    PD_FETCH_W(0)
    PD_FETCH_W(1)
    if constexpr (R > 2) { PD_FETCH_W(2) }
    if constexpr (R > 3) { PD_FETCH_W(3) }
    if constexpr (R > 4) { PD_FETCH_W(4) }
    if constexpr (R > 5) { PD_FETCH_W(5) }
    lds_barrier();

    int cur = 0;
    for (;;) {
        PD_STEP(0)
        if (u == u1) break;
        PD_STEP(1)
        if (u == u1) break;
        if constexpr (R > 2) {
            PD_STEP(2)
            if (u == u1) break;
        }
        if constexpr (R > 3) {
            PD_STEP(3)
            if (u == u1) break;
        }
        if constexpr (R > 4) {
            PD_STEP(4)
            if (u == u1) break;
        }
        if constexpr (R > 5) {
            PD_STEP(5)
            if (u == u1) break;
        }
    }
#undef PD_FETCH_W
#undef PD_W_PTRS
#undef PD_W_LOAD
#undef PD_W_NEXT
#undef PD_A_READ
#undef PD_LOAD_A
#undef PD_STORE_A
#undef PD_MFMA
#undef PD_FOLD
#undef PD_STORE_TILE
#undef PD_STEP
}

// bf16 [B][K] -> block fixed point (test entry pd_qgemm): one wave per (row, chunk)
__global__ __launch_bounds__(256) void quantize_bf16_kernel(const uint16_t* __restrict__ a,
                                                            unsigned char* __restrict__ qa,
                                                            float* __restrict__ scale_t, int K,
                                                            int nd) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.y, j = blockIdx.x * 4 + wave;
    if (j >= (K >> 7)) return;
    const uint32_t two = *reinterpret_cast<const uint32_t*>(a + (size_t)b * K + j * QCHUNK + 2 * lane);
    quantize_chunk_wave(bf16_lo(two), bf16_hi(two), lane, nd,
                        qa + ((size_t)b * K + (size_t)j * QCHUNK) * nd,
                        scale_t + (size_t)j * QSCALE_ROWS + b);
}

// ---- packing ----------------------------------------------------------------

// Column map of the fused input projection: packed column -> canonical column.
// q|k|v keep their place; gate and up are interleaved in 32-column groups
// (gate group m, then up group m) so one workgroup sees both halves of a
// SwiGLU pair.  mode 0 = identity.
__device__ __forceinline__ int col_map(int pn, int mode, int n_qkv, int F) {
    if (mode == 0 || pn < n_qkv) return pn;
    int r = pn - n_qkv, pair = r >> 6, within = r & 63;
    return within < 32 ? n_qkv + pair * 32 + within : n_qkv + F + pair * 32 + (within - 32);
}

__global__ __launch_bounds__(256) void pack_matrix_kernel(const int8_t* __restrict__ w,
                                                          uint4* __restrict__ dst, int K, int N,
                                                          int mode, int n_qkv, int F) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)(N >> 5) * (K >> 5) * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    size_t t = idx >> 6;
    int kb = (int)(t % (size_t)(K >> 5));
    int st = (int)(t / (size_t)(K >> 5));
    int n = col_map(st * 32 + (lane & 31), mode, n_qkv, F);
    int k0 = kb * 32 + (lane >> 5) * 16;
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 16; j++) {
        uint32_t byte = (uint8_t)w[(size_t)(k0 + j) * N + n];
        o[j >> 2] |= byte << (8 * (j & 3));
    }
    dst[idx] = make_uint4(o[0], o[1], o[2], o[3]);
}

__global__ __launch_bounds__(256) void pack_vector_kernel(const uint16_t* __restrict__ src,
                                                          float* __restrict__ dst, int N, int mode,
                                                          int n_qkv, int F) {
    int pn = blockIdx.x * 256 + threadIdx.x;
    if (pn < N) dst[pn] = from_bf16(src[col_map(pn, mode, n_qkv, F)]);
}

// out[b][n] = scale[n] * sum over the slots of n's tile (fixed order)
__global__ __launch_bounds__(256) void qgemm_reduce_kernel(const float* __restrict__ part,
                                                           const float* __restrict__ scale,
                                                           float* __restrict__ out, int B, int N,
                                                           SkqPlan pl) {
    int n = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (n >= N) return;
    const int ns = skq_slots(n / pl.tile_cols, pl.C, pl.T, pl.G);
    float acc = 0.f;
    for (int s = 0; s < ns; s++) acc += part[((size_t)s * B + b) * N + n];
    out[(size_t)b * N + n] = scale[n] * acc;
}

// ---- host launchers -----------------------------------------------------------

void qgemm_config(int B, int* bm, int* ns, int* tile_cols) {
    int blocks = (B + 31) / 32;
    *bm = blocks <= 1 ? 1 : 2;  // more than 64 rows: several row groups
    *ns = 1;
    *tile_cols = (NT / 64) * 32 * *ns;
}

SkqPlan qgemm_skq(int B, int K, int N, int G) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    return SkqPlan{tc, K / 128, (N + tc - 1) / tc, G};
}

// Workgroups per row group and partial slots per tile for a [K][N] projection.
void qgemm_plan(int B, int K, int N, int num_cus, int* G, int* slots) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    const int T = (N + tc - 1) / tc, C = K / 128;
    const long long U = (long long)T * C;
    long long g = num_cus;
    if (g > U) g = U;
    // a tile is shared by at most ceil(G / T) + 1 workgroups: keep that within PD_MAX_SPLITS
    const long long cap = (long long)(PD_MAX_SPLITS - 1) * T;
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    int mx = 1;
    for (int t = 0; t < T; t++) {
        int n = skq_owner((long long)(t + 1) * C - 1, U, (int)g) - skq_owner((long long)t * C, U, (int)g) + 1;
        if (n > mx) mx = n;
    }
    *G = (int)g;
    *slots = mx;
}

hipError_t launch_qgemm(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                        int K, int N, int G, int c_split, int blk0, int blk1, int nd,
                        hipStream_t stream) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    dim3 grid(G, (B + 32 * bm - 1) / (32 * bm)), block(NT);
    const uint4* w4 = reinterpret_cast<const uint4*>(wp);
    const unsigned char* q = reinterpret_cast<const unsigned char*>(qa);
#define PD_LAUNCH(BMv, NSv, PD_RING)                                                                 \
    do {                                                                                    \
        if (nd == 3)                                                                        \
            qgemm_kernel<BMv, NSv, 3, PD_RING><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, c_split, blk0, blk1); \
        else                                                                                \
            qgemm_kernel<BMv, NSv, 2, PD_RING><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, c_split, blk0, blk1); \
    } while (0)
    if (nd != 2 && nd != 3) return hipErrorInvalidValue;
    if (blk0 < 1 || blk0 > 1024 || blk1 < 1 || blk1 > 1024 || c_split < 0 || c_split > K / 128)
        return hipErrorInvalidValue;
    if (bm == 1) PD_LAUNCH(1, 1, 6);
    else PD_LAUNCH(2, 1, 2);
#undef PD_LAUNCH
    return hipGetLastError();
}

hipError_t launch_quantize_bf16(const uint16_t* a, void* qa, float* scale_t, int B, int K, int nd,
                                hipStream_t stream) {
    quantize_bf16_kernel<<<dim3((K / 128 + 3) / 4, B), dim3(256), 0, stream>>>(
        a, reinterpret_cast<unsigned char*>(qa), scale_t, K, nd);
    return hipGetLastError();
}

hipError_t launch_pack_matrix(const int8_t* w, void* dst, int K, int N, int mode, int n_qkv, int F,
                              hipStream_t stream) {
    size_t total = (size_t)(N / 32) * (K / 32) * 64;
    pack_matrix_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
        w, reinterpret_cast<uint4*>(dst), K, N, mode, n_qkv, F);
    return hipGetLastError();
}

hipError_t launch_pack_vector(const uint16_t* src, float* dst, int N, int mode, int n_qkv, int F,
                              hipStream_t stream) {
    pack_vector_kernel<<<dim3((N + 255) / 256), dim3(256), 0, stream>>>(src, dst, N, mode, n_qkv, F);
    return hipGetLastError();
}

hipError_t launch_qgemm_reduce(const float* part, const float* scale, float* out, int B, int K,
                               int N, int G, hipStream_t stream) {
    qgemm_reduce_kernel<<<dim3((N + 255) / 256, B), dim3(256), 0, stream>>>(
        part, scale, out, B, N, qgemm_skq(B, K, N, G));
    return hipGetLastError();
}

}  // namespace pd
