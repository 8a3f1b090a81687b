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
// planes and a power-of-two scale per (row, 128-k chunk), constant over a scale
// block of chunks.  Every digit plane goes through v_mfma_i32_32x32x32_i8 against
// the raw int8 weights -- no weight conversion, exact int32 sums, one int32
// accumulator per plane -- and at the end of a scale block the planes are folded
// into the fp32 sums of the tile:
//     acc += scale[b] * (65536 * float(top) + 256 * float(mid) + float(low)).
// ND = 3 gives 23-bit activations (bf16 rounding of the LayerNorm and SwiGLU
// outputs would otherwise dominate the error of a deep stack) for 1.5x the MFMA
// time of a single bf16 pass.
//
// Data movement (HBM-bound: 1 byte per weight, 2*B flops per byte).
//   - weights are pre-tiled by pd_pack_* so that a wavefront's 16-byte-per-lane
//     load is 1 KiB contiguous and is already an MFMA B operand:
//     packed[(st*(K/32) + kb)*64 + lane] holds W[kb*32 + (lane/32)*16 + 0..15][st*32 + lane%32];
//     each wave keeps R units of its weight stream in flight in registers;
//   - activations (and their scales) are shared by the 4 waves through LDS.
// A = activations (M = batch row), B = weights (N = output channel).
//
// Work split (deterministic stream-K).  The matrix is cut into units = (tile of
// 128*NS columns, 128-k chunk), ordered tile-major; workgroup g of G takes the
// contiguous range [g*U/G, (g+1)*U/G) (rounded to the ring depth).  All workgroups
// stream the same number of bytes (+-1 unit), whatever the matrix shape.  A tile
// covered by several workgroups gets one partial per workgroup, in slot (g - first
// g of the tile); consumers add the slots in index order, so results do not depend
// on timing.
#include "common.h"
#include "kernels.h"

namespace pd {

constexpr int NT = 256;  // threads per GEMM workgroup: 4 waves, one per SIMD, 512 registers each

// BM: 32-row batch blocks held in accumulators; NS: 32-column subtiles per wave;
// ND: digit planes; R: weight units per wave held in a register ring; AD: operand
// reads run AD - 1 MFMA groups ahead.  grid = (G workgroups, row groups of 32*BM
// rows).  One workgroup per compute unit, one wave per SIMD with all 512 registers:
// 256 of them are AGPRs and hold the int32 tiles for the whole unit loop.
//
// Weights go HBM -> registers with non-temporal buffer loads (each is 1 KiB
// contiguous per wave and already a B operand); the loop body is unrolled R
// times so every ring slot is a fixed register range and the compiler's own
// vmcnt bookkeeping keeps the ring in flight.  Every step issues the same loads
// unconditionally (past the end of the range the last unit is fetched again,
// an L2 hit) so that no control-flow join weakens those waits.
template <int BM, int NS, int ND, int R, int AD, int WAUX>
__global__ __launch_bounds__(NT) void qgemm_kernel(const uint4* __restrict__ wp,
                                                      const unsigned char* __restrict__ qa,
                                                      const float* __restrict__ scale_t,
                                                      float* __restrict__ part, int B, int K, int N,
                                                      SkqPlan pl) {
    constexpr int KC = QCHUNK;                  // k-extent of one unit = one LDS stage
    constexpr int ROWS = BM * 32;
    constexpr int PITCH = ND * KC + 16;         // bytes; +16 spreads rows over LDS banks
    constexpr int PPR = ND * KC / 16;           // 16-byte pieces per row per stage
    constexpr int APT = (ROWS * PPR + NT - 1) / NT;  // pieces per thread per stage (tail repeats the last piece)
    constexpr int KB = KC / 32;                 // 32-k blocks per unit
    constexpr int TSUB = (NT / 64) * NS;        // 32-column subtiles per tile
    constexpr int STAGE = ROWS * PITCH + ROWS * 4;  // digits + one scale per row
    static_assert(3 + APT < KB * ND, "stage write fits behind the loads in one unit");
    static_assert(R == 2 || R == 4, "ring depth (even: the activation register stages alternate with the ring slots)");
    static_assert((KB * ND) % AD == 0, "operand slots rotate evenly across the unit boundary");
    static_assert(3 * STAGE + NS * BM * 16 * NT * 4 <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(16))) unsigned char lds[3][STAGE];
    // fp32 sums of the scale blocks of the current tile that this range has finished:
    // thread-private (each thread owns 16 * NS * BM values), kept in LDS because the
    // unit loop leaves no registers for them
    __shared__ f32x4 accl[NS * BM * 4][NT];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: lets addresses stay scalar
    const int g = lane >> 5, l32 = lane & 31;
    const int n_sub = N >> 5;
    const int C = pl.C, T = pl.T;
    const int c_split = pl.c_split, blk0 = pl.blk0, blk1 = pl.blk1;
    // This workgroup's range comes from the plan's device table (the divisions that
    // define it are 64-bit and would run on the vector ALU, here, in every launch).
    // Scalar loads: everything derived from them -- unit counters, buffer offsets,
    // loop exits -- stays scalar.
    const int* rec = pl.nseg + skq_wg_offset(T) + 4 * (int)blockIdx.x;
    const int u0 = __builtin_amdgcn_readfirstlane(rec[0]);
    const int u1 = __builtin_amdgcn_readfirstlane(rec[1]);
    if (u0 >= u1) return;

    // Every global read is a buffer load: a scalar descriptor and a scalar byte
    // offset that moves with the unit, plus a per-lane offset that never changes --
    // no 64-bit address arithmetic in vector registers, and reads past the end of
    // a range return zero instead of faulting.
    const uint32_t lane16 = lane * 16;
    // One descriptor spans the whole packed matrix; the 32-column stream of subtile i
    // and the unit inside it are a scalar byte offset that advances by one unit per
    // step (a constant) and is recomputed only when the fetch moves to the next tile.
    const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(reinterpret_cast<const unsigned char*>(wp)), 0,
        (int)((uint32_t)n_sub * (uint32_t)K * 32u), 0x00020000);
    uint32_t w_so[NS];
    // (tile, chunk) of the unit being computed; of the next weight unit to fetch
    // (saturates at the last unit of the range)
    int t_cur = __builtin_amdgcn_readfirstlane(rec[3]);
    int c_cur = u0 - t_cur * C;
    int t_w = t_cur, c_w = c_cur, u_w = u0;
    u32x4 wreg[R][NS][KB];

    // weight unit (t_w, c_w) -> ring slot s, one 32-k block at a time
#define PD_W_PTRS()                                                                      \
    _Pragma("unroll") for (int i = 0; i < NS; i++) {                                     \
        int st_ = t_w * TSUB + wave * NS + i;                                            \
        st_ = st_ < n_sub ? st_ : n_sub - 1; /* ragged last tile: result dropped */      \
        w_so[i] = (uint32_t)st_ * (uint32_t)(K * 32) + (uint32_t)c_w * (KC * 32);        \
    }
    // WAUX = 2 (non-temporal): each weight byte is read once per step; 0 when several row
    // groups stream the same weights and the later ones are meant to find them in L2
#define PD_W_LOAD(s, kb)                                                                 \
    _Pragma("unroll") for (int i = 0; i < NS; i++)                                       \
        wreg[s][i][kb] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, lane16 + (kb) * 1024, w_so[i], WAUX);
#define PD_W_REFILL(s, kb) PD_W_LOAD(s, kb)
    // (past the end of the range the last unit is fetched again: an L2 hit; selects
    // rather than branches, except for the rare move to the next tile)
#define PD_W_NEXT()                                                                      \
    {                                                                                    \
        const int nu_ = u_w + 1 < u1 - 1 ? u_w + 1 : u1 - 1; /* s_min: no compare result to widen */ \
        const int adv_ = nu_ - u_w;                                                      \
        u_w = nu_;                                                                       \
        c_w += adv_;                                                                     \
        if (c_w == C) {                                                                  \
            c_w = 0;                                                                     \
            t_w++;                                                                       \
            PD_W_PTRS()                                                                  \
        } else {                                                                         \
            _Pragma("unroll") for (int i = 0; i < NS; i++) w_so[i] += adv_ * (KC * 32);  \
        }                                                                                \
    }
#define PD_FETCH_W(s)                                                                    \
    {                                                                                    \
        _Pragma("unroll") for (int kb = 0; kb < KB; kb++) { PD_W_LOAD(s, kb) }           \
        PD_W_NEXT()                                                                      \
    }
    // The first R weight units are requested before anything else is set up: they come
    // from HBM and are what the first unit waits for longest.
    PD_W_PTRS()
    PD_FETCH_W(0)
    PD_FETCH_W(1)
    if constexpr (R > 2) { PD_FETCH_W(2) }
    if constexpr (R > 3) { PD_FETCH_W(3) }
    bool w_fetched = true;
    __builtin_amdgcn_sched_barrier(0);

    const int row0 = blockIdx.y * ROWS;

    // byte offsets (within one chunk column of the activation matrix) of the pieces
    // this thread moves, and where they go in an LDS stage; rows >= B repeat row B-1
    // (their results are never stored)
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
    // (every thread moves a row scale: threads beyond the rows repeat the first ones)
    int srow = row0 + (tid & (ROWS - 1));
    srow = srow < B ? srow : B - 1;
    const uint32_t srow4 = srow * 4, sslot = ROWS * PITCH + (tid & (ROWS - 1)) * 4;
    const __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char*>(qa), 0, B * K * ND, 0x00020000);
    const __amdgpu_buffer_rsrc_t s_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(scale_t), 0, C * QSCALE_ROWS * 4, 0x00020000);
    // partial sums: slots of pl.rows (whole row groups) x N, so stores need no row test
    const __amdgpu_buffer_rsrc_t p_rs = __builtin_amdgcn_make_buffer_rsrc(
        part, 0, (int)((uint32_t)pl.max_slots * (uint32_t)pl.rows * (uint32_t)N * 4u), 0x00020000);
    uint32_t a_so = 0, s_so = 0;  // byte offsets of chunk c_a in the activation and scale arrays

    // The int32 accumulators live in the accumulation registers (AGPRs) for the whole
    // loop.  They are cleared by an MFMA of zeros rather than by moves: the register
    // allocator keeps a loop-carried tile in AGPRs only if every value that flows into
    // it comes out of an MFMA; a single VALU-written zero makes it hold the tiles in
    // VGPRs and copy all of them to and from AGPRs around every unit.
    const i32x4 zero4 = {0, 0, 0, 0};
    const i32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    i32x16 iacc[ND][NS][BM];
#pragma unroll
    for (int p = 0; p < ND; p++)
#pragma unroll
        for (int i = 0; i < NS; i++)
#pragma unroll
            for (int bm = 0; bm < BM; bm++)
                iacc[p][i][bm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(zero4, zero4, zero16, 0, 0, 0);

#pragma unroll
    for (int j = 0; j < NS * BM * 4; j++) accl[j][tid] = (f32x4){0.f, 0.f, 0.f, 0.f};

    u32x4 areg[2][APT];
    float sreg[2] = {0.f, 0.f};
    i32x4 aop[AD][BM];  // operand reads run AD - 1 groups ahead of their MFMAs

    int c_a = c_cur, u = u0, u_a = u0;  // chunk of the next activation stage; unit being computed
    int slot = __builtin_amdgcn_readfirstlane(rec[2]);  // partial slot of this range in tile t_cur

    // end of the scale block that holds chunk c
    auto block_end = [&](int c) {
        int e;
        if (c < c_split) {
            e = (c / blk0 + 1) * blk0;
            e = e < c_split ? e : c_split;
        } else {
            e = c_split + ((c - c_split) / blk1 + 1) * blk1;
            e = e < C ? e : C;
        }
        return __builtin_amdgcn_readfirstlane(e);
    };
    int seg_end = block_end(c_cur);

#define PD_A_NEXT()                                                                      \
    {                                                                                    \
        const int nu_ = u_a + 1 < u1 - 1 ? u_a + 1 : u1 - 1;                             \
        const int adv_ = nu_ - u_a;                                                      \
        u_a = nu_;                                                                       \
        c_a += adv_;                                                                     \
        a_so += adv_ * (ND * KC);                                                        \
        s_so += adv_ * (QSCALE_ROWS * 4);                                                \
        const bool wrap_ = c_a == C;                                                     \
        c_a = wrap_ ? 0 : c_a;                                                           \
        a_so = wrap_ ? 0 : a_so;                                                         \
        s_so = wrap_ ? 0 : s_so;                                                         \
    }
    // activations (and row scales) of chunk c_a -> register stage `as`
#define PD_A_NOW(as)                                                                     \
    {                                                                                    \
        _Pragma("unroll") for (int it = 0; it < APT; it++)                               \
            areg[as][it] = __builtin_amdgcn_raw_buffer_load_b128(a_rs, aoff[it], a_so, 0); \
        sreg[as] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(       \
            s_rs, srow4, s_so, 0));                                                      \
    }
    // ... of the next unit not yet fetched.  Vector-memory operations retire in
    // order, so a load that is waited on must be older than everything that is meant
    // to stay in flight: these registers are written to LDS one step after the loads
    // are issued, with weight units still outstanding behind them, and the LDS stage
    // is read one step after that.
#define PD_LOAD_A(as)                                                                    \
    {                                                                                    \
        PD_A_NEXT()                                                                      \
        PD_A_NOW(as)                                                                     \
    }
#define PD_STORE_A(buf, as)                                                              \
    {                                                                                    \
        _Pragma("unroll") for (int it = 0; it < APT; it++)                               \
            *reinterpret_cast<u32x4*>(&ldsb[(buf) + aslot[it]]) = areg[as][it];              \
        *reinterpret_cast<float*>(&ldsb[(buf) + sslot]) = sreg[as];                          \
    }
    // One unit of MFMAs.  Group gi = (kb, plane p): BM operand reads from LDS feed
    // NS*BM MFMAs; the reads run two groups ahead of the MFMAs (those of groups 0
    // and 1 were issued by the previous step, ahead of the workgroup barrier), and
    // scheduling barriers keep that order (left alone, the scheduler hoists every
    // read of the unit and runs out of registers).  As soon as the last plane of a
    // 32-k block is issued, the ring registers of that block are refilled from the
    // next unit.  Plane 0 of a row chunk is the most significant digit.
#define PD_A_READ(buf, gi, slot_)                                                        \
    _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                                    \
        aop[slot_][bm] = *reinterpret_cast<const i32x4*>(                                \
            &ldsb[(buf) + (bm * 32 + l32) * PITCH + ((gi) % ND) * KC + ((gi) / ND) * 32 + g * 16]);
#define PD_MFMA1(gi, s, i, bm)                                                           \
    iacc[(gi) % ND][i][bm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                      \
        aop[(gi) % AD][bm], __builtin_bit_cast(i32x4, wreg[s][i][(gi) / ND]),            \
        iacc[(gi) % ND][i][bm], 0, 0, 0);                                                \
    __builtin_amdgcn_sched_barrier(0);
#define PD_MFMA(buf, nbuf, s, wbuf, as_load, as_store)                                   \
    {                                                                                    \
        PD_A_NEXT()                                                                      \
        _Pragma("unroll") for (int gi = 0; gi < KB * ND; gi++) {                         \
            /* One wave per SIMD: whatever is not an MFMA has to be issued while an   */ \
            /* MFMA executes, so the other work of the group is spread between its    */ \
            /* MFMAs and pinned there.                                                 */ \
            PD_MFMA1(gi, s, 0, 0)                                                        \
            /* operand reads run AD - 1 groups ahead, across the end of the unit into  */ \
            /* the stage of the next one (published by the previous barrier)           */ \
            if (gi + AD - 1 < KB * ND) { PD_A_READ(buf, gi + AD - 1, (gi + AD - 1) % AD) } \
            else { PD_A_READ(nbuf, gi + AD - 1 - KB * ND, (gi + AD - 1) % AD) }           \
            __builtin_amdgcn_sched_barrier(0);                                           \
            if (BM > 1) { PD_MFMA1(gi, s, 0, BM - 1) }                                   \
            /* in the first three groups the loads of the activations three units     */ \
            /* ahead (ahead of this step's weight loads in the queue, see PD_A_NOW),  */ \
            /* then one piece per group of the stage write of the unit two ahead      */ \
            if (gi < 3) {                                                                \
                _Pragma("unroll") for (int it = 0; it < APT; it++)                       \
                    if (it * 3 / APT == gi)                                              \
                        areg[as_load][it] = __builtin_amdgcn_raw_buffer_load_b128(       \
                            a_rs, aoff[it], a_so, 0);                                    \
                if (gi == 2)                                                             \
                    sreg[as_load] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32( \
                        s_rs, srow4, s_so, 0));                                          \
            } else if (gi - 3 < APT) {                                                   \
                *reinterpret_cast<u32x4*>(&ldsb[(wbuf) + aslot[gi - 3]]) = areg[as_store][gi - 3]; \
            } else if (gi - 3 == APT) {                                                  \
                *reinterpret_cast<float*>(&ldsb[(wbuf) + sslot]) = sreg[as_store];           \
            }                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                           \
            if (NS > 1) {                                                                \
                PD_MFMA1(gi, s, NS - 1, 0)                                               \
                if (BM > 1) { PD_MFMA1(gi, s, NS - 1, BM - 1) }                          \
            }                                                                            \
            if (gi % ND == ND - 1) { PD_W_REFILL(s, gi / ND) }                           \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
        PD_W_NEXT()                                                                      \
    }
    // A scale block ends: facc += scale * sum_p 256^(ND-1-p) * float(iacc[p]).
    // int32 bound per plane and scale block: 128 * 127 * 128 * chunks < 2^31 for blocks
    // of up to 1024 chunks.  D layout of the 32x32 MFMA: register r of lane (l32, g)
    // is row 8*(r/4) + 4*g + r%4, column l32.
    // (`opq` is a zero the compiler cannot see through: what the fold and the stores
    // need is computed from it, here, instead of being hoisted above the unit loop and
    // kept in registers across it.)
#define PD_FOLD(buf)                                                                     \
    {                                                                                    \
        int opq;                                                                         \
        asm volatile("s_mov_b32 %0, 0" : "=s"(opq));                                     \
        const int g_ = g + opq, tid_ = tid + opq;                                        \
        /* the running sums are read one group of four ahead of their use */             \
        f32x4 nx_ = accl[0][tid_];                                                       \
        _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                              \
            f32x4 sc[4];                                                                 \
            _Pragma("unroll") for (int q = 0; q < 4; q++)                                \
                sc[q] = *reinterpret_cast<const f32x4*>(                                 \
                    &ldsb[(buf) + ROWS * PITCH + (bm * 32 + 8 * q + 4 * g_) * 4]);       \
            _Pragma("unroll") for (int i = 0; i < NS; i++) {                             \
                /* The accumulators leave their AGPRs one 32x32 tile at a time, through */ \
                /* an MFMA of zeros that adds them into VGPRs.  (Read by vector ALU     */ \
                /* code directly, the register allocator copies all of them to VGPRs at */ \
                /* the loop exit and spills what the unit loop keeps there.)            */ \
                i32x16 c_[ND];                                                           \
                _Pragma("unroll") for (int p = 0; p < ND; p++)                           \
                    c_[p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(zero4, zero4, iacc[p][i][bm], 0, 0, 0); \
                _Pragma("unroll") for (int q = 0; q < 4; q++) {                          \
                    const int j_ = (bm * NS + i) * 4 + q;                                \
                    f32x4 t_ = nx_;                                                      \
                    if (j_ + 1 < NS * BM * 4) nx_ = accl[j_ + 1][tid_];                  \
                    _Pragma("unroll") for (int k = 0; k < 4; k++) {                      \
                        float v_ = (float)c_[0][4 * q + k];                              \
                        _Pragma("unroll") for (int p = 1; p < ND; p++)                   \
                            v_ = v_ * 256.0f + (float)c_[p][4 * q + k];                  \
                        t_[k] += sc[q][k] * v_;                                          \
                    }                                                                    \
                    accl[j_][tid_] = t_;                                                 \
                }                                                                        \
                __builtin_amdgcn_sched_barrier(0); /* one tile in flight */              \
            }                                                                            \
        }                                                                                \
    }
    // The range leaves the tile (or ends): part[slot] = tile sums, tile sums = 0.
#define PD_STORE_TILE()                                                                  \
    {                                                                                    \
        int opq;                                                                         \
        asm volatile("s_mov_b32 %0, 0" : "=s"(opq));                                     \
        const int g_ = g + opq, l32_ = l32 + opq, tid_ = tid + opq;                      \
        const uint32_t rowb_ = (uint32_t)(N + opq) * 4u; /* bytes of one partial row */  \
        const uint32_t voff_ = (uint32_t)(4 * g_) * rowb_ + l32_ * 4;                    \
        _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                              \
            _Pragma("unroll") for (int i = 0; i < NS; i++) {                             \
                const int st_ = t_cur * TSUB + wave * NS + i;                            \
                if (st_ < n_sub) {                                                       \
                    uint32_t so_ = (uint32_t)(slot * pl.rows + row0 + bm * 32) * rowb_ + st_ * 128; \
                    _Pragma("unroll") for (int q = 0; q < 4; q++) {                      \
                        const f32x4 t_ = accl[(bm * NS + i) * 4 + q][tid_];              \
                        _Pragma("unroll") for (int k = 0; k < 4; k++) {                  \
                            const float f_ = t_[k];                                      \
                            __builtin_amdgcn_raw_buffer_store_b32(                       \
                                __builtin_bit_cast(uint32_t, f_), p_rs, voff_, so_, PD_WRITE_THROUGH);  \
                            so_ += k == 3 ? 5 * rowb_ : rowb_; /* rows 8*q + 4*g + k */  \
                        }                                                                \
                    }                                                                    \
                }                                                                        \
                _Pragma("unroll") for (int q = 0; q < 4; q++)                            \
                    accl[(bm * NS + i) * 4 + q][tid_] = (f32x4){0.f, 0.f, 0.f, 0.f};     \
            }                                                                            \
        }                                                                                \
    }
    // One unit.  LDS holds three activation stages: stage k%3 is read by step k,
    // stage (k+1)%3 was published by the previous barrier, stage (k+2)%3 (last read
    // in step k-1) is written during step k.  The only thing a step waits for at its
    // barrier is the other waves: its own LDS writes have a whole step to land, and
    // the first operand reads of the next step are already in flight across it.
#define PD_STEP(s)                                                                       \
    {                                                                                    \
        const int nxt_ = o_nxt, wr_ = o_wr;                                              \
        PD_MFMA(cur, nxt_, (s) % R, wr_, (s) % 2, ((s) + 1) % 2)                         \
        /* LDS operations of a wave complete in order: all but the (AD-1)*BM reads of   */ \
        /* the next unit's first groups, i.e. this step's stage writes, have landed     */ \
        /* before the barrier                                                           */ \
        asm volatile("s_waitcnt lgkmcnt(%0)\n\ts_barrier" ::"n"((AD - 1) * BM) : "memory"); \
        last = cur;                                                                      \
        o_wr = cur;                                                                      \
        cur = nxt_;                                                                      \
        o_nxt = wr_;                                                                     \
    }
    // A segment = the run of units of one scale block inside this range: clear the
    // int32 accumulators, run its units, fold the int32 sums into the fp32 sums of the
    // tile.  (A fold inside the unit loop would put VALU reads and writes of the
    // accumulators on the loop's back edge and the register allocator would then keep
    // all of them in VGPRs.)
    // byte offsets of the LDS stages: being read, published by the last barrier,
    // being written; they rotate every step
    unsigned char* const ldsb = &lds[0][0];
    int cur = 0, o_nxt = STAGE, o_wr = 2 * STAGE, last = 0;
    // The end of a segment: scales of the segment's scale block from the stage of its
    // last unit; the barrier keeps the next unit's stage write (or the next fill) from
    // overwriting a stage that a slower wave is still reading.
#define PD_END_SEGMENT()                                                                 \
    u += n_units;                                                                        \
    c_cur += n_units;                                                                    \
    PD_FOLD(last)                                                                        \
    if (c_cur == C || u == u1) { PD_STORE_TILE() }                                       \
    lds_barrier();                                                                       \
    if (u == u1) break;                                                                  \
    if (c_cur == C) { c_cur = 0; t_cur++; slot = 0; }                                    \
    seg_end = block_end(c_cur);
    // Outer loop: fill the pipeline.  Inner loop: the segments that run on it -- it
    // keeps running across a segment end as long as the segment was a whole number of
    // turns of the ring, which the plan arranges for the decode shapes by starting
    // workgroup ranges at multiples of the ring; a segment with a remainder ends in
    // its own copy of the segment end and falls out to the fill.  (One copy behind
    // an `if` would let the wait counts of the remainder steps, which have just
    // refilled ring slot 0, reach the head of the unit loop, where slot 0 is read:
    // every turn would then wait for nearly all of its loads.)
    bool done = false;
    while (!done) {
        done = true;

            // fill: R weight units in flight (first: they come from HBM and take longest),
            // activations of the first two units straight into stages 0 and 1, those of the
            // third into register stage 1 (step 0 writes them to stage 2), first operand
            // reads of step 0
            c_a = c_cur;
            u_a = u;
            a_so = (uint32_t)c_cur * (ND * KC);
            s_so = (uint32_t)c_cur * (QSCALE_ROWS * 4);
            if (!w_fetched) {  // (the first fill finds its weights already on their way)
                t_w = t_cur; c_w = c_cur; u_w = u;
                PD_W_PTRS()
                PD_FETCH_W(0)
                PD_FETCH_W(1)
                if constexpr (R > 2) { PD_FETCH_W(2) }
                if constexpr (R > 3) { PD_FETCH_W(3) }
            }
            w_fetched = false;
            PD_A_NOW(0)
            PD_LOAD_A(1)
            PD_STORE_A(0, 0)
            PD_STORE_A(STAGE, 1)
            PD_LOAD_A(1)
            // Everything fetched so far is waited for here, once, so that the compiler's
            // wait counts at the head of the unit loop come from the loop's own back edge
            // alone (merged with this path they drain the ring on every turn).
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
            lds_barrier();
            cur = 0; o_nxt = STAGE; o_wr = 2 * STAGE;
#pragma unroll
            for (int g_ = 0; g_ < AD - 1; g_++) { PD_A_READ(0, g_, g_) }
        
        for (;;) {
            const int rest = u1 - u;
            const int n_units = seg_end - c_cur < rest ? seg_end - c_cur : rest;
#pragma unroll
            for (int p = 0; p < ND; p++)
#pragma unroll
                for (int i = 0; i < NS; i++)
#pragma unroll
                    for (int bm = 0; bm < BM; bm++)
                        iacc[p][i][bm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(zero4, zero4, zero16, 0, 0, 0);
            // whole turns of the ring in a loop with a single exit (exits from the middle
            // of the body make the compiler funnel scalar state through vector registers
            // that have loads in flight, and wait for those), then the last R - 1 units at most
            for (int turns = n_units / R; turns > 0; --turns) {
                PD_STEP(0)
                PD_STEP(1)
                if constexpr (R > 2) {
                    PD_STEP(2)
                    PD_STEP(3)
                }
            }
            const int rem = n_units % R;
            if (rem > 0) {
                PD_STEP(0)
                if constexpr (R > 2) {
                    if (rem > 1) {
                        PD_STEP(1)
                        if (rem > 2) { PD_STEP(2) }
                    }
                }
                // nothing stays in flight from here (the fill that follows waits for all
                // of it anyway): the compiler then has no loads of the remainder steps to
                // account for at the head of the unit loop, where it would otherwise wait
                // for ring slot 0 -- just refilled here -- on every turn
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
                PD_END_SEGMENT()
                done = false;  // refill and go on
                break;
            }
            PD_END_SEGMENT()
        }
    }
#undef PD_END_SEGMENT
#undef PD_FETCH_W
#undef PD_A_NEXT
#undef PD_A_NOW
#undef PD_W_PTRS
#undef PD_W_LOAD
#undef PD_W_REFILL
#undef PD_W_NEXT
#undef PD_A_READ
#undef PD_LOAD_A
#undef PD_STORE_A
#undef PD_MFMA
#undef PD_MFMA1
#undef PD_FOLD
#undef PD_STORE_TILE
#undef PD_STEP
}

// segments (= partial slots) per tile, for the consumers of the partial sums
__global__ __launch_bounds__(256) void skq_table_kernel(SkqPlan pl, int* __restrict__ table) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < pl.T) table[t] = skq_segments(t, pl);
    if (t < pl.G) {
        const long long U = (long long)pl.T * pl.C;
        const long long u0 = skq_begin(t, U, pl.G, pl.align), u1 = skq_begin(t + 1, U, pl.G, pl.align);
        const int t0 = (int)(u0 / pl.C);
        int* rec = table + skq_wg_offset(pl.T) + 4 * t;
        rec[0] = (int)u0;
        rec[1] = (int)u1;
        rec[2] = u0 < u1 ? skq_segments_upto(t0, (int)(u0 - (long long)t0 * pl.C), pl) : 0;
        rec[3] = t0;
    }
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
    int n = packed_col_map(st * 32 + (lane & 31), mode, n_qkv, F);
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
    if (pn < N) dst[pn] = from_bf16(src[packed_col_map(pn, mode, n_qkv, F)]);
}

// out[b][n] = scale[n] * sum over the slots of n's tile (fixed order); scale NULL = ones
__global__ __launch_bounds__(256) void qgemm_reduce_kernel(const float* __restrict__ part,
                                                           const float* __restrict__ scale,
                                                           float* __restrict__ out, int B, int N,
                                                           SkqPlan pl) {
    int n = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (n >= N) return;
    const int ns = pl.nseg[n / pl.tile_cols];
    float acc = 0.f;
    for (int s = 0; s < ns; s++) acc += part[((size_t)s * pl.rows + b) * N + n];
    out[(size_t)b * N + n] = scale ? scale[n] * acc : acc;
}

// ---- host launchers -----------------------------------------------------------

// weight units per wave kept in flight (the R of the kernel instance launch_qgemm picks)
static int qgemm_ring(int bm) { return bm == 1 ? 4 : 2; }

void qgemm_config(int B, int* bm, int* ns, int* tile_cols) {
    int blocks = (B + 31) / 32;
    *bm = blocks <= 1 ? 1 : 2;  // more than 64 rows: several row groups
    *ns = 2;
    *tile_cols = (NT / 64) * 32 * *ns;
}

// Plan of a [K][N] projection for batch B: `workgroups` share the matrix (capped by
// the number of units); returns the largest number of segments in any tile.
SkqPlan qgemm_plan(int B, int K, int N, int workgroups, int c_split, int blk0, int blk1,
                   int* max_slots, int tile_cols) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    if (tile_cols > 0) tc = tile_cols;  // (the bf16-weight kernel's tiles are wider)
    SkqPlan pl;
    pl.tile_cols = tc;
    pl.C = K / 128;
    pl.T = (N + tc - 1) / tc;
    const long long U = (long long)pl.T * pl.C;
    pl.G = (int)(workgroups < U ? (workgroups < 1 ? 1 : workgroups) : U);
    // ranges that start at multiples of the weight ring (qgemm_ring() units) keep the
    // pipeline of the unit loop running across segment ends; only worth it for ranges of
    // many units.  (The ring is also the granularity of the split: ranges differ by at
    // most one ring, which is what the slowest workgroup streams more than the others.)
    const int ring = qgemm_ring(bm);
    pl.align = (U / pl.G >= 16 && pl.C % ring == 0 && c_split % ring == 0 &&
                (c_split == 0 || blk0 % ring == 0) && blk1 % ring == 0) ? ring : 1;
    pl.c_split = c_split;
    pl.blk0 = blk0;
    pl.blk1 = blk1;
    pl.nseg = nullptr;
    pl.rows = (B + 32 * bm - 1) / (32 * bm) * (32 * bm);
    int mx = 1;
    for (int t = 0; t < pl.T; t++) {
        const int n = skq_segments(t, pl);
        if (n > mx) mx = n;
    }
    pl.max_slots = mx;
    if (max_slots) *max_slots = mx;
    return pl;
}

// Automatic workgroup count: at most g_max, at least 7/8 of it, in steps of 8 (one per XCD),
// whichever leaves the longest range shortest relative to an even split.  The kernel is
// bandwidth-bound, so its time follows the longest range times the number of ranges that
// share the bandwidth; a few idle compute units cost less than one ring of extra units on
// the slowest workgroup (62B-shaped input projection: 232 ranges of 80 units beat 256 of
// 72 or 74).
int qgemm_auto_workgroups(int B, int K, int N, int g_max, int c_split, int blk0, int blk1, int tile_cols) {
    if (g_max < 16) return g_max < 1 ? 1 : g_max;
    int best_g = g_max;
    long long best_cost = -1;
    for (int g = g_max; g >= g_max - g_max / 8; g -= 8) {
        const SkqPlan pl = qgemm_plan(B, K, N, g, c_split, blk0, blk1, nullptr, tile_cols);
        const long long U = (long long)pl.T * pl.C;
        long long longest = 0;
        for (int i = 0; i < pl.G; i++) {
            const long long n = skq_begin(i + 1, U, pl.G, pl.align) - skq_begin(i, U, pl.G, pl.align);
            if (n > longest) longest = n;
        }
        const long long cost = longest * pl.G;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_g = g; }
    }
    return best_g;
}

hipError_t launch_skq_table(SkqPlan pl, int* nseg, hipStream_t stream) {
    const int n = pl.T > pl.G ? pl.T : pl.G;
    skq_table_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(pl, nseg);
    return hipGetLastError();
}

hipError_t launch_qgemm(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                        int K, int N, SkqPlan pl, int nd, hipStream_t stream) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    dim3 grid(pl.G, (B + 32 * bm - 1) / (32 * bm)), block(NT);
    const uint4* w4 = reinterpret_cast<const uint4*>(wp);
    const unsigned char* q = reinterpret_cast<const unsigned char*>(qa);
#define PD_LAUNCH(BMv, NSv, RING, ADv, WAUXv)                                                    \
    do {                                                                                    \
        if (nd == 3)                                                                        \
            qgemm_kernel<BMv, NSv, 3, RING, ADv, WAUXv><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, pl); \
        else                                                                                \
            qgemm_kernel<BMv, NSv, 2, RING, ADv, WAUXv><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, pl); \
    } while (0)
    if (nd != 2 && nd != 3) return hipErrorInvalidValue;
    if (pl.blk0 < 1 || pl.blk0 > 1024 || pl.blk1 < 1 || pl.blk1 > 1024 || pl.c_split < 0 || pl.c_split > K / 128)
        return hipErrorInvalidValue;
    // buffer descriptors address 32 bits
    if ((long long)B * K * nd >= (1ll << 31) || (long long)K * N >= (1ll << 32)) return hipErrorInvalidValue;
    if ((long long)pl.T * pl.C >= (1ll << 31)) return hipErrorInvalidValue;
    if ((long long)pl.max_slots * pl.rows * N * 4 >= (1ll << 32)) return hipErrorInvalidValue;
    if (bm == 1) PD_LAUNCH(1, 2, 4, 4, 2);  // rings as in qgemm_ring()
    else if (grid.y > 1) PD_LAUNCH(2, 2, 2, 4, 0);
    else PD_LAUNCH(2, 2, 2, 4, 2);
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

hipError_t launch_qgemm_reduce(const float* part, const float* scale, float* out, int B, int N,
                               SkqPlan pl, hipStream_t stream) {
    qgemm_reduce_kernel<<<dim3((N + 255) / 256, B), dim3(256), 0, stream>>>(part, scale, out, B, N, pl);
    return hipGetLastError();
}

}  // namespace pd
