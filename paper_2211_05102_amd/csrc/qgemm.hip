// int8-weight skinny GEMM for gfx950 (paper Section 3.6: weights stored int8
// with one scale per output channel; Section 3.4: the fused input and output
// projections of the parallel block are the two instances of this product).
//
//   part[s][b][n] = sum_{k in split s} a[b][k] * q8[k][n]          (fp32, unscaled)
//
// The per-channel weight scale s[n] is applied once per output by the consumer
// of the partial sums, which is exact because it does not depend on k.
//
// Activations arrive in block fixed point (common.h): ND int8 digit planes and
// a power-of-two scale per (row, 128-k chunk).  Every digit goes through
// v_mfma_i32_32x32x32_i8 against the raw int8 weights -- no weight conversion,
// exact int32 sums -- and once per chunk the int32 tiles are folded into the
// fp32 accumulator:  acc += scale[b][chunk] * (65536 * float(top) + float((mid << 8) + low)).
// ND = 3 gives 23-bit activations (the bf16 rounding of LayerNorm and SwiGLU
// outputs would otherwise dominate the error of a deep stack) for 1.5x the MFMA
// time of a single bf16 pass; ND = 2 gives 15 bits for 1.0x.
//
// Data movement (HBM-bound: 1 byte per weight, 2*B flops per byte):
//   - weights are pre-tiled by pd_pack_* so that a wavefront's 16-byte-per-lane
//     load is 1 KiB contiguous and is already an MFMA B operand:
//     packed[(st*(K/32) + kb)*64 + lane] holds W[kb*32 + (lane/32)*16 + 0..15][st*32 + lane%32];
//   - activations (and their scales) are shared by the 4 waves through LDS.
// A = activations (M = batch row), B = weights (N = output channel).
#include "common.h"
#include "kernels.h"

namespace pd {

// BM: 32-row batch blocks held in accumulators; NS: 32-column subtiles per wave.
// Workgroup = 4 waves = 128*NS columns x one K-split x one group of 32*BM rows.
// grid = (n_tiles, S, row groups).
template <int BM, int NS, int ND>
__global__ __launch_bounds__(256) void qgemm_kernel(const uint4* __restrict__ wp,
                                                    const unsigned char* __restrict__ qa,
                                                    const float* __restrict__ scale_t,
                                                    float* __restrict__ part, int B, int K, int N,
                                                    int S) {
    constexpr int KC = QCHUNK;                  // k-extent of one LDS stage = one scale block
    constexpr int ROWS = BM * 32;
    constexpr int PITCH = ND * KC + 16;         // bytes; +16 spreads rows over LDS banks
    constexpr int PPR = ND * KC / 16;           // 16-byte pieces per row per stage
    constexpr int APT = ROWS * PPR / 256;       // pieces per thread per stage
    static_assert(ROWS * PPR % 256 == 0, "stage must split evenly over 256 threads");
    constexpr int KB = KC / 32;                 // 32-k blocks per stage
    constexpr int STAGE = ROWS * PITCH + ROWS * 4;  // digits + one scale per row
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int n_sub = N >> 5;                   // 32-column subtiles in the matrix
    const int kblocks = K >> 5;
    const int chunks = K >> 7;
    const int s = blockIdx.y;
    const int row0 = blockIdx.z * ROWS;         // first batch row of this group
    const int c_begin = (int)(((long long)s * chunks) / S);
    const int c_end = (int)(((long long)(s + 1) * chunks) / S);
    const size_t row_pitch = (size_t)K * ND;    // bytes per activation row

    int st[NS];
    bool st_ok[NS];
    const uint4* wptr[NS];
#pragma unroll
    for (int i = 0; i < NS; i++) {
        st[i] = (blockIdx.x * 4 + wave) * NS + i;
        st_ok[i] = st[i] < n_sub;
        int stc = st_ok[i] ? st[i] : n_sub - 1;  // clamp: loads stay in bounds, result dropped
        wptr[i] = wp + ((size_t)stc * kblocks + (size_t)c_begin * KB) * 64 + lane;
    }

    f32x16 acc[NS][BM];
    i32x16 iacc[NS][BM];
#pragma unroll
    for (int i = 0; i < NS; i++)
#pragma unroll
        for (int bm = 0; bm < BM; bm++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                acc[i][bm][r] = 0.f;
                iacc[i][bm][r] = 0;
            }

    uint4 wcur[NS][KB], wnext[NS][KB], areg[APT];
    float sreg = 0.f;

#define PD_LOAD_W(dst, c)                                                                \
    _Pragma("unroll") for (int i = 0; i < NS; i++)                                       \
        _Pragma("unroll") for (int kb = 0; kb < KB; kb++)                                \
            dst[i][kb] = ld_stream(wptr[i] + ((size_t)((c) - c_begin) * KB + kb) * 64)
#define PD_LOAD_A(c)                                                                     \
    _Pragma("unroll") for (int it = 0; it < APT; it++) {                                 \
        const int p_ = it * 256 + tid;                                                   \
        int row_ = row0 + p_ / PPR;                                                      \
        row_ = row_ < B ? row_ : B - 1; /* rows >= B: duplicate, never stored */         \
        areg[it] = *reinterpret_cast<const uint4*>(qa + (size_t)row_ * row_pitch +       \
                                                   (size_t)(c) * (ND * KC) + (p_ % PPR) * 16); \
    }                                                                                    \
    if (tid < ROWS) {                                                                    \
        int row_ = row0 + tid;                                                           \
        row_ = row_ < B ? row_ : B - 1;                                                  \
        sreg = scale_t[(size_t)(c) * QSCALE_ROWS + row_];                                \
    }
#define PD_STORE_A(buf)                                                                  \
    _Pragma("unroll") for (int it = 0; it < APT; it++) {                                 \
        const int p_ = it * 256 + tid;                                                   \
        *reinterpret_cast<uint4*>(&lds[buf][(p_ / PPR) * PITCH + (p_ % PPR) * 16]) = areg[it]; \
    }                                                                                    \
    if (tid < ROWS) *reinterpret_cast<float*>(&lds[buf][ROWS * PITCH + tid * 4]) = sreg;
    // plane 0 of a row chunk is the most significant digit
#define PD_MFMA_PLANE(buf, plane)                                                        \
    _Pragma("unroll") for (int kb = 0; kb < KB; kb++) {                                  \
        i32x4 aop[BM];                                                                   \
        _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                                \
            aop[bm] = *reinterpret_cast<const i32x4*>(                                   \
                &lds[buf][(bm * 32 + l32) * PITCH + (plane) * KC + kb * 32 + g * 16]);   \
        _Pragma("unroll") for (int i = 0; i < NS; i++) {                                 \
            const i32x4 bop = __builtin_bit_cast(i32x4, wcur[i][kb]);                    \
            _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                            \
                iacc[i][bm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aop[bm], bop,        \
                                                                    iacc[i][bm], 0, 0, 0); \
        }                                                                                \
    }
    // acc += (scale * mult) * float(iacc); iacc = 0.  Rows 8*q + 4*g + 0..3 of a
    // block: one float4 of scales per q.
#define PD_FOLD(buf, mult)                                                               \
    _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                                  \
        f32x4 sc[4];                                                                     \
        _Pragma("unroll") for (int q = 0; q < 4; q++)                                    \
            sc[q] = *reinterpret_cast<const f32x4*>(                                     \
                        &lds[buf][ROWS * PITCH + (bm * 32 + 8 * q + 4 * g) * 4]) * (mult); \
        _Pragma("unroll") for (int i = 0; i < NS; i++)                                   \
            _Pragma("unroll") for (int r = 0; r < 16; r++) {                             \
                acc[i][bm][r] += sc[r >> 2][r & 3] * (float)iacc[i][bm][r];              \
                iacc[i][bm][r] = 0;                                                      \
            }                                                                            \
    }
#define PD_SHIFT8()                                                                      \
    _Pragma("unroll") for (int i = 0; i < NS; i++)                                       \
        _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                                \
            _Pragma("unroll") for (int r = 0; r < 16; r++) iacc[i][bm][r] <<= 8;
    // int32 bounds per 128-k chunk: one plane 127*128*128 < 2^21; two planes
    // combined 32640*127*128 < 2^29.  Three planes would overflow, so the top
    // digit of ND = 3 is folded on its own.
#define PD_COMPUTE(buf)                                                                  \
    if (ND == 3) {                                                                       \
        PD_MFMA_PLANE(buf, 0)                                                            \
        PD_FOLD(buf, 65536.0f)                                                           \
    }                                                                                    \
    PD_MFMA_PLANE(buf, ND - 2)                                                           \
    PD_SHIFT8()                                                                          \
    PD_MFMA_PLANE(buf, ND - 1)                                                           \
    PD_FOLD(buf, 1.0f)

    if (c_begin < c_end) {
        PD_LOAD_W(wcur, c_begin);
        PD_LOAD_A(c_begin);
        PD_STORE_A(0);
        __syncthreads();
        int cur = 0;
        // steady state: fetch chunk c + 1 while the MFMAs consume chunk c
        for (int c = c_begin; c + 1 < c_end; c++) {
            PD_LOAD_W(wnext, c + 1);
            PD_LOAD_A(c + 1);
            PD_COMPUTE(cur);
            PD_STORE_A(cur ^ 1);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NS; i++)
#pragma unroll
                for (int kb = 0; kb < KB; kb++) wcur[i][kb] = wnext[i][kb];
            cur ^= 1;
        }
        PD_COMPUTE(cur);  // last chunk, nothing left to fetch
    }
#undef PD_LOAD_W
#undef PD_LOAD_A
#undef PD_STORE_A
#undef PD_MFMA_PLANE
#undef PD_FOLD
#undef PD_SHIFT8
#undef PD_COMPUTE

    // D layout of the 32x32 MFMA: register r of lane (l32, g) is row 8*(r/4) + 4*g + r%4, column l32
#pragma unroll
    for (int i = 0; i < NS; i++) {
        if (!st_ok[i]) continue;
        const int n = st[i] * 32 + l32;
#pragma unroll
        for (int bm = 0; bm < BM; bm++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                int b = row0 + bm * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (b < B) part[((size_t)s * B + b) * N + n] = acc[i][bm][r];
            }
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

// out[b][n] = scale[n] * sum_s part[s][b][n]   (fixed summation order)
__global__ __launch_bounds__(256) void qgemm_reduce_kernel(const float* __restrict__ part,
                                                           const float* __restrict__ scale,
                                                           float* __restrict__ out, int B, int N,
                                                           int S) {
    int n = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (n >= N) return;
    float acc = 0.f;
    for (int s = 0; s < S; s++) acc += part[((size_t)s * B + b) * N + n];
    out[(size_t)b * N + n] = scale[n] * acc;
}

// ---- host launchers -----------------------------------------------------------

void qgemm_config(int B, int* bm, int* ns, int* tile_cols) {
    int blocks = (B + 31) / 32;
    int BMv = blocks <= 1 ? 1 : blocks <= 2 ? 2 : 4;  // more than 128 rows: several row groups
    *bm = BMv;
    *ns = BMv <= 2 ? 2 : 1;
    *tile_cols = 128 * *ns;
}

int qgemm_auto_splits(int B, int K, int N) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    int n_tiles = (N + tc - 1) / tc * ((B + 32 * bm - 1) / (32 * bm));
    int s = (400 + n_tiles / 2) / n_tiles;
    int cap = K / 128 < PD_MAX_SPLITS ? K / 128 : PD_MAX_SPLITS;
    if (s < 1) s = 1;
    if (s > cap) s = cap;
    return s;
}

hipError_t launch_qgemm(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                        int K, int N, int S, int nd, hipStream_t stream) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    dim3 grid((N + tc - 1) / tc, S, (B + 32 * bm - 1) / (32 * bm)), block(256);
    const uint4* w4 = reinterpret_cast<const uint4*>(wp);
    const unsigned char* q = reinterpret_cast<const unsigned char*>(qa);
#define PD_LAUNCH(BMv, NSv)                                                                 \
    do {                                                                                    \
        if (nd == 3)                                                                        \
            qgemm_kernel<BMv, NSv, 3><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, S); \
        else                                                                                \
            qgemm_kernel<BMv, NSv, 2><<<grid, block, 0, stream>>>(w4, q, scale_t, part, B, K, N, S); \
    } while (0)
    if (nd != 2 && nd != 3) return hipErrorInvalidValue;
    if (bm == 1) PD_LAUNCH(1, 2);
    else if (bm == 2) PD_LAUNCH(2, 2);
    else PD_LAUNCH(4, 1);
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
                               int S, hipStream_t stream) {
    qgemm_reduce_kernel<<<dim3((N + 255) / 256, B), dim3(256), 0, stream>>>(part, scale, out, B, N, S);
    return hipGetLastError();
}

}  // namespace pd
