// int8-weight x bf16-activation skinny GEMM for gfx950 (paper Section 3.6:
// weights stored int8 with one scale per output channel, matmul arithmetic
// stays bf16 with fp32 accumulation; Section 3.4: the fused input and output
// projections of the parallel block are the two instances of this product).
//
//   part[s][b][n] = sum_{k in split s} a[b][k] * q8[k][n]          (fp32, unscaled)
//
// The scale s[n] is applied once per output by the consumer of the partial
// sums, which is exact because the scale is per output channel.
//
// Data movement (HBM-bound: 1 byte per weight, 2*B flops per byte):
//   - weights are pre-tiled by pd_pack_* so that a wavefront's 16-byte-per-lane
//     load is 1 KiB contiguous and lands directly in MFMA B-operand order:
//     packed[(st*(K/32) + kb)*64 + lane] holds W[kb*32 + (lane/32)*16 + 0..15][st*32 + lane%32];
//   - int8 -> bf16 in registers (every int8 is exact in bf16), 1.5 VALU ops/weight;
//   - activations are shared by the 4 waves of a workgroup through LDS.
// MFMA: v_mfma_f32_32x32x16_bf16, A = activations (M = batch), B = weights
// (N = output channel).  The contraction index inside one MFMA is permuted the
// same way on both operands (k = kb*32 + g*16 + e2*8 + e), which leaves the sum
// unchanged.
#include "common.h"
#include "kernels.h"

namespace pd {

// 8 int8 (two dwords) -> 8 bf16, element order = byte order
__device__ __forceinline__ bf16x8 cvt_i8x8(uint32_t lo, uint32_t hi) {
    float f0 = (float)(int8_t)(lo & 0xff);
    float f1 = (float)(int8_t)((lo >> 8) & 0xff);
    float f2 = (float)(int8_t)((lo >> 16) & 0xff);
    float f3 = (float)(int8_t)(lo >> 24);
    float f4 = (float)(int8_t)(hi & 0xff);
    float f5 = (float)(int8_t)((hi >> 8) & 0xff);
    float f6 = (float)(int8_t)((hi >> 16) & 0xff);
    float f7 = (float)(int8_t)(hi >> 24);
    uint4 r = {pack_bf16x2(f0, f1), pack_bf16x2(f2, f3), pack_bf16x2(f4, f5), pack_bf16x2(f6, f7)};
    return __builtin_bit_cast(bf16x8, r);
}

// BM: number of 32-row batch blocks held in accumulators; NS: 32-column
// subtiles per wave; KC: k-extent of one LDS stage (multiple of 32).
// Workgroup = 4 waves = 128*NS columns x one K-split.  grid = (n_tiles, S).
template <int BM, int NS, int KC>
__global__ __launch_bounds__(256) void qgemm_kernel(const uint4* __restrict__ wp,
                                                    const uint16_t* __restrict__ a,
                                                    float* __restrict__ part, int B, int K, int N,
                                                    int lda, int S) {
    constexpr int ROWS = BM * 32;
    constexpr int PITCH = KC * 2 + 16;          // bytes; +16 spreads rows over LDS banks
    constexpr int PIECES_PER_ROW = KC / 8;      // 16-byte pieces
    constexpr int APT = ROWS * PIECES_PER_ROW / 256;  // pieces per thread per stage
    constexpr int KB = KC / 32;                 // 32-k blocks per stage
    static_assert(APT >= 1, "tile too small for 256 threads");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][ROWS * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, l32 = lane & 31;
    const int n_sub = N >> 5;                   // 32-column subtiles in the matrix
    const int kblocks = K >> 5;
    // K-split in units of 128
    const int chunks128 = K >> 7;
    const int s = blockIdx.y;
    const int k_begin = (int)(((long long)s * chunks128) / S) << 7;
    const int k_end = (int)(((long long)(s + 1) * chunks128) / S) << 7;

    int st[NS];
    bool st_ok[NS];
    const uint4* wptr[NS];
#pragma unroll
    for (int i = 0; i < NS; i++) {
        st[i] = (blockIdx.x * 4 + wave) * NS + i;
        st_ok[i] = st[i] < n_sub;
        int stc = st_ok[i] ? st[i] : n_sub - 1;  // clamp: loads stay in bounds, result dropped
        wptr[i] = wp + ((size_t)stc * kblocks + (k_begin >> 5)) * 64 + lane;
    }

    f32x16 acc[NS][BM];
#pragma unroll
    for (int i = 0; i < NS; i++)
#pragma unroll
        for (int bm = 0; bm < BM; bm++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][bm][r] = 0.f;

    uint4 wcur[NS][KB], wnext[NS][KB], areg[APT];

#define PD_LOAD_W(dst, k0)                                                               \
    _Pragma("unroll") for (int i = 0; i < NS; i++)                                       \
        _Pragma("unroll") for (int kb = 0; kb < KB; kb++)                                \
            dst[i][kb] = ld_stream(wptr[i] + ((size_t)(((k0) - k_begin) >> 5) + kb) * 64)
#define PD_LOAD_A(k0)                                                                    \
    _Pragma("unroll") for (int it = 0; it < APT; it++) {                                 \
        const int p_ = it * 256 + tid;                                                   \
        int row_ = p_ / PIECES_PER_ROW;                                                  \
        row_ = row_ < B ? row_ : B - 1; /* rows >= B: duplicate, never stored */         \
        areg[it] = *reinterpret_cast<const uint4*>(a + (size_t)row_ * lda + (k0) +       \
                                                   (p_ % PIECES_PER_ROW) * 8);           \
    }
#define PD_STORE_A(buf)                                                                  \
    _Pragma("unroll") for (int it = 0; it < APT; it++) {                                 \
        const int p_ = it * 256 + tid;                                                   \
        *reinterpret_cast<uint4*>(                                                       \
            &lds[buf][(p_ / PIECES_PER_ROW) * PITCH + (p_ % PIECES_PER_ROW) * 16]) = areg[it]; \
    }
#define PD_COMPUTE(buf)                                                                  \
    _Pragma("unroll") for (int kb = 0; kb < KB; kb++) {                                  \
        _Pragma("unroll") for (int e2 = 0; e2 < 2; e2++) {                               \
            bf16x8 aop[BM];                                                              \
            _Pragma("unroll") for (int bm = 0; bm < BM; bm++) {                          \
                uint4 v_ = *reinterpret_cast<const uint4*>(                              \
                    &lds[buf][(bm * 32 + l32) * PITCH + kb * 64 + g * 32 + e2 * 16]);    \
                aop[bm] = __builtin_bit_cast(bf16x8, v_);                                \
            }                                                                            \
            _Pragma("unroll") for (int i = 0; i < NS; i++) {                             \
                const uint4 w_ = wcur[i][kb];                                            \
                const bf16x8 bop = e2 == 0 ? cvt_i8x8(w_.x, w_.y) : cvt_i8x8(w_.z, w_.w); \
                _Pragma("unroll") for (int bm = 0; bm < BM; bm++)                        \
                    acc[i][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[bm], bop,   \
                                                                          acc[i][bm], 0, 0, 0); \
            }                                                                            \
        }                                                                                \
    }

    if (k_begin < k_end) {
        PD_LOAD_W(wcur, k_begin);
        PD_LOAD_A(k_begin);
        PD_STORE_A(0);
        __syncthreads();
        int cur = 0;
        // steady state: fetch stage k0 + KC while the MFMAs consume stage k0
        for (int k0 = k_begin; k0 + KC < k_end; k0 += KC) {
            PD_LOAD_W(wnext, k0 + KC);
            PD_LOAD_A(k0 + KC);
            PD_COMPUTE(cur);
            PD_STORE_A(cur ^ 1);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NS; i++)
#pragma unroll
                for (int kb = 0; kb < KB; kb++) wcur[i][kb] = wnext[i][kb];
            cur ^= 1;
        }
        PD_COMPUTE(cur);  // last stage, nothing left to fetch
    }
#undef PD_LOAD_W
#undef PD_LOAD_A
#undef PD_STORE_A
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
                int b = bm * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (b < B) part[((size_t)s * B + b) * N + n] = acc[i][bm][r];
            }
    }
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
    int BMv = blocks <= 1 ? 1 : blocks <= 2 ? 2 : blocks <= 4 ? 4 : 8;
    int NSv = BMv <= 4 ? 2 : 1;
    *bm = BMv;
    *ns = NSv;
    *tile_cols = 128 * NSv;
}

int qgemm_auto_splits(int B, int K, int N) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    int n_tiles = (N + tc - 1) / tc;
    int s = (400 + n_tiles / 2) / n_tiles;
    int cap = K / 128 < PD_MAX_SPLITS ? K / 128 : PD_MAX_SPLITS;
    if (s < 1) s = 1;
    if (s > cap) s = cap;
    return s;
}

hipError_t launch_qgemm(const void* wp, const uint16_t* a, float* part, int B, int K, int N,
                        int lda, int S, hipStream_t stream) {
    int bm, ns, tc;
    qgemm_config(B, &bm, &ns, &tc);
    dim3 grid((N + tc - 1) / tc, S), block(256);
    const uint4* w4 = reinterpret_cast<const uint4*>(wp);
    if (bm == 1)
        qgemm_kernel<1, 2, 128><<<grid, block, 0, stream>>>(w4, a, part, B, K, N, lda, S);
    else if (bm == 2)
        qgemm_kernel<2, 2, 128><<<grid, block, 0, stream>>>(w4, a, part, B, K, N, lda, S);
    else if (bm == 4)
        qgemm_kernel<4, 2, 64><<<grid, block, 0, stream>>>(w4, a, part, B, K, N, lda, S);
    else
        qgemm_kernel<8, 1, 32><<<grid, block, 0, stream>>>(w4, a, part, B, K, N, lda, S);
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
