// The small kernels between the two projections of the parallel block (paper
// Section 3.4: one LayerNorm per layer feeds both branches, attention and FFN
// outputs are summed by the fused output projection and added to the residual).
//   prep     : per-step rotation table cos/sin(positions[b] * base^(-2i/dh)), position check
//   ln_first : bf16 input -> fp32 residual stream + LayerNorm of layer 0
//   epi_in   : sum K-split partials of the input projection, apply the per-channel
//              scale (Section 3.6), rotate q and k, append k/v to the cache,
//              SwiGLU gate (Section 3.5 names the base-2 Swish)
//   epi_out  : sum partials of the output projection, scale, add the residual,
//              LayerNorm for the next layer (or the final bf16 rounding)
#include "common.h"
#include "kernels.h"

namespace pd {

__global__ __launch_bounds__(128) void prep_kernel(const int32_t* __restrict__ positions, int L_ctx,
                                                   int dh, double rope_base, float* __restrict__ cs,
                                                   int32_t* __restrict__ flag) {
    const int b = blockIdx.x, i = threadIdx.x;
    const int P = positions[b];
    const bool bad = P < 0 || P >= L_ctx;
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

// h = gamma * (x - mean) / sqrt(var + eps), population variance, two passes
__device__ __forceinline__ void layernorm_row(const float* __restrict__ xrow,
                                              const float* __restrict__ gamma, int d, float eps,
                                              float sum, uint16_t* __restrict__ hrow, float* red) {
    const int tid = threadIdx.x;
    const float mean = block_sum_256(sum, red) / (float)d;
    float sq = 0.f;
    for (int c = tid; c < d; c += 256) {
        float t = xrow[c] - mean;
        sq += t * t;
    }
    const float var = block_sum_256(sq, red) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    for (int c = tid; c < d; c += 256) hrow[c] = to_bf16(gamma[c] * (xrow[c] - mean) * rstd);
}

__global__ __launch_bounds__(256) void ln_first_kernel(const uint16_t* __restrict__ x_in,
                                                       const float* __restrict__ gamma, int d,
                                                       float eps, float* __restrict__ xres,
                                                       uint16_t* __restrict__ h) {
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    float* xrow = xres + (size_t)b * d;
    float sum = 0.f;
    for (int c = tid; c < d; c += 256) {
        float v = from_bf16(x_in[(size_t)b * d + c]);
        xrow[c] = v;  // each thread later re-reads only what it wrote itself
        sum += v;
    }
    layernorm_row(xrow, gamma, d, eps, sum, h + (size_t)b * d, red);
}

__device__ __forceinline__ float sum_partials(const float* __restrict__ part, int S, size_t stride,
                                              size_t off) {
    float acc = 0.f;
    for (int s = 0; s < S; s++) acc += part[(size_t)s * stride + off];  // fixed order
    return acc;
}

// Items per batch row: H*dh/2 q pairs | dh/2 k pairs | dh v elements | F FFN elements.
// `part` is in packed column order: q|k|v in place, then 64-column groups of
// (32 gate, 32 up).  Cache element offsets follow the library block layouts.
__global__ __launch_bounds__(256) void epi_in_kernel(
    const float* __restrict__ part, int S, const float* __restrict__ scale,
    const float* __restrict__ cs, const int32_t* __restrict__ positions, int B, int H, int dh, int F,
    int L_ctx, uint16_t* __restrict__ q, uint16_t* __restrict__ kc, uint16_t* __restrict__ vc,
    uint16_t* __restrict__ act, int act_stride) {
    const int b = blockIdx.y;
    const int item = blockIdx.x * 256 + threadIdx.x;
    const int half = dh >> 1;
    const int n_q = H * half, n_k = half, n_v = dh;
    const int n_qkv = H * dh + 2 * dh;
    const int N = n_qkv + 2 * F;
    const size_t stride = (size_t)B * N, rowoff = (size_t)b * N;
    const int P = positions[b];
    const bool ok = P >= 0 && P < L_ctx;

    if (item < n_q + n_k) {
        // rotation pair (i, i + dh/2) of a q head or of k
        const bool is_k = item >= n_q;
        const int pi = is_k ? item - n_q : item;
        const int head = is_k ? 0 : pi / half, i = pi % half;
        const int col = (is_k ? H * dh : head * dh) + i;
        float lo = scale[col] * sum_partials(part, S, stride, rowoff + col);
        float hi = scale[col + half] * sum_partials(part, S, stride, rowoff + col + half);
        const float cn = cs[((size_t)b * half + i) * 2], sn = cs[((size_t)b * half + i) * 2 + 1];
        const float rlo = lo * cn - hi * sn, rhi = hi * cn + lo * sn;
        if (!is_k) {
            uint16_t* qrow = q + ((size_t)b * H + head) * dh;
            qrow[i] = to_bf16(rlo);
            qrow[i + half] = to_bf16(rhi);
        } else if (ok) {
            const size_t blk = ((size_t)b * (L_ctx >> 5) + (P >> 5)) * 32 * dh;
            const int tt = P & 31;
            int c = i;
            kc[blk + (((size_t)(c >> 4) * 2 + ((c & 15) >> 3)) * 32 + tt) * 8 + (c & 7)] = to_bf16(rlo);
            c = i + half;
            kc[blk + (((size_t)(c >> 4) * 2 + ((c & 15) >> 3)) * 32 + tt) * 8 + (c & 7)] = to_bf16(rhi);
        }
    } else if (item < n_q + n_k + n_v) {
        const int c = item - n_q - n_k;
        const int col = H * dh + dh + c;
        float v = scale[col] * sum_partials(part, S, stride, rowoff + col);
        if (ok) {
            const size_t blk = ((size_t)b * (L_ctx >> 5) + (P >> 5)) * 32 * dh;
            const int tt = P & 31;
            vc[blk + ((((size_t)(c >> 5) * 2 + (tt >> 4)) * 2 + ((tt & 7) >> 2)) * 32 + (c & 31)) * 8 +
               4 * ((tt & 15) >> 3) + (tt & 3)] = to_bf16(v);
        }
    } else if (item < n_q + n_k + n_v + F) {
        const int f = item - n_q - n_k - n_v;
        const int pcol = n_qkv + (f >> 5) * 64 + (f & 31);
        float gt = scale[pcol] * sum_partials(part, S, stride, rowoff + pcol);
        float up = scale[pcol + 32] * sum_partials(part, S, stride, rowoff + pcol + 32);
        // swish(g) = g / (1 + e^-g) = g / (1 + 2^(-g log2 e))
        float sw = gt / (1.0f + __builtin_amdgcn_exp2f(-gt * 1.4426950408889634f));
        act[(size_t)b * act_stride + H * dh + f] = to_bf16(sw * up);
    }
}

__global__ __launch_bounds__(256) void epi_out_kernel(const float* __restrict__ part, int S,
                                                      const float* __restrict__ scale,
                                                      float* __restrict__ xres,
                                                      const float* __restrict__ gamma_next, int B,
                                                      int d, float eps, int add_residual,
                                                      uint16_t* __restrict__ h,
                                                      uint16_t* __restrict__ x_out_bf16,
                                                      float* __restrict__ y_out_f32) {
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    float* xrow = xres + (size_t)b * d;
    const size_t stride = (size_t)B * d, rowoff = (size_t)b * d;
    float sum = 0.f;
    for (int c = tid; c < d; c += 256) {
        float y = scale[c] * sum_partials(part, S, stride, rowoff + c);
        float xn = add_residual ? xrow[c] + y : y;
        xrow[c] = xn;
        sum += xn;
        if (x_out_bf16) x_out_bf16[rowoff + c] = to_bf16(xn);
        if (y_out_f32) y_out_f32[rowoff + c] = xn;
    }
    if (gamma_next) layernorm_row(xrow, gamma_next, d, eps, sum, h + rowoff, red);
}

hipError_t launch_prep(const int32_t* positions, int B, int L_ctx, int dh, float rope_base,
                       float* cs, int32_t* flag, hipStream_t stream) {
    prep_kernel<<<dim3(B), dim3(128), 0, stream>>>(positions, L_ctx, dh, (double)rope_base, cs, flag);
    return hipGetLastError();
}

hipError_t launch_ln_first(const uint16_t* x_in, const float* gamma, int B, int d, float eps,
                           float* xres, uint16_t* h, hipStream_t stream) {
    ln_first_kernel<<<dim3(B), dim3(256), 0, stream>>>(x_in, gamma, d, eps, xres, h);
    return hipGetLastError();
}

hipError_t launch_epi_in(const float* part, int S, const float* scale, const float* cs,
                         const int32_t* positions, int B, int H, int dh, int F, int L_ctx,
                         uint16_t* q, void* kc_layer, void* vc_layer, uint16_t* act, int act_stride,
                         hipStream_t stream) {
    int items = H * dh / 2 + dh / 2 + dh + F;
    epi_in_kernel<<<dim3((items + 255) / 256, B), dim3(256), 0, stream>>>(
        part, S, scale, cs, positions, B, H, dh, F, L_ctx, q, reinterpret_cast<uint16_t*>(kc_layer),
        reinterpret_cast<uint16_t*>(vc_layer), act, act_stride);
    return hipGetLastError();
}

hipError_t launch_epi_out(const float* part, int S, const float* scale, float* xres,
                          const float* gamma_next, int B, int d, float eps, int add_residual,
                          uint16_t* h, uint16_t* x_out_bf16, float* y_out_f32, hipStream_t stream) {
    epi_out_kernel<<<dim3(B), dim3(256), 0, stream>>>(part, S, scale, xres, gamma_next, B, d, eps,
                                                      add_residual, h, x_out_bf16, y_out_f32);
    return hipGetLastError();
}

}  // namespace pd
