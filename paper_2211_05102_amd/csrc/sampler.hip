// The tail of a generation step (paper Section 2.2: after each forward pass one new
// token is sampled per sequence and fed back; Section 3.5 lists fast top-k / top-p
// sampling among the low-level optimisations):
//   sample : top-k / top-p draw of one token per row from fp32 logits [B][V]
//   embed  : next hidden state = embedding row of the sampled token; position and
//            step counters advance on the device, so the whole loop replays as a graph
//
// sample_kernel, one workgroup of 1024 threads per row:
//   1. exact k-th largest logit by radix select on an order-preserving integer key
//      (four 8-bit digits, most significant first, 256-bin histograms in LDS);
//   2. the candidates = every entry above that value, plus as many entries equal to it
//      as are needed to reach k, smallest indices first (an ordered, ballot-ranked scan:
//      no dependence on timing);
//   3. the k candidates are ranked (logit descending, index ascending) by one wavefront;
//   4. softmax with temperature over them, the shortest prefix whose mass reaches top_p,
//      and the inverse-CDF draw with the caller's uniform number, serially in fp32 by
//      one lane (k <= 64 terms: fixed order, bit-reproducible).
#include "common.h"
#include "kernels.h"

namespace pd {

constexpr int SM_THREADS = 1024;
constexpr int SM_WAVES = SM_THREADS / 64;

// larger float <-> larger key; -0 and +0 differ by one step, NaNs sort above +inf
// (logits are finite by contract)
__device__ __forceinline__ uint32_t order_key(float v) {
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(SM_THREADS) void sample_kernel(
    const float* __restrict__ logits, int V, int top_k, float top_p, float inv_temperature,
    const float* __restrict__ uniforms, const int32_t* __restrict__ step, int B,
    int32_t* __restrict__ tokens) {
    __shared__ int hist[256];
    __shared__ int wave_eq[SM_WAVES];
    __shared__ uint32_t s_prefix, s_mask;
    __shared__ int s_need, s_cnt;
    __shared__ uint32_t cand_key[PD_MAX_TOP_K];
    __shared__ int cand_idx[PD_MAX_TOP_K];
    __shared__ float sort_logit[PD_MAX_TOP_K];
    __shared__ int sort_idx[PD_MAX_TOP_K];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const float* row = logits + (size_t)b * V;
    const int it = step ? step[0] : 0;  // generation step: selects this step's uniforms and output row

    // ---- 1. radix select: after the loop `prefix` is the key of the k-th largest entry
    if (tid == 0) { s_prefix = 0; s_mask = 0; s_need = top_k; }
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix, mask = s_mask;
        for (int i = tid; i < V; i += SM_THREADS) {
            const uint32_t key = order_key(row[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);  // integer: order-free
        }
        __syncthreads();
        if (tid == 0) {
            int need = s_need, d = 255;
            while (d > 0 && hist[d] < need) { need -= hist[d]; d--; }
            s_need = need;  // entries still to take among those whose digit equals d
            s_prefix = prefix | ((uint32_t)d << shift);
            s_mask = mask | (255u << shift);
        }
        __syncthreads();
    }
    const uint32_t kth = s_prefix;
    const int need_eq = s_need;  // entries equal to the k-th largest that belong to the top k

    // ---- 2. candidates.  Each wave owns a contiguous segment of the row and walks it in
    // 64-wide steps, so (step, lane) order is index order.
    const int seg = (V + SM_WAVES - 1) / SM_WAVES;
    const int lo = wave * seg, hi = lo + seg < V ? lo + seg : V;
    int n_eq = 0;
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const bool eq = i < hi && order_key(row[i]) == kth;
        n_eq += __popcll(__ballot(eq));
    }
    if (tid == 0) s_cnt = 0;
    if (lane == 0) wave_eq[wave] = n_eq;
    __syncthreads();
    int eq_before = 0;  // equal entries in the segments of lower waves
    for (int w = 0; w < wave; w++) eq_before += wave_eq[w];
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? order_key(row[i]) : 0u;
        const bool gt = i < hi && key > kth, eq = i < hi && key == kth;
        const unsigned long long m_eq = __ballot(eq);
        bool take = gt;
        if (eq) take = eq_before + __popcll(m_eq & ((1ull << lane) - 1ull)) < need_eq;
        eq_before += __popcll(m_eq);
        if (take) {
            const int slot = atomicAdd(&s_cnt, 1);  // slot order is irrelevant: ranked below
            cand_key[slot] = key;
            cand_idx[slot] = i;
        }
    }
    __syncthreads();

    // ---- 3. rank by (logit descending, index ascending): exactly top_k candidates
    if (wave == 0) {
        if (lane < top_k) {
            const uint32_t key = cand_key[lane];
            const int idx = cand_idx[lane];
            int rank = 0;
            for (int j = 0; j < top_k; j++) {
                const uint32_t kj = cand_key[j];
                rank += (kj > key || (kj == key && cand_idx[j] < idx)) ? 1 : 0;
            }
            sort_logit[rank] = row[idx];
            sort_idx[rank] = idx;
        }
    }
    __syncthreads();

    // ---- 4. softmax over the k candidates, nucleus, draw
    if (tid == 0) {
        const float z0 = sort_logit[0] * inv_temperature;
        float total = 0.f;
        for (int j = 0; j < top_k; j++)
            total += __builtin_amdgcn_exp2f((sort_logit[j] * inv_temperature - z0) * 1.4426950408889634f);
        // shortest prefix with probability mass >= top_p (unnormalised: mass >= top_p * total)
        const float want = top_p * total;
        float c = 0.f;
        int n = 0;
        while (n < top_k) {
            c += __builtin_amdgcn_exp2f((sort_logit[n] * inv_temperature - z0) * 1.4426950408889634f);
            n++;
            if (c >= want) break;
        }
        const float target = uniforms[(size_t)it * B + b] * c;
        float run = 0.f;
        int pick = n - 1;
        for (int j = 0; j < n; j++) {
            run += __builtin_amdgcn_exp2f((sort_logit[j] * inv_temperature - z0) * 1.4426950408889634f);
            if (run > target) { pick = j; break; }
        }
        tokens[(size_t)it * B + b] = sort_idx[pick];
    }
}

// x_next[b] = embed[token[b]]; positions[b] += 1; the step counter advances once
__global__ __launch_bounds__(256) void embed_advance_kernel(const uint16_t* __restrict__ embed, int d, int V,
                                                            const int32_t* __restrict__ tokens, int B,
                                                            uint16_t* __restrict__ x_next,
                                                            int32_t* __restrict__ positions,
                                                            int32_t* __restrict__ step) {
    const int b = blockIdx.x;
    const int it = step[0];
    int tok = tokens[(size_t)it * B + b];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);  // (the sampler only produces valid ids)
    const uint4* src = reinterpret_cast<const uint4*>(embed + (size_t)tok * d);
    uint4* dst = reinterpret_cast<uint4*>(x_next + (size_t)b * d);
    for (int i = threadIdx.x; i < d / 8; i += 256) dst[i] = src[i];
    if (threadIdx.x == 0) positions[b] += 1;
    // every block has read step[0] before the last block to finish could have changed it:
    // the counter is advanced by a separate one-thread launch
}

__global__ void step_advance_kernel(int32_t* __restrict__ step, int value, int add) {
    if (threadIdx.x == 0 && blockIdx.x == 0) step[0] = add ? step[0] + value : value;
}

hipError_t launch_sample(const float* logits, int B, int V, int top_k, float top_p, float temperature,
                         const float* uniforms, const int32_t* step, int32_t* tokens,
                         hipStream_t stream) {
    if (top_k < 1 || top_k > PD_MAX_TOP_K || top_k > V) return hipErrorInvalidValue;
    sample_kernel<<<dim3(B), dim3(SM_THREADS), 0, stream>>>(logits, V, top_k, top_p, 1.0f / temperature,
                                                           uniforms, step, B, tokens);
    return hipGetLastError();
}

hipError_t launch_embed_advance(const uint16_t* embed, int d, int V, const int32_t* tokens, int B,
                                uint16_t* x_next, int32_t* positions, int32_t* step, hipStream_t stream) {
    embed_advance_kernel<<<dim3(B), dim3(256), 0, stream>>>(embed, d, V, tokens, B, x_next, positions, step);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    step_advance_kernel<<<dim3(1), dim3(64), 0, stream>>>(step, 1, 1);
    return hipGetLastError();
}

hipError_t launch_step_set(int32_t* step, int value, hipStream_t stream) {
    step_advance_kernel<<<dim3(1), dim3(64), 0, stream>>>(step, value, 0);
    return hipGetLastError();
}

}  // namespace pd
