// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"

#define PD_MIN_BLOCKS_PER_SPLIT 4 // 32-token blocks per attention workgroup, lower bound

namespace pd {

// ---- qgemm.hip
void qgemm_config(int B, int* bm, int* ns, int* tile_cols);
// tile_cols = 0: the int8 kernel's tile width; PD_WGEMM_TILE_COLS for the bf16-weight kernel
SkqPlan qgemm_plan(int B, int K, int N, int workgroups, int c_split, int blk0, int blk1,
                   int* max_slots, int tile_cols = 0);
int qgemm_auto_workgroups(int B, int K, int N, int g_max, int c_split, int blk0, int blk1, int tile_cols = 0);
hipError_t launch_skq_table(SkqPlan pl, int* nseg, hipStream_t stream);
hipError_t launch_qgemm(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                        int K, int N, SkqPlan pl, int nd, hipStream_t stream);
hipError_t launch_quantize_bf16(const uint16_t* a, void* qa, float* scale_t, int B, int K, int nd,
                                hipStream_t stream);
hipError_t launch_pack_matrix(const int8_t* w, void* dst, int K, int N, int mode, int n_qkv, int F,
                              hipStream_t stream);
hipError_t launch_pack_vector(const uint16_t* src, float* dst, int N, int mode, int n_qkv, int F,
                              hipStream_t stream);
hipError_t launch_qgemm_reduce(const float* part, const float* scale, float* out, int B, int N,
                               SkqPlan pl, hipStream_t stream);

// ---- wgemm.hip: the same product with bf16 weights (same kind of plan with tiles of
// PD_WGEMM_TILE_COLS columns, same partial slots)
#define PD_WGEMM_TILE_COLS 512
hipError_t launch_wgemm_bf16(const void* wp, const void* qa, const float* scale_t, float* part, int B,
                             int K, int N, SkqPlan pl, int nd, hipStream_t stream);
hipError_t launch_pack_matrix_bf16(const uint16_t* w, void* dst, int K, int N, int mode, int n_qkv, int F,
                                   hipStream_t stream);
hipError_t launch_fill_f32(float* dst, int n, float v, hipStream_t stream);

// ---- attention.hip
hipError_t launch_mqa_attend(const float* q, const void* kc_layer, const void* vc_layer,
                             const int32_t* positions, const int32_t* seq, int cache_rows, int B, int H,
                             int G, int dh, int L_ctx, int bps,
                             float* opart, float* ml, float* o, void* actq, float* acts,
                             int k_out, int blk_o, int nd, hipStream_t stream);
hipError_t launch_kv_convert(const void* src, void* dst, int B, int L_ctx, int dh, int is_v,
                             int to_library, hipStream_t stream);

// ---- pointwise.hip
// `seq` (may be NULL = identity): cache row of each token row; `cache_rows` = rows of the cache
hipError_t launch_prep(const int32_t* positions, int B, int L_ctx, int dh, float rope_base,
                       float* cs, int32_t* flag, const int32_t* seq, int cache_rows, hipStream_t stream);
hipError_t launch_ln_first(const uint16_t* x_in, const float* gamma, int B, int d, float eps,
                           float* xres, void* hq, float* hs, int nd, hipStream_t stream);
hipError_t launch_epi_in(const float* part, SkqPlan pl, const float* scale, const float* cs,
                         const int32_t* positions, const int32_t* seq, int cache_rows, int B, int H, int G,
                         int dh, int F, int L_ctx,
                         float* q, void* kc_layer, void* vc_layer, void* actq, float* acts,
                         int blk_a, int nd, hipStream_t stream);
hipError_t launch_residual(const float* part, SkqPlan pl, const float* scale, float* xres, int B,
                           int d, int add_residual, uint16_t* x_out_bf16, float* y_out_f32,
                           float* stats, hipStream_t stream);
hipError_t launch_ln_slices(const float* xres, const float* gamma, const float* gamma_absmax,
                            const float* stats, int B, int d, float eps, void* hq, float* hs,
                            int nd, hipStream_t stream);
// residual add + LayerNorm of the next layer in one launch; rows of at most
// PD_RESIDUAL_LN_MAX_D columns
#define PD_RESIDUAL_LN_MAX_D 16384
hipError_t launch_residual_ln(const float* part, SkqPlan pl, const float* scale, float* xres, int B,
                              int d, int add_residual, const float* gamma, float eps, void* hq, float* hs,
                              int nd, hipStream_t stream);
hipError_t launch_vec_absmax(const float* v, int n, float* out, hipStream_t stream);

// ---- sampler.hip
#define PD_MAX_TOP_K 64
hipError_t launch_sample(const float* logits, int B, int V, int top_k, float top_p, float temperature,
                         const float* uniforms, const int32_t* step, int32_t* tokens,
                         hipStream_t stream);
hipError_t launch_embed_advance(const uint16_t* embed, int d, int V, const int32_t* tokens, int B,
                                uint16_t* x_next, int32_t* positions, int32_t* step, hipStream_t stream);
hipError_t launch_step_set(int32_t* step, int value, hipStream_t stream);

// ---- probe.hip
hipError_t launch_ceiling_probe(const void* src, size_t bytes, int mfma_per_unit, int random_operands,
                                unsigned* sink, hipStream_t stream);

}  // namespace pd
