/*
 * palmdecode.h -- C ABI of the MI355X (gfx950) int8-weight multiquery decode step.
 *
 * One generate-phase step of a PaLM-style stack (paper Section 2.2: one forward
 * pass over B x 1 tokens; Section 3.4: parallel block
 *     x' = x + Attn(LN(x)) + SwiGLU-FFN(LN(x))
 * with the input projections fused into one matrix and the two output
 * projections fused into another; Section 3.3: multiquery attention, all query
 * heads share one K/V head; Section 3.6: int8 weights, one scale per output
 * channel, arithmetic in bf16/fp32).
 *
 * Conventions
 *   - Every function returns a pd_status (0 = PD_OK, negative = error) and
 *     never throws.  pd_last_error() returns a thread-local text for the last
 *     failure on the calling thread.
 *   - "device" pointers are HIP device memory owned by the CALLER for the whole
 *     call (and until the stream has drained); the library allocates no device
 *     memory.  "host" pointers are ordinary host memory.
 *   - bf16 values are passed as uint16_t bit patterns.
 *   - Device pointers must be 16-byte aligned (256 for packed weights, caches
 *     and workspace).  All argument errors are detected on the host before
 *     anything is enqueued: on error nothing has been launched.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     are asynchronous: they return after enqueueing.
 *
 * Canonical (caller-side) layouts
 *   w_in   [d_model][n_in]  int8 row-major, columns q(H*dh) | k(dh) | v(dh) | gate(F) | up(F)
 *   s_in   [n_in]           bf16, scale of output channel n:  W[k][n] = w_in[k][n] * s_in[n]
 *   w_out  [k_out][d_model] int8 row-major, rows attention-out(H*dh) | FFN activation(F)
 *   s_out  [d_model]        bf16
 *   gamma  [d_model]        bf16 LayerNorm gain (no bias; eps inside the root)
 *   K, V   [B][G][L_ctx][d_head] bf16 per layer (K holds rotated keys), G = n_kv_heads
 *   with n_in = H*dh + 2*G*dh + 2*F (k and v: one block of dh columns per K/V head)
 *   and k_out = H*dh + F.  G = 1 is the multiquery layout of Section 3.3 (all query
 *   heads share one K/V head); G = H is the multihead baseline it is compared with
 *   (Section 3.3, Section 4.2); any G that divides H works (query heads j*H/G ..
 *   (j+1)*H/G - 1 read K/V head j).
 *
 * Library-side layouts (Section 3.5 lists in-memory tensor layout among the
 * low-level optimisations; these are this library's, chosen so that every
 * 64-lane wavefront streams 1 KiB contiguous pieces straight into MFMA operands)
 *   packed layer  = pd_packed_layer_bytes() bytes made by pd_pack_layer().
 *   K cache [n_layers][B*G][L_ctx/32][dh/16][2][32][8] bf16 (K/V head j of row b at b*G + j):
 *       element (l,b,t,c) -> [l][b][t/32][c/16][(c%16)/8][t%32][c%8]
 *   V cache [n_layers][B*G][L_ctx/32][dh/32][2][2][32][8] bf16:
 *       element (l,b,t,c) -> [l][b][t/32][c/32][(t%32)/16][(t%8)/4][c%32][4*((t%16)/8) + t%4]
 *   L_ctx must be a multiple of 32.  pd_kv_import()/pd_kv_export() convert one
 *   layer between canonical and library layout.
 */
#ifndef PALMDECODE_H
#define PALMDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t pd_status;
enum {
    PD_OK = 0,
    PD_ERR_NULL = -1,      /* a required pointer is NULL */
    PD_ERR_ALIGN = -2,     /* a device pointer is not aligned as required */
    PD_ERR_SHAPE = -3,     /* model shape / batch / context not supported */
    PD_ERR_RANGE = -4,     /* an index argument is out of range */
    PD_ERR_WORKSPACE = -5, /* workspace_bytes smaller than pd_workspace_bytes() */
    PD_ERR_HIP = -6,       /* a HIP runtime call failed */
    PD_ERR_POSITION = -7,  /* a device-side positions[b] was outside [0, L_ctx) */
    PD_ERR_STATE = -8      /* call not valid in the handle's current state */
};

/* Model description (Section 2.2 notation: d_model = E, d_ff = F, n_heads = H).
 * Supported: d_model % 128 == 0, d_ff % 128 == 0, (H*d_head) % 128 == 0,
 * d_head in {64, 128, 256}, 1 <= n_heads <= 256, n_kv_heads divides n_heads and at
 * most 32 query heads share a K/V head; each projection
 * matrix smaller than 4 GiB; batch 1..256; L_ctx a multiple of 32.  Anything else
 * is refused with PD_ERR_SHAPE by every call that takes the description. */
/* flags bit: w_in and w_out are bf16 with no scales, the unquantised format that
 * Section 4.4 compares the int8 weights of Section 3.6 with.  Twice the weight
 * bytes per step; everything else (layouts, caches, calls) is unchanged. */
#define PD_FLAG_BF16_WEIGHTS 1

typedef struct pd_model_desc {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_heads;
    int32_t d_head;
    int32_t d_ff;       /* per SwiGLU branch */
    int32_t n_kv_heads; /* 1 = multiquery (Section 3.3), n_heads = multihead */
    float rope_base;    /* 10000 */
    float ln_eps;       /* 1e-6 */
    int32_t flags;      /* 0, or PD_FLAG_BF16_WEIGHTS */
} pd_model_desc;

typedef struct pd_handle pd_handle;

const char* pd_status_string(pd_status code);
const char* pd_last_error(void);

/* ---- sizes: pure host functions ------------------------------------------
 * Section 2 ("Memory costs") counts exactly these two tensors per step: the
 * weights and the KV cache; the third size is this library's own scratch. */

/* Bytes of one packed layer (int8 or bf16 matrices, fp32 scales and gain, 256-aligned).
 * The packed stack is n_layers such blobs back to back. */
pd_status pd_packed_layer_bytes(const pd_model_desc* desc, size_t* bytes);
/* Bytes of EACH of the K cache and the V cache for batch B, capacity L_ctx. */
pd_status pd_kv_cache_bytes(const pd_model_desc* desc, int32_t B, int32_t L_ctx, size_t* bytes);
/* Scratch a decode call needs for batch B, capacity L_ctx. */
pd_status pd_workspace_bytes(const pd_model_desc* desc, int32_t B, int32_t L_ctx, size_t* bytes);

/* ---- handle --------------------------------------------------------------- */

/* Validates and copies `desc` (the model of Section 2.2 / Section 3.4).  The
 * handle owns host state only (launch plan, an optional captured graph). */
pd_status pd_create(const pd_model_desc* desc, pd_handle** out);
pd_status pd_destroy(pd_handle* h);
/* Tuning knobs (not part of the decode contract; defaults are what the
 * benchmark times): "gemm_workgroups_in", "gemm_workgroups_out" (workgroups that
 * share the weight matrix of the input / output projection, 0 = automatic:
 * at most one per compute unit and 64-row group, chosen so that the ranges come
 * out even; values above 256 are rejected),
 * "attn_blocks_per_split" (32-token blocks per attention
 * workgroup, 0 = automatic), "act_digits" (2 or 3 int8 digit planes per
 * projection operand), "profile_kernel" (see pd_profile_read).  Unknown names
 * return PD_ERR_RANGE. */
pd_status pd_set_option(pd_handle* h, const char* name, int32_t value);

/* Event timing of one kernel class, for the roofline report (measurement
 * interface; no passage of the paper defines it).  Option
 * "profile_kernel" = 1 (input projection), 2 (attention + combine), 3 (output
 * projection), 4 (input epilogue), 5 (output epilogue), 0 = off: while on, every
 * launch of that class made by pd_decode_step/pd_decode_layer is bracketed by
 * HIP events on the caller's stream.  pd_profile_read() waits for them, returns
 * the summed duration and the number of launches, and resets the counters. */
pd_status pd_profile_read(pd_handle* h, double* total_ms, int32_t* launches);

/* ---- data preparation ----------------------------------------------------- */

/* Re-tiles one layer's canonical device tensors into the packed blob at
 * `packed_layer` (device, 256-aligned, pd_packed_layer_bytes() bytes).  The
 * canonical buffers may be freed once the stream has drained.  Section 3.5
 * (tensor layouts chosen to avoid padding and copies in the matrix multiplies).
 * With PD_FLAG_BF16_WEIGHTS the two matrices are bf16 (same shapes, passed through
 * the same two pointers) and s_in, s_out are ignored (may be NULL). */
pd_status pd_pack_layer(pd_handle* h, const int8_t* w_in, const uint16_t* s_in,
                        const int8_t* w_out, const uint16_t* s_out, const uint16_t* gamma,
                        void* packed_layer, void* stream);

/* Generic pieces of the same packing for a single [K][N] int8 matrix (K % 128
 * == 0, N % 32 == 0): packed_w gets K*N bytes. */
pd_status pd_pack_matrix(const int8_t* w, int32_t K, int32_t N, void* packed_w, void* stream);
/* The same for a bf16 matrix (the Section 4.4 baseline format): packed_w gets 2*K*N
 * bytes; K*N below 2^31. */
pd_status pd_pack_matrix_bf16(const uint16_t* w, int32_t K, int32_t N, void* packed_w, void* stream);

/* One layer of the cache, canonical [B][L_ctx][dh] <-> library layout, at layer
 * index `layer` of the library-side K or V cache (`is_v` selects the V layout).
 * The cache is the per-sequence K/V store of Section 2 ("Memory costs"), with one
 * K/V head per layer (Section 3.3); the library layout is a permutation of it
 * inside 32-token blocks, so slot (l, b, t) of one is slot (l, b, t) of the other. */
pd_status pd_kv_import(pd_handle* h, const uint16_t* canonical, void* cache, int32_t layer,
                       int32_t B, int32_t L_ctx, int32_t is_v, void* stream);
pd_status pd_kv_export(pd_handle* h, const void* cache, uint16_t* canonical, int32_t layer,
                       int32_t B, int32_t L_ctx, int32_t is_v, void* stream);

/* ---- the hot path --------------------------------------------------------- */

/*
 * One decode step of the whole stack (Section 2.2; Section 3.4 block).
 *   packed_weights  device, n_layers packed layers back to back
 *   k_cache,v_cache device, library layout, in/out: for every layer l and
 *                   sequence b exactly slot (l, b, positions[b]) is written
 *                   (rotated key / value of this token, rounded to bf16) and
 *                   slots 0..positions[b] are read; nothing else is touched
 *   x_in            device [B][d_model] bf16
 *   positions       device [B] int32, index of the token being decoded
 *   x_out           device [B][d_model] bf16 (may alias x_in): hidden state after
 *                   the last block; the residual stream is fp32 inside the call
 *   workspace       device, >= pd_workspace_bytes(desc, B, L_ctx)
 * A positions[b] outside [0, L_ctx) is device data the host cannot see: that
 * row writes nothing to the cache, its x_out row is unspecified, and a flag is
 * raised in the workspace that pd_check_async() reports.
 */
pd_status pd_decode_step(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                         const uint16_t* x_in, const int32_t* positions, int32_t B, int32_t L_ctx,
                         uint16_t* x_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Prefill, whole or incremental (Section 2.2: the input tokens are all present at the
 * start and run through the model in parallel; Section 3.5: incremental processing
 * of sequences during prefill).  n_tokens token rows, each with the cache row
 * (sequence) it belongs to and its position; every row appends its K/V at
 * (seq_ids[r], positions[r]) and attends over slots 0..positions[r] of that cache
 * row -- causal attention, since tokens after it sit at higher slots.  Rows are
 * processed in chunks of 256 in array order; a token's predecessors must be in the
 * cache already or come no later than the token's own chunk (e.g. rows ordered by
 * position), and no (sequence, position) pair may occur twice in a chunk.  Sequences
 * may already hold cached tokens (incremental prefill) and may have different
 * lengths.  The caches have `cache_rows` rows of capacity L_ctx
 * (pd_kv_cache_bytes(desc, cache_rows, L_ctx)); workspace >=
 * pd_workspace_bytes(desc, min(n_tokens, 256), L_ctx).  x_out [n_tokens][d_model] bf16
 * is the hidden state of every token after the last block (may alias x_in).  Device
 * data that is out of range (position, sequence id) skips the row and raises the flag
 * pd_check_async() reports for the last chunk.
 */
pd_status pd_prefill(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                     const uint16_t* x_in, const int32_t* seq_ids, const int32_t* positions,
                     int32_t n_tokens, int32_t cache_rows, int32_t L_ctx, uint16_t* x_out,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * One layer of the step, for per-layer checks and for a weight shard's
 * unreduced partial (Section 3.2.1: a 1D weight-stationary shard over heads
 * and d_ff produces a partial sum that still needs a cross-chip reduction).
 *   layer         index into the caches (the packed blob is passed directly)
 *   y_out         device [B][d_model] fp32: x + block(x) if add_residual != 0,
 *                 else block(x) alone
 */
pd_status pd_decode_layer(pd_handle* h, int32_t layer, const void* packed_layer, void* k_cache,
                          void* v_cache, const uint16_t* x_in, const int32_t* positions, int32_t B,
                          int32_t L_ctx, float* y_out, int32_t add_residual, void* workspace,
                          size_t workspace_bytes, void* stream);

/* Synchronises `stream`, then reports the per-row position flags the most
 * recent step on this `workspace` left: PD_OK or PD_ERR_POSITION.  `workspace`
 * NULL = the scratch of pd_decode_step_static() on the current device.
 * (Section 2.2: a step decodes the token at positions[b]; a position outside
 * the cache has no defined result.) */
pd_status pd_check_async(pd_handle* h, void* workspace, void* stream);

/*
 * For callers that cannot allocate or pass device scratch: code under HIP graph
 * capture that must not call an allocator, tight serving loops, harnesses that
 * forbid allocation.  The same step as pd_decode_step() -- same kernels, same
 * results bit for bit -- with the workspace taken from a fixed array inside the
 * library's device image (64 MiB per GPU, held until the process ends) instead of
 * from the caller.  Calls no allocator of any kind.  Shapes whose
 * pd_workspace_bytes() exceeds 64 MiB are refused with PD_ERR_WORKSPACE and a
 * message that says how much was needed; nothing is enqueued then.
 * All calls on one GPU share that GPU's array: two calls whose execution overlaps
 * on one GPU (different streams, or another thread) race; calls on one stream are
 * ordered and safe.  The array needs no initial contents: every step writes what
 * it later reads.  The device address of the array is looked up on the first
 * call on each device (make that call before starting a stream capture).
 * pd_check_async(h, NULL, stream) reads this step's position flags.
 */
pd_status pd_decode_step_static(pd_handle* h, const void* packed_weights, void* k_cache,
                                void* v_cache, const uint16_t* x_in, const int32_t* positions,
                                int32_t B, int32_t L_ctx, uint16_t* x_out, void* stream);

/* ---- single steps of the path (tests, profiling) -------------------------- */

/* out[b][n] = s[n] * sum_k a[b][k] * w[k][n]   (Section 3.6 weight-only int8)
 *   packed_w from pd_pack_matrix, scale [N] fp32 device, a [B][K] bf16 device,
 *   out [B][N] fp32 device, B <= 256.  workspace >= pd_qgemm_workspace_bytes().
 *   `workgroups` (0 = automatic, else 1..4096) is the number of workgroups the
 *   matrix is shared between; the result is bit-reproducible for a given value.
 *   The activations are converted to the library's 3-digit block fixed point
 *   (23 bits relative to each 128-element chunk's maximum) before the product. */
pd_status pd_qgemm_workspace_bytes(int32_t B, int32_t K, int32_t N, int32_t workgroups, size_t* bytes);

/* Host only (no GPU work): the deterministic work split of a [K][N] projection for
 * batch B over `workgroups` workgroups (0 = automatic), as the kernels use it
 * (Section 3.4's fused projections are the two instances).  Units = (column tile,
 * 128-row chunk of K), tile-major; workgroup g owns units [range_begin[g],
 * range_begin[g + 1]); the part of a tile inside one range is one partial-sum slot.
 *   counts[5] (host, required) = { workgroups used G, tiles T, chunks per tile C,
 *                                  padded rows of a partial slot, most slots in a tile }
 *   range_begin (host, optional) >= G + 1 entries;  first_slot (host, optional) >= G
 *   entries: slot index of range g inside its first tile;  slots_per_tile (host,
 *   optional) >= T entries.  Call once with the optional arrays NULL to size them.
 * c_split / blk0 / blk1: scale blocks of the operand (chunks [0, c_split) in blocks
 * of blk0, the rest in blocks of blk1); they decide how ranges are aligned. */
pd_status pd_qgemm_plan(int32_t B, int32_t K, int32_t N, int32_t workgroups, int32_t c_split,
                        int32_t blk0, int32_t blk1, int32_t* counts, int64_t* range_begin,
                        int32_t* first_slot, int32_t* slots_per_tile);
pd_status pd_qgemm(const void* packed_w, const float* scale, const uint16_t* a, int32_t B,
                   int32_t K, int32_t N, float* out, int32_t workgroups, void* workspace,
                   size_t workspace_bytes, void* stream);
/* out[b][n] = sum_k a[b][k] * w[k][n] with bf16 weights and no scales (the
 * Section 4.4 baseline format): packed_w from pd_pack_matrix_bf16, otherwise as
 * pd_qgemm (same workspace size, same plan). */
pd_status pd_wgemm_bf16(const void* packed_w, const uint16_t* a, int32_t B, int32_t K, int32_t N,
                        float* out, int32_t workgroups, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Ceiling probe (measurement aid of the benchmark; no passage of the paper defines
 * it).  One launch streams `buffer` (device, `bytes` a positive multiple of 8 MiB,
 * read only) once over all compute units and, independent of the data, issues
 * `mfma_per_unit` (a multiple of 6) int8 32x32x32 matrix instructions per wavefront
 * for every 8 KiB the wavefront loads; 48 is the ratio of the weight-only int8
 * projection with three digit planes at 64 rows (384 operations per weight byte,
 * Section 3.6), 0 a plain streaming read.  random_operands = 1: the matrix operands
 * are uniformly random bit patterns that differ between consecutive instructions
 * (largest power draw); 2: operands with the value statistics of the projections
 * (bell-shaped weights and top digits, uniform lower digits); 0: constants.  `sink`: 4 bytes of device memory (never written in
 * practice).  Time the launches yourself (events on `stream`): bytes / time and
 * mfma_per_unit * 65536 * bytes / 8192 / time are the pair the chip sustains. */
pd_status pd_ceiling_probe(const void* buffer, size_t bytes, int32_t mfma_per_unit,
                           int32_t random_operands, void* sink, void* stream);

/* Multiquery attention of one layer over the library-layout cache (Section 3.3):
 *   q [B][H][dh] fp32 (already rotated, unscaled), o [B][H*dh] fp32,
 *   attends over slots 0..positions[b] of layer `layer`. */
pd_status pd_mqa_attend(pd_handle* h, int32_t layer, const float* q, const void* k_cache,
                        const void* v_cache, const int32_t* positions, int32_t B, int32_t L_ctx,
                        float* o, void* workspace, size_t workspace_bytes, void* stream);

/* ---- sampling head and the generation loop --------------------------------
 * Section 2.2: generation is a sequential loop of L_gen steps; each step is one
 * forward pass after which one new token is sampled for each of the B sequences
 * and fed back.  Section 3.5 names fast top-k / top-p sampling for decode.  The
 * model tail is PaLM's by citation; the reading used here: a final LayerNorm
 * (same definition as in the blocks, own gain), logits = LN(x) . W_vocab with
 * W_vocab [d_model][vocab] int8 + one bf16 scale per vocabulary entry (the format
 * of Section 3.6), and the next input = row `token` of an embedding table
 * [vocab][d_model] bf16.
 *
 * Sampling of one row (fp32): order the vocabulary by logit, largest first, equal
 * logits by smaller index; keep the first top_k (1..64); p = softmax(logit /
 * temperature) over them; keep the shortest prefix whose mass reaches top_p; with
 * c_i the running sums over that prefix and c_n its total, the token is the first
 * entry with c_i > u * c_n (u in [0,1) supplied by the caller: the library draws
 * no random numbers).  Logits must be finite.
 */

/* Bytes of the packed head (vocab % 32 == 0, d_model * vocab < 4 GiB). */
pd_status pd_packed_head_bytes(const pd_model_desc* desc, int32_t vocab, size_t* bytes);
/* Scratch of pd_head_logits() for batch B. */
pd_status pd_head_workspace_bytes(const pd_model_desc* desc, int32_t vocab, int32_t B, size_t* bytes);
/* Scratch of pd_generate() for batch B and cache capacity L_ctx (includes the
 * decode step's and the head's). */
pd_status pd_generate_workspace_bytes(const pd_model_desc* desc, int32_t vocab, int32_t B, int32_t L_ctx,
                                      size_t* bytes);
/* Canonical device tensors -> packed head: w_vocab [d_model][vocab] int8 row-major,
 * s_vocab [vocab] bf16, gamma_f [d_model] bf16. */
pd_status pd_pack_head(pd_handle* h, const int8_t* w_vocab, const uint16_t* s_vocab,
                       const uint16_t* gamma_f, int32_t vocab, void* packed_head, void* stream);
/* logits [B][vocab] fp32 (device) = LN_f(x) . deq(W_vocab) for x [B][d_model] bf16. */
pd_status pd_head_logits(pd_handle* h, const void* packed_head, int32_t vocab, const uint16_t* x,
                         int32_t B, float* logits, void* workspace, size_t workspace_bytes,
                         void* stream);
/* tokens[b] (device int32) = the draw defined above from logits [B][vocab] fp32
 * with uniforms[b] (device fp32 in [0,1)).  Bit-reproducible. */
pd_status pd_sample(const float* logits, int32_t B, int32_t vocab, int32_t top_k, float top_p,
                    float temperature, const float* uniforms, int32_t* tokens, void* stream);
/*
 * n_steps generation steps.  Per step i: one decode step of the stack on x at
 * positions (K/V appended as in pd_decode_step), logits, one draw per row with
 * uniforms[i][b], tokens_out[i][b] = the token, x[b] = embed[token], positions[b]
 * += 1.  Everything advances on the device; with use_graph != 0 one step is
 * captured as a HIP graph (owned by the handle) and replayed n_steps times.
 *   x              device [B][d_model] bf16, in: hidden state (embedding) of the
 *                  current token of each sequence; out: embedding of the last draw
 *   positions      device [B] int32, in/out; positions[b] + n_steps <= L_ctx is the
 *                  caller's duty (a row that runs past L_ctx is flagged as in
 *                  pd_decode_step and reported by pd_check_async(h, workspace, ..))
 *   uniforms       device [n_steps][B] fp32;  tokens_out device [n_steps][B] int32
 *   workspace      device, >= pd_generate_workspace_bytes()
 */
pd_status pd_generate(pd_handle* h, const void* packed_weights, const void* packed_head,
                      const uint16_t* embed, void* k_cache, void* v_cache, uint16_t* x,
                      int32_t* positions, int32_t B, int32_t L_ctx, int32_t vocab, int32_t n_steps,
                      int32_t top_k, float top_p, float temperature, const float* uniforms,
                      int32_t* tokens_out, int32_t use_graph, void* workspace,
                      size_t workspace_bytes, void* stream);

/* ---- graph replay ---------------------------------------------------------
 * Section 2.2: generation repeats the same step once per token; replaying a
 * captured step removes the per-kernel launch cost from that loop. */

/* Captures pd_decode_step(...) with these arguments into a HIP graph owned by
 * the handle; pd_graph_replay() launches it.  Valid while every pointer, B and
 * L_ctx stay the same; the CONTENTS of positions, x_in and the caches may change
 * between replays. */
pd_status pd_graph_capture(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                           const uint16_t* x_in, const int32_t* positions, int32_t B, int32_t L_ctx,
                           uint16_t* x_out, void* workspace, size_t workspace_bytes, void* stream);
pd_status pd_graph_replay(pd_handle* h, void* stream);
pd_status pd_graph_release(pd_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* PALMDECODE_H */
