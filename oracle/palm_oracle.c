/*
 * palm_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what one generate-phase (decode) step of
 * a PaLM-style stack computes, written from the paper's definitions:
 *
 *   - parallel block  y = x + Attn(LN(x)) + FFN(LN(x)), one LayerNorm per layer
 *     (Section 3.4);
 *   - fused input projection producing q | k | v | gate | up from LN(x), fused
 *     output projection consuming attention-out | FFN-activation (Section 3.4);
 *   - multiquery attention: n_heads query heads share one K/V head (Section 3.3);
 *   - the KV cache keeps K and V of every past token (Section 1; Section 2
 *     "Memory costs"); a decode step processes one new token per sequence
 *     (Section 2.2);
 *   - weights are int8 with one scale per output channel, arithmetic is not
 *     quantised (Section 3.6);
 *   - Swish gate (Section 3.5 names Swish; SwiGLU = swish(gate) * up).
 *
 * Where the paper is silent the readings are: LayerNorm subtracts the mean,
 * uses the population variance with eps added inside the square root, has a
 * gain and no bias; RoPE rotates the full head with half-split pairing
 * (i, i + d_head/2), angle = position * base^(-2i/d_head), applied to q and k;
 * softmax scale 1/sqrt(d_head); the freshly computed k and v are rounded to
 * bf16 into the cache *before* the step attends, so the step reads them back
 * like any other slot; the residual stream stays fp64 between layers.
 *
 * No blocking, fusion or reordering: every output is its defining sum taken in
 * index order.  OpenMP only spreads independent outputs over cores.
 *
 * Nothing here is shared with the HIP library; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  Pins that check this file
 * against library routines, closed forms and brute force live in tests/.
 * Absolute values of a trained PaLM forward pass: parity unpinned (no weights).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_layers, d_model, n_heads, d_head, d_ff, n_kv_heads;
    double rope_base, ln_eps;
} orc_desc;

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- bf16 --- */

double orc_bf16_to_f64(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* fp64 -> bf16, round to nearest even in ONE rounding (never through fp32). */
uint16_t orc_f64_to_bf16(double v) {
    if (isnan(v)) return 0x7fc0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isinf(a)) return sign | 0x7f80;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = m * 2^e, m in [0.5, 1)  ->  floor(log2 a) = e - 1 */
    int ex = e - 1;
    if (ex < -126) ex = -126;          /* subnormal range shares one quantum */
    double quantum = ldexp(1.0, ex - 7); /* bf16 keeps 8 significant bits */
    double r = nearbyint(a / quantum) * quantum; /* default mode = ties to even */
    if (r >= ldexp(1.0, 128)) return sign | 0x7f80;
    float f = (float)r; /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

void orc_f64_to_bf16_n(const double* v, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; i++) out[i] = orc_f64_to_bf16(v[i]);
}

/* ------------------------------------------------------------ LayerNorm --- */

/* h_i = gamma_i * (x_i - mean) / sqrt(var + eps), population variance.
 * Section 3.4: one LayerNorm per layer feeds both branches. */
void orc_layernorm(const double* x, const uint16_t* gamma, int32_t d, double eps, double* h) {
    double mean = 0.0;
    for (int32_t i = 0; i < d; i++) mean += x[i];
    mean /= (double)d;
    double var = 0.0;
    for (int32_t i = 0; i < d; i++) var += (x[i] - mean) * (x[i] - mean);
    var /= (double)d;
    double rstd = 1.0 / sqrt(var + eps);
    for (int32_t i = 0; i < d; i++) h[i] = orc_bf16_to_f64(gamma[i]) * (x[i] - mean) * rstd;
}

/* ------------------------------------------------- int8-weight projection --- */

/* out[r][n] = scale[n] * sum_k a[r][k] * q8[k][n]      (Section 3.6: int8
 * weight, one scale per output channel n; dequantised weight = q8 * scale).
 * a: [R][K] fp64, q8: [K][N] row-major int8, scale: [N] bf16 bits. */
void orc_qmatmul(const double* a, const int8_t* q8, const uint16_t* scale,
                 int32_t R, int32_t K, int32_t N, double* out) {
    const int32_t NB = 512;
    int32_t nblocks = (N + NB - 1) / NB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t nb = 0; nb < nblocks; nb++) {
        int32_t n0 = nb * NB, n1 = n0 + NB < N ? n0 + NB : N;
        for (int32_t r = 0; r < R; r++) {
            double acc[512];
            for (int32_t n = n0; n < n1; n++) acc[n - n0] = 0.0;
            for (int32_t k = 0; k < K; k++) { /* k ascending for every output */
                double ak = a[(size_t)r * K + k];
                const int8_t* wrow = q8 + (size_t)k * N;
                for (int32_t n = n0; n < n1; n++) acc[n - n0] += ak * (double)wrow[n];
            }
            for (int32_t n = n0; n < n1; n++)
                out[(size_t)r * N + n] = orc_bf16_to_f64(scale[n]) * acc[n - n0];
        }
    }
}

/* out[r][n] = sum_k a[r][k] * w[k][n] with the weights stored in bf16 and no
 * scales: the unquantised baseline the int8 weights are compared with
 * (Section 3.6, Section 4.4).  w: [K][N] row-major bf16 bits. */
void orc_wmatmul_bf16(const double* a, const uint16_t* w, int32_t R, int32_t K, int32_t N, double* out) {
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; n++)
        for (int32_t r = 0; r < R; r++) {
            double acc = 0.0;
            for (int32_t k = 0; k < K; k++) acc += a[(size_t)r * K + k] * orc_bf16_to_f64(w[(size_t)k * N + n]);
            out[(size_t)r * N + n] = acc;
        }
}

/* the projection of a layer in either weight format */
static void orc_project(const double* a, const void* w, const uint16_t* scale, int32_t w16,
                        int32_t R, int32_t K, int32_t N, double* out) {
    if (w16) orc_wmatmul_bf16(a, (const uint16_t*)w, R, K, N, out);
    else orc_qmatmul(a, (const int8_t*)w, scale, R, K, N, out);
}

/* ------------------------------------------------------------------ RoPE --- */

/* Rotate y[0..dh) in place by the angles pos * base^(-2i/dh), pairing element
 * i with element i + dh/2. */
void orc_rope(double* y, int32_t dh, int32_t pos, double base) {
    int32_t half = dh / 2;
    for (int32_t i = 0; i < half; i++) {
        double theta = pow(base, -2.0 * (double)i / (double)dh);
        double phi = (double)pos * theta;
        double c = cos(phi), s = sin(phi);
        double lo = y[i], hi = y[i + half];
        y[i] = lo * c - hi * s;
        y[i + half] = hi * c + lo * s;
    }
}

/* ------------------------------------------------------------- attention --- */

/* Multiquery attention for one sequence (Section 3.3): every one of the H
 * query heads attends over the SAME K and V rows, slots 0..T-1.
 * q: [H][dh] fp64; K, V: [T][dh] bf16 bits; out: [H][dh];
 * probs (may be NULL): [H][T] softmax weights. */
void orc_attend_mqa(const double* q, const uint16_t* K, const uint16_t* V,
                    int32_t H, int32_t dh, int32_t T, double* out, double* probs) {
    double inv = 1.0 / sqrt((double)dh);
    double* s = (double*)malloc((size_t)T * sizeof(double));
    for (int32_t j = 0; j < H; j++) {
        const double* qj = q + (size_t)j * dh;
        double m = -INFINITY;
        for (int32_t t = 0; t < T; t++) {
            double dot = 0.0;
            for (int32_t c = 0; c < dh; c++) dot += qj[c] * orc_bf16_to_f64(K[(size_t)t * dh + c]);
            s[t] = dot * inv;
            if (s[t] > m) m = s[t];
        }
        double z = 0.0;
        for (int32_t t = 0; t < T; t++) { s[t] = exp(s[t] - m); z += s[t]; }
        for (int32_t t = 0; t < T; t++) s[t] /= z;
        if (probs) memcpy(probs + (size_t)j * T, s, (size_t)T * sizeof(double));
        for (int32_t c = 0; c < dh; c++) {
            double o = 0.0;
            for (int32_t t = 0; t < T; t++) o += s[t] * orc_bf16_to_f64(V[(size_t)t * dh + c]);
            out[(size_t)j * dh + c] = o;
        }
    }
    free(s);
}

/* Multihead attention, every head with its OWN K and V: K, V are
 * [H][T][dh].  Written separately from the multiquery routine (scores held as
 * a full [T] row per head, V accumulated token by token) so that "multiquery ==
 * multihead with the K/V head copied H times" is a test of two codes. */
void orc_attend_mha(const double* q, const uint16_t* K, const uint16_t* V,
                    int32_t H, int32_t dh, int32_t T, double* out) {
    for (int32_t j = 0; j < H; j++) {
        const uint16_t* Kj = K + (size_t)j * T * dh;
        const uint16_t* Vj = V + (size_t)j * T * dh;
        double* logits = (double*)malloc((size_t)T * sizeof(double));
        double big = -INFINITY;
        for (int32_t t = 0; t < T; t++) {
            double acc = 0.0;
            for (int32_t c = 0; c < dh; c++)
                acc += q[(size_t)j * dh + c] * orc_bf16_to_f64(Kj[(size_t)t * dh + c]);
            logits[t] = acc / sqrt((double)dh);
            big = logits[t] > big ? logits[t] : big;
        }
        double denom = 0.0;
        for (int32_t t = 0; t < T; t++) denom += exp(logits[t] - big);
        for (int32_t c = 0; c < dh; c++) out[(size_t)j * dh + c] = 0.0;
        for (int32_t t = 0; t < T; t++) {
            double p = exp(logits[t] - big) / denom;
            for (int32_t c = 0; c < dh; c++)
                out[(size_t)j * dh + c] += p * orc_bf16_to_f64(Vj[(size_t)t * dh + c]);
        }
        free(logits);
    }
}

/* ---------------------------------------------------------------- SwiGLU --- */

/* a_f = swish(g_f) * u_f, swish(z) = z * sigmoid(z) = z / (1 + exp(-z)). */
void orc_swiglu(const double* g, const double* u, int32_t F, double* a) {
    for (int32_t f = 0; f < F; f++) a[f] = g[f] / (1.0 + exp(-g[f])) * u[f];
}

/* ------------------------------------------------------- one decode layer --- */

/*
 * One layer of one decode step for R independent sequences (rows never
 * interact in decode, Section 2.2).
 *
 * w_in  [d][n_in] int8, columns q(H*dh) | k(dh) | v(dh) | gate(F) | up(F)
 * s_in  [n_in] bf16 bits;  w_out [H*dh + F][d] int8, rows attn | ffn;  s_out [d]
 * gamma [d] bf16 bits
 * kc, vc: this layer's cache, [rows][n_kv_heads][L_ctx][dh] bf16 bits; row r uses
 *         cache row cache_row[r]; slot positions[r] of every K/V head is WRITTEN,
 *         slots 0..positions[r] are read, nothing else is touched.
 * x:   [R][d] fp64, in/out.  add_residual = 0 stores only the block's
 *      contribution (a shard's unreduced partial) instead of x + contribution.
 * Returns 0, or -1 on a bad argument.
 */
static int orc_decode_layer_impl(const orc_desc* m, int32_t w16, const void* w_in, const uint16_t* s_in,
                                 const void* w_out, const uint16_t* s_out, const uint16_t* gamma,
                                 uint16_t* kc, uint16_t* vc, const int32_t* cache_row,
                                 const int32_t* positions, int32_t R, int32_t L_ctx,
                                 double* x, int32_t add_residual) {
    int32_t d = m->d_model, H = m->n_heads, dh = m->d_head, F = m->d_ff;
    /* K/V heads: 1 = multiquery (Section 3.3), H = multihead (every query head has its
     * own K/V head).  With G heads the columns of w_in are q(H*dh) | k(G*dh) | v(G*dh) |
     * gate | up and a cache row is [G][L_ctx][dh]. */
    int32_t G = m->n_kv_heads;
    if ((G != 1 && G != H) || R < 1 || L_ctx < 1 || (dh & 1)) return -1;
    for (int32_t r = 0; r < R; r++)
        if (positions[r] < 0 || positions[r] >= L_ctx) return -1;
    int32_t n_in = H * dh + 2 * G * dh + 2 * F, k_out = H * dh + F;

    double* h = (double*)malloc((size_t)R * d * sizeof(double));
    double* z = (double*)malloc((size_t)R * n_in * sizeof(double));
    double* oa = (double*)malloc((size_t)R * k_out * sizeof(double));
    double* y = (double*)malloc((size_t)R * d * sizeof(double));
    if (!h || !z || !oa || !y) { free(h); free(z); free(oa); free(y); return -1; }

    for (int32_t r = 0; r < R; r++)
        orc_layernorm(x + (size_t)r * d, gamma, d, m->ln_eps, h + (size_t)r * d);

    orc_project(h, w_in, s_in, w16, R, d, n_in, z);

    for (int32_t r = 0; r < R; r++) {
        double* zr = z + (size_t)r * n_in;
        double* q = zr;
        double* k = zr + (size_t)H * dh;
        double* v = k + (size_t)G * dh;
        double* g = v + (size_t)G * dh;
        double* u = g + F;
        int32_t p = positions[r];
        for (int32_t j = 0; j < H; j++) orc_rope(q + (size_t)j * dh, dh, p, m->rope_base);
        double* oar = oa + (size_t)r * k_out;
        for (int32_t j = 0; j < G; j++) {
            orc_rope(k + (size_t)j * dh, dh, p, m->rope_base);
            uint16_t* Kr = kc + ((size_t)cache_row[r] * G + j) * L_ctx * dh;
            uint16_t* Vr = vc + ((size_t)cache_row[r] * G + j) * L_ctx * dh;
            for (int32_t c = 0; c < dh; c++) {
                Kr[(size_t)p * dh + c] = orc_f64_to_bf16(k[(size_t)j * dh + c]);
                Vr[(size_t)p * dh + c] = orc_f64_to_bf16(v[(size_t)j * dh + c]);
            }
            /* the query heads that share K/V head j: all H of them (multiquery) or head j alone */
            int32_t per = H / G;
            orc_attend_mqa(q + (size_t)j * per * dh, Kr, Vr, per, dh, p + 1, oar + (size_t)j * per * dh, NULL);
        }
        orc_swiglu(g, u, F, oar + (size_t)H * dh);
    }

    orc_project(oa, w_out, s_out, w16, R, k_out, d, y);

    for (size_t i = 0; i < (size_t)R * d; i++) x[i] = add_residual ? x[i] + y[i] : y[i];

    free(h); free(z); free(oa); free(y);
    return 0;
}

int orc_decode_layer(const orc_desc* m, const int8_t* w_in, const uint16_t* s_in,
                     const int8_t* w_out, const uint16_t* s_out, const uint16_t* gamma,
                     uint16_t* kc, uint16_t* vc, const int32_t* cache_row,
                     const int32_t* positions, int32_t R, int32_t L_ctx,
                     double* x, int32_t add_residual) {
    return orc_decode_layer_impl(m, 0, w_in, s_in, w_out, s_out, gamma, kc, vc, cache_row, positions, R,
                                 L_ctx, x, add_residual);
}

/* The same layer with both matrices stored in bf16, no scales (the bf16-weight
 * baseline of Section 4.4). */
int orc_decode_layer_w16(const orc_desc* m, const uint16_t* w_in, const uint16_t* w_out,
                         const uint16_t* gamma, uint16_t* kc, uint16_t* vc, const int32_t* cache_row,
                         const int32_t* positions, int32_t R, int32_t L_ctx, double* x,
                         int32_t add_residual) {
    return orc_decode_layer_impl(m, 1, w_in, NULL, w_out, NULL, gamma, kc, vc, cache_row, positions, R,
                                 L_ctx, x, add_residual);
}

/* --------------------------------------------------- sampling head (f1) --- */

/*
 * The tail of a generation step (Section 2.2: after the forward pass one new
 * token is sampled for each sequence): final LayerNorm of the hidden state,
 * logits = LN(x) . deq(W_vocab) with the same weight-only int8 format as the
 * other matrices (Section 3.6).  The paper gives no formula for this tail (the
 * model is PaLM's by citation); the reading is: the same LayerNorm as in the
 * blocks with its own gain, no bias, a [d][V] int8 matrix with one bf16 scale
 * per vocabulary entry.
 * x: [R][d] fp64 hidden state, logits: [R][V] fp64.
 */
void orc_head_logits(const double* x, const uint16_t* gamma_f, const int8_t* w_vocab,
                     const uint16_t* s_vocab, int32_t R, int32_t d, int32_t V, double eps,
                     double* logits) {
    double* h = (double*)malloc((size_t)R * d * sizeof(double));
    for (int32_t r = 0; r < R; r++) orc_layernorm(x + (size_t)r * d, gamma_f, d, eps, h + (size_t)r * d);
    orc_qmatmul(h, w_vocab, s_vocab, R, d, V, logits);
    free(h);
}

/*
 * Top-k / top-p (nucleus) sampling of ONE token from `logits` [V] (Section 3.5
 * names top-k/top-p decode sampling; the definition written out here is the usual
 * one):
 *   1. order the vocabulary by logit, largest first, equal logits by smaller index;
 *   2. keep the first k entries;
 *   3. p_i = softmax(logit_i / temperature) over the kept entries;
 *   4. keep the shortest prefix whose probabilities sum to at least top_p (at least
 *      one entry);
 *   5. with c_i the running sums over that prefix and c_n its total, return the first
 *      entry with c_i > u * c_n, u in [0, 1) supplied by the caller (the last entry
 *      if rounding leaves none).
 * The random number is an input: the method's random draws do not live here.
 * Plain selection sort of the first k entries: O(k V), obviously correct.
 * Outputs: *token; optionally kept[0] = entries that survived step 4 and
 * margin[0] = distance of u * c_n from the nearest boundary of the chosen entry's
 * interval, relative to c_n (how well-conditioned the draw is).
 * Returns 0, or -1 on a bad argument.
 */
int orc_sample_topk_topp(const double* logits, int32_t V, int32_t k, double top_p,
                         double temperature, double u, int32_t* token, int32_t* kept,
                         double* margin) {
    if (V < 1 || k < 1 || k > V || !(top_p > 0.0) || top_p > 1.0 || !(temperature > 0.0) ||
        !(u >= 0.0) || !(u < 1.0))
        return -1;
    int32_t* idx = (int32_t*)malloc((size_t)k * sizeof(int32_t));
    double* pr = (double*)malloc((size_t)k * sizeof(double));
    char* taken = (char*)calloc((size_t)V, 1);
    for (int32_t i = 0; i < k; i++) { /* i-th largest, ties by smaller index */
        int32_t best = -1;
        for (int32_t v = 0; v < V; v++) {
            if (taken[v]) continue;
            if (best < 0 || logits[v] > logits[best]) best = v;
        }
        taken[best] = 1;
        idx[i] = best;
    }
    double m = logits[idx[0]] / temperature, z = 0.0;
    for (int32_t i = 0; i < k; i++) { pr[i] = exp(logits[idx[i]] / temperature - m); z += pr[i]; }
    for (int32_t i = 0; i < k; i++) pr[i] /= z;
    int32_t n = 0;
    double c = 0.0;
    while (n < k) { c += pr[n]; n++; if (c >= top_p) break; }
    double target = u * c, run = 0.0, lo = 0.0;
    int32_t pick = n - 1;
    for (int32_t i = 0; i < n; i++) {
        lo = run;
        run += pr[i];
        if (run > target) { pick = i; break; }
    }
    *token = idx[pick];
    if (kept) *kept = n;
    if (margin) {
        double a = target - lo, b = run - target;
        *margin = (a < b ? a : b) / c;
    }
    free(idx); free(pr); free(taken);
    return 0;
}

/* --------------------------------------------- full causal forward (pins) --- */

/*
 * The same layer applied to T tokens of ONE sequence at once, the way the
 * prefill phase runs it (Section 2.2): all projections as [T x .] products,
 * keys/values of all T tokens formed first, then a [T x T] score matrix with
 * the causal mask.  Deliberately does not go through the cache-based routine
 * above: "decode step t == row t of this" is a brute-force pin on the cache
 * indexing, the rotation position and the append-before-attend order.
 * Token t sits at position t.  x: [T][d] in/out.
 */
int orc_causal_layer(const orc_desc* m, const int8_t* w_in, const uint16_t* s_in,
                     const int8_t* w_out, const uint16_t* s_out, const uint16_t* gamma,
                     int32_t T, double* x) {
    int32_t d = m->d_model, H = m->n_heads, dh = m->d_head, F = m->d_ff;
    if (m->n_kv_heads != 1 || T < 1) return -1;
    int32_t n_in = H * dh + 2 * dh + 2 * F, k_out = H * dh + F;
    double* h = (double*)malloc((size_t)T * d * sizeof(double));
    double* z = (double*)malloc((size_t)T * n_in * sizeof(double));
    double* Kb = (double*)malloc((size_t)T * dh * sizeof(double));
    double* Vb = (double*)malloc((size_t)T * dh * sizeof(double));
    double* S = (double*)malloc((size_t)T * T * sizeof(double));
    double* oa = (double*)calloc((size_t)T * k_out, sizeof(double));
    double* y = (double*)malloc((size_t)T * d * sizeof(double));

    for (int32_t t = 0; t < T; t++)
        orc_layernorm(x + (size_t)t * d, gamma, d, m->ln_eps, h + (size_t)t * d);
    orc_qmatmul(h, w_in, s_in, T, d, n_in, z);

    for (int32_t t = 0; t < T; t++) { /* keys/values of every token, as cached */
        double* zt = z + (size_t)t * n_in;
        for (int32_t j = 0; j < H; j++) orc_rope(zt + (size_t)j * dh, dh, t, m->rope_base);
        double* k = zt + (size_t)H * dh;
        double* v = k + dh;
        orc_rope(k, dh, t, m->rope_base);
        for (int32_t c = 0; c < dh; c++) {
            Kb[(size_t)t * dh + c] = orc_bf16_to_f64(orc_f64_to_bf16(k[c]));
            Vb[(size_t)t * dh + c] = orc_bf16_to_f64(orc_f64_to_bf16(v[c]));
        }
    }
    for (int32_t j = 0; j < H; j++) {
        for (int32_t t = 0; t < T; t++)
            for (int32_t u = 0; u < T; u++) {
                double dot = 0.0;
                for (int32_t c = 0; c < dh; c++)
                    dot += z[(size_t)t * n_in + (size_t)j * dh + c] * Kb[(size_t)u * dh + c];
                S[(size_t)t * T + u] = (u <= t) ? dot / sqrt((double)dh) : -INFINITY;
            }
        for (int32_t t = 0; t < T; t++) {
            double mx = -INFINITY, den = 0.0;
            for (int32_t u = 0; u < T; u++) if (S[(size_t)t * T + u] > mx) mx = S[(size_t)t * T + u];
            for (int32_t u = 0; u < T; u++) { S[(size_t)t * T + u] = exp(S[(size_t)t * T + u] - mx); den += S[(size_t)t * T + u]; }
            for (int32_t u = 0; u < T; u++) S[(size_t)t * T + u] /= den;
            for (int32_t c = 0; c < dh; c++) {
                double o = 0.0;
                for (int32_t u = 0; u < T; u++) o += S[(size_t)t * T + u] * Vb[(size_t)u * dh + c];
                oa[(size_t)t * k_out + (size_t)j * dh + c] = o;
            }
        }
    }
    for (int32_t t = 0; t < T; t++) {
        double* g = z + (size_t)t * n_in + (size_t)H * dh + 2 * dh;
        orc_swiglu(g, g + F, F, oa + (size_t)t * k_out + (size_t)H * dh);
    }
    orc_qmatmul(oa, w_out, s_out, T, k_out, d, y);
    for (size_t i = 0; i < (size_t)T * d; i++) x[i] += y[i];
    free(h); free(z); free(Kb); free(Vb); free(S); free(oa); free(y);
    return 0;
}
