/* Runs every routine of the fp64 oracle once on small inputs held in heap blocks of
 * exactly the documented sizes, for a build with AddressSanitizer and
 * UndefinedBehaviorSanitizer: a read or write outside any tensor, a signed overflow or
 * a bad shift in the oracle ends the program with a report.  Test infrastructure. */
#include "../../oracle/palm_oracle.c"

#include <stdio.h>

static uint64_t state = 0x2211051020221105ull;
static double uniform01(void) { /* 53-bit LCG output in [0, 1) */
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}
static double* doubles(size_t n, double scale) {
    double* p = (double*)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; i++) p[i] = (uniform01() * 2.0 - 1.0) * scale;
    return p;
}
static uint16_t* bf16s(size_t n, double scale, double offset) {
    uint16_t* p = (uint16_t*)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; i++) p[i] = orc_f64_to_bf16(offset + (uniform01() * 2.0 - 1.0) * scale);
    return p;
}
static int8_t* int8s(size_t n) {
    int8_t* p = (int8_t*)malloc(n);
    for (size_t i = 0; i < n; i++) p[i] = (int8_t)((int)(uniform01() * 255.0) - 127);
    return p;
}
static int finite_all(const double* v, size_t n) {
    for (size_t i = 0; i < n; i++)
        if (!(v[i] == v[i]) || v[i] > 1e300 || v[i] < -1e300) return 0;
    return 1;
}

static int run_layer(int G, int w16) {
    orc_desc m = {1, 64, 4, 16, 32, G, 10000.0, 1e-6};
    const int R = 3, L_ctx = 8, rows = 4;
    const size_t n_in = (size_t)m.n_heads * m.d_head + 2 * (size_t)G * m.d_head + 2 * (size_t)m.d_ff;
    const size_t k_out = (size_t)m.n_heads * m.d_head + m.d_ff;
    void* w_in = w16 ? (void*)bf16s(m.d_model * n_in, 0.02, 0.0) : (void*)int8s(m.d_model * n_in);
    void* w_out = w16 ? (void*)bf16s(k_out * m.d_model, 0.02, 0.0) : (void*)int8s(k_out * m.d_model);
    uint16_t* s_in = bf16s(n_in, 1e-4, 2e-4);
    uint16_t* s_out = bf16s(m.d_model, 1e-4, 2e-4);
    uint16_t* gamma = bf16s(m.d_model, 0.02, 1.0);
#ifdef PLANT_SHORT_CACHE /* the check of the checker: one element too few must be reported */
    const size_t cache = (size_t)rows * G * L_ctx * m.d_head - 1;
#else
    const size_t cache = (size_t)rows * G * L_ctx * m.d_head;
#endif
    uint16_t* kc = bf16s(cache, 1.0, 0.0);
    uint16_t* vc = bf16s(cache, 1.0, 0.0);
    int32_t cache_row[3] = {3, 0, 2};
    int32_t positions[3] = {7, 0, 4}; /* last slot (of the last cache row), first slot, one in between */
    double* x = doubles((size_t)R * m.d_model, 1.0);
    int rc;
    if (w16)
        rc = orc_decode_layer_w16(&m, (const uint16_t*)w_in, (const uint16_t*)w_out, gamma, kc, vc, cache_row,
                                  positions, R, L_ctx, x, 1);
    else
        rc = orc_decode_layer(&m, (const int8_t*)w_in, s_in, (const int8_t*)w_out, s_out, gamma, kc, vc,
                              cache_row, positions, R, L_ctx, x, 1);
    int ok = rc == 0 && finite_all(x, (size_t)R * m.d_model);
    free(w_in); free(w_out); free(s_in); free(s_out); free(gamma); free(kc); free(vc); free(x);
    return ok;
}

int main(void) {
    int ok = 1;
    ok &= run_layer(1, 0);
    ok &= run_layer(4, 0);
    ok &= run_layer(1, 1);
    ok &= run_layer(4, 1);
    { /* prefill-shaped layer */
        orc_desc m = {1, 64, 4, 16, 32, 1, 10000.0, 1e-6};
        const int T = 5;
        const size_t n_in = 64 + 32 + 64, k_out = 64 + 32;
        int8_t* w_in = int8s(m.d_model * n_in);
        int8_t* w_out = int8s(k_out * m.d_model);
        uint16_t* s_in = bf16s(n_in, 1e-4, 2e-4);
        uint16_t* s_out = bf16s(m.d_model, 1e-4, 2e-4);
        uint16_t* gamma = bf16s(m.d_model, 0.02, 1.0);
        double* x = doubles((size_t)T * m.d_model, 1.0);
        ok &= orc_causal_layer(&m, w_in, s_in, w_out, s_out, gamma, T, x) == 0;
        ok &= finite_all(x, (size_t)T * m.d_model);
        free(w_in); free(w_out); free(s_in); free(s_out); free(gamma); free(x);
    }
    { /* sampling head and sampler */
        const int R = 2, d = 64, V = 37;
        double* x = doubles((size_t)R * d, 1.0);
        uint16_t* gamma = bf16s(d, 0.02, 1.0);
        int8_t* w = int8s((size_t)d * V);
        uint16_t* s = bf16s(V, 1e-4, 2e-4);
        double* logits = (double*)malloc((size_t)R * V * sizeof(double));
        orc_head_logits(x, gamma, w, s, R, d, V, 1e-6, logits);
        ok &= finite_all(logits, (size_t)R * V);
        int32_t token = -1, kept = -1;
        double margin = -1.0;
        ok &= orc_sample_topk_topp(logits, V, V, 1.0, 1.0, 0.999999, &token, &kept, &margin) == 0;
        ok &= token >= 0 && token < V && kept >= 1 && kept <= V;
        ok &= orc_sample_topk_topp(logits + V, V, 1, 0.5, 0.7, 0.0, &token, NULL, NULL) == 0;
        ok &= token >= 0 && token < V;
        ok &= orc_sample_topk_topp(logits, V, V + 1, 1.0, 1.0, 0.5, &token, NULL, NULL) == -1;
        free(x); free(gamma); free(w); free(s); free(logits);
    }
    { /* the two attention routines and the small pieces */
        const int H = 3, dh = 8, T = 6;
        double* q = doubles((size_t)H * dh, 1.0);
        uint16_t* K1 = bf16s((size_t)T * dh, 1.0, 0.0);
        uint16_t* V1 = bf16s((size_t)T * dh, 1.0, 0.0);
        uint16_t* KH = bf16s((size_t)H * T * dh, 1.0, 0.0);
        uint16_t* VH = bf16s((size_t)H * T * dh, 1.0, 0.0);
        double* out = (double*)malloc((size_t)H * dh * sizeof(double));
        double* probs = (double*)malloc((size_t)H * T * sizeof(double));
        orc_attend_mqa(q, K1, V1, H, dh, T, out, probs);
        ok &= finite_all(out, (size_t)H * dh) && finite_all(probs, (size_t)H * T);
        orc_attend_mha(q, KH, VH, H, dh, T, out);
        ok &= finite_all(out, (size_t)H * dh);
        orc_rope(q, dh, 1000000, 10000.0);
        double* a = (double*)malloc((size_t)H * dh * sizeof(double));
        orc_swiglu(q, q, H * dh, a);
        ok &= finite_all(a, (size_t)H * dh);
        uint16_t* r = (uint16_t*)malloc((size_t)H * dh * sizeof(uint16_t));
        double edge[4] = {1e39, -1e39, 1e-45, 0.0}; /* beyond bf16's range, below its smallest subnormal */
        orc_f64_to_bf16_n(q, r, (int64_t)H * dh);
        orc_f64_to_bf16_n(edge, r, 4);
        free(q); free(K1); free(V1); free(KH); free(VH); free(out); free(probs); free(a); free(r);
    }
    printf(ok ? "ok\n" : "FAILED\n");
    return ok ? 0 : 1;
}
