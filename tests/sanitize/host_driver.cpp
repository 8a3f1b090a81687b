// Drives the host-only entry points of the library (sizes and work-split plans: no
// device is touched) over a sweep of shapes, for a build whose host code carries
// AddressSanitizer and UndefinedBehaviorSanitizer.  Output arrays are heap blocks of
// exactly the sizes the header documents, so an overrun in the plan code is reported.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "palmdecode.h"

static int failures = 0;
#define EXPECT(cond)                                                   \
    do {                                                               \
        if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); failures++; } \
    } while (0)

static void plan_case(int B, int K, int N, int wg, int c_split, int blk0, int blk1) {
    int32_t counts[5] = {0, 0, 0, 0, 0};
    pd_status rc = pd_qgemm_plan(B, K, N, wg, c_split, blk0, blk1, counts, nullptr, nullptr, nullptr);
    EXPECT(rc == PD_OK);
    if (rc != PD_OK) return;
    const int G = counts[0], T = counts[1], C = counts[2];
    int64_t* begin = static_cast<int64_t*>(std::malloc(sizeof(int64_t) * (G + 1)));
    int32_t* first = static_cast<int32_t*>(std::malloc(sizeof(int32_t) * G));
    int32_t* slots = static_cast<int32_t*>(std::malloc(sizeof(int32_t) * T));
    EXPECT(pd_qgemm_plan(B, K, N, wg, c_split, blk0, blk1, counts, begin, first, slots) == PD_OK);
    EXPECT(begin[0] == 0 && begin[G] == (int64_t)T * C);
    int most = 0;
    for (int g = 0; g < G; g++) EXPECT(begin[g] <= begin[g + 1] && first[g] >= 0);
    for (int t = 0; t < T; t++) { EXPECT(slots[t] >= 1); most = slots[t] > most ? slots[t] : most; }
    EXPECT(most == counts[4]);
    size_t bytes = 0;
    EXPECT(pd_qgemm_workspace_bytes(B, K, N, wg, &bytes) == PD_OK && bytes > 0);
    std::free(begin); std::free(first); std::free(slots);
}

int main() {
    const int batches[] = {1, 8, 32, 33, 64, 65, 130, 256};
    for (int B : batches) {
        plan_case(B, 128, 32, 0, 0, 1, 1);
        plan_case(B, 8192, 81920, 0, 0, 1, 64);
        plan_case(B, 40960, 8192, 0, 64, 16, 16);
        plan_case(B, 1280, 2432, 7, 3, 2, 4);
        plan_case(B, 4096, 544, 4096, 0, 1, 1);
        plan_case(B, 18432, 20480, 255, 0, 1, 144);
    }
    int32_t counts[5];
    EXPECT(pd_qgemm_plan(0, 128, 32, 0, 0, 1, 1, counts, nullptr, nullptr, nullptr) == PD_ERR_SHAPE);
    EXPECT(pd_qgemm_plan(1, 100, 32, 0, 0, 1, 1, counts, nullptr, nullptr, nullptr) == PD_ERR_SHAPE);
    EXPECT(pd_qgemm_plan(1, 128, 32, 5000, 0, 1, 1, counts, nullptr, nullptr, nullptr) == PD_ERR_RANGE);
    EXPECT(pd_qgemm_plan(1, 128, 32, 0, 0, 1, 1, nullptr, nullptr, nullptr, nullptr) == PD_ERR_NULL);

    struct Model { int L, d, H, dh, F, G, flags; };
    const Model models[] = {
        {1, 256, 4, 64, 1024, 1, 0},        {32, 4096, 16, 256, 16384, 1, 0},
        {64, 8192, 32, 256, 32768, 1, 0},   {118, 18432, 6, 256, 9216, 1, 0},
        {64, 8192, 64, 128, 32768, 64, 0},  {64, 8192, 32, 256, 32768, 1, PD_FLAG_BF16_WEIGHTS},
        {2, 128, 256, 64, 128, 8, 0},       {1, 1048576, 2, 64, 128, 1, 0},
    };
    for (const Model& m : models) {
        pd_model_desc d = {m.L, m.d, m.H, m.dh, m.F, m.G, 10000.0f, 1e-6f, m.flags};
        size_t bytes = 0;
        EXPECT(pd_packed_layer_bytes(&d, &bytes) == PD_OK && bytes % 256 == 0);
        for (int B : batches)
            for (int L_ctx : {32, 2048, 8192}) {
                size_t kv = 0, ws = 0, gen = 0, head = 0;
                EXPECT(pd_kv_cache_bytes(&d, B, L_ctx, &kv) == PD_OK);
                EXPECT(kv == (size_t)m.L * B * m.G * L_ctx * m.dh * 2);
                EXPECT(pd_workspace_bytes(&d, B, L_ctx, &ws) == PD_OK && ws % 256 == 0);
                if (m.d <= 32768) {
                    EXPECT(pd_head_workspace_bytes(&d, 32000, B, &head) == PD_OK && head > 0);
                    EXPECT(pd_generate_workspace_bytes(&d, 32000, B, L_ctx, &gen) == PD_OK && gen >= ws);
                }
            }
        EXPECT(pd_packed_head_bytes(&d, 32, &bytes) == PD_OK);
        EXPECT(pd_packed_head_bytes(&d, 31, &bytes) != PD_OK);
    }
    const pd_model_desc bad[] = {
        {1, 200, 4, 64, 1024, 1, 10000.0f, 1e-6f, 0},   {1, 256, 4, 96, 1024, 1, 10000.0f, 1e-6f, 0},
        {1, 256, 4, 64, 1024, 3, 10000.0f, 1e-6f, 0},   {0, 256, 4, 64, 1024, 1, 10000.0f, 1e-6f, 0},
        {1, 256, 4, 64, 1024, 1, 10000.0f, 1e-6f, 2},   {1, 256, 257, 64, 1024, 1, 10000.0f, 1e-6f, 0},
        {1, 1048576, 256, 256, 16777216, 1, 10000.0f, 1e-6f, 0},  // products that overflow 32 bits
        {1, 256, 4, 64, 1024, 1, 1.0f, 1e-6f, 0},       {1, 256, 4, 64, 1024, 1, 10000.0f, 0.0f, 0},
    };
    for (const pd_model_desc& d : bad) {
        size_t bytes = 0;
        EXPECT(pd_packed_layer_bytes(&d, &bytes) == PD_ERR_SHAPE);
        EXPECT(pd_workspace_bytes(&d, 8, 64, &bytes) == PD_ERR_SHAPE);
    }
    pd_model_desc ok = {1, 256, 4, 64, 1024, 1, 10000.0f, 1e-6f, 0};
    size_t bytes = 0;
    EXPECT(pd_kv_cache_bytes(&ok, 0, 64, &bytes) == PD_ERR_SHAPE);
    EXPECT(pd_kv_cache_bytes(&ok, 257, 64, &bytes) == PD_ERR_SHAPE);
    EXPECT(pd_kv_cache_bytes(&ok, 1, 100, &bytes) == PD_ERR_SHAPE);
    EXPECT(pd_kv_cache_bytes(&ok, 1, 64, nullptr) == PD_ERR_NULL);
    EXPECT(pd_packed_layer_bytes(nullptr, &bytes) == PD_ERR_NULL);
    EXPECT(pd_status_string(PD_ERR_SHAPE) != nullptr && pd_last_error() != nullptr);
    std::printf(failures ? "FAILED (%d)\n" : "ok\n", failures);
    return failures ? 1 : 0;
}
