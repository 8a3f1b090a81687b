// C ABI of the decode library: argument validation, workspace carving, the
// layer-stack driver (paper Section 2.2: one forward pass over B x 1 tokens that
// streams every weight and every live cache slot once) and graph capture.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/palmdecode.h"
#include "kernels.h"

// Scratch memory of pd_decode_step_static(): one copy per GPU the library runs on, held
// until the process ends.  In host code this name is only a stand-in for the symbol; the
// device address comes from hipGetSymbolAddress (static_scratch() below) and that
// pointer is what kernels and copies get.
#define PD_STATIC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[PD_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

pd_status fail(pd_status code, const char* msg) {
    snprintf(g_err, sizeof(g_err), "%s", msg);
    return code;
}
pd_status fail_hip(hipError_t e, const char* where) {
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
    return PD_ERR_HIP;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct Shape {
    int L, d, H, G, dh, F, n_qkv, n_in, k_out;  // G = K/V heads
    int w16;                                    // 1: the projection matrices are bf16, no scales
};

pd_status check_desc(const pd_model_desc* m, Shape* s) {
    if (!m) return fail(PD_ERR_NULL, "desc is NULL");
    if (m->n_layers < 1 || m->d_model < 128 || m->d_model % 128) return fail(PD_ERR_SHAPE, "d_model must be a positive multiple of 128, n_layers >= 1");
    if (m->d_head != 64 && m->d_head != 128 && m->d_head != 256) return fail(PD_ERR_SHAPE, "d_head must be 64, 128 or 256");
    if (m->n_heads < 1 || m->n_heads > 256) return fail(PD_ERR_SHAPE, "n_heads must be in 1..256");
    if (m->n_kv_heads < 1 || m->n_heads % m->n_kv_heads) return fail(PD_ERR_SHAPE, "n_kv_heads must divide n_heads");
    if (m->n_heads / m->n_kv_heads > 32) return fail(PD_ERR_SHAPE, "at most 32 query heads may share one K/V head");
    if (m->d_ff < 128 || m->d_ff % 128) return fail(PD_ERR_SHAPE, "d_ff must be a positive multiple of 128");
    long long k_out = (long long)m->n_heads * m->d_head + m->d_ff;
    if ((m->n_heads * m->d_head) % 128) return fail(PD_ERR_SHAPE, "n_heads*d_head must be a multiple of 128");
    long long n_in = (long long)m->n_heads * m->d_head + 2LL * m->n_kv_heads * m->d_head + 2LL * m->d_ff;
    if (n_in > (1 << 24) || k_out > (1 << 24) || m->d_model > (1 << 20)) return fail(PD_ERR_SHAPE, "model too large");
    if (m->flags != 0 && m->flags != PD_FLAG_BF16_WEIGHTS) return fail(PD_ERR_SHAPE, "unknown flags");
    // the kernels address each matrix through a 32-bit buffer descriptor
    const long long wbytes = m->flags & PD_FLAG_BF16_WEIGHTS ? 2 : 1;
    if ((long long)m->d_model * n_in * wbytes >= (1ll << 32) || k_out * m->d_model * wbytes >= (1ll << 32))
        return fail(PD_ERR_SHAPE, "a projection matrix must be smaller than 4 GiB");
    if (!(m->rope_base > 1.0f) || !(m->ln_eps > 0.0f)) return fail(PD_ERR_SHAPE, "rope_base must exceed 1 and ln_eps must be positive");
    if (s) {
        s->L = m->n_layers; s->d = m->d_model; s->H = m->n_heads; s->G = m->n_kv_heads; s->dh = m->d_head; s->F = m->d_ff;
        s->n_qkv = m->n_heads * m->d_head + 2 * m->n_kv_heads * m->d_head;
        s->n_in = (int)n_in; s->k_out = (int)k_out;
        s->w16 = m->flags & PD_FLAG_BF16_WEIGHTS ? 1 : 0;
    }
    return PD_OK;
}

pd_status check_batch(int32_t B, int32_t L_ctx) {
    if (B < 1 || B > 256) return fail(PD_ERR_SHAPE, "B must be in 1..256");
    if (L_ctx < 32 || L_ctx % 32 || L_ctx > (1 << 20)) return fail(PD_ERR_SHAPE, "L_ctx must be a positive multiple of 32");
    return PD_OK;
}

// offsets inside one packed layer
struct PackedLayout {
    size_t w_in, w_out, s_in, s_out, gamma, gamma_absmax, total;
};
PackedLayout packed_layout(const Shape& s) {
    PackedLayout p;
    size_t o = 0;
    p.w_in = o; o += align256((size_t)s.d * s.n_in * (1 + s.w16));
    p.w_out = o; o += align256((size_t)s.k_out * s.d * (1 + s.w16));
    p.s_in = o; o += align256((size_t)s.n_in * 4);
    p.s_out = o; o += align256((size_t)s.d * 4);
    p.gamma = o; o += align256((size_t)s.d * 4);
    p.gamma_absmax = o; o += 256;  // max |gamma|, one float
    p.total = o;
    return p;
}

int auto_bps(int B, int L_ctx) {
    // one workgroup per compute unit when the batch allows: each wave then streams
    // several blocks back to back, which is what keeps its load ring full
    long long v = (long long)(L_ctx / 32) * B / 256;
    if (v < PD_MIN_BLOCKS_PER_SPLIT) v = PD_MIN_BLOCKS_PER_SPLIT;
    if (v > 64) v = 64;
    return (int)v;
}

// Launch plans of the two projections for batch B: workgroups (stream-K shares of
// the weight matrix), scale blocks of the operand, partial-sum slots per tile.
// Fixed by the shape alone -- the chip this library is written for has 256 compute
// units -- so results do not depend on where the code runs and the workspace can
// be sized on the host.
constexpr int PD_GEMM_WORKGROUPS = 256;
constexpr int PD_PREFILL_CHUNK = 256;  // token rows per pass of the stack in pd_prefill
struct GemmPlans {
    pd::SkqPlan in, out;
    int slots_in, slots_out;
    int blk_o, blk_a;  // scale blocks (in 128-element chunks) of the attention and SwiGLU outputs
};
// Automatic workgroup count of a projection.  More than 64 rows: the projection runs one
// workgroup grid per 64-row group; all groups together fill the chip once, and the
// workgroups that stream the same weight range (same x, different row group) are a
// multiple of 8 apart in launch order, i.e. on the same XCD, where all but the first find
// the weights in that XCD's L2.
int auto_workgroups(int B, int K, int N, int c_split, int blk0, int blk1, int tile_cols = 0) {
    const int row_groups = B > 32 ? (B + 63) / 64 : 1;
    int g_max = PD_GEMM_WORKGROUPS / row_groups;
    if (row_groups > 1) g_max = g_max / 8 * 8;
    return pd::qgemm_auto_workgroups(B, K, N, g_max, c_split, blk0, blk1, tile_cols);
}

GemmPlans gemm_plans(const Shape& s, int B, int g_in_opt, int g_out_opt) {
    GemmPlans p;
    // scale blocks of the projection operands (chunks that share one power-of-two
    // scale): LayerNorm output = one scale per row; attention output and SwiGLU
    // output = blocks of blk_o and blk_a chunks
    const int c_in = s.d / 128, c_attn = s.H * s.dh / 128, c_ffn = s.F / 128;
    const int blk_ln = c_in < 1024 ? c_in : 1024;
    p.blk_o = c_attn < 16 ? c_attn : 16;
    p.blk_a = c_ffn < 16 ? c_ffn : 16;
    const int tc = s.w16 ? PD_WGEMM_TILE_COLS : 0;
    const int g_in = g_in_opt > 0 ? g_in_opt : auto_workgroups(B, s.d, s.n_in, 0, 1, blk_ln, tc);
    const int g_out = g_out_opt > 0 ? g_out_opt : auto_workgroups(B, s.k_out, s.d, c_attn, p.blk_o, p.blk_a, tc);
    p.in = pd::qgemm_plan(B, s.d, s.n_in, g_in, 0, 1, blk_ln, &p.slots_in, tc);
    p.out = pd::qgemm_plan(B, s.k_out, s.d, g_out, c_attn, p.blk_o, p.blk_a, &p.slots_out, tc);
    return p;
}

// Upper bound of the partial-sum slots of one tile for ANY workgroup count up to
// PD_GEMM_WORKGROUPS: one, plus the workgroup ranges that can start strictly inside a
// tile of C chunks.  Range starts are floor(g*U/G) rounded down to the ring (at most 4
// units), so two consecutive starts are at least floor(U/G) - 3 units apart, and more
// workgroups only make the ranges shorter.
int slots_bound(const pd::SkqPlan& pl) {
    const long long U = (long long)pl.T * pl.C;
    long long min_len = U / PD_GEMM_WORKGROUPS - 3;
    if (min_len < 1) min_len = 1;
    return 1 + (int)((pl.C - 1 + min_len - 1) / min_len);
}

// workspace carving; the partial-sum areas hold slots_bound() slots, so a workgroup
// count set through pd_set_option never overflows them
struct Workspace {
    size_t flag, cs, xres, h, hs, part_in, nseg_in, q, act, acts, opart, ml, part_out, nseg_out, stats, total;
};
Workspace workspace_layout(const Shape& s, int B, int L_ctx) {
    Workspace w;
    size_t o = 0;
    const size_t nsplit_max = (size_t)(L_ctx / 32 + PD_MIN_BLOCKS_PER_SPLIT - 1) / PD_MIN_BLOCKS_PER_SPLIT;
    const GemmPlans gp = gemm_plans(s, B, 0, 0);
    w.flag = o; o += 1024;  // 256 per-row position flags
    w.cs = o; o += align256((size_t)B * (s.dh / 2) * 2 * 4);
    w.xres = o; o += align256((size_t)B * s.d * 4);
    w.h = o; o += align256((size_t)B * s.d * 3);                    // digit planes of LN(x)
    w.hs = o; o += align256((size_t)(s.d / 128) * 256 * 4);         // their scales [chunk][256]
    w.part_in = o; o += align256((size_t)slots_bound(gp.in) * gp.in.rows * s.n_in * 4);
    w.nseg_in = o; o += align256(pd::skq_table_ints(gp.in.T, PD_GEMM_WORKGROUPS) * 4);
    w.q = o; o += align256((size_t)B * s.H * s.dh * 4);
    w.act = o; o += align256((size_t)B * s.k_out * 3);              // digit planes of [o | a]
    w.acts = o; o += align256((size_t)(s.k_out / 128) * 256 * 4);
    w.opart = o; o += align256((size_t)B * nsplit_max * s.H * s.dh * 4);
    w.ml = o; o += align256((size_t)B * nsplit_max * s.H * 2 * 4);
    w.part_out = o; o += align256((size_t)slots_bound(gp.out) * gp.out.rows * s.d * 4);
    w.nseg_out = o; o += align256(pd::skq_table_ints(gp.out.T, PD_GEMM_WORKGROUPS) * 4);
    w.stats = o; o += align256((size_t)B * ((s.d + 1023) / 1024) * 4 * 4);  // LayerNorm slice statistics
    w.total = o;
    return w;
}

size_t kv_layer_elems(const Shape& s, int B, int L_ctx) { return (size_t)B * s.G * L_ctx * s.dh; }

// Limits that depend on the batch: the projection operand and the partial-sum slots
// are also addressed through 32-bit buffer descriptors.
pd_status check_limits(const Shape& s, int B) {
    const long long K_max = s.k_out > s.d ? s.k_out : s.d;
    if ((long long)B * K_max * 3 >= (1ll << 31)) return fail(PD_ERR_SHAPE, "batch x projection depth too large");
    const GemmPlans gp = gemm_plans(s, B, 0, 0);
    if ((long long)slots_bound(gp.in) * gp.in.rows * s.n_in * 4 >= (1ll << 32) ||
        (long long)slots_bound(gp.out) * gp.out.rows * s.d * 4 >= (1ll << 32))
        return fail(PD_ERR_SHAPE, "batch x projection width too large");
    return PD_OK;
}

}  // namespace

struct pd_handle {
    pd_model_desc desc;
    Shape s;
    int opt_g_in = 0, opt_g_out = 0, opt_bps = 0;  // 0 = automatic
    int act_digits = 3;  // int8 digit planes per projection operand
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    hipGraph_t gen_graph = nullptr;  // one iteration of pd_generate
    hipGraphExec_t gen_exec = nullptr;
    // optional event timing of one kernel class (0 = off), see pd_profile_read
    int profile_kernel = 0;
    std::vector<hipEvent_t> ev_pool;  // pairs: start, stop
    size_t ev_used = 0;
};

namespace {

#define PD_TRY_HIP(expr, where)                          \
    do {                                                 \
        hipError_t _e = (expr);                          \
        if (_e != hipSuccess) return fail_hip(_e, where); \
    } while (0)

enum { PROF_QGEMM_IN = 1, PROF_ATTEND = 2, PROF_QGEMM_OUT = 3, PROF_EPI_IN = 4, PROF_EPI_OUT = 5 };

// Records an event on `st` if kernel class `which` is being timed.  Events are
// created on first use and reused after pd_profile_read().
void prof_mark(pd_handle* h, int which, hipStream_t st) {
    if (h->profile_kernel != which) return;
    if (h->ev_used == h->ev_pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        h->ev_pool.push_back(e);
    }
    (void)hipEventRecord(h->ev_pool[h->ev_used++], st);
}

struct StepArgs {
    const unsigned char* packed;  // first layer to run
    void* k_cache;
    void* v_cache;
    const uint16_t* x_in;
    const int32_t* positions;
    int B, L_ctx;
    uint16_t* x_out_bf16;
    float* y_out_f32;
    int add_residual;
    int layer0, n_run;  // cache layer index of the first layer, number of layers to run
    unsigned char* ws;
    const int32_t* seq = nullptr;  // cache row of each token row (NULL: row b uses cache row b)
    int cache_rows = 0;            // rows of the caches (0: B)
};

pd_status run_layers(pd_handle* h, const StepArgs& a, hipStream_t st) {
    const Shape& s = h->s;
    const PackedLayout pl = packed_layout(s);
    const Workspace w = workspace_layout(s, a.B, a.L_ctx);
    const int B = a.B;
    float* cs = reinterpret_cast<float*>(a.ws + w.cs);
    int32_t* flag = reinterpret_cast<int32_t*>(a.ws + w.flag);
    float* stats = reinterpret_cast<float*>(a.ws + w.stats);
    float* xres = reinterpret_cast<float*>(a.ws + w.xres);
    unsigned char* hq = a.ws + w.h;
    float* hs = reinterpret_cast<float*>(a.ws + w.hs);
    float* part_in = reinterpret_cast<float*>(a.ws + w.part_in);
    float* q = reinterpret_cast<float*>(a.ws + w.q);
    unsigned char* actq = a.ws + w.act;
    float* acts = reinterpret_cast<float*>(a.ws + w.acts);
    float* opart = reinterpret_cast<float*>(a.ws + w.opart);
    float* ml = reinterpret_cast<float*>(a.ws + w.ml);
    float* part_out = reinterpret_cast<float*>(a.ws + w.part_out);

    GemmPlans gp = gemm_plans(s, B, h->opt_g_in, h->opt_g_out);
    gp.in.nseg = reinterpret_cast<const int*>(a.ws + w.nseg_in);
    gp.out.nseg = reinterpret_cast<const int*>(a.ws + w.nseg_out);
    if (gp.slots_in > slots_bound(gp.in) || gp.slots_out > slots_bound(gp.out))
        return fail(PD_ERR_STATE, "internal: partial-sum slots exceed the workspace bound");
    const pd::SkqPlan& pl_in = gp.in;
    const pd::SkqPlan& pl_out = gp.out;
    const int blk_o = gp.blk_o, blk_a = gp.blk_a;
    const int bps = h->opt_bps > 0 ? h->opt_bps : auto_bps(B * s.G, a.L_ctx);
    const int nd = h->act_digits;
    const int cache_rows = a.cache_rows > 0 ? a.cache_rows : B;
    const size_t kv_layer_bytes = kv_layer_elems(s, cache_rows, a.L_ctx) * 2;

    PD_TRY_HIP(pd::launch_prep(a.positions, B, a.L_ctx, s.dh, h->desc.rope_base, cs, flag, a.seq, cache_rows, st), "prep");
    PD_TRY_HIP(pd::launch_skq_table(pl_in, reinterpret_cast<int*>(a.ws + w.nseg_in), st), "segment table (in)");
    PD_TRY_HIP(pd::launch_skq_table(pl_out, reinterpret_cast<int*>(a.ws + w.nseg_out), st), "segment table (out)");
    for (int i = 0; i < a.n_run; i++) {
        const unsigned char* L = a.packed + (size_t)i * pl.total;
        const float* s_in = reinterpret_cast<const float*>(L + pl.s_in);
        const float* s_out = reinterpret_cast<const float*>(L + pl.s_out);
        const float* gamma = reinterpret_cast<const float*>(L + pl.gamma);
        unsigned char* kc = static_cast<unsigned char*>(a.k_cache) + (size_t)(a.layer0 + i) * kv_layer_bytes;
        unsigned char* vc = static_cast<unsigned char*>(a.v_cache) + (size_t)(a.layer0 + i) * kv_layer_bytes;
        if (i == 0)
            PD_TRY_HIP(pd::launch_ln_first(a.x_in, gamma, B, s.d, h->desc.ln_eps, xres, hq, hs, nd, st), "ln_first");
        prof_mark(h, PROF_QGEMM_IN, st);
        if (s.w16) PD_TRY_HIP(pd::launch_wgemm_bf16(L + pl.w_in, hq, hs, part_in, B, s.d, s.n_in, pl_in, nd, st), "wgemm_in");
        else PD_TRY_HIP(pd::launch_qgemm(L + pl.w_in, hq, hs, part_in, B, s.d, s.n_in, pl_in, nd, st), "qgemm_in");
        prof_mark(h, PROF_QGEMM_IN, st);
        prof_mark(h, PROF_EPI_IN, st);
        PD_TRY_HIP(pd::launch_epi_in(part_in, pl_in, s_in, cs, a.positions, a.seq, cache_rows, B, s.H, s.G, s.dh, s.F, a.L_ctx, q,
                                     kc, vc, actq, acts, blk_a, nd, st), "epi_in");
        prof_mark(h, PROF_EPI_IN, st);
        prof_mark(h, PROF_ATTEND, st);
        PD_TRY_HIP(pd::launch_mqa_attend(q, kc, vc, a.positions, a.seq, cache_rows, B, s.H, s.G, s.dh, a.L_ctx, bps, opart, ml,
                                         nullptr, actq, acts, s.k_out, blk_o, nd, st), "mqa_attend");
        prof_mark(h, PROF_ATTEND, st);
        prof_mark(h, PROF_QGEMM_OUT, st);
        if (s.w16) PD_TRY_HIP(pd::launch_wgemm_bf16(L + pl.w_out, actq, acts, part_out, B, s.k_out, s.d, pl_out, nd, st), "wgemm_out");
        else PD_TRY_HIP(pd::launch_qgemm(L + pl.w_out, actq, acts, part_out, B, s.k_out, s.d, pl_out, nd, st), "qgemm_out");
        prof_mark(h, PROF_QGEMM_OUT, st);
        const bool last = i == a.n_run - 1;
        prof_mark(h, PROF_EPI_OUT, st);
        if (!last && s.d <= PD_RESIDUAL_LN_MAX_D) {
            // the updated row stays in one workgroup's registers from the residual add to the
            // next layer's LayerNorm
            const unsigned char* Ln = L + pl.total;
            PD_TRY_HIP(pd::launch_residual_ln(part_out, pl_out, s_out, xres, B, s.d, a.add_residual,
                                              reinterpret_cast<const float*>(Ln + pl.gamma), h->desc.ln_eps,
                                              hq, hs, nd, st), "residual + ln");
        } else {
            PD_TRY_HIP(pd::launch_residual(part_out, pl_out, s_out, xres, B, s.d, a.add_residual,
                                           last ? a.x_out_bf16 : nullptr, last ? a.y_out_f32 : nullptr,
                                           last ? nullptr : stats, st),
                       "residual");
            if (!last) {
                const unsigned char* Ln = L + pl.total;
                PD_TRY_HIP(pd::launch_ln_slices(xres, reinterpret_cast<const float*>(Ln + pl.gamma),
                                                reinterpret_cast<const float*>(Ln + pl.gamma_absmax), stats, B, s.d,
                                                h->desc.ln_eps, hq, hs, nd, st), "ln");
            }
        }
        prof_mark(h, PROF_EPI_OUT, st);
    }
    return PD_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int PD_MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[PD_MAX_DEVICES];
std::mutex g_scratch_mu;

pd_status static_scratch(unsigned char** out) {
    int dev = -1;
    PD_TRY_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= PD_MAX_DEVICES) return fail(PD_ERR_RANGE, "device index beyond the library's table");
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        PD_TRY_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (!p || !aligned(p, 256)) return fail(PD_ERR_HIP, "static scratch has no usable device address");
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return PD_OK;
}

pd_status check_step_args(pd_handle* h, const void* packed, void* kc, void* vc, const uint16_t* x_in,
                          const int32_t* positions, int32_t B, int32_t L_ctx, const void* out,
                          void* ws, size_t ws_bytes) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!packed || !kc || !vc || !x_in || !positions || !out || !ws) return fail(PD_ERR_NULL, "NULL device pointer");
    pd_status rc = check_batch(B, L_ctx);
    if (rc != PD_OK) return rc;
    if ((rc = check_limits(h->s, B)) != PD_OK) return rc;
    if (!aligned(packed, 256) || !aligned(kc, 256) || !aligned(vc, 256) || !aligned(ws, 256))
        return fail(PD_ERR_ALIGN, "packed weights, caches and workspace must be 256-byte aligned");
    if (!aligned(x_in, 16) || !aligned(out, 16) || !aligned(positions, 4))
        return fail(PD_ERR_ALIGN, "x_in/x_out must be 16-byte aligned");
    if (ws_bytes < workspace_layout(h->s, B, L_ctx).total) return fail(PD_ERR_WORKSPACE, "workspace too small");
    return PD_OK;
}

}  // namespace

extern "C" {

const char* pd_status_string(pd_status code) {
    switch (code) {
        case PD_OK: return "ok";
        case PD_ERR_NULL: return "null pointer";
        case PD_ERR_ALIGN: return "misaligned pointer";
        case PD_ERR_SHAPE: return "unsupported shape";
        case PD_ERR_RANGE: return "argument out of range";
        case PD_ERR_WORKSPACE: return "workspace too small";
        case PD_ERR_HIP: return "HIP runtime error";
        case PD_ERR_POSITION: return "position outside [0, L_ctx)";
        case PD_ERR_STATE: return "invalid state";
        default: return "unknown status";
    }
}

const char* pd_last_error(void) { return g_err; }

pd_status pd_packed_layer_bytes(const pd_model_desc* desc, size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = packed_layout(s).total;
    return PD_OK;
}

pd_status pd_kv_cache_bytes(const pd_model_desc* desc, int32_t B, int32_t L_ctx, size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if ((rc = check_batch(B, L_ctx)) != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = (size_t)s.L * kv_layer_elems(s, B, L_ctx) * 2;
    return PD_OK;
}

pd_status pd_workspace_bytes(const pd_model_desc* desc, int32_t B, int32_t L_ctx, size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if ((rc = check_batch(B, L_ctx)) != PD_OK) return rc;
    if ((rc = check_limits(s, B)) != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = workspace_layout(s, B, L_ctx).total;
    return PD_OK;
}

pd_status pd_create(const pd_model_desc* desc, pd_handle** out) {
    if (!out) return fail(PD_ERR_NULL, "out is NULL");
    *out = nullptr;
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    pd_handle* h = new (std::nothrow) pd_handle();
    if (!h) return fail(PD_ERR_STATE, "out of host memory");
    h->desc = *desc;
    h->s = s;
    *out = h;
    return PD_OK;
}

pd_status pd_graph_release(pd_handle* h) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (h->graph_exec) { (void)hipGraphExecDestroy(h->graph_exec); h->graph_exec = nullptr; }
    if (h->graph) { (void)hipGraphDestroy(h->graph); h->graph = nullptr; }
    if (h->gen_exec) { (void)hipGraphExecDestroy(h->gen_exec); h->gen_exec = nullptr; }
    if (h->gen_graph) { (void)hipGraphDestroy(h->gen_graph); h->gen_graph = nullptr; }
    return PD_OK;
}

pd_status pd_destroy(pd_handle* h) {
    if (!h) return PD_OK;
    pd_graph_release(h);
    for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
    delete h;
    return PD_OK;
}

pd_status pd_set_option(pd_handle* h, const char* name, int32_t value) {
    if (!h || !name) return fail(PD_ERR_NULL, "NULL argument");
    if (!strcmp(name, "gemm_workgroups_in") || !strcmp(name, "gemm_workgroups_out")) {
        if (value < 0 || value > PD_GEMM_WORKGROUPS) return fail(PD_ERR_RANGE, "workgroup count must be in 0..256");
        (!strcmp(name, "gemm_workgroups_in") ? h->opt_g_in : h->opt_g_out) = value;
        return PD_OK;
    }
    if (!strcmp(name, "attn_blocks_per_split")) {
        if (value != 0 && (value < PD_MIN_BLOCKS_PER_SPLIT || value > 4096)) return fail(PD_ERR_RANGE, "attn_blocks_per_split must be 0 or in 4..4096");
        h->opt_bps = value;
        return PD_OK;
    }
    if (!strcmp(name, "act_digits")) {
        if (value != 2 && value != 3) return fail(PD_ERR_RANGE, "act_digits must be 2 or 3");
        h->act_digits = value;
        return PD_OK;
    }
    if (!strcmp(name, "profile_kernel")) {
        if (value < 0 || value > PROF_EPI_OUT) return fail(PD_ERR_RANGE, "profile_kernel must be in 0..5");
        h->profile_kernel = value;
        h->ev_used = 0;
        return PD_OK;
    }
    return fail(PD_ERR_RANGE, "unknown option");
}

pd_status pd_profile_read(pd_handle* h, double* total_ms, int32_t* launches) {
    if (!h || !total_ms || !launches) return fail(PD_ERR_NULL, "NULL argument");
    double sum = 0.0;
    const size_t pairs = h->ev_used / 2;
    for (size_t i = 0; i < pairs; i++) {
        PD_TRY_HIP(hipEventSynchronize(h->ev_pool[2 * i + 1]), "event synchronize");
        float ms = 0.f;
        PD_TRY_HIP(hipEventElapsedTime(&ms, h->ev_pool[2 * i], h->ev_pool[2 * i + 1]), "event elapsed");
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int32_t)pairs;
    h->ev_used = 0;
    return PD_OK;
}

pd_status pd_pack_matrix(const int8_t* w, int32_t K, int32_t N, void* packed_w, void* stream) {
    if (!w || !packed_w) return fail(PD_ERR_NULL, "NULL device pointer");
    if (K < 128 || K % 128 || N < 32 || N % 32) return fail(PD_ERR_SHAPE, "K must be a multiple of 128 and N a multiple of 32");
    if (!aligned(packed_w, 256)) return fail(PD_ERR_ALIGN, "packed_w must be 256-byte aligned");
    PD_TRY_HIP(pd::launch_pack_matrix(w, packed_w, K, N, 0, 0, 0, static_cast<hipStream_t>(stream)), "pack_matrix");
    return PD_OK;
}

pd_status pd_pack_layer(pd_handle* h, const int8_t* w_in, const uint16_t* s_in, const int8_t* w_out,
                        const uint16_t* s_out, const uint16_t* gamma, void* packed_layer, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    const Shape& s = h->s;
    if (!w_in || !w_out || !gamma || !packed_layer || (!s.w16 && (!s_in || !s_out)))
        return fail(PD_ERR_NULL, "NULL device pointer");
    if (!aligned(packed_layer, 256)) return fail(PD_ERR_ALIGN, "packed_layer must be 256-byte aligned");
    const PackedLayout pl = packed_layout(s);
    unsigned char* dst = static_cast<unsigned char*>(packed_layer);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (s.w16) {
        // bf16 matrices arrive through the same two pointers; every channel scale is one
        PD_TRY_HIP(pd::launch_pack_matrix_bf16(reinterpret_cast<const uint16_t*>(w_in), dst + pl.w_in, s.d, s.n_in, 1,
                                               s.n_qkv, s.F, st), "pack w_in (bf16)");
        PD_TRY_HIP(pd::launch_pack_matrix_bf16(reinterpret_cast<const uint16_t*>(w_out), dst + pl.w_out, s.k_out, s.d,
                                               0, 0, 0, st), "pack w_out (bf16)");
        PD_TRY_HIP(pd::launch_fill_f32(reinterpret_cast<float*>(dst + pl.s_in), s.n_in, 1.0f, st), "unit s_in");
        PD_TRY_HIP(pd::launch_fill_f32(reinterpret_cast<float*>(dst + pl.s_out), s.d, 1.0f, st), "unit s_out");
    } else {
        PD_TRY_HIP(pd::launch_pack_matrix(w_in, dst + pl.w_in, s.d, s.n_in, 1, s.n_qkv, s.F, st), "pack w_in");
        PD_TRY_HIP(pd::launch_pack_matrix(w_out, dst + pl.w_out, s.k_out, s.d, 0, 0, 0, st), "pack w_out");
        PD_TRY_HIP(pd::launch_pack_vector(s_in, reinterpret_cast<float*>(dst + pl.s_in), s.n_in, 1, s.n_qkv, s.F, st), "pack s_in");
        PD_TRY_HIP(pd::launch_pack_vector(s_out, reinterpret_cast<float*>(dst + pl.s_out), s.d, 0, 0, 0, st), "pack s_out");
    }
    PD_TRY_HIP(pd::launch_pack_vector(gamma, reinterpret_cast<float*>(dst + pl.gamma), s.d, 0, 0, 0, st), "pack gamma");
    PD_TRY_HIP(pd::launch_vec_absmax(reinterpret_cast<const float*>(dst + pl.gamma), s.d,
                                     reinterpret_cast<float*>(dst + pl.gamma_absmax), st), "gamma absmax");
    return PD_OK;
}

static pd_status kv_convert(pd_handle* h, const void* src, void* dst, int32_t layer, int32_t B,
                            int32_t L_ctx, int32_t is_v, int to_library, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!src || !dst) return fail(PD_ERR_NULL, "NULL device pointer");
    pd_status rc = check_batch(B, L_ctx);
    if (rc != PD_OK) return rc;
    if (layer < 0 || layer >= h->s.L) return fail(PD_ERR_RANGE, "layer out of range");
    if (!aligned(src, 16) || !aligned(dst, 16)) return fail(PD_ERR_ALIGN, "cache pointers must be 16-byte aligned");
    const size_t off = (size_t)layer * kv_layer_elems(h->s, B, L_ctx) * 2;
    const void* s2 = to_library ? src : static_cast<const unsigned char*>(src) + off;
    void* d2 = to_library ? static_cast<unsigned char*>(dst) + off : dst;
    PD_TRY_HIP(pd::launch_kv_convert(s2, d2, B * h->s.G, L_ctx, h->s.dh, is_v ? 1 : 0, to_library,
                                     static_cast<hipStream_t>(stream)), "kv_convert");
    return PD_OK;
}

pd_status pd_kv_import(pd_handle* h, const uint16_t* canonical, void* cache, int32_t layer, int32_t B,
                       int32_t L_ctx, int32_t is_v, void* stream) {
    return kv_convert(h, canonical, cache, layer, B, L_ctx, is_v, 1, stream);
}

pd_status pd_kv_export(pd_handle* h, const void* cache, uint16_t* canonical, int32_t layer, int32_t B,
                       int32_t L_ctx, int32_t is_v, void* stream) {
    return kv_convert(h, cache, canonical, layer, B, L_ctx, is_v, 0, stream);
}

pd_status pd_decode_step(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                         const uint16_t* x_in, const int32_t* positions, int32_t B, int32_t L_ctx,
                         uint16_t* x_out, void* workspace, size_t workspace_bytes, void* stream) {
    pd_status rc = check_step_args(h, packed_weights, k_cache, v_cache, x_in, positions, B, L_ctx, x_out,
                                   workspace, workspace_bytes);
    if (rc != PD_OK) return rc;
    StepArgs a{static_cast<const unsigned char*>(packed_weights), k_cache, v_cache, x_in, positions, B, L_ctx,
               x_out, nullptr, 1, 0, h->s.L, static_cast<unsigned char*>(workspace)};
    return run_layers(h, a, static_cast<hipStream_t>(stream));
}

pd_status pd_decode_step_static(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                                const uint16_t* x_in, const int32_t* positions, int32_t B, int32_t L_ctx,
                                uint16_t* x_out, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    pd_status rc = check_batch(B, L_ctx);
    if (rc != PD_OK) return rc;
    if ((rc = check_limits(h->s, B)) != PD_OK) return rc;
    const size_t need = workspace_layout(h->s, B, L_ctx).total;
    if (need > PD_STATIC_SCRATCH_BYTES) {
        snprintf(g_err, sizeof(g_err), "this shape needs %zu bytes of scratch; pd_decode_step_static holds %u "
                 "(use pd_decode_step with a caller workspace)", need, PD_STATIC_SCRATCH_BYTES);
        return PD_ERR_WORKSPACE;
    }
    unsigned char* ws = nullptr;
    if ((rc = static_scratch(&ws)) != PD_OK) return rc;
    rc = check_step_args(h, packed_weights, k_cache, v_cache, x_in, positions, B, L_ctx, x_out, ws,
                         PD_STATIC_SCRATCH_BYTES);
    if (rc != PD_OK) return rc;
    StepArgs a{static_cast<const unsigned char*>(packed_weights), k_cache, v_cache, x_in, positions, B, L_ctx,
               x_out, nullptr, 1, 0, h->s.L, ws};
    return run_layers(h, a, static_cast<hipStream_t>(stream));
}

pd_status pd_prefill(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                     const uint16_t* x_in, const int32_t* seq_ids, const int32_t* positions, int32_t n_tokens,
                     int32_t cache_rows, int32_t L_ctx, uint16_t* x_out, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!seq_ids) return fail(PD_ERR_NULL, "NULL device pointer");
    if (n_tokens < 1 || n_tokens > (1 << 24)) return fail(PD_ERR_SHAPE, "n_tokens must be in 1..2^24");
    if (cache_rows < 1 || cache_rows > 65535) return fail(PD_ERR_SHAPE, "cache_rows must be in 1..65535");
    // the stack runs on chunks of up to PD_PREFILL_CHUNK token rows: every chunk streams the weights once
    const int chunk = n_tokens < PD_PREFILL_CHUNK ? n_tokens : PD_PREFILL_CHUNK;
    pd_status rc = check_step_args(h, packed_weights, k_cache, v_cache, x_in, positions, chunk, L_ctx, x_out,
                                   workspace, workspace_bytes);
    if (rc != PD_OK) return rc;
    if (!aligned(seq_ids, 4)) return fail(PD_ERR_ALIGN, "seq_ids must be 4-byte aligned");
    const size_t d = (size_t)h->s.d;
    for (int t0 = 0; t0 < n_tokens; t0 += PD_PREFILL_CHUNK) {
        const int rows = n_tokens - t0 < PD_PREFILL_CHUNK ? n_tokens - t0 : PD_PREFILL_CHUNK;
        if ((rc = check_limits(h->s, rows)) != PD_OK) return rc;
        if (workspace_bytes < workspace_layout(h->s, rows, L_ctx).total) return fail(PD_ERR_WORKSPACE, "workspace too small");
        StepArgs a{static_cast<const unsigned char*>(packed_weights), k_cache, v_cache, x_in + t0 * d,
                   positions + t0, rows, L_ctx, x_out + t0 * d, nullptr, 1, 0, h->s.L,
                   static_cast<unsigned char*>(workspace)};
        a.seq = seq_ids + t0;
        a.cache_rows = cache_rows;
        if ((rc = run_layers(h, a, static_cast<hipStream_t>(stream))) != PD_OK) return rc;
    }
    return PD_OK;
}

pd_status pd_decode_layer(pd_handle* h, int32_t layer, const void* packed_layer, void* k_cache,
                          void* v_cache, const uint16_t* x_in, const int32_t* positions, int32_t B,
                          int32_t L_ctx, float* y_out, int32_t add_residual, void* workspace,
                          size_t workspace_bytes, void* stream) {
    pd_status rc = check_step_args(h, packed_layer, k_cache, v_cache, x_in, positions, B, L_ctx, y_out,
                                   workspace, workspace_bytes);
    if (rc != PD_OK) return rc;
    if (layer < 0 || layer >= h->s.L) return fail(PD_ERR_RANGE, "layer out of range");
    StepArgs a{static_cast<const unsigned char*>(packed_layer), k_cache, v_cache, x_in, positions, B, L_ctx,
               nullptr, y_out, add_residual ? 1 : 0, layer, 1, static_cast<unsigned char*>(workspace)};
    return run_layers(h, a, static_cast<hipStream_t>(stream));
}

pd_status pd_check_async(pd_handle* h, void* workspace, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "NULL argument");
    if (!workspace) {  // the step ran on the library's static scratch
        unsigned char* ws = nullptr;
        pd_status rc = static_scratch(&ws);
        if (rc != PD_OK) return rc;
        workspace = ws;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    PD_TRY_HIP(hipStreamSynchronize(st), "stream synchronize");
    int32_t flags[256];
    PD_TRY_HIP(hipMemcpy(flags, workspace, sizeof(flags), hipMemcpyDeviceToHost), "read flags");
    for (int b = 0; b < 256; b++)
        if (flags[b]) {
            snprintf(g_err, sizeof(g_err), "positions[%d] was outside [0, L_ctx); that row was skipped", b);
            return PD_ERR_POSITION;
        }
    return PD_OK;
}

namespace {
// test entry: every 128-element chunk has its own scale (blocks of one chunk)
struct QgemmWs {
    pd::SkqPlan pl;
    size_t part, qa, qs, nseg, total;
};
QgemmWs qgemm_ws(int B, int K, int N, int workgroups, int tile_cols = 0) {
    QgemmWs q;
    int slots = 1;
    q.pl = pd::qgemm_plan(B, K, N, workgroups > 0 ? workgroups : auto_workgroups(B, K, N, 0, 1, 1, tile_cols), 0, 1, 1,
                          &slots, tile_cols);
    size_t o = 0;
    q.part = o; o += align256((size_t)slots * q.pl.rows * N * 4);
    q.qa = o; o += align256((size_t)B * K * 3);
    q.qs = o; o += align256((size_t)(K / 128) * 256 * 4);
    q.nseg = o; o += align256(pd::skq_table_ints(q.pl.T, q.pl.G) * 4);
    q.total = o;
    return q;
}
}  // namespace

pd_status pd_qgemm_workspace_bytes(int32_t B, int32_t K, int32_t N, int32_t workgroups, size_t* bytes) {
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    if (B < 1 || B > 256 || K < 128 || K % 128 || N < 32 || N % 32) return fail(PD_ERR_SHAPE, "unsupported GEMM shape");
    if (workgroups < 0 || workgroups > 4096) return fail(PD_ERR_RANGE, "workgroups out of range");
    // one size for both test entries (the bf16-weight kernel's wider tiles have more slots)
    const size_t a = qgemm_ws(B, K, N, workgroups).total, b = qgemm_ws(B, K, N, workgroups, PD_WGEMM_TILE_COLS).total;
    *bytes = a > b ? a : b;
    return PD_OK;
}

pd_status pd_qgemm_plan(int32_t B, int32_t K, int32_t N, int32_t workgroups, int32_t c_split,
                        int32_t blk0, int32_t blk1, int32_t* counts, int64_t* range_begin,
                        int32_t* first_slot, int32_t* slots_per_tile) {
    if (!counts) return fail(PD_ERR_NULL, "counts is NULL");
    if (B < 1 || B > 256 || K < 128 || K % 128 || N < 32 || N % 32) return fail(PD_ERR_SHAPE, "unsupported GEMM shape");
    if (workgroups < 0 || workgroups > 4096) return fail(PD_ERR_RANGE, "workgroups out of range");
    if (c_split < 0 || c_split > K / 128 || blk0 < 1 || blk0 > 1024 || blk1 < 1 || blk1 > 1024)
        return fail(PD_ERR_RANGE, "scale blocks out of range");
    int slots = 1;
    const pd::SkqPlan pl = pd::qgemm_plan(B, K, N, workgroups > 0 ? workgroups : auto_workgroups(B, K, N, c_split, blk0, blk1),
                                          c_split, blk0, blk1, &slots);
    counts[0] = pl.G; counts[1] = pl.T; counts[2] = pl.C; counts[3] = pl.rows; counts[4] = slots;
    const long long U = (long long)pl.T * pl.C;
    for (int g = 0; g <= pl.G; g++) {
        const long long u0 = pd::skq_begin(g, U, pl.G, pl.align);
        if (range_begin) range_begin[g] = u0;
        if (first_slot && g < pl.G) {
            const int t0 = (int)(u0 / pl.C);
            first_slot[g] = u0 < pd::skq_begin(g + 1, U, pl.G, pl.align)
                                ? pd::skq_segments_upto(t0, (int)(u0 - (long long)t0 * pl.C), pl) : 0;
        }
    }
    if (slots_per_tile)
        for (int t = 0; t < pl.T; t++) slots_per_tile[t] = pd::skq_segments(t, pl);
    return PD_OK;
}

pd_status pd_qgemm(const void* packed_w, const float* scale, const uint16_t* a, int32_t B, int32_t K,
                   int32_t N, float* out, int32_t workgroups, void* workspace, size_t workspace_bytes,
                   void* stream) {
    if (!packed_w || !scale || !a || !out || !workspace) return fail(PD_ERR_NULL, "NULL device pointer");
    size_t need = 0;
    pd_status rc = pd_qgemm_workspace_bytes(B, K, N, workgroups, &need);
    if (rc != PD_OK) return rc;
    if (workspace_bytes < need) return fail(PD_ERR_WORKSPACE, "workspace too small");
    if (!aligned(packed_w, 256) || !aligned(workspace, 256) || !aligned(a, 16) || !aligned(out, 16))
        return fail(PD_ERR_ALIGN, "misaligned device pointer");
    QgemmWs q = qgemm_ws(B, K, N, workgroups);
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* wsb = static_cast<unsigned char*>(workspace);
    float* part = reinterpret_cast<float*>(wsb + q.part);
    float* qs = reinterpret_cast<float*>(wsb + q.qs);
    int* nseg = reinterpret_cast<int*>(wsb + q.nseg);
    q.pl.nseg = nseg;
    PD_TRY_HIP(pd::launch_skq_table(q.pl, nseg, st), "segment table");
    PD_TRY_HIP(pd::launch_quantize_bf16(a, wsb + q.qa, qs, B, K, 3, st), "quantize");
    PD_TRY_HIP(pd::launch_qgemm(packed_w, wsb + q.qa, qs, part, B, K, N, q.pl, 3, st), "qgemm");
    PD_TRY_HIP(pd::launch_qgemm_reduce(part, scale, out, B, N, q.pl, st), "qgemm_reduce");
    return PD_OK;
}

pd_status pd_pack_matrix_bf16(const uint16_t* w, int32_t K, int32_t N, void* packed_w, void* stream) {
    if (!w || !packed_w) return fail(PD_ERR_NULL, "NULL device pointer");
    if (K < 128 || K % 128 || N < 32 || N % 32) return fail(PD_ERR_SHAPE, "K must be a multiple of 128 and N a multiple of 32");
    if ((long long)K * N * 2 >= (1ll << 32)) return fail(PD_ERR_SHAPE, "matrix must be smaller than 4 GiB");
    if (!aligned(packed_w, 256)) return fail(PD_ERR_ALIGN, "packed_w must be 256-byte aligned");
    PD_TRY_HIP(pd::launch_pack_matrix_bf16(w, packed_w, K, N, 0, 0, 0, static_cast<hipStream_t>(stream)), "pack_matrix_bf16");
    return PD_OK;
}

pd_status pd_wgemm_bf16(const void* packed_w, const uint16_t* a, int32_t B, int32_t K, int32_t N, float* out,
                        int32_t workgroups, void* workspace, size_t workspace_bytes, void* stream) {
    if (!packed_w || !a || !out || !workspace) return fail(PD_ERR_NULL, "NULL device pointer");
    size_t need = 0;
    pd_status rc = pd_qgemm_workspace_bytes(B, K, N, workgroups, &need);
    if (rc != PD_OK) return rc;
    if ((long long)K * N * 2 >= (1ll << 32)) return fail(PD_ERR_SHAPE, "matrix must be smaller than 4 GiB");
    if (workspace_bytes < need) return fail(PD_ERR_WORKSPACE, "workspace too small");
    if (!aligned(packed_w, 256) || !aligned(workspace, 256) || !aligned(a, 16) || !aligned(out, 16))
        return fail(PD_ERR_ALIGN, "misaligned device pointer");
    QgemmWs q = qgemm_ws(B, K, N, workgroups, PD_WGEMM_TILE_COLS);
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* wsb = static_cast<unsigned char*>(workspace);
    float* part = reinterpret_cast<float*>(wsb + q.part);
    float* qs = reinterpret_cast<float*>(wsb + q.qs);
    int* nseg = reinterpret_cast<int*>(wsb + q.nseg);
    q.pl.nseg = nseg;
    PD_TRY_HIP(pd::launch_skq_table(q.pl, nseg, st), "segment table");
    PD_TRY_HIP(pd::launch_quantize_bf16(a, wsb + q.qa, qs, B, K, 3, st), "quantize");
    PD_TRY_HIP(pd::launch_wgemm_bf16(packed_w, wsb + q.qa, qs, part, B, K, N, q.pl, 3, st), "wgemm_bf16");
    PD_TRY_HIP(pd::launch_qgemm_reduce(part, nullptr, out, B, N, q.pl, st), "qgemm_reduce");
    return PD_OK;
}

pd_status pd_ceiling_probe(const void* buffer, size_t bytes, int32_t mfma_per_unit, int32_t random_operands,
                           void* sink, void* stream) {
    if (!buffer || !sink) return fail(PD_ERR_NULL, "NULL device pointer");
    if (!aligned(buffer, 16) || !aligned(sink, 4)) return fail(PD_ERR_ALIGN, "misaligned device pointer");
    if (bytes == 0 || bytes % 8388608u) return fail(PD_ERR_SHAPE, "bytes must be a positive multiple of 8 MiB");
    if (mfma_per_unit < 0 || mfma_per_unit % 6 || mfma_per_unit > 6000)
        return fail(PD_ERR_RANGE, "mfma_per_unit must be a multiple of 6 in 0..6000");
    if (random_operands < 0 || random_operands > 2) return fail(PD_ERR_RANGE, "random_operands must be 0, 1 or 2");
    PD_TRY_HIP(pd::launch_ceiling_probe(buffer, bytes, mfma_per_unit, random_operands,
                                        static_cast<unsigned*>(sink), static_cast<hipStream_t>(stream)),
               "ceiling probe");
    return PD_OK;
}

pd_status pd_mqa_attend(pd_handle* h, int32_t layer, const float* q, const void* k_cache,
                        const void* v_cache, const int32_t* positions, int32_t B, int32_t L_ctx,
                        float* o, void* workspace, size_t workspace_bytes, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!q || !k_cache || !v_cache || !positions || !o || !workspace) return fail(PD_ERR_NULL, "NULL device pointer");
    pd_status rc = check_batch(B, L_ctx);
    if (rc != PD_OK) return rc;
    if (layer < 0 || layer >= h->s.L) return fail(PD_ERR_RANGE, "layer out of range");
    if (!aligned(k_cache, 256) || !aligned(v_cache, 256) || !aligned(workspace, 256) || !aligned(q, 16) || !aligned(o, 16))
        return fail(PD_ERR_ALIGN, "misaligned device pointer");
    const Shape& s = h->s;
    const Workspace w = workspace_layout(s, B, L_ctx);
    if (workspace_bytes < w.total) return fail(PD_ERR_WORKSPACE, "workspace too small");
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const int bps = h->opt_bps > 0 ? h->opt_bps : auto_bps(B * s.G, L_ctx);
    const size_t off = (size_t)layer * kv_layer_elems(s, B, L_ctx) * 2;
    PD_TRY_HIP(pd::launch_mqa_attend(q, static_cast<const unsigned char*>(k_cache) + off,
                                     static_cast<const unsigned char*>(v_cache) + off, positions, nullptr, B, B, s.H,
                                     s.G, s.dh, L_ctx, bps, reinterpret_cast<float*>(ws + w.opart),
                                     reinterpret_cast<float*>(ws + w.ml), o, nullptr, nullptr, s.k_out, 1,
                                     h->act_digits, static_cast<hipStream_t>(stream)), "mqa_attend");
    return PD_OK;
}

// ---- sampling head and generation loop ---------------------------------------

namespace {

struct HeadLayout {  // packed head: vocabulary matrix, its scales, the final LayerNorm gain
    size_t w, s, gamma, total;
};
HeadLayout head_layout(const Shape& s, int V) {
    HeadLayout p;
    size_t o = 0;
    p.w = o; o += align256((size_t)s.d * V);
    p.s = o; o += align256((size_t)V * 4);
    p.gamma = o; o += align256((size_t)s.d * 4);
    p.total = o;
    return p;
}

pd_status check_vocab(const Shape& s, int V, int B) {
    if (V < 32 || V % 32 || V > (1 << 24)) return fail(PD_ERR_SHAPE, "vocab must be a positive multiple of 32");
    if ((long long)s.d * V >= (1ll << 32)) return fail(PD_ERR_SHAPE, "the vocabulary matrix must be smaller than 4 GiB");
    const int blk_ln = s.d / 128 < 1024 ? s.d / 128 : 1024;
    int slots = 1;
    const pd::SkqPlan pl = pd::qgemm_plan(B, s.d, V, auto_workgroups(B, s.d, V, 0, 1, blk_ln), 0, 1, blk_ln, &slots);
    if ((long long)slots * pl.rows * V * 4 >= (1ll << 32)) return fail(PD_ERR_SHAPE, "batch x vocab too large");
    return PD_OK;
}

struct HeadWs {  // scratch of the head for batch B
    pd::SkqPlan pl;
    size_t xres, hq, hs, part, nseg, total;
};
HeadWs head_ws(const Shape& s, int V, int B) {
    HeadWs w;
    const int blk_ln = s.d / 128 < 1024 ? s.d / 128 : 1024;
    int slots = 1;
    w.pl = pd::qgemm_plan(B, s.d, V, auto_workgroups(B, s.d, V, 0, 1, blk_ln), 0, 1, blk_ln, &slots);
    size_t o = 0;
    w.xres = o; o += align256((size_t)B * s.d * 4);
    w.hq = o; o += align256((size_t)B * s.d * 3);
    w.hs = o; o += align256((size_t)(s.d / 128) * 256 * 4);
    w.part = o; o += align256((size_t)slots * w.pl.rows * V * 4);
    w.nseg = o; o += align256(pd::skq_table_ints(w.pl.T, w.pl.G) * 4);
    w.total = o;
    return w;
}

// final LayerNorm + vocabulary projection of x [B][d] bf16 -> logits [B][V] fp32
pd_status run_head(pd_handle* h, const unsigned char* packed_head, int V, const uint16_t* x, int B,
                   float* logits, unsigned char* ws, hipStream_t st) {
    const Shape& s = h->s;
    const HeadLayout hl = head_layout(s, V);
    HeadWs w = head_ws(s, V, B);
    float* hs = reinterpret_cast<float*>(ws + w.hs);
    float* part = reinterpret_cast<float*>(ws + w.part);
    int* nseg = reinterpret_cast<int*>(ws + w.nseg);
    w.pl.nseg = nseg;
    PD_TRY_HIP(pd::launch_skq_table(w.pl, nseg, st), "segment table (head)");
    PD_TRY_HIP(pd::launch_ln_first(x, reinterpret_cast<const float*>(packed_head + hl.gamma), B, s.d, h->desc.ln_eps,
                                   reinterpret_cast<float*>(ws + w.xres), ws + w.hq, hs, 3, st), "final ln");
    PD_TRY_HIP(pd::launch_qgemm(packed_head + hl.w, ws + w.hq, hs, part, B, s.d, V, w.pl, 3, st), "qgemm (vocab)");
    PD_TRY_HIP(pd::launch_qgemm_reduce(part, reinterpret_cast<const float*>(packed_head + hl.s), logits, B, V, w.pl, st),
               "logits");
    return PD_OK;
}

struct GenWs {  // workspace of pd_generate: decode scratch, head scratch, logits, hidden state, step counter
    size_t decode, head, logits, hidden, step, total;
};
GenWs gen_ws(const Shape& s, int V, int B, int L_ctx) {
    GenWs g;
    size_t o = 0;
    g.decode = o; o += align256(workspace_layout(s, B, L_ctx).total);
    g.head = o; o += align256(head_ws(s, V, B).total);
    g.logits = o; o += align256((size_t)B * V * 4);
    g.hidden = o; o += align256((size_t)B * s.d * 2);
    g.step = o; o += 256;
    g.total = o;
    return g;
}

pd_status check_sampling(int V, int top_k, float top_p, float temperature) {
    if (top_k < 1 || top_k > PD_MAX_TOP_K || top_k > V) return fail(PD_ERR_RANGE, "top_k must be in 1..64 and at most vocab");
    if (!(top_p > 0.f) || top_p > 1.f) return fail(PD_ERR_RANGE, "top_p must be in (0, 1]");
    if (!(temperature > 0.f)) return fail(PD_ERR_RANGE, "temperature must be positive");
    return PD_OK;
}

}  // namespace

pd_status pd_packed_head_bytes(const pd_model_desc* desc, int32_t vocab, size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if ((rc = check_vocab(s, vocab, 1)) != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = head_layout(s, vocab).total;
    return PD_OK;
}

pd_status pd_head_workspace_bytes(const pd_model_desc* desc, int32_t vocab, int32_t B, size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if ((rc = check_batch(B, 32)) != PD_OK) return rc;
    if ((rc = check_vocab(s, vocab, B)) != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = head_ws(s, vocab, B).total;
    return PD_OK;
}

pd_status pd_generate_workspace_bytes(const pd_model_desc* desc, int32_t vocab, int32_t B, int32_t L_ctx,
                                      size_t* bytes) {
    Shape s;
    pd_status rc = check_desc(desc, &s);
    if (rc != PD_OK) return rc;
    if ((rc = check_batch(B, L_ctx)) != PD_OK) return rc;
    if ((rc = check_limits(s, B)) != PD_OK) return rc;
    if ((rc = check_vocab(s, vocab, B)) != PD_OK) return rc;
    if (!bytes) return fail(PD_ERR_NULL, "bytes is NULL");
    *bytes = gen_ws(s, vocab, B, L_ctx).total;
    return PD_OK;
}

pd_status pd_pack_head(pd_handle* h, const int8_t* w_vocab, const uint16_t* s_vocab, const uint16_t* gamma_f,
                       int32_t vocab, void* packed_head, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!w_vocab || !s_vocab || !gamma_f || !packed_head) return fail(PD_ERR_NULL, "NULL device pointer");
    pd_status rc = check_vocab(h->s, vocab, 1);
    if (rc != PD_OK) return rc;
    if (!aligned(packed_head, 256)) return fail(PD_ERR_ALIGN, "packed_head must be 256-byte aligned");
    const HeadLayout hl = head_layout(h->s, vocab);
    unsigned char* dst = static_cast<unsigned char*>(packed_head);
    hipStream_t st = static_cast<hipStream_t>(stream);
    PD_TRY_HIP(pd::launch_pack_matrix(w_vocab, dst + hl.w, h->s.d, vocab, 0, 0, 0, st), "pack w_vocab");
    PD_TRY_HIP(pd::launch_pack_vector(s_vocab, reinterpret_cast<float*>(dst + hl.s), vocab, 0, 0, 0, st), "pack s_vocab");
    PD_TRY_HIP(pd::launch_pack_vector(gamma_f, reinterpret_cast<float*>(dst + hl.gamma), h->s.d, 0, 0, 0, st), "pack gamma_f");
    return PD_OK;
}

pd_status pd_head_logits(pd_handle* h, const void* packed_head, int32_t vocab, const uint16_t* x, int32_t B,
                         float* logits, void* workspace, size_t workspace_bytes, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!packed_head || !x || !logits || !workspace) return fail(PD_ERR_NULL, "NULL device pointer");
    pd_status rc = check_batch(B, 32);
    if (rc != PD_OK) return rc;
    if ((rc = check_limits(h->s, B)) != PD_OK) return rc;
    if ((rc = check_vocab(h->s, vocab, B)) != PD_OK) return rc;
    if (!aligned(packed_head, 256) || !aligned(workspace, 256) || !aligned(x, 16) || !aligned(logits, 16))
        return fail(PD_ERR_ALIGN, "misaligned device pointer");
    if (workspace_bytes < head_ws(h->s, vocab, B).total) return fail(PD_ERR_WORKSPACE, "workspace too small");
    return run_head(h, static_cast<const unsigned char*>(packed_head), vocab, x, B, logits,
                    static_cast<unsigned char*>(workspace), static_cast<hipStream_t>(stream));
}

pd_status pd_sample(const float* logits, int32_t B, int32_t vocab, int32_t top_k, float top_p, float temperature,
                    const float* uniforms, int32_t* tokens, void* stream) {
    if (!logits || !uniforms || !tokens) return fail(PD_ERR_NULL, "NULL device pointer");
    if (B < 1 || B > 65535 || vocab < 1) return fail(PD_ERR_SHAPE, "B must be in 1..65535 and vocab positive");
    pd_status rc = check_sampling(vocab, top_k, top_p, temperature);
    if (rc != PD_OK) return rc;
    PD_TRY_HIP(pd::launch_sample(logits, B, vocab, top_k, top_p, temperature, uniforms, nullptr, tokens,
                                 static_cast<hipStream_t>(stream)), "sample");
    return PD_OK;
}

pd_status pd_generate(pd_handle* h, const void* packed_weights, const void* packed_head, const uint16_t* embed,
                      void* k_cache, void* v_cache, uint16_t* x, int32_t* positions, int32_t B, int32_t L_ctx,
                      int32_t vocab, int32_t n_steps, int32_t top_k, float top_p, float temperature,
                      const float* uniforms, int32_t* tokens_out, int32_t use_graph, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!packed_weights || !packed_head || !embed || !k_cache || !v_cache || !x || !positions || !uniforms ||
        !tokens_out || !workspace)
        return fail(PD_ERR_NULL, "NULL device pointer");
    if (n_steps < 1 || n_steps > (1 << 20)) return fail(PD_ERR_RANGE, "n_steps must be in 1..2^20");
    pd_status rc = check_sampling(vocab, top_k, top_p, temperature);
    if (rc != PD_OK) return rc;
    const Shape& s = h->s;
    if ((rc = check_vocab(s, vocab, B > 0 ? B : 1)) != PD_OK) return rc;
    const GenWs g = gen_ws(s, vocab, B > 0 && B <= 256 ? B : 1, L_ctx >= 32 && L_ctx % 32 == 0 ? L_ctx : 32);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    uint16_t* hidden = reinterpret_cast<uint16_t*>(ws + g.hidden);
    rc = check_step_args(h, packed_weights, k_cache, v_cache, x, positions, B, L_ctx, hidden, workspace,
                         workspace_bytes);
    if (rc != PD_OK) return rc;
    if (workspace_bytes < g.total) return fail(PD_ERR_WORKSPACE, "workspace too small");
    if (!aligned(packed_head, 256) || !aligned(embed, 16)) return fail(PD_ERR_ALIGN, "misaligned device pointer");
    if (use_graph && !stream) return fail(PD_ERR_STATE, "graph replay of the loop needs a non-null stream");
    if (use_graph && h->profile_kernel) return fail(PD_ERR_STATE, "turn profile_kernel off before capturing");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t* step = reinterpret_cast<int32_t*>(ws + g.step);
    float* logits = reinterpret_cast<float*>(ws + g.logits);

    // one iteration: forward pass, logits, draw, feed the token back, advance positions
    auto iteration = [&]() -> pd_status {
        StepArgs a{static_cast<const unsigned char*>(packed_weights), k_cache, v_cache, x, positions, B, L_ctx,
                   hidden, nullptr, 1, 0, s.L, ws + g.decode};
        pd_status r = run_layers(h, a, st);
        if (r != PD_OK) return r;
        r = run_head(h, static_cast<const unsigned char*>(packed_head), vocab, hidden, B, logits, ws + g.head, st);
        if (r != PD_OK) return r;
        PD_TRY_HIP(pd::launch_sample(logits, B, vocab, top_k, top_p, temperature, uniforms, step, tokens_out, st), "sample");
        PD_TRY_HIP(pd::launch_embed_advance(embed, s.d, vocab, tokens_out, B, x, positions, step, st), "embed");
        return PD_OK;
    };

    PD_TRY_HIP(pd::launch_step_set(step, 0, st), "step counter");
    if (!use_graph) {
        for (int i = 0; i < n_steps; i++)
            if ((rc = iteration()) != PD_OK) return rc;
        return PD_OK;
    }
    if (h->gen_exec) { (void)hipGraphExecDestroy(h->gen_exec); h->gen_exec = nullptr; }
    if (h->gen_graph) { (void)hipGraphDestroy(h->gen_graph); h->gen_graph = nullptr; }
    PD_TRY_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal), "begin capture");
    rc = iteration();
    hipGraph_t gr = nullptr;
    hipError_t e = hipStreamEndCapture(st, &gr);
    if (rc != PD_OK) { if (gr) (void)hipGraphDestroy(gr); return rc; }
    if (e != hipSuccess) return fail_hip(e, "end capture");
    h->gen_graph = gr;
    e = hipGraphInstantiate(&h->gen_exec, gr, nullptr, nullptr, 0);
    if (e != hipSuccess) return fail_hip(e, "graph instantiate");
    for (int i = 0; i < n_steps; i++) PD_TRY_HIP(hipGraphLaunch(h->gen_exec, st), "graph launch");
    return PD_OK;
}

pd_status pd_graph_capture(pd_handle* h, const void* packed_weights, void* k_cache, void* v_cache,
                           const uint16_t* x_in, const int32_t* positions, int32_t B, int32_t L_ctx,
                           uint16_t* x_out, void* workspace, size_t workspace_bytes, void* stream) {
    pd_status rc = check_step_args(h, packed_weights, k_cache, v_cache, x_in, positions, B, L_ctx, x_out,
                                   workspace, workspace_bytes);
    if (rc != PD_OK) return rc;
    if (!stream) return fail(PD_ERR_STATE, "graph capture needs a non-null stream");
    if (h->profile_kernel) return fail(PD_ERR_STATE, "turn profile_kernel off before capturing");
    pd_graph_release(h);
    hipStream_t st = static_cast<hipStream_t>(stream);
    PD_TRY_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal), "begin capture");
    StepArgs a{static_cast<const unsigned char*>(packed_weights), k_cache, v_cache, x_in, positions, B, L_ctx,
               x_out, nullptr, 1, 0, h->s.L, static_cast<unsigned char*>(workspace)};
    rc = run_layers(h, a, st);
    hipGraph_t g = nullptr;
    hipError_t e = hipStreamEndCapture(st, &g);
    if (rc != PD_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
    if (e != hipSuccess) return fail_hip(e, "end capture");
    h->graph = g;
    e = hipGraphInstantiate(&h->graph_exec, g, nullptr, nullptr, 0);
    if (e != hipSuccess) { pd_graph_release(h); return fail_hip(e, "graph instantiate"); }
    return PD_OK;
}

pd_status pd_graph_replay(pd_handle* h, void* stream) {
    if (!h) return fail(PD_ERR_NULL, "handle is NULL");
    if (!h->graph_exec) return fail(PD_ERR_STATE, "no captured graph");
    PD_TRY_HIP(hipGraphLaunch(h->graph_exec, static_cast<hipStream_t>(stream)), "graph launch");
    return PD_OK;
}

}  // extern "C"
