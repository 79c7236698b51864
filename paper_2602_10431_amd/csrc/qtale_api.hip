// Host side of the C ABI declared in include/qtale.h: argument validation (before any HIP call),
// workspace carving, and the launch sequence of one token-adaptive layer:
//   router score -> select/compact -> gather+RMSNorm -> q|k|v GEMM -> rotary (+cache append) ->
//   attention over executed tokens -> o GEMM (+residual) -> RMSNorm -> gate/up GEMM (SiLU*up) ->
//   down GEMM (+residual, scatter back).
// In ratio mode the executed count k is known on the host, so every launch shape is static and the
// stack runs without any device->host synchronisation; in threshold mode grids are sized for all T
// tokens and the kernels read the device-side count.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/qtale.h"
#include "qtale_kernels.h"

using namespace qtale;

struct qtale_ctx {
    int mode = QTALE_MODE_RATIO;
    float value = 1.0f;
    bool profiling = false;
    struct Span { int cls; hipEvent_t a, b; };
    std::vector<Span> spans;
    std::vector<hipEvent_t> free_events;
    double ms[QTALE_PROF_CLASSES] = {0};
    int64_t launches[QTALE_PROF_CLASSES] = {0};
};

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Workspace {
    float* z;
    int32_t* idx;
    int32_t* scalars;      // [0] count, [1] n_items
    int32_t* cu_exec;
    int32_t* row_seq;
    int32_t* kv_old;
    void* items;
    void* nbuf;            // [T][H] fp16
    void* qkv;             // [T][(nh+2nkv)d] fp16
    void* attn;            // [T][nh d] fp16
    float* h;              // [T][H] fp32
    void* act;             // [T][I] fp16
    float* attn_part;      // [min(T, kAttnSplitRows)][nh][kAttnSplitMax][d + 2] fp32: key-range partials of decode attention
    float* gemm_part;      // [kGemmPartMax][min(T, kGemmPartRows)][H] fp32: K-part partial tiles of the decode o-/down-proj
    int32_t* inv;          // [min(T, 256)] token -> compact row of small calls (-1 = bypassed)
    size_t total;
};

Workspace carve(const qtale_layer_cfg* c, int T, int B, void* base) {
    Workspace w{};
    size_t off = 0;
    char* p = reinterpret_cast<char*>(base);
    auto take = [&](size_t bytes) {
        void* r = p ? p + off : nullptr;
        off += align_up(bytes, 256);
        return r;
    };
    const size_t Tz = static_cast<size_t>(T);
    w.z = reinterpret_cast<float*>(take(Tz * 4));
    w.idx = reinterpret_cast<int32_t*>(take(Tz * 4));
    w.scalars = reinterpret_cast<int32_t*>(take(256));
    w.cu_exec = reinterpret_cast<int32_t*>(take((static_cast<size_t>(B) + 1) * 4));
    w.row_seq = reinterpret_cast<int32_t*>(take(Tz * 4));
    w.kv_old = reinterpret_cast<int32_t*>(take(static_cast<size_t>(B) * 4 + 4));
    w.items = take((Tz / kAttnBQ + B + 2) * 16);
    w.nbuf = take(Tz * c->hidden * 2);
    w.qkv = take(Tz * (static_cast<size_t>(c->n_heads) + 2 * c->n_kv_heads) * c->head_dim * 2);
    w.attn = take(Tz * c->n_heads * c->head_dim * 2);
    w.h = reinterpret_cast<float*>(take(Tz * c->hidden * 4));
    w.act = take(Tz * c->inter * 2);
    w.attn_part = reinterpret_cast<float*>(take(static_cast<size_t>(T < kAttnSplitRows ? T : kAttnSplitRows) * c->n_heads *
                                                kAttnSplitMax * (c->head_dim + 2) * 4));
    w.gemm_part = reinterpret_cast<float*>(take(static_cast<size_t>(kGemmPartMax) * (T < kGemmPartRows ? T : kGemmPartRows) *
                                                c->hidden * 4));
    w.inv = reinterpret_cast<int32_t*>(take(static_cast<size_t>(T < 256 ? T : 256) * 4));
    w.total = off;
    return w;
}

int check_quant_params(int N, int K, int bits, int group) {
    if (N <= 0 || K <= 0) return QTALE_ERR_INVALID_ARG;
    if (bits != 4 && bits != 3 && bits != 2) return QTALE_ERR_UNSUPPORTED;
    if (group != 32 && group != 64 && group != 128) return QTALE_ERR_UNSUPPORTED;
    if (K % 8 != 0) return QTALE_ERR_SHAPE;
    return QTALE_OK;
}

int check_cfg(const qtale_layer_cfg* c) {
    if (!c) return QTALE_ERR_INVALID_ARG;
    if (c->hidden <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->inter <= 0)
        return QTALE_ERR_INVALID_ARG;
    if (c->bits != 4 && c->bits != 3 && c->bits != 2) return QTALE_ERR_UNSUPPORTED;
    if (c->group != 32 && c->group != 64 && c->group != 128) return QTALE_ERR_UNSUPPORTED;
    if (c->head_dim != 64 && c->head_dim != 128) return QTALE_ERR_UNSUPPORTED;
    if (c->act_dtype != QTALE_ACT_FP16 && c->act_dtype != QTALE_ACT_BF16) return QTALE_ERR_UNSUPPORTED;
    if (c->n_heads % c->n_kv_heads != 0) return QTALE_ERR_SHAPE;
    if (c->hidden % 8 != 0 || c->inter % 8 != 0) return QTALE_ERR_SHAPE;
    if (!(c->rms_eps >= 0.0f) || !(c->rope_base > 0.0f)) return QTALE_ERR_INVALID_ARG;
    return QTALE_OK;
}

int check_linear(const qtale_qlinear& l, int N, int K) {
    if (!l.prepacked) return QTALE_ERR_INVALID_ARG;
    if (l.N != N || l.K != K || N % 8 != 0) return QTALE_ERR_SHAPE;
    return QTALE_OK;
}

int check_weights(const qtale_layer_cfg* c, const qtale_layer_weights* w) {
    if (!w) return QTALE_ERR_INVALID_ARG;
    const int H = c->hidden, qd = c->n_heads * c->head_dim, kd = c->n_kv_heads * c->head_dim;
    int e;
    if ((e = check_linear(w->q, qd, H))) return e;
    if ((e = check_linear(w->k, kd, H))) return e;
    if ((e = check_linear(w->v, kd, H))) return e;
    if ((e = check_linear(w->o, H, qd))) return e;
    if ((e = check_linear(w->gate, c->inter, H))) return e;
    if ((e = check_linear(w->up, c->inter, H))) return e;
    if ((e = check_linear(w->down, H, c->inter))) return e;
    if (!w->norm1 || !w->norm2) return QTALE_ERR_INVALID_ARG;
    if (w->bits != 0 && w->bits != 4 && w->bits != 3 && w->bits != 2) return QTALE_ERR_UNSUPPORTED;
    if (w->router_hidden < 0 || w->router_hidden > 256) return QTALE_ERR_INVALID_ARG;
    if (w->router_hidden > 0) {
        if (!w->router_w1 || !w->router_b1 || !w->router_w2 || !w->router_b2) return QTALE_ERR_INVALID_ARG;
    } else {
        if (!w->router_w || std::isnan(w->router_b)) return QTALE_ERR_INVALID_ARG;
    }
    return QTALE_OK;
}

// k = floor(r*T + 1/2) in double, clamped.
int executed_count(float r, int T) {
    const double v = std::floor(static_cast<double>(r) * static_cast<double>(T) + 0.5);
    if (v <= 0.0) return 0;
    if (v >= static_cast<double>(T)) return T;
    return static_cast<int>(v);
}

float theta_to_logit(float theta) {
    const double t = static_cast<double>(theta);
    if (t <= 0.0) return -INFINITY;
    if (t >= 1.0) return INFINITY;
    return static_cast<float>(std::log(t / (1.0 - t)));
}

struct Prof {
    qtale_ctx* ctx;
    hipStream_t stream;
    int cls;
    hipEvent_t a = nullptr, b = nullptr;
    bool on;
    static hipEvent_t get(qtale_ctx* c) {
        if (!c->free_events.empty()) {
            hipEvent_t e = c->free_events.back();
            c->free_events.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    Prof(qtale_ctx* c, hipStream_t s, int k) : ctx(c), stream(s), cls(k), on(c->profiling) {
        if (!on) return;
        a = get(c);
        b = get(c);
        if (!a || !b) { on = false; return; }
        (void)hipEventRecord(a, stream);
    }
    ~Prof() {
        if (!on) return;
        (void)hipEventRecord(b, stream);
        ctx->spans.push_back({cls, a, b});
    }
};

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return QTALE_ERR_HIP;    \
    } while (0)

// How a layer call is linked to its neighbours inside a stack (decode-sized calls only): the previous layer's last
// kernel may already have written this layer's scores, and this layer's last kernel may write the next layer's.
struct LayerLink {
    bool scores_ready = false;                  // in: z of this layer is already in place
    const qtale_layer_weights* next = nullptr;  // in: the next layer, or null
    float* next_z = nullptr;                    // in: where its scores go
    bool next_scored = false;                   // out: they were written
};

int layer_forward_impl(qtale_ctx* ctx, const qtale_layer_cfg* c, const qtale_layer_weights* w, void* x, int T,
                       const int32_t* seq_offsets, int B, const int32_t* positions, const qtale_kv* kv,
                       int32_t* sel_idx, int32_t* sel_count, float* scores, const Workspace& ws,
                       hipStream_t stream, LayerLink* link = nullptr) {
    const int bf16 = c->act_dtype == QTALE_ACT_BF16;
    const int H = c->hidden, nh = c->n_heads, nkv = c->n_kv_heads, d = c->head_dim, I = c->inter;
    const int ratio_mode = ctx->mode == QTALE_MODE_RATIO;
    const int lbits = w->bits ? w->bits : c->bits;     // per-layer code width (mixed-precision stacks)
    const int k = ratio_mode ? executed_count(ctx->value, T) : 0;
    const int M_max = ratio_mode ? k : T;
    float* z = scores ? scores : ws.z;
    int32_t* count = ws.scalars;

    SelectArgs s{};
    s.z = z; s.T = T; s.mode = ratio_mode ? 0 : 1; s.k = k;
    s.z_thr = ratio_mode ? 0.0f : theta_to_logit(ctx->value);
    s.seq_offsets = seq_offsets; s.B = B;
    s.idx = ws.idx; s.count = count; s.cu_exec = ws.cu_exec; s.row_seq = ws.row_seq;
    s.kv_len = kv ? kv->kv_len : nullptr; s.kv_old = ws.kv_old; s.kv_cap = kv ? kv->cap : 0;
    s.idx_copy = sel_idx; s.count_copy = sel_count;
    if (!(link && link->scores_ready)) {
        Prof pr(ctx, stream, 0);
        if (w->router_hidden > 0)
            HIP_TRY(launch_router_mlp(x, bf16, T, H, w->router_w1, w->router_b1, w->router_w2, w->router_b2,
                                      w->router_hidden, z, stream));
        else
            HIP_TRY(launch_router_score(x, bf16, T, H, w->router_w, w->router_b, z, stream));
    }
    const bool small_call = fused_select_norm_fits(T, M_max);
    if (small_call) {
        // decode-sized call: decision, compaction and gather + RMSNorm 1 in one launch
        s.inv = ws.inv;
        Prof pr(ctx, stream, 1);
        HIP_TRY(launch_select_norm(x, bf16, H, z, w->norm1, c->rms_eps, ws.nbuf, s, M_max, stream));
    } else {
        {
            Prof pr(ctx, stream, 1);
            HIP_TRY(launch_select(s, stream));
        }
        if (M_max == 0) return QTALE_OK;
        {
            Prof pr(ctx, stream, 2);
            HIP_TRY(launch_gather_rmsnorm(x, bf16, H, ws.idx, count, M_max, w->norm1, c->rms_eps, ws.nbuf, stream));
        }
    }
    const int qkv_w = (nh + 2 * nkv) * d;
    int o_parts = 0;
    {
        Prof pr(ctx, stream, 3);
        GemmArgs g{};
        g.A = ws.nbuf; g.count = count; g.M_max = M_max; g.rows_exact = ratio_mode; g.K = H; g.group = c->group; g.bits = lbits; g.n_w = 3;
        g.w[0] = {w->q.prepacked, w->q.N, w->q.K};
        g.w[1] = {w->k.prepacked, w->k.N, w->k.K};
        g.w[2] = {w->v.prepacked, w->v.N, w->v.K};
        g.epilogue = EPI_STORE_F16; g.out = ws.qkv; g.ldo = qkv_w;
        HIP_TRY(launch_gemm_w4a16(g, stream));
    }
    {
        Prof pr(ctx, stream, 4);
        RopeArgs r{};
        r.qkv = ws.qkv; r.nh = nh; r.nkv = nkv; r.d = d; r.base = c->rope_base;
        r.idx = ws.idx; r.positions = positions; r.count = count; r.max_rows = M_max;
        if (kv) { r.k_cache = kv->k_cache; r.v_cache = kv->v_cache; r.cap = kv->cap; }
        r.row_seq = ws.row_seq; r.cu_exec = ws.cu_exec; r.kv_old = ws.kv_old;
        HIP_TRY(launch_rope_append(r, stream));
    }
    {
        Prof pr(ctx, stream, 5);
        AttnArgs a{};
        a.qkv = ws.qkv; a.out = ws.attn; a.nh = nh; a.nkv = nkv; a.d = d; a.count = count; a.max_rows = M_max;
        a.B = B; a.cu_exec = ws.cu_exec; a.row_seq = ws.row_seq;
        if (kv) { a.k_cache = kv->k_cache; a.v_cache = kv->v_cache; a.cap = kv->cap; }
        a.kv_old = ws.kv_old; a.T = T; a.items = ws.items; a.n_items = ws.scalars + 1; a.partials = ws.attn_part;
        HIP_TRY(launch_attention(a, stream));
    }
    {
        Prof pr(ctx, stream, 6);
        GemmArgs g{};
        g.A = ws.attn; g.count = count; g.M_max = M_max; g.rows_exact = ratio_mode; g.K = nh * d; g.group = c->group; g.bits = lbits; g.n_w = 1;
        g.w[0] = {w->o.prepacked, w->o.N, w->o.K};
        g.epilogue = EPI_RESID_F32; g.out = ws.h; g.ldo = H; g.resid = x; g.idx = ws.idx; g.bf16 = bf16;
        g.part = M_max <= kGemmPartRows ? ws.gemm_part : nullptr; g.n_parts = &o_parts;
        HIP_TRY(launch_gemm_w4a16(g, stream));
    }
    {
        Prof pr(ctx, stream, 7);
        if (o_parts > 0)       // the o-proj left K-part partial tiles: add them and the residual here
            HIP_TRY(launch_reduce_rmsnorm(ws.gemm_part, o_parts, x, bf16, ws.idx, H, count, M_max, w->norm2, c->rms_eps,
                                          ws.h, ws.nbuf, stream));
        else
            HIP_TRY(launch_rmsnorm_f32(ws.h, H, count, M_max, w->norm2, bf16, c->rms_eps, ws.nbuf, stream));
    }
    {
        Prof pr(ctx, stream, 8);
        GemmArgs g{};
        g.A = ws.nbuf; g.count = count; g.M_max = M_max; g.rows_exact = ratio_mode; g.K = H; g.group = c->group; g.bits = lbits; g.n_w = 2;
        g.w[0] = {w->gate.prepacked, w->gate.N, w->gate.K};
        g.w[1] = {w->up.prepacked, w->up.N, w->up.K};
        g.epilogue = EPI_SWIGLU_F16; g.out = ws.act; g.ldo = I;
        HIP_TRY(launch_gemm_w4a16(g, stream));
    }
    {
        Prof pr(ctx, stream, 9);
        GemmArgs g{};
        g.A = ws.act; g.count = count; g.M_max = M_max; g.rows_exact = ratio_mode; g.K = I; g.group = c->group; g.bits = lbits; g.n_w = 1;
        g.w[0] = {w->down.prepacked, w->down.N, w->down.K};
        g.epilogue = EPI_RESID_SCATTER; g.out = x; g.ldo = H; g.resid = ws.h; g.idx = ws.idx; g.bf16 = bf16;
        int d_parts = 0;
        g.part = M_max <= kGemmPartRows ? ws.gemm_part : nullptr; g.n_parts = &d_parts;
        HIP_TRY(launch_gemm_w4a16(g, stream));
        if (d_parts > 0) {
            if (link && link->next && link->next->router_hidden == 0 && small_call) {
                HIP_TRY(launch_reduce_scatter_score(ws.gemm_part, d_parts, M_max, ws.h, H, ws.inv, T, x, bf16,
                                                    link->next->router_w, link->next->router_b, link->next_z, stream));
                link->next_scored = true;
            } else {
                HIP_TRY(launch_reduce_scatter(ws.gemm_part, d_parts, ws.h, H, ws.idx, count, M_max, x, bf16, stream));
            }
        }
    }
    return QTALE_OK;
}

int check_forward_args(qtale_ctx* ctx, const qtale_layer_cfg* cfg, void* x, int T, const int32_t* seq_offsets,
                       int B, const int32_t* positions, void* workspace, size_t workspace_bytes) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    int e = check_cfg(cfg);
    if (e) return e;
    if (T < 0 || B < 0) return QTALE_ERR_INVALID_ARG;
    if (T == 0) return QTALE_OK;
    if (!x || !seq_offsets || !positions || B == 0) return QTALE_ERR_INVALID_ARG;
    if (!workspace) return QTALE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return QTALE_ERR_INVALID_ARG;
    if (workspace_bytes < carve(cfg, T, B, nullptr).total) return QTALE_ERR_WORKSPACE_TOO_SMALL;
    return QTALE_OK;
}

int check_kv(const qtale_kv* kv) {
    if (!kv) return QTALE_OK;
    if (!kv->k_cache || !kv->v_cache || !kv->kv_len || kv->cap <= 0) return QTALE_ERR_INVALID_ARG;
    return QTALE_OK;
}

}  // namespace

// ---- threshold calibration helpers (Sec. 3.4) --------------------------------------------------------------
namespace {

float theta_grid(int n) { return static_cast<float>(n / 100.0); }

// Coarse pass n = 5, 10, ..., 50, then the unevaluated n within 4 steps of the best coarse point; the answer is
// the evaluated n with the smallest |R - target|, the larger theta on ties.  table[n] (n = 1..50) keeps every
// evaluated ratio, NaN elsewhere.  eval(n, &ratio) returns a QTALE status.
template <class Eval>
int two_phase_search(Eval&& eval, double target, double* table, int* best_n) {
    for (int n = 0; n <= kThetaGrid; ++n) table[n] = std::nan("");
    auto pick = [&]() {
        int b = -1;
        double bd = INFINITY;
        for (int n = 1; n <= kThetaGrid; ++n) {
            if (std::isnan(table[n])) continue;
            const double d = std::fabs(table[n] - target);
            if (d <= bd) { b = n; bd = d; }
        }
        return b;
    };
    int e;
    for (int n = 5; n <= kThetaGrid; n += 5)
        if ((e = eval(n, &table[n]))) return e;
    const int c = pick();
    for (int n = std::max(1, c - 4); n <= std::min(kThetaGrid, c + 4); ++n)
        if (std::isnan(table[n]) && (e = eval(n, &table[n]))) return e;
    *best_n = pick();
    return QTALE_OK;
}

int finish_calibration(qtale_ctx* ctx, const double* table, int best, float* theta, float* ratio, float* table_out) {
    ctx->mode = QTALE_MODE_THRESHOLD;
    ctx->value = theta_grid(best);
    if (theta) *theta = ctx->value;
    if (ratio) *ratio = static_cast<float>(table[best]);
    if (table_out)
        for (int n = 1; n <= kThetaGrid; ++n) table_out[n - 1] = static_cast<float>(table[n]);
    return QTALE_OK;
}

}  // namespace

extern "C" {

const char* qtale_strerror(int code) {
    switch (code) {
        case QTALE_OK: return "ok";
        case QTALE_ERR_INVALID_ARG: return "invalid argument";
        case QTALE_ERR_SHAPE: return "inconsistent or unsupported shape";
        case QTALE_ERR_UNSUPPORTED: return "unsupported bits / group / head_dim / dtype";
        case QTALE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case QTALE_ERR_HIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

int qtale_create(qtale_ctx** out) {
    if (!out) return QTALE_ERR_INVALID_ARG;
    *out = new (std::nothrow) qtale_ctx();
    return *out ? QTALE_OK : QTALE_ERR_INVALID_ARG;
}

int qtale_destroy(qtale_ctx* ctx) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    for (auto& s : ctx->spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
    for (auto e : ctx->free_events) (void)hipEventDestroy(e);
    delete ctx;
    return QTALE_OK;
}

int qtale_set_exec_ratio(qtale_ctx* ctx, float r) {
    if (!ctx || std::isnan(r) || r < 0.0f || r > 1.0f) return QTALE_ERR_INVALID_ARG;
    ctx->mode = QTALE_MODE_RATIO;
    ctx->value = r;
    return QTALE_OK;
}

int qtale_set_threshold(qtale_ctx* ctx, float theta) {
    if (!ctx || std::isnan(theta)) return QTALE_ERR_INVALID_ARG;
    ctx->mode = QTALE_MODE_THRESHOLD;
    ctx->value = theta;
    return QTALE_OK;
}

int qtale_get_control(const qtale_ctx* ctx, int* mode, float* value) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    if (mode) *mode = ctx->mode;
    if (value) *value = ctx->value;
    return QTALE_OK;
}

size_t qtale_prepacked_bytes(int N, int K, int bits, int group) {
    if (check_quant_params(N, K, bits, group) != QTALE_OK) return 0;
    const PrepackDims d = prepack_dims(N, K, group, bits);
    return d.code_bytes + d.sz_bytes;
}

int qtale_quantize(const float* W, int N, int K, int bits, int group, uint32_t* codes, uint16_t* scales,
                   uint16_t* zeros, void* prepacked, void* stream) {
    const int e = check_quant_params(N, K, bits, group);
    if (e) return e;
    if (!W || !codes || !scales || !zeros) return QTALE_ERR_INVALID_ARG;
    if (prepacked && reinterpret_cast<uintptr_t>(prepacked) % 16 != 0) return QTALE_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    HIP_TRY(launch_quantize(W, N, K, bits, group, codes, scales, zeros, s));
    if (prepacked) HIP_TRY(launch_prepack(codes, scales, zeros, N, K, bits, group, prepacked, s));
    return QTALE_OK;
}

int qtale_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros, int N, int K, int bits,
                  int group, void* prepacked, void* stream) {
    const int e = check_quant_params(N, K, bits, group);
    if (e) return e;
    if (!codes || !scales || !zeros || !prepacked) return QTALE_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(prepacked) % 16 != 0) return QTALE_ERR_INVALID_ARG;
    HIP_TRY(launch_prepack(codes, scales, zeros, N, K, bits, group, prepacked, reinterpret_cast<hipStream_t>(stream)));
    return QTALE_OK;
}

size_t qtale_workspace_bytes(const qtale_layer_cfg* cfg, int max_tokens, int max_seqs) {
    if (check_cfg(cfg) != QTALE_OK || max_tokens < 0 || max_seqs < 0) return 0;
    return carve(cfg, max_tokens, max_seqs, nullptr).total;
}

int qtale_layer_forward(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* w, void* x, int T,
                        const int32_t* seq_offsets, int B, const int32_t* positions, const qtale_kv* kv,
                        int32_t* sel_idx, int32_t* sel_count, float* scores, void* workspace,
                        size_t workspace_bytes, void* stream) {
    int e = check_forward_args(ctx, cfg, x, T, seq_offsets, B, positions, workspace, workspace_bytes);
    if (e) return e;
    if (T == 0) return QTALE_OK;
    if ((e = check_weights(cfg, w))) return e;
    if ((e = check_kv(kv))) return e;
    const Workspace ws = carve(cfg, T, B, workspace);
    return layer_forward_impl(ctx, cfg, w, x, T, seq_offsets, B, positions, kv, sel_idx, sel_count, scores, ws,
                              reinterpret_cast<hipStream_t>(stream));
}

// ---- layer forward on the library's own scratch array (for callers that cannot allocate) ------------------
// The workspace of qtale_layer_forward lives in a file-scope device array instead of a caller buffer.  In host
// code the array's name is only a handle: its device address is looked up once per device with
// hipGetSymbolAddress (every GPU holds its own copy at its own address) and that pointer is what the kernels get.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(QTALE_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (resolved on the first call per device).
int static_scratch(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return QTALE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0) return QTALE_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return QTALE_OK;
}
}  // namespace

size_t qtale_static_scratch_bytes(void) { return kStaticScratchBytes; }

int qtale_layer_forward_static(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* w, void* x, int T,
                               const int32_t* seq_offsets, int B, const int32_t* positions, const qtale_kv* kv,
                               int32_t* sel_idx, int32_t* sel_count, float* scores, void* stream) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    int e = check_cfg(cfg);
    if (e) return e;
    if (T < 0 || B < 0) return QTALE_ERR_INVALID_ARG;
    if (T == 0) return QTALE_OK;
    if (!x || !seq_offsets || !positions || B == 0) return QTALE_ERR_INVALID_ARG;
    if (ctx->profiling) return QTALE_ERR_INVALID_ARG;          // the per-kernel timer creates events
    if (carve(cfg, T, B, nullptr).total > kStaticScratchBytes) return QTALE_ERR_WORKSPACE_TOO_SMALL;
    if ((e = check_weights(cfg, w))) return e;
    if ((e = check_kv(kv))) return e;
    void* base = nullptr;
    if ((e = static_scratch(&base))) return e;
    // Nothing in the workspace has to start at zero: every kernel of the layer writes what it later reads.
    const Workspace ws = carve(cfg, T, B, base);
    return layer_forward_impl(ctx, cfg, w, x, T, seq_offsets, B, positions, kv, sel_idx, sel_count, scores, ws,
                              reinterpret_cast<hipStream_t>(stream));
}

int qtale_stack_forward(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                        int n_layers, void* x, int T, const int32_t* seq_offsets, int B, const int32_t* positions,
                        const qtale_kv* kv_per_layer, int32_t* sel_idx, int32_t* sel_count, float* scores,
                        void* dbg_hidden, void* workspace, size_t workspace_bytes, void* stream) {
    int e = check_forward_args(ctx, cfg, x, T, seq_offsets, B, positions, workspace, workspace_bytes);
    if (e) return e;
    if (n_layers < 0 || (n_layers > 0 && !layers)) return QTALE_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        if ((e = check_weights(cfg, &layers[l]))) return e;
        if (kv_per_layer && (e = check_kv(&kv_per_layer[l]))) return e;
    }
    if (T == 0) return QTALE_OK;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const Workspace ws = carve(cfg, T, B, workspace);
    const size_t row_bytes = static_cast<size_t>(cfg->hidden) * 2;
    bool scores_ready = false;
    for (int l = 0; l < n_layers; ++l) {
        if (dbg_hidden) {
            HIP_TRY(hipMemcpyAsync(reinterpret_cast<char*>(dbg_hidden) + static_cast<size_t>(l) * T * row_bytes, x,
                                   static_cast<size_t>(T) * row_bytes, hipMemcpyDeviceToDevice, s));
        }
        LayerLink link;
        link.scores_ready = scores_ready;
        if (l + 1 < n_layers) {
            link.next = &layers[l + 1];
            link.next_z = scores ? scores + static_cast<size_t>(l + 1) * T : ws.z;
        }
        e = layer_forward_impl(ctx, cfg, &layers[l], x, T, seq_offsets, B, positions,
                               kv_per_layer ? &kv_per_layer[l] : nullptr,
                               sel_idx ? sel_idx + static_cast<size_t>(l) * T : nullptr,
                               sel_count ? sel_count + l : nullptr,
                               scores ? scores + static_cast<size_t>(l) * T : nullptr, ws, s, &link);
        if (e) return e;
        scores_ready = link.next_scored;
    }
    return QTALE_OK;
}

int qtale_router_select(qtale_ctx* ctx, int act_dtype, const void* x, int T, int hidden, const float* router_w,
                        float router_b, const int32_t* seq_offsets, int B, float* scores, int32_t* sel_idx,
                        int32_t* sel_count, int32_t* cu_exec, void* stream) {
    if (!ctx || T < 0 || B < 0 || hidden <= 0) return QTALE_ERR_INVALID_ARG;
    if (act_dtype != QTALE_ACT_FP16 && act_dtype != QTALE_ACT_BF16) return QTALE_ERR_UNSUPPORTED;
    if (hidden % 8 != 0) return QTALE_ERR_SHAPE;
    if (std::isnan(router_b)) return QTALE_ERR_INVALID_ARG;
    if (T == 0) return QTALE_OK;
    if (!x || !router_w || !scores || !sel_idx || !sel_count) return QTALE_ERR_INVALID_ARG;
    if (cu_exec && (!seq_offsets || B == 0)) return QTALE_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    HIP_TRY(launch_router_score(x, act_dtype == QTALE_ACT_BF16, T, hidden, router_w, router_b, scores, s));
    SelectArgs a{};
    a.z = scores; a.T = T;
    a.mode = ctx->mode == QTALE_MODE_RATIO ? 0 : 1;
    a.k = ctx->mode == QTALE_MODE_RATIO ? executed_count(ctx->value, T) : 0;
    a.z_thr = ctx->mode == QTALE_MODE_RATIO ? 0.0f : theta_to_logit(ctx->value);
    a.seq_offsets = seq_offsets; a.B = cu_exec ? B : 0;
    a.idx = sel_idx; a.count = sel_count; a.cu_exec = cu_exec;
    if (!cu_exec) a.B = -1;            // skip the per-sequence tail entirely
    HIP_TRY(launch_select(a, s));
    return QTALE_OK;
}

// ---- threshold calibration (Sec. 3.4) --------------------------------------------------------------------
size_t qtale_calibration_scratch_bytes(int n_layers) {
    if (n_layers < 0) return 0;
    return 1024 + static_cast<size_t>(n_layers) * 4;
}

int qtale_calibrate_threshold_from_scores(qtale_ctx* ctx, const float* scores, int64_t n, float target_ratio,
                                          void* scratch, float* theta, float* ratio, float* table_out, void* stream) {
    if (!ctx || n < 0 || !(target_ratio >= 0.0f && target_ratio <= 1.0f)) return QTALE_ERR_INVALID_ARG;
    if (n == 0 || !scores || !scratch) return QTALE_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned long long* bins = reinterpret_cast<unsigned long long*>(scratch);
    float* zthr_dev = reinterpret_cast<float*>(reinterpret_cast<char*>(scratch) + 512);
    float zthr[kThetaGrid];
    for (int j = 0; j < kThetaGrid; ++j) zthr[j] = theta_to_logit(theta_grid(j + 1));
    HIP_TRY(hipMemcpyAsync(zthr_dev, zthr, sizeof(zthr), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));                  // zthr is a stack array: the copy must have left it
    HIP_TRY(launch_threshold_bins(scores, static_cast<long>(n), zthr_dev, bins, s));
    unsigned long long host_bins[kThetaGrid + 1];
    HIP_TRY(hipMemcpyAsync(host_bins, bins, sizeof(host_bins), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    // a score in bin b reaches thresholds 1..b: count(theta_j) = sum of bins j..50
    unsigned long long reach[kThetaGrid + 2];
    reach[kThetaGrid + 1] = 0;
    for (int j = kThetaGrid; j >= 1; --j) reach[j] = reach[j + 1] + host_bins[j];
    double table[kThetaGrid + 1];
    int best = -1;
    const int e = two_phase_search(
        [&](int j, double* r) {
            *r = static_cast<double>(reach[j]) / static_cast<double>(n);
            return QTALE_OK;
        },
        static_cast<double>(target_ratio), table, &best);
    if (e) return e;
    return finish_calibration(ctx, table, best, theta, ratio, table_out);
}

int qtale_calibrate_threshold(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                              int n_layers, const void* x_calib, void* x_work, int T, const int32_t* seq_offsets,
                              int B, const int32_t* positions, float target_ratio, void* scratch, void* workspace,
                              size_t workspace_bytes, float* theta, float* ratio, float* table_out, void* stream) {
    if (!(target_ratio >= 0.0f && target_ratio <= 1.0f)) return QTALE_ERR_INVALID_ARG;
    int e = check_forward_args(ctx, cfg, x_work, T, seq_offsets, B, positions, workspace, workspace_bytes);
    if (e) return e;
    if (n_layers <= 0 || !layers || T <= 0 || !x_calib || !scratch) return QTALE_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l)
        if ((e = check_weights(cfg, &layers[l]))) return e;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    int32_t* counts_dev = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(scratch) + 1024);
    std::vector<int32_t> counts(static_cast<size_t>(n_layers));
    const size_t x_bytes = static_cast<size_t>(T) * cfg->hidden * 2;
    const int saved_mode = ctx->mode;
    const float saved_value = ctx->value;
    const bool saved_prof = ctx->profiling;
    ctx->profiling = false;
    double table[kThetaGrid + 1];
    int best = -1;
    e = two_phase_search(
        [&](int n, double* r) {
            ctx->mode = QTALE_MODE_THRESHOLD;
            ctx->value = theta_grid(n);
            if (hipMemcpyAsync(x_work, x_calib, x_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) return (int)QTALE_ERR_HIP;
            const int st = qtale_stack_forward(ctx, cfg, layers, n_layers, x_work, T, seq_offsets, B, positions, nullptr,
                                               nullptr, counts_dev, nullptr, nullptr, workspace, workspace_bytes, stream);
            if (st) return st;
            if (hipMemcpyAsync(counts.data(), counts_dev, counts.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess) return (int)QTALE_ERR_HIP;
            if (hipStreamSynchronize(s) != hipSuccess) return (int)QTALE_ERR_HIP;
            long total = 0;
            for (int32_t c : counts) total += c;
            *r = static_cast<double>(total) / (static_cast<double>(n_layers) * static_cast<double>(T));
            return (int)QTALE_OK;
        },
        static_cast<double>(target_ratio), table, &best);
    ctx->profiling = saved_prof;
    if (e) {
        ctx->mode = saved_mode;
        ctx->value = saved_value;
        return e;
    }
    return finish_calibration(ctx, table, best, theta, ratio, table_out);
}

int qtale_router_mlp_scores(int act_dtype, const void* x, int T, int hidden, const float* w1, const float* b1,
                            const float* w2, const float* b2, int router_hidden, float* scores, void* stream) {
    if (T < 0 || hidden <= 0 || router_hidden <= 0 || router_hidden > 256) return QTALE_ERR_INVALID_ARG;
    if (act_dtype != QTALE_ACT_FP16 && act_dtype != QTALE_ACT_BF16) return QTALE_ERR_UNSUPPORTED;
    if (hidden % 8 != 0) return QTALE_ERR_SHAPE;
    if (T == 0) return QTALE_OK;
    if (!x || !w1 || !b1 || !w2 || !b2 || !scores) return QTALE_ERR_INVALID_ARG;
    HIP_TRY(launch_router_mlp(x, act_dtype == QTALE_ACT_BF16, T, hidden, w1, b1, w2, b2, router_hidden, scores,
                              reinterpret_cast<hipStream_t>(stream)));
    return QTALE_OK;
}

int qtale_linear_w4a16(const qtale_qlinear* w, int bits, int group, const void* A, int M, void* out, void* stream) {
    if (!w || M < 0) return QTALE_ERR_INVALID_ARG;
    int e = check_quant_params(w->N, w->K, bits, group);
    if (e) return e;
    if (w->N % 8 != 0) return QTALE_ERR_SHAPE;
    if (M == 0) return QTALE_OK;
    if (!w->prepacked || !A || !out) return QTALE_ERR_INVALID_ARG;
    GemmArgs g{};
    g.A = A; g.M_max = M; g.rows_exact = 1; g.K = w->K; g.group = group; g.bits = bits; g.n_w = 1;
    g.w[0] = {w->prepacked, w->N, w->K};
    g.epilogue = EPI_STORE_F16; g.out = out; g.ldo = w->N;
    HIP_TRY(launch_gemm_w4a16(g, reinterpret_cast<hipStream_t>(stream)));
    return QTALE_OK;
}

int qtale_swiglu_w4a16(const qtale_qlinear* gate, const qtale_qlinear* up, int bits, int group, const void* A, int M,
                       void* out, void* stream) {
    if (!gate || !up || M < 0) return QTALE_ERR_INVALID_ARG;
    int e = check_quant_params(gate->N, gate->K, bits, group);
    if (e) return e;
    if (gate->N != up->N || gate->K != up->K || gate->N % 8 != 0) return QTALE_ERR_SHAPE;
    if (M == 0) return QTALE_OK;
    if (!gate->prepacked || !up->prepacked || !A || !out) return QTALE_ERR_INVALID_ARG;
    GemmArgs g{};
    g.A = A; g.M_max = M; g.rows_exact = 1; g.K = gate->K; g.group = group; g.bits = bits; g.n_w = 2;
    g.w[0] = {gate->prepacked, gate->N, gate->K};
    g.w[1] = {up->prepacked, up->N, up->K};
    g.epilogue = EPI_SWIGLU_F16; g.out = out; g.ldo = gate->N;
    HIP_TRY(launch_gemm_w4a16(g, reinterpret_cast<hipStream_t>(stream)));
    return QTALE_OK;
}

// ---- HIP graph of one stack forward ---------------------------------------------------------------------------
struct qtale_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipStream_t capture_stream = nullptr;
};

void qtale_graph_destroy(qtale_graph* g) {
    if (!g) return;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    if (g->capture_stream) (void)hipStreamDestroy(g->capture_stream);
    delete g;
}

int qtale_graph_capture_stack(qtale_ctx* ctx, const qtale_layer_cfg* cfg, const qtale_layer_weights* layers,
                              int n_layers, void* x, int T, const int32_t* seq_offsets, int B,
                              const int32_t* positions, const qtale_kv* kv_per_layer, int32_t* sel_idx,
                              int32_t* sel_count, float* scores, void* workspace, size_t workspace_bytes,
                              qtale_graph** out) {
    if (!out) return QTALE_ERR_INVALID_ARG;
    *out = nullptr;
    if (!ctx || ctx->profiling) return QTALE_ERR_INVALID_ARG;       // event spans cannot be recorded into a graph
    // validate everything before capture starts, so that a failing call never leaves a capture open
    int e = check_forward_args(ctx, cfg, x, T, seq_offsets, B, positions, workspace, workspace_bytes);
    if (e) return e;
    if (n_layers <= 0 || !layers || T <= 0) return QTALE_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        if ((e = check_weights(cfg, &layers[l]))) return e;
        if (kv_per_layer && (e = check_kv(&kv_per_layer[l]))) return e;
    }
    qtale_graph* g = new (std::nothrow) qtale_graph();
    if (!g) return QTALE_ERR_HIP;
    if (hipStreamCreateWithFlags(&g->capture_stream, hipStreamNonBlocking) != hipSuccess) {
        qtale_graph_destroy(g);
        return QTALE_ERR_HIP;
    }
    if (hipStreamBeginCapture(g->capture_stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
        qtale_graph_destroy(g);
        return QTALE_ERR_HIP;
    }
    e = qtale_stack_forward(ctx, cfg, layers, n_layers, x, T, seq_offsets, B, positions, kv_per_layer, sel_idx,
                            sel_count, scores, nullptr, workspace, workspace_bytes, g->capture_stream);
    const hipError_t he = hipStreamEndCapture(g->capture_stream, &g->graph);   // always close the capture
    if (e || he != hipSuccess || !g->graph) {
        qtale_graph_destroy(g);
        return e ? e : QTALE_ERR_HIP;
    }
    if (hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0) != hipSuccess) {
        qtale_graph_destroy(g);
        return QTALE_ERR_HIP;
    }
    *out = g;
    return QTALE_OK;
}

int qtale_graph_launch(qtale_graph* g, void* stream) {
    if (!g || !g->exec) return QTALE_ERR_INVALID_ARG;
    HIP_TRY(hipGraphLaunch(g->exec, reinterpret_cast<hipStream_t>(stream)));
    return QTALE_OK;
}

int qtale_profile_enable(qtale_ctx* ctx, int on) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    ctx->profiling = on != 0;
    return QTALE_OK;
}

int qtale_profile_read(qtale_ctx* ctx, double* ms, int64_t* launches) {
    if (!ctx) return QTALE_ERR_INVALID_ARG;
    for (auto& s : ctx->spans) {
        float t = 0.0f;
        if (hipEventSynchronize(s.b) != hipSuccess) return QTALE_ERR_HIP;
        if (hipEventElapsedTime(&t, s.a, s.b) != hipSuccess) return QTALE_ERR_HIP;
        ctx->ms[s.cls] += t;
        ctx->launches[s.cls] += 1;
        ctx->free_events.push_back(s.a);
        ctx->free_events.push_back(s.b);
    }
    ctx->spans.clear();
    for (int i = 0; i < QTALE_PROF_CLASSES; ++i) {
        if (ms) ms[i] = ctx->ms[i];
        if (launches) launches[i] = ctx->launches[i];
        ctx->ms[i] = 0.0;
        ctx->launches[i] = 0;
    }
    return QTALE_OK;
}

}  // extern "C"
