// C ABI of the MoE hot path: argument checks, workspace carving and the layer-group driver
// for the chunked (Sec. 2.3) and layered (Sec. 4.1-4.2) prefill schedules.  All arithmetic
// happens in the kernels of router.hip / permute.hip / ffn.hip / combine.hip.
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "common.h"

using namespace moe;

struct moe_ctx {
    moe_config cfg;
    int64_t max_tokens;
    int esz;  // bytes per element
    // workspace slices (device)
    unsigned long long* d_active_total;
    double* logits;
    int32_t *idx, *counts, *offsets, *perm, *inv, *tile_hist;
    float* w;
    void *xa, *xb, *act, *y_perm;
    // host-side counters (everything the host already knows)
    uint64_t router_bytes, tokens_processed;
    uint32_t iterations, layer_passes;
    int ffn_variant;   // moe_ffn_variant_id pinned by moe_set_ffn_variant (MOE_FFN_AUTO: the library's rule)
    // benchmark aid: HIP event pairs around the launches of the kernels selected by timing_mask; pairs are
    // recycled through event_pool, so that steady-state timing creates no events
    uint32_t timing_mask;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> timing[MOE_KERNEL_COUNT];
    std::vector<std::pair<hipEvent_t, hipEvent_t>> event_pool;
};

// Scratch of moe_router_topk_noalloc: the fp64 logits [T, E] of one call.  One copy per GPU, held until the
// process ends; in host code the name below is only a handle for hipGetSymbolAddress, never an address.
constexpr int64_t kNoallocMaxLogits = (int64_t)1 << 19;      // T * E <= 524288: 4 MiB of logits
static __device__ __align__(256) double scratch[kNoallocMaxLogits];

namespace {

constexpr size_t kAlign = 256;
inline size_t up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

moe_status check_cfg(const moe_config* c)
{
    if (!c) return MOE_ERR_NULL;
    if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (c->H <= 0 || c->I <= 0 || c->E <= 0 || c->E > kMaxExperts || c->K <= 0 || c->K > c->E || c->K > kMaxTopK)
        return MOE_ERR_SHAPE;
    if (c->H % 8 || c->I % 8) return MOE_ERR_ALIGN;
    if (c->weight_format != MOE_W_DTYPE && c->weight_format != MOE_W_MXFP4) return MOE_ERR_DTYPE;
    if (c->y_perm_f32 != 0 && c->y_perm_f32 != 1) return MOE_ERR_DTYPE;
    if (c->act_split != 0 && c->act_split != 1) return MOE_ERR_DTYPE;
    // a split intermediate: bf16 contexts with bf16 weights and fp32 expert outputs only
    if (c->act_split && (c->dtype != MOE_BF16 || c->weight_format != MOE_W_DTYPE || !c->y_perm_f32)) return MOE_ERR_DTYPE;
    if (c->weight_format == MOE_W_MXFP4) {
        if (c->dtype != MOE_BF16) return MOE_ERR_DTYPE;
        if (c->H % 64 || c->I % 64) return MOE_ERR_ALIGN;
    }
    return MOE_OK;
}

struct Layout {
    size_t counters, logits, idx, w, counts, offsets, perm, inv, tile_hist, xa, xb, act, y_perm, total;
};

Layout carve(const moe_config& c, int64_t Tm)
{
    const size_t esz = c.dtype == MOE_BF16 ? 2 : 4;
    const size_t Am = (size_t)Tm * c.K;
    const size_t n_tiles = (Am + kPermTile - 1) / kPermTile + 1;
    Layout L;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up(bytes); return at; };
    L.counters = take(256);
    L.logits = take((size_t)Tm * c.E * sizeof(double));
    L.idx = take(Am * 4);
    L.w = take(Am * 4);
    L.counts = take((size_t)c.E * 4);
    L.offsets = take((size_t)(c.E + 1) * 4);
    L.perm = take(Am * 4);
    L.inv = take(Am * 4);
    L.tile_hist = take(n_tiles * c.E * 4);
    L.xa = take((size_t)Tm * c.H * esz);
    L.xb = take((size_t)Tm * c.H * esz);
    L.act = take(Am * c.I * esz * (c.act_split ? 2 : 1));
    L.y_perm = take(Am * c.H * (c.y_perm_f32 ? 4 : esz));
    L.total = o;
    return L;
}

// Records an event before and after one launch when that kernel is being timed.  At most kMaxTimed
// launches per kernel are kept between two reads; later ones go untimed (the mean stays a mean).
constexpr size_t kMaxTimed = 1 << 16;
struct Timed {
    moe_ctx* c; int id; hipStream_t s; bool on; hipEvent_t e0, e1;
    Timed(moe_ctx* c_, int id_, hipStream_t s_) : c(c_), id(id_), s(s_), on(false), e0(nullptr), e1(nullptr)
    {
        if (!(c->timing_mask & (1u << id)) || c->timing[id].size() >= kMaxTimed) return;
        if (!c->event_pool.empty()) {
            e0 = c->event_pool.back().first;
            e1 = c->event_pool.back().second;
            c->event_pool.pop_back();
        } else {
            if (hipEventCreate(&e0) != hipSuccess) { e0 = nullptr; return; }
            if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); e0 = e1 = nullptr; return; }
        }
        on = hipEventRecord(e0, s) == hipSuccess;
    }
    ~Timed()
    {
        if (!e1) return;
        if (on && hipEventRecord(e1, s) == hipSuccess) c->timing[id].emplace_back(e0, e1);
        else c->event_pool.emplace_back(e0, e1);
    }
};

// Forget the recorded launches; their events go back to the pool (or are destroyed with the context).
void drop_timing(moe_ctx* c, bool destroy)
{
    for (auto& v : c->timing) {
        for (auto& p : v) c->event_pool.push_back(p);
        v.clear();
    }
    if (destroy) {
        for (auto& p : c->event_pool) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
        c->event_pool.clear();
    }
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
// the packed codes of MXFP4 weights: rows must start a multiple of 32 bytes into a 128-byte line
inline bool misaligned32(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 31u) != 0; }
inline moe_status dev(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE; }

// One layer on the batch `x` [T,H]; output rows [0,rows0) -> y0, the rest -> y1.
moe_status run_layer(moe_ctx* c, const moe_layer& L, RowSrc x, int64_t T, void* y0, int64_t rows0, void* y1,
                     hipStream_t s)
{
    const moe_config& g = c->cfg;
    const int64_t A = T * g.K;
    // with more than one permutation tile the top-k kernel counts the per-tile expert histograms itself
    const int n_perm_tiles = (int)((A + kPermTile - 1) / kPermTile);
    const bool fused_hist = n_perm_tiles > 1;
    hipError_t e;
    {
        Timed t(c, MOE_KERNEL_ROUTER_LOGITS, s);
        e = launch_router_logits(g.dtype, x, T, g.H, L.w_router, L.router_bias, g.E, c->logits, c->tile_hist,
                                 fused_hist ? n_perm_tiles * g.E : 0, s);
    }
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    {
        Timed t(c, MOE_KERNEL_TOPK, s);
        e = launch_topk(c->logits, T, g.E, g.K, g.renormalize, c->idx, c->w, fused_hist ? c->tile_hist : nullptr, s);
    }
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    {
        Timed t(c, MOE_KERNEL_PERMUTE, s);
        e = launch_permute(c->idx, A, g.E, c->counts, c->offsets, c->perm, c->inv, c->tile_hist, fused_hist,
                           c->d_active_total, s);
    }
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    // the activation rows are gathered inside the gate_up GEMM's tile loads: no x_perm round trip
    const bool w4 = g.weight_format == MOE_W_MXFP4;
    {
        Timed t(c, MOE_KERNEL_GATE_UP, s);
        if (w4)
            e = launch_ffn_gate_up_w4(c->ffn_variant, x, c->perm, g.K, c->offsets, A, g.E, g.H, g.I,
                                      (const uint8_t*)L.w_gate_up, L.s_gate_up, c->act, s);
        else
            e = launch_ffn_gate_up(g.dtype, c->ffn_variant, g.act_split != 0, x, c->perm, g.K, c->offsets, A, g.E, g.H,
                                   g.I, L.w_gate_up, c->act, s);
    }
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    {
        Timed t(c, MOE_KERNEL_DOWN, s);
        if (w4)
            e = launch_ffn_down_w4(c->ffn_variant, g.y_perm_f32 != 0, c->act, c->offsets, A, g.E, g.H, g.I,
                                   (const uint8_t*)L.w_down, L.s_down, c->y_perm, s);
        else
            e = launch_ffn_down(g.dtype, c->ffn_variant, g.y_perm_f32 != 0, g.act_split != 0, c->act, c->offsets, A, g.E,
                                g.H, g.I, L.w_down, c->y_perm, s);
    }
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    {
        Timed t(c, MOE_KERNEL_COMBINE, s);
        e = launch_combine(g.dtype, g.y_perm_f32 != 0, c->y_perm, c->inv, c->w, g.residual != 0, x, T, g.K, g.H, y0,
                           rows0, y1, s);
    }
    return dev(e);
}

// Layers [0, n) of `layers` on the batch `in` [T,H]: the first layer reads `in` where it is, the layers
// between ping-pong through the context's two batch buffers, the last one writes rows [0,rows0) to y0
// and the rest to y1 (either may be the memory `in` points at: a layer's output row is written by the
// combine kernel after every read of that row).
moe_status run_group(moe_ctx* c, const moe_layer* layers, int n, RowSrc in, int64_t T, void* y0, int64_t rows0,
                     void* y1, hipStream_t s)
{
    char* cur = static_cast<char*>(c->xa);
    char* nxt = static_cast<char*>(c->xb);
    for (int l = 0; l < n; ++l) {
        const RowSrc src = (l == 0) ? in : single_src(cur);
        moe_status st;
        if (l + 1 < n) st = run_layer(c, layers[l], src, T, nxt, T, nxt, s);
        else st = run_layer(c, layers[l], src, T, y0, rows0, y1, s);
        if (st != MOE_OK) return st;
        char* t = cur; cur = nxt; nxt = t;
        c->layer_passes += 1;
        c->router_bytes += (uint64_t)c->cfg.E * c->cfg.H * c->esz;
    }
    return MOE_OK;
}

moe_status check_stack_args(const moe_ctx* ctx, const moe_layer* layers, int32_t n_layers, const void* x_decode,
                            int64_t D, const void* x_prefill, int64_t P, const void* y_decode, const void* y_prefill)
{
    if (!ctx || !layers) return MOE_ERR_NULL;
    if (n_layers <= 0 || D < 0 || P < 0) return MOE_ERR_SHAPE;
    if ((D > 0 && (!x_decode || !y_decode)) || (P > 0 && (!x_prefill || !y_prefill))) return MOE_ERR_NULL;
    if ((D > 0 && (misaligned(x_decode) || misaligned(y_decode))) ||
        (P > 0 && (misaligned(x_prefill) || misaligned(y_prefill))))
        return MOE_ERR_ALIGN;
    for (int l = 0; l < n_layers; ++l) {
        if (!layers[l].w_router || !layers[l].w_gate_up || !layers[l].w_down) return MOE_ERR_NULL;
        if (misaligned(layers[l].w_router) || misaligned(layers[l].w_gate_up) || misaligned(layers[l].w_down))
            return MOE_ERR_ALIGN;
        if (ctx->cfg.weight_format == MOE_W_MXFP4) {
            if (!layers[l].s_gate_up || !layers[l].s_down) return MOE_ERR_NULL;
            if (misaligned32(layers[l].w_gate_up) || misaligned32(layers[l].w_down) ||
                misaligned(layers[l].s_gate_up) || misaligned(layers[l].s_down))
                return MOE_ERR_ALIGN;
        }
    }
    return MOE_OK;
}

}  // namespace

extern "C" {

moe_status moe_workspace_bytes(const moe_config* cfg, int64_t max_tokens, size_t* out_bytes)
{
    if (!out_bytes) return MOE_ERR_NULL;
    moe_status st = check_cfg(cfg);
    if (st != MOE_OK) return st;
    if (max_tokens <= 0 || max_tokens > (((int64_t)1 << 31) - 1) / cfg->K) return MOE_ERR_SHAPE;   // A = T*K is counted in 32 bits
    *out_bytes = carve(*cfg, max_tokens).total;
    return MOE_OK;
}

moe_status moe_create(const moe_config* cfg, int64_t max_tokens, void* workspace, size_t workspace_bytes,
                      void* stream, moe_ctx** out_ctx)
{
    if (!out_ctx || !workspace) return MOE_ERR_NULL;
    moe_status st = check_cfg(cfg);
    if (st != MOE_OK) return st;
    if (max_tokens <= 0 || max_tokens > (((int64_t)1 << 31) - 1) / cfg->K) return MOE_ERR_SHAPE;   // A = T*K is counted in 32 bits
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return MOE_ERR_ALIGN;
    const Layout L = carve(*cfg, max_tokens);
    if (workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return MOE_ERR_DEVICE;
    char* b = static_cast<char*>(workspace);
    c->cfg = *cfg;
    c->max_tokens = max_tokens;
    c->esz = cfg->dtype == MOE_BF16 ? 2 : 4;
    c->d_active_total = reinterpret_cast<unsigned long long*>(b + L.counters);
    c->logits = reinterpret_cast<double*>(b + L.logits);
    c->idx = reinterpret_cast<int32_t*>(b + L.idx);
    c->w = reinterpret_cast<float*>(b + L.w);
    c->counts = reinterpret_cast<int32_t*>(b + L.counts);
    c->offsets = reinterpret_cast<int32_t*>(b + L.offsets);
    c->perm = reinterpret_cast<int32_t*>(b + L.perm);
    c->inv = reinterpret_cast<int32_t*>(b + L.inv);
    c->tile_hist = reinterpret_cast<int32_t*>(b + L.tile_hist);
    c->xa = b + L.xa;
    c->xb = b + L.xb;
    c->act = b + L.act;
    c->y_perm = b + L.y_perm;
    c->router_bytes = c->tokens_processed = 0;
    c->iterations = c->layer_passes = 0;
    c->timing_mask = 0;
    c->ffn_variant = MOE_FFN_AUTO;
    if (hipMemsetAsync(b + L.counters, 0, 256, static_cast<hipStream_t>(stream)) != hipSuccess) {
        delete c;
        return MOE_ERR_DEVICE;
    }
    *out_ctx = c;
    return MOE_OK;
}

moe_status moe_destroy(moe_ctx* ctx)
{
    if (!ctx) return MOE_ERR_NULL;
    drop_timing(ctx, true);
    delete ctx;
    return MOE_OK;
}

moe_status moe_router_topk(moe_ctx* ctx, const void* x, int64_t T, const void* w_router, const float* bias,
                           int32_t* topk_idx, float* topk_w, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (T < 0 || T > ctx->max_tokens) return MOE_ERR_SHAPE;
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !topk_idx || !topk_w) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router)) return MOE_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const moe_config& g = ctx->cfg;
    hipError_t e = launch_router_logits(g.dtype, single_src(x), T, g.H, w_router, bias, g.E, ctx->logits, nullptr, 0, s);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    return dev(launch_topk(ctx->logits, T, g.E, g.K, g.renormalize, topk_idx, topk_w, nullptr, s));
}

moe_status moe_router_topk_noalloc(const moe_config* cfg, const void* x, int64_t T, const void* w_router,
                                   const float* bias, int32_t* topk_idx, float* topk_w, void* stream)
{
    moe_status st = check_cfg(cfg);
    if (st != MOE_OK) return st;
    if (T < 0) return MOE_ERR_SHAPE;
    if (T > kNoallocMaxLogits / cfg->E) return MOE_ERR_WORKSPACE;      // the static scratch holds T * E logits (no overflow for any T)
    if (T == 0) return MOE_OK;
    if (!x || !w_router || !topk_idx || !topk_w) return MOE_ERR_NULL;
    if (misaligned(x) || misaligned(w_router)) return MOE_ERR_ALIGN;
    // device address of this GPU's copy of the scratch array, looked up once per device
    static std::mutex mu;
    static double* dev_scratch[kMaxDevices] = {};
    int d = 0;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return MOE_ERR_DEVICE;
    double* logits = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!dev_scratch[d]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOE_ERR_DEVICE;
            dev_scratch[d] = static_cast<double*>(p);
        }
        logits = dev_scratch[d];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_router_logits(cfg->dtype, single_src(x), T, cfg->H, w_router, bias, cfg->E, logits, nullptr, 0, s);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    return dev(launch_topk(logits, T, cfg->E, cfg->K, cfg->renormalize, topk_idx, topk_w, nullptr, s));
}

moe_status moe_permute(moe_ctx* ctx, const void* x, const int32_t* topk_idx, int64_t T, int32_t* counts,
                       int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (T < 0 || T > ctx->max_tokens) return MOE_ERR_SHAPE;
    if (!counts || !offsets) return MOE_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const moe_config& g = ctx->cfg;
    if (T == 0) {
        // fill kernels, not memset nodes: the caller may be capturing the stream
        if (launch_fill_zero(counts, g.E, s) != hipSuccess) return MOE_ERR_DEVICE;
        return dev(launch_fill_zero(offsets, g.E + 1, s));
    }
    if (!topk_idx || !perm || !inv_perm) return MOE_ERR_NULL;
    if (x_perm && (!x || misaligned(x) || misaligned(x_perm))) return x ? MOE_ERR_ALIGN : MOE_ERR_NULL;
    const int64_t A = T * g.K;
    hipError_t e = launch_permute(topk_idx, A, g.E, counts, offsets, perm, inv_perm, ctx->tile_hist, false, nullptr, s);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    if (x_perm) return dev(launch_gather_rows(g.dtype, x, perm, g.K, A, g.H, x_perm, s));
    return MOE_OK;
}

moe_status moe_grouped_ffn(moe_ctx* ctx, const void* x_perm, const int32_t* offsets, int64_t A,
                           const void* w_gate_up, const void* w_down, void* y_perm, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (A < 0 || A > ctx->max_tokens * ctx->cfg.K) return MOE_ERR_SHAPE;
    if (A == 0) return MOE_OK;
    if (!x_perm || !offsets || !w_gate_up || !w_down || !y_perm) return MOE_ERR_NULL;
    if (misaligned(x_perm) || misaligned(w_gate_up) || misaligned(w_down) || misaligned(y_perm)) return MOE_ERR_ALIGN;
    const moe_config& g = ctx->cfg;
    if (g.weight_format != MOE_W_DTYPE) return MOE_ERR_DTYPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_ffn_gate_up(g.dtype, ctx->ffn_variant, g.act_split != 0, single_src(x_perm), nullptr, 1, offsets,
                                      A, g.E, g.H, g.I, w_gate_up, ctx->act, s);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    return dev(launch_ffn_down(g.dtype, ctx->ffn_variant, g.y_perm_f32 != 0, g.act_split != 0, ctx->act, offsets, A, g.E,
                               g.H, g.I, w_down, y_perm, s));
}

moe_status moe_grouped_ffn_mxfp4(moe_ctx* ctx, const void* x_perm, const int32_t* offsets, int64_t A,
                                 const uint8_t* w_gate_up, const uint8_t* s_gate_up, const uint8_t* w_down,
                                 const uint8_t* s_down, void* y_perm, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (A < 0 || A > ctx->max_tokens * ctx->cfg.K) return MOE_ERR_SHAPE;
    if (ctx->cfg.weight_format != MOE_W_MXFP4) return MOE_ERR_DTYPE;
    if (A == 0) return MOE_OK;
    if (!x_perm || !offsets || !w_gate_up || !s_gate_up || !w_down || !s_down || !y_perm) return MOE_ERR_NULL;
    if (misaligned(x_perm) || misaligned32(w_gate_up) || misaligned32(w_down) || misaligned(s_gate_up) ||
        misaligned(s_down) || misaligned(y_perm))
        return MOE_ERR_ALIGN;
    const moe_config& g = ctx->cfg;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_ffn_gate_up_w4(ctx->ffn_variant, single_src(x_perm), nullptr, 1, offsets, A, g.E, g.H, g.I,
                                         w_gate_up, s_gate_up, ctx->act, s);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    return dev(launch_ffn_down_w4(ctx->ffn_variant, g.y_perm_f32 != 0, ctx->act, offsets, A, g.E, g.H, g.I, w_down,
                                  s_down, y_perm, s));
}

moe_status moe_combine(moe_ctx* ctx, const void* y_perm, const int32_t* inv_perm, const float* topk_w,
                       const void* residual, int64_t T, void* y, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (T < 0 || T > ctx->max_tokens) return MOE_ERR_SHAPE;
    if (T == 0) return MOE_OK;
    if (!y_perm || !inv_perm || !topk_w || !y) return MOE_ERR_NULL;
    if (misaligned(y_perm) || misaligned(y) || (residual && misaligned(residual))) return MOE_ERR_ALIGN;
    const moe_config& g = ctx->cfg;
    return dev(launch_combine(g.dtype, g.y_perm_f32 != 0, y_perm, inv_perm, topk_w, residual != nullptr,
                              single_src(residual), T, g.K, g.H, y, T, y, static_cast<hipStream_t>(stream)));
}

moe_status moe_group_forward(moe_ctx* ctx, const moe_layer* layers, int32_t n_layers, const void* x_decode,
                             int64_t D, const void* x_prefill, int64_t P, moe_schedule sched, void* y_decode,
                             void* y_prefill, void* stream)
{
    if (!ctx || !layers) return MOE_ERR_NULL;
    if (n_layers <= 0 || D < 0 || P < 0) return MOE_ERR_SHAPE;
    if (sched.kind != MOE_SCHED_CHUNKED && sched.kind != MOE_SCHED_LAYERED) return MOE_ERR_SCHEDULE;
    if (sched.kind == MOE_SCHED_CHUNKED && sched.chunk <= 0) return MOE_ERR_SCHEDULE;
    // one group that holds every layer: each iteration sends [decode; slice] through all of them
    moe_stack_schedule st;
    st.chunk = sched.kind == MOE_SCHED_CHUNKED ? sched.chunk : 0;
    st.n_groups = 1;
    st.granule = 0;
    return moe_stack_forward(ctx, layers, n_layers, x_decode, D, x_prefill, P, st, y_decode, y_prefill, stream);
}

int32_t moe_num_layer_groups(int64_t prompt_len, int32_t n_layers, int32_t granule)
{
    if (prompt_len < 0 || n_layers <= 0 || granule <= 0) return 0;
    int64_t n = (prompt_len + granule - 1) / granule;
    if (n < 1) n = 1;
    if (n > n_layers) n = n_layers;
    return (int32_t)n;
}

moe_status moe_layer_groups(int32_t n_layers, int32_t n_groups, int32_t* first_layer)
{
    if (!first_layer) return MOE_ERR_NULL;
    if (n_groups < 1 || n_groups > n_layers) return MOE_ERR_SHAPE;
    const int32_t q = n_layers / n_groups, r = n_layers % n_groups;
    int32_t at = 0;
    for (int32_t g = 0; g < n_groups; ++g) {
        first_layer[g] = at;
        at += q + (g < r ? 1 : 0);
    }
    first_layer[n_groups] = at;
    return MOE_OK;
}

moe_status moe_stack_forward(moe_ctx* ctx, const moe_layer* layers, int32_t n_layers, const void* x_decode,
                             int64_t D, const void* x_prefill, int64_t P, moe_stack_schedule sched, void* y_decode,
                             void* y_prefill, void* stream)
{
    moe_status st = check_stack_args(ctx, layers, n_layers, x_decode, D, x_prefill, P, y_decode, y_prefill);
    if (st != MOE_OK) return st;
    if (sched.chunk < 0 || sched.n_groups < 0 || sched.n_groups > n_layers) return MOE_ERR_SCHEDULE;
    if (sched.n_groups == 0 && sched.granule <= 0) return MOE_ERR_SCHEDULE;
    if (D + P == 0) return MOE_OK;
    if ((P > 0 && x_prefill == y_prefill) || (D > 0 && x_decode == y_decode)) return MOE_ERR_SHAPE;
    const int64_t step = (sched.chunk > 0 && P > 0) ? (int64_t)sched.chunk : (P > 0 ? P : 1);
    const int64_t n_slices = (P == 0) ? 1 : (P + step - 1) / step;
    if (D + (P < step ? P : step) > ctx->max_tokens) return MOE_ERR_SHAPE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t row_bytes = (size_t)ctx->cfg.H * ctx->esz;
    std::vector<int32_t> first((size_t)n_layers + 1);
    for (int64_t sl = 0; sl < n_slices; ++sl) {
        const int64_t p0 = sl * step;
        const int64_t pn = (P == 0) ? 0 : ((p0 + step <= P) ? step : P - p0);
        // a decode-only call (no prompt rows) is one iteration whatever the group count
        const int32_t G = (pn == 0) ? 1
                          : (sched.n_groups > 0 ? sched.n_groups : moe_num_layer_groups(pn, n_layers, sched.granule));
        st = moe_layer_groups(n_layers, G, first.data());
        if (st != MOE_OK) return st;
        const char* slice_in = static_cast<const char*>(x_prefill) + p0 * row_bytes;
        char* slice_state = (P > 0) ? static_cast<char*>(y_prefill) + p0 * row_bytes : nullptr;
        for (int32_t g = 0; g < G; ++g) {
            for (int32_t j = 0; j < G; ++j) {
                const moe_layer* gl = layers + first[j];
                const int gn = first[j + 1] - first[j];
                // the decode rows enter group 0 from x_decode and travel on in y_decode
                const void* dec_in = (j == 0) ? x_decode : y_decode;
                if (j == g && pn > 0) {
                    const RowSrc in{dec_in, D, (g == 0) ? slice_in : slice_state};
                    st = run_group(ctx, gl, gn, in, D + pn, y_decode, D, slice_state, s);
                } else if (D > 0) {
                    st = run_group(ctx, gl, gn, single_src(dec_in), D, y_decode, D, nullptr, s);
                }
                if (st != MOE_OK) return st;
            }
            ctx->iterations += 1;
            ctx->tokens_processed += (uint64_t)(D + pn);
        }
    }
    return MOE_OK;
}

moe_status moe_read_counters(moe_ctx* ctx, moe_counters* out, void* stream)
{
    if (!ctx || !out) return MOE_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned long long active = 0;
    if (hipMemcpyAsync(&active, ctx->d_active_total, sizeof(active), hipMemcpyDeviceToHost, s) != hipSuccess)
        return MOE_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return MOE_ERR_DEVICE;
    const moe_config& g = ctx->cfg;
    out->active_experts_total = active;
    const uint64_t hi3 = 3ull * (uint64_t)g.H * (uint64_t)g.I;
    // one expert's weights: dtype elements, or 4-bit codes plus one scale byte per 32 of them
    out->expert_bytes = (uint64_t)active * (g.weight_format == MOE_W_MXFP4 ? hi3 / 2 + hi3 / 32 : hi3 * (uint64_t)ctx->esz);
    out->router_bytes = ctx->router_bytes;
    out->tokens_processed = ctx->tokens_processed;
    out->iterations = ctx->iterations;
    out->layer_passes = ctx->layer_passes;
    return MOE_OK;
}

moe_status moe_reset_counters(moe_ctx* ctx, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    ctx->router_bytes = ctx->tokens_processed = 0;
    ctx->iterations = ctx->layer_passes = 0;
    return dev(launch_fill_zero(ctx->d_active_total, 2, static_cast<hipStream_t>(stream)));
}

moe_status moe_kernel_timing(moe_ctx* ctx, uint32_t kernel_mask)
{
    if (!ctx) return MOE_ERR_NULL;
    if (kernel_mask >> MOE_KERNEL_COUNT) return MOE_ERR_SHAPE;
    drop_timing(ctx, false);
    ctx->timing_mask = kernel_mask;
    return MOE_OK;
}

moe_status moe_read_kernel_timing(moe_ctx* ctx, int32_t kernel, double* total_ms, int64_t* launches, void* stream)
{
    if (!ctx || !total_ms || !launches) return MOE_ERR_NULL;
    if (kernel < 0 || kernel >= MOE_KERNEL_COUNT) return MOE_ERR_SHAPE;
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return MOE_ERR_DEVICE;
    double sum = 0.0;
    for (auto& p : ctx->timing[kernel]) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.first, p.second) != hipSuccess) return MOE_ERR_DEVICE;
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int64_t)ctx->timing[kernel].size();
    return MOE_OK;
}

const char* moe_ffn_variant(const moe_ctx* ctx, int64_t T)
{
    if (!ctx) return "";
    const moe_config& g = ctx->cfg;
    if (g.weight_format == MOE_W_MXFP4) return ffn_w4_variant_name(ctx->ffn_variant, T * g.K, g.E);
    return ffn_variant_name(g.dtype, ctx->ffn_variant, T * g.K, g.E, g.H, g.I);
}

moe_status moe_set_ffn_variant(moe_ctx* ctx, int32_t variant)
{
    if (!ctx) return MOE_ERR_NULL;
    if (variant < MOE_FFN_AUTO || variant > MOE_FFN_W4_STREAM) return MOE_ERR_SHAPE;
    ctx->ffn_variant = variant;
    return MOE_OK;
}

const char* moe_status_string(moe_status s)
{
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "null pointer";
        case MOE_ERR_SHAPE: return "bad shape or size";
        case MOE_ERR_DTYPE: return "unknown dtype";
        case MOE_ERR_ALIGN: return "alignment (H, I multiples of 8, 64 with MXFP4 weights; 16-byte aligned pointers, 32-byte for MXFP4 codes)";
        case MOE_ERR_WORKSPACE: return "workspace too small";
        case MOE_ERR_SCHEDULE: return "bad schedule";
        case MOE_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
