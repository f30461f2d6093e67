// C-ABI layer of libhybridkv: argument validation (host only, before any launch), workspace
// layout, and the sequencing of the kernels of the hybrid-cache decode step
// (KV Gen -> concat -> MHA; Sec. 4.2.2, Eq. 7, 3, 4).
#include "../../include/hybridkv.h"
#include "hk_internal.h"

#include <atomic>
#include <cmath>
#include <cstdint>

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct Plan {
    // sizes
    int64_t M;            // B * L_act
    int64_t BH;           // B * n_heads
    int n_waves;          // wavefronts of the attention kernel
    float scale;
    // workspace offsets (bytes)
    size_t off_k, off_v, off_stats, off_prep, off_partial, total;   // off_prep: per-call prepared layer (0 bytes when unused)
};

int check_shape(const hk_shape *s)
{
    if (!s) return HK_ERR_NULL;
    if (s->dtype != HK_DTYPE_F16 && s->dtype != HK_DTYPE_BF16) return HK_ERR_DTYPE;
    if (s->d <= 0 || s->n_heads <= 0) return HK_ERR_SHAPE;
    if (s->gemm_tile != 0 && s->gemm_tile != 128 && s->gemm_tile != 256) return HK_ERR_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128) return HK_ERR_SHAPE;
    if ((int64_t)s->n_heads * s->head_dim != s->d) return HK_ERR_SHAPE;
    if (s->d > (1 << 20)) return HK_ERR_SHAPE;
    if (s->attn_splits < 0 || s->attn_splits > HK_MAX_SPLITS) return HK_ERR_SHAPE;
    if (!(s->ln_eps >= 0.f) || !std::isfinite(s->ln_eps) || !std::isfinite(s->softmax_scale)) return HK_ERR_SHAPE;
    return HK_OK;
}

struct PreparedLayout {
    size_t off_w, off_c, off_b, total;
};
PreparedLayout prepared_layout(int d);

// Fills the plan; returns HK_OK or a status.  regen_only: plan of hk_regen_kv (no K/V scratch, no partials).
// prep_room = false: the caller brings a prepared layer, no room for one is planned.
int make_plan(const hk_shape *s, int64_t B, int64_t L_kv, int64_t L_act, bool regen_only, Plan *p, bool prep_room = true)
{
    int st = check_shape(s);
    if (st != HK_OK) return st;
    if (B < 0 || L_kv < 0 || L_act < 0) return HK_ERR_SHAPE;
    if (B > (1 << 24) || L_kv > (1 << 28) || L_act > (1 << 28)) return HK_ERR_SHAPE;
    p->M = B * L_act;
    p->BH = B * s->n_heads;
    // element counts must stay addressable and grids launchable
    const long double elems = (long double)B * (long double)(L_kv + L_act) * (long double)s->d;
    if (elems > 4.0e12L || p->M > 0x7fffffffLL || p->BH > 0x7fffffffLL) return HK_ERR_SHAPE;
    p->scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / std::sqrt((float)s->head_dim);
    const size_t kv_bytes = regen_only ? 0 : align_up((size_t)p->M * s->d * 2);
    p->off_k = 0;
    p->off_v = kv_bytes;
    p->off_stats = 2 * kv_bytes;
    size_t end = p->off_stats + align_up((size_t)p->M * sizeof(float2));
    // The large-problem projection kernel works on a prepared layer; room to prepare one per call, for
    // callers that do not bring their own.
    p->off_prep = end;
    if (prep_room && p->M > 0 && hk::kv_gemm_uses_prepared(p->M, s->d, s->gemm_tile, s->dtype)) end += prepared_layout(s->d).total;
    p->off_partial = end;
    p->n_waves = 0;
    if (!regen_only && L_kv + L_act > 0 && p->BH > 0) {
        p->n_waves = hk::attn_wavefronts(p->BH, L_kv + L_act, s->attn_splits);
        end += align_up(((size_t)p->n_waves + (size_t)p->BH) * (s->head_dim + 2) * sizeof(float));
    }
    p->total = end;
    return HK_OK;
}

int check_params(const hk_layer_params *lp)
{
    if (!lp) return HK_ERR_NULL;
    if (!lp->ln_w || !lp->ln_b || !lp->Wkv || !lp->bkv) return HK_ERR_NULL;
    if (!aligned(lp->ln_w, 16) || !aligned(lp->ln_b, 16) || !aligned(lp->Wkv, 16) || !aligned(lp->bkv, 16))
        return HK_ERR_ALIGN;
    if (lp->prepared && !aligned(lp->prepared, kAlign)) return HK_ERR_ALIGN;
    return HK_OK;
}

// Layout of a prepared layer: W' [2d, d] fp16, then c [2d] fp32, then b' [2d] fp32, each 256-byte aligned.
PreparedLayout prepared_layout(int d)
{
    PreparedLayout L;
    L.off_w = 0;
    L.off_c = align_up((size_t)2 * d * d * 2);
    L.off_b = L.off_c + align_up((size_t)2 * d * sizeof(float));
    L.total = L.off_b + align_up((size_t)2 * d * sizeof(float));
    return L;
}

// Optional per-kernel time stamps: events recorded on the call's stream between the kernels.
struct Marks {
    hipEvent_t *ev;
    int n;
    hipStream_t stream;
    bool put(int i) const { return !(ev && i < n && ev[i]) || hipEventRecord(ev[i], stream) == hipSuccess; }
};

int regen_impl(const hk_shape *s, const void *act, int64_t L_act, const hk_layer_params *lp,
               void *K_out, void *V_out, int L_cap, int tok_off, float2 *stats, void *prep_scratch, int64_t M,
               hipStream_t stream, const Marks &mk, int cu_limit = 0)
{
    const void *prepared = lp->prepared;
    if (!prepared && hk::kv_gemm_uses_prepared(M, s->d, s->gemm_tile, s->dtype)) {
        // no prepared layer given: prepare one into the workspace (one pass over the weights)
        const PreparedLayout L = prepared_layout(s->d);
        char *pp = static_cast<char *>(prep_scratch);
        if (hk::launch_prepare_layer(lp->Wkv, lp->bkv, lp->ln_w, lp->ln_b, pp + L.off_w,
                                     reinterpret_cast<float *>(pp + L.off_c), reinterpret_cast<float *>(pp + L.off_b),
                                     s->d, stream, s->dtype) != hipSuccess)
            return HK_ERR_LAUNCH;
        prepared = prep_scratch;
    }
    if (hk::launch_ln_stats(act, stats, M, s->d, s->ln_eps, stream, s->dtype) != hipSuccess) return HK_ERR_LAUNCH;
    if (!mk.put(1)) return HK_ERR_LAUNCH;
    hk::KvGemmArgs g;
    g.act = act; g.stats = stats; g.ln_w = lp->ln_w; g.ln_b = lp->ln_b; g.Wkv = lp->Wkv; g.bkv = lp->bkv;
    g.Wp = nullptr; g.cvec = nullptr; g.bvec = nullptr;
    if (prepared) {
        const PreparedLayout L = prepared_layout(s->d);
        const char *pp = static_cast<const char *>(prepared);
        g.Wp = pp + L.off_w;
        g.cvec = reinterpret_cast<const float *>(pp + L.off_c);
        g.bvec = reinterpret_cast<const float *>(pp + L.off_b);
    }
    g.K_out = K_out; g.V_out = V_out; g.M = M; g.d = s->d; g.n_heads = s->n_heads; g.head_dim = s->head_dim;
    g.L_act = (int)L_act; g.L_cap = L_cap; g.tok_off = tok_off; g.tile = s->gemm_tile; g.dtype = s->dtype;
    g.cu_limit = cu_limit;
    if (hk::launch_kv_gemm(g, stream) != hipSuccess) return HK_ERR_LAUNCH;
    return HK_OK;
}

}  // namespace

extern "C" {

size_t hk_prepared_bytes(const hk_shape *shape)
{
    if (check_shape(shape) != HK_OK) return 0;
    return prepared_layout(shape->d).total;
}

int hk_prepare_layer(const hk_shape *shape, const hk_layer_params *params, void *prepared, size_t prepared_bytes,
                     void *stream)
{
    int st = check_shape(shape);
    if (st != HK_OK) return st;
    st = check_params(params);
    if (st != HK_OK) return st;
    if (!prepared) return HK_ERR_NULL;
    if (!aligned(prepared, kAlign)) return HK_ERR_ALIGN;
    const PreparedLayout L = prepared_layout(shape->d);
    if (prepared_bytes < L.total) return HK_ERR_WORKSPACE;
    char *pp = static_cast<char *>(prepared);
    if (hk::launch_prepare_layer(params->Wkv, params->bkv, params->ln_w, params->ln_b, pp + L.off_w,
                                 reinterpret_cast<float *>(pp + L.off_c), reinterpret_cast<float *>(pp + L.off_b),
                                 shape->d, static_cast<hipStream_t>(stream), shape->dtype) != hipSuccess)
        return HK_ERR_LAUNCH;
    return HK_OK;
}

size_t hk_regen_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_act)
{
    Plan p;
    if (make_plan(shape, B, 0, L_act, true, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

size_t hk_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act)
{
    Plan p;
    if (make_plan(shape, B, L_kv, L_act, false, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

int hk_regen_offsets(const hk_shape *shape, int32_t B, int32_t L_act, size_t *k_offset, size_t *v_offset)
{
    if (!k_offset || !v_offset) return HK_ERR_NULL;
    Plan p;
    const int st = make_plan(shape, B, 0, L_act, false, &p);     // the offsets do not depend on L_kv
    if (st != HK_OK) return st;
    *k_offset = p.off_k;
    *v_offset = p.off_v;
    return HK_OK;
}

int hk_regen_kv(const hk_shape *shape, const void *act, int32_t B, int32_t L_act,
                const hk_layer_params *params, void *K_out, void *V_out, int32_t L_cap, int32_t tok_off,
                void *workspace, size_t workspace_bytes, void *stream)
{
    Plan p;
    int st = make_plan(shape, B, 0, L_act, true, &p);
    if (st != HK_OK) return st;
    if (tok_off < 0 || L_cap < 0 || (int64_t)tok_off + L_act > L_cap) return HK_ERR_SHAPE;
    if ((long double)B * L_cap * shape->d > 4.0e12L) return HK_ERR_SHAPE;
    if (p.M == 0) return HK_OK;
    st = check_params(params);
    if (st != HK_OK) return st;
    if (!act || !K_out || !V_out || !workspace) return HK_ERR_NULL;
    if (!aligned(act, 16) || !aligned(K_out, 16) || !aligned(V_out, 16) || !aligned(workspace, kAlign))
        return HK_ERR_ALIGN;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    return regen_impl(shape, act, L_act, params, K_out, V_out, L_cap, tok_off,
                      reinterpret_cast<float2 *>(ws + p.off_stats), ws + p.off_prep, p.M, static_cast<hipStream_t>(stream),
                      Marks{nullptr, 0, nullptr});
}

int hk_hybrid_decode_attn(const hk_shape *shape, const void *q,
                          const void *K_cache, const void *V_cache, int32_t L_kv,
                          const void *act, int32_t L_act, int32_t B,
                          const hk_layer_params *params, float ratio,
                          void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return hk_hybrid_decode_attn_marked(shape, q, K_cache, V_cache, L_kv, act, L_act, B, params, ratio, out,
                                        workspace, workspace_bytes, stream, nullptr, 0);
}

}  // extern "C"

namespace {

// ---- the step on two streams: the attention over the cached segment beside the regeneration ----
struct TwoStreamPlan {
    Plan base;                 // regenerated K/V, statistics, room for a prepared layer (its partials are not used)
    int waves_c, waves_r;      // wavefronts of the attention over the cached / the regenerated segment
    size_t off_part_c, off_part_r, off_out_c, off_out_r, off_lse_c, off_lse_r, total;
};

int make_two_stream_plan(const hk_shape *s, int64_t B, int64_t L_kv, int64_t L_act, TwoStreamPlan *p)
{
    const int st = make_plan(s, B, L_kv, L_act, false, &p->base);
    if (st != HK_OK) return st;
    const size_t bh = (size_t)p->base.BH;
    size_t end = p->base.off_partial;                          // the single-stream partials are not needed: reuse their place
    auto take = [&](size_t bytes) { const size_t at = end; end += align_up(bytes); return at; };
    p->waves_c = L_kv > 0 && bh > 0 ? hk::attn_wavefronts((int64_t)bh, L_kv, s->attn_splits) : 0;
    p->waves_r = L_act > 0 && bh > 0 ? hk::attn_wavefronts((int64_t)bh, L_act, s->attn_splits) : 0;
    p->off_part_c = take(((size_t)p->waves_c + bh) * (s->head_dim + 2) * sizeof(float));
    p->off_part_r = take(((size_t)p->waves_r + bh) * (s->head_dim + 2) * sizeof(float));
    p->off_out_c = take(bh * s->head_dim * 2);
    p->off_out_r = take(bh * s->head_dim * 2);
    p->off_lse_c = take(bh * sizeof(float2));
    p->off_lse_r = take(bh * sizeof(float2));
    p->total = end > p->base.total ? end : p->base.total;      // never less than the single-stream step needs (the fallback)
    return HK_OK;
}

// ---- the step for callers that cannot allocate: scratch in a static device array of the library ----
// One copy per GPU, held from the loading of the library's code on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[HK_STATIC_SCRATCH_BYTES];

constexpr int kMaxScratchDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxScratchDevices];     // device address of `scratch` on device i (null: not looked up yet)

// Device address of this GPU's copy of `scratch`.  The array's name is only a host-side handle: the address
// comes from the runtime, once per device, with that device current.
int static_scratch_ptr(void **ptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return HK_ERR_LAUNCH;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HK_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return HK_OK;
}

// The hybrid step on a given scratch buffer.  static_scratch: the buffer is the library's own array instead
// (`workspace` is ignored, workspace_bytes is the array's size, and a caller that brings a prepared layer needs no
// room for one); its address is looked up only after every check has passed.
int hybrid_step(const hk_shape *shape, const void *q,
                const void *K_cache, const void *V_cache, int32_t L_kv,
                const void *act, int32_t L_act, int32_t B,
                const hk_layer_params *params, float ratio,
                void *out, void *workspace, size_t workspace_bytes, bool static_scratch, void *stream,
                void **events, int32_t n_events)
{
    Plan p;
    int st = make_plan(shape, B, L_kv, L_act, false, &p, !(static_scratch && params && params->prepared));
    if (st != HK_OK) return st;
    const int64_t L = (int64_t)L_kv + L_act;
    if (L == 0) return HK_ERR_SHAPE;
    if (!(ratio >= 0.f && ratio <= 1.f)) return HK_ERR_RATIO;
    if (std::fabs((double)ratio * (double)L - (double)L_kv) > 0.5 + 1e-6 * (double)L) return HK_ERR_RATIO;
    if (B == 0) return HK_OK;
    if (static_scratch && workspace_bytes < p.total) return HK_ERR_STATIC_LIMIT;      // before the pointer checks: it is about sizes alone
    if (!q || !out || (!workspace && !static_scratch)) return HK_ERR_NULL;
    if (L_kv > 0 && (!K_cache || !V_cache)) return HK_ERR_NULL;
    if (L_act > 0) {
        st = check_params(params);
        if (st != HK_OK) return st;
        if (!act) return HK_ERR_NULL;
        if (!aligned(act, 16)) return HK_ERR_ALIGN;
    }
    if (!aligned(q, 16) || !aligned(out, 16) || (!static_scratch && !aligned(workspace, kAlign))) return HK_ERR_ALIGN;
    if (L_kv > 0 && (!aligned(K_cache, 16) || !aligned(V_cache, 16))) return HK_ERR_ALIGN;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;
    if (static_scratch) {
        st = static_scratch_ptr(&workspace);
        if (st != HK_OK) return st;
    }

    char *ws = static_cast<char *>(workspace);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    void *K_regen = ws + p.off_k, *V_regen = ws + p.off_v;
    const Marks mk{reinterpret_cast<hipEvent_t *>(events), events ? n_events : 0, hs};
    if (!mk.put(0)) return HK_ERR_LAUNCH;
    if (L_act > 0) {
        st = regen_impl(shape, act, L_act, params, K_regen, V_regen, L_act, 0,
                        reinterpret_cast<float2 *>(ws + p.off_stats), ws + p.off_prep, p.M, hs, mk);
        if (st != HK_OK) return st;
    } else if (!mk.put(1)) {
        return HK_ERR_LAUNCH;
    }
    if (!mk.put(2)) return HK_ERR_LAUNCH;
    hk::AttnArgs a;
    a.q = q;
    a.K0 = K_cache; a.V0 = V_cache; a.L0 = L_kv;
    a.K1 = K_regen; a.V1 = V_regen; a.L1 = L_act;
    a.BH = (int)p.BH; a.head_dim = shape->head_dim; a.scale = p.scale;
    a.n_waves = p.n_waves;
    a.partial = reinterpret_cast<float *>(ws + p.off_partial);
    a.out = out;
    a.lse = nullptr;
    a.dtype = shape->dtype;
    a.after_main = (mk.ev && mk.n > 3) ? mk.ev[3] : nullptr;
    if (hk::launch_flash_decode(a, hs) != hipSuccess) return HK_ERR_LAUNCH;
    if (!mk.put(4)) return HK_ERR_LAUNCH;
    return HK_OK;
}

}  // namespace

extern "C" {

int hk_hybrid_decode_attn_marked(const hk_shape *shape, const void *q,
                                 const void *K_cache, const void *V_cache, int32_t L_kv,
                                 const void *act, int32_t L_act, int32_t B,
                                 const hk_layer_params *params, float ratio,
                                 void *out, void *workspace, size_t workspace_bytes, void *stream,
                                 void **events, int32_t n_events)
{
    return hybrid_step(shape, q, K_cache, V_cache, L_kv, act, L_act, B, params, ratio, out, workspace, workspace_bytes, false,
                       stream, events, n_events);
}

size_t hk_two_stream_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act)
{
    TwoStreamPlan p;
    if (make_two_stream_plan(shape, B, L_kv, L_act, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

int hk_hybrid_decode_attn_two_stream(const hk_shape *shape, const void *q,
                                     const void *K_cache, const void *V_cache, int32_t L_kv,
                                     const void *act, int32_t L_act, int32_t B,
                                     const hk_layer_params *params, float ratio,
                                     void *out, void *workspace, size_t workspace_bytes,
                                     void *stream, void *side_stream, void *fork_event, void *join_event, int32_t gemm_cus)
{
    TwoStreamPlan p;
    int st = make_two_stream_plan(shape, B, L_kv, L_act, &p);
    if (st != HK_OK) return st;
    if (gemm_cus < 0) return HK_ERR_SHAPE;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;
    // Only one segment: there is nothing to run side by side, the single-stream step is the step.
    if (L_kv == 0 || L_act == 0 || B == 0)
        return hybrid_step(shape, q, K_cache, V_cache, L_kv, act, L_act, B, params, ratio, out, workspace, workspace_bytes, false,
                           stream, nullptr, 0);
    if (!(ratio >= 0.f && ratio <= 1.f)) return HK_ERR_RATIO;
    const int64_t L = (int64_t)L_kv + L_act;
    if (std::fabs((double)ratio * (double)L - (double)L_kv) > 0.5 + 1e-6 * (double)L) return HK_ERR_RATIO;
    if (!q || !out || !workspace || !K_cache || !V_cache || !act || !fork_event || !join_event) return HK_ERR_NULL;
    st = check_params(params);
    if (st != HK_OK) return st;
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(workspace, kAlign) || !aligned(act, 16) || !aligned(K_cache, 16) ||
        !aligned(V_cache, 16))
        return HK_ERR_ALIGN;

    char *ws = static_cast<char *>(workspace);
    hipStream_t main_s = static_cast<hipStream_t>(stream), side_s = static_cast<hipStream_t>(side_stream);
    hipEvent_t fork = static_cast<hipEvent_t>(fork_event), join = static_cast<hipEvent_t>(join_event);
    // main stream: LayerNorm statistics, fork, projection (on gemm_cus compute units when asked).  The fork sits
    // behind the statistics kernel: that kernel and the attention are both bound by HBM and gain nothing from
    // running side by side, the projection is bound by the matrix cores.
    void *K_regen = ws + p.base.off_k, *V_regen = ws + p.base.off_v;
    hipEvent_t marks[2] = {nullptr, fork};                     // Marks slot 1: recorded after the statistics kernel
    st = regen_impl(shape, act, L_act, params, K_regen, V_regen, L_act, 0, reinterpret_cast<float2 *>(ws + p.base.off_stats),
                    ws + p.base.off_prep, p.base.M, main_s, Marks{marks, 2, main_s}, gemm_cus);
    if (st != HK_OK) return st;
    // side stream: the attention over the cached segment, which needs nothing the regeneration produces
    if (hipStreamWaitEvent(side_s, fork, 0) != hipSuccess) return HK_ERR_LAUNCH;
    hk::AttnArgs a;
    a.q = q;
    a.K0 = K_cache; a.V0 = V_cache; a.L0 = L_kv;
    a.K1 = nullptr; a.V1 = nullptr; a.L1 = 0;
    a.BH = (int)p.base.BH; a.head_dim = shape->head_dim; a.scale = p.base.scale;
    a.n_waves = p.waves_c;
    a.partial = reinterpret_cast<float *>(ws + p.off_part_c);
    a.out = ws + p.off_out_c;
    a.lse = reinterpret_cast<float2 *>(ws + p.off_lse_c);
    a.dtype = shape->dtype;
    a.after_main = nullptr;
    if (hk::launch_flash_decode(a, side_s) != hipSuccess) return HK_ERR_LAUNCH;
    if (hipEventRecord(join, side_s) != hipSuccess) return HK_ERR_LAUNCH;
    // main stream again: the attention over the regenerated rows
    a.K0 = K_regen; a.V0 = V_regen; a.L0 = L_act;
    a.n_waves = p.waves_r;
    a.partial = reinterpret_cast<float *>(ws + p.off_part_r);
    a.out = ws + p.off_out_r;
    a.lse = reinterpret_cast<float2 *>(ws + p.off_lse_r);
    if (hk::launch_flash_decode(a, main_s) != hipSuccess) return HK_ERR_LAUNCH;
    if (hipStreamWaitEvent(main_s, join, 0) != hipSuccess) return HK_ERR_LAUNCH;
    if (hk::launch_segment_join(ws + p.off_out_c, reinterpret_cast<const float2 *>(ws + p.off_lse_c), ws + p.off_out_r,
                                reinterpret_cast<const float2 *>(ws + p.off_lse_r), out, (int)p.base.BH, shape->head_dim,
                                shape->dtype, main_s) != hipSuccess)
        return HK_ERR_LAUNCH;
    return HK_OK;
}

int hk_hybrid_decode_attn_static(const hk_shape *shape, const void *q,
                                 const void *K_cache, const void *V_cache, int32_t L_kv,
                                 const void *act, int32_t L_act, int32_t B,
                                 const hk_layer_params *params, float ratio,
                                 void *out, void *stream)
{
    return hybrid_step(shape, q, K_cache, V_cache, L_kv, act, L_act, B, params, ratio, out, nullptr, HK_STATIC_SCRATCH_BYTES, true,
                       stream, nullptr, 0);
}

namespace {

// Floats of the output projection's partial sums for B sequences (taken kAbsorbMaxBatch at a time).
size_t absorbed_proj_floats(const hk_shape *s, int64_t B)
{
    int parts, steps_per_part;
    hk::absorbed_project_parts(s->d, s->n_heads, &parts, &steps_per_part);
    const size_t rows = (size_t)(B < hk::kAbsorbMaxBatch ? B : hk::kAbsorbMaxBatch);
    return (size_t)parts * rows * s->d;
}

struct AbsorbedPlan {
    int64_t M, BH;
    int n_waves;               // wavefronts of the attention kernel over the cached segment
    int Lp;
    float scale;
    size_t off_stats, off_prep, off_u, off_raw, off_w, off_sums, off_y, off_outc, off_lse, off_proj, off_partial, total;
};

int make_absorbed_plan(const hk_shape *s, int64_t B, int64_t L_kv, int64_t L_act, AbsorbedPlan *p)
{
    Plan base;
    int st = make_plan(s, B, L_kv, L_act, false, &base);
    if (st != HK_OK) return st;
    if (s->n_heads > hk::kAbsorbMaxHeads || B > 65535) return HK_ERR_SHAPE;
    p->M = base.M; p->BH = base.BH; p->scale = base.scale;
    p->Lp = hk::absorbed_row_pitch((int)L_act);
    size_t end = 0;
    auto take = [&](size_t bytes) { const size_t at = end; end += align_up(bytes); return at; };
    p->off_stats = take((size_t)p->M * sizeof(float4));
    p->off_prep = take(L_act > 0 ? prepared_layout(s->d).total : 0);
    const size_t bh = (size_t)p->BH;
    const bool act = L_act > 0;
    p->off_u = take(act ? bh * s->d * 2 : 0);
    p->off_raw = take(act ? bh * p->Lp * 4 : 0);
    p->off_w = take(act ? bh * p->Lp * 2 : 0);
    p->off_sums = take(act ? bh * sizeof(float4) : 0);
    p->off_y = take(act ? bh * s->d * 2 : 0);
    p->off_outc = take(act ? bh * s->head_dim * 2 : 0);
    p->off_lse = take(act ? bh * sizeof(float2) : 0);
    p->off_proj = take(act ? absorbed_proj_floats(s, B) * sizeof(float) : 0);
    p->n_waves = 0;
    p->off_partial = end;
    if (L_kv > 0 && p->BH > 0) {
        p->n_waves = hk::attn_wavefronts(p->BH, L_kv, s->attn_splits);
        take(((size_t)p->n_waves + bh) * (s->head_dim + 2) * sizeof(float));
    }
    p->total = end;
    return HK_OK;
}

}  // namespace

size_t hk_absorbed_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act)
{
    AbsorbedPlan p;
    if (make_absorbed_plan(shape, B, L_kv, L_act, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

int hk_hybrid_decode_attn_absorbed(const hk_shape *shape, const void *q,
                                   const void *K_cache, const void *V_cache, int32_t L_kv,
                                   const void *act, int32_t L_act, int32_t B,
                                   const hk_layer_params *params, float ratio,
                                   void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    AbsorbedPlan p;
    int st = make_absorbed_plan(shape, B, L_kv, L_act, &p);
    if (st != HK_OK) return st;
    const int64_t L = (int64_t)L_kv + L_act;
    if (L == 0) return HK_ERR_SHAPE;
    if (!(ratio >= 0.f && ratio <= 1.f)) return HK_ERR_RATIO;
    if (std::fabs((double)ratio * (double)L - (double)L_kv) > 0.5 + 1e-6 * (double)L) return HK_ERR_RATIO;
    if (B == 0) return HK_OK;
    if (!q || !out || !workspace) return HK_ERR_NULL;
    if (L_kv > 0 && (!K_cache || !V_cache)) return HK_ERR_NULL;
    if (L_act > 0) {
        st = check_params(params);
        if (st != HK_OK) return st;
        if (!act) return HK_ERR_NULL;
        if (!aligned(act, 16)) return HK_ERR_ALIGN;
    }
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(workspace, kAlign)) return HK_ERR_ALIGN;
    if (L_kv > 0 && (!aligned(K_cache, 16) || !aligned(V_cache, 16))) return HK_ERR_ALIGN;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;

    char *ws = static_cast<char *>(workspace);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (L_kv > 0) {
        // the cached segment alone: straight to `out` when there are no checkpoints
        hk::AttnArgs a;
        a.q = q;
        a.K0 = K_cache; a.V0 = V_cache; a.L0 = L_kv;
        a.K1 = nullptr; a.V1 = nullptr; a.L1 = 0;
        a.BH = (int)p.BH; a.head_dim = shape->head_dim; a.scale = p.scale;
        a.n_waves = p.n_waves;
        a.partial = reinterpret_cast<float *>(ws + p.off_partial);
        a.out = L_act > 0 ? static_cast<void *>(ws + p.off_outc) : out;
        a.lse = L_act > 0 ? reinterpret_cast<float2 *>(ws + p.off_lse) : nullptr;
        a.dtype = shape->dtype;
        a.after_main = nullptr;
        if (hk::launch_flash_decode(a, hs) != hipSuccess) return HK_ERR_LAUNCH;
    }
    if (L_act == 0) return HK_OK;

    const PreparedLayout PL = prepared_layout(shape->d);
    const char *pp = static_cast<const char *>(params->prepared);
    if (!pp) {
        char *dst = ws + p.off_prep;
        if (hk::launch_prepare_layer(params->Wkv, params->bkv, params->ln_w, params->ln_b, dst + PL.off_w,
                                     reinterpret_cast<float *>(dst + PL.off_c), reinterpret_cast<float *>(dst + PL.off_b),
                                     shape->d, hs, shape->dtype) != hipSuccess)
            return HK_ERR_LAUNCH;
        pp = dst;
    }
    hk::AbsorbedArgs a;
    a.q = q; a.act = act; a.stats = reinterpret_cast<float4 *>(ws + p.off_stats);
    a.Wp = pp + PL.off_w;
    a.cvec = reinterpret_cast<const float *>(pp + PL.off_c);
    a.bvec = reinterpret_cast<const float *>(pp + PL.off_b);
    a.U = ws + p.off_u;
    a.w_raw = reinterpret_cast<float *>(ws + p.off_raw);
    a.w = ws + p.off_w;
    a.sums = reinterpret_cast<float4 *>(ws + p.off_sums);
    a.Y = ws + p.off_y;
    a.out_c = ws + p.off_outc;
    a.lse_c = reinterpret_cast<const float2 *>(ws + p.off_lse);
    a.out = out;
    a.proj_part = reinterpret_cast<float *>(ws + p.off_proj);
    a.proj_part_floats = absorbed_proj_floats(shape, B);
    a.B = B; a.H = shape->n_heads; a.head_dim = shape->head_dim; a.d = shape->d; a.L_act = L_act; a.L_kv = L_kv;
    a.dt = shape->dtype;
    a.scale = p.scale; a.eps = shape->ln_eps;
    if (hk::launch_absorbed(a, hs) != hipSuccess) return HK_ERR_LAUNCH;
    return HK_OK;
}

size_t hk_qkv_workspace_bytes(const hk_shape *shape, int32_t B)
{
    if (check_shape(shape) != HK_OK || B < 0 || B > (1 << 24)) return 0;
    return kAlign;                                             // the call is one kernel that needs no scratch; the argument stays
}

namespace {

// paged == nullptr: the stores are contiguous (K_dst, V_dst, act_dst with their capacities and positions);
// otherwise they are the pools of *paged and the destination of every row comes from its block table.
int qkv_impl(const hk_shape *shape, const void *x_cur, int32_t B,
             const hk_layer_params *params, const void *Wq, const void *bq,
             void *q_out,
             void *K_dst, void *V_dst, int32_t L_cap, int32_t tok_pos,
             void *act_dst, int32_t act_cap, int32_t act_pos, const hk_paged_cache *paged, const int32_t *store_mask,
             void *workspace, size_t workspace_bytes, void *stream)
{
    int st = check_shape(shape);
    if (st != HK_OK) return st;
    if (B < 0 || B > (1 << 24)) return HK_ERR_SHAPE;
    int blk_log2 = 0;
    if (paged) {
        const int bt = paged->block_tokens;
        if (bt < 16 || bt > 1024 || (bt & (bt - 1)) != 0) return HK_ERR_SHAPE;
        if (paged->P_kv < 0 || paged->P_act < 0 || paged->max_blocks <= 0) return HK_ERR_SHAPE;
        if ((long double)((long double)paged->P_kv + paged->P_act) * bt * shape->d > 4.0e12L) return HK_ERR_SHAPE;
        if ((long double)B * paged->max_blocks > 2.0e9L) return HK_ERR_SHAPE;
        while ((1 << blk_log2) < bt) ++blk_log2;
        // the pools are this call's outputs (the struct declares them const for the calls that only read them)
        K_dst = paged->P_kv > 0 ? const_cast<void *>(paged->K_pool) : nullptr;
        V_dst = paged->P_kv > 0 ? const_cast<void *>(paged->V_pool) : nullptr;
        act_dst = paged->P_act > 0 ? const_cast<void *>(paged->act_pool) : nullptr;
        if (B > 0 && (!paged->block_table || !paged->seq_len)) return HK_ERR_NULL;
        if (B > 0 && paged->P_kv > 0 && (!K_dst || !V_dst)) return HK_ERR_NULL;
        if (B > 0 && paged->P_act > 0 && !act_dst) return HK_ERR_NULL;
        if (!aligned(paged->block_table, 4) || !aligned(paged->seq_len, 4) || !aligned(store_mask, 4)) return HK_ERR_ALIGN;
        L_cap = 1; tok_pos = 0; act_cap = 1; act_pos = 0;
    }
    if ((K_dst == nullptr) != (V_dst == nullptr)) return HK_ERR_NULL;
    if (K_dst && (L_cap <= 0 || tok_pos < 0 || tok_pos >= L_cap)) return HK_ERR_SHAPE;
    if (act_dst && (act_cap <= 0 || act_pos < 0 || act_pos >= act_cap)) return HK_ERR_SHAPE;
    if ((long double)B * (K_dst ? L_cap : 1) * shape->d > 4.0e12L) return HK_ERR_SHAPE;
    if ((long double)B * (act_dst ? act_cap : 1) * shape->d > 4.0e12L) return HK_ERR_SHAPE;
    if (B == 0) return HK_OK;
    st = check_params(params);
    if (st != HK_OK) return st;
    if (!x_cur || !Wq || !bq || !q_out || !workspace) return HK_ERR_NULL;
    if (!aligned(x_cur, 16) || !aligned(Wq, 16) || !aligned(bq, 16) || !aligned(q_out, 16) ||
        !aligned(workspace, kAlign))
        return HK_ERR_ALIGN;
    if (K_dst && (!aligned(K_dst, 16) || !aligned(V_dst, 16))) return HK_ERR_ALIGN;
    if (act_dst && !aligned(act_dst, 16)) return HK_ERR_ALIGN;
    if (workspace_bytes < hk_qkv_workspace_bytes(shape, B)) return HK_ERR_WORKSPACE;

    const int d = shape->d;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    // rows are taken kQkvMaxRows at a time
    for (int32_t b0 = 0; b0 < B; b0 += hk::kQkvMaxRows) {
        hk::QkvArgs a;
        const int rows = B - b0 < hk::kQkvMaxRows ? B - b0 : hk::kQkvMaxRows;
        a.x = static_cast<const char *>(x_cur) + (size_t)b0 * d * 2;
        a.ln_w = params->ln_w; a.ln_b = params->ln_b; a.Wq = Wq; a.bq = bq; a.Wkv = params->Wkv; a.bkv = params->bkv;
        a.q_out = static_cast<char *>(q_out) + (size_t)b0 * d * 2;
        a.K_dst = K_dst ? static_cast<char *>(K_dst) + (paged ? 0 : (size_t)b0 * L_cap * d * 2) : nullptr;
        a.V_dst = V_dst ? static_cast<char *>(V_dst) + (paged ? 0 : (size_t)b0 * L_cap * d * 2) : nullptr;
        a.act_dst = act_dst ? static_cast<char *>(act_dst) + (paged ? 0 : ((size_t)b0 * act_cap + act_pos) * d * 2) : nullptr;
        a.act_row_stride = (int64_t)act_cap * d;
        a.B = rows; a.d = d; a.n_heads = shape->n_heads; a.head_dim = shape->head_dim;
        a.L_cap = L_cap; a.tok_pos = tok_pos; a.eps = shape->ln_eps; a.dtype = shape->dtype;
        a.block_table = nullptr; a.seq_len = nullptr; a.store_mask = nullptr; a.max_blocks = 0; a.blk_log2 = 0; a.P_kv = 0; a.P_act = 0;
        if (paged) {
            a.block_table = paged->block_table + (size_t)b0 * paged->max_blocks; a.seq_len = paged->seq_len + b0;
            a.store_mask = store_mask ? store_mask + b0 : nullptr;
            a.max_blocks = paged->max_blocks; a.blk_log2 = blk_log2; a.P_kv = paged->P_kv; a.P_act = paged->P_act;
        }
        if (hk::launch_qkv_current(a, hs) != hipSuccess) return HK_ERR_LAUNCH;
    }
    return HK_OK;
}

}  // namespace

int hk_qkv_current(const hk_shape *shape, const void *x_cur, int32_t B,
                   const hk_layer_params *params, const void *Wq, const void *bq,
                   void *q_out,
                   void *K_dst, void *V_dst, int32_t L_cap, int32_t tok_pos,
                   void *act_dst, int32_t act_cap, int32_t act_pos,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return qkv_impl(shape, x_cur, B, params, Wq, bq, q_out, K_dst, V_dst, L_cap, tok_pos, act_dst, act_cap, act_pos, nullptr,
                    nullptr, workspace, workspace_bytes, stream);
}

int hk_qkv_current_paged(const hk_shape *shape, const void *x_cur, int32_t B,
                         const hk_layer_params *params, const void *Wq, const void *bq,
                         void *q_out, const hk_paged_cache *cache, const int32_t *store_mask,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cache) return HK_ERR_NULL;
    return qkv_impl(shape, x_cur, B, params, Wq, bq, q_out, nullptr, nullptr, 0, 0, nullptr, 0, 0, cache, store_mask,
                    workspace, workspace_bytes, stream);
}

namespace {

struct PagedPlan {
    int64_t M;                 // rows of the regeneration GEMM: n_act_used * block_tokens
    int n_waves;
    float scale;
    size_t off_k, off_v, off_stats, off_prep, off_partial, total;
};

int make_paged_plan(const hk_shape *s, int64_t B, const hk_paged_cache *c, PagedPlan *p)
{
    int st = check_shape(s);
    if (st != HK_OK) return st;
    if (!c) return HK_ERR_NULL;
    if (B < 0 || B > (1 << 24)) return HK_ERR_SHAPE;
    const int bt = c->block_tokens;
    if (bt < 16 || bt > 1024 || (bt & (bt - 1)) != 0) return HK_ERR_SHAPE;
    if (c->P_kv < 0 || c->P_act < 0 || c->n_act_used < 0 || c->n_act_used > c->P_act || c->max_blocks < 0) return HK_ERR_SHAPE;
    if (c->total_tokens < 0 || c->total_tokens > (int64_t)B * c->max_blocks * bt) return HK_ERR_SHAPE;
    if (c->total_tokens > 0 && c->P_kv == 0 && c->n_act_used == 0) return HK_ERR_SHAPE;      // tokens but no block to hold them
    p->M = (int64_t)c->n_act_used * bt;
    const long double elems = ((long double)c->P_kv + c->P_act) * bt * (long double)s->d;
    if (elems > 4.0e12L || p->M > 0x7fffffffLL || B * s->n_heads > 0x7fffffffLL) return HK_ERR_SHAPE;
    p->scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / std::sqrt((float)s->head_dim);
    const size_t kv_bytes = align_up((size_t)p->M * s->d * 2);
    p->off_k = 0;
    p->off_v = kv_bytes;
    p->off_stats = 2 * kv_bytes;
    size_t end = p->off_stats + align_up((size_t)p->M * sizeof(float2));
    p->off_prep = end;
    if (p->M > 0 && hk::kv_gemm_uses_prepared(p->M, s->d, s->gemm_tile, s->dtype)) end += prepared_layout(s->d).total;
    p->off_partial = end;
    p->n_waves = hk::attn_wavefronts(s->n_heads, c->total_tokens, 0, hk::kPagedResidentWaves);
    end += align_up(((size_t)p->n_waves + (size_t)B * s->n_heads) * (s->head_dim + 2) * sizeof(float));
    p->total = end;
    return HK_OK;
}

}  // namespace

size_t hk_paged_workspace_bytes(const hk_shape *shape, int32_t B, const hk_paged_cache *cache)
{
    PagedPlan p;
    if (make_paged_plan(shape, B, cache, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

int hk_paged_decode_attn(const hk_shape *shape, const void *q, int32_t B, const hk_paged_cache *cache,
                         const hk_layer_params *params, void *out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    PagedPlan p;
    int st = make_paged_plan(shape, B, cache, &p);
    if (st != HK_OK) return st;
    if (B == 0) return HK_OK;
    if (!q || !out || !workspace || !cache->block_table || !cache->seq_len || !cache->cu_tokens) return HK_ERR_NULL;
    if (cache->P_kv > 0 && (!cache->K_pool || !cache->V_pool)) return HK_ERR_NULL;
    if (cache->n_act_used > 0) {
        st = check_params(params);
        if (st != HK_OK) return st;
        if (!cache->act_pool) return HK_ERR_NULL;
        if (!aligned(cache->act_pool, 16)) return HK_ERR_ALIGN;
    }
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(workspace, kAlign)) return HK_ERR_ALIGN;
    if (cache->P_kv > 0 && (!aligned(cache->K_pool, 16) || !aligned(cache->V_pool, 16))) return HK_ERR_ALIGN;
    if (!aligned(cache->block_table, 4) || !aligned(cache->seq_len, 4) || !aligned(cache->cu_tokens, 8)) return HK_ERR_ALIGN;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;

    char *ws = static_cast<char *>(workspace);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    void *K_regen = ws + p.off_k, *V_regen = ws + p.off_v;
    if (cache->n_act_used > 0) {
        // "KV Gen" over the ACT pool: block b of the pool is a sequence of block_tokens checkpoints whose
        // K/V rows land in block b of the regenerated pools, which have the KV pool's layout
        st = regen_impl(shape, cache->act_pool, cache->block_tokens, params, K_regen, V_regen,
                        cache->block_tokens, 0, reinterpret_cast<float2 *>(ws + p.off_stats), ws + p.off_prep, p.M, hs,
                        Marks{nullptr, 0, nullptr});
        if (st != HK_OK) return st;
    }
    hk::PagedAttnArgs a;
    a.q = q;
    a.K_pool = cache->K_pool; a.V_pool = cache->V_pool;
    a.K_regen = cache->n_act_used > 0 ? K_regen : nullptr; a.V_regen = cache->n_act_used > 0 ? V_regen : nullptr;
    a.block_table = cache->block_table; a.seq_len = cache->seq_len; a.cu_tokens = cache->cu_tokens;
    a.total_tokens = cache->total_tokens; a.max_blocks = cache->max_blocks;
    a.P_kv = cache->P_kv; a.P_act = cache->n_act_used; a.block_tokens = cache->block_tokens;
    a.B = B; a.H = shape->n_heads; a.head_dim = shape->head_dim; a.scale = p.scale; a.n_waves = p.n_waves;
    a.partial = reinterpret_cast<float *>(ws + p.off_partial);
    a.out = out;
    // the kernels take the number of tokens from the device (cu_tokens[B]); the host's total_tokens sizes the launch
    a.total_dev = cache->cu_tokens + B; a.lse = nullptr; a.dtype = shape->dtype;
    if (hk::launch_paged_decode(a, hs) != hipSuccess) return HK_ERR_LAUNCH;
    return HK_OK;
}

namespace {

struct PagedAbsorbedPlan {
    int n_waves, Lp;
    float scale;
    size_t off_stats, off_prep, off_u, off_raw, off_w, off_sums, off_y, off_outc, off_lse, off_list, off_count, off_last,
        off_rows, off_kvtab, off_kvlen, off_kvcu, off_proj, off_partial, total;
};

int make_paged_absorbed_plan(const hk_shape *s, int64_t B, const hk_paged_cache *c, PagedAbsorbedPlan *p)
{
    PagedPlan base;                                        // the checks of the paged step
    int st = make_paged_plan(s, B, c, &base);
    if (st != HK_OK) return st;
    if (s->n_heads > hk::kAbsorbMaxHeads || B > 65535) return HK_ERR_SHAPE;
    const int64_t max_rows = (int64_t)c->max_blocks * c->block_tokens;     // the most checkpoint rows a request can have
    if (max_rows > (1 << 28) || B * c->max_blocks > 0x7fffffffLL) return HK_ERR_SHAPE;
    p->scale = base.scale;
    p->Lp = hk::absorbed_row_pitch((int)max_rows);
    const bool act = c->n_act_used > 0;
    const size_t b = (size_t)B, bh = b * s->n_heads;
    size_t end = 0;
    auto take = [&](size_t bytes) { const size_t at = end; end += align_up(bytes); return at; };
    p->off_stats = take(act ? b * p->Lp * sizeof(float4) : 0);
    p->off_prep = take(act ? prepared_layout(s->d).total : 0);
    p->off_u = take(act ? bh * s->d * 2 : 0);
    p->off_raw = take(act ? bh * p->Lp * 4 : 0);
    p->off_w = take(act ? bh * p->Lp * 2 : 0);
    p->off_sums = take(act ? bh * sizeof(float4) : 0);
    p->off_y = take(act ? bh * s->d * 2 : 0);
    p->off_outc = take(act ? bh * s->head_dim * 2 : 0);
    p->off_lse = take(act ? bh * sizeof(float2) : 0);
    p->off_list = take(act ? b * c->max_blocks * sizeof(int32_t) : 0);
    p->off_count = take(act ? b * sizeof(int32_t) : 0);
    p->off_last = take(act ? b * sizeof(int32_t) : 0);
    p->off_rows = take(act ? b * sizeof(int32_t) : 0);
    p->off_kvtab = take(act ? b * c->max_blocks * sizeof(int32_t) : 0);
    p->off_kvlen = take(act ? b * sizeof(int32_t) : 0);
    p->off_kvcu = take(act ? (b + 1) * sizeof(int64_t) : 0);
    p->off_proj = take(act ? absorbed_proj_floats(s, B) * sizeof(float) : 0);
    p->off_partial = end;
    // the attention over the KV blocks alone: sized for every token being cached (the device knows the true number)
    p->n_waves = hk::attn_wavefronts(s->n_heads, c->total_tokens, 0, hk::kPagedResidentWaves);
    take(((size_t)p->n_waves + bh) * (s->head_dim + 2) * sizeof(float));
    p->total = end;
    return HK_OK;
}

}  // namespace

size_t hk_paged_absorbed_workspace_bytes(const hk_shape *shape, int32_t B, const hk_paged_cache *cache)
{
    PagedAbsorbedPlan p;
    if (make_paged_absorbed_plan(shape, B, cache, &p) != HK_OK) return 0;
    return p.total > 0 ? p.total : kAlign;
}

int hk_paged_decode_attn_absorbed(const hk_shape *shape, const void *q, int32_t B, const hk_paged_cache *cache,
                                  const hk_layer_params *params, void *out,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    PagedAbsorbedPlan p;
    int st = make_paged_absorbed_plan(shape, B, cache, &p);
    if (st != HK_OK) return st;
    if (B == 0) return HK_OK;
    if (!q || !out || !workspace || !cache->block_table || !cache->seq_len || !cache->cu_tokens) return HK_ERR_NULL;
    if (cache->P_kv > 0 && (!cache->K_pool || !cache->V_pool)) return HK_ERR_NULL;
    if (cache->n_act_used > 0) {
        st = check_params(params);
        if (st != HK_OK) return st;
        if (!cache->act_pool) return HK_ERR_NULL;
        if (!aligned(cache->act_pool, 16)) return HK_ERR_ALIGN;
    }
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(workspace, kAlign)) return HK_ERR_ALIGN;
    if (cache->P_kv > 0 && (!aligned(cache->K_pool, 16) || !aligned(cache->V_pool, 16))) return HK_ERR_ALIGN;
    if (!aligned(cache->block_table, 4) || !aligned(cache->seq_len, 4) || !aligned(cache->cu_tokens, 8)) return HK_ERR_ALIGN;
    if (workspace_bytes < p.total) return HK_ERR_WORKSPACE;

    char *ws = static_cast<char *>(workspace);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const bool act = cache->n_act_used > 0;
    const bool kv = cache->P_kv > 0;
    hk::PagedAttnArgs t;
    t.q = q;
    t.K_pool = cache->K_pool; t.V_pool = cache->V_pool;
    t.K_regen = nullptr; t.V_regen = nullptr;
    t.block_table = cache->block_table; t.seq_len = cache->seq_len; t.cu_tokens = cache->cu_tokens;
    t.total_tokens = cache->total_tokens; t.max_blocks = cache->max_blocks;
    t.P_kv = cache->P_kv; t.P_act = 0; t.block_tokens = cache->block_tokens;
    t.B = B; t.H = shape->n_heads; t.head_dim = shape->head_dim; t.scale = p.scale; t.n_waves = p.n_waves;
    t.partial = reinterpret_cast<float *>(ws + p.off_partial);
    t.out = out; t.total_dev = cache->cu_tokens ? cache->cu_tokens + B : nullptr; t.lse = nullptr; t.dtype = shape->dtype;
    if (!act) {                                            // no checkpoint block in use: the block-table attention is the whole step
        if (hk::launch_paged_decode(t, hs) != hipSuccess) return HK_ERR_LAUNCH;
        return HK_OK;
    }

    const PreparedLayout PL = prepared_layout(shape->d);
    const char *pp = static_cast<const char *>(params->prepared);
    if (!pp) {
        char *dst = ws + p.off_prep;
        if (hk::launch_prepare_layer(params->Wkv, params->bkv, params->ln_w, params->ln_b, dst + PL.off_w,
                                     reinterpret_cast<float *>(dst + PL.off_c), reinterpret_cast<float *>(dst + PL.off_b),
                                     shape->d, hs, shape->dtype) != hipSuccess)
            return HK_ERR_LAUNCH;
        pp = dst;
    }
    hk::PagedAbsorbedArgs pa;
    hk::AbsorbedArgs &a = pa.abs;
    a.q = q; a.act = cache->act_pool; a.stats = reinterpret_cast<float4 *>(ws + p.off_stats);
    a.Wp = pp + PL.off_w;
    a.cvec = reinterpret_cast<const float *>(pp + PL.off_c);
    a.bvec = reinterpret_cast<const float *>(pp + PL.off_b);
    a.U = ws + p.off_u;
    a.w_raw = reinterpret_cast<float *>(ws + p.off_raw);
    a.w = ws + p.off_w;
    a.sums = reinterpret_cast<float4 *>(ws + p.off_sums);
    a.Y = ws + p.off_y;
    a.out_c = ws + p.off_outc;
    a.lse_c = reinterpret_cast<const float2 *>(ws + p.off_lse);
    a.out = out;
    a.proj_part = reinterpret_cast<float *>(ws + p.off_proj);
    a.proj_part_floats = absorbed_proj_floats(shape, B);
    a.B = B; a.H = shape->n_heads; a.head_dim = shape->head_dim; a.d = shape->d;
    a.L_act = cache->max_blocks * cache->block_tokens; a.L_kv = kv ? 1 : 0;
    a.dt = shape->dtype;
    a.scale = p.scale; a.eps = shape->ln_eps;
    pa.block_table = cache->block_table; pa.seq_len = cache->seq_len;
    pa.max_blocks = cache->max_blocks; pa.block_tokens = cache->block_tokens; pa.n_act_used = cache->n_act_used;
    pa.list = reinterpret_cast<int32_t *>(ws + p.off_list);
    pa.count = reinterpret_cast<int32_t *>(ws + p.off_count);
    pa.last_rows = reinterpret_cast<int32_t *>(ws + p.off_last);
    pa.n_rows = reinterpret_cast<int32_t *>(ws + p.off_rows);
    pa.kv_table = reinterpret_cast<int32_t *>(ws + p.off_kvtab);
    pa.kv_len = reinterpret_cast<int32_t *>(ws + p.off_kvlen);
    pa.kv_cu = reinterpret_cast<int64_t *>(ws + p.off_kvcu);
    if (hk::launch_paged_index(pa, hs) != hipSuccess) return HK_ERR_LAUNCH;
    if (kv) {
        // attention over the cached tokens alone, through the KV view of the table; how many there are only the
        // device knows (the launch is sized for all tokens being cached)
        t.block_table = pa.kv_table; t.seq_len = pa.kv_len; t.cu_tokens = pa.kv_cu; t.total_dev = pa.kv_cu + B;
        t.out = ws + p.off_outc;
        t.lse = reinterpret_cast<float2 *>(ws + p.off_lse);
        if (hk::launch_paged_decode(t, hs) != hipSuccess) return HK_ERR_LAUNCH;
    }
    if (hk::launch_paged_absorbed(pa, hs) != hipSuccess) return HK_ERR_LAUNCH;
    return HK_OK;
}

const char *hk_status_string(int status)
{
    switch (status) {
    case HK_OK: return "HK_OK";
    case HK_ERR_NULL: return "HK_ERR_NULL: a required pointer is NULL";
    case HK_ERR_SHAPE: return "HK_ERR_SHAPE: unsupported or inconsistent sizes";
    case HK_ERR_RATIO: return "HK_ERR_RATIO: ratio outside [0,1] or inconsistent with L_kv, L_act";
    case HK_ERR_ALIGN: return "HK_ERR_ALIGN: pointer not sufficiently aligned";
    case HK_ERR_WORKSPACE: return "HK_ERR_WORKSPACE: workspace too small";
    case HK_ERR_DTYPE: return "HK_ERR_DTYPE: unsupported dtype";
    case HK_ERR_LAUNCH: return "HK_ERR_LAUNCH: HIP reported a launch error";
    case HK_ERR_STATIC_LIMIT: return "HK_ERR_STATIC_LIMIT: the problem needs more scratch than the library's static buffer (HK_STATIC_SCRATCH_BYTES) holds";
    default: return "unknown hk_status";
    }
}

}  // extern "C"

int hk_paged_append(int32_t *block_table, int32_t *seq_len, int64_t *cu_tokens, int32_t *counters, const int32_t *active,
                    int32_t *grew, int32_t B, int32_t max_blocks, int32_t block_tokens, int32_t P_kv, int32_t P_act,
                    int64_t act_host, int64_t kv_host, void *stream)
{
    if (B < 0 || B > 65535 || max_blocks <= 0 || P_kv < 0 || P_act < 0) return HK_ERR_SHAPE;
    if (block_tokens < 16 || block_tokens > 1024 || (block_tokens & (block_tokens - 1)) != 0) return HK_ERR_SHAPE;
    if ((long double)max_blocks * block_tokens > 2.0e9L) return HK_ERR_SHAPE;
    if (act_host < 0 || kv_host < 0 || act_host + kv_host == 0 || act_host > (1LL << 31) || kv_host > (1LL << 31)) return HK_ERR_SHAPE;
    if (B == 0) return HK_OK;
    if (!block_table || !seq_len || !cu_tokens || !counters) return HK_ERR_NULL;
    if (!aligned(block_table, 4) || !aligned(seq_len, 4) || !aligned(cu_tokens, 8) || !aligned(counters, 4) || !aligned(active, 4) ||
        !aligned(grew, 4))
        return HK_ERR_ALIGN;
    hk::PagedAppendArgs a;
    a.block_table = block_table; a.seq_len = seq_len; a.cu_tokens = cu_tokens; a.counters = counters; a.active = active; a.grew = grew;
    a.B = B; a.max_blocks = max_blocks; a.block_tokens = block_tokens; a.P_kv = P_kv; a.P_act = P_act;
    a.act_host = act_host; a.kv_host = kv_host;
    if (hk::launch_paged_append(a, static_cast<hipStream_t>(stream)) != hipSuccess) return HK_ERR_LAUNCH;
    return HK_OK;
}
