// Cache-management policy arithmetic on the host (Sec. 4.3): the linear time models and their
// least-squares fit (the regression over sampled token counts), the two-step host block allocation
// (Algorithm 1), the ratio-keeping choice of the next block type (Eq. 11) and the mini-batch balance
// metric (Eq. 12, 13).  Plain double arithmetic, no device code, no allocation.
#include "../../include/hybridkv.h"

#include <cmath>

namespace {

inline bool finite_line(const hk_line *l) { return l && std::isfinite(l->slope) && std::isfinite(l->offset); }
inline double eval(const hk_line &l, double n) { return l.slope * n + l.offset; }
// n with T(n) = t, not below zero
inline double solve_for(const hk_line &l, double t)
{
    const double n = (t - l.offset) / l.slope;
    return n > 0.0 ? n : 0.0;
}

}  // namespace

extern "C" {

int hk_fit_line(const double *n, const double *t, int32_t count, hk_line *line, double *r2)
{
    if (!n || !t || !line) return HK_ERR_NULL;
    if (count < 2) return HK_ERR_SHAPE;
    double sn = 0, st = 0;
    for (int32_t i = 0; i < count; ++i) { sn += n[i]; st += t[i]; }
    const double mn = sn / count, mt = st / count;
    double snn = 0, snt = 0, stt = 0;
    for (int32_t i = 0; i < count; ++i) {
        const double dn = n[i] - mn, dt = t[i] - mt;
        snn += dn * dn; snt += dn * dt; stt += dt * dt;
    }
    if (!(snn > 0.0) || !std::isfinite(snn) || !std::isfinite(snt)) return HK_ERR_SHAPE;   // all n equal, or bad input
    line->slope = snt / snn;
    line->offset = mt - line->slope * mn;
    if (r2) {
        double res = 0;
        for (int32_t i = 0; i < count; ++i) {
            const double e = t[i] - (line->slope * n[i] + line->offset);
            res += e * e;
        }
        *r2 = stt > 0.0 ? 1.0 - res / stt : 1.0;
    }
    return HK_OK;
}

int hk_host_block_allocation(const hk_alloc_params *p, hk_alloc_result *out)
{
    if (!p || !out) return HK_ERR_NULL;
    if (!finite_line(&p->T_kv_gen) || !finite_line(&p->T_load_kv)) return HK_ERR_SHAPE;
    if (!(p->T_kv_gen.slope > 0.0) || !(p->T_load_kv.slope > 0.0)) return HK_ERR_SHAPE;
    if (!(p->S_kv > 0.0) || !std::isfinite(p->S_kv) || !std::isfinite(p->T_load_w) || !(p->T_load_w >= 0.0)) return HK_ERR_SHAPE;
    if (!(p->n_act_gpu >= 0.0) || !std::isfinite(p->n_act_gpu)) return HK_ERR_SHAPE;
    if (!std::isfinite(p->M_host) || !std::isfinite(p->S_weight) || !(p->S_weight >= 0.0)) return HK_ERR_SHAPE;
    const hk_line &gen = p->T_kv_gen, &load = p->T_load_kv;

    // First stage (Algorithm 1, initial allocation).  While one layer's weights cross the link the GPU
    // regenerates its resident checkpoints; `gap` is how much longer the link is busy.  A positive gap is
    // closed by host checkpoints whose regeneration lasts that long, a negative one by host KV blocks whose
    // transfer lasts that long.  Whole blocks only.
    const double gap = p->T_load_w - eval(gen, p->n_act_gpu);
    const double first_act = gap >= 0.0 ? std::floor(solve_for(gen, gap)) : 0.0;
    const double first_kv = gap >= 0.0 ? 0.0 : std::floor(solve_for(load, -gap));

    // Second stage (Algorithm 1, remaining allocation).  Count the bytes that are left in units of a checkpoint
    // block (half a KV block): u = 2 * bytes / S_kv.  The split (x checkpoint, y KV blocks) fills them,
    //     x + 2 y = u,
    // and takes equal time on both sides,
    //     gen.slope x + gen.offset = load.slope y + load.offset.
    // Eliminating x:  y = (gen.slope u + gen.offset - load.offset) / (load.slope + 2 gen.slope),  x = u - 2 y.
    // A negative count means one kind alone is already the slower side: it gets nothing, the other kind all.
    const double bytes_left = p->M_host - p->S_weight - 0.5 * p->S_kv * first_act - p->S_kv * first_kv;
    double x = 0.0, y = 0.0;
    if (bytes_left > 0.0) {
        const double u = 2.0 * bytes_left / p->S_kv;
        y = (gen.slope * u + gen.offset - load.offset) / (load.slope + 2.0 * gen.slope);
        x = u - 2.0 * y;
        if (x < 0.0) { x = 0.0; y = 0.5 * u; }
        if (y < 0.0) { y = 0.0; x = u; }
    }
    x = std::floor(x);
    y = std::floor(y);
    // counts are reported as 64-bit integers: anything that does not fit comfortably is an input error
    const double limit = 4611686018427387904.0;                           // 2^62
    const double all[4] = {first_act, first_kv, x, y};
    for (double v : all)
        if (!(v >= 0.0) || !(v < limit)) return HK_ERR_SHAPE;
    if (!(first_act + x < limit) || !(first_kv + y < limit)) return HK_ERR_SHAPE;
    out->act_init = (int64_t)first_act;
    out->kv_init = (int64_t)first_kv;
    out->act_remain = (int64_t)x;
    out->kv_remain = (int64_t)y;
    out->act_host = out->act_init + out->act_remain;
    out->kv_host = out->kv_init + out->kv_remain;
    return HK_OK;
}

int hk_next_block_type(int64_t n_act, int64_t n_kv, int64_t act_host, int64_t kv_host)
{
    if (n_act < 0 || n_kv < 0 || act_host < 0 || kv_host < 0 || act_host + kv_host == 0) return HK_ERR_SHAPE;
    if (n_act > (1LL << 31) || n_kv > (1LL << 31) || act_host > (1LL << 31) || kv_host > (1LL << 31)) return HK_ERR_SHAPE;
    if (kv_host == 0) return HK_BLOCK_ACT;
    if (act_host == 0) return HK_BLOCK_KV;
    // After the allocation the request has n + 1 blocks.  Its checkpoint share would be
    // (n_act + 1) / (n + 1) or n_act / (n + 1); take the one nearer act_host / (act_host + kv_host).
    // In integers, with T = act_host + kv_host:  |(n_act + 1) T - act_host (n + 1)|  vs  |n_act T - act_host (n + 1)|.
    const int64_t T = act_host + kv_host, n1 = n_act + n_kv + 1;
    const int64_t dev_act = (n_act + 1) * T - act_host * n1, dev_kv = n_act * T - act_host * n1;
    const int64_t a = dev_act < 0 ? -dev_act : dev_act, k = dev_kv < 0 ? -dev_kv : dev_kv;
    return a <= k ? HK_BLOCK_ACT : HK_BLOCK_KV;                       // a tie goes to the smaller block
}

int hk_minibatch_balance(const hk_line *T_kv_gen, const hk_line *T_load_kv, double n_act_mb, double n_kv_mb,
                         double *balance, double *cost)
{
    if (!T_kv_gen || !T_load_kv || !balance || !cost) return HK_ERR_NULL;
    if (!finite_line(T_kv_gen) || !finite_line(T_load_kv) || !(n_act_mb >= 0.0) || !(n_kv_mb >= 0.0)) return HK_ERR_SHAPE;
    const double tg = eval(*T_kv_gen, n_act_mb), tl = eval(*T_load_kv, n_kv_mb);
    if (!(tg > 0.0) || !(tl > 0.0)) return HK_ERR_SHAPE;
    *balance = tg / tl;
    *cost = *balance > 1.0 / *balance ? *balance : 1.0 / *balance;
    return HK_OK;
}

}  // extern "C"
