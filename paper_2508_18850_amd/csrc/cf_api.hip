// C ABI of libcfdecode: handle, argument validation, work plan, launch.
#include "../../include/cfdecode.h"
#include "cf_params.h"

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

using cf::Params;

struct cf_handle_s {
    cf_config cfg;
    int device = 0;
    int num_cu = 0;
    int G = 1;
    int nqkv = 0;
    int nch = 0;
    // workspace (one allocation)
    char *ws = nullptr;
    size_t ws_bytes = 0;
    size_t counters_bytes = 0;
    size_t exchange_bytes = 0;   // counters + exchange slots: cleared together (stamps restart at 1)
    uint32_t *err = nullptr;
    unsigned long long *done = nullptr;
    uint64_t *p1 = nullptr, *p2 = nullptr, *p3 = nullptr;
    float *dbg_q = nullptr, *dbg_attn = nullptr;
    unsigned long long *dbg_t = nullptr;
    uint16_t *chain[2] = {nullptr, nullptr};   // hidden states between the layers of a stack, [max_batch, d_model] each
    uint64_t *xslots = nullptr;                // the same between the layers of a one-launch stack: stamped fp32, [max_batch, d_model]
    // tuning
    int tune_w = 0, tune_ks = 0, tune_ns = 0;
    int balance_rows = 0, balance_tokens = 32;   // half the length difference between even and odd splits (-1: off)
    long long spin_ticks = 200000000LL;   // 2 s of the 100 MHz wall clock
    int wg_per_cu[6] = {0, 0, 0, 0, 0, 0};   // resident workgroups per CU for batch tiles 1, 4, 16 of the block kernel,
                                          // then of the layer kernel (0 = not probed)
    int last_batch = 0;
    int last_plan[10] = {0};
    int last_hip = 0;
    // cf_decode_block_static: the exchange slots are laid out per call, for the plan in use, inside this area
    char *slot_area = nullptr;
    size_t slot_area_bytes = 0;
};

namespace {

int ceil_div(int a, int b) { return (a + b - 1) / b; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Register tile of the batch rows: 1, 4 (vector units) or 16 (MFMA).  The 16-row tile also wins at batch 3 and 4
// (Llama-3-8B shape, batch 3 / 4: 52.2 / 46.9 against 54.9 / 48.3 us; Llama-2-7B shape, batch 4: 73.4 against 74.8 us).
// Without MFMA tiles (head_dim 64) the 16-row tile is the vector variant with 128 accumulators per thread: there the
// 4-row tile keeps batch 3 and 4.
int batch_tile(int batch, int head_dim) { return batch <= 1 ? 1 : batch <= (cf::mfma_tiles(head_dim, 16) ? 2 : 4) ? 4 : 16; }
int tile_index(int bt) { return bt == 1 ? 0 : bt == 4 ? 1 : 2; }

constexpr int kMaxKS = 32;
constexpr size_t kLdsLimit = 160 * 1024 - 256;   // LDS per workgroup on gfx950, minus the static flags

bool aligned16(const void *p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int default_workgroups(const cf_handle_s *h)
{
    int w = h->tune_w > 0 ? h->tune_w : h->num_cu;
    w -= w % h->cfg.n_kv_heads;
    return w;
}

// Fill the work split of one call.  Returns CF_OK or an error.
int make_plan(const cf_handle_s *h, int batch, int pos, Params *p)
{
    const cf_config &c = h->cfg;
    const int hd = c.head_dim, G = h->G, bt = batch_tile(batch, c.head_dim);
    const int W = default_workgroups(h);
    if (W <= 0) return CF_EUNSUPPORTED;
    const int TS = W / c.n_kv_heads;
    p->W = W;
    p->TS = TS;

    // projection: split the reduction dimension so that (G+2)*KS items balance over TS members
    {
        int best = 0;
        long best_cost = 0;
        for (int ks = 1; ks <= kMaxKS && ks <= TS; ++ks) {
            if (TS % ks) continue;              // every member keeps one slice for all its selectors
            if (h->tune_ks > 0 && ks != h->tune_ks) continue;
            const int rps = ceil_div(c.d_model, ks);
            if (rps < 8 && ks > 1) continue;
            if ((long)(ks - 1) * rps >= c.d_model) continue;   // no empty slice
            const int maxi = bt == 1 ? 4 : (bt <= 4 ? 2 : 1);
            const size_t lds = (cf::x_lds_floats(hd, bt, rps) + (size_t)maxi * cf::kWaves * bt * hd) * sizeof(float);
            if (lds > kLdsLimit) continue;
            const int dsel = TS / ks;
            // rows a member streams, plus what its consumers pay for every further slice: KS partial sums per projected
            // value to fetch, for every batch row (weighed by measurements on the grouped-query shapes: the
            // Llama-3-8B shape takes 8 slices from batch 3 on, 16 below; the Llama-2-70B shape stays at 16)
            const long cost = (long)(ceil_div(G, dsel) + ceil_div(2, dsel)) * rps + 12L * ks * (bt < 4 ? bt : 4);
            if (!best || cost < best_cost) {
                best = ks;
                best_cost = cost;
            }
        }
        if (!best) return h->tune_ks > 0 ? CF_EINVAL : CF_EUNSUPPORTED;
        p->KS = best;
        p->RB = ceil_div(c.d_model, best);
        // uneven slices (see the kernel's workgroup mapping): only when member parity == slice parity
        p->pairmap = (TS % 2 == 0 && W % 2 == 0 && h->balance_rows >= 0) ? 1 : 0;
        p->RD = 0;
        if (p->pairmap && best % 2 == 0 && p->RB * best == c.d_model && p->RB >= 8 * h->balance_rows) {
            const int maxi = bt == 1 ? 4 : (bt <= 4 ? 2 : 1);
            const size_t lds = (cf::x_lds_floats(hd, bt, p->RB + h->balance_rows) + (size_t)maxi * cf::kWaves * bt * hd) * sizeof(float);
            if (lds <= kLdsLimit) p->RD = h->balance_rows;
        }
        p->RPS = p->RB + p->RD;
    }
    // attention: split the cached sequence so that B*NS items balance over TS members
    {
        const int rows_per_step = cf::kThreads / (hd / 8);
        int best = 0;
        long best_cost = 0;
        for (int ns = 1; ns <= cf::kMaxKvSplits; ns *= 2) {
            if (h->tune_ns > 0 && ns != h->tune_ns) continue;
            // One item per member at most, where the batch allows it: a second round of items costs far more than
            // its rows (measured on the Llama-3-8B shape, 8192 rows, 32 members: batch 3 with 8 / 16 / 32 splits 44.1 /
            // 48.9 / 54.9 us, batch 5 with 4 / 8 / 16 / 32 splits 55.2 / 64.7 / 68.0 / 85.8 us, batch 12 with 2 / 4 / 8
            // splits 87.5 / 97.3 / 96.2 us)
            // (with more batch rows than members there are several rounds anyway and the cost below decides: Llama-2-7B
            // shape, 8 members, batch 12: 160.2 us with 2 splits, three full rounds, against 167.8 us with 1)
            if (h->tune_ns == 0 && ns > 1 && batch * ns > TS && batch <= TS) continue;
            int tps = ceil_div(ceil_div(pos, ns), rows_per_step) * rows_per_step;
            if (tps == 0) tps = rows_per_step;
            const long cost = (long)ceil_div(batch * ns, TS) * (tps + 64);
            if (!best || cost < best_cost) {
                best = ns;
                best_cost = cost;
            }
        }
        if (!best) return CF_EINVAL;
        p->NS = best;
        // the member with the last split also sums, rotates, appends and scores the new token:
        // its split is made shorter by about that much work
        const int discount = best > 1 ? 64 : 0;
        int tps = ceil_div(pos + discount, best);
        if (tps * (best - 1) > pos) tps = ceil_div(pos, best);
        p->TPS = tps > 0 ? tps : 1;
        p->TD = 0;
        if (p->pairmap && best % 2 == 0 && TS % best == 0 && p->TPS >= 8 * h->balance_tokens) p->TD = h->balance_tokens;
        // A workgroup walks its split in batches of 8 * rows_per_step cached rows.  When the rows divide into whole
        // batches per split, equal splits keep every workgroup at the same number of batches; the discount and the
        // even/odd difference would push half of them into one more (measured: 0.2 - 0.6 us per step).
        if (pos > 0 && pos % (best * 8 * rows_per_step) == 0) {
            p->TPS = pos / best;
            p->TD = 0;
        }
    }
    // output projection: G heads x NC3 column blocks x RS3 row splits per team
    {
        const int nch = h->nch;
        int best_nc = 0, best_rs = 0;
        double best_cost = 0;
        for (int rs = 1; rs <= 8 && hd / rs >= cf::kWaves; rs *= 2) {
            for (int nc = 1; nc <= nch; nc *= 2) {
                const int cw = ceil_div(nch, nc) * cf::kOutChunk;
                const double cost = (double)ceil_div(G * nc * rs, TS) * (hd / rs) * cw;
                if (!best_nc || cost < best_cost * 0.999) {
                    best_nc = nc;
                    best_rs = rs;
                    best_cost = cost;
                }
            }
        }
        p->NC3 = best_nc;
        p->RS3 = best_rs;
        p->CW3 = ceil_div(nch, best_nc) * cf::kOutChunk;
        p->NC3 = ceil_div(nch * cf::kOutChunk, p->CW3);
    }
    p->DSEL = TS / p->KS;
    auto log2_or_minus1 = [](int v) {
        for (int k = 0; k < 31; ++k)
            if ((1 << k) == v) return k;
        return -1;
    };
    p->sh_nkv = log2_or_minus1(c.n_kv_heads);
    p->sh_ks = log2_or_minus1(p->KS);
    p->sh_dsel = log2_or_minus1(p->DSEL);
    p->sh_ns = log2_or_minus1(p->NS);
    return CF_OK;
}

void fill_static(const cf_handle_s *h, Params *p)
{
    const cf_config &c = h->cfg;
    p->done = h->done;
    p->err = h->err;
    p->p1 = h->p1;
    p->p2 = h->p2;
    p->p3 = h->p3;
    p->rope_log2_base = std::log2((double)c.rope_base);
    p->dbg_q = (c.flags & CF_FLAG_DEBUG_EXPORT) ? h->dbg_q : nullptr;
    p->dbg_attn = (c.flags & CF_FLAG_DEBUG_EXPORT) ? h->dbg_attn : nullptr;
    p->dbg_t = (c.flags & CF_FLAG_DEBUG_EXPORT) ? h->dbg_t : nullptr;
    p->D = c.d_model;
    p->nq = c.n_q_heads;
    p->nkv = c.n_kv_heads;
    p->max_seq = c.max_seq;
    p->nqkv = h->nqkv;
    p->qk_scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)c.head_dim));
    p->spin_ticks = (uint32_t)(h->spin_ticks > 0xffffffffLL ? 0xffffffffLL : h->spin_ticks);
}

int hip_fail(cf_handle_s *h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return CF_EHIP;
}

// Check (once per batch tile) that the whole grid can be resident at the same time.
int check_residency(cf_handle_s *h, const Params &p, int bt, size_t lds_bytes)
{
    const bool layer = cf::wants_layer_kernel(p);
    int &slot = h->wg_per_cu[tile_index(bt) + (layer ? 3 : 0)];
    if (slot == 0) {
        int n = 0;
        hipError_t e = cf::max_workgroups_per_cu(h->cfg.head_dim, h->G, bt, lds_bytes, layer, &n);
        if (e != hipSuccess) return hip_fail(h, e);
        slot = n > 0 ? n : -1;
    }
    if (slot < 0 || (long)slot * h->num_cu < p.W) return CF_EUNSUPPORTED;
    return CF_OK;
}

}  // namespace

extern "C" {

// Shape checks common to cf_create and cf_decode_block_static.
static int check_config(const cf_config &c)
{
    if (c.d_model < 8 || c.d_model % 8 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads ||
        c.max_batch < 1 || c.max_batch > 16 || c.max_seq < 1 || !(c.rope_base > 1.0f))
        return CF_EINVAL;
    if (c.head_dim != 64 && c.head_dim != 128) return CF_EUNSUPPORTED;
    {
        // the kernel addresses each tensor with 32-bit byte offsets
        const unsigned long long lim = 0x7fffffffull;
        const unsigned long long nqkv = (unsigned long long)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
        if (2ull * c.d_model * nqkv + 256ull * (nqkv / c.head_dim) > lim || 2ull * c.n_q_heads * c.head_dim * c.d_model > lim ||
            2ull * c.max_seq * c.head_dim > lim)
            return CF_EUNSUPPORTED;
    }
    const int G = c.n_q_heads / c.n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return CF_EUNSUPPORTED;
    return CF_OK;
}

int cf_create(const cf_config *cfg, cf_handle *out)
{
    if (!cfg || !out) return CF_EINVAL;
    *out = nullptr;
    const cf_config &c = *cfg;
    const int cfg_rc = check_config(c);
    if (cfg_rc != CF_OK) return cfg_rc;
    const int G = c.n_q_heads / c.n_kv_heads;

    cf_handle_s *h = new (std::nothrow) cf_handle_s();
    if (!h) return CF_ENOMEM;
    h->cfg = c;
    h->G = G;
    h->nqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    h->nch = ceil_div(c.d_model, cf::kOutChunk);

    hipError_t e = hipGetDevice(&h->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, h->device);
    if (e != hipSuccess) {
        delete h;
        return CF_EHIP;
    }
    h->num_cu = prop.multiProcessorCount;
    if (c.n_kv_heads > h->num_cu) {
        delete h;
        return CF_EUNSUPPORTED;
    }

    const size_t B = (size_t)c.max_batch, hd = (size_t)c.head_dim;
    // error flag, then one launch counter per workgroup, each in a 128-byte line of its own
    h->counters_bytes = 256 + (size_t)8 * h->num_cu * cf::kCounterStride * sizeof(unsigned long long);
    const size_t p1_bytes = align_up((size_t)kMaxKS * B * h->nqkv * sizeof(uint64_t), 256);
    const size_t p2_bytes = align_up(B * c.n_q_heads * cf::kMaxKvSplits * (hd + cf::kP2Stride) * sizeof(uint64_t), 256);
    const size_t p3_bytes = align_up((size_t)c.n_q_heads * 8 * B * c.d_model * sizeof(uint64_t), 256);
    if (p1_bytes > 0xfffffff0ull || p2_bytes > 0xfffffff0ull || p3_bytes > 0xfffffff0ull) {   // slots are addressed with 32-bit byte offsets
        delete h;
        return CF_EUNSUPPORTED;
    }
    const size_t dbg_bytes = align_up(B * c.n_q_heads * hd * sizeof(float), 256);
    const size_t times_bytes = align_up((size_t)8 * h->num_cu * cf::kStamps * sizeof(unsigned long long), 256);
    h->exchange_bytes = h->counters_bytes + p1_bytes + p2_bytes + p3_bytes;
    const size_t chain_bytes = align_up(B * c.d_model * sizeof(uint16_t), 256);
    const size_t xslot_bytes = align_up(B * c.d_model * sizeof(uint64_t), 256);
    h->exchange_bytes += xslot_bytes;
    h->ws_bytes = h->counters_bytes + p1_bytes + p2_bytes + p3_bytes + xslot_bytes + 2 * dbg_bytes + times_bytes +
                  2 * chain_bytes;
    e = hipMalloc(reinterpret_cast<void **>(&h->ws), h->ws_bytes);
    if (e != hipSuccess) {
        delete h;
        return e == hipErrorOutOfMemory ? CF_ENOMEM : CF_EHIP;
    }
    char *cur = h->ws;
    h->err = reinterpret_cast<uint32_t *>(cur + 128);
    h->done = reinterpret_cast<unsigned long long *>(cur + 256);
    cur += h->counters_bytes;
    h->p1 = reinterpret_cast<uint64_t *>(cur);
    cur += p1_bytes;
    h->p2 = reinterpret_cast<uint64_t *>(cur);
    cur += p2_bytes;
    h->p3 = reinterpret_cast<uint64_t *>(cur);
    cur += p3_bytes;
    h->xslots = reinterpret_cast<uint64_t *>(cur);
    cur += xslot_bytes;
    h->dbg_q = reinterpret_cast<float *>(cur);
    cur += dbg_bytes;
    h->dbg_attn = reinterpret_cast<float *>(cur);
    cur += dbg_bytes;
    h->dbg_t = reinterpret_cast<unsigned long long *>(cur);
    cur += times_bytes;
    h->chain[0] = reinterpret_cast<uint16_t *>(cur);
    h->chain[1] = reinterpret_cast<uint16_t *>(cur + chain_bytes);

    e = hipMemset(h->ws, 0, h->ws_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(h->ws);
        delete h;
        return CF_EHIP;
    }
    *out = h;
    return CF_OK;
}

int cf_destroy(cf_handle h)
{
    if (!h) return CF_EINVAL;
    hipError_t e = hipFree(h->ws);
    delete h;
    return e == hipSuccess ? CF_OK : CF_EHIP;
}

static int decode_impl(cf_handle h, int packed, int32_t batch, const void *x, const void *W_qkv, const void *W_o,
                       void *k_cache, void *v_cache, int32_t pos, void *out, void *stream,
                       const void *norm_weight = nullptr, float eps = 0.f, int residual = 0,
                       const int32_t *row_pos = nullptr, cf::StackArgs *stack = nullptr)
{
    if (!h) return CF_EINVAL;
    if (reinterpret_cast<uintptr_t>(row_pos) & 3u) return CF_EINVAL;
    if ((norm_weight && !aligned16(norm_weight)) || !(eps >= 0.f) || !std::isfinite(eps)) return CF_EINVAL;
    if (norm_weight && h->cfg.d_model > 8 * 2 * cf::kThreads) return CF_EUNSUPPORTED;        // the kernel squares a row with two loads per thread
    if (batch < 1 || batch > h->cfg.max_batch || pos < 0 || pos >= h->cfg.max_seq) return CF_EINVAL;
    if (!aligned16(x) || !aligned16(W_qkv) || !aligned16(W_o) || !aligned16(k_cache) || !aligned16(v_cache) ||
        !aligned16(out))
        return CF_EINVAL;
    Params p;
    std::memset(&p, 0, sizeof p);
    fill_static(h, &p);
    p.x = static_cast<const uint16_t *>(x);
    p.wqkv = static_cast<const uint16_t *>(W_qkv);
    p.wo = static_cast<const uint16_t *>(W_o);
    p.kc = static_cast<uint16_t *>(k_cache);
    p.vc = static_cast<uint16_t *>(v_cache);
    p.out = static_cast<uint16_t *>(out);
    p.gamma = static_cast<const uint16_t *>(norm_weight);
    p.eps = eps;
    p.row_pos = row_pos;
    p.B = batch;
    p.pos = pos;
    p.flags = (packed ? cf::kFlagPacked : 0) | (residual ? cf::kFlagResidual : 0);
    int rc = make_plan(h, batch, pos, &p);
    if (rc != CF_OK) return rc;
    if (h->slot_area) {
        // the three slot arrays, sized for this call's plan, side by side in the fixed area
        const size_t b1 = align_up((size_t)p.KS * batch * h->nqkv * sizeof(uint64_t), 256);
        const size_t b2 = align_up((size_t)batch * h->cfg.n_q_heads * p.NS * (h->cfg.head_dim + cf::kP2Stride) * sizeof(uint64_t), 256);
        const size_t b3 = align_up((size_t)h->cfg.n_q_heads * p.RS3 * batch * h->cfg.d_model * sizeof(uint64_t), 256);
        if (b1 + b2 + b3 > h->slot_area_bytes) return CF_ESCRATCH;
        p.p1 = reinterpret_cast<uint64_t *>(h->slot_area);
        p.p2 = reinterpret_cast<uint64_t *>(h->slot_area + b1);
        p.p3 = reinterpret_cast<uint64_t *>(h->slot_area + b1 + b2);
    }
    const int bt = batch_tile(batch, h->cfg.head_dim);
    const size_t lds = cf::lds_floats(p, h->cfg.head_dim, h->G, bt) * sizeof(float);
    if (lds > kLdsLimit) return CF_EUNSUPPORTED;
    rc = check_residency(h, p, bt, lds);
    if (rc != CF_OK) return rc;
    const int plan[10] = {p.W, p.TS, p.KS, p.RB, p.NS, p.TPS, p.NC3, p.CW3, p.RS3, (int)lds};
    std::memcpy(h->last_plan, plan, sizeof plan);
    h->last_batch = batch;
    hipError_t e;
    if (stack) {
        // one launch for all layers: the table of the other layers' pointers is filled in by the caller
        stack->p = p;
        stack->xslots = h->xslots;
        e = cf::launch_fused_stack(*stack, h->cfg.head_dim, h->G, bt, lds, static_cast<hipStream_t>(stream));
    } else {
        e = cf::launch_fused(p, h->cfg.head_dim, h->G, bt, lds, static_cast<hipStream_t>(stream));
    }
    if (e != hipSuccess) return hip_fail(h, e);
    return CF_OK;
}

int cf_decode_block(cf_handle h, int32_t batch, const void *x, const void *W_qkv, const void *W_o, void *k_cache,
                    void *v_cache, int32_t pos, void *out, void *stream)
{
    return decode_impl(h, 0, batch, x, W_qkv, W_o, k_cache, v_cache, pos, out, stream);
}

int cf_decode_block_packed(cf_handle h, int32_t batch, const void *x, const void *W_qkv_packed,
                           const void *W_o_packed, void *k_cache, void *v_cache, int32_t pos, void *out, void *stream)
{
    return decode_impl(h, 1, batch, x, W_qkv_packed, W_o_packed, k_cache, v_cache, pos, out, stream);
}

int cf_decode_layer(cf_handle h, int32_t batch, const void *x, const void *norm_weight, float eps, int32_t residual,
                    int32_t packed, const void *W_qkv, const void *W_o, void *k_cache, void *v_cache, int32_t pos,
                    void *out, void *stream)
{
    if (residual && x == out) return CF_EINVAL;
    return decode_impl(h, packed != 0, batch, x, W_qkv, W_o, k_cache, v_cache, pos, out, stream, norm_weight, eps,
                       residual);
}

int cf_decode_layer_rows(cf_handle h, int32_t batch, const void *x, const void *norm_weight, float eps, int32_t residual,
                         int32_t packed, const void *W_qkv, const void *W_o, void *k_cache, void *v_cache,
                         const int32_t *row_pos, int32_t max_pos, void *out, void *stream)
{
    if (!row_pos || (residual && x == out)) return CF_EINVAL;
    return decode_impl(h, packed != 0, batch, x, W_qkv, W_o, k_cache, v_cache, max_pos, out, stream, norm_weight, eps,
                       residual, row_pos);
}

int cf_decode_stack(cf_handle h, int32_t n_layers, int32_t batch, const void *x, const void *const *norm_weight, float eps,
                    int32_t residual, int32_t packed, const void *const *W_qkv, const void *const *W_o,
                    void *const *k_cache, void *const *v_cache, int32_t pos, void *out, void *stream)
{
    if (!h || n_layers < 1 || !W_qkv || !W_o || !k_cache || !v_cache || !x || !out || x == out) return CF_EINVAL;
    // all layers are checked before the first one is enqueued (decode_impl checks again, per layer)
    for (int l = 0; l < n_layers; ++l)
        if (!aligned16(W_qkv[l]) || !aligned16(W_o[l]) || !aligned16(k_cache[l]) || !aligned16(v_cache[l]) ||
            (norm_weight && !aligned16(norm_weight[l])))
            return CF_EINVAL;
    if (!norm_weight && !residual && h->cfg.head_dim == 128 && !h->slot_area) {
        // The bare block: up to kMaxStackLayers layers per launch, the hidden state handed from layer to layer
        // inside the kernel; a deeper stack takes several such launches, chained through the two buffers.
        const void *in = x;
        int chunk_index = 0;
        for (int l0 = 0; l0 < n_layers; l0 += cf::kMaxStackLayers, ++chunk_index) {
            const int n = n_layers - l0 < cf::kMaxStackLayers ? n_layers - l0 : cf::kMaxStackLayers;
            void *dst = l0 + n == n_layers ? out : static_cast<void *>(h->chain[chunk_index & 1]);
            cf::StackArgs a;
            std::memset(&a, 0, sizeof a);
            a.n_layers = n;
            for (int l = 0; l < n; ++l) {
                a.tab[l].wqkv = static_cast<const uint16_t *>(W_qkv[l0 + l]);
                a.tab[l].wo = static_cast<const uint16_t *>(W_o[l0 + l]);
                a.tab[l].kc = static_cast<uint16_t *>(k_cache[l0 + l]);
                a.tab[l].vc = static_cast<uint16_t *>(v_cache[l0 + l]);
            }
            const int rc = decode_impl(h, packed != 0, batch, in, W_qkv[l0], W_o[l0], k_cache[l0], v_cache[l0], pos, dst, stream,
                                       nullptr, 0.f, 0, nullptr, &a);
            if (rc != CF_OK) return rc;
            in = dst;
        }
        return CF_OK;
    }
    const void *in = x;
    for (int l = 0; l < n_layers; ++l) {
        void *dst = l == n_layers - 1 ? out : static_cast<void *>(h->chain[l & 1]);
        const int rc = decode_impl(h, packed != 0, batch, in, W_qkv[l], W_o[l], k_cache[l], v_cache[l], pos, dst, stream,
                                   norm_weight ? norm_weight[l] : nullptr, eps, residual);
        if (rc != CF_OK) return rc;
        in = dst;
    }
    return CF_OK;
}

int cf_packed_sizes(cf_handle h, size_t *qkv_bytes, size_t *o_bytes)
{
    if (!h || !qkv_bytes || !o_bytes) return CF_EINVAL;
    *qkv_bytes = (size_t)(h->nqkv / h->cfg.head_dim) * ((size_t)h->cfg.d_model * h->cfg.head_dim * 2 + cf::kQkvBlockPad);
    *o_bytes = (size_t)h->cfg.n_q_heads * h->nch * h->cfg.head_dim * cf::kOutChunk * 2;
    return CF_OK;
}

int cf_pack_weights(cf_handle h, const void *W_qkv, const void *W_o, void *W_qkv_packed, void *W_o_packed, void *stream)
{
    if (!h || !aligned16(W_qkv) || !aligned16(W_o) || !aligned16(W_qkv_packed) || !aligned16(W_o_packed))
        return CF_EINVAL;
    if (W_qkv == W_qkv_packed || W_o == W_o_packed) return CF_EINVAL;   // not in place
    hipError_t e = cf::launch_pack(static_cast<const uint16_t *>(W_qkv), static_cast<const uint16_t *>(W_o),
                                   static_cast<uint16_t *>(W_qkv_packed), static_cast<uint16_t *>(W_o_packed),
                                   h->cfg.d_model, h->nqkv, h->cfg.n_q_heads, h->cfg.head_dim,
                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CF_OK : hip_fail(h, e);
}

int cf_status(cf_handle h, void *stream)
{
    if (!h) return CF_EINVAL;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e);
    uint32_t flag = 0;
    e = hipMemcpy(&flag, h->err, sizeof flag, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e);
    if (flag) {
        // a spin gave up: start from a clean slate (launch counters and all stamps)
        e = hipMemset(h->ws, 0, h->exchange_bytes);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(h, e);
        return CF_ETIMEOUT;
    }
    return CF_OK;
}

int cf_debug_export(cf_handle h, int32_t what, void *host_dst, size_t bytes, void *stream)
{
    if (!h || !host_dst || what < 0 || what > 2) return CF_EINVAL;
    if (!(h->cfg.flags & CF_FLAG_DEBUG_EXPORT) || h->last_batch < 1) return CF_EINVAL;
    const size_t want = what == 2 ? (size_t)h->last_plan[0] * cf::kStamps * sizeof(unsigned long long)
                                  : (size_t)h->last_batch * h->cfg.n_q_heads * h->cfg.head_dim * sizeof(float);
    if (bytes != want) return CF_EINVAL;
    const void *src = what == 0 ? (const void *)h->dbg_q : what == 1 ? (const void *)h->dbg_attn : (const void *)h->dbg_t;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e == hipSuccess) e = hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost);
    return e == hipSuccess ? CF_OK : hip_fail(h, e);
}

int cf_set_tuning(cf_handle h, int32_t workgroups, int32_t k_splits, int32_t kv_splits, int32_t spin_limit_us)
{
    if (!h || workgroups < 0 || k_splits < 0 || kv_splits < 0 || spin_limit_us < -1) return CF_EINVAL;
    auto pow2 = [](int v) { return v > 0 && (v & (v - 1)) == 0; };
    if (workgroups && (workgroups % h->cfg.n_kv_heads || workgroups > 8 * h->num_cu)) return CF_EINVAL;
    if (k_splits > kMaxKS) return CF_EINVAL;
    if (kv_splits && (!pow2(kv_splits) || kv_splits > cf::kMaxKvSplits)) return CF_EINVAL;
    if (workgroups != h->tune_w) {
        // every workgroup counts its own launches; with another grid the counts must start together again
        hipError_t e = hipDeviceSynchronize();
        if (e == hipSuccess) e = hipMemset(h->ws, 0, h->exchange_bytes);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(h, e);
    }
    h->tune_w = workgroups;
    h->tune_ks = k_splits;
    h->tune_ns = kv_splits;
    for (int &v : h->wg_per_cu) v = 0;   // LDS size may change: probe residency again
    if (spin_limit_us) h->spin_ticks = spin_limit_us < 0 ? 0 : (long long)spin_limit_us * 100;
    return CF_OK;
}

int cf_get_plan(cf_handle h, int32_t *dst, int32_t n)
{
    if (!h || !dst || n < 0) return CF_EINVAL;
    for (int i = 0; i < n && i < 10; ++i) dst[i] = h->last_plan[i];
    return CF_OK;
}

int64_t cf_algorithmic_bytes(const cf_config *cfg, int32_t batch, int32_t pos)
{
    if (!cfg) return 0;
    const int64_t D = cfg->d_model, nq = cfg->n_q_heads, nkv = cfg->n_kv_heads, d = cfg->head_dim, B = batch;
    const int64_t weights = 2 * D * (nq + 2 * nkv) * d + 2 * nq * d * D;
    const int64_t kv_read = B * 2 * nkv * (int64_t)pos * d * 2;
    const int64_t appended = B * 2 * nkv * d * 2;
    const int64_t io = 2 * B * D * 2;
    return weights + kv_read + appended + io;
}

// ------------------------------------------------------------------------------------------------
// cf_decode_block_static: the decode step for callers that cannot allocate.  Everything the kernel keeps between
// workgroups (error flag, launch counters, exchange slots) lives in one array of device memory that is part of the
// library's code object; the address each GPU gives it is looked up once per device.
}  // extern "C" (reopened below)

namespace {

constexpr size_t kScratchBytes = (size_t)32 << 20;               // 32 MiB per GPU, held until the process ends
constexpr size_t kScratchCounters = 2048;                         // launch counters: one per possible workgroup
constexpr size_t kScratchHeadBytes = 256 + kScratchCounters * cf::kCounterStride * sizeof(unsigned long long);
constexpr int kMaxDevices = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

struct StaticDevice {
    char *ptr = nullptr;        // device address of `scratch` on this GPU (hipGetSymbolAddress)
    int num_cu = 0;
    int last_w = 0;             // workgroups of the previous launch through this entry point on this GPU
    int wg_per_cu[6] = {0, 0, 0, 0, 0, 0};
    unsigned long long occ_key = 0;   // (head_dim, group, LDS bytes) the residency figures above were taken for
};
StaticDevice g_static[kMaxDevices];

// All launch counters take the largest value any of them holds.  Every workgroup of a launch counts in its own
// line; after a launch with fewer workgroups the lines of the others lag behind, and a launch with more workgroups
// needs them all equal again (the stamp of a launch is count + 1).
__global__ void __launch_bounds__(1024) equalize_counters(unsigned long long *done)
{
    __shared__ unsigned long long part[16];
    unsigned long long v = 0;
    for (size_t i = threadIdx.x; i < kScratchCounters; i += blockDim.x) {
        const unsigned long long c = done[i * cf::kCounterStride];
        v = c > v ? c : v;
    }
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(v, off);
        v = o > v ? o : v;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) v = part[k] > v ? part[k] : v;
    for (size_t i = threadIdx.x; i < kScratchCounters; i += blockDim.x) done[i * cf::kCounterStride] = v;
}

}  // namespace

extern "C" {

int cf_decode_block_static(const cf_config *cfg, int32_t batch, const void *x, const void *W_qkv, const void *W_o,
                           void *k_cache, void *v_cache, int32_t pos, void *out, void *stream)
{
    if (!cfg) return CF_EINVAL;
    int rc = check_config(*cfg);
    if (rc != CF_OK) return rc;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return CF_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return CF_EUNSUPPORTED;
    StaticDevice &sd = g_static[dev];
    if (!sd.ptr) {
        // once per device, with that device current: every GPU holds its own copy of the array at its own address
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CF_EHIP;
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return CF_EHIP;
        sd.num_cu = cus;
        sd.ptr = static_cast<char *>(ptr);
    }
    if ((size_t)sd.num_cu > kScratchCounters) return CF_EUNSUPPORTED;

    // a handle on the stack that points into the array; nothing is allocated and nothing outlives the call
    cf_handle_s h;
    h.cfg = *cfg;
    h.cfg.flags = 0;
    h.device = dev;
    h.num_cu = sd.num_cu;
    h.G = cfg->n_q_heads / cfg->n_kv_heads;
    h.nqkv = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
    h.nch = ceil_div(cfg->d_model, cf::kOutChunk);
    if (cfg->n_kv_heads > h.num_cu) return CF_EUNSUPPORTED;
    h.err = reinterpret_cast<uint32_t *>(sd.ptr + 128);
    h.done = reinterpret_cast<unsigned long long *>(sd.ptr + 256);
    h.slot_area = sd.ptr + kScratchHeadBytes;
    h.slot_area_bytes = kScratchBytes - kScratchHeadBytes;
    const unsigned long long key = ((unsigned long long)cfg->head_dim << 40) ^ ((unsigned long long)h.G << 32);
    if (sd.occ_key == key) std::memcpy(h.wg_per_cu, sd.wg_per_cu, sizeof h.wg_per_cu);
    const int w = default_workgroups(&h);
    if (w != sd.last_w) {
        // (a kernel, not a memset: the call may be recorded into a graph)
        hipLaunchKernelGGL(equalize_counters, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), h.done);
        if (hipGetLastError() != hipSuccess) return CF_EHIP;
        sd.last_w = w;
    }
    rc = decode_impl(&h, 0, batch, x, W_qkv, W_o, k_cache, v_cache, pos, out, stream);
    sd.occ_key = key;
    std::memcpy(sd.wg_per_cu, h.wg_per_cu, sizeof h.wg_per_cu);
    return rc;
}

const char *cf_strerror(int code)
{
    switch (code) {
    case CF_OK: return "ok";
    case CF_EINVAL: return "invalid argument";
    case CF_EUNSUPPORTED: return "unsupported shape or launch configuration";
    case CF_EHIP: return "HIP runtime error";
    case CF_ENOMEM: return "out of memory";
    case CF_ETIMEOUT: return "a cross-workgroup wait inside the kernel timed out";
    case CF_ESCRATCH: return "the call needs more exchange memory than the fixed scratch array of cf_decode_block_static holds";
    default: return "unknown error";
    }
}

int cf_last_hip_error(cf_handle h) { return h ? h->last_hip : 0; }

}  // extern "C"
