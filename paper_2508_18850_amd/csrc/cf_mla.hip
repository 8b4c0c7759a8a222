// Fused decode step of a weight-absorbed Multi-Head Latent Attention block (paper Appendix B, Alg. 4) as ONE
// kernel for gfx950, behind the C ABI (cf_mla_* in include/cfdecode.h).
//
// Alg. 4 runs one cluster per head and moves data between its blocks with three ClusterGathers and three
// ClusterReduces.  Here a head is a team of 16 co-resident workgroups and every hand-over is one hop through
// stamped {value, stamp} slots in global memory (cf_team_device.h), five hops in all:
//
//   A  projections        [q | kv_new] = x [W_Q | W_KV]           16 row slices x 16 column blocks, partial sums
//   B  up-projection      q_lat_i = q_nope_i W_Up[i]              member j: 1/16 of the kv_lora_rank columns
//   C  attention          partial softmax over 1/16 of the tokens  (m, l, acc[kv_lora_rank]) per member;
//                         the last member appends the new row and counts the new token
//   D1 merge              member j merges 1/16 of the latent dimensions of the 16 partials
//   D2 down-projection    a_i = z_i W_Down[i]                      member j: 1/16 of the value columns
//   E  output projection  out = concat(a) W_O                      every workgroup: 1/W of the output columns
//
// This is a first, correctness-first version: weights are read with plain (narrow) loads, nothing is prefetched
// across the hops.  All waits are bounded (CF_ETIMEOUT), all workgroups have to be resident at once.
#include "../../include/cfdecode.h"
#include "cf_rope_device.h"
#include "cf_team_device.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

namespace {

using cf::team::Exchange;
using cf::team::pair_t;
constexpr int NT = 512;             // threads per workgroup
constexpr int NW = NT / 64;
constexpr int TS = 16;              // workgroups per head (team)
constexpr int KS = 16;              // row slices of the projections
constexpr int L = 512;              // kv_lora_rank the lane mapping is written for: 64 lanes x 8 values
constexpr int R = 64;               // rope_dim: 8 lanes x 8 values
constexpr int MAXB = 4;             // largest batch
constexpr int MAXCOLS = 256;        // projection columns per column block
constexpr int MAXA = 2048;          // n_heads * v_head_dim
constexpr int kCounterStride = 16;
constexpr float kNegBig = -1.0e30f;

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

struct MlaArgs {
    const uint16_t *x, *wq, *wkv, *wup, *wdown, *wo;
    uint16_t *cache, *out;
    uint64_t *slots;
    unsigned long long *counters;
    uint32_t *err;
    size_t x1, x2, x3, x4, x5;      // first slot of each exchange area
    int D, nh, n, v, B, pos, max_seq, W;
    int cq, ckv;                    // columns of W_Q / W_KV per column block
    float scale_log2e;              // log2(e) / sqrt(nope_dim + rope_dim)
    double log2_base;
    long long spin_ticks;
};

__device__ __forceinline__ float h2f(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t f2h(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Sum of the n stamped values at idx, idx + stride, ... (in that order); polls go out eight at a time.
__device__ __forceinline__ float take_sum(const Exchange &x, __amdgpu_buffer_rsrc_t r, size_t idx, size_t stride, int n)
{
    float s = 0.f;
    for (int k0 = 0; k0 < n; k0 += 8) {
        pair_t q[8];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < 8; ++k) q[k] = cf::team::peek(r, idx + (size_t)min(k0 + k, n - 1) * stride);
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < 8; ++k) ok &= q[k].y == x.stamp;
            if (ok || cf::team::gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k0 + k < n) s += __builtin_bit_cast(float, q[k].x);
    }
    return s;
}

__device__ __forceinline__ void lds_sync() { __syncthreads(); }

__global__ void __launch_bounds__(NT) fused_mla_decode(const MlaArgs a)
{
    __shared__ float s_a[MAXB * MAXA];                  // stage buffers, reused from stage to stage
    __shared__ float s_b[MAXB * (L + R)];
    __shared__ float s_red[NW * (L + 2)];
    __shared__ float s_small[R + MAXB];                 // cos, sin of the rotary angles; score of the new token per row
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, w = blockIdx.x;
    const int head = w / TS, j = w % TS;
    const int B = a.B, nr = a.n + R, CQq = a.nh * nr, CQ = CQq + L + R;

    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)w * kCounterStride)
                 : "memory");
    const unsigned long long cnt = launches + 1ull;
    const Exchange x = {a.slots, 0, (uint32_t)(cnt + (cnt >> 32)), a.err, a.spin_ticks};
    const __amdgpu_buffer_rsrc_t r = cf::team::slots_rsrc(x);

    // ---- A: partial projections.  Work item (kb, cb): rows [kb*RK, +RK) of x, column block cb of W_Q and of W_KV.
    const int RK = a.D / KS, ncols = a.cq + a.ckv;
    for (int item = w; item < KS * 16; item += a.W) {
        const int kb = item / 16, cb = item % 16;
        lds_sync();
        for (int i = tid; i < B * RK; i += NT) s_a[i] = h2f(a.x[(size_t)(i / RK) * a.D + kb * RK + i % RK]);
        lds_sync();
        const int c = tid % MAXCOLS, half = tid / MAXCOLS;           // two halves of the rows per column
        const bool isq = c < a.cq;
        const int col = isq ? cb * a.cq + c : cb * a.ckv + (c - a.cq);
        const bool live = c < ncols && col < (isq ? CQq : L + R);
        const uint16_t *wp = isq ? a.wq + col : a.wkv + col;
        const size_t ld = isq ? CQq : L + R;
        float acc[MAXB] = {0.f, 0.f, 0.f, 0.f};
        if (live) {
            const int r0 = half * (RK / 2), r1 = half ? RK : RK / 2;
            for (int rr = r0; rr < r1; ++rr) {
                const float wgt = h2f(wp[(size_t)(kb * RK + rr) * ld]);
#pragma unroll
                for (int b = 0; b < MAXB; ++b)
                    if (b < B) acc[b] = fmaf(s_a[b * RK + rr], wgt, acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < MAXB; ++b) s_b[(b * 2 + half) * MAXCOLS + c] = acc[b];
        lds_sync();
        if (half == 0 && live) {
            const int gcol = isq ? col : CQq + col;
            for (int b = 0; b < B; ++b)
                cf::team::put(r, a.x1 + ((size_t)kb * B + b) * CQ + gcol,
                              s_b[(b * 2) * MAXCOLS + c] + s_b[(b * 2 + 1) * MAXCOLS + c], x.stamp);
        }
    }

    // ---- B: up-projection of head `head`, columns [LJ*j, +LJ) of the latent dimension
    constexpr int LJ = L / TS;                                        // 32
    lds_sync();
    for (int i = tid; i < B * a.n; i += NT) {
        const int b = i / a.n, c = i % a.n;
        s_a[i] = take_sum(x, r, a.x1 + (size_t)b * CQ + head * nr + c, (size_t)B * CQ, KS);
    }
    lds_sync();
    {
        const int c = tid % LJ, g = tid / LJ;                         // 16 row groups
        float acc[MAXB] = {0.f, 0.f, 0.f, 0.f};
        for (int row = g; row < a.n; row += NT / LJ) {
            const float wgt = h2f(a.wup[((size_t)head * a.n + row) * L + LJ * j + c]);
#pragma unroll
            for (int b = 0; b < MAXB; ++b)
                if (b < B) acc[b] = fmaf(s_a[b * a.n + row], wgt, acc[b]);
        }
#pragma unroll
        for (int b = 0; b < MAXB; ++b) s_b[(b * (NT / LJ) + g) * LJ + c] = acc[b];
        lds_sync();
        if (tid < LJ * B) {
            const int b = tid / LJ, cc = tid % LJ;
            float s = 0.f;
            for (int g2 = 0; g2 < NT / LJ; ++g2) s += s_b[(b * (NT / LJ) + g2) * LJ + cc];
            cf::team::put(r, a.x2 + ((size_t)b * a.nh + head) * L + LJ * j + cc, s, x.stamp);
        }
    }

    // ---- C: attention over the tokens [t0, t1) of this member; the last member also takes the new token
    lds_sync();
    const bool last = j == TS - 1;
    const int tps = (a.pos + TS - 1) / TS;
    const int t0 = min(j * tps, a.pos), t1 = min(t0 + tps, a.pos);
    // s_a: [B][L + R] the query in the latent space and its rotated rotary part; s_b: [B][L + R] the new row
    for (int i = tid; i < B * L; i += NT) {
        const int b = i / L, d = i % L;
        s_a[b * (L + R) + d] = take_sum(x, r, a.x2 + ((size_t)b * a.nh + head) * L + d, 0, 1);
    }
    for (int i = tid; i < B * R; i += NT) {
        const int b = i / R, d = i % R;
        s_a[b * (L + R) + L + d] = take_sum(x, r, a.x1 + (size_t)b * CQ + head * nr + a.n + d, (size_t)B * CQ, KS);
    }
    if (last)
        for (int i = tid; i < B * (L + R); i += NT) {
            const int b = i / (L + R), d = i % (L + R);
            s_b[i] = take_sum(x, r, a.x1 + (size_t)b * CQ + CQq + d, (size_t)B * CQ, KS);
        }
    if (tid < R / 2) {
        const double inv_freq = exp2(-2.0 * (double)tid / (double)R * a.log2_base);
        cf::rope_cos_sin(a.pos, inv_freq, s_small[tid], s_small[R / 2 + tid]);
    }
    lds_sync();
    for (int i = tid; i < B * (R / 2); i += NT) {                     // RoPE on the rotary parts (pairs d, d + R/2)
        const int b = i / (R / 2), d = i % (R / 2);
        const float c = s_small[d], sn = s_small[R / 2 + d];
        float *q = s_a + b * (L + R) + L;
        const float lo = q[d], hi = q[d + R / 2];
        q[d] = lo * c - hi * sn;
        q[d + R / 2] = hi * c + lo * sn;
        if (last) {
            float *k = s_b + b * (L + R) + L;
            const float klo = k[d], khi = k[d + R / 2];
            k[d] = klo * c - khi * sn;
            k[d + R / 2] = khi * c + klo * sn;
        }
    }
    lds_sync();
    if (last)                                                         // append (Sec. 2.1): row pos of every sequence
        for (int i = tid; i < B * (L + R); i += NT) {
            const int b = i / (L + R), d = i % (L + R);
            a.cache[((size_t)b * a.max_seq + a.pos) * (L + R) + d] = f2h(s_b[i]);
        }
    for (int b = 0; b < B; ++b) {
        const float *q = s_a + b * (L + R);
        float ql[8], qr[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            ql[k] = q[lane * 8 + k] * a.scale_log2e;
            qr[k] = lane < R / 8 ? q[L + lane * 8 + k] * a.scale_log2e : 0.f;
        }
        float m = kNegBig, lsum = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const uint16_t *rows = a.cache + (size_t)b * a.max_seq * (L + R);
        for (int t = t0 + wv; t < t1; t += NW * 4) {                   // four rows of this wavefront in flight
            h8 kl[4], kr[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int tt = min(t + u * NW, t1 - 1);
                kl[u] = *reinterpret_cast<const h8 *>(rows + (size_t)tt * (L + R) + lane * 8);
                kr[u] = *reinterpret_cast<const h8 *>(rows + (size_t)tt * (L + R) + L + (lane & (R / 8 - 1)) * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float d = 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) d = fmaf(ql[k], (float)kl[u][k], d);
#pragma unroll
                for (int k = 0; k < 8; ++k) d = fmaf(qr[k], (float)kr[u][k], d);
                d = wave_sum(d);
                if (t + u * NW < t1) {                                  // uniform over the wavefront
                    const float mn = fmaxf(m, d), f = __builtin_amdgcn_exp2f(m - mn), pw = __builtin_amdgcn_exp2f(d - mn);
                    m = mn;
                    lsum = lsum * f + pw;
#pragma unroll
                    for (int k = 0; k < 8; ++k) acc[k] = fmaf(pw, (float)kl[u][k], acc[k] * f);
                }
            }
        }
        lds_sync();
        if (lane == 0) {
            s_red[wv * (L + 2)] = m;
            s_red[wv * (L + 2) + 1] = lsum;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) s_red[wv * (L + 2) + 2 + lane * 8 + k] = acc[k];
        if (last && wv == 0) {                                        // score of the new token (its row is not rounded)
            const float *kn = s_b + b * (L + R);
            float d = 0.f;
#pragma unroll
            for (int k = 0; k < 8; ++k) d = fmaf(ql[k], kn[lane * 8 + k], d);
#pragma unroll
            for (int k = 0; k < 8; ++k) d = fmaf(qr[k], kn[L + (lane & (R / 8 - 1)) * 8 + k], d);
            d = wave_sum(d);
            if (lane == 0) s_small[R + b] = d;
        }
        lds_sync();
        {
            const int d = tid;                                         // one latent dimension per thread
            float M = last ? s_small[R + b] : kNegBig;
            for (int w8 = 0; w8 < NW; ++w8) M = fmaxf(M, s_red[w8 * (L + 2)]);
            float Ls = 0.f, A = 0.f;
            for (int w8 = 0; w8 < NW; ++w8) {
                const float f = __builtin_amdgcn_exp2f(s_red[w8 * (L + 2)] - M);
                Ls = fmaf(s_red[w8 * (L + 2) + 1], f, Ls);
                A = fmaf(s_red[w8 * (L + 2) + 2 + d], f, A);
            }
            if (last) {
                const float f = __builtin_amdgcn_exp2f(s_small[R + b] - M);
                Ls += f;
                A = fmaf(s_b[b * (L + R) + d], f, A);
            }
            const size_t dst = a.x3 + (((size_t)b * a.nh + head) * TS + j) * (L + 2);
            if (d == 0) {
                cf::team::put(r, dst, M, x.stamp);
                cf::team::put(r, dst + 1, Ls, x.stamp);
            }
            cf::team::put(r, dst + 2 + d, A, x.stamp);
        }
    }

    // ---- D1: merge latent dimensions [LJ*j, +LJ) of the team's partials (online softmax, Alg. 4 steps 8-10)
    if (tid < LJ * B) {
        const int b = tid / LJ, d = LJ * j + tid % LJ;
        const size_t src = a.x3 + ((size_t)b * a.nh + head) * TS * (L + 2);
        float ms[TS], ls[TS], as[TS];
#pragma unroll
        for (int s = 0; s < TS; ++s) ms[s] = take_sum(x, r, src + (size_t)s * (L + 2), 0, 1);
#pragma unroll
        for (int s = 0; s < TS; ++s) ls[s] = take_sum(x, r, src + (size_t)s * (L + 2) + 1, 0, 1);
#pragma unroll
        for (int s = 0; s < TS; ++s) as[s] = take_sum(x, r, src + (size_t)s * (L + 2) + 2 + d, 0, 1);
        float M = kNegBig;
#pragma unroll
        for (int s = 0; s < TS; ++s) M = fmaxf(M, ms[s]);
        float Ls = 0.f, A = 0.f;
#pragma unroll
        for (int s = 0; s < TS; ++s) {
            const float f = __builtin_amdgcn_exp2f(ms[s] - M);
            Ls = fmaf(ls[s], f, Ls);
            A = fmaf(as[s], f, A);
        }
        cf::team::put(r, a.x4 + ((size_t)b * a.nh + head) * L + d, A / Ls, x.stamp);
    }

    // ---- D2: down-projection, value columns [VJ*j, +VJ) of this head
    const int VJ = a.v / TS;                                           // <= 8
    lds_sync();
    for (int i = tid; i < B * L; i += NT)
        s_a[i] = take_sum(x, r, a.x4 + ((size_t)(i / L) * a.nh + head) * L + i % L, 0, 1);
    lds_sync();
    {
        float part[MAXB][8];
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) part[b][c] = 0.f;
        const uint16_t *wrow = a.wdown + ((size_t)head * L + tid) * a.v + VJ * j;      // row tid of W_Down[head]
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float wgt = c < VJ ? h2f(wrow[c]) : 0.f;
#pragma unroll
            for (int b = 0; b < MAXB; ++b)
                if (b < B) part[b][c] = s_a[b * L + tid] * wgt;
        }
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float s = wave_sum(part[b][c]);
                if (lane == 0) s_red[(wv * MAXB + b) * 8 + c] = s;
            }
        lds_sync();
        if (tid < B * VJ) {
            const int b = tid / VJ, c = tid % VJ;
            float s = 0.f;
            for (int w8 = 0; w8 < NW; ++w8) s += s_red[(w8 * MAXB + b) * 8 + c];
            cf::team::put(r, a.x5 + (size_t)b * a.nh * a.v + head * a.v + VJ * j + c, s, x.stamp);
        }
    }

    // ---- E: output projection, columns [CW*w, +CW) of the output
    const int HV = a.nh * a.v, CW = (a.D + a.W - 1) / a.W;             // CW <= 8
    lds_sync();
    for (int i = tid; i < B * HV; i += NT) s_a[i] = take_sum(x, r, a.x5 + i, 0, 1);
    lds_sync();
    {
        float part[MAXB][8];
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) part[b][c] = 0.f;
        const int c0 = CW * w;
        for (int row = tid; row < HV; row += NT) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float wgt = (c < CW && c0 + c < a.D) ? h2f(a.wo[(size_t)row * a.D + c0 + c]) : 0.f;
#pragma unroll
                for (int b = 0; b < MAXB; ++b)
                    if (b < B) part[b][c] = fmaf(s_a[b * HV + row], wgt, part[b][c]);
            }
        }
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float s = wave_sum(part[b][c]);
                if (lane == 0) s_red[(wv * MAXB + b) * 8 + c] = s;
            }
        lds_sync();
        if (tid < B * CW) {
            const int b = tid / CW, c = tid % CW;
            if (c0 + c < a.D) {
                float s = 0.f;
                for (int w8 = 0; w8 < NW; ++w8) s += s_red[(w8 * MAXB + b) * 8 + c];
                a.out[(size_t)b * a.D + c0 + c] = f2h(s);
            }
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

}  // namespace

struct cf_mla_s {
    cf_mla_config cfg;
    int W = 0;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    uint64_t *slots = nullptr;
    unsigned long long *counters = nullptr;
    uint32_t *err = nullptr;
    size_t x1 = 0, x2 = 0, x3 = 0, x4 = 0, x5 = 0;
    long long spin_ticks = 200000000LL;
    int last_hip = 0;
};

extern "C" {

int cf_mla_create(const cf_mla_config *cfg, cf_mla *out)
{
    if (!cfg || !out) return CF_EINVAL;
    *out = nullptr;
    const cf_mla_config &c = *cfg;
    if (c.d_model < 16 || c.n_heads < 1 || c.nope_dim < 1 || c.v_head_dim < 1 || c.max_batch < 1 || c.max_seq < 1 ||
        !(c.rope_base > 1.f))
        return CF_EINVAL;
    // what this first kernel is written for
    const int W = c.n_heads * TS;
    const int CQq = c.n_heads * (c.nope_dim + R);
    const int cq = (CQq + 15) / 16, ckv = (L + R + 15) / 16;
    if (c.kv_lora_rank != L || c.rope_dim != R || c.max_batch > MAXB || c.d_model % (2 * KS) || c.d_model / KS > NT ||
        c.v_head_dim % TS || c.v_head_dim / TS > 8 || c.n_heads * c.v_head_dim > MAXA || cq + ckv > MAXCOLS ||
        c.nope_dim > L || c.d_model > 8 * W)
        return CF_EUNSUPPORTED;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CF_EHIP;
    if (W > prop.multiProcessorCount) return CF_EUNSUPPORTED;        // all workgroups resident, one per compute unit
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fused_mla_decode), NT, 0) !=
            hipSuccess || per_cu < 1)
        return CF_EUNSUPPORTED;
    cf_mla t = new (std::nothrow) cf_mla_s();
    if (!t) return CF_ENOMEM;
    t->cfg = c;
    t->W = W;
    const size_t B = c.max_batch, CQ = (size_t)CQq + L + R;
    t->x1 = 0;
    t->x2 = t->x1 + (size_t)KS * B * CQ;
    t->x3 = t->x2 + B * c.n_heads * L;
    t->x4 = t->x3 + B * c.n_heads * TS * (L + 2);
    t->x5 = t->x4 + B * c.n_heads * L;
    const size_t nslots = t->x5 + B * c.n_heads * c.v_head_dim;
    const size_t head = 256 + (size_t)W * kCounterStride * sizeof(unsigned long long);
    const size_t head_al = (head + 255) / 256 * 256;
    t->ws_bytes = head_al + nslots * sizeof(uint64_t);
    if (nslots * sizeof(uint64_t) > 0xfffffff0ull) {
        delete t;
        return CF_EUNSUPPORTED;
    }
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&t->ws), t->ws_bytes);
    if (e == hipSuccess) e = hipMemset(t->ws, 0, t->ws_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (t->ws) (void)hipFree(t->ws);
        delete t;
        return e == hipErrorOutOfMemory ? CF_ENOMEM : CF_EHIP;
    }
    t->err = reinterpret_cast<uint32_t *>(t->ws + 128);
    t->counters = reinterpret_cast<unsigned long long *>(t->ws + 256);
    t->slots = reinterpret_cast<uint64_t *>(t->ws + head_al);
    *out = t;
    return CF_OK;
}

int cf_mla_destroy(cf_mla t)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipFree(t->ws);
    delete t;
    return e == hipSuccess ? CF_OK : CF_EHIP;
}

int cf_mla_decode(cf_mla t, int32_t batch, const void *x, const void *W_q, const void *W_kv, const void *W_up,
                  const void *W_down, const void *W_o, void *kv_cache, int32_t pos, void *out, void *stream)
{
    if (!t || !x || !W_q || !W_kv || !W_up || !W_down || !W_o || !kv_cache || !out) return CF_EINVAL;
    if (batch < 1 || batch > t->cfg.max_batch || pos < 0 || pos >= t->cfg.max_seq) return CF_EINVAL;
    const void *ptrs[] = {x, W_q, W_kv, W_up, W_down, W_o, kv_cache, out};
    for (const void *p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) & 15u) return CF_EINVAL;
    const cf_mla_config &c = t->cfg;
    MlaArgs a;
    std::memset(&a, 0, sizeof a);
    a.x = static_cast<const uint16_t *>(x);
    a.wq = static_cast<const uint16_t *>(W_q);
    a.wkv = static_cast<const uint16_t *>(W_kv);
    a.wup = static_cast<const uint16_t *>(W_up);
    a.wdown = static_cast<const uint16_t *>(W_down);
    a.wo = static_cast<const uint16_t *>(W_o);
    a.cache = static_cast<uint16_t *>(kv_cache);
    a.out = static_cast<uint16_t *>(out);
    a.slots = t->slots;
    a.counters = t->counters;
    a.err = t->err;
    // the exchange areas are laid out for max_batch; a smaller batch uses the front of each
    a.x1 = t->x1, a.x2 = t->x2, a.x3 = t->x3, a.x4 = t->x4, a.x5 = t->x5;
    a.D = c.d_model, a.nh = c.n_heads, a.n = c.nope_dim, a.v = c.v_head_dim, a.B = batch, a.pos = pos;
    a.max_seq = c.max_seq, a.W = t->W;
    a.cq = (c.n_heads * (c.nope_dim + R) + 15) / 16;
    a.ckv = (L + R + 15) / 16;
    a.scale_log2e = 1.4426950408889634f / std::sqrt((float)(c.nope_dim + R));
    a.log2_base = std::log2((double)c.rope_base);
    a.spin_ticks = t->spin_ticks;
    hipLaunchKernelGGL(fused_mla_decode, dim3(t->W), dim3(NT), 0, static_cast<hipStream_t>(stream), a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    return CF_OK;
}

int cf_mla_status(cf_mla t, void *stream)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    uint32_t flag = 0;
    if (e == hipSuccess) e = hipMemcpy(&flag, t->err, sizeof flag, hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    if (flag) {
        e = hipMemset(t->ws, 0, t->ws_bytes);        // launch counters and all stamps start afresh
        if (e == hipSuccess) e = hipDeviceSynchronize();
        return e == hipSuccess ? CF_ETIMEOUT : CF_EHIP;
    }
    return CF_OK;
}

int cf_mla_set_spin_limit(cf_mla t, int32_t spin_limit_us)
{
    if (!t || spin_limit_us < 1) return CF_EINVAL;
    t->spin_ticks = (long long)spin_limit_us * 100;
    return CF_OK;
}

int64_t cf_mla_algorithmic_bytes(const cf_mla_config *c, int32_t batch, int32_t pos)
{
    if (!c) return 0;
    const int64_t nr = c->nope_dim + c->rope_dim, lr = c->kv_lora_rank + c->rope_dim, B = batch;
    const int64_t weights = (int64_t)c->d_model * (c->n_heads * nr + lr) + (int64_t)c->n_heads * c->nope_dim * c->kv_lora_rank +
                            (int64_t)c->n_heads * c->kv_lora_rank * c->v_head_dim + (int64_t)c->n_heads * c->v_head_dim * c->d_model;
    return 2 * (weights + B * (int64_t)pos * lr + B * lr + 2 * B * c->d_model);
}

}  // extern "C"
