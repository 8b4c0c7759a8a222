// Fused decode-block kernel for gfx950: QKV projection + RoPE + KV append +
// split-KV attention + output projection in one launch (paper Alg. 3).
//
// Mapping.  The paper maps one attention head to a cluster of thread blocks and
// resolves the dependencies between the blocks of a cluster with ClusterGather
// and ClusterReduce over distributed shared memory.  gfx950 has no clusters, so
// a "team" of workgroups (all workgroups whose index is congruent modulo
// n_kv_heads; with 8 | n_kv_heads they share one XCD and its L2) serves one KV
// head together with the query heads that use it:
//   phase 1  every member multiplies a slice of the reduction dimension of the
//            team's q/k/v weight columns (split-K instead of the paper's split
//            of the head dimension: rows of 256 contiguous bytes coalesce, 32
//            columns would not) and leaves an fp32 partial in an exchange slot;
//   phase 2  every member sums the partials it needs (the role of
//            ClusterGather), applies RoPE, and runs online-softmax attention
//            over its slice of the cached sequence (Alg. 3 step 4); the member
//            with the last slice also appends the new key/value and counts the
//            new token; (m, l, acc) partials go to exchange slots;
//   phase 3  every member merges the partials of its head (Alg. 3 steps 5-7,
//            local sums rescaled by exp(m_i - M) before being added), multiplies
//            by its block of W_o rows/columns (step 8) and leaves a per-head
//            partial of the output; the last arriver per 512-column chunk adds
//            the heads in a fixed order (the paper uses atomicAdd) and writes fp16.
// Workgroups of a team meet through two counters in device memory; all
// workgroups of the launch must be resident (checked on the host).  Waits are
// bounded: after spin_ticks a workgroup sets an error flag and goes on, so the
// kernel always ends.
#include "cf_params.h"


namespace cf {
namespace {

constexpr int NT = kThreads;
constexpr int NW = kWaves;
constexpr float kNegBig = -1.0e30f;   // stands for "no score yet"; finite so that differences never give NaN

__device__ __forceinline__ float ld_coh(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

typedef _Float16 h8 __attribute__((ext_vector_type(8)));   // eight fp16 values = one 128-bit load

// Streaming 128-bit load of weights / cache rows that are read exactly once.
__device__ __forceinline__ h8 ld_stream(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const h8 *>(p));
}

__device__ __forceinline__ void unpack8(const h8 &u, float (&f)[8])
{
#pragma unroll
    for (int k = 0; k < 8; ++k) f[k] = (float)u[k];
}

__device__ __forceinline__ float h2f(uint16_t bits)
{
    return (float)__builtin_bit_cast(_Float16, bits);
}
__device__ __forceinline__ uint16_t f2h(float v)
{
    return __builtin_bit_cast(uint16_t, (_Float16)v);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the LPR (8 or 16) consecutive lanes that hold one row; every lane gets the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7-i within 8 lanes
    if (LPR == 16) v += dpp_move<0x140>(v);   // row_mirror: lane i <-> 15-i within 16 lanes
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Publish `n` finished items of this workgroup to the team counter.
__device__ __forceinline__ void team_signal(uint32_t *cnt, uint32_t n)
{
    __syncthreads();   // every thread's exchange stores have completed
    if (threadIdx.x == 0 && n)
        __hip_atomic_fetch_add(cnt, n, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until the counter reaches `target` (counters are zero at launch).
__device__ __forceinline__ void team_wait(const Params &p, uint32_t *cnt, uint32_t target)
{
    if (threadIdx.x == 0) {
        const long long t0 = wall_clock64();
        while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if (wall_clock64() - t0 > p.spin_ticks) {
                __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}

// First weight column of selector `sel` for a team: sel < G query heads, G = key, G+1 = value.
template <int HD, int G>
__device__ __forceinline__ int qkv_col0(const Params &p, int team, int sel)
{
    if (sel < G) return (team * G + sel) * HD;
    if (sel == G) return (p.nq + team) * HD;
    return (p.nq + p.nkv + team) * HD;
}

// ---------------------------------------------------------------------------
// Phase 1: partial projection  y[b][col0 .. col0+HD) += x[b][r0 .. r0+RPS) . W[r0.., col0..]
// (Alg. 3 step 2, split over the reduction dimension)
// ---------------------------------------------------------------------------
template <int HD, int BT>
__device__ void p1_item(const Params &p, int col0, int ks, float *smem)
{
    constexpr int LPR = HD / 8;        // lanes per weight-row segment (16-byte loads)
    constexpr int NG = NT / LPR;       // row groups per workgroup
    constexpr int U = 8;               // loads in flight per thread
    const int tid = threadIdx.x, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const int RPS = p.RPS;
    const int r0 = ks * RPS;
    const int nrows = min(RPS, p.D - r0);
    float *xs = smem;                   // [BT][RPS]
    float *red = smem + BT * RPS;       // [NW][BT][HD]

    for (int i = tid; i < BT * RPS; i += NT) {
        const int b = i / RPS, r = i - b * RPS;
        xs[i] = (b < p.B && r < nrows) ? h2f(p.x[(size_t)b * p.D + r0 + r]) : 0.f;
    }
    __syncthreads();

    float acc[BT][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;

    const uint16_t *wbase = p.wqkv + (size_t)r0 * p.nqkv + col0 + lig * 8;
    const int iters = (nrows + NG - 1) / NG;
    for (int i0 = 0; i0 < iters; i0 += U) {
        h8 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = grp + NG * (i0 + u);
            const int rr = r < nrows ? r : 0;
            w[u] = ld_stream(wbase + (size_t)rr * p.nqkv);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = grp + NG * (i0 + u);
            const bool ok = r < nrows;
            float f[8];
            unpack8(w[u], f);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const float xv = ok ? xs[b * RPS + r] : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(xv, f[j], acc[b][j]);
            }
        }
    }
    // row groups of one wavefront, then the wavefronts through LDS, in a fixed order
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][j] += __shfl_xor(acc[b][j], off);
    if ((tid & 63) < LPR) {
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) red[(wv * BT + b) * HD + lig * 8 + j] = acc[b][j];
    }
    __syncthreads();
    for (int e = tid; e < BT * HD; e += NT) {
        const int b = e / HD, c = e - b * HD;
        if (b < p.B) {
            float s = 0.f;
#pragma unroll
            for (int w8 = 0; w8 < NW; ++w8) s += red[(w8 * BT + b) * HD + c];
            st_coh(p.p1 + ((size_t)ks * p.B + b) * p.nqkv + col0 + c, s);
        }
    }
    __syncthreads();
}

// cos/sin of pos * inv_freq[i] for i < HD/2, angle and range reduction in fp64.
template <int HD>
__device__ void rope_table(const Params &p, float *cs, float *sn)
{
    const int i = threadIdx.x;
    if (i < HD / 2) {
        const double ang = (double)p.pos * p.inv_freq[i];
        const double k = rint(ang * 0.63661977236758134308);              // 2/pi
        double r = fma(-k, 1.57079632679489655800e+00, ang);              // pi/2, high part
        r = fma(-k, 6.12323399573676603587e-17, r);                       // pi/2, low part
        const double r2 = r * r;                                          // |r| <= pi/4: Taylor series
        double s = -1.0 / 1307674368000.0;
        s = fma(s, r2, 1.0 / 6227020800.0);
        s = fma(s, r2, -1.0 / 39916800.0);
        s = fma(s, r2, 1.0 / 362880.0);
        s = fma(s, r2, -1.0 / 5040.0);
        s = fma(s, r2, 1.0 / 120.0);
        s = fma(s, r2, -1.0 / 6.0);
        s = fma(s * r2, r, r);
        double c = 1.0 / 20922789888000.0;
        c = fma(c, r2, -1.0 / 87178291200.0);
        c = fma(c, r2, 1.0 / 479001600.0);
        c = fma(c, r2, -1.0 / 3628800.0);
        c = fma(c, r2, 1.0 / 40320.0);
        c = fma(c, r2, -1.0 / 720.0);
        c = fma(c, r2, 1.0 / 24.0);
        c = fma(c, r2, -0.5);
        c = fma(c, r2, 1.0);
        const int q = (int)((long long)k & 3);
        const double sv = (q == 0) ? s : (q == 1) ? c : (q == 2) ? -s : -c;
        const double cv = (q == 0) ? c : (q == 1) ? -s : (q == 2) ? -c : s;
        cs[i] = (float)cv;
        sn[i] = (float)sv;
    }
}

// ---------------------------------------------------------------------------
// Phase 2: one (batch row, KV split) of the team's KV head, all G query heads
// (Alg. 3 steps 3-4; the new token is counted by the last split only)
// ---------------------------------------------------------------------------
template <int HD, int G>
__device__ void p2_item(const Params &p, int team, int b, int s, float *smem)
{
    constexpr int LPR = HD / 8;
    constexpr int NG = NT / LPR;
    constexpr int U = 4;
    constexpr int PS = HD + kP2Stride;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const bool last = (s == p.NS - 1);

    float *cs = smem;                       // [HD/2]  (filled by rope_table before the first item)
    float *sn = cs + HD / 2;                // [HD/2]
    float *qs = sn + HD / 2;                // [G][HD]
    float *kn = qs + G * HD;                // [HD] rotated new key
    float *vn = kn + HD;                    // [HD] new value
    float *snew = vn + HD;                  // [8]  scores of the new token, log2 domain
    float *redm = snew + 8;                 // [G][NW]
    float *redl = redm + G * NW;            // [G][NW]
    float *redacc = redl + G * NW;          // [G][NW][HD]

    // ---- sum the projection partials this item needs (the gather of Alg. 3 step 3)
    const int nsel = last ? G + 2 : G;
    for (int e = tid; e < nsel * HD; e += NT) {
        const int sel = e / HD, c = e - sel * HD;
        const int col = qkv_col0<HD, G>(p, team, sel) + c;
        const float *src = p.p1 + (size_t)b * p.nqkv + col;
        float v = 0.f;
        for (int k = 0; k < p.KS; ++k) v += ld_coh(src + (size_t)k * p.B * p.nqkv);
        qs[e] = v;                           // qs, kn, vn are contiguous
    }
    __syncthreads();
    // ---- RoPE on the query heads and, for the last split, the new key
    const int nrot = last ? G + 1 : G;
    for (int e = tid; e < nrot * (HD / 2); e += NT) {
        const int sel = e / (HD / 2), i = e - sel * (HD / 2);
        float *v = qs + sel * HD;
        const float lo = v[i], hi = v[i + HD / 2], c = cs[i], sgn = sn[i];
        v[i] = lo * c - hi * sgn;
        v[i + HD / 2] = hi * c + lo * sgn;
    }
    __syncthreads();
    if (last) {
        // ---- append the new key/value (Sec. 2.1) and score the new token
        const size_t row = (((size_t)b * p.nkv + team) * p.max_seq + p.pos) * HD;
        if (tid < HD)
            p.kc[row + tid] = f2h(kn[tid]);
        else if (tid < 2 * HD)
            p.vc[row + tid - HD] = f2h(vn[tid - HD]);
        for (int g = wv; g < G; g += NW) {
            float d = 0.f;
            for (int c = lane; c < HD; c += 64) d = fmaf(qs[g * HD + c], kn[c], d);
            d = wave_sum(d);
            if (lane == 0) snew[g] = d * p.qk_scale_log2e;
        }
        if (p.dbg_q)
            for (int e = tid; e < G * HD; e += NT)
                p.dbg_q[((size_t)b * p.nq + team * G) * HD + e] = qs[e];
    }
    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int j = 0; j < 8; ++j) qf[g][j] = qs[g * HD + lig * 8 + j] * p.qk_scale_log2e;

    // ---- online softmax over this split's cached tokens; one row per LPR lanes
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig;
        l[g] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] = 0.f;
    }
    const int t0 = s * p.TPS;
    const int t1 = min(t0 + p.TPS, p.pos);
    if (t1 > t0) {
        const size_t head = ((size_t)b * p.nkv + team) * p.max_seq * HD;
        const uint16_t *kbase = p.kc + head + lig * 8;
        const uint16_t *vbase = p.vc + head + lig * 8;
        const int iters = (t1 - t0 + NG - 1) / NG;
        for (int i0 = 0; i0 < iters; i0 += U) {
            h8 kr[U], vr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0 + grp + NG * (i0 + u);
                const int tt = t < t1 ? t : t0;
                kr[u] = ld_stream(kbase + (size_t)tt * HD);
                vr[u] = ld_stream(vbase + (size_t)tt * HD);
            }
            float sc[G][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[8];
                unpack8(kr[u], kf);
                const bool ok = (t0 + grp + NG * (i0 + u)) < t1;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int j = 0; j < 8; ++j) d = fmaf(qf[g][j], kf[j], d);
                    d = row_sum<LPR>(d);
                    sc[g][u] = ok ? d : kNegBig;
                }
            }
            float pr[G][U];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mn = m[g];
#pragma unroll
                for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[g][u]);
                const float scale = __builtin_amdgcn_exp2f(m[g] - mn);
                m[g] = mn;
                float ls = l[g] * scale;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool ok = (t0 + grp + NG * (i0 + u)) < t1;
                    pr[g][u] = ok ? __builtin_amdgcn_exp2f(sc[g][u] - mn) : 0.f;
                    ls += pr[g][u];
                }
                l[g] = ls;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[g][j] *= scale;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[8];
                unpack8(vr[u], vf);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pr[g][u], vf[j], acc[g][j]);
            }
        }
    }
    // ---- merge the row groups of a wavefront, then the wavefronts and the new token
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(l[g], off);
            const float mn = fmaxf(m[g], mo);
            const float sa = __builtin_amdgcn_exp2f(m[g] - mn), sb = __builtin_amdgcn_exp2f(mo - mn);
            l[g] = l[g] * sa + lo * sb;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float ao = __shfl_xor(acc[g][j], off);
                acc[g][j] = acc[g][j] * sa + ao * sb;
            }
            m[g] = mn;
        }
    }
    if (lane < LPR) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (lane == 0) {
                redm[g * NW + wv] = m[g];
                redl[g * NW + wv] = l[g];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) redacc[(g * NW + wv) * HD + lig * 8 + j] = acc[g][j];
        }
    }
    __syncthreads();
    for (int e = tid; e < G * HD; e += NT) {
        const int g = e / HD, c = e - g * HD;
        float M = last ? snew[g] : kNegBig;
#pragma unroll
        for (int w8 = 0; w8 < NW; ++w8) M = fmaxf(M, redm[g * NW + w8]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < NW; ++w8) {
            const float f = __builtin_amdgcn_exp2f(redm[g * NW + w8] - M);
            L = fmaf(redl[g * NW + w8], f, L);
            A = fmaf(redacc[(g * NW + w8) * HD + c], f, A);
        }
        if (last) {
            const float f = __builtin_amdgcn_exp2f(snew[g] - M);
            L += f;
            A = fmaf(vn[c], f, A);
        }
        float *dst = p.p2 + (((size_t)b * p.nq + team * G + g) * p.NS + s) * PS;
        if (c == 0) {
            st_coh(dst, M);
            st_coh(dst + 1, L);
        }
        st_coh(dst + kP2Stride + c, A);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Phase 3: merge the split-KV partials of head hq (Alg. 3 steps 5-7), multiply by
// rows [rs*HD/RS3, (rs+1)*HD/RS3) x columns [c3*CW3, (c3+1)*CW3) of that head's
// W_o block (step 8), then add the heads once all partials of a chunk are in.
// ---------------------------------------------------------------------------
template <int HD, int BT>
__device__ void p3_item(const Params &p, int hq, int c3, int rs, float *smem)
{
    constexpr int U = 8;
    constexpr int RB = BT < 4 ? BT : 4;
    constexpr int PS = HD + kP2Stride;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    float *as = smem;                 // [BT][HD] merged, normalised attention output of head hq
    float *red = smem + BT * HD;      // [NW][RB][512]
    __shared__ int s_last;

    for (int e = tid; e < BT * HD; e += NT) {
        const int b = e / HD, c = e - b * HD;
        float a = 0.f;
        if (b < p.B) {
            const float *src = p.p2 + ((size_t)b * p.nq + hq) * p.NS * PS;
            float M = kNegBig;
            for (int s = 0; s < p.NS; ++s) M = fmaxf(M, ld_coh(src + (size_t)s * PS));
            float L = 0.f, A = 0.f;
            for (int s = 0; s < p.NS; ++s) {
                const float f = __builtin_amdgcn_exp2f(ld_coh(src + (size_t)s * PS) - M);
                L = fmaf(ld_coh(src + (size_t)s * PS + 1), f, L);
                A = fmaf(ld_coh(src + (size_t)s * PS + kP2Stride + c), f, A);
            }
            a = A / L;
            if (p.dbg_attn && c3 == 0 && rs == 0) p.dbg_attn[((size_t)b * p.nq + hq) * HD + c] = a;
        }
        as[e] = a;
    }
    __syncthreads();

    const int nrows = HD / p.RS3;
    const int rbeg = rs * nrows;
    const int slot = hq * p.RS3 + rs;
    const int nslots = p.nq * p.RS3;
    const int nchunk = p.CW3 / kOutChunk;
    for (int ch = 0; ch < nchunk; ++ch) {
        const int cbase = c3 * p.CW3 + ch * kOutChunk;
        if (cbase >= p.D) break;
        const int col = cbase + lane * 8;
        const bool cok = col < p.D;
        float acc[BT][8];
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
        const uint16_t *wbase = p.wo + ((size_t)hq * HD + rbeg) * p.D + (cok ? col : 0);
        const int iters = nrows / NW;
        for (int i0 = 0; i0 < iters; i0 += U) {
            h8 w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = wv + NW * (i0 + u);
                const int rr = (i0 + u) < iters ? r : wv;
                w[u] = ld_stream(wbase + (size_t)rr * p.D);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + u < iters) {
                    const int r = rbeg + wv + NW * (i0 + u);
                    float f[8];
                    unpack8(w[u], f);
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        const float av = as[b * HD + r];
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(av, f[j], acc[b][j]);
                    }
                }
            }
        }
        // wavefronts -> one partial row per batch row, RB batch rows at a time
#pragma unroll
        for (int bb = 0; bb < BT; bb += RB) {
#pragma unroll
            for (int b = 0; b < RB; ++b)
#pragma unroll
                for (int j = 0; j < 8; ++j) red[(wv * RB + b) * kOutChunk + lane * 8 + j] = acc[bb + b][j];
            __syncthreads();
            for (int e = tid; e < RB * kOutChunk; e += NT) {
                const int b = e / kOutChunk, cc = e - b * kOutChunk;
                if (bb + b < p.B && cbase + cc < p.D) {
                    float sum = 0.f;
#pragma unroll
                    for (int w8 = 0; w8 < NW; ++w8) sum += red[(w8 * RB + b) * kOutChunk + cc];
                    st_coh(p.p3 + ((size_t)slot * p.B + bb + b) * p.D + cbase + cc, sum);
                }
            }
            __syncthreads();
        }
        // ---- ticket of this 512-column chunk; the last arriver adds all heads' partials
        if (tid == 0) {
            const uint32_t old = __hip_atomic_fetch_add(p.cnt3 + (size_t)(cbase / kOutChunk) * kCounterStride, 1u,
                                                        __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (old == (uint32_t)nslots - 1u);
        }
        __syncthreads();
        if (s_last) {
            for (int e = tid; e < p.B * kOutChunk; e += NT) {
                const int b = e / kOutChunk, cc = e - b * kOutChunk;
                if (cbase + cc < p.D) {
                    const float *src = p.p3 + (size_t)b * p.D + cbase + cc;
                    float sum = 0.f;
                    for (int sl = 0; sl < nslots; ++sl) sum += ld_coh(src + (size_t)sl * p.B * p.D);
                    p.out[(size_t)b * p.D + cbase + cc] = f2h(sum);
                }
            }
        }
        __syncthreads();
    }
}

template <int HD, int G, int BT>
__global__ void __launch_bounds__(NT) fused_decode_block(const Params p)
{
    extern __shared__ float smem[];
    __shared__ int s_flag;
    const int tid = threadIdx.x;
    const int team = blockIdx.x % p.nkv;
    const int member = blockIdx.x / p.nkv;

    // ---- phase 1
    {
        const int n1 = (G + 2) * p.KS;
        uint32_t mine = 0;
        for (int it = member; it < n1; it += p.TS, ++mine)
            p1_item<HD, BT>(p, qkv_col0<HD, G>(p, team, it / p.KS), it % p.KS, smem);
        team_signal(p.cnt1 + (size_t)team * kCounterStride, mine);
    }
    // ---- phase 2
    {
        const int n2 = p.B * p.NS;
        uint32_t mine = 0;
        if (member < n2) {
            rope_table<HD>(p, smem, smem + HD / 2);       // does not depend on phase 1
            team_wait(p, p.cnt1 + (size_t)team * kCounterStride, (uint32_t)((G + 2) * p.KS));
            for (int it = member; it < n2; it += p.TS, ++mine) p2_item<HD, G>(p, team, it / p.NS, it % p.NS, smem);
        }
        team_signal(p.cnt2 + (size_t)team * kCounterStride, mine);
    }
    // ---- phase 3
    {
        const int n3 = G * p.NC3 * p.RS3;
        if (member < n3) {
            team_wait(p, p.cnt2 + (size_t)team * kCounterStride, (uint32_t)(p.B * p.NS));
            for (int it = member; it < n3; it += p.TS) {
                const int g = it / (p.NC3 * p.RS3), rem = it - g * (p.NC3 * p.RS3);
                p3_item<HD, BT>(p, team * G + g, rem / p.RS3, rem % p.RS3, smem);
            }
        }
    }
    // ---- the last workgroup to finish clears the counters for the next launch
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(p.done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        s_flag = (old == (uint32_t)p.W - 1u);
    }
    __syncthreads();
    if (s_flag) {
        for (int i = tid; i < p.nkv; i += NT) {
            __hip_atomic_store(p.cnt1 + (size_t)i * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.cnt2 + (size_t)i * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        for (int i = tid; i < p.NCH; i += NT)
            __hip_atomic_store(p.cnt3 + (size_t)i * kCounterStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid == 0) __hip_atomic_store(p.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

using KernelFn = void (*)(const Params);

template <int HD, int G>
KernelFn pick_bt(int bt)
{
    switch (bt) {
    case 1: return fused_decode_block<HD, G, 1>;
    case 4: return fused_decode_block<HD, G, 4>;
    case 16: return fused_decode_block<HD, G, 16>;
    default: return nullptr;
    }
}

template <int HD>
KernelFn pick_g(int g, int bt)
{
    switch (g) {
    case 1: return pick_bt<HD, 1>(bt);
    case 2: return pick_bt<HD, 2>(bt);
    case 4: return pick_bt<HD, 4>(bt);
    case 8: return pick_bt<HD, 8>(bt);
    default: return nullptr;
    }
}

KernelFn pick(int hd, int g, int bt)
{
    if (hd == 64) return pick_g<64>(g, bt);
    if (hd == 128) return pick_g<128>(g, bt);
    return nullptr;
}

}  // namespace

size_t lds_floats(const Params &p, int hd, int g, int bt)
{
    const size_t rb = bt < 4 ? bt : 4;
    const size_t f1 = (size_t)bt * p.RPS + (size_t)kWaves * bt * hd;
    const size_t f2 = (size_t)hd + (size_t)(g + 2) * hd + 8 + 2 * (size_t)g * kWaves + (size_t)g * kWaves * hd;
    const size_t f3 = (size_t)bt * hd + (size_t)kWaves * rb * kOutChunk;
    size_t f = f1 > f2 ? f1 : f2;
    return f > f3 ? f : f3;
}

hipError_t max_workgroups_per_cu(int hd, int g, int bt, size_t lds_bytes, int *out)
{
    KernelFn fn = pick(hd, g, bt);
    *out = 0;
    if (!fn) return hipSuccess;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void *>(fn), kThreads, lds_bytes);
}

hipError_t launch_fused(const Params &p, int hd, int g, int bt, size_t lds_bytes, hipStream_t stream)
{
    KernelFn fn = pick(hd, g, bt);
    if (!fn) return hipErrorInvalidDeviceFunction;
    hipLaunchKernelGGL(fn, dim3(p.W), dim3(kThreads), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace cf
