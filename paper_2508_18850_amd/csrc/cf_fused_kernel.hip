// Fused decode-block kernel for gfx950: QKV projection + RoPE + KV append +
// split-KV attention + output projection in one launch (paper Alg. 3).
//
// Mapping.  The paper maps one attention head to a cluster of thread blocks and
// resolves the dependencies between the blocks of a cluster with ClusterGather
// and ClusterReduce over distributed shared memory.  gfx950 has no clusters, so
// a "team" of workgroups (all workgroups whose index is congruent modulo
// n_kv_heads; with 8 | n_kv_heads they share one XCD) serves one KV head
// together with the query heads that use it.  Every member streams, in this
// order, so that each dependency falls behind a stream that does not need it:
//   1a  its slice of the reduction dimension of the team's W_q columns
//       (split-K instead of the paper's split of the head dimension: rows of 256
//       contiguous bytes coalesce, 32 columns would not)
//   1b  the same slice of the team's W_k / W_v columns
//   2   the first K/V rows are put in flight, then the q partials of the team
//       are summed (the role of ClusterGather) and rotated; online-softmax
//       attention over the member's slice of the cached sequence (Alg. 3 step
//       4); the member with the last slice also sums the k/v partials, appends
//       the new key/value and counts the new token
//   3   its block of W_o is loaded into registers, then the split-KV partials of
//       the head are merged (Alg. 3 steps 5-7, local sums rescaled by
//       exp(m_i - M) before being added) and multiplied (step 8) into a per-head
//       partial of the output
//   4   every workgroup adds, over all heads and in a fixed order, the partials
//       of its own few output columns (the paper uses atomicAdd) and writes fp16.
// Exchange between workgroups needs no counters: every exchanged fp32 value is
// stored as a 64-bit {value, stamp} pair with one write-through store, the stamp
// being the launch number; a reader polls the pair until the stamp is current.
// The launch number is read from a counter of finished workgroups.  All
// workgroups of the launch must be resident (checked on the host), since
// readers spin.  Spins are bounded: after spin_ticks a thread sets an error
// flag and goes on, so the kernel always ends.
#include "cf_params.h"

namespace cf {
namespace {

constexpr int NT = kThreads;
constexpr int NW = kWaves;
constexpr float kNegBig = -1.0e30f;   // stands for "no score yet"; finite so that differences never give NaN

typedef _Float16 h8 __attribute__((ext_vector_type(8)));   // eight fp16 values = one 128-bit load
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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

__device__ __forceinline__ float h2f(uint16_t bits) { return (float)__builtin_bit_cast(_Float16, bits); }
__device__ __forceinline__ uint16_t f2h(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }

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

// Exchange slots (partials handed from one workgroup to another).  A slot is a 64-bit
// {fp32 bits, stamp} pair written by ONE 8-byte write-through store (agent scope), so a
// reader sees either the old pair or the new one; the stamp of a launch is its number.
struct Xbuf {
    __amdgpu_buffer_rsrc_t r;
    __device__ __forceinline__ explicit Xbuf(const void *base)
        : r(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0xfffffff8u, 0x00020000)) {}
    __device__ __forceinline__ u32x2 ld(size_t idx) const
    {
        return __builtin_amdgcn_raw_buffer_load_b64(r, (unsigned)(idx * 8), 0, 16);
    }
    __device__ __forceinline__ void st(size_t idx, float v, uint32_t stamp) const
    {
        u32x2 d = {__builtin_bit_cast(uint32_t, v), stamp};
        __builtin_amdgcn_raw_buffer_store_b64(d, r, (unsigned)(idx * 8), 0, 16);
    }
};

// Bounded spinning: returns true when the caller should give up.
struct Spin {
    long long t0 = 0;
    __device__ __forceinline__ bool expired(const Params &p)
    {
        __builtin_amdgcn_s_sleep(1);
        const long long now = wall_clock64();
        if (t0 == 0) t0 = now;
        if (now - t0 > p.spin_ticks) {
            __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        return false;
    }
};

// Sum of n stamped slots base, base+stride, ... in index order; spins until all are current.
__device__ __forceinline__ float ll_sum(const Params &p, const Xbuf &x, size_t base, size_t stride, int n,
                                        uint32_t stamp)
{
    Spin spin;
    for (;;) {
        float s = 0.f;
        bool ok = true;
#pragma unroll 8
        for (int k = 0; k < n; ++k) {
            const u32x2 v = x.ld(base + (size_t)k * stride);
            ok &= (v.y == stamp);
            s += __builtin_bit_cast(float, v.x);
        }
        if (ok || spin.expired(p)) return s;
    }
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
// Phase 1 (Alg. 3 step 2, split over the reduction dimension): for the selectors
// sel0, sel0+dsel, ... < sel_end accumulate x[b][r0..r0+nrows) . W[r0.., col0(sel)..+HD)
// and store the partials into slot ks of the exchange buffer.
// ---------------------------------------------------------------------------
template <int HD, int BT>
__device__ __forceinline__ void p1_stream(const Params &p, const float *xs, const uint16_t *wbase, int nrows, int grp,
                                          float (&acc)[BT][8])
{
    constexpr int NG = NT / (HD / 8);
    constexpr int U = 8;
    const int iters = (nrows + NG - 1) / NG;
    auto load = [&](h8(&w)[U], int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = grp + NG * (i0 + u);
            w[u] = ld_stream(wbase + (size_t)(r < nrows ? r : 0) * p.nqkv);
        }
    };
    auto consume = [&](const h8(&w)[U], int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = grp + NG * (i0 + u);
            const bool ok = r < nrows;
            float f[8];
            unpack8(w[u], f);
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const float xv = ok ? xs[b * p.RPS + r] : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(xv, f[j], acc[b][j]);
            }
        }
    };
    h8 wa[U], wb[U];
    if (iters > 0) load(wa, 0);
    for (int i0 = 0; i0 < iters; i0 += 2 * U) {
        if (i0 + U < iters) load(wb, i0 + U);
        consume(wa, i0);
        if (i0 + 2 * U < iters) load(wa, i0 + 2 * U);
        if (i0 + U < iters) consume(wb, i0 + U);
    }
}

template <int HD, int G, int BT>
__device__ void p1_pass(const Params &p, int team, int ks, int sel0, int dsel, int sel_end, uint32_t stamp,
                        const float *xs, float *red)
{
    constexpr int LPR = HD / 8;
    constexpr int MAXI = BT == 1 ? 4 : (BT <= 4 ? 2 : 1);   // items whose wave partials are buffered in LDS
    const int tid = threadIdx.x, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const int r0 = ks * p.RPS;
    const int nrows = min(p.RPS, p.D - r0);
    const Xbuf x1(p.p1);
    int sels[MAXI];
    int nbuf = 0;
    auto flush = [&]() {
        __syncthreads();
        for (int e = tid; e < nbuf * BT * HD; e += NT) {
            const int it = e / (BT * HD), rem = e - it * (BT * HD);
            const int b = rem / HD, c = rem - b * HD;
            if (b < p.B) {
                float s = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < NW; ++w8) s += red[((it * NW + w8) * BT + b) * HD + c];
                int sel = sels[0];
#pragma unroll
                for (int k = 1; k < MAXI; ++k) sel = (it == k) ? sels[k] : sel;
                x1.st(((size_t)ks * p.B + b) * p.nqkv + qkv_col0<HD, G>(p, team, sel) + c, s, stamp);
            }
        }
        __syncthreads();
        nbuf = 0;
    };
    for (int sel = sel0; sel < sel_end; sel += dsel) {
        float acc[BT][8];
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
        const uint16_t *wbase = p.wqkv + (size_t)r0 * p.nqkv + qkv_col0<HD, G>(p, team, sel) + lig * 8;
        p1_stream<HD, BT>(p, xs, wbase, nrows, grp, acc);
        // row groups of one wavefront by shuffles; the wavefronts are added in flush(), in a fixed order
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
                for (int j = 0; j < 8; ++j) red[((nbuf * NW + wv) * BT + b) * HD + lig * 8 + j] = acc[b][j];
        }
#pragma unroll
        for (int k = 0; k < MAXI; ++k)
            if (nbuf == k) sels[k] = sel;
        if (++nbuf == MAXI) flush();
    }
    if (nbuf) flush();
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
__device__ void p2_item(const Params &p, int team, int b, int s, uint32_t stamp, bool first, float *smem)
{
    constexpr int LPR = HD / 8;
    constexpr int NG = NT / LPR;
    constexpr int U = G >= 8 ? 2 : (G >= 4 ? 4 : 8);   // tokens per row group in one batch of loads
    constexpr int PS = HD + kP2Stride;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const bool last = (s == p.NS - 1);
    const Xbuf x1(p.p1), x2(p.p2);

    float *cs = smem;                       // [HD/2]
    float *sn = cs + HD / 2;                // [HD/2]
    float *qs = sn + HD / 2;                // [G][HD]
    float *kn = qs + G * HD;                // [HD] rotated new key
    float *vn = kn + HD;                    // [HD] new value
    float *snew = vn + HD;                  // [8]  scores of the new token, log2 domain
    float *redm = snew + 8;                 // [G][NW]
    float *redl = redm + G * NW;            // [G][NW]
    float *redacc = redl + G * NW;          // [G][NW][HD]

    const int t0 = s * p.TPS;
    const int t1 = min(t0 + p.TPS, p.pos);
    const int iters = t1 > t0 ? (t1 - t0 + NG - 1) / NG : 0;
    const size_t head = ((size_t)b * p.nkv + team) * p.max_seq * HD;
    const uint16_t *kbase = p.kc + head + lig * 8;
    const uint16_t *vbase = p.vc + head + lig * 8;
    auto load = [&](h8(&kr)[U], h8(&vr)[U], int i0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + grp + NG * (i0 + u);
            const size_t off = (size_t)(t < t1 ? t : t0) * HD;
            kr[u] = ld_stream(kbase + off);
            vr[u] = ld_stream(vbase + off);
        }
    };
    // ---- the first batch of K/V rows does not depend on q: put it in flight before waiting
    h8 ka[U], va[U], kb[U], vb[U];
    if (iters > 0) load(ka, va, 0);
    if (first) rope_table<HD>(p, cs, sn);
    // ---- sum the projection partials of the team (the gather of Alg. 3 step 3): q heads, and for
    //      the last split also the new key and value; then RoPE on q and the key
    const int nsel = last ? G + 2 : G;
    for (int e = tid; e < nsel * HD; e += NT) {
        const int sel = e / HD, c = e - sel * HD;
        const size_t src = (size_t)b * p.nqkv + qkv_col0<HD, G>(p, team, sel) + c;
        qs[e] = ll_sum(p, x1, src, (size_t)p.B * p.nqkv, p.KS, stamp);     // qs, kn, vn are contiguous
    }
    __syncthreads();
    const int nrot = last ? G + 1 : G;
    for (int e = tid; e < nrot * (HD / 2); e += NT) {
        const int sel = e / (HD / 2), i = e - sel * (HD / 2);
        float *v = qs + sel * HD;
        const float lo = v[i], hi = v[i + HD / 2], c = cs[i], sgn = sn[i];
        v[i] = lo * c - hi * sgn;
        v[i + HD / 2] = hi * c + lo * sgn;
    }
    __syncthreads();
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
    auto consume = [&](const h8(&kr)[U], const h8(&vr)[U], int i0) {
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
    };
    for (int i0 = 0; i0 < iters; i0 += 2 * U) {
        if (i0 + U < iters) load(kb, vb, i0 + U);
        consume(ka, va, i0);
        if (i0 + 2 * U < iters) load(ka, va, i0 + 2 * U);
        if (i0 + U < iters) consume(kb, vb, i0 + U);
    }
    // ---- merge the row groups of a wavefront
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
    if (last) {
        // ---- the new token: append its key/value (Sec. 2.1) and score it
        const size_t row = head + (size_t)p.pos * HD;
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
            for (int e = tid; e < G * HD; e += NT) p.dbg_q[((size_t)b * p.nq + team * G) * HD + e] = qs[e];
    }
    __syncthreads();
    // ---- the wavefronts and the new token -> one partial (m, l, acc) per query head
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
        const size_t dst = (((size_t)b * p.nq + team * G + g) * p.NS + s) * PS;
        if (c == 0) {
            x2.st(dst, M, stamp);
            x2.st(dst + 1, L, stamp);
        }
        x2.st(dst + kP2Stride + c, A, stamp);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Phase 3: merge the split-KV partials of head hq (Alg. 3 steps 5-7), multiply by
// rows [rs*HD/RS3, (rs+1)*HD/RS3) x columns [c3*CW3, (c3+1)*CW3) of that head's
// W_o block (step 8), then add the heads once all partials of a chunk are in.
// The first 512-column chunk of the first item is loaded before the wait.
// ---------------------------------------------------------------------------
template <int HD>
struct OutTile {
    static constexpr int MAXR = HD / NW;   // W_o rows per wavefront when a head is not split over rows
    h8 w[MAXR];
};

template <int HD>
__device__ __forceinline__ void p3_load(const Params &p, int hq, int c3, int rs, int ch, OutTile<HD> &t)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int nrows = HD / p.RS3;
    const int cbase = c3 * p.CW3 + ch * kOutChunk;
    const int col = cbase + lane * 8;
    const uint16_t *wbase = p.wo + ((size_t)hq * HD + rs * nrows) * p.D + (col < p.D ? col : 0);
    const int iters = nrows / NW;
#pragma unroll
    for (int u = 0; u < OutTile<HD>::MAXR; ++u) {
        const int rr = u < iters ? wv + NW * u : wv;
        t.w[u] = ld_stream(wbase + (size_t)rr * p.D);
    }
}

template <int HD, int BT>
__device__ void p3_item(const Params &p, int hq, int c3, int rs, uint32_t stamp, float *smem)
{
    constexpr int RB = BT < 4 ? BT : 4;
    constexpr int PS = HD + kP2Stride;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    float *as = smem;                 // [BT][HD] merged, normalised attention output of head hq
    float *red = smem + BT * HD;      // [NW][RB][512]
    const Xbuf x2(p.p2), x3(p.p3);

    const int nrows = HD / p.RS3;
    const int rbeg = rs * nrows;
    const int iters = nrows / NW;
    const int slot = hq * p.RS3 + rs;
    const int nchunk = p.CW3 / kOutChunk;

    OutTile<HD> tile;
    p3_load<HD>(p, hq, c3, rs, 0, tile);                 // independent of the attention result

    for (int e = tid; e < BT * HD; e += NT) {
        const int b = e / HD, c = e - b * HD;
        float a = 0.f;
        if (b < p.B) {
            const size_t src = ((size_t)b * p.nq + hq) * p.NS * PS;
            Spin spin;
            for (;;) {
                bool ok = true;
                float M = kNegBig;
#pragma unroll 8
                for (int s = 0; s < p.NS; ++s) {
                    const u32x2 v = x2.ld(src + (size_t)s * PS);
                    ok &= (v.y == stamp);
                    M = fmaxf(M, __builtin_bit_cast(float, v.x));
                }
                float L = 0.f, A = 0.f;
#pragma unroll 8
                for (int s = 0; s < p.NS; ++s) {
                    const u32x2 vm = x2.ld(src + (size_t)s * PS), vl = x2.ld(src + (size_t)s * PS + 1),
                                va = x2.ld(src + (size_t)s * PS + kP2Stride + c);
                    ok &= (vl.y == stamp) & (va.y == stamp);
                    const float f = __builtin_amdgcn_exp2f(__builtin_bit_cast(float, vm.x) - M);
                    L = fmaf(__builtin_bit_cast(float, vl.x), f, L);
                    A = fmaf(__builtin_bit_cast(float, va.x), f, A);
                }
                a = A / L;
                if (ok || spin.expired(p)) break;
            }
            if (p.dbg_attn && c3 == 0 && rs == 0) p.dbg_attn[((size_t)b * p.nq + hq) * HD + c] = a;
        }
        as[e] = a;
    }
    __syncthreads();

    for (int ch = 0; ch < nchunk; ++ch) {
        const int cbase = c3 * p.CW3 + ch * kOutChunk;
        if (cbase >= p.D) break;
        if (ch > 0) p3_load<HD>(p, hq, c3, rs, ch, tile);
        float acc[BT][8];
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
#pragma unroll
        for (int u = 0; u < OutTile<HD>::MAXR; ++u) {
            if (u < iters) {
                const int r = rbeg + wv + NW * u;
                float f[8];
                unpack8(tile.w[u], f);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float av = as[b * HD + r];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(av, f[j], acc[b][j]);
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
                    x3.st(((size_t)slot * p.B + bb + b) * p.D + cbase + cc, sum, stamp);
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------
// Phase 4: every workgroup owns ceil(D/W) output columns and adds the per-head
// partials of those columns in slot order (the cross-head reduction that the paper
// does with atomicAdd), then writes fp16.
// ---------------------------------------------------------------------------
__device__ void final_reduce(const Params &p, uint32_t stamp, float *smem)
{
    const int tid = threadIdx.x;
    const Xbuf x3(p.p3);
    const int nslots = p.nq * p.RS3;
    const int cpw = (p.D + p.W - 1) / p.W;
    const int c0 = blockIdx.x * cpw;
    const int ncol = min(cpw, p.D - c0);
    if (ncol <= 0) return;
    const int nv = ncol * p.B;                       // values this workgroup produces
    for (int v0 = 0; v0 < nv; v0 += NT) {
        const int cb = min(NT, nv - v0);
        const int spt = min(NT / cb, nslots);        // slots read in parallel
        const int v = tid % cb, s0 = tid / cb;
        const int b = (v0 + v) / ncol, c = (v0 + v) - b * ncol;
        if (s0 < spt) {
            const int n = (nslots - s0 + spt - 1) / spt;
            smem[s0 * cb + v] = ll_sum(p, x3, (size_t)s0 * p.B * p.D + (size_t)b * p.D + c0 + c,
                                       (size_t)spt * p.B * p.D, n, stamp);
        }
        __syncthreads();
        if (tid < cb) {
            float sum = 0.f;
            for (int k = 0; k < spt; ++k) sum += smem[k * cb + tid];
            p.out[(size_t)b * p.D + c0 + c] = f2h(sum);
        }
        __syncthreads();
    }
}

template <int HD, int G, int BT>
__global__ void __launch_bounds__(NT) fused_decode_block(const Params p)
{
    extern __shared__ float smem[];
    __shared__ uint32_t s_stamp;
    const int tid = threadIdx.x;
    const int team = blockIdx.x % p.nkv;
    const int member = blockIdx.x / p.nkv;
    auto stamp_t = [&](int k) {
        if (p.dbg_t && tid == 0) p.dbg_t[(size_t)blockIdx.x * 8 + k] = wall_clock64();
    };
    stamp_t(0);
    if (p.dbg_t && tid == 0)   // where this workgroup runs: XCC id and the HW_ID register (CU, SE ...)
        p.dbg_t[(size_t)blockIdx.x * 8 + 7] = ((unsigned long long)__builtin_amdgcn_s_getreg(63508) << 32) |
                                              (unsigned)__builtin_amdgcn_s_getreg(63492);
    // launch number = finished workgroups / workgroups per launch + 1.  A workgroup of this launch
    // that starts late still sees fewer than W finished ones of this launch, hence the same value.
    if (tid == 0) {
        const unsigned long long fin = __hip_atomic_load(p.done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_stamp = (uint32_t)(fin / (unsigned long long)p.W + 1ull);
    }
    __syncthreads();
    const uint32_t stamp = s_stamp;

    // ---- phase 1: this member's slice ks of the reduction dimension, q selectors first, then k / v
    {
        const int ks = member % p.KS;
        const int sel0 = member / p.KS, dsel = p.TS / p.KS;
        const int r0 = ks * p.RPS;
        const int nrows = min(p.RPS, p.D - r0);
        float *xs = smem;                       // [BT][RPS]
        float *red = smem + BT * p.RPS;
        for (int i = tid; i < BT * p.RPS; i += NT) {
            const int b = i / p.RPS, r = i - b * p.RPS;
            xs[i] = (b < p.B && r < nrows) ? h2f(p.x[(size_t)b * p.D + r0 + r]) : 0.f;
        }
        __syncthreads();
        p1_pass<HD, G, BT>(p, team, ks, sel0, dsel, G, stamp, xs, red);
        stamp_t(1);
        p1_pass<HD, G, BT>(p, team, ks, G + sel0, dsel, G + 2, stamp, xs, red);
        stamp_t(2);
    }
    // ---- phase 2
    {
        const int n2 = p.B * p.NS;
        bool first = true;
        for (int it = member; it < n2; it += p.TS, first = false)
            p2_item<HD, G>(p, team, it / p.NS, it % p.NS, stamp, first, smem);
        stamp_t(3);
    }
    // ---- phase 3
    {
        const int n3 = G * p.NC3 * p.RS3;
        for (int it = member; it < n3; it += p.TS) {
            const int g = it / (p.NC3 * p.RS3), rem = it - g * (p.NC3 * p.RS3);
            p3_item<HD, BT>(p, team * G + g, rem / p.RS3, rem % p.RS3, stamp, smem);
        }
        stamp_t(4);
    }
    // ---- phase 4
    final_reduce(p, stamp, smem);
    stamp_t(5);
    if (tid == 0) __hip_atomic_fetch_add(p.done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    stamp_t(6);
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
    const size_t maxi = bt == 1 ? 4 : (bt <= 4 ? 2 : 1);
    const size_t f1 = (size_t)bt * p.RPS + maxi * kWaves * bt * hd;
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
