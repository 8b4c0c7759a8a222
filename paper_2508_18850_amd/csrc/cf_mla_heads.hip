// Fused MLA decode step (paper Appendix B, Alg. 4) with the HEAD as the unit of work, the way Alg. 4 assigns a cluster
// to a head: 16 co-resident workgroups per head, every member scans 1/16 of the cached rows for its head with vector
// arithmetic.  Every head reads every cached row, which the last-level cache absorbs at batch 1 and 2; from batch 3
// on the kernel of cf_mla.hip (token ranges as the unit of work, MFMA tiles over all heads) is the faster one, and
// cf_mla_decode picks between the two.  Same exchange through stamped slots, same stages:
//
//   A  projections        [q | kv_new] = x [W_Q | W_KV]           16 row slices x 16 column blocks, partial sums
//   B  up-projection      q_lat_i = q_nope_i W_Up[i]              member j: 1/16 of the kv_lora_rank columns
//   C  attention          partial softmax over 1/16 of the tokens  (m, l, acc[kv_lora_rank]) per member;
//                         the last member appends the new row and counts the new token
//   D  merge + down-proj. member j merges 1/16 of the latent dimensions of the 16 partials and multiplies them
//                         by the same rows of W_Down[i]: a partial of a_i per member (summed by the reader)
//   E1 output projection  rows of W_O of head i, 1/16 of the output columns per member: a partial of out per head
//   E2 sum over heads     every workgroup: 1/W of the output columns (the paper's atomicAdd)
//
// Each stage requests its weights before it waits for its input.  All waits are bounded (CF_ETIMEOUT), all
// workgroups have to be resident at once.
#include "cf_mla_internal.h"
#include "cf_rope_device.h"
#include "cf_team_device.h"

namespace {

using cf::team::Exchange;
using cf::team::pair_t;
constexpr int NT = 512;             // threads per workgroup
constexpr int NW = NT / 64;
constexpr int TS = 16;              // workgroups per head (team)
constexpr int KS = 16;              // row slices of the projections
constexpr int L = 512;              // kv_lora_rank the lane mapping is written for: 16 lanes x 32 values per cached row
constexpr int R = 64;               // rope_dim: 16 lanes x 4 values
constexpr int MAXB = 4;             // largest batch
constexpr int MAXCOLS = 256;        // projection columns per column block
constexpr int MAXA = 2048;          // floats of the largest stage buffer per batch row
constexpr int kCounterStride = 16;
constexpr int NPART = NW * 4;       // attention partials of a workgroup: four row groups per wavefront
constexpr size_t kDynLds = (size_t)NPART * (L + 2) * sizeof(float);
constexpr float kNegBig = -1.0e30f;

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));


__device__ __forceinline__ float h2f(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t f2h(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the wavefront, the same value in every lane: four data-parallel-primitive steps inside each row of
// 16 lanes, then the four row totals are read out as scalars (no trip through the LDS crossbar).
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror
    const int i = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
    return (r0 + r1) + (r2 + r3);
}

// Sum of the n stamped values at idx, idx + stride, ... (in that order); polls go out sixteen at a time (the
// teams and the row slices have 16 members: one round trip).
__device__ __forceinline__ float take_sum(const Exchange &x, __amdgpu_buffer_rsrc_t r, size_t idx, size_t stride, int n)
{
    constexpr int NP = 16;
    float s = 0.f;
    for (int k0 = 0; k0 < n; k0 += NP) {
        pair_t q[NP];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < NP; ++k) q[k] = cf::team::peek(r, idx + (size_t)min(k0 + k, n - 1) * stride);
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < NP; ++k) ok &= q[k].y == x.stamp;
            if (ok || cf::team::gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < NP; ++k)
            if (k0 + k < n) s += __builtin_bit_cast(float, q[k].x);
    }
    return s;
}

// The stamped value at idx (one poll per try).
__device__ __forceinline__ float take1(const Exchange &x, __amdgpu_buffer_rsrc_t r, size_t idx)
{
    long long t0 = 0;
    for (;;) {
        const pair_t q = cf::team::peek(r, idx);
        if (q.y == x.stamp) return __builtin_bit_cast(float, q.x);
        if (cf::team::gave_up(x, t0)) return 0.f;
    }
}

// Workgroup barrier that orders LDS accesses only (__syncthreads() would also wait until the write-through stores of
// the last hand-over have reached memory); nothing here passes data between the threads of a workgroup through
// global memory.
__device__ __forceinline__ void lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#define MLA_STAMP(k)

__global__ void __launch_bounds__(NT) fused_mla_heads(const cf::mla::HeadsArgs a)
{
    __shared__ float s_a[MAXB * MAXA];                  // stage buffers, reused from stage to stage
    __shared__ float s_b[MAXB * (L + R)];
    __shared__ float s_red[NW * (L + 2)];
    extern __shared__ __align__(16) float s_part[];                  // [NPART][L + 2] attention partials of the row groups (dynamic)
    __shared__ float s_small[R + MAXB];                 // cos, sin of the rotary angles; score of the new token per row
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, w = blockIdx.x;
    const int head = w / TS, j = w % TS;
    const int B = a.B, nr = a.n + R, CQq = a.nh * nr, CQ = CQq + L + R;
    MLA_STAMP(0);

    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)w * kCounterStride)
                 : "memory");
    const unsigned long long cnt = launches + 1ull;
    const Exchange x = {a.slots, 0, (uint32_t)(cnt + (cnt >> 32)), a.err, a.spin_ticks};
    const __amdgpu_buffer_rsrc_t r = cf::team::slots_rsrc(x);

    // ---- A: partial projections.  Work item (kb, cb): rows [kb*RK, +RK) of x, column block cb of W_Q and of W_KV.
    //      A thread owns one 16-byte piece (8 columns) of the block and every 16th row of the slice: lanes run
    //      along the columns, so a row of the block is one contiguous read; the two row groups of a wavefront
    //      are added by a shuffle, the eight wavefronts through LDS.
    const int RK = a.D / KS;
    const int qv = CQq / 8, kvv = (L + R) / 8;                        // 16-byte pieces of a row of W_Q / W_KV
    for (int item = w; item < KS * 16; item += a.W) {
        const int kb = item / 16, cb = item % 16;
        const int pv = tid % 32, g = tid / 32;                        // piece of the block, row group 0..15
        const bool isq = pv < a.cq;
        const int piece = isq ? cb * a.cq + pv : cb * a.ckv + (pv - a.cq);
        const bool live = pv < a.cq + a.ckv && piece < (isq ? qv : kvv);
        const h8 *wp = reinterpret_cast<const h8 *>(isq ? a.wq : a.wkv) + piece;
        const size_t ld = isq ? qv : kvv;                             // row stride in pieces
        float acc[MAXB][8];
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[b][c] = 0.f;
        h8 wr[8];                                                      // eight rows of this thread in flight
        auto request = [&](int r0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int rr = r0 + 16 * k;
                wr[k] = (live && rr < RK) ? wp[(size_t)(kb * RK + rr) * ld] : h8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        };
        request(g);                                                    // the first weights go out before the slice of x
        lds_sync();                                                    // (all threads, whatever their row group)
        for (int i = tid; i < B * RK; i += NT) s_b[i] = h2f(a.x[(size_t)(i / RK) * a.D + kb * RK + i % RK]);
        lds_sync();
        for (int r0 = g; r0 < RK; r0 += 16 * 8) {
            if (r0 != g) request(r0);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int rr = min(r0 + 16 * k, RK - 1);
#pragma unroll
                for (int b = 0; b < MAXB; ++b) {
                    const float xv = b < B ? s_b[b * RK + rr] : 0.f;
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[b][c] = fmaf(xv, (float)wr[k][c], acc[b][c]);
                }
            }
        }
        // (all shuffles of a row first, then the stores: a store between two shuffles makes each one wait for the last)
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
            if (b < B) {
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[b][c] += __shfl_xor(acc[b][c], 32);
                if (lane < 32) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) s_a[(wv * MAXB + b) * MAXCOLS + pv * 8 + c] = acc[b][c];
                }
            }
        lds_sync();
        for (int i = tid; i < B * MAXCOLS; i += NT) {
            const int b = i / MAXCOLS, cc = i % MAXCOLS, p2 = cc / 8;
            const bool q2 = p2 < a.cq;
            const int piece2 = q2 ? cb * a.cq + p2 : cb * a.ckv + (p2 - a.cq);
            if (p2 < a.cq + a.ckv && piece2 < (q2 ? qv : kvv)) {
                float sum = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < NW; ++w8) sum += s_a[(w8 * MAXB + b) * MAXCOLS + cc];
                const int gcol = (q2 ? 0 : CQq) + piece2 * 8 + cc % 8;
                cf::team::put(r, a.x1 + ((size_t)kb * B + b) * CQ + gcol, sum, x.stamp);
            }
        }
    }

    MLA_STAMP(1);           // A done
    // ---- B: up-projection of head `head`, columns [LJ*j, +LJ) of the latent dimension
    constexpr int LJ = L / TS;                                        // 32
    // (the weights of a stage do not depend on what the stage waits for: they are requested first)
    const int pcB = tid % 4, rowB = tid / 4;                          // nope_dim <= 128: one (row, piece) per thread
    const h8 wupr = rowB < a.n ? *reinterpret_cast<const h8 *>(a.wup + ((size_t)head * a.n + rowB) * L + LJ * j + pcB * 8)
                               : h8{0, 0, 0, 0, 0, 0, 0, 0};
    lds_sync();
    for (int i = tid; i < B * a.n; i += NT) {
        const int b = i / a.n, c = i % a.n;
        s_a[i] = take_sum(x, r, a.x1 + (size_t)b * CQ + head * nr + c, (size_t)B * CQ, KS);
    }
    lds_sync();
    MLA_STAMP(2);           // q_nope arrived
    {
        // W_Up[head] rows x this member's 32 columns: four 16-byte pieces per row; lanes with the same piece are
        // added by shuffles, the wavefronts through LDS
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
            if (b < B) {
                const float qv2 = rowB < a.n ? s_a[b * a.n + rowB] : 0.f;
                float t[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) t[c] = qv2 * (float)wupr[c];
#pragma unroll
                for (int off = 4; off < 64; off <<= 1)
#pragma unroll
                    for (int c = 0; c < 8; ++c) t[c] += __shfl_xor(t[c], off);
                if (lane < 4) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) s_b[(wv * MAXB + b) * LJ + pcB * 8 + c] = t[c];
                }
            }
        lds_sync();
        if (tid < LJ * B) {
            const int b = tid / LJ, cc = tid % LJ;
            float sum = 0.f;
            for (int w8 = 0; w8 < NW; ++w8) sum += s_b[(w8 * MAXB + b) * LJ + cc];
            cf::team::put(r, a.x2 + ((size_t)b * a.nh + head) * L + LJ * j + cc, sum, x.stamp);
        }
    }

    MLA_STAMP(3);           // B done
    // ---- C: attention over the tokens [t0, t1) of this member; the last member also takes the new token
    lds_sync();
    const bool last = j == TS - 1;
    const int tps = (a.pos + TS - 1) / TS;
    const int t0 = min(j * tps, a.pos), t1 = min(t0 + tps, a.pos);
    // s_a: [B][L + R] the query in the latent space and its rotated rotary part; s_b: [B][L + R] the new row.
    // First what has been there since stage A (the rotary part of the query, the new row) and the angles, last the
    // latent query, which the other members of the team are still producing.
    if (tid < R / 2) {
        const double inv_freq = exp2(-2.0 * (double)tid / (double)R * a.log2_base);
        cf::rope_cos_sin(a.pos, inv_freq, s_small[tid], s_small[R / 2 + tid]);
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
    for (int i = tid; i < B * L; i += NT) {
        const int b = i / L, d = i % L;
        s_a[b * (L + R) + d] = take1(x, r, a.x2 + ((size_t)b * a.nh + head) * L + d);
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
    MLA_STAMP(4);           // query arrived and rotated
    if (j == 0)                                                       // for cf_mla_debug_export: (q_lat | q_rope) of this head
        for (int i = tid; i < B * (L + R); i += NT)
            a.qdbg[((size_t)(i / (L + R)) * a.nh + head) * (L + R) + i % (L + R)] = s_a[i];
    if (last)                                                         // append (Sec. 2.1): row pos of every sequence
        for (int i = tid; i < B * (L + R); i += NT) {
            const int b = i / (L + R), d = i % (L + R);
            a.cache[((size_t)b * a.max_seq + a.pos) * (L + R) + d] = f2h(s_b[i]);
        }
    for (int b = 0; b < B; ++b) {
        const float *q = s_a + b * (L + R);
        // A row of the cache is handled by 16 lanes (a wavefront takes four rows at a time): lane li of a row group
        // owns the latent dimensions 128 k + 8 li .. + 8 (k < 4) and the rotary dimensions 4 li .. + 4, so a row's
        // score needs only the four in-row steps of a cross-lane sum and one exponential serves 36 multiply-adds.
        const int li = lane & 15, rg = lane >> 4;
        float ql[4][8], qr4[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int c = 0; c < 8; ++c) ql[k][c] = q[128 * k + 8 * li + c] * a.scale_log2e;
#pragma unroll
        for (int c = 0; c < 4; ++c) qr4[c] = q[L + 4 * li + c] * a.scale_log2e;
        float m = kNegBig, lsum = 0.f, acc[4][8];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[k][c] = 0.f;
        const uint16_t *rows = a.cache + (size_t)b * a.max_seq * (L + R);
        // Two rows per row group and batch, two batches in flight.  Rows past the split are read from its last row
        // (finite data) and count for nothing.
        constexpr int UR = 4, RPB = NW * 4;                            // rows of the workgroup per sub-batch
        h8 kl[2][UR][4];
        h4 kr[2][UR];
        const int myrow = wv * 4 + rg;
        auto request = [&](int buf, int t) {
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const uint16_t *row = rows + (size_t)min(t + myrow + u * RPB, t1 - 1) * (L + R);
#pragma unroll
                for (int k = 0; k < 4; ++k) kl[buf][u][k] = *reinterpret_cast<const h8 *>(row + 128 * k + 8 * li);
                kr[buf][u] = *reinterpret_cast<const h4 *>(row + L + 4 * li);
            }
        };
        auto use = [&](int buf, int t) {
            float d[UR];
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                float dd = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < 8; ++c) dd = fmaf(ql[k][c], (float)kl[buf][u][k][c], dd);
#pragma unroll
                for (int c = 0; c < 4; ++c) dd = fmaf(qr4[c], (float)kr[buf][u][c], dd);
                d[u] = dd;
            }
#pragma unroll
            for (int u = 0; u < UR; ++u) {                             // sum over the 16 lanes of the row
                d[u] += dpp_move<0xB1>(d[u]);
                d[u] += dpp_move<0x4E>(d[u]);
                d[u] += dpp_move<0x141>(d[u]);
                d[u] += dpp_move<0x140>(d[u]);
            }
            float mn = m;
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                d[u] = (t + myrow + u * RPB < t1) ? d[u] : kNegBig;
                mn = fmaxf(mn, d[u]);
            }
            const float f = __builtin_amdgcn_exp2f(m - mn);
            m = mn;
            lsum *= f;
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[k][c] *= f;
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                const float pw = (t + myrow + u * RPB < t1) ? __builtin_amdgcn_exp2f(d[u] - mn) : 0.f;
                lsum += pw;
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[k][c] = fmaf(pw, (float)kl[buf][u][k][c], acc[k][c]);
            }
        };
        if (t1 > t0) {                                                 // uniform over the workgroup
            constexpr int step = RPB * UR;
            request(0, t0);
            for (int t = t0; t < t1; t += 2 * step) {
                request(1, t + step);
                use(0, t);
                request(0, t + 2 * step);
                use(1, t + step);
            }
        }
        MLA_STAMP(11);          // rows consumed
        // every row group of every wavefront leaves its (m, l, acc) in LDS: 32 partials, folded below
        lds_sync();
        {
            float *part = s_part + (wv * 4 + rg) * (L + 2);
            if (li == 0) {
                part[0] = m;
                part[1] = lsum;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int c = 0; c < 8; ++c) part[2 + 128 * k + 8 * li + c] = acc[k][c];
        }
        MLA_STAMP(12);          // row groups merged
        if (last && wv == 0) {                                        // score of the new token (its row is not rounded)
            const float *kn = s_b + b * (L + R);
            float d = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int c = 0; c < 8; ++c) d = fmaf(ql[k][c], kn[128 * k + 8 * li + c], d);
#pragma unroll
            for (int c = 0; c < 4; ++c) d = fmaf(qr4[c], kn[L + 4 * li + c], d);
            d += dpp_move<0xB1>(d);
            d += dpp_move<0x4E>(d);
            d += dpp_move<0x141>(d);
            d += dpp_move<0x140>(d);
            if (lane == 0) s_small[R + b] = d;
        }
        lds_sync();
        {
            const int d = tid;                                         // one latent dimension per thread
            // lane w8 of every wavefront takes the maximum and the sum of partial w8; the factors then reach the
            // threads as scalars (one exponential per lane in place of one per thread and partial)
            static_assert(NPART <= 64, "one lane per partial");
            const float pm = lane < NPART ? s_part[lane * (L + 2)] : kNegBig;
            const float pl = lane < NPART ? s_part[lane * (L + 2) + 1] : 0.f;
            float M = pm;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
            if (last) M = fmaxf(M, s_small[R + b]);
            const float fw = __builtin_amdgcn_exp2f(pm - M);           // (0 for the lanes past the partials)
            float Ls = wave_sum(pl * fw), A = 0.f;
#pragma unroll
            for (int w8 = 0; w8 < NPART; ++w8) {
                const float f = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, fw), w8));
                A = fmaf(s_part[w8 * (L + 2) + 2 + d], f, A);
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

    MLA_STAMP(5);           // C done
    // ---- D: merge latent dimensions [LJ*j, +LJ) of the team's partials (online softmax, Alg. 4 steps 8-10) and
    //      multiply them by the same rows of W_Down[head]: a partial of a_head per member, no hop in between
    const int pcsD = a.v / 8, pcD = tid % 16, rowD = tid / 16;        // thread = (row of the slice, 16-byte piece)
    const h8 wdr = pcD < pcsD ? *reinterpret_cast<const h8 *>(a.wdown + ((size_t)head * L + LJ * j + rowD) * a.v + pcD * 8)
                              : h8{0, 0, 0, 0, 0, 0, 0, 0};
    lds_sync();
    if (tid < LJ * B) {
        const int b = tid / LJ, d = LJ * j + tid % LJ;
        const size_t src = a.x3 + ((size_t)b * a.nh + head) * TS * (L + 2);
        pair_t qm[TS], ql2[TS], qa[TS];
        long long tw = 0;
        for (;;) {                                                     // all 48 polls of this thread in one go
#pragma unroll
            for (int s2 = 0; s2 < TS; ++s2) {
                qm[s2] = cf::team::peek(r, src + (size_t)s2 * (L + 2));
                ql2[s2] = cf::team::peek(r, src + (size_t)s2 * (L + 2) + 1);
                qa[s2] = cf::team::peek(r, src + (size_t)s2 * (L + 2) + 2 + d);
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int s2 = 0; s2 < TS; ++s2) ok &= (qm[s2].y == x.stamp) & (ql2[s2].y == x.stamp) & (qa[s2].y == x.stamp);
            if (ok || cf::team::gave_up(x, tw)) break;
        }
        float M = kNegBig;
#pragma unroll
        for (int s2 = 0; s2 < TS; ++s2) M = fmaxf(M, __builtin_bit_cast(float, qm[s2].x));
        float Ls = 0.f, A = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < TS; ++s2) {
            const float f = __builtin_amdgcn_exp2f(__builtin_bit_cast(float, qm[s2].x) - M);
            Ls = fmaf(__builtin_bit_cast(float, ql2[s2].x), f, Ls);
            A = fmaf(__builtin_bit_cast(float, qa[s2].x), f, A);
        }
        s_b[b * LJ + tid % LJ] = A / Ls;                               // z[b][LJ*j + ...]
        a.zdbg[((size_t)b * a.nh + head) * L + d] = A / Ls;
    }
    lds_sync();
    MLA_STAMP(6);           // z slice merged
    {
        // rows [LJ*j, +LJ) of W_Down[head], all v columns: one contiguous block (requested above)
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
            if (b < B) {
                const float zv = s_b[b * LJ + rowD];
                float t[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) t[c] = zv * (float)wdr[c];
#pragma unroll
                for (int c = 0; c < 8; ++c) t[c] += __shfl_xor(t[c], 16);
#pragma unroll
                for (int c = 0; c < 8; ++c) t[c] += __shfl_xor(t[c], 32);
                if (lane < 16) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) s_red[(wv * MAXB + b) * 128 + pcD * 8 + c] = t[c];
                }
            }
        lds_sync();
        for (int i = tid; i < B * a.v; i += NT) {
            const int b = i / a.v, c = i % a.v;
            float sum = 0.f;
#pragma unroll
            for (int w8 = 0; w8 < NW; ++w8) sum += s_red[(w8 * MAXB + b) * 128 + c];
            cf::team::put(r, a.x5 + (((size_t)b * a.nh + head) * TS + j) * a.v + c, sum, x.stamp);
        }
    }
    MLA_STAMP(7);           // D done

    // ---- E1: rows of W_O that belong to this head, column block j of the output: a partial of out per head
    const int dpE = a.D / 8, pcsE = (dpE + TS - 1) / TS;                // 16-byte pieces of an output row; per member
    const int pcE = tid % 16, rgE = tid / 16;                         // 32 row groups
    auto wo_rows = [&](int p0, h8 (&wr)[4]) {                          // v <= 128: at most four rows per thread
        const int piece = j * pcsE + p0 + pcE;
        const bool live = p0 + pcE < pcsE && piece < dpE;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = rgE + 32 * k;
            wr[k] = (live && row < a.v) ? *reinterpret_cast<const h8 *>(a.wo + ((size_t)head * a.v + row) * a.D + piece * 8)
                                        : h8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    };
    h8 wor[4];
    wo_rows(0, wor);
    lds_sync();
    for (int i = tid; i < B * a.v; i += NT) {
        const int b = i / a.v, c = i % a.v;
        s_b[i] = take_sum(x, r, a.x5 + ((size_t)b * a.nh + head) * TS * a.v + c, (size_t)a.v, TS);
    }
    lds_sync();
    MLA_STAMP(8);           // a_head arrived
    for (int p0 = 0; p0 < pcsE; p0 += 16) {
        if (p0 > 0) wo_rows(p0, wor);
        float acc[MAXB][8];
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[b][c] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = min(rgE + 32 * k, a.v - 1);
#pragma unroll
            for (int b = 0; b < MAXB; ++b)
                if (b < B) {
                    const float av = s_b[b * a.v + row];
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[b][c] = fmaf(av, (float)wor[k][c], acc[b][c]);
                }
        }
        lds_sync();
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
            if (b < B) {
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[b][c] += __shfl_xor(acc[b][c], 16);
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[b][c] += __shfl_xor(acc[b][c], 32);
                if (lane < 16) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) s_red[(wv * MAXB + b) * 128 + pcE * 8 + c] = acc[b][c];
                }
            }
        lds_sync();
        for (int i = tid; i < B * 128; i += NT) {
            const int b = i / 128, cc = i % 128, piece2 = j * pcsE + p0 + cc / 8;
            if (p0 + cc / 8 < pcsE && piece2 < dpE) {
                float sum = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < NW; ++w8) sum += s_red[(w8 * MAXB + b) * 128 + cc];
                cf::team::put(r, a.x6 + ((size_t)b * a.nh + head) * a.D + piece2 * 8 + cc % 8, sum, x.stamp);
            }
        }
    }
    MLA_STAMP(10);          // E1 done

    // ---- E2: sum over the heads (what the paper does with atomicAdd), columns [CW*w, +CW) of the output
    {
        const int CW = (a.D + a.W - 1) / a.W;
        if (tid < B * CW) {
            const int b = tid / CW, col = CW * w + tid % CW;
            if (col < a.D)
                a.out[(size_t)b * a.D + col] = f2h(take_sum(x, r, a.x6 + (size_t)b * a.nh * a.D + col, (size_t)a.D, a.nh));
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
    MLA_STAMP(9);
}


}  // namespace

namespace cf {
namespace mla {

size_t heads_layout(const cf_mla_config &c, int B, size_t (&first)[5])
{
    const size_t CQ = (size_t)c.n_heads * (c.nope_dim + R) + L + R;
    first[0] = 0;
    first[1] = first[0] + (size_t)KS * B * CQ;
    first[2] = first[1] + (size_t)B * c.n_heads * L;
    first[3] = first[2] + (size_t)B * c.n_heads * TS * (L + 2);
    first[4] = first[3] + (size_t)B * c.n_heads * TS * c.v_head_dim;
    return first[4] + (size_t)B * c.n_heads * c.d_model;
}

bool heads_prepare()
{
    int per_cu = 0;
    const void *fn = reinterpret_cast<const void *>(fused_mla_heads);
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDynLds) == hipSuccess &&
           hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, NT, kDynLds) == hipSuccess && per_cu >= 1;
}

int heads_launch(const HeadsArgs &a, void *stream)
{
    hipLaunchKernelGGL(fused_mla_heads, dim3(a.W), dim3(NT), kDynLds, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

}  // namespace mla
}  // namespace cf
