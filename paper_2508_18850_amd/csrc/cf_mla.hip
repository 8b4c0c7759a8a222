// Fused decode step of a weight-absorbed Multi-Head Latent Attention block (paper Appendix B, Alg. 4) as ONE
// kernel for gfx950, behind the C ABI (cf_mla_* in include/cfdecode.h).
//
// Alg. 4 runs one cluster per head and moves data between its blocks with three ClusterGathers and three
// ClusterReduces.  Here 16 co-resident workgroups per head share the weights of that head, every hand-over is one
// hop through stamped {value, stamp} slots in global memory (cf_team_device.h), five hops in all, and every weight
// matrix is read in contiguous rows:
//
//   A  projections        [q | kv_new] = x [W_Q | W_KV]           16 row slices x 16 column blocks, partial sums
//   B  up-projection      q_lat_i = q_nope_i W_Up[i]              member j: 1/16 of the kv_lora_rank columns; the same
//                         workgroups finish q_rope_i and the new cache row (sum of the partials, RoPE, append)
//   C  attention          unit of work = (batch row, token range), NOT the head: all heads share every cached row
//                         (one latent "head": MQA), so the scores and the weighted sums of the 16 heads against a tile
//                         of 128 rows are two dense products on MFMA tiles; a row is read from HBM once for all heads
//   D  merge + down-proj. (head i, member j): merges 1/16 of the latent dimensions of the range partials (Alg. 4's
//                         online-softmax reduction) and multiplies them by the same rows of W_Down[i]
//   E1 output projection  rows of W_O of head i, 1/16 of the output columns per member: a partial of out per head
//   E2 sum over heads     every workgroup: 1/W of the output columns (the paper's atomicAdd)
//
// Each stage requests its weights (or cached rows) before it waits for its input.  All waits are bounded
// (CF_ETIMEOUT), all workgroups have to be resident at once.
#include "cf_mfma_device.h"
#include "cf_mla_internal.h"
#include "cf_rope_device.h"
#include "cf_team_device.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace {

using cf::team::Exchange;
using cf::team::pair_t;
constexpr int NT = 512;             // threads per workgroup
constexpr int NW = NT / 64;
constexpr int TS = 16;              // workgroups per head (team)
constexpr int KS = 16;              // row slices of the projections
constexpr int L = 512;              // kv_lora_rank the lane mapping is written for
constexpr int R = 64;               // rope_dim
constexpr int LR = L + R;
constexpr int HT = 16;              // heads of one MFMA tile: the most the kernel takes
constexpr int MAXBATCH = 16;
constexpr int MAXCOLS = 256;        // projection columns per column block
constexpr int kCounterStride = 16;
constexpr int kTile = 64;           // cached rows per attention tile of a workgroup (held in LDS)
constexpr int KSTR = LR + 8;        // row stride (fp16 values) of the tile in LDS
constexpr int kSteps = LR / 32;     // MFMA steps of a score product (contraction over 576 dimensions)
constexpr int kQops = kSteps * 64;  // 16-byte query operands (one per step and lane)
constexpr int PS = kTile + 8;       // row stride (fp16 values) of the probabilities in LDS
constexpr int QS = LR + 8;          // row stride (floats) of the fp32 query in LDS
constexpr int kPart = 2 + L;        // slots of an attention partial per head: m, l, acc[L]
constexpr int kMaxSplits = 32;      // token ranges per batch row at most
constexpr size_t kLdsFloats = 29440;    // 115 KiB: the largest stage (C: query operands, a tile of rows, the rest)
constexpr float kNegBig = -1.0e30f;
constexpr int kHeadsBatch = 1;      // up to this batch cf_mla_decode runs the head-team kernel (measured cross-over)

using cf::mfma::f32x4;
using cf::mfma::h8;
using cf::mfma::mfma16;
using cf::mfma::transpose8;
using cf::mfma::u32x4;
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

struct MlaArgs {
    const uint16_t *x, *wq, *wkv, *wup, *wdown, *wo;
    uint16_t *cache, *out;
    float *zdbg;                    // [B][nh][L]: the normalised latent vectors z of the call (for cf_mla_debug_export)
    uint64_t *slots;
    unsigned long long *counters;
    uint32_t *err;
    size_t x1, xq, xkv, x3, xs, x5, x6, xqn, xa;     // first slot of each exchange area
    int D, nh, n, v, B, pos, max_seq, W;
    int NS, tps, HG;                // token ranges per batch row, cached rows per range, heads per attention item
    int cq, ckv;                    // 16-byte pieces (8 columns) of W_Q / W_KV per column block
    float scale_log2e;              // log2(e) / sqrt(nope_dim + rope_dim)
    double log2_base;
    long long spin_ticks;
};

__device__ __forceinline__ float h2f(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t f2h(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// Sums of NV sets of n <= 16 stamped values each: set v is idx[v], idx[v] + stride, ... (added in that order).
// All NV * 16 polls are in flight together: one round trip when the values are there.
template <int NV>
__device__ __forceinline__ void take_sums(const Exchange &x, __amdgpu_buffer_rsrc_t r, const size_t (&idx)[NV], size_t stride,
                                          int n, float (&out)[NV])
{
    constexpr int NP = 16;
    pair_t q[NV][NP];
    long long t0 = 0;
    for (;;) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int k = 0; k < NP; ++k) q[v][k] = cf::team::peek(r, idx[v] + (size_t)min(k, n - 1) * stride);
        __builtin_amdgcn_sched_barrier(0);
        bool ok = true;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int k = 0; k < NP; ++k) ok &= q[v][k].y == x.stamp;
        if (ok || cf::team::gave_up(x, t0)) break;
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NP; ++k)
            if (k < n) s += __builtin_bit_cast(float, q[v][k].x);
        out[v] = s;
    }
}

// All threads: fetch cnt <= 4 * NT stamped values into LDS, value i (at slot_of(i)) to dst[i]; all polls of a thread are
// in flight together (one round trip).  No barrier inside.
template <class SlotOf>
__device__ __forceinline__ void fetch4(const Exchange &x, __amdgpu_buffer_rsrc_t r, int cnt, float *dst, SlotOf &&slot_of)
{
    pair_t q[4];
    long long t0 = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            q[k] = pair_t{0u, x.stamp};
            if (NT * k < cnt) q[k] = cf::team::peek(r, slot_of(min((int)threadIdx.x + NT * k, cnt - 1)));     // (uniform)
        }
        __builtin_amdgcn_sched_barrier(0);
        bool ok = true;
#pragma unroll
        for (int k = 0; k < 4; ++k) ok &= q[k].y == x.stamp;
        if (ok || cf::team::gave_up(x, t0)) break;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if ((int)threadIdx.x + NT * k < cnt) dst[threadIdx.x + NT * k] = __builtin_bit_cast(float, q[k].x);
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() would also wait for every outstanding global
// access of the wavefront (vmcnt(0)): for the write-through stores of the last hand-over to reach memory and for the
// loads a stage keeps in flight across it.  Nothing here passes data between the threads of a workgroup through
// global memory.
__device__ __forceinline__ void lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Product of the B rows of `in` (LDS, row b at in + b * ld_in, nrows values each) with a [nrows x PCS * 8] block of
// fp16 weights that the threads hold in registers: thread (piece pc = tid % PCS, batch quad bq, row group rg) has
// rows rg, rg + RG, ... of piece pc in wr[].  The partial sums of the row groups are added inside the wavefront by
// shuffles and across wavefronts through s_red ([NW][BT][PCS * 8] floats); sink(b, column, sum) gets the result.
// All threads of the workgroup call; contains barriers.
template <int BT, int PCS, int RPT, class Sink>
__device__ __forceinline__ void small_product(const h8 (&wr)[RPT], const float *in, int ld_in, int nrows, int B, float *s_red,
                                              Sink &&sink)
{
    constexpr int BQ = BT / 4, G = PCS * BQ, RG = NT / G;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int pc = tid % PCS, bq = (tid / PCS) % BQ, rg = tid / G;
    float acc[4][8];
#pragma unroll
    for (int bb = 0; bb < 4; ++bb)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[bb][c] = 0.f;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        const int row = min(rg + RG * k, nrows - 1);                 // rows past the block carry zero weights
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            const float xin = in[min(4 * bq + bb, B - 1) * ld_in + row];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[bb][c] = fmaf(xin, (float)wr[k][c], acc[bb][c]);
        }
    }
#pragma unroll
    for (int bb = 0; bb < 4; ++bb)
        if (BT > 4 || bb < B) {                                       // (BT == 4: the same for all threads)
#pragma unroll
            for (int off = G; off < 64; off <<= 1)
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[bb][c] += __shfl_xor(acc[bb][c], off);
            if (lane < G) {
#pragma unroll
                for (int c = 0; c < 8; ++c) s_red[(wv * BT + 4 * bq + bb) * (PCS * 8) + pc * 8 + c] = acc[bb][c];
            }
        }
    lds_sync();
    for (int i = tid; i < B * PCS * 8; i += NT) {
        const int b = i / (PCS * 8), cc = i % (PCS * 8);
        float sum = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < NW; ++w8) sum += s_red[(w8 * BT + b) * (PCS * 8) + cc];
        sink(b, cc, sum);
    }
}

// Dimension of a cached row that contraction slot (step m, lane group g, element 0) of a score product stands for:
// a lane reads 32 contiguous bytes of the row in two steps, the four groups of a token one 128-byte line.
__device__ __forceinline__ int score_dim(int m, int g) { return 64 * (m >> 1) + 16 * g + 8 * (m & 1); }

// Stage time stamps of every workgroup, only in builds with -DCF_STAMPS=1 (the profiling library).
#ifndef CF_STAMPS
#define CF_STAMPS 0
#endif
#if CF_STAMPS
constexpr int kMlaStamps = 16;
__device__ unsigned long long g_mla_ts[256 * kMlaStamps];
#define MLA_STAMP(k) do { if (threadIdx.x == 0) s_ts[k] = wall_clock64(); } while (0)
#else
#define MLA_STAMP(k)
#endif

// BT: batch rows the register tiles are written for (4 or 16)
template <int BT>
__global__ void __launch_bounds__(NT) fused_mla_decode(const MlaArgs a)
{
    constexpr int BQ = BT / 4;
    extern __shared__ __align__(16) float smem[];                    // carved anew by every stage
    __shared__ float s_rope[R];                         // cos, sin of the rotary angles
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, w = blockIdx.x;
    const int head = w / TS, j = w % TS;
    const int B = a.B, nr = a.n + R, CQq = a.nh * nr, CQ = CQq + LR;
#if CF_STAMPS
    __shared__ unsigned long long s_ts[kMlaStamps];
    if (tid < kMlaStamps) s_ts[tid] = 0;
#endif
    MLA_STAMP(0);

    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)w * kCounterStride)
                 : "memory");
    const unsigned long long cnt = launches + 1ull;
    const Exchange x = {a.slots, 0, (uint32_t)(cnt + (cnt >> 32)), a.err, a.spin_ticks};
    const __amdgpu_buffer_rsrc_t r = cf::team::slots_rsrc(x);
    if (tid < R / 2) {
        const double inv_freq = exp2(-2.0 * (double)tid / (double)R * a.log2_base);
        cf::rope_cos_sin(a.pos, inv_freq, s_rope[tid], s_rope[R / 2 + tid]);
    }

    constexpr int LJ = L / TS;                                         // latent dimensions per member: 32
    constexpr int RPT_B = (128 * 4 * BQ + NT - 1) / NT;                // rows per thread: W_Up (nope_dim <= 128),
    constexpr int RPT_D = (LJ * 16 * BQ + NT - 1) / NT;                //   W_Down slice (LJ rows),
    constexpr int RPT_E = (128 * 16 * BQ + NT - 1) / NT;               //   W_O (v_head_dim <= 128 rows)
    constexpr int G4 = 4 * BQ, RG4 = NT / G4, G16 = 16 * BQ, RG16 = NT / G16;

    // ---- A: partial projections.  Work item (kb, cb): rows [kb*RK, +RK) of x, column block cb of W_Q and of W_KV.
    //      A thread owns one 16-byte piece (8 columns) of the block and every 16th row of the slice: lanes run
    //      along the columns, so a row of the block is one contiguous read; the two row groups of a wavefront
    //      are added by a shuffle, the eight wavefronts through LDS (eight batch rows at a time).
    {
        constexpr int RB = BT < 8 ? BT : 8;
        float *s_x = smem;                                             // [BT][RK], RK <= 512
        float *s_red = smem + BT * 512;                                // [NW][RB][MAXCOLS]; 16-row tile: [4][BT][MAXCOLS]
        const int RK = a.D / KS;
        const int qv = CQq / 8, kvv = LR / 8;                          // 16-byte pieces of a row of W_Q / W_KV
        for (int item = w; item < KS * 16; item += a.W) {
            const int kb = item / 16, cb = item % 16;
            if constexpr (BT == 16) {
                // Matrix cores: one 16 x 16 x 32 step per 32 rows of the slice and eight columns: A = x (batch rows by
                // slice rows, fp16 as given), B = eight rows of a 16-byte piece of the weights, transposed inside
                // the lane; fp32 accumulation.  Wavefront wv takes the pieces [16 (wv & 1), +16) of the block and the
                // steps wv / 2, wv / 2 + 4, ...; the four wavefronts of a piece set are added through LDS.
                const int g = lane >> 4, c = lane & 15, pv = 16 * (wv & 1) + c, sw = wv >> 1;
                const bool isq = pv < a.cq;
                const int piece = isq ? cb * a.cq + pv : cb * a.ckv + (pv - a.cq);
                const bool live = pv < a.cq + a.ckv && piece < (isq ? qv : kvv);
                const h8 *wp = reinterpret_cast<const h8 *>(isq ? a.wq : a.wkv) + piece;
                const size_t ld = isq ? qv : kvv;                      // row stride in pieces
                h8 wr[8];
                auto request = [&](int st) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int rr = 32 * st + 8 * g + u;
                        wr[u] = (live && rr < RK) ? wp[(size_t)(kb * RK + rr) * ld] : h8{0, 0, 0, 0, 0, 0, 0, 0};
                    }
                };
                request(sw);                                            // the first weights go out before the slice of x
                lds_sync();
                for (int i = tid; i < B * RK; i += NT) s_x[i] = h2f(a.x[(size_t)(i / RK) * a.D + kb * RK + i % RK]);
                lds_sync();
                f32x4 acc[8];                                           // [jj][rr]: batch row 4 g + rr, column 8 pv + jj
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) acc[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int st = sw; 32 * st < RK; st += 4) {
                    if (st != sw) request(st);
                    h8 xa;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int rr = 32 * st + 8 * g + i;
                        xa[i] = (c < B && rr < RK) ? (_Float16)s_x[c * RK + rr] : (_Float16)0.f;
                    }
                    h8 f8[8];
                    transpose8(wr, f8);
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj) acc[jj] = mfma16(xa, f8[jj], acc[jj]);
                }
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    float *dst = s_red + (sw * BT + 4 * g + rr) * MAXCOLS + pv * 8;
                    *reinterpret_cast<float4 *>(dst) = make_float4(acc[0][rr], acc[1][rr], acc[2][rr], acc[3][rr]);
                    *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[4][rr], acc[5][rr], acc[6][rr], acc[7][rr]);
                }
                lds_sync();
                for (int i = tid; i < BT * MAXCOLS; i += NT) {
                    const int b = i / MAXCOLS, cc = i % MAXCOLS, p2 = cc / 8;
                    const bool q2 = p2 < a.cq;
                    const int piece2 = q2 ? cb * a.cq + p2 : cb * a.ckv + (p2 - a.cq);
                    if (b < B && p2 < a.cq + a.ckv && piece2 < (q2 ? qv : kvv)) {
                        float sum = 0.f;
#pragma unroll
                        for (int k4 = 0; k4 < 4; ++k4) sum += s_red[(k4 * BT + b) * MAXCOLS + cc];
                        const int gcol = (q2 ? 0 : CQq) + piece2 * 8 + cc % 8;
                        cf::team::put(r, a.x1 + ((size_t)kb * B + b) * CQ + gcol, sum, x.stamp);
                    }
                }
                lds_sync();
            } else {
                const int pv = tid % 32, g = tid / 32;                     // piece of the block, row group 0..15
                const bool isq = pv < a.cq;
                const int piece = isq ? cb * a.cq + pv : cb * a.ckv + (pv - a.cq);
                const bool live = pv < a.cq + a.ckv && piece < (isq ? qv : kvv);
                const h8 *wp = reinterpret_cast<const h8 *>(isq ? a.wq : a.wkv) + piece;
                const size_t ld = isq ? qv : kvv;                          // row stride in pieces
                h8 wr[8];                                                   // eight rows of this thread in flight
                auto request = [&](int r0) {
    #pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int rr = r0 + 16 * k;
                        wr[k] = (live && rr < RK) ? wp[(size_t)(kb * RK + rr) * ld] : h8{0, 0, 0, 0, 0, 0, 0, 0};
                    }
                };
                request(g);                                                 // the first weights go out before the slice of x
                lds_sync();                                                 // (all threads, whatever their row group)
                for (int i = tid; i < B * RK; i += NT) s_x[i] = h2f(a.x[(size_t)(i / RK) * a.D + kb * RK + i % RK]);
                lds_sync();
                // RB batch rows per pass (the accumulators of 16 rows do not fit beside the weights); a slice of up to
                // 128 rows is one batch of loads and stays in registers over the passes
                for (int b0 = 0; b0 < B; b0 += RB) {
                    float acc[RB][8];
    #pragma unroll
                    for (int bb = 0; bb < RB; ++bb)
    #pragma unroll
                        for (int c = 0; c < 8; ++c) acc[bb][c] = 0.f;
                    for (int r0 = g; r0 < RK; r0 += 16 * 8) {
                        if (r0 != g || (b0 > 0 && RK > 16 * 8)) request(r0);
    #pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const int rr = min(r0 + 16 * k, RK - 1);
                            float wf[8];
    #pragma unroll
                            for (int c = 0; c < 8; ++c) wf[c] = (float)wr[k][c];
    #pragma unroll
                            for (int bb = 0; bb < RB; ++bb) {
                                const float xv = s_x[min(b0 + bb, B - 1) * RK + rr];
    #pragma unroll
                                for (int c = 0; c < 8; ++c) acc[bb][c] = fmaf(xv, wf[c], acc[bb][c]);
                            }
                        }
                    }
                    // (all shuffles of a row first, then the stores: a store between two shuffles makes each one wait)
    #pragma unroll
                    for (int bb = 0; bb < RB; ++bb)
                        if (b0 + bb < B) {
    #pragma unroll
                            for (int c = 0; c < 8; ++c) acc[bb][c] += __shfl_xor(acc[bb][c], 32);
                            if (lane < 32) {
    #pragma unroll
                                for (int c = 0; c < 8; ++c) s_red[(wv * RB + bb) * MAXCOLS + pv * 8 + c] = acc[bb][c];
                            }
                        }
                    lds_sync();
                    for (int i = tid; i < RB * MAXCOLS; i += NT) {
                        const int bb = i / MAXCOLS, b = b0 + bb, cc = i % MAXCOLS, p2 = cc / 8;
                        const bool q2 = p2 < a.cq;
                        const int piece2 = q2 ? cb * a.cq + p2 : cb * a.ckv + (p2 - a.cq);
                        if (b < B && p2 < a.cq + a.ckv && piece2 < (q2 ? qv : kvv)) {
                            float sum = 0.f;
    #pragma unroll
                            for (int w8 = 0; w8 < NW; ++w8) sum += s_red[(w8 * RB + bb) * MAXCOLS + cc];
                            const int gcol = (q2 ? 0 : CQq) + piece2 * 8 + cc % 8;
                            cf::team::put(r, a.x1 + ((size_t)kb * B + b) * CQ + gcol, sum, x.stamp);
                        }
                    }
                    lds_sync();
                }
            }
        }
    }

    MLA_STAMP(1);           // A done
    // ---- B: member j of head `head`: columns [LJ*j, +LJ) of the up-projection; RoPE pairs 2j, 2j + 1 of the head's
    //      rotary query; and, spread over all workgroups, the new cache row (latent dimensions w, w + W, ..., rotary
    //      pairs w, w + W, ...): sums of the KS partials, RoPE, the append (Sec. 2.1) and a copy in fp32 for stage C.
    {
        constexpr int NVB = BT == 4 ? 2 : 1;        // (16-row tile: at most 256 jobs, see J3 below)
        // (the weights do not depend on what the stage waits for: they are requested first)
        h8 wupr[RPT_B];
        {
            const int pc = tid % 4, rg = tid / G4;
#pragma unroll
            for (int k = 0; k < RPT_B; ++k) {
                const int row = rg + RG4 * k;
                wupr[k] = row < a.n ? *reinterpret_cast<const h8 *>(a.wup + ((size_t)head * a.n + row) * L + LJ * j + pc * 8)
                                    : h8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
        float *s_job = smem;                                           // sums of the jobs below
        const int nlat = w < L ? (L - w + a.W - 1) / a.W : 0, npair = w < R / 2 ? (R / 2 - w + a.W - 1) / a.W : 0;
        // 16-row tile: the sums of q_nope go in two levels (this member adds the KS partials of 1/16 of the head's
        // nope dimensions and publishes them, then fetches all of them): 16 times fewer polls per workgroup, which at
        // this batch outweighs the extra hand-over
        constexpr bool TWO = BT == 16;
        const int cpm = (a.n + TS - 1) / TS;                           // nope dimensions per member (two levels)
        const int J0 = TWO ? B * cpm : B * a.n, J1 = J0 + 4 * B, J2 = J1 + B * nlat, J3 = J2 + 2 * B * npair;
        float *s_red = smem + (J3 + 3) / 4 * 4;                        // [NW][BT][LJ]
        float *s_qn = TWO ? s_red + NW * BT * LJ : s_job;               // [B][n] q_nope of this head
        auto job_slot = [&](int i) -> size_t {                          // the first of the KS partials of job i
            if (i < J0) {
                const int b = TWO ? i / cpm : i / a.n, c = TWO ? min(cpm * j + i % cpm, a.n - 1) : i % a.n;
                return a.x1 + (size_t)b * CQ + head * nr + c;
            }
            i -= J0;
            if (i < 4 * B) {
                const int k = i % 4;                                    // lo of pair 2j, 2j + 1, then their partners
                return a.x1 + (size_t)(i / 4) * CQ + head * nr + a.n + (k >> 1) * (R / 2) + 2 * j + (k & 1);
            }
            i -= 4 * B;
            if (i < B * nlat) return a.x1 + (size_t)(i / nlat) * CQ + CQq + w + a.W * (i % nlat);
            i -= B * nlat;
            const int k = i % (2 * npair);                              // (lo, hi) of pair w + W * (k / 2)
            return a.x1 + (size_t)(i / (2 * npair)) * CQ + CQq + L + w + a.W * (k >> 1) + (R / 2) * (k & 1);
        };
        lds_sync();
        for (int i0 = tid; i0 < J3; i0 += NT * NVB) {
            size_t idx[NVB];
            float sum[NVB];
#pragma unroll
            for (int v = 0; v < NVB; ++v) idx[v] = job_slot(min(i0 + NT * v, J3 - 1));
            take_sums<NVB>(x, r, idx, (size_t)B * CQ, KS, sum);
#pragma unroll
            for (int v = 0; v < NVB; ++v)
                if (i0 + NT * v < J3) s_job[i0 + NT * v] = sum[v];
        }
        lds_sync();
        if (TWO) {
            for (int i = tid; i < J0; i += NT) {
                const int b = i / cpm, c = cpm * j + i % cpm;
                if (c < a.n) cf::team::put(r, a.xqn + ((size_t)b * a.nh + head) * 128 + c, s_job[i], x.stamp);
            }
            for (int i0 = 0; i0 < B * a.n; i0 += 4 * NT)
                fetch4(x, r, min(4 * NT, B * a.n - i0), s_qn + i0, [&](int i) {
                    return a.xqn + ((size_t)((i0 + i) / a.n) * a.nh + head) * 128 + (i0 + i) % a.n;
                });
            lds_sync();
        }
        MLA_STAMP(2);           // q_nope, q_rope and the new row summed
        for (int i = tid; i < 2 * B; i += NT) {                         // rotary query, pairs (p, p + R/2)
            const int b = i / 2, pp = i % 2, p = 2 * j + pp;
            const float lo = s_job[J0 + 4 * b + pp], hi = s_job[J0 + 4 * b + 2 + pp], c = s_rope[p], sn = s_rope[R / 2 + p];
            const size_t dst = a.xq + ((size_t)b * a.nh + head) * LR + L + p;
            cf::team::put(r, dst, lo * c - hi * sn, x.stamp);
            cf::team::put(r, dst + R / 2, hi * c + lo * sn, x.stamp);
        }
        for (int i = tid; i < B * nlat; i += NT) {                      // latent part of the new row
            const int b = i / nlat, d = w + a.W * (i % nlat);
            const float v = s_job[J1 + i];
            cf::team::put(r, a.xkv + (size_t)b * LR + d, v, x.stamp);
            a.cache[((size_t)b * a.max_seq + a.pos) * LR + d] = f2h(v);
        }
        for (int i = tid; i < B * npair; i += NT) {                     // rotary part of the new row
            const int b = i / npair, p = w + a.W * (i % npair);
            const float lo = s_job[J2 + 2 * i], hi = s_job[J2 + 2 * i + 1], c = s_rope[p], sn = s_rope[R / 2 + p];
            const float rl = lo * c - hi * sn, rh = hi * c + lo * sn;
            cf::team::put(r, a.xkv + (size_t)b * LR + L + p, rl, x.stamp);
            cf::team::put(r, a.xkv + (size_t)b * LR + L + p + R / 2, rh, x.stamp);
            uint16_t *row = a.cache + ((size_t)b * a.max_seq + a.pos) * LR + L + p;
            row[0] = f2h(rl);
            row[R / 2] = f2h(rh);
        }
        small_product<BT, 4, RPT_B>(wupr, s_qn, a.n, a.n, B, s_red, [&](int b, int cc, float sum) {
            cf::team::put(r, a.xq + ((size_t)b * a.nh + head) * LR + LJ * j + cc, sum, x.stamp);
        });
    }

    MLA_STAMP(3);           // B done
    // ---- C: attention.  Work item (b, s): cached rows [t0, t1) of batch row b against the queries of all heads.
    //      A tile is 64 rows, read from memory once and kept in LDS for both products (read twice, the second
    //      read of a row misses the L2 at batch 16 and the stage is bound by that traffic).  Scores: wavefronts
    //      0..3 take 16 rows each, S^T = K Q^T as one 16 x 16 tile (rows = tokens, columns = heads), the contraction
    //      over the 576 dimensions in 18 steps with the query as a pair of fp16 operands (value = hi + lo, so the
    //      fp32 query loses nothing).  Online softmax per head over the tile (the wavefronts exchange their maxima
    //      through LDS).  Weighted sum: wavefront (kq, th) takes the latent dimensions [128 kq, +128) and the rows
    //      [32 th, +32) of the tile: A = probabilities (fp16, from LDS), B = the rows themselves, eight at a time
    //      transposed inside the lane.  The item with s = 0 also scores the new token (its row is taken in fp32
    //      from stage B).
    {
        h8 *qop_hi = reinterpret_cast<h8 *>(smem);                      // [kSteps][64]
        h8 *qop_lo = qop_hi + kQops;
        float *s_m = smem + 2 * kQops * 4;                              // [NW][HT] maxima of the wavefronts' rows
        float *s_l = s_m + NW * HT;                                     // [NW][HT] sums of the wavefronts' probabilities
        float *s_M = s_l + NW * HT;                                     // [HT]
        float *s_kn = s_M + HT;                                         // [LR] the new row
        _Float16 *sP = reinterpret_cast<_Float16 *>(s_kn + LR);         // [HT][PS]
        float *sO = s_kn + LR + HT * PS / 2;                            // [HT][L], at the end of an item
        float *s_q = sO;                                                // [HT][QS], at its start
        _Float16 *sK = reinterpret_cast<_Float16 *>(sO);                // [kTile][KSTR] cached rows, between the two
        const int g = lane >> 4, c = lane & 15, kq = wv & 3, th = wv >> 2;
        const int ngroups = (a.nh + a.HG - 1) / a.HG;
        for (int it = w; it < B * a.NS * ngroups; it += a.W) {
            const int hg = it % ngroups, b = it / ngroups / a.NS, s = it / ngroups % a.NS;
            const int h0 = hg * a.HG, h1 = min(h0 + a.HG, a.nh);        // the heads of this item
            const int t0 = min(s * a.tps, a.pos), t1 = min(t0 + a.tps, a.pos);
            const uint16_t *rows = a.cache + (size_t)b * a.max_seq * LR;
            // A tile of rows goes from memory to LDS once (a thread carries nine 16-byte pieces of it, requested a
            // tile ahead); both products take their operands from there.  Rows past the range are read from its last
            // row (finite data) and get probability 0.
            constexpr int kPieces = kTile * (LR / 8) / NT;              // 9
            h8 kr[kPieces];
            auto request = [&](int T0) {
#pragma unroll
                for (int k = 0; k < kPieces; ++k) {
                    const int pc = tid + NT * k, row = pc / (LR / 8), col = pc % (LR / 8);
                    kr[k] = *reinterpret_cast<const h8 *>(rows + (size_t)min(T0 + row, t1 - 1) * LR + 8 * col);
                }
            };
            auto deposit = [&]() {
#pragma unroll
                for (int k = 0; k < kPieces; ++k) {
                    const int pc = tid + NT * k, row = pc / (LR / 8), col = pc % (LR / 8);
                    *reinterpret_cast<h8 *>(sK + row * KSTR + 8 * col) = kr[k];
                }
            };
            if (t1 > t0) request(t0);                                   // (uniform) the rows do not wait for the query
            lds_sync();                                                 // the previous item has left LDS
            MLA_STAMP(13);
            {
                // the query of the item's heads, [head][LR] fp32 scaled by log2(e) / sqrt(d_k): consecutive lanes poll
                // consecutive slots
                constexpr int NQ = HT * LR / NT;
                const int nq = (h1 - h0) * LR;
                const size_t src = a.xq + ((size_t)b * a.nh + h0) * LR;
                pair_t q[NQ];
                long long tw = 0;
                for (;;) {
#pragma unroll
                    for (int k = 0; k < NQ; ++k) {
                        q[k] = pair_t{0u, x.stamp};
                        if (NT * k < nq) q[k] = cf::team::peek(r, src + min(tid + NT * k, nq - 1));       // (uniform)
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    bool ok = true;
#pragma unroll
                    for (int k = 0; k < NQ; ++k) ok &= q[k].y == x.stamp;
                    if (ok || cf::team::gave_up(x, tw)) break;
                }
#pragma unroll
                for (int k = 0; k < NQ; ++k) {
                    const int i = tid + NT * k;
                    if (i < nq) s_q[(h0 + i / LR) * QS + i % LR] = __builtin_bit_cast(float, q[k].x) * a.scale_log2e;
                }
            }
            if (s == 0) {                                               // the new row, for the score of the new token
                for (int i0 = tid; i0 < LR; i0 += NT) {
                    long long tw = 0;
                    for (;;) {
                        const pair_t q = cf::team::peek(r, a.xkv + (size_t)b * LR + i0);
                        if (q.y == x.stamp || cf::team::gave_up(x, tw)) {
                            s_kn[i0] = __builtin_bit_cast(float, q.x);
                            break;
                        }
                    }
                }
            }
            lds_sync();
            // query operands: entry e = (step m, lane (g2, head c2)) holds the eight dimensions score_dim(m, g2) + 0..7
            // of head c2 as fp16 pairs (value = hi + lo); heads outside the item's group are zero
            for (int e = tid; e < kQops; e += NT) {
                const int m = e >> 6, g2 = (e >> 4) & 3, c2 = e & 15;
                const bool mine = c2 >= h0 && c2 < h1;
                const float *src = s_q + (mine ? c2 : h0) * QS + score_dim(m, g2);
                h8 hi, lo;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float v = mine ? src[i] : 0.f;
                    hi[i] = (_Float16)v;
                    lo[i] = (_Float16)(v - (float)hi[i]);
                }
                qop_hi[e] = hi;
                qop_lo[e] = lo;
            }
            if (s == 0) {
                // score of the new token: 32 lanes per head, 18 dimensions each
                const int h = min(h0 + (tid >> 5), h1 - 1), part = tid & 31;
                float d = 0.f;
#pragma unroll
                for (int k = 0; k < LR / 32; ++k) d = fmaf(s_q[h * QS + part * (LR / 32) + k], s_kn[part * (LR / 32) + k], d);
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) d += __shfl_xor(d, off);
                if (part == 0 && h0 + (tid >> 5) < h1) cf::team::put(r, a.xs + (size_t)b * a.nh + h, d, x.stamp);
            }
            lds_sync();
            MLA_STAMP(4);           // query operands built
            if (t1 > t0) {                                              // uniform over the workgroup
                float M = kNegBig, lw = 0.f;                            // of head c: running maximum; sum over this lane's rows
                f32x4 O[8];                                             // [jj][rr]: head 4 g + rr, dimension 128 kq + 8 c + jj
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) O[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int T0 = t0; T0 < t1; T0 += kTile) {
                    deposit();
                    if (T0 + kTile < t1) request(T0 + kTile);
                    lds_sync();
                    f32x4 S = {0.f, 0.f, 0.f, 0.f};                     // rows = tokens T0 + 16 wv + 4 g + rr, column = head c
                    if (wv < kTile / 16) {                              // (uniform per wavefront)
                        const _Float16 *krow = sK + (16 * wv + c) * KSTR;
#pragma unroll
                        for (int m = 0; m < kSteps; ++m) {
                            const h8 ka = *reinterpret_cast<const h8 *>(krow + score_dim(m, g));
                            S = mfma16(ka, qop_hi[m * 64 + lane], S);
                            S = mfma16(ka, qop_lo[m * 64 + lane], S);
                        }
                        float mx = kNegBig;
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            S[rr] = (T0 + 16 * wv + 4 * g + rr < t1) ? S[rr] : kNegBig;
                            mx = fmaxf(mx, S[rr]);
                        }
                        mx = fmaxf(mx, __shfl_xor(mx, 16));
                        mx = fmaxf(mx, __shfl_xor(mx, 32));
                        if (lane < HT) s_m[wv * HT + c] = mx;
                    }
                    lds_sync();
                    float mt = s_m[c];
#pragma unroll
                    for (int w4 = 1; w4 < kTile / 16; ++w4) mt = fmaxf(mt, s_m[w4 * HT + c]);
                    const float Mn = fmaxf(M, mt);                      // > kNegBig: the tile has a row inside the range
                    const float f = __builtin_amdgcn_exp2f(M - Mn);
                    M = Mn;
                    if (wv < kTile / 16) {
                        float psum = 0.f;
                        h4 ph;
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            const float pw = __builtin_amdgcn_exp2f(S[rr] - Mn);
                            ph[rr] = (_Float16)pw;
                            psum += pw;
                        }
                        lw = fmaf(lw, f, psum);
                        *reinterpret_cast<uint2 *>(sP + c * PS + 16 * wv + 4 * g) = __builtin_bit_cast(uint2, ph);
                    }
                    float fr[4];                                        // factor of the heads this lane accumulates
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) fr[rr] = __shfl(f, 4 * g + rr);
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) O[jj][rr] *= fr[rr];
                    lds_sync();
                    {
                        const h8 pa = *reinterpret_cast<const h8 *>(sP + c * PS + 32 * th + 8 * g);
                        h8 vr[8], f8[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            vr[u] = *reinterpret_cast<const h8 *>(sK + (32 * th + 8 * g + u) * KSTR + 128 * kq + 8 * c);
                        transpose8(vr, f8);
#pragma unroll
                        for (int jj = 0; jj < 8; ++jj) O[jj] = mfma16(pa, f8[jj], O[jj]);
                    }
                    lds_sync();                                         // the tile is consumed: the next one may land
                }
                MLA_STAMP(11);          // rows consumed
                lw += __shfl_xor(lw, 16);
                lw += __shfl_xor(lw, 32);
                if (lane < HT) {
                    s_l[wv * HT + c] = lw;
                    if (wv == 0) s_M[c] = M;
                }
                // the two halves of the tile rows are added through LDS (all wavefronts hold the same maxima)
                if (th == 1) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        float *dst = sO + (4 * g + rr) * L + 128 * kq + 8 * c;
                        *reinterpret_cast<float4 *>(dst) = make_float4(O[0][rr], O[1][rr], O[2][rr], O[3][rr]);
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(O[4][rr], O[5][rr], O[6][rr], O[7][rr]);
                    }
                }
                lds_sync();
                if (th == 0) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        float *dst = sO + (4 * g + rr) * L + 128 * kq + 8 * c;
                        const float4 lo4 = *reinterpret_cast<const float4 *>(dst), hi4 = *reinterpret_cast<const float4 *>(dst + 4);
                        *reinterpret_cast<float4 *>(dst) =
                            make_float4(O[0][rr] + lo4.x, O[1][rr] + lo4.y, O[2][rr] + lo4.z, O[3][rr] + lo4.w);
                        *reinterpret_cast<float4 *>(dst + 4) =
                            make_float4(O[4][rr] + hi4.x, O[5][rr] + hi4.y, O[6][rr] + hi4.z, O[7][rr] + hi4.w);
                    }
                }
                lds_sync();
                MLA_STAMP(12);          // wavefronts merged
                const size_t dst = a.x3 + ((size_t)b * a.NS + s) * HT * kPart;
                for (int i = h0 * L + tid; i < h1 * L; i += NT)
                    cf::team::put(r, dst + (size_t)(i / L) * kPart + 2 + i % L, sO[i], x.stamp);
                if (tid >= h0 && tid < h1) {
                    float ls = 0.f;
#pragma unroll
                    for (int w8 = 0; w8 < NW; ++w8) ls += s_l[w8 * HT + tid];
                    cf::team::put(r, dst + (size_t)tid * kPart, s_M[tid], x.stamp);
                    cf::team::put(r, dst + (size_t)tid * kPart + 1, ls, x.stamp);
                }
            }
        }
    }

    MLA_STAMP(5);           // C done
    // ---- D: merge latent dimensions [LJ*j, +LJ) of head `head` over the token ranges and the new token (online
    //      softmax, Alg. 4 steps 8-10) and multiply them by the same rows of W_Down[head]: a partial of a_head per
    //      member, no hop in between
    {
        float *s_z = smem;                                              // [B][LJ]
        float *s_red = smem + BT * LJ;                                  // [NW][BT][128]
        h8 wdr[RPT_D];
        {
            const int pc = tid % 16, rg = tid / G16;
#pragma unroll
            for (int k = 0; k < RPT_D; ++k) {
                const int row = rg + RG16 * k;
                wdr[k] = (pc < a.v / 8 && row < LJ)
                             ? *reinterpret_cast<const h8 *>(a.wdown + ((size_t)head * L + LJ * j + row) * a.v + pc * 8)
                             : h8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
        lds_sync();
        const int n_used = (a.pos + a.tps - 1) / a.tps;
        if (tid < LJ * B) {
            // lane sl of a group of 32 fetches the maximum and the sum of range sl (at most 32 ranges) and the group
            // shares them by shuffles; every lane fetches its own dimension of all ranges: one round trip in all
            const int b = tid / LJ, sl = tid % LJ, d = LJ * j + sl, nu1 = max(n_used, 1);
            pair_t qa[kMaxSplits], qm, ql, qn, qc;
            long long tw = 0;
            for (;;) {
                const size_t mine = a.x3 + (((size_t)b * a.NS + min(sl, nu1 - 1)) * HT + head) * kPart;
                qm = cf::team::peek(r, mine);
                ql = cf::team::peek(r, mine + 1);
                qn = cf::team::peek(r, a.xs + (size_t)b * a.nh + head);
                qc = cf::team::peek(r, a.xkv + (size_t)b * LR + d);
#pragma unroll
                for (int k = 0; k < kMaxSplits; ++k) {
                    qa[k] = pair_t{0u, x.stamp};
                    if (k < nu1) qa[k] = cf::team::peek(r, a.x3 + (((size_t)b * a.NS + k) * HT + head) * kPart + 2 + d);     // (uniform)
                }
                __builtin_amdgcn_sched_barrier(0);
                bool ok = (qn.y == x.stamp) & (qc.y == x.stamp) & ((sl >= n_used) | ((qm.y == x.stamp) & (ql.y == x.stamp)));
#pragma unroll
                for (int k = 0; k < kMaxSplits; ++k) ok &= (k >= n_used) | (qa[k].y == x.stamp);
                if (ok || cf::team::gave_up(x, tw)) break;
            }
            const float snew = __builtin_bit_cast(float, qn.x);
            const float ms = sl < n_used ? __builtin_bit_cast(float, qm.x) : kNegBig;
            float M = fmaxf(ms, snew);
#pragma unroll
            for (int off = 1; off < LJ; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
            const float fs = sl < n_used ? __builtin_amdgcn_exp2f(ms - M) : 0.f;
            float Ls = __builtin_bit_cast(float, ql.x) * fs;
#pragma unroll
            for (int off = 1; off < LJ; off <<= 1) Ls += __shfl_xor(Ls, off);
            const float fn = __builtin_amdgcn_exp2f(snew - M);          // the new token: weight 1 at its own score
            Ls += fn;
            float A = __builtin_bit_cast(float, qc.x) * fn;
#pragma unroll
            for (int k = 0; k < kMaxSplits; ++k) {
                const float fk = __shfl(fs, (lane & 32) + k);
                A = fmaf(k < n_used ? __builtin_bit_cast(float, qa[k].x) : 0.f, fk, A);
            }
            const float z = A / Ls;
            s_z[b * LJ + sl] = z;
            a.zdbg[((size_t)b * a.nh + head) * L + d] = z;
        }
        lds_sync();
        MLA_STAMP(6);           // z slice merged
        small_product<BT, 16, RPT_D>(wdr, s_z, LJ, LJ, B, s_red, [&](int b, int cc, float sum) {
            if (cc < a.v) cf::team::put(r, a.x5 + (((size_t)b * a.nh + head) * TS + j) * a.v + cc, sum, x.stamp);
        });
    }
    MLA_STAMP(7);           // D done

    // ---- E1: rows of W_O that belong to this head, column block j of the output: a partial of out per head
    {
        constexpr int NVE = BT == 4 ? 1 : 4;
        float *s_a = smem;                                              // [B][v]
        float *s_red = smem + BT * 128;                                 // [NW][BT][128]
        const int dpE = a.D / 8, pcsE = (dpE + TS - 1) / TS;            // 16-byte pieces of an output row; per member
        h8 wor[RPT_E];
        auto wo_rows = [&](int p0) {
            const int pc = tid % 16, rg = tid / G16;
            const int piece = j * pcsE + p0 + pc;
            const bool live = p0 + pc < pcsE && piece < dpE;
#pragma unroll
            for (int k = 0; k < RPT_E; ++k) {
                const int row = rg + RG16 * k;
                wor[k] = (live && row < a.v) ? *reinterpret_cast<const h8 *>(a.wo + ((size_t)head * a.v + row) * a.D + piece * 8)
                                             : h8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        };
        wo_rows(0);
        lds_sync();
        if constexpr (BT == 16) {
            // two levels as for q_nope: this member adds the TS partials of 1/16 of the head's dimensions
            const int cpv = (a.v + TS - 1) / TS;
            for (int i = tid; i < B * cpv; i += NT) {
                const int b = i / cpv, c = cpv * j + i % cpv;
                size_t idx[1] = {a.x5 + ((size_t)b * a.nh + head) * TS * a.v + min(c, a.v - 1)};
                float sum[1];
                take_sums<1>(x, r, idx, (size_t)a.v, TS, sum);
                if (c < a.v) cf::team::put(r, a.xa + ((size_t)b * a.nh + head) * 128 + c, sum[0], x.stamp);
            }
            for (int i0 = 0; i0 < B * a.v; i0 += 4 * NT)
                fetch4(x, r, min(4 * NT, B * a.v - i0), s_a + i0, [&](int i) {
                    return a.xa + ((size_t)((i0 + i) / a.v) * a.nh + head) * 128 + (i0 + i) % a.v;
                });
        } else {
            for (int i0 = tid; i0 < B * a.v; i0 += NT * NVE) {
                size_t idx[NVE];
                float sum[NVE];
#pragma unroll
                for (int v = 0; v < NVE; ++v) {
                    const int i = min(i0 + NT * v, B * a.v - 1);
                    idx[v] = a.x5 + ((size_t)(i / a.v) * a.nh + head) * TS * a.v + i % a.v;
                }
                take_sums<NVE>(x, r, idx, (size_t)a.v, TS, sum);
#pragma unroll
                for (int v = 0; v < NVE; ++v)
                    if (i0 + NT * v < B * a.v) s_a[i0 + NT * v] = sum[v];
            }
        }
        lds_sync();
        MLA_STAMP(8);           // a_head arrived
        for (int p0 = 0; p0 < pcsE; p0 += 16) {
            if (p0 > 0) {
                lds_sync();
                wo_rows(p0);
            }
            small_product<BT, 16, RPT_E>(wor, s_a, a.v, a.v, B, s_red, [&](int b, int cc, float sum) {
                const int piece2 = j * pcsE + p0 + cc / 8;
                if (p0 + cc / 8 < pcsE && piece2 < dpE)
                    cf::team::put(r, a.x6 + ((size_t)b * a.nh + head) * a.D + piece2 * 8 + cc % 8, sum, x.stamp);
            });
        }
    }
    MLA_STAMP(10);          // E1 done

    // ---- E2: sum over the heads (what the paper does with atomicAdd), columns [CW*w, +CW) of the output
    {
        const int CW = (a.D + a.W - 1) / a.W;
        if (tid < B * CW) {
            const int b = tid / CW, col = CW * w + tid % CW;
            if (col < a.D) {
                const size_t idx[1] = {a.x6 + (size_t)b * a.nh * a.D + col};
                float sum[1];
                take_sums<1>(x, r, idx, (size_t)a.D, a.nh, sum);
                a.out[(size_t)b * a.D + col] = f2h(sum[0]);
            }
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
    MLA_STAMP(9);
#if CF_STAMPS
    lds_sync();
    if (tid < kMlaStamps && w < 256) g_mla_ts[w * kMlaStamps + tid] = s_ts[tid];
#endif
}

using MlaFn = void (*)(const MlaArgs);

MlaFn pick(int batch) { return batch <= 4 ? fused_mla_decode<4> : fused_mla_decode<16>; }

}  // namespace

struct cf_mla_s {
    cf_mla_config cfg;
    int W = 0;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    uint64_t *slots = nullptr;
    float *zdbg = nullptr, *qdbg = nullptr;
    unsigned long long *counters = nullptr;
    uint32_t *err = nullptr;
    size_t x1 = 0, xq = 0, xkv = 0, x3 = 0, xs = 0, x5 = 0, x6 = 0, xqn = 0, xa = 0;
    long long spin_ticks = 200000000LL;
    int max_splits = 0;             // 0: chosen by the library
    int last_batch = 0;
    bool last_heads = false;        // the last call ran the head-team kernel
    int last_hip = 0;
};

namespace {

// token ranges of a call: NS ranges of tps cached rows per batch row; and the heads per attention item: as few as
// the number of workgroups allows (an item fetches the queries and publishes the partial results of its heads only:
// per workgroup that traffic, not the arithmetic, is what takes time)
void plan_splits(const cf_mla_s *t, int batch, int pos, int *ns, int *tps, int *hg)
{
    int cap = t->W / batch;
    cap = cap < 1 ? 1 : cap > kMaxSplits ? kMaxSplits : cap;
    if (t->max_splits > 0 && t->max_splits < cap) cap = t->max_splits;
    int per = (pos + cap - 1) / cap;
    per = (per + 15) / 16 * 16;
    if (per < 64 && t->max_splits == 0) per = 64;     // below a tile more ranges only add partials
    if (per < 16) per = 16;
    *tps = per;
    const int n = (pos + per - 1) / per;
    *ns = n < 1 ? 1 : n;                              // range 0 always exists: it scores the new token
    int groups = 1;
    while (2 * groups <= t->cfg.n_heads && batch * *ns * 2 * groups <= t->W) groups *= 2;
    *hg = (t->cfg.n_heads + groups - 1) / groups;
}

}  // namespace

extern "C" {

int cf_mla_create(const cf_mla_config *cfg, cf_mla *out)
{
    if (!cfg || !out) return CF_EINVAL;
    *out = nullptr;
    const cf_mla_config &c = *cfg;
    if (c.d_model < 16 || c.n_heads < 1 || c.nope_dim < 1 || c.v_head_dim < 1 || c.max_batch < 1 || c.max_seq < 1 ||
        !(c.rope_base > 1.f))
        return CF_EINVAL;
    // what the kernel is written for
    const int W = c.n_heads * TS;
    const int CQq = c.n_heads * (c.nope_dim + R);
    const int cq = (CQq / 8 + 15) / 16, ckv = (LR / 8 + 15) / 16;          // 16-byte pieces per column block
    if (c.kv_lora_rank != L || c.rope_dim != R || c.max_batch > MAXBATCH || c.n_heads > HT || c.d_model % (2 * KS) ||
        c.d_model / KS > NT || c.v_head_dim % 8 || c.v_head_dim > 128 || cq + ckv > 32 || c.nope_dim % 8 ||
        c.nope_dim > 128 || c.d_model > 8 * W || c.d_model % 8)
        return CF_EUNSUPPORTED;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CF_EHIP;
    if (W > prop.multiProcessorCount) return CF_EUNSUPPORTED;        // all workgroups resident, one per compute unit
    const size_t lds = kLdsFloats * sizeof(float);
    for (int batch : {1, MAXBATCH}) {
        int per_cu = 0;
        const void *fn = reinterpret_cast<const void *>(pick(batch));
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, NT, lds) != hipSuccess || per_cu < 1)
            return CF_EUNSUPPORTED;
    }
    if (!cf::mla::heads_prepare()) return CF_EUNSUPPORTED;
    cf_mla t = new (std::nothrow) cf_mla_s();
    if (!t) return CF_ENOMEM;
    t->cfg = c;
    t->W = W;
    const size_t B = c.max_batch, CQ = (size_t)CQq + LR, items = (size_t)(W > c.max_batch ? W : c.max_batch);
    t->x1 = 0;
    t->xq = t->x1 + (size_t)KS * B * CQ;
    t->xkv = t->xq + B * c.n_heads * LR;
    t->x3 = t->xkv + B * LR;
    t->xs = t->x3 + items * HT * kPart;
    t->x5 = t->xs + B * c.n_heads;
    t->x6 = t->x5 + B * c.n_heads * TS * c.v_head_dim;
    size_t hfirst[5];
    const size_t hslots = cf::mla::heads_layout(c, c.max_batch < cf::mla::kHeadsMaxBatch ? c.max_batch : cf::mla::kHeadsMaxBatch, hfirst);
    t->xqn = t->x6 + B * c.n_heads * c.d_model;                  // [B][heads][128] summed q_nope (16-row tile)
    t->xa = t->xqn + B * c.n_heads * 128;                         // [B][heads][128] summed a_head (16-row tile)
    const size_t rslots = t->xa + B * c.n_heads * 128;
    const size_t nslots = rslots > hslots ? rslots : hslots;         // the two kernels use the same slots, never together
    const size_t head = 256 + (size_t)W * kCounterStride * sizeof(unsigned long long);
    const size_t head_al = (head + 255) / 256 * 256;
    const size_t slot_bytes = (nslots * sizeof(uint64_t) + 255) / 256 * 256;
    const size_t zbytes = (B * c.n_heads * L * sizeof(float) + 255) / 256 * 256;
    t->ws_bytes = head_al + slot_bytes + zbytes + B * c.n_heads * LR * sizeof(float);
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
    t->zdbg = reinterpret_cast<float *>(t->ws + head_al + slot_bytes);
    t->qdbg = reinterpret_cast<float *>(t->ws + head_al + slot_bytes + zbytes);
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
    if (batch <= kHeadsBatch && t->max_splits == 0) {
        // one or two batch rows: the head-team kernel (every head scans the cached rows itself; see cf_mla_heads.hip)
        cf::mla::HeadsArgs h;
        std::memset(&h, 0, sizeof h);
        h.x = static_cast<const uint16_t *>(x);
        h.wq = static_cast<const uint16_t *>(W_q);
        h.wkv = static_cast<const uint16_t *>(W_kv);
        h.wup = static_cast<const uint16_t *>(W_up);
        h.wdown = static_cast<const uint16_t *>(W_down);
        h.wo = static_cast<const uint16_t *>(W_o);
        h.cache = static_cast<uint16_t *>(kv_cache);
        h.out = static_cast<uint16_t *>(out);
        h.qdbg = t->qdbg, h.zdbg = t->zdbg;
        h.slots = t->slots, h.counters = t->counters, h.err = t->err;
        size_t first[5];
        (void)cf::mla::heads_layout(c, batch, first);
        h.x1 = first[0], h.x2 = first[1], h.x3 = first[2], h.x5 = first[3], h.x6 = first[4];
        h.D = c.d_model, h.nh = c.n_heads, h.n = c.nope_dim, h.v = c.v_head_dim, h.B = batch, h.pos = pos;
        h.max_seq = c.max_seq, h.W = t->W;
        h.cq = (c.n_heads * (c.nope_dim + R) / 8 + 15) / 16;
        h.ckv = (LR / 8 + 15) / 16;
        h.scale_log2e = 1.4426950408889634f / std::sqrt((float)(c.nope_dim + R));
        h.log2_base = std::log2((double)c.rope_base);
        h.spin_ticks = t->spin_ticks;
        t->last_batch = batch, t->last_heads = true;
        const int e = cf::mla::heads_launch(h, stream);
        if (e != (int)hipSuccess) {
            t->last_hip = e;
            return CF_EHIP;
        }
        return CF_OK;
    }
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
    a.zdbg = t->zdbg;
    a.slots = t->slots;
    a.counters = t->counters;
    a.err = t->err;
    // the exchange areas are laid out for max_batch; a smaller batch uses the front of each
    a.x1 = t->x1, a.xq = t->xq, a.xkv = t->xkv, a.x3 = t->x3, a.xs = t->xs, a.x5 = t->x5, a.x6 = t->x6, a.xqn = t->xqn, a.xa = t->xa;
    a.D = c.d_model, a.nh = c.n_heads, a.n = c.nope_dim, a.v = c.v_head_dim, a.B = batch, a.pos = pos;
    a.max_seq = c.max_seq, a.W = t->W;
    plan_splits(t, batch, pos, &a.NS, &a.tps, &a.HG);
    a.cq = (c.n_heads * (c.nope_dim + R) / 8 + 15) / 16;
    a.ckv = (LR / 8 + 15) / 16;
    a.scale_log2e = 1.4426950408889634f / std::sqrt((float)(c.nope_dim + R));
    a.log2_base = std::log2((double)c.rope_base);
    a.spin_ticks = t->spin_ticks;
    t->last_batch = batch, t->last_heads = false;
    hipLaunchKernelGGL(pick(batch), dim3(t->W), dim3(NT), kLdsFloats * sizeof(float), static_cast<hipStream_t>(stream), a);
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

int cf_mla_set_splits(cf_mla t, int32_t max_splits)
{
    if (!t || max_splits < 0 || max_splits > kMaxSplits) return CF_EINVAL;
    t->max_splits = max_splits;
    return CF_OK;
}

int cf_mla_debug_export(cf_mla t, int32_t what, void *host_dst, size_t bytes, void *stream)
{
    if (!t || !host_dst || what < 0 || what > 2 || t->last_batch < 1) return CF_EINVAL;
    const size_t B = t->last_batch, nh = t->cfg.n_heads;
    const size_t per = what == 1 ? R : L;
    if (bytes != B * nh * per * sizeof(float)) return CF_EINVAL;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e == hipSuccess && what == 2) e = hipMemcpy(host_dst, t->zdbg, bytes, hipMemcpyDeviceToHost);
    if (e == hipSuccess && what != 2 && t->last_heads) {
        std::vector<float> q(B * nh * LR);
        e = hipMemcpy(q.data(), t->qdbg, q.size() * sizeof(float), hipMemcpyDeviceToHost);
        float *dst = static_cast<float *>(host_dst);
        if (e == hipSuccess)
            for (size_t i = 0; i < B * nh; ++i)
                std::memcpy(dst + i * per, q.data() + i * LR + (what == 1 ? L : 0), per * sizeof(float));
    } else if (e == hipSuccess && what != 2) {
        // the query of the last call still sits in its exchange slots: [b][head][L + R] {value, stamp} pairs
        std::vector<uint64_t> pairs(B * nh * LR);
        e = hipMemcpy(pairs.data(), t->slots + t->xq, pairs.size() * sizeof(uint64_t), hipMemcpyDeviceToHost);
        float *dst = static_cast<float *>(host_dst);
        if (e == hipSuccess)
            for (size_t b = 0; b < B; ++b)
                for (size_t h = 0; h < nh; ++h)
                    for (size_t k = 0; k < per; ++k) {
                        const uint32_t bits = (uint32_t)pairs[(b * nh + h) * LR + (what == 1 ? L : 0) + k];
                        std::memcpy(dst + (b * nh + h) * per + k, &bits, sizeof bits);
                    }
    }
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    return CF_OK;
}

#if CF_STAMPS
// profiling library only: the stage stamps of the last launch (host buffer of 256 * 16 64-bit words)
int cf_mla_trace_read(void *host_dst)
{
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_mla_ts), sizeof(unsigned long long) * 256 * kMlaStamps);
    return e == hipSuccess ? CF_OK : CF_EHIP;
}
#endif

int cf_mla_set_spin_limit(cf_mla t, int32_t spin_limit_us)
{
    if (!t || spin_limit_us < 0) return CF_EINVAL;
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
