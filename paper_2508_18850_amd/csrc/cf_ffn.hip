// Feed-forward block of a decoder layer (paper Sec. 2.1, FFN(Z) = W3 (sigma(W1 Z) * W2 Z)) for one token per
// sequence as ONE kernel for gfx950, behind the C ABI (cf_ffn_* in include/cfdecode.h).
//
// The paper fuses the attention block and names the FFN as the other part of a layer; here it is built the same
// way: one launch, the hidden vector g = sigma(W1 z) * W2 z never leaves the chip, and the only exchange between
// workgroups is the sum of the per-workgroup partial outputs (stamped {value, stamp} slots, cf_team_device.h),
// the counterpart of the decode block's sum over heads.
//
// All three matrices are stored [d_ff, d_model] (row f = hidden unit f), so hidden unit f is one contiguous row in
// each of them.  Workgroup w owns the hidden units [w F / W, (w + 1) F / W):
//   A  h_f = W1[f] . z, u_f = W2[f] . z for its units: a row is read in 512-column pieces, one piece per wavefront
//      step (64 lanes x 16 bytes, contiguous), the pieces of all rows dealt round-robin to the eight wavefronts;
//      fp16 x fp16 products accumulated in fp32 (v_dot2_f32_f16), summed over the wavefront and, through LDS,
//      over the pieces of a row in a fixed order;  g_f = sigma(h_f) u_f
//   B  partial out = sum over its units of g_f W3[f]: thread t owns eight columns (and eight more per further
//      4096 columns), a row of W3 is one contiguous read of the whole workgroup; no reduction inside the
//      workgroup is needed
//   C  every workgroup adds, in workgroup order, the partials of its own d_model / W output columns and writes fp16.
// The first rows of W3 are requested before the last pieces of stage A are consumed, so the memory pipe does not
// drain at the stage boundary.  All waits are bounded (CF_ETIMEOUT); all workgroups have to be resident at once.
#include "../../include/cfdecode.h"
#include "cf_mfma_device.h"
#include "cf_team_device.h"

#include <cmath>
#include <cstring>
#include <new>

namespace {

using cf::team::Exchange;
using cf::team::pair_t;
constexpr int NT = 512;
constexpr int NW = NT / 64;
constexpr int kChunk = 512;            // columns of one wavefront load: 64 lanes x 8 values
constexpr int kCounterStride = 16;
constexpr int kMaxBatch = 16;          // the batch of Appendix C
constexpr int kVectorBatch = 4;        // the largest batch of the vector-unit kernel
constexpr int kTilesFrom = 2;          // from this batch on the MFMA kernel runs where the shape allows it (measured:
                                       // Llama-2-7B shape, batch 1 / 2 / 4: 46.5 / 52.3 / 75.2 us against 47.8 / 47.8 / 49.0)
constexpr int kNC = 16;                // MFMA kernel: column slices of the output (workgroups per slice of hidden units)
constexpr int kStageRow = 256 + 8;     // MFMA kernel: row stride (fp16 values) of a wavefront's staging area in LDS
constexpr uint32_t kNoLoad = 0x80000000u;

using cf::mfma::f32x4;
using cf::mfma::h8;
using cf::mfma::mfma16;
using cf::mfma::transpose8;
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

struct FfnArgs {
    const uint16_t *z, *w1, *w2, *w3;
    uint16_t *out;
    uint64_t *slots;                   // [W][B][D] partial outputs
    unsigned long long *counters;
    uint32_t *err;
    int D, F, B, W, act;
    int nrmax;                         // most hidden units a workgroup owns
    long long spin_ticks;
    // MFMA kernel only
    size_t xg, xp;                     // first slot of g [d_ff][B] and of the partial outputs [NF][B][D]
    int NF, CW, nRp;                   // slices of hidden units; columns per column slice; units of a slice, padded to 32
};

struct Stream {
    __amdgpu_buffer_rsrc_t r;
    __device__ __forceinline__ Stream(const void *base, uint32_t bytes)
        : r(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000)) {}
    __device__ __forceinline__ h8 ld(uint32_t voff, uint32_t soff) const
    {
        return __builtin_bit_cast(h8, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 2));
    }
};

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the wavefront (the same value in every lane): four steps inside each row of 16 lanes, then the four row
// totals are read out as scalars.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    const int i = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(i, 48));
    return (r0 + r1) + (r2 + r3);
}

// eight fp16 x fp16 products added to acc in fp32
__device__ __forceinline__ float dot8(const h8 &a, const h8 &b, float acc)
{
#pragma unroll
    for (int k = 0; k < 4; ++k)
        acc = __builtin_amdgcn_fdot2(h2{a[2 * k], a[2 * k + 1]}, h2{b[2 * k], b[2 * k + 1]}, acc, false);
    return acc;
}

__device__ __forceinline__ float activate(float a, int act)
{
    if (act == CF_FFN_GELU) return 0.5f * a * (1.0f + erff(a * 0.70710678118654752f));
    return a / (1.0f + __expf(-a));                    // SiLU
}

template <int BT, int NCB>     // batch tile; column blocks of 4096 per thread (d_model <= 4096 NCB)
__global__ void __launch_bounds__(NT) fused_ffn(const FfnArgs a)
{
    extern __shared__ __align__(16) float smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = blockIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int D = a.D, B = a.B;
    const int NCK = (D + kChunk - 1) / kChunk;                    // pieces of a row
    const int Dp = NCK * kChunk;
    const int r0 = (int)((long long)w * a.F / a.W), r1 = (int)((long long)(w + 1) * a.F / a.W), nr = r1 - r0;
    const int NU = nr * NCK;                                      // (row, piece) units of this workgroup, per matrix
    // LDS: z as fp16 [BT][Dp]; partial dot products [2][BT][nrmax][NCK]; g [BT][nrmax]
    _Float16 *z16 = reinterpret_cast<_Float16 *>(smem);
    float *part = smem + BT * Dp / 2;
    float *gl = part + 2 * BT * a.nrmax * NCK;

    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)w * kCounterStride)
                 : "memory");
    const unsigned long long cnt = launches + 1ull;
    const Exchange x = {a.slots, 0, (uint32_t)(cnt + (cnt >> 32)), a.err, a.spin_ticks};
    const __amdgpu_buffer_rsrc_t xr = cf::team::slots_rsrc(x);

    const uint32_t wbytes = (uint32_t)((size_t)a.F * D * 2);
    const Stream W1(a.w1, wbytes), W2(a.w2, wbytes), W3(a.w3, wbytes);

    // ---- stage A.  Units q = wv, wv + 8, ... of this wavefront; unit q is piece q % NCK of row q / NCK.
    constexpr int U = 4;                                          // units per batch of loads (two loads each)
    struct Cursor {
        int r, c;                                                 // row (local), piece
    };
    // a wavefront's next unit is eight units on: branch-free (loads inside branches would make every later
    // wait for a load drain the queue)
    const int dr = NW / NCK, dc = NW % NCK;
    auto advance = [&](Cursor &k) {
        k.c += dc;
        k.r += dr;
        const bool wrap = k.c >= NCK;
        k.c -= wrap ? NCK : 0;
        k.r += wrap ? 1 : 0;
    };
    Cursor lc = {wv / NCK, wv % NCK};
    Cursor cc = lc;
    auto load = [&](h8(&p1)[U], h8(&p2)[U], uint32_t dep) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = lc.r < nr && lc.c * kChunk + lane * 8 < D;
            const uint32_t voff = live ? (uint32_t)lane * 16 + dep : kNoLoad;
            const uint32_t soff = (uint32_t)(((size_t)(r0 + lc.r) * D + (size_t)lc.c * kChunk) * 2);
            p1[u] = W1.ld(voff, lc.r < nr ? soff : 0u);
            p2[u] = W2.ld(voff, lc.r < nr ? soff : 0u);
            advance(lc);
        }
    };
    h8 a1[U], a2[U], b1[U], b2[U];
    load(a1, a2, 0u);
    // z of every batch row -> LDS as it is (fp16), zero past d_model and past the batch
    for (int i = tid; i < BT * Dp / 8; i += NT) {
        const int b = i / (Dp / 8), c8 = i - b * (Dp / 8);
        uint4 v = {0u, 0u, 0u, 0u};
        if (b < B && c8 * 8 < D) v = *reinterpret_cast<const uint4 *>(a.z + (size_t)b * D + c8 * 8);
        *reinterpret_cast<uint4 *>(z16 + (size_t)b * Dp + c8 * 8) = v;
    }
    load(b1, b2, 0u);
    lds_barrier();

    auto consume = [&](const h8(&p1)[U], const h8(&p2)[U]) -> uint32_t {
        float keep = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool live = cc.r < nr;
            const int c = cc.c, r = live ? cc.r : 0;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                const h8 zc = *reinterpret_cast<const h8 *>(z16 + (size_t)b * Dp + c * kChunk + lane * 8);
                const float d1 = wave_sum(dot8(p1[u], zc, 0.f)), d2 = wave_sum(dot8(p2[u], zc, 0.f));
                if (live && lane == 0) {
                    part[(b * a.nrmax + r) * NCK + c] = d1;
                    part[((BT + b) * a.nrmax + r) * NCK + c] = d2;
                }
                keep += d1 + d2;
            }
            advance(cc);
        }
        // the reload of this register batch is made to follow its last use (its offset depends on the sums)
        uint32_t dep = 0;
        asm volatile("" : "+v"(dep) : "v"(keep));
        return dep;
    };

    // ---- stage B set-up: thread t owns columns 8 t + 4096 cb
    constexpr int UB = 8;                                         // rows of W3 per batch of loads
    auto load3 = [&](h8(&p3)[NCB][UB], int row0, uint32_t dep) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int r = row0 + u, col = 8 * tid + 4096 * cb;
                const bool live = r < nr && col < D;
                p3[cb][u] = W3.ld(live ? (uint32_t)col * 2 + dep : kNoLoad, r < nr ? (uint32_t)((size_t)(r0 + r) * D * 2) : 0u);
            }
    };
    h8 t3a[NCB][UB], t3b[NCB][UB];

    const int nsteps = (NU + NW * U - 1) / (NW * U);             // batches of this wavefront (the same for all)
    const int nsteps2 = max(2, (nsteps + 1) & ~1);
    for (int k = 0; k + 2 < nsteps2; k += 2) {
        const uint32_t d0 = consume(a1, a2);
        load(a1, a2, d0);
        const uint32_t d1 = consume(b1, b2);
        load(b1, b2, d1);
    }
    load3(t3a, 0, 0u);                                            // the first rows of W3, before the tail of stage A
    consume(a1, a2);
    load3(t3b, UB, 0u);
    consume(b1, b2);
    lds_barrier();
    // pieces of a row in piece order; activation; g
    for (int e = tid; e < BT * nr; e += NT) {
        const int b = e / nr, r = e - b * nr;
        float h = 0.f, u = 0.f;
        for (int c = 0; c < NCK; ++c) {
            h += part[(b * a.nrmax + r) * NCK + c];
            u += part[((BT + b) * a.nrmax + r) * NCK + c];
        }
        gl[b * a.nrmax + r] = b < B ? activate(h, a.act) * u : 0.f;
    }
    lds_barrier();

    // ---- stage B
    float acc[BT][NCB][8];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][cb][j] = 0.f;
    auto consume3 = [&](const h8(&p3)[NCB][UB], int row0) -> uint32_t {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int r = min(row0 + u, nr - 1);               // a row past the end has zero weights
                float f[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) f[j] = (float)p3[cb][u][j];
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float g = gl[b * a.nrmax + r];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[b][cb][j] = fmaf(g, f[j], acc[b][cb][j]);
                }
            }
        uint32_t dep = 0;
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
                asm volatile("" : "+v"(dep) : "v"(acc[b][cb][0]), "v"(acc[b][cb][1]), "v"(acc[b][cb][2]), "v"(acc[b][cb][3]),
                             "v"(acc[b][cb][4]), "v"(acc[b][cb][5]), "v"(acc[b][cb][6]), "v"(acc[b][cb][7]));
        return dep;
    };
    // two batches of rows in flight; consume and reload are unconditional (a batch past the end is all zeros)
    for (int row0 = 0; row0 < nr; row0 += 2 * UB) {
        const uint32_t d0 = consume3(t3a, row0);
        load3(t3a, row0 + 2 * UB, d0);
        const uint32_t d1 = consume3(t3b, row0 + UB);
        load3(t3b, row0 + 3 * UB, d1);
    }
    // ---- the partial output of this workgroup.  A thread holds eight adjacent columns; stored from there, one store
    //      instruction would touch 64 lines with 8 bytes each.  The values pass through LDS (4096 columns at a time) so
    //      that consecutive lanes write consecutive slots.
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            if (b < B) {                                          // (uniform)
                lds_barrier();
                *reinterpret_cast<float4 *>(smem + 8 * tid) = make_float4(acc[b][cb][0], acc[b][cb][1], acc[b][cb][2], acc[b][cb][3]);
                *reinterpret_cast<float4 *>(smem + 8 * tid + 4) = make_float4(acc[b][cb][4], acc[b][cb][5], acc[b][cb][6], acc[b][cb][7]);
                lds_barrier();
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int col = 4096 * cb + NT * j + tid;
                    if (col < D) cf::team::put(xr, ((size_t)w * B + b) * D + col, smem[NT * j + tid], x.stamp);
                }
            }
        }

    lds_barrier();              // stage C reuses the front of LDS
    // ---- stage C: columns [c0, c0 + ncol) of every batch row, summed over the workgroups in workgroup order
    const int cpw = (D + a.W - 1) / a.W;
    const int c0 = w * cpw, ncol = min(cpw, D - c0);
    if (ncol > 0) {
        const int nv = ncol * B;                                  // values this workgroup produces (<= 512 is checked on the host)
        const int spt = max(1, min(NT / nv, a.W));                // slots read in parallel
        const int v = tid % nv, s0 = tid / nv;
        const int b = v / ncol, c = v - b * ncol;
        if (s0 < spt) {
            constexpr int NP = 8;
            float s = 0.f;
            for (int k0 = s0; k0 < a.W; k0 += NP * spt) {
                pair_t q[NP];
                long long t0 = 0;
                for (;;) {
#pragma unroll
                    for (int k = 0; k < NP; ++k) {
                        const int slot = min(k0 + k * spt, a.W - 1);
                        q[k] = cf::team::peek(xr, ((size_t)slot * B + b) * D + c0 + c);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    bool ok = true;
#pragma unroll
                    for (int k = 0; k < NP; ++k) ok &= (k0 + k * spt >= a.W) | (q[k].y == x.stamp);
                    if (ok || cf::team::gave_up(x, t0)) break;
                }
#pragma unroll
                for (int k = 0; k < NP; ++k)
                    if (k0 + k * spt < a.W) s += __builtin_bit_cast(float, q[k].x);
            }
            smem[s0 * nv + v] = s;
        }
        lds_barrier();
        if (tid < nv) {
            float s = 0.f;
            for (int k = 0; k < spt; ++k) s += smem[k * nv + tid];
            a.out[(size_t)b * D + c0 + c] = __builtin_bit_cast(uint16_t, (_Float16)s);
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

// Stage time stamps of every workgroup, only in builds with -DCF_STAMPS=1 (the profiling library).
#ifndef CF_STAMPS
#define CF_STAMPS 0
#endif
#if CF_STAMPS
constexpr int kFfnStamps = 16;
__device__ unsigned long long g_ffn_ts[256 * kFfnStamps];
#define FFN_STAMP(k) do { if (threadIdx.x == 0) s_ts[k] = wall_clock64(); } while (0)
#else
#define FFN_STAMP(k)
#endif

// ---------------------------------------------------------------------------------------------------------------------
// Batch 2..16: the same block on matrix cores, with the work cut in two directions.  One partial output per workgroup
// (as above) would be W x B x d_model stamped pairs, 134 MB at batch 16; here the W workgroups form NF = W / 16 slices
// of hidden units times 16 slices of output columns:
//   A  as above, workgroup w owns the hidden units [w F / W, (w + 1) F / W): h = W1 z, u = W2 z as 16 x 16 x 32 MFMA
//      steps, A = sixteen rows of the weights (read as they lie in memory and brought into the operand layout through
//      LDS), B = z in fp16 as given, held in registers for the 512 columns of a wavefront; the eight wavefronts
//      (eight column pieces) are added through LDS; g = sigma(h) u goes to stamped slots [d_ff][B]
//   G  workgroup (fi, ci) fetches g of slice fi (the units of 16 workgroups) and keeps it in LDS as fp16 pairs
//      (value = hi + lo, so fp32 g loses nothing)
//   B  partial out [B][columns of slice ci] = g W3[slice fi]: A = g, B = eight rows of a 16-byte piece of W3
//      transposed inside the lane; wavefront (cg, ks) takes 128 columns and every (8 / groups)-th step of 32 units;
//      the wavefronts of a column group are added through LDS; the partial goes to slots [NF][B][d_model]
//   C  workgroup (fi, ci) adds the NF partials of 1/NF of the columns of slice ci, in slice order, and writes fp16.
// Two hand-overs instead of one, NF partials per output value instead of W.
template <int NTL>     // row tiles of 16 hidden units a workgroup owns at most (1..8)
__global__ void __launch_bounds__(NT) fused_ffn_tiles(const FfnArgs a)
{
    extern __shared__ __align__(16) float smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = blockIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int D = a.D, B = a.B;
    const int r0 = (int)((long long)w * a.F / a.W), nr = (int)((long long)(w + 1) * a.F / a.W) - r0;
    const int fi = w / kNC, ci = w % kNC;
    const int R0 = (int)((long long)(fi * kNC) * a.F / a.W), nR = (int)((long long)(fi * kNC + kNC) * a.F / a.W) - R0;
    // n / B for n < 2^28 without a division (B = 1: the reciprocal does not fit 32 bits)
    const uint32_t inv_b = B > 1 ? (uint32_t)((0x100000000ull + (unsigned)B - 1) / (unsigned)B) : 0u;
    auto div_b = [&](int n) { return B > 1 ? (int)__umulhi((uint32_t)n, inv_b) : n; };
#if CF_STAMPS
    __shared__ unsigned long long s_ts[kFfnStamps];
    if (tid < kFfnStamps) s_ts[tid] = 0;
#endif
    FFN_STAMP(0);

    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)w * kCounterStride)
                 : "memory");
    const unsigned long long cnt = launches + 1ull;
    const Exchange x = {a.slots, 0, (uint32_t)(cnt + (cnt >> 32)), a.err, a.spin_ticks};
    const __amdgpu_buffer_rsrc_t xr = cf::team::slots_rsrc(x);
    const uint32_t wbytes = (uint32_t)((size_t)a.F * D * 2);
    const Stream W1(a.w1, wbytes), W2(a.w2, wbytes), W3(a.w3, wbytes);

    // ---- stage A.  A task is sixteen weight rows by 256 columns of one matrix.  The rows are read as they lie in
    //      memory (a load instruction of a wavefront is two rows of 512 contiguous bytes; read in the layout of the MFMA
    //      operand, sixteen rows of 64 bytes per instruction, the same bytes took 4.8 us longer at batch 16) and pass
    //      through a staging area in LDS that belongs to the wavefront alone: no barrier, LDS operations of a wavefront
    //      execute in order.  Contraction slot (step m, group g, element e) of a 512-column piece is its column
    //      32 m + 8 g + e.
    {
        const int NCK = (D + kChunk - 1) / kChunk;
        f32x4 acc[NTL][2];                                        // [tile][matrix]: units 16 t + 4 g + rr, batch row c
#pragma unroll
        for (int t = 0; t < NTL; ++t) acc[t][0] = acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        _Float16 *stg = reinterpret_cast<_Float16 *>(smem) + (size_t)wv * 16 * kStageRow;      // [16][kStageRow]
        const int hi = lane >> 5, lp = lane & 31;
        for (int piece = wv; piece < NCK; piece += NW) {          // (uniform per wavefront)
            h8 zb[16];
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int col = kChunk * piece + 32 * m + 8 * g;
                uint4 v = {0u, 0u, 0u, 0u};
                if (c < B && col < D) v = *reinterpret_cast<const uint4 *>(a.z + (size_t)c * D + col);
                zb[m] = __builtin_bit_cast(h8, v);
            }
            // two tasks in flight; load k of a task: rows 2 k and 2 k + 1 of the tile, 32 lanes each
            auto request = [&](h8(&wr)[8], int task) {
                const int t = task >> 2, mat = (task >> 1) & 1, half = task & 1;
                const bool colok = kChunk * piece + 256 * half + 8 * lp < D;
                const uint32_t soff = 16 * t < nr ? (uint32_t)(((size_t)(r0 + 16 * t) * D + (size_t)kChunk * piece) * 2) : 0u;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int row = 2 * k + hi;                    // rows past the workgroup's units are not read
                    const uint32_t voff = (colok && 16 * t + row < nr) ? (uint32_t)row * (uint32_t)D * 2u + 512u * half + 16u * lp : kNoLoad;
                    wr[k] = mat ? W2.ld(voff, soff) : W1.ld(voff, soff);
                }
            };
            // (the fences and the wave barrier emit nothing: they keep the compiler from moving the reads of other
            // lanes' values across the writes, which it might, seeing that a thread's own addresses differ)
            auto wave_sync = [&]() {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            };
            auto stage = [&](const h8(&wr)[8]) {
                wave_sync();                                       // the previous task's operands have been read
#pragma unroll
                for (int k = 0; k < 8; ++k) *reinterpret_cast<h8 *>(stg + (2 * k + hi) * kStageRow + 8 * lp) = wr[k];
                wave_sync();
            };
            auto consume = [&](int task) {
                const int t = task >> 2, mat = (task >> 1) & 1, half = task & 1;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const h8 wop = *reinterpret_cast<const h8 *>(stg + c * kStageRow + 32 * k + 8 * g);
                    acc[t][mat] = mfma16(wop, zb[8 * half + k], acc[t][mat]);
                }
            };
            h8 wa[8], wb[8];
            request(wa, 0);
            request(wb, 1);
#pragma unroll
            for (int task = 0; task < 4 * NTL; task += 2) {
                stage(wa);
                if (task + 2 < 4 * NTL) request(wa, task + 2);
                consume(task);
                stage(wb);
                if (task + 3 < 4 * NTL) request(wb, task + 3);
                consume(task + 1);
            }
        }
        lds_barrier();                                            // the staging areas are left: the sums below overlay them
        FFN_STAMP(1);       // products of stage A done
        float4 *part = reinterpret_cast<float4 *>(smem);          // [NW][NTL][2][64 lanes]
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
            for (int mat = 0; mat < 2; ++mat)
                part[((wv * NTL + t) * 2 + mat) * 64 + lane] =
                    make_float4(acc[t][mat][0], acc[t][mat][1], acc[t][mat][2], acc[t][mat][3]);
        lds_barrier();
        for (int e = tid; e < nr * B; e += NT) {                  // consecutive threads, consecutive slots
            const int unit = div_b(e), b = e - unit * B;
            const int t = unit >> 4, l = 16 * ((unit >> 2) & 3) + b, rr = unit & 3;
            float h = 0.f, u = 0.f;
#pragma unroll
            for (int w8 = 0; w8 < NW; ++w8) {
                h += smem[(((w8 * NTL + t) * 2 + 0) * 64 + l) * 4 + rr];
                u += smem[(((w8 * NTL + t) * 2 + 1) * 64 + l) * 4 + rr];
            }
            cf::team::put(xr, a.xg + (size_t)(r0 + unit) * B + b, activate(h, a.act) * u, x.stamp);
        }
        lds_barrier();
    }
    FFN_STAMP(2);           // g published

    // ---- stage B set-up: the first rows of W3 are requested before g is waited for
    const int CW = a.CW, c0 = ci * CW, CWi = max(0, min(CW, D - c0));
    const int ncg = (CW + 127) / 128, ncgp = ncg <= 1 ? 1 : ncg <= 2 ? 2 : ncg <= 4 ? 4 : 8, KSPL = NW / ncgp;
    const int cg = wv % ncgp, ks = wv / ncgp;
    const int nst = (nR + 31) / 32;
    const int colp = 128 * cg + 8 * c;                            // first of this lane's eight columns in the slice
    const bool colok = colp < CWi;
    const uint32_t base3 = (uint32_t)(8 * g) * (uint32_t)D * 2u + (uint32_t)(c0 + colp) * 2u;
    auto request3 = [&](h8(&wr)[8], int s) {
        const uint32_t soff = s < nst ? (uint32_t)((size_t)(R0 + 32 * s) * D * 2) : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool live = colok && s < nst && 32 * s + 8 * g + u < nR;
            wr[u] = W3.ld(live ? base3 + (uint32_t)u * (uint32_t)D * 2u : kNoLoad, soff);
        }
    };
    h8 ra[8], rb[8];

    // ---- G: g of the slice into LDS as fp16 pairs [16][nRp] (zero past the batch and past the slice)
    _Float16 *ghi = reinterpret_cast<_Float16 *>(smem), *glo = ghi + 16 * a.nRp;
    for (int i = tid; i < 4 * a.nRp; i += NT) reinterpret_cast<uint4 *>(smem)[i] = uint4{0u, 0u, 0u, 0u};
    lds_barrier();
    // The first two steps of W3 go out before the polls: the polls return behind them, about when g has arrived anyway
    // (all polls of a thread in one round; with two more steps ahead, or with three poll rounds, this order lost).
    request3(ra, ks);
    request3(rb, ks + KSPL);
    constexpr int NPG = 24;                                       // polls of a thread in one round trip
    for (int i0 = 0; i0 < nR * B; i0 += NPG * NT) {
        const int cntv = min(NPG * NT, nR * B - i0);
        pair_t q[NPG];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < NPG; ++k) {
                q[k] = pair_t{0u, x.stamp};
                if (NT * k < cntv) q[k] = cf::team::peek(xr, a.xg + (size_t)R0 * B + i0 + min(tid + NT * k, cntv - 1));   // (uniform)
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < NPG; ++k) ok &= q[k].y == x.stamp;
            if (ok || cf::team::gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < NPG; ++k) {
            const int i = i0 + tid + NT * k;
            if (tid + NT * k < cntv) {
                const int unit = div_b(i), b = i - unit * B;
                const float v = __builtin_bit_cast(float, q[k].x);
                const _Float16 hi = (_Float16)v;
                ghi[b * a.nRp + unit] = hi;
                glo[b * a.nRp + unit] = (_Float16)(v - (float)hi);
            }
        }
    }
    lds_barrier();
    FFN_STAMP(3);           // g of the slice arrived

    // ---- stage B
    f32x4 o[8];                                                   // [jj][rr]: batch row 4 g + rr, column colp + jj
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) o[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto consume3 = [&](const h8(&wr)[8], int s) {
        const int at = c * a.nRp + 32 * min(s, nst - 1) + 8 * g;  // (a step past the end has zero weights)
        const h8 ah = *reinterpret_cast<const h8 *>(ghi + at), al = *reinterpret_cast<const h8 *>(glo + at);
        h8 f8[8];
        transpose8(wr, f8);
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            o[jj] = mfma16(ah, f8[jj], o[jj]);
            o[jj] = mfma16(al, f8[jj], o[jj]);
        }
    };
    for (int s = ks; s < nst; s += 2 * KSPL) {                    // (uniform per wavefront; no barrier inside)
        consume3(ra, s);
        request3(ra, s + 2 * KSPL);
        consume3(rb, s + KSPL);
        request3(rb, s + 3 * KSPL);
    }
    FFN_STAMP(4);           // products of stage B done (this wavefront)
    lds_barrier();                                                // g is consumed: the sums of the wavefronts overlay it
    {
        const int CWp = 128 * ncgp;
        float *red = smem;                                        // [KSPL][16][CWp]
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            float *dst = red + (size_t)(ks * 16 + 4 * g + rr) * CWp + colp;
            *reinterpret_cast<float4 *>(dst) = make_float4(o[0][rr], o[1][rr], o[2][rr], o[3][rr]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(o[4][rr], o[5][rr], o[6][rr], o[7][rr]);
        }
        lds_barrier();
        for (int e = tid; e < B * CWi; e += NT) {
            const int b = e / CWi, col = e - b * CWi;
            float sum = 0.f;
            for (int k = 0; k < KSPL; ++k) sum += red[(size_t)(k * 16 + b) * CWp + col];
            cf::team::put(xr, a.xp + ((size_t)fi * B + b) * D + c0 + col, sum, x.stamp);
        }
    }

    FFN_STAMP(5);           // partial output published
    // ---- stage C: columns [c0 + fi cpf, + cpf) of slice ci, summed over the NF slices of hidden units in slice order
    {
        const int cpf = (CW + a.NF - 1) / a.NF;
        const int q0 = fi * cpf, nq = max(0, min(cpf, CWi - q0));
        if (tid < nq * B) {
            const int b = tid / nq, col = c0 + q0 + tid - b * nq;
            pair_t q[16];
            long long t0 = 0;
            for (;;) {
#pragma unroll
                for (int k = 0; k < 16; ++k) q[k] = cf::team::peek(xr, a.xp + ((size_t)min(k, a.NF - 1) * B + b) * D + col);
                __builtin_amdgcn_sched_barrier(0);
                bool ok = true;
#pragma unroll
                for (int k = 0; k < 16; ++k) ok &= q[k].y == x.stamp;
                if (ok || cf::team::gave_up(x, t0)) break;
            }
            float sum = 0.f;
#pragma unroll
            for (int k = 0; k < 16; ++k)
                if (k < a.NF) sum += __builtin_bit_cast(float, q[k].x);
            a.out[(size_t)b * D + col] = __builtin_bit_cast(uint16_t, (_Float16)sum);
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
    FFN_STAMP(6);
#if CF_STAMPS
    lds_barrier();
    if (tid < kFfnStamps && w < 256) g_ffn_ts[w * kFfnStamps + tid] = s_ts[tid];
#endif
}

using KernelFn = void (*)(const FfnArgs);
KernelFn pick(int bt, int d_model)
{
    if (d_model <= 4096) return bt == 1 ? fused_ffn<1, 1> : bt == 2 ? fused_ffn<2, 1> : fused_ffn<4, 1>;
    return bt == 1 ? fused_ffn<1, 2> : bt == 2 ? fused_ffn<2, 2> : fused_ffn<4, 2>;
}
int batch_tile(int b) { return b <= 1 ? 1 : b <= 2 ? 2 : 4; }
int row_tiles(int nrmax) { return (nrmax + 15) / 16; }
KernelFn pick_tiles(int nrmax)
{
    static const KernelFn fn[8] = {fused_ffn_tiles<1>, fused_ffn_tiles<2>, fused_ffn_tiles<3>, fused_ffn_tiles<4>,
                                   fused_ffn_tiles<5>, fused_ffn_tiles<6>, fused_ffn_tiles<7>, fused_ffn_tiles<8>};
    return fn[row_tiles(nrmax) - 1];
}

}  // namespace

struct cf_ffn_s {
    cf_ffn_config cfg;
    int W = 0, nrmax = 0;
    int NF = 0, CW = 0, nRp = 0;       // MFMA kernel (max_batch >= 2)
    size_t xg = 0, xp = 0, lds_tiles = 0;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    uint32_t *err = nullptr;
    unsigned long long *counters = nullptr;
    uint64_t *slots = nullptr;
    long long spin_ticks = 200000000LL;
    int last_hip = 0;
};

static size_t lds_bytes_of(const cf_ffn_config &c, int bt, int nrmax)
{
    const size_t nck = (c.d_model + kChunk - 1) / kChunk, dp = nck * kChunk;
    const size_t stages_ab = (size_t)bt * dp / 2 + 2 * (size_t)bt * nrmax * nck + (size_t)bt * nrmax;
    return (stages_ab > (size_t)(8 * NT) ? stages_ab : (size_t)(8 * NT)) * sizeof(float);       // the partial output on its way out: 4096 floats
}

extern "C" {

int cf_ffn_create(const cf_ffn_config *cfg, cf_ffn *out)
{
    if (!cfg || !out) return CF_EINVAL;
    *out = nullptr;
    const cf_ffn_config &c = *cfg;
    if (c.d_model < 8 || c.d_model % 8 || c.d_ff < 1 || c.max_batch < 1 ||
        (c.activation != CF_FFN_SILU && c.activation != CF_FFN_GELU))
        return CF_EINVAL;
    if (c.max_batch > kMaxBatch || c.d_model > 8192 || (unsigned long long)c.d_ff * c.d_model * 2 > 0x7fffffffull)
        return CF_EUNSUPPORTED;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return CF_EHIP;
    const int W = c.d_ff < cus ? c.d_ff : cus;
    const int nrmax = (c.d_ff + W - 1) / W;
    const int cpw = (c.d_model + W - 1) / W;
    const int vbatch = c.max_batch < kVectorBatch ? c.max_batch : kVectorBatch;
    if ((size_t)cpw * vbatch > (size_t)NT) return CF_EUNSUPPORTED;            // stage C: one thread per output value
    for (int bt = 1; bt <= kVectorBatch; bt *= 2) {
        if (bt / 2 >= c.max_batch) break;
        const size_t lds = lds_bytes_of(c, bt, nrmax);
        if (lds > 160 * 1024 - 256) return CF_EUNSUPPORTED;
        int per_cu = 0;
        if ((lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void *>(pick(bt, c.d_model)),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(pick(bt, c.d_model)), NT, lds) != hipSuccess ||
            per_cu < 1)
            return CF_EUNSUPPORTED;                                             // all workgroups resident, one per compute unit
    }
    // the MFMA kernel: 16 column slices times W / 16 slices of hidden units
    const int NF = W / kNC, CW = ((c.d_model + kNC - 1) / kNC + 7) / 8 * 8, nRp = (kNC * nrmax + 31) / 32 * 32 + 8;     // (+ 8: the rows of g in LDS start in different banks)
    size_t lds_tiles = 0;
    const bool tiles_fit = W % kNC == 0 && nrmax <= 128 && (size_t)((CW + (NF > 0 ? NF : 1) - 1) / (NF > 0 ? NF : 1)) * c.max_batch <= (size_t)NT;
    if (c.max_batch > kVectorBatch && !tiles_fit) return CF_EUNSUPPORTED;
    if (c.max_batch >= kTilesFrom && tiles_fit) {
        const size_t part = (size_t)row_tiles(nrmax) * 16384, gbytes = 64 * (size_t)nRp, red = 65536;
        lds_tiles = part > gbytes ? part : gbytes;
        lds_tiles = lds_tiles > red ? lds_tiles : red;
        const size_t staging = (size_t)NW * 16 * kStageRow * sizeof(uint16_t);
        lds_tiles = lds_tiles > staging ? lds_tiles : staging;
        int per_cu = 0;
        if (lds_tiles > 160 * 1024 - 256 ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(pick_tiles(nrmax)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_tiles) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(pick_tiles(nrmax)), NT,
                                                         lds_tiles) != hipSuccess ||
            per_cu < 1)
            return CF_EUNSUPPORTED;
    }
    cf_ffn t = new (std::nothrow) cf_ffn_s();
    if (!t) return CF_ENOMEM;
    t->cfg = c;
    t->W = W;
    t->nrmax = nrmax;
    t->NF = NF, t->CW = CW, t->nRp = nRp, t->lds_tiles = lds_tiles;
    t->xg = 0;
    t->xp = (size_t)c.d_ff * c.max_batch;
    const size_t head = (256 + (size_t)W * kCounterStride * sizeof(unsigned long long) + 255) / 256 * 256;
    const size_t vb = c.max_batch < kVectorBatch ? c.max_batch : kVectorBatch;
    const size_t slots_vector = (size_t)W * vb * c.d_model;                   // the two kernels use the same slots, never together
    const size_t slots_tiles = lds_tiles ? t->xp + (size_t)NF * c.max_batch * c.d_model : 0;
    const size_t slot_bytes = (slots_vector > slots_tiles ? slots_vector : slots_tiles) * sizeof(uint64_t);
    if (slot_bytes > 0xfffffff0ull) {
        delete t;
        return CF_EUNSUPPORTED;
    }
    t->ws_bytes = head + slot_bytes;
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
    t->slots = reinterpret_cast<uint64_t *>(t->ws + head);
    *out = t;
    return CF_OK;
}

int cf_ffn_destroy(cf_ffn t)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipFree(t->ws);
    delete t;
    return e == hipSuccess ? CF_OK : CF_EHIP;
}

int cf_ffn_decode(cf_ffn t, int32_t batch, const void *z, const void *W1, const void *W2, const void *W3, void *out,
                  void *stream)
{
    if (!t || !z || !W1 || !W2 || !W3 || !out) return CF_EINVAL;
    if (batch < 1 || batch > t->cfg.max_batch) return CF_EINVAL;
    const void *ptrs[] = {z, W1, W2, W3, out};
    for (const void *p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) & 15u) return CF_EINVAL;
    FfnArgs a;
    std::memset(&a, 0, sizeof a);
    a.z = static_cast<const uint16_t *>(z);
    a.w1 = static_cast<const uint16_t *>(W1);
    a.w2 = static_cast<const uint16_t *>(W2);
    a.w3 = static_cast<const uint16_t *>(W3);
    a.out = static_cast<uint16_t *>(out);
    a.slots = t->slots;
    a.counters = t->counters;
    a.err = t->err;
    a.D = t->cfg.d_model, a.F = t->cfg.d_ff, a.B = batch, a.W = t->W, a.act = t->cfg.activation;
    a.nrmax = t->nrmax;
    a.spin_ticks = t->spin_ticks;
    if (batch >= kTilesFrom && t->lds_tiles) {
        a.xg = t->xg, a.xp = t->xp, a.NF = t->NF, a.CW = t->CW, a.nRp = t->nRp;
        hipLaunchKernelGGL(pick_tiles(t->nrmax), dim3(t->W), dim3(NT), t->lds_tiles, static_cast<hipStream_t>(stream), a);
    } else {
        const int bt = batch_tile(batch);
        hipLaunchKernelGGL(pick(bt, t->cfg.d_model), dim3(t->W), dim3(NT), lds_bytes_of(t->cfg, bt, t->nrmax),
                           static_cast<hipStream_t>(stream), a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    return CF_OK;
}

int cf_ffn_status(cf_ffn t, void *stream)
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

#if CF_STAMPS
// profiling library only: the stage stamps of the last launch of the MFMA kernel (host buffer of 256 * 16 64-bit words)
int cf_ffn_trace_read(void *host_dst)
{
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_ffn_ts), sizeof(unsigned long long) * 256 * kFfnStamps);
    return e == hipSuccess ? CF_OK : CF_EHIP;
}
#endif

int cf_ffn_set_spin_limit(cf_ffn t, int32_t spin_limit_us)
{
    if (!t || spin_limit_us < 0) return CF_EINVAL;
    t->spin_ticks = (long long)spin_limit_us * 100;
    return CF_OK;
}

int64_t cf_ffn_algorithmic_bytes(const cf_ffn_config *c, int32_t batch)
{
    if (!c) return 0;
    return 2 * (3 * (int64_t)c->d_ff * c->d_model + 2 * (int64_t)batch * c->d_model);
}

}  // extern "C"
