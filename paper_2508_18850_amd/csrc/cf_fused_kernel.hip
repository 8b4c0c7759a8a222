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
// Every workgroup counts the launches it has completed; the count gives the launch number.  All
// workgroups of the launch must be resident (checked on the host), since
// readers spin.  Spins are bounded: after spin_ticks a thread sets an error
// flag and goes on, so the kernel always ends.
#include "cf_params.h"
#include "cf_rope_device.h"

#include <cstddef>
#include <cstdlib>
#include <type_traits>

namespace cf {
namespace {

// CF_LAYER=1 compiles the kernel with the RMSNorm prologue, the residual epilogue and per-row positions
// (fused_decode_layer); without it none of that code is in the kernel (fused_decode_block).
#ifndef CF_LAYER
#define CF_LAYER 0
#endif
#if CF_LAYER
#define CF_KERNEL fused_decode_layer
#else
#define CF_KERNEL fused_decode_block
#endif
constexpr bool kLayer = CF_LAYER != 0;
constexpr int NT = kThreads;
constexpr int NW = kWaves;
constexpr float kNegBig = -1.0e30f;   // stands for "no score yet"; finite so that differences never give NaN
#ifndef CF_PREFETCH_NEXT_LAYER
#define CF_PREFETCH_NEXT_LAYER 1
#endif
constexpr bool kPrefetchNextLayer = CF_PREFETCH_NEXT_LAYER != 0;   // stack kernel: next layer's first weights during the tail

typedef _Float16 h8 __attribute__((ext_vector_type(8)));   // eight fp16 values = one 128-bit load
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A read-only tensor that is streamed once: raw buffer resource + 128-bit non-temporal loads.
// The address of a load is base + voff (per lane) + soff (wave-uniform), so no 64-bit
// address registers are needed per load; a lane with nothing to load passes kNoLoad,
// which is beyond the buffer's size: the hardware then skips the access and returns zeros.
constexpr uint32_t kNoLoad = 0x80000000u;
struct Stream {
    __amdgpu_buffer_rsrc_t r;
    __device__ __forceinline__ Stream(const void *base, uint32_t bytes)
        : r(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000)) {}
    __device__ __forceinline__ h8 ld(uint32_t voff, uint32_t soff) const
    {
        return __builtin_bit_cast(h8, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 2));
    }
};

__device__ __forceinline__ void unpack8(const h8 &u, float (&f)[8])
{
#pragma unroll
    for (int k = 0; k < 8; ++k) f[k] = (float)u[k];
}

// Batch tile 16 with head_dim 128: the two projections (Alg. 3 steps 2 and 8) are dense [16 x K] x [K x N]
// products and run on MFMA tiles (v_mfma_f32_16x16x32_f16: A is 16 x 32, B is 32 x 16, fp32 accumulators).
// Operand layout of that instruction: lane l holds, of A, row l % 16 and eight consecutive values of the
// contraction index for group l / 16; of B, column l % 16 and the same eight contraction values; of the
// result, column l % 16 and rows 4 * (l / 16) + 0..3.  The weights stay in the layout the batch-1 path
// streams (a lane loads eight COLUMNS of one row), so eight loaded rows are transposed inside the lane
// into eight operands of one column each (transpose8); the sixteen batch rows are the A operand.
template <int HD, int BT>
struct Mfma {
    static constexpr bool on = mfma_tiles(HD, BT);
};
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16(const h8 &a, const h8 &b, const f32x4 &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// w[u] = row u, eight adjacent columns  ->  f[c] = column c, rows 0..7 (a 8 x 8 transpose of 16-bit values
// inside one lane: one byte permute per result register)
__device__ __forceinline__ void transpose8(const h8 *w, h8 (&f)[8])
{
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) {
        u32x4 e, o;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = __builtin_bit_cast(u32x4, w[2 * d])[c2], hi = __builtin_bit_cast(u32x4, w[2 * d + 1])[c2];
            e[d] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);    // {lo.low half, hi.low half}
            o[d] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);    // {lo.high half, hi.high half}
        }
        f[2 * c2] = __builtin_bit_cast(h8, e);
        f[2 * c2 + 1] = __builtin_bit_cast(h8, o);
    }
}

// v = hi + lo with both parts fp16: the A operand of an MFMA product whose fp32 input must not lose bits
__device__ __forceinline__ void split_hi_lo(const float (&v)[8], h8 &hi, h8 &lo)
{
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        hi[k] = (_Float16)v[k];
        lo[k] = (_Float16)(v[k] - (float)hi[k]);
    }
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

// Workgroup barrier that orders LDS accesses only.  __syncthreads() would also wait for every
// outstanding global load of the wave (vmcnt(0)), which would drain the loads that are kept in
// flight across phases; nothing here passes data between the threads of a workgroup through
// global memory.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
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
//
// Scope: agent (sc1, through to memory), also for slots that only travel inside a team.  Keeping
// those in the L2 of the team's die (workgroup-scope loads and stores) was tried: the per-CU cache
// then serves the polled line and the reader never sees the new stamp.
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
        if (now - t0 >= (long long)p.spin_ticks) {            // a limit of 0 gives up at the first failed look
            __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        return false;
    }
};

// Sum of n stamped slots base, base+stride, ... in index order; spins until all are current.
// Loads go out eight at a time (indices past n repeat the last slot and are ignored) and are consumed
// only after all eight have been issued: written as one loop, each load was waited for on its own.
template <int C = 8>
__device__ __forceinline__ float ll_sum(const Params &p, const Xbuf &x, size_t base, size_t stride, int n,
                                        uint32_t stamp)
{
    Spin spin;
    for (;;) {
        float s = 0.f;
        bool ok = true;
        if (n == 1) {
            const u32x2 v = x.ld(base);
            ok = (v.y == stamp);
            s = __builtin_bit_cast(float, v.x);
        } else {
            for (int k0 = 0; k0 < n; k0 += C) {
                u32x2 v[C];
#pragma unroll
                for (int k = 0; k < C; ++k) v[k] = x.ld(base + (size_t)min(k0 + k, n - 1) * stride);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k = 0; k < C; ++k)
                    if (k0 + k < n) {
                        ok &= (v[k].y == stamp);
                        s += __builtin_bit_cast(float, v[k].x);
                    }
            }
        }
        if (ok || spin.expired(p)) return s;
    }
}

// Division by a plan constant: a shift when the host found a power of two (sh >= 0).  Integer division
// by a run-time value costs some thirty instructions, and a handful of them sat between the start of
// the kernel and its first weight load.
__device__ __forceinline__ int qdiv(int n, int d, int sh) { return sh >= 0 ? (n >> sh) : n / d; }
__device__ __forceinline__ int qmod(int n, int d, int sh) { return sh >= 0 ? (n & (d - 1)) : n % d; }

// First weight column of selector `sel` for a team: sel < G query heads, G = key, G+1 = value.
// Tokens cached for batch row b == index of the row's new token (b is uniform over the workgroup).
// Values outside 0 .. pos are clamped, so that a bad entry cannot make the kernel leave its buffers.
__device__ __forceinline__ int row_pos(const Params &p, int b)
{
    if (kLayer && p.row_pos) return min(max(__builtin_amdgcn_readfirstlane(p.row_pos[b]), 0), p.pos);
    return p.pos;
}

template <int HD, int G>
__device__ __forceinline__ int qkv_col0(const Params &p, int team, int sel)
{
    if (sel < G) return (team * G + sel) * HD;
    if (sel == G) return (p.nq + team) * HD;
    return (p.nq + p.nkv + team) * HD;
}

// The RoPE tables in LDS: [rows][HD] floats, per row HD/2 cosines then HD/2 sines of that row's position.
// One row (the common position) unless the rows of the batch have positions of their own.
template <int HD, int BT>
struct RopeRows {
    static constexpr int ROWS = kLayer ? BT : 1;                      // rows the LDS array has room for
    static constexpr int NE = (ROWS * (HD / 2) + NT - 1) / NT;        // table entries per thread
};

// ---------------------------------------------------------------------------
// Phase 1 (Alg. 3 step 2, split over the reduction dimension).  The member owns the
// row slice ks of W_qkv and, within it, the column blocks ("selectors") sel0, sel0+dsel,
// ... of the team: query heads first, then key / value.  All (selector, row batch)
// steps run as one software pipeline: the loads of step k+1 are issued before step k is
// consumed, also across selectors and across the partial-sum epilogues, and the loads
// of the NEXT phase (issue_next) are issued before the last step is consumed, so the
// memory pipe never drains.
// ---------------------------------------------------------------------------
// Per-phase time stamps (cf_debug_export what = 2) are compiled in only with -DCF_STAMPS=1: their
// `if (thread 0)` blocks cost a quarter of a microsecond per step.  A stamp goes to LDS and is copied to
// memory when the workgroup ends: a store to memory in the first microseconds of a kernel (the first
// version did that) holds up every load behind it for about 3 us and falsifies what it measures.
#ifndef CF_STAMPS
#define CF_STAMPS 0
#endif
#if CF_STAMPS
__shared__ unsigned long long s_ts[kStamps];
#define CF_STAMP(k)                                       \
    do {                                                  \
        if (threadIdx.x == 0) s_ts[k] = wall_clock64();   \
    } while (0)
#else
#define CF_STAMP(k)
#endif

// The launch stamp of layer `layer` of a launch whose first layer has count cnt0 (never 0, the value of a
// cleared slot: the low word plus the number of times it has wrapped).
__device__ __forceinline__ uint32_t stamp_of(unsigned long long cnt0, int layer)
{
    const unsigned long long cnt = cnt0 + (unsigned long long)layer;
    return (uint32_t)(cnt + (cnt >> 32));
}

// The two batches of weight rows that phase 1 keeps in flight, and the cursor of the next batch to load.  They live
// outside p1_all so that, in a stack of layers, the first two batches of the NEXT layer can be requested while the
// current layer still exchanges its last partial results (its memory pipe would idle otherwise).
template <int HD, int BT>
struct P1Cfg {
    static constexpr bool MF = Mfma<HD, BT>::on;
    static constexpr int U = MF ? 8 : (BT > 4 ? 2 : (BT == 4 ? 4 : 8));     // loads per thread and batch
};
// How many of the two batches a stack requests ahead for its next layer: what the registers of the variant allow
// (none with the 16-row tile, one where the attention or a second query head per KV head takes the room).
template <int HD, int G, int BT>
struct P1Ahead {
    static constexpr int n = !kPrefetchNextLayer || BT > 4 ? 0 : (G >= 2 && BT == 1 ? 1 : 2);
};
template <int HD, int BT>
struct P1Regs {
    h8 wa[P1Cfg<HD, BT>::U], wb[P1Cfg<HD, BT>::U];
    int si = 0, i0 = 0;
    uint32_t sbase = 0;
};

// `layer` > 0 (a stack of layers in one launch): the input rows are what the final reduction of the previous layer
// left in the slots xin (stamped fp32 values that are exact fp16 numbers), and cnt0 is known already.
// PART 0: the whole phase (`primed`: its first two batches are in flight already, requested by PART 1 and 2);
// PART 1 / 2: only request the first / second batch of this layer's weights into rg and return.
template <int HD, int G, int BT, bool STACK, int PART, class NextFn>
__device__ __forceinline__ uint32_t p1_all(const Params &p, const LayerPtrs &lp, int tid0, int team, int member, float *smem,
                                           float *rope, int layer, const uint64_t *xin, int n_layers,
                                           unsigned long long &cnt0, P1Regs<HD, BT> &rg, bool primed, NextFn &&issue_next)
{
    constexpr int LPR = HD / 8;
    constexpr int NG = NT / LPR;
    // loads per thread and batch: the 16-row batch tile keeps 128 accumulators per thread, and anything above two
    // loads per batch spills (measured on the 8B shape, batch 16: 202 us with 8, 181 with 4, 177 with 2, 182 with 1);
    // the 4-row tile is best with 4 (8B shape, batch 4: 55.1 us with 8, 53.6 with 4, 53.7 with 2)
    // With MFMA tiles (MF) a batch is eight rows per lane: one 32-row step of the contraction per wavefront.
    constexpr bool MF = P1Cfg<HD, BT>::MF;
    constexpr int U = P1Cfg<HD, BT>::U;
    constexpr int MAXI = BT == 1 ? 4 : (BT <= 4 ? 2 : 1);   // selectors whose wave partials are buffered in LDS
    const int tid = tid0, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const int kg = (tid & 63) >> 4;                         // MF: contraction group of the lane (rows 8 kg .. 8 kg + 7 of a step)
    const int lrow = 32 * wv + 8 * kg;                      // MF: first row of the lane inside a 256-row batch
    const int ks = qmod(member, p.KS, p.sh_ks);
    const int sel0 = qdiv(member, p.KS, p.sh_ks), dsel = p.DSEL;
    // slices with an even index (workgroups on the faster dies, see the workgroup mapping in the
    // kernel) are 2*RD rows longer than those with an odd index
    const int r0 = ks * p.RB + ((ks & 1) ? p.RD : 0);
    const int nrows = min(p.RB + ((ks & 1) ? -p.RD : p.RD), p.D - r0);   // > 0: the host never plans an empty slice
    const int iters = (nrows + NG - 1) / NG;
    const int nb = (iters + U - 1) / U;                     // load batches per selector
    const int nA = sel0 < G ? qdiv(G - sel0 + dsel - 1, dsel, p.sh_dsel) : 0;
    const int nB = sel0 < 2 ? qdiv(2 - sel0 + dsel - 1, dsel, p.sh_dsel) : 0;
    const int nsteps = (nA + nB) * nb;
    auto sel_of = [&](int si) { return si < nA ? sel0 + si * dsel : G + sel0 + (si - nA) * dsel; };
    float *xs = smem;                       // [BT][RPS]
    // MF: x as fp16 MFMA operands, [16][XS] halves (rows padded by 16 bytes: the sixteen lanes of an operand read
    // then fall into different banks), followed by a second array with the low parts of x * gamma (RMSNorm)
    const int XS = xs16_stride(p.RPS);
    _Float16 *xh = reinterpret_cast<_Float16 *>(smem), *xl = xh + 16 * XS;
    float *red = smem + (MF ? 16 * XS : BT * p.RPS);   // [MAXI][NW][BT][HD]
    const Xbuf x1(p.p1);
    const uint32_t blkb = (uint32_t)p.D * HD * 2 + kQkvBlockPad;          // packed: bytes from one block to the next
    const Stream W(lp.wqkv, (p.flags & kFlagPacked) ? (uint32_t)(p.nqkv / HD) * blkb : (uint32_t)((size_t)p.D * p.nqkv * 2));
    // row-major [D][Nqkv]: rows are Nqkv*2 bytes apart and a selector starts at column col0;
    // packed [Nqkv/HD][D][HD] (+ pad): rows are HD*2 bytes apart and a selector is one contiguous block
    const uint32_t rowb = (p.flags & kFlagPacked) ? (uint32_t)HD * 2 : (uint32_t)p.nqkv * 2;
    const uint32_t voff0 = (uint32_t)(MF ? lrow : grp) * rowb + lig * 16;

    // A step is (selector, batch of U row groups).  Steps are loaded and consumed strictly in order,
    // so each side keeps a cursor that is advanced incrementally: no divisions, and the address
    // of a load is one per-lane offset plus a wave-uniform offset that grows by a constant.
    const uint32_t step_b = (uint32_t)NG * rowb;            // bytes between consecutive row groups
    struct Cursor {
        int si, i0;          // selector index, first row group of the batch
        uint32_t sbase;      // uniform byte offset of that row group's first row
    };
    auto blk_base = [&](int si) {
        const uint32_t col0 = (uint32_t)qkv_col0<HD, G>(p, team, sel_of(si));
        return (uint32_t)r0 * rowb + ((p.flags & kFlagPacked) ? (col0 / HD) * blkb : col0 * 2);
    };
    auto advance = [&](Cursor &c) {
        c.i0 += U;
        c.sbase += (uint32_t)U * step_b;
        if (c.i0 >= iters) {
            c.i0 = 0;
            ++c.si;
            c.sbase = blk_base(c.si);
        }
    };
    const int nsel = nA + nB;
    Cursor cc = {0, 0, nsteps > 0 ? blk_base(0) : 0u};      // next step to consume
    Cursor lc = cc;                                         // next step to load
    constexpr int AHEAD = STACK ? P1Ahead<HD, G, BT>::n : 0;
    if (PART == 2 || (PART == 0 && primed && AHEAD > 0)) lc = Cursor{rg.si, rg.i0, rg.sbase};
    // Every call issues exactly U load instructions on one straight-line path, also for a step past
    // the end (all lanes switched off through their offset).  The compiler derives each wait from
    // the number of loads issued after the one it needs, taking the smallest over all paths of the
    // control flow, so a branch around loads would make every later wait drain the queue.
    const int lim = nrows - (MF ? lrow : grp);              // row group i is inside the slice iff NG*i < lim (MF: row NG*i0 + u iff < lim)
    auto load = [&](h8(&w)[U], uint32_t voff) {
        const bool live = lc.si < nsel;
        const int g0 = live ? NG * lc.i0 : 0x40000000;      // uniform
#pragma unroll
        for (int u = 0; u < U; ++u)
            w[u] = W.ld((g0 + (MF ? u : NG * u)) < lim ? voff : kNoLoad, lc.sbase + (uint32_t)u * (MF ? rowb : step_b));
        if (live) advance(lc);
    };

    CF_STAMP(20);           // phase 1 set up
    // Kernel start: the first batch of weights goes out at once, then the small loads (this slice of
    // x, the RoPE frequencies), then the second batch.  Loads return in order: x arrives right behind
    // the first batch and is staged into LDS while the second one streams.
    h8(&wa)[U] = rg.wa;
    h8(&wb)[U] = rg.wb;
    if (PART != 0) {
        // (`primed` here means "there is a next layer"; without one the loads go out with every lane off: the
        // registers are written either way, so that what they held does not stay alive through the caller's loop)
        load(PART == 1 ? wa : wb, primed ? voff0 : kNoLoad);
        rg.si = lc.si;
        rg.i0 = lc.i0;
        rg.sbase = lc.sbase;
        return 0u;
    }
    // (a stack past its first layer has both batches in flight: the branch costs the other path, the first layer
    // of a stack, some exactness of its waits, nothing else)
    if (!(AHEAD >= 1 && primed)) load(wa, voff0);
    __builtin_amdgcn_sched_barrier(0);
    CF_STAMP(12);           // first weight batch issued
    constexpr int XR = BT + 1;                                    // x values per thread kept in registers
    const bool x_in_regs = BT * p.RPS <= XR * NT;
    // (all of them unconditional: a load inside a branch would be waited for at the branch's end)
    uint16_t xr[XR];
    u32x2 xs2[XR];                                                // layer > 0: the stamped slots of the same values
    bool xv[XR];
    const bool from_slots = STACK && layer > 0;
    const Xbuf xsl(xin ? (const void *)xin : (const void *)p.p1);
    // (the same number of loads on both paths, so that the waits behind this branch stay exact)
#pragma unroll
    for (int q = 0; q < XR; ++q) {
        const int i = tid + q * NT, b = BT == 1 ? 0 : i / p.RPS, r = i - b * p.RPS;
        xv[q] = x_in_regs && i < BT * p.RPS && b < p.B && r < nrows;
        xr[q] = 0;
        xs2[q] = u32x2{0u, 0u};
    }
    if (from_slots) {
#pragma unroll
        for (int q = 0; q < XR; ++q) {
            const int i = tid + q * NT, b = BT == 1 ? 0 : i / p.RPS, r = i - b * p.RPS;
            xs2[q] = xsl.ld(xv[q] ? (size_t)b * p.D + r0 + r : 0);
        }
    } else {
#pragma unroll
        for (int q = 0; q < XR; ++q) {
            const int i = tid + q * NT, b = BT == 1 ? 0 : i / p.RPS, r = i - b * p.RPS;
            xr[q] = p.x[xv[q] ? (size_t)b * p.D + r0 + r : 0];
        }
    }
    // RMSNorm in front of the projection (when a weight vector is given): the projection is linear, so the
    // weights gamma go into the staged slice of x and the factor 1/sqrt(mean(x^2) + eps) of a row goes into
    // the partial sums when they are stored.  Every workgroup takes the mean square from the whole row
    // (D*2 bytes: one or two 16-byte loads per thread, issued here with the other small loads).
    const bool norm = kLayer && p.gamma != nullptr;
    const uint16_t *gsrc = norm ? p.gamma : p.x;                  // any readable address when there is no weight
    uint16_t gr[XR];
#pragma unroll
    for (int q = 0; q < XR; ++q) gr[q] = 0;
    if (norm) {             // (a wait behind this branch counts the loads of the path without it: nothing drains)
#pragma unroll
        for (int q = 0; q < XR; ++q) {
            const int i = tid + q * NT, b = BT == 1 ? 0 : i / p.RPS, r = i - b * p.RPS;
            gr[q] = gsrc[xv[q] ? r0 + r : 0];
        }
    }
    float *nrm = red + MAXI * NW * BT * HD;                       // [NW][BT] sums of squares, one per wavefront and row
    constexpr int RG = BT < 4 ? BT : 4;                           // rows whose loads are in flight together
    const int d8 = p.D >> 3;                                      // 16-byte pieces of a row
    const uint4 *x4 = reinterpret_cast<const uint4 *>(p.x);
    uint4 xq[RG][2];                                              // rows b0 .. b0 + RG - 1; needs D <= 2 * 8 * NT
    bool ok[RG][2];
    auto load_rows = [&](int b0) {
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int c = tid + k * NT;
                ok[r][k] = norm && b0 + r < p.B && c < d8;
                xq[r][k] = x4[ok[r][k] ? (size_t)(b0 + r) * d8 + c : 0];
            }
    };
    auto square_rows = [&](int b0) {
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            float ss = 0.f;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                float f[8];
                unpack8(__builtin_bit_cast(h8, xq[r][k]), f);
                float t = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) t = fmaf(f[j], f[j], t);
                ss += ok[r][k] ? t : 0.f;
            }
            ss = wave_sum(ss);
            if ((tid & 63) == 0 && b0 + r < BT) nrm[wv * BT + b0 + r] = ss;
        }
    };
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            xq[r][k] = uint4{0u, 0u, 0u, 0u};
            ok[r][k] = false;
        }
    if (BT <= 4 && norm) load_rows(0);
    // for the RoPE tables, below: the frequency and the position of every table entry of this thread
    constexpr int NE = RopeRows<HD, BT>::NE;
    const bool own_pos = kLayer && p.row_pos != nullptr;
    const int32_t *psrc = own_pos ? p.row_pos : reinterpret_cast<const int32_t *>(p.x);   // any readable address
    int epos[NE];
#pragma unroll
    for (int k = 0; k < NE; ++k) {
        const int e = tid + k * NT, eb = e / (HD / 2);
        epos[k] = psrc[own_pos && eb < p.B ? eb : 0];
    }
    __builtin_amdgcn_sched_barrier(0);
    if (!(AHEAD >= 2 && primed)) load(wb, voff0);
    __builtin_amdgcn_sched_barrier(0);
    CF_STAMP(21);           // second weight batch issued
    if (BT > 4 && norm)     // large batches: four rows at a time, each group waits for its loads
        for (int b0 = 0; b0 < p.B; b0 += RG) {
            load_rows(b0);
            square_rows(b0);
        }
    // Launch number: every workgroup keeps, in a line of its own, the number of launches it has
    // completed; all workgroups of a launch hold the same count, so count + 1 stamps this launch
    // without any shared counter.  (One counter for all was read by 256 workgroups at once and
    // bumped by 256 atomics at the end: both are served one after the other, microseconds in all,
    // and the read sat at the head of the in-order return queue in front of the weights.)  The
    // value was written in an earlier launch, so a scalar load through the cache is good enough,
    // and it does not enter the vector memory queue at all.
    if (layer == 0) {
        unsigned long long launches;
        asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                     : "=s"(launches)
                     : "s"(p.done + (size_t)blockIdx.x * kCounterStride)
                     : "memory");
        cnt0 = launches + 1ull;
    }
    const uint32_t stamp = stamp_of(cnt0, layer);
    if (from_slots) {
        // The slots carry the stamp of the previous layer.  A workgroup whose projection nobody waits for (no
        // column block of its own) may arrive here after its sources have moved on and stamped newer values:
        // any stamp from the previous layer's up to the last layer's of this launch is taken.
        const uint32_t want = stamp_of(cnt0, layer - 1);
        Spin spin;
        for (;;) {
            bool ok = true;
#pragma unroll
            for (int q = 0; q < XR; ++q) ok &= !xv[q] | ((uint32_t)(xs2[q].y - want) <= (uint32_t)n_layers);
            if (ok || spin.expired(p)) break;
#pragma unroll
            for (int q = 0; q < XR; ++q) {
                const int i = tid + q * NT, b = BT == 1 ? 0 : i / p.RPS, r = i - b * p.RPS;
                xs2[q] = xsl.ld(xv[q] ? (size_t)b * p.D + r0 + r : 0);
            }
        }
    }
    // MF: the value goes to row b, column r of the operand array as fp16; without RMSNorm that is x itself,
    // with it the product x * gamma is kept as high + low part, so that nothing is rounded away
    auto stage = [&](int i, float v) {
        if constexpr (MF) {
            const int b = i / p.RPS, r = i - b * p.RPS;
            const _Float16 hi = (_Float16)v;
            xh[b * XS + r] = hi;
            if (norm) xl[b * XS + r] = (_Float16)(v - (float)hi);
        } else {
            xs[i] = v;
        }
    };
    if (x_in_regs) {
#pragma unroll
        for (int q = 0; q < XR; ++q) {
            const int i = tid + q * NT;
            const float xval = from_slots ? __builtin_bit_cast(float, xs2[q].x) : h2f(xr[q]);
            if (i < BT * p.RPS) stage(i, xv[q] ? xval * (norm ? h2f(gr[q]) : 1.f) : 0.f);
        }
    } else {
        const uint32_t want = stamp_of(cnt0, layer - 1);
        for (int i = tid; i < BT * p.RPS; i += NT) {
            const int b = i / p.RPS, r = i - b * p.RPS;
            const bool in = b < p.B && r < nrows;
            float xval = 0.f;
            if (in && from_slots) {
                Spin spin;
                for (;;) {
                    const u32x2 v = xsl.ld((size_t)b * p.D + r0 + r);
                    xval = __builtin_bit_cast(float, v.x);
                    if ((uint32_t)(v.y - want) <= (uint32_t)n_layers || spin.expired(p)) break;
                }
            } else if (in) {
                xval = h2f(p.x[(size_t)b * p.D + r0 + r]);
            }
            stage(i, in ? xval * (norm ? h2f(gsrc[r0 + r]) : 1.f) : 0.f);
        }
    }
    if constexpr (MF) {
        // columns RPS .. XS-1 of every row (an operand read may reach up to seven columns past the slice)
        const int nz = XS - p.RPS;
        for (int e = tid; e < 16 * nz; e += NT) {
            const int b = e / nz, r = p.RPS + (e - b * nz);
            xh[b * XS + r] = (_Float16)0.f;
            xl[b * XS + r] = (_Float16)0.f;
        }
    }
    if (BT <= 4 && norm) square_rows(0);
    // cos / sin of this position while the first weights are still on their way (the same for every layer of a stack)
#pragma unroll
    for (int k = 0; k < NE; ++k) {
        const int e = tid + k * NT, eb = e / (HD / 2), i = e % (HD / 2);
        if (!STACK && eb < (own_pos ? p.B : 1)) {      // (a stack builds the table once, in front of its layers)
            const int pos_e = own_pos ? min(max(epos[k], 0), p.pos) : p.pos;
            // (the frequency is computed here: a table in memory was one more cold page in front of the first wait)
            rope_cos_sin(pos_e, rope_inv_freq(i, HD, p.rope_log2_base), rope[eb * HD + i], rope[eb * HD + HD / 2 + i]);
        }
    }
    lds_barrier();
    CF_STAMP(2);            // x staged

    float acc[MF ? 1 : BT][8];              // FMA tiles: [batch row][column] of this lane's row group
    f32x4 acc4[MF ? 8 : 1];                 // MFMA tiles: [column][batch rows 4 * (lane / 16) + 0..3]
#pragma unroll
    for (int b = 0; b < (MF ? 1 : BT); ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
#pragma unroll
    for (int c = 0; c < (MF ? 8 : 1); ++c) acc4[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    int si_first = 0;                       // selector index of the first buffered item
    int nbuf = 0;
    auto flush = [&]() {
        lds_barrier();
        for (int e = tid; e < nbuf * BT * HD; e += NT) {
            const int it = e / (BT * HD), rem = e - it * (BT * HD);
            const int b = rem / HD, c = rem - b * HD;
            if (b < p.B) {
                float sum = 0.f, ss = 0.f;
#pragma unroll
                for (int w8 = 0; w8 < NW; ++w8) sum += red[((it * NW + w8) * BT + b) * HD + c];
                if (norm) {
#pragma unroll
                    for (int w8 = 0; w8 < NW; ++w8) ss += nrm[w8 * BT + b];
                    sum *= 1.0f / sqrtf(ss / (float)p.D + p.eps);
                }
                x1.st(((size_t)ks * p.B + b) * p.nqkv + qkv_col0<HD, G>(p, team, sel_of(si_first + it)) + c, sum,
                      stamp);
            }
        }
        lds_barrier();
        nbuf = 0;
    };
    auto consume = [&](const h8(&w)[U]) {
        const int i0 = cc.i0;
        if constexpr (MF) {
            // one step of 32 rows: operand A = x[batch row lane % 16][rows of this lane's group], operands B =
            // the eight columns of this lane.  Rows past the slice: their weights are zero (loads switched off)
            // and x is zero up to column XS; a group that starts past the slice reads nothing.
            const int r = NG * i0 + lrow;
            const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
            const int xo = (tid & 15) * XS + min(r, XS - 8);
            const h8 ah = r < nrows ? *reinterpret_cast<const h8 *>(xh + xo) : zero;
            h8 f[8];
            transpose8(w, f);
#pragma unroll
            for (int c = 0; c < 8; ++c) acc4[c] = mfma16(ah, f[c], acc4[c]);
            if (norm) {
                const h8 al = r < nrows ? *reinterpret_cast<const h8 *>(xl + xo) : zero;
#pragma unroll
                for (int c = 0; c < 8; ++c) acc4[c] = mfma16(al, f[c], acc4[c]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // a row past the slice has zero weights (its load was switched off) and any finite x
                const int r = min(grp + NG * (i0 + u), p.RPS - 1);
                float f[8];
                unpack8(w[u], f);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float xv = xs[b * p.RPS + r];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(xv, f[j], acc[b][j]);
                }
            }
        }
    };
    auto finish = [&]() {         // epilogue of the step just consumed, then move the cursor on
        const int si = cc.si, i0 = cc.i0;
        if (si >= nsel) return;                     // padding step: nothing was loaded
        advance(cc);
        if (i0 + U < iters) return;
        if constexpr (MF) {
            // last batch of this selector: the MFMA has already added the four row groups of the wavefront;
            // the lane holds eight adjacent columns of batch rows 4 * kg + 0..3
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float *dst = red + ((nbuf * NW + wv) * BT + 4 * kg + r) * HD + lig * 8;
                *reinterpret_cast<f32x4 *>(dst) = f32x4{acc4[0][r], acc4[1][r], acc4[2][r], acc4[3][r]};
                *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{acc4[4][r], acc4[5][r], acc4[6][r], acc4[7][r]};
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) acc4[c] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (nbuf == 0) si_first = si;
            if (++nbuf == MAXI) flush();
        } else {
            // last batch of this selector: row groups of a wavefront by shuffles; the wavefronts
            // are added in flush(), in a fixed order
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
            for (int b = 0; b < BT; ++b)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
            if (nbuf == 0) si_first = si;           // buffered items are consecutive selectors
            // (flushing as soon as the q heads are done, so that q leaves early, was measured: the two extra
            // barriers in the middle of the stream cost more than the early q gains)
            if (++nbuf == MAXI) flush();
        }
    };

    // Two steps are in flight at the top of every iteration.  The step count is padded to an even
    // number >= 2 (a padding step loads nothing and adds zeros), so that the loop body and the
    // tail are straight-line code with a fixed number of loads.  The scheduling barriers keep the
    // reload of a register batch behind its last use, so the batch stays in the same registers
    // (no branch may sit between consume() and the barrier: the multiply-adds would sink past it).
    const int nsteps2 = max(2, (nsteps + 1) & ~1);
    // the reload of a register batch must follow its last use, or the compiler keeps old and new
    // batch in different registers and copies them (after a full drain) at the end of every
    // iteration: the load offset is made to depend on the accumulators the batch was folded into
    auto after_consume = [&]() {
        uint32_t v = voff0;
        if constexpr (MF) {
#pragma unroll
            for (int c = 0; c < 8; ++c) asm volatile("" : "+v"(v) : "v"(acc4[c]));
        } else {
#pragma unroll
            for (int b = 0; b < BT; ++b)
                asm volatile("" : "+v"(v) : "v"(acc[b][0]), "v"(acc[b][1]), "v"(acc[b][2]), "v"(acc[b][3]),
                             "v"(acc[b][4]), "v"(acc[b][5]), "v"(acc[b][6]), "v"(acc[b][7]));
        }
        return v;
    };
    for (int k = 0; k + 2 < nsteps2; k += 2) {
        consume(wa);
        load(wa, after_consume());
        if (k == 0) CF_STAMP(16);       // first step consumed and reloaded
        finish();
        consume(wb);
        load(wb, after_consume());
        finish();
    }
    // tail: no step of this phase is left to issue, so the first loads of the next phase go out
    // before the last two steps are consumed.  (Not earlier: the partial-sum stores of the final
    // flush queue behind every load issued before them.)
    issue_next(0);
    consume(wa);
    finish();
    consume(wb);
    finish();
    if (nbuf) flush();
    return stamp;
}

// ---------------------------------------------------------------------------
// Phase 2: one (batch row, KV split) of the team's KV head, all G query heads
// (Alg. 3 steps 3-4; the new token is counted by the last split only).
// K/V rows are streamed in batches of U rows per row group, two batches in flight.
// ---------------------------------------------------------------------------
// The loads of the team's q partials are put in flight right behind this workgroup's own partial sums
// (at the end of phase 1, before the second part of the K/V prefetch) and checked when q is needed:
// where the other members were no later than this one, the sum costs no further round trip.  Covers
// value e = threadIdx.x and the first kEarly k-slices; anything else takes the polling path.
constexpr int kEarly = 16;
struct EarlyQ {
    u32x2 v[kEarly];
    bool issued = false;
    template <int HD, int G>
    __device__ __forceinline__ void issue(const Params &p, int tid0, int team, int b)
    {
        const Xbuf x1(p.p1);
        const int e = tid0;
        if (e < G * HD) {
            const int sel = e / HD, c = e - sel * HD;
            const size_t src = (size_t)b * p.nqkv + qkv_col0<HD, G>(p, team, sel) + c;
            // eight loads at a time on a straight-line path (slices past KS repeat the last one)
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = x1.ld(src + (size_t)min(k, p.KS - 1) * p.B * p.nqkv);
            if (p.KS > 8) {
#pragma unroll
                for (int k = 8; k < kEarly; ++k) v[k] = x1.ld(src + (size_t)min(k, p.KS - 1) * p.B * p.nqkv);
            }
        }
        issued = true;
    }
    // sum in slice order; false if a slot was not yet stamped or not covered
    __device__ __forceinline__ bool sum(const Params &p, uint32_t stamp, float &out) const
    {
        bool ok = issued && p.KS <= kEarly;
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < kEarly; ++k)
            if (k < p.KS) {
                ok &= (v[k].y == stamp);
                s += __builtin_bit_cast(float, v[k].x);
            }
        out = s;
        return ok;
    }
};

template <int G>
struct P2Cfg {
    static constexpr int U = G >= 4 ? 2 : 4;    // rows per row group in one batch of loads
    static constexpr int GP = G >= 4 ? 4 : G;   // query heads handled per pass over a batch
    static constexpr int NB = 2;                // batches in flight
};

// Attention on MFMA tiles (head_dim 128, four or more query heads per KV head): the G query heads that share
// a K/V row are the (zero-padded) 16-row edge of two dense products per 32 cached tokens,
//   S^T = K q^T   (A = K rows, B = q, contraction over head_dim in four steps of 32),
//   O  += P V     (A = P, B = V, contraction over the 32 tokens),
// in place of 16 G multiply-adds per loaded 16 bytes on the vector ALU, which is what bounds the plain loop
// from G = 4 on.  A wavefront owns every eighth tile of 32 tokens of the split.  K rows are loaded row by
// row (16 lanes x 16 bytes), put into a tile of LDS that only this wavefront uses and read back as A operands
// (lane l: token l % 16, eight of the 32 dimensions of a step); the result has token 4 (l / 16) + r of each
// 16-token half in register r of lane (head l % 16).  Those eight scores of a lane are, after the softmax,
// exactly the lane's A operand of the second product if contraction index (l / 16, e) stands for token
// 16 (e / 4) + 4 (l / 16) + e % 4, so V rows are loaded in that order and transposed in the lane
// (transpose8), and nothing moves between the two products.
template <int HD, int G>
struct AttnMfma {
    static constexpr bool on = HD == 128 && G >= 4;
    static constexpr int kTile = 32;                   // tokens per tile
    static constexpr int kRowH = HD + 8;               // halves per K row in LDS (16 bytes of padding: bank spread)
    static constexpr int kTileFloats = kTile * kRowH / 2;   // LDS floats per wavefront
};

template <int HD, int G>
struct KvBuf {
    static constexpr bool MA = AttnMfma<HD, G>::on;
    static constexpr int NBd = MA ? 1 : P2Cfg<G>::NB, Ud = MA ? 8 : P2Cfg<G>::U;
    h8 k[NBd][Ud], v[NBd][Ud];
};

template <int HD, int G>
struct P2Stream {
    static constexpr int LPR = HD / 8;
    static constexpr int NG = NT / LPR;
    static constexpr int U = P2Cfg<G>::U;
    static constexpr bool MA = AttnMfma<HD, G>::on;
    int t0, t1, iters, grp, pos, tid;
    uint32_t voff0;
    size_t head;
    Stream K, V;
    // `pos_b`: tokens cached for this batch row.  Rows >= pos_b are outside the buffers: they can never be
    // read.  An inactive stream (a workgroup without an attention item) has an empty row range: its
    // loads are issued with every lane off.  A row shorter than the longest one of the batch uses the
    // same split boundaries: its splits past pos_b are empty.
    __device__ __forceinline__ P2Stream(const Params &p, const LayerPtrs &lp, int tid0, int team, int b, int s, int pos_b,
                                        bool active = true)
        : pos(pos_b), tid(tid0), head(((size_t)b * p.nkv + team) * p.max_seq * HD), K(lp.kc + head, (uint32_t)pos_b * HD * 2),
          V(lp.vc + head, (uint32_t)pos_b * HD * 2)
    {
        const int lig = tid0 % LPR;
        grp = tid0 / LPR;
        t0 = active ? s * p.TPS + ((s & 1) ? p.TD : 0) : 0;         // even splits are 2*TD tokens longer
        t1 = active ? min(t0 + p.TPS + ((s & 1) ? -p.TD : p.TD), pos_b) : 0;
        iters = t1 > t0 ? (t1 - t0 + NG - 1) / NG : 0;
        voff0 = (uint32_t)(grp * HD + lig * 8) * 2;
        if (MA) iters = t1 > t0 ? (t1 - t0 + 32 * NW - 1) / (32 * NW) : 0;   // rounds of one 32-token tile per wavefront
    }
    // MFMA tiles: round `it` gives wavefront wv the tokens t0 + 32 (8 it + wv) + 0..31.  K: load u brings rows
    // 4 u + (lane / 16); V: load u brings rows 16 (u / 4) + 4 (lane / 16) + u % 4 (the order in which the scores
    // come out of the first product).  Eight load instructions each, lanes past the split switched off.
    __device__ __forceinline__ void load_k(h8 (&kr)[8], int it, uint32_t dep) const
    {
        const int wv = tid >> 6, rg = (tid & 63) >> 4, lig = tid & 15;
        const uint32_t voff = (uint32_t)((32 * wv + rg) * HD + lig * 8) * 2 + dep;
        const int tb = t0 + 32 * NW * it;                       // uniform
        const int lim = t1 - 32 * wv - rg;
#pragma unroll
        for (int u = 0; u < 8; ++u) kr[u] = K.ld(tb + 4 * u < lim ? voff : kNoLoad, (uint32_t)(tb + 4 * u) * HD * 2);
    }
    __device__ __forceinline__ void load_v(h8 (&vr)[8], int it, uint32_t dep) const
    {
        const int wv = tid >> 6, rg = (tid & 63) >> 4, lig = tid & 15;
        const uint32_t voff = (uint32_t)((32 * wv + 4 * rg) * HD + lig * 8) * 2 + dep;
        const int tb = t0 + 32 * NW * it;
        const int lim = t1 - 32 * wv - 4 * rg;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = 16 * (u >> 2) + (u & 3);
            vr[u] = V.ld(tb + r < lim ? voff : kNoLoad, (uint32_t)(tb + r) * HD * 2);
        }
    }
    // Always 2*U load instructions on a straight-line path (rows past the split: lane switched off),
    // so that the compiler's wait counts for earlier loads stay exact.
    __device__ __forceinline__ void load(h8 (&kr)[U], h8 (&vr)[U], int i0, uint32_t voff_on) const
    {
        const int lim = t1 - t0 - grp;                         // row NG*i + grp is inside the split iff NG*i < lim
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u;
            const uint32_t soff = (uint32_t)(t0 + NG * i) * HD * 2;   // first row of this step (uniform)
            const uint32_t voff = NG * i < lim ? voff_on : kNoLoad;
            kr[u] = K.ld(voff, soff);
            vr[u] = V.ld(voff, soff);
        }
    }
    // the first NB batches do not depend on q: they are put in flight before q is needed; part 0
    // (two batches) before the last steps of phase 1, part 1 (the rest) once phase 1 has stored
    // its partial sums (stores queue behind every load issued before them)
    __device__ __forceinline__ void prefetch(KvBuf<HD, G> &buf, int part) const
    {
        constexpr int NB = P2Cfg<G>::NB;
        if constexpr (MA) {
            if (part == 0)
                load_k(buf.k[0], 0, 0u);
            else
                load_v(buf.v[0], 0, 0u);
        } else {
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if ((j < 2) == (part == 0)) load(buf.k[j], buf.v[j], j * U, voff0);
        }
    }
};

template <int HD, int G, class TailFn>
__device__ __forceinline__ void p2_item(const Params &p, const LayerPtrs &lp, int tid0, int team, int b, int s, uint32_t stamp, bool first,
                                        const P2Stream<HD, G> &st, KvBuf<HD, G> &buf, const EarlyQ &eq, float *smem,
                                        const float *rope, TailFn &&issue_next)
{
    constexpr int LPR = HD / 8;
    constexpr int NG = NT / LPR;
    constexpr int U = P2Cfg<G>::U;
    constexpr int NB = P2Cfg<G>::NB;
    constexpr int PS = HD + kP2Stride;
    // (the thread index is made opaque per item: everything derived from it would otherwise be computed once in
    // front of the loop over the items, dozens of registers that are then spilled)
    int tid = tid0;
    if (AttnMfma<HD, G>::on) asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wv = tid >> 6, lig = tid % LPR, grp = tid / LPR;
    const bool last = (s == p.NS - 1);
    const Xbuf x1(p.p1), x2(p.p2);

    const float *cs = rope;                 // [HD/2] cos, filled at kernel start
    const float *sn = rope + HD / 2;        // [HD/2] sin
    float *qs = smem;                       // [G][HD]
    float *kn = qs + G * HD;                // [HD] rotated new key
    float *vn = kn + HD;                    // [HD] new value
    float *snew = vn + HD;                  // [8]  scores of the new token, log2 domain
    // Partials that are folded through LDS: one per wavefront (its row groups merged by shuffles first), or, for
    // groups of 8 heads, one per row group: there the shuffle merge of 10 values per head and step runs on
    // spilled registers and costs more than the larger fold (measured: 70B shape 111 -> 105 us; with 4 heads
    // per group the shuffle merge is the faster one, 32.1 against 35.1 us).
    constexpr int RGW = 64 / LPR;                               // row groups of a wavefront
    constexpr bool MA = AttnMfma<HD, G>::on;                    // both products on MFMA tiles: one partial per wavefront
    constexpr bool kFoldRowGroups = G >= 8 && !MA;
    constexpr int NPART = kFoldRowGroups ? NW * RGW : NW;
    float *redm = snew + 8;                 // [G][NPART]
    float *redl = redm + G * NPART;         // [G][NPART]
    float *redacc = redl + G * NPART;       // [G][NPART][HD]
    const int t0 = st.t0, t1 = st.t1, iters = st.iters;

    // ---- sum the projection partials of the team (the gather of Alg. 3 step 3): q heads, and for
    //      the last split also the new key and value; then RoPE on q and the key
    for (int e = tid; e < G * HD; e += NT) {
        const int sel = e / HD, c = e - sel * HD;
        const size_t src = (size_t)b * p.nqkv + qkv_col0<HD, G>(p, team, sel) + c;
        float v;
        if (!(first && e == tid && eq.sum(p, stamp, v)))
            v = ll_sum(p, x1, src, (size_t)p.B * p.nqkv, p.KS, stamp);
        qs[e] = v;
    }
    lds_barrier();
    for (int e = tid; e < G * (HD / 2); e += NT) {
        const int sel = e / (HD / 2), i = e - sel * (HD / 2);
        float *v = qs + sel * HD;
        const float lo = v[i], hi = v[i + HD / 2], c = cs[i], sgn = sn[i];
        v[i] = lo * c - hi * sgn;
        v[i + HD / 2] = hi * c + lo * sgn;
    }
    lds_barrier();
    // q fragments of this lane's 8 columns, pre-scaled by log2(e)/sqrt(d).  Up to GP heads stay in
    // registers; wider groups (G > GP) re-read them from LDS for every pass over a batch.
    constexpr int GP = P2Cfg<G>::GP;
    constexpr bool kQsScaled = !MA && G > GP;                   // qs is overwritten by the scaled q
    float qf[GP][8];
    if constexpr (MA) {
        constexpr int RH = AttnMfma<HD, G>::kRowH;
        _Float16 *kt = reinterpret_cast<_Float16 *>(redacc + G * NPART * HD) + wv * (AttnMfma<HD, G>::kTile * RH);
        const int hq = lane & 15, quad = lane >> 4;             // operand row / column of the lane, contraction group
        // B operands of K q^T: head hq (zero for hq >= G), the lane's eight of the 32 dimensions of each step,
        // pre-scaled by log2(e)/sqrt(d), as high + low fp16 parts so that q keeps its fp32 bits.  They are the
        // same for every wavefront and every tile: kept in LDS ([step][lane], high then low), not in registers.
        h8 *qop = reinterpret_cast<h8 *>(redacc + G * NPART * HD + NW * AttnMfma<HD, G>::kTileFloats);
        if (tid < 256) {
            const int s4 = tid >> 6;
            float a[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = hq < G ? qs[hq * HD + 32 * s4 + 8 * quad + e] * p.qk_scale_log2e : 0.f;
            h8 hi, lo;
            split_hi_lo(a, hi, lo);
            qop[tid] = hi;
            qop[256 + tid] = lo;
        }
        lds_barrier();
        CF_STAMP(14);           // q ready
        float m = kNegBig, l = 0.f;      // of head hq: running maximum (the same in the four lanes of a head), sum of this lane's tokens
        f32x4 O[8];                      // [column of the lane][heads 4 quad + 0..3]
#pragma unroll
        for (int c = 0; c < 8; ++c) O[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < st.iters; ++it) {
            // ---- K rows -> this wavefront's tile in LDS -> A operands; the registers are reloaded at once
#pragma unroll
            for (int u = 0; u < 8; ++u) *reinterpret_cast<h8 *>(kt + (4 * u + quad) * RH + lig * 8) = buf.k[0][u];
            __builtin_amdgcn_sched_barrier(0);
            st.load_k(buf.k[0], it + 1, 0u);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            f32x4 S[2];
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                S[T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    const h8 kf = *reinterpret_cast<const h8 *>(kt + (16 * T + hq) * RH + 32 * s4 + 8 * quad);
                    S[T] = mfma16(kf, qop[s4 * 64 + lane], S[T]);
                    S[T] = mfma16(kf, qop[256 + s4 * 64 + lane], S[T]);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // ---- online softmax of head hq over the lane's eight tokens 16 T + 4 quad + r
            const int tb = t0 + 32 * (NW * it + wv) + 4 * quad;
            float sc[8];
            bool ok[8];
            float mx = kNegBig;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ok[e] = tb + 16 * (e >> 2) + (e & 3) < t1;
                sc[e] = ok[e] ? S[e >> 2][e & 3] : kNegBig;
                mx = fmaxf(mx, sc[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mn = fmaxf(m, mx);
            if (__any(mn > m)) {
                // a maximum has grown (rare after the first tiles): rescale the sum and the accumulators; the lane
                // holds heads 4 quad + r, whose factors are in lanes 4 quad + r
                const float scale = __builtin_amdgcn_exp2f(m - mn);
                l *= scale;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float sr = __shfl(scale, 4 * quad + r);
#pragma unroll
                    for (int c = 0; c < 8; ++c) O[c][r] *= sr;
                }
                m = mn;
            }
            float pv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = ok[e] ? __builtin_amdgcn_exp2f(sc[e] - mn) : 0.f;
                l += pv[e];
            }
            h8 ph, pl;
            split_hi_lo(pv, ph, pl);
            // ---- O += P V
            h8 f[8];
            transpose8(buf.v[0], f);
            __builtin_amdgcn_sched_barrier(0);
            st.load_v(buf.v[0], it + 1, 0u);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                O[c] = mfma16(ph, f[c], O[c]);
                O[c] = mfma16(pl, f[c], O[c]);
            }
        }
        CF_STAMP(15);           // K/V consumed
        if (!last) issue_next(1);
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (hq < G && quad == 0) {
            redm[hq * NPART + wv] = m;
            redl[hq * NPART + wv] = l;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int g = 4 * quad + r;
            if (g < G) {
                float *dst = redacc + (g * NPART + wv) * HD + lig * 8;
                *reinterpret_cast<f32x4 *>(dst) = f32x4{O[0][r], O[1][r], O[2][r], O[3][r]};
                *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{O[4][r], O[5][r], O[6][r], O[7][r]};
            }
        }
    } else {
    if (G > GP) {
        for (int e = tid; e < G * HD; e += NT) qs[e] *= p.qk_scale_log2e;   // qs now holds the scaled q
        lds_barrier();
    } else {
#pragma unroll
        for (int g = 0; g < GP; ++g)
#pragma unroll
            for (int j = 0; j < 8; ++j) qf[g][j] = qs[g * HD + lig * 8 + j] * p.qk_scale_log2e;
    }
    CF_STAMP(14);           // q ready

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
#pragma unroll
        for (int g0 = 0; g0 < G; g0 += GP) {
            if (G > GP) {
#pragma unroll
                for (int g = 0; g < GP; ++g)
#pragma unroll
                    for (int j = 0; j < 8; ++j) qf[g][j] = qs[(g0 + g) * HD + lig * 8 + j];
            }
            float sc[GP][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[8];
                unpack8(kr[u], kf);
                const bool ok = (t0 + grp + NG * (i0 + u)) < t1;
#pragma unroll
                for (int g = 0; g < GP; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int j = 0; j < 8; ++j) d = fmaf(qf[g][j], kf[j], d);
                    d = row_sum<LPR>(d);
                    sc[g][u] = ok ? d : kNegBig;
                }
            }
            float pr[GP][U];
#pragma unroll
            for (int g = 0; g < GP; ++g) {
                float mn = m[g0 + g];
#pragma unroll
                for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[g][u]);
                const float scale = __builtin_amdgcn_exp2f(m[g0 + g] - mn);
                m[g0 + g] = mn;
                float ls = l[g0 + g] * scale;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool ok = (t0 + grp + NG * (i0 + u)) < t1;
                    pr[g][u] = ok ? __builtin_amdgcn_exp2f(sc[g][u] - mn) : 0.f;
                    ls += pr[g][u];
                }
                l[g0 + g] = ls;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[g0 + g][j] *= scale;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[8];
                unpack8(vr[u], vf);
#pragma unroll
                for (int g = 0; g < GP; ++g)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[g0 + g][j] = fmaf(pr[g][u], vf[j], acc[g0 + g][j]);
            }
        }
    };
    // NB batches are in flight at the top of every iteration.  Consume and reload are unconditional
    // (a batch past the split is all zeros with every row masked, its reload has every lane off), and
    // the reload offset is made to depend on the state the batch was folded into: the reload then
    // follows the last use of the registers it overwrites, so no copy and no drain is needed.
    auto after_consume = [&]() {
        uint32_t v = st.voff0;
#pragma unroll
        for (int g = 0; g < G; ++g)
            asm volatile("" : "+v"(v) : "v"(acc[g][0]), "v"(acc[g][1]), "v"(acc[g][2]), "v"(acc[g][3]),
                         "v"(acc[g][4]), "v"(acc[g][5]), "v"(acc[g][6]), "v"(acc[g][7]), "v"(l[g]), "v"(m[g]));
        return v;
    };
    for (int i0 = 0; i0 < iters; i0 += NB * U) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            consume(buf.k[j], buf.v[j], i0 + j * U);
            st.load(buf.k[j], buf.v[j], i0 + (j + NB) * U, after_consume());
        }
    }
    CF_STAMP(15);           // K/V consumed
    // Nothing of this phase is left to load.  Half of the next phase's first tile goes out now and
    // streams while the partial is merged and stored; the other half follows the stored partial.
    // (Not all of it now: the vector memory path of a compute unit returns in order, so the stamped
    // store and the next phase's polls wait for every bulk load issued before them.)  The member with
    // the last split first polls for the new token's key/value sums, for the same reason.
    if (!last) issue_next(1);
    if (kFoldRowGroups) {
        // ---- every row group leaves its partial in LDS
        const int part = wv * RGW + (lane / LPR);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (lig == 0) {
                redm[g * NPART + part] = m[g];
                redl[g * NPART + part] = l[g];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) redacc[(g * NPART + part) * HD + lig * 8 + j] = acc[g][j];
        }
    } else {
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
                    redm[g * NPART + wv] = m[g];
                    redl[g * NPART + wv] = l[g];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) redacc[(g * NPART + wv) * HD + lig * 8 + j] = acc[g][j];
            }
        }
    }
    }   // !MA
    CF_STAMP(8);            // row groups of the wavefront merged
    if (last) {
        // ---- the new token: sum its key/value partials (stored at the end of phase 1, long ago by
        //      now), rotate the key, append both (Sec. 2.1) and score the token
        for (int e = tid; e < 2 * HD; e += NT) {
            const int sel = G + e / HD, c = e % HD;
            const size_t src = (size_t)b * p.nqkv + qkv_col0<HD, G>(p, team, sel) + c;
            kn[e] = ll_sum(p, x1, src, (size_t)p.B * p.nqkv, p.KS, stamp);      // kn and vn are contiguous
        }
        issue_next(1);
        lds_barrier();
        if (tid < HD / 2) {
            const float lo = kn[tid], hi = kn[tid + HD / 2], c = cs[tid], sgn = sn[tid];
            kn[tid] = lo * c - hi * sgn;
            kn[tid + HD / 2] = hi * c + lo * sgn;
        }
        lds_barrier();
        const size_t row = st.head + (size_t)st.pos * HD;
        if (tid < HD)
            lp.kc[row + tid] = f2h(kn[tid]);
        else if (tid < 2 * HD)
            lp.vc[row + tid - HD] = f2h(vn[tid - HD]);
        for (int g = wv; g < G; g += NW) {
            float d = 0.f;
            for (int c = lane; c < HD; c += 64) d = fmaf(qs[g * HD + c], kn[c], d);
            d = wave_sum(d);
            if (lane == 0) snew[g] = kQsScaled ? d : d * p.qk_scale_log2e;
        }
        if (p.dbg_q)
            for (int e = tid; e < G * HD; e += NT)
                p.dbg_q[((size_t)b * p.nq + team * G) * HD + e] =
                    kQsScaled ? qs[e] / p.qk_scale_log2e : qs[e];
    }
    lds_barrier();
    CF_STAMP(9);            // new token handled, wavefronts in step
    // ---- the wavefronts and the new token -> one partial (m, l, acc) per query head
    for (int e = tid; e < G * HD; e += NT) {
        const int g = e / HD, c = e - g * HD;
        float M = last ? snew[g] : kNegBig;
#pragma unroll
        for (int w8 = 0; w8 < NPART; ++w8) M = fmaxf(M, redm[g * NPART + w8]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < NPART; ++w8) {
            const float f = __builtin_amdgcn_exp2f(redm[g * NPART + w8] - M);
            L = fmaf(redl[g * NPART + w8], f, L);
            A = fmaf(redacc[(g * NPART + w8) * HD + c], f, A);
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
    CF_STAMP(10);            // partial stored
    issue_next(2);       // the rest of the tile, behind the stored partial
    lds_barrier();
}

// ---------------------------------------------------------------------------
// Phase 3: merge the split-KV partials of head hq (Alg. 3 steps 5-7), multiply by
// rows [rs*HD/RS3, (rs+1)*HD/RS3) x columns [c3*CW3, (c3+1)*CW3) of that head's
// W_o block (step 8) and leave a per-head partial of the output.  The first
// 512-column chunk is loaded into registers before the attention result is needed.
// ---------------------------------------------------------------------------
template <int HD>
struct OutTile {
    static constexpr int MAXR = HD / NW;   // W_o rows per wavefront when a head is not split over rows
    h8 w[MAXR];
};

// part: 0 = first half of the tile's loads, 1 = second half, 2 = all
// MF (MFMA tiles): wavefront wv takes columns [128 (wv % 4), +128) of the chunk and rows [64 (wv / 4), +64) of the
// item; lane (l % 16, l / 16) loads eight adjacent columns of rows 32 s + 8 (l / 16) + 0..7 for the two steps s
// (the same lane layout as in the projection: eight rows are transposed in the lane into MFMA operands).
template <int HD, bool MF>
__device__ __forceinline__ void p3_load(const Params &p, const LayerPtrs &lp, int tid0, int hq, int c3, int rs, int ch, OutTile<HD> &t, int part = 2)
{
    const int lane = tid0 & 63, wv = tid0 >> 6;
    // row-major [nq*HD][D], or packed [nq][ceil(D/512)][HD][512] (one contiguous tile per head and chunk)
    const int NCH = (p.D + kOutChunk - 1) / kOutChunk;        // 512-column chunks of the output
    const Stream Wo(lp.wo, (p.flags & kFlagPacked) ? (uint32_t)((size_t)p.nq * NCH * HD * kOutChunk * 2)
                                   : (uint32_t)((size_t)p.nq * HD * p.D * 2));
    const int nrows = HD / p.RS3;
    const int cbase = c3 * p.CW3 + ch * kOutChunk;
    const uint32_t rowb = (p.flags & kFlagPacked) ? (uint32_t)kOutChunk * 2 : (uint32_t)p.D * 2;
    uint32_t voff = (cbase + lane * 8) < p.D ? (uint32_t)wv * rowb + lane * 16 : kNoLoad;
    // (opaque to the compiler: it otherwise computes the sixteen per-row offsets of all call sites once, far
    // ahead of the first one, and spills them)
    asm volatile("" : "+v"(voff));
    const uint32_t sbase = (p.flags & kFlagPacked) ? (uint32_t)((hq * NCH + cbase / kOutChunk) * HD + rs * nrows) * rowb
                                    : (uint32_t)(hq * HD + rs * nrows) * rowb + (uint32_t)cbase * 2;
    const int iters = nrows / NW;
    if constexpr (MF) {
        static_assert(OutTile<HD>::MAXR == 16, "two steps of eight rows per lane");
        const int lig = lane & 15, kg = lane >> 4, cb = wv & 3, kh = wv >> 2;
        uint32_t voffm = (cbase + 128 * cb + 8 * lig) < p.D ? (uint32_t)(8 * kg) * rowb + (uint32_t)(128 * cb + 8 * lig) * 2
                                                            : kNoLoad;
        asm volatile("" : "+v"(voffm));
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const bool mine = part == 2 || (part == 0) == (u < 8);
            const int row = 64 * kh + 32 * (u >> 3) + (u & 7);          // + 8 kg: the lane's row inside the item
            if (mine) t.w[u] = Wo.ld(row + 8 * kg < nrows ? voffm : kNoLoad, sbase + (uint32_t)row * rowb);
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < OutTile<HD>::MAXR; ++u) {
        const bool mine = part == 2 || (part == 0) == (u < OutTile<HD>::MAXR / 2);
        if (mine) t.w[u] = Wo.ld(u < iters ? voff : kNoLoad, sbase + (uint32_t)(NW * u) * rowb);
    }
}

template <int HD, int BT>
__device__ __forceinline__ void p3_item(const Params &p, const LayerPtrs &lp, int tid0, int hq, int c3, int rs, uint32_t stamp, OutTile<HD> &tile,
                                        bool prefetched, float *smem)
{
    constexpr int RB = BT < 4 ? BT : 4;
    constexpr int PS = HD + kP2Stride;
    // (the 16-row tile has no register to spare: the thread index is made opaque here, so that what this phase
    // derives from it is computed here and not kept from the start of the kernel)
    int tid = tid0;
    if (Mfma<HD, BT>::on) asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wv = tid >> 6;
    float *as = smem;                 // [BT][HD] merged, normalised attention output of head hq
    float *red = smem + BT * HD;      // [NW][RB][512]; also the (m, l, a) triples of the merge
    const Xbuf x2(p.p2), x3(p.p3);

    const int nrows = HD / p.RS3;
    const int rbeg = rs * nrows;
    const int iters = nrows / NW;
    const int slot = hq * p.RS3 + rs;
    const int nchunk = p.CW3 / kOutChunk;

    constexpr bool MF = Mfma<HD, BT>::on;
    if (!prefetched) p3_load<HD, MF>(p, lp, tid, hq, c3, rs, 0, tile);     // independent of the attention result

    {
        // ---- merge of the split-KV partials (Alg. 3 steps 5-7).  A pass handles up to NV * 512 values v = (batch row,
        //      column).  NV == 1: value v is handled by SG threads, each folding every SG-th split with a running
        //      maximum, MC splits per round trip; the SG (m, l, a) triples are then folded in split order through
        //      LDS.  NV == 4 (more values than threads): a thread folds all splits of four values, so that a batch of
        //      sixteen rows takes one pass (one round trip per MC splits) instead of four.  All loads of a round go
        //      out together.
        const int V = p.B * HD;
        auto run = [&](auto nv_c, auto mc_c) {
            constexpr int NV = decltype(nv_c)::value, MC = decltype(mc_c)::value;
            for (int v0 = 0; v0 < V; v0 += NT * NV) {
                const int cv = min(NT * NV, V - v0);
                const int SG = NV == 1 ? max(1, min(NT / cv, p.NS)) : 1;
                const int v = NV == 1 ? tid % cv : tid, sg = NV == 1 ? tid / cv : 0;
                if (sg < SG) {
                    float mt[NV], lt[NV], at[NV];
                    size_t src[NV];
                    int col[NV];
#pragma unroll
                    for (int n = 0; n < NV; ++n) {
                        mt[n] = kNegBig;
                        lt[n] = 0.f;
                        at[n] = 0.f;
                        const int vi = min(v0 + v + n * NT, V - 1);        // a value past the end repeats the last one
                        const int b = vi / HD;
                        col[n] = vi - b * HD;
                        src[n] = ((size_t)b * p.nq + hq) * p.NS * PS;
                    }
                    for (int sb = sg; sb < p.NS; sb += MC * SG) {
                        Spin spin;
                        float mm[NV][MC], ll[NV][MC], aa[NV][MC];
                        for (;;) {
                            bool ok = true;
#pragma unroll
                            for (int n = 0; n < NV; ++n)
#pragma unroll
                                for (int k = 0; k < MC; ++k) {
                                    const int s = sb + k * SG;
                                    const size_t o = src[n] + (size_t)(s < p.NS ? s : sb) * PS;
                                    const u32x2 vm = x2.ld(o), vl = x2.ld(o + 1), va = x2.ld(o + kP2Stride + col[n]);
                                    ok &= (vm.y == stamp) & (vl.y == stamp) & (va.y == stamp);
                                    mm[n][k] = __builtin_bit_cast(float, vm.x);
                                    ll[n][k] = __builtin_bit_cast(float, vl.x);
                                    aa[n][k] = __builtin_bit_cast(float, va.x);
                                }
                            if (ok || spin.expired(p)) break;
                        }
#pragma unroll
                        for (int n = 0; n < NV; ++n)
#pragma unroll
                            for (int k = 0; k < MC; ++k) {
                                if (sb + k * SG < p.NS) {
                                    const float mn = fmaxf(mt[n], mm[n][k]);
                                    const float fa = __builtin_amdgcn_exp2f(mt[n] - mn), fb = __builtin_amdgcn_exp2f(mm[n][k] - mn);
                                    lt[n] = lt[n] * fa + ll[n][k] * fb;
                                    at[n] = at[n] * fa + aa[n][k] * fb;
                                    mt[n] = mn;
                                }
                            }
                    }
                    if (NV == 1) {
                        red[(sg * cv + v) * 3 + 0] = mt[0];
                        red[(sg * cv + v) * 3 + 1] = lt[0];
                        red[(sg * cv + v) * 3 + 2] = at[0];
                    } else {
#pragma unroll
                        for (int n = 0; n < NV; ++n) {
                            const int vi = v0 + v + n * NT;
                            if (vi < V) {
                                const float a = at[n] / lt[n];
                                as[vi] = a;
                                if (p.dbg_attn && c3 == 0 && rs == 0) p.dbg_attn[((size_t)(vi / HD) * p.nq + hq) * HD + col[n]] = a;
                            }
                        }
                    }
                }
                lds_barrier();
                if (NV == 1) {
                    if (tid < cv) {
                        float mt = kNegBig, lt = 0.f, at = 0.f;
                        for (int k = 0; k < SG; ++k) {
                            const float mk = red[(k * cv + tid) * 3], lk = red[(k * cv + tid) * 3 + 1],
                                        ak = red[(k * cv + tid) * 3 + 2];
                            const float mn = fmaxf(mt, mk);
                            const float fa = __builtin_amdgcn_exp2f(mt - mn), fb = __builtin_amdgcn_exp2f(mk - mn);
                            lt = lt * fa + lk * fb;
                            at = at * fa + ak * fb;
                            mt = mn;
                        }
                        const float a = at / lt;
                        as[v0 + tid] = a;
                        if (p.dbg_attn && c3 == 0 && rs == 0) {
                            const int b = (v0 + tid) / HD, c = (v0 + tid) - b * HD;
                            p.dbg_attn[((size_t)b * p.nq + hq) * HD + c] = a;
                        }
                    }
                    lds_barrier();
                }
            }
        };
        using std::integral_constant;
        // (NV == 1 with eight splits per round trip was measured and is slower than four: a round is repeated as a
        // whole until all its stamps are current, and the partials of a team do not arrive together)
        if (V > NT)
            run(integral_constant<int, 4>{}, integral_constant<int, 2>{});
        else
            run(integral_constant<int, 1>{}, integral_constant<int, 4>{});
        for (int e = V + tid; e < BT * HD; e += NT) as[e] = 0.f;
        lds_barrier();
    }
    CF_STAMP(11);           // attention merged

    for (int ch = 0; ch < nchunk; ++ch) {
        const int cbase = c3 * p.CW3 + ch * kOutChunk;
        if (cbase >= p.D) break;
        if (ch > 0) p3_load<HD, MF>(p, lp, tid, hq, c3, rs, ch, tile);
        if constexpr (MF) {
            // [16 batch rows] x [rows of the item] x [128 columns of this wavefront]: two steps of 32 rows for each
            // half of the rows; the attention output is split into a high and a low fp16 part (two products), so
            // that it enters with all its fp32 bits
            const int lig = lane & 15, kg = lane >> 4, cb = wv & 3, kh = wv >> 2;
            f32x4 acc4[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc4[c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sstep = 0; sstep < 2; ++sstep) {
                const int row = 64 * kh + 32 * sstep + 8 * kg;          // first of the lane's eight rows
                float a[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = row < nrows ? as[(lane & 15) * HD + rbeg + row + e] : 0.f;
                h8 ahi, alo, f[8];
                split_hi_lo(a, ahi, alo);
                transpose8(&tile.w[8 * sstep], f);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    acc4[c] = mfma16(ahi, f[c], acc4[c]);
                    acc4[c] = mfma16(alo, f[c], acc4[c]);
                }
            }
            // the two halves of the rows -> one partial row per batch row
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float *dst = red + ((kh * 16 + 4 * kg + r) * kOutChunk) + 128 * cb + 8 * lig;
                *reinterpret_cast<f32x4 *>(dst) = f32x4{acc4[0][r], acc4[1][r], acc4[2][r], acc4[3][r]};
                *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{acc4[4][r], acc4[5][r], acc4[6][r], acc4[7][r]};
            }
            lds_barrier();
            for (int e = tid; e < 16 * kOutChunk; e += NT) {
                const int b = e / kOutChunk, cc = e - b * kOutChunk;
                if (b < p.B && cbase + cc < p.D)
                    x3.st(((size_t)slot * p.B + b) * p.D + cbase + cc, red[e] + red[16 * kOutChunk + e], stamp);
            }
            CF_STAMP(18);   // output partial stored
            lds_barrier();
            continue;
        }
        float acc[BT][8];
#pragma unroll
        for (int b = 0; b < BT; ++b)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[b][j] = 0.f;
        if (BT <= 4 && nchunk == 1) {
            // straight-line code (a branch per row would serialise the LDS reads): a row past the item
            // has a zero tile entry, its load was switched off, so it may be multiplied by any finite value
#pragma unroll
            for (int u = 0; u < OutTile<HD>::MAXR; ++u) {
                const int r = rbeg + wv + NW * min(u, iters - 1);
                float f[8];
                unpack8(tile.w[u], f);
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    const float av = as[b * HD + r];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[b][j] = fmaf(av, f[j], acc[b][j]);
                }
            }
        } else {
            // the 16-row batch tile has no registers to spare for reads hoisted across rows; with several
            // chunks per item the tile was loaded just now, and row-by-row waits overlap its arrival
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
        }
        // wavefronts -> one partial row per batch row, RB batch rows at a time
#pragma unroll
        for (int bb = 0; bb < BT; bb += RB) {
#pragma unroll
            for (int b = 0; b < RB; ++b)
#pragma unroll
                for (int j = 0; j < 8; ++j) red[(wv * RB + b) * kOutChunk + lane * 8 + j] = acc[bb + b][j];
            lds_barrier();
            for (int e = tid; e < RB * kOutChunk; e += NT) {
                const int b = e / kOutChunk, cc = e - b * kOutChunk;
                if (bb + b < p.B && cbase + cc < p.D) {
                    float sum = 0.f;
#pragma unroll
                    for (int w8 = 0; w8 < NW; ++w8) sum += red[(w8 * RB + b) * kOutChunk + cc];
                    x3.st(((size_t)slot * p.B + bb + b) * p.D + cbase + cc, sum, stamp);
                }
            }
            CF_STAMP(18);   // output partial stored
            lds_barrier();
        }
    }
}

// ---------------------------------------------------------------------------
// Phase 4: every workgroup owns ceil(D/W) output columns and adds the per-head
// partials of those columns in slot order (the cross-head reduction that the paper
// does with atomicAdd), then writes fp16.
// ---------------------------------------------------------------------------
// The residual input of output value v0 + threadIdx.x of this workgroup (0 when there is none).
__device__ __forceinline__ uint16_t residual_input(const Params &p, int tid0, int v0)
{
    const int cpw = (p.D + p.W - 1) / p.W;
    const int c0 = blockIdx.x * cpw;
    const int ncol = min(cpw, p.D - c0);
    const int i = v0 + tid0;
    uint16_t r = 0;
    if (kLayer && (p.flags & kFlagResidual) && ncol > 0 && i < ncol * p.B) {
        const int b = i / ncol, c = i - b * ncol;
        r = p.x[(size_t)b * p.D + c0 + c];
    }
    return r;
}

// xout != null (a layer of a stack that is not the last): the result, rounded to fp16 as `out` would hold it, goes to
// the slots the next layer's projection reads its input from, not to `out`.
template <class HookFn>
__device__ __forceinline__ void final_reduce(const Params &p, int tid0, uint32_t stamp, float *smem, uint64_t *xout, HookFn &&after_polls)
{
    const int tid = tid0;
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
        // the residual input of the value this thread writes below (threads tid < cb have v == tid), on its
        // way while the partials are polled.  (Fetching it before phase 3 was tried: a load inside a branch
        // there makes every later wait for the output-projection tile drain the queue.)
        const uint16_t xres = residual_input(p, tid0, v0);
        if (s0 < spt) {
            const int n = (nslots - s0 + spt - 1) / spt;
            const size_t base = (size_t)s0 * p.B * p.D + (size_t)b * p.D + c0 + c, stride = (size_t)spt * p.B * p.D;
            // (more than eight slots per thread: sixteen polls in flight, one round trip instead of two)
            smem[s0 * cb + v] = nslots > 8 * spt ? ll_sum<16>(p, x3, base, stride, n, stamp) : ll_sum<8>(p, x3, base, stride, n, stamp);
        }
        CF_STAMP(19);           // head partials arrived
        lds_barrier();
        if (v0 == 0) after_polls();
        if (tid < cb) {
            float sum = kLayer && (p.flags & kFlagResidual) ? h2f(xres) : 0.f;
            for (int k = 0; k < spt; ++k) sum += smem[k * cb + tid];
            if (xout)
                Xbuf(xout).st((size_t)b * p.D + c0 + c, h2f(f2h(sum)), stamp);
            else
                p.out[(size_t)b * p.D + c0 + c] = f2h(sum);
        }
        lds_barrier();
    }
}

// One launch = n_layers decode steps in a row (1 for the plain entry points).  Layer l > 0 takes its weights and
// caches from tab[l] and its input from the slots xslots, where the final reduction of layer l - 1 left its result;
// the last layer writes `out`.  Nothing separates the layers but those slots: a workgroup goes on as soon as the
// rows of the input it needs have arrived.  The exchange areas need no second set: a workgroup can post values of
// layer l + 1 only after it has taken in that layer's input, which exists only when every workgroup has finished
// reading what layer l exchanged.
template <int HD, int G, int BT, bool STACK>
__device__ __forceinline__ void decode_steps(const Params &p0, const LayerPtrs *tab, int n_layers_in, uint64_t *xslots)
{
    const int n_layers = STACK ? n_layers_in : 1;
    extern __shared__ __align__(16) float smem[];
    {
        // The compiler loads each kernel argument shortly before its first use: several dependent
        // round trips to cold memory in a row at the start of every launch.  One word of every 64-byte
        // line of the argument block is read here, all at once, so the later reads hit the scalar cache.
        static_assert(sizeof(Params) == 256, "one load per 64-byte line of the argument block below");
        auto ka = __builtin_amdgcn_kernarg_segment_ptr();
        uint32_t t0, t1, t2, t3;
        asm volatile("s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %4, 0x40\n\ts_load_dword %2, %4, 0x80\n\t"
                     "s_load_dword %3, %4, 0xc0\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3)
                     : "s"(ka));
    }
    __shared__ float s_rope[RopeRows<HD, BT>::ROWS * HD];    // cos / sin of the RoPE angles, per row if the rows differ
    const int tid = threadIdx.x;
    // Workgroup w runs on die (XCD) w % 8, and the odd dies get about a tenth less memory
    // bandwidth than the even ones.  With pairmap a team sits on one pair of dies, members with an
    // even index on the even die: those take the longer slices and splits.
#if CF_STAMPS
    if (tid < kStamps) s_ts[tid] = 0;       // same wavefront as thread 0: ordered before its stamps
#endif
    CF_STAMP(0);
#if CF_STAMPS
    if (tid == 0)   // where this workgroup runs: XCC id and the HW_ID register (CU, SE ...)
        s_ts[7] = ((unsigned long long)__builtin_amdgcn_s_getreg(63508) << 32) | (unsigned)__builtin_amdgcn_s_getreg(63492);
#endif

    unsigned long long cnt0 = 0;
    P1Regs<HD, BT> rg;
    bool primed = false;
    if (STACK) {
        // the RoPE table is the same for all layers (one position; a stack has no per-row positions): built here,
        // outside the loop, so that its fp64 constants do not become loop-invariant registers
        for (int e = tid; e < HD / 2; e += NT)
            rope_cos_sin(p0.pos, rope_inv_freq(e, HD, p0.rope_log2_base), s_rope[e], s_rope[HD / 2 + e]);
        lds_barrier();
    }
    for (int layer = 0; layer < n_layers; ++layer) {
    // In a stack the parameters are read through a pointer to the kernel's argument block that is made opaque per
    // layer (as are the thread and workgroup index below): whatever depends only on them is loop-invariant, and
    // the compiler would otherwise compute all of it once in front of the loop over the layers and keep it in
    // registers, hundreds of values, across every phase.
    typedef const __attribute__((address_space(4))) Params *KernargParams;
    KernargParams pk = (KernargParams)__builtin_amdgcn_kernarg_segment_ptr();      // StackArgs begins with Params
    if (STACK) asm volatile("" : "+s"(pk));
    const Params &p = STACK ? *(const Params *)pk : p0;
    const int n2 = p.B * p.NS;                       // attention items of the team
    const int n3 = G * p.NC3 * p.RS3;                // output-projection items of the team
    // (in a stack the thread index is made opaque per layer: everything derived from it would otherwise be computed
    // once in front of the loop over the layers and be kept in registers across all phases)
    int tl = threadIdx.x, w = blockIdx.x;
    if (STACK) asm volatile("" : "+v"(tl), "+s"(w));
    const int team = p.pairmap ? qmod(w >> 1, p.nkv, p.sh_nkv) : qmod(w, p.nkv, p.sh_nkv);
    const int member = p.pairmap ? qdiv(w >> 1, p.nkv, p.sh_nkv) * 2 + (w & 1) : qdiv(w, p.nkv, p.sh_nkv);
    // weights and caches of this layer (layer 0, and the only layer of a plain call: those of the parameters);
    // a reference into the argument block either way, so that each pointer is fetched where it is used
    static_assert(offsetof(Params, wo) == offsetof(Params, wqkv) + 8 && offsetof(Params, kc) == offsetof(Params, wqkv) + 16 &&
                      offsetof(Params, vc) == offsetof(Params, wqkv) + 24, "Params holds a LayerPtrs");
    const LayerPtrs &lp = (STACK && layer > 0) ? tab[layer] : *reinterpret_cast<const LayerPtrs *>(&p.wqkv);
    KvBuf<HD, G> kv;
    OutTile<HD> tile;
    const int b_first = member < n2 ? qdiv(member, p.NS, p.sh_ns) : 0;     // batch row of the first attention item
    const int pos_first = row_pos(p, b_first);
    const int s_first = member < n2 ? qmod(member, p.NS, p.sh_ns) : 0;
    // (with positions per row the stream is set up only where phase 1 first needs it: the position comes from
    // memory, and waiting for it here would hold up the first weight loads)
    const bool own_pos = kLayer && p.row_pos != nullptr;
    P2Stream<HD, G> st2(p, lp, tl, team, b_first, s_first, own_pos ? 0 : p.pos, member < n2 && !own_pos);

    // ---- phase 1 (projection); its last step already starts the K/V stream of phase 2
    EarlyQ eq;
    // (without batches requested ahead the registers of the two batches belong to this layer alone)
    P1Regs<HD, BT> rg_layer;
    P1Regs<HD, BT> &rgu = (STACK && P1Ahead<HD, G, BT>::n > 0) ? rg : rg_layer;
    const uint32_t stamp = p1_all<HD, G, BT, STACK, 0>(p, lp, tl, team, member, smem, s_rope, STACK ? layer : 0, xslots, n_layers, cnt0,
                                             rgu, primed, [&](int stage) {
                                                 if (own_pos) st2 = P2Stream<HD, G>(p, lp, tl, team, b_first, s_first, pos_first, member < n2);
                                                 st2.prefetch(kv, 0);
                                             });
    // a first look at the team's q partials (in a stack only for one batch row and attention on the vector ALU: no
    // registers are left for the sixteen pairs there, they would be spilled as they arrive)
    if (member < n2 && !(STACK && (AttnMfma<HD, G>::on || BT > 1)))
        eq.issue<HD, G>(p, tl, team, qdiv(member, p.NS, p.sh_ns));
    st2.prefetch(kv, 1);
    CF_STAMP(1);
    // ---- phase 2 (attention); the last item already starts the W_o stream of phase 3
    auto p3_args = [&](int it, int &hq, int &c3, int &rs) {
        const int g = it / (p.NC3 * p.RS3), rem = it - g * (p.NC3 * p.RS3);
        hq = team * G + g;
        c3 = rem / p.RS3;
        rs = rem % p.RS3;
    };
    bool tile_ready = false;
    auto p3_prefetch = [&](int part) {
        if (member < n3) {
            int hq, c3, rs;
            p3_args(member, hq, c3, rs);
            p3_load<HD, Mfma<HD, BT>::on>(p, lp, tl, hq, c3, rs, 0, tile, part);
            tile_ready = true;
        }
    };
    for (int it = member; it < n2; it += p.TS) {
        const bool first = (it == member), final_item = (it + p.TS >= n2);
        if (!first) {
            const int b_it = qdiv(it, p.NS, p.sh_ns);
            st2 = P2Stream<HD, G>(p, lp, tl, team, b_it, qmod(it, p.NS, p.sh_ns), row_pos(p, b_it));
            st2.prefetch(kv, 0);
            st2.prefetch(kv, 1);
        }
        // stage 1: first half of the output-projection tile, stage 2: second half
        p2_item<HD, G>(p, lp, tl, team, qdiv(it, p.NS, p.sh_ns), qmod(it, p.NS, p.sh_ns), stamp, first, st2, kv, eq, smem,
                       s_rope + (kLayer && p.row_pos ? qdiv(it, p.NS, p.sh_ns) * HD : 0), [&](int stage) {
            if (final_item) p3_prefetch(stage - 1);
        });
    }
    if (member >= n2) p3_prefetch(2);
    CF_STAMP(3);
    const bool more = STACK && layer + 1 < n_layers;
    auto no_next = [](int) {};
    const LayerPtrs &lpn = STACK ? tab[more ? layer + 1 : layer] : lp;
    constexpr int AHEAD = STACK ? P1Ahead<HD, G, BT>::n : 0;
    // ---- phase 3 (output projection, per-head partials)
    for (int it = member; it < n3; it += p.TS) {
        int hq, c3, rs;
        p3_args(it, hq, c3, rs);
        p3_item<HD, BT>(p, lp, tl, hq, c3, rs, stamp, tile, tile_ready && it == member, smem);
    }
    CF_STAMP(4);
    // ---- phase 4 (sum over heads)
    // In a stack the first two batches of the next layer's weights are requested here: one before the partial
    // outputs of the heads are waited for, one once they have arrived (behind both, their polls would queue for
    // the time the batches take to stream in).
    // (measured on the 7B shape, us per layer: this placement 36.5; both batches before the wait 37.6; the first
    // one already after the merge of the attention partials 37.7; none 37.6)
    if (AHEAD >= 1)
        p1_all<HD, G, BT, STACK, 1>(p, lpn, tl, team, member, smem, s_rope, 0, nullptr, n_layers, cnt0, rg, more, no_next);
    final_reduce(p, tl, stamp, smem, more ? xslots : nullptr, [&]() {
        if (AHEAD >= 2)
            p1_all<HD, G, BT, STACK, 2>(p, lpn, tl, team, member, smem, s_rope, 0, nullptr, n_layers, cnt0, rg, more, no_next);
    });
    primed = more;
    CF_STAMP(5);
    }   // layers
    if (tid == 0) p0.done[(size_t)blockIdx.x * kCounterStride] = cnt0 + (unsigned long long)(n_layers - 1);   // steps completed
#if CF_STAMPS
    CF_STAMP(6);
    lds_barrier();
    if (p0.dbg_t && tid < kStamps) p0.dbg_t[(size_t)blockIdx.x * kStamps + tid] = s_ts[tid];
#endif
}

template <int HD, int G, int BT>
__global__ void __launch_bounds__(NT) CF_KERNEL(const Params p)
{
    decode_steps<HD, G, BT, false>(p, nullptr, 1, nullptr);
}

#if !CF_LAYER
// A stack of layers in one launch: the argument block carries the table of per-layer pointers by value.
template <int HD, int G, int BT>
__global__ void __launch_bounds__(NT) fused_decode_stack(const StackArgs a)
{
    decode_steps<HD, G, BT, true>(a.p, a.tab, a.n_layers, a.xslots);
}
#endif

#if !CF_LAYER
// One-time rearrangement of the weights into per-head contiguous blocks (16 bytes per thread step).
__global__ void pack_qkv_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int D, int nqkv, int hd)
{
    const size_t n = (size_t)D * nqkv / 8;
    const int v_per_row = hd / 8;
    const size_t blk = (size_t)v_per_row * D + kQkvBlockPad / 16;      // block stride in 16-byte units
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t c8 = i % v_per_row, r = (i / v_per_row) % D, cb = i / ((size_t)v_per_row * D);
        dst[cb * blk + r * v_per_row + c8] = src[(r * nqkv + cb * hd) / 8 + c8];
        if (r == 0 && c8 == 0)
            for (int k = 0; k < kQkvBlockPad / 16; ++k) dst[cb * blk + (size_t)v_per_row * D + k] = make_uint4(0, 0, 0, 0);
    }
}

__global__ void pack_o_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int D, int nq, int hd)
{
    const int nch = (D + kOutChunk - 1) / kOutChunk;
    const size_t n = (size_t)nq * nch * hd * (kOutChunk / 8);
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const size_t c8 = i % (kOutChunk / 8), r = (i / (kOutChunk / 8)) % hd;
        const size_t ch = (i / ((size_t)(kOutChunk / 8) * hd)) % nch, h = i / ((size_t)(kOutChunk / 8) * hd * nch);
        const size_t col = ch * kOutChunk + c8 * 8;
        dst[i] = col < (size_t)D ? src[((h * hd + r) * D + col) / 8] : make_uint4(0, 0, 0, 0);
    }
}

#endif  // !CF_LAYER

using KernelFn = void (*)(const Params);

template <int HD, int G>
KernelFn pick_bt(int bt)
{
    switch (bt) {
    case 1: return CF_KERNEL<HD, G, 1>;
    case 4: return CF_KERNEL<HD, G, 4>;
    case 16: return CF_KERNEL<HD, G, 16>;
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

#if !CF_LAYER
using StackFn = void (*)(const StackArgs);

template <int G>
StackFn pick_stack_bt(int bt)
{
    switch (bt) {
    case 1: return fused_decode_stack<128, G, 1>;
    case 4: return fused_decode_stack<128, G, 4>;
    case 16: return fused_decode_stack<128, G, 16>;
    default: return nullptr;
    }
}

// (head_dim 128 only: the shapes whose stacks are worth one launch)
StackFn pick_stack(int hd, int g, int bt)
{
    if (hd != 128) return nullptr;
    switch (g) {
    case 1: return pick_stack_bt<1>(bt);
    case 2: return pick_stack_bt<2>(bt);
    case 4: return pick_stack_bt<4>(bt);
    case 8: return pick_stack_bt<8>(bt);
    default: return nullptr;
    }
}
#endif

}  // namespace

static hipError_t occupancy_of(KernelFn fn, size_t lds_bytes, int *out)
{
    *out = 0;
    if (!fn) return hipSuccess;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void *>(fn), kThreads, lds_bytes);
}

static hipError_t launch_of(KernelFn fn, const Params &p, size_t lds_bytes, hipStream_t stream)
{
    if (!fn) return hipErrorInvalidDeviceFunction;
    hipLaunchKernelGGL(fn, dim3(p.W), dim3(kThreads), lds_bytes, stream, p);
    return hipGetLastError();
}

#if CF_LAYER

hipError_t max_workgroups_per_cu_layer(int hd, int g, int bt, size_t lds_bytes, int *out)
{
    return occupancy_of(pick(hd, g, bt), lds_bytes, out);
}

hipError_t launch_fused_layer(const Params &p, int hd, int g, int bt, size_t lds_bytes, hipStream_t stream)
{
    return launch_of(pick(hd, g, bt), p, lds_bytes, stream);
}

#else

bool wants_layer_kernel(const Params &p)
{
    return p.gamma != nullptr || (p.flags & kFlagResidual) != 0 || p.row_pos != nullptr;
}

size_t lds_floats(const Params &p, int hd, int g, int bt)
{
    const size_t rb = bt < 4 ? bt : 4;
    const size_t maxi = bt == 1 ? 4 : (bt <= 4 ? 2 : 1);
    const size_t f1 = x_lds_floats(hd, bt, p.RPS) + maxi * kWaves * bt * hd + (size_t)kWaves * bt;
    const bool ma = hd == 128 && g >= 4;                                          // attention on MFMA tiles: a K tile per wavefront
    const size_t npart = (g >= 8 && !ma) ? (size_t)kWaves * (64 / (hd / 8)) : kWaves;      // attention partials folded through LDS
    const size_t f2 = (size_t)hd + (size_t)(g + 2) * hd + 8 + 2 * (size_t)g * npart + (size_t)g * npart * hd +
                      (ma ? (size_t)kWaves * 32 * (hd + 8) / 2 + 2 * 256 * 4 : 0);   // K tiles, q operands
    const size_t f3 = (size_t)bt * hd + (size_t)kWaves * rb * kOutChunk;
    size_t f = f1 > f2 ? f1 : f2;
    return f > f3 ? f : f3;
}

hipError_t max_workgroups_per_cu(int hd, int g, int bt, size_t lds_bytes, bool layer, int *out)
{
    if (layer) return max_workgroups_per_cu_layer(hd, g, bt, lds_bytes, out);
    return occupancy_of(pick(hd, g, bt), lds_bytes, out);
}

hipError_t launch_pack(const uint16_t *wqkv, const uint16_t *wo, uint16_t *wqkv_p, uint16_t *wo_p, int D, int nqkv,
                       int nq, int hd, hipStream_t stream)
{
    hipLaunchKernelGGL(pack_qkv_kernel, dim3(2048), dim3(256), 0, stream, reinterpret_cast<const uint4 *>(wqkv),
                       reinterpret_cast<uint4 *>(wqkv_p), D, nqkv, hd);
    hipLaunchKernelGGL(pack_o_kernel, dim3(2048), dim3(256), 0, stream, reinterpret_cast<const uint4 *>(wo),
                       reinterpret_cast<uint4 *>(wo_p), D, nq, hd);
    return hipGetLastError();
}

hipError_t launch_fused_stack(const StackArgs &a, int hd, int g, int bt, size_t lds_bytes, hipStream_t stream)
{
    StackFn fn = pick_stack(hd, g, bt);
    if (!fn || wants_layer_kernel(a.p) || a.n_layers < 1 || a.n_layers > kMaxStackLayers) return hipErrorInvalidDeviceFunction;
    // all workgroups must be resident, as for the one-layer kernel
    int per_cu = 0;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fn), kThreads, lds_bytes);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    if ((long)per_cu * cus < a.p.W) return hipErrorLaunchOutOfResources;
    hipLaunchKernelGGL(fn, dim3(a.p.W), dim3(kThreads), lds_bytes, stream, a);
    return hipGetLastError();
}

hipError_t launch_fused(const Params &p, int hd, int g, int bt, size_t lds_bytes, hipStream_t stream)
{
    if (wants_layer_kernel(p)) return launch_fused_layer(p, hd, g, bt, lds_bytes, stream);
    return launch_of(pick(hd, g, bt), p, lds_bytes, stream);
}

#endif  // CF_LAYER

}  // namespace cf
