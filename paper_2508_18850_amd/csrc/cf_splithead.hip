// The SplitHead dataflow (paper Appendix B, Alg. 5) of the fused decode step as one kernel for gfx950, behind the
// C ABI (cf_splithead_* in include/cfdecode.h).  It is the ablation the paper compares its SplitToken dataflow
// (Alg. 3, the kernel in cf_fused_kernel.hip) with: same inputs, same result, a different division of the work.
//
// A head is a team of N co-resident workgroups (N = 2, 4 or 8) and the members split the head dimension in every
// stage: member b owns the RoPE pairs [b*h2, (b+1)*h2) of the head, h2 = head_dim / (2N), i.e. dimensions
// b*h2 + j and head_dim/2 + b*h2 + j.
//
//   1  projection    its 3 * 2*h2 columns of W_qkv over all of D (weights repacked once so that the columns of a
//                    member are contiguous), RoPE on its pairs, its slice of the new K/V row appended to the caches
//   2  scores        partial q.k over its dimensions for ALL tokens, kept in LDS (Alg. 5's S_b)
//   3  ClusterReduce of the scores (sum): reduce-scatter + all-gather through stamped {value, stamp} slots in
//                    global memory (cf_team_device.h), 2 hops, the schedule with the fewest bytes
//   4  softmax over all tokens (every member, redundantly), then A_b = P . V over its dimensions
//   5  output proj.  partial O_b = A_b . W_o[its rows of the head, :]  (D values)
//   6  ClusterReduce of O_b: the reduce-scatter half only (every column is summed by one member), then the
//                    paper's atomicAdd of the head's result into an fp32 accumulator shared by all heads
//   7  the workgroup whose atomicAdd completes a column slice (an arrival counter per slice) rounds the slice to
//                    fp16, writes it to `out` and clears accumulator and counter for the next launch
//
// Batch 1, one KV head per query head.  All waits are bounded (CF_ETIMEOUT); all workgroups have to be resident
// at once (one per compute unit).
#include "../../include/cfdecode.h"
#include "cf_rope_device.h"
#include "cf_team_device.h"

#include <cmath>
#include <cstring>
#include <new>

namespace {

using cf::team::Exchange;
using cf::team::pair_t;
constexpr int NT = 512;             // threads per workgroup
constexpr int NW = NT / 64;
constexpr int kDoneStride = 16;     // 64-bit words between the launch counts of two workgroups (one 128-byte line each)
constexpr int kRedFloats = NT * 8;  // floats of the cross-thread sum of stage 1

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// Stage time stamps (100 MHz wall clock, thread 0 of every workgroup), only in builds with -DCF_STAMPS=1
#ifndef CF_STAMPS
#define CF_STAMPS 0
#endif
#if CF_STAMPS
constexpr int kShStamps = 16;
__device__ unsigned long long g_sh_ts[256 * kShStamps];
#define SH_STAMP(k) do { if (threadIdx.x == 0) s_ts[k] = wall_clock64(); } while (0)
#else
#define SH_STAMP(k)
#endif

struct SplitArgs {
    const uint16_t *x, *wqkv, *wo;
    uint16_t *kc, *vc, *out;
    uint64_t *slots;
    float *acc;                     // [D] fp32, zero between launches
    uint32_t *arrive;               // [N] arrivals per column slice, zero between launches
    uint32_t *err;
    unsigned long long *done;       // [W][kDoneStride] launches completed, one line per workgroup
    size_t cap;                     // pairs per exchange area
    long long spin_ticks;
    double log2_base;
    float scale_log2e;
    int D, nh, HD, N, pos, max_seq;
    int only_member0;               // test of the error path: the other members of every team leave at once
};

__device__ __forceinline__ uint16_t f2h(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }

__device__ __forceinline__ h8 load8(const uint16_t *p)
{
    return *reinterpret_cast<const h8 *>(p);
}

__device__ __forceinline__ float wave_fold(float v, bool is_max)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const float o = __shfl_xor(v, m);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    return v;
}

// all threads of the workgroup; s_w: NW floats not in use by anything else
__device__ __forceinline__ float block_fold(float v, bool is_max, float *s_w)
{
    v = wave_fold(v, is_max);
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = s_w[0];
#pragma unroll
    for (int k = 1; k < NW; ++k) r = is_max ? fmaxf(r, s_w[k]) : r + s_w[k];
    __syncthreads();
    return r;
}

// PV: 16-byte pieces per half of a member's slice (h2 = 8 * PV)
template <int PV>
__global__ void __launch_bounds__(NT) fused_decode_splithead(const SplitArgs a)
{
    constexpr int H2 = 8 * PV;            // RoPE pairs of a member
    constexpr int SD = 2 * H2;            // dimensions of a member
    constexpr int P = 6 * PV;             // 16-byte pieces of a packed weight row: q lo, q hi, k lo, k hi, v lo, v hi
    constexpr int RPP = NT / P;           // weight rows per pass of the workgroup
    constexpr int UT = 8 / PV;            // cached rows per thread and batch: 16 loads in flight
    extern __shared__ __align__(16) float smem[];
    __shared__ float s_q[SD], s_k[SD], s_v[SD], s_a[SD], s_w[NW], s_part[NW][SD];
    __shared__ uint32_t s_flag;
#if CF_STAMPS
    __shared__ unsigned long long s_ts[kShStamps];
    if (threadIdx.x < kShStamps) s_ts[threadIdx.x] = 0;
    __syncthreads();
#endif
    SH_STAMP(0);
    float *s_x = smem;                    // [D] the hidden state, later the partial output projection
    float *s_s = smem + a.D;              // stage 1: sums across row groups; then the scores / probabilities
    const int tid = threadIdx.x, w = blockIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.N, D = a.D, HD = a.HD, pos = a.pos;
    // a team sits on one XCD (workgroup w runs on XCD w % 8) when the heads divide evenly
    int head, b;
    if ((a.nh & 7) == 0) {
        const int q = w >> 3;
        head = (w & 7) + 8 * (q / N);
        b = q % N;
    } else {
        head = w / N;
        b = w % N;
    }
    const int team_first = head * N;
    // Error-path test: with its peers gone (before they touch anything) member 0 finds none of their posts, and with a
    // wait limit of 0 it gives up at its first look: a timeout that does not depend on timing, and every wait still ends.
    if (a.only_member0 && b != 0) return;
    // The launch stamp comes from device memory, not from the host: every workgroup keeps the number of launches it
    // has completed in a line of its own (all hold the same number), so a launch recorded once in a graph stamps
    // each of its replays afresh.  Written by the previous launch, hence a scalar load through the cache will do.
    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.done + (size_t)w * kDoneStride)
                 : "memory");
    launches += 1ull;
    Exchange x;
    x.slots = a.slots, x.cap = a.cap, x.err = a.err, x.spin_ticks = a.spin_ticks;
    x.stamp = (uint32_t)(launches + (launches >> 32));        // never 0, the value of a cleared slot

    // ---- 1: projection.  Thread (row group g = tid / P, piece c = tid % P) walks rows g, g + RPP, ...
    for (int v = tid; v < D / 8; v += NT) {
        const h8 xv = load8(a.x + (size_t)v * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) s_x[v * 8 + j] = (float)xv[j];
    }
    __syncthreads();
    {
        const bool active = tid < RPP * P;
        const int g = active ? tid / P : 0, c = active ? tid % P : 0;
        const uint16_t *wb = a.wqkv + ((size_t)(head * N + b) * D) * (P * 8) + c * 8;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        constexpr int U = 8;
        for (int r0 = 0; r0 < D; r0 += RPP * U) {
            h8 wv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + g + u * RPP;
                wv[u] = load8(wb + (size_t)(r < D ? r : D - 1) * (P * 8));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + g + u * RPP;
                const float xf = (active && r < D) ? s_x[r] : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(xf, (float)wv[u][j], acc[j]);
            }
        }
        SH_STAMP(1);            // weights consumed
        if (active) {
#pragma unroll
            for (int j = 0; j < 8; ++j) s_s[g * (P * 8) + c * 8 + j] = acc[j];
        }
        __syncthreads();
        float y = 0.f;
        if (tid < P * 8)
            for (int k = 0; k < RPP; ++k) y += s_s[k * (P * 8) + tid];
        __syncthreads();
        if (tid < P * 8) s_s[tid] = y;        // [q lo | q hi | k lo | k hi | v lo | v hi], H2 values each
        __syncthreads();
        if (tid < H2) {
            const int i = b * H2 + tid;       // frequency index of the pair
            const double inv_freq = exp2(-2.0 * (double)i / (double)HD * a.log2_base);
            float cs, sn;
            cf::rope_cos_sin(pos, inv_freq, cs, sn);
            const float qlo = s_s[tid], qhi = s_s[H2 + tid], klo = s_s[2 * H2 + tid], khi = s_s[3 * H2 + tid];
            const float vlo = s_s[4 * H2 + tid], vhi = s_s[5 * H2 + tid];
            const float kl = klo * cs - khi * sn, kh = khi * cs + klo * sn;
            s_q[tid] = qlo * cs - qhi * sn;
            s_q[H2 + tid] = qhi * cs + qlo * sn;
            s_k[tid] = kl, s_k[H2 + tid] = kh;
            s_v[tid] = vlo, s_v[H2 + tid] = vhi;
            const size_t row = ((size_t)head * a.max_seq + pos) * HD + i;
            a.kc[row] = f2h(kl), a.kc[row + HD / 2] = f2h(kh);
            a.vc[row] = f2h(vlo), a.vc[row + HD / 2] = f2h(vhi);
        }
        __syncthreads();
    }

    SH_STAMP(2);                // q, k, v of the new token ready
    // ---- 2: partial scores of all tokens over the member's dimensions
    const uint16_t *kbase = a.kc + (size_t)head * a.max_seq * HD + b * H2;
    const uint16_t *vbase = a.vc + (size_t)head * a.max_seq * HD + b * H2;
    {
        float qf[SD];
#pragma unroll
        for (int j = 0; j < SD; ++j) qf[j] = s_q[j];
        for (int t0 = 0; t0 < pos; t0 += NT * UT) {
            h8 kv[UT][2 * PV];
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                const int t = t0 + tid + NT * u;
                const uint16_t *rp = kbase + (size_t)(t < pos ? t : pos - 1) * HD;
#pragma unroll
                for (int p = 0; p < PV; ++p) {
                    kv[u][p] = load8(rp + 8 * p);
                    kv[u][PV + p] = load8(rp + HD / 2 + 8 * p);
                }
            }
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                const int t = t0 + tid + NT * u;
                float s = 0.f;
#pragma unroll
                for (int p = 0; p < 2 * PV; ++p)
#pragma unroll
                    for (int j = 0; j < 8; ++j) s = fmaf(qf[p * 8 + j], (float)kv[u][p][j], s);
                if (t < pos) s_s[t] = s;
            }
        }
        if (tid == 0) {
            float s = 0.f;
            for (int j = 0; j < SD; ++j) s = fmaf(s_q[j], s_k[j], s);
            s_s[pos] = s;                      // the new token attends to itself
        }
    }
    __syncthreads();

    SH_STAMP(3);                // partial scores done
    // ---- 3: ClusterReduce(S_b, sum) over the team
    const size_t count = (size_t)pos + 1;
    cf::team::reduce_two_hops<cf::team::kSum>(
        x, team_first, N, b, count, [&](size_t i) { return s_s[i]; }, [&](size_t i, float v) { s_s[i] = v; });
    __syncthreads();

    SH_STAMP(4);                // scores reduced
    // ---- 4: softmax over all tokens, A_b = P . V over the member's dimensions
    {
        float m = -3.0e38f;
        for (int t = tid; t <= pos; t += NT) m = fmaxf(m, s_s[t]);
        m = block_fold(m, true, s_w);
        float l = 0.f;
        for (int t = tid; t <= pos; t += NT) {
            const float e = exp2f((s_s[t] - m) * a.scale_log2e);
            s_s[t] = e;
            l += e;
        }
        l = block_fold(l, false, s_w);         // its barriers also order the writes of s_s before the reads below
        SH_STAMP(5);            // softmax done
        float av[SD];
#pragma unroll
        for (int j = 0; j < SD; ++j) av[j] = 0.f;
        for (int t0 = 0; t0 < pos; t0 += NT * UT) {
            h8 vv[UT][2 * PV];
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                const int t = t0 + tid + NT * u;
                const uint16_t *rp = vbase + (size_t)(t < pos ? t : pos - 1) * HD;
#pragma unroll
                for (int p = 0; p < PV; ++p) {
                    vv[u][p] = load8(rp + 8 * p);
                    vv[u][PV + p] = load8(rp + HD / 2 + 8 * p);
                }
            }
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                const int t = t0 + tid + NT * u;
                const float pr = t < pos ? s_s[t] : 0.f;
#pragma unroll
                for (int p = 0; p < 2 * PV; ++p)
#pragma unroll
                    for (int j = 0; j < 8; ++j) av[p * 8 + j] = fmaf(pr, (float)vv[u][p][j], av[p * 8 + j]);
            }
        }
        if (tid == 0) {
            const float pr = s_s[pos];
#pragma unroll
            for (int j = 0; j < SD; ++j) av[j] = fmaf(pr, s_v[j], av[j]);
        }
#pragma unroll
        for (int j = 0; j < SD; ++j) {
            const float s = wave_fold(av[j], false);
            if (lane == 0) s_part[wave][j] = s;
        }
        __syncthreads();
        if (tid < SD) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < NW; ++k) s += s_part[k][tid];
            s_a[tid] = s / l;
        }
        __syncthreads();
    }

    SH_STAMP(6);                // A_b done
    // ---- 5: partial output projection over the member's rows of W_o: s_x[c] = sum_j A_b[j] W_o[row_j, c]
    {
        const uint16_t *wlo = a.wo + ((size_t)head * HD + b * H2) * D;
        const uint16_t *whi = wlo + (size_t)(HD / 2) * D;
        for (int c0 = tid * 8; c0 < D; c0 += NT * 8) {
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = 0.f;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const uint16_t *wr = (half ? whi : wlo) + c0;
#pragma unroll
                for (int r0 = 0; r0 < H2; r0 += 8) {
                    h8 wv[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) wv[r] = load8(wr + (size_t)(r0 + r) * D);
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const float af = s_a[half * H2 + r0 + r];
#pragma unroll
                        for (int j = 0; j < 8; ++j) o[j] = fmaf(af, (float)wv[r][j], o[j]);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) s_x[c0 + j] = o[j];
        }
    }
    __syncthreads();

    SH_STAMP(7);                // O_b done
    // ---- 6: reduce-scatter of O_b over the team (third area of the members' slots), atomicAdd across the heads
    const unsigned sl = (unsigned)((D + N - 1) / N);
    const int lo = min(b * (int)sl, D), hi = min(lo + (int)sl, D);
    {
        const __amdgpu_buffer_rsrc_t r = cf::team::slots_rsrc(x);
        const size_t box = (size_t)cf::team::kMaxRounds * x.cap, area = 2 * x.cap;
        const size_t mine = (size_t)(team_first + b) * box + area;
        for (int i = tid; i < D; i += NT)
            if (i < lo || i >= hi) cf::team::put(r, mine + i, s_x[i], x.stamp);
        constexpr int E = 4;
        for (int first = lo; first < hi; first += NT * E) {
            float d[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int i = first + tid + NT * e;
                d[e] = i < hi ? s_x[i] : 0.f;
            }
            cf::team::fold_posts<E, cf::team::kSum>(x, r, team_first, N, b, area, (size_t)first, (size_t)hi, d);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int i = first + tid + NT * e;
                if (i < hi) {
                    // the returned value is waited for: the addition has been performed where all workgroups see it
                    const float before = __hip_atomic_fetch_add(a.acc + i, d[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    asm volatile("" ::"v"(before));
                }
            }
        }
    }

    SH_STAMP(8);                // O reduced over the team and added
    // ---- 7: the last head to add its slice b finishes it.  No fence: every addition above has returned before the
    // barrier, the counter is incremented after it, and the sums are fetched with an atomic exchange (which also
    // clears them), so nothing here depends on what a cache of this XCD holds.
    __syncthreads();
    if (tid == 0) s_flag = __hip_atomic_fetch_add(a.arrive + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_flag == (uint32_t)a.nh - 1u) {
        for (int i = lo + tid; i < hi; i += NT)
            a.out[i] = f2h(__hip_atomic_exchange(a.acc + i, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if (tid == 0) __hip_atomic_store(a.arrive + b, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid == 0) a.done[(size_t)w * kDoneStride] = launches;
    SH_STAMP(9);
#if CF_STAMPS
    __syncthreads();
    if (tid < kShStamps && w < 256) g_sh_ts[w * kShStamps + tid] = s_ts[tid];
#endif
}

// One-time rearrangement of W_qkv [D, 3 * nh * HD] into per-member blocks [nh][N][D][6 * PV * 8], 16 bytes per step
__global__ void pack_splithead_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int D, int nh, int HD, int N)
{
    const int H2 = HD / (2 * N), RW = 6 * H2 / 8;       // 16-byte pieces per packed row (h2 is a multiple of 8)
    const size_t n = (size_t)nh * N * D * RW;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(i % RW) * 8;
        const size_t r = (i / RW) % D, m = i / ((size_t)RW * D);
        const int b = (int)(m % N), head = (int)(m / N);
        const int sec = e / H2, j = e % H2;             // sec: q lo, q hi, k lo, k hi, v lo, v hi
        const int which = sec >> 1, half = sec & 1;
        const size_t col = (size_t)which * nh * HD + (size_t)head * HD + (size_t)half * (HD / 2) + b * H2 + j;
        dst[i] = src[(r * (size_t)(3 * nh * HD) + col) / 8];
    }
}

using SplitFn = void (*)(const SplitArgs);

SplitFn pick(int pv)
{
    switch (pv) {
    case 1: return fused_decode_splithead<1>;
    case 2: return fused_decode_splithead<2>;
    case 4: return fused_decode_splithead<4>;
    default: return nullptr;
    }
}

}  // namespace

struct cf_splithead_s {
    cf_config cfg;
    int N = 0, W = 0, pv = 0;
    char *ws = nullptr;
    size_t ws_bytes = 0, cap = 0, lds_bytes = 0;
    uint64_t *slots = nullptr;
    float *acc = nullptr;
    uint32_t *arrive = nullptr, *err = nullptr;
    unsigned long long *done = nullptr;
    long long spin_ticks = 200000000LL;
    int only_member0 = 0;
    int last_hip = 0;
};

extern "C" {

int cf_splithead_create(const cf_config *cfg, int32_t team_size, cf_splithead *out)
{
    if (!cfg || !out) return CF_EINVAL;
    *out = nullptr;
    const cf_config &c = *cfg;
    if (c.d_model < 8 || c.d_model % 8 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.max_seq < 1 || c.max_batch < 1 ||
        !(c.rope_base > 1.f) || team_size < 1)
        return CF_EINVAL;
    const int N = team_size;
    if (c.n_q_heads != c.n_kv_heads || c.max_batch != 1 || (c.head_dim != 64 && c.head_dim != 128) ||
        (N != 2 && N != 4 && N != 8) || c.head_dim % (16 * N) || c.d_model > 16384)
        return CF_EUNSUPPORTED;
    const int pv = c.head_dim / (16 * N);
    SplitFn fn = pick(pv);
    if (!fn) return CF_EUNSUPPORTED;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return CF_EHIP;
    const int W = c.n_q_heads * N;
    if (W > prop.multiProcessorCount) return CF_EUNSUPPORTED;         // all workgroups resident, one per compute unit
    const size_t s_floats = (size_t)c.max_seq + 64 > (size_t)kRedFloats ? (size_t)c.max_seq + 64 : (size_t)kRedFloats;
    const size_t lds = ((size_t)c.d_model + s_floats) * sizeof(float);
    if (lds > 150 * 1024) return CF_EUNSUPPORTED;                     // Alg. 5 keeps the scores of all tokens on chip
    int per_cu = 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
            hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(fn), NT, lds) != hipSuccess ||
        per_cu < 1)
        return CF_EUNSUPPORTED;
    cf_splithead t = new (std::nothrow) cf_splithead_s();
    if (!t) return CF_ENOMEM;
    t->cfg = c, t->N = N, t->W = W, t->pv = pv, t->lds_bytes = lds;
    t->cap = (size_t)c.max_seq + 1 > (size_t)c.d_model ? (size_t)c.max_seq + 1 : (size_t)c.d_model;
    const size_t nslots = (size_t)W * cf::team::kMaxRounds * t->cap;
    const size_t acc_end = (512 + (size_t)c.d_model * sizeof(float) + 255) / 256 * 256;
    const size_t head_al = acc_end + (size_t)W * kDoneStride * sizeof(unsigned long long);
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
    t->arrive = reinterpret_cast<uint32_t *>(t->ws + 256);
    t->acc = reinterpret_cast<float *>(t->ws + 512);
    t->done = reinterpret_cast<unsigned long long *>(t->ws + acc_end);
    t->slots = reinterpret_cast<uint64_t *>(t->ws + head_al);
    *out = t;
    return CF_OK;
}

int cf_splithead_destroy(cf_splithead t)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipFree(t->ws);
    delete t;
    return e == hipSuccess ? CF_OK : CF_EHIP;
}

int cf_splithead_pack(cf_splithead t, const void *W_qkv, void *W_qkv_members, void *stream)
{
    if (!t || !W_qkv || !W_qkv_members || W_qkv == W_qkv_members) return CF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(W_qkv) | reinterpret_cast<uintptr_t>(W_qkv_members)) & 15u) return CF_EINVAL;
    const cf_config &c = t->cfg;
    hipLaunchKernelGGL(pack_splithead_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(W_qkv), static_cast<uint4 *>(W_qkv_members), c.d_model, c.n_q_heads,
                       c.head_dim, t->N);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    return CF_OK;
}

int cf_splithead_decode(cf_splithead t, const void *x, const void *W_qkv_members, const void *W_o, void *k_cache,
                        void *v_cache, int32_t pos, void *out, void *stream)
{
    if (!t || !x || !W_qkv_members || !W_o || !k_cache || !v_cache || !out) return CF_EINVAL;
    if (pos < 0 || pos >= t->cfg.max_seq) return CF_EINVAL;
    const void *ptrs[] = {x, W_qkv_members, W_o, k_cache, v_cache, out};
    for (const void *p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) & 15u) return CF_EINVAL;
    const cf_config &c = t->cfg;
    SplitArgs a;
    std::memset(&a, 0, sizeof a);
    a.x = static_cast<const uint16_t *>(x);
    a.wqkv = static_cast<const uint16_t *>(W_qkv_members);
    a.wo = static_cast<const uint16_t *>(W_o);
    a.kc = static_cast<uint16_t *>(k_cache);
    a.vc = static_cast<uint16_t *>(v_cache);
    a.out = static_cast<uint16_t *>(out);
    a.slots = t->slots, a.acc = t->acc, a.arrive = t->arrive, a.err = t->err, a.done = t->done, a.cap = t->cap;
    a.spin_ticks = t->spin_ticks;
    a.log2_base = std::log2((double)c.rope_base);
    a.scale_log2e = 1.4426950408889634f / std::sqrt((float)c.head_dim);
    a.D = c.d_model, a.nh = c.n_q_heads, a.HD = c.head_dim, a.N = t->N, a.pos = pos, a.max_seq = c.max_seq;
    a.only_member0 = t->only_member0;
    hipLaunchKernelGGL(pick(t->pv), dim3(t->W), dim3(NT), t->lds_bytes, static_cast<hipStream_t>(stream), a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        t->last_hip = (int)e;
        return CF_EHIP;
    }
    return CF_OK;
}

int cf_splithead_status(cf_splithead t, void *stream)
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
        e = hipMemset(t->ws, 0, t->ws_bytes);        // accumulator, arrival counters and all stamps start afresh
        if (e == hipSuccess) e = hipDeviceSynchronize();
        return e == hipSuccess ? CF_ETIMEOUT : CF_EHIP;
    }
    return CF_OK;
}

#if CF_STAMPS
// profiling library only: the stage stamps of the last launch (host buffer of 256 * 16 64-bit words)
int cf_splithead_trace_read(void *host_dst)
{
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_sh_ts), sizeof(unsigned long long) * 256 * kShStamps);
    return e == hipSuccess ? CF_OK : CF_EHIP;
}
#endif

int cf_splithead_set_spin_limit(cf_splithead t, int32_t spin_limit_us)
{
    if (!t || spin_limit_us < -1) return CF_EINVAL;
    t->only_member0 = spin_limit_us == -1;
    t->spin_ticks = spin_limit_us == -1 ? 0 : (long long)spin_limit_us * 100;
    return CF_OK;
}

}  // extern "C"
