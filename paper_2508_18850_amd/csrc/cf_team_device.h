// Team collectives for gfx950: what a group of co-resident workgroups can do in place of the paper's
// ClusterReduce (Alg. 1) and ClusterGather (Alg. 2), which run over the distributed shared memory of a
// thread-block cluster.  CDNA4 has no such memory; the nearest thing is an exchange through global
// memory that never leaves the kernel: every fp32 value travels as a 64-bit {value, stamp} pair written
// with one write-through store and polled by the receiver until the stamp is the current one.  No flag,
// no fence, no atomic; a value is either the old pair or the new one.
//
// Two schedules.  The paper's: log2(N) rounds, in round s rank b sends to rank (b + 2^s) mod N and
// receives from rank (b - 2^s) mod N.  And a direct one: every rank posts its data once and reads the
// posts of its N - 1 peers, one hop in place of log2(N); a hop through memory costs microseconds here
// where a hop through a cluster's shared memory costs a fraction of one, so the direct schedule is the one
// the fused decode kernel uses.
//
// Buffers are worked through in chunks of kThreads x E values (E values per thread in registers), so that
// the register use does not grow with the buffer.
//
// These are device functions to be called by all threads of a workgroup; every workgroup of the team
// must be resident at the same time (the caller's launch has to guarantee that), because receivers spin.
#ifndef CF_TEAM_DEVICE_H
#define CF_TEAM_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {
namespace team {

typedef uint32_t pair_t __attribute__((ext_vector_type(2)));

constexpr int kThreads = 512;      // threads per workgroup the functions are written for
constexpr int kMaxRounds = 4;      // N <= 16

enum Op { kSum = 0, kMax = 1 };

// Exchange area of one launch: inbox of rank r, round s = slots[(r * kMaxRounds + s) * cap ...] for the
// reduce, slots[r * cap ...] for the gather (cap = capacity of one inbox in pairs).
struct Exchange {
    uint64_t *slots;     // device memory, cleared once when it is allocated
    size_t cap;          // pairs per inbox
    uint32_t stamp;      // stamp of this launch, never 0
    uint32_t *err;       // set to 1 when a wait gave up
    long long spin_ticks;    // give up after this many ticks of the 100 MHz wall clock (0: at the first failed look)
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t slots_rsrc(const Exchange &x)
{
    return __builtin_amdgcn_make_buffer_rsrc(x.slots, 0, 0xfffffff8u, 0x00020000);
}

__device__ __forceinline__ void put(__amdgpu_buffer_rsrc_t r, size_t idx, float v, uint32_t stamp)
{
    pair_t d = {__builtin_bit_cast(uint32_t, v), stamp};
    __builtin_amdgcn_raw_buffer_store_b64(d, r, (unsigned)(idx * 8), 0, 16);      // sc1: through to memory
}

__device__ __forceinline__ pair_t peek(__amdgpu_buffer_rsrc_t r, size_t idx)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (unsigned)(idx * 8), 0, 16);   // sc1: not from a stale cache
}

// true when the caller should stop waiting (the error flag is set then)
__device__ __forceinline__ bool gave_up(const Exchange &x, long long &t0)
{
    __builtin_amdgcn_s_sleep(1);
    const long long now = wall_clock64();
    if (t0 == 0) t0 = now;
    if (now - t0 >= x.spin_ticks) {                 // a limit of 0 gives up at the first failed look
        __hip_atomic_store(x.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return false;
}

constexpr int kPolls = 32;         // polls a thread keeps in flight: the receive rate is kPolls x 8 bytes per round trip

// Wait for the pairs at base + first + tid + kThreads*e (e < E, first + ... < count) and hand each value to
// use(e, value).  All polls of a batch are issued before the first one is looked at.
template <int E, class Use>
__device__ __forceinline__ void take(const Exchange &x, __amdgpu_buffer_rsrc_t r, size_t base, size_t first, size_t count,
                                     Use &&use)
{
    constexpr int C = E < kPolls ? E : kPolls;
    const size_t tid = threadIdx.x;
#pragma unroll
    for (int e0 = 0; e0 < E; e0 += C) {
        long long t0 = 0;
        pair_t q[C];
        for (;;) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = first + tid + (size_t)kThreads * (e0 + k);
                q[k] = peek(r, base + (i < count ? i : 0));       // out of range: any valid slot, ignored
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = first + tid + (size_t)kThreads * (e0 + k);
                ok &= (i >= count) | (q[k].y == x.stamp);
            }
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) use(e0 + k, __builtin_bit_cast(float, q[k].x));
    }
}

template <int OP>
__device__ __forceinline__ float fold(float a, float b)
{
    return OP == kSum ? a + b : fmaxf(a, b);
}

// Alg. 1: all-reduce of the N ranks' buffers of `count` values, for the chunk that starts at value `first`:
// rank b holds value first + tid + kThreads*e in d[e].  On return every rank holds the reduction of the
// chunk.  fp32, folded in the order of the rounds.
template <int E, int OP>
__device__ __forceinline__ void reduce(const Exchange &x, int team_first_rank, int N, int b, size_t first, size_t count,
                                       float (&d)[E])
{
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    int s = 0;
    for (int stride = 1; stride < N; stride <<= 1, ++s) {
        const int to = (b + stride) % N;
        const size_t outbox = ((size_t)(team_first_rank + to) * kMaxRounds + s) * x.cap;
        const size_t inbox = ((size_t)(team_first_rank + b) * kMaxRounds + s) * x.cap;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = first + tid + (size_t)kThreads * e;
            if (i < count) put(r, outbox + i, d[e], x.stamp);
        }
        // the whole chunk has been sent before any of it is overwritten (Alg. 1 sends D_b, then folds)
        take<E>(x, r, inbox, first, count, [&](int e, float v) { d[e] = fold<OP>(d[e], v); });
    }
}

// Fold what the N ranks of a team have posted at positions first + tid + kThreads*e (< end) of the area that
// starts `area` pairs into every rank's slots, in rank order, the rank's own values d[] at their place.
template <int E, int OP>
__device__ __forceinline__ void fold_posts(const Exchange &x, __amdgpu_buffer_rsrc_t r, int team_first_rank, int N, int b,
                                           size_t area, size_t first, size_t end, float (&d)[E])
{
    const size_t tid = threadIdx.x;
    const size_t box = (size_t)kMaxRounds * x.cap;                    // a rank's whole slot area
    constexpr int P = E >= kPolls ? 1 : kPolls / E;                   // peers polled together
    float acc[E];
    for (int r0 = 0; r0 < N; r0 += P) {
        pair_t q[P][E];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int peer = r0 + p;
#pragma unroll
                for (int e = 0; e < E; ++e) q[p][e] = pair_t{0u, x.stamp};
                if (peer < N && peer != b) {                          // uniform over the workgroup
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const size_t i = first + tid + (size_t)kThreads * e;
                        q[p][e] = peek(r, (size_t)(team_first_rank + peer) * box + area + (i < end ? i : first));
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const size_t i = first + tid + (size_t)kThreads * e;
                    ok &= (i >= end) | (q[p][e].y == x.stamp);
                }
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int peer = r0 + p;
            if (peer < N) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float v = peer == b ? d[e] : __builtin_bit_cast(float, q[p][e].x);
                    acc[e] = peer == 0 ? v : fold<OP>(acc[e], v);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < E; ++e) d[e] = acc[e];
}

// The all-reduce in one hop: every rank posts its chunk in its own slots and folds the N posts in rank order,
// so that all ranks of a team end with the same bits.
template <int E, int OP>
__device__ __forceinline__ void reduce_direct(const Exchange &x, int team_first_rank, int N, int b, size_t first,
                                              size_t count, float (&d)[E])
{
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    const size_t box = (size_t)kMaxRounds * x.cap;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const size_t i = first + tid + (size_t)kThreads * e;
        if (i < count) put(r, (size_t)(team_first_rank + b) * box + i, d[e], x.stamp);
    }
    fold_posts<E, OP>(x, r, team_first_rank, N, b, 0, first, count, d);
}

// The all-reduce in two hops with the fewest bytes: rank b folds slice b of the buffer (count / N values, in
// rank order) from the posts of the others, posts the result, and reads the other slices from their owners.
// A rank receives 2 * (N - 1) / N * count values, against (N - 1) * count in one hop.  own(i) gives value i of
// the rank's buffer, use(i, v) receives value i of the result.
template <int OP, class Own, class Use>
__device__ __forceinline__ void reduce_two_hops(const Exchange &x, int team_first_rank, int N, int b, size_t count,
                                                Own &&own, Use &&use)
{
    constexpr int C = 16, E = 4;
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    const size_t box = (size_t)kMaxRounds * x.cap;
    const size_t mine = (size_t)(team_first_rank + b) * box;
    const unsigned sl = (unsigned)((count + N - 1) / N);              // values of a slice; count <= cap < 2^32
    const size_t lo = (size_t)b * sl < count ? (size_t)b * sl : count;
    const size_t hi = lo + sl < count ? lo + sl : count;
    for (size_t i0 = 0; i0 < count; i0 += (size_t)kThreads * C) {     // post what the owners of the other slices need
        float v[C];
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            v[k] = i < count ? own(i) : 0.f;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i < count && (i < lo || i >= hi)) put(r, mine + i, v[k], x.stamp);
        }
    }
    for (size_t first = lo; first < hi; first += (size_t)kThreads * E) {      // fold the own slice, post it
        float d[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = first + tid + (size_t)kThreads * e;
            d[e] = i < hi ? own(i) : 0.f;
        }
        fold_posts<E, OP>(x, r, team_first_rank, N, b, 0, first, hi, d);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = first + tid + (size_t)kThreads * e;
            if (i < hi) {
                put(r, mine + x.cap + i, d[e], x.stamp);              // second area of the rank's slots
                use(i, d[e]);
            }
        }
    }
    for (size_t i0 = 0; i0 < count; i0 += (size_t)kThreads * C) {     // the other slices, from their owners
        pair_t q[C];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                const bool want = i < count && (i < lo || i >= hi);
                const unsigned owner = (unsigned)i / sl;
                q[k] = want ? peek(r, (size_t)(team_first_rank + owner) * box + x.cap + i) : pair_t{0u, x.stamp};
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < C; ++k) ok &= q[k].y == x.stamp;
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i < count && (i < lo || i >= hi)) use(i, __builtin_bit_cast(float, q[k].x));
        }
    }
}

constexpr int kGatherBatch = 16;   // values per thread and step of the gathers

// Alg. 2: all-gather.  A rank's buffer has N segments of `seg` values; own(i) gives value i < seg of the
// rank's own data; use(p, v) receives value p of the gathered buffer, p in [0, N*seg), where segment j is the
// data of rank (b - j) mod N.  Nothing is held in registers between the rounds: what arrived in the rank's
// inbox in the earlier rounds is read there again when it is passed on.
template <class Own, class Use>
__device__ __forceinline__ void gather(const Exchange &x, int team_first_rank, int N, int b, size_t seg, Own &&own, Use &&use)
{
    constexpr int C = kGatherBatch;
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    const size_t inbox = (size_t)(team_first_rank + b) * x.cap;
    // wait for positions i0 + tid + kThreads*k of the inbox that are in [seg, end); positions below seg are the rank's own
    auto fetch = [&](size_t i0, size_t end, float (&v)[C]) {
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            v[k] = i < seg ? own(i) : 0.f;
        }
        if (i0 + (size_t)kThreads * C <= seg) return;                 // the whole step is own data (uniform)
        pair_t q[C];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                q[k] = peek(r, inbox + (i >= seg && i < end ? i : seg));
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                ok &= (i < seg) | (i >= end) | (q[k].y == x.stamp);
            }
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i >= seg) v[k] = __builtin_bit_cast(float, q[k].x);
        }
    };
    for (int stride = 1; stride < N; stride <<= 1) {
        const int to = (b + stride) % N;
        const size_t have = seg * (size_t)stride;                     // values this rank holds so far
        const size_t outbox = (size_t)(team_first_rank + to) * x.cap + have;    // they become the peer's next segments
        for (size_t i0 = 0; i0 < have; i0 += (size_t)kThreads * C) {
            float v[C];
            fetch(i0, have, v);
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                if (i < have) put(r, outbox + i, v[k], x.stamp);
            }
        }
    }
    const size_t all = seg * (size_t)N;
    for (size_t i0 = 0; i0 < all; i0 += (size_t)kThreads * C) {
        float v[C];
        fetch(i0, all, v);
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i < all) use(i, v[k]);
        }
    }
}

// The same result in one hop: every rank posts its segment in its own outbox and reads the N - 1 others.
template <class Own, class Use>
__device__ __forceinline__ void gather_direct(const Exchange &x, int team_first_rank, int N, int b, size_t seg, Own &&own,
                                              Use &&use)
{
    constexpr int C = kGatherBatch;
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    for (size_t i0 = 0; i0 < seg; i0 += (size_t)kThreads * C) {
        float v[C];
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            v[k] = i < seg ? own(i) : 0.f;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i < seg) {
                put(r, (size_t)(team_first_rank + b) * x.cap + i, v[k], x.stamp);
                use(i, v[k]);
            }
        }
    }
    // positions seg .. N*seg of the result, as one index space: position p is value p % seg of rank (b - p / seg) mod N
    const size_t all = seg * (size_t)N;
    for (size_t i0 = seg; i0 < all; i0 += (size_t)kThreads * C) {
        pair_t q[C];
        long long t0 = 0;
        for (;;) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                const unsigned p = (unsigned)(i < all ? i : seg);      // all <= cap < 2^32
                const unsigned j = p / (unsigned)seg;
                q[k] = peek(r, (size_t)(team_first_rank + (b - (int)j + N) % N) * x.cap + (p - j * (unsigned)seg));
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = i0 + tid + (size_t)kThreads * k;
                ok &= (i >= all) | (q[k].y == x.stamp);
            }
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) {
            const size_t i = i0 + tid + (size_t)kThreads * k;
            if (i < all) use(i, __builtin_bit_cast(float, q[k].x));
        }
    }
}

}  // namespace team
}  // namespace cf
#endif
