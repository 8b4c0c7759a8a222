// Team collectives for gfx950: what a group of co-resident workgroups can do in place of the paper's
// ClusterReduce (Alg. 1) and ClusterGather (Alg. 2), which run over the distributed shared memory of a
// thread-block cluster.  CDNA4 has no such memory; the nearest thing is an exchange through global
// memory that never leaves the kernel: every fp32 value travels as a 64-bit {value, stamp} pair written
// with one write-through store and polled by the receiver until the stamp is the current one.  No flag,
// no fence, no atomic; a value is either the old pair or the new one.
//
// The schedules are the paper's: log2(N) rounds, in round s rank b sends to rank (b + 2^s) mod N and
// receives from rank (b - 2^s) mod N.  The data of a rank stays in registers (E values per thread).
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
    long long spin_ticks;    // give up after this many ticks of the 100 MHz wall clock
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
    if (now - t0 > x.spin_ticks) {
        __hip_atomic_store(x.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    return false;
}

// Wait for the pairs at base + tid + kThreads*e (e < E, index < count) and hand each value to use(e, value).
// Polls go out eight at a time and are looked at only after all eight have been issued.
template <int E, class Use>
__device__ __forceinline__ void take(const Exchange &x, __amdgpu_buffer_rsrc_t r, size_t base, size_t count, Use &&use)
{
    constexpr int C = E < 8 ? E : 8;
    const size_t tid = threadIdx.x;
#pragma unroll
    for (int e0 = 0; e0 < E; e0 += C) {
        long long t0 = 0;
        pair_t q[C];
        for (;;) {
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = tid + (size_t)kThreads * (e0 + k);
                q[k] = peek(r, base + (i < count ? i : 0));       // out of range: any valid slot, ignored
            }
            __builtin_amdgcn_sched_barrier(0);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < C; ++k) {
                const size_t i = tid + (size_t)kThreads * (e0 + k);
                ok &= (i >= count) | (q[k].y == x.stamp);
            }
            if (ok || gave_up(x, t0)) break;
        }
#pragma unroll
        for (int k = 0; k < C; ++k) use(e0 + k, __builtin_bit_cast(float, q[k].x));
    }
}

// Alg. 1: all-reduce of the N ranks' buffers of `count` values (rank `b` holds value i = tid + kThreads*e
// in d[e]).  On return every rank holds the reduction.  fp32, folded in the order of the rounds.
template <int E, int OP>
__device__ __forceinline__ void reduce(const Exchange &x, int team_first_rank, int N, int b, size_t count, float (&d)[E])
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
            const size_t i = tid + (size_t)kThreads * e;
            if (i < count) put(r, outbox + i, d[e], x.stamp);
        }
        // the whole buffer has been sent before any of it is overwritten (Alg. 1 sends D_b, then folds)
        take<E>(x, r, inbox, count, [&](int e, float v) { d[e] = OP == kSum ? d[e] + v : fmaxf(d[e], v); });
    }
}

// Alg. 2: all-gather.  A rank's buffer has N segments of `seg` values; position i = tid + kThreads*e of the
// whole buffer is in g[e]; on entry segment 0 is the rank's own data, on return segment j is the data of
// rank (b - j) mod N.
template <int E>
__device__ __forceinline__ void gather(const Exchange &x, int team_first_rank, int N, int b, size_t seg, float (&g)[E])
{
    const __amdgpu_buffer_rsrc_t r = slots_rsrc(x);
    const size_t tid = threadIdx.x;
    for (int stride = 1; stride < N; stride <<= 1) {
        const int to = (b + stride) % N;
        const size_t have = seg * (size_t)stride;                     // values this rank holds so far
        const size_t outbox = (size_t)(team_first_rank + to) * x.cap + have;    // they become the peer's next segments
        const size_t inbox = (size_t)(team_first_rank + b) * x.cap + have;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = tid + (size_t)kThreads * e;
            if (i < have) put(r, outbox + i, g[e], x.stamp);
        }
        // positions [have, 2*have) arrive now: thread tid owns position have + j for j = tid + kThreads*e - have
#pragma unroll
        for (int e0 = 0; e0 < E; e0 += 8) {
            constexpr int C = E < 8 ? E : 8;
            long long t0 = 0;
            for (;;) {
                pair_t q[C];
#pragma unroll
                for (int k = 0; k < C; ++k) {
                    const size_t i = tid + (size_t)kThreads * (e0 + k);
                    const bool mine = i >= have && i < 2 * have;
                    q[k] = peek(r, (size_t)(team_first_rank + b) * x.cap + (mine ? i : have));
                }
                __builtin_amdgcn_sched_barrier(0);
                bool ok = true;
#pragma unroll
                for (int k = 0; k < C; ++k) {
                    const size_t i = tid + (size_t)kThreads * (e0 + k);
                    const bool mine = i >= have && i < 2 * have;
                    ok &= !mine | (q[k].y == x.stamp);
                    if (mine) g[e0 + k] = __builtin_bit_cast(float, q[k].x);
                }
                if (ok || gave_up(x, t0)) break;
            }
        }
        (void)inbox;
    }
}

}  // namespace team
}  // namespace cf
#endif
