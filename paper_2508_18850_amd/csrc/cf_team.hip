// Team collectives behind the C ABI (cf_team_* in include/cfdecode.h): kernels that run the paper's
// ClusterReduce / ClusterGather schedules (Alg. 1, Alg. 2) among co-resident workgroups through stamped
// exchange slots, one-hop versions of the same collectives, and the two-kernel versions that go through a scratch buffer in global memory instead
// (the "off-chip" column of the paper's Table 1).
#include "../../include/cfdecode.h"
#include "cf_team_device.h"

#include <cstdlib>
#include <new>

namespace {

using cf::team::kThreads;
constexpr int kCounterStride = 16;      // 64-bit words between the launch counters of two workgroups
constexpr size_t kMaxElems = 65536;     // largest buffer of one rank (values)

struct TeamArgs {
    const float *in;
    float *out;
    float *scratch;
    uint64_t *slots;
    unsigned long long *counters;    // [ranks][kCounterStride]
    uint32_t *err;
    size_t cap, count;
    int N;
    long long spin_ticks;
};

// launch stamp from this workgroup's own launch counter (never 0); the counter is written back at the end
__device__ __forceinline__ uint32_t launch_stamp(const TeamArgs &a, unsigned long long &cnt)
{
    unsigned long long launches;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(launches)
                 : "s"(a.counters + (size_t)blockIdx.x * kCounterStride)
                 : "memory");
    cnt = launches + 1ull;
    return (uint32_t)(cnt + (cnt >> 32));
}

// E values per thread and chunk; the buffer is worked through chunk by chunk
template <int E, int OP, bool DIRECT>
__global__ void __launch_bounds__(kThreads) team_reduce_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N, tid = threadIdx.x;
    unsigned long long cnt;
    const cf::team::Exchange x = {a.slots, a.cap, launch_stamp(a, cnt), a.err, a.spin_ticks};
    const float *src = a.in + (size_t)w * a.count;
    float *dst = a.out + (size_t)w * a.count;
    for (size_t first = 0; first < a.count; first += (size_t)kThreads * E) {
        float d[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = first + tid + (size_t)kThreads * e;
            d[e] = i < a.count ? src[i] : 0.f;
        }
        if (DIRECT)
            cf::team::reduce_direct<E, OP>(x, team * a.N, a.N, b, first, a.count, d);
        else
            cf::team::reduce<E, OP>(x, team * a.N, a.N, b, first, a.count, d);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const size_t i = first + tid + (size_t)kThreads * e;
            if (i < a.count) dst[i] = d[e];
        }
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

template <int OP>
__global__ void __launch_bounds__(kThreads) team_reduce_two_hops_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N;
    unsigned long long cnt;
    const cf::team::Exchange x = {a.slots, a.cap, launch_stamp(a, cnt), a.err, a.spin_ticks};
    const float *src = a.in + (size_t)w * a.count;
    float *dst = a.out + (size_t)w * a.count;
    cf::team::reduce_two_hops<OP>(x, team * a.N, a.N, b, a.count, [&](size_t i) { return src[i]; },
                                  [&](size_t i, float v) { dst[i] = v; });
    if (threadIdx.x == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

// count = values of one segment; a rank's output has N segments
template <bool DIRECT>
__global__ void __launch_bounds__(kThreads) team_gather_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N;
    unsigned long long cnt;
    const cf::team::Exchange x = {a.slots, a.cap, launch_stamp(a, cnt), a.err, a.spin_ticks};
    const float *src = a.in + (size_t)w * a.count;
    float *dst = a.out + (size_t)w * a.count * a.N;
    auto own = [&](size_t i) { return src[i]; };
    auto use = [&](size_t p, float v) { dst[p] = v; };
    if (DIRECT)
        cf::team::gather_direct(x, team * a.N, a.N, b, a.count, own, use);
    else
        cf::team::gather(x, team * a.N, a.N, b, a.count, own, use);
    if (threadIdx.x == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

// ---- the two-kernel versions: every rank writes its buffer to global memory, the kernel boundary is the
//      synchronisation, then every rank reads what it needs
// (eight independent loads per thread and step, so that these kernels are bound by bandwidth and not by
// one load latency per value)
constexpr int kU = 8;

__global__ void __launch_bounds__(kThreads) team_stage_kernel(const TeamArgs a)
{
    const size_t w = blockIdx.x;
    for (size_t i0 = threadIdx.x; i0 < a.count; i0 += (size_t)kThreads * kU) {
        float v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const size_t i = i0 + (size_t)kThreads * u;
            v[u] = i < a.count ? a.in[w * a.count + i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const size_t i = i0 + (size_t)kThreads * u;
            if (i < a.count) a.scratch[w * a.count + i] = v[u];
        }
    }
}

template <int OP>
__global__ void __launch_bounds__(kThreads) team_reduce_offchip_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N;
    for (size_t i0 = threadIdx.x; i0 < a.count; i0 += (size_t)kThreads * kU) {
        float v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const size_t i = i0 + (size_t)kThreads * u;
            v[u] = i < a.count ? a.scratch[(size_t)team * a.N * a.count + i] : 0.f;
        }
        for (int r = 1; r < a.N; ++r) {
            float o[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const size_t i = i0 + (size_t)kThreads * u;
                o[u] = i < a.count ? a.scratch[((size_t)team * a.N + r) * a.count + i] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) v[u] = OP == cf::team::kSum ? v[u] + o[u] : fmaxf(v[u], o[u]);
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const size_t i = i0 + (size_t)kThreads * u;
            if (i < a.count) a.out[(size_t)w * a.count + i] = v[u];
        }
    }
}

__global__ void __launch_bounds__(kThreads) team_gather_offchip_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N;
    for (int j = 0; j < a.N; ++j) {
        const int r = (b - j + a.N) % a.N;
        for (size_t i0 = threadIdx.x; i0 < a.count; i0 += (size_t)kThreads * kU) {
            float v[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const size_t i = i0 + (size_t)kThreads * u;
                v[u] = i < a.count ? a.scratch[((size_t)team * a.N + r) * a.count + i] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const size_t i = i0 + (size_t)kThreads * u;
                if (i < a.count) a.out[((size_t)w * a.N + j) * a.count + i] = v[u];
            }
        }
    }
}

using Kernel = void (*)(const TeamArgs);

template <int OP, bool DIRECT>
Kernel pick_reduce(int e)
{
    switch (e) {
    case 1: return team_reduce_kernel<1, OP, DIRECT>;
    case 2: return team_reduce_kernel<2, OP, DIRECT>;
    case 4: return team_reduce_kernel<4, OP, DIRECT>;
    case 8: return team_reduce_kernel<8, OP, DIRECT>;
    }
    return team_reduce_kernel<16, OP, DIRECT>;
}

// values per thread and chunk: enough for the whole buffer in one chunk up to 16
int values_per_thread(size_t values)
{
    const size_t need = (values + kThreads - 1) / kThreads;
    for (int e = 1; e < 16; e *= 2)
        if ((size_t)e >= need) return e;
    return 16;
}

}  // namespace

struct cf_team_s {
    int max_ranks = 0;
    size_t cap = 0;
    int num_cu = 0;
    char *ws = nullptr;
    size_t slots_bytes = 0, clear_bytes = 0;
    uint64_t *slots = nullptr;
    unsigned long long *counters = nullptr;
    uint32_t *err = nullptr;
    float *scratch = nullptr;
    long long spin_ticks = 200000000LL;     // 2 s
    int last_ranks = 0;                     // workgroups of the previous launch
    int last_hip = 0;
};

namespace {

int fail(cf_team t, hipError_t e)
{
    if (t) t->last_hip = (int)e;
    return CF_EHIP;
}

bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int check_call(cf_team t, int32_t teams, int32_t team_size, const void *in, const void *out, size_t elems, int32_t mode)
{
    if (mode != CF_TEAM_ROUNDS && mode != CF_TEAM_TWO_KERNELS && mode != CF_TEAM_DIRECT && mode != CF_TEAM_TWO_HOPS)
        return CF_EINVAL;
    if (!t || !in || !out || teams < 1 || !pow2(team_size) || team_size > 16 || elems < 1) return CF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 3u) return CF_EINVAL;
    if ((long)teams * team_size > t->max_ranks) return CF_EINVAL;
    // receivers spin: all workgroups of the launch must be resident, one per compute unit
    if ((long)teams * team_size > t->num_cu) return CF_EUNSUPPORTED;
    return CF_OK;
}

// Every workgroup counts its own launches and all of a launch must agree on the count: when the number of
// workgroups changes, the counts (and with them all stamps) start together again.
int same_grid(cf_team t, int ranks)
{
    if (ranks == t->last_ranks) return CF_OK;
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemset(t->ws, 0, t->clear_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail(t, e);
    t->last_ranks = ranks;
    return CF_OK;
}

TeamArgs make_args(cf_team t, const float *in, float *out, size_t count, int n)
{
    TeamArgs a;
    a.in = in;
    a.out = out;
    a.scratch = t->scratch;
    a.slots = t->slots;
    a.counters = t->counters;
    a.err = t->err;
    a.cap = t->cap;
    a.count = count;
    a.N = n;
    a.spin_ticks = t->spin_ticks;
    return a;
}

}  // namespace

extern "C" {

int cf_team_create(int32_t max_ranks, size_t max_elems, cf_team *out)
{
    if (!out || max_ranks < 1 || max_elems < 1 || max_elems > kMaxElems) return CF_EINVAL;
    *out = nullptr;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return CF_EHIP;
    cf_team t = new (std::nothrow) cf_team_s();
    if (!t) return CF_ENOMEM;
    t->max_ranks = max_ranks;
    t->cap = max_elems;
    t->num_cu = prop.multiProcessorCount;
    const size_t head = 256 + (size_t)max_ranks * kCounterStride * sizeof(unsigned long long);
    t->slots_bytes = (size_t)max_ranks * cf::team::kMaxRounds * max_elems * sizeof(uint64_t);
    if (t->slots_bytes > 0xfffffff0ull) {            // slots are addressed with 32-bit byte offsets
        delete t;
        return CF_EUNSUPPORTED;
    }
    const size_t head_al = (head + 255) / 256 * 256;
    const size_t scratch_bytes = (size_t)max_ranks * max_elems * sizeof(float);
    t->clear_bytes = head_al + t->slots_bytes;
    e = hipMalloc(reinterpret_cast<void **>(&t->ws), t->clear_bytes + scratch_bytes);
    if (e != hipSuccess) {
        delete t;
        return e == hipErrorOutOfMemory ? CF_ENOMEM : CF_EHIP;
    }
    t->err = reinterpret_cast<uint32_t *>(t->ws + 128);
    t->counters = reinterpret_cast<unsigned long long *>(t->ws + 256);
    t->slots = reinterpret_cast<uint64_t *>(t->ws + head_al);
    t->scratch = reinterpret_cast<float *>(t->ws + t->clear_bytes);
    e = hipMemset(t->ws, 0, t->clear_bytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(t->ws);
        delete t;
        return CF_EHIP;
    }
    *out = t;
    return CF_OK;
}

int cf_team_destroy(cf_team t)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipFree(t->ws);
    delete t;
    return e == hipSuccess ? CF_OK : CF_EHIP;
}

int cf_team_reduce(cf_team t, int32_t teams, int32_t team_size, int32_t op, const float *in, float *out, size_t elems,
                   int32_t mode, void *stream)
{
    int rc = check_call(t, teams, team_size, in, out, elems, mode);
    if (rc != CF_OK) return rc;
    if ((op != CF_TEAM_SUM && op != CF_TEAM_MAX) || elems > t->cap) return CF_EINVAL;
    if (mode != CF_TEAM_TWO_KERNELS && (rc = same_grid(t, teams * team_size)) != CF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const TeamArgs a = make_args(t, in, out, elems, team_size);
    const dim3 grid(teams * team_size), block(kThreads);
    if (mode == CF_TEAM_TWO_KERNELS) {
        hipLaunchKernelGGL(team_stage_kernel, grid, block, 0, s, a);
        if (op == CF_TEAM_SUM)
            hipLaunchKernelGGL(team_reduce_offchip_kernel<cf::team::kSum>, grid, block, 0, s, a);
        else
            hipLaunchKernelGGL(team_reduce_offchip_kernel<cf::team::kMax>, grid, block, 0, s, a);
    } else {
        const int e = values_per_thread(elems);
        Kernel k;
        if (mode == CF_TEAM_TWO_HOPS)
            k = op == CF_TEAM_SUM ? team_reduce_two_hops_kernel<cf::team::kSum> : team_reduce_two_hops_kernel<cf::team::kMax>;
        else if (mode == CF_TEAM_DIRECT)
            k = op == CF_TEAM_SUM ? pick_reduce<cf::team::kSum, true>(e) : pick_reduce<cf::team::kMax, true>(e);
        else
            k = op == CF_TEAM_SUM ? pick_reduce<cf::team::kSum, false>(e) : pick_reduce<cf::team::kMax, false>(e);
        hipLaunchKernelGGL(k, grid, block, 0, s, a);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CF_OK : fail(t, e);
}

int cf_team_gather(cf_team t, int32_t teams, int32_t team_size, const float *in, float *out, size_t elems,
                   int32_t mode, void *stream)
{
    int rc = check_call(t, teams, team_size, in, out, elems, mode);
    if (rc != CF_OK) return rc;
    if (elems * (size_t)team_size > t->cap || mode == CF_TEAM_TWO_HOPS) return CF_EINVAL;
    if (mode != CF_TEAM_TWO_KERNELS && (rc = same_grid(t, teams * team_size)) != CF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const TeamArgs a = make_args(t, in, out, elems, team_size);
    const dim3 grid(teams * team_size), block(kThreads);
    if (mode == CF_TEAM_TWO_KERNELS) {
        hipLaunchKernelGGL(team_stage_kernel, grid, block, 0, s, a);
        hipLaunchKernelGGL(team_gather_offchip_kernel, grid, block, 0, s, a);
    } else if (mode == CF_TEAM_DIRECT) {
        hipLaunchKernelGGL(team_gather_kernel<true>, grid, block, 0, s, a);
    } else {
        hipLaunchKernelGGL(team_gather_kernel<false>, grid, block, 0, s, a);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CF_OK : fail(t, e);
}

int cf_team_status(cf_team t, void *stream)
{
    if (!t) return CF_EINVAL;
    hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(t, e);
    uint32_t flag = 0;
    e = hipMemcpy(&flag, t->err, sizeof flag, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(t, e);
    if (flag) {
        e = hipMemset(t->ws, 0, t->clear_bytes);     // launch counters and all stamps start afresh
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) return fail(t, e);
        return CF_ETIMEOUT;
    }
    return CF_OK;
}

int cf_team_set_spin_limit(cf_team t, int32_t spin_limit_us)
{
    if (!t || spin_limit_us < 0) return CF_EINVAL;
    t->spin_ticks = (long long)spin_limit_us * 100;
    return CF_OK;
}

}  // extern "C"
