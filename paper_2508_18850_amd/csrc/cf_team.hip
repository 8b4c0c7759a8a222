// Team collectives behind the C ABI (cf_team_* in include/cfdecode.h): kernels that run the paper's
// ClusterReduce / ClusterGather schedules (Alg. 1, Alg. 2) among co-resident workgroups through stamped
// exchange slots, and the two-kernel versions that go through a scratch buffer in global memory instead
// (the "off-chip" column of the paper's Table 1).
#include "../../include/cfdecode.h"
#include "cf_team_device.h"

#include <cstdlib>
#include <new>

namespace {

using cf::team::kThreads;
constexpr int kCounterStride = 16;      // 64-bit words between the launch counters of two workgroups

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

template <int E, int OP>
__global__ void __launch_bounds__(kThreads) team_reduce_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N, tid = threadIdx.x;
    unsigned long long cnt;
    const cf::team::Exchange x = {a.slots, a.cap, launch_stamp(a, cnt), a.err, a.spin_ticks};
    const float *src = a.in + (size_t)w * a.count;
    float *dst = a.out + (size_t)w * a.count;
    float d[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const size_t i = tid + (size_t)kThreads * e;
        d[e] = i < a.count ? src[i] : 0.f;
    }
    cf::team::reduce<E, OP>(x, team * a.N, a.N, b, a.count, d);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const size_t i = tid + (size_t)kThreads * e;
        if (i < a.count) dst[i] = d[e];
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

// count = values of one segment; a rank's output has N segments
template <int E>
__global__ void __launch_bounds__(kThreads) team_gather_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N, tid = threadIdx.x;
    unsigned long long cnt;
    const cf::team::Exchange x = {a.slots, a.cap, launch_stamp(a, cnt), a.err, a.spin_ticks};
    const float *src = a.in + (size_t)w * a.count;
    float *dst = a.out + (size_t)w * a.count * a.N;
    float g[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const size_t i = tid + (size_t)kThreads * e;
        g[e] = i < a.count ? src[i] : 0.f;
    }
    cf::team::gather<E>(x, team * a.N, a.N, b, a.count, g);
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const size_t i = tid + (size_t)kThreads * e;
        if (i < a.count * a.N) dst[i] = g[e];
    }
    if (tid == 0) a.counters[(size_t)w * kCounterStride] = cnt;
}

// ---- the two-kernel versions: every rank writes its buffer to global memory, the kernel boundary is the
//      synchronisation, then every rank reads what it needs
__global__ void __launch_bounds__(kThreads) team_stage_kernel(const TeamArgs a)
{
    const size_t w = blockIdx.x;
    for (size_t i = threadIdx.x; i < a.count; i += kThreads) a.scratch[w * a.count + i] = a.in[w * a.count + i];
}

template <int OP>
__global__ void __launch_bounds__(kThreads) team_reduce_offchip_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N;
    for (size_t i = threadIdx.x; i < a.count; i += kThreads) {
        float v = a.scratch[(size_t)team * a.N * a.count + i];
        for (int r = 1; r < a.N; ++r) {
            const float o = a.scratch[((size_t)team * a.N + r) * a.count + i];
            v = OP == cf::team::kSum ? v + o : fmaxf(v, o);
        }
        a.out[(size_t)w * a.count + i] = v;
    }
}

__global__ void __launch_bounds__(kThreads) team_gather_offchip_kernel(const TeamArgs a)
{
    const int w = blockIdx.x, team = w / a.N, b = w % a.N;
    for (int j = 0; j < a.N; ++j) {
        const int r = (b - j + a.N) % a.N;
        for (size_t i = threadIdx.x; i < a.count; i += kThreads)
            a.out[((size_t)w * a.N + j) * a.count + i] = a.scratch[((size_t)team * a.N + r) * a.count + i];
    }
}

using Kernel = void (*)(const TeamArgs);

template <int OP>
Kernel pick_reduce(int e)
{
    switch (e) {
    case 1: return team_reduce_kernel<1, OP>;
    case 2: return team_reduce_kernel<2, OP>;
    case 4: return team_reduce_kernel<4, OP>;
    case 8: return team_reduce_kernel<8, OP>;
    case 16: return team_reduce_kernel<16, OP>;
    case 32: return team_reduce_kernel<32, OP>;
    case 64: return team_reduce_kernel<64, OP>;
    case 128: return team_reduce_kernel<128, OP>;
    }
    return nullptr;
}

Kernel pick_gather(int e)
{
    switch (e) {
    case 1: return team_gather_kernel<1>;
    case 2: return team_gather_kernel<2>;
    case 4: return team_gather_kernel<4>;
    case 8: return team_gather_kernel<8>;
    case 16: return team_gather_kernel<16>;
    case 32: return team_gather_kernel<32>;
    case 64: return team_gather_kernel<64>;
    case 128: return team_gather_kernel<128>;
    }
    return nullptr;
}

// values per thread, rounded up to a compiled variant; 0 if too many
int values_per_thread(size_t values)
{
    const size_t need = (values + kThreads - 1) / kThreads;
    for (int e = 1; e <= 128; e *= 2)
        if ((size_t)e >= need) return e;
    return 0;
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

int check_call(cf_team t, int32_t teams, int32_t team_size, const void *in, const void *out, size_t elems)
{
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
    if (!out || max_ranks < 1 || max_elems < 1 || max_elems > (size_t)kThreads * 128) return CF_EINVAL;
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
                   int32_t offchip, void *stream)
{
    int rc = check_call(t, teams, team_size, in, out, elems);
    if (rc != CF_OK) return rc;
    if ((op != CF_TEAM_SUM && op != CF_TEAM_MAX) || elems > t->cap) return CF_EINVAL;
    if (!offchip && (rc = same_grid(t, teams * team_size)) != CF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const TeamArgs a = make_args(t, in, out, elems, team_size);
    const dim3 grid(teams * team_size), block(kThreads);
    if (offchip) {
        hipLaunchKernelGGL(team_stage_kernel, grid, block, 0, s, a);
        if (op == CF_TEAM_SUM)
            hipLaunchKernelGGL(team_reduce_offchip_kernel<cf::team::kSum>, grid, block, 0, s, a);
        else
            hipLaunchKernelGGL(team_reduce_offchip_kernel<cf::team::kMax>, grid, block, 0, s, a);
    } else {
        const int e = values_per_thread(elems);
        Kernel k = op == CF_TEAM_SUM ? pick_reduce<cf::team::kSum>(e) : pick_reduce<cf::team::kMax>(e);
        if (!k) return CF_EUNSUPPORTED;
        hipLaunchKernelGGL(k, grid, block, 0, s, a);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CF_OK : fail(t, e);
}

int cf_team_gather(cf_team t, int32_t teams, int32_t team_size, const float *in, float *out, size_t elems,
                   int32_t offchip, void *stream)
{
    int rc = check_call(t, teams, team_size, in, out, elems);
    if (rc != CF_OK) return rc;
    if (elems * (size_t)team_size > t->cap) return CF_EINVAL;
    if (!offchip && (rc = same_grid(t, teams * team_size)) != CF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const TeamArgs a = make_args(t, in, out, elems, team_size);
    const dim3 grid(teams * team_size), block(kThreads);
    if (offchip) {
        hipLaunchKernelGGL(team_stage_kernel, grid, block, 0, s, a);
        hipLaunchKernelGGL(team_gather_offchip_kernel, grid, block, 0, s, a);
    } else {
        Kernel k = pick_gather(values_per_thread(elems * (size_t)team_size));
        if (!k) return CF_EUNSUPPORTED;
        hipLaunchKernelGGL(k, grid, block, 0, s, a);
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
    if (!t || spin_limit_us < 1) return CF_EINVAL;
    t->spin_ticks = (long long)spin_limit_us * 100;
    return CF_OK;
}

}  // extern "C"
