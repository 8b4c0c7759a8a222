// What cf_mla.hip (C ABI, the token-range kernel) and cf_mla_heads.hip (the head-team kernel) share.
#ifndef CF_MLA_INTERNAL_H
#define CF_MLA_INTERNAL_H

#include "../../include/cfdecode.h"

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cf {
namespace mla {

constexpr int kHeadsMaxBatch = 4;   // batch rows the head-team kernel's register tiles hold

struct HeadsArgs {
    const uint16_t *x, *wq, *wkv, *wup, *wdown, *wo;
    uint16_t *cache, *out;
    float *qdbg, *zdbg;             // [B][nh][L + R] query (latent | rotated rotary part), [B][nh][L] z: for cf_mla_debug_export
    uint64_t *slots;
    unsigned long long *counters;
    uint32_t *err;
    size_t x1, x2, x3, x5, x6;      // first slot of each exchange area
    int D, nh, n, v, B, pos, max_seq, W;
    int cq, ckv;                    // 16-byte pieces (8 columns) of W_Q / W_KV per column block
    float scale_log2e;              // log2(e) / sqrt(nope_dim + rope_dim)
    double log2_base;
    long long spin_ticks;
};

// first slot of the five exchange areas for batch B; returns the number of slots in all
size_t heads_layout(const cf_mla_config &c, int B, size_t (&first)[5]);
// sets the kernel's LDS attribute; false if no workgroup fits a compute unit
bool heads_prepare();
// enqueues the kernel (a.W workgroups); returns the hipError_t of the launch
int heads_launch(const HeadsArgs &a, void *stream);

}  // namespace mla
}  // namespace cf

#endif
