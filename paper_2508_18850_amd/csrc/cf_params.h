// Internal: kernel argument block and launcher interface shared by the host
// side (cf_api.hip) and the device side (cf_fused_kernel.hip) of libcfdecode.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {

constexpr int kThreads = 512;              // threads per workgroup (8 wavefronts of 64)
constexpr int kWaves = kThreads / 64;
constexpr int kOutChunk = 512;             // output columns one wavefront covers with one 128-bit load per lane
constexpr int kP2Stride = 4;               // floats in front of the accumulator in a split-KV partial: m, l, pad, pad
constexpr int kStamps = 24;                // debug time stamps per workgroup
// Bytes between the end of one per-head block of the packed W_qkv and the start of the next.  With
// power-of-two block sizes all workgroups would walk through the memory channels in step (measured:
// a tenth less bandwidth); 256 bytes shift each block by one channel.
constexpr int kQkvBlockPad = 256;
constexpr int kCounterStride = 16;   // 64-bit words between the launch counters of two workgroups (one 128-byte line each)
constexpr int kMaxKSplits = 64;
constexpr int kMaxKvSplits = 64;

// Batch tile 16 with head_dim 128 runs both projections on MFMA tiles; x then sits in LDS as fp16 operands,
// [16][xs16_stride(rows of the longest split)] halves, twice (high parts, low parts of x * gamma).
__host__ __device__ constexpr bool mfma_tiles(int head_dim, int batch_tile) { return batch_tile == 16 && head_dim == 128; }
__host__ __device__ constexpr int xs16_stride(int rps) { return ((rps + 7) & ~7) + 8; }
// LDS floats that hold x in phase 1
__host__ __device__ constexpr size_t x_lds_floats(int head_dim, int batch_tile, int rps)
{
    return mfma_tiles(head_dim, batch_tile) ? (size_t)16 * xs16_stride(rps) : (size_t)batch_tile * rps;
}

constexpr int kFlagPacked = 1;     // weights are in the packed (per-head contiguous) layout of cf_pack_weights
constexpr int kFlagResidual = 2;   // out = x + block output

// Everything the fused kernel needs, passed by value (256 bytes: four 64-byte lines, fetched together at kernel start).
struct LayerPtrs {             // what differs from layer to layer of a stack
    const uint16_t *wqkv, *wo;
    uint16_t *kc, *vc;
};
struct Params {
    const uint16_t *x;
    const uint16_t *wqkv, *wo; // these four in the order of LayerPtrs: the kernel reads them as one
    uint16_t *kc, *vc;
    const int32_t *row_pos;    // [B] tokens cached for each batch row (at most pos), or null: pos for every row
    const uint16_t *gamma;     // [D] RMSNorm weight applied to x in front of the projection, or null: x is used as it is
    uint16_t *out;
    // workspace
    unsigned long long *done;  // [workgroups][kCounterStride]: launches that workgroup w has completed
    uint32_t *err;         // set to 1 when a spin gave up
    // exchange slots: 64-bit {fp32 bits, launch stamp} pairs
    uint64_t *p1;          // [k_splits][B][Nqkv] partial projections
    uint64_t *p2;          // [B][n_q][kv_splits][head_dim + kP2Stride] split-KV partials
    uint64_t *p3;          // [n_q * row_splits][B][D] per-head partial outputs
    double rope_log2_base; // log2 of the RoPE base: the kernel computes the frequencies base^(-2i/d) itself
    float *dbg_q, *dbg_attn;   // [B][n_q][head_dim] or null
    unsigned long long *dbg_t; // [W][kStamps] wall-clock stamps at phase boundaries, or null
    int D, nq, nkv, B, pos, max_seq, nqkv;
    int W, TS;             // workgroups, workgroups per team (team = one KV head)
    int KS, RPS;           // projection: splits of the reduction dimension, rows of the longest split (LDS stride)
    int RB, RD;            // rows of a split are RB + RD (even split index) or RB - RD (odd)
    int TD;                // attention: tokens of a split are TPS + TD (even split index) or TPS - TD (odd)
    int DSEL;              // TS / KS: selectors advance by this much from one step of a member to the next
    int sh_nkv, sh_ks, sh_dsel, sh_ns;   // log2 of nkv, KS, DSEL, NS where that is a power of two, else -1
    int pairmap;           // workgroup -> (team, member) keeps the parity of the workgroup id in the member id
    int NS, TPS;           // attention: splits of the cached sequence, tokens per split
    int NC3, CW3, RS3;     // output projection: column blocks, columns per block, row splits per head
    int reserved0;
    int flags;             // kFlagPacked, kFlagResidual
    float qk_scale_log2e;  // log2(e)/sqrt(head_dim)
    float eps;             // RMSNorm: added to the mean square
    uint32_t spin_ticks;   // wait limit in 100 MHz ticks (at most 42 s)
};

// A stack of layers in one launch (cf_decode_stack without RMSNorm and residual): the pointers of every layer travel
// by value in the kernel's argument block, behind the parameters of the first layer.
constexpr int kMaxStackLayers = 88;        // 256 + 16 + 88 * 32 bytes = 3088 of the 4096 an argument block may have
struct StackArgs {
    Params p;                  // everything of layer 0, and what all layers share
    uint64_t *xslots;          // [B][D] stamped fp32: the hidden state between two layers
    int n_layers, reserved;
    LayerPtrs tab[kMaxStackLayers];
};

// The kernel exists twice: the block alone, and the block with the RMSNorm prologue, the residual epilogue
// and per-row positions
// (a translation unit of its own, compiled from the same source with -DCF_LAYER=1, so that the block kernel
// carries none of that code).
bool wants_layer_kernel(const Params &p);
// Launch the variant for (head_dim, group size, batch tile).  Returns a hipError_t.
hipError_t launch_fused(const Params &p, int head_dim, int group, int batch_tile, size_t lds_bytes,
                        hipStream_t stream);
// The block kernel over a.n_layers layers in one launch (a.p must not ask for RMSNorm, residual or per-row positions).
hipError_t launch_fused_stack(const StackArgs &a, int head_dim, int group, int batch_tile, size_t lds_bytes,
                              hipStream_t stream);
// Workgroups of that variant that fit on one CU with `lds_bytes` of LDS each (0 = variant missing).
hipError_t max_workgroups_per_cu(int head_dim, int group, int batch_tile, size_t lds_bytes, bool layer, int *out);
// the same two for the layer kernel (defined by the -DCF_LAYER=1 translation unit; called by the two above)
hipError_t launch_fused_layer(const Params &p, int head_dim, int group, int batch_tile, size_t lds_bytes,
                              hipStream_t stream);
hipError_t max_workgroups_per_cu_layer(int head_dim, int group, int batch_tile, size_t lds_bytes, int *out);
// LDS floats needed by the three phases for the given plan.
size_t lds_floats(const Params &p, int head_dim, int group, int batch_tile);
// XCC id of every workgroup of a W-workgroup launch (host buffer of W ints).
// Rearrange row-major weights into the packed layout (see cf_pack_weights in the public header).
hipError_t launch_pack(const uint16_t *wqkv, const uint16_t *wo, uint16_t *wqkv_p, uint16_t *wo_p, int D, int nqkv,
                       int nq, int head_dim, hipStream_t stream);

}  // namespace cf
