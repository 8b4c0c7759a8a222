/*
 * cfdecode - one decode step of a transformer attention block as a single fused
 * HIP kernel for AMD MI355X (gfx950).
 *
 * The block is the one the ClusterFusion paper fuses (Alg. 3; definition Eq. 1,
 * decode semantics Sec. 2.1): QKV projection of the new token's hidden state,
 * RoPE on q and k, append of the new key/value to the KV cache, split-KV
 * attention over cached + new token with an online-softmax merge, and the
 * output projection, summed over heads.
 *
 * C ABI, plain pointers and sizes.  Every tensor pointer is a DEVICE pointer to
 * IEEE binary16 ("fp16") data unless stated otherwise, 16-byte aligned, dense
 * row-major with the shapes given below.  The caller owns all tensors; the
 * library owns only a per-handle workspace in device memory.
 *
 * All functions return 0 (CF_OK) or a negative CF_E* code; nothing aborts or
 * throws across this boundary.
 */
#ifndef CFDECODE_H
#define CFDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CF_OK = 0,
    CF_EINVAL = -1,        /* null or misaligned pointer, bad shape, pos or batch out of range */
    CF_EUNSUPPORTED = -2,  /* shape outside the compiled kernel variants, or the grid cannot be co-resident */
    CF_EHIP = -3,          /* a HIP runtime call failed; see cf_last_hip_error */
    CF_ENOMEM = -4,        /* host or device allocation failed */
    CF_ETIMEOUT = -5,      /* a cross-workgroup wait inside the kernel gave up (reported by cf_status) */
    CF_ESCRATCH = -6       /* cf_decode_block_static: the call needs more exchange memory than the fixed scratch array holds */
};

/* Shape of the block (paper Alg. 3 "Require": hidden size D, heads, head dim). */
typedef struct cf_config {
    int32_t d_model;      /* D; multiple of 8 */
    int32_t n_q_heads;    /* query heads */
    int32_t n_kv_heads;   /* key/value heads; n_q_heads % n_kv_heads == 0, ratio in {1,2,4,8} */
    int32_t head_dim;     /* 64 or 128 */
    int32_t max_batch;    /* largest batch a call may use (1..16) */
    int32_t max_seq;      /* capacity (rows) of each KV-cache head slice */
    float   rope_base;    /* RoPE frequency base, e.g. 10000 or 500000 */
    int32_t flags;        /* bit 0: keep q_rot / attention vectors of the last call for cf_debug_export */
} cf_config;

#define CF_FLAG_DEBUG_EXPORT 1

typedef struct cf_handle_s *cf_handle;

/*
 * Create a handle on the current HIP device: validates the shape, allocates and
 * clears the workspace (exchange slots and counters used between workgroups).
 * Synchronous.  A handle must not be used from two streams at the same time.
 */
int cf_create(const cf_config *cfg, cf_handle *out);

/* Free the workspace.  The caller must have synchronised the streams that used it. */
int cf_destroy(cf_handle h);

/*
 * Enqueue one decode step on `stream` (a hipStream_t, NULL for the default
 * stream) and return without waiting.  Paper Alg. 3 with Eq. 1:
 *
 *   [q | k_new | v_new] = x . W_qkv        columns ordered Q heads, K heads, V heads
 *   q, k_new <- RoPE at position pos       pairs (i, i + head_dim/2), angle pos * rope_base^(-2i/head_dim)
 *   k_cache[b, g, pos, :] = fp16(k_new),  v_cache[b, g, pos, :] = fp16(v_new)
 *   a_i = softmax(K_g q_i / sqrt(head_dim))^T V_g   over rows 0..pos (cached rows + the new one),
 *                                                   g = i / (n_q_heads / n_kv_heads)
 *   out = concat_i(a_i) . W_o
 *
 *   x        [batch, d_model]                                  read
 *   W_qkv    [d_model, (n_q_heads + 2 n_kv_heads) * head_dim]  read
 *   W_o      [n_q_heads * head_dim, d_model]                   read
 *   k_cache  [batch, n_kv_heads, max_seq, head_dim]            rows < pos read, row pos written
 *   v_cache  same
 *   pos      number of tokens already cached == index of the new token, 0 <= pos < max_seq
 *   out      [batch, d_model] fp16, fully overwritten (needs no clearing)
 *
 * Storage is fp16, accumulation fp32.  Rows > pos of the caches are neither
 * read nor written.  No allocation and no host synchronisation happen here.
 * Errors: CF_EINVAL for null/misaligned pointers, batch outside 1..max_batch,
 * pos outside 0..max_seq-1; CF_EHIP if the launch fails.
 * Residency: the workgroups of the launch wait for each other's partial results, so all of them must be on
 * the GPU at the same time (one per compute unit; checked once against the kernel's occupancy).  If other work
 * holds compute units while this kernel runs, a workgroup may never start, every wait for it runs to the spin
 * limit (2 s by default, cf_set_tuning), the output of that call is wrong, and the only report is CF_ETIMEOUT
 * from the next cf_status: run the step on a GPU (or partition) of its own and call cf_status where results count.
 */
int cf_decode_block(cf_handle h, int32_t batch, const void *x, const void *W_qkv, const void *W_o,
                    void *k_cache, void *v_cache, int32_t pos, void *out, void *stream);

/*
 * cf_decode_block for callers that cannot allocate device memory: code under HIP graph capture, serving loops and
 * harnesses that forbid hipMalloc.  No handle and no cf_create: the shape is passed with every call, and what the
 * kernel keeps between its workgroups (launch counters, exchange slots, error flag) lives in a fixed array of device
 * memory inside the library (32 MiB on every GPU the library runs on, held until the process ends) in place of a
 * per-handle workspace.  The call itself makes no hipMalloc / hipFree and no allocating library call, does not
 * synchronise, and enqueues on `stream` the fused kernel, preceded by a one-workgroup kernel that re-aligns the
 * launch counters whenever the number of workgroups differs from the previous call's on this GPU.
 *   cfg      shape as for cf_create (max_batch and max_seq as the caches were allocated; flags ignored)
 *   others   exactly as for cf_decode_block (row-major weights)
 * Limits: the exchange slots of the call's work plan must fit the array:
 *   8 bytes * (k_splits * batch * (n_q + 2 n_kv) * head_dim + batch * n_q * kv_splits * (head_dim + 4)
 *              + n_q * out_row_splits * batch * d_model)  <=  32 MiB - 257 KiB
 * (Llama-2-7B shape, batch 1: 2.1 MB; Llama-3-8B shape, batch 16: 30.5 MB); a call beyond that returns CF_ESCRATCH
 * and enqueues nothing.  All calls on one GPU share the array and it keeps the contents of the last call: calls
 * that overlap in time on one GPU (two streams, two host threads) race and give wrong results; calls on one stream,
 * or otherwise ordered, are fine, also with different shapes.  A wait inside the kernel that gives up (the grid was
 * not co-resident) cannot be reported by this entry point: use a handle and cf_status where that matters.
 * Errors otherwise as for cf_create (shape) and cf_decode_block (arguments).
 */
int cf_decode_block_static(const cf_config *cfg, int32_t batch, const void *x, const void *W_qkv, const void *W_o,
                           void *k_cache, void *v_cache, int32_t pos, void *out, void *stream);

/*
 * Optional layout for the (static) weights that lets every workgroup stream one
 * contiguous block instead of a strided column strip; same bytes, same arithmetic.
 * It is the per-head form of Eq. 1 (W_Qi, W_Ki, W_Vi per head):
 *   W_qkv_packed [(n_q + 2 n_kv)][d_model][head_dim]   block j = columns [j*head_dim, (j+1)*head_dim) of W_qkv;
 *                                                        each block is followed by 256 zero bytes, so that
 *                                                        equal positions in different blocks fall into
 *                                                        different memory channels
 *   W_o_packed   [n_q][ceil(d_model/512)][head_dim][512]  tile (i, c) = rows of head i, columns [512c, 512c+512)
 *                                                          of W_o, zero-filled past d_model
 * cf_packed_sizes gives the two buffer sizes in bytes; cf_pack_weights enqueues the
 * rearrangement on `stream` (source and destination must not overlap);
 * cf_decode_block_packed is cf_decode_block taking the packed weights.
 */
int cf_packed_sizes(cf_handle h, size_t *qkv_bytes, size_t *o_bytes);
int cf_pack_weights(cf_handle h, const void *W_qkv, const void *W_o, void *W_qkv_packed, void *W_o_packed,
                    void *stream);
int cf_decode_block_packed(cf_handle h, int32_t batch, const void *x, const void *W_qkv_packed,
                           const void *W_o_packed, void *k_cache, void *v_cache, int32_t pos, void *out,
                           void *stream);

/*
 * The steps of a pre-norm decoder layer that sit directly around the block, in the same single kernel
 * (the paper fuses the block of Eq. 1 and leaves RMSNorm to other libraries, end of Sec. 3):
 *
 *   n_b   = x_b / sqrt(mean_j(x_bj^2) + eps) * norm_weight        (norm_weight != NULL; else n_b = x_b)
 *   out_b = block(n_b)  [+ x_b  when residual != 0]
 *
 * with block() and all other arguments as in cf_decode_block (packed == 0) or cf_decode_block_packed
 * (packed != 0).  norm_weight: DEVICE [d_model] fp16, 16-byte aligned, read.  The mean square is taken in
 * fp32 from the fp16 values of x and the normalised row enters the projection unrounded.  `out` must not
 * overlap `x` (other workgroups may still be reading x when the first results are written).
 * Errors as for cf_decode_block; in addition CF_EINVAL for eps < 0 or not finite, CF_EUNSUPPORTED for a
 * norm_weight with d_model > 8192.
 */
int cf_decode_layer(cf_handle h, int32_t batch, const void *x, const void *norm_weight, float eps, int32_t residual,
                    int32_t packed, const void *W_qkv, const void *W_o, void *k_cache, void *v_cache, int32_t pos,
                    void *out, void *stream);

/*
 * A stack of n_layers layers in one call: layer 0 reads x, layer l reads the hidden state layer l-1 wrote (two
 * buffers of the handle's workspace, used in turn), the last layer writes `out`.  Each layer is cf_decode_layer
 * with its own weights and caches and the common batch, pos, eps, residual and packed; the launch overhead the
 * paper compares in Sec. 4.2 is that of such a stack.  This version enqueues one launch of the fused kernel per
 * layer on `stream`.
 *   W_qkv, W_o, k_cache, v_cache: HOST arrays of n_layers DEVICE pointers (read during the call only), each as in
 *   cf_decode_layer; norm_weight: NULL (no RMSNorm in any layer) or a HOST array of n_layers DEVICE pointers.
 *   x and out must differ.  Errors as for cf_decode_layer; a pointer of any layer that is null or misaligned is
 *   CF_EINVAL before anything is enqueued; after another error the layers before the failing one have been enqueued.
 */
int cf_decode_stack(cf_handle h, int32_t n_layers, int32_t batch, const void *x, const void *const *norm_weight, float eps,
                    int32_t residual, int32_t packed, const void *const *W_qkv, const void *const *W_o,
                    void *const *k_cache, void *const *v_cache, int32_t pos, void *out, void *stream);

/*
 * cf_decode_layer for a batch whose rows have different lengths (continuous batching): row b has row_pos[b]
 * cached tokens; its query and new key are rotated for position row_pos[b], it attends to its rows
 * 0 .. row_pos[b] and its new key / value go to row row_pos[b] of its cache slice.  Rows of a batch are
 * independent in Eq. 1, so this is the block applied row by row with each row's own position.
 *   row_pos  DEVICE [batch] int32, 4-byte aligned, read by the kernel (it may be written by earlier work on
 *            `stream`); 0 <= row_pos[b] <= max_pos.  Entries outside that range are clamped into it.
 *   max_pos  HOST value, an upper bound of the entries, 0 <= max_pos < max_seq: the work is split as for a batch
 *            with max_pos cached tokens in every row (shorter rows leave their last splits empty).
 * norm_weight may be NULL and residual 0: then this is the bare block with per-row positions.
 */
int cf_decode_layer_rows(cf_handle h, int32_t batch, const void *x, const void *norm_weight, float eps,
                         int32_t residual, int32_t packed, const void *W_qkv, const void *W_o, void *k_cache,
                         void *v_cache, const int32_t *row_pos, int32_t max_pos, void *out, void *stream);

/*
 * Wait for `stream` and report whether any kernel launched through this handle
 * gave up on a cross-workgroup wait (CF_ETIMEOUT) since the last cf_status
 * call.  The fused kernel relies on all its workgroups being resident at once
 * (Alg. 3 has the same requirement for the blocks of a cluster); a wait that
 * exceeds the spin limit sets a flag instead of hanging.
 */
int cf_status(cf_handle h, void *stream);

/*
 * Copy intermediate vectors of the most recent call to HOST memory (handle must
 * have CF_FLAG_DEBUG_EXPORT).  what = 0: rotated queries [batch, n_q_heads,
 * head_dim]; what = 1: per-head attention outputs a_i, same shape (Alg. 3 step
 * 7 result).  fp32.  what = 2: [workgroups][24] uint64 stamps of the 100 MHz wall
 * clock taken by every workgroup (all zero unless the library was built with
 * -DCF_STAMPS=1, as libcfdecode_trace.so is): 0 start, 1 projection done, 2 x staged
 * in LDS, 3 attention done, 4 output projection done, 5 final reduction done, 6 exit,
 * 7 hardware id (XCC / CU) instead of a time, 8 attention row groups merged,
 * 9 new token handled, 10 attention partial stored, 11 attention merged, 12 / 21 first /
 * second weight batch issued, 14 rotated queries ready, 15 K/V stream consumed,
 * 16 first projection step consumed, 17 output tile multiplied, 18 output partial
 * stored, 19 head partials arrived, 20 projection set up; others unused.
 * Synchronises `stream`.  `bytes` must equal the tensor size.
 */
int cf_debug_export(cf_handle h, int32_t what, void *host_dst, size_t bytes, void *stream);

/*
 * Tuning knobs (all optional; 0 keeps the default): workgroups per launch,
 * split count of the projection's reduction dimension, split count of the KV
 * sequence, spin limit of the in-kernel waits in microseconds (-1: every wait gives up at its first
 * unsuccessful look, which makes any launch report CF_ETIMEOUT: for tests of the error path).  Alg. 3's
 * "cluster size" corresponds to workgroups / n_kv_heads.  Returns CF_EINVAL for
 * values the shape cannot use.  A change of the workgroup count waits for the
 * device and clears the workspace, so call it between steps, not inside a hot loop.
 */
int cf_set_tuning(cf_handle h, int32_t workgroups, int32_t k_splits, int32_t kv_splits, int32_t spin_limit_us);

/* Plan of the most recent call, for reports: fills up to n ints
 * {workgroups, team_size, k_splits, rows_per_split, kv_splits, tokens_per_split,
 *  out_col_blocks, out_cols_per_block, out_row_splits, lds_bytes}. */
int cf_get_plan(cf_handle h, int32_t *dst, int32_t n);

/* Algorithmic HBM bytes of one call (weights + cached K/V rows + appended rows + x + out). */
int64_t cf_algorithmic_bytes(const cf_config *cfg, int32_t batch, int32_t pos);

const char *cf_strerror(int code);

/* hipError_t of the most recent failing HIP call made through this handle (0 if none). */
int cf_last_hip_error(cf_handle h);

/* ------------------------------------------------------------------------------------------------
 * Team collectives: the paper's two cluster-level primitives (Sec. 3.2; ClusterReduce, Alg. 1, and
 * ClusterGather, Alg. 2) among co-resident workgroups of one kernel, exchanged through stamped slots in
 * global memory in place of distributed shared memory, and -- for the comparison of the paper's Table 1 --
 * the same results from two kernels that hand the data over through a buffer in global memory.
 *
 * A launch has teams * team_size workgroups ("ranks"); team k consists of ranks k*team_size .. +team_size-1
 * (team_size = N = 1, 2, 4, 8 or 16, as in the paper).  All pointers are DEVICE pointers to fp32, 4-byte
 * aligned; the caller owns them.  Calls are asynchronous on `stream`; a handle must not be used from two
 * streams at once.  All ranks of a launch have to be resident together (one per compute unit): more ranks
 * than compute units is CF_EUNSUPPORTED.
 */
typedef struct cf_team_s *cf_team;
enum { CF_TEAM_SUM = 0, CF_TEAM_MAX = 1 };
/* How the ranks exchange their data (argument `mode`):
 *   CF_TEAM_ROUNDS       one kernel, the paper's schedule: log2(N) rounds, in round s rank b sends to rank
 *                        (b + 2^s) mod N (Alg. 1, Alg. 2);
 *   CF_TEAM_TWO_KERNELS  a kernel that writes every rank's buffer to global memory and a second one that reads
 *                        what each rank needs (the "off-chip" column of Table 1);
 *   CF_TEAM_DIRECT       one kernel, one hop: every rank posts its buffer once and reads the N - 1 others
 *                        (the schedule the fused decode kernel uses: a hop through memory costs microseconds,
 *                        so fewer hops win over fewer bytes for small buffers);
 *   CF_TEAM_TWO_HOPS     reduce only: one kernel, two hops, fewest bytes: rank b folds slice b of the buffer
 *                        from the others' posts, posts the result and reads the other slices from their owners
 *                        (a rank receives 2 (N-1)/N * elems values, against (N-1) * elems in one hop). */
enum { CF_TEAM_ROUNDS = 0, CF_TEAM_TWO_KERNELS = 1, CF_TEAM_DIRECT = 2, CF_TEAM_TWO_HOPS = 3 };

/* max_ranks: most workgroups a launch may have; max_elems: most fp32 values a rank may hold in a reduce,
 * or receive in a gather (team_size * elems), at most 65536.  Allocates and clears the exchange area
 * (max_ranks * 4 * max_elems * 8 bytes) and a scratch buffer for the two-kernel versions.  Synchronous. */
int cf_team_create(int32_t max_ranks, size_t max_elems, cf_team *out);
int cf_team_destroy(cf_team t);

/* All-reduce (Alg. 1):  in, out [teams][team_size][elems];  out[k][b][:] = op over b' of in[k][b'][:], the same
 * for every rank b of team k.  fp32; the sum is folded in the order of Alg. 1's rounds (round s adds the
 * buffer of rank (b - 2^s) mod N as it stands after round s-1), so it is deterministic.  The other modes
 * add the ranks in rank order (all ranks of a team then hold the same bits). */
int cf_team_reduce(cf_team t, int32_t teams, int32_t team_size, int32_t op, const float *in, float *out,
                   size_t elems, int32_t mode, void *stream);

/* All-gather (Alg. 2):  in [teams][team_size][elems], out [teams][team_size][team_size][elems];
 * out[k][b][j][:] = in[k][(b - j) mod N][:]  (segment 0 is the rank's own data, as in Alg. 2). */
int cf_team_gather(cf_team t, int32_t teams, int32_t team_size, const float *in, float *out, size_t elems,
                   int32_t mode, void *stream);

/* Wait for `stream`; CF_ETIMEOUT if a rank gave up waiting for a peer since the last call (the exchange
 * area is cleared then). */
int cf_team_status(cf_team t, void *stream);
/* Limit of the in-kernel waits in microseconds; 0: every wait gives up at its first unsuccessful look (any launch then
 * reports CF_ETIMEOUT: for tests of the error path). */
int cf_team_set_spin_limit(cf_team t, int32_t spin_limit_us);

/* ------------------------------------------------------------------------------------------------
 * Fused decode step of a Multi-Head Latent Attention block in its weight-absorbed form (paper Appendix B:
 * Q = Hidden W_Q W_Up, K = Hidden W_K, V = K[:kv_lora_rank]; Alg. 4), one kernel:
 *
 *   q_i = x W_Q[:, head i] -> (q_nope_i [nope_dim] | q_rope_i [rope_dim]);   kv_new = x W_KV -> (c_new | k_rope_new)
 *   q_rope_i, k_rope_new <- RoPE at position pos (pairs (d, d + rope_dim/2), angle pos * rope_base^(-2d/rope_dim))
 *   kv_cache[b, pos, :] = fp16(c_new | k_rope_new)                            one latent row shared by all heads
 *   q_lat_i = q_nope_i W_Up[i];   s_i = ((q_lat_i | q_rope_i) . K^T) / sqrt(nope_dim + rope_dim)  over rows 0..pos
 *   z_i = softmax(s_i) . K[:, :kv_lora_rank];   a_i = z_i W_Down[i];   out = concat_i(a_i) W_O
 *
 * All pointers are DEVICE pointers to fp16 (IEEE binary16), 16-byte aligned, row-major; the caller owns them:
 *   x [batch, d_model]; W_q [d_model, n_heads * (nope_dim + rope_dim)] (per head: nope part, rope part);
 *   W_kv [d_model, kv_lora_rank + rope_dim]; W_up [n_heads, nope_dim, kv_lora_rank];
 *   W_down [n_heads, kv_lora_rank, v_head_dim]; W_o [n_heads * v_head_dim, d_model];
 *   kv_cache [batch, max_seq, kv_lora_rank + rope_dim]: rows < pos read, row pos written; out [batch, d_model].
 * Storage fp16, accumulation fp32.  Asynchronous on `stream`; no allocation, no host synchronisation.
 * The kernel is written for kv_lora_rank 512, rope_dim 64, n_heads <= 16 (one MFMA tile of heads; 16 workgroups per
 * head, all resident), batch <= 16 (the batch of Appendix C), nope_dim a multiple of 8 up to 128, v_head_dim a
 * multiple of 8 up to 128, d_model a multiple of 32, at most 8192 and at most 128 * n_heads: cf_mla_create returns
 * CF_EUNSUPPORTED otherwise.  cf_mla_status is cf_status for this handle.
 * Two kernels: at batch 1 every head scans the cached rows itself (16 workgroups per head, vector arithmetic);
 *   from batch 2 on the unit of work of the attention stage is a range of cached rows of one batch row, for a group of
 *   heads at once, as two products on MFMA tiles.
 * cf_mla_set_splits: upper limit on the number of token ranges a batch row's cached rows are divided into; 0 = chosen
 *   by the library, at most 32.  A non-zero limit also selects the token-range kernel at batch 1.  For tests of
 *   the range logic and for measurements; CF_EINVAL outside 0..32.
 * cf_mla_debug_export: intermediate results of the last call on this handle, copied to the host buffer as fp32 after
 *   synchronising `stream`: what = 0: q_lat [batch, n_heads, kv_lora_rank] (Alg. 4's absorbed query); 1: q_rope
 *   [batch, n_heads, rope_dim] (rotated); 2: z [batch, n_heads, kv_lora_rank] (the attention result in the latent
 *   space, before W_Down).  `bytes` must equal the tensor size (CF_EINVAL otherwise, and before any call).
 */
typedef struct cf_mla_config {
    int32_t d_model, n_heads, nope_dim, rope_dim, kv_lora_rank, v_head_dim;
    int32_t max_batch, max_seq;
    float rope_base;
} cf_mla_config;
typedef struct cf_mla_s *cf_mla;

int cf_mla_create(const cf_mla_config *cfg, cf_mla *out);
int cf_mla_destroy(cf_mla t);
int cf_mla_decode(cf_mla t, int32_t batch, const void *x, const void *W_q, const void *W_kv, const void *W_up,
                  const void *W_down, const void *W_o, void *kv_cache, int32_t pos, void *out, void *stream);
int cf_mla_status(cf_mla t, void *stream);
int cf_mla_set_spin_limit(cf_mla t, int32_t spin_limit_us);   /* as cf_team_set_spin_limit */
int cf_mla_set_splits(cf_mla t, int32_t max_splits);
int cf_mla_debug_export(cf_mla t, int32_t what, void *host_dst, size_t bytes, void *stream);
/* Algorithmic HBM bytes of one call (all weights + cached rows + appended rows + x + out). */
int64_t cf_mla_algorithmic_bytes(const cf_mla_config *cfg, int32_t batch, int32_t pos);

/* ------------------------------------------------------------------------------------------------
 * The SplitHead dataflow (paper Appendix B, Alg. 5) of the decode step of cf_decode_block: the same operation on
 * the same tensors, with the work divided the other way, as the ablation the paper measures against its
 * SplitToken dataflow (Alg. 3).  A head is a team of `team_size` workgroups (Alg. 5's cluster of N blocks) that
 * split the head dimension in the projection, the attention and the output projection; the partial scores of all
 * tokens and the partial output projection are summed over the team (Alg. 5's two ClusterReduce), the heads are
 * summed with atomicAdd.  One kernel per call.
 *
 * cf_splithead_create: cfg as for cf_create.  Written for batch 1 (max_batch == 1), n_kv_heads == n_q_heads,
 *   head_dim 64 or 128, team_size 2, 4 or 8 with head_dim % (16 * team_size) == 0, n_q_heads * team_size not above
 *   the number of compute units, and (d_model + max_seq + 64) * 4 bytes of LDS at most 150 KiB (the scores of all
 *   tokens stay on chip): CF_EUNSUPPORTED otherwise.  Allocates and clears the exchange workspace; synchronous.
 * cf_splithead_pack: one-time rearrangement of W_qkv [d_model, 3 * n_q_heads * head_dim] (as for cf_decode_block)
 *   into W_qkv_members (same size, caller-owned, must not overlap), where the columns of every team member are
 *   contiguous: [head][member][d_model][q lo | q hi | k lo | k hi | v lo | v hi], each part head_dim / (2 *
 *   team_size) values, "lo" the member's dimensions below head_dim / 2 and "hi" their RoPE partners.  Asynchronous.
 * cf_splithead_decode: x [1, d_model], W_o, k_cache, v_cache [1, n_heads, max_seq, head_dim], pos and out [1,
 *   d_model] as for cf_decode_block (rows < pos read, row pos written).  Asynchronous on `stream`, no allocation.
 *   The stamp of a launch is counted on the device (every workgroup counts the launches it has completed), so a
 *   captured launch can be replayed.  The order of the atomic additions, and with it the last bits of the result, is
 *   not fixed.
 * cf_splithead_status / cf_splithead_set_spin_limit: as cf_team_status / cf_team_set_spin_limit; in addition a limit
 *   of -1 makes every launch report CF_ETIMEOUT whatever the timing (only member 0 of every team runs and gives up at
 *   its first look for the posts of the others): for tests of the error path.  Every wait still ends.
 */
typedef struct cf_splithead_s *cf_splithead;
int cf_splithead_create(const cf_config *cfg, int32_t team_size, cf_splithead *out);
int cf_splithead_destroy(cf_splithead t);
int cf_splithead_pack(cf_splithead t, const void *W_qkv, void *W_qkv_members, void *stream);
int cf_splithead_decode(cf_splithead t, const void *x, const void *W_qkv_members, const void *W_o, void *k_cache,
                        void *v_cache, int32_t pos, void *out, void *stream);
int cf_splithead_status(cf_splithead t, void *stream);
int cf_splithead_set_spin_limit(cf_splithead t, int32_t spin_limit_us);

/* ------------------------------------------------------------------------------------------------
 * The feed-forward block of a decoder layer for one token per sequence, one kernel (paper Sec. 2.1:
 * FFN(Z) = W3 (sigma(W1 Z) * W2 Z), three linear layers with an activation in between, * element-wise):
 *
 *   h = W1 z_b,  u = W2 z_b   [d_ff]      g = sigma(h) * u      out_b = g W3   [d_model]        for every batch row b
 *
 * All pointers are DEVICE pointers to fp16, 16-byte aligned, row-major; the caller owns them:
 *   z [batch, d_model] read;  W1, W2, W3 [d_ff, d_model] read (row f: the weights of hidden unit f into it, for W1 and
 *   W2, and out of it, for W3; for W1 and W2 that is the [out_features, in_features] layout of the paper's "W1 Z");
 *   out [batch, d_model] fully overwritten.  Storage fp16, accumulation fp32; the hidden vector is never rounded.
 * activation: CF_FFN_SILU, sigma(a) = a / (1 + exp(-a)) (the Llama-family layers whose shapes the paper measures), or
 *   CF_FFN_GELU, a Phi(a) in its exact form (the paper's example).
 * cf_ffn_create allocates and clears the exchange workspace (synchronous): CF_EINVAL for d_model not a multiple of 8,
 *   sizes below 1 or an unknown activation; CF_EUNSUPPORTED for max_batch > 16 (the batch of Appendix C), d_model >
 *   8192, matrices of 2 GiB or more; with max_batch > 4 also for fewer workgroups than a multiple of 16 (d_ff below
 *   the number of compute units and not a multiple of 16) and for more than 128 hidden units per workgroup.
 *   Two kernels: the products on the vector units with one partial output per workgroup (batch 1; also 2 to 4 where
 *   the second kernel does not take the shape), and from batch 2 on the products on MFMA tiles, the workgroups cut into
 *   slices of hidden units times slices of output columns.
 * cf_ffn_decode enqueues the kernel on `stream` (no allocation, no synchronisation; the launch can be captured and
 *   replayed): CF_EINVAL for null or misaligned pointers and a batch outside 1..max_batch.  All workgroups must be
 *   resident together (one per compute unit), as for cf_decode_block.
 * cf_ffn_status / cf_ffn_set_spin_limit: as cf_team_status / cf_team_set_spin_limit.
 */
enum { CF_FFN_SILU = 0, CF_FFN_GELU = 1 };
typedef struct cf_ffn_config {
    int32_t d_model, d_ff, max_batch, activation;
} cf_ffn_config;
typedef struct cf_ffn_s *cf_ffn;
int cf_ffn_create(const cf_ffn_config *cfg, cf_ffn *out);
int cf_ffn_destroy(cf_ffn t);
int cf_ffn_decode(cf_ffn t, int32_t batch, const void *z, const void *W1, const void *W2, const void *W3, void *out,
                  void *stream);
int cf_ffn_status(cf_ffn t, void *stream);
int cf_ffn_set_spin_limit(cf_ffn t, int32_t spin_limit_us);
/* Algorithmic HBM bytes of one call (the three matrices + z + out). */
int64_t cf_ffn_algorithmic_bytes(const cf_ffn_config *cfg, int32_t batch);

#ifdef __cplusplus
}
#endif
#endif /* CFDECODE_H */
