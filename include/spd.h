/*
 * spd.h - C ABI of the MI355X (gfx950) Sync-Point-Drop decoder-block library.
 *
 * What the library computes (arXiv 2502.20727).  Tensor parallelism splits every decoder
 * block over `tp_degree` devices: the query/key/value projections by columns (each
 * device owns n_heads / tp_degree whole heads, Sec. 4.2.3), the attention output
 * projection and the MLP down projection by rows (Sec. 4.1.2).  Device i produces a
 * partial attention output Y_i and a partial MLP output Z_i, and a TP block all-reduces
 * both (two sync points per block, Sec. 3, Fig. 1a).  An SPD block (Sec. 4.1.1, Fig. 3a,
 * the design without linear-layer bias) drops the first all-reduce: the device feeds
 * X + Y_i to its MLP, adds Y_i to Z_i before the remaining all-reduce and X after it,
 * giving X + sum_i Y_i + sum_i Z_i.  A per-layer mask (the outcome of Alg. 1) says which
 * blocks are SPD blocks.
 *
 * This library runs ONE device's share ("rank") of such blocks on one GPU.  A sync point
 * that is kept is not a collective between GPUs: it is a sum, in HBM, over `tp_degree`
 * buffers ("slots") of which this rank writes its own and the caller supplies the
 * others.  With rank = SPD_ALL_RANKS the library runs every rank's share in turn and so
 * emulates the whole TP group exactly.
 *
 * Block internals (the paper only says "LLaMA2"): pre-norm RMSNorm with eps inside the
 * square root; rotary embedding, rotate-half convention (pair (j, j + d/2) rotated by
 * pos * rope_base^(-2j/d)), on queries and keys; causal softmax attention with scale
 * 1/sqrt(head_dim) over a KV cache, grouped KV heads (query head j reads KV head
 * j / (q_heads / kv_heads)); SwiGLU MLP (silu(x Wg) * (x Wu)) Wd.
 *
 * General conventions
 *  - Plain C, no exceptions cross the boundary.  Every int-returning call returns SPD_OK
 *    (0) or a negative SPD_E* code; spd_strerror() names it.  All argument checks run on
 *    the host before anything is enqueued, so a failing call has launched nothing.
 *  - The caller owns every buffer.  Forward calls allocate nothing, free nothing and never
 *    synchronise; they only enqueue kernels on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream).  spd_workspace_init() is the only call that copies from
 *    host memory to the device (spd_block_forward_static() does the same copy by itself
 *    when it has to, see there).
 *  - "device" pointers must be device memory of the current HIP device; "host" pointers
 *    are ordinary host memory.  Buffers must be 256-byte aligned.
 *  - Tokens of a call are ordered [batch][q_len]; token b*q_len + t sits at position
 *    positions[b] + t of sequence b.  The residual stream (x_in, x_out, slots) is fp32
 *    for both dtypes.
 *  - An spd_ctx is immutable after spd_create() and may be shared between threads; use
 *    one workspace per stream that runs concurrently.
 */
#ifndef SPD_H
#define SPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPD_F32 0   /* weights, KV cache and activations fp32; plain reference-style kernels */
#define SPD_BF16 1  /* bf16 weights and bf16 KV cache, fp32 accumulation, fp32 residual stream.  The projections run on the
                       matrix cores with fp16 operands: the packed shard holds each bf16 weight w as fp16(2^k w), one power
                       of two per matrix (an exact re-encoding for every weight within 2^-29 of its matrix's largest), and
                       activations between kernels are fp16; attention contracts bf16 */

#define SPD_OK 0
#define SPD_EINVAL (-1)       /* NULL pointer, bad shape, rank, batch, position or mask value */
#define SPD_EUNSUPPORTED (-2) /* a valid request this build does not implement (see spd_create) */
#define SPD_EHIP (-3)         /* a HIP call or kernel launch reported an error */
#define SPD_ETOOBIG (-4)      /* spd_block_forward_static(): the configuration's workspace exceeds the static scratch */

#define SPD_ALL_RANKS (-1)
#define SPD_MAX_BATCH 64

typedef struct spd_config {
    int32_t hidden;      /* model width h */
    int32_t n_q_heads;   /* query heads of the whole model */
    int32_t n_kv_heads;  /* KV heads of the whole model (== n_q_heads: MHA; fewer: grouped) */
    int32_t head_dim;    /* d */
    int32_t ffn;         /* SwiGLU inner width F of the whole model */
    int32_t n_layers;
    int32_t tp_degree;   /* must divide n_q_heads, n_kv_heads and ffn */
    int32_t dtype;       /* SPD_F32 | SPD_BF16 */
    int32_t max_batch;   /* sequences per call, <= SPD_MAX_BATCH */
    int32_t max_ctx;     /* KV-cache capacity in positions; a multiple of 32 */
    int32_t max_tokens;  /* largest batch*q_len of a single call */
    float rms_eps;       /* 1e-5 for LLaMA2 */
    float rope_base;     /* 10000 for LLaMA2 */
    int32_t act_split;   /* SPD_BF16 only: SPD_SPLIT_AUTO | SPD_SPLIT_ALWAYS | SPD_SPLIT_NEVER */
    int32_t o_bias;      /* 1: the attention output projection has a bias (block with bias, Sec. 4.1.2); else 0 */
} spd_config;

/* SPD_BF16 only.  An activation that feeds a projection is rounded to fp16 (11 significant bits).  A "split"
 * activation is kept as a pair hi + lo of fp16 values (lo = the rounding error of hi) and the contraction
 * runs over both, which removes that rounding from the result at the price of a second pass over the
 * matrix cores.  AUTO splits the one input whose rounding shows at the block output: the QKV
 * projection's in calls of more than 16 tokens with q_len > 1 (a prefill attends to keys it produces itself; the
 * softmax amplifies errors of q and k; a decode step of any batch size keeps the single plane).  ALWAYS splits every projection input, NEVER none. */
#define SPD_SPLIT_AUTO 0
#define SPD_SPLIT_ALWAYS 1
#define SPD_SPLIT_NEVER 2

typedef struct spd_ctx spd_ctx;

/* Byte sizes the caller allocates.  All are multiples of 256. */
typedef struct spd_sizes {
    size_t weight_bytes;    /* one rank's packed shard of one layer */
    size_t kv_bytes;        /* one rank's KV cache of one layer (max_batch x max_ctx) */
    size_t workspace_bytes; /* scratch for one stream */
} spd_sizes;

/* One layer's weights on the host, fp32, in the y = x W convention (rows = inputs).
 * `ld_*` is the row stride in elements.  For spd_pack_shard() these are the dense
 * (unsharded) matrices: wq [h, Hq*d], wk/wv [h, Hkv*d], wo [Hq*d, h], wg/wu [h, F],
 * wd [F, h]; for spd_pack_shard_local() they are one rank's slices.  g1/g2 [h] are the
 * gains of the two RMSNorms.  With dtype SPD_BF16 every weight must already be exactly
 * representable in bf16 (SPD_EINVAL otherwise): the packer re-encodes values, it does not round them
 * (only a weight more than 2^29 times smaller than its matrix's largest moves, by < 2^-39 of that largest). */
typedef struct spd_layer_weights {
    const float *wq, *wk, *wv, *wo, *wg, *wu, *wd, *g1, *g2;
    int64_t ld_q, ld_k, ld_v, ld_o, ld_g, ld_u, ld_d;
    const float *bo;     /* [h] bias of the output projection, replicated on every rank (it cannot be split
                            along the rows of W_O); required iff the configuration has o_bias = 1, else NULL.
                            Kept in fp32.  Block with bias (Sec. 4.1.2): the device's MLP input is
                            X + P_r + b, the partial product P_r joins the partial sum before the sync
                            point and b is added once after it. */
} spd_layer_weights;

/* Optional taps: when a pointer is non-NULL the block copies that intermediate of the
 * LAST rank it ran, in fp32 natural layout, to the device buffer.  For tests. */
typedef struct spd_taps {
    float *q;    /* [tokens, q*d]  rotated queries of the rank's heads */
    float *attn; /* [tokens, q*d]  attention output before the O projection */
    float *y;    /* [tokens, h]    partial attention output Y_r */
    float *u;    /* [tokens, f]    SwiGLU output silu(gate) * up of the rank's FFN slice */
} spd_taps;

/* ---------------------------------------------------------------- context (host only) */

/* Validates the configuration and builds an immutable context; touches no device.
 * SPD_EINVAL: NULL, non-positive sizes, odd head_dim, tp_degree not dividing the head
 * counts or ffn, n_q_heads not a multiple of n_kv_heads, max_batch > SPD_MAX_BATCH,
 * max_ctx not a multiple of 32.  SPD_EUNSUPPORTED: n_kv_heads < tp_degree (a KV head
 * shared by several ranks); unknown dtype; for SPD_BF16: hidden or head_dim not a
 * multiple of 32, head_dim above 128, ffn / tp_degree not a multiple of 16, more than 16
 * query heads per KV head.  act_split outside its three values, o_bias outside {0, 1}: SPD_EINVAL. */
int spd_create(const spd_config *cfg, spd_ctx **out);
void spd_destroy(spd_ctx *ctx);
int spd_get_config(const spd_ctx *ctx, spd_config *out);
int spd_get_sizes(const spd_ctx *ctx, spd_sizes *out);
const char *spd_strerror(int code);
/* After a call returned SPD_EHIP: which HIP call of this thread failed and with what error (a
 * string owned by the library, valid until the thread's next failing call).  Empty if none. */
const char *spd_last_hip_error(void);

/* ---------------------------------------------------------------- rank indexing (host only)
 * Sec. 4.2.3: the heads (and FFN columns) of device `rank` are a contiguous block of
 * N / tp_degree of them.  Each call returns the half-open range [*first, *first + *count). */
int spd_rank_q_heads(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count);
int spd_rank_kv_heads(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count);
int spd_rank_ffn_cols(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count);

/* Number of sync points (rank-sums) a model forward with this mask performs: two for a
 * block that keeps its attention sync point (mask 0), one for an SPD block (mask 1),
 * Sec. 3.  mask: host, [n_layers], each 0 or 1.  Returns the count or a negative code. */
int64_t spd_sync_count(const spd_ctx *ctx, const uint8_t *mask);

/* Sync-point drop by sensitivity (Alg. 1, Sec. 4.2): ranks the n_layers blocks by ascending
 * sync sensitivity and lets the first n_spd of the ranking drop their attention sync point.
 * Every dropped block gets a tier from its sensitivity s: SPD_TIER_ISB (s <= tau1: SPD as is),
 * SPD_TIER_SB (s <= tau2: SPD after block-to-block distillation), SPD_TIER_ESB (otherwise: head
 * grouping as well); blocks outside the budget get SPD_TIER_TP.  Blocks of equal sensitivity
 * rank by index.  The sensitivities themselves are measured on calibration data outside this
 * library (Sec. 4.2, Fig. 4); Sec. 5 uses tau1 = 0.05 (0.02 for the largest models), tau2 = 10.
 *   sensitivity  host, [n_layers] doubles, no NaN
 *   mask         host, [n_layers], receives 1 = sync dropped (the mask spd_model_forward takes)
 *   tier         host, [n_layers], receives the SPD_TIER_* codes; may be NULL
 * Host only, no device work.  SPD_EINVAL: NULL sensitivity or mask, n_layers <= 0, n_spd
 * outside [0, n_layers], NaN in the sensitivities or thresholds. */
#define SPD_TIER_TP 0
#define SPD_TIER_ISB 1
#define SPD_TIER_SB 2
#define SPD_TIER_ESB 3
int spd_mask_from_sensitivity(const double *sensitivity, int32_t n_layers, int32_t n_spd, double tau1, double tau2,
                              uint8_t *mask, uint8_t *tier);

/* ---------------------------------------------------------------- packing (host only)
 * Slices rank `rank`'s heads / FFN columns out of the dense layer and lays them out the
 * way the kernels stream them (the values themselves, re-encoded as described at SPD_BF16; zero padding only).
 * `packed_host` receives weight_bytes bytes; the caller then copies them to the device. */
int spd_pack_shard(const spd_ctx *ctx, int32_t rank, const spd_layer_weights *dense, void *packed_host);
/* Same after head grouping (Sec. 4.2.3, Fig. 5): the heads are laid over the devices in the
 * order `kv_heads` (a permutation of 0 .. n_kv_heads-1; device r holds kv_heads[r*kv .. r*kv+kv)
 * with the query heads that attend through them, so that the columns of W_Q, W_K, W_V and the
 * rows of W_O move together with their head), and device r is matched with MLP partition
 * mlp_of_rank[r] (a permutation of 0 .. tp_degree-1; partition m = FFN columns [m*f, m*f+f)).
 * Either array may be NULL = identity; with both NULL this is spd_pack_shard().  How the
 * grouping and the matching are found (attention scores and MLP output norms on calibration
 * data, Eq. 2 and 3) is outside this library.  SPD_EINVAL if an array is not a permutation. */
int spd_pack_shard_grouped(const spd_ctx *ctx, int32_t rank, const spd_layer_weights *dense, const int32_t *kv_heads,
                           const int32_t *mlp_of_rank, void *packed_host);
/* Same, from matrices that already are one rank's slices. */
int spd_pack_shard_local(const spd_ctx *ctx, const spd_layer_weights *shard, void *packed_host);
/* Inverse of spd_pack_shard_local(): writes the rank's slices back in natural layout
 * (pointers in `out` are written through despite the const in the struct). */
int spd_unpack_shard(const spd_ctx *ctx, const void *packed_host, const spd_layer_weights *out);

/* KV cache <-> natural layout.  k, v: host fp32 [batch, kv_heads_per_rank, n_pos, d],
 * positions 0 .. n_pos-1 of each sequence (keys already rotated).  `cache_host` is a host
 * copy of one rank's cache of one layer (kv_bytes bytes); pack leaves other positions as
 * they are.  batch <= max_batch, n_pos <= max_ctx. */
int spd_kv_pack(const spd_ctx *ctx, const float *k, const float *v, int32_t batch, int32_t n_pos, void *cache_host);
int spd_kv_unpack(const spd_ctx *ctx, const void *cache_host, int32_t batch, int32_t n_pos, float *k, float *v);

/* ---------------------------------------------------------------- device calls */

/* The KV cache must be zero-filled once before its first use (positions that were never
 * written are read as padding of the last key block and multiplied by a zero weight).
 *
 * Prepares a workspace (device, workspace_bytes): uploads the rotary table.  Call once per
 * workspace before the first forward; synchronises the stream before returning. */
int spd_workspace_init(const spd_ctx *ctx, void *workspace, void *stream);

/* out = base + (slot[0] + slot[1] + ... + slot[n_slots-1]): the partials are summed in
 * ascending slot order in fp32 and the base is added last (a kept sync point: what an
 * all-reduce delivers to every device, Sec. 3).  The order is fixed, so results are
 * bit-reproducible.  base may be NULL (treated as zero), out may alias base.  slots: device, [n_slots][n_elems] fp32
 * contiguous.  n_slots >= 0, n_elems >= 0 (0 is a no-op). */
int spd_rank_sum(const spd_ctx *ctx, const float *base, const float *slots, int32_t n_slots,
                 int64_t n_elems, float *out, void *stream);

/* One decoder block for one rank (or all of them).
 *   layer          index of the block (only used for error messages and taps)
 *   spd_flag       1: SPD block (attention sync point dropped, Sec. 4.1.1); 0: TP block
 *   rank           0 .. tp_degree-1, or SPD_ALL_RANKS
 *   packed_weights device; the rank's packed shard, or all ranks' shards back to back
 *                  (stride weight_bytes) with SPD_ALL_RANKS
 *   kv_cache       device; the rank's cache of this layer, or all ranks' caches back to
 *                  back (stride kv_bytes).  Keys/values of the call's tokens are appended
 *                  at their positions before attention reads the cache.
 *   positions      host, [batch]: position of each sequence's first token of this call;
 *                  positions[b] + q_len <= max_ctx
 *   x_in           device, fp32 [batch*q_len, hidden]: the block input X, identical on all ranks
 *   slots          device, fp32 [tp_degree][batch*q_len, hidden]: the partial sums met at a
 *                  sync point.  With rank = r the library overwrites slot r only (with Y_r
 *                  and later Z_r in a TP block, with Y_r + Z_r in an SPD block) and reads
 *                  the other slots as the peers' contributions; with SPD_ALL_RANKS it
 *                  writes all of them.
 *   x_out          device, fp32 [batch*q_len, hidden]; may alias x_in
 *   workspace      device, initialised by spd_workspace_init()
 *   taps           NULL or optional debug outputs
 * Errors: SPD_EINVAL for NULL pointers, rank out of range, spd_flag not 0/1, batch or
 * batch*q_len beyond the configured maxima, a position that would overflow max_ctx. */
int spd_block_forward(const spd_ctx *ctx, int32_t layer, int32_t spd_flag, int32_t rank,
                      const void *packed_weights, void *kv_cache, const int32_t *positions,
                      int32_t batch, int32_t q_len, const float *x_in, float *slots,
                      float *x_out, void *workspace, void *stream, const spd_taps *taps);

/* spd_block_forward() for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results without `workspace`: the scratch the kernels need (partial tiles,
 * packed activations, norm statistics, the rotary table) lives in a device array inside the
 * library, SPD_STATIC_WORKSPACE_BYTES large, which every GPU the library runs on holds until the
 * process ends.  The call allocates and frees nothing.
 *  - SPD_ETOOBIG if spd_get_sizes(ctx).workspace_bytes exceeds SPD_STATIC_WORKSPACE_BYTES (64 MiB:
 *    the LLaMA2 shards fit with max_tokens up to 128, long prefills do not); nothing is launched then.
 *  - The first call on a device looks the array up; the first call with a context other than the
 *    one that used the array last uploads that context's rotary table (a host-to-device copy and a
 *    synchronisation of `stream`: make that call outside stream capture).  Later calls only
 *    enqueue kernels.
 *  - All calls on one GPU share the one array: calls that overlap in time on one GPU (two streams,
 *    two threads) race.  Nothing else in the array needs to start at a known value, so a call may
 *    follow one of any other size. */
#define SPD_STATIC_WORKSPACE_BYTES (64u << 20)
int spd_block_forward_static(const spd_ctx *ctx, int32_t layer, int32_t spd_flag, int32_t rank,
                             const void *packed_weights, void *kv_cache, const int32_t *positions,
                             int32_t batch, int32_t q_len, const float *x_in, float *slots,
                             float *x_out, void *stream, const spd_taps *taps);

/* All blocks in order; block l is an SPD block iff spd_mask[l] == 1 (the per-layer outcome
 * of Alg. 1; every other value than 0 or 1 is SPD_EINVAL).
 *   spd_mask       host, [n_layers]
 *   layer_weights  host array [n_layers] of device pointers (as in spd_block_forward)
 *   layer_kv       host array [n_layers] of device pointers
 *   slots          one [tp_degree][tokens, hidden] buffer reused by every layer
 *   n_rank_sums    NULL or host int64 receiving the number of rank-sums enqueued
 * x_out may alias x_in.  The rank-sum that ends block l is fused with the first norm's
 * elementwise work of block l+1.
 * A bf16 prefill (q_len > 1) of at least two sequences whose halves have 1024 tokens or more, for one rank,
 * in a context sized for it, is enqueued as two chains of launches, one half of the sequences each: one on
 * `stream`, one on a stream the library keeps per device (default priority, created on first use), forked
 * from and joined back to `stream` with events, so that `stream` sees one ordered call and the call can be
 * captured into a HIP graph.  Calls of this kind from several threads on one device enqueue one after the
 * other. */
int spd_model_forward(const spd_ctx *ctx, const uint8_t *spd_mask, int32_t rank,
                      const void *const *layer_weights, void *const *layer_kv,
                      const int32_t *positions, int32_t batch, int32_t q_len,
                      const float *x_in, float *slots, float *x_out, void *workspace,
                      void *stream, int64_t *n_rank_sums);

#ifdef __cplusplus
}
#endif
#endif /* SPD_H */
