// Device-facing entry points of the C ABI: argument checks on the host, then the sequence
// of kernel launches that makes up one rank's share of a TP or SPD decoder block.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "spd_internal.h"

namespace {

// what the last failing HIP call of this thread was (spd_last_hip_error())
thread_local char g_hip_msg[256] = "";

#define SPD_HIP(x)                                                                                              \
    do {                                                                                                        \
        const hipError_t e_ = (x);                                                                              \
        if (e_ != hipSuccess) {                                                                                 \
            std::snprintf(g_hip_msg, sizeof(g_hip_msg), "%s (%s) at %s:%d", hipGetErrorName(e_), #x, __FILE__, __LINE__); \
            return SPD_EHIP;                                                                                    \
        }                                                                                                       \
    } while (0)

// launch errors are read with hipGetLastError(), which also returns whatever an earlier, unrelated
// call of this thread left behind: every entry point starts from a clean slate
inline void clear_stale_hip_error() { (void)hipGetLastError(); }

inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15) == 0; }

// Everything a forward call must satisfy before anything is launched.
int check_call(const spd_ctx *ctx, int32_t rank, const int32_t *positions, int32_t batch, int32_t q_len,
               const float *x_in, float *slots, float *x_out, void *workspace, spd_call *c, void *stream) {
    if (!ctx || !positions || !x_in || !slots || !x_out || !workspace) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (rank != SPD_ALL_RANKS && (rank < 0 || rank >= D.tp)) return SPD_EINVAL;
    if (batch < 0 || q_len < 0 || batch > D.max_batch) return SPD_EINVAL;
    if ((int64_t)batch * q_len > D.max_tokens) return SPD_EINVAL;
    if (!aligned16(x_in) || !aligned16(slots) || !aligned16(x_out) || (((uintptr_t)workspace) & 255)) return SPD_EINVAL;
    c->D = &D;
    c->s = (hipStream_t)stream;
    c->batch = batch;
    c->q_len = q_len;
    c->M = batch * q_len;
    c->slot_stride = (size_t)c->M * D.h;
    c->ws = (char *)workspace;
    c->taps = nullptr;
    c->chained = false;
    c->stages = SPD_ALL_STAGES;
    c->timer = nullptr;
    c->max_pos_end = 0;
    {
        const bool bf = D.dtype == SPD_BF16;
        const bool always = bf && ctx->cfg.act_split == SPD_SPLIT_ALWAYS, automatic = bf && ctx->cfg.act_split == SPD_SPLIT_AUTO;
        // AUTO: fp16 activations are precise enough everywhere except the QKV projection's input in calls that
        // attend to keys they produce themselves (prefill), where the softmax amplifies its rounding; a decode
        // step of any batch size attends to one new key per sequence and keeps the single plane
        c->sp_x = always || (automatic && c->M > SPD_AUTO_SPLIT_TOKENS && q_len > 1);
        c->sp_a = always;
        c->sp_m = always;
    }
    c->nch1 = 0;
    std::memset(&c->pos, 0, sizeof(c->pos));
    for (int b = 0; b < batch; ++b) {
        if (positions[b] < 0 || (int64_t)positions[b] + q_len > D.max_ctx) return SPD_EINVAL;
        c->pos.pos[b] = positions[b];
        if (positions[b] + q_len > c->max_pos_end) c->max_pos_end = positions[b] + q_len;
    }
    return SPD_OK;
}

// The part of a block between its input and the rank-sum that ends it.  On return the
// slots hold the partial sums of the final sync point and *base_out is what they are added
// to: X for an SPD block (Sec. 4.1.1: the block input joins after the remaining sync point), R = X + sum Y for a TP
// block.  *syncs is incremented by the number of kept attention sync points (0 or 1).
// With end_sync_out (one rank, bf16 path, at most 16 tokens) the last kernel of the block also
// performs that final rank-sum into x_out (and the next block's first-norm preparation when
// next_g1 is given); *end_done tells the caller whether it did.
int block_core(const spd_ctx *ctx, spd_call &c, int spd, int32_t rank, const char *weights, char *kv,
               const float *x, float *slots, const float **base_out, const float **bias_out, int64_t *syncs,
               float *x_out, const float *next_g1, bool *end_done) {
    const spd_dims &D = ctx->D;
    const size_t slot_n = c.slot_stride;      // distance between two ranks' slots (the whole call's tokens)
    float *ybuf = (float *)(c.ws + D.ws_y), *rbuf = (float *)(c.ws + D.ws_r);
    const int r0 = rank == SPD_ALL_RANKS ? 0 : rank, r1 = rank == SPD_ALL_RANKS ? D.tp : rank + 1;
    const bool all = rank == SPD_ALL_RANKS;
    auto wr = [&](int r) { return weights + (all ? (size_t)r * D.weight_bytes : 0); };
    auto kr = [&](int r) { return kv + (all ? (size_t)r * D.kv_bytes : 0); };

    // block with bias (Sec. 4.1.2): the output projection's bias b joins a sum over the ranks once,
    // after the sync point: the attention one in a TP block, the one that ends the block in an SPD
    // block (whose MLP input X + P_r + b takes it locally)
    const float *bo = D.o_bias ? (const float *)(wr(r0) + D.w_bo) : nullptr;
    *bias_out = spd ? bo : nullptr;
    *end_done = false;
    if (D.dtype == SPD_BF16) {
        spd_bf16::spd_end_sync es;
        es.slots = slots; es.tp = D.tp; es.rank = r0; es.x_out = x_out; es.next_g1 = next_g1; es.bias = *bias_out;
        const spd_bf16::spd_end_sync *fuse = (!all && x_out) ? &es : nullptr;
        if (spd) {
            es.base = x;
            for (int r = r0; r < r1; ++r) {
                SPD_HIP(spd_bf16::attention_half(c, wr(r), kr(r), x, 1, slots + r * slot_n));
                SPD_HIP(spd_bf16::mlp_half(c, wr(r), 1, slots + r * slot_n, fuse, end_done, true));
            }
            *base_out = x;
        } else {
            // kept sync point: R = X + sum_r Y_r (+ bias), with the second norm's elementwise part; for one
            // rank and a call of at most 512 tokens the O projection's epilogue does it, otherwise prep()
            spd_bf16::spd_mid_sync ms;
            ms.slots = slots; ms.tp = D.tp; ms.rank = r0; ms.rbuf = rbuf;
            bool mid_done = false;
            for (int r = r0; r < r1; ++r)
                SPD_HIP(spd_bf16::attention_half(c, wr(r), kr(r), x, 0, slots + r * slot_n, all ? nullptr : &ms, &mid_done));
            if (!mid_done) SPD_HIP(spd_bf16::prep(c, x, slots, D.tp, rbuf, (const float *)(wr(r0) + D.w_g2), true, 1, bo));
            *syncs += 1;
            es.base = rbuf;
            for (int r = r0; r < r1; ++r)
                SPD_HIP(spd_bf16::mlp_half(c, wr(r), 0, slots + r * slot_n, fuse, end_done, mid_done));
            *base_out = rbuf;
        }
        return SPD_OK;
    }
    if (spd) {
        for (int r = r0; r < r1; ++r) {
            SPD_HIP(spd_f32::attention_half(c, wr(r), kr(r), x, ybuf));
            SPD_HIP(spd_common::rank_sum(x, ybuf, 1, (int64_t)c.M * D.h, rbuf, c.s, bo, D.h));   // local fold X + Y_r (+ b)
            SPD_HIP(spd_f32::mlp_half(c, wr(r), rbuf, ybuf, slots + r * slot_n));        // slot = Y_r + Z_r
        }
        *base_out = x;
    } else {
        for (int r = r0; r < r1; ++r) SPD_HIP(spd_f32::attention_half(c, wr(r), kr(r), x, slots + r * slot_n));
        SPD_HIP(spd_common::rank_sum(x, slots, D.tp, (int64_t)slot_n, rbuf, c.s, bo, D.h));   // kept sync point
        *syncs += 1;
        for (int r = r0; r < r1; ++r) SPD_HIP(spd_f32::mlp_half(c, wr(r), rbuf, nullptr, slots + r * slot_n));
        *base_out = rbuf;
    }
    return SPD_OK;
}

// The helper stream of the two-chain model forward and the events that fork to it and join from it: one
// set per device, created on first use with that device current (default priority, non-blocking), never
// destroyed.
struct TwoStreams {
    std::mutex mu;
    hipStream_t helper = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool tried = false, ok = false;
};
TwoStreams *two_streams() {
    constexpr int kMaxDevices = 64;
    static TwoStreams per_device[kMaxDevices];
    static std::mutex create_mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        std::snprintf(g_hip_msg, sizeof(g_hip_msg), "no current device for the helper stream of the two-chain model forward");
        return nullptr;
    }
    TwoStreams &ts = per_device[dev];
    {
        std::lock_guard<std::mutex> lock(create_mu);
        if (!ts.tried) {
            ts.tried = true;
            ts.ok = hipStreamCreateWithFlags(&ts.helper, hipStreamNonBlocking) == hipSuccess &&
                    hipEventCreateWithFlags(&ts.fork, hipEventDisableTiming) == hipSuccess &&
                    hipEventCreateWithFlags(&ts.join, hipEventDisableTiming) == hipSuccess;
        }
    }
    if (!ts.ok) {
        std::snprintf(g_hip_msg, sizeof(g_hip_msg), "could not create the helper stream of the two-chain model forward");
        return nullptr;
    }
    return &ts;
}

// spd_block_forward() and its variant without allocations differ only in where the workspace comes from
int block_forward_impl(const spd_ctx *ctx, int32_t layer, int32_t spd_flag, int32_t rank, const void *packed_weights,
                       void *kv_cache, const int32_t *positions, int32_t batch, int32_t q_len, const float *x_in,
                       float *slots, float *x_out, void *workspace, void *stream, const spd_taps *taps) {
    spd_call c;
    const int rc = check_call(ctx, rank, positions, batch, q_len, x_in, slots, x_out, workspace, &c, stream);
    if (rc != SPD_OK) return rc;
    if (!packed_weights || !kv_cache) return SPD_EINVAL;
    if (spd_flag != 0 && spd_flag != 1) return SPD_EINVAL;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return SPD_EINVAL;
    if (c.M == 0) return SPD_OK;
    clear_stale_hip_error();
    const spd_dims &D = ctx->D;
    c.taps = taps;
    const char *w = (const char *)packed_weights;
    if (D.dtype == SPD_BF16) {
        SPD_HIP(spd_bf16::prep(c, x_in, nullptr, 0, nullptr, (const float *)(w + D.w_g1), true, 0));
        c.nch1 = spd_bf16::prep_chunks(c);
    }
    const float *base = nullptr, *bias = nullptr;
    int64_t syncs = 0;
    bool end_done = false;
    const int rc2 = block_core(ctx, c, spd_flag, rank, w, (char *)kv_cache, x_in, slots, &base, &bias, &syncs, x_out,
                               nullptr, &end_done);
    if (rc2 != SPD_OK) return rc2;
    // the sync point that ends every block, SPD or not
    if (!end_done) SPD_HIP(spd_common::rank_sum(base, slots, D.tp, (int64_t)c.M * D.h, x_out, c.s, bias, D.h));
    return SPD_OK;
}

}  // namespace

extern "C" {

int spd_workspace_init(const spd_ctx *ctx, void *workspace, void *stream) {
    if (!ctx || !workspace || (((uintptr_t)workspace) & 255)) return SPD_EINVAL;
    clear_stale_hip_error();
    const spd_dims &D = ctx->D;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    for (int k = 0; k < (D.ws_dual ? 2 : 1); ++k) {      // a workspace for two chains holds the table twice
        char *half = ws + (size_t)k * D.ws_single;
        SPD_HIP(hipMemcpyAsync(half + D.ws_cos, ctx->rope_cos.data(), ctx->rope_cos.size() * 4, hipMemcpyHostToDevice, s));
        SPD_HIP(hipMemcpyAsync(half + D.ws_sin, ctx->rope_sin.data(), ctx->rope_sin.size() * 4, hipMemcpyHostToDevice, s));
    }
    SPD_HIP(hipStreamSynchronize(s));
    return SPD_OK;
}

int spd_rank_sum(const spd_ctx *ctx, const float *base, const float *slots, int32_t n_slots, int64_t n_elems,
                 float *out, void *stream) {
    if (!ctx || !out || n_slots < 0 || n_elems < 0) return SPD_EINVAL;
    if (n_slots > 0 && !slots) return SPD_EINVAL;
    if (n_elems == 0) return SPD_OK;
    clear_stale_hip_error();
    SPD_HIP(spd_common::rank_sum(base, slots, n_slots, n_elems, out, (hipStream_t)stream));
    return SPD_OK;
}

int spd_block_forward(const spd_ctx *ctx, int32_t layer, int32_t spd_flag, int32_t rank, const void *packed_weights,
                      void *kv_cache, const int32_t *positions, int32_t batch, int32_t q_len, const float *x_in,
                      float *slots, float *x_out, void *workspace, void *stream, const spd_taps *taps) {
    return block_forward_impl(ctx, layer, spd_flag, rank, packed_weights, kv_cache, positions, batch, q_len, x_in, slots,
                              x_out, workspace, stream, taps);
}

int spd_model_forward_staged(const spd_ctx *ctx, const uint8_t *spd_mask, int32_t rank, const void *const *layer_weights,
                             void *const *layer_kv, const int32_t *positions, int32_t batch, int32_t q_len,
                             const float *x_in, float *slots, float *x_out, void *workspace, void *stream,
                             int64_t *n_rank_sums, uint32_t stage_mask, spd_stage_timer *timer, float *layer_out) {
    spd_call c;
    const int rc = check_call(ctx, rank, positions, batch, q_len, x_in, slots, x_out, workspace, &c, stream);
    if (rc != SPD_OK) return rc;
    if (!spd_mask || !layer_weights || !layer_kv) return SPD_EINVAL;
    if (stage_mask & ~SPD_ALL_STAGES) return SPD_EINVAL;
    c.stages = stage_mask;
    c.timer = timer;
    const spd_dims &D = ctx->D;
    const int L = ctx->cfg.n_layers;
    for (int l = 0; l < L; ++l) {
        if (spd_mask[l] > 1) return SPD_EINVAL;
        if (!layer_weights[l] || !layer_kv[l]) return SPD_EINVAL;
    }
    if (n_rank_sums) *n_rank_sums = 0;
    if (c.M == 0) return SPD_OK;
    clear_stale_hip_error();
    const bool bf = D.dtype == SPD_BF16;
    int64_t syncs = 0;

    // One chain of launches per half of the sequences, or a single chain for the whole call.  A prefill is
    // independent from sequence to sequence all the way through the model, and a chain alternates between
    // kernels bound by the matrix cores (the projections) and kernels bound by memory (the rank-sums, the
    // norm preparation, attention's vector work): two chains on two streams let one chain's memory-bound
    // kernels share the compute units with the other's GEMMs.  Each chain has its own workspace half.
    struct Chain {
        spd_call c;
        const float *x_in, *x;
        float *slots, *x_out, *layer_out;
        size_t kv_off;            // byte offset of the chain's first sequence inside a layer's K (and V) region
        size_t row0;              // first token row of the chain in the call
    };
    Chain ch[2];
    int n_chains = 1;
    ch[0].c = c; ch[0].x_in = x_in; ch[0].x = x_in; ch[0].slots = slots; ch[0].x_out = x_out; ch[0].kv_off = 0; ch[0].row0 = 0;
    const bool two = bf && D.ws_dual && rank != SPD_ALL_RANKS && q_len > 1 && batch >= 2 &&
                     (int64_t)(batch / 2) * q_len >= SPD_DUAL_MIN_TOKENS;
    TwoStreams *ts = nullptr;
    std::unique_lock<std::mutex> dual_lock;
    if (two) {
        ts = two_streams();
        if (!ts) return SPD_EHIP;
        dual_lock = std::unique_lock<std::mutex>(ts->mu);     // the helper stream and its events serve one call at a time
        n_chains = 2;
        const int b0 = (batch + 1) / 2, b1 = batch - b0;
        const size_t es = 2, seq_bytes = (size_t)D.kv * D.max_ctx * D.d * es;
        for (int k = 0; k < 2; ++k) {
            Chain &h = ch[k];
            const int bb = k ? b1 : b0, first = k ? b0 : 0;
            h.c = c;
            h.c.chained = true;
            h.c.batch = bb;
            h.c.M = bb * q_len;
            std::memset(&h.c.pos, 0, sizeof(h.c.pos));
            for (int i = 0; i < bb; ++i) h.c.pos.pos[i] = c.pos.pos[first + i];
            h.row0 = (size_t)first * q_len;
            h.x_in = h.x = x_in + h.row0 * D.h;
            h.slots = slots + h.row0 * D.h;
            h.x_out = x_out + h.row0 * D.h;
            h.kv_off = (size_t)first * seq_bytes;
            if (k) {
                h.c.ws = c.ws + D.ws_single;
                h.c.s = ts->helper;
            }
        }
        // fork: the second chain starts when everything enqueued on the caller's stream so far is done
        SPD_HIP(hipEventRecord(ts->fork, c.s));
        SPD_HIP(hipStreamWaitEvent(ts->helper, ts->fork, 0));
    }
    for (int k = 0; k < n_chains; ++k) {
        Chain &h = ch[k];
        h.layer_out = layer_out;
        if (bf) {
            SPD_HIP(spd_bf16::prep(h.c, h.x_in, nullptr, 0, nullptr, (const float *)((const char *)layer_weights[0] + D.w_g1),
                                   true, 0));
            h.c.nch1 = spd_bf16::prep_chunks(h.c);
        }
    }
    for (int l = 0; l < L; ++l) {
        const bool more = l + 1 < L;
        const float *g1 = (bf && more) ? (const float *)((const char *)layer_weights[l + 1] + D.w_g1) : nullptr;
        for (int k = 0; k < n_chains; ++k) {
            Chain &h = ch[k];
            const float *base = nullptr, *bias = nullptr;
            bool end_done = false;
            int64_t kept = 0;
            const int rc2 = block_core(ctx, h.c, spd_mask[l], rank, (const char *)layer_weights[l],
                                       (char *)layer_kv[l] + h.kv_off, h.x, h.slots, &base, &bias, &kept, h.x_out, g1, &end_done);
            if (rc2 != SPD_OK) return rc2;
            if (k == 0) syncs += kept;
            // end-of-block sync point; in the bf16 path it also prepares the next block's first norm
            if (end_done) {
                h.c.nch1 = D.h / 32;                   // the fused epilogue left one partial per pair of n-tiles
            } else if (bf) {
                SPD_HIP(spd_bf16::prep(h.c, base, h.slots, D.tp, h.x_out, g1, more, 0, bias));
                h.c.nch1 = spd_bf16::prep_chunks(h.c);
            } else if (h.c.on(SPD_STAGE_PREP)) {
                SPD_HIP(spd_common::rank_sum(base, h.slots, D.tp, (int64_t)h.c.M * D.h, h.x_out, h.c.s, bias, D.h));
            }
            h.x = h.x_out;
            if (layer_out)       // test tap: every block's output
                SPD_HIP(hipMemcpyAsync(layer_out + ((size_t)l * c.M + h.row0) * D.h, h.x_out, (size_t)h.c.M * D.h * 4,
                                       hipMemcpyDeviceToDevice, h.c.s));
        }
        syncs += 1;
    }
    if (two) {       // join: the caller's stream continues when the second chain is done
        SPD_HIP(hipEventRecord(ts->join, ts->helper));
        SPD_HIP(hipStreamWaitEvent(c.s, ts->join, 0));
    }
    if (n_rank_sums) *n_rank_sums = syncs;
    return SPD_OK;
}

int spd_model_forward(const spd_ctx *ctx, const uint8_t *spd_mask, int32_t rank, const void *const *layer_weights,
                      void *const *layer_kv, const int32_t *positions, int32_t batch, int32_t q_len, const float *x_in,
                      float *slots, float *x_out, void *workspace, void *stream, int64_t *n_rank_sums) {
    return spd_model_forward_staged(ctx, spd_mask, rank, layer_weights, layer_kv, positions, batch, q_len, x_in, slots, x_out,
                                    workspace, stream, n_rank_sums, SPD_ALL_STAGES, nullptr, nullptr);
}

const char *spd_last_hip_error(void) { return g_hip_msg; }

}  // extern "C"

// ------------------------------------------------------------------------------------------
// The entry point that allocates nothing: the workspace of spd_block_forward() lives in a
// file-scope device array instead of caller memory.  Every GPU the library runs on holds its own
// copy of the array at its own address, looked up once per device with hipGetSymbolAddress() (in
// host code the array's name is only a stand-in for that address and is never handed to a kernel
// or a copy).
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SPD_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
struct StaticScratch {
    void *ptr = nullptr;          // device address of `scratch` on this device
    uint64_t tables_of = 0;       // id of the context whose rotary table the array holds (0: none)
};
std::mutex g_static_mu;
StaticScratch g_static[MAX_DEVICES];
}  // namespace

extern "C" int spd_block_forward_static(const spd_ctx *ctx, int32_t layer, int32_t spd_flag, int32_t rank,
                                        const void *packed_weights, void *kv_cache, const int32_t *positions,
                                        int32_t batch, int32_t q_len, const float *x_in, float *slots, float *x_out,
                                        void *stream, const spd_taps *taps) {
    if (!ctx) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (D.workspace_bytes > (size_t)SPD_STATIC_WORKSPACE_BYTES) return SPD_ETOOBIG;     // before any device call
    clear_stale_hip_error();
    int dev = -1;
    SPD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return SPD_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticScratch &st = g_static[dev];
    if (!st.ptr) {
        void *p = nullptr;
        SPD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SPD_EHIP;
        st.ptr = p;
    }
    char *ws = (char *)st.ptr;
    // every argument check of the ordinary entry point, before the array is touched
    {
        spd_call probe;
        const int rc = check_call(ctx, rank, positions, batch, q_len, x_in, slots, x_out, ws, &probe, stream);
        if (rc != SPD_OK) return rc;
        if (!packed_weights || !kv_cache || (spd_flag != 0 && spd_flag != 1) || layer < 0 || layer >= ctx->cfg.n_layers)
            return SPD_EINVAL;
        if (probe.M == 0) return SPD_OK;
    }
    // The array keeps what the last call left.  The only part a forward call reads without having written it
    // is the rotary table, which belongs to a context: upload it when another context used the array last.
    if (st.tables_of != ctx->id) {
        hipStream_t s = (hipStream_t)stream;
        st.tables_of = 0;
        SPD_HIP(hipMemcpyAsync(ws + D.ws_cos, ctx->rope_cos.data(), ctx->rope_cos.size() * 4, hipMemcpyHostToDevice, s));
        SPD_HIP(hipMemcpyAsync(ws + D.ws_sin, ctx->rope_sin.data(), ctx->rope_sin.size() * 4, hipMemcpyHostToDevice, s));
        SPD_HIP(hipStreamSynchronize(s));       // the host table may go away with its context
        st.tables_of = ctx->id;
    }
    return block_forward_impl(ctx, layer, spd_flag, rank, packed_weights, kv_cache, positions, batch, q_len, x_in, slots,
                              x_out, ws, stream, taps);
}

// ------------------------------------------------------------------------------------------
// stage timers (spd_testing.h)
// ------------------------------------------------------------------------------------------
extern "C" {

void spd_stage_timer_destroy(spd_stage_timer *t) {
    if (!t) return;
    for (auto e : t->start) (void)hipEventDestroy(e);
    for (auto e : t->stop) (void)hipEventDestroy(e);
    delete t;
}

int spd_mfma_probe(int32_t iters, int32_t random_data, void *scratch, void *stream, double *tflops, double *mhz) {
    if (iters <= 0 || !scratch || !tflops || !mhz) return SPD_EINVAL;
    clear_stale_hip_error();
    SPD_HIP(spd_bf16::mfma_probe(iters, random_data, scratch, (hipStream_t)stream, tflops, mhz));
    return SPD_OK;
}

int spd_read_probe(const void *buf, size_t chunk_bytes, int32_t n_chunks, int32_t reps, void *sink, void *stream,
                   double *us_per_launch) {
    if (!buf || !sink || !us_per_launch || n_chunks <= 0 || reps <= 0) return SPD_EINVAL;
    if (chunk_bytes == 0 || chunk_bytes % ((size_t)4 << 20) != 0) return SPD_EINVAL;
    clear_stale_hip_error();
    SPD_HIP(spd_bf16::read_probe(buf, chunk_bytes, n_chunks, reps, sink, (hipStream_t)stream, us_per_launch));
    return SPD_OK;
}

int spd_stage_timer_create(int32_t stage, int32_t max_records, spd_stage_timer **out) {
    if (!out || stage < 0 || stage > SPD_STAGE_EMPTY || max_records <= 0) return SPD_EINVAL;
    *out = nullptr;
    spd_stage_timer *t = new (std::nothrow) spd_stage_timer();
    if (!t) return SPD_EINVAL;
    t->stage = stage;
    for (int i = 0; i < max_records; ++i) {
        hipEvent_t a = nullptr, b = nullptr;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            if (a) (void)hipEventDestroy(a);
            spd_stage_timer_destroy(t);
            std::snprintf(g_hip_msg, sizeof(g_hip_msg), "hipEventCreate failed in spd_stage_timer_create");
            return SPD_EHIP;
        }
        t->start.push_back(a);
        t->stop.push_back(b);
    }
    *out = t;
    return SPD_OK;
}

int spd_stage_timer_read(spd_stage_timer *t, int32_t *n_records, double *mean_us, double *min_us) {
    if (!t) return SPD_EINVAL;
    double sum = 0.0, mn = 1e30;
    for (int i = 0; i < t->n; ++i) {
        SPD_HIP(hipEventSynchronize(t->stop[i]));
        float ms = 0.f;
        SPD_HIP(hipEventElapsedTime(&ms, t->start[i], t->stop[i]));
        sum += (double)ms * 1000.0;
        if ((double)ms * 1000.0 < mn) mn = (double)ms * 1000.0;
    }
    if (n_records) *n_records = t->n;
    if (mean_us) *mean_us = t->n ? sum / t->n : 0.0;
    if (min_us) *min_us = t->n ? mn : 0.0;
    t->n = 0;
    return SPD_OK;
}

}  // extern "C"
