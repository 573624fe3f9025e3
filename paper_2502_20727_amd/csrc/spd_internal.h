// Internal declarations shared by the host side and the kernels of the SPD library:
// derived per-rank dimensions, the packed memory layouts, and the launcher prototypes.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "spd.h"
#include "spd_testing.h"

#define SPD_HD __host__ __device__ __forceinline__

// ------------------------------------------------------------------------------------------
// Packed layouts of the bf16 path.
//
// Every matrix operand of an MFMA 16x16x32 (16-bit elements: fp16 for the projections, bf16 for
// attention) is stored as a sequence of 1 KiB
// "fragments": 16 rows x 32 contraction elements, in the register order of the
// instruction.  Lane l of a wavefront owns row (l % 16) and the 8 consecutive contraction
// elements starting at 8 * (l / 16); its 8 bf16 values are contiguous (16 bytes), and the
// 64 lanes follow each other, so one fragment is one fully coalesced 1 KiB load.
//
// A weight matrix W [K, N] (y = x W) is cut into n-tiles of 16 output columns and k-tiles
// of 32 inputs; fragment (nt, kt) sits at ((nt * KT) + kt) * 512 elements, row = column
// n0(nt) + l % 16 of W, contraction element = input kt*32 + 8*(l/16) + j.  Row-major
// activations [M, K] use the same scheme with m-tiles in place of n-tiles.
// ------------------------------------------------------------------------------------------

constexpr int SPD_FRAG_ELEMS = 512;   // 16 x 32
constexpr int SPD_MAX_SPLITS = 64;    // decode attention: context splits per (sequence, KV head)
constexpr int SPD_AUTO_SPLIT_TOKENS = 16;    // SPD_SPLIT_AUTO: calls of more than this many tokens carry the QKV projection's input as a hi + lo pair
constexpr int SPD_MAX_QKV_SLICES = 8;  // K slices of a decode QKV projection that the attention kernel adds up itself
constexpr int SPD_DUAL_MIN_TOKENS = 1024;   // a prefill runs as two chains when each half has at least this many tokens
constexpr int SPD_MAX_KPART = 4096;   // split-K partial tiles (pairs x splits) a GEMV may park in the workspace
constexpr int SPD_MID_KPART = 2304 * 8;   // ... and a call of 17 .. 128 tokens (pairs x splits x m-tiles)

SPD_HD size_t spd_frag_index(int tile, int ktile, int n_ktiles) {
    return ((size_t)tile * (size_t)n_ktiles + (size_t)ktile) * SPD_FRAG_ELEMS;
}
// element offset inside a fragment of (row r in 0..15, contraction index c in 0..31)
SPD_HD int spd_frag_elem(int r, int c) { return ((r + 16 * (c >> 3)) << 3) + (c & 7); }

// QKV n-tiles: the rank's columns are [Q heads | K heads | V heads].  Inside every rotary
// head (Q and K) the d/16 tiles are interleaved so that packed tiles 2i and 2i+1 hold the
// rotary partners: columns [16 i, 16 i + 16) and the same range shifted by d/2.
SPD_HD int spd_qkv_tile_col0(int pt, int q, int kv, int d) {
    const int tph = d >> 4;
    const int head = pt / tph, w = pt % tph;
    if (head < q + kv) return head * d + (((w >> 1) + (w & 1) * (tph >> 1)) << 4);
    return head * d + (w << 4);
}

// KV cache, bf16 path, per (sequence, KV head): max_ctx * d elements for K, same for V.
// K: blocks of 16 positions; block = d/32 fragments with row = position, contraction = d.
SPD_HD size_t spd_kcache_off(int pos, int dcol, int d) {
    return (size_t)(pos >> 4) * (size_t)(16 * d) + (size_t)(dcol >> 5) * SPD_FRAG_ELEMS +
           (size_t)spd_frag_elem(pos & 15, dcol & 31);
}
// V: blocks of 32 positions; block = d/16 fragments with row = d index, contraction =
// position.  The 32 positions of a block are permuted so that the probabilities, as they
// come out of two 16-key score tiles (4 consecutive keys per lane and tile), already are
// the partner operand: contraction slot (g, j) holds key 4g + j (j < 4) or 16 + 4g + j - 4.
SPD_HD size_t spd_vcache_off(int pos, int dcol, int d) {
    const int kl = pos & 31, hi = kl >> 4, r = kl & 15;
    const int g = r >> 2, j = (r & 3) + 4 * hi;
    return (size_t)(pos >> 5) * (size_t)(32 * d) + (size_t)(dcol >> 4) * SPD_FRAG_ELEMS +
           (size_t)(((dcol & 15) + 16 * g) << 3) + (size_t)j;
}

// ------------------------------------------------------------------------------------------
// Order of the tiles of the LDS-tiled GEMM.  Every XCD has its own L2 and workgroup b of a launch
// runs on XCD b % 8, so the tiles are put in an order in which neighbours share operand panels
// (blocks of bn x bm tiles, block rows along N first, a block's tiles along N first; blocks at the
// edges are narrower or shorter) and every XCD works on runs of 32 consecutive tiles of that
// order: the tiles an XCD has in flight then form about one block and fetch bn + bm panels through
// its L2 (256 x 256 tiles, blocks of 4 x 8: 12 panels instead of the 16-17 of a row-major numbering
// with the workgroups dealt round-robin, which cost the gate/up launch of the 70B shard 2.16 instead
// of 1.59 GB of fetches).
// ------------------------------------------------------------------------------------------
struct spd_tile_order {
    int TN, TM, bn, bm;
};
// tile number idx of the order -> tile coordinates
SPD_HD void spd_tile_at(const spd_tile_order &o, int idx, int &tn, int &tm) {
    const int row_tiles = o.TN * o.bm, nbm = (o.TM + o.bm - 1) / o.bm, nbn = (o.TN + o.bn - 1) / o.bn;
    int bj = idx / row_tiles;
    bj = bj < nbm - 1 ? bj : nbm - 1;
    const int rest = o.TM - bj * o.bm, hgt = o.bm < rest ? o.bm : rest;
    const int r1 = idx - bj * row_tiles;
    int bi = r1 / (o.bn * hgt);
    bi = bi < nbn - 1 ? bi : nbn - 1;
    const int restn = o.TN - bi * o.bn, w = o.bn < restn ? o.bn : restn;
    const int r2 = r1 - bi * o.bn * hgt;
    tn = bi * o.bn + r2 % w;
    tm = bj * o.bm + r2 / w;
}
// Workgroup b = 8 q + x of a launch of n_tiles tiles runs on XCD x.  Whole rounds of 256 tiles: the XCDs
// take the runs of 32 consecutive tiles in turn, so that the eight runs in flight are neighbours too (the
// epilogues of a round then write whole rows of the output between them; handing each XCD a far-apart
// eighth of the order cost the O projection 20 %).  The ragged rest: eight equal shares.  Returns the
// tile's number in [0, n_tiles), or -1 for a spare workgroup of a ragged share.
SPD_HD int spd_tile_deal(int b, int n_tiles) {
    const int full = n_tiles & ~255;
    if (b < full) {
        const int x = b & 7, q = b >> 3;
        return (((q >> 5) << 3) + x) * 32 + (q & 31);
    }
    const int x = (b - full) & 7, q = (b - full) >> 3, share = (n_tiles - full + 7) >> 3;
    const int idx = full + x * share + q;
    return (q >= share || idx >= n_tiles) ? -1 : idx;
}
SPD_HD int spd_tile_launch_size(int n_tiles) { return (n_tiles & ~255) + (((n_tiles & 255) + 7) / 8) * 8; }
// block shape for tiles of rn x rm rows: at most 32 tiles, the fewest panel rows per tile in flight
inline void spd_pick_block(int TN, int TM, int rn, int rm, int &bn, int &bm) {
    static const int cand[][2] = {{4, 8}, {8, 4}, {5, 6}, {6, 5}, {3, 10}, {10, 3}, {2, 16}, {16, 2}, {1, 32}, {32, 1}};
    double best = 1e30;
    bn = 1;
    bm = 1;
    for (const auto &cd : cand) {
        const int a = cd[0] < TN ? cd[0] : TN, b = cd[1] < TM ? cd[1] : TM;
        // panel rows per tile; blocks of fewer than 32 tiles drift against the 32 tiles an XCD has in flight
        const double cost = (double)(a * rn + b * rm) / (double)(a * b) * (32.0 / (double)(a * b));
        if (cost < best) {
            best = cost;
            bn = a;
            bm = b;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Derived dimensions of one rank's share, and byte offsets of everything the library lays out.
// ------------------------------------------------------------------------------------------
struct spd_dims {
    int h, q, kv, d, f, f_pad, group, nqkv, tp, dtype;
    int gud_cols, gud_groups;     // decode-only gate/up copy: FFN columns per workgroup and number of groups (0: none)
    size_t w_gud;                 // its offset in a layer's packed weights
    int o_bias;                   // the output projection has a bias, kept at w_bo (fp32, [h])
    size_t w_bo;
    int max_batch, max_ctx, max_tokens, m_pad;
    float eps, rope_base;
    // packed shard (bytes from its start)
    size_t w_g1, w_g2, w_qkv, w_o, w_g, w_u, w_d, weight_bytes;   // w_u: f32 path only (bf16: gate/up interleaved at w_g)
    // bf16 path: the four matrices are stored as round_fp16(2^k w), one k per matrix; w_scale holds the four
    // factors 2^-k (fp32; 0 QKV, 1 O, 2 gate/up incl. its decode-only copy, 3 down) that undo it
    size_t w_scale;
    // KV cache (bytes)
    size_t kv_v, kv_bytes;
    // workspace (bytes)
    size_t ws_cos, ws_sin, ws_xhat, ws_xhat2, ws_q, ws_ahat, ws_y, ws_r, ws_ss1, ws_ss2, ws_uhat,
        ws_apart, ws_kpart, ws_qkv, ws_gu, workspace_bytes;
    // a context for long prefills of several sequences lays out two such workspaces back to back (ws_single bytes
    // each), one per chain of the two-chain model forward
    int ws_dual;
    size_t ws_single;
    // bf16 path: every packed activation buffer has a second plane (the "lo" halves) this many
    // elements after the first
    size_t pl_x, pl_a, pl_u;
    size_t kpart_tiles;           // capacity of ws_kpart in pairs of 16x16 fp32 tiles (2 KiB each)
};

struct spd_ctx {
    uint64_t id;                             // unique per spd_create() in this process, never 0
    spd_config cfg;
    spd_dims D;
    std::vector<float> rope_cos, rope_sin;   // [max_ctx][d/2], built in double on the host
};

struct spd_positions {
    int32_t pos[SPD_MAX_BATCH];
};

inline size_t spd_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Stage selection and timing of one call (test and benchmark aid, declared in spd_testing.h): a call
// launches the stages whose bit is set in `stages`; with a timer, every launch of the timer's stage is
// bracketed by a pair of events on the call's stream.  Both travel with the call, nothing is global.
struct spd_stage_timer {
    int stage = -1;
    int n = 0;
    std::vector<hipEvent_t> start, stop;
};

// ------------------------------------------------------------------------------------------
// Launchers (defined next to their kernels).  All enqueue on `s` and return a hipError_t.
// ------------------------------------------------------------------------------------------
struct spd_call {
    const spd_dims *D;
    hipStream_t s;
    int batch, q_len, M;
    size_t slot_stride;       // elements between two ranks' slots (a chain of a two-chain call keeps the whole call's)
    spd_positions pos;
    int max_pos_end;          // max over sequences of positions[b] + q_len
    // bf16 path: which projection inputs are carried as hi + lo pairs of fp16 values
    bool sp_x;                // first norm's output (input of the QKV projection)
    bool sp_a;                // attention output (input of the O projection)
    bool sp_m;                // second norm's output and SwiGLU output (inputs of the MLP's projections)
    int nch1;                 // number of sum-of-squares partials per token waiting in ss1
    char *ws;                 // workspace
    const spd_taps *taps;
    bool chained;             // one of the two chains of a long prefill: its kernels share the chip with the other chain's
    uint32_t stages;          // bit s set: the kernels of stage s are launched (all set in an ordinary call)
    spd_stage_timer *timer;   // NULL, or the timer that brackets the launches of its stage
    bool on(int stage) const { return (stages >> stage) & 1u; }
};
inline void spd_stage_begin(const spd_call &c, int stage) {
    spd_stage_timer *t = c.timer;
    if (t && t->stage == stage && t->n < (int)t->start.size()) (void)hipEventRecord(t->start[t->n], c.s);
}
inline void spd_stage_end(const spd_call &c, int stage) {
    spd_stage_timer *t = c.timer;
    if (t && t->stage == stage && t->n < (int)t->start.size()) {
        (void)hipEventRecord(t->stop[t->n], c.s);
        ++t->n;
    }
}
struct spd_stage_scope {
    const spd_call &c;
    int stage;
    spd_stage_scope(const spd_call &call, int st) : c(call), stage(st) { spd_stage_begin(c, stage); }
    ~spd_stage_scope() { spd_stage_end(c, stage); }
};

namespace spd_common {
// out = base + (slot_0 + ... ) [+ bias[i % h] when bias is given]
hipError_t rank_sum(const float *base, const float *slots, int n_slots, int64_t n, float *out, hipStream_t s,
                    const float *bias = nullptr, int h = 0);
hipError_t fill_zero_u32(uint32_t *p, size_t n, hipStream_t s);
hipError_t copy2d(const float *src, int lds, float *dst, int ldd, int rows, int cols, hipStream_t s);
}

namespace spd_f32 {
// attention half of a rank's share: X -> Y_r (into ybuf or the slot), fp32 path
hipError_t attention_half(const spd_call &c, const char *w, char *kvc, const float *x, float *y_out);
// MLP half: r_in -> Z_r, out[m][n] = (add ? add[m][n] : 0) + Z_r
hipError_t mlp_half(const spd_call &c, const char *w, const float *r_in, const float *add, float *out);
}

namespace spd_bf16 {
// benchmark aid (spd_testing.h): rate of register-resident MFMAs over a full grid
hipError_t mfma_probe(int iters, int random_data, void *scratch, hipStream_t s, double *tflops, double *mhz);
// benchmark aid (spd_testing.h): mean time of launches that only read chunk_bytes each
hipError_t read_probe(const void *buf, size_t chunk_bytes, int n_chunks, int reps, void *sink, hipStream_t s, double *us);
// out = base + sum slots (optional), xhat = fp16(out * g) packed (optional), partial sums of squares
// which = 0: the block's first norm (xhat, ss1); which = 1: its second norm (xhat2, ss2)
// bias (may be NULL): [h], added to `out` after the sum
hipError_t prep(const spd_call &c, const float *base, const float *slots, int n_slots, float *out,
                const float *gain, bool want_xhat, int which, const float *bias = nullptr);
// QKV + rotary + cache append + attention + O projection.
//   spd = 1: ybuf <- Y_r, xhat2 <- fp16((X + Y_r) g2) and its partial sums of squares
//   spd = 0: slot <- Y_r
// With `mid` (TP block, one rank, calls of at most 512 tokens) the O projection's epilogue also performs
// the kept attention sync point: R = X + sum of the slots (+ bias) -> mid->rbuf, second norm prepared;
// *mid_done tells whether it did (otherwise the caller runs prep()).
struct spd_mid_sync {
    const float *slots;       // [tp][M*h]
    int tp, rank;
    float *rbuf;
};
hipError_t attention_half(const spd_call &c, const char *w, char *kvc, const float *x, int spd, float *slot,
                          const spd_mid_sync *mid = nullptr, bool *mid_done = nullptr);
// The sync point that ends a block, for one rank whose peers' partial sums are already in
// `slots`: x_out = base + (slot_0 + ... + slot_tp-1), optionally followed by the elementwise
// part of the next block's first norm (gain next_g1, may be NULL).
struct spd_end_sync {
    const float *base;        // X (SPD block) or R (TP block)
    const float *slots;       // [tp][M*h]
    int tp, rank;
    float *x_out;
    const float *next_g1;
    const float *bias;        // [h] added once after the sum (SPD block with bias), or NULL
};
// gate/up + SwiGLU + down.  spd = 1: slot <- ybuf + Z_r; spd = 0: slot <- Z_r.  With `fuse`
// (calls of at most 16 tokens) the down projection's epilogue also performs the end-of-block
// sync point; returns through *fused whether it did.
// ss_per_pair: the sums of squares of the MLP input were left per pair of n-tiles (by the O projection's
// epilogue) rather than per prep() chunk
hipError_t mlp_half(const spd_call &c, const char *w, int spd, float *slot, const spd_end_sync *fuse, bool *fused,
                    bool ss_per_pair);
int prep_chunks(const spd_call &c);
}
