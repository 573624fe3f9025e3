// Host side of the SPD library: configuration checks, rank indexing, the sync-point count,
// and the packers that lay one rank's shard and KV cache out the way the kernels read them.
// Nothing in this file touches a device.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>

#include "spd_internal.h"

namespace {

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// fp32 -> bf16 bit pattern; false if the value is not exactly representable
inline bool to_bf16_exact(float v, uint16_t *out) {
    uint32_t u;
    std::memcpy(&u, &v, 4);
    *out = (uint16_t)(u >> 16);
    return (u & 0xFFFFu) == 0;
}
inline float from_bf16(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float v;
    std::memcpy(&v, &u, 4);
    return v;
}

// fp32 -> IEEE binary16 bit pattern, round to nearest even (subnormals kept, overflow to infinity)
inline uint16_t to_f16(float v) {
    uint32_t u;
    std::memcpy(&u, &v, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    u &= 0x7FFFFFFFu;
    if (u >= 0x7F800000u) return (uint16_t)(sign | (u > 0x7F800000u ? 0x7E00u : 0x7C00u));   // NaN / infinity
    if (u >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);                                   // rounds to >= 65520: infinity
    if (u < 0x38800000u) {                            // below 2^-14: a multiple of 2^-24
        if (u < 0x33000000u) return (uint16_t)sign;   // below 2^-25: zero (2^-25 itself ties to even = 0)
        const int e = (int)(u >> 23);                 // biased exponent, 102 .. 112
        const uint32_t m = (u & 0x7FFFFFu) | 0x800000u;
        const int shift = 126 - e;                    // 14 .. 24: value = m * 2^(e-150), unit 2^-24
        const uint32_t q = m >> shift, rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
        return (uint16_t)(sign | (q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u)));
    }
    const uint32_t q = (u - 0x38000000u) >> 13, rem = u & 0x1FFFu;      // rebias 127 -> 15, drop 13 mantissa bits
    return (uint16_t)(sign | (q + ((rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ? 1u : 0u)));
}
inline float from_f16(uint16_t b) {
    const uint32_t sign = (uint32_t)(b & 0x8000u) << 16, e = (b >> 10) & 0x1Fu, m = b & 0x3FFu;
    float v;
    if (e == 0) {
        v = std::ldexp((float)m, -24);
    } else if (e == 31) {
        const uint32_t u = 0x7F800000u | (m << 13);
        std::memcpy(&v, &u, 4);
    } else {
        const uint32_t u = ((e + 112u) << 23) | (m << 13);
        std::memcpy(&v, &u, 4);
    }
    uint32_t u;
    std::memcpy(&u, &v, 4);
    u |= sign;
    std::memcpy(&v, &u, 4);
    return v;
}

template <class F>
void parallel_for(int n, F f) {
    int nt = (int)std::thread::hardware_concurrency();
    if (nt < 1) nt = 1;
    if (nt > 16) nt = 16;
    if (nt > n) nt = n;
    if (nt <= 1) {
        for (int i = 0; i < n; ++i) f(i);
        return;
    }
    std::vector<std::thread> th;
    for (int t = 0; t < nt; ++t)
        th.emplace_back([=]() {
            for (int i = t; i < n; i += nt) f(i);
        });
    for (auto &t : th) t.join();
}

void compute_dims(const spd_config &c, spd_dims &D) {
    std::memset(&D, 0, sizeof(D));
    D.h = c.hidden;
    D.q = c.n_q_heads / c.tp_degree;
    D.kv = c.n_kv_heads / c.tp_degree;
    D.d = c.head_dim;
    D.f = c.ffn / c.tp_degree;
    D.group = D.q / D.kv;
    D.nqkv = (D.q + 2 * D.kv) * D.d;
    D.tp = c.tp_degree;
    D.dtype = c.dtype;
    D.max_batch = c.max_batch;
    D.max_ctx = c.max_ctx;
    D.max_tokens = c.max_tokens;
    D.eps = c.rms_eps;
    D.rope_base = c.rope_base;
    const bool bf = c.dtype == SPD_BF16;
    D.f_pad = bf ? round_up(D.f, 32) : D.f;
    D.m_pad = round_up(c.max_tokens, 16);
    const size_t es = bf ? 2 : 4;
    const size_t h = D.h, qd = (size_t)D.q * D.d, f = D.f_pad;

    size_t o = 0;
    D.w_g1 = o; o = spd_align256(o + h * 4);
    D.w_g2 = o; o = spd_align256(o + h * 4);
    D.o_bias = c.o_bias;
    if (c.o_bias) { D.w_bo = o; o = spd_align256(o + h * 4); }
    if (bf) { D.w_scale = o; o = spd_align256(o + 4 * 4); }
    D.w_qkv = o; o = spd_align256(o + h * (size_t)D.nqkv * es);
    D.w_o = o; o = spd_align256(o + qd * h * es);
    D.w_g = o; o = spd_align256(o + h * f * es);
    D.w_u = o; o = spd_align256(o + h * f * es);     // bf16: second half of the interleaved gate/up block
    D.w_d = o; o = spd_align256(o + f * h * es);
    // Decode streams the gate/up weights with one workgroup per group of FFN columns.  When the
    // 16-column tiles of the block above do not fill a whole number of rounds of the chip's 256
    // compute units, a second copy with narrower groups (c < 16 columns) is kept for decode so
    // that they do: group p holds, for every k-tile, the c gate rows then the c up rows of the
    // columns [c p, c p + c), 16 bytes (8 contraction elements) per row and quarter of the k-tile.
    if (bf) {
        const int pairs = D.f_pad / 16;
        const int want = 256 * ((pairs + 255) / 256);
        const int c = (D.f_pad + want - 1) / want;
        // (from 64 tile pairs on: below that the K-sliced launch of the 16-column tiles does as well)
        if (pairs >= 64 && want != pairs && c < 16) {
            D.gud_cols = c;
            D.gud_groups = (D.f_pad + c - 1) / c;
            D.w_gud = o;
            o = spd_align256(o + (size_t)D.gud_groups * (h / 32) * 2 * 64 * c);
        }
    }
    D.weight_bytes = o;

    const size_t kvn = (size_t)D.max_batch * D.kv * D.max_ctx * D.d;
    D.kv_v = spd_align256(kvn * es);
    D.kv_bytes = D.kv_v + spd_align256(kvn * es);

    const size_t M = D.m_pad;
    o = 0;
    D.ws_cos = o; o = spd_align256(o + (size_t)D.max_ctx * (D.d / 2) * 4);
    D.ws_sin = o; o = spd_align256(o + (size_t)D.max_ctx * (D.d / 2) * 4);
    D.ws_y = o; o = spd_align256(o + M * h * 4);
    D.ws_r = o; o = spd_align256(o + M * h * 4);
    if (bf) {
        D.pl_x = M * h; D.pl_a = M * qd; D.pl_u = M * f;
        D.ws_xhat = o; o = spd_align256(o + 2 * M * h * 2);
        D.ws_xhat2 = o; o = spd_align256(o + 2 * M * h * 2);
        D.ws_q = o; o = spd_align256(o + 2 * M * qd * 2);
        D.ws_ahat = o; o = spd_align256(o + 2 * M * qd * 2);
        D.ws_ss1 = o; o = spd_align256(o + (h / 32) * M * 4);
        D.ws_ss2 = o; o = spd_align256(o + (h / 32) * M * 4);
        D.ws_uhat = o; o = spd_align256(o + 2 * M * f * 2);
        // partial tiles of the K-sliced launches: the decode sizes always, the 17 .. 128 token kind when calls can be that long
        D.kpart_tiles = D.max_tokens > 16 ? (size_t)SPD_MID_KPART : (size_t)SPD_MAX_KPART;
        // ... and, when calls can be longer than 512 tokens, the slice partials of a K-sliced QKV GEMM: up to
        // 8192 (slice, token) rows of fp32
        if (D.max_tokens > 512) D.kpart_tiles = std::max(D.kpart_tiles, (size_t)8192 * D.nqkv / 512 + 1);
        D.ws_kpart = o; o = spd_align256(o + D.kpart_tiles * 512 * 4);
        D.ws_apart = o;
        o = spd_align256(o + (size_t)D.max_batch * D.kv * SPD_MAX_SPLITS * 16 * (D.d + 2) * 4);
    } else {
        D.ws_xhat = o; o = spd_align256(o + M * h * 4);            // normalised activations
        D.ws_qkv = o; o = spd_align256(o + M * (size_t)D.nqkv * 4);
        D.ws_ahat = o; o = spd_align256(o + M * qd * 4);
        D.ws_gu = o; o = spd_align256(o + M * 2 * f * 4);
        D.ws_uhat = o; o = spd_align256(o + M * f * 4);
    }
    D.ws_single = o;
    D.ws_dual = bf && c.max_batch >= 2 && c.max_tokens / 2 >= SPD_DUAL_MIN_TOKENS;
    D.workspace_bytes = D.ws_dual ? 2 * o : o;
}

// Power of two k for a matrix whose largest magnitude is mx: the largest k with mx 2^k < 2^15 (half of
// fp16's range), clamped to what ldexp of a float can undo.
inline int f16_shift(float mx) {
    if (!(mx > 0.f) || !std::isfinite(mx)) return 0;
    int e;
    std::frexp(mx, &e);                       // mx = m 2^e, m in [0.5, 1)
    int k = 15 - e;
    if (k > 60) k = 60;
    if (k < -60) k = -60;
    return k;
}

// One packed matrix: n_tiles x k_tiles fragments of fp16 elements round_fp16(2^k w).  `src(k, tile, r)`
// returns the fp32 value of contraction index k for row r of tile `tile` (0 where padded); it must be a
// bf16 value (the packer copies values, it never rounds one that fp16 can hold: bf16's 8 significant bits
// fit fp16's 11 for every weight within 2^-29 of the matrix's largest; smaller ones land on the subnormal
// grid, at most 2^-25 / 2^k away).
template <class Src>
bool pack_frags(uint16_t *dst, int n_tiles, int k_tiles, int shift, Src src) {
    const float up = std::ldexp(1.0f, shift);
    std::vector<int> bad(n_tiles, 0);
    parallel_for(n_tiles, [&](int nt) {
        uint16_t scratch;
        for (int kt = 0; kt < k_tiles; ++kt) {
            uint16_t *fr = dst + spd_frag_index(nt, kt, k_tiles);
            for (int c = 0; c < 32; ++c)
                for (int r = 0; r < 16; ++r) {
                    const float v = src(kt * 32 + c, nt, r);
                    if (!to_bf16_exact(v, &scratch)) bad[nt] = 1;
                    fr[spd_frag_elem(r, c)] = to_f16(v * up);
                }
        }
    });
    for (int b : bad)
        if (b) return false;
    return true;
}

template <class Dst>
void unpack_frags(const uint16_t *srcp, int n_tiles, int k_tiles, float down, Dst dst) {
    parallel_for(n_tiles, [&](int nt) {
        for (int kt = 0; kt < k_tiles; ++kt) {
            const uint16_t *fr = srcp + spd_frag_index(nt, kt, k_tiles);
            for (int c = 0; c < 32; ++c)
                for (int r = 0; r < 16; ++r) dst(kt * 32 + c, nt, r, from_f16(fr[spd_frag_elem(r, c)]) * down);
        }
    });
}

// largest magnitude of a [rows, cols] matrix with row stride ld
float max_abs(const float *p, int rows, int cols, int64_t ld) {
    float mx = 0.f;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) mx = std::max(mx, std::fabs(p[(size_t)r * ld + c]));
    return mx;
}

bool weights_ok(const spd_layer_weights *w) {
    return w && w->wq && w->wk && w->wv && w->wo && w->wg && w->wu && w->wd && w->g1 && w->g2;     // bo: see bias_ok()
}

bool bias_ok(const spd_ctx *ctx, const spd_layer_weights *w) { return (ctx->D.o_bias != 0) == (w->bo != nullptr); }

}  // namespace

extern "C" {

const char *spd_strerror(int code) {
    switch (code) {
        case SPD_OK: return "ok";
        case SPD_EINVAL: return "invalid argument";
        case SPD_EUNSUPPORTED: return "unsupported configuration";
        case SPD_EHIP: return "HIP runtime error";
        case SPD_ETOOBIG: return "configuration needs more workspace than the static scratch of spd_block_forward_static holds";
        default: return "unknown error code";
    }
}

int spd_create(const spd_config *cfg, spd_ctx **out) {
    if (!cfg || !out) return SPD_EINVAL;
    *out = nullptr;
    const spd_config &c = *cfg;
    if (c.hidden <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 || c.ffn <= 0 ||
        c.n_layers <= 0 || c.tp_degree <= 0 || c.max_batch <= 0 || c.max_ctx <= 0 || c.max_tokens <= 0)
        return SPD_EINVAL;
    if (!(c.rms_eps >= 0.0f) || !(c.rope_base > 0.0f)) return SPD_EINVAL;
    if (c.head_dim % 2) return SPD_EINVAL;
    if (c.n_q_heads % c.n_kv_heads) return SPD_EINVAL;
    if (c.max_batch > SPD_MAX_BATCH || c.max_ctx % 32) return SPD_EINVAL;
    if (c.max_tokens < c.max_batch) return SPD_EINVAL;
    if (c.dtype != SPD_F32 && c.dtype != SPD_BF16) return SPD_EUNSUPPORTED;
    if (c.o_bias != 0 && c.o_bias != 1) return SPD_EINVAL;
    if (c.act_split != SPD_SPLIT_AUTO && c.act_split != SPD_SPLIT_ALWAYS && c.act_split != SPD_SPLIT_NEVER)
        return SPD_EINVAL;
    if (c.n_kv_heads < c.tp_degree) return SPD_EUNSUPPORTED;   // a KV head shared by several ranks
    if (c.n_q_heads % c.tp_degree || c.n_kv_heads % c.tp_degree || c.ffn % c.tp_degree) return SPD_EINVAL;
    if (c.dtype == SPD_BF16) {
        if (c.hidden % 32 || c.head_dim % 32 || (c.ffn / c.tp_degree) % 16) return SPD_EUNSUPPORTED;
        if ((c.n_q_heads / c.n_kv_heads) > 16) return SPD_EUNSUPPORTED;
        if (c.head_dim > 128) return SPD_EUNSUPPORTED;        // the attention kernels exist for 32, 64, 96 and 128
    } else {
        if (c.head_dim > 256 || c.max_ctx > 8192) return SPD_EUNSUPPORTED;
    }
    spd_ctx *ctx = new (std::nothrow) spd_ctx();
    if (!ctx) return SPD_EINVAL;
    static std::atomic<uint64_t> next_id{1};
    ctx->id = next_id.fetch_add(1);
    ctx->cfg = c;
    compute_dims(c, ctx->D);
    const int half = c.head_dim / 2;
    ctx->rope_cos.resize((size_t)c.max_ctx * half);
    ctx->rope_sin.resize((size_t)c.max_ctx * half);
    for (int j = 0; j < half; ++j) {
        const double theta = std::pow((double)c.rope_base, -2.0 * (double)j / (double)c.head_dim);
        for (int p = 0; p < c.max_ctx; ++p) {
            const double a = (double)p * theta;
            ctx->rope_cos[(size_t)p * half + j] = (float)std::cos(a);
            ctx->rope_sin[(size_t)p * half + j] = (float)std::sin(a);
        }
    }
    *out = ctx;
    return SPD_OK;
}

void spd_destroy(spd_ctx *ctx) { delete ctx; }

int spd_get_config(const spd_ctx *ctx, spd_config *out) {
    if (!ctx || !out) return SPD_EINVAL;
    *out = ctx->cfg;
    return SPD_OK;
}

int spd_get_sizes(const spd_ctx *ctx, spd_sizes *out) {
    if (!ctx || !out) return SPD_EINVAL;
    out->weight_bytes = ctx->D.weight_bytes;
    out->kv_bytes = ctx->D.kv_bytes;
    out->workspace_bytes = ctx->D.workspace_bytes;
    return SPD_OK;
}

static int rank_range(const spd_ctx *ctx, int32_t rank, int per_rank, int32_t *first, int32_t *count) {
    if (!ctx || !first || !count) return SPD_EINVAL;
    if (rank < 0 || rank >= ctx->D.tp) return SPD_EINVAL;
    *first = rank * per_rank;
    *count = per_rank;
    return SPD_OK;
}
int spd_rank_q_heads(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count) {
    return rank_range(ctx, rank, ctx ? ctx->D.q : 0, first, count);
}
int spd_rank_kv_heads(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count) {
    return rank_range(ctx, rank, ctx ? ctx->D.kv : 0, first, count);
}
int spd_rank_ffn_cols(const spd_ctx *ctx, int32_t rank, int32_t *first, int32_t *count) {
    return rank_range(ctx, rank, ctx ? ctx->D.f : 0, first, count);
}

int64_t spd_sync_count(const spd_ctx *ctx, const uint8_t *mask) {
    if (!ctx || !mask) return SPD_EINVAL;
    int64_t n = 0;
    for (int l = 0; l < ctx->cfg.n_layers; ++l) {
        if (mask[l] > 1) return SPD_EINVAL;
        n += mask[l] ? 1 : 2;
    }
    return n;
}

int spd_mask_from_sensitivity(const double *sensitivity, int32_t n_layers, int32_t n_spd, double tau1, double tau2,
                              uint8_t *mask, uint8_t *tier) {
    if (!sensitivity || !mask || n_layers <= 0 || n_spd < 0 || n_spd > n_layers) return SPD_EINVAL;
    if (tau1 != tau1 || tau2 != tau2) return SPD_EINVAL;
    for (int l = 0; l < n_layers; ++l)
        if (sensitivity[l] != sensitivity[l]) return SPD_EINVAL;
    std::vector<int32_t> order(n_layers);
    for (int l = 0; l < n_layers; ++l) order[l] = l;
    // ascending sensitivity; a stable sort keeps blocks of equal sensitivity in index order
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return sensitivity[a] < sensitivity[b]; });
    for (int l = 0; l < n_layers; ++l) {
        mask[l] = 0;
        if (tier) tier[l] = SPD_TIER_TP;
    }
    for (int i = 0; i < n_spd; ++i) {
        const int32_t blk = order[i];
        mask[blk] = 1;
        if (tier) tier[blk] = sensitivity[blk] <= tau1 ? SPD_TIER_ISB : (sensitivity[blk] <= tau2 ? SPD_TIER_SB : SPD_TIER_ESB);
    }
    return SPD_OK;
}

int spd_pack_shard_local(const spd_ctx *ctx, const spd_layer_weights *w, void *packed_host) {
    if (!ctx || !weights_ok(w) || !packed_host || !bias_ok(ctx, w)) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    char *base = (char *)packed_host;
    std::memset(base, 0, D.weight_bytes);
    std::memcpy(base + D.w_g1, w->g1, (size_t)D.h * 4);
    std::memcpy(base + D.w_g2, w->g2, (size_t)D.h * 4);
    if (D.o_bias) std::memcpy(base + D.w_bo, w->bo, (size_t)D.h * 4);
    const int h = D.h, d = D.d, q = D.q, kv = D.kv, f = D.f, qd = q * d, kvd = kv * d;
    if (D.dtype == SPD_F32) {
        float *wqkv = (float *)(base + D.w_qkv);
        for (int k = 0; k < h; ++k) {
            std::memcpy(wqkv + (size_t)k * D.nqkv, w->wq + (size_t)k * w->ld_q, (size_t)qd * 4);
            std::memcpy(wqkv + (size_t)k * D.nqkv + qd, w->wk + (size_t)k * w->ld_k, (size_t)kvd * 4);
            std::memcpy(wqkv + (size_t)k * D.nqkv + qd + kvd, w->wv + (size_t)k * w->ld_v, (size_t)kvd * 4);
            std::memcpy((float *)(base + D.w_g) + (size_t)k * f, w->wg + (size_t)k * w->ld_g, (size_t)f * 4);
            std::memcpy((float *)(base + D.w_u) + (size_t)k * f, w->wu + (size_t)k * w->ld_u, (size_t)f * 4);
        }
        for (int k = 0; k < qd; ++k)
            std::memcpy((float *)(base + D.w_o) + (size_t)k * h, w->wo + (size_t)k * w->ld_o, (size_t)h * 4);
        for (int k = 0; k < f; ++k)
            std::memcpy((float *)(base + D.w_d) + (size_t)k * h, w->wd + (size_t)k * w->ld_d, (size_t)h * 4);
        return SPD_OK;
    }
    bool ok = true;
    // one power of two per matrix (the three parts of QKV share one, gate and up share one)
    const int k_qkv = f16_shift(std::max(max_abs(w->wq, h, qd, w->ld_q), std::max(max_abs(w->wk, h, kvd, w->ld_k), max_abs(w->wv, h, kvd, w->ld_v))));
    const int k_o = f16_shift(max_abs(w->wo, qd, h, w->ld_o));
    const int k_gu = f16_shift(std::max(max_abs(w->wg, h, f, w->ld_g), max_abs(w->wu, h, f, w->ld_u)));
    const int k_d = f16_shift(max_abs(w->wd, f, h, w->ld_d));
    float *sc = (float *)(base + D.w_scale);
    sc[0] = std::ldexp(1.0f, -k_qkv); sc[1] = std::ldexp(1.0f, -k_o); sc[2] = std::ldexp(1.0f, -k_gu); sc[3] = std::ldexp(1.0f, -k_d);
    // QKV: contraction = hidden, tiles in the rotary-interleaved order
    ok &= pack_frags((uint16_t *)(base + D.w_qkv), D.nqkv / 16, h / 32, k_qkv, [&](int k, int nt, int r) {
        const int c = spd_qkv_tile_col0(nt, q, kv, d) + r;
        if (c < qd) return w->wq[(size_t)k * w->ld_q + c];
        if (c < qd + kvd) return w->wk[(size_t)k * w->ld_k + (c - qd)];
        return w->wv[(size_t)k * w->ld_v + (c - qd - kvd)];
    });
    // O: contraction = the rank's q*d attention features
    ok &= pack_frags((uint16_t *)(base + D.w_o), h / 16, qd / 32, k_o,
                     [&](int k, int nt, int r) { return w->wo[(size_t)k * w->ld_o + nt * 16 + r]; });
    // gate/up: even tiles gate, odd tiles up, same 16 columns; columns >= f are zero padding
    ok &= pack_frags((uint16_t *)(base + D.w_g), 2 * D.f_pad / 16, h / 32, k_gu, [&](int k, int nt, int r) {
        const int c = (nt >> 1) * 16 + r;
        if (c >= f) return 0.0f;
        return (nt & 1) ? w->wu[(size_t)k * w->ld_u + c] : w->wg[(size_t)k * w->ld_g + c];
    });
    if (D.gud_cols) {
        const int c = D.gud_cols, KT = h / 32;
        const float up = std::ldexp(1.0f, k_gu);
        std::vector<int> bad(D.gud_groups, 0);
        parallel_for(D.gud_groups, [&](int p) {
            uint16_t scratch;
            for (int kt = 0; kt < KT; ++kt)
                for (int t = 0; t < 2; ++t) {
                    uint16_t *fr = (uint16_t *)(base + D.w_gud) + (((size_t)p * KT + kt) * 2 + t) * (size_t)(32 * c);
                    for (int g = 0; g < 4; ++g)
                        for (int r = 0; r < c; ++r)
                            for (int j = 0; j < 8; ++j) {
                                const int col = p * c + r, k = kt * 32 + g * 8 + j;
                                const float v = col >= f ? 0.0f : (t ? w->wu[(size_t)k * w->ld_u + col] : w->wg[(size_t)k * w->ld_g + col]);
                                if (!to_bf16_exact(v, &scratch)) bad[p] = 1;
                                fr[(g * c + r) * 8 + j] = to_f16(v * up);
                            }
                }
        });
        for (int b : bad)
            if (b) ok = false;
    }
    // down: contraction = the rank's FFN slice (zero rows where padded)
    ok &= pack_frags((uint16_t *)(base + D.w_d), h / 16, D.f_pad / 32, k_d, [&](int k, int nt, int r) {
        return k < f ? w->wd[(size_t)k * w->ld_d + nt * 16 + r] : 0.0f;
    });
    return ok ? SPD_OK : SPD_EINVAL;   // a weight that is not a bf16 value
}

static bool is_permutation(const int32_t *p, int n) {
    std::vector<char> seen(n, 0);
    for (int i = 0; i < n; ++i) {
        if (p[i] < 0 || p[i] >= n || seen[p[i]]) return false;
        seen[p[i]] = 1;
    }
    return true;
}

int spd_pack_shard_grouped(const spd_ctx *ctx, int32_t rank, const spd_layer_weights *dense, const int32_t *kv_heads,
                           const int32_t *mlp_of_rank, void *packed_host) {
    if (!ctx || !weights_ok(dense) || !packed_host || !bias_ok(ctx, dense)) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (rank < 0 || rank >= D.tp) return SPD_EINVAL;
    const int n_kv = ctx->cfg.n_kv_heads;
    if (kv_heads && !is_permutation(kv_heads, n_kv)) return SPD_EINVAL;
    if (mlp_of_rank && !is_permutation(mlp_of_rank, D.tp)) return SPD_EINVAL;
    const int h = D.h, d = D.d, kv = D.kv, g = D.group, qd = D.q * d, kvd = kv * d;
    // gather the device's heads into contiguous matrices: columns of W_Q / W_K / W_V, rows of W_O
    std::vector<float> wq((size_t)h * qd), wk((size_t)h * kvd), wv((size_t)h * kvd), wo((size_t)qd * h);
    for (int j = 0; j < kv; ++j) {
        const int head = kv_heads ? kv_heads[rank * kv + j] : rank * kv + j;
        for (int k = 0; k < h; ++k) {
            std::memcpy(&wk[(size_t)k * kvd + j * d], dense->wk + (size_t)k * dense->ld_k + (size_t)head * d, (size_t)d * 4);
            std::memcpy(&wv[(size_t)k * kvd + j * d], dense->wv + (size_t)k * dense->ld_v + (size_t)head * d, (size_t)d * 4);
            std::memcpy(&wq[(size_t)k * qd + (size_t)j * g * d], dense->wq + (size_t)k * dense->ld_q + (size_t)head * g * d,
                        (size_t)g * d * 4);
        }
        for (int r = 0; r < g * d; ++r)
            std::memcpy(&wo[((size_t)j * g * d + r) * h], dense->wo + ((size_t)head * g * d + r) * dense->ld_o, (size_t)h * 4);
    }
    const int m = mlp_of_rank ? mlp_of_rank[rank] : rank;
    spd_layer_weights s = *dense;
    s.wq = wq.data(); s.ld_q = qd;
    s.wk = wk.data(); s.ld_k = kvd;
    s.wv = wv.data(); s.ld_v = kvd;
    s.wo = wo.data(); s.ld_o = h;
    s.wg += (size_t)m * D.f;
    s.wu += (size_t)m * D.f;
    s.wd += (size_t)m * D.f * (size_t)dense->ld_d;
    return spd_pack_shard_local(ctx, &s, packed_host);
}

int spd_pack_shard(const spd_ctx *ctx, int32_t rank, const spd_layer_weights *dense, void *packed_host) {
    if (!ctx || !weights_ok(dense) || !packed_host || !bias_ok(ctx, dense)) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (rank < 0 || rank >= D.tp) return SPD_EINVAL;
    spd_layer_weights s = *dense;
    s.wq += (size_t)rank * D.q * D.d;                      // column-wise split: the rank's heads
    s.wk += (size_t)rank * D.kv * D.d;
    s.wv += (size_t)rank * D.kv * D.d;
    s.wo += (size_t)rank * D.q * D.d * (size_t)dense->ld_o;   // row-wise split
    s.wg += (size_t)rank * D.f;
    s.wu += (size_t)rank * D.f;
    s.wd += (size_t)rank * D.f * (size_t)dense->ld_d;
    return spd_pack_shard_local(ctx, &s, packed_host);
}

int spd_unpack_shard(const spd_ctx *ctx, const void *packed_host, const spd_layer_weights *o) {
    if (!ctx || !weights_ok(o) || !packed_host) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    const char *base = (const char *)packed_host;
    const int h = D.h, d = D.d, q = D.q, kv = D.kv, f = D.f, qd = q * d, kvd = kv * d;
    float *wq = (float *)o->wq, *wk = (float *)o->wk, *wv = (float *)o->wv, *wo = (float *)o->wo;
    float *wg = (float *)o->wg, *wu = (float *)o->wu, *wd = (float *)o->wd;
    std::memcpy((float *)o->g1, base + D.w_g1, (size_t)h * 4);
    std::memcpy((float *)o->g2, base + D.w_g2, (size_t)h * 4);
    if (D.o_bias && o->bo) std::memcpy((float *)o->bo, base + D.w_bo, (size_t)h * 4);
    if (D.dtype == SPD_F32) {
        const float *wqkv = (const float *)(base + D.w_qkv);
        for (int k = 0; k < h; ++k) {
            std::memcpy(wq + (size_t)k * o->ld_q, wqkv + (size_t)k * D.nqkv, (size_t)qd * 4);
            std::memcpy(wk + (size_t)k * o->ld_k, wqkv + (size_t)k * D.nqkv + qd, (size_t)kvd * 4);
            std::memcpy(wv + (size_t)k * o->ld_v, wqkv + (size_t)k * D.nqkv + qd + kvd, (size_t)kvd * 4);
            std::memcpy(wg + (size_t)k * o->ld_g, (const float *)(base + D.w_g) + (size_t)k * f, (size_t)f * 4);
            std::memcpy(wu + (size_t)k * o->ld_u, (const float *)(base + D.w_u) + (size_t)k * f, (size_t)f * 4);
        }
        for (int k = 0; k < qd; ++k)
            std::memcpy(wo + (size_t)k * o->ld_o, (const float *)(base + D.w_o) + (size_t)k * h, (size_t)h * 4);
        for (int k = 0; k < f; ++k)
            std::memcpy(wd + (size_t)k * o->ld_d, (const float *)(base + D.w_d) + (size_t)k * h, (size_t)h * 4);
        return SPD_OK;
    }
    const float *sc = (const float *)(base + D.w_scale);
    unpack_frags((const uint16_t *)(base + D.w_qkv), D.nqkv / 16, h / 32, sc[0], [&](int k, int nt, int r, float v) {
        const int c = spd_qkv_tile_col0(nt, q, kv, d) + r;
        if (c < qd) wq[(size_t)k * o->ld_q + c] = v;
        else if (c < qd + kvd) wk[(size_t)k * o->ld_k + (c - qd)] = v;
        else wv[(size_t)k * o->ld_v + (c - qd - kvd)] = v;
    });
    unpack_frags((const uint16_t *)(base + D.w_o), h / 16, qd / 32, sc[1],
                 [&](int k, int nt, int r, float v) { wo[(size_t)k * o->ld_o + nt * 16 + r] = v; });
    unpack_frags((const uint16_t *)(base + D.w_g), 2 * D.f_pad / 16, h / 32, sc[2], [&](int k, int nt, int r, float v) {
        const int c = (nt >> 1) * 16 + r;
        if (c >= f) return;
        if (nt & 1) wu[(size_t)k * o->ld_u + c] = v;
        else wg[(size_t)k * o->ld_g + c] = v;
    });
    unpack_frags((const uint16_t *)(base + D.w_d), h / 16, D.f_pad / 32, sc[3], [&](int k, int nt, int r, float v) {
        if (k < f) wd[(size_t)k * o->ld_d + nt * 16 + r] = v;
    });
    return SPD_OK;
}

int spd_kv_pack(const spd_ctx *ctx, const float *k, const float *v, int32_t batch, int32_t n_pos, void *cache_host) {
    if (!ctx || !k || !v || !cache_host) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (batch < 0 || batch > D.max_batch || n_pos < 0 || n_pos > D.max_ctx) return SPD_EINVAL;
    const int d = D.d;
    const size_t per_head = (size_t)D.max_ctx * d;
    std::vector<int> bad(batch * D.kv, 0);
    parallel_for(batch * D.kv, [&](int bh) {
        const float *ks = k + (size_t)bh * n_pos * d, *vs = v + (size_t)bh * n_pos * d;
        if (D.dtype == SPD_F32) {
            float *kd = (float *)cache_host + (size_t)bh * per_head;
            float *vd = (float *)((char *)cache_host + D.kv_v) + (size_t)bh * per_head;
            std::memcpy(kd, ks, (size_t)n_pos * d * 4);
            std::memcpy(vd, vs, (size_t)n_pos * d * 4);
            return;
        }
        uint16_t *kd = (uint16_t *)cache_host + (size_t)bh * per_head;
        uint16_t *vd = (uint16_t *)((char *)cache_host + D.kv_v) + (size_t)bh * per_head;
        for (int p = 0; p < n_pos; ++p)
            for (int c = 0; c < d; ++c) {
                if (!to_bf16_exact(ks[(size_t)p * d + c], &kd[spd_kcache_off(p, c, d)])) bad[bh] = 1;
                if (!to_bf16_exact(vs[(size_t)p * d + c], &vd[spd_vcache_off(p, c, d)])) bad[bh] = 1;
            }
    });
    for (int b : bad)
        if (b) return SPD_EINVAL;
    return SPD_OK;
}

int spd_kv_unpack(const spd_ctx *ctx, const void *cache_host, int32_t batch, int32_t n_pos, float *k, float *v) {
    if (!ctx || !k || !v || !cache_host) return SPD_EINVAL;
    const spd_dims &D = ctx->D;
    if (batch < 0 || batch > D.max_batch || n_pos < 0 || n_pos > D.max_ctx) return SPD_EINVAL;
    const int d = D.d;
    const size_t per_head = (size_t)D.max_ctx * d;
    parallel_for(batch * D.kv, [&](int bh) {
        float *ks = k + (size_t)bh * n_pos * d, *vs = v + (size_t)bh * n_pos * d;
        if (D.dtype == SPD_F32) {
            std::memcpy(ks, (const float *)cache_host + (size_t)bh * per_head, (size_t)n_pos * d * 4);
            std::memcpy(vs, (const float *)((const char *)cache_host + D.kv_v) + (size_t)bh * per_head,
                        (size_t)n_pos * d * 4);
            return;
        }
        const uint16_t *kd = (const uint16_t *)cache_host + (size_t)bh * per_head;
        const uint16_t *vd = (const uint16_t *)((const char *)cache_host + D.kv_v) + (size_t)bh * per_head;
        for (int p = 0; p < n_pos; ++p)
            for (int c = 0; c < d; ++c) {
                ks[(size_t)p * d + c] = from_bf16(kd[spd_kcache_off(p, c, d)]);
                vs[(size_t)p * d + c] = from_bf16(vd[spd_vcache_off(p, c, d)]);
            }
    });
    return SPD_OK;
}

}  // extern "C"

extern "C" int spd_gemm_launch_size(int32_t n_tiles) {
    if (n_tiles < 0) return SPD_EINVAL;
    return spd_tile_launch_size(n_tiles);
}

extern "C" int spd_gemm_tile_of(int32_t TN, int32_t TM, int32_t rn, int32_t rm, int32_t tile0, int32_t n_tiles, int32_t b,
                                int32_t *tn, int32_t *tm) {
    if (!tn || !tm || TN <= 0 || TM <= 0 || rn <= 0 || rm <= 0 || tile0 < 0 || n_tiles < 0 || b < 0) return SPD_EINVAL;
    if ((int64_t)tile0 + n_tiles > (int64_t)TN * TM || b >= spd_tile_launch_size(n_tiles)) return SPD_EINVAL;
    spd_tile_order o;
    o.TN = TN;
    o.TM = TM;
    spd_pick_block(TN, TM, rn, rm, o.bn, o.bm);
    const int idx = spd_tile_deal(b, n_tiles);
    if (idx < 0) return 1;
    int a, m;
    spd_tile_at(o, tile0 + idx, a, m);
    *tn = a;
    *tm = m;
    return 0;
}

