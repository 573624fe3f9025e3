// bf16 path: MFMA (16x16x32 bf16, fp32 accumulate) kernels for gfx950 over the packed
// fragment layouts described in spd_internal.h.
//
// Orientation used everywhere: the *weights* (or keys / values) are the first MFMA operand,
// the *activations* (or queries / probabilities) the second, so an accumulator tile is
// D[output feature][token]: lane l holds token (l % 16) and the 4 consecutive output
// features 4*(l/16) .. 4*(l/16)+3.  Four consecutive features per lane is exactly what the
// next contraction wants as its packed operand, so every epilogue stores 8-byte pieces
// straight into the next kernel's fragment layout.
#include "spd_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16((a), (b), (c), 0, 0, 0)

__device__ __forceinline__ bf16x4 cvt4(float a, float b, float c, float d) {
    bf16x4 r;
    r[0] = (__bf16)a; r[1] = (__bf16)b; r[2] = (__bf16)c; r[3] = (__bf16)d;
    return r;
}
__device__ __forceinline__ float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, 64); }

// 1 / sqrt(mean(x^2) + eps) of row m from `nch` partial sums of squares ss[c][m]; the four
// lanes that share a token each add a quarter of the partials (fixed order).
__device__ __forceinline__ float row_rsqrt(const float *__restrict__ ss, int nch, int m_pad, int m, int g, int h,
                                           float eps) {
    float s = 0.f;
    for (int c = g; c < nch; c += 4) s += ss[(size_t)c * m_pad + m];
    s += shfl_xor_f(s, 16);
    s += shfl_xor_f(s, 32);
    return 1.0f / sqrtf(s / (float)h + eps);
}

// ------------------------------------------------------------------------------------------
// prep: out = base + (slot0 + slot1 + ...), xhat = bf16(out * gain) in packed layout, and the
// partial sums of squares of `out` per (k-chunk, token).  One wave per (m-tile, chunk of
// `tpw` k-tiles); lane l handles token l%16 and 8 consecutive features.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_prep(const float *__restrict__ base, const float *__restrict__ slots,
                                              int n_slots, size_t slot_stride, float *__restrict__ out,
                                              const float *__restrict__ gain, __bf16 *__restrict__ xhat,
                                              float *__restrict__ ss, int M, int h, int tpw, int m_pad) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KT = h >> 5;
    const int chunk = blockIdx.x * 4 + wave;
    const int mt = blockIdx.y;
    const int m = mt * 16 + (lane & 15), g = lane >> 4;
    const bool valid = m < M;
    float ssum = 0.f;
    for (int t = 0; t < tpw; ++t) {
        const int kt = chunk * tpw + t;
        if (kt >= KT) break;
        const int col = kt * 32 + g * 8;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.f;
        if (valid) {
            const size_t o = (size_t)m * h + col;
            if (n_slots > 0) {
                float4 a0 = *(const float4 *)(slots + o), a1 = *(const float4 *)(slots + o + 4);
                for (int s = 1; s < n_slots; ++s) {
                    const float4 b0 = *(const float4 *)(slots + s * slot_stride + o);
                    const float4 b1 = *(const float4 *)(slots + s * slot_stride + o + 4);
                    a0.x += b0.x; a0.y += b0.y; a0.z += b0.z; a0.w += b0.w;
                    a1.x += b1.x; a1.y += b1.y; a1.z += b1.z; a1.w += b1.w;
                }
                v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w;
                v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
            }
            if (base) {
                const float4 b0 = *(const float4 *)(base + o), b1 = *(const float4 *)(base + o + 4);
                v[0] = b0.x + v[0]; v[1] = b0.y + v[1]; v[2] = b0.z + v[2]; v[3] = b0.w + v[3];
                v[4] = b1.x + v[4]; v[5] = b1.y + v[5]; v[6] = b1.z + v[6]; v[7] = b1.w + v[7];
            }
            if (out) {
                *(float4 *)(out + o) = make_float4(v[0], v[1], v[2], v[3]);
                *(float4 *)(out + o + 4) = make_float4(v[4], v[5], v[6], v[7]);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) ssum += v[i] * v[i];
        if (xhat) {
            bf16x8 x;
            if (valid) {
                const float4 g0 = *(const float4 *)(gain + col), g1 = *(const float4 *)(gain + col + 4);
                x[0] = (__bf16)(v[0] * g0.x); x[1] = (__bf16)(v[1] * g0.y);
                x[2] = (__bf16)(v[2] * g0.z); x[3] = (__bf16)(v[3] * g0.w);
                x[4] = (__bf16)(v[4] * g1.x); x[5] = (__bf16)(v[5] * g1.y);
                x[6] = (__bf16)(v[6] * g1.z); x[7] = (__bf16)(v[7] * g1.w);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = (__bf16)0.f;
            }
            *(bf16x8 *)(xhat + spd_frag_index(mt, kt, KT) + lane * 8) = x;
        }
    }
    ssum += shfl_xor_f(ssum, 16);
    ssum += shfl_xor_f(ssum, 32);
    if (ss && g == 0 && chunk * tpw < KT) ss[(size_t)chunk * m_pad + m] = ssum;
}

// ------------------------------------------------------------------------------------------
// Epilogues.  Each receives the accumulators of one (pair of n-tiles, m-tile): a = tile
// 2*pair, b = tile 2*pair+1; lane l: token m = mt*16 + l%16, features 4*(l/16) + i.
// ------------------------------------------------------------------------------------------
struct EpiQKV {
    int M, q_len, q, kv, d, h, max_ctx, nch, m_pad;
    float eps;
    const float *ss, *cosT, *sinT;
    __bf16 *qbuf, *kc, *vc;
    spd_positions P;

    __device__ __forceinline__ void operator()(int pair, int mt, f32x4 a, f32x4 b, int lane) const {
        const int m = mt * 16 + (lane & 15), g = lane >> 4;
        const float rs = row_rsqrt(ss, nch, m_pad, m, g, h, eps);
        if (m >= M) return;
        const int tph = d >> 4, half = d >> 1;
        const int head = (2 * pair) / tph;
        const int bseq = m / q_len, pos = P.pos[bseq] + (m % q_len);
        const int ca = spd_qkv_tile_col0(2 * pair, q, kv, d) - head * d + 4 * g;       // column inside the head
        const int cb = spd_qkv_tile_col0(2 * pair + 1, q, kv, d) - head * d + 4 * g;
        a *= rs;
        b *= rs;
        if (head < q + kv) {
            // rotary partners: a holds j = ca .. ca+3 (< d/2), b holds j + d/2
            const float4 c = *(const float4 *)(cosT + (size_t)pos * half + ca);
            const float4 s = *(const float4 *)(sinT + (size_t)pos * half + ca);
            const bf16x4 lo = cvt4(a[0] * c.x - b[0] * s.x, a[1] * c.y - b[1] * s.y, a[2] * c.z - b[2] * s.z,
                                   a[3] * c.w - b[3] * s.w);
            const bf16x4 hi = cvt4(b[0] * c.x + a[0] * s.x, b[1] * c.y + a[1] * s.y, b[2] * c.z + a[2] * s.z,
                                   b[3] * c.w + a[3] * s.w);
            if (head < q) {
                __bf16 *dst = qbuf + (size_t)m * (q * d) + head * d;
                *(bf16x4 *)(dst + ca) = lo;
                *(bf16x4 *)(dst + cb) = hi;
            } else {
                __bf16 *dst = kc + ((size_t)bseq * kv + (head - q)) * (size_t)max_ctx * d;
                *(bf16x4 *)(dst + spd_kcache_off(pos, ca, d)) = lo;
                *(bf16x4 *)(dst + spd_kcache_off(pos, cb, d)) = hi;
            }
        } else {
            __bf16 *dst = vc + ((size_t)bseq * kv + (head - q - kv)) * (size_t)max_ctx * d;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                dst[spd_vcache_off(pos, ca + i, d)] = (__bf16)a[i];
                dst[spd_vcache_off(pos, cb + i, d)] = (__bf16)b[i];
            }
        }
    }
};

struct EpiO {
    int M, h, spd, m_pad;
    const float *x, *g2;
    float *ybuf, *slot, *ss2;
    __bf16 *xhat2;

    __device__ __forceinline__ void operator()(int pair, int mt, f32x4 a, f32x4 b, int lane) const {
        const int r = lane & 15, m = mt * 16 + r, g = lane >> 4;
        const int na = pair * 32 + 4 * g, nb = na + 16;
        const bool valid = m < M;
        if (!spd) {
            if (valid) {
                *(float4 *)(slot + (size_t)m * h + na) = make_float4(a[0], a[1], a[2], a[3]);
                *(float4 *)(slot + (size_t)m * h + nb) = make_float4(b[0], b[1], b[2], b[3]);
            }
            return;
        }
        float ra[4] = {0.f, 0.f, 0.f, 0.f}, rb[4] = {0.f, 0.f, 0.f, 0.f};
        bf16x4 xa = cvt4(0.f, 0.f, 0.f, 0.f), xb = xa;
        if (valid) {
            const size_t o = (size_t)m * h;
            *(float4 *)(ybuf + o + na) = make_float4(a[0], a[1], a[2], a[3]);
            *(float4 *)(ybuf + o + nb) = make_float4(b[0], b[1], b[2], b[3]);
            const float4 x0 = *(const float4 *)(x + o + na), x1 = *(const float4 *)(x + o + nb);
            ra[0] = x0.x + a[0]; ra[1] = x0.y + a[1]; ra[2] = x0.z + a[2]; ra[3] = x0.w + a[3];
            rb[0] = x1.x + b[0]; rb[1] = x1.y + b[1]; rb[2] = x1.z + b[2]; rb[3] = x1.w + b[3];
            const float4 ga = *(const float4 *)(g2 + na), gb = *(const float4 *)(g2 + nb);
            xa = cvt4(ra[0] * ga.x, ra[1] * ga.y, ra[2] * ga.z, ra[3] * ga.w);
            xb = cvt4(rb[0] * gb.x, rb[1] * gb.y, rb[2] * gb.z, rb[3] * gb.w);
        }
        // the pair's 32 features are k-tile `pair` of the next contraction
        __bf16 *fr = xhat2 + spd_frag_index(mt, pair, h >> 5);
        *(bf16x4 *)(fr + spd_frag_elem(r, 4 * g)) = xa;
        *(bf16x4 *)(fr + spd_frag_elem(r, 16 + 4 * g)) = xb;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) s += ra[i] * ra[i] + rb[i] * rb[i];
        s += shfl_xor_f(s, 16);
        s += shfl_xor_f(s, 32);
        if (g == 0) ss2[(size_t)pair * m_pad + m] = s;
    }
};

struct EpiGU {
    int M, h, f_pad, nch, m_pad;
    float eps;
    const float *ss;
    __bf16 *uhat;

    __device__ __forceinline__ void operator()(int pair, int mt, f32x4 a, f32x4 b, int lane) const {
        const int r = lane & 15, m = mt * 16 + r, g = lane >> 4;
        const float rs = row_rsqrt(ss, nch, m_pad, m, g, h, eps);
        bf16x4 u = cvt4(0.f, 0.f, 0.f, 0.f);
        if (m < M) {
            float o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float gt = a[i] * rs, up = b[i] * rs;
                o[i] = gt / (1.0f + __expf(-gt)) * up;
            }
            u = cvt4(o[0], o[1], o[2], o[3]);
        }
        // gate/up pair p covers FFN columns [16p, 16p+16): half of k-tile p/2 of the down projection
        __bf16 *fr = uhat + spd_frag_index(mt, pair >> 1, f_pad >> 5);
        *(bf16x4 *)(fr + spd_frag_elem(r, 16 * (pair & 1) + 4 * g)) = u;
    }
};

struct EpiDown {
    int M, h, spd;
    const float *ybuf;
    float *slot;

    __device__ __forceinline__ void operator()(int pair, int mt, f32x4 a, f32x4 b, int lane) const {
        const int m = mt * 16 + (lane & 15), g = lane >> 4;
        if (m >= M) return;
        const size_t oa = (size_t)m * h + pair * 32 + 4 * g, ob = oa + 16;
        if (spd) {   // Y_r joins the partial sum before the sync point (Sec. 4.1.1)
            const float4 ya = *(const float4 *)(ybuf + oa), yb = *(const float4 *)(ybuf + ob);
            a[0] += ya.x; a[1] += ya.y; a[2] += ya.z; a[3] += ya.w;
            b[0] += yb.x; b[1] += yb.y; b[2] += yb.z; b[3] += yb.w;
        }
        *(float4 *)(slot + oa) = make_float4(a[0], a[1], a[2], a[3]);
        *(float4 *)(slot + ob) = make_float4(b[0], b[1], b[2], b[3]);
    }
};

// ------------------------------------------------------------------------------------------
// GEMM, fragments streamed straight from global memory (no reuse through LDS).
//   out^T[n][m] = sum_k W[k][n] x[m][k]
// grid.x = pairs of n-tiles, grid.y = groups of m-tiles.
// SPLITK = true : the W waves of a workgroup split K, partial accumulators are added through
//                 LDS in fixed wave order (deterministic); one m-group of MT tiles per workgroup.
// SPLITK = false: each wave owns its own MT m-tiles and runs the whole K.
// ------------------------------------------------------------------------------------------
template <int MT, int W, bool SPLITK, class Epi>
__global__ void __launch_bounds__(W * 64) k_gemm(const __bf16 *__restrict__ Wp, const __bf16 *__restrict__ Xp, int KT,
                                                  int n_mtiles, Epi epi) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pair = blockIdx.x;
    const int mt0 = SPLITK ? blockIdx.y * MT : (blockIdx.y * W + wave) * MT;
    int k0 = 0, k1 = KT;
    if (SPLITK) {
        k0 = (int)(((long)wave * KT) / W);
        k1 = (int)(((long)(wave + 1) * KT) / W);
    }
    f32x4 acc[MT][2];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        acc[i][0] = (f32x4){0.f, 0.f, 0.f, 0.f};
        acc[i][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const bf16x8 *wa = (const bf16x8 *)(Wp + spd_frag_index(2 * pair, 0, KT)) + lane;
    const bf16x8 *wb = (const bf16x8 *)(Wp + spd_frag_index(2 * pair + 1, 0, KT)) + lane;
    const bf16x8 *xp[MT];
    bool mv[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        mv[i] = (mt0 + i) < n_mtiles;
        xp[i] = (const bf16x8 *)(Xp + spd_frag_index(mv[i] ? mt0 + i : 0, 0, KT)) + lane;
    }
    if (SPLITK || mv[0]) {
#pragma unroll 4
        for (int kt = k0; kt < k1; ++kt) {
            const bf16x8 fa = wa[(size_t)kt * 64], fb = wb[(size_t)kt * 64];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const bf16x8 fx = xp[i][(size_t)kt * 64];
                acc[i][0] = MFMA(fa, fx, acc[i][0]);
                acc[i][1] = MFMA(fb, fx, acc[i][1]);
            }
        }
    }
    if (SPLITK && W > 1) {
        __shared__ f32x4 red[W][MT * 2][64];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            red[wave][2 * i][lane] = acc[i][0];
            red[wave][2 * i + 1][lane] = acc[i][1];
        }
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            f32x4 s0 = red[0][2 * i][lane], s1 = red[0][2 * i + 1][lane];
            for (int w = 1; w < W; ++w) {
                s0 += red[w][2 * i][lane];
                s1 += red[w][2 * i + 1][lane];
            }
            acc[i][0] = s0;
            acc[i][1] = s1;
        }
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
        if (mv[i]) epi(pair, mt0 + i, acc[i][0], acc[i][1], lane);
}

// ------------------------------------------------------------------------------------------
// Attention.  Scores are computed transposed, S^T[key][col] = K q, so that the probabilities
// leave the MFMA already in the operand layout of the second contraction O^T = V^T P^T.
// A "column" is a (token, query head of the KV group) pair: col = t * group + c.
// ------------------------------------------------------------------------------------------
template <int DT>   // DT = head_dim / 16
struct AttnState {
    f32x4 o[DT];    // O^T[d = dt*16 + 4g + i][col = lane%16], unnormalised
    float m, l;     // running max (of scaled scores) and sum for col = lane%16
};

// one 32-key block: keys [vb*32, vb*32+32) of one (sequence, KV head); n_keys_col = number of
// keys column lane%16 may attend (causal), 0 for a padding column
template <int DT>
__device__ __forceinline__ void attn_block(AttnState<DT> &st, const bf16x8 *__restrict__ qf, const __bf16 *__restrict__ kbase,
                                           const __bf16 *__restrict__ vbase, int vb, int d, int n_keys_col, float scale,
                                           int lane) {
    const int g = lane >> 4;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
    const bf16x8 *k0 = (const bf16x8 *)(kbase + (size_t)(2 * vb) * 16 * d) + lane;
    const bf16x8 *k1 = (const bf16x8 *)(kbase + (size_t)(2 * vb + 1) * 16 * d) + lane;
#pragma unroll
    for (int t = 0; t < DT / 2; ++t) {
        s0 = MFMA(k0[t * 64], qf[t], s0);
        s1 = MFMA(k1[t * 64], qf[t], s1);
    }
    const int key0 = vb * 32 + 4 * g;
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s0[i] = (key0 + i < n_keys_col) ? s0[i] * scale : -INFINITY;
        s1[i] = (key0 + 16 + i < n_keys_col) ? s1[i] * scale : -INFINITY;
        mx = fmaxf(mx, fmaxf(s0[i], s1[i]));
    }
    mx = fmaxf(mx, shfl_xor_f(mx, 16));
    mx = fmaxf(mx, shfl_xor_f(mx, 32));
    const float m_new = fmaxf(st.m, mx);
    // every key of this block masked for this column and nothing seen before: keep the state
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __expf(st.m - m_use);          // exp(-inf) = 0 on the first block
    float p0[4], p1[4], ps = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        p0[i] = __expf(s0[i] - m_use);
        p1[i] = __expf(s1[i] - m_use);
        ps += p0[i] + p1[i];
    }
    ps += shfl_xor_f(ps, 16);
    ps += shfl_xor_f(ps, 32);
    st.l = st.l * alpha + ps;
    st.m = m_new;
    bf16x8 pb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pb[i] = (__bf16)p0[i];
        pb[4 + i] = (__bf16)p1[i];
    }
    const bf16x8 *vf = (const bf16x8 *)(vbase + (size_t)vb * 32 * d) + lane;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        st.o[dt] *= alpha;
        st.o[dt] = MFMA(vf[dt * 64], pb, st.o[dt]);
    }
}

// query fragments of one column tile: col -> (token t, head c); zero for padding columns
template <int DT>
__device__ __forceinline__ void load_q(bf16x8 *qf, const __bf16 *__restrict__ qbuf, int m, int head, int qd, int d,
                                       bool valid, int lane) {
    const int g = lane >> 4;
#pragma unroll
    for (int t = 0; t < DT / 2; ++t) {
        if (valid) {
            qf[t] = *(const bf16x8 *)(qbuf + (size_t)m * qd + head * d + t * 32 + g * 8);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[t][i] = (__bf16)0.f;
        }
    }
}

// Decode (q_len = 1): grid (splits, kv heads, sequences), 4 waves.  The waves of a workgroup
// take the 32-key blocks of their split round-robin; the workgroup writes one partial
// (unnormalised O^T, running max, running sum) per split.
// partial layout: [seq][kvh][split][(d + 2) * 16] floats: O^T[d][16], m[16], l[16]
template <int DT>
__global__ void __launch_bounds__(256) k_attn_decode(const __bf16 *__restrict__ qbuf, const __bf16 *__restrict__ kc,
                                                     const __bf16 *__restrict__ vc, float *__restrict__ part, spd_positions P,
                                                     int q, int kv, int max_ctx, int n_splits) {
    constexpr int d = DT * 16;
    __shared__ float sm[4][(DT * 16 + 2) * 16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int group = q / kv, qd = q * d;
    const int n_keys = P.pos[b] + 1;
    const int nblk = (n_keys + 31) >> 5;
    const int b0 = (int)(((long)split * nblk) / n_splits), b1 = (int)(((long)(split + 1) * nblk) / n_splits);
    const int col = lane & 15, g = lane >> 4;
    const bool cvalid = col < group;
    bf16x8 qf[DT / 2];
    load_q<DT>(qf, qbuf, b, kvh * group + col, qd, d, cvalid, lane);
    const __bf16 *kbase = kc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    const __bf16 *vbase = vc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    AttnState<DT> st;
#pragma unroll
    for (int i = 0; i < DT; ++i) st.o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
    const float scale = 1.0f / sqrtf((float)d);
    for (int vb = b0 + wave; vb < b1; vb += 4) attn_block<DT>(st, qf, kbase, vbase, vb, d, cvalid ? n_keys : 0, scale, lane);
    // merge the four waves
    float *my = sm[wave];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) my[(dt * 16 + 4 * g + i) * 16 + col] = st.o[dt][i];
    if (g == 0) {
        my[d * 16 + col] = st.m;
        my[(d + 1) * 16 + col] = st.l;
    }
    __syncthreads();
    float *dst = part + (((size_t)b * kv + kvh) * n_splits + split) * (size_t)((d + 2) * 16);
    for (int e = threadIdx.x; e < (d + 2) * 16; e += 256) {
        const int c = e & 15, row = e >> 4;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, sm[w][d * 16 + c]);
        float v;
        if (row == d) {
            v = mm;
        } else {
            v = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float mw = sm[w][d * 16 + c];
                const float sc = (mw == -INFINITY) ? 0.f : __expf(mw - mm);
                v += sm[w][row * 16 + c] * sc;
            }
        }
        dst[e] = v;
    }
}

// merge the splits of one (sequence, KV head) and write the normalised output as packed
// activations of the O projection: row = token, contraction index = head*d + dd
__global__ void __launch_bounds__(256) k_attn_combine(const float *__restrict__ part, __bf16 *__restrict__ ahat, int q, int kv,
                                                      int d, int n_splits) {
    const int kvh = blockIdx.x, b = blockIdx.y;
    const int group = q / kv, qd = q * d;
    const size_t pstride = (size_t)(d + 2) * 16;
    const float *src = part + ((size_t)b * kv + kvh) * n_splits * pstride;
    for (int e = threadIdx.x; e < group * d; e += 256) {
        const int c = e / d, dd = e % d;
        float mm = -INFINITY;
        for (int s = 0; s < n_splits; ++s) mm = fmaxf(mm, src[s * pstride + d * 16 + c]);
        float num = 0.f, den = 0.f;
        for (int s = 0; s < n_splits; ++s) {
            const float ms = src[s * pstride + d * 16 + c];
            const float sc = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
            num += src[s * pstride + dd * 16 + c] * sc;
            den += src[s * pstride + (d + 1) * 16 + c] * sc;
        }
        const int kidx = (kvh * group + c) * d + dd;
        ahat[spd_frag_index(b >> 4, kidx >> 5, qd >> 5) + spd_frag_elem(b & 15, kidx & 31)] = (__bf16)(num / den);
    }
}

// Prefill (q_len > 1): grid (column-tile groups, kv heads, sequences), 4 waves, each wave owns
// CT column tiles of 16 (token, head) columns and walks the causal key range once.
template <int DT, int CT>
__global__ void __launch_bounds__(256) k_attn_prefill(const __bf16 *__restrict__ qbuf, const __bf16 *__restrict__ kc,
                                                      const __bf16 *__restrict__ vc, __bf16 *__restrict__ ahat, spd_positions P,
                                                      int q_len, int q, int kv, int max_ctx) {
    constexpr int d = DT * 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int group = q / kv, qd = q * d;
    const int n_cols = q_len * group;
    const int ct0 = (blockIdx.x * 4 + wave) * CT;
    if (ct0 * 16 >= n_cols) return;
    const int g = lane >> 4;
    const int pos0 = P.pos[b];
    bf16x8 qf[CT][DT / 2];
    AttnState<DT> st[CT];
    int nk[CT], mrow[CT], hd[CT];
    int last_key = 0;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const int col = (ct0 + c) * 16 + (lane & 15);
        const bool valid = col < n_cols;
        const int t = col / group;
        hd[c] = kvh * group + col % group;
        mrow[c] = b * q_len + t;
        nk[c] = valid ? pos0 + t + 1 : 0;
        load_q<DT>(qf[c], qbuf, mrow[c], hd[c], qd, d, valid, lane);
#pragma unroll
        for (int i = 0; i < DT; ++i) st[c].o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
        st[c].m = -INFINITY;
        st[c].l = 0.f;
        last_key = max(last_key, nk[c]);
    }
    // the block range must be wave-uniform: take the maximum over the wave's columns
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) last_key = max(last_key, __shfl_xor(last_key, o, 64));
    const __bf16 *kbase = kc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    const __bf16 *vbase = vc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    const float scale = 1.0f / sqrtf((float)d);
    const int nblk = (last_key + 31) >> 5;
    for (int vb = 0; vb < nblk; ++vb) {
#pragma unroll
        for (int c = 0; c < CT; ++c) attn_block<DT>(st[c], qf[c], kbase, vbase, vb, d, nk[c], scale, lane);
    }
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        if (nk[c] == 0) continue;
        const float inv = 1.0f / st[c].l;
        const int mt = mrow[c] >> 4, r = mrow[c] & 15;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int kidx = hd[c] * d + dt * 16 + 4 * g;
            const bf16x4 v = cvt4(st[c].o[dt][0] * inv, st[c].o[dt][1] * inv, st[c].o[dt][2] * inv, st[c].o[dt][3] * inv);
            *(bf16x4 *)(ahat + spd_frag_index(mt, kidx >> 5, qd >> 5) + spd_frag_elem(r, kidx & 31)) = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
// taps (tests only): packed bf16 -> natural fp32
// ------------------------------------------------------------------------------------------
__global__ void k_unpack_act(const __bf16 *__restrict__ src, float *__restrict__ dst, int M, int K_packed, int K_out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)M * K_out) return;
    const int m = (int)(i / K_out), k = (int)(i % K_out);
    dst[i] = (float)src[spd_frag_index(m >> 4, k >> 5, K_packed >> 5) + spd_frag_elem(m & 15, k & 31)];
}
__global__ void k_bf16_to_f32(const __bf16 *__restrict__ src, float *__restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (float)src[i];
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

#define SPD_TRY(x)                       \
    do {                                 \
        hipError_t e_ = (x);             \
        if (e_ != hipSuccess) return e_; \
    } while (0)

template <class Epi>
hipError_t launch_gemm(const __bf16 *Wp, const __bf16 *Xp, int n_pairs, int KT, int M, const Epi &epi, hipStream_t s) {
    const int n_mtiles = (M + 15) / 16;
    if (n_mtiles == 1) {
        // skinny: one m-tile, the waves of a workgroup split K
        constexpr int W = 8;
        hipLaunchKernelGGL((k_gemm<1, W, true, Epi>), dim3(n_pairs, 1), dim3(W * 64), 0, s, Wp, Xp, KT, n_mtiles, epi);
    } else {
        constexpr int MT = 4, W = 4;
        hipLaunchKernelGGL((k_gemm<MT, W, false, Epi>), dim3(n_pairs, cdiv(n_mtiles, MT * W)), dim3(W * 64), 0, s, Wp, Xp,
                           KT, n_mtiles, epi);
    }
    return hipGetLastError();
}

// chunking of the sum-of-squares partials written by prep()
inline int prep_tpw(int M) { return M <= 64 ? 1 : 8; }
inline int prep_nch(int h, int M) { return (int)cdiv(h / 32, prep_tpw(M)); }

}  // namespace

namespace spd_bf16 {

hipError_t prep(const spd_call &c, const float *base, const float *slots, int n_slots, float *out, const float *gain,
                bool want_xhat, int which) {
    const spd_dims &D = *c.D;
    const int tpw = prep_tpw(c.M), nch = prep_nch(D.h, c.M);
    __bf16 *xhat = want_xhat ? (__bf16 *)(c.ws + (which ? D.ws_xhat2 : D.ws_xhat)) : nullptr;
    float *ss = want_xhat ? (float *)(c.ws + (which ? D.ws_ss2 : D.ws_ss1)) : nullptr;
    if (n_slots == 0 && out == base) out = nullptr;   // nothing to rewrite
    spd_profile::scope prof(SPD_STAGE_PREP, c.s);
    hipLaunchKernelGGL(k_prep, dim3(cdiv(nch, 4), cdiv(c.M, 16)), dim3(256), 0, c.s, base, slots, n_slots,
                       (size_t)c.M * D.h, out, gain, xhat, ss, c.M, D.h, tpw, D.m_pad);
    return hipGetLastError();
}

hipError_t attention_half(const spd_call &c, const char *w, char *kvc, const float *x, int spd, float *slot) {
    const spd_dims &D = *c.D;
    const int M = c.M, qd = D.q * D.d;
    const __bf16 *xhat = (const __bf16 *)(c.ws + D.ws_xhat);
    __bf16 *qbuf = (__bf16 *)(c.ws + D.ws_q), *ahat = (__bf16 *)(c.ws + D.ws_ahat);
    __bf16 *kc = (__bf16 *)kvc, *vc = (__bf16 *)(kvc + D.kv_v);
    float *ybuf = (float *)(c.ws + D.ws_y);

    EpiQKV e1;
    e1.M = M; e1.q_len = c.q_len; e1.q = D.q; e1.kv = D.kv; e1.d = D.d; e1.h = D.h; e1.max_ctx = D.max_ctx;
    e1.nch = prep_nch(D.h, M); e1.m_pad = D.m_pad; e1.eps = D.eps;
    e1.ss = (const float *)(c.ws + D.ws_ss1);
    e1.cosT = (const float *)(c.ws + D.ws_cos); e1.sinT = (const float *)(c.ws + D.ws_sin);
    e1.qbuf = qbuf; e1.kc = kc; e1.vc = vc; e1.P = c.pos;
    {
        spd_profile::scope prof(SPD_STAGE_QKV, c.s);
        SPD_TRY(launch_gemm((const __bf16 *)(w + D.w_qkv), xhat, D.nqkv / 32, D.h / 32, M, e1, c.s));
    }

    const int DT = D.d / 16;
    spd_profile::begin(SPD_STAGE_ATTN, c.s);
    if (c.q_len == 1) {
        const int nblk = (c.max_pos_end + 31) / 32;
        int splits = nblk / 4;
        if (splits < 1) splits = 1;
        if (splits > SPD_MAX_SPLITS) splits = SPD_MAX_SPLITS;
        float *part = (float *)(c.ws + D.ws_apart);
        const dim3 grid(splits, D.kv, c.batch);
#define SPD_DECODE(DTV)                                                                                          \
    hipLaunchKernelGGL((k_attn_decode<DTV>), grid, dim3(256), 0, c.s, qbuf, kc, vc, part, c.pos, D.q, D.kv, D.max_ctx, \
                       splits)
        switch (DT) {
            case 2: SPD_DECODE(2); break;
            case 4: SPD_DECODE(4); break;
            case 6: SPD_DECODE(6); break;
            case 8: SPD_DECODE(8); break;
            default: return hipErrorInvalidValue;
        }
#undef SPD_DECODE
        SPD_TRY(hipGetLastError());
        hipLaunchKernelGGL(k_attn_combine, dim3(D.kv, c.batch), dim3(256), 0, c.s, part, ahat, D.q, D.kv, D.d, splits);
        SPD_TRY(hipGetLastError());
    } else {
        constexpr int CT = 2;
        const int n_ct = (c.q_len * D.group + 15) / 16;
        const dim3 grid(cdiv(n_ct, 4 * CT), D.kv, c.batch);
#define SPD_PREFILL(DTV)                                                                                              \
    hipLaunchKernelGGL((k_attn_prefill<DTV, CT>), grid, dim3(256), 0, c.s, qbuf, kc, vc, ahat, c.pos, c.q_len, D.q, D.kv, \
                       D.max_ctx)
        switch (DT) {
            case 2: SPD_PREFILL(2); break;
            case 4: SPD_PREFILL(4); break;
            case 6: SPD_PREFILL(6); break;
            case 8: SPD_PREFILL(8); break;
            default: return hipErrorInvalidValue;
        }
#undef SPD_PREFILL
        SPD_TRY(hipGetLastError());
    }
    spd_profile::end(SPD_STAGE_ATTN, c.s);

    EpiO e2;
    e2.M = M; e2.h = D.h; e2.spd = spd; e2.m_pad = D.m_pad;
    e2.x = x; e2.g2 = (const float *)(w + D.w_g2);
    e2.ybuf = ybuf; e2.slot = slot; e2.ss2 = (float *)(c.ws + D.ws_ss2);
    e2.xhat2 = (__bf16 *)(c.ws + D.ws_xhat2);
    {
        spd_profile::scope prof(SPD_STAGE_O, c.s);
        SPD_TRY(launch_gemm((const __bf16 *)(w + D.w_o), ahat, D.h / 32, qd / 32, M, e2, c.s));
    }

    if (c.taps) {
        if (c.taps->q) {
            hipLaunchKernelGGL(k_bf16_to_f32, dim3(cdiv((int64_t)M * qd, 256)), dim3(256), 0, c.s, qbuf, c.taps->q,
                               (int64_t)M * qd);
            SPD_TRY(hipGetLastError());
        }
        if (c.taps->attn) {
            hipLaunchKernelGGL(k_unpack_act, dim3(cdiv((int64_t)M * qd, 256)), dim3(256), 0, c.s, ahat, c.taps->attn, M, qd, qd);
            SPD_TRY(hipGetLastError());
        }
        if (c.taps->y) SPD_TRY(spd_common::copy2d(spd ? ybuf : slot, D.h, c.taps->y, D.h, M, D.h, c.s));
    }
    return hipSuccess;
}

hipError_t mlp_half(const spd_call &c, const char *w, int spd, float *slot, int nch2) {
    const spd_dims &D = *c.D;
    const int M = c.M;
    const __bf16 *xhat = (const __bf16 *)(c.ws + D.ws_xhat2);
    __bf16 *uhat = (__bf16 *)(c.ws + D.ws_uhat);

    EpiGU e1;
    e1.M = M; e1.h = D.h; e1.f_pad = D.f_pad; e1.nch = nch2; e1.m_pad = D.m_pad; e1.eps = D.eps;
    e1.ss = (const float *)(c.ws + D.ws_ss2);
    e1.uhat = uhat;
    {
        spd_profile::scope prof(SPD_STAGE_GATEUP, c.s);
        SPD_TRY(launch_gemm((const __bf16 *)(w + D.w_g), xhat, D.f_pad / 16, D.h / 32, M, e1, c.s));
    }

    EpiDown e2;
    e2.M = M; e2.h = D.h; e2.spd = spd;
    e2.ybuf = (const float *)(c.ws + D.ws_y); e2.slot = slot;
    {
        spd_profile::scope prof(SPD_STAGE_DOWN, c.s);
        SPD_TRY(launch_gemm((const __bf16 *)(w + D.w_d), uhat, D.h / 32, D.f_pad / 32, M, e2, c.s));
    }

    if (c.taps && c.taps->u) {
        hipLaunchKernelGGL(k_unpack_act, dim3(cdiv((int64_t)M * D.f, 256)), dim3(256), 0, c.s, uhat, c.taps->u, M, D.f_pad, D.f);
        SPD_TRY(hipGetLastError());
    }
    return hipSuccess;
}

hipError_t mlp_half(const spd_call &c, const char *w, int spd, float *slot) {
    // SPD block: the O-projection epilogue wrote one partial per pair of n-tiles (h/32 of them);
    // TP block: prep() wrote them after the kept sync point
    const int nch2 = spd ? c.D->h / 32 : prep_nch(c.D->h, c.M);
    return mlp_half(c, w, spd, slot, nch2);
}

}  // namespace spd_bf16
