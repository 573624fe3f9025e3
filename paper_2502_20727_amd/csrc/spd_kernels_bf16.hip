// bf16 path: MFMA (16x16x32 bf16, fp32 accumulate) kernels for gfx950 over the packed
// fragment layouts described in spd_internal.h.
//
// Orientation used everywhere: the *weights* (or keys / values) are the first MFMA operand,
// the *activations* (or queries / probabilities) the second, so an accumulator tile is
// D[output feature][token]: lane l holds token (l % 16) and the 4 consecutive output
// features 4*(l/16) .. 4*(l/16)+3.  Four consecutive features per lane is exactly what the
// next contraction wants as its packed operand, so every epilogue stores 8-byte pieces
// straight into the next kernel's fragment layout.
//
// "Split" activations: an activation buffer may carry a second plane holding, for every
// element, the bf16 rounding error of the first plane (x = hi + lo up to 2^-17 relative).
// Contractions then run over both planes.
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
// rounding error of cvt4, itself rounded to bf16
__device__ __forceinline__ bf16x4 cvt4_lo(float a, float b, float c, float d, bf16x4 hi) {
    return cvt4(a - (float)hi[0], b - (float)hi[1], c - (float)hi[2], d - (float)hi[3]);
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
// prep: out = base + (slot0 + slot1 + ...), xhat = bf16(out * gain) in packed layout (plus its
// lo plane), and the partial sums of squares of `out` per (k-chunk, token).  One wave per
// (m-tile, chunk of `tpw` k-tiles); lane l handles token l%16 and 8 consecutive features.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_prep(const float *__restrict__ base, const float *__restrict__ slots,
                                              int n_slots, size_t slot_stride, float *__restrict__ out,
                                              const float *__restrict__ gain, __bf16 *__restrict__ xhat,
                                              __bf16 *__restrict__ xlo, float *__restrict__ ss, int M, int h, int tpw,
                                              int m_pad) {
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
            // partials in ascending slot order; the loads of a group of 8 slots are issued together
            for (int s0 = 0; s0 < n_slots; s0 += 8) {
                float4 p0[8], p1[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (s0 + j < n_slots) {
                        p0[j] = *(const float4 *)(slots + (size_t)(s0 + j) * slot_stride + o);
                        p1[j] = *(const float4 *)(slots + (size_t)(s0 + j) * slot_stride + o + 4);
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (s0 + j < n_slots) {
                        if (s0 + j == 0) {
                            v[0] = p0[j].x; v[1] = p0[j].y; v[2] = p0[j].z; v[3] = p0[j].w;
                            v[4] = p1[j].x; v[5] = p1[j].y; v[6] = p1[j].z; v[7] = p1[j].w;
                        } else {
                            v[0] += p0[j].x; v[1] += p0[j].y; v[2] += p0[j].z; v[3] += p0[j].w;
                            v[4] += p1[j].x; v[5] += p1[j].y; v[6] += p1[j].z; v[7] += p1[j].w;
                        }
                    }
                }
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
            bf16x8 x, xl;
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = xl[i] = (__bf16)0.f;
            if (valid) {
                const float4 g0 = *(const float4 *)(gain + col), g1 = *(const float4 *)(gain + col + 4);
                const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float p = v[i] * gg[i];
                    x[i] = (__bf16)p;
                    xl[i] = (__bf16)(p - (float)x[i]);
                }
            }
            const size_t fo = spd_frag_index(mt, kt, KT) + lane * 8;
            *(bf16x8 *)(xhat + fo) = x;
            if (xlo) *(bf16x8 *)(xlo + fo) = xl;
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
    __bf16 *qbuf, *qlo, *kc, *vc;     // queries are kept as hi + lo pairs
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
            const float l0 = a[0] * c.x - b[0] * s.x, l1 = a[1] * c.y - b[1] * s.y, l2 = a[2] * c.z - b[2] * s.z,
                        l3 = a[3] * c.w - b[3] * s.w;
            const float h0 = b[0] * c.x + a[0] * s.x, h1 = b[1] * c.y + a[1] * s.y, h2 = b[2] * c.z + a[2] * s.z,
                        h3 = b[3] * c.w + a[3] * s.w;
            const bf16x4 lo = cvt4(l0, l1, l2, l3), hi = cvt4(h0, h1, h2, h3);
            if (head < q) {
                const size_t o = (size_t)m * (q * d) + head * d;
                *(bf16x4 *)(qbuf + o + ca) = lo;
                *(bf16x4 *)(qbuf + o + cb) = hi;
                *(bf16x4 *)(qlo + o + ca) = cvt4_lo(l0, l1, l2, l3, lo);
                *(bf16x4 *)(qlo + o + cb) = cvt4_lo(h0, h1, h2, h3, hi);
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
    __bf16 *xhat2, *xlo2;      // xlo2 may be NULL

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
        float pa[4] = {0.f, 0.f, 0.f, 0.f}, pb[4] = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            const size_t o = (size_t)m * h;
            *(float4 *)(ybuf + o + na) = make_float4(a[0], a[1], a[2], a[3]);
            *(float4 *)(ybuf + o + nb) = make_float4(b[0], b[1], b[2], b[3]);
            const float4 x0 = *(const float4 *)(x + o + na), x1 = *(const float4 *)(x + o + nb);
            ra[0] = x0.x + a[0]; ra[1] = x0.y + a[1]; ra[2] = x0.z + a[2]; ra[3] = x0.w + a[3];
            rb[0] = x1.x + b[0]; rb[1] = x1.y + b[1]; rb[2] = x1.z + b[2]; rb[3] = x1.w + b[3];
            const float4 ga = *(const float4 *)(g2 + na), gb = *(const float4 *)(g2 + nb);
            pa[0] = ra[0] * ga.x; pa[1] = ra[1] * ga.y; pa[2] = ra[2] * ga.z; pa[3] = ra[3] * ga.w;
            pb[0] = rb[0] * gb.x; pb[1] = rb[1] * gb.y; pb[2] = rb[2] * gb.z; pb[3] = rb[3] * gb.w;
        }
        const bf16x4 xa = cvt4(pa[0], pa[1], pa[2], pa[3]), xb = cvt4(pb[0], pb[1], pb[2], pb[3]);
        // the pair's 32 features are k-tile `pair` of the next contraction
        const size_t fo = spd_frag_index(mt, pair, h >> 5);
        const int ea = spd_frag_elem(r, 4 * g), eb = spd_frag_elem(r, 16 + 4 * g);
        *(bf16x4 *)(xhat2 + fo + ea) = xa;
        *(bf16x4 *)(xhat2 + fo + eb) = xb;
        if (xlo2) {
            *(bf16x4 *)(xlo2 + fo + ea) = cvt4_lo(pa[0], pa[1], pa[2], pa[3], xa);
            *(bf16x4 *)(xlo2 + fo + eb) = cvt4_lo(pb[0], pb[1], pb[2], pb[3], xb);
        }
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
    __bf16 *uhat, *ulo;        // ulo may be NULL

    __device__ __forceinline__ void operator()(int pair, int mt, f32x4 a, f32x4 b, int lane) const {
        const int r = lane & 15, m = mt * 16 + r, g = lane >> 4;
        const float rs = row_rsqrt(ss, nch, m_pad, m, g, h, eps);
        float o[4] = {0.f, 0.f, 0.f, 0.f};
        if (m < M) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float gt = a[i] * rs, up = b[i] * rs;
                o[i] = gt / (1.0f + __expf(-gt)) * up;
            }
        }
        const bf16x4 u = cvt4(o[0], o[1], o[2], o[3]);
        // gate/up pair p covers FFN columns [16p, 16p+16): half of k-tile p/2 of the down projection
        const size_t fo = spd_frag_index(mt, pair >> 1, f_pad >> 5) + spd_frag_elem(r, 16 * (pair & 1) + 4 * g);
        *(bf16x4 *)(uhat + fo) = u;
        if (ulo) *(bf16x4 *)(ulo + fo) = cvt4_lo(o[0], o[1], o[2], o[3], u);
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
// GEMV-like projection for at most 16 tokens (one m-tile): bound by streaming the weights.
//   out^T[n][m] = sum_k W[k][n] x[m][k]
// grid = (pairs of n-tiles, KS).  A workgroup owns one pair and one of KS slices of K; its W
// waves split that slice, each wave streaming its weight fragments straight from HBM into
// registers in batches of U k-tiles (all loads of a batch are issued before the first MFMA).
// The waves' partial tiles are added through LDS in wave order.  With KS > 1 the workgroups
// of a pair park their partial tile in `kpart`, and the last one to arrive (a counter per
// pair) adds the KS tiles in slice order and runs the epilogue: the result does not depend
// on which workgroup came last, so it is bit-reproducible.  No workgroup ever waits.
// ------------------------------------------------------------------------------------------
template <int W, int U, bool SPLIT, class Epi>
__global__ void __launch_bounds__(W * 64) k_gemv(const __bf16 *__restrict__ Wp, const __bf16 *__restrict__ Xhi,
                                                  const __bf16 *__restrict__ Xlo, int KT, int KS,
                                                  float *__restrict__ kpart, unsigned int *__restrict__ counters, Epi epi) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pair = blockIdx.x, ks = blockIdx.y;
    const int kb0 = (int)(((long)ks * KT) / KS), kb1 = (int)(((long)(ks + 1) * KT) / KS);
    const int nk = kb1 - kb0;
    const int k0 = kb0 + (wave * nk) / W, k1 = kb0 + ((wave + 1) * nk) / W;
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    const bf16x8 *wa = (const bf16x8 *)(Wp + spd_frag_index(2 * pair, 0, KT)) + lane;
    const bf16x8 *wb = (const bf16x8 *)(Wp + spd_frag_index(2 * pair + 1, 0, KT)) + lane;
    const bf16x8 *xh = (const bf16x8 *)Xhi + lane;
    const bf16x8 *xl = (const bf16x8 *)Xlo + lane;
    int kt = k0;
    for (; kt + U <= k1; kt += U) {
        bf16x8 fa[U], fb[U], fh[U], fl[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            fa[u] = __builtin_nontemporal_load(wa + (size_t)(kt + u) * 64);
            fb[u] = __builtin_nontemporal_load(wb + (size_t)(kt + u) * 64);
            fh[u] = xh[(size_t)(kt + u) * 64];
            if (SPLIT) fl[u] = xl[(size_t)(kt + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a = MFMA(fa[u], fh[u], a);
            b = MFMA(fb[u], fh[u], b);
            if (SPLIT) {
                a = MFMA(fa[u], fl[u], a);
                b = MFMA(fb[u], fl[u], b);
            }
        }
    }
    for (; kt < k1; ++kt) {
        const bf16x8 fa = __builtin_nontemporal_load(wa + (size_t)kt * 64);
        const bf16x8 fb = __builtin_nontemporal_load(wb + (size_t)kt * 64);
        const bf16x8 fh = xh[(size_t)kt * 64];
        a = MFMA(fa, fh, a);
        b = MFMA(fb, fh, b);
        if (SPLIT) {
            const bf16x8 fl = xl[(size_t)kt * 64];
            a = MFMA(fa, fl, a);
            b = MFMA(fb, fl, b);
        }
    }
    __shared__ f32x4 red[W][2][64];
    red[wave][0][lane] = a;
    red[wave][1][lane] = b;
    __syncthreads();
    if (wave != 0) return;
    a = red[0][0][lane];
    b = red[0][1][lane];
#pragma unroll
    for (int w = 1; w < W; ++w) {
        a += red[w][0][lane];
        b += red[w][1][lane];
    }
    if (KS > 1) {
        // park the partial tile; agent-scope atomics so that another XCD's L2 sees it
        unsigned int *mine = (unsigned int *)(kpart + ((size_t)pair * KS + ks) * 512) + lane;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __hip_atomic_store(mine + i * 64, __float_as_uint(a[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(mine + (4 + i) * 64, __float_as_uint(b[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        unsigned int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(counters + pair, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        old = __shfl(old, 0, 64);
        if (old != (unsigned int)(KS - 1)) return;   // not the last slice of this pair: done
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        a = (f32x4){0.f, 0.f, 0.f, 0.f};
        b = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < KS; ++s) {
            const unsigned int *src = (const unsigned int *)(kpart + ((size_t)pair * KS + s) * 512) + lane;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] += __uint_as_float(__hip_atomic_load(src + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                b[i] += __uint_as_float(__hip_atomic_load(src + (4 + i) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            }
        }
        if (lane == 0) __hip_atomic_store(counters + pair, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    epi(pair, 0, a, b, lane);
}

// ------------------------------------------------------------------------------------------
// GEMM for more than 16 tokens, fragments streamed straight from global memory: each wave owns
// MT m-tiles and one pair of n-tiles and runs the whole K.  grid = (pairs, groups of W*MT m-tiles).
// ------------------------------------------------------------------------------------------
template <int MT, int W, bool SPLIT, class Epi>
__global__ void __launch_bounds__(W * 64) k_gemm(const __bf16 *__restrict__ Wp, const __bf16 *__restrict__ Xhi,
                                                  const __bf16 *__restrict__ Xlo, int KT, int n_mtiles, Epi epi) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pair = blockIdx.x;
    const int mt0 = (blockIdx.y * W + wave) * MT;
    if (mt0 >= n_mtiles) return;
    f32x4 acc[MT][2];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        acc[i][0] = (f32x4){0.f, 0.f, 0.f, 0.f};
        acc[i][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const bf16x8 *wa = (const bf16x8 *)(Wp + spd_frag_index(2 * pair, 0, KT)) + lane;
    const bf16x8 *wb = (const bf16x8 *)(Wp + spd_frag_index(2 * pair + 1, 0, KT)) + lane;
    const bf16x8 *xp[MT], *xq[MT];
    bool mv[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        mv[i] = (mt0 + i) < n_mtiles;
        const size_t o = spd_frag_index(mv[i] ? mt0 + i : mt0, 0, KT);
        xp[i] = (const bf16x8 *)(Xhi + o) + lane;
        xq[i] = (const bf16x8 *)(Xlo + o) + lane;
    }
#pragma unroll 2
    for (int kt = 0; kt < KT; ++kt) {
        const bf16x8 fa = wa[(size_t)kt * 64], fb = wb[(size_t)kt * 64];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const bf16x8 fx = xp[i][(size_t)kt * 64];
            acc[i][0] = MFMA(fa, fx, acc[i][0]);
            acc[i][1] = MFMA(fb, fx, acc[i][1]);
            if (SPLIT) {
                const bf16x8 fl = xq[i][(size_t)kt * 64];
                acc[i][0] = MFMA(fa, fl, acc[i][0]);
                acc[i][1] = MFMA(fb, fl, acc[i][1]);
            }
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

template <int DT>
struct KVFrags {
    bf16x8 k0[DT / 2], k1[DT / 2], v[DT];
};

// all fragments of one 32-key block: 2 x 16 keys x d for K, d x 32 keys for V
template <int DT>
__device__ __forceinline__ void load_kv(KVFrags<DT> &f, const __bf16 *__restrict__ kbase, const __bf16 *__restrict__ vbase,
                                        int vb, int d, int lane) {
    const bf16x8 *k0 = (const bf16x8 *)(kbase + (size_t)(2 * vb) * 16 * d) + lane;
    const bf16x8 *k1 = (const bf16x8 *)(kbase + (size_t)(2 * vb + 1) * 16 * d) + lane;
    const bf16x8 *vf = (const bf16x8 *)(vbase + (size_t)vb * 32 * d) + lane;
#pragma unroll
    for (int t = 0; t < DT / 2; ++t) {
        f.k0[t] = k0[t * 64];
        f.k1[t] = k1[t * 64];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) f.v[dt] = vf[dt * 64];
}

// one 32-key block: keys [vb*32, vb*32+32) of one (sequence, KV head); n_keys_col = number of
// keys column lane%16 may attend (causal), 0 for a padding column
template <int DT>
__device__ __forceinline__ void attn_block(AttnState<DT> &st, const bf16x8 *__restrict__ qf, const KVFrags<DT> &f, int vb,
                                           int n_keys_col, float scale, int lane) {
    // qf[0 .. DT/2) are the hi halves of the query fragments, qf[DT/2 .. DT) the lo halves
    const int g = lane >> 4;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < DT / 2; ++t) {
        s0 = MFMA(f.k0[t], qf[t], s0);
        s1 = MFMA(f.k1[t], qf[t], s1);
        s0 = MFMA(f.k0[t], qf[DT / 2 + t], s0);
        s1 = MFMA(f.k1[t], qf[DT / 2 + t], s1);
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
    bf16x8 pb, pl;      // probabilities as hi + lo pairs
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pb[i] = (__bf16)p0[i];
        pb[4 + i] = (__bf16)p1[i];
        pl[i] = (__bf16)(p0[i] - (float)pb[i]);
        pl[4 + i] = (__bf16)(p1[i] - (float)pb[4 + i]);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        st.o[dt] *= alpha;
        st.o[dt] = MFMA(f.v[dt], pb, st.o[dt]);
        st.o[dt] = MFMA(f.v[dt], pl, st.o[dt]);
    }
}

// query fragments of one column tile: col -> (token t, head c); zero for padding columns
template <int DT>
__device__ __forceinline__ void load_q(bf16x8 *qf, const __bf16 *__restrict__ qbuf, const __bf16 *__restrict__ qlo, int m,
                                       int head, int qd, int d, bool valid, int lane) {
    const int g = lane >> 4;
#pragma unroll
    for (int t = 0; t < DT / 2; ++t) {
        if (valid) {
            const size_t o = (size_t)m * qd + head * d + t * 32 + g * 8;
            qf[t] = *(const bf16x8 *)(qbuf + o);
            qf[DT / 2 + t] = *(const bf16x8 *)(qlo + o);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[t][i] = qf[DT / 2 + t][i] = (__bf16)0.f;
        }
    }
}

// Decode (q_len = 1): grid (splits, kv heads, sequences), 4 waves.  The waves of a workgroup
// take the 32-key blocks of their split round-robin, the next block's fragments being loaded
// while the current one is processed; the workgroup writes one partial (unnormalised O^T,
// running max, running sum) per split.
// partial layout: [seq][kvh][split][(d + 2) * 16] floats: O^T[d][16], m[16], l[16]
template <int DT>
__global__ void __launch_bounds__(256) k_attn_decode(const __bf16 *__restrict__ qbuf, const __bf16 *__restrict__ qlo, const __bf16 *__restrict__ kc,
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
    const __bf16 *kbase = kc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    const __bf16 *vbase = vc + ((size_t)b * kv + kvh) * (size_t)max_ctx * d;
    AttnState<DT> st;
#pragma unroll
    for (int i = 0; i < DT; ++i) st.o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
    const float scale = 1.0f / sqrtf((float)d);
    int vb = b0 + wave;
    if (vb < b1) {
        KVFrags<DT> cur;
        load_kv<DT>(cur, kbase, vbase, vb, d, lane);
        bf16x8 qf[DT];
        load_q<DT>(qf, qbuf, qlo, b, kvh * group + col, qd, d, cvalid, lane);
        for (; vb < b1; vb += 4) {
            KVFrags<DT> nxt;
            const bool more = vb + 4 < b1;
            if (more) load_kv<DT>(nxt, kbase, vbase, vb + 4, d, lane);
            attn_block<DT>(st, qf, cur, vb, cvalid ? n_keys : 0, scale, lane);
            if (more) cur = nxt;
        }
    }
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
// activations of the O projection: row = token, contraction index = head*d + dd.
// grid (kv heads, sequences, d/32): each workgroup produces 32 features of every head of the group.
__global__ void __launch_bounds__(256) k_attn_combine(const float *__restrict__ part, __bf16 *__restrict__ ahat,
                                                      __bf16 *__restrict__ alo, int q, int kv, int d, int n_splits) {
    __shared__ float wgt[SPD_MAX_SPLITS][16];     // exp(m_s - M) per split and column
    __shared__ float den[16];
    const int kvh = blockIdx.x, b = blockIdx.y, dchunk = blockIdx.z;
    const int group = q / kv, qd = q * d;
    const size_t pstride = (size_t)(d + 2) * 16;
    const float *src = part + ((size_t)b * kv + kvh) * n_splits * pstride;
    const int tid = threadIdx.x;
    for (int e = tid; e < n_splits * 16; e += 256) wgt[e >> 4][e & 15] = src[(size_t)(e >> 4) * pstride + d * 16 + (e & 15)];
    __syncthreads();
    if (tid < 16) {
        float mm = -INFINITY;
        for (int s = 0; s < n_splits; ++s) mm = fmaxf(mm, wgt[s][tid]);
        float dn = 0.f;
        for (int s = 0; s < n_splits; ++s) {
            const float ms = wgt[s][tid];
            const float sc = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
            wgt[s][tid] = sc;
            dn += src[(size_t)s * pstride + (d + 1) * 16 + tid] * sc;
        }
        den[tid] = dn;
    }
    __syncthreads();
    // 32 features x 16 columns per workgroup; thread -> (feature, column) pairs, columns fastest
    for (int e = tid; e < 32 * 16; e += 256) {
        const int c = e & 15, dd = dchunk * 32 + (e >> 4);
        if (c >= group) continue;
        float num = 0.f;
        for (int s0 = 0; s0 < n_splits; s0 += 8) {
            float t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (s0 + j < n_splits) ? src[(size_t)(s0 + j) * pstride + dd * 16 + c] : 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (s0 + j < n_splits) num += t[j] * wgt[s0 + j][c];
        }
        const float val = num / den[c];
        const int kidx = (kvh * group + c) * d + dd;
        const size_t o = spd_frag_index(b >> 4, kidx >> 5, qd >> 5) + spd_frag_elem(b & 15, kidx & 31);
        const __bf16 hi = (__bf16)val;
        ahat[o] = hi;
        if (alo) alo[o] = (__bf16)(val - (float)hi);
    }
}

// Prefill (q_len > 1): grid (column-tile groups, kv heads, sequences), 4 waves, each wave owns
// CT column tiles of 16 (token, head) columns and walks the causal key range once.
template <int DT, int CT>
__global__ void __launch_bounds__(256) k_attn_prefill(const __bf16 *__restrict__ qbuf, const __bf16 *__restrict__ qlo, const __bf16 *__restrict__ kc,
                                                      const __bf16 *__restrict__ vc, __bf16 *__restrict__ ahat,
                                                      __bf16 *__restrict__ alo, spd_positions P, int q_len, int q, int kv,
                                                      int max_ctx) {
    constexpr int d = DT * 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int group = q / kv, qd = q * d;
    const int n_cols = q_len * group;
    const int ct0 = (blockIdx.x * 4 + wave) * CT;
    if (ct0 * 16 >= n_cols) return;
    const int g = lane >> 4;
    const int pos0 = P.pos[b];
    bf16x8 qf[CT][DT];
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
        load_q<DT>(qf[c], qbuf, qlo, mrow[c], hd[c], qd, d, valid, lane);
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
        KVFrags<DT> f;
        load_kv<DT>(f, kbase, vbase, vb, d, lane);
#pragma unroll
        for (int c = 0; c < CT; ++c) attn_block<DT>(st[c], qf[c], f, vb, nk[c], scale, lane);
    }
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        if (nk[c] == 0) continue;
        const float inv = 1.0f / st[c].l;
        const int mt = mrow[c] >> 4, r = mrow[c] & 15;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int kidx = hd[c] * d + dt * 16 + 4 * g;
            const float o0 = st[c].o[dt][0] * inv, o1 = st[c].o[dt][1] * inv, o2 = st[c].o[dt][2] * inv,
                        o3 = st[c].o[dt][3] * inv;
            const bf16x4 v = cvt4(o0, o1, o2, o3);
            const size_t o = spd_frag_index(mt, kidx >> 5, qd >> 5) + spd_frag_elem(r, kidx & 31);
            *(bf16x4 *)(ahat + o) = v;
            if (alo) *(bf16x4 *)(alo + o) = cvt4_lo(o0, o1, o2, o3, v);
        }
    }
}

// ------------------------------------------------------------------------------------------
// taps (tests only): packed bf16 (hi [+ lo]) -> natural fp32
// ------------------------------------------------------------------------------------------
__global__ void k_unpack_act(const __bf16 *__restrict__ src, const __bf16 *__restrict__ lo, float *__restrict__ dst, int M,
                             int K_packed, int K_out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)M * K_out) return;
    const int m = (int)(i / K_out), k = (int)(i % K_out);
    const size_t o = spd_frag_index(m >> 4, k >> 5, K_packed >> 5) + spd_frag_elem(m & 15, k & 31);
    dst[i] = (float)src[o] + (lo ? (float)lo[o] : 0.f);
}
__global__ void k_bf16_to_f32(const __bf16 *__restrict__ src, const __bf16 *__restrict__ lo, float *__restrict__ dst,
                              int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (float)src[i] + (float)lo[i];
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

#define SPD_TRY(x)                       \
    do {                                 \
        hipError_t e_ = (x);             \
        if (e_ != hipSuccess) return e_; \
    } while (0)

// Launch shape of a projection.  At most 16 tokens: the weight-streaming kernel; the number of
// K slices is chosen so that about two workgroups per compute unit are in flight.
template <class Epi>
hipError_t launch_proj(const spd_call &c, const __bf16 *Wp, const __bf16 *Xhi, size_t plane, int n_pairs, int KT,
                       const Epi &epi) {
    const spd_dims &D = *c.D;
    const int M = c.M;
    const int n_mtiles = (M + 15) / 16;
    const __bf16 *Xlo = Xhi + plane;
    if (n_mtiles == 1) {
        float *kpart = (float *)(c.ws + D.ws_kpart);
        unsigned int *counters = (unsigned int *)(c.ws + D.ws_counters);
        if (n_pairs > SPD_N_COUNTERS) return hipErrorInvalidValue;
        if (n_pairs >= 192 && KT >= 64) {
            // enough pairs to occupy the chip: one workgroup of 16 waves per pair, no slices
            constexpr int W = 16, U = 4;
            if (c.split)
                hipLaunchKernelGGL((k_gemv<W, U, true, Epi>), dim3(n_pairs, 1), dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, 1,
                                   kpart, counters, epi);
            else
                hipLaunchKernelGGL((k_gemv<W, U, false, Epi>), dim3(n_pairs, 1), dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, 1,
                                   kpart, counters, epi);
        } else {
            constexpr int W = 8, U = 4;
            int KS = (512 + n_pairs - 1) / n_pairs;
            const int ks_max = KT / W > 0 ? KT / W : 1;         // at least one k-tile per wave
            if (KS > ks_max) KS = ks_max;
            if (KS < 1) KS = 1;
            while ((size_t)n_pairs * KS > (size_t)SPD_MAX_KPART && KS > 1) --KS;
            if (c.split)
                hipLaunchKernelGGL((k_gemv<W, U, true, Epi>), dim3(n_pairs, KS), dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, KS,
                                   kpart, counters, epi);
            else
                hipLaunchKernelGGL((k_gemv<W, U, false, Epi>), dim3(n_pairs, KS), dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, KS,
                                   kpart, counters, epi);
        }
    } else {
        constexpr int MT = 4, W = 4;
        const dim3 grid(n_pairs, cdiv(n_mtiles, MT * W));
        if (c.split)
            hipLaunchKernelGGL((k_gemm<MT, W, true, Epi>), grid, dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, n_mtiles, epi);
        else
            hipLaunchKernelGGL((k_gemm<MT, W, false, Epi>), grid, dim3(W * 64), 0, c.s, Wp, Xhi, Xlo, KT, n_mtiles, epi);
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
    __bf16 *xlo = (want_xhat && c.split) ? xhat + D.pl_x : nullptr;
    float *ss = want_xhat ? (float *)(c.ws + (which ? D.ws_ss2 : D.ws_ss1)) : nullptr;
    if (n_slots == 0 && out == base) out = nullptr;   // nothing to rewrite
    spd_profile::scope prof(SPD_STAGE_PREP, c.s);
    hipLaunchKernelGGL(k_prep, dim3(cdiv(nch, 4), cdiv(c.M, 16)), dim3(256), 0, c.s, base, slots, n_slots,
                       (size_t)c.M * D.h, out, gain, xhat, xlo, ss, c.M, D.h, tpw, D.m_pad);
    return hipGetLastError();
}

hipError_t attention_half(const spd_call &c, const char *w, char *kvc, const float *x, int spd, float *slot) {
    const spd_dims &D = *c.D;
    const int M = c.M, qd = D.q * D.d;
    const __bf16 *xhat = (const __bf16 *)(c.ws + D.ws_xhat);
    __bf16 *qbuf = (__bf16 *)(c.ws + D.ws_q), *ahat = (__bf16 *)(c.ws + D.ws_ahat);
    __bf16 *alo = c.split ? ahat + D.pl_a : nullptr;
    __bf16 *qlo = qbuf + D.pl_a;
    __bf16 *kc = (__bf16 *)kvc, *vc = (__bf16 *)(kvc + D.kv_v);
    float *ybuf = (float *)(c.ws + D.ws_y);

    EpiQKV e1;
    e1.M = M; e1.q_len = c.q_len; e1.q = D.q; e1.kv = D.kv; e1.d = D.d; e1.h = D.h; e1.max_ctx = D.max_ctx;
    e1.nch = prep_nch(D.h, M); e1.m_pad = D.m_pad; e1.eps = D.eps;
    e1.ss = (const float *)(c.ws + D.ws_ss1);
    e1.cosT = (const float *)(c.ws + D.ws_cos); e1.sinT = (const float *)(c.ws + D.ws_sin);
    e1.qbuf = qbuf; e1.qlo = qlo; e1.kc = kc; e1.vc = vc; e1.P = c.pos;
    {
        spd_profile::scope prof(SPD_STAGE_QKV, c.s);
        SPD_TRY(launch_proj(c, (const __bf16 *)(w + D.w_qkv), xhat, D.pl_x, D.nqkv / 32, D.h / 32, e1));
    }

    const int DT = D.d / 16;
    spd_profile::begin(SPD_STAGE_ATTN, c.s);
    if (c.q_len == 1) {
        // about 8 key blocks (256 keys) per workgroup, two per wave
        const int nblk = (c.max_pos_end + 31) / 32;
        int splits = (nblk + 7) / 8;
        if (splits < 1) splits = 1;
        if (splits > SPD_MAX_SPLITS) splits = SPD_MAX_SPLITS;
        float *part = (float *)(c.ws + D.ws_apart);
        const dim3 grid(splits, D.kv, c.batch);
#define SPD_DECODE(DTV)                                                                                          \
    hipLaunchKernelGGL((k_attn_decode<DTV>), grid, dim3(256), 0, c.s, qbuf, qlo, kc, vc, part, c.pos, D.q, D.kv, D.max_ctx, \
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
        hipLaunchKernelGGL(k_attn_combine, dim3(D.kv, c.batch, D.d / 32), dim3(256), 0, c.s, part, ahat, alo, D.q, D.kv,
                           D.d, splits);
        SPD_TRY(hipGetLastError());
    } else {
        constexpr int CT = 2;
        const int n_ct = (c.q_len * D.group + 15) / 16;
        const dim3 grid(cdiv(n_ct, 4 * CT), D.kv, c.batch);
#define SPD_PREFILL(DTV)                                                                                              \
    hipLaunchKernelGGL((k_attn_prefill<DTV, CT>), grid, dim3(256), 0, c.s, qbuf, qlo, kc, vc, ahat, alo, c.pos, c.q_len, D.q, \
                       D.kv, D.max_ctx)
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
    e2.xlo2 = c.split ? e2.xhat2 + D.pl_x : nullptr;
    {
        spd_profile::scope prof(SPD_STAGE_O, c.s);
        SPD_TRY(launch_proj(c, (const __bf16 *)(w + D.w_o), ahat, D.pl_a, D.h / 32, qd / 32, e2));
    }

    if (c.taps) {
        if (c.taps->q) {
            hipLaunchKernelGGL(k_bf16_to_f32, dim3(cdiv((int64_t)M * qd, 256)), dim3(256), 0, c.s, qbuf, qlo, c.taps->q,
                               (int64_t)M * qd);
            SPD_TRY(hipGetLastError());
        }
        if (c.taps->attn) {
            hipLaunchKernelGGL(k_unpack_act, dim3(cdiv((int64_t)M * qd, 256)), dim3(256), 0, c.s, ahat, alo, c.taps->attn, M,
                               qd, qd);
            SPD_TRY(hipGetLastError());
        }
        if (c.taps->y) SPD_TRY(spd_common::copy2d(spd ? ybuf : slot, D.h, c.taps->y, D.h, M, D.h, c.s));
    }
    return hipSuccess;
}

hipError_t mlp_half(const spd_call &c, const char *w, int spd, float *slot) {
    const spd_dims &D = *c.D;
    const int M = c.M;
    const __bf16 *xhat = (const __bf16 *)(c.ws + D.ws_xhat2);
    __bf16 *uhat = (__bf16 *)(c.ws + D.ws_uhat);
    __bf16 *ulo = c.split ? uhat + D.pl_u : nullptr;

    EpiGU e1;
    e1.M = M; e1.h = D.h; e1.f_pad = D.f_pad; e1.m_pad = D.m_pad; e1.eps = D.eps;
    // SPD block: the O-projection epilogue wrote one partial per pair of n-tiles (h/32 of them);
    // TP block: prep() wrote them after the kept sync point
    e1.nch = spd ? D.h / 32 : prep_nch(D.h, M);
    e1.ss = (const float *)(c.ws + D.ws_ss2);
    e1.uhat = uhat; e1.ulo = ulo;
    {
        spd_profile::scope prof(SPD_STAGE_GATEUP, c.s);
        SPD_TRY(launch_proj(c, (const __bf16 *)(w + D.w_g), xhat, D.pl_x, D.f_pad / 16, D.h / 32, e1));
    }

    EpiDown e2;
    e2.M = M; e2.h = D.h; e2.spd = spd;
    e2.ybuf = (const float *)(c.ws + D.ws_y); e2.slot = slot;
    {
        spd_profile::scope prof(SPD_STAGE_DOWN, c.s);
        SPD_TRY(launch_proj(c, (const __bf16 *)(w + D.w_d), uhat, D.pl_u, D.h / 32, D.f_pad / 32, e2));
    }

    if (c.taps && c.taps->u) {
        hipLaunchKernelGGL(k_unpack_act, dim3(cdiv((int64_t)M * D.f, 256)), dim3(256), 0, c.s, uhat, ulo, c.taps->u, M,
                           D.f_pad, D.f);
        SPD_TRY(hipGetLastError());
    }
    return hipSuccess;
}

}  // namespace spd_bf16
