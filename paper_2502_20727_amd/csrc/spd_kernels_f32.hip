// fp32 path: small, plain kernels in natural layouts (used by the toy-sized configuration and
// as the library's generic rank-sum), plus helpers shared by both paths.
#include "spd_internal.h"

namespace {

constexpr int TB = 256;

__global__ void k_rank_sum(const float *__restrict__ base, const float *__restrict__ slots, int n_slots,
                           int64_t n, float *__restrict__ out, const float *__restrict__ bias, int h) {
    // partials are summed in ascending slot order, the base is added last
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float acc = 0.0f;
    if (n_slots > 0) {
        acc = slots[i];
        for (int s = 1; s < n_slots; ++s) acc += slots[(int64_t)s * n + i];
    }
    if (base) acc = base[i] + acc;
    if (bias) acc += bias[i % h];          // the output projection's bias, once, after the sum
    out[i] = acc;
}

__global__ void k_rank_sum4(const float4 *__restrict__ base, const float4 *__restrict__ slots, int n_slots,
                            int64_t n4, float4 *__restrict__ out, const float4 *__restrict__ bias, int h4) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n_slots > 0) {
        acc = slots[i];
        for (int s = 1; s < n_slots; ++s) {
            const float4 v = slots[(int64_t)s * n4 + i];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    if (base) {
        const float4 b = base[i];
        acc.x = b.x + acc.x; acc.y = b.y + acc.y; acc.z = b.z + acc.z; acc.w = b.w + acc.w;
    }
    if (bias) {
        const float4 b = bias[i % h4];
        acc.x += b.x; acc.y += b.y; acc.z += b.z; acc.w += b.w;
    }
    out[i] = acc;
}

__global__ void k_fill_zero(uint32_t *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// y[m][:] = x[m][:] * rsqrt(mean(x^2) + eps) * g      one workgroup per row
__global__ void k_rmsnorm(const float *__restrict__ x, const float *__restrict__ g, float *__restrict__ y, int h,
                          float eps) {
    __shared__ float red[TB];
    const float *xr = x + (size_t)blockIdx.x * h;
    float s = 0.f;
    for (int i = threadIdx.x; i < h; i += TB) s += xr[i] * xr[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = TB / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    const float rs = 1.0f / sqrtf(red[0] / (float)h + eps);
    float *yr = y + (size_t)blockIdx.x * h;
    for (int i = threadIdx.x; i < h; i += TB) yr[i] = xr[i] * rs * g[i];
}

// C[M][N] (ldc) = A[M][K] (lda) * W[K][N] (ldw) (+ add[M][N], ldc).  32x32 tiles, 2x2 per thread.
__global__ void k_gemm(const float *__restrict__ A, int lda, const float *__restrict__ W, int ldw,
                       const float *__restrict__ add, float *__restrict__ C, int ldc, int M, int N, int K) {
    __shared__ float As[32][33];
    __shared__ float Ws[32][33];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int i = threadIdx.x; i < 1024; i += TB) {
            const int r = i >> 5, c = i & 31;
            As[r][c] = (m0 + r < M && k0 + c < K) ? A[(size_t)(m0 + r) * lda + k0 + c] : 0.f;
            Ws[r][c] = (k0 + r < K && n0 + c < N) ? W[(size_t)(k0 + r) * ldw + n0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            const float a0 = As[ty][k], a1 = As[ty + 16][k];
            const float b0 = Ws[k][tx], b1 = Ws[k][tx + 16];
            acc[0][0] += a0 * b0; acc[0][1] += a0 * b1;
            acc[1][0] += a1 * b0; acc[1][1] += a1 * b1;
        }
        __syncthreads();
    }
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            const int m = m0 + ty + 16 * i, n = n0 + tx + 16 * j;
            if (m < M && n < N) {
                const size_t o = (size_t)m * ldc + n;
                C[o] = add ? add[o] + acc[i][j] : acc[i][j];
            }
        }
}

// Rotate queries (in place in the qkv buffer) and keys, append keys and values to the cache.
// qkv: [M][nqkv] = [Q heads | K heads | V heads].  One thread per (token, head, j < d/2).
__global__ void k_rope_append(float *__restrict__ qkv, float *__restrict__ kc, float *__restrict__ vc,
                              const float *__restrict__ cosT, const float *__restrict__ sinT, spd_positions P, int M,
                              int q_len, int q, int kv, int d, int nqkv, int max_ctx) {
    const int half = d >> 1;
    const int per_tok = (q + kv) * half;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)M * per_tok) return;
    const int m = (int)(i / per_tok), r = (int)(i % per_tok);
    const int head = r / half, j = r % half;
    const int b = m / q_len, pos = P.pos[b] + (m % q_len);
    const float c = cosT[(size_t)pos * half + j], s = sinT[(size_t)pos * half + j];
    float *v = qkv + (size_t)m * nqkv + head * d;
    const float lo = v[j], hi = v[j + half];
    const float rlo = lo * c - hi * s, rhi = hi * c + lo * s;
    if (head < q) {
        v[j] = rlo;
        v[j + half] = rhi;
    } else {
        const int kh = head - q;
        const size_t o = (((size_t)b * kv + kh) * max_ctx + pos) * d;
        kc[o + j] = rlo;
        kc[o + j + half] = rhi;
        const float *vv = qkv + (size_t)m * nqkv + (q + kv + kh) * d;
        vc[o + j] = vv[j];
        vc[o + j + half] = vv[j + half];
    }
}

// One workgroup per (token, query head): causal softmax attention over the cache.
__global__ void k_attention(const float *__restrict__ qkv, const float *__restrict__ kc, const float *__restrict__ vc,
                            float *__restrict__ out, spd_positions P, int q_len, int q, int kv, int d, int nqkv,
                            int max_ctx) {
    extern __shared__ float sc[];          // [n_keys] scores, then probabilities
    __shared__ float red[TB];
    const int m = blockIdx.x / q, j = blockIdx.x % q;
    const int b = m / q_len, pos = P.pos[b] + (m % q_len);
    const int n_keys = pos + 1;            // causal: key position <= query position
    const int kh = j / (q / kv);
    const float *qv = qkv + (size_t)m * nqkv + j * d;
    const float *K = kc + ((size_t)b * kv + kh) * max_ctx * d;
    const float *V = vc + ((size_t)b * kv + kh) * max_ctx * d;
    const float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int t = threadIdx.x; t < n_keys; t += TB) {
        float s = 0.f;
        for (int c = 0; c < d; ++c) s += qv[c] * K[(size_t)t * d + c];
        s *= scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int o = TB / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + o]);
        __syncthreads();
    }
    mx = red[0];
    __syncthreads();
    float sum = 0.f;
    for (int t = threadIdx.x; t < n_keys; t += TB) {
        const float e = expf(sc[t] - mx);
        sc[t] = e;
        sum += e;
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int o = TB / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    const float inv = 1.0f / red[0];
    for (int c = threadIdx.x; c < d; c += TB) {
        float a = 0.f;
        for (int t = 0; t < n_keys; ++t) a += sc[t] * V[(size_t)t * d + c];
        out[(size_t)m * (q * d) + j * d + c] = a * inv;
    }
}

__global__ void k_swiglu(const float *__restrict__ g, const float *__restrict__ u, float *__restrict__ out, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float x = g[i];
    out[i] = x / (1.0f + expf(-x)) * u[i];
}

__global__ void k_copy2d(const float *__restrict__ src, int lds, float *__restrict__ dst, int ldd, int rows, int cols) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)rows * cols) return;
    const int r = (int)(i / cols), c = (int)(i % cols);
    dst[(size_t)r * ldd + c] = src[(size_t)r * lds + c];
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + TB - 1) / TB); }

hipError_t gemm(const float *A, int lda, const float *W, int ldw, const float *add, float *C, int ldc, int M, int N,
                int K, hipStream_t s) {
    dim3 grid((N + 31) / 32, (M + 31) / 32);
    hipLaunchKernelGGL(k_gemm, grid, dim3(TB), 0, s, A, lda, W, ldw, add, C, ldc, M, N, K);
    return hipGetLastError();
}

}  // namespace

namespace spd_common {

hipError_t rank_sum(const float *base, const float *slots, int n_slots, int64_t n, float *out, hipStream_t s,
                    const float *bias, int h) {
    if (n <= 0) return hipSuccess;
    const bool al = ((((uintptr_t)base) | ((uintptr_t)slots) | ((uintptr_t)out) | ((uintptr_t)bias)) & 15) == 0 &&
                    (n % 4) == 0 && (!bias || h % 4 == 0);
    if (al)
        hipLaunchKernelGGL(k_rank_sum4, dim3(blocks_for(n / 4)), dim3(TB), 0, s, (const float4 *)base,
                           (const float4 *)slots, n_slots, n / 4, (float4 *)out, (const float4 *)bias, h / 4);
    else
        hipLaunchKernelGGL(k_rank_sum, dim3(blocks_for(n)), dim3(TB), 0, s, base, slots, n_slots, n, out, bias, h);
    return hipGetLastError();
}

hipError_t fill_zero_u32(uint32_t *p, size_t n, hipStream_t s) {
    if (!n) return hipSuccess;
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks_for((int64_t)n)), dim3(TB), 0, s, p, n);
    return hipGetLastError();
}

hipError_t copy2d(const float *src, int lds, float *dst, int ldd, int rows, int cols, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_copy2d, dim3(blocks_for((int64_t)rows * cols)), dim3(TB), 0, s, src, lds, dst, ldd, rows, cols);
    return hipGetLastError();
}

}  // namespace spd_common

namespace spd_f32 {

#define SPD_TRY(x)                        \
    do {                                  \
        hipError_t e_ = (x);              \
        if (e_ != hipSuccess) return e_;  \
    } while (0)

hipError_t attention_half(const spd_call &c, const char *w, char *kvc, const float *x, float *y_out) {
    const spd_dims &D = *c.D;
    const int M = c.M, qd = D.q * D.d;
    float *xn = (float *)(c.ws + D.ws_xhat), *qkv = (float *)(c.ws + D.ws_qkv), *att = (float *)(c.ws + D.ws_ahat);
    const float *cosT = (const float *)(c.ws + D.ws_cos), *sinT = (const float *)(c.ws + D.ws_sin);
    float *kc = (float *)kvc, *vc = (float *)(kvc + D.kv_v);
    hipLaunchKernelGGL(k_rmsnorm, dim3(M), dim3(TB), 0, c.s, x, (const float *)(w + D.w_g1), xn, D.h, D.eps);
    SPD_TRY(hipGetLastError());
    SPD_TRY(gemm(xn, D.h, (const float *)(w + D.w_qkv), D.nqkv, nullptr, qkv, D.nqkv, M, D.nqkv, D.h, c.s));
    const int64_t nro = (int64_t)M * (D.q + D.kv) * (D.d / 2);
    hipLaunchKernelGGL(k_rope_append, dim3(blocks_for(nro)), dim3(TB), 0, c.s, qkv, kc, vc, cosT, sinT, c.pos, M,
                       c.q_len, D.q, D.kv, D.d, D.nqkv, D.max_ctx);
    SPD_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_attention, dim3(M * D.q), dim3(TB), (size_t)c.max_pos_end * sizeof(float), c.s, qkv, kc, vc,
                       att, c.pos, c.q_len, D.q, D.kv, D.d, D.nqkv, D.max_ctx);
    SPD_TRY(hipGetLastError());
    SPD_TRY(gemm(att, qd, (const float *)(w + D.w_o), D.h, nullptr, y_out, D.h, M, D.h, qd, c.s));
    if (c.taps) {
        if (c.taps->q) SPD_TRY(spd_common::copy2d(qkv, D.nqkv, c.taps->q, qd, M, qd, c.s));
        if (c.taps->attn) SPD_TRY(spd_common::copy2d(att, qd, c.taps->attn, qd, M, qd, c.s));
        if (c.taps->y) SPD_TRY(spd_common::copy2d(y_out, D.h, c.taps->y, D.h, M, D.h, c.s));
    }
    return hipSuccess;
}

hipError_t mlp_half(const spd_call &c, const char *w, const float *r_in, const float *add, float *out) {
    const spd_dims &D = *c.D;
    const int M = c.M, f = D.f;
    float *xn = (float *)(c.ws + D.ws_xhat), *gu = (float *)(c.ws + D.ws_gu), *u = (float *)(c.ws + D.ws_uhat);
    hipLaunchKernelGGL(k_rmsnorm, dim3(M), dim3(TB), 0, c.s, r_in, (const float *)(w + D.w_g2), xn, D.h, D.eps);
    SPD_TRY(hipGetLastError());
    SPD_TRY(gemm(xn, D.h, (const float *)(w + D.w_g), f, nullptr, gu, f, M, f, D.h, c.s));
    SPD_TRY(gemm(xn, D.h, (const float *)(w + D.w_u), f, nullptr, gu + (size_t)M * f, f, M, f, D.h, c.s));
    hipLaunchKernelGGL(k_swiglu, dim3(blocks_for((int64_t)M * f)), dim3(TB), 0, c.s, gu, gu + (size_t)M * f, u,
                       (int64_t)M * f);
    SPD_TRY(hipGetLastError());
    SPD_TRY(gemm(u, f, (const float *)(w + D.w_d), D.h, add, out, D.h, M, D.h, f, c.s));
    if (c.taps && c.taps->u) SPD_TRY(spd_common::copy2d(u, f, c.taps->u, f, M, f, c.s));
    return hipSuccess;
}

}  // namespace spd_f32
