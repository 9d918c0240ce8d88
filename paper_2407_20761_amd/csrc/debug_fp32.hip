// fp32 debug path: the same block (steps a1-a9, b9-b1) and the same varlen attention with every
// tensor stored in fp32 and every product accumulated in fp32 FMAs.  It exists to check the
// composition, the masks and the analytic backward against the fp64 oracle at a tolerance (1e-4)
// that bf16 storage cannot reach; it is written for clarity, not speed: no MFMA, no fusion, one
// wavefront per attention row, one thread per element elsewhere.
#include <cmath>

#include "ob_internal.h"

namespace ob {
namespace f32 {
namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// block-wide sum over 256 threads (result in every thread)
__device__ __forceinline__ float block_sum(float v, float *sh /* >= 4 floats */) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}

// C[m][n] = sum_k A(m,k) B(n,k) (+ bias[n]) (+ R[m][n]) (+ C[m][n] when accumulate);
// A(m,k) = A[m sam + k sak], B(n,k) = B[n sbn + k sbk].  16x16 threads, one 64x64 tile, 4x4 each.
__global__ __launch_bounds__(256) void gemm_kernel(int M, int N, int K, const float *__restrict__ A,
                                                   long sam, long sak, const float *__restrict__ B,
                                                   long sbn, long sbk, float *__restrict__ C, int ldc,
                                                   const float *__restrict__ bias,
                                                   const float *__restrict__ R, int ldr, int accumulate) {
    __shared__ float As[16][65], Bs[16][65];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = threadIdx.x; i < 16 * 64; i += 256) {
            const int kk = i & 15, r = i >> 4;
            const int k = k0 + kk;
            As[kk][r] = (m0 + r < M && k < K) ? A[(long)(m0 + r) * sam + (long)k * sak] : 0.f;
            Bs[kk][r] = (n0 + r < N && k < K) ? B[(long)(n0 + r) * sbn + (long)k * sbk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m >= M || n >= N) continue;
            float v = acc[i][j];
            if (bias) v += bias[n];
            if (R) v += R[(size_t)m * ldr + n];
            if (accumulate) v += C[(size_t)m * ldc + n];
            C[(size_t)m * ldc + n] = v;
        }
}

// h = (x - mean) rstd g + b (LayerNorm) or x rstd g (RMSNorm); stat[t] = (mean, rstd)
__global__ __launch_bounds__(256) void norm_fwd_kernel(int layernorm, const float *__restrict__ x,
                                                       const float *__restrict__ g,
                                                       const float *__restrict__ b, float *__restrict__ h,
                                                       float *__restrict__ stat, int H, float eps) {
    __shared__ float sh[4];
    const size_t row = (size_t)blockIdx.x * H;
    float s = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) s += x[row + i];
    const float mean = layernorm ? block_sum(s, sh) / H : 0.f;
    float ss = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) { const float c = x[row + i] - mean; ss += c * c; }
    const float rstd = 1.0f / sqrtf(block_sum(ss, sh) / H + eps);
    for (int i = threadIdx.x; i < H; i += 256) {
        float v = (x[row + i] - mean) * rstd * g[i];
        if (b) v += b[i];
        h[row + i] = v;
    }
    if (threadIdx.x == 0) { stat[2 * blockIdx.x] = mean; stat[2 * blockIdx.x + 1] = rstd; }
}

// dx = res + norm_bwd(dh) (res may be null: no residual); xh = (x - mean) rstd, gy = dh g:
//   LayerNorm dx = rstd (gy - mean(gy) - xh mean(gy xh));  RMSNorm dx = rstd (gy - xh mean(gy xh))
__global__ __launch_bounds__(256) void norm_bwd_kernel(int layernorm, const float *__restrict__ dh,
                                                       const float *__restrict__ x,
                                                       const float *__restrict__ stat,
                                                       const float *__restrict__ g,
                                                       const float *__restrict__ res, float *__restrict__ dx,
                                                       int H) {
    __shared__ float sh[4];
    const size_t row = (size_t)blockIdx.x * H;
    const float mean = stat[2 * blockIdx.x], rstd = stat[2 * blockIdx.x + 1];
    float s1 = 0.f, s2 = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) {
        const float gy = dh[row + i] * g[i], xh = (x[row + i] - mean) * rstd;
        s1 += gy;
        s2 += gy * xh;
    }
    const float m1 = layernorm ? block_sum(s1, sh) / H : 0.f;
    const float m2 = block_sum(s2, sh) / H;
    for (int i = threadIdx.x; i < H; i += 256) {
        const float gy = dh[row + i] * g[i], xh = (x[row + i] - mean) * rstd;
        dx[row + i] = (res ? res[row + i] : 0.f) + rstd * (gy - m1 - xh * m2);
    }
}

// dg[c] (+)= sum_t dh[t][c] xh[t][c];  db[c] (+)= sum_t dh[t][c]; one thread per column
__global__ __launch_bounds__(256) void norm_wgrad_kernel(const float *__restrict__ dh,
                                                         const float *__restrict__ x,
                                                         const float *__restrict__ stat, float *__restrict__ dg,
                                                         float *__restrict__ db, int T, int H, int accumulate) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= H) return;
    float sg = 0.f, sb = 0.f;
    for (int t = 0; t < T; ++t) {
        const float d = dh[(size_t)t * H + c];
        sg += d * (x[(size_t)t * H + c] - stat[2 * t]) * stat[2 * t + 1];
        sb += d;
    }
    dg[c] = accumulate ? dg[c] + sg : sg;
    if (db) db[c] = accumulate ? db[c] + sb : sb;
}

__global__ __launch_bounds__(256) void colsum_kernel(const float *__restrict__ src, int T, int C,
                                                     float *__restrict__ out, int accumulate) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    float s = 0.f;
    for (int t = 0; t < T; ++t) s += src[(size_t)t * C + c];
    out[c] = accumulate ? out[c] + s : s;
}

__device__ __forceinline__ int segment_of(const int32_t *cu, int n_seg, int t) {
    int lo = 0, hi = n_seg;  // cu[lo] <= t < cu[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// rotate pairs (i, i + d/2) of the first `heads` heads of every row by sign * pos * base^(-2i/d)
__global__ __launch_bounds__(256) void rotary_kernel(float *__restrict__ qkv, int ld, int T, int heads, int d,
                                                     const int32_t *__restrict__ cu, int n_seg, float base,
                                                     float sign) {
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int half = d / 2;
    if (gid >= (long)T * heads * half) return;
    const int i = (int)(gid % half);
    const int hd = (int)((gid / half) % heads);
    const int t = (int)(gid / ((long)half * heads));
    const int pos = t - cu[segment_of(cu, n_seg, t)];
    // the angle reaches thousands of radians: form it in double so its error stays below the tolerance
    const double ang = (double)sign * (double)pos * exp2(-2.0 * (double)i / (double)d * log2((double)base));
    const float c = (float)cos(ang), s = (float)sin(ang);
    float *p = qkv + (size_t)t * ld + hd * d;
    const float a = p[i], b = p[i + half];
    p[i] = a * c - b * s;
    p[i + half] = b * c + a * s;
}

__device__ __forceinline__ float gelu(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad(float x) {
    return 0.5f * (1.0f + erff(x * 0.70710678118654752f)) + x * 0.3989422804014327f * expf(-0.5f * x * x);
}

// GELU: act = gelu(up[t][c]);  SwiGLU: act = silu(up[t][c]) up[t][F + c]
__global__ __launch_bounds__(256) void act_fwd_kernel(int swiglu, const float *__restrict__ up,
                                                      float *__restrict__ act, long n, int F) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if (!swiglu) { act[i] = gelu(up[i]); return; }
    const long t = i / F; const int c = (int)(i % F);
    const float g = up[t * 2 * F + c], u = up[t * 2 * F + F + c];
    act[i] = g / (1.0f + expf(-g)) * u;
}

__global__ __launch_bounds__(256) void act_bwd_kernel(int swiglu, const float *__restrict__ dact,
                                                      const float *__restrict__ up, float *__restrict__ dup,
                                                      long n, int F) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if (!swiglu) { dup[i] = dact[i] * gelu_grad(up[i]); return; }
    const long t = i / F; const int c = (int)(i % F);
    const float g = up[t * 2 * F + c], u = up[t * 2 * F + F + c], da = dact[i];
    const float sg = 1.0f / (1.0f + expf(-g));
    dup[t * 2 * F + c] = da * u * sg * (1.0f + g * (1.0f - sg));
    dup[t * 2 * F + F + c] = da * g * sg;
}

// ---- attention: one wavefront per (row, head); lanes split the head dimension ------------------
// forward: online softmax over the allowed keys of the row's segment
__global__ __launch_bounds__(256) void attn_fwd_kernel(const float *__restrict__ q, const float *__restrict__ k,
                                                       const float *__restrict__ v, float *__restrict__ o,
                                                       float *__restrict__ lse, int ldq, int ldkv, int ldo,
                                                       const int32_t *__restrict__ cu, int n_seg, int T, int nq,
                                                       int group, int d, float scale, int causal) {
    const long w = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (w >= (long)T * nq) return;
    const int t = (int)(w / nq), head = (int)(w % nq), kvh = head / group;
    const int sj = segment_of(cu, n_seg, t);
    const int lo = cu[sj], hi = causal ? t + 1 : cu[sj + 1];
    const int per = d / 64;  // 1 or 2 elements per lane
    float qv[2] = {0.f, 0.f}, ov[2] = {0.f, 0.f};
    for (int e = 0; e < per; ++e) qv[e] = q[(size_t)t * ldq + head * d + lane + 64 * e];
    float m = -INFINITY, l = 0.f;
    for (int j = lo; j < hi; ++j) {
        float part = 0.f;
        for (int e = 0; e < per; ++e) part += qv[e] * k[(size_t)j * ldkv + kvh * d + lane + 64 * e];
        const float s = wave_sum(part) * scale;
        const float mn = fmaxf(m, s);
        const float alpha = expf(m - mn), p = expf(s - mn);
        l = l * alpha + p;
        for (int e = 0; e < per; ++e) ov[e] = ov[e] * alpha + p * v[(size_t)j * ldkv + kvh * d + lane + 64 * e];
        m = mn;
    }
    for (int e = 0; e < per; ++e) o[(size_t)t * ldo + head * d + lane + 64 * e] = ov[e] / l;
    if (lane == 0) lse[(size_t)head * T + t] = m + logf(l);
}

// delta[head][t] = sum_d dO O
__global__ __launch_bounds__(256) void attn_delta_kernel(const float *__restrict__ d_o, const float *__restrict__ o,
                                                         int ldo, float *__restrict__ delta, int T, int nq, int d) {
    const long w = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (w >= (long)T * nq) return;
    const int t = (int)(w / nq), head = (int)(w % nq);
    float part = 0.f;
    for (int e = 0; e < d / 64; ++e) {
        const size_t off = (size_t)t * ldo + head * d + lane + 64 * e;
        part += d_o[off] * o[off];
    }
    part = wave_sum(part);
    if (lane == 0) delta[(size_t)head * T + t] = part;
}

// dq[t, head] = scale sum_j P_tj (dP_tj - delta_t) k_j
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const float *__restrict__ d_o, const float *__restrict__ q,
                                                          const float *__restrict__ k, const float *__restrict__ v,
                                                          const float *__restrict__ lse, const float *__restrict__ delta,
                                                          float *__restrict__ dq, int ldq, int ldkv, int ldo,
                                                          const int32_t *__restrict__ cu, int n_seg, int T, int nq,
                                                          int group, int d, float scale, int causal) {
    const long w = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (w >= (long)T * nq) return;
    const int t = (int)(w / nq), head = (int)(w % nq), kvh = head / group;
    const int sj = segment_of(cu, n_seg, t);
    const int lo = cu[sj], hi = causal ? t + 1 : cu[sj + 1];
    const int per = d / 64;
    float qv[2] = {0.f, 0.f}, dov[2] = {0.f, 0.f}, acc[2] = {0.f, 0.f};
    for (int e = 0; e < per; ++e) {
        qv[e] = q[(size_t)t * ldq + head * d + lane + 64 * e];
        dov[e] = d_o[(size_t)t * ldo + head * d + lane + 64 * e];
    }
    const float ls = lse[(size_t)head * T + t], dl = delta[(size_t)head * T + t];
    for (int j = lo; j < hi; ++j) {
        float ps = 0.f, pd = 0.f;
        for (int e = 0; e < per; ++e) {
            const size_t off = (size_t)j * ldkv + kvh * d + lane + 64 * e;
            ps += qv[e] * k[off];
            pd += dov[e] * v[off];
        }
        const float p = expf(wave_sum(ps) * scale - ls);
        const float ds = p * (wave_sum(pd) - dl);
        for (int e = 0; e < per; ++e) acc[e] += ds * k[(size_t)j * ldkv + kvh * d + lane + 64 * e];
    }
    for (int e = 0; e < per; ++e) dq[(size_t)t * ldq + head * d + lane + 64 * e] = acc[e] * scale;
}

// dk[j, kvh] = scale sum_{heads of the group} sum_t dS_tj q_t;  dv[j, kvh] = sum sum P_tj dO_t
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const float *__restrict__ d_o, const float *__restrict__ q,
                                                           const float *__restrict__ k, const float *__restrict__ v,
                                                           const float *__restrict__ lse, const float *__restrict__ delta,
                                                           float *__restrict__ dk, float *__restrict__ dv, int ldq,
                                                           int ldkv, int ldo, const int32_t *__restrict__ cu, int n_seg,
                                                           int T, int nkv, int group, int d, float scale, int causal) {
    const long w = ((long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (w >= (long)T * nkv) return;
    const int j = (int)(w / nkv), kvh = (int)(w % nkv);
    const int sj = segment_of(cu, n_seg, j);
    const int lo = causal ? j : cu[sj], hi = cu[sj + 1];
    const int per = d / 64;
    float kv_[2] = {0.f, 0.f}, vv[2] = {0.f, 0.f}, ak[2] = {0.f, 0.f}, av[2] = {0.f, 0.f};
    for (int e = 0; e < per; ++e) {
        kv_[e] = k[(size_t)j * ldkv + kvh * d + lane + 64 * e];
        vv[e] = v[(size_t)j * ldkv + kvh * d + lane + 64 * e];
    }
    for (int head = kvh * group; head < (kvh + 1) * group; ++head)
        for (int t = lo; t < hi; ++t) {
            float ps = 0.f, pd = 0.f, qe[2] = {0.f, 0.f}, de[2] = {0.f, 0.f};
            for (int e = 0; e < per; ++e) {
                qe[e] = q[(size_t)t * ldq + head * d + lane + 64 * e];
                de[e] = d_o[(size_t)t * ldo + head * d + lane + 64 * e];
                ps += qe[e] * kv_[e];
                pd += de[e] * vv[e];
            }
            const float p = expf(wave_sum(ps) * scale - lse[(size_t)head * T + t]);
            const float ds = p * (wave_sum(pd) - delta[(size_t)head * T + t]);
            for (int e = 0; e < per; ++e) { av[e] += p * de[e]; ak[e] += ds * qe[e]; }
        }
    for (int e = 0; e < per; ++e) {
        dk[(size_t)j * ldkv + kvh * d + lane + 64 * e] = ak[e] * scale;
        dv[(size_t)j * ldkv + kvh * d + lane + 64 * e] = av[e];
    }
}

// ---- ViT -> LLM hand-over: patch gather / its adjoint, row scatter / gather ----------------------

// u[i][b Hv + c] = v[row(i, b)][c]: token i = (tile, r, cq) of the (g/2)^2 grid, block b = 2 dr + dc
// takes patch (2r + dr, 2cq + dc); row 0 of every tile (the class token) is skipped
__global__ __launch_bounds__(256) void subsample_gather_kernel(const float *__restrict__ v, float *__restrict__ u,
                                                               long n, int g, int Hv) {
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const int W = 4 * Hv, half = g / 2;
    const long i = e / W;
    const int col = (int)(e % W), b = col / Hv, c = col % Hv;
    const int tile = (int)(i / (half * half)), rem = (int)(i % (half * half)), r = rem / half, cq = rem % half;
    const long row = (long)tile * (g * g + 1) + 1 + (long)(2 * r + (b >> 1)) * g + (2 * cq + (b & 1));
    u[e] = v[row * Hv + c];
}

// the adjoint: every patch row receives its channel block of du, class rows become zero
__global__ __launch_bounds__(256) void subsample_scatter_kernel(const float *__restrict__ du, float *__restrict__ dv,
                                                                long n, int g, int Hv) {
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const int half = g / 2, per_tile = g * g + 1;
    const long row = e / Hv;
    const int c = (int)(e % Hv), tile = (int)(row / per_tile), p = (int)(row % per_tile);
    if (p == 0) { dv[e] = 0.f; return; }
    const int pr = (p - 1) / g, pc = (p - 1) % g;
    const long i = ((long)tile * half + pr / 2) * half + pc / 2;
    const int b = 2 * (pr & 1) + (pc & 1);
    dv[e] = du[i * 4 * Hv + b * Hv + c];
}

// SCATTER: big[rows[i]][:] = small[i][:];  else small[i][:] = big[rows[i]][:]
__global__ __launch_bounds__(256) void rows_copy_kernel(float *__restrict__ small, float *__restrict__ big,
                                                        const int32_t *__restrict__ rows, long n, int C, int scatter) {
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const long i = e / C;
    const int c = (int)(e % C);
    if (scatter) big[(long)rows[i] * C + c] = small[e];
    else small[e] = big[(long)rows[i] * C + c];
}

inline unsigned blocks_for(long threads) { return (unsigned)((threads + 255) / 256); }

void gemm(int layout, int M, int N, int K, const float *A, const float *B, float *C, const float *bias,
          const float *R, int accumulate, hipStream_t s) {
    // layout 0 "NT" A[M,K] B[N,K]; 1 "NN" A[M,K] B[K,N]; 2 "TN" A[K,M] B[K,N]
    const long sam = layout == 2 ? 1 : K, sak = layout == 2 ? M : 1;
    const long sbn = layout == 0 ? K : 1, sbk = layout == 0 ? 1 : N;
    hipLaunchKernelGGL(gemm_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, s, M, N, K, A, sam, sak, B,
                       sbn, sbk, C, N, bias, R, N, accumulate);
}

}  // namespace

void attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int ldq, int ldkv, int ldo,
              const ob_segments *seg, int nq, int nkv, int d, float scale, int mask, hipStream_t s) {
    const int T = seg->total_tokens;
    hipLaunchKernelGGL(attn_fwd_kernel, dim3(blocks_for((long)T * nq * 64)), dim3(256), 0, s, (const float *)q,
                       (const float *)k, (const float *)v, (float *)o, lse, ldq, ldkv, ldo, seg->cu_dev, seg->n_seg, T,
                       nq, nq / nkv, d, scale, mask == OB_MASK_SEG_CAUSAL ? 1 : 0);
}

void attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const void *o, const float *lse,
              void *dq, void *dk, void *dv, float *delta, int ldq, int ldkv, int ldo, const ob_segments *seg, int nq,
              int nkv, int d, float scale, int mask, hipStream_t s) {
    const int T = seg->total_tokens, causal = mask == OB_MASK_SEG_CAUSAL ? 1 : 0;
    hipLaunchKernelGGL(attn_delta_kernel, dim3(blocks_for((long)T * nq * 64)), dim3(256), 0, s, (const float *)d_o,
                       (const float *)o, ldo, delta, T, nq, d);
    hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(blocks_for((long)T * nq * 64)), dim3(256), 0, s, (const float *)d_o,
                       (const float *)q, (const float *)k, (const float *)v, lse, delta, (float *)dq, ldq, ldkv, ldo,
                       seg->cu_dev, seg->n_seg, T, nq, nq / nkv, d, scale, causal);
    hipLaunchKernelGGL(attn_bwd_dkv_kernel, dim3(blocks_for((long)T * nkv * 64)), dim3(256), 0, s, (const float *)d_o,
                       (const float *)q, (const float *)k, (const float *)v, lse, delta, (float *)dk, (float *)dv, ldq,
                       ldkv, ldo, seg->cu_dev, seg->n_seg, T, nkv, nq / nkv, d, scale, causal);
}

// Buffers of the fp32 block: the same members as the bf16 path, four bytes per element.
static size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }
SavedF32 saved_layout(const ob_block_desc *dsc, int T_) {
    const size_t T = T_, H = dsc->hidden, d = dsc->head_dim, nq = dsc->n_q_heads, nkv = dsc->n_kv_heads;
    const size_t F = dsc->mlp_dim, upF = dsc->mlp == OB_SWIGLU ? 2 * F : F, Dq = (nq + 2 * nkv) * d;
    SavedF32 s; size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    s.h1 = take(T * H * 4); s.qkv = take(T * Dq * 4); s.o = take(T * nq * d * 4); s.lse = take(nq * T * 4);
    s.x1 = take(T * H * 4); s.h2 = take(T * H * 4); s.up = take(T * upF * 4); s.act = take(T * F * 4);
    s.stat1 = take(T * 8); s.stat2 = take(T * 8);
    s.total = off;
    return s;
}
WorkF32 work_layout(const ob_block_desc *dsc, int T_) {
    const size_t T = T_, H = dsc->hidden, d = dsc->head_dim, nq = dsc->n_q_heads, nkv = dsc->n_kv_heads;
    const size_t F = dsc->mlp_dim, upF = dsc->mlp == OB_SWIGLU ? 2 * F : F, Dq = (nq + 2 * nkv) * d;
    WorkF32 w; size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    w.dact = take(T * F * 4); w.dup = take(T * upF * 4); w.dh = take(T * H * 4); w.dx1 = take(T * H * 4);
    w.d_o = take(T * nq * d * 4); w.dqkv = take(T * Dq * 4); w.delta = take(nq * T * 4);
    w.total = off;
    return w;
}

#define OB_F(p) ((const float *)(p))
#define OB_FM(p) ((float *)(p))

void block_fwd(const ob_block_desc *dsc, const ob_block_weights *w, const void *x, void *y, void *saved,
               const ob_segments *seg, hipStream_t s) {
    const int T = seg->total_tokens, H = dsc->hidden, d = dsc->head_dim, nq = dsc->n_q_heads, nkv = dsc->n_kv_heads;
    const int F = dsc->mlp_dim, upF = dsc->mlp == OB_SWIGLU ? 2 * F : F, Dq = (nq + 2 * nkv) * d, HD = nq * d;
    const SavedF32 sv = saved_layout(dsc, T);
    unsigned char *b = (unsigned char *)saved;
    float *h1 = OB_FM(b + sv.h1), *qkv = OB_FM(b + sv.qkv), *o = OB_FM(b + sv.o), *lse = OB_FM(b + sv.lse);
    float *x1 = OB_FM(b + sv.x1), *h2 = OB_FM(b + sv.h2), *up = OB_FM(b + sv.up), *act = OB_FM(b + sv.act);
    const bool bias = dsc->has_bias != 0, ln = dsc->norm == OB_LAYERNORM, beta = bias && ln;
    const float scale = 1.0f / sqrtf((float)d);
    hipLaunchKernelGGL(norm_fwd_kernel, dim3(T), dim3(256), 0, s, ln ? 1 : 0, OB_F(x), OB_F(w->n1_g),
                       beta ? OB_F(w->n1_b) : nullptr, h1, OB_FM(b + sv.stat1), H, dsc->norm_eps);
    gemm(0, T, Dq, H, h1, OB_F(w->w_qkv), qkv, bias ? OB_F(w->b_qkv) : nullptr, nullptr, 0, s);
    if (dsc->use_rotary)
        hipLaunchKernelGGL(rotary_kernel, dim3(blocks_for((long)T * (nq + nkv) * (d / 2))), dim3(256), 0, s, qkv, Dq, T,
                           nq + nkv, d, seg->cu_dev, seg->n_seg, dsc->rotary_base, 1.0f);
    attn_fwd(qkv, qkv + HD, qkv + HD + nkv * d, o, lse, Dq, Dq, HD, seg, nq, nkv, d, scale, dsc->mask, s);
    gemm(0, T, H, HD, o, OB_F(w->w_o), x1, bias ? OB_F(w->b_o) : nullptr, OB_F(x), 0, s);
    hipLaunchKernelGGL(norm_fwd_kernel, dim3(T), dim3(256), 0, s, ln ? 1 : 0, x1, OB_F(w->n2_g),
                       beta ? OB_F(w->n2_b) : nullptr, h2, OB_FM(b + sv.stat2), H, dsc->norm_eps);
    gemm(0, T, upF, H, h2, OB_F(w->w_up), up, bias ? OB_F(w->b_up) : nullptr, nullptr, 0, s);
    hipLaunchKernelGGL(act_fwd_kernel, dim3(blocks_for((long)T * F)), dim3(256), 0, s, dsc->mlp == OB_SWIGLU ? 1 : 0, up,
                       act, (long)T * F, F);
    if (y) gemm(0, T, H, F, act, OB_F(w->w_down), OB_FM(y), bias ? OB_F(w->b_down) : nullptr, x1, 0, s);
}

void block_bwd(const ob_block_desc *dsc, const ob_block_weights *w, const ob_block_grads *g, int acc, const void *x,
               const void *dy, void *dx, const void *saved, const ob_segments *seg, void *ws, hipStream_t s) {
    const int T = seg->total_tokens, H = dsc->hidden, d = dsc->head_dim, nq = dsc->n_q_heads, nkv = dsc->n_kv_heads;
    const int F = dsc->mlp_dim, upF = dsc->mlp == OB_SWIGLU ? 2 * F : F, Dq = (nq + 2 * nkv) * d, HD = nq * d;
    const SavedF32 sv = saved_layout(dsc, T);
    const WorkF32 wk = work_layout(dsc, T);
    const unsigned char *b = (const unsigned char *)saved;
    unsigned char *wb = (unsigned char *)ws;
    const float *h1 = OB_F(b + sv.h1), *qkv = OB_F(b + sv.qkv), *o = OB_F(b + sv.o), *lse = OB_F(b + sv.lse);
    const float *x1 = OB_F(b + sv.x1), *h2 = OB_F(b + sv.h2), *up = OB_F(b + sv.up), *act = OB_F(b + sv.act);
    float *dact = OB_FM(wb + wk.dact), *dup = OB_FM(wb + wk.dup), *dh = OB_FM(wb + wk.dh), *dx1 = OB_FM(wb + wk.dx1);
    float *d_o = OB_FM(wb + wk.d_o), *dqkv = OB_FM(wb + wk.dqkv), *delta = OB_FM(wb + wk.delta);
    const bool bias = dsc->has_bias != 0, ln = dsc->norm == OB_LAYERNORM, beta = bias && ln;
    const float scale = 1.0f / sqrtf((float)d);
    auto colsum = [&](const float *src, int C, void *out) {
        hipLaunchKernelGGL(colsum_kernel, dim3(blocks_for(C)), dim3(256), 0, s, src, T, C, OB_FM(out), acc);
    };
    // y = x1 + act W_down^T + b_down
    gemm(1, T, F, H, OB_F(dy), OB_F(w->w_down), dact, nullptr, nullptr, 0, s);
    gemm(2, H, F, T, OB_F(dy), act, OB_FM(g->w_down), nullptr, nullptr, acc, s);
    if (bias) colsum(OB_F(dy), H, g->b_down);
    hipLaunchKernelGGL(act_bwd_kernel, dim3(blocks_for((long)T * F)), dim3(256), 0, s, dsc->mlp == OB_SWIGLU ? 1 : 0,
                       dact, up, dup, (long)T * F, F);
    gemm(2, upF, H, T, dup, h2, OB_FM(g->w_up), nullptr, nullptr, acc, s);
    if (bias) colsum(dup, upF, g->b_up);
    gemm(1, T, H, upF, dup, OB_F(w->w_up), dh, nullptr, nullptr, 0, s);
    // dx1 = dy + norm2_bwd(dh2)
    hipLaunchKernelGGL(norm_bwd_kernel, dim3(T), dim3(256), 0, s, ln ? 1 : 0, dh, x1, OB_F(b + sv.stat2), OB_F(w->n2_g),
                       OB_F(dy), dx1, H);
    hipLaunchKernelGGL(norm_wgrad_kernel, dim3(blocks_for(H)), dim3(256), 0, s, dh, x1, OB_F(b + sv.stat2),
                       OB_FM(g->n2_g), beta ? OB_FM(g->n2_b) : nullptr, T, H, acc);
    // x1 = x + o W_o^T + b_o
    gemm(2, H, HD, T, dx1, o, OB_FM(g->w_o), nullptr, nullptr, acc, s);
    if (bias) colsum(dx1, H, g->b_o);
    gemm(1, T, HD, H, dx1, OB_F(w->w_o), d_o, nullptr, nullptr, 0, s);
    attn_bwd(d_o, qkv, qkv + HD, qkv + HD + nkv * d, o, lse, dqkv, dqkv + HD, dqkv + HD + nkv * d, delta, Dq, Dq, HD,
             seg, nq, nkv, d, scale, dsc->mask, s);
    if (dsc->use_rotary)
        hipLaunchKernelGGL(rotary_kernel, dim3(blocks_for((long)T * (nq + nkv) * (d / 2))), dim3(256), 0, s, dqkv, Dq, T,
                           nq + nkv, d, seg->cu_dev, seg->n_seg, dsc->rotary_base, -1.0f);
    // qkv = h1 W_qkv^T + b_qkv
    gemm(2, Dq, H, T, dqkv, h1, OB_FM(g->w_qkv), nullptr, nullptr, acc, s);
    if (bias) colsum(dqkv, Dq, g->b_qkv);
    gemm(1, T, H, Dq, dqkv, OB_F(w->w_qkv), dh, nullptr, nullptr, 0, s);
    // dx = dx1 + norm1_bwd(dh1)
    hipLaunchKernelGGL(norm_bwd_kernel, dim3(T), dim3(256), 0, s, ln ? 1 : 0, dh, OB_F(x), OB_F(b + sv.stat1),
                       OB_F(w->n1_g), dx1, OB_FM(dx), H);
    hipLaunchKernelGGL(norm_wgrad_kernel, dim3(blocks_for(H)), dim3(256), 0, s, dh, OB_F(x), OB_F(b + sv.stat1),
                       OB_FM(g->n1_g), beta ? OB_FM(g->n1_b) : nullptr, T, H, acc);
}


// ---- hand-over, fp32: the same steps as the bf16 path, every tensor in fp32, u kept in `saved` ----
struct ConnSaved { size_t u, un, h, a, stats, total; };
struct ConnWork { size_t z, da, dh, dun, du, total; };
static ConnSaved conn_saved(long n, int W, int Ht) {
    ConnSaved s; size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    s.u = take(n * W * 4); s.un = take(n * W * 4); s.h = take(n * Ht * 4); s.a = take(n * Ht * 4); s.stats = take(n * 8);
    s.total = off;
    return s;
}
static ConnWork conn_work(long n, int W, int Ht) {
    ConnWork w; size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    w.z = take(n * Ht * 4); w.da = take(n * Ht * 4); w.dh = take(n * Ht * 4); w.dun = take(n * W * 4); w.du = take(n * W * 4);
    w.total = off;
    return w;
}
size_t connector_saved_bytes(long n_tok, int Hv, int Ht) { return conn_saved(n_tok, 4 * Hv, Ht).total; }
size_t connector_work_bytes(long n_tok, int Hv, int Ht) { return conn_work(n_tok, 4 * Hv, Ht).total; }

void connector_fwd(const ob_connector_weights *w, const void *v, int n_tok, int g, int Hv, int Ht, float eps,
                   const int32_t *rows_dev, void *x_llm, void *saved, void *ws, hipStream_t s) {
    const int W = 4 * Hv;
    const ConnSaved sv = conn_saved(n_tok, W, Ht);
    const ConnWork wk = conn_work(n_tok, W, Ht);
    unsigned char *b = (unsigned char *)saved;
    float *u = OB_FM(b + sv.u), *un = OB_FM(b + sv.un), *h = OB_FM(b + sv.h), *a = OB_FM(b + sv.a);
    float *z = OB_FM((unsigned char *)ws + wk.z);
    hipLaunchKernelGGL(subsample_gather_kernel, dim3(blocks_for((long)n_tok * W)), dim3(256), 0, s, OB_F(v), u,
                       (long)n_tok * W, g, Hv);
    hipLaunchKernelGGL(norm_fwd_kernel, dim3(n_tok), dim3(256), 0, s, 1, u, OB_F(w->n_g), OB_F(w->n_b), un,
                       OB_FM(b + sv.stats), W, eps);
    gemm(0, n_tok, Ht, W, un, OB_F(w->w1), h, OB_F(w->b1), nullptr, 0, s);
    hipLaunchKernelGGL(act_fwd_kernel, dim3(blocks_for((long)n_tok * Ht)), dim3(256), 0, s, 0, h, a, (long)n_tok * Ht, Ht);
    gemm(0, n_tok, Ht, Ht, a, OB_F(w->w2), z, OB_F(w->b2), nullptr, 0, s);
    hipLaunchKernelGGL(rows_copy_kernel, dim3(blocks_for((long)n_tok * Ht)), dim3(256), 0, s, z, OB_FM(x_llm), rows_dev,
                       (long)n_tok * Ht, Ht, 1);
}

void connector_bwd(const ob_connector_weights *w, const ob_connector_grads *gr, int acc, const void *dx_llm, void *dv,
                   int n_tok, int n_tiles, int g, int Hv, int Ht, const int32_t *rows_dev, const void *saved, void *ws,
                   hipStream_t s) {
    const int W = 4 * Hv;
    const ConnSaved sv = conn_saved(n_tok, W, Ht);
    const ConnWork wk = conn_work(n_tok, W, Ht);
    const unsigned char *b = (const unsigned char *)saved;
    unsigned char *wb = (unsigned char *)ws;
    const float *u = OB_F(b + sv.u), *un = OB_F(b + sv.un), *h = OB_F(b + sv.h), *a = OB_F(b + sv.a);
    const float *stats = OB_F(b + sv.stats);
    float *dz = OB_FM(wb + wk.z), *da = OB_FM(wb + wk.da), *dh = OB_FM(wb + wk.dh), *dun = OB_FM(wb + wk.dun);
    float *du = OB_FM(wb + wk.du);
    auto colsum = [&](const float *src, int C, void *out) {
        hipLaunchKernelGGL(colsum_kernel, dim3(blocks_for(C)), dim3(256), 0, s, src, n_tok, C, OB_FM(out), acc);
    };
    hipLaunchKernelGGL(rows_copy_kernel, dim3(blocks_for((long)n_tok * Ht)), dim3(256), 0, s, dz,
                       (float *)dx_llm /* read only */, rows_dev, (long)n_tok * Ht, Ht, 0);
    gemm(2, Ht, Ht, n_tok, dz, a, OB_FM(gr->w2), nullptr, nullptr, acc, s);
    colsum(dz, Ht, gr->b2);
    gemm(1, n_tok, Ht, Ht, dz, OB_F(w->w2), da, nullptr, nullptr, 0, s);
    hipLaunchKernelGGL(act_bwd_kernel, dim3(blocks_for((long)n_tok * Ht)), dim3(256), 0, s, 0, da, h, dh,
                       (long)n_tok * Ht, Ht);
    gemm(2, Ht, W, n_tok, dh, un, OB_FM(gr->w1), nullptr, nullptr, acc, s);
    colsum(dh, Ht, gr->b1);
    gemm(1, n_tok, W, Ht, dh, OB_F(w->w1), dun, nullptr, nullptr, 0, s);
    // un = LayerNorm(u): du = norm_bwd(dun), no residual
    hipLaunchKernelGGL(norm_bwd_kernel, dim3(n_tok), dim3(256), 0, s, 1, dun, u, stats, OB_F(w->n_g),
                       (const float *)nullptr, du, W);
    hipLaunchKernelGGL(norm_wgrad_kernel, dim3(blocks_for(W)), dim3(256), 0, s, dun, u, stats, OB_FM(gr->n_g),
                       OB_FM(gr->n_b), n_tok, W, acc);
    const long n_dv = (long)n_tiles * (g * g + 1) * Hv;
    hipLaunchKernelGGL(subsample_scatter_kernel, dim3(blocks_for(n_dv)), dim3(256), 0, s, du, OB_FM(dv), n_dv, g, Hv);
}

}  // namespace f32
}  // namespace ob
