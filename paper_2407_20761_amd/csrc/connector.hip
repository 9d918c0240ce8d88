// Row-wise kernels of the hand-over between a ViT stack and an LLM stack on one mixed pipeline
// stage (App. A; the "token sub-sampling" named in Sec. 5.4): the 2 x 2 patch gather fused with
// the LayerNorm that follows it (forward, backward, gain / beta gradients) and the row
// scatter / gather that places the connector's output on the visual rows of the packed LLM
// batch.  All HBM-bound: every byte is read once and written once, 16 bytes per lane.
//
// Tile layout of the ViT output: g*g + 1 rows per tile, class token first, then the patches
// row-major.  Sub-sampled token (r, c) of a tile, r, c < g/2, has 4 Hv channels; channel block
// 2 dr + dc is patch (2 r + dr, 2 c + dc).
#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

namespace {

constexpr int THREADS = 256;
constexpr int MAX_VEC = 8;  // 8-element vectors per thread: 4 Hv <= 256 * 8 * 8 = 16384

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) t += red[w];
    return t;
}

// first ViT row (patch (2r, 2c)) behind sub-sampled token i
__device__ __forceinline__ long first_patch_row(int i, int g) {
    const int half = g >> 1, per_tile = half * half;
    const int t = i / per_tile, rc = i - t * per_tile, r = rc / half, c = rc - r * half;
    return (long)t * (g * g + 1) + 1 + (long)(2 * r) * g + 2 * c;
}

// element offset into v of the 8 channels [8 c8, 8 c8 + 8) of sub-sampled token whose first
// patch row is row0
__device__ __forceinline__ size_t gather_offset(long row0, int c8, int g, int Hv) {
    const int col = c8 * 8, b = col / Hv, off = col - b * Hv;
    return (size_t)(row0 + (b >> 1) * g + (b & 1)) * Hv + off;
}

// un[i] = LayerNorm(gather(v, i)) * gamma + beta;  stats[i] = (mean, rstd)
__global__ __launch_bounds__(THREADS) void subsample_norm_fwd_kernel(
    const __bf16 *__restrict__ v, const __bf16 *__restrict__ gamma, const __bf16 *__restrict__ beta,
    __bf16 *__restrict__ un, float *__restrict__ stats, int g, int Hv, float eps) {
    __shared__ float red[THREADS / 64];
    const int i = blockIdx.x, W = 4 * Hv, nvec = W / 8;
    const long row0 = first_patch_row(i, g);
    float x[MAX_VEC][8];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < MAX_VEC; ++k) {
        const int c8 = threadIdx.x + k * THREADS;
        if (c8 < nvec) {
            const bf16x8 t = *(const bf16x8 *)(v + gather_offset(row0, c8, g, Hv));
#pragma unroll
            for (int e = 0; e < 8; ++e) { x[k][e] = (float)t[e]; s += x[k][e]; }
        }
    }
    const float mean = block_sum(s, red) / W;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < MAX_VEC; ++k) {
        const int c8 = threadIdx.x + k * THREADS;
        if (c8 < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = x[k][e] - mean; q += d * d; }
        }
    }
    const float rstd = rsqrtf(block_sum(q, red) / W + eps);
    if (threadIdx.x == 0) {
        stats[2 * (size_t)i] = mean;
        stats[2 * (size_t)i + 1] = rstd;
    }
#pragma unroll
    for (int k = 0; k < MAX_VEC; ++k) {
        const int c8 = threadIdx.x + k * THREADS;
        if (c8 < nvec) {
            const bf16x8 gm = *(const bf16x8 *)(gamma + c8 * 8), bt = *(const bf16x8 *)(beta + c8 * 8);
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)((x[k][e] - mean) * rstd * (float)gm[e] + (float)bt[e]);
            *(bf16x8 *)(un + (size_t)i * W + c8 * 8) = o;
        }
    }
}

// Blocks [0, n_tok): du = LayerNorm backward of dun at sub-sampled token i, written to the four
// patch rows of dv it was gathered from.  Blocks [n_tok, n_tok + n_tiles): zero the class row
// of a tile (it feeds nothing).  Together they write every element of dv exactly once.
__global__ __launch_bounds__(THREADS) void subsample_norm_bwd_kernel(
    const __bf16 *__restrict__ dun, const __bf16 *__restrict__ v, const float *__restrict__ stats,
    const __bf16 *__restrict__ gamma, __bf16 *__restrict__ dv, int n_tok, int g, int Hv) {
    __shared__ float red[THREADS / 64];
    const int W = 4 * Hv, nvec = W / 8;
    if ((int)blockIdx.x >= n_tok) {
        const size_t row = (size_t)(blockIdx.x - n_tok) * (g * g + 1);
        bf16x8 z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
        for (int c8 = threadIdx.x; c8 < Hv / 8; c8 += THREADS) *(bf16x8 *)(dv + row * Hv + c8 * 8) = z;
        return;
    }
    const int i = blockIdx.x;
    const long row0 = first_patch_row(i, g);
    const float mean = stats[2 * (size_t)i], rstd = stats[2 * (size_t)i + 1];
    float xh[MAX_VEC][8], dxh[MAX_VEC][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int k = 0; k < MAX_VEC; ++k) {
        const int c8 = threadIdx.x + k * THREADS;
        if (c8 < nvec) {
            const bf16x8 t = *(const bf16x8 *)(v + gather_offset(row0, c8, g, Hv));
            const bf16x8 d = *(const bf16x8 *)(dun + (size_t)i * W + c8 * 8);
            const bf16x8 gm = *(const bf16x8 *)(gamma + c8 * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                xh[k][e] = ((float)t[e] - mean) * rstd;
                dxh[k][e] = (float)d[e] * (float)gm[e];
                s1 += dxh[k][e];
                s2 += dxh[k][e] * xh[k][e];
            }
        }
    }
    s1 = block_sum(s1, red) / W;
    s2 = block_sum(s2, red) / W;
#pragma unroll
    for (int k = 0; k < MAX_VEC; ++k) {
        const int c8 = threadIdx.x + k * THREADS;
        if (c8 < nvec) {
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)(rstd * (dxh[k][e] - s1 - xh[k][e] * s2));
            *(bf16x8 *)(dv + gather_offset(row0, c8, g, Hv)) = o;
        }
    }
}

// partial[blockIdx.y][0][c] = sum over tokens blockIdx.y, +gridDim.y, ... of dun * xhat (gain),
// partial[blockIdx.y][1][c] = the same sum of dun (beta); reduce_partials sums over blockIdx.y.
__global__ __launch_bounds__(THREADS) void subsample_norm_wgrad_kernel(
    const __bf16 *__restrict__ dun, const __bf16 *__restrict__ v, const float *__restrict__ stats,
    float *__restrict__ partial, int n_tok, int g, int Hv) {
    const int W = 4 * Hv, c8 = blockIdx.x * THREADS + threadIdx.x;
    if (c8 * 8 >= W) return;
    float dg[8] = {0, 0, 0, 0, 0, 0, 0, 0}, db[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = blockIdx.y; i < n_tok; i += gridDim.y) {
        const float mean = stats[2 * (size_t)i], rstd = stats[2 * (size_t)i + 1];
        const bf16x8 t = *(const bf16x8 *)(v + gather_offset(first_patch_row(i, g), c8, g, Hv));
        const bf16x8 d = *(const bf16x8 *)(dun + (size_t)i * W + c8 * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            dg[e] += (float)d[e] * (((float)t[e] - mean) * rstd);
            db[e] += (float)d[e];
        }
    }
    float *p = partial + (size_t)blockIdx.y * 2 * W + c8 * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) { p[e] = dg[e]; p[W + e] = db[e]; }
}

// SCATTER: big[rows[i]] = small[i];  otherwise small[i] = big[rows[i]].  One workgroup per row.
template <bool SCATTER>
__global__ __launch_bounds__(THREADS) void rows_copy_kernel(__bf16 *__restrict__ small, __bf16 *__restrict__ big,
                                                            const int32_t *__restrict__ rows, int H) {
    const size_t i = blockIdx.x, r = (size_t)rows[i];
    for (int c8 = threadIdx.x; c8 < H / 8; c8 += THREADS) {
        if (SCATTER) *(bf16x8 *)(big + r * H + c8 * 8) = *(const bf16x8 *)(small + i * H + c8 * 8);
        else *(bf16x8 *)(small + i * H + c8 * 8) = *(const bf16x8 *)(big + r * H + c8 * 8);
    }
}

}  // namespace

int subsample_max_width() { return THREADS * 8 * MAX_VEC; }

void launch_subsample_norm_fwd(const void *v, const void *gamma, const void *beta, void *un, float *stats,
                               int n_tok, int g, int Hv, float eps, hipStream_t s) {
    ProfScope prof(K_CONN_FWD, s, 16.0 * n_tok * Hv);   // 4 Hv bf16 in, 4 Hv bf16 out
    hipLaunchKernelGGL(subsample_norm_fwd_kernel, dim3(n_tok), dim3(THREADS), 0, s, (const __bf16 *)v,
                       (const __bf16 *)gamma, (const __bf16 *)beta, (__bf16 *)un, stats, g, Hv, eps);
}

void launch_subsample_norm_bwd(const void *dun, const void *v, const float *stats, const void *gamma, void *dv,
                               int n_tok, int n_tiles, int g, int Hv, hipStream_t s) {
    ProfScope prof(K_CONN_BWD, s, 24.0 * n_tok * Hv);   // dun and v in, dv out
    hipLaunchKernelGGL(subsample_norm_bwd_kernel, dim3(n_tok + n_tiles), dim3(THREADS), 0, s, (const __bf16 *)dun,
                       (const __bf16 *)v, stats, (const __bf16 *)gamma, (__bf16 *)dv, n_tok, g, Hv);
}

int subsample_wgrad_partials(int n_tok) { return n_tok < 64 ? n_tok : 64; }

void launch_subsample_norm_wgrad(const void *dun, const void *v, const float *stats, float *partial, int n_tok,
                                 int g, int Hv, hipStream_t s) {
    ProfScope prof(K_CONN_BWD, s, 16.0 * n_tok * Hv);
    const int W = 4 * Hv;
    hipLaunchKernelGGL(subsample_norm_wgrad_kernel, dim3((W / 8 + THREADS - 1) / THREADS, subsample_wgrad_partials(n_tok)),
                       dim3(THREADS), 0, s, (const __bf16 *)dun, (const __bf16 *)v, stats, partial, n_tok, g, Hv);
}

void launch_rows_scatter(const void *small, void *big, const int32_t *rows_dev, int n_rows, int H, hipStream_t s) {
    ProfScope prof(K_ROWS, s, 4.0 * n_rows * H);
    hipLaunchKernelGGL(rows_copy_kernel<true>, dim3(n_rows), dim3(THREADS), 0, s, (__bf16 *)small, (__bf16 *)big,
                       rows_dev, H);
}

void launch_rows_gather(void *small, const void *big, const int32_t *rows_dev, int n_rows, int H, hipStream_t s) {
    ProfScope prof(K_ROWS, s, 4.0 * n_rows * H);
    hipLaunchKernelGGL(rows_copy_kernel<false>, dim3(n_rows), dim3(THREADS), 0, s, (__bf16 *)small, (__bf16 *)big,
                       rows_dev, H);
}

}  // namespace ob
