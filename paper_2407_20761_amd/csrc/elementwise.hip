// HBM-bound row-wise and elementwise kernels of the block (steps a1, a3, a6, a8 and their
// backward counterparts b1, b3, b6, b8, bias-gradient column sums).
// bf16 in / out, fp32 arithmetic, 16-byte loads and stores; one workgroup per token row for the
// row-wise ones so every byte is read once and written once.
#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

constexpr int NORM_THREADS = 256;
constexpr int MAX_VEC = 4;  // 8-element vectors per thread: H <= 256 * 8 * 4 = 8192

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// sum over the workgroup; every thread gets the result.  `red` holds one float per wave.
__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < nw; ++w) t += red[w];
    return t;
}

template <bool LAYERNORM>
__global__ __launch_bounds__(NORM_THREADS) void norm_fwd_kernel(
    const __bf16 *__restrict__ x, const __bf16 *__restrict__ gamma, const __bf16 *__restrict__ beta,
    __bf16 *__restrict__ h, float *__restrict__ stats, int T, int H, float eps) {
    __shared__ float red[NORM_THREADS / 64];
    const int row = blockIdx.x;
    const int nvec = H / 8;
    const __bf16 *xr = x + (size_t)row * H;
    float v[MAX_VEC][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAX_VEC; ++i) {
        const int c = threadIdx.x + i * NORM_THREADS;
        if (c < nvec) {
            const bf16x8 t = *(const bf16x8 *)(xr + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[i][e] = (float)t[e];
                s += LAYERNORM ? v[i][e] : v[i][e] * v[i][e];
            }
        }
    }
    s = block_sum(s, red);
    float mean = 0.f, rstd;
    if (LAYERNORM) {
        mean = s / H;
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < MAX_VEC; ++i) {
            const int c = threadIdx.x + i * NORM_THREADS;
            if (c < nvec) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float dlt = v[i][e] - mean;
                    q += dlt * dlt;
                }
            }
        }
        q = block_sum(q, red);
        rstd = rsqrtf(q / H + eps);
    } else {
        rstd = rsqrtf(s / H + eps);
    }
    if (threadIdx.x == 0) {
        stats[2 * (size_t)row] = mean;
        stats[2 * (size_t)row + 1] = rstd;
    }
#pragma unroll
    for (int i = 0; i < MAX_VEC; ++i) {
        const int c = threadIdx.x + i * NORM_THREADS;
        if (c < nvec) {
            const bf16x8 g = *(const bf16x8 *)(gamma + c * 8);
            bf16x8 o;
            if (LAYERNORM && beta) {
                const bf16x8 b = *(const bf16x8 *)(beta + c * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    o[e] = (__bf16)((v[i][e] - mean) * rstd * (float)g[e] + (float)b[e]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (__bf16)((v[i][e] - mean) * rstd * (float)g[e]);
            }
            *(bf16x8 *)(h + (size_t)row * H + c * 8) = o;
        }
    }
}

// The same forward for narrow rows (H <= 2048): a workgroup per row would leave most lanes idle and
// pay two workgroup barriers per row, so a wavefront owns a row (NV vectors of 8 per lane, row sums
// by wave reduction), walks rows slot, slot + n_slots, ... with the next row's loads in flight, and
// keeps gamma and beta in registers.
template <bool LAYERNORM, int NV>
__global__ __launch_bounds__(256) void norm_fwd_wave_kernel(
    const __bf16 *__restrict__ x, const __bf16 *__restrict__ gamma, const __bf16 *__restrict__ beta,
    __bf16 *__restrict__ h, float *__restrict__ stats, int T, int H, float eps) {
    const int nvec = H / 8, lane = threadIdx.x & 63;
    const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), n_slots = gridDim.x * 4;
    bf16x8 g[NV], b[NV], nx[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        g[i] = c < nvec ? *(const bf16x8 *)(gamma + c * 8) : bf16x8{};
        b[i] = LAYERNORM && beta && c < nvec ? *(const bf16x8 *)(beta + c * 8) : bf16x8{};
        nx[i] = bf16x8{};
    }
    auto fetch = [&](int row) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (lane + 64 * i < nvec) nx[i] = *(const bf16x8 *)(x + (size_t)row * H + (lane + 64 * i) * 8);
    };
    if (slot < T) fetch(slot);
    for (int row = slot; row < T; row += n_slots) {
        float v[NV][8];
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i)      // lanes past the end of the row hold zeros
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[i][e] = (float)nx[i][e];
                sum += LAYERNORM ? v[i][e] : v[i][e] * v[i][e];
            }
        if (row + n_slots < T) fetch(row + n_slots);
        sum = wave_sum(sum);
        float mean = 0.f, rstd;
        if (LAYERNORM) {
            mean = sum / H;
            float q = 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i)
                if (lane + 64 * i < nvec)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float dlt = v[i][e] - mean;
                        q += dlt * dlt;
                    }
            rstd = rsqrtf(wave_sum(q) / H + eps);
        } else {
            rstd = rsqrtf(sum / H + eps);
        }
        if (lane == 0) {
            stats[2 * (size_t)row] = mean;
            stats[2 * (size_t)row + 1] = rstd;
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nvec) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (__bf16)((v[i][e] - mean) * rstd * (float)g[i][e] + (float)b[i][e]);
                *(bf16x8 *)(h + (size_t)row * H + c * 8) = o;
            }
        }
    }
}

// dx = dres + rstd * (dxhat - mean(dxhat) [LayerNorm only] - xhat * mean(dxhat * xhat)),
// dxhat = dh * gamma.  Each workgroup walks rows blockIdx.x, +gridDim.x, ... and keeps its
// column sums of dh * xhat (dgamma) and dh (dbeta) in registers; they are written once to
// partial[blockIdx.x][2][H] and summed by reduce_partials_kernel.
// CSUM: the kernel also leaves the column sums of dres and of its output dx (as stored, after rounding) in
// csum[blockIdx.x][2][H]: the bias gradients of the two linears around the norm, which would otherwise
// each take a pass of their own over a [T, H] tensor the kernel has in registers anyway.
template <bool LAYERNORM, bool CSUM>
__global__ __launch_bounds__(NORM_THREADS) void norm_bwd_kernel(
    const __bf16 *__restrict__ dh, const __bf16 *__restrict__ x, const float *__restrict__ stats,
    const __bf16 *__restrict__ gamma, const __bf16 *__restrict__ dres, __bf16 *__restrict__ dx,
    float *__restrict__ partial, float *__restrict__ csum, int T, int H) {
    __shared__ float red[NORM_THREADS / 64];
    const int nvec = H / 8;
    float g[MAX_VEC][8], dg[MAX_VEC][8], db[MAX_VEC][8];
    float sr[CSUM ? MAX_VEC : 1][8], sx[CSUM ? MAX_VEC : 1][8];
#pragma unroll
    for (int i = 0; i < (CSUM ? MAX_VEC : 1); ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) sr[i][e] = sx[i][e] = 0.f;
#pragma unroll
    for (int i = 0; i < MAX_VEC; ++i) {
        const int c = threadIdx.x + i * NORM_THREADS;
#pragma unroll
        for (int e = 0; e < 8; ++e) dg[i][e] = db[i][e] = g[i][e] = 0.f;
        if (c < nvec) {
            const bf16x8 t = *(const bf16x8 *)(gamma + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) g[i][e] = (float)t[e];
        }
    }
    // the loads of a row are issued one row ahead (x, dh) or in front of the row's two reductions
    // (dres), so that the barriers of the reductions never leave the memory pipe empty
    bf16x8 nx[MAX_VEC], nd[MAX_VEC];
    float nmean = 0.f, nrstd = 0.f;
    auto fetch = [&](int row) {
        nmean = stats[2 * (size_t)row];
        nrstd = stats[2 * (size_t)row + 1];
#pragma unroll
        for (int i = 0; i < MAX_VEC; ++i) {
            const int c = threadIdx.x + i * NORM_THREADS;
            if (c < nvec) {
                nx[i] = *(const bf16x8 *)(x + (size_t)row * H + c * 8);
                nd[i] = *(const bf16x8 *)(dh + (size_t)row * H + c * 8);
            }
        }
    };
    if ((int)blockIdx.x < T) fetch(blockIdx.x);
    for (int row = blockIdx.x; row < T; row += gridDim.x) {
        const float mean = nmean, rstd = nrstd;
        float xh[MAX_VEC][8], dxh[MAX_VEC][8];
        bf16x8 tr[MAX_VEC];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < MAX_VEC; ++i) {
            const int c = threadIdx.x + i * NORM_THREADS;
            if (c < nvec) {
                const bf16x8 tx = nx[i], td = nd[i];
                tr[i] = *(const bf16x8 *)(dres + (size_t)row * H + c * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = (float)td[e];
                    xh[i][e] = ((float)tx[e] - mean) * rstd;
                    dxh[i][e] = d * g[i][e];
                    dg[i][e] += d * xh[i][e];
                    db[i][e] += d;
                    s1 += dxh[i][e];
                    s2 += dxh[i][e] * xh[i][e];
                }
            }
        }
        if (row + (int)gridDim.x < T) fetch(row + gridDim.x);
        s2 = block_sum(s2, red) / H;
        s1 = LAYERNORM ? block_sum(s1, red) / H : 0.f;
#pragma unroll
        for (int i = 0; i < MAX_VEC; ++i) {
            const int c = threadIdx.x + i * NORM_THREADS;
            if (c < nvec) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    o[e] = (__bf16)((float)tr[i][e] + rstd * (dxh[i][e] - s1 - xh[i][e] * s2));
                *(bf16x8 *)(dx + (size_t)row * H + c * 8) = o;
                if (CSUM) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        sr[i][e] += (float)tr[i][e];
                        sx[i][e] += (float)o[e];
                    }
                }
            }
        }
    }
    float *pg = partial + (size_t)blockIdx.x * 2 * H, *pb = pg + H;
#pragma unroll
    for (int i = 0; i < MAX_VEC; ++i) {
        const int c = threadIdx.x + i * NORM_THREADS;
        if (c < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pg[c * 8 + e] = dg[i][e];
                pb[c * 8 + e] = db[i][e];
            }
            if (CSUM) {
                float *cr = csum + (size_t)blockIdx.x * 2 * H, *cx = cr + H;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    cr[c * 8 + e] = sr[i][e];
                    cx[c * 8 + e] = sx[i][e];
                }
            }
        }
    }
}

// The same backward with one wavefront per row (H <= 64 * 8 * NV): no workgroup barrier in the walk, the
// row sums are wave reductions, and the next row's loads are in flight while the current row is
// worked on (24 KB per wave in flight at H = 4096).  Every wave keeps its own column sums.  W = 4: every
// wave writes its own partial, partial[(blockIdx.x * 4 + wave)][2][H].  W = 8 (narrow rows, where four
// waves per CU have too few bytes in flight to fill the memory pipes): the workgroup's eight waves add
// their column sums in LDS, in wave order, and leave ONE partial, partial[blockIdx.x][2][H]: twice the
// rows in flight for a quarter of the partial sums written here and read again by the final reduction.
template <bool LAYERNORM, int NV, bool CSUM, int W>
__global__ __launch_bounds__(64 * W) void norm_bwd_wave_kernel(
    const __bf16 *__restrict__ dh, const __bf16 *__restrict__ x, const float *__restrict__ stats,
    const __bf16 *__restrict__ gamma, const __bf16 *__restrict__ dres, __bf16 *__restrict__ dx,
    float *__restrict__ partial, float *__restrict__ csum, int T, int H) {
    const int nvec = H / 8, lane = threadIdx.x & 63;
    const int slot = blockIdx.x * W + (threadIdx.x >> 6), n_slots = gridDim.x * W;
    bf16x8 g[NV];
    float dg[NV][8], db[NV][8];
    float sr[CSUM ? NV : 1][8], sx[CSUM ? NV : 1][8];   // column sums of dres and of dx (see norm_bwd_kernel)
#pragma unroll
    for (int i = 0; i < (CSUM ? NV : 1); ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) sr[i][e] = sx[i][e] = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
#pragma unroll
        for (int e = 0; e < 8; ++e) dg[i][e] = db[i][e] = 0.f;
        g[i] = c < nvec ? *(const bf16x8 *)(gamma + c * 8) : bf16x8{};
    }
    bf16x8 nx[NV], nd[NV], nr[NV];
    float nmean = 0.f, nrstd = 0.f;
    auto fetch = [&](int row) {
        nmean = stats[2 * (size_t)row];
        nrstd = stats[2 * (size_t)row + 1];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nvec) {
                nx[i] = *(const bf16x8 *)(x + (size_t)row * H + c * 8);
                nd[i] = *(const bf16x8 *)(dh + (size_t)row * H + c * 8);
                nr[i] = *(const bf16x8 *)(dres + (size_t)row * H + c * 8);
            }
        }
    };
    if (slot < T) fetch(slot);
    for (int row = slot; row < T; row += n_slots) {
        const float mean = nmean, rstd = nrstd;
        bf16x8 cx[NV], cd[NV], cr[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) { cx[i] = nx[i]; cd[i] = nd[i]; cr[i] = nr[i]; }
        if (row + n_slots < T) fetch(row + n_slots);
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (lane + 64 * i < nvec) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float d = (float)cd[i][e];
                    const float xh = ((float)cx[i][e] - mean) * rstd;
                    const float dxh = d * (float)g[i][e];
                    dg[i][e] += d * xh;
                    db[i][e] += d;
                    s1 += dxh;
                    s2 += dxh * xh;
                }
            }
        }
        s2 = wave_sum(s2) / H;
        s1 = LAYERNORM ? wave_sum(s1) / H : 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nvec) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float xh = ((float)cx[i][e] - mean) * rstd;
                    const float dxh = (float)cd[i][e] * (float)g[i][e];
                    o[e] = (__bf16)((float)cr[i][e] + rstd * (dxh - s1 - xh * s2));
                }
                *(bf16x8 *)(dx + (size_t)row * H + c * 8) = o;
                if (CSUM) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        sr[i][e] += (float)cr[i][e];
                        sx[i][e] += (float)o[e];
                    }
                }
            }
        }
    }
    if constexpr (W == 4) {
        float *pg = partial + (size_t)slot * 2 * H, *pb = pg + H;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = lane + 64 * i;
            if (c < nvec) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pg[c * 8 + e] = dg[i][e];
                    pb[c * 8 + e] = db[i][e];
                }
                if (CSUM) {
                    float *pr = csum + (size_t)slot * 2 * H, *px = pr + H;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        pr[c * 8 + e] = sr[i][e];
                        px[c * 8 + e] = sx[i][e];
                    }
                }
            }
        }
    } else {
        constexpr int HMAX = 64 * 8 * NV;
        __shared__ float red[W][2][HMAX];
        const int wave = threadIdx.x >> 6;
        auto fold = [&](const float (&a)[NV][8], const float (&b)[NV][8], float *__restrict__ out) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int c = lane + 64 * i;
                if (c < nvec) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        red[wave][0][c * 8 + e] = a[i][e];
                        red[wave][1][c * 8 + e] = b[i][e];
                    }
                }
            }
            __syncthreads();
            for (int c = threadIdx.x; c < 2 * H; c += 64 * W) {
                const int which = c >= H ? 1 : 0, col = c - which * H;
                float sum = red[0][which][col];
#pragma unroll
                for (int w = 1; w < W; ++w) sum += red[w][which][col];
                out[c] = sum;   // [2][H]
            }
            __syncthreads();
        };
        fold(dg, db, partial + (size_t)blockIdx.x * 2 * H);
        if constexpr (CSUM) fold(sr, sx, csum + (size_t)blockIdx.x * 2 * H);
    }
}

// out[c] = (accumulate ? out[c] : 0) + sum_p partial[p * stride + c]; fixed summation order.
// A workgroup owns 32 columns; its RG groups of 32 lanes each sum every RG-th partial (eight
// independent chains per lane to keep loads in flight: the kernel is a chain of dependent memory
// latencies, a few hundred partials deep), then the RG sums are combined in LDS.
constexpr int REDUCE_THREADS = 512, RG = REDUCE_THREADS / 32;
__device__ __forceinline__ void reduce_columns(const float *__restrict__ partial, int n_part, int stride,
                                               __bf16 *__restrict__ out, int C, int accumulate) {
    __shared__ float red[RG][32];
    const int col = threadIdx.x & 31, pl = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + col;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (c < C) {
        int p = pl;
        for (; p + 7 * RG < n_part; p += 8 * RG) {
#pragma unroll
            for (int u = 0; u < 8; ++u) s[u] += partial[(size_t)(p + u * RG) * stride + c];
        }
        for (; p < n_part; p += RG) s[0] += partial[(size_t)p * stride + c];
    }
    red[pl][col] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
    __syncthreads();
    if (pl == 0 && c < C) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < RG; ++i) t += red[i][col];
        if (accumulate) t += (float)out[c];
        out[c] = (__bf16)t;
    }
}

__global__ __launch_bounds__(REDUCE_THREADS) void reduce_partials_kernel(const float *__restrict__ partial,
                                                              int n_part, int stride,
                                                              __bf16 *__restrict__ out, int C,
                                                              int accumulate) {
    reduce_columns(partial, n_part, stride, out, C, accumulate);
}

// the reductions of one block's backward pass in one launch: blockIdx.y picks the job
__global__ __launch_bounds__(REDUCE_THREADS) void reduce_batch_kernel(ReduceBatch b, int accumulate) {
    const ReduceJob j = b.job[blockIdx.y];
    if ((int)blockIdx.x * 32 >= j.C) return;
    reduce_columns(j.partial, j.n_part, j.stride, (__bf16 *)j.out, j.C, accumulate);
}

// partial[blockIdx.y][c] = sum over the rows blockIdx.y, +gridDim.y, ... of in[row][c]
__global__ __launch_bounds__(256) void colsum_kernel(const __bf16 *__restrict__ in, int T, int C,
                                                     int ld, float *__restrict__ partial) {
    const int c8 = blockIdx.x * 256 + threadIdx.x;  // 8-column vector index
    if (c8 * 8 >= C) return;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const __bf16 *src = in + c8 * 8;
    const int g = gridDim.y;
    int row = blockIdx.y;
    // four rows' loads in flight; the rows are added in the order they are walked
    for (; row + 3 * g < T; row += 4 * g) {
        bf16x8 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = *(const bf16x8 *)(src + (size_t)(row + u * g) * ld);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += (float)t[u][e];
    }
    for (; row < T; row += g) {
        const bf16x8 t = *(const bf16x8 *)(src + (size_t)row * ld);
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += (float)t[e];
    }
    float *dst = partial + (size_t)blockIdx.y * C + c8 * 8;
    *(f32x4 *)dst = f32x4{s[0], s[1], s[2], s[3]};
    *(f32x4 *)(dst + 4) = f32x4{s[4], s[5], s[6], s[7]};
}

// segment index of token t: the j with cu[j] <= t < cu[j+1]
__device__ __forceinline__ int find_segment(const int32_t *__restrict__ cu, int n_seg, int t) {
    int lo = 0, hi = n_seg;  // invariant: cu[lo] <= t < cu[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// In-place rotation of the first n_heads_rot heads of each row of qkv (the q heads then the k
// heads are contiguous there): pair (i, i + d/2) by sign * pos * base^(-2 i / d).
// One workgroup per token.  The angle depends on (token, i) only, so its cosine and sine are
// computed once per token (d/2 values, in LDS) and shared by all heads; the token's position is
// its distance to the largest segment start not behind it, found by one wave in parallel.
__global__ __launch_bounds__(256) void rotary_kernel(__bf16 *__restrict__ qkv, int ld, int T,
                                                     int n_heads_rot, int d,
                                                     const int32_t *__restrict__ cu, int n_seg,
                                                     float log2_base, float sign) {
    const int t = blockIdx.x;
    const int half = d / 2;   // <= 64
    __shared__ float cs_s[64], sn_s[64];
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        int start = 0;
        for (int j0 = 0; j0 < n_seg; j0 += 64) {
            const int j = j0 + lane;
            const int c = j < n_seg ? cu[j] : 0;
            start = max(start, c <= t ? c : 0);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) start = max(start, __shfl_xor(start, o));
        if (lane < half) {
            const float theta = exp2f(-2.0f * (float)lane / (float)d * log2_base);
            float sn, cs;
            sincosf((float)(t - start) * theta, &sn, &cs);
            cs_s[lane] = cs;
            sn_s[lane] = sn * sign;
        }
    }
    __syncthreads();
    const int per_head = half / 8;
    for (int w = threadIdx.x; w < n_heads_rot * per_head; w += blockDim.x) {
        const int head = w / per_head, i0 = (w % per_head) * 8;
        __bf16 *p = qkv + (size_t)t * ld + head * d + i0;
        const bf16x8 a = *(const bf16x8 *)p, b = *(const bf16x8 *)(p + half);
        bf16x8 oa, obb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float cs = cs_s[i0 + e], sn = sn_s[i0 + e];
            const float x1 = (float)a[e], x2 = (float)b[e];
            oa[e] = (__bf16)(x1 * cs - x2 * sn);
            obb[e] = (__bf16)(x2 * cs + x1 * sn);
        }
        *(bf16x8 *)p = oa;
        *(bf16x8 *)(p + half) = obb;
    }
}

__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
    return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * __expf(-0.5f * z * z) * 0.3989422804014327f;
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + __expf(-z)); }

// GELU: act[t, f] = gelu(up[t, f]).  SwiGLU: up row = [gate (F) | up (F)], act = silu(gate) * up.
template <bool SWIGLU>
__global__ __launch_bounds__(256) void act_fwd_kernel(const __bf16 *__restrict__ up,
                                                      __bf16 *__restrict__ act, long n_vec, int F) {
    const int fv = F / 8;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (long)gridDim.x * 256) {
        const long t = i / fv;
        const int c = (int)(i % fv) * 8;
        bf16x8 o;
        if (SWIGLU) {
            const bf16x8 g = *(const bf16x8 *)(up + t * 2 * F + c);
            const bf16x8 u = *(const bf16x8 *)(up + t * 2 * F + F + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gz = (float)g[e];
                o[e] = (__bf16)(gz * sigmoid_f(gz) * (float)u[e]);
            }
        } else {
            const bf16x8 u = *(const bf16x8 *)(up + t * F + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)gelu_f((float)u[e]);
        }
        *(bf16x8 *)(act + t * F + c) = o;
    }
}

template <bool SWIGLU>
__global__ __launch_bounds__(256) void act_bwd_kernel(const __bf16 *__restrict__ dact,
                                                      const __bf16 *__restrict__ up,
                                                      __bf16 *__restrict__ dup, long n_vec, int F) {
    const int fv = F / 8;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (long)gridDim.x * 256) {
        const long t = i / fv;
        const int c = (int)(i % fv) * 8;
        const bf16x8 da = *(const bf16x8 *)(dact + t * F + c);
        if (SWIGLU) {
            const bf16x8 g = *(const bf16x8 *)(up + t * 2 * F + c);
            const bf16x8 u = *(const bf16x8 *)(up + t * 2 * F + F + c);
            bf16x8 og, ou;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gz = (float)g[e], sg = sigmoid_f(gz), d = (float)da[e];
                og[e] = (__bf16)(d * (float)u[e] * sg * (1.0f + gz * (1.0f - sg)));
                ou[e] = (__bf16)(d * gz * sg);
            }
            *(bf16x8 *)(dup + t * 2 * F + c) = og;
            *(bf16x8 *)(dup + t * 2 * F + F + c) = ou;
        } else {
            const bf16x8 u = *(const bf16x8 *)(up + t * F + c);
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)da[e] * gelu_grad_f((float)u[e]));
            *(bf16x8 *)(dup + t * F + c) = o;
        }
    }
}

__global__ __launch_bounds__(256) void mask_kernel(const int32_t *__restrict__ cu, int n_seg, int T,
                                                   int causal, uint8_t *__restrict__ out) {
    const int i = blockIdx.x;
    const int seg = find_segment(cu, n_seg, i);
    const int a = cu[seg], b = causal ? i + 1 : cu[seg + 1];
    for (int j = threadIdx.x; j < T; j += 256) out[(size_t)i * T + j] = (j >= a && j < b) ? 1 : 0;
}

}  // namespace

template <int NV>
static void launch_norm_fwd_wave(int norm, const void *x, const void *gamma, const void *beta, void *h, float *stats,
                                 int T, int H, float eps, int groups, hipStream_t s) {
    if (norm == OB_LAYERNORM)
        hipLaunchKernelGGL((norm_fwd_wave_kernel<true, NV>), dim3(groups), dim3(256), 0, s, (const __bf16 *)x,
                           (const __bf16 *)gamma, (const __bf16 *)beta, (__bf16 *)h, stats, T, H, eps);
    else
        hipLaunchKernelGGL((norm_fwd_wave_kernel<false, NV>), dim3(groups), dim3(256), 0, s, (const __bf16 *)x,
                           (const __bf16 *)gamma, (const __bf16 *)nullptr, (__bf16 *)h, stats, T, H, eps);
}

void launch_norm_fwd(int norm, const void *x, const void *gamma, const void *beta, void *h,
                     float *stats, int T, int H, float eps, hipStream_t s) {
    ProfScope prof(K_NORM_FWD, s, 4.0 * T * H);
    if (H <= 2048) {
        const int groups = (T + 3) / 4 < 1024 ? (T + 3) / 4 : 1024;      // 4 rows at a time per workgroup
        if (H <= 512) launch_norm_fwd_wave<1>(norm, x, gamma, beta, h, stats, T, H, eps, groups, s);
        else if (H <= 1024) launch_norm_fwd_wave<2>(norm, x, gamma, beta, h, stats, T, H, eps, groups, s);
        else launch_norm_fwd_wave<4>(norm, x, gamma, beta, h, stats, T, H, eps, groups, s);
        return;
    }
    if (norm == OB_LAYERNORM)
        hipLaunchKernelGGL(norm_fwd_kernel<true>, dim3(T), dim3(NORM_THREADS), 0, s, (const __bf16 *)x,
                           (const __bf16 *)gamma, (const __bf16 *)beta, (__bf16 *)h, stats, T, H, eps);
    else
        hipLaunchKernelGGL(norm_fwd_kernel<false>, dim3(T), dim3(NORM_THREADS), 0, s, (const __bf16 *)x,
                           (const __bf16 *)gamma, (const __bf16 *)nullptr, (__bf16 *)h, stats, T, H, eps);
}

// rows of H <= 1024 elements, enough of them: 256 workgroups of eight row-walking waves, one partial each
static bool norm_bwd_folds(int T, int H) { return H <= 1024 && T >= 2048; }
int norm_bwd_partials(int T, int H) { return norm_bwd_folds(T, H) ? 256 : T < 1024 ? T : 1024; }

template <int NV, int W>
static void launch_norm_bwd_wave(int norm, const void *dh, const void *x, const float *stats, const void *gamma,
                                 const void *dres, void *dx, float *partial, float *csum, int T, int H, int wgs,
                                 hipStream_t s) {
#define OB_NBW(LN, CS)                                                                                          \
    hipLaunchKernelGGL((norm_bwd_wave_kernel<LN, NV, CS, W>), dim3(wgs), dim3(64 * W), 0, s, (const __bf16 *)dh, \
                       (const __bf16 *)x, stats, (const __bf16 *)gamma, (const __bf16 *)dres, (__bf16 *)dx,     \
                       partial, csum, T, H)
    if (norm == OB_LAYERNORM) { if (csum) OB_NBW(true, true); else OB_NBW(true, false); }
    else { if (csum) OB_NBW(false, true); else OB_NBW(false, false); }
#undef OB_NBW
}

// csum (may be null): [norm_bwd_partials(T, H)][2][H] fp32, column sums of dres and of dx per partial
void launch_norm_bwd(int norm, const void *dh, const void *x, const float *stats, const void *gamma,
                     const void *dres, void *dx, float *partial, int T, int H, hipStream_t s, float *csum) {
    ProfScope prof(K_NORM_BWD, s, 8.0 * T * H);
    const int nb = norm_bwd_partials(T, H);
    if (norm_bwd_folds(T, H)) {
        launch_norm_bwd_wave<2, 8>(norm, dh, x, stats, gamma, dres, dx, partial, csum, T, H, nb, s);
        return;
    }
    // a wave per row while a row fits 8 vectors per lane and there are whole workgroups of rows
    if (H <= 4096 && nb % 4 == 0) {
        if (H <= 1024) launch_norm_bwd_wave<2, 4>(norm, dh, x, stats, gamma, dres, dx, partial, csum, T, H, nb / 4, s);
        else if (H <= 2048) launch_norm_bwd_wave<4, 4>(norm, dh, x, stats, gamma, dres, dx, partial, csum, T, H, nb / 4, s);
        else launch_norm_bwd_wave<8, 4>(norm, dh, x, stats, gamma, dres, dx, partial, csum, T, H, nb / 4, s);
        return;
    }
#define OB_NB(LN, CS)                                                                                          \
    hipLaunchKernelGGL((norm_bwd_kernel<LN, CS>), dim3(nb), dim3(NORM_THREADS), 0, s, (const __bf16 *)dh,       \
                       (const __bf16 *)x, stats, (const __bf16 *)gamma, (const __bf16 *)dres, (__bf16 *)dx,    \
                       partial, csum, T, H)
    if (norm == OB_LAYERNORM) { if (csum) OB_NB(true, true); else OB_NB(true, false); }
    else { if (csum) OB_NB(false, true); else OB_NB(false, false); }
#undef OB_NB
}

void launch_reduce_partials(const float *partial, int n_part, int stride, void *out, int C,
                            int accumulate, hipStream_t s) {
    ProfScope prof(K_REDUCE, s, 4.0 * n_part * C);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((C + 31) / 32), dim3(REDUCE_THREADS), 0, s, partial, n_part,
                       stride, (__bf16 *)out, C, accumulate);
}

int launch_reduce_batch(const ReduceBatch &b, int accumulate, hipStream_t s) {
    if (b.overflow) return fail(OB_EINVAL, "reduce batch: more than %d column reductions in one launch", ReduceBatch::MAX);
    if (b.n == 0) return OB_OK;
    double work = 0.0;
    int max_c = 0;
    for (int i = 0; i < b.n; ++i) {
        work += 4.0 * b.job[i].n_part * b.job[i].C;
        if (b.job[i].C > max_c) max_c = b.job[i].C;
    }
    ProfScope prof(K_REDUCE, s, work);
    hipLaunchKernelGGL(reduce_batch_kernel, dim3((max_c + 31) / 32, b.n), dim3(REDUCE_THREADS), 0, s, b, accumulate);
    return OB_OK;
}

int colsum_partials(int T) { return T < 256 ? T : 256; }

void launch_colsum(const void *in, int T, int C, int ld, float *partial, hipStream_t s) {
    ProfScope prof(K_COLSUM, s, 2.0 * T * C);
    dim3 grid((C / 8 + 255) / 256, colsum_partials(T));
    hipLaunchKernelGGL(colsum_kernel, grid, dim3(256), 0, s, (const __bf16 *)in, T, C, ld, partial);
}

void launch_rotary(void *qkv, int ld, int T, int n_heads_rot, int d, const int32_t *cu_dev, int n_seg,
                   float base, float sign, hipStream_t s) {
    ProfScope prof(K_ROTARY, s, 4.0 * T * n_heads_rot * d);
    hipLaunchKernelGGL(rotary_kernel, dim3(T), dim3(256), 0, s, (__bf16 *)qkv, ld, T, n_heads_rot, d,
                       cu_dev, n_seg, log2f(base), sign);
}

void launch_act_fwd(int mlp, const void *up, void *act, int T, int F, hipStream_t s) {
    ProfScope prof(K_ACT_FWD, s, (mlp == OB_SWIGLU ? 6.0 : 4.0) * T * F);
    const long n_vec = (long)T * (F / 8);
    const int blocks = (int)((n_vec + 255) / 256 < 65536 ? (n_vec + 255) / 256 : 65536);
    if (mlp == OB_SWIGLU)
        hipLaunchKernelGGL(act_fwd_kernel<true>, dim3(blocks), dim3(256), 0, s, (const __bf16 *)up,
                           (__bf16 *)act, n_vec, F);
    else
        hipLaunchKernelGGL(act_fwd_kernel<false>, dim3(blocks), dim3(256), 0, s, (const __bf16 *)up,
                           (__bf16 *)act, n_vec, F);
}

void launch_act_bwd(int mlp, const void *dact, const void *up, void *dup, int T, int F, hipStream_t s) {
    ProfScope prof(K_ACT_BWD, s, (mlp == OB_SWIGLU ? 10.0 : 6.0) * T * F);
    const long n_vec = (long)T * (F / 8);
    const int blocks = (int)((n_vec + 255) / 256 < 65536 ? (n_vec + 255) / 256 : 65536);
    if (mlp == OB_SWIGLU)
        hipLaunchKernelGGL(act_bwd_kernel<true>, dim3(blocks), dim3(256), 0, s, (const __bf16 *)dact,
                           (const __bf16 *)up, (__bf16 *)dup, n_vec, F);
    else
        hipLaunchKernelGGL(act_bwd_kernel<false>, dim3(blocks), dim3(256), 0, s, (const __bf16 *)dact,
                           (const __bf16 *)up, (__bf16 *)dup, n_vec, F);
}

void launch_mask(const int32_t *cu_dev, int n_seg, int T, int mask, uint8_t *out, hipStream_t s) {
    hipLaunchKernelGGL(mask_kernel, dim3(T), dim3(256), 0, s, cu_dev, n_seg, T,
                       mask == OB_MASK_SEG_CAUSAL ? 1 : 0, out);
}

}  // namespace ob
