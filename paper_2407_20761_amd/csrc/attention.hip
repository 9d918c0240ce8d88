// Flash-style variable-length attention for gfx950 (steps a4 and b4 of the block).
//
// A packed batch is a concatenation of segments (cu offsets); a token attends only inside its own
// segment, bidirectionally (ViT tile) or causally (LLM sample).  Work is tiled per segment, so
// score tiles that would straddle two segments are never formed, and causal tiles above the
// diagonal are skipped.
//
// All matrix products run on the 32x32x16 bf16 MFMA in "transposed" form: the wavefront's 32 query
// rows (forward, dQ) or 32 key rows (dK/dV) sit on the MFMA's column index, which is the lane
// index.  Each lane therefore owns ONE row of the softmax: row max / row sum are in-register
// reductions plus a single exchange between lane l and lane l+32, and the probabilities a lane
// holds in its accumulator registers are, without any data movement, exactly the 8-value k-slices
// the next MFMA wants as its second operand.  The accumulator's row order
// (8 (r/4) + 4 (l/32) + r%4) fixes which k index each slot carries; the other operand is staged
// in LDS transposed with its 16-element groups permuted to the same order.
#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;
constexpr int QT = 128;  // rows owned by a workgroup (4 waves x 32)
constexpr int ST = 64;   // rows of the streamed tile held in LDS

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// [rows][D] bf16 tile, 16-byte chunks XOR-swizzled so 32 consecutive rows read conflict-free
template <int D>
__device__ __forceinline__ int swz_rows(int row, int chunk) {
    return D == 128 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}
// [D][64] transposed tile: 8 chunks of 16 bytes per row
__device__ __forceinline__ int swz_t(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Stage rows [row0, row0 + 64) of a [*, ld] matrix (columns col0 .. col0 + D) into LDS, as a
// row-major swizzled tile (`normal`) and/or transposed (`transposed`, [D][64]).  Rows past
// row_last are replaced by row_last (their contribution is masked by the callers).
// In the transposed tile the 64 positions of a row are grouped by 16; inside a group, source
// index 8a + 4h + c sits at 8h + 4a + c, which is the order in which an MFMA accumulator lane
// (half h) holds its eight values of that group.
template <int D>
__device__ __forceinline__ void stage_tile(const __bf16 *__restrict__ g, int ld, int row0,
                                           int row_last, unsigned char *normal,
                                           unsigned char *transposed) {
    constexpr int CH = D / 8;
#pragma unroll
    for (int p = 0; p < ST * CH / 256; ++p) {
        const int qd = threadIdx.x + p * 256, row = qd / CH, c = qd % CH;
        const int gr = min(row0 + row, row_last);
        const u32x4 val = *(const u32x4 *)(g + (size_t)gr * ld + c * 8);
        if (normal) *(u32x4 *)(normal + row * (D * 2) + swz_rows<D>(row, c) * 16) = val;
        if (transposed) {
            const int grp = row >> 4, a = (row >> 3) & 1, h = (row >> 2) & 1, cc = row & 3;
            const int chunk = 2 * grp + h, elem = 4 * a + cc;
            const unsigned short *e16 = (const unsigned short *)&val;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int dd = 8 * c + e;
                *(unsigned short *)(transposed + dd * 128 + swz_t(dd, chunk) * 16 + elem * 2) = e16[e];
            }
        }
    }
}

template <int D>
__device__ __forceinline__ bf16x8 frag_rows(const unsigned char *tile, int row, int chunk) {
    return *(const bf16x8 *)(tile + row * (D * 2) + swz_rows<D>(row, chunk) * 16);
}
__device__ __forceinline__ bf16x8 frag_t(const unsigned char *tile, int row, int chunk) {
    return *(const bf16x8 *)(tile + row * 128 + swz_t(row, chunk) * 16);
}

// accumulator registers 8 (u % 2) .. +7 of a 32x32 tile -> the 8-slot second operand of k-step u
__device__ __forceinline__ bf16x8 pack8(const f32x16 &a, int base) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)a[base + e];
    return o;
}

// which segment-aligned tile (of `tile_rows` rows) is blockIdx.x
struct TileInfo { int seg_start, seg_end, row0, local; };
__device__ __forceinline__ TileInfo find_tile(const int32_t *__restrict__ cu, int n_seg, int tile_rows,
                                              int *sh) {
    if (threadIdx.x == 0) {
        int acc = 0, j = 0, a = 0, b = 0, loc = 0;
        for (; j < n_seg; ++j) {
            a = cu[j];
            b = cu[j + 1];
            const int nt = (b - a + tile_rows - 1) / tile_rows;
            if ((int)blockIdx.x < acc + nt) { loc = blockIdx.x - acc; break; }
            acc += nt;
        }
        sh[0] = a; sh[1] = b; sh[2] = loc; sh[3] = (j < n_seg) ? 1 : 0;
    }
    __syncthreads();
    TileInfo t;
    t.seg_start = sh[0]; t.seg_end = sh[1]; t.local = sh[2];
    t.row0 = sh[3] ? t.seg_start + t.local * tile_rows : -1;
    return t;
}

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    __bf16 *__restrict__ o, float *__restrict__ lse, int ldq, int ldkv, int ldo,
    const int32_t *__restrict__ cu, int n_seg, int T, int group, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned char k_s[ST * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char vt_s[D * ST * 2];
    __shared__ int sh[4];
    const TileInfo ti = find_tile(cu, n_seg, QT, sh);
    if (ti.row0 < 0) return;
    const int head = blockIdx.y, kvh = head / group;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lx = lane & 31, lh = lane >> 5;
    const int q_row = min(ti.row0 + wave * 32 + lx, ti.seg_end - 1);
    const bool q_live = ti.row0 + wave * 32 + lx < ti.seg_end;
    const int wave_q_last = min(ti.row0 + wave * 32 + 31, ti.seg_end - 1);
    const float sl2 = scale * LOG2E;

    bf16x8 qf[D / 16];
#pragma unroll
    for (int t = 0; t < D / 16; ++t)
        qf[t] = *(const bf16x8 *)(q + (size_t)q_row * ldq + head * D + 16 * t + 8 * lh);

    f32x16 acc_o[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;
    float m_run = NEG_BIG, l_run = 0.f;

    const int kv_end = CAUSAL ? min(ti.seg_end, ti.row0 + QT) : ti.seg_end;
    for (int kv0 = ti.seg_start; kv0 < kv_end; kv0 += ST) {
        __syncthreads();
        stage_tile<D>(k + kvh * D, ldkv, kv0, ti.seg_end - 1, k_s, nullptr);
        stage_tile<D>(v + kvh * D, ldkv, kv0, ti.seg_end - 1, nullptr, vt_s);
        __syncthreads();
        if (CAUSAL && kv0 > wave_q_last) continue;

        f32x16 acc_s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[mt][r] = 0.f;
#pragma unroll
            for (int t = 0; t < D / 16; ++t)
                acc_s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_rows<D>(k_s, mt * 32 + lx, 2 * t + lh), qf[t], acc_s[mt], 0, 0, 0);
        }
        float mx = NEG_BIG;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = kv0 + mt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const bool ok = kv < ti.seg_end && (!CAUSAL || kv <= q_row);
                const float s = ok ? acc_s[mt][r] * sl2 : NEG_BIG;
                acc_s[mt][r] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(acc_s[mt][r] - m_new);
                acc_s[mt][r] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
#pragma unroll
        for (int u = 0; u < ST / 16; ++u) {
            const bf16x8 pb = pack8(acc_s[u >> 1], 8 * (u & 1));
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
                acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_t(vt_s, dt * 32 + lx, 2 * u + lh), pb, acc_o[dt], 0, 0, 0);
        }
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!q_live) return;
    const float inv = 1.0f / l_tot;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc_o[dt][4 * g + e] * inv);
            *(bf16x4 *)(o + (size_t)q_row * ldo + head * D + dt * 32 + g * 8 + lh * 4) = ov;
        }
    if (lh == 0) lse[(size_t)head * T + q_row] = (m_run + __builtin_amdgcn_logf(l_tot)) * LN2;
}

// ------------------------------------------------------------------------------------------------
// backward, part 1: dQ.  Same ownership as the forward (a wave owns 32 query rows and streams the
// segment's keys); P is rebuilt from the saved log-sum-exp.
//   S^T = K Q^T,  P = exp(scale S - lse),  dP^T = V dO^T,  dS^T = P (dP^T - Delta),  dQ^T += K^T dS^T
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(
    const __bf16 *__restrict__ d_o, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k,
    const __bf16 *__restrict__ v, const float *__restrict__ lse, const float *__restrict__ delta,
    __bf16 *__restrict__ dq, int ldq, int ldkv, int ldo, const int32_t *__restrict__ cu, int n_seg,
    int T, int group, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned char k_s[ST * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char v_s[ST * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char kt_s[D * ST * 2];
    __shared__ int sh[4];
    const TileInfo ti = find_tile(cu, n_seg, QT, sh);
    if (ti.row0 < 0) return;
    const int head = blockIdx.y, kvh = head / group;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lx = lane & 31, lh = lane >> 5;
    const int q_row = min(ti.row0 + wave * 32 + lx, ti.seg_end - 1);
    const bool q_live = ti.row0 + wave * 32 + lx < ti.seg_end;
    const int wave_q_last = min(ti.row0 + wave * 32 + 31, ti.seg_end - 1);
    const float sl2 = scale * LOG2E;

    bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        qf[t] = *(const bf16x8 *)(q + (size_t)q_row * ldq + head * D + 16 * t + 8 * lh);
        dof[t] = *(const bf16x8 *)(d_o + (size_t)q_row * ldo + head * D + 16 * t + 8 * lh);
    }
    const float lse2 = lse[(size_t)head * T + q_row] * LOG2E;
    const float dlt = delta[(size_t)head * T + q_row];

    f32x16 acc_dq[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_dq[i][r] = 0.f;

    const int kv_end = CAUSAL ? min(ti.seg_end, ti.row0 + QT) : ti.seg_end;
    for (int kv0 = ti.seg_start; kv0 < kv_end; kv0 += ST) {
        __syncthreads();
        stage_tile<D>(k + kvh * D, ldkv, kv0, ti.seg_end - 1, k_s, kt_s);
        stage_tile<D>(v + kvh * D, ldkv, kv0, ti.seg_end - 1, v_s, nullptr);
        __syncthreads();
        if (CAUSAL && kv0 > wave_q_last) continue;
        f32x16 acc_s[2], acc_dp[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[mt][r] = acc_dp[mt][r] = 0.f;
#pragma unroll
            for (int t = 0; t < D / 16; ++t) {
                acc_s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_rows<D>(k_s, mt * 32 + lx, 2 * t + lh), qf[t], acc_s[mt], 0, 0, 0);
                acc_dp[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_rows<D>(v_s, mt * 32 + lx, 2 * t + lh), dof[t], acc_dp[mt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = kv0 + mt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const bool ok = kv < ti.seg_end && (!CAUSAL || kv <= q_row);
                const float p = ok ? fast_exp2(acc_s[mt][r] * sl2 - lse2) : 0.f;
                acc_s[mt][r] = p * (acc_dp[mt][r] - dlt);
            }
#pragma unroll
        for (int u = 0; u < ST / 16; ++u) {
            const bf16x8 dsb = pack8(acc_s[u >> 1], 8 * (u & 1));
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
                acc_dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_t(kt_s, dt * 32 + lx, 2 * u + lh), dsb, acc_dq[dt], 0, 0, 0);
        }
    }
    if (!q_live) return;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc_dq[dt][4 * g + e] * scale);
            *(bf16x4 *)(dq + (size_t)q_row * ldq + head * D + dt * 32 + g * 8 + lh * 4) = ov;
        }
}

// ------------------------------------------------------------------------------------------------
// backward, part 2: dK, dV.  A wave owns 32 key rows of one KV head and streams, for every query
// head of the group, the segment's query rows (from the diagonal on when causal):
//   S = Q K^T,  P = exp(scale S - lse),  dV^T += dO^T P,  dP = dO V^T,  dS = P (dP - Delta),
//   dK^T += Q^T dS.   The sum over the group's query heads happens in the accumulators.
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(
    const __bf16 *__restrict__ d_o, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k,
    const __bf16 *__restrict__ v, const float *__restrict__ lse, const float *__restrict__ delta,
    __bf16 *__restrict__ dk, __bf16 *__restrict__ dv, int ldq, int ldkv, int ldo,
    const int32_t *__restrict__ cu, int n_seg, int T, int group, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned char q_s[ST * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char do_s[ST * D * 2];
    __shared__ __attribute__((aligned(16))) unsigned char qt_s[D * ST * 2];
    __shared__ __attribute__((aligned(16))) unsigned char dot_s[D * ST * 2];
    __shared__ __attribute__((aligned(16))) float lse_s[ST];
    __shared__ __attribute__((aligned(16))) float dlt_s[ST];
    __shared__ int sh[4];
    const TileInfo ti = find_tile(cu, n_seg, QT, sh);
    if (ti.row0 < 0) return;
    const int kvh = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lx = lane & 31, lh = lane >> 5;
    const int kv_row = min(ti.row0 + wave * 32 + lx, ti.seg_end - 1);
    const bool kv_live = ti.row0 + wave * 32 + lx < ti.seg_end;
    const int wave_kv_first = ti.row0 + wave * 32;
    const float sl2 = scale * LOG2E;

    bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        kf[t] = *(const bf16x8 *)(k + (size_t)kv_row * ldkv + kvh * D + 16 * t + 8 * lh);
        vf[t] = *(const bf16x8 *)(v + (size_t)kv_row * ldkv + kvh * D + 16 * t + 8 * lh);
    }
    f32x16 acc_dk[D / 32], acc_dv[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_dk[i][r] = acc_dv[i][r] = 0.f;

    // causal: query rows before this workgroup's first key row see none of its keys
    const int q_begin = CAUSAL ? ti.seg_start + ((ti.row0 - ti.seg_start) / ST) * ST : ti.seg_start;
    for (int hg = 0; hg < group; ++hg) {
        const int head = kvh * group + hg;
        for (int q0 = q_begin; q0 < ti.seg_end; q0 += ST) {
            __syncthreads();
            stage_tile<D>(q + head * D, ldq, q0, ti.seg_end - 1, q_s, qt_s);
            stage_tile<D>(d_o + head * D, ldo, q0, ti.seg_end - 1, do_s, dot_s);
            if (threadIdx.x < ST) {
                const int r = min(q0 + (int)threadIdx.x, ti.seg_end - 1);
                lse_s[threadIdx.x] = lse[(size_t)head * T + r] * LOG2E;
                dlt_s[threadIdx.x] = delta[(size_t)head * T + r];
            }
            __syncthreads();
            // a 64-row query tile entirely before this wave's keys contributes nothing
            if (CAUSAL && q0 + ST - 1 < wave_kv_first) continue;
            f32x16 acc_s[2], acc_dp[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_s[mt][r] = acc_dp[mt][r] = 0.f;
#pragma unroll
                for (int t = 0; t < D / 16; ++t) {
                    acc_s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(q_s, mt * 32 + lx, 2 * t + lh), kf[t], acc_s[mt], 0, 0, 0);
                    acc_dp[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(do_s, mt * 32 + lx, 2 * t + lh), vf[t], acc_dp[mt], 0, 0, 0);
                }
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int qi = mt * 32 + 8 * g + 4 * lh;  // 4 consecutive query rows
                    const f32x4 l4 = *(const f32x4 *)(lse_s + qi);
                    const f32x4 d4 = *(const f32x4 *)(dlt_s + qi);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * g + e;
                        const int qr = q0 + qi + e;
                        const bool ok = qr < ti.seg_end && (!CAUSAL || kv_row <= qr);
                        const float p = ok ? fast_exp2(acc_s[mt][r] * sl2 - l4[e]) : 0.f;
                        acc_s[mt][r] = p;
                        acc_dp[mt][r] = p * (acc_dp[mt][r] - d4[e]);
                    }
                }
#pragma unroll
            for (int u = 0; u < ST / 16; ++u) {
                const bf16x8 pb = pack8(acc_s[u >> 1], 8 * (u & 1));
                const bf16x8 dsb = pack8(acc_dp[u >> 1], 8 * (u & 1));
#pragma unroll
                for (int dt = 0; dt < D / 32; ++dt) {
                    acc_dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_t(dot_s, dt * 32 + lx, 2 * u + lh), pb, acc_dv[dt], 0, 0, 0);
                    acc_dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_t(qt_s, dt * 32 + lx, 2 * u + lh), dsb, acc_dk[dt], 0, 0, 0);
                }
            }
        }
    }
    if (!kv_live) return;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 ok_, ov_;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ok_[e] = (__bf16)(acc_dk[dt][4 * g + e] * scale);
                ov_[e] = (__bf16)acc_dv[dt][4 * g + e];
            }
            const size_t off = (size_t)kv_row * ldkv + kvh * D + dt * 32 + g * 8 + lh * 4;
            *(bf16x4 *)(dk + off) = ok_;
            *(bf16x4 *)(dv + off) = ov_;
        }
}

// algorithmic forward FLOPs: 4 nq d sum_seg A(s), A = s^2 or s (s + 1) / 2 (causal)
double attn_flops(const ob_segments *seg, int nq, int d, bool causal) {
    double area = 0;
    for (int j = 0; j < seg->n_seg; ++j) {
        const double len = seg->cu_host[j + 1] - seg->cu_host[j];
        area += causal ? len * (len + 1) / 2 : len * len;
    }
    return 4.0 * nq * d * area;
}

int count_tiles(const ob_segments *seg, int tile_rows) {
    long n = 0;
    for (int j = 0; j < seg->n_seg; ++j)
        n += (seg->cu_host[j + 1] - seg->cu_host[j] + tile_rows - 1) / tile_rows;
    return (int)n;
}

}  // namespace

#define OB_ATTN_DISPATCH(KERNEL, GRID, ...)                                                        \
    do {                                                                                           \
        if (d == 64 && causal)                                                                     \
            hipLaunchKernelGGL((KERNEL<64, true>), GRID, dim3(256), 0, s, __VA_ARGS__);            \
        else if (d == 64)                                                                          \
            hipLaunchKernelGGL((KERNEL<64, false>), GRID, dim3(256), 0, s, __VA_ARGS__);           \
        else if (causal)                                                                           \
            hipLaunchKernelGGL((KERNEL<128, true>), GRID, dim3(256), 0, s, __VA_ARGS__);           \
        else                                                                                       \
            hipLaunchKernelGGL((KERNEL<128, false>), GRID, dim3(256), 0, s, __VA_ARGS__);          \
    } while (0)

void launch_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int ldq,
                     int ldkv, int ldo, const ob_segments *seg, int nq, int nkv, int d, float scale,
                     int mask, hipStream_t s) {
    const bool causal = mask == OB_MASK_SEG_CAUSAL;
    ProfScope prof(K_ATTN_FWD, s, attn_flops(seg, nq, d, causal));
    const dim3 grid(count_tiles(seg, QT), nq);
    OB_ATTN_DISPATCH(attn_fwd_kernel, grid, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v,
                     (__bf16 *)o, lse, ldq, ldkv, ldo, seg->cu_dev, seg->n_seg, seg->total_tokens,
                     nq / nkv, scale);
}

void launch_attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const float *lse,
                     const float *delta, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                     const ob_segments *seg, int nq, int nkv, int d, float scale, int mask,
                     hipStream_t s) {
    const bool causal = mask == OB_MASK_SEG_CAUSAL;
    const int tiles = count_tiles(seg, QT);
    const dim3 grid_q(tiles, nq), grid_kv(tiles, nkv);
    {
    ProfScope prof(K_ATTN_BWD_DQ, s, 0.5 * attn_flops(seg, nq, d, causal));  // dQ = dS K: 1 of the 4 bwd products
    OB_ATTN_DISPATCH(attn_bwd_dq_kernel, grid_q, (const __bf16 *)d_o, (const __bf16 *)q,
                     (const __bf16 *)k, (const __bf16 *)v, lse, delta, (__bf16 *)dq, ldq, ldkv, ldo,
                     seg->cu_dev, seg->n_seg, seg->total_tokens, nq / nkv, scale);
    }
    ProfScope prof(K_ATTN_BWD_DKV, s, 1.5 * attn_flops(seg, nq, d, causal));  // dV, dP, dK
    OB_ATTN_DISPATCH(attn_bwd_dkv_kernel, grid_kv, (const __bf16 *)d_o, (const __bf16 *)q,
                     (const __bf16 *)k, (const __bf16 *)v, lse, delta, (__bf16 *)dk, (__bf16 *)dv, ldq,
                     ldkv, ldo, seg->cu_dev, seg->n_seg, seg->total_tokens, nq / nkv, scale);
}

}  // namespace ob
