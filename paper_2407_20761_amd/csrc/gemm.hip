// bf16 MFMA GEMM for gfx950 (steps a2, a5, a7, a9 and their dgrad / wgrad counterparts).
//
//   C[M,N] = A[M,K] * B[N,K]^T (+ bias[N]) (+ R[M,N])      bf16 in, fp32 accumulate, bf16 out
//
// One workgroup owns a BM x BN tile of C and walks K in steps of 64.  Both operands are
// K-contiguous, so a 16-byte global load is 8 consecutive k of one row; tiles are staged in LDS
// as [row][64 k] with the 16-byte chunk index XOR-swizzled by the row so that the 32 rows a
// wavefront reads for one MFMA operand fall into different banks.  The MFMA is 32x32x16 bf16:
// lane l supplies row (l % 32), k = 8 (l / 32) .. +7 of each operand, i.e. one 16-byte LDS read.
// The weight rows are fed as the MFMA's first operand so that a lane's four consecutive
// accumulator registers are four consecutive columns n of one output row m (8-byte stores).
#include <cmath>

#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

#define OB_LDS __attribute__((address_space(3)))

constexpr int BK = 64;           // k per LDS stage: 8 chunks of 16 bytes = 128 bytes per row
constexpr int ROW_BYTES = BK * 2;

// tile id -> (tile_m, tile_n): each XCD (blocks are dealt round-robin to the 8 XCDs) gets one
// contiguous range of tile ids, and ids walk groups of GM tile-rows column by column, so the
// tiles resident on one XCD at a time share A and B panels in that XCD's L2.
__device__ __forceinline__ void tile_coords(int tiles_m, int tiles_n, int &tm, int &tn) {
    const int nblk = gridDim.x, pid = blockIdx.x;
    const int per = nblk >> 3, rem = nblk & 7;
    const int xcd = pid & 7, loc = pid >> 3;
    const int tile = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + loc;
    constexpr int GM = 8;
    const int width = GM * tiles_n;
    const int group = tile / width;
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = tile - group * width;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

template <int BM, int BN, int WM, int WN>
struct Cfg {
    static constexpr int NW = WM * WN, NT = NW * 64;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // 32x32 MFMA tiles per wave
    // a wave instruction of the LDS-direct load fills 1 KB = 8 rows of a tile
    static constexpr int A_LD = BM / 8 / NW, B_LD = BN / 8 / NW;
    static constexpr int STAGE = (BM + BN) * ROW_BYTES;
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile / wave count mismatch");
};

// Per-thread addressing state.  LDS tiles are [row][8 chunks of 16 B]; the chunk stored at
// physical position p of row r is logical chunk p ^ f(r), f(r) = (r ^ ((r >> 3) & 1)) & 7, which
// keeps the 16-byte reads of 8 as well as of 16 consecutive rows on distinct banks.
template <int BM, int BN, int WM, int WN>
struct Ctx {
    using C = Cfg<BM, BN, WM, WN>;
    const unsigned char *a_base, *b_base;        // tile origin in A / B (wave-uniform)
    uint32_t a_off[C::A_LD], b_off[C::B_LD];     // this lane's byte offset for each of its loads
    int wave;
    int xa[BK / 16], xb[BK / 16];                // this lane's LDS read offset for k-step t
};

// Asynchronous global -> LDS copy of one K-step's A and B tiles: lane l of a wave instruction
// supplies the global address of the 16 bytes that land at LDS base + 16 l.
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void issue_loads(unsigned char OB_LDS *__restrict__ dst,
                                            const Ctx<BM, BN, WM, WN> &c, int kbytes) {
    using C = Cfg<BM, BN, WM, WN>;
#pragma unroll
    for (int p = 0; p < C::A_LD; ++p)
        __builtin_amdgcn_global_load_lds(c.a_base + kbytes + c.a_off[p],
                                         dst + (c.wave * C::A_LD + p) * 1024, 16, 0, 0);
#pragma unroll
    for (int p = 0; p < C::B_LD; ++p)
        __builtin_amdgcn_global_load_lds(c.b_base + kbytes + c.b_off[p],
                                         dst + BM * ROW_BYTES + (c.wave * C::B_LD + p) * 1024, 16, 0, 0);
}

template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void load_frags(const unsigned char OB_LDS *__restrict__ src,
                                           const Ctx<BM, BN, WM, WN> &c, int t,
                                           bf16x8 (&af)[Cfg<BM, BN, WM, WN>::TM],
                                           bf16x8 (&bfr)[Cfg<BM, BN, WM, WN>::TN]) {
    using C = Cfg<BM, BN, WM, WN>;
#pragma unroll
    for (int i = 0; i < C::TM; ++i) af[i] = *(const bf16x8 OB_LDS *)(src + c.xa[t] + i * 32 * ROW_BYTES);
#pragma unroll
    for (int j = 0; j < C::TN; ++j) bfr[j] = *(const bf16x8 OB_LDS *)(src + c.xb[t] + j * 32 * ROW_BYTES);
}

// Multiply one LDS stage (4 k-steps of 16).  The fragments of k-step t+1 are read while the
// MFMAs of k-step t run; the scheduling groups pin "one LDS read, one MFMA" pairs at the front of
// each k-step so every read has at least half a k-step of MFMA work to hide behind.
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void compute_stage(const unsigned char OB_LDS *__restrict__ src,
                                              const Ctx<BM, BN, WM, WN> &c,
                                              f32x16 (&acc)[Cfg<BM, BN, WM, WN>::TM][Cfg<BM, BN, WM, WN>::TN]) {
    using C = Cfg<BM, BN, WM, WN>;
    bf16x8 af[2][C::TM], bfr[2][C::TN];
    load_frags<BM, BN, WM, WN>(src, c, 0, af[0], bfr[0]);
#pragma unroll
    for (int t = 0; t < BK / 16; ++t) {
        if (t + 1 < BK / 16) load_frags<BM, BN, WM, WN>(src, c, t + 1, af[(t + 1) & 1], bfr[(t + 1) & 1]);
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[t & 1][j], af[t & 1][i],
                                                                   acc[i][j], 0, 0, 0);
        if (t + 1 < BK / 16) {
#pragma unroll
            for (int r = 0; r < C::TM + C::TN; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// C[M,N] = A[M,K] B[N,K]^T (+bias) (+R).  Two LDS stages; the copy of K-step kt+1 is in flight
// while K-step kt is multiplied; one barrier per K-step.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_nt_kernel(
    int M, int N, int K, const __bf16 *__restrict__ A, int lda, const __bf16 *__restrict__ B,
    int ldb, __bf16 *__restrict__ Cm, int ldc, const __bf16 *__restrict__ bias,
    const __bf16 *R, int ldr, int tiles_m, int tiles_n) {
    using C = Cfg<BM, BN, WM, WN>;
    __shared__ __attribute__((aligned(1024))) unsigned char st0[C::STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[C::STAGE];

    int tile_m, tile_n;
    tile_coords(tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    Ctx<BM, BN, WM, WN> c;
    c.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = c.wave / WN, wn = c.wave % WN;
    const int lx = lane & 31, lh = lane >> 5;

    // rows past the matrix edge are clamped onto its last row: they are multiplied as duplicate
    // data and never stored
    c.a_base = (const unsigned char *)(A + (size_t)m0 * lda);
    c.b_base = (const unsigned char *)(B + (size_t)n0 * ldb);
#pragma unroll
    for (int p = 0; p < C::A_LD; ++p) {
        const int blk = c.wave * C::A_LD + p, row = blk * 8 + (lane >> 3);
        const int ch = (lane & 7) ^ (((lane >> 3) ^ (blk & 1)) & 7);
        c.a_off[p] = ((uint32_t)min(row, M - 1 - m0) * (uint32_t)lda + ch * 8) * 2u;
    }
#pragma unroll
    for (int p = 0; p < C::B_LD; ++p) {
        const int blk = c.wave * C::B_LD + p, row = blk * 8 + (lane >> 3);
        const int ch = (lane & 7) ^ (((lane >> 3) ^ (blk & 1)) & 7);
        c.b_off[p] = ((uint32_t)min(row, N - 1 - n0) * (uint32_t)ldb + ch * 8) * 2u;
    }
    const int f = (lx ^ ((lx >> 3) & 1)) & 7;
#pragma unroll
    for (int t = 0; t < BK / 16; ++t) {
        c.xa[t] = (wm * (BM / WM) + lx) * ROW_BYTES + (((2 * t + lh) ^ f) * 16);
        c.xb[t] = BM * ROW_BYTES + (wn * (BN / WN) + lx) * ROW_BYTES + (((2 * t + lh) ^ f) * 16);
    }

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    unsigned char OB_LDS *s0 = (unsigned char OB_LDS *)st0;
    unsigned char OB_LDS *s1 = (unsigned char OB_LDS *)st1;
    const int nk = K / BK;
    constexpr int WAIT_VM0 = 0x0F70;  // s_waitcnt vmcnt(0) only
    issue_loads<BM, BN, WM, WN>(s0, c, 0);
    int kt = 0;
    for (; kt + 2 <= nk; kt += 2) {
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        __syncthreads();
        issue_loads<BM, BN, WM, WN>(s1, c, (kt + 1) * ROW_BYTES);
        compute_stage<BM, BN, WM, WN>(s0, c, acc);
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        __syncthreads();
        if (kt + 2 < nk) issue_loads<BM, BN, WM, WN>(s0, c, (kt + 2) * ROW_BYTES);
        compute_stage<BM, BN, WM, WN>(s1, c, acc);
    }
    if (kt < nk) {
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);
        __syncthreads();
        compute_stage<BM, BN, WM, WN>(s0, c, acc);
    }

    // Epilogue.  A lane holds, per MFMA tile, output row m = lx and columns n = 8 g + 4 lh + (0..3):
    // stored directly, every lane of a store would touch a different cache line.  Instead each
    // wave transposes 32-row slabs of its tile through its share of the (now idle) stage buffers
    // as fp32, and reads them back so that 16 (or 8) consecutive lanes cover one contiguous row
    // segment; bias and residual are added on the way out, then one rounding to bf16.
    __syncthreads();  // every wave is done reading the last stage
    constexpr int CW = BN / WN;            // columns of the wave's tile
    constexpr int RSTR = CW * 4 + 16;      // fp32 row stride in LDS, padded against bank conflicts
    constexpr int LPR = CW / 8;            // lanes per row on the way out (8 columns each)
    constexpr int RPI = 64 / LPR;          // rows per read instruction
    static_assert(32 * RSTR <= C::STAGE / (C::NW / 2), "slab does not fit the wave's LDS share");
    unsigned char OB_LDS *slab = (c.wave < C::NW / 2 ? s0 : s1) + (c.wave % (C::NW / 2)) * (C::STAGE / (C::NW / 2));
    const int n_out = n0 + wn * CW + (lane % LPR) * 8;
    float bv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bv[e] = 0.f;
    if (bias && n_out < N) {
        const bf16x8 b8 = *(const bf16x8 *)(bias + n_out);
#pragma unroll
        for (int e = 0; e < 8; ++e) bv[e] = (float)b8[e];
    }
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][g * 4 + e];
                *(f32x4 OB_LDS *)(slab + lx * RSTR + (j * 32 + g * 8 + lh * 4) * 4) = v;
            }
#pragma unroll
        for (int r = 0; r < 32 / RPI; ++r) {
            const int row = r * RPI + lane / LPR;
            const f32x4 lo = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32);
            const f32x4 hi = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32 + 16);
            const int m = m0 + wm * (BM / WM) + i * 32 + row;
            if (m < M && n_out < N) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[e] = lo[e] + bv[e]; v[4 + e] = hi[e] + bv[4 + e]; }
                if (R) {
                    const bf16x8 r8 = *(const bf16x8 *)(R + (size_t)m * ldr + n_out);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] += (float)r8[e];
                }
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
                *(bf16x8 *)(Cm + (size_t)m * ldc + n_out) = o;
            }
        }
    }
}

// out[c][r] = in[r][c]; rows r in [rows, rows_pad) are written as zero.  64x64 tiles via LDS.
__global__ __launch_bounds__(256) void transpose_pad_kernel(const unsigned short *__restrict__ in,
                                                            int rows, int cols, int ld_in,
                                                            unsigned short *__restrict__ out,
                                                            int rows_pad) {
    __shared__ unsigned short tile[64][66];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? in[(size_t)r * ld_in + c] : (unsigned short)0;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows_pad) out[(size_t)c * rows_pad + r] = tile[tx][i];
    }
}

template <int BM, int BN, int WM, int WN>
void launch_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
               const void *bias, const void *R, int ldr, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    auto kern = gemm_nt_kernel<BM, BN, WM, WN>;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WM * WN * 64), 0, s, M, N, K,
                       (const __bf16 *)A, lda, (const __bf16 *)B, ldb, (__bf16 *)C, ldc,
                       (const __bf16 *)bias, (const __bf16 *)R, ldr, tiles_m, tiles_n);
}

}  // namespace

void launch_gemm_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C,
                    int ldc, const void *bias, const void *R, int ldr, hipStream_t s, int k_algo) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * (k_algo > 0 ? k_algo : K));
    // 256x256 tiles run one workgroup per CU, 128x128 tiles two; take the shape whose last round
    // of tiles leaves fewer CUs idle (the small tile pays ~15 % in operand re-reads)
    const double big = (double)((M + 255) / 256) * ((N + 255) / 256);
    const double small = (double)((M + 127) / 128) * ((N + 127) / 128);
    const double eff_big = big / (ceil(big / 256.0) * 256.0);
    const double eff_small = 0.85 * small / (ceil(small / 512.0) * 512.0);
    if (eff_big >= eff_small)
        launch_nt<256, 256, 2, 2>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
    else
        launch_nt<128, 128, 2, 2>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
}

void launch_transpose_pad(const void *in, int rows, int cols, int ld_in, void *out, int rows_pad,
                          hipStream_t s) {
    ProfScope prof(K_TRANSPOSE, s, 2.0 * rows * cols + 2.0 * rows_pad * cols);
    dim3 grid((rows_pad + 63) / 64, (cols + 63) / 64);
    hipLaunchKernelGGL(transpose_pad_kernel, grid, dim3(256), 0, s, (const unsigned short *)in,
                       rows, cols, ld_in, (unsigned short *)out, rows_pad);
}

size_t gemm_workspace_bytes(int layout, int M, int N, int K) {
    if (layout == 1) return align_up((size_t)N * K * 2, 256);
    if (layout == 2) {
        const size_t kp = align_up((size_t)K, 64);
        return align_up((size_t)M * kp * 2, 256) + align_up((size_t)N * kp * 2, 256);
    }
    return 0;
}

// layout 0: A[M,K] B[N,K]; 1: A[M,K] B[K,N]; 2: A[K,M] B[K,N].  NN / TN operands are re-laid
// out K-contiguous in `ws` first (zero-padded along K to a multiple of 64 for TN).
int gemm_any(int layout, int M, int N, int K, const void *A, const void *B, void *C,
             const void *bias, const void *R, void *ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < gemm_workspace_bytes(layout, M, N, K))
        return fail(OB_EWORKSPACE, "gemm: workspace too small");
    if (layout == 0) {
        launch_gemm_nt(M, N, K, A, K, B, K, C, N, bias, R, N, s);
    } else if (layout == 1) {
        launch_transpose_pad(B, K, N, N, ws, K, s);  // B[K,N] -> Bt[N,K]
        launch_gemm_nt(M, N, K, A, K, ws, K, C, N, bias, R, N, s);
    } else {
        const int kp = (int)align_up((size_t)K, 64);
        unsigned char *at = (unsigned char *)ws;
        unsigned char *bt = at + align_up((size_t)M * kp * 2, 256);
        launch_transpose_pad(A, K, M, M, at, kp, s);  // A[K,M] -> At[M,kp]
        launch_transpose_pad(B, K, N, N, bt, kp, s);  // B[K,N] -> Bt[N,kp]
        launch_gemm_nt(M, N, kp, at, kp, bt, kp, C, N, bias, R, N, s, K);
    }
    return check_launch("gemm");
}

}  // namespace ob
