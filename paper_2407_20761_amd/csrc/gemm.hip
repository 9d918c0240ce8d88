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
#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

namespace {

constexpr int BK = 64;  // k per LDS stage: 8 chunks of 16 bytes per row

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

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
__global__ __launch_bounds__(WM * WN * 64) void gemm_nt_kernel(
    int M, int N, int K, const __bf16 *__restrict__ A, int lda, const __bf16 *__restrict__ B,
    int ldb, __bf16 *__restrict__ C, int ldc, const __bf16 *__restrict__ bias,
    const __bf16 *R, int ldr, int tiles_m, int tiles_n) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;  // 32-row MFMA tiles per wave along m
    constexpr int TN = BN / WN / 32;
    constexpr int A_CHUNKS = BM * 8 / NT;  // 16-byte chunks per thread per stage
    constexpr int B_CHUNKS = BN * 8 / NT;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/thread mismatch");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // [2 stages][A tile BM*64 | B tile BN*64] bf16
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    auto a_tile = [&](int s) { return smem + s * STAGE_BYTES; };
    auto b_tile = [&](int s) { return smem + s * STAGE_BYTES + BM * BK * 2; };

    int tile_m, tile_n;
    tile_coords(tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lx = lane & 31, lh = lane >> 5;

    // global -> register staging addresses (row clamped into the matrix; out-of-range rows are
    // computed on duplicate data and never stored)
    const __bf16 *a_src[A_CHUNKS];
    const __bf16 *b_src[B_CHUNKS];
    int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
#pragma unroll
    for (int p = 0; p < A_CHUNKS; ++p) {
        const int q = tid + p * NT, row = q >> 3, c = q & 7;
        a_src[p] = A + (size_t)min(m0 + row, M - 1) * lda + c * 8;
        a_dst[p] = row * (BK * 2) + swz(row, c) * 16;
    }
#pragma unroll
    for (int p = 0; p < B_CHUNKS; ++p) {
        const int q = tid + p * NT, row = q >> 3, c = q & 7;
        b_src[p] = B + (size_t)min(n0 + row, N - 1) * ldb + c * 8;
        b_dst[p] = row * (BK * 2) + swz(row, c) * 16;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 a_reg[A_CHUNKS], b_reg[B_CHUNKS];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_CHUNKS; ++p) a_reg[p] = *(const u32x4 *)(a_src[p] + k0);
#pragma unroll
        for (int p = 0; p < B_CHUNKS; ++p) b_reg[p] = *(const u32x4 *)(b_src[p] + k0);
    };
    auto store_lds = [&](int s) {
#pragma unroll
        for (int p = 0; p < A_CHUNKS; ++p) *(u32x4 *)(a_tile(s) + a_dst[p]) = a_reg[p];
#pragma unroll
        for (int p = 0; p < B_CHUNKS; ++p) *(u32x4 *)(b_tile(s) + b_dst[p]) = b_reg[p];
    };

    const int nk = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int s = kt & 1;
        if (kt + 1 < nk) load_global((kt + 1) * BK);
        const unsigned char *as = a_tile(s) + (wm * (BM / WM)) * (BK * 2);
        const unsigned char *bs = b_tile(s) + (wn * (BN / WN)) * (BK * 2);
#pragma unroll
        for (int t = 0; t < BK / 16; ++t) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = i * 32 + lx;
                af[i] = *(const bf16x8 *)(as + row * (BK * 2) +
                                          swz(wm * (BM / WM) + row, 2 * t + lh) * 16);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = j * 32 + lx;
                bfr[j] = *(const bf16x8 *)(bs + row * (BK * 2) +
                                           swz(wn * (BN / WN) + row, 2 * t + lh) * 16);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j],
                                                                       0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(s ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, per MFMA tile, column m = lx and rows n = 8 g + 4 lh + (0..3)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * (BM / WM) + i * 32 + lx;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * (BN / WN) + j * 32 + g * 8 + lh * 4;
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][g * 4 + e];
                if (bias) {
                    const bf16x4 bv = *(const bf16x4 *)(bias + n);
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += (float)bv[e];
                }
                if (R) {
                    const bf16x4 rv = *(const bf16x4 *)(R + (size_t)m * ldr + n);
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += (float)rv[e];
                }
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
                *(bf16x4 *)(C + (size_t)m * ldc + n) = o;
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
    constexpr int smem = 2 * (BM + BN) * BK * 2;
    auto kern = gemm_nt_kernel<BM, BN, WM, WN>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WM * WN * 64), smem, s, M, N, K,
                       (const __bf16 *)A, lda, (const __bf16 *)B, ldb, (__bf16 *)C, ldc,
                       (const __bf16 *)bias, (const __bf16 *)R, ldr, tiles_m, tiles_n);
}

}  // namespace

void launch_gemm_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C,
                    int ldc, const void *bias, const void *R, int ldr, hipStream_t s, int k_algo) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * (k_algo > 0 ? k_algo : K));
    // big tiles when they still fill the 256 CUs a few times over, smaller ones otherwise
    const long tiles_big = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (tiles_big >= 512)
        launch_nt<256, 256, 2, 4>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
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
