// bf16 MFMA GEMM for gfx950 (steps a2, a5, a7, a9 and their dgrad / wgrad counterparts).
//
//   C[M,N] = op(A) * op(B) (+ bias[N]) (+ R[M,N])      bf16 in, fp32 accumulate, bf16 out
//   "NT" A[M,K] B[N,K] (forward)   "NN" A[M,K] B[K,N] (dgrad)   "TN" A[K,M] B[K,N] (wgrad, K = tokens)
//
// One workgroup (4 wavefronts, each a 128x128 block of 4x4 MFMA 32x32x16 tiles, 256 accumulator
// registers) owns a 256x256 tile of C and walks K in steps of 64 over two LDS stages.  Tiles go
// global -> registers -> LDS: every wave issues one 16-byte-per-lane buffer load after every few
// MFMAs, all K step long, and writes each vector to LDS one whole K step after it was requested,
// so the memory pipeline sees a steady stream (a burst of a K step's loads blocks the wave's
// instruction issue, MFMAs included, until the cache has taken them) and no wait ever meets a
// load in flight.  The hardware range check of the buffer descriptor turns every access past the end
// of an operand (row tails of M / N, the ragged token tail of K) into zeros.  A K-contiguous operand
// is staged as [row][64 k] and a fragment is one 16-byte LDS read; a K-major operand is staged as
// it lies in memory, [k][rows], and the fragment comes out of two transposing LDS reads, so dgrad
// and wgrad need no re-layout pass.  16-byte chunks are XOR-swizzled on the way in (the global
// address of each lane's chunk is free to choose) so that LDS reads are bank-conflict free.
// The weight-side rows are the MFMA's first operand, so a lane's accumulators are runs of four
// consecutive output columns; the epilogue transposes them through LDS into full-row stores.
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
    // a wave instruction of the LDS-direct load fills 1 KB of a tile; a tile is X rows x 64 k
    static constexpr int A_LD = BM / 8 / NW, B_LD = BN / 8 / NW;
    static constexpr int STAGE = (BM + BN) * ROW_BYTES;
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile / wave count mismatch");
};

// One operand's tile in LDS, in one of two layouts.
//
// KMAJOR = false: the source is [X, K] with k contiguous.  LDS holds [x][8 chunks of 16 B]; the
//   chunk at physical position p of row x is logical chunk p ^ f(x), f(x) = (x ^ ((x >> 3) & 1)) & 7,
//   so the 16-byte reads of 16 consecutive rows hit distinct banks.  A fragment (row x, 8
//   consecutive k) is one 16-byte read.
// KMAJOR = true: the source is [K, X] with x contiguous.  LDS holds [k][X / 8 chunks of 16 B]
//   (8 x-values per chunk); the chunk at physical position p of row k is logical chunk
//   p ^ 4 (k & 3).  A fragment is two transposing 8-byte reads (ds_read_b64_tr_b16): inside a
//   group of 16 lanes, lane 4 k' + c addresses the 4 x-values [4c, 4c+4) of row k' of a 4 x 16
//   block, and lane p receives column p, i.e. 4 consecutive k of one x.
template <int X, int NW, bool KMAJOR>
struct Operand {
    static constexpr int LD = X / 8 / NW;        // wave-level 1 KB loads per stage
    static constexpr int ROWB = X * 2;           // LDS bytes per k-row (k-major layout)
    const unsigned char *base;                   // advances every K step
    uint32_t nrec, step;                         // bytes left from `base`; bytes per K step
    uint32_t voff[LD];                           // this lane's byte offset for each of its loads
    int rd[KMAJOR ? X / 32 : BK / 16];           // this lane's LDS read offsets (per tile i / per k-step t)

    // ld = source leading dimension (elements); x0 = first tile row; extent = rows (k-major: K)
    __device__ __forceinline__ void init(const __bf16 *src, int ld, int x0, long total_bytes, int wave,
                                         int lane, int wave_x0, int tiles) {
        if (!KMAJOR) {
            base = (const unsigned char *)(src + (size_t)x0 * ld);
            const long left = total_bytes - (long)x0 * ld * 2;
            nrec = (uint32_t)(left > 0xFFFFFFFFl ? 0xFFFFFFFFl : left);
            step = ROW_BYTES;
#pragma unroll
            for (int p = 0; p < LD; ++p) {
                const int blk = wave * LD + p, row = blk * 8 + (lane >> 3);
                const int ch = (lane & 7) ^ (((lane >> 3) ^ (blk & 1)) & 7);
                voff[p] = ((uint32_t)row * (uint32_t)ld + ch * 8) * 2u;
            }
            const int lx = lane & 31, lh = lane >> 5;
            const int f = (lx ^ ((lx >> 3) & 1)) & 7;
#pragma unroll
            for (int t = 0; t < BK / 16; ++t) rd[t] = (wave_x0 + lx) * ROW_BYTES + (((2 * t + lh) ^ f) * 16);
        } else {
            base = (const unsigned char *)(src + x0);
            const long left = total_bytes - (long)x0 * 2;
            nrec = (uint32_t)(left > 0xFFFFFFFFl ? 0xFFFFFFFFl : left);
            step = (uint32_t)BK * (uint32_t)ld * 2u;
            constexpr int KPB = 1024 / ROWB, CPR = ROWB / 16;   // k-rows per 1 KB load, chunks per row
#pragma unroll
            for (int p = 0; p < LD; ++p) {
                const int blk = wave * LD + p, k = blk * KPB + lane / CPR;
                const int ch = (lane % CPR) ^ (4 * (k & 3));
                voff[p] = ((uint32_t)k * (uint32_t)ld + ch * 8) * 2u;
            }
            const int b = lane >> 4, q = lane & 15, kq = q >> 2, c = q & 3, hb = b >> 1, nb = 16 * (b & 1);
#pragma unroll
            for (int i = 0; i < X / 32; ++i) {
                if (i >= tiles) { rd[i] = 0; continue; }
                const int chunk = (wave_x0 + 32 * i + nb) / 8 + (c >> 1);
                rd[i] = (8 * hb + kq) * ROWB + ((chunk ^ (4 * kq)) * 16) + (c & 1) * 8;
            }
        }
    }
    __device__ __forceinline__ void advance() {
        base += step;
        nrec = nrec > step ? nrec - step : 0u;
    }
    // descriptor of the current K step; must sit in scalar registers: pin its (uniform) parts explicitly
    // (live = false: an empty range, every load returns zeros without touching memory)
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t descriptor(bool live) const {
        const uint64_t b = (uint64_t)base;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
        return __builtin_amdgcn_make_buffer_rsrc((void *)(((uint64_t)hi << 32) | lo), 0,
                                                 live ? (int)__builtin_amdgcn_readfirstlane(nrec) : 0, 0x00020000);
    }
    // piece p (1 KB per wave) of this wave's share of the K step behind `rsrc`: global -> registers;
    // loads past the end of the source (rows beyond M / N / K) deliver zeros
    __device__ __forceinline__ u32x4 load(__amdgpu_buffer_rsrc_t rsrc, int p) const {
        return __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff[p], 0, 0);
    }
    // registers -> its place in the stage (lane-linear inside the 1 KB piece: the swizzle was applied
    // by the choice of each lane's global address)
    __device__ __forceinline__ void store(unsigned char OB_LDS *__restrict__ dst, int wave, int lane, int p, u32x4 v) const {
        *(u32x4 OB_LDS *)(dst + (wave * LD + p) * 1024 + lane * 16) = v;
    }
    // fragment for MFMA tile i (32 x-values) at k-step t: lane l holds x = l % 32, k = 8 (l / 32) .. +7
    __device__ __forceinline__ bf16x8 frag(const unsigned char OB_LDS *__restrict__ tile, int i, int t) const {
        if (!KMAJOR) {
            return *(const bf16x8 OB_LDS *)(tile + rd[t] + i * 32 * ROW_BYTES);
        } else {
#if defined(__HIP_DEVICE_COMPILE__)  // the gfx950-only builtin must not be seen by the host pass
            typedef __attribute__((ext_vector_type(4))) short s16x4;
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 OB_LDS *)(tile + rd[i] + (16 * t) * ROWB));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 OB_LDS *)(tile + rd[i] + (16 * t + 4) * ROWB));
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
#else
            return bf16x8{};
#endif
        }
    }
};

// The copy stream of one wave: G = A_LD + B_LD vectors in flight, vector g < A_LD is piece g of A,
// the others pieces of B.  A "copy group" writes vector g (requested one K step ago) to the stage
// being refilled and re-issues its load for the K step after.
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
struct CopyStream {
    using C = Cfg<BM, BN, WM, WN>;
    static constexpr int G = C::A_LD + C::B_LD;
    static_assert(G % 4 == 0, "copy groups are dealt to the four k-steps of a K step");
    u32x4 v[G];
    __amdgpu_buffer_rsrc_t ra, rb;
    int k_left;   // K steps not yet given a descriptor

    __device__ __forceinline__ void next_k(Operand<BM, WM * WN, AK> &opa, Operand<BN, WM * WN, BKM> &opb) {
        const bool live = k_left > 0;
        --k_left;
        ra = opa.descriptor(live);
        rb = opb.descriptor(live);
        opa.advance();
        opb.advance();
    }
    __device__ __forceinline__ void request(const Operand<BM, WM * WN, AK> &opa, const Operand<BN, WM * WN, BKM> &opb, int g) {
        v[g] = g < C::A_LD ? opa.load(ra, g) : opb.load(rb, g - C::A_LD);
    }
    __device__ __forceinline__ void deliver(const Operand<BM, WM * WN, AK> &opa, const Operand<BN, WM * WN, BKM> &opb,
                                            unsigned char OB_LDS *__restrict__ dst, int wave, int lane, int g) const {
        if (g < C::A_LD) opa.store(dst, wave, lane, g, v[g]);
        else opb.store(dst + BM * ROW_BYTES, wave, lane, g - C::A_LD, v[g]);
    }
};

// One k-step (16 k): the MFMAs on the fragments in (af_use, bf_use), cut into as many runs as the
// k-step has copy groups.  Each run opens with its share of the fragment reads of k-step t_rd of
// `rd` (into af_rd / bf_rd; READ = false: none), then copy group q * GROUPS + run: deliver to
// `fill`, request the next K step (COPY = false: none), placed between the run's MFMAs.  The runs are
// kept in this order so that buffer loads and LDS traffic leave the wave evenly spaced between MFMAs.
template <int BM, int BN, int WM, int WN, bool AK, bool BKM, bool READ, bool COPY>
__device__ __forceinline__ void k_step(const unsigned char OB_LDS *__restrict__ rd, int t_rd,
                                       unsigned char OB_LDS *__restrict__ fill, int q,
                                       CopyStream<BM, BN, WM, WN, AK, BKM> &cs,
                                       const Operand<BM, WM * WN, AK> &opa,
                                       const Operand<BN, WM * WN, BKM> &opb, int wave, int lane,
                                       bf16x8 (&af_rd)[Cfg<BM, BN, WM, WN>::TM], bf16x8 (&bf_rd)[Cfg<BM, BN, WM, WN>::TN],
                                       const bf16x8 (&af_use)[Cfg<BM, BN, WM, WN>::TM],
                                       const bf16x8 (&bf_use)[Cfg<BM, BN, WM, WN>::TN],
                                       f32x16 (&acc)[Cfg<BM, BN, WM, WN>::TM][Cfg<BM, BN, WM, WN>::TN]) {
    using C = Cfg<BM, BN, WM, WN>;
    constexpr int GROUPS = (C::A_LD + C::B_LD) / 4;
    constexpr int RUN = C::TM * C::TN / GROUPS;       // MFMAs per run
    constexpr int FPR = (C::TM + C::TN) / GROUPS;     // fragments read per run
    static_assert(C::TM * C::TN % GROUPS == 0 && (C::TM + C::TN) % GROUPS == 0, "uneven runs");
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        if (READ) {
#pragma unroll
            // read order a0 b0 b1 .. b(TN-1) a1 a2 ..: the order in which the next k-step's MFMAs
            // first touch them, so the fragments read last are the ones needed last
            for (int f = g * FPR; f < (g + 1) * FPR; ++f) {
                if (f == 0) af_rd[0] = opa.frag(rd, 0, t_rd);
                else if (f <= C::TN) bf_rd[f - 1] = opb.frag(rd + BM * ROW_BYTES, f - 1, t_rd);
                else af_rd[f - C::TN] = opa.frag(rd, f - C::TN, t_rd);
            }
        }
        // the copy group sits in the middle of the run's MFMAs: an LDS write issued right behind the
        // LDS reads costs 3 % (random data) to 10 % (zeros, full clock) of the whole kernel
#pragma unroll
        for (int m = g * RUN; m < g * RUN + RUN / 2; ++m)
            acc[m / C::TN][m % C::TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_use[m % C::TN], af_use[m / C::TN],
                                                                               acc[m / C::TN][m % C::TN], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (COPY) {
            cs.deliver(opa, opb, fill, wave, lane, q * GROUPS + g);
            cs.request(opa, opb, q * GROUPS + g);
        }
#pragma unroll
        for (int m = g * RUN + RUN / 2; m < (g + 1) * RUN; ++m)
            acc[m / C::TN][m % C::TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_use[m % C::TN], af_use[m / C::TN],
                                                                               acc[m / C::TN][m % C::TN], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__device__ __forceinline__ void read_frags(const unsigned char OB_LDS *__restrict__ src,
                                           const Operand<BM, WM * WN, AK> &opa,
                                           const Operand<BN, WM * WN, BKM> &opb, int t,
                                           bf16x8 (&af)[Cfg<BM, BN, WM, WN>::TM],
                                           bf16x8 (&bfr)[Cfg<BM, BN, WM, WN>::TN]) {
    using C = Cfg<BM, BN, WM, WN>;
#pragma unroll
    for (int i = 0; i < C::TM; ++i) af[i] = opa.frag(src, i, t);
#pragma unroll
    for (int j = 0; j < C::TN; ++j) bfr[j] = opb.frag(src + BM * ROW_BYTES, j, t);
}

// quarter q of the copy groups: deliver to `fill`, request the K step behind the stream's descriptors
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__device__ __forceinline__ void copy_quarter(CopyStream<BM, BN, WM, WN, AK, BKM> &cs,
                                             const Operand<BM, WM * WN, AK> &opa,
                                             const Operand<BN, WM * WN, BKM> &opb,
                                             unsigned char OB_LDS *__restrict__ fill, int wave, int lane, int q) {
    constexpr int GROUPS = CopyStream<BM, BN, WM, WN, AK, BKM>::G / 4;
#pragma unroll
    for (int g = q * GROUPS; g < (q + 1) * GROUPS; ++g) {
        cs.deliver(opa, opb, fill, wave, lane, g);
        cs.request(opa, opb, g);
    }
}

// k-steps 0 .. 2 of the stage in `cur`: the fragments of k-step 0 are already in af[0] / bfr[0];
// on return the fragments of k-step 3 are in af[1] / bfr[1] and `cur` is not read again.  Copy
// quarters 1 .. 3 go to `fill` (the other stage).
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__device__ __forceinline__ void stage_front(const unsigned char OB_LDS *__restrict__ cur,
                                            unsigned char OB_LDS *__restrict__ fill,
                                            CopyStream<BM, BN, WM, WN, AK, BKM> &cs,
                                            const Operand<BM, WM * WN, AK> &opa,
                                            const Operand<BN, WM * WN, BKM> &opb, int wave, int lane,
                                            bf16x8 (&af)[2][Cfg<BM, BN, WM, WN>::TM],
                                            bf16x8 (&bfr)[2][Cfg<BM, BN, WM, WN>::TN],
                                            f32x16 (&acc)[Cfg<BM, BN, WM, WN>::TM][Cfg<BM, BN, WM, WN>::TN]) {
#pragma unroll
    for (int t = 0; t < 3; ++t)
        k_step<BM, BN, WM, WN, AK, BKM, true, true>(cur, t + 1, fill, t + 1, cs, opa, opb, wave, lane, af[(t + 1) & 1],
                                                    bfr[(t + 1) & 1], af[t & 1], bfr[t & 1], acc);
}

// k-step 3 of the current stage (fragments in af[1] / bfr[1]) overlapped with the fragment reads
// of k-step 0 of the stage in `nxt` (into af[0] / bfr[0]) and copy quarter 0 into `fill` (the
// stage just left).
template <int BM, int BN, int WM, int WN, bool AK, bool BKM, bool NEXT>
__device__ __forceinline__ void stage_back(const unsigned char OB_LDS *__restrict__ nxt,
                                           unsigned char OB_LDS *__restrict__ fill,
                                           CopyStream<BM, BN, WM, WN, AK, BKM> &cs,
                                           const Operand<BM, WM * WN, AK> &opa,
                                           const Operand<BN, WM * WN, BKM> &opb, int wave, int lane,
                                           bf16x8 (&af)[2][Cfg<BM, BN, WM, WN>::TM],
                                           bf16x8 (&bfr)[2][Cfg<BM, BN, WM, WN>::TN],
                                           f32x16 (&acc)[Cfg<BM, BN, WM, WN>::TM][Cfg<BM, BN, WM, WN>::TN]) {
    k_step<BM, BN, WM, WN, AK, BKM, NEXT, NEXT>(nxt, 0, fill, 0, cs, opa, opb, wave, lane, af[0], bfr[0], af[1], bfr[1], acc);
}

// C[M,N] = op(A) op(B) (+bias) (+R): A is [M,K] (AK = false) or [K,M] (AK = true); B is [N,K]
// (BKM = false) or [K,N] (BKM = true).
//
// Two LDS stages.  The barrier of K step s sits between its third and fourth k-step: by then the
// step's last LDS reads have been issued (their data is needed only by the MFMAs after the
// barrier), so behind the barrier the stage can be refilled, and the first fragments of step
// s + 1 are read while the fourth k-step's MFMAs run.  The refill of a stage takes the four
// k-steps between two barriers (the fourth of step s, the first three of step s + 1) and writes K
// step s + 2, whose vectors were requested during the same four k-steps one K step earlier; the
// registers freed by each write take the request for K step s + 3 right away.  Requests past the
// last K step fall outside the descriptor's range: zeros, no memory access.
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(
    int M, int N, int K, const __bf16 *__restrict__ A, int lda, const __bf16 *__restrict__ B,
    int ldb, __bf16 *__restrict__ Cm, int ldc, const __bf16 *__restrict__ bias,
    const __bf16 *R, int ldr, int tiles_m, int tiles_n) {
    using C = Cfg<BM, BN, WM, WN>;
    __shared__ __attribute__((aligned(1024))) unsigned char st0[C::STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[C::STAGE];

    int tile_m, tile_n;
    tile_coords(tiles_m, tiles_n, tile_m, tile_n);
    // the divisions above run on the vector ALU; pin the (uniform) results to scalar registers so
    // the buffer descriptors built from them are scalar too
    const int m0 = __builtin_amdgcn_readfirstlane(tile_m) * BM;
    const int n0 = __builtin_amdgcn_readfirstlane(tile_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int lx = lane & 31, lh = lane >> 5;

    Operand<BM, C::NW, AK> opa;
    Operand<BN, C::NW, BKM> opb;
    opa.init(A, lda, m0, (AK ? (long)K : (long)M) * lda * 2, wave, lane, wm * (BM / WM), C::TM);
    opb.init(B, ldb, n0, (BKM ? (long)K : (long)N) * ldb * 2, wave, lane, wn * (BN / WN), C::TN);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    unsigned char OB_LDS *s0 = (unsigned char OB_LDS *)st0;
    unsigned char OB_LDS *s1 = (unsigned char OB_LDS *)st1;
    const int nk = (K + BK - 1) / BK;
    using CS = CopyStream<BM, BN, WM, WN, AK, BKM>;
    CS cs;
    cs.k_left = nk;
    // own LDS traffic done (reads landed in registers, writes in the stage), then the barrier;
    // buffer loads stay in flight across it
#define OB_SYNC()                                  \
    do {                                           \
        __builtin_amdgcn_s_waitcnt(0xC07F);        \
        __syncthreads();                           \
    } while (0)
    bf16x8 af[2][C::TM], bfr[2][C::TN];
    // prologue: K step 0 into stage 0; K step 1 requested, its first quarter delivered to stage 1
    // and re-requested for K step 2 -- the state every trip of the loop starts from
    cs.next_k(opa, opb);
#pragma unroll
    for (int g = 0; g < CS::G; ++g) cs.request(opa, opb, g);
#pragma unroll
    for (int g = 0; g < CS::G; ++g) cs.deliver(opa, opb, s0, wave, lane, g);
    cs.next_k(opa, opb);
#pragma unroll
    for (int g = 0; g < CS::G; ++g) cs.request(opa, opb, g);
    cs.next_k(opa, opb);
    copy_quarter<BM, BN, WM, WN, AK, BKM>(cs, opa, opb, s1, wave, lane, 0);
    OB_SYNC();
    read_frags<BM, BN, WM, WN, AK, BKM>(s0, opa, opb, 0, af[0], bfr[0]);
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) {       // two K steps per trip: stage 0 then stage 1, both with successors
        stage_front<BM, BN, WM, WN, AK, BKM>(s0, s1, cs, opa, opb, wave, lane, af, bfr, acc);
        cs.next_k(opa, opb);             // scalar work, kept off the path behind the barrier
        OB_SYNC();                       // stage 1 written everywhere; nobody reads stage 0 any more
        stage_back<BM, BN, WM, WN, AK, BKM, true>(s1, s0, cs, opa, opb, wave, lane, af, bfr, acc);
        stage_front<BM, BN, WM, WN, AK, BKM>(s1, s0, cs, opa, opb, wave, lane, af, bfr, acc);
        cs.next_k(opa, opb);
        OB_SYNC();
        stage_back<BM, BN, WM, WN, AK, BKM, true>(s0, s1, cs, opa, opb, wave, lane, af, bfr, acc);
    }
    // here kt is even, stage 0 holds K step kt (its first fragments are in registers) and stage 1
    // is receiving K step kt + 1 (zeros when that is past the end)
    stage_front<BM, BN, WM, WN, AK, BKM>(s0, s1, cs, opa, opb, wave, lane, af, bfr, acc);
    if (kt + 1 < nk) {
        cs.next_k(opa, opb);
        OB_SYNC();
        stage_back<BM, BN, WM, WN, AK, BKM, true>(s1, s0, cs, opa, opb, wave, lane, af, bfr, acc);
        stage_front<BM, BN, WM, WN, AK, BKM>(s1, s0, cs, opa, opb, wave, lane, af, bfr, acc);
    }
    stage_back<BM, BN, WM, WN, AK, BKM, false>(s0, s0, cs, opa, opb, wave, lane, af, bfr, acc);
#undef OB_SYNC

    // Epilogue.  A lane holds, per MFMA tile, output row m = lx and columns n = 8 g + 4 lh + (0..3):
    // stored directly, every lane of a store would touch a different cache line.  Instead each
    // wave transposes 32-row slabs of its tile through its share of the (now idle) stage buffers
    // as fp32, and reads them back so that 16 (or 8) consecutive lanes cover one contiguous row
    // segment; bias and residual are added on the way out, then one rounding to bf16.
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();  // every wave is done reading the last stage and writing the other one
    constexpr int CW = BN / WN;            // columns of the wave's tile
    constexpr int RSTR = CW * 4 + 16;      // fp32 row stride in LDS, padded against bank conflicts
    constexpr int LPR = CW / 8;            // lanes per row on the way out (8 columns each)
    constexpr int RPI = 64 / LPR;          // rows per read instruction
    static_assert(32 * RSTR <= C::STAGE / (C::NW / 2), "slab does not fit the wave's LDS share");
    unsigned char OB_LDS *slab = (wave < C::NW / 2 ? s0 : s1) + (wave % (C::NW / 2)) * (C::STAGE / (C::NW / 2));
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
                __builtin_nontemporal_store(o, (bf16x8 *)(Cm + (size_t)m * ldc + n_out));
            }
        }
    }
}

// Explicit instantiations: without them hipcc's host pass references but does not emit the launch
// stubs of the variants whose only use sits two templates deep.
#define OB_GEMM_INSTANCE(BM, BN, AK, BKM)                                                          \
    template __global__ void gemm_kernel<BM, BN, 2, 2, AK, BKM>(                                   \
        int, int, int, const __bf16 *, int, const __bf16 *, int, __bf16 *, int, const __bf16 *,    \
        const __bf16 *, int, int, int);
OB_GEMM_INSTANCE(256, 256, false, false)
OB_GEMM_INSTANCE(128, 128, false, false)
OB_GEMM_INSTANCE(256, 256, false, true)
OB_GEMM_INSTANCE(128, 128, false, true)
OB_GEMM_INSTANCE(256, 256, true, true)
OB_GEMM_INSTANCE(128, 128, true, true)
#undef OB_GEMM_INSTANCE

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
void launch_tile(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
                 const void *bias, const void *R, int ldr, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, AK, BKM>), dim3(tiles_m * tiles_n), dim3(WM * WN * 64),
                       0, s, M, N, K, (const __bf16 *)A, lda, (const __bf16 *)B, ldb, (__bf16 *)C, ldc,
                       (const __bf16 *)bias, (const __bf16 *)R, ldr, tiles_m, tiles_n);
}

template <bool AK, bool BKM>
void launch_layout(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
                   const void *bias, const void *R, int ldr, hipStream_t s) {
    // 256x256 tiles run one workgroup per CU, 128x128 tiles two; take the shape whose last round
    // of tiles leaves fewer CUs idle (the small tile pays ~15 % in operand re-reads)
    const double big = (double)((M + 255) / 256) * ((N + 255) / 256);
    const double small = (double)((M + 127) / 128) * ((N + 127) / 128);
    const double eff_big = big / (ceil(big / 256.0) * 256.0);
    const double eff_small = 0.85 * small / (ceil(small / 512.0) * 512.0);
    if (eff_big >= eff_small)
        launch_tile<256, 256, 2, 2, AK, BKM>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
    else
        launch_tile<128, 128, 2, 2, AK, BKM>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
}

}  // namespace

void launch_gemm_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C,
                    int ldc, const void *bias, const void *R, int ldr, hipStream_t s, int k_algo) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * (k_algo > 0 ? k_algo : K));
    launch_layout<false, false>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, s);
}

size_t gemm_workspace_bytes(int, int, int, int) { return 0; }

// layout 0 ("NT"): A[M,K] B[N,K]; 1 ("NN"): A[M,K] B[K,N]; 2 ("TN"): A[K,M] B[K,N].  All three
// run natively: a K-major operand is staged as it lies in memory and transposed by the LDS read.
int gemm_any(int layout, int M, int N, int K, const void *A, const void *B, void *C,
             const void *bias, const void *R, void *, size_t, hipStream_t s) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * K);
    if (layout == 0)
        launch_layout<false, false>(M, N, K, A, K, B, K, C, N, bias, R, N, s);
    else if (layout == 1)
        launch_layout<false, true>(M, N, K, A, K, B, N, C, N, bias, R, N, s);
    else
        launch_layout<true, true>(M, N, K, A, M, B, N, C, N, bias, R, N, s);
    return check_launch("gemm");
}

}  // namespace ob
