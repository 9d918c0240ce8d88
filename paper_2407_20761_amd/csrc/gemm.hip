// bf16 MFMA GEMM for gfx950 (steps a2, a5, a7, a9 and their dgrad / wgrad counterparts).
//
//   C[M,N] = op(A) * op(B) (+ bias[N]) (+ R[M,N])      bf16 in, fp32 accumulate, bf16 out
//   "NT" A[M,K] B[N,K] (forward)   "NN" A[M,K] B[K,N] (dgrad)   "TN" A[K,M] B[K,N] (wgrad, K = tokens)
//
// One workgroup (4 wavefronts, each a 128x128 block of 8x8 MFMA 16x16x32 tiles, 256 accumulator
// registers) owns a 256x256 tile of C and walks K in steps of 64 over two LDS stages.  The 16x16x32
// shape reads and writes half the accumulator registers per FLOP of the 32x32x16 one; under
// sustained load the chip is power-limited, and a register-fed loop of it sustains 2010 against
// 1725-1790 TFLOP/s on random data.
//
// Tiles go global -> registers -> LDS: every wave issues one 16-byte-per-lane buffer load per run of
// 8 MFMAs, all K step long, and writes each vector to LDS one whole K step after it was requested,
// so the memory pipeline sees a steady stream (a burst of a K step's loads blocks the wave's
// instruction issue, MFMAs included, until the cache has taken them) and no wait ever meets a
// load in flight.  The hardware range check of the buffer descriptor turns every access past the end
// of an operand into zeros: whole rows beyond M / N of a K-contiguous operand, the ragged token tail
// of K and K steps past the last.  (Columns beyond M / N of a K-major operand wrap into its next row
// instead; they only feed outputs beyond M / N, which are never stored.)  A K-contiguous operand
// is staged as [row][64 k] and a fragment is one 16-byte LDS read; a K-major operand is staged as
// it lies in memory, [k][rows], and the fragment comes out of two transposing LDS reads, so dgrad
// and wgrad need no re-layout pass.  16-byte chunks are XOR-swizzled on the way in (the global
// address of each lane's chunk is free to choose) so that LDS reads are bank-conflict free.
// The weight-side rows are the MFMA's first operand, so a lane's accumulators are runs of four
// consecutive output columns; the epilogue transposes them through LDS into full-row stores.
#include <algorithm>
#include <cmath>

#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

#define OB_LDS __attribute__((address_space(3)))

constexpr int BK = 64;           // k per LDS stage: 8 chunks of 16 bytes = 128 bytes per row
constexpr int ROW_BYTES = BK * 2;

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous range of the `count`
// work items that the workgroups [first, first + count) of a launch stand for (first % 8 == 0).
__device__ __forceinline__ int xcd_chunk(int pid, int count, bool interleave) {
    const int per = count >> 3, rem = count & 7;
    const int xcd = pid & 7, loc = pid >> 3;
    // interleave: blocks of 32 consecutive items (what one XCD holds at a time) are dealt round-robin
    // to the XCDs instead, so that at any time the 8 XCDs work on neighbouring blocks
    if (interleave && (count & 255) == 0) return (((loc >> 5) << 3) + xcd) * 32 + (loc & 31);
    return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + loc;
}
// contractions at least this long deal their patches round-robin to the XCDs (measured: shorter ones
// lose up to 1.8 %, longer ones gain 2.4 - 3.5 %)
constexpr int INTERLEAVE_MIN_K = 8192;
// tile id -> (tile_m, tile_n): ids walk groups of GM tile-rows column by column, so the tiles
// resident on one XCD at a time share A and B panels in that XCD's L2.
__device__ __forceinline__ void tile_of_id(int tile, int tiles_m, int tiles_n, int &tm, int &tn) {
    constexpr int GM = 8;
    const int width = GM * tiles_n;
    const int group = tile / width;
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = tile - group * width;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
}

// The tiles [n_full, n_full + n_tail) of a GEMM, those of an incomplete last round, have their
// contraction cut into `splits` slices of k_chunk K steps; a slice leaves the fp32 sums of its
// BM x BN tile at part[slice][tile - n_full] and tail_sum_kernel adds the slices.
struct TailSplit {
    float *part;          // null: no tile is split
    int n_full, n_tail, splits, k_chunk;
};

template <int BM, int BN, int WM, int WN>
struct Cfg {
    static constexpr int NW = WM * WN;
    static constexpr int T = BM / WM / 16;        // 16x16 MFMA tiles per wave, each way
    static constexpr int A_LD = BM / 8 / NW, B_LD = BN / 8 / NW;
    static constexpr int G = A_LD + B_LD;         // copy groups of one wave per K step
    static constexpr int STAGE = (BM + BN) * ROW_BYTES;
    static_assert(BM / WM == BN / WN, "square wave tiles");
    static_assert(G == 2 * T, "one copy group per run of T MFMAs");
};

// One operand's tile in LDS, in one of two layouts; a fragment of the 16x16x32 MFMA is 16 x-values by
// 32 k, lane l holding x = l % 16, k = 8 (l / 16) .. +7.
//
// KMAJOR = false: the source is [X, K] with k contiguous.  LDS holds [x][8 chunks of 16 B], chunks
//   swizzled by row (see row_swizzle).  A fragment is one 16-byte read per lane.
// KMAJOR = true: the source is [K, X] with x contiguous.  LDS holds [k][X / 8 chunks of 16 B]
//   (8 x-values per chunk); the chunk at physical position p of row k is logical chunk
//   p ^ 4 (k & 3) ^ 2 ((k >> 3 ^ k >> 4) & 1).  A fragment is two transposing 8-byte reads
//   (ds_read_b64_tr_b16): inside a group of 16 lanes, lane 4 k' + c addresses the 4 x-values
//   [4c, 4c + 4) of row k' of a 4 x 16 block, and lane p receives column p, i.e. 4 consecutive k of
//   one x.  The four groups of a read sit at k, k + 8, k + 16, k + 24 over the same x; the second
//   swizzle term puts any two of them that could be served together 32 bytes apart.
template <int X, int NW, int T, bool KMAJOR>
struct Operand {
    static constexpr int LD = X / 8 / NW;
    static constexpr int ROWB = X * 2;
    const unsigned char *base;
    long left;                                   // bytes from `base` to the end of the source
    uint32_t step;                               // bytes per K step
    uint32_t voff[LD];
    int rd[KMAJOR ? T : BK / 32];                // LDS read offsets: per tile i (k-major) / per k-step u

    // k-contiguous layout: the chunk at physical position p of row x is logical chunk
    // p ^ row_swizzle(x).  The LDS serves a 16-byte read 16 lanes at a time (measured with a probe
    // of lane pairs): within each half of the wavefront, first the lanes whose index bits 2, 3, 4 have
    // even parity, then the others.  For these fragments such a group is all 16 rows, the rows with
    // bit 2 ^ bit 3 = 0 at chunk c and the others at c ^ 1 (or the other way round); rows alternate
    // between the two 128-byte halves of the banks, so among the 8 rows of one parity
    // swizzle(x) ^ bit 2 ^ bit 3 has to take 8 different values.
    static __device__ __forceinline__ int row_swizzle(int x) { return (x >> 1) & 7; }

    // ld = source leading dimension (elements); x0 = first tile row; total_bytes = size of the
    // source; wave_x0 = first x-value of this wave's part of the tile
    __device__ __forceinline__ void init(const __bf16 *src, int ld, int x0, long total_bytes, int wave,
                                         int lane, int wave_x0) {
        if (!KMAJOR) {
            base = (const unsigned char *)(src + (size_t)x0 * ld);
            left = total_bytes - (long)x0 * ld * 2;
            step = ROW_BYTES;
#pragma unroll
            for (int p = 0; p < LD; ++p) {
                const int blk = wave * LD + p, row = blk * 8 + (lane >> 3);
                const int ch = (lane & 7) ^ row_swizzle(row);
                voff[p] = ((uint32_t)row * (uint32_t)ld + ch * 8) * 2u;
            }
            const int lx = lane & 15, lq = lane >> 4;
            const int f = row_swizzle(lx);
#pragma unroll
            for (int u = 0; u < BK / 32; ++u) rd[u] = (wave_x0 + lx) * ROW_BYTES + (((4 * u + lq) ^ f) * 16);
        } else {
            base = (const unsigned char *)(src + x0);
            left = total_bytes - (long)x0 * 2;
            step = (uint32_t)BK * (uint32_t)ld * 2u;
            constexpr int KPB = 1024 / ROWB, CPR = ROWB / 16;
#pragma unroll
            for (int p = 0; p < LD; ++p) {
                const int blk = wave * LD + p, k = blk * KPB + lane / CPR;
                const int ch = (lane % CPR) ^ (4 * (k & 3)) ^ (2 * (((k >> 3) ^ (k >> 4)) & 1));
                voff[p] = ((uint32_t)k * (uint32_t)ld + ch * 8) * 2u;
            }
            // group b of 16 lanes reads k = 8 b + (0..3) (and + 4 with the second read); inside the
            // group lane 4 kq + c addresses x-values [4c, 4c + 4) of row kq
            const int b = lane >> 4, q = lane & 15, kq = q >> 2, c = q & 3;
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const int chunk = (wave_x0 + 16 * i) / 8 + (c >> 1);
                rd[i] = (8 * b + kq) * ROWB + ((chunk ^ (4 * kq) ^ (2 * ((b ^ (b >> 1)) & 1))) * 16) + (c & 1) * 8;
            }
        }
    }
    __device__ __forceinline__ void advance() {
        base += step;
        left -= step;
    }
    // start the contraction `steps` K steps into the source
    __device__ __forceinline__ void skip(int steps) {
        base += (long)steps * step;
        left -= (long)steps * step;
    }
    // descriptor of the current K step; must sit in scalar registers: pin its (uniform) parts explicitly
    // (live = false: an empty range, every load returns zeros without touching memory)
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t descriptor(bool live) const {
        const uint64_t b = (uint64_t)base;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
        // the range a descriptor can check is 32 bits wide: a source with more than 4 GB left is
        // clamped (no access of a K step reaches that far from `base`), one past its end is empty
        const long cl = left < 0 ? 0 : (left > 0xFFFFFFFFl ? 0xFFFFFFFFl : left);
        return __builtin_amdgcn_make_buffer_rsrc((void *)(((uint64_t)hi << 32) | lo), 0,
                                                 live ? (int)__builtin_amdgcn_readfirstlane((uint32_t)cl) : 0, 0x00020000);
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
    // fragment for MFMA tile i (16 x-values) at k-step u (32 k)
    __device__ __forceinline__ bf16x8 frag(const unsigned char OB_LDS *__restrict__ tile, int i, int u) const {
        if (!KMAJOR) {
            return *(const bf16x8 OB_LDS *)(tile + rd[u] + i * 16 * ROW_BYTES);
        } else {
#if defined(__HIP_DEVICE_COMPILE__)
            typedef __attribute__((ext_vector_type(4))) short s16x4;
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 OB_LDS *)(tile + rd[i] + (32 * u) * ROWB));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 OB_LDS *)(tile + rd[i] + (32 * u + 4) * ROWB));
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
#else
            return bf16x8{};
#endif
        }
    }
};

// acc += first x second, in place in the accumulation registers.  Written as an instruction: the
// builtin's destination is not tied to its addend for this shape, and the register allocator then
// moves accumulators around the loop.
__device__ __forceinline__ void mfma(f32x4 &acc, bf16x8 first, bf16x8 second) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(first), "v"(second));
}

// State of one wave in the K loop.  A K step (64 k, one LDS stage) is two k-steps of T runs; run g
// multiplies A fragment g with all T B fragments, and carries one copy group (deliver the vector
// requested one K step ago, request the same piece of the K step after) between its MFMAs and two
// or three fragment reads for the next k-step in front of them: the next B fragments into the
// other B set, the next A fragment g - 1 into the register run g - 1 has just finished with.
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
struct KLoop {
    using C = Cfg<BM, BN, WM, WN>;
    static constexpr int T = C::T;
    Operand<BM, C::NW, T, AK> opa;
    Operand<BN, C::NW, T, BKM> opb;
    u32x4 v[C::G];
    __amdgpu_buffer_rsrc_t ra, rb;
    int k_left;
    int wave, lane;
    bf16x8 af[T], bfr[2][T];

    __device__ __forceinline__ void next_k() {
        const bool live = k_left > 0;
        --k_left;
        ra = opa.descriptor(live);
        rb = opb.descriptor(live);
        opa.advance();
        opb.advance();
    }
    __device__ __forceinline__ void request(int g) {
        v[g] = g < C::A_LD ? opa.load(ra, g) : opb.load(rb, g - C::A_LD);
    }
    __device__ __forceinline__ void deliver(unsigned char OB_LDS *__restrict__ dst, int g) const {
        if (g < C::A_LD) opa.store(dst, wave, lane, g, v[g]);
        else opb.store(dst + BM * ROW_BYTES, wave, lane, g - C::A_LD, v[g]);
    }
    __device__ __forceinline__ bf16x8 a_frag(const unsigned char OB_LDS *__restrict__ stage, int i, int u) const {
        return opa.frag(stage, i, u);
    }
    __device__ __forceinline__ bf16x8 b_frag(const unsigned char OB_LDS *__restrict__ stage, int j, int u) const {
        return opb.frag(stage + BM * ROW_BYTES, j, u);
    }
    // The fragment reads that run g carries.  KIND 0: none.  1: first k-step, reading the second
    // one of the same stage.  2: run 0 of the second k-step (its own last A fragment; the barrier
    // follows).  3: second k-step, reading the first one of the next stage (one B read more in run 1,
    // which makes up for run 0).
    template <int KIND>
    __device__ __forceinline__ void read_b(const unsigned char OB_LDS *__restrict__ src, int g) {
        if (KIND == 1) bfr[1][g] = b_frag(src, g, 1);
        if (KIND == 3) bfr[0][g] = b_frag(src, g, 0);
    }
    template <int KIND>
    __device__ __forceinline__ void read_a(const unsigned char OB_LDS *__restrict__ src, int g) {
        if (KIND == 1) {
            if (g == 0) af[T - 1] = a_frag(src, T - 1, 0);
            else af[g - 1] = a_frag(src, g - 1, 1);
        }
        if (KIND == 2) af[T - 1] = a_frag(src, T - 1, 1);
        if (KIND == 3) af[g - 1] = a_frag(src, g - 1, 0);
    }
    template <int KIND>
    __device__ __forceinline__ void read_extra(const unsigned char OB_LDS *__restrict__ src, int g) {
        if (KIND == 3 && g == 1) bfr[0][0] = b_frag(src, 0, 0);
    }
    // Run g: the T MFMAs of A fragment g with B set `set`, and between them, never more than one
    // memory instruction between two MFMAs (a 16x16x32 MFMA keeps the pipe busy for four issue slots
    // of a lone wave, and whatever sits between two of them beyond three slots is lost): the run's
    // fragment reads, then the delivery of copy group `grp` to `fill` (well behind the reads: an LDS
    // write right after LDS reads stalls), then its next request (COPY = false: no copy group).
    template <int KIND, bool COPY>
    __device__ __forceinline__ void run(f32x4 (&acc)[T][T], int g, int set, const unsigned char OB_LDS *__restrict__ src,
                                        unsigned char OB_LDS *__restrict__ fill, int grp) {
        constexpr int AT_RB = 0, AT_RA = 1, AT_RX = T >= 8 ? 2 : 1, AT_DL = T / 2, AT_RQ = T >= 8 ? T / 2 + 2 : T - 1;
#pragma unroll
        for (int j = 0; j < T; ++j) {
            mfma(acc[g][j], bfr[set][j], af[g]);
            __builtin_amdgcn_sched_barrier(0);
            if (j == AT_RB) read_b<KIND>(src, g);
            if (j == AT_RA) read_a<KIND>(src, g);
            if (j == AT_RX) read_extra<KIND>(src, g);
            if (COPY && j == AT_DL) deliver(fill, grp);
            if (COPY && j == AT_RQ) request(grp);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // One K step out of stage `cur`.  On entry bfr[0] and af[0 .. T-2] hold the fragments of its
    // first k-step.  NEXT: stage `nxt` holds (after the barrier) the K step behind, and on return
    // the registers hold that one's first fragments; the copy groups in front of the barrier go
    // to `nxt`, those behind it to `cur`, which by then nobody reads.
    template <bool NEXT>
    __device__ __forceinline__ void stage(f32x4 (&acc)[T][T], unsigned char OB_LDS *__restrict__ cur,
                                          unsigned char OB_LDS *__restrict__ nxt) {
#pragma unroll
        for (int g = 0; g < T; ++g) run<1, true>(acc, g, 0, cur, nxt, g);   // k-step 0
        run<2, true>(acc, 0, 1, cur, nxt, T);
        if (NEXT) {
            next_k();                          // scalar work, kept off the path behind the barrier
            // own LDS traffic done (reads landed, writes in the stage), then the barrier: `nxt` is
            // complete everywhere and nobody reads `cur` any more; buffer loads stay in flight
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __syncthreads();
        }
#pragma unroll
        for (int g = 1; g < T; ++g) run<NEXT ? 3 : 0, NEXT>(acc, g, 1, nxt, cur, T + g);   // rest of k-step 1
    }
};

// One workgroup's work: tile (tile_m, tile_n) of C, whole, or (sliced) K steps [kz k_chunk, ...) of it with
// the fp32 sums left at part[kz][tail_tile].
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__device__ __forceinline__ void gemm_tile(
    int M, int N, int K, const __bf16 *__restrict__ A, int lda, const __bf16 *__restrict__ B,
    int ldb, __bf16 *__restrict__ Cm, int ldc, const __bf16 *__restrict__ bias,
    const __bf16 *R, int ldr, int tile_m, int tile_n, bool sliced, int kz, int tail_tile, const TailSplit &ts) {
    using C = Cfg<BM, BN, WM, WN>;
    constexpr int T = C::T;
    __shared__ __attribute__((aligned(1024))) unsigned char st0[C::STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[C::STAGE];
    const int m0 = __builtin_amdgcn_readfirstlane(tile_m) * BM;
    const int n0 = __builtin_amdgcn_readfirstlane(tile_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    KLoop<BM, BN, WM, WN, AK, BKM> lp;
    lp.wave = wave;
    lp.lane = lane;
    lp.opa.init(A, lda, m0, (AK ? (long)K : (long)M) * lda * 2, wave, lane, wm * (BM / WM));
    lp.opb.init(B, ldb, n0, (BKM ? (long)K : (long)N) * ldb * 2, wave, lane, wn * (BN / WN));

    f32x4 acc[T][T];
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    unsigned char OB_LDS *s0 = (unsigned char OB_LDS *)st0;
    unsigned char OB_LDS *s1 = (unsigned char OB_LDS *)st1;
    // a slice covers K steps [k_first, k_first + nk)
    const int k_first = kz * ts.k_chunk;
    const int nk = sliced ? min(ts.k_chunk, (K + BK - 1) / BK - k_first) : (K + BK - 1) / BK;
    lp.opa.skip(k_first);
    lp.opb.skip(k_first);
    lp.k_left = nk;
    // prologue: K step 0 into stage 0; K step 1 requested, the copy groups that follow a barrier
    // delivered to stage 1 and re-requested for K step 2: the state behind the barrier of a K step
    lp.next_k();
#pragma unroll
    for (int g = 0; g < C::G; ++g) lp.request(g);
#pragma unroll
    for (int g = 0; g < C::G; ++g) lp.deliver(s0, g);
    lp.next_k();
#pragma unroll
    for (int g = 0; g < C::G; ++g) lp.request(g);
    lp.next_k();
#pragma unroll
    for (int g = T + 1; g < C::G; ++g) {
        lp.deliver(s1, g);
        lp.request(g);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < T; ++j) lp.bfr[0][j] = lp.b_frag(s0, j, 0);
#pragma unroll
    for (int i = 0; i < T - 1; ++i) lp.af[i] = lp.a_frag(s0, i, 0);

    // two K steps per trip: a single straight path with immediate stage addresses.  There is no
    // separate tail (several ways into the epilogue make the register allocator move the
    // accumulators between homes): the last K step also reads ahead and copies (fragments that
    // are never used, zeros from past the end of K), and an odd count of K steps is rounded up
    // with a K step of zeros.
    for (int kt = 0; kt < nk; kt += 2) {
        lp.template stage<true>(acc, s0, s1);
        lp.template stage<true>(acc, s1, s0);
    }

    // the MFMAs above are opaque to the compiler's hazard handling: let the last ones retire before
    // the accumulators are read
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");
    // every wave is done reading the last stage and writing the other one; then the stages serve as
    // transposition slabs.  A lane holds, per MFMA tile, output row m = lane % 16 and columns
    // n = 4 (lane / 16) + (0..3): stored directly, every lane of a store would touch a different
    // cache line.  Each wave writes two tile rows (32 output rows) to its slab as fp32 and reads
    // them back so that 16 (or 8) consecutive lanes cover one contiguous row segment; bias and
    // residual are added on the way out, then one rounding to bf16.
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads();
    constexpr int CW = BN / WN;            // columns of the wave's tile
    constexpr int RSTR = CW * 4 + 16;      // fp32 row stride in LDS, padded against bank conflicts
    constexpr int LPR = CW / 8;            // lanes per row on the way out (8 columns each)
    constexpr int RPI = 64 / LPR;          // rows per read instruction
    static_assert(32 * RSTR <= C::STAGE / (C::NW / 2), "slab does not fit the wave's LDS share");
    unsigned char OB_LDS *slab = (wave < C::NW / 2 ? s0 : s1) + (wave % (C::NW / 2)) * (C::STAGE / (C::NW / 2));
    const int lx = lane & 15, lq = lane >> 4;
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
    for (int ii = 0; ii < T / 2; ++ii) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < T; ++j)
                *(f32x4 OB_LDS *)(slab + (16 * h + lx) * RSTR + (j * 16 + lq * 4) * 4) = acc[2 * ii + h][j];
#pragma unroll
        for (int r = 0; r < 32 / RPI; ++r) {
            const int row = r * RPI + lane / LPR;
            const f32x4 lo = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32);
            const f32x4 hi = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32 + 16);
            const int m = m0 + wm * (BM / WM) + ii * 32 + row;
            if (sliced) {   // the whole tile; sums beyond M and N are never read by tail_sum_kernel
                float *dst = ts.part + ((size_t)(kz * ts.n_tail + tail_tile) * BM + (m - m0)) * BN + (n_out - n0);
                *(f32x4 *)dst = lo;
                *(f32x4 *)(dst + 4) = hi;
            } else if (m < M && n_out < N) {
                float o8[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) { o8[e] = lo[e] + bv[e]; o8[4 + e] = hi[e] + bv[4 + e]; }
                if (R) {
                    const bf16x8 r8 = *(const bf16x8 *)(R + (size_t)m * ldr + n_out);
#pragma unroll
                    for (int e = 0; e < 8; ++e) o8[e] += (float)r8[e];
                }
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (__bf16)o8[e];
                __builtin_nontemporal_store(o, (bf16x8 *)(Cm + (size_t)m * ldc + n_out));
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(
    int M, int N, int K, const __bf16 *__restrict__ A, int lda, const __bf16 *__restrict__ B,
    int ldb, __bf16 *__restrict__ Cm, int ldc, const __bf16 *__restrict__ bias,
    const __bf16 *R, int ldr, int tiles_m, int tiles_n, TailSplit ts) {
    // workgroups [0, n_full): whole tiles; then slice after slice of the tail tiles
    const int pid = blockIdx.x, n_whole = ts.part ? ts.n_full : (int)gridDim.x;
    const bool sliced = pid >= n_whole;
    const int kz = sliced ? (pid - n_whole) / ts.n_tail : 0;
    const bool interleave = K >= INTERLEAVE_MIN_K;
    const int tail_tile = sliced ? xcd_chunk((pid - n_whole) % ts.n_tail, ts.n_tail, interleave) : 0;
    int tile_m, tile_n;
    tile_of_id(sliced ? n_whole + tail_tile : xcd_chunk(pid, n_whole, interleave), tiles_m, tiles_n, tile_m, tile_n);
    gemm_tile<BM, BN, WM, WN, AK, BKM>(M, N, K, A, lda, B, ldb, Cm, ldc, bias, R, ldr, tile_m, tile_n, sliced, kz,
                                       tail_tile, ts);
}

// Several GEMMs of one layout over the same contraction length K in ONE launch (the weight gradients of a
// block: K = tokens).  Their tiles are numbered one GEMM after the other and dealt to the chip as one list,
// so the chip sees one incomplete last round (cut into slices as for a single GEMM) instead of one per GEMM:
// for a narrow model every weight gradient alone is less than a round of tiles.
struct GemmGroup {
    static constexpr int MAX = 4;
    int n;
    int first[MAX + 1];   // first[p]: number of the first tile of GEMM p; first[n]: all tiles
    int M[MAX], N[MAX], lda[MAX], ldb[MAX], ldc[MAX], ldr[MAX], tiles_m[MAX], tiles_n[MAX];
    const __bf16 *A[MAX], *B[MAX], *R[MAX];
    __bf16 *C[MAX];
};
__device__ __forceinline__ int group_member(const GemmGroup &g, int tile) {
    int p = 0;
#pragma unroll
    for (int i = 1; i < GemmGroup::MAX; ++i) p += (i < g.n && tile >= g.first[i]) ? 1 : 0;
    return __builtin_amdgcn_readfirstlane(p);
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM * WN * 64) void gemm_group_kernel(GemmGroup g, int K, TailSplit ts) {
    const int pid = blockIdx.x, n_whole = ts.part ? ts.n_full : (int)gridDim.x;
    const bool sliced = pid >= n_whole;
    const int kz = sliced ? (pid - n_whole) / ts.n_tail : 0;
    const bool interleave = K >= INTERLEAVE_MIN_K;
    const int tail_tile = sliced ? xcd_chunk((pid - n_whole) % ts.n_tail, ts.n_tail, interleave) : 0;
    const int tile = sliced ? n_whole + tail_tile : xcd_chunk(pid, n_whole, interleave);
    const int p = group_member(g, tile);
    int tile_m, tile_n;
    tile_of_id(tile - g.first[p], g.tiles_m[p], g.tiles_n[p], tile_m, tile_n);
    gemm_tile<BM, BN, WM, WN, AK, BKM>(g.M[p], g.N[p], K, g.A[p], g.lda[p], g.B[p], g.ldb[p], g.C[p], g.ldc[p], nullptr,
                                       g.R[p], g.ldr[p], tile_m, tile_n, sliced, kz, tail_tile, ts);
}
template __global__ void gemm_group_kernel<256, 256, 2, 2, true, true>(GemmGroup, int, TailSplit);

#define OB_GEMM_INSTANCE(BM, BN, AK, BKM)                                                        \
    template __global__ void gemm_kernel<BM, BN, 2, 2, AK, BKM>(                                 \
        int, int, int, const __bf16 *, int, const __bf16 *, int, __bf16 *, int, const __bf16 *,    \
        const __bf16 *, int, int, int, TailSplit);
OB_GEMM_INSTANCE(256, 256, false, false)
OB_GEMM_INSTANCE(128, 128, false, false)
OB_GEMM_INSTANCE(256, 256, false, true)
OB_GEMM_INSTANCE(128, 128, false, true)
OB_GEMM_INSTANCE(256, 256, true, true)
OB_GEMM_INSTANCE(128, 128, true, true)
#undef OB_GEMM_INSTANCE

// C = sum over the slices of the tail tiles' fp32 sums (+ bias) (+ R); 8 outputs per lane, slices
// added in order
template <int BM, int BN>
__global__ __launch_bounds__(256) void tail_sum_kernel(TailSplit ts, int M, int N, int tiles_m, int tiles_n,
                                                       const __bf16 *__restrict__ bias, const __bf16 *R, int ldr,
                                                       __bf16 *__restrict__ Cm, int ldc) {
    constexpr int PER_TILE = BM * BN / 8 / 256;      // workgroups per tile
    const int t = blockIdx.x / PER_TILE;
    const int e = ((blockIdx.x % PER_TILE) * 256 + threadIdx.x) * 8;
    int tile_m, tile_n;
    tile_of_id(ts.n_full + t, tiles_m, tiles_n, tile_m, tile_n);
    const int m = tile_m * BM + e / BN, n = tile_n * BN + e % BN;
    if (m >= M || n >= N) return;
    const float *src = ts.part + (size_t)t * (BM * BN) + e;
    const size_t slice = (size_t)ts.n_tail * (BM * BN);
    f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
    for (int z = 1; z < ts.splits; ++z) {
        lo += *(const f32x4 *)(src + z * slice);
        hi += *(const f32x4 *)(src + z * slice + 4);
    }
    float o8[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { o8[i] = lo[i]; o8[4 + i] = hi[i]; }
    if (bias) {
        const bf16x8 b8 = *(const bf16x8 *)(bias + n);
#pragma unroll
        for (int i = 0; i < 8; ++i) o8[i] += (float)b8[i];
    }
    if (R) {
        const bf16x8 r8 = *(const bf16x8 *)(R + (size_t)m * ldr + n);
#pragma unroll
        for (int i = 0; i < 8; ++i) o8[i] += (float)r8[i];
    }
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)o8[i];
    *(bf16x8 *)(Cm + (size_t)m * ldc + n) = o;
}

// the same for the tail tiles of a group of GEMMs
template <int BM, int BN>
__global__ __launch_bounds__(256) void tail_sum_group_kernel(TailSplit ts, GemmGroup g) {
    constexpr int PER_TILE = BM * BN / 8 / 256;
    const int t = blockIdx.x / PER_TILE;
    const int e = ((blockIdx.x % PER_TILE) * 256 + threadIdx.x) * 8;
    const int tile = ts.n_full + t;
    const int p = group_member(g, tile);
    int tile_m, tile_n;
    tile_of_id(tile - g.first[p], g.tiles_m[p], g.tiles_n[p], tile_m, tile_n);
    const int m = tile_m * BM + e / BN, n = tile_n * BN + e % BN;
    if (m >= g.M[p] || n >= g.N[p]) return;
    const float *src = ts.part + (size_t)t * (BM * BN) + e;
    const size_t slice = (size_t)ts.n_tail * (BM * BN);
    f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
    for (int z = 1; z < ts.splits; ++z) {
        lo += *(const f32x4 *)(src + z * slice);
        hi += *(const f32x4 *)(src + z * slice + 4);
    }
    float o8[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { o8[i] = lo[i]; o8[4 + i] = hi[i]; }
    const __bf16 *R = g.R[p];
    if (R) {
        const bf16x8 r8 = *(const bf16x8 *)(R + (size_t)m * g.ldr[p] + n);
#pragma unroll
        for (int i = 0; i < 8; ++i) o8[i] += (float)r8[i];
    }
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)o8[i];
    *(bf16x8 *)(g.C[p] + (size_t)m * g.ldc[p] + n) = o;
}

// How a GEMM is cut into workgroups: tile size, and which tiles have their contraction split.
struct Plan {
    bool big;
    int n_full, n_tail, splits, k_chunk;   // splits == 1: every tile whole
    size_t part_bytes() const { return splits > 1 ? (size_t)splits * n_tail * (big ? 256 * 256 : 128 * 128) * 4 : 0; }
};

// 256x256 tiles run one workgroup per CU, 128x128 tiles two.  Both the tile size and the split are
// chosen by an estimate of the launch's duration in microseconds, fitted to launches measured on a
// mostly idle chip:
//  * big tiles come in rounds of one per CU, and the tiles of an incomplete last round take as long
//    as a full one (over 16325 tokens: 4096 x 12288, 3 rounds, 1409 TFLOP/s; 4096 x 14336, 3.5
//    rounds, 1178; 4096 x 5120, 1.25 rounds, 1008); a K step takes 1.3, prologue and epilogue as
//    much as 5 more (nothing else runs on the CU meanwhile);
//  * a small tile with a CU to itself takes 0.47 per K step (+3); two to a CU 0.9 each (about 0.72
//    of a big tile's rate: twice the fragment reads per MFMA), but the one's epilogue hides behind the
//    other's K loop (+1) and, out of step as they are, they fill the last round gradually (0.4 of a
//    round on top of tiles / 512).  Measured: 12300 x 4096 x 1024 (3.06 rounds of big tiles) 109
//    against 118; 12300 x 1024 x 4096 (0.77 rounds) 112 against 86; 6144 x 4096 x 16325 808 against 712;
//  * when the caller has room for fp32 sums (`can_split`), the contraction of the tiles of the last
//    round can be cut into as many slices as fill the round, each slice a workgroup with a shorter K
//    loop; a second kernel adds the slices.  A GEMM of less than one round (the hidden x hidden
//    weight gradients of a narrow model over all tokens of the batch) is all tail.  The sums cost 4
//    bytes per element and slice at 4 TB/s (measured: 14 us for 64 MiB) and 3 for the second launch;
//    a split has to promise 7 %.
// compute units of the current device, asked once (256 on MI355X, also when no device answers: the
// size queries must work on a host without a GPU)
int compute_units() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        (void)hipGetLastError();
        return n;
    }();
    return cus;
}

double estimate_us(bool big, int nk, double n_full, double n_tail, int splits, int k_chunk) {
    const double area = big ? 65536.0 : 16384.0;
    const double sums = splits > 1 ? splits * n_tail * area * 4.0 / 4e6 + 3.0 : 0.0;
    const int k_tail = splits > 1 ? k_chunk : nk;
    const double cus = compute_units(), slots2 = 2.0 * cus;
    if (big) return n_full / cus * (nk + 5) * 1.3 + ceil(n_tail * splits / cus) * (k_tail + 5) * 1.3 + sums;
    if (n_full == 0 && n_tail * splits <= cus) return (k_tail + 3) * 0.47 + sums;
    if (splits == 1) return ((n_full + n_tail) / slots2 + 0.4) * (nk + 1) * 0.9;
    return n_full / slots2 * (nk + 1) * 0.9 + ceil(n_tail * splits / slots2) * (k_tail + 1) * 0.9 + sums;
}

Plan make_plan(int M, int N, int K, bool can_split) {
    const int big = ((M + 255) / 256) * ((N + 255) / 256);
    const int small = ((M + 127) / 128) * ((N + 127) / 128);
    const int nk = (K + BK - 1) / BK;
    const double t_big = estimate_us(true, nk, 0, big, 1, 0), t_small = estimate_us(false, nk, 0, small, 1, 0);
    const bool use_big = t_big <= t_small;
    Plan p{use_big, use_big ? big : small, 0, 1, 0};
    if (can_split && nk >= 16) {
        double best = 0.93 * (use_big ? t_big : t_small);
        for (int tile_big = 0; tile_big < 2; ++tile_big) {
            const int tiles = tile_big ? big : small, slots = (tile_big ? 1 : 2) * compute_units();
            const int n_tail = tiles % slots, n_full = tiles - n_tail;
            if (n_tail == 0) continue;
            for (int z = 2; z <= 8 && nk / z >= 8; ++z) {
                const int chunk = ((nk + z - 1) / z + 1) & ~1;       // whole trips of the two-step loop
                const int slices = (nk + chunk - 1) / chunk;         // every slice has at least one K step
                if (slices < 2) continue;
                const double t = estimate_us(tile_big, nk, n_full, n_tail, slices, chunk);
                if (t < best) { best = t; p = Plan{tile_big != 0, n_full, n_tail, slices, chunk}; }
            }
        }
    }
    return p;
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
void launch_tile(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
                 const void *bias, const void *R, int ldr, float *part, const Plan &p, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const TailSplit ts{p.splits > 1 ? part : nullptr, p.n_full, p.n_tail, p.splits, p.k_chunk};
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, AK, BKM>), dim3(p.n_full + p.n_tail * p.splits),
                       dim3(WM * WN * 64), 0, s, M, N, K, (const __bf16 *)A, lda, (const __bf16 *)B, ldb,
                       (__bf16 *)C, ldc, (const __bf16 *)bias, (const __bf16 *)R, ldr, tiles_m, tiles_n, ts);
    if (p.splits > 1)
        hipLaunchKernelGGL((tail_sum_kernel<BM, BN>), dim3(p.n_tail * (BM * BN / 8 / 256)), dim3(256), 0, s, ts, M, N,
                           tiles_m, tiles_n, (const __bf16 *)bias, (const __bf16 *)R, ldr, (__bf16 *)C, ldc);
}

// `part` (may be null: nothing is split) has room for the plan's fp32 sums
template <bool AK, bool BKM>
void launch_layout(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
                   const void *bias, const void *R, int ldr, float *part, hipStream_t s) {
    const Plan p = make_plan(M, N, K, part != nullptr);
    if (p.big)
        launch_tile<256, 256, 2, 2, AK, BKM>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, part, p, s);
    else
        launch_tile<128, 128, 2, 2, AK, BKM>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, part, p, s);
}

// A group of "TN" GEMMs over one K, 256 x 256 tiles: the whole tiles of the full rounds of the combined
// list, then the slices of its tail (same rule and estimate as for a single GEMM).
Plan make_group_plan(int total_tiles, int K) {
    const int nk = (K + BK - 1) / BK, slots = compute_units();
    const int n_tail = total_tiles % slots, n_full = total_tiles - n_tail;
    Plan p{true, total_tiles, 0, 1, 0};
    if (n_tail == 0 || nk < 16) return p;
    double best = 0.93 * estimate_us(true, nk, 0, total_tiles, 1, 0);
    for (int z = 2; z <= 8 && nk / z >= 8; ++z) {
        const int chunk = ((nk + z - 1) / z + 1) & ~1;
        const int slices = (nk + chunk - 1) / chunk;
        if (slices < 2) continue;
        const double t = estimate_us(true, nk, n_full, n_tail, slices, chunk);
        if (t < best) { best = t; p = Plan{true, n_full, n_tail, slices, chunk}; }
    }
    return p;
}

}  // namespace

// fp32 sums of the slices of the tiles whose contraction is split; 0 for a GEMM without such tiles
size_t gemm_workspace_bytes(int, int M, int N, int K) { return make_plan(M, N, K, true).part_bytes(); }

// ws (may be null): gemm_workspace_bytes(0, M, N, K) bytes
void launch_gemm_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C,
                    int ldc, const void *bias, const void *R, int ldr, hipStream_t s, int k_algo, void *ws) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * (k_algo > 0 ? k_algo : K));
    launch_layout<false, false>(M, N, K, A, lda, B, ldb, C, ldc, bias, R, ldr, (float *)ws, s);
}

// The weight gradients of a block in one launch: C_p[M_p, N_p] = A_p[K, M_p]^T B_p[K, N_p] (+ R_p), p < count
// <= 4, all over the same K.  Worth it when the GEMMs' own last rounds of tiles are a sizeable part of them:
// the estimate (as for single GEMMs) has to promise 10 % (measured: the 300M-class ViT's four weight
// gradients, 192 tiles in all, 38.0 -> 35.3 ms per 24-block step; the 6B-class ViT's, where it promises
// 5 %, lose 0.4 %); otherwise, or without scratch, they are launched one by one.
size_t gemm_tn_group_workspace_bytes(int count, const GemmTN *g, int K) {
    int total = 0;
    size_t single = 0;
    for (int i = 0; i < count; ++i) {
        total += ((g[i].M + 255) / 256) * ((g[i].N + 255) / 256);
        const size_t b = gemm_workspace_bytes(2, g[i].M, g[i].N, K);
        if (b > single) single = b;
    }
    const size_t grouped = make_group_plan(total, K).part_bytes();
    return grouped > single ? grouped : single;
}

int gemm_tn_group(int count, const GemmTN *g, int K, void *ws, size_t ws_bytes, hipStream_t s) {
    if (count < 1 || count > GemmGroup::MAX) return fail(OB_EINVAL, "gemm group: %d members", count);
    const int nk = (K + BK - 1) / BK;
    GemmGroup grp{};
    grp.n = count;
    double t_single = 0.0, flops = 0.0;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        grp.first[i] = total;
        grp.M[i] = g[i].M; grp.N[i] = g[i].N;
        grp.A[i] = (const __bf16 *)g[i].A; grp.lda[i] = g[i].M;
        grp.B[i] = (const __bf16 *)g[i].B; grp.ldb[i] = g[i].N;
        grp.C[i] = (__bf16 *)g[i].C; grp.ldc[i] = g[i].N;
        grp.R[i] = (const __bf16 *)g[i].R; grp.ldr[i] = g[i].N;
        grp.tiles_m[i] = (g[i].M + 255) / 256; grp.tiles_n[i] = (g[i].N + 255) / 256;
        total += grp.tiles_m[i] * grp.tiles_n[i];
        const Plan p1 = make_plan(g[i].M, g[i].N, K, ws != nullptr);
        const int t1 = p1.n_full + p1.n_tail;
        t_single += estimate_us(p1.big, nk, p1.splits > 1 ? p1.n_full : 0, p1.splits > 1 ? p1.n_tail : t1, p1.splits, p1.k_chunk) + 3.0;
        flops += 2.0 * g[i].M * g[i].N * K;
    }
    for (int i = count; i <= GemmGroup::MAX; ++i) grp.first[i] = total;
    const Plan p = make_group_plan(total, K);
    const double t_group = estimate_us(true, nk, p.splits > 1 ? p.n_full : 0, p.splits > 1 ? p.n_tail : total, p.splits, p.k_chunk);
    if (count == 1 || !ws || ws_bytes < p.part_bytes() || t_group > 0.9 * t_single) {
        for (int i = 0; i < count; ++i)
            if (int rc = gemm_any(2, g[i].M, g[i].N, K, g[i].A, g[i].B, g[i].C, nullptr, g[i].R, ws, ws_bytes, s)) return rc;
        return OB_OK;
    }
    ProfScope prof(K_GEMM, s, flops);
    const TailSplit ts{p.splits > 1 ? (float *)ws : nullptr, p.n_full, p.n_tail, p.splits, p.k_chunk};
    hipLaunchKernelGGL((gemm_group_kernel<256, 256, 2, 2, true, true>), dim3(p.n_full + p.n_tail * p.splits), dim3(256), 0,
                       s, grp, K, ts);
    if (p.splits > 1)
        hipLaunchKernelGGL((tail_sum_group_kernel<256, 256>), dim3(p.n_tail * (256 * 256 / 8 / 256)), dim3(256), 0, s, ts, grp);
    return check_launch("gemm group");
}

// layout 0 ("NT"): A[M,K] B[N,K]; 1 ("NN"): A[M,K] B[K,N]; 2 ("TN"): A[K,M] B[K,N].  All three
// run natively: a K-major operand is staged as it lies in memory and transposed by the LDS read.
// The timed span of a GEMM with split tiles includes the kernel that sums the slices.
int gemm_any(int layout, int M, int N, int K, const void *A, const void *B, void *C,
             const void *bias, const void *R, void *ws, size_t ws_bytes, hipStream_t s) {
    ProfScope prof(K_GEMM, s, 2.0 * M * N * K);
    float *part = ws && ws_bytes >= gemm_workspace_bytes(layout, M, N, K) ? (float *)ws : nullptr;
    if (layout == 0)
        launch_layout<false, false>(M, N, K, A, K, B, K, C, N, bias, R, N, part, s);
    else if (layout == 1)
        launch_layout<false, true>(M, N, K, A, K, B, N, C, N, bias, R, N, part, s);
    else
        launch_layout<true, true>(M, N, K, A, M, B, N, C, N, bias, R, N, part, s);
    return check_launch("gemm");
}

}  // namespace ob
