// bf16 MFMA GEMM for gfx950 (steps a2, a5, a7, a9 and their dgrad / wgrad counterparts).
//
//   C[M,N] = op(A) * op(B) (+ bias[N]) (+ R[M,N])      bf16 in, fp32 accumulate, bf16 out
//   "NT" A[M,K] B[N,K] (forward)   "NN" A[M,K] B[K,N] (dgrad)   "TN" A[K,M] B[K,N] (wgrad, K = tokens)
//
// One workgroup (4 wavefronts, each a 128x128 block of 8x8 MFMA 16x16x32 tiles, 256 accumulator
// registers) owns a 256x256 tile of C and walks K in steps of 32 over a ring of four LDS slots.  The
// 16x16x32 shape reads and writes half the accumulator registers per FLOP of the 32x32x16 one; under
// sustained load the chip is power-limited, and a register-fed loop of it sustains 2010 against
// 1725-1790 TFLOP/s on random data.
//
// A wave has its SIMD to itself, so every instruction that is not an MFMA takes an issue slot that
// only the gaps between MFMAs can hide (three per gap), and what moves data through registers costs
// more than its slot: a 16-byte-per-lane LDS write holds the issue back for as long as its kilobyte
// takes to leave the registers (with both operands staged through registers the loop ran 7 - 12 %
// longer).  Hence
//  * every tile goes global -> LDS directly (buffer loads that write to LDS), one load per run of
//    8 MFMAs, issued one to two slots before its use;
//  * a K-major operand ([k][rows], as it lies in memory: B of "NN", both of "TN") has four slots of 32 k
//    and its fragments come out of transposing LDS reads, so dgrad and wgrad need no re-layout pass;
//  * a K-contiguous operand ([row][k]: A of "NT" and "NN", B of "NT") moves in whole 128-byte rows, two
//    slots at a time (a slot at a time it would fetch every cache line twice); a fragment is one
//    16-byte LDS read.  A has a ring of three such pairs of slots, so its loads have two slots to land;
//    B of "NT" has two (160 KB of LDS hold 96 + 64 KB), its loads go out as soon as the barrier has
//    freed their pair and have a slot and a half;
//  * the descriptor arithmetic of the next slot is a dozen scalar instructions dealt over the gaps of
//    one run (left to the compiler it was some 35 instructions with 64-bit vector compares in one
//    place, 5 % of the loop).
// The hardware range check of the buffer descriptor turns every access past the end of an operand into
// zeros: whole rows beyond M / N of a K-contiguous operand, the ragged token tail of K and slots past
// the last.  (Columns beyond M / N of a K-major operand wrap into its next row instead; they only
// feed outputs beyond M / N, which are never stored.)  16-byte chunks are XOR-swizzled on the way in
// (the global address of each lane's chunk is free to choose) so that LDS reads are bank-conflict free.
// The weight-side rows are the MFMA's first operand, so a lane's accumulators are runs of four
// consecutive output columns; the epilogue transposes them through LDS into full-row stores.
#include <algorithm>
#include <cmath>
#include <type_traits>

#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

#define OB_LDS __attribute__((address_space(3)))

constexpr int BK = 32;           // k per ring slot: 4 chunks of 16 bytes = 64 bytes per row of a K-contiguous operand
constexpr int ROW_BYTES = BK * 2;
constexpr int NS = 4;            // ring slots
constexpr int KSTEP = 64;        // k per "K step", the unit the host's plan counts and slices in (two slots)

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
    static constexpr int SLOT = (BM + BN) * ROW_BYTES;
    static_assert(BM / WM == BN / WN, "square wave tiles");
    static_assert(BM == BN && BM / 16 / NW * 2 == T, "T / 2 pieces of 1 KB per wave, operand and slot");
};

// One operand's part of the ring; a fragment of the 16x16x32 MFMA is 16 x-values by 32 k, lane l
// holding x = l % 16, k = 8 (l / 16) .. +7.
//
// KMAJOR = true: the source is [K, X] with x contiguous.  A slot holds [32 k][X / 8 chunks of 16 B]
//   (8 x-values per chunk) and is filled by buffer loads that write straight to LDS: the 64 lanes
//   of one load deliver 16 bytes each to 1 KB of consecutive LDS addresses (lane i at 16 i), and which
//   16 bytes of global memory a lane asks for is free to choose: the chunk at physical position p
//   of row k is logical chunk p ^ 4 (k & 3) ^ 2 ((k >> 3 ^ k >> 4) & 1).  A fragment is two
//   transposing 8-byte reads (ds_read_b64_tr_b16): inside a group of 16 lanes, lane 4 k' + c
//   addresses the 4 x-values [4c, 4c + 4) of row k' of a 4 x 16 block, and lane p receives column p,
//   i.e. 4 consecutive k of one x.  The four groups of a read sit at k, k + 8, k + 16, k + 24 over
//   the same x; the second swizzle term puts any two of them that could be served together 32 bytes
//   apart.
// KMAJOR = false: the source is [X, K] with k contiguous.  A load that filled 16 rows of one slot would
//   take 64 bytes of each: half a cache line, whose other half the load for the next slot would
//   fetch again once the line has left the first-level cache (measured: a quarter slower than whole
//   lines).  So this operand's slots come in pairs, [x][8 chunks of 16 B] (64 k), the chunk c of row x
//   at position c ^ row_swizzle(x), filled a pair at a time: one load takes 8 rows of 128 bytes and
//   lands lane-linear in a 1 KB piece of LDS (the swizzle is applied by the choice of each lane's
//   global address).  A fragment is one 16-byte read per lane, from the chunks 0-3 (even slot) or
//   4-7 (odd slot).
template <int X, int NW, int T, bool KMAJOR>
struct Operand {
    static constexpr int LD = KMAJOR ? X / 16 / NW : X / 8 / NW;   // loads per wave: per slot / per two slots
    static constexpr int ROWB = X * 2;
    uint64_t base;                               // (uniform) address of the slot / pair of slots to describe next
    long left;                                   // bytes from there to the end of the source (may be negative)
    uint32_t step;                               // bytes from one to the next
    uint32_t num;                                // checked range of the one at hand
    uint32_t voff[LD];
    int rd[KMAJOR ? T : 2];                      // LDS read offsets (from the ring's start): per tile i (k-major) / per slot of the pair

    // k-contiguous layout.  The LDS serves a 16-byte read 16 lanes at a time (measured with a probe
    // of lane pairs): within each half of the wavefront, first the lanes whose index bits 2, 3, 4 have
    // even parity, then the others.  For these fragments such a group is all 16 rows, the rows with
    // bit 2 ^ bit 3 = 0 at chunk c and the others at c ^ 1 (or the other way round); rows alternate
    // between the two 128-byte halves of the banks, so among the 8 rows of one parity
    // swizzle(x) ^ bit 2 ^ bit 3 has to take 8 different values.
    static __device__ __forceinline__ int row_swizzle(int x) { return (x >> 1) & 7; }

    // ld = source leading dimension (elements); x0 = first tile row; total_bytes = size of the
    // source; wave_x0 = first x-value of this wave's part of the tile; region = where in the ring this
    // operand's slots start (part of every per-lane offset, so that what is added per slot, tile and
    // piece fits an instruction's 16-bit offset field)
    __device__ __forceinline__ void init(const __bf16 *src, int ld, int x0, long total_bytes, int wave,
                                         int lane, int wave_x0, int region) {
        if (!KMAJOR) {
            set((const unsigned char *)(src + (size_t)x0 * ld), total_bytes - (long)x0 * ld * 2, 2 * ROW_BYTES, 0);
#pragma unroll
            for (int p = 0; p < LD; ++p) {
                const int row = (wave * LD + p) * 8 + (lane >> 3);
                const int ch = (lane & 7) ^ row_swizzle(row);
                voff[p] = ((uint32_t)row * (uint32_t)ld + ch * 8) * 2u;
            }
            const int lx = lane & 15, lq = lane >> 4;
#pragma unroll
            for (int h = 0; h < 2; ++h) rd[h] = region + (wave_x0 + lx) * 2 * ROW_BYTES + (((4 * h + lq) ^ row_swizzle(lx)) * 16);
        } else {
            set((const unsigned char *)(src + x0), total_bytes - (long)x0 * 2, (uint32_t)BK * (uint32_t)ld * 2u, 0);
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
                rd[i] = region + (8 * b + kq) * ROWB + ((chunk ^ (4 * kq) ^ (2 * ((b ^ (b >> 1)) & 1))) * 16) + (c & 1) * 8;
            }
        }
    }
    // the contraction starts `first` steps into the source (all arguments uniform)
    __device__ __forceinline__ void set(const unsigned char *b, long l, uint32_t step_bytes, int first) {
        base = (uint64_t)b + (uint64_t)first * step_bytes;
        left = l - (long)first * step_bytes;
        step = step_bytes;
    }
    // start the contraction `ksteps` K steps (64 k) into the source
    __device__ __forceinline__ void skip(int ksteps) {
        set((const unsigned char *)base, left, step, KMAJOR ? 2 * ksteps : ksteps);
    }
    // Descriptor of the slot (pair) at hand, then on to the next one, in five steps of two to four scalar
    // instructions (to be placed between different pairs of MFMAs).  The range a descriptor can check is
    // 32 bits wide: a source with more than 4 GB left is clamped (no access of a slot reaches that far
    // from the base), one past its end is empty, and so is any slot when k_left < 1 (every load
    // returns zeros without touching memory).  Written as scalar instructions: the compiler's own
    // 64-bit compares go through the vector unit, a few dozen instructions per slot that a wave alone
    // on its SIMD cannot hide.
    template <int STEP>
    __device__ __forceinline__ void next_step(int k_left, __amdgpu_buffer_rsrc_t &r) {
#if defined(__HIP_DEVICE_COMPILE__)
        if (STEP == 0)
            asm("s_cmp_eq_u32 %2, 0\n\ts_cselect_b32 %0, %1, -1"
                : "=s"(num) : "s"((uint32_t)left), "s"((int32_t)(left >> 32)) : "scc");
        if (STEP == 1)
            asm("s_cmp_lt_i32 %1, 0\n\ts_cselect_b32 %0, 0, %0" : "+s"(num) : "s"((int32_t)(left >> 32)) : "scc");
        if (STEP == 2) asm("s_cmp_gt_i32 %1, 0\n\ts_cselect_b32 %0, %0, 0" : "+s"(num) : "s"(k_left) : "scc");
#endif
        if (STEP == 3) r = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)num, 0x00020000);
        if (STEP == 4) {
            base += step;
            left -= step;
        }
    }
    // k-major: piece p (1 KB per wave) of this wave's share of the slot behind `rsrc`: global -> LDS,
    // lane i to byte 16 i of the piece; lanes past the end of the source (rows beyond K) deliver zeros
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, unsigned char OB_LDS *__restrict__ dst, int wave, int p) const {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void OB_LDS *)(dst + (wave * LD + p) * 1024), 16, voff[p], 0, 0, 0);
    }
    // k-contiguous: piece p (8 rows of 64 k) of this wave's share of the pair of slots behind `rsrc`
    // (rows beyond M / N deliver zeros): global -> the pair at `dst` (this operand's region included)
    __device__ __forceinline__ void load_pair(__amdgpu_buffer_rsrc_t rsrc, unsigned char OB_LDS *__restrict__ dst, int wave, int p) const {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void OB_LDS *)(dst + (wave * LD + p) * 1024), 16, voff[p], 0, 0, 0);
    }
    // fragment for MFMA tile i (16 x-values) out of the slot at `tile` (k-contiguous: slot h of the
    // pair at `tile`)
    __device__ __forceinline__ bf16x8 frag(const unsigned char OB_LDS *__restrict__ tile, int i, int h) const {
        if (!KMAJOR) {
            return *(const bf16x8 OB_LDS *)(tile + rd[h] + i * 16 * 2 * ROW_BYTES);
        } else {
#if defined(__HIP_DEVICE_COMPILE__)
            typedef __attribute__((ext_vector_type(4))) short s16x4;
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 OB_LDS *)(tile + rd[i]));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 OB_LDS *)(tile + rd[i] + 4 * ROWB));
            const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v8);
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

// The bare barrier instruction: __syncthreads() carries a fence as well, which waits for every load
// to LDS still in flight, the ones for the slots further ahead included.  What has to be complete at a
// barrier is said by the s_waitcnt in front of it; the empty statement keeps the compiler from moving
// LDS accesses across.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt operand: at most `vm` vector-memory operations and `lgkm` LDS operations still pending
constexpr int waitcnt(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | 0x70 | (lgkm << 8); }

// State of one wave in the K loop.  The contraction advances one ring slot (32 k) at a time: T runs,
// run g multiplying A fragment g with all T B fragments.  Between its MFMAs a run carries two or
// three fragment reads for the slot after (the next B fragment g into the other B set, the next A
// fragment g - 1 into the register run g - 1 has just finished with) and one step of the refill:
//  * a k-major operand refills, for NS slots ahead, the slot whose last reader has passed the barrier
//    behind run 0: its T / 2 loads go straight to LDS, from run 1 on (A first; with both operands k-major
//    the last load of B falls into run 0 of the slot after);
//  * a k-contiguous operand refills two slots at a time, T loads, straight to LDS as well: between the
//    barrier of an odd slot, when both slots of a pair are free, and the barrier two slots on there
//    are 2 T runs.  A has three pairs: the pair freed last is filled for three K steps further on, so
//    any of those runs will do.  B has two: the pair freed is the one read next but one, so its loads
//    go out in the odd slot's own runs and the barrier two slots on waits for them.
template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
struct KLoop {
    using C = Cfg<BM, BN, WM, WN>;
    static constexpr int T = C::T;
    Operand<BM, C::NW, T, AK> opa;
    Operand<BN, C::NW, T, BKM> opb;
    __amdgpu_buffer_rsrc_t ra, rb, ra_n, rb_n;
    int ka_left, kb_left;                        // slots (k-major) / pairs of slots (k-contiguous) not yet described
    int wave;
    bf16x8 af[T], bfr[2][T];

    // The descriptors of the next slot (pair), ten steps (five per operand, see Operand::next_step); ra_n
    // and rb_n take over behind run 0 of the slot they are for.
    template <int STEP>
    __device__ __forceinline__ void next_step() {
        if (STEP < 5) opa.template next_step<STEP>(ka_left, ra_n);
        else opb.template next_step<STEP - 5>(kb_left, rb_n);
        if (STEP == 4) --ka_left;
        if (STEP == 9) --kb_left;
    }
    __device__ __forceinline__ void prepare_a() {
        next_step<0>();
        next_step<1>();
        next_step<2>();
        next_step<3>();
        next_step<4>();
    }
    __device__ __forceinline__ void prepare_b() {
        next_step<5>();
        next_step<6>();
        next_step<7>();
        next_step<8>();
        next_step<9>();
    }
    __device__ __forceinline__ void next_a() {
        prepare_a();
        ra = ra_n;
    }
    __device__ __forceinline__ void next_b() {
        prepare_b();
        rb = rb_n;
    }
    // The ring holds A's slots, then B's: a k-major operand's NS one after the other, a k-contiguous
    // one's in pairs: B's two, A's three (160 KB of LDS hold 64 + 96 KB).  A's pairs are used in turn,
    // which does not go into the four slots of a trip: where k-contiguous A is read and filled are
    // run-time offsets.
    static constexpr int A_SLOT = BM * ROW_BYTES, B_SLOT = BN * ROW_BYTES, A_PAIRS = 3;
    static constexpr int A_BYTES = AK ? NS * A_SLOT : A_PAIRS * 2 * A_SLOT, RING_BYTES = A_BYTES + NS * B_SLOT;
    static constexpr int A_BASE = AK ? 0 : NS * B_SLOT, B_BASE = AK ? A_BYTES : 0;   // (transposing reads stay in the lower 128 KB)
    int a_cur, a_nxt, a_fill;                    // k-contiguous A: the pair of the slot at hand, of the one after, the one being filled
    // fragment i of operand A (j of B) out of the slot in ring position S (`own`: the slot at hand, else the one after it)
    __device__ __forceinline__ bf16x8 a_frag(const unsigned char OB_LDS *__restrict__ ring, int S, int i, bool own) const {
        if (AK) return opa.frag(ring + S * A_SLOT, i, 0);
        return opa.frag(ring + (own || (S & 1) ? a_cur : a_nxt), i, S & 1);
    }
    __device__ __forceinline__ bf16x8 b_frag(const unsigned char OB_LDS *__restrict__ ring, int S, int j) const {
        return opb.frag(ring + (BKM ? S : S & ~1) * B_SLOT, j, S & 1);       // (the operand's offsets start at its region)
    }
    // Position of run g of slot S among the 2 T runs between the barrier of an odd slot and the barrier
    // two slots on: the odd slot's runs 1 .. T-1, the even slot's runs, run 0 of the next odd slot.
    static constexpr int position(int S, int g) { return (S & 1) ? (g == 0 ? 2 * T - 1 : g - 1) : T - 1 + g; }
    // the piece of k-contiguous A that the run at position q loads (-1: none): next to k-contiguous B
    // the even slot's runs; next to k-major B, whose loads sit in runs 1 .. T/2 of every slot, the
    // other runs
    static constexpr int piece_a(int q) {
        if (AK) return -1;
        if (!BKM) return q >= T - 1 && q < 2 * T - 1 ? q - (T - 1) : -1;         // the even slot's runs
        return q >= T / 2 && q < T ? q - T / 2 : (q >= T + T / 2 ? q - T : -1);
    }
    // (B k-contiguous: A is as well, there is no layout with A alone k-major.)  B's pieces go out in the
    // odd slot's runs 1 .. T-1, as early as its pair is free, the last one as a second load of run 1
    static constexpr int piece_b(int q) {
        if (BKM) return -1;
        return q < T - 1 ? q : -1;
    }
    // the pair of slots (0: slots 0 and 1; 1: slots 2 and 3) that the runs of slot S refill
    static constexpr int pair_of(int S, int g) { return (S & 1) ? (g == 0 ? ((S + 1) / 2) & 1 : (S - 1) / 2) : ((S / 2) + 1) & 1; }

    // Run g of the slot in ring position S: its T MFMAs and between them, never more than one memory
    // instruction between two MFMAs (a 16x16x32 MFMA keeps the pipe busy for four issue slots of a
    // lone wave, and whatever sits between two of them beyond three slots is lost: scalar
    // instructions count).  Run 0 reads its slot's own last A fragment (the register was busy until
    // now) and moves the descriptors on; the others read ahead in the slot after (run 1 one B fragment
    // more, which makes up for run 0).
    template <int S, int g>
    __device__ __forceinline__ void run(f32x4 (&acc)[T][T], unsigned char OB_LDS *__restrict__ ring) {
        constexpr int AT_RB = 0, AT_RA = 1, AT_RX = T >= 8 ? 2 : 1, AT_DL = T / 2, AT_RQ = T >= 8 ? T / 2 + 2 : T - 1;
        constexpr int set = S & 1, q = position(S, g), pa = piece_a(q), pb = piece_b(q);
        constexpr int N = (S + 1) % NS, P = (S + NS - 1) % NS, pair = pair_of(S, g);
#pragma unroll
        for (int j = 0; j < T; ++j) {
            mfma(acc[g][j], bfr[set][j], af[g]);
            __builtin_amdgcn_sched_barrier(0);
            if (g == 0) {
                if (j == AT_RA) af[T - 1] = a_frag(ring, S, T - 1, true);
                // the last load of the slot before, when both operands go straight to LDS
                if (AK && BKM && j == 2) opb.load(rb, ring + B_BASE + P * B_SLOT, wave, T / 2 - 1);
                // (small tiles: the descriptors of this slot's loads are worked out here, see below)
                if (T < 8 && (AK || (S & 1)) && j == 0) prepare_a();
                if (T < 8 && (BKM || (S & 1)) && j == 2) prepare_b();
            } else {
                if (j == AT_RB) bfr[set ^ 1][g] = b_frag(ring, N, g);
                if (j == AT_RA) af[g - 1] = a_frag(ring, N, g - 1, false);
                if (j == AT_RX && g == 1) bfr[set ^ 1][0] = b_frag(ring, N, 0);
                if (j == AT_RQ) {
                    if (AK && g - 1 < T / 2) opa.load(ra, ring + A_BASE + S * A_SLOT, wave, g - 1);
                    if (BKM && !AK && g - 1 < T / 2) opb.load(rb, ring + B_BASE + S * B_SLOT, wave, g - 1);
                    if (BKM && AK && g - 1 >= T / 2) opb.load(rb, ring + B_BASE + S * B_SLOT, wave, g - 1 - T / 2);
                }
            }
            // Descriptors: a k-major operand moves on every slot, a k-contiguous one every other, behind run 0.
            // The ten steps of working the next ones out are dealt over the gaps of runs 2 - 4 of the slot
            // before that no memory instruction uses (a wave alone on its SIMD has three issue slots per gap).
            if (T >= 8 && g >= 2 && g <= 4 && (j == 3 || j == 4 || j == 5 || j == 7)) {
                constexpr int first = (g - 2) * 4;
                const int step_no = first + (j == 7 ? 3 : j - 3);
                if (AK || !(S & 1)) {
                    if (step_no == 0) next_step<0>();
                    if (step_no == 1) next_step<1>();
                    if (step_no == 2) next_step<2>();
                    if (step_no == 3) next_step<3>();
                    if (step_no == 4) next_step<4>();
                }
                if (BKM || !(S & 1)) {
                    if (step_no == 5) next_step<5>();
                    if (step_no == 6) next_step<6>();
                    if (step_no == 7) next_step<7>();
                    if (step_no == 8) next_step<8>();
                    if (step_no == 9) next_step<9>();
                }
            }
            if (pa >= 0 && j == AT_RQ) opa.load_pair(ra, ring + A_BASE + a_fill, wave, pa);
            if (pb >= 0 && j == AT_RQ) opb.load_pair(rb, ring + B_BASE + pair * 2 * B_SLOT, wave, pb);
            if (pb == 0 && j == AT_DL + 1) opb.load_pair(rb, ring + B_BASE + pair * 2 * B_SLOT, wave, T - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (g == 0) {
            if (AK || (S & 1)) ra = ra_n;
            if (BKM || (S & 1)) rb = rb_n;
            // behind the barrier of an odd slot its pair is free: the runs from here on fill it, and
            // read the pair after it
            if (!AK && (S & 1)) {
                a_fill = a_cur;
                a_nxt = a_cur == (A_PAIRS - 1) * 2 * A_SLOT ? 0 : a_cur + 2 * A_SLOT;
            }
        }
        if (!AK && (S & 1) && g == T - 1) a_cur = a_nxt;
    }
    template <int S, int g>
    __device__ __forceinline__ void runs_from(f32x4 (&acc)[T][T], unsigned char OB_LDS *__restrict__ ring) {
        if constexpr (g < T) {
            run<S, g>(acc, ring);
            runs_from<S, g + 1>(acc, ring);
        }
    }
    // the loads of at most this many slots, the newest, may still be on their way at a barrier
    // (both operands k-contiguous: at the barrier of an odd slot, behind which B's pair filled two slots
    // before is read, the T loads of A since; at that of an even slot nothing new is read)
    static constexpr int vm_pending(int S) { return AK || BKM ? T * (NS - 2) : (S & 1) ? T : 63; }
    // The slot in ring position S.  On entry bfr[S & 1] and af[0 .. T-2] hold its fragments; on return
    // those of the slot after.
    template <int S>
    __device__ __forceinline__ void slot(f32x4 (&acc)[T][T], unsigned char OB_LDS *__restrict__ ring) {
        run<S, 0>(acc, ring);
        // own reads of this slot and own writes to LDS landed, own loads to the slot after in LDS (every
        // run issues one load, and the last one to the slot after went out NS - 2 slots ago or earlier),
        // then the barrier: the slot after is complete and nobody reads this one any more
        __builtin_amdgcn_s_waitcnt(waitcnt(vm_pending(S), 0));
        wg_barrier();
        runs_from<S, 1>(acc, ring);
    }
    // Before the first slot: the ring filled as the loop expects to find it, what the first slot needs
    // requested first.  k-major: the first NS slots, all but what run 0 of the first slot issues.
    // k-contiguous B: its two pairs.  k-contiguous A: the first two pairs and of the third what the runs
    // in front of the loop's first would have asked for (positions 0 .. T-2).
    // prologue_later(): the number of loads it issues after the last one that the first slot needs.
    static constexpr int prologue_later() {
        if (!AK && !BKM) return 2 * T;
        int n = 0;
        for (int q = 0; q < T - 1; ++q) n += piece_a(q) >= 0 ? 1 : 0;
        n += AK ? (NS - 1) * T / 2 : T;
        n += (NS - 1) * T / 2 - (AK ? 1 : 0);
        return n;
    }
    __device__ __forceinline__ void prologue(unsigned char OB_LDS *__restrict__ ring) {
        next_a();
#pragma unroll
        for (int p = 0; p < (AK ? T / 2 : T); ++p) {
            if (AK) opa.load(ra, ring + A_BASE, wave, p);
            else opa.load_pair(ra, ring + A_BASE, wave, p);
        }
        next_b();
#pragma unroll
        for (int p = 0; p < (BKM ? T / 2 : T); ++p) {
            if (BKM) opb.load(rb, ring + B_BASE, wave, p);
            else opb.load_pair(rb, ring + B_BASE, wave, p);
        }
        // the rest in the order of its use: a barrier of the loop waits for all but a fixed number of
        // the newest loads
#pragma unroll
        for (int sl = 1; sl < NS; ++sl) {
            if (AK) {
                next_a();
#pragma unroll
                for (int p = 0; p < T / 2; ++p) opa.load(ra, ring + A_BASE + sl * A_SLOT, wave, p);
            }
            if (BKM) {
                next_b();
#pragma unroll
                for (int p = 0; p < T / 2; ++p)
                    if (!(AK && sl == NS - 1 && p == T / 2 - 1)) opb.load(rb, ring + B_BASE + sl * B_SLOT, wave, p);
            }
            if (!BKM && sl == 1) {
                next_b();
#pragma unroll
                for (int p = 0; p < T; ++p) opb.load_pair(rb, ring + B_BASE + 2 * B_SLOT, wave, p);
            }
            if (!AK && sl == 1) {
                next_a();
#pragma unroll
                for (int p = 0; p < T; ++p) opa.load_pair(ra, ring + A_BASE + 2 * A_SLOT, wave, p);
            }
            if (!AK && sl == NS - 1) {
                next_a();
#pragma unroll
                for (int q = 0; q < T - 1; ++q)
                    if (piece_a(q) >= 0) opa.load_pair(ra, ring + A_BASE + 4 * A_SLOT, wave, piece_a(q));
                a_cur = a_nxt = 0;
                a_fill = 4 * A_SLOT;
            }
        }
        // what runs 2 - 4 of the slot before the first would have left: the descriptors that take over
        // behind run 0 of the first slot
        if (T >= 8 && AK) prepare_a();
        if (T >= 8 && BKM) prepare_b();
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
    __shared__ __attribute__((aligned(1024))) unsigned char ring_mem[KLoop<BM, BN, WM, WN, AK, BKM>::RING_BYTES];
    const int m0 = __builtin_amdgcn_readfirstlane(tile_m) * BM;
    const int n0 = __builtin_amdgcn_readfirstlane(tile_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    KLoop<BM, BN, WM, WN, AK, BKM> lp;
    lp.wave = wave;
    lp.opa.init(A, lda, m0, (AK ? (long)K : (long)M) * lda * 2, wave, lane, wm * (BM / WM), lp.A_BASE);
    lp.opb.init(B, ldb, n0, (BKM ? (long)K : (long)N) * ldb * 2, wave, lane, wn * (BN / WN), lp.B_BASE);

    f32x4 acc[T][T];
    unsigned char OB_LDS *ring = (unsigned char OB_LDS *)ring_mem;
    // a slice covers K steps [k_first, k_first + nk); two ring slots to the K step
    const int k_first = kz * ts.k_chunk;
    const int nk = sliced ? min(ts.k_chunk, (K + KSTEP - 1) / KSTEP - k_first) : (K + KSTEP - 1) / KSTEP;
    lp.opa.skip(k_first);
    lp.opb.skip(k_first);
    lp.ka_left = AK ? 2 * nk : nk;
    lp.kb_left = BKM ? 2 * nk : nk;
    lp.prologue(ring);
    // the accumulators are cleared while the first loads are on their way (the empty statement pins the 256
    // moves here: left alone they sink behind the wait for those loads)
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
            asm volatile("" : "+a"(acc[i][j]));
        }
    constexpr int later = KLoop<BM, BN, WM, WN, AK, BKM>::prologue_later();
    __builtin_amdgcn_s_waitcnt(waitcnt(later < 63 ? later : 63, 0));
    wg_barrier();
#pragma unroll
    for (int j = 0; j < T; ++j) lp.bfr[0][j] = lp.b_frag(ring, 0, j);
#pragma unroll
    for (int i = 0; i < T - 1; ++i) lp.af[i] = lp.a_frag(ring, 0, i, true);

    // once round the ring per trip: a single straight path with immediate LDS addresses.  There is no
    // separate tail (several ways into the epilogue make the register allocator move the
    // accumulators between homes): the last slots also read ahead and load (fragments that are never
    // used, zeros from past the end of K), and the count of slots is rounded up to whole trips with
    // slots of zeros.
    for (int kt = 0; kt < 2 * nk; kt += NS) {
        lp.template slot<0>(acc, ring);
        lp.template slot<1>(acc, ring);
        lp.template slot<2>(acc, ring);
        lp.template slot<3>(acc, ring);
    }
    static_assert(NS == 4, "the trip above names the slots");

    // the MFMAs above are opaque to the compiler's hazard handling: let the last ones retire before
    // the accumulators are read
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");
    // every wave is done reading the ring and every load still in flight has landed in it (zeros from
    // past the end of K); then the ring serves as transposition slabs.  A lane holds, per MFMA tile, output row m = lane % 16 and columns
    // n = 4 (lane / 16) + (0..3): stored directly, every lane of a store would touch a different
    // cache line.  Each wave writes two tile rows (32 output rows) to its slab as fp32 and reads
    // them back so that 16 (or 8) consecutive lanes cover one contiguous row segment; bias and
    // residual are added on the way out, then one rounding to bf16.
    __builtin_amdgcn_s_waitcnt(waitcnt(0, 0));
    __syncthreads();
    constexpr int CW = BN / WN;            // columns of the wave's tile
    constexpr int RSTR = CW * 4 + 16;      // fp32 row stride in LDS, padded against bank conflicts
    constexpr int LPR = CW / 8;            // lanes per row on the way out (8 columns each)
    constexpr int RPI = 64 / LPR;          // rows per read instruction
    static_assert(32 * RSTR <= NS * C::SLOT / C::NW, "slab does not fit the wave's LDS share");
    unsigned char OB_LDS *slab = ring + wave * (NS * C::SLOT / C::NW);
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
    auto put = [&](int ii) {   // tile rows 2 ii and 2 ii + 1 of the wave into its slab
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < T; ++j)
                *(f32x4 OB_LDS *)(slab + (16 * h + lx) * RSTR + (j * 16 + lq * 4) * 4) = acc[2 * ii + h][j];
    };
    // One straight path per kind of output (MODE 0: bf16; 1: bf16 with the residual added; 2: the fp32 sums
    // of a slice, the whole tile: sums beyond M and N are never read by tail_sum_kernel) and per kind of
    // tile (CHECK: some rows or columns lie past M or N): with the choices inside the loop every row read
    // was a round trip to LDS of its own.  All reads of a pair of tile rows are issued together; the next
    // pair is written to the slab behind them (a wave's LDS accesses execute in order) while the rows
    // just read are rounded and stored.
    auto out = [&](auto mode, auto check) {
        constexpr int MODE = decltype(mode)::value;
        constexpr bool CHECK = decltype(check)::value;
        constexpr int NR = 32 / RPI;
        put(0);
#pragma unroll
        for (int ii = 0; ii < T / 2; ++ii) {
            f32x4 lo[NR], hi[NR];
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int row = r * RPI + lane / LPR;
                lo[r] = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32);
                hi[r] = *(const f32x4 OB_LDS *)(slab + row * RSTR + (lane % LPR) * 32 + 16);
            }
            if (ii + 1 < T / 2) put(ii + 1);
            const int m_first = m0 + wm * (BM / WM) + ii * 32 + lane / LPR;
            bf16x8 r8[NR];
            if (MODE == 1) {
#pragma unroll
                for (int r = 0; r < NR; ++r)
                    if (!CHECK || (m_first + r * RPI < M && n_out < N))
                        r8[r] = *(const bf16x8 *)(R + (size_t)(m_first + r * RPI) * ldr + n_out);
            }
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int m = m_first + r * RPI;
                if (MODE == 2) {
                    float *dst = ts.part + ((size_t)(kz * ts.n_tail + tail_tile) * BM + (m - m0)) * BN + (n_out - n0);
                    *(f32x4 *)dst = lo[r];
                    *(f32x4 *)(dst + 4) = hi[r];
                } else if (!CHECK || (m < M && n_out < N)) {
                    float o8[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { o8[e] = lo[r][e] + bv[e]; o8[4 + e] = hi[r][e] + bv[4 + e]; }
                    if (MODE == 1) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) o8[e] += (float)r8[r][e];
                    }
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (__bf16)o8[e];
                    __builtin_nontemporal_store(o, (bf16x8 *)(Cm + (size_t)m * ldc + n_out));
                }
            }
        }
    };
    using std::integral_constant;
    const bool inside = m0 + BM <= M && n0 + BN <= N;
    if (sliced) out(integral_constant<int, 2>{}, integral_constant<bool, false>{});
    else if (inside && R) out(integral_constant<int, 1>{}, integral_constant<bool, false>{});
    else if (inside) out(integral_constant<int, 0>{}, integral_constant<bool, false>{});
    else if (R) out(integral_constant<int, 1>{}, integral_constant<bool, true>{});
    else out(integral_constant<int, 0>{}, integral_constant<bool, true>{});
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
    const int nk = (K + KSTEP - 1) / KSTEP;
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
    const int nk = (K + KSTEP - 1) / KSTEP, slots = compute_units();
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
    const int nk = (K + KSTEP - 1) / KSTEP;
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
