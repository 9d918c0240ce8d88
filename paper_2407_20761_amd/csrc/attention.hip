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
// the next MFMA wants as its second operand (accumulator register 8 (u%2) + e of row-tile u/2
// carries streamed row 16 u + 8 (e/4) + 4 (l/32) + e%4, and the other operand is fetched from LDS
// in that same order).
//
// The streamed 64-row tiles (K and V; Q and dO in the dK/dV kernel) are copied global -> LDS
// asynchronously (buffer loads that write LDS directly, two stages, the next tile in flight while
// the current one is multiplied) in their natural [row][D] layout.  Products that contract over D
// read 16-byte fragments; products that contract over the streamed rows read the same tile with
// the transposing LDS read (ds_read_b64_tr_b16), so no tile is ever stored twice.  16-byte chunks
// are XOR-swizzled by the row so that both kinds of read are free of bank conflicts.
#include <algorithm>
#include <type_traits>

#include "ob_internal.h"

namespace ob {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

#define OB_LDS __attribute__((address_space(3)))

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;
constexpr float RESCALE_LOG2 = 8.0f;  // the forward's reference maximum may lag the row maximum by this much (base-2 log)
constexpr int QT = 128;  // rows owned by a workgroup (4 waves x 32)
constexpr int ST = 64;   // rows of a streamed tile
constexpr int WAIT_VM0 = 0x0F70;  // s_waitcnt vmcnt(0) only

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The value of lane l ^ 32, in one vector instruction (v_permlane32_swap exchanges the upper half of its
// first register with the lower half of its second; given the same value twice, every lane ends up with
// its own value in one of the two results and its partner's in the other): __shfl_xor goes through the
// LDS crossbar, a round trip in the middle of the forward's dependent chain maximum -> exponentials.
__device__ __forceinline__ void both_halves(float x, float &a, float &b) {
#if defined(__HIP_DEVICE_COMPILE__)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
#else
    a = b = x;
#endif
}
__device__ __forceinline__ float max_halves(float x) {
    float a, b;
    both_halves(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float sum_halves(float x) {
    float a, b;
    both_halves(x, a, b);
    return a + b;
}

// XOR applied to the 16-byte chunk index of tile row r.  D = 128 (16 chunks per 256-byte row):
// 16 consecutive rows get 16 different values (conflict-free fragment reads) and the 4 rows of a
// transposing read differ in bits 2-3 (they land in different 64-byte groups).  D = 64 (8 chunks
// per 128-byte row, two rows per bank window): the same two properties with 3 bits.
template <int D>
__device__ __forceinline__ int swz(int r) {
    return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

// Per-lane addressing of one streamed [64][D] tile family.
template <int D>
struct Tile {
    static constexpr int RB = D * 2;            // bytes per tile row
    static constexpr int BYTES = ST * RB;
    static constexpr int CPR = RB / 16;         // chunks per row
    static constexpr int RPI = 1024 / RB;       // rows filled by one wave-level load
    static constexpr int LD = ST / RPI / 4;     // wave-level loads per wave per tile
    uint32_t voff[LD];                          // global byte offset of this lane's chunk (row-in-tile part)
    int rr[D / 16];                             // LDS offset of the 16-byte fragment read, per D-step t
    int tro[2][D / 32];                         // LDS offset of the transposing read, per half s and D-tile dt

    __device__ __forceinline__ void init(int ld, int wave, int lane) {
#pragma unroll
        for (int p = 0; p < LD; ++p) {
            const int row = (wave * LD + p) * RPI + lane / CPR;
            const int ch = (lane % CPR) ^ swz<D>(row);
            voff[p] = ((uint32_t)row * (uint32_t)ld + ch * 8) * 2u;
        }
        const int x = lane & 31, h = lane >> 5;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) rr[t] = x * RB + (((2 * t + h) ^ swz<D>(x)) * 16);
        const int b = lane >> 4, q = lane & 15, kq = q >> 2, c = q & 3, hb = b >> 1;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) {
                const int row = 8 * s + 4 * hb + kq;  // + 16 u
                const int chunk = 4 * dt + 2 * (b & 1) + (c >> 1);
                tro[s][dt] = row * RB + ((chunk ^ swz<D>(row)) * 16) + (c & 1) * 8;
            }
    }
    // asynchronous copy of rows [row0, row0 + 64) of a [*, ld] matrix (column offset folded into
    // `base`); rows past the end of the matrix arrive as zeros
    __device__ __forceinline__ void issue(const unsigned char *base, long bytes_left,
                                          unsigned char OB_LDS *__restrict__ dst, int wave) const {
        const uint64_t b = (uint64_t)base;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
        // the checked range: bytes_left clamped to [0, 2^32 - 1], in scalar instructions (the compiler's own
        // 64-bit compares go through the vector unit)
        uint32_t num = 0;
#if defined(__HIP_DEVICE_COMPILE__)
        asm("s_cmp_eq_u32 %2, 0\n\ts_cselect_b32 %0, %1, -1\n\ts_cmp_lt_i32 %2, 0\n\ts_cselect_b32 %0, 0, %0"
            : "=&s"(num)
            : "s"(__builtin_amdgcn_readfirstlane((uint32_t)bytes_left)),
              "s"(__builtin_amdgcn_readfirstlane((int32_t)(bytes_left >> 32)))
            : "scc");
#endif
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(((uint64_t)hi << 32) | lo), 0, (int)num, 0x00020000);
#pragma unroll
        for (int p = 0; p < LD; ++p)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst + (wave * LD + p) * 1024, 16, voff[p], 0, 0, 0);
    }
    // lane l: tile row 32 mt + l % 32, elements 16 t + 8 (l / 32) .. +7
    __device__ __forceinline__ bf16x8 frag_row(const unsigned char OB_LDS *__restrict__ tile, int mt, int t) const {
        return *(const bf16x8 OB_LDS *)(tile + rr[t] + mt * 32 * RB);
    }
    // lane l: column 32 dt + l % 32, rows 16 u + 8 (e / 4) + 4 (l / 32) + e % 4 for e = 0..7
    __device__ __forceinline__ bf16x8 frag_tr(const unsigned char OB_LDS *__restrict__ tile, int dt, int u) const {
#if defined(__HIP_DEVICE_COMPILE__)  // gfx950-only builtin, hidden from the host pass
        typedef __attribute__((ext_vector_type(4))) short s16x4;
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 OB_LDS *)(tile + tro[0][dt] + u * 16 * RB));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 OB_LDS *)(tile + tro[1][dt] + u * 16 * RB));
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#else
        return bf16x8{};
#endif
    }
};

// accumulator registers 8 (u % 2) .. +7 of a 32x32 tile -> the 8-slot second operand of step u
__device__ __forceinline__ bf16x8 pack8(const f32x16 &a, int base) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)a[base + e];
    return o;
}

// Rotary backward folded into the epilogues of the backward kernels.  A lane holds, of one token's head
// row, accumulator (dt, r) = column 32 dt + 8 (r / 4) + 4 lh + r % 4: the rotary pair (i, i + D/2) is
// (dt, r) and (dt + D/64, r) of the same lane.  The gradient is rotated by minus the token's angle
// pos * base^(-2 i / D), pos = distance to the segment's first token (log2_base <= 0: no rotary).
// Sine and cosine come from the hardware's functions of the angle in revolutions, reduced to [0, 1)
// first: an absolute error of a few 1e-4 rad at positions in the thousands, an order of magnitude
// below the bf16 rounding of the result.
template <int D>
__device__ __forceinline__ void rotary_bwd_row(f32x16 (&acc)[D / 32], int pos, float log2_base, int lh) {
    constexpr int H = D / 64;   // accumulator tiles per half of the head dimension
#pragma unroll
    for (int dt = 0; dt < H; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int i = 32 * dt + 8 * (r >> 2) + 4 * lh + (r & 3);
            const float theta = __builtin_amdgcn_exp2f(-2.0f * (float)i / (float)D * log2_base);
            float rev = (float)pos * theta * 0.15915494309189535f;
            rev -= floorf(rev);
            const float sn = __builtin_amdgcn_sinf(rev), cs = __builtin_amdgcn_cosf(rev);
            const float x1 = acc[dt][r], x2 = acc[dt + H][r];
            acc[dt][r] = x1 * cs + x2 * sn;
            acc[dt + H][r] = x2 * cs - x1 * sn;
        }
}

// Which workgroup does which tile.  The launch is one-dimensional: workgroup b works on tile
// b / heads for head slot b % heads, so all heads of a tile are dispatched together, and (workgroups
// being dealt round-robin to the 8 XCDs) head slot hs runs on XCD hs % 8: with a head count that is a
// multiple of 8 the slots are renumbered so that an XCD only ever sees heads [x heads/8, (x+1) heads/8),
// i.e. the query heads of one key/value group (and that group's K and V) stay in one XCD's L2.
__device__ __forceinline__ int head_of_slot(int hs, int heads) {
    return (heads & 7) == 0 ? (hs & 7) * (heads >> 3) + (hs >> 3) : hs;
}

// Order of the tiles: heaviest first.  The work of a tile is the number of streamed tiles it walks;
// in a causal batch that differs by an order of magnitude between the first and the last tile of a
// long segment, and a launch that hands out the tiles segment by segment ends with a few workgroups
// on the heaviest tiles of the last segment while the rest of the chip idles (simulated on the
// benchmark's batches: 20 % of the forward's and 40 % of the dK/dV kernel's duration).  The host
// sorts the tiles by work (ties: natural order) and passes the order as a kernel argument:
// entry = segment << 16 | tile in segment.  n == 0 (more tiles than the table holds, or a segment or
// tile number beyond 16 bits): natural order, found by find_tile.
struct TileOrder {
    static constexpr int CAP = 896;
    int n;
    uint32_t e[CAP];
};

// Which segment-aligned tile (of `tile_rows` rows) has number `tile` when tiles are numbered segment
// by segment.  Thread j looks at segment j (256 segments per round), an inclusive scan over the
// workgroup gives each segment's first tile number, and the thread whose range holds `tile`
// publishes the answer -- one global-memory round trip instead of a serial walk over cu.
struct TileInfo { int seg_start, seg_end, row0; };
__device__ __forceinline__ TileInfo find_tile(const int32_t *__restrict__ cu, int n_seg, int tile_rows,
                                              int *sh /* >= 8 ints */, int tile) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool scans = tid < 256;  // waves past the fourth only take part in the barriers
    if (tid == 0) sh[2] = -1;
    int base = 0;  // tiles in the segments of earlier rounds
    for (int j0 = 0; j0 < n_seg; j0 += 256) {
        const int j = j0 + tid;
        int a = 0, b = 0, nt = 0;
        if (scans && j < n_seg) {
            a = cu[j];
            b = cu[j + 1];
            nt = (b - a + tile_rows - 1) / tile_rows;
        }
        int incl = nt;  // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        __syncthreads();  // sh[4..7] free (previous round consumed)
        if (scans && lane == 63) sh[4 + wave] = incl;
        __syncthreads();
        int before = base;
        for (int w = 0; w < (wave & 3); ++w) before += sh[4 + w];
        const int first = before + incl - nt;  // number of this segment's first tile
        if (scans && nt > 0 && tile >= first && tile < first + nt) {
            sh[0] = a;
            sh[1] = b;
            sh[2] = a + (tile - first) * tile_rows;
        }
        base += sh[4] + sh[5] + sh[6] + sh[7];
    }
    __syncthreads();
    TileInfo t;
    t.seg_start = __builtin_amdgcn_readfirstlane(sh[0]);
    t.seg_end = __builtin_amdgcn_readfirstlane(sh[1]);
    t.row0 = __builtin_amdgcn_readfirstlane(sh[2]);
    return t;
}

// tile number `rank` in the order of work
__device__ __forceinline__ TileInfo pick_tile(const TileOrder &ord, int rank, const int32_t *__restrict__ cu,
                                              int n_seg, int tile_rows, int *sh) {
    if (ord.n == 0) return find_tile(cu, n_seg, tile_rows, sh, rank);
    const uint32_t e = ord.e[rank];
    const int seg = (int)(e >> 16);
    TileInfo t;
    t.seg_start = __builtin_amdgcn_readfirstlane(cu[seg]);
    t.seg_end = __builtin_amdgcn_readfirstlane(cu[seg + 1]);
    t.row0 = t.seg_start + (int)(e & 0xFFFFu) * tile_rows;
    return t;
}

// ------------------------------------------------------------------------------------------------
// forward:  S^T = K Q^T,  online softmax per lane,  O^T += V^T P^T
// ------------------------------------------------------------------------------------------------
// LDS reads are issued one batch ahead of the MFMAs that consume them (explicit double buffers and
// scheduling groups): left alone, the compiler emits read / wait / MFMA triples and every MFMA
// pays a full LDS round trip.
#define OB_SCHED_READS_THEN_MFMA(n_reads, n_mfma)                 \
    do {                                                          \
        __builtin_amdgcn_sched_group_barrier(0x100, (n_reads), 0); \
        __builtin_amdgcn_sched_group_barrier(0x008, (n_mfma), 0);  \
        __builtin_amdgcn_sched_barrier(0);                         \
    } while (0)

template <int D, bool CAUSAL, bool MASK>
__device__ __forceinline__ void fwd_tile(const unsigned char OB_LDS *__restrict__ ks,
                                         const unsigned char OB_LDS *__restrict__ vs, const Tile<D> &tl,
                                         const bf16x8 (&qf)[D / 16], f32x16 (&acc_o)[D / 32], float &m_run,
                                         float &l_run, int kv0, int seg_end, int q_row, float sl2) {
    const int lh = (threadIdx.x & 63) >> 5;
    constexpr int HB = 2;                 // K fragments (D-steps) per batch
    constexpr int R = D == 128 ? 3 : 2;   // batches in flight (ring depth)
    constexpr int PER = (D / 16) / HB;    // batches per 32-row tile
    constexpr int NB = 2 * PER;
    constexpr int DT = D / 32;
    f32x16 acc_s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_s[mt][r] = 0.f;
    bf16x8 fa[R][HB], fb[2][DT];
#pragma unroll
    for (int b = 0; b < R - 1; ++b)
#pragma unroll
        for (int i = 0; i < HB; ++i) fa[b][i] = tl.frag_row(ks, b / PER, (b % PER) * HB + i);
#pragma unroll
    for (int b = 0; b < NB; ++b) {  // batch b: row tile b / PER, D-steps (b % PER) HB ..
        constexpr int AHEAD = R - 1;
        if (b + AHEAD < NB) {
#pragma unroll
            for (int i = 0; i < HB; ++i)
                fa[(b + AHEAD) % R][i] = tl.frag_row(ks, (b + AHEAD) / PER, ((b + AHEAD) % PER) * HB + i);
        } else if (b + AHEAD == NB) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) fb[0][dt] = tl.frag_tr(vs, dt, 0);
        }
#pragma unroll
        for (int i = 0; i < HB; ++i)
            acc_s[b / PER] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[b % R][i], qf[(b % PER) * HB + i], acc_s[b / PER], 0, 0, 0);
        if (b + AHEAD < NB) OB_SCHED_READS_THEN_MFMA(HB, HB);
        else if (b + AHEAD == NB) OB_SCHED_READS_THEN_MFMA(2 * DT, HB);
        else OB_SCHED_READS_THEN_MFMA(0, HB);
    }
    // the running maximum is kept on the raw scores; the softmax scale rides in the exponent's FMA
    float mx = NEG_BIG;
    if (MASK) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = kv0 + mt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const bool ok = kv < seg_end && (!CAUSAL || kv <= q_row);
                const float s = ok ? acc_s[mt][r] : NEG_BIG;
                acc_s[mt][r] = s;
                mx = fmaxf(mx, s);
            }
    } else {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[mt][r]);
    }
    mx = max_halves(mx);
    // The reference maximum m_run of a row only has to keep the exponentials in range, it need not be
    // the true maximum: it follows the row maximum when that has outgrown it by more than 2^RESCALE_LOG2
    // in some row of the wave (probabilities then reach at most 2^RESCALE_LOG2, harmless in fp32 sums
    // and in bf16 operands), so the accumulators are rescaled a few times per row instead of at almost
    // every tile (with random scores some row of 32 finds a new maximum in nearly every tile).
    if (__any((mx - m_run) * sl2 > RESCALE_LOG2)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * sl2);
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
        m_run = m_new;
    }
    const float c = m_run * sl2;
    float psum = 0.f;
    // The exponentials of contraction step u + 1 (8 per lane, then their rounding to bf16) are issued
    // between the MFMAs of step u, one MFMA to a few vector instructions: a wave's own element-wise
    // work then runs in the shadow of its own matrix instructions.
    auto probs = [&](int u) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float p = fast_exp2(acc_s[u >> 1][8 * (u & 1) + e] * sl2 - c);
            psum += p;
            o[e] = (__bf16)p;
        }
        return o;
    };
    bf16x8 pb = probs(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < ST / 16; ++u) {
        bf16x8 pn = pb;
        if (u + 1 < ST / 16) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) fb[(u + 1) & 1][dt] = tl.frag_tr(vs, dt, u + 1);
            pn = probs(u + 1);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[u & 1][dt], pb, acc_o[dt], 0, 0, 0);
        if (u + 1 < ST / 16) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * DT, 0);        // next step's V fragments
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, (28 + DT - 1) / DT, 0);   // its share of 28 vector instructions
            }
            __builtin_amdgcn_sched_barrier(0);
        } else {
            OB_SCHED_READS_THEN_MFMA(0, DT);
        }
        pb = pn;
    }
    l_run += psum;
}

// (D = 64: 128 registers, four waves on a SIMD)
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, D == 64 ? 4 : 2) void attn_fwd_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    __bf16 *__restrict__ o, float *__restrict__ lse, int ldq, int ldkv, int ldo,
    const int32_t *__restrict__ cu, int n_seg, int T, int group, float scale, int heads, TileOrder ord) {
    __shared__ __attribute__((aligned(1024))) unsigned char k_s0[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_s0[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char k_s1[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_s1[Tile<D>::BYTES];
    __shared__ int sh[8];
    const int rank = blockIdx.x / heads;
    const TileInfo ti = pick_tile(ord, rank, cu, n_seg, QT, sh);
    if (ti.row0 < 0) return;
    const int head = head_of_slot(blockIdx.x - rank * heads, heads), kvh = head / group;
    const int lane = threadIdx.x & 63, lx = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q_row = min(ti.row0 + wave * 32 + lx, ti.seg_end - 1);
    const bool q_live = ti.row0 + wave * 32 + lx < ti.seg_end;
    const int wave_q_last = min(ti.row0 + wave * 32 + 31, ti.seg_end - 1);
    const float sl2 = scale * LOG2E;

    Tile<D> tl;
    tl.init(ldkv, wave, lane);
    const unsigned char *kbase = (const unsigned char *)(k + kvh * D);
    const unsigned char *vbase = (const unsigned char *)(v + kvh * D);
    const long kv_bytes = (long)T * ldkv * 2 - (long)kvh * D * 2;  // from kbase / vbase to the end

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
    const int n_tiles = (kv_end - ti.seg_start + ST - 1) / ST;
    unsigned char OB_LDS *const ks0 = (unsigned char OB_LDS *)k_s0, *const ks1 = (unsigned char OB_LDS *)k_s1;
    unsigned char OB_LDS *const vs0 = (unsigned char OB_LDS *)v_s0, *const vs1 = (unsigned char OB_LDS *)v_s1;
    {
        const long off = (long)ti.seg_start * ldkv * 2;
        tl.issue(kbase + off, kv_bytes - off, ks0, wave);
        tl.issue(vbase + off, kv_bytes - off, vs0, wave);
    }
    // Tiles before the workgroup's first row (causal) or before the ragged end need no mask; they
    // run in a loop of their own whose body is a single straight path (with several paths per
    // iteration the register allocator shuffles the accumulators between homes every iteration).
    const int n_main = CAUSAL ? (ti.row0 - ti.seg_start) / ST : (ti.seg_end - ti.seg_start) / ST;
    int j = 0;
#define OB_FWD_ITER(MASKED, KS, VS, KS_NEXT, VS_NEXT)                                                     \
    {                                                                                                    \
        const int kv0 = ti.seg_start + j * ST;                                                           \
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);                                                            \
        __syncthreads();                                                                                 \
        if (j + 1 < n_tiles) {                                                                           \
            const long off = (long)(kv0 + ST) * ldkv * 2;                                                \
            tl.issue(kbase + off, kv_bytes - off, (KS_NEXT), wave);                                      \
            tl.issue(vbase + off, kv_bytes - off, (VS_NEXT), wave);                                      \
        }                                                                                                \
        if (!(MASKED))                                                                                   \
            fwd_tile<D, CAUSAL, false>((KS), (VS), tl, qf, acc_o, m_run, l_run, kv0, ti.seg_end, q_row,  \
                                       sl2);                                                             \
        else if (!(CAUSAL && kv0 > wave_q_last))                                                         \
            fwd_tile<D, CAUSAL, true>((KS), (VS), tl, qf, acc_o, m_run, l_run, kv0, ti.seg_end, q_row,   \
                                      sl2);                                                              \
        ++j;                                                                                             \
    }
    // two tiles per trip: the stage buffers are then compile-time constants and every LDS address is
    // a register plus an immediate offset
    while (j + 1 < n_main) {
        OB_FWD_ITER(false, ks0, vs0, ks1, vs1)
        OB_FWD_ITER(false, ks1, vs1, ks0, vs0)
    }
#define OB_FWD_ANY(MASKED) OB_FWD_ITER(MASKED, (j & 1) ? ks1 : ks0, (j & 1) ? vs1 : vs0, (j & 1) ? ks0 : ks1, (j & 1) ? vs0 : vs1)
    while (j < n_main) OB_FWD_ANY(false)
    while (j < n_tiles) OB_FWD_ANY(true)
#undef OB_FWD_ANY
#undef OB_FWD_ITER
    const float l_tot = sum_halves(l_run);
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
    if (lh == 0) lse[(size_t)head * T + q_row] = (m_run * sl2 + __builtin_amdgcn_logf(l_tot)) * LN2;
}

// ------------------------------------------------------------------------------------------------
// backward, part 1: dQ.  A workgroup owns 128 query rows of one head (four wavefronts, 32 rows
// each) and streams the segment's 64-row key/value tiles (up to the diagonal when causal); P is
// rebuilt from the saved log-sum-exp.  A wave takes the two 32-row halves of a streamed tile one
// after the other through the three products
//   S^T = K Q^T,  P = 2^(scale log2(e) S - lse2),  dP^T = V dO^T,  dS^T = P (dP^T - Delta),
//   dQ^T += K^T dS^T
// so its state between the products is that of a 32 x 32 block (two such waves fit on a SIMD; two
// workgroups share a CU and, as nothing synchronises them, their phases drift apart).  Every K / V
// tile a workgroup copies serves 128 query rows: the first layout, two waves per 32 query rows each
// on one half of the tile with their partial dQ added at the end, asked the L2 for twice the bytes
// per MFMA (4.7 GB per launch on the 7B-shaped batch, 10 TB/s) and had a barrier per 24 MFMAs.
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL, bool MASK>
__device__ __forceinline__ void dq_half(const unsigned char OB_LDS *__restrict__ ks,
                                        const unsigned char OB_LDS *__restrict__ vs, const Tile<D> &tl,
                                        const bf16x8 (&qf)[D / 16], const bf16x8 (&dof)[D / 16],
                                        f32x16 (&acc_dq)[D / 32], float lse2, float dlt, int kv_first,
                                        int seg_end, int q_row, float sl2) {
    // ks / vs point at a 32-row half of the K / V tile; kv_first is its first key row
    const int lh = (threadIdx.x & 63) >> 5;
    constexpr int HB = 2;             // D-steps per batch (a batch reads HB fragments of K and HB of V)
    constexpr int NB = (D / 16) / HB;
    constexpr int DT = D / 32;
    f32x16 acc_s, acc_dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_s[r] = acc_dp[r] = 0.f;
    bf16x8 fk[2][HB], fv[2][HB], fb[2][DT];
#pragma unroll
    for (int i = 0; i < HB; ++i) {
        fk[0][i] = tl.frag_row(ks, 0, i);
        fv[0][i] = tl.frag_row(vs, 0, i);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b + 1 < NB) {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                fk[(b + 1) & 1][i] = tl.frag_row(ks, 0, (b + 1) * HB + i);
                fv[(b + 1) & 1][i] = tl.frag_row(vs, 0, (b + 1) * HB + i);
            }
        } else {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) fb[0][dt] = tl.frag_tr(ks, dt, 0);
        }
#pragma unroll
        for (int i = 0; i < HB; ++i) {
            acc_s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[b & 1][i], qf[b * HB + i], acc_s, 0, 0, 0);
            acc_dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[b & 1][i], dof[b * HB + i], acc_dp, 0, 0, 0);
        }
        if (b + 1 < NB) OB_SCHED_READS_THEN_MFMA(2 * HB, 2 * HB); else OB_SCHED_READS_THEN_MFMA(2 * DT, 2 * HB);
    }
    // dS of contraction step h (8 values per lane, rounded to bf16); step 1's are worked out between the
    // MFMAs of step 0, so the wave's own element-wise work runs in the shadow of its matrix instructions
    auto dscores = [&](int h) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int r = 8 * h + e;
            bool ok = true;
            if (MASK) {
                const int kv = kv_first + 8 * (r >> 2) + 4 * lh + (r & 3);
                ok = kv < seg_end && (!CAUSAL || kv <= q_row);
            }
            const float p = ok ? fast_exp2(acc_s[r] * sl2 - lse2) : 0.f;
            o[e] = (__bf16)(p * (acc_dp[r] - dlt));
        }
        return o;
    };
    const bf16x8 ds0 = dscores(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) fb[1][dt] = tl.frag_tr(ks, dt, 1);
    const bf16x8 ds1 = dscores(1);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        acc_dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][dt], ds0, acc_dq[dt], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * DT, 0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, (MASK ? 60 : 36) / DT, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        acc_dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][dt], ds1, acc_dq[dt], 0, 0, 0);
    OB_SCHED_READS_THEN_MFMA(0, DT);
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(
    const __bf16 *__restrict__ d_o, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k,
    const __bf16 *__restrict__ v, const __bf16 *__restrict__ o, const float *__restrict__ lse,
    float *__restrict__ lse2_all, float *__restrict__ delta, __bf16 *__restrict__ dq, int ldq, int ldkv, int ldo,
    const int32_t *__restrict__ cu, int n_seg, int T, int group, float scale, float rot_log2_base, int heads,
    TileOrder ord) {
    __shared__ __attribute__((aligned(1024))) unsigned char k_s0[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_s0[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char k_s1[Tile<D>::BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char v_s1[Tile<D>::BYTES];
    __shared__ int sh[8];
    const int rank = blockIdx.x / heads;
    const TileInfo ti = pick_tile(ord, rank, cu, n_seg, QT, sh);
    if (ti.row0 < 0) return;
    const int head = head_of_slot(blockIdx.x - rank * heads, heads), kvh = head / group;
    const int lane = threadIdx.x & 63, lx = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q_row = min(ti.row0 + wave * 32 + lx, ti.seg_end - 1);
    const bool q_live = ti.row0 + wave * 32 + lx < ti.seg_end;
    const int wave_q_last = min(ti.row0 + wave * 32 + 31, ti.seg_end - 1);
    const bool wave_live = ti.row0 + wave * 32 < ti.seg_end;   // a wave past the segment's end only copies
    const float sl2 = scale * LOG2E;
    constexpr int DT = D / 32, HALF = 32 * Tile<D>::RB;

    Tile<D> tl;
    tl.init(ldkv, wave, lane);
    const unsigned char *kbase = (const unsigned char *)(k + kvh * D);
    const unsigned char *vbase = (const unsigned char *)(v + kvh * D);
    const long kv_bytes = (long)T * ldkv * 2 - (long)kvh * D * 2;

    bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        qf[t] = *(const bf16x8 *)(q + (size_t)q_row * ldq + head * D + 16 * t + 8 * lh);
        dof[t] = *(const bf16x8 *)(d_o + (size_t)q_row * ldo + head * D + 16 * t + 8 * lh);
    }
    // The row statistics of the backward: Delta = sum_d dO O and the log-sum-exp in base-2 units.  The
    // wave holds its rows of dO already; each lane adds its half of the row, the other half sits 32
    // lanes away.  Both are also written out: the dK / dV kernel, launched behind this one, reads them.
    const float lse2 = lse[(size_t)head * T + q_row] * LOG2E;
    float dlt = 0.f;
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        const bf16x8 of = *(const bf16x8 *)(o + (size_t)q_row * ldo + head * D + 16 * t + 8 * lh);
#pragma unroll
        for (int e = 0; e < 8; ++e) dlt += (float)dof[t][e] * (float)of[e];
    }
    dlt = sum_halves(dlt);
    if (q_live && lh == 0) {
        lse2_all[(size_t)head * T + q_row] = lse2;
        delta[(size_t)head * T + q_row] = dlt;
    }
    f32x16 acc_dq[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_dq[i][r] = 0.f;

    const int kv_end = CAUSAL ? min(ti.seg_end, ti.row0 + QT) : ti.seg_end;
    const int n_tiles = (kv_end - ti.seg_start + ST - 1) / ST;
    unsigned char OB_LDS *const ks0 = (unsigned char OB_LDS *)k_s0, *const ks1 = (unsigned char OB_LDS *)k_s1;
    unsigned char OB_LDS *const vs0 = (unsigned char OB_LDS *)v_s0, *const vs1 = (unsigned char OB_LDS *)v_s1;
    {
        const long off = (long)ti.seg_start * ldkv * 2;
        tl.issue(kbase + off, kv_bytes - off, ks0, wave);
        tl.issue(vbase + off, kv_bytes - off, vs0, wave);
    }
    const int n_main = CAUSAL ? (ti.row0 - ti.seg_start) / ST : (ti.seg_end - ti.seg_start) / ST;
    int j = 0;
#define OB_DQ_ITER(MASKED, KS, VS, KS_NEXT, VS_NEXT)                                                          \
    {                                                                                                        \
        const int kv0 = ti.seg_start + j * ST;                                                               \
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);                                                                \
        __syncthreads();                                                                                     \
        if (j + 1 < n_tiles) {                                                                               \
            const long off = (long)(kv0 + ST) * ldkv * 2;                                                    \
            tl.issue(kbase + off, kv_bytes - off, (KS_NEXT), wave);                                          \
            tl.issue(vbase + off, kv_bytes - off, (VS_NEXT), wave);                                          \
        }                                                                                                    \
        _Pragma("unroll") for (int hf = 0; hf < 2; ++hf) {                                                   \
            const int kv_first = kv0 + 32 * hf;                                                              \
            if (!(MASKED)) {                                                                                 \
                if (wave_live)                                                                               \
                    dq_half<D, CAUSAL, false>((KS) + hf * HALF, (VS) + hf * HALF, tl, qf, dof, acc_dq, lse2,  \
                                              dlt, kv_first, ti.seg_end, q_row, sl2);                        \
            } else if (wave_live && kv_first < ti.seg_end && !(CAUSAL && kv_first > wave_q_last))            \
                dq_half<D, CAUSAL, true>((KS) + hf * HALF, (VS) + hf * HALF, tl, qf, dof, acc_dq, lse2, dlt,  \
                                         kv_first, ti.seg_end, q_row, sl2);                                  \
        }                                                                                                    \
        ++j;                                                                                                 \
    }
    while (j + 1 < n_main) {  // two tiles per trip: the stage buffers are compile-time constants
        OB_DQ_ITER(false, ks0, vs0, ks1, vs1)
        OB_DQ_ITER(false, ks1, vs1, ks0, vs0)
    }
#define OB_DQ_ANY(MASKED) OB_DQ_ITER(MASKED, (j & 1) ? ks1 : ks0, (j & 1) ? vs1 : vs0, (j & 1) ? ks0 : ks1, (j & 1) ? vs0 : vs1)
    while (j < n_main) OB_DQ_ANY(false)
    while (j < n_tiles) OB_DQ_ANY(true)
#undef OB_DQ_ANY
#undef OB_DQ_ITER
    if (!q_live) return;
    if (rot_log2_base > 0.f) rotary_bwd_row<D>(acc_dq, q_row - ti.seg_start, rot_log2_base, lh);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc_dq[dt][4 * g + e] * scale);
            *(bf16x4 *)(dq + (size_t)q_row * ldq + head * D + dt * 32 + g * 8 + lh * 4) = ov;
        }
}

// ------------------------------------------------------------------------------------------------
// backward, part 2: dK, dV.  A workgroup owns 128 key rows of one head and streams the segment's
// 64-row query tiles (from the diagonal on when causal).  Its eight wavefronts form four pairs, one
// pair per 32 key rows, and the two waves of a pair split the four products between them:
//   role P (waves 0-3):  S = Q K^T,  P = 2^(scale log2(e) S - lse2),  dV^T += dO^T P
//   role G (waves 4-7):  dP = dO V^T,  dS = P (dP - Delta),           dK^T += Q^T dS
// P travels from the first to the second through LDS in the packed operand layout both use.  Each
// wave keeps half of the state a single wave would need (so two fit on a SIMD and one's MFMAs hide
// the other's element-wise work and LDS waits), and no product is computed twice.  Both roles run
// "row-fragment tile x held rows -> 32x32 scores" and "transposed tile x packed scores -> output";
// role G does the second one tile late (see the kernel), so that it never waits for its partner.
// ------------------------------------------------------------------------------------------------
// scores of a 64-row streamed tile against the 32 held rows: acc[mt] = rows 32 mt .. of the tile
template <int D>
__device__ __forceinline__ void dkv_scores(const unsigned char OB_LDS *__restrict__ tile, const Tile<D> &tl,
                                           const bf16x8 (&held)[D / 16], f32x16 (&acc)[2]) {
    constexpr int HB = D / 32, NB = 2 * (D / 16) / HB, PER = NB / 2;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
    bf16x8 fr[2][HB];
#pragma unroll
    for (int i = 0; i < HB; ++i) fr[0][i] = tl.frag_row(tile, 0, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        if (b + 1 < NB) {
#pragma unroll
            for (int i = 0; i < HB; ++i)
                fr[(b + 1) & 1][i] = tl.frag_row(tile, (b + 1) / PER, ((b + 1) % PER) * HB + i);
        }
#pragma unroll
        for (int i = 0; i < HB; ++i)
            acc[b / PER] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[b & 1][i], held[(b % PER) * HB + i], acc[b / PER], 0, 0, 0);
        if (b + 1 < NB) OB_SCHED_READS_THEN_MFMA(HB, HB); else OB_SCHED_READS_THEN_MFMA(0, HB);
    }
}

// role P: probabilities of the 64 x 32 score tile, packed as the second operands of the four
// 16-row contraction steps (pk[mt][h] serves step 2 mt + h)
template <bool CAUSAL, bool MASK>
__device__ __forceinline__ void dkv_probs(const f32x16 (&s)[2], const float OB_LDS *__restrict__ lse2_s,
                                          int q0, int seg_end, int kv_row, float sl2, bf16x8 (&pk)[2][2]) {
    const int lh = (threadIdx.x & 63) >> 5;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        f32x16 p;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 l4 = *(const f32x4 OB_LDS *)(lse2_s + mt * 32 + 8 * g + 4 * lh);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bool ok = true;
                if (MASK) {
                    const int qr = q0 + mt * 32 + 8 * g + 4 * lh + e;
                    ok = qr < seg_end && (!CAUSAL || kv_row <= qr);
                }
                p[4 * g + e] = ok ? fast_exp2(s[mt][4 * g + e] * sl2 - l4[e]) : 0.f;
            }
        }
        pk[mt][0] = pack8(p, 0);
        pk[mt][1] = pack8(p, 8);
    }
}

// role G: dS = P (dP - Delta), in place of the packed probabilities
__device__ __forceinline__ void dkv_dscores(const f32x16 (&dp)[2], const float OB_LDS *__restrict__ dlt_s,
                                            bf16x8 (&pk)[2][2]) {
    const int lh = (threadIdx.x & 63) >> 5;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        f32x16 ds;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 d4 = *(const f32x4 OB_LDS *)(dlt_s + mt * 32 + 8 * g + 4 * lh);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * g + e;
                ds[r] = (float)pk[mt][r >> 3][r & 7] * (dp[mt][r] - d4[e]);
            }
        }
        pk[mt][0] = pack8(ds, 0);
        pk[mt][1] = pack8(ds, 8);
    }
}

// out^T += tile^T x packed scores, contracting over the tile's 64 rows
template <int D>
__device__ __forceinline__ void dkv_outputs(const unsigned char OB_LDS *__restrict__ tile, const Tile<D> &tl,
                                            const bf16x8 (&pk)[2][2], f32x16 (&acc_out)[D / 32]) {
    constexpr int DT = D / 32;
    bf16x8 tf[2][DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) tf[0][dt] = tl.frag_tr(tile, dt, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < ST / 16; ++u) {
        if (u + 1 < ST / 16) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) tf[(u + 1) & 1][dt] = tl.frag_tr(tile, dt, u + 1);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            acc_out[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[u & 1][dt], pk[u >> 1][u & 1], acc_out[dt], 0, 0, 0);
        if (u + 1 < ST / 16) OB_SCHED_READS_THEN_MFMA(2 * DT, DT); else OB_SCHED_READS_THEN_MFMA(0, DT);
    }
}

// one wave-level load of 64 consecutive floats into LDS (lanes past the end deliver zeros)
__device__ __forceinline__ void issue_row_stats(const float *base, long floats_left,
                                                float OB_LDS *__restrict__ dst, int lane) {
    const uint64_t b = (uint64_t)base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const long cl = floats_left < 0 ? 0 : floats_left * 4;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(((uint64_t)hi << 32) | lo), 0, (int)__builtin_amdgcn_readfirstlane((uint32_t)cl), 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 4, lane * 4, 0, 0, 0);
}

// pairs of waves per workgroup of the dK / dV kernel, each owning 32 key rows: with D = 64 a wave needs few
// enough registers for three on a SIMD, so six pairs (192 key rows) share every streamed tile
constexpr int dkv_pairs(int d) { return d == 64 ? 6 : 4; }
template <int D, bool CAUSAL>
__global__ __launch_bounds__(128 * dkv_pairs(D)) void attn_bwd_dkv_kernel(
    const __bf16 *__restrict__ d_o, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k,
    const __bf16 *__restrict__ v, const float *__restrict__ lse2_all, const float *__restrict__ delta,
    __bf16 *__restrict__ dk, __bf16 *__restrict__ dv, int ldq, int ldkv, int ldo,
    const int32_t *__restrict__ cu, int n_seg, int T, int group, float scale, float rot_log2_base, int heads,
    TileOrder ord) {
    // three stages of the streamed Q and dO tiles (the dK side works one tile behind the dV side, see
    // below), two buffers for the probabilities on their way from one to the other, row statistics
    __shared__ __attribute__((aligned(1024))) unsigned char tiles_s[6 * Tile<D>::BYTES];
    constexpr int NP = dkv_pairs(D), KVT = 32 * NP;                              // pairs; key rows of the workgroup
    __shared__ __attribute__((aligned(1024))) unsigned char p_s[2 * NP * 4096];  // [buffer][pair]: 4 x 64 lanes x 16 B
    __shared__ __attribute__((aligned(256))) float stat_s[6 * ST];              // lse2 x 3 stages, Delta x 3 stages
    __shared__ int sh[8];
    const int rank = blockIdx.x / heads;
    const TileInfo ti = pick_tile(ord, rank, cu, n_seg, KVT, sh);
    if (ti.row0 < 0) return;
    // one workgroup per key/value head: the group's query heads run one after another
    const int kvh = head_of_slot(blockIdx.x - rank * heads, heads);
    const int lane = threadIdx.x & 63, lx = lane & 31, lh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool role_g = wave >= NP;  // false: S, P, dV;  true: dP, dS, dK
    const int pair = role_g ? wave - NP : wave;
    const int kv_row = min(ti.row0 + pair * 32 + lx, ti.seg_end - 1);
    const bool kv_live = ti.row0 + pair * 32 + lx < ti.seg_end;
    const int pair_kv_first = ti.row0 + pair * 32;
    const float sl2 = scale * LOG2E;
    constexpr int KT = D / 16, DT = D / 32;

    // the wave copies the tile it reads row fragments from: Q (role P) or dO (role G)
    Tile<D> tl;
    tl.init(role_g ? ldo : ldq, pair, lane);
    const unsigned char *const own_base = role_g ? (const unsigned char *)d_o : (const unsigned char *)q;
    const long own_ld2 = (role_g ? (long)ldo : (long)ldq) * 2;
    const long own_total = (long)T * own_ld2;

    // held rows: K (role P) or V (role G)
    bf16x8 kvf[KT];
    {
        const __bf16 *src = (role_g ? v : k) + (size_t)kv_row * ldkv + kvh * D + 8 * lh;
#pragma unroll
        for (int t = 0; t < KT; ++t) kvf[t] = *(const bf16x8 *)(src + 16 * t);
    }
    f32x16 acc_out[DT];  // dV^T (role P) or dK^T (role G)
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_out[i][r] = 0.f;

    constexpr int BYTES = Tile<D>::BYTES;
    unsigned char OB_LDS *const tiles = (unsigned char OB_LDS *)tiles_s;
    float OB_LDS *const stats = (float OB_LDS *)stat_s;
#define OB_QS(S) (tiles + (S) * BYTES)
#define OB_DOS(S) (tiles + (3 + (S)) * BYTES)
#define OB_LSES(S) (stats + (S) * ST)
#define OB_DLTS(S) (stats + (3 + (S)) * ST)
    unsigned char OB_LDS *const p_mine = (unsigned char OB_LDS *)p_s + pair * 4096 + lane * 16;

    // causal: query rows before this workgroup's first key row see none of its keys
    const int q_begin = CAUSAL ? ti.seg_start + ((ti.row0 - ti.seg_start) / ST) * ST : ti.seg_start;
    const int n_iter = (ti.seg_end - q_begin + ST - 1) / ST;
#define OB_ISSUE_DKV(hq_, it_, S)                                                                             \
    do {                                                                                                      \
        const int head_ = kvh * group + (hq_);                                                                \
        const int q0_ = q_begin + (it_) * ST;                                                                 \
        const long off_ = (long)q0_ * own_ld2 + (long)head_ * D * 2;                                          \
        /* four waves of each role copy a tile */                                                            \
        if (pair < 4) tl.issue(own_base + off_, own_total - off_, role_g ? OB_DOS(S) : OB_QS(S), pair);       \
        if (wave == 0) issue_row_stats(lse2_all + (size_t)head_ * T + q0_, (long)T - q0_, OB_LSES(S), lane);  \
        if (wave == NP) issue_row_stats(delta + (size_t)head_ * T + q0_, (long)T - q0_, OB_DLTS(S), lane);    \
    } while (0)
    // causal: only the first KVT / ST query tiles touch some pair's diagonal; either way only the last
    // tile can be ragged.  The tiles in between need no mask.
    const int n_head = CAUSAL ? min(KVT / ST, n_iter) : 0;
    const int n_mid_end = max(n_head, n_iter - (((ti.seg_end - q_begin) % ST) ? 1 : 0));
    // Order of work: first the masked tiles of every query head of the group (phase 0), then the
    // mask-free ones of every head (phase 1) in one single-path loop -- the sums do not care, and one
    // loop nest per phase keeps the accumulators in place (a loop over the heads around the per-head
    // loops made the register allocator spill them).  A cursor names a tile: (phase, head in group, j).
    const int cnt0 = n_head + (n_iter - n_mid_end), cnt1 = n_mid_end - n_head;
    struct Cursor { int phase, hq, j; };
    auto tile_of = [&](const Cursor &c) { return c.phase ? n_head + c.j : (c.j < n_head ? c.j : n_mid_end + c.j - n_head); };
    auto step = [&](Cursor &c) {   // to the next tile in the order of work; phase 2 = past the end
        const int cnt = c.phase ? cnt1 : cnt0;
        if (c.j + 1 < cnt) { ++c.j; return; }
        c.j = 0;
        if (c.hq + 1 < group) { ++c.hq; return; }
        c.hq = 0;
        ++c.phase;
        if (c.phase == 1 && cnt1 == 0) c.phase = 2;
    };
    // the whole walk once per role, chosen outside the loops: each role's loop then carries only its own
    // registers (role G keeps dP across trips, role P does not)
    auto walk = [&](auto role_tag) {
    constexpr bool RG = decltype(role_tag)::value;
    Cursor cur = {0, 0, 0};
    if (cnt0 == 0) cur.phase = cnt1 ? 1 : 2;
    Cursor nxt = cur;
    step(nxt);
    OB_ISSUE_DKV(cur.hq, tile_of(cur), 0);
    // The dK side runs one tile behind: in the trip of tile n the role-P wave does S, P, dV of tile n
    // and leaves P in buffer n % 2, while the role-G wave first finishes tile n - 1 (dS from the P it
    // finds in buffer (n - 1) % 2 and the dP it kept in registers, then dK) and then forms dP of tile
    // n.  One barrier per tile instead of two, the role-G wave never waits for its partner inside a
    // trip, and the two waves of a SIMD start a trip in different kinds of work (MFMAs / element-wise).
    // Stage n % 3 holds tile n: the load of tile n + 1 overwrites tile n - 2, which nobody needs any more.
    int gi = 0, st = 0;        // tiles done; stage of the current tile
    int left1 = group * cnt1;  // mask-free tiles not yet done
    bool live_prev = false;    // role G: tile n - 1 took part
    f32x16 dp_keep[2];         // role G: dP of tile n - 1
#define OB_DKV_ITER(MASKED, S, PREV, NEXT)                                                                   \
    {                                                                                                       \
        const int q0 = q_begin + tile_of(cur) * ST;                                                         \
        __builtin_amdgcn_s_waitcnt(WAIT_VM0);                                                               \
        __syncthreads();                                                                                    \
        if (nxt.phase < 2) OB_ISSUE_DKV(nxt.hq, tile_of(nxt), NEXT);                                        \
        /* a masked tile entirely before this pair's keys contributes nothing */                            \
        const bool live = !((MASKED) && CAUSAL && q0 + ST - 1 < pair_kv_first);                             \
        if constexpr (!RG) {                                                                                \
            if (live) {                                                                                     \
                f32x16 acc_x[2];                                                                            \
                bf16x8 pk[2][2];                                                                            \
                dkv_scores<D>(OB_QS(S), tl, kvf, acc_x);                                                    \
                dkv_probs<CAUSAL, MASKED>(acc_x, OB_LSES(S), q0, ti.seg_end, kv_row, sl2, pk);              \
                _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                            \
                    *(bf16x8 OB_LDS *)(p_mine + (gi & 1) * (NP * 4096) + i_ * 1024) = pk[i_ >> 1][i_ & 1];        \
                dkv_outputs<D>(OB_DOS(S), tl, pk, acc_out);                                                 \
            }                                                                                               \
        } else {                                                                                            \
            if (live_prev) {                                                                                \
                bf16x8 pk[2][2];                                                                            \
                _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                            \
                    pk[i_ >> 1][i_ & 1] = *(const bf16x8 OB_LDS *)(p_mine + ((gi - 1) & 1) * (NP * 4096) + i_ * 1024); \
                dkv_dscores(dp_keep, OB_DLTS(PREV), pk);                                                    \
                dkv_outputs<D>(OB_QS(PREV), tl, pk, acc_out);                                               \
            }                                                                                               \
            if (live) dkv_scores<D>(OB_DOS(S), tl, kvf, dp_keep);                                           \
            live_prev = live;                                                                               \
        }                                                                                                   \
        if (cur.phase == 1) --left1;                                                                        \
        cur = nxt;                                                                                          \
        step(nxt);                                                                                          \
        ++gi;                                                                                               \
        st = (NEXT);                                                                                        \
    }
#define OB_DKV_ANY(MASKED)                                                                                   \
    {                                                                                                       \
        const int s_ = st, p_ = st == 0 ? 2 : st - 1, n_ = st == 2 ? 0 : st + 1;                            \
        OB_DKV_ITER(MASKED, s_, p_, n_)                                                                     \
    }
    while (cur.phase == 0) OB_DKV_ANY(true)
    while (st != 0 && cur.phase == 1) OB_DKV_ANY(false)   // the three-tile loop below starts on stage 0
    while (left1 >= 3) {  // three tiles per trip: constant stage addresses, a single straight path
        OB_DKV_ITER(false, 0, 2, 1)
        OB_DKV_ITER(false, 1, 0, 2)
        OB_DKV_ITER(false, 2, 1, 0)
    }
    while (cur.phase == 1) OB_DKV_ANY(false)
    // the dK side still owes the last tile
    __syncthreads();
    if (RG && live_prev) {
        const int p_ = st == 0 ? 2 : st - 1;
        bf16x8 pk[2][2];
#pragma unroll
        for (int i_ = 0; i_ < 4; ++i_)
            pk[i_ >> 1][i_ & 1] = *(const bf16x8 OB_LDS *)(p_mine + ((gi - 1) & 1) * (NP * 4096) + i_ * 1024);
        dkv_dscores(dp_keep, OB_DLTS(p_), pk);
        dkv_outputs<D>(OB_QS(p_), tl, pk, acc_out);
    }
    };
    if (role_g) walk(std::true_type{}); else walk(std::false_type{});
#undef OB_DKV_ANY
#undef OB_DKV_ITER
#undef OB_ISSUE_DKV
#undef OB_DLTS
#undef OB_LSES
#undef OB_DOS
#undef OB_QS
    if (!kv_live) return;
    // dV^T / dK^T of the whole group of query heads sit in the accumulators: one rounding to bf16
    const float out_scale = role_g ? scale : 1.0f;
    __bf16 *const dst = role_g ? dk : dv;
    if (role_g && rot_log2_base > 0.f) rotary_bwd_row<D>(acc_out, kv_row - ti.seg_start, rot_log2_base, lh);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 ov;
#pragma unroll
            for (int e = 0; e < 4; ++e) ov[e] = (__bf16)(acc_out[dt][4 * g + e] * out_scale);
            *(bf16x4 *)(dst + (size_t)kv_row * ldkv + kvh * D + dt * 32 + g * 8 + lh * 4) = ov;
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

// Order of work of a launch whose workgroups own `tile_rows` rows of a segment and stream 64-row
// tiles of the other side: descending number of streamed tiles, ties in natural order.  `kv_side`:
// the workgroup owns key rows and streams query tiles (from its diagonal on when causal); otherwise
// it owns query rows and streams key tiles (up to its diagonal when causal).  No heap memory.
void make_order(const ob_segments *seg, int tile_rows, bool causal, bool kv_side, int n_tiles, TileOrder &ord) {
    ord.n = 0;
    if (n_tiles > TileOrder::CAP || seg->n_seg > 0xFFFF) return;
    uint64_t key[TileOrder::CAP];
    int n = 0;
    for (int j = 0; j < seg->n_seg; ++j) {
        const int a = seg->cu_host[j], len = seg->cu_host[j + 1] - a;
        const int nt = (len + tile_rows - 1) / tile_rows;
        if (nt > 0xFFFF) return;
        for (int t = 0; t < nt; ++t) {
            int rows = len;                                            // streamed rows
            if (causal && kv_side) rows = len - (t * tile_rows) / ST * ST;
            else if (causal) rows = std::min(len, (t + 1) * tile_rows);
            const uint32_t w = (uint32_t)((rows + ST - 1) / ST);
            // ascending sort of (~work, natural index); the entry rides in the low half
            key[n] = ((uint64_t)(0xFFFFFu - w) << 44) | ((uint64_t)n << 32) | ((uint32_t)j << 16) | (uint32_t)t;
            ++n;
        }
    }
    std::sort(key, key + n);
    for (int i = 0; i < n; ++i) ord.e[i] = (uint32_t)key[i];
    ord.n = n;
}

// explicit instantiations (the host pass otherwise drops launch stubs of kernels reached only
// through the dispatch macro below)
#define OB_ATTN_INSTANCES(D, C)                                                                               \
    template __global__ void attn_fwd_kernel<D, C>(const __bf16 *, const __bf16 *, const __bf16 *, __bf16 *,  \
                                                   float *, int, int, int, const int32_t *, int, int, int,    \
                                                   float, int, TileOrder);                                    \
    template __global__ void attn_bwd_dq_kernel<D, C>(const __bf16 *, const __bf16 *, const __bf16 *,         \
                                                      const __bf16 *, const __bf16 *, const float *, float *, \
                                                      float *, __bf16 *, int, int, int, const int32_t *, int, \
                                                      int, int, float, float, int, TileOrder);                \
    template __global__ void attn_bwd_dkv_kernel<D, C>(const __bf16 *, const __bf16 *, const __bf16 *,        \
                                                       const __bf16 *, const float *, const float *,          \
                                                       __bf16 *, __bf16 *, int, int, int,                     \
                                                       const int32_t *, int, int, int, float, float, int,     \
                                                       TileOrder);
OB_ATTN_INSTANCES(64, true)
OB_ATTN_INSTANCES(64, false)
OB_ATTN_INSTANCES(128, true)
OB_ATTN_INSTANCES(128, false)
#undef OB_ATTN_INSTANCES

}  // namespace

#define OB_ATTN_DISPATCH(KERNEL, GRID, THREADS, ...)                                                      \
    do {                                                                                           \
        if (d == 64 && causal)                                                                     \
            hipLaunchKernelGGL((KERNEL<64, true>), GRID, dim3(THREADS), 0, s, __VA_ARGS__);            \
        else if (d == 64)                                                                          \
            hipLaunchKernelGGL((KERNEL<64, false>), GRID, dim3(THREADS), 0, s, __VA_ARGS__);           \
        else if (causal)                                                                           \
            hipLaunchKernelGGL((KERNEL<128, true>), GRID, dim3(THREADS), 0, s, __VA_ARGS__);           \
        else                                                                                       \
            hipLaunchKernelGGL((KERNEL<128, false>), GRID, dim3(THREADS), 0, s, __VA_ARGS__);          \
    } while (0)

void launch_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int ldq,
                     int ldkv, int ldo, const ob_segments *seg, int nq, int nkv, int d, float scale,
                     int mask, hipStream_t s) {
    const bool causal = mask == OB_MASK_SEG_CAUSAL;
    ProfScope prof(K_ATTN_FWD, s, attn_flops(seg, nq, d, causal));
    const int tiles = count_tiles(seg, QT);
    TileOrder ord;
    make_order(seg, QT, causal, false, tiles, ord);
    const dim3 grid((unsigned)tiles * nq);
OB_ATTN_DISPATCH(attn_fwd_kernel, grid, 256, (const __bf16 *)q, (const __bf16 *)k, (const __bf16 *)v,
                     (__bf16 *)o, lse, ldq, ldkv, ldo, seg->cu_dev, seg->n_seg, seg->total_tokens,
                     nq / nkv, scale, nq, ord);
}

void launch_attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const void *o, const float *lse,
                     float *lse2, float *delta, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                     const ob_segments *seg, int nq, int nkv, int d, float scale, int mask, float rotary_base,
                     hipStream_t s) {
    const bool causal = mask == OB_MASK_SEG_CAUSAL;
    const int tiles = count_tiles(seg, QT);
    const int T = seg->total_tokens, group = nq / nkv;
    const float rot = rotary_base > 1.f ? log2f(rotary_base) : 0.f;
    {
        // dQ = dS K: 1 of the 4 backward products; the kernel also forms Delta and the base-2 log-sum-exp
        ProfScope prof(K_ATTN_BWD_DQ, s, 0.5 * attn_flops(seg, nq, d, causal));
        TileOrder ord;
        make_order(seg, QT, causal, false, tiles, ord);
        const dim3 grid_q((unsigned)tiles * nq);
        OB_ATTN_DISPATCH(attn_bwd_dq_kernel, grid_q, 256, (const __bf16 *)d_o, (const __bf16 *)q,
                         (const __bf16 *)k, (const __bf16 *)v, (const __bf16 *)o, lse, lse2, delta, (__bf16 *)dq, ldq,
                         ldkv, ldo, seg->cu_dev, seg->n_seg, seg->total_tokens, nq / nkv, scale, rot, nq, ord);
    }
    ProfScope prof(K_ATTN_BWD_DKV, s, 1.5 * attn_flops(seg, nq, d, causal));  // dV, dP, dK
    TileOrder ord;
    const int kvt = 32 * dkv_pairs(d), tiles_kv = count_tiles(seg, kvt);
    make_order(seg, kvt, causal, true, tiles_kv, ord);
    const dim3 grid_kv((unsigned)tiles_kv * nkv);
    OB_ATTN_DISPATCH(attn_bwd_dkv_kernel, grid_kv, 4 * kvt, (const __bf16 *)d_o, (const __bf16 *)q,
                     (const __bf16 *)k, (const __bf16 *)v, lse2, delta, (__bf16 *)dk, (__bf16 *)dv, ldq, ldkv,
                     ldo, seg->cu_dev, seg->n_seg, T, group, scale, rot, nkv, ord);
}

}  // namespace ob
