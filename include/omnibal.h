/*
 * omnibal.h -- C ABI of the MI355X (gfx950) hot path behind OmniBal-style balanced VLM training:
 * forward + backward of pre-norm transformer blocks over ONE packed, padding-free,
 * variable-length mini-batch, plus the host-side balanced grouping that produces the batch.
 *
 * What the paper fixes: samples stay whole and a mini-batch carries no padding (Sec. 3 "Data
 * Imbalance"; Sec. 4.1; Table 3, ISF row: PadRatio 0), the grouping algorithm (Alg. 1) and its
 * metrics (Eq. 1, Eq. 2).  The block arithmetic is the textbook pre-norm transformer block:
 *     x1 = x  + Attn(N1(x)) W_o^T (+ b_o)        y = x1 + MLP(N2(x1))
 * with attention confined to each segment of the packed batch: one ViT image tile (bidirectional)
 * or one LLM sample (causal), rotary positions restarting at 0 in every segment.
 *
 * Conventions for every device entry point
 *   - All tensor pointers are DEVICE pointers unless the name ends in _host.  The caller owns every
 *     buffer; the library never allocates or frees device memory, never synchronises, never
 *     changes the current device.  All work is enqueued on `hip_stream` (a hipStream_t cast to
 *     void*; NULL = the default stream).
 *   - Tensors are dense row-major.  Activations [T, H]; weights [out_features, in_features];
 *     bf16 storage (OB_BF16) with fp32 accumulation; row statistics and log-sum-exp are fp32.
 *     OB_FP32 selects the debug path of the attention and block entry points: every tensor
 *     (activations, weights, gradients, saved members) is fp32 and every product is a plain
 *     fp32 FMA loop: slow, no MFMA, meant for checking against the oracle at 1e-4.
 *   - Every call validates its arguments on the host first and returns a non-zero ob_status
 *     WITHOUT launching anything when validation fails.  ob_last_error() gives the text.
 *   - Feature dimensions (hidden, mlp_dim, head_dim * heads) must be multiples of 64; head_dim
 *     must be 64 or 128; the token count T is arbitrary (1 .. 2^22).
 */
#ifndef OMNIBAL_H
#define OMNIBAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OB_OK = 0,
    OB_EINVAL = 1,       /* null pointer, non-positive size, inconsistent head counts ...      */
    OB_ESEGMENTS = 2,    /* cu_seqlens not starting at 0, not strictly increasing, wrong total  */
    OB_EUNSUPPORTED = 3, /* head_dim not in {64,128}, dimension not a multiple of 64             */
    OB_EWORKSPACE = 4,   /* workspace / saved buffer smaller than the query functions report    */
    OB_EHIP = 5          /* a HIP launch failed; text in ob_last_error()                         */
} ob_status;

typedef enum { OB_BF16 = 0, OB_FP32 = 1 } ob_dtype;
typedef enum { OB_MASK_SEG_BIDIR = 0, OB_MASK_SEG_CAUSAL = 1 } ob_mask;
typedef enum { OB_LAYERNORM = 0, OB_RMSNORM = 1 } ob_norm;
typedef enum { OB_GELU = 0, OB_SWIGLU = 1 } ob_mlp;

/* One block's static description.  has_bias: all four linears carry a bias and (LayerNorm only)
 * the norms carry beta; otherwise every bias/beta pointer is ignored and may be NULL. */
typedef struct {
    int hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim;
    int norm;          /* ob_norm  */
    int mlp;           /* ob_mlp   */
    int mask;          /* ob_mask  */
    int dtype;         /* ob_dtype */
    int use_rotary;    /* rotate q,k pairs (i, i+d/2) by pos * base^(-2i/d), pos = t - cu[seg(t)] */
    float rotary_base;
    float norm_eps;
    int has_bias;
} ob_block_desc;

/* Weights [out, in]: w_qkv [(nq+2nkv)d, H] rows ordered q heads | k heads | v heads;
 * w_o [H, nq d]; w_up [F, H] (GELU) or [2F, H] = gate rows then up rows (SwiGLU); w_down [H, F].
 * Norm gains n?_g [H] (bf16), betas n?_b [H]. */
typedef struct {
    const void *n1_g, *n1_b, *w_qkv, *b_qkv, *w_o, *b_o, *n2_g, *n2_b, *w_up, *b_up, *w_down, *b_down;
} ob_block_weights;
typedef struct {
    void *n1_g, *n1_b, *w_qkv, *b_qkv, *w_o, *b_o, *n2_g, *n2_b, *w_up, *b_up, *w_down, *b_down;
} ob_block_grads;

/* Segment layout of one packed mini-batch: cu[0] = 0 < cu[1] < ... < cu[n_seg] = total_tokens.
 * cu_host is read during validation and launch planning; cu_dev must hold the same n_seg+1
 * int32 values in device memory.  max_seqlen >= the longest segment. */
typedef struct {
    const int32_t *cu_host;
    const int32_t *cu_dev;
    int n_seg, total_tokens, max_seqlen;
} ob_segments;

const char *ob_last_error(void);
/* 1 when the library was built with its gfx950 kernels (always, for the shipped build). */
int ob_has_device_code(void);

/* ---- opt-in per-kernel timing for the bench's roofline lines ----------------------------------
 * Between ob_prof_begin and ob_prof_end every kernel the library launches is bracketed by a pair
 * of HIP events on its own stream.  ob_prof_end waits for them and returns, per kernel class
 * (ob_prof_class_name), the summed duration in ms, the launch count and the summed algorithmic
 * work (FLOPs for the MFMA classes gemm / attn_*, bytes for the HBM-bound classes).  Not thread
 * safe; at most max_launches launches are recorded (more -> OB_EWORKSPACE from ob_prof_end). */
int ob_prof_num_classes(void);
const char *ob_prof_class_name(int cls);
int ob_prof_begin(int max_launches);
int ob_prof_end(double *ms_per_class, int64_t *launches_per_class, double *work_per_class,
                int n_classes);

/* ---- varlen attention (step a4 / b4 of the block) --------------------------------------------
 * For query head a, KV head a / (nq / nkv):  S_ij = scale * q_i . k_j;  allowed(i, j) <=>
 * same segment (and j <= i when causal);  o_i = sum_j softmax_j(S_ij) v_j over allowed j;
 * lse[a, i] = log sum_j exp(S_ij) (natural log), layout [nq, T] fp32.
 * q, o, d_o, dq: rows of nq*d elements with row strides ldq / ldo (in elements); k, v, dk, dv:
 * rows of nkv*d elements with row stride ldkv -- so q,k,v may be column slices of one
 * [T, (nq+2nkv) d] buffer.  Cross-segment score tiles are never computed.
 * The backward needs ob_varlen_attn_bwd_workspace_bytes() bytes of scratch: Delta_i = sum_d dO_i O_i
 * and the log-sum-exp in base-2 units ([nq, T] fp32 each).  With nq > nkv the workgroup that owns a
 * tile of key rows walks the query heads of its group in order and keeps dK / dV in registers
 * (no atomics, no partial sums in memory: results are bitwise reproducible). */
int ob_varlen_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
                       int ldq, int ldkv, int ldo, const ob_segments *seg, int nq, int nkv, int d,
                       float scale, int mask, int dtype, void *hip_stream);
size_t ob_varlen_attn_bwd_workspace_bytes(int total_tokens, int nq, int nkv, int d);
int ob_varlen_attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const void *o,
                       const float *lse, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                       const ob_segments *seg, int nq, int nkv, int d, float scale, int mask,
                       int dtype, void *ws, size_t ws_bytes, void *hip_stream);

/* The same backward for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Its scratch is a static
 * device array of OB_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the
 * process ends); the call allocates and frees nothing.  Limit: total_tokens * n_q_heads * 8 bytes
 * (rounded up to 512) must fit the array (4 Mi query-head rows: e.g. 32768 tokens x 128 heads);
 * beyond it the call returns OB_EWORKSPACE without launching anything.  Inputs, outputs and results
 * are those of ob_varlen_attn_bwd.  All calls on one GPU share that GPU's array: calls that overlap
 * in time on one GPU (different streams or threads) race; serialise them. */
#define OB_STATIC_SCRATCH_BYTES (32u << 20)
int ob_varlen_attn_bwd_static(const void *d_o, const void *q, const void *k, const void *v, const void *o,
                              const float *lse, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                              const ob_segments *seg, int nq, int nkv, int d, float scale, int mask,
                              int dtype, void *hip_stream);

/* ---- one transformer block (steps a1..a9 / b9..b1) -------------------------------------------
 * ob_block_fwd:  y = Block(x); keeps in `saved` (ob_block_saved_bytes) what the backward needs.
 * ob_block_bwd:  given dy, the same x, weights and `saved`, writes dx and every weight gradient
 * (bf16, after fp32 accumulation).  `flags` is a bit set:
 *   OB_BWD_ACCUMULATE  add into the existing gradient buffers instead of overwriting them;
 *   OB_BWD_RECOMPUTE   re-computation (Sec. 4.3): `saved` need not hold this block's forward data
 *                      (one buffer may serve every block); the forward is replayed from x into it
 *                      first (every step but the last GEMM), then the backward runs as usual, so
 *                      the results are bit-identical to the non-recomputed ones.
 * x/y and dy/dx may not alias each other or `saved`/`ws`.  Besides the activations, `saved` holds
 * the scratch of the forward GEMMs (the slice sums of split contractions, see ob_gemm_bf16), `ws`
 * that of the backward GEMMs: both are counted in the two size functions. */
enum { OB_BWD_ACCUMULATE = 1, OB_BWD_RECOMPUTE = 2 };
size_t ob_block_saved_bytes(const ob_block_desc *desc, int total_tokens);
size_t ob_block_workspace_bytes(const ob_block_desc *desc, int total_tokens);
int ob_block_fwd(const ob_block_desc *desc, const ob_block_weights *w, const void *x, void *y,
                 void *saved, size_t saved_bytes, const ob_segments *seg, void *ws, size_t ws_bytes,
                 void *hip_stream);
int ob_block_bwd(const ob_block_desc *desc, const ob_block_weights *w, const ob_block_grads *g,
                 int flags, const void *x, const void *dy, void *dx, void *saved,
                 size_t saved_bytes, const ob_segments *seg, void *ws, size_t ws_bytes,
                 void *hip_stream);

/* Views into `saved` for tests and profiling: byte offset of a named intermediate
 * ("h1","qkv","o","lse","x1","h2","up","act","stat1","stat2"); returns (size_t)-1 if unknown. */
size_t ob_block_saved_offset(const ob_block_desc *desc, int total_tokens, const char *name);

/* ---- building blocks exposed for tests and the bench's per-kernel roofline lines --------------
 * C[M,N] = op(A) op(B) (+ bias[N]) (+ R[M,N]), bf16 in / fp32 accumulate / bf16 out.
 *   layout 0 ("NT"): A [M,K], B [N,K]        -- forward  y = a W^T
 *   layout 1 ("NN"): A [M,K], B [K,N]        -- dgrad    da = dy W
 *   layout 2 ("TN"): A [K,M], B [K,N]        -- wgrad    dW = dy^T a   (K = tokens)
 * `R` may equal `C` (in-place accumulate).  N and the feature side of K must be multiples of 64.
 * All three layouts run natively (a K-major operand is transposed by the LDS read).
 * The output tiles of an incomplete last round of the chip (all tiles, for the weight gradients of
 * a narrow model) may have their contraction split along K: the slices leave fp32 sums in `ws`
 * (device memory, ob_gemm_workspace_bytes() bytes: 0 for a GEMM that is not split, never more than
 * 510 MiB) and a second kernel adds them, bias and R in a fixed order.  ws == NULL: the GEMM runs
 * unsplit, whatever its shape; a non-NULL ws of fewer bytes than that is OB_EWORKSPACE. */
size_t ob_gemm_workspace_bytes(int layout, int M, int N, int K);
int ob_gemm_bf16(int layout, int M, int N, int K, const void *A, const void *B, void *C,
                 const void *bias, const void *R, void *ws, size_t ws_bytes, void *hip_stream);

/* ---- ViT -> LLM hand-over of a mixed stage (App. A; the "token sub-sampling" of Sec. 5.4) ------
 * The paper names the step but fixes neither it nor the connector; what runs here is
 *   c1  per tile of grid*grid + 1 ViT rows (class token first, patches row-major): drop the class
 *       token; sub-sampled token (r, c), r, c < grid/2, is the channel-wise concatenation of the
 *       patches (2r + dr, 2c + dc), channel block 2 dr + dc   -> [n_tok, 4 Hv], n_tok = n_tiles grid^2/4
 *   c2  LayerNorm over the 4 Hv channels (n_g, n_b)
 *   c3  h = un W1^T + b1,  a = GELU(h)            w1 [Ht, 4 Hv]
 *   c4  z = a W2^T + b2                            w2 [Ht, Ht]
 *   c5  row i of z is written to row dst_rows[i] of x_llm [llm_tokens, Ht]; other rows (text) are
 *       left as the caller filled them.
 * dst_rows (int32, n_tok entries, host and device copies like cu_seqlens) must be distinct and
 * inside [0, llm_tokens): checked on the host.  dtype OB_BF16, or OB_FP32 for the debug variant
 * (every tensor, weight and gradient fp32; plain kernels, same steps); vit_hidden and
 * llm_hidden multiples of 64, 4 vit_hidden <= 16384, grid even.
 * ob_connector_bwd: given dx_llm [llm_tokens, Ht] it reads the rows dst_rows, writes every row of
 * dv [n_tiles (grid^2 + 1), Hv] (class rows: zeros) and all six weight gradients (flags:
 * OB_BWD_ACCUMULATE only).  `saved` carries un, h, a and the row statistics from the forward. */
typedef struct {
    int vit_hidden, llm_hidden, grid;
    int dtype;         /* ob_dtype */
    float norm_eps;
} ob_connector_desc;
typedef struct { const void *n_g, *n_b, *w1, *b1, *w2, *b2; } ob_connector_weights;
typedef struct { void *n_g, *n_b, *w1, *b1, *w2, *b2; } ob_connector_grads;
size_t ob_connector_saved_bytes(const ob_connector_desc *desc, int n_tiles);
size_t ob_connector_workspace_bytes(const ob_connector_desc *desc, int n_tiles);
int ob_connector_fwd(const ob_connector_desc *desc, const ob_connector_weights *w, const void *v,
                     int n_tiles, const int32_t *dst_rows_host, const int32_t *dst_rows_dev,
                     void *x_llm, int llm_tokens, void *saved, size_t saved_bytes, void *ws,
                     size_t ws_bytes, void *hip_stream);
int ob_connector_bwd(const ob_connector_desc *desc, const ob_connector_weights *w,
                     const ob_connector_grads *g, int flags, const void *v, const void *dx_llm,
                     void *dv, int n_tiles, const int32_t *dst_rows_host,
                     const int32_t *dst_rows_dev, int llm_tokens, const void *saved,
                     size_t saved_bytes, void *ws, size_t ws_bytes, void *hip_stream);

/* T x T byte mask (1 = allowed): allowed(i, j) <=> i and j lie in the same segment (and j <= i when
 * causal), evaluated per entry from cu_seqlens by a small kernel of its own (the attention kernels
 * never form the mask: they tile each segment separately and compare row indices inside the
 * diagonal and ragged tiles).  For bit-exact tests of the segment layout, T <= 4096. */
int ob_debug_materialize_mask(const ob_segments *seg, int mask, uint8_t *mask_dev, void *hip_stream);

/* ---- host side: balanced dynamic mini-batches (Alg. 1, ISF) -----------------------------------
 * Inputs: per-sample image-tile count n_img[i] = |x_i| and LLM-side token count n_tok[i] = |y_i|.
 * Sampling stage: walk a random permutation of the not-yet-grouped samples, appending to the
 * open group until the tile total would exceed Qv or the token total would exceed Qt; the group
 * still open at the end is a candidate too.  Filtering stage: a candidate is accepted iff its
 * tile total >= Qv_min or its token total >= Qt_min; accepted samples leave the pool.  Repeated
 * `iters` times (Sec. 4.1; 10 in App. G).  randperm = Fisher-Yates (i = n-1..1, j uniform in
 * [0, i] by rejection) over splitmix64 seeded with seed + iteration; the pool is kept in
 * ascending sample-id order between iterations.
 * Outputs (host arrays, caller-allocated): group_offsets[n_samples+1], sample_ids[n_samples]
 * (group g = sample_ids[group_offsets[g] .. group_offsets[g+1])), leftover_ids[n_samples],
 * groups_per_iter[iters] (may be NULL).  A sample with n_img > Qv or n_tok > Qt -> OB_EINVAL. */
int ob_pack_isf(const int32_t *n_img, const int32_t *n_tok, int64_t n_samples, int64_t Qv,
                int64_t Qt, int64_t Qv_min, int64_t Qt_min, int iters, uint64_t seed,
                int64_t *group_offsets, int64_t *n_groups, int64_t *sample_ids,
                int64_t *leftover_ids, int64_t *n_leftover, int64_t *groups_per_iter);
/* Baseline arm (Sec. 5.4, method 1): consecutive runs of B samples of one random permutation. */
int ob_pack_random(int64_t n_samples, int64_t B, uint64_t seed, int64_t *group_offsets,
                   int64_t *n_groups, int64_t *sample_ids, int64_t *leftover_ids,
                   int64_t *n_leftover);
/* Sec. 5.4, method 2 (Length-Group): samples sorted by token count (ties by id), cut into runs of
 * B, the mini-batches then put in a seeded random order.  Method 3 (Device-Group): the random
 * arm's mini-batches ordered by their token totals, so consecutive mini-batches (the ones a step
 * hands to its devices) are close in size.  Outputs as for ob_pack_random. */
int ob_pack_length_group(const int32_t *n_tok, int64_t n_samples, int64_t B, uint64_t seed,
                         int64_t *group_offsets, int64_t *n_groups, int64_t *sample_ids,
                         int64_t *leftover_ids, int64_t *n_leftover);
int ob_pack_device_group(const int32_t *n_tok, int64_t n_samples, int64_t B, uint64_t seed,
                         int64_t *group_offsets, int64_t *n_groups, int64_t *sample_ids,
                         int64_t *leftover_ids, int64_t *n_leftover);
/* Segment offsets of one packed mini-batch: one segment per sample (LLM) / per tile (ViT). */
int ob_build_cu_seqlens_llm(const int64_t *group_ids, int64_t n, const int32_t *n_tok,
                            int32_t *cu_out, int32_t *max_seqlen_out);
int ob_build_cu_seqlens_vit(int64_t n_tiles, int32_t tile_len, int32_t *cu_out);
/* Eq. 1 and Eq. 2 (same form): sum_i (max - v_i) / (max * n). */
double ob_pad_ratio(const int64_t *tokens_per_sample, int64_t n);
double ob_dist_ratio(const int64_t *tokens_per_minibatch, int64_t n);


/* ---- host side: adaptive re-computation, Step 4 (Sec. 4.3) -----------------------------------
 * With re-computation on everywhere a stage has free_bytes (M_r) left; keeping the activations of
 * one ViT / LLM layer costs saved_bytes_vit / saved_bytes_llm (M_v / M_t, e.g.
 * ob_block_saved_bytes) and saves that layer's forward replay (fwd_ms_*).  Returns the counts of
 * layers that may skip re-computation: the pair that saves the most replay time within the budget
 * (ties: fewer bytes, then fewer ViT layers).  Each failed trial run of the caller adds one to
 * extra_recompute: one more kept layer is given up, the kind with the larger footprint first. */
int ob_recompute_plan(int64_t free_bytes, int n_vit, int64_t saved_bytes_vit, double fwd_ms_vit,
                      int n_llm, int64_t saved_bytes_llm, double fwd_ms_llm, int extra_recompute,
                      int *keep_vit, int *keep_llm);

/* ---- host side: balanced model partitioning (Sec. 4.2) ---------------------------------------
 * Layers are numbered 1..L, the pipeline has N stages, a partition is P = (P1 < ... < P(N-1)) with
 * P0 = 1 and PN = L + 1; stage i holds layers P(i-1) <= l < P(i).  fwd_ms[l-1] = profiled forward
 * time of layer l, activ[l-1] = size of its output activation (the volume sent if a cut follows).
 * ob_bmp_anchor: greedy anchor P+, cut i where the running time is closest to i/N of the total
 * among positions that leave every stage a layer (ties: the earlier).  P_out[N-1].
 * ob_bmp_search: every partition within radius r of the anchor that is valid (n_candidates of
 * them; 27 for r = 1, N = 4 when none falls off the ends), scored by
 *   VAR(fwd_time) + comm_weight * SUM(comm)      (Eq. 4 + Eq. 5; the variance as printed, no 1/N)
 * and the top_k lowest returned in ascending order (ties: lexicographic in P):
 * cand_out[top_k][N-1], score_out[top_k], n_returned = min(top_k, n_candidates).  Timing the
 * returned candidates and picking the fastest (Eq. 3) is the caller's step. */
int ob_bmp_anchor(const double *fwd_ms, int L, int N, int *P_out);
int ob_bmp_search(const double *fwd_ms, const double *activ, int L, int N, int r, double comm_weight,
                  int top_k, int *cand_out, double *score_out, int64_t *n_candidates,
                  int *n_returned);

#ifdef __cplusplus
}
#endif
#endif /* OMNIBAL_H */
