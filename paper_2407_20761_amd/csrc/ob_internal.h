// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/omnibal.h"

namespace ob {

// thread-local error text behind ob_last_error()
int fail(int status, const char *fmt, ...);
int check_launch(const char *what);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// host-side checks shared by the attention entry points (api.cpp); OB_OK or a status with the text set
int validate_attn(const ob_segments *seg, int nq, int nkv, int d, int ldq, int ldkv, int ldo,
                  int mask, int dtype, const char *who);

// ---- opt-in per-kernel-class timing (ob_prof_begin / ob_prof_end) --------------------------
enum KClass {
    K_GEMM = 0, K_ATTN_FWD, K_ATTN_BWD_DQ, K_ATTN_BWD_DKV, K_NORM_FWD,
    K_NORM_BWD, K_ROTARY, K_ACT_FWD, K_ACT_BWD, K_COLSUM, K_REDUCE, K_CONN_FWD, K_CONN_BWD, K_ROWS, K_COUNT
};
// Brackets one kernel launch with a pair of events on its stream while profiling is on;
// `work` is the launch's algorithmic FLOPs (MFMA kernels) or bytes (HBM-bound kernels).
struct ProfScope {
    ProfScope(int cls, hipStream_t s, double work);
    ~ProfScope();
    int slot;
    hipStream_t stream;
};

// ---- GEMM (gemm.hip) ---------------------------------------------------------------------
// C[M,N] = A[M,K] B[N,K]^T (+bias[N]) (+R[M,N]); K % 64 == 0, N % 8 == 0, any M.
// k_algo (<= K, 0 = K): the contraction length that counts as algorithmic work when K is padded.
// ws (may be null): gemm_workspace_bytes(0, M, N, K) bytes of scratch for a split contraction.
void launch_gemm_nt(int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C,
                    int ldc, const void *bias, const void *R, int ldr, hipStream_t s,
                    int k_algo = 0, void *ws = nullptr);
size_t gemm_workspace_bytes(int layout, int M, int N, int K);
int gemm_any(int layout, int M, int N, int K, const void *A, const void *B, void *C,
             const void *bias, const void *R, void *ws, size_t ws_bytes, hipStream_t s);

// C[M, N] = A[K, M]^T B[K, N] (+ R): one weight gradient; up to 4 of them over the same K go out as one
// launch (gemm_tn_group), with ws of gemm_tn_group_workspace_bytes() bytes
struct GemmTN { int M, N; const void *A, *B; void *C; const void *R; };
size_t gemm_tn_group_workspace_bytes(int count, const GemmTN *g, int K);
int gemm_tn_group(int count, const GemmTN *g, int K, void *ws, size_t ws_bytes, hipStream_t s);

// ---- elementwise (elementwise.hip) -----------------------------------------------------------
// stats: LayerNorm [T,2] = (mean, rstd); RMSNorm [T,2] = (unused, rstd)
void launch_norm_fwd(int norm, const void *x, const void *gamma, const void *beta, void *h,
                     float *stats, int T, int H, float eps, hipStream_t s);
// dx = dres + norm_bwd(dh); partial [n_part, 2, H] fp32 sums of dgamma / dbeta
int norm_bwd_partials(int T, int H);
// csum (may be null): [norm_bwd_partials(T, H)][2][H] fp32 column sums of dres and of dx (the bias gradients
// of the linears on either side of the norm), formed in the same pass
void launch_norm_bwd(int norm, const void *dh, const void *x, const float *stats, const void *gamma,
                     const void *dres, void *dx, float *partial, int T, int H, hipStream_t s,
                     float *csum = nullptr);
// out[c] (bf16) = (accumulate ? out[c] : 0) + sum_p partial[p * stride + c]
void launch_reduce_partials(const float *partial, int n_part, int stride, void *out, int C,
                            int accumulate, hipStream_t s);
// several such reductions in one launch (they are latency-bound: few columns, a few hundred partials)
struct ReduceJob { const float *partial; int n_part, stride; void *out; int C; };
struct ReduceBatch {
    static constexpr int MAX = 8;
    ReduceJob job[MAX];
    int n = 0;
    bool overflow = false;   // a job did not fit: launch_reduce_batch refuses the whole batch
    void add(const float *partial, int n_part, int stride, void *out, int C) {
        if (n >= MAX) { overflow = true; return; }
        job[n++] = ReduceJob{partial, n_part, stride, out, C};
    }
};
// OB_EINVAL (nothing launched) when a job was dropped by add()
int launch_reduce_batch(const ReduceBatch &b, int accumulate, hipStream_t s);
int colsum_partials(int T);
void launch_colsum(const void *in, int T, int C, int ld, float *partial, hipStream_t s);
void launch_rotary(void *qkv, int ld, int T, int n_heads_rot, int d, const int32_t *cu_dev,
                   int n_seg, float base, float sign, hipStream_t s);
void launch_act_fwd(int mlp, const void *up, void *act, int T, int F, hipStream_t s);
void launch_act_bwd(int mlp, const void *dact, const void *up, void *dup, int T, int F,
                    hipStream_t s);
void launch_mask(const int32_t *cu_dev, int n_seg, int T, int mask, uint8_t *out, hipStream_t s);

// ---- ViT -> LLM hand-over (connector.hip) ------------------------------------------------------
// n_tok = n_tiles * (g/2)^2 sub-sampled tokens of 4 Hv channels; stats [n_tok, 2] = (mean, rstd)
int subsample_max_width();
void launch_subsample_norm_fwd(const void *v, const void *gamma, const void *beta, void *un, float *stats,
                               int n_tok, int g, int Hv, float eps, hipStream_t s);
// writes every row of dv [n_tiles (g^2 + 1), Hv] (class rows: zeros)
void launch_subsample_norm_bwd(const void *dun, const void *v, const float *stats, const void *gamma, void *dv,
                               int n_tok, int n_tiles, int g, int Hv, hipStream_t s);
// partial [subsample_wgrad_partials(n_tok)][2][4 Hv] fp32: gain sums, then beta sums
int subsample_wgrad_partials(int n_tok);
void launch_subsample_norm_wgrad(const void *dun, const void *v, const float *stats, float *partial, int n_tok,
                                 int g, int Hv, hipStream_t s);
// big[rows[i]] = small[i]  /  small[i] = big[rows[i]];  rows of H bf16 elements, H % 8 == 0
void launch_rows_scatter(const void *small, void *big, const int32_t *rows_dev, int n_rows, int H, hipStream_t s);
void launch_rows_gather(void *small, const void *big, const int32_t *rows_dev, int n_rows, int H, hipStream_t s);

// ---- attention (attention.hip) ---------------------------------------------------------------
void launch_attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int ldq,
                     int ldkv, int ldo, const ob_segments *seg, int nq, int nkv, int d, float scale,
                     int mask, hipStream_t s);
// o, lse (natural log): the forward's results; lse2, delta: [nq][T] floats of scratch each, written by the
// dQ kernel (base-2 log-sum-exp, Delta = sum_d dO O) and read by the dK / dV kernel behind it.
// rotary_base > 1: dq and dk leave the kernels already rotated back by the tokens' rotary angles.
void launch_attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const void *o, const float *lse,
                     float *lse2, float *delta, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                     const ob_segments *seg, int nq, int nkv, int d, float scale, int mask, float rotary_base,
                     hipStream_t s);

// ---- fp32 debug path (debug_fp32.hip): every tensor fp32, plain FMA kernels --------------------
namespace f32 {
struct SavedF32 { size_t h1, qkv, o, lse, x1, h2, up, act, stat1, stat2, total; };
struct WorkF32 { size_t dact, dup, dh, dx1, d_o, dqkv, delta, total; };
SavedF32 saved_layout(const ob_block_desc *dsc, int T);
WorkF32 work_layout(const ob_block_desc *dsc, int T);
void attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int ldq, int ldkv, int ldo,
              const ob_segments *seg, int nq, int nkv, int d, float scale, int mask, hipStream_t s);
// delta: nq * T floats of scratch
void attn_bwd(const void *d_o, const void *q, const void *k, const void *v, const void *o, const float *lse,
              void *dq, void *dk, void *dv, float *delta, int ldq, int ldkv, int ldo, const ob_segments *seg, int nq,
              int nkv, int d, float scale, int mask, hipStream_t s);
void block_fwd(const ob_block_desc *dsc, const ob_block_weights *w, const void *x, void *y, void *saved,
               const ob_segments *seg, hipStream_t s);
void block_bwd(const ob_block_desc *dsc, const ob_block_weights *w, const ob_block_grads *g, int accumulate,
               const void *x, const void *dy, void *dx, const void *saved, const ob_segments *seg, void *ws,
               hipStream_t s);
// the ViT -> LLM hand-over with every tensor in fp32 (n_tok = n_tiles (g/2)^2 sub-sampled tokens)
size_t connector_saved_bytes(long n_tok, int Hv, int Ht);
size_t connector_work_bytes(long n_tok, int Hv, int Ht);
void connector_fwd(const ob_connector_weights *w, const void *v, int n_tok, int g, int Hv, int Ht, float eps,
                   const int32_t *rows_dev, void *x_llm, void *saved, void *ws, hipStream_t s);
void connector_bwd(const ob_connector_weights *w, const ob_connector_grads *gr, int accumulate, const void *dx_llm,
                   void *dv, int n_tok, int n_tiles, int g, int Hv, int Ht, const int32_t *rows_dev, const void *saved,
                   void *ws, hipStream_t s);
}  // namespace f32

}  // namespace ob
