// Stand-ins for the device half of the library, for the host-only sanitizer build: the size helpers
// return plain values, and every launcher aborts -- the driver only exercises calls that must be
// refused by validation before anything is launched.
#include <cstdio>
#include <cstdlib>

#include "../../paper_2407_20761_amd/csrc/ob_internal.h"

#define OB_STUB(name)                                                   \
    do {                                                                \
        std::fprintf(stderr, "device launcher reached: %s\n", name);    \
        std::abort();                                                   \
    } while (0)

namespace ob {

void launch_gemm_nt(int, int, int, const void *, int, const void *, int, void *, int, const void *, const void *, int,
                    hipStream_t, int, void *) { OB_STUB("launch_gemm_nt"); }
size_t gemm_workspace_bytes(int, int, int, int) { return 0; }
size_t gemm_tn_group_workspace_bytes(int, const GemmTN *, int) { return 0; }
int gemm_tn_group(int, const GemmTN *, int, void *, size_t, hipStream_t) { OB_STUB("gemm_tn_group"); }
int gemm_any(int, int, int, int, const void *, const void *, void *, const void *, const void *, void *, size_t,
             hipStream_t) { OB_STUB("gemm_any"); }
void launch_norm_fwd(int, const void *, const void *, const void *, void *, float *, int, int, float, hipStream_t) { OB_STUB("launch_norm_fwd"); }
int norm_bwd_partials(int T, int H) { return (H <= 1024 && T >= 2048) ? 256 : T < 1024 ? T : 1024; }
void launch_norm_bwd(int, const void *, const void *, const float *, const void *, const void *, void *, float *, int,
                     int, hipStream_t, float *) { OB_STUB("launch_norm_bwd"); }
void launch_reduce_partials(const float *, int, int, void *, int, int, hipStream_t) { OB_STUB("launch_reduce_partials"); }
int launch_reduce_batch(const ReduceBatch &, int, hipStream_t) { OB_STUB("launch_reduce_batch"); }
int colsum_partials(int T) { return T < 256 ? T : 256; }
void launch_colsum(const void *, int, int, int, float *, hipStream_t) { OB_STUB("launch_colsum"); }
void launch_rotary(void *, int, int, int, int, const int32_t *, int, float, float, hipStream_t) { OB_STUB("launch_rotary"); }
void launch_act_fwd(int, const void *, void *, int, int, hipStream_t) { OB_STUB("launch_act_fwd"); }
void launch_act_bwd(int, const void *, const void *, void *, int, int, hipStream_t) { OB_STUB("launch_act_bwd"); }
void launch_mask(const int32_t *, int, int, int, uint8_t *, hipStream_t) { OB_STUB("launch_mask"); }
int subsample_max_width() { return 16384; }
void launch_subsample_norm_fwd(const void *, const void *, const void *, void *, float *, int, int, int, float, hipStream_t) { OB_STUB("launch_subsample_norm_fwd"); }
void launch_subsample_norm_bwd(const void *, const void *, const float *, const void *, void *, int, int, int, int, hipStream_t) { OB_STUB("launch_subsample_norm_bwd"); }
int subsample_wgrad_partials(int n_tok) { return n_tok < 256 ? n_tok : 256; }
void launch_subsample_norm_wgrad(const void *, const void *, const float *, float *, int, int, int, hipStream_t) { OB_STUB("launch_subsample_norm_wgrad"); }
void launch_rows_scatter(const void *, void *, const int32_t *, int, int, hipStream_t) { OB_STUB("launch_rows_scatter"); }
void launch_rows_gather(void *, const void *, const int32_t *, int, int, hipStream_t) { OB_STUB("launch_rows_gather"); }
void launch_attn_fwd(const void *, const void *, const void *, void *, float *, int, int, int, const ob_segments *, int,
                     int, int, float, int, hipStream_t) { OB_STUB("launch_attn_fwd"); }
void launch_attn_bwd(const void *, const void *, const void *, const void *, const void *, const float *, float *,
                     float *, void *, void *, void *, int, int, int, const ob_segments *, int, int, int, float, int,
                     float, hipStream_t) { OB_STUB("launch_attn_bwd"); }

namespace f32 {
SavedF32 saved_layout(const ob_block_desc *d, int T) {
    SavedF32 s{};
    s.total = (size_t)T * d->hidden * 64;
    return s;
}
WorkF32 work_layout(const ob_block_desc *d, int T) {
    WorkF32 w{};
    w.total = (size_t)T * d->hidden * 64;
    return w;
}
void attn_fwd(const void *, const void *, const void *, void *, float *, int, int, int, const ob_segments *, int, int,
              int, float, int, hipStream_t) { OB_STUB("f32::attn_fwd"); }
void attn_bwd(const void *, const void *, const void *, const void *, const void *, const float *, void *, void *,
              void *, float *, int, int, int, const ob_segments *, int, int, int, float, int, hipStream_t) { OB_STUB("f32::attn_bwd"); }
void block_fwd(const ob_block_desc *, const ob_block_weights *, const void *, void *, void *, const ob_segments *,
               hipStream_t) { OB_STUB("f32::block_fwd"); }
void block_bwd(const ob_block_desc *, const ob_block_weights *, const ob_block_grads *, int, const void *,
               const void *, void *, const void *, const ob_segments *, void *, hipStream_t) { OB_STUB("f32::block_bwd"); }
size_t connector_saved_bytes(long n_tok, int Hv, int Ht) { return (size_t)n_tok * (4 * Hv + 2 * Ht + 2) * 4; }
size_t connector_work_bytes(long n_tok, int Hv, int Ht) { return (size_t)n_tok * (4 * Hv + 3 * Ht) * 4; }
void connector_fwd(const ob_connector_weights *, const void *, int, int, int, int, float, const int32_t *, void *,
                   void *, void *, hipStream_t) { OB_STUB("f32::connector_fwd"); }
void connector_bwd(const ob_connector_weights *, const ob_connector_grads *, int, const void *, void *, int, int, int,
                   int, int, const int32_t *, const void *, void *, hipStream_t) { OB_STUB("f32::connector_bwd"); }
}  // namespace f32
}  // namespace ob
