// ob_varlen_attn_bwd_static: the attention backward for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels
// as ob_varlen_attn_bwd; the scratch they need (Delta and the base-2 log-sum-exp, [nq, T] fp32 each)
// lives in a file-scope device array instead of a caller-provided workspace.
//
// Every GPU the library is loaded on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle: the device address is asked for once
// per device with hipGetSymbolAddress and only that pointer is handed to kernels.
#include <mutex>

#include "ob_internal.h"

namespace {

constexpr size_t SCRATCH_BYTES = OB_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *g_scratch[MAX_DEVICES];   // per device: address of that device's copy of `scratch`
std::mutex g_mu;

// address of the current device's scratch array (asked for on the first call on that device)
int scratch_of_current_device(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return ob::fail(OB_EHIP, "ob_varlen_attn_bwd_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return ob::fail(OB_EUNSUPPORTED, "ob_varlen_attn_bwd_static: device %d not in [0, %d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return ob::fail(OB_EHIP, "ob_varlen_attn_bwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch[dev] = p;
    }
    *out = g_scratch[dev];
    return OB_OK;
}

}  // namespace

extern "C" int ob_varlen_attn_bwd_static(const void *d_o, const void *q, const void *k, const void *v, const void *o,
                                         const float *lse, void *dq, void *dk, void *dv, int ldq, int ldkv, int ldo,
                                         const ob_segments *seg, int nq, int nkv, int d, float scale, int mask,
                                         int dtype, void *hip_stream) {
    using namespace ob;
    if (!d_o || !q || !k || !v || !o || !lse || !dq || !dk || !dv)
        return fail(OB_EINVAL, "ob_varlen_attn_bwd_static: null tensor pointer");
    if (int rc = validate_attn(seg, nq, nkv, d, ldq, ldkv, ldo, mask, dtype, "ob_varlen_attn_bwd_static")) return rc;
    const size_t rows = align_up((size_t)seg->total_tokens * nq * 4, 256);
    if (2 * rows > SCRATCH_BYTES)
        return fail(OB_EWORKSPACE, "ob_varlen_attn_bwd_static: total_tokens * n_q_heads = %zu needs %zu bytes of scratch, "
                    "the static array holds %zu (use ob_varlen_attn_bwd with a workspace)",
                    (size_t)seg->total_tokens * nq, 2 * rows, SCRATCH_BYTES);
    void *base = nullptr;
    if (int rc = scratch_of_current_device(&base)) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == OB_FP32) {
        f32::attn_bwd(d_o, q, k, v, o, lse, dq, dk, dv, (float *)base, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, s);
        return check_launch("ob_varlen_attn_bwd_static");
    }
    // both halves are written (by the dQ kernel, for every row of every head) before the dK / dV kernel
    // reads them: nothing of an earlier call's contents is ever read
    float *delta = (float *)base, *lse2 = (float *)((unsigned char *)base + rows);
    launch_attn_bwd(d_o, q, k, v, o, lse, lse2, delta, dq, dk, dv, ldq, ldkv, ldo, seg, nq, nkv, d, scale, mask, 0.f, s);
    return check_launch("ob_varlen_attn_bwd_static");
}
