// C ABI of the CCE- library: argument checks, workspace layout, dispatch.  See include/cce_neg.h for the contract.
#include <hip/hip_runtime.h>

#include "cce_device.hpp"
#include "cce_kernels.hpp"

namespace cce {
namespace {

constexpr size_t kHeaderBytes = 256;  // status word + padding; keeps what follows 256-byte aligned

__global__ void fill_zero_kernel(int32_t *dst, size_t words)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) dst[i] = 0;
}

cce_status check_desc(const cce_desc *d)
{
    if (!d) return CCE_ERR_NULL;
    if (d->N < 0 || d->V <= 0 || d->V > 0x7fffffffLL || d->N > 0x7fffffffLL) return CCE_ERR_SHAPE;
    if (d->d < 8 || d->d > 512 || (d->d % 8) != 0) return CCE_ERR_SHAPE;
    if (d->neg_mode != CCE_NEG_SHARED && d->neg_mode != CCE_NEG_PER_POSITION && d->neg_mode != CCE_NEG_FULL)
        return CCE_ERR_SHAPE;
    if (d->neg_mode != CCE_NEG_FULL && d->K < 0) return CCE_ERR_SHAPE;
    if (d->in_dtype != CCE_F32 && d->in_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->dH_dtype != CCE_F32 && d->dH_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->dH_dtype == CCE_BF16 && d->in_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->algo != CCE_ALGO_AUTO && d->algo != CCE_ALGO_GATHER && d->algo != CCE_ALGO_TILE) return CCE_ERR_UNSUPPORTED;
    if (d->algo == CCE_ALGO_TILE) return CCE_ERR_UNSUPPORTED;  // matrix-core path not built yet
    return CCE_OK;
}

cce_status check_common(const cce_desc *d, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                        void *workspace, size_t workspace_bytes)
{
    const cce_status st = check_desc(d);
    if (st != CCE_OK) return st;
    if (!H || !E || !tgt) return CCE_ERR_NULL;
    if (d->neg_mode != CCE_NEG_FULL && d->K > 0 && !neg) return CCE_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < cce_neg_workspace_bytes(d))
        return CCE_ERR_WORKSPACE;
    return CCE_OK;
}

Params make_params(const cce_desc *d, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                   const uint8_t *mask, void *workspace)
{
    Params p{};
    p.H = H;
    p.E = E;
    p.tgt = tgt;
    p.neg = neg;
    p.mask = mask;
    p.status = static_cast<int32_t *>(workspace);
    p.N = d->N;
    p.V = d->V;
    p.d = d->d;
    p.K = (d->neg_mode == CCE_NEG_FULL) ? 0 : d->K;
    p.neg_mode = d->neg_mode;
    p.collide = d->mask_target_collisions ? 1 : 0;
    p.validate = d->validate_indices ? 1 : 0;
    p.dH_bf16 = (d->dH_dtype == CCE_BF16) ? 1 : 0;
    return p;
}

}  // namespace

hipError_t launch_fill_zero(int32_t *dst, size_t words, hipStream_t stream)
{
    if (words == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, dst, words);
    return hipGetLastError();
}

}  // namespace cce

extern "C" {

size_t cce_neg_workspace_bytes(const cce_desc *desc)
{
    if (cce::check_desc(desc) != CCE_OK) return 0;
    return cce::kHeaderBytes;
}

cce_status cce_neg_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace) return CCE_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < cce::kHeaderBytes) return CCE_ERR_WORKSPACE;
    const hipError_t e = cce::launch_fill_zero(static_cast<int32_t *>(workspace), cce::kHeaderBytes / 4,
                                               static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

cce_status cce_neg_forward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                           const uint8_t *mask, float *loss, float *lse, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    const cce_status st = cce::check_common(desc, H, E, tgt, neg, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!loss || !lse) return CCE_ERR_NULL;
    cce::Params p = cce::make_params(desc, H, E, tgt, neg, mask, workspace);
    p.loss = loss;
    p.lse = lse;
    const hipError_t e = cce::launch_gather(false, desc->in_dtype == CCE_BF16, p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

cce_status cce_neg_backward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                            const uint8_t *mask, const float *lse, const float *grad_loss, void *dH, float *dE,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const cce_status st = cce::check_common(desc, H, E, tgt, neg, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!lse || !dH || !dE) return CCE_ERR_NULL;
    cce::Params p = cce::make_params(desc, H, E, tgt, neg, mask, workspace);
    p.lse_in = lse;
    p.g = grad_loss;
    p.dH = dH;
    p.dE = dE;
    const hipError_t e = cce::launch_gather(true, desc->in_dtype == CCE_BF16, p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

cce_status cce_neg_index_status(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace) return CCE_ERR_NULL;
    if (workspace_bytes < cce::kHeaderBytes) return CCE_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t word = 0;
    if (hipMemcpyAsync(&word, workspace, sizeof word, hipMemcpyDeviceToHost, s) != hipSuccess) return CCE_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CCE_ERR_HIP;
    if (word != 0) {
        if (cce::launch_fill_zero(static_cast<int32_t *>(workspace), 1, s) != hipSuccess) return CCE_ERR_HIP;
        if (hipStreamSynchronize(s) != hipSuccess) return CCE_ERR_HIP;
        return CCE_ERR_INDEX;
    }
    return CCE_OK;
}

const char *cce_status_string(cce_status status)
{
    switch (status) {
    case CCE_OK: return "ok";
    case CCE_ERR_NULL: return "a required pointer is NULL";
    case CCE_ERR_SHAPE: return "invalid shape (N, V, K, d or neg_mode)";
    case CCE_ERR_DTYPE: return "invalid dtype combination";
    case CCE_ERR_INDEX: return "an id of a valid position is outside [0, V)";
    case CCE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CCE_ERR_UNSUPPORTED: return "requested algorithm cannot run this descriptor";
    case CCE_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
