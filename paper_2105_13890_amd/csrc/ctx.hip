// Context, status word, error strings, zero-fill.
#include "common.h"

#include <new>

__global__ void fill_zero_kernel(uint32_t *p, size_t n_words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_words; i += stride) p[i] = 0u;
}

extern "C" int eoq_create(eoq_ctx **out, void *hip_stream)
{
    if (!out) return EOQ_ERR_ARG;
    eoq_ctx *c = new (std::nothrow) eoq_ctx();
    if (!c) return EOQ_ERR_ARG;
    c->stream = (hipStream_t)hip_stream;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return EOQ_ERR_HIP; }
    if (wgrad_static_scratch_init(c->device, &c->static_scratch) != EOQ_OK) { delete c; return EOQ_ERR_HIP; }
    if (hipMalloc((void **)&c->d_status, 256) != hipSuccess) { delete c; return EOQ_ERR_HIP; }
    if (hipMalloc((void **)&c->d_scratch, sizeof(int32_t) * EOQ_SCRATCH_SLOTS) != hipSuccess) {
        (void)hipFree(c->d_status);
        delete c;
        return EOQ_ERR_HIP;
    }
    if (hipMalloc((void **)&c->d_partials, sizeof(int64_t) * EOQ_PARTIAL_SLOTS) != hipSuccess) {
        (void)hipFree(c->d_status);
        (void)hipFree(c->d_scratch);
        delete c;
        return EOQ_ERR_HIP;
    }
    if (hipMemset(c->d_status, 0, 256) != hipSuccess ||
        hipMemset(c->d_scratch, 0, sizeof(int32_t) * EOQ_SCRATCH_SLOTS) != hipSuccess) {
        (void)hipFree(c->d_status);
        (void)hipFree(c->d_scratch);
        (void)hipFree(c->d_partials);
        delete c;
        return EOQ_ERR_HIP;
    }
    *out = c;
    return EOQ_OK;
}

extern "C" int eoq_destroy(eoq_ctx *c)
{
    if (!c) return EOQ_ERR_ARG;
    (void)hipFree(c->d_status);
    (void)hipFree(c->d_scratch);
    (void)hipFree(c->d_partials);
    delete c;
    return EOQ_OK;
}

extern "C" const char *eoq_strerror(int code)
{
    switch (code) {
    case EOQ_OK: return "ok";
    case EOQ_ERR_ARG: return "invalid argument";
    case EOQ_ERR_SHAPE: return "shape not supported";
    case EOQ_ERR_WORKSPACE: return "workspace missing or too small";
    case EOQ_ERR_RANGE: return "range violation reported by the device";
    case EOQ_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

extern "C" int eoq_status(eoq_ctx *c, uint32_t *flags)
{
    if (!c) return EOQ_ERR_ARG;
    uint32_t h = 0;
    EOQ_HIP(hipStreamSynchronize(c->stream));
    EOQ_HIP(hipMemcpy(&h, c->d_status, sizeof(h), hipMemcpyDeviceToHost));
    if (h) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(64), 0, c->stream, c->d_status, (size_t)1);
        EOQ_LAUNCH_CHECK();
        EOQ_HIP(hipStreamSynchronize(c->stream));
    }
    if (flags) *flags = h;
    return h ? EOQ_ERR_RANGE : EOQ_OK;
}

extern "C" int eoq_spec_counters(eoq_ctx *c, int64_t *hits, int64_t *misses)
{
    if (!c) return EOQ_ERR_ARG;
    int32_t h[2] = {0, 0};
    EOQ_HIP(hipStreamSynchronize(c->stream));
    EOQ_HIP(hipMemcpy(h, c->d_scratch + EOQ_SLOT_SPEC_HITS, sizeof(h), hipMemcpyDeviceToHost));
    if (hits) *hits = h[0];
    if (misses) *misses = h[1];
    return EOQ_OK;
}

extern "C" int eoq_fill_zero(eoq_ctx *c, void *ptr, size_t bytes)
{
    if (!c || (!ptr && bytes) || (bytes & 3) || ((uintptr_t)ptr & 3)) return EOQ_ERR_ARG;
    if (!bytes) return EOQ_OK;
    size_t words = bytes / 4;
    size_t blocks = (words + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, c->stream, (uint32_t *)ptr, words);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
