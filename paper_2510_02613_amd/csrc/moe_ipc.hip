// Zero-copy attach of a weight pool from a second process (the paper's zero-copy primitive,
// Sec. 4.6, and its export_handle / open_tensor pair, App. D): the process that owns the experts
// exports a handle of the device allocation that holds a pool, a serving process opens it and hands
// the resulting address to moe_layer_create as w13 / w2 -- the weights are never copied, and a
// serving process can be replaced (a scale-up starts a new one) while the owner keeps the tensors.
// Built on hipIpcGetMemHandle / hipIpcOpenMemHandle.
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstring>

#include "elasticmoe.h"

namespace emoe {
moe_status_t set_error(moe_status_t st, const char *fmt, va_list ap);   // moe_api.hip
}

namespace {

moe_status_t fail(moe_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    emoe::set_error(st, fmt, ap);
    va_end(ap);
    return st;
}

static_assert(sizeof(hipIpcMemHandle_t) == MOE_IPC_HANDLE_BYTES, "the handle travels as MOE_IPC_HANDLE_BYTES opaque bytes");
constexpr size_t kMaxShared = (size_t)2 << 30;   // allocations of 2 GiB and more are not opened across processes

}  // namespace

extern "C" {

moe_status_t moe_pool_export(const void *dev_ptr, void *handle, size_t *offset)
{
    if (!dev_ptr || !handle || !offset) return fail(MOE_ERR_ARG, "dev_ptr, handle and offset must be non-NULL");
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    hipError_t e = hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)const_cast<void *>(dev_ptr));
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipMemGetAddressRange: %s (is dev_ptr device memory of this process?)", hipGetErrorString(e));
    if (size >= kMaxShared)
        return fail(MOE_ERR_UNSUPPORTED, "the allocation that holds dev_ptr has %zu bytes; pools are shared in allocations under 2 GiB", size);
    hipIpcMemHandle_t h;
    e = hipIpcGetMemHandle(&h, base);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipIpcGetMemHandle: %s", hipGetErrorString(e));
    memcpy(handle, &h, sizeof h);
    *offset = (size_t)((const char *)dev_ptr - (const char *)base);
    return MOE_OK;
}

moe_status_t moe_pool_open(const void *handle, size_t offset, void **dev_ptr)
{
    if (!handle || !dev_ptr) return fail(MOE_ERR_ARG, "handle and dev_ptr must be non-NULL");
    *dev_ptr = nullptr;
    hipIpcMemHandle_t h;
    memcpy(&h, handle, sizeof h);
    void *base = nullptr;
    const hipError_t e = hipIpcOpenMemHandle(&base, h, hipIpcMemLazyEnablePeerAccess);
    if (e != hipSuccess || !base) return fail(MOE_ERR_HIP, "hipIpcOpenMemHandle: %s", hipGetErrorString(e));
    *dev_ptr = (char *)base + offset;
    return MOE_OK;
}

moe_status_t moe_pool_close(void *dev_ptr, size_t offset)
{
    if (!dev_ptr) return fail(MOE_ERR_ARG, "dev_ptr is NULL");
    const hipError_t e = hipIpcCloseMemHandle((char *)dev_ptr - offset);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipIpcCloseMemHandle: %s", hipGetErrorString(e));
    return MOE_OK;
}

}  // extern "C"
