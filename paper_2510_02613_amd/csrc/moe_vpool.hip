// A weight pool as ONE contiguous virtual tensor over separately allocated physical pages
// (the paper's Virtual Expert Management, Sec. 3.2, and its vpage-remap primitive, Sec. 4.6 /
// App. D): kernels see slots 0..n-1 back to back, while which physical page lies under a slot
// can be changed in O(1) -- map a fresh page behind the existing ones to grow, or exchange the
// pages under two slots to re-place experts without moving a byte.  Built on HIP's virtual
// memory management (hipMemAddressReserve / hipMemCreate / hipMemMap / hipMemSetAccess).
//
// Mapping calls are host operations, not stream ordered: a slot may only be unmapped when no
// kernel that can read it is in flight (the paper likewise switches at a step boundary).
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdio>
#include <vector>

#include "elasticmoe.h"

namespace emoe {
moe_status_t set_error(moe_status_t st, const char *fmt, va_list ap);   // moe_api.hip
void layer_drop_vpool(moe_layer *layer, const moe_vpool *pool);         // moe_api.hip
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

struct Page {
    hipMemGenericAllocationHandle_t handle;
    bool live = false;     // allocated and not yet freed
    int32_t vslot = -1;    // virtual slot it is mapped under, or -1
};

}  // namespace

struct moe_vpool {
    int device = 0;
    size_t slot_bytes = 0;
    int32_t n_vslots = 0;
    void *base = nullptr;
    std::vector<int32_t> page_of;   // per virtual slot: page id or -1
    std::vector<Page> pages;
    hipMemAllocationProp prop = {};
    std::vector<moe_layer *> bound;  // layers that check their placements against this pool
};

namespace emoe {
bool vpool_backed(const moe_vpool *p, int32_t slot) { return slot >= 0 && slot < p->n_vslots && p->page_of[slot] >= 0; }
void vpool_bind(moe_vpool *p, moe_layer *l)
{
    for (moe_layer *b : p->bound) if (b == l) return;
    p->bound.push_back(l);
}
void vpool_unbind(moe_vpool *p, moe_layer *l)
{
    for (size_t i = 0; i < p->bound.size(); ++i)
        if (p->bound[i] == l) { p->bound.erase(p->bound.begin() + i); return; }
}
}  // namespace emoe

extern "C" {

moe_status_t moe_vpool_create(size_t slot_bytes, int32_t n_vslots, moe_vpool_t **out)
{
    if (!out) return fail(MOE_ERR_ARG, "out is NULL");
    *out = nullptr;
    if (slot_bytes == 0 || n_vslots <= 0) return fail(MOE_ERR_ARG, "slot_bytes and n_vslots must be positive");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    int supported = 0;
    e = hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, dev);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipDeviceGetAttribute: %s", hipGetErrorString(e));
    if (!supported) return fail(MOE_ERR_UNSUPPORTED, "device %d has no virtual memory management", dev);
    moe_vpool *p = new moe_vpool;
    p->device = dev;
    p->prop.type = hipMemAllocationTypePinned;
    p->prop.location.type = hipMemLocationTypeDevice;
    p->prop.location.id = dev;
    size_t gran = 0;
    e = hipMemGetAllocationGranularity(&gran, &p->prop, hipMemAllocationGranularityMinimum);
    if (e != hipSuccess || gran == 0) { delete p; return fail(MOE_ERR_HIP, "hipMemGetAllocationGranularity: %s", hipGetErrorString(e)); }
    if (slot_bytes % gran != 0) {
        delete p;
        return fail(MOE_ERR_UNSUPPORTED, "slot_bytes %zu is not a multiple of the mapping granularity %zu: slots could not lie back to back",
                    slot_bytes, gran);
    }
    e = hipMemAddressReserve(&p->base, slot_bytes * (size_t)n_vslots, 0, nullptr, 0);
    if (e != hipSuccess) { delete p; return fail(MOE_ERR_HIP, "hipMemAddressReserve of %zu bytes: %s", slot_bytes * (size_t)n_vslots, hipGetErrorString(e)); }
    p->slot_bytes = slot_bytes;
    p->n_vslots = n_vslots;
    p->page_of.assign(n_vslots, -1);
    *out = p;
    return MOE_OK;
}

void *moe_vpool_base(const moe_vpool_t *p) { return p ? p->base : nullptr; }

int32_t moe_vpool_page_of(const moe_vpool_t *p, int32_t vslot)
{
    if (!p || vslot < 0 || vslot >= p->n_vslots) return -1;
    return p->page_of[vslot];
}

moe_status_t moe_vpool_page_alloc(moe_vpool_t *p, int32_t *page)
{
    if (!p || !page) return fail(MOE_ERR_ARG, "pool or page is NULL");
    Page pg;
    hipError_t e = hipMemCreate(&pg.handle, p->slot_bytes, &p->prop, 0);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipMemCreate of %zu bytes: %s", p->slot_bytes, hipGetErrorString(e));
    pg.live = true;
    for (size_t i = 0; i < p->pages.size(); ++i)
        if (!p->pages[i].live) { p->pages[i] = pg; *page = (int32_t)i; return MOE_OK; }
    p->pages.push_back(pg);
    *page = (int32_t)p->pages.size() - 1;
    return MOE_OK;
}

moe_status_t moe_vpool_page_free(moe_vpool_t *p, int32_t page)
{
    if (!p) return fail(MOE_ERR_ARG, "pool is NULL");
    if (page < 0 || page >= (int32_t)p->pages.size() || !p->pages[page].live) return fail(MOE_ERR_ARG, "page %d does not exist", page);
    if (p->pages[page].vslot >= 0) return fail(MOE_ERR_MAP, "page %d is still mapped under slot %d", page, p->pages[page].vslot);
    hipError_t e = hipMemRelease(p->pages[page].handle);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipMemRelease: %s", hipGetErrorString(e));
    p->pages[page].live = false;
    return MOE_OK;
}

moe_status_t moe_vpool_map(moe_vpool_t *p, int32_t vslot, int32_t page)
{
    if (!p) return fail(MOE_ERR_ARG, "pool is NULL");
    if (vslot < 0 || vslot >= p->n_vslots) return fail(MOE_ERR_ARG, "slot %d is outside [0, %d)", vslot, p->n_vslots);
    if (page < 0 || page >= (int32_t)p->pages.size() || !p->pages[page].live) return fail(MOE_ERR_ARG, "page %d does not exist", page);
    if (p->page_of[vslot] >= 0) return fail(MOE_ERR_MAP, "slot %d already has page %d under it", vslot, p->page_of[vslot]);
    if (p->pages[page].vslot >= 0) return fail(MOE_ERR_MAP, "page %d is already mapped under slot %d", page, p->pages[page].vslot);
    char *va = (char *)p->base + (size_t)vslot * p->slot_bytes;
    hipError_t e = hipMemMap(va, p->slot_bytes, 0, p->pages[page].handle, 0);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipMemMap: %s", hipGetErrorString(e));
    hipMemAccessDesc acc = {};
    acc.location = p->prop.location;
    acc.flags = hipMemAccessFlagsProtReadWrite;
    e = hipMemSetAccess(va, p->slot_bytes, &acc, 1);
    if (e != hipSuccess) {
        (void)hipMemUnmap(va, p->slot_bytes);
        return fail(MOE_ERR_HIP, "hipMemSetAccess: %s", hipGetErrorString(e));
    }
    p->page_of[vslot] = page;
    p->pages[page].vslot = vslot;
    return MOE_OK;
}

moe_status_t moe_vpool_unmap(moe_vpool_t *p, int32_t vslot)
{
    if (!p) return fail(MOE_ERR_ARG, "pool is NULL");
    if (vslot < 0 || vslot >= p->n_vslots) return fail(MOE_ERR_ARG, "slot %d is outside [0, %d)", vslot, p->n_vslots);
    const int32_t page = p->page_of[vslot];
    if (page < 0) return fail(MOE_ERR_MAP, "slot %d has no page under it", vslot);
    hipError_t e = hipMemUnmap((char *)p->base + (size_t)vslot * p->slot_bytes, p->slot_bytes);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipMemUnmap: %s", hipGetErrorString(e));
    p->page_of[vslot] = -1;
    p->pages[page].vslot = -1;
    return MOE_OK;
}

size_t moe_vpool_slot_bytes(const moe_vpool_t *p) { return p ? p->slot_bytes : 0; }
int32_t moe_vpool_slots(const moe_vpool_t *p) { return p ? p->n_vslots : 0; }

moe_status_t moe_vpool_destroy(moe_vpool_t *p)
{
    if (!p) return MOE_OK;
    for (moe_layer *l : p->bound) emoe::layer_drop_vpool(l, p);   // those layers stop checking against this pool
    hipError_t first = hipSuccess;
    for (int32_t s = 0; s < p->n_vslots; ++s)
        if (p->page_of[s] >= 0) {
            hipError_t e = hipMemUnmap((char *)p->base + (size_t)s * p->slot_bytes, p->slot_bytes);
            if (e != hipSuccess && first == hipSuccess) first = e;
        }
    for (Page &pg : p->pages)
        if (pg.live) {
            hipError_t e = hipMemRelease(pg.handle);
            if (e != hipSuccess && first == hipSuccess) first = e;
        }
    hipError_t e = hipMemAddressFree(p->base, p->slot_bytes * (size_t)p->n_vslots);
    if (e != hipSuccess && first == hipSuccess) first = e;
    delete p;
    if (first != hipSuccess) return fail(MOE_ERR_HIP, "releasing the pool: %s", hipGetErrorString(first));
    return MOE_OK;
}

}  // extern "C"
