// Host-side buffers with lazy host<->device synchronisation, after the DualView of Section 4.3
// of the paper: a host buffer and a device buffer of the same size, one "modified" flag per
// side, `sync` copies only if the other side was modified since the last sync, `modify` only
// sets a flag; sub-views alias their parent's memory, share its flags and keep it alive.
// Contracts of the entry points are in include/lapis.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>
#include <string>

#include "../../include/lapis.h"
#include "internal.hpp"

namespace {

using lapis::fail;

// The allocation and the state shared by a view and all its sub-views.
struct DualRoot {
    void *h = nullptr;            // pinned host memory
    void *d = nullptr;            // device memory
    int64_t bytes = 0;
    bool host_modified = false, device_modified = false;
    int64_t h2d_copies = 0, d2h_copies = 0;
    int refs = 1;
};

void release(DualRoot *r)
{
    if (--r->refs > 0) return;
    (void)hipHostFree(r->h);
    (void)hipFree(r->d);
    delete r;
}

}  // namespace

struct lapis_dualview {
    DualRoot *root;
    int64_t offset, bytes;
};

extern "C" {

int lapis_dualview_create(lapis_dualview_t **out, int64_t bytes)
{
    if (!out) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_create: out is NULL");
    *out = nullptr;
    if (bytes < 0) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_create: negative size");
    DualRoot *r = new (std::nothrow) DualRoot();
    lapis_dualview *v = new (std::nothrow) lapis_dualview();
    if (!r || !v) { delete r; delete v; return fail(LAPIS_ERR_ALLOC, "lapis_dualview_create: out of host memory"); }
    r->bytes = bytes;
    const size_t n = bytes ? (size_t)bytes : 1;
    if (hipHostMalloc(&r->h, n, hipHostMallocDefault) != hipSuccess || hipMalloc(&r->d, n) != hipSuccess) {
        (void)hipGetLastError();
        release(r);
        delete v;
        return fail(LAPIS_ERR_ALLOC, "lapis_dualview_create: cannot allocate " + std::to_string(bytes) + " bytes on both sides");
    }
    v->root = r; v->offset = 0; v->bytes = bytes;
    *out = v;
    return LAPIS_OK;
}

int lapis_dualview_subview(lapis_dualview_t **out, lapis_dualview_t *parent, int64_t offset_bytes, int64_t bytes)
{
    if (!out) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_subview: out is NULL");
    *out = nullptr;
    if (!parent || offset_bytes < 0 || bytes < 0 || offset_bytes > parent->bytes || bytes > parent->bytes - offset_bytes)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_subview: range is not inside the parent");
    lapis_dualview *v = new (std::nothrow) lapis_dualview();
    if (!v) return fail(LAPIS_ERR_ALLOC, "lapis_dualview_subview: out of host memory");
    v->root = parent->root;
    v->offset = parent->offset + offset_bytes;
    v->bytes = bytes;
    ++v->root->refs;
    *out = v;
    return LAPIS_OK;
}

void *lapis_dualview_host(lapis_dualview_t *v) { return v ? static_cast<char *>(v->root->h) + v->offset : nullptr; }
void *lapis_dualview_device(lapis_dualview_t *v) { return v ? static_cast<char *>(v->root->d) + v->offset : nullptr; }

int lapis_dualview_modify_host(lapis_dualview_t *v)
{
    if (!v) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_modify_host: view is NULL");
    v->root->host_modified = true;
    return LAPIS_OK;
}

int lapis_dualview_modify_device(lapis_dualview_t *v)
{
    if (!v) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_modify_device: view is NULL");
    v->root->device_modified = true;
    return LAPIS_OK;
}

// A sync of a sub-view is a sync of the whole parent allocation (they share the flags).
int lapis_dualview_sync_device(lapis_dualview_t *v, void *hip_stream)
{
    if (!v) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_sync_device: view is NULL");
    DualRoot *r = v->root;
    if (!r->host_modified) return LAPIS_OK;                 // the cost of a sync with nothing to do: one flag
    if (r->device_modified)                                 // both sides changed: no copy can be right
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_sync_device: host and device copies are both modified");
    if (r->bytes > 0 &&
        hipMemcpyAsync(r->d, r->h, (size_t)r->bytes, hipMemcpyHostToDevice, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return fail(LAPIS_ERR_DEVICE, "lapis_dualview_sync_device: host-to-device copy failed");
    r->host_modified = false;
    ++r->h2d_copies;
    return LAPIS_OK;
}

int lapis_dualview_sync_host(lapis_dualview_t *v, void *hip_stream)
{
    if (!v) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_sync_host: view is NULL");
    DualRoot *r = v->root;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (!r->device_modified) return LAPIS_OK;
    if (r->host_modified)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_sync_host: host and device copies are both modified");
    if (r->bytes > 0 && hipMemcpyAsync(r->h, r->d, (size_t)r->bytes, hipMemcpyDeviceToHost, s) != hipSuccess)
        return fail(LAPIS_ERR_DEVICE, "lapis_dualview_sync_host: device-to-host copy failed");
    if (hipStreamSynchronize(s) != hipSuccess)              // the host may read right away
        return fail(LAPIS_ERR_DEVICE, "lapis_dualview_sync_host: stream synchronisation failed");
    r->device_modified = false;
    ++r->d2h_copies;
    return LAPIS_OK;
}

int lapis_dualview_copy_counts(const lapis_dualview_t *v, int64_t *h2d, int64_t *d2h)
{
    if (!v) return fail(LAPIS_ERR_INVALID_ARG, "lapis_dualview_copy_counts: view is NULL");
    if (h2d) *h2d = v->root->h2d_copies;
    if (d2h) *d2h = v->root->d2h_copies;
    return LAPIS_OK;
}

int lapis_dualview_destroy(lapis_dualview_t *v)
{
    if (!v) return LAPIS_OK;
    release(v->root);
    delete v;
    return LAPIS_OK;
}

int lapis_spmv_dualview(const lapis_csr_t *A, double alpha, lapis_dualview_t *x, double beta,
                        lapis_dualview_t *y, void *hip_stream)
{
    if (!A || !x || !y) return fail(LAPIS_ERR_INVALID_ARG, "lapis_spmv_dualview: NULL argument");
    if (x->root == y->root && x->offset < y->offset + y->bytes && y->offset < x->offset + x->bytes)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_spmv_dualview: x and y overlap");
    int64_t x_bytes, y_bytes;
    lapis::vector_bytes(A, &x_bytes, &y_bytes);
    if (x->bytes < x_bytes || y->bytes < y_bytes)
        return fail(LAPIS_ERR_INVALID_ARG, "lapis_spmv_dualview: a view is smaller than its operand (x needs " +
                                               std::to_string(x_bytes) + " bytes, y " + std::to_string(y_bytes) + ")");
    int rc = lapis_dualview_sync_device(x, hip_stream);
    // y is overwritten when beta == 0: its host copy need not travel if the product rewrites the
    // whole allocation (an allocation longer than the operand keeps host-side bytes past the
    // operand that only a copy can bring to the device)
    const bool y_discarded = beta == 0.0 && y->offset == 0 && y_bytes == y->root->bytes && y->root != x->root;
    if (rc == LAPIS_OK && !y_discarded) rc = lapis_dualview_sync_device(y, hip_stream);
    if (rc != LAPIS_OK) return rc;
    if (y_discarded) y->root->host_modified = false;
    rc = lapis_spmv(A, alpha, lapis_dualview_device(x), beta, lapis_dualview_device(y), hip_stream);
    if (rc != LAPIS_OK) return rc;
    return lapis_dualview_modify_device(y);
}

}  // extern "C"
