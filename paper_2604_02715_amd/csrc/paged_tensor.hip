// PagedTensor on HIP virtual memory management (paper Sec. 4.1): every rank-local expert tensor
// of every layer gets a stable virtual address; pageable layers alias two reusable physical
// blocks per tensor type, uncompressed-resident layers own a dedicated block.  Only residency
// changes touch mappings; materialization only writes block contents.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "fluxmoe_internal.h"

using fluxmoe::set_error;

#define PT_HIP(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return set_error(FLUXMOE_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

struct fluxmoe_paged_tensor {
    fluxmoe_desc d{};
    int device = 0;
    uint64_t g = 0, A[2] = {0, 0}, S[2] = {0, 0}, sigma[2] = {0, 0};
    uint8_t* v0[2] = {nullptr, nullptr};       // N layer ranges of S bytes each
    uint8_t* window[2] = {nullptr, nullptr};   // a second view of the two reusable blocks, back to back
    hipMemGenericAllocationHandle_t reusable[2][2] = {};
    bool reusable_made[2][2] = {};
    std::vector<hipMemGenericAllocationHandle_t> dedicated[2];   // per layer, valid if uncompressed
    std::vector<uint8_t> uncompressed;         // [N]
    std::vector<uint8_t> mapped[2];            // [N] the layer range currently has a mapping
    bool window_mapped[2][2] = {};
    hipMemAllocationProp prop{};
    hipMemAccessDesc access{};
};

namespace {

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

int layout(const fluxmoe_desc* d, uint64_t g, uint32_t n_unc, fluxmoe_paged_tensor_info* out) {
    if (!d || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (g == 0) return set_error(FLUXMOE_EINVAL, "granularity must be positive");
    if (d->n_layers == 0 || d->n_experts == 0 || d->hidden == 0 || d->ffn == 0)
        return set_error(FLUXMOE_EINVAL, "n_layers, n_experts, hidden, ffn must be positive");
    if (n_unc > d->n_layers) return set_error(FLUXMOE_ERANGE, "more uncompressed layers than layers");
    *out = fluxmoe_paged_tensor_info{};
    out->granularity = g;
    const uint64_t sigma2 = uint64_t(d->hidden) * d->ffn * 2, sigma1 = 2 * sigma2;
    const uint64_t sig[2] = {sigma1, sigma2};
    for (int t = 0; t < 2; ++t) {
        out->A[t] = uint64_t(d->n_experts) * sig[t];
        out->S[t] = align_up(out->A[t], g);
        out->virtual_bytes += uint64_t(d->n_layers) * out->S[t];
        out->physical_bytes += (uint64_t(n_unc) + 2) * out->S[t];
        out->pad_bytes += (uint64_t(n_unc) + 2) * (out->S[t] - out->A[t]);
    }
    out->n_uncompressed = n_unc;
    out->n_pageable = d->n_layers - n_unc;
    return FLUXMOE_OK;
}

int map_range(fluxmoe_paged_tensor* p, uint8_t* va, uint64_t bytes, hipMemGenericAllocationHandle_t h) {
    PT_HIP(hipMemMap(va, bytes, 0, h, 0));
    PT_HIP(hipMemSetAccess(va, bytes, &p->access, 1));
    return FLUXMOE_OK;
}

int map_layer(fluxmoe_paged_tensor* p, uint32_t layer) {
    for (int t = 0; t < 2; ++t) {
        if (p->mapped[t][layer]) continue;
        hipMemGenericAllocationHandle_t h;
        if (p->uncompressed[layer]) {
            PT_HIP(hipMemCreate(&p->dedicated[t][layer], p->S[t], &p->prop, 0));
            h = p->dedicated[t][layer];
        } else {
            h = p->reusable[t][layer & 1];
        }
        if (int rc = map_range(p, p->v0[t] + uint64_t(layer) * p->S[t], p->S[t], h)) return rc;
        p->mapped[t][layer] = 1;
    }
    return FLUXMOE_OK;
}

int unmap_layer(fluxmoe_paged_tensor* p, uint32_t layer) {
    for (int t = 0; t < 2; ++t) {
        if (!p->mapped[t][layer]) continue;
        PT_HIP(hipMemUnmap(p->v0[t] + uint64_t(layer) * p->S[t], p->S[t]));
        p->mapped[t][layer] = 0;
        if (p->uncompressed[layer]) PT_HIP(hipMemRelease(p->dedicated[t][layer]));
    }
    return FLUXMOE_OK;
}

}  // namespace

extern "C" {

int fluxmoe_paged_tensor_layout(const fluxmoe_desc* desc, uint64_t granularity, uint32_t n_uncompressed,
                                fluxmoe_paged_tensor_info* out) {
    return layout(desc, granularity, n_uncompressed, out);
}

int fluxmoe_paged_tensor_destroy(fluxmoe_paged_tensor* p) {
    if (!p) return FLUXMOE_OK;
    int rc = FLUXMOE_OK;
    auto keep = [&](int r) { if (r && !rc) rc = r; };
    for (uint32_t l = 0; l < p->mapped[0].size(); ++l) keep(unmap_layer(p, l));
    for (int t = 0; t < 2; ++t) {
        for (int b = 0; b < 2; ++b) {
            if (p->window_mapped[t][b] && hipMemUnmap(p->window[t] + uint64_t(b) * p->S[t], p->S[t]) != hipSuccess)
                keep(set_error(FLUXMOE_EHIP, "hipMemUnmap of the reusable window failed"));
            if (p->reusable_made[t][b] && hipMemRelease(p->reusable[t][b]) != hipSuccess)
                keep(set_error(FLUXMOE_EHIP, "hipMemRelease failed"));
        }
        if (p->v0[t]) (void)hipMemAddressFree(p->v0[t], uint64_t(p->d.n_layers) * p->S[t]);
        if (p->window[t]) (void)hipMemAddressFree(p->window[t], 2 * p->S[t]);
    }
    delete p;
    return rc;
}

int fluxmoe_paged_tensor_create(const fluxmoe_desc* desc, const uint8_t* uncompressed,
                                fluxmoe_paged_tensor** out) {
    if (!desc || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    fluxmoe_paged_tensor* p = new (std::nothrow) fluxmoe_paged_tensor;
    if (!p) return set_error(FLUXMOE_ENOMEM, "out of host memory");
    p->d = *desc;
    const uint32_t N = desc->n_layers;
    auto fail = [&](int rc) { fluxmoe_paged_tensor_destroy(p); return rc; };
    if (hipGetDevice(&p->device) != hipSuccess) return fail(set_error(FLUXMOE_EHIP, "hipGetDevice failed"));
    int supported = 0;
    if (hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, p->device) != hipSuccess ||
        !supported)
        return fail(set_error(FLUXMOE_EHIP, "the device does not support virtual memory management"));
    p->prop.type = hipMemAllocationTypePinned;
    p->prop.location.type = hipMemLocationTypeDevice;
    p->prop.location.id = p->device;
    p->access.location = p->prop.location;
    p->access.flags = hipMemAccessFlagsProtReadWrite;
    size_t g = 0;
    if (hipMemGetAllocationGranularity(&g, &p->prop, hipMemAllocationGranularityMinimum) != hipSuccess || g == 0)
        return fail(set_error(FLUXMOE_EHIP, "hipMemGetAllocationGranularity failed"));
    fluxmoe_paged_tensor_info li;
    if (int rc = layout(desc, g, 0, &li)) return fail(rc);
    p->g = g;
    p->uncompressed.assign(N, 0);
    if (uncompressed)
        for (uint32_t l = 0; l < N; ++l) p->uncompressed[l] = uncompressed[l] ? 1 : 0;
    for (int t = 0; t < 2; ++t) {
        p->A[t] = li.A[t];
        p->S[t] = li.S[t];
        p->sigma[t] = li.A[t] / desc->n_experts;
        p->mapped[t].assign(N, 0);
        p->dedicated[t].assign(N, hipMemGenericAllocationHandle_t{});
        void* va = nullptr;
        if (hipMemAddressReserve(&va, uint64_t(N) * p->S[t], g, nullptr, 0) != hipSuccess)
            return fail(set_error(FLUXMOE_EHIP, "hipMemAddressReserve of %llu bytes failed",
                                  (unsigned long long)(uint64_t(N) * p->S[t])));
        p->v0[t] = static_cast<uint8_t*>(va);
        if (hipMemAddressReserve(&va, 2 * p->S[t], g, nullptr, 0) != hipSuccess)
            return fail(set_error(FLUXMOE_EHIP, "hipMemAddressReserve of the reusable window failed"));
        p->window[t] = static_cast<uint8_t*>(va);
        for (int b = 0; b < 2; ++b) {
            if (hipMemCreate(&p->reusable[t][b], p->S[t], &p->prop, 0) != hipSuccess)
                return fail(set_error(FLUXMOE_ENOMEM, "hipMemCreate of a %llu-byte reusable block failed",
                                      (unsigned long long)p->S[t]));
            p->reusable_made[t][b] = true;
            if (int rc = map_range(p, p->window[t] + uint64_t(b) * p->S[t], p->S[t], p->reusable[t][b])) return fail(rc);
            p->window_mapped[t][b] = true;
        }
    }
    for (uint32_t l = 0; l < N; ++l)
        if (int rc = map_layer(p, l)) return fail(rc);
    *out = p;
    return FLUXMOE_OK;
}

int fluxmoe_paged_tensor_info_get(const fluxmoe_paged_tensor* p, fluxmoe_paged_tensor_info* out) {
    if (!p || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    uint32_t n_unc = 0;
    for (uint8_t u : p->uncompressed) n_unc += u;
    if (int rc = layout(&p->d, p->g, n_unc, out)) return rc;
    for (int t = 0; t < 2; ++t) {
        out->v0[t] = uint64_t(uintptr_t(p->v0[t]));
        out->reusable_window[t] = uint64_t(uintptr_t(p->window[t]));
    }
    return FLUXMOE_OK;
}

int fluxmoe_paged_tensor_address(const fluxmoe_paged_tensor* p, uint32_t layer, int type, uint32_t expert,
                                 void** out) {
    if (!p || !out) return set_error(FLUXMOE_EINVAL, "NULL argument");
    if (type != 1 && type != 2) return set_error(FLUXMOE_EINVAL, "type must be 1 or 2");
    if (layer >= p->d.n_layers || expert >= p->d.n_experts)
        return set_error(FLUXMOE_ERANGE, "layer %u / expert %u out of range", layer, expert);
    const int t = type - 1;
    *out = p->v0[t] + uint64_t(layer) * p->S[t] + uint64_t(expert) * p->sigma[t];
    return FLUXMOE_OK;
}

int fluxmoe_paged_tensor_set_class(fluxmoe_paged_tensor* p, uint32_t layer, int uncompressed) {
    if (!p) return set_error(FLUXMOE_EINVAL, "paged tensor is NULL");
    if (layer >= p->d.n_layers) return set_error(FLUXMOE_ERANGE, "layer %u out of range", layer);
    const uint8_t want = uncompressed ? 1 : 0;
    if (p->uncompressed[layer] == want) return FLUXMOE_OK;
    PT_HIP(hipDeviceSynchronize());          // no kernel may still use the old mapping
    if (int rc = unmap_layer(p, layer)) return rc;
    p->uncompressed[layer] = want;
    return map_layer(p, layer);
}

}  // extern "C"
