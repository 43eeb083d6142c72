// zm_layer: the compressed experts of one MoE layer, resident in device memory (ZipMoE, arXiv 2601.21198,
// Sec. 3.1: the serialised objects made offline are what the run-time system holds).  The handle keeps what
// the hot call otherwise takes as arrays -- device addresses, chunk tables, tensor descriptions -- so that a
// caller hands over expert ids and output buffers only.  It owns no device memory: the blobs live in an arena the
// caller provides.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>
#include <vector>

#include "zipmoe.h"

struct zm_layer {
    int n_experts = 0, tensors_per_expert = 0;
    std::vector<zm_tensor_info> infos;
    std::vector<const void *> blobs;                // device address of every blob
    std::vector<const uint64_t *> tables;           // device address of every chunk table (inside the blob)
    size_t bytes = 0;                               // of the arena in use
};

namespace {

constexpr size_t kAlign = 256;

inline size_t aligned(size_t n) { return (n + kAlign - 1) & ~(kAlign - 1); }

}  // namespace

extern "C" {

int zm_layer_arena_bytes(const size_t *blob_sizes, int n_tensors, size_t *bytes)
{
    if (!blob_sizes || !bytes || n_tensors <= 0) return ZM_E_ARG;
    size_t total = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const size_t a = aligned(blob_sizes[i]);
        if (a < blob_sizes[i] || total + a < total) return ZM_E_ARG;
        total += a;
    }
    *bytes = total;
    return ZM_OK;
}

int zm_layer_create(const void *const *host_blobs, const size_t *blob_sizes, int n_experts, int tensors_per_expert,
                    void *arena, size_t arena_bytes, zm_layer **out)
{
    if (out) *out = nullptr;
    if (!host_blobs || !blob_sizes || !arena || !out || n_experts <= 0 || tensors_per_expert <= 0 ||
        static_cast<int64_t>(n_experts) * tensors_per_expert > (1 << 24) ||
        (reinterpret_cast<uintptr_t>(arena) & (kAlign - 1))) return ZM_E_ARG;
    const int n = n_experts * tensors_per_expert;
    size_t need = 0;
    int rc = zm_layer_arena_bytes(blob_sizes, n, &need);
    if (rc != ZM_OK) return rc;
    if (need > arena_bytes) return ZM_E_SIZE;
    zm_layer *L = new (std::nothrow) zm_layer;
    if (!L) return ZM_E_NOMEM;
    try {
        L->infos.resize(n);
        L->blobs.resize(n);
        L->tables.resize(n);
    } catch (const std::bad_alloc &) {
        delete L;
        return ZM_E_NOMEM;
    }
    L->n_experts = n_experts;
    L->tensors_per_expert = tensors_per_expert;
    // every blob is checked in full before the first byte is uploaded: the kernels trust what is resident
    for (int i = 0; i < n; ++i) {
        if (!host_blobs[i]) rc = ZM_E_ARG;
        if (rc == ZM_OK) rc = zm_validate_blob(host_blobs[i], blob_sizes[i]);
        if (rc == ZM_OK) rc = zm_blob_info(host_blobs[i], blob_sizes[i], &L->infos[i]);
        if (rc == ZM_OK && L->infos[i].blob_size != blob_sizes[i]) rc = ZM_E_FORMAT;
        if (rc != ZM_OK) {
            delete L;
            return rc;
        }
    }
    uint8_t *at = static_cast<uint8_t *>(arena);
    for (int i = 0; i < n; ++i) {
        if (hipMemcpy(at, host_blobs[i], blob_sizes[i], hipMemcpyHostToDevice) != hipSuccess) {
            delete L;
            return ZM_E_HIP;
        }
        L->blobs[i] = at;
        L->tables[i] = reinterpret_cast<const uint64_t *>(at + L->infos[i].table_offset);
        at += aligned(blob_sizes[i]);
    }
    L->bytes = need;
    *out = L;
    return ZM_OK;
}

int zm_layer_tensor_info(const zm_layer *layer, int expert, int tensor, zm_tensor_info *info_out, const void **device_blob_out)
{
    if (!layer || !info_out || expert < 0 || expert >= layer->n_experts || tensor < 0 || tensor >= layer->tensors_per_expert)
        return ZM_E_ARG;
    const size_t i = static_cast<size_t>(expert) * layer->tensors_per_expert + tensor;
    *info_out = layer->infos[i];
    if (device_blob_out) *device_blob_out = layer->blobs[i];
    return ZM_OK;
}

int zm_layer_decode(const zm_layer *layer, const int32_t *expert_ids, int n_selected, void *const *out_bf16, int stores,
                    void *stream)
{
    if (!layer) return ZM_E_ARG;
    return zm_decode_experts_stores(layer->blobs.data(), layer->tables.data(), layer->infos.data(), layer->n_experts,
                                    layer->tensors_per_expert, expert_ids, n_selected, out_bf16, stores, stream);
}

void zm_layer_destroy(zm_layer *layer) { delete layer; }

}  // extern "C"
