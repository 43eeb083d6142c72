// zm_decode_host_tensors: the decode of tensors whose serialised form lies in host memory, for callers that
// can not allocate device memory.  The compressed bytes are staged in a fixed device array that is part of
// the library's image, copied there on the caller's stream, and decoded from there by the same kernels as
// zm_decode_tensors; the call allocates nothing.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "zipmoe.h"

namespace {

// The staging area.  Every device the library runs on holds its own copy of this array, at its own address,
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) uint8_t scratch[ZM_STAGING_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<uint8_t *> g_scratch[kMaxDevices];      // device address of `scratch` on each device, once known

// Address of the current device's staging area; asked of the runtime on the first call on that device.
uint8_t *staging_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    uint8_t *p = g_scratch[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
    p = static_cast<uint8_t *>(sym);
    g_scratch[dev].store(p, std::memory_order_release);     // two first calls at once store the same address
    return p;
}

constexpr int kMaxTensors = 256;

}  // namespace

extern "C" int zm_decode_host_tensors(const void *const *host_blobs, const zm_tensor_info *infos, int n_tensors,
                                      void *const *out_bf16, void *stream)
{
    if (n_tensors == 0) return ZM_OK;
    if (!host_blobs || !infos || !out_bf16 || n_tensors < 0 || n_tensors > kMaxTensors) return ZM_E_ARG;
    // every blob keeps its section alignment when it starts at a multiple of 256 (blob sizes are multiples of 256)
    uint64_t total = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const zm_tensor_info &t = infos[i];
        if (t.n_values == 0) continue;
        if (!host_blobs[i] || (t.blob_size & 255) || t.lut_offset > t.table_offset || t.table_offset > t.sm_offset ||
            t.sm_offset > t.e_offset || t.e_offset > t.blob_size) return ZM_E_ARG;
        total += t.blob_size;
        if (total > ZM_STAGING_BYTES) return ZM_E_SIZE;
    }
    uint8_t *base = staging_of_current_device();
    if (!base) return ZM_E_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    zm_tensor_parts parts[kMaxTensors];
    uint64_t at = 0;
    for (int i = 0; i < n_tensors; ++i) {
        const zm_tensor_info &t = infos[i];
        parts[i] = zm_tensor_parts{nullptr, nullptr, nullptr, nullptr};
        if (t.n_values == 0) continue;
        uint8_t *dst = base + at;
        // header and code lengths are not needed on the device: the copy starts at the decode table
        if (hipMemcpyAsync(dst + t.lut_offset, static_cast<const uint8_t *>(host_blobs[i]) + t.lut_offset,
                           t.blob_size - t.lut_offset, hipMemcpyHostToDevice, s) != hipSuccess) return ZM_E_HIP;
        parts[i] = zm_tensor_parts{dst + t.lut_offset, dst + t.table_offset, dst + t.sm_offset, dst + t.e_offset};
        at += t.blob_size;
    }
    return zm_decode_tensors(parts, infos, n_tensors, out_bf16, stream);
}
