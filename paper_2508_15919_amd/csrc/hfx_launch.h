// Host-callable launch helpers implemented next to the kernels (internal).
#pragma once
#include <hip/hip_runtime_api.h>

#include "hfx_desc.h"

namespace hfx {

hipError_t max_resident_workgroups(int head_dim, int* per_cu);
hipError_t launch_mixed_attention(const HfxHeader& header, int grid, void* desc, const void* q, const void* pool,
                                  void* ws, void* out, hipStream_t stream);
// Device address, on the current device, of the library's fixed workspace of HFX_STATIC_WS_BYTES
// (looked up once per device, then cached).
hipError_t static_workspace(void** ptr);
hipError_t launch_gather_kv(const void* desc, const void* pool, int request, long elements, void* k_out,
                            void* v_out, hipStream_t stream);

hipError_t launch_append_kv(const HfxHeader& h, const void* desc, const void* k_new, const void* v_new, void* pool,
                            hipStream_t stream);

hipError_t launch_copy_pages(const void* pairs, long n_pairs, int units_per_page, const void* src, void* dst,
                             hipStream_t stream);

}  // namespace hfx
