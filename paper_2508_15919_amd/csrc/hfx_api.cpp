// C ABI of libhfxattn (see include/hfxattn.h): argument checking, descriptor upload, launches.
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/hfxattn.h"
#include "hfx_desc.h"
#include "hfx_launch.h"
#include "hfx_plan.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// header of a descriptor this library wrote, matching `shape`
hfx_status check_header(const hfx_shape* shape, const void* host_desc, HfxHeader* out) {
  hfx_status st = hfx::check_shape(shape);
  if (st != HFX_OK) return st;
  if (!host_desc) return HFX_ERR_NULL;
  std::memcpy(out, host_desc, sizeof(HfxHeader));
  if (out->magic != HFX_DESC_MAGIC || out->version != HFX_DESC_VERSION) return HFX_ERR_DESC;
  if (out->num_q_heads != shape->num_q_heads || out->num_kv_heads != shape->num_kv_heads ||
      out->head_dim != shape->head_dim || out->page_size != shape->page_size ||
      out->num_pages != shape->num_pages)
    return HFX_ERR_SHAPE;
  return HFX_OK;
}

// Workgroups of the persistent launch on the current device: what fits on the chip at once (cached per
// device), but never more than the width the planner laid the queue out for -- its first rounds deal
// queue positions b and b + HFX_PLAN_WGS to workgroup b.
hfx_status persistent_grid(int head_dim, int* grid) {
  static std::mutex mu;
  static int cache[HFX_MAX_DEVICES][2];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return HFX_ERR_DEVICE;
  if (dev < 0 || dev >= HFX_MAX_DEVICES) return HFX_ERR_DEVICE;
  const int slot = head_dim == 128 ? 1 : 0;
  std::lock_guard<std::mutex> lock(mu);
  if (cache[dev][slot] == 0) {
    int cus = 0, per_cu = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return HFX_ERR_DEVICE;
    if (hfx::max_resident_workgroups(head_dim, &per_cu) != hipSuccess) return HFX_ERR_DEVICE;
    if (cus < 1 || per_cu < 1) return HFX_ERR_DEVICE;
    cache[dev][slot] = cus * per_cu < HFX_PLAN_WGS ? cus * per_cu : HFX_PLAN_WGS;
  }
  *grid = cache[dev][slot];
  return HFX_OK;
}

}  // namespace

namespace {

// The attention call proper; `h` is the descriptor's header, already checked against the shape.
hfx_status run_attention(const HfxHeader& h, const void* q, const void* kv_pool, void* device_desc, void* workspace,
                         size_t workspace_bytes, void* out, void* stream) {
  hfx_status st;
  if (h.workspace_bytes > 0 && !workspace) return HFX_ERR_NULL;
  if (workspace_bytes < h.workspace_bytes) return HFX_ERR_BUFSIZE;
  if (!aligned16(q) || !aligned16(kv_pool) || !aligned16(device_desc) || !aligned16(out) ||
      (h.workspace_bytes > 0 && !aligned16(workspace)))
    return HFX_ERR_ALIGN;
  if (h.n_items < 1) return HFX_ERR_DESC;
  if ((h.queue_classes != 1 && h.queue_classes != HFX_QUEUE_CLASSES) || h.n_ctrl <= HFX_QUEUE_CLASSES) return HFX_ERR_DESC;
  int grid = 0;
  st = persistent_grid(h.head_dim, &grid);
  if (st != HFX_OK) return st;
  if (grid > h.n_items) grid = h.n_items;
  if (hfx::launch_mixed_attention(h, grid, device_desc, q, kv_pool, workspace, out, static_cast<hipStream_t>(stream)) !=
      hipSuccess)
    return HFX_ERR_DEVICE;
  return HFX_OK;
}

}  // namespace

extern "C" {

const char* hfx_status_string(hfx_status s) {
  switch (s) {
    case HFX_OK: return "ok";
    case HFX_ERR_NULL: return "null pointer";
    case HFX_ERR_SHAPE: return "unsupported or inconsistent shape";
    case HFX_ERR_KIND: return "request kind is neither decode nor prefill";
    case HFX_ERR_LEN: return "query-chunk / context length out of range";
    case HFX_ERR_PAGES: return "block table malformed or too short";
    case HFX_ERR_PAGE_ID: return "page id outside the pool";
    case HFX_ERR_BUFSIZE: return "buffer too small";
    case HFX_ERR_DEVICE: return "HIP runtime error";
    case HFX_ERR_DESC: return "not a batch descriptor of this library version";
    case HFX_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case HFX_ERR_MODEL: return "latency model or SLO values not usable";
    default: return "unknown status";
  }
}

hfx_status hfx_version(int32_t* major, int32_t* minor) {
  if (major) *major = 0;
  if (minor) *minor = (int32_t)HFX_DESC_VERSION;
  return HFX_OK;
}

// One planner scratch per host thread: its vectors keep their capacity, so steady-state calls do
// not touch the allocator (fresh pages for a megabyte of items cost more than planning them).
static hfx::Plan& tls_plan() {
  static thread_local hfx::Plan plan;
  return plan;
}

hfx_status hfx_batch_desc_sizes(const hfx_shape* shape, int32_t num_requests, const int32_t* kind,
                                const int32_t* q_len, const int32_t* ctx_len, size_t* host_desc_bytes,
                                size_t* device_desc_bytes, size_t* device_workspace_bytes) {
  if (!host_desc_bytes || !device_desc_bytes || !device_workspace_bytes) return HFX_ERR_NULL;
  hfx::Plan& plan = tls_plan();
  hfx_status st = hfx::plan_step(shape, num_requests, kind, q_len, ctx_len, &plan);
  if (st != HFX_OK) return st;
  HfxHeader h;
  hfx::layout_blob(shape, plan, &h);
  *host_desc_bytes = (size_t)h.total_bytes;
  *device_desc_bytes = (size_t)h.total_bytes;
  *device_workspace_bytes = (size_t)h.workspace_bytes;
  return HFX_OK;
}

hfx_status hfx_fill_batch_desc(const hfx_shape* shape, int32_t num_requests, const int32_t* kind,
                               const int32_t* q_len, const int32_t* ctx_len, const int32_t* bt_indptr,
                               const int32_t* bt_pages, void* host_desc, size_t host_desc_bytes) {
  hfx::Plan& plan = tls_plan();
  hfx_status st = hfx::plan_step(shape, num_requests, kind, q_len, ctx_len, &plan);
  if (st != HFX_OK) return st;
  return hfx::fill_blob(shape, plan, bt_indptr, bt_pages, host_desc, host_desc_bytes);
}

hfx_status hfx_build_batch_desc(const hfx_shape* shape, int32_t num_requests, const int32_t* kind,
                                const int32_t* q_len, const int32_t* ctx_len, const int32_t* bt_indptr,
                                const int32_t* bt_pages, void* host_desc, size_t host_desc_bytes,
                                void* device_desc, size_t device_desc_bytes, void* stream) {
  if (!device_desc) return HFX_ERR_NULL;
  if (!aligned16(device_desc)) return HFX_ERR_ALIGN;
  hfx_status st = hfx_fill_batch_desc(shape, num_requests, kind, q_len, ctx_len, bt_indptr, bt_pages, host_desc,
                                      host_desc_bytes);
  if (st != HFX_OK) return st;
  HfxHeader h;
  std::memcpy(&h, host_desc, sizeof h);
  if (device_desc_bytes < h.total_bytes) return HFX_ERR_BUFSIZE;
  if (hipMemcpyAsync(device_desc, host_desc, (size_t)h.total_bytes, hipMemcpyHostToDevice,
                     static_cast<hipStream_t>(stream)) != hipSuccess)
    return HFX_ERR_DEVICE;
  return HFX_OK;
}

hfx_status hfx_mixed_paged_attention(const hfx_shape* shape, const void* q, const void* kv_pool,
                                     const void* host_desc, void* device_desc, void* workspace,
                                     size_t workspace_bytes, void* out, void* stream) {
  if (!q || !kv_pool || !device_desc || !out) return HFX_ERR_NULL;
  HfxHeader h;
  hfx_status st = check_header(shape, host_desc, &h);
  if (st != HFX_OK) return st;
  return run_attention(h, q, kv_pool, device_desc, workspace, workspace_bytes, out, stream);
}

hfx_status hfx_mixed_paged_attention_static(const hfx_shape* shape, const void* q, const void* kv_pool,
                                            const void* host_desc, void* device_desc, void* out,
                                            void* stream) {
  if (!q || !kv_pool || !device_desc || !out) return HFX_ERR_NULL;
  HfxHeader h;
  hfx_status st = check_header(shape, host_desc, &h);
  if (st != HFX_OK) return st;
  if (h.workspace_bytes > (uint64_t)HFX_STATIC_WS_BYTES) return HFX_ERR_BUFSIZE;
  void* ws = nullptr;
  if (hfx::static_workspace(&ws) != hipSuccess) return HFX_ERR_DEVICE;
  return run_attention(h, q, kv_pool, device_desc, ws, (size_t)HFX_STATIC_WS_BYTES, out, stream);
}

hfx_status hfx_gather_kv(const hfx_shape* shape, const void* kv_pool, const void* host_desc,
                         const void* device_desc, int32_t request, void* k_out, void* v_out, void* stream) {
  if (!kv_pool || !device_desc || !k_out || !v_out) return HFX_ERR_NULL;
  HfxHeader h;
  hfx_status st = check_header(shape, host_desc, &h);
  if (st != HFX_OK) return st;
  if (request < 0 || request >= h.num_requests) return HFX_ERR_LEN;
  const HfxReq* reqs = reinterpret_cast<const HfxReq*>(static_cast<const char*>(host_desc) + h.off_req);
  const long elements = (long)reqs[request].ctx_len * h.num_kv_heads * h.head_dim;
  if (hfx::launch_gather_kv(device_desc, kv_pool, request, elements, k_out, v_out,
                            static_cast<hipStream_t>(stream)) != hipSuccess)
    return HFX_ERR_DEVICE;
  return HFX_OK;
}

hfx_status hfx_append_kv(const hfx_shape* shape, const void* k_new, const void* v_new, void* kv_pool,
                         const void* host_desc, const void* device_desc, void* stream) {
  if (!k_new || !v_new || !kv_pool || !device_desc) return HFX_ERR_NULL;
  HfxHeader h;
  hfx_status st = check_header(shape, host_desc, &h);
  if (st != HFX_OK) return st;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(kv_pool) || !aligned16(device_desc)) return HFX_ERR_ALIGN;
  if (hfx::launch_append_kv(h, device_desc, k_new, v_new, kv_pool, static_cast<hipStream_t>(stream)) != hipSuccess)
    return HFX_ERR_DEVICE;
  return HFX_OK;
}

hfx_status hfx_copy_pages(const hfx_shape* shape, const void* src_pool, void* dst_pool, int32_t dst_num_pages,
                          int32_t num_pairs, const int32_t* src_ids, const int32_t* dst_ids, void* host_stage,
                          void* device_stage, size_t stage_bytes, void* stream) {
  hfx_status st = hfx::check_shape(shape);
  if (st != HFX_OK) return st;
  if (num_pairs < 0 || dst_num_pages < 1) return HFX_ERR_SHAPE;
  if (num_pairs == 0) return HFX_OK;
  if (!src_pool || !dst_pool || !src_ids || !dst_ids || !host_stage || !device_stage) return HFX_ERR_NULL;
  if (stage_bytes < 8ull * (size_t)num_pairs) return HFX_ERR_BUFSIZE;
  if (!aligned16(src_pool) || !aligned16(dst_pool) || !aligned16(device_stage)) return HFX_ERR_ALIGN;
  // a destination page is written once; inside one pool it is not read either
  static thread_local std::vector<uint8_t> mark;
  mark.assign((size_t)dst_num_pages, 0);
  for (int i = 0; i < num_pairs; ++i) {
    if (src_ids[i] < 0 || src_ids[i] >= shape->num_pages || dst_ids[i] < 0 || dst_ids[i] >= dst_num_pages)
      return HFX_ERR_PAGE_ID;
    if (mark[(size_t)dst_ids[i]]) return HFX_ERR_PAGES;
    mark[(size_t)dst_ids[i]] = 1;
  }
  if (src_pool == dst_pool)
    for (int i = 0; i < num_pairs; ++i)
      if (src_ids[i] < dst_num_pages && mark[(size_t)src_ids[i]]) return HFX_ERR_PAGES;
  int32_t* stage = static_cast<int32_t*>(host_stage);
  for (int i = 0; i < num_pairs; ++i) {
    stage[2 * i] = src_ids[i];
    stage[2 * i + 1] = dst_ids[i];
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(device_stage, host_stage, 8ull * (size_t)num_pairs, hipMemcpyHostToDevice, s) != hipSuccess)
    return HFX_ERR_DEVICE;
  const int units_per_page = shape->num_kv_heads * 2 * HFX_PAGE * shape->head_dim * 2 / 16;
  if (hfx::launch_copy_pages(device_stage, num_pairs, units_per_page, src_pool, dst_pool, s) != hipSuccess)
    return HFX_ERR_DEVICE;
  return HFX_OK;
}

}  // extern "C"
