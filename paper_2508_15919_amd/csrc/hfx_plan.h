// Host planner interface (internal).  See hfx_plan.cpp.
#pragma once
#include <stddef.h>

#include <vector>

#include "../../include/hfxattn.h"
#include "hfx_desc.h"

namespace hfx {

struct Plan {
  std::vector<HfxReq> reqs;
  std::vector<HfxItem> items;
  std::vector<HfxGroup> groups;
  std::vector<HfxUnit> units;
  int32_t total_q = 0, n_bt = 0, n_partial_rows = 0, n_decode_items = 0, n_prefill_items = 0, n_runs = 0;
  int32_t queue_classes = 1;            // 1: plain queue; HFX_QUEUE_CLASSES: one list per die, interleaved by position
  // scratch of plan_step, kept so that a reused Plan allocates nothing once it has grown
  std::vector<uint64_t> sort_keys;
  std::vector<uint32_t> order;          // queue position -> index into items
  std::vector<int32_t> split_cost;
  std::vector<uint32_t> order_dec, order_pre;
  std::vector<uint32_t> item_unit;      // item -> sharing unit (see the queue order in plan_step)
  std::vector<float> item_frac;         // prefill item -> its row tile's place in the chunk, in [0, 1)
  std::vector<int64_t> unit_cost;
  std::vector<uint32_t> unit_fill, unit_start;
  std::vector<uint64_t> unit_keys;
};

hfx_status check_shape(const hfx_shape* shape);
hfx_status plan_step(const hfx_shape* shape, int32_t num_requests, const int32_t* kind, const int32_t* q_len,
                     const int32_t* ctx_len, Plan* out);
void layout_blob(const hfx_shape* shape, const Plan& plan, HfxHeader* header);
hfx_status fill_blob(const hfx_shape* shape, Plan& plan, const int32_t* bt_indptr, const int32_t* bt_pages,
                     void* host_desc, size_t host_desc_bytes);

}  // namespace hfx
