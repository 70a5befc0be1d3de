// Internal layout of the batch descriptor shared by the host planner and the kernels.
// Plain-old-data, position independent: the blob is built on the host and copied verbatim.
#pragma once
#include <stdint.h>

#define HFX_DESC_MAGIC 0x31584648u /* "HFX1" */
#define HFX_DESC_VERSION 15u
#define HFX_PAGE 16
#define HFX_WG_THREADS 256
#define HFX_PLAN_WGS 512         /* planning width: 256 compute units x 2 resident workgroups */
#define HFX_KEY_TILE 64          /* key ranges of prefill items start at multiples of this */
#define HFX_STAGE_KEYS 32        /* keys per prefill pipeline stage (2 pages) */
#define HFX_BT_PAD 16            /* stored block-table entries after a request's last page, all naming that page */
#define HFX_WAVE_ROWS 32         /* query rows one wavefront owns in a prefill item (one MFMA row block) */
#define HFX_QUEUE_CLASSES 8      /* queue positions p with equal p % 8 form a class: one per accelerator die (XCD), each with an L2 of its own */

#define HFX_STATIC_WS_BYTES (64u << 20) /* fixed workspace of the entry point that allocates nothing */
#define HFX_MAX_DEVICES 64

enum { HFX_ITEM_DECODE = 0, HFX_ITEM_PREFILL = 1 };

struct HfxHeader {
  uint32_t magic, version;
  int32_t num_requests, total_q;
  int32_t num_q_heads, num_kv_heads, head_dim, page_size, num_pages;
  float softmax_scale;
  int32_t n_items, n_decode_items, n_prefill_items, n_groups;
  int32_t n_partial_rows;       /* workspace rows: one (query row, q-head) partial each */
  int32_t n_bt;                 /* page ids stored */
  uint32_t off_ctrl, off_req, off_bt, off_items, off_groups;
  uint32_t n_ctrl;              /* control words: [c], c < queue_classes: tickets of class c handed out past the two dealt
                                   to each workgroup by index; [HFX_QUEUE_CLASSES]: finished workgroups */
  uint64_t total_bytes;
  uint64_t workspace_bytes;
  uint64_t ws_off_ml;           /* byte offset of the (m, l) pairs inside the workspace; acc rows start at 0 */
  int32_t max_group_rows;       /* largest rows_per_split over the groups */
  int32_t n_units;              /* merge work units (one workgroup each) */
  uint32_t off_units;
  int32_t n_runs;               /* append runs: the new tokens of the step, cut at page boundaries */
  uint32_t off_runs;
  uint32_t queue_classes;       /* 1 or HFX_QUEUE_CLASSES: how many classes the queue positions past the dealt ones fall into */
  uint32_t reserved[2];
};

struct HfxReq {
  int32_t kind, q_len, ctx_len;
  int32_t q_start;              /* first packed query row */
  int32_t bt_start;             /* first entry in the stored block table; a multiple of 4 */
  int32_t n_pages;              /* ceil(ctx_len / 16) */
  int32_t bt_len;               /* entries stored: n_pages rounded up to 4, plus HFX_BT_PAD; those past
                                   n_pages repeat the last page, so that a tile's four ids can be fetched
                                   as one aligned quad without clamping, a little way past the end */
  int32_t pad1;
};

// The new tokens of one request that fall into one page: packed query rows [row0, row0 + n) go to
// slots [slot0, slot0 + n) of physical page `page`.  What the KV append walks.
struct HfxRun {
  int32_t row0, n, page, slot0;
};

// One unit of work for one workgroup.
//  decode : h0 = first kv-head, hn = kv-heads covered (1, 2 or 4; one wavefront per head, the
//           remaining wavefronts split the pages), kb/ke = request-relative page range.
//  prefill: h0 = first q-head, hn = q-heads covered (1, 2 or 4), row0 = first chunk row,
//           nrows = rows covered (32 * 4 / hn), kb/ke = key range in tokens (kb % 64 == 0).
//  group >= 0: the item is one of several splits; its partial goes to workspace rows
//           [slot_row, slot_row + rows) and the merge kernel combines the group afterwards.
//  home   : the queue class (0 .. HFX_QUEUE_CLASSES-1) whose workgroups the planner meant the item
//           for, or -1 where the queue order has no classes; planner bookkeeping, kernels ignore it.
//  The request's record is repeated inside the item so that a workgroup needs one dependent load
//  less between taking a ticket and issuing its first KV load.
struct HfxItem {
  int32_t type, req, group, slot_row;
  int32_t h0, hn, row0, nrows;
  int32_t kb, ke, cost, home;
  HfxReq rq;
};

// One merge group: nsplit partials of rows_per_split rows each, split s at workspace rows
// base_row + s * rows_per_split.  type/req/h0/hn/row0 are those of the group's items and say
// which output rows the merged result belongs to.

struct HfxGroup {
  int32_t nsplit;
  int32_t base_row;
  int32_t rows_per_split;
  int32_t type, req, h0, hn, row0;
  int32_t q_start, q_len;       /* of the request, so that the merge launch needs no third table */
};

// One workgroup of the merge launch: 8 / lanes rows of a group starting at row chunk * (8 / lanes),
// where lanes (8 or 1) is how many threads share the splits of one row.
struct HfxUnit {
  int32_t group, chunk;
};
