/*
 * libhfxattn -- mixed prefill/decode attention over a block-paged bf16 KV cache,
 * for one scheduled serving step, on one AMD MI355X (gfx950).
 *
 * The operation behind this interface is the device work of one engine step as
 * HFX (arXiv 2508.15919) frames it: Section 2.1 names the two phases of a step
 * (prompt processing with full-sequence attention, compute bound; token
 * generation over cached KV states, memory-bandwidth bound), Section 3.3.1
 * fixes what a scheduler hands down for a step (which requests run, and how
 * many new tokens each contributes under the token budget), and Sections
 * 3.3.3 / 3.4 state that the KV cache is managed in fixed-size blocks.  The
 * paper does not define the attention operator further; the result computed
 * here is textbook scaled-dot-product attention with a causal mask and
 * grouped-query head sharing, defined precisely at hfx_mixed_paged_attention.
 *
 * C ABI only: plain pointers and sizes.  Every pointer argument is tagged
 * [host] or [device] below.  The library never allocates or frees device
 * memory and never synchronises a stream; the only memory it keeps between
 * calls is a host-side planner scratch per calling thread.  No function throws or
 * aborts; every failure is a negative hfx_status and, when it is a validation
 * failure, nothing has been enqueued on the stream.
 */
#ifndef HFXATTN_H
#define HFXATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t hfx_status;

enum {
  HFX_OK = 0,
  HFX_ERR_NULL = -1,     /* a required pointer is NULL                                  */
  HFX_ERR_SHAPE = -2,    /* hfx_shape is inconsistent or unsupported                    */
  HFX_ERR_KIND = -3,     /* kind[r] is neither HFX_DECODE nor HFX_PREFILL               */
  HFX_ERR_LEN = -4,      /* q_len / ctx_len violate 1 <= q_len <= ctx_len (decode: q=1) */
  HFX_ERR_PAGES = -5,    /* block table malformed or too short for ctx_len              */
  HFX_ERR_PAGE_ID = -6,  /* a page id needed by some request is outside [0, num_pages)  */
  HFX_ERR_BUFSIZE = -7,  /* a caller-provided buffer is too small                       */
  HFX_ERR_DEVICE = -8,   /* the HIP runtime reported an error                           */
  HFX_ERR_DESC = -9,     /* the descriptor blob is not one this library version wrote   */
  HFX_ERR_ALIGN = -10,   /* a device pointer is not 16-byte aligned                     */
  HFX_ERR_MODEL = -11    /* latency model or SLO values are not usable (see hfx_token_budget) */
};

/* Request kinds of a scheduled step (Section 3.3.1: in-flight decoding requests
 * versus newly admitted requests whose prompt tokens are processed). */
enum { HFX_DECODE = 0, HFX_PREFILL = 1 };

/* Shape constants of one attention layer and its page pool. */
typedef struct {
  int32_t num_q_heads;   /* Hq;  Hq % Hkv == 0, group size G = Hq/Hkv <= 16               */
  int32_t num_kv_heads;  /* Hkv; 1, 2, or a multiple of 4                                 */
  int32_t head_dim;      /* D in {64, 128}                                                */
  int32_t page_size;     /* tokens per KV block; must be 16                               */
  int32_t num_pages;     /* physical pages in the pool                                    */
  float softmax_scale;   /* multiplier of q.k before softmax; <= 0 selects 1/sqrt(D)      */
} hfx_shape;

/*
 * KV page pool layout (bf16, one device allocation, 16-byte aligned):
 *
 *   pool[num_pages][Hkv][2][16 * D]
 *
 * For page P and kv-head g the first 16*D elements are the keys, blocked by
 * groups of 16 dimensions: K[slot][d] at ((d / 16) * 16 + slot) * 16 + d % 16
 * (for each 16-dimension group, the 16 slots' 32-byte pieces are contiguous).
 * The second 16*D elements are the values, dimension-major: V[slot][d] at
 * (d * 16 + slot).  Both are the order in which the matrix cores consume the
 * operands, so a page streams into them without a transpose.  Logical token t
 * of a request lives in page bt_pages[bt_indptr[r] + t / 16] at slot t % 16
 * (block-managed cache, Sections 3.3.3 and 3.4).  Slots at or past ctx_len in
 * a request's last page, and pages no block table names, may hold anything
 * (including NaN) and never influence a result.
 */

/* Human-readable name of a status code (a utility of this interface; no passage of the paper behind
 * it).  Returns a static string. */
const char* hfx_status_string(hfx_status status);

/* Library version: major, and the descriptor layout version as minor (utility; no passage of the
 * paper behind it).  Either pointer may be NULL. [host] */
hfx_status hfx_version(int32_t* major, int32_t* minor);

/*
 * Sizes, in bytes, of the three caller-owned buffers a step needs.  Pure host
 * integer work; touches no device.
 *   host_desc_bytes        staging buffer for hfx_build_batch_desc (pinned memory
 *                          makes the upload asynchronous; pageable also works)
 *   device_desc_bytes      device buffer that receives the descriptor
 *   device_workspace_bytes device scratch for split partial results (may be 0)
 * kind, q_len, ctx_len: [host] arrays of num_requests entries, as below.
 * Errors: HFX_ERR_NULL, HFX_ERR_SHAPE, HFX_ERR_KIND, HFX_ERR_LEN.
 */
hfx_status hfx_batch_desc_sizes(const hfx_shape* shape, int32_t num_requests,
                                const int32_t* kind, const int32_t* q_len,
                                const int32_t* ctx_len, size_t* host_desc_bytes,
                                size_t* device_desc_bytes,
                                size_t* device_workspace_bytes);

/*
 * Turns the scheduler's statement of a step (Section 3.3.1: the admitted
 * requests and the number of new tokens each contributes, next to the
 * in-flight decodes) into the device-side batch descriptor: validated
 * per-request records, the block table, and the cost-ordered list of work
 * items (decode ranges, prefill tiles, split/merge groups) one launch drains.
 * Integer work only.
 *
 *   kind       [host][R]   HFX_DECODE or HFX_PREFILL
 *   q_len      [host][R]   query-chunk length; exactly 1 for HFX_DECODE
 *   ctx_len    [host][R]   KV tokens visible to the chunk's last query,
 *                          the chunk's own tokens included; >= q_len
 *   bt_indptr  [host][R+1] CSR offsets into bt_pages, bt_indptr[0] == 0,
 *                          non-decreasing; request r owns at least
 *                          ceil(ctx_len[r]/16) entries (extra ones are ignored)
 *   bt_pages   [host]      physical page ids in logical order; the ones a
 *                          request needs must lie in [0, num_pages).  Two
 *                          requests may name the same page (shared prefix).
 *   host_desc  [host]      staging memory, host_desc_bytes as reported above
 *   device_desc [device]   receives the descriptor, 16-byte aligned
 *   stream                 hipStream_t (NULL = default stream)
 *
 * The descriptor is written into host_desc and one asynchronous host-to-device
 * copy of it is enqueued on `stream`; host_desc must stay untouched until that
 * copy has completed.  The five input arrays are consumed before return.  The
 * descriptor is position independent (offsets, no pointers) and holds a few
 * control words that launches use and restore to zero, so one descriptor may
 * serve any number of launches (e.g. every layer of a step) as long as they
 * do not overlap in time.
 * Errors: every code above; nothing is enqueued unless HFX_OK is returned.
 */
hfx_status hfx_build_batch_desc(const hfx_shape* shape, int32_t num_requests,
                                const int32_t* kind, const int32_t* q_len,
                                const int32_t* ctx_len, const int32_t* bt_indptr,
                                const int32_t* bt_pages, void* host_desc,
                                size_t host_desc_bytes, void* device_desc,
                                size_t device_desc_bytes, void* stream);

/*
 * The host half of hfx_build_batch_desc alone: validates and writes the
 * descriptor into host_desc, touching no device and no stream.  For callers
 * that upload the blob themselves (total size: host_desc_bytes as reported by
 * hfx_batch_desc_sizes) -- e.g. as a copy node of their own.  Same inputs,
 * same errors except HFX_ERR_DEVICE / HFX_ERR_ALIGN.
 */
hfx_status hfx_fill_batch_desc(const hfx_shape* shape, int32_t num_requests,
                               const int32_t* kind, const int32_t* q_len,
                               const int32_t* ctx_len, const int32_t* bt_indptr,
                               const int32_t* bt_pages, void* host_desc,
                               size_t host_desc_bytes);

/*
 * Executes the attention of one scheduled step: one persistent launch drains
 * the step's work items, and, when the plan split some of them, one small
 * launch behind it on the same stream merges the partial results.
 *
 * With T = sum of q_len, requests packed in order (request r owns query rows
 * [sum_{s<r} q_len[s], +q_len[r])):
 *   q    [device] bf16 [T][Hq][D]
 *   out  [device] bf16 [T][Hq][D]
 * For request r, chunk row i (0 <= i < q_len[r]) and q-head h, let
 * g = h / (Hq/Hkv), n = ctx_len[r] - q_len[r] + i + 1 (the causal horizon; the
 * whole context for a decode), k_j / v_j the key / value of logical token j
 * and kv-head g fetched through the block table.  Then
 *   s_j = softmax_scale * <q, k_j>,  j in [0, n)
 *   out = sum_j softmax(s)_j * v_j
 * (Section 2.1: full-sequence attention for the prompt phase, attention over
 * cached KV states for the generation phase.)  Scores, softmax and the
 * weighted sum accumulate in fp32 (softmax weights are rounded to bf16 for the
 * second contraction); the result is rounded to bf16 nearest-even.
 *
 *   host_desc      [host]   the staging buffer hfx_build_batch_desc filled; only
 *                           its header is read (launch geometry), on the host
 *   device_desc    [device] descriptor uploaded by hfx_build_batch_desc
 * Pairing rule: host_desc and device_desc must hold the SAME descriptor, the one
 * written by one hfx_build_batch_desc (or hfx_fill_batch_desc plus the caller's
 * own upload) call.  The launch takes its item, group, merge-unit and run counts
 * and its table offsets from host_desc's header and walks device_desc with them;
 * it cannot see whether the two match.  A caller that refills a staging buffer
 * for the next step while an older device_desc is still being launched must
 * keep one staging buffer per device descriptor (the header is read during the
 * call itself, not later: once the call has returned host_desc may be reused).
 * The same rule holds for hfx_mixed_paged_attention_static, hfx_gather_kv and
 * hfx_append_kv.
 *   workspace      [device] device_workspace_bytes of scratch, 16-byte aligned;
 *                           contents need no initialisation; may be NULL when 0
 *
 * Asynchronous on `stream`; allocates nothing and synchronises nothing.
 * Errors: HFX_ERR_NULL, HFX_ERR_SHAPE (shape differs from the descriptor's),
 * HFX_ERR_DESC, HFX_ERR_BUFSIZE, HFX_ERR_ALIGN, HFX_ERR_DEVICE.
 */
hfx_status hfx_mixed_paged_attention(const hfx_shape* shape, const void* q,
                                     const void* kv_pool, const void* host_desc,
                                     void* device_desc, void* workspace,
                                     size_t workspace_bytes, void* out,
                                     void* stream);

/*
 * hfx_mixed_paged_attention for callers that cannot allocate device memory or
 * carry a workspace of their own: code under stream capture, tight serving
 * loops, harnesses that forbid allocation.  Same inputs, same kernels and same
 * result bits as hfx_mixed_paged_attention, but the split partials go to a
 * fixed workspace that lives inside the library's code object: 64 MiB
 * (67108864 bytes) per GPU, held from the library's first use on that GPU
 * until the process ends.  A step whose device_workspace_bytes (as
 * hfx_batch_desc_sizes reports it) exceeds that returns HFX_ERR_BUFSIZE and
 * enqueues nothing.
 *
 * The call allocates and frees nothing and calls no allocating routine; its
 * first call on a device looks the workspace's device address up once and
 * keeps it.  The workspace needs no clearing between calls (every partial a
 * merge reads was written by the same call first).  All calls on one GPU share
 * that one workspace: two of them, or one of them and nothing else that uses it,
 * must not overlap in time on that GPU (calls on one stream never do; calls on
 * different streams race).  hfx_mixed_paged_attention with a caller-owned
 * workspace is not affected and may overlap with it.
 * Errors: those of hfx_mixed_paged_attention.
 */
hfx_status hfx_mixed_paged_attention_static(const hfx_shape* shape, const void* q,
                                            const void* kv_pool, const void* host_desc,
                                            void* device_desc, void* out, void* stream);

/*
 * Paging check hook: copies the keys and values of request `request`, tokens
 * [0, ctx_len), all kv-heads, out of the page pool into token-major contiguous
 * buffers, walking the same device descriptor the attention kernel walks
 * (block-managed KV cache, Sections 3.3.3 and 3.4).  A pure byte copy.
 *   k_out, v_out [device] bf16 [ctx_len][Hkv][D] each
 * Errors: HFX_ERR_NULL, HFX_ERR_SHAPE, HFX_ERR_DESC, HFX_ERR_LEN (request out of
 * range), HFX_ERR_DEVICE.
 */
hfx_status hfx_gather_kv(const hfx_shape* shape, const void* kv_pool,
                         const void* host_desc, const void* device_desc,
                         int32_t request, void* k_out, void* v_out, void* stream);

/*
 * Writes the step's new keys and values into the page pool: the step just
 * before the attention of a scheduled step (Section 3.4: the instance's
 * execution loop fills its block-managed KV cache as tokens are processed;
 * Section 3.3.1: each request contributes q_len new tokens).  For request r the
 * chunk's rows i in [0, q_len[r]) are the logical tokens ctx_len[r] - q_len[r] + i;
 * token t goes to page bt_pages[bt_indptr[r] + t / 16], slot t % 16, in the pool
 * layout described above.  A pure byte move (bit-exact).
 *   k_new, v_new [device] bf16 [T][Hkv][D], rows packed like Q
 *   kv_pool      [device] the page pool, written in place
 *   host_desc / device_desc: the step's descriptor, as for the attention call
 * Pages shared between requests must not be written by two requests of the same
 * step (the caller's block manager guarantees this; it is not checked).
 * Asynchronous on `stream`; allocates nothing.
 * Errors: HFX_ERR_NULL, HFX_ERR_SHAPE, HFX_ERR_DESC, HFX_ERR_ALIGN, HFX_ERR_DEVICE.
 */
hfx_status hfx_append_kv(const hfx_shape* shape, const void* k_new, const void* v_new,
                         void* kv_pool, const void* host_desc, const void* device_desc,
                         void* stream);

/*
 * Copies whole KV pages between two pools of the same geometry (Hkv, D, page size), or inside
 * one pool: page src_ids[i] of src_pool becomes page dst_ids[i] of dst_pool, bit for bit.
 * This is the device half of handing a request's KV blocks from the instance that prefilled
 * it to the instance that decodes it (Section 3.3.1, disaggregated mode; Section 3.4), with
 * both pools on this GPU; the block table of the receiving side is dst_ids.
 *
 *   shape          geometry; shape->num_pages is the size of src_pool
 *   src_pool       [device] source pool, layout as at the top of this file
 *   dst_pool       [device] destination pool with dst_num_pages pages (may equal src_pool)
 *   src_ids, dst_ids [host] num_pairs page ids each.  dst ids are pairwise distinct; when the
 *                  pools are the same buffer no dst id is also a src id (HFX_ERR_PAGES)
 *   host_stage     [host]   >= 8*num_pairs bytes, written here and read by the upload: leave
 *                  it alone until the stream has passed this call (pinned memory keeps the
 *                  call asynchronous)
 *   device_stage   [device] >= 8*num_pairs bytes, 16-byte aligned
 *   stage_bytes    size of each staging buffer
 *
 * Asynchronous on `stream`; allocates no device memory.  num_pairs == 0 is a no-op.
 * Errors: HFX_ERR_NULL, HFX_ERR_SHAPE, HFX_ERR_PAGE_ID, HFX_ERR_PAGES, HFX_ERR_BUFSIZE,
 * HFX_ERR_ALIGN, HFX_ERR_DEVICE; on a validation error nothing is enqueued.
 */
hfx_status hfx_copy_pages(const hfx_shape* shape, const void* src_pool, void* dst_pool,
                          int32_t dst_num_pages, int32_t num_pairs, const int32_t* src_ids,
                          const int32_t* dst_ids, void* host_stage, void* device_stage,
                          size_t stage_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Step composition (host only): the closed forms of Section 3.3.1 that decide how many
 * prompt tokens a step may carry, and a one-instance form of the dispatching steps that
 * turns a waiting queue into the arrays hfx_build_batch_desc takes.
 * All times are in seconds.  Nothing here touches a device.
 * ---------------------------------------------------------------------------------------- */

/* Latency model of one instance (Section 3.3.1): a prefill batch of n prompt tokens takes
 * E_p = a + b*n (the linear model the paper adopts), a decode iteration of the current
 * running batch takes the constant E_d. */
typedef struct {
  double a;    /* fixed cost of a prefill batch, >= 0   */
  double b;    /* cost per prompt token, > 0            */
  double e_d;  /* duration of one decode iteration, >= 0 */
} hfx_latency_model;

/*
 * Token budget, Eq. (3): the largest integer n with 2*E_p + k*E_d <= TTFT, where
 * E_p = a + b*n and k = E_p / (TPOT - E_d), i.e.
 *   n <= (TPOT - E_d)*TTFT / ((2*TPOT - E_d)*b) - a/b.
 * Writes floor of the bound, clamped to [0, INT64_MAX/2], to *n_token.  When the decode
 * iteration leaves no slack (E_d >= TPOT) the budget is 0: no prefill can be absorbed.
 * Errors: HFX_ERR_NULL; HFX_ERR_MODEL if ttft or tpot <= 0, b <= 0, a < 0, e_d < 0, or any
 * value is not finite.
 */
hfx_status hfx_token_budget(double ttft, double tpot, const hfx_latency_model* model,
                            int64_t* n_token);

/*
 * Maturity time (Section 3.3.1): after a prefill batch of duration e_p, k = e_p/(TPOT - E_d)
 * decode iterations rebuild the slack the batch consumed (k is kept real-valued, as in the
 * paper's formula); the instance can admit again at  maturity = e_p + k*E_d.
 * Writes k and maturity (either pointer may be NULL).  With E_d >= TPOT there is no slack to
 * rebuild: returns HFX_ERR_MODEL.  Other errors as hfx_token_budget.
 */
hfx_status hfx_maturity_time(double e_p, double tpot, double e_d, double* k, double* maturity);

/*
 * Least-squares fit of E_p = a + b*n to measured prefill batches (n_token[i], seconds[i]),
 * i < count, count >= 2 with at least two distinct n_token.  Also writes the coefficient of
 * determination R^2 (may be NULL): the check of the paper's claim that the quadratic term
 * is negligible.  e_d of *model is left untouched.  a is clamped at 0.
 * Errors: HFX_ERR_NULL, HFX_ERR_MODEL (degenerate input or b <= 0).
 */
hfx_status hfx_fit_latency_model(int32_t count, const int64_t* n_token, const double* seconds,
                                 hfx_latency_model* model, double* r_squared);

/*
 * One dispatching decision for one instance (the four steps of Section 3.3.1 with a single
 * instance, so step 1 is trivial): compute the token budget from the strictest TTFT / TPOT
 * given, scan the waiting queue in ascending `urgency` (ties: queue order) and admit every
 * request whose prompt still fits in what is left of the budget, then predict E_p, k and the
 * new maturity time of the instance.
 *
 *   n_running, running_ctx   [host] in-flight decode requests and the KV tokens each has now
 *   n_waiting, prompt_len    [host] waiting requests and their prompt lengths (>= 1)
 *   urgency                  [host] smaller = more urgent (e.g. TTFT deadline); NULL = queue order
 *   mixed                    0: the step is the admitted prompts alone (the prefill batch that
 *                               pre-empts decoding, as in the paper's colocated mode);
 *                            1: the running requests' next decode tokens ride in the same step
 *   admitted                 [host] out, n_waiting flags (1 = dispatched in this step)
 *   kind, q_len, ctx_len     [host] out, capacity n_running + n_waiting each: the step in the
 *                            form hfx_batch_desc_sizes / hfx_build_batch_desc take.  Decodes
 *                            first (q 1, ctx running_ctx+1), then admitted prompts in scan
 *                            order (q = ctx = prompt_len)
 *   n_step                   [host] out, number of requests in the step (0 = nothing to run)
 *   decision                 [host] out, may be NULL
 * Errors: HFX_ERR_NULL, HFX_ERR_LEN (a length < 1), HFX_ERR_MODEL.
 */
typedef struct {
  int64_t budget;       /* Eq. (3)                                  */
  int64_t n_token;      /* prompt tokens admitted (<= budget)       */
  double e_p;           /* a + b*n_token (0 if nothing admitted)    */
  double k;             /* decode iterations until maturity         */
  double maturity;      /* e_p + k*E_d                              */
} hfx_decision;

hfx_status hfx_compose_step(double ttft, double tpot, const hfx_latency_model* model,
                            int32_t n_running, const int32_t* running_ctx, int32_t n_waiting,
                            const int32_t* prompt_len, const double* urgency, int32_t mixed,
                            int32_t* admitted, int32_t* kind, int32_t* q_len, int32_t* ctx_len,
                            int32_t* n_step, hfx_decision* decision);

#ifdef __cplusplus
}
#endif
#endif /* HFXATTN_H */
