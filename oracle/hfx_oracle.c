/*
 * CPU oracle for mixed prefill/decode attention over a block-paged bf16 KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of the result,
 * in fp64, that the GPU library is checked against.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may build, load or call it.
 * It shares no code, header, table or helper with the GPU library.
 *
 * What is computed (HFX, arXiv 2508.15919): Section 2.1 says a step's prompt
 * phase runs full-sequence attention and its generation phase attends over
 * cached KV states; Sections 3.3.3 / 3.4 say the cache is held in blocks;
 * Section 3.3.1 says a step consists of requests each contributing a number of
 * new tokens.  The paper defines nothing beyond that, so the result is the
 * textbook one: for request r with chunk length q and context length c (the
 * chunk's tokens included), chunk row i sits at position c-q+i and attends
 * keys 0..c-q+i; q-head h reads kv-head h / (Hq/Hkv);
 *     s_j = scale * <q, k_j>,  w_j = exp(s_j - max s),  out = sum w_j v_j / sum w_j.
 * Every step is carried out in double precision on the exact values of the
 * bf16 inputs; the output is left in double.  No blocking, no splitting, no
 * reordering: one pass for the scores, one for the maximum, one for the
 * weights and the weighted sum.  OpenMP spreads independent (request, row,
 * head) units over cores and changes no arithmetic inside a unit.
 *
 * Pool layout read here: page-major, then kv-head, then K block, then V block;
 * a K block holds, for each group of 16 dimensions in turn, the 16 slots' 16
 * values (element (slot, d) at ((d/16)*16 + slot)*16 + d%16); a V block is
 * dimension-major (D rows of 16 slots).  Token t of request r: page
 * bt_pages[bt_indptr[r] + t/16], slot t%16.
 *
 * Pins (tests/test_oracle_pins.py): dense brute force on un-paged KV written
 * in numpy, torch's scaled_dot_product_attention in float64, single-token
 * context returns V bit-for-bit, page-permutation invariance, uniform-key and
 * constant-value closed forms, dominant-key limit, shift invariance,
 * chunk-split / decode-as-prefill / row-as-decode equivalences, GQA
 * duplicate-head equality, NaN poison in unreachable slots.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_PAGE 16

static double widen(uint16_t bits) {
  uint32_t u = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

typedef struct {
  int Hq, Hkv, D;
  long num_pages;
  const int32_t *bt_indptr, *bt_pages;
  const uint16_t* pool;
} orc_ctx;

/* element offset of the K block (which = 0) or V block (which = 1) of (page, kv-head) */
static size_t block_base(const orc_ctx* c, long page, int g, int which) {
  size_t blk = (size_t)ORC_PAGE * (size_t)c->D;
  return (((size_t)page * (size_t)c->Hkv + (size_t)g) * 2u + (size_t)which) * blk;
}

/* element offset of (slot, d) inside a K block */
static size_t k_offset(int slot, int d) { return ((size_t)(d / 16) * ORC_PAGE + (size_t)slot) * 16u + (size_t)(d % 16); }

static double key_at(const orc_ctx* c, int r, long t, int g, int d) {
  long page = c->bt_pages[c->bt_indptr[r] + t / ORC_PAGE];
  int slot = (int)(t % ORC_PAGE);
  return widen(c->pool[block_base(c, page, g, 0) + k_offset(slot, d)]);
}

static double value_at(const orc_ctx* c, int r, long t, int g, int d) {
  long page = c->bt_pages[c->bt_indptr[r] + t / ORC_PAGE];
  int slot = (int)(t % ORC_PAGE);
  return widen(c->pool[block_base(c, page, g, 1) + (size_t)d * ORC_PAGE + slot]);
}

/* one (request, chunk row, q-head) unit; n = number of visible keys; s = scratch of n doubles */
static void one_unit(const orc_ctx* c, double scale, int r, long n, int h, const uint16_t* qrow,
                     double* s, double* out) {
  int D = c->D;
  int g = h / (c->Hq / c->Hkv);
  for (long j = 0; j < n; ++j) {
    double dot = 0.0;
    for (int d = 0; d < D; ++d) dot += widen(qrow[d]) * key_at(c, r, j, g, d);
    s[j] = scale * dot;
  }
  double m = s[0];
  for (long j = 1; j < n; ++j)
    if (s[j] > m) m = s[j];
  double ell = 0.0;
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  for (long j = 0; j < n; ++j) {
    double w = exp(s[j] - m);
    ell += w;
    for (int d = 0; d < D; ++d) out[d] += w * value_at(c, r, j, g, d);
  }
  for (int d = 0; d < D; ++d) out[d] /= ell;
}

static int check_inputs(int Hq, int Hkv, int D, long num_pages, int R, const int32_t* kind,
                        const int32_t* q_len, const int32_t* ctx_len, const int32_t* bt_indptr,
                        const int32_t* bt_pages) {
  if (Hq <= 0 || Hkv <= 0 || D <= 0 || D % 16 != 0 || Hq % Hkv != 0 || num_pages <= 0 || R < 0) return -2;
  if (bt_indptr[0] != 0) return -5;
  for (int r = 0; r < R; ++r) {
    if (kind[r] != 0 && kind[r] != 1) return -3;
    if (q_len[r] < 1 || ctx_len[r] < q_len[r]) return -4;
    if (kind[r] == 0 && q_len[r] != 1) return -4;
    long have = (long)bt_indptr[r + 1] - bt_indptr[r];
    long need = ((long)ctx_len[r] + ORC_PAGE - 1) / ORC_PAGE;
    if (have < need) return -5;
    for (long i = 0; i < need; ++i) {
      long p = bt_pages[bt_indptr[r] + i];
      if (p < 0 || p >= num_pages) return -6;
    }
  }
  return 0;
}

int hfx_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* out: double [T][Hq][D], T = sum q_len, requests packed in order.  scale <= 0 means 1/sqrt(D). */
int hfx_oracle_attention(int Hq, int Hkv, int D, long num_pages, double scale, int R,
                         const int32_t* kind, const int32_t* q_len, const int32_t* ctx_len,
                         const int32_t* bt_indptr, const int32_t* bt_pages, const uint16_t* q,
                         const uint16_t* pool, double* out) {
  int rc = check_inputs(Hq, Hkv, D, num_pages, R, kind, q_len, ctx_len, bt_indptr, bt_pages);
  if (rc) return rc;
  if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
  orc_ctx c = {Hq, Hkv, D, num_pages, bt_indptr, bt_pages, pool};
  long T = 0, cmax = 0;
  for (int r = 0; r < R; ++r) {
    T += q_len[r];
    if (ctx_len[r] > cmax) cmax = ctx_len[r];
  }
  /* flat list of (request, row) so that the parallel loop has independent units */
  int32_t* unit_r = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
  int32_t* unit_i = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
  if (!unit_r || !unit_i) { free(unit_r); free(unit_i); return -7; }
  long u = 0;
  for (int r = 0; r < R; ++r)
    for (int i = 0; i < q_len[r]; ++i) { unit_r[u] = r; unit_i[u] = i; ++u; }
  int fail = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(cmax > 0 ? cmax : 1));
    if (!s) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (long t = 0; t < T; ++t)
      for (int h = 0; h < Hq; ++h) {
        if (!s) continue;
        int r = unit_r[t], i = unit_i[t];
        long n = (long)ctx_len[r] - q_len[r] + i + 1;
        one_unit(&c, scale, r, n, h, q + ((size_t)t * Hq + h) * D, s, out + ((size_t)t * Hq + h) * D);
      }
    free(s);
  }
  free(unit_r);
  free(unit_i);
  return fail ? -7 : 0;
}

/* Selected outputs only: sample k is (request sample_req[k], chunk row sample_row[k], q-head
 * sample_head[k]); out: double [n_samples][D].  Same arithmetic as the full call. */
int hfx_oracle_attention_rows(int Hq, int Hkv, int D, long num_pages, double scale, int R,
                              const int32_t* kind, const int32_t* q_len, const int32_t* ctx_len,
                              const int32_t* bt_indptr, const int32_t* bt_pages, const uint16_t* q,
                              const uint16_t* pool, long n_samples, const int32_t* sample_req,
                              const int32_t* sample_row, const int32_t* sample_head, double* out) {
  int rc = check_inputs(Hq, Hkv, D, num_pages, R, kind, q_len, ctx_len, bt_indptr, bt_pages);
  if (rc) return rc;
  if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
  orc_ctx c = {Hq, Hkv, D, num_pages, bt_indptr, bt_pages, pool};
  long cmax = 0;
  long* q_start = (long*)malloc(sizeof(long) * (size_t)(R + 1));
  if (!q_start) return -7;
  q_start[0] = 0;
  for (int r = 0; r < R; ++r) {
    q_start[r + 1] = q_start[r] + q_len[r];
    if (ctx_len[r] > cmax) cmax = ctx_len[r];
  }
  for (long k = 0; k < n_samples; ++k) {
    int r = sample_req[k];
    if (r < 0 || r >= R || sample_row[k] < 0 || sample_row[k] >= q_len[r] || sample_head[k] < 0 ||
        sample_head[k] >= Hq) {
      free(q_start);
      return -4;
    }
  }
  int fail = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(cmax > 0 ? cmax : 1));
    if (!s) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (long k = 0; k < n_samples; ++k) {
      if (!s) continue;
      int r = sample_req[k], i = sample_row[k], h = sample_head[k];
      long n = (long)ctx_len[r] - q_len[r] + i + 1;
      long t = q_start[r] + i;
      one_unit(&c, scale, r, n, h, q + ((size_t)t * Hq + h) * D, s, out + (size_t)k * D);
    }
    free(s);
  }
  free(q_start);
  return fail ? -7 : 0;
}

/* Un-pages request `request`: k_out, v_out are uint16 [ctx_len][Hkv][D], bit copies. */
int hfx_oracle_gather_kv(int Hkv, int D, long num_pages, int R, const int32_t* ctx_len,
                         const int32_t* bt_indptr, const int32_t* bt_pages, const uint16_t* pool,
                         int request, uint16_t* k_out, uint16_t* v_out) {
  if (request < 0 || request >= R) return -4;
  if (D <= 0 || D % 16 != 0) return -2;
  orc_ctx c = {Hkv, Hkv, D, num_pages, bt_indptr, bt_pages, pool};
  long n = ctx_len[request];
  for (long t = 0; t < n; ++t) {
    long page = bt_pages[bt_indptr[request] + t / ORC_PAGE];
    if (page < 0 || page >= num_pages) return -6;
    int slot = (int)(t % ORC_PAGE);
    for (int g = 0; g < Hkv; ++g)
      for (int d = 0; d < D; ++d) {
        size_t o = ((size_t)t * Hkv + g) * D + d;
        k_out[o] = pool[block_base(&c, page, g, 0) + k_offset(slot, d)];
        v_out[o] = pool[block_base(&c, page, g, 1) + (size_t)d * ORC_PAGE + slot];
      }
  }
  return 0;
}

/* Writes the new tokens of every request into the pool (in place): chunk row i of request r is
 * logical token ctx_len - q_len + i (Section 3.4: the engine loop fills the block-managed cache;
 * Section 3.3.1: q_len new tokens per request).  k_new, v_new: uint16 [T][Hkv][D]. */
int hfx_oracle_append_kv(int Hkv, int D, long num_pages, int R, const int32_t* q_len,
                         const int32_t* ctx_len, const int32_t* bt_indptr, const int32_t* bt_pages,
                         const uint16_t* k_new, const uint16_t* v_new, uint16_t* pool) {
  if (D <= 0 || D % 16 != 0 || Hkv <= 0) return -2;
  orc_ctx c = {Hkv, Hkv, D, num_pages, bt_indptr, bt_pages, pool};
  long row = 0;
  for (int r = 0; r < R; ++r) {
    if (q_len[r] < 1 || ctx_len[r] < q_len[r]) return -4;
    for (int i = 0; i < q_len[r]; ++i, ++row) {
      long t = (long)ctx_len[r] - q_len[r] + i;
      long page = bt_pages[bt_indptr[r] + t / ORC_PAGE];
      if (page < 0 || page >= num_pages) return -6;
      int slot = (int)(t % ORC_PAGE);
      for (int g = 0; g < Hkv; ++g)
        for (int d = 0; d < D; ++d) {
          size_t src = ((size_t)row * Hkv + g) * D + d;
          pool[block_base(&c, page, g, 0) + k_offset(slot, d)] = k_new[src];
          pool[block_base(&c, page, g, 1) + (size_t)d * ORC_PAGE + slot] = v_new[src];
        }
    }
  }
  return 0;
}

/* Page copy between two pools of one geometry: page src_ids[i] of src becomes page dst_ids[i] of
 * dst, element by element (the KV blocks of a request handed from a prefill instance to a decode
 * instance, Section 3.3.1 disaggregated mode / Section 3.4).  A page is Hkv*2*16*D elements. */
int hfx_oracle_copy_pages(int Hkv, int D, long src_num_pages, long dst_num_pages, long n,
                          const int32_t* src_ids, const int32_t* dst_ids, const uint16_t* src,
                          uint16_t* dst) {
  if (D <= 0 || Hkv <= 0) return -2;
  const size_t page_elems = (size_t)Hkv * 2 * ORC_PAGE * (size_t)D;
  for (long i = 0; i < n; ++i) {
    if (src_ids[i] < 0 || src_ids[i] >= src_num_pages || dst_ids[i] < 0 || dst_ids[i] >= dst_num_pages) return -6;
    for (size_t e = 0; e < page_elems; ++e)
      dst[(size_t)dst_ids[i] * page_elems + e] = src[(size_t)src_ids[i] * page_elems + e];
  }
  return 0;
}
