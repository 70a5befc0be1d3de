// Host planner: turns the scheduler's statement of a step (HFX Section 3.3.1: which requests
// run and how many new tokens each contributes) into the batch descriptor one persistent launch
// drains.  Integer work only; no device calls in this file.
#include "hfx_plan.h"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace hfx {

// Relative cost model, in nanoseconds of one resident workgroup when the whole chip runs that
// kind of work: decode streams KV bytes (about 6 TB/s over HFX_PLAN_WGS workgroups), prefill
// does MFMA flops (about 1 PFLOP/s over HFX_PLAN_WGS workgroups).  Only ratios matter: they
// order the queue and size the splits.
static const double kDecodeBytesPerNs = 12.0;
static const double kPrefillFlopsPerNs = 2000.0;
static const double kMinItemNs = 32000.0;
static const int kMinDecodeTokens = 128;
static const int kMinPrefillKeys = 256;
static const int kMaxSplits = 64;
static const int kDecodeItemsPerWg = 4;    // decode partials are small (rows of D + 2 floats per q-head)
// Which prefill-dominated steps get a queue per die (see the queue order in plan_step), by items per
// workgroup of the planning width.  Steps of many short items gain nothing from it (their time
// goes into item hand-overs, not into key traffic).  In the first rounds all workgroups of a die
// start together, and those that read the same keys then move in step: every cache line is a
// first touch for all of them at once, its full memory latency shows in each, and a tile takes up
// to twice as long as when neighbours run a little ahead and leave the lines in the L2.  Later
// rounds start staggered.  Steps of fewer than three rounds therefore keep the plain order.
static const int kClassRoundsMin = 3;
static const int kClassRoundsMax = 8;
static const int kFitRounds = 6;           // steps with fewer rounds of prefill items than this get whole rounds
static const int kPrefillItemsPerWg = 2;   // prefill partials are 128 rows: split only where balance needs it
static const uint32_t kNoUnit = 0x0fffffffu;   // items that share keys with no other item

static int kv_heads_per_item(int Hkv) { return (Hkv % 4 == 0) ? 4 : (Hkv % 2 == 0 ? 2 : 1); }
static int q_heads_per_item(int G) { return (G % 4 == 0) ? 4 : (G % 2 == 0 ? 2 : 1); }

hfx_status check_shape(const hfx_shape* s) {
  if (!s) return HFX_ERR_NULL;
  if (s->num_q_heads <= 0 || s->num_kv_heads <= 0) return HFX_ERR_SHAPE;
  if (s->num_q_heads % s->num_kv_heads != 0) return HFX_ERR_SHAPE;
  if (s->num_q_heads / s->num_kv_heads > 16) return HFX_ERR_SHAPE;
  if (s->num_kv_heads > 2 && s->num_kv_heads % 4 != 0) return HFX_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return HFX_ERR_SHAPE;
  if (s->page_size != HFX_PAGE) return HFX_ERR_SHAPE;
  if (s->num_pages < 1) return HFX_ERR_SHAPE;
  if (!(s->softmax_scale == s->softmax_scale)) return HFX_ERR_SHAPE;
  return HFX_OK;
}

// visible (row, key) pairs of chunk rows [r0, r1) against keys [kb, ke); row i sees keys <= p+i.
// Rows below i_lo see nothing of the range, rows from i_hi on see all of it, the rows between
// see p+i+1-kb keys (an arithmetic series).
static int64_t pairs_in(int64_t p, int64_t r0, int64_t r1, int64_t kb, int64_t ke) {
  if (ke <= kb || r1 <= r0) return 0;
  const int64_t i_lo = std::min(r1, std::max(r0, kb - p));
  const int64_t i_hi = std::min(r1, std::max(i_lo, ke - p - 1));
  const int64_t n = i_hi - i_lo;
  return n * (p + 1 - kb) + (i_lo + i_hi - 1) * n / 2 + (r1 - i_hi) * (ke - kb);
}

// How the keys a row tile (chunk rows [r0, r1) behind p earlier tokens) sees are cut into items
// of at most about cap_ns each: nsplit pieces of tiles_per key tiles (the last may be shorter).
static void prefill_splits(int64_t p, int64_t r0, int64_t r1, int D, int hpw, double cap_ns, int64_t* nsplit_out,
                           int64_t* tiles_per_out) {
  const int64_t kmax = p + r1;
  const int64_t ntiles = (kmax + HFX_KEY_TILE - 1) / HFX_KEY_TILE;
  const double ns_all = 4.0 * D * hpw * (double)pairs_in(p, r0, r1, 0, kmax) / kPrefillFlopsPerNs;
  int64_t nsplit = (int64_t)std::ceil(ns_all / cap_ns);
  nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, kMaxSplits));
  int64_t tiles_per = (ntiles + nsplit - 1) / nsplit;
  tiles_per = std::max<int64_t>(tiles_per, kMinPrefillKeys / HFX_KEY_TILE);
  *nsplit_out = (ntiles + tiles_per - 1) / tiles_per;
  *tiles_per_out = tiles_per;
}

static int32_t clamp_cost(double ns) {
  if (ns < 1.0) return 1;
  if (ns > 2.0e9) return 2000000000;
  return (int32_t)ns;
}

hfx_status plan_step(const hfx_shape* shape, int32_t R, const int32_t* kind, const int32_t* q_len,
                     const int32_t* ctx_len, Plan* out) {
  hfx_status st = check_shape(shape);
  if (st != HFX_OK) return st;
  if (!kind || !q_len || !ctx_len || !out) return HFX_ERR_NULL;
  if (R < 1) return HFX_ERR_SHAPE;
  const int Hq = shape->num_q_heads, Hkv = shape->num_kv_heads, D = shape->head_dim;
  const int G = Hq / Hkv;

  Plan& P = *out;
  P.reqs.assign((size_t)R, HfxReq());
  P.items.clear();
  P.groups.clear();
  P.item_unit.clear();
  P.item_frac.clear();
  int64_t T = 0, nbt = 0;
  double dec_ns = 0.0, pre_ns = 0.0;   // modelled time of each kind of work
  for (int r = 0; r < R; ++r) {
    if (kind[r] != HFX_DECODE && kind[r] != HFX_PREFILL) return HFX_ERR_KIND;
    if (q_len[r] < 1 || ctx_len[r] < q_len[r]) return HFX_ERR_LEN;
    if (kind[r] == HFX_DECODE && q_len[r] != 1) return HFX_ERR_LEN;
    HfxReq& q = P.reqs[(size_t)r];
    q.kind = kind[r];
    q.q_len = q_len[r];
    q.ctx_len = ctx_len[r];
    q.n_pages = (int32_t)(((int64_t)ctx_len[r] + HFX_PAGE - 1) / HFX_PAGE);
    q.bt_len = ((q.n_pages + 3) & ~3) + HFX_BT_PAD;
    if (T > 0x7fffffff - q_len[r] || nbt > 0x7fffffff - q.bt_len) return HFX_ERR_LEN;
    q.q_start = (int32_t)T;
    q.bt_start = (int32_t)nbt;
    T += q_len[r];
    nbt += q.bt_len;
    if (kind[r] == HFX_DECODE) {
      dec_ns += (double)ctx_len[r] * Hkv * D * 4.0 / kDecodeBytesPerNs;
    } else {
      double ql = q_len[r], p = ctx_len[r] - q_len[r];
      pre_ns += 4.0 * D * Hq * (ql * p + ql * (ql + 1) / 2) / kPrefillFlopsPerNs;
    }
  }
  P.total_q = (int32_t)T;
  P.n_bt = (int32_t)nbt;
  int64_t n_runs = 0;   // pages touched by each request's new tokens
  for (int r = 0; r < R; ++r)
    n_runs += (ctx_len[r] - 1) / HFX_PAGE - (ctx_len[r] - q_len[r]) / HFX_PAGE + 1;
  P.n_runs = (int32_t)n_runs;
  const double total_ns = dec_ns + pre_ns;
  // Decode pieces are sized against the decode work alone (in a step dominated by prefill they stay
  // small and fill the gaps between the large prefill items), for a whole number of rounds of the
  // planning width: as many rounds as fit pieces of at least the minimum size, at most
  // kDecodeItemsPerWg.  A step with work for 2.4 rounds of minimum-size pieces is better served by
  // two rounds of larger ones than by a third, half-empty round.
  double rounds = std::floor(dec_ns / (HFX_PLAN_WGS * kMinItemNs));
  rounds = std::min<double>(std::max(rounds, 1.0), kDecodeItemsPerWg);
  const double cap_ns = std::max(dec_ns / (HFX_PLAN_WGS * rounds), kMinItemNs);
  double cap_prefill_ns = std::max(total_ns / (HFX_PLAN_WGS * kPrefillItemsPerWg), kMinItemNs);
  // In a decode-dominated step the prefill items run beside the decode stream on CUs of their own
  // (see the queue order below) and only have to be done when it is: pieces of up to 0.6 of the
  // step's expected duration save partials and merge work (1 % on the Llama-8B-shaped mixed step;
  // at 0.75, unsplit there, the longest item starts to decide the step).
  if (dec_ns > pre_ns) cap_prefill_ns = std::max(cap_prefill_ns, 0.6 * total_ns / HFX_PLAN_WGS);

  const int ngc = kv_heads_per_item(Hkv);
  const int hpw = q_heads_per_item(G);
  const int rows_wg = HFX_WAVE_ROWS * (4 / hpw);
  // A prefill-dominated step of few, about equally expensive items per workgroup lasts a whole
  // number of items: 2.25 items per workgroup take as long as 3.  Where the cut above leaves a
  // partly filled last round, the cap is raised (by up to a half) to the smallest value at which
  // the prefill items fill whole rounds of the planning width.
  if (pre_ns > dec_ns) {
    auto count_items = [&](double cap) {
      int64_t count = 0;
      for (int r = 0; r < R; ++r) {
        if (kind[r] != HFX_PREFILL) continue;
        const int64_t p = ctx_len[r] - q_len[r];
        const int n_rt = (q_len[r] + rows_wg - 1) / rows_wg;
        for (int rt = 0; rt < n_rt; ++rt) {
          const int64_t r0 = (int64_t)rt * rows_wg, r1 = std::min<int64_t>(q_len[r], r0 + rows_wg);
          int64_t nsplit, tiles_per;
          prefill_splits(p, r0, r1, D, hpw, cap, &nsplit, &tiles_per);
          count += nsplit * Hkv * (G / hpw);
        }
      }
      return count;
    };
    const int64_t n0 = count_items(cap_prefill_ns);
    const int64_t whole = n0 / HFX_PLAN_WGS * HFX_PLAN_WGS;
    if (whole >= HFX_PLAN_WGS && n0 > whole && n0 < (int64_t)kFitRounds * HFX_PLAN_WGS) {
      double lo = cap_prefill_ns, hi = 1.5 * cap_prefill_ns;   // count(lo) > whole; is count(hi) <= whole?
      if (count_items(hi) <= whole) {
        for (int it = 0; it < 12; ++it) {
          const double mid = 0.5 * (lo + hi);
          (count_items(mid) <= whole ? hi : lo) = mid;
        }
        cap_prefill_ns = hi;
      }
    }
  }

  int64_t rows = 0;
  std::vector<int32_t>& split_cost = P.split_cost;
  int64_t pre_ord = 0;              // prefill requests seen so far
  for (int r = 0; r < R; ++r) {
    const HfxReq& q = P.reqs[(size_t)r];
    if (q.kind == HFX_DECODE) {
      const double ns_per_token = (double)ngc * D * 4.0 / kDecodeBytesPerNs;
      int64_t L = (int64_t)(cap_ns / ns_per_token);
      L = std::max<int64_t>(L, kMinDecodeTokens);
      L = std::max<int64_t>(L, ((int64_t)q.ctx_len + kMaxSplits - 1) / kMaxSplits);
      int64_t pages_per = (L + HFX_PAGE - 1) / HFX_PAGE;
      pages_per += pages_per & 1;                     // page pairs stay aligned across splits
      int nsplit = (int)((q.n_pages + pages_per - 1) / pages_per);
      // even out the pieces
      pages_per = (q.n_pages + nsplit - 1) / nsplit;
      pages_per += pages_per & 1;
      nsplit = (int)((q.n_pages + pages_per - 1) / pages_per);
      HfxItem proto;                  // what all items of the request share
      std::memset(&proto, 0, sizeof proto);
      proto.type = HFX_ITEM_DECODE;
      proto.req = r;
      proto.hn = ngc;
      proto.rq = q;
      for (int g0 = 0; g0 < Hkv; g0 += ngc) {
        int group = -1;
        if (nsplit > 1) {
          group = (int)P.groups.size();
          HfxGroup gr = {nsplit, (int32_t)rows, ngc * G, HFX_ITEM_DECODE, r, g0, ngc, 0, q.q_start, q.q_len};
          P.groups.push_back(gr);
        }
        for (int s = 0; s < nsplit; ++s) {
          HfxItem it = proto;
          it.group = group;
          it.slot_row = (nsplit > 1) ? (int32_t)(rows + (int64_t)s * ngc * G) : -1;
          it.h0 = g0;
          it.kb = (int32_t)(s * pages_per);
          it.ke = (int32_t)std::min<int64_t>(q.n_pages, (int64_t)(s + 1) * pages_per);
          int64_t toks = std::min<int64_t>(q.ctx_len, (int64_t)it.ke * HFX_PAGE) - (int64_t)it.kb * HFX_PAGE;
          it.cost = clamp_cost((double)toks * ns_per_token + 2000.0);
          it.home = -1;
          P.items.push_back(it);
          P.item_unit.push_back(kNoUnit);
          P.item_frac.push_back(0.f);
        }
        if (nsplit > 1) rows += (int64_t)nsplit * ngc * G;
      }
    } else {
      const int64_t p = q.ctx_len - q.q_len;
      const int n_rt = (q.q_len + rows_wg - 1) / rows_wg;
      for (int rt = 0; rt < n_rt; ++rt) {
        const int64_t r0 = (int64_t)rt * rows_wg, r1 = std::min<int64_t>(q.q_len, r0 + rows_wg);
        const int64_t kmax = p + r1;
        int64_t nsplit, tiles_per;
        prefill_splits(p, r0, r1, D, hpw, cap_prefill_ns, &nsplit, &tiles_per);
        split_cost.resize((size_t)nsplit);
        for (int64_t s = 0; s < nsplit; ++s) {
          const int64_t kb = s * tiles_per * HFX_KEY_TILE, ke = std::min<int64_t>(kmax, (s + 1) * tiles_per * HFX_KEY_TILE);
          split_cost[(size_t)s] = clamp_cost(4.0 * D * hpw * (double)pairs_in(p, r0, r1, kb, ke) / kPrefillFlopsPerNs + 3000.0);
        }
        HfxItem proto;                // what all items of the row tile share
        std::memset(&proto, 0, sizeof proto);
        proto.type = HFX_ITEM_PREFILL;
        proto.req = r;
        proto.hn = hpw;
        proto.row0 = (int32_t)r0;
        proto.nrows = rows_wg;
        proto.rq = q;
        for (int g = 0; g < Hkv; ++g)
          for (int hb = 0; hb < G / hpw; ++hb) {
            int group = -1;
            if (nsplit > 1) {
              group = (int)P.groups.size();
              HfxGroup gr = {(int32_t)nsplit, (int32_t)rows, 4 * HFX_WAVE_ROWS, HFX_ITEM_PREFILL, r, g * G + hb * hpw, hpw, (int32_t)r0, q.q_start, q.q_len};
              P.groups.push_back(gr);
            }
            for (int64_t s = 0; s < nsplit; ++s) {
              HfxItem it = proto;
              it.group = group;
              it.slot_row = (nsplit > 1) ? (int32_t)(rows + s * 4 * HFX_WAVE_ROWS) : -1;
              it.h0 = g * G + hb * hpw;
              it.kb = (int32_t)(s * tiles_per * HFX_KEY_TILE);
              it.ke = (int32_t)std::min<int64_t>(kmax, (s + 1) * tiles_per * HFX_KEY_TILE);
              it.cost = split_cost[(size_t)s];
              it.home = -1;
              P.items.push_back(it);
              // the row tiles and head blocks that read the s-th piece of the keys of (request, kv-head)
              const int64_t unit = (pre_ord * Hkv + g) * kMaxSplits + s;
              P.item_unit.push_back(unit < (int64_t)kNoUnit ? (uint32_t)unit : kNoUnit);
              P.item_frac.push_back((float)rt / (float)n_rt);
            }
            if (nsplit > 1) rows += nsplit * 4 * HFX_WAVE_ROWS;
          }
      }
      ++pre_ord;
    }
    if (rows > 0x7fffffff / 2 || P.items.size() > 0x3fffffffu) return HFX_ERR_LEN;
  }
  P.n_partial_rows = (int32_t)rows;
  // queue order: descending cost, ties in creation order: a stable radix sort (11-bit digits) of
  // (inverted cost, index) keys, then one permutation of the item records.
  {
    const size_t n = P.items.size();
    std::vector<uint64_t>& key = P.sort_keys;
    key.resize(2 * n);
    uint64_t* a = key.data();
    uint64_t* b = a + n;
    // keys count down from the largest cost, so that the number of digit passes follows the range
    // of costs in the step and not the width of the field
    uint32_t max_cost = 0;
    for (size_t i = 0; i < n; ++i) max_cost = std::max(max_cost, (uint32_t)P.items[i].cost);
    uint32_t top = 0;
    for (size_t i = 0; i < n; ++i) {
      const uint32_t inv = max_cost - (uint32_t)P.items[i].cost;
      a[i] = ((uint64_t)inv << 32) | (uint64_t)i;
      top |= inv;
    }
    for (int shift = 0; shift < 31 && (top >> shift) != 0; shift += 11) {
      uint32_t count[2048] = {0};
      for (size_t i = 0; i < n; ++i) count[(a[i] >> (32 + shift)) & 2047u]++;
      uint32_t sum = 0;
      for (int d = 0; d < 2048; ++d) {
        const uint32_t c = count[d];
        count[d] = sum;
        sum += c;
      }
      for (size_t i = 0; i < n; ++i) b[count[(a[i] >> (32 + shift)) & 2047u]++] = a[i];
      std::swap(a, b);
    }
    // the queue order is kept as a permutation; the records are put in that order when the blob is written
    std::vector<uint32_t>& order = P.order;
    order.resize(n);
    P.queue_classes = 1;
    if (dec_ns > pre_ns && pre_ns > 0.0) {
      // A step whose decode work outweighs its prefill work.  The first two items of workgroup b
      // are queue positions b and b + HFX_PLAN_WGS, and workgroups b and b + HFX_PLAN_WGS/2 share a
      // CU.  Over those two rounds the prefill items (largest first) go to the workgroups of the
      // first `pair_cus` CUs, both workgroups of a CU, and the decode items to all the others:
      // the matrix work then runs in the shadow of the memory-bound stream without sharing a
      // CU's memory path with it (a prefill workgroup next to a decode workgroup on one CU saw its
      // tiles take 2.5 times as long; measured on the Llama-8B-shaped mixed step, this layout takes
      // 6 % less time than one workgroup of each kind per CU, which in turn took 5 % less than plain
      // descending order).  pair_cus is sized so that the two rounds hold all prefill items, up to
      // half the CUs.  Behind the two rounds the kinds alternate in blocks of half the planning
      // width, decode first, each kind still in descending cost.  On prefill-dominated steps any
      // such interleave costs 2-13 %, so they keep the plain order.
      constexpr size_t kBlockItems = HFX_PLAN_WGS / 2;
      std::vector<uint32_t>& dec = P.order_dec;
      std::vector<uint32_t>& pre = P.order_pre;
      dec.clear();
      pre.clear();
      for (size_t i = 0; i < n; ++i) {
        const uint32_t idx = (uint32_t)(a[i] & 0xffffffffu);
        (P.items[idx].type == HFX_ITEM_DECODE ? dec : pre).push_back(idx);
      }
      const size_t pair_cus = std::min<size_t>((pre.size() + 3) / 4, kBlockItems / 2);
      size_t di = 0, pi = 0, o = 0;
      for (int round = 0; round < 2; ++round)
        for (size_t b = 0; b < (size_t)HFX_PLAN_WGS && o < n; ++b) {
          const bool prefill_slot = (b % kBlockItems) < pair_cus;
          if ((prefill_slot && pi < pre.size()) || di >= dec.size()) order[o++] = pre[pi++];
          else order[o++] = dec[di++];
        }
      while (di < dec.size() || pi < pre.size()) {
        for (size_t k = 0; k < kBlockItems && di < dec.size(); ++k) order[o++] = dec[di++];
        for (size_t k = 0; k < kBlockItems && pi < pre.size(); ++k) order[o++] = pre[pi++];
      }
    } else if (pre_ns > 0.0 && n >= (size_t)kClassRoundsMin * HFX_PLAN_WGS && n <= (size_t)kClassRoundsMax * HFX_PLAN_WGS &&
               pre_ord * Hkv * kMaxSplits < (int64_t)kNoUnit) {
      // A step whose prefill work outweighs its decode work.  Many prefill items read the same
      // keys: all row tiles (and q-head blocks) of one request and kv-head that hold the same
      // piece of the key range.  Call that set a unit.  The chip has HFX_QUEUE_CLASSES dies, each
      // with an L2 of its own, and workgroup b runs on die b % HFX_QUEUE_CLASSES; the kernel hands
      // queue position p to a workgroup of die p % HFX_QUEUE_CLASSES (as long as that die has work).
      // So the queue is built per class: every unit gets a home class (largest total cost first,
      // each to the class with the least cost so far), a class lists the items homed there in
      // descending cost, and the classes are interleaved position by position.  Items of a unit
      // that cost about the same then run side by side on one die and fetch their keys from
      // memory once instead of once per die and round, while the queue as a whole still goes
      // from the most to the least expensive items.  A decode item is a unit of its own.  When
      // a class runs out of items before the others, its positions are filled from the tail of
      // the class that has most left.
      const size_t n_slots = (size_t)(pre_ord * Hkv * kMaxSplits);
      std::vector<int64_t>& ucost = P.unit_cost;
      std::vector<uint32_t>& ufill = P.unit_fill;
      std::vector<uint32_t>& ustart = P.unit_start;
      std::vector<uint64_t>& ukeys = P.unit_keys;
      // A unit that would be a large share of a class's work is cut into sub-units of consecutive
      // row tiles, each at most about half of one class's share of the step, so that there is
      // something to balance with (a long prompt on one kv-head has as few units as it has splits).
      ucost.assign(n_slots, 0);
      int64_t all_cost = 0;
      for (size_t i = 0; i < n; ++i) {
        all_cost += P.items[i].cost;
        if (P.item_unit[i] != kNoUnit) ucost[P.item_unit[i]] += P.items[i].cost;
      }
      const int64_t sub_cost = std::max<int64_t>(1, all_cost / (2 * HFX_QUEUE_CLASSES));
      ufill.assign(n_slots, 0);     // sub-units of the slot
      ustart.assign(n_slots, 0);    // index of its first sub-unit
      size_t n_units = 0;
      for (size_t u = 0; u < n_slots; ++u)
        if (ucost[u] > 0) {
          ufill[u] = (uint32_t)std::min<int64_t>((ucost[u] + sub_cost - 1) / sub_cost, 4 * HFX_QUEUE_CLASSES);
          ustart[u] = (uint32_t)n_units;
          n_units += ufill[u];
        }
      // decode items (and anything else without a unit) get singleton units behind those
      for (size_t i = 0; i < n; ++i) {
        const uint32_t u = P.item_unit[i];
        if (u == kNoUnit) P.item_unit[i] = (uint32_t)n_units++;
        else P.item_unit[i] = ustart[u] + std::min<uint32_t>(ufill[u] - 1, (uint32_t)(P.item_frac[i] * (float)ufill[u]));
      }
      ucost.assign(n_units, 0);     // total cost of the unit; once it has a home, the home
      ustart.assign(n_units, 0);    // items in the unit
      for (size_t i = 0; i < n; ++i) {
        const uint32_t u = P.item_unit[i];
        ucost[u] += P.items[i].cost;
        ustart[u]++;
      }
      // home classes: units by descending total cost (36 bits of it, saturating; the low 28 bits
      // of a key hold the unit's index)
      ukeys.clear();
      const int64_t kCostTop = (1ll << 36) - 1;
      for (size_t u = 0; u < n_units; ++u)
        if (ustart[u]) ukeys.push_back(((uint64_t)(kCostTop - std::min(ucost[u], kCostTop)) << 28) | (uint64_t)u);
      std::sort(ukeys.begin(), ukeys.end());
      int64_t load[HFX_QUEUE_CLASSES] = {0};
      for (uint64_t& k : ukeys) {
        const uint32_t u = (uint32_t)(k & 0x0fffffffu);
        int home = 0;
        for (int c = 1; c < HFX_QUEUE_CLASSES; ++c)
          if (load[c] < load[home]) home = c;
        load[home] += ucost[u];
        ucost[u] = home;
      }
      // The items are in descending cost (a[]); a class's list is those of them that are homed
      // there, in that order (a stable counting sort by class into b[]).
      size_t head[HFX_QUEUE_CLASSES], tail[HFX_QUEUE_CLASSES];
      for (int c = 0; c < HFX_QUEUE_CLASSES; ++c) tail[c] = 0;
      for (size_t i = 0; i < n; ++i) {
        const uint32_t idx = (uint32_t)(a[i] & 0xffffffffu);
        const int home = (int)ucost[P.item_unit[idx]];
        P.items[idx].home = home;
        tail[home]++;
      }
      for (int c = 0, at = 0; c < HFX_QUEUE_CLASSES; ++c) {
        head[c] = (size_t)at;
        at += (int)tail[c];
        tail[c] = head[c];          // fill cursor; ends up one past the class's last item
      }
      for (size_t i = 0; i < n; ++i) b[tail[P.items[(uint32_t)(a[i] & 0xffffffffu)].home]++] = a[i];
      std::swap(a, b);
      P.queue_classes = HFX_QUEUE_CLASSES;
      for (size_t o = 0; o < n; ++o) {
        const int c = (int)(o % HFX_QUEUE_CLASSES);
        if (head[c] < tail[c]) {
          order[o] = (uint32_t)(a[head[c]++] & 0xffffffffu);
        } else {
          int from = 0;
          for (int y = 1; y < HFX_QUEUE_CLASSES; ++y)
            if (tail[y] - head[y] > tail[from] - head[from]) from = y;
          order[o] = (uint32_t)(a[--tail[from]] & 0xffffffffu);
        }
      }
    } else {
      for (size_t i = 0; i < n; ++i) order[i] = (uint32_t)(a[i] & 0xffffffffu);
    }
  }
  // merge work units: groups with many splits get 8 threads per (row, column) and one row per
  // workgroup, groups with few splits one thread per (row, column) and 8 rows per workgroup
  P.units.clear();
  for (size_t gi = 0; gi < P.groups.size(); ++gi) {
    const int rows_per_unit = P.groups[gi].nsplit > 8 ? 1 : 8;
    for (int c = 0; c * rows_per_unit < P.groups[gi].rows_per_split; ++c) {
      HfxUnit u = {(int32_t)gi, c};
      P.units.push_back(u);
    }
  }
  P.n_decode_items = P.n_prefill_items = 0;
  for (const HfxItem& it : P.items) (it.type == HFX_ITEM_DECODE ? P.n_decode_items : P.n_prefill_items)++;
  return HFX_OK;
}

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

void layout_blob(const hfx_shape* shape, const Plan& P, HfxHeader* h) {
  std::memset(h, 0, sizeof *h);
  h->magic = HFX_DESC_MAGIC;
  h->version = HFX_DESC_VERSION;
  h->num_requests = (int32_t)P.reqs.size();
  h->total_q = P.total_q;
  h->num_q_heads = shape->num_q_heads;
  h->num_kv_heads = shape->num_kv_heads;
  h->head_dim = shape->head_dim;
  h->page_size = shape->page_size;
  h->num_pages = shape->num_pages;
  h->softmax_scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / std::sqrt((float)shape->head_dim);
  h->n_items = (int32_t)P.items.size();
  h->n_decode_items = P.n_decode_items;
  h->n_prefill_items = P.n_prefill_items;
  h->n_groups = (int32_t)P.groups.size();
  h->n_partial_rows = P.n_partial_rows;
  h->n_bt = P.n_bt;
  h->n_ctrl = 16;
  h->queue_classes = (uint32_t)P.queue_classes;
  h->max_group_rows = 0;
  for (const HfxGroup& g : P.groups) h->max_group_rows = std::max(h->max_group_rows, g.rows_per_split);
  uint64_t off = align_up(sizeof(HfxHeader), 256);
  h->off_ctrl = (uint32_t)off;
  off = align_up(off + 4ull * h->n_ctrl, 64);
  h->off_req = (uint32_t)off;
  off = align_up(off + sizeof(HfxReq) * P.reqs.size(), 64);
  h->off_bt = (uint32_t)off;
  off = align_up(off + 4ull * (uint64_t)P.n_bt, 64);
  h->off_items = (uint32_t)off;
  off = align_up(off + sizeof(HfxItem) * P.items.size(), 64);
  h->off_groups = (uint32_t)off;
  off = align_up(off + sizeof(HfxGroup) * P.groups.size(), 64);
  h->off_units = (uint32_t)off;
  h->n_units = (int32_t)P.units.size();
  off = align_up(off + sizeof(HfxUnit) * P.units.size(), 64);
  h->off_runs = (uint32_t)off;
  h->n_runs = P.n_runs;
  off = align_up(off + sizeof(HfxRun) * (uint64_t)P.n_runs, 256);
  h->total_bytes = off;
  uint64_t acc_bytes = align_up((uint64_t)P.n_partial_rows * shape->head_dim * 4ull, 256);
  h->ws_off_ml = acc_bytes;
  h->workspace_bytes = P.n_partial_rows ? acc_bytes + align_up((uint64_t)P.n_partial_rows * 8ull, 256) : 0;
}

hfx_status fill_blob(const hfx_shape* shape, Plan& P, const int32_t* bt_indptr, const int32_t* bt_pages,
                     void* host_desc, size_t host_desc_bytes) {
  if (!bt_indptr || !bt_pages || !host_desc) return HFX_ERR_NULL;
  HfxHeader h;
  layout_blob(shape, P, &h);
  if (h.total_bytes > 0xffffffffull) return HFX_ERR_LEN;
  if (host_desc_bytes < h.total_bytes) return HFX_ERR_BUFSIZE;
  const int R = (int)P.reqs.size();
  if (bt_indptr[0] != 0) return HFX_ERR_PAGES;
  for (int r = 0; r < R; ++r) {
    if (bt_indptr[r + 1] < bt_indptr[r]) return HFX_ERR_PAGES;
    if ((int64_t)bt_indptr[r + 1] - bt_indptr[r] < P.reqs[(size_t)r].n_pages) return HFX_ERR_PAGES;
  }
  for (int r = 0; r < R; ++r) {
    const int32_t* src = bt_pages + bt_indptr[r];
    for (int i = 0; i < P.reqs[(size_t)r].n_pages; ++i)
      if (src[i] < 0 || src[i] >= shape->num_pages) return HFX_ERR_PAGE_ID;
  }
  char* base = (char*)host_desc;
  // every byte of the blob is written: sections by copy, the padding between them with zeros
  auto put = [base](uint64_t off, const void* src, uint64_t bytes, uint64_t next_off) {
    if (bytes) std::memcpy(base + off, src, (size_t)bytes);
    std::memset(base + off + bytes, 0, (size_t)(next_off - off - bytes));
  };
  put(0, &h, sizeof h, h.off_ctrl);
  put(h.off_ctrl, nullptr, 0, h.off_req);
  put(h.off_req, P.reqs.data(), sizeof(HfxReq) * P.reqs.size(), h.off_bt);
  int32_t* bt = (int32_t*)(base + h.off_bt);
  for (int r = 0; r < R; ++r) {
    const HfxReq& q = P.reqs[(size_t)r];
    int32_t* dst = bt + q.bt_start;
    std::memcpy(dst, bt_pages + bt_indptr[r], 4ull * (size_t)q.n_pages);
    for (int i = q.n_pages; i < q.bt_len; ++i) dst[i] = dst[q.n_pages - 1];
  }
  put(h.off_bt + 4ull * (uint64_t)P.n_bt, nullptr, 0, h.off_items);
  HfxItem* queue = (HfxItem*)(base + h.off_items);
  for (size_t i = 0; i < P.items.size(); ++i) queue[i] = P.items[P.order[i]];
  put(h.off_items + sizeof(HfxItem) * P.items.size(), nullptr, 0, h.off_groups);
  put(h.off_groups, P.groups.data(), sizeof(HfxGroup) * P.groups.size(), h.off_units);
  put(h.off_units, P.units.data(), sizeof(HfxUnit) * P.units.size(), h.off_runs);
  // append runs: each request's new tokens, cut at page boundaries
  HfxRun* run = (HfxRun*)(base + h.off_runs);
  for (int r = 0; r < R; ++r) {
    const HfxReq& q = P.reqs[(size_t)r];
    const int32_t* pages = bt_pages + bt_indptr[r];
    int32_t t = q.ctx_len - q.q_len;
    while (t < q.ctx_len) {
      const int32_t slot0 = t % HFX_PAGE;
      const int32_t n = std::min<int32_t>(HFX_PAGE - slot0, q.ctx_len - t);
      *run++ = HfxRun{q.q_start + (t - (q.ctx_len - q.q_len)), n, pages[t / HFX_PAGE], slot0};
      t += n;
    }
  }
  put(h.off_runs + sizeof(HfxRun) * (uint64_t)P.n_runs, nullptr, 0, h.total_bytes);
  return HFX_OK;
}

}  // namespace hfx
