// Device code of libhfxattn for gfx950 (MI355X): one persistent kernel that drains the
// cost-ordered work items of a scheduled step -- decode ranges (HBM-bound streaming of KV
// pages: the token-generation phase of HFX Section 2.1) and prefill tiles (dense bf16 MFMA
// contraction with a causal mask: its prompt phase) -- plus the split merge, the page gather
// hook, the KV append and the page copy.  Wavefronts are 64 lanes wide; every tiling below is
// written for that.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "hfx_desc.h"
#include "hfx_launch.h"

namespace hfx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define NEG_INF (-__builtin_inff())

struct KArgs {
  const char* desc;      // device descriptor blob (read-only here; the control words go through `ctrl`)
  const __bf16* q;       // [T][Hq][D]
  const __bf16* pool;    // [pages][Hkv][2][16*D]
  float* ws;             // split partials
  __bf16* out;           // [T][Hq][D]
};

template <int D>
struct Smem {
  // prefill: two stage buffers of 32 keys (two pages) each, the halves of a 64-key tile.  A stage holds the keys in
  // operand order ([D/16][2 dimension halves][32 keys][8 dims], 1 KB per 16-dimension group) followed by
  // the two pages' V blocks as they lie in the pool ([D dims][16 slots] each).
  static constexpr int kKBytes = HFX_STAGE_KEYS * D * 2;
  static constexpr int kPageVBytes = HFX_PAGE * D * 2;
  static constexpr int kStageBytes = kKBytes + 2 * kPageVBytes;
  static constexpr int kStages = 2;
  static constexpr int kCopies = D / 32;         // 16-byte pieces per lane that a wavefront moves per stage
  // decode: per-wavefront partial rows [4][16][D + 4] floats (same memory; an item is one or the other)
  static constexpr int kPartStride = D + 4;
  static constexpr int kPartBytes = 4 * 16 * kPartStride * 4;
  static constexpr int kBytes = kStages * kStageBytes > kPartBytes ? kStages * kStageBytes : kPartBytes;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ bf16x8 ld16(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }

// `x` where keep, -inf elsewhere, as a select on the bit pattern: the scores of masked keys may be
// NaN (unused slots hold anything), and the file is compiled with -fno-honor-nans, under which a
// floating-point select of a NaN is not defined.
__device__ __forceinline__ float keep_or_neg_inf(float x, bool keep) {
  const unsigned u = keep ? __builtin_bit_cast(unsigned, x) : 0xff800000u;
  return __builtin_bit_cast(float, u);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Exchange between lane n and lane n ^ 32 with the swap instruction gfx950 has for it (the upper half
// of one register against the lower half of another); a shuffle would go through LDS and put
// its latency, and a wait for every LDS read in flight, into the softmax of every stage.
// swap32(x): {x of the lower-half lane of the pair, x of its upper-half lane}, in both lanes.
// The copies in and out are hidden from the optimizer, which otherwise folds the swap of a value
// with itself, and whatever combines its two results, into the value.
struct Pair32 {
  float lo, hi;
};
__device__ __forceinline__ Pair32 swap32(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  unsigned u2 = u;
  asm volatile("" : "+v"(u2));
  const auto r = __builtin_amdgcn_permlane32_swap(u, u2, false, false);
  unsigned a = r[0], b = r[1];
  asm volatile("" : "+v"(a), "+v"(b));
  Pair32 p;
  p.lo = __builtin_bit_cast(float, a);
  p.hi = __builtin_bit_cast(float, b);
  return p;
}
__device__ __forceinline__ float max_xor32(float x) {
  const Pair32 p = swap32(x);
  return fmaxf(p.lo, p.hi);
}
__device__ __forceinline__ float sum_xor32(float x) {
  const Pair32 p = swap32(x);
  return p.lo + p.hi;
}

// zero the elements e >= nv of an 8-element bf16 vector (nv may be <= 0 or >= 8)
__device__ __forceinline__ bf16x8 keep_first(bf16x8 v, int nv) {
  u32x4 u = __builtin_bit_cast(u32x4, v);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    uint32_t m = (2 * w < nv ? 0x0000ffffu : 0u) | (2 * w + 1 < nv ? 0xffff0000u : 0u);
    u[w] &= m;
  }
  return __builtin_bit_cast(bf16x8, u);
}

// ----------------------------------------------------------------------------------------------
// Split merge (runs as its own small launch after the persistent kernel, so the partials are
// ordered by the kernel boundary and no fences or arrival counters are needed).  One workgroup
// per merge unit combines a few rows of a group's partials (m, l, acc):
//   m* = max m_s,  l* = sum l_s 2^(m_s - m*),  out = sum acc_s 2^(m_s - m*) / l*
// (m is kept in the base-2 domain throughout), rounds to bf16 and stores.  A thread owns one
// float4 column of a row; for groups with many splits 8 threads share the splits of that column
// (one row per workgroup) so that all loads are in flight together, for groups with at most 8
// splits one thread takes them all (8 rows per workgroup).
// ----------------------------------------------------------------------------------------------
// The body of the merge for a group whose threads see at most N splits each.
template <int D, int N>
__device__ __forceinline__ void merge_rows(const HfxUnit& un, const HfxGroup& gr, const float* __restrict__ ws, const float* __restrict__ ml,
                                           int Hq, int G, __bf16* __restrict__ out, float* s_max, float* s_l,
                                           f32x4 (*s_acc)[D / 4]) {
  constexpr int C4 = D / 4;                       // float4 columns of a row
  const int tid = threadIdx.x;
  const int col = tid % C4, q = tid / C4;
  const bool wide = N == 8 && gr.nsplit > 8;      // only the first 8 thread rows are used below
  const int SL = wide ? 8 : 1;                    // threads sharing one row's splits
  const int sl = wide ? q : 0;
  const int row = wide ? un.chunk : un.chunk * 8 + q;
  const bool row_ok = q < 8 && row < gr.rows_per_split;
  const int rows = gr.rows_per_split, ns = gr.nsplit, base = gr.base_row;
  // All loads are issued without lane predicates (a thread without a split in a slot, or outside
  // the group's rows, reads a neighbour's partial and gives it weight 0): under per-lane
  // conditions the compiler waits for each slot's loads before it asks for the next.
  const int row_c = row < rows ? row : rows - 1;
  float mv[N], lv[N];
  f32x4 av[N];
  bool ok[N];
#pragma unroll
  for (int i = 0; i < N; ++i) {                   // the planner never makes more than 64 splits
    const int s = sl + i * SL;
    ok[i] = row_ok && s < ns;
    const long pr = (long)base + (long)(s < ns ? s : ns - 1) * rows + row_c;
    const float2 t = *reinterpret_cast<const float2*>(ml + pr * 2);
    mv[i] = t.x;
    lv[i] = t.y;
    av[i] = *reinterpret_cast<const f32x4*>(ws + pr * D + col * 4);
  }
  float mloc = NEG_INF;
#pragma unroll
  for (int i = 0; i < N; ++i) mloc = fmaxf(mloc, ok[i] ? mv[i] : NEG_INF);
  float mm = mloc;
  if (wide) {
    if (col == 0) s_max[q] = mloc;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) mm = fmaxf(mm, s_max[i]);
  }
  float ll = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float w = ok[i] ? fast_exp2(mv[i] - mm) : 0.f;
    ll += lv[i] * w;
    o += av[i] * w;
  }
  if (wide) {
    s_acc[q][col] = o;
    if (col == 0) s_l[q] = ll;
    __syncthreads();
    if (q != 0) return;
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      o += s_acc[i][col];
      ll += s_l[i];
    }
  }
  if (!row_ok) return;
  long orow;
  if (gr.type == HFX_ITEM_DECODE) {
    orow = (long)gr.q_start * Hq + gr.h0 * G + row;
  } else {
    const int w = row / HFX_WAVE_ROWS, nn = row % HFX_WAVE_ROWS;
    const int head = gr.h0 + w % gr.hn;
    const int qrow = gr.row0 + (w / gr.hn) * HFX_WAVE_ROWS + nn;
    if (qrow >= gr.q_len) return;
    orow = ((long)gr.q_start + qrow) * Hq + head;
  }
  const float inv = 1.0f / ll;
  bf16x4 ob;
#pragma unroll
  for (int e = 0; e < 4; ++e) ob[e] = (__bf16)(o[e] * inv);
  *reinterpret_cast<bf16x4*>(out + orow * D + col * 4) = ob;
}

template <int D>
__global__ __launch_bounds__(HFX_WG_THREADS) void merge_kernel(const HfxUnit* __restrict__ units,
                                                               const HfxGroup* __restrict__ groups,
                                                               const float* __restrict__ ws,
                                                               const float* __restrict__ ml, int Hq, int G,
                                                               __bf16* __restrict__ out) {
  constexpr int Q = HFX_WG_THREADS / (D / 4);     // threads per column: 8 (D = 128) or 16 (D = 64)
  __shared__ float s_max[Q];
  __shared__ float s_l[Q];
  __shared__ f32x4 s_acc[Q][D / 4];
  // Everything the launch can know on the host comes in as an argument: unit -> group -> partials
  // is the whole chain of dependent loads, and the (m, l) pairs and the accumulator rows of all
  // splits are asked for together.  One copy of the body per number of slots, so that a group of
  // two splits does not pay for eight.  (A unit record that carried a copy of its group saved one
  // trip, about a microsecond, and cost the host ten to write and upload.)
  const HfxUnit un = units[blockIdx.x];
  const HfxGroup gr = groups[un.group];
  const int ns = gr.nsplit;
  if (ns <= 2) merge_rows<D, 2>(un, gr, ws, ml, Hq, G, out, s_max, s_l, s_acc);
  else if (ns <= 4) merge_rows<D, 4>(un, gr, ws, ml, Hq, G, out, s_max, s_l, s_acc);
  else merge_rows<D, 8>(un, gr, ws, ml, Hq, G, out, s_max, s_l, s_acc);
}

// ----------------------------------------------------------------------------------------------
// Decode item.  One wavefront per kv-head (hn of them), the other 4/hn wavefronts of the
// workgroup interleave over page pairs.  Per pair (32 tokens) and kv-head a wavefront issues
// 16 coalesced 16-byte loads per lane and 16 MFMA 16x16x32:
//   S^T[token][head] = K[token][:] . Q[head][:]      (A = K rows, B = Q^T)
//   O^T[d][head]    += V^T[d][token] . P^T[token][head]   (A = V^T rows, B = P^T)
// The two 16-token score tiles take their rows from the page pair such that, in the MFMA
// result layout, each lane ends up holding 8 consecutive tokens of one page -- exactly the
// 16 bytes of a dimension-major V row that the second contraction needs, with no shuffles.
// ----------------------------------------------------------------------------------------------
// Work-queue tickets of a workgroup.  It holds the item it is processing and the item after it
// (whose record is therefore known while the current item runs, so that a prefill item can
// request the first tiles of its successor before it ends).  The ticket after those is asked
// for by thread 0 shortly before the current item ends, published through LDS ahead of a
// barrier the item crosses anyway, and taken at the hand-over.  Asking late matters: a
// workgroup that asks at the start of a long item reserves work it will not touch for a long
// time, and in a step with about three items per workgroup that left half the chip idle while
// the other half worked through its reservations.  The first two tickets of a workgroup are its
// index plus 0 and 1 grids (the queue is in descending cost, so this deals the largest items
// out evenly, and a workgroup starts without a round trip to a counter).
constexpr int kDealtTickets = 2;
struct Tickets {
  int cur, nxt;
  int pending;   // meaningful in thread 0 only: the counter's reply, an offset from the dealt tickets
  int parity;
};

// Queue positions past the dealt ones fall into `nc` classes (1 or HFX_QUEUE_CLASSES, the
// planner's choice per step), position p into class p % nc, each with a counter of its own, and a
// workgroup asks the counter of the class of its index.  Workgroups are placed on the chip's dies
// round-robin by index, so with HFX_QUEUE_CLASSES classes a class is served by the workgroups of
// one die, and the planner puts items that read the same keys into one class: they then share
// that die's L2.
//
// Thread 0 asks its class's counter for one more ticket (when `ask`); the reply is first touched by
// tickets_publish.  The other lanes, and a call with ask == false, set the field to zero rather
// than keep what it held: keeping it reads the register the previous request wrote, and for that
// the compiler puts a wait for everything in flight in front of this request.
__device__ __forceinline__ void tickets_reserve(Tickets& t, int* ctrl, int nc, bool ask = true) {
  int r = 0;
  if (ask && threadIdx.x == 0) r = atomicAdd(ctrl + ((int)blockIdx.x & (nc - 1)), 1);
  t.pending = r;
}
// Thread 0 puts the reserved ticket into LDS (two slots alternate, so one barrier per hand-over is
// enough).  A reply past the end of the queue means the workgroup's class is empty.  It then reads
// all counters (one round trip) and asks the class that has most positions left for one, so
// that a die that finishes early helps the others; when other workgroups got there first (the
// reply is past the end again) it looks again, a few times.  Giving up early costs balance, not
// correctness: every class is drained by its own workgroups whether or not others help.
constexpr int kStealAttempts = 4;
__device__ __forceinline__ void tickets_publish(const Tickets& t, int* s_tk, int* ctrl, int n_items, int nc) {
  if (threadIdx.x == 0) {
    const int base = kDealtTickets * (int)gridDim.x;
    int pos = base + t.pending * nc + ((int)blockIdx.x & (nc - 1));
    if (nc > 1) {
      for (int attempt = 0; attempt < kStealAttempts && pos >= n_items; ++attempt) {
        int best = 0, best_left = 0;
        for (int k = 0; k < HFX_QUEUE_CLASSES; ++k) {
          const int taken = __hip_atomic_load(ctrl + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          // positions base + r * classes + k below n_items with r >= taken
          const int left = (n_items - base - k + HFX_QUEUE_CLASSES - 1) / HFX_QUEUE_CLASSES - taken;
          if (left > best_left) {
            best_left = left;
            best = k;
          }
        }
        if (best_left <= 0) break;
        pos = base + atomicAdd(ctrl + best, 1) * HFX_QUEUE_CLASSES + best;
      }
    }
    s_tk[t.parity] = pos;
  }
}
// ... after a workgroup barrier that follows tickets_publish
__device__ __forceinline__ void tickets_take(Tickets& t, int* s_tk) {
  t.cur = t.nxt;
  t.nxt = uniform(s_tk[t.parity]);
  t.parity ^= 1;
}

template <int D>
struct PairRegs {
  bf16x8 ka[D / 32], kb[D / 32], v[D / 16];
};

template <int D>
__device__ __forceinline__ void decode_load(PairRegs<D>& r, const __bf16* pool, int pg0, int pg1, int Hkv, int g,
                                            int k_sel, int k_off, int v_sel, int v_off) {
  constexpr long kBlock = 16 * D;
  const __bf16* kp = pool + (((long)(k_sel ? pg1 : pg0) * Hkv + g) * 2) * kBlock + k_off;
  const __bf16* vp = pool + (((long)(v_sel ? pg1 : pg0) * Hkv + g) * 2 + 1) * kBlock + v_off;
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) {   // 32 dimensions = two 16-dimension groups of 256 elements each
    r.ka[kk] = ld16(kp + kk * 512);
    r.kb[kk] = ld16(kp + kk * 512 + 4 * 16);
  }
#pragma unroll
  for (int b = 0; b < D / 16; ++b) r.v[b] = ld16(vp + b * 256);
}

template <int D>
__device__ __forceinline__ void decode_compute(PairRegs<D>& r, const bf16x8* qf, f32x4* o, float& m, float& l,
                                               float sl2, int nv) {
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.ka[kk], qf[kk], sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.kb[kk], qf[kk], sb, 0, 0, 0);
  }
  float s[8];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s[e] = sa[e] * sl2;
    s[4 + e] = sb[e] * sl2;
  }
  if (nv < 8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = keep_or_neg_inf(s[e], e < nv);
  }
  float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float mn = fmaxf(m, mx);
  const float alpha = fast_exp2(m - mn);
  float ps = 0.f;
  bf16x8 pb;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float p = fast_exp2(s[e] - mn);
    ps += p;
    pb[e] = (__bf16)p;
  }
  l = l * alpha + ps;
  m = mn;
#pragma unroll
  for (int b = 0; b < D / 16; ++b) {
    o[b] *= alpha;
    const bf16x8 vv = (nv < 8) ? keep_first(r.v[b], nv) : r.v[b];
    o[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, pb, o[b], 0, 0, 0);
  }
}

// What a wavefront derives from a decode item: its kv-head, its share of the page pairs, and the
// pages of its first two pairs.
struct DecodeWave {
  int g;          // kv-head
  int step;       // pages between two pairs of this wavefront
  int pp, pe;     // next page (pair-aligned) and end of the item's page range
  int tend;       // tokens of the context that the item may see (end of its range or of the context)
  int bt0, last_page;
  int a0, a1, b0, b1;   // page ids of the pair at pp and of the one after it
};

__device__ __forceinline__ int decode_page(const int* __restrict__ bt, const DecodeWave& d, int i) {
  return bt[d.bt0 + (i < d.last_page ? i : d.last_page)];
}

__device__ __forceinline__ DecodeWave decode_wave(const int* __restrict__ bt, const HfxItem& it, int wave) {
  DecodeWave d;
  const int HW = it.hn, TW = 4 / HW;
  d.g = it.h0 + wave % HW;
  d.step = 2 * TW;
  d.pp = it.kb + 2 * (wave / HW);
  d.pe = it.ke;
  d.tend = min(it.ke * HFX_PAGE, it.rq.ctx_len);
  d.bt0 = it.rq.bt_start;
  d.last_page = it.rq.n_pages - 1;
  d.a0 = decode_page(bt, d, d.pp);
  d.a1 = decode_page(bt, d, d.pp + 1);
  d.b0 = decode_page(bt, d, d.pp + d.step);
  d.b1 = decode_page(bt, d, d.pp + d.step + 1);
  return d;
}

// Runs the decode item t.cur and carries on for as long as the workgroup's next item is a decode
// item too: the first KV pair of the next item is requested before the current item's partial
// results are combined and stored, so the KV stream of a workgroup does not stop between items.
// Returns with t.cur at the first item it did not process.
template <int D>
__device__ void decode_run(const KArgs& a, const HfxHeader* H, const HfxItem* __restrict__ items, int n_items,
                           Tickets& t, int* s_tk, int* ctrl, char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int Hq = H->num_q_heads, Hkv = H->num_kv_heads;
  const int G = Hq / Hkv;
  const int n = lane & 15, j = lane >> 4;
  const float sl2 = H->softmax_scale * 1.4426950408889634f;
  const int* bt = reinterpret_cast<const int*>(a.desc + H->off_bt);
  // K rows of the two score tiles: row rho of tile A is (page rho>>3, token ((rho>>2)&1)*8 + (rho&3)),
  // tile B the same + 4 tokens.  V: lane group j reads tokens (j&1)*8.. of page j>>1 for row d = 16b + n.
  const int k_sel = n >> 3;
  const int k_off = (j >> 1) * 256 + (((n >> 2) & 1) * 8 + (n & 3)) * 16 + (j & 1) * 8;
  const int v_sel = j >> 1;
  const int v_off = n * 16 + (j & 1) * 8;
  const int tok_lane = (j >> 1) * 16 + (j & 1) * 8;   // first of this lane's 8 tokens inside the pair

  HfxItem it = items[t.cur];
  DecodeWave d = decode_wave(bt, it, wave);
  PairRegs<D> r0, r1;
  if (d.pp < d.pe) decode_load<D>(r0, a.pool, d.a0, d.a1, Hkv, d.g, k_sel, k_off, v_sel, v_off);
  bf16x8 qf[D / 32];
  auto q_load = [&](const HfxItem& item, int g) {
    const int hh = n < G ? n : G - 1;
    const __bf16* qrow = a.q + ((long)item.rq.q_start * Hq + g * G + hh) * D + j * 8;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      bf16x8 tq = ld16(qrow + kk * 32);
      qf[kk] = keep_first(tq, n < G ? 8 : 0);
    }
  };
  q_load(it, d.g);

  for (;;) {
    // the record of the next item and, if it is a decode item, this wavefront's share of it
    const HfxItem nx = items[t.nxt < n_items ? t.nxt : t.cur];
    const bool carry_on = t.nxt < n_items && nx.type == HFX_ITEM_DECODE;
    const DecodeWave dn = decode_wave(bt, nx, wave);

    f32x4 o[D / 16];
#pragma unroll
    for (int b = 0; b < D / 16; ++b) o[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, l = 0.f;
    const int step = d.step, pe = d.pe, tend = d.tend, g = d.g;
    int pp = d.pp;
    int a0 = d.a0, a1 = d.a1, b0 = d.b0, b1 = d.b1;
    bool reserved = false;
    // page ids are fetched one pair ahead of the KV loads that need them
    while (pp < pe) {
      if (!reserved && pp + 4 * step >= pe) {   // a few pairs before the end (thread 0 sits in the first wavefront, which always has pairs)
        tickets_reserve(t, ctrl, (int)H->queue_classes);
        reserved = true;
      }
      if (pp + step < pe) decode_load<D>(r1, a.pool, b0, b1, Hkv, g, k_sel, k_off, v_sel, v_off);
      if (pp + 2 * step < pe) {
        a0 = decode_page(bt, d, pp + 2 * step);
        a1 = decode_page(bt, d, pp + 2 * step + 1);
      }
      {
        const int nv = tend - (pp * HFX_PAGE + tok_lane);
        if ((pp + 2) * HFX_PAGE <= tend) decode_compute<D>(r0, qf, o, m, l, sl2, 8);
        else decode_compute<D>(r0, qf, o, m, l, sl2, nv);
      }
      pp += step;
      if (pp >= pe) break;
      if (pp + step < pe) decode_load<D>(r0, a.pool, a0, a1, Hkv, g, k_sel, k_off, v_sel, v_off);
      if (pp + 2 * step < pe) {
        b0 = decode_page(bt, d, pp + 2 * step);
        b1 = decode_page(bt, d, pp + 2 * step + 1);
      }
      {
        const int nv = tend - (pp * HFX_PAGE + tok_lane);
        if ((pp + 2) * HFX_PAGE <= tend) decode_compute<D>(r1, qf, o, m, l, sl2, 8);
        else decode_compute<D>(r1, qf, o, m, l, sl2, nv);
      }
      pp += step;
    }
    // The reply to the ticket request has come back in front of the last pairs' loads (returns
    // are in order), so publishing it here waits for nothing; after the requests below it would
    // wait for them.  The barriers of the epilogue stand between this write and its readers.
    tickets_publish(t, s_tk, ctrl, n_items, (int)H->queue_classes);
    // both register sets and the Q operand are free now: start on the next item
    if (carry_on) {
      if (dn.pp < dn.pe) decode_load<D>(r0, a.pool, dn.a0, dn.a1, Hkv, dn.g, k_sel, k_off, v_sel, v_off);
      q_load(nx, dn.g);
    }
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);

    // wavefront partial -> LDS: part[wave][head n][D + 4]; o[b][v] is dimension 16b + 4j + v
    constexpr int PS = Smem<D>::kPartStride;
    float* part = reinterpret_cast<float*>(smem);
    if (n < G) {
      float* dst = part + ((wave * 16 + n) * PS);
#pragma unroll
      for (int b = 0; b < D / 16; ++b) *reinterpret_cast<f32x4*>(dst + b * 16 + 4 * j) = o[b];
      if (j == 0) {
        dst[D] = m;
        dst[D + 1] = l;
      }
    }
    __syncthreads();

    // combine the TW token partitions of each head; row = hwi * G + hh
    const int HW = it.hn, TW = 4 / HW;
    const int rows = HW * G;
    float* ws_acc = a.ws;
    float* ws_ml = reinterpret_cast<float*>(reinterpret_cast<char*>(a.ws) + H->ws_off_ml);
    constexpr int C4 = D / 4;
    for (int idx = tid; idx < rows * C4; idx += HFX_WG_THREADS) {
      const int row = idx / C4, d4 = (idx % C4) * 4;
      const int hwi = row / G, hh = row % G;
      float mm = NEG_INF;
      for (int tt = 0; tt < TW; ++tt) mm = fmaxf(mm, part[((tt * HW + hwi) * 16 + hh) * PS + D]);
      float ll = 0.f;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      for (int tt = 0; tt < TW; ++tt) {
        const float* src = part + ((tt * HW + hwi) * 16 + hh) * PS;
        const float wgt = fast_exp2(src[D] - mm);
        ll += src[D + 1] * wgt;
        acc += *reinterpret_cast<const f32x4*>(src + d4) * wgt;
      }
      if (it.group < 0) {
        const float inv = 1.0f / ll;
        bf16x4 ob;
#pragma unroll
        for (int e = 0; e < 4; ++e) ob[e] = (__bf16)(acc[e] * inv);
        *reinterpret_cast<bf16x4*>(a.out + ((long)it.rq.q_start * Hq + it.h0 * G + row) * D + d4) = ob;
      } else {
        const long pr = (long)it.slot_row + row;
        *reinterpret_cast<f32x4*>(ws_acc + pr * D + d4) = acc;
        if (d4 == 0) {
          ws_ml[pr * 2] = mm;
          ws_ml[pr * 2 + 1] = ll;
        }
      }
    }
    __syncthreads();                  // frees the LDS partials; the ticket was published before the one above
    tickets_take(t, s_tk);
    if (!carry_on) break;
    it = nx;
    d = dn;
  }
}

// ----------------------------------------------------------------------------------------------
// Prefill item.  Four wavefronts, each owning 32 chunk rows of one q-head; all four share the
// kv-head.  Both contractions take their streamed operand from LDS, which on CDNA4 delivers 16-byte
// reads at about 256 bytes per clock and CU, four times what the vector-memory path gives a wavefront
// (about 64 bytes per clock and CU, measured): with 32 rows per wavefront every MFMA 32x32x16 needs a
// fresh 1 KB operand, 128 bytes per clock and CU at full matrix rate.
//   S^T[key][row]  = K[key][:] . Q[row][:]        A = K rows out of the stage buffer, B = Q^T in registers;
//   O^T[d][row]   += V^T[d][key] . P^T[key][row]  A = V^T rows out of the stage buffer (a dimension-major
//                                                 V block is the operand layout), B = P^T from the
//                                                 score registers.
// The workgroup fills a stage (32 keys: two pages' K and V blocks, 16 KB at D = 128) once with
// direct-to-LDS loads, two stages ahead of the one being multiplied; the global-to-LDS traffic is a
// quarter of what four wavefronts loading their own fragments would move.
// Each lane owns one query row (a column of S^T and O^T), so the running maximum, sum and rescale
// are lane-local up to one exchange with lane ^ 32.  The K rows of a score tile are taken in the
// order that leaves every lane with 8 consecutive keys of one page per 16-key MFMA step.
// ----------------------------------------------------------------------------------------------
struct StagePages {     // the two pages of a 32-key stage
  int pg0, pg1;
};

// What a lane contributes to every stage copy; fixed for the lifetime of the kernel.  Wavefronts 0
// and 1 copy the keys (D/32 groups of 16 dimensions each: 1 KB per instruction, the 32-byte pieces of
// 32 keys, lanes 16-31 and 48-63 taking the second page), wavefronts 2 and 3 copy the V block of the
// first and of the second page (1 KB per instruction, as it lies).
struct CopyLane {
  unsigned src_off;    // byte offset of the lane's first piece inside the (page, kv-head) K|V block pair
  unsigned lds_off;    // where the lane's pieces start inside a stage buffer
  bool second;         // the lane reads the stage's second page
};

template <int D>
__device__ __forceinline__ CopyLane copy_lane(int wave, int lane) {
  CopyLane c;
  if (wave < 2) {
    const int kk0 = wave * Smem<D>::kCopies;
    // lane l fills LDS slot l of a 1 KB group: slot = 32 * (dimension half) + key, so that the 16
    // lanes the LDS serves together later read 16 different bank groups
    c.src_off = (unsigned)(((kk0 * 16 + (lane & 15)) * 16 + (lane >> 5) * 8) * 2);
    c.lds_off = (unsigned)(kk0 * 1024 + lane * 16);
    c.second = (lane >> 4) & 1;
  } else {
    c.src_off = (unsigned)(HFX_PAGE * D * 2 + lane * 16);
    // A lane holds one half (8 slots, 16 bytes) of one dimension's 32-byte V row; the halves of rows
    // 8-15 and 24-31 of a 1 KB group change places in LDS, so that the 16 lanes the LDS serves together
    // hit 16 different bank groups both when the pieces are written (8 rows, both halves) and when the
    // MFMA fragments are read (16 rows, one half); laid out as in the pool the reads collide in pairs.
    const int row = lane >> 1, half = lane & 1;
    c.lds_off = (unsigned)(Smem<D>::kKBytes + (wave - 2) * Smem<D>::kPageVBytes + (2 * row + (half ^ ((row >> 3) & 1))) * 16);
    c.second = wave == 3;
  }
  return c;
}

// A wavefront's share of one 32-key stage on its way from the pool to LDS: D/32 pieces of 16 bytes per lane.
template <int D>
struct StageRegs {
  u32x4 r[Smem<D>::kCopies];
};

// Requests this wavefront's pieces of the stage made of pages pg0, pg1 of kv-head g.
template <int D>
__device__ __forceinline__ void stage_load(StageRegs<D>& sr, const __bf16* pool, const StagePages& sp, int Hkv, int g,
                                           const CopyLane& cl, int wave) {
  constexpr long kPairBytes = 2L * HFX_PAGE * D * 2;   // K block + V block of one (page, kv-head)
  // the block addresses of the two pages are formed in scalar registers; a lane only picks its page
  const uintptr_t b0 = reinterpret_cast<uintptr_t>(pool) + ((long)sp.pg0 * Hkv + g) * kPairBytes;
  const uintptr_t b1 = reinterpret_cast<uintptr_t>(pool) + ((long)sp.pg1 * Hkv + g) * kPairBytes;
  // (an address formed from integers has to be told that it is a global one, or the loads come out as flat loads)
  typedef const __attribute__((address_space(1))) char* gptr;
  gptr src = reinterpret_cast<gptr>((cl.second ? b1 : b0) + cl.src_off);
  const int step = wave < 2 ? 512 : 1024;   // keys: the next 16-dimension group is 512 bytes on in the page; values: 1 KB
#pragma unroll
  for (int i = 0; i < Smem<D>::kCopies; ++i)
    sr.r[i] = *reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(src + i * step);
}

// ... and puts them into the stage buffer `buf` (1 KB per instruction, lane l at 16 l).
template <int D>
__device__ __forceinline__ void stage_write(char* buf, const StageRegs<D>& sr, const CopyLane& cl, int lane) {
  char* dst = buf + cl.lds_off;
#pragma unroll
  for (int i = 0; i < Smem<D>::kCopies; ++i) *reinterpret_cast<u32x4*>(dst + i * 1024) = sr.r[i];
}

// Per-wavefront state of a prefill item that lives across key tiles.
template <int D>
struct PrefillWave {
  f32x16 o[D / 32];        // O^T accumulators per 32-dimension block
  bf16x8 qf[D / 16];       // Q^T operand fragments
  float m, l;              // reference exponent (base-2 domain) and running sum
  int pos;                 // last key this lane's row may see
};

// Softmax of 32 scores (one MFMA result tile) of this lane's row.  `m` is the reference exponent
// of the running sums; it is only raised -- and O, l rescaled -- when some row's maximum has
// grown by more than 2^8 over it, which keeps every weight below 2^8 and makes the rescale rare.
// s[v] is key key0 + (v>>3)*16 + (v&7)   (key0 already includes the lane's 8j).
template <int D>
__device__ __forceinline__ void softmax_block(f32x16& s, PrefillWave<D>& w, bf16x8* pb, float sl2, bool masked,
                                              int key0) {
  if (masked) {                // wave-uniform; the empty asm keeps the compiler from turning the rare
    asm volatile("" ::: );     // masking into selects executed on every tile
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = key0 + (v >> 3) * 16 + (v & 7);
      s[v] = keep_or_neg_inf(s[v], key <= w.pos);
    }
  }
  float mx = fmaxf(s[0], s[1]);
#pragma unroll
  for (int v = 2; v < 16; v += 2) mx = fmaxf(fmaxf(mx, s[v]), s[v + 1]);   // v_max3_f32
  mx = max_xor32(mx) * sl2;
  if (__any(mx > w.m + 8.0f)) {
    const float mn = fmaxf(w.m, mx);
    const float alpha = fast_exp2(w.m - (mn == NEG_INF ? 0.f : mn));
    w.l *= alpha;
#pragma unroll
    for (int b = 0; b < D / 32; ++b) w.o[b] *= alpha;
    w.m = mn;
  }
  const float mneg = w.m == NEG_INF ? 0.f : -w.m;
  // The weights are summed in fp32 with plain adds, four partial sums.  (The two-element dot-product
  // instruction would sum the rounded weights in half as many instructions, but it does not issue
  // while a matrix instruction executes -- measured: 28 of them interleaved with 4 MFMA 32x32x16
  // take the sum of both times, every other instruction of this function the maximum -- and so
  // serialises the softmax of one wavefront with the MFMAs of both wavefronts of its SIMD.)
  float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int v = 0; v < 16; v += 2) {
    const float p0 = fast_exp2(__builtin_fmaf(s[v], sl2, mneg));
    const float p1 = fast_exp2(__builtin_fmaf(s[v + 1], sl2, mneg));
    ps[(v >> 1) & 3] += p0 + p1;
    pb[v >> 3][v & 7] = (__bf16)p0;
    pb[v >> 3][(v & 7) + 1] = (__bf16)p1;
  }
  w.l += (ps[0] + ps[1]) + (ps[2] + ps[3]);
}

// One 32-key stage out of the LDS buffer `buf` against the wavefront's 32 rows; key0 is the stage's
// first key.  k_lane / v_lane: byte offsets of this lane's K row and V^T fragment inside the buffer.
template <int D>
__device__ __forceinline__ void prefill_stage(PrefillWave<D>& w, const char* buf, int k_lane, int v_lane, bool masked,
                                              bool past_ctx, int key0, int ctx_len, int j, float sl2, char* fill,
                                              const StageRegs<D>& sr, const CopyLane& cl, int lane) {
  bf16x8 kf[D / 16];
  bf16x8 vf[2][D / 32];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(buf + kk * 1024 + k_lane);
#pragma unroll
  for (int sp = 0; sp < 2; ++sp)
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
      vf[sp][b] = *reinterpret_cast<const bf16x8*>(buf + Smem<D>::kKBytes + sp * Smem<D>::kPageVBytes + b * 1024 + v_lane);
  // keep all the reads in front of the MFMA chain that consumes them: left alone, the scheduler
  // sinks each read next to its MFMA to save registers and exposes the LDS latency every time
  __builtin_amdgcn_sched_barrier(0);
  f32x16 s;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    if (kk == 0) {
      f32x16 z;
#pragma unroll
      for (int v = 0; v < 16; ++v) z[v] = 0.f;
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], w.qf[kk], z, 0, 0, 0);
    } else {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], w.qf[kk], s, 0, 0, 0);
    }
  }
  // the pieces of the stage after next go to the other buffer while the score MFMAs run
  stage_write<D>(fill, sr, cl, lane);
  __builtin_amdgcn_sched_barrier(0);
  if (past_ctx) {              // the stage runs past the context: unused V slots may hold anything
    asm volatile("" ::: );
#pragma unroll
    for (int sp = 0; sp < 2; ++sp)
#pragma unroll
      for (int b = 0; b < D / 32; ++b) vf[sp][b] = keep_first(vf[sp][b], ctx_len - (key0 + sp * 16 + j * 8));
  }
  bf16x8 pb[2];
  softmax_block<D>(s, w, pb, sl2, masked, key0 + j * 8);
#pragma unroll
  for (int sp = 0; sp < 2; ++sp)
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
      w.o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[sp][b], pb[sp], w.o[b], 0, 0, 0);
}

// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters left at their maxima)
#define HFX_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | (7 << 4) | (15 << 8))

// Wave-uniform description of where the workgroup's tile stream goes: the current prefill item
// and, when the next item of this workgroup is a prefill item too, that one.
struct TileStream {
  int bt0;            // start of the current item's request in the stored block table
  int g;              // kv-head
  int end;            // first key past the current item's last (whole) 64-key tile
  bool next_ok;
  int bt0_n, g_n, kb_n, len_n;   // the same for the next item, its first key and its length in whole tiles' keys
};

// Page ids of the 64-key tile that starts `kt` keys into a request (kt a multiple of 64): one aligned
// quad out of the step's stored block table.  The stored table repeats a request's last page for
// HFX_BT_PAD entries behind it, so the quad needs no clamping a tile past the end.
typedef int i32x4 __attribute__((ext_vector_type(4)));
struct TilePages {
  StagePages half[2];
};

// Pages and kv-head of the tile that starts `kt` keys into the stream.  The tile after an item's
// last is the first tile of the workgroup's next item (key ranges of items start at multiples of
// 64).  `known` says whether the position lies in the current or in the next item; past those (the
// item after next has no ticket yet), and with no next prefill item at all, the stored table is read
// on into its padding, which repeats a request's last page: readable pages whose data is never used.
__device__ __forceinline__ TilePages stream_pages(const int* __restrict__ bt, const TileStream& ts, int kt,
                                                  int& g_out, bool& known) {
  const bool into_next = kt >= ts.end && ts.next_ok;
  const int off = kt - ts.end;
  known = kt < ts.end || (ts.next_ok && off < ts.len_n);
  const int bt0 = into_next ? ts.bt0_n : ts.bt0;
  const int k = into_next ? ts.kb_n + off : kt;
  g_out = into_next ? ts.g_n : ts.g;
  const i32x4 v = *reinterpret_cast<const i32x4*>(bt + bt0 + k / HFX_PAGE);
  TilePages t;
  t.half[0].pg0 = v[0];
  t.half[0].pg1 = v[1];
  t.half[1].pg0 = v[2];
  t.half[1].pg1 = v[3];
  return t;
}

// What a wavefront derives from a prefill item: its q-head and rows, and the key ranges that
// decide whether a tile is worked on and whether it needs masks.
struct WaveRows {
  int head, qrow, wave_kend, wave_pmin;
  bool store;    // qrow is a real row of the chunk
};

template <int D>
__device__ __forceinline__ WaveRows wave_rows(const HfxItem& it, int wave, int n) {
  WaveRows r;
  r.head = it.h0 + wave % it.hn;
  const int r0 = it.row0 + (wave / it.hn) * HFX_WAVE_ROWS;
  const int p = it.rq.ctx_len - it.rq.q_len;
  r.wave_kend = r0 < it.rq.q_len ? p + min(r0 + HFX_WAVE_ROWS, it.rq.q_len) : 0;   // keys >= this: nothing to do
  r.wave_pmin = p + r0;                                                            // keys <= this are visible to every row
  r.qrow = r0 + n;
  r.store = r.qrow < it.rq.q_len;
  return r;
}

// Q^T operand fragments of this lane's row (rows past the chunk read the last row and are never stored)
template <int D>
__device__ __forceinline__ void q_load(PrefillWave<D>& w, const KArgs& a, const HfxItem& it, const WaveRows& r, int Hq,
                                       int j) {
  const int qc = r.store ? r.qrow : it.rq.q_len - 1;
  w.pos = it.rq.ctx_len - it.rq.q_len + qc;
  const __bf16* qp = a.q + (((long)it.rq.q_start + qc) * Hq + r.head) * D + j * 8;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) w.qf[kk] = ld16(qp + kk * 16);
}

// Result of a finished item: normalised bf16 rows, or (m, l, acc) partial rows when the item is one split of a group.
// A lane holds 4-dimension pieces of its own row, so stored straight from the registers every
// instruction would touch 32 rows with 16 bytes each, and the write path takes one request per
// (instruction, line): measured, the 16 stores of an item took longer to issue than two of its
// tiles took to compute.  The bf16 rows therefore go through `stage` (4 KB of LDS owned by this
// wavefront, 64 dimensions of its 32 rows at a time) and leave as whole 128-byte lines, 8 rows per
// instruction.  The 8-byte pieces of a row are swizzled by the row number to spread the LDS banks.
template <int D>
__device__ __forceinline__ void prefill_store(const KArgs& a, const HfxHeader* H, const HfxItem& it, const WaveRows& r,
                                              const PrefillWave<D>& w, int Hq, int wave, int lane, char* stage) {
  // o[b][v] is dimension 32b + (v>>2)*8 + 4j + (v&3) of chunk row `qrow`
  const float lsum = sum_xor32(w.l);
  // The lane's parts of the destination addresses are formed here, per call: left visible, the
  // compiler hoists them out of the item loop, runs out of registers and parks them in scratch
  // memory, and the reload at every hand-over waits for every load the tile stream has in flight.
  asm volatile("" : "+v"(lane));
  const int n = lane & 31, j = lane >> 5;
  if (it.group < 0) {
    const float inv = 1.0f / lsum;
    const int row0 = r.qrow - n;                 // first chunk row of this wavefront
    const int rr = lane >> 3, u = lane & 7;      // read-back: row rr + 8i, 16-byte piece u
    __bf16* dst = a.out + (((long)it.rq.q_start + row0 + rr) * Hq + r.head) * D + u * 8;
#pragma unroll
    for (int p = 0; p < D / 64; ++p) {
#pragma unroll
      for (int bb = 0; bb < 2; ++bb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 ob;
#pragma unroll
          for (int e = 0; e < 4; ++e) ob[e] = (__bf16)(w.o[2 * p + bb][q4 * 4 + e] * inv);
          const int c = 8 * bb + 2 * q4 + j;     // 8-byte piece of the 128-byte half row
          *reinterpret_cast<bf16x4*>(stage + n * 128 + ((c ^ ((n & 7) << 1)) * 8)) = ob;
        }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = rr + 8 * i;
        const bf16x8 line = *reinterpret_cast<const bf16x8*>(stage + row * 128 + ((u ^ (row & 7)) * 16));
        if (row0 + row < it.rq.q_len)
          *reinterpret_cast<bf16x8*>(dst + (long)i * 8 * Hq * D + p * 64) = line;
      }
    }
  } else {
    float* ws_acc = a.ws;
    float* ws_ml = reinterpret_cast<float*>(reinterpret_cast<char*>(a.ws) + H->ws_off_ml);
    const long pr = (long)it.slot_row + wave * HFX_WAVE_ROWS + n;
    float* dst = ws_acc + pr * D + 4 * j;
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 t = {w.o[b][q4 * 4], w.o[b][q4 * 4 + 1], w.o[b][q4 * 4 + 2], w.o[b][q4 * 4 + 3]};
        *reinterpret_cast<f32x4*>(dst + b * 32 + q4 * 8) = t;
      }
    if (j == 0) {
      ws_ml[pr * 2] = w.m;
      ws_ml[pr * 2 + 1] = lsum;
    }
  }
}

// Runs the prefill item t.cur and, for as long as the workgroup's next item is a prefill item as
// well, carries straight on into it: the K/V pipeline does not drain between items, only the
// per-row state (Q, O, m, l) is swapped.  Returns with t.cur at the first item it did not process.
//
// The pipeline, per 64-key tile (two stages, buffers 0 and 1):
//   first stage  : request the next tile's first half from the pool into register set A; multiply
//                  buffer 0; put register set B (this tile's second half, requested a tile ago) into
//                  buffer 1; barrier.
//   second stage : request the next tile's second half into register set B; multiply buffer 1; put
//                  register set A into buffer 0; barrier.
// Every piece therefore has two stages between its request and its use, and ordinary loads are
// used on purpose: the direct-to-LDS form of the load moved about 16 bytes per clock and CU here,
// a quarter of the ordinary path, and bounded the loop.  "Next tile" is a position in the
// workgroup's tile stream: past the end of the item it is the first tile of the next prefill item.
template <int D>
__device__ void prefill_run(const KArgs& a, const HfxHeader* H, const HfxItem* __restrict__ items, int n_items,
                            Tickets& t, int* s_tk, int* ctrl, char* smem, char* o_stage) {
  constexpr int SK = HFX_STAGE_KEYS;
  constexpr int SB = Smem<D>::kStageBytes;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int Hq = H->num_q_heads, Hkv = H->num_kv_heads;
  const int G = Hq / Hkv;
  const int n = lane & 31, j = lane >> 5;
  // The result rows are staged in buffer 1 at the hand-over: its stage has been multiplied, and the
  // slice a wavefront stages its rows in is the slice that only its own next pieces go to.
  char* stage = D == 128 ? smem + SB + wave * 4096 : o_stage + wave * 4096;
  const float sl2 = H->softmax_scale * 1.4426950408889634f;
  const int* bt_all = reinterpret_cast<const int*>(a.desc + H->off_bt);
  // row of this lane's key inside the stage's 32 keys
  const int krow = (n >> 4) * 16 + ((n >> 2) & 1) * 8 + ((n >> 3) & 1) * 4 + (n & 3);
  const int k_lane = (j * 32 + krow) * 16;
  const int v_lane = (n * 2 + (j ^ ((n >> 3) & 1))) * 16;   // V^T rows 32b + n, keys 8j.. of a page, at their swizzled place (copy_lane)
  const CopyLane cl = copy_lane<D>(wave, lane);

  HfxItem it = items[t.cur];
  HfxItem nx = items[t.nxt < n_items ? t.nxt : t.cur];
  TileStream ts;
  auto set_stream = [&]() {
    ts.bt0 = it.rq.bt_start;
    ts.g = it.h0 / G;
    ts.end = it.kb + (it.ke - it.kb + HFX_KEY_TILE - 1) / HFX_KEY_TILE * HFX_KEY_TILE;
    ts.next_ok = t.nxt < n_items && nx.type == HFX_ITEM_PREFILL;
    ts.bt0_n = nx.rq.bt_start;
    ts.g_n = nx.h0 / G;
    ts.kb_n = nx.kb;
    ts.len_n = (nx.ke - nx.kb + HFX_KEY_TILE - 1) / HFX_KEY_TILE * HFX_KEY_TILE;
  };
  set_stream();
  // Tiles (by first key) at whose start the next ticket is published and asked for: published at
  // the last tile but one, asked for a tile earlier.  Items of one or two tiles ask at the
  // hand-over and publish at their first tile.
  int publish_kt, reserve_kt;
  auto set_ticket_points = [&]() {
    const int n_tiles = (it.ke - it.kb + HFX_KEY_TILE - 1) / HFX_KEY_TILE;
    const int ip = n_tiles > 2 ? n_tiles - 2 : 0;
    publish_kt = it.kb + ip * HFX_KEY_TILE;
    reserve_kt = ip > 0 ? publish_kt - HFX_KEY_TILE : -1;
    tickets_reserve(t, ctrl, (int)H->queue_classes, ip == 0);   // the field is dead here: the last publish has read it
  };
  set_ticket_points();

  PrefillWave<D> w;
  WaveRows wr = wave_rows<D>(it, wave, n);
  int wave_end = min(wr.wave_kend, it.ke);   // keys from here on: nothing to do for this wavefront
  q_load<D>(w, a, it, wr, Hq, j);
#pragma unroll
  for (int b = 0; b < D / 32; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) w.o[b][v] = 0.f;
  w.m = NEG_INF;
  w.l = 0.f;

  // cold start: the first tile's first half goes to buffer 0, its second half is requested; the
  // page ids of the tile after it are looked up (they are always asked for a tile before the loads
  // that need them, so that no tile starts by waiting for a scalar load)
  int kt = it.kb;
  StageRegs<D> ra, rb;
  TilePages tn;
  int gn;
  bool tn_known;
  {
    int gq;
    bool known;
    const TilePages tp = stream_pages(bt_all, ts, kt, gq, known);
    stage_load<D>(ra, a.pool, tp.half[0], Hkv, gq, cl, wave);
    stage_load<D>(rb, a.pool, tp.half[1], Hkv, gq, cl, wave);
    tn = stream_pages(bt_all, ts, kt + HFX_KEY_TILE, gn, tn_known);
    stage_write<D>(smem, ra, cl, lane);
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wavefront's pieces are in LDS
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  for (;;) {
    if (kt == publish_kt) {
      // The ticket asked for earlier is published ahead of this tile's barriers, so that the
      // hand-over at the end of the item needs no barrier of its own.  Reading the counter's reply
      // makes the wavefront wait for what it had in flight when it asked.
      tickets_publish(t, s_tk, ctrl, n_items, (int)H->queue_classes);
    }
    if (kt == reserve_kt) tickets_reserve(t, ctrl, (int)H->queue_classes);   // never in the publishing tile
    // ---- first stage: keys kt .. kt + 31 out of buffer 0
    stage_load<D>(ra, a.pool, tn.half[0], Hkv, gn, cl, wave);
    if (kt < wave_end) {
      prefill_stage<D>(w, smem, k_lane, v_lane, kt + SK - 1 > wr.wave_pmin, kt + SK > it.rq.ctx_len, kt,
                       it.rq.ctx_len, j, sl2, smem + SB, rb, cl, lane);
    } else {
      stage_write<D>(smem + SB, rb, cl, lane);
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();   // bare barrier: LDS is only written by the pieces ordered above
    asm volatile("" ::: "memory");  // keep the next stage's LDS reads below the barrier
    // ---- second stage: keys kt + 32 .. kt + 63 out of buffer 1
    stage_load<D>(rb, a.pool, tn.half[1], Hkv, gn, cl, wave);
    // the tile after next, for the next tile's loads
    tn = stream_pages(bt_all, ts, kt + 2 * HFX_KEY_TILE, gn, tn_known);
    if (kt + SK < wave_end) {
      prefill_stage<D>(w, smem + SB, k_lane, v_lane, kt + 2 * SK - 1 > wr.wave_pmin, kt + 2 * SK > it.rq.ctx_len,
                       kt + SK, it.rq.ctx_len, j, sl2, smem, ra, cl, lane);
    } else {
      stage_write<D>(smem, ra, cl, lane);
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    kt += HFX_KEY_TILE;
    if (kt < it.ke) continue;

    // hand-over: the item is finished; its successor's first tile is in buffer 0 and on its way
    const bool carry_on = ts.next_ok;
    prefill_store<D>(a, H, it, wr, w, Hq, wave, lane, stage);
    tickets_take(t, s_tk);
    if (!carry_on) break;
    it = nx;
    nx = items[t.nxt < n_items ? t.nxt : t.cur];   // asked for here, first looked at behind the wait for Q
    set_ticket_points();
    wr = wave_rows<D>(it, wave, n);
    wave_end = min(wr.wave_kend, it.ke);
    q_load<D>(w, a, it, wr, Hq, j);
    // Q is needed by the very next MFMA.  Waiting for it here, in so many words, also tells the
    // compiler that nothing is in flight when the tile loop is re-entered; left to itself it
    // carries the Q loads into the loop as pending and drains the queue down to them on every tile.
    HFX_WAIT_VMCNT(0);
    set_stream();
    // the page ids for the tile after this item's first were asked for while the item after this one
    // had no ticket yet, if this item is one tile long: asked for again, now that it has
    if (!tn_known) tn = stream_pages(bt_all, ts, it.kb + HFX_KEY_TILE, gn, tn_known);
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) w.o[b][v] = 0.f;
    w.m = NEG_INF;
    w.l = 0.f;
    kt = it.kb;
  }
  __syncthreads();     // every wavefront is done with the stage buffers before the LDS is used for anything else
}

// ----------------------------------------------------------------------------------------------
// The persistent kernel: workgroups pull items in descending modelled cost until the queue is
// empty.  A workgroup always knows its next item (see Tickets).  The queue counters live in the
// descriptor; the last workgroup to leave restores them to zero so the descriptor can serve the
// next launch.
// ----------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(HFX_WG_THREADS, 2) void mixed_attention_kernel(
    const HfxHeader hdr, const char* __restrict__ desc, int* __restrict__ ctrl, const __bf16* __restrict__ q,
    const __bf16* __restrict__ pool, float* __restrict__ ws, __bf16* __restrict__ out) {
  // The descriptor's header travels as a kernel argument (the host has it anyway), which takes one
  // dependent load off the start of every workgroup.
  // The descriptor tables are read-only and distinct from everything written here, which lets
  // the compiler fetch them with scalar loads that do not queue behind the KV stream
  KArgs a;
  a.desc = desc;
  a.q = q;
  a.pool = pool;
  a.ws = ws;
  a.out = out;
  __shared__ __attribute__((aligned(1024))) char smem[Smem<D>::kBytes];
  __shared__ int s_tk[2];
  // result rows on their way out (prefill_store): at D = 128 they go through a free stage buffer
  __shared__ __attribute__((aligned(128))) char s_ostage[D == 128 ? 128 : 4 * 4096];
  const HfxHeader* H = &hdr;
  const HfxItem* items = reinterpret_cast<const HfxItem*>(a.desc + H->off_items);
  const int n_items = H->n_items;
  Tickets t;
  t.cur = (int)blockIdx.x;
  t.nxt = (int)(blockIdx.x + gridDim.x);
  t.pending = 0;
  t.parity = 0;
  while (t.cur < n_items) {
    if (items[t.cur].type == HFX_ITEM_DECODE) {
      decode_run<D>(a, H, items, n_items, t, s_tk, &ctrl[0], smem);
    } else {
      prefill_run<D>(a, H, items, n_items, t, s_tk, &ctrl[0], smem, s_ostage);
    }
  }
  // the ticket fetched last is never used; it must have reached the counter before this
  // workgroup reports itself finished, or it could land after the reset below
  HFX_WAIT_VMCNT(0);
  asm volatile("" ::: "memory");
  if (threadIdx.x == 0) {
    const int done = atomicAdd(&ctrl[HFX_QUEUE_CLASSES], 1);
    if (done == (int)gridDim.x - 1) {
      for (int c = 0; c <= HFX_QUEUE_CLASSES; ++c) atomicExch(&ctrl[c], 0);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Page copy: pool pages named by (src, dst) id pairs move between two pools of the same
// geometry (or inside one).  The device half of handing a request's KV blocks from the
// instance that prefilled it to the instance that decodes it (HFX Section 3.3.1,
// disaggregated mode; Section 3.4).  16-byte units; a workgroup moves 16 KB with all of its
// loads in flight before the first store.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_pages_kernel(const int2* __restrict__ pairs, long n_units,
                                                         int units_per_page, const u32x4* __restrict__ src,
                                                         u32x4* __restrict__ dst) {
  const long base = (long)blockIdx.x * 1024 + threadIdx.x;
  u32x4 v[4];
  long to[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const long u = base + 256 * j;
    to[j] = -1;
    if (u < n_units) {
      const long pr = u / units_per_page;
      const int off = (int)(u - pr * units_per_page);
      const int2 id = pairs[pr];
      v[j] = __builtin_nontemporal_load(src + (long)id.x * units_per_page + off);
      to[j] = (long)id.y * units_per_page + off;
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (to[j] >= 0) __builtin_nontemporal_store(v[j], dst + to[j]);
}

// Page gather hook: one thread per (token, kv-head, dimension); a pure 2-byte copy through the
// same request record and block table the attention kernel walks.
__global__ void gather_kv_kernel(const char* desc, const uint16_t* pool, int request, uint16_t* k_out,
                                 uint16_t* v_out) {
  const HfxHeader* H = reinterpret_cast<const HfxHeader*>(desc);
  const HfxReq rq = reinterpret_cast<const HfxReq*>(desc + H->off_req)[request];
  const int* bt = reinterpret_cast<const int*>(desc + H->off_bt) + rq.bt_start;
  const int Hkv = H->num_kv_heads, D = H->head_dim;
  const long total = (long)rq.ctx_len * Hkv * D;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int d = (int)(i % D);
    const int g = (int)((i / D) % Hkv);
    const long t = i / ((long)D * Hkv);
    const long pg = bt[t / HFX_PAGE];
    const int slot = (int)(t % HFX_PAGE);
    const long blk = ((pg * Hkv + g) * 2) * (16L * D);
    k_out[i] = pool[blk + ((long)(d / 16) * HFX_PAGE + slot) * 16 + d % 16];
    v_out[i] = pool[blk + 16L * D + (long)d * HFX_PAGE + slot];
  }
}

// KV append: one workgroup per (run, kv-head), a run being the new tokens of one request that fall
// into one page (at most 16 consecutive slots).  The tokens' K and V rows for the head are read in
// whole rows into LDS and leave in the pool's block order: a K piece of 16 dimensions is 32
// contiguous bytes per slot, and a V row (one dimension) gets its run of slots as one contiguous
// piece -- stored token by token, the dimension-major V block took one 2-byte request per
// (token, dimension), which was most of the launch.  D threads; rows are padded by one word in LDS
// so that a column walk does not stay on one bank.
template <int D>
__global__ __launch_bounds__(D) void append_kv_kernel(const HfxRun* __restrict__ runs, int Hkv,
                                                      const uint16_t* __restrict__ k_new,
                                                      const uint16_t* __restrict__ v_new,
                                                      uint16_t* __restrict__ pool) {
  constexpr int LD = D + 2;                       // LDS row stride in elements
  __shared__ uint16_t sk[HFX_PAGE * LD];
  __shared__ uint16_t sv[HFX_PAGE * LD];
  const HfxRun run = runs[blockIdx.x];
  const int g = blockIdx.y;
  const int tid = threadIdx.x;
  // rows in: thread t takes 2 elements of each token's row (4-byte loads, a row is D*2 bytes contiguous)
  for (int i = tid; i < run.n * (D / 2); i += D) {
    const int tok = i / (D / 2), e2 = i % (D / 2);
    const long src = ((long)(run.row0 + tok) * Hkv + g) * D + e2 * 2;
    *reinterpret_cast<uint32_t*>(&sk[tok * LD + e2 * 2]) = *reinterpret_cast<const uint32_t*>(k_new + src);
    *reinterpret_cast<uint32_t*>(&sv[tok * LD + e2 * 2]) = *reinterpret_cast<const uint32_t*>(v_new + src);
  }
  __syncthreads();
  uint16_t* kblk = pool + (((long)run.page * Hkv + g) * 2) * (16L * D);
  uint16_t* vblk = kblk + 16L * D;
  // K block [D/16][16 slots][16]: 2 D pieces of 16 bytes, piece u = (dimension group u / 32, slot
  // (u % 32) / 2, half u % 2); consecutive threads write consecutive pieces
#pragma unroll
  for (int u = tid; u < 2 * D; u += D) {
    const int slot = (u % 32) / 2;
    if (slot >= run.slot0 && slot < run.slot0 + run.n) {
      const uint16_t* src = &sk[(slot - run.slot0) * LD + (u / 32) * 16 + (u % 2) * 8];
      u32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const uint32_t*>(src + 2 * e);
      *reinterpret_cast<u32x4*>(kblk + u * 8) = v;
    }
  }
  // V block [D][16 slots]: a row (one dimension) is 32 bytes
  if (run.slot0 == 0 && run.n == HFX_PAGE) {
    // a whole page: 2 D pieces of 16 bytes, piece u = (dimension u / 2, slots 8 (u % 2) ..)
#pragma unroll
    for (int u = tid; u < 2 * D; u += D) {
      const int d = u >> 1, s0 = (u & 1) * 8;
      u32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        v[e] = (uint32_t)sv[(s0 + 2 * e) * LD + d] | ((uint32_t)sv[(s0 + 2 * e + 1) * LD + d] << 16);
      *reinterpret_cast<u32x4*>(vblk + u * 8) = v;
    }
  } else {
    // part of a page: thread d writes its row's slots, two at a time where both belong to the run
    const int d = tid;
    uint16_t* dst = vblk + (long)d * HFX_PAGE;
    const int lo = run.slot0, hi = run.slot0 + run.n;
#pragma unroll
    for (int w = 0; w < HFX_PAGE / 2; ++w) {
      const int a = 2 * w, b = 2 * w + 1;
      const bool in_a = a >= lo && a < hi, in_b = b >= lo && b < hi;
      if (in_a && in_b)
        *reinterpret_cast<uint32_t*>(dst + a) = (uint32_t)sv[(a - lo) * LD + d] | ((uint32_t)sv[(b - lo) * LD + d] << 16);
      else if (in_a)
        dst[a] = sv[(a - lo) * LD + d];
      else if (in_b)
        dst[b] = sv[(b - lo) * LD + d];
    }
  }
}

// ------------------------------------------------------------------ static workspace
// Split partials for callers that cannot allocate device memory: a fixed array inside the code
// object, one copy per GPU, held until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; the device address it yields (per device) is what launches get.
static __device__ __align__(256) unsigned char scratch[HFX_STATIC_WS_BYTES];

hipError_t static_workspace(void** ptr) {
  static std::mutex mu;
  static void* addr[HFX_MAX_DEVICES];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= HFX_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

// ------------------------------------------------------------------ host-side launch helpers
hipError_t max_resident_workgroups(int head_dim, int* per_cu) {
  if (head_dim == 128)
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, mixed_attention_kernel<128>, HFX_WG_THREADS, 0);
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, mixed_attention_kernel<64>, HFX_WG_THREADS, 0);
}

hipError_t launch_mixed_attention(const HfxHeader& h, int grid, void* desc, const void* q, const void* pool, void* ws,
                                  void* out, hipStream_t stream) {
  const int head_dim = h.head_dim, n_units = h.n_units;
  const char* d = static_cast<const char*>(desc);
  int* ctrl = reinterpret_cast<int*>(static_cast<char*>(desc) + h.off_ctrl);
  const __bf16* qp = static_cast<const __bf16*>(q);
  const __bf16* pp = static_cast<const __bf16*>(pool);
  float* wp = static_cast<float*>(ws);
  __bf16* op = static_cast<__bf16*>(out);
  if (head_dim == 128)
    hipLaunchKernelGGL(mixed_attention_kernel<128>, dim3(grid), dim3(HFX_WG_THREADS), 0, stream, h, d, ctrl, qp, pp, wp, op);
  else
    hipLaunchKernelGGL(mixed_attention_kernel<64>, dim3(grid), dim3(HFX_WG_THREADS), 0, stream, h, d, ctrl, qp, pp, wp, op);
  if (n_units > 0) {
    const HfxUnit* units = reinterpret_cast<const HfxUnit*>(d + h.off_units);
    const HfxGroup* groups = reinterpret_cast<const HfxGroup*>(d + h.off_groups);
    const float* ml = reinterpret_cast<const float*>(static_cast<const char*>(ws) + h.ws_off_ml);
    const int Hq = h.num_q_heads, G = h.num_q_heads / h.num_kv_heads;
    if (head_dim == 128)
      hipLaunchKernelGGL(merge_kernel<128>, dim3(n_units), dim3(HFX_WG_THREADS), 0, stream, units, groups, wp, ml, Hq, G, op);
    else
      hipLaunchKernelGGL(merge_kernel<64>, dim3(n_units), dim3(HFX_WG_THREADS), 0, stream, units, groups, wp, ml, Hq, G, op);
  }
  return hipGetLastError();
}

hipError_t launch_copy_pages(const void* pairs, long n_pairs, int units_per_page, const void* src, void* dst,
                             hipStream_t stream) {
  const long n_units = n_pairs * units_per_page;
  if (n_units == 0) return hipSuccess;
  const long blocks = (n_units + 1023) / 1024;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(copy_pages_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     static_cast<const int2*>(pairs), n_units, units_per_page, static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst));
  return hipGetLastError();
}

hipError_t launch_gather_kv(const void* desc, const void* pool, int request, long elements, void* k_out,
                            void* v_out, hipStream_t stream) {
  long blocks = (elements + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_kv_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     static_cast<const char*>(desc), static_cast<const uint16_t*>(pool), request,
                     static_cast<uint16_t*>(k_out), static_cast<uint16_t*>(v_out));
  return hipGetLastError();
}

hipError_t launch_append_kv(const HfxHeader& h, const void* desc, const void* k_new, const void* v_new, void* pool,
                            hipStream_t stream) {
  if (h.n_runs <= 0) return hipSuccess;
  const HfxRun* runs = reinterpret_cast<const HfxRun*>(static_cast<const char*>(desc) + h.off_runs);
  const dim3 grid((unsigned)h.n_runs, (unsigned)h.num_kv_heads);
  if (h.head_dim == 128)
    hipLaunchKernelGGL(append_kv_kernel<128>, grid, dim3(128), 0, stream, runs, h.num_kv_heads,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(pool));
  else
    hipLaunchKernelGGL(append_kv_kernel<64>, grid, dim3(64), 0, stream, runs, h.num_kv_heads,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                       static_cast<uint16_t*>(pool));
  return hipGetLastError();
}

}  // namespace hfx
