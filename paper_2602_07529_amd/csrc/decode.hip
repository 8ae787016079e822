// Branch-parallel decode over a paged KV cache (paper section 3.2: tokens carry KV-cache
// references; section 4.3 Fork: sibling branches share the prefix KV without copying).
//
// dag_kv_append_rope : store each live branch's new (rotated) key and value into its tail page.
// dag_attn_decode    : cascade attention.  One launch of independent single-wave work items:
//     shared items  (group, kv head, 32-row block, page split): the queries of ALL siblings of the
//                   group (siblings x query heads of the kv head, stacked as MFMA columns) against
//                   a slice of the shared pages -- each shared page is fetched once per group;
//     own items     (branch, kv head, page split): the branch's query heads against its own pages.
//   Every item writes an un-normalised partial (o, m, l); a second launch merges the partials of
//   each (branch, head) by log-sum-exp.
//
// Pool formats (bf16, 16 tokens per page) are chosen so that global loads land directly in MFMA
// operand layout, fully coalesced, with no LDS staging:
//   K pool [P][hkv][D/8][16][8] : for a fixed 8-wide d-chunk the 16 keys of a page are contiguous;
//                                 one load instruction of a wave reads 2 x 512 contiguous bytes.
//   V pool [P][hkv][D][16]      : for a fixed d the 16 keys of a page are contiguous (the
//                                 contraction dimension of P.V); one load reads 1 KiB contiguous.
// Scores are computed transposed (S^T = K Q^T, 32 keys x 32 query rows per MFMA block) and MFMA
// row i is mapped to key pi(i), so the probabilities come out of the first product already in the
// B-operand layout of the second (O^T = V^T P^T).
#include <stdlib.h>

#include <mutex>

#include "common.h"

namespace {

constexpr int PAGE = DAG_PAGE_SIZE;

struct DecodeArgs {
  const int32_t* group_branch_off;
  const int32_t* shared_page_off;
  const int32_t* shared_pages;
  const int32_t* shared_len;
  const int32_t* branch_page_off;
  const int32_t* branch_pages;
  const int32_t* branch_len;
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  uint16_t* out;
  float* part_o_a;   // [items_a][32][D]
  float* part_ml_a;  // [items_a][32][2]
  float* part_o_b;   // [items_b][G][D]
  float* part_ml_b;  // [items_b][G][2]
  int n_groups, n_live, hq, hkv, G;
  int rb_max;        // 32-row blocks per (group, kv head)
  int chunk_a, splits_a, chunk_b, splits_b;
  int items_a, items_b;
  int item_base;     // first work item of this launch (k_decode)
  int wide_shared;   // k_decode_wide: workgroups that take shared items (the rest take own pages)
  float sc;          // softmax_scale * log2(e)
  float th;          // 8 / sc: how far a score may exceed the reference maximum before it is raised
  float scale;
};

// Decode over lists of KV segments: a segment is a page list with a token count and the set of
// live branches that read it; a branch's context is the union of the segments it reads.
struct SegItem {  // one work item: a slice of a segment's pages against one 32-row block of its readers' rows
  int32_t page_off, len, e0, nrows, row0, split, pad0, pad1;
};
struct SegArgs {
  const int32_t* seg_page_off;
  const int32_t* seg_pages;
  const int32_t* seg_len;
  const int32_t* seg_reader_off;
  const int32_t* seg_readers;
  const int32_t* seg_reader_len;  // optional: leading tokens of the segment each reader-list entry sees
  const int32_t* branch_entry_off;
  const int32_t* branch_entries;
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  uint16_t* out;
  float* part_o;   // [splits][total_readers][hq][D]
  float* part_ml;  // [splits][total_readers][hq][2]
  SegItem* items;        // [item_cap] compact list of (segment, row block, slice), written by k_seg_plan
  int32_t* item_total;   // number of list entries
  int32_t* entry_nsplit; // [total_readers] slices of the segment of each reader-list entry
  int item_cap;
  int n_segments, n_live, hq, hkv, G;
  int rb_max;      // 32-row blocks per (segment, kv head)
  int chunk, splits, total_readers;
  float sc, th;
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
typedef __attribute__((ext_vector_type(8))) float f32x8;

// MFMA row i (0..31) of a 32-key block -> (page 0/1, slot 0..15): registers 0..7 / 8..15 of the
// transposed score block then hold slots 8H..8H+7 of page 0 / page 1.
__device__ __forceinline__ int key_of_row(int i) {
  const int a = i >> 3, hh = (i >> 2) & 1, c = i & 3;
  return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}

template <int D>
struct KVBlock {           // one 32-key block (2 pages) in operand layout
  bf16x8 k[D / 16];        // k[s]: d-chunk 2s+H of key pi(L)
  bf16x8 v[2][D / 32];     // v[page][db]: keys 8H..8H+7 of dimension 32db+L
};

// pgv: page ids of the item's slice, lane i holds page p0 + (i % 64) of the current 64-page window
// (fetched once per window, so that no page-table load sits in front of every K/V load)
template <int D, typename A>
__device__ __forceinline__ void load_block(KVBlock<D>& blk, const A& a, int pgv, int pb_rel, int last_rel,
                                           int hk, int L, int H, int kpage_sel, int kslot) {
  const int pg0 = __builtin_amdgcn_readlane(pgv, pb_rel & 63);
  const int pg1 = __builtin_amdgcn_readlane(pgv, min(pb_rel + 1, last_rel) & 63);
  const size_t kbase0 = ((size_t)pg0 * a.hkv + hk) * (size_t)(D * PAGE);
  const size_t kbase1 = ((size_t)pg1 * a.hkv + hk) * (size_t)(D * PAGE);
  const uint16_t* kp = a.k_pool + (kpage_sel ? kbase1 : kbase0) + kslot * 8 + H * (PAGE * 8);
#pragma unroll
  for (int s = 0; s < D / 16; ++s) blk.k[s] = *(const bf16x8*)(kp + s * (2 * PAGE * 8));
  const uint16_t* vp0 = a.v_pool + kbase0 + L * PAGE + H * 8;
  const uint16_t* vp1 = a.v_pool + kbase1 + L * PAGE + H * 8;
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    blk.v[0][db] = *(const bf16x8*)(vp0 + db * 32 * PAGE);
    blk.v[1][db] = *(const bf16x8*)(vp1 + db * 32 * PAGE);
  }
}

// qop(s): the query operand of MFMA step s.  k_decode keeps the operands in LDS, qs[s * 64 + lane]
// (they are needed once per 32-key block; keeping them out of the register file lets two waves
// share a SIMD, which doubles the bytes in flight); k_decode_wide keeps them in registers.
// First phase of a 32-key block: scores against the key operands, online softmax bookkeeping
// (accumulators rescaled when the reference maximum moves), probabilities as the two B operands
// of the second phase.
template <int D, typename QF>
__device__ __forceinline__ void block_scores(const bf16x8 (&kop)[D / 16], QF&& qop, f32x16* O, float& m, float& l,
                                             float sc, float th, int key0, int len, int lim, int H,
                                             bf16x8& pb0, bf16x8& pb1) {
  f32x16 S;
#pragma unroll
  for (int r = 0; r < 16; ++r) S[r] = 0.f;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) S = mfma32(kop[s], qop(s), S);
  if (key0 + 32 > len) {  // len: wave-uniform, the smallest of the rows' limits; lim: this lane's row
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = key0 + 16 * (r >> 3) + 8 * H + (r & 7);
      S[r] = key < lim ? S[r] : -INFINITY;
    }
  }
  float bm = S[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) bm = fmaxf(bm, S[r]);
  bm = fmaxf(bm, __shfl_xor(bm, 32));
  // The reference maximum m is raised only when some row of the wave exceeds it by more than 2^8
  // (in the exponent's units); the rescale of the accumulators is then rare, and probabilities up
  // to 2^8 are absorbed exactly by fp32 accumulation and the final division.
  if (__builtin_amdgcn_ballot_w64(bm > m + th) != 0) {
    const float m_new = fmaxf(m, bm);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * sc);
    m = m_new;
    l *= alpha;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[db][r] *= alpha;
  }
  const float msc = m * sc;
  f32x8 p0, p1;
  float rowsum = 0.f;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    p0[r] = __builtin_amdgcn_exp2f(fmaf(S[r], sc, -msc));
    p1[r] = __builtin_amdgcn_exp2f(fmaf(S[8 + r], sc, -msc));
    rowsum += p0[r] + p1[r];
  }
  l += rowsum;
  pb0 = __builtin_convertvector(p0, bf16x8);
  pb1 = __builtin_convertvector(p1, bf16x8);
}

// Second phase: O^T += V^T P^T with the value operands of the block's two pages.
template <int D>
__device__ __forceinline__ void block_pv(const bf16x8 (&v0)[D / 32], const bf16x8 (&v1)[D / 32], bf16x8 pb0,
                                         bf16x8 pb1, f32x16* O) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    O[db] = mfma32(v0[db], pb0, O[db]);
    O[db] = mfma32(v1[db], pb1, O[db]);
  }
}

// Value operands of a block that reaches past the `vlen` tokens its page list holds: the slots
// behind the last token (and the page that a slice with an odd page count reads twice) may hold
// anything, NaN or infinity bit patterns included, and a zero probability does not neutralise
// those in the product, so their elements are cleared.  v0 / v1 hold keys 8 H .. 8 H + 7 of the
// block's first / second page.
template <int D>
__device__ __forceinline__ void clear_unused_values(bf16x8 (&v0)[D / 32], bf16x8 (&v1)[D / 32], int key0, int vlen,
                                                    int H) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {  // 32-bit word w of an operand = keys 8 H + 2 w, 8 H + 2 w + 1 of the page
    const int k0 = key0 + 8 * H + 2 * w, k1 = k0 + 16;
    const uint32_t m0 = (k0 < vlen ? 0x0000ffffu : 0u) | (k0 + 1 < vlen ? 0xffff0000u : 0u);
    const uint32_t m1 = (k1 < vlen ? 0x0000ffffu : 0u) | (k1 + 1 < vlen ? 0xffff0000u : 0u);
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      u32x4 a = __builtin_bit_cast(u32x4, v0[db]), b = __builtin_bit_cast(u32x4, v1[db]);
      a[w] &= m0;
      b[w] &= m1;
      v0[db] = __builtin_bit_cast(bf16x8, a);
      v1[db] = __builtin_bit_cast(bf16x8, b);
    }
  }
}

// vlen: tokens the page list holds (wave-uniform); len <= vlen: the smallest of the rows' limits.
// The block's value operands are cleared in place where they reach past vlen (the block is dead
// after this call: its registers are refilled by the next load).
template <int D, typename QF>
__device__ __forceinline__ void compute_block(KVBlock<D>& blk, QF&& qop, f32x16* O, float& m, float& l,
                                              float sc, float th, int key0, int len, int lim, int vlen, int H) {
  bf16x8 pb0, pb1;
  block_scores<D>(blk.k, qop, O, m, l, sc, th, key0, len, lim, H, pb0, pb1);
  if (key0 + 32 > vlen) clear_unused_values<D>(blk.v[0], blk.v[1], key0, vlen, H);
  block_pv<D>(blk.v[0], blk.v[1], pb0, pb1, O);
}

// The loop of a single-wave work item: pages [p0, p1) of one page list, 32 keys (two pages) per
// step, the next block's loads in flight while the current one is computed.  `lim` is the number
// of leading tokens of the list that this lane's row sees (keys at or past it are masked), `len`
// the smallest `lim` of the wave, `vlen` the number of tokens the list holds.  Leaves the un-normalised partial
// (O, reference maximum m, row sum l of this lane's half) in registers.
template <int D, typename A, typename QF>
__device__ __forceinline__ void stream_slice(const A& a, const int32_t* pages, int p0, int p1, int len, int lim,
                                             int vlen, int hk, int lane, QF&& qop, f32x16* O, float& m, float& l) {
  const int L = lane & 31, H = lane >> 5;
  const int kr = key_of_row(L);
  const int kpage_sel = kr >> 4, kslot = kr & 15;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
  m = -1e30f;
  l = 0.f;

  // Page ids in windows of 64 (lane i: page p0 + 64 w + i); a block never straddles a window
  // because windows and blocks both start at even offsets.
  const int np = p1 - p0;
  int pgv = pages[p0 + min(lane, np - 1)];
  asm volatile("" ::"v"(pgv));  // arrived: a wait for it inside the loop would also wait for the K/V loads in flight
  KVBlock<D> b0, b1;
  load_block<D>(b0, a, pgv, 0, np - 1, hk, L, H, kpage_sel, kslot);
  int pb = 0;  // relative to p0
  while (true) {
    if (pb + 2 < np) {
      if (((pb + 2) & 63) == 0) {
        pgv = pages[p0 + min(pb + 2 + lane, np - 1)];
        asm volatile("" ::"v"(pgv));
      }
      load_block<D>(b1, a, pgv, pb + 2, np - 1, hk, L, H, kpage_sel, kslot);
    }
    compute_block<D>(b0, qop, O, m, l, a.sc, a.th, (p0 + pb) * PAGE, len, lim, vlen, H);
    pb += 2;
    if (pb >= np) break;
    if (pb + 2 < np) {
      if (((pb + 2) & 63) == 0) {
        pgv = pages[p0 + min(pb + 2 + lane, np - 1)];
        asm volatile("" ::"v"(pgv));
      }
      load_block<D>(b0, a, pgv, pb + 2, np - 1, hk, L, H, kpage_sel, kslot);
    }
    compute_block<D>(b1, qop, O, m, l, a.sc, a.th, (p0 + pb) * PAGE, len, lim, vlen, H);
    pb += 2;
    if (pb >= np) break;
  }
}

template <int D>
__global__ void __launch_bounds__(64, 2) k_decode(DecodeArgs a) {
  __shared__ bf16x8 qs_all[(D / 16) * 64];
  const int item = blockIdx.x + a.item_base;
  const int lane = threadIdx.x, L = lane & 31, H = lane >> 5;
  const bool is_a = item < a.items_a;
  int hk, split, chunk, len, nrows, row0, branch0;
  const int32_t* pages;
  if (is_a) {
    int x = item;
    split = x % a.splits_a; x /= a.splits_a;
    const int rb = x % a.rb_max; x /= a.rb_max;
    hk = x % a.hkv;
    const int g = x / a.hkv;
    branch0 = a.group_branch_off[g];
    nrows = (a.group_branch_off[g + 1] - branch0) * a.G;
    row0 = rb * 32;
    pages = a.shared_pages + a.shared_page_off[g];
    len = a.shared_len[g];
    chunk = a.chunk_a;
  } else {
    int x = item - a.items_a;
    split = x % a.splits_b; x /= a.splits_b;
    hk = x % a.hkv;
    branch0 = x / a.hkv;
    nrows = a.G;
    row0 = 0;
    pages = a.branch_pages + a.branch_page_off[branch0];
    len = a.branch_len[branch0];
    chunk = a.chunk_b;
  }
  const int npages = (len + PAGE - 1) / PAGE;
  const int p0 = split * chunk, p1 = min(p0 + chunk, npages);
  const int row = row0 + L;
  const bool row_ok = row < nrows;

  float* po;
  float* pml;
  if (is_a) {
    po = a.part_o_a + ((size_t)item * 32 + L) * D;
    pml = a.part_ml_a + ((size_t)item * 32 + L) * 2;
  } else {
    po = a.part_o_b + ((size_t)(item - a.items_a) * a.G + L) * D;
    pml = a.part_ml_b + ((size_t)(item - a.items_a) * a.G + L) * 2;
  }
  if (p0 >= p1 || row0 >= nrows) {  // empty slice: neutral partial
    if (row_ok && H == 0) {
      pml[0] = -1e30f;
      pml[1] = 0.f;
    }
    return;
  }

  const bf16x8* qf = qs_all + lane;
  {
    const int rr = row_ok ? row : 0;
    const int br = branch0 + rr / a.G, head = hk * a.G + rr % a.G;
    const uint16_t* qp = a.q + ((size_t)br * a.hq + head) * D + 8 * H;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qs_all[s * 64 + lane] = *(const bf16x8*)(qp + 16 * s);
  }
  auto qop = [&](int s) { return qf[s * 64]; };
  f32x16 O[D / 32];
  float m, l;
  stream_slice<D>(a, pages, p0, p1, len, len, len, hk, lane, qop, O, m, l);

  const float l_tot = l + __shfl_xor(l, 32);
  if (row_ok) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 o = {O[db][4 * r4], O[db][4 * r4 + 1], O[db][4 * r4 + 2], O[db][4 * r4 + 3]};
        *(f32x4*)(po + 32 * db + 8 * r4 + 4 * H) = o;
      }
    if (H == 0) {
      pml[0] = m;
      pml[1] = l_tot;
    }
  }
}

// Segment form, step 1: the work items.  Segment lengths and reader counts live in device memory,
// so a launch sized by the host bounds would consist mostly of items that find nothing to do, and
// those cost time even when they exit at once (they sit between the real items in the dispatch
// order and hold wave slots while their loads return).  One workgroup therefore writes the compact
// list: for every segment, in the caller's order, its slices x row blocks (exclusive scan of the
// counts), and for every reader-list entry the number of slices its segment has.
constexpr int PLAN_THREADS = 1024;
__global__ void __launch_bounds__(PLAN_THREADS) k_seg_plan(SegArgs a) {
  __shared__ int s_wave[PLAN_THREADS / 64];
  __shared__ int s_carry;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int base = 0; base < a.n_segments; base += PLAN_THREADS) {
    const int s = base + tid;
    int len = 0, e0 = 0, nr = 0, nsp = 0, rbs = 0;
    if (s < a.n_segments) {
      len = max(a.seg_len[s], 0);
      e0 = a.seg_reader_off[s];
      nr = max(a.seg_reader_off[s + 1] - e0, 0);
      const int npages = (len + PAGE - 1) / PAGE;
      nsp = min((npages + a.chunk - 1) / a.chunk, a.splits);
      rbs = min((nr * a.G + 31) / 32, a.rb_max);
    }
    const int cnt = nsp * rbs;
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) s_wave[w] = incl;
    __syncthreads();
    int start = s_carry + incl - cnt;
    for (int i = 0; i < w; ++i) start += s_wave[i];
    if (s < a.n_segments) {
      int k = start;
      for (int sp = nsp - 1; sp >= 0; --sp)
        for (int rb = 0; rb < rbs; ++rb, ++k)
          if (k < a.item_cap) a.items[k] = SegItem{a.seg_page_off[s], len, e0, nr * a.G, rb * 32, sp, 0, 0};
      for (int e = e0; e < e0 + nr; ++e)
        if (e >= 0 && e < a.total_readers) a.entry_nsplit[e] = nsp;
    }
    __syncthreads();
    if (tid == PLAN_THREADS - 1) s_carry = min(start + cnt, a.item_cap);
    __syncthreads();
  }
  if (tid == 0) *a.item_total = s_carry;
}

// Step 2: one wave per (work item, kv head).  Row j * G + g of a segment is query head hk * G + g
// of its j-th reader; the partial of a row goes to the reader's entry in the reader list, which is
// where the combination step looks for it.  The launch covers the host's bound on the list; the
// workgroups past its end exit.
template <int D>
__global__ void __launch_bounds__(64, 2) k_decode_seg(SegArgs a) {
  __shared__ bf16x8 qs_all[(D / 16) * 64];
  const int lane = threadIdx.x, L = lane & 31, H = lane >> 5;
  const int hk = blockIdx.x % a.hkv, idx = blockIdx.x / a.hkv;
  if (idx >= *a.item_total) return;
  const SegItem it = a.items[idx];
  const int len = it.len, e0 = it.e0, nrows = it.nrows, row0 = it.row0, split = it.split;
  const int npages = (len + PAGE - 1) / PAGE;
  const int p0 = split * a.chunk;
  int p1 = min(p0 + a.chunk, npages);
  if (row0 >= nrows || p0 >= p1) return;  // (never listed)
  const int row = row0 + L;
  const bool row_ok = row < nrows;
  const int rr = row_ok ? row : row0;
  const int entry = e0 + rr / a.G, head = hk * a.G + rr % a.G;
  const bool store_ok = row_ok && entry < a.total_readers;  // (a reader list longer than announced: no partial)
  const size_t pbase = ((size_t)split * a.total_readers + entry) * a.hq + head;
  // per-reader visible prefix of the segment (a token of a node being prefilled sees the node's
  // tokens up to itself): the slice ends at the longest prefix of the wave's rows
  int lim = len, lim_min = len;
  if (a.seg_reader_len) {
    lim = min(max(a.seg_reader_len[entry], 0), len);
    int lim_max = lim;
    lim_min = lim;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      lim_max = max(lim_max, __shfl_xor(lim_max, o));
      lim_min = min(lim_min, __shfl_xor(lim_min, o));
    }
    p1 = min(p1, (lim_max + PAGE - 1) / PAGE);
    if (p0 >= p1) {  // no row of this block sees a token of the slice: neutral partial
      if (store_ok && H == 0) {
        a.part_ml[pbase * 2] = -1e30f;
        a.part_ml[pbase * 2 + 1] = 0.f;
      }
      return;
    }
  }
  const int br = min(max(a.seg_readers[entry], 0), a.n_live - 1);

  const bf16x8* qf = qs_all + lane;
  {
    const uint16_t* qp = a.q + ((size_t)br * a.hq + head) * D + 8 * H;
#pragma unroll
    for (int t = 0; t < D / 16; ++t) qs_all[t * 64 + lane] = *(const bf16x8*)(qp + 16 * t);
  }
  auto qop = [&](int t) { return qf[t * 64]; };
  f32x16 O[D / 32];
  float m, l;
  stream_slice<D>(a, a.seg_pages + it.page_off, p0, p1, lim_min, lim, len, hk, lane, qop, O, m, l);

  const float l_tot = l + __shfl_xor(l, 32);
  if (store_ok) {
    float* po = a.part_o + pbase * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 o = {O[db][4 * r4], O[db][4 * r4 + 1], O[db][4 * r4 + 2], O[db][4 * r4 + 3]};
        *(f32x4*)(po + 32 * db + 8 * r4 + 4 * H) = o;
      }
    if (H == 0) {
      a.part_ml[pbase * 2] = m;
      a.part_ml[pbase * 2 + 1] = l_tot;
    }
  }
}

// Step 3: one wave per (branch, query head): log-sum-exp combination over the slices of every
// segment the branch reads.  The branch's entries in the reader lists name its partials (and how
// many slices each has); the lanes fetch the
// (maximum, sum) pairs of up to 64 (entry, split) pairs at once, the wave agrees on the maximum
// and the weights, and the weighted partial outputs are added pair by pair.  A branch without any
// key gets zeros.
template <int D>
__global__ void __launch_bounds__(64) k_decode_seg_merge(SegArgs a) {
  const int r = blockIdx.x / a.hq, head = blockIdx.x % a.hq;
  const int lane = threadIdx.x;
  constexpr int PER = D / 64;  // output elements per lane
  float acc[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) acc[e] = 0.f;
  float mx = -1e30f, lsum = 0.f;
  const int e0 = a.branch_entry_off[r];
  const int npairs = (a.branch_entry_off[r + 1] - e0) * a.splits;
  for (int b = 0; b < npairs; b += 64) {
    const int i = b + lane;
    float ms = -1e30f, ls = 0.f;
    uint32_t base = 0;
    if (i < npairs) {
      const int entry = a.branch_entries[e0 + i / a.splits];
      if (entry >= 0 && entry < a.total_readers && i % a.splits < a.entry_nsplit[entry]) {
        base = (uint32_t)(((size_t)(i % a.splits) * a.total_readers + entry) * a.hq + head);
        const float2 ml = *(const float2*)(a.part_ml + (size_t)base * 2);
        if (ml.y > 0.f) {
          ms = ml.x;
          ls = ml.y;
        }
      }
    }
    float cm = ms;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) cm = fmaxf(cm, __shfl_xor(cm, o));
    const float mn = fmaxf(mx, cm);
    const float keep = __builtin_amdgcn_exp2f((mx - mn) * a.sc);
    const float wgt = ls > 0.f ? __builtin_amdgcn_exp2f((ms - mn) * a.sc) : 0.f;
    float part = ls * wgt;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    lsum = lsum * keep + part;
    mx = mn;
#pragma unroll
    for (int t = 0; t < PER; ++t) acc[t] *= keep;
    unsigned long long live = __builtin_amdgcn_ballot_w64(ls > 0.f);
    while (live) {
      const int j = __builtin_ctzll(live);
      live &= live - 1;
      const float wj = __shfl(wgt, j);
      const uint32_t bj = (uint32_t)__shfl((int)base, j);
#pragma unroll
      for (int t = 0; t < PER; ++t) acc[t] += wj * a.part_o[(size_t)bj * D + lane * PER + t];
    }
  }
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  uint16_t* o = a.out + ((size_t)r * a.hq + head) * D + lane * PER;
  if (PER == 2) {
    *(uint32_t*)o = dag_pack_bf2(acc[0] * inv, acc[PER - 1] * inv);
  } else {
    o[0] = (uint16_t)dag_f2bf(acc[0] * inv);
  }
}

// Shared items of wide sibling groups (more than 32 stacked query rows per KV head, e.g. 32 siblings
// x 5 query heads): one workgroup per (group, kv head, page split) with one wave per 32-row
// block.  The waves share the K/V blocks through a ring in LDS (global -> LDS directly, 16 bytes
// per lane; a page of the pools is already the operand image), so the shared pages are streamed
// once per group whatever the number of rows, and up to RING blocks are in flight per workgroup
// instead of one per wave.  A row block is served by `nsub` waves that take the key blocks in
// turn (wave `sub` of a row block computes blocks sub, sub + nsub, ...), each with accumulators
// of its own that are put together through LDS at the end: a wave's chain of LDS reads, score
// MFMAs, softmax arithmetic and P V MFMAs is long and serial, so a SIMD needs two or three of
// them to stay busy.  The workgroup meets at a barrier once per round of nsub blocks.  Writes the
// same partials as the shared items of k_decode.
constexpr int WIDE_RING = 6;                    // 32-key blocks in the ring (96 KiB of LDS at head_dim 128; behind it the query operands)
constexpr int WIDE_MAX_WAVES = 8;               // row blocks of a workgroup
constexpr int WIDE_MAX_THREADS = 768;           // three waves per SIMD (the register budget is set for that)
constexpr int WIDE_OWN_WAVES = WIDE_RING / 2;   // waves that share the own pages of a branch
template <int D>
constexpr int wide_block_bytes() { return 4 * PAGE * D * 2; }  // K and V of two pages
// waves per row block: as many as fit into twelve waves, and their accumulators (64 lanes x
// (D / 2 + 4) floats per wave) into the ring for the final combination
// (a round's blocks are issued a round ahead, so the ring holds two rounds)
inline int wide_nsub(int rb_max, int D) {
  int n = (WIDE_MAX_THREADS / 64) / rb_max;
  if (n > WIDE_RING / 2) n = WIDE_RING / 2;
  while (n > 1 && (size_t)(n - 1) * rb_max * 64 * (D / 2 + 4) * 4 > (size_t)WIDE_RING * 4 * PAGE * D * 2) --n;
  return n < 1 ? 1 : n;
}
// dynamic LDS of a launch: the ring, then the query operands of every row block
inline int wide_lds_bytes(int rb_max, int D) { return WIDE_RING * 4 * PAGE * D * 2 + rb_max * (D / 16) * 1024; }
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {  // s_waitcnt vmcnt(n), n <= 56, wave-uniform
  // vmcnt is split over bits 3:0 and 15:14 of the immediate (gfx9 encoding)
  switch (n >> 2) {
#define DAG_VM_CASE(q)                                                                         \
  case q:                                                                                       \
    switch (n & 3) {                                                                            \
      case 0: __builtin_amdgcn_s_waitcnt(0x0F70 | ((4 * q + 0) & 15) | (((4 * q + 0) >> 4) << 14)); break; \
      case 1: __builtin_amdgcn_s_waitcnt(0x0F70 | ((4 * q + 1) & 15) | (((4 * q + 1) >> 4) << 14)); break; \
      case 2: __builtin_amdgcn_s_waitcnt(0x0F70 | ((4 * q + 2) & 15) | (((4 * q + 2) >> 4) << 14)); break; \
      default: __builtin_amdgcn_s_waitcnt(0x0F70 | ((4 * q + 3) & 15) | (((4 * q + 3) >> 4) << 14)); break; \
    }                                                                                           \
    break;
    DAG_VM_CASE(0) DAG_VM_CASE(1) DAG_VM_CASE(2) DAG_VM_CASE(3) DAG_VM_CASE(4) DAG_VM_CASE(5) DAG_VM_CASE(6)
    DAG_VM_CASE(7) DAG_VM_CASE(8) DAG_VM_CASE(9) DAG_VM_CASE(10) DAG_VM_CASE(11) DAG_VM_CASE(12) DAG_VM_CASE(13)
#undef DAG_VM_CASE
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;  // vmcnt(0)
  }
}

template <int D>
__global__ void __launch_bounds__(WIDE_MAX_THREADS) __attribute__((amdgpu_waves_per_eu(3, 3))) k_decode_wide(DecodeArgs a) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
  constexpr int BB = wide_block_bytes<D>();       // bytes of a block in the ring: K page 0, K page 1, V page 0, V page 1
  constexpr int PB = PAGE * D * 2;                // bytes of one page of one kv head in a pool
  constexpr int LOADS = BB / 1024;                // wave-level loads per block
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int L = lane & 31, H = lane >> 5;
  // The first wide_shared workgroups take the shared items; the ones after them take the own
  // pages of one (branch, kv head, split) each, as a single row block whose waves (six at most,
  // the others leave at once) take the key blocks in turn: they follow the shared items in the
  // same launch and fill the compute units as those run out.
  const bool own = (int)blockIdx.x >= a.wide_shared;
#ifdef DAGATTN_ABL_NOOWN  // (development: timing of the shared items alone; results are wrong)
  if (own) return;
#endif
#ifdef DAGATTN_ABL_NOSHARED
  if (!own) return;
#endif
  int nw, nsub, rb, sub, split, hk, branch0, nrows, len, chunk;
  const int32_t* pages;
  float *po, *pml;
  if (!own) {
    nw = blockDim.x >> 6;
    nsub = nw / a.rb_max; rb = w % a.rb_max; sub = w / a.rb_max;
    int x = blockIdx.x;
    split = x % a.splits_a; x /= a.splits_a;
    hk = x % a.hkv;
    const int g = x / a.hkv;
    branch0 = a.group_branch_off[g];
    nrows = (a.group_branch_off[g + 1] - branch0) * a.G;
    pages = a.shared_pages + a.shared_page_off[g];
    len = a.shared_len[g];
    chunk = a.chunk_a;
    const size_t item = (((size_t)g * a.hkv + hk) * a.rb_max + rb) * a.splits_a + split;
    po = a.part_o_a + (item * 32 + L) * D;
    pml = a.part_ml_a + (item * 32 + L) * 2;
  } else {
    nw = min((int)(blockDim.x >> 6), WIDE_OWN_WAVES);
    if (w >= nw) return;
    nsub = nw; rb = 0; sub = w;
    int x = (int)blockIdx.x - a.wide_shared;
    const size_t item = (size_t)x;  // the order of k_decode's own items: (branch, kv head, split)
    split = x % a.splits_b; x /= a.splits_b;
    hk = x % a.hkv;
    branch0 = x / a.hkv;
    nrows = a.G;
    pages = a.branch_pages + a.branch_page_off[branch0];
    len = a.branch_len[branch0];
    chunk = a.chunk_b;
    po = a.part_o_b + (item * a.G + L) * D;
    pml = a.part_ml_b + (item * a.G + L) * 2;
  }
  const int npages = (len + PAGE - 1) / PAGE;
  const int p0 = split * chunk, p1 = min(p0 + chunk, npages);
  const int row = 32 * rb + L;
  const bool row_ok = row < nrows;
  const int rbm = own ? 1 : a.rb_max;  // row blocks of the workgroup
  if (p0 >= p1) {  // empty slice (the same for every wave of the workgroup): neutral partials
    if (row_ok && H == 0 && sub == 0) {
      pml[0] = -1e30f;
      pml[1] = 0.f;
    }
    return;
  }

  // The query operands of the row block live in LDS behind the ring (operand s of lane i at
  // (s 64 + i) 16 bytes), written by the block's first wave and read again for every key block:
  // with them in registers three waves would not fit on a SIMD.
  const uint32_t qbase = WIDE_RING * BB + rb * (D / 16) * 1024;
  if (sub == 0) {
    const int rr = row_ok ? row : 0;
    const int br = branch0 + rr / a.G, head = hk * a.G + rr % a.G;
    const uint16_t* qp = a.q + ((size_t)br * a.hq + head) * D + 8 * H;
    bf16x8 qreg[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qreg[s] = *(const bf16x8*)(qp + 16 * s);
#pragma unroll
    for (int s = 0; s < D / 16; ++s) *(bf16x8*)(ring + qbase + (s * 64 + lane) * 16) = qreg[s];
  }
  __builtin_amdgcn_s_waitcnt(0);  // (written before the first barrier of the block loop, which every wave passes before it reads them)

  // Loads of a block: piece j (0 .. LOADS - 1) = 1 KiB number j % (LOADS / 4) of {K page 0, K page 1,
  // V page 0, V page 1}[j / (LOADS / 4)]; wave w issues the pieces w, w + nw, ...  Every wave
  // issues the same number of loads per block (the last ones of some waves repeat a piece), so
  // that the number of loads a wave may leave in flight is the same for all.
  const int lpw = (LOADS + nw - 1) / nw;
  const int np = p1 - p0, nblk = (np + 1) / 2;
  int pgv = pages[p0 + min(lane, np - 1)];  // page ids, a 64-page window per register (as in k_decode)
  asm volatile("" ::"v"(pgv));             // arrived (a wait for it inside the loops would drain the ring's loads)
  int pgv_first = 0;                        // first page (relative) of the window in pgv
  // A V piece (32 dimensions x 16 keys) is fetched so that the 16 lanes which read an operand
  // together find it in 256 consecutive bytes: LDS position u of the piece holds dimension
  // 16 (u / 32) + u % 16, key half (u / 16) % 2 (a row of the pool has 32 bytes: read as it lies,
  // those lanes would hit every bank twice).
  const uint32_t vsrc = (2 * (16 * (lane / 32) + lane % 16) + (lane / 16) % 2) * 16;
  auto issue_block = [&](int b) {
    const int pr = 2 * b;
    if (pr - pgv_first >= 64) {  // next window (blocks are issued in order)
      pgv_first += 64;
      pgv = pages[p0 + min(pgv_first + lane, np - 1)];
      asm volatile("" ::"v"(pgv));
    }
    const int pg0 = __builtin_amdgcn_readlane(pgv, (pr - pgv_first) & 63);
    const int pg1 = __builtin_amdgcn_readlane(pgv, (min(pr + 1, np - 1) - pgv_first) & 63);
    const size_t base0 = ((size_t)pg0 * a.hkv + hk) * (size_t)PB, base1 = ((size_t)pg1 * a.hkv + hk) * (size_t)PB;
    unsigned char* slot = ring + (b % WIDE_RING) * BB;
    for (int i = 0; i < lpw; ++i) {
      const int j = min(w + i * nw, LOADS - 1);
      const int part = j / (LOADS / 4), piece = j % (LOADS / 4);
      const unsigned char* src = (const unsigned char*)(part < 2 ? a.k_pool : a.v_pool) + ((part & 1) ? base1 : base0) +
                                 piece * 1024 + (part < 2 ? lane * 16 : vsrc);
      __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) const void*)src,
                                       (__attribute__((address_space(3))) void*)(slot + j * 1024), 16, 0, 0);
    }
  };

  const int kr = key_of_row(L);
  // operand addresses inside a block: K[s] = chunk 2 s + H of key pi(L); V[page][db] = keys 8 H .. of
  // dimension 32 db + L, which lies at position 32 (L / 16) + 16 H + L % 16 of its 1 KiB piece
  const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)ring;
  const uint32_t koff = (kr >> 4) * PB + H * (PAGE * 16) + (kr & 15) * 16;
  const uint32_t voff = 2 * PB + (L / 16) * 512 + H * 256 + (L % 16) * 16;

  f32x16 O[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
  float m = -1e30f, l = 0.f;
  bf16x8 qcur[D / 16];
  auto qop = [&](int s) { return qcur[s]; };

  // Operands come from LDS right before their product (inline assembly: for plain LDS reads the
  // compiler would first wait for every global-to-LDS load in flight).  Nothing else happens
  // between a read and its wait: the compiler does not know that the registers are not there yet
  // (it might spill one in between).
  bf16x8 pb0, pb1;
  auto score_phase = [&](int b) __attribute__((always_inline)) {  // scores and probabilities of block b
    const uint32_t sb = ring0 + (b % WIDE_RING) * BB;
    bf16x8 kop[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(kop[s]) : "v"(sb + koff), "n"(s * 2 * PAGE * 16));
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(qcur[s]) : "v"(ring0 + qbase + lane * 16), "n"(s * 1024));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" : "+v"(kop[s]), "+v"(qcur[s]));
    block_scores<D>(kop, qop, O, m, l, a.sc, a.th, (p0 + 2 * b) * PAGE, len, len, H, pb0, pb1);
  };
  auto value_phase = [&](int b) __attribute__((always_inline)) {  // O += V^T P^T of block b
    const uint32_t sb = ring0 + (b % WIDE_RING) * BB;
    bf16x8 v0[D / 32], v1[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v0[db]) : "v"(sb + voff), "n"(db * 32 * PAGE * 2));
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v1[db]) : "v"(sb + voff), "n"(PB + db * 32 * PAGE * 2));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int db = 0; db < D / 32; ++db) asm volatile("" : "+v"(v0[db]), "+v"(v1[db]));
    if ((p0 + 2 * b) * PAGE + 32 > len) clear_unused_values<D>(v0, v1, (p0 + 2 * b) * PAGE, len, H);
    block_pv<D>(v0, v1, pb0, pb1, O);
  };
  // The barrier of a round puts every wave at the same point, and waves that then all read LDS,
  // all run their score MFMAs, all do the softmax arithmetic at the same time leave each of those
  // units idle for most of the round.  When the ring holds three rounds, the waves with an odd
  // `sub` therefore run half a block behind: after the barrier they first finish the block of the
  // round before (its values), then take the scores of their new block, while the others do it
  // the usual way round; a round's slots are then refilled a round later.
  const bool skew = WIDE_RING >= 3 * nsub;
  const bool late = skew && (sub & 1);
  const int keep = skew ? 1 : 0;  // rounds before the current one whose blocks are still read
  int issued = 0;
  for (; issued < nblk && issued < WIDE_RING - keep * nsub; ++issued) issue_block(issued);
  const int nrounds = (nblk + nsub - 1) / nsub;
  auto round_sync = [&](int r) __attribute__((always_inline)) {
    // this wave's loads of the round's blocks have landed when at most the loads of the blocks after them are in flight
    wait_vmcnt_dyn(max(issued - min((r + 1) * nsub, nblk), 0) * lpw);
    __builtin_amdgcn_s_barrier();  // the round's blocks are complete; every wave has finished the round before (late ones: its scores)
    asm volatile("" ::: "memory");
    // the next loads, into the slots that nobody reads any more
    for (; issued < nblk && issued - (r - keep) * nsub < WIDE_RING; ++issued) issue_block(issued);
  };
  // (every wave passes one barrier per round, the late ones between the two halves of a block)
  round_sync(0);
  for (int r = 0; r < nrounds; ++r) {
    const int b = r * nsub + sub;
    const bool mine = b < nblk;
    if (mine) score_phase(b);
    if (late && r + 1 < nrounds) round_sync(r + 1);
    if (mine) value_phase(b);
    if (!late && r + 1 < nrounds) round_sync(r + 1);
  }

  // The waves of a row block put their accumulators together: waves 1 .. nsub - 1 leave theirs in
  // LDS (the ring is free once every load has landed and every wave is past its last block), lane
  // by lane, and wave 0 adds them in the order of `sub` with the usual change of reference maximum.
  if (nsub > 1) {
    wait_vmcnt_dyn(0);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    float* const slot = (float*)ring + ((size_t)((sub - 1) * rbm + rb) * 64 + lane) * (D / 2 + 4);
    if (sub > 0) {
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(f32x4*)(slot + 16 * db + 4 * r4) = f32x4{O[db][4 * r4], O[db][4 * r4 + 1], O[db][4 * r4 + 2], O[db][4 * r4 + 3]};
      slot[D / 2] = m;
      slot[D / 2 + 1] = l;
    }
    __syncthreads();
    if (sub > 0) return;
    for (int s2 = 1; s2 < nsub; ++s2) {
      const float* const other = (const float*)ring + ((size_t)((s2 - 1) * rbm + rb) * 64 + lane) * (D / 2 + 4);
      const float m2 = other[D / 2], l2 = other[D / 2 + 1];
      const float m_new = fmaxf(m, m2);
      const float a1 = __builtin_amdgcn_exp2f((m - m_new) * a.sc), a2 = __builtin_amdgcn_exp2f((m2 - m_new) * a.sc);
      m = m_new;
      l = l * a1 + l2 * a2;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 o2 = *(const f32x4*)(other + 16 * db + 4 * r4);
#pragma unroll
          for (int e = 0; e < 4; ++e) O[db][4 * r4 + e] = O[db][4 * r4 + e] * a1 + o2[e] * a2;
        }
    }
  }

  const float l_tot = l + __shfl_xor(l, 32);
  if (row_ok) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 o = {O[db][4 * r4], O[db][4 * r4 + 1], O[db][4 * r4 + 2], O[db][4 * r4 + 3]};
        *(f32x4*)(po + 32 * db + 8 * r4 + 4 * H) = o;
      }
    if (H == 0) {
      pml[0] = m;
      pml[1] = l_tot;
    }
  }
}

// One wave per (branch, query head): log-sum-exp combination of its partials.
template <int D>
__global__ void __launch_bounds__(64) k_decode_merge(DecodeArgs a) {
  const int r = blockIdx.x / a.hq, head = blockIdx.x % a.hq;
  const int hk = head / a.G, j = head % a.G;
  const int lane = threadIdx.x;
  const int g = dag_find_segment(a.group_branch_off, a.n_groups, r);
  const int row = (r - a.group_branch_off[g]) * a.G + j;
  const int rb = row >> 5, rr = row & 31;
  const size_t ia0 = (((size_t)g * a.hkv + hk) * a.rb_max + rb) * a.splits_a;
  const size_t ib0 = ((size_t)r * a.hkv + hk) * a.splits_b;
  constexpr int PER = D / 64;  // output elements per lane
  const int np = a.splits_a + a.splits_b;
  // partial p of this (branch, head): shared split p, then own split p - splits_a
  auto ml_of = [&](int p) {
    return p < a.splits_a ? a.part_ml_a + ((ia0 + p) * 32 + rr) * 2 : a.part_ml_b + ((ib0 + (p - a.splits_a)) * a.G + j) * 2;
  };
  auto o_of = [&](int p) {
    return p < a.splits_a ? a.part_o_a + ((ia0 + p) * 32 + rr) * D : a.part_o_b + ((ib0 + (p - a.splits_a)) * a.G + j) * D;
  };
  float acc[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) acc[e] = 0.f;
  // The reference maximum first (64 partials at a time, one per lane, so that their loads are in
  // flight together), then the weighted sums in the fixed order of the partials: the weights of
  // a group of 64 come from the lanes, and the loads of the partial outputs do not depend on
  // each other (a partial without a visible key has l = 0 and weight 0; what it holds is read
  // and dropped).
  float mx = -1e30f;
  for (int p0 = 0; p0 < np; p0 += 64) {
    const float mv = p0 + lane < np ? ml_of(p0 + lane)[0] : -1e30f;
    mx = fmaxf(mx, mv);
  }
#pragma unroll
  for (int off = 32; off; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float lsum = 0.f;
  for (int p0 = 0; p0 < np; p0 += 64) {
    float wl = 0.f, wgt = 0.f;
    if (p0 + lane < np) {
      const float* ml = ml_of(p0 + lane);
      const float ls = ml[1];
      if (ls > 0.f) {
        wgt = __builtin_amdgcn_exp2f((ml[0] - mx) * a.sc);
        wl = ls * wgt;
      }
    }
    const int n = min(64, np - p0);
#pragma unroll 4
    for (int i = 0; i < n; ++i) {
      const float wi = __shfl(wgt, i);
      lsum += __shfl(wl, i);
      const float* o = o_of(p0 + i) + lane * PER;  // (read in any case, so that the loads of several partials overlap)
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const float x = o[e];
        acc[e] += wi != 0.f ? wi * x : 0.f;
      }
    }
  }
  const float inv = 1.f / lsum;
  uint16_t* o = a.out + ((size_t)r * a.hq + head) * D + lane * PER;
  if (PER == 2) {
    *(uint32_t*)o = dag_pack_bf2(acc[0] * inv, acc[PER - 1] * inv);
  } else {
    o[0] = (uint16_t)dag_f2bf(acc[0] * inv);
  }
}

// One block per live branch: rotate the new key at the branch's adaptive position and scatter
// key and value into the pool formats.  The angles depend on the position and the frequency index
// only, so D / 2 threads compute them once (fp64) and the block shares them through LDS.
__global__ void __launch_bounds__(256) k_kv_append(const int32_t* branch_page_off, const int32_t* branch_pages,
                                                   const int32_t* branch_len, const int32_t* branch_pos,
                                                   const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                                                   uint16_t* v_pool, int hkv, int D, float theta) {
  __shared__ float s_cos[64], s_sin[64];  // D / 2 <= 64 (the entry point admits head_dim 64 and 128 only)
  const int r = blockIdx.x;
  const int idx = branch_len[r] - 1;
  if (idx < 0) return;
  const int page = branch_pages[branch_page_off[r] + idx / PAGE];
  const int slot = idx % PAGE;
  const int half = D / 2;
  if ((int)threadIdx.x < half) {
    double sn, cs;
    sincos((double)branch_pos[r] * pow((double)theta, -2.0 * (double)threadIdx.x / (double)D), &sn, &cs);
    s_cos[threadIdx.x] = (float)cs;
    s_sin[threadIdx.x] = (float)sn;
  }
  __syncthreads();
  for (int x = threadIdx.x; x < hkv * half; x += blockDim.x) {
    const int h = x / half, mi = x % half;
    const size_t src = ((size_t)r * hkv + h) * D;
    const float lo = __uint_as_float((uint32_t)k_new[src + mi] << 16);
    const float hi = __uint_as_float((uint32_t)k_new[src + mi + half] << 16);
    const float c = s_cos[mi], s = s_sin[mi];
    const size_t pb = ((size_t)page * hkv + h) * (size_t)(D * PAGE);
    const int d0 = mi, d1 = mi + half;
    k_pool[pb + (size_t)(d0 >> 3) * (PAGE * 8) + slot * 8 + (d0 & 7)] = (uint16_t)dag_f2bf(lo * c - hi * s);
    k_pool[pb + (size_t)(d1 >> 3) * (PAGE * 8) + slot * 8 + (d1 & 7)] = (uint16_t)dag_f2bf(hi * c + lo * s);
    v_pool[pb + (size_t)d0 * PAGE + slot] = v_new[src + d0];
    v_pool[pb + (size_t)d1 * PAGE + slot] = v_new[src + d1];
  }
}

struct DecodePlan {
  int rb_max, chunk_a, splits_a, chunk_b, splits_b, items_a, items_b;
  bool wide;  // shared items by k_decode_wide (one workgroup per group, kv head and split)
  size_t off_o_a, off_ml_a, off_o_b, off_ml_b, bytes;
};

// Development knobs (pages per decode work item), read from the environment once per process;
// 0 = not set, the split sizes then follow the shape of the batch.
struct DecodeKnobs {
  int chunk_a, chunk_b, chunk_seg;
};
int env_int(const char* name) {
  const char* s = getenv(name);
  if (!s || !*s) return 0;
  const int v = atoi(s);
  return v > 0 ? v : 0;
}
const DecodeKnobs& decode_knobs() {
  static const DecodeKnobs k = {env_int("DAGATTN_DECODE_CHUNK_A"), env_int("DAGATTN_DECODE_CHUNK_B"),
                                env_int("DAGATTN_DECODE_CHUNK_SEG")};
  return k;
}

// Split sizes: slices as long as the batch allows (every work item pays a start-up latency and
// writes a partial, so fewer and longer items stream better) while still giving the GPU about two
// waves per SIMD; both even so that a 32-key block never straddles a split.
int make_plan(const dag_decode_desc_t* d, int hq, int hkv, int D, DecodePlan* p) {
  if (!d) return DAG_ERR_NULL;
  if (d->n_groups < 0 || d->n_live < 0 || d->max_shared_pages < 0 || d->max_branch_pages < 0 || d->max_group_size < 0)
    return DAG_ERR_BAD_LEN;
  if (d->page_size != PAGE) return DAG_ERR_UNSUPPORTED;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || hq / hkv > 32) return DAG_ERR_UNSUPPORTED;
  if (D != 64 && D != 128) return DAG_ERR_UNSUPPORTED;
  const int G = hq / hkv;
  p->rb_max = (int)dag_ceil_div((int64_t)d->max_group_size * G, 32);
  if (p->rb_max < 1) p->rb_max = 1;
  const int64_t base_a = (int64_t)d->n_groups * hkv * p->rb_max;
  const int64_t base_b = (int64_t)d->n_live * hkv;
  const DecodeKnobs& knobs = decode_knobs();
  int ca = knobs.chunk_a ? knobs.chunk_a : 128, cb = knobs.chunk_b ? knobs.chunk_b : 64;
  ca += ca & 1;
  cb += cb & 1;
  p->wide = p->rb_max >= 2 && p->rb_max <= WIDE_MAX_WAVES;
  if (!knobs.chunk_a) {
    if (p->wide)  // about one workgroup per compute unit
      while (ca > 8 && (int64_t)d->n_groups * hkv * dag_ceil_div(d->max_shared_pages, ca) < 256) ca /= 2;
    else
      while (ca > 8 && base_a * dag_ceil_div(d->max_shared_pages, ca) < 512) ca /= 2;
  }
  if (!knobs.chunk_b)  // (wide: the own items are workgroups of several waves, about two per compute unit)
    while (cb > 4 && base_b * dag_ceil_div(d->max_branch_pages, cb) < (p->wide ? 512 : 1024)) cb /= 2;
  p->chunk_a = ca;
  p->chunk_b = cb;
  p->splits_a = d->max_shared_pages > 0 ? (int)dag_ceil_div(d->max_shared_pages, ca) : 0;
  p->splits_b = d->max_branch_pages > 0 ? (int)dag_ceil_div(d->max_branch_pages, cb) : 0;
  const int64_t ia = base_a * p->splits_a, ib = base_b * p->splits_b;
  if (ia + ib > INT32_MAX) return DAG_ERR_UNSUPPORTED;
  p->items_a = (int)ia;
  p->items_b = (int)ib;
  size_t off = 0;
  p->off_o_a = off;  off += dag_align_up((size_t)ia * 32 * D * 4, 256);
  p->off_ml_a = off; off += dag_align_up((size_t)ia * 32 * 2 * 4, 256);
  p->off_o_b = off;  off += dag_align_up((size_t)ib * G * D * 4, 256);
  p->off_ml_b = off; off += dag_align_up((size_t)ib * G * 2 * 4, 256);
  p->bytes = off + 256;
  return DAG_OK;
}

}  // namespace

extern "C" size_t dag_decode_workspace_bytes(const dag_decode_desc_t* desc, int32_t hq, int32_t hkv,
                                             int32_t head_dim) {
  DecodePlan p;
  if (make_plan(desc, hq, hkv, head_dim, &p) != DAG_OK) return 0;
  return p.bytes;
}

extern "C" int dag_kv_append_rope(const dag_decode_desc_t* d, const void* k_new, const void* v_new, void* k_pool,
                                  void* v_pool, int32_t hkv, int32_t head_dim, float theta, void* stream_) {
  if (!d) return DAG_ERR_NULL;
  if (d->n_live < 0) return DAG_ERR_BAD_LEN;
  if (d->page_size != PAGE) return DAG_ERR_UNSUPPORTED;
  if (hkv < 1 || (head_dim != 64 && head_dim != 128) || !(theta > 0.f)) return DAG_ERR_UNSUPPORTED;
  if (d->n_live == 0) return DAG_OK;
  if (!k_new || !v_new || !k_pool || !v_pool || !d->branch_page_off || !d->branch_pages || !d->branch_len ||
      !d->branch_pos)
    return DAG_ERR_NULL;
  hipLaunchKernelGGL(k_kv_append, dim3(d->n_live), dim3(256), 0, (hipStream_t)stream_, d->branch_page_off,
                     d->branch_pages, d->branch_len, d->branch_pos, (const uint16_t*)k_new, (const uint16_t*)v_new,
                     (uint16_t*)k_pool, (uint16_t*)v_pool, hkv, head_dim, theta);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

namespace {

// Scratch of dag_attn_decode_static: the partial results live in this array instead of a caller
// workspace.  Every GPU the library runs on holds its own copy at its own address until the
// process ends; host code never uses the array's name as an address, only what
// hipGetSymbolAddress returned for the current device.
static __device__ __align__(256) unsigned char scratch[DAG_DECODE_STATIC_SCRATCH_BYTES];

int static_scratch(void** out) {
  constexpr int MAX_DEV = 64;
  static void* ptr[MAX_DEV];
  static bool ready[MAX_DEV];
  static std::mutex mu;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return DAG_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ready[dev]) {  // once per device, with that device current
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DAG_ERR_HIP;
    ptr[dev] = p;
    ready[dev] = true;
  }
  *out = ptr[dev];
  return DAG_OK;
}

// static_ws: the partials go to the library's own scratch array (ws / ws_bytes ignored).
int decode_impl(const dag_decode_desc_t* d, const void* q, const void* k_pool, const void* v_pool, void* out,
                int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale, void* ws, size_t ws_bytes,
                void* stream_, bool static_ws) {
  DecodePlan p;
  const int rc = make_plan(d, hq, hkv, head_dim, &p);
  if (rc != DAG_OK) return rc;
  if (d->n_live == 0) return DAG_OK;
  if (!q || !k_pool || !v_pool || !out || !d->group_branch_off || !d->branch_page_off || !d->branch_pages ||
      !d->branch_len)
    return DAG_ERR_NULL;
  if (d->n_groups < 1) return DAG_ERR_BAD_LEN;
  if (p.items_a > 0 && (!d->shared_page_off || !d->shared_pages || !d->shared_len)) return DAG_ERR_NULL;
  if (p.items_a + p.items_b == 0) return DAG_ERR_BAD_LEN;  // a query needs at least its own token
  if (!dag_aligned16(q) || !dag_aligned16(k_pool) || !dag_aligned16(v_pool) || !dag_aligned16(out))
    return DAG_ERR_ALIGN;
  if (static_ws) {
    if (p.bytes > (size_t)DAG_DECODE_STATIC_SCRATCH_BYTES) return DAG_ERR_WORKSPACE;
    const int rs = static_scratch(&ws);
    if (rs != DAG_OK) return rs;
  } else if (!ws || ws_bytes < p.bytes) {
    return DAG_ERR_WORKSPACE;
  }
  char* base = (char*)dag_align_up((size_t)(uintptr_t)ws, 256);
  DecodeArgs a;
  a.group_branch_off = d->group_branch_off;
  a.shared_page_off = d->shared_page_off;
  a.shared_pages = d->shared_pages;
  a.shared_len = d->shared_len;
  a.branch_page_off = d->branch_page_off;
  a.branch_pages = d->branch_pages;
  a.branch_len = d->branch_len;
  a.q = (const uint16_t*)q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.out = (uint16_t*)out;
  a.part_o_a = (float*)(base + p.off_o_a);
  a.part_ml_a = (float*)(base + p.off_ml_a);
  a.part_o_b = (float*)(base + p.off_o_b);
  a.part_ml_b = (float*)(base + p.off_ml_b);
  a.n_groups = d->n_groups;
  a.n_live = d->n_live;
  a.hq = hq;
  a.hkv = hkv;
  a.G = hq / hkv;
  a.rb_max = p.rb_max;
  a.chunk_a = p.chunk_a;
  a.splits_a = p.splits_a;
  a.chunk_b = p.chunk_b;
  a.splits_b = p.splits_b;
  a.items_a = p.items_a;
  a.items_b = p.items_b;
  a.scale = softmax_scale;
  a.sc = softmax_scale * 1.4426950408889634f;
  a.th = 8.f / a.sc;
  hipStream_t stream = (hipStream_t)stream_;
  const unsigned nout = (unsigned)(d->n_live * hq);
  a.item_base = 0;
  unsigned items = (unsigned)(p.items_a + p.items_b);
  if (p.wide && p.items_a > 0) {
    // Wide sibling groups: one launch of workgroups that share their K/V blocks through LDS, the
    // shared items first (one workgroup streams a slice of the shared pages once for all rows),
    // the own items behind them.
    const unsigned shared_wgs = (unsigned)(d->n_groups * hkv * p.splits_a);
    const unsigned threads = 64u * (unsigned)(p.rb_max * wide_nsub(p.rb_max, head_dim));
    const int sm = wide_lds_bytes(p.rb_max, head_dim);
    a.wide_shared = (int)shared_wgs;
    if (head_dim == 128) {
      if (hipFuncSetAttribute((const void*)k_decode_wide<128>, hipFuncAttributeMaxDynamicSharedMemorySize, sm) != hipSuccess)
        return DAG_ERR_HIP;
      hipLaunchKernelGGL(k_decode_wide<128>, dim3(shared_wgs + (unsigned)p.items_b), dim3(threads), sm, stream, a);
    } else {
      if (hipFuncSetAttribute((const void*)k_decode_wide<64>, hipFuncAttributeMaxDynamicSharedMemorySize, sm) != hipSuccess)
        return DAG_ERR_HIP;
      hipLaunchKernelGGL(k_decode_wide<64>, dim3(shared_wgs + (unsigned)p.items_b), dim3(threads), sm, stream, a);
    }
    DAG_LAUNCH_CHECK();
    items = 0;
  }
  if (items > 0) {
    if (head_dim == 128) hipLaunchKernelGGL(k_decode<128>, dim3(items), dim3(64), 0, stream, a);
    else hipLaunchKernelGGL(k_decode<64>, dim3(items), dim3(64), 0, stream, a);
    DAG_LAUNCH_CHECK();
  }
  if (head_dim == 128) hipLaunchKernelGGL(k_decode_merge<128>, dim3(nout), dim3(64), 0, stream, a);
  else hipLaunchKernelGGL(k_decode_merge<64>, dim3(nout), dim3(64), 0, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

}  // namespace

extern "C" int dag_attn_decode(const dag_decode_desc_t* d, const void* q, const void* k_pool, const void* v_pool,
                               void* out, int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale, void* ws,
                               size_t ws_bytes, void* stream_) {
  return decode_impl(d, q, k_pool, v_pool, out, hq, hkv, head_dim, softmax_scale, ws, ws_bytes, stream_, false);
}

extern "C" int dag_attn_decode_static(const dag_decode_desc_t* d, const void* q, const void* k_pool,
                                      const void* v_pool, void* out, int32_t hq, int32_t hkv, int32_t head_dim,
                                      float softmax_scale, void* stream_) {
  return decode_impl(d, q, k_pool, v_pool, out, hq, hkv, head_dim, softmax_scale, nullptr, 0, stream_, true);
}

namespace {

struct SegPlan {
  int rb_max, chunk, splits;
  long items;  // bound on the work items (per kv head)
  size_t off_o, off_ml, off_items, off_total, off_nsplit, bytes;
};

// One split size for all segments (their lengths live in device memory): as long as possible
// while the launch still has about a thousand items if every segment were the longest one.
int make_seg_plan(const dag_decode_seg_desc_t* d, int hq, int hkv, int D, SegPlan* p) {
  if (!d) return DAG_ERR_NULL;
  if (d->n_live < 0 || d->n_segments < 0 || d->max_seg_pages < 0 || d->max_readers < 0 || d->total_readers < 0)
    return DAG_ERR_BAD_LEN;
  if (d->page_size != PAGE) return DAG_ERR_UNSUPPORTED;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || hq / hkv > 32) return DAG_ERR_UNSUPPORTED;
  if (D != 64 && D != 128) return DAG_ERR_UNSUPPORTED;
  const int G = hq / hkv;
  p->rb_max = (int)dag_ceil_div((int64_t)d->max_readers * G, 32);
  if (p->rb_max < 1) p->rb_max = 1;
  const int knob = decode_knobs().chunk_seg;
  int c = knob ? knob : 128;
  c += c & 1;
  const int64_t base = (int64_t)d->n_segments * hkv * p->rb_max;
  if (!knob)
    while (c > 8 && base * dag_ceil_div(d->max_seg_pages, c) < 1024) c /= 2;
  p->chunk = c;
  p->splits = d->max_seg_pages > 0 ? (int)dag_ceil_div(d->max_seg_pages, c) : 0;
  const int64_t items = (int64_t)d->n_segments * p->rb_max * p->splits;
  if (items * hkv > INT32_MAX) return DAG_ERR_UNSUPPORTED;
  p->items = (long)items;
  size_t off = 0;
  const size_t rows = (size_t)p->splits * (size_t)d->total_readers * hq;
  if (rows > (size_t)INT32_MAX) return DAG_ERR_UNSUPPORTED;
  p->off_o = off;  off += dag_align_up(rows * D * 4, 256);
  p->off_ml = off; off += dag_align_up(rows * 2 * 4, 256);
  p->off_items = off;  off += dag_align_up((size_t)items * sizeof(SegItem), 256);
  p->off_total = off;  off += 256;
  p->off_nsplit = off; off += dag_align_up((size_t)d->total_readers * 4, 256);
  p->bytes = off + 256;
  return DAG_OK;
}

}  // namespace

extern "C" size_t dag_decode_segments_workspace_bytes(const dag_decode_seg_desc_t* desc, int32_t hq, int32_t hkv,
                                                      int32_t head_dim) {
  SegPlan p;
  if (make_seg_plan(desc, hq, hkv, head_dim, &p) != DAG_OK) return 0;
  return p.bytes;
}

extern "C" int dag_attn_decode_segments(const dag_decode_seg_desc_t* d, const void* q, const void* k_pool,
                                        const void* v_pool, void* out, int32_t hq, int32_t hkv, int32_t head_dim,
                                        float softmax_scale, void* ws, size_t ws_bytes, void* stream_) {
  SegPlan p;
  const int rc = make_seg_plan(d, hq, hkv, head_dim, &p);
  if (rc != DAG_OK) return rc;
  if (d->n_live == 0) return DAG_OK;
  if (!q || !k_pool || !v_pool || !out || !d->branch_entry_off || !d->branch_entries) return DAG_ERR_NULL;
  if (d->n_segments > 0 &&
      (!d->seg_page_off || !d->seg_pages || !d->seg_len || !d->seg_reader_off || !d->seg_readers))
    return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k_pool) || !dag_aligned16(v_pool) || !dag_aligned16(out))
    return DAG_ERR_ALIGN;
  if (!ws || ws_bytes < p.bytes) return DAG_ERR_WORKSPACE;
  char* base = (char*)dag_align_up((size_t)(uintptr_t)ws, 256);
  SegArgs a;
  a.seg_page_off = d->seg_page_off;
  a.seg_pages = d->seg_pages;
  a.seg_len = d->seg_len;
  a.seg_reader_off = d->seg_reader_off;
  a.seg_readers = d->seg_readers;
  a.seg_reader_len = d->seg_reader_len;
  a.branch_entry_off = d->branch_entry_off;
  a.branch_entries = d->branch_entries;
  a.q = (const uint16_t*)q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.out = (uint16_t*)out;
  a.part_o = (float*)(base + p.off_o);
  a.part_ml = (float*)(base + p.off_ml);
  a.items = (SegItem*)(base + p.off_items);
  a.item_total = (int32_t*)(base + p.off_total);
  a.entry_nsplit = (int32_t*)(base + p.off_nsplit);
  a.item_cap = (int)p.items;
  a.n_segments = d->n_segments;
  a.n_live = d->n_live;
  a.hq = hq;
  a.hkv = hkv;
  a.G = hq / hkv;
  a.rb_max = p.rb_max;
  a.chunk = p.chunk;
  a.splits = p.splits;
  a.total_readers = d->total_readers;
  a.sc = softmax_scale * 1.4426950408889634f;
  a.th = 8.f / a.sc;
  hipStream_t stream = (hipStream_t)stream_;
  if (p.items > 0) {
    hipLaunchKernelGGL(k_seg_plan, dim3(1), dim3(PLAN_THREADS), 0, stream, a);
    DAG_LAUNCH_CHECK();
    const unsigned grid = (unsigned)(p.items * hkv);
    if (head_dim == 128) hipLaunchKernelGGL(k_decode_seg<128>, dim3(grid), dim3(64), 0, stream, a);
    else hipLaunchKernelGGL(k_decode_seg<64>, dim3(grid), dim3(64), 0, stream, a);
    DAG_LAUNCH_CHECK();
  }
  const unsigned nout = (unsigned)(d->n_live * hq);
  if (head_dim == 128) hipLaunchKernelGGL(k_decode_seg_merge<128>, dim3(nout), dim3(64), 0, stream, a);
  else hipLaunchKernelGGL(k_decode_seg_merge<64>, dim3(nout), dim3(64), 0, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}
