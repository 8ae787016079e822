// Backward of the DAG-masked prefill attention (the paper fine-tunes through the mask of Eq. 3,
// section 4.2): with P = softmax_row(scale Q K^T + M), O = P V and the incoming gradient dO,
//     delta_i = sum_d dO_id O_id,   dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),
//     dQ = scale dS K,   dK = scale dS^T Q        (a KV head sums over its query heads).
// P is recomputed from the forward's log-sum-exp; the block map of the forward skips the tiles
// without a visible pair.  bf16 operands on the 32x32x16 MFMA, fp32 accumulation.  The kernels:
//   k_bwd_delta   delta and -lse log2(e) per (token, query head)
//   k_bwd_tokvis, k_bwd_weights, k_bwd_order   small tables: first visibility word per token; weight
//                 and launch rank of the key-tile pairs (the dK/dV workgroups start heaviest first)
//   k_bwd_dq2     head dimension 128: one workgroup per (64-row query tile, KV head, four of its
//                 query heads), eight waves; the K / V tiles of the tile's row of the forward's
//                 FULL-first CSR stream through an LDS ring and every tile is a fixed sequence of
//                 48 slots (described at the kernel).  The heads that the groups of four leave
//                 over (G not a multiple of four) run as k_bwd_dq2<true>: one head on four
//                 consecutive query tiles per workgroup, with tile lists from k_bwd_wide_rows
//   k_bwd_dkv2    head dimension 128: one workgroup per (pair of 64-key tiles, KV head), four
//                 waves; the Q / dO tiles of the query tiles that see the pair stream through an LDS
//                 ring, one (tile, query head) = 64 slots (described at the kernel); nothing is
//                 accumulated through atomics, so the results do not depend on the order of execution
//   k_bwd_dq, k_bwd_dkv   the first versions (tiles staged through registers, compiler-scheduled):
//                 head dimension 64, and inside the two kernels above the "general walk" over
//                 masked tiles of sequences with more than one visibility word per node
// Register layout of a 32x32 MFMA result C = A B:  lane (L, H) = (lane % 32, lane / 32) holds
// column L and the 16 rows rho_H(e) = 8 (e / 4) + 4 H + e % 4.  A result is used again as the B
// operand of the next product (contraction over its rows) straight from the registers; the A
// operand of that product is then gathered from LDS in the same row order.
// Those A operands are transposed tiles (K^T for dQ; Q^T and dO^T for dK and dV): they are read
// from the row-major tiles in LDS with the transposing LDS load of gfx950, two 8-byte reads per
// operand, in the row order rho asks for.
// fp32 inputs take the plain kernels at the end of the file (the accuracy path).
#include <stdlib.h>
#include <type_traits>

#include "common.h"

namespace {

constexpr int BM = 64, BN = 64;  // tile shape of the bf16 block map
constexpr float LOG2E = 1.4426950408889634f;

struct BwdArgs {
  const uint16_t *q, *k, *v, *out, *dout;
  const float* lse;
  uint16_t *dq, *dk, *dv;
  float* delta;  // [T][hq]
  float* nlse2;  // [T][hq]  -lse log2(e)
  int32_t *kt_weight, *kt_order;        // [total key tiles] launch order of the dK/dV workgroups
  uint64_t* tok_vis0;                   // [T] first visibility word of every token's node
  int total_ktiles;
  const int32_t *cu_seqlens, *node_start, *tok_node, *qtile_start, *ktile_start;
  const int32_t* qtile_order;  // the forward's launch order: query tiles by descending number of visible key tiles
  const int32_t* qtile_desc;   // [launch slot][8]: token offset and length of the sequence, first row of the tile, CSR row start,
                               // tiles in the row, leading tiles without mask (FULL, not reaching past the end), node offset, -
  const int32_t* qtile_col;    // CSR of the visible key tiles of every query tile, the FULL ones first
  const uint8_t* qtile_flag;
  const uint64_t* node_vis;
  const int64_t* block_map_off;
  const uint8_t* block_map;
  int n_seqs, W, hq, hkv, G;
  long total_rows;  // T * hq
  float scale, sc;  // sc = scale * log2(e)
  // dQ: heads 0 .. dq_narrow - 1 of a KV head run four at a time on one query tile, the others one
  // at a time on four query tiles (k_bwd_dq2<true>), whose tile lists k_bwd_wide_rows writes: the
  // list of the tiles 4 c .. 4 c + 3 of a sequence lies where row 4 c of its dense block map does
  int dq_narrow;
  int total_qtiles;
  int32_t* wide_col;    // [dense map] key tiles that one of the four query tiles sees, those that all four see in full first
  uint8_t* wide_flag;   // [dense map] block-map entries of the four query tiles, two bits each
  int32_t *wide_n, *wide_nfast;  // [total query tiles] length of the list, leading entries without tests (at every fourth tile)
  int32_t* wide_list;   // [total query tiles + 1] the first tiles of the groups of four, sequence after sequence; last element: their number
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ int rho(int e, int H) { return 8 * (e >> 2) + 4 * H + (e & 3); }

__device__ __forceinline__ bf16x8 pack8(const float* x) {
  typedef __attribute__((ext_vector_type(8))) float f32x8;
  const f32x8 f = {x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7]};
  return __builtin_convertvector(f, bf16x8);
}

// Eq. 3 for a (query token i of node ni, key token j of node nj) pair of one sequence.  With at
// most 64 nodes per sequence (one visibility word) the test is a few selects, no branch and no load.
__device__ __forceinline__ bool visible(const BwdArgs& a, int nbase, int ni, int i, int nj, int j, uint64_t vis0) {
  if (a.W == 1) {
    const bool anc = (vis0 >> (nj & 63)) & 1u;
    return nj == ni ? j <= i : anc;
  }
  if (nj == ni) return j <= i;
  const uint64_t w = nj < 64 ? vis0 : a.node_vis[(int64_t)(nbase + ni) * a.W + (nj >> 6)];
  return (w >> (nj & 63)) & 1u;
}

// Tables kept in LDS per workgroup hold this many tiles (262,144 tokens); longer sequences read the
// rest from global memory.  (A build with a small DAG_BWD_LDS_TILES runs the tests through that path.)
#ifndef DAG_BWD_LDS_TILES
#define DAG_BWD_LDS_TILES 4096
#endif
constexpr int MAX_QT_LDS = DAG_BWD_LDS_TILES;  // query tiles of a sequence whose block-map column is kept in LDS

// A operand of a product whose contraction runs over the ROWS of a row-major LDS tile (K^T for dQ;
// Q^T and dO^T for dK and dV), read with the transposing LDS load of gfx950 (ds_read_b64_tr_b16):
// within 16 consecutive lanes, lane p hands in the address of four consecutive 16-bit elements and
// lane i receives, as component j, element i % 4 of the four that lane 4 j + i / 4 pointed at.
// With lane p pointing at tile[row 4 H + p / 4 (+ 8)][col 16 (lane / 16 % 2) + 4 (p % 4)], lane
// (L, H) of the wave gets tile[4 H + j (+ 8)][L], j = 0 .. 3: column L of the rows rho_H(0 .. 7), the
// row order in which the B operand (a previous result) holds its eight contraction elements.
// `tile` points at the first of the 16 rows and the first of the 32 columns of the operand.
template <int LD>
__device__ __forceinline__ bf16x8 read_transposed(const uint16_t* tile, int lane) {
  typedef short v4i16 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) v4i16* lds_v4_t;
  const int p = lane & 15, g = lane >> 4;
  const uint16_t* a0 = tile + (4 * (g >> 1) + (p >> 2)) * LD + 16 * (g & 1) + 4 * (p & 3);
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)a0);
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)(a0 + 8 * LD));
  typedef short v8i16 __attribute__((ext_vector_type(8)));
  const v8i16 x = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, x);
}

template <int D>
__global__ void __launch_bounds__(256) k_bwd_delta(BwdArgs a) {
  // D / 8 lanes per (token, query head) row, 16 bytes of out and of dout per lane
  constexpr int LPR = D / 8, RPB = 256 / LPR;
  const long row = (long)blockIdx.x * RPB + threadIdx.x / LPR;
  const int part = threadIdx.x % LPR;
  float s = 0.f;
  if (row < a.total_rows) {
    const u32x4 o = *(const u32x4*)(a.out + (size_t)row * D + part * 8);
    const u32x4 g = *(const u32x4*)(a.dout + (size_t)row * D + part * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) s += dag_bf_lo(o[e]) * dag_bf_lo(g[e]) + dag_bf_hi(o[e]) * dag_bf_hi(g[e]);
  }
#pragma unroll
  for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (part == 0 && row < a.total_rows) {
    a.delta[row] = s;
    a.nlse2[row] = -a.lse[row] * LOG2E;
  }
}

// The per-wave state of a dQ workgroup (64-row query tile x KV head x up to 4 of its query heads;
// two waves per head, each with 32 query rows: one row per lane and half wave).
template <int D>
struct DqLane {
  bf16x8 qf[D / 16], dof[D / 16];  // the row's Q and dO as B operands
  float lse2, dl;                  // its log-sum-exp (log2 units) and delta
  int i, ni;                       // its index in the sequence and its node
  uint64_t vis0;                   // first visibility word of that node
  bool row_ok;
  size_t qoff;                     // element offset of the row in q / dout / dq
};

template <int D>
__device__ __forceinline__ void dq_store(const BwdArgs& a, const DqLane<D>& me, int H, const f32x16* dQ) {
  if (!me.row_ok) return;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      u32x2 o;
      o[0] = dag_pack_bf2(dQ[db][4 * e4] * a.scale, dQ[db][4 * e4 + 1] * a.scale);
      o[1] = dag_pack_bf2(dQ[db][4 * e4 + 2] * a.scale, dQ[db][4 * e4 + 3] * a.scale);
      *(u32x2*)(a.dq + me.qoff + 32 * db + 8 * e4 + 4 * H) = o;
    }
}

// The visible key tiles of a query tile, FULL ones first (the forward's CSR row), copied to LDS at
// set-up; rows longer than the arrays read the rest from global memory.  get() is an
// inline-assembly LDS read that waits for itself: the loads of k_bwd_dq2's ring write LDS too, and
// a compiler-visible LDS read might be made to wait for all of them.
constexpr int MAX_ROW_LDS = DAG_BWD_LDS_TILES;
struct TileList {
  const int32_t* col;   // the row in global memory
  const uint8_t* flag;
  uint32_t lds_col, lds_flag;  // LDS byte addresses of the copies
  template <int NT>
  __device__ __forceinline__ void fill(int32_t* sCol, uint8_t* sFlg, int n) {
    for (int x = threadIdx.x; x < min(n, MAX_ROW_LDS); x += NT) {
      sCol[x] = col[x];
      sFlg[x] = flag[x];
    }
    lds_col = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)sCol;
    lds_flag = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)sFlg;
  }
  __device__ __forceinline__ int tile(int n) const {
    if (n < MAX_ROW_LDS) {
      uint32_t v;
      asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_col + 4u * (uint32_t)n) : "memory");
      return __builtin_amdgcn_readfirstlane((int)v);
    }
    return __builtin_amdgcn_readfirstlane(col[n]);
  }
  __device__ __forceinline__ int flag_of(int n) const {
    if (n < MAX_ROW_LDS) {
      uint32_t v;
      asm volatile("ds_read_u8 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_flag + (uint32_t)n) : "memory");
      return __builtin_amdgcn_readfirstlane((int)v);
    }
    return __builtin_amdgcn_readfirstlane((int)flag[n]);
  }
};

// The walk of a dQ workgroup over entries n0 .. n1 - 1 of its tile list, one key tile at a time:
// the tile's K and V rows go through LDS (row-major, padded) for all the waves; the next tile is
// fetched into registers while the current one is multiplied (constant per-thread offsets, rows
// past the end re-read the last row and are zeroed on the way to LDS, no load depends on another).
// (fshift >= 0: a list entry's flag holds the block-map entries of four query tiles, this wave's at
// that bit; a wave whose query tile does not see the key tile only helps to stage it)
template <int D, int NT>
__device__ __forceinline__ void dq_general_walk(const BwdArgs& a, unsigned char* smem, const TileList& tl, int n0, int n1, int T,
                                                int cu, int hk, int nbase, const DqLane<D>& me, f32x16* dQ, int fshift = -1) {
  constexpr int LD = D + 8;  // padded rows: the 16-byte operand reads of 32 consecutive rows spread over the banks
  uint16_t* const sK = (uint16_t*)smem;   // [BN][LD]
  uint16_t* const sV = sK + BN * LD;      // [BN][LD]
  int* const sNode = (int*)(sV + BN * LD);
  const int tid = threadIdx.x, lane = tid & 63, L = lane & 31, H = lane >> 5;
  constexpr int NPQ = (BN * (D / 8) + NT - 1) / NT;  // 16-byte pieces per thread and staged tile
  u32x4 rk[NPQ], rv[NPQ];
  int r_node = 0;
  uint32_t row_off[NPQ];
#pragma unroll
  for (int x = 0; x < NPQ; ++x) {
    const int c = min(tid + NT * x, BN * (D / 8) - 1);
    row_off[x] = (uint32_t)(c / (D / 8)) * (uint32_t)(a.hkv * D) + (uint32_t)(c % (D / 8)) * 8;
  }
  const uint32_t one_row = (uint32_t)(a.hkv * D);
  auto fetch = [&](int kt) {
    const int j0 = kt * BN, n_in = min(BN, T - j0);
    const size_t slab = ((size_t)(cu + j0) * a.hkv + hk) * D;
    const uint16_t* pk = a.k + slab;
    const uint16_t* pv = a.v + slab;
#pragma unroll
    for (int x = 0; x < NPQ; ++x) {
      const int c = min(tid + NT * x, BN * (D / 8) - 1), r = c / (D / 8);
      const uint32_t off = r < n_in ? row_off[x] : row_off[x] - (uint32_t)(r - (n_in - 1)) * one_row;
      rk[x] = *(const u32x4*)(pk + off);
      rv[x] = *(const u32x4*)(pv + off);
    }
    if (tid < BN) r_node = a.tok_node[cu + j0 + min(tid, n_in - 1)];
  };
  auto commit = [&](int kt) {
    const int n_in = min(BN, T - kt * BN);
#pragma unroll
    for (int x = 0; x < NPQ; ++x) {
      const int c = tid + NT * x, r = c / (D / 8), ch = c % (D / 8);
      if (c < BN * (D / 8)) {
        if (r >= n_in) rk[x] = rv[x] = u32x4{0, 0, 0, 0};
        *(u32x4*)(sK + r * LD + ch * 8) = rk[x];
        *(u32x4*)(sV + r * LD + ch * 8) = rv[x];
      }
    }
    if (tid < BN) sNode[tid] = r_node;
  };
  if (n0 >= n1) return;
  int kt_next = tl.tile(n0);
  fetch(kt_next);
  for (int n = n0; n < n1; ++n) {
    const int kt = kt_next;
    int flag = tl.flag_of(n);
    if (fshift >= 0) flag = (flag >> fshift) & 3;
    const int j0 = kt * BN;
    __syncthreads();  // everybody is done with the tile in LDS
    commit(kt);
    __syncthreads();
    if (n + 1 < n1) {
      kt_next = tl.tile(n + 1);
      fetch(kt_next);  // in flight during the products below
    }
    if (flag == 0) continue;
    const bool need_mask = flag == 1;
#pragma unroll 1
    for (int hh = 0; hh < 2; ++hh) {
      f32x16 S, dP;
#pragma unroll
      for (int e = 0; e < 16; ++e) S[e] = dP[e] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {  // S^T = K Q^T, dP^T = V dO^T: rows = keys, column = this lane's query row
        S = mfma32(*(const bf16x8*)(sK + (32 * hh + L) * LD + 16 * s + 8 * H), me.qf[s], S);
        dP = mfma32(*(const bf16x8*)(sV + (32 * hh + L) * LD + 16 * s + 8 * H), me.dof[s], dP);
      }
      float ds[16];
      if (!need_mask && j0 + BN <= T) {  // every in-range row sees every key of the tile: no tests
#pragma unroll
        for (int e = 0; e < 16; ++e) ds[e] = __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -me.lse2)) * (dP[e] - me.dl);
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int kk = 32 * hh + rho(e, H), j = j0 + kk;
          bool ok = me.row_ok && j < T;
          if (need_mask) ok = ok & visible(a, nbase, me.ni, me.i, sNode[kk], j, me.vis0);
          const float p = __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -me.lse2));
          ds[e] = ok ? p * (dP[e] - me.dl) : 0.f;
        }
      }
      const bf16x8 b0 = pack8(ds), b1 = pack8(ds + 8);
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {  // dQ^T += K^T dS^T
        dQ[db] = mfma32(read_transposed<LD>(sK + (32 * hh) * LD + 32 * db, lane), b0, dQ[db]);
        dQ[db] = mfma32(read_transposed<LD>(sK + (32 * hh + 16) * LD + 32 * db, lane), b1, dQ[db]);
      }
    }
  }
}

// The set-up both dQ kernels share: the descriptor of the launch slot, then which row this lane
// owns and what it needs of it (no load depends on more than the descriptor).
struct DqTile {
  int cu, T, row0, c0, N, nfast, nbase;
};
__device__ __forceinline__ DqTile dq_tile(const BwdArgs& a) {
  const int32_t* d = a.qtile_desc + (size_t)blockIdx.x * 8;  // heaviest tiles first
  DqTile t;
  t.cu = d[0], t.T = d[1], t.row0 = d[2], t.c0 = d[3], t.N = d[4], t.nfast = d[5], t.nbase = d[6];
  return t;
}
// (g: query head of the KV head, row0: first row of this wave pair's 64-row query tile)
template <int D>
__device__ __forceinline__ void dq_setup_at(const BwdArgs& a, const DqTile& t, int hk, int g, bool head_ok, int row0, DqLane<D>& me) {
  const int h = hk * a.G + min(g, a.G - 1);
  const int tid = threadIdx.x, w = (tid >> 6) & 1, lane = tid & 63, L = lane & 31, H = lane >> 5;
  me.i = row0 + 32 * w + L;
  me.row_ok = me.i < t.T && head_ok;
  const int ic = min(me.i, t.T - 1);
  me.qoff = ((size_t)(t.cu + ic) * a.hq + h) * D;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    me.qf[s] = *(const bf16x8*)(a.q + me.qoff + 16 * s + 8 * H);
    me.dof[s] = *(const bf16x8*)(a.dout + me.qoff + 16 * s + 8 * H);
  }
  me.lse2 = a.lse[(size_t)(t.cu + ic) * a.hq + h] * LOG2E;
  me.dl = a.delta[(size_t)(t.cu + ic) * a.hq + h];
  me.ni = a.tok_node[t.cu + ic];
  me.vis0 = a.tok_vis0[t.cu + ic];
}
template <int D, int HG>
__device__ __forceinline__ void dq_setup(const BwdArgs& a, const DqTile& t, int hk, DqLane<D>& me) {
  const int g = blockIdx.z * HG + (threadIdx.x >> 7);  // two waves per query head
  dq_setup_at<D>(a, t, hk, g, g < a.dq_narrow, t.row0, me);
}

// First dQ kernel (every head dimension and head grouping): the general walk over all tiles.
template <int D, int HG>
__global__ void __launch_bounds__(128 * HG) k_bwd_dq(BwdArgs a) {
  constexpr int NT = 128 * HG;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int32_t sCol[MAX_ROW_LDS];
  __shared__ uint8_t sFlg[MAX_ROW_LDS];
  const DqTile t = dq_tile(a);
  const int hk = blockIdx.y;
  DqLane<D> me;
  dq_setup<D, HG>(a, t, hk, me);
  f32x16 dQ[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dQ[db][e] = 0.f;
  TileList tl;
  tl.col = a.qtile_col + t.c0;
  tl.flag = a.qtile_flag + t.c0;
  tl.fill<NT>(sCol, sFlg, t.N);
  __syncthreads();
  dq_general_walk<D, NT>(a, smem, tl, 0, t.N, t.T, t.cu, hk, t.nbase, me, dQ);
  dq_store<D>(a, me, (threadIdx.x & 63) >> 5, dQ);
}

// Launch order of the dK/dV workgroups: heaviest first.  A workgroup takes a pair of key tiles
// (the even tile of a sequence and its successor); its weight is the number of query tiles that
// see the pair (the prefix keys of a plan are seen by every later tile, the keys of a branch by a
// few), odd tiles get -1 and sort last.  One wave per key tile, twice: weights, then ranks by
// counting (ties by index), which is fine for the few thousand tiles of a batch.
__global__ void __launch_bounds__(64) k_bwd_weights(BwdArgs a) {
  const int kt = blockIdx.x, lane = threadIdx.x;
  const int b = dag_find_segment(a.ktile_start, a.n_seqs, kt);
  const int ktl = kt - a.ktile_start[b];
  const int T = a.cu_seqlens[b + 1] - a.cu_seqlens[b];
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  int n = 0;
  if (!(ktl & 1))
    for (int qt = lane; qt < QT; qt += 64)
      n += (bm[(int64_t)qt * KT + ktl] | (ktl + 1 < KT ? bm[(int64_t)qt * KT + ktl + 1] : 0)) != 0;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) n += __shfl_xor(n, o);
  if (lane == 0) a.kt_weight[kt] = (ktl & 1) ? -1 : n;
}
// First visibility word of every token's node, so that the dK/dV kernel can fetch it for the rows
// of a tile without a load that depends on another load.
__global__ void __launch_bounds__(256) k_bwd_tokvis(BwdArgs a, int total_tokens) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= total_tokens) return;
  const int b = dag_find_segment(a.cu_seqlens, a.n_seqs, t);
  a.tok_vis0[t] = a.node_vis[(int64_t)(a.node_start[b] + a.tok_node[t]) * a.W];
}
__global__ void __launch_bounds__(64) k_bwd_order(BwdArgs a) {
  const int kt = blockIdx.x, lane = threadIdx.x;
  const int mine = a.kt_weight[kt];
  int rank = 0;
  for (int x = lane; x < a.total_ktiles; x += 64) {
    const int w = a.kt_weight[x];
    rank += w > mine || (w == mine && x < kt);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) rank += __shfl_xor(rank, o);
  if (lane == 0) a.kt_order[rank] = kt;
}

template <int D>
constexpr int dkv_smem_bytes() {
  // Q and dO rows of one query tile for one query head and their transposed images, lse / delta of
  // the rows, node ids and first visibility words of the rows
  return 2 * BM * (D + 8) * 2 + 2 * BM * 4 + BM * 4 + BM * 8;
}

// The walk of one workgroup of the dK/dV kernels (pair of key tiles x KV head; wave w owns keys
// 32 w .. 32 w + 31 of the pair, with their K and V rows as B operands in registers and dK^T, dV^T
// accumulators for them) over the query tiles from the last one down and over the query heads of
// the group, one (tile, head) at a time: its Q and dO rows go through LDS (row-major, padded) for
// all four waves, the next (tile, head) is fetched into registers while the current one is
// computed.  `pair_flag(qt)` returns flag of tile 0 | flag of tile 1 << 2 of the pair for query
// tile qt, or 0 where the walk is to leave the tile out.  Pairs of a tile that are all visible
// run without a single test, the others evaluate Eq. 3 and the sequence end per element.
template <int D, typename PairFlag>
__device__ __forceinline__ void dkv_general_walk(const BwdArgs& a, unsigned char* smem, PairFlag&& pair_flag, int QT, int T,
                                                 int cu, int hk, int nbase, int my_kt, int nj, int j, bool key_ok,
                                                 const bf16x8* kf, const bf16x8* vf, f32x16* dK, f32x16* dV) {
  constexpr int LD = D + 8, DB = D / 32;
  constexpr int NP = BM * (D / 8) / 256;  // 16-byte pieces per thread and staged tile
  uint16_t* const sQ = (uint16_t*)smem;                  // [BM][LD]
  uint16_t* const sdO = sQ + BM * LD;                    // [BM][LD]
  float* const sLse = (float*)(sdO + BM * LD);           // [BM]  (log2 units)
  float* const sDl = sLse + BM;                          // [BM]
  int* const sNodeR = (int*)(sDl + BM);                  // [BM]
  uint64_t* const sVis0 = (uint64_t*)(sNodeR + BM);      // [BM]
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, L = lane & 31, H = lane >> 5;
  auto next_tile = [&](int qt) {  // last query tile <= qt with a visible pair, -1 if none
    while (qt >= 0 && pair_flag(qt) == 0) --qt;
    return qt;
  };
  // register stage of one (tile, head)
  // (addresses: a wave-uniform 64-bit base per tile and head plus 32-bit per-thread offsets that
  // never change; rows past the end of the sequence re-read its last row and are zeroed afterwards,
  // so no load sits under a branch; no load depends on another one: a wait for the first would
  // also wait for everything issued before it)
  u32x4 rq[NP], rdo[NP];
  float r_lse = 0.f, r_dl = 0.f;
  int r_node = 0;
  uint64_t r_vis = 0;
  uint32_t row_off[NP];  // element offset of this thread's piece x inside a 64-row slab of q / dout
#pragma unroll
  for (int x = 0; x < NP; ++x) {
    const int c = tid + 256 * x;
    row_off[x] = (uint32_t)(c / (D / 8)) * (uint32_t)(a.hq * D) + (uint32_t)(c % (D / 8)) * 8;
  }
  const uint32_t last_off = (uint32_t)(a.hq * D);  // one row
  auto fetch = [&](int qt, int g) {
    const int r0 = qt * BM;
    const int h = hk * a.G + g;
    const size_t slab = ((size_t)(cu + r0) * a.hq + h) * D;
    const uint16_t* pq = a.q + slab;
    const uint16_t* pdo = a.dout + slab;
    const int n_in = min(BM, T - r0);  // rows of the tile inside the sequence (>= 1)
#pragma unroll
    for (int x = 0; x < NP; ++x) {
      const int c = tid + 256 * x, r = c / (D / 8);
      const uint32_t off = r < n_in ? row_off[x] : row_off[x] - (uint32_t)(r - (n_in - 1)) * last_off;
      rq[x] = *(const u32x4*)(pq + off);
      rdo[x] = *(const u32x4*)(pdo + off);
    }
    if (tid < BM) {
      const int rr = min(tid, n_in - 1);
      const size_t row = (size_t)(cu + r0 + rr) * a.hq + h;
      r_lse = a.lse[row];
      r_dl = a.delta[row];
      r_node = a.tok_node[cu + r0 + rr];
      r_vis = a.tok_vis0[cu + r0 + rr];
    }
  };
  auto commit = [&](int qt_of_regs) {
    const int n_in = min(BM, T - qt_of_regs * BM);
#pragma unroll
    for (int x = 0; x < NP; ++x) {
      const int c = tid + 256 * x, r = c / (D / 8), ch = c % (D / 8);
      if (r >= n_in) rq[x] = rdo[x] = u32x4{0, 0, 0, 0};
      *(u32x4*)(sQ + r * LD + ch * 8) = rq[x];
      *(u32x4*)(sdO + r * LD + ch * 8) = rdo[x];
    }
    if (tid < BM) {
      sLse[tid] = tid < n_in ? r_lse * LOG2E : 0.f;
      sDl[tid] = tid < n_in ? r_dl : 0.f;
      sNodeR[tid] = r_node;
      sVis0[tid] = r_vis;
    }
  };

  int qt = next_tile(QT - 1), g = 0;
  if (qt >= 0) fetch(qt, g);
  while (qt >= 0) {
    __syncthreads();  // everybody is done with the tile in LDS
    commit(qt);
    __syncthreads();
    const int cur_qt = qt;
    // (every global load the products depend on comes before the fetch: a wait for a later load
    // would also wait for the fetch, the counter being in order)
    const int flag = __builtin_amdgcn_readfirstlane((pair_flag(cur_qt) >> (2 * (w >> 1))) & 3);
    if (++g == a.G) {
      g = 0;
      qt = next_tile(qt - 1);
    }
    if (qt >= 0) fetch(qt, g);  // in flight during the products below
    if (flag != 0) {
      const int r0 = cur_qt * BM;
      const bool need_mask = flag == 1;
#pragma unroll 1
      for (int rb = 0; rb < BM / 32; ++rb) {
        f32x16 S, dP;
#pragma unroll
        for (int e = 0; e < 16; ++e) S[e] = dP[e] = 0.f;
        // (all operand reads of a phase are issued before its first MFMA: one wave per SIMD has
        // nobody to hide the LDS latency behind, so the reads are kept far ahead of their use)
        bf16x8 aq[D / 16], ado[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
          aq[s] = *(const bf16x8*)(sQ + (32 * rb + L) * LD + 16 * s + 8 * H);
          ado[s] = *(const bf16x8*)(sdO + (32 * rb + L) * LD + 16 * s + 8 * H);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {  // S = Q K^T, dP = dO V^T: rows = query rows, column = this lane's key
          S = mfma32(aq[s], kf[s], S);
          dP = mfma32(ado[s], vf[s], dP);
        }
        // the transposed operands of the second phase: on their way during the exponentials
        bf16x8 at_do[2 * DB], at_q[2 * DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          at_do[2 * db] = read_transposed<LD>(sdO + (32 * rb) * LD + 32 * db, lane);
          at_do[2 * db + 1] = read_transposed<LD>(sdO + (32 * rb + 16) * LD + 32 * db, lane);
          at_q[2 * db] = read_transposed<LD>(sQ + (32 * rb) * LD + 32 * db, lane);
          at_q[2 * db + 1] = read_transposed<LD>(sQ + (32 * rb + 16) * LD + 32 * db, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
        float p[16], ds[16];
        // lse and delta of the 16 rows of this lane: four groups of four consecutive rows
        f32x4 l4[4], d4[4];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          l4[e4] = *(const f32x4*)(sLse + 32 * rb + 8 * e4 + 4 * H);
          d4[e4] = *(const f32x4*)(sDl + 32 * rb + 8 * e4 + 4 * H);
        }
        if (!need_mask && r0 + BM <= T && (my_kt + 1) * BN <= T) {  // every pair of the tile is visible: no tests
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -l4[e >> 2][e & 3]));
            ds[e] = p[e] * (dP[e] - d4[e >> 2][e & 3]);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r = 32 * rb + rho(e, H), i = r0 + r;
            bool ok = key_ok && i < T;
            if (need_mask) ok = ok & visible(a, nbase, sNodeR[r], i, nj, j, sVis0[r]);
            const float pe = __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -l4[e >> 2][e & 3]));
            p[e] = ok ? pe : 0.f;
            ds[e] = p[e] * (dP[e] - d4[e >> 2][e & 3]);
          }
        }
        const bf16x8 p0 = pack8(p), p1 = pack8(p + 8), s0 = pack8(ds), s1 = pack8(ds + 8);
#pragma unroll
        for (int db = 0; db < DB; ++db) {  // dV^T += dO^T P, dK^T += Q^T dS
          dV[db] = mfma32(at_do[2 * db], p0, dV[db]);
          dV[db] = mfma32(at_do[2 * db + 1], p1, dV[db]);
          dK[db] = mfma32(at_q[2 * db], s0, dK[db]);
          dK[db] = mfma32(at_q[2 * db + 1], s1, dK[db]);
        }
      }
    }
  }
}

// Writes the dK and dV rows of a wave's 32 keys (column = this lane's key, rows = d: every lane
// writes its key's row).
template <int D>
__device__ __forceinline__ void dkv_store(const BwdArgs& a, size_t koff, bool key_ok, int H, const f32x16* dK, const f32x16* dV) {
  if (!key_ok) return;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      u32x2 ok2, ov2;
      ok2[0] = dag_pack_bf2(dK[db][4 * e4] * a.scale, dK[db][4 * e4 + 1] * a.scale);
      ok2[1] = dag_pack_bf2(dK[db][4 * e4 + 2] * a.scale, dK[db][4 * e4 + 3] * a.scale);
      ov2[0] = dag_pack_bf2(dV[db][4 * e4], dV[db][4 * e4 + 1]);
      ov2[1] = dag_pack_bf2(dV[db][4 * e4 + 2], dV[db][4 * e4 + 3]);
      *(u32x2*)(a.dk + koff + 32 * db + 8 * e4 + 4 * H) = ok2;
      *(u32x2*)(a.dv + koff + 32 * db + 8 * e4 + 4 * H) = ov2;
    }
}

// First dK/dV kernel (every head dimension; the only one for 64): the general walk over all tiles.
template <int D>
__global__ void __launch_bounds__(256) k_bwd_dkv(BwdArgs a) {
  constexpr int DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ uint8_t sFlag[MAX_QT_LDS];                  // block-map column of the pair: flag of tile 0 | flag of tile 1 << 2
  // (the KV head is the fast index of the launch: workgroups go to the XCDs round robin, so with 8
  // KV heads every XCD's L2 holds the Q / dO tiles of one head group only, and the workgroups of a
  // group walk over the query tiles from the last one down, i.e. side by side)
  const int hk = blockIdx.x % a.hkv, kt = a.kt_order[blockIdx.x / a.hkv];  // heaviest pairs first
  const int b = dag_find_segment(a.ktile_start, a.n_seqs, kt);
  const int ktl = kt - a.ktile_start[b];
  if (ktl & 1) return;  // the workgroup of the even tile takes the pair (odd tiles come last in the order)
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  const int nbase = a.node_start[b];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, L = lane & 31, H = lane >> 5;
  const int my_kt = ktl + (w >> 1);          // this wave's key tile
  const int j = ktl * BN + 32 * w + L;       // this lane's key
  const bool key_ok = j < T;
  const int jc = min(j, T - 1);
  const size_t koff = ((size_t)(cu + jc) * a.hkv + hk) * D;
  bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kf[s] = *(const bf16x8*)(a.k + koff + 16 * s + 8 * H);
    vf[s] = *(const bf16x8*)(a.v + koff + 16 * s + 8 * H);
  }
  const int nj = a.tok_node[cu + jc];
  f32x16 dK[DB], dV[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dK[db][e] = dV[db][e] = 0.f;

  // (the map is read once: a load of it inside the loop would sit, with its full latency, in front
  // of every tile; sequences with more query tiles than the array holds read the map directly)
  const bool flags_in_lds = QT <= MAX_QT_LDS;
  if (flags_in_lds) {
    for (int x = tid; x < QT; x += 256) {
      const int f0 = bm[(int64_t)x * KT + ktl];
      const int f1 = ktl + 1 < KT ? bm[(int64_t)x * KT + ktl + 1] : 0;
      sFlag[x] = (uint8_t)(f0 | (f1 << 2));
    }
    __syncthreads();
  }
  auto pair_flag = [&](int qt) {
    if (flags_in_lds) return (int)sFlag[qt];
    const int f0 = bm[(int64_t)qt * KT + ktl];
    const int f1 = ktl + 1 < KT ? bm[(int64_t)qt * KT + ktl + 1] : 0;
    return f0 | (f1 << 2);
  };
  dkv_general_walk<D>(a, smem, pair_flag, QT, T, cu, hk, nbase, my_kt, nj, j, key_ok, kf, vf, dK, dV);
  dkv_store<D>(a, koff, key_ok, H, dK, dV);
}

// ---------------------------------------------------------------------------------------------
// k_bwd_dkv2: the dK/dV kernel for head dimension 128 with the data movement and the instruction
// order of the forward kernel.  Same decomposition as k_bwd_dkv (pair of key tiles x KV head, wave
// w owns keys 32 w .. 32 w + 31, iteration = (query tile, query head)), but
//   * the Q and dO tiles go from global memory straight into LDS (16 bytes per lane, no staging
//     registers) through a ring of NST stages; one bare s_barrier per iteration, in its middle:
//     it publishes the stage of the NEXT iteration (every wave has waited for its own loads of
//     that stage before) and frees the stage of the previous one, which the loads of iteration
//     n + NST - 1 then fill, one load per MFMA slot;
//   * a wave-level load writes 1 KiB of consecutive LDS, a block of 4 rows laid out
//     [chunk / 4][row % 4][chunk % 4][16 B], blocks 1024 + 16 bytes apart: four consecutive lanes
//     fetch 64 consecutive bytes, the 16-byte row reads (A operands of S = Q K^T, dP = dO V^T) of 16
//     consecutive rows and the 8-byte transposing reads (A operands of dV^T += dO^T P,
//     dK^T += Q^T dS) of 16 consecutive lanes both fall into 16 different bank groups;
//   * an iteration is written slot by slot (operand read of the MFMA PF slots ahead, wait, one
//     MFMA, a share of the exponentials; a scheduling barrier after every slot): scores and dP of
//     the two 32-row halves (32 MFMAs), then dV / dK of the two halves (32 MFMAs), with the
//     exponentials of half 0 in the slots of the score MFMAs of half 1 and those of half 1 in the
//     slots of the dV / dK MFMAs of half 0.  The operand reads are inline assembly with explicit
//     lgkmcnt waits (LDS reads return in order); nothing branches while such reads are in flight,
//     so no copy of a register that is still being written can be made
//     (tests/test_asm_lds_reads.py checks the generated code for exactly that);
//   * two such loops run one after the other: the iterations whose pairs are all visible (both key
//     tiles FULL, nothing past the end of the sequence), then, when a node has one visibility
//     word, the masked and ragged ones: Eq. 3 of a (query tile, key) pair is one 64-bit word per
//     lane, built once per query tile from the runs of equal node ids among its rows
//     (tile_visibility) and applied with two instructions per element; the ancestor test uses the
//     key's column of the visibility matrix, built once per workgroup.  Both loops find their
//     tiles through a bitmap per kind of the pair's block-map column.
//     With more words per node the masked iterations take the general walk of k_bwd_dkv.
// Every iteration passes the barrier once and issues LPS loads per wave (past the end of the walk:
// loads of the sequence's first tile, never consumed), so the vmcnt waits are constants.
// With one wave per SIMD (the accumulators and the K / V operands of 32 keys need 192 registers)
// nothing of a wave overlaps its own MFMAs: an iteration costs the 64 MFMAs plus the time to
// issue everything else.
namespace dkv2 {
constexpr int NST = 4;              // ring depth
constexpr int LPS = 9;              // wave-level loads per stage and wave: 4 Q blocks, 4 dO blocks, 1 of row data
constexpr int PF = 5;               // operands in flight ahead of their MFMA
constexpr int BLK = 1024 + 16;
constexpr int TILEB = 16 * BLK;     // 64 rows x 128 dims
constexpr int RD = 2 * TILEB;       // row data: -lse log2(e) [64], delta [64], node id [64]
constexpr int STAGEB = RD + 768;
constexpr int NSLOT = 64;
constexpr int VAHEAD = 8;           // the row data of four rows are read this many slots before their first use
constexpr int XR = 2;               // row-data reads per group of four rows: -lse and delta
constexpr int opnd_reads(int o) { return o < 32 ? 1 : 2; }
// The scores of rows 4 x .. 4 x + 3 of half h are taken in slots 16 + 16 h + 4 x ..; the XR reads of their
// row data go out VAHEAD slots earlier, i.e. before the operand read that slot waits for, so they have
// arrived with it.
constexpr int extra_reads(int slot) { return slot >= 16 - VAHEAD && slot < 48 - VAHEAD && slot % 4 == 0 ? XR : 0; }
constexpr int issued_through(int k) {  // LDS reads issued up to and including those of operand k
  int t = 0;
  for (int o = 0; o <= k; ++o) t += (o >= PF ? extra_reads(o - PF) : 0) + opnd_reads(o);
  return t;
}
constexpr int wait_at(int i) {  // reads that may still be pending when MFMA i starts
  const int last = i + PF < NSLOT ? i + PF : NSLOT - 1;
  const int n = issued_through(last) - issued_through(i);
  return n < 15 ? n : 15;
}
// byte offset (after the per-lane part) of operand i of the fast iteration
constexpr int row_imm(int i) {  // i < 32: row operand of half i / 16, k-step (i % 16) / 2, of Q (even) or dO (odd)
  return (i & 1) * TILEB + 8 * (i / 16) * BLK + (((i % 16) / 2) / 2) * 256 + (((i % 16) / 2) % 2) * 32;
}
constexpr int tr_imm(int i) {  // i >= 32: transposed operand (dims 32 db .., 16 rows) of dO (even) or Q (odd)
  const int j = i - 32, h = j / 16, jj = j % 16, db = jj / 4, hh = (jj / 2) % 2;
  return ((jj & 1) ? 0 : TILEB) + (8 * h + 4 * hh) * BLK + db * 256;
}
}  // namespace dkv2

// Eq. 3 for one 64 x 64 tile as a 64-bit word per lane (one visibility word per node): bit c says
// whether element c of the tile -- query row c for a lane that holds a key, key c for a lane that
// holds a query row -- and the lane's own token see each other.  The tokens of a sequence lie node
// after node, so the tile's 64 elements are a few runs of one node each: the runs are found with
// one ballot over the node ids (LDS, `ids`: byte address of the 64 ids) and every run is switched
// on as a whole -- for the lane's own node the elements that pass the causal test (`own`), for
// another node n all or nothing by bit n of `word` (the lane's row or column of the visibility
// matrix).  Elements from n_in on lie behind the end of the sequence.  Called where no operand read
// is in flight (the LDS reads here wait for themselves; the loop branches on wave-uniform values).
__device__ __forceinline__ uint64_t tile_visibility(uint32_t ids, int lane, uint32_t my_node, uint64_t word, uint64_t own,
                                                    int n_in) {
  uint32_t n_here, n_before;
  asm volatile("ds_read_b32 %0, %2\n\tds_read_b32 %1, %3\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(n_here), "=&v"(n_before)
               : "v"(ids + 4u * (uint32_t)lane), "v"(ids + 4u * (uint32_t)max(lane - 1, 0))
               : "memory");
  uint64_t starts = __builtin_amdgcn_ballot_w64(lane == 0 || n_here != n_before);
  uint64_t m = 0;
  while (starts != 0) {
    const int s0 = __builtin_ctzll(starts);
    starts &= starts - 1;
    const int s1 = starts != 0 ? __builtin_ctzll(starts) : 64;
    const uint32_t n = (uint32_t)__builtin_amdgcn_readlane((int)n_here, s0);
    const uint64_t run = (s1 == 64 ? ~0ull : (1ull << s1) - 1) & ~((1ull << s0) - 1);
    const uint64_t sel = n == my_node ? own : 0ull - ((word >> (n & 63u)) & 1ull);
    m |= run & sel;
  }
  return n_in >= 64 ? m : m & ((1ull << n_in) - 1);
}
// x when bit BIT of the word is set, else 0: the bit as a signed one-bit field (0 or all ones), then
// one AND -- no comparison, no condition register (written out: from the plain expression the
// compiler makes a test, a compare and a select).
template <int BIT>
__device__ __forceinline__ float keep_if_bit(float x, uint32_t word) {
  float r;
  asm("v_bfe_i32 %0, %2, %3, 1\n\tv_and_b32 %0, %0, %1" : "=&v"(r) : "v"(x), "v"(word), "n"(BIT));
  return r;
}

// The score MFMAs of k_bwd_dkv2 written out, with their results in vector registers and the B
// operand (the K / V rows of the wave's keys, fixed for the workgroup) in accumulation registers.
// A kernel with more than 256 registers gets the accumulation-register form for every MFMA the
// compiler selects, and the vector instructions that turn scores into probabilities would first
// have to copy every score out of there; the dK / dV accumulators stay where they are.  The
// compiler does not know what these statements are: the last MFMA of a chain is followed by 20
// idle states, more than the 19 a vector instruction must keep from a 16-pass MFMA whose result
// it reads; a chain's own accumulation is two MFMAs apart (the S and dP chains alternate).
__device__ __forceinline__ f32x16 mfma32_first_v(bf16x8 a, bf16x8 b_acc) {
  f32x16 d;
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b_acc));
  return d;
}
__device__ __forceinline__ f32x16 mfma32_next_v(bf16x8 a, bf16x8 b_acc, f32x16 c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b_acc));
  return c;
}
__device__ __forceinline__ f32x16 mfma32_last_v(bf16x8 a, bf16x8 b_acc, f32x16 c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\ts_nop 15\n\ts_nop 3" : "+v"(c) : "v"(a), "v"(b_acc));
  return c;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_only() {  // s_waitcnt vmcnt(N) (gfx9 encoding)
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
template <int N>
__device__ __forceinline__ void wait_lgkmcnt_only() {
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {  // byte address inside LDS of a __shared__ pointer
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
template <int A, int B, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (A < B) {
    f(std::integral_constant<int, A>{});
    static_for<A + 1, B>(f);
  }
}

__global__ void __launch_bounds__(256) k_bwd_dkv2(BwdArgs a) {
  using namespace dkv2;
  constexpr int D = 128, DB = D / 32;
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
  typedef short v4i16 __attribute__((ext_vector_type(4)));
  typedef short v8i16 __attribute__((ext_vector_type(8)));
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int KIND_WORDS = (MAX_QT_LDS + 63) / 64;
  __shared__ uint8_t sFlag[MAX_QT_LDS];  // block-map column of the pair: flag of tile 0 | flag of tile 1 << 2
  __shared__ uint64_t sKind[3][KIND_WORDS];
  const int hk = blockIdx.x % a.hkv, kt = a.kt_order[blockIdx.x / a.hkv];  // heaviest pairs first
  const int b = dag_find_segment(a.ktile_start, a.n_seqs, kt);
  const int ktl = kt - a.ktile_start[b];
  if (ktl & 1) return;  // the workgroup of the even tile takes the pair
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  const int nbase = a.node_start[b];
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, L = lane & 31, H = lane >> 5;
  const int my_kt = ktl + (w >> 1);
  const int j = ktl * BN + 32 * w + L;  // this lane's key
  const bool key_ok = j < T;
  const int jc = min(j, T - 1);
  const size_t koff = ((size_t)(cu + jc) * a.hkv + hk) * D;
  bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kf[s] = *(const bf16x8*)(a.k + koff + 16 * s + 8 * H);
    vf[s] = *(const bf16x8*)(a.v + koff + 16 * s + 8 * H);
  }
  const int nj = a.tok_node[cu + jc];
  // (one visibility word per node) the nodes that see this lane's key: bit ni of `seen_by` = bit nj
  // of node ni's word, i.e. the key's column of the sequence's visibility matrix
  uint64_t seen_by = 0;
  if (a.W == 1) {
    const int n_nodes = a.node_start[b + 1] - nbase;
    const uint64_t word = lane < n_nodes ? a.node_vis[nbase + lane] : 0;
#pragma unroll
    for (int ni = 0; ni < 64; ++ni) {
      const uint64_t wn = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(word >> 32), ni) << 32) |
                          (uint32_t)__builtin_amdgcn_readlane((int)word, ni);
      seen_by |= ((wn >> (nj & 63)) & 1ull) << ni;
    }
  }
  f32x16 dK[DB], dV[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dK[db][e] = dV[db][e] = 0.f;

  // bit 4 of a pair's flags: the iteration runs in the steady-state loop (both key tiles exist, every
  // pair of both is visible, nothing reaches past the end of the sequence)
  auto with_fast_bit = [&](int qt, int f) {
    return f | ((f == (2 | (2 << 2)) && (qt + 1) * BM <= T && (ktl + 2) * BN <= T) ? 16 : 0);
  };
  // Two pipelined loops: the iterations without tests, then (when a node has one visibility word)
  // the masked ones; with more words per node the masked ones go to the general walk.
  const bool masks_in_loop = a.W == 1;
  auto kind_of = [&](int f) { return (f & 16) ? 0 : ((f & 15) != 0 && masks_in_loop) ? 1 : 2; };  // 2: general walk or nothing
  // The column is kept in LDS as the flags and as one bitmap per kind of iteration (bit qt % 64 of
  // word qt / 64: tile qt has a visible pair and is of that kind), so that a walk finds its next
  // tile with one 64-bit read per 64 tiles instead of one probe per tile.
  const bool flags_in_lds = QT <= MAX_QT_LDS;
  if (flags_in_lds) {
    for (int x0 = 0; x0 < QT; x0 += 256) {
      const int x = x0 + tid;
      int f = 0;
      if (x < QT) {
        const int f0 = bm[(int64_t)x * KT + ktl];
        const int f1 = ktl + 1 < KT ? bm[(int64_t)x * KT + ktl + 1] : 0;
        f = with_fast_bit(x, f0 | (f1 << 2));
        sFlag[x] = (uint8_t)f;
      }
      const int kind = (f & 15) != 0 ? kind_of(f) : 3;
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const uint64_t word = __builtin_amdgcn_ballot_w64(kind == k);
        if (lane == 0 && x0 + 64 * w < QT) sKind[k][(x0 >> 6) + w] = word;
      }
    }
  }
  __syncthreads();
  const uint32_t flag_base = lds_addr(sFlag), kind_base = lds_addr(sKind);
  // (the flags are read with an inline-assembly LDS read that waits for itself: the ring's loads
  // write LDS too, and a compiler-visible LDS read might be made to wait for all of them)
  auto pair_flag = [&](int qt) {
    if (flags_in_lds) {
      uint32_t v;
      asm volatile("ds_read_u8 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(flag_base + (uint32_t)qt) : "memory");
      return __builtin_amdgcn_readfirstlane((int)v);
    }
    const int f0 = bm[(int64_t)qt * KT + ktl];
    const int f1 = ktl + 1 < KT ? bm[(int64_t)qt * KT + ktl + 1] : 0;
    return __builtin_amdgcn_readfirstlane(with_fast_bit(qt, f0 | (f1 << 2)));
  };
  auto kind_word = [&](int kind, int wi) {
    uint64_t v;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(kind_base + (uint32_t)(kind * KIND_WORDS + wi) * 8u) : "memory");
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  };
  auto last_of_kind = [&](int kind, int qt) {  // last query tile <= qt of the kind (with a visible pair), -1 if none
    if (!flags_in_lds) {
      for (; qt >= 0; --qt) {
        const int f = pair_flag(qt);
        if ((f & 15) != 0 && kind_of(f) == kind) break;
      }
      return qt;
    }
    if (qt < 0) return -1;
    int wi = qt >> 6;
    uint64_t word = kind_word(kind, wi) & (~0ull >> (63 - (qt & 63)));
    while (word == 0) {
      if (--wi < 0) return -1;
      word = kind_word(kind, wi);
    }
    return 64 * wi + 63 - __builtin_clzll(word);
  };

  // ---- loads of one stage, in LPS pieces per wave (piece p of (tile qt, head g) into stage st)
  const uint32_t row_stride = (uint32_t)(a.hq * D);  // elements
  const uint32_t chunk8 = (uint32_t)(4 * (lane >> 4) + (lane & 3)) * 8;  // this lane's 16-byte chunk of a row
  const int rsub = (lane >> 2) & 3;
  // Row data, 4 bytes per lane, one load per wave: wave 0 fetches -lse log2(e), wave 1 delta, wave 2
  // the node ids of the rows (for the masked iterations), wave 3 -lse log2(e) once more (every wave
  // issues the same number of loads, so that the vmcnt waits are the same constants for all).
  // Element index in the source: (token of the row) * rd_mul + head * rd_hmul -- no branch where
  // the loads are issued.
  const float* rd_src = w == 1 ? a.delta : w == 2 ? (const float*)a.tok_node : a.nlse2;
  const int rd_mul = w == 2 ? 1 : a.hq, rd_hmul = w == 2 ? 0 : 1, rd_dst = w == 1 ? 256 : w == 2 ? 512 : 0;
  // The addresses of a stage's loads are prepared once per iteration, outside the slots (wave-uniform
  // bases, four per-lane row offsets, one per-lane row-data pointer); a slot then only sets the LDS
  // destination and issues its load.
  struct IssueCtx {
    const uint16_t *qb, *dob;  // first row of the tile, this head
    uint32_t voff[4];          // element offset of this lane's chunk in block w + 4 i (rows past the sequence end re-read its last row)
    const float* rd;           // this lane's row-data word
  };
  auto prepare_issue = [&](int qt, int g) __attribute__((always_inline)) {
    IssueCtx c;
    const int qv = max(qt, 0);
    const int r0 = qv * BM, n_in = min(BM, T - r0), h = hk * a.G + g;
    const size_t slab = ((size_t)(cu + r0) * a.hq + h) * D;
    c.qb = a.q + slab;
    c.dob = a.dout + slab;
#pragma unroll
    for (int i = 0; i < 4; ++i) c.voff[i] = (uint32_t)min(4 * (w + 4 * i) + rsub, n_in - 1) * row_stride + chunk8;
    c.rd = rd_src + ((size_t)(cu + r0 + min(lane, n_in - 1)) * rd_mul + rd_hmul * h);
    return c;
  };
  auto issue_piece = [&](int p, const IssueCtx& c, int st) __attribute__((always_inline)) {
    unsigned char* const sb = smem + st * STAGEB;
    if (p < 8) {
      const int blk = w + 4 * (p & 3);
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)((p < 4 ? c.qb : c.dob) + c.voff[p & 3]),
                                       (lds_ptr_t)(sb + (p < 4 ? 0 : TILEB) + blk * BLK), 16, 0, 0);
    } else {
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)c.rd, (lds_ptr_t)(sb + RD + rd_dst), 4, 0, 0);
    }
  };
  auto sync_mid = [&]() __attribute__((always_inline)) {
    wait_vmcnt_only<LPS>();        // this wave's loads of the next iteration's stage have landed
    __builtin_amdgcn_s_barrier();  // (bare: a __syncthreads would drain the loads in flight)
    asm volatile("" ::: "memory");
  };

  // per-lane parts of the LDS operand addresses
  const uint32_t roff = (uint32_t)((L >> 2) * BLK + (L & 3) * 64 + H * 16);
  const uint32_t toff = (uint32_t)(((lane >> 5) & 1) * BLK + ((lane & 15) >> 2) * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8);
  const uint32_t smem_base = lds_addr(smem);
  const float sc = a.sc;

  // ---- the iteration without tests, slot by slot
  // (with masks: vis_lo / vis_hi = this lane's visibility word of the tile, shifted so that bit
  // 32 h + 8 (e / 4) + e % 4 belongs to element e of half h, i.e. to row 64 qt + 4 H + that number)
  auto pipelined_iter = [&](auto msk_c, int cs, const IssueCtx& ictx, int is, uint32_t vis_lo, uint32_t vis_hi) __attribute__((always_inline)) {
    constexpr bool MSK = decltype(msk_c)::value;
    const uint32_t sbase = smem_base + (uint32_t)cs * STAGEB;
    const uint32_t ra = sbase + roff, ta = sbase + toff, va = sbase + RD + 16 * H;
    bf16x8 op[NSLOT];
    v4i16 lo[NSLOT], hi[NSLOT];
    f32x4 nl[2][4], dl[2][4];
    f32x16 S[2], dP[2];
    float pt[2][16], dt[2][16];
    bf16x8 pp[2][2], dss[2][2];
    // row data of rows 32 h + 8 x + 4 H .. + 3: -lse, delta, node ids
    auto fetch_val = [&](auto hc, auto xc) __attribute__((always_inline)) {
      constexpr int h = decltype(hc)::value, x = decltype(xc)::value;
      const uint32_t v = va;  // (named here: captures inside discarded branches trip the compiler)
      f32x4(*const nlp)[4] = nl;
      f32x4(*const dlp)[4] = dl;
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(nlp[h][x]) : "v"(v), "n"(128 * h + 32 * x));
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dlp[h][x]) : "v"(v), "n"(256 + 128 * h + 32 * x));
    };
    auto fetch = [&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      const uint32_t r = ra, t = ta;
      bf16x8* const opp = op;
      v4i16* const lop = lo;
      v4i16* const hip_ = hi;
      if constexpr (i < 32)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(opp[i]) : "v"(r), "n"(row_imm(i)));
      else if constexpr (i < NSLOT)
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(lop[i]), "=&v"(hip_[i])
                     : "v"(t), "n"(tr_imm(i)), "n"(tr_imm(i) + 2 * BLK));
    };
    static_for<0, PF>(fetch);
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NSLOT>([&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      if constexpr (i == 32) {
        sync_mid();
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (extra_reads(i) != 0) {
        constexpr int u = (i + VAHEAD - 16) / 4;  // rows 4 u .. 4 u + 3 of the 64
        fetch_val(std::integral_constant<int, u / 4>{}, std::integral_constant<int, u % 4>{});
      }
      fetch(std::integral_constant<int, i + PF>{});
      wait_lgkmcnt_only<wait_at(i)>();
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 32) {
        constexpr int rb = i / 16, s = (i % 16) / 2;
        const bf16x8 b_acc = (i & 1) == 0 ? kf[s] : vf[s];
        f32x16& acc = (i & 1) == 0 ? S[rb] : dP[rb];
        if constexpr (s == 0)
          acc = mfma32_first_v(op[i], b_acc);
        else if constexpr (s < D / 16 - 1)
          acc = mfma32_next_v(op[i], b_acc, acc);
        else
          acc = mfma32_last_v(op[i], b_acc, acc);
      } else {
        constexpr int jx = i - 32, h = jx / 16, jj = jx % 16, db = jj / 4, hh = (jj / 2) % 2;
        const v8i16 x = {lo[i][0], lo[i][1], lo[i][2], lo[i][3], hi[i][0], hi[i][1], hi[i][2], hi[i][3]};
        const bf16x8 opx = __builtin_bit_cast(bf16x8, x);
        if constexpr ((jj & 1) == 0)
          dV[db] = mfma32(opx, pp[h][hh], dV[db]);
        else
          dK[db] = mfma32(opx, dss[h][hh], dK[db]);
      }
      if constexpr (i >= 32 && i < 32 + LPS) issue_piece(i - 32, ictx, is);
      if constexpr (i >= 16 && i < 48) {  // one score of half 0 (slots 16..31) or half 1 (slots 32..47)
        constexpr int h = (i - 16) / 16, e = (i - 16) % 16;
        float pe = __builtin_amdgcn_exp2f(fmaf(S[h][e], sc, nl[h][e >> 2][e & 3]));
        if constexpr (MSK) pe = keep_if_bit<8 * (e >> 2) + (e & 3)>(pe, h == 0 ? vis_lo : vis_hi);  // Eq. 3 and the end of the sequence
        pt[h][e] = pe;
        dt[h][e] = pe * (dP[h][e] - dl[h][e >> 2][e & 3]);
        if constexpr ((e & 1) == 1) {
          const uint32_t pw = dag_pack_bf2(pt[h][e - 1], pt[h][e]), dw = dag_pack_bf2(dt[h][e - 1], dt[h][e]);
          typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
          const bf16x2 pb = __builtin_bit_cast(bf16x2, pw), db2 = __builtin_bit_cast(bf16x2, dw);
          pp[h][e >> 3][(e & 7) - 1] = pb[0];
          pp[h][e >> 3][e & 7] = pb[1];
          dss[h][e >> 3][(e & 7) - 1] = db2[0];
          dss[h][e >> 3][e & 7] = db2[1];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // ---- the walk of one kind of iteration: query tiles from the last one down, the heads of the group inside
  auto ring_loop = [&](auto msk_c) __attribute__((always_inline)) {
    constexpr int KIND = decltype(msk_c)::value ? 1 : 0;
    auto next_tile = [&](int qt) { return last_of_kind(KIND, qt); };
    auto advance = [&](int& qt, int& g) {
      if (qt < 0) return;
      if (++g == a.G) {
        g = 0;
        qt = next_tile(qt - 1);
      }
    };
    int cq = next_tile(QT - 1), cg = 0;  // the iteration being computed
    if (cq < 0) return;
    int iq = cq, ig = 0;                 // the iteration whose loads are issued next
#pragma unroll 1
    for (int st = 0; st < NST - 1; ++st) {
      const IssueCtx c = prepare_issue(iq, ig);
#pragma unroll
      for (int p = 0; p < LPS; ++p) issue_piece(p, c, st);
      advance(iq, ig);
    }
    wait_vmcnt_only<(NST - 2) * LPS>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int cs = 0, is = NST - 1;
    // (register classes, at the top of every iteration: the dK / dV accumulators stay in the
    // accumulation registers over the whole loop; without the hint the allocator moves three of
    // the eight back and forth every iteration)
    while (cq >= 0) {  // one query tile: (with masks) its visibility word once, then an iteration per head
      bool active = true;  // a visible pair in this wave's key tile
      uint64_t vis = 0;
      if constexpr (KIND == 1) {
        active = ((pair_flag(cq) >> (2 * (w >> 1))) & 3) != 0;
        if (active) {
          // the rows of tile cq that this lane's key is visible to: own node from the key's row on
          const int first = j - cq * BM;  // first such row of the tile (may lie before or behind it)
          const uint64_t own = first <= 0 ? ~0ull : first >= 64 ? 0ull : ~0ull << first;
          vis = tile_visibility(smem_base + (uint32_t)cs * STAGEB + RD + 512, lane, (uint32_t)nj, seen_by, own, T - cq * BM);
          vis = key_ok ? vis >> (4 * H) : 0ull;  // bit 32 h + 8 (e / 4) + e % 4: element e of half h
        }
      }
#pragma unroll 1
      for (int g = 0; g < a.G; ++g) {
#pragma unroll
        for (int db = 0; db < DB; ++db) asm volatile("" : "+a"(dK[db]), "+a"(dV[db]));
        const IssueCtx ic = prepare_issue(iq, ig);
        if (KIND == 0 || active) {
          pipelined_iter(msk_c, cs, ic, is, (uint32_t)vis, (uint32_t)(vis >> 32));
        } else {  // only the ring's business
          sync_mid();
#pragma unroll
          for (int p = 0; p < LPS; ++p) issue_piece(p, ic, is);
        }
        advance(iq, ig);
        cs = cs + 1 == NST ? 0 : cs + 1;
        is = is + 1 == NST ? 0 : is + 1;
      }
      cq = next_tile(cq - 1);
    }
    wait_vmcnt_only<0>();  // (the loads past the end of the walk)
    __builtin_amdgcn_s_barrier();  // every wave is done with the ring before the next loop refills it
    asm volatile("" ::: "memory");
  };
  ring_loop(std::false_type{});
  if (masks_in_loop) ring_loop(std::true_type{});
  __syncthreads();  // the ring is free: the general walk lays its own tiles over it
  // ---- everything else: the general walk over the tiles the loop above left out
  auto rest_flag = [&](int qt) {
    const int f = pair_flag(qt);
    return kind_of(f) == 2 ? (f & 15) : 0;
  };
  if (last_of_kind(2, QT - 1) >= 0)  // (the same for every thread)
    dkv_general_walk<D>(a, smem, rest_flag, QT, T, cu, hk, nbase, my_kt, nj, j, key_ok, kf, vf, dK, dV);
  dkv_store<D>(a, koff, key_ok, H, dK, dV);
}

// Tile lists of the dQ workgroups that take one query head on four query tiles (the heads that do
// not fill a group of four): one wave per query tile of the batch, those of every fourth tile of a
// sequence work.  The list of tiles 4 c .. 4 c + 3 holds every key tile that one of them sees, with
// the four block-map entries as its flag; the key tiles that all four see in full, with all their
// rows and keys inside the sequence, come first (they run without tests), both parts ascending.
__global__ void __launch_bounds__(64) k_bwd_wide_rows(BwdArgs a) {
  const int x = blockIdx.x, lane = threadIdx.x;
  const int b = dag_find_segment(a.qtile_start, a.n_seqs, x);
  const int qt = x - a.qtile_start[b];
  if (qt & 3) return;
  const int T = a.cu_seqlens[b + 1] - a.cu_seqlens[b];
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  const int64_t base = a.block_map_off[b] + (int64_t)qt * KT;
  const bool rows_in = (qt + 4) * BM <= T;
  auto entries = [&](int kt) {
    int f8 = 0;
    if (kt < KT)
      for (int i = 0; i < 4; ++i)
        if (qt + i < QT) f8 |= (int)bm[(int64_t)(qt + i) * KT + kt] << (2 * i);
    return f8;
  };
  int n = 0, nfast = 0;
  for (int k0 = 0; k0 < KT; k0 += 64) {
    const int kt = k0 + lane, f8 = entries(kt);
    nfast += __builtin_popcountll(__builtin_amdgcn_ballot_w64(rows_in && f8 == 0xAA && (kt + 1) * BN <= T));
    n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(f8 != 0));
  }
  int at_fast = 0, at_rest = nfast;
  const uint64_t below = (1ull << lane) - 1;
  for (int k0 = 0; k0 < KT; k0 += 64) {
    const int kt = k0 + lane, f8 = entries(kt);
    const bool fast = rows_in && f8 == 0xAA && (kt + 1) * BN <= T, rest = f8 != 0 && !fast;
    const uint64_t mf = __builtin_amdgcn_ballot_w64(fast), mr = __builtin_amdgcn_ballot_w64(rest);
    if (fast || rest) {
      const int64_t at = base + (fast ? at_fast + __builtin_popcountll(mf & below) : at_rest + __builtin_popcountll(mr & below));
      a.wide_col[at] = kt;
      a.wide_flag[at] = (uint8_t)f8;
    }
    at_fast += __builtin_popcountll(mf);
    at_rest += __builtin_popcountll(mr);
  }
  if (lane == 0) {
    a.wide_n[x] = n;
    a.wide_nfast[x] = nfast;
    // the groups of the batch, numbered through (the launch of the dQ workgroups runs over these
    // numbers: over the query tiles, with three of four workgroups leaving at once, the ones that
    // stay would all have the same index modulo four and land on two of the eight XCDs)
    int before = 0;
    for (int bb = 0; bb < b; ++bb) before += (a.qtile_start[bb + 1] - a.qtile_start[bb] + 3) / 4;
    a.wide_list[before + qt / 4] = x;
    if (qt == 0 && a.qtile_start[b + 1] == a.total_qtiles) a.wide_list[a.total_qtiles] = before + (QT + 3) / 4;  // (the last sequence with tokens)
  }
}

// ---------------------------------------------------------------------------------------------
// k_bwd_dq2: the dQ kernel for head dimension 128 and four query heads per workgroup, with the data
// movement and instruction order of k_bwd_dkv2.  Eight waves (head g = wave / 2, query rows
// 32 (wave % 2) ..), two per SIMD, so that the vector and LDS instructions of one overlap the
// MFMAs of the other.  The K and V tiles of the key tiles whose pairs are all visible go through
// a ring of NST stages in the block layout described at k_bwd_dkv2 (4 loads per wave and stage),
// one bare barrier per tile in its middle; a tile is 48 slots: S^T = K Q^T and dP^T = V dO^T of
// the two 32-key halves (32 MFMAs, 16-byte row reads), then dQ^T += K^T dS^T of the two halves
// (16 MFMAs, transposing reads), with the exponentials of half 0 under the score MFMAs of half 1
// and those of half 1 under the dQ MFMAs of half 0.  The masked and ragged tiles follow in a second
// such loop when a node has one visibility word (Eq. 3 of the tile as one 64-bit word per lane, a
// lane being a query row here: tile_visibility over the node ids of the tile's keys, which ride
// the ring as a fifth load), else in the general walk.
namespace dq2 {
constexpr int NST = 4, NSLOT = 48;
constexpr int PF = 4;                // operands in flight ahead of their MFMA
constexpr int BLK = dkv2::BLK, TILEB = dkv2::TILEB;
constexpr int ND = 2 * TILEB;        // node ids of the tile's keys [64] (masked tiles)
constexpr int STAGEB = ND + 256;     // K tile, V tile, node ids
constexpr int opnd_reads(int o) { return o < 32 ? 1 : 2; }
constexpr int issued_through(int k) {  // LDS reads issued up to and including those of operand k
  int t = 0;
  for (int o = 0; o <= k; ++o) t += opnd_reads(o);
  return t;
}
constexpr int wait_at(int i) {  // reads that may still be pending when MFMA i starts
  const int last = i + PF < NSLOT ? i + PF : NSLOT - 1;
  const int n = issued_through(last) - issued_through(i);
  return n < 15 ? n : 15;
}
constexpr int row_imm(int i) { return dkv2::row_imm(i); }  // half i / 16, k-step (i % 16) / 2, of K (even) or V (odd)
constexpr int tr_imm(int i) {  // i >= 32: K^T operand of key half (i - 32) / 8, 16-key group x, dims 32 db ..
  const int j = i - 32, hh = j / 8, x = (j % 8) / 4, db = j % 4;
  return (8 * hh + 4 * x) * BLK + db * 256;
}
}  // namespace dq2

// WIDE: the same workgroup turned by ninety degrees -- one query head on four consecutive query
// tiles (wave pair p takes tile 4 c + p), for the heads that do not fill a group of four: the
// waves still share every staged K / V tile.  The tile list is the one k_bwd_wide_rows wrote.
template <bool WIDE>
__global__ void __launch_bounds__(512) k_bwd_dq2(BwdArgs a) {
  using namespace dq2;
  constexpr int D = 128, HG = 4, NT = 512;
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
  typedef short v4i16 __attribute__((ext_vector_type(4)));
  typedef short v8i16 __attribute__((ext_vector_type(8)));
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int32_t sCol[MAX_ROW_LDS];
  __shared__ uint8_t sFlg[MAX_ROW_LDS];
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, L = lane & 31, H = lane >> 5;
  const int pair = w >> 1;  // (WIDE) which of the four query tiles
  DqTile t;
  int64_t wide_base = 0;
  if constexpr (!WIDE) {
    t = dq_tile(a);
  } else {
    const int groups = a.wide_list[a.total_qtiles];
    if ((int)blockIdx.x >= groups) return;  // (the whole workgroup: the launch is sized by a bound)
    const int x = a.wide_list[groups - 1 - (int)blockIdx.x];  // the long rows at the end of a sequence first
    const int b = dag_find_segment(a.qtile_start, a.n_seqs, x);
    const int qt = x - a.qtile_start[b];
    t.cu = a.cu_seqlens[b], t.T = a.cu_seqlens[b + 1] - t.cu, t.row0 = qt * BM, t.c0 = 0;
    t.N = a.wide_n[x], t.nfast = a.wide_nfast[x], t.nbase = a.node_start[b];
    wide_base = a.block_map_off[b] + (int64_t)qt * ((t.T + BN - 1) / BN);
  }
  const int hk = blockIdx.y, cu = t.cu, T = t.T;
  DqLane<D> me;
  if constexpr (!WIDE)
    dq_setup<D, HG>(a, t, hk, me);
  else
    dq_setup_at<D>(a, t, hk, a.dq_narrow + (int)blockIdx.z, true, t.row0 + BM * pair, me);
  f32x16 dQ[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dQ[db][e] = 0.f;
  TileList tl;
  tl.col = WIDE ? a.wide_col + wide_base : a.qtile_col + t.c0;
  tl.flag = WIDE ? a.wide_flag + wide_base : a.qtile_flag + t.c0;
  tl.fill<NT>(sCol, sFlg, t.N);
  __syncthreads();
  const int NF = t.nfast;  // entries 0 .. NF - 1 of the list: every pair visible, inside the sequence

  // ---- loads of one stage: wave w fetches blocks w and w + 8 of the K tile and of the V tile; for
  // masked tiles every wave also fetches the node ids of the keys (the same 256 bytes from all
  // eight: the number of loads a wave has in flight must not depend on the wave)
  const uint32_t row_stride = (uint32_t)(a.hkv * D);
  const uint32_t chunk8 = (uint32_t)(4 * (lane >> 4) + (lane & 3)) * 8;
  const int rsub = (lane >> 2) & 3;
  struct IssueCtx {
    const uint16_t *kb, *vb;
    uint32_t voff[2];
    const int32_t* nodes;  // this lane's key of the tile
  };
  auto prepare_issue = [&](int n, int n_end) __attribute__((always_inline)) {
    IssueCtx c;
    const int kv = n < n_end ? tl.tile(n) : 0;  // (past the end of the walk: the sequence's first tile, never consumed)
    const int j0 = kv * BN, n_in = min(BN, T - j0);
    const size_t slab = ((size_t)(cu + j0) * a.hkv + hk) * D;
    c.kb = a.k + slab;
    c.vb = a.v + slab;
#pragma unroll
    for (int i = 0; i < 2; ++i) c.voff[i] = (uint32_t)min(4 * (w + 8 * i) + rsub, n_in - 1) * row_stride + chunk8;
    c.nodes = a.tok_node + cu + j0 + min(lane, n_in - 1);
    return c;
  };
  auto issue_piece = [&](int p, const IssueCtx& c, int st) __attribute__((always_inline)) {
    unsigned char* const sb = smem + st * STAGEB;
    if (p < 4) {
      const int blk = w + 8 * (p & 1);
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)((p < 2 ? c.kb : c.vb) + c.voff[p & 1]),
                                       (lds_ptr_t)(sb + (p < 2 ? 0 : TILEB) + blk * BLK), 16, 0, 0);
    } else {
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)c.nodes, (lds_ptr_t)(sb + ND), 4, 0, 0);
    }
  };
  const uint32_t roff = (uint32_t)((L >> 2) * BLK + (L & 3) * 64 + H * 16);
  const uint32_t toff = (uint32_t)(((lane >> 5) & 1) * BLK + ((lane & 15) >> 2) * 64 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8);
  const uint32_t smem_base = lds_addr(smem);
  const float sc = a.sc, nl = -me.lse2, dl = me.dl;
  const int nq = me.ni, iq_row = me.i;
  const uint64_t vis0 = me.vis0;
  const bool row_ok = me.row_ok;

  // ---- one key tile, slot by slot; MSK: with Eq. 3 (one visibility word per node) and the end of the
  // sequence applied per element from the lane's visibility word of the tile
  // (with masks: vis_lo / vis_hi = this lane's visibility word of the tile, shifted so that bit
  // 32 hh + 8 (e / 4) + e % 4 belongs to element e of half hh, i.e. to key 64 kt + 4 H + that number)
  auto pipelined_tile = [&](auto msk_c, int cs, const IssueCtx& ictx, int is, uint32_t vis_lo, uint32_t vis_hi) __attribute__((always_inline)) {
    constexpr bool MSK = decltype(msk_c)::value;
    constexpr int LPS = MSK ? 5 : 4, PFM = PF;
    const uint32_t sbase = smem_base + (uint32_t)cs * STAGEB;
    const uint32_t ra = sbase + roff, ta = sbase + toff;
    bf16x8 op[NSLOT];
    v4i16 lo[NSLOT], hi[NSLOT];
    f32x16 S[2], dP[2];
    float dt[2][16];
    bf16x8 bds[2][2];
    auto fetch = [&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      const uint32_t r = ra, t = ta;  // (named here: captures inside discarded branches trip the compiler)
      bf16x8* const opp = op;
      v4i16* const lop = lo;
      v4i16* const hip_ = hi;
      if constexpr (i < 32)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(opp[i]) : "v"(r), "n"(row_imm(i)));
      else if constexpr (i < NSLOT)
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(lop[i]), "=&v"(hip_[i])
                     : "v"(t), "n"(tr_imm(i)), "n"(tr_imm(i) + 2 * BLK));
    };
    auto score = [&](auto hc, auto ec) __attribute__((always_inline)) {  // dS of key e of half h (this lane's row), packed in pairs
      constexpr int h = decltype(hc)::value, e = decltype(ec)::value;
      float p = __builtin_amdgcn_exp2f(fmaf(S[h][e], sc, nl));
      if constexpr (MSK) p = keep_if_bit<8 * (e >> 2) + (e & 3)>(p, h == 0 ? vis_lo : vis_hi);  // Eq. 3 and the end of the sequence
      dt[h][e] = p * (dP[h][e] - dl);
      if constexpr ((e & 1) == 1) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        const bf16x2 pk = __builtin_bit_cast(bf16x2, dag_pack_bf2(dt[h][e - 1], dt[h][e]));
        bds[h][e >> 3][(e & 7) - 1] = pk[0];
        bds[h][e >> 3][e & 7] = pk[1];
      }
    };
    static_for<0, PFM>(fetch);
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NSLOT>([&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      if constexpr (i == 32) {
        wait_vmcnt_only<LPS>();        // this wave's loads of the next tile's stage have landed
        __builtin_amdgcn_s_barrier();  // (bare: a __syncthreads would drain the loads in flight)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
      }
      fetch(std::integral_constant<int, i + PFM>{});
      wait_lgkmcnt_only<wait_at(i)>();
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (i < 32) {
        constexpr int hh = i / 16, s = (i % 16) / 2;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if constexpr ((i & 1) == 0)
          S[hh] = mfma32(op[i], me.qf[s], s == 0 ? zero : S[hh]);
        else
          dP[hh] = mfma32(op[i], me.dof[s], s == 0 ? zero : dP[hh]);
      } else {
        constexpr int j = i - 32, hh = j / 8, x = (j % 8) / 4, db = j % 4;
        const v8i16 t8 = {lo[i][0], lo[i][1], lo[i][2], lo[i][3], hi[i][0], hi[i][1], hi[i][2], hi[i][3]};
        dQ[db] = mfma32(__builtin_bit_cast(bf16x8, t8), bds[hh][x], dQ[db]);
      }
      if constexpr (i >= 32 && i < 32 + LPS) issue_piece(i - 32, ictx, is);
      if constexpr (i >= 16 && i < 32) score(std::integral_constant<int, 0>{}, std::integral_constant<int, i - 16>{});
      if constexpr (i >= 32 && i < 40) {
        score(std::integral_constant<int, 1>{}, std::integral_constant<int, 2 * (i - 32)>{});
        score(std::integral_constant<int, 1>{}, std::integral_constant<int, 2 * (i - 32) + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // ---- the pipelined walk over entries n0 .. n1 - 1 of the tile list
  auto ring_loop = [&](auto msk_c, int n0, int n1) __attribute__((always_inline)) {
    constexpr int LPS = decltype(msk_c)::value ? 5 : 4;
    if (n0 >= n1) return;
    int in = n0;  // list entry whose loads are issued next
#pragma unroll 1
    for (int st = 0; st < NST - 1; ++st, ++in) {
      const IssueCtx c = prepare_issue(in, n1);
#pragma unroll
      for (int p = 0; p < LPS; ++p) issue_piece(p, c, st);
    }
    wait_vmcnt_only<(NST - 2) * LPS>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int cs = 0, is = NST - 1;
    for (int n = n0; n < n1; ++n, ++in) {
      const IssueCtx ic = prepare_issue(in, n1);
      uint64_t vis = 0;
      if constexpr (decltype(msk_c)::value) {
        // the keys of the tile that this lane's row sees: own node up to the row itself
        // (WIDE: none at all when the wave pair's own query tile does not see the key tile -- the
        // few such tiles along the diagonal are multiplied through with zeros)
        const int kt = tl.tile(n);
        const int last = iq_row - kt * BN;  // last such key of the tile (may lie before or behind it)
        const uint64_t own = last < 0 ? 0ull : last >= 63 ? ~0ull : (2ull << last) - 1;
        vis = tile_visibility(smem_base + (uint32_t)cs * STAGEB + ND, lane, (uint32_t)nq, vis0, own, T - kt * BN);
        vis = row_ok ? vis >> (4 * H) : 0ull;
      }
      pipelined_tile(msk_c, cs, ic, is, (uint32_t)vis, (uint32_t)(vis >> 32));
      cs = cs + 1 == NST ? 0 : cs + 1;
      is = is + 1 == NST ? 0 : is + 1;
    }
    wait_vmcnt_only<0>();          // (the loads past the end of the walk)
    __builtin_amdgcn_s_barrier();  // every wave is done with the ring before it is filled again
    asm volatile("" ::: "memory");
  };
  ring_loop(std::false_type{}, 0, NF);
  // the masked and the ragged tiles: pipelined as well when a node has one visibility word, else the general walk
  const int NM = a.W == 1 ? t.N : NF;
  ring_loop(std::true_type{}, NF, NM);
  __syncthreads();  // the ring is free: the general walk lays its own tiles over it
  dq_general_walk<D, NT>(a, smem, tl, NM, t.N, T, cu, hk, t.nbase, me, dQ, WIDE ? 2 * pair : -1);
  dq_store<D>(a, me, H, dQ);
}

template <int D, int HG>
int launch_dq(const BwdArgs& a, long total_qtiles, hipStream_t stream) {
  constexpr int sm = 2 * BN * (D + 8) * 2 + BN * 4;
  if (hipFuncSetAttribute((const void*)k_bwd_dq<D, HG>, hipFuncAttributeMaxDynamicSharedMemorySize, sm) != hipSuccess)
    return DAG_ERR_HIP;
  hipLaunchKernelGGL((k_bwd_dq<D, HG>), dim3((unsigned)total_qtiles, (unsigned)a.hkv, (unsigned)((a.G + HG - 1) / HG)),
                     dim3(128 * HG), sm, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

// Query heads per KV head that the dQ kernel takes one at a time on four query tiles.
int bwd_wide_heads(int G) { return G % 4; }

// Development switch, read once: DAGATTN_BWD_V1=1 runs the first dQ and dK/dV kernels for every shape.
bool bwd_first_version() {
  static const bool v = [] {
    const char* e = getenv("DAGATTN_BWD_V1");
    return e && e[0] == '1';
  }();
  return v;
}

template <int D>
int launch_bwd(const BwdArgs& args, long total_qtiles, long total_ktiles, hipStream_t stream) {
  BwdArgs a = args;
  constexpr int RPB = 256 / (D / 8);  // rows per workgroup of k_bwd_delta
  hipLaunchKernelGGL((k_bwd_delta<D>), dim3((unsigned)((a.total_rows + RPB - 1) / RPB)), dim3(256), 0, stream, a);
  const int total_tokens = (int)(a.total_rows / a.hq);
  hipLaunchKernelGGL(k_bwd_tokvis, dim3((unsigned)((total_tokens + 255) / 256)), dim3(256), 0, stream, a, total_tokens);
  DAG_LAUNCH_CHECK();
  int rc;
  a.dq_narrow = a.G;
  if (D == 128 && !bwd_first_version()) {
    // the heads left over by the groups of four take four query tiles each
    const int wide = bwd_wide_heads(a.G);
    a.dq_narrow = a.G - wide;
    constexpr int sm2 = dq2::NST * dq2::STAGEB;
    if (hipFuncSetAttribute((const void*)k_bwd_dq2<false>, hipFuncAttributeMaxDynamicSharedMemorySize, sm2) != hipSuccess ||
        hipFuncSetAttribute((const void*)k_bwd_dq2<true>, hipFuncAttributeMaxDynamicSharedMemorySize, sm2) != hipSuccess)
      return DAG_ERR_HIP;
    if (a.dq_narrow > 0)
      hipLaunchKernelGGL(k_bwd_dq2<false>, dim3((unsigned)total_qtiles, (unsigned)a.hkv, (unsigned)((a.dq_narrow + 3) / 4)),
                         dim3(512), sm2, stream, a);
    if (wide > 0) {
      hipLaunchKernelGGL(k_bwd_wide_rows, dim3((unsigned)total_qtiles), dim3(64), 0, stream, a);
      const long groups_bound = std::min(total_qtiles, (total_qtiles + 3) / 4 + a.n_seqs);
      hipLaunchKernelGGL(k_bwd_dq2<true>, dim3((unsigned)groups_bound, (unsigned)a.hkv, (unsigned)wide), dim3(512), sm2, stream, a);
    }
    rc = hipGetLastError() == hipSuccess ? DAG_OK : DAG_ERR_HIP;
  } else {
    rc = a.G >= 3 ? launch_dq<D, 4>(a, total_qtiles, stream)
                  : a.G == 2 ? launch_dq<D, 2>(a, total_qtiles, stream) : launch_dq<D, 1>(a, total_qtiles, stream);
  }
  if (rc != DAG_OK) return rc;
  constexpr int sm = dkv_smem_bytes<D>();
  if (hipFuncSetAttribute((const void*)k_bwd_dkv<D>, hipFuncAttributeMaxDynamicSharedMemorySize, sm) != hipSuccess)
    return DAG_ERR_HIP;
  hipLaunchKernelGGL(k_bwd_weights, dim3((unsigned)total_ktiles), dim3(64), 0, stream, a);
  hipLaunchKernelGGL(k_bwd_order, dim3((unsigned)total_ktiles), dim3(64), 0, stream, a);
  DAG_LAUNCH_CHECK();
  if (D == 128 && !bwd_first_version()) {
    constexpr int sm2 = dkv2::NST * dkv2::STAGEB;
    if (hipFuncSetAttribute((const void*)k_bwd_dkv2, hipFuncAttributeMaxDynamicSharedMemorySize, sm2) != hipSuccess)
      return DAG_ERR_HIP;
    hipLaunchKernelGGL(k_bwd_dkv2, dim3((unsigned)(total_ktiles * a.hkv)), dim3(256), sm2, stream, a);
  } else {
    hipLaunchKernelGGL((k_bwd_dkv<D>), dim3((unsigned)(total_ktiles * a.hkv)), dim3(256), sm, stream, a);
  }
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

// ---------------------------------------------------------------------------------------------
// fp32 backward: the accuracy path beside k_prefill_f32 (plain vector arithmetic, exact expf, the
// same 64 x 64 tiles and block map).  Four threads share a row (a query row in k_bwd_dq_f32, a key
// in k_bwd_dkv_f32), each owning a quarter of the head dimension.  Not a performance path.
struct BwdArgsF32 {
  const float *q, *k, *v, *out, *dout, *lse;
  float *dq, *dk, *dv, *delta;
  const int32_t *cu_seqlens, *node_start, *tok_node, *qtile_start, *ktile_start;
  const uint64_t* node_vis;
  const int64_t* block_map_off;
  const uint8_t* block_map;
  int n_seqs, W, hq, hkv, G;
  float scale;
};

__device__ __forceinline__ float quad_sum(float x) {  // over the four threads of a row
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

template <int D>
__global__ void __launch_bounds__(256) k_bwd_dq_f32(BwdArgsF32 a) {
  extern __shared__ float smem_f[];
  float* Ks = smem_f;            // [BN][D]
  float* Vs = smem_f + BN * D;   // [BN][D]
  int* s_node = (int*)(Vs + BN * D);
  constexpr int DP = D / 4;
  const int qt = blockIdx.x, head = blockIdx.y, hk = head / a.G;
  const int b = dag_find_segment(a.qtile_start, a.n_seqs, qt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int qtl = qt - a.qtile_start[b], KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b] + (int64_t)qtl * KT;
  const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
  const int i = qtl * BM + r, ic = min(i, T - 1);
  const int ni = a.tok_node[cu + ic];
  const uint64_t* vis_row = a.node_vis + (int64_t)(a.node_start[b] + ni) * a.W;
  const size_t row = (size_t)(cu + ic) * a.hq + head;
  float qr[DP], dor[DP], dq[DP];
  float dl = 0.f;
#pragma unroll
  for (int d = 0; d < DP; ++d) {
    qr[d] = a.q[row * D + part * DP + d];
    dor[d] = a.dout[row * D + part * DP + d];
    dl += dor[d] * a.out[row * D + part * DP + d];
    dq[d] = 0.f;
  }
  dl = quad_sum(dl);
  if (i < T && part == 0) a.delta[row] = dl;  // for the dK / dV kernel
  const float lse = a.lse[row];
  for (int kt = 0; kt < KT; ++kt) {
    const int flag = bm[kt];
    if (flag == 0) continue;
    const int j0 = kt * BN;
    __syncthreads();
    for (int idx = threadIdx.x; idx < BN * (D / 4); idx += 256) {
      const int rr = idx / (D / 4), c4 = idx % (D / 4);
      const size_t g = ((size_t)(cu + min(j0 + rr, T - 1)) * a.hkv + hk) * D + c4 * 4;
      *(f32x4*)(Ks + rr * D + c4 * 4) = *(const f32x4*)(a.k + g);
      *(f32x4*)(Vs + rr * D + c4 * 4) = *(const f32x4*)(a.v + g);
    }
    if (threadIdx.x < BN) s_node[threadIdx.x] = a.tok_node[cu + min(j0 + (int)threadIdx.x, T - 1)];
    __syncthreads();
    const int jn = min(BN, T - j0);
    for (int jj = 0; jj < jn; ++jj) {
      const int j = j0 + jj, nj = s_node[jj];
      const bool ok = flag == 2 || (nj == ni ? j <= i : (bool)((vis_row[nj >> 6] >> (nj & 63)) & 1));
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < DP; ++d) {
        s += qr[d] * Ks[jj * D + part * DP + d];
        dp += dor[d] * Vs[jj * D + part * DP + d];
      }
      s = quad_sum(s);
      dp = quad_sum(dp);
      if (ok) {
        const float ds = expf(s * a.scale - lse) * (dp - dl);
#pragma unroll
        for (int d = 0; d < DP; ++d) dq[d] += ds * Ks[jj * D + part * DP + d];
      }
    }
  }
  if (i < T)
#pragma unroll
    for (int d = 0; d < DP; ++d) a.dq[row * D + part * DP + d] = dq[d] * a.scale;
}

template <int D>
__global__ void __launch_bounds__(256) k_bwd_dkv_f32(BwdArgsF32 a) {
  extern __shared__ float smem_f[];
  float* Qs = smem_f;             // [BM][D]
  float* dOs = smem_f + BM * D;   // [BM][D]
  float* s_lse = dOs + BM * D;    // [BM]
  float* s_dl = s_lse + BM;       // [BM]
  int* s_node = (int*)(s_dl + BM);
  constexpr int DP = D / 4;
  const int kt = blockIdx.x, hk = blockIdx.y;
  const int b = dag_find_segment(a.ktile_start, a.n_seqs, kt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int ktl = kt - a.ktile_start[b];
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  const int nbase = a.node_start[b];
  const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
  const int j = ktl * BN + r, jc = min(j, T - 1);
  const int nj = a.tok_node[cu + jc];
  const size_t krow = (size_t)(cu + jc) * a.hkv + hk;
  float kr[DP], vr[DP], dk[DP], dv[DP];
#pragma unroll
  for (int d = 0; d < DP; ++d) {
    kr[d] = a.k[krow * D + part * DP + d];
    vr[d] = a.v[krow * D + part * DP + d];
    dk[d] = dv[d] = 0.f;
  }
  for (int qt = 0; qt < QT; ++qt) {
    const int flag = bm[(int64_t)qt * KT + ktl];
    if (flag == 0) continue;
    const int r0 = qt * BM;
    for (int g = 0; g < a.G; ++g) {
      const int head = hk * a.G + g;
      __syncthreads();
      for (int idx = threadIdx.x; idx < BM * (D / 4); idx += 256) {
        const int rr = idx / (D / 4), c4 = idx % (D / 4);
        const size_t o = ((size_t)(cu + min(r0 + rr, T - 1)) * a.hq + head) * D + c4 * 4;
        *(f32x4*)(Qs + rr * D + c4 * 4) = *(const f32x4*)(a.q + o);
        *(f32x4*)(dOs + rr * D + c4 * 4) = *(const f32x4*)(a.dout + o);
      }
      if (threadIdx.x < BM) {
        const size_t o = (size_t)(cu + min(r0 + (int)threadIdx.x, T - 1)) * a.hq + head;
        s_lse[threadIdx.x] = a.lse[o];
        s_dl[threadIdx.x] = a.delta[o];
        s_node[threadIdx.x] = a.tok_node[cu + min(r0 + (int)threadIdx.x, T - 1)];
      }
      __syncthreads();
      const int in = min(BM, T - r0);
      for (int ii = 0; ii < in; ++ii) {
        const int i = r0 + ii, ni = s_node[ii];
        bool ok = j < T;
        if (flag != 2 && ok)
          ok = nj == ni ? j <= i : (bool)((a.node_vis[(int64_t)(nbase + ni) * a.W + (nj >> 6)] >> (nj & 63)) & 1);
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < DP; ++d) {
          s += kr[d] * Qs[ii * D + part * DP + d];
          dp += vr[d] * dOs[ii * D + part * DP + d];
        }
        s = quad_sum(s);
        dp = quad_sum(dp);
        if (ok) {
          const float p = expf(s * a.scale - s_lse[ii]);
          const float ds = p * (dp - s_dl[ii]);
#pragma unroll
          for (int d = 0; d < DP; ++d) {
            dv[d] += p * dOs[ii * D + part * DP + d];
            dk[d] += ds * Qs[ii * D + part * DP + d];
          }
        }
      }
    }
  }
  if (j < T)
#pragma unroll
    for (int d = 0; d < DP; ++d) {
      a.dk[krow * D + part * DP + d] = dk[d] * a.scale;
      a.dv[krow * D + part * DP + d] = dv[d];
    }
}

template <int D>
int launch_bwd_f32(const BwdArgsF32& a, long total_qtiles, long total_ktiles, hipStream_t stream) {
  const int sm_q = 2 * BN * D * 4 + BN * 4, sm_k = 2 * BM * D * 4 + 3 * BM * 4;
  if (hipFuncSetAttribute((const void*)k_bwd_dq_f32<D>, hipFuncAttributeMaxDynamicSharedMemorySize, sm_q) != hipSuccess ||
      hipFuncSetAttribute((const void*)k_bwd_dkv_f32<D>, hipFuncAttributeMaxDynamicSharedMemorySize, sm_k) != hipSuccess)
    return DAG_ERR_HIP;
  hipLaunchKernelGGL((k_bwd_dq_f32<D>), dim3((unsigned)total_qtiles, (unsigned)a.hq), dim3(256), sm_q, stream, a);
  hipLaunchKernelGGL((k_bwd_dkv_f32<D>), dim3((unsigned)total_ktiles, (unsigned)a.hkv), dim3(256), sm_k, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

}  // namespace

extern "C" size_t dag_prefill_bwd_workspace_bytes(const dag_meta_t* m, int32_t hq, int32_t hkv, int32_t head_dim) {
  if (!m || hq < 1 || hkv < 1 || head_dim < 1 || m->sizes.total_tokens < 0 || m->sizes.total_qtiles < 0 ||
      m->sizes.total_ktiles < 0)
    return 0;
  // delta and -lse log2(e) [T][hq] fp32 each, weight and launch order of the key tiles, first visibility word per token
  size_t n = 2 * dag_align_up((size_t)m->sizes.total_tokens * hq * 4, 256) +
             2 * dag_align_up((size_t)m->sizes.total_ktiles * 4, 256) +
             dag_align_up((size_t)m->sizes.total_tokens * 8, 256) + 256;
  // head groupings that leave heads over (G not a multiple of four) at head dimension 128: the tile lists of the dQ
  // workgroups that take four query tiles (an int32 and a byte per entry of the dense block map,
  // three int32 per query tile)
  if (head_dim == 128 && hq % hkv == 0 && bwd_wide_heads(hq / hkv) > 0 && m->sizes.total_tiles >= 0)
    n += dag_align_up((size_t)m->sizes.total_tiles * 4, 256) + dag_align_up((size_t)m->sizes.total_tiles, 256) +
         3 * dag_align_up((size_t)(m->sizes.total_qtiles + 1) * 4, 256);
  return n;
}

extern "C" int dag_attn_prefill_bwd(const dag_meta_t* m, const void* q, const void* k, const void* v, const void* out,
                                    const void* dout, const float* lse, void* dq, void* dk, void* dv, int32_t hq,
                                    int32_t hkv, int32_t head_dim, float softmax_scale, dag_dtype_t dtype, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!m) return DAG_ERR_NULL;
  if (dtype != DAG_BF16 && dtype != DAG_F32) return DAG_ERR_UNSUPPORTED;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || (head_dim != 64 && head_dim != 128)) return DAG_ERR_UNSUPPORTED;
  if (m->tile_m != BM || m->tile_n != BN) return DAG_ERR_UNSUPPORTED;
  if (m->n_seqs < 0 || m->sizes.total_tokens < 0 || m->words_per_node < 1) return DAG_ERR_BAD_LEN;
  if (m->n_seqs == 0 || m->sizes.total_tokens == 0) return DAG_OK;
  if (!q || !k || !v || !out || !dout || !lse || !dq || !dk || !dv) return DAG_ERR_NULL;
  if (!m->cu_seqlens || !m->node_start || !m->tok_node || !m->node_vis || !m->qtile_start || !m->ktile_start ||
      !m->block_map_off || !m->block_map || !m->qtile_order || !m->qtile_desc || !m->qtile_col || !m->qtile_flag)
    return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k) || !dag_aligned16(v) || !dag_aligned16(out) || !dag_aligned16(dout) ||
      !dag_aligned16(dq) || !dag_aligned16(dk) || !dag_aligned16(dv))
    return DAG_ERR_ALIGN;
  if (m->sizes.total_tokens * (int64_t)hq > INT32_MAX) return DAG_ERR_UNSUPPORTED;
  if (m->sizes.total_qtiles != m->sizes.total_ktiles) return DAG_ERR_BAD_LEN;  // (both tilings are 64 rows)
  const size_t need = dag_prefill_bwd_workspace_bytes(m, hq, hkv, head_dim);
  if (!ws || ws_bytes < need) return DAG_ERR_WORKSPACE;
  if (dtype == DAG_F32) {
    BwdArgsF32 f;
    f.q = (const float*)q; f.k = (const float*)k; f.v = (const float*)v;
    f.out = (const float*)out; f.dout = (const float*)dout; f.lse = lse;
    f.dq = (float*)dq; f.dk = (float*)dk; f.dv = (float*)dv;
    f.delta = (float*)dag_align_up((size_t)(uintptr_t)ws, 256);
    f.cu_seqlens = m->cu_seqlens; f.node_start = m->node_start; f.tok_node = m->tok_node;
    f.qtile_start = m->qtile_start; f.ktile_start = m->ktile_start;
    f.node_vis = m->node_vis; f.block_map_off = m->block_map_off; f.block_map = m->block_map;
    f.n_seqs = m->n_seqs; f.W = m->words_per_node; f.hq = hq; f.hkv = hkv; f.G = hq / hkv;
    f.scale = softmax_scale;
    hipStream_t s32 = (hipStream_t)stream;
    return head_dim == 128 ? launch_bwd_f32<128>(f, m->sizes.total_qtiles, m->sizes.total_ktiles, s32)
                           : launch_bwd_f32<64>(f, m->sizes.total_qtiles, m->sizes.total_ktiles, s32);
  }
  BwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.out = (const uint16_t*)out; a.dout = (const uint16_t*)dout;
  a.lse = lse;
  a.dq = (uint16_t*)dq; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.delta = (float*)dag_align_up((size_t)(uintptr_t)ws, 256);
  a.nlse2 = (float*)((char*)a.delta + dag_align_up((size_t)m->sizes.total_tokens * hq * 4, 256));
  a.kt_weight = (int32_t*)((char*)a.nlse2 + dag_align_up((size_t)m->sizes.total_tokens * hq * 4, 256));
  a.kt_order = a.kt_weight + dag_align_up((size_t)m->sizes.total_ktiles * 4, 256) / 4;
  a.total_ktiles = (int)m->sizes.total_ktiles;
  a.tok_vis0 = (uint64_t*)(a.kt_order + dag_align_up((size_t)m->sizes.total_ktiles * 4, 256) / 4);
  a.wide_col = (int32_t*)((char*)a.tok_vis0 + dag_align_up((size_t)m->sizes.total_tokens * 8, 256));
  a.wide_flag = (uint8_t*)((char*)a.wide_col + dag_align_up((size_t)m->sizes.total_tiles * 4, 256));
  a.wide_n = (int32_t*)((char*)a.wide_flag + dag_align_up((size_t)m->sizes.total_tiles, 256));
  a.wide_nfast = a.wide_n + dag_align_up((size_t)(m->sizes.total_qtiles + 1) * 4, 256) / 4;
  a.wide_list = a.wide_nfast + dag_align_up((size_t)(m->sizes.total_qtiles + 1) * 4, 256) / 4;
  a.total_qtiles = (int)m->sizes.total_qtiles;
  a.dq_narrow = hq / hkv;
  a.cu_seqlens = m->cu_seqlens; a.node_start = m->node_start; a.tok_node = m->tok_node;
  a.qtile_start = m->qtile_start; a.ktile_start = m->ktile_start;
  a.qtile_order = m->qtile_order;
  a.qtile_desc = m->qtile_desc; a.qtile_col = m->qtile_col; a.qtile_flag = m->qtile_flag;
  a.node_vis = m->node_vis; a.block_map_off = m->block_map_off; a.block_map = m->block_map;
  a.n_seqs = m->n_seqs; a.W = m->words_per_node; a.hq = hq; a.hkv = hkv; a.G = hq / hkv;
  a.total_rows = (long)m->sizes.total_tokens * hq;
  a.scale = softmax_scale; a.sc = softmax_scale * LOG2E;
  hipStream_t s = (hipStream_t)stream;
  return head_dim == 128 ? launch_bwd<128>(a, m->sizes.total_qtiles, m->sizes.total_ktiles, s)
                         : launch_bwd<64>(a, m->sizes.total_qtiles, m->sizes.total_ktiles, s);
}
