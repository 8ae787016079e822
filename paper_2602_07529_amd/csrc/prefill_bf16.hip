// bf16 DAG attention prefill for gfx950 (paper Eq. 2 + Eq. 3), MFMA 32x32x16 with fp32 accumulation.
//
// Work decomposition.  A work item is one query tile of one KV head with some of that KV head's
// query heads, eight waves, each wave one 32-row block of one head, so every wave of the workgroup
// consumes the same K/V tiles: 64-row tiles x 4 heads for full groups of four heads, 256-row tiles
// x 1 head for one or two heads left over (their rows over the key tiles are derived from the
// 64 x 64 block map, see k_wide_rows).  The kernel is persistent: the grid has one workgroup per
// CU; workgroup g processes items g and g + grid of the launch list (query tiles heavy first, the
// KV heads of a tile next to each other) and takes every further item from a counter, one item
// ahead of its use.  The K/V stream of the next item is prefetched while the current one finishes.
//
// Only the key tiles the block map lists are visited.  The CSR row of a query tile lists its FULL
// tiles first: after the first tile they run through a steady-state loop without any test but an
// after-the-fact overflow check; PARTIAL tiles (and a ragged last tile) follow and go through the
// general step with a per-token mask, leaving out the 32 x 32 blocks that the mask hides entirely.
//
// Software pipeline.  The matrix pipe and the vector ALU of a SIMD run concurrently only if one
// instruction stream feeds both, so a wave works in steps of half a key tile (32 keys) and each
// step interleaves three independent pieces:  scores of half g + 1 (MFMA),  the exponentials of
// half g (vector ALU),  and the P V product of half g - 1 (MFMA).  A step is written slot by slot
// (one LDS operand read, one MFMA, a few vector instructions) with a scheduling barrier after
// every slot, so the instruction order in the binary is the one written here.
//
// Data movement.  K tiles (64 keys x D) and V^T tiles (D x 64 keys, from a key-tile-wise
// transposed copy of V that a small pre-pass writes into the workspace) go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane, no staging registers) through a ring of
// NSTAGE buffers.  Bare s_barrier + explicit vmcnt waits keep the ring's loads in flight (a
// __syncthreads would drain them).  A wave-level load writes 1 KiB of consecutive LDS (a "block");
// which 16-byte chunk of which row a lane fetches is chosen so that (a) four consecutive lanes
// read 64 consecutive bytes of global memory (the texture path looks up one cache line per
// such group; with four lines per group the waves stall issuing their loads), (b) the 16-byte
// operand reads of the block are spread evenly over the LDS banks, and (c) their addresses are one
// register plus immediates for all reads of a tile:
//   K block = R keys x C chunks (R = 1024 / (2 D)), stride 1024 + 16 bytes:
//             [chunk / 4][key % R][chunk % 4][16 B]
//   V^T block = 8 output dimensions x 8 key groups, stride 1024 + 128 bytes: [key group][dim % 8][16 B]
//             (the workspace copy is stored in this order, so its loads are linear)
//
// Register layout.  Scores are computed transposed, S^T = K Q^T, so that after the MFMA a lane
// holds one query row (lane % 32) and 16 keys of the 32-key half in registers: the softmax row
// reductions are in-register plus one exchange between the two half waves, and the probabilities
// already sit in the B-operand layout of the second product O^T = V^T P^T.  MFMA row i of a
// 32-key block is mapped to key pi(i) so that registers 0..7 / 8..15 of a score block hold 8
// consecutive keys.
//
// Softmax.  Online softmax in the log2 domain on scores that are relative to a per-row reference
// maximum (the accumulator of the score product starts at minus the reference).  The reference is
// only raised when some row of the wave exceeds it by more than 2^8 (general step) or when a row's
// probabilities of a half sum to 2^10 or more (steady state, found afterwards); probabilities may
// exceed 1 by such a factor, which fp32 accumulation and the final division absorb exactly.
#include <stdlib.h>
#include <type_traits>

#include "common.h"
#include "prefill_launch.h"

namespace {

constexpr int TN = 64;
constexpr int TM = 64;
constexpr int NSTAGE = 4;  // ring depth: two tiles in use by the pipeline, two in flight
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef std::true_type yes_t;
typedef std::false_type no_t;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// MFMA row i (0..31) of a 32-key block -> key index inside the block.
__device__ __forceinline__ int key_of_row(int i) {
  const int a = i >> 3, hh = (i >> 2) & 1, c = i & 3;
  return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N) only (gfx9 encoding)
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ void wait_lgkmcnt(int n) {  // s_waitcnt lgkmcnt(n) only, n = 0..3 (folds when n is constant)
  switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(0xC07F); break;
    case 1: __builtin_amdgcn_s_waitcnt(0xC17F); break;
    case 2: __builtin_amdgcn_s_waitcnt(0xC27F); break;
    case 3: __builtin_amdgcn_s_waitcnt(0xC37F); break;
    case 4: __builtin_amdgcn_s_waitcnt(0xC47F); break;
    case 5: __builtin_amdgcn_s_waitcnt(0xC57F); break;
    default: __builtin_amdgcn_s_waitcnt(0xC67F); break;
  }
}

__device__ __forceinline__ int sgpr(int x) { return __builtin_amdgcn_readfirstlane(x); }

// f(integral_constant<int, I>) for I = A .. B - 1, each a separate instantiation
template <int A, int B, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (A < B) {
    f(std::integral_constant<int, A>{});
    static_for<A + 1, B>(f);
  }
}

__device__ __forceinline__ uint32_t lds_addr(const void* p) {  // byte address inside LDS of a __shared__ pointer
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// LDS byte offsets of the MFMA operands inside a tile, after the per-lane part (koff / voff in the
// kernel, where the layouts are described): K operand of MFMA step s of key half h, and V^T
// operand of key step st (16 keys) for output block db.
template <int D, bool PAGED>
__device__ constexpr int k_imm(int h, int s) {
  constexpr int KPB = 64 / (D / 8), BLKK = 1024 + 16, IPK = (TN / KPB) / 8;
  return PAGED ? (4 * h + (s >> 1) / IPK + 8 * ((s >> 1) % IPK)) * BLKK + (s & 1) * 512
               : h * (32 / KPB) * BLKK + (s >> 1) * 64 * KPB + (s & 1) * 32;
}
template <int D, bool PAGED>
__device__ constexpr int v_imm(int st, int db) {
  constexpr int BLKV = 1024 + 16 * 8, IPV = (D / 8) / 8;
  return PAGED ? (2 * st + db / IPV + 8 * (db % IPV)) * BLKV : db * 4 * BLKV + st * 256;
}

struct Item {  // wave-uniform description of a work item
  int cu, T, row0, c0, N, nfast, nstart, ktb, hk, hs;
};


// ---------------------------------------------------------------------------------------------
// Pre-pass: V [T][hkv][D] -> V^T tiles [key tile][kv head][D / 8][8 key groups][8 dims][8 keys]
// (keys past the end of the sequence are zero): the tile is stored as the image it has in LDS, so
// the attention kernel streams it with fully linear reads.  One block per (key tile, kv head).
template <int D>
__global__ void __launch_bounds__(256) k_vt_prepare(const uint16_t* __restrict__ v, uint16_t* __restrict__ vt,
                                                    const int32_t* __restrict__ ktile_start,
                                                    const int32_t* __restrict__ cu_seqlens, int n_seqs, int hkv,
                                                    int32_t* __restrict__ sched) {
  constexpr int LD = D + 8;  // padded row (elements)
  __shared__ __attribute__((aligned(16))) uint16_t s[TN * LD];
  const int tile = blockIdx.x, h = blockIdx.y;
  if (tile == 0 && h == 0 && threadIdx.x < DAG_SCHED_INTS) sched[threadIdx.x] = 0;  // work counters of the attention kernel
  const int b = dag_find_segment(ktile_start, n_seqs, tile);
  const int T = cu_seqlens[b + 1] - cu_seqlens[b];
  const int j0 = (tile - ktile_start[b]) * TN;
  for (int c = threadIdx.x; c < TN * (D / 8); c += 256) {
    const int r = c / (D / 8), ch = c % (D / 8);
    u32x4 x = {0, 0, 0, 0};
    if (j0 + r < T) x = *(const u32x4*)(v + ((size_t)(cu_seqlens[b] + j0 + r) * hkv + h) * D + ch * 8);
    *(u32x4*)(s + r * LD + ch * 8) = x;
  }
  __syncthreads();
  uint16_t* o = vt + ((size_t)tile * hkv + h) * (size_t)(D * TN);
  // 16-byte piece c of the tile image = dimension d, keys 8 kc .. 8 kc + 7: a column of the staged
  // tile, fetched with the transposing LDS read (16 lanes point at four rows x 16 dimensions and
  // lane i of them receives dimension i of those four rows; two reads give the eight keys).
  typedef short v4i16 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) v4i16* lds_v4_t;
  const int p = threadIdx.x & 15;
  for (int g = threadIdx.x >> 4; g < (D / 16) * (TN / 8); g += 16) {
    const int dg = g % (D / 16), kc = g / (D / 16);
    const uint16_t* a0 = s + (8 * kc + (p >> 2)) * LD + 16 * dg + 4 * (p & 3);
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)a0);
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_t)(a0 + 4 * LD));
    const int d = 16 * dg + p, c = 64 * (d / 8) + 8 * kc + d % 8;
    typedef short v8i16 __attribute__((ext_vector_type(8)));
    *(v8i16*)(o + (size_t)c * 8) = v8i16{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
}

// 256-row query tiles.  Query heads that do not fill a four-head item are computed one head at a
// time on four stacked 64-row tiles of the block map (eight waves = eight 32-row blocks).  The row
// of such a tile over the key tiles follows from the dense map: a key tile is skipped when all
// four 64-row tiles skip it, needs no mask when all of them (those inside the sequence) are FULL,
// and takes the mask path otherwise.  Rows are stored like the 64-row ones (tiles without mask
// first, each class ascending), the row that starts at 64-row tile qt at position rowptr[qt] of
// its own column array: it cannot be longer than the four rows it is made of.  One wave per 64-row
// tile; those that start no 256-row tile mark themselves with a count of -1.
__global__ void __launch_bounds__(256) k_wide_rows(int n_seqs, int total_qtiles, const int32_t* __restrict__ qtile_start,
                                                   const int64_t* __restrict__ block_map_off,
                                                   const int32_t* __restrict__ cu_seqlens,
                                                   const int32_t* __restrict__ node_start,
                                                   const int32_t* __restrict__ ktile_start,
                                                   const uint8_t* __restrict__ block_map,
                                                   const int32_t* __restrict__ rowptr, int32_t* __restrict__ wide_cnt,
                                                   int32_t* __restrict__ wide_pre, int32_t* __restrict__ wide_col) {
  const int qt = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (qt >= total_qtiles) return;
  const int b = dag_find_segment(qtile_start, n_seqs, qt);
  const int ql = qt - qtile_start[b];
  if (ql % 4 != 0) {
    if (lane == 0) wide_cnt[qt] = -1;
    return;
  }
  const int T = cu_seqlens[b + 1] - cu_seqlens[b];
  const int KT = (T + TN - 1) / TN, QT = qtile_start[b + 1] - qtile_start[b];
  const int nsub = min(4, QT - ql);
  const uint8_t* rows = block_map + block_map_off[b] + (int64_t)ql * KT;
  const int c0 = rowptr[qt];
  int out = c0, nf = 0, last_full = -1;
  for (int pass = 0; pass < 2; ++pass) {
    for (int k0 = 0; k0 < KT; k0 += 64) {
      const int k = k0 + lane;
      bool any = false, all_full = true;
      if (k < KT)
        for (int i = 0; i < nsub; ++i) {
          const uint8_t f = rows[(int64_t)i * KT + k];
          any = any || f != DAG_TILE_SKIP;
          all_full = all_full && f == DAG_TILE_FULL;
        }
      const bool want = any && (pass == 0 ? all_full : !all_full);
      const uint64_t m = __ballot(want);
      if (want) wide_col[out + __popcll(m & ((1ull << lane) - 1))] = k;
      out += __popcll(m);
      if (pass == 0 && m) last_full = k0 + 63 - __builtin_clzll(m);
    }
    if (pass == 0) nf = out - c0;
  }
  if (lane != 0) return;
  if (nf > 0 && (last_full + 1) * TN > T) --nf;  // a ragged last key tile needs the mask path
  wide_cnt[qt] = out - c0;
  int32_t* d = wide_pre + (int64_t)qt * 8;
  d[0] = cu_seqlens[b];
  d[1] = T;
  d[2] = ql * 64;
  d[3] = c0;
  d[4] = out - c0;
  d[5] = nf;
  d[6] = node_start[b];
  d[7] = ktile_start[b];
}

// Launch order of the 256-row tiles: by descending tile count (ties: ascending index), as for the
// 64-row ones; also counts them.  One wave per 64-row tile.
__global__ void __launch_bounds__(256) k_wide_order(int total_qtiles, const int32_t* __restrict__ wide_cnt,
                                                    const int32_t* __restrict__ wide_pre,
                                                    int32_t* __restrict__ wide_desc, int32_t* __restrict__ wide_count) {
  const int qt = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (qt >= total_qtiles) return;
  const int mine = wide_cnt[qt];
  if (mine < 0 && qt != 0) return;
  int oi = 0, n = 0;
  for (int j = lane; j < total_qtiles; j += 64) {
    const int o = wide_cnt[j];
    oi += (o > mine) || (o == mine && j < qt);
    n += o >= 0;
  }
  for (int off = 32; off; off >>= 1) {
    oi += __shfl_xor(oi, off);
    n += __shfl_xor(n, off);
  }
  if (mine >= 0 && lane < 8) wide_desc[(int64_t)oi * 8 + lane] = wide_pre[(int64_t)qt * 8 + lane];
  if (qt == 0 && lane == 0) *wide_count = n;
}

// Work items of the paged prefill (section 4.3, phase II: the new tokens of a node are prefilled
// against the cached KV of its predecessors, which is only referenced, never copied).  One wave
// per (node, 64-row tile of its new tokens); slots past the node's last tile mark themselves with
// a count of -1.  The context of the node is cut into tiles of four pages in its own order; the
// row of a query tile lists the tiles up to the last row's own position, those that need no mask
// first (four full pages, all in front of the first row's position).  An entry is {four page
// ids, their token counts (one byte each), tile index, 0, 0}; pages past the end of the context
// repeat its first page with a count of zero, page ids are clamped to the pool.
__global__ void __launch_bounds__(256) k_paged_rows(int n_nodes, int qt_max, int nt_max, int n_pages,
                                                    const int32_t* __restrict__ q_off,
                                                    const int32_t* __restrict__ ctx_page_off,
                                                    const int32_t* __restrict__ ctx_pages,
                                                    const int32_t* __restrict__ ctx_page_len,
                                                    const int32_t* __restrict__ own_page,
                                                    const int32_t* __restrict__ own_len, int32_t* __restrict__ sched,
                                                    int32_t* __restrict__ cnt_out, int32_t* __restrict__ pre,
                                                    int32_t* __restrict__ tiles) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (blockIdx.x == 0 && threadIdx.x < DAG_SCHED_INTS) sched[threadIdx.x] = 0;  // work counters of the attention kernel
  if (slot >= n_nodes * qt_max) return;
  const int node = slot / qt_max, qt = slot % qt_max;
  const int n = q_off[node + 1] - q_off[node];
  const int p0 = ctx_page_off[node], np = ctx_page_off[node + 1] - p0;
  if (qt * TM >= n || np < 1) {
    if (lane == 0) cnt_out[slot] = -1;
    return;
  }
  const int nstart = own_page[node] * 16 + own_len[node] - n;  // context slot of the node's first new token
  const int lim_first = nstart + qt * TM, lim_last = nstart + min(qt * TM + TM - 1, n - 1);
  const int NT = min(min(lim_last / TN + 1, (np + 3) / 4), nt_max);
  int32_t* const row = tiles + (int64_t)slot * nt_max * 8;
  int out = 0, nf = 0;
  for (int pass = 0; pass < 2; ++pass) {
    for (int t0 = 0; t0 < NT; t0 += 64) {
      const int t = t0 + lane;
      int pg[4], ln[4];
      bool full = t < NT && t * TN + TN - 1 <= lim_first;
      for (int i = 0; i < 4; ++i) {
        const bool have = t < NT && 4 * t + i < np;
        pg[i] = min(max(ctx_pages[p0 + (have ? 4 * t + i : 0)], 0), n_pages - 1);
        ln[i] = have ? min(max(ctx_page_len[p0 + 4 * t + i], 0), 16) : 0;
        full = full && ln[i] == 16;
      }
      const bool want = t < NT && (pass == 0 ? full : !full);
      const uint64_t m = __ballot(want);
      if (want) {
        int32_t* e = row + (int64_t)(out + __popcll(m & ((1ull << lane) - 1))) * 8;
        for (int i = 0; i < 4; ++i) e[i] = pg[i];
        e[4] = ln[0] | ln[1] << 8 | ln[2] << 16 | ln[3] << 24;
        e[5] = t;
        e[6] = e[7] = 0;
      }
      out += __popcll(m);
    }
    if (pass == 0) nf = out;
  }
  if (lane != 0) return;
  cnt_out[slot] = out;
  int32_t* d = pre + (int64_t)slot * 8;
  d[0] = q_off[node];
  d[1] = n;
  d[2] = qt * TM;
  d[3] = slot * nt_max;
  d[4] = out;
  d[5] = nf;
  d[6] = nstart;
  d[7] = 0;
}

// ---------------------------------------------------------------------------------------------
#ifdef DAGATTN_TIMING
__device__ unsigned long long g_tlog[4096];
#endif
// PAGED: K and V^T tiles come from the paged pools of the decode path through a list of pages per
// work item instead of from the packed sequence (see k_paged_rows); the pipeline is the same.
template <int D, int HG, int NRG, bool PAGED>
__global__ void __launch_bounds__(64 * HG * NRG, 1) k_prefill_bf16(PrefillArgs a) {
  constexpr int RB = 1;                      // 32-row blocks per wave
  constexpr int NW = HG * NRG;               // waves: NRG row blocks x HG query heads
  constexpr int CH = D / 8;                  // 16-byte chunks per K row
  constexpr int KSTEPS = D / 16;             // MFMA steps of the score product
  constexpr int DB = D / 32;                 // 32-row blocks of O^T
  constexpr int KPB = 64 / CH;               // keys per K block
  constexpr int NBK = TN / KPB;              // K blocks per tile
  constexpr int NBV = D / 8;                 // V^T blocks per tile (8 output dimensions each)
  // Every wave issues its share of the K/V loads of a tile: the waves meet at a barrier once per
  // tile, so the tile takes as long as its slowest wave, and the load issue (with the cursor
  // arithmetic in front of it) is what makes a wave slow.
  constexpr int NISS = NW;
  constexpr int IPK = NBK / NISS, IPV = NBV / NISS;  // blocks per tile and issuing wave
  constexpr int LPT = IPK + IPV;             // loads per tile and wave
  constexpr int BLKK = 1024 + 16;            // block strides (skewed so that reads are conflict free)
  constexpr int BLKV = 1024 + 16 * 8;
  constexpr int KTILE = NBK * BLKK, VTILE = NBV * BLKV;
  constexpr float TH_LOG2 = 8.f;
  static_assert(IPK >= 1 && IPK * NISS == NBK && IPV >= 1 && IPV * NISS == NBV, "tile loads must divide over the waves");
  static_assert((NSTAGE - 2) * LPT < 64 && NSTAGE >= 3, "vmcnt range / ring depth");
  static_assert(!PAGED || NW == 8, "the paged tile layout is laid out for eight issuing waves");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* const Kbase = smem;                    // K[NSTAGE][KTILE]
  unsigned char* const Vbase = smem + NSTAGE * KTILE;   // V^T[NSTAGE][VTILE]
  unsigned char* const Abase = smem + NSTAGE * (KTILE + VTILE);  // node ids of the keys [NSTAGE][64]
  // after them: the two-slot item mailbox (16 bytes)

  // The launch covers query heads head0 .. head0 + heads - 1 of every KV head's group: HS items
  // of HG heads per (query tile, KV head), the last one padded when heads is no multiple of HG.
  // The number of query tiles is known to the host for the 64-row tiles of the block map and
  // read from the workspace for the 256-row tiles derived from it.
  const int G = a.hq / a.hkv;
  const int HS = (a.heads + HG - 1) / HG;
  const int nhw = a.hkv * HS;
  const long n_items = (long)(a.n_tiles_dev ? sgpr(*a.n_tiles_dev) : (int)a.total_qtiles) * nhw;

  const int tid = threadIdx.x, w = sgpr(tid >> 6), lane = tid & 63;
  const int L = lane & 31, H = lane >> 5;
  const int rg = w / HG, hj = w % HG;

  const uint16_t* qg = (const uint16_t*)a.q;
  const unsigned char* kg = (const unsigned char*)a.k;
  const unsigned char* vtg = (const unsigned char*)a.vt;
  const uint32_t rowbytes = (uint32_t)a.hkv * D * 2;

  // Work distribution.  The items are the (query tile, head group) pairs in launch order, the
  // head groups of a query tile next to each other; the list is sorted heavy first.  Workgroup b
  // takes items b and b + grid statically and every further one from a counter in the workspace,
  // so whoever is free next takes the heaviest item left (the compute units do not all run at the
  // same speed, and the items differ by more than a factor of ten).
  const int nb = (int)gridDim.x;
  const int my_rank = (int)blockIdx.x;
  const long n_list = n_items;
  int32_t* const ctr = a.sched;
  auto load_item = [&](long it) __attribute__((always_inline)) {
    const int oi = (int)(it / nhw), hw = (int)(it % nhw);
    const int32_t* d = a.qtile_desc + (size_t)oi * 8;
    Item I;
    I.cu = sgpr(d[0]); I.T = sgpr(d[1]); I.row0 = sgpr(d[2]); I.c0 = sgpr(d[3]);
    I.N = sgpr(d[4]); I.nfast = sgpr(d[5]); I.nstart = sgpr(d[6]); I.ktb = sgpr(d[7]);
    I.hk = sgpr(hw / HS); I.hs = sgpr(hw % HS);
    return I;
  };
  auto row_of = [&](const Item& I, int r) __attribute__((always_inline)) { return I.row0 + 32 * (rg * RB + r) + L; };  // row inside the sequence
  auto token_of = [&](const Item& I, int r) __attribute__((always_inline)) { return I.cu + min(row_of(I, r), I.T - 1); };
  // The waves beyond the last head of a padded item repeat that head (they load valid rows and
  // take part in every barrier) and store nothing.
  auto head_of = [&](const Item& I) __attribute__((always_inline)) { return I.hk * G + a.head0 + min(I.hs * HG + hj, a.heads - 1); };
  auto head_is_mine = [&](const Item& I) __attribute__((always_inline)) { return I.hs * HG + hj < a.heads; };

  // What this lane fetches in a wave-level load (LDS position 16*lane inside the block):
  //   K:   key (lane / 4) % KPB of the block, chunk 4 * (lane / (4 * KPB)) + lane % 4: four
  //        consecutive lanes fetch 64 consecutive bytes of one row (one cache-line lookup)
  //   V^T: piece `lane` of the block (the workspace copy already has the LDS order)
  // Addresses are a wave-uniform 64-bit base plus one 32-bit per-lane offset.
  // PAGED: a load fetches a 1 KiB piece of a page, the pools' layouts being what the MFMA operands
  // need: K piece = 4 chunks x 16 tokens x 16 bytes, fetched as it lies; V piece = 32 dimensions x
  // 16 tokens, of which LDS position u holds dimension 16 (u / 32) + u % 16, token half (u / 16) % 2
  // (the 16 lanes that read an operand together then read 256 consecutive bytes).
  const int kkey = (lane >> 2) % KPB;
  const uint32_t kchunk = (4 * (lane / (4 * KPB)) + (lane & 3)) * 16;
  const uint32_t ksrc = PAGED ? lane * 16 : kkey * rowbytes + kchunk;
  const uint32_t vsrc = PAGED ? (2 * (16 * (lane / 32) + lane % 16) + (lane / 16) % 2) * 16 : lane * 16;
  constexpr uint32_t VSTEP = PAGED ? 1024 : NISS * 1024;  // from a wave's V^T load to its next one
  // The steady state issues its loads without a decision: the row a lane fetches in K load i of
  // a tile (clamped to the tile's last valid row, which only matters in a ragged tile) and the
  // per-lane offset of V^T load i.
  int kvrow[IPK];
  uint32_t vvo[IPV];
#pragma unroll
  for (int i = 0; i < IPK; ++i) kvrow[i] = (w + NISS * i) * KPB + kkey;
#pragma unroll
  for (int i = 0; i < IPV; ++i) vvo[i] = (uint32_t)i * VSTEP + vsrc;

  // kbase / vbase: the cursor item's K rows (token cu, head hk) and V^T tiles (tile ktb, head hk,
  // this wave's block); the tile adds a multiple of its index.
  // PAGED: the pools' bases at the KV head and at this wave's pieces; the page adds a multiple of
  // its id (a page holds 16 tokens: D * 32 bytes per head in either pool).
  const uint32_t kt_kstride = PAGED ? (uint32_t)a.hkv * (D * 32) : (uint32_t)TN * rowbytes;
  const uint32_t kt_vstride = PAGED ? (uint32_t)a.hkv * (D * 32) : (uint32_t)a.hkv * (D * TN * 2);
  // Issuing a tile is split into a set-up (addresses of the tile, optional node-id record) and
  // LPT single loads, so that the pipeline can spread them over the slots of a step, in the
  // shadow of the MFMAs; issue_loads does all of it at once.
  // The tiles of all items of a workgroup form one stream; "group" g of the stream is the K tile g
  // together with the V^T tile g - 1: the scores of a tile are computed one tile before its P V
  // product, and the first K operands of the next tile are read at the end of the current one, so
  // K is needed a tile earlier than V^T.  Group g lives in K slot g % NSTAGE and V^T slot
  // (g - 1) % NSTAGE.  Every group has the same number of loads (the vmcnt waits count loads): the
  // first group of the stream fetches its own V^T tile into the slot in front of it, the last one
  // (V^T of the last tile) fetches that tile's K once more; neither copy is ever read.
  const unsigned char *p_ktile = nullptr, *p_vtile = nullptr;  // pending group (wave-uniform)
  const unsigned char* v_saved = nullptr;                      // V^T tile of the group issued last
  unsigned char *p_kl = nullptr, *p_vl = nullptr;
  int p_last = 0;
  bool p_ragged = false;
  auto issue_setup = [&](unsigned g, const unsigned char* kbase, const unsigned char* vbase, int cu, int T, int kt,
                         bool with_nodes) __attribute__((always_inline)) {
    const unsigned slot = g % NSTAGE, vslot = (g + NSTAGE - 1) % NSTAGE;
    const int j0 = kt * TN;
    if (!PAGED && with_nodes) {  // a tile that needs the mask: node ids of its 64 keys (every wave writes the same record)
      const int32_t* np = a.tok_node + cu + min(j0 + lane, T - 1);
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)np, (lds_ptr_t)(Abase + slot * 256), 4, 0, 0);
    }
    p_ktile = kbase + (uint64_t)(uint32_t)kt * kt_kstride;
    const unsigned char* const v_mine = vbase + (uint64_t)(uint32_t)kt * kt_vstride;
    p_vtile = g == 0 ? v_mine : v_saved;
    v_saved = v_mine;
    p_kl = Kbase + slot * KTILE + w * BLKK;
    p_vl = Vbase + vslot * VTILE + w * BLKV;
    p_ragged = !PAGED && j0 + TN > T;  // ragged last tile: rows past the end re-read the last valid row (masked later)
    p_last = PAGED ? TN - 1 : T - 1 - j0;
  };
  auto issue_setup_flush = [&](unsigned g) __attribute__((always_inline)) {  // the stream's last group: V^T of the last tile (its K once more)
    p_vtile = v_saved;
    p_kl = Kbase + (g % NSTAGE) * KTILE + w * BLKK;
    p_vl = Vbase + ((g + NSTAGE - 1) % NSTAGE) * VTILE + w * BLKV;
  };
  auto issue_part = [&](int i) __attribute__((always_inline)) {  // i = 0 .. LPT - 1, a compile-time constant at every call site
    if (i < IPK) {
      if (PAGED) {
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_ktile + (i * 1024 + ksrc)), (lds_ptr_t)(p_kl + i * NISS * BLKK), 16, 0, 0);
      } else if (!p_ragged) {
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_ktile + (size_t)((w + NISS * i) * KPB) * rowbytes + ksrc),
                                         (lds_ptr_t)(p_kl + i * NISS * BLKK), 16, 0, 0);
      } else {
        const int rk = min((w + NISS * i) * KPB + kkey, p_last);
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_ktile + ((uint32_t)rk * rowbytes + kchunk)),
                                         (lds_ptr_t)(p_kl + i * NISS * BLKK), 16, 0, 0);
      }
    } else {  // the transposed copy is zero padded: no ragged case
      const int iv = i - IPK;
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_vtile + (iv * VSTEP + vsrc)),
                                       (lds_ptr_t)(p_vl + iv * NISS * BLKV), 16, 0, 0);
    }
  };

  // LDS read addresses (bytes inside a tile); every other read of the tile is an immediate away.
  //   K, MFMA step s of key half h:      koff + h * (32 / KPB) * BLKK + (s / 2) * 64 * KPB + (s % 2) * 32
  //   V^T, key step st, output block db: voff + db * 4 * BLKV + st * 256
  // PAGED: wave w's load i of a tile (LDS block w + NISS i) is piece (w % 2) IPK + i of page w / 2,
  // so piece s of page p sits in block 2 p + s / IPK + NISS (s % IPK).  K chunk 2 s + H of key k:
  // page k / 16, piece s / 2, position (2 (s % 2) + H) 256 + (k % 16) 16; V^T dimensions of output
  // block db, keys of step st: page st, piece db, position 512 (L / 16) + 256 H + 16 (L % 16).
  const int krow = key_of_row(L);
  const uint32_t koff = PAGED ? 2 * (krow / 16) * BLKK + (krow % 16) * 16 + H * 256
                              : (krow / KPB) * BLKK + (krow % KPB) * 64 + H * 16;
  const uint32_t voff = PAGED ? (L / 16) * 512 + H * 256 + (L % 16) * 16 : (L / 8) * BLKV + (L % 8) * 16 + H * 128;

  f32x16 O[RB][DB];
  // Scores are kept relative to a reference maximum per row, in the exponent's units: the Q rows
  // are scaled by scale * log2(e) when they are loaded, and the accumulator of the score product
  // starts at -M (the C operand of its first MFMA), so a probability is exp2 of a score register
  // with no further arithmetic.  M is the reference (0 until a row has seen a key), negM holds -M
  // in all 16 registers of an accumulator.
  float M[RB], l[RB], bmax[RB];  // reference maximum, row sum, maximum of the last score half (relative to M)
  f32x16 negM[RB];
  bf16x8 P0[RB][2], P1[RB][2];  // probabilities of the two key halves (B operands)
  auto reset_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[r][db][e] = 0.f;
      M[r] = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) negM[r][e] = 0.f;
      l[r] = 0.f;
    }
  };
  reset_acc();
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        P0[r][j][e] = (__bf16)0.f;
        P1[r][j][e] = (__bf16)0.f;
      }
  const float sc = a.scale * 1.4426950408889634f;

  // The Q rows of an item: fetched as they are into the registers they stay in (all loads of a
  // row in flight together; with the scaling attached to each load the compiler handed them out
  // one by one, each behind a wait for the one before and for every tile load in flight), scaled
  // in place once they have arrived.
  bf16x8 qf[RB][KSTEPS];
  auto load_q = [&](const Item& I) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const uint16_t* qp = qg + ((size_t)token_of(I, r) * a.hq + head_of(I)) * D + 8 * H;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) qf[r][s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + 16 * s));
    }
  };
  auto scale_q = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const u32x4 raw = __builtin_bit_cast(u32x4, qf[r][s]);
        u32x4 scaled;
#pragma unroll
        for (int e = 0; e < 4; ++e) scaled[e] = dag_pack_bf2(dag_bf_lo(raw[e]) * sc, dag_bf_hi(raw[e]) * sc);
        qf[r][s] = __builtin_bit_cast(bf16x8, scaled);
      }
  };

  // row maxima of a half; true when some row of the wave exceeds its reference maximum by the
  // threshold (or lies that far below it while the row has not accumulated anything yet)
  auto row_max = [&](const f32x16* S) __attribute__((always_inline)) {
    bool need = false;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float bm = max3(S[r][0], S[r][1], S[r][2]);
#pragma unroll
      for (int e = 3; e < 15; e += 2) bm = max3(bm, S[r][e], S[r][e + 1]);
      bm = fmaxf(bm, S[r][15]);
      bmax[r] = bm;  // this lane's 16 keys only; the other half wave has the rest of the row
      need |= bm > TH_LOG2 || (l[r] == 0.f && bm < -TH_LOG2 && bm > -1e30f);
    }
    return __builtin_amdgcn_ballot_w64(need) != 0;
  };

  // Mask of the key tile whose scores are being computed, for PARTIAL and ragged tiles: bit j of
  // rmsk[r] says whether this lane's row r may see key j + 8 H of the tile (set by tile_mask in the
  // item loop); msk_on is wave-uniform and false for the tiles that need no mask.
  bool msk_on = false;
  bool msk_full[2] = {false, false};  // (wave-uniform) the mask of that key half hides nothing from this wave's rows
  // (wave-uniform) parts of a step that are wanted: a part whose 32 x 32 block of the mask hides
  // everything keeps its slots and operand reads (the read counters stay as they are) and leaves
  // out the arithmetic
  bool qk_on = true, pv_on = true, ex_on = true;
  uint64_t rmsk[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) rmsk[r] = 0;
  auto apply_mask = [&](f32x16* S, int half) __attribute__((always_inline)) {  // masked scores become -inf
#ifdef DAGATTN_ABL_NOAPPLY  // (development: timing without the mask application; results are wrong)
    return;
#endif
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const uint32_t word = half ? (uint32_t)(rmsk[r] >> 32) : (uint32_t)rmsk[r];
#pragma unroll
      for (int e = 0; e < 16; ++e) {  // this lane's key 32 half + 16 (e / 8) + 8 H + e % 8
        const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)word, 16 * (e >> 3) + (e & 7), 1);
        S[r][e] = __uint_as_float((__float_as_uint(S[r][e]) & keep) | (0xff800000u & ~keep));
      }
    }
  };

  // ---- one pipeline step, written slot by slot (a scheduling barrier after every slot keeps the
  // order): slot = the LDS read of the operand needed PF slots later, RB MFMAs on one operand,
  // and a share of the step's exponentials.  Pieces (each optional):
  //   QK: Sn[r]  = K_h Q_r^T      scores of key half HQ of the tile at Kb (first KSTEPS slots)
  //   PV: O[r]  += V_h^T Pp[r]    the 32 keys of half HV of the tile at Vb (last 2 DB slots)
  //   EX: Pc[r]  = exp2(Sc[r])    probabilities of a half (scores are relative to M), row sums added to l
  // `extra(slot, slots)` runs in every slot (used to issue the next K/V tile loads piecewise, in
  // the shadow of the MFMAs).
  // With QK, the row maxima of Sn are taken two slots after the last score MFMA (after the mask of
  // the tile, if it has one, has been applied to Sn) and the return value says whether they call
  // for a rescale.
  auto step = [&](auto qk_c, auto pv_c, auto ex_c, auto hq_c, auto hv_c, const unsigned char* Kb, f32x16* Sn,
                  const unsigned char* Vb, const bf16x8 (*Pp)[2], const f32x16* Sc, bf16x8 (*Pc)[2], auto&& extra) {
    constexpr bool QK = decltype(qk_c)::value, PV = decltype(pv_c)::value, EX = decltype(ex_c)::value;
    constexpr int HQ = decltype(hq_c)::value, HV = decltype(hv_c)::value;
    constexpr int NQ = QK ? KSTEPS : 0, NSLOT = NQ + (PV ? 2 * DB : 0), NU = EX ? 8 * RB : 0;
    constexpr int PF = 3;  // operand reads in flight ahead of the MFMA that uses them
    constexpr int MAXSLOT = NQ + 2 < NSLOT ? NQ + 2 : NSLOT;  // where the row maxima are taken
    bf16x8 opnd[NSLOT];
    float rs[RB];
    bool need = false;
#pragma unroll
    for (int r = 0; r < RB; ++r) rs[r] = 0.f;
    // The operand reads are inline assembly with explicit lgkmcnt waits: LDS reads return in
    // order, so before the MFMA of slot i exactly the reads of the slots after it may be pending
    // (the compiler's own bookkeeping waits for all of them, which exposes the LDS latency).
    const uint32_t kaddr = QK ? lds_addr(Kb) + koff : 0, vaddr = PV ? lds_addr(Vb) + voff : 0;
    auto fetch = [&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      const uint32_t ka = kaddr, va = vaddr;  // (named here: captures inside discarded branches trip the compiler)
      bf16x8* const op = opnd;
      if constexpr (i < NQ)
        asm volatile("ds_read_b128 %0, %1 offset:%2"
                     : "=v"(op[i])
                     : "v"(ka), "n"(k_imm<D, PAGED>(HQ, i)));
      else if constexpr (i < NSLOT)
        asm volatile("ds_read_b128 %0, %1 offset:%2"
                     : "=v"(op[i])
                     : "v"(va), "n"(v_imm<D, PAGED>(2 * HV + (i - NQ) / DB, (i - NQ) % DB)));
    };
    static_for<0, (PF < NSLOT ? PF : NSLOT)>(fetch);
    __builtin_amdgcn_sched_barrier(0);
    // (the slots are instantiated one by one, not left to the loop unroller: the immediate offsets
    // of the reads above have to be compile-time constants whatever `extra` contains)
    static_for<0, NSLOT>([&](auto ic) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      fetch(std::integral_constant<int, i + PF>{});
      wait_lgkmcnt(NSLOT - 1 - i < PF ? NSLOT - 1 - i : PF);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        if (i < NQ) {
          if (qk_on) Sn[r] = mfma32(opnd[i], qf[r][i < NQ ? i : 0], i == 0 ? negM[r] : Sn[r]);
        } else {
          if (pv_on) O[r][(i - NQ) % DB] = mfma32(opnd[i], Pp[r][(i - NQ) / DB], O[r][(i - NQ) % DB]);
        }
      }
      extra(i, NSLOT);
      if (QK && i == MAXSLOT && qk_on) {
        if (msk_on && !msk_full[HQ]) apply_mask(Sn, HQ);
        need = row_max(Sn);
      }
      if (ex_on)
#pragma unroll
      for (int u = i * NU / NSLOT; u < (i + 1) * NU / NSLOT; ++u) {  // two probabilities of one row
        const int r = u / 8, e = 2 * (u % 8);
        f32x2 p;
        p[0] = __builtin_amdgcn_exp2f(Sc[r][e]);
        p[1] = __builtin_amdgcn_exp2f(Sc[r][e + 1]);
        rs[r] += p[0] + p[1];
        asm volatile("" : "+v"(rs[r]));  // keep the running sum (no sum tree at the end of the step)
        const bf16x2 pk = __builtin_convertvector(p, bf16x2);
        Pc[r][e >> 3][e & 7] = pk[0];
        Pc[r][e >> 3][(e & 7) + 1] = pk[1];
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if (QK && MAXSLOT == NSLOT && qk_on) {
      if (msk_on && !msk_full[HQ]) apply_mask(Sn, HQ);
      need = row_max(Sn);
    }
    if (EX && ex_on) {
#pragma unroll
      for (int r = 0; r < RB; ++r) l[r] += rs[r];
    }
    return need;
  };
  typedef std::integral_constant<int, 0> h0_t;
  typedef std::integral_constant<int, 1> h1_t;
  auto nothing = [](int, int) {};
  // raise the running maxima to bmax and rescale everything accumulated so far, including the
  // probabilities that are still waiting for their P V product (rare after the first tiles)
  auto rescale = [&](f32x16* Sn) __attribute__((always_inline)) {  // Sn: the score half whose maxima called for it (still relative to the old M)
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      float d = fmaxf(bmax[r], __shfl_xor(bmax[r], 32));  // maximum of the half over the whole row, relative to M
      const bool fresh = l[r] + __shfl_xor(l[r], 32) == 0.f;  // nothing accumulated yet: M may go down too
      d = d > -1e30f ? (fresh ? d : fmaxf(d, 0.f)) : 0.f;      // (a half without a visible key leaves M alone)
      const float alpha = __builtin_amdgcn_exp2f(-d);
      M[r] += d;
      l[r] *= alpha;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        negM[r][e] -= d;
        Sn[r][e] -= d;
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[r][db][e] *= alpha;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        P0[r][j] = __builtin_convertvector(__builtin_convertvector(P0[r][j], f32x8) * alpha, bf16x8);
        P1[r][j] = __builtin_convertvector(__builtin_convertvector(P1[r][j], f32x8) * alpha, bf16x8);
      }
    }
  };
  // ---------------------------------------------------------------- persistent loop over items
  // Reporting done: the workgroup that finishes last puts the counters back to zero for the next
  // launch.  Relaxed on purpose: only the order of these atomic operations matters, and a release
  // would write back and invalidate the L2 under the workgroups that are still running.
  auto report_done = [&]() __attribute__((always_inline)) {
    int32_t* const done = a.sched + DAG_SCHED_INTS / 2;
    const bool last = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1;
    if (last) {
      __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return last;
  };
  // (a launch sized on the host has at most one workgroup per item; one sized on an upper bound
  // of the item count may have workgroups without any)
  if (my_rank >= n_list) {
    if (tid == 0) report_done();
    return;
  }
  Item cur = load_item(my_rank);
  bool has_next = (long)my_rank + nb < n_list;
  Item nxt = has_next ? load_item(my_rank + nb) : cur;
  // The last wave takes the items after the second from the counter, one item ahead: asked for
  // at the start of an item, handed to the other waves through `mbox` before its last tile.
  const bool grabber = w == NW - 1;
  int grabbed = 0;
  uint32_t* const mbox = (uint32_t*)(Abase + NSTAGE * 256);
  // after the mailbox: per wave, the piece of LDS that its output rows pass through
  constexpr int OROW = 64 + 16;
  unsigned char* const Obase = Abase + NSTAGE * 256 + 16 + w * (32 * OROW);
  int mslot = 0;

  // The K/V tile stream runs ahead of the computation, across the item boundary: `ti` groups have
  // been issued (group g = K tile g + V^T tile g - 1), tile `tc` is the one whose scores are being
  // computed; tile t lives in ring slot t % NSTAGE of its ring.
  unsigned ti = 0, tc = 0;
  bool flushed = false;  // the last group of the stream (V^T of its last tile) has been issued
  int iss_next = 0, iss_idx = 0;  // issue cursor: item (0 current / 1 next) and tile index in its row
  // The cursor's item, field by field (scalar registers), with the bases of its K rows and V^T
  // tiles, and 64 key-tile indices of its row in a vector register (lane e holds entry
  // (iss_idx & ~63) + e; a scalar or vector load inside the tile loop would drain the K/V
  // prefetches with its wait).  col_nxt is the same for the first 64 entries of the next item.
  int is_cu, is_T, is_c0, is_N, is_nfast, col_iss, col_nxt;
  const unsigned char *is_kbase, *is_vbase;
  // PAGED: an entry of the item's list is a tile of four pages {page ids, token counts (a byte
  // each), tile index in the context, -}; a wave only needs the page it fetches pieces of.
  auto col_at = [&](int c0, int N, int first) __attribute__((always_inline)) {
    const int e = c0 + min(first + lane, N - 1);
    return PAGED ? a.col[(size_t)e * 8 + (w >> 1)] : a.col[e];
  };
  auto load_cols = [&](const Item& I, int first) __attribute__((always_inline)) { return col_at(I.c0, I.N, first); };
  auto cursor_enter = [&](const Item& I, int cols) __attribute__((always_inline)) {
    is_cu = I.cu; is_T = I.T; is_c0 = I.c0; is_N = I.N; is_nfast = I.nfast;
    if (PAGED) {
      is_kbase = kg + (size_t)I.hk * (D * 32) + (w & 1) * (IPK * 1024);
      is_vbase = vtg + (size_t)I.hk * (D * 32) + (w & 1) * (IPV * 1024);
    } else {
      is_kbase = kg + ((size_t)I.cu * a.hkv + I.hk) * (D * 2);
      is_vbase = vtg + ((size_t)I.ktb * a.hkv + I.hk) * (size_t)(D * TN * 2) + w * 1024;
    }
    col_iss = cols;
    iss_idx = 0;
  };
  cursor_enter(cur, load_cols(cur, 0));
  col_nxt = has_next ? load_cols(nxt, 0) : 0;
  const bool issuer = w < NISS;
  // First half of issuing the next tile of the stream: cursor, tile index, addresses.  The LPT
  // loads follow through issue_part (at once in try_issue, slot by slot in the pipeline).
  auto try_issue_begin = [&]() __attribute__((always_inline)) {
    if (!issuer) return false;
    bool flush = false;
    if (iss_idx >= is_N) {
      if (iss_next) return false;  // (the item after the next one is not known yet)
      if (has_next) {
        iss_next = 1;
        cursor_enter(nxt, col_nxt);
      } else {                     // end of the stream: its last group
        if (flushed) return false;
        flushed = true;
        flush = true;
      }
    }
    if (flush) {
      issue_setup_flush(ti);
    } else {
      if ((iss_idx & 63) == 0 && iss_idx != 0) {  // rows with more than 64 tiles: next 64 entries
        col_iss = col_at(is_c0, is_N, iss_idx);
        asm volatile("" ::"v"(col_iss));  // the wait for this load belongs here, not on the common path
      }
      const int kt = __builtin_amdgcn_readlane(col_iss, iss_idx & 63);
      issue_setup(ti, is_kbase, is_vbase, is_cu, is_T, kt, iss_idx >= is_nfast);
      iss_idx = iss_idx + 1;
    }
    ti = ti + 1;
    return true;
  };
  auto try_issue = [&]() __attribute__((always_inline)) {
    if (!try_issue_begin()) return false;
#pragma unroll
    for (int i = 0; i < LPT; ++i) issue_part(i);
    return true;
  };
  // Moves on to the next tile of the stream: afterwards group tc + 1 (K tile tc + 1, whose first
  // operands are read at the end of tile tc, and V^T tile tc) is visible to the whole workgroup,
  // every wave has finished what it did before the call, and the ring slots that this frees are
  // refilled.  The pipeline reads K tiles tc and tc + 1 and V^T tile tc - 1, so groups up to
  // tc + NSTAGE - 1 may be in the rings.
#ifdef DAGATTN_TIMING
  unsigned long long tacc[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  unsigned long long t_mid = 0;
  const unsigned long long t_begin = __builtin_amdgcn_s_memrealtime();
  const unsigned long long c_begin = __builtin_amdgcn_s_memtime();  // shader clock
#define TSTAMP(x) const unsigned long long x = __builtin_amdgcn_s_memrealtime()
#define TACC(i, a0, a1) tacc[i] += (a1) - (a0)
#define TCOUNT(i) tacc[i] += 1
#else
#define TSTAMP(x)
#define TACC(i, a0, a1)
#define TCOUNT(i)
#endif
#if defined(DAGATTN_TIMING) && DAGATTN_TIMING >= 2  // stamps inside the tile loops (they disturb what they measure)
#define TSTAMP2(x) TSTAMP(x)
#define TACC2(i, a0, a1) TACC(i, a0, a1)
#else
#define TSTAMP2(x)
#define TACC2(i, a0, a1)
#endif
  auto sync_next = [&]() __attribute__((always_inline)) {
    ++tc;
    TSTAMP2(tw0);
    const int younger = (int)(ti - tc) - 2;  // groups issued after the one needed now (group tc + 1)
    if (!issuer) {
    } else if (younger >= 2) wait_vmcnt<2 * LPT>();
    else if (younger == 1) wait_vmcnt<LPT>();
    else wait_vmcnt<0>();
    TSTAMP2(tw1);
    TACC2(8, tw0, tw1);
    // Bare barrier (no memory fence: __syncthreads would drain every outstanding prefetch).
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    TSTAMP2(tw2);
    TACC2(9, tw1, tw2);
  };
  // One more tile into the slot that a sync_next has freed, spread over the slots of a pipeline step with NS slots (slot 1: set-up, the slots
  // after it: the loads), so that the scalar work and the load issue hide behind the MFMAs.
  // The texture path takes a 1 KiB load every 16 cycles at best, so the loads are spaced out: the
  // K loads over the first step of a tile, the V^T loads over the second.
  bool refill_pending = false;
  auto refill_slot = [&](int i, int NS) __attribute__((always_inline)) {  // first step: set-up in slot 1, K load x in slot 2 + x (NS - 2) / IPK
    if (i == 1) {
      refill_pending = (ti - tc < NSTAGE) && try_issue_begin();
    } else if (i >= 2 && refill_pending) {
#pragma unroll
      for (int x = 0; x < IPK; ++x)
        if (2 + x * (NS - 2) / IPK == i) issue_part(x);
    }
  };
  auto refill_slot_v = [&](int i, int NS) __attribute__((always_inline)) {  // second step: V^T load x in slot x NS / IPV
    if (refill_pending) {
#pragma unroll
      for (int x = 0; x < IPV; ++x)
        if (x * NS / IPV == i) issue_part(IPK + x);
    }
  };

#pragma unroll 1
  while (ti < NSTAGE && try_issue()) {
  }
  load_q(cur);
  // Row data for the mask: node of each row (rnode), word 0 of that node's visibility bitset
  // (vis0), and the nodes of the next item's rows, fetched one item ahead so that the dependent
  // vis0 load can go out together with the next Q rows.
  int rnode[RB], rnode_nxt[RB];
  uint64_t vis0[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) {
    rnode[r] = PAGED ? 0 : a.tok_node[token_of(cur, r)];
    rnode_nxt[r] = !PAGED && has_next ? a.tok_node[token_of(nxt, r)] : 0;
  }
#pragma unroll
  for (int r = 0; r < RB; ++r) vis0[r] = PAGED ? 0 : a.node_vis[(int64_t)(cur.nstart + rnode[r]) * a.W];
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  while (true) {
    // The Q rows and the row data were loaded with ordinary global loads; make them "arrive"
    // here, outside the tile loops, so that no conservative wait on them ends up inside (that
    // wait would also drain the K/V prefetches every tile).
#pragma unroll
    for (int r = 0; r < RB; ++r) {
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) asm volatile("" ::"v"(qf[r][s]));
      asm volatile("" ::"v"(vis0[r]), "v"(rnode_nxt[r]));
    }
    asm volatile("" ::"v"(col_iss), "v"(col_nxt));
    // Refill the rings (the cursor could not go past the end of the old `nxt`): group g goes into
    // the slots of K tile g - NSTAGE and V^T tile g - 1 - NSTAGE, both read for the last time before
    // the old item's last barrier.  Here, behind the arrival of the row data and not at the end of
    // the item before: that arrival waits for every load in flight, and these loads have the whole
    // first tile to land.
#pragma unroll 1
    while (ti - tc < NSTAGE && try_issue()) {
    }
    scale_q();
    TCOUNT(11);
    TSTAMP(t_top);
    if (grabber && has_next && lane == 0)  // the item after `nxt`; the answer is needed at the end of this item only
      grabbed = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    const int F = cur.nfast;
    f32x16 SA[RB], SB[RB];
    auto Kt = [&](unsigned t) __attribute__((always_inline)) { return Kbase + (t % NSTAGE) * KTILE; };
    auto Vt = [&](unsigned t) __attribute__((always_inline)) { return Vbase + (t % NSTAGE) * VTILE; };
    const yes_t Y;
    const no_t N_;
    const h0_t H0;
    const h1_t H1;
    const bf16x8 (*const nop)[2] = nullptr;

    // ---- PARTIAL tiles (and a ragged last tile) carry a per-token mask.  The mask of a row is built
    // as a 64-bit word over the keys of the tile: the key tile is cut into its node segments (node
    // ids come with the tile, through the ring) and each segment is switched on for the rows whose
    // node sees the segment's node (Eq. 3); the causal / length limit is one more AND.  Called
    // when tile n of the row (ring tile tc) has become visible, before its scores are masked.
    auto tile_mask = [&](int n, unsigned ring_tile, uint64_t* rm) __attribute__((always_inline)) {
#ifdef DAGATTN_ABL_NOTILEMASK  // (development: timing without the mask construction; results are wrong)
#pragma unroll
      for (int r = 0; r < RB; ++r) rm[r] = ~0ull;
      return;
#endif
      if constexpr (PAGED) {
        // A page of the context holds its first `count` tokens (a byte per page in the entry's word
        // 4); row i of the node's new tokens sees the slots of the context up to nstart + i (its
        // own position: everything in front belongs to its ancestors or to itself).
        int cw, tix;
        const int32_t* ep = a.col + (size_t)sgpr(cur.c0 + n) * 8 + 4;
        asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %2, 0x4\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(cw), "=&s"(tix)
                     : "s"(ep)
                     : "memory");
        uint64_t valid = 0;
#pragma unroll
        for (int p = 0; p < 4; ++p) valid |= ((1ull << ((cw >> (8 * p)) & 31)) - 1) << (16 * p);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
          const int cnt = cur.nstart + min(row_of(cur, r), cur.T - 1) - tix * TN + 1;
          const uint64_t lim = cnt >= 64 ? ~0ull : (cnt <= 0 ? 0ull : ((1ull << cnt) - 1));
          rm[r] = (valid & lim) >> (8 * H);
        }
        return;
      }
      int kt;
      const int32_t* cp = a.col + sgpr(cur.c0 + n);
      asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(kt) : "s"(cp) : "memory");
      const int j0 = kt * TN;
      // node of key j0 + lane (inline assembly: for a plain LDS read the compiler would first wait
      // for every global-to-LDS load in flight, i.e. drain the ring; the record of this tile has
      // landed, the barrier that published the tile covers it)
      int nj;
      asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                   : "=v"(nj)
                   : "v"(lds_addr(Abase + (ring_tile % NSTAGE) * 256 + lane * 4))
                   : "memory");
      const int prev = __shfl_up(nj, 1);
      uint64_t starts = __builtin_amdgcn_ballot_w64(lane == 0 || nj != prev);
      uint64_t rowmask[RB];
#pragma unroll
      for (int r = 0; r < RB; ++r) rowmask[r] = 0;
      while (starts) {  // wave-uniform loop over the node segments of the key tile
        const int s0 = __builtin_ctzll(starts);
        starts &= starts - 1;
        const int s1 = starts ? __builtin_ctzll(starts) : 64;
        const int ns = __builtin_amdgcn_readlane(nj, s0);
        const uint64_t range = (s1 == 64 ? ~0ull : ((1ull << s1) - 1)) & ~((1ull << s0) - 1);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
          uint64_t word = vis0[r];
          if (a.W != 1) {  // more than 64 nodes: fetch the word (the wait for it stays in this branch)
            word = a.node_vis[(int64_t)(cur.nstart + rnode[r]) * a.W + (ns >> 6)];
            asm volatile("" ::"v"(word));
          }
          if ((word >> (ns & 63)) & 1) rowmask[r] |= range;
        }
      }
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const int cnt = min(row_of(cur, r), cur.T - 1) - j0 + 1;  // keys j0 .. j0 + cnt - 1 are not in the future
        const uint64_t lim = cnt >= 64 ? ~0ull : (cnt <= 0 ? 0ull : ((1ull << cnt) - 1));
        rm[r] = (rowmask[r] & lim) >> (8 * H);
      }
    };
    // What a mask means for this wave's rows, per key half: hides everything (the half's score
    // MFMAs, exponentials and P V MFMAs can be left out), hides nothing (no need to apply it).
    auto mask_census = [&](const uint64_t* rm, bool* live, bool* full) __attribute__((always_inline)) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        bool some = false, gap = false;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
          const uint32_t mine = (uint32_t)(rm[r] >> (32 * h)) & 0x00ff00ffu;  // this lane's 16 keys of the half
          some |= mine != 0;
          gap |= mine != 0x00ff00ffu;
        }
        live[h] = __builtin_amdgcn_ballot_w64(some) != 0;
        full[h] = __builtin_amdgcn_ballot_w64(gap) == 0;
      }
    };

    // ---- every tile of the row goes through the software pipeline, in steps of half a tile;
    // the CSR row lists the tiles that need no mask first (F of them)
    // The mask of a tile is needed only after the score MFMAs of its first half, so it is built
    // inside that step, in the shadow of the MFMAs, and the two waves of a SIMD do it in different
    // slots (while one builds its mask the other one keeps the matrix pipe busy).
    const int NT = cur.N;
    const int mask_slot = w < NW / 2 ? KSTEPS - 2 : 0;  // (a slot of the score part: the first tile's step has no other)
    auto first_tile_extra = [&](int i, int) __attribute__((always_inline)) {
      if (msk_on && i == mask_slot) tile_mask(0, tc, rmsk);
    };
    msk_on = F == 0;
    msk_full[0] = msk_full[1] = false;
    if (step(Y, N_, N_, H0, H0, Kt(tc), SA, nullptr, nop, nullptr, nullptr, first_tile_extra)) rescale(SA);
    bool need = step(Y, N_, Y, H1, H0, Kt(tc), SB, nullptr, nop, SA, P0, nothing);
    TSTAMP(t_first);
    TACC(0, t_top, t_first);
    int n = 0;
    {
      // ---- the mask-free tiles after the first one: the steady state of the kernel.  One
      // straight run of 2 (KSTEPS + 2 DB) slots per tile with no test in it but the two overflow
      // checks; the operand reads run PF slots ahead of their MFMAs without a break, across the
      // two halves and into the next tile (whose K tile is published a tile ahead for that).
#ifndef DAGATTN_NOFAST
      if (1 < F) {
        constexpr int NS = KSTEPS + 2 * DB;
#ifdef DAGATTN_PF
        constexpr int PF = DAGATTN_PF, RING = DAGATTN_PF < 4 ? 4 : 8;
#else
        constexpr int PF = 3, RING = 4;
#endif
        static_assert((2 * NS) % RING == 0 && KSTEPS >= PF - 4 && PF < RING, "operand ring");
        if (need) rescale(SB);
        bf16x8 opr[RING];
        auto ffetch = [&](auto ic, uint32_t ka, uint32_t va, uint32_t kn) __attribute__((always_inline)) {  // operand of slot ic (2 NS ..: next tile)
          constexpr int i = decltype(ic)::value;
          bf16x8* const op = opr;
          if constexpr (i >= 2 * NS) {
            constexpr int q = i - 2 * NS;
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(op[i % RING]) : "v"(kn), "n"(k_imm<D, PAGED>(0, q)));
          } else if constexpr (i % NS < KSTEPS) {
            constexpr int st = i / NS, j = i % NS;
            asm volatile("ds_read_b128 %0, %1 offset:%2"
                         : "=v"(op[i % RING])
                         : "v"(ka), "n"(k_imm<D, PAGED>(st, j)));
          } else {
            constexpr int st = i / NS, j = i % NS - KSTEPS;
            asm volatile("ds_read_b128 %0, %1 offset:%2"
                         : "=v"(op[i % RING])
                         : "v"(va), "n"(v_imm<D, PAGED>(2 * st + j / DB, j % DB)));
          }
        };
        // The reference maximum is not looked after before the exponentials here: a row's sum of
        // the 16 probabilities a lane has just computed tells afterwards whether a score left the
        // range (a sum above 2^10, infinity or NaN); only then are the row maxima of that half
        // taken, the accumulators and the other half's scores shifted and the half's probabilities
        // computed again (they have not been used yet).  Sc: the scores the probabilities Pc came
        // from, Sn: the other half's scores (relative to the same reference), rs: this lane's sums.
        auto overflow_fix = [&](const f32x16* Sc, bf16x8 (*Pc)[2], f32x16* Sn, float* rs) __attribute__((always_inline)) {
#pragma unroll
          for (int r = 0; r < RB; ++r) {
            float bm = max3(Sc[r][0], Sc[r][1], Sc[r][2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) bm = max3(bm, Sc[r][e], Sc[r][e + 1]);
            bm = fmaxf(bm, Sc[r][15]);
            const float d = fmaxf(fmaxf(bm, __shfl_xor(bm, 32)), 0.f);  // the row's maximum relative to M (M never goes down here)
            const float alpha = __builtin_amdgcn_exp2f(-d);
            M[r] += d;
            l[r] *= alpha;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              negM[r][e] -= d;
              Sn[r][e] -= d;
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
              for (int e = 0; e < 16; ++e) O[r][db][e] *= alpha;
            rs[r] = 0.f;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
              f32x2 pp;
              pp[0] = __builtin_amdgcn_exp2f(Sc[r][e] - d);
              pp[1] = __builtin_amdgcn_exp2f(Sc[r][e + 1] - d);
              rs[r] += pp[0] + pp[1];
              const bf16x2 pk = __builtin_convertvector(pp, bf16x2);
              Pc[r][e >> 3][e & 7] = pk[0];
              Pc[r][e >> 3][(e & 7) + 1] = pk[1];
            }
          }
        };
        {
          const uint32_t kn = lds_addr(Kt(tc + 1)) + koff;
          static_for<0, (PF < KSTEPS ? PF : KSTEPS)>([&](auto ic) __attribute__((always_inline)) {
            ffetch(std::integral_constant<int, 2 * NS + decltype(ic)::value>{}, 0u, 0u, kn);
          });
        }
        // One tile of the steady state.  In one slot of its first half (the two waves of a SIMD
        // take different slots, so that one of them always feeds the matrix pipe) the wave moves
        // the cursor on: the common case -- a tile of the cursor's item that needs no mask, so it
        // is not ragged either, inside the 64 entries of the row the wave holds -- costs a handful
        // of scalar instructions; anything else is left to the general code after the tile
        // (`other` set).  In its second half the tile always issues this wave's LPT loads of the
        // group that p_ktile / p_vtile / p_kl / p_vl / p_last describe, without a test: normally
        // the group that has just been set up; when none was (the rings are full, the stream has
        // ended, the general code issues its group itself) the last group once more, which puts
        // the bytes that are there already into the same places.
        const int setup_slot = w < NW / 2 || NW == 1 ? 1 : NS / 2 + 1;
        bool other = false;
        auto fast_tile = [&]() __attribute__((always_inline)) {
          const uint32_t ka = lds_addr(Kt(tc)) + koff, va = lds_addr(Vt(tc - 1)) + voff, kn = lds_addr(Kt(tc + 1)) + koff;
          float rs[RB], pprev[RB], plast[RB];  // sums, the even partner of a pair, the exponential of the slot before
#pragma unroll
          for (int r = 0; r < RB; ++r) rs[r] = pprev[r] = plast[r] = 0.f;
          // (operands KSTEPS .. PF - 1 of this tile, when the reads run further ahead than the K
          // operands of the next tile that the previous tile could fetch)
          static_for<(PF < KSTEPS ? PF : KSTEPS), PF>([&](auto ic) __attribute__((always_inline)) {
            ffetch(ic, ka, va, kn);
          });
          static_for<0, 2 * NS>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value, st = i / NS, j = i % NS;
            constexpr int ahead = i + PF < 2 * NS + KSTEPS ? PF : 2 * NS + KSTEPS - 1 - i;  // reads in flight after this slot's
            if constexpr (i + PF < 2 * NS + KSTEPS) ffetch(std::integral_constant<int, i + PF>{}, ka, va, kn);
            wait_lgkmcnt(ahead);
            __builtin_amdgcn_sched_barrier(0);
            f32x16* const Sn = st ? SB : SA;
            const f32x16* const Sc = st ? SA : SB;
            bf16x8 (*const Pp)[2] = st ? P1 : P0;
            bf16x8 (*const Pc)[2] = st ? P0 : P1;
#pragma unroll
            for (int r = 0; r < RB; ++r) {
              if constexpr (j < KSTEPS) Sn[r] = mfma32(opr[i % RING], qf[r][j < KSTEPS ? j : 0], j == 0 ? negM[r] : Sn[r]);
              else O[r][(j - KSTEPS) % DB] = mfma32(opr[i % RING], Pp[r][(j - KSTEPS) / DB], O[r][(j - KSTEPS) % DB]);
            }
            if constexpr (st == 0 && (j == 1 || j == NS / 2 + 1)) {
              if (j == setup_slot && ti - tc < NSTAGE) {
                if (iss_idx < is_nfast && ((iss_idx & 63) != 0 || iss_idx == 0)) {
                  const uint32_t kt = (uint32_t)__builtin_amdgcn_readlane(col_iss, iss_idx & 63);
                  p_ktile = is_kbase + (uint64_t)kt * kt_kstride;
                  p_vtile = v_saved;  // (ti > 0 here: the first tile of the stream never runs through this loop)
                  v_saved = is_vbase + (uint64_t)kt * kt_vstride;
                  p_kl = Kbase + (ti % NSTAGE) * KTILE + w * BLKK;
                  p_vl = Vbase + ((ti + NSTAGE - 1) % NSTAGE) * VTILE + w * BLKV;
                  p_ragged = false;
                  p_last = TN - 1;
                  iss_idx = iss_idx + 1;
                  ti = ti + 1;
                } else {
                  other = true;
                }
              }
            }
#ifndef DAGATTN_ABL_NOLOADS  // (development: timing without the steady state's loads; results are wrong)
            if constexpr (st == 1) {  // load x of the group (K first, then V^T) in slot x NS / LPT of the second half
              static_assert(LPT <= NS, "at most one load per slot");
              static_for<0, LPT>([&](auto xc) __attribute__((always_inline)) {
                constexpr int x = decltype(xc)::value;
                if constexpr (x * NS / LPT + (NS / LPT > 1 ? 1 : 0) == j) {
                  if constexpr (x < IPK) {
                    const uint32_t off = PAGED ? x * 1024 + ksrc : __umul24((uint32_t)min(kvrow[x], p_last), rowbytes) + kchunk;  // (rows and row sizes are far below 2^24)
                    __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_ktile + off), (lds_ptr_t)(p_kl + x * NISS * BLKK), 16, 0, 0);
                  } else {
                    __builtin_amdgcn_global_load_lds((gbl_ptr_t)(p_vtile + vvo[x - IPK]), (lds_ptr_t)(p_vl + (x - IPK) * NISS * BLKV), 16, 0, 0);
                  }
                }
              });
            }
#endif
#pragma unroll
            for (int r = 0; r < RB; ++r) {
#pragma unroll
              for (int e = j * 16 / NS; e < (j + 1) * 16 / NS; ++e) {
#ifdef DAGATTN_ABL_NOEXP  // (development: timing without the exponentials; results are wrong)
                const float pe = Sc[r][e];
#else
                const float pe = __builtin_amdgcn_exp2f(Sc[r][e]);
#endif
                rs[r] += plast[r];  // (the one before: its result is there, this one's is not yet)
                plast[r] = pe;
                asm volatile("" : "+v"(rs[r]));  // keep the running sum
                if (e & 1) {
                  const f32x2 pp = {pprev[r], pe};
                  const bf16x2 pk = __builtin_convertvector(pp, bf16x2);
                  Pc[r][e >> 3][(e & 7) - 1] = pk[0];
                  Pc[r][e >> 3][e & 7] = pk[1];
                } else {
                  pprev[r] = pe;
                }
              }
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (j == NS - 1) {
              bool over = false;
#pragma unroll
              for (int r = 0; r < RB; ++r) {
                rs[r] += plast[r];
                plast[r] = 0.f;
                over |= !(rs[r] < 1024.f);
              }
              if (__builtin_amdgcn_ballot_w64(over) != 0) overflow_fix(Sc, Pc, Sn, rs);
#pragma unroll
              for (int r = 0; r < RB; ++r) {
                l[r] += rs[r];
                rs[r] = 0.f;
              }
            }
          });
        };
#pragma unroll 1
        for (; n + 1 < F; ++n) {
          TSTAMP2(tf0);
          sync_next();
          TSTAMP2(tf1);
          TACC2(1, tf0, tf1);
          fast_tile();
          if (other) {  // (a tile with a mask or a ragged one, the next item, the next 64 entries, the end of the stream)
            other = false;
            try_issue();
          }
          TSTAMP2(tf2);
          TACC2(3, tf1, tf2);
          TCOUNT(10);
          TCOUNT(7);
        }
        // The operands fetched ahead for a tile that takes the other path: nobody will use them, so
        // the compiler takes their registers for the temporaries of what follows -- which must not
        // start before these reads have written them (the scheduling barrier keeps it behind the wait).
        wait_lgkmcnt(0);
        __builtin_amdgcn_sched_barrier(0);
        need = row_max(SB);
        TSTAMP(t_fast);
        TACC(1, t_first, t_fast);
      }
#endif
    }
    // ---- the tiles with a mask.  The mask of a tile is built a tile ahead (its node ids are in
    // the ring by then, the K tiles being published a tile ahead), in a slot of the second half's
    // step, in the shadow of the MFMAs -- the two waves of a SIMD in different slots; only the
    // first one is built on the spot, after the barrier that publishes its tile -- so that
    // it is known before the tile's first step which of the wave's two 32 x 32 blocks of the tile
    // see nothing at all: such a block's score MFMAs, its exponentials a step later and its P V
    // MFMAs two steps later are left out (lvA / lvB / lvP0 / lvP1: whether SA, SB, P0, P1 hold
    // something that counts); the wave still takes part in the tile's barrier and load issue.
    uint64_t rm_nxt[RB];
    bool lvA = true, lvB = true, lvP0 = true, lvP1 = true;
    bool mask_built = false;  // rm_nxt holds the mask of the tile the loop turns to
    auto step_sel = [&](bool qk, bool pv, bool ex, auto qk_c, auto hq_c, auto hv_c, const unsigned char* Kb, f32x16* Sn,
                        const unsigned char* Vb, const bf16x8 (*Pp)[2], const f32x16* Sc, bf16x8 (*Pc)[2],
                        auto&& extra) __attribute__((always_inline)) {
      qk_on = qk;
      pv_on = pv;
      ex_on = ex;
      const bool nd = step(qk_c, Y, Y, hq_c, hv_c, Kb, Sn, Vb, Pp, Sc, Pc, extra);
      qk_on = pv_on = ex_on = true;
      return nd;
    };
#pragma unroll 1
    for (; n + 1 < NT; ++n) {
      sync_next();  // tile tc - 1 is the one in flight through the pipeline, tc the new one
      msk_on = n + 1 >= F;
      bool live[2] = {true, true};
      if (msk_on) {
        if (!mask_built) tile_mask(n + 1, tc, rm_nxt);
#pragma unroll
        for (int r = 0; r < RB; ++r) rmsk[r] = rm_nxt[r];
        mask_census(rmsk, live, msk_full);
      }
      const bool mask_ahead = n + 2 < NT && n + 2 >= F;
      mask_built = mask_ahead;
      auto second_half_extra = [&](int i, int NS) __attribute__((always_inline)) {
        if (mask_ahead && i == mask_slot) tile_mask(n + 2, tc + 1, rm_nxt);
        refill_slot_v(i, NS);
      };
      if (need) rescale(SB);
      need = step_sel(live[0], lvP0, lvB, Y, H0, H0, Kt(tc), SA, Vt(tc - 1), P0, SB, P1, refill_slot);
      lvA = live[0];
      lvP1 = lvB;
      if (need) rescale(SA);
      need = step_sel(live[1], lvP1, lvA, Y, H1, H1, Kt(tc), SB, Vt(tc - 1), P1, SA, P0, second_half_extra);
      lvB = live[1];
      lvP0 = lvA;
      TCOUNT(7);
    }
    msk_on = false;
    TSTAMP(t_loop);
    TACC(2, t_first, t_loop);
    // The item after `nxt`: the last wave publishes what the counter gave it (-1: the list is
    // exhausted).  Done here, in front of the item's last barrier, which makes it visible: a
    // wait on the answer placed later would also wait for the next item's Q rows or for the
    // output stores.  Two slots, used in turn: a wave may still have to read the one written an
    // item ago.
    if (grabber && has_next) {
      asm volatile("" ::"v"(grabbed));  // the wait for the counter's answer belongs here
      const long g = 2L * nb + __builtin_amdgcn_readfirstlane(grabbed);
      const int v = g < n_list ? (int)g : -1;
      asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(lds_addr(mbox + mslot)), "v"(v) : "memory");
    }
    TSTAMP(te0);
    sync_next();
    TSTAMP(te1);
    // The last scores of the item are done: the Q registers and the mask words are free for the
    // next item's rows (its node ids were loaded an item ago).  Placed after the loop above on
    // purpose (a load of the Q registers in front of it would make the compiler wait for
    // everything in flight there) and after the wait of sync_next, which counts tile loads only.
    if (has_next) {
      load_q(nxt);
      if (!PAGED) {
#pragma unroll
        for (int r = 0; r < RB; ++r) vis0[r] = a.node_vis[(int64_t)(nxt.nstart + rnode_nxt[r]) * a.W];
      }
    }
    if (need) rescale(SB);
    TSTAMP(te2);
    step_sel(true, lvP0, lvB, N_, H0, H0, nullptr, nullptr, Vt(tc - 1), P0, SB, P1, refill_slot);
    pv_on = lvB;  // (P1 comes from SB)
    step(N_, Y, N_, H0, H1, nullptr, nullptr, Vt(tc - 1), P1, nullptr, nullptr, refill_slot_v);
    pv_on = true;
    TSTAMP(t_p1);
    TACC(4, t_loop, t_p1);
    TACC(8, t_loop, te0);
    TACC(9, te0, te1);
    TACC(3, te1, te2);
    // ---- output.  A lane holds one row in 8-byte pieces (four consecutive dimensions).  Stored
    // as they are, a store instruction writes 16 bytes of each of 32 rows, 4096 such fragments per
    // item, and the stores took 3.7 us of the item (the compute units take the fragments one by
    // one).  So the rows go through a private piece of LDS, 32 dimensions at a time ([32 rows][64
    // bytes + 16 of padding]), and leave as 64-byte runs: four lanes per row, 16 rows per store.
    // LDS is reached by inline assembly only (plain accesses would make the compiler wait for
    // every tile load in flight); the piece belongs to this wave, so no barrier is involved.
    const int head = head_of(cur);
    const bool store = head_is_mine(cur);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      const float l_tot = l[r] + __shfl_xor(l[r], 32);
      const float inv = 1.f / l_tot;
      const bool mine = store && row_of(cur, r) < cur.T;
      if (a.lse && mine && H == 0)
        a.lse[(size_t)token_of(cur, r) * a.hq + head] = M[r] * 0.6931471805599453f + logf(l_tot);
      const uint32_t ow = lds_addr(Obase) + L * OROW + 8 * H;          // this lane's row in the piece
      const uint32_t ord = lds_addr(Obase) + (lane >> 2) * OROW + (lane & 3) * 16;  // row lane / 4 (+ 16), 16-byte part lane % 4
      uint16_t* orow[2];
      bool omine[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int rr = cur.row0 + 32 * (rg * RB + r) + 16 * jj + (lane >> 2);
        omine[jj] = store && rr < cur.T;
        orow[jj] = (uint16_t*)a.out + ((size_t)(cur.cu + min(rr, cur.T - 1)) * a.hq + head) * D + 8 * (lane & 3);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {  // dimensions 32 db + 8 r4 + 4 H .. + 3
          u32x2 o;
          o[0] = dag_pack_bf2(O[r][db][4 * r4] * inv, O[r][db][4 * r4 + 1] * inv);
          o[1] = dag_pack_bf2(O[r][db][4 * r4 + 2] * inv, O[r][db][4 * r4 + 3] * inv);
          asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(ow), "v"(o), "n"(16 * r4) : "memory");
        }
        u32x4 x0, x1;
        asm volatile("s_waitcnt lgkmcnt(0)\n\tds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:%3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(x0), "=&v"(x1)
                     : "v"(ord), "n"(16 * OROW)
                     : "memory");
#ifdef DAGATTN_ABL_NOSTORE  // (development: timing without the output stores; results are missing)
        asm volatile("" ::"v"(x0), "v"(x1));
#else
        if (omine[0]) *(u32x4*)(orow[0] + 32 * db) = x0;
        if (omine[1]) *(u32x4*)(orow[1] + 32 * db) = x1;
#endif
      }
    }
    TSTAMP(t_o);
    TACC(6, t_p1, t_o);
    if (!has_next) break;
    reset_acc();
    int after_next;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(after_next) : "v"(lds_addr(mbox + mslot)) : "memory");
    mslot ^= 1;
    after_next = sgpr(after_next);
    cur = nxt;
    has_next = after_next >= 0;
    if (has_next) nxt = load_item(after_next);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
      rnode[r] = rnode_nxt[r];
      if (!PAGED && has_next) rnode_nxt[r] = a.tok_node[token_of(nxt, r)];
    }
    if (iss_next) iss_next = 0;     // the cursor was already in what is now the current item
    else cursor_enter(cur, col_nxt);  // (all tiles of the old item were issued: start of the new one)
    if (has_next) col_nxt = load_cols(nxt, 0);
    TSTAMP(t_sw);
    TACC(5, t_o, t_sw);
  }
  // Every answer from the counters has arrived by now (each was waited for at the end of its
  // item), so this workgroup's requests were served before it reports itself done.
#ifdef DAGATTN_TIMING
  if (tid == 0) {  // begin, end and tile count of every workgroup, printed by the one that finishes last
    __hip_atomic_store(&g_tlog[blockIdx.x * 4 + 0], t_begin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&g_tlog[blockIdx.x * 4 + 1], __builtin_amdgcn_s_memrealtime(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&g_tlog[blockIdx.x * 4 + 2], tacc[7], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&g_tlog[blockIdx.x * 4 + 3], tacc[11], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0);
  }
#endif
  if (tid == 0) {
    if (report_done()) {
#ifdef DAGATTN_TIMING
      unsigned long long t0 = ~0ull;
      for (unsigned b = 0; b < gridDim.x; ++b) {
        const unsigned long long x = __hip_atomic_load(&g_tlog[b * 4], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t0 = x < t0 ? x : t0;
      }
      for (unsigned b = 0; b < gridDim.x; ++b)
        printf("blk %u begin %llu end %llu tiles %llu items %llu\n", b,
               __hip_atomic_load(&g_tlog[b * 4], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - t0,
               __hip_atomic_load(&g_tlog[b * 4 + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - t0,
               __hip_atomic_load(&g_tlog[b * 4 + 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
               __hip_atomic_load(&g_tlog[b * 4 + 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
#endif
    }
  }
#ifdef DAGATTN_TIMING
  if (blockIdx.x == 0 && lane == 0) {
    const unsigned long long t_end = __builtin_amdgcn_s_memrealtime();
    const unsigned long long c_end = __builtin_amdgcn_s_memtime();
    if (w == 0) printf("shader clock during the kernel: %.0f MHz\n", (double)(c_end - c_begin) / (double)(t_end - t_begin) * 100.0);
    printf("wave %d total %llu | first tile %llu tile loop %llu last tile + epilogue %llu out %llu switch %llu | tiles in the loop %llu items %llu epi: mailbox %llu sync %llu q+rescale %llu | fast tiles %llu fast loop %llu (epi q) %llu (x10ns)\n",
           w, t_end - t_begin, tacc[0], tacc[2], tacc[4], tacc[6], tacc[5], tacc[7], tacc[11], tacc[8], tacc[9], tacc[10], tacc[1], tacc[3]);
  }
#endif
}

// How a KV head's G query heads are divided: `narrow` heads in items of four heads x 64 rows (the
// last item padded when narrow is no multiple of 4), `wide` heads one at a time on 256 rows.  A
// padded item wastes (4 - narrow % 4) / 4 of its time, a 256-row tile takes the mask path in more
// of its tiles and idles more at the end of a short sequence; every left-over head goes wide (three
// of them measured against the padded item: 16 % less time on long fork-joins, the same on short
// random DAGs).
void split_heads(int g, int* narrow, int* wide) {
  static const int force = [] {
    const char* e = getenv("DAGATTN_WIDE_HEADS");  // development: 0 = never wide, 2 = one or two left-over heads only
    return e ? atoi(e) : -1;
  }();
  const int rem = g % 4;
  *wide = force == 0 ? 0 : (force == 2 && rem == 3) ? 0 : rem;
  *narrow = g - *wide;
}

template <int D, int HG, int NRG, bool PAGED = false>
int launch_one(const PrefillArgs& a, long max_tiles, hipStream_t stream) {
  constexpr int KPB = 64 / (D / 8);
  constexpr size_t sm = (size_t)NSTAGE * ((TN / KPB) * (1024 + 16) + (D / 8) * (1024 + 128) + 256) + 16 +
                        (size_t)HG * NRG * 32 * (64 + 16);  // rings + node-id records + item mailbox + output pieces
  if (hipFuncSetAttribute((const void*)k_prefill_bf16<D, HG, NRG, PAGED>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sm) != hipSuccess)
    return DAG_ERR_HIP;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    return DAG_ERR_HIP;
  const long n_items = max_tiles * a.hkv * ((a.heads + HG - 1) / HG);
  const unsigned grid = (unsigned)(n_items < n_cu ? n_items : n_cu);
  hipLaunchKernelGGL((k_prefill_bf16<D, HG, NRG, PAGED>), dim3(grid), dim3(64 * HG * NRG), sm, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

template <int D>
int launch_d(const PrefillArgs& a, hipStream_t stream) {
  int narrow, wide;
  split_heads(a.hq / a.hkv, &narrow, &wide);
  if (narrow > 0) {  // eight waves = 2 row blocks x 4 query heads
    PrefillArgs b = a;
    b.head0 = 0;
    b.heads = narrow;
    const int rc = launch_one<D, 4, 2>(b, (long)a.total_qtiles, stream);
    if (rc != DAG_OK) return rc;
  }
  if (wide > 0) {  // eight waves = 8 row blocks of one query head; starts when the launch above has ended
    PrefillArgs b = a;
    b.head0 = narrow;
    b.heads = wide;
    b.col = a.wide_col;
    b.qtile_desc = a.wide_desc;
    b.n_tiles_dev = a.wide_count;
    // (every sequence has at most a quarter of its 64-row tiles, rounded up, as 256-row tiles)
    return launch_one<D, 1, 8>(b, ((long)a.total_qtiles + 3) / 4 + a.n_seqs, stream);
  }
  return DAG_OK;
}

}  // namespace

template <int D>
int launch_prepare_v(const PrefillArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL((k_vt_prepare<D>), dim3((unsigned)a.total_ktiles, (unsigned)a.hkv), dim3(256), 0, stream,
                     (const uint16_t*)a.v, (uint16_t*)a.vt, a.ktile_start, a.cu_seqlens, a.n_seqs, a.hkv, a.sched);
  DAG_LAUNCH_CHECK();
  int narrow, wide;
  split_heads(a.hq / a.hkv, &narrow, &wide);
  if (wide > 0) {
    const unsigned nblk = (unsigned)((a.total_qtiles + 3) / 4);
    hipLaunchKernelGGL(k_wide_rows, dim3(nblk), dim3(256), 0, stream, a.n_seqs, (int)a.total_qtiles, a.qtile_start,
                       a.block_map_off, a.cu_seqlens, a.node_start, a.ktile_start, a.block_map, a.rowptr, a.wide_cnt,
                       a.wide_pre, a.wide_col);
    DAG_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_wide_order, dim3(nblk), dim3(256), 0, stream, (int)a.total_qtiles, a.wide_cnt, a.wide_pre,
                       a.wide_desc, a.wide_count);
    DAG_LAUNCH_CHECK();
  }
  return DAG_OK;
}

int launch_prefill_bf16_prepare_v(const PrefillArgs& a, int head_dim, hipStream_t stream) {
  return head_dim == 128 ? launch_prepare_v<128>(a, stream) : launch_prepare_v<64>(a, stream);
}

int launch_prefill_paged(const PagedPrefillArgs& pa, int head_dim, hipStream_t stream) {
  const int slots = pa.n_nodes * pa.qt_max;
  const unsigned nblk = (unsigned)((slots + 3) / 4);
  const PrefillArgs& a = pa.a;
  hipLaunchKernelGGL(k_paged_rows, dim3(nblk), dim3(256), 0, stream, pa.n_nodes, pa.qt_max, pa.nt_max, pa.n_pages,
                     pa.q_off, pa.ctx_page_off, pa.ctx_pages, pa.ctx_page_len, pa.own_page, pa.own_len, a.sched,
                     a.wide_cnt, a.wide_pre, a.wide_col);
  DAG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_wide_order, dim3(nblk), dim3(256), 0, stream, slots, a.wide_cnt, a.wide_pre, a.wide_desc,
                     a.wide_count);
  DAG_LAUNCH_CHECK();
  PrefillArgs b = a;
  b.col = a.wide_col;
  b.qtile_desc = a.wide_desc;
  b.n_tiles_dev = a.wide_count;
  // (query heads in items of four, the last item padded)
  return head_dim == 128 ? launch_one<128, 4, 2, true>(b, slots, stream) : launch_one<64, 4, 2, true>(b, slots, stream);
}

int launch_prefill_bf16(const PrefillArgs& a, int head_dim, hipStream_t stream) {
  if (head_dim == 128) return launch_d<128>(a, stream);
  return launch_d<64>(a, stream);
}
