// bf16 DAG attention prefill for gfx950 (paper Eq. 2 + Eq. 3), MFMA 32x32x16 with fp32 accumulation.
//
// Work decomposition.  A work item is one 64-row query tile of one KV head with HG of that KV
// head's query heads stacked: wave w handles the 32-row block w / HG of head w % HG, so every wave
// of the workgroup consumes the same K/V tiles.  With HG = 4 that is eight waves, two per SIMD, so
// that one wave's softmax (vector ALU) overlaps the other's MFMAs.  The kernel is persistent: the
// grid has one workgroup per CU slot and workgroup g processes items g, g + grid, ... of the
// launch list (sequences in order, heavy query tiles first).  The K/V stream of the next item is
// prefetched while the current one finishes; and because workgroups are placed round-robin on
// the eight XCDs, an XCD keeps working on one KV head of one sequence at a time, whose K/V then
// stay in its L2.
//
// Only the key tiles the block map lists are visited.  The CSR row of a query tile lists its FULL
// tiles first: those need no mask; PARTIAL tiles (and a ragged last tile) follow and evaluate the
// per-token mask.
//
// Data movement.  K tiles (64 keys x D) and V^T tiles (D x 64 keys, from a key-tile-wise
// transposed copy of V that a small pre-pass writes into the workspace) go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane, no staging registers) through a ring of
// NSTAGE buffers.  Bare s_barrier + explicit vmcnt waits keep up to NSTAGE-1 tiles in flight (a
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
// The MFMA A operand of both products is then one ds_read_b128 per instruction: LDS bandwidth, not
// the matrix pipe, is the scarce resource here (a 32x32x16 MFMA consumes a 1 KiB operand per wave
// every 32 cycles), which is why V is transposed once in global memory instead of with the slower
// LDS transpose loads.
//
// Register layout.  Scores are computed transposed, S^T = K Q^T, so that after the MFMA a lane
// holds one query row (lane % 32) and 16 keys of each 32-key block in registers: the softmax row
// reductions are in-register plus one exchange between the two half waves, and the probabilities
// already sit in the B-operand layout of the second product O^T = V^T P^T.  MFMA row i of a
// 32-key block is mapped to key pi(i) so that registers 0..7 / 8..15 of a score block hold 8
// consecutive keys.
//
// Softmax.  Online softmax in the log2 domain.  The running maximum is only raised when some row
// of the wave exceeds it by more than 2^8 (the accumulator rescale is then rare); probabilities
// may exceed 1 by that factor, which fp32 accumulation and the final division absorb exactly.
#include "common.h"
#include "prefill_launch.h"

namespace {

constexpr int TN = 64;
constexpr int TM = 64;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(8))) int i32x8;

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
                                                    const int32_t* __restrict__ cu_seqlens, int n_seqs, int hkv) {
  constexpr int LD = D + 8;  // padded row (elements)
  __shared__ __attribute__((aligned(16))) uint16_t s[TN * LD];
  const int tile = blockIdx.x, h = blockIdx.y;
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
  for (int c = threadIdx.x; c < D * (TN / 8); c += 256) {  // 16-byte piece c of the tile image
    const int d = 8 * (c / 64) + (c % 8), kc = (c / 8) % 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      w[e] = (uint32_t)s[(8 * kc + 2 * e) * LD + d] | ((uint32_t)s[(8 * kc + 2 * e + 1) * LD + d] << 16);
    *(u32x4*)(o + (size_t)c * 8) = u32x4{w[0], w[1], w[2], w[3]};
  }
}

// ---------------------------------------------------------------------------------------------
template <int D, int HG, int NSTAGE>
__global__ void __launch_bounds__(128 * HG, (HG == 4 ? 1 : 2)) k_prefill_bf16(PrefillArgs a) {
  constexpr int NW = 2 * HG;                 // waves: two 32-row blocks x HG heads
  constexpr int CH = D / 8;                  // 16-byte chunks per K row
  constexpr int KSTEPS = D / 16;             // MFMA steps of the score product
  constexpr int DB = D / 32;                 // 32-row blocks of O^T
  constexpr int KPB = 64 / CH;               // keys per K block
  constexpr int NBK = TN / KPB;              // K blocks per tile
  constexpr int NBV = D / 8;                 // V^T blocks per tile (8 output dimensions each)
  constexpr int IPK = NBK / NW, IPV = NBV / NW;  // blocks per tile and wave
  constexpr int LPT = IPK + IPV;             // loads per tile and wave
  constexpr int BLKK = 1024 + 16;            // block strides (skewed so that reads are conflict free)
  constexpr int BLKV = 1024 + 16 * 8;
  constexpr int KTILE = NBK * BLKK, VTILE = NBV * BLKV;
  constexpr float TH_LOG2 = 8.f;
  static_assert(IPK >= 1 && IPK * NW == NBK && IPV >= 1 && IPV * NW == NBV, "tile loads must divide over the waves");
  static_assert((NSTAGE - 1) * LPT < 64 && NSTAGE >= 2 && NSTAGE <= 4, "vmcnt range / ring depth");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* const Kbase = smem;                    // K[NSTAGE][KTILE]
  unsigned char* const Vbase = smem + NSTAGE * KTILE;   // V^T[NSTAGE][VTILE]

  const int G = a.hq / a.hkv;
  const int HS = G / HG;  // items per (query tile, KV head)
  const int nhw = a.hkv * HS;
  const long n_items = (long)a.total_qtiles * nhw;

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int L = lane & 31, H = lane >> 5;
  const int rb = w / HG, hj = w % HG;

  const uint16_t* qg = (const uint16_t*)a.q;
  const unsigned char* kg = (const unsigned char*)a.k;
  const unsigned char* vtg = (const unsigned char*)a.vt;
  const uint32_t rowbytes = (uint32_t)a.hkv * D * 2;

  auto load_item = [&](long it) {
    const int oi = (int)(it / nhw), hw = (int)(it % nhw);
    const int32_t* d = a.qtile_desc + (size_t)oi * 8;
    Item I;
    I.cu = d[0]; I.T = d[1]; I.row0 = d[2]; I.c0 = d[3]; I.N = d[4]; I.nfast = d[5]; I.nstart = d[6]; I.ktb = d[7];
    I.hk = hw / HS; I.hs = hw % HS;
    return I;
  };
  auto token_of = [&](const Item& I) { return I.cu + min(I.row0 + 32 * rb + L, I.T - 1); };
  auto head_of = [&](const Item& I) { return I.hk * G + I.hs * HG + hj; };

  // What this lane fetches in a wave-level load (LDS position 16*lane inside the block):
  //   K:   key (lane / 4) % KPB of the block, chunk 4 * (lane / (4 * KPB)) + lane % 4: four
  //        consecutive lanes fetch 64 consecutive bytes of one row (one cache-line lookup)
  //   V^T: piece `lane` of the block (the workspace copy already has the LDS order)
  const int kkey = (lane >> 2) % KPB;
  const uint32_t kchunk = (4 * (lane / (4 * KPB)) + (lane & 3)) * 16;
  const uint32_t ksrc = (w * KPB + kkey) * rowbytes + kchunk;
  const uint32_t vsrc = w * 1024 + lane * 16;

  auto issue_loads = [&](int buf, int cu, int T, int hk, int ktb, int kt) {
    const int j0 = kt * TN;
    const unsigned char* ktile = kg + ((size_t)(cu + j0) * a.hkv + hk) * (D * 2);
    const unsigned char* vtile = vtg + ((size_t)(ktb + kt) * a.hkv + hk) * (size_t)(D * TN * 2);
    unsigned char* kl = Kbase + buf * KTILE + w * BLKK;
    unsigned char* vl = Vbase + buf * VTILE + w * BLKV;
    if (j0 + TN <= T) {
#pragma unroll
      for (int i = 0; i < IPK; ++i)
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(ktile + (size_t)i * (NW * KPB) * rowbytes + ksrc),
                                         (lds_ptr_t)(kl + i * NW * BLKK), 16, 0, 0);
    } else {  // ragged last tile: rows past the end re-read the last valid row (masked later)
      const int last = T - 1 - j0;
#pragma unroll
      for (int i = 0; i < IPK; ++i) {
        const int rk = min((w + NW * i) * KPB + kkey, last);
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(ktile + (uint32_t)rk * rowbytes + kchunk),
                                         (lds_ptr_t)(kl + i * NW * BLKK), 16, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < IPV; ++i)  // the transposed copy is zero padded: no ragged case
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)(vtile + i * (NW * 1024) + vsrc),
                                       (lds_ptr_t)(vl + i * NW * BLKV), 16, 0, 0);
  };

  // LDS read addresses (bytes inside a tile); every other read of the tile is an immediate away.
  //   K, MFMA step s of key block kb:   koff + kb * (32 / KPB) * BLKK + (s / 2) * 64 * KPB + (s % 2) * 32
  //   V^T, key step st, output block db: voff + db * 4 * BLKV + st * 256
  const int krow = key_of_row(L);
  const uint32_t koff = (krow / KPB) * BLKK + (krow % KPB) * 64 + H * 16;
  const uint32_t voff = (L / 8) * BLKV + (L % 8) * 16 + H * 128;

  f32x16 O[DB];
  float m, l;
  auto reset_acc = [&]() {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
    m = -1e30f;
    l = 0.f;
  };
  reset_acc();
  const float sc = a.scale * 1.4426950408889634f;
  const float th = TH_LOG2 / sc;  // threshold in raw score units

  bf16x8 qf[KSTEPS];
  auto load_q = [&](const Item& I) {
    const uint16_t* qp = qg + ((size_t)token_of(I) * a.hq + head_of(I)) * D + 8 * H;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);
  };

  // LDS operand reads are issued a few MFMAs ahead of their use (software prefetch enforced with
  // scheduling groups), so that the LDS latency is hidden behind the matrix pipe.
  auto scores = [&](const unsigned char* Kb, f32x16* S) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
    // the two key blocks alternate so that consecutive MFMAs never depend on each other
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 kf = *(const bf16x8*)(Kb + koff + kb * (32 / KPB) * BLKK + (s >> 1) * 64 * KPB + (s & 1) * 32);
        S[kb] = mfma32(kf, qf[s], S[kb]);
      }
    constexpr int NM = 2 * KSTEPS, PF = 4;
    __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
#pragma unroll
    for (int i = 0; i < NM - PF; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PF, 0);
  };

  // online softmax of one tile whose scores are in S: raises the running maximum (rarely) and
  // returns the probabilities as bf16 B operands
  auto softmax = [&](const f32x16* S, bf16x8* pb) {
    float bm = max3(S[0][0], S[0][1], S[0][2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) bm = max3(bm, S[0][r], S[0][r + 1]);
    bm = fmaxf(bm, S[0][15]);
#pragma unroll
    for (int r = 0; r < 16; r += 2) bm = max3(bm, S[1][r], S[1][r + 1]);
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    if (__builtin_amdgcn_ballot_w64(bm > m + th) != 0) {  // rare after the first tiles
      const float m_new = fmaxf(m, bm);
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * sc);
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[db][r] *= alpha;
    }
    const float msc = m * sc;
    float rowsum = 0.f;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      f32x8 p;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(fmaf(S[st >> 1][8 * (st & 1) + e], sc, -msc));
        rowsum += p[e];
      }
      pb[st] = __builtin_convertvector(p, bf16x8);
    }
    l += rowsum;
  };

  auto accumulate = [&](const unsigned char* Vb, const bf16x8* pb) {
#pragma unroll
    for (int st = 0; st < 4; ++st)  // keys 16*st + 8H .. +7
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 vf = *(const bf16x8*)(Vb + voff + db * 4 * BLKV + st * 256);
        O[db] = mfma32(vf, pb[st], O[db]);
      }
    constexpr int NM = 4 * DB, PF = 4;
    __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
#pragma unroll
    for (int i = 0; i < NM - PF; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PF, 0);
  };

  // ---------------------------------------------------------------- persistent loop over items
  long item = blockIdx.x;
  if (item >= n_items) return;
  Item cur = load_item(item);
  bool has_next = item + gridDim.x < n_items;
  Item nxt = has_next ? load_item(item + gridDim.x) : cur;

  // The K/V tile stream runs ahead of the computation, across the item boundary: `ti` tiles have
  // been issued, `tc` consumed; tile t lives in ring slot t % NSTAGE.
  int ti = 0, tc = 0;
  int iss_next = 0, iss_idx = 0;  // issue cursor: item (0 current / 1 next) and tile index in its row
  // the cursor's item, field by field (scalar registers)
  int is_cu = cur.cu, is_T = cur.T, is_c0 = cur.c0, is_N = cur.N, is_hk = cur.hk, is_ktb = cur.ktb;
  auto cursor_enter = [&](const Item& I) {
    is_cu = I.cu; is_T = I.T; is_c0 = I.c0; is_N = I.N; is_hk = I.hk; is_ktb = I.ktb;
    iss_idx = 0;
  };
  i32x8 colv = {0, 0, 0, 0, 0, 0, 0, 0};  // key-tile indices iss_idx & ~7 .. +7 of the cursor's row
  auto try_issue = [&]() {
    if (iss_idx >= is_N) {
      if (iss_next || !has_next) return false;
      iss_next = 1;
      cursor_enter(nxt);
    }
    const int cu = is_cu, T = is_T, c0 = is_c0, hk = is_hk, ktb = is_ktb;
    // Scalar load of the key-tile indices, eight at a time so that the load latency is paid once
    // per eight tiles (the compiler would use a vector load here, whose wait drains the K/V
    // prefetches, because it cannot prove the table is not written by the kernel).  The table
    // has eight spare entries at its end, so the load never leaves it.
    const int sub = iss_idx & 7;
    if (sub == 0) {
      const int32_t* cp = a.col + __builtin_amdgcn_readfirstlane(c0 + iss_idx);
      asm volatile("s_load_dwordx8 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(colv) : "s"(cp) : "memory");
    }
    int kt = colv[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) kt = (sub == e) ? colv[e] : kt;
#if defined(DAGATTN_ABL) && (DAGATTN_ABL & 16)
    kt = iss_idx;
#endif
#if defined(DAGATTN_ABL) && (DAGATTN_ABL & 8)
    (void)cu; (void)T; (void)hk; (void)ktb;
#else
    issue_loads(ti % NSTAGE, cu, T, hk, ktb, kt);
#endif
    ++ti;
    ++iss_idx;
    return true;
  };
#pragma unroll
  for (int p = 0; p < NSTAGE - 1; ++p) try_issue();
  load_q(cur);

  while (true) {
    const int i_row = cur.row0 + 32 * rb + L;  // row inside the sequence
    const int tok = token_of(cur), head = head_of(cur);
    const uint64_t* vis_row = nullptr;
    uint64_t vis0 = 0;
    if (cur.nfast < cur.N) {  // some tile of this item needs the per-token mask
      vis_row = a.node_vis + (int64_t)(cur.nstart + a.tok_node[tok]) * a.W;
      vis0 = vis_row[0];
    }

    // The Q rows were loaded with ordinary global loads; make them "arrive" here, outside the
    // tile loop, so that no conservative wait on them ends up inside it (that wait would also
    // drain the K/V prefetches every tile).
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) asm volatile("" ::"v"(qf[s]));
    for (int n = 0; n < cur.N; ++n) {
      if (ti == tc) try_issue();  // nothing in flight (only right after very short items)
      const int younger = ti - tc - 1;  // tiles issued after the one needed now
      if (NSTAGE > 3 && younger >= 3) wait_vmcnt<(NSTAGE > 3 ? 3 : 0) * LPT>();
      else if (NSTAGE > 2 && younger == 2) wait_vmcnt<(NSTAGE > 2 ? 2 : 0) * LPT>();
      else if (younger == 1) wait_vmcnt<LPT>();
      else wait_vmcnt<0>();
      // Bare barrier (no memory fence: __syncthreads would drain every outstanding prefetch).
      // Everyone's loads of tile tc have landed (each wave waited for its own above) and
      // everyone has left tile tc-1.
#if !defined(DAGATTN_ABL) || !(DAGATTN_ABL & 32)
      __builtin_amdgcn_s_barrier();
#endif
      asm volatile("" ::: "memory");
      while (ti - tc < NSTAGE && try_issue()) {
      }
      const int buf = tc % NSTAGE;
      f32x16 S[2];
      bf16x8 pb[4];
#ifdef DAGATTN_ABL  // development ablations: bit 0 no scores, 1 no softmax, 2 no accumulate
      if (DAGATTN_ABL & 1) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) S[kb][r] = (float)(n + r);
      } else {
        scores(Kbase + buf * KTILE, S);
      }
      if (n == cur.N - 1 && has_next) load_q(nxt);
      if (DAGATTN_ABL & 2) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = S[st >> 1][8 * (st & 1) + e];
          pb[st] = __builtin_convertvector(p, bf16x8);
        }
      } else {
        softmax(S, pb);
      }
      if (DAGATTN_ABL & 4) {
        O[0][0] += (float)pb[0][0];
      } else {
        accumulate(Vbase + buf * VTILE, pb);
      }
      ++tc;
      continue;
#endif
      scores(Kbase + buf * KTILE, S);
      if (n == cur.N - 1 && has_next) load_q(nxt);  // the Q registers are free from here on
      if (n >= cur.nfast) {
        const int j0 = a.col[__builtin_amdgcn_readfirstlane(cur.c0 + n)] * TN;
        const int32_t* tn = a.tok_node + cur.cu;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = j0 + 32 * kb + 16 * (r >> 3) + 8 * H + (r & 7);
            const int nj = tn[min(j, cur.T - 1)];
            const uint64_t word = (a.W == 1) ? vis0 : vis_row[nj >> 6];
            const bool ok = (j <= i_row) && (j < cur.T) && ((word >> (nj & 63)) & 1);
            S[kb][r] = ok ? S[kb][r] : -INFINITY;
          }
      }
      softmax(S, pb);
      accumulate(Vbase + buf * VTILE, pb);
      ++tc;
    }

    const float l_tot = l + __shfl_xor(l, 32);
    if (i_row < cur.T) {
      const float inv = 1.f / l_tot;
      uint16_t* og = (uint16_t*)a.out + ((size_t)tok * a.hq + head) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 o;
          o[0] = dag_pack_bf2(O[db][4 * r4] * inv, O[db][4 * r4 + 1] * inv);
          o[1] = dag_pack_bf2(O[db][4 * r4 + 2] * inv, O[db][4 * r4 + 3] * inv);
          *(u32x2*)(og + 32 * db + 8 * r4 + 4 * H) = o;
        }
      if (a.lse && H == 0) a.lse[(size_t)tok * a.hq + head] = m * a.scale + logf(l_tot);
    }
    if (!has_next) break;
    reset_acc();
    item += gridDim.x;
    cur = nxt;
    has_next = item + gridDim.x < n_items;
    if (has_next) nxt = load_item(item + gridDim.x);
    if (iss_next) iss_next = 0;  // the cursor was already in what is now the current item
    else cursor_enter(cur);      // (all tiles of the old item were issued: start of the new one)
  }
}

template <int D, int HG, int NSTAGE>
int launch_one(const PrefillArgs& a, int hs, hipStream_t stream) {
  constexpr int KPB = 64 / (D / 8);
  constexpr size_t sm = (size_t)NSTAGE * ((TN / KPB) * (1024 + 16) + (D / 8) * (1024 + 128));
  if (hipFuncSetAttribute((const void*)k_prefill_bf16<D, HG, NSTAGE>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sm) != hipSuccess)
    return DAG_ERR_HIP;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    return DAG_ERR_HIP;
  hipLaunchKernelGGL((k_vt_prepare<D>), dim3((unsigned)a.total_ktiles, (unsigned)a.hkv), dim3(256), 0, stream,
                     (const uint16_t*)a.v, (uint16_t*)a.vt, a.ktile_start, a.cu_seqlens, a.n_seqs, a.hkv);
  DAG_LAUNCH_CHECK();
  const long n_items = (long)a.total_qtiles * a.hkv * hs;
  const long slots = (long)n_cu * (HG == 4 ? 1 : 2);
  const unsigned grid = (unsigned)(n_items < slots ? n_items : slots);
  hipLaunchKernelGGL((k_prefill_bf16<D, HG, NSTAGE>), dim3(grid), dim3(128 * HG), sm, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

template <int D>
int launch_d(const PrefillArgs& a, hipStream_t stream) {
  const int g = a.hq / a.hkv;
  if (g % 4 == 0) return launch_one<D, 4, 4>(a, g / 4, stream);  // 8 waves, one workgroup per CU
  if (g % 2 == 0) return launch_one<D, 2, 2>(a, g / 2, stream);  // 4 waves, two workgroups per CU
  return launch_one<D, 1, 2>(a, g, stream);                       // 2 waves per workgroup
}

}  // namespace

int launch_prefill_bf16(const PrefillArgs& a, int head_dim, hipStream_t stream) {
  if (head_dim == 128) return launch_d<128>(a, stream);
  return launch_d<64>(a, stream);
}
