// bf16 DAG attention prefill for gfx950 (paper Eq. 2 + Eq. 3), MFMA 32x32x16 with fp32 accumulation.
//
// Work decomposition.  A workgroup owns one 64-row query tile of one KV head and stacks HG of that
// KV head's query heads: wave w handles the 32-row block w / HG of head w % HG, so every wave of
// the workgroup consumes the same K/V tiles.  With HG = 4 that is eight waves, two per SIMD, so
// that one wave's softmax (vector ALU) overlaps the other's MFMAs.  Only the key tiles the block
// map lists are visited.  The CSR row of a query tile lists its FULL tiles first: those run in a
// loop that contains no mask code at all; the PARTIAL tiles (and a ragged last tile) follow in a
// second loop that evaluates the per-token mask.
//
// Data movement.  K and V tiles of 64 tokens go from global memory straight into LDS
// (global_load_lds, 16 bytes per lane, no staging registers) through a ring of NSTAGE buffers:
// the loads of the next NSTAGE-1 tiles are in flight while a tile is computed, one barrier per
// tile.  A wave-level load writes 1 KiB of consecutive LDS, so the bank-conflict-avoiding XOR
// swizzle is applied to the *source* address each lane fetches:
//   K tile [64 keys][D]  16-byte chunk c of key r is stored at chunk c ^ swzK(r)
//   V tile [64 keys][D]  16-byte chunk c of key r is stored at chunk c ^ swzV(r)
//
// Register layout.  Scores are computed transposed, S^T = K Q^T, so that after the MFMA a lane
// holds one query row (lane % 32) and 16 keys of each 32-key block in registers: the softmax row
// reductions are in-register plus one exchange between the two half waves, and the probabilities
// already sit in the B-operand layout of the second product O^T = V^T P^T.  MFMA row i of a
// 32-key block is mapped to key pi(i) so that registers 0..7 / 8..15 of a score block hold 8
// consecutive keys.  The V^T operand (8 keys of one output dimension per lane) is read from the
// row-major V tile with the LDS transpose load ds_read_tr16_b64.
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
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(8))) float f32x8;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// MFMA row i (0..31) of a 32-key block -> key index inside the block.
__device__ __forceinline__ int key_of_row(int i) {
  const int a = i >> 3, hh = (i >> 2) & 1, c = i & 3;
  return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}
template <int D>
__device__ __forceinline__ int swzK(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int swzV(int row) {
  return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1);
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // s_waitcnt vmcnt(N) only (gfx9 encoding)
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <int D, int HG, int NSTAGE>
__global__ void __launch_bounds__(128 * HG, (HG == 4 ? 1 : 2)) k_prefill_bf16(PrefillArgs a) {
  constexpr int NW = 2 * HG;                 // waves: two 32-row blocks x HG heads
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  constexpr int KSTEPS = D / 16;             // MFMA steps of the score product
  constexpr int DB = D / 32;                 // 32-row blocks of O^T
  constexpr int RPI = 64 / CH;               // tile rows covered by one wave-level load
  constexpr int IPW = TN / RPI / NW;         // wave-level loads per tile, tensor and wave
  constexpr int LPT = 2 * IPW;               // loads per tile and wave (K and V)
  constexpr int TILE_BYTES = TN * D * 2;
  constexpr float TH_LOG2 = 8.f;
  static_assert(IPW >= 1 && IPW * RPI * NW == TN, "tile loads must divide evenly over the waves");
  static_assert((NSTAGE - 2) * LPT < 64, "vmcnt range");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // layout: K[NSTAGE][TILE_BYTES], V[NSTAGE][TILE_BYTES]
  unsigned char* const Kbase = smem;
  unsigned char* const Vbase = smem + NSTAGE * TILE_BYTES;

  const int G = a.hq / a.hkv;
  const int HS = G / HG;  // workgroups per KV head
  const int nhw = a.hkv * HS;
  const int oi = blockIdx.x / nhw, hw = blockIdx.x % nhw;
  const int hk = hw / HS, hs = hw % HS;
  const int qt = a.qtile_order[oi];
  const int b = dag_find_segment(a.qtile_start, a.n_seqs, qt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int row0 = (qt - a.qtile_start[b]) * TM;

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int L = lane & 31, H = lane >> 5;
  const int rb = w / HG, hj = w % HG;
  const int head = hk * G + hs * HG + hj;
  const int i_row = row0 + 32 * rb + L;  // row inside the sequence
  const int tok = cu + min(i_row, T - 1);

  const uint16_t* qg = (const uint16_t*)a.q;
  const unsigned char* kg = (const unsigned char*)a.k;
  const unsigned char* vg = (const unsigned char*)a.v;
  const uint32_t rowbytes = (uint32_t)a.hkv * D * 2;

  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s)
    qf[s] = *(const bf16x8*)(qg + ((size_t)tok * a.hq + head) * D + 16 * s + 8 * H);

  // Source offsets of this lane's tile loads.  Load i of the wave covers rows RPI*(w + NW*i) ...;
  // when NW is a multiple of 4 the swizzle terms do not depend on i and one offset serves all.
  constexpr bool UNIFORM_SRC = (NW % 4 == 0);
  constexpr int NSRC = UNIFORM_SRC ? 1 : IPW;
  const int pos = lane % CH;
  uint32_t ksrc[NSRC], vsrc[NSRC];
#pragma unroll
  for (int i = 0; i < NSRC; ++i) {
    const int r = (w + NW * i) * RPI + lane / CH;
    ksrc[i] = r * rowbytes + ((pos ^ swzK<D>(r)) * 16);
    vsrc[i] = r * rowbytes + ((pos ^ swzV<D>(r)) * 16);
  }

  auto issue_loads = [&](int buf, int j0) {
    const unsigned char* kt = kg + ((size_t)(cu + j0) * a.hkv + hk) * (D * 2);
    const unsigned char* vt = vg + ((size_t)(cu + j0) * a.hkv + hk) * (D * 2);
    unsigned char* kl = Kbase + buf * TILE_BYTES + w * 1024;
    unsigned char* vl = Vbase + buf * TILE_BYTES + w * 1024;
    if (j0 + TN <= T) {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const size_t step = UNIFORM_SRC ? (size_t)i * (RPI * NW) * rowbytes : 0;
        const uint32_t ks = ksrc[UNIFORM_SRC ? 0 : i], vs = vsrc[UNIFORM_SRC ? 0 : i];
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(kt + step + ks), (lds_ptr_t)(kl + i * NW * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(vt + step + vs), (lds_ptr_t)(vl + i * NW * 1024), 16, 0, 0);
      }
    } else {  // ragged last tile: rows past the end re-read the last valid row (masked later)
      const int last = T - 1 - j0;
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int r = (w + NW * i) * RPI + lane / CH;
        const uint32_t rc = (uint32_t)min(r, last) * rowbytes;
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(kt + rc + ((pos ^ swzK<D>(r)) * 16)),
                                         (lds_ptr_t)(kl + i * NW * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(vt + rc + ((pos ^ swzV<D>(r)) * 16)),
                                         (lds_ptr_t)(vl + i * NW * 1024), 16, 0, 0);
      }
    }
  };

  // per-lane LDS read offsets (bytes inside a tile)
  const int krow = key_of_row(L);
  uint32_t koff[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) koff[s] = krow * (D * 2) + (((2 * s + H) ^ swzK<D>(krow)) * 16);
  // transpose read: within a 16-lane group, lane j = 4e + c addresses key e (of 4), 8-byte piece c
  const int tr_e = (lane & 15) >> 2, tr_c = lane & 3, dhalf = (lane >> 4) & 1;
  uint32_t voff[2][DB];  // [rd][db]: keys 8H + 4rd + e of the first 16-key step; a step adds 16 rows
#pragma unroll
  for (int rd = 0; rd < 2; ++rd)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int key = 8 * H + 4 * rd + tr_e;
      const int c16 = 4 * db + 2 * dhalf + (tr_c >> 1);
      voff[rd][db] = key * (D * 2) + ((c16 ^ swzV<D>(key)) * 16) + (tr_c & 1) * 8;
    }

  f32x16 O[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
  float m = -1e30f, l = 0.f;
  const float sc = a.scale * 1.4426950408889634f;
  const float th = TH_LOG2 / sc;  // threshold in raw score units

  auto scores = [&](const unsigned char* Kb, f32x16* S) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 kf = *(const bf16x8*)(Kb + kb * 32 * (D * 2) + koff[s]);
        S[kb] = mfma32(kf, qf[s], S[kb]);
      }
    }
  };

  // online softmax + accumulation of one tile whose scores are in S
  auto softmax_accumulate = [&](const unsigned char* Vb, const f32x16* S) {
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
    bf16x8 pb[4];
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
#pragma unroll
    for (int st = 0; st < 4; ++st) {  // keys 16*st + 8H .. +7
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(Vb + st * 16 * (D * 2) + voff[0][db]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(Vb + st * 16 * (D * 2) + voff[1][db]));
        const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        O[db] = mfma32(__builtin_bit_cast(bf16x8, v8), pb[st], O[db]);
      }
    }
  };

  const int c0 = a.rowptr[qt], c1 = a.rowptr[qt + 1];
  // FULL tiles come first in the row; a ragged last key tile needs the masked loop as well
  int c_fast = c0 + a.nfull[qt];
  if (c_fast > c0 && a.col[c_fast - 1] * TN + TN > T) --c_fast;

  // Ring pipeline step shared by both loops: wait for tile `it`, barrier, refill the freed buffer.
  auto advance = [&](int it) {
    const int ahead = min(NSTAGE - 2, c1 - 1 - it);  // later tiles whose loads may stay in flight
    if (NSTAGE > 3 && ahead >= 2) wait_vmcnt<(NSTAGE > 3 ? 2 : 0) * LPT>();
    else if (NSTAGE > 2 && ahead == 1) wait_vmcnt<(NSTAGE > 2 ? 1 : 0) * LPT>();
    else wait_vmcnt<0>();
    __syncthreads();  // everyone's loads have landed, and everyone has left the buffer refilled next
    if (it + NSTAGE - 1 < c1) issue_loads((it - c0 + NSTAGE - 1) % NSTAGE, a.col[it + NSTAGE - 1] * TN);
  };

#pragma unroll
  for (int p = 0; p < NSTAGE - 1; ++p)
    if (c0 + p < c1) issue_loads(p, a.col[c0 + p] * TN);

  for (int it = c0; it < c_fast; ++it) {  // FULL tiles: no mask
    advance(it);
    const int buf = (it - c0) % NSTAGE;
    f32x16 S[2];
    scores(Kbase + buf * TILE_BYTES, S);
    softmax_accumulate(Vbase + buf * TILE_BYTES, S);
  }

  if (c_fast < c1) {  // PARTIAL / ragged tiles: per-token mask
    const uint64_t* vis_row = a.node_vis + (int64_t)(a.node_start[b] + a.tok_node[tok]) * a.W;
    const uint64_t vis0 = vis_row[0];
    const int32_t* tn = a.tok_node + cu;
    for (int it = c_fast; it < c1; ++it) {
      advance(it);
      const int buf = (it - c0) % NSTAGE;
      const int j0 = a.col[it] * TN;
      f32x16 S[2];
      scores(Kbase + buf * TILE_BYTES, S);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + 32 * kb + 16 * (r >> 3) + 8 * H + (r & 7);
          const int nj = tn[min(j, T - 1)];
          const uint64_t word = (a.W == 1) ? vis0 : vis_row[nj >> 6];
          const bool ok = (j <= i_row) && (j < T) && ((word >> (nj & 63)) & 1);
          S[kb][r] = ok ? S[kb][r] : -INFINITY;
        }
      softmax_accumulate(Vbase + buf * TILE_BYTES, S);
    }
  }

  const float l_tot = l + __shfl_xor(l, 32);
  if (i_row < T) {
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
}

template <int D, int HG, int NSTAGE>
int launch_one(const PrefillArgs& a, int hs, hipStream_t stream) {
  constexpr size_t sm = (size_t)2 * NSTAGE * TN * D * 2;
  if (hipFuncSetAttribute((const void*)k_prefill_bf16<D, HG, NSTAGE>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sm) != hipSuccess)
    return DAG_ERR_HIP;
  const unsigned grid = (unsigned)(a.total_qtiles * a.hkv * hs);
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
