// bf16 DAG attention prefill for gfx950 (paper Eq. 2 + Eq. 3), MFMA 32x32x16 with fp32 accumulation.
//
// Work decomposition.  A workgroup owns one query tile (32*RB token rows) of one KV head and stacks
// HG of that KV head's query heads: wave w handles row block w / HG and head w % HG, so every wave
// of the workgroup consumes the same K/V tiles.  K/V tiles of 64 tokens are staged through LDS
// (double buffered, one barrier per tile); only the tiles the CSR block map lists are visited and
// only PARTIAL (or ragged) tiles evaluate the per-token mask.
//
// Register layout.  Scores are computed transposed, S^T = K Q^T, so that after the MFMA a lane
// holds one query row (lane % 32) and 16 keys of each 32-key block in registers: the softmax
// row reductions are in-register plus one exchange between the two half waves, and the
// probabilities already sit in the B-operand layout of the second product O^T = V^T P^T.
// The MFMA row i of a 32-key block is mapped to key pi(i) so that registers 0..7 / 8..15 of the
// score block hold 8 consecutive keys; V is transposed while it is staged so that a lane reads its
// 8 keys for one output dimension with a single 16-byte LDS load.
//
// LDS layouts (XOR swizzles at 16-byte granularity; reads are conflict free):
//   K tile  [64 keys][D]      chunk' = chunk ^ fK(key)
//   V^T tile [D][64 keys]     chunk' = chunk ^ gV(d)
#include "common.h"
#include "prefill_launch.h"

namespace {

constexpr int TN = 64;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(8))) float f32x8;

__device__ __forceinline__ bf16x8 cvt8(const float* p) {
  f32x8 v = {p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]};
  return __builtin_convertvector(v, bf16x8);
}

// MFMA row i (0..31) of a 32-key block -> key index inside the block.
__device__ __forceinline__ int key_of_row(int i) {
  const int a = i >> 3, hh = (i >> 2) & 1, c = i & 3;
  return 16 * (a >> 1) + 8 * hh + 4 * (a & 1) + c;
}

template <int D>
__device__ __forceinline__ int fK(int key) {
  return D == 128 ? (key & 15) : ((key >> 1) & 7);
}
__device__ __forceinline__ int gV(int d) {
  const int L = d & 31;
  return ((L >> 1) ^ (L >> 4)) & 7;
}

template <int D, int HG, int RB>
__global__ void __launch_bounds__(64 * HG * RB) k_prefill_bf16(PrefillArgs a) {
  constexpr int NW = HG * RB, NT = 64 * NW, TM = 32 * RB;
  constexpr int CH = D / 8;       // 16-byte chunks per K row
  constexpr int KSTEPS = D / 16;  // MFMA steps of the score product
  constexpr int DB = D / 32;      // 32-row blocks of O^T
  constexpr int KCHUNKS = TN * CH, NKC = (KCHUNKS + NT - 1) / NT;
  constexpr int VTASKS = (TN / 8) * (D / 4), NVT = (VTASKS + NT - 1) / NT;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  uint16_t* Ks = (uint16_t*)smem_raw;          // [2][TN*D]
  uint16_t* Vs = Ks + 2 * TN * D;              // [2][D*TN]
  int* s_node = (int*)(Vs + 2 * D * TN);       // [2][TN]

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
  const int i_row = row0 + 32 * rb + L;         // row inside the sequence
  const int tok = cu + min(i_row, T - 1);

  const uint16_t* qg = (const uint16_t*)a.q;
  const uint16_t* kg = (const uint16_t*)a.k;
  const uint16_t* vg = (const uint16_t*)a.v;

  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s)
    qf[s] = *(const bf16x8*)(qg + ((size_t)tok * a.hq + head) * D + 16 * s + 8 * H);

  const int node_i = a.tok_node[tok];
  const uint64_t* vis_row = a.node_vis + (int64_t)(a.node_start[b] + node_i) * a.W;
  const uint64_t vis0 = vis_row[0];

  // per-lane LDS read offsets (elements)
  const int krow = key_of_row(L);
  int koff[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) koff[s] = krow * D + (((2 * s + H) ^ fK<D>(krow)) * 8);
  int voff[4];  // index 2*kb + t: chunk 4kb + 2t + H of V^T row L
#pragma unroll
  for (int c = 0; c < 4; ++c) voff[c] = L * TN + ((((2 * c + H) ^ gV(L)) & 7) * 8);

  f32x16 O[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
  float m = -1e30f, l = 0.f;
  const float sc = a.scale * 1.4426950408889634f;

  // staging registers
  u32x4 kst[NKC];
  u32x2 vst[NVT][8];
  int nst = 0;

  auto stage_load = [&](int kt) {
    const int j0 = kt * TN;
#pragma unroll
    for (int n = 0; n < NKC; ++n) {
      const int c = tid + n * NT;
      if (KCHUNKS % NT == 0 || c < KCHUNKS) {
        const int row = c / CH, ch = c % CH;
        const int jc = min(j0 + row, T - 1);
        kst[n] = *(const u32x4*)(kg + ((size_t)(cu + jc) * a.hkv + hk) * D + ch * 8);
      }
    }
#pragma unroll
    for (int n = 0; n < NVT; ++n) {
      const int c = tid + n * NT;
      if (VTASKS % NT == 0 || c < VTASKS) {
        const int kgp = c / (D / 4), dg = c % (D / 4);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int jc = min(j0 + 8 * kgp + e, T - 1);
          vst[n][e] = *(const u32x2*)(vg + ((size_t)(cu + jc) * a.hkv + hk) * D + dg * 4);
        }
      }
    }
    if (tid < TN) nst = a.tok_node[cu + min(j0 + tid, T - 1)];
  };

  auto stage_store = [&](int buf) {
    uint16_t* Kb = Ks + buf * TN * D;
    uint16_t* Vb = Vs + buf * D * TN;
#pragma unroll
    for (int n = 0; n < NKC; ++n) {
      const int c = tid + n * NT;
      if (KCHUNKS % NT == 0 || c < KCHUNKS) {
        const int row = c / CH, ch = c % CH;
        *(u32x4*)(Kb + row * D + ((ch ^ fK<D>(row)) * 8)) = kst[n];
      }
    }
#pragma unroll
    for (int n = 0; n < NVT; ++n) {
      const int c = tid + n * NT;
      if (VTASKS % NT == 0 || c < VTASKS) {
        const int kgp = c / (D / 4), dg = c % (D / 4);
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
          u32x4 o;
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t lo = vst[n][2 * e2][dd >> 1], hi = vst[n][2 * e2 + 1][dd >> 1];
            o[e2] = (dd & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
          }
          const int d = dg * 4 + dd;
          *(u32x4*)(Vb + d * TN + ((kgp ^ gV(d)) * 8)) = o;
        }
      }
    }
    if (tid < TN) s_node[buf * TN + tid] = nst;
  };

  const int c0 = a.rowptr[qt], c1 = a.rowptr[qt + 1];
  if (c0 < c1) {
    stage_load(a.col[c0]);
    stage_store(0);
  }
  __syncthreads();

  for (int it = c0; it < c1; ++it) {
    const int buf = (it - c0) & 1;
    const int kt = a.col[it];
    const int j0 = kt * TN;
    const bool need_mask = (a.flag[it] != DAG_TILE_FULL) || (j0 + TN > T);
    const bool has_next = it + 1 < c1;
    if (has_next) stage_load(a.col[it + 1]);

    const uint16_t* Kb = Ks + buf * TN * D;
    const uint16_t* Vb = Vs + buf * D * TN;

    f32x16 S[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[kb][r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 kf = *(const bf16x8*)(Kb + kb * 32 * D + koff[s]);
        S[kb] = mfma32(kf, qf[s], S[kb]);
      }
    }

    if (need_mask) {
      const int* sn = s_node + buf * TN;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kl = 32 * kb + 16 * (r >> 3) + 8 * H + (r & 7);
          const int j = j0 + kl;
          const int nj = sn[kl];
          const uint64_t word = (a.W == 1) ? vis0 : vis_row[nj >> 6];
          const bool ok = (j <= i_row) && (j < T) && ((word >> (nj & 63)) & 1);
          S[kb][r] = ok ? S[kb][r] : -INFINITY;
        }
    }

    float bm = S[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) bm = fmaxf(bm, S[kb][r]);
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    const float m_new = fmaxf(m, bm);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * sc);
    const float msc = m_new * sc;
    m = m_new;
    float rowsum = 0.f;
    float P[2][16];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(S[kb][r], sc, -msc));
        P[kb][r] = p;
        rowsum += p;
      }
    l = l * alpha + rowsum;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[db][r] *= alpha;

#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pb = cvt8(&P[kb][8 * t]);
        const int vo = voff[2 * kb + t];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 vf = *(const bf16x8*)(Vb + db * 32 * TN + vo);
          O[db] = mfma32(vf, pb, O[db]);
        }
      }

    if (has_next) stage_store(buf ^ 1);
    __syncthreads();
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

template <int D, int HG, int RB>
int launch_one(const PrefillArgs& a, int hs, hipStream_t stream) {
  constexpr size_t sm = (size_t)2 * TN * D * 2 * 2 + 2 * TN * 4;
  if (hipFuncSetAttribute((const void*)k_prefill_bf16<D, HG, RB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sm) != hipSuccess)
    return DAG_ERR_HIP;
  const unsigned grid = (unsigned)(a.total_qtiles * a.hkv * hs);
  hipLaunchKernelGGL((k_prefill_bf16<D, HG, RB>), dim3(grid), dim3(64 * HG * RB), sm, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

template <int D>
int launch_d(const PrefillArgs& a, hipStream_t stream) {
  const int g = a.hq / a.hkv;
  if (g % 4 == 0) return launch_one<D, 4, 1>(a, g / 4, stream);
  if (g == 5) return launch_one<D, 5, 1>(a, 1, stream);
  if (g % 2 == 0) return launch_one<D, 2, 2>(a, g / 2, stream);
  return launch_one<D, 1, 4>(a, g, stream);
}

}  // namespace

int launch_prefill_bf16(const PrefillArgs& a, int head_dim, hipStream_t stream) {
  if (head_dim == 128) return launch_d<128>(a, stream);
  return launch_d<64>(a, stream);
}
