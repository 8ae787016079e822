// Backward of the DAG-masked prefill attention (the paper fine-tunes through the mask of Eq. 3,
// section 4.2): with P = softmax_row(scale Q K^T + M), O = P V and the incoming gradient dO,
//     delta_i = sum_d dO_id O_id,   dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),
//     dQ = scale dS K,   dK = scale dS^T Q        (a KV head sums over its query heads).
// P is recomputed from the forward's log-sum-exp; the block map of the forward skips the tiles
// without a visible pair.  bf16 operands on the 32x32x16 MFMA, fp32 accumulation.  Three kernels:
//   k_bwd_delta   delta per (token, query head)
//   k_bwd_dq      one workgroup per (64-row query tile, query head), loop over its key tiles
//   k_bwd_dkv     one workgroup per (64-key tile, KV head), loop over the query tiles that see it
//                 and the query heads of the group; nothing is accumulated through atomics, so
//                 the results do not depend on the order of execution.
// Register layout of a 32x32 MFMA result C = A B:  lane (L, H) = (lane % 32, lane / 32) holds
// column L and the 16 rows rho_H(e) = 8 (e / 4) + 4 H + e % 4.  A result is used again as the B
// operand of the next product (contraction over its rows) straight from the registers; the A
// operand of that product is then gathered from LDS in the same row order.
// First version: tiles are staged with plain loads between two workgroup barriers (no software
// pipeline) and the transposed operands are gathered element by element from LDS.
#include "common.h"

namespace {

constexpr int BM = 64, BN = 64;  // tile shape of the bf16 block map
constexpr float LOG2E = 1.4426950408889634f;

struct BwdArgs {
  const uint16_t *q, *k, *v, *out, *dout;
  const float* lse;
  uint16_t *dq, *dk, *dv;
  float* delta;  // [T][hq]
  const int32_t *cu_seqlens, *node_start, *tok_node, *qtile_start, *ktile_start;
  const uint64_t* node_vis;
  const int64_t* block_map_off;
  const uint8_t* block_map;
  int n_seqs, W, hq, hkv, G;
  long total_rows;  // T * hq
  float scale, sc;  // sc = scale * log2(e)
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

// Eq. 3 for a (query token i of node ni, key token j of node nj) pair of one sequence
__device__ __forceinline__ bool visible(const BwdArgs& a, int nbase, int ni, int i, int nj, int j, uint64_t vis0) {
  if (nj == ni) return j <= i;
  const uint64_t w = nj < 64 ? vis0 : a.node_vis[(int64_t)(nbase + ni) * a.W + (nj >> 6)];
  return (w >> (nj & 63)) & 1u;
}

// 8 elements of column `col` of a row-major LDS tile (row stride LD), rows r0 + rho_H(8 ks + e):
// the A operand of a product whose contraction runs over the rows of a previous result
template <int LD>
__device__ __forceinline__ bf16x8 gather_col(const uint16_t* tile, int r0, int ks, int H, int col) {
  typedef __attribute__((ext_vector_type(8))) uint16_t u16x8;
  u16x8 x;
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = tile[(r0 + rho(8 * ks + e, H)) * LD + col];
  return __builtin_bit_cast(bf16x8, x);
}

template <int D>
__global__ void __launch_bounds__(64) k_bwd_delta(BwdArgs a) {
  const long row = blockIdx.x;  // (token, query head)
  const int lane = threadIdx.x;
  constexpr int PER = D / 64;
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const size_t idx = (size_t)row * D + lane * PER + e;
    s += __uint_as_float((uint32_t)a.out[idx] << 16) * __uint_as_float((uint32_t)a.dout[idx] << 16);
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (lane == 0) a.delta[row] = s;
}

template <int D>
__global__ void __launch_bounds__(128) k_bwd_dq(BwdArgs a) {
  constexpr int LD = D + 8;  // padded rows: the 16-byte operand reads of 32 consecutive rows spread over the banks
  __shared__ __attribute__((aligned(16))) uint16_t sK[BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sV[BN * LD];
  __shared__ int sNode[BN];
  const int qt = blockIdx.x, h = blockIdx.y, hk = h / a.G;
  const int b = dag_find_segment(a.qtile_start, a.n_seqs, qt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int qtl = qt - a.qtile_start[b];
  const int KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b] + (int64_t)qtl * KT;
  const int nbase = a.node_start[b];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, L = lane & 31, H = lane >> 5;
  const int i = qtl * BM + 32 * w + L;  // this lane's query row
  const bool row_ok = i < T;
  const int ic = min(i, T - 1);
  const size_t qoff = ((size_t)(cu + ic) * a.hq + h) * D;
  bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    qf[s] = *(const bf16x8*)(a.q + qoff + 16 * s + 8 * H);
    dof[s] = *(const bf16x8*)(a.dout + qoff + 16 * s + 8 * H);
  }
  const float lse2 = a.lse[(size_t)(cu + ic) * a.hq + h] * LOG2E;
  const float dl = a.delta[(size_t)(cu + ic) * a.hq + h];
  const int ni = a.tok_node[cu + ic];
  const uint64_t vis0 = a.node_vis[(int64_t)(nbase + ni) * a.W];
  f32x16 dQ[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) dQ[db][e] = 0.f;

  for (int kt = 0; kt < KT; ++kt) {
    const int flag = bm[kt];
    if (flag == 0) continue;
    const int j0 = kt * BN;
    __syncthreads();
    for (int c = tid; c < BN * (D / 8); c += 128) {
      const int r = c / (D / 8), ch = c % (D / 8);
      u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
      if (j0 + r < T) {
        const size_t off = ((size_t)(cu + j0 + r) * a.hkv + hk) * D + ch * 8;
        x = *(const u32x4*)(a.k + off);
        y = *(const u32x4*)(a.v + off);
      }
      *(u32x4*)(sK + r * LD + ch * 8) = x;
      *(u32x4*)(sV + r * LD + ch * 8) = y;
    }
    if (tid < BN) sNode[tid] = a.tok_node[cu + min(j0 + tid, T - 1)];
    __syncthreads();
    const bool need_mask = flag == 1;
#pragma unroll 1
    for (int hh = 0; hh < 2; ++hh) {
      f32x16 S, dP;
#pragma unroll
      for (int e = 0; e < 16; ++e) S[e] = dP[e] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {  // S^T = K Q^T, dP^T = V dO^T: rows = keys, column = this lane's query row
        S = mfma32(*(const bf16x8*)(sK + (32 * hh + L) * LD + 16 * s + 8 * H), qf[s], S);
        dP = mfma32(*(const bf16x8*)(sV + (32 * hh + L) * LD + 16 * s + 8 * H), dof[s], dP);
      }
      float ds[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kk = 32 * hh + rho(e, H), j = j0 + kk;
        bool ok = row_ok && j < T;
        if (need_mask && ok) ok = visible(a, nbase, ni, i, sNode[kk], j, vis0);
        const float p = ok ? __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -lse2)) : 0.f;
        ds[e] = p * (dP[e] - dl);
      }
      const bf16x8 b0 = pack8(ds), b1 = pack8(ds + 8);
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {  // dQ^T += K^T dS^T
        dQ[db] = mfma32(gather_col<LD>(sK, 32 * hh, 0, H, 32 * db + L), b0, dQ[db]);
        dQ[db] = mfma32(gather_col<LD>(sK, 32 * hh, 1, H, 32 * db + L), b1, dQ[db]);
      }
    }
  }
  if (row_ok) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        u32x2 o;
        o[0] = dag_pack_bf2(dQ[db][4 * e4] * a.scale, dQ[db][4 * e4 + 1] * a.scale);
        o[1] = dag_pack_bf2(dQ[db][4 * e4 + 2] * a.scale, dQ[db][4 * e4 + 3] * a.scale);
        *(u32x2*)(a.dq + qoff + 32 * db + 8 * e4 + 4 * H) = o;
      }
  }
}

template <int D>
constexpr int dkv_smem_bytes() {
  // Q and dO rows of one query tile for two query heads, their lse / delta, node ids and first
  // visibility words of the rows; the area is reused for the final reduction over the two head sets
  return 2 * 2 * BM * (D + 8) * 2 + 2 * 2 * BM * 4 + BM * 4 + BM * 8;
}

template <int D>
__global__ void __launch_bounds__(256) k_bwd_dkv(BwdArgs a) {
  constexpr int LD = D + 8, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* const sQ = (uint16_t*)smem;                  // [2][BM][LD]
  uint16_t* const sdO = sQ + 2 * BM * LD;                // [2][BM][LD]
  float* const sLse = (float*)(sdO + 2 * BM * LD);       // [2][BM]  (log2 units)
  float* const sDl = sLse + 2 * BM;                      // [2][BM]
  int* const sNodeR = (int*)(sDl + 2 * BM);              // [BM]
  uint64_t* const sVis0 = (uint64_t*)(sNodeR + BM);      // [BM]
  const int kt = blockIdx.x, hk = blockIdx.y;
  const int b = dag_find_segment(a.ktile_start, a.n_seqs, kt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int ktl = kt - a.ktile_start[b];
  const int QT = (T + BM - 1) / BM, KT = (T + BN - 1) / BN;
  const uint8_t* bm = a.block_map + a.block_map_off[b];
  const int nbase = a.node_start[b];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, L = lane & 31, H = lane >> 5;
  const int kh = w & 1, hs = w >> 1;  // key half of the tile, set of query heads (even / odd within the group)
  const int j = ktl * BN + 32 * kh + L;  // this lane's key
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

  for (int qt = 0; qt < QT; ++qt) {
    const int flag = bm[(int64_t)qt * KT + ktl];
    if (flag == 0) continue;
    const int r0 = qt * BM;
    const bool need_mask = flag == 1;
    for (int gi = 0; 2 * gi < a.G; ++gi) {
      __syncthreads();
      for (int c = tid; c < 2 * BM * (D / 8); c += 256) {  // rows of the tile for heads 2 gi and 2 gi + 1 of the group
        const int sub = c / (BM * (D / 8)), r = (c / (D / 8)) % BM, ch = c % (D / 8);
        const int g = 2 * gi + sub;
        u32x4 x = {0, 0, 0, 0}, y = {0, 0, 0, 0};
        if (r0 + r < T && g < a.G) {
          const size_t off = ((size_t)(cu + r0 + r) * a.hq + hk * a.G + g) * D + ch * 8;
          x = *(const u32x4*)(a.q + off);
          y = *(const u32x4*)(a.dout + off);
        }
        *(u32x4*)(sQ + (sub * BM + r) * LD + ch * 8) = x;
        *(u32x4*)(sdO + (sub * BM + r) * LD + ch * 8) = y;
      }
      if (tid < 2 * BM) {
        const int sub = tid / BM, r = tid % BM, g = 2 * gi + sub;
        float l2 = 0.f, dl = 0.f;
        if (r0 + r < T && g < a.G) {
          const size_t row = (size_t)(cu + r0 + r) * a.hq + hk * a.G + g;
          l2 = a.lse[row] * LOG2E;
          dl = a.delta[row];
        }
        sLse[tid] = l2;
        sDl[tid] = dl;
      }
      if (tid < BM) {
        const int n = a.tok_node[cu + min(r0 + tid, T - 1)];
        sNodeR[tid] = n;
        sVis0[tid] = a.node_vis[(int64_t)(nbase + n) * a.W];
      }
      __syncthreads();
      if (2 * gi + hs < a.G) {
        const uint16_t* tQ = sQ + hs * BM * LD;
        const uint16_t* tdO = sdO + hs * BM * LD;
#pragma unroll 1
        for (int rb = 0; rb < BM / 32; ++rb) {
          f32x16 S, dP;
#pragma unroll
          for (int e = 0; e < 16; ++e) S[e] = dP[e] = 0.f;
#pragma unroll
          for (int s = 0; s < D / 16; ++s) {  // S = Q K^T, dP = dO V^T: rows = query rows, column = this lane's key
            S = mfma32(*(const bf16x8*)(tQ + (32 * rb + L) * LD + 16 * s + 8 * H), kf[s], S);
            dP = mfma32(*(const bf16x8*)(tdO + (32 * rb + L) * LD + 16 * s + 8 * H), vf[s], dP);
          }
          float p[16], ds[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r = 32 * rb + rho(e, H), i = r0 + r;
            bool ok = key_ok && i < T;
            if (need_mask && ok) ok = visible(a, nbase, sNodeR[r], i, nj, j, sVis0[r]);
            p[e] = ok ? __builtin_amdgcn_exp2f(fmaf(S[e], a.sc, -sLse[hs * BM + r])) : 0.f;
            ds[e] = p[e] * (dP[e] - sDl[hs * BM + r]);
          }
          const bf16x8 p0 = pack8(p), p1 = pack8(p + 8), s0 = pack8(ds), s1 = pack8(ds + 8);
#pragma unroll
          for (int db = 0; db < DB; ++db) {  // dV^T += dO^T P, dK^T += Q^T dS
            dV[db] = mfma32(gather_col<LD>(tdO, 32 * rb, 0, H, 32 * db + L), p0, dV[db]);
            dV[db] = mfma32(gather_col<LD>(tdO, 32 * rb, 1, H, 32 * db + L), p1, dV[db]);
            dK[db] = mfma32(gather_col<LD>(tQ, 32 * rb, 0, H, 32 * db + L), s0, dK[db]);
            dK[db] = mfma32(gather_col<LD>(tQ, 32 * rb, 1, H, 32 * db + L), s1, dK[db]);
          }
        }
      }
    }
  }
  // the two head sets of a key half add up through LDS, then the even set writes the rows out
  __syncthreads();
  float* const red = (float*)smem;  // [2 key halves][2 tensors][DB][16][64 lanes]
  if (hs == 1) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        red[(((kh * 2 + 0) * DB + db) * 16 + e) * 64 + lane] = dK[db][e];
        red[(((kh * 2 + 1) * DB + db) * 16 + e) * 64 + lane] = dV[db][e];
      }
  }
  __syncthreads();
  if (hs == 0 && key_ok) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        float xk[4], xv[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int e = 4 * e4 + t;
          xk[t] = (dK[db][e] + red[(((kh * 2 + 0) * DB + db) * 16 + e) * 64 + lane]) * a.scale;
          xv[t] = dV[db][e] + red[(((kh * 2 + 1) * DB + db) * 16 + e) * 64 + lane];
        }
        u32x2 ok2, ov2;
        ok2[0] = dag_pack_bf2(xk[0], xk[1]); ok2[1] = dag_pack_bf2(xk[2], xk[3]);
        ov2[0] = dag_pack_bf2(xv[0], xv[1]); ov2[1] = dag_pack_bf2(xv[2], xv[3]);
        *(u32x2*)(a.dk + koff + 32 * db + 8 * e4 + 4 * H) = ok2;
        *(u32x2*)(a.dv + koff + 32 * db + 8 * e4 + 4 * H) = ov2;
      }
  }
}

template <int D>
int launch_bwd(const BwdArgs& a, long total_qtiles, long total_ktiles, hipStream_t stream) {
  hipLaunchKernelGGL((k_bwd_delta<D>), dim3((unsigned)a.total_rows), dim3(64), 0, stream, a);
  DAG_LAUNCH_CHECK();
  hipLaunchKernelGGL((k_bwd_dq<D>), dim3((unsigned)total_qtiles, (unsigned)a.hq), dim3(128), 0, stream, a);
  DAG_LAUNCH_CHECK();
  constexpr int sm = dkv_smem_bytes<D>();
  static_assert(sm >= 2 * 2 * (D / 32) * 16 * 64 * 4, "the staging area also holds the final reduction");
  if (hipFuncSetAttribute((const void*)k_bwd_dkv<D>, hipFuncAttributeMaxDynamicSharedMemorySize, sm) != hipSuccess)
    return DAG_ERR_HIP;
  hipLaunchKernelGGL((k_bwd_dkv<D>), dim3((unsigned)total_ktiles, (unsigned)a.hkv), dim3(256), sm, stream, a);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

}  // namespace

extern "C" size_t dag_prefill_bwd_workspace_bytes(const dag_meta_t* m, int32_t hq) {
  if (!m || hq < 1 || m->sizes.total_tokens < 0) return 0;
  return (size_t)m->sizes.total_tokens * hq * 4 + 256;
}

extern "C" int dag_attn_prefill_bwd(const dag_meta_t* m, const void* q, const void* k, const void* v, const void* out,
                                    const void* dout, const float* lse, void* dq, void* dk, void* dv, int32_t hq,
                                    int32_t hkv, int32_t head_dim, float softmax_scale, dag_dtype_t dtype, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!m) return DAG_ERR_NULL;
  if (dtype != DAG_BF16) return DAG_ERR_UNSUPPORTED;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || (head_dim != 64 && head_dim != 128)) return DAG_ERR_UNSUPPORTED;
  if (m->tile_m != BM || m->tile_n != BN) return DAG_ERR_UNSUPPORTED;
  if (m->n_seqs < 0 || m->sizes.total_tokens < 0 || m->words_per_node < 1) return DAG_ERR_BAD_LEN;
  if (m->n_seqs == 0 || m->sizes.total_tokens == 0) return DAG_OK;
  if (!q || !k || !v || !out || !dout || !lse || !dq || !dk || !dv) return DAG_ERR_NULL;
  if (!m->cu_seqlens || !m->node_start || !m->tok_node || !m->node_vis || !m->qtile_start || !m->ktile_start ||
      !m->block_map_off || !m->block_map)
    return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k) || !dag_aligned16(v) || !dag_aligned16(out) || !dag_aligned16(dout) ||
      !dag_aligned16(dq) || !dag_aligned16(dk) || !dag_aligned16(dv))
    return DAG_ERR_ALIGN;
  if (m->sizes.total_tokens * (int64_t)hq > INT32_MAX) return DAG_ERR_UNSUPPORTED;
  const size_t need = dag_prefill_bwd_workspace_bytes(m, hq);
  if (!ws || ws_bytes < need) return DAG_ERR_WORKSPACE;
  BwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.out = (const uint16_t*)out; a.dout = (const uint16_t*)dout;
  a.lse = lse;
  a.dq = (uint16_t*)dq; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.delta = (float*)dag_align_up((size_t)(uintptr_t)ws, 256);
  a.cu_seqlens = m->cu_seqlens; a.node_start = m->node_start; a.tok_node = m->tok_node;
  a.qtile_start = m->qtile_start; a.ktile_start = m->ktile_start;
  a.node_vis = m->node_vis; a.block_map_off = m->block_map_off; a.block_map = m->block_map;
  a.n_seqs = m->n_seqs; a.W = m->words_per_node; a.hq = hq; a.hkv = hkv; a.G = hq / hkv;
  a.total_rows = (long)m->sizes.total_tokens * hq;
  a.scale = softmax_scale; a.sc = softmax_scale * LOG2E;
  hipStream_t s = (hipStream_t)stream;
  return head_dim == 128 ? launch_bwd<128>(a, m->sizes.total_qtiles, m->sizes.total_ktiles, s)
                         : launch_bwd<64>(a, m->sizes.total_qtiles, m->sizes.total_ktiles, s);
}
