// fp32 DAG attention prefill (paper Eq. 2 + Eq. 3): the accuracy path.  Plain vector arithmetic,
// fp32 everywhere, exact expf.  A workgroup owns one 64-row query tile of one head; four threads
// share a row, each owning a quarter of the head dimension.  Key/value tiles of 64 tokens are
// staged in LDS; tiles the block map marks SKIP are never touched, FULL tiles skip the mask test.
#include "common.h"
#include "prefill_launch.h"

namespace {

constexpr int TM = 64, TN = 64;

template <int D>
__global__ void __launch_bounds__(256) k_prefill_f32(PrefillArgs a) {
  extern __shared__ float smem[];
  float* Ks = smem;             // [TN][D]
  float* Vs = smem + TN * D;    // [TN][D]
  int* s_node = (int*)(Vs + TN * D);  // [TN]
  constexpr int DP = D / 4;     // dims per thread

  const int oi = blockIdx.x / a.hq, head = blockIdx.x % a.hq;
  const int hk = head / (a.hq / a.hkv);
  const int qt = a.qtile_order[oi];
  const int b = dag_find_segment(a.qtile_start, a.n_seqs, qt);
  const int cu = a.cu_seqlens[b], T = a.cu_seqlens[b + 1] - cu;
  const int row0 = (qt - a.qtile_start[b]) * TM;
  const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
  const int i = row0 + r;                 // row inside the sequence
  const int ic = min(i, T - 1);
  const int node_i = a.tok_node[cu + ic];
  const uint64_t* vis_row = a.node_vis + (int64_t)(a.node_start[b] + node_i) * a.W;

  const float* q = (const float*)a.q + ((size_t)(cu + ic) * a.hq + head) * D + part * DP;
  float qreg[DP], o[DP];
#pragma unroll
  for (int d = 0; d < DP; ++d) {
    qreg[d] = q[d];
    o[d] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  const int c0 = a.rowptr[qt], c1 = a.rowptr[qt + 1];
  for (int it = c0; it < c1; ++it) {
    const int kt = a.col[it];
    const bool full = a.flag[it] == DAG_TILE_FULL;
    const int j0 = kt * TN;
    __syncthreads();
    for (int idx = threadIdx.x; idx < TN * (D / 4); idx += 256) {
      const int row = idx / (D / 4), c4 = idx % (D / 4);
      const int jc = min(j0 + row, T - 1);
      const size_t g = ((size_t)(cu + jc) * a.hkv + hk) * D + c4 * 4;
      *(f32x4*)(Ks + row * D + c4 * 4) = *(const f32x4*)((const float*)a.k + g);
      *(f32x4*)(Vs + row * D + c4 * 4) = *(const f32x4*)((const float*)a.v + g);
    }
    if (threadIdx.x < TN) s_node[threadIdx.x] = a.tok_node[cu + min(j0 + (int)threadIdx.x, T - 1)];
    __syncthreads();
    const int jn = min(TN, T - j0);
    for (int jj = 0; jj < jn; ++jj) {
      const int j = j0 + jj;
      bool ok = true;
      if (!full) {
        const int nj = s_node[jj];
        ok = (j <= i) && ((vis_row[nj >> 6] >> (nj & 63)) & 1);
      }
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < DP; ++d) s += qreg[d] * Ks[jj * D + part * DP + d];
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      if (ok) {
        const float x = s * a.scale;
        if (x > m) {
          const float alpha = expf(m - x);  // expf(-inf) = 0 on the first visible key
          l *= alpha;
#pragma unroll
          for (int d = 0; d < DP; ++d) o[d] *= alpha;
          m = x;
        }
        const float p = expf(x - m);
        l += p;
#pragma unroll
        for (int d = 0; d < DP; ++d) o[d] += p * Vs[jj * D + part * DP + d];
      }
    }
  }
  if (i < T) {
    const float inv = 1.f / l;
    float* out = (float*)a.out + ((size_t)(cu + i) * a.hq + head) * D + part * DP;
#pragma unroll
    for (int d = 0; d < DP; ++d) out[d] = o[d] * inv;
    if (a.lse && part == 0) a.lse[(size_t)(cu + i) * a.hq + head] = m + logf(l);
  }
}

}  // namespace

int launch_prefill_f32(const PrefillArgs& a, int head_dim, hipStream_t stream) {
  const unsigned grid = (unsigned)(a.total_qtiles * a.hq);
  if (head_dim == 64) {
    const size_t sm = (size_t)2 * TN * 64 * 4 + TN * 4;
    hipLaunchKernelGGL(k_prefill_f32<64>, dim3(grid), dim3(256), sm, stream, a);
  } else {
    const size_t sm = (size_t)2 * TN * 128 * 4 + TN * 4;
    if (hipFuncSetAttribute((const void*)k_prefill_f32<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm) != hipSuccess)
      return DAG_ERR_HIP;
    hipLaunchKernelGGL(k_prefill_f32<128>, dim3(grid), dim3(256), sm, stream, a);
  }
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}
