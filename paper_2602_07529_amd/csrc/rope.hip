// dag_rope_qk: rotary position embedding (the P(i) of the paper's Eq. 2) evaluated at the adaptive
// position ids of section 4.2.  Memory-bound pre-pass, in place: each block handles a few tokens,
// computes their cos/sin tables once (fp64 angle, so that positions of tens of thousands lose no
// accuracy) and applies them to every query and key head with 16-byte loads and stores.
#include "common.h"

namespace {

constexpr int kRopeTokens = 4;   // tokens per block
constexpr int kRopeMaxHalf = 128;

template <bool BF16>
__global__ void __launch_bounds__(256) k_rope(const int32_t* __restrict__ pos_ids, int64_t n_tokens,
                                              void* __restrict__ q, void* __restrict__ k, int hq, int hkv,
                                              int D, float theta) {
  __shared__ double s_freq[kRopeMaxHalf];
  __shared__ float s_cos[kRopeTokens][kRopeMaxHalf];
  __shared__ float s_sin[kRopeTokens][kRopeMaxHalf];
  const int half = D / 2;
  const int64_t t0 = (int64_t)blockIdx.x * kRopeTokens;
  for (int m = threadIdx.x; m < half; m += blockDim.x)
    s_freq[m] = pow((double)theta, -2.0 * (double)m / (double)D);
  __syncthreads();
  for (int idx = threadIdx.x; idx < kRopeTokens * half; idx += blockDim.x) {
    const int tt = idx / half, m = idx % half;
    const int64_t t = t0 + tt;
    if (t < n_tokens) {
      double sn, cs;
      sincos((double)pos_ids[t] * s_freq[m], &sn, &cs);
      s_cos[tt][m] = (float)cs;
      s_sin[tt][m] = (float)sn;
    }
  }
  __syncthreads();
  constexpr int EPV = BF16 ? 8 : 4;          // elements per 16-byte vector
  const int upr = half / EPV;                // vectors per half row
  const int rows_q = q ? hq : 0, rows_k = k ? hkv : 0;
  const int rows = rows_q + rows_k;
  const int total = kRopeTokens * rows * upr;
  for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
    const int u = idx % upr;
    const int row = (idx / upr) % rows;
    const int tt = idx / (upr * rows);
    const int64_t t = t0 + tt;
    if (t >= n_tokens) continue;
    const float* cs = &s_cos[tt][u * EPV];
    const float* sn = &s_sin[tt][u * EPV];
    if (BF16) {
      uint16_t* base = row < rows_q ? (uint16_t*)q + ((size_t)t * hq + row) * D
                                    : (uint16_t*)k + ((size_t)t * hkv + (row - rows_q)) * D;
      u32x4* plo = (u32x4*)(base + u * EPV);
      u32x4* phi = (u32x4*)(base + half + u * EPV);
      u32x4 lo = *plo, hi = *phi, olo, ohi;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float l0 = dag_bf_lo(lo[w]), l1 = dag_bf_hi(lo[w]);
        const float h0 = dag_bf_lo(hi[w]), h1 = dag_bf_hi(hi[w]);
        const float c0 = cs[2 * w], c1 = cs[2 * w + 1], s0 = sn[2 * w], s1 = sn[2 * w + 1];
        olo[w] = dag_pack_bf2(l0 * c0 - h0 * s0, l1 * c1 - h1 * s1);
        ohi[w] = dag_pack_bf2(h0 * c0 + l0 * s0, h1 * c1 + l1 * s1);
      }
      *plo = olo;
      *phi = ohi;
    } else {
      float* base = row < rows_q ? (float*)q + ((size_t)t * hq + row) * D
                                 : (float*)k + ((size_t)t * hkv + (row - rows_q)) * D;
      f32x4* plo = (f32x4*)(base + u * EPV);
      f32x4* phi = (f32x4*)(base + half + u * EPV);
      f32x4 lo = *plo, hi = *phi, olo, ohi;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        olo[w] = lo[w] * cs[w] - hi[w] * sn[w];
        ohi[w] = hi[w] * cs[w] + lo[w] * sn[w];
      }
      *plo = olo;
      *phi = ohi;
    }
  }
}

}  // namespace

extern "C" int dag_rope_qk(const int32_t* pos_ids, int64_t n_tokens, void* q, void* k, int32_t hq, int32_t hkv,
                           int32_t head_dim, float theta, dag_dtype_t dtype, void* stream_) {
  if (n_tokens < 0) return DAG_ERR_BAD_LEN;
  if (dtype != DAG_F32 && dtype != DAG_BF16) return DAG_ERR_UNSUPPORTED;
  if (head_dim < 16 || head_dim > 2 * kRopeMaxHalf || head_dim % 16 != 0) return DAG_ERR_UNSUPPORTED;
  if ((q && hq < 1) || (k && hkv < 1) || !(theta > 0.f)) return DAG_ERR_UNSUPPORTED;
  if (n_tokens == 0 || (!q && !k)) return DAG_OK;
  if (!pos_ids) return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k)) return DAG_ERR_ALIGN;
  hipStream_t stream = (hipStream_t)stream_;
  const unsigned grid = (unsigned)dag_ceil_div(n_tokens, kRopeTokens);
  if (dtype == DAG_BF16)
    hipLaunchKernelGGL(k_rope<true>, dim3(grid), dim3(256), 0, stream, pos_ids, n_tokens, q, k, hq, hkv, head_dim, theta);
  else
    hipLaunchKernelGGL(k_rope<false>, dim3(grid), dim3(256), 0, stream, pos_ids, n_tokens, q, k, hq, hkv, head_dim, theta);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}
