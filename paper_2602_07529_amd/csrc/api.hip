// C-ABI entry points that only validate and dispatch: dag_attn_prefill (and its two halves), dag_strerror, dag_version.
#include "common.h"
#include "prefill_launch.h"

extern "C" size_t dag_prefill_workspace_bytes(const dag_meta_t* m, int32_t hkv, int32_t head_dim,
                                              dag_dtype_t dtype) {
  if (!m || dtype != DAG_BF16 || hkv < 1 || head_dim < 1 || m->sizes.total_ktiles < 0) return 0;
  // key-tile-wise transposed copy of V: [key tile][kv head][head_dim][tile_n] bf16, then the
  // work-distribution counters and the tables of the 256-row query tiles, plus slack for
  // aligning the caller's pointer to 256 bytes
  if (m->sizes.total_qtiles < 0 || m->sizes.csr_capacity < 0) return 0;
  return (size_t)m->sizes.total_ktiles * hkv * head_dim * m->tile_n * 2 +
         prefill_bf16_table_bytes(m->sizes.total_qtiles, m->sizes.csr_capacity) + 256;
}

namespace {

// Validation shared by the prefill entry points; fills the kernel argument block.
int prefill_args(const dag_meta_t* m, const void* q, const void* k, const void* v, void* out, float* lse, int32_t hq,
                 int32_t hkv, int32_t head_dim, float softmax_scale, dag_dtype_t dtype, void* ws, size_t ws_bytes,
                 bool need_qko, PrefillArgs* a, bool* empty) {
  *empty = false;
  if (!m) return DAG_ERR_NULL;
  if (dtype != DAG_F32 && dtype != DAG_BF16) return DAG_ERR_UNSUPPORTED;
  int32_t tm = 0, tn = 0;
  const int rc = dag_prefill_tile_shape(hq, hkv, head_dim, dtype, &tm, &tn);
  if (rc != DAG_OK) return rc;
  if (m->tile_m != tm || m->tile_n != tn) return DAG_ERR_UNSUPPORTED;
  if (m->n_seqs < 0 || m->sizes.total_tokens < 0 || m->sizes.total_qtiles < 0 || m->words_per_node < 1)
    return DAG_ERR_BAD_LEN;
  if (m->n_seqs == 0 || m->sizes.total_tokens == 0) {
    *empty = true;
    return DAG_OK;
  }
  if (need_qko && (!q || !k || !out)) return DAG_ERR_NULL;
  if (!v) return DAG_ERR_NULL;
  if (!m->cu_seqlens || !m->node_start || !m->tok_node || !m->node_vis || !m->qtile_start || !m->ktile_start ||
      !m->qtile_rowptr || !m->qtile_col || !m->qtile_flag || !m->qtile_nfull || !m->qtile_order || !m->qtile_desc ||
      !m->block_map_off || !m->block_map)
    return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k) || !dag_aligned16(v) || !dag_aligned16(out)) return DAG_ERR_ALIGN;
  if (m->sizes.total_qtiles * (int64_t)hq > INT32_MAX) return DAG_ERR_UNSUPPORTED;
  const size_t need = dag_prefill_workspace_bytes(m, hkv, head_dim, dtype);
  if (need > 0 && (!ws || ws_bytes < need)) return DAG_ERR_WORKSPACE;
  a->q = q;
  a->k = k;
  a->v = v;
  a->out = out;
  a->lse = lse;
  a->vt = need > 0 ? (void*)dag_align_up((size_t)(uintptr_t)ws, 256) : nullptr;
  a->sched = need > 0 ? (int32_t*)((char*)a->vt + (size_t)m->sizes.total_ktiles * hkv * head_dim * m->tile_n * 2) : nullptr;
  a->wide_count = need > 0 ? a->sched + DAG_SCHED_INTS : nullptr;
  a->wide_cnt = need > 0 ? a->wide_count + 64 : nullptr;
  a->wide_pre = need > 0 ? a->wide_cnt + m->sizes.total_qtiles : nullptr;
  a->wide_desc = need > 0 ? a->wide_pre + 8 * m->sizes.total_qtiles : nullptr;
  a->wide_col = need > 0 ? a->wide_desc + 8 * m->sizes.total_qtiles : nullptr;
  a->head0 = 0;
  a->heads = hq / hkv;
  a->n_tiles_dev = nullptr;
  a->block_map_off = m->block_map_off;
  a->block_map = m->block_map;
  a->cu_seqlens = m->cu_seqlens;
  a->node_start = m->node_start;
  a->tok_node = m->tok_node;
  a->node_vis = m->node_vis;
  a->qtile_start = m->qtile_start;
  a->ktile_start = m->ktile_start;
  a->rowptr = m->qtile_rowptr;
  a->col = m->qtile_col;
  a->flag = m->qtile_flag;
  a->nfull = m->qtile_nfull;
  a->qtile_order = m->qtile_order;
  a->qtile_desc = m->qtile_desc;
  a->n_seqs = m->n_seqs;
  a->W = m->words_per_node;
  a->hq = hq;
  a->hkv = hkv;
  a->total_qtiles = m->sizes.total_qtiles;
  a->total_ktiles = m->sizes.total_ktiles;
  a->scale = softmax_scale;
  return DAG_OK;
}

}  // namespace

extern "C" int dag_prefill_prepare_v(const dag_meta_t* m, const void* v, int32_t hq, int32_t hkv, int32_t head_dim,
                                     dag_dtype_t dtype, void* ws, size_t ws_bytes, void* stream_) {
  PrefillArgs a;
  bool empty;
  const int rc = prefill_args(m, nullptr, nullptr, v, nullptr, nullptr, hq, hkv, head_dim, 1.f, dtype, ws, ws_bytes,
                              false, &a, &empty);
  if (rc != DAG_OK || empty || dtype == DAG_F32) return rc;  // the fp32 path reads V as it is
  return launch_prefill_bf16_prepare_v(a, head_dim, (hipStream_t)stream_);
}

extern "C" int dag_attn_prefill_prepared(const dag_meta_t* m, const void* q, const void* k, const void* v, void* out,
                                         float* lse, int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale,
                                         dag_dtype_t dtype, void* ws, size_t ws_bytes, void* stream_) {
  PrefillArgs a;
  bool empty;
  const int rc = prefill_args(m, q, k, v, out, lse, hq, hkv, head_dim, softmax_scale, dtype, ws, ws_bytes, true, &a,
                              &empty);
  if (rc != DAG_OK || empty) return rc;
  hipStream_t stream = (hipStream_t)stream_;
  return dtype == DAG_F32 ? launch_prefill_f32(a, head_dim, stream) : launch_prefill_bf16(a, head_dim, stream);
}

extern "C" int dag_attn_prefill(const dag_meta_t* m, const void* q, const void* k, const void* v, void* out,
                                float* lse, int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale,
                                dag_dtype_t dtype, void* ws, size_t ws_bytes, void* stream_) {
  PrefillArgs a;
  bool empty;
  const int rc = prefill_args(m, q, k, v, out, lse, hq, hkv, head_dim, softmax_scale, dtype, ws, ws_bytes, true, &a,
                              &empty);
  if (rc != DAG_OK || empty) return rc;
  hipStream_t stream = (hipStream_t)stream_;
  if (dtype == DAG_F32) return launch_prefill_f32(a, head_dim, stream);
  const int rp = launch_prefill_bf16_prepare_v(a, head_dim, stream);
  return rp != DAG_OK ? rp : launch_prefill_bf16(a, head_dim, stream);
}

namespace {
// slots of (node, query tile) and tiles per slot that the host bounds allow
bool paged_dims(const dag_paged_prefill_desc_t* d, int64_t* slots, int64_t* nt_max) {
  if (!d || d->n_nodes < 0 || d->max_new < 0 || d->max_ctx_pages < 0 || d->page_size != 16) return false;
  *slots = (int64_t)d->n_nodes * ((d->max_new + 63) / 64);
  *nt_max = (d->max_ctx_pages + 3) / 4;
  return *slots * 8 * *nt_max <= INT32_MAX;  // (entries are indexed with 32-bit integers)
}
}  // namespace

extern "C" size_t dag_prefill_paged_workspace_bytes(const dag_paged_prefill_desc_t* d) {
  int64_t slots, nt_max;
  if (!paged_dims(d, &slots, &nt_max)) return 0;
  // counters, item count, per slot: tile count, two descriptors, its row of tile entries
  return (size_t)(DAG_SCHED_INTS + 64 + slots * (17 + 8 * nt_max)) * 4 + 256;
}

extern "C" int dag_attn_prefill_paged(const dag_paged_prefill_desc_t* d, const void* q, const void* k_pool,
                                      const void* v_pool, int32_t n_pages, void* out, float* lse, int32_t hq,
                                      int32_t hkv, int32_t head_dim, float softmax_scale, void* ws, size_t ws_bytes,
                                      void* stream_) {
  if (!d) return DAG_ERR_NULL;
  if (d->page_size != 16) return DAG_ERR_UNSUPPORTED;
  if (hq < 1 || hkv < 1 || hq % hkv != 0 || (head_dim != 64 && head_dim != 128)) return DAG_ERR_UNSUPPORTED;
  int64_t slots, nt_max;
  if (d->n_nodes < 0 || d->max_new < 0 || d->max_ctx_pages < 0 || n_pages < 0) return DAG_ERR_BAD_LEN;
  if (!paged_dims(d, &slots, &nt_max)) return DAG_ERR_UNSUPPORTED;
  if (slots == 0) return DAG_OK;  // no new token anywhere
  if (nt_max == 0 || n_pages == 0) return DAG_ERR_BAD_LEN;  // new tokens live in pages of their own
  if (!q || !k_pool || !v_pool || !out || !d->q_off || !d->ctx_page_off || !d->ctx_pages || !d->ctx_page_len ||
      !d->own_page || !d->own_len)
    return DAG_ERR_NULL;
  if (!dag_aligned16(q) || !dag_aligned16(k_pool) || !dag_aligned16(v_pool) || !dag_aligned16(out)) return DAG_ERR_ALIGN;
  if (!ws || ws_bytes < dag_prefill_paged_workspace_bytes(d)) return DAG_ERR_WORKSPACE;
  PagedPrefillArgs pa = {};
  PrefillArgs& a = pa.a;
  a.q = q;
  a.k = k_pool;
  a.vt = const_cast<void*>(v_pool);
  a.out = out;
  a.lse = lse;
  a.sched = (int32_t*)dag_align_up((size_t)(uintptr_t)ws, 256);
  a.wide_count = a.sched + DAG_SCHED_INTS;
  a.wide_cnt = a.wide_count + 64;
  a.wide_pre = a.wide_cnt + slots;
  a.wide_desc = a.wide_pre + 8 * slots;
  a.wide_col = a.wide_desc + 8 * slots;
  a.W = 1;
  a.hq = hq;
  a.hkv = hkv;
  a.head0 = 0;
  a.heads = hq / hkv;
  a.scale = softmax_scale;
  pa.n_nodes = d->n_nodes;
  pa.qt_max = (d->max_new + 63) / 64;
  pa.nt_max = (int)nt_max;
  pa.n_pages = n_pages;
  pa.q_off = d->q_off;
  pa.ctx_page_off = d->ctx_page_off;
  pa.ctx_pages = d->ctx_pages;
  pa.ctx_page_len = d->ctx_page_len;
  pa.own_page = d->own_page;
  pa.own_len = d->own_len;
  return launch_prefill_paged(pa, head_dim, (hipStream_t)stream_);
}

namespace {
__global__ void __launch_bounds__(256) k_copy_calibration(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
}  // namespace

extern "C" int dag_copy_calibration(void* dst, const void* src, size_t bytes, void* stream_) {
  if (!dst || !src) return DAG_ERR_NULL;
  if (!dag_aligned16(dst) || !dag_aligned16(src) || bytes % 16 != 0) return DAG_ERR_ALIGN;
  if (bytes == 0) return DAG_OK;
  hipLaunchKernelGGL(k_copy_calibration, dim3(4096), dim3(256), 0, (hipStream_t)stream_, (const u32x4*)src, (u32x4*)dst,
                     bytes / 16);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}

extern "C" const char* dag_strerror(int code) {
  switch (code) {
    case DAG_OK: return "ok";
    case DAG_ERR_NULL: return "a required pointer is NULL";
    case DAG_ERR_BAD_LEN: return "bad length or inconsistent size";
    case DAG_ERR_NOT_TOPOLOGICAL: return "ancestor bitset is not in topological order (or the graph has a cycle)";
    case DAG_ERR_NOT_CLOSED: return "ancestor bitset is not transitively closed";
    case DAG_ERR_POS_OVERFLOW: return "token or position count exceeds int32";
    case DAG_ERR_WORKSPACE: return "workspace missing or too small";
    case DAG_ERR_UNSUPPORTED: return "unsupported configuration";
    case DAG_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case DAG_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

extern "C" int dag_version(void) { return 100; }
