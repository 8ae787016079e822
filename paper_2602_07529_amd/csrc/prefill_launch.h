// Kernel argument block shared by the prefill kernels (internal).
#pragma once
#include "common.h"

constexpr int DAG_SCHED_INTS = 128;  // [0..63] item counters, [64] finished workgroups

struct PrefillArgs {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  float* lse;
  void* vt;  // workspace: key-tile-wise transposed V in the LDS tile order (bf16 path)
  int32_t* sched;  // workspace: work-distribution counters of the bf16 kernel, DAG_SCHED_INTS ints, zero between launches
  const int32_t* cu_seqlens;
  const int32_t* node_start;
  const int32_t* tok_node;
  const uint64_t* node_vis;
  const int32_t* qtile_start;
  const int32_t* ktile_start;
  const int32_t* rowptr;
  const int32_t* col;
  const uint8_t* flag;
  const int32_t* nfull;
  const int32_t* qtile_order;
  const int32_t* qtile_desc;  // [total_qtiles][8], see dag_meta_t
  const int64_t* block_map_off;
  const uint8_t* block_map;
  int n_seqs, W, hq, hkv;
  int64_t total_qtiles, total_ktiles;
  float scale;
  // bf16 path: the query heads of every KV head that one launch covers (set per launch)
  int head0, heads;
  const int32_t* n_tiles_dev;  // null, or where the launch reads its number of query tiles
  // bf16 path, workspace: the 256-row query tiles derived from the block map (see k_wide_rows)
  int32_t* wide_count;  // [1] number of 256-row tiles
  int32_t* wide_cnt;    // [total_qtiles] tiles in the row starting at this 64-row tile, -1: none starts here
  int32_t* wide_pre;    // [total_qtiles][8] descriptor of that row
  int32_t* wide_desc;   // [total_qtiles][8] descriptors in launch order (wide_count of them)
  int32_t* wide_col;    // [csr_capacity] key tiles of the rows, row of tile qt at rowptr[qt]
};

// Workspace of the bf16 path behind the transposed V: counters, then the tables above.
inline size_t prefill_bf16_table_bytes(int64_t total_qtiles, int64_t csr_capacity) {
  return (size_t)(DAG_SCHED_INTS + 64 + 17 * total_qtiles + csr_capacity) * 4;
}

// Paged prefill: the kernel argument block (q, k = K pool, vt = V pool, out, lse, sched, hq, hkv,
// scale, head0 / heads, and the five table pointers, of which wide_col holds the tile entries)
// plus what the table kernel reads.
struct PagedPrefillArgs {
  PrefillArgs a;
  int n_nodes, qt_max, nt_max, n_pages;
  const int32_t *q_off, *ctx_page_off, *ctx_pages, *ctx_page_len, *own_page, *own_len;
};
int launch_prefill_paged(const PagedPrefillArgs& pa, int head_dim, hipStream_t stream);

int launch_prefill_f32(const PrefillArgs& a, int head_dim, hipStream_t stream);
int launch_prefill_bf16_prepare_v(const PrefillArgs& a, int head_dim, hipStream_t stream);  // V -> workspace copy
int launch_prefill_bf16(const PrefillArgs& a, int head_dim, hipStream_t stream);            // needs the copy
