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
  int n_seqs, W, hq, hkv;
  int64_t total_qtiles, total_ktiles;
  float scale;
};

int launch_prefill_f32(const PrefillArgs& a, int head_dim, hipStream_t stream);
int launch_prefill_bf16_prepare_v(const PrefillArgs& a, int head_dim, hipStream_t stream);  // V -> workspace copy
int launch_prefill_bf16(const PrefillArgs& a, int head_dim, hipStream_t stream);            // needs the copy
