// dag_meta_sizes / dag_build_meta: node table + ancestor bitsets -> per-token node ids, adaptive
// position ids (paper section 4.2), per-node visibility sets (Eq. 3 in ancestor-closure form),
// tile-level block map (dense + CSR), launch order, visible-pair counts.  Integer work only.
#include <vector>

#include "common.h"

namespace {

struct SeqDims {
  int64_t tokens, qtiles, ktiles;
};

// Host: sums and validation of the counts.  Returns DAG_OK or an error.
int host_dims(const dag_desc_t* d, std::vector<SeqDims>* per_seq, dag_meta_sizes_t* out) {
  if (!d || !out) return DAG_ERR_NULL;
  if (d->n_seqs < 0) return DAG_ERR_BAD_LEN;
  if (d->tile_m < 1 || d->tile_n < 1 || d->tile_m > 1024 || d->tile_n > 1024) return DAG_ERR_UNSUPPORTED;
  if (d->words_per_node < 1) return DAG_ERR_BAD_LEN;
  dag_meta_sizes_t s = {};
  if (d->n_seqs > 0 && (!d->node_offsets || !d->node_len || !d->anc_bits)) return DAG_ERR_NULL;
  if (d->n_seqs > 0 && d->node_offsets[0] != 0) return DAG_ERR_BAD_LEN;
  int64_t max_nodes = 0;
  for (int b = 0; b < d->n_seqs; ++b) {
    int64_t n0 = d->node_offsets[b], n1 = d->node_offsets[b + 1];
    if (n1 < n0) return DAG_ERR_BAD_LEN;
    if (n1 - n0 > max_nodes) max_nodes = n1 - n0;
    int64_t T = 0;
    for (int64_t v = n0; v < n1; ++v) {
      if (d->node_len[v] < 1) return DAG_ERR_BAD_LEN;
      T += d->node_len[v];
    }
    if (T > INT32_MAX) return DAG_ERR_POS_OVERFLOW;
    SeqDims sd;
    sd.tokens = T;
    sd.qtiles = dag_ceil_div(T, d->tile_m);
    sd.ktiles = dag_ceil_div(T, d->tile_n);
    if (per_seq) per_seq->push_back(sd);
    s.total_tokens += T;
    s.total_qtiles += sd.qtiles;
    s.total_ktiles += sd.ktiles;
    s.total_tiles += sd.qtiles * sd.ktiles;
    for (int64_t a = 0; a < sd.qtiles; ++a) {
      int64_t last_row = (a + 1) * d->tile_m < T ? (a + 1) * d->tile_m : T;
      s.csr_capacity += (last_row - 1) / d->tile_n + 1;  // key tiles that start at or before the last row
    }
  }
  s.csr_capacity += 8;  // spare entries: the prefill kernel reads the column list eight entries at a time
  if (s.total_tokens > INT32_MAX || s.total_qtiles > INT32_MAX || s.csr_capacity > INT32_MAX)
    return DAG_ERR_POS_OVERFLOW;
  if (d->n_seqs > 0) s.total_nodes = d->node_offsets[d->n_seqs];
  if (max_nodes > (int64_t)d->words_per_node * 64) return DAG_ERR_BAD_LEN;
  if (max_nodes > 16384) return DAG_ERR_UNSUPPORTED;  // per-sequence node table is kept in LDS
  size_t ws = 0;
  ws += dag_align_up((size_t)(d->n_seqs + 1) * 4, 16);
  ws += dag_align_up((size_t)s.total_nodes * 4, 16);
  ws += dag_align_up((size_t)s.total_nodes * d->words_per_node * 8, 16);
  ws += dag_align_up((size_t)(s.total_qtiles + 1) * 4, 16);
  s.workspace_bytes = (int64_t)ws + 16;
  *out = s;
  return DAG_OK;
}

int host_validate_bits(const dag_desc_t* d) {
  const int W = d->words_per_node;
  for (int b = 0; b < d->n_seqs; ++b) {
    const int64_t n0 = d->node_offsets[b];
    const int n = d->node_offsets[b + 1] - d->node_offsets[b];
    for (int v = 0; v < n; ++v) {
      const uint64_t* row = d->anc_bits + (n0 + v) * W;
      // bits above v must be clear; the self bit is ignored
      for (int w = 0; w < W; ++w) {
        uint64_t allowed;
        int lo = w * 64;
        if (v < lo) allowed = 0;
        else if (v >= lo + 63) allowed = ~0ull;
        else allowed = (2ull << (v - lo)) - 1;  // bits 0..v-lo (includes the self bit)
        if (row[w] & ~allowed) return DAG_ERR_NOT_TOPOLOGICAL;
      }
      if (d->flags & DAG_STRICT_CLOSURE) {
        for (int u = 0; u < v; ++u) {
          if (!((row[u >> 6] >> (u & 63)) & 1)) continue;
          const uint64_t* ru = d->anc_bits + (n0 + u) * W;
          for (int w = 0; w < W; ++w) {
            uint64_t need = ru[w];
            if ((u >> 6) == w) need &= ~(1ull << (u & 63));  // u's own self bit does not count
            if (need & ~row[w]) return DAG_ERR_NOT_CLOSED;
          }
        }
      }
    }
  }
  return DAG_OK;
}

// ------------------------------------------------------------------------------------ kernels
// One block: per-sequence token counts and the three prefix sums over sequences; zeroes the
// per-row tile counts that k_blockmap adds up.
__device__ void seq_block(int n_seqs, const int32_t* node_off, const int32_t* node_len, int tile_m, int tile_n,
                          int32_t* cu_seqlens, int32_t* qtile_start, int64_t* block_map_off, int32_t* node_start,
                          int32_t* ktile_start, int32_t* cnt, int total_qtiles) {
  for (int i = threadIdx.x; i < total_qtiles; i += blockDim.x) cnt[i] = 0;
  for (int b = threadIdx.x; b <= n_seqs; b += blockDim.x) node_start[b] = node_off[b];
  for (int b = threadIdx.x; b < n_seqs; b += blockDim.x) {
    int t = 0;
    for (int v = node_off[b]; v < node_off[b + 1]; ++v) t += node_len[v];
    cu_seqlens[b + 1] = t;  // turned into a prefix sum below
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int cu = 0, qs = 0, ks = 0;
    int64_t mo = 0;
    cu_seqlens[0] = 0;
    qtile_start[0] = 0;
    ktile_start[0] = 0;
    block_map_off[0] = 0;
    for (int b = 0; b < n_seqs; ++b) {
      int t = cu_seqlens[b + 1];
      int qt = (t + tile_m - 1) / tile_m, kt = (t + tile_n - 1) / tile_n;
      cu += t;
      qs += qt;
      ks += kt;
      mo += (int64_t)qt * kt;
      cu_seqlens[b + 1] = cu;
      qtile_start[b + 1] = qs;
      ktile_start[b + 1] = ks;
      block_map_off[b + 1] = mo;
    }
  }
}

// One wave per sequence: node token starts (scan), visibility sets, adaptive position starts
// (section 4.2: 0 without ancestors, else one past the largest ancestor position), pair counts.
// One more block (the last) does the per-sequence sums of seq_block.
__global__ void __launch_bounds__(64) k_seq_node(int n_seqs, const int32_t* node_off, const int32_t* node_len,
                                                 const uint64_t* anc, int W, int tile_m, int tile_n,
                                                 int32_t* cu_seqlens, int32_t* qtile_start, int64_t* block_map_off,
                                                 int32_t* node_start, int32_t* ktile_start, int32_t* cnt,
                                                 int total_qtiles, int32_t* node_tok_start,
                                                 int32_t* node_pos_start, uint64_t* node_vis,
                                                 int64_t* useful_pairs, int anc_in_lds) {
  extern __shared__ uint64_t s_anc[];  // [n][W] ancestor words of the sequence, then int32 [n] + [n] below
  if ((int)blockIdx.x == n_seqs) {
    seq_block(n_seqs, node_off, node_len, tile_m, tile_n, cu_seqlens, qtile_start, block_map_off, node_start,
              ktile_start, cnt, total_qtiles);
    return;
  }
  const int b = blockIdx.x, lane = threadIdx.x;
  const int n0 = node_off[b], n = node_off[b + 1] - n0;
  // (the copy of the ancestor words is skipped for node tables too large for LDS; the walk below
  // then reads them from global memory, one dependent load per node)
  int32_t* s_pos_end = (int32_t*)(s_anc + (anc_in_lds ? (size_t)n * W : 0));  // [n] last position used by each node
  int32_t* s_len = s_pos_end + n;                                              // [n]
  const uint64_t* anc_rows = anc_in_lds ? s_anc : anc + (int64_t)n0 * W;
  if (anc_in_lds)
    for (int i = lane; i < n * W; i += 64) s_anc[i] = anc[(int64_t)n0 * W + i];
  int run = 0;
  for (int c = 0; c < n; c += 64) {
    int v = c + lane;
    int x = v < n ? node_len[n0 + v] : 0;
    int incl = x;
    for (int off = 1; off < 64; off <<= 1) {
      int y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    if (v < n) {
      node_tok_start[n0 + v] = run + incl - x;
      s_len[v] = x;
    }
    run += __shfl(incl, 63);
  }
  for (int v = lane; v < n; v += 64)
    for (int w = 0; w < W; ++w) {
      uint64_t bits = anc[(int64_t)(n0 + v) * W + w];  // (this lane's own row: no need to wait for the LDS copy)
      if ((v >> 6) == w) bits |= 1ull << (v & 63);
      node_vis[(int64_t)(n0 + v) * W + w] = bits;
    }
  __syncthreads();
  long long pairs = 0;
  for (int v = 0; v < n; ++v) {
    int best = -1;          // largest ancestor end position seen by this lane
    long long anc_tokens = 0;
    for (int w = 0; w * 64 <= v; ++w) {
      uint64_t bits = anc_rows[(size_t)v * W + w];
      int u = w * 64 + lane;
      if (u < v && ((bits >> lane) & 1)) {
        int e = s_pos_end[u];
        best = e > best ? e : best;
        anc_tokens += s_len[u];
      }
    }
    for (int off = 32; off >= 1; off >>= 1) {
      int o = __shfl_xor(best, off);
      best = o > best ? o : best;
      anc_tokens += __shfl_xor(anc_tokens, off);
    }
    const int start = best + 1;  // -1 + 1 = 0 for a node without ancestors
    const int len = s_len[v];
    if (lane == 0) {
      node_pos_start[n0 + v] = start;
      s_pos_end[v] = start + len - 1;
      pairs += (long long)len * anc_tokens + (long long)len * (len + 1) / 2;
    }
    __syncthreads();
  }
  if (lane == 0) useful_pairs[b] = pairs;
}

// One block per node: expand to tokens.
__global__ void k_tokens(int n_seqs, const int32_t* node_off, const int32_t* node_len,
                         const int32_t* cu_seqlens, const int32_t* node_tok_start,
                         const int32_t* node_pos_start, int32_t* tok_node, int32_t* pos_ids) {
  const int gv = blockIdx.x;
  const int b = dag_find_segment(node_off, n_seqs, gv);
  const int v = gv - node_off[b];
  const int base = cu_seqlens[b] + node_tok_start[gv];
  const int p0 = node_pos_start[gv], len = node_len[gv];
  for (int o = threadIdx.x; o < len; o += blockDim.x) {
    tok_node[base + o] = v;
    pos_ids[base + o] = p0 + o;
  }
}

// One thread per (query tile, key tile): exact count of visible pairs among the in-range pairs
// => SKIP / PARTIAL / FULL.  Also adds up the non-skip tiles of every query tile's row (cnt, zeroed
// before): tiles are numbered row after row, so a block touches at most blockDim.x consecutive
// rows; it counts them in LDS and adds each row's share to cnt once.
__global__ void __launch_bounds__(256) k_blockmap(int n_seqs, int64_t total_tiles, const int64_t* block_map_off,
                                                  const int32_t* cu_seqlens, const int32_t* node_off,
                                                  const int32_t* tok_node, const int32_t* node_tok_start,
                                                  const uint64_t* node_vis, int W, int tile_m, int tile_n,
                                                  const int32_t* qtile_start, uint8_t* block_map, int32_t* cnt) {
  __shared__ int s_rows[256];
  __shared__ int s_first;
  s_rows[threadIdx.x] = 0;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool valid = idx < total_tiles;
  int gq = 0;  // query tile (row of the block map) over the whole batch
  uint8_t state = DAG_TILE_SKIP;
  if (valid) {
    const int b = dag_find_segment(block_map_off, n_seqs, idx);
    const int T = cu_seqlens[b + 1] - cu_seqlens[b];
    const int KT = (T + tile_n - 1) / tile_n;
    const int64_t loc = idx - block_map_off[b];
    const int a = (int)(loc / KT), kb = (int)(loc % KT);
    gq = qtile_start[b] + a;
    const int i0 = a * tile_m, i1 = min(T, i0 + tile_m);
    const int j0 = kb * tile_n, j1 = min(T, j0 + tile_n);
    if (j0 <= i1 - 1) {  // else entirely in the future of every row
      const int32_t* tn = tok_node + cu_seqlens[b];
      const int n0 = node_off[b];
      const int nn = node_off[b + 1] - n0;
      const int u_lo = tn[i0], u_hi = tn[i1 - 1], w_lo = tn[j0], w_hi = tn[j1 - 1];
      long long allowed = 0;
      for (int u = u_lo; u <= u_hi; ++u) {
        const int us = node_tok_start[n0 + u];
        const int ue = (u + 1 < nn) ? node_tok_start[n0 + u + 1] : T;
        const int r0 = max(i0, us), r1 = min(i1, ue);
        for (int w = w_lo; w <= w_hi && w <= u; ++w) {
          const int ws = node_tok_start[n0 + w];
          const int we = (w + 1 < nn) ? node_tok_start[n0 + w + 1] : T;
          const int c0 = max(j0, ws), c1 = min(j1, we);
          if (w == u) {
            for (int i = r0; i < r1; ++i) {  // causal inside the node
              int c = min(i + 1, c1) - c0;
              if (c > 0) allowed += c;
            }
          } else if ((node_vis[(int64_t)(n0 + u) * W + (w >> 6)] >> (w & 63)) & 1) {
            allowed += (long long)(r1 - r0) * (c1 - c0);
          }
        }
      }
      const long long total = (long long)(i1 - i0) * (j1 - j0);
      state = allowed == 0 ? DAG_TILE_SKIP : (allowed == total ? DAG_TILE_FULL : DAG_TILE_PARTIAL);
    }
    block_map[idx] = state;
  }
  if (threadIdx.x == 0) s_first = gq;  // thread 0 is always valid (the grid covers total_tiles)
  __syncthreads();
  if (state != DAG_TILE_SKIP) atomicAdd(&s_rows[gq - s_first], 1);
  __syncthreads();
  if (s_rows[threadIdx.x] != 0) atomicAdd(cnt + s_first + threadIdx.x, s_rows[threadIdx.x]);
}

// One block: exclusive scan of the per-row counts (only used for a batch without tokens).
__global__ void __launch_bounds__(1024) k_csr_scan(int total_qtiles, const int32_t* cnt, int32_t* rowptr) {
  __shared__ int s[1024];
  __shared__ int carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int c0 = 0; c0 < total_qtiles; c0 += 1024) {
    int i = c0 + threadIdx.x;
    int x = i < total_qtiles ? cnt[i] : 0;
    s[threadIdx.x] = x;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      int y = threadIdx.x >= off ? s[threadIdx.x - off] : 0;
      __syncthreads();
      s[threadIdx.x] += y;
      __syncthreads();
    }
    if (i < total_qtiles) rowptr[i] = carry + s[threadIdx.x] - x;
    __syncthreads();
    if (threadIdx.x == 1023) carry += s[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) rowptr[total_qtiles] = carry;
}

// One wave per query tile, given the number of non-skip tiles of every row (cnt):
//  * CSR row start = sum of the counts in front of it, and launch slot = number of query tiles in
//    front of it in the order (tile count descending, index ascending), both from one pass over
//    cnt shared by the lanes.  The prefill kernel hands the launch list out dynamically, and with
//    the heaviest items first the workgroups finish within the duration of one of the lightest;
//  * ordered compaction of the row's non-skip tiles -- FULL tiles first (key tiles ascending),
//    then PARTIAL tiles (ascending) -- and the number of FULL tiles;
//  * the tile's launch record in its slot: everything the prefill kernel needs to start the
//    query tile, in 32 bytes {token offset of the sequence, tokens in the sequence, first row of
//    the tile, CSR row start, tiles in the row, tiles that need no mask, node offset of the
//    sequence, first key tile of the sequence}.
__global__ void __launch_bounds__(256) k_csr_order_desc(int n_seqs, int total_qtiles, int tile_m, int tile_n,
                                                        const int32_t* cnt, const int32_t* qtile_start,
                                                        const int64_t* block_map_off, const int32_t* cu_seqlens,
                                                        const int32_t* node_start, const int32_t* ktile_start,
                                                        const uint8_t* block_map, int32_t* rowptr, int32_t* col,
                                                        uint8_t* flag, int32_t* nfull, int32_t* order,
                                                        int32_t* desc) {
  const int qt = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (qt >= total_qtiles) return;
  const int mine = cnt[qt];
  int oi = 0, c0 = 0;
  for (int j = lane; j < total_qtiles; j += 64) {
    const int o = cnt[j];
    oi += (o > mine) || (o == mine && j < qt);
    c0 += j < qt ? o : 0;
  }
  for (int off = 32; off; off >>= 1) {
    oi += __shfl_xor(oi, off);
    c0 += __shfl_xor(c0, off);
  }
  const int b = dag_find_segment(qtile_start, n_seqs, qt);
  const int T = cu_seqlens[b + 1] - cu_seqlens[b];
  const int KT = (T + tile_n - 1) / tile_n;
  const uint8_t* row = block_map + block_map_off[b] + (int64_t)(qt - qtile_start[b]) * KT;
  int out = c0, nf = 0, last_full = -1;
  for (int pass = 0; pass < 2; ++pass) {
    const uint8_t want = pass == 0 ? DAG_TILE_FULL : DAG_TILE_PARTIAL;
    for (int k0 = 0; k0 < KT; k0 += 64) {
      const int k = k0 + lane;
      const uint8_t f = k < KT ? row[k] : (uint8_t)DAG_TILE_SKIP;
      const uint64_t m = __ballot(f == want);
      if (f == want) {
        const int p = out + __popcll(m & ((1ull << lane) - 1));
        col[p] = k;
        flag[p] = f;
      }
      out += __popcll(m);
      if (pass == 0 && m) last_full = k0 + 63 - __builtin_clzll(m);
    }
    if (pass == 0) nf = out - c0;
  }
  if (lane != 0) return;
  rowptr[qt] = c0;
  if (qt == total_qtiles - 1) rowptr[total_qtiles] = c0 + mine;
  nfull[qt] = nf;
  order[oi] = qt;
  if (nf > 0 && (last_full + 1) * tile_n > T) --nf;  // a ragged last key tile needs the mask path
  int32_t* d = desc + (int64_t)oi * 8;
  d[0] = cu_seqlens[b];
  d[1] = T;
  d[2] = (qt - qtile_start[b]) * tile_m;
  d[3] = c0;
  d[4] = mine;
  d[5] = nf;
  d[6] = node_start[b];
  d[7] = ktile_start[b];
}

}  // namespace

extern "C" int dag_prefill_tile_shape(int32_t hq, int32_t hkv, int32_t head_dim, dag_dtype_t dtype,
                                      int32_t* tile_m, int32_t* tile_n) {
  if (!tile_m || !tile_n) return DAG_ERR_NULL;
  if (hq < 1 || hkv < 1 || hq % hkv != 0) return DAG_ERR_UNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return DAG_ERR_UNSUPPORTED;
  if (dtype == DAG_F32) {
    *tile_m = 64;
    *tile_n = 64;
    return DAG_OK;
  }
  if (dtype != DAG_BF16) return DAG_ERR_UNSUPPORTED;
  // The block map is 64 x 64 for every head configuration: four-head items work on 64 query rows,
  // and the 256-row tiles of left-over heads are derived from four rows of this map.
  *tile_m = 64;
  *tile_n = 64;
  return DAG_OK;
}

extern "C" int dag_meta_sizes(const dag_desc_t* desc, dag_meta_sizes_t* out) {
  return host_dims(desc, nullptr, out);
}

extern "C" int dag_build_meta(const dag_desc_t* d, const dag_meta_t* m, void* ws, size_t ws_bytes,
                              void* stream_) {
  if (!d || !m) return DAG_ERR_NULL;
  dag_meta_sizes_t s;
  int rc = host_dims(d, nullptr, &s);
  if (rc != DAG_OK) return rc;
  if (m->n_seqs != d->n_seqs || m->words_per_node != d->words_per_node || m->tile_m != d->tile_m ||
      m->tile_n != d->tile_n || m->sizes.total_tokens != s.total_tokens ||
      m->sizes.total_qtiles != s.total_qtiles || m->sizes.total_tiles != s.total_tiles ||
      m->sizes.csr_capacity != s.csr_capacity || m->sizes.total_nodes != s.total_nodes)
    return DAG_ERR_BAD_LEN;
  if (d->n_seqs == 0) return DAG_OK;
  if (!m->cu_seqlens || !m->node_start || !m->qtile_start || !m->ktile_start || !m->block_map_off ||
      !m->qtile_rowptr || !m->useful_pairs)
    return DAG_ERR_NULL;
  if (s.total_tokens > 0 && (!m->tok_node || !m->pos_ids || !m->node_tok_start || !m->node_pos_start ||
                             !m->node_vis || !m->block_map || !m->qtile_col || !m->qtile_flag || !m->qtile_nfull || !m->qtile_order || !m->qtile_desc))
    return DAG_ERR_NULL;
  rc = host_validate_bits(d);
  if (rc != DAG_OK) return rc;
  if (!ws || ws_bytes < (size_t)s.workspace_bytes) return DAG_ERR_WORKSPACE;

  hipStream_t stream = (hipStream_t)stream_;
  const int W = d->words_per_node;
  char* p = (char*)dag_align_up((size_t)(uintptr_t)ws, 16);
  int32_t* d_off = (int32_t*)p;
  p += dag_align_up((size_t)(d->n_seqs + 1) * 4, 16);
  int32_t* d_len = (int32_t*)p;
  p += dag_align_up((size_t)s.total_nodes * 4, 16);
  uint64_t* d_anc = (uint64_t*)p;
  p += dag_align_up((size_t)s.total_nodes * W * 8, 16);
  int32_t* d_cnt = (int32_t*)p;

  DAG_HIP_CHECK(hipMemcpyAsync(d_off, d->node_offsets, (size_t)(d->n_seqs + 1) * 4, hipMemcpyHostToDevice, stream));
  if (s.total_nodes > 0) {
    DAG_HIP_CHECK(hipMemcpyAsync(d_len, d->node_len, (size_t)s.total_nodes * 4, hipMemcpyHostToDevice, stream));
    DAG_HIP_CHECK(hipMemcpyAsync(d_anc, d->anc_bits, (size_t)s.total_nodes * W * 8, hipMemcpyHostToDevice, stream));
  }
  int max_nodes = 0;
  for (int b = 0; b < d->n_seqs; ++b) {
    int n = d->node_offsets[b + 1] - d->node_offsets[b];
    if (n > max_nodes) max_nodes = n;
  }
  const unsigned QT = (unsigned)s.total_qtiles;
  const size_t anc_bytes = (size_t)max_nodes * W * 8;
  const int anc_in_lds = anc_bytes <= 32768;
  hipLaunchKernelGGL(k_seq_node, dim3(d->n_seqs + 1), dim3(64), (size_t)max_nodes * 8 + 8 + (anc_in_lds ? anc_bytes : 0), stream, d->n_seqs, d_off,
                     d_len, d_anc, W, d->tile_m, d->tile_n, m->cu_seqlens, m->qtile_start, m->block_map_off,
                     m->node_start, m->ktile_start, d_cnt, (int)QT, m->node_tok_start, m->node_pos_start, m->node_vis,
                     m->useful_pairs, anc_in_lds);
  DAG_LAUNCH_CHECK();
  if (s.total_tokens == 0) {
    hipLaunchKernelGGL(k_csr_scan, dim3(1), dim3(1024), 0, stream, 0, d_cnt, m->qtile_rowptr);
    DAG_LAUNCH_CHECK();
    return DAG_OK;
  }
  hipLaunchKernelGGL(k_tokens, dim3((unsigned)s.total_nodes), dim3(256), 0, stream, d->n_seqs, d_off, d_len,
                     m->cu_seqlens, m->node_tok_start, m->node_pos_start, m->tok_node, m->pos_ids);
  DAG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_blockmap, dim3((unsigned)dag_ceil_div(s.total_tiles, 256)), dim3(256), 0, stream, d->n_seqs,
                     s.total_tiles, m->block_map_off, m->cu_seqlens, d_off, m->tok_node, m->node_tok_start,
                     m->node_vis, W, d->tile_m, d->tile_n, m->qtile_start, m->block_map, d_cnt);
  DAG_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_csr_order_desc, dim3((QT + 3) / 4), dim3(256), 0, stream, d->n_seqs, (int)QT, d->tile_m,
                     d->tile_n, d_cnt, m->qtile_start, m->block_map_off, m->cu_seqlens, m->node_start, m->ktile_start,
                     m->block_map, m->qtile_rowptr, m->qtile_col, m->qtile_flag, m->qtile_nfull, m->qtile_order,
                     m->qtile_desc);
  DAG_LAUNCH_CHECK();
  return DAG_OK;
}
