/*
 * dagattn -- DAG-structured attention for AMD MI355X (gfx950).  C ABI.
 *
 * The operation is the attention of MedVerse (arXiv 2602.07529), section 4.2: a token sequence is
 * organised as a DAG of reasoning nodes (the places of the Petri net of section 3.2); a token
 * attends causally inside its own node and fully to every ancestor node (Eq. 3 in its
 * ancestor-closure form, i.e. the Fork/Join semantics of sections 3.3 and 4.3), and carries an
 * adaptive position index (section 4.2, "Adaptive Position Indices"): sibling branches restart at
 * their fork point and a join resumes one past the largest position of its predecessors.
 *
 * General conventions
 *   - Every function returns DAG_OK (0) or a negative dag_status_t; dag_strerror() names it.
 *   - "HOST" pointers are read synchronously during the call.  "DEVICE" pointers are caller-owned
 *     GPU memory (for instance torch tensors); the library never allocates or frees device memory,
 *     scratch comes from a caller-provided workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All GPU work is
 *     enqueued on it and the call returns without synchronising.  Host-side validation happens
 *     before anything is enqueued; on a validation error no GPU work has been submitted.
 *   - Tensors are token-major packed variable-length: q [T][Hq][D], k/v [T][Hkv][D], contiguous,
 *     16-byte aligned.  Sequences are concatenated; tokens of a sequence are stored node after
 *     node in node-id order and node ids must be a topological order of the DAG.
 *   - Process-wide state: none that a result depends on.  What the library keeps until the
 *     process ends is (a) per device, the address of the scratch array of
 *     dag_attn_decode_static (see there), (b) attributes set on its own kernels, and (c) the
 *     development knobs of the decode split sizes and of the prefill head split, read from the
 *     environment once.  It creates no streams and no events.  Calls on different streams may
 *     overlap if their buffers (workspaces included) do not.
 */
#ifndef DAGATTN_H
#define DAGATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DAG_PAGE_SIZE 16

typedef enum {
  DAG_OK = 0,
  DAG_ERR_NULL = -1,            /* a required pointer is NULL                                   */
  DAG_ERR_BAD_LEN = -2,         /* a node length < 1, a negative count, or an inconsistent size  */
  DAG_ERR_NOT_TOPOLOGICAL = -3, /* ancestor bit u >= v set in row v (also rejects cycles)        */
  DAG_ERR_NOT_CLOSED = -4,      /* DAG_STRICT_CLOSURE set and the bitsets are not transitive     */
  DAG_ERR_POS_OVERFLOW = -5,    /* a sequence has more tokens than fit an int32 position         */
  DAG_ERR_WORKSPACE = -6,       /* workspace missing or too small                                */
  DAG_ERR_UNSUPPORTED = -7,     /* head_dim / head counts / page size / tile shape not supported */
  DAG_ERR_ALIGN = -8,           /* a tensor pointer is not 16-byte aligned                       */
  DAG_ERR_HIP = -9              /* the HIP runtime reported an error at launch                   */
} dag_status_t;

typedef enum { DAG_F32 = 0, DAG_BF16 = 1 } dag_dtype_t;

/* dag_desc_t.flags */
#define DAG_STRICT_CLOSURE 1u /* reject ancestor bitsets that are not transitively closed */

/* Block-map tile classes */
#define DAG_TILE_SKIP 0
#define DAG_TILE_PARTIAL 1
#define DAG_TILE_FULL 2

/* Node table of a batch of DAGs (sections 3.1-3.2: nodes = reasoning states).  HOST memory. */
typedef struct {
  int32_t n_seqs;
  const int32_t* node_offsets; /* [n_seqs+1] prefix sum of node counts                          */
  const int32_t* node_len;     /* [total_nodes] tokens per node, each >= 1                      */
  const uint64_t* anc_bits;    /* [total_nodes][words_per_node]; bit u of row v set <=> node u
                                  (local id within the sequence) is an ancestor of node v.  The
                                  self bit is ignored.                                           */
  int32_t words_per_node;      /* >= ceil(max nodes per sequence / 64)                          */
  int32_t tile_m, tile_n;      /* block-map tile shape; use dag_prefill_tile_shape()            */
  uint32_t flags;
} dag_desc_t;

/* Element counts a caller needs to allocate dag_meta_t (all filled by dag_meta_sizes). */
typedef struct {
  int64_t total_nodes;
  int64_t total_tokens;    /* T                                                                */
  int64_t total_qtiles;    /* sum over sequences of ceil(T_b / tile_m)                         */
  int64_t total_ktiles;    /* sum over sequences of ceil(T_b / tile_n)                         */
  int64_t total_tiles;     /* sum over sequences of QT_b * KT_b  (bytes of the dense map)      */
  int64_t csr_capacity;    /* upper bound on the number of non-skip tiles, plus 8 spare entries */
  int64_t workspace_bytes; /* device scratch needed by dag_build_meta                          */
} dag_meta_sizes_t;

/* Derived per-token / per-tile tables.  The struct lives on the HOST; every pointer is DEVICE
 * memory allocated by the caller with the element counts of dag_meta_sizes_t.  Written by
 * dag_build_meta, read by dag_rope_qk (pos_ids) and dag_attn_prefill. */
typedef struct {
  /* scalars copied from the description / sizes by the caller */
  int32_t n_seqs, words_per_node, tile_m, tile_n;
  dag_meta_sizes_t sizes;
  /* device arrays */
  int32_t* cu_seqlens;     /* [n_seqs+1] token offset of each sequence                         */
  int32_t* node_start;     /* [n_seqs+1] device copy of the node offsets                       */
  int32_t* tok_node;       /* [T] node id (local to the sequence) of every token               */
  int32_t* pos_ids;        /* [T] adaptive position of every token                             */
  int32_t* node_tok_start; /* [total_nodes] first token of the node, relative to its sequence  */
  int32_t* node_pos_start; /* [total_nodes] adaptive position of the node's first token        */
  uint64_t* node_vis;      /* [total_nodes][words_per_node] ancestors | self                   */
  int32_t* qtile_start;    /* [n_seqs+1] index of each sequence's first query tile             */
  int32_t* ktile_start;    /* [n_seqs+1] index of each sequence's first key tile               */
  int64_t* block_map_off;  /* [n_seqs+1] offset of each sequence's dense map                   */
  uint8_t* block_map;      /* [total_tiles] per sequence row-major [QT_b][KT_b], DAG_TILE_*    */
  int32_t* qtile_rowptr;   /* [total_qtiles+1] CSR over non-skip tiles; within a row the FULL
                              tiles come first (key tiles ascending), then the PARTIAL ones   */
  int32_t* qtile_col;      /* [csr_capacity] key-tile index                                    */
  uint8_t* qtile_flag;     /* [csr_capacity] DAG_TILE_PARTIAL or DAG_TILE_FULL                 */
  int32_t* qtile_nfull;    /* [total_qtiles] number of FULL tiles in the row                   */
  int32_t* qtile_order;    /* [total_qtiles] launch order: all query tiles by descending tile
                              count (ties: ascending index)                                    */
  int32_t* qtile_desc;     /* [total_qtiles][8] per launch slot: token offset of the sequence,
                              its token count, first row of the tile, CSR row start, tiles in
                              the row, leading tiles that need no mask (FULL and not ragged),
                              node offset of the sequence, first key tile of the sequence      */
  int64_t* useful_pairs;   /* [n_seqs] number of visible (query, key) pairs                    */
} dag_meta_t;

/* Tile shape the prefill kernel for this head configuration works on (section 4.2 gives no
 * kernel; the block map is this library's own device for skipping fully masked tiles).
 * Output pointers are HOST. */
int dag_prefill_tile_shape(int32_t hq, int32_t hkv, int32_t head_dim, dag_dtype_t dtype,
                           int32_t* tile_m, int32_t* tile_n);

/* Sizes of everything dag_build_meta writes.  Host only; validates lengths and counts. */
int dag_meta_sizes(const dag_desc_t* desc, dag_meta_sizes_t* out);

/* Section 4.2 (Eq. 3 + adaptive position indices): from the node table derive, on the GPU, the
 * per-token node ids and position ids, the per-node visibility bitsets, the tile-level block map
 * (dense + CSR), the launch order and the visible-pair counts.  The host validates the DAG first
 * (lengths >= 1, topological bitsets -- the paper's DAG validity check of its data pipeline,
 * section 4.1 --, optional closure check) and returns an error before any GPU work is enqueued.
 * `ws` is DEVICE scratch of at least sizes.workspace_bytes, 16-byte aligned. */
int dag_build_meta(const dag_desc_t* desc, const dag_meta_t* meta, void* ws, size_t ws_bytes,
                   void* stream);

/* Eq. 2's position embedding P(i) as rotary embedding at the adaptive positions: rotates q
 * [n_tokens][hq][head_dim] and k [n_tokens][hkv][head_dim] in place (either may be NULL) by the
 * angle pos_ids[t] * theta^(-2m/head_dim), pairing elements (m, m + head_dim/2).  All DEVICE.
 * head_dim must be even and <= 256. */
int dag_rope_qk(const int32_t* pos_ids, int64_t n_tokens, void* q, void* k, int32_t hq,
                int32_t hkv, int32_t head_dim, float theta, dag_dtype_t dtype, void* stream);

/* Eq. 2 + Eq. 3: out[i] = sum_j softmax_j(q_i . k_j * softmax_scale + M_ij) v_j, where M is the
 * DAG mask described by `meta`.  q/out [T][hq][head_dim], k/v [T][hkv][head_dim] DEVICE, already
 * rotated; lse (nullable) [T][hq] fp32 receives log sum exp of the scaled scores.  Fully masked
 * tiles are skipped through the block map; only PARTIAL tiles evaluate per-token masks.
 * Supported: DAG_BF16 with head_dim 64 or 128 (MFMA path, fp32 accumulation); DAG_F32 with
 * head_dim 64 or 128; hq a multiple of hkv.  meta->tile_m/tile_n must equal
 * dag_prefill_tile_shape() for the same configuration.  `ws` is DEVICE scratch of at least
 * dag_prefill_workspace_bytes() bytes, 256-byte aligned (the bf16 path keeps a key-tile-wise
 * transposed copy of V there); it may be NULL when that size is 0. */
int dag_attn_prefill(const dag_meta_t* meta, const void* q, const void* k, const void* v,
                     void* out, float* lse, int32_t hq, int32_t hkv, int32_t head_dim,
                     float softmax_scale, dag_dtype_t dtype, void* ws, size_t ws_bytes,
                     void* stream);

/* The two halves of dag_attn_prefill (Eq. 2 + Eq. 3), for callers that want them as separate
 * launches, e.g. to time the attention kernel alone or to prepare V while Q and K are still being
 * produced.  dag_prefill_prepare_v writes the key-tile-wise transposed copy of v [T][hkv][head_dim]
 * into `ws` (a no-op for DAG_F32); dag_attn_prefill_prepared is dag_attn_prefill without that
 * step: it expects `ws` as dag_prefill_prepare_v left it for the same meta, v, hkv, head_dim and
 * dtype.  Arguments, layouts, errors and the workspace size are those of dag_attn_prefill.
 * The workspace also holds the attention kernel's work-distribution counters: dag_prefill_prepare_v
 * zeroes them and every attention launch leaves them zeroed, so a workspace must go through
 * dag_prefill_prepare_v (or dag_attn_prefill) once before dag_attn_prefill_prepared uses it, and
 * two attention launches must not use one workspace at the same time. */
int dag_prefill_prepare_v(const dag_meta_t* meta, const void* v, int32_t hq, int32_t hkv,
                          int32_t head_dim, dag_dtype_t dtype, void* ws, size_t ws_bytes, void* stream);
int dag_attn_prefill_prepared(const dag_meta_t* meta, const void* q, const void* k, const void* v,
                              void* out, float* lse, int32_t hq, int32_t hkv, int32_t head_dim,
                              float softmax_scale, dag_dtype_t dtype, void* ws, size_t ws_bytes,
                              void* stream);

/* Bytes of DEVICE workspace dag_attn_prefill needs (host only; 0 for the fp32 path). */
size_t dag_prefill_workspace_bytes(const dag_meta_t* meta, int32_t hkv, int32_t head_dim,
                                   dag_dtype_t dtype);

/* Backward of dag_attn_prefill (section 4.2: the model is fine-tuned through the mask of Eq. 3):
 * from the incoming gradient dout [T][hq][head_dim] of the attention output, the forward's inputs
 * (q and k rotated, as the forward took them), its output `out` and log-sum-exp `lse` [T][hq]
 * (natural log, as dag_attn_prefill writes it), compute
 *   dq [T][hq][head_dim], dk and dv [T][hkv][head_dim]   (gradients w.r.t. the rotated q and k; a KV
 *   head's gradient is the sum over its query heads)
 * with P recomputed from lse: dV = P^T dO, dS = P o (dO V^T - rowsum(dO o O)), dQ = scale dS K,
 * dK = scale dS^T Q, only over the tiles the block map marks visible.  DAG_BF16 (MFMA, fp32
 * accumulation; gradients bf16) or DAG_F32 (plain fp32 arithmetic, the accuracy path; gradients
 * fp32), head_dim 128 or 64; all tensors DEVICE, 16-byte aligned; `ws` DEVICE scratch of
 * dag_prefill_bwd_workspace_bytes.  `meta` is the one dag_build_meta filled for the forward: the
 * bf16 path reads its block map, launch order, tile descriptors and FULL-first CSR.  No atomics:
 * results are bit-identical from run to run.  Errors as dag_attn_prefill. */
size_t dag_prefill_bwd_workspace_bytes(const dag_meta_t* meta, int32_t hq, int32_t hkv, int32_t head_dim);
int dag_attn_prefill_bwd(const dag_meta_t* meta, const void* q, const void* k, const void* v,
                         const void* out, const void* dout, const float* lse, void* dq, void* dk,
                         void* dv, int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale,
                         dag_dtype_t dtype, void* ws, size_t ws_bytes, void* stream);

/* One decode step over a paged KV cache (section 3.2: a token carries KV-cache indices, not
 * copies; section 4.3 Fork: sibling branches share the prefix KV without copying).  The struct
 * lives on the HOST; arrays are DEVICE int32.  A sibling group is a set of live branches that
 * share one context (list of pages); each live branch additionally owns a page list.
 * Pool storage formats (bf16, page size 16), P = number of pages:
 *   K pool [P][hkv][head_dim/8][16][8]   element (page, h, slot, d) at [page][h][d/8][slot][d%8]
 *   V pool [P][hkv][head_dim][16]        element (page, h, slot, d) at [page][h][d][slot]       */
typedef struct {
  int32_t n_groups, n_live, page_size;
  int32_t max_shared_pages; /* HOST upper bound on pages of any group's shared context          */
  int32_t max_branch_pages; /* HOST upper bound on pages owned by any live branch               */
  int32_t max_group_size;   /* HOST upper bound on live branches in any group                   */
  const int32_t* group_branch_off; /* [n_groups+1] live branches of group g are contiguous     */
  const int32_t* shared_page_off;  /* [n_groups+1] into shared_pages                           */
  const int32_t* shared_pages;     /* page ids of the shared contexts, in token order          */
  const int32_t* shared_len;       /* [n_groups] tokens in the shared context                  */
  const int32_t* branch_page_off;  /* [n_live+1] into branch_pages                             */
  const int32_t* branch_pages;     /* page ids owned by each live branch                       */
  const int32_t* branch_len;       /* [n_live] tokens in own pages, incl. the one being decoded */
  const int32_t* branch_pos;       /* [n_live] adaptive position of the token being decoded    */
} dag_decode_desc_t;

/* Section 3.2 (a fired transition's new KV blocks are added to the cache references its token
 * carries): store the new token of every live branch -- key rotated at branch_pos (Eq. 2's P(i)),
 * value as is -- into slot branch_len-1 of the branch's own page list.  k_new/v_new
 * [n_live][hkv][head_dim] bf16 DEVICE; head_dim 64 or 128 (DAG_ERR_UNSUPPORTED otherwise).
 * Slots of a page that no token has been stored in yet may hold anything, non-finite bit patterns
 * included: the decode kernels never let them reach a result. */
int dag_kv_append_rope(const dag_decode_desc_t* desc, const void* k_new, const void* v_new,
                       void* k_pool, void* v_pool, int32_t hkv, int32_t head_dim, float theta,
                       void* stream);

/* Bytes of DEVICE workspace dag_attn_decode needs for this description (0 on bad arguments). */
size_t dag_decode_workspace_bytes(const dag_decode_desc_t* desc, int32_t hq, int32_t hkv,
                                  int32_t head_dim);

/* Attention of every live branch's query over (shared context, own tokens): Eq. 2 without a mask
 * other than membership.  The shared pages of a group are streamed once for all its siblings
 * (section 4.3 Fork), own pages once per branch, and the partial results are combined by
 * log-sum-exp.  q/out [n_live][hq][head_dim] bf16 DEVICE, q already rotated.  head_dim 128 or
 * 64, page_size 16, hq a multiple of hkv with hq/hkv <= 32.
 * Everything is enqueued on `stream` (two launches: the partial results, their combination);
 * the call allocates nothing and does not synchronise. */
int dag_attn_decode(const dag_decode_desc_t* desc, const void* q, const void* k_pool,
                    const void* v_pool, void* out, int32_t hq, int32_t hkv, int32_t head_dim,
                    float softmax_scale, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): dag_attn_decode with its partial
 * results kept in a device array of the library itself, DAG_DECODE_STATIC_SCRATCH_BYTES long,
 * which every GPU the library runs on holds until the process ends.  Arguments, results (bit for
 * bit), layouts and errors as dag_attn_decode, except:
 *   - DAG_ERR_WORKSPACE when dag_decode_workspace_bytes() for this description exceeds
 *     DAG_DECODE_STATIC_SCRATCH_BYTES (benchmark configs 3 and 5 need 11 and 24 MiB);
 *   - the call allocates nothing and frees nothing.  Its first call on a device looks up the
 *     array's address there (hipGetSymbolAddress), so make one call per device outside a capture;
 *   - all calls on one GPU share the array, which keeps the last call's contents (every partial
 *     that is read has been written by the same call, so nothing needs clearing): calls that
 *     overlap on one GPU, on whatever streams, race -- order them. */
#define DAG_DECODE_STATIC_SCRATCH_BYTES (32u << 20)
int dag_attn_decode_static(const dag_decode_desc_t* desc, const void* q, const void* k_pool,
                           const void* v_pool, void* out, int32_t hq, int32_t hkv, int32_t head_dim,
                           float softmax_scale, void* stream);

/* One decode step over a general DAG frontier, contexts given as lists of KV segments (section
 * 3.2: a token carries references to cached blocks, not copies; section 4.3: a Fork hands every
 * child the same context, a Join reads the histories of all its predecessors and the context
 * before them, without padding or copying).  A segment is a page list with a token count (its last
 * page may be partly filled) and the list of live branches that read it; a live branch's context
 * is the union of the segments it reads, e.g. the segments of its ancestors and its own (which
 * holds the token being decoded).  Any number of sharing levels: a root segment read by all
 * branches, a mid-level one by a sub-group, an own one by a single branch.  Each branch also
 * lists where it appears in the reader lists (the inverse relation, as positions in seg_readers):
 * that is how its partial results are found.
 * The struct lives on the HOST; arrays are DEVICE int32; pools as for dag_attn_decode.
 * Appending a branch's new token is dag_kv_append_rope with branch_page_off / branch_pages /
 * branch_len / branch_pos describing the branches' own (tail) segments.
 * seg_reader_len turns the step into the incremental prefill of newly forked or joined nodes
 * against the cached context: the n new tokens of a node are n "live branches" that read the
 * ancestors' segments in full and the first L - n + i + 1 tokens of the node's own segment
 * (token i of the new ones, L the segment's length after all n were appended), which is the
 * node's causal part of Eq. 3. */
typedef struct {
  int32_t n_live, n_segments, page_size;
  int32_t max_seg_pages;  /* HOST upper bound on pages of any segment                            */
  int32_t max_readers;    /* HOST upper bound on readers of any segment                          */
  int32_t total_readers;  /* HOST: seg_reader_off[n_segments] (= branch_entry_off[n_live])       */
  const int32_t* seg_page_off;   /* [n_segments+1] into seg_pages                               */
  const int32_t* seg_pages;      /* page ids of each segment, in token order                    */
  const int32_t* seg_len;        /* [n_segments] tokens in the segment (0 allowed)              */
  const int32_t* seg_reader_off; /* [n_segments+1] into seg_readers                             */
  const int32_t* seg_readers;    /* live branches reading each segment, each once, any order    */
  const int32_t* branch_entry_off; /* [n_live+1] into branch_entries                            */
  const int32_t* branch_entries; /* for each live branch r: the positions e in seg_readers with
                                    seg_readers[e] == r, one per segment it reads, any order    */
  const int32_t* seg_reader_len; /* NULL, or [total_readers]: how many leading tokens of the
                                    segment the reader of entry e sees (clamped to seg_len)     */
} dag_decode_seg_desc_t;

/* Bytes of DEVICE workspace dag_attn_decode_segments needs for this description (0 on bad
 * arguments). */
size_t dag_decode_segments_workspace_bytes(const dag_decode_seg_desc_t* desc, int32_t hq, int32_t hkv,
                                           int32_t head_dim);

/* Attention of every live branch's query over the tokens of the segments it reads: Eq. 2 with
 * membership as the only mask.  Every segment is streamed once per 32 stacked query rows of its
 * readers (readers x hq/hkv rows per KV head), in slices, and the partial results of a branch are
 * combined by log-sum-exp.  q/out [n_live][hq][head_dim] bf16 DEVICE, q already rotated; a branch
 * that reads no token gets zeros.  head_dim 128 or 64, page_size 16, hq a multiple of hkv with
 * hq/hkv <= 32.  Errors as dag_attn_decode; the host bounds are trusted (a reader list longer
 * than max_readers loses rows, entries past total_readers are dropped).  Everything is enqueued
 * on `stream`; the call allocates nothing and does not synchronise. */
int dag_attn_decode_segments(const dag_decode_seg_desc_t* desc, const void* q, const void* k_pool,
                             const void* v_pool, void* out, int32_t hq, int32_t hkv, int32_t head_dim,
                             float softmax_scale, void* ws, size_t ws_bytes, void* stream);

/* Prefill of new tokens against cached, paged KV (section 4.3, phase II: when a step header or
 * a join prompt is given, its tokens are prefilled in one pass over the KV of all predecessor
 * paths and the preceding context, concatenated by reference, without padding or copying).  Each
 * of the n_nodes nodes has n_i >= 0 new tokens whose K/V are already in the node's own pages
 * (dag_kv_append_rope); its context is a list of pages in token order -- the segments it reads,
 * then its own pages -- with the number of tokens each page holds (a segment's last page may be
 * partly filled).  New token i of a node sees every token of the pages in front of its own and
 * its own node's tokens 0 .. own_len - n_i + i: Eq. 3 for a node whose ancestors are cached.
 * All arrays DEVICE int32; the two bounds are HOST values the launch is sized by (a node with
 * more new tokens or pages than the bounds say loses the excess). */
typedef struct {
  int32_t n_nodes, page_size;  /* page_size must be 16                                            */
  int32_t max_new;             /* HOST upper bound on the new tokens of any node                 */
  int32_t max_ctx_pages;       /* HOST upper bound on the pages in any node's context            */
  const int32_t* q_off;        /* [n_nodes+1] rows of q / out that are node i's new tokens       */
  const int32_t* ctx_page_off; /* [n_nodes+1] into ctx_pages / ctx_page_len                      */
  const int32_t* ctx_pages;    /* page ids of every context, own pages last                      */
  const int32_t* ctx_page_len; /* tokens in each of these pages, 0..16                           */
  const int32_t* own_page;     /* [n_nodes] index inside its context of the node's first own page */
  const int32_t* own_len;      /* [n_nodes] tokens in the node's own pages, the new ones included */
} dag_paged_prefill_desc_t;

/* Bytes of DEVICE workspace dag_attn_prefill_paged needs (0 on bad arguments). */
size_t dag_prefill_paged_workspace_bytes(const dag_paged_prefill_desc_t* desc);

/* q / out [q_off[n_nodes]][hq][head_dim] bf16 DEVICE (q already rotated), lse NULL or
 * [q_off[n_nodes]][hq] fp32 DEVICE (natural logarithm of the softmax denominator, as in
 * dag_attn_prefill); pools as in dag_attn_decode, n_pages = pages in each pool (page ids outside
 * are clamped, never followed).  head_dim 64 or 128, hq a multiple of hkv.  The tables of work
 * items are built on the device from the description; everything is enqueued on `stream`, the
 * call allocates nothing and does not synchronise.  Errors: DAG_ERR_NULL, DAG_ERR_BAD_LEN,
 * DAG_ERR_UNSUPPORTED, DAG_ERR_ALIGN, DAG_ERR_WORKSPACE, DAG_ERR_HIP. */
int dag_attn_prefill_paged(const dag_paged_prefill_desc_t* desc, const void* q, const void* k_pool,
                           const void* v_pool, int32_t n_pages, void* out, float* lse, int32_t hq,
                           int32_t hkv, int32_t head_dim, float softmax_scale, void* ws,
                           size_t ws_bytes, void* stream);

/* Host-side scheduler of the execution phase (section 3.2: the plan as a Petri net whose places
 * are the DAG nodes, one transition per node with its parents as input places; section 3.3, Eq. 1:
 * the enabled-transition frontier fires as a whole and the marking advances when all of it is
 * complete; Fork = children read the parent's pages by reference, Join = a node reads the
 * histories of all its predecessors).  Pure HOST code, no GPU call: it decides which transitions
 * are live, hands out pages of the KV pool (never copied, never moved), assigns adaptive positions
 * (section 4.2) and writes, per step, the descriptions dag_kv_append_rope and
 * dag_attn_decode_segments take.  The caller uploads them and runs the model between steps.
 *
 * dag_sched_create: nodes in topological order (parents[parent_off[v] .. parent_off[v+1]) < v,
 * else DAG_ERR_NOT_TOPOLOGICAL; DAG_ERR_POS_OVERFLOW when an adaptive position would not fit an
 * int32 -- positions depend on the plan only, so this is the one place where that is reported); node_len[v] >= 1 tokens to produce for node v; chunk[v] >= 1
 * tokens per step (NULL: 1 everywhere = token-by-token generation; more for a node whose text is
 * given, e.g. the prompt or a step header, which is then prefilled in pieces); n_pages pages of
 * page_size (16) tokens in the pool, handed out in ascending order.  All arrays HOST, copied.
 * dag_sched_destroy frees the object (NULL allowed). */
typedef struct dag_sched dag_sched_t;
int dag_sched_create(int32_t n_nodes, const int32_t* parent_off, const int32_t* parents,
                     const int32_t* node_len, const int32_t* chunk, int32_t n_pages, int32_t page_size,
                     dag_sched_t** out);
void dag_sched_destroy(dag_sched_t* sched);

/* One step: n_live new tokens ("live branches"; 0 = the net has no enabled transition left).
 * Entry r is token live_token[r] of node live_node[r]; the caller feeds the model with these
 * tokens, stores their K/V with dag_kv_append_rope (branch_* arrays: the node's page list, the
 * token count of the node including entry r, its adaptive position) and attends with
 * dag_attn_decode_segments (seg_* / branch_entr* arrays and the four host bounds; segment i holds
 * node seg_node[i]).  All pointers are HOST memory owned by the scheduler, valid until the next
 * call on it; the caller copies them to the device.  DAG_ERR_WORKSPACE when the pool has too few
 * free pages for the step: no page is handed out and no token is counted then (the marking may
 * already have advanced to the step's frontier, which a repeated call finds unchanged). */
typedef struct {
  int32_t n_live, layer;          /* layer: index k of the frontier F_k the step belongs to         */
  int32_t n_segments, max_seg_pages, max_readers, total_readers;
  int32_t n_branch_pages, n_seg_pages, pages_in_use;
  const int32_t* live_node;       /* [n_live]                                                       */
  const int32_t* live_token;      /* [n_live] index of the token inside its node                    */
  const int32_t* branch_page_off; /* [n_live+1] into branch_pages                                   */
  const int32_t* branch_pages;    /* [n_branch_pages]                                               */
  const int32_t* branch_len;      /* [n_live]                                                       */
  const int32_t* branch_pos;      /* [n_live]                                                       */
  const int32_t* seg_node;        /* [n_segments]                                                   */
  const int32_t* seg_page_off;    /* [n_segments+1] into seg_pages                                  */
  const int32_t* seg_pages;       /* [n_seg_pages]                                                  */
  const int32_t* seg_len;         /* [n_segments]                                                   */
  const int32_t* seg_reader_off;  /* [n_segments+1]                                                 */
  const int32_t* seg_readers;     /* [total_readers]                                                */
  const int32_t* seg_reader_len;  /* [total_readers]                                                */
  const int32_t* branch_entry_off;/* [n_live+1]                                                     */
  const int32_t* branch_entries;  /* [total_readers]                                                */
} dag_sched_step_t;
int dag_sched_step(dag_sched_t* sched, dag_sched_step_t* out);

/* Measurement aid, not part of the attention path: a plain device-to-device copy of `bytes`
 * (a multiple of 16; both pointers DEVICE, 16-byte aligned, not overlapping) by a kernel of the
 * library's own, k_copy_calibration.  Its reading of a hardware counter (HBM bytes fetched or
 * written) under a profiler gives the scale of that counter on the machine at hand: it reads
 * and writes exactly `bytes`.  Enqueued on `stream`; DAG_ERR_NULL / DAG_ERR_ALIGN. */
int dag_copy_calibration(void* dst, const void* src, size_t bytes, void* stream);

const char* dag_strerror(int code);
int dag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DAGATTN_H */
