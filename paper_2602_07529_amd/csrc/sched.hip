// Host-side scheduler of the execution phase (sections 3.2-3.3): the plan is a Petri net whose
// places are the DAG nodes and whose transitions produce one node each from its parents; the
// enabled-transition frontier (Eq. 1) fires as a whole, every transition of it advancing by its
// chunk of tokens per step, and the marking advances when the whole frontier is complete.  The
// scheduler owns the bookkeeping the engine text describes: which transitions are live, where
// their tokens go in the paged KV pool (pages are handed out from a free list and never copied:
// a child reads its ancestors' pages by reference), the adaptive position of every new token
// (section 4.2), and, per step, the descriptions dag_kv_append_rope and dag_attn_decode_segments
// take.  Pure host code: all arrays it returns are host memory, valid until the next call.
#include <stdint.h>

#include <algorithm>
#include <new>
#include <vector>

#include "dagattn.h"

struct dag_sched {
  int n = 0, words = 0, page_size = 16;
  std::vector<int32_t> parent_off, parents, len, chunk;
  std::vector<uint64_t> anc;  // [n][words], transitive closure of the parents
  std::vector<int32_t> free_pages;
  std::vector<std::vector<int32_t>> pages;
  std::vector<int32_t> done, pos_start;
  std::vector<char> marked;
  std::vector<int32_t> frontier;
  int layer = -1;
  int64_t steps = 0;
  // buffers of the current step
  std::vector<int32_t> live_node, live_token, b_page_off, b_pages, b_len, b_pos;
  std::vector<int32_t> seg_node, seg_page_off, seg_pages, seg_len, seg_reader_off, seg_readers, seg_reader_len;
  std::vector<int32_t> entry_off, entries;
  std::vector<int32_t> seg_of_node;
  std::vector<std::vector<int32_t>> entries_of;

  bool is_anc(int v, int u) const { return (anc[(size_t)v * words + (u >> 6)] >> (u & 63)) & 1u; }
};

extern "C" int dag_sched_create(int32_t n_nodes, const int32_t* parent_off, const int32_t* parents,
                                const int32_t* node_len, const int32_t* chunk, int32_t n_pages, int32_t page_size,
                                dag_sched_t** out) {
  if (!out) return DAG_ERR_NULL;
  *out = nullptr;
  if (n_nodes < 0 || n_pages < 0) return DAG_ERR_BAD_LEN;
  if (page_size != 16) return DAG_ERR_UNSUPPORTED;
  if (n_nodes > 0 && (!parent_off || !node_len)) return DAG_ERR_NULL;
  if (n_nodes > 0 && parent_off[0] != 0) return DAG_ERR_BAD_LEN;
  for (int v = 0; v < n_nodes; ++v) {
    if (parent_off[v + 1] < parent_off[v]) return DAG_ERR_BAD_LEN;
    if (node_len[v] < 1 || (chunk && chunk[v] < 1)) return DAG_ERR_BAD_LEN;
    if (parent_off[v + 1] > parent_off[v] && !parents) return DAG_ERR_NULL;
    for (int e = parent_off[v]; e < parent_off[v + 1]; ++e)
      if (parents[e] < 0 || parents[e] >= v) return DAG_ERR_NOT_TOPOLOGICAL;  // (also rejects cycles)
  }
  dag_sched* s = new (std::nothrow) dag_sched;
  if (!s) return DAG_ERR_WORKSPACE;
  try {  // (no exception may cross the C boundary: running out of host memory is reported as an error)
  s->n = n_nodes;
  s->words = std::max(1, (n_nodes + 63) / 64);
  s->page_size = page_size;
  s->parent_off.assign(parent_off, parent_off + (n_nodes > 0 ? n_nodes + 1 : 0));
  if (n_nodes > 0) s->parents.assign(parents, parents + parent_off[n_nodes]);
  s->len.assign(node_len, node_len + n_nodes);
  s->chunk.assign(n_nodes, 1);
  if (chunk) s->chunk.assign(chunk, chunk + n_nodes);
  s->anc.assign((size_t)n_nodes * s->words, 0);
  for (int v = 0; v < n_nodes; ++v)
    for (int e = parent_off[v]; e < parent_off[v + 1]; ++e) {
      const int p = parents[e];
      for (int w = 0; w < s->words; ++w) s->anc[(size_t)v * s->words + w] |= s->anc[(size_t)p * s->words + w];
      s->anc[(size_t)v * s->words + (p >> 6)] |= 1ull << (p & 63);
    }
  s->free_pages.resize(n_pages);
  for (int i = 0; i < n_pages; ++i) s->free_pages[i] = n_pages - 1 - i;  // handed out in ascending order
  s->pages.resize(n_nodes);
  s->done.assign(n_nodes, 0);
  // adaptive positions (section 4.2): one past the largest position of any predecessor, 0 without
  // one; the parents suffice because positions grow along every edge.  They depend on the plan
  // only, so they are fixed (and checked against the int32 range) here, not while stepping.
  s->pos_start.assign(n_nodes, 0);
  for (int v = 0; v < n_nodes; ++v) {
    int64_t start = 0;
    for (int e = parent_off[v]; e < parent_off[v + 1]; ++e)
      start = std::max<int64_t>(start, (int64_t)s->pos_start[parents[e]] + node_len[parents[e]]);
    if (start + node_len[v] > INT32_MAX) {
      delete s;
      return DAG_ERR_POS_OVERFLOW;
    }
    s->pos_start[v] = (int32_t)start;
  }
  s->marked.assign(n_nodes, 0);
  s->seg_of_node.assign(n_nodes, -1);
  } catch (...) {
    delete s;
    return DAG_ERR_WORKSPACE;
  }
  *out = s;
  return DAG_OK;
}

extern "C" void dag_sched_destroy(dag_sched_t* s) { delete s; }

static int sched_step(dag_sched_t* s, dag_sched_step_t* out);

extern "C" int dag_sched_step(dag_sched_t* s, dag_sched_step_t* out) {
  if (!s || !out) return DAG_ERR_NULL;
  try {
    return sched_step(s, out);
  } catch (...) {  // host memory exhausted while growing the step's arrays
    return DAG_ERR_WORKSPACE;
  }
}

static int sched_step(dag_sched_t* s, dag_sched_step_t* out) {
  // advance the marking when the whole frontier is complete, then recompute the frontier (Eq. 1)
  bool complete = true;
  for (int v : s->frontier) complete = complete && s->done[v] >= s->len[v];
  if (complete) {
    for (int v : s->frontier) s->marked[v] = 1;
    s->frontier.clear();
    for (int v = 0; v < s->n; ++v) {
      if (s->marked[v]) continue;  // output place already holds a token
      bool enabled = true;
      for (int e = s->parent_off[v]; e < s->parent_off[v + 1]; ++e) enabled = enabled && s->marked[s->parents[e]];
      if (enabled) s->frontier.push_back(v);
    }
    if (!s->frontier.empty()) s->layer++;
  }

  s->live_node.clear(); s->live_token.clear();
  s->b_page_off.assign(1, 0); s->b_pages.clear(); s->b_len.clear(); s->b_pos.clear();
  s->seg_node.clear(); s->seg_page_off.assign(1, 0); s->seg_pages.clear(); s->seg_len.clear();
  s->seg_reader_off.assign(1, 0); s->seg_readers.clear(); s->seg_reader_len.clear();
  s->entry_off.assign(1, 0); s->entries.clear();

  // the step's new tokens: pages first (all or nothing), then the bookkeeping
  int64_t need = 0;
  for (int v : s->frontier) {
    const int n_new = std::min(s->chunk[v], s->len[v] - s->done[v]);
    if (n_new > 0) need += (s->done[v] + n_new + s->page_size - 1) / s->page_size - (int64_t)s->pages[v].size();
  }
  if (need > (int64_t)s->free_pages.size()) return DAG_ERR_WORKSPACE;  // page pool exhausted; nothing changed
  std::vector<int32_t> live_nodes;
  for (int v : s->frontier) {
    const int n_new = std::min(s->chunk[v], s->len[v] - s->done[v]);
    if (n_new <= 0) continue;
    while ((int64_t)s->pages[v].size() * s->page_size < s->done[v] + n_new) {
      s->pages[v].push_back(s->free_pages.back());
      s->free_pages.pop_back();
    }
    live_nodes.push_back(v);
    for (int i = 0; i < n_new; ++i) {
      s->live_node.push_back(v);
      s->live_token.push_back(s->done[v] + i);
      // (the append kernel takes one page list per entry: the node's list, once per new token)
      s->b_pages.insert(s->b_pages.end(), s->pages[v].begin(), s->pages[v].end());
      s->b_page_off.push_back((int32_t)s->b_pages.size());
      s->b_len.push_back(s->done[v] + i + 1);
      s->b_pos.push_back(s->pos_start[v] + s->done[v] + i);
    }
    s->done[v] += n_new;
  }
  const int n_live = (int)s->live_node.size();

  // segments: every node some live transition reads (its ancestors and itself), in node order
  for (int v : live_nodes) {
    s->seg_of_node[v] = 0;
    for (int u = 0; u < v; ++u)
      if (s->is_anc(v, u)) s->seg_of_node[u] = 0;
  }
  for (int u = 0; u < s->n; ++u)
    if (s->seg_of_node[u] == 0) {
      s->seg_of_node[u] = (int32_t)s->seg_node.size();
      s->seg_node.push_back(u);
    }
  s->entries_of.assign(n_live, std::vector<int32_t>());
  int max_seg_pages = 0, max_readers = 0;
  for (size_t si = 0; si < s->seg_node.size(); ++si) {
    const int u = s->seg_node[si];
    s->seg_pages.insert(s->seg_pages.end(), s->pages[u].begin(), s->pages[u].end());
    s->seg_page_off.push_back((int32_t)s->seg_pages.size());
    s->seg_len.push_back(s->done[u]);
    max_seg_pages = std::max(max_seg_pages, (int)s->pages[u].size());
    for (int r = 0; r < n_live; ++r) {
      const int v = s->live_node[r];
      if (v != u && !s->is_anc(v, u)) continue;
      s->entries_of[r].push_back((int32_t)s->seg_readers.size());
      s->seg_readers.push_back(r);
      // a new token sees its own node up to itself, every other segment in full
      s->seg_reader_len.push_back(v == u ? s->live_token[r] + 1 : s->done[u]);
    }
    s->seg_reader_off.push_back((int32_t)s->seg_readers.size());
    max_readers = std::max(max_readers, s->seg_reader_off[si + 1] - s->seg_reader_off[si]);
  }
  for (int r = 0; r < n_live; ++r) {
    s->entries.insert(s->entries.end(), s->entries_of[r].begin(), s->entries_of[r].end());
    s->entry_off.push_back((int32_t)s->entries.size());
  }
  for (int u : s->seg_node) s->seg_of_node[u] = -1;
  if (n_live > 0) s->steps++;

  out->n_live = n_live;
  out->layer = s->layer;
  out->n_segments = (int32_t)s->seg_node.size();
  out->max_seg_pages = max_seg_pages;
  out->max_readers = max_readers;
  out->total_readers = (int32_t)s->seg_readers.size();
  out->pages_in_use = (int32_t)0;
  for (int v = 0; v < s->n; ++v) out->pages_in_use += (int32_t)s->pages[v].size();
  out->live_node = s->live_node.data();
  out->live_token = s->live_token.data();
  out->branch_page_off = s->b_page_off.data();
  out->branch_pages = s->b_pages.data();
  out->branch_len = s->b_len.data();
  out->branch_pos = s->b_pos.data();
  out->seg_node = s->seg_node.data();
  out->seg_page_off = s->seg_page_off.data();
  out->seg_pages = s->seg_pages.data();
  out->seg_len = s->seg_len.data();
  out->seg_reader_off = s->seg_reader_off.data();
  out->seg_readers = s->seg_readers.data();
  out->seg_reader_len = s->seg_reader_len.data();
  out->branch_entry_off = s->entry_off.data();
  out->branch_entries = s->entries.data();
  out->n_branch_pages = (int32_t)s->b_pages.size();
  out->n_seg_pages = (int32_t)s->seg_pages.size();
  return DAG_OK;
}
