// Host side of the library: block pool, prefixes, streams, batch descriptors, and the
// C ABI declared in include/oxy.h.  The paper's manager (Sec. 3.2; App. A.2) stores one
// resumable state per request; here the KV part of that state is a reference to a
// refcounted prefix plus an own block table and length, so that Batch (Alg. 1) is a
// descriptor build and UnBatch is a no-op.
#include "../../include/oxy.h"
#include "oxy_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int32_t hip_fail(hipError_t e, const char* what) {
  return fail(OXY_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Prefix {
  std::vector<int32_t> blocks;
  int32_t len = 0;
  bool sealed = false;
  bool handle = true;  // creator's reference still held
  int32_t n_streams = 0;
  int32_t frozen = 0;  // tokens below this position are shared with a fork: read-only
};

struct Stream {
  int32_t prefix_id = -1;
  int32_t kind = 0;
  std::vector<int32_t> blocks;
  int32_t len = 0;
  uint64_t stamp = 0;  // last batch build that listed this stream
};

// One descriptor slot in the caller's workspace plus its staging buffer.
struct DescSlot {
  bool in_use = false;
  int32_t* staging = nullptr;   // pinned (or malloc in host-only mode), desc_words ints
  hipEvent_t uploaded = nullptr;
  bool event_pending = false;
  char* d_base = nullptr;       // device: descriptor, then partial accumulators, then (m,l)
};

// Everything a recorded step depends on: two steps with equal keys issue identical launches.
struct StepKey {
  const void* d_base = nullptr;
  const void *k_new = nullptr, *v_new = nullptr, *q = nullptr, *out = nullptr, *lse = nullptr;
  size_t kv_stride = 0, q_stride = 0, lse_stride = 0;
  float scale = 0.f;
  int32_t layer_begin = 0, layer_end = 0, mode = 0;   // mode: 0 separate, 1 fused, 2 folded
  int32_t n_work = 0, n_tokens = 0, n_fresh = 0, off_work = 0, off_tables = 0, off_part_off = 0,
          off_n_parts = 0;
  bool operator==(const StepKey& o) const {
    return d_base == o.d_base && k_new == o.k_new && v_new == o.v_new && q == o.q &&
           out == o.out && lse == o.lse && kv_stride == o.kv_stride && q_stride == o.q_stride &&
           lse_stride == o.lse_stride && scale == o.scale && layer_begin == o.layer_begin &&
           layer_end == o.layer_end && mode == o.mode && n_work == o.n_work &&
           n_tokens == o.n_tokens && n_fresh == o.n_fresh && off_work == o.off_work && off_tables == o.off_tables &&
           off_part_off == o.off_part_off && off_n_parts == o.off_n_parts;
  }
  // same number and kinds of launches in the same order: an instantiated graph can be updated
  // in place from a recording of the other
  bool same_topology(const StepKey& o) const {
    return layer_end - layer_begin == o.layer_end - o.layer_begin && mode == o.mode &&
           (n_tokens > 0) == (o.n_tokens > 0) && (n_fresh > 0) == (o.n_fresh > 0);
  }
};
struct StepGraph {
  StepKey key;
  hipGraphExec_t exec = nullptr;
  uint64_t last_use = 0;
};
constexpr size_t kMaxStepGraphs = 8;

}  // namespace

struct oxy_pool {
  oxy_pool_config cfg;
  bool host_only = false;
  std::vector<int32_t> free_stack;  // top = back
  std::vector<int32_t> ref;
  std::unordered_map<int32_t, Prefix> prefixes;
  std::unordered_map<int32_t, Stream> streams;
  int32_t next_prefix = 0;
  int32_t next_stream = 0;
  size_t desc_words = 0;
  size_t per_batch_bytes = 0;
  size_t acc_offset = 0, ml_offset = 0;
  std::vector<DescSlot> slots;
  int32_t live_batches = 0;
  uint64_t build_seq = 0;
  // recorded launch sequences of oxy_step_layers (OXY_STEP_GRAPH)
  std::vector<StepGraph> graphs;
  hipStream_t record_stream = nullptr;   // launches are recorded here, never executed here
  uint64_t graph_clock = 0;
  int32_t graph_instantiations = 0, graph_updates = 0, graph_replays = 0;
};

struct oxy_batch {
  oxy_pool* pool = nullptr;
  int32_t slot = -1;
  int32_t flags = 0;
  int32_t n_items = 0, n_tokens = 0, n_work = 0, n_partials = 0;
  int32_t n_launch = 0;   // n_work rounded up to a multiple of 64 with padding records: the grid
  int32_t n_fresh = 0;    // tokens of items whose own-phase tiles read k_new / v_new (folded append)
  int32_t off_fresh = 0;
  bool append_foldable = false;   // every item has <= 2 new tokens or an empty own history
  // word offsets inside the descriptor
  int32_t off_slots = 0, off_work = 0, off_toks = 0, off_tables = 0, off_part_off = 0,
          off_n_parts = 0;
  std::vector<int32_t> host;  // full descriptor image (kept for introspection)
};

namespace {

using oxy::kPage;

int32_t blocks_for(int32_t n_tokens) { return (n_tokens + kPage - 1) / kPage; }

bool resolve_config(const oxy_pool_config* in, oxy_pool_config* c) {
  if (!in) return false;
  *c = *in;
  if (c->n_layers < 1 || c->n_q_heads != oxy::kHeads || c->n_kv_heads != 1 ||
      c->head_dim != oxy::kDim || c->page_size != kPage || c->num_blocks < 1 ||
      c->num_blocks > (1 << 26))
    return false;
  if (c->max_live_batches == 0) c->max_live_batches = 2;
  if (c->max_q_tokens == 0) c->max_q_tokens = 1024;
  if (c->max_append_tokens == 0) c->max_append_tokens = kPage * c->num_blocks;
  if (c->max_work_items == 0) c->max_work_items = 16384;
  if (c->max_partials == 0) c->max_partials = 32 * c->max_q_tokens;
  // split_tokens == 0 stays 0: the tile path then sizes its splits from the length of the KV
  // source alone (see tile_split_for), which keeps an item's arithmetic independent of its batch
  // stream_split_tokens == 0 becomes split_tokens; both 0: by the item's length (stream_split_for)
  if (c->stream_split_tokens == 0) c->stream_split_tokens = c->split_tokens;
  // query token ids travel in 23 bits of a work-record word (kPathRowShift)
  if (c->max_q_tokens > (1 << 20) || c->max_append_tokens > (1 << 26)) return false;
  if (c->max_live_batches < 1 || c->max_live_batches > 64 || c->max_q_tokens < 1 ||
      c->max_append_tokens < 1 || c->max_work_items < 1 || c->max_partials < 1 ||
      (c->split_tokens != 0 && (c->split_tokens < 32 || c->split_tokens % 32 != 0)) ||
      c->split_tokens > 1024 ||
      (c->stream_split_tokens != 0 &&
       (c->stream_split_tokens < 32 || c->stream_split_tokens % 32 != 0)) ||
      c->stream_split_tokens > 1024)
    return false;
  return true;
}

// Capacity of a batch's flat block tables.  Every block sits in one table, except blocks
// shared by forked prefixes, which every such prefix lists: twice the pool covers one fork
// level of everything.
size_t table_words_of(const oxy_pool_config& c) { return 2 * (size_t)c.num_blocks; }

size_t desc_words_of(const oxy_pool_config& c) {
  return (size_t)c.max_append_tokens + (size_t)oxy::kWorkWords * c.max_work_items +
         2 * (size_t)c.max_q_tokens /* token lists */ + table_words_of(c) /* tables */ +
         3 * (size_t)c.max_q_tokens /* part_off, n_parts, fresh tokens */;
}

void layout_of(const oxy_pool_config& c, size_t* acc_off, size_t* ml_off, size_t* total) {
  size_t desc = align_up(desc_words_of(c) * 4, 256);
  size_t acc = align_up((size_t)c.max_partials * oxy::kHeads * oxy::kDim * sizeof(uint16_t), 256);
  size_t ml = align_up((size_t)c.max_partials * oxy::kHeads * 4 * sizeof(float), 256);
  *acc_off = desc;
  *ml_off = desc + acc;
  *total = desc + acc + ml;
}

void unref_table(oxy_pool* p, const std::vector<int32_t>& table) {
  for (int32_t b : table) {
    if (--p->ref[b] == 0) p->free_stack.push_back(b);
  }
}

void maybe_drop_prefix(oxy_pool* p, int32_t pid) {
  auto it = p->prefixes.find(pid);
  if (it != p->prefixes.end() && !it->second.handle && it->second.n_streams == 0)
    p->prefixes.erase(it);
}

// Split size of the shared-tile path for a KV source of `len` tokens.  With a configured
// split_tokens it is that; otherwise about an eighth of the source, between 64 and 256 tokens:
// short sources (an 832-token prefix, a 50-token chunk) get short dependent chains per
// workgroup, long ones (2048 tokens) keep the number of partials per query down.
int32_t tile_split_for(const oxy_pool_config& c, int32_t len) {
  if (c.split_tokens) return c.split_tokens;
  int32_t s = ((len + 7) / 8 + 31) / 32 * 32;
  return std::max(64, std::min(256, s));
}

// Streaming path on an item's own history.  A history of at most 512 tokens is cut into
// 128-token work items (one step per wavefront: steps that wait for memory one after the other
// are what such a launch is made of), a longer one into 256-token work items (two steps per
// wavefront; halves the work items and split results of a launch that is bound by bytes).
int32_t stream_split_for(const oxy_pool_config& c, int32_t len) {
  if (c.stream_split_tokens) return c.stream_split_tokens;
  return len <= 512 ? 128 : 256;
}

char* layer_base(const oxy_pool* p, int32_t layer) {
  return (char*)p->cfg.kv_base + (size_t)layer * p->cfg.num_blocks * oxy::kBlockBytes;
}

}  // namespace

extern "C" {

const char* oxy_last_error(void) { return g_err; }
__attribute__((visibility("hidden"))) void oxy_internal_set_error(const char* msg) { snprintf(g_err, sizeof(g_err), "%s", msg); }
int32_t oxy_version(void) { return 1; }

size_t oxy_kv_bytes(const oxy_pool_config* cfg) {
  oxy_pool_config c;
  if (!resolve_config(cfg, &c)) return 0;
  return (size_t)c.n_layers * c.num_blocks * oxy::kBlockBytes;
}

size_t oxy_workspace_bytes(const oxy_pool_config* cfg) {
  oxy_pool_config c;
  if (!resolve_config(cfg, &c)) return 0;
  size_t a, m, total;
  layout_of(c, &a, &m, &total);
  return total * c.max_live_batches;
}

int32_t oxy_pool_create(const oxy_pool_config* cfg, oxy_pool** out) {
  if (!out) return fail(OXY_ERR_INVALID_ARG, "pool_create: out is null");
  *out = nullptr;
  oxy_pool_config c;
  if (!resolve_config(cfg, &c))
    return fail(OXY_ERR_INVALID_ARG,
                "pool_create: unsupported geometry or sizes (need 8 q heads, 1 kv head, "
                "head_dim 256, page 16, split_tokens a multiple of 32)");
  const bool host_only = (c.flags & OXY_POOL_HOST_ONLY) != 0;
  if (!host_only) {
    if (!c.kv_base || c.kv_bytes < oxy_kv_bytes(cfg) || ((uintptr_t)c.kv_base & 255))
      return fail(OXY_ERR_INVALID_ARG, "pool_create: kv buffer missing, misaligned or < %zu bytes",
                  oxy_kv_bytes(cfg));
    if (!c.workspace || c.workspace_bytes < oxy_workspace_bytes(cfg) ||
        ((uintptr_t)c.workspace & 255))
      return fail(OXY_ERR_INVALID_ARG,
                  "pool_create: workspace missing, misaligned or < %zu bytes",
                  oxy_workspace_bytes(cfg));
  }
  std::vector<int32_t> order(c.num_blocks);
  if (c.free_order) {
    std::vector<char> seen(c.num_blocks, 0);
    for (int32_t i = 0; i < c.num_blocks; ++i) {
      int32_t b = c.free_order[i];
      if (b < 0 || b >= c.num_blocks || seen[b])
        return fail(OXY_ERR_INVALID_ARG, "pool_create: free_order is not a permutation");
      seen[b] = 1;
      order[i] = b;
    }
  } else {
    for (int32_t i = 0; i < c.num_blocks; ++i) order[i] = i;
  }
  oxy_pool* p = new (std::nothrow) oxy_pool();
  if (!p) return fail(OXY_ERR_INVALID_ARG, "pool_create: out of host memory");
  p->cfg = c;
  p->cfg.free_order = nullptr;
  p->host_only = host_only;
  p->free_stack.assign(order.rbegin(), order.rend());  // first element of free_order on top
  p->ref.assign(c.num_blocks, 0);
  p->desc_words = desc_words_of(c);
  layout_of(c, &p->acc_offset, &p->ml_offset, &p->per_batch_bytes);
  p->slots.resize(c.max_live_batches);
  for (int32_t i = 0; i < c.max_live_batches; ++i) {
    DescSlot& s = p->slots[i];
    if (host_only) {
      s.staging = (int32_t*)malloc(p->desc_words * 4);
      if (!s.staging) {
        oxy_pool_destroy(p);
        return fail(OXY_ERR_INVALID_ARG, "pool_create: out of host memory");
      }
    } else {
      hipError_t e = hipHostMalloc((void**)&s.staging, p->desc_words * 4, hipHostMallocDefault);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&s.uploaded, hipEventDisableTiming);
      if (e != hipSuccess) {
        oxy_pool_destroy(p);
        return hip_fail(e, "pool_create: pinned staging");
      }
      s.d_base = (char*)c.workspace + (size_t)i * p->per_batch_bytes;
    }
  }
  if (!host_only) {   // set-up of oxy_mixed_attention_static for this device, so that the call
                      // itself never has to ask the runtime for the address
    uint16_t* acc;
    float* ml;
    hipError_t e = oxy::static_scratch(&acc, &ml);
    if (e != hipSuccess) {
      oxy_pool_destroy(p);
      return hip_fail(e, "pool_create: static split-result buffer");
    }
  }
  *out = p;
  return OXY_OK;
}

int32_t oxy_pool_destroy(oxy_pool* p) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "pool_destroy: null");
  if (p->live_batches > 0) return fail(OXY_ERR_BUSY, "pool_destroy: %d batches alive", p->live_batches);
  for (DescSlot& s : p->slots) {
    if (p->host_only) {
      free(s.staging);
    } else {
      if (s.uploaded) {
        if (s.event_pending) (void)hipEventSynchronize(s.uploaded);
        (void)hipEventDestroy(s.uploaded);
      }
      if (s.staging) (void)hipHostFree(s.staging);
    }
  }
  for (StepGraph& g : p->graphs)
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (p->record_stream) (void)hipStreamDestroy(p->record_stream);
  delete p;
  return OXY_OK;
}

// ---- prefixes -------------------------------------------------------------------------
int32_t oxy_prefix_create(oxy_pool* p, int32_t* prefix_id) {
  if (!p || !prefix_id) return fail(OXY_ERR_INVALID_ARG, "prefix_create: null argument");
  int32_t id = p->next_prefix++;
  p->prefixes.emplace(id, Prefix());
  *prefix_id = id;
  return OXY_OK;
}

namespace {
// Appends tokens [pos0, pos0+n) of layers [layer_begin, layer_end): blocks are allocated on first
// touch, then one launch per 512 blocks covers all the layers.
int32_t prefix_append_impl(oxy_pool* p, int32_t pid, int32_t layer_begin, int32_t layer_end,
                           const void* k, const void* v, size_t src_layer_stride, int32_t n_tokens,
                           int32_t pos0, void* hip_stream, const char* who) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "%s: null pool", who);
  auto it = p->prefixes.find(pid);
  if (it == p->prefixes.end() || !it->second.handle)
    return fail(OXY_ERR_BAD_ID, "%s: no prefix %d", who, pid);
  Prefix& px = it->second;
  if (layer_begin < 0 || layer_end > p->cfg.n_layers || layer_begin >= layer_end || n_tokens < 1 ||
      pos0 < 0 || pos0 > px.len || (int64_t)pos0 + n_tokens > (int64_t)kPage * p->cfg.num_blocks)
    return fail(OXY_ERR_INVALID_ARG, "%s: layers [%d, %d), n %d, pos0 %d (len %d)", who, layer_begin,
                layer_end, n_tokens, pos0, px.len);
  if (!p->host_only && (!k || !v)) return fail(OXY_ERR_INVALID_ARG, "%s: null k/v", who);
  if (px.sealed) return fail(OXY_ERR_SEALED, "%s: prefix %d has streams attached", who, pid);
  if (pos0 < px.frozen)
    return fail(OXY_ERR_SEALED, "%s: tokens below %d of prefix %d are shared with a fork", who,
                px.frozen, pid);
  int32_t need = blocks_for(pos0 + n_tokens) - (int32_t)px.blocks.size();
  if (need > (int32_t)p->free_stack.size())
    return fail(OXY_ERR_NO_BLOCKS, "%s: need %d blocks, %zu free", who, need, p->free_stack.size());
  const size_t old_blocks = px.blocks.size();
  const int32_t old_len = px.len;
  for (int32_t i = 0; i < need; ++i) {
    int32_t b = p->free_stack.back();
    p->free_stack.pop_back();
    p->ref[b] = 1;
    px.blocks.push_back(b);
  }
  px.len = std::max(px.len, pos0 + n_tokens);
  if (p->host_only) return OXY_OK;
  // a launch that fails leaves the pool as it was: the blocks go back in reverse order of
  // their pops, which restores the free stack exactly
  auto roll_back = [&]() {
    while (px.blocks.size() > old_blocks) {
      p->ref[px.blocks.back()] = 0;
      p->free_stack.push_back(px.blocks.back());
      px.blocks.pop_back();
    }
    px.len = old_len;
  };
  // device copy, at most kMaxInlineBlocks blocks per launch (block ids travel by value)
  const char* kp = (const char*)k;
  const char* vp = (const char*)v;
  const size_t pool_layer_stride = (size_t)p->cfg.num_blocks * oxy::kBlockBytes;
  int32_t done = 0;
  while (done < n_tokens) {
    int32_t pos = pos0 + done;
    int32_t first_block = pos / kPage;
    int32_t max_tok = (first_block + oxy::kMaxInlineBlocks) * kPage - pos;
    int32_t n = std::min(n_tokens - done, max_tok);
    oxy::InlineIds ids;
    int32_t nb = blocks_for(pos + n) - first_block;
    for (int32_t i = 0; i < nb; ++i) ids.v[i] = px.blocks[first_block + i];
    hipError_t e = oxy::launch_append_inline(
        kp + (size_t)done * oxy::kDim * 2, vp + (size_t)done * oxy::kDim * 2, ids,
        pos - first_block * kPage, n, layer_base(p, layer_begin), layer_end - layer_begin,
        src_layer_stride, pool_layer_stride, (hipStream_t)hip_stream);
    if (e != hipSuccess) {
      roll_back();
      return hip_fail(e, "prefix_append: launch");
    }
    done += n;
  }
  return OXY_OK;
}
}  // namespace

int32_t oxy_prefix_append(oxy_pool* p, int32_t pid, int32_t layer, const void* k, const void* v,
                          int32_t n_tokens, int32_t pos0, void* hip_stream) {
  return prefix_append_impl(p, pid, layer, layer + 1, k, v, 0, n_tokens, pos0, hip_stream,
                            "prefix_append");
}

int32_t oxy_prefix_append_layers(oxy_pool* p, int32_t pid, int32_t layer_begin, int32_t layer_end,
                                 const void* k, const void* v, size_t layer_stride, int32_t n_tokens,
                                 int32_t pos0, void* hip_stream) {
  return prefix_append_impl(p, pid, layer_begin, layer_end, k, v, layer_stride, n_tokens, pos0,
                            hip_stream, "prefix_append_layers");
}

int32_t oxy_prefix_fork(oxy_pool* p, int32_t parent_id, int32_t n_tokens, int32_t* prefix_id) {
  if (!p || !prefix_id) return fail(OXY_ERR_INVALID_ARG, "prefix_fork: null argument");
  auto it = p->prefixes.find(parent_id);
  if (it == p->prefixes.end()) return fail(OXY_ERR_BAD_ID, "prefix_fork: no prefix %d", parent_id);
  if (n_tokens < 0 || n_tokens % kPage != 0 || n_tokens > it->second.len)
    return fail(OXY_ERR_INVALID_ARG, "prefix_fork: %d tokens of prefix %d (len %d, page %d)", n_tokens,
                parent_id, it->second.len, kPage);
  Prefix child;
  child.blocks.assign(it->second.blocks.begin(), it->second.blocks.begin() + n_tokens / kPage);
  child.len = child.frozen = n_tokens;
  it->second.frozen = std::max(it->second.frozen, n_tokens);
  for (int32_t b : child.blocks) p->ref[b]++;
  int32_t id = p->next_prefix++;
  p->prefixes.emplace(id, std::move(child));   // may rehash: `it` is not used after this
  *prefix_id = id;
  return OXY_OK;
}

int32_t oxy_prefix_release(oxy_pool* p, int32_t pid) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "prefix_release: null pool");
  auto it = p->prefixes.find(pid);
  if (it == p->prefixes.end() || !it->second.handle)
    return fail(OXY_ERR_BAD_ID, "prefix_release: no prefix %d", pid);
  it->second.handle = false;
  unref_table(p, it->second.blocks);
  maybe_drop_prefix(p, pid);
  return OXY_OK;
}

// ---- streams --------------------------------------------------------------------------
int32_t oxy_stream_create(oxy_pool* p, int32_t pid, int32_t kind, int32_t* stream_id) {
  if (!p || !stream_id) return fail(OXY_ERR_INVALID_ARG, "stream_create: null argument");
  if (kind != OXY_KIND_ACTION && kind != OXY_KIND_DECODE)
    return fail(OXY_ERR_INVALID_ARG, "stream_create: kind %d", kind);
  if (pid != -1) {
    auto it = p->prefixes.find(pid);
    if (it == p->prefixes.end() || !it->second.handle)
      return fail(OXY_ERR_BAD_ID, "stream_create: no prefix %d", pid);
    Prefix& px = it->second;
    px.sealed = true;
    px.n_streams++;
    for (int32_t b : px.blocks) p->ref[b]++;
  }
  int32_t id = p->next_stream++;
  Stream s;
  s.prefix_id = pid;
  s.kind = kind;
  p->streams.emplace(id, std::move(s));
  *stream_id = id;
  return OXY_OK;
}

int32_t oxy_stream_release(oxy_pool* p, int32_t sid) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "stream_release: null pool");
  auto it = p->streams.find(sid);
  if (it == p->streams.end()) return fail(OXY_ERR_BAD_ID, "stream_release: no stream %d", sid);
  Stream s = std::move(it->second);
  p->streams.erase(it);
  unref_table(p, s.blocks);
  if (s.prefix_id != -1) {
    Prefix& px = p->prefixes.at(s.prefix_id);
    unref_table(p, px.blocks);
    px.n_streams--;
    maybe_drop_prefix(p, s.prefix_id);
  }
  return OXY_OK;
}

int32_t oxy_stream_rewind(oxy_pool* p, int32_t sid, int32_t new_len) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "stream_rewind: null pool");
  auto it = p->streams.find(sid);
  if (it == p->streams.end()) return fail(OXY_ERR_BAD_ID, "stream_rewind: no stream %d", sid);
  if (new_len < 0 || new_len > it->second.len)
    return fail(OXY_ERR_INVALID_ARG, "stream_rewind: %d not in [0, %d]", new_len, it->second.len);
  it->second.len = new_len;
  return OXY_OK;
}

// ---- batch ------------------------------------------------------------------------------
int32_t oxy_batch_build(oxy_pool* p, const oxy_item* items, int32_t n_items, int32_t flags,
                        void* hip_stream, oxy_batch** out) {
  if (!p || !items || !out || n_items < 1)
    return fail(OXY_ERR_INVALID_ARG, "batch_build: null argument or no items");
  *out = nullptr;
  const bool append_only = (flags & OXY_BATCH_APPEND_ONLY) != 0;
  if (flags & ~OXY_BATCH_APPEND_ONLY) return fail(OXY_ERR_INVALID_ARG, "batch_build: flags");
  const oxy_pool_config& c = p->cfg;

  // ---- validate everything before touching state
  struct Plan {
    Stream* s;
    int32_t old_len, new_len, need, tok0;
    int32_t len_before;   // the stream's length when the call began (an ACTION item is rewound)
  };
  std::vector<Plan> plan;
  plan.reserve(n_items);
  const uint64_t stamp = ++p->build_seq;   // marks the streams of this build (duplicate check)
  int64_t need_total = 0, n_tokens = 0;
  for (int32_t i = 0; i < n_items; ++i) {
    auto it = p->streams.find(items[i].stream_id);
    if (it == p->streams.end())
      return fail(OXY_ERR_BAD_ID, "batch_build: no stream %d", items[i].stream_id);
    Stream& s = it->second;
    if (items[i].n_new < 1 || s.stamp == stamp)
      return fail(OXY_ERR_INVALID_ARG, "batch_build: item %d: n_new %d or duplicate stream", i,
                  items[i].n_new);
    s.stamp = stamp;
    int32_t old_len = s.kind == OXY_KIND_ACTION ? 0 : s.len;
    int64_t new_len = (int64_t)old_len + items[i].n_new;
    if (new_len > (int64_t)kPage * c.num_blocks)
      return fail(OXY_ERR_NO_BLOCKS, "batch_build: stream %d would exceed the pool", items[i].stream_id);
    int32_t need = std::max(0, blocks_for((int32_t)new_len) - (int32_t)s.blocks.size());
    plan.push_back({&s, old_len, (int32_t)new_len, need, (int32_t)n_tokens, s.len});
    need_total += need;
    n_tokens += items[i].n_new;
  }
  if (need_total > (int64_t)p->free_stack.size())
    return fail(OXY_ERR_NO_BLOCKS, "batch_build: need %lld blocks, %zu free", (long long)need_total,
                p->free_stack.size());
  if (n_tokens > c.max_append_tokens)
    return fail(OXY_ERR_WORKSPACE, "batch_build: %lld new tokens > max_append_tokens %d",
                (long long)n_tokens, c.max_append_tokens);
  if (!append_only && n_tokens > c.max_q_tokens)
    return fail(OXY_ERR_WORKSPACE, "batch_build: %lld query tokens > max_q_tokens %d",
                (long long)n_tokens, c.max_q_tokens);

  // ---- work list on the lengths the step will have (state still untouched).  Records are
  // kept as their eight header words until the order is known.
  constexpr int kHdr = 8;
  std::vector<int32_t> hdr, toks, n_parts(append_only ? 0 : n_tokens, 0);
  std::vector<int32_t> fresh_toks;   // tokens whose rows the merge launch writes under a folded append
  struct TableRef {
    int32_t off;
    const std::vector<int32_t>* src;
    int32_t count;
  };
  std::vector<TableRef> table_refs;
  std::vector<int32_t> order;   // final order of the records; -1 = padding record
  int32_t tbl_words = 0;
  bool foldable = !append_only;
  if (!append_only) {
    hdr.reserve(1024 * kHdr);
    toks.reserve(2 * n_tokens);
    table_refs.reserve(n_items + 8);
    auto add_work = [&](int32_t tok_off, int32_t n_tok, int32_t tbl_off, int32_t b, int32_t e,
                        int32_t q0, int32_t part, int32_t path) {
      const int32_t w[kHdr] = {tok_off, n_tok, tbl_off, b, e, q0, part, path};
      hdr.insert(hdr.end(), w, w + kHdr);
    };
    // Which path evaluates a query depends on its item and its prefix only (kind, n_new, phase,
    // prefix length), never on its batch mates, so an item's arithmetic is the same in every
    // batch it can appear in:
    //   prefix phase, prefix longer than kStreamPrefixMax -> all queries attached to the prefix
    //                   share tiles of 8 tokens (64 MFMA rows), which fetch the prefix pages once
    //                   for all of them;
    //   prefix phase, shorter prefix -> streaming path: a decode item (<= 2 new tokens) on its
    //                   own, the other queries (an action chunk) two tokens at a time.  With a
    //                   short prefix the launch is bound by latency, CUs are idle, and the
    //                   re-reads hit L2; four steps in flight per workgroup beat a tile's two;
    //   own phase    -> items with <= 2 new tokens (decode) stream their own pages; larger
    //                   items (action chunks, multi-token decode) use tiles: 8 tokens on a long
    //                   KV source, 4 (two wavefronts compute, all four move pages) on one of at
    //                   most 1024 tokens, where few workgroups exist anyway and a step is
    //                   bound by the tile's own LDS reads and arithmetic.
    auto tile_tok_for = [](int32_t source_len) { return source_len <= 1024 ? 4 : 8; };
    constexpr int32_t kStreamPrefixMax = 1024;
    struct Group {
      int32_t pid;
      const Prefix* px;
      std::vector<int32_t> toks;
      std::vector<std::pair<int32_t, int32_t>> solo;   // (first token, count) of streaming items
    };
    std::vector<Group> groups;   // in order of first appearance; a batch touches few prefixes
    groups.reserve(16);
    for (const Plan& pl : plan) {
      const int32_t pid = pl.s->prefix_id;
      if (pid == -1) continue;
      Group* g = nullptr;
      for (Group& x : groups)
        if (x.pid == pid) {
          g = &x;
          break;
        }
      if (!g) {
        const Prefix& px = p->prefixes.at(pid);
        if (px.len == 0) continue;
        groups.push_back({pid, &px, {}, {}});
        g = &groups.back();
      }
      const int32_t n_new = pl.new_len - pl.old_len;
      if (n_new <= 2 && g->px->len <= kStreamPrefixMax)
        g->solo.push_back({pl.tok0, n_new});
      else
        for (int32_t t = 0; t < n_new; ++t) g->toks.push_back(pl.tok0 + t);
    }
    for (const Group& g : groups) {
      const Prefix& px = *g.px;
      const int32_t tbl_off = tbl_words;
      table_refs.push_back({tbl_off, &px.blocks, blocks_for(px.len)});
      tbl_words += blocks_for(px.len);
      const int32_t split = tile_split_for(c, px.len);
      const int32_t nsplit = (px.len + split - 1) / split;
      const bool pairs = px.len <= kStreamPrefixMax;   // short prefix: pairs on the streaming path
      const int32_t tile_tok = pairs ? 2 : tile_tok_for(px.len);
      for (size_t t0 = 0; t0 < g.toks.size(); t0 += tile_tok) {
        const int32_t n = (int32_t)std::min<size_t>(tile_tok, g.toks.size() - t0);
        const int32_t tok_off = (int32_t)toks.size();
        toks.insert(toks.end(), g.toks.begin() + t0, g.toks.begin() + t0 + n);
        for (int32_t s = 0; s < nsplit; ++s)
          add_work(tok_off, n, tbl_off, s * split, std::min(px.len, (s + 1) * split),
                   oxy::kNoCausal, s, pairs ? oxy::PATH_STREAM : oxy::PATH_TILE);
      }
      for (int32_t t : g.toks) n_parts[t] = nsplit;
      for (const auto& so : g.solo) {
        const int32_t tok_off = (int32_t)toks.size();
        for (int32_t t = 0; t < so.second; ++t) toks.push_back(so.first + t);
        for (int32_t s = 0; s < nsplit; ++s)
          add_work(tok_off, so.second, tbl_off, s * split, std::min(px.len, (s + 1) * split),
                   oxy::kNoCausal, s, oxy::PATH_STREAM);
        for (int32_t t = 0; t < so.second; ++t) n_parts[so.first + t] = nsplit;
      }
    }
    for (const Plan& pl : plan) {
      const int32_t tbl_off = tbl_words;
      table_refs.push_back({tbl_off, &pl.s->blocks, blocks_for(pl.new_len)});
      tbl_words += blocks_for(pl.new_len);
      const int32_t n_new = pl.new_len - pl.old_len;
      const bool causal = pl.s->kind == OXY_KIND_DECODE;
      int32_t path = n_new <= 2 ? (oxy::PATH_STREAM | oxy::kPathAppends) : oxy::PATH_TILE;
      if ((path & oxy::kPathMask) == oxy::PATH_TILE) {
        if (pl.old_len == 0) {
          path |= oxy::kPathFresh | (pl.tok0 << oxy::kPathRowShift);
          for (int32_t t = 0; t < n_new; ++t) fresh_toks.push_back(pl.tok0 + t);
        }
        else
          foldable = false;   // old and new keys in one tile: only the separate append covers it
      }
      // a short chunk on an empty history (see below): single 32-key steps, so all four
      // wavefronts of a tile get rows (8 tokens) -- half as many workgroups to place
      const bool short_chunk = n_new > 2 && pl.old_len == 0 && pl.new_len <= 64 && !c.split_tokens;
      const int32_t step_tok = n_new <= 2 ? 2 : (short_chunk ? 8 : tile_tok_for(pl.new_len));
      int32_t split = n_new <= 2 ? stream_split_for(c, pl.new_len) : tile_split_for(c, pl.new_len);
      // A short chunk on an empty history (an action chunk, Sec. 3.2) is cut into single 32-key
      // steps: its tiles start last (their keys are this step's new rows) and would otherwise
      // be the workgroups the launch ends with.  Depends on the item alone, like every split.
      if (short_chunk) split = 32;
      for (int32_t t0 = 0; t0 < n_new; t0 += step_tok) {
        const int32_t n = std::min(step_tok, n_new - t0);
        const int32_t tok_off = (int32_t)toks.size();
        for (int32_t t = 0; t < n; ++t) toks.push_back(pl.tok0 + t0 + t);
        const int32_t q0 = pl.old_len + t0;
        const int32_t kv_hi = causal ? q0 + n : pl.new_len;
        const int32_t nsplit = (kv_hi + split - 1) / split;
        const int32_t base = n_parts[pl.tok0 + t0];
        for (int32_t s = 0; s < nsplit; ++s)
          add_work(tok_off, n, tbl_off, s * split, std::min(kv_hi, (s + 1) * split),
                   causal ? q0 : oxy::kNoCausal, base + s, path);
        for (int32_t t = 0; t < n; ++t) n_parts[pl.tok0 + t0 + t] += nsplit;
      }
    }
    // Order of the work list.  Workgroup i runs on XCD i % 8 and every XCD has its own L2, so
    // tiles that read the same pages (same table, same split) are given indices of one residue
    // class; within a class the longest work comes first, and the classes are balanced by cost
    // (longest-processing-time rule over the groups).  Padding records keep the pattern intact.
    {
      const int32_t nw = (int32_t)(hdr.size() / kHdr);
      constexpr int kXcd = 8, kCuPerXcd = 32;
      struct Rec {
        int64_t key;     // readers of shared pages: (table, split begin); others: unique
        int32_t idx, cost;
        bool tile;
      };
      std::vector<Rec> recs(nw);
      for (int32_t i = 0; i < nw; ++i) {
        const int32_t* r = &hdr[(size_t)i * kHdr];
        const int32_t steps = (r[oxy::W_KV_END] - r[oxy::W_KV_BEGIN] + 31) / 32;
        const bool tile = (r[oxy::W_PATH] & oxy::kPathMask) == oxy::PATH_TILE;
        // work items that read pages others read too: tiles (not those that take their keys from
        // the step's new rows: they read no pages, and dealt out as one group they would sit two
        // to a CU on one XCD), and streaming items on prefix pages
        const bool fresh = (r[oxy::W_PATH] & oxy::kPathFresh) != 0;
        const bool shares = fresh ? false : (tile || !(r[oxy::W_PATH] & oxy::kPathAppends));
        recs[i].idx = i;
        recs[i].cost = tile ? 2 * steps : steps;
        recs[i].tile = tile && !fresh;
        recs[i].key = shares ? (((int64_t)r[oxy::W_TBL_OFF] << 32) | (uint32_t)r[oxy::W_KV_BEGIN])
                             : -(int64_t)i - 1;
      }
      std::stable_sort(recs.begin(), recs.end(),
                       [](const Rec& a, const Rec& b) { return a.key < b.key; });
      struct Grp {
        int32_t first, count;
        int64_t cost;
      };
      std::vector<Grp> grps;
      grps.reserve(nw);
      for (int32_t i = 0; i < nw;) {
        int32_t j = i;
        int64_t cst = 0;
        while (j < nw && recs[j].key == recs[i].key) cst += recs[j++].cost;
        // A tile that is the only reader of its pages fetches all of them from HBM itself (a
        // tile that shares its split finds most of them on their way into the L2 already) and
        // is the slowest kind of work item per step: it counts half as much again, which makes
        // the pairing below give it the smallest partner on its CU, or none.
        if (j - i == 1 && recs[i].tile) {
          recs[i].cost = recs[i].cost * 3 / 2;
          cst = recs[i].cost;
        }
        grps.push_back({i, j - i, cst});
        i = j;
      }
      std::stable_sort(grps.begin(), grps.end(), [&](const Grp& a, const Grp& b) {
        return a.cost != b.cost ? a.cost > b.cost : recs[a.first].idx < recs[b.first].idx;
      });
      std::vector<Rec> queue[kXcd];
      int64_t qcost[kXcd] = {0};
      for (int x = 0; x < kXcd; ++x) queue[x].reserve(nw / kXcd + 16);
      for (const Grp& g : grps) {
        // least loaded XCD among those that still have a resident slot for every record of the
        // group (two workgroups on each of 32 CUs); any XCD if none has
        int best = -1;
        for (int x = 0; x < kXcd; ++x)
          if (queue[x].size() + g.count <= (size_t)2 * kCuPerXcd && (best < 0 || qcost[x] < qcost[best]))
            best = x;
        if (best < 0) {
          best = 0;
          for (int x = 1; x < kXcd; ++x)
            if (qcost[x] < qcost[best]) best = x;
        }
        queue[best].insert(queue[best].end(), recs.begin() + g.first,
                           recs.begin() + g.first + g.count);
        qcost[best] += g.cost;
      }
      size_t longest = 0;
      for (int x = 0; x < kXcd; ++x) {
        std::stable_sort(queue[x].begin(), queue[x].end(), [](const Rec& a, const Rec& b) {
          return a.cost != b.cost ? a.cost > b.cost : a.idx < b.idx;
        });
        // Inside an XCD the dispatcher hands workgroups to the 32 CUs in turn, so while at most
        // two are resident per CU, positions j and j + 32 of a class share a CU, and a CU's
        // share of the memory system is what bounds its workgroups.  Pair the largest of the
        // first round with the smallest of the second; first-round items without a partner are
        // the largest ones.  Anything past 64 follows in descending order (it back-fills).
        std::vector<Rec>& q = queue[x];
        if (q.size() > (size_t)kCuPerXcd) {
          const size_t top = std::min(q.size(), (size_t)2 * kCuPerXcd), m = top - kCuPerXcd;
          const std::vector<Rec> r(q.begin(), q.begin() + top);
          for (size_t j = 0; j < m; ++j) q[j] = r[kCuPerXcd - m + j];
          for (size_t j = m; j < (size_t)kCuPerXcd; ++j) q[j] = r[j - m];
          for (size_t j = 0; j < m; ++j) q[kCuPerXcd + j] = r[top - 1 - j];
        }
        longest = std::max(longest, queue[x].size());
      }
      order.reserve(longest * kXcd);
      size_t last_real = 0;
      for (size_t k = 0; k < longest; ++k)
        for (int x = 0; x < kXcd; ++x) {
          if (k < queue[x].size()) {
            order.push_back(queue[x][k].idx);
            last_real = order.size();
          } else {
            order.push_back(-1);
          }
        }
      order.resize(last_real);
    }
  }
  const int32_t n_work = (int32_t)order.size();
  int64_t n_partials = 0;
  std::vector<int32_t> part_off(n_parts.size());
  for (size_t t = 0; t < n_parts.size(); ++t) {
    part_off[t] = (int32_t)n_partials;
    n_partials += n_parts[t];
  }
  if (n_work > c.max_work_items)
    return fail(OXY_ERR_WORKSPACE, "batch_build: %d work items > max_work_items %d", n_work,
                c.max_work_items);
  if (n_partials > c.max_partials)
    return fail(OXY_ERR_WORKSPACE, "batch_build: %lld partials > max_partials %d",
                (long long)n_partials, c.max_partials);
  if ((size_t)tbl_words > table_words_of(c))
    return fail(OXY_ERR_WORKSPACE,
                "batch_build: the block tables of this batch list %d entries > %zu (forked "
                "prefixes list shared blocks once each)", tbl_words, table_words_of(c));

  // ---- a free descriptor slot
  int32_t slot = -1;
  for (int32_t i = 0; i < (int32_t)p->slots.size(); ++i)
    if (!p->slots[i].in_use) {
      slot = i;
      break;
    }
  if (slot < 0)
    return fail(OXY_ERR_BUSY, "batch_build: %d batches alive (max_live_batches)", p->live_batches);
  oxy_batch* b = new (std::nothrow) oxy_batch();
  if (!b) return fail(OXY_ERR_INVALID_ARG, "batch_build: out of host memory");

  // ---- commit: take blocks in item order; the descriptor image is filled in place
  b->pool = p;
  b->slot = slot;
  b->flags = flags;
  b->n_items = n_items;
  b->n_tokens = (int32_t)n_tokens;
  b->n_work = n_work;
  b->n_partials = (int32_t)n_partials;
  b->off_slots = 0;
  b->append_foldable = foldable;
  // Sections in the order slots | work | part_off | n_parts | fresh tokens | token lists | tables: the block
  // tables, whose size changes whenever a stream takes a new block, come last, so that the
  // device addresses of all sections stay the same from step to step while the shape of the
  // batch (tokens, work items, tile token lists) does -- a recorded launch sequence
  // (OXY_STEP_GRAPH) can then be replayed unchanged.
  // The grid is the work list rounded up to a multiple of 64 records (padding records end at
  // once): the launch shape then changes only every 64 work items, not whenever a history
  // crosses a split boundary.
  b->n_launch = std::max(n_work, std::min((n_work + 63) / 64 * 64, c.max_work_items));
  b->off_work = b->off_slots + (int32_t)n_tokens;
  b->off_part_off = b->off_work + b->n_launch * oxy::kWorkWords;
  b->off_n_parts = b->off_part_off + (int32_t)part_off.size();
  b->n_fresh = (int32_t)fresh_toks.size();
  b->off_fresh = b->off_n_parts + (int32_t)n_parts.size();
  b->off_toks = b->off_fresh + b->n_fresh;
  b->off_tables = b->off_toks + (int32_t)toks.size();
  std::vector<int32_t>& h = b->host;
  h.resize((size_t)b->off_tables + tbl_words);
  if (h.size() > p->desc_words) {   // cannot happen: every section was bounded above
    delete b;
    return fail(OXY_ERR_WORKSPACE, "batch_build: descriptor overflow (internal)");
  }
  {
    int32_t* sl = &h[b->off_slots];
    for (Plan& pl : plan) {
      for (int32_t i = 0; i < pl.need; ++i) {
        int32_t blk = p->free_stack.back();
        p->free_stack.pop_back();
        p->ref[blk] = 1;
        pl.s->blocks.push_back(blk);
      }
      pl.s->len = pl.new_len;
      for (int32_t t = pl.old_len; t < pl.new_len; ++t)
        *sl++ = pl.s->blocks[t / kPage] * kPage + t % kPage;
    }
  }
  int32_t* tables = h.data() + b->off_tables;
  for (const TableRef& tr : table_refs)
    std::copy(tr.src->begin(), tr.src->begin() + tr.count, tables + tr.off);
  std::copy(toks.begin(), toks.end(), h.begin() + b->off_toks);
  std::copy(fresh_toks.begin(), fresh_toks.end(), h.begin() + b->off_fresh);
  std::copy(part_off.begin(), part_off.end(), h.begin() + b->off_part_off);
  std::copy(n_parts.begin(), n_parts.end(), h.begin() + b->off_n_parts);
  // Work records, 128 bytes each: header, then inline copies of the tile's token ids and of the
  // block ids of the split's first pages, so a workgroup needs one load before its first pages.
  for (int32_t i = 0; i < b->n_launch; ++i) {
    int32_t* w = &h[(size_t)b->off_work + (size_t)i * oxy::kWorkWords];
    if (i >= n_work || order[i] < 0) {
      const int32_t noop[kHdr] = {0, 0, 0, 0, 0, oxy::kNoCausal, 0, oxy::PATH_NOOP};
      std::copy(noop, noop + kHdr, w);
      std::fill(w + kHdr, w + oxy::kWorkWords, 0);
      continue;
    }
    const int32_t* r = &hdr[(size_t)order[i] * kHdr];
    std::copy(r, r + kHdr, w);
    for (int32_t k = 0; k < oxy::kWorkInlineToks; ++k)
      w[8 + k] = toks[r[oxy::W_TOK_OFF] + std::min(k, r[oxy::W_N_TOK] - 1)];
    const int32_t pg0 = r[oxy::W_KV_BEGIN] / kPage;
    const int32_t npg = blocks_for(r[oxy::W_KV_END]) - pg0;
    for (int32_t k = 0; k < oxy::kWorkInlinePages; ++k)
      w[16 + k] = tables[r[oxy::W_TBL_OFF] + pg0 + std::min(k, npg - 1)];
  }

  DescSlot& ds = p->slots[slot];
  if (!p->host_only) {
    if (ds.event_pending) {
      (void)hipEventSynchronize(ds.uploaded);  // staging of an earlier batch fully consumed
      ds.event_pending = false;
    }
    memcpy(ds.staging, h.data(), h.size() * 4);
    hipError_t e = hipMemcpyAsync(ds.d_base, ds.staging, h.size() * 4, hipMemcpyHostToDevice,
                                  (hipStream_t)hip_stream);
    if (e == hipSuccess) e = hipEventRecord(ds.uploaded, (hipStream_t)hip_stream);
    if (e != hipSuccess) {
      // a failing call changes no pool state: lengths back, blocks back in reverse order of
      // their pops (which restores the free stack exactly)
      for (auto it = plan.rbegin(); it != plan.rend(); ++it) {
        for (int32_t i = 0; i < it->need; ++i) {
          p->ref[it->s->blocks.back()] = 0;
          p->free_stack.push_back(it->s->blocks.back());
          it->s->blocks.pop_back();
        }
        it->s->len = it->len_before;
      }
      delete b;
      return hip_fail(e, "batch_build: descriptor upload");
    }
    ds.event_pending = true;
  }
  ds.in_use = true;
  p->live_batches++;
  *out = b;
  return OXY_OK;
}

int32_t oxy_batch_destroy(oxy_batch* b) {
  if (!b) return fail(OXY_ERR_INVALID_ARG, "batch_destroy: null");
  b->pool->slots[b->slot].in_use = false;
  b->pool->live_batches--;
  delete b;
  return OXY_OK;
}

int32_t oxy_stream_append(oxy_pool* p, const oxy_batch* b, int32_t layer, const void* k_new,
                          const void* v_new, void* hip_stream) {
  if (!p || !b || b->pool != p || !k_new || !v_new || p->host_only)
    return fail(OXY_ERR_INVALID_ARG, "stream_append: null argument, foreign batch or host-only pool");
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(OXY_ERR_INVALID_ARG, "stream_append: layer %d", layer);
  const int32_t* d_desc = (const int32_t*)p->slots[b->slot].d_base;
  hipError_t e = oxy::launch_append(k_new, v_new, d_desc + b->off_slots, b->n_tokens,
                                    layer_base(p, layer), (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "stream_append: launch");
  return OXY_OK;
}

namespace {
oxy::AttnArgs attn_args(const oxy_pool* p, const oxy_batch* b, int32_t layer, const void* q, void* out,
                        float* lse, float scale) {
  const DescSlot& ds = p->slots[b->slot];
  const int32_t* d = (const int32_t*)ds.d_base;
  oxy::AttnArgs a;
  a.layer_base = layer_base(p, layer);
  a.q = q;
  a.out = out;
  a.lse = lse;
  a.work = d + b->off_work;
  a.tables = d + b->off_tables;
  a.part_off = d + b->off_part_off;
  a.n_parts = d + b->off_n_parts;
  a.part_acc = (uint16_t*)(ds.d_base + p->acc_offset);
  a.part_ml = (float*)(ds.d_base + p->ml_offset);
  a.n_work = b->n_launch;
  a.n_q = b->n_tokens;
  a.scale = scale;
  a.k_new = a.v_new = nullptr;
  a.d_slots = nullptr;
  return a;
}
}  // namespace

int32_t oxy_mixed_attention(oxy_pool* p, const oxy_batch* b, int32_t layer, const void* q,
                            void* out, float* lse, float scale, void* hip_stream) {
  if (!p || !b || b->pool != p || !q || !out || p->host_only)
    return fail(OXY_ERR_INVALID_ARG, "mixed_attention: null argument, foreign batch or host-only pool");
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(OXY_ERR_INVALID_ARG, "mixed_attention: layer %d", layer);
  if (b->flags & OXY_BATCH_APPEND_ONLY)
    return fail(OXY_ERR_INVALID_ARG, "mixed_attention: batch was built append-only");
  hipError_t e = oxy::launch_attention(attn_args(p, b, layer, q, out, lse, scale),
                                       (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "mixed_attention: launch");
  return OXY_OK;
}

int32_t oxy_mixed_attention_static(oxy_pool* p, const oxy_batch* b, int32_t layer, const void* q,
                                   void* out, float* lse, float scale, void* hip_stream) {
  if (!p || !b || b->pool != p || !q || !out || p->host_only)
    return fail(OXY_ERR_INVALID_ARG,
                "mixed_attention_static: null argument, foreign batch or host-only pool");
  if (layer < 0 || layer >= p->cfg.n_layers)
    return fail(OXY_ERR_INVALID_ARG, "mixed_attention_static: layer %d", layer);
  if (b->flags & OXY_BATCH_APPEND_ONLY)
    return fail(OXY_ERR_INVALID_ARG, "mixed_attention_static: batch was built append-only");
  if (b->n_partials > oxy::kStaticMaxPartials)
    return fail(OXY_ERR_WORKSPACE,
                "mixed_attention_static: the batch has %d split results, the static buffer holds %d",
                b->n_partials, oxy::kStaticMaxPartials);
  oxy::AttnArgs a = attn_args(p, b, layer, q, out, lse, scale);
  hipError_t e = oxy::static_scratch(&a.part_acc, &a.part_ml);
  if (e != hipSuccess) return hip_fail(e, "mixed_attention_static: static buffer");
  e = oxy::launch_attention(a, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "mixed_attention_static: launch");
  return OXY_OK;
}

namespace {
struct StepCall {
  oxy_pool* p;
  const oxy_batch* b;
  int32_t layer_begin, layer_end;
  const void *k_new, *v_new;
  size_t kv_layer_stride;
  const void* q;
  void* out;
  size_t q_layer_stride;
  float* lse;
  size_t lse_layer_stride;
  float scale;
  bool fold, fuse;
  void* const* events;
};

// The launches of one step, in order, on stream s.  Same effects as the per-layer calls.  With
// `fuse`, the merge of layer l and the append of layer l+1 (disjoint memory) share one launch;
// with `fold`, the work items do the append.
int32_t issue_step(const StepCall& c, hipStream_t s) {
  oxy_pool* p = c.p;
  const oxy_batch* b = c.b;
  const int32_t* d_desc = (const int32_t*)p->slots[b->slot].d_base;
  auto append_of = [&](int32_t layer) {
    oxy::AppendArgs ap;
    ap.k_new = (const char*)c.k_new + (size_t)layer * c.kv_layer_stride;
    ap.v_new = (const char*)c.v_new + (size_t)layer * c.kv_layer_stride;
    ap.d_slots = d_desc + b->off_slots;
    ap.n_tokens = b->n_tokens;
    ap.layer_base = layer_base(p, layer);
    ap.tok_list = nullptr;
    return ap;
  };
  auto append_now = [&](int32_t layer) {
    oxy::AppendArgs ap = append_of(layer);
    return oxy::launch_append(ap.k_new, ap.v_new, ap.d_slots, ap.n_tokens, ap.layer_base, s);
  };
  if (c.fuse) {
    hipError_t e = append_now(c.layer_begin);
    if (e != hipSuccess) return hip_fail(e, "step_layers: append");
  }
  for (int32_t layer = c.layer_begin; layer < c.layer_end; ++layer) {
    const size_t i = (size_t)(layer - c.layer_begin);
    hipError_t e = hipSuccess;
    if (!c.fuse && !c.fold) {
      e = append_now(layer);
      if (e != hipSuccess) return hip_fail(e, "step_layers: append");
    }
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    if (c.events)
      for (int j = 0; j < 4; ++j) ev[j] = (hipEvent_t)c.events[4 * i + j];
    oxy::AttnArgs a =
        attn_args(p, b, layer, (const char*)c.q + (size_t)layer * c.q_layer_stride,
                  (char*)c.out + (size_t)layer * c.q_layer_stride,
                  c.lse ? (float*)((char*)c.lse + (size_t)layer * c.lse_layer_stride) : nullptr,
                  c.scale);
    if (c.fold) {
      const oxy::AppendArgs ap = append_of(layer);
      a.k_new = ap.k_new;
      a.v_new = ap.v_new;
      a.d_slots = ap.d_slots;
    }
    e = oxy::launch_attention_work(a, s, ev[0], ev[1]);
    if (e != hipSuccess) return hip_fail(e, "step_layers: attention");
    if (c.fuse && layer + 1 < c.layer_end) {
      oxy::AppendArgs nx = append_of(layer + 1);
      e = oxy::launch_merge_append(a, &nx, s, ev[2], ev[3]);
    } else if (c.fold && b->n_fresh > 0) {
      // items whose tiles took their keys from k_new / v_new: their rows go to the pool here
      oxy::AppendArgs fr = append_of(layer);
      fr.n_tokens = b->n_fresh;
      fr.tok_list = d_desc + b->off_fresh;
      e = oxy::launch_merge_append(a, &fr, s, ev[2], ev[3]);
    } else {
      e = oxy::launch_merge_append(a, nullptr, s, ev[2], ev[3]);
    }
    if (e != hipSuccess) return hip_fail(e, "step_layers: merge");
  }
  return OXY_OK;
}

// OXY_STEP_GRAPH: the launches of the step are recorded once (stream capture on a stream of the
// library's own; nothing runs there) and replayed with one graph launch on the caller's stream.
// A step whose key equals a recorded one replays it as it is; otherwise the step is recorded
// again and, where a recording with the same sequence of launches exists and the cache is
// full, that one is updated in place instead of instantiating another.
int32_t replay_step(const StepCall& c, hipStream_t s) {
  oxy_pool* p = c.p;
  const oxy_batch* b = c.b;
  StepKey key;
  key.d_base = p->slots[b->slot].d_base;
  key.k_new = c.k_new;
  key.v_new = c.v_new;
  key.q = c.q;
  key.out = c.out;
  key.lse = c.lse;
  key.kv_stride = c.kv_layer_stride;
  key.q_stride = c.q_layer_stride;
  key.lse_stride = c.lse_layer_stride;
  key.scale = c.scale;
  key.layer_begin = c.layer_begin;
  key.layer_end = c.layer_end;
  key.mode = c.fold ? 2 : c.fuse ? 1 : 0;
  key.n_work = b->n_launch;
  key.n_tokens = b->n_tokens;
  key.n_fresh = b->n_fresh;
  key.off_work = b->off_work;
  key.off_tables = b->off_tables;
  key.off_part_off = b->off_part_off;
  key.off_n_parts = b->off_n_parts;
  const uint64_t now = ++p->graph_clock;
  StepGraph* hit = nullptr;
  for (StepGraph& g : p->graphs)
    if (g.key == key) {
      hit = &g;
      break;
    }
  if (!hit) {
    hipError_t e = hipSuccess;
    if (!p->record_stream) {
      e = hipStreamCreateWithFlags(&p->record_stream, hipStreamNonBlocking);
      if (e != hipSuccess) return hip_fail(e, "step_layers: stream for recording");
    }
    e = hipStreamBeginCapture(p->record_stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return hip_fail(e, "step_layers: begin recording");
    const int32_t rc = issue_step(c, p->record_stream);
    hipGraph_t graph = nullptr;
    e = hipStreamEndCapture(p->record_stream, &graph);   // always: leaves recording mode
    if (rc != OXY_OK) {
      if (graph) (void)hipGraphDestroy(graph);
      return rc;
    }
    if (e != hipSuccess || !graph) return hip_fail(e, "step_layers: end recording");
    // a victim to update in place: least recently used recording with the same launch sequence,
    // taken only when the cache is full
    StepGraph* victim = nullptr;
    if (p->graphs.size() >= kMaxStepGraphs) {
      for (StepGraph& g : p->graphs)
        if (g.key.same_topology(key) && (!victim || g.last_use < victim->last_use)) victim = &g;
      if (!victim) {   // none fits: drop the least recently used one
        size_t lru = 0;
        for (size_t i = 1; i < p->graphs.size(); ++i)
          if (p->graphs[i].last_use < p->graphs[lru].last_use) lru = i;
        (void)hipGraphExecDestroy(p->graphs[lru].exec);
        p->graphs.erase(p->graphs.begin() + lru);
      }
    }
    if (victim) {
      hipGraphNode_t bad = nullptr;
      hipGraphExecUpdateResult res = hipGraphExecUpdateSuccess;
      e = hipGraphExecUpdate(victim->exec, graph, &bad, &res);
      if (e == hipSuccess && res == hipGraphExecUpdateSuccess) {
        victim->key = key;
        hit = victim;
        p->graph_updates++;
      } else {
        (void)hipGetLastError();
        (void)hipGraphExecDestroy(victim->exec);
        p->graphs.erase(p->graphs.begin() + (victim - p->graphs.data()));
      }
    }
    if (!hit) {
      hipGraphExec_t exec = nullptr;
      e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      if (e != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return hip_fail(e, "step_layers: instantiate the recorded step");
      }
      p->graphs.push_back(StepGraph{key, exec, now});
      hit = &p->graphs.back();
      p->graph_instantiations++;
    }
    (void)hipGraphDestroy(graph);
  }
  hit->last_use = now;
  hipError_t e = hipGraphLaunch(hit->exec, s);
  if (e != hipSuccess) return hip_fail(e, "step_layers: replay");
  p->graph_replays++;
  return OXY_OK;
}
}  // namespace

int32_t oxy_step_layers(oxy_pool* p, const oxy_batch* b, int32_t layer_begin, int32_t layer_end,
                        const void* k_new, const void* v_new, size_t kv_layer_stride,
                        const void* q, void* out, size_t q_layer_stride, float* lse,
                        size_t lse_layer_stride, float scale, int32_t flags, void* const* events,
                        void* hip_stream) {
  if (flags & ~(OXY_STEP_FUSE_ACROSS_LAYERS | OXY_STEP_FOLD_APPEND | OXY_STEP_GRAPH))
    return fail(OXY_ERR_INVALID_ARG, "step_layers: flags");
  if (!p || !b || b->pool != p || !k_new || !v_new || !q || !out || p->host_only)
    return fail(OXY_ERR_INVALID_ARG, "step_layers: null argument, foreign batch or host-only pool");
  if (layer_begin < 0 || layer_end > p->cfg.n_layers || layer_begin >= layer_end)
    return fail(OXY_ERR_INVALID_ARG, "step_layers: layers [%d, %d)", layer_begin, layer_end);
  if (b->flags & OXY_BATCH_APPEND_ONLY)
    return fail(OXY_ERR_INVALID_ARG, "step_layers: batch was built append-only");
  if ((flags & OXY_STEP_GRAPH) && events)
    return fail(OXY_ERR_INVALID_ARG, "step_layers: timing events cannot go into a recorded step");
  StepCall c;
  c.p = p;
  c.b = b;
  c.layer_begin = layer_begin;
  c.layer_end = layer_end;
  c.k_new = k_new;
  c.v_new = v_new;
  c.kv_layer_stride = kv_layer_stride;
  c.q = q;
  c.out = out;
  c.q_layer_stride = q_layer_stride;
  c.lse = lse;
  c.lse_layer_stride = lse_layer_stride;
  c.scale = scale;
  c.fold = (flags & OXY_STEP_FOLD_APPEND) != 0 && b->append_foldable;
  c.fuse = (flags & OXY_STEP_FUSE_ACROSS_LAYERS) != 0 && !c.fold;
  c.events = events;
  if (flags & OXY_STEP_GRAPH) return replay_step(c, (hipStream_t)hip_stream);
  return issue_step(c, (hipStream_t)hip_stream);
}

int32_t oxy_step_graph_stats(oxy_pool* p, int32_t* instantiations, int32_t* updates,
                             int32_t* replays) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "step_graph_stats: null");
  if (instantiations) *instantiations = p->graph_instantiations;
  if (updates) *updates = p->graph_updates;
  if (replays) *replays = p->graph_replays;
  return OXY_OK;
}

int32_t oxy_append_attention(oxy_pool* p, const oxy_batch* b, int32_t layer, const void* k_new,
                             const void* v_new, const void* q, void* out, float* lse, float scale,
                             void* hip_stream) {
  if (layer < 0 || !p || layer >= p->cfg.n_layers)
    return fail(OXY_ERR_INVALID_ARG, "append_attention: null pool or layer %d", layer);
  // one layer of oxy_step_layers with the append folded in (layer strides 0: the pointers are
  // this layer's own)
  return oxy_step_layers(p, b, layer, layer + 1, k_new, v_new, 0, q, out, 0, lse, 0, scale,
                         OXY_STEP_FOLD_APPEND, nullptr, hip_stream);
}

int32_t oxy_gather_kv(oxy_pool* p, int32_t layer, const int64_t* slots, int32_t n, void* k_out,
                      void* v_out, void* hip_stream) {
  if (!p || !slots || n < 1 || !k_out || !v_out || p->host_only)
    return fail(OXY_ERR_INVALID_ARG, "gather_kv: null argument or host-only pool");
  if (layer < 0 || layer >= p->cfg.n_layers) return fail(OXY_ERR_INVALID_ARG, "gather_kv: layer %d", layer);
  const int64_t n_slots = (int64_t)p->cfg.num_blocks * kPage;
  for (int32_t i = 0; i < n; ++i)
    if (slots[i] < 0 || slots[i] >= n_slots)
      return fail(OXY_ERR_INVALID_ARG, "gather_kv: slot %lld out of range", (long long)slots[i]);
  for (int32_t done = 0; done < n; done += oxy::kMaxInlineBlocks) {
    int32_t m = std::min(oxy::kMaxInlineBlocks, n - done);
    oxy::InlineIds ids;
    for (int32_t i = 0; i < m; ++i) ids.v[i] = (int32_t)slots[done + i];
    hipError_t e = oxy::launch_gather_inline(layer_base(p, layer), ids, m,
                                             (char*)k_out + (size_t)done * oxy::kDim * 2,
                                             (char*)v_out + (size_t)done * oxy::kDim * 2,
                                             (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "gather_kv: launch");
  }
  return OXY_OK;
}

// ---- introspection ------------------------------------------------------------------------
int32_t oxy_stream_info(oxy_pool* p, int32_t sid, int32_t* prefix_id, int32_t* kind,
                        int32_t* own_len, int32_t* n_blocks) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "stream_info: null pool");
  auto it = p->streams.find(sid);
  if (it == p->streams.end()) return fail(OXY_ERR_BAD_ID, "stream_info: no stream %d", sid);
  if (prefix_id) *prefix_id = it->second.prefix_id;
  if (kind) *kind = it->second.kind;
  if (own_len) *own_len = it->second.len;
  if (n_blocks) *n_blocks = (int32_t)it->second.blocks.size();
  return OXY_OK;
}

int32_t oxy_stream_blocks(oxy_pool* p, int32_t sid, int32_t* out, int32_t cap) {
  if (!p || !out) return fail(OXY_ERR_INVALID_ARG, "stream_blocks: null argument");
  auto it = p->streams.find(sid);
  if (it == p->streams.end()) return fail(OXY_ERR_BAD_ID, "stream_blocks: no stream %d", sid);
  if (cap < (int32_t)it->second.blocks.size()) return fail(OXY_ERR_INVALID_ARG, "stream_blocks: cap");
  std::copy(it->second.blocks.begin(), it->second.blocks.end(), out);
  return OXY_OK;
}

int32_t oxy_prefix_info(oxy_pool* p, int32_t pid, int32_t* len, int32_t* n_blocks,
                        int32_t* sealed, int32_t* n_streams) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "prefix_info: null pool");
  auto it = p->prefixes.find(pid);
  if (it == p->prefixes.end()) return fail(OXY_ERR_BAD_ID, "prefix_info: no prefix %d", pid);
  if (len) *len = it->second.len;
  if (n_blocks) *n_blocks = (int32_t)it->second.blocks.size();
  if (sealed) *sealed = it->second.sealed ? 1 : 0;
  if (n_streams) *n_streams = it->second.n_streams;
  return OXY_OK;
}

int32_t oxy_prefix_blocks(oxy_pool* p, int32_t pid, int32_t* out, int32_t cap) {
  if (!p || !out) return fail(OXY_ERR_INVALID_ARG, "prefix_blocks: null argument");
  auto it = p->prefixes.find(pid);
  if (it == p->prefixes.end()) return fail(OXY_ERR_BAD_ID, "prefix_blocks: no prefix %d", pid);
  if (cap < (int32_t)it->second.blocks.size()) return fail(OXY_ERR_INVALID_ARG, "prefix_blocks: cap");
  std::copy(it->second.blocks.begin(), it->second.blocks.end(), out);
  return OXY_OK;
}

int32_t oxy_block_refcounts(oxy_pool* p, int32_t* out, int32_t cap) {
  if (!p || !out || cap < p->cfg.num_blocks) return fail(OXY_ERR_INVALID_ARG, "block_refcounts: cap");
  std::copy(p->ref.begin(), p->ref.end(), out);
  return OXY_OK;
}

int32_t oxy_free_blocks(oxy_pool* p, int32_t* out, int32_t cap) {
  if (!p || !out || cap < (int32_t)p->free_stack.size()) return fail(OXY_ERR_INVALID_ARG, "free_blocks: cap");
  std::copy(p->free_stack.rbegin(), p->free_stack.rend(), out);
  return OXY_OK;
}

int32_t oxy_pool_stats(oxy_pool* p, int32_t* free_blocks, int32_t* live_prefixes,
                       int32_t* live_streams) {
  if (!p) return fail(OXY_ERR_INVALID_ARG, "pool_stats: null pool");
  if (free_blocks) *free_blocks = (int32_t)p->free_stack.size();
  if (live_prefixes) *live_prefixes = (int32_t)p->prefixes.size();
  if (live_streams) *live_streams = (int32_t)p->streams.size();
  return OXY_OK;
}

int32_t oxy_batch_info(const oxy_batch* b, int32_t* n_items, int32_t* n_tokens, int32_t* n_work,
                       int32_t* n_partials) {
  if (!b) return fail(OXY_ERR_INVALID_ARG, "batch_info: null");
  if (n_items) *n_items = b->n_items;
  if (n_tokens) *n_tokens = b->n_tokens;
  if (n_work) *n_work = b->n_work;
  if (n_partials) *n_partials = b->n_partials;
  return OXY_OK;
}

int32_t oxy_batch_slots(const oxy_batch* b, int64_t* out, int32_t cap) {
  if (!b || !out || cap < b->n_tokens) return fail(OXY_ERR_INVALID_ARG, "batch_slots: cap");
  for (int32_t i = 0; i < b->n_tokens; ++i) out[i] = b->host[b->off_slots + i];
  return OXY_OK;
}

int32_t oxy_batch_work(const oxy_batch* b, int32_t* out, int32_t cap_items) {
  if (!b || !out || cap_items < b->n_work) return fail(OXY_ERR_INVALID_ARG, "batch_work: cap");
  for (int32_t i = 0; i < b->n_work; ++i) {   // the eight header words of each record
    std::copy(b->host.begin() + b->off_work + (size_t)i * oxy::kWorkWords,
              b->host.begin() + b->off_work + (size_t)i * oxy::kWorkWords + 8, out + (size_t)i * 8);
    out[(size_t)i * 8 + oxy::W_PATH] &= oxy::kPathMask;
  }
  return OXY_OK;
}

}  // extern "C"
