// Internal interface between the host pool (oxy_pool.cpp) and the HIP kernels
// (oxy_kernels.hip).  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oxy {

constexpr int kHeads = 8;        // query heads sharing the one KV head
constexpr int kDim = 256;        // head_dim
constexpr int kPage = 16;        // tokens per page
constexpr int kPageBytes = kPage * kDim * 2;      // one K page or one V page (bf16)
constexpr int kBlockBytes = 2 * kPageBytes;       // K page + V page of one layer
constexpr int kNoCausal = 0x3fffffff;
constexpr int kWorkWords = 32;             // one 128-byte line per work record
constexpr int kWorkInlineToks = 8;         // words 8..15: query token ids of the tile
constexpr int kWorkInlinePages = 16;       // words 16..31: block ids of the first 16 pages
constexpr int kMaxInlineBlocks = 512;             // block ids passed by value to append/gather

// work record fields (words 0..7)
enum { W_TOK_OFF = 0, W_N_TOK, W_TBL_OFF, W_KV_BEGIN, W_KV_END, W_CAUSAL_Q0, W_PART_IDX, W_PATH };
// paths
enum { PATH_STREAM = 0,  // <=2 query tokens (16 rows): 4 wavefronts split the keys, KV to registers
       PATH_TILE = 1,    // <=8 query tokens (64 rows): 4 wavefronts share the keys through LDS
       PATH_NOOP = 2 };  // padding that keeps the index -> XCD pattern of the work list intact
// The path sits in the low four bits of word W_PATH.  kPathFresh marks an own-phase tile of an
// item whose own history was empty before this step: all of its keys are rows of this step's
// k_new / v_new, row = (word >> kPathRowShift) + own position.
// kPathAppends marks a streaming work item on an item's own pages: its query tokens are the new
// rows that a folded append has to write (a streaming item on prefix pages appends nothing).
constexpr int kPathMask = 15, kPathFresh = 16, kPathAppends = 32, kPathRowShift = 8;

struct InlineIds {
  int32_t v[kMaxInlineBlocks];
};

// Scatter n_tokens rows of K and V (natural [token][256] bf16) into the slots of one layer.
hipError_t launch_append(const void* k_new, const void* v_new, const int32_t* d_slots,
                         int32_t n_tokens, void* layer_base, hipStream_t s);
// Same, slots = blocks.v[(pos0+t)/16]*16 + (pos0+t)%16 with the block ids passed by value.
// n_layers consecutive layers in one launch: layer i reads k_new/v_new + i*src_layer_stride and
// writes layer_base + i*pool_layer_stride (bytes).
hipError_t launch_append_inline(const void* k_new, const void* v_new, const InlineIds& blocks,
                                int32_t pos0, int32_t n_tokens, void* layer_base, int32_t n_layers,
                                size_t src_layer_stride, size_t pool_layer_stride, hipStream_t s);
// Gather rows back to natural order; slot ids passed by value (<= kMaxInlineBlocks per call).
hipError_t launch_gather_inline(const void* layer_base, const InlineIds& slots, int32_t n,
                                void* k_out, void* v_out, hipStream_t s);

struct AttnArgs {
  const void* layer_base;   // KV of this layer
  const void* q;            // [n_q][8][256] bf16
  void* out;                // [n_q][8][256] bf16
  float* lse;               // [n_q][8] or null
  const int32_t* work;      // [n_work][32]: one 128-byte record per work item
  const int32_t* tables;
  const int32_t* part_off;  // [n_q]
  const int32_t* n_parts;   // [n_q]
  uint16_t* part_acc;       // [n_partials][8][256] fp16: accumulator / row scale
  float* part_ml;           // [n_partials][8][4]: reference max (log2 domain), sum, row scale, -
  int32_t n_work;
  int32_t n_q;
  float scale;
  // Append folded into the work items (all three null otherwise): this step's new rows
  // [n_q][256] bf16 and their slots.  A streaming work item first writes the new rows that lie
  // in its key range into the pool; a fresh tile reads its keys from the new rows themselves
  // (the merge launch of the layer writes those rows to the pool).
  const void* k_new;
  const void* v_new;
  const int32_t* d_slots;
};
hipError_t launch_attention(const AttnArgs& a, hipStream_t s);       // work items, then merge
// Split-result buffers in static device memory of the current device (kStaticMaxPartials
// entries, shared by every call on that device).  The first call on a device looks the address
// up; later calls make no HIP call other than hipGetDevice.
constexpr int kStaticMaxPartials = 2048;
hipError_t static_scratch(uint16_t** part_acc, float** part_ml);
// work items only; start/stop (may be null) receive the kernel's own begin/end timestamps
hipError_t launch_attention_work(const AttnArgs& a, hipStream_t s, hipEvent_t start = nullptr,
                                 hipEvent_t stop = nullptr);
struct AppendArgs {
  const void* k_new;
  const void* v_new;
  const int32_t* d_slots;
  int32_t n_tokens;
  void* layer_base;
  const int32_t* tok_list;   // null: tokens 0..n_tokens-1; else the n_tokens token ids to append
};
// merge of `a`, and in the same launch the append described by `next` (may be null)
hipError_t launch_merge_append(const AttnArgs& a, const AppendArgs* next, hipStream_t s,
                               hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

}  // namespace oxy
