// HIP kernels for gfx950 (MI355X): KV append / gather and the mixed-mask paged attention.
//
// What is computed is the attention inside the paper's ActionDenoise and
// BatchedLanguageDecode passes (App. A.1, Eq. 5-6) for queries of several tasks at once,
// all reading one shared prefill cache (Sec. 3.2, cross-task KV sharing) plus their own
// tokens.  Visibility: prefix always; own tokens causally for decode queries, all of the
// chunk for action queries.
//
// Evaluation scheme.  The visible set of a query is cut into (prefix | own) and each part
// into fixed-size splits.  A work item is (query rows that share one KV source, one split of
// that source); it yields an un-normalised partial (reference max m in the log2 domain, sum
// l, accumulator acc[256]).  A second kernel merges a query's partials by the log-sum-exp
// rule.  The split size is fixed per pool and the path that evaluates a query depends on
// its item only, so the arithmetic of a query never depends on what else is in the batch.
//
// MFMA mapping (v_mfma_f32_16x16x32_bf16, lane = 16*g + n, keys taken 32 at a time = page A
// and page B of the block table):
//   S^T[key][row]  = sum_d K[key][d] * Q[row][d]      A = K chunks, B = Q rows
//       tile hf (0,1): A-row r is key 8hf + r%8 of page r/8, so lane (n = row, g) receives
//       the logits of keys 8hf + 4(g%2) + e, e < 4, of page g/2
//   O^T[d][row]   += sum_key V[key][d] * P[row][key]  A = V chunk, B = P
//       lane (g) contracts exactly the eight keys it holds logits for, all of one page, so
//       its V operand is ONE 16-byte chunk of that page and P needs no cross-lane movement
//       -> lane (n = row, g) accumulates d = 16c+4g..16c+4g+3
// Both results keep "row = lane % 16", so the softmax state (m, l, rescale factor) is a
// per-lane scalar.  The pool pages are stored in exactly the operand order these products
// want (see oxy.h): every MFMA operand is one aligned 16-byte load.
#include "oxy_internal.h"

#include <hip/hip_ext.h>

#include <mutex>

namespace oxy {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// two floats -> packed bf16 pair, round to nearest even (inputs are finite here)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
  f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two floats -> packed fp16 pair (round to nearest even)
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2;
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_;
  const f32x2_ f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
}
__device__ __forceinline__ void unpack_f16(uint32_t u, float& lo, float& hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2;
  const f16x2 h = __builtin_bit_cast(f16x2, u);
  lo = (float)h[0];
  hi = (float)h[1];
}

// max over the four lanes {n, n+16, n+32, n+48} that hold one query row: two register swaps
// between lane halves (v_permlane16_swap, v_permlane32_swap), no LDS round trip
__device__ __forceinline__ float row_max4(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const uint32_t v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
// sum over the same four lanes, same two swaps: every lane adds its own value and its partner's
__device__ __forceinline__ float row_sum4(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const uint32_t v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// max over the 16 lanes of a row (lanes 16r .. 16r+15): four DPP moves, no LDS round trip.
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror: after each step twice
// as many neighbouring lanes hold the same value, so the mirrors act like xor 4 and xor 8.
__device__ __forceinline__ float lanes16_max(float x) {
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x4E, 0xF, 0xF, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x141, 0xF, 0xF, true)));
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x140, 0xF, 0xF, true)));
  return x;
}

// ------------------------------------------------------------------------------------------
// page layout (see oxy.h)
// ------------------------------------------------------------------------------------------
// K page: chunk (j, hf, g, k8) holds K[8hf+k8][32j+8g .. +7]
__device__ __forceinline__ int k_chunk_offset(int j, int hf, int g, int k8) {
  return ((((j * 2 + hf) * 4 + g) * 8) + k8) * 16;
}
// V page: chunk (c, gp, m) holds V[4gp..4gp+3][16c+m] then V[8+4gp..8+4gp+3][16c+m]
__device__ __forceinline__ int v_chunk_offset(int c, int gp, int m) {
  return (((c * 2 + gp) * 16) + m) * 16;
}
__device__ __forceinline__ int v_slot_of_key(int key) { return ((key >> 3) << 2) | (key & 3); }

// ------------------------------------------------------------------------------------------
// append / gather
// ------------------------------------------------------------------------------------------
// One row of K and V on its way into a page: thread t of 256 carries 16 bytes of K (t < 32)
// and one element of V.  Load and store are separate so that callers can keep several rows in
// flight before the first store.
struct RowPart {
  u32x4 k;
  uint16_t v;
};
__device__ __forceinline__ RowPart load_row(const uint16_t* __restrict__ k_row,
                                            const uint16_t* __restrict__ v_row, int t) {
  RowPart r;
  r.k = *(const u32x4*)(k_row + (t & 31) * 8);
  r.v = v_row[t];
  return r;
}
__device__ __forceinline__ void store_row(const RowPart& r, int32_t slot,
                                          char* __restrict__ layer_base, int t) {
  const int blk = slot >> 4, key = slot & 15;
  char* kp = layer_base + (size_t)blk * kBlockBytes;
  char* vp = kp + kPageBytes;
  if (t < 32) *(u32x4*)(kp + k_chunk_offset(t >> 2, key >> 3, t & 3, key & 7)) = r.k;
  *(uint16_t*)(vp + v_chunk_offset(t >> 4, (key >> 2) & 1, t & 15) + v_slot_of_key(key) * 2) = r.v;
}
__device__ __forceinline__ void append_row(const uint16_t* __restrict__ k_row,
                                           const uint16_t* __restrict__ v_row, int32_t slot,
                                           char* __restrict__ layer_base, int t) {
  store_row(load_row(k_row, v_row, t), slot, layer_base, t);
}

__global__ __launch_bounds__(256) void append_kernel(const uint16_t* __restrict__ k_new,
                                                     const uint16_t* __restrict__ v_new,
                                                     const int32_t* __restrict__ slots,
                                                     char* __restrict__ layer_base) {
  const int tok = blockIdx.x;
  append_row(k_new + (size_t)tok * kDim, v_new + (size_t)tok * kDim, slots[tok], layer_base,
             threadIdx.x);
}

// Append of a run of consecutive positions of one table (a prefix): one workgroup per block.
// A block that is covered completely is written as whole 16-byte chunks (V transposed through
// LDS); a partly covered block falls back to the per-row scatter so that nothing else in the
// page is touched.
// blockIdx.y = layer relative to the first one: sources advance by src_layer_stride bytes, the
// pool by pool_layer_stride bytes per layer.
__global__ __launch_bounds__(256) void append_blocks_kernel(const uint16_t* __restrict__ k_new,
                                                            const uint16_t* __restrict__ v_new,
                                                            const InlineIds blocks, int32_t pos0,
                                                            int32_t n_tokens,
                                                            char* __restrict__ layer_base,
                                                            size_t src_layer_stride,
                                                            size_t pool_layer_stride) {
  __shared__ __align__(16) uint16_t v_s[kPage][kDim + 8];   // +8: rows land in different banks
  const int t = threadIdx.x;
  k_new = (const uint16_t*)((const char*)k_new + blockIdx.y * src_layer_stride);
  v_new = (const uint16_t*)((const char*)v_new + blockIdx.y * src_layer_stride);
  layer_base += blockIdx.y * pool_layer_stride;
  const int first_page = pos0 >> 4;
  const int page = first_page + blockIdx.x;
  const int lo = max(pos0, page * kPage), hi = min(pos0 + n_tokens, (page + 1) * kPage);
  const int blk = blocks.v[blockIdx.x];
  if (hi - lo < kPage) {
    for (int pos = lo; pos < hi; ++pos)
      append_row(k_new + (size_t)(pos - pos0) * kDim, v_new + (size_t)(pos - pos0) * kDim,
                 blk * kPage + (pos & 15), layer_base, t);
    return;
  }
  char* kp = layer_base + (size_t)blk * kBlockBytes;
  char* vp = kp + kPageBytes;
  const uint16_t* k_src = k_new + (size_t)(lo - pos0) * kDim;
  const uint16_t* v_src = v_new + (size_t)(lo - pos0) * kDim;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = t + 256 * i, key = idx >> 5, cd = idx & 31;
    *(u32x4*)(kp + k_chunk_offset(cd >> 2, key >> 3, cd & 3, key & 7)) =
        *(const u32x4*)(k_src + (size_t)key * kDim + cd * 8);
    *(u32x4*)(&v_s[key][cd * 8]) = *(const u32x4*)(v_src + (size_t)key * kDim + cd * 8);
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ci = t + 256 * i, c = ci >> 5, gp = (ci >> 4) & 1, m = ci & 15, d = 16 * c + m;
    u32x4 out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k0 = (e < 2 ? 4 * gp : 8 + 4 * gp) + 2 * (e & 1);
      out[e] = (uint32_t)v_s[k0][d] | ((uint32_t)v_s[k0 + 1][d] << 16);
    }
    *(u32x4*)(vp + v_chunk_offset(c, gp, m)) = out;
  }
}

__global__ __launch_bounds__(256) void gather_inline_kernel(const char* __restrict__ layer_base,
                                                            const InlineIds slots,
                                                            uint16_t* __restrict__ k_out,
                                                            uint16_t* __restrict__ v_out) {
  const int tok = blockIdx.x, t = threadIdx.x;
  const int slot = slots.v[tok];
  const int blk = slot >> 4, key = slot & 15;
  const char* kp = layer_base + (size_t)blk * kBlockBytes;
  const char* vp = kp + kPageBytes;
  if (t < 32)
    *(u32x4*)(k_out + (size_t)tok * kDim + t * 8) =
        *(const u32x4*)(kp + k_chunk_offset(t >> 2, key >> 3, t & 3, key & 7));
  v_out[(size_t)tok * kDim + t] =
      *(const uint16_t*)(vp + v_chunk_offset(t >> 4, (key >> 2) & 1, t & 15) + v_slot_of_key(key) * 2);
}

hipError_t launch_append(const void* k_new, const void* v_new, const int32_t* d_slots,
                         int32_t n_tokens, void* layer_base, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  append_kernel<<<n_tokens, 256, 0, s>>>((const uint16_t*)k_new, (const uint16_t*)v_new, d_slots,
                                         (char*)layer_base);
  return hipGetLastError();
}

hipError_t launch_append_inline(const void* k_new, const void* v_new, const InlineIds& blocks,
                                int32_t pos0, int32_t n_tokens, void* layer_base, int32_t n_layers,
                                size_t src_layer_stride, size_t pool_layer_stride, hipStream_t s) {
  if (n_tokens <= 0 || n_layers <= 0) return hipSuccess;
  // blocks.v[i] is the block of page (pos0 / 16 + i)
  const int32_t n_pages = ((pos0 + n_tokens + kPage - 1) >> 4) - (pos0 >> 4);
  append_blocks_kernel<<<dim3(n_pages, n_layers), 256, 0, s>>>(
      (const uint16_t*)k_new, (const uint16_t*)v_new, blocks, pos0, n_tokens, (char*)layer_base,
      src_layer_stride, pool_layer_stride);
  return hipGetLastError();
}

hipError_t launch_gather_inline(const void* layer_base, const InlineIds& slots, int32_t n,
                                void* k_out, void* v_out, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  gather_inline_kernel<<<n, 256, 0, s>>>((const char*)layer_base, slots, (uint16_t*)k_out,
                                         (uint16_t*)v_out);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// attention work items
// ------------------------------------------------------------------------------------------
// LDS stage of the tile path: K page A, K page B, V page A, V page B.  K page B is skewed by
// 128 bytes so that the 16 lanes served together (8 keys of page A, 8 of page B) hit
// different banks.
constexpr int kOffKA = 0;
constexpr int kOffKB = kPageBytes + 128;
constexpr int kOffVA = 2 * kPageBytes + 256;
constexpr int kOffVB = kOffVA + kPageBytes;
constexpr int kStageBytes = kOffVB + kPageBytes;      // 33024
constexpr int kMergeStride = kDim + 4;                // floats per row in the LDS merge buffer
constexpr int kEpilogueStride = kDim * 2 + 16;        // bytes per fp16 row in the tile epilogue
constexpr int kSmemBytes = 4 * 16 * kMergeStride * 4; // 66560 >= 2 * kStageBytes
static_assert(2 * kStageBytes <= kSmemBytes, "two stages must fit");
constexpr float kGrow = 8.f;  // the reference max only moves when a logit exceeds it by 2^8

// One 32-key step of the online softmax for the 16 rows of a wavefront.  s0/s1 hold the raw
// dot products of this lane's row with keys pos + 16(g/2) + 8hf + 4(g%2) + e (hf = 0 / 1).
// m is the reference max of the row in the scaled log2 domain.  It only moves when a logit
// exceeds it by more than kGrow, so the 64-register rescale of acc is rare; P is then at most
// 2^kGrow, well inside fp32/bf16 range.  P is returned as hi+lo bf16: a single bf16 rounding
// (2^-9 relative) is too coarse for queries that see only a handful of keys.
__device__ __forceinline__ void softmax_step(const f32x4 s0, const f32x4 s1, const bool need_mask,
                                             const int pos, const int kv_end, const int qpos,
                                             const int g, const float sl2, float& m, float& l,
                                             f32x4 (&acc)[16], u32x4& pf, u32x4& pl) {
  const float ninf = -__builtin_inff();
  float t[8];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    t[e] = s0[e] * sl2;
    t[4 + e] = s1[e] * sl2;
  }
  if (need_mask) {  // wave-uniform: only the last step of a split or the causal diagonal
    const int k0 = pos + 16 * (g >> 1) + 4 * (g & 1);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int ka = k0 + e, kb = k0 + 8 + e;
      t[e] = (ka < kv_end && ka <= qpos) ? t[e] : ninf;
      t[4 + e] = (kb < kv_end && kb <= qpos) ? t[4 + e] : ninf;
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])),
                   fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
  mx = row_max4(mx);
  const bool grow = mx > m + kGrow;   // also true for the first finite logit (m = -inf)
  if (__any(grow)) {
    const float m_new = grow ? mx : m;
    const float alpha = grow ? fast_exp2(m - m_new) : 1.f;   // m = -inf gives 0
    l *= alpha;
    // a wavefront whose rows have seen no finite logit yet (the first step of every work item)
    // holds zeros: scaling them changes nothing
    if (__any(m != ninf)) {
#pragma unroll
      for (int c = 0; c < 16; ++c) acc[c] *= alpha;
    }
    m = m_new;
  }
  const float m_use = (m == ninf) ? 0.f : m;
  float p[8], sum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    p[e] = fast_exp2(t[e] - m_use);
    sum += p[e];
  }
  l += sum;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    pf[i] = pack_bf16(p[2 * i], p[2 * i + 1]);
    pl[i] = pack_bf16(p[2 * i] - __uint_as_float(pf[i] << 16),
                      p[2 * i + 1] - __uint_as_float(pf[i] & 0xffff0000u));
  }
}

// Values of keys at or beyond kv_end may be stale bits (never-written slots, freed blocks):
// they are selected to zero, not multiplied by zero.  `left` = valid keys in this step.
__device__ __forceinline__ u32x4 value_mask(const int left, const int g) {
  const int k0 = 16 * (g >> 1) + 4 * (g & 1);
  u32x4 mask;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    mask[i] = (k0 + 2 * i < left ? 0xffffu : 0u) | (k0 + 2 * i + 1 < left ? 0xffff0000u : 0u);
    mask[2 + i] = (k0 + 8 + 2 * i < left ? 0xffffu : 0u) | (k0 + 8 + 2 * i + 1 < left ? 0xffff0000u : 0u);
  }
  return mask;
}


struct WorkItem {
  int n_tok, kv_begin, kv_end, q0, part_idx;
  const int32_t* tbl;
  int rec;   // this lane's word of the 32-word record (lanes 32..63 mirror 0..31)
};

// Block ids of the split, one per lane: the first 16 pages are words 16..31 of the record itself
// (no dependent load), all pages (a split has at most 64) come from the block table.  The table load is
// issued whether or not the split has more than 16 pages: a load under a condition would make
// the compiler wait for EVERYTHING in flight wherever the two paths meet again (it counts
// outstanding loads per control-flow path), and that wait would sit in front of the first pages.
struct SplitIds {
  int lo, hi;
};
__device__ __forceinline__ SplitIds split_block_ids(const WorkItem& wi, const int lane, const int npg) {
  SplitIds ids;
  ids.lo = wi.rec;
  ids.hi = wi.tbl[(wi.kv_begin >> 4) + (lane < npg ? lane : npg - 1)];
  return ids;
}
// pi is wave-uniform
__device__ __forceinline__ int block_of(const SplitIds& ids, const int pi) {
  return pi < kWorkInlinePages ? __builtin_amdgcn_readlane(ids.lo, 16 + pi)
                               : __builtin_amdgcn_readlane(ids.hi, pi);
}

// ---- tile path: <= 8 query tokens (64 rows); the four wavefronts share every KV page through
// LDS (double-buffered, one barrier per 32-key step) and own 16 rows each.
// kFresh: the keys are rows of this step's k_new / v_new (row0 + own position) instead of pool
// pages; they are brought into the same register image, so everything after the fetch is shared.
// The pool receives those rows from the merge launch of the same layer (nothing reads them from
// the pool during this launch, and the tiles are the last workgroups of a small launch to end).
template <bool kFresh>
__device__ __forceinline__ void tile_path(const AttnArgs& a, const WorkItem& wi, char* smem,
                                          const int row0) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int n = lane & 15, g = lane >> 4;
  const int ts = 2 * wv + (n >> 3), h = n & 7;
  const bool row_valid = ts < wi.n_tok;
  const bool wave_active = 2 * wv < wi.n_tok;
  // token ids sit in words 8..15 of the record: this wavefront's two, and the tile's first for
  // rows past its tokens (wave-uniform lane reads instead of a shuffle through LDS)
  const int tok_a = __builtin_amdgcn_readlane(wi.rec, 8 + 2 * wv);
  const int tok_b = __builtin_amdgcn_readlane(wi.rec, 9 + 2 * wv);
  const int tok_z = __builtin_amdgcn_readlane(wi.rec, 8);
  const int tok = row_valid ? ((n >> 3) ? tok_b : tok_a) : tok_z;
  const int qpos = wi.q0 + ts;
  // first partial slot of this wavefront's two tokens (words past the tile's tokens repeat its
  // last one): needed only at the end, loaded now (two scalar loads) so that the epilogue does
  // not wait for them
  const int part_a = a.part_off[tok_a] + wi.part_idx, part_b = a.part_off[tok_b] + wi.part_idx;
  u32x4 qf[8];
  float m = -__builtin_inff(), l = 0.f;
  f32x4 acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;
  const char* __restrict__ base = (const char*)a.layer_base;
  const int nsteps = (wi.kv_end - wi.kv_begin + 31) >> 5;

  // Each thread moves 8 x 16 B per step: K page A (2), K page B (2), V page A (2), V page B (2).
  // Two steps are kept in flight in registers on top of the step being computed from LDS.
  u32x4 st0[8], st1[8];
  // block ids of the whole split, one per lane (a split has at most 64 pages): fetched once,
  // then read with v_readlane, so no step waits on a scalar load before issuing its pages
  const int npg = ((wi.kv_end + 15) >> 4) - (wi.kv_begin >> 4);
  const SplitIds ids = split_block_ids(wi, lane, npg);
  // Every fetch issues exactly eight loads and no fetch is conditional: the compiler counts
  // outstanding loads per control-flow path, and a conditional load would make it wait for
  // everything at the next join.  A step past the end re-reads one hot 4 KiB (eight times the
  // same 16 B per thread); a missing page B re-reads page A.  Neither is ever used.
  // kFresh only: the V part of a step in two halves, so that the loads of several steps can be
  // issued before the first transpose waits for any of them.
  // r[e] = dims vdim..vdim+3 of key e of this thread's chunks (keys 4gp+e, then 8+4gp+e-4).
  typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
  auto fetch_fresh_k = [&](const int s, u32x4 (&st)[8]) {
    const int pos0 = wi.kv_begin + 32 * s, last = wi.kv_end - 1;
    const uint16_t* kn = (const uint16_t*)a.k_new + (size_t)row0 * kDim;
    const int kkey = ((tid >> 5) & 1) * 8 + (tid & 7);
    const int kdim = (tid >> 6) * 32 + ((tid >> 3) & 3) * 8;
#pragma unroll
    for (int pgi = 0; pgi < 2; ++pgi) {
      const uint16_t* ksrc = kn + (size_t)min(pos0 + 16 * pgi + kkey, last) * kDim + kdim;
      st[2 * pgi] = *(const u32x4*)ksrc;
      st[2 * pgi + 1] = *(const u32x4*)(ksrc + 128);
    }
  };
  auto fresh_v_load = [&](const int s, u32x2 (&r)[8]) {
    const uint16_t* vn = (const uint16_t*)a.v_new + (size_t)row0 * kDim;
    const int q = tid & 127, gp = (q >> 2) & 1, last = wi.kv_end - 1;
    const int vpos = wi.kv_begin + 32 * s + 16 * (tid >> 7) + 4 * gp;
    const int vdim = 16 * (q >> 3) + 4 * (q & 3);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      r[e] = *(const u32x2*)(vn + (size_t)min(vpos + (e < 4 ? e : e + 4), last) * kDim + vdim);
  };
  auto fresh_v_assemble = [&](const u32x2 (&r)[8], u32x4 (&st)[8]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {   // chunk j = dim vdim + j: halfword j of every key
      u32x4 c;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t lo = r[2 * w][j >> 1], hi = r[2 * w + 1][j >> 1];
        c[w] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
      st[4 + j] = c;
    }
  };
  auto fetch = [&](const int s, u32x4 (&st)[8]) {
    const bool real = s < nsteps;
    if constexpr (kFresh) {
      // K: thread tid holds chunks tid and tid+256 of each page as everywhere (a K chunk = 8 dims
      // of one key = one 16-byte load from the row).  V: a chunk is one dim of 8 keys, so here a
      // thread takes FOUR NEIGHBOURING chunks (dims d..d+3, same eight keys) of ONE page: eight
      // 8-byte loads and a 4x8 transpose in registers instead of thirty-two 2-byte gathers.
      // Thread tid: page tid / 128, chunks 4q..4q+3 with q = tid % 128 (see commit / sanitize).
      // Positions at or beyond the split's end re-read its last row; they are masked like stale
      // slots.  A step past the end loads nothing: the rows sit in L2 and a fresh tile has few
      // steps, so the wait that a conditional load costs is cheap.
      if (!real) return;
      fetch_fresh_k(s, st);
      u32x2 r[8];
      fresh_v_load(s, r);
      fresh_v_assemble(r, st);
      return;
    }
    const int pi = real ? 2 * s : 0;                      // page index inside the split
    const int o = real ? 1 : 0;
    const int blk_a = block_of(ids, pi);
    const int blk_b = block_of(ids, (real && pi + 1 < npg) ? pi + 1 : pi);
    const char* pa = base + (size_t)blk_a * kBlockBytes + tid * 16;
    const char* pb = base + (size_t)blk_b * kBlockBytes + tid * 16;
    st[0] = *(const u32x4*)(pa);
    st[1] = *(const u32x4*)(pa + o * 4096);
    st[2] = *(const u32x4*)(pb);
    st[3] = *(const u32x4*)(pb + o * 4096);
    st[4] = *(const u32x4*)(pa + o * kPageBytes);
    st[5] = *(const u32x4*)(pa + o * (kPageBytes + 4096));
    st[6] = *(const u32x4*)(pb + o * kPageBytes);
    st[7] = *(const u32x4*)(pb + o * (kPageBytes + 4096));
  };
  // Values of keys beyond the split's end are zero-selected once, on their way into LDS (only
  // the last step of a split can have any); the asm statement keeps this a real branch.
  // Thread tid holds V chunks tid and tid+256 of each page: chunk ci = (c, gp, m) with gp =
  // (ci >> 4) & 1, i.e. keys 4gp..4gp+3 and 8+4gp..8+4gp+3 of that page.
  auto sanitize = [&](const int s, u32x4 (&st)[8]) {
    const int left = wi.kv_end - (wi.kv_begin + 32 * s);
    if (s < nsteps && left < 32) {
      asm volatile("" ::: "memory");
      if constexpr (kFresh) {   // four chunks of page tid / 128, all with the same eight keys
        const int k0 = 16 * (tid >> 7) + 4 * (((tid & 127) >> 2) & 1);
        u32x4 mask;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          mask[i] = (k0 + 2 * i < left ? 0xffffu : 0u) | (k0 + 2 * i + 1 < left ? 0xffff0000u : 0u);
          mask[2 + i] = (k0 + 8 + 2 * i < left ? 0xffffu : 0u) | (k0 + 9 + 2 * i < left ? 0xffff0000u : 0u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) st[4 + j] &= mask;
        return;
      }
      const int gp = (tid >> 4) & 1;
#pragma unroll
      for (int pgi = 0; pgi < 2; ++pgi) {
        const int k0 = 16 * pgi + 4 * gp;
        u32x4 mask;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          mask[i] = (k0 + 2 * i < left ? 0xffffu : 0u) | (k0 + 2 * i + 1 < left ? 0xffff0000u : 0u);
          mask[2 + i] = (k0 + 8 + 2 * i < left ? 0xffffu : 0u) | (k0 + 9 + 2 * i < left ? 0xffff0000u : 0u);
        }
        st[4 + 2 * pgi] &= mask;
        st[5 + 2 * pgi] &= mask;
      }
    }
  };
  auto commit = [&](const int stage, const u32x4 (&st)[8]) {
    char* dst = smem + stage * kStageBytes + tid * 16;
    *(u32x4*)(dst + kOffKA) = st[0];
    *(u32x4*)(dst + kOffKA + 4096) = st[1];
    *(u32x4*)(dst + kOffKB) = st[2];
    *(u32x4*)(dst + kOffKB + 4096) = st[3];
    if constexpr (kFresh) {   // chunks 4q..4q+3 of page tid / 128
      char* vd = smem + stage * kStageBytes + ((tid >> 7) ? kOffVB : kOffVA) + (tid & 127) * 64;
#pragma unroll
      for (int j = 0; j < 4; ++j) *(u32x4*)(vd + j * 16) = st[4 + j];
      return;
    }
    *(u32x4*)(dst + kOffVA) = st[4];
    *(u32x4*)(dst + kOffVA + 4096) = st[5];
    *(u32x4*)(dst + kOffVB) = st[6];
    *(u32x4*)(dst + kOffVB + 4096) = st[7];
  };
  // per-lane LDS offsets of this lane's operands: K of key n%8 in page n/8, V of page g/2
  const int lds_k = ((n >> 3) ? kOffKB : kOffKA) + (g * 8 + (n & 7)) * 16;
  const int lds_v = ((g >> 1) ? kOffVB : kOffVA) + ((g & 1) * 16 + n) * 16;
  auto compute = [&](const int s) {
    const int pos = wi.kv_begin + 32 * s;
    const int left = wi.kv_end - pos;
    const char* sk = smem + (s & 1) * kStageBytes;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      s0 = mfma16(*(const u32x4*)(sk + lds_k + j * 1024), qf[j], s0);
      s1 = mfma16(*(const u32x4*)(sk + lds_k + j * 1024 + 512), qf[j], s1);
    }
    // eight operand reads ahead of the products: left to itself the compiler keeps two in
    // flight, and every product then waits a full LDS round trip
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    u32x4 pf, pl;
    softmax_step(s0, s1, left < 32 || pos + 31 > wi.q0, pos, wi.kv_end, qpos, g, sl2, m, l, acc,
                 pf, pl);
#pragma unroll
    for (int c = 0; c < 16; ++c) {   // V was sanitised on its way into LDS
      const u32x4 v = *(const u32x4*)(sk + lds_v + c * 512);
      acc[c] = mfma16(v, pl, mfma16(v, pf, acc[c]));
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 1);   // as above: eight reads ahead
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 1);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 16, 1);
  };
  // body(s, cur, nxt): cur's content (step s) already sits in LDS, nxt holds step s+1 in
  // flight.  The scheduling barriers keep the order "issue s+2, compute s, then wait for s+1",
  // otherwise the wait would be hoisted above the compute.
  auto body = [&](const int s, u32x4 (&cur)[8], u32x4 (&nxt)[8]) {
    fetch(s + 2, cur);
    __builtin_amdgcn_sched_barrier(0);
    if (wave_active && s < nsteps) compute(s);
    __builtin_amdgcn_sched_barrier(0);
    if (s + 1 < nsteps) {   // after the last step only the barrier is left: the epilogue reuses LDS
      sanitize(s + 1, nxt);
      commit((s + 1) & 1, nxt);
    }
    __syncthreads();
  };
  auto load_q = [&]() {
    const char* qrow = (const char*)a.q + ((size_t)tok * kHeads + h) * (kDim * 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      // unconditional (a row past the tile's tokens re-reads its last token's row, see `tok`)
      // and zeroed afterwards: see split_block_ids for why no load sits under a condition
      const u32x4 z = {0, 0, 0, 0};
      const u32x4 x = *(const u32x4*)(qrow + j * 64 + g * 16);
      qf[j] = row_valid ? x : z;
    }
  };
  if constexpr (kFresh) {
    // Step 0 first: its rows have to pass through the transpose, LDS and a barrier before the
    // first product, the query rows only have to be in registers by then.  Every load of steps
    // 0 and 1 goes out before the first transpose waits for its rows.
    u32x2 r0[8], r1[8];
    fetch_fresh_k(0, st0);
    fresh_v_load(0, r0);
    __builtin_amdgcn_sched_barrier(0);
    load_q();
    __builtin_amdgcn_sched_barrier(0);
    if (nsteps > 1) {
      fetch_fresh_k(1, st1);
      fresh_v_load(1, r1);
    }
    __builtin_amdgcn_sched_barrier(0);
    fresh_v_assemble(r0, st0);
    if (nsteps > 1) fresh_v_assemble(r1, st1);
  } else {
    // the query rows are requested first: loads complete in order per wavefront, and the
    // first product should wait for step 0 only, not for step 1 as well
    load_q();
    __builtin_amdgcn_sched_barrier(0);
    fetch(0, st0);
    fetch(1, st1);
  }
  __builtin_amdgcn_sched_barrier(0);
  sanitize(0, st0);
  commit(0, st0);
  __syncthreads();
  for (int s = 0; s < nsteps; s += 2) {   // steps in pairs: the two register stages swap roles
    body(s, st0, st1);
    if (s + 1 < nsteps) body(s + 1, st1, st0);
  }
  l = row_sum4(l);
  // The partial leaves as (m, l, scale, acc / scale in fp16): half the bytes of fp32, and the
  // per-row scale (max |acc| of the row) keeps it independent of the magnitude of the values.
  float amax = 0.f;
#pragma unroll
  for (int c = 0; c < 16; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) amax = fmaxf(amax, fabsf(acc[c][e]));
  amax = row_max4(amax);
  const float inv = amax > 0.f ? 1.f / amax : 0.f;
  // Each lane holds 4-dim pieces of its row; written as they are, a store would touch 16 rows
  // with 32 bytes each.  The rows go through LDS instead (the stages are free after the loop's
  // last barrier; every wavefront uses a region of its own, so no barrier is needed) and leave
  // as whole rows: 32 lanes x 16 bytes per row.
  typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
  char* ep = smem + wv * (16 * kEpilogueStride);
#pragma unroll
  for (int c = 0; c < 16; ++c) {
    const u32x2 v = {pack_f16(acc[c][0] * inv, acc[c][1] * inv),
                     pack_f16(acc[c][2] * inv, acc[c][3] * inv)};
    *(u32x2*)(ep + n * kEpilogueStride + (16 * c + 4 * g) * 2) = v;
  }
  asm volatile("" ::: "memory");   // the reads below are of another type: keep them behind the writes
  const int slot_lane = (n >> 3) ? part_b : part_a;   // of this lane's row n
  if (row_valid && g == 0)
    *(f32x4*)(a.part_ml + ((size_t)slot_lane * kHeads + h) * 4) = (f32x4){m, l, amax, 0.f};
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = 2 * it + (lane >> 5);              // row of this wavefront's 16
    const int slot_row = (it >> 2) ? part_b : part_a;  // rows 0..7: first token, 8..15: second
    const u32x4 v = *(const u32x4*)(ep + row * kEpilogueStride + (lane & 31) * 16);
    if (2 * wv + (row >> 3) < wi.n_tok)
      *(u32x4*)(a.part_acc + ((size_t)slot_row * kHeads + (row & 7)) * kDim + (lane & 31) * 8) = v;
  }
}

// ---- stream path: <= 2 query tokens (16 rows, the decode case).  Nothing is shared, so the
// four wavefronts take the 32-key steps of the split round-robin, stream their pages straight
// into registers one step ahead, and combine their four results through LDS.
// kOwnPages: the key range lies in the item's own pages, which no other workgroup of the launch
// reads (and which receive the item's new rows when the append is folded in); otherwise the
// pages are a prefix's and other workgroups read them too.
template <bool kOwnPages>
__device__ __forceinline__ void stream_path(const AttnArgs& a, const WorkItem& wi, char* smem,
                                            float (*sml)[16][2], char* qs) {
  constexpr bool appends = kOwnPages;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int n = lane & 15, g = lane >> 4;
  const int ts = n >> 3, h = n & 7;
  const bool row_valid = ts < wi.n_tok;
  const int tok_a = __builtin_amdgcn_readlane(wi.rec, 8), tok_b = __builtin_amdgcn_readlane(wi.rec, 9);
  const int tok = (row_valid && ts) ? tok_b : tok_a;
  const int qpos = wi.q0 + ts;
  // In the epilogue thread tid writes 16 dims of row tid / 16; the first partial slot of that
  // row's token is loaded now so that the epilogue does not wait for it.
  const int otok = ((wv >> 1) && wi.n_tok > 1) ? tok_b : tok_a;
  const int part_base = a.part_off[otok];
  float m = -__builtin_inff(), l = 0.f;
  f32x4 acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;
  const char* __restrict__ base = (const char*)a.layer_base;
  const int nsteps = (wi.kv_end - wi.kv_begin + 31) >> 5;

  u32x4 kr[16], vr[16];   // kr[2j+hf]: K chunk of (j, hf); vr[c]: V chunk of block c
  const int npg = ((wi.kv_end + 15) >> 4) - (wi.kv_begin >> 4);
  const SplitIds ids = split_block_ids(wi, lane, npg);
  const int lane_k = (g * 8 + (n & 7)) * 16;
  const int lane_v = kPageBytes + ((g & 1) * 16 + n) * 16;
  // A wavefront has at most one step in flight beyond the one it computes, and it waits for all
  // of it before the next product, so (unlike the tile path) nothing is lost when the load of
  // a step past the end is simply skipped; a missing page B re-reads page A and is masked.
  // Own pages are read once per launch, by this workgroup alone: their loads carry the
  // non-temporal hint, so that they do not push the pages that other workgroups share out of
  // the L2.
  auto page_load = [](const char* p) {
    if constexpr (kOwnPages) return __builtin_nontemporal_load((const u32x4*)p);
    return *(const u32x4*)p;
  };
  auto load_k_at = [&](const int s) {
    const int pi = 2 * s;
    const int blk_a = block_of(ids, pi);
    const int blk_b = block_of(ids, pi + 1 < npg ? pi + 1 : pi);
    const char* p = base + (size_t)((n >> 3) ? blk_b : blk_a) * kBlockBytes + lane_k;
#pragma unroll
    for (int i = 0; i < 16; ++i) kr[i] = page_load(p + i * 512);
  };
  auto load_v_at = [&](const int s) {
    const int pi = 2 * s;
    const int blk_a = block_of(ids, pi);
    const int blk_b = block_of(ids, pi + 1 < npg ? pi + 1 : pi);
    const char* p = base + (size_t)((g >> 1) ? blk_b : blk_a) * kBlockBytes + lane_v;
#pragma unroll
    for (int c = 0; c < 16; ++c) vr[c] = page_load(p + c * 512);
  };
  auto load_k = [&](const int s) {
    if (s < nsteps) load_k_at(s);
  };
  auto load_v = [&](const int s) {
    if (s < nsteps) load_v_at(s);
  };
  // Folded append: the query tokens of a streaming item are its new rows.  Those inside this
  // split's key range are written to the pool by this workgroup (no other workgroup reads
  // them in this launch), and a workgroup barrier orders the writes before the page loads that
  // cover them.  The first new row sits in step `first_new`: when that step is loaded after the
  // barrier below anyway, the stores wait there; otherwise they go out, with a barrier of their
  // own, before the first page load.
  RowPart rows[2];
  int32_t slot2 = 0;   // lane j % 2: pool slot of the record's token j
  bool row_mine[2] = {false, false};
  bool early = false;
  const bool fold = a.k_new && appends;
  if (fold) {
    const int pos0 = (wi.q0 == kNoCausal ? 0 : wi.q0);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int pos = pos0 + t;
      row_mine[t] = t < wi.n_tok && pos >= wi.kv_begin && pos < wi.kv_end;
      const int tk = __builtin_amdgcn_readlane(wi.rec, 8 + t);
      rows[t] = load_row((const uint16_t*)a.k_new + (size_t)tk * kDim,
                         (const uint16_t*)a.v_new + (size_t)tk * kDim, tid);
    }
    slot2 = a.d_slots[(lane & 1) ? tok_b : tok_a];   // one load per lane, read with v_readlane
    const int first_new = (max(pos0, wi.kv_begin) - wi.kv_begin) >> 5;
    early = first_new < 4;
    if (early) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
        if (row_mine[t])
          store_row(rows[t], __builtin_amdgcn_readlane(slot2, t), (char*)a.layer_base, tid);
      __syncthreads();
    }
  }
  // The 16 query rows are the same for all four wavefronts: their MFMA fragments live in LDS
  // (registers are needed for the pages in flight).  The query loads are issued BEFORE the first
  // pages: loads complete in order per wavefront, so the barrier below then waits for the
  // queries only, not for the slowest wavefront's first 32 KiB.
  u32x4 qtmp[2];
  {
    const char* qrow = (const char*)a.q + ((size_t)tok * kHeads + h) * (kDim * 2);
    const u32x4 z = {0, 0, 0, 0};
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {   // unconditional, zeroed afterwards (see split_block_ids)
      const u32x4 x = *(const u32x4*)(qrow + (2 * wv + jj) * 64 + g * 16);
      qtmp[jj] = row_valid ? x : z;
    }
  }
  int s = wv;
  // The first step's loads are unconditional as well: a wavefront without a step of its own
  // (a split of fewer than four steps) re-reads the split's last step and never uses it.  With
  // the number of loads in flight known, the store of the queries below waits for the queries
  // only, and the barrier after it no longer ties the four wavefronts to the slowest first step.
  load_k_at(s < nsteps ? s : nsteps - 1);
  load_v_at(s < nsteps ? s : nsteps - 1);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) *(u32x4*)(qs + (2 * wv + jj) * 1024 + lane * 16) = qtmp[jj];
  if (fold && !early) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (row_mine[t])
        store_row(rows[t], __builtin_amdgcn_readlane(slot2, t), (char*)a.layer_base, tid);
  }
  __syncthreads();
  const char* qf = qs + lane * 16;
  for (; s < nsteps; s += 4) {
    const int pos = wi.kv_begin + 32 * s;
    const int left = wi.kv_end - pos;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32x4 q = *(const u32x4*)(qf + j * 1024);
      s0 = mfma16(kr[2 * j], q, s0);
      s1 = mfma16(kr[2 * j + 1], q, s1);
    }
    // four query reads ahead of the products (see the tile path)
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 2);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 2);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 2);
    u32x4 pf, pl;
    softmax_step(s0, s1, left < 32 || pos + 31 > wi.q0, pos, wi.kv_end, qpos, g, sl2, m, l, acc,
                 pf, pl);
    __builtin_amdgcn_sched_barrier(0);  // the next K pages reuse kr[]: issue only after S
    load_k(s + 4);
    __builtin_amdgcn_sched_barrier(0);
    if (left < 32) {   // wave-uniform; only the last step of a split (asm: keep it a branch)
      asm volatile("" ::: "memory");
      const u32x4 mask = value_mask(left, g);
#pragma unroll
      for (int c = 0; c < 16; ++c) vr[c] &= mask;
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] = mfma16(vr[c], pl, mfma16(vr[c], pf, acc[c]));
    __builtin_amdgcn_sched_barrier(0);  // likewise vr[]
    load_v(s + 4);
    __builtin_amdgcn_sched_barrier(0);
  }
  l = row_sum4(l);
  // combine the four wavefronts' results (log-sum-exp rule) and write one partial
  float* sm = (float*)smem;
#pragma unroll
  for (int c = 0; c < 16; ++c)
    *(f32x4*)(sm + (wv * 16 + n) * kMergeStride + 16 * c + 4 * g) = acc[c];
  if (g == 0) {
    sml[wv][n][0] = m;
    sml[wv][n][1] = l;
  }
  __syncthreads();
  // thread tid: row tid / 16, dims [8t, 8t+8) and [128+8t, 128+8t+8) with t = tid % 16, so that
  // the 16 threads of a row write 256 contiguous bytes per store
  const int r = tid >> 4, seg = (tid & 15) * 8;
  if ((r >> 3) < wi.n_tok) {
    const float ninf = -__builtin_inff();
    float big = ninf;
#pragma unroll
    for (int w = 0; w < 4; ++w) big = fmaxf(big, sml[w][r][0]);
    float wgt[4], total = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      wgt[w] = (sml[w][r][0] == ninf) ? 0.f : fast_exp2(sml[w][r][0] - big);
      total = __builtin_fmaf(wgt[w], sml[w][r][1], total);
    }
    const size_t slot = (size_t)part_base + wi.part_idx;
    uint16_t* dst = a.part_acc + (slot * kHeads + (r & 7)) * kDim + seg;
    f32x4 o[4];
    float amax = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int d = seg + 4 * (q & 1) + 128 * (q >> 1);
      o[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const f32x4 x = *(const f32x4*)(sm + (w * 16 + r) * kMergeStride + d);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[q][e] = __builtin_fmaf(wgt[w], x[e], o[q][e]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) amax = fmaxf(amax, fabsf(o[q][e]));
    }
    // row scale over the 16 threads that hold this row (the branch is uniform per wavefront)
    amax = lanes16_max(amax);
    const float inv = amax > 0.f ? 1.f / amax : 0.f;
    const u32x4 lo = {pack_f16(o[0][0] * inv, o[0][1] * inv), pack_f16(o[0][2] * inv, o[0][3] * inv),
                      pack_f16(o[1][0] * inv, o[1][1] * inv), pack_f16(o[1][2] * inv, o[1][3] * inv)};
    const u32x4 hi = {pack_f16(o[2][0] * inv, o[2][1] * inv), pack_f16(o[2][2] * inv, o[2][3] * inv),
                      pack_f16(o[3][0] * inv, o[3][1] * inv), pack_f16(o[3][2] * inv, o[3][3] * inv)};
    *(u32x4*)(dst) = lo;
    *(u32x4*)(dst + 128) = hi;
    if ((tid & 15) == 0)
      *(f32x4*)(a.part_ml + (slot * kHeads + (r & 7)) * 4) = (f32x4){big, total, amax, 0.f};
  }
}

__global__ __launch_bounds__(256, 2) void attn_kernel(const AttnArgs a) {
  __shared__ __align__(16) char smem[kSmemBytes];
  __shared__ float sml[4][16][2];
  __shared__ __align__(16) char qs[16 * kDim * 2];
  // one 128-byte load brings the whole record; its fields are read out lane-wise
  WorkItem wi;
  wi.rec = a.work[(size_t)blockIdx.x * kWorkWords + (threadIdx.x & 31)];
  wi.n_tok = __builtin_amdgcn_readlane(wi.rec, W_N_TOK);
  wi.tbl = a.tables + __builtin_amdgcn_readlane(wi.rec, W_TBL_OFF);
  wi.kv_begin = __builtin_amdgcn_readlane(wi.rec, W_KV_BEGIN);
  wi.kv_end = __builtin_amdgcn_readlane(wi.rec, W_KV_END);
  wi.q0 = __builtin_amdgcn_readlane(wi.rec, W_CAUSAL_Q0);
  wi.part_idx = __builtin_amdgcn_readlane(wi.rec, W_PART_IDX);
  const int path_word = __builtin_amdgcn_readlane(wi.rec, W_PATH);
  const int path = path_word & kPathMask;
  if (path == PATH_TILE) {
    __builtin_amdgcn_s_setprio(2);   // compute-heavy: issue ahead of co-resident streaming waves
    if (a.k_new && (path_word & kPathFresh))
      tile_path<true>(a, wi, smem, path_word >> kPathRowShift);
    else
      tile_path<false>(a, wi, smem, 0);
  } else if (path == PATH_STREAM) {
    if (path_word & kPathAppends)
      stream_path<true>(a, wi, smem, sml, qs);
    else
      stream_path<false>(a, wi, smem, sml, qs);
  } else {
    return;   // padding record
  }
}

// ------------------------------------------------------------------------------------------
// merge of a query token's partials (log-sum-exp rule).  One workgroup per token; a thread owns
// eight consecutive output dims of one head and has every load of the first sixteen partials in
// flight at once.
// (A merge fused into attn_kernel by "last arriver merges" was built twice and measured: with
// device-scope fences every workgroup pays a whole-L2 write-back + invalidate (165 us per
// launch); with scoped write-through stores and no fences it is correct and fence-free, but the
// tile workgroups finish last and then merge their eight tokens serially (53 us).  Hence its own
// kernel.)
// ------------------------------------------------------------------------------------------
constexpr int kMergeAhead = 16;   // partials whose loads are all issued before anything is used

// One workgroup per token; thread t owns head t/32 and eight consecutive output dims.
__device__ __forceinline__ void merge_block(const AttnArgs& a, const int tok) {
  const int t = threadIdx.x;
  const int h = t >> 5, d0 = (t & 31) * 8;
  const int np = a.n_parts[tok];
  const size_t base = (size_t)a.part_off[tok];
  const float* ml = a.part_ml + (base * kHeads + h) * 4;
  const uint16_t* src = a.part_acc + (base * kHeads + h) * kDim + d0;
  const size_t stride = (size_t)kHeads * kDim;
  const float ninf = -__builtin_inff();
  // one round trip for the common case: every load of the first 16 partials is in flight at once
  u32x4 x[kMergeAhead];
  f32x4 w[kMergeAhead];
#pragma unroll
  for (int u = 0; u < kMergeAhead; ++u) {
    const int p = u < np ? u : 0;
    x[u] = *(const u32x4*)(src + (size_t)p * stride);
    w[u] = *(const f32x4*)(ml + (size_t)p * kHeads * 4);
  }
  float big = ninf;
#pragma unroll
  for (int u = 0; u < kMergeAhead; ++u) big = fmaxf(big, u < np ? w[u][0] : ninf);
  for (int p = kMergeAhead; p < np; ++p) big = fmaxf(big, ml[(size_t)p * kHeads * 4]);
  float total = 0.f;
  float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto add = [&](const f32x4& mls, const u32x4& v) {   // mls = (m, l, scale, -)
    const float wgt = (mls[0] == ninf) ? 0.f : fast_exp2(mls[0] - big);
    total = __builtin_fmaf(wgt, mls[1], total);
    const float ws = wgt * mls[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float lo, hi;
      unpack_f16(v[i], lo, hi);
      o[2 * i] = __builtin_fmaf(ws, lo, o[2 * i]);
      o[2 * i + 1] = __builtin_fmaf(ws, hi, o[2 * i + 1]);
    }
  };
#pragma unroll
  for (int u = 0; u < kMergeAhead; ++u)
    if (u < np) add(w[u], x[u]);
  for (int p = kMergeAhead; p < np; ++p)
    add(*(const f32x4*)(ml + (size_t)p * kHeads * 4), *(const u32x4*)(src + (size_t)p * stride));
  const float inv = 1.f / total;
  const u32x4 packed = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv),
                        pack_bf16(o[4] * inv, o[5] * inv), pack_bf16(o[6] * inv, o[7] * inv)};
  *(u32x4*)((uint16_t*)a.out + ((size_t)tok * kHeads + h) * kDim + d0) = packed;
  if (a.lse && (t & 31) == 0)
    a.lse[(size_t)tok * kHeads + h] = (big + __builtin_amdgcn_logf(total)) * 0.6931471805599453f;
}

__global__ __launch_bounds__(256) void merge_kernel(const AttnArgs a) { merge_block(a, blockIdx.x); }

// merge of one layer and, in the same launch, an append that touches other memory than the
// merge: the next layer's new rows (cross-layer fusion), or this layer's rows of the items whose
// tiles read their keys from k_new / v_new (nx.tok_list names their tokens)
__global__ __launch_bounds__(256) void merge_append_kernel(const AttnArgs a, const AppendArgs nx) {
  const int n_merge = a.n_q;
  if ((int)blockIdx.x < n_merge) {
    merge_block(a, blockIdx.x);
  } else {
    const int i = blockIdx.x - n_merge;
    const int tok = nx.tok_list ? nx.tok_list[i] : i;
    append_row((const uint16_t*)nx.k_new + (size_t)tok * kDim,
               (const uint16_t*)nx.v_new + (size_t)tok * kDim, nx.d_slots[tok],
               (char*)nx.layer_base, threadIdx.x);
  }
}

hipError_t launch_attention_work(const AttnArgs& a, hipStream_t s, hipEvent_t start,
                                 hipEvent_t stop) {
  if (a.n_work <= 0 || a.n_q <= 0) return hipErrorInvalidValue;
  if (start || stop)
    hipExtLaunchKernelGGL(attn_kernel, dim3(a.n_work), dim3(256), 0, s, start, stop, 0, a);
  else
    attn_kernel<<<a.n_work, 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_merge_append(const AttnArgs& a, const AppendArgs* next, hipStream_t s,
                               hipEvent_t start, hipEvent_t stop) {
  if (a.n_q <= 0) return hipErrorInvalidValue;
  const bool timed = start || stop;
  if (next && next->n_tokens > 0) {
    const dim3 grid(a.n_q + next->n_tokens);
    if (timed)
      hipExtLaunchKernelGGL(merge_append_kernel, grid, dim3(256), 0, s, start, stop, 0, a, *next);
    else
      merge_append_kernel<<<grid, 256, 0, s>>>(a, *next);
  } else {
    if (timed)
      hipExtLaunchKernelGGL(merge_kernel, dim3(a.n_q), dim3(256), 0, s, start, stop, 0, a);
    else
      merge_kernel<<<a.n_q, 256, 0, s>>>(a);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Split results in static device memory, for callers that cannot allocate (see
// oxy_mixed_attention_static in oxy.h).  Every GPU the library runs on holds its own copy of
// the array, at its own address, until the process ends; that address is looked up once per
// device, with the device current, and is what host code passes on from then.
// ------------------------------------------------------------------------------------------
constexpr size_t kStaticAccBytes = (size_t)kStaticMaxPartials * kHeads * kDim * sizeof(uint16_t);
constexpr size_t kStaticMlBytes = (size_t)kStaticMaxPartials * kHeads * 4 * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kStaticAccBytes + kStaticMlBytes];

hipError_t static_scratch(uint16_t** part_acc, float** part_ml) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    ptr_of_device[dev] = ptr;
  }
  *part_acc = (uint16_t*)ptr_of_device[dev];
  *part_ml = (float*)((char*)ptr_of_device[dev] + kStaticAccBytes);
  return hipSuccess;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  hipError_t e = launch_attention_work(a, s);
  if (e != hipSuccess) return e;
  return launch_merge_append(a, nullptr, s);
}

}  // namespace oxy
