// HIP kernels for gfx950 (MI355X): KV append / gather and the mixed-mask paged attention.
//
// What is computed is the attention inside the paper's ActionDenoise and
// BatchedLanguageDecode passes (App. A.1, Eq. 5-6) for queries of several tasks at once,
// all reading one shared prefill cache (Sec. 3.2, cross-task KV sharing) plus their own
// tokens.  Visibility: prefix always; own tokens causally for decode queries, all of the
// chunk for action queries.
//
// Evaluation scheme.  The visible set of a query is cut into (prefix | own) and each part
// into fixed-size splits.  A work item is (<=16 query rows that share one KV source, one
// split of that source); it yields an un-normalised partial (running max m in the log2
// domain, sum l, accumulator acc[256]).  A second kernel merges a query's partials by the
// log-sum-exp rule.  Because the split size is fixed per pool, the arithmetic of a query
// never depends on what else is in the batch.
//
// MFMA mapping (v_mfma_f32_16x16x32_bf16, lane = 16*g + n):
//   S^T[key][row]  = sum_d K[key][d] * Q[row][d]      A = K page chunk, B = Q rows
//       -> lane (n = row, g) receives keys 4g..4g+3 of the page
//   O^T[d][row]   += sum_key V[key][d] * P[row][key]  A = V chunk, B = P
//       -> lane (n = row, g) accumulates d = 16c+4g..4g+3
// Both results keep "row = lane % 16", so the softmax state (m, l, rescale factor) is a
// per-lane scalar and P feeds the second product without any cross-lane movement.  The
// pool pages are stored in exactly the operand order these products want (see oxy.h), so
// every wave-wide load is one contiguous KiB.
#include "oxy_internal.h"

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

// ------------------------------------------------------------------------------------------
// append / gather
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void append_row(const uint16_t* __restrict__ k_row,
                                           const uint16_t* __restrict__ v_row, int32_t slot,
                                           char* __restrict__ layer_base, int t) {
  const int blk = slot >> 4, key = slot & 15;
  char* kp = layer_base + (size_t)blk * kBlockBytes;
  char* vp = kp + kPageBytes;
  if (t < 32) *(u32x4*)(kp + (t * 16 + key) * 16) = *(const u32x4*)(k_row + t * 8);
  const int d = t, c = d >> 5, hi = (d >> 4) & 1, m = d & 15, g = key >> 2, e = key & 3;
  *(uint16_t*)(vp + ((c * 4 + g) * 16 + m) * 16 + hi * 8 + e * 2) = v_row[d];
}

__global__ __launch_bounds__(256) void append_kernel(const uint16_t* __restrict__ k_new,
                                                     const uint16_t* __restrict__ v_new,
                                                     const int32_t* __restrict__ slots,
                                                     char* __restrict__ layer_base) {
  const int tok = blockIdx.x;
  append_row(k_new + (size_t)tok * kDim, v_new + (size_t)tok * kDim, slots[tok], layer_base,
             threadIdx.x);
}

__global__ __launch_bounds__(256) void append_inline_kernel(const uint16_t* __restrict__ k_new,
                                                            const uint16_t* __restrict__ v_new,
                                                            const InlineIds blocks, int32_t pos0,
                                                            char* __restrict__ layer_base) {
  const int tok = blockIdx.x;
  const int pos = pos0 + tok;
  append_row(k_new + (size_t)tok * kDim, v_new + (size_t)tok * kDim,
             blocks.v[pos >> 4] * kPage + (pos & 15), layer_base, threadIdx.x);
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
  if (t < 32) *(u32x4*)(k_out + (size_t)tok * kDim + t * 8) = *(const u32x4*)(kp + (t * 16 + key) * 16);
  const int d = t, c = d >> 5, hi = (d >> 4) & 1, m = d & 15, g = key >> 2, e = key & 3;
  v_out[(size_t)tok * kDim + d] =
      *(const uint16_t*)(vp + ((c * 4 + g) * 16 + m) * 16 + hi * 8 + e * 2);
}

hipError_t launch_append(const void* k_new, const void* v_new, const int32_t* d_slots,
                         int32_t n_tokens, void* layer_base, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  append_kernel<<<n_tokens, 256, 0, s>>>((const uint16_t*)k_new, (const uint16_t*)v_new, d_slots,
                                         (char*)layer_base);
  return hipGetLastError();
}

hipError_t launch_append_inline(const void* k_new, const void* v_new, const InlineIds& blocks,
                                int32_t pos0, int32_t n_tokens, void* layer_base, hipStream_t s) {
  if (n_tokens <= 0) return hipSuccess;
  append_inline_kernel<<<n_tokens, 256, 0, s>>>((const uint16_t*)k_new, (const uint16_t*)v_new,
                                                blocks, pos0, (char*)layer_base);
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
constexpr int kStageBytes = 4 * kPageBytes;          // K page A, K page B, V page A, V page B
constexpr int kMergeStride = kDim + 4;               // floats per row in the LDS merge buffer
constexpr int kSmemBytes = 4 * 16 * kMergeStride * 4;  // >= 2 * kStageBytes

// One 32-key step of the online softmax for the 16 rows of a wavefront.  sa/sb hold the raw
// dot products of this lane's row with keys pos+4g+e (page A) and pos+16+4g+e (page B).
// Updates the running max m (log2 domain), the lane-partial sum l and rescales acc; returns P
// as hi+lo bf16 (a single bf16 rounding of P, 2^-9 relative, is too coarse for queries that see
// only a handful of keys).
__device__ __forceinline__ void softmax_step(const f32x4 sa, const f32x4 sb, const bool has_b,
                                             const int pos, const int kv_end, const int qpos,
                                             const int g, const float sl2, float& m, float& l,
                                             f32x4 (&acc)[16], u32x4& pf, u32x4& pl) {
  const float ninf = -__builtin_inff();
  float s[8];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int ka = pos + 4 * g + e, kb = ka + 16;
    s[e] = (ka < kv_end && ka <= qpos) ? sa[e] * sl2 : ninf;
    s[4 + e] = (has_b && kb < kv_end && kb <= qpos) ? sb[e] * sl2 : ninf;
  }
  float mx = s[0];
#pragma unroll
  for (int e = 1; e < 8; ++e) mx = fmaxf(mx, s[e]);
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  const float m_use = (m_new == ninf) ? 0.f : m_new;
  const float alpha = fast_exp2(m - m_use);
  float p[8], sum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    p[e] = fast_exp2(s[e] - m_use);
    sum += p[e];
  }
  l = l * alpha + sum;
  m = m_new;
  if (__any(alpha != 1.f)) {
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] *= alpha;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    pf[i] = pack_bf16(p[2 * i], p[2 * i + 1]);
    pl[i] = pack_bf16(p[2 * i] - __uint_as_float(pf[i] << 16),
                      p[2 * i + 1] - __uint_as_float(pf[i] & 0xffff0000u));
  }
}

// Values of keys at or beyond kv_end may be stale bits (never-written slots, freed blocks):
// they are selected to zero, not multiplied by zero.
__device__ __forceinline__ void value_masks(const int left, const int g, uint32_t (&mask)[4]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int k0 = 4 * g + 2 * i;
    mask[i] = (k0 < left ? 0xffffu : 0u) | (k0 + 1 < left ? 0xffff0000u : 0u);
    mask[2 + i] = (k0 + 16 < left ? 0xffffu : 0u) | (k0 + 17 < left ? 0xffff0000u : 0u);
  }
}

__device__ __forceinline__ void pv_block(f32x4 (&acc)[16], const int c, u32x4 va, u32x4 vb,
                                         const uint32_t (&mask)[4], const bool masked,
                                         const u32x4 pf, const u32x4 pl) {
  if (masked) {
    va[0] &= mask[0]; va[1] &= mask[1]; va[2] &= mask[0]; va[3] &= mask[1];
    vb[0] &= mask[2]; vb[1] &= mask[3]; vb[2] &= mask[2]; vb[3] &= mask[3];
  }
  const u32x4 v0 = {va[0], va[1], vb[0], vb[1]};
  const u32x4 v1 = {va[2], va[3], vb[2], vb[3]};
  acc[2 * c] = mfma16(v0, pl, mfma16(v0, pf, acc[2 * c]));
  acc[2 * c + 1] = mfma16(v1, pl, mfma16(v1, pf, acc[2 * c + 1]));
}

struct WorkItem {
  int tok_off, n_tok, kv_begin, kv_end, q0, part_idx;
  const int32_t* tbl;
};

// ---- tile path: <= 8 query tokens (64 rows); the four wavefronts share every KV page through
// LDS (double-buffered, one barrier per 32-key step) and own 16 rows each.
__device__ __forceinline__ void tile_path(const AttnArgs& a, const WorkItem& wi, char* smem) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int n = lane & 15, g = lane >> 4;
  const int ts = 2 * wv + (n >> 3), h = n & 7;
  const bool row_valid = ts < wi.n_tok;
  const bool wave_active = 2 * wv < wi.n_tok;
  const int tok = row_valid ? a.tok_list[wi.tok_off + ts] : 0;
  const int qpos = wi.q0 + ts;
  u32x4 qf[8];
  {
    const char* qrow = (const char*)a.q + ((size_t)tok * kHeads + h) * (kDim * 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32x4 z = {0, 0, 0, 0};
      qf[j] = row_valid ? *(const u32x4*)(qrow + j * 64 + g * 16) : z;
    }
  }
  float m = -__builtin_inff(), l = 0.f;
  f32x4 acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;
  const char* __restrict__ base = (const char*)a.layer_base;
  const int nsteps = (wi.kv_end - wi.kv_begin + 31) >> 5;

  // Each thread moves 8 x 16 B per step: K page A (2), K page B (2), V page A (2), V page B (2).
  // Two steps are kept in flight in registers on top of the step being computed from LDS, so a
  // workgroup has up to 64 KiB outstanding and a split costs about half as many memory
  // latencies as it has steps.
  u32x4 st0[8], st1[8];
  auto fetch = [&](const int s, u32x4 (&st)[8]) {
    const int pos = wi.kv_begin + 32 * s;
    const bool has_b = pos + 16 < wi.kv_end;
    const char* pa = base + (size_t)wi.tbl[pos >> 4] * kBlockBytes;
    st[0] = *(const u32x4*)(pa + tid * 16);
    st[1] = *(const u32x4*)(pa + 4096 + tid * 16);
    st[4] = *(const u32x4*)(pa + kPageBytes + tid * 16);
    st[5] = *(const u32x4*)(pa + kPageBytes + 4096 + tid * 16);
    if (has_b) {
      const char* pb = base + (size_t)wi.tbl[(pos >> 4) + 1] * kBlockBytes;
      st[2] = *(const u32x4*)(pb + tid * 16);
      st[3] = *(const u32x4*)(pb + 4096 + tid * 16);
      st[6] = *(const u32x4*)(pb + kPageBytes + tid * 16);
      st[7] = *(const u32x4*)(pb + kPageBytes + 4096 + tid * 16);
    }
  };
  auto commit = [&](const int stage, const u32x4 (&st)[8]) {
    char* dst = smem + stage * kStageBytes + tid * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) *(u32x4*)(dst + (i >> 1) * kPageBytes + (i & 1) * 4096) = st[i];
  };
  auto compute = [&](const int s) {
    const int pos = wi.kv_begin + 32 * s;
    const bool has_b = pos + 16 < wi.kv_end;
    const char* sk = smem + (s & 1) * kStageBytes + lane * 16;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) sa = mfma16(*(const u32x4*)(sk + j * 1024), qf[j], sa);
    if (has_b) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        sb = mfma16(*(const u32x4*)(sk + kPageBytes + j * 1024), qf[j], sb);
    }
    u32x4 pf, pl;
    softmax_step(sa, sb, has_b, pos, wi.kv_end, qpos, g, sl2, m, l, acc, pf, pl);
    const int left = wi.kv_end - pos;
    uint32_t mask[4];
    value_masks(left, g, mask);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const u32x4 va = *(const u32x4*)(sk + 2 * kPageBytes + c * 1024);
      u32x4 vb = {0, 0, 0, 0};
      if (has_b) vb = *(const u32x4*)(sk + 3 * kPageBytes + c * 1024);
      pv_block(acc, c, va, vb, mask, left < 32, pf, pl);
    }
  };
  // body(s, cur, nxt): cur's content (step s) already sits in LDS; nxt holds step s+1 in flight
  auto body = [&](const int s, u32x4 (&cur)[8], const u32x4 (&nxt)[8]) {
    if (s + 2 < nsteps) fetch(s + 2, cur);
    if (wave_active) compute(s);
    if (s + 1 < nsteps) commit((s + 1) & 1, nxt);
    __syncthreads();
  };
  fetch(0, st0);
  if (nsteps > 1) fetch(1, st1);
  commit(0, st0);
  __syncthreads();
  for (int s = 0; s < nsteps; s += 2) {
    body(s, st0, st1);
    if (s + 1 < nsteps) body(s + 1, st1, st0);
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (row_valid) {
    const size_t slot = (size_t)a.part_off[tok] + wi.part_idx;
    float* dst = a.part_acc + (slot * kHeads + h) * kDim;
#pragma unroll
    for (int c = 0; c < 16; ++c) *(f32x4*)(dst + 16 * c + 4 * g) = acc[c];
    if (g == 0) {
      a.part_ml[(slot * kHeads + h) * 2] = m;
      a.part_ml[(slot * kHeads + h) * 2 + 1] = l;
    }
  }
}

// ---- stream path: <= 2 query tokens (16 rows, the decode case).  Nothing is shared, so the
// four wavefronts take the 32-key steps of the split round-robin, stream their pages straight
// into registers one step ahead, and combine their four results through LDS.
__device__ __forceinline__ void stream_path(const AttnArgs& a, const WorkItem& wi, char* smem,
                                            float (*sml)[16][2], char* qs) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int n = lane & 15, g = lane >> 4;
  const int ts = n >> 3, h = n & 7;
  const bool row_valid = ts < wi.n_tok;
  const int tok = row_valid ? a.tok_list[wi.tok_off + ts] : 0;
  const int qpos = wi.q0 + ts;
  // the 16 query rows are the same for all four wavefronts: keep their MFMA fragments in LDS
  // (registers are needed for the pages in flight)
  {
    const char* qrow = (const char*)a.q + ((size_t)tok * kHeads + h) * (kDim * 2);
    const u32x4 z = {0, 0, 0, 0};
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int j = 2 * wv + jj;
      *(u32x4*)(qs + j * 1024 + lane * 16) = row_valid ? *(const u32x4*)(qrow + j * 64 + g * 16) : z;
    }
  }
  __syncthreads();
  const char* qf = qs + lane * 16;
  float m = -__builtin_inff(), l = 0.f;
  f32x4 acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;
  const char* __restrict__ base = (const char*)a.layer_base + lane * 16;
  const int nsteps = (wi.kv_end - wi.kv_begin + 31) >> 5;

  u32x4 kr[16], vr[16];
  auto load_k = [&](const int s) {
    const int pos = wi.kv_begin + 32 * s;
    const char* pa = base + (size_t)wi.tbl[pos >> 4] * kBlockBytes;
#pragma unroll
    for (int j = 0; j < 8; ++j) kr[j] = *(const u32x4*)(pa + j * 1024);
    if (pos + 16 < wi.kv_end) {
      const char* pb = base + (size_t)wi.tbl[(pos >> 4) + 1] * kBlockBytes;
#pragma unroll
      for (int j = 0; j < 8; ++j) kr[8 + j] = *(const u32x4*)(pb + j * 1024);
    }
  };
  auto load_v = [&](const int s) {
    const int pos = wi.kv_begin + 32 * s;
    const char* pa = base + (size_t)wi.tbl[pos >> 4] * kBlockBytes + kPageBytes;
#pragma unroll
    for (int c = 0; c < 8; ++c) vr[c] = *(const u32x4*)(pa + c * 1024);
    if (pos + 16 < wi.kv_end) {
      const char* pb = base + (size_t)wi.tbl[(pos >> 4) + 1] * kBlockBytes + kPageBytes;
#pragma unroll
      for (int c = 0; c < 8; ++c) vr[8 + c] = *(const u32x4*)(pb + c * 1024);
    }
  };
  int s = wv;
  if (s < nsteps) {
    load_k(s);
    load_v(s);
  }
  for (; s < nsteps; s += 4) {
    const int pos = wi.kv_begin + 32 * s;
    const bool has_b = pos + 16 < wi.kv_end;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) sa = mfma16(kr[j], *(const u32x4*)(qf + j * 1024), sa);
    if (has_b) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sb = mfma16(kr[8 + j], *(const u32x4*)(qf + j * 1024), sb);
    }
    u32x4 pf, pl;
    softmax_step(sa, sb, has_b, pos, wi.kv_end, qpos, g, sl2, m, l, acc, pf, pl);
    __builtin_amdgcn_sched_barrier(0);  // the next K pages reuse kr[]: issue only after S
    if (s + 4 < nsteps) load_k(s + 4);
    __builtin_amdgcn_sched_barrier(0);
    const int left = wi.kv_end - pos;
    uint32_t mask[4];
    value_masks(left, g, mask);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      u32x4 vb = {0, 0, 0, 0};
      if (has_b) vb = vr[8 + c];
      pv_block(acc, c, vr[c], vb, mask, left < 32, pf, pl);
    }
    __builtin_amdgcn_sched_barrier(0);  // likewise vr[]
    if (s + 4 < nsteps) load_v(s + 4);
    __builtin_amdgcn_sched_barrier(0);
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
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
  const int r = tid >> 4, seg = (tid & 15) * 16;
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
    const int otok = a.tok_list[wi.tok_off + (r >> 3)];
    const size_t slot = (size_t)a.part_off[otok] + wi.part_idx;
    float* dst = a.part_acc + (slot * kHeads + (r & 7)) * kDim + seg;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const f32x4 x = *(const f32x4*)(sm + (w * 16 + r) * kMergeStride + seg + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = __builtin_fmaf(wgt[w], x[e], o[e]);
      }
      *(f32x4*)(dst + 4 * q) = o;
    }
    if ((tid & 15) == 0) {
      a.part_ml[(slot * kHeads + (r & 7)) * 2] = big;
      a.part_ml[(slot * kHeads + (r & 7)) * 2 + 1] = total;
    }
  }
}

__global__ __launch_bounds__(256, 2) void attn_kernel(const AttnArgs a) {
  __shared__ __align__(16) char smem[kSmemBytes];
  __shared__ float sml[4][16][2];
  __shared__ __align__(16) char qs[16 * kDim * 2];
  const int32_t* __restrict__ w = a.work + (size_t)blockIdx.x * kWorkWords;
  WorkItem wi;
  wi.tok_off = w[W_TOK_OFF];
  wi.n_tok = w[W_N_TOK];
  wi.tbl = a.tables + w[W_TBL_OFF];
  wi.kv_begin = w[W_KV_BEGIN];
  wi.kv_end = w[W_KV_END];
  wi.q0 = w[W_CAUSAL_Q0];
  wi.part_idx = w[W_PART_IDX];
  const int path = w[W_PATH];
  if (path == PATH_TILE)
    tile_path(a, wi, smem);
  else if (path == PATH_STREAM)
    stream_path(a, wi, smem, sml, qs);
}

// ------------------------------------------------------------------------------------------
// merge of a query token's partials (log-sum-exp rule), one workgroup per token
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merge_kernel(const AttnArgs a) {
  const int tok = blockIdx.x, t = threadIdx.x;
  const int h = t >> 5, d0 = (t & 31) * 8;
  const int np = a.n_parts[tok];
  const size_t base = (size_t)a.part_off[tok];
  float big = -__builtin_inff();
  for (int p = 0; p < np; ++p) big = fmaxf(big, a.part_ml[((base + p) * kHeads + h) * 2]);
  float total = 0.f;
  float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < np; ++p) {
    const float mp = a.part_ml[((base + p) * kHeads + h) * 2];
    const float lp = a.part_ml[((base + p) * kHeads + h) * 2 + 1];
    const float wgt = fast_exp2(mp - big);
    total += wgt * lp;
    const float* src = a.part_acc + ((base + p) * kHeads + h) * kDim + d0;
    const f32x4 x = *(const f32x4*)src, y = *(const f32x4*)(src + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      o[e] += wgt * x[e];
      o[4 + e] += wgt * y[e];
    }
  }
  const float inv = 1.f / total;
  const u32x4 packed = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv),
                        pack_bf16(o[4] * inv, o[5] * inv), pack_bf16(o[6] * inv, o[7] * inv)};
  *(u32x4*)((uint16_t*)a.out + ((size_t)tok * kHeads + h) * kDim + d0) = packed;
  if (a.lse && (t & 31) == 0)
    a.lse[(size_t)tok * kHeads + h] = (big + __builtin_amdgcn_logf(total)) * 0.6931471805599453f;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  if (a.n_work <= 0 || a.n_q <= 0) return hipErrorInvalidValue;
  attn_kernel<<<a.n_work, 256, 0, s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  merge_kernel<<<a.n_q, 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace oxy
