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
// attention, wave path: one wavefront per work item, <= 16 rows (2 tokens x 8 heads)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attn_wave_kernel(const AttnArgs a) {
  const int lane = threadIdx.x;
  const int n = lane & 15, g = lane >> 4;
  const int32_t* __restrict__ w = a.work + (size_t)blockIdx.x * kWorkWords;
  const int tok_off = w[W_TOK_OFF], n_tok = w[W_N_TOK], tbl_off = w[W_TBL_OFF];
  const int kv_begin = w[W_KV_BEGIN], kv_end = w[W_KV_END], q0 = w[W_CAUSAL_Q0];
  const int part_idx = w[W_PART_IDX];
  const int ts = n >> 3, h = n & 7;
  const bool row_valid = ts < n_tok;
  const int tok = row_valid ? a.tok_list[tok_off + ts] : 0;
  const int qpos = q0 + ts;  // own position of this row's query; huge when not causal

  u32x4 qf[8];
  {
    const char* qrow = (const char*)a.q + ((size_t)tok * kHeads + h) * (kDim * 2);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      u32x4 z = {0, 0, 0, 0};
      qf[j] = row_valid ? *(const u32x4*)(qrow + j * 64 + g * 16) : z;
    }
  }
  const float ninf = -__builtin_inff();
  float m = ninf, l = 0.f;
  f32x4 acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;
  const int32_t* __restrict__ tbl = a.tables + tbl_off;
  const char* __restrict__ base = (const char*)a.layer_base;

  for (int pos = kv_begin; pos < kv_end; pos += 32) {
    const bool has_b = pos + 16 < kv_end;
    const int blk_a = tbl[pos >> 4];
    const int blk_b = has_b ? tbl[(pos >> 4) + 1] : blk_a;
    const char* pa = base + (size_t)blk_a * kBlockBytes;
    const char* pb = base + (size_t)blk_b * kBlockBytes;

    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) sa = mfma16(*(const u32x4*)(pa + j * 1024 + lane * 16), qf[j], sa);
    if (has_b) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sb = mfma16(*(const u32x4*)(pb + j * 1024 + lane * 16), qf[j], sb);
    }
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
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] *= alpha;
    // P enters the second product as bf16.  A single rounding (2^-9 relative) is too coarse
    // when a query sees only a handful of keys, so P = hi + lo with both parts in bf16.
    u32x4 pf, pl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pf[i] = pack_bf16(p[2 * i], p[2 * i + 1]);
      pl[i] = pack_bf16(p[2 * i] - __uint_as_float(pf[i] << 16),
                        p[2 * i + 1] - __uint_as_float(pf[i] & 0xffff0000u));
    }

    // values of keys at or beyond kv_end may be stale bits: select them to zero
    const int left = kv_end - pos;  // >= 1
    uint32_t mask[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
    if (left < 32) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int k0 = 4 * g + 2 * i;
        mask[i] = (k0 < left ? 0xffffu : 0u) | (k0 + 1 < left ? 0xffff0000u : 0u);
        mask[2 + i] = (k0 + 16 < left ? 0xffffu : 0u) | (k0 + 17 < left ? 0xffff0000u : 0u);
      }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      u32x4 va = *(const u32x4*)(pa + kPageBytes + c * 1024 + lane * 16);
      u32x4 vb = {0, 0, 0, 0};
      if (has_b) vb = *(const u32x4*)(pb + kPageBytes + c * 1024 + lane * 16);
      const u32x4 v0 = {va[0] & mask[0], va[1] & mask[1], vb[0] & mask[2], vb[1] & mask[3]};
      const u32x4 v1 = {va[2] & mask[0], va[3] & mask[1], vb[2] & mask[2], vb[3] & mask[3]};
      acc[2 * c] = mfma16(v0, pl, mfma16(v0, pf, acc[2 * c]));
      acc[2 * c + 1] = mfma16(v1, pl, mfma16(v1, pf, acc[2 * c + 1]));
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (row_valid) {
    const size_t slot = (size_t)a.part_off[tok] + part_idx;
    float* dst = a.part_acc + (slot * kHeads + h) * kDim;
#pragma unroll
    for (int c = 0; c < 16; ++c) *(f32x4*)(dst + 16 * c + 4 * g) = acc[c];
    if (g == 0) {
      a.part_ml[(slot * kHeads + h) * 2] = m;
      a.part_ml[(slot * kHeads + h) * 2 + 1] = l;
    }
  }
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
  attn_wave_kernel<<<a.n_work, 64, 0, s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  merge_kernel<<<a.n_q, 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace oxy
