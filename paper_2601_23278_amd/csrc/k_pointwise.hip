// Row-wise and element-wise kernels of the decode step: embedding lookup, RMSNorm, rotary embedding fused
// with the K/V cache write, row gather for the packed batch, SiLU(gate)*up, and small state set-up kernels.
// All are bandwidth-bound; one workgroup handles one row with 16-byte accesses where the layout allows.
#include "focus_internal.h"

namespace fk {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v) { return (T)v; }

__device__ __forceinline__ int n_rows(Rows r) { return r.count ? min(*r.count, r.cap) : r.cap; }

__device__ __forceinline__ float block_sum_256(float v, float *sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

// ---------------------------------------------------------------------------------------------
// Block input (Alg. 1 "Masked Block X"): mask embedding where masked, committed token's embedding elsewhere.
template <typename T>
__global__ __launch_bounds__(256) void k_embed(const T *table, int hidden, Rows rows, RowIndex ri, SlotState st,
                                               int mask_id, float *resid) {
  int r = blockIdx.x;
  if (r >= n_rows(rows)) return;
  int rm = ri.row_map[r], b = rm / ri.B, p = rm % ri.B;
  int slot = slot_of(ri.seq_slot, b, st);
  int tok = ((st.mask_bits[slot] >> p) & 1ull) ? mask_id : st.tokens[slot * ri.B + p];
  const T *src = table + (size_t)tok * hidden;
  float *dst = resid + (size_t)r * hidden;
  for (int i = threadIdx.x; i < hidden; i += 256) dst[i] = to_f(src[i]);
}

void embed(hipStream_t s, int dtype, const void *table, int hidden, Rows rows, RowIndex ri, SlotState st,
           int mask_id, float *resid) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_F32)
    k_embed<float><<<rows.cap, 256, 0, s>>>((const float *)table, hidden, rows, ri, st, mask_id, resid);
  else
    k_embed<bf16_t><<<rows.cap, 256, 0, s>>>((const bf16_t *)table, hidden, rows, ri, st, mask_id, resid);
}

// ---------------------------------------------------------------------------------------------
// y = x / sqrt(mean(x^2) + eps) * w, x fp32 residual stream, y in the activation type.
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float *x, const T *w, T *y, int hidden, float eps, Rows rows) {
  __shared__ float sh[4];
  int r = blockIdx.x;
  if (r >= n_rows(rows)) return;
  const float *xr = x + (size_t)r * hidden;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < hidden; i += 1024) {
    float4 v = *(const float4 *)(xr + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum_256(ss, sh);
  float inv = 1.0f / sqrtf(ss / (float)hidden + eps);
  T *yr = y + (size_t)r * hidden;
  for (int i = threadIdx.x * 4; i < hidden; i += 1024) {
    float4 v = *(const float4 *)(xr + i);
    yr[i + 0] = from_f<T>(v.x * inv * to_f(w[i + 0]));
    yr[i + 1] = from_f<T>(v.y * inv * to_f(w[i + 1]));
    yr[i + 2] = from_f<T>(v.z * inv * to_f(w[i + 2]));
    yr[i + 3] = from_f<T>(v.w * inv * to_f(w[i + 3]));
  }
}

// bf16 output, hidden <= 8192: the row is read once (kept in registers between the two phases) and written
// as 16-byte vectors.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(256) void k_rmsnorm_bf16(const float *x, const bf16_t *w, bf16_t *y, int hidden, float eps, Rows rows) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  if (r >= n_rows(rows)) return;
  const float *xr = x + (size_t)r * hidden;
  float v[4][8];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = (it * 256 + threadIdx.x) * 8;
    if (i < hidden) {
      const float4 a = *(const float4 *)(xr + i), b = *(const float4 *)(xr + i + 4);
      v[it][0] = a.x; v[it][1] = a.y; v[it][2] = a.z; v[it][3] = a.w;
      v[it][4] = b.x; v[it][5] = b.y; v[it][6] = b.z; v[it][7] = b.w;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += v[it][e] * v[it][e];
    }
  }
  ss = block_sum_256(ss, sh);
  const float inv = 1.0f / sqrtf(ss / (float)hidden + eps);
  bf16_t *yr = y + (size_t)r * hidden;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = (it * 256 + threadIdx.x) * 8;
    if (i < hidden) {
      const bf16x8_t wv = *(const bf16x8_t *)(w + i);
      bf16x8_t o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(v[it][e] * inv * (float)wv[e]);
      *(bf16x8_t *)(yr + i) = o;
    }
  }
}

void rmsnorm(hipStream_t s, int dtype, const float *x, const void *w, void *y, int hidden, float eps, Rows rows) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_BF16 && hidden % 8 == 0 && hidden <= 8192 && (((uintptr_t)x | (uintptr_t)w | (uintptr_t)y) & 15) == 0) {
    k_rmsnorm_bf16<<<rows.cap, 256, 0, s>>>(x, (const bf16_t *)w, (bf16_t *)y, hidden, eps, rows);
    return;
  }
  if (dtype == FOCUS_F32)
    k_rmsnorm<float><<<rows.cap, 256, 0, s>>>(x, (const float *)w, (float *)y, hidden, eps, rows);
  else
    k_rmsnorm<bf16_t><<<rows.cap, 256, 0, s>>>(x, (const bf16_t *)w, (bf16_t *)y, hidden, eps, rows);
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding (rotate-half) of the q and k heads of one row, in place, and the K/V cache write of the
// row's k (rotated) and v into the slot of its absolute position (App. C: the K/V of a layer is filled for
// every row that enters the layer, before anything is evicted).
template <typename T>
__global__ __launch_bounds__(256) void k_rope_kv_write(T *qkv, int Hq, Rows rows, RowIndex ri, SlotState st, KvLayer kv,
                                                       const float2 *rope) {
  int r = blockIdx.x;
  if (r >= n_rows(rows)) return;
  const int D = kv.head_dim, half = D / 2, Hkv = kv.n_kv_heads, P = kv.page_size;
  int rm = ri.row_map[r], b = rm / ri.B, p = rm % ri.B;
  int slot = slot_of(ri.seq_slot, b, st);
  int pos = st.prefix_len[slot] + p;
  int page = st.page_table[(size_t)slot * st.table_stride + pos / P], off = pos % P;
  T *row = qkv + (size_t)r * (Hq + 2 * Hkv) * D;
  T *cache = (T *)kv.base + (size_t)page * 2 * Hkv * P * D;
  const float2 *cs = rope + (size_t)pos * half;
  // q and k heads: one (head, pair) per thread step
  for (int i = threadIdx.x; i < (Hq + Hkv) * half; i += 256) {
    int h = i / half, d = i % half;
    float2 c = cs[d];
    float x1 = to_f(row[h * D + d]), x2 = to_f(row[h * D + d + half]);
    T y1 = from_f<T>(x1 * c.x - x2 * c.y), y2 = from_f<T>(x2 * c.x + x1 * c.y);
    row[h * D + d] = y1;
    row[h * D + d + half] = y2;
    if (h >= Hq) {
      T *dst = cache + ((size_t)(h - Hq) * P + off) * D;
      dst[d] = y1;
      dst[d + half] = y2;
    }
  }
  const T *v = row + (size_t)(Hq + Hkv) * D;
  T *vc = cache + (size_t)Hkv * P * D;
  for (int i = threadIdx.x; i < Hkv * D; i += 256) {
    int h = i / D, d = i % D;
    vc[((size_t)h * D + d) * P + off] = v[i];       // V is kept transposed: [H_kv][D][page_size]
  }
}

// bf16: eight rotation pairs per thread step, 16-byte loads and stores (q, k in place; k also into its cache row).
__device__ __forceinline__ void rope_kv_write_row(int r, bf16_t *qkv, int Hq, Rows rows, RowIndex ri, SlotState st, KvLayer kv,
                                                  const float2 *rope, int write_v) {
  if (r >= n_rows(rows)) return;
  const int D = kv.head_dim, half = D / 2, Hkv = kv.n_kv_heads, P = kv.page_size, upr = half / 8;   // units per head
  const int rm = ri.row_map[r], b = rm / ri.B, p = rm % ri.B;
  const int slot = slot_of(ri.seq_slot, b, st);
  const int pos = st.prefix_len[slot] + p;
  const int page = st.page_table[(size_t)slot * st.table_stride + pos / P], off = pos % P;
  bf16_t *row = qkv + (size_t)r * (Hq + 2 * Hkv) * D;
  bf16_t *cache = (bf16_t *)kv.base + (size_t)page * 2 * Hkv * P * D;
  const float2 *cs = rope + (size_t)pos * half;
  for (int u = threadIdx.x; u < (Hq + Hkv) * upr; u += 256) {
    const int h = u / upr, d = (u % upr) * 8;
    bf16x8_t x1 = *(const bf16x8_t *)(row + h * D + d), x2 = *(const bf16x8_t *)(row + h * D + d + half), y1, y2;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float2 c = cs[d + e];
      const float a = (float)x1[e], bb = (float)x2[e];
      y1[e] = (bf16_t)(a * c.x - bb * c.y);
      y2[e] = (bf16_t)(bb * c.x + a * c.y);
    }
    *(bf16x8_t *)(row + h * D + d) = y1;
    *(bf16x8_t *)(row + h * D + d + half) = y2;
    if (h >= Hq) {
      bf16_t *dst = cache + ((size_t)(h - Hq) * P + off) * D;
      *(bf16x8_t *)(dst + d) = y1;
      *(bf16x8_t *)(dst + d + half) = y2;
    }
  }
  if (write_v) {
    const bf16_t *v = row + (size_t)(Hq + Hkv) * D;
    bf16_t *vc = cache + (size_t)Hkv * P * D;
    for (int i = threadIdx.x; i < Hkv * D; i += 256) vc[(size_t)i * P + off] = v[i];   // V transposed: [H_kv][D][page_size]
  }
}

// V cache write of all rows of one (sequence, kv head).  V is kept transposed, [H_kv][D][page_size], so the values of
// one row are 128 bytes apart; eight neighbouring lanes take eight rows of the same d, which fall into the same
// 128-byte line (one write transaction instead of eight).
__device__ __forceinline__ void v_write_group(int b, int hk, const bf16_t *qkv, int Hq, const int32_t *cu, RowIndex ri, SlotState st, KvLayer kv) {
  const int r0 = cu[b], nr = cu[b + 1] - r0;
  if (nr <= 0) return;
  const int D = kv.head_dim, Hkv = kv.n_kv_heads, P = kv.page_size, stride = (Hq + 2 * Hkv) * D;
  const int slot = slot_of(ri.seq_slot, b, st);
  const int L = st.prefix_len[slot];
  const int32_t *pt = st.page_table + (size_t)slot * st.table_stride;
  for (int rb = 0; rb < nr; rb += 8) {
    const int r = rb + (threadIdx.x & 7);
    if (r >= nr) continue;
    const int pos = L + ri.row_map[r0 + r] % ri.B;
    bf16_t *vc = (bf16_t *)kv.base + (size_t)pt[pos / P] * 2 * Hkv * P * D + (size_t)Hkv * P * D + (size_t)hk * D * P + pos % P;
    const bf16_t *v = qkv + (size_t)(r0 + r) * stride + (size_t)(Hq + Hkv + hk) * D;
    for (int d = threadIdx.x >> 3; d < D; d += 32) vc[(size_t)d * P] = v[d];
  }
}

// One launch for both: the first n_seq * H_kv workgroups write V (they read columns the rotation does not touch), the rest
// rotate one row each and write its K.
__global__ __launch_bounds__(256) void k_rope_kv_write_bf16(bf16_t *qkv, int Hq, Rows rows, RowIndex ri, SlotState st, KvLayer kv,
                                                            const float2 *rope, int n_seq, const int32_t *cu) {
  const int v_groups = n_seq * kv.n_kv_heads;
  if ((int)blockIdx.x < v_groups) v_write_group(blockIdx.x / kv.n_kv_heads, blockIdx.x % kv.n_kv_heads, qkv, Hq, cu, ri, st, kv);
  else rope_kv_write_row(blockIdx.x - v_groups, qkv, Hq, rows, ri, st, kv, rope, n_seq > 0 ? 0 : 1);
}

void rope_kv_write(hipStream_t s, int dtype, void *qkv, int n_q_heads, Rows rows, RowIndex ri, SlotState st,
                   KvLayer kv, const float2 *rope_table, int n_seq, const int32_t *cu) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_BF16 && kv.head_dim % 16 == 0 && (((uintptr_t)qkv | (uintptr_t)kv.base) & 15) == 0) {
    const bool by_seq = cu != nullptr && n_seq > 0;      // the V scatter per (sequence, kv head) when the row ranges are known
    const int groups = by_seq ? n_seq * kv.n_kv_heads : 0;
    k_rope_kv_write_bf16<<<groups + rows.cap, 256, 0, s>>>((bf16_t *)qkv, n_q_heads, rows, ri, st, kv, rope_table, by_seq ? n_seq : 0, cu);
    return;
  }
  if (dtype == FOCUS_F32)
    k_rope_kv_write<float><<<rows.cap, 256, 0, s>>>((float *)qkv, n_q_heads, rows, ri, st, kv, rope_table);
  else
    k_rope_kv_write<bf16_t><<<rows.cap, 256, 0, s>>>((bf16_t *)qkv, n_q_heads, rows, ri, st, kv, rope_table);
}

// ---------------------------------------------------------------------------------------------
// Gather of the retained rows (Sec. 4.2): residual stream and the layer-e queries, into packed order.
template <typename T>
__global__ __launch_bounds__(256) void k_gather(Rows rows, const int32_t *row_map, int B, const int32_t *src_cu, const uint64_t *src_bits,
                                                const float *resid, float *resid_p, int hidden, const T *qkv, int qkv_stride, T *q_p,
                                                int q_width) {
  int r = blockIdx.x;
  if (r >= n_rows(rows)) return;
  int src = row_map[r];
  if (src_bits) {       // the source rows are themselves a packed subset of the block positions
    const int b = src / B, p = src % B;
    src = src_cu[b] + __popcll(src_bits[b] & ((1ull << p) - 1));
  }
  const float4 *a = (const float4 *)(resid + (size_t)src * hidden);
  float4 *o = (float4 *)(resid_p + (size_t)r * hidden);
  const T *q = qkv + (size_t)src * qkv_stride;
  T *qo = q_p + (size_t)r * q_width;
  constexpr int QV = 16 / sizeof(T);                       // query elements per 16-byte piece
  const bool qvec = q_width % QV == 0 && qkv_stride % QV == 0 && (((size_t)qkv | (size_t)q_p) & 15) == 0;
  const int n4 = hidden / 4, nq = qvec ? q_width / QV : 0;
  // plain load-store pairs: all workgroups of the launch start together, and a kernel that first reads its whole row and then
  // writes it makes the chip alternate between a read phase and a write phase (measured: 35 us against 23 us for 100 MB)
  for (int i = threadIdx.x; i < n4; i += 256) o[i] = a[i];
  for (int i = threadIdx.x; i < nq; i += 256) ((float4 *)qo)[i] = ((const float4 *)q)[i];
  if (!qvec)
    for (int i = threadIdx.x; i < q_width; i += 256) qo[i] = q[i];
}

void gather_rows(hipStream_t s, int dtype, Rows rows, const int32_t *row_map, int B, const int32_t *src_cu, const uint64_t *src_bits,
                 const float *resid, float *resid_p, int hidden, const void *qkv, int qkv_stride, void *q_p, int q_width) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_F32)
    k_gather<float><<<rows.cap, 256, 0, s>>>(rows, row_map, B, src_cu, src_bits, resid, resid_p, hidden, (const float *)qkv, qkv_stride,
                                             (float *)q_p, q_width);
  else
    k_gather<bf16_t><<<rows.cap, 256, 0, s>>>(rows, row_map, B, src_cu, src_bits, resid, resid_p, hidden, (const bf16_t *)qkv, qkv_stride,
                                              (bf16_t *)q_p, q_width);
}

// ---------------------------------------------------------------------------------------------
// act = silu(gate) * up over the fused [rows, 2F] projection.
template <typename T>
__global__ __launch_bounds__(256) void k_silu_mul(const T *gu, T *act, int ffn, Rows rows) {
  int r = blockIdx.y;
  if (r >= n_rows(rows)) return;
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= ffn) return;
  float g = to_f(gu[(size_t)r * 2 * ffn + i]), u = to_f(gu[(size_t)r * 2 * ffn + ffn + i]);
  act[(size_t)r * ffn + i] = from_f<T>(g / (1.0f + __expf(-g)) * u);
}

void silu_mul(hipStream_t s, int dtype, const void *gate_up, void *act, int ffn, Rows rows) {
  if (rows.cap <= 0) return;
  dim3 grid((ffn + 255) / 256, rows.cap);
  if (dtype == FOCUS_F32)
    k_silu_mul<float><<<grid, 256, 0, s>>>((const float *)gate_up, (float *)act, ffn, rows);
  else
    k_silu_mul<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)gate_up, (bf16_t *)act, ffn, rows);
}

// ---------------------------------------------------------------------------------------------
// state set-up

__global__ void k_fill_u64(uint64_t *p, int n, uint64_t v) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void k_add_counts(int n, const int32_t *counts, int64_t *totals) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) totals[i] += counts[i];
}

void add_counts(hipStream_t s, int n, const int32_t *counts, int64_t *totals) {
  if (n > 0) k_add_counts<<<(n + 255) / 256, 256, 0, s>>>(n, counts, totals);
}

void fill_u64(hipStream_t s, uint64_t *p, int n, uint64_t v) {
  if (n > 0) k_fill_u64<<<(n + 255) / 256, 256, 0, s>>>(p, n, v);
}

// Row map of the full (not yet evicted) batch: row r is (b, p) = (r / B, r % B); cu[b] = b * B.
__global__ void k_iota_rows(int32_t *row_map, int32_t *cu, int n_seq, int B, int32_t *total) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_seq * B) row_map[i] = i;
  if (i <= n_seq) cu[i] = i * B;
  if (i == 0) *total = n_seq * B;
}
void iota_rows(hipStream_t s, int32_t *row_map, int32_t *cu, int n_seq, int B, int32_t *total) {
  k_iota_rows<<<(n_seq * B + 256) / 256, 256, 0, s>>>(row_map, cu, n_seq, B, total);
}

// Longest-first launch order for the attention workgroups: with a handful of workgroups per CU and an 8x
// spread of prefix lengths, starting the long sequences first keeps the tail of the launch short.
__global__ __launch_bounds__(256) void k_length_order(int n_seq, const int32_t *seq_slot, SlotState st, int32_t *order) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= n_seq) return;
  const int len = st.prefix_len[slot_of(seq_slot, b, st)];
  int rank = 0;
  for (int o = 0; o < n_seq; ++o) {
    const int lo = st.prefix_len[slot_of(seq_slot, o, st)];
    rank += (lo > len || (lo == len && o < b)) ? 1 : 0;
  }
  order[rank] = b;
}
void length_order(hipStream_t s, int n_seq, const int32_t *seq_slot, SlotState st, int32_t *order) {
  if (n_seq > 0) k_length_order<<<(n_seq + 255) / 256, 256, 0, s>>>(n_seq, seq_slot, st, order);
}

// New block: every position masked, nothing processed; statistics kept or cleared.
__global__ void k_reset_block(int n_seq, int B, const int32_t *seq_slot, SlotState st, const int32_t *prefix_len,
                              int mask_id, int keep_stats) {
  int b = blockIdx.x;
  int slot = slot_of(seq_slot, b, st);
  if (threadIdx.x < B) st.tokens[slot * B + threadIdx.x] = mask_id;
  if (threadIdx.x == 0) {
    st.prefix_len[slot] = prefix_len[b];
    st.mask_bits[slot] = B >= 64 ? ~0ull : ((1ull << B) - 1);
    st.processed_bits[slot] = 0;
    st.cached_bits[slot] = 0;
    if (!keep_stats) {
      st.token_sum[slot] = 0;
      st.total_steps[slot] = 0;
    }
  }
}
void reset_block_state(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st,
                       const int32_t *prefix_len, int mask_id, int keep_stats) {
  if (n_seq > 0) k_reset_block<<<n_seq, 64, 0, s>>>(n_seq, B, seq_slot, st, prefix_len, mask_id, keep_stats);
}

__global__ void k_finalize_pick(int n_seq, int B, int P, const int32_t *seq_slot, SlotState st, uint64_t *keep_bits, int32_t *finalized) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= n_seq) return;
  const int slot = slot_of(seq_slot, b, st);
  const uint64_t all = B >= 64 ? ~0ull : ((1ull << B) - 1);
  const int L = st.prefix_len[slot];
  const bool done = (st.mask_bits[slot] & all) == 0 && L + B <= st.max_prefix_len && (long)L + 2 * B <= (long)st.page_count[slot] * P;
  keep_bits[b] = done ? all & ~st.cached_bits[slot] : 0;      // frozen positions keep the K/V they have (Sec. 4.3)
  if (finalized) finalized[b] = done ? 1 : 0;
}
void finalize_pick(hipStream_t s, int n_seq, int B, int page_size, const int32_t *seq_slot, SlotState st, uint64_t *keep_bits,
                   int32_t *finalized) {
  if (n_seq > 0) k_finalize_pick<<<(n_seq + 63) / 64, 64, 0, s>>>(n_seq, B, page_size, seq_slot, st, keep_bits, finalized);
}

__global__ void k_finalize_advance(int n_seq, int B, const int32_t *seq_slot, SlotState st, const int32_t *finalized, int mask_id) {
  const int b = blockIdx.x;
  if (!finalized[b]) return;
  const int slot = slot_of(seq_slot, b, st);
  if ((int)threadIdx.x < B) st.tokens[slot * B + threadIdx.x] = mask_id;
  if (threadIdx.x == 0) {
    st.prefix_len[slot] += B;
    st.mask_bits[slot] = B >= 64 ? ~0ull : ((1ull << B) - 1);
    st.processed_bits[slot] = 0;
    st.cached_bits[slot] = 0;
  }
}
void finalize_advance(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st, const int32_t *finalized, int mask_id) {
  if (n_seq > 0) k_finalize_advance<<<n_seq, 64, 0, s>>>(n_seq, B, seq_slot, st, finalized, mask_id);
}

// Prefill: chunk c of each prompt becomes the (fully unmasked) block at prefix_len = c * B; sequences whose
// prompt has ended contribute no rows.
__global__ void k_prefill_chunk(int n_seq, int B, int chunk, const int32_t *seq_slot, SlotState st, const int32_t *prompt,
                                const int32_t *prompt_offset, const int32_t *prompt_len, uint64_t *keep_bits) {
  int b = blockIdx.x;
  int slot = slot_of(seq_slot, b, st);
  int start = chunk * B;
  int nr = min(max(prompt_len[b] - start, 0), B);
  if ((int)threadIdx.x < nr) st.tokens[slot * B + threadIdx.x] = prompt[prompt_offset[b] + start + threadIdx.x];
  if (threadIdx.x == 0) {
    st.prefix_len[slot] = start;
    st.mask_bits[slot] = 0;
    st.cached_bits[slot] = 0;
    keep_bits[b] = nr >= 64 ? ~0ull : ((1ull << nr) - 1);
  }
}
void prefill_chunk_setup(hipStream_t s, int n_seq, int B, int chunk, const int32_t *seq_slot, SlotState st,
                         const int32_t *prompt, const int32_t *prompt_offset, const int32_t *prompt_len,
                         uint64_t *keep_bits) {
  if (n_seq > 0)
    k_prefill_chunk<<<n_seq, 64, 0, s>>>(n_seq, B, chunk, seq_slot, st, prompt, prompt_offset, prompt_len, keep_bits);
}

}  // namespace fk
