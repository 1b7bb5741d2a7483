// Block-diffusion attention over the paged K/V cache, and the token-importance reduction of Eq. 2.
//
// A query row (sequence b, block position p) attends to the sequence's whole prefix [0, L) and to the
// in-block positions whose bit is set in the sequence's visibility set (all B in the layers up to the
// eviction layer; the processed positions above it).  There is no mask inside the block (Sec. 1-2).
#include "focus_internal.h"

namespace fk {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }

__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ---------------------------------------------------------------------------------------------
// One wavefront per (row, query head): lanes split the head dimension, tokens are visited in order with an
// online softmax.  Exact to fp32 rounding; used for fp32 models and as the fallback path.
template <typename T, int NE>   // NE = D / 64 elements per lane
__global__ __launch_bounds__(64) void k_attn_rowwave(const T *__restrict__ q, int q_stride, int Hq, Rows rows, RowIndex ri,
                                                     SlotState st, const uint64_t *vis_by_b, KvLayer kv, T *out) {
  const int r = blockIdx.x;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  if (r >= M) return;
  const int hq = blockIdx.y, lane = threadIdx.x;
  const int D = NE * 64, Hkv = kv.n_kv_heads, P = kv.page_size;
  const int hk = hq / (Hq / Hkv);
  const int rm = ri.row_map[r], b = rm / ri.B;
  const int slot = slot_of(ri.seq_slot, b, st);
  const int L = st.prefix_len[slot];
  const uint64_t vis = vis_by_b ? vis_by_b[b] : ~0ull;
  const int32_t *pt = st.page_table + (size_t)slot * st.table_stride;
  const float scale = 1.0f / sqrtf((float)D);

  float qv[NE], o[NE];
  const T *qr = q + (size_t)r * q_stride + (size_t)hq * D;
  for (int e = 0; e < NE; ++e) qv[e] = to_f(qr[lane + 64 * e]) * scale, o[e] = 0.f;
  float m = -INFINITY, l = 0.f;
  const size_t page_elems = (size_t)2 * Hkv * P * D;
  for (int t = 0; t < L + ri.B; ++t) {
    if (t >= L && !((vis >> (t - L)) & 1ull)) continue;
    const T *kp = (const T *)kv.base + (size_t)pt[t / P] * page_elems + ((size_t)hk * P + (t % P)) * D;
    const T *vp = kp + (size_t)Hkv * P * D;
    float s = 0.f;
    for (int e = 0; e < NE; ++e) s += qv[e] * to_f(kp[lane + 64 * e]);
    s = wave_sum(s);
    float mn = fmaxf(m, s);
    float corr = __expf(m - mn), pr = __expf(s - mn);
    l = l * corr + pr;
    for (int e = 0; e < NE; ++e) o[e] = o[e] * corr + pr * to_f(vp[lane + 64 * e]);
    m = mn;
  }
  T *orow = out + (size_t)r * Hq * D + (size_t)hq * D;
  float inv = l > 0.f ? 1.0f / l : 0.f;
  for (int e = 0; e < NE; ++e) orow[lane + 64 * e] = (T)(o[e] * inv);
}

void attention(hipStream_t s, int dtype, const void *q, int q_stride, int n_q_heads, Rows rows, RowIndex ri,
               SlotState st, const uint64_t *vis_by_b, KvLayer kv, void *out) {
  if (rows.cap <= 0) return;
  dim3 grid(rows.cap, n_q_heads);
  const int ne = kv.head_dim / 64;
  if (dtype == FOCUS_F32) {
    if (ne == 1) k_attn_rowwave<float, 1><<<grid, 64, 0, s>>>((const float *)q, q_stride, n_q_heads, rows, ri, st, vis_by_b, kv, (float *)out);
    else k_attn_rowwave<float, 2><<<grid, 64, 0, s>>>((const float *)q, q_stride, n_q_heads, rows, ri, st, vis_by_b, kv, (float *)out);
  } else {
    if (ne == 1) k_attn_rowwave<bf16_t, 1><<<grid, 64, 0, s>>>((const bf16_t *)q, q_stride, n_q_heads, rows, ri, st, vis_by_b, kv, (bf16_t *)out);
    else k_attn_rowwave<bf16_t, 2><<<grid, 64, 0, s>>>((const bf16_t *)q, q_stride, n_q_heads, rows, ri, st, vis_by_b, kv, (bf16_t *)out);
  }
}

// ---------------------------------------------------------------------------------------------
// Token importance, Eq. 2: for one (sequence, query head), S_ij = q_i . k_j / sqrt(D) over the block's own
// B x B scores, MaxPool1D (window 3, same length) along j, softmax along j, column sums over i.
// Output partial[b, h, j]; the head sum is taken later in a fixed order (no atomics, so it is reproducible).
// The fused qkv buffer of the full block is read after the rotary embedding has been applied in place.
template <typename T, int MAXB, int MAXD>
__global__ __launch_bounds__(256) void k_importance(const T *__restrict__ qkv, int B, int Hq, int Hkv, int D, int pool_k,
                                                    float *partial) {
  __shared__ float ks[MAXB * (MAXD + 1)];
  __shared__ float S[MAXB][MAXB + 1];
  const int b = blockIdx.x, h = blockIdx.y, hk = h / (Hq / Hkv);
  const int stride = (Hq + 2 * Hkv) * D;
  const T *base = qkv + (size_t)b * B * stride;
  for (int i = threadIdx.x; i < B * D; i += 256) {
    int j = i / D, d = i % D;
    ks[j * (D + 1) + d] = to_f(base[(size_t)j * stride + (size_t)(Hq + hk) * D + d]);
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)D);
  // thread -> query row i = tid / 4 and keys j = (tid % 4) + 4 * jj
  const int i = threadIdx.x >> 2, j0 = threadIdx.x & 3;
  if (i < B) {
    float acc[MAXB / 4];
    for (int jj = 0; jj < MAXB / 4; ++jj) acc[jj] = 0.f;
    const T *qi = base + (size_t)i * stride + (size_t)h * D;
    for (int d = 0; d < D; ++d) {
      float qd = to_f(qi[d]);
#pragma unroll
      for (int jj = 0; jj < MAXB / 4; ++jj) {
        int j = j0 + 4 * jj;
        if (j < B) acc[jj] += qd * ks[j * (D + 1) + d];
      }
    }
#pragma unroll
    for (int jj = 0; jj < MAXB / 4; ++jj) {
      int j = j0 + 4 * jj;
      if (j < B) S[i][j] = acc[jj] * scale;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < B) {
    const int row = threadIdx.x;
    float m = -INFINITY;                        // max of the pooled row equals max of the row
    for (int j = 0; j < B; ++j) m = fmaxf(m, S[row][j]);
    float sum = 0.f;
    {
      float a = -INFINITY, c0 = S[row][0];
      for (int j = 0; j < B; ++j) {
        float nx = (j + 1 < B) ? S[row][j + 1] : -INFINITY;
        float pooled = pool_k == 3 ? fmaxf(fmaxf(a, c0), nx) : c0;
        sum += __expf(pooled - m);
        a = c0; c0 = nx;
      }
    }
    float inv = 1.0f / sum;
    float a = -INFINITY, c0 = S[row][0];
    for (int j = 0; j < B; ++j) {
      float nx = (j + 1 < B) ? S[row][j + 1] : -INFINITY;
      float pooled = pool_k == 3 ? fmaxf(fmaxf(a, c0), nx) : c0;
      S[row][j] = __expf(pooled - m) * inv;
      a = c0; c0 = nx;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < B) {
    const int j = threadIdx.x;
    float col = 0.f;
    for (int ii = 0; ii < B; ++ii) col += S[ii][j];
    partial[((size_t)b * Hq + h) * B + j] = col;
  }
}

void importance(hipStream_t s, int dtype, const void *qkv, int n_seq, int B, int n_q_heads, int n_kv_heads,
                int head_dim, int maxpool_k, float *partial) {
  if (n_seq <= 0) return;
  dim3 grid(n_seq, n_q_heads);
  if (dtype == FOCUS_F32)
    k_importance<float, 64, 128><<<grid, 256, 0, s>>>((const float *)qkv, B, n_q_heads, n_kv_heads, head_dim, maxpool_k, partial);
  else
    k_importance<bf16_t, 64, 128><<<grid, 256, 0, s>>>((const bf16_t *)qkv, B, n_q_heads, n_kv_heads, head_dim, maxpool_k, partial);
}

}  // namespace fk
