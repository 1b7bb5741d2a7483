// Integer-exact stages of the FOCUS step: budget (Eq. 4-5), top-K selection with the structural constraints
// of Sec. 4.2 (Alg. 1 phase 3), prefix-sum packing of the retained rows, confidence over the vocabulary,
// and the confidence-based commit with the running statistics of App. E.3.1.
//
// One 64-lane wavefront owns one sequence: lane j holds block position j (B <= 64), sets of positions are
// 64-bit ballots, ranks come from lane-to-lane reads.  Every decision is a comparison of the given fp32
// values (ties: lower index), so identical scores give identical indices on any implementation.
#include "focus_internal.h"

namespace fk {

__device__ __forceinline__ uint64_t low_bits(int n) { return n >= 64 ? ~0ull : ((1ull << n) - 1); }

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_select(SelectArgs a) {
  __shared__ float dsh[64];
  const int b = blockIdx.x, j = threadIdx.x, B = a.B;
  const int slot = slot_of(a.seq_slot, b, a.st);
  const bool in = j < B;

  // importance of the two layers: sum of the per-head column sums in head order; delta (Eq. 3)
  float d = 0.f;
  if (a.delta_in) {
    d = in ? a.delta_in[(size_t)b * B + j] : 0.f;
  } else {
    float ie = 0.f, ip = 0.f;
    if (in) {
      for (int h = 0; h < a.n_q_heads; ++h) ie += a.partial_evict[((size_t)b * a.n_q_heads + h) * B + j];
      if (a.importance_mode == 0)
        for (int h = 0; h < a.n_q_heads; ++h) ip += a.partial_prev[((size_t)b * a.n_q_heads + h) * B + j];
      if (a.imp_out) a.imp_out[(size_t)b * B + j] = ie;
      if (a.imp_prev_out) a.imp_prev_out[(size_t)b * B + j] = ip;
    }
    d = ie - ip;
  }
  if (in && a.delta_out) a.delta_out[(size_t)b * B + j] = d;

  const uint64_t all = low_bits(B);
  const uint64_t masked = a.st.mask_bits[slot] & all;
  const bool is_masked = (masked >> j) & 1ull;
  // delayed intra-block cache (Sec. 4.3): frozen positions have left the rows; decoded positions that are not frozen
  // yet are owed the forward with their final token in every layer
  const uint64_t frozen = a.intra_block_cache ? a.st.cached_bits[slot] & all : 0ull;
  const uint64_t owed = a.intra_block_cache ? all & ~frozen & ~masked : 0ull;
  uint64_t keep;
  int K;

  if (a.keep_override) {
    keep = a.keep_override[b] & all;
    K = __popcll(keep);
  } else {
    // budget
    if (a.budget_mode == FOCUS_BUDGET_OVERRIDE) {
      K = a.k_override[b];
    } else if (a.budget_mode == FOCUS_BUDGET_DYNAMIC) {
      // N_sigma (Eq. 5): masked positions with delta >= block mean + population std, both accumulated in
      // fp64 in index order with separately rounded operations
      dsh[j] = d;
      __syncthreads();
      double thr = 0.0;
      if (j == 0) {
        double s = 0.0;
        for (int i = 0; i < B; ++i) s = __dadd_rn(s, (double)dsh[i]);
        double mu = s / (double)B;
        double ss = 0.0;
        for (int i = 0; i < B; ++i) {
          double e = __dsub_rn((double)dsh[i], mu);
          ss = __dadd_rn(ss, __dmul_rn(e, e));
        }
        thr = __dadd_rn(mu, sqrt(ss / (double)B));
      }
      thr = __shfl(thr, 0);
      int n_sigma = __popcll(__ballot(in && is_masked && (double)d >= thr));
      // Eq. 4: historical term ceil(alpha * mean decoded per step), 1 on the first step
      int steps = a.st.total_steps[slot];
      double nbar = steps > 0 ? (double)a.st.token_sum[slot] / (double)steps : 1.0;
      int k_hist = (int)ceil(__dmul_rn((double)a.alpha, nbar));
      K = max(k_hist, n_sigma);
    } else {
      K = a.K_fixed;
    }
    K = max(0, min(B, K));

    if (K >= B) {
      keep = all & ~frozen;                      // no eviction: the whole block (what is left of it) stays
    } else {
      // rank of position j among the masked positions: number that order before it
      int rank = 0;
      if (a.selection == FOCUS_SELECT_RANDOM) {
        // control of Sec. 5.2: SplitMix64 output number c + 1 from the seed, c = (slot * 2^32 + step) * 64 + j
        const uint64_t c = ((((uint64_t)slot << 32) + (uint64_t)(uint32_t)a.st.total_steps[slot]) << 6) + (uint64_t)j;
        uint64_t z = (uint64_t)a.selection_seed + (c + 1) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        const unsigned lo = (unsigned)z, hi = (unsigned)(z >> 32);
        for (int i = 0; i < B; ++i) {
          const uint64_t zi = ((uint64_t)__shfl(hi, i) << 32) | __shfl(lo, i);
          const bool mi = (masked >> i) & 1ull;
          rank += (mi && (zi > z || (zi == z && i < j))) ? 1 : 0;
        }
      } else {
        float v = (a.selection == FOCUS_SELECT_BOTTOM) ? -d : d;   // BOTTOM: smallest delta first
        v = (v != v) ? -INFINITY : v;                              // NaN ranks last
        for (int i = 0; i < B; ++i) {
          float vi = __shfl(v, i);
          bool mi = (masked >> i) & 1ull;
          rank += (mi && (vi > v || (vi == v && i < j))) ? 1 : 0;
        }
      }
      const uint64_t top = __ballot(in && is_masked && rank < K);
      keep = top;
      if (keep) {
        if (a.constraints & FOCUS_KEEP_AR_CONTEXT) keep |= (top >> 1) & ~frozen;   // predecessor of every pick
        if (a.constraints & FOCUS_KEEP_PLACEHOLDERS) {
          int mx = 63 - __clzll((long long)keep);
          keep |= masked & low_bits(mx);                                      // masked positions below max(S)
        }
      }
      keep |= owed;
    }
  }
  if (j == 0) {
    a.K_out[b] = K;
    a.keep_out[b] = keep;
    a.n_keep_out[b] = __popcll(keep);
    if (a.update_state || a.vis_out) {
      const uint64_t proc = a.st.processed_bits[slot] | keep;
      if (a.update_state) a.st.processed_bits[slot] = proc;
      if (a.vis_out) a.vis_out[b] = proc;
    }
  }
}

void select(hipStream_t s, const SelectArgs &a) {
  if (a.n_seq > 0) k_select<<<a.n_seq, 64, 0, s>>>(a);
}

// ---------------------------------------------------------------------------------------------
// Packed order of the retained rows: exclusive prefix sum of the per-sequence counts (one workgroup, each lane
// scans a contiguous chunk of sequences), then row_map[cu[b] + i] = b * B + (i-th set bit of keep[b]).
__global__ __launch_bounds__(256) void k_scan_compact(int n_seq, int B, const uint64_t *keep_bits, int32_t *cu,
                                                      int32_t *row_map, int32_t *total) {
  __shared__ int part[256];
  const int t = threadIdx.x;
  const int chunk = (n_seq + 255) / 256;
  const int b0 = t * chunk, b1 = min(b0 + chunk, n_seq);
  int sum = 0;
  for (int b = b0; b < b1; ++b) sum += __popcll(keep_bits[b]);
  part[t] = sum;
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int i = 0; i < 256; ++i) { int v = part[i]; part[i] = run; run += v; }
    cu[n_seq] = run;
    *total = run;
  }
  __syncthreads();
  int at = part[t];
  for (int b = b0; b < b1; ++b) {
    cu[b] = at;
    uint64_t k = keep_bits[b];
    while (k) {
      int p = __ffsll((long long)k) - 1;
      row_map[at++] = b * B + p;
      k &= k - 1;
    }
  }
}

void scan_compact(hipStream_t s, int n_seq, int B, const uint64_t *keep_bits, int32_t *cu, int32_t *row_map,
                  int32_t *total) {
  k_scan_compact<<<1, 256, 0, s>>>(n_seq, B, keep_bits, cu, row_map, total);
}

// ---------------------------------------------------------------------------------------------
// Confidence of a row of logits: arg-max (lowest id on ties) and 1 / sum exp(logit - max).
// One pass over the row: every lane keeps a running maximum (with its index: ascending index per lane, so the first
// maximum is kept) and the sum of exp(x - maximum so far), rescaled when the maximum grows; lanes are merged as
// (maximum, sum) pairs, lowest index on equal maxima.
__device__ __forceinline__ void conf_push(float v, int i, float &m, int &mi, float &s) {
  if (v > m) { s = s * __expf(m - v) + 1.0f; m = v; mi = i; }
  else s += v == -INFINITY ? 0.f : __expf(v - m);     // (a row that starts with -inf: exp(-inf + inf) is not a number)
}
__device__ __forceinline__ void conf_merge(float om, int oi, float os, float &m, int &mi, float &s) {
  const float big = fmaxf(m, om);
  const float a = m == big ? 1.0f : __expf(m - big), b = om == big ? 1.0f : __expf(om - big);
  s = s * a + os * b;
  if (om > m || (om == m && oi < mi)) mi = oi;
  m = big;
}
__global__ __launch_bounds__(256) void k_confidence(const float *__restrict__ logits, int vocab, Rows rows, float *conf,
                                                    int32_t *argmax) {
  __shared__ float smax[4], ssum[4];
  __shared__ int sidx[4];
  const int r = blockIdx.x;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  if (r >= M) return;
  const float *x = logits + (size_t)r * vocab;
  const int nv = ((size_t)x & 15) == 0 ? vocab / 4 : 0;       // 16-byte pieces when the row is aligned
  float m = -INFINITY, sum = 0.f;
  int mi = 0x7fffffff;
  for (int i = threadIdx.x; i < nv; i += 256) {
    const float4 v = ((const float4 *)x)[i];
    conf_push(v.x, 4 * i, m, mi, sum);
    conf_push(v.y, 4 * i + 1, m, mi, sum);
    conf_push(v.z, 4 * i + 2, m, mi, sum);
    conf_push(v.w, 4 * i + 3, m, mi, sum);
  }
  for (int i = 4 * nv + threadIdx.x; i < vocab; i += 256) conf_push(x[i], i, m, mi, sum);
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o), os = __shfl_xor(sum, o);
    const int oi = __shfl_xor(mi, o);
    conf_merge(om, oi, os, m, mi, sum);
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { smax[w] = m; sidx[w] = mi; ssum[w] = sum; }
  __syncthreads();
  if (threadIdx.x == 0) {
    m = smax[0]; mi = sidx[0]; sum = ssum[0];
    for (int i = 1; i < 4; ++i) conf_merge(smax[i], sidx[i], ssum[i], m, mi, sum);
    conf[r] = 1.0f / sum;
    argmax[r] = mi;
  }
}

// Few rows: one workgroup per row leaves most of the chip idle while it walks 150 000 logits, so a row is cut into
// kConfParts column ranges.  A part records its own maximum (lowest index on ties), where it is, and the sum of
// exp(x - its maximum); the merge takes the overall maximum and adds the rescaled sums in part order.
constexpr int kConfParts = 16;
__global__ __launch_bounds__(256) void k_confidence_part(const float *__restrict__ logits, int vocab, Rows rows, float *part) {
  __shared__ float smax[4], ssum[4];
  __shared__ int sidx[4];
  const int r = blockIdx.x, p = blockIdx.y;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  if (r >= M) return;
  const int chunk = ((vocab + kConfParts - 1) / kConfParts + 3) & ~3;
  const int c0 = min(p * chunk, vocab), c1 = min(c0 + chunk, vocab);
  const float *x = logits + (size_t)r * vocab;
  const bool vec = (((size_t)x) & 15) == 0;
  float m = -INFINITY;
  int mi = 0x7fffffff;
  const int nv = vec ? (c1 - c0) / 4 : 0;
  for (int i = threadIdx.x; i < nv; i += 256) {
    const float4 v = ((const float4 *)(x + c0))[i];
    const int at = c0 + 4 * i;
    if (v.x > m) { m = v.x; mi = at; }
    if (v.y > m) { m = v.y; mi = at + 1; }
    if (v.z > m) { m = v.z; mi = at + 2; }
    if (v.w > m) { m = v.w; mi = at + 3; }
  }
  for (int i = c0 + 4 * nv + threadIdx.x; i < c1; i += 256) {
    const float v = x[i];
    if (v > m) { m = v; mi = i; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o);
    const int oi = __shfl_xor(mi, o);
    if (om > m || (om == m && oi < mi)) { m = om; mi = oi; }
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { smax[w] = m; sidx[w] = mi; }
  __syncthreads();
  m = smax[0]; mi = sidx[0];
  for (int i = 1; i < 4; ++i)
    if (smax[i] > m || (smax[i] == m && sidx[i] < mi)) { m = smax[i]; mi = sidx[i]; }
  float sum = 0.f;
  for (int i = threadIdx.x; i < nv; i += 256) {
    const float4 v = ((const float4 *)(x + c0))[i];
    sum += __expf(v.x - m) + __expf(v.y - m) + __expf(v.z - m) + __expf(v.w - m);
  }
  for (int i = c0 + 4 * nv + threadIdx.x; i < c1; i += 256) sum += __expf(x[i] - m);
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if ((threadIdx.x & 63) == 0) ssum[w] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    float *o = part + ((size_t)r * kConfParts + p) * 3;
    o[0] = m;
    o[1] = __int_as_float(mi);
    o[2] = c1 > c0 ? ssum[0] + ssum[1] + ssum[2] + ssum[3] : 0.f;
  }
}

__global__ __launch_bounds__(256) void k_confidence_merge(const float *__restrict__ part, Rows rows, float *conf, int32_t *argmax) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  if (r >= M) return;
  const float *p = part + (size_t)r * kConfParts * 3;
  float m = -INFINITY;
  int mi = 0x7fffffff;
  for (int i = 0; i < kConfParts; ++i) {
    const float pm = p[3 * i];
    const int pi = __float_as_int(p[3 * i + 1]);
    if (pm > m || (pm == m && pi < mi)) { m = pm; mi = pi; }
  }
  float sum = 0.f;
  for (int i = 0; i < kConfParts; ++i) sum += p[3 * i + 2] * __expf(p[3 * i] - m);   // an empty part has sum 0 and maximum -inf: adds 0
  conf[r] = 1.0f / sum;
  argmax[r] = mi;
}

// Merge of the per-wavefront triples that the fused vocabulary projection leaves (gemm_conf_partials): one wavefront per row,
// lane l folds slots l, l + 64, ... in ascending order, then the lanes are merged; equal maxima keep the lower column.
__global__ __launch_bounds__(256) void k_confidence_slots(const float *__restrict__ part, int n_slots, Rows rows, float *conf, int32_t *argmax) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  if (r >= M) return;
  const float *p = part + (size_t)r * n_slots * 3;
  float m = -INFINITY, sum = 0.f;
  int mi = 0x7fffffff;
  for (int i = lane; i < n_slots; i += 64) conf_merge(p[3 * i], __float_as_int(p[3 * i + 2]), p[3 * i + 1], m, mi, sum);
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o), os = __shfl_xor(sum, o);
    const int oi = __shfl_xor(mi, o);
    conf_merge(om, oi, os, m, mi, sum);
  }
  if (lane == 0) {
    conf[r] = 1.0f / sum;
    argmax[r] = mi;
  }
}

void confidence_from_partials(hipStream_t s, const float *part, int n_slots, Rows rows, float *conf, int32_t *argmax) {
  if (rows.cap > 0) k_confidence_slots<<<(rows.cap + 3) / 4, 256, 0, s>>>(part, n_slots, rows, conf, argmax);
}

void confidence(hipStream_t s, const float *logits, int vocab, Rows rows, float *conf, int32_t *argmax, Scratch scratch) {
  if (rows.cap <= 0) return;
  if (rows.cap <= 512 && vocab >= 16384 && scratch.ptr && scratch.bytes >= (size_t)rows.cap * kConfParts * 12) {
    k_confidence_part<<<dim3(rows.cap, kConfParts), 256, 0, s>>>(logits, vocab, rows, (float *)scratch.ptr);
    k_confidence_merge<<<(rows.cap + 255) / 256, 256, 0, s>>>((const float *)scratch.ptr, rows, conf, argmax);
    return;
  }
  k_confidence<<<rows.cap, 256, 0, s>>>(logits, vocab, rows, conf, argmax);
}

// ---------------------------------------------------------------------------------------------
// Decode_and_Verify (Alg. 1) per sequence: lane i holds the i-th retained row.  Masked survivors with
// confidence >= threshold are unmasked with their arg-max token; if none passes, the most confident masked
// survivor is (ties: lower position), so a block always makes progress.  Statistics (App. E.3.1):
// token_sum += number unmasked, total_steps += 1, for every sequence that had rows in this step.
__global__ __launch_bounds__(64) void k_commit(CommitArgs a) {
  const int b = blockIdx.x, i = threadIdx.x, B = a.B;
  const int slot = slot_of(a.seq_slot, b, a.st);
  const uint64_t keep = a.keep_bits[b] & low_bits(B);
  const int nk = __popcll(keep);
  uint64_t masked = a.st.mask_bits[slot];
  int n_dec = 0;
  if (nk > 0) {
    // position of lane i's row: the i-th set bit of keep
    int p = -1;
    if (i < nk) {
      uint64_t k = keep;
      for (int c = 0; c < i; ++c) k &= k - 1;
      p = __ffsll((long long)k) - 1;
    }
    const int row = a.cu[b] + i;
    const float c = i < nk ? a.conf[row] : -INFINITY;
    const int tok = i < nk ? a.argmax[row] : 0;
    const bool cand = i < nk && ((masked >> p) & 1ull);
    uint64_t pass = __ballot(cand && c >= a.threshold);
    const uint64_t cands = __ballot(cand);
    if (!pass && cands) {
      // most confident candidate, lower lane (= lower position) on ties
      float best = -INFINITY;
      int bi = -1;
      for (int l = 0; l < nk; ++l) {
        float cl = __shfl(c, l);
        if (((cands >> l) & 1ull) && (bi < 0 || cl > best)) { best = cl; bi = l; }
      }
      pass = 1ull << bi;
    }
    const bool mine = (pass >> i) & 1ull;
    if (mine) a.st.tokens[slot * B + p] = tok;
    uint64_t cleared = 0;
    for (int l = 0; l < nk; ++l) {
      int pl = __shfl(p, l);
      if ((pass >> l) & 1ull) cleared |= 1ull << pl;
    }
    masked &= ~cleared;
    n_dec = __popcll(pass);
    if (i == 0) {
      const uint64_t before = a.st.mask_bits[slot];
      a.st.mask_bits[slot] = masked;
      a.st.token_sum[slot] += n_dec;
      a.st.total_steps[slot] += 1;
      if (a.intra_block_cache) {
        // neighbour-aware stability (Sec. 4.3): a retained position that was decoded before this step, and whose right
        // neighbour was too (the last position has none), went through this forward with its final context: freeze it
        const uint64_t all = low_bits(B), unm = all & ~before;
        a.st.cached_bits[slot] |= keep & unm & ((unm >> 1) | (1ull << (B - 1)));
      }
    }
  }
  __syncthreads();
  if (a.tokens_out && i < B) {
    bool m = (masked >> i) & 1ull;
    a.tokens_out[(size_t)b * B + i] = m ? a.mask_id : a.st.tokens[slot * B + i];
  }
  if (i == 0) {
    if (a.mask_out) a.mask_out[b] = masked;
    if (a.n_decoded_out) a.n_decoded_out[b] = n_dec;
  }
}

__global__ void k_uncached_bits(int n_seq, int B, const int32_t *seq_slot, SlotState st, uint64_t *bits) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < n_seq) bits[b] = low_bits(B) & ~st.cached_bits[slot_of(seq_slot, b, st)];
}

void uncached_bits(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st, uint64_t *bits) {
  if (n_seq > 0) k_uncached_bits<<<(n_seq + 255) / 256, 256, 0, s>>>(n_seq, B, seq_slot, st, bits);
}

void commit(hipStream_t s, const CommitArgs &a) {
  if (a.n_seq > 0) k_commit<<<a.n_seq, 64, 0, s>>>(a);
}

}  // namespace fk
