// Mixture-of-experts feed-forward (the second model of Sec. 5.1 is an MoE; the layer is the common token-choice one):
// routing, sorting the (row, expert) entries by expert, the two grouped projections of the SwiGLU experts, and the
// weighted sum back into the residual stream.
//
// With k of E experts per row and a few thousand rows per step an expert sees a few dozen rows, so the grouped
// projections are bound by streaming the expert weights from HBM once, not by the matrix cores: the kernel keeps two
// K-slabs of weights in flight per workgroup and two workgroups per CU (LDS stages filled by direct-to-LDS loads), and
// the matrix work hides underneath.  Everything is deterministic: entries are placed by prefix sums, never in the order
// atomics happen to arrive, and a row's result does not depend on which other rows share its tile.
#include <algorithm>

#include "focus_internal.h"

namespace fk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ int moe_rows(const Rows &rows) { return rows.count ? min(*rows.count, rows.cap) : rows.cap; }

// ---------------------------------------------------------------------------------------------
// Routing: one wavefront per row.  The k largest router logits in descending order (ties: lower expert), or the
// caller's forced list; weights = softmax over the chosen logits (the full softmax's denominator cancels in the
// renormalised top-k probabilities), times route_scale.  E <= 512: lane l holds experts l, l + 64, ...
__global__ __launch_bounds__(256) void k_moe_route(MoeArgs a) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int M = moe_rows(a.rows), E = a.n_experts, k = a.k;
  if (row >= M) return;
  const float *lg = a.logits + (size_t)row * E;
  const int rid = a.row_map ? a.row_map[row] : row;
  float val = -INFINITY;      // lane j < k ends up with the j-th chosen logit and expert
  int idx = 0;
  if (a.route_override) {
    if (lane < k) {
      idx = min(max(a.route_override[(size_t)rid * k + lane], 0), E - 1);
      val = lg[idx];
    }
  } else {
    float v[8];
    unsigned gone = 0;        // bit i: expert lane + 64 i is taken or does not exist
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = lane + 64 * i;
      v[i] = e < E ? lg[e] : -INFINITY;
      v[i] = v[i] != v[i] ? -INFINITY : v[i];
      gone |= e < E ? 0u : 1u << i;
    }
    for (int j = 0; j < k; ++j) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (!((gone >> i) & 1u) && (bi == 0x7fffffff || v[i] > bv)) { bv = v[i]; bi = lane + 64 * i; }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        const float ov = __shfl_xor(bv, d);
        const int oi = __shfl_xor(bi, d);
        if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
      }
      if ((bi & 63) == lane) gone |= 1u << (bi >> 6);
      if (lane == j) { val = bv; idx = bi; }
    }
  }
  // softmax over the chosen logits, summed in choice order
  float m = -INFINITY;
  for (int j = 0; j < k; ++j) m = fmaxf(m, __shfl(val, j));
  const float ex = lane < k ? __expf(val - m) : 0.f;
  float sum = 0.f;
  for (int j = 0; j < k; ++j) sum += __shfl(ex, j);
  if (lane < k) {
    const float w = a.route_scale * ex / sum;
    a.topk_idx[(size_t)row * k + lane] = idx;
    a.topk_w[(size_t)row * k + lane] = w;
    if (a.out_experts) a.out_experts[(size_t)rid * k + lane] = idx;
    if (a.out_weights) a.out_weights[(size_t)rid * k + lane] = w;
  }
}

void moe_route(hipStream_t s, const MoeArgs &a) {
  if (a.rows.cap > 0) k_moe_route<<<(a.rows.cap + 3) / 4, 256, 0, s>>>(a);
}

// ---------------------------------------------------------------------------------------------
// Entries of expert e = blockIdx.x, in a fixed order: the workgroup walks all M * k entries, 1024 per trip (lane t looks
// at entries 4 t .. 4 t + 3 of the trip), and places the matches by ballot prefix sums.
__global__ __launch_bounds__(256) void k_moe_list(MoeArgs a) {
  __shared__ int wave_cnt[4];
  const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = moe_rows(a.rows) * a.k;
  int32_t *list = a.list + (size_t)e * a.rows.cap;
  int base = 0;
  for (int i0 = 0; i0 < n; i0 += 1024) {
    const int i = i0 + tid * 4;
    const int4 t = *(const int4 *)(a.topk_idx + i);        // the buffer is padded; entries beyond n are masked
    const int ids[4] = {t.x, t.y, t.z, t.w};
    int before = 0, mine[4];
    bool hit[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      hit[j] = i + j < n && ids[j] == e;
      const uint64_t b = __ballot(hit[j]);
      mine[j] = before + __popcll(b & ((1ull << lane) - 1));
      before += __popcll(b);
    }
    wave_cnt[wave] = before;
    __syncthreads();
    int off = base, total = 0;
    for (int w = 0; w < 4; ++w) { off += w < wave ? wave_cnt[w] : 0; total += wave_cnt[w]; }
    // a row names an expert at most once, so an expert has at most rows.cap entries; a forced list that repeats an
    // expert could exceed that: the surplus is dropped rather than written past the list
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (hit[j] && off + mine[j] < a.rows.cap) list[off + mine[j]] = i + j;
    base += total;
    __syncthreads();
  }
  if (tid == 0) a.count[e] = min(base, a.rows.cap);
}

// Expert-sorted rows: offs = exclusive prefix sum of the counts; entry list[e][j] becomes row offs[e] + j.  Also the list
// of (expert, first row) tiles of kMoeTileRows rows that the grouped projections walk.
__global__ __launch_bounds__(256) void k_moe_place(MoeArgs a) {
  __shared__ int s_sum[4];     // rows before this expert, tiles before it, all rows, all tiles (integer adds: order-free)
  const int e = blockIdx.x, tid = threadIdx.x, E = a.n_experts;
  if (tid < 4) s_sum[tid] = 0;
  __syncthreads();
  int rows_lt = 0, tiles_lt = 0, rows_all = 0, tiles_all = 0;
  for (int i = tid; i < E; i += 256) {
    const int c = a.count[i], t = (c + kMoeTileRows - 1) / kMoeTileRows;
    rows_all += c; tiles_all += t;
    if (i < e) { rows_lt += c; tiles_lt += t; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    rows_lt += __shfl_xor(rows_lt, o); tiles_lt += __shfl_xor(tiles_lt, o);
    rows_all += __shfl_xor(rows_all, o); tiles_all += __shfl_xor(tiles_all, o);
  }
  if ((tid & 63) == 0) {
    atomicAdd(&s_sum[0], rows_lt); atomicAdd(&s_sum[1], tiles_lt); atomicAdd(&s_sum[2], rows_all); atomicAdd(&s_sum[3], tiles_all);
  }
  __syncthreads();
  const int off = s_sum[0], first_tile = s_sum[1], cnt = a.count[e], k = a.k;
  if (tid == 0) {
    a.offs[e] = off;
    if (e == 0) { a.offs[E] = s_sum[2]; *a.n_tiles = min(s_sum[3], a.n_tile_slots); }
  }
  const int32_t *list = a.list + (size_t)e * a.rows.cap;
  for (int j = tid; j < cnt; j += 256) {
    const int ent = list[j];
    a.pos[ent] = off + j;
    a.arow[off + j] = ent / k;
    a.aexp[off + j] = e;
  }
  for (int m = tid; m * kMoeTileRows < cnt; m += 256)
    if (first_tile + m < a.n_tile_slots) { a.tile_e[first_tile + m] = e; a.tile_m0[first_tile + m] = m * kMoeTileRows; }
}

void moe_group(hipStream_t s, const MoeArgs &a) {
  if (a.rows.cap <= 0) return;
  k_moe_list<<<a.n_experts, 256, 0, s>>>(a);
  k_moe_place<<<a.n_experts, 256, 0, s>>>(a);
}

// ---------------------------------------------------------------------------------------------
// Grouped projection on the matrix cores: out[row] = A[src(row)] * W[expert(row)]^T for the expert-sorted rows.
// A workgroup (4 wavefronts, 2 x 2, each 64 x 64) takes one tile of up to 128 rows of one expert and 128 rows of that
// expert's weight matrix, so that with the usual few dozen rows per expert every weight byte is fetched by exactly one
// workgroup.  K-slabs of 64 go straight into LDS (buffer_load_dwordx4 ... lds, chunk-swizzled like the dense kernel):
// three stages for the weights (two slabs in flight: they come from HBM), two for the rows (one in flight: they come
// from the L2), 80 KB in all, so two workgroups share a CU and one streams while the other starts or stores.
// Rows beyond the expert's count and weight rows beyond N fall outside the buffer descriptors and read as zero.
//   GG_GATE_UP: W = [Fe gate rows; Fe up rows] per expert; LDS weight rows 64 c .. 64 c + 31 are the gate rows of output
//               columns 32 c .., the next 32 the matching up rows; out[bf16][row, col] = silu(gate) * up.
//   GG_DOWN:    out[f32][row, col] = acc.
//   GG_DENSE_PARTIAL, GG_DENSE_PARTIAL_SILU: the same stream for a dense projection of few rows: one weight matrix, rows in
//               place, K cut into `splits` ranges of which a workgroup takes one; fp32 partial sums out (gemm_stream_partial).
struct GroupGemm {
  const bf16_t *A;
  unsigned a_bytes;            // size of A (for the descriptor)
  const int32_t *src;          // expert-sorted row -> row of A, or null (identity)
  const bf16_t *W;             // [E, N, K]
  int N, K;
  const int32_t *offs, *count, *tile_e, *tile_m0, *n_tiles;
  int tiles_n;
  void *out;
  int ldo;
  // dense modes (one weight matrix, rows in place, K cut into `splits` parts that write fp32 partial sums)
  Rows rows;
  int tiles_m, splits;
  size_t split_stride;
};
enum { GG_DOWN = 0, GG_GATE_UP = 1, GG_DENSE_PARTIAL = 2, GG_DENSE_PARTIAL_SILU = 3 };

#define FK_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }   // s_waitcnt vmcnt(n) only
constexpr int kGroupLds = (2 * kMoeTileRows + 3 * 128) * 128;

template <int MODE>
__global__ __launch_bounds__(256, 2) void k_group_gemm(GroupGemm g) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer-resource builtins exist in the device pass only
  constexpr bool GATE_UP = MODE == GG_GATE_UP || MODE == GG_DENSE_PARTIAL_SILU, DENSE = MODE >= GG_DENSE_PARTIAL;
  constexpr int BM = kMoeTileRows, BN = 128, ASTAGE = BM * 128, WSTAGE = BN * 128, WBASE = 2 * ASTAGE;
  constexpr int IA = BM / 8 / 4, IB = BN / 8 / 4;   // load instructions per wavefront and slab
  static_assert(BM == 128, "wavefront layout below is 2 x 2 of 64 x 64");
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_group[];
  unsigned char *const lds = lds_group;
  // work item = weight tile nt of row tile t, nt fastest; XCD x (workgroups x, x + 8, ...) takes a contiguous range, so
  // the workgroups that read the same rows share an L2
  const int splits = DENSE ? g.splits : 1;
  const int n_tiles = DENSE ? g.tiles_m : *g.n_tiles, total = n_tiles * g.tiles_n * splits, per_xcd = (total + 7) / 8;
  const int item = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if ((int)(blockIdx.x / 8) >= per_xcd || item >= total) return;
  const int split = item % splits, t = item / splits / g.tiles_n, nt = item / splits % g.tiles_n;
  int e = 0, m0 = t * BM, row0 = m0, valid;
  if (DENSE) {
    valid = min(BM, (g.rows.count ? min(*g.rows.count, g.rows.cap) : g.rows.cap) - m0);
    if (valid <= 0) return;
  } else {
    e = g.tile_e[t]; m0 = g.tile_m0[t];
    row0 = g.offs[e] + m0; valid = min(BM, g.count[e] - m0);
  }
  const int N = g.N, K = g.K, n0 = nt * (GATE_UP ? BN / 2 : BN);
  const int nk = K / 64 / splits;                      // slabs of this workgroup
  const unsigned k_base = (unsigned)split * (unsigned)nk * 128u;
  float *const out_part = (float *)g.out + (size_t)split * g.split_stride;   // dense modes
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)g.A, 0, g.a_bytes, 0x00020000);
  __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)(g.W + (size_t)e * N * K), 0, (unsigned)N * (unsigned)K * 2u, 0x00020000);
  unsigned voa[IA], vob[IB];
#pragma unroll
  for (int q = 0; q < IA; ++q) {
    const int r = (wave * IA + q) * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    const int srow = r < valid ? (g.src ? g.src[row0 + r] : row0 + r) : -1;
    voa[q] = srow < 0 ? 0x80000000u : (unsigned)srow * (unsigned)K * 2u + k_base + c * 16;
  }
#pragma unroll
  for (int q = 0; q < IB; ++q) {
    const int r = (wave * IB + q) * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    const int wrow = GATE_UP ? ((r >> 5) & 1) * (N / 2) + n0 + (r / 64) * 32 + (r & 31) : n0 + r;
    const bool ok = GATE_UP ? n0 + (r / 64) * 32 + (r & 31) < N / 2 : wrow < N;
    vob[q] = ok ? (unsigned)wrow * (unsigned)K * 2u + k_base + c * 16 : 0x80000000u;
  }
  // slab kt of an operand into a stage; beyond the last slab the offset is out of range: nothing moves
  auto issue_a = [&](int kt, int stage) {
    const unsigned so = kt < nk ? (unsigned)kt * 128u : 0x80000000u;
#pragma unroll
    for (int q = 0; q < IA; ++q)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, FK_LDS_PTR(lds + stage * ASTAGE + (wave * IA + q) * 1024), 16, voa[q], so, 0, 0);
  };
  auto issue_w = [&](int kt, int stage) {
    const unsigned so = kt < nk ? (unsigned)kt * 128u : 0x80000000u;
#pragma unroll
    for (int q = 0; q < IB; ++q)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, FK_LDS_PTR(lds + WBASE + stage * WSTAGE + (wave * IB + q) * 1024), 16, vob[q], so, 0, 0);
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int frow = lane & 31, fch = lane >> 5, sw = (frow >> 1) & 7;
  issue_a(0, 0);
  issue_w(0, 0);
  issue_w(1, 1);
  int ws = 0;   // weight stage of slab kt
  for (int kt = 0; kt < nk; ++kt) {
    // loads are issued in the order ... rows(kt), weights(kt + 1): all but the youngest IB have landed = slab kt is complete
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(IB));
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // ... for every wavefront; and everyone has finished slab kt - 1
    issue_a(kt + 1, (kt + 1) & 1);                    // into the stages slab kt - 1 occupied
    issue_w(kt + 2, ws == 0 ? 2 : ws - 1);
    const unsigned char *sa = lds + (kt & 1) * ASTAGE, *sb = lds + WBASE + ws * WSTAGE;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[2], fb[2];
      const int ch = ((2 * ks + fch) ^ sw) << 4;
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = *(const bf16x8 *)(sa + (wm + i * 32 + frow) * 128 + ch);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = *(const bf16x8 *)(sb + (wn + j * 32 + frow) * 128 + ch);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    ws = ws == 2 ? 0 : ws + 1;
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  // accumulator register r of lane l is C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of its 32 x 32 tile
  const int erow = wm + 4 * (lane >> 5), ecol = lane & 31;
  if (MODE == GG_DENSE_PARTIAL_SILU) {   // fp32 partial sums in weight-row order: gate of column c at c, up at N / 2 + c
    const int gn = n0 + (wn / 64) * 32 + ecol;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
        if (gm < valid && gn < N / 2) {
          out_part[(size_t)(row0 + gm) * g.ldo + gn] = acc[i][0][r];
          out_part[(size_t)(row0 + gm) * g.ldo + N / 2 + gn] = acc[i][1][r];
        }
      }
  } else if (GATE_UP) {
    const int gn = n0 + (wn / 64) * 32 + ecol;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
        const float ga = acc[i][0][r], up = acc[i][1][r];
        if (gm < valid && gn < N / 2) ((bf16_t *)g.out)[(size_t)(row0 + gm) * g.ldo + gn] = (bf16_t)(ga / (1.0f + __expf(-ga)) * up);
      }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int gn = n0 + wn + j * 32 + ecol;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
          if (gm < valid && gn < N) (DENSE ? out_part : (float *)g.out)[(size_t)(row0 + gm) * g.ldo + gn] = acc[i][j][r];
        }
      }
  }
#endif
}

// Any element type, any shape: one output element per lane (fp32 models of the oracle-check size).
template <typename T, bool GATE_UP>
__global__ __launch_bounds__(256) void k_group_gemm_valu(const T *A, const int32_t *src, const T *W, int N, int K, const int32_t *offs,
                                                         const int32_t *aexp, int n_experts, void *out, int ldo) {
  const int row = blockIdx.x, total = offs[n_experts];
  if (row >= total) return;
  const int ncol = GATE_UP ? N / 2 : N;
  const int col = blockIdx.y * 256 + threadIdx.x;
  if (col >= ncol) return;
  const T *a = A + (size_t)(src ? src[row] : row) * K;
  const T *w = W + (size_t)aexp[row] * N * K;
  float d0 = 0.f, d1 = 0.f;
  for (int i = 0; i < K; ++i) {
    const float x = (float)a[i];
    d0 += x * (float)w[(size_t)col * K + i];
    if (GATE_UP) d1 += x * (float)w[(size_t)(N / 2 + col) * K + i];
  }
  if (GATE_UP) ((T *)out)[(size_t)row * ldo + col] = (T)(d0 / (1.0f + __expf(-d0)) * d1);
  else ((float *)out)[(size_t)row * ldo + col] = d0;
}

template <int MODE>
static bool launch_group(hipStream_t s, const GroupGemm &g, int n_tile_slots) {
  constexpr int kLds = kGroupLds;
  static bool ready = false;             // the dynamic LDS size has to be allowed once per kernel
  if (!ready) {
    if (hipFuncSetAttribute((const void *)k_group_gemm<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess) return false;
    ready = true;
  }
  k_group_gemm<MODE><<<((n_tile_slots * g.tiles_n * (MODE >= GG_DENSE_PARTIAL ? g.splits : 1) + 7) / 8) * 8, 256, kLds, s>>>(g);
  return true;
}

// Dense projection of few rows (at most a few 128-row tiles) as fp32 partial sums of `splits` K ranges, part[split][row][N]
// (SiLU variant: gate and up sums in weight-row order): the weight-streaming kernel above with one "expert".
bool gemm_stream_partial(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, bool silu, int splits, float *part) {
  if (K % (64 * splits) || (double)rows.cap * K * 2 >= 2.0e9 || (double)N * K * 2 >= 4.0e9 || ((uintptr_t)A & 15) || ((uintptr_t)W & 15)) return false;
  GroupGemm g{};
  g.A = (const bf16_t *)A; g.a_bytes = (unsigned)((size_t)rows.cap * K * 2); g.W = (const bf16_t *)W; g.N = N; g.K = K;
  g.tiles_n = silu ? (N / 2 + 63) / 64 : (N + 127) / 128;
  g.out = part; g.ldo = N; g.rows = rows; g.tiles_m = (rows.cap + kMoeTileRows - 1) / kMoeTileRows; g.splits = splits;
  g.split_stride = (size_t)rows.cap * N;
  return silu ? launch_group<GG_DENSE_PARTIAL_SILU>(s, g, g.tiles_m) : launch_group<GG_DENSE_PARTIAL>(s, g, g.tiles_m);
}

void moe_experts(hipStream_t s, const MoeArgs &a) {
  if (a.rows.cap <= 0) return;
  const int Fe = a.expert_ffn, h = a.hidden, cap = a.rows.cap * a.k;
  const bool mfma = a.dtype == FOCUS_BF16 && h % 64 == 0 && Fe % 64 == 0 && ((uintptr_t)a.u & 15) == 0 && ((uintptr_t)a.w_gate_up & 15) == 0 &&
                    ((uintptr_t)a.w_down & 15) == 0 && (double)a.rows.cap * h * 2 < 2.0e9 && (double)cap * Fe * 2 < 2.0e9 &&
                    (double)2 * Fe * h * 2 < 2.0e9;
  if (mfma) {
    GroupGemm g{(const bf16_t *)a.u, (unsigned)((size_t)a.rows.cap * h * 2), a.arow, (const bf16_t *)a.w_gate_up, 2 * Fe, h,
                a.offs, a.count, a.tile_e, a.tile_m0, a.n_tiles, (Fe + 63) / 64, a.act, Fe};
    GroupGemm d{(const bf16_t *)a.act, (unsigned)((size_t)cap * Fe * 2), nullptr, (const bf16_t *)a.w_down, h, Fe,
                a.offs, a.count, a.tile_e, a.tile_m0, a.n_tiles, (h + 127) / 128, a.y, h};
    if (launch_group<GG_GATE_UP>(s, g, a.n_tile_slots) && launch_group<GG_DOWN>(s, d, a.n_tile_slots)) return;
  }
  if (a.dtype == FOCUS_BF16) {
    k_group_gemm_valu<bf16_t, true><<<dim3(cap, (Fe + 255) / 256), 256, 0, s>>>((const bf16_t *)a.u, a.arow, (const bf16_t *)a.w_gate_up, 2 * Fe, h, a.offs, a.aexp, a.n_experts, a.act, Fe);
    k_group_gemm_valu<bf16_t, false><<<dim3(cap, (h + 255) / 256), 256, 0, s>>>((const bf16_t *)a.act, nullptr, (const bf16_t *)a.w_down, h, Fe, a.offs, a.aexp, a.n_experts, a.y, h);
  } else {
    k_group_gemm_valu<float, true><<<dim3(cap, (Fe + 255) / 256), 256, 0, s>>>((const float *)a.u, a.arow, (const float *)a.w_gate_up, 2 * Fe, h, a.offs, a.aexp, a.n_experts, a.act, Fe);
    k_group_gemm_valu<float, false><<<dim3(cap, (h + 255) / 256), 256, 0, s>>>((const float *)a.act, nullptr, (const float *)a.w_down, h, Fe, a.offs, a.aexp, a.n_experts, a.y, h);
  }
}

// ---------------------------------------------------------------------------------------------
// resid[row] += sum_j w[row, j] * y[pos[row * k + j]], j ascending (one workgroup per row)
__global__ __launch_bounds__(256) void k_moe_combine(MoeArgs a) {
  const int row = blockIdx.x;
  if (row >= moe_rows(a.rows)) return;
  const int k = a.k, h = a.hidden;
  float *r = a.resid + (size_t)row * h;
  for (int c = threadIdx.x * 4; c < h; c += 1024) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
      const float w = a.topk_w[(size_t)row * k + j];
      const float4 v = *(const float4 *)(a.y + (size_t)a.pos[(size_t)row * k + j] * h + c);
      acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
    }
    float4 o = *(float4 *)(r + c);
    o.x += acc.x; o.y += acc.y; o.z += acc.z; o.w += acc.w;
    *(float4 *)(r + c) = o;
  }
}

void moe_combine(hipStream_t s, const MoeArgs &a) {
  if (a.rows.cap > 0) k_moe_combine<<<a.rows.cap, 256, 0, s>>>(a);
}

}  // namespace fk
