// Block-diffusion attention over the paged K/V cache, and the token-importance reduction of Eq. 2.
//
// A query row (sequence b, block position p) attends to the sequence's whole prefix [0, L) and to the
// in-block positions whose bit is set in the sequence's visibility set (all B in the layers up to the
// eviction layer; the processed positions above it).  There is no mask inside the block (Sec. 1-2).
#include "focus_internal.h"

namespace fk {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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
    const T *vp = (const T *)kv.base + (size_t)pt[t / P] * page_elems + (size_t)(Hkv + hk) * P * D + (t % P);
    float s = 0.f;
    for (int e = 0; e < NE; ++e) s += qv[e] * to_f(kp[lane + 64 * e]);
    s = wave_sum(s);
    float mn = fmaxf(m, s);
    float corr = __expf(m - mn), pr = __expf(s - mn);
    l = l * corr + pr;
    for (int e = 0; e < NE; ++e) o[e] = o[e] * corr + pr * to_f(vp[(size_t)(lane + 64 * e) * P]);
    m = mn;
  }
  T *orow = out + (size_t)r * Hq * D + (size_t)hq * D;
  float inv = l > 0.f ? 1.0f / l : 0.f;
  for (int e = 0; e < NE; ++e) orow[lane + 64 * e] = (T)(o[e] * inv);
}

// ---------------------------------------------------------------------------------------------
// bf16 attention on the matrix cores, one workgroup per (sequence, kv head, K/V split).
//
// All query rows of the sequence that share the kv head (rows x group heads, up to 32 per wavefront) are
// multiplied against each 64-token K/V tile, so the K/V stream is read from HBM once per (sequence, kv head)
// whatever the number of rows: the kernel is bound by that stream.
//
// Per tile and wavefront:  S^T = K Q^T  (v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q held in
// registers), so that a lane owns one query row and its scores sit in its own registers: the online-softmax
// max/sum are in-lane reductions plus one exchange between lanes l and l + 32.  O^T = V^T P^T then takes
// the probabilities straight from those registers as the B operand.  For that, lane l of the first product
// loads K row sigma(l % 32) (bits 2 and 3 swapped) instead of l % 32, which makes the eight probabilities a
// lane holds for one product belong to eight consecutive tokens; V is cached transposed ([D][tokens]), so
// the matching A operand is one 16-byte LDS read.
//
// LDS: K tile [64 tokens][128] and V^T tile [128][64 tokens], 16-byte chunks XOR-swizzled against bank
// conflicts; the next tile is fetched into registers while the current one is used.
// A page (64 tokens) is one tile.  Long sequences are cut into splits of `chunk` tokens; a split writes
// un-normalised partial outputs and (max, sum), merged in split order by k_attn_combine.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int sigma32(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// s_waitcnt immediate that waits for at most n outstanding vector-memory operations and for nothing else
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

#define FK_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define FK_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// BJ > 0: the kernel also reduces the in-block score tile to the token importance of Eq. 2 (blocks of up to BJ positions); its LDS
// is then dynamic: the two tile buffers, a score patch of 32 x (BJ + 1) floats per wavefront, and per-wavefront column sums.
template <int NW, int BJ = 0>
__global__ __launch_bounds__(NW * 64, 2) void k_attn_mfma(AttnArgs a) {
  constexpr int D = 128, P = 64, IPW = 16 / NW;       // 1 KB load instructions per wavefront for K, and for V
  constexpr bool IMP = BJ > 0;
  __shared__ __attribute__((aligned(1024))) unsigned char lds_fixed[IMP ? 1024 : 32768];
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_imp[];
  unsigned char *const lds = IMP ? lds_imp : lds_fixed;
  const int Hkv = a.kv.n_kv_heads, Hq = a.n_q_heads, g = Hq / Hkv;
  const int bo = blockIdx.x / Hkv, hk = blockIdx.x % Hkv, split = blockIdx.y;
  const int b = a.order ? a.order[bo] : bo;
  const int r0 = a.cu[b], nr = a.cu[b + 1] - r0;
  if (nr <= 0) {
    if (BJ > 0 && a.imp_partial && split == 0)           // a sequence without query rows: its importance sums are zero
      for (int i = threadIdx.x; i < g * a.ri.B; i += NW * 64) a.imp_partial[((size_t)b * Hq + hk * g) * a.ri.B + i] = 0.f;
    return;
  }
  const int slot = slot_of(a.ri.seq_slot, b, a.st);
  const int L = a.st.prefix_len[slot], total = L + a.ri.B;
  // Splits that have tokens: the sequence's own length decides (it is read here, on the device), bounded by the number of
  // split workgroups this launch has; the last one takes everything that is left.  So a launch whose geometry was fixed when
  // the prefixes were shorter (a captured graph replayed after blocks became prefix) still attends to every token.
  const int nsplit = min((total + a.chunk - 1) / a.chunk, (int)gridDim.y);
  if (split >= nsplit) return;
  const int t0 = split * a.chunk;
  const int t1 = split == nsplit - 1 ? total : t0 + a.chunk;
  const uint64_t vis = a.vis_by_b ? a.vis_by_b[b] : ~0ull;
  const int32_t *pt = a.st.page_table + (size_t)slot * a.st.table_stride;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, col = lane & 31;
  // fused importance: only the workgroup of the last K/V range of the sequence (it is the one that ends with the block's tokens)
  const bool do_imp = IMP && a.imp_partial != nullptr && split == nsplit - 1;
  float *const imp_scores = (float *)(lds + 32768) + wave * 32 * (BJ + 1);              // [32 pairs][BJ + 1]
  float *const imp_wsum = (float *)(lds + 32768) + NW * 32 * (BJ + 1);                  // [NW][g][BJ]
  if (do_imp)
    for (int i = tid; i < NW * g * BJ; i += NW * 64) imp_wsum[i] = 0.f;                  // (barriers of the tile loop order this)

  // Tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l of an instruction fills
  // the 16-byte slot l of a 1 KB LDS block), so the swizzle is applied on the global side: the lane that owns
  // slot (row, position p) fetches the chunk that belongs there.  K block = 4 token rows x 16 chunks,
  // chunk c of token t sits at position c ^ (t & 15); V^T block = 8 d rows x 8 chunks, chunk c of row d at
  // position c ^ ((d >> 1) & 7).  Both make the 16 rows that one LDS read cycle serves hit 16 distinct
  // 16-byte bank groups.
  const size_t page_bytes = (size_t)2 * Hkv * P * D * 2;
  const unsigned char *pool = (const unsigned char *)a.kv.base;
  const size_t k_head = (size_t)hk * P * D * 2, v_head = ((size_t)Hkv * P * D + (size_t)hk * D * P) * 2;
  int gk[IPW], gv[IPW];                                // per-lane byte offsets inside the K / V^T tile
#pragma unroll
  for (int q = 0; q < IPW; ++q) {
    const int blk = wave * IPW + q;
    const int tok = 4 * blk + (lane >> 4), pk = lane & 15;
    gk[q] = tok * 256 + ((pk ^ (tok & 15)) << 4);
    const int d = 8 * blk + (lane >> 3), pv = lane & 7;
    gv[q] = d * 128 + ((pv ^ ((d >> 1) & 7)) << 4);
  }
  unsigned char *const Ks = lds, *const Vs = lds + 16384;
  // Page ids of the next 64 tiles are kept in one register (lane i = tile base + i) and broadcast with
  // readlane, so a tile's loads never wait for a dependent page-table read.
  const int tile0 = t0 / 64, tile1 = (t1 + 63) / 64;
  int ptreg = pt[min(tile0 + lane, tile1 - 1)];
  auto page_of = [&](int tile) { return (size_t)__builtin_amdgcn_readlane(ptreg, (tile - tile0) & 63); };
  auto issue_k = [&](int tile) {
    const unsigned char *pg = pool + page_of(tile) * page_bytes + k_head;
#pragma unroll
    for (int q = 0; q < IPW; ++q)
      __builtin_amdgcn_global_load_lds(FK_GLB_PTR(pg + gk[q]), FK_LDS_PTR(Ks + (wave * IPW + q) * 1024), 16, 0, 0);
  };
  auto issue_v = [&](int tile) {
    const unsigned char *pg = pool + page_of(tile) * page_bytes + v_head;
#pragma unroll
    for (int q = 0; q < IPW; ++q)
      __builtin_amdgcn_global_load_lds(FK_GLB_PTR(pg + gv[q]), FK_LDS_PTR(Vs + (wave * IPW + q) * 1024), 16, 0, 0);
  };

  const float sc = 1.4426950408889634f / sqrtf((float)D);      // scores in the log2 domain
  // The workgroup holds NW * 32 (row, group head) pairs at a time.  The launch is sized for the rows a sequence is expected
  // to have; a sequence with more takes further passes over its K/V range (correct for any row count, one stream per pass).
  const int RT = nr * g;
  for (int q0 = 0; q0 < RT; q0 += NW * 32) {
  const int R = min(RT - q0, NW * 32);
  const int qi = q0 + wave * 32 + col;
  const bool wave_has_rows = wave * 32 < R, qvalid = wave * 32 + col < R;
  const int qrow = r0 + (qvalid ? qi / g : 0), qhead = hk * g + (qvalid ? qi % g : 0);
  bf16x8 qf[8];
  {
    const bf16_t *qp = (const bf16_t *)a.q + (size_t)qrow * a.q_stride + (size_t)qhead * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 v = qvalid ? *(const u32x4 *)(qp + 16 * ks) : (u32x4){0, 0, 0, 0};
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  if (q0 > 0) {                                                // a further pass starts from the first tile again
    ptreg = pt[min(tile0 + lane, tile1 - 1)];
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();
  }
  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  // One K buffer and one V^T buffer, refilled as soon as the product that reads them is done: the K tile of
  // the next step streams in during this step's softmax and P V product, the V tile during the next step's
  // K Q^T product.  Loads complete in issue order, so "at most IPW outstanding" means the older tile landed.
  issue_k(tile0);
  issue_v(tile0);
  for (int tile = tile0; tile < tile1; ++tile) {
    const bool more = tile + 1 < tile1;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(IPW));          // K(tile) is in LDS
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    f32x16 sacc[2];
    if (wave_has_rows) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
        const int tl = 32 * u + sigma32(col);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const int ch = 2 * ks + half;
          bf16x8 kf = *(const bf16x8 *)(Ks + tl * 256 + ((ch ^ (tl & 15)) << 4));
          sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[u], 0, 0, 0);
        }
      }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();                        // every wavefront has read the K tile
    if (more && ((tile + 1 - tile0) & 63) == 0) {        // next batch of page ids (drains the queue: once per 64 tiles)
      ptreg = pt[min(tile + 1 + lane, tile1 - 1)];
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    if (more) issue_k(tile + 1);
    bf16x8 pf[4];
    if (wave_has_rows) {
      // mask, running maximum (of the raw scores: the scale is positive and is folded into the exponent's multiply-add)
      const bool need_mask = tile * 64 + 64 > L;
      float mx = -INFINITY;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float s = sacc[u][r];
          if (need_mask) {
            const int tok = tile * 64 + 32 * u + sigma32(8 * (r >> 2) + 4 * half + (r & 3));
            const bool ok = tok < L || (tok < total && ((vis >> (tok - L)) & 1ull));
            s = ok ? s : -INFINITY;
            sacc[u][r] = s;
          }
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * sc;
      const float m_new = fmaxf(m, mx);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m - m_use);
      m = m_new;
      float ls = 0.f;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[u][r], sc, -m_use));
          ls += p;
          pf[2 * u + (r >> 3)][r & 7] = (bf16_t)p;
        }
      l = l * corr + ls;
      // the 64 output accumulators are rescaled only when some row's maximum moved (after the first tiles it rarely does)
      if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
      }
    }
    if (more) __builtin_amdgcn_s_waitcnt(vmcnt_imm(IPW)); else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // V(tile) is in LDS
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (wave_has_rows) {
#pragma unroll
      for (int ds = 0; ds < 4; ++ds) {
        const int vr = 32 * ds + col;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          bf16x8 vf = *(const bf16x8 *)(Vs + vr * 128 + (((2 * kk + half) ^ ((vr >> 1) & 7)) << 4));
          oacc[ds] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kk], oacc[ds], 0, 0, 0);
        }
      }
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();                        // every wavefront has read the V tile
    if (more) issue_v(tile + 1);
  }

  const float l_tot = l + __shfl_xor(l, 32);
  if (qvalid) {
  if (nsplit == 1) {
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    bf16_t *orow = (bf16_t *)a.out + (size_t)qrow * Hq * D + (size_t)qhead * D;
#pragma unroll
    for (int ds = 0; ds < 4; ++ds)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(oacc[ds][4 * q4 + e] * inv);
        *(bf16x4 *)(orow + 32 * ds + 8 * q4 + 4 * half) = v;
      }
  } else {
    const size_t pi = ((size_t)qrow * Hq + qhead) * a.max_splits + split;
    float *po = a.part_o + pi * D;
#pragma unroll
    for (int ds = 0; ds < 4; ++ds)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = make_float4(oacc[ds][4 * q4], oacc[ds][4 * q4 + 1], oacc[ds][4 * q4 + 2], oacc[ds][4 * q4 + 3]);
        *(float4 *)(po + 32 * ds + 8 * q4 + 4 * half) = v;
      }
    if (half == 0) {
      a.part_ml[pi * 2] = m;
      a.part_ml[pi * 2 + 1] = l_tot;
    }
  }
  }   // qvalid
  if constexpr (IMP) {
    if (do_imp) {
      // Eq. 2 for this pass's (row, head) pairs: scores against the block's own B keys (the one or two tiles that hold positions
      // L .. L + B - 1 are fetched again: they were just streamed and sit in the L2), MaxPool1D along the keys, softmax over the
      // B keys, sums over the rows of every head.  The query fragments are still in registers.
      const int B = a.ri.B, tb0 = L / 64, tb1 = (total - 1) / 64;
      for (int tile = tb0; tile <= tb1; ++tile) {
        __builtin_amdgcn_s_barrier();                      // the K buffer is free
        const unsigned char *pg = pool + (size_t)__builtin_amdgcn_readfirstlane(pt[tile]) * page_bytes + k_head;
#pragma unroll
        for (int q = 0; q < IPW; ++q)
          __builtin_amdgcn_global_load_lds(FK_GLB_PTR(pg + gk[q]), FK_LDS_PTR(Ks + (wave * IPW + q) * 1024), 16, 0, 0);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (wave_has_rows) {
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            f32x16 sc2;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc2[r] = 0.f;
            const int tl = 32 * u + sigma32(col);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
              const int ch = 2 * ks + half;
              bf16x8 kf = *(const bf16x8 *)(Ks + tl * 256 + ((ch ^ (tl & 15)) << 4));
              sc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc2, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int j = tile * 64 + 32 * u + sigma32(8 * (r >> 2) + 4 * half + (r & 3)) - L;
              if (j >= 0 && j < B) imp_scores[col * (BJ + 1) + j] = sc2[r] * sc;     // log2 domain
            }
          }
        }
        asm volatile("" ::: "memory");
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
      if (wave_has_rows) {
        float row[BJ];
#pragma unroll
        for (int j = 0; j < BJ; ++j) row[j] = j < B ? imp_scores[col * (BJ + 1) + j] : -INFINITY;
        float mrow = -INFINITY;
#pragma unroll
        for (int j = 0; j < BJ; ++j) mrow = fmaxf(mrow, row[j]);                     // the pooled row has the same maximum
        float pooled[BJ], sum = 0.f;
#pragma unroll
        for (int j = 0; j < BJ; ++j) {
          float v = row[j];
          if (a.imp_pool_k == 3) {
            if (j > 0) v = fmaxf(v, row[j - 1]);
            if (j + 1 < BJ) v = fmaxf(v, row[j + 1]);
          }
          v = j < B ? __builtin_amdgcn_exp2f(v - mrow) : 0.f;                        // no position beyond the block takes part
          pooled[j] = v;
          sum += v;
        }
        const float inv = qvalid ? 1.0f / sum : 0.f;                                // lanes without a pair add nothing
#pragma unroll
        for (int j = 0; j < BJ; ++j) {
          float v = pooled[j] * inv;
          for (int o = g; o < 32; o <<= 1) v += __shfl_xor(v, o);                    // over the rows: lanes with the same col % g
          if (half == 0 && col < g && j < B) imp_wsum[(wave * g + col) * BJ + j] += v;
        }
      }
    }
  }
  }   // passes
  if constexpr (IMP) {
    if (do_imp) {
      __syncthreads();
      const int B = a.ri.B;
      for (int i = tid; i < g * BJ; i += NW * 64) {
        const int hq = i / BJ, j = i % BJ;
        float v = 0.f;
        for (int w = 0; w < NW; ++w) v += imp_wsum[(w * g + hq) * BJ + j];           // wavefront order: reproducible
        if (j < B) a.imp_partial[((size_t)b * Hq + hk * g + hq) * B + j] = v;
      }
    }
  }
  // the last workgroups to start (the shortest sequences), once through their own K/V, pull the next projection's
  // weights into the memory-side cache: any earlier and the K/V stream would push them out again
  const unsigned warm_acc = warm_touch(a.warm.ptr, a.warm.bytes, NW * 64);
  if (warm_acc == 0x9e3779b9u && a.chunk < 0) ((unsigned *)a.out)[0] = warm_acc;   // never true: keeps the loads
}

// Merge of the K/V splits of one (row, head): out = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), in split order.
__global__ __launch_bounds__(128) void k_attn_combine(AttnArgs a) {
  const int r = blockIdx.x, hq = blockIdx.y, d = threadIdx.x;
  const int M = a.rows.count ? min(*a.rows.count, a.rows.cap) : a.rows.cap;
  if (r >= M) return;
  const int b = a.ri.row_map[r] / a.ri.B;
  const int slot = slot_of(a.ri.seq_slot, b, a.st);
  const int total = a.st.prefix_len[slot] + a.ri.B;
  const int nsplit = min((total + a.chunk - 1) / a.chunk, a.max_splits);   // as in k_attn_mfma
  if (nsplit <= 1) return;
  const size_t pi = ((size_t)r * a.n_q_heads + hq) * a.max_splits;
  float mm = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mm = fmaxf(mm, a.part_ml[(pi + s) * 2]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = a.part_ml[(pi + s) * 2];
    const float w = ms == -INFINITY ? 0.f : exp2f(ms - mm);
    num += a.part_o[(pi + s) * 128 + d] * w;
    den += a.part_ml[(pi + s) * 2 + 1] * w;
  }
  ((bf16_t *)a.out)[((size_t)r * a.n_q_heads + hq) * 128 + d] = (bf16_t)(den > 0.f ? num / den : 0.f);
}

template <int NW, int BJ>
static bool launch_attn_imp(hipStream_t s, dim3 grid, const AttnArgs &a, int g) {
  const int bytes = 32768 + NW * 32 * (BJ + 1) * 4 + NW * g * BJ * 4;
  static int allowed = 0;                // LDS beyond 64 KB has to be allowed once per kernel
  if (bytes > allowed) {
    if (hipFuncSetAttribute((const void *)k_attn_mfma<NW, BJ>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    allowed = bytes;
  }
  k_attn_mfma<NW, BJ><<<grid, NW * 64, bytes, s>>>(a);
  return true;
}

bool attention(hipStream_t s, const AttnArgs &a) {
  if (a.rows.cap <= 0 || a.n_seq <= 0) return false;
  const int g = a.n_q_heads / a.kv.n_kv_heads;
  const bool mfma = a.dtype == FOCUS_BF16 && a.kv.head_dim == 128 && a.kv.page_size == 64 && a.q_stride % 8 == 0 && a.part_o != nullptr;
  if (mfma) {
    dim3 grid(a.n_seq * a.kv.n_kv_heads, a.launch_splits);
    const int R = a.max_rows_per_seq * g;
    bool fused = false;
    // importance rides along when the group size divides the 32 pairs of a wavefront (rows of one head are then the lanes with
    // equal lane % g) and the score patches fit the LDS
    if (a.imp_partial && (g == 1 || g == 2 || g == 4 || g == 8) && a.ri.B <= 64) {
      const bool small = a.ri.B <= 32;
      if (R <= 32) fused = small ? launch_attn_imp<1, 32>(s, grid, a, g) : launch_attn_imp<1, 64>(s, grid, a, g);
      else if (R <= 64) fused = small ? launch_attn_imp<2, 32>(s, grid, a, g) : launch_attn_imp<2, 64>(s, grid, a, g);
      else if (R <= 128) fused = small ? launch_attn_imp<4, 32>(s, grid, a, g) : launch_attn_imp<4, 64>(s, grid, a, g);
      else fused = small ? launch_attn_imp<8, 32>(s, grid, a, g) : launch_attn_imp<8, 64>(s, grid, a, g);
    }
    if (!fused) {
      if (R <= 32) k_attn_mfma<1><<<grid, 64, 0, s>>>(a);
      else if (R <= 64) k_attn_mfma<2><<<grid, 128, 0, s>>>(a);
      else if (R <= 128) k_attn_mfma<4><<<grid, 256, 0, s>>>(a);
      else k_attn_mfma<8><<<grid, 512, 0, s>>>(a);
    }
    if (a.launch_splits > 1) k_attn_combine<<<dim3(a.rows.cap, a.n_q_heads), 128, 0, s>>>(a);
    return fused;
  }
  dim3 grid(a.rows.cap, a.n_q_heads);
  const int ne = a.kv.head_dim / 64;
  if (a.dtype == FOCUS_F32) {
    if (ne == 1) k_attn_rowwave<float, 1><<<grid, 64, 0, s>>>((const float *)a.q, a.q_stride, a.n_q_heads, a.rows, a.ri, a.st, a.vis_by_b, a.kv, (float *)a.out);
    else k_attn_rowwave<float, 2><<<grid, 64, 0, s>>>((const float *)a.q, a.q_stride, a.n_q_heads, a.rows, a.ri, a.st, a.vis_by_b, a.kv, (float *)a.out);
  } else {
    if (ne == 1) k_attn_rowwave<bf16_t, 1><<<grid, 64, 0, s>>>((const bf16_t *)a.q, a.q_stride, a.n_q_heads, a.rows, a.ri, a.st, a.vis_by_b, a.kv, (bf16_t *)a.out);
    else k_attn_rowwave<bf16_t, 2><<<grid, 64, 0, s>>>((const bf16_t *)a.q, a.q_stride, a.n_q_heads, a.rows, a.ri, a.st, a.vis_by_b, a.kv, (bf16_t *)a.out);
  }
  return false;
}

// ---------------------------------------------------------------------------------------------
// Token importance, Eq. 2: for one (sequence, query head), S_ij = q_i . k_j / sqrt(D) over the block's own
// B x B scores, MaxPool1D (window 3, same length) along j, softmax along j, column sums over i.
// Output partial[b, h, j]; the head sum is taken later in a fixed order (no atomics, so it is reproducible).
// Queries: the sequence's rows of the fused qkv buffer (after the rotary embedding), i.e. all B positions, or, with the
// delayed intra-block cache (Sec. 4.3), the positions that are not frozen.  Keys: the B block positions of the layer's
// K cache, which holds the key every row just wrote and the frozen positions' keys.
struct ImpArgs {
  const void *qkv;
  const int32_t *cu;       // query rows of batch entry b: cu[b] .. cu[b + 1]
  int B, Hq, Hkv, D, pool_k;
  const int32_t *seq_slot;
  SlotState st;
  KvLayer kv;
  float *partial;
};

// K cache row of block position j of the sequence in slot `slot`, kv head hk
template <typename T>
__device__ __forceinline__ const T *block_key_row(const ImpArgs &a, int slot, int hk, int j) {
  const int P = a.kv.page_size, pos = a.st.prefix_len[slot] + j;
  const int page = a.st.page_table[(size_t)slot * a.st.table_stride + pos / P];
  return (const T *)a.kv.base + (size_t)page * 2 * a.Hkv * P * a.D + ((size_t)hk * P + pos % P) * a.D;
}

template <typename T, int MAXB, int MAXD>
__global__ __launch_bounds__(256) void k_importance(ImpArgs a) {
  __shared__ float ks[MAXB * (MAXD + 1)];
  __shared__ float S[MAXB][MAXB + 1];
  const int B = a.B, Hq = a.Hq, Hkv = a.Hkv, D = a.D, pool_k = a.pool_k;
  float *partial = a.partial;
  const int b = blockIdx.x, h = blockIdx.y, hk = h / (Hq / Hkv);
  const int slot = slot_of(a.seq_slot, b, a.st);
  const int stride = (Hq + 2 * Hkv) * D;
  const int r0 = a.cu[b], nq = min(a.cu[b + 1] - r0, B);
  const T *base = (const T *)a.qkv + (size_t)r0 * stride;
  for (int i = threadIdx.x; i < B * D; i += 256) {
    int j = i / D, d = i % D;
    ks[j * (D + 1) + d] = to_f(block_key_row<T>(a, slot, hk, j)[d]);
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)D);
  // thread -> query row i = tid / 4 and keys j = (tid % 4) + 4 * jj
  const int i = threadIdx.x >> 2, j0 = threadIdx.x & 3;
  if (i < nq) {
    float acc[MAXB / 4];
    for (int jj = 0; jj < MAXB / 4; ++jj) acc[jj] = 0.f;
    const T *qi = base + (size_t)i * stride + (size_t)h * D;
    constexpr int VE = 16 / sizeof(T);            // the query row is read in 16-byte pieces
    for (int d0 = 0; d0 < D; d0 += VE) {
      T qv[VE];
      *(u32x4 *)qv = *(const u32x4 *)(qi + d0);
#pragma unroll
      for (int e = 0; e < VE; ++e) {
        const float qd = to_f(qv[e]);
#pragma unroll
        for (int jj = 0; jj < MAXB / 4; ++jj) {
          int j = j0 + 4 * jj;
          if (j < B) acc[jj] += qd * ks[j * (D + 1) + d0 + e];
        }
      }
    }
#pragma unroll
    for (int jj = 0; jj < MAXB / 4; ++jj) {
      int j = j0 + 4 * jj;
      if (j < B) S[i][j] = acc[jj] * scale;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < nq) {
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
    for (int ii = 0; ii < nq; ++ii) col += S[ii][j];
    partial[((size_t)b * Hq + h) * B + j] = col;
  }
}

// bf16, D = 128: the same reduction on the matrix cores, one wavefront per (sequence, query head).
// S^T = K Q^T puts a query row in each lane (both lane halves hold the row of query l % 32 after one exchange),
// so pooling, max, exp and normalisation run in registers; the column sums are 5-step lane reductions, the lower
// lane half finishing the lower half of the keys and the upper half the rest.
template <int NJ>   // key tiles of 32: B <= 32 * NJ
__global__ __launch_bounds__(64) void k_importance_mfma(ImpArgs a) {
  constexpr int D = 128, BJ = 32 * NJ, HJ = BJ / 2;
  const int B = a.B, Hq = a.Hq, Hkv = a.Hkv, pool_k = a.pool_k;
  float *partial = a.partial;
  const int b = blockIdx.x, h = blockIdx.y, hk = h / (Hq / Hkv);
  const int slot = slot_of(a.seq_slot, b, a.st);
  const int lane = threadIdx.x, half = lane >> 5, col = lane & 31;
  const int stride = (Hq + 2 * Hkv) * D;
  const int r0 = a.cu[b], nq = min(a.cu[b + 1] - r0, B);
  const bf16_t *base = (const bf16_t *)a.qkv + (size_t)r0 * stride;
  const float sc = 1.4426950408889634f / sqrtf((float)D);
  bf16x8 kf[NJ][8];
#pragma unroll
  for (int jt = 0; jt < NJ; ++jt) {
    const bf16_t *kp = block_key_row<bf16_t>(a, slot, hk, min(32 * jt + col, B - 1)) + 8 * half;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[jt][ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(kp + 16 * ks));
  }
  float acc[HJ];
#pragma unroll
  for (int jj = 0; jj < HJ; ++jj) acc[jj] = 0.f;

  for (int it = 0; it * 32 < nq; ++it) {
    const int i = 32 * it + col;
    bf16x8 qf[8];
    const bf16_t *qp = base + (size_t)min(i, max(nq - 1, 0)) * stride + (size_t)h * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + 16 * ks));
    // full score row of query i in every lane: own registers for the keys of this lane half, the partner's for the rest
    float row[BJ];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) {
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[jt][ks], qf[ks], sacc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float mine = sacc[r] * sc, other = __shfl_xor(mine, 32);
        const int j0 = 32 * jt + 8 * (r >> 2) + (r & 3);          // key of register r in lane half 0; half 1 holds j0 + 4
        row[j0] = half ? other : mine;
        row[j0 + 4] = half ? mine : other;
      }
    }
#pragma unroll
    for (int j = 0; j < BJ; ++j) row[j] = j < B ? row[j] : -INFINITY;
    float pooled[BJ], m = -INFINITY;
#pragma unroll
    for (int j = 0; j < BJ; ++j) {
      float v = row[j];
      if (pool_k == 3) {
        if (j > 0) v = fmaxf(v, row[j - 1]);
        if (j + 1 < BJ) v = fmaxf(v, row[j + 1]);
      }
      v = j < B ? v : -INFINITY;                                  // no position beyond the block takes part in the softmax
      pooled[j] = v;
      m = fmaxf(m, v);
    }
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < BJ; ++j) {
      pooled[j] = exp2f(pooled[j] - m);
      sum += pooled[j];
    }
    const float inv = i < nq ? 1.0f / sum : 0.f;                  // lanes beyond the sequence's rows add nothing
#pragma unroll
    for (int jj = 0; jj < HJ; ++jj) {
      float v = (half ? pooled[jj + HJ] : pooled[jj]) * inv;
      for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o);     // over the 32 queries of this lane half
      acc[jj] += v;
    }
  }
#pragma unroll
  for (int jj = 0; jj < HJ; ++jj) {
    const int j = half * HJ + jj;
    if (col == (jj & 31) && j < B) partial[((size_t)b * Hq + h) * B + j] = acc[jj];
  }
}

void importance(hipStream_t s, int dtype, const void *qkv, const int32_t *cu, int n_seq, int B, int n_q_heads, int n_kv_heads,
                int head_dim, int maxpool_k, const int32_t *seq_slot, SlotState st, KvLayer kv, float *partial) {
  if (n_seq <= 0) return;
  dim3 grid(n_seq, n_q_heads);
  const ImpArgs a{qkv, cu, B, n_q_heads, n_kv_heads, head_dim, maxpool_k, seq_slot, st, kv, partial};
  if (dtype == FOCUS_BF16 && head_dim == 128 && (((uintptr_t)qkv | (uintptr_t)kv.base) & 15) == 0) {
    if (B <= 32) k_importance_mfma<1><<<grid, 64, 0, s>>>(a);
    else k_importance_mfma<2><<<grid, 64, 0, s>>>(a);
    return;
  }
  if (dtype == FOCUS_F32) k_importance<float, 64, 128><<<grid, 256, 0, s>>>(a);
  else k_importance<bf16_t, 64, 128><<<grid, 256, 0, s>>>(a);
}

}  // namespace fk
