// Dense projections  C[M, N] = A[M, K] * W[N, K]^T  (activations times [out, in] weights), fp32 accumulate.
//
// Two kernels:
//   k_gemm_valu  any element type, any shape: LDS-tiled 64x64x16, 4x4 outputs per lane on the vector ALU.
//                Used for fp32 models (the tiny oracle-check configuration) and for shapes the MFMA kernel
//                does not take.
//   k_gemm_mfma  bf16 on the matrix cores (see below).
// M is read from device memory when the row count is only known on the device (packed batch after eviction).
#include <algorithm>

#include "focus_internal.h"

namespace fk {

template <typename T> __device__ __forceinline__ float to_f(T v) { return (float)v; }

template <typename T, int EPI>
__device__ __forceinline__ void store_out(void *out, size_t idx, float acc) {
  if (EPI == EPI_STORE) ((T *)out)[idx] = (T)acc;
  else if (EPI == EPI_ADD_F32) ((float *)out)[idx] += acc;
  else ((float *)out)[idx] = acc;
}

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_valu(const T *__restrict__ A, const T *__restrict__ W, int N, int K, Rows rows,
                                                   void *out, int ldo) {
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= M) return;
  __shared__ float As[16][65], Ws[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 1024; i += 256) {
      int rr = i >> 4, kk = i & 15;
      int gm = m0 + rr, gn = n0 + rr, gk = k0 + kk;
      As[kk][rr] = (gm < M && gk < K) ? to_f(A[(size_t)gm * K + gk]) : 0.f;
      Ws[kk][rr] = (gn < N && gk < K) ? to_f(W[(size_t)gn * K + gk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i], w[i] = Ws[kk][tx * 4 + i];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn < N) store_out<T, EPI>(out, (size_t)gm * ldo + gn, acc[i][j]);
    }
  }
}

template <typename T>
static void launch_valu(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, int epi, void *out, int ldo) {
  dim3 grid((N + 63) / 64, (rows.cap + 63) / 64);
  if (epi == EPI_STORE)
    k_gemm_valu<T, EPI_STORE><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
  else if (epi == EPI_ADD_F32)
    k_gemm_valu<T, EPI_ADD_F32><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
  else
    k_gemm_valu<T, EPI_STORE_F32><<<grid, 256, 0, s>>>((const T *)A, (const T *)W, N, K, rows, out, ldo);
}

// ---------------------------------------------------------------------------------------------
// bf16 on the matrix cores.
//
// Workgroup = 4 wavefronts (2 x 2), macro tile BM x BN x 64; each wavefront owns a (BM/2) x (BN/2) patch as
// 32x32 accumulator tiles of v_mfma_f32_32x32x16_bf16.  Both operands are K-contiguous, so A rows and W rows
// feed the instruction the same way: lane l supplies row l % 32, eight consecutive k starting at 8 * (l / 32).
//
// LDS holds one K-slab of each operand, rows of 64 bf16 = 128 B = eight 16-byte chunks; chunk c of row r is
// stored at chunk position c ^ ((r >> 1) & 7), so the 32 rows read by one ds_read_b128 spread over all banks and
// the 8 lanes that fill a row write distinct chunks.  The next K-slab is fetched from global memory into
// registers while the current one is multiplied (two workgroups per CU overlap each other's barriers).
//
// Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id is remapped so that each XCD
// works on one contiguous range of tiles (ordered in groups of 8 tile rows), which keeps the A and W panels a
// range touches inside that XCD's own L2.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256, 2) void k_gemm_mfma(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, int N, int K,
                                                      Rows rows, void *out, int ldo, int tiles_m, int tiles_n) {
  constexpr int BK = 64, WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int CA = BM * 8 / 256, CB = BN * 8 / 256;      // 16-byte chunks per thread and K-slab
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * 128];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * 128];

  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  // XCD-aware tile order over the tile rows that hold valid rows (the grid is sized for rows.cap; with a row count that
  // only the device knows, the live tiles still spread over all 8 XCDs and the workgroups beyond them exit)
  tiles_m = min(tiles_m, (M + BM - 1) / BM);
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (blockIdx.x / 8 >= per_xcd || tile >= total) return;
  constexpr int GROUP = 8;
  const int in_group = tile % (GROUP * tiles_n), first_m = (tile / (GROUP * tiles_n)) * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int m0 = (first_m + in_group % gsz) * BM, n0 = (in_group / gsz) * (EPI == EPI_SILU_MUL ? BN / 2 : BN);
  if (m0 >= M) return;
  static_assert(EPI != EPI_SILU_MUL || BN == 128, "the fused SiLU*up epilogue pairs the two column tiles of a wavefront");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;

  // global -> register -> LDS staging: chunk id = tid + 256 * i -> (row, chunk)
  const bf16_t *ga[CA], *gb[CB];
  int sa[CA], sb[CB];
#pragma unroll
  for (int i = 0; i < CA; ++i) {
    int c = tid + 256 * i, r = c >> 3, ch = c & 7;
    ga[i] = A + (size_t)min(m0 + r, M - 1) * K + ch * 8;
    sa[i] = r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int i = 0; i < CB; ++i) {
    int c = tid + 256 * i, r = c >> 3, ch = c & 7;
    // fused SiLU*up: the two 32-column accumulator tiles of a wavefront are the gate and the up projection of
    // the same 32 activation columns, so LDS row r holds gate row n0 + ... for even 32-row groups and the
    // matching up row (F rows further) for odd ones
    const int wrow = EPI == EPI_SILU_MUL ? ((r >> 5) & 1) * (N / 2) + n0 + (r / WN) * 32 + (r & 31) : n0 + r;
    gb[i] = W + (size_t)min(wrow, N - 1) * K + ch * 8;
    sb[i] = r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
  }
  u32x4 ra[CA], rb[CB];
#pragma unroll
  for (int i = 0; i < CA; ++i) ra[i] = *(const u32x4 *)(ga[i]);
#pragma unroll
  for (int i = 0; i < CB; ++i) rb[i] = *(const u32x4 *)(gb[i]);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment addresses: row = base + (lane & 31), logical chunk = 2 * ks + (lane >> 5)
  const int frow = lane & 31, fch = lane >> 5;
  const int nk = K / BK;
  for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
    for (int i = 0; i < CA; ++i) *(u32x4 *)(As + sa[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *(u32x4 *)(Bs + sb[i]) = rb[i];
    __syncthreads();
    {
      // the last iteration re-reads its own slab: an unconditional load keeps the staging registers in VGPRs
      const size_t koff = (size_t)min(kt + 1, nk - 1) * BK;
#pragma unroll
      for (int i = 0; i < CA; ++i) ra[i] = *(const u32x4 *)(ga[i] + koff);
#pragma unroll
      for (int i = 0; i < CB; ++i) rb[i] = *(const u32x4 *)(gb[i] + koff);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int r = wm + i * 32 + frow;
        af[i] = *(const bf16x8 *)(As + r * 128 + (((2 * ks + fch) ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int r = wn + j * 32 + frow;
        bfr[j] = *(const bf16x8 *)(Bs + r * 128 + (((2 * ks + fch) ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue: accumulator register r of lane l is C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of its 32x32 tile
  if (EPI == EPI_SILU_MUL) {
    const int gn = n0 + (wn / WN) * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const float g = acc[i][0][r], u = acc[i][TN - 1][r];
        if (gm < M && gn < N / 2) ((bf16_t *)out)[(size_t)gm * ldo + gn] = (bf16_t)(g / (1.0f + __expf(-g)) * u);
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int gn = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (gm < M && gn < N) store_out<bf16_t, EPI>(out, (size_t)gm * ldo + gn, acc[i][j][r]);
      }
    }
}

template <int BM, int BN>
static void launch_mfma(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, int epi, void *out, int ldo) {
  const int tiles_m = (rows.cap + BM - 1) / BM;
  const int tiles_n = epi == EPI_SILU_MUL ? (N / 2 + BN / 2 - 1) / (BN / 2) : (N + BN - 1) / BN;
  const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
  const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
  if (epi == EPI_SILU_MUL) k_gemm_mfma<BM, BN, EPI_SILU_MUL><<<grid, 256, 0, s>>>(a, w, N, K, rows, out, ldo, tiles_m, tiles_n);
  else if (epi == EPI_STORE) k_gemm_mfma<BM, BN, EPI_STORE><<<grid, 256, 0, s>>>(a, w, N, K, rows, out, ldo, tiles_m, tiles_n);
  else if (epi == EPI_ADD_F32) k_gemm_mfma<BM, BN, EPI_ADD_F32><<<grid, 256, 0, s>>>(a, w, N, K, rows, out, ldo, tiles_m, tiles_n);
  else k_gemm_mfma<BM, BN, EPI_STORE_F32><<<grid, 256, 0, s>>>(a, w, N, K, rows, out, ldo, tiles_m, tiles_n);
}

// ---------------------------------------------------------------------------------------------
// Large problems: BM x 256 x 64 tiles (BM = 256 or 128), 8 wavefronts (2 x 4), K-slabs loaded straight into LDS
// (buffer_load_dwordx4 ... lds: lane l of an instruction fills the 16-byte slot l of a 1 KB block = 8 tile rows, so
// the bank swizzle is applied by choosing which chunk a lane fetches; rows beyond the matrix fall outside the buffer
// descriptor and read as zero), two LDS stages, software-pipelined by hand:
//   * the fragments of k-step s + 1 are read from LDS while the MFMAs of step s run (two register sets);
//   * one barrier per slab, placed before the last k-step: by then every wavefront has read all of the current slab
//     and the next one has landed, so the loads of the slab after the next start right behind the barrier;
//   * loads are spread between the MFMAs (a burst of 8 direct-to-LDS loads per wavefront stalls the matrix pipe for
//     longer than the loads take on their own: measured 37 % of the MFMA rate against 100 % when interleaved);
//   * the loop handles two slabs per trip, so the stage is a compile-time constant, LDS addresses are loop-invariant
//     registers plus immediates, and the loads take their slab offset from a scalar register: no vector ALU work
//     competes with the MFMAs for issue slots.
// The waits for the loads are explicit: the compiler does not order LDS reads behind direct-to-LDS loads.
// LDS layout: A stage 0, A stage 1, W stage 0, W stage 1 (so that both stages of an operand are within the 16-bit
// immediate offset of one base register).
#define FK_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// Workgroup barrier that orders LDS traffic only: outstanding global loads (which the kernel waits for by count) are
// not drained, unlike with __syncthreads().
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Lane exchanges inside a row of 16 lanes without LDS: CTRL is a data-parallel-primitive pattern (0xB1 / 0x4E: lanes l ^ 1 / l ^ 2
// of a quad, 0x141: lane 7 - l of eight, 0x140: lane 15 - l of sixteen).  All four are permutations, so every lane has a source.
template <int CTRL> __device__ __forceinline__ float lane_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ void lane_max_step(float &m, int &mi) {
  const float om = lane_dpp<CTRL>(m);
  const int oi = __builtin_amdgcn_update_dpp(0, mi, CTRL, 0xF, 0xF, false);
  if (om > m || (om == m && oi < mi)) { m = om; mi = oi; }     // equal maxima: the lower column
}

template <int BM, int NW, int EPI, int BN = 256>
__global__ __launch_bounds__(NW * 64, NW == 8 ? 2 : 1) void k_gemm_pipe(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, int N, int K,
                                                      Rows rows, void *out, int ldo, int tiles_m, int tiles_n, const void *warm,
                                                      unsigned warm_bytes, int splits, size_t split_stride) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer-resource builtins exist in the device pass only
  // splits > 1: the K range is cut into `splits` parts, one workgroup each; part s writes its fp32 sums to
  // out + s * split_stride and a second kernel adds the parts in order (EPI is then EPI_STORE_F32 or EPI_PARTIAL_SILU)
  constexpr bool SILU_W = EPI == EPI_SILU_MUL || EPI == EPI_PARTIAL_SILU;
  // NW = 8: wavefronts 2 x 4, each BM/2 x 64;  NW = 4: wavefronts 2 x 2, each BM/2 x 128 (a third fewer LDS reads per MFMA,
  // accumulators in the 256 accumulation registers a lone wavefront per SIMD can have)
  // BN = 192 (4 wavefronts of 128 x 96) exists for launches whose 256-wide tiles would leave a quarter of the CUs idle
  constexpr int BK = 64, WCOLS = NW / 2, WM = BM / 2, WN = BN / WCOLS, TM = WM / 32, TN = WN / 32;
  static_assert(WN % 32 == 0 && (BN / 8) % NW == 0 && (!SILU_W || TN % 2 == 0), "tile shape");
  constexpr int IA = BM / 8 / NW, IB = BN / 8 / NW, NI = IA + IB;
  constexpr int ASTAGE = BM * 128, WSTAGE = BN * 128, WBASE = 2 * ASTAGE, NMF = TM * TN;
  // loads issued in the k-step right behind the barrier; the rest follow in the first k-step of the next slab
  constexpr int L0 = NI / 2, L1 = NI - L0;
  static_assert(L0 <= NMF && L1 <= NMF && TM + TN <= NMF, "one load and one fragment read per MFMA at most");
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_pipe[];
  unsigned char *const lds = lds_pipe;
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  // the tile list covers the tile rows that hold valid rows: the grid is sized for rows.cap, and with a row count that only the
  // device knows the live tiles still spread evenly over the 8 XCDs (workgroups beyond them exit at once)
  tiles_m = min(tiles_m, (M + BM - 1) / BM);
  const int total = tiles_m * tiles_n * splits;
  const int per_xcd = (total + 7) / 8;
  const int work = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (blockIdx.x / 8 >= per_xcd || work >= total) return;
  const int live_grid = per_xcd * 8;
  const int tile = work / splits, split = work % splits;
  constexpr int GROUP = 8;
  const int in_group = tile % (GROUP * tiles_n), first_m = (tile / (GROUP * tiles_n)) * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int m0 = (first_m + in_group % gsz) * BM, n0 = (in_group / gsz) * (SILU_W ? BN / 2 : BN);
  if (m0 >= M) return;
  out = (void *)((float *)out + (size_t)split * split_stride);   // (split is 0 unless the output is fp32 partial sums)
  const int nk = K / BK / splits;                                 // slabs of this workgroup; even (checked by the host)
  const unsigned k_base = (unsigned)split * (unsigned)nk * (BK * 2);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / WCOLS) * WM, wn = (wave % WCOLS) * WN;
  // raw buffers over the valid rows: an offset at or beyond the size reads zero without touching memory
  __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (unsigned)M * (unsigned)K * 2u, 0x00020000);
  __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (unsigned)N * (unsigned)K * 2u, 0x00020000);
  // per-lane byte offsets of this wavefront's load instructions: instruction q covers tile rows (wave * I + q) * 8 .. + 7
  unsigned voa[IA], vob[IB];
#pragma unroll
  for (int q = 0; q < IA; ++q) {
    const int r = (wave * IA + q) * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    voa[q] = (unsigned)(m0 + r) * (unsigned)K * 2u + k_base + c * 16;
  }
#pragma unroll
  for (int q = 0; q < IB; ++q) {
    const int r = (wave * IB + q) * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    // fused SiLU*up: LDS rows 64 c .. 64 c + 31 hold the gate rows of output columns 32 c .. 32 c + 31, the next 32 rows the
    // matching up rows, so that a wavefront's column tiles 2 p and 2 p + 1 are gate and up of the same columns
    const int wrow = SILU_W ? ((r >> 5) & 1) * (N / 2) + n0 + (r / 64) * 32 + (r & 31) : n0 + r;
    vob[q] = (unsigned)wrow * (unsigned)K * 2u + k_base + c * 16;
  }
  // Optional: touch `warm_bytes` bytes at `warm` (the weights of the next projection) so that they wait in the memory-side
  // cache; weights are read once per step and a projection that finds them in HBM runs up to 1.5 times longer.  A
  // workgroup's share is spread over its slabs: on a "hit" slab each wavefront reads one dword of 64
  // consecutive 128-byte lines.  The loads go through a descriptor of exactly warm_bytes, so shares beyond the end (and
  // all of them when there is nothing to warm) are out of range and move no data.  A result is folded into a dummy value
  // one slab later, when the load has long returned, so nothing waits for it.
  __amdgpu_buffer_rsrc_t rs_p = __builtin_amdgcn_make_buffer_rsrc((void *)warm, 0, warm_bytes, 0x00020000);
  // only the workgroups of the last round (one workgroup per CU) take part: what earlier rounds fetch is pushed out of the
  // cache again by the kernel's own traffic before the next kernel starts
  const int warm_groups = min(live_grid, 256), warm_rank = (int)blockIdx.x - (live_grid - warm_groups);
  constexpr unsigned HIT = NW * 8192;   // bytes per hit: NW wavefronts x 64 lines
  const unsigned warm_hits = warm_rank < 0 ? 0u : ((warm_bytes + warm_groups - 1) / warm_groups + HIT - 1) / HIT;
  const int warm_stride = warm_hits ? max(1, nk / (int)warm_hits) : 1;
  unsigned warm_off = (unsigned)max(warm_rank, 0) * (warm_hits * HIT), warm_left = warm_hits;
  int warm_next = 0;
  unsigned warm_sink = 0, warm_prev = 0;
  const unsigned warm_lane = lane * 128 + wave * 8192;
  auto gl = [&](int i, int soff, int buf) {   // load instruction i (A: 0 .. IA-1, W: IA .. NI-1) of the slab at byte offset soff
    if (i < IA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, FK_LDS_PTR(lds + buf * ASTAGE + (wave * IA + (i < IA ? i : 0)) * 1024), 16, voa[i < IA ? i : 0], soff, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, FK_LDS_PTR(lds + WBASE + buf * WSTAGE + (wave * IB + (i < IA ? 0 : i - IA)) * 1024), 16,
                                               vob[i < IA ? 0 : i - IA], soff, 0, 0);
  };
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // fragment addresses: row = base + (lane & 31), logical chunk 2 * ks + (lane >> 5), swizzled with the row (all 32-row
  // tiles start at a multiple of 32, so the swizzle depends on the lane only)
  const int frow = lane & 31, fch = lane >> 5, sw = (frow >> 1) & 7;
  const unsigned char *pa[4], *pb[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    pa[ks] = lds + (wm + frow) * 128 + (((2 * ks + fch) ^ sw) << 4);
    pb[ks] = lds + WBASE + (wn + frow) * 128 + (((2 * ks + fch) ^ sw) << 4);
  }
  bf16x8 fa[2][TM], fb[2][TN];
  auto rd = [&](int s, int ks, int buf, int slot) {   // s-th fragment read of a k-step, in the order the MFMAs need them
    const int f = s == 0 ? TM : (s == 1 ? 0 : (s <= TN ? TM + s - 1 : s - TN));   // W0, A0, W1 .. W(TN-1), A1 .. A(TM-1)
    if (f < TM) fa[slot][f < TM ? f : 0] = *(const bf16x8 *)(pa[ks] + buf * ASTAGE + (f < TM ? f : 0) * 4096);
    else fb[slot][f < TM ? 0 : f - TM] = *(const bf16x8 *)(pb[ks] + buf * WSTAGE + (f < TM ? 0 : f - TM) * 4096);
  };
  const int last = (nk - 1) * (BK * 2);
#pragma unroll
  for (int i = 0; i < NI; ++i) gl(i, 0, 0);
#pragma unroll
  for (int i = 0; i < L0; ++i) gl(i, min(BK * 2, last), 1);
  __builtin_amdgcn_s_waitcnt(0x0F70 | L0);   // vmcnt(L0): slab 0 has landed
  lds_barrier(); 
#pragma unroll
  for (int s = 0; s < TM + TN; ++s) rd(s, 0, 0, 0);

  // one k-step: the MFMAs on register set `cur`; behind MFMA s, fragment read s of the next k-step, and (when nl > 0)
  // a load on every NMF / nl-th MFMA
#define FK_STEP(cur, next_ks, next_buf, nl, lfirst, lsoff, lbuf)                                        \
  {                                                                                                     \
    _Pragma("unroll") for (int s = 0; s < NMF; ++s) {                                                   \
      const int i = s / TN, j = s % TN;                                                                 \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);  \
      if (s < TM + TN) rd(s, next_ks, next_buf, (cur) ^ 1);                                             \
      if ((nl) > 0 && s % (NMF / ((nl) > 0 ? (nl) : 1)) == NMF / ((nl) > 0 ? (nl) : 1) - 1 && s / (NMF / ((nl) > 0 ? (nl) : 1)) < (nl)) \
        gl((lfirst) + s / (NMF / ((nl) > 0 ? (nl) : 1)), lsoff, lbuf);                                  \
      __builtin_amdgcn_sched_barrier(0);                                                                \
    }                                                                                                   \
  }
  // one slab held in stage `buf`; beyond the last slab the loads repeat it (into a stage nobody reads any more), so the
  // loop body has no branches
#define FK_SLAB(buf, kt)                                                                                \
  {                                                                                                     \
    const int so1 = min(((kt) + 1) * (BK * 2), last), so2 = min(((kt) + 2) * (BK * 2), last);           \
    FK_STEP(0, 1, buf, L1, L0, so1, (buf) ^ 1)                                                          \
    {                                                                                                   \
      const bool hit = (kt) == warm_next && warm_left > 0;                                              \
      const unsigned so = hit ? warm_off : 0x80000000u;                                                 \
      warm_sink ^= warm_prev;                                                                           \
      warm_prev = __builtin_amdgcn_raw_buffer_load_b32(rs_p, warm_lane, so, 0);                         \
      warm_off += hit ? HIT : 0u; warm_left -= hit ? 1u : 0u; warm_next += hit ? warm_stride : 0;       \
    }                                                                                                   \
    FK_STEP(1, 2, buf, 0, 0, so1, (buf) ^ 1)                                                            \
    FK_STEP(0, 3, buf, 0, 0, so1, (buf) ^ 1)                                                            \
    __builtin_amdgcn_s_waitcnt(0x0F71); /* vmcnt(1): all but the warm-up load: this wavefront's part of the next slab has landed */ \
    lds_barrier();                     /* ... and everyone's; everyone has read all of this slab */    \
    FK_STEP(1, 0, (buf) ^ 1, L0, 0, so2, buf)                                                           \
  }
  for (int kt = 0; kt < nk; kt += 2) {
    FK_SLAB(0, kt)
    FK_SLAB(1, kt + 1)
  }
#undef FK_SLAB
#undef FK_STEP
  __builtin_amdgcn_s_waitcnt(0x0F70);
  if ((warm_sink ^ warm_prev) == 0x9e3779b9u && warm_bytes == 1) ((unsigned *)out)[0] = warm_sink;   // keeps the warm-up loads alive; never true
  // epilogue: accumulator register r of lane l is C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of its 32x32 tile.
  // A tile that lies inside the matrix takes the path without per-element bounds checks; there the accumulating
  // epilogue reads a whole row of 32x32 tiles before it adds and stores (one memory round trip per tile row instead
  // of one per element).
  const bool inside = m0 + BM <= M && n0 + (SILU_W ? BN / 2 : BN) <= (SILU_W ? N / 2 : N);
  const int erow = m0 + wm + 4 * (lane >> 5), ecol = lane & 31;
  if (EPI == EPI_SILU_MUL) {
#pragma unroll
    for (int jp = 0; jp < TN / 2; ++jp) {
      const int gn = n0 + (wn / 64 + jp) * 32 + ecol;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
          const float g = acc[i][2 * jp][r], u = acc[i][2 * jp + 1][r];
          if (inside || (gm < M && gn < N / 2)) ((bf16_t *)out)[(size_t)gm * ldo + gn] = (bf16_t)(g / (1.0f + __expf(-g)) * u);
        }
    }
    return;
  }
  if (EPI == EPI_PARTIAL_SILU) {   // fp32 partial sums in weight-row order: gate of column c at c, up at N / 2 + c
#pragma unroll
    for (int jp = 0; jp < TN / 2; ++jp) {
      const int gn = n0 + (wn / 64 + jp) * 32 + ecol;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
          if (inside || (gm < M && gn < N / 2)) {
            ((float *)out)[(size_t)gm * ldo + gn] = acc[i][2 * jp][r];
            ((float *)out)[(size_t)gm * ldo + N / 2 + gn] = acc[i][2 * jp + 1][r];
          }
        }
    }
    return;
  }
  if (EPI == EPI_CONF) {
    // per row: (maximum, sum exp(x - maximum), lowest column of the maximum) over this wavefront's WN columns.  The accumulators
    // hold a row spread over 32 lanes; each 32 x WN patch goes through a private LDS area (the operand stages are free: every
    // load has landed) and comes back with two lanes per row, each holding half of the row's columns in order, so that the
    // reductions run inside a lane and one exchange with the neighbour lane finishes them.
    constexpr int XS = WN + 4;                               // padded row: two lanes per row read 16-byte pieces
    static_assert(NW * 32 * XS * 4 <= 2 * (BM + BN) * 128, "transpose area");
    lds_barrier();                                           // everybody's loads have landed, nobody reads operands any more
    float *xp = (float *)lds + wave * (32 * XS);
    const int slot = (n0 / BN) * WCOLS + wn / WN;
    const int xrow = lane >> 1, xpart = lane & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const bool ok = n0 + wn + j * 32 + ecol < N;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          xp[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * XS + j * 32 + ecol] = ok ? acc[i][j][r] : -INFINITY;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
      const float4 *src = (const float4 *)(xp + xrow * XS + xpart * (WN / 2));
      float4 v[WN / 8];
#pragma unroll
      for (int k = 0; k < WN / 8; ++k) v[k] = src[k];
      float m = -INFINITY;
      int mi = 0x7fffffff;
      const int c0 = n0 + wn + xpart * (WN / 2);
#pragma unroll
      for (int k = 0; k < WN / 8; ++k) {                     // ascending columns: the first maximum stays
        if (v[k].x > m) { m = v[k].x; mi = c0 + 4 * k; }
        if (v[k].y > m) { m = v[k].y; mi = c0 + 4 * k + 1; }
        if (v[k].z > m) { m = v[k].z; mi = c0 + 4 * k + 2; }
        if (v[k].w > m) { m = v[k].w; mi = c0 + 4 * k + 3; }
      }
      lane_max_step<0xB1>(m, mi);                            // the row's other half (lane l ^ 1)
      float sum = 0.f;
      if (m > -INFINITY) {
#pragma unroll
        for (int k = 0; k < WN / 8; ++k) sum += __expf(v[k].x - m) + __expf(v[k].y - m) + __expf(v[k].z - m) + __expf(v[k].w - m);
      }
      sum += lane_dpp<0xB1>(sum);
      const int gm = m0 + wm + i * 32 + xrow;
      if (xpart == 0 && gm < M) {
        float *p = (float *)out + ((size_t)gm * ldo + slot) * 3;
        p[0] = m; p[1] = sum; p[2] = __int_as_float(mi);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
      __builtin_amdgcn_wave_barrier();                       // the patch is rewritten by the next row tile
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
    }
    return;
  }
  if (EPI == EPI_ADD_F32 && inside) {
    float *o = (float *)out + (size_t)erow * ldo + n0 + wn + ecol;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float old[TN][16];
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) old[j][r] = o[(size_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * ldo + j * 32];
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[(size_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * ldo + j * 32] = old[j][r] + acc[i][j][r];
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int gn = n0 + wn + j * 32 + ecol;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gm = erow + i * 32 + 8 * (r >> 2) + (r & 3);
        if (inside || (gm < M && gn < N)) store_out<bf16_t, EPI == EPI_PARTIAL_SILU ? EPI_STORE_F32 : EPI>(out, (size_t)gm * ldo + gn, acc[i][j][r]);
      }
    }
#endif
}

// Adds the fp32 partial sums of a K-split projection in split order and applies the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void k_splitk_reduce(const float *__restrict__ part, int splits, size_t split_stride, Rows rows, int N,
                                                       void *out, int ldo) {
  const int M = rows.count ? min(*rows.count, rows.cap) : rows.cap;
  const int ncol = EPI == EPI_SILU_MUL ? N / 2 : N, per_row = ncol / 4;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int m = (int)(idx / per_row), c = (int)(idx % per_row) * 4;
  if (m >= M) return;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
  for (int s = 0; s < splits; ++s) {
    const float *p = part + s * split_stride + (size_t)m * N + c;
    const float4 v = *(const float4 *)p;
    a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    if (EPI == EPI_SILU_MUL) {
      const float4 u = *(const float4 *)(p + N / 2);
      b.x += u.x; b.y += u.y; b.z += u.z; b.w += u.w;
    }
  }
  const float r[4] = {a.x, a.y, a.z, a.w}, u[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const size_t o = (size_t)m * ldo + c + i;
    if (EPI == EPI_SILU_MUL) ((bf16_t *)out)[o] = (bf16_t)(r[i] / (1.0f + __expf(-r[i])) * u[i]);
    else store_out<bf16_t, EPI>(out, o, r[i]);
  }
}

template <int BM, int NW, int EPI, int BN = 256>
static bool launch_pipe_epi(hipStream_t s, const bf16_t *a, const bf16_t *w, int N, int K, Rows rows, void *out, int ldo, int tiles_m, int tiles_n, Warm warm,
                            int splits = 1, size_t split_stride = 0) {
  constexpr int kLds = 2 * (BM + BN) * 128;
  static bool ready = false;             // the dynamic LDS size has to be allowed once per kernel
  if (!ready) {
    if (hipFuncSetAttribute((const void *)k_gemm_pipe<BM, NW, EPI, BN>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess) return false;
    ready = true;
  }
  const int grid = ((tiles_m * tiles_n * splits + 7) / 8) * 8;
  k_gemm_pipe<BM, NW, EPI, BN><<<grid, NW * 64, kLds, s>>>(a, w, N, K, rows, out, ldo, tiles_m, tiles_n, warm.ptr, (unsigned)std::min<size_t>(warm.bytes, 0x7fffffffu),
                                                      splits, split_stride);
  return true;
}

// K-split launch for problems with too few tiles to occupy the chip (few rows: the projection is bound by streaming W,
// and a CU cannot pull more than a fraction of a percent of the HBM bandwidth on its own): `splits` workgroups per tile
// write fp32 partial sums to the scratch buffer, k_splitk_reduce adds them in a fixed order.
static void launch_reduce(hipStream_t s, int N, Rows rows, int epi, void *out, int ldo, int splits, const float *scratch) {
  const size_t stride = (size_t)rows.cap * N;
  const size_t quads = (size_t)rows.cap * ((epi == EPI_SILU_MUL ? N / 2 : N) / 4);
  const unsigned grid = (unsigned)((quads + 255) / 256);
  if (epi == EPI_SILU_MUL) k_splitk_reduce<EPI_SILU_MUL><<<grid, 256, 0, s>>>(scratch, splits, stride, rows, N, out, ldo);
  else if (epi == EPI_STORE) k_splitk_reduce<EPI_STORE><<<grid, 256, 0, s>>>(scratch, splits, stride, rows, N, out, ldo);
  else if (epi == EPI_ADD_F32) k_splitk_reduce<EPI_ADD_F32><<<grid, 256, 0, s>>>(scratch, splits, stride, rows, N, out, ldo);
  else k_splitk_reduce<EPI_STORE_F32><<<grid, 256, 0, s>>>(scratch, splits, stride, rows, N, out, ldo);
}

static bool launch_split(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, int epi, void *out, int ldo, Warm warm,
                         int splits, float *scratch) {
  const int tiles_m = (rows.cap + 127) / 128;
  const int tiles_n = epi == EPI_SILU_MUL ? (N / 2 + 127) / 128 : (N + 255) / 256;
  const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
  const size_t stride = (size_t)rows.cap * N;
  const bool ok = epi == EPI_SILU_MUL ? launch_pipe_epi<128, 8, EPI_PARTIAL_SILU>(s, a, w, N, K, rows, scratch, N, tiles_m, tiles_n, warm, splits, stride)
                                      : launch_pipe_epi<128, 8, EPI_STORE_F32>(s, a, w, N, K, rows, scratch, N, tiles_m, tiles_n, warm, splits, stride);
  if (!ok) return false;
  launch_reduce(s, N, rows, epi, out, ldo, splits, scratch);
  return true;
}

template <int BM, int NW>
static bool launch_pipe(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, int epi, void *out, int ldo, Warm warm) {
  const int tiles_m = (rows.cap + BM - 1) / BM;
  const int tiles_n = epi == EPI_SILU_MUL ? (N / 2 + 127) / 128 : (N + 255) / 256;
  const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
  if (epi == EPI_SILU_MUL) return launch_pipe_epi<BM, NW, EPI_SILU_MUL>(s, a, w, N, K, rows, out, ldo, tiles_m, tiles_n, warm);
  if (epi == EPI_STORE) return launch_pipe_epi<BM, NW, EPI_STORE>(s, a, w, N, K, rows, out, ldo, tiles_m, tiles_n, warm);
  if (epi == EPI_ADD_F32) return launch_pipe_epi<BM, NW, EPI_ADD_F32>(s, a, w, N, K, rows, out, ldo, tiles_m, tiles_n, warm);
  return launch_pipe_epi<BM, NW, EPI_STORE_F32>(s, a, w, N, K, rows, out, ldo, tiles_m, tiles_n, warm);
}

bool gemm_conf_partials(hipStream_t s, int dtype, const void *A, const void *W, int N, int K, Rows rows, float *part, size_t part_bytes,
                        int *n_slots) {
  if (rows.cap <= 0 || dtype != FOCUS_BF16 || K % 64 || (((uintptr_t)A | (uintptr_t)W) & 15)) return false;
  if (!((double)std::max(rows.cap + 256, N + 256) * K * 2 < 4.0e9 && (K / 64) % 2 == 0)) return false;
  const int est = rows.expected(), tn = (N + 255) / 256;
  const long t256 = (long)((est + 255) / 256) * tn, t128 = (long)((est + 127) / 128) * tn;
  const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
  // same tile choice as gemm(): the largest tile that gives every compute unit work; four wavefronts where a unit takes several tiles
  if (t256 >= 160) {
    const bool four = t256 > 256;
    const int slots = tn * (four ? 2 : 4), tm = (rows.cap + 255) / 256;
    if ((size_t)rows.cap * slots * 12 > part_bytes) return false;
    *n_slots = slots;
    return four ? launch_pipe_epi<256, 4, EPI_CONF>(s, a, w, N, K, rows, part, slots, tm, tn, Warm())
                : launch_pipe_epi<256, 8, EPI_CONF>(s, a, w, N, K, rows, part, slots, tm, tn, Warm());
  }
  if (t128 >= 160) {
    const int slots = tn * 4, tm = (rows.cap + 127) / 128;
    if ((size_t)rows.cap * slots * 12 > part_bytes) return false;
    *n_slots = slots;
    return launch_pipe_epi<128, 8, EPI_CONF>(s, a, w, N, K, rows, part, slots, tm, tn, Warm());
  }
  return false;
}

bool gemm_fuses_silu_mul(int dtype, const void *A, const void *W, int N, int K) {
  return dtype == FOCUS_BF16 && K % 64 == 0 && N % 2 == 0 && ((uintptr_t)A & 15) == 0 && ((uintptr_t)W & 15) == 0;
}

void gemm(hipStream_t s, int dtype, const void *A, const void *W, int N, int K, Rows rows, int epilogue,
          void *out, int ldo, Warm warm, Scratch scratch) {
  if (rows.cap <= 0) return;
  if (dtype == FOCUS_F32) { launch_valu<float>(s, A, W, N, K, rows, epilogue, out, ldo); return; }
  const bool aligned = K % 64 == 0 && ((uintptr_t)A & 15) == 0 && ((uintptr_t)W & 15) == 0;
  if (!aligned) { launch_valu<bf16_t>(s, A, W, N, K, rows, epilogue, out, ldo); return; }
  // tile choice: the pipelined kernels run one workgroup per CU; take the largest tile that still gives every CU work
  // (byte offsets of rows must fit 32 bits there, and the slab count must be even), else the register-staged kernel with smaller tiles
  const long n_tiles = epilogue == EPI_SILU_MUL ? (N / 2 + 127) / 128 : (N + 255) / 256;
  const bool fits32 = (double)std::max(rows.cap + 256, N + 256) * K * 2 < 4.0e9 && (K / 64) % 2 == 0;
  // (tile shapes are chosen for the expected row count; the grids below cover rows.cap)
  const int est = rows.expected();
  const long t256 = (long)((est + 255) / 256) * n_tiles, t128 = (long)((est + 127) / 128) * n_tiles;
  const int choice = t256 >= 160 ? 256 : (t128 >= 160 ? 128 : 0);
  // four wavefronts of 128 x 128 read a third less from LDS per MFMA: measured 2-5 % faster where the launch takes more
  // than one round of workgroups (gate/up, vocabulary projection, full-block layers), no gain on single-round launches
  const bool four = t256 > 256;
  // one round of 256-wide tiles that leaves CUs idle (the QKV projection of 2048 rows: 192 tiles): 192-wide tiles fill them
  const long t192 = N % 192 == 0 ? (long)((est + 255) / 256) * (N / 192) : 0;
  if (fits32 && choice == 256 && !four && t256 < 240 && t192 > t256 && t192 <= 256 && epilogue != EPI_SILU_MUL) {
    const int tm = (rows.cap + 255) / 256, tn = N / 192;
    const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
    const bool ok = epilogue == EPI_STORE ? launch_pipe_epi<256, 4, EPI_STORE, 192>(s, a, w, N, K, rows, out, ldo, tm, tn, warm)
                  : epilogue == EPI_ADD_F32 ? launch_pipe_epi<256, 4, EPI_ADD_F32, 192>(s, a, w, N, K, rows, out, ldo, tm, tn, warm)
                                            : launch_pipe_epi<256, 4, EPI_STORE_F32, 192>(s, a, w, N, K, rows, out, ldo, tm, tn, warm);
    if (ok) return;
  }
  if (fits32 && choice == 256 && (four ? launch_pipe<256, 4>(s, A, W, N, K, rows, epilogue, out, ldo, warm) : launch_pipe<256, 8>(s, A, W, N, K, rows, epilogue, out, ldo, warm))) return;
  if (fits32 && choice == 128 && launch_pipe<128, 8>(s, A, W, N, K, rows, epilogue, out, ldo, warm)) return;
  if (fits32 && choice == 0 && scratch.ptr && N % 8 == 0 && rows.cap <= 128) {
    // one tile of rows: pure weight streaming.  The expert-projection kernel (two workgroups per CU, two weight slabs in
    // flight each) with K cut so that about two workgroups per CU exist
    const int nk = K / 64, tn = epilogue == EPI_SILU_MUL ? (N / 2 + 63) / 64 : (N + 127) / 128;
    int splits = 1;
    while (splits < 16 && (long)tn * (splits * 2) <= 512 && nk % (splits * 2) == 0 && nk / (splits * 2) >= 4 &&
           (size_t)(splits * 2) * rows.cap * N * 4 <= scratch.bytes)
      splits *= 2;
    if ((size_t)splits * rows.cap * N * 4 <= scratch.bytes &&
        gemm_stream_partial(s, A, W, N, K, rows, epilogue == EPI_SILU_MUL, splits, (float *)scratch.ptr)) {
      launch_reduce(s, N, rows, epilogue, out, ldo, splits, (const float *)scratch.ptr);
      return;
    }
  }
  if (fits32 && choice == 0 && scratch.ptr && N % 8 == 0) {
    // too few tiles for the chip: cut K so that about one workgroup per CU exists (each part an even number of slabs, at least 4)
    const int nk = K / 64;
    int splits = 1;
    while (splits < 16 && t128 * (splits * 2) <= 256 && nk % (splits * 4) == 0 && nk / (splits * 2) >= 4 &&
           (size_t)(splits * 2) * rows.cap * N * 4 <= scratch.bytes)
      splits *= 2;
    if (splits > 1 && launch_split(s, A, W, N, K, rows, epilogue, out, ldo, warm, splits, (float *)scratch.ptr)) return;
    if (launch_pipe<128, 8>(s, A, W, N, K, rows, epilogue, out, ldo, warm)) return;
  }
  const long tiles_big = (long)((est + 255) / 256) * ((N + 127) / 128);
  if (tiles_big >= 512) launch_mfma<256, 128>(s, A, W, N, K, rows, epilogue, out, ldo);
  else launch_mfma<128, 128>(s, A, W, N, K, rows, epilogue, out, ldo);
}

}  // namespace fk
