// Internal declarations shared by the translation units of libfocus: the context, the workspace
// plan and the host-side launch wrappers of every kernel.  Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "focus.h"

typedef __bf16 bf16_t;

namespace fk {

// Number of valid rows of a launch: the grid is sized for `cap` rows; kernels read the actual count
// from `count` (device memory, written earlier on the same stream) when it is not null.
struct Rows {
  int cap;
  const int32_t *count;
  int hint = 0;   // the host's guess of *count (0: none, plan for cap).  Tile shapes and K splits are chosen for it; a wrong
                  // guess costs time, never correctness: grids are sized for cap and kernels work from *count
  int expected() const { return hint > 0 && hint < cap ? hint : cap; }
};

// Device arrays indexed by sequence slot.
struct SlotState {
  int32_t *prefix_len;
  int32_t *page_table;    // [max_batch, table_stride]
  int32_t table_stride;
  int32_t *tokens;        // [max_batch, B]
  uint64_t *mask_bits;
  uint64_t *processed_bits;
  int64_t *token_sum;
  int32_t *total_steps;
  int32_t max_batch;
  int32_t *page_count;    // pages each slot's table really holds
  int32_t max_prefix_len;
  uint64_t *cached_bits;  // positions whose K/V is frozen in every layer (delayed intra-block cache, Sec. 4.3)
};

// Slot of batch entry b.  A caller-supplied slot list lives in device memory and cannot be checked on the
// host, so it is clamped into range here: a bad entry aliases another slot instead of leaving the workspace.
__device__ __forceinline__ int slot_of(const int32_t *seq_slot, int b, const SlotState &st) {
  if (!seq_slot) return b;
  int s = seq_slot[b];
  return s < 0 ? 0 : (s >= st.max_batch ? st.max_batch - 1 : s);
}

// How a kernel maps a row to its sequence: row_map[r] = b * B + p, slot = seq_slot ? seq_slot[b] : b.
struct RowIndex {
  const int32_t *row_map;
  const int32_t *seq_slot;
  int B;
};

// Geometry of the paged K/V pool for one layer.
struct KvLayer {
  void *base;             // start of this layer's pages
  int page_size, n_kv_heads, head_dim;
};

enum Epilogue {
  EPI_STORE = 0,     // out[dtype] = acc
  EPI_ADD_F32 = 1,   // out[f32] += acc
  EPI_STORE_F32 = 2, // out[f32] = acc
  EPI_SILU_MUL = 3,  // W = [gate rows; up rows] (N = 2F): out[dtype][m, f] = silu(gate) * up; only where gemm_fuses_silu_mul()
  EPI_PARTIAL_SILU = 4,  // internal to the K-split path: fp32 sums of the gate and up columns, weight-row order
  EPI_CONF = 5           // vocabulary projection without logits: per row and column range (max, sum exp(x - max), arg-max); only
                         // through gemm_conf_partials()
};
// Vocabulary projection fused with the first half of the confidence computation (Alg. 1 Decode_and_Verify): every wavefront of a
// projection tile reduces its columns of a row to (maximum, sum of exp(logit - maximum), lowest index of the maximum) and writes
// that triple to part[row * n_slots + slot] (3 floats, the index as int bits); confidence_from_partials() merges a row's slots in
// slot order.  The logits never reach memory.  False when the shape is not taken (few rows, fp32 model): the caller then
// materialises the logits and runs confidence().
bool gemm_conf_partials(hipStream_t s, int dtype, const void *A, const void *W, int N, int K, Rows rows, float *part, size_t part_bytes,
                        int *n_slots);
void confidence_from_partials(hipStream_t s, const float *part, int n_slots, Rows rows, float *conf, int32_t *argmax);
bool gemm_fuses_silu_mul(int dtype, const void *A, const void *W, int N, int K);

void embed(hipStream_t s, int dtype, const void *table, int hidden, Rows rows, RowIndex ri, SlotState st,
           int mask_id, float *resid);
void rmsnorm(hipStream_t s, int dtype, const float *x, const void *w, void *y, int hidden, float eps, Rows rows);
// Memory the kernel may touch on the side so that the next kernel finds it in the memory-side cache (a hint: kernels
// that cannot do it ignore it).
struct Warm {
  const void *ptr = nullptr;
  size_t bytes = 0;
};
// Device memory a projection may use for the fp32 partial sums of a K-split launch (none: no such launches).
struct Scratch {
  void *ptr = nullptr;
  size_t bytes = 0;
};
void gemm(hipStream_t s, int dtype, const void *A, const void *W, int N, int K, Rows rows, int epilogue,
          void *out, int ldo, Warm warm = Warm(), Scratch scratch = Scratch());
// Warm-up helper for kernels with one- or two-dimensional grids of short workgroups: the workgroups of the last round
// (the last min(grid, 256) in launch order) each read one dword of every 128-byte line of their share.  Returns a value
// the caller must keep alive (e.g. store it under a condition that never holds).
__device__ __forceinline__ unsigned warm_touch(const void *ptr, size_t bytes, int n_threads) {
  if (!ptr || !bytes) return 0;
  const long n_groups = (long)gridDim.x * gridDim.y, id = blockIdx.x + (long)blockIdx.y * gridDim.x;
  const long shares = n_groups < 256 ? n_groups : 256, share = id - (n_groups - shares);
  if (share < 0) return 0;
  const size_t lines = (bytes + 127) / 128, per = (lines + shares - 1) / shares;
  const size_t l0 = (size_t)share * per, l1 = l0 + per < lines ? l0 + per : lines;
  unsigned acc = 0;
  for (size_t l = l0 + threadIdx.x; l < l1; l += n_threads) acc ^= __builtin_nontemporal_load((const unsigned *)((const char *)ptr + l * 128));
  return acc;
}
// Rotates q and k rows of the fused qkv buffer in place and stores k, v of every row into its cache slot.
// n_seq, cu: the row range of every batch entry (rows cu[b] .. cu[b + 1]), or 0 / null when not known.
void rope_kv_write(hipStream_t s, int dtype, void *qkv, int n_q_heads, Rows rows, RowIndex ri, SlotState st,
                   KvLayer kv, const float2 *rope_table, int n_seq = 0, const int32_t *cu = nullptr);
struct AttnArgs {
  int dtype;
  const void *q;                 // [rows, q_stride] rotated queries, head h at column h * D
  int q_stride, n_q_heads;
  int n_seq;
  const int32_t *cu;             // rows of sequence b are cu[b] .. cu[b + 1]
  int max_rows_per_seq;          // rows per sequence the launch is shaped for (wavefronts per workgroup); a sequence with
                                 // more rows takes several passes over its K/V
  Rows rows;
  RowIndex ri;
  SlotState st;
  const uint64_t *vis_by_b;      // visible in-block positions per batch entry, null = all
  KvLayer kv;
  void *out;                     // [rows, H_q * D]
  float *part_o, *part_ml;       // split-K/V partials: [rows, H_q, max_splits, D] and [.., 2]
  int chunk, max_splits, launch_splits;
  const int32_t *order;          // batch entries sorted by descending prefix length (longest first), or null
  Warm warm;                     // weights of the projection that follows (bf16 kernel only)
  // Eq. 2 fused into this pass (the layer below the eviction layer, whose attention runs over the whole block anyway): when not
  // null, the workgroup that holds a sequence's last K/V range also reduces the in-block score tile of its query heads to
  // imp_partial[b, h, j] (the layout importance() writes).  attention() says whether it did.
  float *imp_partial = nullptr;
  int imp_pool_k = 3;
};
// Returns true when imp_partial was asked for and has been written by the attention launch itself.
bool attention(hipStream_t s, const AttnArgs &a);
// Eq. 2 per (sequence, query head): partial[b, h, j] = sum over the sequence's query rows (rows cu[b] .. cu[b + 1] of the
// fused qkv buffer, after the rotary embedding) of the pooled block-local softmax over the B in-block keys, which
// are read from the layer's K cache (every row's key has been written there; frozen positions keep theirs).
void importance(hipStream_t s, int dtype, const void *qkv, const int32_t *cu, int n_seq, int B, int n_q_heads, int n_kv_heads,
                int head_dim, int maxpool_k, const int32_t *seq_slot, SlotState st, KvLayer kv, float *partial);
// bits[b] = block positions of batch entry b that are not frozen
void uncached_bits(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st, uint64_t *bits);
struct SelectArgs {
  int n_seq, B, n_q_heads;
  const float *partial_prev, *partial_evict;   // [n, Hq, B] or null (then delta_in is used)
  const float *delta_in;                       // [n, B] or null
  int importance_mode, budget_mode, K_fixed, constraints;
  float alpha;
  const int32_t *k_override;
  const uint64_t *keep_override;
  const int32_t *seq_slot;
  SlotState st;
  int intra_block_cache;                       // Sec. 4.3: frozen positions are never retained, decoded unfrozen ones always
  int selection;                               // FOCUS_SELECT_*: pick by largest delta, by a random key, by smallest delta
  uint32_t selection_seed;
  int update_state;                            // processed_bits |= keep
  float *imp_prev_out, *imp_out, *delta_out;   // [n, B] or null
  int32_t *K_out;
  uint64_t *keep_out;
  int32_t *n_keep_out;
  uint64_t *vis_out;                           // [n] processed bits after the update, by batch index
};
void select(hipStream_t s, const SelectArgs &a);
// cu[b] = exclusive prefix sum of n_keep, row_map, cu[n] also to *total.
void scan_compact(hipStream_t s, int n_seq, int B, const uint64_t *keep_bits, int32_t *cu, int32_t *row_map,
                  int32_t *total);
// Packed row r = (b, p) is copied from row src_cu[b] + (number of src_bits[b] below p) of the source buffers
// (src_bits null: from row b * B + p).
void gather_rows(hipStream_t s, int dtype, Rows rows, const int32_t *row_map, int B, const int32_t *src_cu, const uint64_t *src_bits,
                 const float *resid, float *resid_p, int hidden, const void *qkv, int qkv_stride, void *q_p, int q_width);
void silu_mul(hipStream_t s, int dtype, const void *gate_up, void *act, int ffn, Rows rows);

// Mixture-of-experts feed-forward on normalised rows (token-choice routing: every row goes through its k best experts
// of E, each a SwiGLU feed-forward of inner width Fe; the outputs are mixed with the renormalised router probabilities).
// Work buffers, all in the workspace; "entry" i = row * k + j is the j-th expert choice of a row.
constexpr int kMoeTileRows = 128;     // rows of one expert that a workgroup of the grouped projections takes
struct MoeArgs {
  int dtype, n_experts, k, expert_ffn, hidden;
  float route_scale;
  Rows rows;
  const int32_t *row_map;             // row -> row id b * B + p (names the row in route_override and in the outputs)
  const void *u;                      // [rows, hidden] normalised rows
  const float *logits;                // [rows, E] router logits
  const int32_t *route_override;      // [row ids, k] experts to use instead of the router's pick, or null
  int32_t *topk_idx;                  // [rows * k (+4)] expert of every entry
  float *topk_w;                      // [rows * k] mixing weight of every entry
  int32_t *list;                      // [E, rows.cap] entries of every expert
  int32_t *count;                     // [E]
  int32_t *offs;                      // [E + 1] first expert-sorted row of every expert
  int32_t *tile_e, *tile_m0;          // [n_tile_slots] row tiles of the grouped projections: expert and first row inside it
  int32_t *n_tiles;                   // [1]
  int n_tile_slots;                   // host bound: rows.cap * k / kMoeTileRows + E
  int32_t *pos;                       // [rows * k] entry -> expert-sorted row
  int32_t *arow;                      // [rows * k] expert-sorted row -> row of u
  int32_t *aexp;                      // [rows * k] expert-sorted row -> expert
  const void *w_gate_up, *w_down;     // [E, 2 Fe, hidden], [E, hidden, Fe]
  void *act;                          // [rows * k, Fe] expert-sorted rows
  float *y;                           // [rows * k, hidden] expert outputs, expert-sorted rows
  float *resid;                       // [rows, hidden] += sum_j weight_j * y[pos[row * k + j]]
  int32_t *out_experts;               // optional outputs [row ids, k]
  float *out_weights;
};
// fp32 partial sums part[split][row][N] of a dense projection of few rows, by the weight-streaming kernel of the expert
// projections (false: shape not taken)
bool gemm_stream_partial(hipStream_t s, const void *A, const void *W, int N, int K, Rows rows, bool silu, int splits, float *part);
void moe_route(hipStream_t s, const MoeArgs &a);      // picks and weights
void moe_group(hipStream_t s, const MoeArgs &a);      // entries sorted by expert, tile list
void moe_experts(hipStream_t s, const MoeArgs &a);    // the two grouped projections
void moe_combine(hipStream_t s, const MoeArgs &a);    // weighted sum into the residual stream
void confidence(hipStream_t s, const float *logits, int vocab, Rows rows, float *conf, int32_t *argmax, Scratch scratch = Scratch());
struct CommitArgs {
  int n_seq, B;
  const int32_t *seq_slot;
  SlotState st;
  const uint64_t *keep_bits;
  const int32_t *cu;
  const float *conf;
  const int32_t *argmax;
  float threshold;
  int mask_id;
  int intra_block_cache;     // freeze positions by the neighbour-aware stability criterion (Sec. 4.3)
  int32_t *tokens_out;       // [n, B] or null
  uint64_t *mask_out;
  int32_t *n_decoded_out;
};
void commit(hipStream_t s, const CommitArgs &a);
// Prefill helper: installs chunk c of every prompt as the block (unmasked tokens, prefix_len = c * B).
void prefill_chunk_setup(hipStream_t s, int n_seq, int B, int chunk, const int32_t *seq_slot, SlotState st,
                         const int32_t *prompt, const int32_t *prompt_offset, const int32_t *prompt_len,
                         uint64_t *keep_bits);
void reset_block_state(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st,
                       const int32_t *prefix_len, int mask_id, int keep_stats);
// Multi-block generation: picks the sequences whose block is complete (and that have room for another block),
// and, after their last forward, turns the block into prefix and starts a new all-masked block.
void finalize_pick(hipStream_t s, int n_seq, int B, int page_size, const int32_t *seq_slot, SlotState st, uint64_t *keep_bits,
                   int32_t *finalized);
void finalize_advance(hipStream_t s, int n_seq, int B, const int32_t *seq_slot, SlotState st, const int32_t *finalized, int mask_id);
void fill_u64(hipStream_t s, uint64_t *p, int n, uint64_t v);
void add_counts(hipStream_t s, int n, const int32_t *counts, int64_t *totals);   // totals[i] += counts[i]
void iota_rows(hipStream_t s, int32_t *row_map, int32_t *cu, int n_seq, int B, int32_t *total);
// order[rank] = batch entry, ranked by descending prefix length (ties: lower entry first)
void length_order(hipStream_t s, int n_seq, const int32_t *seq_slot, SlotState st, int32_t *order);

}  // namespace fk
