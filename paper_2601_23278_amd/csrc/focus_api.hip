// C ABI of libfocus: argument checks, the workspace plan, and the order in which the kernels of one FOCUS
// step (Algorithm 1) are enqueued.  All arithmetic lives in the kernels.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "focus_internal.h"

namespace {

std::string g_error;   // last error of a call that had no context

// Scratch of focus_select_compact_noalloc: per-sequence retained counts and the packed row total.  One copy per GPU, held
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device address of
// each GPU's copy is looked up once per device (scratch_of_current_device) and that pointer is what kernels get.
constexpr int kNoallocScratchInts = FOCUS_NOALLOC_MAX_SEQ + 64;
static __device__ __align__(256) int32_t scratch[kNoallocScratchInts];
constexpr int kMaxDevices = 64;
int32_t *g_scratch_ptr[kMaxDevices];

constexpr int kMaxTimed = 4096;
constexpr int kTargetAttnGroups = 2048;   // (sequence, kv head, split) workgroups the attention launch aims for

struct Plan {
  size_t off_prefix_len, off_page_count, off_page_table, off_tokens, off_mask, off_processed, off_cached, off_token_sum, off_total_steps;
  size_t off_rope, off_resid, off_resid_p, off_normed, off_qkv, off_q_p, off_attn, off_gate_up, off_act, off_logits;
  size_t off_partial, off_delta, off_K, off_keep, off_n_keep, off_vis, off_cu, off_cu_full, off_row_map,
      off_row_map_full, off_total, off_total_full, off_conf, off_argmax, off_prompt, off_prompt_off, off_prompt_len,
      off_slot_list, off_part_o, off_part_ml, off_order, off_uncached, off_finalized;
  // mixture-of-experts work buffers (zero-sized for a dense model)
  size_t off_moe_logits, off_moe_idx, off_moe_w, off_moe_list, off_moe_count, off_moe_offs, off_moe_tile_e, off_moe_tile_m0,
      off_moe_ntiles, off_moe_pos, off_moe_arow, off_moe_aexp, off_moe_act, off_moe_y;
  size_t off_n_dec;                  // tokens decoded by the current step of focus_run_steps
  size_t off_splitk, splitk_bytes;   // fp32 partial sums of K-split projections (launches with few rows)
  size_t bytes, part_entries;
  int table_stride, max_rows, max_pos, moe_tile_slots;
};

size_t esize(int dtype) { return dtype == FOCUS_F32 ? 4 : 2; }

Plan make_plan(const focus_config &c) {
  Plan p{};
  size_t at = 0;
  auto take = [&](size_t bytes) { size_t o = at; at += (bytes + 255) & ~(size_t)255; return o; };
  const size_t nb = c.max_batch, B = c.block_size, rows = nb * B, es = esize(c.dtype);
  const size_t qkv_w = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, q_w = (size_t)c.n_q_heads * c.head_dim;
  p.table_stride = (c.max_prefix_len + c.block_size + c.page_size - 1) / c.page_size;
  p.max_rows = (int)rows;
  p.max_pos = c.max_prefix_len + c.block_size;
  p.off_prefix_len = take(nb * 4);
  p.off_page_count = take(nb * 4);
  p.off_page_table = take(nb * p.table_stride * 4);
  p.off_tokens = take(rows * 4);
  p.off_mask = take(nb * 8);
  p.off_processed = take(nb * 8);
  p.off_cached = take(nb * 8);
  p.off_token_sum = take(nb * 8);
  p.off_total_steps = take(nb * 4);
  p.off_rope = take((size_t)p.max_pos * (c.head_dim / 2) * sizeof(float2));
  p.off_resid = take(rows * c.hidden * 4);
  p.off_resid_p = take(rows * c.hidden * 4);
  p.off_normed = take(rows * c.hidden * es);
  p.off_qkv = take(rows * qkv_w * es);
  p.off_q_p = take(rows * q_w * es);
  p.off_attn = take(rows * q_w * es);
  const size_t ffn_w = c.n_experts > 0 ? (size_t)std::max(c.ffn, c.shared_ffn) : (size_t)c.ffn;   // dense and shared-expert feed-forward
  p.off_gate_up = take(rows * 2 * ffn_w * es);
  p.off_act = take(rows * ffn_w * es);
  p.off_logits = take(rows * (size_t)c.vocab * 4);
  p.off_partial = take(2 * nb * c.n_q_heads * B * 4);
  p.off_delta = take(rows * 4);
  p.off_K = take(nb * 4);
  p.off_keep = take(nb * 8);
  p.off_n_keep = take(nb * 4);
  p.off_vis = take(nb * 8);
  p.off_cu = take((nb + 1) * 4);
  p.off_cu_full = take((nb + 1) * 4);
  p.off_row_map = take(rows * 4);
  p.off_row_map_full = take(rows * 4);
  p.off_total = take(4);
  p.off_total_full = take(4);
  p.off_conf = take(rows * 4);
  p.off_argmax = take(rows * 4);
  p.off_prompt = take(nb * (size_t)c.max_prefix_len * 4);
  p.off_prompt_off = take(nb * 4);
  p.off_prompt_len = take(nb * 4);
  p.off_slot_list = take(nb * 4);
  // split-K/V partials of the attention: (row, head, split) entries; the launch policy keeps
  // rows * H_q * splits within  B * group * kTargetAttnGroups + max_rows * H_q
  p.part_entries = c.dtype == FOCUS_BF16 ? (size_t)B * (c.n_q_heads / c.n_kv_heads) * kTargetAttnGroups + rows * c.n_q_heads : 0;
  p.off_part_o = take(p.part_entries * c.head_dim * 4);
  p.off_part_ml = take(p.part_entries * 2 * 4);
  p.off_order = take(nb * 4);
  p.off_uncached = take(nb * 8);
  p.off_finalized = take(nb * 4);
  p.off_n_dec = take(nb * 4);
  p.splitk_bytes = c.dtype == FOCUS_BF16 ? (size_t)64 << 20 : 0;
  p.off_splitk = take(p.splitk_bytes);
  if (c.n_experts > 0) {
    const size_t E = c.n_experts, ent = rows * c.experts_per_token;
    p.moe_tile_slots = (int)(ent / fk::kMoeTileRows + E);
    p.off_moe_logits = take(rows * E * 4);
    p.off_moe_idx = take((ent + 1024) * 4);          // read in 1024-entry trips
    p.off_moe_w = take(ent * 4);
    p.off_moe_list = take(E * rows * 4);
    p.off_moe_count = take(E * 4);
    p.off_moe_offs = take((E + 1) * 4);
    p.off_moe_tile_e = take((size_t)p.moe_tile_slots * 4);
    p.off_moe_tile_m0 = take((size_t)p.moe_tile_slots * 4);
    p.off_moe_ntiles = take(4);
    p.off_moe_pos = take(ent * 4);
    p.off_moe_arow = take(ent * 4);
    p.off_moe_aexp = take(ent * 4);
    p.off_moe_act = take(ent * c.expert_ffn * es);
    p.off_moe_y = take(ent * c.hidden * 4);
  }
  p.bytes = at;
  return p;
}

const char *check_config(const focus_config &c) {
  if (c.n_layers < 1 || c.hidden < 8 || c.hidden % 8) return "hidden must be a positive multiple of 8";
  if (c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
  if (c.head_dim != 64 && c.head_dim != 128) return "head_dim must be 64 or 128";
  if (c.ffn < 8 || c.ffn % 8 || c.vocab < 2) return "ffn must be a multiple of 8 and vocab at least 2";
  if (c.dtype != FOCUS_F32 && c.dtype != FOCUS_BF16) return "dtype must be FOCUS_F32 or FOCUS_BF16";
  if (c.block_size < 1 || c.block_size > FOCUS_MAX_BLOCK) return "block_size must be in 1..64";
  if (c.mask_token_id < 0 || c.mask_token_id >= c.vocab) return "mask_token_id outside the vocabulary";
  if (c.max_batch < 1 || c.max_prefix_len < 0 || c.page_size < 1 || c.n_pages < 1) return "bad batch / prefix / page sizes";
  if ((size_t)c.max_batch * c.block_size > (1u << 24)) return "max_batch * block_size too large";
  if (c.importance_mode != 0 && c.importance_mode != 1) return "importance_mode must be 0 or 1";
  if (c.evict_layer < (c.importance_mode == 0 ? 1 : 0) || c.evict_layer >= c.n_layers)
    return "evict_layer must satisfy 1 <= e < n_layers (0 <= e with importance_mode 1)";
  if (c.maxpool_k != 1 && c.maxpool_k != 3) return "maxpool_k must be 1 or 3";
  if (c.budget_mode < 0 || c.budget_mode > 3) return "unknown budget_mode";
  if (c.constraints & ~3) return "unknown constraint bits";
  if (c.intra_block_cache != 0 && c.intra_block_cache != 1) return "intra_block_cache must be 0 or 1";
  if (c.selection < FOCUS_SELECT_TOP || c.selection > FOCUS_SELECT_BOTTOM) return "selection must be a FOCUS_SELECT_* value";
  if (!(c.rms_eps > 0.f) || !(c.rope_base > 1.f)) return "rms_eps must be > 0 and rope_base > 1";
  if (c.n_experts < 0 || c.n_experts > 512) return "n_experts must be in 0..512";
  if (c.n_experts > 0) {
    if (c.experts_per_token < 1 || c.experts_per_token > c.n_experts || c.experts_per_token > 32) return "experts_per_token must be in 1..min(n_experts, 32)";
    if (c.expert_ffn < 8 || c.expert_ffn % 8 || c.shared_ffn < 0 || c.shared_ffn % 8) return "expert_ffn and shared_ffn must be multiples of 8";
    if (c.first_moe_layer < 0 || c.first_moe_layer > c.n_layers) return "first_moe_layer must be in 0..n_layers";
    if (!(c.route_scale > 0.f)) return "route_scale must be > 0";
    if ((double)c.max_batch * c.block_size * c.experts_per_token > (double)(1u << 26)) return "max_batch * block_size * experts_per_token too large";
  }
  return nullptr;
}

}  // namespace

struct focus_ctx {
  focus_config cfg;
  Plan plan;
  char *ws;
  char *kv_pool;
  const void *embed, *lm_head, *final_norm;
  std::vector<const void *> attn_norm, w_qkv, w_o, mlp_norm, w_gate_up, w_down;
  std::vector<const void *> w_router, w_expert_gate_up, w_expert_down, w_shared_gate_up, w_shared_down;
  // forced routing (focus_set_route_override) and the routing outputs of the running step; planes of max_batch * B * k per layer
  const int32_t *route_override = nullptr;
  int32_t *out_route_experts = nullptr;
  float *out_route_weights = nullptr;
  bool route_by_row_id = false;         // inside focus_step / focus_run_layers: rows are block positions of the step's batch
  std::string error;
  // timing
  bool timing = false;
  std::vector<hipEvent_t> ev;          // pairs
  std::vector<int> ev_class;
  int n_timed = 0;
  hipStream_t last_stream = nullptr;
  int max_total = 0;                   // host-side bound of prefix_len + B over the installed sequences
  int hint_rows = 0, hint_rows_per_seq = 0;   // focus_set_row_hint: expected packed rows of a step / per sequence (0: none)

  template <typename T> T *at(size_t off) const { return (T *)(ws + off); }
  fk::SlotState slots() const {
    return {at<int32_t>(plan.off_prefix_len), at<int32_t>(plan.off_page_table), plan.table_stride,
            at<int32_t>(plan.off_tokens), at<uint64_t>(plan.off_mask), at<uint64_t>(plan.off_processed),
            at<int64_t>(plan.off_token_sum), at<int32_t>(plan.off_total_steps), cfg.max_batch,
            at<int32_t>(plan.off_page_count), cfg.max_prefix_len, at<uint64_t>(plan.off_cached)};
  }
  fk::Scratch scratch() const { return fk::Scratch{plan.splitk_bytes ? ws + plan.off_splitk : nullptr, plan.splitk_bytes}; }
  bool moe_layer(int l) const { return cfg.n_experts > 0 && l >= cfg.first_moe_layer; }
  fk::KvLayer kv_layer(int l) const {
    size_t layer_bytes = (size_t)cfg.n_pages * 2 * cfg.n_kv_heads * cfg.page_size * cfg.head_dim * esize(cfg.dtype);
    return {kv_pool + (size_t)l * layer_bytes, cfg.page_size, cfg.n_kv_heads, cfg.head_dim};
  }
};

namespace {

int fail(focus_ctx *ctx, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  (ctx ? ctx->error : g_error) = buf;
  return code;
}

#define HIP_TRY(ctx, expr)                                                                         \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(ctx, FOCUS_EHIP, "%s: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

// Device address of the current GPU's copy of `scratch`, looked up on the first call per device (focus_init does it for the
// device a context is created on).  Null with the error stored when the lookup fails.
int32_t *scratch_of_current_device(focus_ctx *ctx) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(ctx, FOCUS_EHIP, "hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    return nullptr;
  }
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fail(ctx, FOCUS_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = (int32_t *)p;
  }
  return g_scratch_ptr[dev];
}

// Brackets the launches of one kernel class with an event pair when timing is on.
struct Timed {
  focus_ctx *c;
  hipStream_t s;
  int idx = -1;
  Timed(focus_ctx *c_, hipStream_t s_, int kclass) : c(c_), s(s_) {
    if (c->timing && c->n_timed < kMaxTimed) {
      idx = c->n_timed++;
      c->ev_class[idx] = kclass;
      (void)hipEventRecord(c->ev[2 * idx], s);
    }
  }
  ~Timed() {
    if (idx >= 0) (void)hipEventRecord(c->ev[2 * idx + 1], s);
  }
};

// While alive, the rows of the layers are block positions of the caller's batch: forced routing applies and the routing
// outputs are written.  Prefill and block finalisation run without it.
struct RouteScope {
  focus_ctx *c;
  RouteScope(focus_ctx *c_, int32_t *experts, float *weights) : c(c_) {
    c->route_by_row_id = true; c->out_route_experts = experts; c->out_route_weights = weights;
  }
  ~RouteScope() { c->route_by_row_id = false; c->out_route_experts = nullptr; c->out_route_weights = nullptr; }
};

struct RowSet {        // a set of rows the layers run on
  fk::Rows rows;
  fk::RowIndex ri;
  int n_seq;
  const int32_t *cu;   // rows of sequence b: cu[b] .. cu[b + 1]
  int max_rows_per_seq;
  const int32_t *order;   // attention launch order (longest sequence first) or null
};

// K/V split size for the attention launch: whole sequences when there are enough (sequence, kv head) groups
// to fill the chip, otherwise cut so that about kTargetAttnGroups workgroups exist; always a multiple of the
// 64-token tile and never so small that the partial buffer would overflow.
void attention_split(const focus_ctx *c, int n_seq, int rows_cap, int *chunk, int *splits);

// rmsnorm -> QKV projection -> rotary + K/V write, for every row of the set (App. C ordering).
void layer_qkv(focus_ctx *c, hipStream_t s, int l, const RowSet &rs, const float *resid) {
  const focus_config &g = c->cfg;
  const int qkv_w = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
  void *normed = c->at<char>(c->plan.off_normed), *qkv = c->at<char>(c->plan.off_qkv);
  { Timed t(c, s, FOCUS_KC_POINTWISE); fk::rmsnorm(s, g.dtype, resid, c->attn_norm[l], normed, g.hidden, g.rms_eps, rs.rows); }
  { Timed t(c, s, FOCUS_KC_GEMM); fk::gemm(s, g.dtype, normed, c->w_qkv[l], qkv_w, g.hidden, rs.rows, fk::EPI_STORE, qkv, qkv_w, fk::Warm(), c->scratch()); }
  { Timed t(c, s, FOCUS_KC_KV_WRITE);
    fk::rope_kv_write(s, g.dtype, qkv, g.n_q_heads, rs.rows, rs.ri, c->slots(), c->kv_layer(l), c->at<float2>(c->plan.off_rope), rs.n_seq, rs.cu); }
}

void swiglu_ffn(focus_ctx *c, hipStream_t s, const RowSet &rs, const void *normed, const void *w_gate_up, const void *w_down, int ffn,
                float *resid, fk::Warm warm_after);
void moe_ffn(focus_ctx *c, hipStream_t s, int l, const RowSet &rs, float *resid, const void *normed);

// attention -> O projection (+residual) -> rmsnorm -> feed-forward (+residual).
// imp_partial: Eq. 2 of this layer is wanted at that address ([n, H_q, B] per-head sums); the attention launch computes it on the
// way when it can, else the stand-alone kernel runs.
void layer_rest(focus_ctx *c, hipStream_t s, int l, const RowSet &rs, float *resid, const void *q, int q_stride,
                const uint64_t *vis_by_b, float *imp_partial = nullptr) {
  const focus_config &g = c->cfg;
  const int q_w = g.n_q_heads * g.head_dim;
  void *normed = c->at<char>(c->plan.off_normed), *attn = c->at<char>(c->plan.off_attn);
  { Timed t(c, s, FOCUS_KC_ATTENTION);
    fk::AttnArgs a{};
    a.dtype = g.dtype; a.q = q; a.q_stride = q_stride; a.n_q_heads = g.n_q_heads; a.n_seq = rs.n_seq; a.cu = rs.cu;
    a.max_rows_per_seq = rs.max_rows_per_seq; a.rows = rs.rows; a.ri = rs.ri; a.st = c->slots(); a.vis_by_b = vis_by_b;
    a.kv = c->kv_layer(l); a.out = attn;
    a.part_o = c->plan.part_entries ? c->at<float>(c->plan.off_part_o) : nullptr;
    a.part_ml = c->plan.part_entries ? c->at<float>(c->plan.off_part_ml) : nullptr;
    a.order = rs.order;
    a.warm = fk::Warm{c->w_o[l], (size_t)g.hidden * q_w * esize(g.dtype)};
    attention_split(c, rs.n_seq, rs.rows.cap, &a.chunk, &a.launch_splits);
    a.max_splits = a.launch_splits;
    a.imp_partial = imp_partial; a.imp_pool_k = g.maxpool_k;
    if (fk::attention(s, a)) imp_partial = nullptr; }
  if (imp_partial) {
    Timed t(c, s, FOCUS_KC_IMPORTANCE);
    fk::importance(s, g.dtype, q, rs.cu, rs.n_seq, g.block_size, g.n_q_heads, g.n_kv_heads, g.head_dim, g.maxpool_k, rs.ri.seq_slot, c->slots(), c->kv_layer(l), imp_partial);
  }
  { Timed t(c, s, FOCUS_KC_GEMM); fk::gemm(s, g.dtype, attn, c->w_o[l], g.hidden, q_w, rs.rows, fk::EPI_ADD_F32, resid, g.hidden, fk::Warm(), c->scratch()); }
  { Timed t(c, s, FOCUS_KC_POINTWISE); fk::rmsnorm(s, g.dtype, resid, c->mlp_norm[l], normed, g.hidden, g.rms_eps, rs.rows); }
  const size_t qkv_bytes = (size_t)(g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim * g.hidden * esize(g.dtype);
  const fk::Warm next_qkv = l + 1 < g.n_layers ? fk::Warm{c->w_qkv[l + 1], qkv_bytes} : fk::Warm();
  if (c->moe_layer(l)) {
    moe_ffn(c, s, l, rs, resid, normed);
    return;
  }
  swiglu_ffn(c, s, rs, normed, c->w_gate_up[l], c->w_down[l], g.ffn, resid, next_qkv);
}

// SwiGLU feed-forward on normalised rows, added to the residual stream: gate/up -> SiLU*up -> down.
void swiglu_ffn(focus_ctx *c, hipStream_t s, const RowSet &rs, const void *normed, const void *w_gate_up, const void *w_down, int ffn,
                float *resid, fk::Warm warm_after) {
  const focus_config &g = c->cfg;
  void *gate_up = c->at<char>(c->plan.off_gate_up), *act = c->at<char>(c->plan.off_act);
  if (fk::gemm_fuses_silu_mul(g.dtype, normed, w_gate_up, 2 * ffn, g.hidden)) {
    Timed t(c, s, FOCUS_KC_GEMM);
    fk::gemm(s, g.dtype, normed, w_gate_up, 2 * ffn, g.hidden, rs.rows, fk::EPI_SILU_MUL, act, ffn,
             fk::Warm{w_down, (size_t)g.hidden * ffn * esize(g.dtype)}, c->scratch());
  } else {
    { Timed t(c, s, FOCUS_KC_GEMM); fk::gemm(s, g.dtype, normed, w_gate_up, 2 * ffn, g.hidden, rs.rows, fk::EPI_STORE, gate_up, 2 * ffn, fk::Warm(), c->scratch()); }
    { Timed t(c, s, FOCUS_KC_POINTWISE); fk::silu_mul(s, g.dtype, gate_up, act, ffn, rs.rows); }
  }
  { Timed t(c, s, FOCUS_KC_GEMM); fk::gemm(s, g.dtype, act, w_down, g.hidden, ffn, rs.rows, fk::EPI_ADD_F32, resid, g.hidden, warm_after, c->scratch()); }
}

// Mixture-of-experts feed-forward on normalised rows, added to the residual stream: router logits -> picks and weights ->
// entries sorted by expert -> grouped gate/up and down projections -> weighted sum; plus the shared expert, if any.
void moe_ffn(focus_ctx *c, hipStream_t s, int l, const RowSet &rs, float *resid, const void *normed) {
  const focus_config &g = c->cfg;
  const Plan &pl = c->plan;
  const size_t plane = (size_t)g.max_batch * g.block_size * g.experts_per_token;
  fk::MoeArgs a{};
  a.dtype = g.dtype; a.n_experts = g.n_experts; a.k = g.experts_per_token; a.expert_ffn = g.expert_ffn; a.hidden = g.hidden;
  a.route_scale = g.route_scale; a.rows = rs.rows; a.row_map = rs.ri.row_map; a.u = normed;
  a.logits = c->at<float>(pl.off_moe_logits);
  a.route_override = c->route_by_row_id && c->route_override ? c->route_override + (size_t)l * plane : nullptr;
  a.topk_idx = c->at<int32_t>(pl.off_moe_idx); a.topk_w = c->at<float>(pl.off_moe_w);
  a.list = c->at<int32_t>(pl.off_moe_list); a.count = c->at<int32_t>(pl.off_moe_count); a.offs = c->at<int32_t>(pl.off_moe_offs);
  a.tile_e = c->at<int32_t>(pl.off_moe_tile_e); a.tile_m0 = c->at<int32_t>(pl.off_moe_tile_m0); a.n_tiles = c->at<int32_t>(pl.off_moe_ntiles);
  a.n_tile_slots = std::min(pl.moe_tile_slots, rs.rows.cap * g.experts_per_token / fk::kMoeTileRows + g.n_experts);
  a.pos = c->at<int32_t>(pl.off_moe_pos); a.arow = c->at<int32_t>(pl.off_moe_arow); a.aexp = c->at<int32_t>(pl.off_moe_aexp);
  a.w_gate_up = c->w_expert_gate_up[l]; a.w_down = c->w_expert_down[l];
  a.act = c->at<char>(pl.off_moe_act); a.y = c->at<float>(pl.off_moe_y); a.resid = resid;
  a.out_experts = c->route_by_row_id && c->out_route_experts ? c->out_route_experts + (size_t)l * plane : nullptr;
  a.out_weights = c->route_by_row_id && c->out_route_weights ? c->out_route_weights + (size_t)l * plane : nullptr;
  { Timed t(c, s, FOCUS_KC_GEMM);
    fk::gemm(s, g.dtype, normed, c->w_router[l], g.n_experts, g.hidden, rs.rows, fk::EPI_STORE_F32, c->at<float>(pl.off_moe_logits), g.n_experts, fk::Warm(), c->scratch()); }
  { Timed t(c, s, FOCUS_KC_ROUTE); fk::moe_route(s, a); fk::moe_group(s, a); }
  { Timed t(c, s, FOCUS_KC_EXPERTS); fk::moe_experts(s, a); }
  // the shared expert adds into the residual stream before the routed sum (both orders are the same sum)
  if (g.shared_ffn > 0) swiglu_ffn(c, s, rs, normed, c->w_shared_gate_up[l], c->w_shared_down[l], g.shared_ffn, resid, fk::Warm());
  { Timed t(c, s, FOCUS_KC_ROUTE); fk::moe_combine(s, a); }
}

void attention_split(const focus_ctx *c, int n_seq, int rows_cap, int *chunk, int *splits) {
  const focus_config &g = c->cfg;
  const int max_total = c->max_total > 0 ? c->max_total : g.max_prefix_len + g.block_size;
  const long groups = (long)n_seq * g.n_kv_heads;
  long want = (groups >= kTargetAttnGroups) ? 1 : (kTargetAttnGroups + groups - 1) / groups;   // splits per sequence
  // with several hundred (sequence, kv head) groups a split of fewer than 4096 tokens costs more in start-up and in the merge
  // than its extra workgroups gain (measured: batch 128 with prefixes up to 2048 runs 8 % faster unsplit, batch 64 with
  // prefixes up to 32768 15 % slower with two splits than with four); a handful of sequences needs every workgroup it can get
  want = std::max(1L, std::min(want, (long)max_total / (groups >= 512 ? 4096 : 512)));
  long ch = ((max_total + want - 1) / want + 63) / 64 * 64;
  if (ch < 256) ch = 256;
  // partial buffer: rows * H_q * splits entries
  while (c->plan.part_entries && (long)rows_cap * g.n_q_heads * ((max_total + ch - 1) / ch) > (long)c->plan.part_entries) ch *= 2;
  *chunk = (int)ch;
  *splits = (int)((max_total + ch - 1) / ch);
}

int check_batch(focus_ctx *ctx, int n_seq) {
  if (!ctx) return fail(nullptr, FOCUS_EINVAL, "null context");
  if (n_seq < 0 || n_seq > ctx->cfg.max_batch) return fail(ctx, FOCUS_EINVAL, "n_seq %d outside 0..max_batch %d", n_seq, ctx->cfg.max_batch);
  return FOCUS_OK;
}

int fixed_budget(const focus_config &g) {
  if (g.budget_mode == FOCUS_BUDGET_TOPK) return g.topk;
  if (g.budget_mode == FOCUS_BUDGET_RATIO) return (int)ceil((double)g.keep_ratio * (double)g.block_size);
  return g.block_size;
}

// Upper bound of the packed row count that the host can know without reading the device.
int packed_cap(const focus_config &g, int n_seq, bool overridden) {
  if (overridden || g.constraints || g.intra_block_cache || g.budget_mode >= FOCUS_BUDGET_DYNAMIC) return n_seq * g.block_size;
  int k = fixed_budget(g);
  k = k < 0 ? 0 : (k > g.block_size ? g.block_size : k);
  return n_seq * k;
}

}  // namespace

extern "C" {

int focus_workspace_bytes(const focus_config *cfg, size_t *bytes) {
  if (!cfg || !bytes) return fail(nullptr, FOCUS_EINVAL, "null argument");
  if (const char *m = check_config(*cfg)) return fail(nullptr, FOCUS_EINVAL, "%s", m);
  *bytes = make_plan(*cfg).bytes;
  return FOCUS_OK;
}

int focus_kv_pool_bytes(const focus_config *cfg, size_t *bytes) {
  if (!cfg || !bytes) return fail(nullptr, FOCUS_EINVAL, "null argument");
  if (const char *m = check_config(*cfg)) return fail(nullptr, FOCUS_EINVAL, "%s", m);
  *bytes = (size_t)cfg->n_layers * cfg->n_pages * 2 * cfg->n_kv_heads * cfg->page_size * cfg->head_dim * esize(cfg->dtype);
  return FOCUS_OK;
}

int focus_init(const focus_config *cfg, const focus_weights *w, void *kv_pool, size_t kv_pool_bytes, void *workspace,
               size_t workspace_bytes, focus_ctx **out) {
  if (!cfg || !w || !kv_pool || !workspace || !out) return fail(nullptr, FOCUS_EINVAL, "null argument");
  if (const char *m = check_config(*cfg)) return fail(nullptr, FOCUS_EINVAL, "%s", m);
  const bool all_moe = cfg->n_experts > 0 && cfg->first_moe_layer == 0;
  if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->w_qkv || !w->w_o || !w->mlp_norm ||
      (!all_moe && (!w->w_gate_up || !w->w_down)))
    return fail(nullptr, FOCUS_EINVAL, "null weight pointer");
  const bool moe = cfg->n_experts > 0;
  if (moe && (!w->w_router || !w->w_expert_gate_up || !w->w_expert_down || (cfg->shared_ffn > 0 && (!w->w_shared_gate_up || !w->w_shared_down))))
    return fail(nullptr, FOCUS_EINVAL, "null expert weight pointer");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const bool ml = moe && l >= cfg->first_moe_layer;
    if (!w->attn_norm[l] || !w->w_qkv[l] || !w->w_o[l] || !w->mlp_norm[l] || (!ml && (!w->w_gate_up[l] || !w->w_down[l])))
      return fail(nullptr, FOCUS_EINVAL, "null weight pointer in layer %d", l);
    if (ml && (!w->w_router[l] || !w->w_expert_gate_up[l] || !w->w_expert_down[l] ||
               (cfg->shared_ffn > 0 && (!w->w_shared_gate_up[l] || !w->w_shared_down[l]))))
      return fail(nullptr, FOCUS_EINVAL, "null expert weight pointer in layer %d", l);
  }
  if (((uintptr_t)workspace & 255) || ((uintptr_t)kv_pool & 15)) return fail(nullptr, FOCUS_EINVAL, "workspace must be 256-byte and kv_pool 16-byte aligned");
  Plan plan = make_plan(*cfg);
  size_t need_kv;
  focus_kv_pool_bytes(cfg, &need_kv);
  if (workspace_bytes < plan.bytes) return fail(nullptr, FOCUS_ENOMEM, "workspace too small: %zu < %zu", workspace_bytes, plan.bytes);
  if (kv_pool_bytes < need_kv) return fail(nullptr, FOCUS_ENOMEM, "kv pool too small: %zu < %zu", kv_pool_bytes, need_kv);

  focus_ctx *c = new (std::nothrow) focus_ctx();
  if (!c) return fail(nullptr, FOCUS_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  c->plan = plan;
  c->ws = (char *)workspace;
  c->kv_pool = (char *)kv_pool;
  c->embed = w->embed; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
  c->attn_norm.assign(w->attn_norm, w->attn_norm + cfg->n_layers);
  c->w_qkv.assign(w->w_qkv, w->w_qkv + cfg->n_layers);
  c->w_o.assign(w->w_o, w->w_o + cfg->n_layers);
  c->mlp_norm.assign(w->mlp_norm, w->mlp_norm + cfg->n_layers);
  c->w_gate_up.assign(cfg->n_layers, nullptr);
  c->w_down.assign(cfg->n_layers, nullptr);
  for (int l = 0; l < cfg->n_layers && !all_moe; ++l) { c->w_gate_up[l] = w->w_gate_up[l]; c->w_down[l] = w->w_down[l]; }
  if (moe) {
    c->w_router.assign(w->w_router, w->w_router + cfg->n_layers);
    c->w_expert_gate_up.assign(w->w_expert_gate_up, w->w_expert_gate_up + cfg->n_layers);
    c->w_expert_down.assign(w->w_expert_down, w->w_expert_down + cfg->n_layers);
    if (cfg->shared_ffn > 0) {
      c->w_shared_gate_up.assign(w->w_shared_gate_up, w->w_shared_gate_up + cfg->n_layers);
      c->w_shared_down.assign(w->w_shared_down, w->w_shared_down + cfg->n_layers);
    }
  }

  // rotary table in fp64 on the host: (cos, sin)(pos * base^(-2i/D)), rounded once to fp32
  const int half = cfg->head_dim / 2;
  std::vector<float2> rope((size_t)plan.max_pos * half);
  for (int pos = 0; pos < plan.max_pos; ++pos)
    for (int i = 0; i < half; ++i) {
      double ang = (double)pos * pow((double)cfg->rope_base, -2.0 * i / cfg->head_dim);
      rope[(size_t)pos * half + i] = make_float2((float)cos(ang), (float)sin(ang));
    }
  hipError_t e = hipMemcpy(c->ws + plan.off_rope, rope.data(), rope.size() * sizeof(float2), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemset(c->ws, 0, plan.off_rope);   // slot state
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    int rc = fail(nullptr, FOCUS_EHIP, "focus_init: %s", hipGetErrorString(e));
    delete c;
    return rc;
  }
  if (!scratch_of_current_device(nullptr)) {   // set-up for focus_select_compact_noalloc on this device
    delete c;
    return FOCUS_EHIP;
  }
  *out = c;
  return FOCUS_OK;
}

int focus_free(focus_ctx *ctx) {
  if (!ctx) return FOCUS_OK;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
  return FOCUS_OK;
}

const char *focus_last_error(const focus_ctx *ctx) { return ctx ? ctx->error.c_str() : g_error.c_str(); }

int focus_set_timing(focus_ctx *ctx, int32_t enable) {
  if (!ctx) return fail(nullptr, FOCUS_EINVAL, "null context");
  if (enable && ctx->ev.empty()) {
    ctx->ev.resize(2 * kMaxTimed);
    ctx->ev_class.resize(kMaxTimed);
    for (auto &e : ctx->ev) HIP_TRY(ctx, hipEventCreate(&e));
  }
  ctx->timing = enable != 0;
  ctx->n_timed = 0;
  return FOCUS_OK;
}

int focus_get_kernel_time(focus_ctx *ctx, int32_t kclass, float *total_ms, int32_t *launches) {
  if (!ctx || !total_ms || !launches) return fail(ctx, FOCUS_EINVAL, "null argument");
  if (kclass < 0 || kclass >= FOCUS_KC_COUNT) return fail(ctx, FOCUS_EINVAL, "unknown kernel class %d", kclass);
  HIP_TRY(ctx, hipStreamSynchronize(ctx->last_stream));
  float sum = 0.f;
  int n = 0;
  for (int i = 0; i < ctx->n_timed; ++i)
    if (ctx->ev_class[i] == kclass) {
      float ms = 0.f;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->ev[2 * i], ctx->ev[2 * i + 1]));
      sum += ms;
      ++n;
    }
  *total_ms = sum;
  *launches = n;
  return FOCUS_OK;
}

int focus_get_state(focus_ctx *ctx, int32_t slot, focus_seq_state *st) {
  if (!ctx || !st) return fail(ctx, FOCUS_EINVAL, "null argument");
  if (slot < 0 || slot >= ctx->cfg.max_batch) return fail(ctx, FOCUS_EINVAL, "slot %d outside 0..%d", slot, ctx->cfg.max_batch - 1);
  fk::SlotState s = ctx->slots();
  const int B = ctx->cfg.block_size;
  memset(st, 0, sizeof *st);
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(&st->prefix_len, s.prefix_len + slot, 4, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(&st->total_steps, s.total_steps + slot, 4, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(&st->token_sum, s.token_sum + slot, 8, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(&st->mask_bits, s.mask_bits + slot, 8, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(&st->processed_bits, s.processed_bits + slot, 8, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(&st->cached_bits, s.cached_bits + slot, 8, hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(st->tokens, s.tokens + (size_t)slot * B, 4 * B, hipMemcpyDeviceToHost));
  return FOCUS_OK;
}

int focus_set_state(focus_ctx *ctx, int32_t slot, const focus_seq_state *st) {
  if (!ctx || !st) return fail(ctx, FOCUS_EINVAL, "null argument");
  if (slot < 0 || slot >= ctx->cfg.max_batch) return fail(ctx, FOCUS_EINVAL, "slot %d outside 0..%d", slot, ctx->cfg.max_batch - 1);
  if (st->prefix_len < 0 || st->prefix_len > ctx->cfg.max_prefix_len) return fail(ctx, FOCUS_EINVAL, "prefix_len %d outside 0..%d", st->prefix_len, ctx->cfg.max_prefix_len);
  fk::SlotState s = ctx->slots();
  const int B = ctx->cfg.block_size;
  for (int p = 0; p < B; ++p)
    if (st->tokens[p] < 0 || st->tokens[p] >= ctx->cfg.vocab) return fail(ctx, FOCUS_EINVAL, "token id %d at position %d outside the vocabulary", st->tokens[p], p);
  HIP_TRY(ctx, hipDeviceSynchronize());
  if (st->prefix_len + B > ctx->max_total) ctx->max_total = st->prefix_len + B;
  HIP_TRY(ctx, hipMemcpy(s.prefix_len + slot, &st->prefix_len, 4, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.total_steps + slot, &st->total_steps, 4, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.token_sum + slot, &st->token_sum, 8, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.mask_bits + slot, &st->mask_bits, 8, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.processed_bits + slot, &st->processed_bits, 8, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.cached_bits + slot, &st->cached_bits, 8, hipMemcpyHostToDevice));
  HIP_TRY(ctx, hipMemcpy(s.tokens + (size_t)slot * B, st->tokens, 4 * B, hipMemcpyHostToDevice));
  return FOCUS_OK;
}

int focus_prefill_kv(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const int32_t *prefix_len,
                     const int32_t *page_table, int32_t table_stride, const int32_t *prompt_tokens, int32_t keep_stats) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (n_seq == 0) return FOCUS_OK;
  if (!prefix_len || !page_table) return fail(ctx, FOCUS_EINVAL, "null argument");
  const focus_config &g = ctx->cfg;
  const Plan &pl = ctx->plan;
  hipStream_t s = (hipStream_t)hip_stream;
  const int B = g.block_size;
  // host-side checks: slots distinct and in range, lengths in range, pages in range and enough of them
  std::vector<char> used(g.max_batch, 0);
  std::vector<int32_t> slots(n_seq), table((size_t)n_seq * pl.table_stride, 0), offs(n_seq), counts(n_seq);
  long long total_prompt = 0;
  int max_len = 0;
  for (int b = 0; b < n_seq; ++b) {
    int slot = seq_slot ? seq_slot[b] : b;
    if (slot < 0 || slot >= g.max_batch || used[slot]) return fail(ctx, FOCUS_EINVAL, "sequence %d: slot %d out of range or repeated", b, slot);
    used[slot] = 1;
    slots[b] = slot;
    int L = prefix_len[b];
    if (L < 0 || L > g.max_prefix_len) return fail(ctx, FOCUS_EINVAL, "sequence %d: prefix_len %d outside 0..%d", b, L, g.max_prefix_len);
    int need = (L + B + g.page_size - 1) / g.page_size;
    if (need > table_stride) return fail(ctx, FOCUS_EINVAL, "sequence %d: needs %d pages, table_stride is %d", b, need, table_stride);
    int have = 0;                              // leading valid entries; a negative entry ends the list
    for (int i = 0; i < table_stride && i < pl.table_stride; ++i) {
      int pg = page_table[(size_t)b * table_stride + i];
      if (pg < 0 && i >= need) break;
      if (pg < 0 || pg >= g.n_pages) return fail(ctx, FOCUS_EINVAL, "sequence %d: page %d outside 0..%d", b, pg, g.n_pages - 1);
      table[(size_t)b * pl.table_stride + i] = pg;
      have = i + 1;
    }
    counts[b] = have;
    offs[b] = (int32_t)total_prompt;
    total_prompt += L;
    max_len = L > max_len ? L : max_len;
  }
  if (prompt_tokens) {
    if (total_prompt > (long long)g.max_batch * g.max_prefix_len) return fail(ctx, FOCUS_EINVAL, "prompts longer than the plan");
    for (long long i = 0; i < total_prompt; ++i)
      if (prompt_tokens[i] < 0 || prompt_tokens[i] >= g.vocab) return fail(ctx, FOCUS_EINVAL, "prompt token %lld outside the vocabulary", i);
  }
  ctx->max_total = (max_len + B > ctx->max_total) ? max_len + B : ctx->max_total;
  fk::SlotState st = ctx->slots();
  // page tables: one row per slot
  for (int b = 0; b < n_seq; ++b)
    HIP_TRY(ctx, hipMemcpyAsync(st.page_table + (size_t)slots[b] * pl.table_stride, table.data() + (size_t)b * pl.table_stride,
                                (size_t)pl.table_stride * 4, hipMemcpyHostToDevice, s));
  for (int b = 0; b < n_seq; ++b)
    HIP_TRY(ctx, hipMemcpyAsync(st.page_count + slots[b], &counts[b], 4, hipMemcpyHostToDevice, s));
  int32_t *d_len = ctx->at<int32_t>(pl.off_prompt_len), *d_off = ctx->at<int32_t>(pl.off_prompt_off);
  int32_t *d_slots = ctx->at<int32_t>(pl.off_slot_list);
  HIP_TRY(ctx, hipMemcpyAsync(d_len, prefix_len, (size_t)n_seq * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(ctx, hipMemcpyAsync(d_off, offs.data(), (size_t)n_seq * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(ctx, hipMemcpyAsync(d_slots, slots.data(), (size_t)n_seq * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(ctx, hipStreamSynchronize(s));     // host vectors go out of scope / are reused below

  if (prompt_tokens && total_prompt > 0) {
    HIP_TRY(ctx, hipMemcpyAsync(ctx->at<int32_t>(pl.off_prompt), prompt_tokens, (size_t)total_prompt * 4, hipMemcpyHostToDevice, s));
    uint64_t *keep = ctx->at<uint64_t>(pl.off_keep);
    int32_t *cu = ctx->at<int32_t>(pl.off_cu), *row_map = ctx->at<int32_t>(pl.off_row_map), *total = ctx->at<int32_t>(pl.off_total);
    float *resid = ctx->at<float>(pl.off_resid_p);
    RowSet rs{{n_seq * B, total}, {row_map, d_slots, B}, n_seq, cu, B, nullptr};
    const int qkv_w = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
    for (int c0 = 0; c0 * B < max_len; ++c0) {
      fk::prefill_chunk_setup(s, n_seq, B, c0, d_slots, st, ctx->at<int32_t>(pl.off_prompt), d_off, d_len, keep);
      fk::scan_compact(s, n_seq, B, keep, cu, row_map, total);
      fk::embed(s, g.dtype, ctx->embed, g.hidden, rs.rows, rs.ri, st, g.mask_token_id, resid);
      for (int l = 0; l < g.n_layers; ++l) {
        layer_qkv(ctx, s, l, rs, resid);
        layer_rest(ctx, s, l, rs, resid, ctx->at<char>(pl.off_qkv), qkv_w, keep);
      }
    }
  }
  fk::reset_block_state(s, n_seq, B, d_slots, st, d_len, g.mask_token_id, keep_stats);
  HIP_TRY(ctx, hipStreamSynchronize(s));
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_step(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const int32_t *k_override,
               const uint64_t *keep_override, const focus_step_out *out) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  const focus_config &g = ctx->cfg;
  if (g.budget_mode == FOCUS_BUDGET_OVERRIDE && !k_override && !keep_override)
    return fail(ctx, FOCUS_EINVAL, "budget_mode OVERRIDE needs k_override");
  if (n_seq == 0) return FOCUS_OK;
  const Plan &pl = ctx->plan;
  hipStream_t s = (hipStream_t)hip_stream;
  ctx->last_stream = s;
  ctx->n_timed = 0;
  static const focus_step_out none{};
  const focus_step_out &o = out ? *out : none;
  RouteScope route_scope(ctx, o.route_experts, o.route_weights);
  const int B = g.block_size, e = g.evict_layer, T0 = n_seq * B;
  const int qkv_w = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim, q_w = g.n_q_heads * g.head_dim;
  fk::SlotState st = ctx->slots();
  float *resid = ctx->at<float>(pl.off_resid), *resid_p = ctx->at<float>(pl.off_resid_p);
  char *qkv = ctx->at<char>(pl.off_qkv), *q_p = ctx->at<char>(pl.off_q_p);
  float *partial = ctx->at<float>(pl.off_partial);
  const size_t partial_stride = (size_t)g.max_batch * g.n_q_heads * B;
  int32_t *cu = o.cu_seqlens ? o.cu_seqlens : ctx->at<int32_t>(pl.off_cu);
  int32_t *row_map = o.row_map ? o.row_map : ctx->at<int32_t>(pl.off_row_map);
  int32_t *total = ctx->at<int32_t>(pl.off_total);
  uint64_t *keep = o.keep_bits ? o.keep_bits : ctx->at<uint64_t>(pl.off_keep);
  uint64_t *vis = ctx->at<uint64_t>(pl.off_vis);
  float *conf = o.conf ? o.conf : ctx->at<float>(pl.off_conf);
  int32_t *amax = o.argmax ? o.argmax : ctx->at<int32_t>(pl.off_argmax);
  float *logits = o.logits ? o.logits : ctx->at<float>(pl.off_logits);

  // phase 1: whole block through layers 0 .. e-1, layer e up to its K/V fill, importance of layers e-1 and e
  // rows of the layers up to e: every block position, or, with the delayed intra-block cache, those not frozen
  const bool dc = g.intra_block_cache != 0;
  uint64_t *uncached = ctx->at<uint64_t>(pl.off_uncached);
  int32_t *cu_full = ctx->at<int32_t>(pl.off_cu_full), *total_full = ctx->at<int32_t>(pl.off_total_full);
  RowSet full{{T0, dc ? total_full : nullptr}, {ctx->at<int32_t>(pl.off_row_map_full), seq_slot, B}, n_seq, cu_full, B, ctx->at<int32_t>(pl.off_order)};
  { Timed t(ctx, s, FOCUS_KC_POINTWISE);
    if (dc) {
      fk::uncached_bits(s, n_seq, B, seq_slot, st, uncached);
      fk::scan_compact(s, n_seq, B, uncached, cu_full, ctx->at<int32_t>(pl.off_row_map_full), total_full);
    } else {
      fk::iota_rows(s, ctx->at<int32_t>(pl.off_row_map_full), cu_full, n_seq, B, total_full);
    }
    fk::length_order(s, n_seq, seq_slot, st, ctx->at<int32_t>(pl.off_order));
    fk::embed(s, g.dtype, ctx->embed, g.hidden, full.rows, full.ri, st, g.mask_token_id, resid); }
  for (int l = 0; l < e; ++l) {
    layer_qkv(ctx, s, l, full, resid);
    // Eq. 2 of layer e - 1 rides on that layer's attention pass over the whole block
    layer_rest(ctx, s, l, full, resid, qkv, qkv_w, nullptr, l == e - 1 && g.importance_mode == 0 ? partial : nullptr);
  }
  if (o.hidden_full)
    (void)hipMemcpyAsync(o.hidden_full, resid, (size_t)T0 * g.hidden * 4, hipMemcpyDeviceToDevice, s);
  layer_qkv(ctx, s, e, full, resid);

  // phase 2 + 3a: delta, budget, selection, packing, gather
  { Timed t(ctx, s, FOCUS_KC_IMPORTANCE);
    fk::importance(s, g.dtype, qkv, cu_full, n_seq, B, g.n_q_heads, g.n_kv_heads, g.head_dim, g.maxpool_k, seq_slot, st, ctx->kv_layer(e),
                   partial + partial_stride); }
  {
    Timed t(ctx, s, FOCUS_KC_SELECT);
    fk::SelectArgs a{};
    a.n_seq = n_seq; a.B = B; a.n_q_heads = g.n_q_heads;
    a.partial_prev = partial; a.partial_evict = partial + partial_stride; a.delta_in = nullptr;
    a.importance_mode = g.importance_mode; a.budget_mode = g.budget_mode; a.K_fixed = fixed_budget(g);
    a.constraints = g.constraints; a.alpha = g.alpha; a.k_override = k_override; a.keep_override = keep_override;
    a.seq_slot = seq_slot; a.st = st; a.update_state = 1; a.intra_block_cache = g.intra_block_cache;
    a.selection = g.selection; a.selection_seed = g.selection_seed;
    a.imp_prev_out = o.importance_prev; a.imp_out = o.importance;
    a.delta_out = o.delta_I ? o.delta_I : ctx->at<float>(pl.off_delta);
    a.K_out = o.K ? o.K : ctx->at<int32_t>(pl.off_K);
    a.keep_out = keep; a.n_keep_out = ctx->at<int32_t>(pl.off_n_keep); a.vis_out = vis;
    fk::select(s, a);
    fk::scan_compact(s, n_seq, B, keep, cu, row_map, total);
  }
  // the packed row count is read from device memory by every kernel; `cap` bounds it (grids, buffers), the caller's hint,
  // when there is one, shapes tiles, K splits and the attention's wavefront count
  const int cap = packed_cap(g, n_seq, keep_override != nullptr);
  const int rows_per_seq_cap = n_seq > 0 ? (cap + n_seq - 1) / n_seq : 0;
  const int rows_per_seq = ctx->hint_rows_per_seq > 0 ? std::min(ctx->hint_rows_per_seq, rows_per_seq_cap) : rows_per_seq_cap;
  RowSet packed{{cap, total, ctx->hint_rows}, {row_map, seq_slot, B}, n_seq, cu, rows_per_seq, ctx->at<int32_t>(pl.off_order)};
  { Timed t(ctx, s, FOCUS_KC_GATHER);
    fk::gather_rows(s, g.dtype, packed.rows, row_map, B, cu_full, dc ? uncached : nullptr, resid, resid_p, g.hidden, qkv, qkv_w, q_p, q_w); }

  // phase 3b: rest of layer e (all B fresh keys of layer e are visible), then the layers above on packed rows
  layer_rest(ctx, s, e, packed, resid_p, q_p, q_w, nullptr);
  for (int l = e + 1; l < g.n_layers; ++l) {
    layer_qkv(ctx, s, l, packed, resid_p);
    layer_rest(ctx, s, l, packed, resid_p, qkv, qkv_w, vis);
  }
  if (o.hidden_packed)
    (void)hipMemcpyAsync(o.hidden_packed, resid_p, (size_t)cap * g.hidden * 4, hipMemcpyDeviceToDevice, s);

  // decode and verify
  void *normed = ctx->at<char>(pl.off_normed);
  { Timed t(ctx, s, FOCUS_KC_POINTWISE); fk::rmsnorm(s, g.dtype, resid_p, ctx->final_norm, normed, g.hidden, g.rms_eps, packed.rows); }
  // without a logits output the projection reduces every row to (max, sum exp, arg-max) triples per column range in its epilogue
  // and the logits never reach memory; the triples take the place of the logits in the workspace
  int conf_slots = 0;
  bool fused_conf = false;
  if (!o.logits) {
    Timed t(ctx, s, FOCUS_KC_GEMM);
    fused_conf = fk::gemm_conf_partials(s, g.dtype, normed, ctx->lm_head, g.vocab, g.hidden, packed.rows, ctx->at<float>(pl.off_logits),
                                        (size_t)ctx->plan.max_rows * g.vocab * 4, &conf_slots);
  }
  if (!fused_conf) { Timed t(ctx, s, FOCUS_KC_GEMM); fk::gemm(s, g.dtype, normed, ctx->lm_head, g.vocab, g.hidden, packed.rows, fk::EPI_STORE_F32, logits, g.vocab, fk::Warm(), ctx->scratch()); }
  {
    Timed t(ctx, s, FOCUS_KC_DECODE);
    if (fused_conf) fk::confidence_from_partials(s, ctx->at<float>(pl.off_logits), conf_slots, packed.rows, conf, amax);
    else fk::confidence(s, logits, g.vocab, packed.rows, conf, amax, ctx->scratch());
    fk::CommitArgs ca{n_seq, B, seq_slot, st, keep, cu, conf, amax, g.conf_threshold, g.mask_token_id, g.intra_block_cache, o.tokens, o.mask_bits, o.n_decoded};
    fk::commit(s, ca);
  }
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_select_compact(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const float *delta_I,
                         const int32_t *k_override, const focus_step_out *out) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (!delta_I || !out || !out->K || !out->keep_bits || !out->cu_seqlens || !out->row_map)
    return fail(ctx, FOCUS_EINVAL, "delta_I and out->K, keep_bits, cu_seqlens, row_map are required");
  const focus_config &g = ctx->cfg;
  if (g.budget_mode == FOCUS_BUDGET_OVERRIDE && !k_override) return fail(ctx, FOCUS_EINVAL, "budget_mode OVERRIDE needs k_override");
  if (n_seq == 0) return FOCUS_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  fk::SelectArgs a{};
  a.n_seq = n_seq; a.B = g.block_size; a.n_q_heads = g.n_q_heads;
  a.delta_in = delta_I;
  a.importance_mode = g.importance_mode; a.budget_mode = g.budget_mode; a.K_fixed = fixed_budget(g);
  a.constraints = g.constraints; a.alpha = g.alpha; a.k_override = k_override; a.keep_override = nullptr;
  a.seq_slot = seq_slot; a.st = ctx->slots(); a.update_state = 0; a.intra_block_cache = g.intra_block_cache;
  a.selection = g.selection; a.selection_seed = g.selection_seed;
  a.delta_out = nullptr; a.K_out = out->K; a.keep_out = out->keep_bits;
  a.n_keep_out = ctx->at<int32_t>(ctx->plan.off_n_keep); a.vis_out = nullptr;
  fk::select(s, a);
  fk::scan_compact(s, n_seq, g.block_size, out->keep_bits, out->cu_seqlens, out->row_map, ctx->at<int32_t>(ctx->plan.off_total));
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_select_compact_noalloc(const focus_config *cfg, void *hip_stream, int32_t n_seq, const float *delta_I,
                                 const uint64_t *mask_bits, const uint64_t *cached_bits, const int64_t *token_sum,
                                 const int32_t *total_steps, const int32_t *k_override, const focus_step_out *out) {
  if (!cfg || !delta_I || !mask_bits || !out || !out->K || !out->keep_bits || !out->cu_seqlens || !out->row_map)
    return fail(nullptr, FOCUS_EINVAL, "cfg, delta_I, mask_bits and out->K, keep_bits, cu_seqlens, row_map are required");
  const focus_config &g = *cfg;
  if (g.block_size < 1 || g.block_size > FOCUS_MAX_BLOCK) return fail(nullptr, FOCUS_EINVAL, "block_size must be in 1..64");
  if (g.budget_mode < 0 || g.budget_mode > 3 || (g.constraints & ~3) || (g.intra_block_cache & ~1) ||
      g.selection < FOCUS_SELECT_TOP || g.selection > FOCUS_SELECT_BOTTOM)
    return fail(nullptr, FOCUS_EINVAL, "unknown budget_mode, constraint bits, intra_block_cache or selection");
  if (n_seq < 0 || n_seq > FOCUS_NOALLOC_MAX_SEQ)
    return fail(nullptr, FOCUS_EINVAL, "n_seq %d outside 0..FOCUS_NOALLOC_MAX_SEQ (%d)", n_seq, FOCUS_NOALLOC_MAX_SEQ);
  if (n_seq == 0) return FOCUS_OK;
  if (g.budget_mode == FOCUS_BUDGET_OVERRIDE && !k_override) return fail(nullptr, FOCUS_EINVAL, "budget_mode OVERRIDE needs k_override");
  if (g.budget_mode == FOCUS_BUDGET_DYNAMIC && (!token_sum || !total_steps)) return fail(nullptr, FOCUS_EINVAL, "budget_mode DYNAMIC needs token_sum and total_steps");
  if (g.selection == FOCUS_SELECT_RANDOM && !total_steps) return fail(nullptr, FOCUS_EINVAL, "selection RANDOM needs total_steps");
  if (g.intra_block_cache && !cached_bits) return fail(nullptr, FOCUS_EINVAL, "intra_block_cache needs cached_bits");
  int32_t *sc = scratch_of_current_device(nullptr);
  if (!sc) return FOCUS_EHIP;
  hipStream_t s = (hipStream_t)hip_stream;
  // the caller's arrays stand in for the slot state, batch entry b = slot b; nothing of it is written
  fk::SlotState st{};
  st.mask_bits = const_cast<uint64_t *>(mask_bits);
  st.cached_bits = const_cast<uint64_t *>(cached_bits);
  st.token_sum = const_cast<int64_t *>(token_sum);
  st.total_steps = const_cast<int32_t *>(total_steps);
  st.max_batch = n_seq;
  fk::SelectArgs a{};
  a.n_seq = n_seq; a.B = g.block_size; a.n_q_heads = g.n_q_heads;
  a.delta_in = delta_I;
  a.importance_mode = g.importance_mode; a.budget_mode = g.budget_mode; a.K_fixed = fixed_budget(g);
  a.constraints = g.constraints; a.alpha = g.alpha; a.k_override = k_override; a.keep_override = nullptr;
  a.seq_slot = nullptr; a.st = st; a.update_state = 0; a.intra_block_cache = g.intra_block_cache;
  a.selection = g.selection; a.selection_seed = g.selection_seed;
  a.delta_out = nullptr; a.K_out = out->K; a.keep_out = out->keep_bits;
  a.n_keep_out = sc; a.vis_out = nullptr;                     // scratch: [0, n_seq) retained counts, [MAX_SEQ] packed total
  fk::select(s, a);
  fk::scan_compact(s, n_seq, g.block_size, out->keep_bits, out->cu_seqlens, out->row_map, sc + FOCUS_NOALLOC_MAX_SEQ);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, FOCUS_EHIP, "focus_select_compact_noalloc: %s", hipGetErrorString(e));
  return FOCUS_OK;
}

int focus_run_layers(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const uint64_t *keep_bits,
                     const uint64_t *vis_bits, int32_t layer_begin, int32_t layer_end, float *hidden) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (!keep_bits || !vis_bits || !hidden) return fail(ctx, FOCUS_EINVAL, "null argument");
  const focus_config &g = ctx->cfg;
  if (layer_begin <= g.evict_layer || layer_end > g.n_layers || layer_begin > layer_end)
    return fail(ctx, FOCUS_EINVAL, "layers [%d, %d) must lie in (evict_layer, n_layers]", layer_begin, layer_end);
  if (n_seq == 0) return FOCUS_OK;
  const Plan &pl = ctx->plan;
  hipStream_t s = (hipStream_t)hip_stream;
  const int B = g.block_size, cap = n_seq * B;
  const int qkv_w = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
  int32_t *cu = ctx->at<int32_t>(pl.off_cu), *row_map = ctx->at<int32_t>(pl.off_row_map), *total = ctx->at<int32_t>(pl.off_total);
  float *resid_p = ctx->at<float>(pl.off_resid_p);
  RouteScope route_scope(ctx, nullptr, nullptr);
  fk::scan_compact(s, n_seq, B, keep_bits, cu, row_map, total);
  HIP_TRY(ctx, hipMemcpyAsync(resid_p, hidden, (size_t)cap * g.hidden * 4, hipMemcpyDeviceToDevice, s));
  RowSet packed{{cap, total}, {row_map, seq_slot, B}, n_seq, cu, B, nullptr};
  for (int l = layer_begin; l < layer_end; ++l) {
    layer_qkv(ctx, s, l, packed, resid_p);
    layer_rest(ctx, s, l, packed, resid_p, ctx->at<char>(pl.off_qkv), qkv_w, vis_bits);
  }
  HIP_TRY(ctx, hipMemcpyAsync(hidden, resid_p, (size_t)cap * g.hidden * 4, hipMemcpyDeviceToDevice, s));
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_finalize_blocks(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, int32_t *finalized) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (n_seq == 0) return FOCUS_OK;
  const focus_config &g = ctx->cfg;
  const Plan &pl = ctx->plan;
  hipStream_t s = (hipStream_t)hip_stream;
  const int B = g.block_size;
  const int qkv_w = (g.n_q_heads + 2 * g.n_kv_heads) * g.head_dim;
  fk::SlotState st = ctx->slots();
  uint64_t *keep = ctx->at<uint64_t>(pl.off_keep);
  int32_t *cu = ctx->at<int32_t>(pl.off_cu), *row_map = ctx->at<int32_t>(pl.off_row_map), *total = ctx->at<int32_t>(pl.off_total);
  float *resid = ctx->at<float>(pl.off_resid_p);
  // the prefixes may grow by one block: keep the host-side bound the attention launch is sized with
  ctx->max_total = std::min(ctx->max_total + B, g.max_prefix_len + B);
  int32_t *done = ctx->at<int32_t>(pl.off_finalized);
  fk::finalize_pick(s, n_seq, B, g.page_size, seq_slot, st, keep, done);
  if (finalized) HIP_TRY(ctx, hipMemcpyAsync(finalized, done, (size_t)n_seq * 4, hipMemcpyDeviceToDevice, s));
  fk::scan_compact(s, n_seq, B, keep, cu, row_map, total);
  RowSet rs{{n_seq * B, total}, {row_map, seq_slot, B}, n_seq, cu, B, nullptr};
  fk::embed(s, g.dtype, ctx->embed, g.hidden, rs.rows, rs.ri, st, g.mask_token_id, resid);
  for (int l = 0; l < g.n_layers; ++l) {
    layer_qkv(ctx, s, l, rs, resid);
    layer_rest(ctx, s, l, rs, resid, ctx->at<char>(pl.off_qkv), qkv_w, nullptr);   // a finished block sees all of itself
  }
  fk::finalize_advance(s, n_seq, B, seq_slot, st, done, g.mask_token_id);
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_run_steps(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, int32_t n_steps, int32_t finalize,
                    int64_t *decoded, const focus_step_out *out) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (n_steps < 0) return fail(ctx, FOCUS_EINVAL, "n_steps %d is negative", n_steps);
  if (ctx->cfg.budget_mode == FOCUS_BUDGET_OVERRIDE) return fail(ctx, FOCUS_EINVAL, "budget_mode OVERRIDE takes its budgets per step: use focus_step");
  if (n_seq == 0) return FOCUS_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  focus_step_out inner{};
  inner.n_decoded = ctx->at<int32_t>(ctx->plan.off_n_dec);
  for (int i = 0; i < n_steps; ++i) {
    focus_step_out o = (i == n_steps - 1 && out) ? *out : inner;
    if (!o.n_decoded) o.n_decoded = inner.n_decoded;
    if (int rc = focus_step(ctx, hip_stream, n_seq, seq_slot, nullptr, nullptr, &o)) return rc;
    if (decoded) fk::add_counts(s, n_seq, o.n_decoded, decoded);
    if (finalize)
      if (int rc = focus_finalize_blocks(ctx, hip_stream, n_seq, seq_slot, nullptr)) return rc;
  }
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

int focus_set_row_hint(focus_ctx *ctx, int32_t packed_rows, int32_t rows_per_seq) {
  if (!ctx) return fail(nullptr, FOCUS_EINVAL, "null context");
  if (packed_rows < 0 || rows_per_seq < 0) return fail(ctx, FOCUS_EINVAL, "row hints must be >= 0");
  ctx->hint_rows = packed_rows;
  ctx->hint_rows_per_seq = rows_per_seq;
  return FOCUS_OK;
}

int focus_set_route_override(focus_ctx *ctx, const int32_t *experts) {
  if (!ctx) return fail(nullptr, FOCUS_EINVAL, "null context");
  if (experts && ctx->cfg.n_experts == 0) return fail(ctx, FOCUS_EINVAL, "the model has no mixture-of-experts layers");
  ctx->route_override = experts;
  return FOCUS_OK;
}

int focus_commit(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const uint64_t *keep_bits,
                 const int32_t *cu_seqlens, const float *conf, const int32_t *argmax, const focus_step_out *out) {
  if (int rc = check_batch(ctx, n_seq)) return rc;
  if (!keep_bits || !cu_seqlens || !conf || !argmax) return fail(ctx, FOCUS_EINVAL, "null argument");
  if (n_seq == 0) return FOCUS_OK;
  const focus_config &g = ctx->cfg;
  static const focus_step_out none{};
  const focus_step_out &o = out ? *out : none;
  fk::CommitArgs ca{n_seq, g.block_size, seq_slot, ctx->slots(), keep_bits, cu_seqlens, conf, argmax, g.conf_threshold,
                    g.mask_token_id, g.intra_block_cache, o.tokens, o.mask_bits, o.n_decoded};
  fk::commit((hipStream_t)hip_stream, ca);
  HIP_TRY(ctx, hipGetLastError());
  return FOCUS_OK;
}

}  // extern "C"
