/*
 * focus.h - C ABI of the MI355X (gfx950) FOCUS decode-step library.
 *
 * One call of focus_step() is one inference step of FOCUS (arXiv 2601.23278, Algorithm 1) for a batch
 * of block-diffusion sequences that share one model: the whole block of B tokens runs through the layers
 * up to the eviction layer e, the token importance (Eq. 2) of layers e-1 and e gives the importance
 * delta (Eq. 3), a per-sequence budget K (Eq. 4-5, or a fixed budget) and the top-K / structural
 * constraints of Sec. 4.2 pick the retained positions, the retained rows of all sequences are packed
 * into one ragged batch, the rest of layer e and all later layers run on the packed rows only, and the
 * confidence-based decoding commits tokens and updates the running statistics of App. E.3.1.
 *
 * Conventions
 *   - Every function returns FOCUS_OK (0) or a negative FOCUS_E* code; focus_last_error() gives the text.
 *     Nothing throws, nothing aborts.
 *   - "device" pointers are HIP device memory of the current device, "host" pointers ordinary memory.
 *   - Weights, the K/V pool and the workspace are BORROWED: the caller allocates them, keeps them alive
 *     until focus_free(), and must not touch the workspace in between.
 *   - focus_step / focus_select_compact / focus_commit only enqueue work on the given stream: no allocation,
 *     no host synchronisation; outputs are valid once the caller has synchronised the stream.
 *   - HIP graphs: a step records no memset node (device-to-device copies only for the hidden-state outputs, when they are
 *     asked for), allocates nothing and never synchronises with the host, and
 *     every kernel reads the packed row count from device memory, so one captured step serves every later step whatever
 *     the number of retained rows.  The K/V split geometry of the attention launches is fixed at capture from the
 *     longest prefix installed then; the kernels read the real lengths on the device and the last split of a sequence
 *     takes whatever lies beyond, so a replay stays correct after prefixes have grown (focus_finalize_blocks), up to
 *     max_prefix_len, with the split sizes of the capture.  The first launch of some kernels in a process sets their dynamic-LDS attribute, which
 *     is not a stream operation: run one step eagerly before capturing.
 *   - A context is not thread-safe.  The same calls on the same inputs give bitwise identical results
 *     (no floating-point atomics anywhere).
 *
 * Layouts
 *   - Matrices are row-major [out_features, in_features]; element type per focus_config.dtype.
 *   - w_qkv rows: H_q*D query rows, then H_kv*D key rows, then H_kv*D value rows.
 *     w_gate_up rows: F gate rows, then F up rows.
 *   - K/V pool: [n_layers][n_pages] pages, element type per dtype.  A page holds K as [H_kv][page_size][D]
 *     (after the rotary embedding) followed by V transposed, [H_kv][D][page_size], so that both operands of
 *     the attention contractions are contiguous along the contracted index.  A sequence's token t lives in
 *     page page_table[t / page_size] at row (K) / column (V) t % page_size; the current block occupies tokens
 *     prefix_len .. prefix_len + B - 1.
 *   - Bit sets over block positions are uint64_t, bit p = position p (B <= 64).
 *   - Packed rows: sequences in batch order, positions ascending; row_map[r] = b * B + p.
 */
#ifndef FOCUS_H
#define FOCUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FOCUS_MAX_BLOCK 64

enum { FOCUS_OK = 0, FOCUS_EINVAL = -1, FOCUS_ENOMEM = -2, FOCUS_EHIP = -3 };
enum { FOCUS_F32 = 0, FOCUS_BF16 = 1 };
enum { FOCUS_BUDGET_TOPK = 0, FOCUS_BUDGET_RATIO = 1, FOCUS_BUDGET_DYNAMIC = 2, FOCUS_BUDGET_OVERRIDE = 3 };
enum { FOCUS_KEEP_AR_CONTEXT = 1, FOCUS_KEEP_PLACEHOLDERS = 2 };
enum { FOCUS_SELECT_TOP = 0, FOCUS_SELECT_RANDOM = 1, FOCUS_SELECT_BOTTOM = 2 };

typedef struct focus_ctx focus_ctx;

/* Plain data, copied by focus_init. */
typedef struct focus_config {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t dtype;            /* FOCUS_F32 or FOCUS_BF16: weights, activations and K/V; the residual stream,
                               softmax, importance and logits are fp32 in both */
  float   rms_eps;
  float   rope_base;        /* rotate-half pairing (i, i + D/2), angle pos * base^(-2i/D) */
  int32_t block_size;       /* B, 1..64 */
  int32_t mask_token_id;
  int32_t max_batch;        /* number of sequence slots */
  int32_t max_prefix_len;   /* longest prefix any slot will hold */
  int32_t page_size;        /* tokens per K/V page */
  int32_t n_pages;          /* pages per layer in the K/V pool */
  int32_t evict_layer;      /* e (Alg. 1 uses 1); 1 <= e < n_layers when importance_mode is 0 */
  int32_t importance_mode;  /* 0: delta I(e) - I(e-1) (Eq. 3); 1: raw I(e) */
  int32_t maxpool_k;        /* MaxPool1D window of Eq. 2: 3 (App. F.1) or 1 (off) */
  int32_t budget_mode;      /* FOCUS_BUDGET_* */
  int32_t topk;             /* FOCUS_BUDGET_TOPK */
  float   keep_ratio;       /* FOCUS_BUDGET_RATIO: K = ceil(keep_ratio * B) */
  float   alpha;            /* FOCUS_BUDGET_DYNAMIC: expansion factor of Eq. 4 */
  int32_t constraints;      /* FOCUS_KEEP_* bits (Sec. 4.2) */
  float   conf_threshold;   /* commit when confidence >= threshold */
  int32_t intra_block_cache;/* 1: delayed intra-block K/V cache with the neighbour-aware stability criterion (Sec. 4.3,
                               App. E.3.1): a position whose token and right neighbour were decoded before a step it
                               took part in keeps that step's K/V in every layer from then on and leaves the rows of
                               all later steps of the block; decoded positions not yet frozen are always retained */
  int32_t selection;        /* FOCUS_SELECT_*: which min(K, |M|) masked positions the budget picks.  TOP is the method
                               (largest delta).  BOTTOM (smallest delta) and RANDOM are the controls of the selection
                               validation (Sec. 5.2); ties go to the lower position, the structural constraints apply
                               to the pick unchanged */
  uint32_t selection_seed;  /* RANDOM: position j of slot s is ranked by output number c + 1 of the SplitMix64 generator
                               started at selection_seed, c = (s * 2^32 + total_steps of the slot before the step) * 64 + j */
  /* Mixture-of-experts feed-forward (the second model of Sec. 5.1 is an MoE; the paper does not spell out its layer, this is
     the common token-choice one).  In layers first_moe_layer .. n_layers - 1 a row's feed-forward is
       route_scale * sum_j g_j * Expert_{e_j}(u)  +  Shared(u)
     where u is the normalised row, e_1 .. e_k are the k experts with the largest router logit w_router u (descending; ties:
     lower expert), g = softmax over all E logits restricted to the chosen ones and renormalised to sum to one, and every
     expert (the shared one too) is a SwiGLU feed-forward.  Layers below first_moe_layer keep the dense feed-forward. */
  int32_t n_experts;        /* E, 0..512; 0 = dense model, the members below are ignored */
  int32_t experts_per_token;/* k, 1..min(E, 32) */
  int32_t expert_ffn;       /* F_e, inner width of a routed expert */
  int32_t shared_ffn;       /* F_s, inner width of the shared expert; 0 = none */
  int32_t first_moe_layer;  /* 0..n_layers */
  float   route_scale;
} focus_config;

/* Device pointers.  The per-layer members are HOST arrays of n_layers device pointers. */
typedef struct focus_weights {
  const void *embed;        /* [vocab, hidden] */
  const void *lm_head;      /* [vocab, hidden] */
  const void *final_norm;   /* [hidden] */
  const void *const *attn_norm;   /* [hidden] */
  const void *const *w_qkv;       /* [(H_q + 2 H_kv) D, hidden] */
  const void *const *w_o;         /* [hidden, H_q D] */
  const void *const *mlp_norm;    /* [hidden] */
  const void *const *w_gate_up;   /* [2 F, hidden] */
  const void *const *w_down;      /* [hidden, F] */
  /* mixture-of-experts layers (n_experts > 0; entries of dense layers are ignored, and so are w_gate_up / w_down entries of
     mixture-of-experts layers) */
  const void *const *w_router;          /* [E, hidden] */
  const void *const *w_expert_gate_up;  /* [E, 2 F_e, hidden]: per expert F_e gate rows, then F_e up rows */
  const void *const *w_expert_down;     /* [E, hidden, F_e] */
  const void *const *w_shared_gate_up;  /* [2 F_s, hidden] (shared_ffn > 0) */
  const void *const *w_shared_down;     /* [hidden, F_s] */
} focus_weights;

/* Optional outputs of a step; every member is a caller-allocated device pointer or NULL.  n = n_seq,
 * T' = cu_seqlens[n] <= n * B. */
typedef struct focus_step_out {
  int32_t  *tokens;         /* [n, B]   block token ids after the commit (mask id where still masked) */
  uint64_t *mask_bits;      /* [n]      still-masked positions after the commit */
  int32_t  *n_decoded;      /* [n]      tokens unmasked by this step */
  float    *importance_prev;/* [n, B]   Eq. 2 at layer e-1 (importance_mode 0) */
  float    *importance;     /* [n, B]   Eq. 2 at layer e */
  float    *delta_I;        /* [n, B]   Eq. 3 */
  int32_t  *K;              /* [n]      budget */
  uint64_t *keep_bits;      /* [n]      retained set S */
  int32_t  *cu_seqlens;     /* [n + 1]  exclusive prefix sum of |S| */
  int32_t  *row_map;        /* [n * B]  first T' entries valid */
  float    *conf;           /* [n * B]  first T' entries valid: probability of the arg-max token */
  int32_t  *argmax;         /* [n * B]  first T' entries valid */
  float    *hidden_full;    /* [n * B, hidden]  residual stream entering layer e: row b * B + p, or, with the
                               intra-block cache, the rows of the positions that are not frozen, packed in batch order */
  float    *hidden_packed;  /* [n * B, hidden]  first T' rows valid: residual stream after the last layer */
  float    *logits;         /* [n * B, vocab]   first T' rows valid.  NULL (the normal case): a bf16 model with enough rows for
                               the tiled projection never writes the logits; the projection's epilogue reduces each tile to
                               (max, sum exp, arg-max) and conf / argmax come from those */
  int32_t  *route_experts;  /* [n_layers, max_batch * B, k]  mixture-of-experts layers: the experts row b * B + p used, in the
                               order of their weights; written for the rows that ran in the layer, other entries untouched */
  float    *route_weights;  /* [n_layers, max_batch * B, k]  their mixing weights (route_scale included) */
} focus_step_out;

/* Host copy of one slot's block state (App. E.3.1 plus the block's tokens). */
typedef struct focus_seq_state {
  int32_t  prefix_len;
  int32_t  total_steps;
  int64_t  token_sum;
  uint64_t mask_bits;
  uint64_t processed_bits;  /* positions that have K/V in the layers above e */
  uint64_t cached_bits;     /* positions whose K/V is frozen in every layer (intra_block_cache) */
  int32_t  tokens[FOCUS_MAX_BLOCK];
} focus_seq_state;

/* Infrastructure (no passage of the paper: the paper's engine keeps this state in its serving framework, App. E.3.1 only lists
 * what the state is).  Sizes the caller must allocate; both need only the shape members of cfg.  The workspace holds the
 * per-slot state of App. E.3.1 (masked / processed / frozen sets, token_sum, total_steps, block tokens, prefix lengths, page
 * tables), the rotary table and every activation buffer of a step. */
int focus_workspace_bytes(const focus_config *cfg, size_t *bytes);
int focus_kv_pool_bytes(const focus_config *cfg, size_t *bytes);

/* Infrastructure.  Creates a context over borrowed device memory.  Builds the rotary table and zeroes the slot state
 * (synchronous).  EINVAL: bad shape / unsupported switch / NULL; ENOMEM: a buffer is too small. */
int focus_init(const focus_config *cfg, const focus_weights *weights, void *kv_pool, size_t kv_pool_bytes,
               void *workspace, size_t workspace_bytes, focus_ctx **out);

/* Installs n_seq sequences and resets their block state (all B positions masked, nothing processed; the
 * running statistics are reset too unless keep_stats != 0, App. E.3.1 "state persistence").
 *   seq_slot      host [n_seq] slot of each sequence, or NULL for 0..n_seq-1
 *   prefix_len    host [n_seq]
 *   page_table    host [n_seq, table_stride]: physical pages covering at least prefix_len + B tokens; further
 *                 entries up to the first negative one are pages for the blocks generated later
 *   prompt_tokens host, the prompts concatenated in order (sum of prefix_len ids), or NULL.
 *                 Not NULL: computes the exact prefix K/V of every layer (the prompt is cut into blocks of
 *                 B tokens, each attends to all earlier blocks and bidirectionally to itself; Sec. 2).
 *                 NULL: the pool already holds the prefix K/V (e.g. seeded synthetic pages).
 * Synchronises the stream before returning. */
int focus_prefill_kv(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot,
                     const int32_t *prefix_len, const int32_t *page_table, int32_t table_stride,
                     const int32_t *prompt_tokens, int32_t keep_stats);

/* One FOCUS step (Algorithm 1) for sequences seq_slot[0..n_seq) in that batch order.
 *   seq_slot      device [n_seq] or NULL for slots 0..n_seq-1
 *   k_override    device [n_seq] budgets for FOCUS_BUDGET_OVERRIDE, else NULL
 *   keep_override device [n_seq] retained sets to use instead of budget + selection, or NULL
 *   out           host struct of device pointers, or NULL */
int focus_step(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot,
               const int32_t *k_override, const uint64_t *keep_override, const focus_step_out *out);

/* Stage entry: budget (Eq. 4-5), selection (Alg. 1 phase 3) and packing on caller-given scores, using the
 * slots' current mask bits and statistics.  Writes out->K, keep_bits, cu_seqlens, row_map.  Does not change
 * the slot state.
 *   delta_I       device [n_seq, B] fp32 */
int focus_select_compact(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot,
                         const float *delta_I, const int32_t *k_override, const focus_step_out *out);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc) and that hold no context: the same budget + selection + packing as focus_select_compact, on caller-given
 * scores AND caller-given block state, enqueued on the stream.  It calls no hipMalloc / hipFree and needs no workspace: its
 * scratch (per-sequence retained counts and the packed total) is a fixed array inside the library, one copy per GPU held
 * until the process ends (FOCUS_NOALLOC_MAX_SEQ + 64 ints = 64.25 KB).  Every call on a GPU uses that one array: calls
 * that overlap on one GPU (two streams, two threads) race; calls on one stream are ordered and fine.  The array keeps
 * the last call's contents; nothing in it has to start at zero.
 *   cfg           only block_size, budget_mode, topk, keep_ratio, alpha, constraints, intra_block_cache, selection and
 *                 selection_seed are read
 *   n_seq         0..FOCUS_NOALLOC_MAX_SEQ, EINVAL beyond
 *   delta_I       device [n_seq, B] fp32
 *   mask_bits     device [n_seq] still-masked positions of batch entry b
 *   cached_bits   device [n_seq] frozen positions (intra_block_cache), else may be NULL
 *   token_sum, total_steps  device [n_seq] running statistics (FOCUS_BUDGET_DYNAMIC; total_steps also for
 *                 FOCUS_SELECT_RANDOM, whose keys take the batch index as the slot), else may be NULL
 *   k_override    device [n_seq] for FOCUS_BUDGET_OVERRIDE, else NULL
 *   out           K, keep_bits, cu_seqlens, row_map are required and written; nothing else is touched
 * Errors are reported through focus_last_error(NULL). */
#define FOCUS_NOALLOC_MAX_SEQ 16384
int focus_select_compact_noalloc(const focus_config *cfg, void *hip_stream, int32_t n_seq, const float *delta_I,
                                 const uint64_t *mask_bits, const uint64_t *cached_bits, const int64_t *token_sum,
                                 const int32_t *total_steps, const int32_t *k_override, const focus_step_out *out);

/* Stage entry: runs layers [layer_begin, layer_end) of the reduced forward pass (Alg. 1 phase 3, "Forward(H_reduced,
 * C, Layers = 1_suffix ... L)") on caller-given hidden states, so that deep layers can be compared with a
 * reference fed the same input.  layer_begin must be above the eviction layer.  Rows are the positions in
 * keep_bits, packed as focus_step packs them; their K/V in those layers is rewritten; in-block keys visible to the
 * attention are vis_bits.  The slot state is not changed.
 *   keep_bits, vis_bits  device [n_seq]
 *   hidden               device [T', hidden] fp32, residual stream entering layer_begin; overwritten with the
 *                        residual stream leaving layer_end - 1 */
int focus_run_layers(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, const uint64_t *keep_bits,
                     const uint64_t *vis_bits, int32_t layer_begin, int32_t layer_end, float *hidden);

/* Multi-block generation (the loop around Alg. 1; App. E.3.1 "state persistence and reset").  Every listed
 * sequence whose block has no masked position left gets one last forward of the whole block with its committed
 * tokens through all layers, so that the K/V it leaves behind is the exact K/V of those tokens; then the block
 * becomes prefix (prefix_len += B) and a new all-masked block starts; the running statistics persist.  Sequences
 * that still have masked positions are untouched, and so are sequences without room: the new prefix must not exceed
 * max_prefix_len and the page list given to focus_prefill_kv must cover prefix_len + 2 B tokens.
 *   finalized     device [n_seq] out: 1 where the block was finalized, else 0; or NULL
 * Enqueues only (no host synchronisation). */
int focus_finalize_blocks(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, int32_t *finalized);

/* Several steps per host call with the state updated on the device after every step (the "in-loop state update" that
 * App. E.3.4 proposes so that a multi-loop engine can run the method): n_steps times focus_step and, when finalize != 0,
 * focus_finalize_blocks, enqueued back to back.  Every step sees the statistics, the masked / processed / frozen sets and
 * the prefix lengths that the step before it left, exactly as n_steps separate calls would; nothing returns to the host.
 * Not for FOCUS_BUDGET_OVERRIDE (its budgets are per step).
 *   decoded       device [n_seq] int64, += tokens each sequence decoded in these steps; or NULL
 *   out           outputs of the LAST step, or NULL */
int focus_run_steps(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot, int32_t n_steps, int32_t finalize,
                    int64_t *decoded, const focus_step_out *out);

/* Launch-shape hint for steps whose packed row count only the device knows (Eq. 4-5 dynamic budget, the structural constraints
 * of Sec. 4.2, the intra-block cache of Sec. 4.3, per-sequence budgets): without it every launch of the reduced forward pass is
 * shaped for the worst case n_seq * B.  packed_rows = rows the next steps are expected to retain in total (e.g. the last step's
 * cu_seqlens[n_seq]), rows_per_seq = the most a single sequence is expected to retain; 0 = no hint.  Only tile shapes, K splits
 * and wavefront counts follow the hint: results do not depend on it in any way other than the rounding order of K-split
 * projections, and a step that retains more rows than hinted is still computed in full (more workgroups per projection, several
 * passes of the attention over that sequence's K/V).  Applies to every later focus_step / focus_run_steps of the context. */
int focus_set_row_hint(focus_ctx *ctx, int32_t packed_rows, int32_t rows_per_seq);

/* Teacher forcing for mixture-of-experts layers: from now on focus_step and focus_run_layers use, for the row of block
 * position p of batch entry b in layer l, the experts experts[(l * max_batch * B + b * B + p) * k + j], j < k (distinct,
 * in 0..E-1; out-of-range values are clamped), with weights computed from the router logits as for the router's own pick.
 * Prefill and block finalisation always route by themselves.  NULL switches it off.
 *   experts       device [n_layers, max_batch * B, k], borrowed until replaced */
int focus_set_route_override(focus_ctx *ctx, const int32_t *experts);

/* Stage entry: confidence-based commit (Alg. 1 Decode_and_Verify, App. E.3.1 statistics) on caller-given
 * confidences.  Updates the slot state and writes out->tokens, mask_bits, n_decoded.
 *   keep_bits     device [n_seq]; cu_seqlens device [n_seq + 1]; conf, argmax device [cu_seqlens[n_seq]] */
int focus_commit(focus_ctx *ctx, void *hip_stream, int32_t n_seq, const int32_t *seq_slot,
                 const uint64_t *keep_bits, const int32_t *cu_seqlens, const float *conf,
                 const int32_t *argmax, const focus_step_out *out);

/* Infrastructure for tests and schedulers: one slot's block state (the fields App. E.3.1 names, plus the block's tokens) read
 * from / written to the device (synchronous copies; not for use between the steps of a timed loop). */
int focus_get_state(focus_ctx *ctx, int32_t slot, focus_seq_state *state);
int focus_set_state(focus_ctx *ctx, int32_t slot, const focus_seq_state *state);

/* Infrastructure for measurement (no passage).  Per-kernel-class device time of the last focus_step.  With timing enabled every kernel launch of a step
 * is bracketed by a pair of HIP events on the step's stream (this adds small gaps between kernels, so time
 * whole steps with timing off).  focus_get_kernel_time synchronises the stream and returns the summed
 * duration and the number of launches of one class. */
enum { FOCUS_KC_GEMM = 0,      /* dense projections: QKV, O, gate/up, down, lm_head */
       FOCUS_KC_ATTENTION = 1, /* block attention over the paged K/V */
       FOCUS_KC_IMPORTANCE = 2,/* token importance of layers e-1 and e (Eq. 2) */
       FOCUS_KC_POINTWISE = 3, /* embedding, RMSNorm, SiLU*up, row bookkeeping */
       FOCUS_KC_DECODE = 4,    /* confidence over the vocabulary, commit */
       FOCUS_KC_ROUTE = 5,     /* mixture-of-experts: picks, sorting by expert, weighted sum */
       FOCUS_KC_EXPERTS = 6,   /* mixture-of-experts: the grouped gate/up and down projections of the routed experts
                                  (router and shared expert are dense projections, FOCUS_KC_GEMM) */
       FOCUS_KC_SELECT = 7,    /* delta, budget, selection (Eq. 3-5, Alg. 1 phase 3) and the prefix-sum packing */
       FOCUS_KC_GATHER = 8,    /* gather of the retained rows into the packed batch */
       FOCUS_KC_KV_WRITE = 9,  /* rotary embedding + scatter of K and V into the paged cache */
       FOCUS_KC_COUNT = 10 };
int focus_set_timing(focus_ctx *ctx, int32_t enable);
int focus_get_kernel_time(focus_ctx *ctx, int32_t kernel_class, float *total_ms, int32_t *launches);

/* Infrastructure.  Destroys the context; the borrowed buffers stay the caller's. */
int focus_free(focus_ctx *ctx);
/* Infrastructure.  Text of the last error of ctx, or of the last failed call without a context when ctx is NULL. */
const char *focus_last_error(const focus_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* FOCUS_H */
