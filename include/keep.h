/*
 * keep.h -- C ABI of the selective-KV-recompute prefill library for MI355X (gfx950).
 *
 * The library implements the hot path of KEEP (arxiv 2602.23592): memory groups
 * whose KV caches were computed independently (Section 4.1) are joined into one
 * prompt, instruction last (Section 1); at every layer only the memories in the
 * current relevant set are recomputed over the joined cache (Section 4.2,
 * "Selective Recomputation"; Section 5, `prefill_layer`), the set for the next
 * layer is found by multi-hop importance propagation over group-to-group
 * attention (Section 4.2, the four steps; Section 5, `importance_evaluation`),
 * and group caches held in host memory are loaded layer by layer, overlapped
 * with compute (Section 4.3; Section 5, `load_memory`).
 *
 * Conventions
 *   - Plain C types only.  Every pointer argument says whether it is a HOST or a
 *     DEVICE pointer.  The caller owns every buffer it passes in or gets results
 *     in; the library never frees caller memory.  A context owns its workspace
 *     (sized at keep_init from max_tokens / max_groups) and its RoPE table.
 *   - Weights and the embedding table are borrowed for the context's lifetime.
 *   - Tensors are dense row-major.  `dtype` (KEEP_F32 or KEEP_BF16) is the storage
 *     type of weights, caches, hidden rows; arithmetic accumulates in fp32.
 *   - Every function returns a keep_status and never throws or aborts;
 *     keep_last_error() gives the text of the last failure on that context (or of
 *     the last failed keep_init when passed NULL).
 *   - Device outputs are ordered on the compute stream given to keep_init; host
 *     outputs are valid on return.  One context must not be used from two threads
 *     at once.
 *   - Token positions are indices into the joined prompt: group g starts at
 *     off_g = len_0 + ... + len_{g-1}; instruction rows follow the last group.
 *     N_mem = sum of group_len, N = N_mem + instr_len.
 *   - A "relevant set" is a strictly ascending list of group indices.  The rows
 *     recomputed at a layer are the tokens of those groups in prompt order followed
 *     by every instruction row; n_rows = sum of their lengths + instr_len.
 */
#ifndef KEEP_H
#define KEEP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct keep_ctx keep_ctx; /* opaque, library-owned */

typedef enum {
  KEEP_OK = 0,
  KEEP_ERR_INVALID_ARG = 1, /* NULL pointer, out-of-range scalar, unsorted set, bad ratio schedule */
  KEEP_ERR_SHAPE = 2,       /* model or prompt shape the kernels cannot take */
  KEEP_ERR_STATE = 3,       /* call out of order (scores asked before the layer was computed) */
  KEEP_ERR_WORKSPACE = 4,   /* prompt larger than max_tokens / max_groups given at init */
  KEEP_ERR_HIP = 5,         /* a HIP runtime call failed; text in keep_last_error */
  KEEP_ERR_UNSUPPORTED = 6
} keep_status;

typedef enum { KEEP_F32 = 0, KEEP_BF16 = 1 } keep_dtype;
typedef enum { KEEP_KV_DEVICE = 0, KEEP_KV_PINNED_HOST = 1 } keep_kv_location;

/* How a ratio becomes a budget (Section 4.2: each layer keeps the top share r_i of the memories):
 * a number of memories, ceil(ratio * n_groups - 1e-3), or a number of tokens,
 * floor(ratio * N_mem + 1e-3), filled by walking the importance order. */
typedef enum { KEEP_BUDGET_GROUP_COUNT = 0, KEEP_BUDGET_TOKENS = 1 } keep_budget_mode;

/* Host->device loading of group caches (Section 4.3, Fig. 8 a/b/c):
 * SERIAL: load layer l, then compute it.  NEXT_LAYER: while layer l computes, load
 * layer l+1 for the groups outside the current set.  LAYER_BALANCED: as NEXT_LAYER,
 * and while compute is still running keep pre-loading later layers for groups that
 * can no longer be recomputed.  All three give bit-identical results. */
typedef enum { KEEP_LOAD_SERIAL = 0, KEEP_LOAD_NEXT_LAYER = 1, KEEP_LOAD_LAYER_BALANCED = 2 } keep_load_mode;

/* Kernel family.  AUTO: MFMA kernels when dtype is bf16 and head_dim is 128 and
 * hidden, ffn_dim are multiples of 64; otherwise the generic kernels.  GENERIC:
 * always the scalar-FMA kernels (any head_dim that is even, fp32 or bf16). */
typedef enum { KEEP_KERNELS_AUTO = 0, KEEP_KERNELS_GENERIC = 1 } keep_kernel_path;

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  float rope_theta; /* RoPE base; rotate-half pairing (j, j + head_dim/2) */
  float rms_eps;
  int32_t dtype;       /* keep_dtype */
  int32_t max_tokens;  /* largest N of any prompt given to this context */
  int32_t max_groups;  /* largest n_groups */
  int32_t kernel_path; /* keep_kernel_path */
} keep_model_desc;

/* One decoder layer (pre-norm, GQA, SwiGLU).  DEVICE pointers, torch.nn.Linear
 * layout [out_features, in_features] row-major.  bq/bk/bv may be NULL (no bias).
 * ln1/ln2: RMSNorm weights [hidden]. */
typedef struct {
  const void *ln1, *wq, *wk, *wv, *bq, *bk, *bv, *wo, *ln2, *wgate, *wup, *wdown;
} keep_layer_weights;

/* The joined prompt (Section 1: retrieved memory then instruction). */
typedef struct {
  int32_t n_groups;          /* G >= 0 */
  const int32_t* group_len;  /* HOST [G], each >= 1: a static group or one dynamic segment (Section 4.1) */
  const uint8_t* group_kind; /* HOST [G] or NULL: 0 static, 1 dynamic (bookkeeping only) */
  int32_t instr_len;         /* >= 1 */
  const int32_t* token_ids;  /* HOST [N]: groups in order, then the instruction */
  /* [n_layers * G], index layer*G + g: that group's cached K and V of that layer,
   * each [len_g, n_kv_heads, head_dim], K rotated at group-local positions 0..len_g-1.
   * The arrays of pointers are HOST arrays; the blocks are DEVICE memory
   * (KEEP_KV_DEVICE) or pinned HOST memory (KEEP_KV_PINNED_HOST). */
  const void* const* k_blocks;
  const void* const* v_blocks;
  int32_t kv_location; /* keep_kv_location */
} keep_prompt;

#define KEEP_REPORT_MAX_LAYERS 128
/* Filled by keep_prefill when a report is asked for (caller-allocated, HOST).
 * Times are device times between HIP events recorded on the stream the kernels run
 * on (compute stream; eval stream for ms_score), in milliseconds, per layer. */
#define KEEP_REPORT_EVENTS_ALL 0     /* events around every kernel: all ms_* fields are filled */
#define KEEP_REPORT_EVENTS_GATE_UP 1 /* events around the gate/up GEMM only (ms_gateup): ~2 ms less intrusive at 48 layers */
typedef struct {
  int32_t events_in;                           /* IN: KEEP_REPORT_EVENTS_*; the only field read by the library */
  int32_t n_layers;
  int32_t used_mfma;                           /* 1 if the MFMA kernel family ran */
  float ms_total;                              /* whole call, host clock */
  int32_t rows[KEEP_REPORT_MAX_LAYERS];        /* n_rows recomputed at each layer */
  int32_t set_size[KEEP_REPORT_MAX_LAYERS];    /* groups recomputed at each layer */
  int32_t hops_run[KEEP_REPORT_MAX_LAYERS];    /* selections run after each layer */
  int32_t realign_rows[KEEP_REPORT_MAX_LAYERS];/* cache rows re-aligned (groups outside the set) */
  int32_t ffn_rows[KEEP_REPORT_MAX_LAYERS];    /* rows the output projection + FFN ran on: rows[l], or the
                                                  next layer's rows when evaluation went first (see keep_prefill);
                                                  at the last layer the instruction's rows */
  int32_t attn_rows[KEEP_REPORT_MAX_LAYERS];   /* rows the attention ran on: rows[l], or fewer where only the rows
                                                  whose scores or outputs are read were attended (see keep_prefill:
                                                  layers that score on demand, and the last layer) */
  uint64_t attn_keys[KEEP_REPORT_MAX_LAYERS];  /* keys those rows see in all: sum of (position + 1) */
  float ms_realign[KEEP_REPORT_MAX_LAYERS];    /* re-align + concatenate kernel */
  float ms_prep[KEEP_REPORT_MAX_LAYERS];       /* row table, gather, first RMSNorm */
  float ms_qkv_gemm[KEEP_REPORT_MAX_LAYERS];   /* QKV projection GEMM alone */
  float ms_rope[KEEP_REPORT_MAX_LAYERS];       /* bias + RoPE + scatter kernel */
  float ms_attn[KEEP_REPORT_MAX_LAYERS];       /* sparse-row attention kernel */
  float ms_oproj[KEEP_REPORT_MAX_LAYERS];      /* output projection GEMM (+ residual) */
  float ms_norm2[KEEP_REPORT_MAX_LAYERS];      /* second RMSNorm */
  float ms_gateup[KEEP_REPORT_MAX_LAYERS];     /* gate/up GEMM with fused SwiGLU */
  float ms_down[KEEP_REPORT_MAX_LAYERS];       /* down GEMM (+ residual) */
  float ms_score[KEEP_REPORT_MAX_LAYERS];      /* score reduction + selection, eval stream */
  uint64_t bytes_loaded[KEEP_REPORT_MAX_LAYERS]; /* host->device bytes enqueued for this layer's turn */
} keep_report;

/* Create a context.  desc, layers[n_layers]: HOST structs holding DEVICE pointers;
 * embed_table: DEVICE [vocab, hidden].  The three streams are hipStream_t handles
 * (NULL = the default stream) for layer compute, importance evaluation (runs beside
 * the FFN, Section 4.2 "System advantage") and host->device loading (Section 5,
 * the three pipelined threads).  All must be at the default priority.
 * Errors: INVALID_ARG (NULL, non-positive sizes, n_q_heads not a multiple of
 * n_kv_heads, odd head_dim), SHAPE (head_dim > 256, n_layers > 128, max_groups > 6000), HIP. */
keep_status keep_init(const keep_model_desc* desc, const keep_layer_weights* layers, const void* embed_table,
                      void* stream_compute, void* stream_eval, void* stream_copy, keep_ctx** out);

/* Waits for the context's streams, frees workspace and RoPE table.  NULL is OK. */
keep_status keep_destroy(keep_ctx* ctx);

/* HOST string owned by the library, valid until the next call on that context. */
const char* keep_last_error(const keep_ctx* ctx);

/* 1 if this context runs the MFMA kernel family, 0 if the generic one, -1 if ctx is NULL. */
int32_t keep_uses_mfma(const keep_ctx* ctx);

/* Device bytes a context for this description allocates (0 if desc is invalid). */
uint64_t keep_workspace_bytes(const keep_model_desc* desc);

/* Options of a context (keep_set_option).
 * KEEP_OPT_PROPAGATION_SOURCES: which rows of the normalised score matrix the importance propagation of
 *   Section 4.2 averages from the second selection on.
 *   KEEP_SOURCES_QUERY_AND_SET (default): the query's row and the rows of the current relevant set (the
 *     query keeps anchoring the importance, so first-hop memories are not evicted by their neighbours);
 *   KEEP_SOURCES_SET_ONLY: the rows of the current relevant set alone, which is the section's propagation
 *     step taken word for word (the query's row only initialises the importance). */
typedef enum { KEEP_OPT_PROPAGATION_SOURCES = 0 } keep_option;
typedef enum { KEEP_SOURCES_QUERY_AND_SET = 0, KEEP_SOURCES_SET_ONLY = 1 } keep_propagation_sources;

/* Sets an option for every later keep_score_groups / keep_select_groups / keep_prefill on this context.
 * Errors: INVALID_ARG (NULL context, unknown option or value). */
keep_status keep_set_option(keep_ctx* ctx, int32_t option, int32_t value);

/* What keep_read_layer_state copies out: the state keep_recompute_layer leaves in the workspace. */
typedef enum {
  KEEP_STATE_ATTN_OUT = 0, /* attention output of the recomputed rows, [n_rows, n_q_heads * head_dim], storage dtype */
  KEEP_STATE_LSE = 1       /* log-sum-exp of each row's scaled scores, [n_rows, n_q_heads], float */
} keep_layer_state;

/* Copies a piece of the state that the last keep_recompute_layer left in the workspace (Section 5: the
 * attention of a layer is what its importance evaluation reads) to HOST memory, for inspection and tests.
 * Waits for the compute stream.  dst: HOST, capacity `bytes`, which must equal the size given above for
 * the rows of that call.
 * Errors: STATE (no keep_recompute_layer since the last call that overwrote the workspace),
 * INVALID_ARG (NULL, unknown `what`, wrong size), HIP. */
keep_status keep_read_layer_state(keep_ctx* ctx, int32_t what, void* dst, uint64_t bytes);

/* `prefill_layer` (Section 5): one layer of selective recomputation.
 *   groups[n_sel]: HOST, ascending: the relevant set R of this layer.
 *   x_in:  DEVICE [n_rows, hidden] hidden rows of the recomputed tokens in prompt
 *          order; NULL at layer 0 = embedding rows of those tokens.
 *   x_out: DEVICE [n_rows, hidden] hidden rows after the layer (may equal x_in).
 *   k_cache_l, v_cache_l: DEVICE [N, n_kv_heads, head_dim], written in full: rows of
 *          groups outside R get the cached K rotated on by the group's offset and the
 *          cached V (position re-alignment); rows of R and of the instruction get the
 *          refreshed K (RoPE at the global position) and V.
 * Steps: re-align + concatenate, RMSNorm, QKV projection of the n_rows rows, RoPE,
 * scatter, causal attention of those rows over all N cache rows, output projection,
 * residual, RMSNorm, SwiGLU FFN, residual.  Leaves q, k and the softmax
 * log-sum-exp of this layer in the workspace for keep_score_groups.
 * With KEEP_KV_PINNED_HOST blocks the call copies the needed blocks itself.
 * Errors: INVALID_ARG, WORKSPACE (N > max_tokens, G > max_groups), HIP. */
keep_status keep_recompute_layer(keep_ctx* ctx, const keep_prompt* prompt, int32_t layer, const int32_t* groups,
                                 int32_t n_sel, const void* x_in, void* x_out, void* k_cache_l, void* v_cache_l);

/* `importance_evaluation` (Section 5; Section 4.2 steps 1-3) for the layer last given
 * to keep_recompute_layer, with the same `groups`.
 *   S[a, b] = attention probability from the rows of a to the keys of b averaged over
 *   heads, rows and keys; a over groups[] then the instruction (last row), b over
 *   groups[]; S[a, a] = 0.  Then: row-normalise, importance = query row, relevant set =
 *   top of the importance order within the budget, importance = mean of the normalised
 *   rows of the query and of the relevant set, repeat until the set repeats or `hops`
 *   selections were made (hops = 1: initialisation only).  Ties: lower group index.
 *   ratio_next: share of the prompt's memories (or memory tokens) kept for the next layer.
 *   S_out: HOST [(n_sel+1) * n_sel] or NULL.  next_groups: HOST, capacity n_sel,
 *   ascending subset of groups[].  n_next, hops_run: HOST scalars.
 * Errors: STATE if `layer`/`groups` differ from the last keep_recompute_layer,
 * INVALID_ARG, HIP. */
keep_status keep_score_groups(keep_ctx* ctx, const keep_prompt* prompt, int32_t layer, const int32_t* groups,
                              int32_t n_sel, float ratio_next, int32_t hops, int32_t budget_mode, float* S_out,
                              int32_t* next_groups, int32_t* n_next, int32_t* hops_run);

/* The selection steps alone (Section 4.2 steps 1-3) on a caller-supplied score
 * matrix S: HOST [(n_sel+1) * n_sel], last row the query; group_len: HOST
 * [n_groups_total] lengths of all the prompt's groups.  Same outputs as above. */
keep_status keep_select_groups(keep_ctx* ctx, const float* S, const int32_t* groups, int32_t n_sel,
                               const int32_t* group_len, int32_t n_groups_total, float ratio_next, int32_t hops,
                               int32_t budget_mode, int32_t* next_groups, int32_t* n_next, int32_t* hops_run);

#define KEEP_STATIC_MAX_CANDIDATES 4096
/* keep_select_groups for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It needs no context: the scratch that the selection uses
 * beyond its inputs and outputs (the candidates' lengths and their token total) lives in a device array built
 * into the library (16.25 KiB, held by every GPU the library runs on until the process ends), and the call
 * makes no allocation, on the device or through any library.  Inputs and outputs are DEVICE memory:
 *   S:         DEVICE [(n_sel + 1) * n_sel], last row the query (as keep_select_groups, but on the device).
 *   groups:    DEVICE [n_sel], strictly ascending group ids below n_groups_total (not checked; ids are clamped
 *              into range when the lengths are looked up).
 *   group_len: DEVICE [n_groups_total] lengths of all the prompt's groups; mem_tokens: their sum (the token
 *              budget is a share of it).
 *   propagation_sources: keep_propagation_sources (there is no context to hold the option).
 *   result:    DEVICE [n_sel + 2]: result[0] = n_next, result[1] = selections run (0 where the budget keeps all
 *              or none of the candidates), result[2 .. 2 + n_next) = the kept group ids, ascending.
 *   stream:    hipStream_t or NULL; the kernels are enqueued on it and the call does not wait for them.
 * Every call on one GPU shares that GPU's scratch array: calls that overlap on one GPU (two streams, two
 * threads) race; calls on one stream are ordered and need nothing cleared in between.
 * Errors (text at keep_last_error(NULL)): INVALID_ARG (NULL pointer, unknown mode, ratio outside [0, 1],
 * hops < 1, n_sel outside [0, n_groups_total], mem_tokens < n_groups_total), WORKSPACE (n_sel above
 * KEEP_STATIC_MAX_CANDIDATES), HIP. */
keep_status keep_select_groups_static(const float* S, const int32_t* groups, int32_t n_sel, const int32_t* group_len,
                                      int32_t n_groups_total, int32_t mem_tokens, float ratio_next, int32_t hops,
                                      int32_t budget_mode, int32_t propagation_sources, int32_t* result, void* stream);

/* Whole selective prefill (Section 4.2 + 4.3 + 5): for l = 0..n_layers-1 recompute
 * the relevant set of layer l, evaluate importance beside the FFN, load what layer
 * l+1 needs.  Evaluation runs beside the output projection and FFN (Section 4.2), except where the
 * budget says that at most half of a layer's rows survive (typically after layer 0): there it runs
 * first and the output projection and FFN are computed for the surviving rows only, which gives the
 * same result because the hidden rows of dropped memories are discarded (Section 4.3).  At such a layer, when
 * there are also 64 or more candidates, the score matrix is formed hop by hop for the rows the propagation
 * reads (the query's, then those of each hop's relevant set), and the attention runs only for those rows and
 * for the rows that survive: neither the scores nor the outputs of the other rows are ever read.  The same
 * holds for the last layer, whose memory rows feed nothing: K and V of its set are refreshed, attention,
 * output projection and FFN run for the instruction's rows.
 *   ratios: HOST [n_layers]; ratios[0] is 1 (recompute every memory at the first
 *           layer, Section 4.2) or 0 (pure reuse); ratios[1..] non-increasing (a memory
 *           dropped once is never recomputed, Section 4.3).
 *   k_cache, v_cache: DEVICE [n_layers][N, n_kv_heads, head_dim], written in full.
 *   x_final: DEVICE [instr_len, hidden]: hidden rows of the instruction after the
 *           last layer (before any final norm).
 *   sel_groups: HOST [n_layers * n_groups] or NULL; row l holds the set of layer l.
 *   sel_counts: HOST [n_layers] or NULL.  report: HOST or NULL.
 * Errors: INVALID_ARG (schedule), WORKSPACE, SHAPE, HIP. */
keep_status keep_prefill(keep_ctx* ctx, const keep_prompt* prompt, const float* ratios, int32_t hops,
                         int32_t budget_mode, int32_t load_mode, void* k_cache, void* v_cache, void* x_final,
                         int32_t* sel_groups, int32_t* sel_counts, keep_report* report);

/* The token-granularity scheme that Section 3 and Section 4.2 ("System advantage") set the method against, on the
 * same kernels: single tokens, not memories, are recomputed.  Every cached block of every layer is loaded and
 * re-aligned (the whole cache is joined), the recomputed tokens' K/V are written over their rows in place, and
 * the memory tokens of layer l+1 are the ceil(ratios[l+1] * N_mem) tokens of layer l whose recomputed K/V state
 * lies furthest from the cached one: deviation = sum over KV heads and dimensions of (k_new - k_cached)^2 +
 * (v_new - v_cached)^2 on the values as stored, summed in binary32 in a fixed order; ties: the lower position.
 * Instruction tokens are recomputed at every layer.  The deviation of a layer is known after its K/V
 * projection, so the attention, the output projection and the FFN of a layer run for the tokens that stay.
 * (At layer 0 the deviation is zero up to rounding: K/V of the first layer depend on the token alone.  A
 * schedule that means anything keeps ratios[1] = 1 and starts selecting from layer 1.)
 *   ratios, k_cache, v_cache, x_final, report: as keep_prefill.  load_mode: SERIAL loads layer l+1 after layer
 *           l's compute, the other two modes load it beside layer l (the whole of it, whatever is selected).
 *   sel_rows: HOST [n_layers * N_mem] or NULL; row l holds the ascending positions of the memory tokens
 *           recomputed at layer l.  sel_counts: HOST [n_layers] or NULL.
 *   deviation_out: HOST [n_layers * N_mem] or NULL; row l holds the deviation of the tokens of sel_rows row l
 *           (costs one device-to-host copy and a wait per layer).
 * Errors: INVALID_ARG (schedule), WORKSPACE, SHAPE, HIP. */
keep_status keep_prefill_tokens(keep_ctx* ctx, const keep_prompt* prompt, const float* ratios, int32_t load_mode,
                                void* k_cache, void* v_cache, void* x_final, int32_t* sel_rows, int32_t* sel_counts,
                                float* deviation_out, keep_report* report);

/* The token selection alone on caller-supplied deviations: deviation HOST [n], kept HOST [k] receives the
 * ascending indices of the k largest (ties: lower index).  Errors: INVALID_ARG (k outside [0, n], NULL),
 * WORKSPACE (n above max_tokens), HIP. */
keep_status keep_select_tokens(keep_ctx* ctx, const float* deviation, int32_t n, int32_t k, int32_t* kept);

/* keep_prefill into caches with room for decoded tokens: as keep_prefill, but layer l of k_cache / v_cache
 * starts at row l * cache_rows (cache_rows >= N); rows N..cache_rows-1 of every layer are left untouched.
 * Errors: as keep_prefill, INVALID_ARG if cache_rows < N. */
keep_status keep_prefill_padded(keep_ctx* ctx, const keep_prompt* prompt, const float* ratios, int32_t hops,
                                int32_t budget_mode, int32_t load_mode, void* k_cache, void* v_cache,
                                int32_t cache_rows, void* x_final, int32_t* sel_groups, int32_t* sel_counts,
                                keep_report* report);

#define KEEP_DECODE_MAX_TOKENS 64
/* First token and short greedy decoding over the joined cache (Section 1: after the long prompt the
 * planner emits a short action; Section 5: the decoder continues on the cache that prefill_layer updated).
 * Token 0 = argmax over the vocabulary of lm_head . RMSNorm(x_last); token t > 0 comes from running
 * token t-1 at position n_ctx + t - 1 through every layer: its K/V are written to row n_ctx + t - 1 of
 * the caches and it attends to rows 0 .. n_ctx + t - 1.  Equal logits: the lowest token id.
 *   final_norm: DEVICE [hidden]; lm_head: DEVICE [vocab, hidden] (row-major, as torch.nn.Linear).
 *   x_last: DEVICE [hidden]: hidden row of the last prompt token (last row of keep_prefill's x_final).
 *   k_cache, v_cache: DEVICE [n_layers][cache_rows, n_kv_heads, head_dim], rows 0..n_ctx-1 valid
 *     (keep_prefill_padded's output); rows n_ctx .. n_ctx + n_new - 2 are written.
 *   n_new: 1..KEEP_DECODE_MAX_TOKENS.  tokens_out: HOST [n_new], valid on return.
 *   logits_out: DEVICE [n_new, vocab] fp32 or NULL.
 *   forced_tokens: HOST [n_new - 1] or NULL; when given, forced_tokens[t] is fed forward instead of
 *     token t (tokens_out still holds the greedy choices).
 * Errors: INVALID_ARG (NULL, n_new out of range, n_ctx < 1, n_ctx + n_new - 1 above cache_rows),
 * WORKSPACE (n_ctx + n_new - 1 above the context's max_tokens), HIP. */
keep_status keep_decode(keep_ctx* ctx, const void* final_norm, const void* lm_head, const void* x_last,
                        void* k_cache, void* v_cache, int32_t cache_rows, int32_t n_ctx, int32_t n_new,
                        int32_t* tokens_out, float* logits_out, const int32_t* forced_tokens);

/* ---- INT4 weight-only matrices (Section 6.1: the 32B model is run with INT4 weight-only quantisation) ----
 * Format of one matrix W[rows, K] (rows a multiple of 32, K a multiple of 128), all DEVICE memory, caller-owned:
 *   codes       rows * K / 2 bytes: 4-bit codes q in 0..15, stored in blocks of 32 rows x 128 input features.
 *               Block (row / 32, feature / 128) starts at byte ((row / 32) * (K / 128) + feature / 128) * 2048;
 *               inside it row r % 32 takes bytes 64 (r % 32) .. + 63; within each run of 8 consecutive input
 *               features, byte t (t < 4) holds feature t in its low nibble and feature t + 4 in its high one;
 *   scale_zero  rows * K / 128 uint32, one per (row, group of 128 features), in the same block order, 32 words
 *               per block: word ((row / 32) * (K / 128) + group) * 32 + row % 32; bits 0..15 the bfloat16
 *               pattern of the group's scale s, bits 16..19 its zero point z, other bits 0.
 *   (A request for 32 bytes of each of 32 consecutive rows is then one contiguous 2 KB block instead of 32
 *   pieces K/2 bytes apart.)
 * The weight the model computes with is  w = bf16((q - z) * s), rounded to nearest even: the 4-bit form is
 * a compact storage of exactly those bfloat16 values.  The calibration that chooses q, z, s is not part of
 * this library (weights arrive quantised). */
typedef struct {
  const void* codes;
  const void* scale_zero;
} keep_int4_matrix;

/* The seven projections of one layer, shapes as in keep_layer_weights. */
typedef struct {
  keep_int4_matrix wq, wk, wv, wo, wgate, wup, wdown;
} keep_layer_weights_int4;

/* out[rows, K] (DEVICE, bfloat16) = the weights of an INT4 matrix.  With these as the keep_layer_weights
 * of keep_init, the launches that are bound by the matrix cores (many rows) run on the expanded copy.
 *   stream: hipStream_t or NULL (default stream); the call does not wait for the kernel.
 * Errors: INVALID_ARG (NULL, rows not a positive multiple of 32, K not a positive multiple of 128), HIP.  Needs no context:
 * the message of a failure is at keep_last_error(NULL). */
keep_status keep_dequantize_int4(const void* codes, const void* scale_zero, int32_t rows, int32_t K, void* out,
                                 void* stream);

/* Registers the INT4 form of every layer's projections with a context whose keep_layer_weights are their
 * bfloat16 expansion (keep_dequantize_int4).  From then on the launches that are bound by reading the
 * weights (at most 48 rows: keep_decode, keep_precompute_group of a short segment, prompts of a few rows)
 * read the 4-bit form, a quarter of the bytes, and expand it in registers to the same bfloat16 values, so
 * results differ from the bfloat16 launches only by the order of the fp32 accumulation.
 *   layers: HOST array [n_layers] of DEVICE pointers, borrowed until keep_destroy; NULL detaches.
 *   The LM head of keep_decode stays bfloat16.
 * Errors: INVALID_ARG (a NULL pointer inside), UNSUPPORTED (context not on the bf16 MFMA path),
 * SHAPE (hidden, ffn_dim or n_q_heads * head_dim not a multiple of 128, n_kv_heads * head_dim not of 64). */
keep_status keep_attach_int4(keep_ctx* ctx, const keep_layer_weights_int4* layers);

#ifdef __cplusplus
}
#endif
#endif /* KEEP_H */
