/*
 * keep_memory.h -- C ABI of the static-dynamic memory construction (KEEP, arxiv 2602.23592,
 * Section 4.1) and of the cache computation it triggers.
 *
 * A memory store holds segments (token sequences) clustered into groups.  A group is STATIC
 * when nothing about it changed during the recent `window_t` steps, else DYNAMIC; a new group
 * starts dynamic.  A static group is cached as ONE unit (its segments concatenated in ascending
 * segment id, full attention between them); a dynamic group is cached one segment per unit, so
 * an update invalidates that segment only.  When a group changes category, its units are
 * recomputed the new way.  The units are also what retrieval hands to the prompt: a static group
 * as a whole, a dynamic segment on its own (they become the `group_len` / `group_kind` entries of
 * a keep_prompt).
 *
 * The store is host-side bookkeeping: every pointer here is a HOST pointer except where
 * keep_precompute_group says DEVICE.  Which group a segment belongs to is the caller's decision
 * (the paper clusters with a sentence encoder).  "Changed" = new content, a segment added to or
 * removed from the group; writing back identical tokens is not a change.  Steps are counted by
 * keep_memory_end_step: a change made while step s is open has age 0 when s closes, and a group is
 * static when the age of its newest change is >= window_t.
 * Functions return a keep_status; keep_memory_last_error gives the text of the last failure.
 * A store must not be used from two threads at once.
 */
#ifndef KEEP_MEMORY_H
#define KEEP_MEMORY_H

#include "keep.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct keep_memory keep_memory; /* opaque, library-owned */

typedef enum { KEEP_UNIT_STATIC_GROUP = 0, KEEP_UNIT_DYNAMIC_SEGMENT = 1 } keep_unit_kind;

typedef struct {
  int32_t kind;       /* keep_unit_kind */
  int32_t id;         /* group id (static group) or segment id (dynamic segment) */
  int32_t group;      /* the group it belongs to */
  int32_t n_segments; /* segments it concatenates (1 for a dynamic segment) */
  int32_t n_tokens;
  int32_t dirty;      /* 1: its KV cache has to be (re)computed, see keep_memory_mark_computed */
} keep_memory_unit;

typedef struct {
  int32_t step;         /* index of the step that was closed */
  int32_t n_static, n_dynamic; /* groups in each state after the step */
  int32_t n_to_dynamic; /* groups that left the static state at this step */
  int32_t n_to_static;  /* groups that became static at this step */
  int32_t dirty_units;  /* units whose KV has to be computed now ... */
  int64_t dirty_tokens; /* ... and their tokens: the cost of this step's memory update */
} keep_memory_step_report;

/* window_t >= 0: steps without a change after which a group is static (the paper uses 10). */
keep_status keep_memory_create(int32_t window_t, keep_memory** out);
keep_status keep_memory_destroy(keep_memory* mem);
const char* keep_memory_last_error(const keep_memory* mem);

/* Add segment `segment_id` to group `group_id`, or replace its content (Section 4.1: a memory
 * update).  token_ids: HOST [n_tokens], n_tokens >= 1, copied.  *changed (may be NULL) is set to 0
 * when the tokens equal the stored ones.  Errors: INVALID_ARG (NULL, n_tokens < 1, negative ids,
 * segment already in another group). */
keep_status keep_memory_put(keep_memory* mem, int32_t group_id, int32_t segment_id, const int32_t* token_ids,
                            int32_t n_tokens, int32_t* changed);
/* Remove a segment; a group left without segments disappears.  Errors: INVALID_ARG (unknown id). */
keep_status keep_memory_remove(keep_memory* mem, int32_t segment_id);

/* Close the open step: re-classify every group (static <=> unchanged for window_t steps),
 * invalidate the units of groups that changed category, count what has to be computed.
 * report may be NULL.  to_dynamic / to_static (may be NULL, capacity cap_* ids) receive the ids
 * of the groups that changed category, ascending. */
keep_status keep_memory_end_step(keep_memory* mem, keep_memory_step_report* report, int32_t* to_dynamic,
                                 int32_t cap_to_dynamic, int32_t* to_static, int32_t cap_to_static);

/* Units in prompt order: groups by ascending id; a dynamic group's segments by ascending id. */
int32_t keep_memory_unit_count(const keep_memory* mem);
keep_status keep_memory_unit_info(const keep_memory* mem, int32_t unit, keep_memory_unit* out);
/* Token ids of a unit into out[cap]; *n_tokens gets the count.  Errors: INVALID_ARG, WORKSPACE (cap too small). */
keep_status keep_memory_unit_tokens(const keep_memory* mem, int32_t unit, int32_t* out, int32_t cap,
                                    int32_t* n_tokens);
/* The caller has computed and stored this unit's KV (keep_precompute_group): clear its dirty flag. */
keep_status keep_memory_mark_computed(keep_memory* mem, int32_t unit);

/* KV cache of one unit computed on its own (Section 4.1: a static group jointly, a dynamic segment
 * individually): dense causal prefill of the unit's tokens at positions 0..n_tokens-1 through every
 * layer of the context's model.
 *   token_ids: HOST [n_tokens].
 *   k_blocks, v_blocks: DEVICE [n_layers][n_tokens, n_kv_heads, head_dim], written in full; layer l
 *     is the unit's block of layer l as keep_prompt expects it (K rotated at the local positions).
 *   report: HOST or NULL (per-layer times as for keep_prefill).
 * Output is ordered on the compute stream.  Errors: INVALID_ARG, WORKSPACE (n_tokens above the
 * context's max_tokens), HIP. */
keep_status keep_precompute_group(keep_ctx* ctx, const int32_t* token_ids, int32_t n_tokens, void* k_blocks,
                                  void* v_blocks, keep_report* report);

/* The same for several units in one pass (a static group that turned dynamic needs every segment cached
 * on its own; a first build of the memory needs every unit): unit u's tokens follow unit u-1's in
 * token_ids, and its blocks follow in k_blocks / v_blocks, so layer l of unit u starts at row
 * (l * total + off_u) with off_u = unit_len[0] + ... + unit_len[u-1], total = sum of unit_len.  Every unit
 * is rotated at its own local positions and attends to its own tokens only, as if computed alone.
 *   unit_len: HOST [n_units], each >= 1; token_ids: HOST [total].
 *   k_blocks, v_blocks: DEVICE [n_layers][total, n_kv_heads, head_dim], written in full.
 * Errors: INVALID_ARG, WORKSPACE (total above the context's max_tokens), HIP. */
keep_status keep_precompute_groups(keep_ctx* ctx, int32_t n_units, const int32_t* unit_len, const int32_t* token_ids,
                                   void* k_blocks, void* v_blocks, keep_report* report);

#ifdef __cplusplus
}
#endif
#endif /* KEEP_MEMORY_H */
