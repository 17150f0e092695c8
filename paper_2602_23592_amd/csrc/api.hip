// C ABI of libkeep_hip.so: argument checks, workspace, per-layer orchestration of the
// kernels over three HIP streams (layer compute / importance evaluation / host->device
// loading), following the pipeline of Section 5 of the paper.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <string>
#include <type_traits>
#include <vector>

#include "keep_internal.h"
#include "keep_memory.h"

using namespace keep;

namespace {

thread_local std::string g_init_error;

constexpr double BUDGET_EPS = 1.0e-3;
// events per layer: 0 begin, 1 re-align done, 2 rows/gather/norm done, 3 QKV GEMM done, 4 RoPE+scatter done,
// 5 attention done, 6 output projection done, 7 second norm done, 8 gate/up done, 9 down done, 10/11 score begin/end,
// 12 output projection begins
constexpr int EV_PER_LAYER = 13;
// Host->device pre-loads are enqueued only while fewer bytes than this are in flight,
// so that the copies a layer is waiting for never queue behind a long run of pre-loads.
constexpr size_t PRELOAD_INFLIGHT_CAP = 48u << 20;

struct Staging {  // pinned host mirror of the small per-layer device arrays
  int32_t* set_off;
  int32_t* row_start;
  int32_t* gather_src;
  int32_t* gather_dst;
  int32_t* cand_len;
  int32_t* score_tiles;  // row-tile table of the MFMA score pass
  int32_t* attn_items;   // work list of the MFMA attention
  RealignSeg* segs;
  hipEvent_t done;
  bool used;
};

}  // namespace

// Layout of the per-layer table block: three int arrays of G + 2, then G re-align segments (16-byte aligned).
static inline size_t table_seg_offset_ints(size_t G) { return (3 * (G + 2) + 3) & ~(size_t)3; }
static inline size_t table_block_bytes(size_t G) { return table_seg_offset_ints(G) * 4 + G * sizeof(keep::RealignSeg); }

struct keep_ctx {
  keep_model_desc d;
  std::vector<keep_layer_weights> w;
  std::vector<keep_layer_weights_int4> w4;  // empty: no INT4 form attached
  const void* embed = nullptr;
  hipStream_t s_comp = nullptr, s_eval = nullptr, s_copy = nullptr;
  bool mfma = false;
  size_t esz = 4;
  std::string err;

  // device workspace
  std::vector<void*> allocs;
  size_t bytes = 0;
  float *rope_cos = nullptr, *rope_sin = nullptr;
  int32_t *d_token_ids = nullptr, *d_row_pos = nullptr, *d_row_slot = nullptr;
  int32_t *d_set_off = nullptr, *d_row_start = nullptr, *d_gather_src = nullptr, *d_cand_len = nullptr;
  RealignSeg* d_segs = nullptr;
  void *xa = nullptr, *xb = nullptr, *hbuf = nullptr, *q = nullptr, *kc = nullptr, *o = nullptr, *x1 = nullptr,
       *act = nullptr, *attn_scratch = nullptr, *skinny_ws = nullptr;
  float *qkv_raw = nullptr, *lse = nullptr, *score_scratch = nullptr, *S = nullptr, *sel_work = nullptr;
  int32_t *sel_iwork = nullptr, *sel_out = nullptr;

  // pinned host
  std::vector<Staging> stage;       // one slot per layer
  int32_t* h_sel_out = nullptr;     // [max_groups + 2]
  int32_t* h_row_list = nullptr;    // pinned [max_tokens]: rows of an attention launch on part of a layer
  int32_t* d_row_list = nullptr;
  hipEvent_t ev_part[16] = {};      // begin / end pairs of such launches (timing)
  int32_t* h_row_lo = nullptr;      // pinned [max_tokens]: first visible key per row (batched unit caching)
  int32_t* d_row_lo = nullptr;
  float* d_dev = nullptr;           // [max_tokens] per-row K/V deviation (token-granularity selection)
  int32_t *d_tok_flags = nullptr, *d_tok_list = nullptr;  // [max_tokens] each
  int32_t* h_tok_list = nullptr;    // pinned [max_tokens]
  float* h_dev = nullptr;           // pinned [max_tokens]
  hipEvent_t ev_rowlist = nullptr;  // the last upload from h_row_list has been read by the device
  bool rowlist_pending = false;
  bool set_only = false;            // KEEP_OPT_PROPAGATION_SOURCES = KEEP_SOURCES_SET_ONLY
  bool ev_light = false;            // record only the events around the gate/up GEMM (keep_report.events_in = 1)
  bool units_mode = false;          // rows attend only from their unit's first row on
  int32_t* h_dec = nullptr;         // pinned [4 * KEEP_DECODE_MAX_TOKENS]: positions, fed tokens, results
  int32_t* d_dec = nullptr;         // device mirror
  float* dec_logits = nullptr;      // [vocab]
  float* h_S = nullptr;             // [(max_groups+1) * max_groups]
  int32_t* h_token_ids = nullptr;   // [max_tokens]

  std::vector<hipEvent_t> ev;       // EV_PER_LAYER per layer
  hipEvent_t ev_attn = nullptr, ev_eval = nullptr, ev_load = nullptr, ev_comp = nullptr, ev_tok = nullptr;
  bool tok_pending = false;          // an upload from h_token_ids may still be in flight
  std::vector<hipEvent_t> ev_chunk; // ring for pre-load flow control

  // work list of the last whole-layer MFMA attention, still in attn_scratch: the next layer reuses it when its
  // rows sit at the same positions (equal sets; the layers of a pure-reuse prompt)
  AttnPlan att_plan;
  std::vector<int32_t> att_plan_row_start, att_plan_set_off;
  int att_plan_n_mem = -1;

  // state left by keep_recompute_layer for keep_score_groups
  int last_layer = -1;
  std::vector<int32_t> last_groups;
  std::vector<int32_t> last_row_start;  // host copy, m+2 entries
  int last_n_rows = 0;
  const void* tokens_uploaded_for = nullptr;  // prompt token array currently in d_token_ids
  int tokens_uploaded_n = 0;
};

namespace {

}  // namespace

namespace keep {
// message behind keep_last_error(NULL), for entry points that have no context
void set_init_error(const char* text) { g_init_error = text; }
}  // namespace keep

namespace {

keep_status fail(keep_ctx* c, keep_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c)
    c->err = buf;
  else
    g_init_error = buf;
  return st;
}

#define HIP_TRY(c, expr)                                                                             \
  do {                                                                                               \
    hipError_t e__ = (expr);                                                                         \
    if (e__ != hipSuccess)                                                                           \
      return fail((c), KEEP_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

// INT4 form of a GEMM's weight parts, where the context has one
inline void set_w4(GemmB& b, int part, const keep_int4_matrix& m) {
  b.has_w4 = true;
  b.w4_codes[part] = m.codes;
  b.w4_scale_zero[part] = m.scale_zero;
}
inline void set_w4_b2(GemmB& b, const keep_int4_matrix& m) {
  b.w4_codes_b2 = m.codes;
  b.w4_scale_zero_b2 = m.scale_zero;
}

keep_status check_desc(const keep_model_desc* d, const char** why) {
  *why = "";
  if (!d) {
    *why = "desc is NULL";
    return KEEP_ERR_INVALID_ARG;
  }
  if (d->n_layers <= 0 || d->hidden <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 ||
      d->ffn_dim <= 0 || d->vocab <= 0 || d->max_tokens <= 0 || d->max_groups < 0) {
    *why = "non-positive size in keep_model_desc";
    return KEEP_ERR_INVALID_ARG;
  }
  if (d->n_q_heads % d->n_kv_heads) {
    *why = "n_q_heads must be a multiple of n_kv_heads";
    return KEEP_ERR_INVALID_ARG;
  }
  if (d->max_groups > 6000) {
    *why = "max_groups above 6000 (the selector keeps its per-memory arrays in LDS)";
    return KEEP_ERR_SHAPE;
  }
  if (d->dtype != KEEP_F32 && d->dtype != KEEP_BF16) {
    *why = "dtype must be KEEP_F32 or KEEP_BF16";
    return KEEP_ERR_INVALID_ARG;
  }
  if (d->kernel_path != KEEP_KERNELS_AUTO && d->kernel_path != KEEP_KERNELS_GENERIC) {
    *why = "unknown kernel_path";
    return KEEP_ERR_INVALID_ARG;
  }
  if (!(d->rope_theta > 0.f) || !(d->rms_eps >= 0.f)) {
    *why = "rope_theta must be > 0 and rms_eps >= 0";
    return KEEP_ERR_INVALID_ARG;
  }
  if (d->head_dim % 16 || d->head_dim > 256) {
    *why = "head_dim must be a multiple of 16 and at most 256";
    return KEEP_ERR_SHAPE;
  }
  if (d->hidden % 8 || d->ffn_dim % 8) {
    *why = "hidden and ffn_dim must be multiples of 8";
    return KEEP_ERR_SHAPE;
  }
  if (d->n_layers > KEEP_REPORT_MAX_LAYERS) {
    *why = "n_layers above 128";
    return KEEP_ERR_SHAPE;
  }
  return KEEP_OK;
}

bool wants_mfma(const keep_model_desc* d) {
  return d->kernel_path == KEEP_KERNELS_AUTO && d->dtype == KEEP_BF16 && d->head_dim == 128 && d->hidden % 64 == 0 &&
         d->ffn_dim % 64 == 0;
}

struct Sizes {
  size_t M, G, d, qd, kvd, F, esz;
};
Sizes sizes_of(const keep_model_desc* d) {
  Sizes z;
  z.M = (size_t)d->max_tokens;
  z.G = (size_t)std::max(1, d->max_groups);
  z.d = (size_t)d->hidden;
  z.qd = (size_t)d->n_q_heads * d->head_dim;
  z.kvd = (size_t)d->n_kv_heads * d->head_dim;
  z.F = (size_t)d->ffn_dim;
  z.esz = d->dtype == KEEP_BF16 ? 2 : 4;
  return z;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// list of (bytes) in a fixed order; used both to size and to carve the workspace
size_t score_scratch_bytes(const keep_model_desc* d) {
  Sizes z = sizes_of(d);
  size_t generic = z.M * z.G * sizeof(float);
  size_t mf = wants_mfma(d) ? score_mfma_scratch_bytes((int32_t)z.M, (int32_t)z.G) : 0;
  return std::max(generic, mf);
}

uint64_t workspace_bytes(const keep_model_desc* d) {
  Sizes z = sizes_of(d);
  size_t half = (size_t)d->head_dim / 2;
  size_t t = 0;
  t += 2 * align256(z.M * half * sizeof(float));                       // rope cos, sin
  t += 3 * align256(z.M * sizeof(int32_t));                            // token ids, row_pos, row_slot
  t += 4 * align256((z.G + 2) * sizeof(int32_t));                      // set_off, row_start, gather_src, cand_len
  t += align256(z.G * sizeof(RealignSeg));
  t += 4 * align256(z.M * z.d * z.esz);                                // xa, xb, h, x1
  t += 2 * align256(z.M * z.qd * z.esz);                               // q, o
  t += align256(z.M * z.kvd * z.esz);                                  // k compact
  t += align256(z.M * z.F * z.esz);                                    // act
  t += align256(z.M * (z.qd + 2 * z.kvd) * sizeof(float));             // qkv_raw
  t += align256(z.M * (size_t)d->n_q_heads * sizeof(float));           // lse
  t += align256(score_scratch_bytes(d));
  if (wants_mfma(d)) t += align256(attn_mfma_scratch_bytes((int32_t)z.M, d->n_q_heads, d->n_kv_heads));
  if (wants_mfma(d)) t += align256(gemm_ws_bytes());
  t += align256((z.G + 1) * z.G * sizeof(float));                      // S
  t += align256(((z.G + 1) * z.G + 2 * z.G) * sizeof(float));          // sel_work
  t += align256(4 * z.G * sizeof(int32_t)) + align256((z.G + 2) * sizeof(int32_t));
  t += align256(4 * KEEP_DECODE_MAX_TOKENS * 4) + align256((size_t)d->vocab * sizeof(float));  // decode
  t += 2 * align256(z.M * sizeof(int32_t));                            // row_lo, row_list
  t += 3 * align256(z.M * sizeof(int32_t));                            // token deviation, flags, kept list
  return t;
}

template <typename P>
keep_status dev_alloc(keep_ctx* c, P** p, size_t bytes) {
  void* v = nullptr;
  HIP_TRY(c, hipMalloc(&v, align256(std::max<size_t>(bytes, 256))));
  c->allocs.push_back(v);
  c->bytes += align256(bytes);
  *p = reinterpret_cast<P*>(v);
  return KEEP_OK;
}

template <typename P>
keep_status pin_alloc(keep_ctx* c, P** p, size_t bytes) {
  void* v = nullptr;
  HIP_TRY(c, hipHostMalloc(&v, std::max<size_t>(bytes, 64), hipHostMallocDefault));
  *p = reinterpret_cast<P*>(v);
  return KEEP_OK;
}

struct PromptInfo {
  int G = 0, Lq = 0, n_mem = 0, N = 0;
  std::vector<int32_t> off;  // G+1
};

keep_status check_prompt(keep_ctx* c, const keep_prompt* p, PromptInfo* pi, bool need_blocks) {
  if (!p) return fail(c, KEEP_ERR_INVALID_ARG, "prompt is NULL");
  if (p->n_groups < 0) return fail(c, KEEP_ERR_INVALID_ARG, "n_groups is negative");
  if (p->instr_len < 1) return fail(c, KEEP_ERR_INVALID_ARG, "instr_len must be at least 1 (the query drives the selection)");
  if (p->n_groups > 0 && !p->group_len) return fail(c, KEEP_ERR_INVALID_ARG, "group_len is NULL");
  if (!p->token_ids) return fail(c, KEEP_ERR_INVALID_ARG, "token_ids is NULL");
  if (p->kv_location != KEEP_KV_DEVICE && p->kv_location != KEEP_KV_PINNED_HOST)
    return fail(c, KEEP_ERR_INVALID_ARG, "unknown kv_location");
  if (need_blocks && p->n_groups > 0 && (!p->k_blocks || !p->v_blocks))
    return fail(c, KEEP_ERR_INVALID_ARG, "k_blocks / v_blocks is NULL");
  if (p->n_groups > c->d.max_groups)
    return fail(c, KEEP_ERR_WORKSPACE, "n_groups %d above max_groups %d", p->n_groups, c->d.max_groups);
  pi->G = p->n_groups;
  pi->Lq = p->instr_len;
  pi->off.assign(pi->G + 1, 0);
  int64_t tot = 0;
  for (int g = 0; g < pi->G; ++g) {
    if (p->group_len[g] < 1) return fail(c, KEEP_ERR_INVALID_ARG, "group_len[%d] = %d, must be >= 1", g, p->group_len[g]);
    tot += p->group_len[g];
    if (tot + p->instr_len > c->d.max_tokens)
      return fail(c, KEEP_ERR_WORKSPACE, "prompt longer than max_tokens %d", c->d.max_tokens);
    pi->off[g + 1] = (int32_t)tot;
  }
  if (tot + p->instr_len > c->d.max_tokens)
    return fail(c, KEEP_ERR_WORKSPACE, "prompt longer than max_tokens %d", c->d.max_tokens);
  pi->n_mem = (int)tot;
  pi->N = pi->n_mem + pi->Lq;
  for (int i = 0; i < pi->N; ++i)
    if (p->token_ids[i] < 0 || p->token_ids[i] >= c->d.vocab)
      return fail(c, KEEP_ERR_INVALID_ARG, "token_ids[%d] = %d outside the vocabulary", i, p->token_ids[i]);
  return KEEP_OK;
}

keep_status check_set(keep_ctx* c, const PromptInfo& pi, const int32_t* groups, int n_sel) {
  if (n_sel < 0 || n_sel > pi.G) return fail(c, KEEP_ERR_INVALID_ARG, "n_sel %d outside [0, n_groups]", n_sel);
  if (n_sel > 0 && !groups) return fail(c, KEEP_ERR_INVALID_ARG, "groups is NULL");
  for (int i = 0; i < n_sel; ++i) {
    if (groups[i] < 0 || groups[i] >= pi.G) return fail(c, KEEP_ERR_INVALID_ARG, "groups[%d] = %d out of range", i, groups[i]);
    if (i && groups[i] <= groups[i - 1]) return fail(c, KEEP_ERR_INVALID_ARG, "groups must be strictly ascending");
  }
  return KEEP_OK;
}

int budget_count(float ratio, int n_groups_total, int n_cand) {
  int k = (int)ceil((double)ratio * (double)n_groups_total - BUDGET_EPS);
  return std::max(0, std::min(n_cand, k));
}
int budget_tokens(float ratio, int mem_tokens) { return (int)floor((double)ratio * (double)mem_tokens + BUDGET_EPS); }

// --- typed dispatch helpers -------------------------------------------------
template <typename T>
struct Typed {
  static T* p(void* v) { return reinterpret_cast<T*>(v); }
  static const T* p(const void* v) { return reinterpret_cast<const T*>(v); }
};

keep_status upload_tokens(keep_ctx* c, const keep_prompt* p, const PromptInfo& pi) {
  // token ids go through pinned memory so the async copy does not read caller memory later
  if (c->tok_pending) HIP_TRY(c, hipEventSynchronize(c->ev_tok));
  memcpy(c->h_token_ids, p->token_ids, (size_t)pi.N * sizeof(int32_t));
  HIP_TRY(c, hipMemcpyAsync(c->d_token_ids, c->h_token_ids, (size_t)pi.N * sizeof(int32_t), hipMemcpyHostToDevice,
                            c->s_comp));
  HIP_TRY(c, hipEventRecord(c->ev_tok, c->s_comp));
  c->tok_pending = true;
  return KEEP_OK;
}

struct LayerPlan {
  int m = 0, n_rows = 0, n_realign_rows = 0, n_segs = 0;
  std::vector<int32_t> row_start;  // m+2
};

// Fill the layer's staging slot (set offsets, compact row starts, re-align segments) and
// enqueue its upload on the compute stream.
keep_status stage_layer(keep_ctx* c, const keep_prompt* p, const PromptInfo& pi, int layer, const int32_t* groups,
                        int m, const void* k_cache_l, const void* v_cache_l, bool blocks_at_dst, LayerPlan* plan) {
  Staging& st = c->stage[layer];
  if (st.used) HIP_TRY(c, hipEventSynchronize(st.done));
  plan->m = m;
  plan->row_start.assign(m + 2, 0);
  int acc = 0;
  for (int i = 0; i < m; ++i) {
    st.set_off[i] = pi.off[groups[i]];
    st.cand_len[i] = p->group_len[groups[i]];
    st.row_start[i] = acc;
    plan->row_start[i] = acc;
    acc += p->group_len[groups[i]];
  }
  st.row_start[m] = plan->row_start[m] = acc;
  acc += pi.Lq;
  st.row_start[m + 1] = plan->row_start[m + 1] = acc;
  plan->n_rows = acc;
  // groups outside the set: re-align segments
  const size_t row_bytes = (size_t)c->d.n_kv_heads * c->d.head_dim * c->esz;
  int ns = 0, rows = 0, gi = 0;
  for (int g = 0; g < pi.G; ++g) {
    if (gi < m && groups[gi] == g) {
      ++gi;
      continue;
    }
    RealignSeg& sg = st.segs[ns++];
    if (blocks_at_dst) {
      sg.k_src = (const char*)k_cache_l + (size_t)pi.off[g] * row_bytes;
      sg.v_src = (const char*)v_cache_l + (size_t)pi.off[g] * row_bytes;
    } else {
      sg.k_src = p->k_blocks[(size_t)layer * pi.G + g];
      sg.v_src = p->v_blocks[(size_t)layer * pi.G + g];
      if (!sg.k_src || !sg.v_src)
        return fail(c, KEEP_ERR_INVALID_ARG, "k_blocks/v_blocks entry of layer %d group %d is NULL", layer, g);
    }
    sg.dst_off = pi.off[g];
    sg.len = p->group_len[g];
    sg.row_start = rows;
    sg.pad = 0;
    rows += sg.len;
  }
  plan->n_segs = ns;
  plan->n_realign_rows = rows;
  hipStream_t s = c->s_comp;
  // one upload: the three int arrays and the segments that are in use
  const size_t G_cap = (size_t)std::max(1, c->d.max_groups);
  HIP_TRY(c, hipMemcpyAsync(c->d_set_off, st.set_off, table_seg_offset_ints(G_cap) * 4 + (size_t)ns * sizeof(RealignSeg),
                            hipMemcpyHostToDevice, s));
  return KEEP_OK;
}

// Steps of one layer on the compute stream, up to and including attention.
template <typename T>
keep_status layer_front(keep_ctx* c, const PromptInfo& pi, int layer, const LayerPlan& plan, const void* x_in,
                        void* k_cache_l, void* v_cache_l, hipEvent_t* evs, bool skip_attention = false) {
  const keep_model_desc& d = c->d;
  const keep_layer_weights& w = c->w[layer];
  hipStream_t s = c->s_comp;
  const int n = plan.n_rows;
  if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[0], s));
  launch_realign<T>(c->d_segs, plan.n_segs, plan.n_realign_rows, d.n_kv_heads, d.head_dim, c->rope_cos, c->rope_sin,
                    Typed<T>::p(k_cache_l), Typed<T>::p(v_cache_l), s);
  if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[1], s));
  launch_build_rows(c->d_set_off, c->d_row_start, plan.m, pi.n_mem, n, c->d_row_pos, c->d_row_slot, s);
  const T* x = Typed<T>::p(x_in);
  if (!x) {
    launch_embed_gather<T>(Typed<T>::p(c->embed), c->d_token_ids, c->d_row_pos, n, d.hidden, Typed<T>::p(c->xa), s);
    x = Typed<T>::p(c->xa);
  }
  launch_rmsnorm<T>(x, Typed<T>::p(w.ln1), n, d.hidden, d.rms_eps, Typed<T>::p(c->hbuf), s);
  if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[2], s));
  GemmB b{};
  b.n_parts = 3;
  b.ptr[0] = w.wq; b.ptr[1] = w.wk; b.ptr[2] = w.wv;
  b.bias[0] = w.bq; b.bias[1] = w.bk; b.bias[2] = w.bv;
  b.n_rows[0] = d.n_q_heads * d.head_dim;
  b.n_rows[1] = b.n_rows[2] = d.n_kv_heads * d.head_dim;
  if (!c->w4.empty()) {
    set_w4(b, 0, c->w4[layer].wq);
    set_w4(b, 1, c->w4[layer].wk);
    set_w4(b, 2, c->w4[layer].wv);
  }
  const int n_qkv = b.n_rows[0] + 2 * b.n_rows[1];
  if (c->mfma && gemm_mfma_fuses_qkv(n, d.hidden, b, n_qkv, c->skinny_ws != nullptr)) {
    // bias, RoPE, the compact q / k rows and the scatter of K and V into the cache are the projection's epilogue
    QkvEpilogue qe{};
    qe.row_pos = c->d_row_pos;
    qe.row_lo = c->units_mode ? c->d_row_lo : nullptr;
    qe.rope_cos = c->rope_cos;
    qe.rope_sin = c->rope_sin;
    qe.bias[0] = w.bq; qe.bias[1] = w.bk; qe.bias[2] = w.bv;
    qe.q = c->q;
    qe.k_compact = c->kc;
    qe.k_cache = k_cache_l;
    qe.v_cache = v_cache_l;
    qe.q_dim = b.n_rows[0];
    qe.kv_dim = b.n_rows[1];
    launch_gemm_mfma(reinterpret_cast<const bf16_t*>(c->hbuf), n, d.hidden, b, nullptr, n_qkv, EPI_QKV_ROPE, nullptr,
                     nullptr, s, c->skinny_ws, &qe);
    if (evs && !c->ev_light) {
      HIP_TRY(c, hipEventRecord(evs[3], s));
      HIP_TRY(c, hipEventRecord(evs[4], s));
    }
  } else {
    if (c->mfma)
      launch_gemm_mfma(reinterpret_cast<const bf16_t*>(c->hbuf), n, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32, nullptr,
                       c->qkv_raw, s, c->skinny_ws);
    else
      launch_gemm_generic<T>(Typed<T>::p(c->hbuf), n, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32, nullptr, c->qkv_raw, s);
    if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[3], s));
    launch_rope_scatter<T>(c->qkv_raw, Typed<T>::p(w.bq), Typed<T>::p(w.bk), Typed<T>::p(w.bv), c->d_row_pos, n,
                           d.n_q_heads, d.n_kv_heads, d.head_dim, c->rope_cos, c->rope_sin, Typed<T>::p(c->q),
                           Typed<T>::p(c->kc), Typed<T>::p(k_cache_l), Typed<T>::p(v_cache_l), s,
                           c->units_mode ? c->d_row_lo : nullptr);
    if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[4], s));
  }
  if (skip_attention) {  // the caller attends the rows as they turn out to be needed
    if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[5], s));
    HIP_TRY(c, hipGetLastError());
    return KEEP_OK;
  }
  if (c->mfma)
  {
    const int32_t* set_off = c->stage[layer].set_off;
    const bool same = c->att_plan.valid && !c->units_mode && c->att_plan_n_mem == pi.n_mem &&
                      c->att_plan_row_start == plan.row_start && (int)c->att_plan_set_off.size() == plan.m &&
                      std::equal(set_off, set_off + plan.m, c->att_plan_set_off.begin());
    if (!same) {
      c->att_plan.valid = false;
      c->att_plan_row_start = plan.row_start;
      c->att_plan_set_off.assign(set_off, set_off + plan.m);
      c->att_plan_n_mem = pi.n_mem;
    }
    launch_attn_mfma(reinterpret_cast<const bf16_t*>(c->q), reinterpret_cast<const bf16_t*>(k_cache_l),
                     reinterpret_cast<const bf16_t*>(v_cache_l), c->d_row_pos, plan.row_start.data(), set_off, plan.m,
                     pi.n_mem, n, pi.N, d.n_q_heads, d.n_kv_heads, d.max_tokens, c->stage[layer].attn_items,
                     c->attn_scratch, reinterpret_cast<bf16_t*>(c->o), c->lse, s, c->units_mode ? c->h_row_lo : nullptr,
                     c->units_mode ? c->d_row_lo : nullptr, c->units_mode ? nullptr : &c->att_plan);
    if (c->units_mode) c->att_plan.valid = false;
  } else
    launch_attn_generic<T>(Typed<T>::p(c->q), Typed<T>::p(k_cache_l), Typed<T>::p(v_cache_l), c->d_row_pos, n,
                           d.n_q_heads, d.n_kv_heads, d.head_dim, Typed<T>::p(c->o), c->lse, s,
                           c->units_mode ? c->d_row_lo : nullptr);
  if (evs && !c->ev_light) HIP_TRY(c, hipEventRecord(evs[5], s));
  HIP_TRY(c, hipGetLastError());
  return KEEP_OK;
}

// Attention of the rows of the flagged blocks only (blocks 0..m-1 the layer's memories, m the instruction),
// on the compute stream; MFMA family.  No earlier upload from h_row_list that is
// still pending is overwritten (it waits for that upload's event).  rows_out / keys_out: how many rows were attended and how many keys they see in all.
keep_status attend_blocks(keep_ctx* c, const PromptInfo& pi, int layer, const LayerPlan& plan, const uint8_t* flags,
                          void* k_cache_l, void* v_cache_l, hipEvent_t ev_begin, hipEvent_t ev_end, int* rows_out,
                          uint64_t* keys_out) {
  const keep_model_desc& d = c->d;
  hipStream_t s = c->s_comp;
  int n = 0;
  uint64_t keys = 0;
  // the pinned list is about to be rewritten: the previous upload from it must have been read
  if (c->rowlist_pending) {
    HIP_TRY(c, hipEventSynchronize(c->ev_rowlist));
    c->rowlist_pending = false;
  }
  for (int a = 0; a <= plan.m; ++a)
    if (flags[a]) {
      const int64_t first = a < plan.m ? c->stage[layer].set_off[a] : pi.n_mem;  // position of the block's first row
      const int64_t len = plan.row_start[a + 1] - plan.row_start[a];
      keys += (uint64_t)(len * (2 * first + len + 1) / 2);
      for (int r = plan.row_start[a]; r < plan.row_start[a + 1]; ++r) c->h_row_list[n++] = r;
    }
  *rows_out = n;
  *keys_out = keys;
  if (n == 0) return KEEP_OK;
  c->att_plan.valid = false;  // this launch's work list replaces the one in attn_scratch
  HIP_TRY(c, hipMemcpyAsync(c->d_row_list, c->h_row_list, (size_t)n * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipEventRecord(c->ev_rowlist, s));
  c->rowlist_pending = true;
  if (ev_begin) HIP_TRY(c, hipEventRecord(ev_begin, s));
  launch_attn_mfma(reinterpret_cast<const bf16_t*>(c->q), reinterpret_cast<const bf16_t*>(k_cache_l),
                   reinterpret_cast<const bf16_t*>(v_cache_l), c->d_row_pos, plan.row_start.data(),
                   c->stage[layer].set_off, plan.m, pi.n_mem, plan.n_rows, pi.N, d.n_q_heads, d.n_kv_heads, d.max_tokens,
                   c->stage[layer].attn_items, c->attn_scratch, reinterpret_cast<bf16_t*>(c->o), c->lse, s, nullptr,
                   nullptr, nullptr, c->h_row_list, c->d_row_list, n);
  if (ev_end) HIP_TRY(c, hipEventRecord(ev_end, s));
  HIP_TRY(c, hipGetLastError());
  return KEEP_OK;
}

// Output projection + residual, RMSNorm, SwiGLU FFN + residual on the compute stream.
template <typename T>
keep_status layer_back(keep_ctx* c, int layer, int n, const void* o_rows, const void* x_in, void* x_out,
                       hipEvent_t* evs) {
  const keep_model_desc& d = c->d;
  const keep_layer_weights& w = c->w[layer];
  hipStream_t s = c->s_comp;
  const int qd = d.n_q_heads * d.head_dim;
  GemmB bo{}; bo.n_parts = 1; bo.ptr[0] = w.wo; bo.n_rows[0] = d.hidden;
  GemmB bg{}; bg.n_parts = 1; bg.ptr[0] = w.wgate; bg.n_rows[0] = d.ffn_dim;
  GemmB bd{}; bd.n_parts = 1; bd.ptr[0] = w.wdown; bd.n_rows[0] = d.hidden;
  if (!c->w4.empty()) {
    set_w4(bo, 0, c->w4[layer].wo);
    set_w4(bg, 0, c->w4[layer].wgate);
    set_w4_b2(bg, c->w4[layer].wup);
    set_w4(bd, 0, c->w4[layer].wdown);
  }
#define EV(i) \
  if (evs && (!c->ev_light || (i) == 7 || (i) == 8)) HIP_TRY(c, hipEventRecord(evs[i], s))
  EV(12);
  if (c->mfma) {
    auto B = [](const void* p) { return reinterpret_cast<const bf16_t*>(p); };
    launch_gemm_mfma(B(o_rows), n, qd, bo, nullptr, d.hidden, EPI_RESIDUAL_STORE, B(x_in), c->x1, s, c->skinny_ws);
    EV(6);
    launch_rmsnorm<bf16_t>(B(c->x1), B(w.ln2), n, d.hidden, d.rms_eps, reinterpret_cast<bf16_t*>(c->hbuf), s);
    EV(7);
    launch_gemm_mfma(B(c->hbuf), n, d.hidden, bg, w.wup, d.ffn_dim, EPI_SWIGLU_STORE, nullptr, c->act, s, c->skinny_ws);
    EV(8);
    launch_gemm_mfma(B(c->act), n, d.ffn_dim, bd, nullptr, d.hidden, EPI_RESIDUAL_STORE, B(c->x1), x_out, s, c->skinny_ws);
  } else {
    launch_gemm_generic<T>(Typed<T>::p(o_rows), n, qd, bo, nullptr, d.hidden, EPI_RESIDUAL_STORE, Typed<T>::p(x_in),
                           c->x1, s);
    EV(6);
    launch_rmsnorm<T>(Typed<T>::p(c->x1), Typed<T>::p(w.ln2), n, d.hidden, d.rms_eps, Typed<T>::p(c->hbuf), s);
    EV(7);
    launch_gemm_generic<T>(Typed<T>::p(c->hbuf), n, d.hidden, bg, w.wup, d.ffn_dim, EPI_SWIGLU_STORE, nullptr, c->act,
                           s);
    EV(8);
    launch_gemm_generic<T>(Typed<T>::p(c->act), n, d.ffn_dim, bd, nullptr, d.hidden, EPI_RESIDUAL_STORE,
                           Typed<T>::p(c->x1), x_out, s);
  }
  EV(9);
#undef EV
  HIP_TRY(c, hipGetLastError());
  return KEEP_OK;
}

// Score matrix of the layer whose q / k / lse are in the workspace, on stream s.
// h_want (MFMA family only): flags of the source blocks whose rows of S are wanted, NULL = all.
template <typename T>
keep_status score_matrix(keep_ctx* c, int layer, const LayerPlan& plan, hipStream_t s, const uint8_t* h_want = nullptr) {
  const keep_model_desc& d = c->d;
  if (plan.m == 0) return KEEP_OK;
  if (c->mfma) {
    launch_score_mfma(reinterpret_cast<const bf16_t*>(c->q), reinterpret_cast<const bf16_t*>(c->kc), c->lse,
                      plan.row_start.data(), c->d_row_start, plan.m, plan.n_rows, d.n_q_heads, d.n_kv_heads,
                      c->stage[layer].score_tiles, c->score_scratch, d.max_tokens, std::max(1, d.max_groups), c->S, s,
                      h_want);
  } else {
    launch_score_rows_generic<T>(Typed<T>::p(c->q), Typed<T>::p(c->kc), c->lse, c->d_row_start, plan.m, plan.n_rows,
                                 d.n_q_heads, d.n_kv_heads, d.head_dim, c->score_scratch, s);
    launch_score_finish(c->score_scratch, c->d_row_start, plan.m, d.n_q_heads, c->S, s);
  }
  HIP_TRY(c, hipGetLastError());
  return KEEP_OK;
}

// Decide the next set.  Returns immediately (no device work) when the budget takes all
// or none of the candidates.  Otherwise enqueues the selection on stream s and the
// read-back of its result into c->h_sel_out; the caller waits and calls finish_select.
enum SelectKind { SEL_ALL, SEL_NONE, SEL_DEVICE };
constexpr int LAZY_MIN_CANDIDATES = 64;  // below this the whole score matrix is cheap
SelectKind classify_budget(const PromptInfo& pi, const keep_prompt* p, const int32_t* groups, int m, float ratio,
                           int mode, int* k_count, int* tok_budget) {
  *k_count = budget_count(ratio, pi.G, m);
  *tok_budget = budget_tokens(ratio, pi.n_mem);
  if (m == 0) return SEL_NONE;
  if (mode == KEEP_BUDGET_GROUP_COUNT) {
    if (*k_count >= m) return SEL_ALL;
    if (*k_count == 0) return SEL_NONE;
  } else {
    int64_t tot = 0;
    for (int i = 0; i < m; ++i) tot += p->group_len[groups[i]];
    if (*tok_budget >= tot) return SEL_ALL;
    if (*tok_budget <= 0) return SEL_NONE;
  }
  return SEL_DEVICE;
}

keep_status enqueue_select(keep_ctx* c, int m, int k_count, int tok_budget, int mode, int hops, hipStream_t s) {
  launch_select(c->S, m, c->d_cand_len, k_count, tok_budget, mode, hops, c->sel_work, c->sel_iwork, c->sel_out, s,
                c->set_only);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipMemcpyAsync(c->h_sel_out, c->sel_out, (size_t)(m + 2) * 4, hipMemcpyDeviceToHost, s));
  return KEEP_OK;
}

template <typename F>
keep_status by_dtype(keep_ctx* c, F&& f) {
  return c->d.dtype == KEEP_BF16 ? f((bf16_t*)nullptr) : f((float*)nullptr);
}


// Greedy decoding of n_new tokens over the joined cache.  The whole chain is enqueued on the compute
// stream without a host round trip: each token id stays on the device (argmax output -> embedding gather).
// For the attention the new token is a one-row "instruction" behind n_ctx + t - 1 cached tokens.
template <typename T>
keep_status decode_impl(keep_ctx* c, const void* final_norm, const void* lm_head, const void* x_last, void* k_cache,
                        void* v_cache, int32_t cache_rows, int32_t n_ctx, int32_t n_new, int32_t* tokens_out,
                        float* logits_out, const int32_t* forced_tokens) {
  const keep_model_desc& d = c->d;
  hipStream_t s = c->s_comp;
  constexpr int CAP = KEEP_DECODE_MAX_TOKENS;
  // pinned / device ints: [0, CAP) positions, [CAP, 2 CAP) fed tokens (forced), [2 CAP, 3 CAP) results, [3 CAP] zero
  int32_t* h = c->h_dec;
  for (int t = 0; t < CAP; ++t) {
    h[t] = n_ctx + t;
    h[CAP + t] = (forced_tokens && t + 1 < n_new) ? forced_tokens[t] : 0;
    h[2 * CAP + t] = 0;
  }
  h[3 * CAP] = 0;
  HIP_TRY(c, hipMemcpyAsync(c->d_dec, h, (size_t)(3 * CAP + 1) * 4, hipMemcpyHostToDevice, s));
  const size_t row_bytes = (size_t)d.n_kv_heads * d.head_dim * c->esz;
  const size_t layer_bytes = (size_t)cache_rows * row_bytes;
  GemmB bh{};
  bh.n_parts = 1;
  bh.ptr[0] = lm_head;
  bh.n_rows[0] = d.vocab;
  PromptInfo pi;
  pi.G = 0;
  pi.Lq = 1;
  pi.off.assign(1, 0);
  LayerPlan plan;
  plan.m = 0;
  plan.n_rows = 1;
  plan.row_start = {0, 1};
  const void* x = x_last;
  AttnPlan att_plan;
  c->att_plan.valid = false;  // the decode steps put their own work lists into attn_scratch
  for (int t = 0; t < n_new; ++t) {
    // vocabulary projection of the newest hidden row, greedy choice
    float* lg = logits_out ? logits_out + (size_t)t * d.vocab : c->dec_logits;
    launch_rmsnorm<T>(Typed<T>::p(x), Typed<T>::p(final_norm), 1, d.hidden, d.rms_eps, Typed<T>::p(c->hbuf), s);
    if (c->mfma)
      launch_gemm_mfma(reinterpret_cast<const bf16_t*>(c->hbuf), 1, d.hidden, bh, nullptr, d.vocab, EPI_STORE_F32,
                       nullptr, lg, s, c->skinny_ws);
    else
      launch_gemm_generic<T>(Typed<T>::p(c->hbuf), 1, d.hidden, bh, nullptr, d.vocab, EPI_STORE_F32, nullptr, lg, s);
    launch_argmax(lg, d.vocab, c->d_dec + 2 * CAP + t, s);
    HIP_TRY(c, hipGetLastError());
    if (t + 1 == n_new) break;
    // the chosen (or forced) token at position n_ctx + t through every layer
    const int32_t* d_tok = c->d_dec + (forced_tokens ? CAP : 2 * CAP) + t;
    const int32_t* d_pos = c->d_dec + t;
    pi.n_mem = n_ctx + t;
    pi.N = n_ctx + t + 1;
    launch_embed_gather<T>(Typed<T>::p(c->embed), d_tok, c->d_dec + 3 * CAP, 1, d.hidden, Typed<T>::p(c->xa), s);
    void* x_cur = c->xa;
    void* x_nxt = c->xb;
    for (int l = 0; l < d.n_layers; ++l) {
      const keep_layer_weights& w = c->w[l];
      char* kl = (char*)k_cache + (size_t)l * layer_bytes;
      char* vl = (char*)v_cache + (size_t)l * layer_bytes;
      // The work list of the attention depends on the position only: layer 0 of the step plans and uploads
      // it (through staging slot t % n_layers, free again once its event has fired), the other layers reuse it.
      Staging& sg = c->stage[t % d.n_layers];
      if (l == 0) {
        if (sg.used) HIP_TRY(c, hipEventSynchronize(sg.done));
        att_plan.valid = false;
      }
      launch_rmsnorm<T>(Typed<T>::p(x_cur), Typed<T>::p(w.ln1), 1, d.hidden, d.rms_eps, Typed<T>::p(c->hbuf), s);
      GemmB b{};
      b.n_parts = 3;
      b.ptr[0] = w.wq; b.ptr[1] = w.wk; b.ptr[2] = w.wv;
      b.bias[0] = w.bq; b.bias[1] = w.bk; b.bias[2] = w.bv;
      b.n_rows[0] = d.n_q_heads * d.head_dim;
      b.n_rows[1] = b.n_rows[2] = d.n_kv_heads * d.head_dim;
      if (!c->w4.empty()) {
        set_w4(b, 0, c->w4[l].wq);
        set_w4(b, 1, c->w4[l].wk);
        set_w4(b, 2, c->w4[l].wv);
      }
      const int n_qkv = b.n_rows[0] + 2 * b.n_rows[1];
      if (c->mfma)
        launch_gemm_mfma(reinterpret_cast<const bf16_t*>(c->hbuf), 1, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32,
                         nullptr, c->qkv_raw, s, c->skinny_ws);
      else
        launch_gemm_generic<T>(Typed<T>::p(c->hbuf), 1, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32, nullptr, c->qkv_raw, s);
      launch_rope_scatter<T>(c->qkv_raw, Typed<T>::p(w.bq), Typed<T>::p(w.bk), Typed<T>::p(w.bv), d_pos, 1, d.n_q_heads,
                             d.n_kv_heads, d.head_dim, c->rope_cos, c->rope_sin, Typed<T>::p(c->q), Typed<T>::p(c->kc),
                             Typed<T>::p(kl), Typed<T>::p(vl), s);
      if (c->mfma)
        launch_attn_mfma(reinterpret_cast<const bf16_t*>(c->q), reinterpret_cast<const bf16_t*>(kl),
                         reinterpret_cast<const bf16_t*>(vl), d_pos, plan.row_start.data(), sg.set_off, 0, pi.n_mem, 1,
                         pi.N, d.n_q_heads, d.n_kv_heads, d.max_tokens, sg.attn_items, c->attn_scratch,
                         reinterpret_cast<bf16_t*>(c->o), c->lse, s, nullptr, nullptr, &att_plan);
      else
        launch_attn_generic<T>(Typed<T>::p(c->q), Typed<T>::p(kl), Typed<T>::p(vl), d_pos, 1, d.n_q_heads, d.n_kv_heads,
                               d.head_dim, Typed<T>::p(c->o), c->lse, s);
      HIP_TRY(c, hipGetLastError());
      if (l == 0) {
        HIP_TRY(c, hipEventRecord(sg.done, s));
        sg.used = true;
      }
      keep_status st = layer_back<T>(c, l, 1, c->o, x_cur, x_nxt, nullptr);
      if (st != KEEP_OK) return st;
      std::swap(x_cur, x_nxt);
    }
    x = x_cur;
  }
  HIP_TRY(c, hipMemcpyAsync(h + 2 * CAP, c->d_dec + 2 * CAP, (size_t)n_new * 4, hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  for (int t = 0; t < n_new; ++t) tokens_out[t] = h[2 * CAP + t];
  return KEEP_OK;
}

}  // namespace

// ===========================================================================
// public functions
// ===========================================================================
namespace {
keep_status prefill_impl(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t hops, int32_t budget_mode,
                         int32_t load_mode, void* k_cache, void* v_cache, int32_t cache_rows, void* x_final,
                         int32_t* sel_groups, int32_t* sel_counts, keep_report* report);
template <typename T>
keep_status prefill_tokens_impl(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t load_mode, void* k_cache,
                                void* v_cache, void* x_final, int32_t* sel_rows, int32_t* sel_counts,
                                float* deviation_out, keep_report* report);
}  // namespace

extern "C" {

const char* keep_last_error(const keep_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

int32_t keep_uses_mfma(const keep_ctx* ctx) { return ctx ? (ctx->mfma ? 1 : 0) : -1; }

uint64_t keep_workspace_bytes(const keep_model_desc* desc) {
  const char* why;
  if (check_desc(desc, &why) != KEEP_OK) return 0;
  return workspace_bytes(desc);
}

keep_status keep_destroy(keep_ctx* c) {
  if (!c) return KEEP_OK;
  (void)hipStreamSynchronize(c->s_comp);
  (void)hipStreamSynchronize(c->s_eval);
  (void)hipStreamSynchronize(c->s_copy);
  for (void* p : c->allocs) (void)hipFree(p);
  for (Staging& st : c->stage) {
    if (st.set_off) (void)hipHostFree(st.set_off);  // the block also holds cand_len, row_start and segs
    if (st.gather_src) (void)hipHostFree(st.gather_src);
    if (st.gather_dst) (void)hipHostFree(st.gather_dst);
    if (st.score_tiles) (void)hipHostFree(st.score_tiles);
    if (st.attn_items) (void)hipHostFree(st.attn_items);
    if (st.done) (void)hipEventDestroy(st.done);
  }
  if (c->h_sel_out) (void)hipHostFree(c->h_sel_out);
  if (c->h_dec) (void)hipHostFree(c->h_dec);
  if (c->h_row_lo) (void)hipHostFree(c->h_row_lo);
  if (c->h_row_list) (void)hipHostFree(c->h_row_list);
  if (c->h_tok_list) (void)hipHostFree(c->h_tok_list);
  if (c->h_dev) (void)hipHostFree(c->h_dev);
  for (hipEvent_t e : c->ev_part)
    if (e) (void)hipEventDestroy(e);
  if (c->h_S) (void)hipHostFree(c->h_S);
  if (c->h_token_ids) (void)hipHostFree(c->h_token_ids);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_chunk) (void)hipEventDestroy(e);
  for (hipEvent_t e : {c->ev_attn, c->ev_eval, c->ev_load, c->ev_comp, c->ev_tok, c->ev_rowlist})
    if (e) (void)hipEventDestroy(e);
  delete c;
  return KEEP_OK;
}

keep_status keep_init(const keep_model_desc* desc, const keep_layer_weights* layers, const void* embed_table,
                      void* stream_compute, void* stream_eval, void* stream_copy, keep_ctx** out) {
  if (!out) return fail(nullptr, KEEP_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  const char* why;
  keep_status st = check_desc(desc, &why);
  if (st != KEEP_OK) return fail(nullptr, st, "%s", why);
  if (!layers || !embed_table) return fail(nullptr, KEEP_ERR_INVALID_ARG, "layers or embed_table is NULL");
  for (int l = 0; l < desc->n_layers; ++l) {
    const keep_layer_weights& w = layers[l];
    if (!w.ln1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.ln2 || !w.wgate || !w.wup || !w.wdown)
      return fail(nullptr, KEEP_ERR_INVALID_ARG, "a weight pointer of layer %d is NULL", l);
  }
  int n_dev = 0;
  hipError_t he = hipGetDeviceCount(&n_dev);
  if (he != hipSuccess || n_dev < 1)
    return fail(nullptr, KEEP_ERR_HIP, "no HIP device available (%s)", hipGetErrorString(he));

  keep_ctx* c = new keep_ctx();
  c->d = *desc;
  c->w.assign(layers, layers + desc->n_layers);
  c->embed = embed_table;
  c->s_comp = (hipStream_t)stream_compute;
  c->s_eval = (hipStream_t)stream_eval;
  c->s_copy = (hipStream_t)stream_copy;
  c->mfma = wants_mfma(desc);
  c->esz = desc->dtype == KEEP_BF16 ? 2 : 4;
  const Sizes z = sizes_of(desc);
  const size_t half = (size_t)desc->head_dim / 2;

#define TRY_INIT(expr)                       \
  do {                                       \
    keep_status s__ = (expr);                \
    if (s__ != KEEP_OK) {                    \
      g_init_error = c->err;                 \
      keep_destroy(c);                       \
      return s__;                            \
    }                                        \
  } while (0)

  TRY_INIT(dev_alloc(c, &c->rope_cos, z.M * half * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->rope_sin, z.M * half * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->d_token_ids, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_row_pos, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_row_slot, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_set_off, table_block_bytes(z.G)));
  c->d_cand_len = c->d_set_off + (z.G + 2);
  c->d_row_start = c->d_cand_len + (z.G + 2);
  c->d_segs = reinterpret_cast<RealignSeg*>(c->d_set_off + table_seg_offset_ints(z.G));
  TRY_INIT(dev_alloc(c, &c->d_gather_src, (z.G + 2) * 4));
  TRY_INIT(dev_alloc(c, &c->xa, z.M * z.d * z.esz));
  TRY_INIT(dev_alloc(c, &c->xb, z.M * z.d * z.esz));
  TRY_INIT(dev_alloc(c, &c->hbuf, z.M * z.d * z.esz));
  TRY_INIT(dev_alloc(c, &c->x1, z.M * z.d * z.esz));
  TRY_INIT(dev_alloc(c, &c->q, z.M * z.qd * z.esz));
  TRY_INIT(dev_alloc(c, &c->o, z.M * z.qd * z.esz));
  TRY_INIT(dev_alloc(c, &c->kc, z.M * z.kvd * z.esz));
  TRY_INIT(dev_alloc(c, &c->act, z.M * z.F * z.esz));
  TRY_INIT(dev_alloc(c, &c->qkv_raw, z.M * (z.qd + 2 * z.kvd) * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->lse, z.M * (size_t)desc->n_q_heads * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->score_scratch, score_scratch_bytes(desc)));
  if (c->mfma) {
    TRY_INIT(dev_alloc(c, reinterpret_cast<char**>(&c->attn_scratch),
                       attn_mfma_scratch_bytes((int32_t)z.M, desc->n_q_heads, desc->n_kv_heads)));
    TRY_INIT(dev_alloc(c, reinterpret_cast<char**>(&c->skinny_ws), gemm_ws_bytes()));
  }
  TRY_INIT(dev_alloc(c, &c->S, (z.G + 1) * z.G * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->sel_work, ((z.G + 1) * z.G + 2 * z.G) * sizeof(float)));
  TRY_INIT(dev_alloc(c, &c->sel_iwork, 4 * z.G * 4));
  TRY_INIT(dev_alloc(c, &c->sel_out, (z.G + 2) * 4));

  // RoPE table: angle = position * theta^(-2j/head_dim), evaluated in double, stored fp32
  {
    std::vector<float> hc(z.M * half), hs(z.M * half);
    std::vector<double> freq(half);
    for (size_t j = 0; j < half; ++j) freq[j] = pow((double)desc->rope_theta, -2.0 * (double)j / (double)desc->head_dim);
    for (size_t p = 0; p < z.M; ++p)
      for (size_t j = 0; j < half; ++j) {
        const double a = (double)p * freq[j];
        hc[p * half + j] = (float)cos(a);
        hs[p * half + j] = (float)sin(a);
      }
    auto up = [&](float* dst, const std::vector<float>& src) -> keep_status {
      HIP_TRY(c, hipMemcpy(dst, src.data(), src.size() * sizeof(float), hipMemcpyHostToDevice));
      return KEEP_OK;
    };
    TRY_INIT(up(c->rope_cos, hc));
    TRY_INIT(up(c->rope_sin, hs));
  }

  c->stage.resize(desc->n_layers);
  for (Staging& sg : c->stage) {
    sg = Staging{};
    // set_off | cand_len | row_start | segs share one block, mirrored on the device: one upload per layer
    TRY_INIT(pin_alloc(c, &sg.set_off, table_block_bytes(z.G)));
    sg.cand_len = sg.set_off + (z.G + 2);
    sg.row_start = sg.cand_len + (z.G + 2);
    sg.segs = reinterpret_cast<RealignSeg*>(sg.set_off + table_seg_offset_ints(z.G));
    TRY_INIT(pin_alloc(c, &sg.gather_src, (z.G + 2) * 4));
    TRY_INIT(pin_alloc(c, &sg.gather_dst, (z.G + 2) * 4));
    if (c->mfma) {
      TRY_INIT(pin_alloc(c, &sg.score_tiles, score_mfma_stage_ints((int32_t)z.M, (int32_t)z.G) * 4));
      TRY_INIT(pin_alloc(c, &sg.attn_items, attn_mfma_stage_ints((int32_t)z.M, desc->n_q_heads, desc->n_kv_heads) * 4));
    }
    auto mk = [&]() -> keep_status {
      HIP_TRY(c, hipEventCreateWithFlags(&sg.done, hipEventDisableTiming));
      return KEEP_OK;
    };
    TRY_INIT(mk());
  }
  TRY_INIT(pin_alloc(c, &c->h_sel_out, (z.G + 2) * 4));
  TRY_INIT(pin_alloc(c, &c->h_dec, 4 * KEEP_DECODE_MAX_TOKENS * 4));
  TRY_INIT(pin_alloc(c, &c->h_row_lo, z.M * 4));
  TRY_INIT(pin_alloc(c, &c->h_row_list, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_row_list, z.M * 4));
  {
    auto mk = [&]() -> keep_status {
      for (hipEvent_t& e : c->ev_part) HIP_TRY(c, hipEventCreate(&e));
      return KEEP_OK;
    };
    TRY_INIT(mk());
  }
  TRY_INIT(dev_alloc(c, &c->d_row_lo, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_dev, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_tok_flags, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_tok_list, z.M * 4));
  TRY_INIT(pin_alloc(c, &c->h_tok_list, z.M * 4));
  TRY_INIT(pin_alloc(c, &c->h_dev, z.M * 4));
  TRY_INIT(dev_alloc(c, &c->d_dec, 4 * KEEP_DECODE_MAX_TOKENS * 4));
  TRY_INIT(dev_alloc(c, &c->dec_logits, (size_t)desc->vocab * sizeof(float)));
  TRY_INIT(pin_alloc(c, &c->h_S, (z.G + 1) * z.G * sizeof(float)));
  TRY_INIT(pin_alloc(c, &c->h_token_ids, z.M * 4));
  auto mk_events = [&]() -> keep_status {
    c->ev.resize((size_t)desc->n_layers * EV_PER_LAYER);
    for (hipEvent_t& e : c->ev) HIP_TRY(c, hipEventCreate(&e));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_attn, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_eval, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_load, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_comp, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_tok, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_rowlist, hipEventDisableTiming));
    c->ev_chunk.resize(64);
    for (hipEvent_t& e : c->ev_chunk) HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    return KEEP_OK;
  };
  TRY_INIT(mk_events());
#undef TRY_INIT
  *out = c;
  return KEEP_OK;
}

// ---------------------------------------------------------------------------
// host->device copies of group blocks (Section 5, load_memory)
// ---------------------------------------------------------------------------
namespace {
struct Loader {
  keep_ctx* c;
  const keep_prompt* p;
  const PromptInfo* pi;
  char* k_cache;
  char* v_cache;
  size_t row_bytes, layer_bytes;
  std::vector<uint8_t> loaded;  // [L * G]
  size_t inflight_head = 0, inflight_tail = 0;  // ring of chunk events
  std::vector<size_t> chunk_bytes;
  size_t inflight = 0;
  uint64_t bytes_total = 0;

  // Copy the blocks of groups [g0, g1) of one layer.  Consecutive groups are consecutive rows of the
  // cache; when their host blocks are consecutive in host memory too (one pinned slab per layer, the
  // usual case), the run goes out as ONE copy for K and one for V instead of two per group.
  static constexpr size_t MAX_RUN_BYTES = 16u << 20;
  keep_status copy_run(int layer, int g0, int g1) {
    int g = g0;
    while (g < g1) {
      const size_t idx0 = (size_t)layer * pi->G + g;
      if (loaded[idx0]) {
        ++g;
        continue;
      }
      if (!p->k_blocks[idx0] || !p->v_blocks[idx0])
        return fail(c, KEEP_ERR_INVALID_ARG, "k_blocks/v_blocks entry of layer %d group %d is NULL", layer, g);
      size_t nb = (size_t)p->group_len[g] * row_bytes;
      int e = g + 1;
      while (e < g1 && nb < MAX_RUN_BYTES && !loaded[(size_t)layer * pi->G + e] &&
             (const char*)p->k_blocks[(size_t)layer * pi->G + e] == (const char*)p->k_blocks[idx0] + nb &&
             (const char*)p->v_blocks[(size_t)layer * pi->G + e] == (const char*)p->v_blocks[idx0] + nb) {
        nb += (size_t)p->group_len[e] * row_bytes;
        ++e;
      }
      const size_t dst = (size_t)layer * layer_bytes + (size_t)pi->off[g] * row_bytes;
      HIP_TRY(c, hipMemcpyAsync(k_cache + dst, p->k_blocks[idx0], nb, hipMemcpyHostToDevice, c->s_copy));
      HIP_TRY(c, hipMemcpyAsync(v_cache + dst, p->v_blocks[idx0], nb, hipMemcpyHostToDevice, c->s_copy));
      for (int i = g; i < e; ++i) loaded[(size_t)layer * pi->G + i] = 1;
      bytes_total += 2 * nb;
      // flow control bookkeeping
      const size_t slot = inflight_head % c->ev_chunk.size();
      if (inflight_head - inflight_tail == c->ev_chunk.size()) {  // ring full: retire the oldest
        HIP_TRY(c, hipEventSynchronize(c->ev_chunk[inflight_tail % c->ev_chunk.size()]));
        inflight -= chunk_bytes[inflight_tail % c->ev_chunk.size()];
        ++inflight_tail;
      }
      HIP_TRY(c, hipEventRecord(c->ev_chunk[slot], c->s_copy));
      chunk_bytes[slot] = 2 * nb;
      inflight += 2 * nb;
      ++inflight_head;
      g = e;
    }
    return KEEP_OK;
  }
  keep_status copy_group(int layer, int g) { return copy_run(layer, g, g + 1); }
  void retire() {
    while (inflight_tail < inflight_head) {
      const size_t slot = inflight_tail % c->ev_chunk.size();
      if (hipEventQuery(c->ev_chunk[slot]) != hipSuccess) break;
      inflight -= chunk_bytes[slot];
      ++inflight_tail;
    }
  }
  // every group of `layer` outside `set` (ascending) that is not loaded yet
  keep_status copy_outside(int layer, const std::vector<int32_t>& set) {
    int g = 0;
    for (size_t gi = 0; gi <= set.size(); ++gi) {
      const int stop = gi < set.size() ? set[gi] : pi->G;  // groups [g, stop) are outside the set
      if (stop > g) {
        keep_status st = copy_run(layer, g, stop);
        if (st != KEEP_OK) return st;
      }
      g = stop + 1;
    }
    return KEEP_OK;
  }
};
}  // namespace

keep_status keep_recompute_layer(keep_ctx* c, const keep_prompt* p, int32_t layer, const int32_t* groups, int32_t n_sel,
                                 const void* x_in, void* x_out, void* k_cache_l, void* v_cache_l) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (layer < 0 || layer >= c->d.n_layers) return fail(c, KEEP_ERR_INVALID_ARG, "layer %d out of range", layer);
  if (!x_out || !k_cache_l || !v_cache_l) return fail(c, KEEP_ERR_INVALID_ARG, "x_out / k_cache_l / v_cache_l is NULL");
  PromptInfo pi;
  keep_status st = check_prompt(c, p, &pi, true);
  if (st != KEEP_OK) return st;
  st = check_set(c, pi, groups, n_sel);
  if (st != KEEP_OK) return st;
  c->last_layer = -1;

  const bool host_kv = p->kv_location == KEEP_KV_PINNED_HOST;
  if (host_kv) {
    // bring the blocks of the groups outside the set to their place in the cache
    // (the caller gave this layer's slice of the cache: layer stride 0)
    Loader ld{c, p, &pi, (char*)k_cache_l, (char*)v_cache_l, (size_t)c->d.n_kv_heads * c->d.head_dim * c->esz, 0};
    ld.loaded.assign((size_t)c->d.n_layers * pi.G, 0);
    ld.chunk_bytes.assign(c->ev_chunk.size(), 0);
    std::vector<int32_t> set(groups, groups + n_sel);
    st = ld.copy_outside(layer, set);
    if (st != KEEP_OK) return st;
    HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
    HIP_TRY(c, hipStreamWaitEvent(c->s_comp, c->ev_load, 0));
  }
  st = upload_tokens(c, p, pi);
  if (st != KEEP_OK) return st;
  LayerPlan plan;
  st = stage_layer(c, p, pi, layer, groups, n_sel, k_cache_l, v_cache_l, host_kv, &plan);
  if (st != KEEP_OK) return st;
  st = by_dtype(c, [&](auto* tag) {
    using T = std::remove_pointer_t<decltype(tag)>;
    keep_status s2 = layer_front<T>(c, pi, layer, plan, x_in, k_cache_l, v_cache_l, nullptr);
    if (s2 != KEEP_OK) return s2;
    return layer_back<T>(c, layer, plan.n_rows, c->o, x_in ? x_in : c->xa, x_out, nullptr);
  });
  if (st != KEEP_OK) return st;
  Staging& sg = c->stage[layer];
  HIP_TRY(c, hipEventRecord(sg.done, c->s_comp));
  sg.used = true;
  c->last_layer = layer;
  c->last_groups.assign(groups, groups + n_sel);
  c->last_row_start = plan.row_start;
  c->last_n_rows = plan.n_rows;
  return KEEP_OK;
}

keep_status keep_score_groups(keep_ctx* c, const keep_prompt* p, int32_t layer, const int32_t* groups, int32_t n_sel,
                              float ratio_next, int32_t hops, int32_t budget_mode, float* S_out, int32_t* next_groups,
                              int32_t* n_next, int32_t* hops_run) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!n_next || !hops_run || (n_sel > 0 && !next_groups))
    return fail(c, KEEP_ERR_INVALID_ARG, "next_groups / n_next / hops_run is NULL");
  if (budget_mode != KEEP_BUDGET_GROUP_COUNT && budget_mode != KEEP_BUDGET_TOKENS)
    return fail(c, KEEP_ERR_INVALID_ARG, "unknown budget_mode");
  if (!(ratio_next >= 0.f && ratio_next <= 1.f)) return fail(c, KEEP_ERR_INVALID_ARG, "ratio_next outside [0, 1]");
  if (hops < 1) return fail(c, KEEP_ERR_INVALID_ARG, "hops must be at least 1");
  PromptInfo pi;
  keep_status st = check_prompt(c, p, &pi, false);
  if (st != KEEP_OK) return st;
  st = check_set(c, pi, groups, n_sel);
  if (st != KEEP_OK) return st;
  if (c->last_layer != layer || (int)c->last_groups.size() != n_sel ||
      !std::equal(c->last_groups.begin(), c->last_groups.end(), groups))
    return fail(c, KEEP_ERR_STATE, "keep_score_groups(layer %d) needs keep_recompute_layer of that layer and set first",
                layer);
  LayerPlan plan;
  plan.m = n_sel;
  plan.n_rows = c->last_n_rows;
  plan.row_start = c->last_row_start;
  // attention of the layer must be complete before its scores are read (second
  // dependency of the paper's pipeline): order the eval stream after the compute stream
  HIP_TRY(c, hipEventRecord(c->ev_attn, c->s_comp));
  HIP_TRY(c, hipStreamWaitEvent(c->s_eval, c->ev_attn, 0));
  st = by_dtype(c, [&](auto* tag) {
    using T = std::remove_pointer_t<decltype(tag)>;
    return score_matrix<T>(c, layer, plan, c->s_eval);
  });
  if (st != KEEP_OK) return st;
  if (S_out && n_sel > 0)
    HIP_TRY(c, hipMemcpyAsync(c->h_S, c->S, (size_t)(n_sel + 1) * n_sel * sizeof(float), hipMemcpyDeviceToHost,
                              c->s_eval));
  int k_count, tok;
  const SelectKind kind = classify_budget(pi, p, groups, n_sel, ratio_next, budget_mode, &k_count, &tok);
  if (kind == SEL_DEVICE) {
    st = enqueue_select(c, n_sel, k_count, tok, budget_mode, hops, c->s_eval);
    if (st != KEEP_OK) return st;
  }
  HIP_TRY(c, hipStreamSynchronize(c->s_eval));
  if (S_out && n_sel > 0) memcpy(S_out, c->h_S, (size_t)(n_sel + 1) * n_sel * sizeof(float));
  if (kind == SEL_ALL) {
    for (int i = 0; i < n_sel; ++i) next_groups[i] = groups[i];
    *n_next = n_sel;
    *hops_run = 0;
  } else if (kind == SEL_NONE) {
    *n_next = 0;
    *hops_run = 0;
  } else {
    *n_next = c->h_sel_out[0];
    *hops_run = c->h_sel_out[1];
    for (int i = 0; i < *n_next; ++i) next_groups[i] = groups[c->h_sel_out[2 + i]];
  }
  return KEEP_OK;
}

keep_status keep_set_option(keep_ctx* c, int32_t option, int32_t value) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (option == KEEP_OPT_PROPAGATION_SOURCES) {
    if (value != KEEP_SOURCES_QUERY_AND_SET && value != KEEP_SOURCES_SET_ONLY)
      return fail(c, KEEP_ERR_INVALID_ARG, "unknown value %d for KEEP_OPT_PROPAGATION_SOURCES", value);
    c->set_only = value == KEEP_SOURCES_SET_ONLY;
    return KEEP_OK;
  }
  return fail(c, KEEP_ERR_INVALID_ARG, "unknown option %d", option);
}

keep_status keep_read_layer_state(keep_ctx* c, int32_t what, void* dst, uint64_t bytes) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!dst) return fail(c, KEEP_ERR_INVALID_ARG, "dst is NULL");
  if (c->last_layer < 0)
    return fail(c, KEEP_ERR_STATE, "keep_read_layer_state needs a keep_recompute_layer whose state is still in the workspace");
  const void* src = nullptr;
  uint64_t want = 0;
  if (what == KEEP_STATE_ATTN_OUT) {
    src = c->o;
    want = (uint64_t)c->last_n_rows * c->d.n_q_heads * c->d.head_dim * c->esz;
  } else if (what == KEEP_STATE_LSE) {
    src = c->lse;
    want = (uint64_t)c->last_n_rows * c->d.n_q_heads * sizeof(float);
  } else {
    return fail(c, KEEP_ERR_INVALID_ARG, "unknown layer state %d", what);
  }
  if (bytes != want)
    return fail(c, KEEP_ERR_INVALID_ARG, "state %d of the last layer holds %llu bytes, the buffer %llu", what,
                (unsigned long long)want, (unsigned long long)bytes);
  HIP_TRY(c, hipStreamSynchronize(c->s_comp));
  HIP_TRY(c, hipMemcpy(dst, src, (size_t)bytes, hipMemcpyDeviceToHost));
  return KEEP_OK;
}

keep_status keep_select_groups(keep_ctx* c, const float* S, const int32_t* groups, int32_t n_sel,
                               const int32_t* group_len, int32_t n_groups_total, float ratio_next, int32_t hops,
                               int32_t budget_mode, int32_t* next_groups, int32_t* n_next, int32_t* hops_run) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!n_next || !hops_run || !group_len || (n_sel > 0 && (!next_groups || !S || !groups)))
    return fail(c, KEEP_ERR_INVALID_ARG, "a pointer argument is NULL");
  if (budget_mode != KEEP_BUDGET_GROUP_COUNT && budget_mode != KEEP_BUDGET_TOKENS)
    return fail(c, KEEP_ERR_INVALID_ARG, "unknown budget_mode");
  if (!(ratio_next >= 0.f && ratio_next <= 1.f)) return fail(c, KEEP_ERR_INVALID_ARG, "ratio_next outside [0, 1]");
  if (hops < 1) return fail(c, KEEP_ERR_INVALID_ARG, "hops must be at least 1");
  if (n_groups_total < 0 || n_groups_total > c->d.max_groups)
    return fail(c, KEEP_ERR_WORKSPACE, "n_groups_total %d above max_groups %d", n_groups_total, c->d.max_groups);
  if (n_sel < 0 || n_sel > n_groups_total) return fail(c, KEEP_ERR_INVALID_ARG, "n_sel outside [0, n_groups_total]");
  PromptInfo pi;
  pi.G = n_groups_total;
  int64_t tot = 0;
  for (int g = 0; g < n_groups_total; ++g) {
    if (group_len[g] < 1) return fail(c, KEEP_ERR_INVALID_ARG, "group_len[%d] must be >= 1", g);
    tot += group_len[g];
  }
  pi.n_mem = (int)tot;
  for (int i = 0; i < n_sel; ++i) {
    if (groups[i] < 0 || groups[i] >= n_groups_total) return fail(c, KEEP_ERR_INVALID_ARG, "groups[%d] out of range", i);
    if (i && groups[i] <= groups[i - 1]) return fail(c, KEEP_ERR_INVALID_ARG, "groups must be strictly ascending");
  }
  keep_prompt fake{};
  fake.group_len = group_len;
  int k_count, tok;
  const SelectKind kind = classify_budget(pi, &fake, groups, n_sel, ratio_next, budget_mode, &k_count, &tok);
  if (kind == SEL_ALL) {
    for (int i = 0; i < n_sel; ++i) next_groups[i] = groups[i];
    *n_next = n_sel;
    *hops_run = 0;
    return KEEP_OK;
  }
  if (kind == SEL_NONE) {
    *n_next = 0;
    *hops_run = 0;
    return KEEP_OK;
  }
  c->last_layer = -1;  // the score workspace is overwritten
  hipStream_t s = c->s_eval;
  memcpy(c->h_S, S, (size_t)(n_sel + 1) * n_sel * sizeof(float));
  HIP_TRY(c, hipMemcpyAsync(c->S, c->h_S, (size_t)(n_sel + 1) * n_sel * sizeof(float), hipMemcpyHostToDevice, s));
  std::vector<int32_t> cl(n_sel);
  for (int i = 0; i < n_sel; ++i) cl[i] = group_len[groups[i]];
  HIP_TRY(c, hipMemcpyAsync(c->d_cand_len, cl.data(), (size_t)n_sel * 4, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipStreamSynchronize(s));  // cl is pageable host memory
  keep_status st = enqueue_select(c, n_sel, k_count, tok, budget_mode, hops, s);
  if (st != KEEP_OK) return st;
  HIP_TRY(c, hipStreamSynchronize(s));
  *n_next = c->h_sel_out[0];
  *hops_run = c->h_sel_out[1];
  for (int i = 0; i < *n_next; ++i) next_groups[i] = groups[c->h_sel_out[2 + i]];
  return KEEP_OK;
}

keep_status keep_prefill(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t hops, int32_t budget_mode,
                         int32_t load_mode, void* k_cache, void* v_cache, void* x_final, int32_t* sel_groups,
                         int32_t* sel_counts, keep_report* report) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!x_final) return fail(c, KEEP_ERR_INVALID_ARG, "x_final is NULL");
  return prefill_impl(c, p, ratios, hops, budget_mode, load_mode, k_cache, v_cache, 0, x_final, sel_groups,
                      sel_counts, report);
}

keep_status keep_prefill_padded(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t hops,
                                int32_t budget_mode, int32_t load_mode, void* k_cache, void* v_cache,
                                int32_t cache_rows, void* x_final, int32_t* sel_groups, int32_t* sel_counts,
                                keep_report* report) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!x_final) return fail(c, KEEP_ERR_INVALID_ARG, "x_final is NULL");
  if (cache_rows < 1) return fail(c, KEEP_ERR_INVALID_ARG, "cache_rows must be positive");
  return prefill_impl(c, p, ratios, hops, budget_mode, load_mode, k_cache, v_cache, cache_rows, x_final, sel_groups,
                      sel_counts, report);
}

keep_status keep_prefill_tokens(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t load_mode, void* k_cache,
                                void* v_cache, void* x_final, int32_t* sel_rows, int32_t* sel_counts,
                                float* deviation_out, keep_report* report) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!x_final) return fail(c, KEEP_ERR_INVALID_ARG, "x_final is NULL");
  return by_dtype(c, [&](auto* tag) {
    using T = std::remove_pointer_t<decltype(tag)>;
    return prefill_tokens_impl<T>(c, p, ratios, load_mode, k_cache, v_cache, x_final, sel_rows, sel_counts,
                                  deviation_out, report);
  });
}

keep_status keep_select_tokens(keep_ctx* c, const float* deviation, int32_t n, int32_t k, int32_t* kept) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (n < 0 || k < 0 || k > n) return fail(c, KEEP_ERR_INVALID_ARG, "need 0 <= k <= n");
  if (n > c->d.max_tokens) return fail(c, KEEP_ERR_WORKSPACE, "n %d above max_tokens %d", n, c->d.max_tokens);
  if ((n > 0 && !deviation) || (k > 0 && !kept)) return fail(c, KEEP_ERR_INVALID_ARG, "deviation / kept is NULL");
  if (k == 0) return KEEP_OK;
  hipStream_t s = c->s_comp;
  HIP_TRY(c, hipStreamSynchronize(s));  // the pinned staging buffers are free
  memcpy(c->h_dev, deviation, (size_t)n * sizeof(float));
  HIP_TRY(c, hipMemcpyAsync(c->d_dev, c->h_dev, (size_t)n * sizeof(float), hipMemcpyHostToDevice, s));
  launch_select_tokens(c->d_dev, n, k, 0, c->d_tok_flags, c->d_tok_list, s);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipMemcpyAsync(c->h_tok_list, c->d_tok_list, (size_t)k * 4, hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  memcpy(kept, c->h_tok_list, (size_t)k * 4);
  return KEEP_OK;
}

keep_status keep_decode(keep_ctx* c, const void* final_norm, const void* lm_head, const void* x_last, void* k_cache,
                        void* v_cache, int32_t cache_rows, int32_t n_ctx, int32_t n_new, int32_t* tokens_out,
                        float* logits_out, const int32_t* forced_tokens) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!final_norm || !lm_head || !x_last || !k_cache || !v_cache || !tokens_out)
    return fail(c, KEEP_ERR_INVALID_ARG, "final_norm / lm_head / x_last / k_cache / v_cache / tokens_out is NULL");
  if (n_new < 1 || n_new > KEEP_DECODE_MAX_TOKENS)
    return fail(c, KEEP_ERR_INVALID_ARG, "n_new %d outside [1, %d]", n_new, KEEP_DECODE_MAX_TOKENS);
  if (n_ctx < 1) return fail(c, KEEP_ERR_INVALID_ARG, "n_ctx must be at least 1");
  if ((int64_t)n_ctx + n_new - 1 > cache_rows)
    return fail(c, KEEP_ERR_INVALID_ARG, "n_ctx + n_new - 1 = %lld rows do not fit cache_rows %d",
                (long long)n_ctx + n_new - 1, cache_rows);
  if ((int64_t)n_ctx + n_new - 1 > c->d.max_tokens)
    return fail(c, KEEP_ERR_WORKSPACE, "n_ctx + n_new - 1 above max_tokens %d", c->d.max_tokens);
  if (forced_tokens)
    for (int t = 0; t + 1 < n_new; ++t)
      if (forced_tokens[t] < 0 || forced_tokens[t] >= c->d.vocab)
        return fail(c, KEEP_ERR_INVALID_ARG, "forced_tokens[%d] = %d outside the vocabulary", t, forced_tokens[t]);
  c->last_layer = -1;
  return by_dtype(c, [&](auto* tag) {
    using T = std::remove_pointer_t<decltype(tag)>;
    return decode_impl<T>(c, final_norm, lm_head, x_last, k_cache, v_cache, cache_rows, n_ctx, n_new, tokens_out,
                          logits_out, forced_tokens);
  });
}

keep_status keep_dequantize_int4(const void* codes, const void* scale_zero, int32_t rows, int32_t K, void* out,
                                 void* stream) {
  if (!codes || !scale_zero || !out) return fail(nullptr, KEEP_ERR_INVALID_ARG, "codes / scale_zero / out is NULL");
  if (rows < 32 || rows % 32 || K < 128 || K % 128)
    return fail(nullptr, KEEP_ERR_INVALID_ARG, "rows %d must be a positive multiple of 32 and K %d of 128", rows, K);
  launch_dequant_int4(codes, scale_zero, rows, K, out, reinterpret_cast<hipStream_t>(stream));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, KEEP_ERR_HIP, "dequantisation launch failed: %s", hipGetErrorString(e));
  return KEEP_OK;
}

keep_status keep_attach_int4(keep_ctx* c, const keep_layer_weights_int4* layers) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!layers) {
    c->w4.clear();
    return KEEP_OK;
  }
  if (!c->mfma) return fail(c, KEEP_ERR_UNSUPPORTED, "the INT4 form is read by the bf16 matrix-core path only");
  if (c->d.hidden % 128 || c->d.ffn_dim % 128 || (c->d.n_q_heads * c->d.head_dim) % 128 ||
      (c->d.n_kv_heads * c->d.head_dim) % 64)
    return fail(c, KEEP_ERR_SHAPE, "hidden, ffn_dim and n_q_heads * head_dim must be multiples of the group length 128, "
                                    "n_kv_heads * head_dim of 64");
  for (int l = 0; l < c->d.n_layers; ++l) {
    const keep_layer_weights_int4& w = layers[l];
    for (const keep_int4_matrix* m : {&w.wq, &w.wk, &w.wv, &w.wo, &w.wgate, &w.wup, &w.wdown})
      if (!m->codes || !m->scale_zero) return fail(c, KEEP_ERR_INVALID_ARG, "an INT4 pointer of layer %d is NULL", l);
  }
  c->w4.assign(layers, layers + c->d.n_layers);
  return KEEP_OK;
}

keep_status keep_precompute_group(keep_ctx* c, const int32_t* token_ids, int32_t n_tokens, void* k_blocks,
                                  void* v_blocks, keep_report* report) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!token_ids || !k_blocks || !v_blocks) return fail(c, KEEP_ERR_INVALID_ARG, "token_ids / k_blocks / v_blocks is NULL");
  if (n_tokens < 1) return fail(c, KEEP_ERR_INVALID_ARG, "a unit needs at least one token");
  // A prompt without memories whose "instruction" is the unit: every row is recomputed at every layer
  // over its own causal prefix at positions 0..n-1, which is the dense prefill of the unit on its own;
  // the joined cache of that prompt is the unit's block of every layer.
  keep_prompt pr;
  memset(&pr, 0, sizeof pr);
  pr.n_groups = 0;
  pr.instr_len = n_tokens;
  pr.token_ids = token_ids;
  pr.kv_location = KEEP_KV_DEVICE;
  std::vector<float> ratios((size_t)c->d.n_layers, 0.f);
  return prefill_impl(c, &pr, ratios.data(), 1, KEEP_BUDGET_GROUP_COUNT, KEEP_LOAD_SERIAL, k_blocks, v_blocks, 0, nullptr,
                      nullptr, nullptr, report);
}

keep_status keep_precompute_groups(keep_ctx* c, int32_t n_units, const int32_t* unit_len, const int32_t* token_ids,
                                   void* k_blocks, void* v_blocks, keep_report* report) {
  if (!c) return KEEP_ERR_INVALID_ARG;
  if (!unit_len || !token_ids || !k_blocks || !v_blocks)
    return fail(c, KEEP_ERR_INVALID_ARG, "unit_len / token_ids / k_blocks / v_blocks is NULL");
  if (n_units < 1) return fail(c, KEEP_ERR_INVALID_ARG, "n_units must be at least 1");
  int64_t total = 0;
  for (int u = 0; u < n_units; ++u) {
    if (unit_len[u] < 1) return fail(c, KEEP_ERR_INVALID_ARG, "unit_len[%d] = %d, must be >= 1", u, unit_len[u]);
    total += unit_len[u];
    if (total > c->d.max_tokens) return fail(c, KEEP_ERR_WORKSPACE, "units longer than max_tokens %d", c->d.max_tokens);
  }
  // One pass for all the units: the rows are every token in order, row t of unit u sits at cache row
  // off_u + t, is rotated at its local position t and attends to rows off_u .. off_u + t only.
  // (The bounds sit in pinned memory until the upload has run: wait for the stream's earlier work first.)
  HIP_TRY(c, hipStreamSynchronize(c->s_comp));
  int row = 0;
  for (int u = 0; u < n_units; ++u) {
    const int start = row;
    for (int t = 0; t < unit_len[u]; ++t) c->h_row_lo[row++] = start;
  }
  HIP_TRY(c, hipMemcpyAsync(c->d_row_lo, c->h_row_lo, (size_t)total * 4, hipMemcpyHostToDevice, c->s_comp));
  keep_prompt pr;
  memset(&pr, 0, sizeof pr);
  pr.n_groups = 0;
  pr.instr_len = (int32_t)total;
  pr.token_ids = token_ids;
  pr.kv_location = KEEP_KV_DEVICE;
  std::vector<float> ratios((size_t)c->d.n_layers, 0.f);
  c->units_mode = true;
  const keep_status st = prefill_impl(c, &pr, ratios.data(), 1, KEEP_BUDGET_GROUP_COUNT, KEEP_LOAD_SERIAL, k_blocks,
                                      v_blocks, 0, nullptr, nullptr, nullptr, report);
  c->units_mode = false;
  return st;
}

}  // extern "C"

namespace {

// ---------------------------------------------------------------------------
// keep_prefill: the per-layer pipeline (Section 5: compute / evaluate / load)
// ---------------------------------------------------------------------------
// How one layer is ordered.  Decided in one place, plan_order(), from the next layer's budget alone.
struct LayerOrder {
  SelectKind kind = SEL_NONE;  // SEL_DEVICE: the next set needs scores and the selector; otherwise it is all or none
  int k_count = 0, tok = 0;    // the next layer's budget in memories and in tokens
  // Output projection + FFN normally run beside the evaluation (Section 4.2).  When the budget says that at most
  // half of this layer's rows survive into the next set, evaluation goes first and they run on the surviving rows
  // only: the hidden rows of dropped memories are discarded anyway (Section 4.3).
  bool eval_first = false;
  // With many candidates only a few rows of S are ever read: the query's, and those of the memories that enter a
  // relevant set during the hops (Section 4.2: propagation averages the rows of the current relevant set).  They
  // are formed hop by hop, as the sets become known; the selector re-runs hops 1..h each time, so the result is
  // that of one run (with a single selection only the query's row is ever formed).  (Worth it only where the budget keeps at most half of the candidates' rows: otherwise
  // nearly every row is read anyway and the hop-by-hop round trips are pure overhead.)
  bool lazy_scores = false;
  // Where both hold, the attention itself is needed only for the rows whose scores are read and for the rows
  // that survive: it runs for the instruction first and for each hop's new memories after that.
  bool lazy_attn = false;
};

struct PrefillRun {
  keep_ctx* c;
  const keep_prompt* p;
  const float* ratios;
  int hops, budget_mode, load_mode;
  char *k_cache, *v_cache;
  void* x_final;
  int32_t *sel_groups, *sel_counts;
  keep_report* report;

  PromptInfo pi;
  int L = 0;
  bool host_kv = false;
  size_t row_bytes = 0, layer_bytes = 0;
  Loader ld{};
  std::vector<int32_t> cur, nxt;  // the relevant set of this layer / of the next
  void *x_cur = nullptr, *x_nxt = nullptr;  // hidden rows of the current layer (compact) / the other row buffer
  bool x_from_embed = true;
  LayerPlan plan;
  std::vector<float> part_attn_ms;  // attention launches on parts of a layer
  std::vector<uint8_t> want, have;  // source blocks of S wanted now / formed so far (block m = the instruction)

  // state of the layer in hand
  int l = 0;
  hipEvent_t* evs = nullptr;
  char *kl = nullptr, *vl = nullptr;
  LayerOrder ord;
  int part_launches = 0;  // attention launches on parts of the layer (timed with c->ev_part)
  long attn_rows = 0;
  uint64_t attn_keys = 0;

  bool timed() const { return evs && !c->ev_light; }

  LayerOrder plan_order() const {
    LayerOrder o;
    if (l + 1 == L) return o;
    const int m = (int)cur.size();
    o.kind = classify_budget(pi, p, cur.data(), m, ratios[l + 1], budget_mode, &o.k_count, &o.tok);
    if (o.kind != SEL_DEVICE) return o;
    const long mem_rows = plan.n_rows - pi.Lq;
    const long keep_rows = budget_mode == KEEP_BUDGET_TOKENS ? std::min<long>(o.tok, mem_rows)
                                                             : mem_rows * o.k_count / std::max(1, m);
    o.eval_first = (keep_rows + pi.Lq) * 2 <= plan.n_rows;
    o.lazy_scores = c->mfma && m >= LAZY_MIN_CANDIDATES && keep_rows * 2 <= mem_rows;
    o.lazy_attn = o.lazy_scores && o.eval_first;
    return o;
  }

  // ---- compute stream: everything up to attention (up to RoPE/scatter where the attention runs on demand)
  keep_status front() {
    const void* x_in = x_from_embed ? nullptr : x_cur;
    return by_dtype(c, [&](auto* tag) {
      using T = std::remove_pointer_t<decltype(tag)>;
      return layer_front<T>(c, pi, l, plan, x_in, kl, vl, evs, ord.lazy_attn);
    });
  }

  // attention of the rows of the flagged blocks (on-demand layers)
  keep_status attend(const uint8_t* flags) {
    int n_att = 0;
    uint64_t n_keys = 0;
    const int slot = std::min(part_launches, 7);
    keep_status st = attend_blocks(c, pi, l, plan, flags, kl, vl, timed() ? c->ev_part[2 * slot] : nullptr,
                                   timed() ? c->ev_part[2 * slot + 1] : nullptr, &n_att, &n_keys);
    if (st != KEEP_OK) return st;
    if (n_att > 0) {
      attn_rows += n_att;
      attn_keys += n_keys;
      if (part_launches < 8) ++part_launches;
    }
    return KEEP_OK;
  }

  keep_status scores(const uint8_t* h_want) {
    return by_dtype(c, [&](auto* tag) {
      using T = std::remove_pointer_t<decltype(tag)>;
      return score_matrix<T>(c, l, plan, c->s_eval, h_want);
    });
  }

  // the eval stream follows the compute stream's attention (second dependency of Section 5's pipeline)
  keep_status eval_after_attention() {
    HIP_TRY(c, hipEventRecord(c->ev_attn, c->s_comp));
    HIP_TRY(c, hipStreamWaitEvent(c->s_eval, c->ev_attn, 0));
    return KEEP_OK;
  }

  // ---- eval stream: first score pass + selector (all hops, or the first selection where rows come on demand)
  keep_status start_evaluation() {
    const int m = (int)cur.size();
    keep_status st;
    if (ord.lazy_scores) {
      want.assign((size_t)m + 1, 0);
      have.assign((size_t)m + 1, 0);
      want[m] = have[m] = 1;
    }
    if (ord.lazy_attn) {
      attn_rows = 0;
      attn_keys = 0;
      st = attend(want.data());  // the instruction's rows
      if (st != KEEP_OK) return st;
    }
    st = eval_after_attention();
    if (st != KEEP_OK) return st;
    if (timed()) HIP_TRY(c, hipEventRecord(evs[10], c->s_eval));
    if (ord.lazy_scores) HIP_TRY(c, hipMemsetAsync(c->S, 0, (size_t)(m + 1) * m * sizeof(float), c->s_eval));
    st = scores(ord.lazy_scores ? want.data() : nullptr);
    if (st != KEEP_OK) return st;
    st = enqueue_select(c, m, ord.k_count, ord.tok, budget_mode, ord.lazy_scores ? 1 : hops, c->s_eval);
    if (st != KEEP_OK) return st;
    if (timed()) HIP_TRY(c, hipEventRecord(evs[11], c->s_eval));
    HIP_TRY(c, hipEventRecord(c->ev_eval, c->s_eval));
    return KEEP_OK;
  }

  // ---- compute stream: output projection + FFN on n_rows rows
  keep_status back(int n_rows, const void* o_rows, const void* x_in, void* x_out) {
    keep_status st = by_dtype(c, [&](auto* tag) {
      using T = std::remove_pointer_t<decltype(tag)>;
      return layer_back<T>(c, l, n_rows, o_rows, x_in, x_out, evs);
    });
    if (st != KEEP_OK) return st;
    if (report) report->ffn_rows[l] = n_rows;
    Staging& sg = c->stage[l];
    HIP_TRY(c, hipEventRecord(sg.done, c->s_comp));
    sg.used = true;
    return KEEP_OK;
  }

  // Layer-balanced loading (Section 4.3): while the host waits for the selection the loader is idle, and the
  // memories outside the current set can never come back, so their blocks of later layers are pre-loaded,
  // layer by layer, with a bounded number of bytes in flight so that the copies the next layer is waiting
  // for never queue behind a long run of pre-loads.
  keep_status preload_while_waiting() {
    int preload_layer = l + 2, preload_group = 0;
    while (hipEventQuery(c->ev_eval) == hipErrorNotReady) {
      ld.retire();
      if (preload_layer >= L || ld.inflight >= PRELOAD_INFLIGHT_CAP) continue;
      bool issued = false;
      while (preload_layer < L && !issued) {
        while (preload_group < pi.G && std::binary_search(cur.begin(), cur.end(), preload_group)) ++preload_group;
        if (preload_group >= pi.G) {
          ++preload_layer;
          preload_group = 0;
          continue;
        }
        // the run of groups outside the set that starts at the cursor (at most 8 of them per chunk)
        int run_end = preload_group + 1;
        while (run_end < pi.G && run_end < preload_group + 8 && !std::binary_search(cur.begin(), cur.end(), run_end))
          ++run_end;
        bool any = false;
        for (int gg = preload_group; gg < run_end; ++gg) any |= !ld.loaded[(size_t)preload_layer * pi.G + gg];
        if (any) {
          keep_status st = ld.copy_run(preload_layer, preload_group, run_end);
          if (st != KEEP_OK) return st;
          issued = true;
        }
        preload_group = run_end;
      }
    }
    return KEEP_OK;
  }

  // flags of the selector's current set that have no score row (and no attention) yet; marks them as had
  bool flag_new_members() {
    bool any = false;
    std::fill(want.begin(), want.end(), 0);
    for (int i = 0; i < c->h_sel_out[0]; ++i) {
      const int a = c->h_sel_out[2 + i];
      if (!have[a]) want[a] = have[a] = 1, any = true;
    }
    return any;
  }

  // ---- host: wait for the selection (it sizes the next layer's launches); on-demand layers go round by round
  keep_status await_selection() {
    const int m = (int)cur.size();
    keep_status st;
    if (host_kv && load_mode == KEEP_LOAD_LAYER_BALANCED) {
      st = preload_while_waiting();
      if (st != KEEP_OK) return st;
    }
    HIP_TRY(c, hipEventSynchronize(c->ev_eval));
    if (ord.lazy_scores) {
      std::vector<int32_t> prev_set;
      for (int h = 1; h < hops; ++h) {
        // the set repeated: converged (the selector would stop here as well)
        std::vector<int32_t> this_set(c->h_sel_out + 2, c->h_sel_out + 2 + c->h_sel_out[0]);
        if (c->h_sel_out[1] < h || (h > 1 && this_set == prev_set)) break;
        prev_set.swap(this_set);
        // rows of the memories selected at hop h that are not there yet
        if (flag_new_members()) {
          if (ord.lazy_attn) {  // their attention first: the scores need its log-sum-exp
            st = attend(want.data());
            if (st != KEEP_OK) return st;
            st = eval_after_attention();
            if (st != KEEP_OK) return st;
          }
          st = scores(want.data());
          if (st != KEEP_OK) return st;
        }
        st = enqueue_select(c, m, ord.k_count, ord.tok, budget_mode, h + 1, c->s_eval);
        if (st != KEEP_OK) return st;
        if (timed()) HIP_TRY(c, hipEventRecord(evs[11], c->s_eval));
        HIP_TRY(c, hipStreamSynchronize(c->s_eval));
      }
    }
    nxt.clear();
    const int nn = c->h_sel_out[0];
    for (int i = 0; i < nn; ++i) nxt.push_back(cur[c->h_sel_out[2 + i]]);
    if (report) report->hops_run[l] = c->h_sel_out[1];
    if (ord.lazy_attn) {
      // members of the final set that no hop has needed yet: their outputs are needed now
      if (flag_new_members()) {
        st = attend(want.data());
        if (st != KEEP_OK) return st;
      }
      st = note_part_attention();
      if (st != KEEP_OK) return st;
    }
    return KEEP_OK;
  }

  // rows and keys of the layer's attention launches on parts of its rows, and their time
  keep_status note_part_attention() {
    if (report) {
      report->attn_rows[l] = (int32_t)attn_rows;
      report->attn_keys[l] = attn_keys;
    }
    if (timed() && part_launches > 0) {  // the events are reused by later layers: read them now
      HIP_TRY(c, hipEventSynchronize(c->ev_part[2 * (part_launches - 1) + 1]));
      for (int i = 0; i < part_launches; ++i) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, c->ev_part[2 * i], c->ev_part[2 * i + 1]);
        part_attn_ms[l] += ms;
      }
    }
    return KEEP_OK;
  }

  // The last layer.  Behind it only the instruction's hidden rows are read (Section 5: the prefill hands the
  // decoder the updated cache and the instruction's state), and none at all where the caller wants the caches
  // alone (a memory unit cached on its own).  K/V of the whole set are refreshed as in every layer; attention,
  // output projection and FFN run for the instruction's rows only, which are the tail of the compact layout.
  keep_status last_layer_tail() {
    const keep_model_desc& d = c->d;
    const int m = (int)cur.size();
    const bool rows_wanted = x_final != nullptr;
    ord.lazy_attn = c->mfma || !rows_wanted;  // front() stops before the attention
    keep_status st = front();
    if (st != KEEP_OK) return st;
    attn_rows = ord.lazy_attn ? 0 : plan.n_rows;
    if (ord.lazy_attn) attn_keys = 0;
    if (rows_wanted && c->mfma) {
      want.assign((size_t)m + 1, 0);
      want[m] = 1;
      st = attend(want.data());
      if (st != KEEP_OK) return st;
    }
    st = note_part_attention();
    if (st != KEEP_OK) return st;
    if (!rows_wanted) {
      if (report) report->ffn_rows[l] = 0;
      return KEEP_OK;
    }
    const size_t first = (size_t)(plan.n_rows - pi.Lq);
    const size_t o_off = first * d.n_q_heads * d.head_dim * c->esz, x_off = first * d.hidden * c->esz;
    return back(pi.Lq, (const char*)c->o + o_off, (const char*)x_cur + x_off, (char*)x_nxt + x_off);
  }

  // ---- copy stream: the groups that just left the set complete layer l+1 (first dependency of the pipeline)
  keep_status finish_loading(uint64_t bytes_before) {
    if (load_mode == KEEP_LOAD_SERIAL) {  // load strictly after this layer's compute
      HIP_TRY(c, hipEventRecord(c->ev_comp, c->s_comp));
      HIP_TRY(c, hipStreamWaitEvent(c->s_copy, c->ev_comp, 0));
    }
    keep_status st = ld.copy_outside(l + 1, nxt);
    if (st != KEEP_OK) return st;
    HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
    HIP_TRY(c, hipStreamWaitEvent(c->s_comp, c->ev_load, 0));
    if (report) report->bytes_loaded[l + 1] = ld.bytes_total - bytes_before;
    return KEEP_OK;
  }

  // ---- hidden rows of the next set; where evaluation went first this is also where this layer's output
  // projection + FFN run (on the survivors)
  keep_status next_rows() {
    const keep_model_desc& d = c->d;
    const int m = (int)cur.size();
    keep_status st;
    if (nxt.size() == cur.size()) {  // same rows: this layer's output is the next layer's input
      if (ord.eval_first) {
        st = back(plan.n_rows, c->o, x_cur, x_nxt);
        if (st != KEEP_OK) return st;
      }
      std::swap(x_cur, x_nxt);
      return KEEP_OK;
    }
    // compact start of each kept block in the current layout and in the next one
    Staging& sg = c->stage[l];
    std::vector<int32_t> dst_start(nxt.size() + 2);
    int acc = 0;
    size_t ci = 0;
    for (size_t i = 0; i < nxt.size(); ++i) {
      while (cur[ci] != nxt[i]) ++ci;
      sg.gather_src[i] = plan.row_start[ci];
      dst_start[i] = acc;
      acc += p->group_len[nxt[i]];
    }
    sg.gather_src[nxt.size()] = plan.row_start[m];
    dst_start[nxt.size()] = acc;
    acc += pi.Lq;
    dst_start[nxt.size() + 1] = acc;
    // (the destination starts are the next layer's row_start; nothing still reads the old one)
    memcpy(sg.gather_dst, dst_start.data(), dst_start.size() * 4);
    HIP_TRY(c, hipMemcpyAsync(c->d_gather_src, sg.gather_src, (nxt.size() + 1) * 4, hipMemcpyHostToDevice, c->s_comp));
    HIP_TRY(c, hipMemcpyAsync(c->d_row_start, sg.gather_dst, dst_start.size() * 4, hipMemcpyHostToDevice, c->s_comp));
    const int n_blocks = (int)nxt.size() + 1;
    if (!ord.eval_first) {
      void* x_out_buf = x_nxt;  // this layer's output
      void* x_dst = x_cur;      // this layer's input buffer is free once the layer is done
      st = by_dtype(c, [&](auto* tag) {
        using T = std::remove_pointer_t<decltype(tag)>;
        launch_rows_gather<T>(Typed<T>::p(x_out_buf), c->d_gather_src, c->d_row_start, n_blocks, acc, d.hidden,
                              Typed<T>::p(x_dst), c->s_comp);
        return KEEP_OK;
      });
      HIP_TRY(c, hipGetLastError());
      HIP_TRY(c, hipEventRecord(sg.done, c->s_comp));
      x_cur = x_dst;
      return KEEP_OK;
    }
    // survivors first: gather their attention rows (into the q buffer, free now that the scores are done) and
    // their input rows, then output projection + FFN on them alone
    const int qd = d.n_q_heads * d.head_dim;
    st = by_dtype(c, [&](auto* tag) {
      using T = std::remove_pointer_t<decltype(tag)>;
      launch_rows_gather<T>(Typed<T>::p(c->o), c->d_gather_src, c->d_row_start, n_blocks, acc, qd, Typed<T>::p(c->q),
                            c->s_comp);
      launch_rows_gather<T>(Typed<T>::p(x_cur), c->d_gather_src, c->d_row_start, n_blocks, acc, d.hidden,
                            Typed<T>::p(x_nxt), c->s_comp);
      return KEEP_OK;
    });
    HIP_TRY(c, hipGetLastError());
    return back(acc, c->q, x_nxt, x_cur);  // output lands in x_cur, already in the next layout
  }

  void read_event_times() {
    for (int ll = 0; ll < L; ++ll) {
      hipEvent_t* e = &c->ev[(size_t)ll * EV_PER_LAYER];
      (void)hipEventElapsedTime(&report->ms_gateup[ll], e[7], e[8]);
      if (c->ev_light) continue;
      (void)hipEventElapsedTime(&report->ms_realign[ll], e[0], e[1]);
      (void)hipEventElapsedTime(&report->ms_prep[ll], e[1], e[2]);
      (void)hipEventElapsedTime(&report->ms_qkv_gemm[ll], e[2], e[3]);
      (void)hipEventElapsedTime(&report->ms_rope[ll], e[3], e[4]);
      (void)hipEventElapsedTime(&report->ms_attn[ll], e[4], e[5]);
      report->ms_attn[ll] += part_attn_ms[ll];
      (void)hipEventElapsedTime(&report->ms_oproj[ll], e[12], e[6]);
      (void)hipEventElapsedTime(&report->ms_norm2[ll], e[6], e[7]);
      (void)hipEventElapsedTime(&report->ms_down[ll], e[8], e[9]);
      if (report->hops_run[ll] > 0) (void)hipEventElapsedTime(&report->ms_score[ll], e[10], e[11]);
    }
  }

  keep_status one_layer() {
    evs = report ? &c->ev[(size_t)l * EV_PER_LAYER] : nullptr;
    kl = k_cache + (size_t)l * layer_bytes;
    vl = v_cache + (size_t)l * layer_bytes;
    const int m = (int)cur.size();
    if (sel_counts) sel_counts[l] = m;
    if (sel_groups)
      for (int i = 0; i < m; ++i) sel_groups[(size_t)l * pi.G + i] = cur[i];
    keep_status st = stage_layer(c, p, pi, l, cur.data(), m, kl, vl, host_kv, &plan);
    if (st != KEEP_OK) return st;
    if (report) {
      report->rows[l] = plan.n_rows;
      report->set_size[l] = m;
      report->realign_rows[l] = plan.n_realign_rows;
    }
    ord = plan_order();
    part_launches = 0;
    attn_rows = plan.n_rows;
    attn_keys = (uint64_t)((int64_t)pi.Lq * (2 * (int64_t)pi.n_mem + pi.Lq + 1) / 2);
    for (int i = 0; i < m; ++i) {
      const int64_t first = pi.off[cur[i]], len = p->group_len[cur[i]];
      attn_keys += (uint64_t)(len * (2 * first + len + 1) / 2);
    }
    if (l + 1 == L && (plan.n_rows > pi.Lq || !x_final)) return last_layer_tail();
    st = front();
    if (st != KEEP_OK) return st;
    if (ord.kind == SEL_DEVICE) {
      st = start_evaluation();
      if (st != KEEP_OK) return st;
    }
    if (!ord.eval_first) {  // output projection + FFN beside the evaluation
      st = back(plan.n_rows, c->o, x_cur, x_nxt);
      if (st != KEEP_OK) return st;
    }
    if (report && !ord.lazy_attn) {
      report->attn_rows[l] = (int32_t)attn_rows;
      report->attn_keys[l] = attn_keys;
    }
    if (l + 1 == L) return KEEP_OK;

    // loading for the layers ahead, while this layer computes: groups outside the current set can never come
    // back, so their blocks of layer l+1 are needed for sure
    const uint64_t bytes_before = ld.bytes_total;
    if (host_kv && load_mode != KEEP_LOAD_SERIAL) {
      st = ld.copy_outside(l + 1, cur);
      if (st != KEEP_OK) return st;
    }
    if (ord.kind == SEL_DEVICE) {
      st = await_selection();
      if (st != KEEP_OK) return st;
    } else if (ord.kind == SEL_ALL) {
      nxt = cur;
    } else {
      nxt.clear();
    }
    if (host_kv) {
      st = finish_loading(bytes_before);
      if (st != KEEP_OK) return st;
    }
    st = next_rows();
    if (st != KEEP_OK) return st;
    x_from_embed = false;
    cur.swap(nxt);
    return KEEP_OK;
  }

  keep_status run(int32_t cache_rows) {
    const auto t_begin = std::chrono::steady_clock::now();
    const keep_model_desc& d = c->d;
    L = d.n_layers;
    if (!ratios || !k_cache || !v_cache) return fail(c, KEEP_ERR_INVALID_ARG, "ratios / k_cache / v_cache is NULL");
    if (budget_mode != KEEP_BUDGET_GROUP_COUNT && budget_mode != KEEP_BUDGET_TOKENS)
      return fail(c, KEEP_ERR_INVALID_ARG, "unknown budget_mode");
    if (load_mode < KEEP_LOAD_SERIAL || load_mode > KEEP_LOAD_LAYER_BALANCED)
      return fail(c, KEEP_ERR_INVALID_ARG, "unknown load_mode");
    if (hops < 1) return fail(c, KEEP_ERR_INVALID_ARG, "hops must be at least 1");
    if (ratios[0] != 0.f && ratios[0] != 1.f)
      return fail(c, KEEP_ERR_INVALID_ARG, "ratios[0] must be 1 (recompute all memories at the first layer) or 0");
    for (int i = 1; i < L; ++i) {
      if (!(ratios[i] >= 0.f && ratios[i] <= 1.f)) return fail(c, KEEP_ERR_INVALID_ARG, "ratios[%d] outside [0, 1]", i);
      if (ratios[i] > ratios[i - 1])
        return fail(c, KEEP_ERR_INVALID_ARG, "ratios must not increase (ratios[%d] > ratios[%d])", i, i - 1);
    }
    keep_status st = check_prompt(c, p, &pi, true);
    if (st != KEEP_OK) return st;
    c->last_layer = -1;
    host_kv = p->kv_location == KEEP_KV_PINNED_HOST;
    row_bytes = (size_t)d.n_kv_heads * d.head_dim * c->esz;
    if (cache_rows != 0 && cache_rows < pi.N)
      return fail(c, KEEP_ERR_INVALID_ARG, "cache_rows %d below the prompt's %d tokens", cache_rows, pi.N);
    layer_bytes = (size_t)(cache_rows ? cache_rows : pi.N) * row_bytes;
    c->ev_light = false;
    if (report) {
      c->ev_light = report->events_in == KEEP_REPORT_EVENTS_GATE_UP;
      const int32_t events_in = report->events_in;
      memset(report, 0, sizeof *report);
      report->events_in = events_in;
      report->n_layers = L;
      report->used_mfma = c->mfma ? 1 : 0;
    }
    ld = Loader{c, p, &pi, k_cache, v_cache, row_bytes, layer_bytes};
    if (host_kv) {
      ld.loaded.assign((size_t)L * pi.G, 0);
      ld.chunk_bytes.assign(c->ev_chunk.size(), 0);
    }
    st = upload_tokens(c, p, pi);
    if (st != KEEP_OK) return st;
    if (ratios[0] == 1.f)
      for (int g = 0; g < pi.G; ++g) cur.push_back(g);
    x_cur = c->xa;
    x_nxt = c->xb;
    part_attn_ms.assign((size_t)L, 0.f);
    if (host_kv) {  // what layer 0 needs must be there before it starts
      st = ld.copy_outside(0, cur);
      if (st != KEEP_OK) return st;
      HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
      HIP_TRY(c, hipStreamWaitEvent(c->s_comp, c->ev_load, 0));
      if (report) report->bytes_loaded[0] = ld.bytes_total;
    }
    for (l = 0; l < L; ++l) {
      st = one_layer();
      if (st != KEEP_OK) return st;
    }
    if (x_final) {  // final hidden rows of the instruction
      const char* src = (const char*)x_nxt + (size_t)(plan.n_rows - pi.Lq) * d.hidden * c->esz;
      HIP_TRY(c, hipMemcpyAsync(x_final, src, (size_t)pi.Lq * d.hidden * c->esz, hipMemcpyDeviceToDevice, c->s_comp));
    }
    HIP_TRY(c, hipStreamSynchronize(c->s_copy));
    HIP_TRY(c, hipStreamSynchronize(c->s_eval));
    HIP_TRY(c, hipStreamSynchronize(c->s_comp));
    if (report) {
      report->ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
      read_event_times();
    }
    return KEEP_OK;
  }
};

// x_final may be NULL (the hidden rows are not wanted).  cache_rows: rows per layer of the caches, 0 = N.
keep_status prefill_impl(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t hops, int32_t budget_mode,
                         int32_t load_mode, void* k_cache, void* v_cache, int32_t cache_rows, void* x_final,
                         int32_t* sel_groups, int32_t* sel_counts, keep_report* report) {
  PrefillRun run{c, p, ratios, hops, budget_mode, load_mode, (char*)k_cache, (char*)v_cache, x_final, sel_groups,
                 sel_counts, report};
  return run.run(cache_rows);
}


// Token-granularity prefill (the comparison scheme of Section 3 and Section 4.2, "System advantage"): the rows of
// a layer are single tokens; every cached block is loaded and re-aligned, the recomputed tokens' K/V are written
// over their rows in place, and the tokens of the next layer are the ones whose K/V moved furthest.  The
// deviation is known right after the K/V projection, so the selection runs before the attention and the
// attention, output projection and FFN are computed for the surviving tokens only (the others' hidden rows
// would be discarded).
template <typename T>
keep_status prefill_tokens_impl(keep_ctx* c, const keep_prompt* p, const float* ratios, int32_t load_mode, void* k_cache,
                                void* v_cache, void* x_final, int32_t* sel_rows, int32_t* sel_counts,
                                float* deviation_out, keep_report* report) {
  const auto t_begin = std::chrono::steady_clock::now();
  const keep_model_desc& d = c->d;
  const int L = d.n_layers;
  if (!ratios || !k_cache || !v_cache) return fail(c, KEEP_ERR_INVALID_ARG, "ratios / k_cache / v_cache is NULL");
  if (load_mode < KEEP_LOAD_SERIAL || load_mode > KEEP_LOAD_LAYER_BALANCED)
    return fail(c, KEEP_ERR_INVALID_ARG, "unknown load_mode");
  if (ratios[0] != 0.f && ratios[0] != 1.f)
    return fail(c, KEEP_ERR_INVALID_ARG, "ratios[0] must be 1 (recompute every token at the first layer) or 0");
  for (int l = 1; l < L; ++l) {
    if (!(ratios[l] >= 0.f && ratios[l] <= 1.f)) return fail(c, KEEP_ERR_INVALID_ARG, "ratios[%d] outside [0, 1]", l);
    if (ratios[l] > ratios[l - 1])
      return fail(c, KEEP_ERR_INVALID_ARG, "ratios must not increase (ratios[%d] > ratios[%d])", l, l - 1);
  }
  PromptInfo pi;
  keep_status st = check_prompt(c, p, &pi, true);
  if (st != KEEP_OK) return st;
  c->last_layer = -1;
  c->att_plan.valid = false;
  const bool host_kv = p->kv_location == KEEP_KV_PINNED_HOST;
  const size_t row_bytes = (size_t)d.n_kv_heads * d.head_dim * c->esz;
  const size_t layer_bytes = (size_t)pi.N * row_bytes;
  const int qd = d.n_q_heads * d.head_dim;
  hipStream_t s = c->s_comp;
  c->ev_light = false;
  if (report) {
    memset(report, 0, sizeof *report);
    report->n_layers = L;
    report->used_mfma = c->mfma ? 1 : 0;
  }
  Loader ld{c, p, &pi, (char*)k_cache, (char*)v_cache, row_bytes, layer_bytes};
  if (host_kv) {
    ld.loaded.assign((size_t)L * pi.G, 0);
    ld.chunk_bytes.assign(c->ev_chunk.size(), 0);
  }
  st = upload_tokens(c, p, pi);
  if (st != KEEP_OK) return st;
  const std::vector<int32_t> nothing;
  std::vector<int32_t> cur, nxt;  // positions of the memory tokens recomputed at this layer / the next
  if (ratios[0] == 1.f)
    for (int t = 0; t < pi.n_mem; ++t) cur.push_back(t);
  void* x_cur = c->xa;
  void* x_nxt = c->xb;
  bool from_embed = true;
  int n_out = 0;
  LayerPlan plan;
  auto upload_positions = [&](const std::vector<int32_t>& mem_pos) -> keep_status {
    if (c->rowlist_pending) {
      HIP_TRY(c, hipEventSynchronize(c->ev_rowlist));
      c->rowlist_pending = false;
    }
    const int nm = (int)mem_pos.size();
    if (nm) memcpy(c->h_row_list, mem_pos.data(), (size_t)nm * 4);
    for (int j = 0; j < pi.Lq; ++j) c->h_row_list[nm + j] = pi.n_mem + j;
    HIP_TRY(c, hipMemcpyAsync(c->d_row_pos, c->h_row_list, (size_t)(nm + pi.Lq) * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(c, hipEventRecord(c->ev_rowlist, s));
    c->rowlist_pending = true;
    return KEEP_OK;
  };
  auto attend_rows = [&](const void* q_rows, int n_rows, void* kl, void* vl) -> keep_status {
    if (c->mfma)
      launch_attn_mfma(reinterpret_cast<const bf16_t*>(q_rows), reinterpret_cast<const bf16_t*>(kl),
                       reinterpret_cast<const bf16_t*>(vl), c->d_row_pos, nullptr, nullptr, 0, pi.n_mem, n_rows, pi.N,
                       d.n_q_heads, d.n_kv_heads, d.max_tokens, c->stage[0].attn_items, c->attn_scratch,
                       reinterpret_cast<bf16_t*>(c->o), c->lse, s, nullptr, nullptr, nullptr, nullptr, nullptr, 0,
                       c->h_row_list);
    else
      launch_attn_generic<T>(Typed<T>::p(q_rows), Typed<T>::p(kl), Typed<T>::p(vl), c->d_row_pos, n_rows, d.n_q_heads,
                             d.n_kv_heads, d.head_dim, Typed<T>::p(c->o), c->lse, s);
    HIP_TRY(c, hipGetLastError());
    return KEEP_OK;
  };

  if (host_kv) {  // the whole cache of layer 0
    st = ld.copy_outside(0, nothing);
    if (st != KEEP_OK) return st;
    HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
    HIP_TRY(c, hipStreamWaitEvent(s, c->ev_load, 0));
    if (report) report->bytes_loaded[0] = ld.bytes_total;
  }
  for (int l = 0; l < L; ++l) {
    hipEvent_t* evs = report ? &c->ev[(size_t)l * EV_PER_LAYER] : nullptr;
    char* kl = (char*)k_cache + (size_t)l * layer_bytes;
    char* vl = (char*)v_cache + (size_t)l * layer_bytes;
    const keep_layer_weights& w = c->w[l];
    const int n_mem_rows = (int)cur.size();
    const int n = n_mem_rows + pi.Lq;
    if (sel_counts) sel_counts[l] = n_mem_rows;
    if (sel_rows && n_mem_rows) memcpy(sel_rows + (size_t)l * pi.n_mem, cur.data(), (size_t)n_mem_rows * 4);
    // the next layer's blocks are all needed whatever is selected: their load runs beside this layer
    const uint64_t bytes_before = ld.bytes_total;
    if (host_kv && l + 1 < L && load_mode != KEEP_LOAD_SERIAL) {
      st = ld.copy_outside(l + 1, nothing);
      if (st != KEEP_OK) return st;
      HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
    }
    // every group is re-aligned (the whole cache is joined, then tokens are overwritten in place)
    st = stage_layer(c, p, pi, l, nullptr, 0, kl, vl, host_kv, &plan);
    if (st != KEEP_OK) return st;
    // (the work list of the attention goes through staging slot 0: wait for its previous user)
    if (l > 0 && c->stage[0].used) HIP_TRY(c, hipEventSynchronize(c->stage[0].done));
    st = upload_positions(cur);
    if (st != KEEP_OK) return st;
    if (evs) HIP_TRY(c, hipEventRecord(evs[0], s));
    launch_realign<T>(c->d_segs, plan.n_segs, plan.n_realign_rows, d.n_kv_heads, d.head_dim, c->rope_cos, c->rope_sin,
                      Typed<T>::p(kl), Typed<T>::p(vl), s);
    if (evs) HIP_TRY(c, hipEventRecord(evs[1], s));
    if (from_embed)
      launch_embed_gather<T>(Typed<T>::p(c->embed), c->d_token_ids, c->d_row_pos, n, d.hidden, Typed<T>::p(x_cur), s);
    launch_rmsnorm<T>(Typed<T>::p(x_cur), Typed<T>::p(w.ln1), n, d.hidden, d.rms_eps, Typed<T>::p(c->hbuf), s);
    if (evs) HIP_TRY(c, hipEventRecord(evs[2], s));
    GemmB b{};
    b.n_parts = 3;
    b.ptr[0] = w.wq; b.ptr[1] = w.wk; b.ptr[2] = w.wv;
    b.n_rows[0] = qd;
    b.n_rows[1] = b.n_rows[2] = d.n_kv_heads * d.head_dim;
    if (!c->w4.empty()) {
      set_w4(b, 0, c->w4[l].wq);
      set_w4(b, 1, c->w4[l].wk);
      set_w4(b, 2, c->w4[l].wv);
    }
    const int n_qkv = qd + 2 * b.n_rows[1];
    if (c->mfma)
      launch_gemm_mfma(reinterpret_cast<const bf16_t*>(c->hbuf), n, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32, nullptr,
                       c->qkv_raw, s, c->skinny_ws);
    else
      launch_gemm_generic<T>(Typed<T>::p(c->hbuf), n, d.hidden, b, nullptr, n_qkv, EPI_STORE_F32, nullptr, c->qkv_raw, s);
    if (evs) HIP_TRY(c, hipEventRecord(evs[3], s));
    const int k_next = l + 1 < L ? std::max(0, std::min(n_mem_rows, (int)ceil((double)ratios[l + 1] * pi.n_mem - BUDGET_EPS)))
                                 : n_mem_rows;
    const bool shrink = l + 1 < L && k_next < n_mem_rows;
    const bool want_dev = (shrink || deviation_out) && n_mem_rows > 0;
    launch_rope_scatter<T>(c->qkv_raw, Typed<T>::p(w.bq), Typed<T>::p(w.bk), Typed<T>::p(w.bv), c->d_row_pos, n,
                           d.n_q_heads, d.n_kv_heads, d.head_dim, c->rope_cos, c->rope_sin, Typed<T>::p(c->q),
                           Typed<T>::p(c->kc), Typed<T>::p(kl), Typed<T>::p(vl), s, nullptr, want_dev ? c->d_dev : nullptr);
    HIP_TRY(c, hipGetLastError());
    if (evs) {
      HIP_TRY(c, hipEventRecord(evs[4], s));
      HIP_TRY(c, hipEventRecord(evs[10], s));
    }
    if (deviation_out && n_mem_rows) {
      HIP_TRY(c, hipMemcpyAsync(c->h_dev, c->d_dev, (size_t)n_mem_rows * 4, hipMemcpyDeviceToHost, s));
      HIP_TRY(c, hipStreamSynchronize(s));
      memcpy(deviation_out + (size_t)l * pi.n_mem, c->h_dev, (size_t)n_mem_rows * 4);
    }
    int n_back = n;
    if (shrink) {
      // kept rows (ascending compact indices) followed by the instruction rows
      launch_select_tokens(c->d_dev, n_mem_rows, k_next, pi.Lq, c->d_tok_flags, c->d_tok_list, s);
      HIP_TRY(c, hipGetLastError());
      if (k_next) HIP_TRY(c, hipMemcpyAsync(c->h_tok_list, c->d_tok_list, (size_t)k_next * 4, hipMemcpyDeviceToHost, s));
      n_back = k_next + pi.Lq;
      // q rows into the projection's fp32 buffer (free once RoPE has read it), hidden rows into the other row buffer
      launch_rows_gather_list<T>(Typed<T>::p(c->q), c->d_tok_list, n_back, qd, Typed<T>::p(c->qkv_raw), s);
      launch_rows_gather_list<T>(Typed<T>::p(x_cur), c->d_tok_list, n_back, d.hidden, Typed<T>::p(x_nxt), s);
      HIP_TRY(c, hipGetLastError());
      HIP_TRY(c, hipStreamSynchronize(s));  // the host needs the kept rows to plan the attention and the next layer
      nxt.resize(k_next);
      for (int i = 0; i < k_next; ++i) nxt[i] = cur[c->h_tok_list[i]];
      st = upload_positions(nxt);
      if (st != KEEP_OK) return st;
    }
    if (evs) HIP_TRY(c, hipEventRecord(evs[11], s));
    st = attend_rows(shrink ? (const void*)c->qkv_raw : (const void*)c->q, n_back, kl, vl);
    if (st != KEEP_OK) return st;
    if (evs) HIP_TRY(c, hipEventRecord(evs[5], s));
    HIP_TRY(c, hipEventRecord(c->stage[0].done, s));
    c->stage[0].used = true;
    if (shrink) {
      st = layer_back<T>(c, l, n_back, c->o, x_nxt, x_cur, evs);  // output lands in x_cur, in the next layer's layout
      cur.swap(nxt);
    } else {
      st = layer_back<T>(c, l, n_back, c->o, x_cur, x_nxt, evs);
      std::swap(x_cur, x_nxt);
    }
    if (st != KEEP_OK) return st;
    Staging& sg = c->stage[l];
    HIP_TRY(c, hipEventRecord(sg.done, s));
    sg.used = true;
    from_embed = false;
    n_out = n_back;
    if (report) {
      report->rows[l] = n;
      report->set_size[l] = n_mem_rows;
      report->realign_rows[l] = plan.n_realign_rows;
      report->attn_rows[l] = n_back;
      report->ffn_rows[l] = n_back;
    }
    if (host_kv && l + 1 < L) {
      if (load_mode == KEEP_LOAD_SERIAL) {  // load strictly after this layer's compute
        HIP_TRY(c, hipEventRecord(c->ev_comp, s));
        HIP_TRY(c, hipStreamWaitEvent(c->s_copy, c->ev_comp, 0));
        st = ld.copy_outside(l + 1, nothing);
        if (st != KEEP_OK) return st;
        HIP_TRY(c, hipEventRecord(c->ev_load, c->s_copy));
      }
      HIP_TRY(c, hipStreamWaitEvent(s, c->ev_load, 0));
      if (report) report->bytes_loaded[l + 1] = ld.bytes_total - bytes_before;
    }
  }
  {
    const char* src = (const char*)x_cur + (size_t)(n_out - pi.Lq) * d.hidden * c->esz;
    HIP_TRY(c, hipMemcpyAsync(x_final, src, (size_t)pi.Lq * d.hidden * c->esz, hipMemcpyDeviceToDevice, s));
  }
  HIP_TRY(c, hipStreamSynchronize(c->s_copy));
  HIP_TRY(c, hipStreamSynchronize(s));
  if (report) {
    report->ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    for (int l = 0; l < L; ++l) {
      hipEvent_t* e = &c->ev[(size_t)l * EV_PER_LAYER];
      (void)hipEventElapsedTime(&report->ms_realign[l], e[0], e[1]);
      (void)hipEventElapsedTime(&report->ms_prep[l], e[1], e[2]);
      (void)hipEventElapsedTime(&report->ms_qkv_gemm[l], e[2], e[3]);
      (void)hipEventElapsedTime(&report->ms_rope[l], e[3], e[4]);
      (void)hipEventElapsedTime(&report->ms_score[l], e[10], e[11]);
      (void)hipEventElapsedTime(&report->ms_attn[l], e[11], e[5]);
      (void)hipEventElapsedTime(&report->ms_oproj[l], e[12], e[6]);
      (void)hipEventElapsedTime(&report->ms_norm2[l], e[6], e[7]);
      (void)hipEventElapsedTime(&report->ms_gateup[l], e[7], e[8]);
      (void)hipEventElapsedTime(&report->ms_down[l], e[8], e[9]);
    }
  }
  return KEEP_OK;
}

}  // namespace
