// C ABI of libsart (see include/sart.h): argument checks, device memory, the
// staging of small host arrays, and kernel launches.  No arithmetic of the
// method happens on the host.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "sart_internal.h"

using namespace sart;

namespace {

thread_local char g_err[512] = "";

sart_status fail(sart_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
sart_status fail(sart_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

#define HIP_TRY(expr)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) return fail(SART_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr int kStageSlots = 8;
// share of the mean range moved from odd-XCD workgroups to even-XCD ones (measured on MI355X)
constexpr int kDefaultSkewPermille = 80;   // swept 30..110 on configs 2 and 4: 70-90 is the flat optimum

struct StageSlot {
  int* host = nullptr;  // pinned
  int* dev = nullptr;
  hipEvent_t done = nullptr;
};

}  // namespace

struct sart_cache {
  Ctx ctx;
  sart_cache_desc desc;
  int device = 0;
  bool owns_pool = false;
  std::vector<void*> allocs;         // every hipMalloc'ed block except the staging slots
  StageSlot stage[kStageSlots];
  size_t stage_ints = 0;
  int next_slot = 0;
  int call_seq = 0;
  size_t layer_bytes = 0;              // pool bytes of one layer
  float k_scale = 1.0f, v_scale = 1.0f; // 8-bit float caches: stored code * scale is the value
  // the last layer-0 append, which the same step's appends to the other layers must repeat
  int last_kind = -1, last_n_seqs = 0, last_has_ids = 0, last_has_ntok = 0;
  long long last_total = 0;
  std::vector<int> last_ids, last_ntok;
  hipStream_t last_stream = nullptr;
  float* partials = nullptr;
  long long partial_cap = 0;
  PlanCfg plan{0, 0, 0};               // launch shape of the decode plan
  int stagger_prompt = 1;              // see sart_set_prompt_stagger
  int merge_mode = 0;                  // 1: merged inside the attention kernel where it can be, 0: by the merge kernel (faster, measured)
  int max_wg = 0;
  int profiling = 0;                   // 0 off, n >= 1: events around n attention launches
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  bool ev_valid = false;
  int* host_nactive = nullptr;         // pinned host int the kernels store the active count to (sart_active_count_hint)
};

namespace {

template <typename T>
sart_status dev_alloc(sart_cache* c, T** p, size_t n) {
  void* q = nullptr;
  HIP_TRY(hipMalloc(&q, (n ? n : 1) * sizeof(T)));
  c->allocs.push_back(q);
  *p = (T*)q;
  return SART_OK;
}

// Takes the next staging slot (waiting for the call that used it last) and
// returns its pinned host buffer.
sart_status stage_begin(sart_cache* c, StageSlot** slot) {
  StageSlot* s = &c->stage[c->next_slot];
  c->next_slot = (c->next_slot + 1) % kStageSlots;
  HIP_TRY(hipEventSynchronize(s->done));
  *slot = s;
  return SART_OK;
}

sart_status stage_upload(sart_cache* c, StageSlot* s, size_t n_ints, hipStream_t st) {
  (void)c;
  if (n_ints) HIP_TRY(hipMemcpyAsync(s->dev, s->host, n_ints * sizeof(int), hipMemcpyHostToDevice, st));
  return SART_OK;
}

sart_status check_desc(const sart_cache_desc* d) {
  if (!d) return fail(SART_E_INVALID, "null description");
  if (d->n_layers < 1 || d->n_layers > 1024) return fail(SART_E_INVALID, "n_layers must be in [1, 1024]");
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads)
    return fail(SART_E_INVALID, "n_q_heads must be a positive multiple of n_kv_heads");
  if (d->head_dim <= 0 || d->head_dim % 8 || d->head_dim > 256)
    return fail(SART_E_INVALID, "head_dim must be a multiple of 8, at most 256");
  if (d->page_tokens <= 0 || d->num_pages <= 0 || d->max_requests <= 0 || d->branches_per_request <= 0)
    return fail(SART_E_INVALID, "page_tokens, num_pages, max_requests, branches_per_request must be positive");
  if (d->max_pages_per_branch <= 0 || d->max_prefix_pages <= 0)
    return fail(SART_E_INVALID, "max_pages_per_branch and max_prefix_pages must be positive");
  if (d->kv_dtype != SART_F32 && d->kv_dtype != SART_BF16 && d->kv_dtype != SART_FP8_E4M3)
    return fail(SART_E_INVALID, "unknown kv_dtype");
  if (d->kv_dtype == SART_FP8_E4M3 &&
      (d->page_tokens != 16 || (d->head_dim != 64 && d->head_dim != 128) || d->n_q_heads / d->n_kv_heads > kMaxGroup ||
       d->force_natural_layout))
    return fail(SART_E_INVALID, "SART_FP8_E4M3 needs page_tokens 16, head_dim 64 or 128, Hq/Hkv <= 16, no forced layout");
  if ((long long)d->max_requests * d->branches_per_request > (1 << 22))
    return fail(SART_E_INVALID, "max_requests * branches_per_request too large");
  return SART_OK;
}

int pick_layout(const sart_cache_desc* d) {
  const int G = d->n_q_heads / d->n_kv_heads;
  if (d->kv_dtype == SART_FP8_E4M3) return SART_LAYOUT_MFMA16_FP8;
  if (!d->force_natural_layout && d->kv_dtype == SART_BF16 && d->page_tokens == 16 &&
      (d->head_dim == 64 || d->head_dim == 128) && G <= kMaxGroup)
    return SART_LAYOUT_MFMA16;
  return SART_LAYOUT_NATURAL;
}

void note_stream(sart_cache* c, void* stream) { c->last_stream = (hipStream_t)stream; }

}  // namespace

extern "C" {

const char* sart_last_error(void) { return g_err; }

size_t sart_pool_bytes(const sart_cache_desc* d) {
  if (!d) return 0;
  const size_t es = d->kv_dtype == SART_F32 ? 4 : (d->kv_dtype == SART_FP8_E4M3 ? 1 : 2);
  return (size_t)(d->n_layers > 0 ? d->n_layers : 1) * d->num_pages * d->page_tokens * 2 * d->n_kv_heads * d->head_dim * es;
}

// The layer's slice of the pool: [layer][page][kv head][K tile | V tile].
static Ctx layer_ctx(const sart_cache* c, int layer) {
  Ctx x = c->ctx;
  x.pool = (char*)c->ctx.pool + (size_t)layer * c->layer_bytes;
  return x;
}

sart_status sart_alloc_cache(const sart_cache_desc* d, sart_cache** out) {
  if (!out) return fail(SART_E_INVALID, "null out");
  *out = nullptr;
  sart_status st = check_desc(d);
  if (st != SART_OK) return st;
  const size_t pool_bytes = sart_pool_bytes(d);
  if (d->kv_pool && d->kv_pool_bytes < pool_bytes)
    return fail(SART_E_INVALID, "kv_pool_bytes %zu < required %zu", d->kv_pool_bytes, pool_bytes);
  if (d->initial_free_order) {
    std::vector<char> seen(d->num_pages, 0);
    for (int i = 0; i < d->num_pages; ++i) {
      const int p = d->initial_free_order[i];
      if (p < 0 || p >= d->num_pages || seen[p]) return fail(SART_E_INVALID, "initial_free_order is not a permutation");
      seen[p] = 1;
    }
  }
  sart_cache* c = new sart_cache();
  // any early return below (a failed HIP call, a failed allocation) releases what exists so far
  struct Guard {
    sart_cache* c;
    ~Guard() { if (c) sart_free_cache(c); }
  } guard{c};
  c->desc = *d;
  c->layer_bytes = pool_bytes / d->n_layers;
  c->desc.initial_free_order = nullptr;
  HIP_TRY(hipGetDevice(&c->device));
  Dims& dm = c->ctx.dm;
  dm.Hq = d->n_q_heads; dm.Hkv = d->n_kv_heads; dm.G = dm.Hq / dm.Hkv; dm.d = d->head_dim;
  dm.pt = d->page_tokens; dm.num_pages = d->num_pages; dm.max_req = d->max_requests;
  dm.Nb = d->branches_per_request; dm.Q = d->finish_quota; dm.max_bp = d->max_pages_per_branch;
  dm.max_pp = d->max_prefix_pages; dm.H = dm.max_req * dm.Nb; dm.dtype = d->kv_dtype;
  dm.layout = pick_layout(d); dm.esize = d->kv_dtype == SART_F32 ? 4 : (d->kv_dtype == SART_FP8_E4M3 ? 1 : 2);
  c->k_scale = d->kv_dtype == SART_FP8_E4M3 && d->k_scale > 0.f ? d->k_scale : 1.0f;
  c->v_scale = d->kv_dtype == SART_FP8_E4M3 && d->v_scale > 0.f ? d->v_scale : 1.0f;
  dm.k_scale = c->k_scale; dm.v_scale = c->v_scale;
  dm.start_waiting = d->branches_start_waiting != 0;
  dm.tile_elems = (long long)dm.pt * dm.d;
  dm.page_elems = (long long)dm.Hkv * 2 * dm.tile_elems;

  Tables& tb = c->ctx.tb;
  const size_t H = dm.H, R = dm.max_req;
#define ALLOC(ptr, n)                                           \
  do {                                                          \
    st = dev_alloc(c, &(ptr), (n));                             \
    if (st != SART_OK) return st;                               \
  } while (0)
  ALLOC(tb.scal, S_COUNT);
  ALLOC(tb.free_stack, dm.num_pages);
  ALLOC(tb.req_used, R); ALLOC(tb.prefix_len, R); ALLOC(tb.prefix_table, R * dm.max_pp);
  ALLOC(tb.refcnt, R); ALLOC(tb.nact, R); ALLOC(tb.req_tmp, R); ALLOC(tb.num_completed, R); ALLOC(tb.num_pruned, R); ALLOC(tb.branch_appended, R);
  ALLOC(tb.br_state, H); ALLOC(tb.active_idx_of, H); ALLOC(tb.active, H); ALLOC(tb.seq_len, H);
  ALLOC(tb.bt[0], H * dm.max_bp); ALLOC(tb.bt[1], H * dm.max_bp);
  ALLOC(tb.new_state, H); ALLOC(tb.mv_push_off, H); ALLOC(tb.mv_new_idx, H);
  ALLOC(tb.tmp_a, H); ALLOC(tb.tmp_b, H);
  ALLOC(tb.req_first, R); ALLOC(tb.req_push_off, R); ALLOC(tb.req_touched, R);
  ALLOC(tb.ap_id, H); ALLOC(tb.ap_start, H);
  ALLOC(tb.page_cum, H + 1); ALLOC(tb.live_req, R); ALLOC(tb.live_item_start, R + 1);

  if (d->kv_pool) {
    c->ctx.pool = d->kv_pool;
  } else {
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, pool_bytes);
    if (e != hipSuccess) return fail(SART_E_HIP, "hipMalloc(pool %zu B): %s", pool_bytes, hipGetErrorString(e));
    c->allocs.push_back(p);
    c->ctx.pool = p;
    c->owns_pool = true;
  }

  // decode launch shape: a persistent grid of kAttnWaves-wave workgroups
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, c->device));
  const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c->max_wg = cus * 16;
  c->plan.n_wg = cus;                // one 4-wave workgroup per CU, one wave per SIMD
  // prompt blocks read once per tile of 16 query rows of the request (matrix-core layouts), per branch otherwise
  c->plan.prompt_mode = dm.layout == SART_LAYOUT_NATURAL ? 1 : 0;    // 0: the planning kernel chooses per step
  c->plan.skew_permille = kDefaultSkewPermille;
  ALLOC(tb.wave_row, (size_t)2 * c->max_wg * kAttnWaves);
  ALLOC(tb.req_pstart, R);
  ALLOC(tb.wave_desc, (size_t)16 * c->max_wg * kAttnWaves);
  ALLOC(tb.row_desc, 8 * H);
  ALLOC(tb.pf_seq, 4 * R);
  ALLOC(tb.mv_first, H);
  ALLOC(tb.page_extra, (size_t)dm.num_pages);
  ALLOC(tb.page_owner, (size_t)dm.num_pages);
  HIP_TRY(hipMemset(tb.mv_first, 0, H * sizeof(int)));
  HIP_TRY(hipMemset(tb.page_extra, 0, (size_t)dm.num_pages * sizeof(int)));
  HIP_TRY(hipMemset(tb.page_owner, 0xff, (size_t)dm.num_pages * sizeof(int)));
  ALLOC(tb.seg_count, H * dm.Hkv);
  HIP_TRY(hipMemset(tb.seg_count, 0, H * dm.Hkv * sizeof(int)));
  HIP_TRY(hipHostMalloc((void**)&c->host_nactive, 64, hipHostMallocMapped));
  *c->host_nactive = 0;
  HIP_TRY(hipHostGetDevicePointer((void**)&tb.host_nactive, c->host_nactive, 0));
  // partial slots: one per own range (wave), one per (row, kv head) a range boundary falls in, and the prompts'
  // blocks, which the planning kernel keeps to max(S, 4 per wave)
  const long long S = (long long)H * dm.Hkv, max_waves = (long long)c->max_wg * kAttnWaves;
  c->partial_cap = max_waves + S + (S > 4 * max_waves ? S : 4 * max_waves);
  const long long pf = (long long)dm.G * dm.d + ((2 * dm.G + 3) & ~3);
  ALLOC(c->partials, (size_t)(c->partial_cap * pf));
#undef ALLOC

  // staging slots for small host arrays (ids, counts, offsets, policy arrays)
  c->stage_ints = 3 * H + 4 * R + 16;
  for (int i = 0; i < kStageSlots; ++i) {
    HIP_TRY(hipHostMalloc((void**)&c->stage[i].host, c->stage_ints * sizeof(int), hipHostMallocDefault));
    HIP_TRY(hipMalloc((void**)&c->stage[i].dev, c->stage_ints * sizeof(int)));
    HIP_TRY(hipEventCreateWithFlags(&c->stage[i].done, hipEventDisableTiming));
  }
  for (int i = 0; i < 4; ++i) HIP_TRY(hipEventCreate(&c->ev[i]));

  // tables + zero-filled pool
  int* order_dev = nullptr;
  if (d->initial_free_order) {
    st = dev_alloc(c, &order_dev, (size_t)dm.num_pages);     // in the cache's list: released on every error path
    if (st != SART_OK) return st;
    HIP_TRY(hipMemcpy(order_dev, d->initial_free_order, (size_t)dm.num_pages * sizeof(int), hipMemcpyHostToDevice));
  }
  launch_init_tables(c->ctx, order_dev, nullptr);
  launch_plan(c->ctx, c->plan, nullptr);
  HIP_TRY(hipMemsetAsync(c->ctx.pool, 0, pool_bytes, nullptr));
  HIP_TRY(hipStreamSynchronize(nullptr));
  if (order_dev) {
    c->allocs.pop_back();                                     // the last block allocated
    HIP_TRY(hipFree(order_dev));
  }
  HIP_TRY(hipGetLastError());
  guard.c = nullptr;
  *out = c;
  return SART_OK;
}

sart_status sart_free_cache(sart_cache* c) {
  if (!c) return SART_OK;
  (void)hipDeviceSynchronize();
  for (void* p : c->allocs) (void)hipFree(p);
  for (int i = 0; i < kStageSlots; ++i) {
    if (c->stage[i].host) (void)hipHostFree(c->stage[i].host);
    if (c->stage[i].dev) (void)hipFree(c->stage[i].dev);
    if (c->stage[i].done) (void)hipEventDestroy(c->stage[i].done);
  }
  for (int i = 0; i < 4; ++i)
    if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
  if (c->host_nactive) (void)hipHostFree(c->host_nactive);
  delete c;
  return SART_OK;
}

int32_t sart_cache_layout(const sart_cache* c) { return c ? c->ctx.dm.layout : -1; }

// One token for every active branch, the count read on the device.  n_seqs = -rows of k and v; by_handle: the
// rows are addressed by branch handle (then rows = max_requests * Nb).
static sart_status append_all_active(sart_cache* c, int n_seqs, int by_handle, const void* k, const void* v, int32_t layer,
                                     void* stream) {
  const Dims& dm = c->ctx.dm;
  const int kind = SART_SEQ_BRANCH;
  if (!k || !v) return fail(SART_E_INVALID, "null k or v");
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  AppendArgs a{};
  a.kind = kind; a.n_seqs = n_seqs; a.total_rows = n_seqs < -dm.H ? dm.H : -n_seqs; a.k = k; a.v = v;
  a.call_seq = ++c->call_seq;
  a.write_only = layer > 0;
  a.by_handle = by_handle;
  const long long mark = by_handle ? -2 : -1;               // what a layer > 0 append of the same step must repeat
  if (layer == 0) { c->last_kind = kind; c->last_n_seqs = n_seqs; c->last_has_ids = 0; c->last_has_ntok = 0; c->last_total = mark; }
  else if (c->last_kind != kind || c->last_n_seqs != n_seqs || c->last_total != mark)
    return fail(SART_E_INVALID, "an append to layer %d must repeat the step's layer-0 append", layer);
  launch_append(layer_ctx(c, layer), c->plan, a, st);
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_append_tokens(sart_cache* c, int32_t kind, int32_t n_seqs, const int32_t* ids,
                               const int32_t* n_tokens, const void* k, const void* v, int32_t layer,
                               void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  const Dims& dm = c->ctx.dm;
  if (layer < 0 || layer >= c->desc.n_layers) return fail(SART_E_INVALID, "layer out of range");
  if (kind != SART_SEQ_PREFIX && kind != SART_SEQ_BRANCH) return fail(SART_E_INVALID, "unknown sequence kind");
  if (n_seqs < 0 && kind == SART_SEQ_BRANCH && !ids && !n_tokens)     // SART_ALL_ACTIVE(rows)
    return append_all_active(c, n_seqs, 0, k, v, layer, stream);
  if (n_seqs < 0) return fail(SART_E_INVALID, "negative n_seqs");
  if (kind == SART_SEQ_PREFIX && !ids && n_seqs > 0) return fail(SART_E_INVALID, "prefix append needs request ids");
  const int limit = kind == SART_SEQ_PREFIX ? dm.max_req : dm.H;
  if (n_seqs > limit) return fail(SART_E_INVALID, "more sequences than exist");
  long long total = 0;
  if (ids) {
    std::vector<char> seen(limit, 0);
    for (int i = 0; i < n_seqs; ++i) {
      if (ids[i] < 0 || ids[i] >= limit) return fail(SART_E_INVALID, "id %d out of range at %d", ids[i], i);
      if (seen[ids[i]]) return fail(SART_E_INVALID, "duplicate id %d", ids[i]);
      seen[ids[i]] = 1;
    }
  }
  if (n_tokens) {
    for (int i = 0; i < n_seqs; ++i) {
      if (n_tokens[i] < 0) return fail(SART_E_INVALID, "negative token count at %d", i);
      total += n_tokens[i];
    }
    if (total > 0x7fffffffLL) return fail(SART_E_INVALID, "too many tokens in one call");
  } else {
    total = n_seqs;
  }
  if (total > 0 && (!k || !v)) return fail(SART_E_INVALID, "null k or v");
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  AppendArgs a{};
  a.kind = kind; a.n_seqs = n_seqs; a.total_rows = total; a.k = k; a.v = v; a.call_seq = ++c->call_seq;
  a.write_only = layer > 0;
  if (layer == 0) {
    c->last_kind = kind; c->last_n_seqs = n_seqs; c->last_has_ids = ids != nullptr; c->last_has_ntok = n_tokens != nullptr;
    c->last_total = total;
    c->last_ids.assign(ids ? ids : nullptr, ids ? ids + n_seqs : nullptr);
    c->last_ntok.assign(n_tokens ? n_tokens : nullptr, n_tokens ? n_tokens + n_seqs : nullptr);
  } else if (c->last_kind != kind || c->last_n_seqs != n_seqs || c->last_has_ids != (ids != nullptr) ||
             c->last_has_ntok != (n_tokens != nullptr) || c->last_total != total ||
             (ids && memcmp(ids, c->last_ids.data(), (size_t)n_seqs * sizeof(int)) != 0) ||
             (n_tokens && memcmp(n_tokens, c->last_ntok.data(), (size_t)n_seqs * sizeof(int)) != 0)) {
    return fail(SART_E_INVALID, "an append to layer %d must repeat the step's layer-0 append (kind, ids, counts)", layer);
  }
  const Ctx lctx = layer_ctx(c, layer);
  if (ids || n_tokens) {
    StageSlot* s;
    sart_status rc = stage_begin(c, &s);
    if (rc != SART_OK) return rc;
    size_t off = 0;
    if (ids) { memcpy(s->host + off, ids, (size_t)n_seqs * sizeof(int)); a.ids = s->dev + off; off += n_seqs; }
    if (n_tokens) {
      memcpy(s->host + off, n_tokens, (size_t)n_seqs * sizeof(int));
      a.ntok = s->dev + off; off += n_seqs;
      int run = 0;
      for (int i = 0; i < n_seqs; ++i) { s->host[off + i] = run; run += n_tokens[i]; }
      a.tok_off = s->dev + off; off += n_seqs;
    }
    rc = stage_upload(c, s, off, st);
    if (rc != SART_OK) return rc;
    launch_append(lctx, c->plan, a, st);
    HIP_TRY(hipEventRecord(s->done, st));
  } else {
    launch_append(lctx, c->plan, a, st);
  }
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_append_active_by_handle(sart_cache* c, const void* k, const void* v, int32_t layer, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (layer < 0 || layer >= c->desc.n_layers) return fail(SART_E_INVALID, "layer out of range");
  return append_all_active(c, -c->ctx.dm.H, 1, k, v, layer, stream);
}

int32_t sart_active_count_hint(const sart_cache* c) {
  return c && c->host_nactive ? *(volatile const int*)c->host_nactive : -1;
}

// Shared by the two decode entry points: `partials` / `partial_cap` name the scratch the kernels use.
static sart_status decode_common(sart_cache* c, int32_t layer, const void* q, float* out, int32_t n_rows, float scale,
                                 void* stream, float* partials, long long partial_cap, int* seg_count, bool profile,
                                 bool by_handle = false) {
  const Dims& dm = c->ctx.dm;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)dm.d);
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  DecodeArgs a{};
  a.q = q; a.out = out; a.n_rows = n_rows;
  a.scale_log2 = scale * 1.44269504088896340736f * c->k_scale;
  a.v_scale = c->v_scale;
  a.n_wg = c->plan.n_wg;
  a.partials = partials; a.partial_cap = partial_cap; a.seg_count = seg_count;
  a.fused_merge = c->merge_mode;
  a.stagger_prompt = c->stagger_prompt;
  a.by_handle = by_handle;
  a.call_seq = ++c->call_seq;
  for (int i = 0; i < 4; ++i) a.ev[i] = profile && c->profiling ? c->ev[i] : nullptr;
  a.repeats = profile ? c->profiling : 0;
  launch_decode(layer_ctx(c, layer), a, st);
  if (profile) c->ev_valid = c->profiling > 0;
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

static sart_status check_decode_args(sart_cache* c, int32_t layer, const void* q, float* out, int32_t n_rows) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (layer < 0 || layer >= c->desc.n_layers) return fail(SART_E_INVALID, "layer out of range");
  if (n_rows < 0) return fail(SART_E_INVALID, "negative n_rows");
  if (n_rows > 0 && (!q || !out)) return fail(SART_E_INVALID, "null q or out");
  return SART_OK;
}

sart_status sart_decode_attention(sart_cache* c, int32_t layer, const void* q, float* out, int32_t n_rows,
                                  float scale, void* stream) {
  sart_status rc = check_decode_args(c, layer, q, out, n_rows);
  if (rc != SART_OK) return rc;
  return decode_common(c, layer, q, out, n_rows, scale, stream, c->partials, c->partial_cap, c->ctx.tb.seg_count, true);
}

sart_status sart_decode_attention_by_handle(sart_cache* c, int32_t layer, const void* q, float* out, float scale,
                                            void* stream) {
  const int n_rows = c ? c->ctx.dm.H : 0;
  sart_status rc = check_decode_args(c, layer, q, out, n_rows);
  if (rc != SART_OK) return rc;
  return decode_common(c, layer, q, out, n_rows, scale, stream, c->partials, c->partial_cap, c->ctx.tb.seg_count, true, true);
}

sart_status sart_decode_attention_static(sart_cache* c, int32_t layer, const void* q, float* out, int32_t n_rows,
                                         float scale, void* stream) {
  sart_status rc = check_decode_args(c, layer, q, out, n_rows);
  if (rc != SART_OK) return rc;
  const Dims& dm = c->ctx.dm;
  // the current device's copy of the scratch array (looked up once per device)
  int dev = -1;
  void* scratch_ptr = nullptr;
  HIP_TRY(static_scratch(&dev, &scratch_ptr));
  if (dev != c->device) return fail(SART_E_INVALID, "the cache lives on device %d but device %d is current", c->device, dev);
  // The array holds the merge's arrival counters (one int per (row, kv head), zero between kernels: the
  // image starts zeroed and every kernel leaves them so), then the partial results.  What a step over
  // n_rows rows can need at most (see refresh_decode_plan): own pieces, then prompt blocks.
  const long long pf_bytes = partial_floats(dm.G, dm.d) * (long long)sizeof(float);
  const long long cap = (long long)(kStaticScratchBytes - kStaticCounterBytes) / pf_bytes;
  const long long rows = n_rows < dm.H ? n_rows : dm.H, S = rows * dm.Hkv, waves = (long long)c->plan.n_wg * kAttnWaves;
  const long long need = waves + S + (S > 4 * waves ? S : 4 * waves);
  if (need > cap || S * (long long)sizeof(int) > (long long)kStaticCounterBytes)
    return fail(SART_E_INVALID, "n_rows %d with %d kv heads and %d workgroups may need %lld partial results of %lld bytes: "
                "more than the static scratch of %zu bytes holds (%lld, and %zu (row, kv head) pairs)", n_rows, dm.Hkv,
                c->plan.n_wg, need, pf_bytes, (size_t)kStaticScratchBytes, cap, (size_t)kStaticCounterBytes / sizeof(int));
  return decode_common(c, layer, q, out, n_rows, scale, stream, (float*)((char*)scratch_ptr + kStaticCounterBytes), cap,
                       (int*)scratch_ptr, false);
}

sart_status sart_prefill_attention(sart_cache* c, int32_t layer, int32_t n_seqs, const int32_t* request_ids,
                                   const int32_t* n_q, const void* q, float* out, float scale, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (layer < 0 || layer >= c->desc.n_layers) return fail(SART_E_INVALID, "layer out of range");
  const Dims& dm = c->ctx.dm;
  if (n_seqs < 0 || n_seqs > dm.max_req || n_seqs > 65535) return fail(SART_E_INVALID, "n_seqs out of range (at most max_requests and 65535)");
  if (n_seqs > 0 && (!request_ids || !n_q)) return fail(SART_E_INVALID, "null request_ids or n_q");
  long long total = 0, max_nq = 0;
  for (int i = 0; i < n_seqs; ++i) {
    if (request_ids[i] < 0 || request_ids[i] >= dm.max_req)
      return fail(SART_E_INVALID, "request %d out of range at %d", request_ids[i], i);
    if (n_q[i] < 0 || n_q[i] > dm.max_pp * dm.pt) return fail(SART_E_INVALID, "n_q out of range at %d", i);
    total += n_q[i];
    if (n_q[i] > max_nq) max_nq = n_q[i];
  }
  const int rows_per_tile = prefill_tile_rows(dm, max_nq * dm.G);     // the matrix-core kernel's workgroup tile
  long long tiles_per_head = (max_nq * dm.G + rows_per_tile - 1) / rows_per_tile;
  if (rows_per_tile == 2 * kPfTileRows) tiles_per_head = (tiles_per_head + 1) / 2;   // those workgroups take two tiles each
  const long long max_tiles = (long long)dm.Hkv * tiles_per_head;                    // grid x: workgroups of the longest sequence
  if (total > 0x7fffffffLL / dm.Hq || max_tiles > 0x7fffffffLL) return fail(SART_E_INVALID, "too many queries in one call");
  if (total > 0 && (!q || !out)) return fail(SART_E_INVALID, "null q or out");
  if (n_seqs == 0) return SART_OK;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)dm.d);
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  StageSlot* s;
  sart_status rc = stage_begin(c, &s);
  if (rc != SART_OK) return rc;
  PrefillArgs a{};
  a.n_seqs = n_seqs; a.q = q; a.out = out; a.call_seq = ++c->call_seq;
  a.scale_log2 = scale * 1.44269504088896340736f * c->k_scale;
  a.v_scale = c->v_scale;
  a.total_q = (int)total; a.max_tiles = (int)max_tiles; a.tile_rows = rows_per_tile;
  int* hbuf = s->host;
  int qo = 0;
  for (int i = 0; i < n_seqs; ++i) {
    hbuf[i] = request_ids[i];
    hbuf[n_seqs + i] = n_q[i];
    hbuf[2 * n_seqs + i] = qo;
    qo += n_q[i];
  }
  a.ids = s->dev; a.nq = s->dev + n_seqs; a.q_off = s->dev + 2 * n_seqs;
  rc = stage_upload(c, s, (size_t)3 * n_seqs, st);
  if (rc != SART_OK) return rc;
  launch_prefill(layer_ctx(c, layer), a, st);
  HIP_TRY(hipEventRecord(s->done, st));
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_prune_branches(sart_cache* c, const sart_prune_policy* pol, const float* scores,
                                int32_t n_scores, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (!pol) return fail(SART_E_INVALID, "null policy");
  if (pol->mode < 0 || pol->mode > 2) return fail(SART_E_INVALID, "unknown prune mode");
  if (!scores || n_scores < 0) return fail(SART_E_INVALID, "null scores");
  if (pol->mode == SART_PRUNE_THRESHOLD && !pol->threshold) return fail(SART_E_INVALID, "threshold mode needs thresholds");
  if (pol->mode != SART_PRUNE_THRESHOLD && !pol->k_per_request && pol->k < 0) return fail(SART_E_INVALID, "negative k");
  const Dims& dm = c->ctx.dm;
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  PruneArgs a{};
  a.mode = pol->mode; a.k = pol->k; a.scores = scores; a.n_scores = n_scores; a.call_seq = ++c->call_seq;
  const bool need_stage = pol->k_per_request || pol->max_pruned || pol->mode == SART_PRUNE_THRESHOLD;
  if (need_stage) {
    StageSlot* s;
    sart_status rc = stage_begin(c, &s);
    if (rc != SART_OK) return rc;
    size_t off = 0;
    const size_t R = dm.max_req;
    if (pol->mode != SART_PRUNE_THRESHOLD && pol->k_per_request) {
      memcpy(s->host + off, pol->k_per_request, R * sizeof(int)); a.k_per_req = s->dev + off; off += R;
    }
    if (pol->mode == SART_PRUNE_THRESHOLD) {
      memcpy(s->host + off, pol->threshold, R * sizeof(float)); a.thr = (const float*)(s->dev + off); off += R;
    }
    if (pol->max_pruned) {
      memcpy(s->host + off, pol->max_pruned, R * sizeof(int)); a.maxp = s->dev + off; off += R;
    }
    rc = stage_upload(c, s, off, st);
    if (rc != SART_OK) return rc;
    launch_prune(c->ctx, c->plan, a, st);
    HIP_TRY(hipEventRecord(s->done, st));
  } else {
    launch_prune(c->ctx, c->plan, a, st);
  }
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_finish_branch(sart_cache* c, int32_t n, const int32_t* handles, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  const Dims& dm = c->ctx.dm;
  if (n < 0 || (n > 0 && !handles)) return fail(SART_E_INVALID, "bad handle list");
  if (n > dm.H) return fail(SART_E_INVALID, "more handles than branches");
  if (n == 0) return SART_OK;  // nothing completes: the state does not change
  {
    std::vector<char> seen(dm.H, 0);
    for (int i = 0; i < n; ++i) {
      if (handles[i] < 0 || handles[i] >= dm.H) return fail(SART_E_INVALID, "handle %d out of range", handles[i]);
      if (seen[handles[i]]) return fail(SART_E_INVALID, "duplicate handle %d", handles[i]);
      seen[handles[i]] = 1;
    }
  }
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  StageSlot* s;
  sart_status rc = stage_begin(c, &s);
  if (rc != SART_OK) return rc;
  if (n) memcpy(s->host, handles, (size_t)n * sizeof(int));
  rc = stage_upload(c, s, n, st);
  if (rc != SART_OK) return rc;
  launch_finish(c->ctx, c->plan, n, s->dev, nullptr, ++c->call_seq, st);
  HIP_TRY(hipEventRecord(s->done, st));
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

// Shared by sart_start_branches (src == null) and sart_fork_branches.
static sart_status start_common(sart_cache* c, int32_t n, const int32_t* handles, const int32_t* src, void* stream) {
  const Dims& dm = c->ctx.dm;
  if (!dm.start_waiting) return fail(SART_E_INVALID, "the cache was not created with branches_start_waiting");
  if (n < 0 || (n > 0 && !handles)) return fail(SART_E_INVALID, "bad handle list");
  if (n > dm.H) return fail(SART_E_INVALID, "more handles than branches");
  if (n == 0) return SART_OK;
  {
    std::vector<char> seen(dm.H, 0);
    for (int i = 0; i < n; ++i) {
      if (handles[i] < 0 || handles[i] >= dm.H) return fail(SART_E_INVALID, "handle %d out of range", handles[i]);
      if (seen[handles[i]]) return fail(SART_E_INVALID, "duplicate handle %d", handles[i]);
      seen[handles[i]] = 1;
      if (!src) continue;
      if (src[i] < 0 || src[i] >= dm.H) return fail(SART_E_INVALID, "source handle %d out of range", src[i]);
      if (src[i] / dm.Nb != handles[i] / dm.Nb)
        return fail(SART_E_INVALID, "branch %d cannot continue branch %d of another request", handles[i], src[i]);
    }
  }
  hipStream_t st = (hipStream_t)stream;
  note_stream(c, stream);
  StageSlot* s;
  sart_status rc = stage_begin(c, &s);
  if (rc != SART_OK) return rc;
  memcpy(s->host, handles, (size_t)n * sizeof(int));
  if (src) memcpy(s->host + n, src, (size_t)n * sizeof(int));
  rc = stage_upload(c, s, src ? 2 * (size_t)n : (size_t)n, st);
  if (rc != SART_OK) return rc;
  launch_start(c->ctx, c->plan, n, s->dev, src ? s->dev + n : nullptr, c->desc.n_layers, c->layer_bytes, ++c->call_seq, st);
  HIP_TRY(hipEventRecord(s->done, st));
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_start_branches(sart_cache* c, int32_t n, const int32_t* handles, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  return start_common(c, n, handles, nullptr, stream);
}

sart_status sart_fork_branches(sart_cache* c, int32_t n, const int32_t* src, const int32_t* dst, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (n > 0 && !src) return fail(SART_E_INVALID, "null source list");
  return start_common(c, n, dst, src, stream);
}

sart_status sart_finish_reached(sart_cache* c, const int32_t* target_len, void* stream) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (!target_len) return fail(SART_E_INVALID, "null target_len");
  note_stream(c, stream);
  launch_finish(c->ctx, c->plan, 0, nullptr, target_len, ++c->call_seq, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

static sart_status read_and_clear_status(sart_cache* c, int* scal_host) {
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  HIP_TRY(hipMemcpy(scal_host, c->ctx.tb.scal, S_COUNT * sizeof(int), hipMemcpyDeviceToHost));
  if (scal_host[S_ERR] != 0) {
    const int zero[2] = {0, 0};
    HIP_TRY(hipMemcpy(c->ctx.tb.scal + S_ERR, zero, 2 * sizeof(int), hipMemcpyHostToDevice));
    fail((sart_status)scal_host[S_ERR], "device-side status %d raised by call #%d on this cache",
         scal_host[S_ERR], scal_host[S_ERRCALL]);
  }
  return (sart_status)scal_host[S_ERR];
}

sart_status sart_sync_status(sart_cache* c) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  int scal[S_COUNT];
  return read_and_clear_status(c, scal);
}

sart_status sart_get_state(sart_cache* c, int32_t* n_active, int32_t* active_handles, int32_t* seq_lens,
                           int32_t* block_tables, int32_t* free_stack, int32_t* free_top,
                           int32_t* prefix_tables, int32_t* prefix_lens, int32_t* prefix_refcnt,
                           int32_t* branch_state, int32_t* req_counters) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  const Dims& dm = c->ctx.dm;
  const Tables& tb = c->ctx.tb;
  int scal[S_COUNT];
  sart_status status = read_and_clear_status(c, scal);
  if (status == SART_E_HIP) return status;
  const size_t H = dm.H, R = dm.max_req;
  if (n_active) *n_active = scal[S_NACTIVE];
  if (free_top) *free_top = scal[S_FREETOP];
#define D2H(dst, src, n) HIP_TRY(hipMemcpy((dst), (src), (n) * sizeof(int), hipMemcpyDeviceToHost))
  if (active_handles) D2H(active_handles, tb.active, H);
  if (seq_lens) D2H(seq_lens, tb.seq_len, H);
  if (block_tables) D2H(block_tables, tb.bt[scal[S_BTSEL]], H * dm.max_bp);
  if (free_stack) {
    D2H(free_stack, tb.free_stack, (size_t)dm.num_pages);
    for (int i = scal[S_FREETOP]; i < dm.num_pages; ++i) free_stack[i] = -1;  // popped entries are not part of the state
  }
  if (prefix_tables) D2H(prefix_tables, tb.prefix_table, R * dm.max_pp);
  if (prefix_lens) D2H(prefix_lens, tb.prefix_len, R);
  if (prefix_refcnt) D2H(prefix_refcnt, tb.refcnt, R);
  if (branch_state) D2H(branch_state, tb.br_state, H);
  if (req_counters) {
    std::vector<int> a(R), b(R);
    D2H(a.data(), tb.num_completed, R);
    D2H(b.data(), tb.num_pruned, R);
    for (size_t r = 0; r < R; ++r) { req_counters[2 * r] = a[r]; req_counters[2 * r + 1] = b[r]; }
  }
#undef D2H
  return status;
}

sart_status sart_set_profiling(sart_cache* c, int32_t on) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (on < 0 || on > 1000) return fail(SART_E_INVALID, "profiling repeats out of range");
  c->profiling = on;
  c->ev_valid = false;
  return SART_OK;
}

sart_status sart_last_decode_ms(sart_cache* c, float* ms_attn, float* ms_total) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (!c->ev_valid) return fail(SART_E_STATE, "no profiled decode call yet");
  HIP_TRY(hipEventSynchronize(c->ev[3]));
  if (ms_attn) {
    HIP_TRY(hipEventElapsedTime(ms_attn, c->ev[1], c->ev[2]));
    *ms_attn /= (float)(c->profiling > 1 ? c->profiling : 1);
  }
  if (ms_total) HIP_TRY(hipEventElapsedTime(ms_total, c->ev[0], c->ev[3]));
  return SART_OK;
}

sart_status sart_device_views(sart_cache* c, const int32_t** active_handles, const int32_t** n_active) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (active_handles) *active_handles = c->ctx.tb.active;
  if (n_active) *n_active = c->ctx.tb.scal + S_NACTIVE;
  return SART_OK;
}

sart_status sart_read_probe(const void* buf, size_t bytes, const int32_t* chunk_order, void* stream) {
  return sart_read_probe_shaped(buf, bytes, chunk_order, 2048, 4, 0, 0, stream);
}

sart_status sart_read_probe_shaped(const void* buf, size_t bytes, const int32_t* chunk_order, int32_t n_workgroups,
                                   int32_t depth, int32_t flavour, int32_t interleave, void* stream) {
  if (!buf || bytes < 8192) return fail(SART_E_INVALID, "the probe needs a device buffer of at least 8 KiB");
  if (n_workgroups < 1 || n_workgroups > 65536) return fail(SART_E_INVALID, "probe workgroups out of range");
  if (depth != 1 && depth != 2 && depth != 4 && depth != 8) return fail(SART_E_INVALID, "probe depth must be 1, 2, 4 or 8");
  if (flavour < 0 || flavour > 1) return fail(SART_E_INVALID, "probe flavour must be 0 (plain) or 1 (non-temporal)");
  launch_read_probe(buf, (long long)(bytes / 8192), chunk_order, n_workgroups, depth, flavour, interleave != 0,
                    (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_mfma_probe(const void* operands, int64_t rounds, int32_t n_workgroups, int32_t shape, float* sink, void* stream) {
  if (!operands || !sink) return fail(SART_E_INVALID, "the matrix-core probe needs its operand and result buffers");
  if (rounds < 1 || rounds > (1ll << 30)) return fail(SART_E_INVALID, "probe rounds out of range");
  if (n_workgroups < 1 || n_workgroups > 65536) return fail(SART_E_INVALID, "probe workgroups out of range");
  if (shape < 0 || shape > 2) return fail(SART_E_INVALID, "probe shape must be 0 (32x32x16), 1 (16x16x32) or 2 (16x16x32 with the softmax)");
  launch_mfma_probe(operands, rounds, n_workgroups, shape, sink, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

sart_status sart_set_prompt_stagger(sart_cache* c, int32_t on) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  c->stagger_prompt = on != 0;
  return SART_OK;
}

sart_status sart_set_merge_mode(sart_cache* c, int32_t in_kernel) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  c->merge_mode = in_kernel != 0;
  return SART_OK;
}

sart_status sart_set_decode_launch(sart_cache* c, int32_t n_workgroups, int32_t prompt_mode, int32_t skew_permille) {
  if (!c) return fail(SART_E_INVALID, "null cache");
  if (prompt_mode < -1 || prompt_mode > 2) return fail(SART_E_INVALID, "prompt_mode must be -1, 0, 1 or 2");
  if (skew_permille < -500 || skew_permille > 500) return fail(SART_E_INVALID, "skew_permille out of range");
  if (n_workgroups > c->max_wg) return fail(SART_E_INVALID, "at most %d workgroups", c->max_wg);
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, c->device));
  const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (prompt_mode >= 0) c->plan.prompt_mode = c->ctx.dm.layout == SART_LAYOUT_NATURAL ? 1 : prompt_mode;   // natural layout: per-branch blocks only
  c->plan.skew_permille = skew_permille;
  c->plan.n_wg = n_workgroups > 0 ? n_workgroups : cus;
  launch_plan(c->ctx, c->plan, c->last_stream);   // the plan follows the launch shape
  HIP_TRY(hipGetLastError());
  return SART_OK;
}

}  // extern "C"
