/*
 * sart_oracle.c - TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU statement of what the SART hot path computes:
 * per-branch softmax attention through a paged KV cache with a shared prompt,
 * and the bookkeeping that removes branches from the batch.  It shares no code
 * with the HIP library; only tests, the smoke check and the benchmark's CPU
 * baseline leg may load it.
 *
 * What follows the paper (arXiv 2505.13326):
 *   - Algorithm 1, Prefill: after prefilling a request, N branches are created
 *     and pushed into the queue of awaiting branches; the main workflow moves
 *     awaiting branches into the batch one by one while it has room (so a
 *     request's branches need not start decoding together: Section 4).
 *   - Algorithm 1, Decode: completed branches are removed and counted; an
 *     incomplete branch is pruned iff num_pruned < max_num_pruned and its
 *     reward < threshold; a request is finished when num_completed >= M or
 *     num_completed + num_pruned == N.
 *   - Section 3, Solution 1: once M responses complete, the remaining branches
 *     are terminated.
 *   - Section 4: the prefix KV cache is shared across the branches of a
 *     request; a branch's KV cache is released as soon as it is pruned,
 *     early-stopped or completed; the prefix is released only when all
 *     branches have terminated.
 *   - Section 2 (tree-based search, e.g. Rebase, which the evaluation compares
 *     against: a reasoning trajectory is expanded into several continuations):
 *     orc_fork lets a branch split, the copies sharing the KV pages of what they
 *     have in common; a shared page is released when its last holder ends.
 *   - Section 4 (prefilling is done as in plain LLM inference) and Section 2
 *     (one token generated per decode step): the attention is the
 *     textbook one, softmax(q K^T / sqrt(d)) V of one query over all cached
 *     tokens, written out below as that definition.
 *
 * The paper names N sampled branches and M required completions; here they are
 * Nb and Q.
 *
 * Readings the paper leaves open (fixed here):
 *   - pages hold page_tokens tokens; a prompt whose length is not a page
 *     multiple leaves its last page partly filled and private tokens start on
 *     a fresh page;
 *   - the free list is a LIFO stack; pops and pushes happen in the order
 *     written in the functions below;
 *   - ties between equal scores are broken by branch handle; NaN scores
 *     compare as +infinity;
 *   - the cap of Algorithm 1 binds in ascending active index.
 *
 * Storage: pool[page][slot][kv_head][K|V][d] raw elements (float or bf16 bits),
 * block tables and lengths by branch handle, `active` an ordered list of
 * handles.  Compaction is list filtering.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_OK = 0, ORC_E_INVALID = 1, ORC_E_OOM_PAGES = 2, ORC_E_STATE = 3 };
enum { BR_UNUSED = 0, BR_ACTIVE = 1, BR_COMPLETED = 2, BR_PRUNED = 3, BR_EARLY_STOPPED = 4, BR_WAITING = 5 };
enum { SEQ_PREFIX = 0, SEQ_BRANCH = 1 };
enum { PRUNE_DROP_LOWEST_K = 0, PRUNE_KEEP_TOP_K = 1, PRUNE_THRESHOLD = 2 };
enum { DT_F32 = 0, DT_BF16 = 1 };

typedef struct {
  int Hq, Hkv, d, pt, num_pages, max_req, Nb, Q, max_bp, max_pp, dtype;
  size_t esize;
  int start_waiting;    /* 1: a request's branches are created WAITING (awaiting branches of Algorithm 1) and join
                           the batch through orc_start; 0: they are created ACTIVE, all at once */
  int fp8;              /* 1: the cache keeps K and V as 8-bit floats (inputs stay bf16) */
  double kv_scale[2];   /* fp8: stored code = round(x / scale); K, V */
  unsigned char* pool;
  int* free_stack;
  int free_top;
  /* per request */
  int* req_used;        /* 0 never created, 1 created */
  int* prefix_len;      /* P_r */
  int* prefix_table;    /* [max_req][max_pp], -1 padded */
  int* refcnt;          /* branches of the request that still hold its prefix: active and waiting ones */
  int* num_completed;
  int* num_pruned;
  int* branch_appended; /* a branch of r already received tokens */
  /* per branch, by handle r*Nb + j */
  int* state;
  int* seq_len;
  int* block_table;     /* [max_req*Nb][max_bp], -1 padded */
  int* page_ref;        /* [num_pages] branches whose block table holds the page (0: not a branch's page) */
  /* active list */
  int n_active;
  int* active;
} orc;

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

static int* ints(size_t n, int fill) {
  int* p = (int*)malloc((n ? n : 1) * sizeof(int));
  for (size_t i = 0; i < n; ++i) p[i] = fill;
  return p;
}

orc* orc_create(int Hq, int Hkv, int d, int pt, int num_pages, int max_req, int Nb, int Q,
                int max_bp, int max_pp, int dtype, const int* free_order) {
  if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || pt <= 0 || num_pages < 0 || max_req <= 0 ||
      Nb <= 0 || max_bp < 0 || max_pp < 0 || (dtype != DT_F32 && dtype != DT_BF16))
    return NULL;
  orc* o = (orc*)calloc(1, sizeof(orc));
  o->Hq = Hq; o->Hkv = Hkv; o->d = d; o->pt = pt; o->num_pages = num_pages;
  o->max_req = max_req; o->Nb = Nb; o->Q = Q; o->max_bp = max_bp; o->max_pp = max_pp;
  o->dtype = dtype;
  o->esize = dtype == DT_F32 ? 4 : 2;
  o->pool = (unsigned char*)calloc((size_t)num_pages * pt * Hkv * 2 * d + 1, o->esize);
  /* first pop returns free_order[0]: the stack holds the order reversed */
  o->free_stack = ints(num_pages, -1);
  for (int i = 0; i < num_pages; ++i)
    o->free_stack[i] = free_order ? free_order[num_pages - 1 - i] : num_pages - 1 - i;
  o->free_top = num_pages;
  size_t H = (size_t)max_req * Nb;
  o->req_used = ints(max_req, 0);
  o->prefix_len = ints(max_req, 0);
  o->prefix_table = ints((size_t)max_req * max_pp, -1);
  o->refcnt = ints(max_req, 0);
  o->num_completed = ints(max_req, 0);
  o->num_pruned = ints(max_req, 0);
  o->branch_appended = ints(max_req, 0);
  o->state = ints(H, BR_UNUSED);
  o->seq_len = ints(H, 0);
  o->block_table = ints(H * max_bp, -1);
  o->page_ref = ints(num_pages, 0);
  o->n_active = 0;
  o->active = ints(H, -1);
  return o;
}

void orc_destroy(orc* o) {
  if (!o) return;
  free(o->pool); free(o->free_stack); free(o->req_used); free(o->prefix_len);
  free(o->prefix_table); free(o->refcnt); free(o->num_completed); free(o->num_pruned);
  free(o->branch_appended); free(o->state); free(o->seq_len); free(o->block_table); free(o->page_ref);
  free(o->active); free(o);
}

static int pop_page(orc* o) { return o->free_stack[--o->free_top]; }
static void push_page(orc* o, int p) { o->free_stack[o->free_top++] = p; }

/* address of the d elements of K (which=0) or V (which=1) of one cached token */
static unsigned char* token_ptr(const orc* o, int page, int slot, int head, int which) {
  size_t e = ((((size_t)page * o->pt + slot) * o->Hkv + head) * 2 + which) * o->d;
  return o->pool + e * o->esize;
}

/*
 * 8-bit float cache (an extension beyond the paper, which keeps KV in the
 * model's dtype): OCP FP8 E4M3 - 1 sign, 4 exponent bits (bias 7), 3 mantissa
 * bits, subnormals, no infinities, S.1111.111 = NaN, largest finite 448.
 * value(code): e == 0: m/8 * 2^-6; else (1 + m/8) * 2^(e-7).
 * A value is stored as the nearest code of the quotient x / scale (ties to the
 * even code, |x / scale| clamped to 448 first) and read back as value(code) *
 * scale.  scale is the cache's float32 scale, widened exactly.  The quotient is
 * taken in float64; that decides every code as the exact quotient would: x has
 * 8 significant bits, scale 24 and a boundary between two codes at most 5, so a
 * quotient that is not on a boundary is at least 2^-29 (relative) away from it,
 * far more than the 2^-53 the float64 division can move it.
 */
static double e4m3_value(unsigned code) {
  const unsigned e = (code >> 3) & 15, m = code & 7;
  const double mag = e == 0 ? ldexp(m / 8.0, -6) : ldexp(1.0 + m / 8.0, (int)e - 7);
  return (code & 0x80) ? -mag : mag;
}
static unsigned e4m3_nearest(double x) {
  const unsigned sign = signbit(x) ? 0x80u : 0u;
  double a = fabs(x);
  if (a > 448.0) a = 448.0;
  /* codes 0..126 are the finite magnitudes in ascending order: take the nearest, ties to the even code.
   * The nearest code's value is within a factor 2 of a, so only the codes of the binades next to a's
   * need looking at (exponent field E = ilogb(a) + 7; everything below 2^-6 is the subnormal binade). */
  int E = a > 0 ? ilogb(a) + 7 : 0;
  if (E < 1) E = 1;
  unsigned first = (unsigned)(E - 1) * 8, last = (unsigned)(E + 1) * 8 + 7;
  if (last > 126) last = 126;
  unsigned best = first;
  double best_err = fabs(e4m3_value(first) - a);
  for (unsigned c = first + 1; c <= last; ++c) {
    const double err = fabs(e4m3_value(c) - a);
    if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
  }
  return sign | best;
}
static double bf16_bits_value(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}
static uint16_t value_bf16_bits(double v) {   /* exact for every E4M3 value */
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}
/* the codec by itself, for tests: bf16 bits in, codes and read-back values out */
void orc_fp8_roundtrip(const uint16_t* in, int n, double scale, unsigned char* codes, double* values) {
  for (int i = 0; i < n; ++i) {
    const unsigned c = e4m3_nearest(bf16_bits_value(in[i]) / scale);
    if (codes) codes[i] = (unsigned char)c;
    if (values) values[i] = e4m3_value(c) * scale;
  }
}
/* switches a bf16 cache to 8-bit float storage (before the first append) */
int orc_set_fp8(orc* o, double k_scale, double v_scale) {
  if (o->dtype != DT_BF16 || !(k_scale > 0) || !(v_scale > 0)) return ORC_E_INVALID;
  o->fp8 = 1;
  o->kv_scale[0] = k_scale;
  o->kv_scale[1] = v_scale;
  return ORC_OK;
}

static double widen(const orc* o, const unsigned char* p, int c) {
  if (o->dtype == DT_F32) {
    float f;
    memcpy(&f, p + 4 * (size_t)c, 4);
    return (double)f;
  }
  uint16_t b;
  memcpy(&b, p + 2 * (size_t)c, 2);
  uint32_t u = (uint32_t)b << 16; /* bf16 is the top half of a float */
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* a cached element as the attention reads it: the stored value, times the scale of an 8-bit float cache */
static double cached(const orc* o, const unsigned char* p, int c, int which) {
  const double x = widen(o, p, c);
  return o->fp8 ? x * o->kv_scale[which] : x;
}

static int is_dup(const int* ids, int n, int limit) {
  unsigned char* seen = (unsigned char*)calloc(limit ? limit : 1, 1);
  int dup = 0;
  for (int i = 0; i < n && !dup; ++i) {
    if (seen[ids[i]]) dup = 1;
    seen[ids[i]] = 1;
  }
  free(seen);
  return dup;
}

/*
 * Append tokens.  Algorithm 1 (Prefill) for SEQ_PREFIX: the first prefix
 * append of a request creates its Nb branches.  Section 2 (decode adds one
 * token per step) for SEQ_BRANCH.  The whole call is validated first; on any
 * error nothing changes.
 * k, v: [sum n][Hkv][d] raw elements.
 */
int orc_append(orc* o, int kind, int n_seqs, const int* ids, const int* n_tokens,
               const void* k, const void* v) {
  if (n_seqs < 0 || (kind != SEQ_PREFIX && kind != SEQ_BRANCH)) return ORC_E_INVALID;
  if (kind == SEQ_PREFIX && !ids && n_seqs > 0) return ORC_E_INVALID;
  if (!ids && n_seqs != o->n_active) return ORC_E_INVALID;
  const int limit = kind == SEQ_PREFIX ? o->max_req : o->max_req * o->Nb;
  int* id = ints(n_seqs, 0);
  for (int i = 0; i < n_seqs; ++i) id[i] = ids ? ids[i] : o->active[i];
  int rc = ORC_OK;
  long need = 0;
  for (int i = 0; i < n_seqs && rc == ORC_OK; ++i) {
    int n = n_tokens ? n_tokens[i] : 1;
    if (id[i] < 0 || id[i] >= limit || n < 0) rc = ORC_E_INVALID;
  }
  if (rc == ORC_OK && is_dup(id, n_seqs, limit)) rc = ORC_E_INVALID;
  for (int i = 0; i < n_seqs && rc == ORC_OK; ++i) {
    int n = n_tokens ? n_tokens[i] : 1;
    if (kind == SEQ_PREFIX) {
      int r = id[i];
      if (o->req_used[r] && (o->refcnt[r] == 0 || o->branch_appended[r])) { rc = ORC_E_STATE; break; }
      int have = ceil_div(o->prefix_len[r], o->pt), want = ceil_div(o->prefix_len[r] + n, o->pt);
      if (want > o->max_pp) { rc = ORC_E_INVALID; break; }
      need += want - have;
    } else {
      int b = id[i];
      if (o->state[b] != BR_ACTIVE) { rc = ORC_E_STATE; break; }
      int have = ceil_div(o->seq_len[b], o->pt), want = ceil_div(o->seq_len[b] + n, o->pt);
      if (want > o->max_bp) { rc = ORC_E_INVALID; break; }
      need += want - have;
    }
  }
  if (rc == ORC_OK && need > o->free_top) rc = ORC_E_OOM_PAGES;
  if (rc != ORC_OK) { free(id); return rc; }

  const size_t row = (size_t)o->Hkv * o->d * o->esize; /* bytes of one token of K (or V) */
  size_t tok = 0;
  for (int i = 0; i < n_seqs; ++i) {
    int n = n_tokens ? n_tokens[i] : 1;
    int* table; int* len;
    if (kind == SEQ_PREFIX) {
      int r = id[i];
      if (!o->req_used[r]) {
        o->req_used[r] = 1;
        o->refcnt[r] = o->Nb;
        for (int j = 0; j < o->Nb; ++j) {
          int b = r * o->Nb + j;
          o->seq_len[b] = 0;
          if (o->start_waiting) {
            o->state[b] = BR_WAITING;              /* pushed into the queue of awaiting branches */
          } else {
            o->state[b] = BR_ACTIVE;
            o->active[o->n_active++] = b;
          }
        }
      }
      table = o->prefix_table + (size_t)r * o->max_pp;
      len = &o->prefix_len[r];
    } else {
      int b = id[i];
      if (n > 0) o->branch_appended[b / o->Nb] = 1;
      table = o->block_table + (size_t)b * o->max_bp;
      len = &o->seq_len[b];
    }
    for (int t = 0; t < n; ++t, ++tok) {
      int pos = *len;
      if (pos % o->pt == 0) {                                  /* first token of a new page */
        table[pos / o->pt] = pop_page(o);
        if (kind == SEQ_BRANCH) o->page_ref[table[pos / o->pt]] = 1;
      }
      int page = table[pos / o->pt], slot = pos % o->pt;
      for (int h = 0; h < o->Hkv; ++h) {
        size_t src = tok * row + (size_t)h * o->d * o->esize;
        if (!o->fp8) {
          memcpy(token_ptr(o, page, slot, h, 0), (const unsigned char*)k + src, o->d * o->esize);
          memcpy(token_ptr(o, page, slot, h, 1), (const unsigned char*)v + src, o->d * o->esize);
        } else {
          /* keep value(code) as bf16 bits (exact): the scale is applied when the element is read */
          for (int w = 0; w < 2; ++w) {
            const uint16_t* in = (const uint16_t*)((const unsigned char*)(w ? v : k) + src);
            uint16_t* dst = (uint16_t*)token_ptr(o, page, slot, h, w);
            for (int c = 0; c < o->d; ++c)
              dst[c] = value_bf16_bits(e4m3_value(e4m3_nearest(bf16_bits_value(in[c]) / o->kv_scale[w])));
          }
        }
      }
      *len = pos + 1;
    }
  }
  free(id);
  return ORC_OK;
}

/*
 * Decode-step attention by its definition.  For active row a (branch b of
 * request r), query head h, KV head g = h / (Hq/Hkv), context = the P_r prompt
 * tokens of r followed by the seq_len[b] private tokens of b:
 *     s_t = scale * sum_c q[a,h,c] K[t,g,c]
 *     w_t = exp(s_t - max s) / sum_t exp(s_t - max s)
 *     out[a,h,:] = sum_t w_t V[t,g,:]
 * all in float64 from the exactly widened stored values.
 * q: [n_rows][Hq][d] raw elements.  rows: n_sel active indices to compute, or
 * NULL for all active rows (then n_sel is ignored).  out: [n_out][Hq][d]
 * doubles where n_out = n_sel or n_active, written in the order of `rows`.
 * wsum (optional): [n_out][Hq] sums of the normalised weights.
 * scale <= 0 means 1/sqrt(d).  An empty context gives zeros.
 */
int orc_attention(const orc* o, const void* q, int n_rows, double scale, const int* rows,
                  int n_sel, double* out, double* wsum) {
  if (n_rows < o->n_active) return ORC_E_INVALID;
  int n_out = rows ? n_sel : o->n_active;
  for (int i = 0; i < n_out; ++i) {
    int a = rows ? rows[i] : i;
    if (a < 0 || a >= o->n_active) return ORC_E_INVALID;
  }
  if (scale <= 0) scale = 1.0 / sqrt((double)o->d);
  const int G = o->Hq / o->Hkv, d = o->d;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < n_out; ++i) {
    for (int h = 0; h < o->Hq; ++h) {
      int a = rows ? rows[i] : i;
      int b = o->active[a], r = b / o->Nb, g = h / G;
      int P = o->prefix_len[r], L = o->seq_len[b], T = P + L;
      const unsigned char* qrow = (const unsigned char*)q + ((size_t)a * o->Hq + h) * d * o->esize;
      double* orow = out + ((size_t)i * o->Hq + h) * d;
      for (int c = 0; c < d; ++c) orow[c] = 0.0;
      if (wsum) wsum[(size_t)i * o->Hq + h] = 0.0;
      if (T == 0) continue;
      double* s = (double*)malloc((size_t)T * sizeof(double));
      double smax = -INFINITY;
      for (int t = 0; t < T; ++t) {
        int page = t < P ? o->prefix_table[(size_t)r * o->max_pp + t / o->pt]
                         : o->block_table[(size_t)b * o->max_bp + (t - P) / o->pt];
        int slot = t < P ? t % o->pt : (t - P) % o->pt;
        const unsigned char* kp = token_ptr(o, page, slot, g, 0);
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += widen(o, qrow, c) * cached(o, kp, c, 0);
        s[t] = scale * dot;
        if (s[t] > smax) smax = s[t];
      }
      double Z = 0.0;
      for (int t = 0; t < T; ++t) { s[t] = exp(s[t] - smax); Z += s[t]; }
      double ws = 0.0;
      for (int t = 0; t < T; ++t) {
        int page = t < P ? o->prefix_table[(size_t)r * o->max_pp + t / o->pt]
                         : o->block_table[(size_t)b * o->max_bp + (t - P) / o->pt];
        int slot = t < P ? t % o->pt : (t - P) % o->pt;
        const unsigned char* vp = token_ptr(o, page, slot, g, 1);
        double w = s[t] / Z;
        ws += w;
        for (int c = 0; c < d; ++c) orow[c] += w * cached(o, vp, c, 1);
      }
      if (wsum) wsum[(size_t)i * o->Hq + h] = ws;
      free(s);
    }
  }
  return ORC_OK;
}

/*
 * Prefill attention (Algorithm 1, Prefill; Section 4 calls the prefill phase
 * the same as in plain LLM inference, so this is ordinary causal
 * self-attention over the prompt).  The queries are the last n_q prompt tokens
 * of request r: query i sits at prompt position p = P_r - n_q + i and attends
 * to prompt tokens 0..p (itself included), read through the prefix table:
 *   s_t = scale * q_i . K[t],  w_t = exp(s_t - max) / sum,  out_i = sum_t w_t V[t].
 * With n_q < P_r this is one chunk of a chunked prefill (append a chunk of the
 * prompt, then attend with that chunk's queries).
 * q: [n_q][Hq][d] in the cache dtype; out: [n_q][Hq][d] double; wsum optional.
 */
int orc_prefill_attention(const orc* o, int r, const void* q, int n_q, double scale, double* out, double* wsum) {
  if (r < 0 || r >= o->max_req || n_q < 0) return ORC_E_INVALID;
  if (!o->req_used[r] || o->refcnt[r] == 0) return ORC_E_STATE;
  const int P = o->prefix_len[r];
  if (n_q > P) return ORC_E_INVALID;
  if (scale <= 0) scale = 1.0 / sqrt((double)o->d);
  const int G = o->Hq / o->Hkv, d = o->d;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < n_q; ++i) {
    for (int h = 0; h < o->Hq; ++h) {
      const int g = h / G, T = P - n_q + i + 1;      /* tokens 0..p */
      const unsigned char* qrow = (const unsigned char*)q + ((size_t)i * o->Hq + h) * d * o->esize;
      double* orow = out + ((size_t)i * o->Hq + h) * d;
      for (int c = 0; c < d; ++c) orow[c] = 0.0;
      double* s = (double*)malloc((size_t)T * sizeof(double));
      double smax = -INFINITY;
      for (int t = 0; t < T; ++t) {
        const unsigned char* kp = token_ptr(o, o->prefix_table[(size_t)r * o->max_pp + t / o->pt], t % o->pt, g, 0);
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += widen(o, qrow, c) * cached(o, kp, c, 0);
        s[t] = scale * dot;
        if (s[t] > smax) smax = s[t];
      }
      double Z = 0.0;
      for (int t = 0; t < T; ++t) { s[t] = exp(s[t] - smax); Z += s[t]; }
      double ws = 0.0;
      for (int t = 0; t < T; ++t) {
        const unsigned char* vp = token_ptr(o, o->prefix_table[(size_t)r * o->max_pp + t / o->pt], t % o->pt, g, 1);
        const double w = s[t] / Z;
        ws += w;
        for (int c = 0; c < d; ++c) orow[c] += w * cached(o, vp, c, 1);
      }
      if (wsum) wsum[(size_t)i * o->Hq + h] = ws;
      free(s);
    }
  }
  return ORC_OK;
}

/*
 * Remove a set of active branches (Section 4, immediate release).
 * new_state[a] != 0 marks active index a as leaving with that state.
 *  (1) in ascending active index: push the branch's private pages in ascending
 *      logical order, set its state, drop one reference on its request;
 *  (2) then, in ascending request id, requests whose last branch left push
 *      their prefix pages in ascending logical order;
 *  (3) the active list keeps the survivors in their old relative order.
 */
static void terminate(orc* o, const int* new_state, const unsigned char* stop_waiting) {
  unsigned char* touched = (unsigned char*)calloc(o->max_req, 1);
  for (int a = 0; a < o->n_active; ++a) {
    if (!new_state[a]) continue;
    int b = o->active[a], r = b / o->Nb;
    int* bt = o->block_table + (size_t)b * o->max_bp;
    int np = ceil_div(o->seq_len[b], o->pt);
    for (int p = 0; p < np; ++p) {                              /* a page shared after a fork goes with its last holder */
      if (--o->page_ref[bt[p]] == 0) push_page(o, bt[p]);
      bt[p] = -1;
    }
    o->seq_len[b] = 0;
    o->state[b] = new_state[a];
    o->refcnt[r]--;
    touched[r] = 1;
  }
  /* awaiting branches of a request that is stopped early never start: they hold no pages of their own */
  for (int r = 0; stop_waiting && r < o->max_req; ++r) {
    if (!stop_waiting[r]) continue;
    for (int j = 0; j < o->Nb; ++j) {
      int b = r * o->Nb + j;
      if (o->state[b] != BR_WAITING) continue;
      o->state[b] = BR_EARLY_STOPPED;
      o->refcnt[r]--;
      touched[r] = 1;
    }
  }
  for (int r = 0; r < o->max_req; ++r) {
    if (!touched[r] || o->refcnt[r] != 0) continue;
    int* ptab = o->prefix_table + (size_t)r * o->max_pp;
    int np = ceil_div(o->prefix_len[r], o->pt);
    for (int p = 0; p < np; ++p) { push_page(o, ptab[p]); ptab[p] = -1; }
  }
  int w = 0;
  for (int a = 0; a < o->n_active; ++a)
    if (!new_state[a]) o->active[w++] = o->active[a];
  for (int a = w; a < o->n_active; ++a) o->active[a] = -1;
  o->n_active = w;
  free(touched);
}

/*
 * A waiting branch joins the batch (Algorithm 1, main workflow: while the batch
 * has room, an awaiting branch is popped from the branch queue and appended to
 * the current batch).  The listed branches, all WAITING, become ACTIVE in list
 * order; each is placed right after the last active branch of its request, or at
 * the end of the active list when the request has none (so a request's branches
 * stay neighbours in the list, in the order they started).
 */
int orc_start(orc* o, int n, const int* handles) {
  const int H = o->max_req * o->Nb;
  if (n < 0 || (n > 0 && !handles)) return ORC_E_INVALID;
  for (int i = 0; i < n; ++i)
    if (handles[i] < 0 || handles[i] >= H) return ORC_E_INVALID;
  if (is_dup(handles, n, H)) return ORC_E_INVALID;
  for (int i = 0; i < n; ++i)
    if (o->state[handles[i]] != BR_WAITING) return ORC_E_STATE;
  for (int i = 0; i < n; ++i) {
    const int b = handles[i], r = b / o->Nb;
    int pos = o->n_active;                       /* no active branch of r: the end of the list */
    for (int a = 0; a < o->n_active; ++a)
      if (o->active[a] / o->Nb == r) pos = a + 1;
    for (int a = o->n_active; a > pos; --a) o->active[a] = o->active[a - 1];
    o->active[pos] = b;
    o->n_active++;
    o->state[b] = BR_ACTIVE;
    o->seq_len[b] = 0;
  }
  return ORC_OK;
}

/*
 * A branch splits (tree search over reasoning trajectories, Section 2: a
 * trajectory is expanded into several continuations).  dst[i], a WAITING branch
 * of the request of src[i], joins the batch as a copy of the ACTIVE branch
 * src[i]: same private tokens so far.  The two share the pages that are full at
 * this moment (a page is then held by several block tables, at the same logical
 * index in each, and goes back to the free stack when its last holder ends); a
 * partly filled last page is copied into a fresh page, so every branch appends
 * into a page of its own.  List entries are handled in order: dst[i] takes its
 * place in the batch as in orc_start (behind its request's last active branch),
 * then pops its page, if it needs one.  The same src may be listed several times.
 */
int orc_fork(orc* o, int n, const int* src, const int* dst) {
  const int H = o->max_req * o->Nb;
  if (n < 0 || (n > 0 && (!src || !dst))) return ORC_E_INVALID;
  for (int i = 0; i < n; ++i) {
    if (src[i] < 0 || src[i] >= H || dst[i] < 0 || dst[i] >= H) return ORC_E_INVALID;
    if (src[i] / o->Nb != dst[i] / o->Nb) return ORC_E_INVALID;      /* a branch splits within its request */
  }
  if (is_dup(dst, n, H)) return ORC_E_INVALID;
  int need = 0;
  for (int i = 0; i < n; ++i) {
    if (o->state[src[i]] != BR_ACTIVE || o->state[dst[i]] != BR_WAITING) return ORC_E_STATE;
    need += o->seq_len[src[i]] % o->pt != 0;
  }
  if (need > o->free_top) return ORC_E_OOM_PAGES;
  const size_t page_bytes = (size_t)o->pt * o->Hkv * 2 * o->d * o->esize;
  for (int i = 0; i < n; ++i) {
    const int one = dst[i];
    int rc = orc_start(o, 1, &one);
    if (rc != ORC_OK) return rc;                                     /* cannot happen: checked above */
    const int L = o->seq_len[src[i]], full = L / o->pt;
    const int* from = o->block_table + (size_t)src[i] * o->max_bp;
    int* to = o->block_table + (size_t)dst[i] * o->max_bp;
    for (int p = 0; p < full; ++p) { to[p] = from[p]; o->page_ref[from[p]]++; }
    if (L % o->pt) {
      const int page = pop_page(o);
      o->page_ref[page] = 1;
      to[full] = page;
      memcpy(o->pool + (size_t)page * page_bytes, o->pool + (size_t)from[full] * page_bytes, page_bytes);
    }
    o->seq_len[dst[i]] = L;
  }
  return ORC_OK;
}

/* Branches are created WAITING from now on (before the first request is created). */
int orc_set_start_waiting(orc* o, int on) {
  for (int r = 0; r < o->max_req; ++r)
    if (o->req_used[r]) return ORC_E_STATE;
  o->start_waiting = on != 0;
  return ORC_OK;
}

/*
 * Completion and early stop (Algorithm 1, Decode: completed branches are
 * removed and counted; Section 3, Solution 1: when Q responses are complete
 * the remaining branches of the request are terminated).
 */
int orc_finish(orc* o, int n, const int* handles) {
  const int H = o->max_req * o->Nb;
  if (n < 0 || (n > 0 && !handles)) return ORC_E_INVALID;
  for (int i = 0; i < n; ++i)
    if (handles[i] < 0 || handles[i] >= H) return ORC_E_INVALID;
  if (is_dup(handles, n, H)) return ORC_E_INVALID;
  for (int i = 0; i < n; ++i)
    if (o->state[handles[i]] != BR_ACTIVE) return ORC_E_STATE;
  int* new_state = ints(o->n_active, 0);
  unsigned char* listed = (unsigned char*)calloc(H ? H : 1, 1);
  for (int i = 0; i < n; ++i) {
    listed[handles[i]] = 1;
    o->num_completed[handles[i] / o->Nb]++;
  }
  const int quota_on = o->Q >= 1 && o->Q <= o->Nb;
  unsigned char* stop_waiting = (unsigned char*)calloc(o->max_req, 1);
  for (int a = 0; a < o->n_active; ++a) {
    int b = o->active[a], r = b / o->Nb;
    if (listed[b]) new_state[a] = BR_COMPLETED;
    else if (quota_on && o->num_completed[r] >= o->Q) new_state[a] = BR_EARLY_STOPPED;
  }
  for (int i = 0; i < n; ++i) {
    int r = handles[i] / o->Nb;
    if (quota_on && o->num_completed[r] >= o->Q) stop_waiting[r] = 1;   /* the remaining branches, awaiting ones too */
  }
  terminate(o, new_state, stop_waiting);
  free(new_state);
  free(listed);
  free(stop_waiting);
  return ORC_OK;
}

/* key order for pruning: score ascending (NaN as +inf), then handle ascending */
static int key_less(float sa, int ha, float sb, int hb) {
  if (sa != sa) sa = INFINITY;
  if (sb != sb) sb = INFINITY;
  if (sa < sb) return 1;
  if (sa > sb) return 0;
  return ha < hb;
}

/*
 * Pruning (Algorithm 1, Decode, the loop over incomplete branches).
 * scores: [n_scores] floats in active order.  k_per_req / thr / maxp: per
 * request arrays (k_per_req and maxp may be NULL).
 */
int orc_prune(orc* o, int mode, int k, const int* k_per_req, const float* thr, const int* maxp,
              const float* scores, int n_scores) {
  if (mode < 0 || mode > 2 || !scores || n_scores < o->n_active) return ORC_E_INVALID;
  if (mode == PRUNE_THRESHOLD && !thr) return ORC_E_INVALID;
  if (mode != PRUNE_THRESHOLD && !k_per_req && k < 0) return ORC_E_INVALID;
  int* new_state = ints(o->n_active, 0);
  int* members = ints(o->Nb, 0);
  for (int r = 0; r < o->max_req; ++r) {
    int live = 0;
    for (int a = 0; a < o->n_active; ++a)
      if (o->active[a] / o->Nb == r) members[live++] = a; /* ascending active index */
    if (!live) continue;
    if (mode == PRUNE_THRESHOLD) {
      for (int i = 0; i < live; ++i) {
        int a = members[i];
        int room = !maxp || o->num_pruned[r] < maxp[r];
        if (room && scores[a] < thr[r]) { /* NaN < x is false: never pruned */
          new_state[a] = BR_PRUNED;
          o->num_pruned[r]++;
        }
      }
      continue;
    }
    int kk = k_per_req ? k_per_req[r] : k;
    if (kk < 0) kk = 0;
    if (kk > live) kk = live;
    int n_victims = mode == PRUNE_DROP_LOWEST_K ? kk : live - kk;
    if (maxp) {
      int room = maxp[r] - o->num_pruned[r];
      if (room < 0) room = 0;
      if (n_victims > room) n_victims = room;
    }
    /* sort the request's live rows by key (insertion sort), take the lowest */
    for (int i = 1; i < live; ++i) {
      int a = members[i], j = i;
      while (j > 0 && key_less(scores[a], o->active[a], scores[members[j - 1]], o->active[members[j - 1]])) {
        members[j] = members[j - 1];
        --j;
      }
      members[j] = a;
    }
    for (int i = 0; i < n_victims; ++i) new_state[members[i]] = BR_PRUNED;
    o->num_pruned[r] += n_victims;
  }
  terminate(o, new_state, NULL);
  free(new_state);
  free(members);
  return ORC_OK;
}

/* Algorithm 1, Decode, last test: the request's output can be produced. */
int orc_request_done(const orc* o, int r) {
  if (r < 0 || r >= o->max_req || !o->req_used[r]) return 0;
  int quota_on = o->Q >= 1 && o->Q <= o->Nb;
  return (quota_on && o->num_completed[r] >= o->Q) ||
         o->num_completed[r] + o->num_pruned[r] == o->Nb;
}

/* Canonical state, same shapes and padding as the product's readback. */
void orc_get_state(const orc* o, int* n_active, int* active_handles, int* seq_lens,
                   int* block_tables, int* free_stack, int* free_top, int* prefix_tables,
                   int* prefix_lens, int* prefix_refcnt, int* branch_state, int* req_counters) {
  const int H = o->max_req * o->Nb;
  if (n_active) *n_active = o->n_active;
  if (free_top) *free_top = o->free_top;
  for (int a = 0; a < H; ++a) {
    int b = a < o->n_active ? o->active[a] : -1;
    if (active_handles) active_handles[a] = b;
    if (seq_lens) seq_lens[a] = b >= 0 ? o->seq_len[b] : 0;
    if (block_tables)
      for (int p = 0; p < o->max_bp; ++p)
        block_tables[(size_t)a * o->max_bp + p] = b >= 0 ? o->block_table[(size_t)b * o->max_bp + p] : -1;
  }
  if (free_stack)
    for (int i = 0; i < o->num_pages; ++i) free_stack[i] = i < o->free_top ? o->free_stack[i] : -1;
  if (prefix_tables) memcpy(prefix_tables, o->prefix_table, (size_t)o->max_req * o->max_pp * sizeof(int));
  if (prefix_lens) memcpy(prefix_lens, o->prefix_len, (size_t)o->max_req * sizeof(int));
  if (prefix_refcnt) memcpy(prefix_refcnt, o->refcnt, (size_t)o->max_req * sizeof(int));
  if (branch_state) memcpy(branch_state, o->state, (size_t)H * sizeof(int));
  if (req_counters)
    for (int r = 0; r < o->max_req; ++r) {
      req_counters[2 * r] = o->num_completed[r];
      req_counters[2 * r + 1] = o->num_pruned[r];
    }
}

int orc_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
