// Decode-step attention over the active branches (the paper's "batch decoding"
// step, Algorithm 1, Decode; arXiv 2505.13326).  The paper leaves the attention
// itself to the serving engine (Section 4: same as vanilla inference), so what
// is computed is softmax(q K^T * scale) V of one query per (branch, head) over
// the request's shared prompt tokens followed by the branch's own tokens
// (Section 4: the prefix KV cache is shared across a request's branches).
//
// Design for MI355X (gfx950):
//   * The work is HBM-bound: every KV byte is used once per step.  The kernel
//     is a persistent grid; each wave streams (page, kv-head) tiles straight
//     from HBM into registers with 1 KiB coalesced loads that already are
//     matrix-core operands (SART_LAYOUT_MFMA16), so K and V never pass through
//     LDS on the private path.
//   * QK^T and PV run on the matrix cores (16x16x32 and 16x16x16 bf16) with
//     the GQA group (<= 16 query heads) as one tile dimension; the vector ALUs
//     only do the online softmax.  S^T = K Q^T leaves each lane holding the
//     scores of 4 tokens of one head, which is exactly the B operand PV needs.
//   * Length-aware partitioning: all private (page, kv head) units of the
//     step are laid on one line and cut into equal ranges, one per wave
//     (a range may cross branch boundaries); each piece yields a partial
//     (m, l, o) that a merge kernel combines.
//   * Shared prompt pages are staged in LDS once per (request, kv head,
//     chunk) workgroup and reused by the request's branches (one wave each)
//     and all query heads of the group.
#include "sart_internal.h"

namespace sart {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline int ceil_div_i(int a, int b) { return (a + b - 1) / b; }

__device__ inline int wave_incl_scan_i(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int n = __shfl_up(v, off, 64);
    if (lane >= off) v += n;
  }
  return v;
}
__device__ inline int block_excl_scan_i(int v, int* lds, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = (blockDim.x + 63) >> 6;
  int incl = wave_incl_scan_i(v);
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    int t = lane < nw ? lds[lane] : 0;
    int ti = wave_incl_scan_i(t);
    if (lane < nw) lds[lane] = ti - t;
    if (lane == nw - 1) lds[16] = ti;
  }
  __syncthreads();
  total = lds[16];
  return incl - v + lds[wave];
}

// floats of one partial: o[G][d], then m[G], l[G]
__host__ __device__ inline long long partial_floats(int G, int d) { return (long long)G * d + 2 * G; }

// ---------------------------------------------------------------------------
// A3: partition plan (one workgroup).
//   page_cum[a]      exclusive scan of the pages each active row contributes
//                    (private pages; plus the prompt's pages when the prompt
//                    is read inline by the generic kernel)
//   units            page_cum[nA] * Hkv, cut into ranges of per_wave units
//   prefix items     one per (live request, kv head, prompt chunk, group of
//                    kAttnWaves branches)
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_decode_plan(Ctx c, DecodeArgs a, int inline_prefix) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  __shared__ int lds[17];
  __shared__ int s_npc;
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  if (a.n_rows < nA) {
    if (tid == 0) {
      if (scal[S_ERR] == 0) { scal[S_ERR] = SART_E_INVALID; scal[S_ERRCALL] = a.call_seq; }
      scal[S_CALLOK] = 0;
    }
    return;
  }
  if (tid == 0) s_npc = 0;
  // first active index of each live request
  for (int i = tid; i < nA; i += kPlanThreads) {
    const int r = tb.active[i] / dm.Nb;
    if (i == 0 || tb.active[i - 1] / dm.Nb != r) tb.req_first[r] = i;
  }
  int carry = 0;
  for (int base = 0; base < nA; base += kPlanThreads) {
    const int i = base + tid;
    int np = 0;
    if (i < nA) {
      np = ceil_div_i(tb.seq_len[i], dm.pt);
      if (inline_prefix) np += ceil_div_i(tb.prefix_len[tb.active[i] / dm.Nb], dm.pt);
    }
    int tot;
    const int ex = block_excl_scan_i(np, lds, tot);
    if (i < nA) tb.page_cum[i] = carry + ex;
    carry += tot;
  }
  if (tid == 0) tb.page_cum[nA] = carry;
  const long long units = (long long)carry * dm.Hkv;
  const int n_waves = a.n_wg * kAttnWaves;
  int per_wave = (int)((units + n_waves - 1) / n_waves);
  if (per_wave < 1) per_wave = 1;

  int n_items = 0, n_live = 0, chunk = 0;
  if (!inline_prefix) {
    // pass 1: total prompt work, to size the chunk so that the items about fill the grid
    int w_carry = 0;
    for (int base = 0; base < nA; base += kPlanThreads) {
      const int i = base + tid;
      int w = 0;
      if (i < nA) {
        const int r = tb.active[i] / dm.Nb;
        if (tb.req_first[r] == i)
          w = ceil_div_i(tb.prefix_len[r], dm.pt) * ceil_div_i(tb.refcnt[r], kAttnWaves) * dm.Hkv;
      }
      int tot;
      block_excl_scan_i(w, lds, tot);
      w_carry += tot;
    }
    chunk = a.chunk_pages;
    if (chunk <= 0) chunk = ceil_div_i(w_carry, a.n_wg > 0 ? a.n_wg : 1);
    chunk = ceil_div_i(chunk < 1 ? 1 : chunk, kStagePages) * kStagePages;
    // pass 2: the live-request list and its item offsets
    int l_carry = 0, i_carry = 0;
    for (int base = 0; base < nA; base += kPlanThreads) {
      const int i = base + tid;
      int is_live = 0, items = 0, r = 0;
      if (i < nA) {
        r = tb.active[i] / dm.Nb;
        const int pp = ceil_div_i(tb.prefix_len[r], dm.pt);
        if (tb.req_first[r] == i && pp > 0) {
          is_live = 1;
          const int nck = ceil_div_i(pp, chunk);
          items = dm.Hkv * nck * ceil_div_i(tb.refcnt[r], kAttnWaves);
          atomicMax(&s_npc, nck);
        }
      }
      int tl, ti;
      const int exl = block_excl_scan_i(is_live, lds, tl);
      const int exi = block_excl_scan_i(items, lds, ti);
      if (is_live) { tb.live_req[l_carry + exl] = r; tb.live_item_start[l_carry + exl] = i_carry + exi; }
      l_carry += tl;
      i_carry += ti;
    }
    n_live = l_carry;
    n_items = i_carry;
    if (tid == 0) tb.live_item_start[n_live] = n_items;
  }
  __syncthreads();
  if (tid == 0) {
    scal[S_D_NA] = nA;
    scal[S_D_UNITS] = (int)units;
    scal[S_D_PER_WAVE] = per_wave;
    scal[S_D_NITEMS] = n_items;
    scal[S_D_NLIVE] = n_live;
    scal[S_D_CHUNK] = chunk;
    scal[S_D_NPC] = s_npc;
    scal[S_CALLOK] = 1;
  }
}

// ---------------------------------------------------------------------------
// Online-softmax state of one wave for one (row, kv head): the 16 x d tile
// O^T as matrix-core accumulators, running max m and per-lane partial sum l.
// Lane (r = lane & 15, g = lane >> 4) holds head r, tokens 4g..4g+3 of a page
// and output columns d = 16*blk + 4g + j.
// ---------------------------------------------------------------------------
template <int D>
struct WaveState {
  f32x4 o[D / 16];
  float m, l;
  __device__ inline void reset() {
#pragma unroll
    for (int b = 0; b < D / 16; ++b) o[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    m = -__builtin_inff();
    l = 0.f;
  }
};

// One 16-token page: kq[i] / vq[i] are the 16-byte chunks this lane loaded
// (chunk i*64 + lane of the K resp. V tile), qreg the Q^T operand.
template <int D>
__device__ inline void process_page(WaveState<D>& st, const uint4* kq, const uint4* vq, const uint4* qreg,
                                    int nvalid, float scale_log2) {
  const int g = (threadIdx.x & 63) >> 4;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kq[i]),
                                                __builtin_bit_cast(bf16x8, qreg[i]), s, 0, 0, 0);
  float sv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) sv[j] = s[j] * scale_log2;
  uint4 vloc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i) vloc[i] = vq[i];
  if (nvalid < 16) {  // wave-uniform: only the last page of a sequence
    const int t0 = 4 * g;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (t0 + j >= nvalid) sv[j] = -__builtin_inff();
    const unsigned m01 = (t0 + 0 < nvalid ? 0x0000ffffu : 0u) | (t0 + 1 < nvalid ? 0xffff0000u : 0u);
    const unsigned m23 = (t0 + 2 < nvalid ? 0x0000ffffu : 0u) | (t0 + 3 < nvalid ? 0xffff0000u : 0u);
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      vloc[i].x &= m01; vloc[i].y &= m23; vloc[i].z &= m01; vloc[i].w &= m23;
    }
  }
  float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(st.m, mx);          // finite: a page holds >= 1 valid token
  const float alpha = exp2f(st.m - m_new);      // 0 on the first page (m = -inf)
  st.m = m_new;
  f32x4 p;
#pragma unroll
  for (int j = 0; j < 4; ++j) p[j] = exp2f(sv[j] - m_new);
  st.l = st.l * alpha + (p[0] + p[1]) + (p[2] + p[3]);
  if (__any(alpha != 1.0f)) {
#pragma unroll
    for (int b = 0; b < D / 16; ++b) st.o[b] *= alpha;
  }
  const s16x4 pb = __builtin_bit_cast(s16x4, __builtin_convertvector(p, bf16x4));
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    const uint2 lo = {vloc[i].x, vloc[i].y}, hi = {vloc[i].z, vloc[i].w};
    st.o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, lo), pb, st.o[2 * i], 0, 0, 0);
    st.o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, hi), pb, st.o[2 * i + 1], 0, 0, 0);
  }
}

template <int D>
__device__ inline void load_q(uint4* qreg, const uint16_t* q, const Dims& dm, int row, int head) {
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    qreg[i] = uint4{0u, 0u, 0u, 0u};
    if (r < dm.G)
      qreg[i] = *(const uint4*)(q + ((long long)row * dm.Hq + head * dm.G + r) * D + i * 32 + g * 8);
  }
}

template <int D>
__device__ inline void store_partial(const WaveState<D>& st, float* partials, long long slot, const Dims& dm) {
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  float l = st.l;
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  if (r >= dm.G) return;
  float* base = partials + slot * partial_floats(dm.G, D);
#pragma unroll
  for (int b = 0; b < D / 16; ++b) *(f32x4*)(base + (long long)r * D + b * 16 + 4 * g) = st.o[b];
  if (g == 0) {
    base[(long long)dm.G * D + r] = st.m;
    base[(long long)dm.G * D + dm.G + r] = l;
  }
}

// ---------------------------------------------------------------------------
// A4 + A5: persistent attention kernel (bf16, SART_LAYOUT_MFMA16, 16-token pages).
// ---------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kAttnThreads)
k_attn_mfma(Ctx c, DecodeArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  constexpr int KQ = D / 32;                       // 16-byte chunks per lane per tile
  constexpr int kTileBytes = 16 * D * 2;           // one K (or V) tile
  constexpr int kPageBytes = 2 * kTileBytes;       // K tile + V tile of one kv head
  __shared__ __attribute__((aligned(16))) unsigned char lds_kv[2][kStagePages][kPageBytes];

  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nA = scal[S_D_NA];
  const int chunk = scal[S_D_CHUNK], npc = scal[S_D_NPC];
  const int n_items = scal[S_D_NITEMS], n_live = scal[S_D_NLIVE];
  const int n_waves = gridDim.x * kAttnWaves;
  const long long S = (long long)nA * dm.Hkv;
  const long long prefix_base = (long long)n_waves + S;
  const uint16_t* q = (const uint16_t*)a.q;
  const unsigned char* pool = (const unsigned char*)c.pool;
  const int* bt = tb.bt[scal[S_BTSEL]];
  WaveState<D> st;
  uint4 qreg[KQ];

  // ---- shared prompt items -------------------------------------------------
  for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
    int lo = 0, hi = n_live - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (tb.live_item_start[mid] <= it) lo = mid; else hi = mid - 1;
    }
    const int r = tb.live_req[lo];
    int local = it - tb.live_item_start[lo];
    const int cnt = tb.refcnt[r], first = tb.req_first[r];
    const int plen = tb.prefix_len[r];
    const int pp = ceil_div_i(plen, 16);
    const int nck = ceil_div_i(pp, chunk), ngr = ceil_div_i(cnt, kAttnWaves);
    const int bg = local % ngr; local /= ngr;
    const int ck = local % nck;
    const int h = local / nck;
    const int p0 = ck * chunk, p1 = min(pp, p0 + chunk);
    const int slot_in_req = bg * kAttnWaves + wv;
    const bool have_row = slot_in_req < cnt;
    const int row = first + slot_in_req;
    const int* ptab = tb.prefix_table + (long long)r * dm.max_pp;
    if (have_row) { load_q<D>(qreg, q, dm, row, h); st.reset(); }

    const int nst = ceil_div_i(p1 - p0, kStagePages);
    const bool loader = threadIdx.x * 16 < kPageBytes;
    uint4 greg[kStagePages];
    auto g_load = [&](int stg) {
#pragma unroll
      for (int k = 0; k < kStagePages; ++k) {
        const int p = p0 + stg * kStagePages + k;
        if (p < p1 && loader) {
          const long long off = (tile_base(dm, ptab[p], h) * 2) + threadIdx.x * 16;
          greg[k] = *(const uint4*)(pool + off);
        }
      }
    };
    auto l_store = [&](int stg) {
#pragma unroll
      for (int k = 0; k < kStagePages; ++k) {
        const int p = p0 + stg * kStagePages + k;
        if (p < p1 && loader) *(uint4*)(&lds_kv[stg & 1][k][threadIdx.x * 16]) = greg[k];
      }
    };
    __syncthreads();   // the previous item's readers are done with both buffers
    g_load(0);
    l_store(0);
    __syncthreads();
    for (int stg = 0; stg < nst; ++stg) {
      if (stg + 1 < nst) g_load(stg + 1);
      if (have_row) {
#pragma unroll
        for (int k = 0; k < kStagePages; ++k) {
          const int p = p0 + stg * kStagePages + k;
          if (p < p1) {
            uint4 kq[KQ], vq[KQ];
#pragma unroll
            for (int i = 0; i < KQ; ++i) {
              kq[i] = *(const uint4*)(&lds_kv[stg & 1][k][i * 1024 + lane * 16]);
              vq[i] = *(const uint4*)(&lds_kv[stg & 1][k][kTileBytes + i * 1024 + lane * 16]);
            }
            const int nvalid = min(16, plen - p * 16);
            process_page<D>(st, kq, vq, qreg, nvalid, a.scale_log2);
          }
        }
      }
      if (stg + 1 < nst) l_store(stg + 1);
      __syncthreads();
    }
    if (have_row)
      store_partial<D>(st, a.partials, prefix_base + ((long long)row * dm.Hkv + h) * npc + ck, dm);
  }

  // ---- private pages: this wave's range of (page, kv head) units ------------
  const long long units = (long long)tb.page_cum[nA] * dm.Hkv;
  const int per = scal[S_D_PER_WAVE];
  const long long w = (long long)blockIdx.x * kAttnWaves + wv;
  long long u = w * per;
  const long long u1 = min(units, u + per);
  if (u >= u1) return;
  // row containing unit u: last row with Hkv * page_cum[row] <= u and pages > 0
  int row;
  {
    int lo = 0, hi = nA - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((long long)tb.page_cum[mid] * dm.Hkv <= u) lo = mid; else hi = mid - 1;
    }
    row = lo;
  }
  while (u < u1) {
    int pages = tb.page_cum[row + 1] - tb.page_cum[row];
    long long rem = u - (long long)tb.page_cum[row] * dm.Hkv;
    while (pages == 0 || rem >= (long long)pages * dm.Hkv) {  // skip rows without private pages
      ++row;
      pages = tb.page_cum[row + 1] - tb.page_cum[row];
      rem = u - (long long)tb.page_cum[row] * dm.Hkv;
    }
    const int h = (int)(rem / pages);
    const int p0 = (int)(rem % pages);
    const int n = (int)min((long long)(pages - p0), u1 - u);
    const int len = tb.seq_len[row];
    const int* table = bt + (long long)row * dm.max_bp;
    load_q<D>(qreg, q, dm, row, h);
    st.reset();
    const long long head_off = (long long)h * kPageBytes + lane * 16;
    const long long page_bytes = dm.page_elems * 2;

    auto load_page = [&](uint4* kq, uint4* vq, int pid) {
      const unsigned char* base = pool + (long long)pid * page_bytes + head_off;
#pragma unroll
      for (int i = 0; i < KQ; ++i) {
        kq[i] = *(const uint4*)(base + i * 1024);
        vq[i] = *(const uint4*)(base + kTileBytes + i * 1024);
      }
    };
    // pages are taken 64 at a time: one coalesced read of the block table,
    // then page ids are broadcast from lanes
    for (int b0 = 0; b0 < n; b0 += 64) {
      const int nb = min(64, n - b0);
      const int my_pid = lane < nb ? table[p0 + b0 + lane] : 0;
      uint4 k0[KQ], v0[KQ], k1[KQ], v1[KQ];
      load_page(k0, v0, __shfl(my_pid, 0, 64));
      for (int i = 0; i < nb; i += 2) {
        if (i + 1 < nb) load_page(k1, v1, __shfl(my_pid, i + 1, 64));
        {
          const int p = p0 + b0 + i;
          process_page<D>(st, k0, v0, qreg, min(16, len - p * 16), a.scale_log2);
        }
        if (i + 2 < nb) load_page(k0, v0, __shfl(my_pid, i + 2, 64));
        if (i + 1 < nb) {
          const int p = p0 + b0 + i + 1;
          process_page<D>(st, k1, v1, qreg, min(16, len - p * 16), a.scale_log2);
        }
      }
    }
    store_partial<D>(st, a.partials, w + (long long)row * dm.Hkv + h, dm);
    u += n;
  }
}

// ---------------------------------------------------------------------------
// Generic kernel (any dtype, SART_LAYOUT_NATURAL, any page size and head dim
// <= 256): same unit line and partial format; one wave per range; the prompt
// is read inline as the first pages of every row.  Used for fp32 caches and
// for shapes the matrix-core tile does not cover; not a tuned path.
// ---------------------------------------------------------------------------
template <typename T> __device__ inline float to_f32(T x);
template <> __device__ inline float to_f32<float>(float x) { return x; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t x) { return __uint_as_float((unsigned)x << 16); }

template <typename T>
__global__ void __launch_bounds__(kAttnThreads)
k_attn_generic(Ctx c, DecodeArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nA = scal[S_D_NA];
  const int* bt = tb.bt[scal[S_BTSEL]];
  const T* pool = (const T*)c.pool;
  const T* q = (const T*)a.q;
  const int D = dm.d, pt = dm.pt;
  const long long units = (long long)tb.page_cum[nA] * dm.Hkv;
  const int per = scal[S_D_PER_WAVE];
  const long long w = (long long)blockIdx.x * kAttnWaves + wv;
  long long u = w * per;
  const long long u1 = min(units, u + per);
  if (u >= u1) return;
  int row;
  {
    int lo = 0, hi = nA - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((long long)tb.page_cum[mid] * dm.Hkv <= u) lo = mid; else hi = mid - 1;
    }
    row = lo;
  }
  while (u < u1) {
    int pages = tb.page_cum[row + 1] - tb.page_cum[row];
    long long rem = u - (long long)tb.page_cum[row] * dm.Hkv;
    while (pages == 0 || rem >= (long long)pages * dm.Hkv) {
      ++row;
      pages = tb.page_cum[row + 1] - tb.page_cum[row];
      rem = u - (long long)tb.page_cum[row] * dm.Hkv;
    }
    const int h = (int)(rem / pages);
    const int p0 = (int)(rem % pages);
    const int n = (int)min((long long)(pages - p0), u1 - u);
    const int req = tb.active[row] / dm.Nb;
    const int plen = tb.prefix_len[req], len = tb.seq_len[row];
    const int pp = ceil_div_i(plen, pt);
    const int* ptab = tb.prefix_table + (long long)req * dm.max_pp;
    const int* table = bt + (long long)row * dm.max_bp;
    float* pbase = a.partials + (w + (long long)row * dm.Hkv + h) * partial_floats(dm.G, D);
    for (int r = 0; r < dm.G; ++r) {
      const T* qrow = q + ((long long)row * dm.Hq + h * dm.G + r) * D;
      float m = -__builtin_inff(), l = 0.f;
      float o[4] = {0.f, 0.f, 0.f, 0.f};   // d = lane + 64*c
      for (int p = p0; p < p0 + n; ++p) {
        const bool in_prompt = p < pp;
        const int page = in_prompt ? ptab[p] : table[p - pp];
        const int nvalid = in_prompt ? min(pt, plen - p * pt) : min(pt, len - (p - pp) * pt);
        const long long kb = tile_base(dm, page, h), vb = kb + dm.tile_elems;
        for (int t0 = 0; t0 < nvalid; t0 += 64) {
          const int t = t0 + lane;
          float s = -__builtin_inff();
          if (t < nvalid) {
            float dot = 0.f;
            for (int d = 0; d < D; ++d) dot = fmaf(to_f32<T>(qrow[d]), to_f32<T>(pool[kb + (long long)t * D + d]), dot);
            s = dot * a.scale_log2;
          }
          float mx = s;
#pragma unroll
          for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
          const float m_new = fmaxf(m, mx);
          const float alpha = exp2f(m - m_new);
          const float pw = t < nvalid ? exp2f(s - m_new) : 0.f;
          float ps = pw;
#pragma unroll
          for (int off = 32; off >= 1; off >>= 1) ps += __shfl_xor(ps, off, 64);
          l = l * alpha + ps;
          m = m_new;
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) o[cc] *= alpha;
          const int nt = min(64, nvalid - t0);
          for (int j = 0; j < nt; ++j) {
            const float pj = __shfl(pw, j, 64);
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
              const int d = lane + 64 * cc;
              if (d < D) o[cc] = fmaf(pj, to_f32<T>(pool[vb + (long long)(t0 + j) * D + d]), o[cc]);
            }
          }
        }
      }
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int d = lane + 64 * cc;
        if (d < D) pbase[(long long)r * D + d] = o[cc];
      }
      if (lane == 0) {
        pbase[(long long)dm.G * D + r] = m;
        pbase[(long long)dm.G * D + dm.G + r] = l;
      }
    }
    u += n;
  }
}

// ---------------------------------------------------------------------------
// A6: merge.  One wave per output row (active row, query head):
//   m = max m_i,  l = sum l_i 2^(m_i - m),  out = sum o_i 2^(m_i - m) / l
// over the prompt-chunk partials and the private pieces, in slot order.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_merge(Ctx c, DecodeArgs a, int inline_prefix, int n_attn_waves) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  const int lane = threadIdx.x & 63;
  const int nA = scal[S_D_NA];
  const int chunk = scal[S_D_CHUNK], npc = scal[S_D_NPC], per = scal[S_D_PER_WAVE];
  const int D = dm.d, G = dm.G;
  const long long pf = partial_floats(G, D);
  const long long S = (long long)nA * dm.Hkv;
  const long long prefix_base = (long long)n_attn_waves + S;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
  for (long long orow = wave; orow < (long long)nA * dm.Hq; orow += nwaves) {
    const int row = (int)(orow / dm.Hq), qh = (int)(orow % dm.Hq);
    const int h = qh / G, r = qh % G;
    const long long seg = (long long)row * dm.Hkv + h;
    // slot ranges: [pa, pa+pn) prompt chunks, [sa, sa+sn) private pieces
    long long pa = 0, sa = 0;
    int pn = 0, sn = 0;
    if (!inline_prefix) {
      const int pp = ceil_div_i(tb.prefix_len[tb.active[row] / dm.Nb], dm.pt);
      pn = pp > 0 ? ceil_div_i(pp, chunk) : 0;
      pa = prefix_base + seg * npc;
    }
    const int pages = tb.page_cum[row + 1] - tb.page_cum[row];
    if (pages > 0) {
      const long long us = (long long)tb.page_cum[row] * dm.Hkv + (long long)h * pages;
      const long long w0 = us / per, w1 = (us + pages - 1) / per;
      sa = w0 + seg;
      sn = (int)(w1 - w0 + 1);
    }
    float m = -__builtin_inff();
    for (int i = 0; i < pn + sn; ++i) {
      const long long slot = i < pn ? pa + i : sa + (i - pn);
      m = fmaxf(m, a.partials[slot * pf + (long long)G * D + r]);
    }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int i = 0; i < pn + sn; ++i) {
      const long long slot = i < pn ? pa + i : sa + (i - pn);
      const float* pb = a.partials + slot * pf;
      const float wgt = exp2f(pb[(long long)G * D + r] - m);
      l += wgt * pb[(long long)G * D + G + r];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int d = lane + 64 * cc;
        if (d < D) acc[cc] = fmaf(wgt, pb[(long long)r * D + d], acc[cc]);
      }
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      const int d = lane + 64 * cc;
      if (d < D) a.out[orow * D + d] = acc[cc] * inv;
    }
  }
}

void launch_decode(const Ctx& c, const DecodeArgs& a, hipStream_t s) {
  const Dims& dm = c.dm;
  const bool mfma = dm.layout == SART_LAYOUT_MFMA16;
  const int inline_prefix = mfma ? 0 : 1;
  if (a.ev[0]) (void)hipEventRecord(a.ev[0], s);
  hipLaunchKernelGGL(k_decode_plan, dim3(1), dim3(kPlanThreads), 0, s, c, a, inline_prefix);
  if (a.ev[1]) (void)hipEventRecord(a.ev[1], s);
  if (mfma) {
    if (dm.d == 128)
      hipLaunchKernelGGL(k_attn_mfma<128>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
    else
      hipLaunchKernelGGL(k_attn_mfma<64>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
  } else if (dm.dtype == SART_F32) {
    hipLaunchKernelGGL(k_attn_generic<float>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
  } else {
    hipLaunchKernelGGL(k_attn_generic<uint16_t>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
  }
  if (a.ev[2]) (void)hipEventRecord(a.ev[2], s);
  const long long out_rows = (long long)dm.H * dm.Hq;
  long long blocks = (out_rows + 3) / 4;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_merge, dim3((unsigned)blocks), dim3(256), 0, s, c, a, inline_prefix, a.n_wg * kAttnWaves);
  if (a.ev[3]) (void)hipEventRecord(a.ev[3], s);
}

}  // namespace sart
