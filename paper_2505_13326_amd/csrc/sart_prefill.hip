// Prefill attention over a request's prompt (Algorithm 1, Prefill; arXiv
// 2505.13326).  The paper treats the prefill phase as that of plain LLM
// inference (Section 4), so what is computed is causal self-attention: the
// query of the prompt token at position p reads prompt tokens 0..p through the
// request's prefix table.  A call names requests and, for each, how many of its
// last prompt tokens are the queries (all of them: whole prefill; fewer: one
// chunk of a chunked prefill, after that chunk's K/V was appended).
//
// Design for MI355X (gfx950).  Unlike decode this is a dense contraction with
// reuse: a K/V page serves every later query.  The rows of one kv head -
// (query, head of the GQA group), query-major - are cut into tiles of
// kPfTileRows, one workgroup per tile, on the matrix-core tile the decode kernel
// uses (S^T = K Q^T and O^T += V^T P^T as 16x16x32 bf16 products; online softmax
// on the vector ALUs).  Pages are taken two at a time (32 tokens): one update of
// the maximum per 32 tokens.  Blocks skip pairs that lie wholly after their
// rows' positions and mask scores only on the pairs that straddle them.  No
// split over the sequence: one wave sees a row's whole context, so there is no
// merge.  Two kernels: k_prefill_mfma (8-bit float caches: every wave loads its
// page pairs into registers and expands them there) and k_prefill_lds8 (bf16
// caches: pairs staged once per workgroup in LDS, 8 waves per tile).
#include <type_traits>

#include "sart_attn_tile.h"

namespace sart {

constexpr int kPfRowsPerWave = 16 * kPfBlocks;
constexpr int kPfRowsPerWg = kPfRowsPerWave * kAttnWaves;       // = kPfTileRows

// Device-side validation of the call (one workgroup): every listed request must
// be live and hold at least as many prompt tokens as it has queries.
__global__ void __launch_bounds__(256)
k_prefill_check(Ctx c, PrefillArgs a) {
  const Tables& tb = c.tb;
  __shared__ int s_err;
  if (threadIdx.x == 0) s_err = 0x7fffffff;
  __syncthreads();
  for (int i = threadIdx.x; i < a.n_seqs; i += blockDim.x) {
    const int r = a.ids[i];
    int err = 0;
    if (!tb.req_used[r] || tb.refcnt[r] == 0) err = SART_E_STATE;
    else if (a.nq[i] > tb.prefix_len[r]) err = SART_E_INVALID;
    if (err) atomicMin(&s_err, (i << 2) | err);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (s_err != 0x7fffffff) record_error(tb.scal, s_err & 3, a.call_seq);
    else tb.scal[S_CALLOK] = 1;
  }
}

// index of the last entry of the ascending array v[0..n) that is <= x (v[0] <= x)
__device__ inline int last_le(const int* v, int n, int x) {
  int lo = 0, hi = n - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (v[mid] <= x) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// (Launched for 8-bit float caches; bf16 caches take k_prefill_lds8 below.)
template <int D, bool FP8>
__global__ void __launch_bounds__(kAttnThreads, 2)
k_prefill_mfma(Ctx c, PrefillArgs a, const int* __restrict__ prefix_table) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  if (!tb.scal[S_CALLOK]) return;
  constexpr int KQ = D / 32;
  constexpr int KR = raw_chunks<D, FP8>();                 // 16-byte chunks per lane per tile as stored
  constexpr int kTileBytes = 16 * D * (FP8 ? 1 : 2), kPageBytes = 2 * kTileBytes;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r16 = lane & 15, g4 = lane >> 4;
  // tile -> (sequence, kv head, row tile); a sequence's later rows (longer contexts) come first
  const int tile = blockIdx.x;
  const int i = last_le(a.tile_start, a.n_seqs, tile);
  const int req = a.ids[i], nq = a.nq[i], plen = tb.prefix_len[req];
  const int n_rows = nq * dm.G;
  const int tiles_per_head = ceil_div(n_rows, kPfRowsPerWg);
  const int local = tile - a.tile_start[i];
  const int h = local / tiles_per_head;
  const int rt = tiles_per_head - 1 - local % tiles_per_head;
  const int row_w0 = rt * kPfRowsPerWg + wv * kPfRowsPerWave;
  if (row_w0 >= n_rows) return;
  const int p_first = plen - nq;                           // prompt position of the call's first query
  const long long q_row0 = a.q_off[i];
  const uint16_t* q = (const uint16_t*)a.q;
  const unsigned char* pool = (const unsigned char*)c.pool;
  const int* __restrict__ table = prefix_table + (long long)req * dm.max_pp;
  const long long page_bytes = dm.page_elems * (FP8 ? 1 : 2);
  const long long head_off = (long long)h * kPageBytes + lane * 16;

  // per 16-row block: this lane's row, its position, the block's position range
  WaveState<D> st[kPfBlocks];
  uint4 qreg[kPfBlocks][KQ];
  int pos[kPfBlocks], lo_pos[kPfBlocks], hi_pos[kPfBlocks];
  long long out_row[kPfBlocks];                            // element offset of this lane's output row, -1: no row
#pragma unroll
  for (int b = 0; b < kPfBlocks; ++b) {
    const int row0 = row_w0 + 16 * b;
    const int row = row0 + r16;
    const bool have = row < n_rows;
    const int rc = have ? row : n_rows - 1;               // rows past the end shadow the last one, and are not stored
    const int ql = rc / dm.G, g = rc % dm.G;
    pos[b] = p_first + ql;
    lo_pos[b] = row0 < n_rows ? p_first + row0 / dm.G : -1;
    hi_pos[b] = row0 < n_rows ? p_first + min(row0 + 15, n_rows - 1) / dm.G : -1;
    const long long qrow = ((q_row0 + ql) * dm.Hq + h * dm.G + g) * D;
    out_row[b] = have ? qrow : -1;
#pragma unroll
    for (int k = 0; k < KQ; ++k) qreg[b][k] = *(const uint4*)(q + qrow + k * 32 + g4 * 8);
    st[b].reset();
  }
  const int last_pos = p_first + min(row_w0 + kPfRowsPerWave - 1, n_rows - 1) / dm.G;
  const int n_pages = last_pos / 16 + 1;

  // Pages are taken two at a time (32 tokens); an odd last page is paired with itself, masked.
  // One register buffer per operand: K of the next pair is requested as soon as the scores of all
  // blocks are done, V after the last O^T product, so each load has half a turn to arrive.  Every
  // load is unconditional (past the end the last pair again).
  const int n_pairs = (n_pages + 1) >> 1;
  // K as stored; V as stored (8-bit float caches) or, for bf16, loaded in 8-byte halves straight into
  // the layout of the O^T product's operand (v0 = lo, v1 = hi of pair_pv_lohi): no register shuffling
  uint4 k0[KR], k1[KR], v0[KR], v1[KR];
  auto load_k = [&](int pr) {
    const unsigned char* b0 = pool + (long long)table[2 * pr] * page_bytes + head_off;
    const unsigned char* b1 = pool + (long long)table[min(2 * pr + 1, n_pages - 1)] * page_bytes + head_off;
#pragma unroll
    for (int k = 0; k < KR; ++k) { k0[k] = *(const uint4*)(b0 + k * 1024); k1[k] = *(const uint4*)(b1 + k * 1024); }
  };
  auto load_v = [&](int pr) {
    const unsigned char* b0 = pool + (long long)table[2 * pr] * page_bytes + head_off + kTileBytes;
    const unsigned char* b1 = pool + (long long)table[min(2 * pr + 1, n_pages - 1)] * page_bytes + head_off + kTileBytes;
#pragma unroll
    for (int k = 0; k < KR; ++k) {
      if constexpr (FP8) {
        v0[k] = *(const uint4*)(b0 + k * 1024);
        v1[k] = *(const uint4*)(b1 + k * 1024);
      } else {
        const uint2 a_lo = *(const uint2*)(b0 + k * 1024), a_hi = *(const uint2*)(b0 + k * 1024 + 8);
        const uint2 b_lo = *(const uint2*)(b1 + k * 1024), b_hi = *(const uint2*)(b1 + k * 1024 + 8);
        v0[k] = uint4{a_lo.x, a_lo.y, b_lo.x, b_lo.y};
        v1[k] = uint4{a_hi.x, a_hi.y, b_hi.x, b_hi.y};
      }
    }
  };
  // the bf16 operands of a tile: the registers as loaded, or their expansion
  auto operands = [&](const uint4* raw, uint4* tmp) -> const uint4* {
    if constexpr (FP8) { expand_fp8<D>(raw, tmp); return tmp; } else { return raw; }
  };
  // O^T += V^T P^T of one block, FULL or masked by the tokens the pair holds
  auto pv = [&](WaveState<D>& stb, bf16x8 ppb, auto full, int nvalid) {
    constexpr bool FULLV = decltype(full)::value;
    if constexpr (FP8) {
      uint4 tv0[KQ], tv1[KQ];
      expand_fp8<D>(v0, tv0);
      expand_fp8<D>(v1, tv1);
      pair_pv<D, FULLV>(stb, tv0, tv1, ppb, nvalid);
    } else {
      pair_pv_lohi<D, FULLV>(stb, v0, v1, ppb, nvalid);
    }
  };
  load_k(0);
  load_v(0);
  for (int pr = 0; pr < n_pairs; ++pr) {
    const int t0 = pr * 32;
    const int nxt = min(pr + 1, n_pairs - 1);
    uint4 tk0[FP8 ? KQ : 1], tk1[FP8 ? KQ : 1];
    f32x4 s0[kPfBlocks], s1[kPfBlocks];
    bf16x8 pp[kPfBlocks];
    const uint4* q0 = operands(k0, tk0);
    const uint4* q1 = operands(k1, tk1);
    if (t0 + 31 <= lo_pos[0]) {
      // every row of the wave sees the whole pair: phase by phase over the wave's independent blocks
#pragma unroll
      for (int b = 0; b < kPfBlocks; ++b) pair_scores<D, 1>(q0, q1, qreg[b], s0[b], s1[b]);
      load_k(nxt);
#pragma unroll
      for (int b = 0; b < kPfBlocks; ++b) pp[b] = pair_softmax<D, true>(st[b], s0[b], s1[b], 32, a.scale_log2);
#pragma unroll
      for (int b = 0; b < kPfBlocks; ++b) pv(st[b], pp[b], std::true_type{}, 32);
      load_v(nxt);
    } else {
      // pairs that straddle some row's position: block by block, scores masked per row
      const int nvalid = min(32, min(plen, n_pages * 16) - t0);      // tokens the pair holds
#pragma unroll
      for (int b = 0; b < kPfBlocks; ++b) {
        if (t0 > hi_pos[b]) continue;                        // the pair lies after every row of the block
        pair_scores<D, 1>(q0, q1, qreg[b], s0[b], s1[b]);
        if (t0 + 31 <= lo_pos[b]) {
          pp[b] = pair_softmax<D, true>(st[b], s0[b], s1[b], 32, a.scale_log2);
          pv(st[b], pp[b], std::true_type{}, 32);
        } else {
          pp[b] = pair_softmax<D, false>(st[b], s0[b], s1[b], min(nvalid, pos[b] + 1 - t0), a.scale_log2);
          pv(st[b], pp[b], std::false_type{}, nvalid);
        }
      }
      load_k(nxt);
      load_v(nxt);
    }
  }
#pragma unroll
  for (int b = 0; b < kPfBlocks; ++b) {
    const float l = sum_over_rows(st[b].l);
    if (out_row[b] < 0) continue;
    const float inv = a.v_scale / l;                       // every row sees at least its own token
    float* o = a.out + out_row[b];
#pragma unroll
    for (int k = 0; k < D / 16; ++k) *(f32x4*)(o + k * 16 + 4 * g4) = st[b].o[k] * inv;
  }
}

// The same computation for bf16 caches with K and V staged in LDS by the workgroup
// and more waves in flight: the tile's 128 rows go to 8 waves of 16 rows (112
// registers, so four waves share a SIMD and there is always one to switch to
// while another waits for a product, an LDS read or the barrier), and each page
// pair is fetched from memory once per workgroup - one 16-byte chunk of two tiles
// per thread - into a ring of three LDS stages (pair p is computed on while pair
// p + 1 is written and pair p + 2 is in flight: one barrier per pair).  V is
// written to LDS already in the layout of the O^T product's operand; operands are
// read from LDS slab by slab, right before their products.  Measured against the
// register kernel above: 452 vs 433 TFLOP/s on 64 x 1024-token prompts, 684 vs
// 605 on 64 x 8192.
template <int D>
__global__ void __launch_bounds__(512, 4)
k_prefill_lds8(Ctx c, PrefillArgs a, const int* __restrict__ prefix_table) {
  constexpr int NW = 8, NB = 1;
  static_assert(16 * NB * NW == kPfTileRows, "the host sizes the grid for tiles of kPfTileRows rows");
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  if (!tb.scal[S_CALLOK]) return;
  constexpr int KQ = D / 32;
  constexpr int kTileBytes = 16 * D * 2, kPageBytes = 2 * kTileBytes;
  constexpr int kChunks = kTileBytes / 16;                 // 16-byte chunks of one K (or V) tile
  constexpr int kStages = 3;
  // one stage: K of the pair's first and second page as stored, then V lo and V hi operands
  __shared__ uint4 lds[kStages][4][kChunks];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, g4 = lane >> 4;
  const int tile = blockIdx.x;
  const int i = last_le(a.tile_start, a.n_seqs, tile);
  const int req = a.ids[i], nq = a.nq[i], plen = tb.prefix_len[req];
  const int n_rows = nq * dm.G;
  const int tiles_per_head = ceil_div(n_rows, (16 * NB * NW));
  const int local = tile - a.tile_start[i];
  const int h = local / tiles_per_head;
  const int rt = tiles_per_head - 1 - local % tiles_per_head;
  const int row_w0 = rt * (16 * NB * NW) + wv * (16 * NB);
  const bool wave_has_rows = row_w0 < n_rows;              // a wave without rows still helps to load
  const int p_first = plen - nq;
  const long long q_row0 = a.q_off[i];
  const uint16_t* q = (const uint16_t*)a.q;
  const unsigned char* pool = (const unsigned char*)c.pool;
  const int* __restrict__ table = prefix_table + (long long)req * dm.max_pp;
  const long long page_bytes = dm.page_elems * 2;

  f32x4 lsum = {0.f, 0.f, 0.f, 0.f};                   // softmax denominators of the lane's query row (see pair_softmax_lagging)
  WaveState<D> st[NB];
  uint4 qreg[NB][KQ];
  int pos[NB], lo_pos[NB], hi_pos[NB];
  long long out_row[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int row0 = row_w0 + 16 * b;
    const int row = row0 + r16;
    const bool have = row < n_rows;
    const int rc = have ? row : n_rows - 1;
    const int ql = rc / dm.G, g = rc % dm.G;
    pos[b] = p_first + ql;
    lo_pos[b] = row0 < n_rows ? p_first + row0 / dm.G : -1;
    hi_pos[b] = row0 < n_rows ? p_first + min(row0 + 15, n_rows - 1) / dm.G : -1;
    const long long qrow = ((q_row0 + ql) * dm.Hq + h * dm.G + g) * D;
    out_row[b] = have ? qrow : -1;
#pragma unroll
    for (int k = 0; k < KQ; ++k) qreg[b][k] = *(const uint4*)(q + qrow + k * 32 + g4 * 8);
    st[b].reset();
  }
  // pages the tile needs (its last row's context) and those this wave needs
  const int tile_last_pos = p_first + min((rt + 1) * (16 * NB * NW) - 1, n_rows - 1) / dm.G;
  const int n_pages = tile_last_pos / 16 + 1;
  const int n_pairs = (n_pages + 1) >> 1;
  const int wave_last_pos = wave_has_rows ? p_first + min(row_w0 + (16 * NB) - 1, n_rows - 1) / dm.G : -1;
  const int wave_pairs = wave_has_rows ? wave_last_pos / 32 + 1 : 0;

  // loader: threads 0..kChunks-1 move chunk t of the two K tiles, the next kChunks threads chunk t of the two V tiles
  static_assert(2 * kChunks <= NW * 64, "one chunk pair per thread");
  uint4 ga, gb;
  const bool ld_k = tid < kChunks, ld_v = tid >= kChunks && tid < 2 * kChunks;
  const int lch = ld_k ? tid : tid - kChunks;
  auto g_load = [&](int pr) {
    const unsigned char* b0 = pool + (long long)table[2 * pr] * page_bytes + (long long)h * kPageBytes + (ld_v ? kTileBytes : 0);
    const unsigned char* b1 = pool + (long long)table[min(2 * pr + 1, n_pages - 1)] * page_bytes + (long long)h * kPageBytes + (ld_v ? kTileBytes : 0);
    if (ld_k || ld_v) { ga = *(const uint4*)(b0 + lch * 16); gb = *(const uint4*)(b1 + lch * 16); }
  };
  auto l_store = [&](int stage) {
    if (ld_k) { lds[stage][0][lch] = ga; lds[stage][1][lch] = gb; }
    if (ld_v) {
      lds[stage][2][lch] = uint4{ga.x, ga.y, gb.x, gb.y};
      lds[stage][3][lch] = uint4{ga.z, ga.w, gb.z, gb.w};
    }
  };
  g_load(0);
  l_store(0);
  g_load(min(1, n_pairs - 1));
  __syncthreads();
  for (int pr = 0; pr < n_pairs; ++pr) {
    const int stage = pr % kStages;
    l_store((pr + 1) % kStages);                           // pair pr + 1 (loaded a turn ago), read a turn from now
    g_load(min(pr + 2, n_pairs - 1));
    if (pr < wave_pairs) {
      const int t0 = pr * 32;
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < KQ; ++k) {
        const bf16x8 qk = __builtin_bit_cast(bf16x8, qreg[0][k]);
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lds[stage][0][k * 64 + lane]), qk, s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lds[stage][1][k * 64 + lane]), qk, s1, 0, 0, 0);
      }
      const bool full = t0 + 31 <= lo_pos[0];
      const int nvalid = min(32, min(plen, n_pages * 16) - t0);
      const bf16x8 pp = full ? pair_softmax_lagging<D, true>(st[0], lsum, s0, s1, 32, a.scale_log2)
                             : pair_softmax_lagging<D, false>(st[0], lsum, s0, s1, min(nvalid, pos[0] + 1 - t0), a.scale_log2);
      if (full) {
#pragma unroll
        for (int k = 0; k < KQ; ++k) {
          st[0].o[2 * k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lds[stage][2][k * 64 + lane]), pp, st[0].o[2 * k], 0, 0, 0);
          st[0].o[2 * k + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lds[stage][3][k * 64 + lane]), pp, st[0].o[2 * k + 1], 0, 0, 0);
        }
      } else {   // tokens the pair does not hold may be anything: zero their V
        uint4 lo[KQ], hi[KQ];
#pragma unroll
        for (int k = 0; k < KQ; ++k) { lo[k] = lds[stage][2][k * 64 + lane]; hi[k] = lds[stage][3][k * 64 + lane]; }
        pair_pv_lohi<D, false>(st[0], lo, hi, pp, nvalid);
      }
    }
    __syncthreads();
  }
  if (!wave_has_rows) return;
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const float l = lsum[0];
    if (out_row[b] < 0) continue;
    const float inv = a.v_scale / l;
    float* o = a.out + out_row[b];
#pragma unroll
    for (int k = 0; k < D / 16; ++k) *(f32x4*)(o + k * 16 + 4 * g4) = st[b].o[k] * inv;
  }
}

// Any dtype, SART_LAYOUT_NATURAL: one wave per (query, kv head), the heads of
// the group one after the other on the vector ALUs.  Not a tuned path.
template <typename T>
__global__ void __launch_bounds__(kAttnThreads)
k_prefill_generic(Ctx c, PrefillArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  if (!tb.scal[S_CALLOK]) return;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const T* pool = (const T*)c.pool;
  const T* q = (const T*)a.q;
  const int D = dm.d;
  const long long units = (long long)a.total_q * dm.Hkv;
  for (long long u = (long long)blockIdx.x * kAttnWaves + wv; u < units; u += (long long)gridDim.x * kAttnWaves) {
    const int gq = (int)(u / dm.Hkv), h = (int)(u % dm.Hkv);
    const int i = last_le(a.q_off, a.n_seqs, gq);
    const int req = a.ids[i];
    const int tokens = tb.prefix_len[req] - a.nq[i] + (gq - a.q_off[i]) + 1;     // prompt tokens 0..p
    const int* table = tb.prefix_table + (long long)req * dm.max_pp;
    for (int r = 0; r < dm.G; ++r) {
      const long long row = ((long long)gq * dm.Hq + h * dm.G + r) * D;
      float m = -__builtin_inff(), l = 0.f;
      float o[4] = {0.f, 0.f, 0.f, 0.f};
      generic_row<T>(dm, pool, table, 0, ceil_div(tokens, dm.pt), tokens, h, q + row, a.scale_log2, m, l, o);
      const float inv = a.v_scale / l;
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int d = lane + 64 * cc;
        if (d < D) a.out[row + d] = o[cc] * inv;
      }
    }
  }
}

void launch_prefill(const Ctx& c, const PrefillArgs& a, hipStream_t s) {
  const Dims& dm = c.dm;
  hipLaunchKernelGGL(k_prefill_check, dim3(1), dim3(256), 0, s, c, a);
  if (a.total_q <= 0) return;
  if (dm.layout != SART_LAYOUT_NATURAL) {
    auto go = [&](auto kern) {
      hipLaunchKernelGGL(kern, dim3(a.n_tiles), dim3(kAttnThreads), 0, s, c, a, c.tb.prefix_table);
    };
    const bool fp8 = dm.layout == SART_LAYOUT_MFMA16_FP8;
    if (!fp8) {   // bf16: the LDS-staged kernel with 8 waves per tile
      if (dm.d == 128) hipLaunchKernelGGL(k_prefill_lds8<128>, dim3(a.n_tiles), dim3(512), 0, s, c, a, c.tb.prefix_table);
      else hipLaunchKernelGGL(k_prefill_lds8<64>, dim3(a.n_tiles), dim3(512), 0, s, c, a, c.tb.prefix_table);
      return;
    }
    if (dm.d == 128) go(k_prefill_mfma<128, true>); else go(k_prefill_mfma<64, true>);   // 8-bit float caches
  } else {
    long long blocks = ((long long)a.total_q * dm.Hkv + kAttnWaves - 1) / kAttnWaves;
    if (blocks > 65536) blocks = 65536;
    if (dm.dtype == SART_F32)
      hipLaunchKernelGGL(k_prefill_generic<float>, dim3((unsigned)blocks), dim3(kAttnThreads), 0, s, c, a);
    else
      hipLaunchKernelGGL(k_prefill_generic<uint16_t>, dim3((unsigned)blocks), dim3(kAttnThreads), 0, s, c, a);
  }
}

}  // namespace sart
