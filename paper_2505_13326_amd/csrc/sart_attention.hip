// Decode-step attention over the active branches (the batched decoding
// step of Algorithm 1, Decode; arXiv 2505.13326).  The paper leaves the attention
// itself to the serving engine (Section 4: as in plain LLM inference), so what
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
//   * Shared prompt pages are read in blocks of pages, once per tile of 16
//     query rows of the request (rows = (branch, head of the GQA group)), the
//     work items ordered (request, kv head, chunk, tile) and served by every
//     wave before its own range, so the tiles' re-reads of a chunk are
//     neighbours in time and on one XCD and hit in its L2 (default).  The
//     other mode: one block per (chunk, branch).  (Staging prompt chunks in LDS
//     was built and measured: 2.5 to 3 times slower on the prompt-heavy
//     workloads and about twice the fetches; it is not in the library.)
#include <mutex>
#include <type_traits>

#include "sart_attn_tile.h"

namespace sart {

// A prompt of pp pages is read in nck = ceil(pp / pb) chunks (pb: the plan's block size); the chunks are made
// equal, ceil(pp / nck) pages rounded up to whole rings of 4 (never more than pb, so still nck chunks), rather
// than nck - 1 of pb pages and a short one: the work items over the chunks then take the same time.
__device__ inline int prompt_chunk_pages(int pp, int nck) { return ceil_div(ceil_div(pp, nck), 4) * 4; }

// partial slots the current plan writes: own pieces (one per range and per (row, kv head) it crosses),
// then the prompts' blocks
__device__ inline long long slots_needed(const int* scal, int Hkv) {
  return (long long)scal[S_D_NOWN] + (long long)scal[S_D_NA] * Hkv + (long long)scal[S_D_NBLOCKS];
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

// Partial results that another wave of the same kernel reads back (the in-kernel merge) are written and
// read with device-scope relaxed atomic accesses, one float each: such stores go through to memory and such
// loads do not take a stale line of the reader's L2 (the 8 XCDs have one L2 each, not coherent with each
// other for ordinary accesses), so no cache has to be written back or invalidated as a whole - a device-scope
// fence does exactly that and, measured, costs about 25 us per piece (config 2 kernel 0.336 against 0.244 ms).
// A partial result is a few KB per piece; the float-wise accesses do not show in the kernel's time.
template <bool COHERENT>
__device__ inline void put_f32x4(float* p, f32x4 v) {
  if constexpr (COHERENT) {
#pragma unroll
    for (int k = 0; k < 4; ++k) __hip_atomic_store(p + k, v[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    *(f32x4*)p = v;
  }
}
template <bool COHERENT>
__device__ inline void put_f32(float* p, float v) {
  if constexpr (COHERENT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
template <bool COHERENT>
__device__ inline f32x4 get_f32x4(const float* p) {
  if constexpr (COHERENT) {
    f32x4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = __hip_atomic_load(p + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return v;
  } else {
    return *(const f32x4*)p;
  }
}
template <bool COHERENT>
__device__ inline float get_f32(const float* p) {
  if constexpr (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

template <int D, bool COHERENT>
__device__ inline void store_partial(const WaveState<D>& st, float* partials, long long slot, const Dims& dm) {
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const float l = sum_over_rows(st.l);
  if (r >= dm.G) return;
  float* base = partials + slot * partial_floats(dm.G, D);
#pragma unroll
  for (int b = 0; b < D / 16; ++b) put_f32x4<COHERENT>(base + (long long)r * D + b * 16 + 4 * g, st.o[b]);
  if (g == 0) {
    put_f32<COHERENT>(base + (long long)dm.G * D + r, st.m);
    put_f32<COHERENT>(base + (long long)dm.G * D + dm.G + r, l);
  }
}

// ---------------------------------------------------------------------------
// A6 inside the attention kernel.  Every piece (a wave's part of one (row, kv
// head), or a prompt block) stores its partial result, then counts itself in
// for that (row, kv head); the plan says how many writers there are, so the
// writer that arrives last knows it is last and folds all the partial results
// in slot order (prompt chunks, then own pieces: the order does not depend on
// who arrived when, so the output is reproducible bit for bit) and writes the
// output rows.  No wave ever waits for another.  The counter is back to zero
// when the kernel ends.
// ---------------------------------------------------------------------------
struct RowInfo { int cum, pages, seq, prompt_writers, pslot, cnt, nck, handle; };   // see refresh_decode_plan (row_desc)
__device__ inline RowInfo load_row_info(const int* __restrict__ row_desc, int row) {
  const int4 x = ((const int4*)(row_desc + 8LL * row))[0], y = ((const int4*)(row_desc + 8LL * row))[1];
  return RowInfo{x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
}
// The row of q and out that belongs to active row `row`: the row itself, or the branch's handle when the
// caller addresses its buffers by handle.
__device__ inline int io_row(const DecodeArgs& a, const RowInfo& ri, int row) { return a.by_handle ? ri.handle : row; }
__device__ inline int io_row(const DecodeArgs& a, const int* __restrict__ row_desc, int row) {
  return a.by_handle ? row_desc[8LL * row + 7] : row;
}
// the own-line pieces of (row, kv head h): first range w0 and their number sn
__device__ inline void own_pieces(const Cut& cut, int Hkv, const RowInfo& ri, int h, long long& w0, int& sn) {
  w0 = 0; sn = 0;
  if (ri.pages == 0) return;
  const long long us = (long long)ri.cum * Hkv + (long long)h * ri.pages;
  w0 = own_of_unit(cut, us);
  sn = (int)(own_of_unit(cut, us + ri.pages - 1) - w0) + 1;
}
// Folds, for query head r of the group and output columns 4 d4 .. 4 d4 + 3, the partial results at slots
// pa + i * pstride (i < pn: prompt pieces) and then sa + i (i < sn: own pieces) with the running form of
//   m = max m_i,  l = sum l_i 2^(m_i - m),  out = sum o_i 2^(m_i - m) / l
// and writes the four outputs.  The loads of successive partial results are independent, so they overlap.
template <bool COHERENT>
__device__ inline void fold_columns(const float* partials, float* __restrict__ out_row, long long pf, int G, int D,
                                    int r, int d4, long long pa, long long pstride, int pn, long long sa, int sn, float v_scale) {
  float m = -__builtin_inff(), l = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int i = 0; i < pn + sn; ++i) {
    const long long slot = i < pn ? pa + i * pstride : sa + (i - pn);
    const float* pb = partials + slot * pf;
    const float mi = get_f32<COHERENT>(pb + (long long)G * D + r);
    const float li = get_f32<COHERENT>(pb + (long long)G * D + G + r);
    const f32x4 oi = get_f32x4<COHERENT>(pb + (long long)r * D + 4 * d4);
    const float mn = fmaxf(m, mi);
    const float ws = __builtin_amdgcn_exp2f(m - mn), wi = __builtin_amdgcn_exp2f(mi - mn);
    l = l * ws + li * wi;
    acc = acc * ws + oi * wi;
    m = mn;
  }
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  *(f32x4*)(out_row + 4 * d4) = acc * (inv * v_scale);
}
// Counts this wave's piece in for its (row, kv head); true for the writer that completes it (all lanes alike).
__device__ inline bool arrive_last(int* counter, int expected) {
  // the wave's partial-result stores (device-scope, see above) have completed before it counts itself in
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  int old = 0;
  if ((threadIdx.x & 63) == 0) old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != expected - 1) return false;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if ((threadIdx.x & 63) == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}
// One wave folds (row, kv head h) and writes its G output rows.
template <int D>
__device__ inline void fold_segment(const DecodeArgs& a, const Dims& dm, long long prompt_slot_base, int row, int h,
                                    const RowInfo& ri, long long w0, int sn) {
  const int lane = threadIdx.x & 63;
  constexpr int D4 = D / 4;
  const long long pf = partial_floats(dm.G, D);
  const long long sa = w0 + (long long)row * dm.Hkv + h;
  const long long pa = prompt_slot_base + ri.pslot + (long long)h * ri.nck * ri.cnt;
  for (int e = lane; e < dm.G * D4; e += 64) {
    const int r = e / D4, d4 = e % D4;
    fold_columns<true>(a.partials, a.out + ((long long)io_row(a, ri, row) * dm.Hq + h * dm.G + r) * D, pf, dm.G, D, r, d4, pa, ri.cnt, ri.nck, sa,
                       sn, a.v_scale);
  }
}
// End of a piece of (row, kv head h) whose state is st: the only piece writes the output rows itself; otherwise
// the partial result goes to `slot` and the last writer merges.
template <int D>
__device__ inline void finish_piece(const DecodeArgs& a, const Dims& dm, const Cut& cut, long long prompt_slot_base,
                                    const WaveState<D>& st, long long slot, int row, int h, const RowInfo& ri) {
  long long w0;
  int sn;
  own_pieces(cut, dm.Hkv, ri, h, w0, sn);
  const int expected = ri.prompt_writers + sn;
  if (expected == 1) {
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const float l = sum_over_rows(st.l);
    if (r >= dm.G) return;
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    float* orow = a.out + ((long long)io_row(a, ri, row) * dm.Hq + h * dm.G + r) * D;
#pragma unroll
    for (int b = 0; b < D / 16; ++b) *(f32x4*)(orow + b * 16 + 4 * g) = st.o[b] * (inv * a.v_scale);
    return;
  }
  store_partial<D, true>(st, a.partials, slot, dm);
  if (arrive_last(a.seg_count + ((long long)row * dm.Hkv + h), expected))
    fold_segment<D>(a, dm, prompt_slot_base, row, h, ri, w0, sn);
}

// ---------------------------------------------------------------------------
// A4 + A5: persistent attention kernel (SART_LAYOUT_MFMA16 / _FP8, 16-token pages).
// One 4-wave workgroup per CU, one wave per SIMD: two waves on a SIMD do not
// share it fairly (the older one streams about 1.5x faster, measured), which a
// static partition cannot absorb; memory-level parallelism comes from the
// per-wave ring of page buffers instead.  Every wave serves its share of the
// prompt work items and its range of the own line.
// bt0 / bt1 are the two block-table buffers again, as noalias kernel arguments:
// the compiler may then read page ids with scalar loads, which do not queue
// behind the in-flight vector loads of K/V tiles.
// ---------------------------------------------------------------------------
// FP8: an 8-bit float cache (SART_LAYOUT_MFMA16_FP8): half the bytes per tile, expanded
// to bf16 operands in registers.
template <int D, bool FP8>
__global__ void __launch_bounds__(kAttnThreads)
k_attn_mfma(Ctx c, DecodeArgs a, const int* __restrict__ bt0, const int* __restrict__ bt1,
            const int* __restrict__ prefix_table, const int* __restrict__ wave_desc, const int* __restrict__ row_desc) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  constexpr int KQ = D / 32;                       // 16-byte bf16 chunks per lane per tile
  constexpr int KR = raw_chunks<D, FP8>();         // 16-byte chunks per lane per tile as stored
  constexpr int kRing = 4;                         // pages in flight per wave while streaming (3, 5 and 6 take the same time,
                                                   // measured; 8 on 8-bit float caches is slower)
  constexpr int kTileBytes = 16 * D * (FP8 ? 1 : 2);   // one K (or V) tile
  constexpr int kPageBytes = 2 * kTileBytes;       // K tile + V tile of one kv head

  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nA = scal[S_D_NA];
  if (a.n_rows < scal[S_NACTIVE] || scal[S_D_NWG] != (int)gridDim.x || slots_needed(scal, dm.Hkv) > a.partial_cap) {
    // a row buffer smaller than the active list, a launch that does not match the plan, or a scratch
    // buffer too small for the plan's partial results
    if (blockIdx.x == 0 && threadIdx.x == 0) record_error(scal, SART_E_INVALID, a.call_seq);
    return;
  }
  const long long S = (long long)nA * dm.Hkv;
  const int n_waves = gridDim.x * kAttnWaves;
  const long long prompt_slot_base = (long long)scal[S_D_NOWN] + S;
  const uint16_t* q = (const uint16_t*)a.q;
  const unsigned char* pool = (const unsigned char*)c.pool;
  const int* __restrict__ bt = scal[S_BTSEL] ? bt1 : bt0;
  WaveState<D> st;
  uint4 qreg[KQ];

  {
    // ---- this wave's prompt work items and its range of the own line; one partial result per piece -------
    const Cut cut = load_cut(scal);
    const int prompt_mode = scal[S_D_PMODE];             // how the plan had this step's prompts read
    const long long wave_id = (long long)blockIdx.x * kAttnWaves + wv;
    // where the wave starts, resolved by the planning kernel: one load instead of a chain of lookups
    const int4 wd0 = ((const int4*)(wave_desc + 16LL * wave_id))[0];
    const int4 wd2 = ((const int4*)(wave_desc + 16LL * wave_id))[2];
    const int4 wd3 = ((const int4*)(wave_desc + 16LL * wave_id))[3];
    const long long page_bytes = dm.page_elems * (FP8 ? 1 : 2);
    // Streams pages [r0, r0 + rn) of `table` (kv head h) through kRing register
    // buffers in a software pipeline: kRing pages (8 KiB each) are in flight per
    // wave.  The steady-state loop and its preheader have no conditional loads,
    // so the compiler can wait for the oldest buffer only (s_waitcnt
    // vmcnt(8*kRing-1 ...)) while the newer pages are still in flight; page ids
    // are wave-uniform scalar reads of the table.  full(k, v): a page of 16
    // valid tokens; part(k, v, nv): a page that may hold fewer (the last one).
    // once: a branch's own pages are read once per step, so their loads carry the non-temporal hint (measured
    // on plain reads of 8 KiB chunks: 6.7 against 6.0 TB/s); prompt pages are read again by the request's
    // other row tiles and stay ordinary loads that the L2 keeps.
    auto stream_pages = [&](auto once, const int* __restrict__ table, int r0, int rn, int n_last, int h, auto&& full, auto&& part) {
      const long long head_off = (long long)h * kPageBytes + lane * 16;
      auto load_page = [&](uint4* kq, uint4* vq, int pid) {
        const unsigned char* base = pool + (long long)pid * page_bytes + head_off;
#pragma unroll
        for (int i = 0; i < KR; ++i) {
          if constexpr (decltype(once)::value) {
            kq[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(base + i * 1024)));
            vq[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4*)(base + kTileBytes + i * 1024)));
          } else {
            kq[i] = *(const uint4*)(base + i * 1024);
            vq[i] = *(const uint4*)(base + kTileBytes + i * 1024);
          }
        }
      };
      uint4 kb[kRing][KR], vb[kRing][KR];
      int i = 0;
      if (rn >= 2 * kRing) {
#pragma unroll
        for (int j = 0; j < kRing; ++j) load_page(kb[j], vb[j], table[r0 + j]);
        do {   // at the top: buffer j holds page i+j (all full pages), i + 2*kRing <= rn
          int pid[kRing];
#pragma unroll
          for (int j = 0; j < kRing; ++j) pid[j] = table[r0 + i + kRing + j];
#pragma unroll
          for (int j = 0; j < kRing; ++j) {
            full(kb[j], vb[j]);
            load_page(kb[j], vb[j], pid[j]);
          }
          i += kRing;
        } while (i + 2 * kRing <= rn);
#pragma unroll
        for (int j = 0; j < kRing; ++j) part(kb[j], vb[j], i + j == rn - 1 ? n_last : 16);
        i += kRing;
      }
      while (i < rn) {   // fewer than 2*kRing pages left: groups of up to kRing, requested up front
        const int cnt = min(kRing, rn - i);
#pragma unroll
        for (int j = 0; j < kRing; ++j)
          if (j < cnt) load_page(kb[j], vb[j], table[r0 + i + j]);
#pragma unroll
        for (int j = 0; j < kRing; ++j)
          if (j < cnt) part(kb[j], vb[j], i + j == rn - 1 ? n_last : 16);
        i += cnt;
      }
    };

    // One piece: pages [r0, r0 + rn) of `table` for the G query heads of (row, kv head h); its partial
    // result goes to `slot` (or, merged, to the output).  `table` is passed down from a kernel argument in
    // every call, so that the page ids stay scalar loads in each instance of the streaming loop.
    auto run_piece = [&](auto once, const int* __restrict__ table, int row, int h, int r0, int rn, int n_last, long long slot,
                         const RowInfo& ri) {
      load_q<D>(qreg, q, dm, io_row(a, ri, row), h);
      st.reset();
      stream_pages(once, table, r0, rn, n_last, h,
                   [&](const uint4* kq, const uint4* vq) { process_raw<D, FP8, true>(st, kq, vq, qreg, 16, 16, a.scale_log2); },
                   [&](const uint4* kq, const uint4* vq, int nv) { process_raw<D, FP8, false>(st, kq, vq, qreg, nv, nv, a.scale_log2); });
      if (a.fused_merge) finish_piece<D>(a, dm, cut, prompt_slot_base, st, slot, row, h, ri);
      else store_partial<D, false>(st, a.partials, slot, dm);
    };

    // The wave's prompt work and its own range are two parts; which comes first alternates between groups of 8
    // workgroups (one per XCD): while one half of the waves is in its prompt part, which is bound by latency
    // (a few pages, mostly L2 hits), the other half keeps HBM busy, and at the end of the kernel the same
    // the other way round.  The waves of a workgroup take the same order, so the row tiles of a chunk, which
    // they serve, still read it at the same time.
    const bool prompt_part_first = !a.stagger_prompt || ((blockIdx.x >> 3) & 1) == 0;
    for (int turn = 0; turn < 2; ++turn) {
      if ((turn == 0) == prompt_part_first) {
        // ---- shared-rows prompt mode: a work item is (request, kv head, chunk of pb prompt pages, tile of up
        //      to 16 * kSharedBlocks query rows); its pages are read once and every page feeds the tile's
        //      blocks (rows = (branch, head of the group), branch-major).  One partial per (branch, kv head,
        //      chunk), in the slots the per-branch blocks would have used. -------------------------------
        if (prompt_mode == 2 && wave_id >= n_waves - cut.n_prompt) {
          const int r16 = lane & 15, g4 = lane >> 4;
          const long long pf = partial_floats(dm.G, D);
          int cursor = wd3.z;
          bool resolved = wd3.w != 0;                                  // the first item's request came with the descriptor
          for (long long item = prompt_range_of_wave(wave_id - (n_waves - cut.n_prompt), cut.n_prompt); item < cut.n_pitems;
               item += cut.n_prompt) {
            int r = wd2.x, cnt = wd2.y, plen = wd2.z, first_row = wd2.w, pstart = wd3.x, istart = wd3.y;
            if (!resolved) {                                           // rare: more items than waves
              while (item >= tb.live_item_start[cursor + 1]) ++cursor; // the live request owning the item
              r = tb.live_req[cursor];
              cnt = tb.nact[r]; plen = tb.prefix_len[r]; first_row = tb.req_first[r]; pstart = tb.req_pstart[r];
              istart = tb.live_item_start[cursor];
            }
            resolved = false;
            const int pp = ceil_div(plen, 16), nck = ceil_div(pp, cut.pb);
            const int rows = cnt * dm.G, ntile = ceil_div(rows, 16 * kSharedBlocks);
            const int local = (int)(item - istart);
            const int rt = local % ntile, ck = (local / ntile) % nck, h = local / (ntile * nck);
            const int cs = prompt_chunk_pages(pp, nck), r0 = ck * cs, rn = min(cs, pp - r0);
            const int n_last = min(16, plen - (r0 + rn - 1) * 16);
            const int row0 = rt * 16 * kSharedBlocks;
            const int nb = min(kSharedBlocks, ceil_div(rows - row0, 16));          // blocks with rows (wave-uniform)
            WaveState<D> sb[kSharedBlocks];
            uint4 qb[kSharedBlocks][KQ];
            int br[kSharedBlocks], hd[kSharedBlocks];                              // this lane's branch and head per block, -1: no row
    #pragma unroll
            for (int b = 0; b < kSharedBlocks; ++b) {
              const int flat = row0 + 16 * b + r16;
              const bool have = flat < rows;
              const int fc = have ? flat : rows - 1;                               // lanes past the end shadow the last row
              const int j = fc / dm.G, g = fc % dm.G;
              br[b] = have ? j : -1;
              hd[b] = g;
              const uint16_t* qrow = q + ((long long)io_row(a, row_desc, first_row + j) * dm.Hq + h * dm.G + g) * D;
    #pragma unroll
              for (int i = 0; i < KQ; ++i) qb[b][i] = *(const uint4*)(qrow + i * 32 + g4 * 8);
              sb[b].reset();
            }
            stream_pages(std::false_type{}, prefix_table + (long long)r * dm.max_pp, r0, rn, n_last, h,
                         [&](const uint4* kq, const uint4* vq) {
    #pragma unroll
                           for (int b = 0; b < kSharedBlocks; ++b)
                             if (b < nb) process_raw<D, FP8, true>(sb[b], kq, vq, qb[b], 16, 16, a.scale_log2);
                         },
                         [&](const uint4* kq, const uint4* vq, int nv) {
    #pragma unroll
                           for (int b = 0; b < kSharedBlocks; ++b)
                             if (b < nb) process_raw<D, FP8, false>(sb[b], kq, vq, qb[b], nv, nv, a.scale_log2);
                         });
            const long long slot0 = prompt_slot_base + pstart + ((long long)h * nck + ck) * cnt;
    #pragma unroll
            for (int b = 0; b < kSharedBlocks; ++b) {
              if (b >= nb) continue;
              const float l = sum_over_rows(sb[b].l);
              if (br[b] < 0) continue;
              float* base = a.partials + (slot0 + br[b]) * pf;
              if (a.fused_merge) {
    #pragma unroll
                for (int k = 0; k < D / 16; ++k) put_f32x4<true>(base + (long long)hd[b] * D + k * 16 + 4 * g4, sb[b].o[k]);
                if (g4 == 0) {
                  put_f32<true>(base + (long long)dm.G * D + hd[b], sb[b].m);
                  put_f32<true>(base + (long long)dm.G * D + dm.G + hd[b], l);
                }
              } else {
    #pragma unroll
                for (int k = 0; k < D / 16; ++k) put_f32x4<false>(base + (long long)hd[b] * D + k * 16 + 4 * g4, sb[b].o[k]);
                if (g4 == 0) {
                  put_f32<false>(base + (long long)dm.G * D + hd[b], sb[b].m);
                  put_f32<false>(base + (long long)dm.G * D + dm.G + hd[b], l);
                }
              }
            }
            if (a.fused_merge) {
              // one lane per branch of the tile (the one holding the branch's first row in the tile) counts the
              // tile in for (branch, kv head); the branches completed by that are merged by the whole wave in turn
              static_assert(kSharedBlocks == 1, "the in-kernel merge expects one 16-row block per prompt item");
              __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // the tile's partial results have been stored
              __builtin_amdgcn_s_waitcnt(0);
              bool last = false;
              const int j = br[0], flat = row0 + r16;
              if (j >= 0 && g4 == 0 && flat == max(row0, j * dm.G)) {
                const RowInfo ri = load_row_info(row_desc, first_row + j);
                long long w0;
                int sn;
                own_pieces(cut, dm.Hkv, ri, h, w0, sn);
                const int old = __hip_atomic_fetch_add(a.seg_count + ((long long)(first_row + j) * dm.Hkv + h), 1, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                last = old == ri.prompt_writers + sn - 1;
              }
              unsigned long long done = __ballot(last);
              if (done) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                while (done) {
                  const int ln = __builtin_ctzll(done);
                  done &= done - 1;
                  const int row = first_row + __builtin_amdgcn_readlane(j, ln);
                  const RowInfo ri = load_row_info(row_desc, row);
                  long long w0;
                  int sn;
                  own_pieces(cut, dm.Hkv, ri, h, w0, sn);
                  if (lane == 0) __hip_atomic_store(a.seg_count + ((long long)row * dm.Hkv + h), 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  fold_segment<D>(a, dm, prompt_slot_base, row, h, ri, w0, sn);
                }
              }
            }
          }
        }

        // ---- per-branch prompt blocks (prompt mode 1): block u is (request, kv head, chunk, branch); served before
        //      the own range, all waves at the same time, so that the branches' re-reads of a chunk hit in L2 -----
        if (prompt_mode == 1 && wave_id >= n_waves - cut.n_prompt) {
          const long long i = wave_id - (n_waves - cut.n_prompt);
          int cursor = tb.wave_row[n_waves + i];                       // live request index
          for (long long u = prompt_range_of_wave(i, cut.n_prompt); u < cut.n_blocks; u += cut.n_prompt) {
            while (u >= tb.live_item_start[cursor + 1]) ++cursor;      // the live request owning block u
            const int r = tb.live_req[cursor];
            const int cnt = tb.nact[r], plen = tb.prefix_len[r];
            const int pp = ceil_div(plen, 16), nck = ceil_div(pp, cut.pb);
            const int local = (int)(u - tb.live_item_start[cursor]);
            const int j = local % cnt, ck = (local / cnt) % nck, h = local / (cnt * nck);
            const int cs = prompt_chunk_pages(pp, nck), r0 = ck * cs, rn = min(cs, pp - r0);
            const int row = tb.req_first[r] + j;
            RowInfo ri{};
            if (a.fused_merge || a.by_handle) ri = load_row_info(row_desc, row);
            run_piece(std::false_type{}, prefix_table + (long long)r * dm.max_pp, row, h, r0, rn, min(16, plen - (r0 + rn - 1) * 16),
                      prompt_slot_base + u, ri);
          }
        }

      } else {
        // ---- own line: this wave's range [u, u1) of the (row, kv head, page) units, one piece per (row, kv head) it
        //      crosses; piece of range x for (row, h) goes to slot x + row * Hkv + h ---------------------------------
        if (wave_id < cut.n_own) {
          const long long x = wave_id, u1 = own_end(cut, x);
          long long u = own_start(cut, x);
          int cursor = wd0.x, c_cum = wd0.y, c_pages = wd0.z, c_seq = wd0.w;   // active row, its page_cum, private pages, tokens
          RowInfo ri{};
          if (u < u1) ri = load_row_info(row_desc, cursor);          // the merge's facts about the row: needed when a piece ends
          while (u < u1) {
            long long rem = u - (long long)c_cum * dm.Hkv;
            while (c_pages == 0 || rem >= (long long)c_pages * dm.Hkv) {   // next row (skipping rows without private pages)
              ++cursor;
              ri = load_row_info(row_desc, cursor);
              c_cum = ri.cum;
              c_pages = ri.pages;
              c_seq = ri.seq;
              rem = u - (long long)c_cum * dm.Hkv;
            }
            const int row = cursor, h = (int)(rem / c_pages), r0 = (int)(rem % c_pages);
            const int rn = (int)min((long long)(c_pages - r0), u1 - u);
            run_piece(std::true_type{}, bt + (long long)row * dm.max_bp, row, h, r0, rn, min(16, c_seq - (r0 + rn - 1) * 16),
                      x + (long long)row * dm.Hkv + h, ri);
            u += rn;
          }
        }
      }
    }
    // (row, kv head) pairs without any context have no writer: their output rows are zero
    if (a.fused_merge && wv == 0) {
      for (long long seg = blockIdx.x; seg < S; seg += gridDim.x) {
        const int row = (int)(seg / dm.Hkv), h = (int)(seg % dm.Hkv);
        const RowInfo ri = load_row_info(row_desc, row);
        if (ri.pages != 0 || ri.prompt_writers != 0) continue;
        for (int e = lane; e < dm.G * (D / 4); e += 64)
          *(f32x4*)(a.out + ((long long)io_row(a, ri, row) * dm.Hq + h * dm.G) * D + 4LL * e) = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Generic kernel (any dtype, SART_LAYOUT_NATURAL, any page size and head dim
// <= 256): same unit line and partial format; one wave per range; the prompt
// is read inline as the first pages of every row.  Used for fp32 caches and
// for shapes the matrix-core tile does not cover; not a tuned path.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kAttnThreads)
k_attn_generic(Ctx c, DecodeArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  if (a.n_rows < scal[S_NACTIVE] || scal[S_D_NWG] != (int)gridDim.x || slots_needed(scal, dm.Hkv) > a.partial_cap) {
    if (blockIdx.x == 0 && threadIdx.x == 0) record_error(scal, SART_E_INVALID, a.call_seq);
    return;
  }
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int* bt = tb.bt[scal[S_BTSEL]];
  const T* pool = (const T*)c.pool;
  const T* q = (const T*)a.q;
  const int D = dm.d, pt = dm.pt;
  const Cut cut = load_cut(scal);
  const int n_waves = gridDim.x * kAttnWaves;
  const long long S = (long long)scal[S_D_NA] * dm.Hkv;
  const long long prompt_slot_base = (long long)cut.n_own + S;
  const long long wave_id = (long long)blockIdx.x * kAttnWaves + wv;
  for (int line = 1; line >= 0; --line) {   // prompt blocks first, as in the matrix-core kernel
    long long x, u, u1;
    int cursor;
    if (line == 0) {
      if (wave_id >= cut.n_own) continue;
      x = wave_id; u = own_start(cut, x); u1 = own_end(cut, x);
      if (u >= u1) continue;
      cursor = tb.wave_row[x];
    } else {
      if (wave_id < n_waves - cut.n_prompt) continue;
      const long long i = wave_id - (n_waves - cut.n_prompt);
      x = 0; u = prompt_range_of_wave(i, cut.n_prompt); u1 = cut.n_blocks;   // u counts prompt blocks here
      if (u >= u1) continue;
      cursor = tb.wave_row[n_waves + i];
    }
    while (u < u1) {
      int row, h, r0, rn, tokens;
      long long slot;
      const int* table;
      if (line == 0) {
        int pages = tb.page_cum[cursor + 1] - tb.page_cum[cursor];
        long long rem = u - (long long)tb.page_cum[cursor] * dm.Hkv;
        while (pages == 0 || rem >= (long long)pages * dm.Hkv) {
          ++cursor;
          pages = tb.page_cum[cursor + 1] - tb.page_cum[cursor];
          rem = u - (long long)tb.page_cum[cursor] * dm.Hkv;
        }
        row = cursor;
        h = (int)(rem / pages);
        r0 = (int)(rem % pages);
        rn = (int)min((long long)(pages - r0), u1 - u);
        tokens = tb.seq_len[row];
        table = bt + (long long)row * dm.max_bp;
        slot = x + (long long)row * dm.Hkv + h;
      } else {
        while (u >= tb.live_item_start[cursor + 1]) ++cursor;
        const int r = tb.live_req[cursor];
        const int cnt = tb.nact[r];
        tokens = tb.prefix_len[r];
        const int pp = ceil_div(tokens, pt), nck = ceil_div(pp, cut.pb);
        const int local = (int)(u - tb.live_item_start[cursor]);
        const int j = local % cnt, ck = (local / cnt) % nck;
        h = local / (cnt * nck);
        const int cs = prompt_chunk_pages(pp, nck);
        r0 = ck * cs;
        rn = min(cs, pp - r0);
        row = tb.req_first[r] + j;
        table = tb.prefix_table + (long long)r * dm.max_pp;
        slot = prompt_slot_base + u;
      }
      float* pbase = a.partials + slot * partial_floats(dm.G, D);
      for (int r = 0; r < dm.G; ++r) {
        const T* qrow = q + ((long long)io_row(a, tb.row_desc, row) * dm.Hq + h * dm.G + r) * D;
        float m = -__builtin_inff(), l = 0.f;
        float o[4] = {0.f, 0.f, 0.f, 0.f};   // d = lane + 64*c
        generic_row<T>(dm, pool, table, r0, rn, tokens, h, qrow, a.scale_log2, m, l, o);
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
      u += line == 0 ? rn : cut.n_prompt;
    }
  }
}

// ---------------------------------------------------------------------------
// A6: merge.  One workgroup per (active row, kv head); each thread owns four
// consecutive output columns of one query head and folds the partials of that
// head in slot order (prompt chunks, then private pieces) with the running
// form of  m = max m_i,  l = sum l_i 2^(m_i - m),  out = sum o_i 2^(m_i - m) / l.
// The loads of successive partials are independent, so they overlap.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_merge(Ctx c, DecodeArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (a.n_rows < scal[S_NACTIVE] || scal[S_D_NWG] != a.n_wg || slots_needed(scal, dm.Hkv) > a.partial_cap) return;
  const int nA = scal[S_D_NA];
  const Cut cut = load_cut(scal);
  const int D = dm.d, G = dm.G, D4 = D >> 2;
  const long long pf = partial_floats(G, D);
  const long long S = (long long)nA * dm.Hkv;
  const long long prompt_slot_base = (long long)cut.n_own + S;
  for (long long seg = blockIdx.x; seg < S; seg += gridDim.x) {
    const int row = (int)(seg / dm.Hkv), h = (int)(seg % dm.Hkv);
    // slot ranges: [pa, pa + pn * pstride) prompt pieces (one block per prompt chunk: first slot of the row +
    // (head * chunks + chunk) * branches), [sa, sa + sn) own pieces; the row's facts come from the plan's
    // descriptor (one load), so that the partial results can be requested right after it
    const RowInfo ri = load_row_info(tb.row_desc, row);
    const int pn = ri.nck;
    const long long pstride = ri.cnt, pa = prompt_slot_base + ri.pslot + (long long)h * ri.nck * ri.cnt;
    long long sa, w0;
    int sn;
    own_pieces(cut, dm.Hkv, ri, h, w0, sn);
    sa = w0 + seg;
    for (int e = threadIdx.x; e < G * D4; e += blockDim.x) {
      const int r = e / D4, d4 = e % D4;
      fold_columns<false>(a.partials, a.out + ((long long)io_row(a, ri, row) * dm.Hq + h * G + r) * D, pf, G, D, r, d4, pa, pstride, pn, sa, sn,
                          a.v_scale);
    }
  }
}

void launch_decode(const Ctx& c, const DecodeArgs& a_in, hipStream_t s) {
  const Dims& dm = c.dm;
  const bool mfma = dm.layout != SART_LAYOUT_NATURAL;
  DecodeArgs a = a_in;
  // the matrix-core kernel can merge in its own last writers; the generic kernel always leaves its partial
  // results to the merge kernel
  a.fused_merge = a_in.fused_merge && mfma;
  if (a.ev[0]) (void)hipEventRecord(a.ev[0], s);
  if (a.ev[1]) (void)hipEventRecord(a.ev[1], s);
  // profiling with repeats > 1 launches the (idempotent) attention kernel that many times
  // back to back between the two events, so their dispatch overhead is amortised
  for (int rep = 0; rep < (a.repeats > 1 ? a.repeats : 1); ++rep) {
  if (mfma) {
    auto go = [&](auto kern) {
      hipLaunchKernelGGL(kern, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a, c.tb.bt[0], c.tb.bt[1],
                         c.tb.prefix_table, c.tb.wave_desc, c.tb.row_desc);
    };
    const bool fp8 = dm.layout == SART_LAYOUT_MFMA16_FP8;
    if (dm.d == 128) { if (fp8) go(k_attn_mfma<128, true>); else go(k_attn_mfma<128, false>); }
    else { if (fp8) go(k_attn_mfma<64, true>); else go(k_attn_mfma<64, false>); }
  } else if (dm.dtype == SART_F32) {
    hipLaunchKernelGGL(k_attn_generic<float>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
  } else {
    hipLaunchKernelGGL(k_attn_generic<uint16_t>, dim3(a.n_wg), dim3(kAttnThreads), 0, s, c, a);
  }
  }
  if (a.ev[2]) (void)hipEventRecord(a.ev[2], s);
  if (!a.fused_merge) {
    long long blocks = (long long)dm.H * dm.Hkv;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_merge, dim3((unsigned)blocks), dim3(256), 0, s, c, a);
  }
  if (a.ev[3]) (void)hipEventRecord(a.ev[3], s);
}


// ---------------------------------------------------------------------------
// Scratch of sart_decode_attention_static: the partial results live in this
// array instead of the cache's own allocation.  Every GPU the library runs on
// holds its own copy at its own address (until the process ends); the array's
// name is only a host-side stand-in, so host code asks the runtime once per
// device, with that device current, where the copy is and uses that address
// from then on.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t static_scratch(int* device, void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // the current device's copy
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *device = dev;
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace sart
