// Device-side helpers shared by the planning kernels: block scans, the sticky
// error word, and the decode plan (the partition of one decode step's work),
// which every state-changing planning kernel refreshes before it ends so that
// sart_decode_attention needs no planning launch of its own.
#pragma once

#include "sart_internal.h"

namespace sart {

__device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

__device__ inline int wave_incl_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int n = __shfl_up(v, off, 64);
    if (lane >= off) v += n;
  }
  return v;
}

// Exclusive prefix of v over the workgroup (up to 1024 threads) and the total.
// lds holds 17 ints.  Every thread of the workgroup must call it.
__device__ inline int block_excl_scan(int v, int* lds, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = (blockDim.x + 63) >> 6;
  const int incl = wave_incl_scan(v);
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    const int t = lane < nw ? lds[lane] : 0;
    const int ti = wave_incl_scan(t);
    if (lane < nw) lds[lane] = ti - t;
    if (lane == nw - 1) lds[16] = ti;
  }
  __syncthreads();
  total = lds[16];
  return incl - v + lds[wave];
}

// Three exclusive scans at once (same barriers as one).  lds holds 3*17 ints.
__device__ inline void block_excl_scan3(int v0, int v1, int v2, int* lds, int* ex, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = (blockDim.x + 63) >> 6;
  const int v[3] = {v0, v1, v2};
  int incl[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) incl[k] = wave_incl_scan(v[k]);
  __syncthreads();
  if (lane == 63) {
#pragma unroll
    for (int k = 0; k < 3; ++k) lds[17 * k + wave] = incl[k];
  }
  __syncthreads();
  if (wave < 3) {
    const int t = lane < nw ? lds[17 * wave + lane] : 0;
    const int ti = wave_incl_scan(t);
    if (lane < nw) lds[17 * wave + lane] = ti - t;
    if (lane == nw - 1) lds[17 * wave + 16] = ti;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    total[k] = lds[17 * k + 16];
    ex[k] = incl[k] - v[k] + lds[17 * k + wave];
  }
}

// First error of a call wins and stays until the host reads it.
// The active count as the host may peek at it without waiting for the device: one int in pinned host
// memory, stored (through to the host) by the thread that changes the count.
__device__ inline void publish_active_count(const Tables& tb, int n) {
  __hip_atomic_store(tb.host_nactive, n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ inline void record_error(int* scal, int code, int call_seq) {
  if (scal[S_ERR] == 0) {
    scal[S_ERR] = code;
    scal[S_ERRCALL] = call_seq;
  }
  scal[S_CALLOK] = 0;
}

// ---------------------------------------------------------------------------
// A3: the decode plan (run by one 1024-thread workgroup; ends with a barrier).
//
//   page_cum[a]   exclusive scan over active rows of their private pages; the
//                 own line has page_cum[nA] * Hkv units.
//   prompt blocks blocks of pb pages, pb sized so that the
//                 blocks about fill the prompt waves once; request r owns blocks
//                 req_pstart[r] + ((head * chunks + chunk) * branches + branch);
//                 live_req[k] lists the live requests with a prompt in active
//                 order, live_item_start[k] their first work item (a block, or, with
//                 shared rows, a (request, kv head, chunk, row tile)).
//   cut           see Cut; wave_row[w] = active row holding the first unit of own
//                 range w; wave_row[n_waves + i] = index k of the live request
//                 owning the first work item of wave i.
// ---------------------------------------------------------------------------
constexpr int kPlanLdsRows = 4096;   // active rows whose page_cum and lengths the plan keeps in LDS
constexpr int kPlanLdsLive = 1024;   // live requests whose fields the plan keeps in LDS

// What the plan's first pass reads of the first kPlanThreads rows, for a caller that requested it earlier
// (together with the flags that decide whether it plans at all: one trip to memory instead of three).
struct PlanPre { int nA, b, b_prev, len, pm_choice, pm_a, pm_b, pm_c, ok, deferred; };
__device__ inline PlanPre plan_preload(const Ctx& c) {
  static_assert(S_COUNT <= 64, "the scalar block is read by one wave, a lane per entry");
  const Tables& tb = c.tb;
  const int ti = min((int)threadIdx.x, c.dm.H - 1);          // (rows past the active ones: any entry, unused)
  // the whole scalar block with one load (lane l holds entry l), and this thread's row: four loads in flight
  // together, all waited for here (the compiler would otherwise move each load to its first use, behind
  // the branches on the earlier ones)
  const int sv = tb.scal[min((int)threadIdx.x & 63, (int)S_COUNT - 1)];
  const int b = tb.active[ti], b_prev = tb.active[max(ti - 1, 0)], len = tb.seq_len[ti];
  asm volatile("" ::"v"(sv), "v"(b), "v"(b_prev), "v"(len));
  PlanPre p;
  p.b = b; p.b_prev = b_prev; p.len = len;
  p.nA = __builtin_amdgcn_readlane(sv, S_NACTIVE);
  p.ok = __builtin_amdgcn_readlane(sv, S_CALLOK);
  p.deferred = __builtin_amdgcn_readlane(sv, S_PLAN_DEFERRED);
  p.pm_choice = __builtin_amdgcn_readlane(sv, S_PM_CHOICE);
  p.pm_a = __builtin_amdgcn_readlane(sv, S_PM_SIG_A);
  p.pm_b = __builtin_amdgcn_readlane(sv, S_PM_SIG_B);
  p.pm_c = __builtin_amdgcn_readlane(sv, S_PM_SIG_C);
  return p;
}

template <bool PRE = false>
__device__ inline void refresh_decode_plan(const Ctx& c, const PlanCfg& pc, int* lds, PlanPre pre = PlanPre{}) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  const int tid = threadIdx.x;
  __shared__ int s_scan[3 * 17];
  __shared__ int s_cum[kPlanLdsRows + 1];
  __shared__ int s_seq[kPlanLdsRows];         // tokens of the active rows
  // live requests with a prompt, by live index: request, live branches, prompt tokens, first active
  // row, first partial slot, first work item (searched per wave)
  __shared__ int s_lreq[kPlanLdsLive], s_lcnt[kPlanLdsLive], s_lplen[kPlanLdsLive], s_lfirst[kPlanLdsLive],
      s_lpstart[kPlanLdsLive], s_item[kPlanLdsLive + 1];
  __shared__ int s_w2;                          // prompt pages read with one read per row tile, summed over the live requests
  __shared__ int s_it1, s_it2;                  // work items of the two ways to read the prompts (estimate)
  (void)lds;
  if (tid == 0) { s_w2 = 0; s_it1 = 0; s_it2 = 0; }
  __syncthreads();                       // the caller's table updates are visible
  if (!PRE) { pre.nA = scal[S_NACTIVE]; pre.pm_choice = scal[S_PM_CHOICE]; pre.pm_a = scal[S_PM_SIG_A]; pre.pm_b = scal[S_PM_SIG_B]; pre.pm_c = scal[S_PM_SIG_C]; }
  const int nA = pre.nA;
  // w: weight of a live request with a prompt, on its first row: the prompt pages its work items read when
  // every branch reads them; w2: when every tile of 16 * kSharedBlocks query rows does
  int carry = 0, w_carry = 0, l_carry = 0;
  int my_handle = -1, my_live = -1;      // of active row tid (the first chunk of rows): its branch, the live index its request would have
  for (int base = 0; base < nA; base += kPlanThreads) {
    const int i = base + tid;
    int np = 0, w = 0, first = 0, r = 0, cnt = 0, plen = 0;
    if (i < nA) {
      const bool have = PRE && base == 0;                  // this row's entries came with the preload
      const int b = have ? pre.b : tb.active[i];
      if (base == 0) my_handle = b;
      r = b / dm.Nb;
      first = i == 0 || (have ? pre.b_prev : tb.active[i - 1]) / dm.Nb != r;
      const int len = have ? pre.len : tb.seq_len[i];
      if (i < kPlanLdsRows) s_seq[i] = len;
      np = ceil_div(len, dm.pt);
      if (first) {
        plen = tb.prefix_len[r];
        cnt = tb.nact[r];
        const int pp = ceil_div(plen, dm.pt);
        // pages read for the request's prompt, per kv head: once per branch, or once per tile of
        // 16 * kSharedBlocks query rows (shared rows)
        w = pp * cnt;
        tb.req_first[r] = i;
      }
    }
    int ex3[3], tot3[3];
    block_excl_scan3(np, w, w > 0, s_scan, ex3, tot3);
    if (i < nA) {
      tb.page_cum[i] = carry + ex3[0];
      if (i <= kPlanLdsRows) s_cum[i] = carry + ex3[0];
    }
    if (w > 0) {
      const int k = l_carry + ex3[2];
      tb.live_req[k] = r;
      if (k < kPlanLdsLive) { s_lreq[k] = r; s_lcnt[k] = cnt; s_lplen[k] = plen; s_lfirst[k] = i; }
    }
    // a request's rows are neighbours: the last live request that starts at or before row i is row i's own, if it has a prompt
    if (base == 0) my_live = l_carry + ex3[2] + (w > 0) - 1;
    carry += tot3[0];
    w_carry += tot3[1];
    l_carry += tot3[2];
  }
  if (tid == 0) {
    tb.page_cum[nA] = carry;
    if (nA <= kPlanLdsRows) s_cum[nA] = carry;
  }
  const int n_live = l_carry;
  const int n_waves = pc.n_wg * kAttnWaves;
  Cut cut;
  cut.u_own = (long long)carry * dm.Hkv;
  __syncthreads();
  // How the prompts are read this step (unless the caller fixed it).  Per branch (1): every branch of a
  // request reads every chunk of its prompt, all but the first read hitting in L2.  Per row tile (2): a chunk
  // is read once for 16 query rows of the request's branches: 16 / G branches share a read.  Measured, the
  // prompts' pages are cheap while the other half of the waves streams private pages (L2 hits: about a tenth
  // of a private page's time) and the per-branch form, with its longer items, is the faster one by 3-12 us
  // over a grid of shapes (2-32 branches per request, prompts of 256-2048 tokens, G = 5 and 7) - unless the
  // tiles save a wave about 48 or more prompt pages, or the step has little private work to hide the prompts
  // behind (then every prompt page saved counts).  cost = most prompt pages a wave reads, whole items.
  // sums over the live requests (their fields are in LDS for the first kPlanLdsLive): within the wave first,
  // then one LDS atomic per wave (many lanes adding to one LDS word take tens of cycles each)
  auto live_sums = [&](auto&& term, int* s_a, int* s_b) {
    int a1 = 0, a2 = 0;
    for (int k = tid; k < n_live; k += kPlanThreads) {
      const bool in_lds = k < kPlanLdsLive;
      const int r = in_lds ? s_lreq[k] : tb.live_req[k];
      const int plen = in_lds ? s_lplen[k] : tb.prefix_len[r], cnt = in_lds ? s_lcnt[k] : tb.nact[r];
      term(ceil_div(plen, dm.pt), cnt, a1, a2);
    }
    if (tid < ((n_live + 63) & ~63)) {
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) { a1 += __shfl_xor(a1, off, 64); a2 += __shfl_xor(a2, off, 64); }
      if ((tid & 63) == 0) { atomicAdd(s_a, a1); if (s_b) atomicAdd(s_b, a2); }
    }
    __syncthreads();
  };
  const long long u1 = (long long)w_carry * dm.Hkv;
  auto block_pages = [&](long long u) {
    int pb = u > 0 ? (int)div_nn(u + n_waves - 1, n_waves) : 1;
    return ceil_div(pb < 1 ? 1 : pb, 4) * 4;              // whole rings of page buffers
  };
  int mode = pc.prompt_mode;
  long long u2 = 0;
  // (the estimate is two more passes over the live requests: it is repeated only when what it rests on changed)
  const long long own_per_wave = div_nn(cut.u_own + n_waves - 1, n_waves);
  const int sig_a = nA, sig_b = w_carry;
  const int sig_c = (int)((unsigned)n_live * 64u + (unsigned)(own_per_wave < 48 ? own_per_wave : 48) + (unsigned)pc.n_wg * 1000003u);
  const bool automatic = mode != 1 && mode != 2;
  const bool known = automatic && pre.pm_choice != 0 && pre.pm_a == sig_a && pre.pm_b == sig_b && pre.pm_c == sig_c;
  if (known) mode = pre.pm_choice;
  if (mode != 1 && u1 > 0) {
    live_sums([&](int pp, int cnt, int& a1, int&) { a1 += pp * ceil_div(cnt * dm.G, 16 * kSharedBlocks); }, &s_w2, nullptr);
    u2 = (long long)__builtin_amdgcn_readfirstlane(s_w2) * dm.Hkv;
  }
  if (mode != 1 && mode != 2) {
    mode = 1;
    if (u1 > 0) {
      const int pb1 = block_pages(u1), pb2 = block_pages(u2);
      live_sums([&](int pp, int cnt, int& a1, int& a2) {
        a1 += dm.Hkv * ceil_div(pp, pb1) * cnt;
        a2 += dm.Hkv * ceil_div(pp, pb2) * ceil_div(cnt * dm.G, 16 * kSharedBlocks);
      }, &s_it1, &s_it2);
      const int it1 = __builtin_amdgcn_readfirstlane(s_it1), it2 = __builtin_amdgcn_readfirstlane(s_it2);   // uniform, and known to be so
      const long long cost1 = (long long)ceil_div(it1, n_waves) * pb1, cost2 = (long long)ceil_div(it2, n_waves) * pb2;
      if (cost1 - cost2 >= (own_per_wave < 48 ? own_per_wave : 48)) mode = 2;
    }
  }
  if (automatic && !known && tid == 0) {
    scal[S_PM_CHOICE] = mode; scal[S_PM_SIG_A] = sig_a; scal[S_PM_SIG_B] = sig_b; scal[S_PM_SIG_C] = sig_c;
  }
  const long long u_prompt = mode == 2 ? u2 : u1;           // prompt units of the step
  // every wave serves both its share of the prompt work items and its range of the own line
  cut.n_own = n_waves;
  cut.n_prompt = u_prompt > 0 ? n_waves : 0;
  cut.pb = block_pages(u_prompt);
  cut.n_blocks = 0;
  cut.n_pitems = 0;
  int per_wave = (int)div_nn(cut.u_own + cut.n_own - 1, cut.n_own > 0 ? cut.n_own : 1);
  if (per_wave < 1) per_wave = 1;
  // even / odd workgroups: pe + po = 2 * per_wave, po >= 1; an odd number of
  // own workgroups leaves the last one without a partner, so no skew then
  cut.pe = cut.po = per_wave;
  if (((cut.n_own / kAttnWaves) & 1) == 0) {
    int sk = (int)(((long long)per_wave * pc.skew_permille) / 1000);
    if (sk > per_wave - 1) sk = per_wave - 1;
    if (sk < 1 - per_wave) sk = 1 - per_wave;
    cut.pe = per_wave + sk;
    cut.po = per_wave - sk;
  }
  __syncthreads();                       // live_req, req_first, page_cum, req_pstart written
  {
    // first prompt block (partial slot) and first work item of every live request.  The blocks are the
    // prompts' partial results, one slot each: should there be more than max(4 per wave, one per (row, kv
    // head)), the block size is doubled until they fit (one block per prompt at the latest), so that
    //   n_own + nA * Hkv + max(nA * Hkv, 4 * n_waves)
    // partial slots always hold a decode step (what callers with a fixed scratch size rely on).
    const long long max_blocks = (long long)nA * dm.Hkv > 4LL * n_waves ? (long long)nA * dm.Hkv : 4LL * n_waves;
    int b_carry = 0, i_carry = 0;
    for (;;) {
      b_carry = 0; i_carry = 0;
      for (int base = 0; base < n_live; base += kPlanThreads) {
        const int k = base + tid;
        int blocks = 0, items = 0, r = 0;
        if (k < n_live) {
          const bool in_lds = k < kPlanLdsLive;
          r = in_lds ? s_lreq[k] : tb.live_req[k];
          const int plen = in_lds ? s_lplen[k] : tb.prefix_len[r], cnt = in_lds ? s_lcnt[k] : tb.nact[r];
          const int nck = ceil_div(ceil_div(plen, dm.pt), cut.pb);
          blocks = dm.Hkv * nck * cnt;
          items = mode == 2 ? dm.Hkv * nck * ceil_div(cnt * dm.G, 16 * kSharedBlocks) : blocks;
        }
        int ex3[3], tot3[3];
        block_excl_scan3(blocks, items, 0, s_scan, ex3, tot3);
        const int ex = ex3[0], ex_i = ex3[1], tot = tot3[0], tot_i = tot3[1];
        if (k < n_live) {
          tb.live_item_start[k] = i_carry + ex_i;
          tb.req_pstart[r] = b_carry + ex;
          if (k < kPlanLdsLive) { s_item[k] = i_carry + ex_i; s_lpstart[k] = b_carry + ex; }
        }
        b_carry += tot;
        i_carry += tot_i;
      }
      if (b_carry <= max_blocks || cut.pb >= dm.max_pp) break;     // uniform: the scans' totals
      cut.pb *= 2;
    }
    cut.n_blocks = b_carry;
    cut.n_pitems = i_carry;
    if (tid == 0) {
      tb.live_item_start[n_live] = i_carry;
      if (n_live <= kPlanLdsLive) s_item[n_live] = i_carry;
    }
    __syncthreads();
  }
  // What the pieces of a row need to merge in the attention kernel itself, 8 ints per active row:
  //   [0] page_cum of the row  [1] its private pages  [2] its private tokens
  //   [3] writers of prompt partial results per kv head: chunks x row tiles holding the branch's rows
  //       (shared rows), chunks (per-branch blocks), 0 without a prompt
  //   [4] first prompt partial slot of the row, relative to the prompts' slots: chunk ck of kv head h is
  //       slot [4] + (h * [6] + ck) * [5]   [5] live branches of the request   [6] prompt chunks   [7] the branch's handle
  for (int i = tid; i < nA; i += kPlanThreads) {
    int handle, r, j, cnt, pp, pstart;
    if (i == tid && my_live < kPlanLdsLive) {
      // the first chunk of rows, from registers and the LDS copies: no dependent trips to memory
      handle = my_handle; r = handle / dm.Nb;
      const bool live = my_live >= 0 && s_lreq[my_live] == r;
      j = live ? i - s_lfirst[my_live] : 0;
      cnt = live ? s_lcnt[my_live] : 0;
      pp = live ? ceil_div(s_lplen[my_live], dm.pt) : 0;
      pstart = live ? s_lpstart[my_live] : 0;
    } else {
      handle = tb.active[i]; r = handle / dm.Nb;
      j = i - tb.req_first[r]; cnt = tb.nact[r];
      pp = ceil_div(tb.prefix_len[r], dm.pt);
      pstart = tb.req_pstart[r];
    }
    const int nck = pp > 0 ? ceil_div(pp, cut.pb) : 0;
    const int tiles = mode == 2 ? ((j + 1) * dm.G - 1) / (16 * kSharedBlocks) - (j * dm.G) / (16 * kSharedBlocks) + 1 : 1;
    const int c0 = nA <= kPlanLdsRows ? s_cum[i] : tb.page_cum[i], c1 = nA <= kPlanLdsRows ? s_cum[i + 1] : tb.page_cum[i + 1];
    int4* rd = (int4*)(tb.row_desc + 8LL * i);
    rd[0] = make_int4(c0, c1 - c0, i < kPlanLdsRows ? s_seq[i] : tb.seq_len[i], nck * tiles);
    rd[1] = make_int4(nck ? pstart + j : 0, cnt, nck, handle);
  }
  // Where every wave starts.  wave_row (generic kernel): active row of an own
  // range's first unit and, after those entries, the live request of a prompt
  // wave's first work item.  wave_desc (matrix-core kernel), 16 ints per wave,
  // holds what the wave would otherwise look up through a chain of dependent
  // loads before its first tile load:
  //   [0..3]   own range: active row of its first unit, page_cum of that row,
  //            private pages of the row, tokens of the row
  //   [8..15]  first prompt item: request, its live branches,
  //            prompt tokens, first active row, first partial slot of the
  //            request, first work item of the request, live request index,
  //            1 if the wave has an item
  for (int w = tid; w < n_waves; w += kPlanThreads) {
    int v = 0;
    int4 d0 = make_int4(0, 0, 0, 0), d2 = d0, d3 = d0;
    if (w < cut.n_own) {
      const long long u = own_start(cut, w);
      if (u < cut.u_own) {
        const int* cum = nA <= kPlanLdsRows ? s_cum : tb.page_cum;   // uniform choice
        int lo = 0, hi = nA - 1;
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if ((long long)cum[mid] * dm.Hkv <= u) lo = mid; else hi = mid - 1;
        }
        v = lo;
        d0 = make_int4(lo, cum[lo], cum[lo + 1] - cum[lo], lo < kPlanLdsRows ? s_seq[lo] : tb.seq_len[lo]);
      }
      tb.wave_row[w] = v;
    }
    if (w >= n_waves - cut.n_prompt) {
      const int i = w - (n_waves - cut.n_prompt);
      const long long b = prompt_range_of_wave(i, cut.n_prompt);
      int k = 0;
      if (b < cut.n_pitems) {
        const bool in_lds = n_live <= kPlanLdsLive;                              // uniform choice
        const int* its = in_lds ? s_item : tb.live_item_start;
        int lo = 0, hi = n_live - 1;
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (its[mid] <= b) lo = mid; else hi = mid - 1;
        }
        k = lo;
        if (in_lds) {
          d2 = make_int4(s_lreq[k], s_lcnt[k], s_lplen[k], s_lfirst[k]);
          d3 = make_int4(s_lpstart[k], its[k], k, 1);
        } else {
          const int r = tb.live_req[k];
          d2 = make_int4(r, tb.nact[r], tb.prefix_len[r], tb.req_first[r]);
          d3 = make_int4(tb.req_pstart[r], its[k], k, 1);
        }
      }
      tb.wave_row[n_waves + i] = k;
    }
    int4* wd = (int4*)(tb.wave_desc + 16LL * w);
    wd[0] = d0; wd[2] = d2; wd[3] = d3;
  }
  if (tid == 0) {
    scal[S_D_NA] = nA;
    scal[S_D_PER_EVEN] = cut.pe;
    scal[S_D_PER_ODD] = cut.po;
    scal[S_D_UOWN] = (int)cut.u_own;
    scal[S_D_NOWN] = cut.n_own;
    scal[S_D_NPROMPT] = cut.n_prompt;
    scal[S_D_PB] = cut.pb;
    scal[S_D_NBLOCKS] = cut.n_blocks;
    scal[S_D_NPITEMS] = cut.n_pitems;
    scal[S_D_PMODE] = mode;
    scal[S_D_NLIVE] = n_live;
    scal[S_D_NWG] = pc.n_wg;
  }
  __syncthreads();
}

// The cut of the current plan, as the attention and merge kernels read it.
__device__ inline Cut load_cut(const int* scal) {
  Cut k;
  k.pe = scal[S_D_PER_EVEN]; k.po = scal[S_D_PER_ODD]; k.u_own = scal[S_D_UOWN]; k.n_own = scal[S_D_NOWN];
  k.n_prompt = scal[S_D_NPROMPT]; k.pb = scal[S_D_PB]; k.n_blocks = scal[S_D_NBLOCKS]; k.n_pitems = scal[S_D_NPITEMS];
  return k;
}

}  // namespace sart
