// Cache bookkeeping kernels: table initialisation, token append, and the
// terminate pass shared by pruning and completion / early stop.
//
// The paper (arXiv 2505.13326) states the rules these kernels implement:
// Algorithm 1 (Prefill creates a request's Nb branches; Decode removes
// completed branches, applies the prune predicate, tests for termination),
// Section 3 Solution 1 (early stop once Q branches complete) and Section 4
// (shared prefix KV, immediate release of a leaving branch's KV, prefix
// released with the request's last branch).
//
// Every planning kernel is ONE workgroup of 1024 threads: the integer state
// is a few thousand entries, and a single workgroup makes the order of every
// pop and push a plain prefix sum, hence reproducible bit for bit.  The bulk
// work (KV rows, block-table rows, free-stack pushes) is done by wide
// kernels that read the plan.
#include "sart_device.h"

namespace sart {

// ---------------------------------------------------------------------------
// A0: initial tables
// ---------------------------------------------------------------------------
__global__ void k_init_tables(Ctx c, const int* free_order) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long nth = (long long)gridDim.x * blockDim.x;
  // page free_order[0] is popped first, so it sits on top of the stack
  for (long long i = tid; i < dm.num_pages; i += nth) {
    int j = dm.num_pages - 1 - (int)i;
    tb.free_stack[i] = free_order ? free_order[j] : j;
  }
  for (long long i = tid; i < dm.max_req; i += nth) {
    tb.req_used[i] = 0; tb.prefix_len[i] = 0; tb.refcnt[i] = 0; tb.nact[i] = 0; tb.req_tmp[i] = 0; tb.num_completed[i] = 0;
    tb.num_pruned[i] = 0; tb.branch_appended[i] = 0; tb.req_first[i] = 0; tb.req_push_off[i] = -1;
    tb.req_touched[i] = 0;
  }
  for (long long i = tid; i < (long long)dm.max_req * dm.max_pp; i += nth) tb.prefix_table[i] = -1;
  for (long long i = tid; i < dm.H; i += nth) {
    tb.br_state[i] = SART_BRANCH_UNUSED; tb.active_idx_of[i] = -1; tb.active[i] = -1; tb.seq_len[i] = 0;
  }
  for (long long i = tid; i < (long long)dm.H * dm.max_bp; i += nth) { tb.bt[0][i] = -1; tb.bt[1][i] = -1; }
  if (tid < S_COUNT) tb.scal[tid] = tid == S_FREETOP ? dm.num_pages : (tid == S_CALLOK ? 1 : 0);
}

void launch_init_tables(const Ctx& c, const int* free_order_dev, hipStream_t s) {
  hipLaunchKernelGGL(k_init_tables, dim3(1024), dim3(256), 0, s, c, free_order_dev);
}

// ---------------------------------------------------------------------------
// A1/A2: append plan.  Validates the whole list, pops pages by prefix sum,
// creates requests, updates lengths.  Sequence i takes
// free_stack[top-1-(off_i+k)] as its k-th new page: exactly the pages a
// sequential pop loop in list order would hand out.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_append_plan(Ctx c, PlanCfg pc, AppendArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  __shared__ int lds[17];
  __shared__ int s_err;     // (list index << 2) | status of the first failing sequence
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  const int top = scal[S_FREETOP];
  if (tid == 0) { s_err = 0x7fffffff; scal[S_APPENDOK] = 0; scal[S_PLAN_DEFERRED] = 0; }
  __syncthreads();
  if (!a.ids && a.n_seqs >= 0 && a.n_seqs != nA) {
    if (tid == 0) record_error(scal, SART_E_INVALID, a.call_seq);
    return;
  }
  if (a.n_seqs < 0) {                     // "all active branches, however many there are now"; -n_seqs rows given
    if (nA > -a.n_seqs) {
      if (tid == 0) record_error(scal, SART_E_INVALID, a.call_seq);
      return;
    }
    a.n_seqs = nA;
  }
  // The decode step's append - one token for every active row, at most one chunk of rows - in one pass:
  // row i is sequence i, so nothing needs to be stashed and looked up again.
  if (a.kind == SART_SEQ_BRANCH && !a.ids && !a.ntok && nA <= kPlanThreads) {
    int len = 0, need = 0, bad = 0, b = 0;
    if (tid < nA) {
      len = tb.seq_len[tid];
      b = tb.active[tid];
      need = len % dm.pt == 0;                        // the token opens a new page
      bad = need && len / dm.pt + 1 > dm.max_bp;
      tb.ap_id[tid] = b;
      tb.ap_start[tid] = len;
    }
    int total;
    const int ex = block_excl_scan(need, lds, total);
    if (__syncthreads_or(bad)) {
      if (tid == 0) record_error(scal, SART_E_INVALID, a.call_seq);
      return;
    }
    if (total > top) {
      if (tid == 0) record_error(scal, SART_E_OOM_PAGES, a.call_seq);
      return;
    }
    if (tid < nA) {
      if (need) tb.bt[scal[S_BTSEL]][(long long)tid * dm.max_bp + len / dm.pt] = tb.free_stack[top - 1 - ex];
      tb.seq_len[tid] = len + 1;
      tb.branch_appended[b / dm.Nb] = 1;
    }
    __syncthreads();
    if (tid == 0) {
      scal[S_FREETOP] = top - total;
      scal[S_CALLOK] = 1;
      scal[S_APPENDOK] = 1;
      if (a.defer_plan) scal[S_PLAN_DEFERRED] = 1;
    }
    // the decode plan of the lengthened rows: here, or (decode step) by one more workgroup of the kernel that
    // writes the rows, so that the two run side by side instead of one after the other
    if (!a.defer_plan) refresh_decode_plan(c, pc, lds);
    return;
  }
  // pass 1: validate, compute pages needed, stash id / start length
  int carry = 0, carry_new = 0;
  for (int base = 0; base < a.n_seqs; base += kPlanThreads) {
    const int i = base + tid;
    int need = 0, creates = 0;
    if (i < a.n_seqs) {
      const int id = a.ids ? a.ids[i] : tb.active[i];
      const int n = a.ntok ? a.ntok[i] : 1;
      int err = 0, len = 0, cap = 0;
      if (a.kind == SART_SEQ_PREFIX) {
        if (tb.req_used[id] && (tb.refcnt[id] == 0 || tb.branch_appended[id])) err = SART_E_STATE;
        len = tb.prefix_len[id];
        cap = dm.max_pp;
        creates = !tb.req_used[id];
      } else {
        if (!a.ids) len = tb.seq_len[i];                 // the active list itself: row i, known active
        else if (tb.br_state[id] != SART_BRANCH_ACTIVE) err = SART_E_STATE;
        else len = tb.seq_len[tb.active_idx_of[id]];
        cap = dm.max_bp;
      }
      const int have = ceil_div(len, dm.pt), want = ceil_div(len + n, dm.pt);
      if (!err && want > cap) err = SART_E_INVALID;
      if (err) atomicMin(&s_err, (i << 2) | err);
      need = want - have;
      tb.ap_id[i] = id;
      tb.ap_start[i] = len;
    }
    int tot, tot_new;
    const int ex = block_excl_scan(need, lds, tot);
    const int ex_new = block_excl_scan(creates, lds, tot_new);
    if (i < a.n_seqs) { tb.tmp_a[i] = carry + ex; tb.tmp_b[i] = carry_new + ex_new; }
    carry += tot;
    carry_new += tot_new;
  }
  __syncthreads();
  if (s_err != 0x7fffffff) {
    if (tid == 0) record_error(scal, s_err & 3, a.call_seq);
    return;
  }
  if (carry > top) {
    if (tid == 0) record_error(scal, SART_E_OOM_PAGES, a.call_seq);
    return;
  }
  // pass 2: apply
  int* bt = tb.bt[scal[S_BTSEL]];
  for (int i = tid; i < a.n_seqs; i += kPlanThreads) {
    const int id = tb.ap_id[i];
    const int n = a.ntok ? a.ntok[i] : 1;
    const int len = tb.ap_start[i];
    const int have = ceil_div(len, dm.pt), want = ceil_div(len + n, dm.pt);
    const int off = tb.tmp_a[i];
    int* table;
    if (a.kind == SART_SEQ_PREFIX) {
      table = tb.prefix_table + (long long)id * dm.max_pp;
      tb.prefix_len[id] = len + n;
      if (!tb.req_used[id]) {
        // Algorithm 1, Prefill: the request's Nb branches exist from now on, either in the batch at once or
        // awaiting (holding the prompt, but no place in the active list until sart_start_branches)
        tb.req_used[id] = 1;
        tb.refcnt[id] = dm.Nb;
        tb.nact[id] = dm.start_waiting ? 0 : dm.Nb;
        const int first = nA + tb.tmp_b[i] * dm.Nb;
        for (int j = 0; j < dm.Nb; ++j) {
          const int b = id * dm.Nb + j;
          if (dm.start_waiting) {
            tb.br_state[b] = SART_BRANCH_WAITING;
            continue;
          }
          tb.br_state[b] = SART_BRANCH_ACTIVE;
          tb.active[first + j] = b;
          tb.seq_len[first + j] = 0;
          tb.active_idx_of[b] = first + j;
        }
      }
    } else {
      const int row = tb.active_idx_of[id];
      table = bt + (long long)row * dm.max_bp;
      tb.seq_len[row] = len + n;
      if (n > 0) tb.branch_appended[id / dm.Nb] = 1;
    }
    for (int k = 0; k < want - have; ++k) table[have + k] = tb.free_stack[top - 1 - (off + k)];
  }
  __syncthreads();
  if (tid == 0) {
    const int na_new = nA + (dm.start_waiting ? 0 : carry_new * dm.Nb);
    scal[S_NACTIVE] = na_new;
    publish_active_count(tb, na_new);
    scal[S_FREETOP] = top - carry;
    const int sel = scal[S_BTSEL];
    if (scal[S_BTHI0 + sel] < na_new) scal[S_BTHI0 + sel] = na_new;
    scal[S_CALLOK] = 1;
    scal[S_APPENDOK] = 1;
  }
  refresh_decode_plan(c, pc, lds);
}

// OCP E4M3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, largest finite
// 448) nearest to x / scale, ties to the even code, magnitude clamped to 448.  The quotient is taken
// in float64 and rounded to the code's 4 significant bits in one step (v_rndne_f64), so the code is
// the one the exact quotient has: x carries 8 significant bits (bf16), scale 24, and a boundary
// between two codes at most 5, so a quotient that is not on a boundary is at least 2^-29 (relative)
// away from it, which the float64 division (2^-53) cannot bridge.  A float32 division can: it turns
// quotients within 2^-24 of a boundary into false ties.
__device__ inline unsigned e4m3_code_of_quotient(float x, float scale) {
  const double t = (double)x / (double)scale;
  double a = __builtin_fabs(t);
  if (!(a <= 448.0)) a = 448.0;
  unsigned code;
  if (a < 0x1p-6) {
    code = (unsigned)__builtin_rint(a * 512.0);            // subnormal codes count 2^-9; 8 is the first normal code
  } else {
    const int e = (int)((__double_as_longlong(a) >> 52) & 0x7ff) - 1023;      // a is normal: 2^-6 <= a <= 448
    const double s = __longlong_as_double(__double_as_longlong(a) - ((long long)(e - 3) << 52));   // a * 2^(3-e) in [8, 16)
    code = (unsigned)((e + 7) << 3) + ((unsigned)__builtin_rint(s) - 8u);     // a carry runs into the exponent field
  }
  return (__double_as_longlong(t) < 0 ? 0x80u : 0u) | code;
}

// One wave copies one (token, kv head) row of K and V into its page slot; the calling kernel's waves are
// numbered wave = 0 .. nwaves - 1.
template <typename T>
__device__ inline void append_write_rows(const Ctx& c, const AppendArgs& a, long long wave, long long nwaves) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int lane = threadIdx.x & 63;
  // n_seqs < 0: one row per active branch (a branch append leaves the active list as it is)
  const long long units = (a.n_seqs < 0 ? (long long)tb.scal[S_NACTIVE] : a.total_rows) * dm.Hkv;
  const int* bt = tb.bt[tb.scal[S_BTSEL]];
  T* pool = (T*)c.pool;
  for (long long u = wave; u < units; u += nwaves) {
    const long long row = u / dm.Hkv;
    const int head = (int)(u % dm.Hkv);
    // sequence owning this row: last i with tok_off[i] <= row
    int i;
    if (a.tok_off) {
      int lo = 0, hi = a.n_seqs - 1;
      while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if ((long long)a.tok_off[mid] <= row) lo = mid; else hi = mid - 1;
      }
      i = lo;
    } else {
      i = (int)row;
    }
    const int t = (int)(row - (a.tok_off ? a.tok_off[i] : i));
    const int pos = tb.ap_start[i] + t;
    // without an id list the sequences are the active rows themselves: no lookups of the handle and its row
    const int* table = a.kind == SART_SEQ_PREFIX ? tb.prefix_table + (long long)tb.ap_id[i] * dm.max_pp
                       : a.ids ? bt + (long long)tb.active_idx_of[tb.ap_id[i]] * dm.max_bp
                               : bt + (long long)i * dm.max_bp;
    const int page = table[pos / dm.pt], slot = pos % dm.pt;
    const long long kb = tile_base(dm, page, head), vb = kb + dm.tile_elems;
    const long long src = a.by_handle ? (long long)tb.ap_id[i] : row;      // rows of k and v by handle or in list order
    const T* ksrc = (const T*)a.k + (src * dm.Hkv + head) * dm.d;
    const T* vsrc = (const T*)a.v + (src * dm.Hkv + head) * dm.d;
    if (dm.dtype == SART_FP8_E4M3) {
      // bf16 in, one byte out: nearest E4M3 code of x / scale (ties to even), magnitude clamped to 448
      if constexpr (sizeof(T) == 2) {
        unsigned char* pool8 = (unsigned char*)c.pool;
        for (int d = lane; d < dm.d; d += 64) {
          pool8[kb + k_elem_off(dm.layout, dm.d, slot, d)] =
              (unsigned char)e4m3_code_of_quotient(__uint_as_float((unsigned)ksrc[d] << 16), dm.k_scale);
          pool8[vb + v_elem_off(dm.layout, dm.d, slot, d)] =
              (unsigned char)e4m3_code_of_quotient(__uint_as_float((unsigned)vsrc[d] << 16), dm.v_scale);
        }
      }
      continue;
    }
    for (int d = lane; d < dm.d; d += 64) {
      pool[kb + k_elem_off(dm.layout, dm.d, slot, d)] = ksrc[d];
      pool[vb + v_elem_off(dm.layout, dm.d, slot, d)] = vsrc[d];
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
k_append_write(Ctx c, AppendArgs a) {
  const Tables& tb = c.tb;
  if (!tb.scal[a.write_only ? S_APPENDOK : S_CALLOK]) {
    // a write to a layer > 0 whose layer-0 append failed on the device, or after rows moved (a finish or
    // prune since): nothing is written, and the caller is told (sticky)
    if (a.write_only && blockIdx.x == 0 && threadIdx.x == 0) record_error(tb.scal, SART_E_STATE, a.call_seq);
    return;
  }
  append_write_rows<T>(c, a, ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6, ((long long)gridDim.x * blockDim.x) >> 6);
}

// The decode step's form: the first workgroup computes the decode plan the append plan left to it, the others
// write the rows - neither needs the other's result.
template <typename T>
__global__ void __launch_bounds__(kPlanThreads)
k_append_write_and_plan(Ctx c, PlanCfg pc, AppendArgs a) {
  const Tables& tb = c.tb;
  if (blockIdx.x == 0) {                          // dispatched first: it is the longer of the two jobs
    __shared__ int lds[17];
    // the flags and what the plan's first pass reads are requested together: the append plan's kernel has
    // ended, so they are final (one trip to memory, where flag, count and rows would be three in a row)
    const PlanPre pre = plan_preload(c);
    if (pre.ok && pre.deferred) refresh_decode_plan<true>(c, pc, lds, pre);
    return;
  }
  if (!tb.scal[S_CALLOK]) return;
  append_write_rows<T>(c, a, ((long long)(blockIdx.x - 1) * blockDim.x + threadIdx.x) >> 6,
                       ((long long)(gridDim.x - 1) * blockDim.x) >> 6);
}

void launch_append(const Ctx& c, const PlanCfg& pc, const AppendArgs& a_in, hipStream_t s) {
  AppendArgs a = a_in;
  // the decode step's append (one token for every active row, no lists): plan and writes side by side
  a.defer_plan = !a.write_only && a.kind == SART_SEQ_BRANCH && !a.ids && !a.ntok && a.total_rows > 0;
  if (!a.write_only) hipLaunchKernelGGL(k_append_plan, dim3(1), dim3(kPlanThreads), 0, s, c, pc, a);
  if (a.total_rows <= 0) return;
  const long long units = a.total_rows * c.dm.Hkv;
  if (a.defer_plan) {
    long long wb = (units + 15) / 16;                    // 16 waves per workgroup
    if (wb > 2048) wb = 2048;
    if (c.dm.dtype == SART_F32)
      hipLaunchKernelGGL(k_append_write_and_plan<float>, dim3((unsigned)wb + 1), dim3(kPlanThreads), 0, s, c, pc, a);
    else
      hipLaunchKernelGGL(k_append_write_and_plan<uint16_t>, dim3((unsigned)wb + 1), dim3(kPlanThreads), 0, s, c, pc, a);
    return;
  }
  long long blocks = (units + 3) / 4;
  if (blocks > 8192) blocks = 8192;
  if (c.dm.dtype == SART_F32)
    hipLaunchKernelGGL(k_append_write<float>, dim3((unsigned)blocks), dim3(256), 0, s, c, a);
  else
    hipLaunchKernelGGL(k_append_write<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, c, a);
}

// ---------------------------------------------------------------------------
// Terminate pass, planning half (device function run by the single planning
// workgroup after victims were marked in new_state[]).
//  (1) victims in ascending active index push their private pages in
//      ascending logical order;
//  (2) then requests that lost their last branch, in ascending request id,
//      push their prefix pages;
//  (3) survivors keep their relative order.
// The pushes themselves and the block-table rows are moved by k_terminate_move.
// ---------------------------------------------------------------------------
__device__ void terminate_plan(const Ctx& c, const PlanCfg& pc, int* lds, bool stop_waiting) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  const int top = scal[S_FREETOP];
  for (int r = tid; r < dm.max_req; r += kPlanThreads) { tb.req_touched[r] = 0; tb.req_push_off[r] = -1; }
  __syncthreads();
  // Branches that were split share pages: a page goes back to the free stack with its last holder, at that
  // holder's turn.  Holders of a page hold every earlier page of theirs together too, so the pages a victim
  // releases are the tail [mv_first, pages) of its row.  One wave per victim row: (1) every page loses a
  // holder and notes the highest victim row holding it; (2) a row counts its leading pages that stay (someone
  // else still holds them, or a later victim releases them); (3) the releasing row resets the page's counters.
  const bool shared_pages = scal[S_ANY_FORK] != 0;
  if (shared_pages) {
    const int* bt_cur = tb.bt[scal[S_BTSEL]];
    const int lane = tid & 63, wave = tid >> 6, n_waves = kPlanThreads >> 6;
    for (int a = wave; a < nA; a += n_waves) {
      if (!tb.new_state[a]) continue;
      const int np = ceil_div(tb.seq_len[a], dm.pt);
      for (int l = lane; l < np; l += 64) {
        const int pg = bt_cur[(long long)a * dm.max_bp + l];
        atomicSub(&tb.page_extra[pg], 1);
        atomicMax(&tb.page_owner[pg], a);
      }
    }
    __syncthreads();
    for (int a = wave; a < nA; a += n_waves) {
      if (!tb.new_state[a]) continue;
      const int np = ceil_div(tb.seq_len[a], dm.pt);
      int stay = 0;
      for (int l = lane; l < np; l += 64) {
        const int pg = bt_cur[(long long)a * dm.max_bp + l];
        stay += !(tb.page_extra[pg] < 0 && tb.page_owner[pg] == a);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) stay += __shfl_xor(stay, off, 64);
      if (lane == 0) tb.mv_first[a] = stay;
    }
    __syncthreads();
    for (int a = wave; a < nA; a += n_waves) {
      if (!tb.new_state[a]) continue;
      const int np = ceil_div(tb.seq_len[a], dm.pt);
      for (int l = lane; l < np; l += 64) {
        const int pg = bt_cur[(long long)a * dm.max_bp + l];
        if (tb.page_owner[pg] != a) continue;
        if (tb.page_extra[pg] < 0) tb.page_extra[pg] = 0;
        tb.page_owner[pg] = -1;
      }
    }
    __syncthreads();
  }
  // scans over active rows: pages pushed by victims, new index of survivors
  int carry_p = 0, carry_s = 0;
  for (int base = 0; base < nA; base += kPlanThreads) {
    const int a = base + tid;
    int np = 0, keep = 0;
    if (a < nA) {
      if (tb.new_state[a]) np = ceil_div(tb.seq_len[a], dm.pt) - (shared_pages ? tb.mv_first[a] : 0); else keep = 1;
    }
    int tp, ts;
    const int exp_ = block_excl_scan(np, lds, tp);
    const int exs = block_excl_scan(keep, lds, ts);
    if (a < nA) {
      tb.mv_push_off[a] = tb.new_state[a] ? carry_p + exp_ : -1;
      tb.mv_new_idx[a] = tb.new_state[a] ? -1 : carry_s + exs;
    }
    carry_p += tp;
    carry_s += ts;
  }
  const int na_new = carry_s, priv_pages = carry_p;
  // victims: state, reference counts
  for (int a = tid; a < nA; a += kPlanThreads) {
    if (!tb.new_state[a]) continue;
    const int b = tb.active[a], r = b / dm.Nb;
    tb.br_state[b] = tb.new_state[a];
    tb.active_idx_of[b] = -1;
    atomicSub(&tb.refcnt[r], 1);
    atomicSub(&tb.nact[r], 1);
    tb.req_touched[r] = 1;
  }
  // a request that reached its quota is over: its awaiting branches never start (they hold no pages of their own)
  if (stop_waiting && dm.start_waiting && dm.Q >= 1 && dm.Q <= dm.Nb) {
    for (int b = tid; b < dm.H; b += kPlanThreads) {
      const int r = b / dm.Nb;
      if (tb.br_state[b] != SART_BRANCH_WAITING || tb.num_completed[r] < dm.Q) continue;
      tb.br_state[b] = SART_BRANCH_EARLY_STOPPED;
      atomicSub(&tb.refcnt[r], 1);
      tb.req_touched[r] = 1;
    }
  }
  __syncthreads();
  // requests whose last branch left: prefix pushes in ascending request id
  int carry_r = 0;
  for (int base = 0; base < dm.max_req; base += kPlanThreads) {
    const int r = base + tid;
    int np = 0, dead = 0;
    if (r < dm.max_req && tb.req_touched[r] && tb.refcnt[r] == 0) {
      dead = 1;
      np = ceil_div(tb.prefix_len[r], dm.pt);
    }
    int tr;
    const int ex = block_excl_scan(np, lds, tr);
    if (dead) tb.req_push_off[r] = carry_r + ex;
    carry_r += tr;
  }
  // compact the small active-order arrays through scratch
  for (int a = tid; a < nA; a += kPlanThreads) {
    const int ni = tb.mv_new_idx[a];
    if (ni >= 0) { tb.tmp_a[ni] = tb.active[a]; tb.tmp_b[ni] = tb.seq_len[a]; }
  }
  __syncthreads();
  for (int a = tid; a < nA; a += kPlanThreads) {
    if (a < na_new) {
      const int b = tb.tmp_a[a];
      tb.active[a] = b;
      tb.seq_len[a] = tb.tmp_b[a];
      tb.active_idx_of[b] = a;
    } else {
      tb.active[a] = -1;
      tb.seq_len[a] = 0;
    }
  }
  __syncthreads();
  if (tid == 0) {
    const int old_sel = scal[S_BTSEL], new_sel = old_sel ^ 1;
    scal[S_T_NA_OLD] = nA;
    scal[S_T_NA_NEW] = na_new;
    scal[S_T_TOP_OLD] = top;
    scal[S_T_PRIV_PAGES] = priv_pages;
    scal[S_T_BT_OLD] = old_sel;
    scal[S_T_CLEAR_HI] = scal[S_BTHI0 + new_sel];
    scal[S_BTHI0 + new_sel] = na_new;
    scal[S_BTSEL] = new_sel;
    scal[S_NACTIVE] = na_new;
    publish_active_count(tb, na_new);
    scal[S_FREETOP] = top + priv_pages + carry_r;
    scal[S_CALLOK] = 1;
  }
  refresh_decode_plan(c, pc, lds);
}

// Terminate pass, bulk half: one workgroup per old row / dead request.
__global__ void __launch_bounds__(256)
k_terminate_move(Ctx c) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  const int na_old = scal[S_T_NA_OLD], na_new = scal[S_T_NA_NEW], top = scal[S_T_TOP_OLD];
  const int priv = scal[S_T_PRIV_PAGES], clear_hi = scal[S_T_CLEAR_HI];
  const int* bt_old = tb.bt[scal[S_T_BT_OLD]];
  int* bt_new = tb.bt[scal[S_T_BT_OLD] ^ 1];
  const int rows_hi = na_old > clear_hi ? na_old : clear_hi;
  const int units = rows_hi + dm.max_req;
  for (int u = blockIdx.x; u < units; u += gridDim.x) {
    if (u < rows_hi) {
      // (a) old row u: push its pages or move it to its new place
      if (u < na_old) {
        const int* src = bt_old + (long long)u * dm.max_bp;
        const int off = tb.mv_push_off[u];
        if (off >= 0) {
          const int first = scal[S_ANY_FORK] ? tb.mv_first[u] : 0;      // earlier pages stay with other holders
          for (int p = first + threadIdx.x; p < dm.max_bp; p += blockDim.x) {
            const int page = src[p];
            if (page >= 0) tb.free_stack[top + off + p - first] = page;
          }
        } else {
          int* dst = bt_new + (long long)tb.mv_new_idx[u] * dm.max_bp;
          for (int p = threadIdx.x; p < dm.max_bp; p += blockDim.x) dst[p] = src[p];
        }
      }
      // (b) row u of the new buffer beyond the survivors goes back to -1
      if (u >= na_new && u < clear_hi) {
        int* dst = bt_new + (long long)u * dm.max_bp;
        for (int p = threadIdx.x; p < dm.max_bp; p += blockDim.x) dst[p] = -1;
      }
    } else {
      const int r = u - rows_hi;
      const int off = tb.req_push_off[r];
      if (off >= 0) {
        int* ptab = tb.prefix_table + (long long)r * dm.max_pp;
        for (int p = threadIdx.x; p < dm.max_pp; p += blockDim.x) {
          const int page = ptab[p];
          if (page >= 0) { tb.free_stack[top + priv + off + p] = page; ptab[p] = -1; }
        }
      }
    }
  }
}

static void launch_move(const Ctx& c, hipStream_t s) {
  int units = c.dm.H + c.dm.max_req;
  int blocks = units < 2048 ? units : 2048;
  hipLaunchKernelGGL(k_terminate_move, dim3(blocks), dim3(256), 0, s, c);
}

// first active index of every live request (a request's branches are
// contiguous in the active list: created together, compaction is stable)
__device__ inline void find_request_starts(const Ctx& c, int nA) {
  const Tables& tb = c.tb;
  for (int a = threadIdx.x; a < nA; a += kPlanThreads) {
    const int r = tb.active[a] / c.dm.Nb;
    if (a == 0 || tb.active[a - 1] / c.dm.Nb != r) tb.req_first[r] = a;
  }
}

__device__ inline bool key_less(float sa, int ha, float sb, int hb) {
  if (sa != sa) sa = __builtin_inff();
  if (sb != sb) sb = __builtin_inff();
  if (sa < sb) return true;
  if (sa > sb) return false;
  return ha < hb;
}

// ---------------------------------------------------------------------------
// A7: prune.  Victim selection per request, then the terminate plan.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_prune_plan(Ctx c, PlanCfg pc, PruneArgs a) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  __shared__ int lds[17];
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  if (tid == 0) scal[S_APPENDOK] = 0;      // rows of the last append may move: no more writes to other layers
  if (a.n_scores < nA) {
    if (tid == 0) record_error(scal, SART_E_INVALID, a.call_seq);
    return;
  }
  find_request_starts(c, nA);
  __syncthreads();
  for (int i = tid; i < nA; i += kPlanThreads) {
    const int b = tb.active[i], r = b / dm.Nb;
    const int first = tb.req_first[r], live = tb.nact[r];
    const float sc = a.scores[i];
    int room = 0x7fffffff;
    if (a.maxp) { room = a.maxp[r] - tb.num_pruned[r]; if (room < 0) room = 0; }
    int victim;
    if (a.mode == SART_PRUNE_THRESHOLD) {
      // Algorithm 1's predicate walked in ascending active index: the branches
      // before this one that qualify use up the room first.
      const float th = a.thr[r];
      int earlier = 0;
      for (int j = first; j < i; ++j) earlier += a.scores[j] < th;
      victim = (sc < th) && earlier < room;
    } else {
      int rank = 0;
      for (int j = first; j < first + live; ++j)
        rank += key_less(a.scores[j], tb.active[j], sc, b);
      int kk = a.k_per_req ? a.k_per_req[r] : a.k;
      kk = kk < 0 ? 0 : (kk > live ? live : kk);
      int nv = a.mode == SART_PRUNE_DROP_LOWEST_K ? kk : live - kk;
      if (nv > room) nv = room;
      victim = rank < nv;
    }
    tb.new_state[i] = victim ? SART_BRANCH_PRUNED : 0;
  }
  __syncthreads();
  for (int i = tid; i < nA; i += kPlanThreads)
    if (tb.new_state[i]) atomicAdd(&tb.num_pruned[tb.active[i] / dm.Nb], 1);
  __syncthreads();
  terminate_plan(c, pc, lds, false);
}

void launch_prune(const Ctx& c, const PlanCfg& pc, const PruneArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_prune_plan, dim3(1), dim3(kPlanThreads), 0, s, c, pc, a);
  launch_move(c, s);
}

// ---------------------------------------------------------------------------
// A8: completion + early stop, then the terminate plan.
// ---------------------------------------------------------------------------
// Who completes: the listed handles, or (targets != null, no list) every active
// branch whose length has reached targets[handle]; in that form a step with no
// such branch changes nothing and the move kernel that follows does nothing.
__global__ void __launch_bounds__(kPlanThreads)
k_finish_plan(Ctx c, PlanCfg pc, int n, const int* handles, const int* targets, int call_seq) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  __shared__ int lds[17];
  __shared__ int s_bad, s_any;
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  if (tid == 0) { s_bad = 0; s_any = 0; }
  __syncthreads();
  for (int i = tid; i < n; i += kPlanThreads)
    if (tb.br_state[handles[i]] != SART_BRANCH_ACTIVE) s_bad = 1;
  __syncthreads();
  if (s_bad) {
    if (tid == 0) record_error(scal, SART_E_STATE, call_seq);
    return;
  }
  for (int a = tid; a < nA; a += kPlanThreads) tb.new_state[a] = 0;
  __syncthreads();
  if (targets) {
    for (int a = tid; a < nA; a += kPlanThreads) {
      const int b = tb.active[a];
      if (tb.seq_len[a] >= targets[b]) {
        tb.new_state[a] = SART_BRANCH_COMPLETED;
        atomicAdd(&tb.num_completed[b / dm.Nb], 1);
        s_any = 1;
      }
    }
    __syncthreads();
    if (!s_any) {
      if (tid == 0) scal[S_CALLOK] = 0;     // not an error: nothing for the move kernel to do
      return;
    }
  }
  if (tid == 0) scal[S_APPENDOK] = 0;        // rows move: no more writes to other layers for the last append
  for (int i = tid; i < n; i += kPlanThreads) {
    const int b = handles[i];
    tb.new_state[tb.active_idx_of[b]] = SART_BRANCH_COMPLETED;
    atomicAdd(&tb.num_completed[b / dm.Nb], 1);
  }
  __syncthreads();
  if (dm.Q >= 1 && dm.Q <= dm.Nb) {
    for (int a = tid; a < nA; a += kPlanThreads)
      if (!tb.new_state[a] && tb.num_completed[tb.active[a] / dm.Nb] >= dm.Q)
        tb.new_state[a] = SART_BRANCH_EARLY_STOPPED;
  }
  __syncthreads();
  terminate_plan(c, pc, lds, true);
}

void launch_finish(const Ctx& c, const PlanCfg& pc, int n, const int* handles_dev, const int* targets_dev, int call_seq,
                   hipStream_t s) {
  hipLaunchKernelGGL(k_finish_plan, dim3(1), dim3(kPlanThreads), 0, s, c, pc, n, handles_dev, targets_dev, call_seq);
  launch_move(c, s);
}

// ---------------------------------------------------------------------------
// Waiting branches join the batch (Algorithm 1, main workflow: while the batch
// has room, an awaiting branch is popped from the branch queue and appended to
// the current batch).  The listed branches, all WAITING, become ACTIVE; each is
// placed right after the last active branch of its request, or, when the
// request has none, at the end of the list (request by request in the order of
// first appearance in the list): what inserting them one by one in list order
// gives.  So a request's rows stay neighbours in the active list.
//   new index of old row a   = a + started branches of the requests whose rows end before a
//   place of list entry i    = new index of its request's last row + 1 + rank of i among the
//                              list's entries of that request, or
//                              old rows + all branches placed behind rows + offset of the
//                              request's group among the row-less requests + rank
// The block-table rows move with their branches into the other buffer
// (k_start_move); a started branch's row is empty.
// ---------------------------------------------------------------------------
// A split (src != null; tree search expands a trajectory into several
// continuations, Section 2): list entry i joins as a copy of the ACTIVE branch
// src[i] - its length, its block-table row (copied by k_start_move like a moved
// row), sharing the pages that are full; a partly filled last page is replaced
// by a freshly popped page that k_fork_fix fills (pages popped in list order).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_start_plan(Ctx c, PlanCfg pc, int n, const int* handles, const int* src, int call_seq) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  int* scal = tb.scal;
  __shared__ int lds[17];
  __shared__ int s_bad;
  const int tid = threadIdx.x;
  const int nA = scal[S_NACTIVE];
  const int top = scal[S_FREETOP];
  if (tid == 0) s_bad = 0;
  __syncthreads();
  for (int i = tid; i < n; i += kPlanThreads) {
    if (tb.br_state[handles[i]] != SART_BRANCH_WAITING) s_bad = 1;
    if (src && tb.br_state[src[i]] != SART_BRANCH_ACTIVE) s_bad = 1;
  }
  __syncthreads();
  if (s_bad) {
    if (tid == 0) record_error(scal, SART_E_STATE, call_seq);
    return;
  }
  int fork_pages = 0;                          // pages the copies of partly filled last pages need
  if (src) {
    for (int base = 0; base < n; base += kPlanThreads) {
      const int i = base + tid;
      int need = 0;
      if (i < n) {
        const int old_row = tb.active_idx_of[src[i]];
        tb.mv_first[i] = old_row;              // (the rows move below: kept for the entry's length and row copy; scratch)
        need = tb.seq_len[old_row] % dm.pt != 0;
      }
      int tot;
      const int ex = block_excl_scan(need, lds, tot);
      if (i < n) tb.tmp_b[i] = need ? fork_pages + ex : -1;      // which pop is the entry's, for now
      fork_pages += tot;
    }
    if (fork_pages > top) {
      if (tid == 0) record_error(scal, SART_E_OOM_PAGES, call_seq);
      return;
    }
  }
  if (tid == 0) scal[S_APPENDOK] = 0;        // rows move: no more writes to other layers for the last append
  for (int r = tid; r < dm.max_req; r += kPlanThreads) { tb.req_touched[r] = 0; tb.req_tmp[r] = 0; }
  find_request_starts(c, nA);
  __syncthreads();
  // per list entry: its rank among the list's entries of its request; per request: how many of its branches start
  for (int i = tid; i < n; i += kPlanThreads) {
    const int r = handles[i] / dm.Nb;
    int rank = 0;
    for (int j = 0; j < i; ++j) rank += handles[j] / dm.Nb == r;
    tb.tmp_a[i] = rank;
    atomicAdd(&tb.req_touched[r], 1);
  }
  __syncthreads();
  // old rows: shifted by the branches placed behind the requests that end before them; scratch copies of the
  // small active-order arrays
  int carry = 0;
  for (int base = 0; base < nA; base += kPlanThreads) {
    const int a = base + tid;
    int v = 0;
    if (a < nA) {
      tb.new_state[a] = tb.active[a];
      tb.mv_push_off[a] = tb.seq_len[a];
      if (a > 0) {
        const int r = tb.active[a] / dm.Nb, prev = tb.active[a - 1] / dm.Nb;
        if (prev != r) v = tb.req_touched[prev];
      }
    }
    int tot;
    const int ex = block_excl_scan(v, lds, tot);
    if (a < nA) tb.mv_new_idx[a] = a + carry + ex + v;
    carry += tot;
  }
  __syncthreads();
  const int behind_rows = carry + (nA > 0 ? tb.req_touched[tb.active[nA - 1] / dm.Nb] : 0);
  // requests without a row: groups at the end, in order of first appearance in the list
  int carry_g = 0;
  for (int base = 0; base < n; base += kPlanThreads) {
    const int i = base + tid;
    int v = 0, r = 0;
    if (i < n) {
      r = handles[i] / dm.Nb;
      if (tb.nact[r] == 0 && tb.tmp_a[i] == 0) v = tb.req_touched[r];
    }
    int tot;
    const int ex = block_excl_scan(v, lds, tot);
    if (v > 0) tb.req_tmp[r] = carry_g + ex;
    carry_g += tot;
  }
  __syncthreads();
  const int na_new = nA + n;
  for (int u = tid; u < na_new; u += kPlanThreads) tb.ap_id[u] = -1;     // new row -> old row it comes from (-1: a started branch)
  __syncthreads();
  for (int a = tid; a < nA; a += kPlanThreads) {
    const int ni = tb.mv_new_idx[a], b = tb.new_state[a];
    tb.active[ni] = b;
    tb.seq_len[ni] = tb.mv_push_off[a];
    tb.active_idx_of[b] = ni;
    tb.ap_id[ni] = a;
  }
  for (int i = tid; i < n; i += kPlanThreads) {
    const int b = handles[i], r = b / dm.Nb;
    const int pos = tb.nact[r] > 0 ? tb.mv_new_idx[tb.req_first[r] + tb.nact[r] - 1] + 1 + tb.tmp_a[i]
                                   : nA + behind_rows + tb.req_tmp[r] + tb.tmp_a[i];
    tb.active[pos] = b;
    tb.seq_len[pos] = src ? tb.mv_push_off[tb.mv_first[i]] : 0;      // a copy starts with its source's length
    if (src) tb.ap_id[pos] = tb.mv_first[i];                          // and its row of the block table
    tb.active_idx_of[b] = pos;
    tb.br_state[b] = SART_BRANCH_ACTIVE;
  }
  __syncthreads();
  if (src) {
    // what k_fork_fix needs per entry: its row (tmp_a) and the page popped for it (tmp_b, -1: none)
    for (int i = tid; i < n; i += kPlanThreads) {
      tb.tmp_a[i] = tb.active_idx_of[handles[i]];
      if (tb.tmp_b[i] >= 0) tb.tmp_b[i] = tb.free_stack[top - 1 - tb.tmp_b[i]];
    }
  }
  for (int r = tid; r < dm.max_req; r += kPlanThreads) tb.nact[r] += tb.req_touched[r];
  if (tid == 0) {
    if (src) { scal[S_FREETOP] = top - fork_pages; scal[S_ANY_FORK] = 1; }
    const int old_sel = scal[S_BTSEL], new_sel = old_sel ^ 1;
    scal[S_T_NA_OLD] = nA;
    scal[S_T_NA_NEW] = na_new;
    scal[S_T_BT_OLD] = old_sel;
    scal[S_T_CLEAR_HI] = scal[S_BTHI0 + new_sel];
    scal[S_BTHI0 + new_sel] = na_new;
    scal[S_BTSEL] = new_sel;
    scal[S_NACTIVE] = na_new;
    publish_active_count(tb, na_new);
    scal[S_CALLOK] = 1;
  }
  refresh_decode_plan(c, pc, lds);
}

// The block-table rows of the start plan: one workgroup per row of the new buffer.
__global__ void __launch_bounds__(256)
k_start_move(Ctx c) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  const int na_new = scal[S_T_NA_NEW], clear_hi = scal[S_T_CLEAR_HI];
  const int* bt_old = tb.bt[scal[S_T_BT_OLD]];
  int* bt_new = tb.bt[scal[S_T_BT_OLD] ^ 1];
  const int rows = na_new > clear_hi ? na_new : clear_hi;
  for (int u = blockIdx.x; u < rows; u += gridDim.x) {
    const int src = u < na_new ? tb.ap_id[u] : -1;        // rows past the new list go back to -1
    int* dst = bt_new + (long long)u * dm.max_bp;
    for (int p = threadIdx.x; p < dm.max_bp; p += blockDim.x) dst[p] = src >= 0 ? bt_old[(long long)src * dm.max_bp + p] : -1;
  }
}

// After a split's rows were copied: entry i's row shares its full pages (one more holder each) and, where the
// source's last page is partly filled, gets the page popped for it with that page's contents in every layer.
__global__ void __launch_bounds__(256)
k_fork_fix(Ctx c, int n, int n_layers, long long layer_bytes) {
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  const int* scal = tb.scal;
  if (!scal[S_CALLOK]) return;
  int* bt = tb.bt[scal[S_BTSEL]];
  const long long page_bytes = dm.page_elems * dm.esize;
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const int row = tb.tmp_a[i], len = tb.seq_len[row], full = len / dm.pt;
    int* my = bt + (long long)row * dm.max_bp;
    for (int p = threadIdx.x; p < full; p += blockDim.x) atomicAdd(&tb.page_extra[my[p]], 1);
    const int fresh = tb.tmp_b[i];
    if (fresh < 0) continue;
    const int old = my[full];
    for (int l = 0; l < n_layers; ++l) {
      const uint4* from = (const uint4*)((const unsigned char*)c.pool + l * layer_bytes + old * page_bytes);
      uint4* to = (uint4*)((unsigned char*)c.pool + l * layer_bytes + fresh * page_bytes);
      for (long long x = threadIdx.x; x < page_bytes / 16; x += blockDim.x) to[x] = from[x];
    }
    __syncthreads();                           // every thread has read `old`
    if (threadIdx.x == 0) my[full] = fresh;
  }
}

void launch_start(const Ctx& c, const PlanCfg& pc, int n, const int* handles_dev, const int* src_dev, int n_layers,
                  size_t layer_bytes, int call_seq, hipStream_t s) {
  hipLaunchKernelGGL(k_start_plan, dim3(1), dim3(kPlanThreads), 0, s, c, pc, n, handles_dev, src_dev, call_seq);
  const int blocks = c.dm.H < 2048 ? c.dm.H : 2048;
  hipLaunchKernelGGL(k_start_move, dim3(blocks), dim3(256), 0, s, c);
  if (src_dev && n > 0)
    hipLaunchKernelGGL(k_fork_fix, dim3(n < 2048 ? n : 2048), dim3(256), 0, s, c, n, n_layers, (long long)layer_bytes);
}

// Stand-alone refresh of the decode plan (after sart_alloc_cache and when the
// launch shape changes).
__global__ void __launch_bounds__(kPlanThreads)
k_decode_plan(Ctx c, PlanCfg pc) {
  __shared__ int lds[17];
  refresh_decode_plan(c, pc, lds);
}

void launch_plan(const Ctx& c, const PlanCfg& pc, hipStream_t s) {
  hipLaunchKernelGGL(k_decode_plan, dim3(1), dim3(kPlanThreads), 0, s, c, pc);
}

}  // namespace sart
