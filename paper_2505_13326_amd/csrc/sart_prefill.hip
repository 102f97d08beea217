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
// kPfTileRows rows (twice that for long bf16 prompts, then two tiles per
// workgroup), on the matrix-core tile the decode kernel
// uses (S^T = K Q^T and O^T += V^T P^T as 16x16x32 bf16 products; online softmax
// on the vector ALUs).  Pages are taken two at a time (32 tokens): one update of
// the maximum per 32 tokens.  Blocks skip pairs that lie wholly after their
// rows' positions and mask scores only on the pairs that straddle them.  No
// split over the sequence: one wave sees a row's whole context, so there is no
// merge.  Two kernels: k_prefill_mfma (8-bit float caches: every wave loads its
// page pairs into registers and expands them there) and k_prefill_b16 (bf16
// caches: pairs staged once per workgroup in LDS, two 16-row blocks per wave).
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
    // what a tile's workgroup needs to know of its sequence, in one 16-byte load
    ((int4*)tb.pf_seq)[i] = make_int4(r, a.nq[i], a.q_off[i], tb.prefix_len[r]);
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

// The grid of the matrix-core kernels is (workgroups of the longest listed sequence, sequences): block (x, y)
// is workgroup x of sequence y, or nothing when that sequence has fewer.  Here (8-bit float caches) a workgroup
// is one tile of tile_rows rows of one kv head; a sequence's later rows (longer contexts) come first.
struct PfTile { int req, nq, plen, h, rt; long long q_row0; };
__device__ inline bool prefill_tile(const Dims& dm, const Tables& tb, int tile_rows, PfTile& t) {
  const int4 sq = ((const int4*)tb.pf_seq)[blockIdx.y];
  t.req = sq.x; t.nq = sq.y; t.q_row0 = sq.z; t.plen = sq.w;
  const int tiles_per_head = ceil_div(t.nq * dm.G, tile_rows);
  const int local = blockIdx.x;
  if (local >= tiles_per_head * dm.Hkv) return false;
  // Neighbouring blocks take the kv heads in turn: workgroups are dealt to the 8 XCDs round-robin, so with 8
  // kv heads (or a divisor of 8) every XCD serves few heads and the K/V pages that a head's tiles share stay
  // in that XCD's L2 (measured on 64 x 1024-token prompts, 8 kv heads: with head-major order the workgroups
  // pulled 8 TB/s of K/V through the fabric and waited for it)
  t.h = local % dm.Hkv;
  t.rt = tiles_per_head - 1 - local / dm.Hkv;
  return true;
}

// (Launched for 8-bit float caches; bf16 caches take k_prefill_b16 below.)
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
  PfTile pt;
  if (!prefill_tile(dm, tb, a.tile_rows, pt)) return;
  const int req = pt.req, nq = pt.nq, plen = pt.plen, h = pt.h, rt = pt.rt;
  const int n_rows = nq * dm.G;
  const int row_w0 = rt * kPfRowsPerWg + wv * kPfRowsPerWave;
  if (row_w0 >= n_rows) return;
  const int p_first = plen - nq;                           // prompt position of the call's first query
  const long long q_row0 = pt.q_row0;
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

typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
// bf16 caches: NW waves of 32 query rows (a tile of 128 or 256 rows of one kv head), two waves per SIMD with
// the whole tile state in registers.  A page pair is fetched once per workgroup into a ring of three LDS stages
// (one barrier per pair); a wave's 32 rows are two blocks of 16 on the 16x16x32 product, and every K and V
// operand read from LDS serves both blocks.  Lane (r = l % 16, g = l / 16) holds, per block, row r: its Q^T
// operands, the scores of tokens 4 g .. 4 g + 3 of either page, and the output columns 16 j + 4 g .. + 3 of
// every 16-column slab j.
//   S^T (16 tokens x 16 rows) = K (16 x 32 per step) Q^T per page and block: the A operand of step i is chunk
//        i * 64 + l of the page's K tile as stored;
//   O^T (16 of d x 16 rows) += V^T P^T per slab and block over the pair's 32 tokens: contraction index
//        g * 8 + e is token 4 g + e % 4 of page e / 4, so P^T is the lane's own 4 + 4 weights, and the A operand
//        of slab 2 i + half is that half of chunk i * 64 + l of the first page's V tile, then of the second's:
//        the loader writes the chunks' halves into LDS in that order.
// Softmax against a lagging reference: the reference of a row is raised, and its accumulators rescaled, only
// when some score exceeds it by 2^kLag (one wave vote per pair over both blocks); until then a weight may
// exceed 1, which is harmless in fp32 and bf16, and l and O / l do not depend on the reference.  A row's
// tokens are spread over the four lanes r, r + 16, r + 32, r + 48: the denominator is summed per lane from
// the bf16-rounded weights with the packed dot product (v_dot2c_f32_bf16) and joined at the end.
// TPW = 2 (8 waves, one workgroup per CU): a workgroup takes two tiles of one kv head one after the other, the
// j-th heaviest and the j-th lightest (every workgroup of a sequence then has the same number of page pairs),
// and the K/V stream runs on across the two: while the first tile's last pairs are computed the second tile's
// first pairs are already on their way into the ring, its Q rows are requested before the first tile's output
// is staged, and what a tile costs before its first product (descriptor, addresses, the first loads: 4-5 us)
// is paid once per two tiles.  The output staging then has an LDS area of its own.
template <int D, int NW, int TPW>
__global__ void __launch_bounds__(64 * NW, 8 / NW)
k_prefill_b16(Ctx c, PrefillArgs a, const int* __restrict__ prefix_table) {
  constexpr int ROWS = 32, NB = 2;
  static_assert(NW == 4 || NW == 8, "one or two workgroups of two waves per SIMD");
  static_assert(TPW == 1 || (TPW == 2 && NW == 8), "a second tile needs the staging area of its own that one workgroup per CU has room for");
  const Dims& dm = c.dm;
  const Tables& tb = c.tb;
  if (!tb.scal[S_CALLOK]) return;
  constexpr int KQ = D / 32;                               // steps of a score product = chunks per lane and tile
  constexpr int NS = D / 16;                               // 16-column slabs of O^T
  constexpr int kTileBytes = 16 * D * 2, kPageBytes = 2 * kTileBytes;
  constexpr int kChunks = kTileBytes / 16;                 // 16-byte chunks of one K (or V) tile
  constexpr int kStages = 3;
  // one stage: the K tiles of the pair's two pages as stored, then the V operands (2 * kChunks slots of two
  // 8-byte pieces).  With one tile per workgroup the ring also stages the output at the end (d = 64: that
  // needs more than the three stages).
  constexpr int kRowStride = 64 + 4;                       // floats per staged output row: 64 columns + padding
  constexpr int kOutFloats = ROWS * kRowStride + 2 * ROWS; // per wave: 32 rows, then their output offsets
  constexpr int kStagesOut = (NW * kOutFloats * 4 + 64 * kChunks - 1) / (64 * kChunks);
  constexpr int kStagesAlloc = TPW == 1 && kStagesOut > kStages ? kStagesOut : kStages;
  __shared__ uint4 lds[kStagesAlloc][4 * kChunks];
  __shared__ float s_out[TPW == 2 ? NW * kOutFloats : 4];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, g4 = lane >> 4;
  // the workgroup's tiles: block (x, y) is item x of sequence y; neighbouring items take the kv heads in turn
  const int4 sq = ((const int4*)tb.pf_seq)[blockIdx.y];
  const int req = sq.x, nq = sq.y, plen = sq.w;
  const long long q_row0 = sq.z;
  const int n_rows = nq * dm.G;
  const int tiles_per_head = ceil_div(n_rows, ROWS * NW);
  const int items_per_head = TPW == 2 ? (tiles_per_head + 1) >> 1 : tiles_per_head;
  if ((int)blockIdx.x >= items_per_head * dm.Hkv) return;
  const int h = blockIdx.x % dm.Hkv, item = blockIdx.x / dm.Hkv;
  const int rt0 = tiles_per_head - 1 - item;               // a sequence's later rows (longer contexts) come first
  const int rt1 = item;                                    // the second tile, if it is another one
  const int n_tiles = TPW == 2 && rt1 < rt0 ? 2 : 1;
  const int p_first = plen - nq;
  const uint16_t* q = (const uint16_t*)a.q;
  const unsigned char* pool = (const unsigned char*)c.pool;
  const int* __restrict__ table = prefix_table + (long long)req * dm.max_pp;
  const long long page_bytes = dm.page_elems * 2;

  // pages a tile needs: its last row's context
  auto pages_of = [&](int rt) { return (p_first + min((rt + 1) * (ROWS * NW) - 1, n_rows - 1) / dm.G) / 16 + 1; };
  const int n_pages0 = pages_of(rt0), n_pages1 = n_tiles == 2 ? pages_of(rt1) : 0;
  const int n_pairs0 = (n_pages0 + 1) >> 1, n_pairs1 = (n_pages1 + 1) >> 1;
  const int total_pairs = n_pairs0 + n_pairs1;

  // this lane's two query rows of the current tile: (query, head of the group), query-major; rows past the end
  // shadow the last one
  int pos[NB];
  long long qrow[NB];
  bool have[NB];
  uint4 qreg[NB][KQ];
  f32x4 O[NB][NS];
  float m_ref[NB], lsum[NB];
  auto rows_of = [&](int rt, int (&pos_)[NB], long long (&qrow_)[NB], bool (&have_)[NB]) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int row = rt * (ROWS * NW) + wv * ROWS + 16 * b + r16;
      have_[b] = row < n_rows;
      const int rc = have_[b] ? row : n_rows - 1;
      const int ql = rc / dm.G, g = rc % dm.G;
      pos_[b] = p_first + ql;
      qrow_[b] = ((q_row0 + ql) * dm.Hq + h * dm.G + g) * D;
    }
  };
  auto load_q = [&](const long long (&qrow_)[NB]) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < KQ; ++i) qreg[b][i] = *(const uint4*)(q + qrow_[b] + i * 32 + g4 * 8);
  };
  auto reset_state = [&]() {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
      for (int j = 0; j < NS; ++j) O[b][j] = f32x4{0.f, 0.f, 0.f, 0.f};
      m_ref[b] = -__builtin_inff();
      lsum[b] = 0.f;
    }
  };
  rows_of(rt0, pos, qrow, have);
  load_q(qrow);
  reset_state();

  // loader: the pair's two pages go to the two halves of the workgroup (the first 32 NW threads: first page,
  // the others: second page); a thread moves kPerThread stored chunks of its page's K tile (to the same place in the stage)
  // and as many of its V tile (each as two 8-byte pieces, to where the products' operand reads find them:
  // every operand read is one contiguous KiB per wave).  A thread reads the id of its page itself, with a
  // vector load two turns ahead: scalar loads return out of order, and one in flight would turn every wait
  // for an LDS operand into a wait for everything.  The pairs of the workgroup's tiles are one sequence,
  // gp = 0 .. total_pairs - 1, through the same page table.
  constexpr int kHalf = 32 * NW;                           // threads per page
  constexpr int kPerThread = kChunks / kHalf;              // chunks of a tile per thread
  static_assert(kPerThread * kHalf == kChunks && (kPerThread == 1 || (kPerThread == 2 && kHalf == 128)), "unsupported tile / workgroup shape");
  const int pg = tid / kHalf, lt = tid % kHalf;
  const int v_dst0 = (((2 * (lt >> 6)) * 64 + (lt & 63)) << 1) + pg;        // uint2 index of the low half of chunk lt
  const int* my_ids = table + pg;                           // my_ids[2 p]: this thread's page of a tile's pair p
  auto page_index = [&](int gp) {                           // an odd last page is paired with itself
    const bool second = TPW == 2 && gp >= n_pairs0;
    return min(2 * (second ? gp - n_pairs0 : gp), (second ? n_pages1 : n_pages0) - 1 - pg);
  };
  uint4 gk0, gk1, gv0, gv1;                                 // (named registers: arrays captured by the lambdas end up in scratch memory)
  gk1 = gv1 = uint4{0u, 0u, 0u, 0u};
  int pid = my_ids[page_index(0)], pid_next = my_ids[page_index(min(1, total_pairs - 1))];
  auto g_load = [&](int gp_after_next) {   // fetches the pair whose id is in pid; requests the id of a later pair
    const unsigned char* b = pool + (long long)pid * page_bytes + (long long)h * kPageBytes + lt * 16;
    gk0 = *(const uint4*)b;
    gv0 = *(const uint4*)(b + kTileBytes);
    if constexpr (kPerThread == 2) {
      gk1 = *(const uint4*)(b + 128 * 16);
      gv1 = *(const uint4*)(b + kTileBytes + 128 * 16);
    }
    pid = pid_next;
    pid_next = my_ids[page_index(gp_after_next)];
  };
  auto l_store = [&](int stage) {
    uint2* vdst = (uint2*)&lds[stage][2 * kChunks];
    lds[stage][pg * kChunks + lt] = gk0;
    vdst[v_dst0] = uint2{gv0.x, gv0.y};
    vdst[v_dst0 + 128] = uint2{gv0.z, gv0.w};              // the high half: the next slab's operand, 64 slots on
    if constexpr (kPerThread == 2) {
      lds[stage][pg * kChunks + lt + 128] = gk1;
      vdst[v_dst0 + 512] = uint2{gv1.x, gv1.y};            // chunk lt + 128: two slab pairs (4 x 64 slots) on
      vdst[v_dst0 + 512 + 128] = uint2{gv1.z, gv1.w};
    }
  };

  g_load(min(2, total_pairs - 1));                         // pair 0
  l_store(0);
  g_load(min(3, total_pairs - 1));                         // pair 1
  __syncthreads();
  int gp = 0;
  for (int t = 0; t < n_tiles; ++t) {
    const int rt = t ? rt1 : rt0;
    const int n_pages = t ? n_pages1 : n_pages0, n_pairs = t ? n_pairs1 : n_pairs0;
    const int row_w0 = rt * (ROWS * NW) + wv * ROWS;
    const bool wave_has_rows = row_w0 < n_rows;            // a wave without rows still helps to load
    const int lo_pos = wave_has_rows ? p_first + row_w0 / dm.G : -1;
    const int wave_last_pos = wave_has_rows ? p_first + min(row_w0 + ROWS - 1, n_rows - 1) / dm.G : -1;
    const int wave_pairs = wave_has_rows ? wave_last_pos / 32 + 1 : 0;     // pairs this wave needs
    const int bound = min(plen, n_pages * 16);             // tokens that exist in the pages the tile reads
    for (int pr = 0; pr < n_pairs; ++pr, ++gp) {
      const int stage = gp % kStages;
      l_store((gp + 1) % kStages);                         // pair gp + 1 (loaded a turn ago), read a turn from now
      g_load(min(gp + 4, total_pairs - 1));                // pair gp + 2 (or the last pair again)
      if (pr < wave_pairs) {
        const int t0 = pr * 32;
        uint4 kop[2][KQ], vop[NS];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
          for (int i = 0; i < KQ; ++i) kop[p][i] = lds[stage][p * kChunks + i * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);                 // all K operands are requested before anything else is scheduled
#pragma unroll
        for (int j = 0; j < NS; ++j) vop[j] = lds[stage][2 * kChunks + j * 64 + lane];
        f32x4 S[NB][2];
#pragma unroll
        for (int b = 0; b < NB; ++b) S[b][0] = S[b][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < KQ; ++i)
#pragma unroll
          for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int b = 0; b < NB; ++b)
              S[b][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kop[p][i]), __builtin_bit_cast(bf16x8, qreg[b][i]), S[b][p], 0, 0, 0);
        const bool full = t0 + 31 <= lo_pos;
        if (!full) {
          // element j of the lane is token 4 g + j of the first page resp. 16 + 4 g + j (second page): masked past
          // the row's position and past the tokens that exist; the V of tokens that do not exist may be anything: zeroed
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const int lim = min(pos[b] + 1, bound) - t0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              if (4 * g4 + j >= lim) S[b][0][j] = -__builtin_inff();
              if (16 + 4 * g4 + j >= lim) S[b][1][j] = -__builtin_inff();
            }
          }
          const int nvalid = bound - t0, tk = 4 * g4;
          const unsigned a01 = (tk + 0 < nvalid ? 0x0000ffffu : 0u) | (tk + 1 < nvalid ? 0xffff0000u : 0u);
          const unsigned a23 = (tk + 2 < nvalid ? 0x0000ffffu : 0u) | (tk + 3 < nvalid ? 0xffff0000u : 0u);
          const unsigned b01 = (tk + 16 < nvalid ? 0x0000ffffu : 0u) | (tk + 17 < nvalid ? 0xffff0000u : 0u);
          const unsigned b23 = (tk + 18 < nvalid ? 0x0000ffffu : 0u) | (tk + 19 < nvalid ? 0xffff0000u : 0u);
#pragma unroll
          for (int j = 0; j < NS; ++j) { vop[j].x &= a01; vop[j].y &= a23; vop[j].z &= b01; vop[j].w &= b23; }
        }
        float mine[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
          mine[b] = fmaxf(fmaxf(fmaxf(S[b][0][0], S[b][0][1]), fmaxf(S[b][0][2], S[b][0][3])),
                          fmaxf(fmaxf(S[b][1][0], S[b][1][1]), fmaxf(S[b][1][2], S[b][1][3])));
        if (__any(mine[0] * a.scale_log2 > m_ref[0] + kLag || mine[1] * a.scale_log2 > m_ref[1] + kLag)) {   // also the first pair: the references are -inf
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const float mx = max_over_rows(mine[b]) * a.scale_log2;
            const float m_new = fmaxf(m_ref[b], mx);
            const float alpha = __builtin_amdgcn_exp2f(m_ref[b] - m_new);
            m_ref[b] = m_new;
            lsum[b] *= alpha;
#pragma unroll
            for (int j = 0; j < NS; ++j) O[b][j] *= alpha;
          }
        }
        uint4 pp[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          unsigned pk[4];
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[b][w >> 1][2 * (w & 1)], a.scale_log2, -m_ref[b]));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[b][w >> 1][2 * (w & 1) + 1], a.scale_log2, -m_ref[b]));
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            const bf16x2v pb = __builtin_convertvector(f32x2{p0, p1}, bf16x2v);
            pk[w] = __builtin_bit_cast(unsigned, pb);
            lsum[b] = __builtin_amdgcn_fdot2_f32_bf16(pb, __builtin_bit_cast(bf16x2v, 0x3f803f80u), lsum[b], false);
          }
          pp[b] = uint4{pk[0], pk[1], pk[2], pk[3]};
        }
#pragma unroll
        for (int j = 0; j < NS; ++j)
#pragma unroll
          for (int b = 0; b < NB; ++b)
            O[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vop[j]), __builtin_bit_cast(bf16x8, pp[b]), O[b][j], 0, 0, 0);
      }
      __syncthreads();
    }
    // The next tile's rows: their Q is requested now (the registers are free) and arrives while this tile's
    // output is staged.
    int pos_n[NB];
    long long qrow_n[NB];
    bool have_n[NB];
    if (t + 1 < n_tiles) {
      rows_of(rt1, pos_n, qrow_n, have_n);
      load_q(qrow_n);
    }
    // Output.  A lane holds 4-column pieces of its two rows: stored from the registers, a wave's store would
    // touch 64 separate 16-byte pieces.  The tile goes through LDS instead (with one tile per workgroup the
    // ring's stages, free now: every wave is past the last barrier), 64 columns at a time, each wave in a
    // region of its own, rows padded to 272 bytes, and leaves in stores of four 256-byte row segments each.
    if (wave_has_rows) {
      float* wreg = (TPW == 2 ? s_out : (float*)&lds[0][0]) + wv * kOutFloats;
      long long* row_off = (long long*)(wreg + ROWS * kRowStride);      // element offset of every row's output, -1: no row
      float inv[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        inv[b] = a.v_scale / sum_over_rows(lsum[b]);       // every row sees at least its own token
        if (g4 == 0) row_off[16 * b + r16] = have[b] ? qrow[b] : -1;
      }
#pragma unroll
      for (int half = 0; half < D / 64; ++half) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            *(f32x4*)(wreg + (16 * b + r16) * kRowStride + 16 * j + 4 * g4) = O[b][4 * half + j] * inv[b];
        // (a wave reads only what it wrote itself: no barrier, the compiler's wait for the LDS writes suffices)
#pragma unroll
        for (int it = 0; it < ROWS / 4; ++it) {
          const int r = 4 * it + (lane >> 4), dc = (lane & 15) * 4;
          const long long off = row_off[r];
          const f32x4 v = *(const f32x4*)(wreg + r * kRowStride + dc);
          if (off >= 0) *(f32x4*)(a.out + off + 64 * half + dc) = v;
        }
      }
    }
    if (t + 1 < n_tiles) {
#pragma unroll
      for (int b = 0; b < NB; ++b) { pos[b] = pos_n[b]; qrow[b] = qrow_n[b]; have[b] = have_n[b]; }
      reset_state();
    }
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

// bf16 caches with head_dim 128: tiles of 256 rows (8 waves, one workgroup per CU: a page pair fetched from the
// pool serves twice the rows) once a sequence has several of them; 128 rows (4 waves, two workgroups per CU)
// for short ones and for every other shape.
int prefill_tile_rows(const Dims& dm, long long max_rows) {
  if (dm.layout == SART_LAYOUT_MFMA16 && dm.d == 128 && max_rows >= 4 * 2 * kPfTileRows) return 2 * kPfTileRows;
  return kPfTileRows;
}

void launch_prefill(const Ctx& c, const PrefillArgs& a, hipStream_t s) {
  const Dims& dm = c.dm;
  hipLaunchKernelGGL(k_prefill_check, dim3(1), dim3(256), 0, s, c, a);
  if (a.total_q <= 0) return;
  if (dm.layout != SART_LAYOUT_NATURAL) {
    auto go = [&](auto kern) {
      hipLaunchKernelGGL(kern, dim3(a.max_tiles, a.n_seqs), dim3(kAttnThreads), 0, s, c, a, c.tb.prefix_table);
    };
    const bool fp8 = dm.layout == SART_LAYOUT_MFMA16_FP8;
    if (!fp8) {   // bf16: the LDS-staged kernel
      const dim3 grid(a.max_tiles, a.n_seqs);
      if (a.tile_rows == 2 * kPfTileRows) hipLaunchKernelGGL((k_prefill_b16<128, 8, 2>), grid, dim3(512), 0, s, c, a, c.tb.prefix_table);
      else if (dm.d == 128) hipLaunchKernelGGL((k_prefill_b16<128, 4, 1>), grid, dim3(256), 0, s, c, a, c.tb.prefix_table);
      else hipLaunchKernelGGL((k_prefill_b16<64, 4, 1>), grid, dim3(256), 0, s, c, a, c.tb.prefix_table);
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
