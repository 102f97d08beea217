// Internal declarations shared by the HIP sources of libsart (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sart.h"
#include "sart_bench.h"

namespace sart {

constexpr int kWave = 64;
constexpr int kPlanThreads = 1024;     // single-workgroup planning kernels
constexpr int kAttnWaves = 4;          // waves per attention workgroup (one per SIMD, one workgroup per CU)
constexpr int kAttnThreads = kAttnWaves * kWave;
constexpr int kPfBlocks = 2;           // prefill: 16-row blocks per wave (two waves per SIMD fit the registers)
constexpr int kPfTileRows = 16 * kPfBlocks * kAttnWaves;   // prefill: rows of one workgroup tile
constexpr int kSharedBlocks = 1;       // shared-rows prompt mode: 16-row blocks of a row tile (1: every wave gets a
                                       // tile's worth of prompt work; 4 read the prompt less often but left
                                       // three waves in four without prompt work, measured slower)
constexpr int kMaxGroup = 16;          // query heads per KV head the MFMA tile holds

// Indices into the device scalar block.
enum Scalar {
  S_NACTIVE = 0,
  S_FREETOP,
  S_BTSEL,        // which of the two block-table buffers is current
  S_ERR,          // sticky status of the first failed call
  S_ERRCALL,      // sequence number of that call
  S_CALLOK,       // the call now running passed its device-side validation
  S_BTHI0,        // rows of block-table buffer 0 that may hold non -1 entries
  S_BTHI1,
  // plan of the terminate pass (written by the plan kernel, read by the move kernel)
  S_T_NA_OLD,
  S_T_NA_NEW,
  S_T_TOP_OLD,
  S_T_PRIV_PAGES, // pages pushed by branches; prefix pushes start after them
  S_T_BT_OLD,     // buffer index holding the rows to move
  S_T_CLEAR_HI,   // rows [na_new, clear_hi) of the new buffer must be reset to -1
  // plan of the decode pass
  S_D_NA,
  S_APPENDOK,     // the last layer-0 append passed its validation and no call changed the state since
  S_D_PER_EVEN,   // units per wave of an even workgroup
  S_D_PER_ODD,    // units per wave of an odd workgroup
  S_D_NLIVE,      // live requests with a non-empty prompt
  S_D_NWG,        // attention workgroups the plan was made for
  S_D_UOWN,       // units of the own region (branches' private pages)
  S_D_NOWN,       // ranges (waves) serving the own region
  S_D_NPROMPT,    // waves serving the prompt work items (all of them, or 0 without prompts)
  S_D_PB,         // pages per prompt block
  S_D_NBLOCKS,    // prompt blocks (partial slots of the prompts)
  S_D_NPITEMS,    // prompt work items of the streaming phase (= blocks unless rows are shared)
  S_D_PMODE,      // how the step's prompts are read: 1 per branch, 2 per tile of 16 query rows (chosen by the plan)
  S_PLAN_DEFERRED,// the append plan left the decode plan to the write kernel's extra workgroup
  S_ANY_FORK,     // some branch was split since the cache was created: branch pages may be shared
  // the plan's last choice of how prompts are read, and what it was made from (the estimate behind it is
  // repeated only when one of these changes)
  S_PM_CHOICE,
  S_PM_SIG_A,     // active rows
  S_PM_SIG_B,     // prompt pages over the live requests' branches
  S_PM_SIG_C,     // live requests, private units per wave (up to the rule's cap), attention workgroups
  S_COUNT = 40
};

struct Dims {
  int Hq, Hkv, G, d, pt, num_pages, max_req, Nb, Q, max_bp, max_pp, H, dtype, layout, esize;
  int start_waiting;      // a request's branches are created WAITING and join the batch through sart_start_branches
  long long tile_elems;   // pt * d: elements of one K (or V) tile
  long long page_elems;   // Hkv * 2 * tile_elems
  float k_scale, v_scale;           // 8-bit float caches: K and V are stored as codes of x / scale
};

struct Tables {
  int* scal;
  int* free_stack;
  // per request
  int* req_used;
  int* prefix_len;
  int* prefix_table;     // [max_req][max_pp]
  int* refcnt;           // branches that hold the request's prefix: active and waiting ones
  int* nact;             // the request's rows in the active list
  int* req_tmp;          // [max_req] scratch of the start plan
  int* num_completed;
  int* num_pruned;
  int* branch_appended;
  // per branch handle
  int* br_state;
  int* active_idx_of;    // handle -> active index, -1 when not active
  // active order
  int* active;           // handles
  int* seq_len;
  int* bt[2];            // [H][max_bp] ping-pong block tables
  // scratch of the planning kernels
  int* new_state;        // [H]
  int* mv_push_off;      // [H]  -1 for survivors
  int* mv_new_idx;       // [H]
  int* mv_first;         // [H] a terminating row's first page that goes back to the free stack (0 unless pages are shared)
  int* page_extra;       // [num_pages] holders of a branch page beyond the first (0 unless branches were split)
  int* page_owner;       // [num_pages] scratch of the terminate pass, -1 between passes
  int* tmp_a;            // [H]
  int* tmp_b;            // [H]
  int* req_first;        // [max_req] first active index of the request
  int* req_push_off;     // [max_req] -1 unless the request died in this pass
  int* req_touched;      // [max_req]
  // append plan
  int* ap_id;            // [H] resolved sequence ids
  int* ap_start;         // [H] length before the append
  // decode plan
  int* page_cum;         // [H+1] exclusive scan of private pages over active rows
  int* live_req;         // [max_req] live requests with prompt, active order
  int* live_item_start;  // [max_req+1] exclusive scan of prefix items
  int* wave_row;         // [max attention waves] own ranges: active row of the first unit; prompt ranges: live request index
  int* req_pstart;       // [max_req] first prompt block of the request
  int* wave_desc;        // [max attention waves][16] where each wave starts (see refresh_decode_plan)
  int* row_desc;         // [H][8] per active row: what a piece of the row needs to know to merge (see refresh_decode_plan)
  int* pf_seq;           // [max_req][4] prefill: request, queries, first q row, prompt tokens of every listed sequence
  int* host_nactive;     // one int in pinned host memory: the active count, stored again whenever it changes
  int* seg_count;        // [H * Hkv] arrivals per (row, kv head) in the running attention kernel; 0 between kernels
};

// Launch shape the decode plan is made for (host-chosen, passed to every
// planning kernel).
struct PlanCfg {
  int n_wg;           // persistent attention workgroups
  int prompt_mode;    // how the prompts are read: 1 in blocks per (chunk, branch), 2 in blocks whose pages are read once
                      // for a tile of 16 query rows of the request (shared rows)
  int skew_permille;  // even workgroups take (1000+skew)/1000 of the mean range, odd ones the rest
};

struct Ctx {
  Dims dm;
  Tables tb;
  void* pool;
};

// ---- work of one decode step -> waves ------------------------------------------
// The work is a set of (page, kv head) units of 8 KiB (d = 128).
//   own line      every active row's private pages, ordered (row, kv head, page),
//                 cut into one contiguous range per wave (a range may cross rows;
//                 a long row is split over many waves).
//   prompt blocks every live request's prompt is read in blocks of pb pages,
//                 once per branch or once per tile of 16 query rows of the
//                 request; the work items over one chunk are neighbours, go to
//                 waves of one workgroup (or of workgroups on one XCD) and are
//                 read at the same time, so all but the first reader hit in cache.
// Every wave serves its prompt work item(s) and its own-line range.  Workgroups are
// dispatched round-robin over the 8 XCDs and on MI355X the odd XCDs stream
// measurably slower than the even ones, so own ranges come in pairs of
// workgroups: waves of an even workgroup take pe units, those of the following
// odd workgroup po units.
struct Cut {
  int pe, po;            // units per own range of even / odd workgroups
  long long u_own;       // units on the own line
  int n_own;             // ranges [0, n_own) serve the own line
  int n_prompt;          // waves serving prompt work items (all, or 0)
  int pb;                // pages per prompt block
  int n_blocks;          // prompt blocks; block b's partial goes to slot n_own + S + b
  int n_pitems;          // prompt work items: the blocks themselves, or (request, kv head, chunk, row tile)
                         // items that each write the blocks of up to 64 query rows (shared-rows mode)
};
__host__ __device__ inline long long own_start(const Cut& k, long long w) {
  const long long b = w / kAttnWaves, wv = w % kAttnWaves;
  const long long pair = b >> 1;
  return pair * kAttnWaves * (k.pe + k.po) + ((b & 1) ? (long long)kAttnWaves * k.pe + wv * k.po : wv * k.pe);
}
__host__ __device__ inline long long own_end(const Cut& k, long long w) {
  const long long e = own_start(k, w) + (((w / kAttnWaves) & 1) ? k.po : k.pe);
  return e < k.u_own ? e : k.u_own;
}
// Non-negative 64-bit quotient; operands that fit 32 bits (every count of this library on any realistic
// cache) take the 32-bit division, which costs the GPU a tenth of the instructions of the 64-bit one.
__host__ __device__ inline long long div_nn(long long a, long long b) {
  return (((unsigned long long)a | (unsigned long long)b) >> 32) ? a / b : (long long)((unsigned)a / (unsigned)b);
}
__host__ __device__ inline long long own_of_unit(const Cut& k, long long u) {
  const long long span = (long long)kAttnWaves * (k.pe + k.po);
  const long long pair = div_nn(u, span), off = u - pair * span;
  if (off < (long long)kAttnWaves * k.pe) return pair * 2 * kAttnWaves + div_nn(off, k.pe);
  return pair * 2 * kAttnWaves + kAttnWaves + div_nn(off - (long long)kAttnWaves * k.pe, k.po);
}
// Which prompt block the i-th prompt wave serves first (then every n_prompt-th
// after it).  Workgroup b runs on XCD b % 8, and neighbouring blocks read the
// same pages, so they go to workgroups of one XCD (one L2): with a multiple of
// 8 workgroups, the blocks are dealt to XCD 0's workgroups first, then XCD 1's, ...
__host__ __device__ inline long long prompt_range_of_wave(long long i, int n_prompt) {
  const long long nwg = n_prompt / kAttnWaves;
  if (nwg % 8) return i;
  const long long b = i / kAttnWaves, wv = i % kAttnWaves;
  const long long per_xcd = nwg / 8;
  return ((b % 8) * per_xcd + b / 8) * kAttnWaves + wv;
}

// ---- layout: element offsets inside one K or V tile ------------------------
// NATURAL: [token][d].   MFMA16: see sart.h.
__host__ __device__ inline long long k_elem_off(int layout, int d_dim, int token, int d) {
  if (layout == SART_LAYOUT_NATURAL) return (long long)token * d_dim + d;
  if (layout == SART_LAYOUT_MFMA16_FP8)
    return ((long long)(d >> 6) * 64 + ((d >> 3) & 3) * 16 + token) * 16 + ((d >> 5) & 1) * 8 + (d & 7);
  return ((long long)(d >> 3) * 16 + token) * 8 + (d & 7);
}
__host__ __device__ inline long long v_elem_off(int layout, int d_dim, int token, int d) {
  if (layout == SART_LAYOUT_NATURAL) return (long long)token * d_dim + d;
  if (layout == SART_LAYOUT_MFMA16_FP8)
    return ((long long)(d >> 6) * 64 + (token >> 2) * 16 + (d & 15)) * 16 + ((d >> 5) & 1) * 8 + ((d >> 4) & 1) * 4 + (token & 3);
  int chunk = (d >> 5) * 64 + (token >> 2) * 16 + (d & 15);
  int e = (token & 3) + (((d >> 4) & 1) << 2);
  return (long long)chunk * 8 + e;
}
// element offset of the K tile of (page, kv head); the V tile follows it
__host__ __device__ inline long long tile_base(const Dims& dm, int page, int head) {
  return (long long)page * dm.page_elems + (long long)head * 2 * dm.tile_elems;
}

// ---- kernels' launchers (defined in the .hip files) ------------------------
struct AppendArgs {
  int kind, n_seqs;
  const int* ids;      // device or null
  const int* ntok;     // device or null
  const int* tok_off;  // device or null (null: one token per sequence)
  long long total_rows;
  const void* k;
  const void* v;
  int call_seq;
  int write_only;      // layer > 0: write the rows of the last layer-0 append again, into this layer's pool
  int defer_plan;      // decode step's append: the write kernel's extra workgroup computes the decode plan, beside the writes
  int by_handle;       // all-active form: the row of k and v that belongs to a branch is its handle, not its active index
};
void launch_append(const Ctx& c, const PlanCfg& pc, const AppendArgs& a, hipStream_t s);

struct PruneArgs {
  int mode, k;
  const int* k_per_req;  // device or null
  const float* thr;      // device or null
  const int* maxp;       // device or null
  const float* scores;
  int n_scores;
  int call_seq;
};
void launch_prune(const Ctx& c, const PlanCfg& pc, const PruneArgs& a, hipStream_t s);
void launch_finish(const Ctx& c, const PlanCfg& pc, int n, const int* handles_dev, const int* targets_dev, int call_seq,
                   hipStream_t s);
void launch_plan(const Ctx& c, const PlanCfg& pc, hipStream_t s);
// src_dev != null: the listed branches join as copies of the branches src_dev lists (a split); the pool has
// n_layers layers, layer_bytes apart
void launch_start(const Ctx& c, const PlanCfg& pc, int n, const int* handles_dev, const int* src_dev, int n_layers,
                  size_t layer_bytes, int call_seq, hipStream_t s);

struct DecodeArgs {
  const void* q;
  float* out;
  int n_rows;
  float scale_log2;     // scale * log2(e)
  int n_wg;             // persistent attention workgroups (the plan's)
  float* partials;      // scratch
  long long partial_cap; // partial slots available
  int* seg_count;       // scratch: arrival counters of the in-kernel merge, one per (row, kv head), zero between kernels
  int fused_merge;      // the attention kernel's last writer of a (row, kv head) merges its partial results
  int stagger_prompt;   // half of the workgroups serve their prompt work after their own range instead of before
  int by_handle;        // rows of q and out are addressed by branch handle instead of by active index
  int call_seq;
  float v_scale;        // 8-bit float caches: what the output is multiplied by (1 otherwise)
  hipEvent_t ev[4];     // optional profiling events (null: none)
  int repeats;          // profiling: attention launches between ev[1] and ev[2]
};
void launch_decode(const Ctx& c, const DecodeArgs& a, hipStream_t s);
// floats of one partial result: o[G][d], then m[G], l[G], padded to a 16-byte multiple
__host__ __device__ inline long long partial_floats(int G, int d) { return (long long)G * d + ((2 * G + 3) & ~3); }
// the fixed scratch of sart_decode_attention_static (bytes), and where the current device keeps it
constexpr size_t kStaticScratchBytes = SART_STATIC_SCRATCH_BYTES;
constexpr size_t kStaticCounterBytes = 256u << 10;    // its first part: the in-kernel merge's arrival counters
hipError_t static_scratch(int* device, void** ptr);

struct PrefillArgs {
  int n_seqs;
  const int* ids;         // device: request of every listed sequence
  const int* nq;          // device: queries per sequence (its last nq prompt tokens)
  const int* q_off;       // device: first row of the sequence in q / out
  const void* q;
  float* out;
  float scale_log2;
  float v_scale;          // 8-bit float caches: what the output is multiplied by (1 otherwise)
  int call_seq;
  int max_tiles;          // workgroups of the listed sequence that has most (matrix-core kernels: grid x)
  int tile_rows;          // rows of a workgroup tile (prefill_tile_rows)
  int total_q;
};
void launch_prefill(const Ctx& c, const PrefillArgs& a, hipStream_t s);
int prefill_tile_rows(const Dims& dm, long long max_rows);   // rows of one kv head per workgroup tile of the prefill kernel, for a call whose longest sequence has max_rows rows per kv head

void launch_init_tables(const Ctx& c, const int* free_order_dev, hipStream_t s);
void launch_read_probe(const void* buf, long long n_chunks, const int* order, int n_workgroups, int depth, int flavour,
                       int interleave, hipStream_t s);
void launch_mfma_probe(const void* operands, long long iters, int n_workgroups, int shape, float* sink, hipStream_t s);

}  // namespace sart
