/*
 * sart_bench.h - measurement and tuning aids of libsart.  NOT part of the
 * method's interface (that is sart.h): nothing here is needed to serve requests.
 * bench.py and the tests that sweep launch shapes call these; a serving loop
 * never does.
 */
#ifndef SART_BENCH_H
#define SART_BENCH_H

#include "sart.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launch statistics of the last sart_decode_attention on this cache, measured
 * with HIP events on the stream the kernels ran on (for bench harnesses).
 * sart_set_profiling(cache, n): n = 0 off; n = 1 each decode call records
 * events around its dominant (attention) kernel; n > 1 the call launches that
 * kernel n times back to back between the events (it is idempotent), which
 * amortises the events' own dispatch overhead; ms_attn is then the average per
 * launch.  ms_total: the whole call's device work.  sart_last_decode_ms waits
 * for the events. */
sart_status sart_set_profiling(sart_cache* cache, int32_t on);
sart_status sart_last_decode_ms(sart_cache* cache, float* ms_attn, float* ms_total);

/* Measurement aid, no part of the method: reads `bytes` (a multiple of 8 KiB is
 * used) of a DEVICE buffer with plain coalesced loads, in 8 KiB chunks, in
 * ascending order or in the order chunk_order gives (DEVICE, bytes / 8192
 * entries, each a chunk number below that; NULL: ascending).  Asynchronous on
 * `stream`; the caller times it.  bench.py reports the attention kernel's rate
 * against this one's on the same box. */
sart_status sart_read_probe(const void* buf, size_t bytes, const int32_t* chunk_order, void* stream);

/* The same probe with its launch shape given, for the sweep that looks for the
 * best rate plain reads reach (bench.py --workload probe): n_workgroups of 256
 * threads (4 waves; 256 workgroups = one wave per SIMD), depth = 8 KiB chunks in
 * flight per wave (1, 2, 4 or 8), flavour 0 = plain loads, 1 = loads with the
 * non-temporal hint, interleave 0 = a wave reads a contiguous run of chunks,
 * 1 = wave w reads chunks w, w + waves, ... (neighbouring waves read
 * neighbouring chunks at the same time).  sart_read_probe is the shape
 * (2048, 4, plain, contiguous). */
sart_status sart_read_probe_shaped(const void* buf, size_t bytes, const int32_t* chunk_order, int32_t n_workgroups,
                                   int32_t depth, int32_t flavour, int32_t interleave, void* stream);

/* Measurement aid, no part of the method: n_workgroups of 4 waves (a CU takes two of them: 256 workgroups =
 * one wave per SIMD on MI355X, 512 = two) each run `rounds` rounds of 524288 flops of bf16 matrix-core products
 * on operands held in registers.  shape 0: 16 products 32x32x16 per round, 8 into one
 * accumulator and 8 into four others (the prefill kernel's own sequence of products); shape 1: 32 products
 * 16x16x32 into 8 accumulators in turn; shape 2: the arithmetic of the bf16 prefill kernel's loop over page pairs
 * for head_dim 128 and nothing else of it (16 score products 16x16x32 of two 16-row blocks against two pages,
 * the softmax of the lane's 16 scores: exp2, conversion to bf16, denominators; 16 output products), the
 * same flops per round.  A wave holds 8 A and 8 B operands per lane, read once from
 * `operands` (DEVICE, 16 KiB: operand i of lane l at byte (i * 64 + l) * 16, A operands first; the same for
 * every wave).  sink (DEVICE, n_workgroups * 256 floats) receives a sum per lane.  Asynchronous on `stream`;
 * the caller times it.  The rate depends on the operand values (zeros draw less power, and the clock follows
 * the power): bench.py reports the prefill kernel's rate against this one's on the same box. */
sart_status sart_mfma_probe(const void* operands, int64_t rounds, int32_t n_workgroups, int32_t shape, float* sink,
                            void* stream);

/* Tuning knobs of the decode launch (defaults are chosen for MI355X):
 *   n_workgroups   persistent attention grid of 4-wave workgroups (<= 0: one per
 *                  CU);
 *   prompt_mode    how the shared prompt is read, in blocks of prompt pages.
 *                  1 = one read of a block per branch of the request (G of the
 *                  matrix-core tile's 16 rows used); 2 = one read per tile of 16
 *                  query rows of the request (rows = (branch, head of the GQA
 *                  group), branch-major: with G = 7 and 8 branches, 4 tiles
 *                  instead of 8 per-branch reads).  In both the items are
 *                  ordered so that the readers of a block run at the same time
 *                  on one XCD and all but the first read hit in its L2.
 *                  0 (default on the matrix-core layouts) = the planning kernel
 *                  chooses per step: per branch, whose longer items stream
 *                  better, unless the tiles save a wave about 48 prompt pages or
 *                  more, or the step has little private work to hide the prompts
 *                  behind (measured over a grid of shapes).  Natural-layout
 *                  caches always use 1.  -1 = keep the current setting.  (A mode
 *                  that staged each prompt chunk in LDS once per workgroup was
 *                  measured 2.5 to 3 times slower on prompt-heavy workloads and
 *                  is not in the library.)
 *   skew_permille  work moved from odd to even workgroups, in 1/1000 of the
 *                  mean per-wave range (workgroups go round-robin to the 8 XCDs,
 *                  and the odd XCDs stream about 10 % slower); default 80,
 *                  0 = equal. */
sart_status sart_set_decode_launch(sart_cache* cache, int32_t n_workgroups, int32_t prompt_mode, int32_t skew_permille);

/* Order of a wave's two parts in the matrix-core attention kernel, its share of
 * the prompts and its range of the branches' own pages.  on != 0 (default):
 * groups of 8 workgroups alternate, prompts first / own range first, so that at
 * any time half of the waves at most are in the latency-bound prompt part;
 * 0: every wave serves its prompt work first. */
sart_status sart_set_prompt_stagger(sart_cache* cache, int32_t on);

/* Where the partial results of a decode step are merged: in_kernel = 0 (the
 * default): by the separate merge kernel; != 0: by the attention kernel's own
 * last writers where the kernel can (the matrix-core kernel with the prompts
 * read inline): every piece counts itself in for its (row, kv head) and the
 * last one folds.  Same results bit for bit.  Measured on MI355X the in-kernel
 * form is the slower one (7B-like config: call 0.2595 against 0.2547 ms;
 * 32B-like: 1.656 against 1.611 ms): each piece waits for its stores and for the
 * counter's round trip while no other wave can use its SIMD. */
sart_status sart_set_merge_mode(sart_cache* cache, int32_t in_kernel);

#ifdef __cplusplus
}
#endif
#endif /* SART_BENCH_H */
