// Tiles shared by the attention kernels (gfx950).  Matrix-core tile: one
// 16-token page of K and V against 16 query rows, with the online-softmax state
// of those rows.  Vector-ALU row routine for the untuned generic path.
#pragma once

#include "sart_device.h"

namespace sart {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

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

// max over the four 16-lane rows of a wave for every column (lane & 15), on
// the vector ALU: v_permlane32_swap / v_permlane16_swap exchange half-waves and
// odd/even rows between two registers; feeding the same value twice and taking
// the max of both results is the pairwise max whichever half is swapped.
__device__ inline float max_over_rows(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned v = __float_as_uint(x);
  const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ inline float sum_over_rows(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const unsigned v = __float_as_uint(x);
  const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// One 16-token page: kq[i] / vq[i] are the 16-byte chunks this lane loaded
// (chunk i*64 + lane of the K resp. V tile), qreg the Q^T operand.  FULL: all
// 16 tokens are valid (no masking code).  Scores are kept in the log2 domain:
// p = 2^(s*c - m) with c = scale*log2(e).
// Not FULL: tokens >= nvalid of the page do not exist (their K/V bytes may be
// anything): their scores are masked and their V rows zeroed; nvalid is
// wave-uniform.  nvalid_row (per lane, by its query row lane & 15; <= nvalid)
// masks further scores of that row only: the causal bound of prefill.
template <int D, bool FULL>
__device__ inline void process_page(WaveState<D>& st, const uint4* kq, const uint4* vq, const uint4* qreg,
                                    int nvalid, int nvalid_row, float scale_log2) {
  const int g = (threadIdx.x & 63) >> 4;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < D / 32; ++i)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kq[i]),
                                                __builtin_bit_cast(bf16x8, qreg[i]), s, 0, 0, 0);
  uint4 vloc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i) vloc[i] = vq[i];
  if (!FULL) {
    const int t0 = 4 * g;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (t0 + j >= nvalid_row) s[j] = -__builtin_inff();
    const unsigned m01 = (t0 + 0 < nvalid ? 0x0000ffffu : 0u) | (t0 + 1 < nvalid ? 0xffff0000u : 0u);
    const unsigned m23 = (t0 + 2 < nvalid ? 0x0000ffffu : 0u) | (t0 + 3 < nvalid ? 0xffff0000u : 0u);
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      vloc[i].x &= m01; vloc[i].y &= m23; vloc[i].z &= m01; vloc[i].w &= m23;
    }
  }
  float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
  mx = max_over_rows(mx) * scale_log2;           // scale > 0: max commutes with the scaling
  const float m_new = fmaxf(st.m, mx);           // finite: a page holds >= 1 valid token
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // 0 on the first page (m = -inf)
  st.m = m_new;
  f32x4 p;
#pragma unroll
  for (int j = 0; j < 4; ++j) p[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[j], scale_log2, -m_new));
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

// 8-bit float caches (SART_LAYOUT_MFMA16_FP8): a 16-byte chunk of the tile holds
// what two bf16 chunks hold.  expand_fp8 turns the D/64 raw chunks of a lane into
// the D/32 bf16 chunks process_page expects (E4M3 values are exact in bf16; the
// cache's scales are applied to the scores and to the output, not here).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline unsigned fp8x2_to_bf16x2(unsigned codes, bool high_half) {
  return high_half ? __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, true))
                   : __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false));
}
template <int D>
__device__ inline void expand_fp8(const uint4* raw, uint4* out) {
#pragma unroll
  for (int c = 0; c < D / 64; ++c) {
    out[2 * c] = uint4{fp8x2_to_bf16x2(raw[c].x, false), fp8x2_to_bf16x2(raw[c].x, true),
                       fp8x2_to_bf16x2(raw[c].y, false), fp8x2_to_bf16x2(raw[c].y, true)};
    out[2 * c + 1] = uint4{fp8x2_to_bf16x2(raw[c].z, false), fp8x2_to_bf16x2(raw[c].z, true),
                           fp8x2_to_bf16x2(raw[c].w, false), fp8x2_to_bf16x2(raw[c].w, true)};
  }
}
// chunks a lane loads per K (or V) tile, and process_page on them as loaded
template <int D, bool FP8> constexpr int raw_chunks() { return FP8 ? D / 64 : D / 32; }
template <int D, bool FP8, bool FULL>
__device__ inline void process_raw(WaveState<D>& st, const uint4* rk, const uint4* rv, const uint4* qreg,
                                   int nvalid, int nvalid_row, float scale_log2) {
  if constexpr (FP8) {
    uint4 kq[D / 32], vq[D / 32];
    expand_fp8<D>(rk, kq);
    expand_fp8<D>(rv, vq);
    process_page<D, FULL>(st, kq, vq, qreg, nvalid, nvalid_row, scale_log2);
  } else {
    process_page<D, FULL>(st, rk, rv, qreg, nvalid, nvalid_row, scale_log2);
  }
}

// Two consecutive pages (32 tokens) at once, for the compute-bound prefill:
// one running-max update per 32 tokens, and O^T += V^T P^T as 16x16x32
// products.  The contraction index of that product is (lane >> 4, e): e < 4 is
// token 4 (lane >> 4) + e of the first page, e >= 4 the same token of the second
// page, for the V operand (built from the two pages' chunks of this lane) and
// for the P operand (this lane's 4 + 4 scores) alike, so no data crosses lanes.
// nvalid / nvalid_row count tokens from the first page's start (up to 32).
// The three phases are separate functions so that a caller with several
// independent 16-row blocks can run each phase for all blocks in turn (scores of
// all blocks, then their softmax updates, then their O^T products): many
// independent matrix-core operations in a row, and K (resp. V) registers that
// are free for the next loads after the first (resp. last) phase.
// qv: this lane's Q^T chunks, QSTRIDE uint4 apart (1 in registers; 64 in an LDS tile of 64 lanes)
template <int D, int QSTRIDE>
__device__ inline void pair_scores(const uint4* kq0, const uint4* kq1, const uint4* qv, f32x4& s0, f32x4& s1) {
  s0 = f32x4{0.f, 0.f, 0.f, 0.f};
  s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    const bf16x8 qi = __builtin_bit_cast(bf16x8, qv[i * QSTRIDE]);
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kq0[i]), qi, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kq1[i]), qi, s1, 0, 0, 0);
  }
}
// online-softmax update of the block's state from the 32 scores; returns P^T as the B operand
template <int D, bool FULL>
__device__ inline bf16x8 pair_softmax(WaveState<D>& st, f32x4 s0, f32x4 s1, int nvalid_row, float scale_log2) {
  if (!FULL) {
    const int t0 = 4 * ((threadIdx.x & 63) >> 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (t0 + j >= nvalid_row) s0[j] = -__builtin_inff();
      if (16 + t0 + j >= nvalid_row) s1[j] = -__builtin_inff();
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])), fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
  mx = max_over_rows(mx) * scale_log2;
  const float m_new = fmaxf(st.m, mx);
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  st.m = m_new;
  f32x4 p0, p1;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    p0[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[j], scale_log2, -m_new));
    p1[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[j], scale_log2, -m_new));
  }
  st.l = st.l * alpha + ((p0[0] + p0[1]) + (p0[2] + p0[3])) + ((p1[0] + p1[1]) + (p1[2] + p1[3]));
  // always rescaled: a branch around the accumulator registers makes the compiler spill them when
  // two waves share a SIMD (measured on 8192-token prompts: 150 vs 470 TFLOP/s), and where it does
  // not spill (16 rows per wave) the test costs more than it saves (669 vs 684 TFLOP/s)
#pragma unroll
  for (int b = 0; b < D / 16; ++b) st.o[b] *= alpha;
  const uint2 pa = __builtin_bit_cast(uint2, __builtin_convertvector(p0, bf16x4));
  const uint2 pb = __builtin_bit_cast(uint2, __builtin_convertvector(p1, bf16x4));
  return __builtin_bit_cast(bf16x8, uint4{pa.x, pa.y, pb.x, pb.y});
}
constexpr float kLag = 24.f;     // prefill on bf16 caches: how far (in binary orders) a score may exceed the softmax reference
template <int D, bool FULL>
__device__ inline void pair_pv(WaveState<D>& st, const uint4* vq0, const uint4* vq1, bf16x8 pp, int nvalid) {
  uint4 va[D / 32], vb[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i) { va[i] = vq0[i]; vb[i] = vq1[i]; }
  if (!FULL) {
    const int t0 = 4 * ((threadIdx.x & 63) >> 4);
    const unsigned a01 = (t0 + 0 < nvalid ? 0x0000ffffu : 0u) | (t0 + 1 < nvalid ? 0xffff0000u : 0u);
    const unsigned a23 = (t0 + 2 < nvalid ? 0x0000ffffu : 0u) | (t0 + 3 < nvalid ? 0xffff0000u : 0u);
    const unsigned b01 = (t0 + 16 < nvalid ? 0x0000ffffu : 0u) | (t0 + 17 < nvalid ? 0xffff0000u : 0u);
    const unsigned b23 = (t0 + 18 < nvalid ? 0x0000ffffu : 0u) | (t0 + 19 < nvalid ? 0xffff0000u : 0u);
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      va[i].x &= a01; va[i].y &= a23; va[i].z &= a01; va[i].w &= a23;
      vb[i].x &= b01; vb[i].y &= b23; vb[i].z &= b01; vb[i].w &= b23;
    }
  }
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    const uint4 lo = {va[i].x, va[i].y, vb[i].x, vb[i].y}, hi = {va[i].z, va[i].w, vb[i].z, vb[i].w};
    st.o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lo), pp, st.o[2 * i], 0, 0, 0);
    st.o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, hi), pp, st.o[2 * i + 1], 0, 0, 0);
  }
}
// The same product with the V operands already in the product's layout: lo[i] / hi[i] hold, for
// head-dim slab i, this lane's four tokens of the first page then of the second page, for
// column d % 16 resp. 16 + d % 16 (what loading the two pages' chunks in 8-byte halves gives).
template <int D, bool FULL>
__device__ inline void pair_pv_lohi(WaveState<D>& st, const uint4* lo, const uint4* hi, bf16x8 pp, int nvalid) {
  unsigned a01 = ~0u, a23 = ~0u, b01 = ~0u, b23 = ~0u;
  if (!FULL) {
    const int t0 = 4 * ((threadIdx.x & 63) >> 4);
    a01 = (t0 + 0 < nvalid ? 0x0000ffffu : 0u) | (t0 + 1 < nvalid ? 0xffff0000u : 0u);
    a23 = (t0 + 2 < nvalid ? 0x0000ffffu : 0u) | (t0 + 3 < nvalid ? 0xffff0000u : 0u);
    b01 = (t0 + 16 < nvalid ? 0x0000ffffu : 0u) | (t0 + 17 < nvalid ? 0xffff0000u : 0u);
    b23 = (t0 + 18 < nvalid ? 0x0000ffffu : 0u) | (t0 + 19 < nvalid ? 0xffff0000u : 0u);
  }
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    uint4 l = lo[i], h = hi[i];
    if (!FULL) {
      l.x &= a01; l.y &= a23; l.z &= b01; l.w &= b23;
      h.x &= a01; h.y &= a23; h.z &= b01; h.w &= b23;
    }
    st.o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, l), pp, st.o[2 * i], 0, 0, 0);
    st.o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, h), pp, st.o[2 * i + 1], 0, 0, 0);
  }
}
template <int D, bool FULL, int QSTRIDE>
__device__ inline void process_pair(WaveState<D>& st, const uint4* kq0, const uint4* vq0, const uint4* kq1,
                                    const uint4* vq1, const uint4* qv, int nvalid, int nvalid_row, float scale_log2) {
  f32x4 s0, s1;
  pair_scores<D, QSTRIDE>(kq0, kq1, qv, s0, s1);
  const bf16x8 pp = pair_softmax<D, FULL>(st, s0, s1, nvalid_row, scale_log2);
  pair_pv<D, FULL>(st, vq0, vq1, pp, nvalid);
}

// ---------------------------------------------------------------------------
// Vector-ALU path (any dtype, SART_LAYOUT_NATURAL, any page size, head dim <=
// 256): one wave folds pages [r0, r0 + rn) of `table` into the online-softmax
// state (m, l, o) of one query row; `tokens` = tokens of the sequence the
// table describes (the last page may be partly filled).  Lane holds output
// columns d = lane + 64 c.  Not a tuned path.
// ---------------------------------------------------------------------------
template <typename T> __device__ inline float to_f32(T x);
template <> __device__ inline float to_f32<float>(float x) { return x; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t x) { return __uint_as_float((unsigned)x << 16); }

template <typename T>
__device__ inline void generic_row(const Dims& dm, const T* pool, const int* table, int r0, int rn, int tokens, int h,
                                   const T* qrow, float scale_log2, float& m, float& l, float (&o)[4]) {
  const int lane = threadIdx.x & 63, D = dm.d, pt = dm.pt;
  for (int p = r0; p < r0 + rn; ++p) {
    const int page = table[p];
    const int nvalid = min(pt, tokens - p * pt);
    const long long kb = tile_base(dm, page, h), vb = kb + dm.tile_elems;
    for (int t0 = 0; t0 < nvalid; t0 += 64) {
      const int t = t0 + lane;
      float s = -__builtin_inff();
      if (t < nvalid) {
        float dot = 0.f;
        for (int d = 0; d < D; ++d) dot = fmaf(to_f32<T>(qrow[d]), to_f32<T>(pool[kb + (long long)t * D + d]), dot);
        s = dot * scale_log2;
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
}

}  // namespace sart
