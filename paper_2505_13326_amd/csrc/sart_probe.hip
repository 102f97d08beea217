// Measurement aid (not part of the method): plain read kernels over a caller's
// buffer in 8 KiB chunks, sequential or in a given chunk order.  bench.py times
// them to report what fraction of the rate plain reads reach on the same box the
// attention kernel achieves, and sweeps their launch shape (workgroups, chunks in
// flight per wave, load flavour, chunk-to-wave assignment) to find that rate.
// And a matrix-core kernel that does nothing but 32x32x16 bf16 products on operands it holds in registers:
// the rate the matrix cores sustain on this machine for given operand values (the clock follows the power drawn,
// and the power follows the values), which the prefill kernel's rate is reported against.
#include "sart_internal.h"

namespace sart {

constexpr int kProbeChunk = 8192;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// DEPTH chunks (8 KiB each) in flight per wave; NT: loads carry the non-temporal hint.
// interleave = 0: wave w reads a contiguous run of chunks; 1: chunks w, w + n_waves, ...
template <int DEPTH, bool NT>
__global__ void __launch_bounds__(256)
k_read_probe(const u32x4* __restrict__ buf, const int* __restrict__ order, long long n_chunks, int interleave,
             unsigned* sink) {
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long n_waves = ((long long)gridDim.x * blockDim.x) >> 6;
  const long long per = (n_chunks + n_waves - 1) / n_waves;
  const long long first = interleave ? wave : wave * per;
  const long long step = interleave ? n_waves : 1;
  const long long count = interleave ? (wave < n_chunks ? (n_chunks - wave + n_waves - 1) / n_waves : 0)
                                     : (first < n_chunks ? (first + per < n_chunks ? per : n_chunks - first) : 0);
  constexpr int V = kProbeChunk / 1024;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (long long i = 0; i < count; i += DEPTH) {
    u32x4 r[DEPTH][V];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (i + d < count) {
        const long long cc = first + (i + d) * step;
        const long long ci = order ? order[cc] : cc;
        const u32x4* p = buf + ci * (kProbeChunk / 16) + lane;
#pragma unroll
        for (int v = 0; v < V; ++v) r[d][v] = NT ? __builtin_nontemporal_load(p + v * 64) : p[v * 64];
      }
    }
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (i + d < count) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc ^= r[d][v];
      }
    }
  }
  const unsigned s = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (s == 0x12345678u && sink) sink[0] = s;     // keeps the loads alive; never true for the probe's data
}

void launch_read_probe(const void* buf, long long n_chunks, const int* order, int n_workgroups, int depth, int flavour,
                       int interleave, hipStream_t s) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(n_workgroups), dim3(256), 0, s, (const u32x4*)buf, order, n_chunks, interleave,
                       (unsigned*)nullptr);
  };
  const bool nt = flavour == 1;
  switch (depth) {
    case 1: if (nt) go(k_read_probe<1, true>); else go(k_read_probe<1, false>); break;
    case 2: if (nt) go(k_read_probe<2, true>); else go(k_read_probe<2, false>); break;
    case 8: if (nt) go(k_read_probe<8, true>); else go(k_read_probe<8, false>); break;
    default: if (nt) go(k_read_probe<4, true>); else go(k_read_probe<4, false>); break;
  }
}

// Every wave: 8 A and 8 B operands (16 bytes per lane each) from `operands` (the same 16 KiB for every wave),
// then `iters` rounds of 524288 flops.  SHAPE 0: 16 products 32x32x16, 8 into one accumulator (a dependent
// chain, as a score tile over head_dim 128) and 8 into four others (as an output tile): the prefill kernel's
// own sequence with everything but the products taken out.  SHAPE 1: 32 products 16x16x32 into 8
// accumulators in turn.  Nothing else: no loads, no LDS, no vector work.
typedef __bf16 pbf16x8 __attribute__((ext_vector_type(8)));
typedef float pf32x16 __attribute__((ext_vector_type(16)));
typedef float pf32x4 __attribute__((ext_vector_type(4)));
typedef float pf32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 pbf16x2 __attribute__((ext_vector_type(2)));
template <int SHAPE>
__global__ void __launch_bounds__(256, 2)
k_mfma_probe(const u32x4* __restrict__ operands, long long iters, float scale, float* sink) {
  const int lane = threadIdx.x & 63;
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = operands[i * 64 + lane];
    b[i] = operands[(8 + i) * 64 + lane];
  }
  float t = 0.f;
  if constexpr (SHAPE == 0) {
    pf32x16 s, o[4];
#pragma unroll
    for (int e = 0; e < 16; ++e) { s[e] = 0.f; o[0][e] = o[1][e] = o[2][e] = o[3][e] = 0.f; }
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pbf16x8, a[i]), __builtin_bit_cast(pbf16x8, b[i]), s, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pbf16x8, b[i]), __builtin_bit_cast(pbf16x8, a[(i + 3) & 7]), o[i & 3], 0, 0, 0);
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) t += s[e] + o[0][e] + o[1][e] + o[2][e] + o[3][e];
  } else if constexpr (SHAPE == 2) {
    pf32x4 o[2][8];
    float m_ref[2] = {4.f, 4.f}, lsum[2] = {0.f, 0.f};
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int j = 0; j < 8; ++j) o[blk][j] = pf32x4{0.f, 0.f, 0.f, 0.f};
    for (long long it = 0; it < iters; ++it) {
      pf32x4 sc[2][2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) sc[blk][0] = sc[blk][1] = pf32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk)
            sc[blk][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pbf16x8, a[p * 4 + i]), __builtin_bit_cast(pbf16x8, b[blk * 4 + i]), sc[blk][p], 0, 0, 0);
      float mine[2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
        mine[blk] = fmaxf(fmaxf(fmaxf(sc[blk][0][0], sc[blk][0][1]), fmaxf(sc[blk][0][2], sc[blk][0][3])),
                          fmaxf(fmaxf(sc[blk][1][0], sc[blk][1][1]), fmaxf(sc[blk][1][2], sc[blk][1][3])));
      if (__any(mine[0] * scale > m_ref[0] + 24.f || mine[1] * scale > m_ref[1] + 24.f)) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          const float m_new = fmaxf(m_ref[blk], mine[blk] * scale), alpha = __builtin_amdgcn_exp2f(m_ref[blk] - m_new);
          m_ref[blk] = m_new;
          lsum[blk] *= alpha;
#pragma unroll
          for (int j = 0; j < 8; ++j) o[blk][j] *= alpha;
        }
      }
      u32x4 pp[2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        unsigned pk[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[blk][w >> 1][2 * (w & 1)], scale, -m_ref[blk]));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[blk][w >> 1][2 * (w & 1) + 1], scale, -m_ref[blk]));
          const pbf16x2 pb = __builtin_convertvector(pf32x2{p0, p1}, pbf16x2);
          pk[w] = __builtin_bit_cast(unsigned, pb);
          lsum[blk] = __builtin_amdgcn_fdot2_f32_bf16(pb, __builtin_bit_cast(pbf16x2, 0x3f803f80u), lsum[blk], false);
        }
        pp[blk] = u32x4{pk[0], pk[1], pk[2], pk[3]};
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
          o[blk][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pbf16x8, a[(j + 3) & 7]), __builtin_bit_cast(pbf16x8, pp[blk]), o[blk][j], 0, 0, 0);
    }
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      t += lsum[blk];
#pragma unroll
      for (int j = 0; j < 8; ++j) t += o[blk][j][0] + o[blk][j][1] + o[blk][j][2] + o[blk][j][3];
    }
  } else {
    pf32x4 o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = pf32x4{0.f, 0.f, 0.f, 0.f};
    for (long long it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 32; ++i)
        o[i & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(pbf16x8, a[i & 7]), __builtin_bit_cast(pbf16x8, b[(i + (i >> 3)) & 7]), o[i & 7], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) t += o[j][0] + o[j][1] + o[j][2] + o[j][3];
  }
  if (sink) sink[(long long)blockIdx.x * blockDim.x + threadIdx.x] = t;
}

void launch_mfma_probe(const void* operands, long long iters, int n_workgroups, int shape, float* sink, hipStream_t s) {
  const float scale = 0.1275174f;   // log2(e) / sqrt(128): what a head_dim of 128 multiplies its scores by
  auto go = [&](auto kern) { hipLaunchKernelGGL(kern, dim3(n_workgroups), dim3(256), 0, s, (const u32x4*)operands, iters, scale, sink); };
  if (shape == 0) go(k_mfma_probe<0>); else if (shape == 1) go(k_mfma_probe<1>); else go(k_mfma_probe<2>);
}

}  // namespace sart
