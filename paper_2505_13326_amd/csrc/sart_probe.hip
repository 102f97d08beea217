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
template <int SHAPE>
__global__ void __launch_bounds__(256, 2)
k_mfma_probe(const u32x4* __restrict__ operands, long long iters, float* sink) {
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
  if (shape == 0) hipLaunchKernelGGL(k_mfma_probe<0>, dim3(n_workgroups), dim3(256), 0, s, (const u32x4*)operands, iters, sink);
  else hipLaunchKernelGGL(k_mfma_probe<1>, dim3(n_workgroups), dim3(256), 0, s, (const u32x4*)operands, iters, sink);
}

}  // namespace sart
