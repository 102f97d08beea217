// Measurement aid (not part of the method): plain read kernels over a caller's
// buffer in 8 KiB chunks, sequential or in a given chunk order.  bench.py times
// them to report what fraction of the rate plain reads reach on the same box the
// attention kernel achieves, and sweeps their launch shape (workgroups, chunks in
// flight per wave, load flavour, chunk-to-wave assignment) to find that rate.
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

}  // namespace sart
