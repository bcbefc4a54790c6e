// LDS streaming microkernel for CDNA4 / gfx950 (the analogue of the shared-memory benchmark
// subject in the paper's Table 1; the definition is stated in include/opal.h).
//
// One workgroup per tile of kLdsTileVectors 16-byte vectors.  The tile lives in two LDS
// buffers (2 x 16 KiB); a round reads buffer `cur` with ds_read_b128 at lane-consecutive
// addresses (bank-conflict free), adds c, writes buffer `cur ^ 1` with ds_write_b128, and one
// workgroup barrier separates rounds (the next round only writes the buffer everybody has
// finished reading).  Every value crosses lanes (and, at wavefront borders, wavefronts) each
// round, so nothing can stay in registers: LDS traffic is 32 bytes per vector per round.
// Bound by LDS bandwidth once rep is large; global traffic is one read and one write of the tile.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

#include "stream_kernels.hpp"

namespace opal {

constexpr int kLdsTileVectors = 1024;

// BLOCK threads, V = kLdsTileVectors / BLOCK vectors per thread; thread t owns vectors t, t + BLOCK, ...
template <typename T, int BLOCK>
__global__ __launch_bounds__(BLOCK) void lds_stream_kernel(const T* __restrict__ in, T* __restrict__ out, T c,
                                                           unsigned rep) {
  typedef typename Vec16<T>::type V16;
  constexpr int L = Vec16<T>::lanes;
  constexpr int V = kLdsTileVectors / BLOCK;
  static_assert(kLdsTileVectors % BLOCK == 0, "whole vectors per thread");
  __shared__ V16 buf[2][kLdsTileVectors];
  const unsigned t = threadIdx.x;
  const size_t e0 = wave_uniform((size_t)blockIdx.x * kLdsTileVectors * L);
  const V16 cv = (V16)(c);

#pragma unroll
  for (int u = 0; u < V; ++u) buf[0][t + u * BLOCK] = load16<T, true, false>(in + e0 + (size_t)(t + u * BLOCK) * L);
  __syncthreads();

  unsigned cur = 0;
  for (unsigned r = 0; r < rep; ++r) {
    V16 x[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      unsigned j = t + u * BLOCK + 1;
      if (j == (unsigned)kLdsTileVectors) j = 0;
      x[u] = buf[cur][j];
    }
#pragma unroll
    for (int u = 0; u < V; ++u) buf[cur ^ 1][t + u * BLOCK] = x[u] + cv;
    __syncthreads();
    cur ^= 1;
  }

#pragma unroll
  for (int u = 0; u < V; ++u) store16<T, false>(out + e0 + (size_t)(t + u * BLOCK) * L, buf[cur][t + u * BLOCK]);
}

}  // namespace opal
