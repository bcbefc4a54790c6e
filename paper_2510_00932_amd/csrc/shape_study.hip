// shape_study: the launch shapes that were weighed against each other for the streaming kernels,
// side by side, as one small program that rocprofv3 can profile (every alternative is a kernel of
// its own name, so counters separate them).  It exists to put counter evidence behind the design
// choices of stream_kernels.hpp; the library itself only contains the shapes that won.
//
//   shape_study [log2_n (default 28)] [launches per variant (default 5)]
//
// fp64 only.  Alternatives for Copy and Triad (Table 1):
//   wave64_nt        one 16-byte vector per lane, 64-lane workgroups, non-temporal   (the library's choice)
//   wave64_temporal  same without the non-temporal hint
//   block256_nt      256-lane workgroups
//   block1024_nt     1024-lane workgroups
//   wave64_2vec_nt   two vectors per lane (2 KiB per wavefront)
//   gridstride_nt    persistent: 8 workgroups of 256 lanes per compute unit, 4 vectors per lane per step
// and for Dot:
//   dot_1_per_cu     persistent, one 256-thread workgroup per compute unit               (the library's choice)
//   dot_8_per_cu     persistent, eight per compute unit
//   dot_tile         one tile per workgroup (131072 workgroups)
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "stream_kernels.hpp"

using namespace opal;

#define CHECK(x)                                                                              \
  do {                                                                                        \
    hipError_t e_ = (x);                                                                      \
    if (e_ != hipSuccess) {                                                                   \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
      exit(1);                                                                                \
    }                                                                                         \
  } while (0)

namespace study {

// Two vectors per lane, wave-sized workgroups (what "more bytes in flight per wavefront" costs).
template <Op OP>
__global__ __launch_bounds__(64) void wave64_2vec_nt(double* __restrict__ out, const double* __restrict__ in0,
                                                     const double* __restrict__ in1, double s, size_t nvec) {
  const size_t v0 = (size_t)blockIdx.x * 128 + threadIdx.x;
  d2_t x[2], y[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const size_t v = v0 + u * 64;
    if (v < nvec) {
      x[u] = load16<double, true, true>(in0 + v * 2);
      y[u] = kTwoInputs<OP> ? load16<double, true, true>(in1 + v * 2) : x[u];
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const size_t v = v0 + u * 64;
    if (v < nvec) store16<double, true>(out + v * 2, apply<OP, d2_t>(x[u], y[u], (d2_t)(s)));
  }
}

// Persistent grid-stride: workgroup g takes tiles g, g + G, ... of blockDim.x * 4 vectors.
template <Op OP>
__global__ __launch_bounds__(256) void gridstride_nt(double* __restrict__ out, const double* __restrict__ in0,
                                                     const double* __restrict__ in1, double s, size_t nvec) {
  constexpr int U = 4;
  const size_t tile_vecs = (size_t)blockDim.x * U;
  const size_t tiles = nvec / tile_vecs;     // the study's n is a whole number of tiles
  for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t e0 = wave_uniform(tile * tile_vecs * 2);
    d2_t x[U], y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned e = (threadIdx.x + u * blockDim.x) * 2;
      x[u] = load16<double, true, true>(in0 + e0 + e);
      y[u] = kTwoInputs<OP> ? load16<double, true, true>(in1 + e0 + e) : x[u];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned e = (threadIdx.x + u * blockDim.x) * 2;
      store16<double, true>(out + e0 + e, apply<OP, d2_t>(x[u], y[u], (d2_t)(s)));
    }
  }
}

__global__ void fill(double* p, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.5 + (double)(i & 1023) * 9.765625e-4;
}

}  // namespace study

int main(int argc, char** argv) {
  const int lg = argc > 1 ? atoi(argv[1]) : 28;
  const int launches = argc > 2 ? atoi(argv[2]) : 5;
  if (lg < 16 || lg > 30 || launches < 1) {
    fprintf(stderr, "usage: shape_study [log2_n 16..30] [launches >= 1]\n");
    return 2;
  }
  const size_t n = (size_t)1 << lg, nvec = n / 2, bytes = n * 8, skew = 1024;
  int cus = 0;
  CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  char* pool = nullptr;
  CHECK(hipMalloc(&pool, 3 * (bytes + skew)));
  double* a = (double*)pool;
  double* b = (double*)(pool + bytes + skew);
  double* c = (double*)(pool + 2 * (bytes + skew));
  double *partials = nullptr, *result = nullptr;
  CHECK(hipMalloc(&partials, (size_t)8 << 20));
  CHECK(hipMalloc(&result, 8));
  study::fill<<<4096, 256>>>((double*)pool, 3 * (bytes + skew) / 8);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));

  printf("n = 2^%d fp64, %d compute units, %d launches per variant (median reported)\n", lg, cus, launches);
  printf("%-8s %-18s %12s %10s %8s\n", "kernel", "variant", "time us", "GB/s", "of peak");
  auto timed = [&](const char* kernel, const char* variant, double bytes_moved, auto&& launch) {
    std::vector<float> ms;
    launch();
    for (int i = 0; i < launches; ++i) {
      CHECK(hipEventRecord(e0, 0));
      launch();
      CHECK(hipEventRecord(e1, 0));
      CHECK(hipEventSynchronize(e1));
      float t;
      CHECK(hipEventElapsedTime(&t, e0, e1));
      ms.push_back(t);
    }
    CHECK(hipGetLastError());
    std::sort(ms.begin(), ms.end());
    const double us = ms[ms.size() / 2] * 1e3;
    printf("%-8s %-18s %12.1f %10.0f %7.1f%%\n", kernel, variant, us, bytes_moved / us / 1e3, bytes_moved / us / 1e3 / 80.0);
    fflush(stdout);
  };

  const double s = 0.4;
  const unsigned g64 = (unsigned)((nvec + 63) / 64), g256 = (unsigned)((nvec + 255) / 256),
                 g1024 = (unsigned)((nvec + 1023) / 1024), g2 = (unsigned)((nvec + 127) / 128);
  // Copy: c = a
  timed("copy", "wave64_nt", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 64, true, true><<<g64, 64>>>(c, a, nullptr, s, 0u, nvec, n); });
  timed("copy", "wave64_temporal", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 64, true, false><<<g64, 64>>>(c, a, nullptr, s, 0u, nvec, n); });
  timed("copy", "block256_nt", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 256, true, true><<<g256, 256>>>(c, a, nullptr, s, 0u, nvec, n); });
  timed("copy", "block1024_nt", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 1024, true, true><<<g1024, 1024>>>(c, a, nullptr, s, 0u, nvec, n); });
  timed("copy", "wave64_2vec_nt", 16.0 * n, [&] { study::wave64_2vec_nt<Op::Copy><<<g2, 64>>>(c, a, nullptr, s, nvec); });
  timed("copy", "gridstride_nt", 16.0 * n, [&] { study::gridstride_nt<Op::Copy><<<cus * 8, 256>>>(c, a, nullptr, s, nvec); });
  // Triad: a = b + s * c
  timed("triad", "wave64_nt", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 64, true, true><<<g64, 64>>>(a, b, c, s, 0u, nvec, n); });
  timed("triad", "wave64_temporal", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 64, true, false><<<g64, 64>>>(a, b, c, s, 0u, nvec, n); });
  timed("triad", "block256_nt", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 256, true, true><<<g256, 256>>>(a, b, c, s, 0u, nvec, n); });
  timed("triad", "block1024_nt", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 1024, true, true><<<g1024, 1024>>>(a, b, c, s, 0u, nvec, n); });
  timed("triad", "wave64_2vec_nt", 24.0 * n, [&] { study::wave64_2vec_nt<Op::Triad><<<g2, 64>>>(a, b, c, s, nvec); });
  timed("triad", "gridstride_nt", 24.0 * n, [&] { study::gridstride_nt<Op::Triad><<<cus * 8, 256>>>(a, b, c, s, nvec); });
  // Dot
  const size_t tiles = nvec / (256 * 4);
  auto dot = [&](unsigned groups) {
    const plan::Tiled t = plan::tiled(plan::Split{0u, nvec, 0u}, 256, 4, groups);
    dot_partial_kernel<double, 4, true, true><<<t.groups, 256>>>(a, b, partials, t);
    dot_final_kernel<<<1, 256>>>(partials, t.groups, result);
  };
  timed("dot", "dot_1_per_cu", 16.0 * n, [&] { dot((unsigned)std::min<size_t>(tiles, cus)); });
  timed("dot", "dot_8_per_cu", 16.0 * n, [&] { dot((unsigned)std::min<size_t>(tiles, (size_t)cus * 8)); });
  timed("dot", "dot_tile", 16.0 * n, [&] { dot((unsigned)tiles); });
  CHECK(hipDeviceSynchronize());
  return 0;
}
