// shape_study: the launch shapes that were weighed against each other for the streaming kernels, and
// the ceilings they are measured against, side by side, as one small program that rocprofv3 can
// profile (every alternative is a kernel of its own name, so counters separate them).  It exists to
// put counter evidence behind the design choices of stream_kernels.hpp / pacing.hpp; the library
// itself only contains the shapes that won.
//
//   shape_study [log2_n (default 28)] [launches per variant (default 9)] [group: all|ceilings|copy|triad|dot|lds]
//
// fp64 only.
// Ceilings (kernels that only read or only write):
//   read1_ordered    one array, one 16-byte vector per lane, 64-lane workgroups in index order
//   read1_tiled      one array, persistent: one 256-thread workgroup per compute unit, 8 vectors per lane per tile
//   read2_tiled      two arrays, 4 vectors of each per lane per tile (what a dot has to read)
//   read2_paced      two arrays, persistent wavefronts on the clock timetable (the library's dot, first pass)
//   write_ordered    one array written, 64-lane workgroups in index order
//   write_tiled      one array written, persistent
//   pair             read1_ordered of `a` on one stream while write_ordered of `c` runs on another:
//                    what a 1:1 read/write mix reaches when reads and writes are not coupled in one wavefront
// Copy and Triad (Table 1):
//   wave64_nt        one vector per lane, 64-lane workgroups in index order, non-temporal (the library's shape below the paced threshold)
//   wave64_temporal  same without the non-temporal hint
//   block256_nt      256-lane workgroups
//   wave64_2vec_nt   two vectors per lane
//   gridstride_nt    persistent: 8 workgroups of 256 lanes per compute unit, 4 vectors per lane per step
//   burst            persistent wavefronts, K loads then K stores, no timetable (K = 8 / 4, 2048 wavefronts)
//   paced_open       the same on the clock timetable, no feedback
//   paced_mixed      timetable and feedback, but every compute unit hosts both sets
//   paced            timetable with feedback, whole compute units per set (the library's shape for large arrays)
// Dot:
//   dot_1_per_cu     tiled, one 256-thread workgroup per compute unit (the library's shape below the paced threshold)
//   dot_8_per_cu     tiled, eight per compute unit
//   dot_tile         one tile per workgroup
//   dot_paced        the library's shape for large arrays
// LDS (group lds, not part of `all`; log2_n is ignored: 10240 tiles of 1024 vectors, 600 rounds, as the LDS bench):
//   lds_stream       the library's LDS kernel: per round one 16-byte read and one 16-byte write per vector
//   lds_stream_128, _512, _1024   the same with other workgroup sizes (the library uses 256)
//   lds_mixed        the same rounds in this file's kernel, which also reads the clocks
//   lds_read         the reads of a round only (same tile, same launch, same barrier per round)
//   lds_write        the writes of a round only
//   lds_write_b64, lds_write_b32   the same bytes written as 8-byte and 4-byte stores per lane
//   lds_read2, lds_write2   twice the reads (writes) per round and barrier: both buffers
//   clocks           what the two wave-readable counters count, and a chain of dependent fp32 adds per SIMD
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "launch_shapes.hpp"
#include "lds_kernel.hpp"
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

// A load must feed something the compiler cannot drop: a store that never happens.
__device__ __forceinline__ void keep(d2_t x, double* sink) {
  if (x[0] == -1.2345e300) sink[0] = x[1];
}

__global__ __launch_bounds__(64) void read1_ordered(const double* __restrict__ a, double* __restrict__ sink) {
  const size_t e0 = wave_uniform((size_t)blockIdx.x * 128);
  keep(load16<double, true, true>(a + e0 + threadIdx.x * 2), sink);
}

__global__ __launch_bounds__(64) void write_ordered(double* __restrict__ c, double v) {
  const size_t e0 = wave_uniform((size_t)blockIdx.x * 128);
  store16<double, true>(c + e0 + threadIdx.x * 2, d2_t{v, v});
}

// Persistent: workgroup g takes tiles g, g + G, ... of blockDim.x * U vectors; U * STREAMS = 8 loads in
// flight per lane (32 KiB per compute unit) in both cases.
template <int STREAMS>
__global__ __launch_bounds__(256) void read_tiled(const double* __restrict__ a, const double* __restrict__ b,
                                                  double* __restrict__ sink, size_t nvec) {
  constexpr int U = 8 / STREAMS;
  const size_t tile_vecs = (size_t)blockDim.x * U;
  const size_t tiles = nvec / tile_vecs;
  d2_t acc = {0.0, 0.0};
  for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t e0 = wave_uniform(tile * tile_vecs * 2);
    d2_t x[U], y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned e = (threadIdx.x + u * blockDim.x) * 2;
      x[u] = load16<double, true, true>(a + e0 + e);
      y[u] = STREAMS == 2 ? load16<double, true, true>(b + e0 + e) : x[u];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) acc += x[u] * y[u];
  }
  keep(acc, sink);
}

__global__ __launch_bounds__(256) void write_tiled(double* __restrict__ c, double v, size_t nvec) {
  constexpr int U = 8;
  const size_t tile_vecs = (size_t)blockDim.x * U;
  const size_t tiles = nvec / tile_vecs;
  for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t e0 = wave_uniform(tile * tile_vecs * 2);
#pragma unroll
    for (int u = 0; u < U; ++u) store16<double, true>(c + e0 + (threadIdx.x + u * blockDim.x) * 2, d2_t{v, v});
  }
}

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

// The library's paced kernels under names of their own per variant, so that profiles tell them apart.
template <Op OP, int K, int VARIANT>
__global__ __launch_bounds__(64) void paced_variant(double* out, const double* in0, const double* in1, double s,
                                                    plan::Paced p, Pace pace) {
  paced_stream_body<double, OP, K, true>(out, in0, in1, s, p, pace);
}

// The rounds of lds_stream_kernel, whole (MODE 0), reads only (1) or writes only (2): same tile, same
// workgroup, one barrier per round.  TWICE: the reads (writes) of a round go to both buffers, which
// halves the barriers per byte (modes 1 and 2 only).  Thread 0 of every workgroup notes how far the shader clock
// counter (s_memtime) and the constant-rate counter (s_memrealtime) advance over the rounds.
template <int MODE, bool TWICE = false>
__global__ __launch_bounds__(256) void lds_rounds(const double* __restrict__ in, double* __restrict__ out, double c,
                                                  unsigned rep, unsigned long long* __restrict__ ticks) {
  constexpr int BLOCK = 256, V = kLdsTileVectors / BLOCK;
  __shared__ d2_t buf[2][kLdsTileVectors];
  const unsigned t = threadIdx.x;
  const size_t e0 = (size_t)blockIdx.x * kLdsTileVectors * 2;
  const d2_t cv = (d2_t)(c);
#pragma unroll
  for (int u = 0; u < V; ++u) {
    const d2_t v = load16<double, true, false>(in + e0 + (size_t)(t + u * BLOCK) * 2);
    buf[0][t + u * BLOCK] = v;
    buf[1][t + u * BLOCK] = v;
  }
  __syncthreads();
  const unsigned long long m0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  unsigned cur = 0;
  d2_t x[V];
#pragma unroll
  for (int u = 0; u < V; ++u) x[u] = cv;
  for (unsigned r = 0; r < rep; ++r) {
    if (MODE != 2) {
      d2_t y[V];
#pragma unroll
      for (int u = 0; u < V; ++u) {
        unsigned j = t + u * BLOCK + 1;
        if (j == (unsigned)kLdsTileVectors) j = 0;
        y[u] = buf[cur][j];
      }
#pragma unroll
      for (int u = 0; u < V; ++u) x[u] = MODE == 0 ? y[u] + cv : x[u] + y[u];
      if (MODE == 1 && TWICE) {
#pragma unroll
        for (int u = 0; u < V; ++u) {
          unsigned j = t + u * BLOCK + 1;
          if (j == (unsigned)kLdsTileVectors) j = 0;
          y[u] = buf[cur ^ 1][j];
        }
#pragma unroll
        for (int u = 0; u < V; ++u) x[u] += y[u];
      }
    } else {
#pragma unroll
      for (int u = 0; u < V; ++u) x[u] += cv;
    }
    if (MODE != 1) {
#pragma unroll
      for (int u = 0; u < V; ++u) buf[cur ^ 1][t + u * BLOCK] = x[u];
      if (MODE == 2 && TWICE) {
#pragma unroll
        for (int u = 0; u < V; ++u) buf[cur][t + u * BLOCK] = x[u] + cv;
      }
    }
    __syncthreads();
    cur ^= 1;
  }
  const unsigned long long m1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  if (t == 0) {
    ticks[2 * blockIdx.x] = m1 - m0;
    ticks[2 * blockIdx.x + 1] = r1 - r0;
  }
#pragma unroll
  for (int u = 0; u < V; ++u)
    store16<double, false>(out + e0 + (size_t)(t + u * BLOCK) * 2, MODE == 1 ? x[u] : buf[cur][t + u * BLOCK]);
}

// Writes only, in pieces of W bytes per lane (8 or 4) at lane-consecutive addresses: the same 16 KiB per
// round and barrier as lds_rounds<2>, as 2 or 4 times as many narrower stores.
template <typename E>
__global__ __launch_bounds__(256) void lds_write_narrow(const double* __restrict__ in, double* __restrict__ out, double c,
                                                        unsigned rep, unsigned long long* __restrict__ ticks) {
  constexpr int BLOCK = 256, N = kLdsTileVectors * 16 / sizeof(E), V = N / BLOCK;
  __shared__ E buf[2][N];
  const unsigned t = threadIdx.x;
  const size_t e0 = (size_t)blockIdx.x * kLdsTileVectors * 2;
  E x[V];
#pragma unroll
  for (int u = 0; u < V; ++u) {
    x[u] = (E)in[e0 + (t + u * BLOCK) % (kLdsTileVectors * 2)];
    buf[0][t + u * BLOCK] = x[u];
    buf[1][t + u * BLOCK] = x[u];
  }
  __syncthreads();
  const unsigned long long m0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  unsigned cur = 0;
  for (unsigned r = 0; r < rep; ++r) {
#pragma unroll
    for (int u = 0; u < V; ++u) x[u] += (E)c;
#pragma unroll
    for (int u = 0; u < V; ++u) buf[cur ^ 1][t + u * BLOCK] = x[u];
    __syncthreads();
    cur ^= 1;
  }
  const unsigned long long m1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  if (t == 0) {
    ticks[2 * blockIdx.x] = m1 - m0;
    ticks[2 * blockIdx.x + 1] = r1 - r0;
  }
  double sum = 0;
#pragma unroll
  for (int u = 0; u < V; ++u) sum += (double)buf[cur][t + u * BLOCK];
  out[e0 + t] = sum;
}

// One wavefront per SIMD (256-thread workgroups, one per compute unit) runs `ops` dependent fp32 adds.
__global__ __launch_bounds__(256) void add_chain(float* __restrict__ out, float c, unsigned ops,
                                                 unsigned long long* __restrict__ ticks) {
  float x = (float)threadIdx.x;
  const unsigned long long m0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (unsigned i = 0; i < ops; i += 16) {
#pragma unroll
    for (int k = 0; k < 16; ++k) asm volatile("v_add_f32 %0, %0, %1" : "+v"(x) : "v"(c));
  }
  const unsigned long long m1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  if (threadIdx.x == 0) {
    ticks[2 * blockIdx.x] = m1 - m0;
    ticks[2 * blockIdx.x + 1] = r1 - r0;
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = x;
}

__global__ void fill(double* p, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.5 + (double)(i & 1023) * 9.765625e-4;
}

}  // namespace study

static Pace make_pace(const PacedShape& sh, unsigned streams, bool timetable, bool feedback, unsigned long long* words) {
  Pace pace{};
  if (!timetable) return pace;   // period 0: no clock use at all
  const double bytes = (double)sh.waves * sh.k * 1024.0 * streams;
  pace.period = (uint32_t)(bytes / sh.bytes_per_us * 100.0 + 0.5);   // 100 ticks per microsecond
  pace.second_input = (uint32_t)(sh.second_input_at * pace.period);
  pace.store = (uint32_t)(sh.store_at * pace.period);
  pace.gap = (uint32_t)(sh.gap * pace.period);
  pace.tolerance = sh.tolerance;
  pace.feedback = feedback ? words : nullptr;
  return pace;
}

// LDS rates in bytes per clock per compute unit, against the two clocks a wave can read.
static int lds_study(int launches) {
  const unsigned tiles = 10240, rep = 600;
  const size_t n = (size_t)tiles * kLdsTileVectors * 2;
  int cus = 0, khz = 0;
  CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  CHECK(hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, 0));
  double *in = nullptr, *out = nullptr;
  unsigned long long* ticks = nullptr;
  CHECK(hipMalloc(&in, n * 8));
  CHECK(hipMalloc(&out, n * 8));
  CHECK(hipMalloc(&ticks, (size_t)tiles * 16));
  study::fill<<<4096, 256>>>(in, n);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  std::vector<unsigned long long> host((size_t)tiles * 2);
  printf("LDS: %u tiles of %d vectors, %u rounds, %d compute units, reported clock %.0f MHz, %d launches per variant\n",
         tiles, kLdsTileVectors, rep, cus, khz / 1e3, launches);
  printf("%-16s %10s %10s %12s %14s %16s\n", "variant", "median us", "LDS GB/s", "B/clk/CU at", "s_memtime per", "B per s_memtime");
  printf("%-16s %10s %10s %12s %14s %16s\n", "", "", "", "reported clk", "s_memrealtime", "tick per CU");
  auto run = [&](const char* name, double bytes_per_vector_round, unsigned groups, auto&& launch) {
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
    const double total = bytes_per_vector_round * tiles * (double)kLdsTileVectors * rep;
    double ratio = 0, per_tick = 0;
    if (groups) {
      CHECK(hipMemcpy(host.data(), ticks, (size_t)groups * 16, hipMemcpyDeviceToHost));
      double m = 0, r = 0;
      for (unsigned g = 0; g < groups; ++g) {
        m += (double)host[2 * g];
        r += (double)host[2 * g + 1];
      }
      ratio = m / r;
      // s_memtime ticks of the whole launch = ratio * (100 ticks per us) * us
      per_tick = total / (ratio * 100.0 * us) / cus;
    }
    if (groups)
      printf("%-16s %10.1f %10.0f %12.1f %14.3f %16.1f\n", name, us, total / us / 1e3, total / us / 1e3 / (khz / 1e6) / cus,
             ratio, per_tick);
    else
      printf("%-16s %10.1f %10.0f %12.1f %14s %16s\n", name, us, total / us / 1e3, total / us / 1e3 / (khz / 1e6) / cus, "-", "-");
    fflush(stdout);
  };
  run("lds_stream", 32.0, 0, [&] { lds_stream_kernel<double, 256><<<tiles, 256>>>(in, out, 0.5, rep); });
  run("lds_stream_128", 32.0, 0, [&] { lds_stream_kernel<double, 128><<<tiles, 128>>>(in, out, 0.5, rep); });
  run("lds_stream_512", 32.0, 0, [&] { lds_stream_kernel<double, 512><<<tiles, 512>>>(in, out, 0.5, rep); });
  run("lds_stream_1024", 32.0, 0, [&] { lds_stream_kernel<double, 1024><<<tiles, 1024>>>(in, out, 0.5, rep); });
  run("lds_mixed", 32.0, tiles, [&] { study::lds_rounds<0><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_read", 16.0, tiles, [&] { study::lds_rounds<1><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_write", 16.0, tiles, [&] { study::lds_rounds<2><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_write_b64", 16.0, tiles, [&] { study::lds_write_narrow<double><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_write_b32", 16.0, tiles, [&] { study::lds_write_narrow<float><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_read2", 32.0, tiles, [&] { study::lds_rounds<1, true><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  run("lds_write2", 32.0, tiles, [&] { study::lds_rounds<2, true><<<tiles, 256>>>(in, out, 0.5, rep, ticks); });
  // clocks: `ops` dependent fp32 adds on one wavefront per SIMD
  const unsigned ops = 1u << 20;
  float* fout = nullptr;
  CHECK(hipMalloc(&fout, (size_t)cus * 256 * 4));
  std::vector<float> ms;
  for (int i = 0; i < launches + 1; ++i) {
    CHECK(hipEventRecord(e0, 0));
    study::add_chain<<<cus, 256>>>(fout, 1.0f, ops, ticks);
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float t;
    CHECK(hipEventElapsedTime(&t, e0, e1));
    if (i) ms.push_back(t);
  }
  CHECK(hipGetLastError());
  std::sort(ms.begin(), ms.end());
  CHECK(hipMemcpy(host.data(), ticks, (size_t)cus * 16, hipMemcpyDeviceToHost));
  double m = 0, r = 0;
  for (int g = 0; g < cus; ++g) {
    m += (double)host[2 * g];
    r += (double)host[2 * g + 1];
  }
  printf("clocks: a chain of %u dependent fp32 adds (one wavefront per SIMD) takes %.1f us by events, %.0f s_memrealtime ticks "
         "and %.0f s_memtime ticks per wavefront: %.3f s_memtime ticks per add, %.3f s_memtime per s_memrealtime tick "
         "(s_memrealtime counts at 100 MHz)\n",
         ops, ms[ms.size() / 2] * 1e3, r / cus, m / cus, m / cus / ops, m / r);
  CHECK(hipDeviceSynchronize());
  return 0;
}

int main(int argc, char** argv) {
  const int lg = argc > 1 ? atoi(argv[1]) : 28;
  const int launches = argc > 2 ? atoi(argv[2]) : 9;
  const char* group = argc > 3 ? argv[3] : "all";
  if (lg < 24 || lg > 30 || launches < 1) {
    fprintf(stderr, "usage: shape_study [log2_n 24..30] [launches >= 1] [all|ceilings|copy|triad|dot|lds]\n");
    return 2;
  }
  if (!strcmp(group, "lds")) return lds_study(launches);
  auto want = [&](const char* g) { return !strcmp(group, "all") || !strcmp(group, g); };
  const size_t n = (size_t)1 << lg, nvec = n / 2, bytes = n * 8, skew = 1024;
  int cus = 0;
  CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  char* pool = nullptr;
  CHECK(hipMalloc(&pool, 3 * (bytes + skew)));
  double* a = (double*)pool;
  double* b = (double*)(pool + bytes + skew);
  double* c = (double*)(pool + 2 * (bytes + skew));
  double *partials = nullptr, *result = nullptr;
  unsigned long long* words = nullptr;
  CHECK(hipMalloc(&partials, (size_t)8 << 20));
  CHECK(hipMalloc(&result, 8));
  CHECK(hipMalloc(&words, kFeedbackWords * 8));
  CHECK(hipMemset(words, 0, kFeedbackWords * 8));
  study::fill<<<4096, 256>>>((double*)pool, 3 * (bytes + skew) / 8);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1, e2;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  CHECK(hipEventCreate(&e2));
  hipStream_t sa, sb;
  CHECK(hipStreamCreate(&sa));
  CHECK(hipStreamCreate(&sb));

  printf("n = 2^%d fp64, %d compute units, %d launches per variant\n", lg, cus, launches);
  printf("%-8s %-16s %10s %10s %8s %8s %10s\n", "kernel", "variant", "median us", "GB/s", "of peak", "mean", "max us");
  auto report = [&](const char* kernel, const char* variant, double bytes_moved, std::vector<float>& ms) {
    double mean = 0;
    for (float t : ms) mean += t;
    mean /= ms.size();
    std::sort(ms.begin(), ms.end());
    const double us = ms[ms.size() / 2] * 1e3;
    printf("%-8s %-16s %10.1f %10.0f %7.1f%% %7.1f%% %10.1f\n", kernel, variant, us, bytes_moved / us / 1e3,
           bytes_moved / us / 1e3 / 80.0, bytes_moved / (mean * 1e3) / 1e3 / 80.0, ms.back() * 1e3);
    fflush(stdout);
  };
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
    report(kernel, variant, bytes_moved, ms);
  };

  const double s = 0.4;
  const unsigned g64 = (unsigned)((nvec + 63) / 64), g256 = (unsigned)((nvec + 255) / 256),
                 g2 = (unsigned)((nvec + 127) / 128);
  const plan::Split whole{0u, nvec, 0u};

  if (want("ceilings")) {
    timed("read", "read1_ordered", 8.0 * n, [&] { study::read1_ordered<<<g64, 64>>>(a, result); });
    timed("read", "read1_tiled", 8.0 * n, [&] { study::read_tiled<1><<<cus, 256>>>(a, b, result, nvec); });
    timed("read", "read2_tiled", 16.0 * n, [&] { study::read_tiled<2><<<cus, 256>>>(a, b, result, nvec); });
    {
      const plan::Paced p = plan::paced(whole, kPacedDot.waves, kPacedKDot, kPacedDot.set_bit);
      const Pace pace = make_pace(kPacedDot, 2, true, false, words);
      timed("read", "read2_paced", 16.0 * n, [&] { paced_dot_kernel<double, kPacedKDot, true><<<kPacedDot.waves, 64>>>(a, b, partials, p, pace); });
    }
    timed("write", "write_ordered", 8.0 * n, [&] { study::write_ordered<<<g64, 64>>>(c, 1.5); });
    timed("write", "write_tiled", 8.0 * n, [&] { study::write_tiled<<<cus, 256>>>(c, 1.5, nvec); });
    // a read-only and a write-only kernel at the same time, on two streams of equal priority
    std::vector<float> ms;
    for (int i = 0; i < launches + 1; ++i) {
      CHECK(hipDeviceSynchronize());
      CHECK(hipEventRecord(e0, sa));
      CHECK(hipStreamWaitEvent(sb, e0, 0));
      study::read1_ordered<<<g64, 64, 0, sa>>>(a, result);
      study::write_ordered<<<g64, 64, 0, sb>>>(c, 1.5);
      CHECK(hipEventRecord(e1, sa));
      CHECK(hipEventRecord(e2, sb));
      CHECK(hipEventSynchronize(e1));
      CHECK(hipEventSynchronize(e2));
      float ta, tb;
      CHECK(hipEventElapsedTime(&ta, e0, e1));
      CHECK(hipEventElapsedTime(&tb, e0, e2));
      if (i) ms.push_back(std::max(ta, tb));
    }
    report("1R:1W", "pair", 16.0 * n, ms);
    CHECK(hipDeviceSynchronize());
    study::fill<<<4096, 256>>>((double*)pool, 3 * (bytes + skew) / 8);
    CHECK(hipDeviceSynchronize());
  }

  if (want("copy")) {
    timed("copy", "wave64_nt", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 64, true, true><<<g64, 64>>>(c, a, nullptr, s, 0u, nvec, n); });
    timed("copy", "wave64_temporal", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 64, true, false><<<g64, 64>>>(c, a, nullptr, s, 0u, nvec, n); });
    timed("copy", "block256_nt", 16.0 * n, [&] { stream_kernel<double, Op::Copy, 256, true, true><<<g256, 256>>>(c, a, nullptr, s, 0u, nvec, n); });
    timed("copy", "wave64_2vec_nt", 16.0 * n, [&] { study::wave64_2vec_nt<Op::Copy><<<g2, 64>>>(c, a, nullptr, s, nvec); });
    timed("copy", "gridstride_nt", 16.0 * n, [&] { study::gridstride_nt<Op::Copy><<<cus * 8, 256>>>(c, a, nullptr, s, nvec); });
    const PacedShape sh = kPacedOneInput;
    const plan::Paced p = plan::paced(whole, sh.waves, kPacedK1, sh.set_bit);
    const plan::Paced pmixed = plan::paced(whole, sh.waves, kPacedK1, 8);
    const Pace none = make_pace(sh, 2, false, false, words), open = make_pace(sh, 2, true, false, words),
               closed = make_pace(sh, 2, true, true, words);
    timed("copy", "burst", 16.0 * n, [&] { study::paced_variant<Op::Copy, kPacedK1, 0><<<sh.waves, 64>>>(c, a, nullptr, s, p, none); });
    timed("copy", "paced_open", 16.0 * n, [&] { study::paced_variant<Op::Copy, kPacedK1, 1><<<sh.waves, 64>>>(c, a, nullptr, s, p, open); });
    timed("copy", "paced_mixed", 16.0 * n, [&] { study::paced_variant<Op::Copy, kPacedK1, 2><<<sh.waves, 64>>>(c, a, nullptr, s, pmixed, closed); });
    timed("copy", "paced", 16.0 * n, [&] { paced_stream_kernel<double, Op::Copy, kPacedK1, true><<<sh.waves, 64>>>(c, a, nullptr, s, p, closed); });
  }

  if (want("triad")) {
    timed("triad", "wave64_nt", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 64, true, true><<<g64, 64>>>(a, b, c, s, 0u, nvec, n); });
    timed("triad", "wave64_temporal", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 64, true, false><<<g64, 64>>>(a, b, c, s, 0u, nvec, n); });
    timed("triad", "block256_nt", 24.0 * n, [&] { stream_kernel<double, Op::Triad, 256, true, true><<<g256, 256>>>(a, b, c, s, 0u, nvec, n); });
    timed("triad", "wave64_2vec_nt", 24.0 * n, [&] { study::wave64_2vec_nt<Op::Triad><<<g2, 64>>>(a, b, c, s, nvec); });
    timed("triad", "gridstride_nt", 24.0 * n, [&] { study::gridstride_nt<Op::Triad><<<cus * 8, 256>>>(a, b, c, s, nvec); });
    const PacedShape sh = kPacedTwoInputs;
    const plan::Paced p = plan::paced(whole, sh.waves, kPacedK2, sh.set_bit);
    const plan::Paced pmixed = plan::paced(whole, sh.waves, kPacedK2, 8);
    const Pace none = make_pace(sh, 3, false, false, words), open = make_pace(sh, 3, true, false, words),
               closed = make_pace(sh, 3, true, true, words);
    timed("triad", "burst", 24.0 * n, [&] { study::paced_variant<Op::Triad, kPacedK2, 0><<<sh.waves, 64>>>(a, b, c, s, p, none); });
    timed("triad", "paced_open", 24.0 * n, [&] { study::paced_variant<Op::Triad, kPacedK2, 1><<<sh.waves, 64>>>(a, b, c, s, p, open); });
    timed("triad", "paced_mixed", 24.0 * n, [&] { study::paced_variant<Op::Triad, kPacedK2, 2><<<sh.waves, 64>>>(a, b, c, s, pmixed, closed); });
    timed("triad", "paced", 24.0 * n, [&] { paced_stream_kernel<double, Op::Triad, kPacedK2, true><<<sh.waves, 64>>>(a, b, c, s, p, closed); });
  }

  if (want("dot")) {
    auto dot = [&](unsigned groups) {
      const plan::Tiled t = plan::tiled(whole, 256, 4, groups);
      dot_partial_kernel<double, 4, true, true><<<t.groups, 256>>>(a, b, partials, t);
      dot_final_kernel<<<1, 256>>>(partials, t.groups, result);
    };
    const size_t tiles = nvec / (256 * 4);
    timed("dot", "dot_1_per_cu", 16.0 * n, [&] { dot((unsigned)std::min<size_t>(tiles, cus)); });
    timed("dot", "dot_8_per_cu", 16.0 * n, [&] { dot((unsigned)std::min<size_t>(tiles, (size_t)cus * 8)); });
    timed("dot", "dot_tile", 16.0 * n, [&] { dot((unsigned)tiles); });
    const plan::Paced p = plan::paced(whole, kPacedDot.waves, kPacedKDot, kPacedDot.set_bit);
    const Pace pace = make_pace(kPacedDot, 2, true, false, words);
    timed("dot", "dot_paced", 16.0 * n, [&] {
      paced_dot_kernel<double, kPacedKDot, true><<<kPacedDot.waves, 64>>>(a, b, partials, p, pace);
      dot_final_kernel<<<1, 256>>>(partials, kPacedDot.waves, result);
    });
  }
  CHECK(hipDeviceSynchronize());
  return 0;
}
