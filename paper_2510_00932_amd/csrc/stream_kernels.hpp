// Device code for the five streaming vector kernels (Table 1: Copy, Mul, Add,
// Triad, Dot), written for CDNA4 / gfx950 only: 64-lane wavefronts, 128-bit
// non-temporal global loads and stores, no LDS on the elementwise path, DPP
// lane exchanges for the dot reduction.  Nothing here is a contraction, so no
// MFMA.
//
// Work split (done on the host, same for all kernels)
//   An array of n elements is cut into
//     head : scalar elements up to the first 1 KiB boundary of the array that
//            steers the split (the output; for dot, `a`), so that every
//            wavefront's 1 KiB run is one aligned DRAM interleave unit
//            (a body that starts 128 or 256 bytes off costs about 1 %)
//     body : nvec 16-byte vectors (double2 / float4)
//     tail : the < one-vector remainder.
//
// Elementwise kernels: one vector per lane, one wavefront per workgroup
//   Workgroup g moves vectors 64g .. 64g+63: one contiguous 1 KiB run per
//   array.  Nothing loops.  The hardware dispatcher hands workgroups out in
//   index order to whichever wavefront slot frees up, so at any moment the
//   whole chip works inside one narrow window that slides through each array
//   (few DRAM pages and TLB entries live at a time), consecutive 1 KiB runs go
//   to different XCDs, and no software schedule can drift.  Measured on
//   MI355X this beats every persistent / grid-stride shape tried (256-1024
//   threads, 1-8 vectors per lane, 1-16 workgroups per CU) by 3-20 %; more
//   than one vector in flight per lane lowers the bandwidth.
//   The last workgroup also moves the head and tail scalars.
//   Arrays small enough to stay in the 256 MB Infinity Cache from one kernel to
//   the next (a few million elements: the regime where the dispatch rate of
//   wave-sized workgroups, about 4.7 per ns, becomes the floor) use the same
//   kernel with 256 lanes per workgroup and without the non-temporal hint.
//
// Paced kernels (arrays far larger than the caches): persistent wavefronts on a timetable
//   `waves` one-wavefront workgroups in two sets; the full 1 KiB runs of the body are cut
//   into chunks of (waves/2) * K runs, set s takes the chunks of parity s and wavefront j of
//   a set moves runs j, j + waves/2, ... of each of its chunks: K loads in one burst, then K
//   stores in one burst.  When a burst is issued is decided by a timetable on the chip-wide
//   constant-rate counter (pacing.hpp), so that HBM sees the load burst of one set, then the
//   store burst of the other, and so on: one stream and one direction at a time.  Measured on
//   MI355X at n = 2^28 fp64 this moves 2-3 % more bytes per second than the dispatcher-ordered
//   shape (dot: 3-4 %).  Kernels with two inputs issue the loads of the second one in the order
//   in which their memory-channel classes match the first one's (launch_plan.hpp), which keeps
//   that gain wherever the two arrays lie relative to each other.  The rest (less than a chunk,
//   a ragged run, head and tail scalars) is moved after the timetable part, unpaced, by all
//   wavefronts together.
//
// Dot on arrays that fit the caches: tiled, a few workgroups per compute unit
//   The body is cut into tiles of blockDim.x * U vectors; workgroup g takes
//   tiles g, g + G, g + 2G, ...  Lane l of the workgroup reads vectors
//   l, l + B, ..., l + (U-1)B of a tile, so every wavefront-wide load is one
//   contiguous 1 KiB run and each lane has 2U independent loads in flight.
//   The workgroup whose turn comes after the last full tile also takes the ragged rest.
//
// Compile with -ffp-contract=off: Triad must round s*c and then b + (s*c).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "launch_plan.hpp"
#include "pacing.hpp"

namespace opal {

enum class Op : int { Copy = 0, Scale = 1, Add = 2, Triad = 3 };

constexpr int kMaxBlock = 1024;
constexpr int kWave = 64;

typedef double d2_t __attribute__((ext_vector_type(2)));
typedef float f4_t __attribute__((ext_vector_type(4)));

template <typename T> struct Vec16;
template <> struct Vec16<double> {
  typedef d2_t type;
  typedef d2_t loose __attribute__((aligned(8)));   // element-aligned only
  static constexpr int lanes = 2;
};
template <> struct Vec16<float> {
  typedef f4_t type;
  typedef f4_t loose __attribute__((aligned(4)));
  static constexpr int lanes = 4;
};

// 16-byte load.  ALIGNED: p is 16-byte aligned.  Otherwise p is only
// element-aligned; gfx950 global loads accept that (unaligned access mode), the
// type just has to say so.  NT marks the access non-temporal (streamed, no reuse).
template <typename T, bool ALIGNED, bool NT>
__device__ __forceinline__ typename Vec16<T>::type load16(const T* p) {
  typedef typename Vec16<T>::type V;
  typedef typename Vec16<T>::loose VL;
  if constexpr (ALIGNED) {
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
    else return *reinterpret_cast<const V*>(p);
  } else {
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const VL*>(p));
    else return *reinterpret_cast<const VL*>(p);
  }
}

template <typename T, bool NT>
__device__ __forceinline__ void store16(T* p, typename Vec16<T>::type v) {
  typedef typename Vec16<T>::type V;
  if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<V*>(p));
  else *reinterpret_cast<V*>(p) = v;
}

// One element of one kernel.  x = first input, y = second input (Add: b; Triad: c).
//   Copy : x            Scale: s * x
//   Add  : x + y        Triad: x + s * y   (x = b[i], y = c[i])
template <Op OP, typename X>
__device__ __forceinline__ X apply(X x, X y, X s) {
  if constexpr (OP == Op::Copy) return x;
  else if constexpr (OP == Op::Scale) return s * x;
  else if constexpr (OP == Op::Add) return x + y;
  else {
    const X t = s * y;   // rounded product
    return x + t;        // rounded sum; contraction is off, so this stays two instructions
  }
}

template <Op OP> constexpr bool kTwoInputs = (OP == Op::Add || OP == Op::Triad);

// The head and tail scalars of a split, element by element, by `threads` cooperating lanes.
template <typename T, Op OP>
__device__ __forceinline__ void edge_elements(T* __restrict__ out, const T* __restrict__ in0,
                                              const T* __restrict__ in1, T s, const plan::Split& sp,
                                              unsigned lane, unsigned threads) {
  constexpr unsigned L = 16 / sizeof(T);
  for (unsigned k = lane; k < sp.head + sp.tail; k += threads) {
    const size_t i = plan::edge_element(sp, L, k);
    const T x = in0[i];
    T y = x;
    if constexpr (kTwoInputs<OP>) y = in1[i];
    out[i] = apply<OP, T>(x, y, s);
  }
}

// Tells the compiler that a wave-uniform 64-bit value lives in scalar registers.
// Tile base addresses built from it stay in SGPRs, and each access becomes
// "scalar base + 32-bit lane offset" instead of a 64-bit pointer per lane.
__device__ __forceinline__ size_t wave_uniform(size_t x) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(x >> 32));
  return ((size_t)hi << 32) | lo;
}

// Elementwise kernel, launched with BLOCK threads per workgroup and
// max(1, ceil(nvec / BLOCK)) workgroups; lane l of workgroup g moves vector
// g * BLOCK + l.  out/in0/in1 point at element 0.
//   head : scalars before the vector body;  nvec : vectors in the body;
//   n    : total elements (tail = n - head - nvec*lanes < lanes).
// (out + head) is 16-byte aligned; ALIGNED says (in0 + head) and (in1 + head) are too.
// NT: loads and stores carry the non-temporal hint (arrays that are streamed
// from and to HBM); without it lines stay in L2 / Infinity Cache for the next
// kernel (arrays small enough to live there).
template <typename T, Op OP, int BLOCK, bool ALIGNED, bool NT>
__global__ __launch_bounds__(BLOCK) void stream_kernel(
    T* __restrict__ out, const T* __restrict__ in0, const T* __restrict__ in1, T s,
    unsigned head, size_t nvec, size_t n) {
  typedef typename Vec16<T>::type V;
  constexpr int L = Vec16<T>::lanes;
  static_assert(BLOCK % kWave == 0 && BLOCK >= kWave, "whole wavefronts");
  const unsigned lane = threadIdx.x;
  const size_t v0 = wave_uniform(plan::stream_vector(BLOCK, blockIdx.x, 0));   // first vector of this workgroup

  if (v0 + lane < nvec) {
    const size_t e0 = (size_t)head + v0 * L;
    const unsigned e = lane * L;
    const V x = load16<T, ALIGNED, NT>(in0 + e0 + e);
    V y = x;
    if constexpr (kTwoInputs<OP>) y = load16<T, ALIGNED, NT>(in1 + e0 + e);
    store16<T, NT>(out + e0 + e, apply<OP, V>(x, y, (V)(s)));
  }

  // Head and tail scalars (fewer than 1024/sizeof(T) + lanes of them), by the last workgroup.
  if (blockIdx.x == gridDim.x - 1) {
    const plan::Split sp{head, nvec, (unsigned)(n - head - nvec * L)};
    edge_elements<T, OP>(out, in0, in1, s, sp, lane, BLOCK);
  }
}

// Paced elementwise kernel: gridDim.x = p.waves one-wavefront workgroups (see the file header).
// Same pointer and alignment conventions as stream_kernel; all accesses non-temporal.
// Kernels with two inputs load the runs of the second input in the order in which their memory-channel
// classes match those of the first (plan::matched_run), keep them in the registers of the slot they
// were issued in, and store in slot order, picking the first input's run that belongs to each slot:
// the data of a slot can be stored as soon as its second-input load has arrived, as without the matching.
template <typename T, Op OP, int K, bool ALIGNED>
__device__ __forceinline__ void paced_stream_body(
    T* __restrict__ out, const T* __restrict__ in0, const T* __restrict__ in1, T s, const plan::Paced& p,
    const Pace& pace) {
  typedef typename Vec16<T>::type V;
  constexpr int L = Vec16<T>::lanes;
  constexpr unsigned RUN = plan::kRunVectors * L;   // elements per run
  const unsigned lane = threadIdx.x;
  const unsigned wave = blockIdx.x;
  const unsigned set = plan::paced_set(wave, p.set_bit), index = plan::paced_index(wave, p.set_bit);
  const bool reporter = pace_reporter(wave);
  T* const obody = out + p.split.head;
  const T* const xbody = in0 + p.split.head;
  const T* const ybody = kTwoInputs<OP> ? in1 + p.split.head : in0;
  const unsigned e = lane * L;

  // Which of the two matched orders this launch uses (pacing.hpp: learnt per pair of input arrays).
  OrderChoice choice{};
  if constexpr (kTwoInputs<OP> && K == (int)plan::kMatchedRuns) {
    if (p.matched && pace.period)
      choice = order_begin(pace, reinterpret_cast<uintptr_t>(xbody), reinterpret_cast<uintptr_t>(ybody), p.split.nvec,
                           p.flip0);
  }
  const unsigned flip = choice.slot != nullptr ? choice.flip : p.flip0;
  PaceState st{};
  if (pace.period) st = pace_begin(pace, set);
  for (size_t chunk = set; chunk < p.nchunks; chunk += 2) {
    V x[K], y[K];      // x[k]: run k of the first input; y[k]: the run of the second input issued in slot k
    unsigned order[K];  // which run that is (wave-uniform)
#pragma unroll
    for (int k = 0; k < K; ++k) order[k] = (unsigned)k;
    uint32_t turn = 0;
    unsigned long long word = 0;
    if (pace.period) {
      turn = pace_turn(pace, st, reporter);
      word = pace_feedback_load(pace, wave);
    }
    // one input after the other, so that each burst is a single stream
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const size_t e0 = wave_uniform(plan::paced_run(p, chunk, index, (unsigned)k) * RUN);
      if (pace.gap && k) pace_wait_until(turn + (uint32_t)k * pace.gap);
      x[k] = load16<T, ALIGNED, true>(xbody + e0 + e);
    }
    if constexpr (kTwoInputs<OP>) {
      if (pace.period && pace.second_input) pace_wait_until(turn + pace.second_input);
      if constexpr (K == (int)plan::kMatchedRuns) {
        if (p.matched) {
          const size_t r0 = wave_uniform(plan::paced_run(p, chunk, index, 0u) * RUN);
          const uintptr_t a0 = reinterpret_cast<uintptr_t>(xbody + r0), a1 = reinterpret_cast<uintptr_t>(ybody + r0);
#pragma unroll
          for (int k = 0; k < K; ++k)
            order[k] = (unsigned)__builtin_amdgcn_readfirstlane((int)plan::matched_run(a0, a1, (unsigned)k, flip));
        }
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const size_t e0 = wave_uniform(plan::paced_run(p, chunk, index, order[k]) * RUN);
        if (pace.gap && k) pace_wait_until(turn + pace.second_input + (uint32_t)k * pace.gap);
        y[k] = load16<T, ALIGNED, true>(ybody + e0 + e);
      }
    } else {
#pragma unroll
      for (int k = 0; k < K; ++k) y[k] = x[k];
    }
    if (pace.period) {
      pace_adopt(pace, st, word);   // needs the feedback word, hence every load of this burst
      if (pace.store) {
        // the clock must not be read before the data is here
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        pace_wait_until(turn + pace.store);
      }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const size_t e0 = wave_uniform(plan::paced_run(p, chunk, index, order[k]) * RUN);
      if (pace.gap && pace.store && k) pace_wait_until(turn + pace.store + (uint32_t)k * pace.gap);
      V xs = x[k];
      if constexpr (kTwoInputs<OP>) {
        // the first input's run that belongs to this slot (all of them arrived before the second burst's)
        xs = x[0];
#pragma unroll
        for (int j = 1; j < K; ++j) xs = (order[k] == (unsigned)j) ? x[j] : xs;
      }
      store16<T, true>(obody + e0 + e, apply<OP, V>(xs, y[k], (V)(s)));
    }
  }

  // The rest: runs rest_run0 + wave, + waves, ...; the last of them may be ragged.
  for (size_t run = p.rest_run0 + wave; run < p.total_runs; run += p.waves) {
    const size_t e0 = wave_uniform(run * RUN);
    if (run * plan::kRunVectors + lane < p.split.nvec) {
      const V x = load16<T, ALIGNED, true>(xbody + e0 + e);
      V y = x;
      if constexpr (kTwoInputs<OP>) y = load16<T, ALIGNED, true>(ybody + e0 + e);
      store16<T, true>(obody + e0 + e, apply<OP, V>(x, y, (V)(s)));
    }
  }
  if (wave == p.waves - 1) {
    edge_elements<T, OP>(out, in0, in1, s, p.split, lane, kWave);
    order_end(choice);
  }
}

template <typename T, Op OP, int K, bool ALIGNED>
__global__ __launch_bounds__(kWave) void paced_stream_kernel(
    T* __restrict__ out, const T* __restrict__ in0, const T* __restrict__ in1, T s, plan::Paced p, Pace pace) {
  paced_stream_body<T, OP, K, ALIGNED>(out, in0, in1, s, p, pace);
}

// ---------------------------------------------------------------------------
// Dot.

__device__ __forceinline__ double fma_t(double x, double y, double z) { return __builtin_fma(x, y, z); }
__device__ __forceinline__ float fma_t(float x, float y, float z) { return __builtin_fmaf(x, y, z); }

// Lane exchange inside a 16-lane row through the DPP path of the vector ALU
// (no LDS traffic).  CTRL: 0xB1 = quad_perm[1,0,3,2], 0x4E = quad_perm[2,3,0,1],
// 0x141 = row_half_mirror, 0x140 = row_mirror.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const uint64_t bits = __builtin_bit_cast(uint64_t, v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)bits, CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(bits >> 32), CTRL, 0xF, 0xF, true);
  return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

__device__ __forceinline__ float read_lane(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ double read_lane(double v, int lane) {
  const uint64_t bits = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(bits >> 32), lane);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Sum over the 64 lanes of a wavefront, same value in every lane, fixed order:
// pairs, quads, 8s and 16s by DPP butterflies inside each row of 16 lanes, then
// the four row sums read out of lanes 0/16/32/48 and added as (r0+r1)+(r2+r3).
// Must be reached by all 64 lanes.
template <typename X>
__device__ __forceinline__ X wave_sum(X v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  const X r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
  return (r0 + r1) + (r2 + r3);
}

// Sum over a workgroup in fp64: wavefront sums go through LDS, thread 0 adds
// them in wavefront order.  Valid in thread 0 only.  blockDim.x is a multiple of 64.
__device__ __forceinline__ double block_sum(double wave_total, double* lds /* kMaxBlock/kWave */) {
  const unsigned wave = threadIdx.x / kWave;
  const unsigned nwaves = blockDim.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) lds[wave] = wave_total;
  __syncthreads();
  double total = 0.0;
  if (threadIdx.x == 0) {
    for (unsigned w = 0; w < nwaves; ++w) total += lds[w];
  }
  return total;
}

// Combines a thread's U vector accumulators into one value in a fixed order: lanes of each
// accumulator pairwise, then accumulators pairwise.
template <typename T, int U>
__device__ __forceinline__ T thread_total(const typename Vec16<T>::type (&acc)[U]) {
  constexpr int L = Vec16<T>::lanes;
  T t[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if constexpr (L == 2) t[u] = acc[u][0] + acc[u][1];
    else t[u] = (acc[u][0] + acc[u][1]) + (acc[u][2] + acc[u][3]);
  }
#pragma unroll
  for (int w = 1; w < U; w *= 2) {
#pragma unroll
    for (int u = 0; u + w < U; u += 2 * w) t[u] += t[u + w];
  }
  return t[0];
}

// First pass, tiled shape: partials[g] = sum of a[i]*b[i] over the elements workgroup g owns
// (plan::Tiled; launched with t.groups workgroups of t.block threads, U == t.unroll).
// Same decomposition as stream_kernel, steered by `a` ((a + head) is 16-byte
// aligned; ALIGNED says (b + head) is too).  Each thread keeps U*lanes
// independent accumulators of type T, updated with fused multiply-adds; they
// are combined in a fixed order, then across the wavefront in T, then across
// the workgroup in fp64.
template <typename T, int U, bool ALIGNED, bool NT_LD>
__global__ __launch_bounds__(kMaxBlock) void dot_partial_kernel(
    const T* __restrict__ a, const T* __restrict__ b, double* __restrict__ partials, plan::Tiled t) {
  typedef typename Vec16<T>::type V;
  constexpr int L = Vec16<T>::lanes;
  __shared__ double lds[kMaxBlock / kWave];
  const unsigned B = blockDim.x;
  const unsigned tid = threadIdx.x;
  const T* const abody = a + t.split.head;
  const T* const bbody = b + t.split.head;

  V acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = (V)((T)0);

  for (size_t tile = blockIdx.x; tile < t.full_tiles; tile += gridDim.x) {
    const size_t e0 = wave_uniform(tile * t.tile_vectors * L);
    const T* ap = abody + e0;
    const T* bp = bbody + e0;
    V x[U], y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned v = (tid + u * B) * L;
      x[u] = load16<T, true, NT_LD>(ap + v);
      y[u] = load16<T, ALIGNED, NT_LD>(bp + v);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int l = 0; l < L; ++l) acc[u][l] = fma_t(x[u][l], y[u][l], acc[u][l]);
    }
  }

  if (blockIdx.x == plan::tiled_ragged_group(t)) {
    const size_t v0 = t.full_tiles * t.tile_vectors;
    for (size_t v = v0 + tid; v < t.split.nvec; v += B) {
      const V x = load16<T, true, false>(abody + v * L);
      const V y = load16<T, ALIGNED, false>(bbody + v * L);
#pragma unroll
      for (int l = 0; l < L; ++l) acc[0][l] = fma_t(x[l], y[l], acc[0][l]);
    }
    for (unsigned k = tid; k < t.split.head + t.split.tail; k += B) {
      const size_t i = plan::edge_element(t.split, L, k);
      acc[0][0] = fma_t(a[i], b[i], acc[0][0]);
    }
  }

  const T wave_total = wave_sum<T>(thread_total<T, U>(acc));
  const double total = block_sum((double)wave_total, lds);
  if (tid == 0) partials[blockIdx.x] = total;
}

// First pass, paced shape (plan::Paced; p.waves one-wavefront workgroups, K == p.k): the load
// burst of `a` and the load burst of `b` of a chunk are issued on the timetable (pace.second_input
// apart), the products are accumulated while the other set's bursts are in flight.  Accumulation
// as in dot_partial_kernel; partials[wave] = the wavefront's sum as fp64 (the single wavefront
// of the workgroup still goes through block_sum's LDS slot so that both shapes share one path).
template <typename T, int K, bool ALIGNED>
__global__ __launch_bounds__(kWave) void paced_dot_kernel(
    const T* __restrict__ a, const T* __restrict__ b, double* __restrict__ partials, plan::Paced p, Pace pace) {
  typedef typename Vec16<T>::type V;
  constexpr int L = Vec16<T>::lanes;
  constexpr unsigned RUN = plan::kRunVectors * L;
  __shared__ double lds[kMaxBlock / kWave];
  const unsigned lane = threadIdx.x;
  const unsigned wave = blockIdx.x;
  const unsigned set = plan::paced_set(wave, p.set_bit), index = plan::paced_index(wave, p.set_bit);
  const bool reporter = pace_reporter(wave);
  const T* const abody = a + p.split.head;
  const T* const bbody = b + p.split.head;
  const unsigned e = lane * L;

  V acc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) acc[k] = (V)((T)0);

  PaceState st{};
  if (pace.period) st = pace_begin(pace, set);
  for (size_t chunk = set; chunk < p.nchunks; chunk += 2) {
    V x[K], y[K];
    uint32_t turn = 0;
    unsigned long long word = 0;
    if (pace.period) {
      turn = pace_turn(pace, st, reporter);
      word = pace_feedback_load(pace, wave);
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const size_t e0 = wave_uniform(plan::paced_run(p, chunk, index, (unsigned)k) * RUN);
      if (pace.gap && k) pace_wait_until(turn + (uint32_t)k * pace.gap);
      x[k] = load16<T, true, true>(abody + e0 + e);
    }
    if (pace.period && pace.second_input) pace_wait_until(turn + pace.second_input);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const size_t e0 = wave_uniform(plan::paced_run(p, chunk, index, (unsigned)k) * RUN);
      if (pace.gap && k) pace_wait_until(turn + pace.second_input + (uint32_t)k * pace.gap);
      y[k] = load16<T, ALIGNED, true>(bbody + e0 + e);
    }
    if (pace.period) pace_adopt(pace, st, word);
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
      for (int l = 0; l < L; ++l) acc[k][l] = fma_t(x[k][l], y[k][l], acc[k][l]);
    }
  }

  for (size_t run = p.rest_run0 + wave; run < p.total_runs; run += p.waves) {
    const size_t e0 = wave_uniform(run * RUN);
    if (run * plan::kRunVectors + lane < p.split.nvec) {
      const V x = load16<T, true, true>(abody + e0 + e);
      const V y = load16<T, ALIGNED, true>(bbody + e0 + e);
#pragma unroll
      for (int l = 0; l < L; ++l) acc[0][l] = fma_t(x[l], y[l], acc[0][l]);
    }
  }
  if (wave == p.waves - 1) {
    for (unsigned k = lane; k < p.split.head + p.split.tail; k += kWave) {
      const size_t i = plan::edge_element(p.split, L, k);
      acc[0][0] = fma_t(a[i], b[i], acc[0][0]);
    }
  }

  const T wave_total = wave_sum<T>(thread_total<T, K>(acc));
  const double total = block_sum((double)wave_total, lds);
  if (lane == 0) partials[wave] = total;
}

// Second pass, one workgroup: result = sum of partials[0..count) in a fixed order
// (thread t adds partials t, t+B, ... in turn; then wavefront and workgroup sums).
// count == 0 stores 0.0.
__global__ __launch_bounds__(kMaxBlock) void dot_final_kernel(
    const double* __restrict__ partials, unsigned count, double* __restrict__ result) {
  __shared__ double lds[kMaxBlock / kWave];
  double acc = 0.0;
  for (unsigned i = threadIdx.x; i < count; i += blockDim.x) acc += partials[i];
  const double total = block_sum(wave_sum<double>(acc), lds);
  if (threadIdx.x == 0) *result = total;
}

}  // namespace opal
