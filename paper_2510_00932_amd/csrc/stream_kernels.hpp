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
// Dot: persistent, one workgroup per compute unit
//   The body is cut into tiles of blockDim.x * U vectors; workgroup g takes
//   tiles g, g + G, g + 2G, ...  Lane l of the workgroup reads vectors
//   l, l + B, ..., l + (U-1)B of a tile, so every wavefront-wide load is one
//   contiguous 1 KiB run and each lane has 2U independent loads in flight.
//   Reads alone run fastest with about 32 KiB in flight per compute unit,
//   which is 256 lanes x 4 vectors x 2 arrays.  The workgroup whose turn comes
//   after the last full tile also takes the ragged rest.
//
// Compile with -ffp-contract=off: Triad must round s*c and then b + (s*c).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

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

// Workgroup that takes the ragged rest: full_tiles mod gridDim.x.  full_tiles is
// below gridDim.x or far above it, so compare first and only then divide.
__device__ __forceinline__ unsigned ragged_group(size_t full_tiles) {
  return full_tiles < gridDim.x ? (unsigned)full_tiles : (unsigned)(full_tiles % gridDim.x);
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
  const size_t v0 = wave_uniform((size_t)blockIdx.x * BLOCK);   // first vector of this workgroup

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
    const size_t tail0 = (size_t)head + nvec * L;
    const unsigned tail = (unsigned)(n - tail0);
    for (unsigned k = lane; k < head + tail; k += BLOCK) {
      const size_t i = k < head ? (size_t)k : tail0 + (k - head);
      const T x = in0[i];
      T y = x;
      if constexpr (kTwoInputs<OP>) y = in1[i];
      out[i] = apply<OP, T>(x, y, s);
    }
  }
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

// First pass: partials[g] = sum of a[i]*b[i] over the elements workgroup g owns.
// Same decomposition as stream_kernel, steered by `a` ((a + head) is 16-byte
// aligned; ALIGNED says (b + head) is too).  Each thread keeps U*lanes
// independent accumulators of type T, updated with fused multiply-adds; they
// are combined in a fixed order, then across the wavefront in T, then across
// the workgroup in fp64.
template <typename T, int U, bool ALIGNED, bool NT_LD>
__global__ __launch_bounds__(kMaxBlock) void dot_partial_kernel(
    const T* __restrict__ a, const T* __restrict__ b, double* __restrict__ partials,
    unsigned head, size_t nvec, size_t full_tiles, size_t n) {
  typedef typename Vec16<T>::type V;
  constexpr int L = Vec16<T>::lanes;
  __shared__ double lds[kMaxBlock / kWave];
  const unsigned B = blockDim.x;
  const unsigned tid = threadIdx.x;
  const size_t tile_vecs = (size_t)B * U;
  const T* const abody = a + head;
  const T* const bbody = b + head;

  V acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = (V)((T)0);

  for (size_t tile = blockIdx.x; tile < full_tiles; tile += gridDim.x) {
    const size_t e0 = wave_uniform(tile * tile_vecs * L);
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

  if (blockIdx.x == ragged_group(full_tiles)) {
    const size_t v0 = full_tiles * tile_vecs;
    for (size_t v = v0 + tid; v < nvec; v += B) {
      const V x = load16<T, true, false>(abody + v * L);
      const V y = load16<T, ALIGNED, false>(bbody + v * L);
#pragma unroll
      for (int l = 0; l < L; ++l) acc[0][l] = fma_t(x[l], y[l], acc[0][l]);
    }
    const size_t tail0 = (size_t)head + nvec * L;
    const unsigned tail = (unsigned)(n - tail0);
    for (unsigned k = tid; k < head + tail; k += B) {
      const size_t i = k < head ? (size_t)k : tail0 + (k - head);
      acc[0][0] = fma_t(a[i], b[i], acc[0][0]);
    }
  }

  // Thread total: lanes of each accumulator pairwise, then accumulators pairwise.
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
  const T wave_total = wave_sum<T>(t[0]);
  const double total = block_sum((double)wave_total, lds);
  if (tid == 0) partials[blockIdx.x] = total;
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
