// Host side of libopal: argument checks, work split and kernel launches for the
// five streaming vector kernels (Table 1: Copy, Mul, Add, Triad, Dot).  The
// interface contract is written out in include/opal.h.
//
// Built for gfx950 only:
//   hipcc --offload-arch=gfx950 -O3 -ffp-contract=off \
//         -Xclang -target-feature -Xclang -packed-fp32-ops -shared -fPIC

#include <atomic>

#include "../../include/opal.h"
#include "launch_shapes.hpp"
#include "lds_kernel.hpp"
#include "stream_kernels.hpp"

namespace {

using namespace opal;

constexpr int kMaxDevices = 64;

// Last HIP error this thread met inside the library (hipSuccess if none yet).
thread_local hipError_t g_last_hip_error = hipSuccess;

bool hip_ok(hipError_t e) {
  if (e != hipSuccess) g_last_hip_error = e;
  return e == hipSuccess;
}

// Launches through the call that returns its own status, so an error left behind
// by some earlier, unrelated runtime call of the process is never mistaken for ours.
template <typename... Params, typename... Args>
bool launch(void (*kernel)(Params...), unsigned grid, unsigned block, hipStream_t stream, Args... args) {
  auto pack = [&](Params... p) {
    void* argv[] = {static_cast<void*>(&p)...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3(grid), dim3(block), argv, 0, stream);
  };
  return hip_ok(pack(args...));
}

// Compute units of the current device (cached per device id); 0 on failure.
unsigned compute_units() {
  static std::atomic<int> cached[kMaxDevices];   // zero-initialised; any thread may fill an entry
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return 0;
  const bool slot = dev >= 0 && dev < kMaxDevices;
  if (slot) {
    const int known = cached[dev].load(std::memory_order_relaxed);
    if (known > 0) return (unsigned)known;
  }
  int cus = 0;
  if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) || cus <= 0)
    return 0;
  if (slot) cached[dev].store(cus, std::memory_order_relaxed);
  return (unsigned)cus;
}

struct Split {
  unsigned head;   // scalar elements before the body
  size_t nvec;     // 16-byte vectors in the body
};

// Head = elements from `steer` up to its next kBodyAlign-byte boundary (or all n).
template <typename T>
Split split(const void* steer, size_t n) {
  constexpr size_t L = 16 / sizeof(T);
  const uintptr_t addr = reinterpret_cast<uintptr_t>(steer);
  size_t head = ((kBodyAlign - (addr % kBodyAlign)) % kBodyAlign) / sizeof(T);
  if (head > n) head = n;
  return Split{(unsigned)head, (n - head) / L};
}

bool aligned16_after(const void* p, unsigned head, size_t elem) {
  return ((reinterpret_cast<uintptr_t>(p) + (uintptr_t)head * elem) & 15u) == 0;
}

size_t dot_full_tiles(size_t nvec, unsigned block) { return nvec / ((size_t)block * (size_t)kDotUnroll); }

template <typename T>
bool cache_resident(size_t n) { return n * sizeof(T) <= kCacheResidentBytes; }

int check_ptr(const void* p, size_t n, size_t elem) {
  if (n == 0) return OPAL_OK;
  if (p == nullptr) return OPAL_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(p) % elem != 0) return OPAL_ERR_ALIGN;
  return OPAL_OK;
}

template <typename T, Op OP, int BLOCK, bool NT>
int launch_stream_shape(T* out, const T* in0, const T* in1, T s, size_t n, hipStream_t stream) {
  const Split sp = split<T>(out, n);
  const bool aligned = aligned16_after(in0, sp.head, sizeof(T)) &&
                       (!kTwoInputs<OP> || aligned16_after(in1, sp.head, sizeof(T)));
  size_t groups = (sp.nvec + BLOCK - 1) / BLOCK;
  if (groups < 1) groups = 1;
  if (groups > kMaxGrid) return OPAL_ERR_SIZE;
  const bool ok = aligned ? launch(stream_kernel<T, OP, BLOCK, true, NT>, (unsigned)groups, (unsigned)BLOCK, stream,
                                   out, in0, in1, s, sp.head, sp.nvec, n)
                          : launch(stream_kernel<T, OP, BLOCK, false, NT>, (unsigned)groups, (unsigned)BLOCK, stream,
                                   out, in0, in1, s, sp.head, sp.nvec, n);
  return ok ? OPAL_OK : OPAL_ERR_LAUNCH;
}

template <typename T, Op OP>
int launch_stream(T* out, const T* in0, const T* in1, T s, size_t n, hipStream_t stream) {
  return cache_resident<T>(n) ? launch_stream_shape<T, OP, kResidentBlock, false>(out, in0, in1, s, n, stream)
                              : launch_stream_shape<T, OP, kStreamBlock, true>(out, in0, in1, s, n, stream);
}

template <Op OP>
int elementwise(void* out, const void* in0, const void* in1, double s, size_t n, int dtype, void* stream) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return OPAL_ERR_DTYPE;
  const size_t elem = dtype == OPAL_F64 ? 8 : 4;
  int st = check_ptr(out, n, elem);
  if (st == OPAL_OK) st = check_ptr(in0, n, elem);
  if (st == OPAL_OK && kTwoInputs<OP>) st = check_ptr(in1, n, elem);
  if (st != OPAL_OK) return st;
  if (n == 0) return OPAL_OK;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (dtype == OPAL_F64) {
    return launch_stream<double, OP>(static_cast<double*>(out), static_cast<const double*>(in0),
                                     static_cast<const double*>(in1), s, n, hs);
  }
  return launch_stream<float, OP>(static_cast<float*>(out), static_cast<const float*>(in0),
                                  static_cast<const float*>(in1), (float)s, n, hs);
}

// Upper bound, from n alone, on the workgroups of dot's first pass.
unsigned dot_groups_bound(size_t n, int dtype) {
  const size_t lanes = dtype == OPAL_F64 ? 2 : 4;
  const size_t tiles = n / ((size_t)kDotBlock * kDotUnroll * lanes);
  size_t g = tiles < 1 ? 1 : tiles;
  if (g > kDotMaxGroups) g = kDotMaxGroups;
  return (unsigned)g;
}

template <typename T, bool NT>
bool launch_dot_pass1(const T* a, const T* b, size_t n, double* partials, unsigned block, unsigned cus,
                      unsigned* groups_out, hipStream_t stream) {
  const Split sp = split<T>(a, n);
  const bool aligned = aligned16_after(b, sp.head, sizeof(T));
  const size_t tiles = dot_full_tiles(sp.nvec, block);
  size_t g = tiles < 1 ? 1 : tiles;
  const unsigned bound = dot_groups_bound(n, sizeof(T) == 8 ? OPAL_F64 : OPAL_F32);
  if (g > (size_t)cus * kDotGroupsPerCU) g = (size_t)cus * kDotGroupsPerCU;
  if (g > bound) g = bound;
  *groups_out = (unsigned)g;
  return aligned ? launch(dot_partial_kernel<T, kDotUnroll, true, NT>, (unsigned)g, block, stream, a, b, partials,
                          sp.head, sp.nvec, tiles, n)
                 : launch(dot_partial_kernel<T, kDotUnroll, false, NT>, (unsigned)g, block, stream, a, b, partials,
                          sp.head, sp.nvec, tiles, n);
}

template <typename T>
int launch_dot(const T* a, const T* b, size_t n, double* partials, double* result, hipStream_t stream) {
  unsigned groups = 0;
  if (n > 0) {
    const unsigned cus = compute_units();
    if (cus == 0) return OPAL_ERR_LAUNCH;
    const bool ok = cache_resident<T>(n)
                        ? launch_dot_pass1<T, false>(a, b, n, partials, kDotResidentBlock, cus, &groups, stream)
                        : launch_dot_pass1<T, true>(a, b, n, partials, kDotBlock, cus, &groups, stream);
    if (!ok) return OPAL_ERR_LAUNCH;
  }
  const double* cpartials = partials;
  return launch(dot_final_kernel, 1u, kFinalBlock, stream, cpartials, groups, result) ? OPAL_OK : OPAL_ERR_LAUNCH;
}

constexpr int kLdsBlock = 256;   // 4 vectors per thread; 32 KiB of LDS per workgroup, 5 workgroups per CU

template <typename T>
int launch_lds(const T* in, T* out, T c, size_t n, unsigned rep, hipStream_t stream) {
  const size_t tile = (size_t)kLdsTileVectors * (16 / sizeof(T));
  const size_t tiles = n / tile;
  if (tiles > kMaxGrid) return OPAL_ERR_SIZE;
  return launch(lds_stream_kernel<T, kLdsBlock>, (unsigned)tiles, (unsigned)kLdsBlock, stream, in, out, c, rep)
             ? OPAL_OK
             : OPAL_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int opal_copy(const void* a, void* c, size_t n, int dtype, void* stream) {
  return elementwise<Op::Copy>(c, a, nullptr, 0.0, n, dtype, stream);
}

int opal_scale(void* b, const void* c, double s, size_t n, int dtype, void* stream) {
  return elementwise<Op::Scale>(b, c, nullptr, s, n, dtype, stream);
}

int opal_add(const void* a, const void* b, void* c, size_t n, int dtype, void* stream) {
  return elementwise<Op::Add>(c, a, b, 0.0, n, dtype, stream);
}

int opal_triad(void* a, const void* b, const void* c, double s, size_t n, int dtype, void* stream) {
  return elementwise<Op::Triad>(a, b, c, s, n, dtype, stream);
}

size_t opal_dot_workspace_bytes(size_t n, int dtype) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return 0;
  return (size_t)dot_groups_bound(n, dtype) * sizeof(double);
}

int opal_dot(const void* a, const void* b, size_t n, int dtype, void* workspace, size_t workspace_bytes,
             double* result, void* stream) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return OPAL_ERR_DTYPE;
  const size_t elem = dtype == OPAL_F64 ? 8 : 4;
  int st = check_ptr(a, n, elem);
  if (st == OPAL_OK) st = check_ptr(b, n, elem);
  if (st != OPAL_OK) return st;
  if (result == nullptr || workspace == nullptr) return OPAL_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(result) % 8 != 0 || reinterpret_cast<uintptr_t>(workspace) % 8 != 0)
    return OPAL_ERR_ALIGN;
  if (workspace_bytes < opal_dot_workspace_bytes(n, dtype)) return OPAL_ERR_WORKSPACE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  double* partials = static_cast<double*>(workspace);
  if (dtype == OPAL_F64) {
    return launch_dot<double>(static_cast<const double*>(a), static_cast<const double*>(b), n, partials, result, hs);
  }
  return launch_dot<float>(static_cast<const float*>(a), static_cast<const float*>(b), n, partials, result, hs);
}

size_t opal_lds_tile_elements(int dtype) {
  if (dtype == OPAL_F64) return (size_t)kLdsTileVectors * 2;
  if (dtype == OPAL_F32) return (size_t)kLdsTileVectors * 4;
  return 0;
}

int opal_lds_stream(const void* in, void* out, double c, size_t n, unsigned rep, int dtype, void* stream) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return OPAL_ERR_DTYPE;
  if (n == 0) return OPAL_OK;
  if (in == nullptr || out == nullptr) return OPAL_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(in) % 16 != 0 || reinterpret_cast<uintptr_t>(out) % 16 != 0) return OPAL_ERR_ALIGN;
  if (n % opal_lds_tile_elements(dtype) != 0) return OPAL_ERR_SIZE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (dtype == OPAL_F64)
    return launch_lds<double>(static_cast<const double*>(in), static_cast<double*>(out), c, n, rep, hs);
  return launch_lds<float>(static_cast<const float*>(in), static_cast<float*>(out), (float)c, n, rep, hs);
}

const char* opal_status_string(int status) {
  switch (status) {
    case OPAL_OK: return "ok";
    case OPAL_ERR_NULL: return "a required pointer is NULL";
    case OPAL_ERR_DTYPE: return "dtype is neither OPAL_F64 nor OPAL_F32";
    case OPAL_ERR_ALIGN: return "a pointer is not aligned to its element size";
    case OPAL_ERR_WORKSPACE: return "dot workspace is smaller than opal_dot_workspace_bytes(n, dtype)";
    case OPAL_ERR_LAUNCH: return "the HIP runtime refused a query or a kernel launch";
    case OPAL_ERR_SIZE: return "n is larger than one launch can cover, or not a whole number of LDS tiles";
    default: return "unknown status";
  }
}

const char* opal_last_hip_error(void) { return hipGetErrorName(g_last_hip_error); }

size_t opal_bytes_per_element(int kernel, int dtype) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return 0;
  const size_t w = dtype == OPAL_F64 ? 8 : 4;
  switch (kernel) {
    case 0: case 1: case 4: return 2 * w;
    case 2: case 3: return 3 * w;
    default: return 0;
  }
}

}  // extern "C"
