// Host side of libopal: argument checks, work split and kernel launches for the
// five streaming vector kernels (Table 1: Copy, Mul, Add, Triad, Dot).  The
// interface contract is written out in include/opal.h.
//
// Built for gfx950 only:
//   hipcc --offload-arch=gfx950 -O3 -ffp-contract=off \
//         -Xclang -target-feature -Xclang -packed-fp32-ops -shared -fPIC

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/opal.h"
#include "launch_plan.hpp"
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

// Device words of the pacing feedback and of the learnt matched orders (pacing.hpp) and the scratch of opal_dot_static: file-scope
// device arrays, one copy per GPU, held until the process ends.  In host code an array's name is
// only a stand-in; its device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned long long pace_words[kFeedbackWords];
static __device__ __align__(256) unsigned order_words[plan::kOrderWords];
constexpr size_t kStaticScratchBytes = (size_t)kDotMaxGroups * sizeof(double);   // 64 KiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// What the library needs to know about a device, looked up on the first call made with that
// device current and cached by device id.
struct DeviceInfo {
  unsigned cus = 0;                       // compute units
  unsigned ticks_per_us = 0;              // rate of the constant counter the timetable runs on
  bool paced = false;                     // the paced shapes were measured on this kind of device
  unsigned long long* feedback = nullptr; // device address of pace_words
  unsigned* order_words = nullptr;        // device address of order_words
  double* scratch = nullptr;              // device address of scratch
};

const DeviceInfo* device_info() {
  static DeviceInfo info[kMaxDevices];
  static std::atomic<int> ready[kMaxDevices];   // zero-initialised; 1 once info[dev] is complete
  static thread_local DeviceInfo overflow;      // device ids beyond the table: looked up per call
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return nullptr;
  const bool slot = dev >= 0 && dev < kMaxDevices;
  if (slot && ready[dev].load(std::memory_order_acquire)) return &info[dev];
  DeviceInfo d;
  int cus = 0, khz = 0;
  if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) || cus <= 0) return nullptr;
  d.cus = (unsigned)cus;
  if (hip_ok(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev)) && khz >= 1000)
    d.ticks_per_us = (unsigned)(khz / 1000);
  hipDeviceProp_t prop;
  const bool gfx950 = hip_ok(hipGetDeviceProperties(&prop, dev)) && std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
  void* ptr = nullptr;
  if (hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(pace_words)))) d.feedback = static_cast<unsigned long long*>(ptr);
  ptr = nullptr;
  if (hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(order_words)))) d.order_words = static_cast<unsigned*>(ptr);
  ptr = nullptr;
  if (hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)))) d.scratch = static_cast<double*>(ptr);
  d.paced = gfx950 && d.cus == kPacedCUs && d.ticks_per_us > 0 && d.feedback != nullptr;
  if (!slot) {
    overflow = d;
    return &overflow;
  }
  static std::mutex fill;
  std::lock_guard<std::mutex> lock(fill);
  if (!ready[dev].load(std::memory_order_acquire)) {
    info[dev] = d;
    ready[dev].store(1, std::memory_order_release);
  }
  return &info[dev];
}

// Run-time copies of the paced shapes (opal_pacing_configure may change the rates) and the switch.
PacedShape g_shapes[3] = {kPacedOneInput, kPacedTwoInputs, kPacedDot};
std::atomic<int> g_matched{1};   // two-input paced kernels: second input in class-matched order (plan::matched_run)
std::atomic<unsigned> g_order_epoch{0};   // changes whenever the setting does: what was learnt before no longer applies
std::atomic<int> g_pacing{-1};   // -1: not decided yet (environment), 0: off, 1: on, 2: on at every size the shape can hold

int pacing_mode() {
  int v = g_pacing.load(std::memory_order_relaxed);
  if (v < 0) {
    const char* env = std::getenv("OPAL_PACING");
    v = (env != nullptr && env[0] == '0') ? 0 : (env != nullptr && env[0] == '2') ? 2 : 1;
    g_pacing.store(v, std::memory_order_relaxed);
  }
  return v;
}

// Timetable of a paced launch: `streams` arrays, each moved waves * k KiB per period.
Pace make_pace(const PacedShape& sh, unsigned streams, const DeviceInfo& dev) {
  const double bytes = (double)sh.waves * sh.k * 1024.0 * streams;
  const double period = bytes / sh.bytes_per_us * dev.ticks_per_us;
  Pace pace;
  pace.period = period < 16.0 ? 16u : (uint32_t)(period + 0.5);
  pace.second_input = (uint32_t)(sh.second_input_at * pace.period);
  pace.store = (uint32_t)(sh.store_at * pace.period);
  pace.gap = (uint32_t)(sh.gap * pace.period);
  pace.tolerance = sh.tolerance;
  pace.feedback = sh.feedback ? dev.feedback : nullptr;
  pace.order_words = dev.order_words;
  pace.order_epoch = g_order_epoch.load(std::memory_order_relaxed);
  return pace;
}

bool aligned16_after(const void* p, unsigned head, size_t elem) {
  return ((reinterpret_cast<uintptr_t>(p) + (uintptr_t)head * elem) & 15u) == 0;
}

template <typename T>
bool cache_resident(size_t n) { return n * sizeof(T) <= kCacheResidentBytes; }

// The paced shapes apply to arrays well beyond the caches, on the device they were measured on.
template <typename T>
bool use_paced(size_t n, const DeviceInfo* dev, const PacedShape& sh) {
  const int mode = pacing_mode();
  if (dev == nullptr || !dev->paced || mode == 0) return false;
  if (mode == 1 && n < sh.min_bytes / sizeof(T)) return false;
  return n / ((size_t)(sh.waves / 2) * sh.k * (1024 / sizeof(T))) >= 16;   // at least 16 chunks
}

int check_ptr(const void* p, size_t n, size_t elem) {
  if (n == 0) return OPAL_OK;
  if (p == nullptr) return OPAL_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(p) % elem != 0) return OPAL_ERR_ALIGN;
  return OPAL_OK;
}

// n * sizeof(T) must be addressable; anything else cannot be a real array.
template <typename T>
bool size_ok(size_t n) { return n <= (~(size_t)0 >> 1) / sizeof(T); }

// Dispatcher-ordered shape: one launch per segment of the body (plan::segment).
template <typename T, Op OP, int BLOCK, bool NT>
int launch_stream_shape(T* out, const T* in0, const T* in1, T s, size_t n, hipStream_t stream) {
  constexpr unsigned L = 16 / sizeof(T);
  const plan::Split sp = plan::split(reinterpret_cast<uintptr_t>(out), n, sizeof(T));
  const bool aligned = aligned16_after(in0, sp.head, sizeof(T)) &&
                       (!kTwoInputs<OP> || aligned16_after(in1, sp.head, sizeof(T)));
  const size_t count = plan::segment_count(sp, BLOCK);
  for (size_t i = 0; i < count; ++i) {
    const plan::Segment g = plan::segment(sp, L, BLOCK, i);
    T* o = out + g.elem_offset;
    const T* x = in0 + g.elem_offset;
    const T* y = kTwoInputs<OP> ? in1 + g.elem_offset : nullptr;
    const bool ok = aligned ? launch(stream_kernel<T, OP, BLOCK, true, NT>, g.groups, (unsigned)BLOCK, stream,
                                     o, x, y, s, g.head, g.nvec, g.n)
                            : launch(stream_kernel<T, OP, BLOCK, false, NT>, g.groups, (unsigned)BLOCK, stream,
                                     o, x, y, s, g.head, g.nvec, g.n);
    if (!ok) return OPAL_ERR_LAUNCH;
  }
  return OPAL_OK;
}

template <typename T, Op OP>
int launch_paced(T* out, const T* in0, const T* in1, T s, size_t n, const DeviceInfo& dev, const PacedShape& sh,
                 hipStream_t stream) {
  constexpr int K = kTwoInputs<OP> ? kPacedK2 : kPacedK1;
  const plan::Split sp = plan::split(reinterpret_cast<uintptr_t>(out), n, sizeof(T));
  const bool aligned = aligned16_after(in0, sp.head, sizeof(T)) &&
                       (!kTwoInputs<OP> || aligned16_after(in1, sp.head, sizeof(T)));
  plan::Paced p = plan::paced(sp, sh.waves, K, sh.set_bit);
  const int matched = g_matched.load(std::memory_order_relaxed);
  p.matched = p.matched && matched != 0;
  p.flip0 = matched == 2 ? 1u : 0u;
  const Pace pace = make_pace(sh, kTwoInputs<OP> ? 3u : 2u, dev);
  const bool ok = aligned ? launch(paced_stream_kernel<T, OP, K, true>, sh.waves, (unsigned)kWave, stream,
                                   out, in0, in1, s, p, pace)
                          : launch(paced_stream_kernel<T, OP, K, false>, sh.waves, (unsigned)kWave, stream,
                                   out, in0, in1, s, p, pace);
  return ok ? OPAL_OK : OPAL_ERR_LAUNCH;
}

template <typename T, Op OP>
int launch_stream(T* out, const T* in0, const T* in1, T s, size_t n, hipStream_t stream) {
  if (!size_ok<T>(n)) return OPAL_ERR_SIZE;
  if (cache_resident<T>(n)) return launch_stream_shape<T, OP, kResidentBlock, false>(out, in0, in1, s, n, stream);
  const PacedShape sh = g_shapes[kTwoInputs<OP> ? 1 : 0];
  if (pacing_mode() != 0) {
    const DeviceInfo* dev = device_info();
    if (use_paced<T>(n, dev, sh)) return launch_paced<T, OP>(out, in0, in1, s, n, *dev, sh, stream);
  }
  return launch_stream_shape<T, OP, kStreamBlock, true>(out, in0, in1, s, n, stream);
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
bool launch_dot_tiled(const T* a, const T* b, size_t n, double* partials, unsigned block, unsigned cus,
                      unsigned* groups_out, hipStream_t stream) {
  const plan::Split sp = plan::split(reinterpret_cast<uintptr_t>(a), n, sizeof(T));
  const bool aligned = aligned16_after(b, sp.head, sizeof(T));
  unsigned cap = dot_groups_bound(n, sizeof(T) == 8 ? OPAL_F64 : OPAL_F32);
  if (cap > cus * kDotGroupsPerCU) cap = cus * kDotGroupsPerCU;
  const plan::Tiled t = plan::tiled(sp, block, kDotUnroll, cap);
  *groups_out = t.groups;
  return aligned ? launch(dot_partial_kernel<T, kDotUnroll, true, NT>, t.groups, block, stream, a, b, partials, t)
                 : launch(dot_partial_kernel<T, kDotUnroll, false, NT>, t.groups, block, stream, a, b, partials, t);
}

template <typename T>
bool launch_dot_paced(const T* a, const T* b, size_t n, double* partials, const DeviceInfo& dev,
                      const PacedShape& sh, hipStream_t stream) {
  const plan::Split sp = plan::split(reinterpret_cast<uintptr_t>(a), n, sizeof(T));
  const bool aligned = aligned16_after(b, sp.head, sizeof(T));
  const plan::Paced p = plan::paced(sp, sh.waves, kPacedKDot, sh.set_bit);
  const Pace pace = make_pace(sh, 2u, dev);
  return aligned ? launch(paced_dot_kernel<T, kPacedKDot, true>, sh.waves, (unsigned)kWave, stream, a, b, partials, p, pace)
                 : launch(paced_dot_kernel<T, kPacedKDot, false>, sh.waves, (unsigned)kWave, stream, a, b, partials, p, pace);
}

template <typename T>
int launch_dot(const T* a, const T* b, size_t n, double* partials, double* result, hipStream_t stream) {
  if (!size_ok<T>(n)) return OPAL_ERR_SIZE;
  unsigned groups = 0;
  if (n > 0) {
    const DeviceInfo* dev = device_info();
    if (dev == nullptr) return OPAL_ERR_LAUNCH;
    const PacedShape sh = g_shapes[2];
    bool ok;
    if (use_paced<T>(n, dev, sh) && sh.waves <= dot_groups_bound(n, sizeof(T) == 8 ? OPAL_F64 : OPAL_F32)) {
      groups = sh.waves;
      ok = launch_dot_paced<T>(a, b, n, partials, *dev, sh, stream);
    } else if (cache_resident<T>(n)) {
      ok = launch_dot_tiled<T, false>(a, b, n, partials, kDotResidentBlock, dev->cus, &groups, stream);
    } else {
      ok = launch_dot_tiled<T, true>(a, b, n, partials, kDotBlock, dev->cus, &groups, stream);
    }
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
  if (tiles > plan::kMaxWorkItems / kLdsBlock) return OPAL_ERR_SIZE;
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

size_t opal_dot_static_scratch_bytes(void) { return kStaticScratchBytes; }

int opal_dot_static(const void* a, const void* b, size_t n, int dtype, double* result, void* stream) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return OPAL_ERR_DTYPE;
  const size_t elem = dtype == OPAL_F64 ? 8 : 4;
  int st = check_ptr(a, n, elem);
  if (st == OPAL_OK) st = check_ptr(b, n, elem);
  if (st != OPAL_OK) return st;
  if (result == nullptr) return OPAL_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(result) % 8 != 0) return OPAL_ERR_ALIGN;
  if (opal_dot_workspace_bytes(n, dtype) > kStaticScratchBytes) return OPAL_ERR_WORKSPACE;
  const DeviceInfo* dev = device_info();
  if (dev == nullptr || dev->scratch == nullptr) return OPAL_ERR_LAUNCH;
  double* partials = dev->scratch;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (dtype == OPAL_F64) {
    return launch_dot<double>(static_cast<const double*>(a), static_cast<const double*>(b), n, partials, result, hs);
  }
  return launch_dot<float>(static_cast<const float*>(a), static_cast<const float*>(b), n, partials, result, hs);
}

void opal_set_pacing(int mode) { g_pacing.store(mode <= 0 ? 0 : mode >= 2 ? 2 : 1, std::memory_order_relaxed); }

int opal_matched_order_state(const void* out, const void* in0, const void* in1, size_t n, int dtype,
                             unsigned state[4]) {
  if (dtype != OPAL_F64 && dtype != OPAL_F32) return OPAL_ERR_DTYPE;
  if (out == nullptr || in0 == nullptr || in1 == nullptr || state == nullptr) return OPAL_ERR_NULL;
  const DeviceInfo* dev = device_info();
  if (dev == nullptr || dev->order_words == nullptr) return OPAL_ERR_LAUNCH;
  const size_t elem = dtype == OPAL_F64 ? 8 : 4;
  const plan::Split sp = plan::split(reinterpret_cast<uintptr_t>(out), n, elem);   // as the kernels split
  const plan::OrderKey key =
      plan::order_key(reinterpret_cast<uintptr_t>(in0) + (uintptr_t)sp.head * elem,
                      reinterpret_cast<uintptr_t>(in1) + (uintptr_t)sp.head * elem, sp.nvec,
                      g_order_epoch.load(std::memory_order_relaxed));
  unsigned words[plan::kOrderSlotWords];
  if (!hip_ok(hipMemcpy(words, dev->order_words + (size_t)key.slot * plan::kOrderSlotWords, sizeof(words),
                        hipMemcpyDeviceToHost)))
    return OPAL_ERR_LAUNCH;
  const bool known = words[0] == key.lo && words[1] == key.hi;
  state[0] = known ? words[2] : 0u;
  state[1] = known ? words[3] : 0xFFFFFFFFu;
  state[2] = known ? words[4] : 0xFFFFFFFFu;
  const unsigned first = g_matched.load(std::memory_order_relaxed) == 2 ? 1u : 0u;
  state[3] = plan::order_of_launch(state[0], first, state[1], state[2]);
  return OPAL_OK;
}

void opal_set_matched_order(int on) {
  g_matched.store(on == 2 ? 2 : on != 0, std::memory_order_relaxed);
  g_order_epoch.fetch_add(1u, std::memory_order_relaxed);
}

int opal_get_pacing(void) { return pacing_mode(); }

int opal_pacing_configure(int kind, double terabytes_per_second, double store_at, double second_input_at,
                          double gap, unsigned tolerance_ticks, int feedback, unsigned set_bit) {
  if (kind < 0 || kind > 2) return OPAL_ERR_SIZE;
  if (!(terabytes_per_second >= 0.5 && terabytes_per_second <= 64.0)) return OPAL_ERR_SIZE;
  if (!(store_at >= 0.0 && store_at < 1.0) || !(second_input_at >= 0.0 && second_input_at < 1.0)) return OPAL_ERR_SIZE;
  if (!(gap >= 0.0 && gap < 0.25)) return OPAL_ERR_SIZE;
  if (set_bit > 8 || g_shapes[kind].waves % (2u << set_bit) != 0) return OPAL_ERR_SIZE;
  PacedShape sh = g_shapes[kind];
  sh.bytes_per_us = terabytes_per_second * 1e6;
  sh.store_at = store_at;
  sh.second_input_at = second_input_at;
  sh.gap = gap;
  sh.set_bit = set_bit;
  sh.tolerance = tolerance_ticks;
  sh.feedback = feedback != 0;
  g_shapes[kind] = sh;
  return OPAL_OK;
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
