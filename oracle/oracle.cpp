// CPU oracle for the five streaming vector kernels (Copy, Mul, Add, Triad, Dot)
// that the paper lists as its simple memory-bound benchmark subjects
// (Table 1; Section 5.2).
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain definition of
// each kernel written out as one loop on one host core.  It shares no code,
// header, table or helper with the GPU library, and only the test-suite, the
// smoke check and the benchmark's CPU-baseline leg may call it.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC
//   -ffp-contract=off : the compiler may never fuse s*c[i] + b[i] into one FMA,
//                       so Triad rounds twice, exactly as the definition says.
//   x86-64 SSE2       : float/double expressions are evaluated in their own
//                       type (FLT_EVAL_METHOD == 0); long double is the 80-bit
//                       x87 format with a 64-bit significand.
//
// Operand roles (the paper gives only the kernel names; roles follow the
// usual STREAM convention):
//   copy : c[i] = a[i]
//   mul  : b[i] = s * c[i]            (called "scale" in the library's API)
//   add  : c[i] = a[i] + b[i]
//   triad: a[i] = b[i] + s * c[i]     (multiply rounded, then add rounded)
//   dot  : sum_i a[i] * b[i]
//
// Also here: the LDS-streaming microkernel (the analogue of the shared-memory
// benchmark subject of Table 1), defined further down.
//
// Parity pins for every function here live in tests/test_oracle_pins.py and
// tests/test_oracle_lds_pins.py: closed forms on constant and ramp fills,
// exact rational arithmetic on small random inputs, a vector on which fused
// and unfused Triad differ, a dyadic chain whose every step is exact, and for
// the LDS kernel pure rotations, exact adds and composition of calls.

#include <cstddef>
#include <cstdint>

namespace {

template <typename T>
void copy_loop(const T* a, T* c, size_t n) {
  for (size_t i = 0; i < n; ++i) c[i] = a[i];
}

template <typename T>
void scale_loop(T* b, const T* c, T s, size_t n) {
  for (size_t i = 0; i < n; ++i) b[i] = s * c[i];
}

template <typename T>
void add_loop(const T* a, const T* b, T* c, size_t n) {
  for (size_t i = 0; i < n; ++i) c[i] = a[i] + b[i];
}

template <typename T>
void triad_loop(T* a, const T* b, const T* c, T s, size_t n) {
  for (size_t i = 0; i < n; ++i) {
    const T t = s * c[i];  // first rounding
    a[i] = b[i] + t;       // second rounding
  }
}

// Dot product accumulated in long double with Neumaier's compensation, also
// carried in long double.  Each product is formed in long double: exact for
// float inputs (48-bit product), rounded to 64 bits for double inputs
// (relative error <= 2^-64 per term).  The compensated sum's error is about
// 2^-63 of the result plus n^2 * 2^-128 of sum|a[i]*b[i]|, i.e. far below the
// 1e-12 relative bound the GPU result is held to, for every n used here.
// -ffast-math must stay off: it would let the optimiser cancel the
// compensation terms algebraically.
template <typename T>
long double dot_loop(const T* a, const T* b, size_t n) {
  long double sum = 0.0L;
  long double comp = 0.0L;
  for (size_t i = 0; i < n; ++i) {
    const long double x = (long double)a[i] * (long double)b[i];
    const long double t = sum + x;
    const long double abs_sum = sum < 0 ? -sum : sum;
    const long double abs_x = x < 0 ? -x : x;
    if (abs_sum >= abs_x) {
      comp += (sum - t) + x;
    } else {
      comp += (x - t) + sum;
    }
    sum = t;
  }
  return sum + comp;
}

// The uncompensated long-double running sum: the brute-force definition the
// compensated loop is cross-checked against on small n.
template <typename T>
long double dot_plain_loop(const T* a, const T* b, size_t n) {
  long double sum = 0.0L;
  for (size_t i = 0; i < n; ++i) sum += (long double)a[i] * (long double)b[i];
  return sum;
}

// sum_i |a[i]*b[i]|, for reporting the condition number of a dot product.
template <typename T>
long double dot_abs_loop(const T* a, const T* b, size_t n) {
  long double sum = 0.0L;
  for (size_t i = 0; i < n; ++i) {
    const long double x = (long double)a[i] * (long double)b[i];
    sum += x < 0 ? -x : x;
  }
  return sum;
}

// LDS streaming microkernel (the library's own definition of the shared-memory
// benchmark subject of Table 1; the paper gives none).  Arrays are cut into
// tiles of 1024 16-byte vectors; `per_vec` = elements per vector (2 for double,
// 4 for float).  One round: x'[j] = x[(j + 1) mod 1024] + c on whole vectors,
// i.e. every element moves one vector down and gets c added once (one rounded
// add).  `rep` rounds, done literally, round by round, on a scratch copy of
// the tile.  n must be a whole number of tiles (returns -1 otherwise).
template <typename T>
int lds_stream_loop(const T* in, T* out, T c, size_t n, unsigned rep) {
  const size_t tile_vecs = 1024;
  const size_t per_vec = 16 / sizeof(T);
  const size_t tile = tile_vecs * per_vec;
  if (n % tile != 0) return -1;
  T* cur = new T[tile];
  T* next = new T[tile];
  for (size_t t0 = 0; t0 < n; t0 += tile) {
    for (size_t e = 0; e < tile; ++e) cur[e] = in[t0 + e];
    for (unsigned r = 0; r < rep; ++r) {
      for (size_t j = 0; j < tile_vecs; ++j) {
        const size_t src = (j + 1) % tile_vecs;
        for (size_t l = 0; l < per_vec; ++l) next[j * per_vec + l] = cur[src * per_vec + l] + c;
      }
      T* tmp = cur; cur = next; next = tmp;
    }
    for (size_t e = 0; e < tile; ++e) out[t0 + e] = cur[e];
  }
  delete[] cur;
  delete[] next;
  return 0;
}

}  // namespace

extern "C" {

// fp64 -----------------------------------------------------------------------
void oracle_copy_f64(const double* a, double* c, size_t n) { copy_loop(a, c, n); }
void oracle_scale_f64(double* b, const double* c, double s, size_t n) { scale_loop(b, c, s, n); }
void oracle_add_f64(const double* a, const double* b, double* c, size_t n) { add_loop(a, b, c, n); }
void oracle_triad_f64(double* a, const double* b, const double* c, double s, size_t n) {
  triad_loop(a, b, c, s, n);
}
// Writes the long-double value to *out_ld (16 bytes of storage, may be NULL)
// and returns it rounded once to double.
double oracle_dot_f64(const double* a, const double* b, size_t n, long double* out_ld) {
  const long double r = dot_loop(a, b, n);
  if (out_ld) *out_ld = r;
  return (double)r;
}
double oracle_dot_plain_f64(const double* a, const double* b, size_t n) {
  return (double)dot_plain_loop(a, b, n);
}
double oracle_dot_abs_f64(const double* a, const double* b, size_t n) {
  return (double)dot_abs_loop(a, b, n);
}

// fp32: the scalar crosses the interface as double and is rounded once to
// float here, before the loop. -------------------------------------------------
void oracle_copy_f32(const float* a, float* c, size_t n) { copy_loop(a, c, n); }
void oracle_scale_f32(float* b, const float* c, double s, size_t n) { scale_loop(b, c, (float)s, n); }
void oracle_add_f32(const float* a, const float* b, float* c, size_t n) { add_loop(a, b, c, n); }
void oracle_triad_f32(float* a, const float* b, const float* c, double s, size_t n) {
  triad_loop(a, b, c, (float)s, n);
}
double oracle_dot_f32(const float* a, const float* b, size_t n, long double* out_ld) {
  const long double r = dot_loop(a, b, n);
  if (out_ld) *out_ld = r;
  return (double)r;
}
double oracle_dot_plain_f32(const float* a, const float* b, size_t n) {
  return (double)dot_plain_loop(a, b, n);
}
double oracle_dot_abs_f32(const float* a, const float* b, size_t n) {
  return (double)dot_abs_loop(a, b, n);
}

int oracle_lds_stream_f64(const double* in, double* out, double c, size_t n, unsigned rep) {
  return lds_stream_loop(in, out, c, n, rep);
}
int oracle_lds_stream_f32(const float* in, float* out, double c, size_t n, unsigned rep) {
  return lds_stream_loop(in, out, (float)c, n, rep);
}

}  // extern "C"
