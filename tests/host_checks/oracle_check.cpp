// The CPU oracle (oracle/oracle.cpp, linked in) run natively under AddressSanitizer and
// UndefinedBehaviorSanitizer on exactly-sized heap arrays: every loop bound, every index and
// every scratch buffer of the oracle is exercised for the edge sizes (0, 1, odd, one tile,
// several tiles), and the results are compared with facts that need no second implementation:
// constant fills have scalar closed forms, ramps are their own index, integer-valued data
// makes every dot sum exact.  Built and run by tests/test_host_checks.py.
#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
void oracle_copy_f64(const double* a, double* c, size_t n);
void oracle_scale_f64(double* b, const double* c, double s, size_t n);
void oracle_add_f64(const double* a, const double* b, double* c, size_t n);
void oracle_triad_f64(double* a, const double* b, const double* c, double s, size_t n);
double oracle_dot_f64(const double* a, const double* b, size_t n, long double* out_ld);
double oracle_dot_plain_f64(const double* a, const double* b, size_t n);
double oracle_dot_abs_f64(const double* a, const double* b, size_t n);
void oracle_copy_f32(const float* a, float* c, size_t n);
void oracle_scale_f32(float* b, const float* c, double s, size_t n);
void oracle_add_f32(const float* a, const float* b, float* c, size_t n);
void oracle_triad_f32(float* a, const float* b, const float* c, double s, size_t n);
double oracle_dot_f32(const float* a, const float* b, size_t n, long double* out_ld);
double oracle_dot_plain_f32(const float* a, const float* b, size_t n);
double oracle_dot_abs_f32(const float* a, const float* b, size_t n);
int oracle_lds_stream_f64(const double* in, double* out, double c, size_t n, unsigned rep);
int oracle_lds_stream_f32(const float* in, float* out, double c, size_t n, unsigned rep);
}

static int g_failures = 0;
#define EXPECT(cond, ...)                                           \
  do {                                                              \
    if (!(cond)) {                                                  \
      if (g_failures < 20) {                                        \
        std::printf("FAIL %s:%d %s | ", __FILE__, __LINE__, #cond); \
        std::printf(__VA_ARGS__);                                   \
        std::printf("\n");                                          \
      }                                                             \
      ++g_failures;                                                 \
    }                                                               \
  } while (0)

template <typename T> struct Api;
template <> struct Api<double> {
  static void copy(const double* a, double* c, size_t n) { oracle_copy_f64(a, c, n); }
  static void scale(double* b, const double* c, double s, size_t n) { oracle_scale_f64(b, c, s, n); }
  static void add(const double* a, const double* b, double* c, size_t n) { oracle_add_f64(a, b, c, n); }
  static void triad(double* a, const double* b, const double* c, double s, size_t n) { oracle_triad_f64(a, b, c, s, n); }
  static double dot(const double* a, const double* b, size_t n) { return oracle_dot_f64(a, b, n, nullptr); }
  static double dot_plain(const double* a, const double* b, size_t n) { return oracle_dot_plain_f64(a, b, n); }
  static double dot_abs(const double* a, const double* b, size_t n) { return oracle_dot_abs_f64(a, b, n); }
  static int lds(const double* in, double* out, double c, size_t n, unsigned rep) { return oracle_lds_stream_f64(in, out, c, n, rep); }
};
template <> struct Api<float> {
  static void copy(const float* a, float* c, size_t n) { oracle_copy_f32(a, c, n); }
  static void scale(float* b, const float* c, double s, size_t n) { oracle_scale_f32(b, c, s, n); }
  static void add(const float* a, const float* b, float* c, size_t n) { oracle_add_f32(a, b, c, n); }
  static void triad(float* a, const float* b, const float* c, double s, size_t n) { oracle_triad_f32(a, b, c, s, n); }
  static double dot(const float* a, const float* b, size_t n) { return oracle_dot_f32(a, b, n, nullptr); }
  static double dot_plain(const float* a, const float* b, size_t n) { return oracle_dot_plain_f32(a, b, n); }
  static double dot_abs(const float* a, const float* b, size_t n) { return oracle_dot_abs_f32(a, b, n); }
  static int lds(const float* in, float* out, double c, size_t n, unsigned rep) { return oracle_lds_stream_f32(in, out, c, n, rep); }
};

// volatile: the scalar closed forms must be rounded operation by operation, like the oracle's
template <typename T>
static void check_type(const char* name) {
  const size_t sizes[] = {0, 1, 2, 3, 5, 64, 65, 1000, 4097};
  const T a0 = (T)1.25, b0 = (T)0.3, c0 = (T)2.7;
  const double s = 0.4;
  const T sT = (T)s;
  for (size_t n : sizes) {
    std::vector<T> a(n, a0), b(n, b0), c(n, c0);   // exactly n elements on the heap
    Api<T>::copy(a.data(), c.data(), n);
    for (size_t i = 0; i < n; ++i) EXPECT(c[i] == a0, "%s copy n=%zu i=%zu", name, n, i);
    Api<T>::scale(b.data(), c.data(), s, n);
    volatile T prod = sT * a0;
    for (size_t i = 0; i < n; ++i) EXPECT(b[i] == prod, "%s scale n=%zu i=%zu", name, n, i);
    Api<T>::add(a.data(), b.data(), c.data(), n);
    volatile T sum = a0 + prod;
    for (size_t i = 0; i < n; ++i) EXPECT(c[i] == sum, "%s add n=%zu i=%zu", name, n, i);
    Api<T>::triad(a.data(), b.data(), c.data(), s, n);
    volatile T t1 = sT * sum;
    volatile T t2 = prod + t1;
    for (size_t i = 0; i < n; ++i) EXPECT(a[i] == t2, "%s triad n=%zu i=%zu", name, n, i);
    // ramp: element i is its own index; integer data keeps every dot sum exact
    std::vector<T> r(n), ones(n, (T)1), out(n, (T)-1);
    for (size_t i = 0; i < n; ++i) r[i] = (T)(i % 1024);
    Api<T>::copy(r.data(), out.data(), n);
    for (size_t i = 0; i < n; ++i) EXPECT(out[i] == (T)(i % 1024), "%s ramp copy n=%zu i=%zu", name, n, i);
    double want = 0.0;
    for (size_t i = 0; i < n; ++i) want += (double)(i % 1024);
    EXPECT(Api<T>::dot(r.data(), ones.data(), n) == want, "%s dot ramp n=%zu", name, n);
    EXPECT(Api<T>::dot_plain(r.data(), ones.data(), n) == want, "%s dot_plain ramp n=%zu", name, n);
    EXPECT(Api<T>::dot_abs(r.data(), ones.data(), n) == want, "%s dot_abs ramp n=%zu", name, n);
    std::vector<T> h(n, (T)1.5), two(n, (T)2);
    EXPECT(Api<T>::dot(h.data(), two.data(), n) == 3.0 * (double)n, "%s dot const n=%zu", name, n);
    for (size_t i = 0; i < n; ++i) two[i] = (i & 1) ? (T)-2 : (T)2;
    EXPECT(Api<T>::dot(h.data(), two.data(), n) == ((n & 1) ? 3.0 : 0.0), "%s dot alternating n=%zu", name, n);
    EXPECT(Api<T>::dot_abs(h.data(), two.data(), n) == 3.0 * (double)n, "%s dot_abs alternating n=%zu", name, n);
  }
  // LDS microkernel: whole tiles only; rotation by rep vectors with c added rep times
  const size_t per_vec = 16 / sizeof(T), tile = 1024 * per_vec;
  for (size_t tiles : {(size_t)0, (size_t)1, (size_t)3})
    for (unsigned rep : {0u, 1u, 5u, 1025u}) {
      const size_t n = tiles * tile;
      std::vector<T> in(n), out(n, (T)-7);
      for (size_t i = 0; i < n; ++i) in[i] = (T)((i / per_vec) % 1024 + 4096 * (i / tile));   // vector index within its tile, tagged by tile
      EXPECT(Api<T>::lds(in.data(), out.data(), 1.0, n, rep) == 0, "%s lds status", name);
      for (size_t i = 0; i < n; ++i) {
        const size_t j = (i / per_vec) % 1024, t = i / tile;
        const T expect = (T)((j + rep) % 1024 + 4096 * t + rep);   // small integers: exact
        EXPECT(out[i] == expect, "%s lds tiles=%zu rep=%u i=%zu got %g want %g", name, tiles, rep, i, (double)out[i], (double)expect);
      }
    }
  std::vector<T> ragged(tile + 1), out(tile + 1);
  EXPECT(Api<T>::lds(ragged.data(), out.data(), 0.0, tile + 1, 1) == -1, "%s lds must refuse a ragged size", name);
}

int main() {
  check_type<double>("f64");
  check_type<float>("f32");
  // compensation: 1e30 + 1 - 1e30 is 1 for the compensated sum, 0 for the plain long-double one... in double inputs
  {
    std::vector<double> a = {1e30, 1.0, -1e30}, b = {1.0, 1.0, 1.0};
    EXPECT(oracle_dot_f64(a.data(), b.data(), 3, nullptr) == 1.0, "compensated dot");
  }
  if (g_failures) {
    std::printf("oracle check: %d failure(s)\n", g_failures);
    return 1;
  }
  std::printf("oracle ok\n");
  return 0;
}
