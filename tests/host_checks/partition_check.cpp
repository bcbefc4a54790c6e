// Host-only check of the work decomposition in paper_2510_00932_amd/csrc/launch_plan.hpp: for every
// launch shape, replay which lane of which workgroup touches which element (the same index
// functions the kernels call) and verify that every element of the array is touched exactly
// once, nothing outside it is touched, and no launch exceeds what one dispatch can hold.
// Small arrays are replayed element by element; huge element counts (up to 2^62) are checked
// through the segment and chunk arithmetic.  Built by tests/test_host_checks.py, also with
// -fsanitize=address,undefined.  Prints "partition ok ..." and returns 0, or the first failure.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "launch_plan.hpp"

using namespace opal::plan;

static int g_failures = 0;
#define EXPECT(cond, ...)                                      \
  do {                                                         \
    if (!(cond)) {                                             \
      if (g_failures < 20) {                                   \
        std::printf("FAIL %s:%d %s | ", __FILE__, __LINE__, #cond); \
        std::printf(__VA_ARGS__);                              \
        std::printf("\n");                                     \
      }                                                        \
      ++g_failures;                                            \
    }                                                          \
  } while (0)

struct Cover {
  std::vector<uint8_t> count;
  size_t outside = 0;
  explicit Cover(size_t n) : count(n, 0) {}
  void touch(size_t i) {
    if (i < count.size()) { if (count[i] < 255) ++count[i]; } else ++outside;
  }
  bool exact() const {
    if (outside) return false;
    for (uint8_t c : count) if (c != 1) return false;
    return true;
  }
};

// stream_kernel: lane l of workgroup g moves vector g*block + l if it is below nvec; the last
// workgroup moves the head and tail scalars.  One launch per segment, on shifted pointers.
static void replay_stream(uintptr_t addr, size_t n, unsigned elem, unsigned block, size_t max_items, Cover& c) {
  const unsigned lanes = 16 / elem;
  const Split sp = split(addr, n, elem);
  const size_t count = segment_count(sp, block, max_items);
  for (size_t s = 0; s < count; ++s) {
    const Segment g = segment(sp, lanes, block, s, max_items);
    EXPECT((uint64_t)g.groups * block <= max_items, "groups %u block %u", g.groups, block);
    const Split local{g.head, g.nvec, (unsigned)(g.n - g.head - g.nvec * lanes)};
    for (unsigned grp = 0; grp < g.groups; ++grp) {
      for (unsigned l = 0; l < block; ++l) {
        const size_t v = stream_vector(block, grp, l);
        if (v < g.nvec)
          for (unsigned e = 0; e < lanes; ++e) c.touch(g.elem_offset + g.head + v * lanes + e);
      }
      if (grp == g.groups - 1)
        for (unsigned k = 0; k < local.head + local.tail; ++k) c.touch(g.elem_offset + edge_element(local, lanes, k));
    }
  }
}

// paced_stream_kernel / paced_dot_kernel.
static void replay_paced(uintptr_t addr, size_t n, unsigned elem, unsigned waves, unsigned k, unsigned set_bit, Cover& c) {
  const unsigned lanes = 16 / elem;
  const Split sp = split(addr, n, elem);
  const Paced p = paced(sp, waves, k, set_bit);
  for (unsigned w = 0; w < waves; ++w) {
    const unsigned set = paced_set(w, set_bit), index = paced_index(w, set_bit);
    EXPECT(index < waves / 2, "wave %u index %u", w, index);
    for (size_t chunk = set; chunk < p.nchunks; chunk += 2)
      for (unsigned kk = 0; kk < k; ++kk) {
        const size_t run = paced_run(p, chunk, index, kk);
        for (unsigned l = 0; l < kRunVectors; ++l)
          for (unsigned e = 0; e < lanes; ++e) c.touch(sp.head + (run * kRunVectors + l) * lanes + e);
      }
    for (size_t run = p.rest_run0 + w; run < p.total_runs; run += waves)
      for (unsigned l = 0; l < kRunVectors; ++l)
        if (run * kRunVectors + l < sp.nvec)
          for (unsigned e = 0; e < lanes; ++e) c.touch(sp.head + (run * kRunVectors + l) * lanes + e);
    if (w == waves - 1)
      for (unsigned i = 0; i < sp.head + sp.tail; ++i) c.touch(edge_element(sp, lanes, i));
  }
}

// The order in which a two-input paced kernel loads its second input and stores (matched_run): for
// every wavefront and chunk the K slots must name every run 0..K-1 once, and, where adding a slot's
// stride stays inside address bits 20-21, the run named for slot k must share the upper two class
// bits of the first input's run k.
static void check_matched(uintptr_t in0, uintptr_t in1, size_t chunks) {
  const size_t stride = (size_t)1 << kMatchedStrideShift;
  for (size_t chunk = 0; chunk < chunks; ++chunk)
    for (unsigned index = 0; index < 1024; index += 37) {
      const uintptr_t a0 = in0 + chunk * kMatchedRuns * stride + (uintptr_t)index * kBodyAlignBytes;
      const uintptr_t a1 = in1 + chunk * kMatchedRuns * stride + (uintptr_t)index * kBodyAlignBytes;
      unsigned seen = 0;
      for (unsigned k = 0; k < kMatchedRuns; ++k) {
        const unsigned kk = matched_run(a0, a1, k);
        EXPECT(kk < kMatchedRuns, "matched_run out of range: %u", kk);
        seen |= 1u << kk;
        // class equality as far as the model goes: compare on addresses whose bits 20-21 hold the slot numbers
        // themselves (no carry out of the field), all other bits as in a0 / a1
        const uintptr_t field = (uintptr_t)3 << kMatchedStrideShift;
        const uintptr_t x0 = (a0 & ~field) | ((((a0 >> kMatchedStrideShift) + k) & 3u) << kMatchedStrideShift);
        const uintptr_t x1 = (a1 & ~field) | ((((a1 >> kMatchedStrideShift) + kk) & 3u) << kMatchedStrideShift);
        EXPECT(((channel_class(x0) ^ channel_class(x1)) & 0xCu) == 0u, "classes differ: a0 %zx a1 %zx k %u kk %u",
               (size_t)a0, (size_t)a1, k, kk);
      }
      EXPECT(seen == (1u << kMatchedRuns) - 1u, "not a permutation: a0 %zx a1 %zx", (size_t)a0, (size_t)a1);
      unsigned seen_flipped = 0;
      for (unsigned k = 0; k < kMatchedRuns; ++k) seen_flipped |= 1u << matched_run(a0, a1, k, 1u);
      EXPECT(seen_flipped == (1u << kMatchedRuns) - 1u, "not a permutation under the other assumption: a0 %zx a1 %zx",
             (size_t)a0, (size_t)a1);
    }
}

// dot_partial_kernel (tiled).
static void replay_tiled(uintptr_t addr, size_t n, unsigned elem, unsigned block, unsigned unroll, unsigned max_groups,
                         Cover& c) {
  const unsigned lanes = 16 / elem;
  const Split sp = split(addr, n, elem);
  const Tiled t = tiled(sp, block, unroll, max_groups);
  EXPECT(t.groups >= 1 && t.groups <= max_groups, "groups %u", t.groups);
  for (unsigned g = 0; g < t.groups; ++g) {
    for (size_t tile = g; tile < t.full_tiles; tile += t.groups)
      for (unsigned tid = 0; tid < block; ++tid)
        for (unsigned u = 0; u < unroll; ++u) {
          const size_t v = tile * t.tile_vectors + tid + (size_t)u * block;
          for (unsigned e = 0; e < lanes; ++e) c.touch(sp.head + v * lanes + e);
        }
    if (g == tiled_ragged_group(t)) {
      for (size_t v = t.full_tiles * t.tile_vectors; v < sp.nvec; ++v)
        for (unsigned e = 0; e < lanes; ++e) c.touch(sp.head + v * lanes + e);
      for (unsigned i = 0; i < sp.head + sp.tail; ++i) c.touch(edge_element(sp, lanes, i));
    }
  }
}

static void check_split(uintptr_t addr, size_t n, unsigned elem) {
  const unsigned lanes = 16 / elem;
  const Split sp = split(addr, n, elem);
  EXPECT((size_t)sp.head + sp.nvec * lanes + sp.tail == n, "addr %zu n %zu", (size_t)addr, n);
  EXPECT(sp.tail < lanes, "tail %u", sp.tail);
  EXPECT(sp.head < kBodyAlignBytes / elem, "head %u", sp.head);
  if (sp.nvec > 0 || sp.tail > 0) EXPECT((addr + (uintptr_t)sp.head * elem) % kBodyAlignBytes == 0, "body not on a 1 KiB boundary");
}

// Arithmetic-only checks for element counts no array could be replayed for.
static void check_huge(uintptr_t addr, size_t n, unsigned elem) {
  const unsigned lanes = 16 / elem;
  check_split(addr, n, elem);
  const Split sp = split(addr, n, elem);
  for (unsigned block : {64u, 256u}) {
    const size_t count = segment_count(sp, block);
    // look at the first few and the last few segments; the middle ones are all alike
    size_t expect_off = 0, covered = 0;
    for (size_t s = 0; s < count; ++s) {
      if (s > 3 && s + 3 < count) {   // skip the middle: full segments of segment_vectors each
        const size_t skip = count - 3 - s;
        expect_off += skip * segment_vectors(block) * lanes;
        covered += skip * segment_vectors(block) * lanes;
        s += skip - 1;
        continue;
      }
      const Segment g = segment(sp, lanes, block, s);
      EXPECT((uint64_t)g.groups * block <= kMaxWorkItems, "segment %zu groups %u", s, g.groups);
      EXPECT((size_t)g.groups * block >= g.nvec, "segment %zu does not cover its vectors", s);
      EXPECT(g.elem_offset == expect_off, "segment %zu offset %zu expected %zu", s, g.elem_offset, expect_off);
      EXPECT(s == 0 || g.head == 0, "only segment 0 has a head");
      expect_off = g.elem_offset + g.n;
      covered += g.n;
    }
    EXPECT(covered == n, "segments cover %zu of %zu", covered, n);
  }
  for (unsigned waves : {1024u, 2048u})
    for (unsigned k : {4u, 8u}) {
      const Paced p = paced(sp, waves, k, 3);
      EXPECT(p.rest_run0 == p.nchunks * p.chunk_runs, "rest");
      EXPECT(p.rest_run0 <= p.total_runs && p.total_runs - p.rest_run0 <= p.chunk_runs, "rest larger than a chunk");
      EXPECT(p.total_runs * kRunVectors >= sp.nvec && (p.total_runs == 0 || (p.total_runs - 1) * kRunVectors < sp.nvec), "runs");
      if (p.nchunks > 0) {
        EXPECT(paced_run(p, p.nchunks - 1, waves / 2 - 1, k - 1) == p.rest_run0 - 1, "last run of the last chunk");
        EXPECT(paced_run(p, 0, 0, 0) == 0, "first run");
      }
    }
  const Tiled t = tiled(sp, 256, 4, 256);
  EXPECT(t.full_tiles * t.tile_vectors <= sp.nvec && sp.nvec - t.full_tiles * t.tile_vectors < t.tile_vectors, "tiles");
  EXPECT(tiled_ragged_group(t) < t.groups, "ragged group");
}

// Where a learnt order is remembered and which order a launch uses (order_key, order_of_launch).
static void check_order_learning() {
  unsigned used[kOrderSlots] = {0};
  for (uintptr_t a0 = 0x7f0000000000ull; a0 < 0x7f0000000000ull + ((uintptr_t)64 << 21); a0 += (uintptr_t)1 << 21)
    for (uintptr_t d : {(uintptr_t)1 << 31, ((uintptr_t)1 << 31) + 1024, (uintptr_t)3 << 30}) {
      const OrderKey k = order_key(a0, a0 + d, (size_t)1 << 27, 0u);
      EXPECT(k.hi != 0u && k.slot < kOrderSlots, "key %x %x slot %u", k.lo, k.hi, k.slot);
      ++used[k.slot];
      const OrderKey again = order_key(a0, a0 + d, (size_t)1 << 27, 0u);
      EXPECT(again.lo == k.lo && again.hi == k.hi && again.slot == k.slot, "key not a function of its arguments");
      const OrderKey swapped = order_key(a0 + d, a0, (size_t)1 << 27, 0u), other_n = order_key(a0, a0 + d, ((size_t)1 << 27) + 64, 0u),
                     later = order_key(a0, a0 + d, (size_t)1 << 27, 1u);
      EXPECT(swapped.lo != k.lo || swapped.hi != k.hi, "swapped inputs share a key");
      EXPECT(other_n.lo != k.lo || other_n.hi != k.hi, "another n shares a key");
      EXPECT(later.lo != k.lo || later.hi != k.hi, "another epoch shares a key");
    }
  unsigned most = 0, nonempty = 0;
  for (unsigned u : used) { most = u > most ? u : most; nonempty += u != 0; }
  EXPECT(nonempty >= kOrderSlots / 2 && most <= 12, "192 keys fall into %u slots, %u into one", nonempty, most);
  for (unsigned first : {0u, 1u}) {
    for (uint32_t cycle : {0u, kOrderCycle, 5u * kOrderCycle}) {
      for (uint32_t i = 0; i < 4; ++i)
        EXPECT(order_of_launch(cycle + i, first, 10u, 20u) == ((first ^ i) & 1u), "launch %u of a cycle, first %u", i, first);
      for (uint32_t i = 4; i < kOrderCycle; i += 41) {
        EXPECT(order_of_launch(cycle + i, first, 10u, 20u) == 0u, "faster order 0 not taken");
        EXPECT(order_of_launch(cycle + i, first, 20u, 10u) == 1u, "faster order 1 not taken");
        EXPECT(order_of_launch(cycle + i, first, 10u, 10u) == 0u, "tie");
      }
    }
  }
}

int main() {
  size_t cases = 0;
  check_order_learning();
  const size_t sizes[] = {0, 1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513,
                          1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8193, 12289, 16385, 20000, 40961};
  for (unsigned elem : {8u, 4u})
    for (uintptr_t mis : {0u, 1u, 2u, 3u, 5u, 63u, 127u, 128u, 255u})
      for (size_t n : sizes) {
        const uintptr_t addr = 0x10000 + mis * elem;
        check_split(addr, n, elem);
        for (unsigned block : {64u, 256u})
          for (size_t max_items : {kMaxWorkItems, (size_t)256, (size_t)1024}) {   // one launch, or several small ones
            Cover c(n);
            replay_stream(addr, n, elem, block, max_items, c);
            EXPECT(c.exact(), "stream elem %u mis %zu n %zu block %u max %zu", elem, (size_t)mis, n, block, max_items);
            ++cases;
          }
        // small wave counts so that small arrays still have several chunks, a rest and a ragged run
        for (unsigned waves : {16u, 64u})
          for (unsigned k : {1u, 4u, 8u})
            for (unsigned set_bit : {0u, 3u}) {
              Cover c(n);
              replay_paced(addr, n, elem, waves, k, set_bit, c);
              EXPECT(c.exact(), "paced elem %u mis %zu n %zu waves %u k %u bit %u", elem, (size_t)mis, n, waves, k, set_bit);
              ++cases;
            }
        for (unsigned block : {64u, 256u})
          for (unsigned max_groups : {1u, 3u, 256u}) {
            Cover c(n);
            replay_tiled(addr, n, elem, block, 4, max_groups, c);
            EXPECT(c.exact(), "tiled elem %u mis %zu n %zu block %u groups<=%u", elem, (size_t)mis, n, block, max_groups);
            ++cases;
          }
      }
  // paced shape on arrays of several chunks (256 or 512 runs per chunk at k = 1) with ragged ends
  for (unsigned elem : {8u, 4u})
    for (uintptr_t mis : {0u, 1u, 3u})
      for (size_t n : {(size_t)65539, (size_t)300001, (size_t)1048576 + 77})
        for (unsigned waves : {512u, 1024u})
          for (unsigned k : {1u, 4u})
            for (unsigned set_bit : {0u, 2u, 3u, 8u}) {
              Cover c(n);
              replay_paced(0x30000 + mis * elem, n, elem, waves, k, set_bit, c);
              EXPECT(c.exact(), "paced elem %u mis %zu n %zu waves %u k %u bit %u", elem, (size_t)mis, n, waves, k, set_bit);
              ++cases;
            }
  // the library's own wave counts on a mid-sized array (several chunks of 1024 * 8 runs)
  for (unsigned elem : {8u, 4u}) {
    const size_t n = ((size_t)3 << 22) / elem * 8 + 77;   // 24 MiB and a bit
    for (unsigned waves : {1024u, 2048u})
      for (unsigned k : {4u, 8u}) {
        Cover c(n);
        replay_paced(0x20000 + elem, n, elem, waves, k, 3, c);
        EXPECT(c.exact(), "paced mid elem %u waves %u k %u", elem, waves, k);
        ++cases;
      }
  }
  // element counts beyond any replay: every boundary of the segment arithmetic up to 2^62
  for (unsigned elem : {8u, 4u})
    for (int lg = 28; lg <= 62 - (elem == 8 ? 3 : 2); ++lg)
      for (long d : {-17L, -1L, 0L, 1L, 2049L})
        for (uintptr_t mis : {0u, 1u, 3u}) {
          check_huge(0x40000 + mis * elem, ((size_t)1 << lg) + (size_t)d, elem);
          ++cases;
        }
  for (size_t n : {((size_t)1 << 33), ((size_t)1 << 40), ((size_t)1 << 33) * 3 + 5}) {
    const Split sp = split(0x1000, n, 8);
    EXPECT(segment_count(sp, 64) == (sp.nvec + segment_vectors(64) - 1) / segment_vectors(64), "segment count");
    EXPECT(segment_count(sp, 64) > 1, "2^33 fp64 elements need more than one launch");
  }
  // matched order of the second input: aligned and misaligned pairs of arrays, distances with every class bit
  {
    const uintptr_t base = (uintptr_t)0x7f42ull << 32;
    const uintptr_t distances[] = {0, 4096, 8192, 12288, 1024, 3072, 15360, (uintptr_t)1 << 20, (uintptr_t)2 << 20, (uintptr_t)3 << 20,
                                   ((uintptr_t)1 << 20) + 4096, ((uintptr_t)2 << 20) + 8192, (uintptr_t)256 << 20,
                                   ((uintptr_t)256 << 20) + 8192, (uintptr_t)2400001280u, 8, 4104, (uintptr_t)0x123456789};
    for (uintptr_t d : distances) {
      check_matched(base, base + ((uintptr_t)1 << 31) + d, 96);
      check_matched(base + 8 + d, base, 96);
      ++cases;
    }
    const Split whole{0u, (size_t)1 << 27, 0u};
    EXPECT(paced(whole, 2048, 4, 3).matched, "the two-input shape in use is matched");
    EXPECT(!paced(whole, 2048, 8, 3).matched && !paced(whole, 1024, 4, 3).matched, "other shapes are not");
  }
  if (g_failures) {
    std::printf("partition check: %d failure(s)\n", g_failures);
    return 1;
  }
  std::printf("partition ok: %zu cases\n", cases);
  return 0;
}
