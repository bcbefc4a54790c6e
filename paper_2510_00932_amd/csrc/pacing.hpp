// Clock-paced issue for the persistent ("paced") launch shapes, CDNA4 / gfx950.
//
// Why.  HBM moves most bytes when, chip-wide, it sees one stream at a time in large bursts: a
// burst of reads, then a burst of writes, instead of reads and writes of all wavefronts mixed
// at random (every change of direction on a DRAM channel costs bus turnaround time, and
// interleaved streams disturb each other's open rows).  No wavefront can see what the others
// do, but all of them can read the same constant-rate counter (s_memrealtime, 100 MHz on
// MI355X, the same value on every compute unit to within a few ticks).  So the wavefronts of a
// paced kernel agree on a timetable instead of on messages: time is cut into periods, set 0
// issues its load burst at the start of a period and its store burst three quarters of a
// period later, set 1 does the same half a period later, and the memory system sees
// load(0) store(1) load(1) store(0) ... with nothing else in between.
//
// The timetable is open loop, so two things keep it honest.  (1) A wavefront that reaches its
// load point late does not wait: it goes at once and catches up with the slack of the next
// periods.  (2) If memory falls behind the timetable for longer (a backlog of stores that
// have not drained), late wavefronts would keep issuing into the wrong phase and the whole
// kernel would degrade into unordered traffic for good.  A few "reporter" wavefronts therefore
// publish how late they are (beyond a tolerance) in a small block of device words, every
// wavefront reads one of those words per period, and all of them push their timetable back by
// the largest lateness published: a common pause in which the backlog drains, after which the
// timetable holds again.  The words are replicated (one copy per reader class, on different
// memory channels) so that reading them is not itself a hot spot.
//
// Nothing here affects results: the timetable only decides when a wavefront issues loads and
// stores it would issue anyway.  Every wait is bounded by a poll count, so a kernel ends even
// if the counter stood still.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch_plan.hpp"

namespace opal {

constexpr unsigned kFeedbackCopies = 64;           // one per lane of a reporting wavefront
constexpr unsigned kFeedbackStrideWords = 544;     // 4352 bytes apart: different channels and banks
constexpr unsigned kFeedbackWords = kFeedbackCopies * kFeedbackStrideWords;
constexpr unsigned kReporterShift = 26;            // about one wavefront in 64 reports (pace_reporter)
constexpr int kPacePolls = 4096;                   // bound of one wait (a legitimate wait is a few periods)
constexpr unsigned kStretchBits = 20;              // a feedback word is  launch stamp << 20 | stretch

// Timetable of one kernel, in ticks of the constant-rate counter.  period == 0: unpaced.
struct Pace {
  uint32_t period;        // one load burst and one store burst of each set per period
  uint32_t second_input;  // offset of the burst that loads the second input (0: together with the first)
  uint32_t store;         // offset of the store burst (0: store as soon as the data is there)
  uint32_t gap;           // ticks between the accesses of one burst (0: all at once)
  uint32_t tolerance;     // lateness beyond which a reporter pushes the timetable back
  unsigned long long* feedback;   // kFeedbackWords device words, or nullptr (no feedback)
  unsigned* order_words;          // plan::kOrderWords device words, or nullptr (matched order: nothing is learnt)
  uint32_t order_epoch;           // part of the key under which an order is remembered: a new value starts afresh
};

__device__ __forceinline__ uint64_t pace_clock64() { return __builtin_amdgcn_s_memrealtime(); }
__device__ __forceinline__ uint32_t pace_clock() { return (uint32_t)__builtin_amdgcn_s_memrealtime(); }

// Returns when the counter has reached `when` (wrap-safe), or after kPacePolls polls.
__device__ __forceinline__ void pace_wait_until(uint32_t when) {
  for (int i = 0; i < kPacePolls; ++i) {
    if ((int32_t)(pace_clock() - when) >= 0) return;
    __builtin_amdgcn_s_sleep(1);
  }
}

// Which wavefronts report lateness: a fixed pseudo-random 1/64 of them, so that reporters sit on
// every XCD, in both sets and on unrelated compute units (any regular stride would pick one XCD
// or one set, because workgroups are dealt out round-robin).
__device__ __forceinline__ bool pace_reporter(unsigned wave) { return ((wave * 0x9E3779B1u) >> kReporterShift) == 0u; }

// Per-wavefront state of the timetable (all members wave-uniform).
struct PaceState {
  uint32_t next;      // time of this wavefront's next load burst, before stretch
  uint32_t stretch;   // how far the timetable has been pushed back so far
  uint64_t stamp;     // identifies the launch in feedback words
};

__device__ __forceinline__ PaceState pace_begin(const Pace& p, unsigned set) {
  PaceState st;
  const uint64_t t = pace_clock64();
  // Period boundaries are counted on the 64-bit counter, so that wavefronts starting on either
  // side of a wrap of its low 32 bits still agree on them.
  st.next = (uint32_t)((t / p.period + 1u) * p.period) + set * (p.period / 2u);
  st.stretch = 0;
  st.stamp = (t >> 9) & (((uint64_t)1 << 44) - 1);
  return st;
}

// Call before a load burst: waits for the wavefront's turn, or, if it is late by more than the
// tolerance and this wavefront is a reporter, publishes the lateness.  Returns the time base
// (turn + stretch) that second_input / store offsets are relative to.
__device__ __forceinline__ uint32_t pace_turn(const Pace& p, PaceState& st, bool reporter) {
  const uint32_t turn = st.next + st.stretch;
  const int32_t late = (int32_t)(pace_clock() - turn);
  if (late > (int32_t)p.tolerance) {
    if (reporter && p.feedback != nullptr) {
      uint32_t s = st.stretch + (uint32_t)late;
      if (s >= (1u << kStretchBits)) s = (1u << kStretchBits) - 1u;
      const unsigned long long word = (st.stamp << kStretchBits) | s;
      __hip_atomic_fetch_max(p.feedback + (size_t)threadIdx.x * kFeedbackStrideWords, word, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
    }
  } else if (late < 0) {
    pace_wait_until(turn);
  }
  st.next += p.period;
  return turn;
}

// The feedback word this wavefront reads (issue together with a load burst, consume after it).
__device__ __forceinline__ unsigned long long pace_feedback_load(const Pace& p, unsigned wave) {
  if (p.feedback == nullptr) return 0ull;
  return __hip_atomic_load(p.feedback + (size_t)(wave & (kFeedbackCopies - 1)) * kFeedbackStrideWords,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Which of the two matched orders (plan::matched_run, `flip`) suits a pair of input arrays is learnt
// from the duration of whole launches, because nothing visible to a kernel tells it: the orders differ
// by 4-5 % of a launch, launches of one order by a few tenths of a percent (one in ten by more, hence
// the shortest of two).  A slot of device words (plan::order_key) holds for its pair the number of
// launches so far and the shortest duration seen with each order in the current cycle of
// plan::kOrderCycle launches; plan::order_of_launch() says which order a launch uses.  Every wavefront
// reads the slot when it starts (an earlier kernel wrote it, so plain loads see it); the last
// wavefront times itself, which is the launch's duration to within a period because the timetable
// keeps all of them in step, and writes the slot when it is done.  Kernels that overlap on one GPU and
// share a slot, or pairs whose keys fall into one slot, may learn nothing or the wrong order: that
// costs speed, never correctness.
struct OrderChoice {
  unsigned* slot;      // nullptr: nothing is learnt
  uint32_t key_lo, key_hi;
  uint32_t launches;   // of this pair, before this one
  uint32_t best[2];
  uint32_t begin;
  unsigned flip;       // this launch's order
};

__device__ __forceinline__ uint32_t order_uniform(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }

__device__ __forceinline__ OrderChoice order_begin(const Pace& p, uintptr_t a0, uintptr_t a1, size_t n, unsigned first) {
  OrderChoice c{};
  if (p.order_words == nullptr) return c;
  c.begin = pace_clock();
  const plan::OrderKey key = plan::order_key(a0, a1, n, p.order_epoch);
  c.key_lo = key.lo;
  c.key_hi = key.hi;
  c.slot = p.order_words + (size_t)key.slot * plan::kOrderSlotWords;
  typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
  const u4_t w = *reinterpret_cast<const u4_t*>(c.slot);
  const uint32_t w4 = c.slot[4];
  const bool known = order_uniform(w.x) == c.key_lo && order_uniform(w.y) == c.key_hi;
  c.launches = known ? order_uniform(w.z) : 0u;
  c.best[0] = order_uniform(w.w);
  c.best[1] = order_uniform(w4);
  if (!known || c.launches % plan::kOrderCycle == 0u) c.best[0] = c.best[1] = 0xFFFFFFFFu;
  c.flip = plan::order_of_launch(c.launches, first, c.best[0], c.best[1]);
  return c;
}

// Call in one wavefront of the launch, when it has issued its last access.
__device__ __forceinline__ void order_end(const OrderChoice& c) {
  if (c.slot == nullptr || threadIdx.x != 0) return;
  const uint32_t ticks = pace_clock() - c.begin;
  uint32_t best[2] = {c.best[0], c.best[1]};
  if (ticks < best[c.flip]) best[c.flip] = ticks;
  c.slot[0] = c.key_lo;
  c.slot[1] = c.key_hi;
  c.slot[2] = c.launches + 1u;
  c.slot[3] = best[0];
  c.slot[4] = best[1];
}

// Adopt a published stretch if it belongs to this launch (stamps of one launch differ by at
// most one unit), is larger than ours, and is plausible (at most eight periods more).
__device__ __forceinline__ void pace_adopt(const Pace& p, PaceState& st, unsigned long long word) {
  if (p.feedback == nullptr) return;
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)word);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(word >> 32));
  const uint64_t w = ((uint64_t)hi << 32) | lo;
  const int64_t dstamp = (int64_t)(w >> kStretchBits) - (int64_t)st.stamp;
  const uint32_t s = (uint32_t)(w & ((1u << kStretchBits) - 1u));
  if (dstamp >= -1 && dstamp <= 1 && s > st.stretch && s - st.stretch <= 8u * p.period) st.stretch = s;
}

}  // namespace opal
