// Launch shapes of the streaming kernels: everything that, together with stream_kernels.hpp,
// pacing.hpp and launch_plan.hpp, decides what the GPU executes for a given call.  Kept in a
// file of its own so that measured figures can be tied to exactly these choices.
#pragma once

#include <stddef.h>

#include "stream_kernels.hpp"

namespace opal {

// Three regimes, by the size of one array (chosen by measurement on MI355X):
//
//   up to kCacheResidentBytes  (three such arrays fit the 256 MB Infinity Cache together, so the
//       next call is expected to find them there): temporal accesses, 256-lane workgroups in
//       dispatcher order (wave-sized ones would make the dispatcher the bottleneck at these
//       sizes), tiled dot with 512-thread workgroups.  Measured crossover, chain of the five
//       kernels back to back: temporal wins by 5-8 % up to 92 MiB per array and loses by 10 %
//       from 128 MiB on.
//   larger, up to the paced shape's own threshold (PacedShape::min_bytes): non-temporal accesses,
//       wave-sized workgroups in dispatcher order, one 16-byte vector per lane; tiled dot, one
//       256-thread workgroup per compute unit.
//   above: the paced shapes (persistent wavefronts on a clock timetable), when the device is
//       the one the timetable was measured on; otherwise as the middle regime.  Measured
//       crossover at n = 2^25 ... 2^28 fp64: Dot gains from 384 MiB per array on, Add and Triad
//       from 512 MiB, Copy and Mul from 768 MiB; below, the ramp of the timetable (a period at
//       each end) and its pauses cost more than the ordering gains.
constexpr size_t kCacheResidentBytes = (size_t)96 << 20;

constexpr int kStreamBlock = kWave;
constexpr int kResidentBlock = 256;
constexpr unsigned kDotBlock = 256;
constexpr unsigned kDotResidentBlock = 512;
constexpr int kDotUnroll = 4;
constexpr unsigned kDotGroupsPerCU = 1;
constexpr unsigned kDotMaxGroups = 8192;   // 64 KiB of fp64 partials at most
constexpr unsigned kFinalBlock = 256;

// Paced shapes.  Rates are what the timetable asks of the memory system, in bytes per
// microsecond (7.0e6 is 7.0 TB/s): slightly more than HBM sustains, so the timetable, not the
// queues, orders the traffic, and the feedback of pacing.hpp absorbs the difference.  Measured
// optimum on MI355X (8 TB/s HBM3E, 256 compute units, 100 MHz counter).
//
// Placement.  Both elementwise shapes hand XCD x the 1 KiB runs whose index is x modulo 8, so an
// XCD keeps reaching the same memory channels of an array.  For kernels with two inputs the
// distance between the input arrays then matters (launch_plan.hpp: channel classes).  The paced
// kernels load the runs of their second input in the order that matches the first input's
// classes (plan::matched_run), which holds Add at 86-88 % of the HBM peak and Triad at 86-87.5 %
// for nearly every distance; what remains are distances that differ in the lower two class bits
// or by odd multiples of 1 MiB (Triad), at 81-85 %.  The index-ordered shape behaves the other way
// round (84-85 % where the inputs differ by 4-12 KiB modulo 16 KiB, 81-83 % where they agree).
struct PacedShape {
  unsigned waves;          // persistent wavefronts (8 or 4 per compute unit)
  unsigned k;              // 1 KiB runs per wavefront per burst
  unsigned set_bit;        // bit of the workgroup index that selects the set (plan::paced_set)
  double bytes_per_us;     // timetable rate
  double store_at;         // store burst at this fraction of the period (0: as soon as data is there)
  double second_input_at;  // burst of the second input at this fraction of the period after the first
  double gap;              // accesses of a burst this fraction of the period apart (0: all at once)
  unsigned tolerance;      // ticks of lateness before reporters push the timetable back
  size_t min_bytes;        // smallest array (bytes) the shape is used for
  bool feedback;
};
// Rates and gaps were settled by interleaved comparisons (the settings alternate from launch to
// launch inside one process, 120-150 launches each, chain of the five kernels at 2 GiB per array):
// what differs between settings is mostly how many launches have one XCD fall behind the
// timetable (such a launch is 5-20 % slow), not the speed of a good launch.
constexpr unsigned kPacedCUs = 256;             // the timetable is for this chip only
constexpr int kPacedK1 = 8;                     // one-input kernels (copy, scale): K
constexpr int kPacedK2 = 4;                     // two-input kernels (add, triad): K
constexpr int kPacedKDot = 8;
constexpr PacedShape kPacedOneInput = {2048, kPacedK1, 3, 7.10e6, 0.75, 0.0, 0.035, 400, (size_t)768 << 20, true};
constexpr PacedShape kPacedTwoInputs = {2048, kPacedK2, 3, 7.10e6, 0.0, 0.0, 0.03, 400, (size_t)512 << 20, true};
constexpr PacedShape kPacedDot = {1024, kPacedKDot, 3, 7.60e6, 0.0, 0.25, 0.0, 0, (size_t)384 << 20, false};

}  // namespace opal
