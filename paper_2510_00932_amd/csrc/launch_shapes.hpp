// Launch shapes of the streaming kernels: everything that, together with
// stream_kernels.hpp, decides what the GPU executes for a given call.  Kept in a
// file of its own so that measured figures can be tied to exactly these choices.
#pragma once

#include <stddef.h>

#include "stream_kernels.hpp"

namespace opal {

// Launch shapes (chosen by measurement on MI355X at n = 2^28 fp64).
// Elementwise: wavefront-sized workgroups, one 16-byte vector per lane, as many
// workgroups as the body has 1 KiB runs; loads and stores non-temporal.
// Dot: one workgroup of kDotBlock threads per compute unit, each looping over
// tiles of kDotBlock * kDotUnroll vectors.
//
// Arrays of at most kCacheResidentBytes each (three of them fit the 256 MB
// Infinity Cache together) are expected to be touched again by the next call:
// they get temporal accesses, 256-lane workgroups (wave-sized ones would make
// the dispatcher the bottleneck at these sizes) and 512-thread dot workgroups.
// Measured crossover on MI355X, chain of the five kernels back to back: temporal
// wins by 5-8 % up to 92 MiB per array and loses by 10 % from 128 MiB on.
constexpr size_t kCacheResidentBytes = (size_t)96 << 20;
constexpr int kStreamBlock = kWave;
constexpr int kResidentBlock = 256;
constexpr unsigned kDotBlock = 256;
constexpr unsigned kDotResidentBlock = 512;
constexpr int kDotUnroll = 4;
constexpr unsigned kDotGroupsPerCU = 1;
constexpr unsigned kDotMaxGroups = 8192;   // 64 KiB of fp64 partials at most
constexpr unsigned kFinalBlock = 256;
constexpr unsigned kBodyAlign = 1024;      // the vector body starts on a 1 KiB boundary
constexpr size_t kMaxGrid = 0x7fffffffu;

}  // namespace opal
