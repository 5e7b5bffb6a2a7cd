// Definitions shared by the kernel headers of libbcsched (included by bcsched.hip only, in this order:
// common, sched, expand, allgather).  Everything sits in the unnamed namespace of that one translation unit.
#ifndef BCS_KERNELS_COMMON_H
#define BCS_KERNELS_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bcsched.h"
#include "bcs_core.h"

namespace {

using namespace bcs;
typedef int v4i __attribute__((ext_vector_type(4)));
// An entry of the slot-major receive table kept in scratch memory: schedule entries lie in [-q, q-1], q <= 31.
typedef int8_t slot_t;
// Rank-major byte rows for the expansion of long rows (scratch as well): row r holds T[k] = entry[k] - k for the q
// slots, then T[0..2] once more, padded to a multiple of 4 bytes.  T lies in [-2q, q), q <= 31.
constexpr int byte_row_stride(int q) { return (q + 3 + 3) & ~3; }
// The byte rows pay while a table of them stays in cache (measured: 25 MB at p = 2^20+1 gives 0.83-0.93 of the
// separate kernels' time for every row length, 50 MB at p = 2^21+1 gives 1.08-1.2).
constexpr uint64_t kByteRowsMax = 32ull << 20;
static_assert(kMaxQ == BCS_MAX_Q, "header and core disagree");
constexpr int kBlock = 256;              // lanes (= ranks) per workgroup

}  // namespace

#endif  // BCS_KERNELS_COMMON_H
