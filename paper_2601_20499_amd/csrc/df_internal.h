// Internal declarations shared by the translation units of the library.
// Nothing here is part of the public ABI (see include/df.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "df.h"

namespace df {

constexpr int kMaxHeads = DF_MAX_HEADS;

// 16-byte row alignment: pointers must be multiples of 16 bytes and strides
// multiples of 8 bf16 elements, so that every row of d elements can be moved
// with 128-bit accesses.
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool stride_ok(int64_t s) { return s > 0 && (s % 8) == 0; }

inline df_status launch_status() {
  return hipGetLastError() == hipSuccess ? DF_OK : DF_ERR_LAUNCH;
}

}  // namespace df
