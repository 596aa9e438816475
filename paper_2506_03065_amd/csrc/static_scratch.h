// The library's own scratch buffer in device memory, for the entry point that
// must not allocate (callers under stream capture, serving loops and harnesses
// that forbid hipMalloc).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>

namespace svd {

// Size of the buffer every GPU the library runs on holds until the process ends.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(64) << 20;

// Address of the current device's copy of the buffer (each device has its own,
// at its own address; resolved once per device and kept) and its size.
hipError_t static_scratch(void** ptr, size_t* bytes);

}  // namespace svd
