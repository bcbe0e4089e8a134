// Device allocations of the library, with optional guard zones around each for debugging.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>

namespace lop {

// hipMalloc / hipFree. With the environment variable LOP_GUARD_BYTES=<n> (read once, n a
// multiple of 256) every allocation gets n bytes of a fixed pattern in front and behind;
// dev_free (and lop_debug_guard_check) compare them and count every allocation whose guard
// was overwritten: a kernel that stores outside the buffer it was given shows up there instead
// of in whatever happens to live next to it.
hipError_t dev_alloc(void** p, size_t bytes);
hipError_t dev_free(void* p);

}  // namespace lop
