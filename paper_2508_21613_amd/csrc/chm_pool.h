// Small caching allocator for the library's own device and pinned host buffers.
//
// A scenario handle owns about a dozen buffers; hipMalloc, hipHostMalloc and hipFree cost tens to hundreds
// of microseconds each, which is as much as a whole bounded search.  Blocks released by one handle are kept
// (per device, by size class) and handed to the next; what is kept is bounded, the rest goes back to the
// runtime.  Thread-safe.
#ifndef CHM_POOL_H
#define CHM_POOL_H
#include <cstddef>

// Device memory of the current device, at least `bytes` long, 256-byte aligned; nullptr on failure.
void *pool_device_alloc(size_t bytes);
// Pinned host memory; nullptr on failure.
void *pool_pinned_alloc(size_t bytes);
// Gives a block of either kind back (nullptr is ignored).  As with hipFree, work that still uses the block
// must have finished: the call waits for the device the block belongs to before the block can be reused,
// unless the caller has just done so itself for all the blocks it is about to release (device_idle).
void pool_release(void *p, bool device_idle = false);
#endif
