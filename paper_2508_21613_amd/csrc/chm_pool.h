// Small caching allocator for the library's own device and pinned host buffers.
//
// A scenario handle owns about a dozen buffers; hipMalloc, hipHostMalloc and hipFree cost tens to hundreds
// of microseconds each, which is as much as a whole bounded search, and hipFree waits for the whole device.
// Blocks released by one handle are kept (per device, by size class) and handed to the next; what is kept
// is bounded (2 GiB of device memory, 96 MiB of pinned memory, blocks of at most 512 MiB), the rest goes back
// to the runtime.  Thread-safe.
#ifndef CHM_POOL_H
#define CHM_POOL_H
#include <cstddef>

// Device memory of the current device, at least `bytes` long, 256-byte aligned; nullptr on failure.
void *pool_device_alloc(size_t bytes);
// Pinned host memory; nullptr on failure.
void *pool_pinned_alloc(size_t bytes);
// Gives a block of either kind back (nullptr is ignored).  Unlike hipFree this does not wait for anything:
// the caller guarantees that all work that reads or writes the block has finished (it has waited for the
// streams it launched that work on), since the block may be handed to another owner at once.
void pool_release(void *p);
#endif
