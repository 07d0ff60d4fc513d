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

// A pinned staging area for host-to-device copies at load.  A copy from pageable memory keeps the host busy until
// the data has left; staged (a memcpy into pinned memory, then the copy) it is queued and done.  `used` counts
// the bytes of the area taken so far: the caller resets it once the stream has been waited for.
struct PoolStage { unsigned char *base = nullptr; size_t bytes = 0, used = 0; };
// Queues the copy of `bytes` from src (host) to dst (device) on `stream` (a hipStream_t), through the staging
// area when it still has room, directly otherwise (src must then outlive the copy, as always).  False when HIP fails.
bool pool_staged_upload(PoolStage *stage, void *dst, const void *src, size_t bytes, void *stream);
#endif
