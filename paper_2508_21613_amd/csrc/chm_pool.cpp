// See chm_pool.h.
#include "chm_pool.h"

#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <unordered_map>
#include <vector>

namespace {

constexpr size_t KEEP_BLOCK_MAX = 512u << 20;                 // larger blocks are never kept
constexpr size_t KEEP_TOTAL_MAX[2] = {2048ull << 20, 96u << 20};   // bytes kept over all devices: device memory, pinned host memory

struct Block { int device; bool pinned; size_t size; };

std::mutex g_lock;
std::unordered_map<void *, Block> g_live;                            // blocks handed out
std::map<std::tuple<int, bool, size_t>, std::vector<void *>> g_kept; // (device, pinned, size class) -> free blocks
size_t g_kept_bytes[2] = {0, 0};

size_t size_class(size_t bytes) {
  size_t c = 256;
  while (c < bytes) c <<= 1;
  return c;
}

void *take(size_t bytes, bool pinned) {
  if (bytes == 0) bytes = 1;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return nullptr;
  const size_t cls = bytes <= KEEP_BLOCK_MAX ? size_class(bytes) : bytes;
  {
    std::lock_guard<std::mutex> hold(g_lock);
    auto it = g_kept.find(std::make_tuple(pinned ? -1 : device, pinned, cls));
    if (it != g_kept.end() && !it->second.empty()) {
      void *p = it->second.back();
      it->second.pop_back();
      g_kept_bytes[pinned] -= cls;
      g_live[p] = Block{device, pinned, cls};
      return p;
    }
  }
  void *p = nullptr;
  const hipError_t rc = pinned ? hipHostMalloc(&p, cls, hipHostMallocDefault) : hipMalloc(&p, cls);
  if (rc != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
  std::lock_guard<std::mutex> hold(g_lock);
  g_live[p] = Block{device, pinned, cls};
  return p;
}

}  // namespace

void *pool_device_alloc(size_t bytes) { return take(bytes, false); }
void *pool_pinned_alloc(size_t bytes) { return take(bytes, true); }

void pool_release(void *p) {
  if (!p) return;
  Block b;
  {
    std::lock_guard<std::mutex> hold(g_lock);
    auto it = g_live.find(p);
    if (it == g_live.end()) return;               // not ours
    b = it->second;
    g_live.erase(it);
    if (b.size <= KEEP_BLOCK_MAX && g_kept_bytes[b.pinned] + b.size <= KEEP_TOTAL_MAX[b.pinned]) {
      g_kept[std::make_tuple(b.pinned ? -1 : b.device, b.pinned, b.size)].push_back(p);
      g_kept_bytes[b.pinned] += b.size;
      return;
    }
  }
  // beyond what is kept: back to the runtime (which waits for the device on its own)
  if (b.pinned) (void)hipHostFree(p);
  else (void)hipFree(p);
}

bool pool_staged_upload(PoolStage *stage, void *dst, const void *src, size_t bytes, void *stream) {
  const void *from = src;
  if (stage && stage->base) {
    const size_t at = (stage->used + 255) & ~(size_t)255;
    if (at + bytes <= stage->bytes) {
      memcpy(stage->base + at, src, bytes);
      from = stage->base + at;
      stage->used = at + bytes;
    }
  }
  return hipMemcpyAsync(dst, from, bytes, hipMemcpyHostToDevice, (hipStream_t)stream) == hipSuccess;
}
