// Measured VALU integer issue rates on the device the library runs on: what the roofline of the
// plan-scoring kernels is checked against.  Register-only kernels, no memory traffic, 16 waves
// queued per SIMD.  On gfx950 simple operations (v_add_u32) issue about twice as fast as
// v_max_i32 / v_mul_u32_u24 / three-operand operations, and a stream that mixes the two classes
// runs at the slower rate throughout.
#include <hip/hip_runtime.h>

#include "../../include/chm.h"
#include "../../include/chm_measure.h"

namespace {

#define CHM_ASM8(OP)                                                                                    \
  OP " %0, %0, %8\n\t" OP " %1, %1, %8\n\t" OP " %2, %2, %8\n\t" OP " %3, %3, %8\n\t" OP " %4, %4, %8\n\t" \
  OP " %5, %5, %8\n\t" OP " %6, %6, %8\n\t" OP " %7, %7, %8\n\t"

// kind 0: v_add_u32 only; kind 1: v_max_i32 only (8 independent accumulators each)
template <int KIND>
__global__ void __launch_bounds__(256) k_probe_op(uint32_t iters, uint32_t seed, uint32_t *sink) {
  uint32_t a0 = threadIdx.x, a1 = seed, a2 = 3, a3 = 4, a4 = 5, a5 = 6, a6 = 7, a7 = 8;
  const uint32_t b = seed | 1u;
  for (uint32_t i = 0; i < iters; ++i) {
    if (KIND == 0) {
      asm volatile(CHM_ASM8("v_add_u32") CHM_ASM8("v_add_u32") CHM_ASM8("v_add_u32") CHM_ASM8("v_add_u32")
                   : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(b));
    } else {
      asm volatile(CHM_ASM8("v_max_i32") CHM_ASM8("v_max_i32") CHM_ASM8("v_max_i32") CHM_ASM8("v_max_i32")
                   : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(b));
    }
  }
  const uint32_t r = a0 ^ a1 ^ a2 ^ a3 ^ a4 ^ a5 ^ a6 ^ a7;
  if (r == 0x12345678u) sink[0] = r;     // never true in practice; keeps the chains alive
}

// kind 2: the recurrence cell, e = max(e, x) + f, as one dependent chain of 64 cells per iteration
__global__ void __launch_bounds__(256) k_probe_cell(uint32_t iters, uint32_t seed, uint32_t *sink) {
  int e[8], f[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) { e[s] = (int)(threadIdx.x + s); f[s] = (int)((seed >> s) & 1023) + 1; }
  for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int x = 0;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int m = e[s] > x ? e[s] : x;
        e[s] = m + f[s];
        x = e[s];
      }
    }
  }
  int r = 0;
#pragma unroll
  for (int s = 0; s < 8; ++s) r ^= e[s];
  if (r == 0x12345678) sink[0] = (uint32_t)r;
}

}  // namespace

extern "C" int chm_valu_probe(int32_t kind, uint32_t iters, double *lane_ops_per_s, void *hip_stream) {
  if (kind < 0 || kind > 2 || iters == 0 || !lane_ops_per_s) return CHM_ERR_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  uint32_t *sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipMalloc((void **)&sink, 64) != hipSuccess) return CHM_ERR_HIP;
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  const uint32_t blocks = 256 * 16, threads = 256;            // 16 waves per SIMD queued on 256 CUs
  const double ops_per_iter = kind == 2 ? 128 : 32;
  for (int rep = 0; rep < 2 && ok; ++rep) {                    // first pass warms up, second is timed
    ok = ok && hipEventRecord(e0, st) == hipSuccess;
    if (kind == 0) hipLaunchKernelGGL((k_probe_op<0>), dim3(blocks), dim3(threads), 0, st, iters, 12345u, sink);
    if (kind == 1) hipLaunchKernelGGL((k_probe_op<1>), dim3(blocks), dim3(threads), 0, st, iters, 12345u, sink);
    if (kind == 2) hipLaunchKernelGGL(k_probe_cell, dim3(blocks), dim3(threads), 0, st, iters, 12345u, sink);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
  }
  float ms = 0;
  ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0;
  if (ok) *lane_ops_per_s = (double)blocks * threads * iters * ops_per_iter / (ms * 1e-3);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  return ok ? CHM_OK : CHM_ERR_HIP;
}
