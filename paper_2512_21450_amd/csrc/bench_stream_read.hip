// Measurement aid of bench.py, not part of the decode-attention library (built into a shared object of
// its own): a loads-only kernel with the K/V-streaming kernel's access pattern, i.e. what the memory
// system delivers to 2048 wavefronts that each walk a private contiguous region in steps of 16 KB
// (16 nontemporal 16-byte loads per lane, one step in flight per wavefront, two workgroups of four
// wavefronts per compute unit).  Its rate is the streaming-read ceiling the decode step is set against.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int STEP_B = 16384;       // bytes per wavefront and step
constexpr int N_WG = 512, WG_THREADS = 256, LDS_B = 65536;

__global__ void __launch_bounds__(WG_THREADS, 2) stream_read_kernel(const char* __restrict__ src, size_t bytes_per_wave,
                                                                     int steps, unsigned* sink) {
  extern __shared__ char lds[];                              // requested only to hold two workgroups per compute unit
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * (WG_THREADS / 64) + (threadIdx.x >> 6);
  const char* p = src + wave * bytes_per_wave + lane * 16;
  u32x4 acc = {0, 0, 0, 0}, v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + i * 1024));
  for (int s = 0; s < steps; ++s) {
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // all loads of the step have landed
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= v[i];
    if (s + 1 < steps) {
      const char* q = p + (size_t)(s + 1) * STEP_B;
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + i * 1024));
    }
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) {  // keeps the loads; practically never true
    sink[wave] = acc[0];
    lds[threadIdx.x] = (char)acc[1];
  }
}

}  // namespace

extern "C" {

// Bytes one launch reads from `bytes` of source: whole 16 KB steps for each of the 2048 wavefronts.
size_t bench_stream_read_bytes(size_t bytes) {
  const size_t waves = (size_t)N_WG * (WG_THREADS / 64);
  return (bytes / waves / STEP_B) * STEP_B * waves;
}

// Enqueue one pass over `src` (device memory, `bytes` long, 16-byte aligned) on `hip_stream`.  `sink`: device
// memory of at least 8 KB (never written in practice).  Returns 0, -1 (bad argument) or -5 (HIP error).
int bench_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  const size_t waves = (size_t)N_WG * (WG_THREADS / 64);
  const size_t steps = bytes / waves / STEP_B;
  if (!src || !sink || steps == 0 || steps > 0x7fffffff) return -1;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(stream_read_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            LDS_B) != hipSuccess) return -5;
    attr_done = true;
  }
  hipLaunchKernelGGL(stream_read_kernel, dim3(N_WG), dim3(WG_THREADS), LDS_B, static_cast<hipStream_t>(hip_stream),
                     static_cast<const char*>(src), steps * STEP_B, (int)steps, static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // extern "C"
