// Measurement kernels, in a library of their own (libarkv_measure.so): plain streaming reads and a plain copy
// of known size.  They give the practical bandwidth ceiling of a box for a launch of a given size, and they are
// the kernels of known traffic against which bench.py's hardware-counter figures are calibrated.  Nothing of the
// method is in here, and the product library does not contain them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "arkv_measure.h"

namespace arkv_measure {

// Plain streaming read: each workgroup reads a contiguous share, 8 x 16 bytes per lane in flight.
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ src, unsigned n_per_wg, unsigned* sink) {
  const uint4* p = src + (size_t)blockIdx.x * n_per_wg;
  unsigned acc = 0;
  for (unsigned i = threadIdx.x; i < n_per_wg; i += 256 * 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { const unsigned j = i + u * 256; v[u] = p[j < n_per_wg ? j : n_per_wg - 1]; }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9E3779B9u) sink[blockIdx.x] = acc;   // practically never: keeps the loads alive
}

// The same bytes in the key-operand layout of k_decode_attend: rows of 256 bytes, a wave covers 16
// rows per tile with 4 instructions, lane = row lane%16, chunk lane/16 of each 64 bytes.
__global__ __launch_bounds__(256) void k_stream_read_operand(const uint4* __restrict__ src, unsigned rows_per_wg, unsigned* sink) {
  const uint4* p = src + (size_t)blockIdx.x * rows_per_wg * 16;
  const unsigned lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  unsigned acc = 0;
  for (unsigned r0 = w * 16; r0 < rows_per_wg; r0 += 128) {
    uint4 v[8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      unsigned row = r0 + t * 64 + (lane & 15);
      if (row >= rows_per_wg) row = rows_per_wg - 1;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) v[t * 4 + kk] = p[row * 16 + kk * 4 + (lane >> 4)];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9E3779B9u) sink[blockIdx.x] = acc;
}

// Plain copy: reads bytes/2 and writes bytes/2 (the second half of the window), coalesced.
__global__ __launch_bounds__(256) void k_stream_copy(uint4* __restrict__ buf, unsigned n_per_wg, unsigned half) {
  uint4* p = buf + (size_t)blockIdx.x * n_per_wg;
  for (unsigned i = threadIdx.x; i < n_per_wg; i += 256 * 4) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) { const unsigned j = i + u * 256; v[u] = p[j < n_per_wg ? j : n_per_wg - 1]; }
#pragma unroll
    for (int u = 0; u < 4; ++u) { const unsigned j = i + u * 256; if (j < n_per_wg) p[(size_t)half + j] = v[u]; }
  }
}

hipError_t launch_stream_read(const void* buf, size_t offset_bytes, size_t bytes, int pattern, unsigned* sink, hipStream_t s) {
  if (pattern == 2) {
    const unsigned wgs = 2048;
    uint4* b = reinterpret_cast<uint4*>(const_cast<char*>(static_cast<const char*>(buf)) + offset_bytes);
    hipLaunchKernelGGL(k_stream_copy, dim3(wgs), dim3(256), 0, s, b, (unsigned)(bytes / 2 / 16 / wgs), (unsigned)(bytes / 2 / 16));
    return hipGetLastError();
  }
  const unsigned wgs = 2048;
  const uint4* src = reinterpret_cast<const uint4*>(static_cast<const char*>(buf) + offset_bytes);
  if (pattern == 0) {
    hipLaunchKernelGGL(k_stream_read, dim3(wgs), dim3(256), 0, s, src, (unsigned)(bytes / 16 / wgs), sink);
  } else {
    hipLaunchKernelGGL(k_stream_read_operand, dim3(wgs), dim3(256), 0, s, src, (unsigned)(bytes / 256 / wgs), sink);
  }
  return hipGetLastError();
}


}  // namespace arkv_measure

using arkv_measure::launch_stream_read;

extern "C" int arkv_measure_stream_read(void* buf, uint64_t buf_bytes, uint64_t bytes_per_launch, int32_t launches,
                                        int32_t pattern, void* hip_stream, float* avg_us) {
  if (!buf || !avg_us || launches < 1 || bytes_per_launch == 0 || bytes_per_launch % 524288 != 0 ||
      bytes_per_launch > buf_bytes || pattern < 0 || pattern > 2)
    return ARKV_MEASURE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&sink), 2048 * sizeof(unsigned));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  const uint64_t windows = buf_bytes / bytes_per_launch;
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {          // pass 0 warms up
    if (pass == 1) e = hipEventRecord(e0, st);
    const int n = pass == 0 ? std::min(launches, 8) : launches;
    for (int i = 0; i < n && e == hipSuccess; ++i)
      e = launch_stream_read(buf, (size_t)((uint64_t)i % windows) * bytes_per_launch, (size_t)bytes_per_launch, pattern, sink, st);
    if (pass == 1 && e == hipSuccess) e = hipEventRecord(e1, st);
  }
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  if (e == hipSuccess) *avg_us = ms * 1000.0f / (float)launches;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  return e == hipSuccess ? ARKV_MEASURE_OK : ARKV_MEASURE_EHIP;
}
