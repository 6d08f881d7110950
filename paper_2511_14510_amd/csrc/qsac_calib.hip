// Measurement aids (include/qsac_calib.h): a copy and a read-only kernel of known size.  Not part of the
// QSAC step; built into a library of their own.
#include "qsac_calib.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t v4u;  // one 16-byte load

// Plain 16-byte-per-lane copy of n vectors: the known-size kernel that hardware counters are
// calibrated against.
__global__ __launch_bounds__(256) void qsac_copy_kernel(v4u* __restrict__ dst, const v4u* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Read-only counterpart: every workgroup reads a contiguous span, eight non-temporal 16-byte loads
// per thread in flight.  The XOR of everything read goes to `sink` only if it equals a magic value,
// so the loads stay.
__global__ __launch_bounds__(256) void qsac_read_kernel(const v4u* __restrict__ src, size_t n, uint32_t* __restrict__ sink) {
  const size_t span = (n + gridDim.x - 1) / gridDim.x;
  const size_t b = (size_t)blockIdx.x * span, e = b + span < n ? b + span : n;
  uint32_t acc = 0;
  for (size_t i = b + threadIdx.x; i < e; i += 256 * 8) {
    v4u v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (i + u * 256 < e) ? __builtin_nontemporal_load(src + i + u * 256) : v4u{0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int qsac_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return -2;
  if (!aligned16(dst) || !aligned16(src) || (bytes & 15u)) return -7;
  if (bytes == 0) return 0;
  qsac_copy_kernel<<<4096, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<v4u*>(dst), static_cast<const v4u*>(src), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

int qsac_calibration_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return -2;
  if (!aligned16(src) || (bytes & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return -7;
  if (bytes == 0) return 0;
  qsac_read_kernel<<<2048, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const v4u*>(src), bytes / 16,
                                                                      static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // extern "C"
