// Seeded synthetic-input generator, device side (test/bench harness; not part of the decode
// library).  Same integer recipe as synth_cpu.c: element i of tensor `tid` is
// table[mix64(seed, tid, i) >> 48], so device-filled tensors are bit-identical to host-filled
// ones.  Lets 100+ GB of weights be created in HBM without ever existing on the host.
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ uint64_t synth_mix64(uint64_t seed, uint64_t tid, uint64_t i) {
  uint64_t z = seed * 0x9E3779B97F4A7C15ull + tid * 0xD1B54A32D192ED03ull + i;
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

__global__ void synth_fill_kernel(uint16_t* __restrict__ out, uint64_t seed, uint64_t tid,
                                  uint64_t i0, uint64_t n, const uint16_t* __restrict__ table) {
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride)
    out[k] = table[synth_mix64(seed, tid, i0 + k) >> 48];
}

// out, table: device pointers.  Asynchronous on `stream`.  Returns the hipError_t value.
extern "C" int synth_fill_bf16_device(void* out, uint64_t seed, uint64_t tid, uint64_t i0,
                                      uint64_t n, const void* table, void* stream) {
  if (n == 0) return 0;
  uint64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     (hipStream_t)stream, (uint16_t*)out, seed, tid, i0, n,
                     (const uint16_t*)table);
  return (int)hipGetLastError();
}

// Plain copy of n 16-byte words (counter calibration: a kernel whose HBM traffic is known, to
// scale profiler byte counters by).  Asynchronous on `stream`.
__global__ void synth_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, uint64_t n) {
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) dst[k] = src[k];
}

extern "C" int synth_copy_device(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (bytes == 0 || (bytes & 15)) return bytes ? 1 : 0;
  hipLaunchKernelGGL(synth_copy_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)src, (uint4*)dst, bytes / 16);
  return (int)hipGetLastError();
}
