// Yardstick for the re-layout kernels: what this chip does on a plain copy of the same shape
// (one-wavefront workgroups, one 16-byte non-temporal load and one 16-byte store per lane, then
// end of program), on reads alone and on writes alone.  Not part of the library: built into its
// own shared object, driven by `bench.py --copy-ceiling`.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define YARD_GLOBAL __attribute__((address_space(1)))

namespace {

__global__ __launch_bounds__(64, 8) void copy_kernel(const u32x4* __restrict__ src,
                                                     u32x4* __restrict__ dst) {
  const size_t x = (size_t)blockIdx.x * 64 + threadIdx.x;
  const u32x4 v = __builtin_nontemporal_load((const YARD_GLOBAL u32x4*)(src + x));
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt"
               :: "v"((YARD_GLOBAL u32x4*)(dst + x)), "v"(v) : "memory");
}

// Reads alone and writes alone: four vectors per lane (4 KiB per workgroup), or the rate at which
// one-wavefront workgroups can be started (about 4.7 per nanosecond) would be measured instead
// of the memory.
__global__ __launch_bounds__(64, 8) void read_kernel(const u32x4* __restrict__ src,
                                                     uint32_t* __restrict__ sink) {
  const size_t x = (size_t)blockIdx.x * 256 + threadIdx.x;
  u32x4 acc = {0, 0, 0, 0};
#pragma unroll
  for (int k = 0; k < 4; ++k) acc |= __builtin_nontemporal_load((const YARD_GLOBAL u32x4*)(src + x + 64 * k));
  // never true for the fill pattern the benchmark uses; keeps the loads alive
  if ((acc.x & acc.y & acc.z & acc.w) == 0xdeadbeefu) sink[threadIdx.x] = acc.x;
}

__global__ __launch_bounds__(64, 8) void write_kernel(u32x4* __restrict__ dst, uint32_t value) {
  const size_t x = (size_t)blockIdx.x * 256 + threadIdx.x;
  const u32x4 v = {value, value + 1, value + 2, value + 3};
#pragma unroll
  for (int k = 0; k < 4; ++k)
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt"
                 :: "v"((YARD_GLOBAL u32x4*)(dst + x + 64 * k)), "v"(v) : "memory");
}

}  // namespace

// bytes must be a multiple of 4096 and at most 2^31 - 1 KiB-slices; device pointers 16-byte
// aligned; `sink` holds at least 64 words.  Returns a hipError_t.
extern "C" int yardstick_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
  if (bytes % 1024 || bytes / 1024 > 0x7fffffffull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)(bytes / 1024)), dim3(64), 0, (hipStream_t)stream,
                     (const u32x4*)src, (u32x4*)dst);
  return (int)hipGetLastError();
}
extern "C" int yardstick_read(const void* src, void* sink, uint64_t bytes, void* stream) {
  if (bytes % 4096 || bytes / 1024 > 0x7fffffffull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(read_kernel, dim3((unsigned)(bytes / 4096)), dim3(64), 0, (hipStream_t)stream,
                     (const u32x4*)src, (uint32_t*)sink);
  return (int)hipGetLastError();
}
extern "C" int yardstick_write(void* dst, uint64_t bytes, void* stream) {
  if (bytes % 4096 || bytes / 1024 > 0x7fffffffull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(write_kernel, dim3((unsigned)(bytes / 4096)), dim3(64), 0, (hipStream_t)stream,
                     (u32x4*)dst, 1u);
  return (int)hipGetLastError();
}
