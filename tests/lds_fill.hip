// Test helper (not part of the library): leaves a chosen bit pattern in the LDS of every compute
// unit, so that a GPU test can show that the step kernels' results do not depend on what a
// previous kernel left there.  Built by __graft_entry__.build() into tests/liblds_fill.so.
#include <hip/hip_runtime.h>
#include <stdint.h>

__global__ void lds_fill_kernel(uint32_t pattern, int words, uint32_t* sink) {
  extern __shared__ uint32_t lds[];
  // pattern 0xdeadbeef: a different pseudo-random word everywhere
  for (int i = threadIdx.x; i < words; i += blockDim.x)
    lds[i] = pattern == 0xdeadbeefu ? (uint32_t)i * 2654435761u + blockIdx.x : pattern;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = lds[(blockIdx.x * 7) % words];   // (keeps the stores alive)
}

// sink: device memory for 2048 words; returns the HIP error code of the launch
extern "C" int lds_fill(uint32_t pattern, void* sink, void* stream) {
  const int bytes = 160 * 1024;
  hipError_t rc = hipFuncSetAttribute((const void*)lds_fill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (rc != hipSuccess) return (int)rc;
  hipLaunchKernelGGL(lds_fill_kernel, dim3(2048), dim3(256), bytes, (hipStream_t)stream, pattern, bytes / 4, (uint32_t*)sink);
  return (int)hipGetLastError();
}
