#include <hip/hip_runtime.h>
#include <cstdio>
// Instruction issue rate of one wavefront on this GPU: chains of fp32 FMAs with 1, 2, 4 or 8
// independent accumulators per thread, 1, 4, 8 or 16 wavefronts per compute unit.  Prints the cycles
// (clock64, calibrated against the 100 MHz wall clock) one wavefront needs per instruction.  The
// step kernel's design rests on the outcome: a wavefront issues an instruction every five to
// seven cycles whether its neighbours on the SIMD are busy or not and whatever its ILP, so a phase
// gets shorter by spreading its work over more lanes, not by packing more work into a lane.
template <int ILP>
__global__ void chain(float* out, long long* cyc, int n, float a, float b) {
  float x[ILP];
  for (int k = 0; k < ILP; ++k) x[k] = threadIdx.x * 0.001f + k;
  long long t0 = clock64(); long long w0 = wall_clock64();
  for (int i = 0; i < n; ++i) {
#pragma unroll
    for (int r = 0; r < 16 / ILP; ++r)
#pragma unroll
      for (int k = 0; k < ILP; ++k) x[k] = __builtin_fmaf(x[k], a, b);
  }
  long long t1 = clock64(); long long w1 = wall_clock64();
  float s = 0; for (int k = 0; k < ILP; ++k) s += x[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = t1 - t0; cyc[1] = w1 - w0; }
}
template <int ILP> void run(int threads, int n, float* out, long long* cyc) {
  hipLaunchKernelGGL(chain<ILP>, dim3(256), dim3(threads), 0, 0, out, cyc, n, 1.0001f, 0.5f);
  (void)hipDeviceSynchronize();
  hipLaunchKernelGGL(chain<ILP>, dim3(256), dim3(threads), 0, 0, out, cyc, n, 1.0001f, 0.5f);
  (void)hipDeviceSynchronize();
  long long c2[2]; (void)hipMemcpy(c2, cyc, 16, hipMemcpyDeviceToHost); long long c = c2[0];
  printf("ILP %d threads/WG %4d: %.2f cycles per FMA instruction (per wave)\n", ILP, threads, (double)c / (16.0 * n)); printf("   clock64 ticks %lld, wall_clock64 ticks (100 MHz) %lld -> clock64 at %.1f MHz, %.2f ns per instruction\n", c2[0], c2[1], 100.0 * c2[0] / c2[1], 10.0 * c2[1] / (16.0 * n));
}
int main() {
  float* out; long long* cyc;
  if (hipMalloc(&out, 256 * 1024 * 4) != hipSuccess || hipMalloc(&cyc, 16) != hipSuccess) { printf("no GPU memory\n"); return 1; }
  int n = 4096;
  for (int threads : {64, 256, 512, 1024}) { run<1>(threads, n, out, cyc); run<2>(threads, n, out, cyc); run<4>(threads, n, out, cyc); run<8>(threads, n, out, cyc); }
  return 0;
}
