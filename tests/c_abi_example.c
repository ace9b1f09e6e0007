/* A caller of the C interface written in plain C (no Python, no torch): the built-in humanoid on
 * the plane, a few env-steps with zero actions, the observations copied back and printed as a
 * checksum that tests/test_gpu_c_caller.py compares with the Python binding's result for the same
 * set-up.  Built by __graft_entry__.build() into tests/c_abi_example.  Usage: c_abi_example N STEPS */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sim.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define SIM_OK_(x) do { int r_ = (x); if (r_ != SIM_OK) { fprintf(stderr, "%s: %d %s\n", #x, r_, sim_last_error()); return 3; } } while (0)

int main(int argc, char** argv) {
  const int n = argc > 1 ? atoi(argv[1]) : 64, steps = argc > 2 ? atoi(argv[2]) : 5;
  sim_desc_t d;
  SIM_OK_(sim_default_params(&d));
  SIM_OK_(sim_builtin_robot(SIM_ROBOT_HUMANOID, &d));
  double* origins = (double*)calloc((size_t)n * 3, sizeof(double));
  for (int e = 0; e < n; ++e) { origins[3 * e] = 5.0 * (e % 8); origins[3 * e + 1] = 5.0 * (e / 8); }
  d.env_origins = origins;

  size_t bytes = 0;
  SIM_OK_(sim_workspace_bytes(&d, n, &bytes));
  void* workspace = NULL;
  HIP_OK(hipMalloc(&workspace, bytes));          /* hipMalloc returns 256-byte aligned memory */
  sim_t* sim = NULL;
  SIM_OK_(sim_create(&d, n, workspace, bytes, &sim));
  free(origins);                                 /* the description was copied */

  const int od = sim_obs_dim(sim);
  float *obs_dev = NULL, *rew_dev = NULL;
  uint8_t* done_dev = NULL;
  HIP_OK(hipMalloc((void**)&obs_dev, (size_t)n * od * sizeof(float)));
  HIP_OK(hipMalloc((void**)&rew_dev, (size_t)n * sizeof(float)));
  HIP_OK(hipMalloc((void**)&done_dev, (size_t)n));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  SIM_OK_(sim_reset(sim, NULL, 7, stream));
  for (int s = 0; s < steps; ++s)
    SIM_OK_(sim_step_obs(sim, NULL /* zero actions */, 1.0f / 60.0f, 4, 20, obs_dev, rew_dev, done_dev, stream));
  SIM_OK_(sim_check(sim, stream));

  float* obs = (float*)malloc((size_t)n * od * sizeof(float));
  float* rew = (float*)malloc((size_t)n * sizeof(float));
  HIP_OK(hipMemcpy(obs, obs_dev, (size_t)n * od * sizeof(float), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(rew, rew_dev, (size_t)n * sizeof(float), hipMemcpyDeviceToHost));
  /* order-dependent checksum over the bit patterns: equal only if every number is */
  uint64_t h = 1469598103934665603ull;
  for (size_t i = 0; i < (size_t)n * od; ++i) { uint32_t w; memcpy(&w, &obs[i], 4); h = (h ^ w) * 1099511628211ull; }
  for (int i = 0; i < n; ++i) { uint32_t w; memcpy(&w, &rew[i], 4); h = (h ^ w) * 1099511628211ull; }
  printf("envs %d obs_dim %d act_dim %d steps %d checksum %016llx root_height0 %.6f\n", n, od, sim_act_dim(sim), steps,
         (unsigned long long)h, obs[0]);

  SIM_OK_(sim_destroy(sim));
  HIP_OK(hipStreamDestroy(stream));
  hipFree(obs_dev); hipFree(rew_dev); hipFree(done_dev); hipFree(workspace);
  free(obs); free(rew);
  return 0;
}
