/* The C ABI used from plain C, without Python or PyTorch: one weight matrix, a few APOLLO steps.
 *
 *   gcc -std=c99 -I include -I /opt/rocm/include -D__HIP_PLATFORM_AMD__ \
 *       paper_2412_05270_amd/examples/c_abi_example.c \
 *       -L paper_2412_05270_amd -lapollo_mi355x -L /opt/rocm/lib -lamdhip64 -lm -o c_abi_example
 *
 * Inputs are a fixed integer pattern (no random numbers), so the printed sums are reproducible:
 * tests compare them with the same steps driven through the Python binding. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "apollo.h"

#define CHECK_HIP(x)                                                              \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));              \
      return 2;                                                                   \
    }                                                                             \
  } while (0)

/* the same pattern as the test: element k of step t */
static float weight_value(int64_t k) { return (float)((k * 37 + 11) % 201 - 100) * 1e-4f; }
static float grad_value(int64_t k, int t) { return (float)((k * 53 + 29 * t) % 127 - 63) * 1e-4f; }

int main(int argc, char** argv) {
  const int64_t rows = 256, cols = 512;
  const int rank = argc > 1 ? atoi(argv[1]) : 32;
  const int steps = 3;
  apollo_config_t cfg = {0};
  cfg.rank = rank;
  cfg.mode = rank == 1 ? APOLLO_TENSOR : APOLLO_CHANNEL;
  cfg.seed = 2024;
  cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f;
  cfg.scale = rank == 1 ? sqrtf(128.0f) : 1.0f;
  cfg.nl_gamma = 1.01f;
  cfg.refresh_interval = 2;
  cfg.bias_correction = 1;
  apollo_shape_t shape = {rows, cols, APOLLO_F32, 0};

  const size_t state_bytes = apollo_state_bytes(&cfg, &shape, 1);
  const size_t ws_bytes = apollo_workspace_bytes(&cfg, &shape, 1);
  if (!state_bytes || !ws_bytes) { fprintf(stderr, "%s\n", apollo_last_error(NULL)); return 1; }

  const size_t n = (size_t)(rows * cols);
  float* hw = (float*)malloc(n * sizeof(float));
  float* hg = (float*)malloc(n * sizeof(float));
  void *dw, *dg, *dstate, *dws;
  CHECK_HIP(hipMalloc(&dw, n * sizeof(float)));
  CHECK_HIP(hipMalloc(&dg, n * sizeof(float)));
  CHECK_HIP(hipMalloc(&dstate, state_bytes));
  CHECK_HIP(hipMalloc(&dws, ws_bytes));
  for (size_t k = 0; k < n; ++k) hw[k] = weight_value((int64_t)k);
  CHECK_HIP(hipMemcpy(dw, hw, n * sizeof(float), hipMemcpyHostToDevice));

  apollo_handle_t* h = NULL;
  if (apollo_init(&h, &cfg, &shape, 1, dstate, state_bytes, dws, ws_bytes, 1, NULL) != APOLLO_OK) {
    fprintf(stderr, "apollo_init: %s\n", apollo_last_error(NULL));
    return 1;
  }
  apollo_tensor_t tensor = {dw, dg, NULL};
  for (int t = 1; t <= steps; ++t) {
    for (size_t k = 0; k < n; ++k) hg[k] = grad_value((int64_t)k, t);
    CHECK_HIP(hipMemcpy(dg, hg, n * sizeof(float), hipMemcpyHostToDevice));
    if (apollo_step(h, &tensor, 1, t, 1e-2f, NULL) != APOLLO_OK) {
      fprintf(stderr, "apollo_step: %s\n", apollo_last_error(h));
      return 1;
    }
  }
  CHECK_HIP(hipDeviceSynchronize());
  CHECK_HIP(hipMemcpy(hw, dw, n * sizeof(float), hipMemcpyDeviceToHost));
  double sum = 0.0, sum_abs = 0.0;
  for (size_t k = 0; k < n; ++k) { sum += hw[k]; sum_abs += fabs((double)hw[k]); }
  printf("rank %d steps %d sum %.9e sum_abs %.9e w0 %.9e w_last %.9e\n", rank, steps, sum, sum_abs, (double)hw[0], (double)hw[n - 1]);
  apollo_destroy(h);
  CHECK_HIP(hipFree(dw)); CHECK_HIP(hipFree(dg)); CHECK_HIP(hipFree(dstate)); CHECK_HIP(hipFree(dws));
  free(hw); free(hg);
  return 0;
}
