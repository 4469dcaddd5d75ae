/*
 * dppf_cli -- the DPPF library used from plain C, with nothing but the HIP runtime API for
 * device memory: reads M workers' tensors from a file, runs one fused round (local momentum-SGD
 * step + pull-push update, Sec. 5 Eq. 5) through the C ABI of include/dppf.h and writes the
 * results.  It exists to show (and test) that the boundary carries no PyTorch types.
 *
 *   dppf_cli <input file> <output file>
 *
 * Input  (little endian): int32 M, int32 T, int64 numel[T], float32 lr, momentum, weight_decay,
 *                         pull, push, then x, v, g -- each as M consecutive vectors of d floats
 *                         (the T tensors of a worker back to back, d = sum numel).
 * Output: x (M*d floats), v (M*d floats), r (M floats), c (M floats).
 * Every tensor is given its own device allocation, as a model's parameter list would have.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "dppf.h"

#define CHECK_HIP(call)                                                              \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) {                                                          \
      fprintf(stderr, "dppf_cli: %s failed: %s\n", #call, hipGetErrorString(e_));    \
      return 3;                                                                      \
    }                                                                                \
  } while (0)

#define CHECK_DPPF(call)                                                             \
  do {                                                                               \
    int rc_ = (call);                                                                \
    if (rc_ != DPPF_OK) {                                                            \
      fprintf(stderr, "dppf_cli: %s failed: %s\n", #call, dppf_strerror(rc_));       \
      return 4;                                                                      \
    }                                                                                \
  } while (0)

static int read_exact(FILE* f, void* dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes ? 0 : -1; }

int main(int argc, char** argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: dppf_cli <input file> <output file>\n");
    return 2;
  }
  FILE* in = fopen(argv[1], "rb");
  if (!in) {
    fprintf(stderr, "dppf_cli: cannot open %s\n", argv[1]);
    return 2;
  }
  int32_t M = 0, T = 0;
  if (read_exact(in, &M, 4) || read_exact(in, &T, 4) || M < 1 || T < 0 || M > DPPF_MAX_WORKERS || T > (1 << 20)) {
    fprintf(stderr, "dppf_cli: bad header\n");
    return 2;
  }
  int64_t* numel = (int64_t*)calloc((size_t)T + 1, sizeof(int64_t));
  float hyper[5];
  if (!numel || read_exact(in, numel, (size_t)T * 8) || read_exact(in, hyper, sizeof hyper)) {
    fprintf(stderr, "dppf_cli: bad header\n");
    return 2;
  }
  int64_t d = 0;
  for (int t = 0; t < T; ++t) {
    if (numel[t] < 0) return 2;
    d += numel[t];
  }
  const size_t n = (size_t)M * (size_t)d;
  float* host[3];                     /* x, v, g */
  for (int a = 0; a < 3; ++a) {
    host[a] = (float*)malloc((n + 1) * sizeof(float));
    if (!host[a] || read_exact(in, host[a], n * sizeof(float))) {
      fprintf(stderr, "dppf_cli: input file too short\n");
      return 2;
    }
  }
  fclose(in);

  /* one device allocation per tensor, pointer tables worker-major */
  const size_t slots = (size_t)M * (size_t)T;
  float** table[3];
  for (int a = 0; a < 3; ++a) {
    table[a] = (float**)calloc(slots + 1, sizeof(float*));
    if (!table[a]) return 2;
    size_t pos = 0;
    for (int m = 0; m < M; ++m)
      for (int t = 0; t < T; ++t) {
        const size_t bytes = (size_t)numel[t] * sizeof(float);
        float* dev = NULL;
        if (bytes) {
          CHECK_HIP(hipMalloc((void**)&dev, bytes));
          CHECK_HIP(hipMemcpy(dev, host[a] + pos, bytes, hipMemcpyHostToDevice));
        }
        table[a][(size_t)m * T + t] = dev;
        pos += (size_t)numel[t];
      }
  }
  float *r_dev = NULL, *c_dev = NULL;
  CHECK_HIP(hipMalloc((void**)&r_dev, (size_t)M * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&c_dev, (size_t)M * sizeof(float)));

  dppf_plan* plan = NULL;
  CHECK_DPPF(dppf_plan_create(&plan, M, T, numel));
  hipStream_t stream;
  CHECK_HIP(hipStreamCreate(&stream));
  CHECK_DPPF(dppf_round(plan, table[0], table[1], (const float* const*)table[2], hyper[0], hyper[1], hyper[2],
                        hyper[3], hyper[4], r_dev, c_dev, NULL, (void*)stream));
  CHECK_HIP(hipStreamSynchronize(stream));

  FILE* out = fopen(argv[2], "wb");
  if (!out) {
    fprintf(stderr, "dppf_cli: cannot open %s\n", argv[2]);
    return 2;
  }
  for (int a = 0; a < 2; ++a) {
    size_t pos = 0;
    for (int m = 0; m < M; ++m)
      for (int t = 0; t < T; ++t) {
        const size_t bytes = (size_t)numel[t] * sizeof(float);
        if (bytes) CHECK_HIP(hipMemcpy(host[a] + pos, table[a][(size_t)m * T + t], bytes, hipMemcpyDeviceToHost));
        pos += (size_t)numel[t];
      }
    fwrite(host[a], sizeof(float), n, out);
  }
  float* small = (float*)malloc(2 * (size_t)M * sizeof(float));
  if (!small) return 2;
  CHECK_HIP(hipMemcpy(small, r_dev, (size_t)M * sizeof(float), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(small + M, c_dev, (size_t)M * sizeof(float), hipMemcpyDeviceToHost));
  fwrite(small, sizeof(float), 2 * (size_t)M, out);
  fclose(out);

  CHECK_DPPF(dppf_plan_destroy(plan));
  CHECK_HIP(hipStreamDestroy(stream));
  for (int a = 0; a < 3; ++a) {
    for (size_t i = 0; i < slots; ++i)
      if (table[a][i]) CHECK_HIP(hipFree(table[a][i]));
    free(table[a]);
    free(host[a]);
  }
  CHECK_HIP(hipFree(r_dev));
  CHECK_HIP(hipFree(c_dev));
  free(small);
  free(numel);
  return 0;
}
