/*
 * The C ABI used from plain C, without Python or PyTorch: build a k-NN graph of
 * n seeded pseudo-random points with gnnd_build, check it against gnnd_exact_knn
 * on every node, print one line.  Device memory comes from hipMalloc here; the
 * library itself never allocates any.
 *
 *   abi_demo [n] [d] [k] [p] [iterations]      (defaults 20000 16 16 8 8)
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "gnnd.h"

#define CHECK_HIP(call)                                                        \
  do {                                                                         \
    hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) {                                                    \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));               \
      return 2;                                                                \
    }                                                                          \
  } while (0)

static unsigned long long next_random(unsigned long long* state) {
  unsigned long long z = (*state += 0x9e3779b97f4a7c15ULL);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ULL;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebULL;
  return z ^ (z >> 31);
}

int main(int argc, char** argv) {
  const long long n = argc > 1 ? atoll(argv[1]) : 20000;
  const int d = argc > 2 ? atoi(argv[2]) : 16;
  const int k = argc > 3 ? atoi(argv[3]) : 16;
  const int p = argc > 4 ? atoi(argv[4]) : 8;
  const int iters = argc > 5 ? atoi(argv[5]) : 8;
  const int K = 10; /* recall is judged on the first 10 neighbours */

  float* x = (float*)malloc(sizeof(float) * (size_t)n * d);
  unsigned long long state = 7;
  for (long long i = 0; i < n * d; ++i) x[i] = (float)(next_random(&state) >> 40) / 16777216.0f;

  gnnd_params prm;
  memset(&prm, 0, sizeof prm);
  prm.n = n;
  prm.d = d;
  prm.k = k;
  prm.p = p;
  prm.metric = GNND_L2SQ_F32;
  prm.seed = 42;
  prm.join_path = GNND_JOIN_AUTO;
  prm.update_mode = GNND_UPDATE_SELECTIVE;
  const size_t need = gnnd_workspace_bytes(&prm);
  if (need == 0) {
    fprintf(stderr, "invalid parameters\n");
    return 2;
  }

  float *x_dev, *dist_dev, *truth_dist_dev;
  int32_t *ids_dev, *truth_ids_dev, *queries_dev;
  void* workspace;
  CHECK_HIP(hipMalloc((void**)&x_dev, sizeof(float) * (size_t)n * d));
  CHECK_HIP(hipMalloc(&workspace, need));
  CHECK_HIP(hipMalloc((void**)&ids_dev, sizeof(int32_t) * (size_t)n * k));
  CHECK_HIP(hipMalloc((void**)&dist_dev, sizeof(float) * (size_t)n * k));
  CHECK_HIP(hipMalloc((void**)&queries_dev, sizeof(int32_t) * (size_t)n));
  CHECK_HIP(hipMalloc((void**)&truth_ids_dev, sizeof(int32_t) * (size_t)n * K));
  CHECK_HIP(hipMalloc((void**)&truth_dist_dev, sizeof(float) * (size_t)n * K));
  CHECK_HIP(hipMemcpy(x_dev, x, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice));
  prm.workspace_dev = workspace;
  prm.workspace_bytes = need;

  gnnd_ctx* ctx = NULL;
  gnnd_iter_stats last;
  if (gnnd_create(&ctx, &prm, x_dev) != GNND_OK || gnnd_build(ctx, iters, 0.0f, &last) != GNND_OK ||
      gnnd_get_graph(ctx, ids_dev, dist_dev, NULL) != GNND_OK) {
    fprintf(stderr, "gnnd: %s\n", gnnd_last_error(ctx));
    return 1;
  }

  int32_t* q = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  for (long long i = 0; i < n; ++i) q[i] = (int32_t)i;
  CHECK_HIP(hipMemcpy(queries_dev, q, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
  if (gnnd_exact_knn(x_dev, n, d, GNND_L2SQ_F32, queries_dev, n, K, truth_ids_dev, truth_dist_dev,
                     NULL) != GNND_OK) {
    fprintf(stderr, "gnnd: %s\n", gnnd_last_error(NULL));
    return 1;
  }
  CHECK_HIP(hipDeviceSynchronize());

  float* dist = (float*)malloc(sizeof(float) * (size_t)n * k);
  float* truth = (float*)malloc(sizeof(float) * (size_t)n * K);
  int32_t* ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * k);
  CHECK_HIP(hipMemcpy(dist, dist_dev, sizeof(float) * (size_t)n * k, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(ids, ids_dev, sizeof(int32_t) * (size_t)n * k, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(truth, truth_dist_dev, sizeof(float) * (size_t)n * K, hipMemcpyDeviceToHost));

  /* Recall@10 with ties: a listed neighbour counts when it is no farther than the exact 10-th */
  long long hits = 0, bad = 0;
  for (long long i = 0; i < n; ++i) {
    const float limit = truth[i * K + K - 1];
    for (int j = 0; j < K && j < k; ++j) hits += dist[i * k + j] <= limit;
    for (int j = 0; j < k; ++j) {
      bad += ids[i * k + j] == (int32_t)i || ids[i * k + j] < 0 || ids[i * k + j] >= n;
      if (j > 0) bad += dist[i * k + j] < dist[i * k + j - 1];
    }
  }
  const double recall = (double)hits / (double)(n * K);
  printf("abi_demo n=%lld d=%d k=%d p=%d iterations=%d recall@10=%.4f malformed=%lld "
         "inserts_last=%llu\n", n, d, k, p, last.iter, recall, bad,
         (unsigned long long)last.inserts);

  gnnd_destroy(ctx);
  hipFree(x_dev); hipFree(workspace); hipFree(ids_dev); hipFree(dist_dev);
  hipFree(queries_dev); hipFree(truth_ids_dev); hipFree(truth_dist_dev);
  free(x); free(q); free(dist); free(truth); free(ids);
  return (bad == 0 && recall > 0.9) ? 0 : 1;
}
