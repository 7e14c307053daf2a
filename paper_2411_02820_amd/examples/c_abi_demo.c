/*
 * The C ABI of libdsk used from plain C, with the HIP runtime alone for device memory (no Python, no torch):
 * a small fp32 model, a selective prefill of layers [1, 3) of 4 over one 96-token prefix whose other layers are
 * spliced from a synthetic sender cache (Sec. 4.1), then the suffix pass over 8 new tokens.  Prints "ok" when the
 * spliced layers are the sender's bytes and every output is finite.
 *
 * Built by `python -m paper_2411_02820_amd.build` as paper_2411_02820_amd/dsk_c_demo.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "dsk.h"

#define HIP_OK(call)                                                          \
  do {                                                                        \
    hipError_t e_ = (call);                                                   \
    if (e_ != hipSuccess) {                                                   \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));              \
      return 1;                                                               \
    }                                                                         \
  } while (0)
#define DSK_OK_(call)                                                         \
  do {                                                                        \
    int s_ = (call);                                                          \
    if (s_ != DSK_OK) {                                                       \
      fprintf(stderr, "%s: %s (hip %d)\n", #call, dsk_strerror(s_), dsk_last_hip_error()); \
      return 1;                                                               \
    }                                                                         \
  } while (0)

enum { L = 4, D = 256, HQ = 4, HKV = 2, DH = 64, F = 688, T = 96, S = 8, ROWS = T + S };

int main(void) {
  dsk_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L; cfg.hidden = D; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = DH; cfg.ffn = F;
  cfg.rope_base = 10000.0; cfg.rms_eps = 1e-5; cfg.dtype = DSK_F32;

  dsk_model_t* model = NULL;
  DSK_OK_(dsk_model_create(&cfg, T, ROWS, &model));
  DSK_OK_(dsk_model_init_random(model, 0, 0.16f, NULL));

  const size_t kvw = (size_t)HKV * DH, layer_elems = 2 * (size_t)ROWS * kvw, kv_bytes = L * layer_elems * sizeof(float);
  float *hidden_in, *hidden_out, *suffix_in, *suffix_out, *kv_sender, *kv_out;
  HIP_OK(hipMalloc((void**)&hidden_in, (size_t)T * D * sizeof(float)));
  HIP_OK(hipMalloc((void**)&hidden_out, (size_t)T * D * sizeof(float)));
  HIP_OK(hipMalloc((void**)&suffix_in, (size_t)S * D * sizeof(float)));
  HIP_OK(hipMalloc((void**)&suffix_out, (size_t)S * D * sizeof(float)));
  HIP_OK(hipMalloc((void**)&kv_sender, kv_bytes));
  HIP_OK(hipMalloc((void**)&kv_out, kv_bytes));
  HIP_OK(hipMemset(kv_out, 0, kv_bytes));
  DSK_OK_(dsk_fill_normal(hidden_in, (int64_t)T * D, 2, 0, 1.0f, 0.0f, 0, DSK_F32, NULL));
  DSK_OK_(dsk_fill_normal(suffix_in, (int64_t)S * D, 4, 0, 1.0f, 0.0f, 0, DSK_F32, NULL));
  DSK_OK_(dsk_fill_normal(kv_sender, (int64_t)(L * layer_elems), 3, 0, 1.0f, 0.0f, 0, DSK_F32, NULL));

  /* one sequence: prefix rows 0..T-1 at positions 0..T-1, suffix rows at positions T..T+S-1 */
  int32_t cu_prefix[2] = {0, T}, cu_suffix[2] = {0, S}, pos[T + S];
  for (int i = 0; i < T + S; ++i) pos[i] = i;
  int32_t *cu_prefix_dev, *cu_suffix_dev, *pos_dev;
  HIP_OK(hipMalloc((void**)&cu_prefix_dev, sizeof cu_prefix));
  HIP_OK(hipMalloc((void**)&cu_suffix_dev, sizeof cu_suffix));
  HIP_OK(hipMalloc((void**)&pos_dev, sizeof pos));
  HIP_OK(hipMemcpy(cu_prefix_dev, cu_prefix, sizeof cu_prefix, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(cu_suffix_dev, cu_suffix, sizeof cu_suffix, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(pos_dev, pos, sizeof pos, hipMemcpyHostToDevice));
  dsk_batch_t prefix = {1, T, cu_prefix, cu_prefix_dev, pos_dev};
  dsk_batch_t suffix = {1, S, cu_suffix, cu_suffix_dev, pos_dev + T};

  dsk_kv_t reused = {kv_sender, DSK_MEM_DEVICE, (int64_t)(layer_elems * sizeof(float)), (int64_t)(ROWS * kvw * sizeof(float)), ROWS};
  dsk_kv_t mixed = {kv_out, DSK_MEM_DEVICE, (int64_t)(layer_elems * sizeof(float)), (int64_t)(ROWS * kvw * sizeof(float)), ROWS};

  DSK_OK_(dsk_partial_prefill(model, hidden_in, DSK_MEM_DEVICE, 1, 3, &reused, &mixed, &prefix, hidden_out, 0, NULL));
  DSK_OK_(dsk_suffix_prefill(model, suffix_in, &mixed, &prefix, &suffix, T, suffix_out, NULL));
  HIP_OK(hipDeviceSynchronize());

  /* layer 0 is reused: its first T K rows are the sender's bytes; layer 1 was recomputed: they are not */
  const size_t n_check = (size_t)T * kvw;
  float *a = malloc(n_check * sizeof(float)), *b = malloc(n_check * sizeof(float));
  float* out_host = malloc((size_t)S * D * sizeof(float));
  if (!a || !b || !out_host) return 1;
  HIP_OK(hipMemcpy(a, kv_out, n_check * sizeof(float), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(b, kv_sender, n_check * sizeof(float), hipMemcpyDeviceToHost));
  const int spliced = memcmp(a, b, n_check * sizeof(float)) == 0;
  HIP_OK(hipMemcpy(a, kv_out + layer_elems, n_check * sizeof(float), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(b, kv_sender + layer_elems, n_check * sizeof(float), hipMemcpyDeviceToHost));
  const int recomputed = memcmp(a, b, n_check * sizeof(float)) != 0;
  HIP_OK(hipMemcpy(out_host, suffix_out, (size_t)S * D * sizeof(float), hipMemcpyDeviceToHost));
  int finite = 1;
  double norm = 0.0;
  for (size_t i = 0; i < (size_t)S * D; ++i) {
    if (!isfinite(out_host[i])) finite = 0;
    norm += (double)out_host[i] * out_host[i];
  }
  printf("reused layer spliced bit for bit: %d, recomputed layer fresh: %d, suffix output finite: %d (rms %.4f)\n", spliced,
         recomputed, finite, sqrt(norm / (S * D)));

  DSK_OK_(dsk_model_destroy(model));
  free(a); free(b); free(out_host);
  hipFree(hidden_in); hipFree(hidden_out); hipFree(suffix_in); hipFree(suffix_out); hipFree(kv_sender); hipFree(kv_out);
  hipFree(cu_prefix_dev); hipFree(cu_suffix_dev); hipFree(pos_dev);
  if (!(spliced && recomputed && finite)) return 1;
  printf("ok\n");
  return 0;
}
