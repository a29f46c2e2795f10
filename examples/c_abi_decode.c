/* The C-ABI on its own: plain C, HIP runtime calls for memory, no Python, no PyTorch.
 *
 * One layer, two sequences, 8 query / 2 KV heads (group size 4), fp32; KV head 0 keeps its full
 * history, KV head 1 keeps 4 sink tokens and a ring of the 12 most recent ones (paper Sec. 3.3 /
 * App. B).  A 40-token prompt is appended, then three decode steps run through
 * rlkv_append_decode; every step's output is checked against softmax attention written out on
 * the host over the positions each head may see (Eq. 1 with the gate at 1 or 0).
 *
 * Build (done by `python -m paper_2510_08525_amd.build`):
 *   gcc -std=c11 -O2 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude examples/c_abi_decode.c \
 *       -Lpaper_2510_08525_amd -lrlkv -L/opt/rocm/lib -lamdhip64 -lm -o examples/c_abi_decode
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "rlkv.h"

enum { L = 1, HQ = 8, HKV = 2, D = 128, B = 2, S = 4, R = 12, PROMPT = 40, STEPS = 3, CAP = PROMPT + STEPS };

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP: %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define RLKV_OK_(x) do { rlkv_status_t s_ = (x); if (s_ != RLKV_OK) { fprintf(stderr, "rlkv: %s (line %d)\n", rlkv_status_string(s_), __LINE__); return 3; } } while (0)

static unsigned lcg_state = 12345u;
static float next_value(void) {                       /* uniform in [-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(lcg_state >> 8) / 8388608.0f - 1.0f;
}

/* history[b][h][pos][d], kept on the host for the check */
static float k_hist[B][HKV][CAP][D], v_hist[B][HKV][CAP][D];

static double check(const float* q, const float* out, int n, const unsigned char* mask, float scale) {
  double worst = 0.0;
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < HQ; ++i) {
      const int h = i / (HQ / HKV);
      double s[CAP], m = -1e300, z = 0.0, o[D];
      int seen[CAP];
      for (int j = 0; j < n; ++j) {
        seen[j] = mask[h] || j < S || j >= n - R;
        if (!seen[j]) continue;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += (double)q[(b * HQ + i) * D + d] * k_hist[b][h][j][d];
        s[j] = dot * scale;
        if (s[j] > m) m = s[j];
      }
      memset(o, 0, sizeof o);
      for (int j = 0; j < n; ++j) {
        if (!seen[j]) continue;
        const double w = exp(s[j] - m);
        z += w;
        for (int d = 0; d < D; ++d) o[d] += w * v_hist[b][h][j][d];
      }
      for (int d = 0; d < D; ++d) {
        const double err = fabs(o[d] / z - (double)out[(b * HQ + i) * D + d]);
        if (err > worst) worst = err;
      }
    }
  return worst;
}

int main(void) {
  const unsigned char mask[L * HKV] = {1, 0};
  const int32_t max_len[B] = {CAP, CAP};
  rlkv_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = D; cfg.batch = B;
  cfg.sink = S; cfg.recent = R; cfg.dtype = RLKV_F32; cfg.kernel = RLKV_KERNEL_AUTO; cfg.device = 0;
  cfg.full_mask = mask; cfg.max_len = max_len;
  cfg.arena_bytes = rlkv_cache_required_bytes(&cfg);
  if (cfg.arena_bytes == 0) { fprintf(stderr, "configuration rejected\n"); return 1; }
  HIP_OK(hipSetDevice(0));
  HIP_OK(hipMalloc(&cfg.arena, cfg.arena_bytes));        /* the caller's memory; the library never frees it */
  rlkv_cache_t* cache = NULL;
  RLKV_OK_(rlkv_cache_create(&cfg, &cache));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  /* prompt: [batch][n_kv_heads][PROMPT][D] */
  static float k_prompt[B][HKV][PROMPT][D], v_prompt[B][HKV][PROMPT][D];
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < HKV; ++h)
      for (int p = 0; p < PROMPT; ++p)
        for (int d = 0; d < D; ++d) {
          k_hist[b][h][p][d] = k_prompt[b][h][p][d] = next_value();
          v_hist[b][h][p][d] = v_prompt[b][h][p][d] = next_value();
        }
  float *dk, *dv, *dq, *dout, *dk1, *dv1;
  HIP_OK(hipMalloc((void**)&dk, sizeof k_prompt));
  HIP_OK(hipMalloc((void**)&dv, sizeof v_prompt));
  HIP_OK(hipMalloc((void**)&dk1, sizeof(float) * B * HKV * D));
  HIP_OK(hipMalloc((void**)&dv1, sizeof(float) * B * HKV * D));
  HIP_OK(hipMalloc((void**)&dq, sizeof(float) * B * HQ * D));
  HIP_OK(hipMalloc((void**)&dout, sizeof(float) * B * HQ * D));
  HIP_OK(hipMemcpyAsync(dk, k_prompt, sizeof k_prompt, hipMemcpyHostToDevice, stream));
  HIP_OK(hipMemcpyAsync(dv, v_prompt, sizeof v_prompt, hipMemcpyHostToDevice, stream));
  RLKV_OK_(rlkv_append(cache, 0, dk, dv, PROMPT, stream));

  const float scale = 1.0f / sqrtf((float)D);
  double worst = 0.0;
  for (int step = 0; step < STEPS; ++step) {
    const int n = PROMPT + step + 1;                     /* cached positions after this step's append */
    static float k1[B][HKV][D], v1[B][HKV][D], q[B * HQ * D], out[B * HQ * D];
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < HKV; ++h)
        for (int d = 0; d < D; ++d) {
          k_hist[b][h][n - 1][d] = k1[b][h][d] = next_value();
          v_hist[b][h][n - 1][d] = v1[b][h][d] = next_value();
        }
    for (int i = 0; i < B * HQ * D; ++i) q[i] = 4.0f * next_value();
    HIP_OK(hipMemcpyAsync(dk1, k1, sizeof k1, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dv1, v1, sizeof v1, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dq, q, sizeof q, hipMemcpyHostToDevice, stream));
    RLKV_OK_(rlkv_append_decode(cache, 0, dk1, dv1, dq, dout, scale, stream));
    HIP_OK(hipMemcpyAsync(out, dout, sizeof out, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    const double err = check(q, out, n, mask, scale);
    printf("step %d: %d positions cached, worst |error| %.3g\n", step, n, err);
    if (err > worst) worst = err;
  }
  int32_t lengths[B];
  RLKV_OK_(rlkv_get_lengths(cache, 0, lengths));
  printf("lengths %d %d, resident store bytes %zu\n", lengths[0], lengths[1], rlkv_resident_bytes(cache));
  RLKV_OK_(rlkv_cache_destroy(cache));
  HIP_OK(hipFree(cfg.arena));
  HIP_OK(hipFree(dk)); HIP_OK(hipFree(dv)); HIP_OK(hipFree(dk1)); HIP_OK(hipFree(dv1)); HIP_OK(hipFree(dq)); HIP_OK(hipFree(dout));
  HIP_OK(hipStreamDestroy(stream));
  if (worst > 1e-5 || lengths[0] != CAP || lengths[1] != CAP) { printf("FAILED\n"); return 1; }
  printf("OK\n");
  return 0;
}
