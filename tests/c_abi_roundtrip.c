/*
 * The C ABI used from plain C, with no Python and no PyTorch in the process: device memory from the HIP runtime, one
 * small multimodal prompt through akvq_select_salient -> akvq_quantize_append -> akvq_decode_attention (grouped-query,
 * two KV splits), checked against the CPU oracle linked into the same program: cache bit-exact, attention within
 * 2e-3.  Test infrastructure (it links the oracle); built by __graft_entry__.build(), run by tests/test_gpu_c_abi.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "akvq.h"
#include "akvq_oracle.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_AKVQ(x) do { int s_ = (x); if (s_ != AKVQ_OK) { \
  fprintf(stderr, "akvq error %d (%s) at %s:%d\n", s_, akvq_strerror(s_), __FILE__, __LINE__); return 3; } } while (0)

static uint32_t lcg_state = 2501u;
static float next_uniform(void) {  /* [-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(int32_t)lcg_state * (1.0f / 2147483648.0f);
}

int main(void) {
  enum { B = 2, Hkv = 2, Hq = 4, G = 128, T = 150, T_cap = 192, S_cap = 64, D = 128, n_split = 2 };
  const float clip = 0.8f, sm_scale = 0.08838834764831845f;
  const size_t n_kv = (size_t)B * Hkv * T * D, n_q = (size_t)B * Hq * D;

  /* inputs: uniform values, one outlier channel per head, the first 6 and the last 4 positions are text */
  uint16_t *k = malloc(n_kv * 2), *v = malloc(n_kv * 2), *q = malloc(n_q * 2);
  uint8_t *is_text = calloc((size_t)B * T, 1);
  for (size_t i = 0; i < n_kv; ++i) {
    float x = 2.0f * next_uniform();
    if (i % D == 5) x *= 10.0f;
    k[i] = orc_float_to_half_rne(x);
    v[i] = orc_float_to_half_rne(2.0f * next_uniform());
  }
  for (size_t i = 0; i < n_q; ++i) q[i] = orc_float_to_half_rne(next_uniform());
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t) is_text[b * T + t] = (t < 6 || t >= T - 4);

  /* ---- the library, on the GPU ---- */
  akvq_cache gc = {B, Hkv, G, T_cap, S_cap, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  size_t bytes[8];
  CHECK_AKVQ(akvq_cache_bytes(&gc, bytes));
  void *dev[8];
  for (int i = 0; i < 8; ++i) {
    CHECK_HIP(hipMalloc(&dev[i], bytes[i]));
    CHECK_HIP(hipMemset(dev[i], 0, bytes[i]));
  }
  gc.k_codes = dev[0]; gc.v_codes = dev[1]; gc.k_meta = dev[2]; gc.v_meta = dev[3];
  gc.k_sal = dev[4]; gc.v_sal = dev[5]; gc.sal_idx = dev[6]; gc.sal_cnt = dev[7];
  void *d_k, *d_v, *d_q, *d_text, *d_out, *d_lse, *d_ws;
  const size_t ws_bytes = akvq_decode_workspace_bytes(B, Hq, n_split);
  CHECK_HIP(hipMalloc(&d_k, n_kv * 2)); CHECK_HIP(hipMalloc(&d_v, n_kv * 2)); CHECK_HIP(hipMalloc(&d_q, n_q * 2));
  CHECK_HIP(hipMalloc(&d_text, (size_t)B * T)); CHECK_HIP(hipMalloc(&d_out, n_q * 4));
  CHECK_HIP(hipMalloc(&d_lse, (size_t)B * Hq * 4)); CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
  CHECK_HIP(hipMemcpy(d_k, k, n_kv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_v, v, n_kv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_q, q, n_q * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_text, is_text, (size_t)B * T, hipMemcpyHostToDevice));

  if (akvq_quantize_append(&gc, d_k, d_v, 0, clip, 0, NULL) != AKVQ_ERR_INVALID_ARG) {  /* rejected on the host */
    fprintf(stderr, "an empty append was not rejected\n");
    return 4;
  }
  CHECK_AKVQ(akvq_select_salient(&gc, AKVQ_MODE_TSA, d_text, NULL, Hkv, NULL, T, 0, 0, 0.0f, NULL, NULL, 0, NULL));
  CHECK_AKVQ(akvq_quantize_append(&gc, d_k, d_v, T, clip, 0, NULL));
  gc.T_len = T;
  CHECK_AKVQ(akvq_decode_attention(&gc, d_q, Hq, sm_scale, d_out, d_lse, n_split, d_ws, ws_bytes, 0, NULL));
  CHECK_HIP(hipDeviceSynchronize());

  /* ---- the oracle, on the CPU ---- */
  orc_cache oc = {B, Hkv, G, T_cap, S_cap, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  void *host[8];
  for (int i = 0; i < 8; ++i) host[i] = calloc(bytes[i], 1);
  oc.k_codes = host[0]; oc.v_codes = host[1]; oc.k_meta = host[2]; oc.v_meta = host[3];
  oc.k_sal = host[4]; oc.v_sal = host[5]; oc.sal_idx = host[6]; oc.sal_cnt = host[7];
  orc_select_tsa(&oc, is_text, T);
  orc_quantize_append(&oc, k, v, T, clip, ORC_ROT_K | ORC_ROT_V);
  oc.T_len = T;
  double *ref = malloc(n_q * sizeof(double)), *ref_lse = malloc((size_t)B * Hq * sizeof(double));
  orc_decode_attention(&oc, Hq, q, (double)sm_scale, ORC_ROT_Q | ORC_ROT_OUT, ref, ref_lse);

  /* ---- compare ---- */
  static const char *names[8] = {"k_codes", "v_codes", "k_meta", "v_meta", "k_sal", "v_sal", "sal_idx", "sal_cnt"};
  int bad = 0;
  for (int i = 0; i < 8; ++i) {
    void *got = malloc(bytes[i]);
    CHECK_HIP(hipMemcpy(got, dev[i], bytes[i], hipMemcpyDeviceToHost));
    if (i == 6) {  /* only the first sal_cnt entries of a list are defined */
      const int32_t *g = got, *o = host[6], *cnt = host[7];
      for (int u = 0; u < B * Hkv; ++u)
        if (memcmp(g + (size_t)u * S_cap, o + (size_t)u * S_cap, (size_t)cnt[u] * 4) != 0) { ++bad; printf("sal_idx differs\n"); }
    } else if (i == 7) {
      if (memcmp(got, host[7], (size_t)B * Hkv * 4) != 0) { ++bad; printf("sal_cnt differs\n"); }
    } else if (memcmp(got, host[i], bytes[i]) != 0) {
      ++bad;
      printf("%s differs\n", names[i]);
    }
    free(got);
  }
  float *out = malloc(n_q * 4), *lse = malloc((size_t)B * Hq * 4);
  CHECK_HIP(hipMemcpy(out, d_out, n_q * 4, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(lse, d_lse, (size_t)B * Hq * 4, hipMemcpyDeviceToHost));
  double worst = 0.0;
  for (int r = 0; r < B * Hq; ++r) {
    double err = 0.0, scale = 1e-6;
    for (int d = 0; d < D; ++d) {
      err = fmax(err, fabs((double)out[r * D + d] - ref[r * D + d]));
      scale = fmax(scale, fabs(ref[r * D + d]));
    }
    worst = fmax(worst, err / scale);
    if (fabs((double)lse[r] - ref_lse[r]) > 2e-3) { ++bad; printf("lse of row %d differs\n", r); }
  }
  if (worst > 2e-3) { ++bad; printf("attention error %.3e\n", worst); }
  if (bad) { printf("FAIL c_abi_roundtrip\n"); return 1; }
  printf("PASS c_abi_roundtrip: cache bit-exact, attention rel err %.2e\n", worst);
  return 0;
}
