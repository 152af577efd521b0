/* Plain-C user of the C ABI in include/sale.h: quantize -> select -> sparse attention -> dense attention on a
 * small seeded problem, with the checks a C caller can make without the oracle (status codes, counts = popcount
 * of the mask, sink / diagonal bits, finite outputs, "every block kept" == dense bit for bit).
 * Built with gcc by paper_2505_24179_amd/build.py; run by tests/test_gpu_c_abi.py.  Exit code 0 = all checks held. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "sale.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "abi_check: line %d: %s failed\n", __LINE__, #cond); \
      return 1;                                                            \
    }                                                                      \
  } while (0)
#define HIP(call) CHECK((call) == hipSuccess)

static uint32_t lcg(uint32_t* s) { *s = *s * 1664525u + 1013904223u; return *s; }
/* a value in about [-2, 2) as bf16 bits */
static uint16_t next_bf16(uint32_t* s) {
  const float x = (float)((int)(lcg(s) >> 8) - (1 << 23)) / (float)(1 << 22);
  uint32_t u;
  memcpy(&u, &x, 4);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
static float bf16_to_float(uint16_t b) { const uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return f; }
static int popcount64(uint64_t x) { int c = 0; while (x) { x &= x - 1; ++c; } return c; }

int main(void) {
  const int N = 512, HQ = 4, HKV = 2, D = 128, NQ = N / 64;
  sale_params_t p = {1, HQ, HKV, N, D, 64, 64, 1, 4, 0};
  CHECK(strcmp(sale_status_string(SALE_OK), "ok") == 0);
  sale_params_t bad = p;
  bad.seq_len = 500;
  CHECK(sale_quantize_qk(&bad, (void*)16, (void*)16, (uint8_t*)16, (uint8_t*)16, (float*)16, (float*)16, NULL) == SALE_ERR_BAD_SHAPE);
  CHECK(sale_workspace_bytes(&bad, SALE_WS_SELECT) == 0);

  const size_t nq_el = (size_t)HQ * N * D, nkv_el = (size_t)HKV * N * D;
  uint16_t* hq = malloc(nq_el * 2), *hk = malloc(nkv_el * 2), *hv = malloc(nkv_el * 2), *ho = malloc(nq_el * 2), *ho2 = malloc(nq_el * 2);
  CHECK(hq && hk && hv && ho && ho2);
  uint32_t seed = 2505u;
  for (size_t e = 0; e < nq_el; ++e) hq[e] = next_bf16(&seed);
  for (size_t e = 0; e < nkv_el; ++e) hk[e] = next_bf16(&seed);
  for (size_t e = 0; e < nkv_el; ++e) hv[e] = next_bf16(&seed);

  void *q, *k, *v, *o, *ws_sel, *ws_att;
  uint8_t *q4, *k4;
  float *qs, *ks, *tau;
  uint64_t* mask;
  int32_t* counts;
  const size_t sel_bytes = sale_workspace_bytes(&p, SALE_WS_SELECT), att_bytes = sale_workspace_bytes(&p, SALE_WS_SPARSE_ATTN);
  CHECK(sel_bytes > 0 && att_bytes > 0 && att_bytes > sale_workspace_bytes(&p, SALE_WS_DENSE_ATTN));
  CHECK(sale_workspace_bytes(&p, SALE_WS_SPARSE_ATTN_MIN) + (size_t)p.n_q_heads * (p.seq_len / 64) * SALE_PARKED_ROW_BYTES == att_bytes);
  HIP(hipMalloc(&q, nq_el * 2)); HIP(hipMalloc(&k, nkv_el * 2)); HIP(hipMalloc(&v, nkv_el * 2)); HIP(hipMalloc(&o, nq_el * 2));
  HIP(hipMalloc((void**)&q4, nq_el / 2)); HIP(hipMalloc((void**)&k4, nkv_el / 2));
  HIP(hipMalloc((void**)&qs, (size_t)HQ * NQ * 4)); HIP(hipMalloc((void**)&ks, (size_t)HKV * NQ * 4));
  HIP(hipMalloc((void**)&tau, 4)); HIP(hipMalloc((void**)&mask, (size_t)HQ * NQ * 8)); HIP(hipMalloc((void**)&counts, (size_t)HQ * NQ * 4));
  HIP(hipMalloc(&ws_sel, sel_bytes)); HIP(hipMalloc(&ws_att, att_bytes));
  HIP(hipMemcpy(q, hq, nq_el * 2, hipMemcpyHostToDevice));
  HIP(hipMemcpy(k, hk, nkv_el * 2, hipMemcpyHostToDevice));
  HIP(hipMemcpy(v, hv, nkv_el * 2, hipMemcpyHostToDevice));
  const float tau_h = 0.004f;
  HIP(hipMemcpy(tau, &tau_h, 4, hipMemcpyHostToDevice));

  CHECK(sale_quantize_qk(&p, q, k, q4, k4, qs, ks, NULL) == SALE_OK);
  CHECK(sale_select(&p, q, k, q4, k4, qs, ks, tau, 1, mask, counts, NULL, NULL, ws_sel, sel_bytes - 1, NULL) == SALE_ERR_WORKSPACE);
  CHECK(sale_select(&p, q, k, q4, k4, qs, ks, tau, 1, mask, counts, NULL, NULL, ws_sel, sel_bytes, NULL) == SALE_OK);
  CHECK(sale_sparse_attn(&p, q, k, v, mask, counts, o, NULL, ws_att, att_bytes, NULL) == SALE_OK);
  HIP(hipDeviceSynchronize());

  uint64_t hmask[4 * 8];
  int32_t hcounts[4 * 8];
  float hqs[4 * 8];
  HIP(hipMemcpy(hmask, mask, sizeof hmask, hipMemcpyDeviceToHost));
  HIP(hipMemcpy(hcounts, counts, sizeof hcounts, hipMemcpyDeviceToHost));
  HIP(hipMemcpy(hqs, qs, sizeof hqs, hipMemcpyDeviceToHost));
  HIP(hipMemcpy(ho, o, nq_el * 2, hipMemcpyDeviceToHost));
  for (int h = 0; h < HQ; ++h)
    for (int i = 0; i < NQ; ++i) {
      const uint64_t m = hmask[h * NQ + i];
      CHECK(popcount64(m) == hcounts[h * NQ + i]);
      CHECK((m >> (i + 1)) == 0);                       /* nothing above the diagonal */
      CHECK((m & 1u) && ((m >> i) & 1u));               /* sink and diagonal kept */
      CHECK(hqs[h * NQ + i] > 0.0f && hqs[h * NQ + i] < 1.0f);   /* scale = amax / 7 with |x| < 2 */
    }
  for (size_t e = 0; e < nq_el; ++e) CHECK(isfinite(bf16_to_float(ho[e])) && fabsf(bf16_to_float(ho[e])) <= 2.0f);

  /* every causal block kept == the dense kernel, bit for bit */
  uint64_t ones[4 * 8];
  for (int e = 0; e < 4 * 8; ++e) ones[e] = ~0ull;
  HIP(hipMemcpy(mask, ones, sizeof ones, hipMemcpyHostToDevice));
  CHECK(sale_sparse_attn(&p, q, k, v, mask, NULL, o, NULL, ws_att, att_bytes, NULL) == SALE_OK);
  HIP(hipMemcpy(ho, o, nq_el * 2, hipMemcpyDeviceToHost));
  CHECK(sale_dense_attn(&p, q, k, v, o, NULL, ws_att, att_bytes, NULL) == SALE_OK);
  HIP(hipMemcpy(ho2, o, nq_el * 2, hipMemcpyDeviceToHost));
  CHECK(memcmp(ho, ho2, nq_el * 2) == 0);
  /* row 0 attends to key 0 only: O[0] = V[0] */
  for (int h = 0; h < HQ; ++h) CHECK(memcmp(ho2 + (size_t)h * N * D, hv + (size_t)(h / (HQ / HKV)) * N * D, D * 2) == 0);

  printf("abi_check: ok\n");
  return 0;
}
