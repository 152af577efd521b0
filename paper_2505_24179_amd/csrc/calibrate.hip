// Per-head threshold calibration (Sec. 3.3): Err(tau) = ||O - O~||_1 / N between full attention and
// SALE, tau starting at tau0 and halved until Err(tau) < theta.
//
// An offline procedure built from the path's own calls: quantize once, dense attention once, then per
// round select -> sparse attention -> L1 distance per head, with the per-head decision taken on the host.
// Both outputs are taken in fp32 (before the bf16 rounding of the output), otherwise the rounding noise
// of two bf16 tensors (about 2^-8 |o| per differing element) would drown the distances being compared.
#include <stdlib.h>
#include <string.h>

#include "sale_common.h"

namespace sale {

// One workgroup per flattened (batch, head): err[bh] = sum |a - b| over its N x d elements, in a fixed
// order (each thread strides over 16-byte chunks, then a tree over the workgroup).
__global__ __launch_bounds__(1024) void l1_distance_kernel(const f32x4* __restrict__ a, const f32x4* __restrict__ b,
                                                           size_t chunks_per_head, double* __restrict__ err) {
  __shared__ double part[1024];
  const f32x4* pa = a + (size_t)blockIdx.x * chunks_per_head;
  const f32x4* pb = b + (size_t)blockIdx.x * chunks_per_head;
  double s = 0.0;
  for (size_t i = threadIdx.x; i < chunks_per_head; i += 1024) {
    const f32x4 x = pa[i], y = pb[i];
    s += (double)(fabsf(x[0] - y[0]) + fabsf(x[1] - y[1])) + (double)(fabsf(x[2] - y[2]) + fabsf(x[3] - y[3]));
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) err[blockIdx.x] = part[0];
}

struct CalibWs {
  uint8_t *q4, *k4;
  float *qs, *ks, *tau, *o_full, *o_sale;
  uint64_t* mask;
  int32_t* counts;
  double* err;
  void *ws_sel, *ws_att;
  size_t sel_bytes, att_bytes, total;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static CalibWs carve(const sale_params_t* p, void* base) {
  const size_t B = p->batch, Hq = p->n_q_heads, Hkv = p->n_kv_heads, N = p->seq_len;
  const size_t nq = N / kBlockQ, nk = N / (size_t)p->block_k, words = (nk + 63) / 64;
  CalibWs c;
  size_t off = 0;
  auto take = [&](size_t bytes) { uint8_t* ptr = (uint8_t*)base + off; off += align256(bytes); return ptr; };
  c.q4 = take(B * Hq * N * 64);
  c.k4 = take(B * Hkv * N * 64);
  c.qs = (float*)take(B * Hq * nq * 4);
  c.ks = (float*)take(B * Hkv * nk * 4);
  c.tau = (float*)take(Hq * 4);
  c.o_full = (float*)take(B * Hq * N * kHeadDim * 4);
  c.o_sale = (float*)take(B * Hq * N * kHeadDim * 4);
  c.mask = (uint64_t*)take(B * Hq * nq * words * 8);
  c.counts = (int32_t*)take(B * Hq * nq * 4);
  c.err = (double*)take(B * Hq * 8);
  c.sel_bytes = sale_workspace_bytes(p, SALE_WS_SELECT);
  c.att_bytes = sale_workspace_bytes(p, SALE_WS_SPARSE_ATTN);
  c.ws_sel = take(c.sel_bytes);
  c.ws_att = take(c.att_bytes);
  c.total = off;
  return c;
}

size_t calibrate_workspace_bytes(const sale_params_t* p) { return carve(p, nullptr).total; }

}  // namespace sale

using namespace sale;

extern "C" int sale_calibrate_tau(const sale_params_t* p, const void* q, const void* k, const void* v, float tau0,
                                  float theta, int32_t max_halvings, float* tau_out, float* err_out,
                                  int32_t* halvings_out, void* ws, size_t ws_bytes, void* stream) {
  if (!p || !q || !k || !v || !tau_out) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  if (!(tau0 > 0.0f && tau0 < 1.0f) || !(theta > 0.0f) || max_halvings < 0 || max_halvings > 64) return SALE_ERR_BAD_SHAPE;
  if (p->n_q_heads > 4096 || p->batch > 4096 || p->n_seqs > 0) return SALE_ERR_UNSUPPORTED;
  const size_t need = sale_workspace_bytes(p, SALE_WS_CALIBRATE);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 255)) return SALE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const CalibWs c = carve(p, ws);
  const int B = p->batch, Hq = p->n_q_heads;
  const size_t N = p->seq_len;

  float* tau_h = (float*)malloc(sizeof(float) * Hq);
  double* err_h = (double*)malloc(sizeof(double) * (size_t)B * Hq);
  float* err_head = (float*)malloc(sizeof(float) * Hq);
  int32_t* halv = (int32_t*)malloc(sizeof(int32_t) * Hq);
  char* done = (char*)calloc(Hq, 1);
  auto finish = [&](int code) {
    free(tau_h); free(err_h); free(err_head); free(halv); free(done);
    return code;
  };
  if (!tau_h || !err_h || !err_head || !halv || !done) return finish(SALE_ERR_HIP);
  for (int h = 0; h < Hq; ++h) { tau_h[h] = tau0; halv[h] = 0; err_head[h] = 0.0f; }

  rc = sale_quantize_qk(p, q, k, c.q4, c.k4, c.qs, c.ks, stream);
  if (rc != SALE_OK) return finish(rc);
  sale_params_t full = *p;      // O of Sec. 3.3 is full attention in full precision
  full.flags &= ~(SALE_FLAG_ATTN_INT8_QK | SALE_FLAG_ATTN_FP8_PV);
  rc = launch_attn_rows(&full, q, k, v, nullptr, nullptr, nullptr, c.o_full, nullptr, c.ws_att, c.att_bytes, st);
  if (rc != SALE_OK) return finish(rc);

  for (int round = 0; round <= max_halvings; ++round) {
    if (hipMemcpyAsync(c.tau, tau_h, sizeof(float) * Hq, hipMemcpyHostToDevice, st) != hipSuccess) return finish(SALE_ERR_HIP);
    rc = sale_select(p, q, k, c.q4, c.k4, c.qs, c.ks, c.tau, Hq, c.mask, c.counts, nullptr, nullptr, c.ws_sel, c.sel_bytes,
                     stream);
    if (rc != SALE_OK) return finish(rc);
    rc = launch_attn_rows(p, q, k, v, c.mask, c.counts, nullptr, c.o_sale, nullptr, c.ws_att, c.att_bytes, st);
    if (rc != SALE_OK) return finish(rc);
    l1_distance_kernel<<<dim3((unsigned)(B * Hq)), dim3(1024), 0, st>>>((const f32x4*)c.o_full, (const f32x4*)c.o_sale,
                                                                        N * kHeadDim / 4, c.err);
    if (hipGetLastError() != hipSuccess) return finish(SALE_ERR_HIP);
    if (hipMemcpyAsync(err_h, c.err, sizeof(double) * (size_t)B * Hq, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
      return finish(SALE_ERR_HIP);
    bool all_done = true;
    for (int h = 0; h < Hq; ++h) {
      if (done[h]) continue;
      double worst = 0.0;      // every sample (batch entry) has to satisfy the bound
      for (int b = 0; b < B; ++b) worst = err_h[(size_t)b * Hq + h] > worst ? err_h[(size_t)b * Hq + h] : worst;
      err_head[h] = (float)(worst / (double)N);
      if (err_head[h] < theta || round == max_halvings) {
        done[h] = 1;
      } else {
        tau_h[h] *= 0.5f;
        halv[h] = round + 1;
        all_done = false;
      }
    }
    if (all_done) break;
  }
  if (hipMemcpyAsync(tau_out, tau_h, sizeof(float) * Hq, hipMemcpyHostToDevice, st) != hipSuccess) return finish(SALE_ERR_HIP);
  if (err_out && hipMemcpyAsync(err_out, err_head, sizeof(float) * Hq, hipMemcpyHostToDevice, st) != hipSuccess)
    return finish(SALE_ERR_HIP);
  if (halvings_out && hipMemcpyAsync(halvings_out, halv, sizeof(int32_t) * Hq, hipMemcpyHostToDevice, st) != hipSuccess)
    return finish(SALE_ERR_HIP);
  if (hipStreamSynchronize(st) != hipSuccess) return finish(SALE_ERR_HIP);   // the host buffers are freed below
  return finish(SALE_OK);
}
