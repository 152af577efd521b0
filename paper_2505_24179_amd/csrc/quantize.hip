// Quantization stage (Sec. 3.2, "4-bit attention weight approximation"):
// per (head, row-block) symmetric 4-bit codes of Q and K with one fp32 scale.
//
// HBM-bound: every bf16 element is read once (16-byte loads, kept in
// registers between the amax reduction and the rounding) and every packed
// byte written once.  One workgroup handles one block of ROWS x 128 elements.
#include "sale_common.h"

namespace sale {

template <int ROWS>
__global__ __launch_bounds__(256) void quantize_kernel(int seq, const uint16_t* __restrict__ xa, Strided la,
                                                       uint32_t* __restrict__ ca, float* __restrict__ sa, int n_blocks_a,
                                                       const uint16_t* __restrict__ xb, Strided lb,
                                                       uint32_t* __restrict__ cb, float* __restrict__ sb) {
  constexpr int CH = ROWS * 16 / 256;   // 16-byte chunks per thread
  __shared__ float wave_max[4];
  int blk = blockIdx.x;
  const uint16_t* x = xa;
  Strided lay = la;
  uint32_t* codes = ca;
  float* scale = sa;
  if (blk >= n_blocks_a) { blk -= n_blocks_a; x = xb; lay = lb; codes = cb; scale = sb; }
  const size_t base = (size_t)blk * (ROWS * 16);      // 16-byte chunk (input) / dword (codes) index of the block
  const int t = threadIdx.x;
  // block blk = rows (blk % bph) * ROWS .. of flat head blk / bph; chunk t + 256 i = row (t / 16 + 16 i), chunk t % 16
  const int bph = seq / ROWS;
  const uint16_t* first = x + row_off(lay, blk / bph, (blk % bph) * ROWS + (t >> 4)) + 8 * (t & 15);

  u32x4 raw[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) raw[i] = __builtin_nontemporal_load((const u32x4*)(first + (size_t)(16 * i) * lay.st));

  float v[CH][8];
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const uint32_t w[4] = {raw[i][0], raw[i][1], raw[i][2], raw[i][3]};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[i][2 * e] = __builtin_bit_cast(float, w[e] << 16);
      v[i][2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xFFFF0000u);
      amax = fmaxf(amax, fmaxf(fabsf(v[i][2 * e]), fabsf(v[i][2 * e + 1])));
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
  if ((t & 63) == 0) wave_max[t >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));

  const bool zero = amax == 0.0f;
  const float inv = zero ? 0.0f : 7.0f / amax;          // IEEE fp32 divide
  if (t == 0) scale[blk] = zero ? 1.0f : amax / 7.0f;

#pragma unroll
  for (int i = 0; i < CH; ++i) {
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float r = rintf(v[i][e] * inv);                   // one multiply, ties to even
      r = fminf(fmaxf(r, -7.0f), 7.0f);
      packed |= ((uint32_t)(int)r & 0xFu) << (4 * e);
    }
    __builtin_nontemporal_store(packed, &codes[base + t + 256 * i]);
  }
}

template <int ROWS>
static int launch_quant(int seq, const void* xa, const Strided& la, uint8_t* ca, float* sa, long blocks_a, const void* xb,
                        const Strided& lb, uint8_t* cb, float* sb, long blocks_b, hipStream_t st) {
  long total = blocks_a + blocks_b;
  if (total == 0) return SALE_OK;
  quantize_kernel<ROWS><<<dim3((unsigned)total), dim3(256), 0, st>>>(seq, (const uint16_t*)xa, la, (uint32_t*)ca, sa,
                                                                    (int)blocks_a, (const uint16_t*)xb, lb, (uint32_t*)cb, sb);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

}  // namespace sale

using namespace sale;

extern "C" int sale_quantize_qk(const sale_params_t* p, const void* q, const void* k, uint8_t* q4, uint8_t* k4,
                                float* q_scale, float* k_scale, void* stream) {
  if (!p || !q || !k || !q4 || !k4 || !q_scale || !k_scale) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomQuantize);
  if (rc != SALE_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const Geo g = make_geo(p);
  const int n = p->seq_len;
  const long rows_q = (long)p->batch * p->n_q_heads * p->seq_len;
  const long rows_k = (long)p->batch * p->n_kv_heads * p->seq_len;
  if (p->block_q == p->block_k) {
    return p->block_q == 64 ? launch_quant<64>(n, q, g.sq, q4, q_scale, rows_q / 64, k, g.sk, k4, k_scale, rows_k / 64, st)
                            : launch_quant<32>(n, q, g.sq, q4, q_scale, rows_q / 32, k, g.sk, k4, k_scale, rows_k / 32, st);
  }
  rc = p->block_q == 64 ? launch_quant<64>(n, q, g.sq, q4, q_scale, rows_q / 64, nullptr, g.sq, nullptr, nullptr, 0, st)
                        : launch_quant<32>(n, q, g.sq, q4, q_scale, rows_q / 32, nullptr, g.sq, nullptr, nullptr, 0, st);
  if (rc != SALE_OK) return rc;
  return p->block_k == 64 ? launch_quant<64>(n, k, g.sk, k4, k_scale, rows_k / 64, nullptr, g.sk, nullptr, nullptr, 0, st)
                          : launch_quant<32>(n, k, g.sk, k4, k_scale, rows_k / 32, nullptr, g.sk, nullptr, nullptr, 0, st);
}
