// Operands of the quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention"): the mean key of
// every KV head is subtracted from its keys (the softmax cancels the shift), then Q and the smoothed K get
// symmetric 8-bit codes in [-127, 127] with one fp32 scale per (head, 64-row block) - the arithmetic of the
// 4-bit quantizer with 127 in place of 7.
//
// All three kernels are HBM-bound and tiny next to the attention they feed (K is read twice, Q once).
#include "sale_common.h"

namespace sale {

// Exact column sums: bf16 values summed in fp64 lose nothing for any realistic value range, so the result
// does not depend on the order of the additions.  One workgroup per (KV head, 64-row tile): partial[c].
__global__ __launch_bounds__(256) void ksum_kernel(const uint16_t* __restrict__ k, Strided lk, int tiles_per_head,
                                                   double* __restrict__ partial) {
  __shared__ double other[128];
  const int c = threadIdx.x & 127, phase = threadIdx.x >> 7;
  const uint16_t* rows = k + row_off(lk, blockIdx.x / tiles_per_head, (blockIdx.x % tiles_per_head) * 64 + phase * 32) + c;
  double s = 0.0;
#pragma unroll 8
  for (int r = 0; r < 32; ++r) s += (double)bf16_bits_to_float(rows[(size_t)r * lk.st]);
  if (phase == 1) other[c] = s;
  __syncthreads();
  if (phase == 0) partial[(size_t)blockIdx.x * 128 + c] = s + other[c];
}

// mean[kvh][c] = fp32(sum over the head's tiles / N).  One workgroup per KV head.
__global__ __launch_bounds__(128) void kmean_kernel(const double* __restrict__ partial, int tiles, int seq,
                                                    float* __restrict__ mean) {
  const int c = threadIdx.x;
  const double* p = partial + (size_t)blockIdx.x * tiles * 128 + c;
  double s = 0.0;
  for (int t = 0; t < tiles; ++t) s += p[(size_t)t * 128];
  mean[blockIdx.x * 128 + c] = (float)(s / (double)seq);
}

// One workgroup per (head, 64-row block).  Thread t holds 32 channels (32 (t % 4) ..) of row t / 4.
// FRAG: codes go out in the operand order of v_mfma_i32_32x32x32_i8 for the keys-as-rows product,
//   [head][tile][mt 0..1][ks 0..3][lane 0..63] 16 bytes: channels 32ks + 16(lane/32) .. of key row 32mt + lane%32;
// otherwise row-major [head][row][128 bytes].
template <bool FRAG>
__global__ __launch_bounds__(256) void quantize8_kernel(const uint16_t* __restrict__ x, Strided lx,
                                                        const float* __restrict__ mean, int tiles_per_head,
                                                        int8_t* __restrict__ codes, float* __restrict__ scale) {
  __shared__ float wave_max[4];
  const int t = threadIdx.x, r = t >> 2, cq = t & 3;
  const size_t blk = blockIdx.x;
  const u32x4* src = (const u32x4*)(x + row_off(lx, (int)(blk / tiles_per_head), (int)(blk % tiles_per_head) * 64 + r) + 32 * cq);
  float v[32];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u32x4 w = __builtin_nontemporal_load(&src[i]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[8 * i + 2 * e] = __builtin_bit_cast(float, w[e] << 16);
      v[8 * i + 2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xFFFF0000u);
    }
  }
  if (mean) {
    const float* m = mean + (blk / tiles_per_head) * 128 + 32 * cq;
#pragma unroll
    for (int e = 0; e < 32; ++e) v[e] = v[e] - m[e];
  }
  float amax = 0.0f;
#pragma unroll
  for (int e = 0; e < 32; ++e) amax = fmaxf(amax, fabsf(v[e]));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
  if ((t & 63) == 0) wave_max[t >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
  const bool zero = amax == 0.0f;
  const float inv = zero ? 0.0f : 127.0f / amax;      // IEEE division, as in the definition
  if (t == 0) scale[blk] = zero ? 1.0f : amax / 127.0f;
  uint32_t packed[8];
#pragma unroll
  for (int w = 0; w < 8; ++w) {
    uint32_t word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const float y = rintf(v[4 * w + b] * inv);
      const int code = (int)fminf(fmaxf(y, -127.0f), 127.0f);
      word |= (uint32_t)(code & 0xFF) << (8 * b);
    }
    packed[w] = word;
  }
  u32x4 lo, hi;
  lo[0] = packed[0]; lo[1] = packed[1]; lo[2] = packed[2]; lo[3] = packed[3];
  hi[0] = packed[4]; hi[1] = packed[5]; hi[2] = packed[6]; hi[3] = packed[7];
  if (FRAG) {
    u32x4* dst = (u32x4*)codes + blk * 512 + ((r >> 5) * 4 + cq) * 64 + (r & 31);
    dst[0] = lo;      // channels 32cq .. +15   -> lanes 0..31
    dst[32] = hi;     // channels 32cq+16 .. +31 -> lanes 32..63
  } else {
    u32x4* dst = (u32x4*)(codes + (blk * 64 + r) * kHeadDim + 32 * cq);
    dst[0] = lo;
    dst[1] = hi;
  }
}

size_t int8_operand_bytes(const sale_params_t* p) {
  const size_t rows = (size_t)p->batch * p->n_q_heads * p->seq_len;
  const size_t kvrows = (size_t)p->batch * p->n_kv_heads * p->seq_len;
  // Q codes | K codes | Q scales | K scales | key means | column-sum partials (fp64)
  return rows * kHeadDim + kvrows * kHeadDim + (rows / 64 + kvrows / 64) * sizeof(float) +
         (size_t)p->batch * p->n_kv_heads * 128 * sizeof(float) + (kvrows / 64) * 128 * sizeof(double) + 64;
}

Int8Operands carve_int8_operands(const sale_params_t* p, void* base) {
  const size_t rows = (size_t)p->batch * p->n_q_heads * p->seq_len;
  const size_t kvrows = (size_t)p->batch * p->n_kv_heads * p->seq_len;
  Int8Operands w;
  uint8_t* b = (uint8_t*)base;
  w.q8 = (int8_t*)b;                       b += rows * kHeadDim;
  w.k8 = (int8_t*)b;                       b += kvrows * kHeadDim;
  w.partial = (double*)b;                  b += (kvrows / 64) * 128 * sizeof(double);   // 8-byte aligned: all sizes above are multiples of 64
  w.q_scale = (float*)b;                   b += (rows / 64) * sizeof(float);
  w.k_scale = (float*)b;                   b += (kvrows / 64) * sizeof(float);
  w.k_mean = (float*)b;
  return w;
}

// Fills the operand copies: Q codes row-major, K codes in fragment order (frag_k) or row-major.
int launch_int8_operands(const sale_params_t* p, const void* q, const void* k, const Int8Operands& w, bool frag_k,
                         hipStream_t st) {
  const int n_kvh = p->batch * p->n_kv_heads, n_qh = p->batch * p->n_q_heads, tiles = p->seq_len / 64;
  const Geo g = make_geo(p);
  ksum_kernel<<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)k, g.sk, tiles, w.partial);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  kmean_kernel<<<dim3((unsigned)n_kvh), dim3(128), 0, st>>>(w.partial, tiles, p->seq_len, w.k_mean);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  quantize8_kernel<false><<<dim3((unsigned)(n_qh * tiles)), dim3(256), 0, st>>>((const uint16_t*)q, g.sq, nullptr, tiles,
                                                                               w.q8, w.q_scale);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  if (frag_k)
    quantize8_kernel<true><<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)k, g.sk, w.k_mean, tiles,
                                                                                 w.k8, w.k_scale);
  else
    quantize8_kernel<false><<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)k, g.sk, w.k_mean, tiles,
                                                                                  w.k8, w.k_scale);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

}  // namespace sale

using namespace sale;

extern "C" int sale_attn_int8_operands(const sale_params_t* p, const void* q, const void* k, int8_t* q8, int8_t* k8,
                                       float* q_scale8, float* k_scale8, float* k_mean, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (!p || !q || !k || !q8 || !k8 || !q_scale8 || !k_scale8 || !k_mean) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  const size_t need = sale_workspace_bytes(p, SALE_WS_INT8_OPERANDS);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  Int8Operands w;
  w.q8 = q8; w.k8 = k8; w.q_scale = q_scale8; w.k_scale = k_scale8; w.k_mean = k_mean;
  w.partial = (double*)ws;
  return launch_int8_operands(p, q, k, w, false, (hipStream_t)stream);
}
