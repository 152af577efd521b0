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

// mean[kvh][c] = fp32(sum over the head's tiles / N).  One workgroup of 1024 threads per KV head: 8 threads per
// channel take every 8th tile each, four loads in flight, and meet in LDS.  (The partial sums are fp64 sums of
// bf16 values: exact for any data whose exponents span less than 53 - 8 - log2(N) bits, so the order is free.)
__global__ __launch_bounds__(1024) void kmean_kernel(const double* __restrict__ partial, int tiles, int seq,
                                                     float* __restrict__ mean) {
  __shared__ double part[8][128];
  const int c = threadIdx.x & 127, ph = threadIdx.x >> 7;
  const double* p = partial + (size_t)blockIdx.x * tiles * 128 + c;
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  int t = ph;
  for (; t + 24 < tiles; t += 32) {
    s0 += p[(size_t)t * 128]; s1 += p[(size_t)(t + 8) * 128]; s2 += p[(size_t)(t + 16) * 128]; s3 += p[(size_t)(t + 24) * 128];
  }
  for (; t < tiles; t += 8) s0 += p[(size_t)t * 128];
  part[ph][c] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (ph == 0) {
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += part[i][c];
    mean[blockIdx.x * 128 + c] = (float)(s / (double)seq);
  }
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

// ---------------------------------------------------------------------------
// V of the low-precision second product: OCP FP8 E4M3 values with one fp32 scale per (KV head, channel),
//   amax = max over the head's N tokens of |v|;  scale = amax / 448;  value = fp8(v * (448 / amax))
// (IEEE fp32, one multiply, round to nearest even; an all-zero channel gets scale 1 and values 0).
// ---------------------------------------------------------------------------
// Per (KV head, 64-row tile): partial[c] = max |v| over the tile's rows.
__global__ __launch_bounds__(256) void vamax_kernel(const uint16_t* __restrict__ v, Strided lv, int tiles_per_head,
                                                    float* __restrict__ partial) {
  __shared__ float other[128];
  const int c = threadIdx.x & 127, phase = threadIdx.x >> 7;
  const uint16_t* rows = v + row_off(lv, blockIdx.x / tiles_per_head, (blockIdx.x % tiles_per_head) * 64 + phase * 32) + c;
  float m = 0.0f;
#pragma unroll 8
  for (int r = 0; r < 32; ++r) m = fmaxf(m, fabsf(bf16_bits_to_float(rows[(size_t)r * lv.st])));
  if (phase == 1) other[c] = m;
  __syncthreads();
  if (phase == 0) partial[(size_t)blockIdx.x * 128 + c] = fmaxf(m, other[c]);
}

// Per KV head: scale[c] = amax / 448 and inv[c] = 448 / amax (1 and 0 for an all-zero channel).  1024 threads as
// in kmean_kernel.
__global__ __launch_bounds__(1024) void vscale_kernel(const float* __restrict__ partial, int tiles, float* __restrict__ scale,
                                                      float* __restrict__ inv) {
  __shared__ float part[8][128];
  const int c = threadIdx.x & 127, ph = threadIdx.x >> 7;
  const float* p = partial + (size_t)blockIdx.x * tiles * 128 + c;
  float m0 = 0.0f, m1 = 0.0f, m2 = 0.0f, m3 = 0.0f;
  int t = ph;
  for (; t + 24 < tiles; t += 32) {
    m0 = fmaxf(m0, p[(size_t)t * 128]); m1 = fmaxf(m1, p[(size_t)(t + 8) * 128]);
    m2 = fmaxf(m2, p[(size_t)(t + 16) * 128]); m3 = fmaxf(m3, p[(size_t)(t + 24) * 128]);
  }
  for (; t < tiles; t += 8) m0 = fmaxf(m0, p[(size_t)t * 128]);
  part[ph][c] = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
  __syncthreads();
  if (ph == 0) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, part[i][c]);
    const bool zero = amax == 0.0f;
    scale[blockIdx.x * 128 + c] = zero ? 1.0f : amax / 448.0f;
    inv[blockIdx.x * 128 + c] = zero ? 0.0f : 448.0f / amax;
  }
}

__device__ __forceinline__ uint32_t fp8x4(float a, float b, float c, float d) {
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
  return (uint32_t)w;
}

// One workgroup per (KV head, 64-key tile).
// FRAG: the values go out as the A operand of v_mfma_f32_32x32x64_f8f6f4 for O^T += V^T P^T,
//   [head][tile][dt 0..3][j 0..1][lane 0..63] 16 bytes: channel 32 dt + lane % 32 of the 16 keys
//   32 j + 8 (e / 4) + 4 (lane / 32) + e % 4, e = 0..15
// (the order in which the S^T accumulator registers of half-tile j hand P^T to the second product);
// otherwise row-major [head][key][128 bytes].
template <bool FRAG>
__global__ __launch_bounds__(256) void quantize_v8_kernel(const uint16_t* __restrict__ v, Strided lv, int tiles_per_head,
                                                          const float* __restrict__ inv, uint8_t* __restrict__ out) {
  __shared__ float sv[64 * (kHeadDim + 1)];      // v * inv, rows padded by one bank
  const int tid = threadIdx.x;
  const size_t tile = blockIdx.x;
  const int head = (int)(tile / tiles_per_head);
  const uint16_t* vt = v + row_off(lv, head, (int)(tile % tiles_per_head) * 64);
  const float* iv = inv + (size_t)head * 128;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int chunk = tid + 256 * r;
    const int row = chunk >> 4, col = (chunk & 15) * 8;
    const u32x4 w = *(const u32x4*)(vt + (size_t)row * lv.st + col);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sv[row * (kHeadDim + 1) + col + 2 * e] = __builtin_bit_cast(float, w[e] << 16) * iv[col + 2 * e];
      sv[row * (kHeadDim + 1) + col + 2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xFFFF0000u) * iv[col + 2 * e + 1];
    }
  }
  __syncthreads();
  if (FRAG) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int oc = tid + 256 * r;
      const int lane = oc & 63, j = (oc >> 6) & 1, dt = oc >> 7;
      const int d = 32 * dt + (lane & 31), h = lane >> 5;
      u32x4 o4;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int key = 32 * j + 8 * w + 4 * h;      // e = 4 w .. 4 w + 3
        o4[w] = fp8x4(sv[key * (kHeadDim + 1) + d], sv[(key + 1) * (kHeadDim + 1) + d], sv[(key + 2) * (kHeadDim + 1) + d],
                      sv[(key + 3) * (kHeadDim + 1) + d]);
      }
      ((u32x4*)out)[tile * 512 + oc] = o4;
    }
  } else {
    const int row = tid >> 2, cq = tid & 3;
    const float* src = sv + row * (kHeadDim + 1) + 32 * cq;
    u32x4 lo, hi;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      lo[w] = fp8x4(src[4 * w], src[4 * w + 1], src[4 * w + 2], src[4 * w + 3]);
      hi[w] = fp8x4(src[16 + 4 * w], src[17 + 4 * w], src[18 + 4 * w], src[19 + 4 * w]);
    }
    u32x4* dst = (u32x4*)(out + (tile * 64 + row) * kHeadDim + 32 * cq);
    dst[0] = lo;
    dst[1] = hi;
  }
}

size_t fp8_operand_bytes(const sale_params_t* p) {
  const size_t kvrows = (size_t)p->batch * p->n_kv_heads * p->seq_len;
  // V values | scales | inverse scales | per-tile maxima
  return kvrows * kHeadDim + 2 * (size_t)p->batch * p->n_kv_heads * 128 * sizeof(float) + (kvrows / 64) * 128 * sizeof(float) + 64;
}

Fp8Operands carve_fp8_operands(const sale_params_t* p, void* base) {
  const size_t kvrows = (size_t)p->batch * p->n_kv_heads * p->seq_len;
  const size_t heads = (size_t)p->batch * p->n_kv_heads;
  Fp8Operands w;
  uint8_t* b = (uint8_t*)base;
  w.v8 = b;                   b += kvrows * kHeadDim;
  w.v_scale = (float*)b;      b += heads * 128 * sizeof(float);
  w.v_inv = (float*)b;        b += heads * 128 * sizeof(float);
  w.partial = (float*)b;
  return w;
}

int launch_fp8_operands(const sale_params_t* p, const void* v, const Fp8Operands& w, bool frag, hipStream_t st) {
  const int n_kvh = p->batch * p->n_kv_heads, tiles = p->seq_len / 64;
  const Geo g = make_geo(p);
  vamax_kernel<<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)v, g.sv, tiles, w.partial);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  vscale_kernel<<<dim3((unsigned)n_kvh), dim3(1024), 0, st>>>(w.partial, tiles, w.v_scale, w.v_inv);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  if (frag)
    quantize_v8_kernel<true><<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)v, g.sv, tiles, w.v_inv, w.v8);
  else
    quantize_v8_kernel<false><<<dim3((unsigned)(n_kvh * tiles)), dim3(256), 0, st>>>((const uint16_t*)v, g.sv, tiles, w.v_inv, w.v8);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
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
  kmean_kernel<<<dim3((unsigned)n_kvh), dim3(1024), 0, st>>>(w.partial, tiles, p->seq_len, w.k_mean);
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

extern "C" int sale_attn_fp8_operands(const sale_params_t* p, const void* v, uint8_t* v8, float* v_scale, void* ws,
                                      size_t ws_bytes, void* stream) {
  if (!p || !v || !v8 || !v_scale) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  const size_t need = sale_workspace_bytes(p, SALE_WS_FP8_OPERANDS);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  Fp8Operands w;
  w.v8 = v8; w.v_scale = v_scale;
  w.v_inv = (float*)ws;
  w.partial = w.v_inv + (size_t)p->batch * p->n_kv_heads * 128;
  return launch_fp8_operands(p, v, w, false, (hipStream_t)stream);
}
