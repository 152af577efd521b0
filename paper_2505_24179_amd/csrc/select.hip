// Selection-Pass (Alg. 1): sink-local statistics from the unquantized Q, K,
// then the 4-bit Q~ K~^T estimate of every middle block scored against
// thr_r = ln(tau l~_r) + m~_r (Eq. 3 in the log form of Eq. 4), written as one
// bit per (query block, key block).
//
// Both kernels compute the TRANSPOSED tile, keys x queries (A operand = K rows,
// B operand = Q rows).  In the 32x32 MFMA accumulator layout a lane then owns
// 16 keys of ONE query column, so the per-query maximum over a key block is an
// in-lane max chain, the per-query threshold is a single register, and the
// "any row of the block passes" reduction is the wave-wide compare mask.
//
// CDNA4 has no int4 MFMA: the integer products run, exactly, on the FP6 MFMA
// (see below).
#include "sale_common.h"

namespace sale {

__device__ __forceinline__ bool in_sink_local(const Geo& g, int j, int j_last) {
  return j < g.sink_blocks || j > j_last - g.local_blocks;
}

// ---------------------------------------------------------------------------
// Sink-local statistics (display equation of Sec. 3.2; first loop of Alg. 1)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stats_kernel(Geo g, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                    const float* __restrict__ tau, int tau_len, float* __restrict__ thr,
                                                    float* __restrict__ m_out, float* __restrict__ l_out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const Unit u = unit_of(g, blockIdx.x, wave);
  if (!u.valid) return;
  const int c = lane & 31, h = lane >> 5;
  const float rsd = 0.08838834764831845f;   // 1 / sqrt(128)

  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + ((size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c) * kHeadDim + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }
  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.0f, 0.0f};
  const int j_last = u.i;   // b_q == b_k
  for (int j = 0; j <= j_last; ++j) {
    if (!in_sink_local(g, j, j_last)) { j = j_last - g.local_blocks; continue; }
    f32x16 acc[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const uint16_t* row = k + ((size_t)u.kvh * g.seq + j * 64 + 32 * mt + c) * kHeadDim + 8 * h;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8 a = *(const bf16x8*)(row + 16 * s);
        acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], acc[mt][1], 0, 0, 0);
      }
    }
    const bool mask_diag = g.stats_causal && j == j_last;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float s[32];
      float mx = -INFINITY;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float x = acc[mt][nt][r] * rsd;
          if (mask_diag && (32 * mt + mfma32_row(r, lane)) > (32 * nt + c)) x = -INFINITY;
          s[mt * 16 + r] = x;
          mx = fmaxf(mx, x);
        }
      const float m_new = fmaxf(m[nt], mx);
      const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
      float sum = 0.0f;
#pragma unroll
      for (int e = 0; e < 32; ++e) sum += __expf(s[e] - m_safe);
      l[nt] = l[nt] * __expf(m[nt] - m_safe) + sum;
      m[nt] = m_new;
    }
  }
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float m_o = swap_half(m[nt]), l_o = swap_half(l[nt]);
    const float m_t = fmaxf(m[nt], m_o);
    const float m_safe = m_t == -INFINITY ? 0.0f : m_t;
    const float l_t = l[nt] * __expf(m[nt] - m_safe) + l_o * __expf(m_o - m_safe);
    if (h == 0) {
      const size_t idx = (size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c;
      const float t = tau[tau_len == 1 ? 0 : u.qh % g.hq_per_b];
      thr[idx] = __logf(t * l_t) + m_t;
      if (m_out) m_out[idx] = m_t;
      if (l_out) l_out[idx] = l_t;
    }
  }
}

// ---------------------------------------------------------------------------
// 4-bit estimate on the FP6 (E2M3) MFMA
// ---------------------------------------------------------------------------
// CDNA4 has no int4 MFMA.  Every integer in [-7, 7] is exactly representable in
// FP6 E2M3 (1 sign, 2 exponent, 3 mantissa bits, bias 1: 1 = 0b001000, 2 =
// 0b010000, 3 = 0b010100, 4 = 0b011000, 5 = 0b011010, 6 = 0b011100, 7 =
// 0b011110), products are at most 49 and a 128-term sum at most 6272 < 2^24, so
// v_mfma_f32_32x32x64_f8f6f4 with both operands in E2M3 and unit scales returns
// the integer product EXACTLY in its fp32 accumulator (checked on hardware
// against integer arithmetic, including all-(+-7) operands) at twice the int8
// MFMA rate.  A pre-pass re-encodes the nibble codes once into MFMA operand
// order ("X6"): per 64-row block 4 fragments f = 2*t + ks (rows 32t.., channels
// 64ks..); lane l of a fragment owns row 32t + l%32, channels 64ks + 32(l/32) +
// e, e = 0..31, as 32 six-bit codes = 6 dwords, stored as
//   [block][f][lane] 16 bytes (dwords 0..3)  followed by  [block][f][lane] 8 bytes (dwords 4..5).
constexpr int kX6BlockBytes = 4 * 64 * 24;   // 6144

// E2M3 code of a 4-bit two's-complement nibble n (-7..7).
__device__ __forceinline__ uint32_t e2m3_of_nibble(uint32_t n) {
  const uint32_t sign = (n >> 3) & 1u;
  const uint32_t mag = ((n ^ (0u - sign)) + sign) & 7u;          // |value|
  return (sign << 5) | (((0xFEDCA840u >> (4u * mag)) & 0xFu) << 1);
}

// 16 packed bytes (32 nibble codes, channel order) -> 32 six-bit codes in 6 dwords.
__device__ __forceinline__ void pack_fp6(const u32x4 w, uint32_t out[6]) {
  uint64_t acc = 0;
  int bits = 0, o = 0;
#pragma unroll
  for (int e = 0; e < 32; ++e) {
    const uint32_t nib = (w[e >> 3] >> (4 * (e & 7))) & 0xFu;
    acc |= (uint64_t)e2m3_of_nibble(nib) << bits;
    bits += 6;
    if (bits >= 32) {
      out[o++] = (uint32_t)acc;
      acc >>= 32;
      bits -= 32;
    }
  }
}

// One thread per (block, fragment, lane) of a nibble-packed [rows][64-byte] matrix.
__global__ __launch_bounds__(256) void pack_fp6_kernel(const uint8_t* __restrict__ xa, uint8_t* __restrict__ ya,
                                                       long blocks_a, const uint8_t* __restrict__ xb,
                                                       uint8_t* __restrict__ yb) {
  long blk = blockIdx.x;
  const uint8_t* x = xa;
  uint8_t* y = ya;
  if (blk >= blocks_a) { blk -= blocks_a; x = xb; y = yb; }
  const int f = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = f >> 1, ks = f & 1;
  const u32x4 w = *(const u32x4*)(x + ((size_t)blk * 64 + 32 * t + (lane & 31)) * 64 + 32 * ks + 16 * (lane >> 5));
  uint32_t d[6];
  pack_fp6(w, d);
  uint8_t* yb_ = y + (size_t)blk * kX6BlockBytes;
  u32x4 lo;
  lo[0] = d[0]; lo[1] = d[1]; lo[2] = d[2]; lo[3] = d[3];
  u32x2 hi;
  hi[0] = d[4]; hi[1] = d[5];
  *(u32x4*)(yb_ + (f * 64 + lane) * 16) = lo;
  *(u32x2*)(yb_ + 4096 + (f * 64 + lane) * 8) = hi;
}

// The 4 operand fragments of block `blk` of an X6 array.
__device__ __forceinline__ void load_x6(const uint8_t* __restrict__ base, size_t blk, int lane, i32x8 f[4]) {
  const uint8_t* b = base + blk * kX6BlockBytes;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u32x4 lo = *(const u32x4*)(b + (i * 64 + lane) * 16);
    const u32x2 hi = *(const u32x2*)(b + 4096 + (i * 64 + lane) * 8);
    f[i][0] = lo[0]; f[i][1] = lo[1]; f[i][2] = lo[2]; f[i][3] = lo[3];
    f[i][4] = hi[0]; f[i][5] = hi[1]; f[i][6] = 0; f[i][7] = 0;
  }
}

// acc[mt][nt] = (K~ tile mt) (Q~ tile nt)^T, keys x queries, exact integers held in fp32.
__device__ __forceinline__ void qk_tile_fp6(const i32x8 kf[4], const i32x8 qf[4], f32x16 acc[2][2]) {
  // the two k-steps of a tile depend on each other: issue the four tiles' first steps, then their second
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const f32x16 z = {0};
      acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[2 * mt], qf[2 * nt], z, 2, 2, 0, 0, 0, 0);
    }
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
      acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[2 * mt + 1], qf[2 * nt + 1], acc[mt][nt], 2, 2, 0, 0, 0, 0);
}

// One wave scores HPW query heads of one GQA group at the same query block, so every K~ fragment it
// loads feeds HPW x 2 MFMAs.  A workgroup is 4 such waves (consecutive head sets / query blocks of one
// KV head); workgroups go round-robin over KV heads, longest rows first.
// (At least 2 waves per SIMD caps the register file at 256 VGPRs, which lets the MFMA results land in
// ordinary VGPRs instead of AGPRs that the max chain would have to copy out one by one.)
template <int HPW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void select_kernel(Geo g, const uint8_t* __restrict__ q6, const uint8_t* __restrict__ k6,
                                                     const float* __restrict__ q_scale, const float* __restrict__ k_scale,
                                                     const float* __restrict__ thr, uint64_t* __restrict__ mask,
                                                     int32_t* __restrict__ row_counts) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = lane & 31;
  const int sets = g.group / HPW;                 // head sets per (KV head, query block)
  const int units = g.n_qb * sets;
  const int tiles = (units + 3) / 4;
  const int kvh = blockIdx.x % g.n_kvh;
  const int id = (tiles - 1 - blockIdx.x / g.n_kvh) * 4 + wave;
  if (id >= units) return;
  const int i = id / sets;
  const int qh0 = kvh * g.group + (id % sets) * HPW;

  i32x8 qf[HPW][4];
  float th[HPW][2], cq[HPW];
#pragma unroll
  for (int a = 0; a < HPW; ++a) {
    load_x6(q6, (size_t)(qh0 + a) * g.n_qb + i, lane, qf[a]);
    th[a][0] = thr[(size_t)(qh0 + a) * g.seq + i * 64 + c];
    th[a][1] = thr[(size_t)(qh0 + a) * g.seq + i * 64 + 32 + c];
    cq[a] = q_scale[(size_t)(qh0 + a) * g.n_qb + i] * 0.08838834764831845f;   // s_q / sqrt(d)
  }
  const float* ks = k_scale + (size_t)kvh * g.n_kb;
  const size_t kblk0 = (size_t)kvh * g.n_kb;

  const int j_last = i;
  int count[HPW];
#pragma unroll
  for (int a = 0; a < HPW; ++a) count[a] = 0;
  for (int wc = 0; wc < g.words; ++wc) {
    uint64_t word[HPW];
#pragma unroll
    for (int a = 0; a < HPW; ++a) word[a] = 0;
    const int j_end = min(64, j_last + 1 - wc * 64);
    for (int jj = 0; jj < j_end; ++jj) {
      const int j = wc * 64 + jj;
      if (in_sink_local(g, j, j_last)) {
#pragma unroll
        for (int a = 0; a < HPW; ++a) word[a] |= 1ull << jj;
        continue;
      }
      i32x8 kf[4];
      load_x6(k6, kblk0 + j, lane, kf);
      const float sk = ks[j];
#pragma unroll
      for (int a = 0; a < HPW; ++a) {
        f32x16 acc[2][2];
        qk_tile_fp6(kf, qf[a], acc);
        const float cj = cq[a] * sk;
        bool pass = false;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          float mx = fmaxf(acc[0][nt][0], acc[1][nt][0]);
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, acc[0][nt][r]), acc[1][nt][r]);
          pass = pass || (mx * cj >= th[a][nt]);
        }
        word[a] |= (uint64_t)(__ballot(pass) != 0ull) << jj;
      }
    }
#pragma unroll
    for (int a = 0; a < HPW; ++a) {
      if (lane == 0) mask[((size_t)(qh0 + a) * g.n_qb + i) * g.words + wc] = word[a];
      count[a] += __popcll(word[a]);
    }
  }
#pragma unroll
  for (int a = 0; a < HPW; ++a)
    if (lane == 0) row_counts[(size_t)(qh0 + a) * g.n_qb + i] = count[a];
}

// Appendix E ablation ("w/o QK Quant"): the same rule with the estimate taken from the 16-bit Q, K
// themselves (S~ = S, bf16 MFMA with fp32 accumulation): four times the MFMA work of the FP6 estimate.
__global__ __launch_bounds__(256) void select16_kernel(Geo g, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                       const float* __restrict__ thr, uint64_t* __restrict__ mask,
                                                       int32_t* __restrict__ row_counts) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const Unit u = unit_of(g, blockIdx.x, wave);
  if (!u.valid) return;
  const int c = lane & 31, h = lane >> 5;
  const float rsd = 0.08838834764831845f;   // 1 / sqrt(128)
  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + ((size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c) * kHeadDim + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }
  float th[2];
  th[0] = thr[(size_t)u.qh * g.seq + u.i * 64 + c];
  th[1] = thr[(size_t)u.qh * g.seq + u.i * 64 + 32 + c];
  uint64_t* mrow = mask + ((size_t)u.qh * g.n_qb + u.i) * g.words;
  const int j_last = u.i;
  int count = 0;
  for (int wc = 0; wc < g.words; ++wc) {
    uint64_t word = 0;
    const int j_end = min(64, j_last + 1 - wc * 64);
    for (int jj = 0; jj < j_end; ++jj) {
      const int j = wc * 64 + jj;
      if (in_sink_local(g, j, j_last)) { word |= 1ull << jj; continue; }
      f32x16 acc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const uint16_t* row = k + ((size_t)u.kvh * g.seq + j * 64 + 32 * mt + c) * kHeadDim + 8 * h;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bf16x8 a = *(const bf16x8*)(row + 16 * s);
          acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], acc[mt][0], 0, 0, 0);
          acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], acc[mt][1], 0, 0, 0);
        }
      }
      bool pass = false;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        float mx = fmaxf(acc[0][nt][0], acc[1][nt][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, acc[0][nt][r]), acc[1][nt][r]);
        pass = pass || (mx * rsd >= th[nt]);
      }
      word |= (uint64_t)(__ballot(pass) != 0ull) << jj;
    }
    if (lane == 0) mrow[wc] = word;
    count += __popcll(word);
  }
  if (lane == 0) row_counts[(size_t)u.qh * g.n_qb + u.i] = count;
}

// Parity hook: the integer products themselves, one wave per key block, through the same
// re-encoding and the same MFMA as the Selection-Pass.
__global__ __launch_bounds__(64) void products_kernel(const uint8_t* __restrict__ q4_head, const uint8_t* __restrict__ k4_head,
                                                      int q_block, int k_begin, int n_kblocks, int32_t* __restrict__ out) {
  const int lane = threadIdx.x, c = lane & 31;
  const int jb = blockIdx.x;
  i32x8 qf[4], kf[4];
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    const int t = f >> 1, ks = f & 1;
    const size_t off = (size_t)(32 * t + c) * 64 + 32 * ks + 16 * (lane >> 5);
    uint32_t d[6];
    pack_fp6(*(const u32x4*)(q4_head + (size_t)q_block * 4096 + off), d);
#pragma unroll
    for (int e = 0; e < 6; ++e) qf[f][e] = d[e];
    qf[f][6] = 0; qf[f][7] = 0;
    pack_fp6(*(const u32x4*)(k4_head + (size_t)(k_begin + jb) * 4096 + off), d);
#pragma unroll
    for (int e = 0; e < 6; ++e) kf[f][e] = d[e];
    kf[f][6] = 0; kf[f][7] = 0;
  }
  f32x16 acc[2][2];
  qk_tile_fp6(kf, qf, acc);
  const size_t ld = (size_t)n_kblocks * 64;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 32 * mt + mfma32_row(r, lane), qr = 32 * nt + c;
        out[(size_t)qr * ld + jb * 64 + key] = (int32_t)acc[mt][nt][r];
      }
}

}  // namespace sale

using namespace sale;

extern "C" int sale_select(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4, const uint8_t* k4,
                           const float* q_scale, const float* k_scale, const float* tau, int32_t tau_len,
                           uint64_t* block_mask, int32_t* row_counts, float* m_out, float* l_out, void* ws,
                           size_t ws_bytes, void* stream) {
  if (!p || !q || !k || !tau || !block_mask || !row_counts) return SALE_ERR_NULL_ARG;
  const bool est16 = (p->flags & SALE_FLAG_SELECT_16BIT) != 0;
  if (!est16 && (!q4 || !k4 || !q_scale || !k_scale)) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, true);
  if (rc != SALE_OK) return rc;
  if (tau_len != 1 && tau_len != p->n_q_heads) return SALE_ERR_BAD_SHAPE;
  const size_t need = sale_workspace_bytes(p, SALE_WS_SELECT);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  const Geo g = make_geo(p);
  hipStream_t st = (hipStream_t)stream;
  const int tiles = (g.n_qb * g.group + 3) / 4;
  float* thr = (float*)ws;
  uint8_t* q6 = (uint8_t*)ws + (size_t)g.n_qh * g.seq * sizeof(float);
  uint8_t* k6 = q6 + (size_t)g.n_qh * g.n_qb * kX6BlockBytes;
  const long qblocks = (long)g.n_qh * g.n_qb, kblocks = (long)g.n_kvh * g.n_kb;
  if (!est16) {
    pack_fp6_kernel<<<dim3((unsigned)(qblocks + kblocks)), dim3(256), 0, st>>>(q4, q6, qblocks, k4, k6);
    if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  }
  stats_kernel<<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k, tau,
                                                                       tau_len, thr, m_out, l_out);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  if (est16) {
    select16_kernel<<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k, thr,
                                                                            block_mask, row_counts);
  } else if (g.group % 2 == 0) {
    const int t2 = (g.n_qb * (g.group / 2) + 3) / 4;
    select_kernel<2><<<dim3((unsigned)(t2 * g.n_kvh)), dim3(256), 0, st>>>(g, q6, k6, q_scale, k_scale, thr, block_mask,
                                                                          row_counts);
  } else {
    select_kernel<1><<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, q6, k6, q_scale, k_scale, thr, block_mask,
                                                                             row_counts);
  }
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

extern "C" int sale_qk_int4_products(const sale_params_t* p, const uint8_t* q4, const uint8_t* k4, int32_t q_head,
                                     int32_t q_block, int32_t k_block_begin, int32_t k_block_end, int32_t* out,
                                     void* stream) {
  if (!p || !q4 || !k4 || !out) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, true);
  if (rc != SALE_OK) return rc;
  const Geo g = make_geo(p);
  if (q_head < 0 || q_head >= g.n_qh || q_block < 0 || q_block >= g.n_qb) return SALE_ERR_BAD_SHAPE;
  if (k_block_begin < 0 || k_block_end > g.n_kb || k_block_begin > k_block_end) return SALE_ERR_BAD_SHAPE;
  const int nkb = k_block_end - k_block_begin;
  if (nkb == 0) return SALE_OK;
  products_kernel<<<dim3((unsigned)nkb), dim3(64), 0, (hipStream_t)stream>>>(
      q4 + (size_t)q_head * g.seq * 64, k4 + (size_t)(q_head / g.group) * g.seq * 64, q_block, k_block_begin, nkb, out);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}
