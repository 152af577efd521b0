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
// CDNA4 has no int4 MFMA.  The 4-bit codes are expanded on the fly to int8
// holding 16*code (one AND / one shift+AND per four codes: the nibble simply
// becomes the byte's high half), multiplied on the int8 MFMA with int32
// accumulation, and the exact integer product is acc / 256.
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
// 4-bit estimate on the int8 MFMA
// ---------------------------------------------------------------------------
// A lane's 16 packed bytes (32 codes) become the operands of two k-steps of
// 16 int8 each.  Which channel lands in which k slot does not matter as long
// as Q~ and K~ use the same expansion: the contraction sums over all of them.
__device__ __forceinline__ void expand16(const u32x4 w, i32x4& s0, i32x4& s1) {
  s0[0] = (int)((w[0] << 4) & 0xF0F0F0F0u); s0[1] = (int)(w[0] & 0xF0F0F0F0u);
  s0[2] = (int)((w[1] << 4) & 0xF0F0F0F0u); s0[3] = (int)(w[1] & 0xF0F0F0F0u);
  s1[0] = (int)((w[2] << 4) & 0xF0F0F0F0u); s1[1] = (int)(w[2] & 0xF0F0F0F0u);
  s1[2] = (int)((w[3] << 4) & 0xF0F0F0F0u); s1[3] = (int)(w[3] & 0xF0F0F0F0u);
}

// Rows row0 + 32*t + lane%32 (t = 0, 1) of a packed [rows][64-byte] matrix.
__device__ __forceinline__ void load_frags(const uint8_t* __restrict__ base, size_t row0, int lane, i32x4 f[2][4]) {
  const int c = lane & 31, h = lane >> 5;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint8_t* row = base + (row0 + 32 * t + c) * 64 + 16 * h;
#pragma unroll
    for (int c16 = 0; c16 < 2; ++c16) {
      const u32x4 w = *(const u32x4*)(row + 32 * c16);
      expand16(w, f[t][2 * c16], f[t][2 * c16 + 1]);
    }
  }
}

// acc[mt][nt] = 256 * (K~ tile mt) (Q~ tile nt)^T, keys x queries.
__device__ __forceinline__ void qk_tile(const i32x4 kf[2][4], const i32x4 qf[2][4], i32x16 acc[2][2]) {
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      i32x16 a = {0};
#pragma unroll
      for (int s = 0; s < 4; ++s) a = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[mt][s], qf[nt][s], a, 0, 0, 0);
      acc[mt][nt] = a;
    }
}

__global__ __launch_bounds__(256) void select_kernel(Geo g, const uint8_t* __restrict__ q4, const uint8_t* __restrict__ k4,
                                                     const float* __restrict__ q_scale, const float* __restrict__ k_scale,
                                                     const float* __restrict__ thr, uint64_t* __restrict__ mask,
                                                     int32_t* __restrict__ row_counts) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const Unit u = unit_of(g, blockIdx.x, wave);
  if (!u.valid) return;
  const int c = lane & 31;

  i32x4 qf[2][4];
  load_frags(q4 + (size_t)u.qh * g.seq * 64, (size_t)u.i * 64, lane, qf);
  float th[2];
  th[0] = thr[(size_t)u.qh * g.seq + u.i * 64 + c];
  th[1] = thr[(size_t)u.qh * g.seq + u.i * 64 + 32 + c];
  // dequantization factor of the block pair, without the key scale: s_q / sqrt(d) / 256
  const float cq = q_scale[(size_t)u.qh * g.n_qb + u.i] * (0.08838834764831845f / 256.0f);
  const float* ks = k_scale + (size_t)u.kvh * g.n_kb;
  const uint8_t* kbase = k4 + (size_t)u.kvh * g.seq * 64;
  uint64_t* mrow = mask + ((size_t)u.qh * g.n_qb + u.i) * g.words;

  const int j_last = u.i;
  int count = 0;
  for (int wc = 0; wc < g.words; ++wc) {
    uint64_t word = 0;
    const int j_end = min(64, j_last + 1 - wc * 64);
    for (int jj = 0; jj < j_end; ++jj) {
      const int j = wc * 64 + jj;
      bool keep;
      if (in_sink_local(g, j, j_last)) {
        keep = true;
      } else {
        i32x4 kf[2][4];
        load_frags(kbase, (size_t)j * 64, lane, kf);
        i32x16 acc[2][2];
        qk_tile(kf, qf, acc);
        const float cj = cq * ks[j];
        bool pass = false;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          int mx = acc[0][nt][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = max(mx, acc[0][nt][r]);
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = max(mx, acc[1][nt][r]);
          pass = pass || ((float)mx * cj >= th[nt]);
        }
        keep = __ballot(pass) != 0ull;
      }
      word |= (uint64_t)keep << jj;
    }
    if (lane == 0) mrow[wc] = word;
    count += __popcll(word);
  }
  if (lane == 0) row_counts[(size_t)u.qh * g.n_qb + u.i] = count;
}

// Parity hook: the integer products themselves, one wave per key block.
__global__ __launch_bounds__(64) void products_kernel(const uint8_t* __restrict__ q4_head, const uint8_t* __restrict__ k4_head,
                                                      int q_block, int k_begin, int n_kblocks, int32_t* __restrict__ out) {
  const int lane = threadIdx.x, c = lane & 31;
  const int jb = blockIdx.x;
  i32x4 qf[2][4], kf[2][4];
  load_frags(q4_head, (size_t)q_block * 64, lane, qf);
  load_frags(k4_head, (size_t)(k_begin + jb) * 64, lane, kf);
  i32x16 acc[2][2];
  qk_tile(kf, qf, acc);
  const size_t ld = (size_t)n_kblocks * 64;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 32 * mt + mfma32_row(r, lane), qr = 32 * nt + c;
        out[(size_t)qr * ld + jb * 64 + key] = acc[mt][nt][r] >> 8;
      }
}

}  // namespace sale

using namespace sale;

extern "C" int sale_select(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4, const uint8_t* k4,
                           const float* q_scale, const float* k_scale, const float* tau, int32_t tau_len,
                           uint64_t* block_mask, int32_t* row_counts, float* m_out, float* l_out, void* ws,
                           size_t ws_bytes, void* stream) {
  if (!p || !q || !k || !q4 || !k4 || !q_scale || !k_scale || !tau || !block_mask || !row_counts) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, true);
  if (rc != SALE_OK) return rc;
  if (tau_len != 1 && tau_len != p->n_q_heads) return SALE_ERR_BAD_SHAPE;
  const size_t need = sale_workspace_bytes(p, SALE_WS_SELECT);
  if (!ws || ws_bytes < need) return SALE_ERR_WORKSPACE;
  const Geo g = make_geo(p);
  hipStream_t st = (hipStream_t)stream;
  const int tiles = (g.n_qb * g.group + 3) / 4;
  const dim3 grid((unsigned)(tiles * g.n_kvh));
  float* thr = (float*)ws;
  stats_kernel<<<grid, dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k, tau, tau_len, thr, m_out, l_out);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  select_kernel<<<grid, dim3(256), 0, st>>>(g, q4, k4, q_scale, k_scale, thr, block_mask, row_counts);
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
