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
#include <mutex>

#include "sale_common.h"

namespace sale {

// Key blocks may be 64 or 32 tokens (MT = b_k / 32 MFMA row tiles per block); query blocks are 64 rows.
__device__ __forceinline__ int j_last_of(const Geo& g, int i) { return (i + 1) * (kBlockQ / g.bk) - 1; }

// Number of local key blocks of a row whose last visible key block is j_last.  With segments (Appendix C:
// the middle blocks are handled in groups of g.seg and the blocks left over at the end of the row are
// treated as local) the local area grows by that remainder.
__device__ __forceinline__ int local_of(const Geo& g, int j_last) {
  const int middle = j_last + 1 - g.sink_blocks - g.local_blocks;
  return g.local_blocks + (g.seg > 0 && middle > 0 ? middle % g.seg : 0);
}

__device__ __forceinline__ bool in_sink_local(const Geo& g, int j, int j_last, int local) {
  return j < g.sink_blocks || j > j_last - local;
}

// ---------------------------------------------------------------------------
// Sink-local statistics (display equation of Sec. 3.2; first loop of Alg. 1)
// ---------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(256) void stats_kernel(Geo g, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                    const float* __restrict__ tau, int tau_len, float* __restrict__ thr,
                                                    float* __restrict__ m_out, float* __restrict__ l_out) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform by construction
  const Unit u = unit_of(g, blockIdx.x, wave);
  if (!u.valid) return;
  const int c = lane & 31, h = lane >> 5;
  const float rsd = 0.08838834764831845f;   // 1 / sqrt(128)

  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + row_off(g.sq, u.qh, u.i * 64 + 32 * nt + c) + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }
  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.0f, 0.0f};
  const SeqPos sp = seq_pos(g, u.i);               // (variable-length batches: block indices inside the row's sequence)
  const int j_last = j_last_of(g, sp.il), local = local_of(g, j_last);
  // The sink-local blocks of the row, numbered t = 0 ..: the sink blocks that are not local ones, then the local
  // ones up to the diagonal.  They are swept in half-blocks of 32 keys (hs = t * MT + mt) with the operands of the
  // next half requested before the current one is multiplied: two register sets that swap roles, the last half
  // requesting itself again so that every step issues the same loads.
  const int lo_local = max(j_last - local + 1, 0);
  const int n_s = min(g.sink_blocks, lo_local);
  const int n_hs = (n_s + j_last - lo_local + 1) * MT;
  auto block_of = [&](int hs) { const int t = hs / MT; return t < n_s ? t : lo_local + (t - n_s); };
  auto fetch = [&](int hs, bf16x8 (&kk)[8]) __attribute__((always_inline)) {
    const uint16_t* row = k + row_off(g.sk, u.kvh, (sp.kb0 + block_of(hs)) * g.bk + 32 * (hs % MT) + c) + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) kk[s] = *(const bf16x8*)(row + 16 * s);
  };
  const float kLog2e = 1.4426950408889634f;
  auto half = [&](int hs, const bf16x8 (&kk)[8], bf16x8 (&kn)[8]) __attribute__((always_inline)) {
    fetch(min(hs + 1, n_hs - 1), kn);
    f32x16 acc[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kk[s], qf[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kk[s], qf[1][s], acc[1], 0, 0, 0);
    }
    const int j = block_of(hs), mt = hs % MT;
    // keys of this half that lie after a query row (only with SALE_FLAG_STATS_CAUSAL)
    const int ahead = j * g.bk + 32 * mt - sp.il * 64;      // first key of the half minus first query row
    if (g.stats_causal && ahead + 31 > 0) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (ahead + mfma32_row(r, lane) > 32 * nt + c) acc[nt][r] = -INFINITY;
    }
    // (VALU-bound: per score one half of a v_max3, one FMA that folds 1 / sqrt(d), log2(e) and the maximum,
    // one v_exp_f32 and one add)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float mx = fmaxf(acc[nt][0], acc[nt][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, acc[nt][r]), acc[nt][r + 1]);
      const float m_new = fmaxf(m[nt], mx * rsd);      // rsd > 0: the maximum of the products is the product of the maximum
      const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
      const float mb = m_safe * kLog2e;
      float sum = 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[nt][r], rsd * kLog2e, -mb));
      l[nt] = l[nt] * __builtin_amdgcn_exp2f(m[nt] * kLog2e - mb) + sum;
      m[nt] = m_new;
    }
  };
  {
    bf16x8 ka[8], kb[8];
    fetch(0, ka);                                   // (n_hs >= 1: the diagonal block is always local)
    for (int hs = 0; hs < n_hs; hs += 2) {
      half(hs, ka, kb);
      if (hs + 1 < n_hs) half(hs + 1, kb, ka);
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

// The same statistics for GQA groups of a multiple of 4 heads: the 4 waves of a workgroup are then 4 heads of one
// KV head at the SAME query block (unit_of), i.e. they need the same key rows.  The kernel above is bound by the
// bytes its waves pull through the vector memory path (each wave reads its 5 key blocks itself); here a half-block of
// K (32 keys, 8 KB) is fetched ONCE per workgroup, staged through registers into LDS in MFMA operand order (two
// buffers, one barrier per half-block, the next half's global loads in flight meanwhile) and read from there by all
// four waves: 2.7 times fewer bytes from L2 / L1.
template <int MT>
__global__ __launch_bounds__(256) void stats_shared_kernel(Geo g, const uint16_t* __restrict__ q,
                                                           const uint16_t* __restrict__ k, const float* __restrict__ tau,
                                                           int tau_len, float* __restrict__ thr, float* __restrict__ m_out,
                                                           float* __restrict__ l_out) {
  __shared__ bf16x8 k_lds[2][8 * 64];                // [buffer][s][lane] 16 bytes: the A operands of one half-block
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const Unit u = unit_of(g, blockIdx.x, wave);       // (group % 4 == 0: every wave is valid, all four share u.i and u.kvh)
  const int c = lane & 31, h = lane >> 5;
  const float rsd = 0.08838834764831845f;   // 1 / sqrt(128)

  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + row_off(g.sq, u.qh, u.i * 64 + 32 * nt + c) + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }
  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.0f, 0.0f};
  const SeqPos sp = seq_pos(g, u.i);
  const int j_last = j_last_of(g, sp.il), local = local_of(g, j_last);
  const int lo_local = max(j_last - local + 1, 0);
  const int n_s = min(g.sink_blocks, lo_local);
  const int n_hs = (n_s + j_last - lo_local + 1) * MT;
  auto block_of = [&](int hs) { const int t = hs / MT; return t < n_s ? t : lo_local + (t - n_s); };
  // Thread tid brings in chunks tid and tid + 256 of a half-block: chunk (s, lane') = the 16 bytes lane' of
  // fragment s needs (key row lane' % 32, channels 16 s + 8 (lane' / 32) ..).
  bf16x8 kreg[2];
  auto fetch = [&](int hs) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int id = tid + 256 * r, s = id >> 6, ln = id & 63;
      kreg[r] = *(const bf16x8*)(k + row_off(g.sk, u.kvh, (sp.kb0 + block_of(hs)) * g.bk + 32 * (hs % MT) + (ln & 31)) +
                                 16 * s + 8 * (ln >> 5));
    }
  };
  auto stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 2; ++r) k_lds[buf][tid + 256 * r] = kreg[r];
  };
  const float kLog2e = 1.4426950408889634f;
  fetch(0);
  stage(0);
  fetch(min(1, n_hs - 1));
  __syncthreads();
  for (int hs = 0; hs < n_hs; ++hs) {
    // the next half goes into the other buffer (every wave finished reading it before the last barrier), and
    // the one after next is requested
    stage((hs + 1) & 1);
    fetch(min(hs + 2, n_hs - 1));
    const bf16x8* kk = k_lds[hs & 1] + lane;
    f32x16 acc[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 a = kk[s * 64];
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], acc[1], 0, 0, 0);
    }
    const int j = block_of(hs), mt = hs % MT;
    const int ahead = j * g.bk + 32 * mt - sp.il * 64;      // first key of the half minus first query row
    if (g.stats_causal && ahead + 31 > 0) {                 // (only with SALE_FLAG_STATS_CAUSAL)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (ahead + mfma32_row(r, lane) > 32 * nt + c) acc[nt][r] = -INFINITY;
    }
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float mx = fmaxf(acc[nt][0], acc[nt][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, acc[nt][r]), acc[nt][r + 1]);
      const float m_new = fmaxf(m[nt], mx * rsd);
      const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
      const float mb = m_safe * kLog2e;
      float sum = 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[nt][r], rsd * kLog2e, -mb));
      l[nt] = l[nt] * __builtin_amdgcn_exp2f(m[nt] * kLog2e - mb) + sum;
      m[nt] = m_new;
    }
    __syncthreads();
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
// MFMA rate.  A pre-pass re-encodes the nibble codes of K~ once into MFMA operand
// order ("X6"; Q~ is re-encoded by the wave that uses it): per group of 32 rows 2 fragments ks (channels 64ks..); lane l of a
// fragment owns row l%32 of the group, channels 64ks + 32(l/32) + e, e = 0..31, as
// 32 six-bit codes = 6 dwords, stored as
//   [group][ks][lane] 16 bytes (dwords 0..3)  followed by  [group][ks][lane] 8 bytes (dwords 4..5).
constexpr int kX6GroupBytes = 2 * 64 * 24;   // 3072 bytes per 32 rows

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

// One thread per (32-row group, fragment, lane) of a nibble-packed [rows][64-byte] matrix; a workgroup
// handles two groups.  (Two matrices in one launch; the second may be empty.)
__global__ __launch_bounds__(256) void pack_fp6_kernel(const uint8_t* __restrict__ xa, uint8_t* __restrict__ ya,
                                                       long groups_a, const uint8_t* __restrict__ xb,
                                                       uint8_t* __restrict__ yb, long groups_b) {
  long grp = (long)blockIdx.x * 2 + (threadIdx.x >> 7);
  const uint8_t* x = xa;
  uint8_t* y = ya;
  if (grp >= groups_a) { grp -= groups_a; x = xb; y = yb; if (grp >= groups_b) return; }
  const int ks = (threadIdx.x >> 6) & 1, lane = threadIdx.x & 63;
  const u32x4 w = *(const u32x4*)(x + ((size_t)grp * 32 + (lane & 31)) * 64 + 32 * ks + 16 * (lane >> 5));
  uint32_t d[6];
  pack_fp6(w, d);
  uint8_t* yg = y + (size_t)grp * kX6GroupBytes;
  u32x4 lo;
  lo[0] = d[0]; lo[1] = d[1]; lo[2] = d[2]; lo[3] = d[3];
  u32x2 hi;
  hi[0] = d[4]; hi[1] = d[5];
  *(u32x4*)(yg + (ks * 64 + lane) * 16) = lo;
  *(u32x2*)(yg + 2048 + (ks * 64 + lane) * 8) = hi;
}

// The 2 operand fragments (ks = 0, 1) of 32-row group `grp` of an X6 array.
__device__ __forceinline__ void load_x6(const uint8_t* __restrict__ base, size_t grp, int lane, i32x8 f[2]) {
  const uint8_t* b = base + grp * kX6GroupBytes;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const u32x4 lo = *(const u32x4*)(b + (ks * 64 + lane) * 16);
    const u32x2 hi = *(const u32x2*)(b + 2048 + (ks * 64 + lane) * 8);
    f[ks][0] = lo[0]; f[ks][1] = lo[1]; f[ks][2] = lo[2]; f[ks][3] = lo[3];
    f[ks][4] = hi[0]; f[ks][5] = hi[1]; f[ks][6] = 0; f[ks][7] = 0;
  }
}

// acc[mt][nt] = (K~ row tile mt) (Q~ row tile nt)^T, keys x queries, exact integers held in fp32.
template <int MT>
__device__ __forceinline__ void qk_tile_fp6(const i32x8 kf[MT][2], const i32x8 qf[2][2], f32x16 acc[MT][2]) {
  // the two k-steps of a tile depend on each other: issue all tiles' first steps, then their second
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const f32x16 z = {0};
      acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[mt][0], qf[nt][0], z, 2, 2, 0, 0, 0, 0);
    }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
      acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[mt][1], qf[nt][1], acc[mt][nt], 2, 2, 0, 0, 0, 0);
}

// Maximum over the keys of a block of what one lane holds for query tile nt.
template <int MT>
__device__ __forceinline__ float lane_max(const f32x16 acc[MT][2], int nt) {
  float mx = acc[0][nt][0];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = (mt == 0 ? 1 : 0); r < 16; ++r) mx = fmaxf(mx, acc[mt][nt][r]);
  return mx;
}

// One wave scores HPW query heads of one GQA group at the same query block, so every K~ fragment it
// loads feeds HPW x 2 MFMAs (HPW = 4 when the group allows).  A workgroup is 4 such waves (consecutive head sets / query blocks of one
// KV head); workgroups go round-robin over KV heads, longest rows first.
// (At least 2 waves per SIMD caps the register file at 256 VGPRs, which lets the MFMA results land in
// ordinary VGPRs instead of AGPRs that the max chain would have to copy out one by one.)
template <int HPW, int MT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void select_kernel(
    Geo g, const uint8_t* __restrict__ q4, const uint8_t* __restrict__ k6, const float* __restrict__ q_scale,
    const float* __restrict__ k_scale, const float* __restrict__ thr, uint64_t* __restrict__ mask,
    int32_t* __restrict__ row_counts) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform by construction
  const int c = lane & 31;
  const int sets = g.group / HPW;                 // head sets per (KV head, query block)
  const int units = g.n_qb * sets;
  const int tiles = (units + 3) / 4;
  const int kvh = blockIdx.x % g.n_kvh;
  const int id = (tiles - 1 - blockIdx.x / g.n_kvh) * 4 + wave;
  if (id >= units) return;
  const int i = id / sets;
  const int qh0 = kvh * g.group + (id % sets) * HPW;

  i32x8 qf[HPW][2][2];
  float th[HPW][2], cq[HPW];
#pragma unroll
  for (int a = 0; a < HPW; ++a) {
    // Q~ is used by this wave alone: its nibble codes are re-encoded here, once per row (K~, which every query
    // block reads again, comes re-encoded from the pre-pass).  Lane (c, h) of fragment (row tile nt, ks) owns row
    // 32 nt + c, channels 64 ks + 32 h ..: 16 bytes of the row.
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const uint8_t* row = q4 + ((size_t)(qh0 + a) * g.seq + i * 64 + 32 * nt + c) * 64 + 16 * (lane >> 5);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        uint32_t d[6];
        pack_fp6(*(const u32x4*)(row + 32 * ks), d);
#pragma unroll
        for (int e = 0; e < 6; ++e) qf[a][nt][ks][e] = d[e];
        qf[a][nt][ks][6] = 0; qf[a][nt][ks][7] = 0;
      }
    }
    th[a][0] = thr[(size_t)(qh0 + a) * g.seq + i * 64 + c];
    th[a][1] = thr[(size_t)(qh0 + a) * g.seq + i * 64 + 32 + c];
    cq[a] = q_scale[(size_t)(qh0 + a) * g.n_qb + i] * 0.08838834764831845f;   // s_q / sqrt(d)
  }
  const float* ks = k_scale + (size_t)kvh * g.n_kb;
  const size_t kgrp0 = (size_t)kvh * g.n_kb * MT;

  const SeqPos sp = seq_pos(g, i);
  const int j_last = j_last_of(g, sp.il), local = local_of(g, j_last);
  const int mid_lo = g.sink_blocks, mid_hi = j_last - local;      // the middle blocks (inclusive), scored below
  int count[HPW];
  uint64_t word[HPW];
  int wc = 0;                                                       // mask word being assembled
  // Bits of word wc that are set without scoring: the sink and local blocks the row can see.
  auto fixed_bits = [&]() -> uint64_t {
    auto span = [&](int lo, int hi) -> uint64_t {                   // bits of blocks lo..hi that fall into word wc
      lo = max(lo - wc * 64, 0); hi = min(hi - wc * 64, 63);
      return lo > hi ? 0ull : ((~0ull >> (63 - hi)) & (~0ull << lo));
    };
    return span(0, min(g.sink_blocks - 1, j_last)) | span(max(mid_hi + 1, 0), j_last);
  };
  // Completes word wc (store, count) and starts the next one.
  auto flush = [&]() {
#pragma unroll
    for (int a = 0; a < HPW; ++a) {
      if (lane == 0) mask[((size_t)(qh0 + a) * g.n_qb + i) * g.words + wc] = word[a];
      count[a] += __popcll(word[a]);
    }
    ++wc;
    const uint64_t fb = fixed_bits();
#pragma unroll
    for (int a = 0; a < HPW; ++a) word[a] = fb;
  };
  {
    const uint64_t fb = fixed_bits();
#pragma unroll
    for (int a = 0; a < HPW; ++a) { count[a] = 0; word[a] = fb; }
  }
  // The operands of a key block are requested one block ahead (two register sets that swap roles): the loads of
  // block j + 1 are in flight while block j is scored.  The last block requests itself again, so every step
  // issues the same loads and the wait counts stay exact.
  i32x8 kfa[MT][2], kfb[MT][2];
  float ska = 0.0f, skb = 0.0f;
  auto fetch = [&](int j, i32x8 (&kf)[MT][2], float& sk) __attribute__((always_inline)) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) load_x6(k6, kgrp0 + (size_t)(sp.kb0 + j) * MT + mt, lane, kf[mt]);
    sk = ks[sp.kb0 + j];
  };
  auto score = [&](int j, const i32x8 (&kf)[MT][2], float sk, i32x8 (&kn)[MT][2], float& skn) __attribute__((always_inline)) {
    fetch(min(j + 1, mid_hi), kn, skn);
    while (wc < (j >> 6)) flush();
#pragma unroll
    for (int a = 0; a < HPW; ++a) {
      f32x16 acc[MT][2];
      qk_tile_fp6<MT>(kf, qf[a], acc);
      const float cj = cq[a] * sk;
      // (both halves always: a short-circuit would put the second maximum chain behind a branch, where it
      // cannot be interleaved with the next head's MFMAs; most blocks fail the first test anyway)
      const bool p0 = lane_max<MT>(acc, 0) * cj >= th[a][0];
      const bool p1 = lane_max<MT>(acc, 1) * cj >= th[a][1];
      word[a] |= (uint64_t)(__ballot(p0 | p1) != 0ull) << (j & 63);
    }
  };
  if (mid_lo <= mid_hi) {
    fetch(mid_lo, kfa, ska);
    for (int j = mid_lo; j <= mid_hi; j += 2) {
      score(j, kfa, ska, kfb, skb);
      if (j + 1 <= mid_hi) score(j + 1, kfb, skb, kfa, ska);
    }
  }
  while (wc < g.words) flush();
#pragma unroll
  for (int a = 0; a < HPW; ++a)
    if (lane == 0) row_counts[(size_t)(qh0 + a) * g.n_qb + i] = count[a];
}

// Appendix E ablation ("w/o QK Quant"): the same rule with the estimate taken from the 16-bit Q, K
// themselves (S~ = S, bf16 MFMA with fp32 accumulation): four times the MFMA work of the FP6 estimate.
template <int MT>
__global__ __launch_bounds__(256) void select16_kernel(Geo g, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                       const float* __restrict__ thr, uint64_t* __restrict__ mask,
                                                       int32_t* __restrict__ row_counts) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform by construction
  const Unit u = unit_of(g, blockIdx.x, wave);
  if (!u.valid) return;
  const int c = lane & 31, h = lane >> 5;
  const float rsd = 0.08838834764831845f;   // 1 / sqrt(128)
  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + row_off(g.sq, u.qh, u.i * 64 + 32 * nt + c) + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }
  float th[2];
  th[0] = thr[(size_t)u.qh * g.seq + u.i * 64 + c];
  th[1] = thr[(size_t)u.qh * g.seq + u.i * 64 + 32 + c];
  uint64_t* mrow = mask + ((size_t)u.qh * g.n_qb + u.i) * g.words;
  const SeqPos sp = seq_pos(g, u.i);
  const int j_last = j_last_of(g, sp.il), local = local_of(g, j_last);
  int count = 0;
  for (int wc = 0; wc < g.words; ++wc) {
    uint64_t word = 0;
    const int j_end = min(64, j_last + 1 - wc * 64);
    for (int jj = 0; jj < j_end; ++jj) {
      const int j = wc * 64 + jj;
      if (in_sink_local(g, j, j_last, local)) { word |= 1ull << jj; continue; }
      f32x16 acc[MT][2];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const uint16_t* row = k + row_off(g.sk, u.kvh, (sp.kb0 + j) * g.bk + 32 * mt + c) + 8 * h;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bf16x8 a = *(const bf16x8*)(row + 16 * s);
          acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], acc[mt][0], 0, 0, 0);
          acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], acc[mt][1], 0, 0, 0);
        }
      }
      const bool pass = (lane_max<MT>(acc, 0) * rsd >= th[0]) || (lane_max<MT>(acc, 1) * rsd >= th[1]);
      word |= (uint64_t)(__ballot(pass) != 0ull) << jj;
    }
    if (lane == 0) mrow[wc] = word;
    count += __popcll(word);
  }
  if (lane == 0) row_counts[(size_t)u.qh * g.n_qb + u.i] = count;
}

// Parity hook: the integer products themselves, one wave per key block, through the same
// re-encoding and the same MFMA as the Selection-Pass.
template <int MT>
__global__ __launch_bounds__(64) void products_kernel(const uint8_t* __restrict__ q4_head, const uint8_t* __restrict__ k4_head,
                                                      int q_block, int k_begin, int n_kblocks, int32_t* __restrict__ out) {
  const int lane = threadIdx.x, c = lane & 31;
  const int jb = blockIdx.x;
  auto frag = [&](const uint8_t* rows32, int ks, i32x8& f) __attribute__((always_inline)) {
    uint32_t d[6];
    pack_fp6(*(const u32x4*)(rows32 + (size_t)c * 64 + 32 * ks + 16 * (lane >> 5)), d);
#pragma unroll
    for (int e = 0; e < 6; ++e) f[e] = d[e];
    f[6] = 0; f[7] = 0;
  };
  i32x8 qf[2][2], kf[MT][2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) frag(q4_head + ((size_t)q_block * 2 + nt) * 2048, ks, qf[nt][ks]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) frag(k4_head + ((size_t)(k_begin + jb) * MT + mt) * 2048, ks, kf[mt][ks]);
  }
  f32x16 acc[MT][2];
  qk_tile_fp6<MT>(kf, qf, acc);
  const size_t ld = (size_t)n_kblocks * (32 * MT);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 32 * mt + mfma32_row(r, lane), qr = 32 * nt + c;
        out[(size_t)qr * ld + jb * (32 * MT) + key] = (int32_t)acc[mt][nt][r];
      }
}

}  // namespace sale

using namespace sale;

namespace {

template <int MT>
int launch_select(const Geo& g, bool est16, const void* q, const void* k, const uint8_t* q4, const uint8_t* k6,
                  const float* q_scale, const float* k_scale, const float* tau, int tau_len, const float* thr_c,
                  float* thr, uint64_t* block_mask, int32_t* row_counts, float* m_out, float* l_out, hipStream_t st) {
  const int tiles = (g.n_qb * g.group + 3) / 4;
  if (g.group % 4 == 0)      // (then every workgroup holds 4 heads of one KV head at one query block: they share K)
    stats_shared_kernel<MT><<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k,
                                                                                    tau, tau_len, thr, m_out, l_out);
  else
    stats_kernel<MT><<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k, tau,
                                                                             tau_len, thr, m_out, l_out);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  if (est16) {
    select16_kernel<MT><<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k,
                                                                                thr_c, block_mask, row_counts);
  } else if (MT == 2 && g.group % 4 == 0) {     // (with 32-key blocks two heads per wave are faster: 15.8 against 17.1 ms at 128K)
    const int t4 = (g.n_qb * (g.group / 4) + 3) / 4;
    select_kernel<4, MT><<<dim3((unsigned)(t4 * g.n_kvh)), dim3(256), 0, st>>>(g, q4, k6, q_scale, k_scale, thr_c,
                                                                              block_mask, row_counts);
  } else if (g.group % 2 == 0) {
    const int t2 = (g.n_qb * (g.group / 2) + 3) / 4;
    select_kernel<2, MT><<<dim3((unsigned)(t2 * g.n_kvh)), dim3(256), 0, st>>>(g, q4, k6, q_scale, k_scale, thr_c,
                                                                              block_mask, row_counts);
  } else {
    select_kernel<1, MT><<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, q4, k6, q_scale, k_scale, thr_c,
                                                                                 block_mask, row_counts);
  }
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

}  // namespace

namespace {

// Checks shared by the two Selection-Pass entry points (everything but the workspace).
int check_select_args(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4, const uint8_t* k4,
                      const float* q_scale, const float* k_scale, const float* tau, int32_t tau_len,
                      const uint64_t* block_mask, const int32_t* row_counts) {
  if (!p || !q || !k || !tau || !block_mask || !row_counts) return SALE_ERR_NULL_ARG;
  const bool est16 = (p->flags & SALE_FLAG_SELECT_16BIT) != 0;
  if (!est16 && (!q4 || !k4 || !q_scale || !k_scale)) return SALE_ERR_NULL_ARG;
  const int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  if (tau_len != 1 && tau_len != p->n_q_heads) return SALE_ERR_BAD_SHAPE;
  return SALE_OK;
}

// The Selection-Pass on a workspace that has been checked.  Every byte of the workspace that a kernel reads is
// written earlier in the same call (thresholds by the statistics kernel, operand copies by the packing kernel),
// so nothing in it has to be cleared.
int run_select(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4, const uint8_t* k4,
               const float* q_scale, const float* k_scale, const float* tau, int32_t tau_len, uint64_t* block_mask,
               int32_t* row_counts, float* m_out, float* l_out, void* ws, hipStream_t st) {
  const bool est16 = (p->flags & SALE_FLAG_SELECT_16BIT) != 0;
  Geo g = make_geo(p);
  float* thr = (float*)ws;
  uint8_t* k6 = (uint8_t*)ws + (size_t)g.n_qh * g.seq * sizeof(float);
  if (p->n_seqs > 0) {      // the per-block sequence table follows the operand copy
    int32_t* table = (int32_t*)(k6 + (size_t)g.n_kvh * (g.seq / 32) * kX6GroupBytes);
    const int rc = build_seq_table(p, table, st);
    if (rc != SALE_OK) return rc;
    g.seq_start = table;
  }
  const long kgroups = (long)g.n_kvh * (g.seq / 32);
  if (!est16) {
    pack_fp6_kernel<<<dim3((unsigned)((kgroups + 1) / 2)), dim3(256), 0, st>>>(k4, k6, kgroups, nullptr, nullptr, 0);
    if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  }
  return g.bk == 64 ? launch_select<2>(g, est16, q, k, q4, k6, q_scale, k_scale, tau, tau_len, thr, thr, block_mask,
                                       row_counts, m_out, l_out, st)
                    : launch_select<1>(g, est16, q, k, q4, k6, q_scale, k_scale, tau, tau_len, thr, thr, block_mask,
                                       row_counts, m_out, l_out, st);
}

}  // namespace

extern "C" int sale_select(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4, const uint8_t* k4,
                           const float* q_scale, const float* k_scale, const float* tau, int32_t tau_len,
                           uint64_t* block_mask, int32_t* row_counts, float* m_out, float* l_out, void* ws,
                           size_t ws_bytes, void* stream) {
  const int rc = check_select_args(p, q, k, q4, k4, q_scale, k_scale, tau, tau_len, block_mask, row_counts);
  if (rc != SALE_OK) return rc;
  const size_t need = sale_workspace_bytes(p, SALE_WS_SELECT);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  return run_select(p, q, k, q4, k4, q_scale, k_scale, tau, tau_len, block_mask, row_counts, m_out, l_out, ws,
                    (hipStream_t)stream);
}

// ---------------------------------------------------------------------------
// Selection-Pass for callers that cannot allocate: the workspace is a static device array of the library.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SALE_SELECT_STATIC_MAX_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];      // per device: the address of that GPU's copy of `scratch`

// Device address of the current device's copy of `scratch` (in host code the array's name is only a handle:
// the address has to be asked for, once per device, with that device current).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SALE_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SALE_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SALE_OK;
}

}  // namespace

extern "C" int sale_select_static(const sale_params_t* p, const void* q, const void* k, const uint8_t* q4,
                                  const uint8_t* k4, const float* q_scale, const float* k_scale, const float* tau,
                                  int32_t tau_len, uint64_t* block_mask, int32_t* row_counts, float* m_out,
                                  float* l_out, void* stream) {
  int rc = check_select_args(p, q, k, q4, k4, q_scale, k_scale, tau, tau_len, block_mask, row_counts);
  if (rc != SALE_OK) return rc;
  if (sale_workspace_bytes(p, SALE_WS_SELECT) > (size_t)SALE_SELECT_STATIC_MAX_BYTES) return SALE_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != SALE_OK) return rc;
  return run_select(p, q, k, q4, k4, q_scale, k_scale, tau, tau_len, block_mask, row_counts, m_out, l_out, ws,
                    (hipStream_t)stream);
}

extern "C" int sale_qk_int4_products(const sale_params_t* p, const uint8_t* q4, const uint8_t* k4, int32_t q_head,
                                     int32_t q_block, int32_t k_block_begin, int32_t k_block_end, int32_t* out,
                                     void* stream) {
  if (!p || !q4 || !k4 || !out) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  const Geo g = make_geo(p);
  if (q_head < 0 || q_head >= g.n_qh || q_block < 0 || q_block >= g.n_qb) return SALE_ERR_BAD_SHAPE;
  if (k_block_begin < 0 || k_block_end > g.n_kb || k_block_begin > k_block_end) return SALE_ERR_BAD_SHAPE;
  const int nkb = k_block_end - k_block_begin;
  if (nkb == 0) return SALE_OK;
  const uint8_t* qh = q4 + (size_t)q_head * g.seq * 64;
  const uint8_t* kh = k4 + (size_t)(q_head / g.group) * g.seq * 64;
  if (g.bk == 64)
    products_kernel<2><<<dim3((unsigned)nkb), dim3(64), 0, (hipStream_t)stream>>>(qh, kh, q_block, k_block_begin, nkb, out);
  else
    products_kernel<1><<<dim3((unsigned)nkb), dim3(64), 0, (hipStream_t)stream>>>(qh, kh, q_block, k_block_begin, nkb, out);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}
