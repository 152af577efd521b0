// Computation-Pass (Sec. 3.1, Eq. 1 with the block mask of Eq. 2) and the dense
// causal kernel of the same design (every causally visible block kept).
//
// Design for gfx950
// -----------------
// * One workgroup = 4 waves = 4 units (query head, 64-row query block) that
//   share one KV head: with GQA group 4 these are the 4 query heads of the
//   group at the same query block, so every K/V tile staged in LDS feeds 256
//   query rows.  Workgroups are dealt round-robin over KV heads (blockIdx %
//   n_kv_heads: one KV head per XCD / L2 when there are 8) and longest rows
//   first.
// * The workgroup walks the UNION of its waves' mask rows; a wave whose own bit
//   is clear skips the tile's arithmetic (a skipped block costs that wave
//   nothing but the barrier).  The dense kernel is the same code with the
//   causal mask synthesised in place of a loaded one.
// * Each wave computes the TRANSPOSED score tile S^T = K Q^T (keys x queries)
//   with v_mfma_f32_32x32x16_bf16: a lane then owns 16 keys of one query
//   column, so row max / row sum / rescale factors are per-lane scalars and
//   the only cross-lane traffic of the online softmax is one exchange with
//   lane^32.  The accumulator layout of S^T is, register for register, the B
//   operand layout of the second product O^T = V^T P^T (up to a permutation
//   of the contraction index that is applied to V^T as well), so P never
//   leaves registers.  V^T operands come straight from the row-major V tile
//   with the LDS transpose read ds_read_b64_tr_b16.
// * Softmax in fp32 with exp2 and the scale folded in; O accumulates in fp32.
#include "sale_common.h"

namespace sale {

constexpr int KS = 136;   // LDS row stride of the K tile in elements (272 B: conflict-free 16-byte row reads)
constexpr int VS = 144;   // LDS row stride of the V tile in elements (288 B: conflict-free transpose reads)

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__global__ __launch_bounds__(256) void attn_kernel(Geo g, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                   const uint16_t* __restrict__ v, const uint64_t* __restrict__ mask,
                                                   uint16_t* __restrict__ o, float* __restrict__ lse) {
  __shared__ __attribute__((aligned(16))) uint16_t sK[64 * KS];
  __shared__ __attribute__((aligned(16))) uint16_t sV[64 * VS];
  __shared__ uint64_t sWords[4][kMaskWordsMax];
  __shared__ uint64_t sUnion[kMaskWordsMax];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 31, h = lane >> 5;
  const Unit u = unit_of(g, blockIdx.x, wave);

  // ---- mask rows of the four units and their union -------------------------------------
  for (int wc = lane; wc < g.words; wc += 64) {
    uint64_t word = 0;
    if (u.valid) {
      const int lo = wc * 64;
      const uint64_t causal = u.i >= lo + 63 ? ~0ull : (u.i < lo ? 0ull : ((2ull << (u.i - lo)) - 1ull));
      word = mask ? (mask[((size_t)u.qh * g.n_qb + u.i) * g.words + wc] & causal) : causal;
    }
    sWords[wave][wc] = word;
  }
  __syncthreads();
  for (int wc = tid; wc < g.words; wc += 256) sUnion[wc] = sWords[0][wc] | sWords[1][wc] | sWords[2][wc] | sWords[3][wc];
  __syncthreads();

  // ---- Q as the B operand of S^T = K Q^T ------------------------------------------------
  bf16x8 qf[2][8];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const uint16_t* row = q + ((size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c) * kHeadDim + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
  }

  f32x16 oacc[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][nt][r] = 0.0f;
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};
  const float cs = 0.08838834764831845f * 1.4426950408889634f;   // log2(e) / sqrt(d)

  // ---- iteration over the union of kept blocks ------------------------------------------
  int wc_it = 0;
  uint64_t cur = sUnion[0];
  auto next_block = [&]() -> int {
    while (cur == 0) {
      if (++wc_it >= g.words) return -1;
      cur = sUnion[wc_it];
    }
    const int b = __builtin_ctzll(cur);
    cur &= cur - 1;
    return wc_it * 64 + b;
  };

  const uint16_t* kh = k + (size_t)u.kvh * g.seq * kHeadDim;
  const uint16_t* vh = v + (size_t)u.kvh * g.seq * kHeadDim;
  uint4 kreg[4], vreg[4];
  auto load_tile = [&](int j) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int chunk = tid + 256 * t;
      const size_t off = ((size_t)j * 64 + (chunk >> 4)) * kHeadDim + (chunk & 15) * 8;
      kreg[t] = *(const uint4*)(kh + off);
      vreg[t] = *(const uint4*)(vh + off);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int chunk = tid + 256 * t;
      const int row = chunk >> 4, col = (chunk & 15) * 8;
      *(uint4*)&sK[row * KS + col] = kreg[t];
      *(uint4*)&sV[row * VS + col] = vreg[t];
    }
  };

  int j_cur = next_block();
  if (j_cur >= 0) load_tile(j_cur);
  while (j_cur >= 0) {
    store_tile();
    __syncthreads();
    const int j_next = next_block();
    if (j_next >= 0) load_tile(j_next);

    const bool active = (sWords[wave][j_cur >> 6] >> (j_cur & 63)) & 1ull;
    if (active) {
      // S^T tile: keys x queries
      f32x16 sacc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[mt][nt][r] = 0.0f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bf16x8 a = *(const bf16x8*)&sK[(32 * mt + c) * KS + 16 * s + 8 * h];
          sacc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], sacc[mt][0], 0, 0, 0);
          sacc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], sacc[mt][1], 0, 0, 0);
        }
      }
      const bool diag = j_cur == u.i;
      bf16x8 pf[2][4];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        if (diag) {
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (32 * mt + mfma32_row(r, lane) > 32 * nt + c) sacc[mt][nt][r] = -INFINITY;
        }
        float mx = sacc[0][nt][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[0][nt][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[1][nt][r]);
        mx = fmaxf(mx, swap_half(mx));
        const float m_new = fmaxf(m_run[nt], mx);          // finite: key 0 of a kept block is visible to every row
        const float alpha = __builtin_amdgcn_exp2f((m_run[nt] - m_new) * cs);
        const float mb = m_new * cs;
        float sum = 0.0f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(sacc[mt][nt][r] * cs - mb);
            sacc[mt][nt][r] = p;
            sum += p;
          }
        l_run[nt] = l_run[nt] * alpha + sum;
        m_run[nt] = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
        // P^T as the B operand of O^T = V^T P^T: k-step s takes registers 8*(s%2).. of tile s/2
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int e = 0; e < 8; ++e) pf[nt][s][e] = (__bf16)sacc[s >> 1][nt][8 * (s & 1) + e];
      }
      // O^T += V^T P^T.  k-step s, lane half h covers keys 16s + 4h + {0..3} and 16s + 8 + 4h + {0..3}.
      const int tr_row = (lane & 15) >> 2, tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const uint16_t* pa = &sV[(16 * s + 4 * h + tr_row) * VS + 32 * dt + tr_col];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)pa);
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(pa + 8 * VS));
          const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          oacc[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[0][s], oacc[dt][0], 0, 0, 0);
          oacc[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[1][s], oacc[dt][1], 0, 0, 0);
        }
      }
    }
    __syncthreads();
    j_cur = j_next;
  }

  // ---- epilogue ---------------------------------------------------------------------------
  if (!u.valid) return;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float l_tot = l_run[nt] + swap_half(l_run[nt]);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    const size_t row = (size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c;
    uint16_t* orow = o + row * kHeadDim + 4 * h;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[dt][nt][4 * q4 + e] * inv);
        *(bf16x4*)(orow + 32 * dt + 8 * q4) = w;
      }
    if (lse && h == 0) lse[row] = l_tot > 0.0f ? m_run[nt] * 0.08838834764831845f + __logf(l_tot) : -INFINITY;
  }
}

static int launch_attn(const sale_params_t* p, const void* q, const void* k, const void* v, const uint64_t* mask, void* o,
                       float* lse, hipStream_t st) {
  const Geo g = make_geo(p);
  const int tiles = (g.n_qb * g.group + 3) / 4;
  attn_kernel<<<dim3((unsigned)(tiles * g.n_kvh)), dim3(256), 0, st>>>(g, (const uint16_t*)q, (const uint16_t*)k,
                                                                      (const uint16_t*)v, mask, (uint16_t*)o, lse);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

}  // namespace sale

using namespace sale;

extern "C" int sale_sparse_attn(const sale_params_t* p, const void* q, const void* k, const void* v,
                                const uint64_t* block_mask, const int32_t* row_counts, void* o, float* lse, void* ws,
                                size_t ws_bytes, void* stream) {
  (void)row_counts;
  if (!p || !q || !k || !v || !block_mask || !o) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, true);
  if (rc != SALE_OK) return rc;
  const size_t need = sale_workspace_bytes(p, SALE_WS_SPARSE_ATTN);
  if (need > 0 && (!ws || ws_bytes < need)) return SALE_ERR_WORKSPACE;
  return launch_attn(p, q, k, v, block_mask, o, lse, (hipStream_t)stream);
}

extern "C" int sale_dense_attn(const sale_params_t* p, const void* q, const void* k, const void* v, void* o, float* lse,
                               void* stream) {
  if (!p || !q || !k || !v || !o) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, true);
  if (rc != SALE_OK) return rc;
  return launch_attn(p, q, k, v, nullptr, o, lse, (hipStream_t)stream);
}
