// Computation-Pass (Sec. 3.1, Eq. 1 with the block mask of Eq. 2) and the dense
// causal kernel of the same design (every causally visible block kept).
//
// Design for gfx950
// -----------------
// * One wave = one unit (query head, 64-row query block) walking its OWN mask
//   row.  The masks of the query heads that share a KV head differ block by
//   block, so staging a tile once for several heads only pays when their bits
//   coincide; instead each wave streams the operands of exactly the blocks its
//   row keeps straight from global memory into MFMA operand registers: no LDS
//   staging, no barriers, a skipped block costs nothing.
// * To make those loads full 1 KB coalesced transactions (and to get V
//   transposed for free) a pre-pass copies K and V once into "fragment order"
//   (layouts at rearrange_kv_kernel).
// * Each wave computes the TRANSPOSED score tile S^T = K Q^T (keys x queries)
//   with v_mfma_f32_32x32x16_bf16: a lane then owns 16 keys of one query
//   column, so row max / row sum / rescale factors are per-lane scalars and
//   the only cross-lane traffic of the online softmax is one exchange with
//   lane^32.  The accumulator layout of S^T is, register for register, the B
//   operand layout of the second product O^T = V^T P^T (up to a permutation
//   of the contraction index that the V copy applies as well), so P never
//   leaves registers.
// * Softmax in fp32 with exp2 and the scale folded in; the O rescale is skipped
//   (exactly) whenever no row maximum grew; O accumulates in fp32.  The finished
//   bf16 tile is transposed through LDS (each wave its own 17 KB, no barrier) so
//   that it leaves as whole 256-byte rows.
// * Scheduling.  Dense: a workgroup is the 4 units of one GQA group at the same
//   query block (they read the same blocks in step, so three of four loads hit
//   L1), longest rows first, workgroups round-robin over KV heads (blockIdx %
//   n_kv_heads: one KV head per XCD / L2 when there are 8).
//   Sparse: row lengths are heavy-tailed (a query block with one weak row keeps
//   everything) and differ between heads, so every unit is its own 64-thread
//   workgroup.  Short sequences: one sweep per row, rows issued by decreasing
//   kept-block count (a counting sort of row_counts).  Longer ones: the long
//   rows are swept window by window (a window of K', V' fits an XCD's L2) with
//   their accumulators parked in the workspace in between, every window launch
//   is balanced over the XCDs by a table that moves rows of over-loaded heads to
//   the lanes of under-loaded ones, and the short rows ride at the tail of the
//   window launches (details at launch_sparse_rows and balance_kernel).
#include <type_traits>

#include "sale_common.h"

namespace sale {

// ---------------------------------------------------------------------------
// Computation-Pass proper: every wave walks its OWN mask row.
//
// The masks of the query heads that share a KV head differ block by block, so
// staging a tile once for several heads only pays when their bits coincide.
// Here each wave streams the operands of exactly the blocks its row keeps,
// straight from global memory into MFMA operand registers: no LDS, no
// barriers, a skipped block costs nothing.  To make those loads full 1 KB
// coalesced transactions (and to get V transposed for free) a pre-pass copies
// K and V once into "fragment order":
//   K' [kv head][block j][mt 0..1][s 0..7][lane 0..63] : 8 channels 16s + 8(lane/32).. of key row 32mt + lane%32
//   V' [kv head][block j][dt 0..3][s 0..3][lane 0..63] : channel 32dt + lane%32 of the 8 keys
//                                                        16s + 8(e/4) + 4(lane/32) + e%4,  e = 0..7
// (the key order inside V' is the order in which the S^T accumulator registers
// hand P^T to the second product).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rearrange_kv_kernel(int seq, const uint16_t* __restrict__ k, Strided lk,
                                                           const uint16_t* __restrict__ v, Strided lv,
                                                           u32x4* __restrict__ kp, u32x4* __restrict__ vp,
                                                           int* __restrict__ slot_counter) {
  __shared__ uint16_t sv[64 * (kHeadDim + 2)];
  const int tid = threadIdx.x;
  if (slot_counter && blockIdx.x == 0 && tid == 0) *slot_counter = 0;      // (for order_units_kernel, next on the stream)
  const size_t tile = blockIdx.x;                      // flattened (kv head, block j): rows tile*64 .. +63
  const int tiles_per_head = seq / 64;
  const uint16_t* kt = k + row_off(lk, (int)(tile / tiles_per_head), (int)(tile % tiles_per_head) * 64);
  const uint16_t* vt = v + row_off(lv, (int)(tile / tiles_per_head), (int)(tile % tiles_per_head) * 64);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int chunk = tid + 256 * r;                   // V tile -> LDS, rows padded by one bank
    const int row = chunk >> 4, col = (chunk & 15) * 8;
    const u32x4 w = *(const u32x4*)(vt + (size_t)row * lv.st + col);
    uint32_t* d = (uint32_t*)&sv[row * (kHeadDim + 2) + col];
    d[0] = w[0]; d[1] = w[1]; d[2] = w[2]; d[3] = w[3];
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int oc = tid + 256 * r;
    const int lane = oc & 63, s = (oc >> 6) & 7, mt = oc >> 9;
    kp[tile * 1024 + oc] = *(const u32x4*)(kt + (size_t)(32 * mt + (lane & 31)) * lk.st + 16 * s + 8 * (lane >> 5));
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int oc = tid + 256 * r;
    const int lane = oc & 63, s = (oc >> 6) & 3, dt = oc >> 8;
    const int d = 32 * dt + (lane & 31), h = lane >> 5;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int e = 2 * e2;
      const int key = 16 * s + 8 * (e >> 2) + 4 * h + (e & 3);
      w[e2] = (uint32_t)sv[key * (kHeadDim + 2) + d] | ((uint32_t)sv[(key + 1) * (kHeadDim + 2) + d] << 16);
    }
    u32x4 out;
    out[0] = w[0]; out[1] = w[1]; out[2] = w[2]; out[3] = w[3];
    vp[tile * 1024 + oc] = out;
  }
}

// Which rows a launch handles and which part of them.  win_word < 0: the whole row in one go.
// win_word >= 0: only the key blocks of that 64-block mask word; a row then resumes from the state
// (fp32 O^T accumulators, running max and sum, exactly the register contents) that the launch of the
// previous word parked in its slot of the workspace, and parks it again unless this word holds its diagonal block.
// slot_of (window launches): the parking slot of every row block, or -1 for the rows that are swept whole: the
// short ones, and the long ones that found no slot in the caller's workspace.
// Workgroups from number tail_from on (tail_from >= 0) form the tail of a window launch: they take the
// rows without a slot, whole, rank tail_phase + k * tail_stride of each KV head's
// sorted list, so that every window launch ends with its share of short rows and its last long rows do
// not leave the chip idle.
struct RowFilter {
  const int32_t* slot_of;
  int win_word;    // first mask word of the window, or < 0
  int win_words;   // words per window
  int tail_from, tail_stride, tail_phase;
};

// order: optional [kv head][rank] -> unit id within the KV head (block * group + head-in-group).
// BK32: the mask has one bit per 32 keys (b_k = 32) instead of one per 64.  The kernel always works on
// pairs of 32-key half-tiles; with b_k = 64 a pair is the two halves of one block, with b_k = 32 it is any
// two kept half-tiles of the row (the operand copies K', V' are addressable by half-tile).
// QK8: the first product runs on the 8-bit operands of the quantized Computation-Pass (Sec. 3.4 "Integration
// with SageAttention") with v_mfma_i32_32x32x32_i8: half the K bytes and half the MFMA time of that product.
struct Qk8 {
  const int8_t* q8;       // [q head][N][128]
  const u32x4* k8p;       // fragment order, 8 KB per 64 keys
  const float* q_scale;   // [q head][N / 64]
  const float* k_scale;   // [kv head][N / 64]
  const float* k_mean;    // [kv head][128]: the mean key taken out of K before quantization
  const u32x4* v8p;       // FP8 V in fragment order, 8 KB per 64 keys (PV8 only)
  const float* v_scale;   // [kv head][128] (PV8 only)
};
// PV8 (with QK8, 64-key blocks): the second product in FP8 with v_mfma_f32_32x32x64_f8f6f4 - a quarter of the V
// bytes and half the MFMA time of that product; see the PV8 section of the kernel.
constexpr float kIntOffset = 12582912.0f;            // 1.5 * 2^23, bit pattern 0x4B400000 (see qk_half)

template <int WAVES, bool BK32, bool QK8, bool PV8 = false>
__global__ __launch_bounds__(WAVES * 64) void attn_rows_kernel(Geo g, const uint16_t* __restrict__ q,
                                                               const bf16x8* __restrict__ kp,
                                                               const bf16x8* __restrict__ vp, Qk8 q8o,
                                                               const uint64_t* __restrict__ mask,
                                                               const int32_t* __restrict__ order,
                                                               const int32_t* __restrict__ assign,
                                                               uint16_t* __restrict__ o, float* __restrict__ o32,
                                                               float* __restrict__ lse,
                                                               RowFilter flt, f32x4* __restrict__ st_o,
                                                               float* __restrict__ st_ml) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane & 31, h = lane >> 5;
  const int units = g.n_qb * g.group;
  Unit u;
  const bool tail = WAVES == 1 && flt.tail_from >= 0 && (int)blockIdx.x >= flt.tail_from;
  {
    const int b = tail ? (int)blockIdx.x - flt.tail_from : (int)blockIdx.x;
    u.kvh = b % g.n_kvh;
    const int rank = tail ? (b / g.n_kvh) * flt.tail_stride + flt.tail_phase : (b / g.n_kvh) * WAVES + wave;
    u.valid = rank < units;
    int id = !u.valid ? 0 : (order ? order[(size_t)u.kvh * units + rank] : units - 1 - rank);
    if (assign && !tail) {
      // balanced issue: slot `rank` of lane blockIdx % n_kvh holds a unit of ANY KV head (or nothing)
      const int entry = u.valid ? assign[(size_t)u.kvh * units + rank] : -1;
      u.valid = entry >= 0;
      u.kvh = u.valid ? entry / units : 0;
      id = u.valid ? entry % units : 0;
    }
    u.i = id / g.group;
    u.qh = u.kvh * g.group + id % g.group;
  }
  if (!u.valid) return;
  const size_t unit_flat = (size_t)u.qh * g.n_qb + u.i;
  const int slot = flt.slot_of ? flt.slot_of[unit_flat] : -1;
  if (tail && slot >= 0) return;      // (rows with a slot are swept window by window through the tables)

  // ---- this wave's list of kept blocks: the set bits of its mask row, below the diagonal ----
  const uint64_t* mrow = mask ? mask + ((size_t)u.qh * g.n_qb + u.i) * g.words : nullptr;
  const SeqPos sp = seq_pos(g, u.i);                // (variable-length batches: block indices inside the row's sequence)
  const int il = sp.il;
  const int j_last = BK32 ? 2 * il + 1 : il;        // last causally visible mask bit of the row
  const int last_word = j_last >> 6;
  const int win_word = tail ? -1 : flt.win_word;
  if (win_word > last_word) return;
  const int word_lo = win_word >= 0 ? win_word : 0;
  const int word_hi = win_word >= 0 ? min(win_word + flt.win_words - 1, last_word) : last_word;
  const bool park = win_word >= 0 && word_hi < last_word;
  auto row_word = [&](int wc) -> uint64_t {
    const int lo = wc * 64;
    const uint64_t causal = j_last >= lo + 63 ? ~0ull : ((2ull << (j_last - lo)) - 1ull);
    return mrow ? (mrow[wc] & causal) : causal;
  };
  // A row takes part only in the windows where it keeps a block (and in its last one): it resumes iff an
  // earlier window held one of its blocks.
  bool resume = false;
  if (win_word > 0) {
    const uint64_t nonzero = __builtin_amdgcn_ballot_w64(lane < word_lo && row_word(lane) != 0ull);
    resume = nonzero != 0ull;
  }

  // ---- operands -----------------------------------------------------------------------
  // Q fragments (B operand of S^T = K Q^T), resident for the whole row.
  bf16x8 qf[QK8 ? 1 : 2][QK8 ? 1 : 8];
  i32x4 qf8[QK8 ? 2 : 1][QK8 ? 4 : 1];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    if constexpr (QK8) {
      const int8_t* row = q8o.q8 + ((size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c) * kHeadDim + 16 * h;
#pragma unroll
      for (int s = 0; s < 4; ++s) qf8[nt][s] = *(const i32x4*)(row + 32 * s);
    } else {
      const uint16_t* row = q + row_off(g.sq, u.qh, u.i * 64 + 32 * nt + c) + 8 * h;
#pragma unroll
      for (int s = 0; s < 8; ++s) qf[nt][s] = *(const bf16x8*)(row + 16 * s);
    }
  }
  const float cs = 0.08838834764831845f * 1.4426950408889634f;   // log2(e) / sqrt(d)
  // Logits are handled in log2 units: x = (raw product) * cl[slot], cl = log2(e) / sqrt(d), times the
  // scales of the 8-bit operands of the slot's key block when QK8.
  float cl[2] = {cs, cs};
  float ks_pend[2] = {1.0f, 1.0f};      // QK8: K scale of the half-tile whose operands were requested last
  float sq_cs = cs;
  const i32x4* k8t = nullptr;
  const float* ks8 = nullptr;
  if constexpr (QK8) {
    sq_cs = q8o.q_scale[unit_flat] * cs;
    k8t = (const i32x4*)q8o.k8p + ((size_t)u.kvh * g.seq + (size_t)(u.i - il) * 64) * 8 + lane;     // 512 16-byte chunks per 64 keys
    ks8 = q8o.k_scale + (size_t)u.kvh * (g.seq / 64) + (u.i - il);
  }
  // (the sequence's first key tile: u.i - il 64-row blocks into the KV head)
  const bf16x8* kt = kp + ((size_t)u.kvh * g.seq + (size_t)(u.i - il) * 64) * 16 + lane;     // 1024 16-byte chunks per 64 keys
  const bf16x8* vt = vp + ((size_t)u.kvh * g.seq + (size_t)(u.i - il) * 64) * 16 + lane;
  // Work proceeds in pairs of 32-key half-tiles held in slots 0 and 1; half-tile hb covers keys
  // 32hb .. 32hb+31 (half hb % 2 of the 64-key tile hb / 2 of K', V').  K operands of slot mt: kf[mt][s];
  // V operands of slot mt: vf[mt][dt][s2].
  bf16x8 kf[QK8 ? 1 : 2][QK8 ? 1 : 8], vf[2][4][2];
  i32x4 kf8[QK8 ? 2 : 1][QK8 ? 4 : 1];
  auto load_k = [&](int hb, int mt) __attribute__((always_inline)) {
    if constexpr (QK8) {
      const i32x4* t = k8t + (size_t)hb * 256;
#pragma unroll
      for (int s = 0; s < 4; ++s) kf8[mt][s] = t[s * 64];
      ks_pend[mt] = ks8[hb >> 1];
    } else {
      const bf16x8* t = kt + (size_t)hb * 512;
#pragma unroll
      for (int s = 0; s < 8; ++s) kf[mt][s] = t[s * 64];
    }
  };
  auto load_v = [&](int hb, int mt) __attribute__((always_inline)) {
    const bf16x8* t = vt + (size_t)(hb >> 1) * 1024 + (hb & 1) * 128;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) vf[mt][dt][s2] = t[(dt * 4 + s2) * 64];
  };

  f32x16 oacc[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][nt][r] = 0.0f;
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};      // m_run in log2 units

  if (resume) {
    const f32x4* so = st_o + (size_t)slot * 2048 + lane;       // [dt][nt][quarter][lane] 16-byte chunks
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const f32x4 w = so[((dt * 2 + nt) * 4 + qd) * 64];
#pragma unroll
          for (int e = 0; e < 4; ++e) oacc[dt][nt][4 * qd + e] = w[e];
        }
    const float* sml = st_ml + (size_t)slot * 256 + lane;       // [m nt0, m nt1, l nt0, l nt1][lane]
    m_run[0] = sml[0]; m_run[1] = sml[64]; l_run[0] = sml[128]; l_run[1] = sml[192];
  }
  int wc_it = word_lo;
  uint64_t cur = row_word(word_lo);
  auto next_block = [&]() -> int {
    while (cur == 0) {
      if (++wc_it > word_hi) return -1;
      cur = row_word(wc_it);
    }
    const int b = __builtin_ctzll(cur);
    cur &= cur - 1;
    return wc_it * 64 + b;
  };

  if constexpr (PV8) {
    // ---- fully quantized pass: 8-bit first product, FP8 second product ---------------------------------
    // One 64-key block per step, nothing deferred: S^T = K8 Q8^T (16 MFMAs), causal mask on the diagonal block,
    // ONE row maximum over the block's 64 keys, rescale, P8 = fp8(448 * exp2(x - m)) packed straight into the B
    // operand of the FP8 MFMA (a lane's 16 + 16 accumulator values of the two half-tiles are its 32 contraction
    // elements; the V8' copy is in the same key order), O^T += V8^T P8^T (8 MFMAs, K = 64).  The row sums are
    // one more MFMA per query tile with an all-ones A operand: numerator and denominator are then sums of the
    // SAME rounded probabilities.  The next block's K8 is requested once the first product has consumed this
    // block's, the next V8 once the second product has.
    static_assert(QK8 && !BK32, "the FP8 second product comes with the 8-bit first product on 64-key blocks");
    const u32x4* const v8t = q8o.v8p + ((size_t)u.kvh * g.seq + (size_t)(u.i - il) * 64) * 8 + lane;   // 512 chunks per 64 keys
    const float kLog2Top = 8.807354922057604f;      // log2(448)
    i32x4 k8[2][4];
    u32x4 v8[4][2];
    float k_sc = 1.0f;
    auto fetch_k = [&](int j) __attribute__((always_inline)) {
      const i32x4* t = k8t + (size_t)j * 512;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int s = 0; s < 4; ++s) k8[mt][s] = t[(mt * 4 + s) * 64];
      k_sc = ks8[j];
    };
    auto fetch_v = [&](int j) __attribute__((always_inline)) {
      const u32x4* t = v8t + (size_t)j * 512;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) v8[dt][jj] = t[(dt * 2 + jj) * 64];
    };
    f32x16 lacc[2];      // every register: sum over the row's keys of P8 (all 32 rows of the ones product are equal)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) lacc[nt][r] = 2.0f * l_run[nt];      // (parked as half the sum: see below)
    i32x8 ones8;
#pragma unroll
    for (int w = 0; w < 8; ++w) ones8[w] = 0x38383838;                   // 1.0 in E4M3
    i32x16 magic;
#pragma unroll
    for (int r = 0; r < 16; ++r) magic[r] = 0x4B400000;
    // one block; `diag`: apply the causal mask (the diagonal block) - a variant of its own, so that the other
    // blocks pay nothing for it
    auto step8 = [&](int jn_or_j, auto diag) __attribute__((always_inline)) {
      // (the accumulators start at the bit pattern of kIntOffset and are read as floats, as in qk_half)
      i32x16 a[2][2];
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            a[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(k8[mt][s], qf8[nt][s], s == 0 ? magic : a[mt][nt], 0, 0, 0);
      const float cj = k_sc * sq_cs;                 // raw integer product -> logit in log2 units
      const float off = kIntOffset * cj;                 // what the offset amounts to in logit units
      fetch_k(jn_or_j);                              // (unconditional: the last block re-reads its own)
      float S[2][2][16];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            S[mt][nt][r] = int_bits_as_float(a[mt][nt][r]);
            if constexpr (decltype(diag)::value) {
              if (32 * mt + mfma32_row(r, lane) > 32 * nt + c) S[mt][nt][r] = -INFINITY;
            }
          }
      float mx[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        float v = fmaxf(S[0][nt][0], S[1][nt][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) v = fmaxf(fmaxf(v, S[0][nt][r]), S[1][nt][r]);
        mx[nt] = __builtin_fmaf(max_with_other_half(v), cj, -off);
      }
      if (__builtin_amdgcn_ballot_w64(mx[0] > m_run[0] || mx[1] > m_run[1]) != 0ull) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const float m_new = fmaxf(m_run[nt], mx[nt]);
          const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new);
          m_run[nt] = m_new;
#pragma unroll
          for (int r = 0; r < 16; ++r) lacc[nt][r] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
        }
      }
      i32x8 p8[2];
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float mb = m_run[nt] - kLog2Top + off;       // exp2(x - m) * 448, x = (S - offset) * cj
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mt][nt][4 * w], cj, -mb));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mt][nt][4 * w + 1], cj, -mb));
            const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mt][nt][4 * w + 2], cj, -mb));
            const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[mt][nt][4 * w + 3], cj, -mb));
            int word = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, 0, false);
            word = __builtin_amdgcn_cvt_pk_fp8_f32(p2, p3, word, true);
            p8[nt][4 * mt + w] = word;
          }
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        i32x8 va;
#pragma unroll
        for (int w = 0; w < 4; ++w) { va[w] = (int)v8[dt][0][w]; va[4 + w] = (int)v8[dt][1][w]; }
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
          oacc[dt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, p8[nt], oacc[dt][nt], 0, 0, 0, 0, 0, 0);
      }
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
        lacc[nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones8, p8[nt], lacc[nt], 0, 0, 0, 0, 0, 0);
      fetch_v(jn_or_j);                              // (unconditional as well: every path leaves the same loads in flight,
                                                     // so the next step waits for exactly the K8 it needs, not for everything)
    };
    int j = next_block();
    if (j >= 0) {
      fetch_k(j);
      fetch_v(j);
      while (true) {
        const int jn = next_block();
        if (j == il) step8(jn >= 0 ? jn : j, std::true_type{}); else step8(jn >= 0 ? jn : j, std::false_type{});
        if (jn < 0) break;
        j = jn;
      }
    }
    // the common tail adds the two lane halves' partial sums; here every lane already holds the whole sum
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) l_run[nt] = 0.5f * lacc[nt][0];
  } else {
  // ---- pipeline stages ----------------------------------------------------------------
  // Half-tile score accumulators S[mt][nt] (keys 32mt.. x queries 32nt..) and the bf16 P^T operands
  // P[mt][nt][s2] made from them.  The MFMA stream and the softmax VALU stream of DIFFERENT half-tiles
  // are written side by side so that they overlap inside one wave:
  //   stage A: O += V^T P^T of the previous block's half 1   ||  row max of S[0], rescale test
  //   stage B: S[1] = K Q^T of this block's half 1            ||  P[0] = exp2(S[0] - max), row sums
  //   stage C: O += V^T P^T of this block's half 0            ||  row max of S[1], rescale test
  //   stage D: S[0] = K Q^T of the NEXT block's half 0        ||  P[1] = exp2(S[1] - max), row sums
  f32x16 S[2][2];
  bf16x8 P[2][2][2];

  auto qk_half = [&](int mt) __attribute__((always_inline)) {                       // S[mt][*] = K(half mt) Q^T
    if constexpr (QK8) {
      // The integer accumulators start at the bit pattern of kIntOffset = 1.5 * 2^23: an integer x with |x| < 2^22
      // added to it (the sums are below 127 * 127 * 128 < 2^21) gives the bit pattern of the FLOAT kIntOffset + x,
      // so the sums are read as floats without a conversion each; the offset leaves with the scaling FMAs.
      i32x16 a0, a1;
#pragma unroll
      for (int r = 0; r < 16; ++r) a0[r] = a1[r] = 0x4B400000;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        a0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf8[mt][s], qf8[0][s], a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf8[mt][s], qf8[1][s], a1, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        S[mt][0][r] = int_bits_as_float(a0[r]);
        S[mt][1][r] = int_bits_as_float(a1[r]);
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[mt][nt][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        S[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][s], qf[0][s], S[mt][0], 0, 0, 0);
        S[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][s], qf[1][s], S[mt][1], 0, 0, 0);
      }
    }
  };
  auto pv_half = [&](int mt) __attribute__((always_inline)) {                       // O^T += V^T(half mt) P^T(half mt)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        oacc[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mt][dt][s2], P[mt][0][s2], oacc[dt][0], 0, 0, 0);
        oacc[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mt][dt][s2], P[mt][1][s2], oacc[dt][1], 0, 0, 0);
      }
  };
  // Row maxima of the half-tile in slot mt (after causal masking where `diag` asks for it): mx[nt].
  // koff[mt]: first key of the slot's half-tile minus the first query row of the block (b_k = 32 only;
  // with b_k = 64 the masked pair is the diagonal block: 0 and 32).  A huge koff empties the slot.
  float mx[2];
  int koff[2] = {0, 32};
  auto max_half = [&](int mt, auto diag) __attribute__((always_inline)) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      if constexpr (decltype(diag)::value) {
        const int ko = BK32 ? koff[mt] : 32 * mt;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (ko + mfma32_row(r, lane) > 32 * nt + c) S[mt][nt][r] = -INFINITY;
      }
      float v = fmaxf(S[mt][nt][0], S[mt][nt][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) v = fmaxf(fmaxf(v, S[mt][nt][r]), S[mt][nt][r + 1]);
      if constexpr (QK8) mx[nt] = __builtin_fmaf(max_with_other_half(v), cl[mt], -kIntOffset * cl[mt]);
      else mx[nt] = max_with_other_half(v) * cl[mt];
    }
  };
  // Lazy rescale: O and l are rescaled only when some row's maximum grew (exact: otherwise the factor
  // is 1).  Rows of the diagonal block that see no key of a half keep their (finite) maximum.
  auto rescale = [&]() __attribute__((always_inline)) {
    if (__builtin_amdgcn_ballot_w64(mx[0] > m_run[0] || mx[1] > m_run[1]) != 0ull) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float m_new = fmaxf(m_run[nt], mx[nt]);
        float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new);
        // b_k = 32: a query row may have seen no key yet (its first half-tile lies above the diagonal)
        if constexpr (BK32) alpha = m_new == -INFINITY ? 1.0f : alpha;
        l_run[nt] *= alpha;
        m_run[nt] = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][nt][r] *= alpha;
      }
    }
  };
  // Interleave hint for the instruction scheduler: n times {1 MFMA, `valu` VALU, `vmem` loads}.
#define SALE_PIPE(n, valu, vmem)                                        \
  _Pragma("unroll") for (int i_ = 0; i_ < (n); ++i_) {                   \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   \
    if ((valu) > 0) __builtin_amdgcn_sched_group_barrier(0x002, (valu), 0); \
    if ((vmem) > 0) __builtin_amdgcn_sched_group_barrier(0x020, (vmem), 0); \
  }
  auto exp_half = [&](int mt) __attribute__((always_inline)) {                      // P[mt] = exp2(S[mt] * cs - m * cs), l += row sums
    bf16x2 ones;
    ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const float ch = cl[mt];
      float mb = (BK32 && m_run[nt] == -INFINITY) ? 0.0f : m_run[nt];
      if constexpr (QK8) mb += kIntOffset * ch;        // S carries the accumulators' offset
      float sum = l_run[nt];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        u32x4 packed;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          const int r = 8 * s2 + 2 * e2;
          bf16x2 pk;
          pk[0] = (__bf16)__builtin_amdgcn_exp2f(S[mt][nt][r] * ch - mb);
          pk[1] = (__bf16)__builtin_amdgcn_exp2f(S[mt][nt][r + 1] * ch - mb);
          sum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, sum, false);   // row sum of the rounded P
          packed[e2] = __builtin_bit_cast(unsigned, pk);
        }
        P[mt][nt][s2] = __builtin_bit_cast(bf16x8, packed);
      }
      l_run[nt] = sum;
    }
  };

  // One pair of half-tiles (slot 0: cur.a, slot 1: cur.b).  first: no previous pair whose slot 1 is still
  // to be multiplied.  last: no next pair (nxt is then unused).  diag: apply the causal mask (and, with
  // b_k = 32, the emptying of a slot that has no half-tile).
  // Every load and MFMA of a variant is unconditional, so the compiler can count outstanding loads
  // exactly and never has to drain the queue.
  struct Pair { int a, b; };
  auto block_step = [&](Pair cur, Pair nxt, auto first, auto last, auto diag) __attribute__((always_inline)) {
    constexpr bool kLast = decltype(last)::value;
    // stage A
    if constexpr (!decltype(first)::value) pv_half(1);
    max_half(0, diag);
    load_v(cur.b, 1);
    if constexpr (!decltype(first)::value) { SALE_PIPE(16, 2, 1) }
    rescale();
    // stage B
    qk_half(1);
    exp_half(0);
    // stage C
    if constexpr (QK8) cl[1] = ks_pend[1] * sq_cs;      // scale of slot 1's key block, requested a step ago
    pv_half(0);
    max_half(1, diag);
    if constexpr (!kLast) { load_k(nxt.b, 1); load_v(nxt.a, 0); }
    SALE_PIPE(16, 6, 0)
    SALE_PIPE(16, 2, 1)
    rescale();
    // stage D (kf[0] of the next pair was requested before stage A)
    if constexpr (!kLast) qk_half(0);
    exp_half(1);
    if constexpr (!kLast) {
      if constexpr (QK8) { SALE_PIPE(8, 14, 0) } else { SALE_PIPE(16, 6, 0) }      // 8 MFMAs in the 8-bit first product
    }
    if constexpr (QK8 && !kLast) cl[0] = ks_pend[0] * sq_cs;      // slot 0 now holds the next pair's first half-tile
  };
  const auto T = std::true_type{};
  const auto F = std::false_type{};

  // b_k = 32: an odd number of kept half-tiles leaves one without a partner.  It goes FIRST, next to an
  // emptied slot 1 (which re-reads the same half-tile), so that every later pair is complete and the
  // half-tiles of the diagonal block, the largest indices of a row, fall into the last pair.  The first
  // and the last pair of a sweep take the masked variant.
  bool lone_first = false;
  if constexpr (BK32) {
    const int wcl = word_lo + lane;
    const int bits = wcl <= word_hi ? __popcll(row_word(wcl)) : 0;
    lone_first = (__popcll(__builtin_amdgcn_ballot_w64((bits & 1) != 0)) & 1) != 0;
  }
  constexpr int kEmptySlot = 1 << 24;
  auto next_pair = [&](Pair& pr) -> bool {
    const int a = next_block();
    if (a < 0) return false;
    if constexpr (BK32) {
      pr.a = a;
      const int b = next_block();
      pr.b = b < 0 ? a : b;      // (b < 0 cannot happen once the lone half-tile has gone first)
    } else {
      pr.a = 2 * a;
      pr.b = 2 * a + 1;
    }
    return true;
  };
  auto set_koff = [&](Pair pr, bool empty_b) {
    if constexpr (BK32) {
      koff[0] = (pr.a - 2 * il) * 32;
      koff[1] = empty_b ? kEmptySlot : (pr.b - 2 * il) * 32;
    }
  };

  Pair pc = {0, 0}, pn = {0, 0}, pa = {0, 0};
  bool have;
  if (BK32 && lone_first) {
    const int a = next_block();
    have = a >= 0;
    pc.a = pc.b = a;
  } else {
    have = next_pair(pc);
  }
  if (have) {
    load_k(pc.a, 0);
    load_k(pc.b, 1);
    load_v(pc.a, 0);
    qk_half(0);
    if constexpr (QK8) cl[0] = ks_pend[0] * sq_cs;
    bool has_next = next_pair(pn);
    set_koff(pc, lone_first);
    if (!has_next) {
      if (BK32 || pc.a == 2 * il) block_step(pc, pc, T, T, T); else block_step(pc, pc, T, T, F);
    } else {
      // the list is read one pair ahead of the loads so that no control flow separates the stages
      load_k(pn.a, 0);
      bool has_aft = next_pair(pa);
      if constexpr (BK32) block_step(pc, pn, T, F, T); else block_step(pc, pn, T, F, F);
      pc = pn; pn = pa; has_next = has_aft;
      while (has_next) {
        load_k(pn.a, 0);
        has_aft = next_pair(pa);
        block_step(pc, pn, F, F, F);
        pc = pn; pn = pa; has_next = has_aft;
      }
      set_koff(pc, false);
      if (BK32 || pc.a == 2 * il) block_step(pc, pc, F, T, T); else block_step(pc, pc, F, T, F);
    }
    pv_half(1);
  }

  }

  if (park) {
    f32x4* so = st_o + (size_t)slot * 2048 + lane;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          f32x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = oacc[dt][nt][4 * qd + e];
          so[((dt * 2 + nt) * 4 + qd) * 64] = w;
        }
    float* sml = st_ml + (size_t)slot * 256 + lane;
    sml[0] = m_run[0]; sml[64] = m_run[1]; sml[128] = l_run[0]; sml[192] = l_run[1];
    return;
  }
  // Output.  A lane holds, per (nt, dt, q4), four consecutive channels of one query row: stored from there a
  // store instruction touches 32 rows, 16 bytes each.  The bf16 tile goes through LDS instead (rows padded by
  // four banks) and leaves as whole 256-byte rows, 4 rows per instruction.
  constexpr int kRowPad = kHeadDim + 8;      // bf16 elements per LDS row
  __shared__ __attribute__((aligned(16))) uint16_t o_lds[WAVES * 64 * kRowPad];
  uint16_t* const tile = o_lds + wave * 64 * kRowPad;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float l_tot = l_run[nt] + swap_half(l_run[nt]);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    if constexpr (PV8) {      // O = v_scale[channel] * (sum P8 V8) / (sum P8)
      const float* vs = q8o.v_scale + (size_t)u.kvh * kHeadDim + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 sc = *(const f32x4*)(vs + 32 * dt + 8 * q4);
#pragma unroll
          for (int e = 0; e < 4; ++e) oacc[dt][nt][4 * q4 + e] *= sc[e];
        }
    }
    const size_t row = (size_t)u.qh * g.seq + u.i * 64 + 32 * nt + c;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        if (o32) {     // calibration reads the output before it is rounded to bf16
          f32x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = oacc[dt][nt][4 * q4 + e] * inv;
          *(f32x4*)(o32 + row * kHeadDim + 4 * h + 32 * dt + 8 * q4) = w;
        } else {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(oacc[dt][nt][4 * q4 + e] * inv);
          *(bf16x4*)(tile + (32 * nt + c) * kRowPad + 4 * h + 32 * dt + 8 * q4) = w;
        }
      }
    if (lse && h == 0) {
      // (PV8: the sum is that of 448 p)
      float v = l_tot > 0.0f ? m_run[nt] * 0.6931471805599453f + __logf(PV8 ? l_tot * (1.0f / 448.0f) : l_tot) : -INFINITY;
      if constexpr (QK8) {
        // The 8-bit logits are those of K minus its mean key, i.e. Eq. 1's logits of this row minus q_r . mean /
        // sqrt(d) (which the softmax cancels in O); lse is reported for Eq. 1's S, so the shift goes back in.
        const uint16_t* qr = q + row_off(g.sq, u.qh, u.i * 64 + 32 * nt + c);
        const float* mean = q8o.k_mean + (size_t)u.kvh * kHeadDim;
        float dot = 0.0f;
        for (int ch = 0; ch < kHeadDim; ++ch) dot = __builtin_fmaf(bf16_bits_to_float(qr[ch]), mean[ch], dot);
        v += dot * 0.08838834764831845f;
      }
      lse[row] = v;
    }
  }
  if (!o32) {
    // (each wave reads back only its own tile: no barrier, LDS operations of a wave complete in order)
    uint16_t* const out = o + row_off(g.so, u.qh, u.i * 64);
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int r = 4 * it + (lane >> 4), ch = 8 * (lane & 15);
      *(u32x4*)(out + (size_t)r * g.so.st + ch) = *(const u32x4*)(tile + r * kRowPad + ch);
    }
  }
}

// Counting sort of the units of each KV head by kept-block count, descending:
// order[kvh][rank] = unit id (block * group + head-in-group).  One workgroup per KV head.
// slot_of (optional): rows keeping more than long_count blocks draw a parking slot from *slot_counter (cleared by
// the K' / V' copy that precedes this kernel) as long as there are slots; every other row gets -1.
__global__ __launch_bounds__(1024) void order_units_kernel(Geo g, const int32_t* __restrict__ row_counts,
                                                           int32_t* __restrict__ order, int32_t* __restrict__ slot_of,
                                                           int long_count, int n_slots, int* __restrict__ slot_counter) {
  __shared__ int bin[kMaskWordsMax * 64 + 2];
  const int kvh = blockIdx.x, units = g.n_qb * g.group;
  const int max_count = min(g.n_kb, g.words * 64);      // (a row keeps at most the key blocks of its own sequence)
  const int nbins = max_count + 1;
  for (int b = threadIdx.x; b < nbins; b += blockDim.x) bin[b] = 0;
  __syncthreads();
  auto count_of = [&](int id) {
    const int c = row_counts[(size_t)(kvh * g.group + id % g.group) * g.n_qb + id / g.group];
    return min(max(c, 0), max_count);
  };
  for (int id = threadIdx.x; id < units; id += blockDim.x) atomicAdd(&bin[count_of(id)], 1);
  __syncthreads();
  if (threadIdx.x == 0) {          // start offset of every bin, largest count first
    int run = 0;
    for (int b = nbins - 1; b >= 0; --b) { const int n = bin[b]; bin[b] = run; run += n; }
  }
  __syncthreads();
  for (int id = threadIdx.x; id < units; id += blockDim.x) {
    const int cnt = count_of(id);
    order[(size_t)kvh * units + atomicAdd(&bin[cnt], 1)] = id;
    if (slot_of) {
      int slot = -1;
      if (cnt > long_count && n_slots > 0) {
        slot = atomicAdd(slot_counter, 1);
        if (slot >= n_slots) slot = -1;
      }
      slot_of[(size_t)(kvh * g.group + id % g.group) * g.n_qb + id / g.group] = slot;
    }
  }
}

// All three in units of 64 keys (scaled by 64 / b_k for a mask with one bit per b_k keys).
// Workgroups go to the XCDs round-robin, so "lane" blockIdx % n_kvh of a launch always runs on the same XCDs.
// With lane = KV head an XCD's L2 serves one head's K', V', but the heads of a layer keep very different
// numbers of blocks (1.6x between the lightest and the heaviest at 128K here) and the light XCDs would idle.
// For every window launch (one workgroup of this kernel each) a table moves a representative sample (every
// so-many-th of the sorted list) of the units of every over-loaded head to the lanes of the under-loaded
// ones, in proportion to the work they lack in THAT window:
//   assign[window][lane][slot] = kvh * units + unit id, or -1.
// A unit takes part in a window if its row has a parking slot (a long row) and keeps a block there, or if the
// window holds its diagonal block (where the row is finished whatever it keeps).
// Falls back to lane = KV head when there are too many lanes or a lane would overflow.
constexpr int kMaxLanes = 256;
struct LaneLoad { unsigned long long work; int n_in; int pad; };      // per (window, KV head)
constexpr size_t kLaneLoadBytes = (size_t)(kMaskWordsMax / 2) * kMaxLanes * sizeof(LaneLoad);      // 128 KB

// Shared by the two kernels below: the units of ONE head in ONE window, 1024 threads, thread t looks at the
// ranks t * per .. of the head's sorted list.
struct WindowScan {
  const Geo& g;
  const uint64_t* mask;
  const int32_t* slot_of;
  const int32_t* order;
  int w0, w1, bits_per_q, units;
  // blocks the unit at rank r of head h keeps in this window (-1: it does not take part)
  __device__ int in_window(int h, int r, int& id) const {
    id = order[(size_t)h * units + r];
    const int i = id / g.group, qh = h * g.group + id % g.group;
    if (slot_of[(size_t)qh * g.n_qb + i] < 0) return -1;      // swept whole, in a tail
    const int j_last = (seq_pos(g, i).il + 1) * bits_per_q - 1, last_word = j_last >> 6;
    if (w0 > last_word) return -1;
    const uint64_t* mrow = mask + ((size_t)qh * g.n_qb + i) * g.words;
    int c = 0;
    for (int wc = w0; wc < min(w1, last_word + 1); ++wc) {
      const int lo = wc * 64;
      const uint64_t causal = j_last >= lo + 63 ? ~0ull : ((2ull << (j_last - lo)) - 1ull);
      c += __popcll(mrow[wc] & causal);
    }
    return (c > 0 || w1 > last_word) ? c : -1;
  }
};

// exclusive prefix over a 1024-thread workgroup of a per-thread count; total in `sum`
__device__ __forceinline__ int block_scan_1024(int v, int* wave_sum, int& sum) {
  const int lane_id = threadIdx.x & 63, wave_id = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(inc, off, 64);
    if (lane_id >= off) inc += o;
  }
  __syncthreads();
  if (lane_id == 63) wave_sum[wave_id] = inc;
  __syncthreads();
  int base = 0, all = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int x = wave_sum[w];
    if (w < wave_id) base += x;
    all += x;
  }
  sum = all;
  return base + inc - v;
}

// Workgroup (window, head): number of participating units and their work in the window; clears the head's
// own lane of the window's table.
__global__ __launch_bounds__(1024) void window_load_kernel(Geo g, const uint64_t* __restrict__ mask,
                                                           const int32_t* __restrict__ slot_of,
                                                           const int32_t* __restrict__ order, int win_words,
                                                           int bits_per_q, LaneLoad* __restrict__ load,
                                                           int32_t* __restrict__ assign_all) {
  __shared__ int wave_sum[16];
  __shared__ unsigned long long work;
  const int units = g.n_qb * g.group, lanes = g.n_kvh;
  const int win = blockIdx.x / lanes, h = blockIdx.x % lanes;
  const int tid = threadIdx.x, per = (units + 1023) / 1024;
  const WindowScan ws = {g, mask, slot_of, order, win * win_words, (win + 1) * win_words, bits_per_q, units};
  int32_t* mine = assign_all + ((size_t)win * lanes + h) * units;
  for (int e = tid; e < units; e += 1024) mine[e] = -1;
  if (tid == 0) work = 0;
  int n_mine = 0;
  unsigned long long w_mine = 0;
  for (int r = tid * per; r < min((tid + 1) * per, units); ++r) {
    int id;
    const int c = ws.in_window(h, r, id);
    if (c >= 0) { ++n_mine; w_mine += (unsigned long long)c; }
  }
  int n_tot;
  block_scan_1024(n_mine, wave_sum, n_tot);      // (its barriers also publish work = 0)
  if (w_mine) atomicAdd(&work, w_mine);
  __syncthreads();
  if (tid == 0 && h < kMaxLanes) { load[win * kMaxLanes + h].work = work; load[win * kMaxLanes + h].n_in = n_tot; }
}

// Workgroup (window, head): places the head's participating units in the window's table.
__global__ __launch_bounds__(1024) void balance_kernel(Geo g, const uint64_t* __restrict__ mask,
                                                       const int32_t* __restrict__ slot_of,
                                                       const int32_t* __restrict__ order, int win_words,
                                                       int bits_per_q, const LaneLoad* __restrict__ load,
                                                       int32_t* __restrict__ assign_all) {
  __shared__ int n_shed_h, shed_off_h, n_in_h, recv_lo[kMaxLanes + 1];
  __shared__ int wave_sum[16];
  const int units = g.n_qb * g.group, lanes = g.n_kvh;
  const int win = blockIdx.x / lanes, h = blockIdx.x % lanes;
  const int tid = threadIdx.x, per = (units + 1023) / 1024;
  const WindowScan ws = {g, mask, slot_of, order, win * win_words, (win + 1) * win_words, bits_per_q, units};
  int32_t* assign = assign_all + (size_t)win * lanes * units;
  const bool balance = lanes <= kMaxLanes && lanes > 1;
  if (tid == 0) {
    n_shed_h = 0; shed_off_h = 0; n_in_h = 1;
    for (int l = 0; l <= min(lanes, kMaxLanes); ++l) recv_lo[l] = 0;
    if (balance) {
      const LaneLoad* ld = load + win * kMaxLanes;
      unsigned long long sum = 0;
      for (int l = 0; l < lanes; ++l) sum += ld[l].work;
      const double target = (double)sum / lanes;
      double lack_total = 0.0;
      int shed_total = 0, my_shed = 0, my_off = 0;
      for (int l = 0; l < lanes; ++l) {
        const double w = (double)ld[l].work;
        const int ns = w > target ? (int)((double)ld[l].n_in * (w - target) / w) : 0;
        if (l == h) { my_shed = ns; my_off = shed_total; }
        shed_total += ns;
        if (w < target) lack_total += target - w;
      }
      // the shed units, numbered (offset of their head) + k, go to the lanes that lack work, in proportion
      double lack_run = 0.0;
      bool ok = lack_total > 0.0;
      for (int l = 0; l < lanes && ok; ++l) {
        recv_lo[l] = (int)((double)shed_total * (lack_run / lack_total));
        const double w = (double)ld[l].work;
        if (w < target) lack_run += target - w;
      }
      recv_lo[lanes] = shed_total;
      for (int l = 0; l < lanes && ok; ++l) {
        const double w = (double)ld[l].work;
        const int ns = w > target ? (int)((double)ld[l].n_in * (w - target) / w) : 0;
        ok = ld[l].n_in - ns + recv_lo[l + 1] - recv_lo[l] <= units;
      }
      if (ok) { n_shed_h = my_shed; shed_off_h = my_off; n_in_h = max(ld[h].n_in, 1); }
      else for (int l = 0; l <= lanes; ++l) recv_lo[l] = 0;
    }
  }
  int n_mine = 0;
  for (int rr = tid * per; rr < min((tid + 1) * per, units); ++rr) {
    int id;
    if (ws.in_window(h, rr, id) >= 0) ++n_mine;
  }
  int n_tot;
  int r = block_scan_1024(n_mine, wave_sum, n_tot);      // (its barriers also publish thread 0's parameters)
  // r counts the participating units of the head in sorted order (longest rows first)
  for (int rr = tid * per; rr < min((tid + 1) * per, units); ++rr) {
    int id;
    if (ws.in_window(h, rr, id) < 0) continue;
    int lane = h, pos = r;
    if (balance) {
      const long long ns = n_shed_h, n = n_in_h;
      const int before = (int)((long long)r * ns / n), upto = (int)((long long)(r + 1) * ns / n);
      if (upto > before) {                      // this unit is shed: global shed number p
        const int p = shed_off_h + before;
        int l = 0;
        while (l + 1 < lanes && recv_lo[l + 1] <= p) ++l;
        lane = l;
        // Received units go first in their new lane: all lanes then read the shedding head's window at the
        // start of a launch, together (interleaving them with the lane's own units was 6 % slower).
        pos = p - recv_lo[l];
      } else {
        pos = (recv_lo[h + 1] - recv_lo[h]) + (r - before);
      }
    }
    assign[(size_t)lane * units + pos] = h * units + id;
    ++r;
  }
}

constexpr int kLongRow = 192;        // rows keeping more than this (12K tokens) are swept window by window
constexpr int kWindowWords = 2;      // window width in mask words of 64 x 64 keys: 8K tokens, 4 MB of K', V' per KV head
constexpr int kWindowMinWords = 4;   // sequences of up to 16K tokens use one sweep per row

namespace {

template <bool BK32, bool QK8, bool PV8 = false>
int launch_sparse_rows(const Geo& g, const uint16_t* q, const bf16x8* kp, const bf16x8* vp, Qk8 q8o, const uint64_t* mask,
                       const int32_t* row_counts, int32_t* order, int32_t* assign, LaneLoad* load, int32_t* slot_of,
                       int* slot_counter, int n_slots, uint16_t* o, float* o32, float* lse, f32x4* st_o, float* st_ml,
                       hipStream_t st) {
  const int units = g.n_qb * g.group;
  const int f = BK32 ? 2 : 1;          // mask bits per 64 keys
  const dim3 grid((unsigned)(units * g.n_kvh));
  const RowFilter all = {nullptr, -1, 0, -1, 0, 0};
  // Without a single parking slot in the workspace every row is swept whole.
  const bool windows = row_counts && g.words > kWindowMinWords * f && n_slots > 0;
  if (row_counts) {
    order_units_kernel<<<dim3((unsigned)g.n_kvh), dim3(1024), 0, st>>>(g, row_counts, order, windows ? slot_of : nullptr,
                                                                       kLongRow * f, n_slots, slot_counter);
    if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  }
  if (!windows) {
    // (one sweep per row: every row reads K', V' of the whole sequence, and moving rows to another XCD costs
    // more L2 misses than the balance gains: 3.1 against 2.7 ms at 32K)
    attn_rows_kernel<1, BK32, QK8, PV8><<<grid, dim3(64), 0, st>>>(g, q, kp, vp, q8o, mask, row_counts ? order : nullptr, nullptr,
                                                             o, o32, lse, all, nullptr, nullptr);
    return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
  }

  // Long rows carry most of the work and keep scattered blocks over the whole sequence: swept
  // independently they miss L2 on most loads.  They are processed one window of 8K tokens (4 MB of K', V'
  // per KV head: the size of an XCD's L2) at a time, all rows together, so that the window is served by
  // the L2 of the XCD that owns the KV head; their accumulators wait in the workspace in between.
  // Measured at 128K tokens (L2 fills / time of the call): one sweep per row 218 GB / 50.7 ms; windows of
  // 16K tokens 121 GB / 37.5 ms; 8K tokens 57 GB / 37.4 ms; 4K tokens 50 GB / 39.1 ms (the parked state
  // then costs more than the window saves).  At 32K tokens windows (with the balancing below) and one sweep
  // per row are within 2 % of each other; shorter sequences use one sweep.
  // Short rows keep little besides the sink, the local band and the heavy columns everyone shares.
  // They are dealt over the window launches: launch number n ends with ranks n, n + launches, ... of every
  // KV head's sorted list (the tail of the grid), which fill the chip while its last long rows finish.
  const int step = kWindowWords * f, launches = (g.words + step - 1) / step;
  const int tail_wgs = ((units + launches - 1) / launches) * g.n_kvh;
  window_load_kernel<<<dim3((unsigned)(launches * g.n_kvh)), dim3(1024), 0, st>>>(g, mask, slot_of, order, step, f, load,
                                                                                 assign);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  balance_kernel<<<dim3((unsigned)(launches * g.n_kvh)), dim3(1024), 0, st>>>(g, mask, slot_of, order, step, f, load, assign);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  for (int n = 0; n < launches; ++n) {
    // (the table holds the rows with a parking slot; the tail takes the others)
    const RowFilter flt = {slot_of, n * step, step, (int)grid.x, launches, n};
    attn_rows_kernel<1, BK32, QK8, PV8><<<dim3(grid.x + (unsigned)tail_wgs), dim3(64), 0, st>>>(
        g, q, kp, vp, q8o, mask, order, assign + (size_t)n * grid.x, o, o32, lse, flt, st_o, st_ml);
    if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  }
  return SALE_OK;
}

}  // namespace

// Workspace of the attention calls.  Fixed part: K' | V' | (sparse: unit order | parking slot per row block | balanced
// issue tables, room for 32 window launches | per-window head loads | slot counter) | 8-bit operand copies | FP8 copy
// of V | per-block sequence table; then (sparse) the parking slots, 33 KB each: as many as the caller's workspace holds.
namespace {
struct AttnWs {
  u32x4 *kp, *vp;
  int32_t *order, *slot_of, *assign;
  LaneLoad* load;
  int* slot_counter;
  uint8_t *ops8, *ops_fp8;
  int32_t* seq_table;
  uint8_t* parked;
  size_t fixed_bytes;
};
AttnWs carve_attn_ws(const sale_params_t* p, bool sparse, void* base) {
  const size_t tile_bytes = (size_t)p->batch * p->n_kv_heads * p->seq_len * kHeadDim * sizeof(uint16_t);
  const size_t n_units = (size_t)p->batch * p->n_q_heads * (p->seq_len / kBlockQ);
  AttnWs w = {};
  size_t off = 0;
  auto take = [&](size_t bytes) { uint8_t* ptr = (uint8_t*)base + off; off += (bytes + 63) & ~(size_t)63; return ptr; };
  w.kp = (u32x4*)take(tile_bytes);
  w.vp = (u32x4*)take(tile_bytes);
  if (sparse) {
    w.order = (int32_t*)take(n_units * sizeof(int32_t));
    w.slot_of = (int32_t*)take(n_units * sizeof(int32_t));
    w.assign = (int32_t*)take(n_units * (kMaskWordsMax / 2) * sizeof(int32_t));
    w.load = (LaneLoad*)take(kLaneLoadBytes);
    w.slot_counter = (int*)take(sizeof(int));
  }
  if (p->flags & SALE_FLAG_ATTN_INT8_QK) w.ops8 = take(int8_operand_bytes(p));
  if (p->flags & SALE_FLAG_ATTN_FP8_PV) w.ops_fp8 = take(fp8_operand_bytes(p));
  if (p->n_seqs > 0) w.seq_table = (int32_t*)take(seq_table_bytes(p));
  w.parked = (uint8_t*)base + off;
  w.fixed_bytes = off;
  return w;
}
}  // namespace

size_t attn_fixed_bytes(const sale_params_t* p, bool sparse) { return carve_attn_ws(p, sparse, nullptr).fixed_bytes; }

// o: bf16 output, or (o32 != nullptr) fp32 output instead.  mask == nullptr: dense causal attention
// (independent of b_k).  ws_bytes >= attn_fixed_bytes (checked by the callers); what lies beyond holds parking slots.
int launch_attn_rows(const sale_params_t* p, const void* q, const void* k, const void* v, const uint64_t* mask,
                     const int32_t* row_counts, void* o, float* o32, float* lse, void* ws, size_t ws_bytes, hipStream_t st) {
  Geo g = make_geo(p);
  const AttnWs w = carve_attn_ws(p, mask != nullptr, ws);
  if (ws_bytes < w.fixed_bytes) return SALE_ERR_WORKSPACE;
  if (p->n_seqs > 0) {
    const int rc = build_seq_table(p, w.seq_table, st);
    if (rc != SALE_OK) return rc;
    g.seq_start = w.seq_table;
  }
  u32x4 *kp = w.kp, *vp = w.vp;
  const size_t n_units = (size_t)g.n_qh * g.n_qb;
  const size_t n_slots_z = mask ? (ws_bytes - w.fixed_bytes) / kParkedRowBytes : 0;
  const int n_slots = (int)(n_slots_z < n_units ? n_slots_z : n_units);
  f32x4* st_o = (f32x4*)w.parked;                               // [slot] 32 KB
  float* st_ml = (float*)(w.parked + (size_t)n_slots * 2048 * 16);      // [slot] 1 KB
  int32_t *order = w.order, *assign = w.assign;
  rearrange_kv_kernel<<<dim3((unsigned)(g.n_kvh * (g.seq / 64))), dim3(256), 0, st>>>(g.seq, (const uint16_t*)k, g.sk,
                                                                                    (const uint16_t*)v, g.sv, kp, vp,
                                                                                    w.slot_counter);
  if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  const bool qk8 = (p->flags & SALE_FLAG_ATTN_INT8_QK) != 0;
  const bool pv8 = (p->flags & SALE_FLAG_ATTN_FP8_PV) != 0;      // (validated: only with qk8 and 64-key blocks)
  Qk8 q8o = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  if (qk8) {
    const Int8Operands w8i = carve_int8_operands(p, (void*)w.ops8);
    int rc = launch_int8_operands(p, q, k, w8i, true, st);
    if (rc != SALE_OK) return rc;
    q8o = {w8i.q8, (const u32x4*)w8i.k8, w8i.q_scale, w8i.k_scale, w8i.k_mean, nullptr, nullptr};
    if (pv8) {
      const Fp8Operands w8 = carve_fp8_operands(p, (void*)w.ops_fp8);
      rc = launch_fp8_operands(p, v, w8, true, st);
      if (rc != SALE_OK) return rc;
      q8o.v8p = (const u32x4*)w8.v8;
      q8o.v_scale = w8.v_scale;
    }
  }
  const uint16_t* qq = (const uint16_t*)q;
  const bf16x8 *kpp = (const bf16x8*)kp, *vpp = (const bf16x8*)vp;
  if (mask) {
#define SALE_SPARSE_ARGS g, qq, kpp, vpp, q8o, mask, row_counts, order, assign, w.load, w.slot_of, w.slot_counter, n_slots, \
                         (uint16_t*)o, o32, lse, st_o, st_ml, st
    if (g.bk == 32) return qk8 ? launch_sparse_rows<true, true>(SALE_SPARSE_ARGS) : launch_sparse_rows<true, false>(SALE_SPARSE_ARGS);
    if (pv8) return launch_sparse_rows<false, true, true>(SALE_SPARSE_ARGS);
    return qk8 ? launch_sparse_rows<false, true>(SALE_SPARSE_ARGS) : launch_sparse_rows<false, false>(SALE_SPARSE_ARGS);
#undef SALE_SPARSE_ARGS
  }
  const int units = g.n_qb * g.group;
  const RowFilter all = {nullptr, -1, 0, -1, 0, 0};
  const dim3 grid((unsigned)(((units + 3) / 4) * g.n_kvh));
  if (pv8)
    attn_rows_kernel<4, false, true, true><<<grid, dim3(256), 0, st>>>(g, qq, kpp, vpp, q8o, nullptr, nullptr, nullptr, (uint16_t*)o,
                                                                      o32, lse, all, nullptr, nullptr);
  else if (qk8)
    attn_rows_kernel<4, false, true><<<grid, dim3(256), 0, st>>>(g, qq, kpp, vpp, q8o, nullptr, nullptr, nullptr, (uint16_t*)o, o32,
                                                                lse, all, nullptr, nullptr);
  else
    attn_rows_kernel<4, false, false><<<grid, dim3(256), 0, st>>>(g, qq, kpp, vpp, q8o, nullptr, nullptr, nullptr, (uint16_t*)o, o32,
                                                                 lse, all, nullptr, nullptr);
  return hipGetLastError() == hipSuccess ? SALE_OK : SALE_ERR_HIP;
}

}  // namespace sale

using namespace sale;

extern "C" int sale_sparse_attn(const sale_params_t* p, const void* q, const void* k, const void* v,
                                const uint64_t* block_mask, const int32_t* row_counts, void* o, float* lse, void* ws,
                                size_t ws_bytes, void* stream) {
  if (!p || !q || !k || !v || !block_mask || !o) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  // (any size from SALE_WS_SPARSE_ATTN_MIN on: what lies beyond the fixed part holds parking slots)
  const size_t need = sale_workspace_bytes(p, SALE_WS_SPARSE_ATTN_MIN);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  return launch_attn_rows(p, q, k, v, block_mask, row_counts, o, nullptr, lse, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int sale_dense_attn(const sale_params_t* p, const void* q, const void* k, const void* v, void* o, float* lse,
                               void* ws, size_t ws_bytes, void* stream) {
  if (!p || !q || !k || !v || !o) return SALE_ERR_NULL_ARG;
  int rc = validate_common(p, kGeomPath);
  if (rc != SALE_OK) return rc;
  const size_t need = sale_workspace_bytes(p, SALE_WS_DENSE_ATTN);
  if (!ws || ws_bytes < need || ((uintptr_t)ws & 15)) return SALE_ERR_WORKSPACE;
  return launch_attn_rows(p, q, k, v, nullptr, nullptr, o, nullptr, lse, ws, ws_bytes, (hipStream_t)stream);
}
