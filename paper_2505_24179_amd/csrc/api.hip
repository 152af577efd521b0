// Argument validation, geometry and the small query entry points of the C ABI.
#include "sale_common.h"

namespace sale {

int validate_common(const sale_params_t* p, GeomClass cls) {
  if (p->batch <= 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->seq_len <= 0) return SALE_ERR_BAD_SHAPE;
  if (p->block_q <= 0 || p->block_k <= 0) return SALE_ERR_BAD_SHAPE;
  if (p->seq_len % p->block_q != 0 || p->seq_len % p->block_k != 0) return SALE_ERR_BAD_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return SALE_ERR_BAD_SHAPE;
  if (p->sink_blocks < 0 || p->local_blocks < 1) return SALE_ERR_BAD_SHAPE;
  if (p->head_dim != kHeadDim) return SALE_ERR_UNSUPPORTED;
  if (p->flags & ~(SALE_FLAG_STATS_CAUSAL | SALE_FLAG_SELECT_16BIT | SALE_FLAG_SEGMENT_LOCAL | SALE_FLAG_ATTN_INT8_QK | SALE_FLAG_ATTN_FP8_PV)) return SALE_ERR_UNSUPPORTED;
  if ((p->block_q != 32 && p->block_q != 64) || (p->block_k != 32 && p->block_k != 64)) return SALE_ERR_UNSUPPORTED;
  if (p->n_seqs < 0 || (p->n_seqs > 0 && !p->cu_seqlens)) return SALE_ERR_BAD_SHAPE;
  int longest = p->seq_len;
  if (p->n_seqs > 0) {
    if (p->batch != 1 || p->cu_seqlens[0] != 0 || p->cu_seqlens[p->n_seqs] != p->seq_len) return SALE_ERR_BAD_SHAPE;
    longest = 0;
    for (int s = 0; s < p->n_seqs; ++s) {
      const int len = p->cu_seqlens[s + 1] - p->cu_seqlens[s];
      if (len <= 0 || len % 64 != 0) return SALE_ERR_BAD_SHAPE;
      longest = len > longest ? len : longest;
    }
    if (p->flags & SALE_FLAG_ATTN_INT8_QK) return SALE_ERR_UNSUPPORTED;
  }
  // the FP8 second product belongs to the fully quantized pass (8-bit first product) on 64-key blocks
  if ((p->flags & SALE_FLAG_ATTN_FP8_PV) && (!(p->flags & SALE_FLAG_ATTN_INT8_QK) || p->block_k != kBlockK))
    return SALE_ERR_UNSUPPORTED;
  if (cls != kGeomQuantize) {
    if (p->block_q != kBlockQ) return SALE_ERR_UNSUPPORTED;
    if (longest / p->block_k > kMaskWordsMax * 64) return SALE_ERR_UNSUPPORTED;
  }
  // strides: all zero (contiguous) or non-negative multiples of 8 elements with whole rows apart
  const int64_t* triples[4] = {p->q_stride, p->k_stride, p->v_stride, p->o_stride};
  const int heads_of[4] = {p->n_q_heads, p->n_kv_heads, p->n_kv_heads, p->n_q_heads};
  for (int x = 0; x < 4; ++x) {
    const int64_t* st = triples[x];
    if (st[0] == 0 && st[1] == 0 && st[2] == 0) continue;
    for (int e = 0; e < 3; ++e)
      if (st[e] < 0 || (st[e] & 7)) return SALE_ERR_BAD_SHAPE;
    if (st[2] < p->head_dim) return SALE_ERR_BAD_SHAPE;
    if ((heads_of[x] > 1 && st[1] == 0) || (p->batch > 1 && st[0] == 0)) return SALE_ERR_BAD_SHAPE;
  }
  // 32-bit index guards used by the kernels
  if ((long)p->batch * p->n_q_heads * (long)(p->seq_len / 32) > 0x7FFFFFFFL) return SALE_ERR_UNSUPPORTED;
  return SALE_OK;
}

Geo make_geo(const sale_params_t* p) {
  Geo g;
  g.n_qh = p->batch * p->n_q_heads;
  g.n_kvh = p->batch * p->n_kv_heads;
  g.hq_per_b = p->n_q_heads;
  g.group = p->n_q_heads / p->n_kv_heads;
  g.seq = p->seq_len;
  g.n_qb = p->seq_len / kBlockQ;
  g.bk = p->block_k;
  g.n_kb = p->seq_len / p->block_k;
  int longest = p->seq_len;
  if (p->n_seqs > 0) {
    longest = 0;
    for (int s = 0; s < p->n_seqs; ++s) longest = max(longest, p->cu_seqlens[s + 1] - p->cu_seqlens[s]);
  }
  g.words = (longest / p->block_k + 63) / 64;
  g.seq_start = nullptr;
  g.sink_blocks = p->sink_blocks;
  g.local_blocks = p->local_blocks;
  g.seg = (p->flags & SALE_FLAG_SEGMENT_LOCAL) ? kSegmentBlocks : 0;
  g.stats_causal = (p->flags & SALE_FLAG_STATS_CAUSAL) ? 1 : 0;
  auto layout = [&](const int64_t* st, int heads) {
    Strided s;
    s.heads = heads;
    if (st[0] == 0 && st[1] == 0 && st[2] == 0) {
      s.st = kHeadDim; s.sh = (long long)p->seq_len * kHeadDim; s.sb = s.sh * heads;
    } else {
      s.sb = st[0]; s.sh = st[1]; s.st = st[2];
    }
    return s;
  };
  g.sq = layout(p->q_stride, p->n_q_heads);
  g.sk = layout(p->k_stride, p->n_kv_heads);
  g.sv = layout(p->v_stride, p->n_kv_heads);
  g.so = layout(p->o_stride, p->n_q_heads);
  return g;
}

size_t seq_table_bytes(const sale_params_t* p) {
  return p->n_seqs > 0 ? (((size_t)(p->seq_len / kBlockQ) * sizeof(int32_t) + 15) & ~(size_t)15) : 0;
}

namespace {

// Up to kSeqChunk sequences per launch travel as kernel arguments (copied at launch: no host buffer has to
// outlive the call, nothing is staged or synchronised).
constexpr int kSeqChunk = 255;
struct SeqChunk {
  int n;
  int start_blk[kSeqChunk + 1];      // first 64-row block of every sequence of the chunk, and the end of the last
};

__global__ __launch_bounds__(256) void seq_table_kernel(SeqChunk c, int32_t* __restrict__ table) {
  const int b = c.start_blk[0] + blockIdx.x * 256 + threadIdx.x;
  if (b >= c.start_blk[c.n]) return;
  int lo = 0, hi = c.n;              // the sequence s with start_blk[s] <= b < start_blk[s + 1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (c.start_blk[mid] <= b) lo = mid; else hi = mid;
  }
  table[b] = c.start_blk[lo];
}

}  // namespace

int build_seq_table(const sale_params_t* p, int32_t* table, hipStream_t st) {
  for (int s0 = 0; s0 < p->n_seqs; s0 += kSeqChunk) {
    SeqChunk c;
    c.n = min(kSeqChunk, p->n_seqs - s0);
    for (int e = 0; e <= c.n; ++e) c.start_blk[e] = p->cu_seqlens[s0 + e] / kBlockQ;
    const int blocks = c.start_blk[c.n] - c.start_blk[0];
    seq_table_kernel<<<dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, st>>>(c, table);
    if (hipGetLastError() != hipSuccess) return SALE_ERR_HIP;
  }
  return SALE_OK;
}

}  // namespace sale

using namespace sale;

extern "C" size_t sale_workspace_bytes(const sale_params_t* p, int which_call) {
  if (!p || validate_common(p, kGeomPath) != SALE_OK) return 0;
  const size_t rows = (size_t)p->batch * p->n_q_heads * p->seq_len;
  switch (which_call) {
    case SALE_WS_SELECT:
      // thr_r = ln(tau l~_r) + m~_r per query row, and the FP6 operand copy of K~ (96 B per row)
      return rows * sizeof(float) + (size_t)p->batch * p->n_kv_heads * p->seq_len * 96 + seq_table_bytes(p);
    case SALE_WS_SPARSE_ATTN:
      // K and V copied once into MFMA fragment order, the order in which rows are issued, the tables (one per
      // window launch, at most 32) that balance them over the XCDs, the 8-bit operand copies of the quantized
      // Computation-Pass - and one parking slot (fp32 O^T accumulators and max / sum per lane: 33 KB) per 64-row block
      return attn_fixed_bytes(p, true) + (rows / kBlockQ) * kParkedRowBytes;
    case SALE_WS_SPARSE_ATTN_MIN:      // the same without parking slots
      return attn_fixed_bytes(p, true);
    case SALE_WS_DENSE_ATTN:           // K', V' (+ the 8-bit operand copies)
      return attn_fixed_bytes(p, false);
    case SALE_WS_CALIBRATE:
      return calibrate_workspace_bytes(p);
    case SALE_WS_INT8_OPERANDS:
      return (size_t)p->batch * p->n_kv_heads * (p->seq_len / 64) * 128 * sizeof(double);
    case SALE_WS_FP8_OPERANDS:      // inverse scales + per-tile maxima
      return (size_t)p->batch * p->n_kv_heads * (1 + p->seq_len / 64) * 128 * sizeof(float);
    default:
      return 0;
  }
}

extern "C" const char* sale_status_string(int status) {
  switch (status) {
    case SALE_OK: return "ok";
    case SALE_ERR_NULL_ARG: return "a required pointer argument is NULL";
    case SALE_ERR_BAD_SHAPE: return "invalid shape (non-positive size, or seq_len / heads not divisible)";
    case SALE_ERR_UNSUPPORTED: return "geometry or flag not supported by this build";
    case SALE_ERR_WORKSPACE: return "workspace missing or too small";
    case SALE_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}
