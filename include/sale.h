/*
 * sale.h - C ABI of the MI355X (gfx950) implementation of SALE's prefill
 * attention path (arXiv 2505.24179):
 *
 *   quantize Q,K to 4 bit  ->  Selection-Pass (block mask)  ->  Computation-Pass
 *   (block-sparse causal attention), plus a dense causal kernel of the same
 *   design used as the speed-up denominator.
 *
 * Conventions shared by every call
 * --------------------------------
 * - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *   never allocates or frees memory.  Scratch comes from a caller-provided
 *   workspace (16-byte aligned) whose size sale_workspace_bytes() reports.
 * - Calls are asynchronous on the given hipStream_t (passed as void*; NULL =
 *   the default stream), never synchronise (sale_calibrate_tau excepted) and
 *   keep no global state (sale_select_static excepted: its scratch memory is a
 *   static device array of the library).
 * - Q, K, V and O are addressed through element strides (sale_params_t):
 *     Q, O : bf16 (batch, n_q_heads,  seq_len, head_dim)
 *     K, V : bf16 (batch, n_kv_heads, seq_len, head_dim)
 *   element (b, h, t, c) of X lies at  x + b * x_stride[0] + h * x_stride[1] +
 *   t * x_stride[2] + c  (the last dimension is always contiguous), so both the
 *   [batch][head][token][d] layout and the [batch][token][head][d] layout of a
 *   projection output are read and written in place.  A stride triple that is
 *   all zero means contiguous [batch][heads][seq_len][head_dim].  Strides are
 *   non-negative multiples of 8 elements (16-byte rows), the token stride at
 *   least head_dim; rows must not overlap.  Every OTHER tensor (codes, scales,
 *   masks, counts, statistics, lse) is contiguous, row-major, in the layout
 *   stated at its call.
 *   Query head h reads KV head h / (n_q_heads / n_kv_heads)  (GQA).
 * - Return value: SALE_OK (0) or a negative sale_status.  Arguments are checked
 *   before anything is launched; a failed check launches nothing.
 * - Supported geometry: head_dim = 128; block_q = 64; block_k = 64, or 32
 *   (the paper's shape, Sec. 4.1) in every call (the dense kernel does not
 *   depend on it); seq_len a multiple of 64 and at most 4096 key
 *   blocks; n_q_heads a multiple of n_kv_heads.  (sale_quantize_qk alone also
 *   accepts block_q = 32.)  Anything else returns SALE_ERR_UNSUPPORTED.
 *   A sequence whose length is not a multiple of 64 is passed zero-padded to
 *   the next multiple: attention is causal, so no valid query row ever sees a
 *   padded key and the outputs of the valid rows are those of the unpadded
 *   sequence under the returned mask; only the mask row of the last query
 *   block is then chosen with its padded (all-zero) query rows taking part, and
 *   the statistics of its valid rows see the padded keys of the diagonal block
 *   unless SALE_FLAG_STATS_CAUSAL is set.
 *
 * Notation follows the paper: N = seq_len, d = head_dim, b_q / b_k block sizes,
 * N_q = N / b_q, N_k = N / b_k, M_bs the block-level sparse mask (Sec. 3.1),
 * m~ / l~ the sink-local statistics and tau the threshold (Sec. 3.2).
 */
#ifndef SALE_H_
#define SALE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sale_status {
  SALE_OK = 0,
  SALE_ERR_NULL_ARG = -1,     /* a required pointer is NULL                       */
  SALE_ERR_BAD_SHAPE = -2,    /* non-positive size, N not a multiple of the block */
  SALE_ERR_UNSUPPORTED = -3,  /* valid but not implemented geometry / flag        */
  SALE_ERR_WORKSPACE = -4,    /* workspace NULL, misaligned or smaller than required */
  SALE_ERR_HIP = -5           /* a HIP runtime call or kernel launch failed       */
} sale_status;

/* The sink-local statistics see only keys at or before each query row.  Default
 * (flag clear) follows Alg. 1's comment: the statistics ignore the causal mask
 * inside the sink-local blocks. */
#define SALE_FLAG_STATS_CAUSAL 1u
/* sale_select estimates the attention weights of the middle blocks from the 16-bit Q, K instead of the
 * 4-bit codes (the "w/o QK Quant" ablation of Appendix E); q4, k4 and the scales are then unused and may
 * be NULL. */
#define SALE_FLAG_SELECT_16BIT 2u
/* Segment rule for the local area (Appendix C): the middle key blocks of a row (those after the sink
 * blocks) are taken in segments of 4; the fewer-than-4 blocks left over before the local_blocks
 * diagonal-side blocks join the local area, i.e. with j_last the last causally visible key block
 *   local(i) = local_blocks + max(0, j_last + 1 - sink_blocks - local_blocks) mod 4.
 * They are always kept and feed the statistics like the other local blocks. */
#define SALE_FLAG_SEGMENT_LOCAL 4u
/* Quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention"): sale_sparse_attn, sale_dense_attn and
 * the sparse leg of sale_calibrate_tau take the attention weights from 8-bit operands,
 *   S = (Q8 K8^T) q_scale8 k_scale8 / sqrt(d),
 * Q8 / K8 the symmetric codes in [-127, 127] of Q and of K minus its head's mean key, one fp32 scale per
 * (head, 64-row block), exact integer products; mask, softmax and the product with V (bf16) are unchanged.
 * The operands are made inside the call (see sale_attn_int8_operands for their definition). */
#define SALE_FLAG_ATTN_INT8_QK 8u
/* Low-precision second product of the quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention"; only
 * together with SALE_FLAG_ATTN_INT8_QK and block_k = 64): V and the probabilities in OCP FP8 E4M3, fp32 accumulation.
 *   V8 = fp8(V * 448 / amax) with amax per (KV head, channel) over all tokens (see sale_attn_fp8_operands);
 *   the kept 64-key blocks of a row are visited in ascending order; with m the row's running maximum after a
 *   block, that block's probabilities are P8 = fp8(448 * exp(S - m)), and
 *   O[r][c] = (amax[c] / 448) * (sum_k P8[r][k] V8[k][c]) / (sum_k P8[r][k]),  lse = m + ln(sum_k P8 / 448),
 *   both sums rescaled by exp(m_old - m_new) whenever m grows.
 * This goes beyond the 16-bit second product of the default pass: every probability and every value of V carries a
 * relative rounding error of up to 2^-4 (they average out over the keys), and the matrix unit adds the 64 products
 * of an instruction with about 2^-14 relative precision.  The codes P8 are decided in fp32 with the hardware exp2:
 * a probability within rounding distance of the midpoint of two codes may take either, which moves lse by at most
 * (that term's share of the row sum) / 8; apart from such rows lse keeps the accuracy stated at sale_sparse_attn. */
#define SALE_FLAG_ATTN_FP8_PV 16u

typedef struct sale_params {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t seq_len;      /* N                                                     */
  int32_t head_dim;     /* d, must be 128                                        */
  int32_t block_q;      /* b_q                                                   */
  int32_t block_k;      /* b_k                                                   */
  int32_t sink_blocks;  /* key blocks at the start of every row that are always
                           kept and feed the statistics (Alg. 1: block 0)        */
  int32_t local_blocks; /* key blocks ending at, and including, the diagonal one
                           that are always kept and feed the statistics          */
  uint32_t flags;       /* SALE_FLAG_*                                           */
  /* element strides of (batch, head, token); all zero = contiguous [batch][heads][N][d] */
  int64_t q_stride[3];
  int64_t k_stride[3];
  int64_t v_stride[3];
  int64_t o_stride[3];
  /* Variable-length batch (optional; n_seqs = 0: every batch entry is one sequence of seq_len tokens).
   * n_seqs > 0 packs n_seqs sequences of different lengths one after the other along the token axis of a
   * batch = 1 call: seq_len is then the TOTAL number of tokens and cu_seqlens, a HOST pointer read during
   * the call, holds n_seqs + 1 ascending token offsets, cu_seqlens[0] = 0, cu_seqlens[n_seqs] = seq_len.
   * Every sequence length is a positive multiple of 64 (pad shorter ones as for a single sequence) and at
   * most 4096 key blocks.  Attention, statistics and selection never cross a sequence boundary: key block j
   * of a mask row is the j-th block OF THAT ROW'S SEQUENCE, and the mask has ceil(longest / (64 b_k)) words
   * per row.  Per-token and per-block tensors (codes, scales, counts, statistics, lse) are indexed by the
   * packed position.  Not combined with SALE_FLAG_ATTN_INT8_QK or sale_calibrate_tau (SALE_ERR_UNSUPPORTED). */
  int32_t n_seqs;
  const int32_t* cu_seqlens;
} sale_params_t;

/* Which call a workspace is for. */
#define SALE_WS_SELECT 1
#define SALE_WS_SPARSE_ATTN 2
#define SALE_WS_DENSE_ATTN 3
#define SALE_WS_CALIBRATE 4
#define SALE_WS_INT8_OPERANDS 5
#define SALE_WS_FP8_OPERANDS 6
/* sale_sparse_attn without parking slots (see there); one slot more per SALE_PARKED_ROW_BYTES. */
#define SALE_WS_SPARSE_ATTN_MIN 7
#define SALE_PARKED_ROW_BYTES 33792u

/* Bytes of workspace `which_call` needs for `p` (0 if the call needs none or the
 * parameters are invalid). */
size_t sale_workspace_bytes(const sale_params_t* p, int which_call);

/* Static description of a status code. */
const char* sale_status_string(int status);

/*
 * Quantization stage (Sec. 3.2 "4-bit attention weight approximation"; inputs
 * Q~, K~ of Alg. 1).  For every block of block_q rows of one Q head (block_k
 * rows of one K head), over all rows*d elements x of the block, in IEEE fp32:
 *   amax = max|x|; scale = amax / 7; code = clamp(rint(x * (7 / amax)), -7, 7)
 * (round half to even; an all-zero block gets scale 1 and codes 0).
 *
 *   q, k     in : bf16, strided as above
 *   q4       out: uint8 [batch][n_q_heads ][N][d/2]; byte c of a row holds channel
 *                 2c in bits 0..3 and channel 2c+1 in bits 4..7 (two's complement)
 *   k4       out: uint8 [batch][n_kv_heads][N][d/2], same packing
 *   q_scale  out: fp32 [batch][n_q_heads ][N / block_q]
 *   k_scale  out: fp32 [batch][n_kv_heads][N / block_k]
 */
int sale_quantize_qk(const sale_params_t* p, const void* q, const void* k,
                     uint8_t* q4, uint8_t* k4, float* q_scale, float* k_scale,
                     void* stream);

/*
 * Selection-Pass (Alg. 1; Eq. 3; Eq. 4; Sec. 3.4 "Reduction in dequantization
 * operations").  For every query head and query block i:
 *   1. I_SL(i) = the first sink_blocks key blocks and the local_blocks key
 *      blocks ending at the diagonal block; those bits are set to 1 and the
 *      statistics m~_r = max S[r,c], l~_r = sum exp(S[r,c] - m~_r) over their
 *      key tokens are taken from the unquantized Q, K (S = Q K^T / sqrt(d)).
 *   2. every other causally visible key block j is kept iff some row r has
 *      max_c  A[r,c] * q_scale[i] * k_scale[j] / sqrt(d)  >=  ln(tau * l~_r) + m~_r,
 *      A = Q~_i K~_j^T in exact integer arithmetic (the log form of
 *      "max relative attention score >= tau").
 *   3. key blocks past the diagonal are 0.
 *
 *   tau         in : fp32, DEVICE pointer, tau_len = 1 (shared) or n_q_heads
 *   block_mask  out: uint64 [batch][n_q_heads][N_q][ceil(N_k/64)]; bit (j mod 64)
 *                    of word j/64 is M_bs[i][j]  (variable-length batches: N_k of
 *                    the longest sequence, j counted inside the row's sequence)
 *   row_counts  out: int32 [batch][n_q_heads][N_q], number of kept blocks per row
 *   m_out,l_out out: optional (may be NULL) fp32 [batch][n_q_heads][N]: m~, l~
 *   ws             : workspace of sale_workspace_bytes(p, SALE_WS_SELECT) bytes
 */
int sale_select(const sale_params_t* p, const void* q, const void* k,
                const uint8_t* q4, const uint8_t* k4,
                const float* q_scale, const float* k_scale,
                const float* tau, int32_t tau_len,
                uint64_t* block_mask, int32_t* row_counts,
                float* m_out, float* l_out,
                void* ws, size_t ws_bytes, void* stream);

/*
 * sale_select for callers that cannot allocate device memory or own a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and checks as sale_select, without the
 * workspace: the scratch memory is a static device array inside the library,
 * SALE_SELECT_STATIC_MAX_BYTES large, that every GPU the library runs on holds
 * until the process ends.  The call allocates and frees nothing.
 * - Geometries whose sale_workspace_bytes(p, SALE_WS_SELECT) exceeds
 *   SALE_SELECT_STATIC_MAX_BYTES return SALE_ERR_WORKSPACE and launch nothing
 *   (64 MiB covers 32 query / 8 KV heads up to 65536 tokens).
 * - The device whose stream is passed must be the current device.  The first
 *   call on a device looks up that device's copy of the array.
 * - All calls on one GPU share that GPU's array: calls that overlap in time on
 *   one GPU (different streams or threads) race.  Nothing in the array has to
 *   be cleared between calls: every byte a kernel reads is written earlier in
 *   the same call.
 */
#define SALE_SELECT_STATIC_MAX_BYTES (64u << 20)
int sale_select_static(const sale_params_t* p, const void* q, const void* k,
                       const uint8_t* q4, const uint8_t* k4,
                       const float* q_scale, const float* k_scale,
                       const float* tau, int32_t tau_len,
                       uint64_t* block_mask, int32_t* row_counts,
                       float* m_out, float* l_out, void* stream);

/*
 * Computation-Pass (Sec. 3.1, Eq. 1 with the block mask of Eq. 2):
 *   O = Softmax(Q K^T / sqrt(d) + M_c + M_s) V, computed only on the key blocks
 * whose bit is set in block_mask (bf16 operands, fp32 accumulation and softmax).
 * A query block whose diagonal bit is clear would leave rows without any key;
 * the Selection-Pass never produces that, and for such rows O is 0 and lse -inf.
 *
 *   block_mask in : layout of sale_select
 *   row_counts in : optional (may be NULL) per-row kept-block counts, used only
 *                   to order work
 *   o          out: bf16, strided by o_stride
 *   lse        out: optional (may be NULL) fp32 [batch][n_q_heads][N], natural-log
 *                   sum-exp of the kept logits S[r,c] = q_r . k_c / sqrt(d) of each row
 *                   (Sec. 3.1).  Accuracy: within 5e-3 absolute of the exact value.
 *                   The kernel sums the probabilities AFTER rounding them to bf16
 *                   (the values it multiplies with V, so that numerator and
 *                   denominator of O agree); bf16 keeps 8 significant bits, so
 *                   the sum is within 2^-8 relative and its logarithm within
 *                   3.9e-3.  A caller that merges partial results by lse
 *                   inherits that 2^-8 relative weight error.  With
 *                   SALE_FLAG_ATTN_INT8_QK the logits are the 8-bit estimates;
 *                   the per-row shift q_r . k_mean / sqrt(d) that the K smoothing
 *                   takes out is added back, so lse still refers to S above.
 *   ws            : workspace (K and V are copied into it once per call in the
 *                   kernel's operand order, 2 * sizeof(K) bytes; tables; then parking
 *                   slots).  Any ws_bytes >= sale_workspace_bytes(p, SALE_WS_SPARSE_ATTN_MIN)
 *                   is accepted.  Above 16K tokens, rows keeping more than 192 x 64 keys
 *                   are swept window by window (so that a window of K, V stays in L2)
 *                   with their accumulators parked in a slot of SALE_PARKED_ROW_BYTES
 *                   in between; the slots are what lies beyond the MIN size.  A long
 *                   row that finds no slot is swept in one go instead: the same result
 *                   bit for bit, slower.  SALE_WS_SPARSE_ATTN is the size with one slot
 *                   per 64-row block (never short of slots); a caller that knows how
 *                   many rows of row_counts exceed 192 x (64 / block_k) passes
 *                   MIN + that many * SALE_PARKED_ROW_BYTES.
 */
int sale_sparse_attn(const sale_params_t* p, const void* q, const void* k, const void* v,
                     const uint64_t* block_mask, const int32_t* row_counts,
                     void* o, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Dense causal attention (Eq. 1 with M = M_c): the same kernel with every
 * causally visible block kept.  The denominator of every reported speed-up.
 *   ws : workspace of sale_workspace_bytes(p, SALE_WS_DENSE_ATTN) bytes
 */
int sale_dense_attn(const sale_params_t* p, const void* q, const void* k, const void* v,
                    void* o, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Parity hook: the exact integer products of the Selection-Pass,
 *   out[r][c] = sum_t Q~[q_block*b_q + r][t] * K~[k_block_begin*b_k + c][t]
 * for one (batch*head) index `q_head` (flattened batch*n_q_heads), computed
 * with the same matrix instructions and operand handling the Selection-Pass
 * uses.  out: int32 [b_q][(k_block_end - k_block_begin) * b_k].
 */
int sale_qk_int4_products(const sale_params_t* p, const uint8_t* q4, const uint8_t* k4,
                          int32_t q_head, int32_t q_block,
                          int32_t k_block_begin, int32_t k_block_end,
                          int32_t* out, void* stream);

/*
 * Parity hook: the 8-bit operands of the quantized Computation-Pass (SALE_FLAG_ATTN_INT8_QK), made by the
 * kernels the attention calls use.  Per KV head, k_mean[c] = fp32(exact sum over the N keys of channel c / N);
 * K' = K - k_mean in fp32; then for every 64-row block of a Q head (of K' of a KV head), in IEEE fp32:
 *   amax = max|x|; scale = amax / 127; code = clamp(rint(x * (127 / amax)), -127, 127)
 * (round half to even; an all-zero block gets scale 1 and codes 0).
 *
 *   q8        out: int8 [batch][n_q_heads ][N][d]
 *   k8        out: int8 [batch][n_kv_heads][N][d]
 *   q_scale8  out: fp32 [batch][n_q_heads ][N / 64]
 *   k_scale8  out: fp32 [batch][n_kv_heads][N / 64]
 *   k_mean    out: fp32 [batch][n_kv_heads][d]
 *   ws           : workspace of sale_workspace_bytes(p, SALE_WS_INT8_OPERANDS) bytes
 */
int sale_attn_int8_operands(const sale_params_t* p, const void* q, const void* k,
                            int8_t* q8, int8_t* k8, float* q_scale8, float* k_scale8, float* k_mean,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * Parity hook: the FP8 operand of the low-precision second product (SALE_FLAG_ATTN_FP8_PV), made by the kernels the
 * attention calls use.  Per (KV head, channel c), in IEEE fp32:
 *   amax = max over the N tokens of |v|; v_scale = amax / 448; value = fp8_e4m3(v * (448 / amax))
 * (OCP FP8 E4M3, round to nearest even; an all-zero channel gets scale 1 and values 0).
 *
 *   v8       out: uint8 [batch][n_kv_heads][N][d] bit patterns (sign, 4 exponent bits, 3 mantissa bits)
 *   v_scale  out: fp32 [batch][n_kv_heads][d]
 *   ws          : workspace of sale_workspace_bytes(p, SALE_WS_FP8_OPERANDS) bytes
 */
int sale_attn_fp8_operands(const sale_params_t* p, const void* v, uint8_t* v8, float* v_scale,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Per-head threshold calibration (Sec. 3.3).  For every query head, starting from tau0 (the paper uses
 * 0.008), tau is halved until Err(tau) = ||O - O~||_1 / N < theta, where O is full causal attention and
 * O~ the SALE output (Selection-Pass with that tau + Computation-Pass) of the same inputs, both taken in
 * fp32 before the output rounding; at most max_halvings halvings (0..64).  With batch > 1 the batch
 * entries are calibration samples and every one of them has to satisfy the bound (Appendix C).
 * This is an offline procedure: unlike the other calls it SYNCHRONISES `stream` (once per round) and
 * uses host memory for Hq-sized bookkeeping.
 *
 *   tau_out      out: fp32 [n_q_heads] (device), the calibrated thresholds
 *   err_out      out: optional fp32 [n_q_heads] (device), Err at the returned tau (worst sample)
 *   halvings_out out: optional int32 [n_q_heads] (device), number of halvings taken
 *   ws              : workspace of sale_workspace_bytes(p, SALE_WS_CALIBRATE) bytes, 256-byte aligned
 */
int sale_calibrate_tau(const sale_params_t* p, const void* q, const void* k, const void* v,
                       float tau0, float theta, int32_t max_halvings,
                       float* tau_out, float* err_out, int32_t* halvings_out,
                       void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SALE_H_ */
