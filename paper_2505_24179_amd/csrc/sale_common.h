// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sale.h"

namespace sale {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kHeadDim = 128;   // d
constexpr int kBlockQ = 64;     // b_q
constexpr int kBlockK = 64;     // b_k of the Computation-Pass (the Selection-Pass also takes 32)
constexpr int kSegmentBlocks = 4;            // key blocks per segment (Appendix C)
constexpr int kMaskWordsMax = 64;            // longest mask row, in 64-bit words
constexpr int kMaxSeqLen = kMaskWordsMax * 64 * kBlockK;   // 262144 tokens (131072 with b_k = 32)

// How one of Q, K, V, O is laid out: element (flat head f = b * heads + h, token t, channel c) lies at
// (f / heads) * sb + (f % heads) * sh + t * st + c.
struct Strided {
  long long sb, sh, st;
  int heads;
};
__host__ __device__ __forceinline__ size_t row_off(const Strided& s, int flat_head, int token) {
  return (size_t)(flat_head / s.heads) * (size_t)s.sb + (size_t)(flat_head % s.heads) * (size_t)s.sh +
         (size_t)token * (size_t)s.st;
}

// Flattened geometry handed to kernels.
struct Geo {
  int n_qh;        // batch * n_q_heads
  int n_kvh;       // batch * n_kv_heads
  int hq_per_b;    // n_q_heads (to index tau)
  int group;       // n_q_heads / n_kv_heads
  int seq;         // N
  int n_qb;        // N / 64
  int bk;          // b_k: 64 or 32
  int n_kb;        // N / b_k
  int words;       // ceil(n_kb / 64)
  int sink_blocks;
  int local_blocks;
  int seg;         // segment size in key blocks (0 = no segment rule for the local area)
  int stats_causal;
  Strided sq, sk, sv, so;   // layouts of Q, K, V, O
  // Variable-length batch: [n_qb] first 64-row block of the sequence that block i belongs to (device), or
  // nullptr when every (batch, head) is one sequence.  n_qb, n_kb, seq then count the packed total and
  // `words` the mask words of the longest sequence.
  const int32_t* seq_start;
};

// Query block i of the packed token axis -> (its index inside its sequence, first key block of that sequence).
struct SeqPos { int il, kb0; };
__device__ __forceinline__ SeqPos seq_pos(const Geo& g, int i) {
  const int s0 = g.seq_start ? g.seq_start[i] : 0;
  SeqPos r;
  r.il = i - s0;
  r.kb0 = s0 * (kBlockQ / g.bk);
  return r;
}

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __builtin_bit_cast(float, (unsigned)b << 16);
}

// Accumulator register r of lane `lane` in a 32x32 MFMA tile holds row
// 8*(r/4) + 4*(lane/32) + r%4 of column lane%32.
__device__ __forceinline__ int mfma32_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Value held by the other half of the wave (lane ^ 32).
__device__ __forceinline__ float swap_half(float x) { return __shfl_xor(x, 32, 64); }

// Reads an integer register as a float.  The empty statement hides the value's origin from the optimizer: with
// this compiler, float arithmetic on elements 1.. of an integer vector that an intrinsic returned and that is
// reinterpreted as floats was folded away as if those elements were NaN (only element 0 survived a maximum).
__device__ __forceinline__ float int_bits_as_float(int x) {
  asm("" : "+v"(x));
  return __builtin_bit_cast(float, x);
}

// max(x, x of lane ^ 32) without going through LDS: v_permlane32_swap exchanges the upper 32 lanes of its
// first register with the lower 32 lanes of its second, so with x in both it leaves the lower half's values in
// both halves of one register and the upper half's in the other.  Written as inline assembly on purpose: through
// the builtin the compiler kept the instruction but dropped the maximum of the two results (it used the first
// alone), which went unnoticed as long as every consumer only needed SOME common reference value per row.
// (s_nop 1: the wait states the instruction needs after the VALU write of its operands.)
__device__ __forceinline__ float max_with_other_half(float x) {
  float lo = x, hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
  return fmaxf(lo, hi);
}

// Unit = (flattened query head, 64-row query block): the work of one wave.
// Units of one KV head are numbered block-major, head-in-group minor, so the
// four waves of a workgroup share their K (and V) rows.  Workgroups are dealt
// round-robin over KV heads (one KV head per XCD / L2 when there are 8) and
// longest rows first.
struct Unit {
  int kvh;     // flattened batch * kv head
  int qh;      // flattened batch * q head
  int i;       // query block
  bool valid;  // false for the padding waves of the last workgroup
};

__device__ __forceinline__ Unit unit_of(const Geo& g, int block, int wave) {
  const int units = g.n_qb * g.group;
  const int tiles = (units + 3) / 4;
  Unit u;
  u.kvh = block % g.n_kvh;
  const int t = tiles - 1 - block / g.n_kvh;
  const int id = t * 4 + wave;
  u.valid = id < units;
  u.i = u.valid ? id / g.group : 0;
  u.qh = u.kvh * g.group + (u.valid ? id % g.group : 0);
  return u;
}

// Which geometry a call accepts: any mix of 32 / 64 (quantization alone), b_q = 64 with b_k = 64 or 32
// and at most 4096 key blocks (everything else).
enum GeomClass { kGeomQuantize, kGeomPath };
int validate_common(const sale_params_t* p, GeomClass cls);
// attention launcher shared by the attention entry points and the calibration (attention.hip)
int launch_attn_rows(const sale_params_t* p, const void* q, const void* k, const void* v, const uint64_t* mask,
                     const int32_t* row_counts, void* o, float* o32, float* lse, void* ws, size_t ws_bytes, hipStream_t st);
// Bytes of an attention workspace without parking slots (sparse) / of the dense kernel's workspace.
size_t attn_fixed_bytes(const sale_params_t* p, bool sparse);
constexpr size_t kParkedRowBytes = 2048 * 16 + 256 * 4;      // fp32 O^T accumulators + running max / sum of one row block
Geo make_geo(const sale_params_t* p);
// Variable-length batches: bytes of the per-block sequence table at the end of a workspace (0 without one), and
// the kernel launches that fill it from the host offsets.
size_t seq_table_bytes(const sale_params_t* p);
int build_seq_table(const sale_params_t* p, int32_t* table, hipStream_t st);
size_t calibrate_workspace_bytes(const sale_params_t* p);

// 8-bit operands of the quantized Computation-Pass (quantize8.hip).
struct Int8Operands {
  int8_t* q8;        // [q head][N][128] codes, row-major
  int8_t* k8;        // codes of the smoothed K: MFMA fragment order (attention) or row-major (parity hook)
  float* q_scale;    // [q head][N / 64]
  float* k_scale;    // [kv head][N / 64]
  float* k_mean;     // [kv head][128]
  double* partial;   // [kv head][N / 64][128] column sums per tile
};
// FP8 V of the low-precision second product (quantize8.hip).
struct Fp8Operands {
  uint8_t* v8;       // values: MFMA fragment order (attention) or row-major (parity hook)
  float* v_scale;    // [kv head][128]
  float* v_inv;      // [kv head][128]: 448 / amax
  float* partial;    // [kv head][N / 64][128] per-tile maxima
};
size_t fp8_operand_bytes(const sale_params_t* p);
Fp8Operands carve_fp8_operands(const sale_params_t* p, void* base);
int launch_fp8_operands(const sale_params_t* p, const void* v, const Fp8Operands& w, bool frag, hipStream_t st);
size_t int8_operand_bytes(const sale_params_t* p);
Int8Operands carve_int8_operands(const sale_params_t* p, void* base);
int launch_int8_operands(const sale_params_t* p, const void* q, const void* k, const Int8Operands& w, bool frag_k,
                         hipStream_t st);

}  // namespace sale
