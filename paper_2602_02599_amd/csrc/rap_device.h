// Shared device-side helpers and the argument blocks of the librap kernels (gfx950 only).
#ifndef RAP_DEVICE_H_
#define RAP_DEVICE_H_

#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>

#include "rap_arith.h"

namespace rap {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxPairs = 64;        // P <= 64  (d_k <= 128)
constexpr int kMaxDv = 128;
constexpr int kMaxGroup = 8;         // query heads per KV head: vector-ALU kernel, fused query rotation, one-call step
constexpr int kMaxGroupWide = 16;    // the same for the matrix-core attention kernels (16 columns per instruction)
constexpr int kSplitQuantum = 128;   // rows_per_split granularity

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// two fp32 -> two bf16 (round to nearest even) in one dword, first argument in the low half
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// eight E4M3 codes (c0: elements 0..3, c1: elements 4..7, lowest byte first) -> eight bf16, exact:
// v_cvt_scalef32_pk_bf16_fp8 turns two codes into two bf16 in one instruction (with a scale of 1.0
// it gives, for every pair of codes, the bits of the conversion to fp32 followed by the rounding
// to bf16, NaN codes included: checked on the device over all 65536 pairs)
__device__ __forceinline__ uint4 widen_e4m3x8(uint32_t c0, uint32_t c1) {
  return make_uint4(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c0, 1.0f, false)),
                    __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c0, 1.0f, true)),
                    __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c1, 1.0f, false)),
                    __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c1, 1.0f, true)));
}

// Angular frequency of compact pair idx = h * P + c: from the caller's table when there is one
// (every entry is valid, 0 means "do not rotate"), else theta^(-2j/D) = 2^(j * (-2 log2(theta) / D))
// at the pair's original index j; false when that index lies outside [0, D/2).
__device__ __forceinline__ bool pair_frequency(const int32_t* keep, const double* pair_freq, double neg2_log2_theta_over_d,
                                               int d_head, int idx, double* f) {
  if (pair_freq != nullptr) {
    *f = pair_freq[idx];
    return true;
  }
  const int j = keep[idx];
  const bool ok = j >= 0 && j < d_head / 2;
  *f = ok ? exp2(static_cast<double>(j) * neg2_log2_theta_over_d) : 0.0;
  return ok;
}

struct AppendArgs {
  const uint16_t* k_new;
  const uint16_t* v_new;
  const int32_t* pos;
  const int32_t* keep;
  const double* pair_freq;          // [H_kv, P] radians per position, or null: theta_j from keep
  const int32_t* block_table;       // paged caches: [B, max_pages], or null
  const float* k_scale;             // fp8 caches: [H_kv] scales of the codes, or null
  const float* v_scale;
  uint8_t* k_scales4;               // 4-bit caches: scale bytes [B, H_kv, cap, 4], or null
  uint8_t* v_scales4;
  int32_t page_shift, n_pages, max_pages;
  uint16_t* k_cache;
  uint16_t* v_cache;
  int32_t batch, n_new, n_kv, d_head, n_pairs, d_v;
  int32_t group;                    // query rows only: heads per row of keep / pair_freq
  int64_t cap;
  double neg2_log2_theta_over_d;    // -2 log2(theta_base) / D, so that theta_j = 2^(j * this)
};

struct DecodeArgs {
  const uint16_t* q;
  const int32_t* q_pos;     // [B] or null: when given, q is un-rotated and is rotated at q_pos[b] first
  const int32_t* keep;      // [H_kv, P] original pair indices (only with q_pos)
  const double* pair_freq;  // [H_kv, P] radians per position, or null: theta_j from keep
  double neg2_log2_theta_over_d;
  int32_t d_head;
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  const int32_t* seq_lens;
  // fp8 caches (null otherwise): per-KV-head scales of the E4M3 codes
  const float* k_scale;
  const float* v_scale;
  // 4-bit caches (null otherwise): k_cache / v_cache hold the code blocks, these the scale bytes,
  // [B, H_kv, cap, 4] each
  const uint8_t* k_scales4;
  const uint8_t* v_scales4;
  // paged caches (block_table null otherwise): pools [n_pages, H_kv, 1 << page_shift, d]
  const int32_t* block_table;   // [B, max_pages]
  int32_t page_shift, n_pages, max_pages;
  // one-call decode step (all null otherwise): the new token of every sequence.  The attention
  // kernel leaves cache row new_pos[b] out of its scan; its first workgroup of each (b, h) rotates
  // the new K row, writes it and the V row into the caches and leaves the token's score and V row
  // as one more partial (slot n_split) for the combining kernel.
  const uint16_t* k_new;    // [B, H_kv, 2P] before rotation
  const uint16_t* v_new;    // [B, H_kv, d_v]
  const int32_t* new_pos;   // [B]
  uint16_t* k_cache_w;
  uint16_t* v_cache_w;
  int32_t direct_out;       // one range and no combining kernel: the attention kernel writes out itself
  // Several query tokens per sequence (n_tok > 1, n_tok * group <= 16; matrix-core kernel only):
  // q is [B, n_tok, H_q, d_k], out [B, n_tok, H_q, d_v], the tokens are the last n_tok rows of
  // their sequence and are already in the cache.  The scan covers the rows in front of them, which
  // every token attends, with the n_tok * group query rows side by side as the columns of the
  // matrix instruction; the causal part among the tokens themselves is added by the combining
  // kernel, which always runs.  "Query row" below is then (b * n_tok + token) * H_q + head.
  int32_t n_tok;
  int32_t all_slots;        // combining kernel: every slot of every query row was written (prefill key ranges)
  int32_t group_inv16;      // ceil(65536 / group): (c * group_inv16) >> 16 == c / group for c < 16
  float* out;          // [B, H_q, d_v]
  float* part_acc;     // [query rows, n_slots, d_v]   un-normalised accumulators
  float* part_ml;      // [query rows, n_slots, 2]     (running max in log2 units, running sum)
  int32_t batch, n_q, n_kv, group, n_pairs, d_k, d_v;
  int32_t max_len, rows_per_split, n_split;
  int32_t n_slots;          // partial slots per query head: n_split, plus one in the decode step
  int32_t lds_wave_bytes;   // matrix-core kernel: LDS slice of one wavefront
  int64_t cap;
  float scale_log2e;   // softmax scale * log2(e): exponentials are taken as exp2
};

struct PrefillArgs {
  const uint16_t* q;        // [B, n_new, H_q, d_k] rotated
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  const int32_t* seq_lens;
  float* out;               // [B, n_new, H_q, d_v]
  // fp8 caches (null otherwise): per-KV-head scales of the E4M3 codes
  const float* k_scale;
  const float* v_scale;
  // paged caches (block_table null otherwise): pools [n_pages, H_kv, 1 << page_shift, d], pages of
  // at least 64 rows so that a staged tile never straddles two of them
  const int32_t* block_table;   // [B, max_pages]
  int32_t page_shift, n_pages, max_pages;
  int32_t batch, n_new, n_q, n_kv, group, d_k, d_v, max_len;
  int32_t tok_per_wg;       // query tokens per workgroup: (64 NQ) / G
  int32_t n_qblk;           // ceil(n_new / tok_per_wg)
  int32_t lds_buf_bytes;    // one K + V tile buffer
  int32_t pad_k, pad_v;     // LDS row padding in bytes (0 or 16)
  int64_t cap;
  float scale_log2e;
  // Key ranges (n_ksplit > 1, for launches whose query blocks alone would not fill the chip): a
  // query block is served by n_ksplit workgroups, each over tiles_per_split 64-row tiles of the
  // rows it sees, which leave partials in the form of the decode kernel's (every slot of every
  // query row is written, an empty range as reference -inf and sum 0); a combining launch follows.
  int32_t n_ksplit;
  int32_t tiles_per_split;
  float* part_acc;          // [B * n_new * H_q, n_ksplit, d_v] un-normalised accumulators
  float* part_ml;           // [B * n_new * H_q, n_ksplit, 2]   (reference in log2 units, sum)
};

// Key ranges per query block of a prefill launch, a function of the shape alone: none while the
// query blocks number at least one and a half per CU or the context is short, else enough for
// about 512 workgroups, none shorter than four tiles.
struct PrefillPlan {
  int tok_per_wg, n_qblk, n_ksplit, tiles_per_split;
};
// Column blocks (of 16 query columns) per wavefront in the prefill kernel: four where the registers
// hold their accumulators, three at d_k > 96 or d_v > 96.  The plan and the kernel's table of
// instantiations both go by these.
constexpr int kPrefillBlocks = 4, kPrefillBlocksWide = 3;
PrefillPlan prefill_plan(int batch, int n_kv, int group, int d_k, int d_v, int n_new, int max_len);

// fp64 -> E4M3 code (finite-only 8-bit float: 4 exponent bits, bias 7, 3 mantissa bits, no
// infinity, S.1111.111 = NaN): nearest value, ties to the even mantissa, magnitudes above 448
// saturate, NaN -> 0x7f.  Two steps that together round once: the fp64 value is first brought to
// fp32 by rounding to odd (truncate towards zero, then set the last mantissa bit if anything was
// cut off), which keeps every fact a later rounding to a format at least two bits shorter needs;
// the conversion instruction of the part then rounds that fp32 to E4M3, nearest-even, subnormal
// codes included.  The instruction agrees with a bit-by-bit software rounding on every fp32
// pattern of magnitude up to 464 (checked exhaustively on the device); above that it no longer
// saturates, hence the clamp to 448 in front of it.
__device__ __forceinline__ uint8_t f64_to_e4m3(double y) {
  if (y != y) return 0x7f;
  return static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_fp8_f32(f64_to_f32_odd_clamped448(y), 0.f, 0, false) & 0xff);
}

// value of one E4M3 code
__device__ __forceinline__ float e4m3_to_f32(uint8_t code) {
  return __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(code), false)[0];
}

// Row of the K / V cache that holds position t of sequence b for KV head h: a row of the dense
// [B, H_kv, cap] arrangement, or, with a block table, of the pool [n_pages, H_kv, page_rows] (a page
// number outside the pool is clamped into it).
__device__ __forceinline__ long long cache_row(const AppendArgs& a, int b, int h, int t) {
  if (a.block_table == nullptr) return (static_cast<long long>(b) * a.n_kv + h) * a.cap + t;
  int pg = a.block_table[static_cast<long long>(b) * a.max_pages + (t >> a.page_shift)];
  pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);
  return ((static_cast<long long>(pg) * a.n_kv + h) << a.page_shift) + (t & ((1 << a.page_shift) - 1));
}

// Index-aware RoPE of the G query rows of KV head h of sequence b, into LDS as bf16 in the
// compact order (Eq. (latent-score): the query side of RoPE(X W~_q) . RoPE(X W~_k)^T).  Same
// arithmetic as the cache append: angle pos * theta^(-2 j / D) with j the ORIGINAL index of the
// kept pair, fp64 throughout, one rounding to bf16, so the rows are bit-identical to what a
// separate rotation kernel storing bf16 would have produced.  A pair whose index lies outside
// [0, D/2) is taken as zero.  Called by every thread of the workgroup; the caller synchronises.
__device__ __forceinline__ void rotate_queries_to_lds(const DecodeArgs& a, int b, int h, int tid, int nthreads,
                                                      uint16_t* s_q) {
  const int P = a.n_pairs, G = a.group;
  const int t = a.q_pos[b];
  for (int e = tid; e < G * P; e += nthreads) {
    const int g = e / P, c = e - g * P;
    const uint16_t* qrow = a.q + (static_cast<long long>(b) * a.n_q + h * G + g) * (2 * P);
    double f;
    uint16_t r0 = 0, r1 = 0;
    if (pair_frequency(a.keep, a.pair_freq, a.neg2_log2_theta_over_d, a.d_head, h * P + c, &f)) {
      const double phi = static_cast<double>(t) * f;
      double sn, cs;
      sincos_f64(phi, &sn, &cs);
      const double x = static_cast<double>(bf16_to_f32(qrow[c]));
      const double y = static_cast<double>(bf16_to_f32(qrow[c + P]));
      r0 = f64_to_bf16_rne(x * cs - y * sn);
      r1 = f64_to_bf16_rne(x * sn + y * cs);
    }
    s_q[g * 2 * P + c] = r0;
    s_q[g * 2 * P + c + P] = r1;
  }
}

// Host side: a kernel that wants more than the default 64 KB of dynamic LDS has its limit raised
// before the launch.  The setting belongs to the (kernel, device) pair, so what has been done is
// remembered per device, one slot per call site (a template instantiation each); a lost race
// between two host threads only repeats the call.
constexpr int kMaxDevicesRemembered = 64;
inline hipError_t raise_lds_limit_impl(const void* kernel, int bytes, std::atomic<int>* done) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) dev = -1;
  const bool remembered = dev >= 0 && dev < kMaxDevicesRemembered;
  if (remembered && done[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && remembered) done[dev].store(bytes, std::memory_order_relaxed);
  return e;
}
#define raise_lds_limit(kernel, bytes)                                \
  ([&]() -> hipError_t {                                              \
    static std::atomic<int> done_[::rap::kMaxDevicesRemembered];      \
    return ::rap::raise_lds_limit_impl((kernel), (bytes), done_);     \
  }())

}  // namespace rap
#endif  // RAP_DEVICE_H_
