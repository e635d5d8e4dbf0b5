// C ABI of librap: host-side validation, split planning and kernel dispatch.  See include/rap.h
// for the contract of every entry point.  Each exported function fills a request record and hands
// it to one of the two shared bodies below (append_impl, decode_impl); nothing here allocates,
// synchronises or keeps state between calls (rap_decode_attn_static remembers, per device, where
// its scratch array lives).
#include <math.h>
#include <string.h>

#include "../../include/rap.h"
#include "rap_device.h"

namespace rap {
hipError_t launch_append(const AppendArgs& a, hipStream_t stream);
hipError_t launch_rope_queries(const AppendArgs& a, hipStream_t stream);
hipError_t launch_decode_valu(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_decode_mfma(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_merge(const DecodeArgs& a, hipStream_t stream);
hipError_t launch_prefill(const PrefillArgs& a, hipStream_t stream);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_stream_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t launch_validate(const int32_t* pos, long long n_pos, long long cap, const int32_t* keep, int n_kv, int n_pairs,
                           int half, const int32_t* seq_lens, int batch, long long max_len, uint32_t* flags, hipStream_t stream);
int mfma_lds_wave_bytes(int d_k, int d_v, bool q8, int cols, bool mx4);
}  // namespace rap

namespace {

constexpr int kCUs = 256;                          // MI355X; what is assumed when no device can be asked
constexpr float kLog2e = 1.4426950408889634f;
constexpr int64_t kInt32Max = 0x7fffffffLL;

bool misaligned(const void* p, uintptr_t bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) != 0; }

rap_status_t hip_status(hipError_t e) { return e == hipSuccess ? RAP_OK : RAP_ERR_HIP; }

rap_status_t check_shape(const rap_shape_t* s) {
  if (!s) return RAP_ERR_NULL;
  if (s->batch < 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->d_head <= 0 || (s->d_head & 1) ||
      s->n_pairs <= 0 || s->d_v <= 0 || s->cache_cap <= 0 || !(s->rope_theta > 0.0))
    return RAP_ERR_SHAPE;
  if (s->n_q_heads % s->n_kv_heads != 0) return RAP_ERR_SHAPE;
  if (s->n_pairs > s->d_head / 2) return RAP_ERR_SHAPE;
  if (s->cache_cap % 8 != 0) return RAP_ERR_SHAPE;
  if (s->n_pairs > rap::kMaxPairs || s->d_v > rap::kMaxDv || s->n_q_heads / s->n_kv_heads > rap::kMaxGroupWide)
    return RAP_ERR_UNSUPPORTED;
  if (s->cache_cap > kInt32Max - 1024 || s->batch > 65535 || s->n_kv_heads > 65535) return RAP_ERR_UNSUPPORTED;
  return RAP_OK;
}

// Exponent of the rotation frequencies: theta_j = 2^(j * this), Eq. (rope).
double neg2_log2_theta_over_d(const rap_shape_t* s) {
  return -2.0 * log2(s->rope_theta) / static_cast<double>(s->d_head);
}

// A rotation needs either the kept pair indices or the caller's frequency table.
bool no_rotation_rule(const rap_shape_t* s, const int32_t* keep_pair_idx) {
  return !keep_pair_idx && !s->pair_inv_freq;
}

struct Plan {
  int rows_per_split;
  int n_split;
  int kernel;   // 1 vector ALU, 2 matrix core
};

// Compute units of the current device, asked once per device (256 on MI355X, which is also the
// answer when no device can be asked: the workspace query is host-only arithmetic).
int device_cus() {
  static std::atomic<int> known[rap::kMaxDevicesRemembered];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= rap::kMaxDevicesRemembered) return kCUs;
  int n = known[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return kCUs;
  known[dev].store(n, std::memory_order_relaxed);
  return n;
}

// Row range per workgroup.  A workgroup whose range starts at or beyond its sequence's length
// exits at once, so ragged batches cost only empty launches.  Measured on MI355X: a workgroup
// should stream for a long time (its fixed cost is a few microseconds), and when the whole job
// fits in one round of resident workgroups their number should be a multiple of the compute
// units.  So: about two workgroups per compute unit when the (b, h) count allows it, ranges never
// shorter than 512 rows nor longer than 4096 (longer ranges only lengthen the tail of a ragged
// batch) - except when that ceiling would leave a second, partly filled round of workgroups
// (more than the chip holds at once, fewer than twice that): then ranges of up to 8192 rows bring
// the job back into a single round of two workgroups per compute unit (cfg4 shape, 4 x 8 slabs of
// 131072 rows: 1024 workgroups of 4096 rows over 768 places took 195 us, 512 of 8192 rows 189 us).
rap_status_t make_plan(const rap_shape_t* s, int64_t max_seq_len, const rap_tuning_t* t, Plan* p) {
  int rps = t ? t->rows_per_split : 0;
  if (rps < 0 || (rps % rap::kSplitQuantum) != 0) return RAP_ERR_SHAPE;
  const int kernel = t ? t->kernel : 0;
  if (kernel < 0 || kernel > 2) return RAP_ERR_SHAPE;
  if (rps == 0) {
    const int cus = device_cus();
    const int64_t slabs = static_cast<int64_t>(s->batch) * s->n_kv_heads;
    int64_t per_slab = slabs > 0 ? (2LL * cus) / slabs : 1;            // ranges per (b, h)
    if (per_slab < 1) per_slab = 1;
    int64_t r = (max_seq_len + per_slab - 1) / per_slab;
    r = (r + rap::kSplitQuantum - 1) / rap::kSplitQuantum * rap::kSplitQuantum;
    const int64_t single_round = r;
    if (r < 512) r = 512;
    if (r > 4096) r = 4096;
    // workgroups the chip holds at once: three per compute unit up to d_k = 96, else two
    const int64_t places = static_cast<int64_t>(cus) * (2 * s->n_pairs <= 96 ? 3 : 2);
    const int64_t n_wg = slabs * ((max_seq_len + r - 1) / r);
    if (n_wg > places && n_wg < 2 * places && single_round <= 8192) r = single_round;
    rps = static_cast<int>(r);
  }
  p->rows_per_split = rps;
  p->n_split = static_cast<int>((max_seq_len + rps - 1) / rps);
  p->kernel = kernel == 0 ? 2 : kernel;
  return RAP_OK;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace = accumulators [B, H_q, n_split + 1, d_v], then (reference, sum) pairs
// [B, H_q, n_split + 1, 2], fp32, each block rounded up to 256 bytes; the extra slot is the new
// token's in the one-call step.
// With n_tok query tokens per sequence there are n_tok times as many query rows.
size_t part_acc_bytes(const rap_shape_t* s, const Plan& p, int n_tok = 1) {
  return align_up(static_cast<size_t>(s->batch) * n_tok * s->n_q_heads * (p.n_split + 1) * s->d_v * sizeof(float), 256);
}
size_t part_ml_bytes(const rap_shape_t* s, const Plan& p, int n_tok = 1) {
  return align_up(static_cast<size_t>(s->batch) * n_tok * s->n_q_heads * (p.n_split + 1) * 2 * sizeof(float), 256);
}
size_t workspace_need(const rap_shape_t* s, const Plan& p, int n_tok = 1) {
  return part_acc_bytes(s, p, n_tok) + part_ml_bytes(s, p, n_tok) + 256;
}

// page_rows a power of two in [32, 65536], table present, logical capacity consistent
rap_status_t check_paging(const rap_shape_t* s, const rap_paging_t* pg, int* shift) {
  if (!pg) return RAP_ERR_NULL;
  if (pg->page_rows < 32 || pg->page_rows > 65536 || (pg->page_rows & (pg->page_rows - 1)) != 0) return RAP_ERR_SHAPE;
  if (pg->n_pages <= 0 || pg->max_pages <= 0) return RAP_ERR_SHAPE;
  if (static_cast<int64_t>(pg->max_pages) * pg->page_rows != s->cache_cap) return RAP_ERR_SHAPE;
  if (s->batch > 0 && !pg->block_table) return RAP_ERR_NULL;
  int sh = 0;
  while ((1 << sh) < pg->page_rows) ++sh;
  *shift = sh;
  return RAP_OK;
}

// ---- append ---------------------------------------------------------------------------------

struct AppendRequest {
  const rap_shape_t* shape = nullptr;
  const rap_paging_t* paging = nullptr;    // paged pools instead of dense caches
  int32_t n_new = 0;
  const void* k_new = nullptr;
  const void* v_new = nullptr;
  const int32_t* pos = nullptr;
  const int32_t* keep_pair_idx = nullptr;
  void* k_cache = nullptr;
  void* v_cache = nullptr;
  bool fp8 = false;                        // caches hold E4M3 codes, scales required
  const float* k_scale = nullptr;
  const float* v_scale = nullptr;
  void* k_scales4 = nullptr;               // 4-bit caches: k_cache / v_cache hold the code blocks, these the scale bytes
  void* v_scales4 = nullptr;
  bool mx4 = false;
  void* stream = nullptr;
};

// Shared body of rap_rope_append and its paged, fp8 and 4-bit variants.
rap_status_t append_impl(const AppendRequest& r) {
  const rap_shape_t* shape = r.shape;
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  int page_shift = 0;
  if (r.paging && (st = check_paging(shape, r.paging, &page_shift)) != RAP_OK) return st;
  if (r.n_new < 0) return RAP_ERR_SHAPE;
  if (r.n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!r.k_new || !r.v_new || !r.pos || no_rotation_rule(shape, r.keep_pair_idx) || !r.k_cache || !r.v_cache)
    return RAP_ERR_NULL;
  if (static_cast<int64_t>(shape->batch) * r.n_new > kInt32Max) return RAP_ERR_UNSUPPORTED;
  if (misaligned(r.k_new, 4) || misaligned(r.v_new, 4) || misaligned(r.k_cache, 4) || misaligned(r.v_cache, 4))
    return RAP_ERR_SHAPE;
  rap::AppendArgs a;
  memset(&a, 0, sizeof(a));
  if (r.paging) {
    a.block_table = r.paging->block_table;
    a.page_shift = page_shift;
    a.n_pages = r.paging->n_pages;
    a.max_pages = r.paging->max_pages;
  }
  if (r.fp8) {
    if (!r.k_scale || !r.v_scale) return RAP_ERR_NULL;
    if (shape->cache_cap % 16 != 0) return RAP_ERR_SHAPE;
    a.k_scale = r.k_scale;
    a.v_scale = r.v_scale;
  }
  if (r.mx4) {
    if (!r.k_scales4 || !r.v_scales4) return RAP_ERR_NULL;
    if (r.paging || r.fp8) return RAP_ERR_UNSUPPORTED;
    if (misaligned(r.k_cache, 16) || misaligned(r.v_cache, 16) || misaligned(r.k_scales4, 4) || misaligned(r.v_scales4, 4))
      return RAP_ERR_SHAPE;
    a.k_scales4 = static_cast<uint8_t*>(r.k_scales4);
    a.v_scales4 = static_cast<uint8_t*>(r.v_scales4);
  }
  a.k_new = static_cast<const uint16_t*>(r.k_new);
  a.v_new = static_cast<const uint16_t*>(r.v_new);
  a.pos = r.pos;
  a.keep = r.keep_pair_idx;
  a.pair_freq = shape->pair_inv_freq;
  a.k_cache = static_cast<uint16_t*>(r.k_cache);
  a.v_cache = static_cast<uint16_t*>(r.v_cache);
  a.batch = shape->batch;
  a.n_new = r.n_new;
  a.n_kv = shape->n_kv_heads;
  a.d_head = shape->d_head;
  a.n_pairs = shape->n_pairs;
  a.d_v = shape->d_v;
  a.group = 1;
  a.cap = shape->cache_cap;
  a.neg2_log2_theta_over_d = neg2_log2_theta_over_d(shape);
  return hip_status(rap::launch_append(a, static_cast<hipStream_t>(r.stream)));
}

// ---- decode attention -------------------------------------------------------------------------

struct DecodeRequest {
  const rap_shape_t* shape = nullptr;
  const rap_paging_t* paging = nullptr;    // paged pools instead of dense caches
  const void* q = nullptr;
  const int32_t* q_pos = nullptr;          // non-null: q arrives un-rotated and is rotated in the prologue
  const int32_t* keep_pair_idx = nullptr;
  const void* k_cache = nullptr;
  const void* v_cache = nullptr;
  bool fp8 = false;                        // caches hold E4M3 codes, scales required
  const float* k_scale = nullptr;
  const float* v_scale = nullptr;
  const void* k_scales4 = nullptr;         // 4-bit caches: k_cache / v_cache hold the code blocks, these the scale bytes
  const void* v_scales4 = nullptr;
  bool mx4 = false;
  const void* k_new = nullptr;             // one-call step: the token to append first (with v_new, new_pos)
  const void* v_new = nullptr;
  const int32_t* new_pos = nullptr;
  int32_t n_tok = 1;                       // query tokens per sequence: the last n_tok rows, already appended
  const int32_t* seq_lens = nullptr;
  int64_t max_seq_len = 0;
  void* out = nullptr;
  float scale = 0.f;
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  const rap_tuning_t* tuning = nullptr;
  void* stream = nullptr;
};

// Shared body of rap_decode_attn, rap_decode_attn_rope, the paged and fp8 variants,
// rap_decode_step and rap_decode_attn_multi.
rap_status_t decode_impl(const DecodeRequest& r) {
  const rap_shape_t* shape = r.shape;
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  int page_shift = 0;
  if (r.paging && (st = check_paging(shape, r.paging, &page_shift)) != RAP_OK) return st;
  if (r.max_seq_len < 1) return RAP_ERR_SHAPE;
  if (r.max_seq_len > shape->cache_cap) return RAP_ERR_CAPACITY;
  if (shape->batch == 0) return RAP_OK;
  const bool step = r.k_new || r.v_new || r.new_pos;
  const bool multi = r.n_tok > 1;
  if (r.n_tok < 1) return RAP_ERR_SHAPE;
  if (!r.q || !r.k_cache || !r.v_cache || !r.seq_lens || !r.out) return RAP_ERR_NULL;
  if (step && (!r.k_new || !r.v_new || !r.new_pos)) return RAP_ERR_NULL;
  if ((r.q_pos || step) && no_rotation_rule(shape, r.keep_pair_idx)) return RAP_ERR_NULL;
  if (misaligned(r.k_cache, 16) || misaligned(r.v_cache, 16) || misaligned(r.q, 4) || misaligned(r.out, 4))
    return RAP_ERR_SHAPE;
  Plan p;
  st = make_plan(shape, r.max_seq_len, r.tuning, &p);
  if (st != RAP_OK) return st;
  // the one-call step on the matrix-core kernel hands the new token to the combining kernel, which
  // therefore always runs
  const bool fused_step = step && p.kernel == 2;
  // several query tokens: their rows are the columns of the matrix instruction, 16 at most, and
  // the part among the tokens themselves is added by the combining kernel, which always runs
  if (multi && (p.kernel != 2 || step || r.q_pos ||
                static_cast<int64_t>(r.n_tok) * (shape->n_q_heads / shape->n_kv_heads) > 16))
    return RAP_ERR_UNSUPPORTED;
  const bool combine = p.n_split > 1 || fused_step || multi;
  if (combine) {
    if (!r.workspace || r.workspace_bytes < workspace_need(shape, p, r.n_tok)) return RAP_ERR_WORKSPACE;
    if (misaligned(r.workspace, 256)) return RAP_ERR_WORKSPACE;
  }
  if (p.n_split > 65535 || (static_cast<int64_t>(p.n_split) + 1) * shape->n_kv_heads * shape->batch > kInt32Max)
    return RAP_ERR_UNSUPPORTED;
  // combinations no kernel is built for
  if ((r.fp8 || r.paging) && p.kernel != 2) return RAP_ERR_UNSUPPORTED;   // the vector-ALU kernel reads dense bf16 caches only
  // more than 8 query heads per KV head: the matrix-core kernel with rotated queries only
  if (shape->n_q_heads / shape->n_kv_heads > rap::kMaxGroup && (p.kernel != 2 || step || r.q_pos)) return RAP_ERR_UNSUPPORTED;
  if (r.fp8) {
    if (shape->cache_cap % 16 != 0) return RAP_ERR_SHAPE;
    if (!r.k_scale || !r.v_scale) return RAP_ERR_NULL;
  }
  if (r.mx4) {
    // 4-bit caches: the plain attention call on the matrix-core kernel over dense caches
    if (!r.k_scales4 || !r.v_scales4) return RAP_ERR_NULL;
    if (p.kernel != 2 || r.fp8 || r.paging || step || multi || r.q_pos) return RAP_ERR_UNSUPPORTED;
    if (misaligned(r.k_scales4, 4) || misaligned(r.v_scales4, 4)) return RAP_ERR_SHAPE;
  }

  rap::DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.q = static_cast<const uint16_t*>(r.q);
  a.q_pos = r.q_pos;
  a.keep = r.keep_pair_idx;
  a.pair_freq = shape->pair_inv_freq;
  a.neg2_log2_theta_over_d = neg2_log2_theta_over_d(shape);
  a.d_head = shape->d_head;
  a.k_cache = static_cast<const uint16_t*>(r.k_cache);
  a.v_cache = static_cast<const uint16_t*>(r.v_cache);
  a.seq_lens = r.seq_lens;
  a.out = static_cast<float*>(r.out);
  a.part_acc = static_cast<float*>(r.workspace);
  a.part_ml = r.workspace ? reinterpret_cast<float*>(static_cast<char*>(r.workspace) + part_acc_bytes(shape, p, r.n_tok)) : nullptr;
  a.n_tok = r.n_tok;
  a.group_inv16 = (65536 + (shape->n_q_heads / shape->n_kv_heads) - 1) / (shape->n_q_heads / shape->n_kv_heads);
  a.batch = shape->batch;
  a.n_q = shape->n_q_heads;
  a.n_kv = shape->n_kv_heads;
  a.group = shape->n_q_heads / shape->n_kv_heads;
  a.n_pairs = shape->n_pairs;
  a.d_k = 2 * shape->n_pairs;
  a.d_v = shape->d_v;
  a.max_len = static_cast<int32_t>(r.max_seq_len);
  a.rows_per_split = p.rows_per_split;
  a.n_split = p.n_split;
  a.n_slots = fused_step ? p.n_split + 1 : p.n_split;
  a.cap = shape->cache_cap;
  a.scale_log2e = r.scale * kLog2e;
  a.lds_wave_bytes = rap::mfma_lds_wave_bytes(a.d_k, a.d_v, r.fp8, r.n_tok * a.group, r.mx4);
  a.k_scales4 = r.mx4 ? static_cast<const uint8_t*>(r.k_scales4) : nullptr;
  a.v_scales4 = r.mx4 ? static_cast<const uint8_t*>(r.v_scales4) : nullptr;
  a.k_scale = r.fp8 ? r.k_scale : nullptr;
  a.v_scale = r.fp8 ? r.v_scale : nullptr;
  if (r.paging) {
    a.block_table = r.paging->block_table;
    a.page_shift = page_shift;
    a.n_pages = r.paging->n_pages;
    a.max_pages = r.paging->max_pages;
  }
  a.direct_out = combine ? 0 : 1;
  if (fused_step) {
    a.k_new = static_cast<const uint16_t*>(r.k_new);
    a.v_new = static_cast<const uint16_t*>(r.v_new);
    a.new_pos = r.new_pos;
    a.k_cache_w = static_cast<uint16_t*>(const_cast<void*>(r.k_cache));
    a.v_cache_w = static_cast<uint16_t*>(const_cast<void*>(r.v_cache));
  }

  hipStream_t s = static_cast<hipStream_t>(r.stream);
  if (step && !fused_step) {
    // vector-ALU kernel: the append is a launch of its own ahead of the attention
    AppendRequest ar;
    ar.shape = shape;
    ar.n_new = 1;
    ar.k_new = r.k_new;
    ar.v_new = r.v_new;
    ar.pos = r.new_pos;
    ar.keep_pair_idx = r.keep_pair_idx;
    ar.k_cache = const_cast<void*>(r.k_cache);
    ar.v_cache = const_cast<void*>(r.v_cache);
    ar.stream = r.stream;
    if ((st = append_impl(ar)) != RAP_OK) return st;
  }
  const rap_tuning_t* t = r.tuning;
  if (t && t->ev_main_start && hipEventRecord(static_cast<hipEvent_t>(t->ev_main_start), s) != hipSuccess)
    return RAP_ERR_HIP;
  const hipError_t e = p.kernel == 1 ? rap::launch_decode_valu(a, s) : rap::launch_decode_mfma(a, s);
  if (e != hipSuccess) return RAP_ERR_HIP;
  if (t && t->ev_main_stop && hipEventRecord(static_cast<hipEvent_t>(t->ev_main_stop), s) != hipSuccess)
    return RAP_ERR_HIP;
  if (combine && rap::launch_merge(a, s) != hipSuccess) return RAP_ERR_HIP;
  return RAP_OK;
}

// ---- scratch for the entry point that allocates nothing ------------------------------------------
// The array lives in the device image of the library: each GPU holds its own copy at its own
// address.  On the host its name is only a handle for hipGetSymbolAddress, never a device address;
// kernels get the looked-up pointer as an argument, like any caller's workspace.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[RAP_STATIC_SCRATCH_BYTES];

std::atomic<void*> g_scratch_ptr[rap::kMaxDevicesRemembered];

// Address of `scratch` on the current device, looked up once per device.
rap_status_t static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= rap::kMaxDevicesRemembered) return RAP_ERR_HIP;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return RAP_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // a lost race between host threads repeats the lookup
  }
  *out = ptr;
  return RAP_OK;
}

// rap_decode_attn_rope and its relatives take q_pos and keep_pair_idx as a pair: an argument the
// call needs and does not get is RAP_ERR_NULL, but only once the shape itself has passed.
rap_status_t null_after_shape(const rap_shape_t* shape) {
  const rap_status_t st = check_shape(shape);
  return st != RAP_OK ? st : RAP_ERR_NULL;
}

bool live_call(const rap_shape_t* shape, int64_t max_seq_len) { return shape && shape->batch > 0 && max_seq_len >= 1; }

// ---- prefill attention ----------------------------------------------------------------------------

// Shared body of rap_prefill_attn, rap_prefill_attn_paged and rap_prefill_attn_ex (k_scale and
// v_scale non-null: the caches hold E4M3 codes).
// Workspace of the prefill attention with key ranges: partial accumulators [B * n_new * H_q,
// n_ksplit, d_v] and (reference, sum) pairs, fp32, each block rounded up to 256 bytes; nothing
// when the launch is not split.
size_t prefill_part_acc_bytes(const rap_shape_t* s, int32_t n_new, const rap::PrefillPlan& p) {
  return align_up(static_cast<size_t>(s->batch) * n_new * s->n_q_heads * p.n_ksplit * s->d_v * sizeof(float), 256);
}
size_t prefill_workspace_need(const rap_shape_t* s, int32_t n_new, const rap::PrefillPlan& p) {
  if (p.n_ksplit <= 1) return 0;
  return prefill_part_acc_bytes(s, n_new, p) +
         align_up(static_cast<size_t>(s->batch) * n_new * s->n_q_heads * p.n_ksplit * 2 * sizeof(float), 256) + 256;
}
rap::PrefillPlan prefill_plan_of(const rap_shape_t* s, int32_t n_new, int64_t max_seq_len) {
  return rap::prefill_plan(s->batch, s->n_kv_heads, s->n_q_heads / s->n_kv_heads, 2 * s->n_pairs, s->d_v, n_new,
                           static_cast<int>(max_seq_len));
}

// `split`: the caller offers a workspace, so a launch whose query blocks would not fill the chip
// is cut into key ranges as well and combined by a second launch.
rap_status_t prefill_impl(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new, const void* q,
                          const void* k_cache, const void* v_cache, const int32_t* seq_lens, int64_t max_seq_len,
                          void* out, float scale, void* stream, const float* k_scale = nullptr,
                          const float* v_scale = nullptr, bool split = false, void* workspace = nullptr,
                          size_t workspace_bytes = 0) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  if ((k_scale == nullptr) != (v_scale == nullptr)) return RAP_ERR_NULL;
  if (k_scale && shape->cache_cap % 16 != 0) return RAP_ERR_SHAPE;
  int page_shift = 0;
  if (paging) {
    if ((st = check_paging(shape, paging, &page_shift)) != RAP_OK) return st;
    if (paging->page_rows < 64) return RAP_ERR_UNSUPPORTED;     // a 64-row tile must not straddle pages
  }
  if (n_new < 0 || max_seq_len < 1) return RAP_ERR_SHAPE;
  if (max_seq_len > shape->cache_cap) return RAP_ERR_CAPACITY;
  if (n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!q || !k_cache || !v_cache || !seq_lens || !out) return RAP_ERR_NULL;
  if (misaligned(k_cache, 16) || misaligned(v_cache, 16) || misaligned(q, 4) || misaligned(out, 4)) return RAP_ERR_SHAPE;
  if (static_cast<int64_t>(shape->batch) * n_new > kInt32Max) return RAP_ERR_UNSUPPORTED;
  rap::PrefillPlan plan = prefill_plan_of(shape, n_new, max_seq_len);
  if (!split) plan.n_ksplit = 1;
  if (plan.n_ksplit > 1) {
    if (!workspace || workspace_bytes < prefill_workspace_need(shape, n_new, plan) || misaligned(workspace, 256))
      return RAP_ERR_WORKSPACE;
    if (static_cast<int64_t>(shape->batch) * n_new * shape->n_q_heads > kInt32Max) return RAP_ERR_UNSUPPORTED;
  }
  rap::PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = static_cast<const uint16_t*>(q);
  a.k_cache = static_cast<const uint16_t*>(k_cache);
  a.v_cache = static_cast<const uint16_t*>(v_cache);
  a.seq_lens = seq_lens;
  a.out = static_cast<float*>(out);
  a.batch = shape->batch;
  a.n_new = n_new;
  a.n_q = shape->n_q_heads;
  a.n_kv = shape->n_kv_heads;
  a.group = shape->n_q_heads / shape->n_kv_heads;
  a.d_k = 2 * shape->n_pairs;
  a.d_v = shape->d_v;
  a.max_len = static_cast<int32_t>(max_seq_len);
  a.cap = shape->cache_cap;
  a.scale_log2e = scale * kLog2e;
  a.k_scale = k_scale;
  a.v_scale = v_scale;
  if (paging) {
    a.block_table = paging->block_table;
    a.page_shift = page_shift;
    a.n_pages = paging->n_pages;
    a.max_pages = paging->max_pages;
  }
  a.n_ksplit = plan.n_ksplit;
  if (plan.n_ksplit > 1) {
    a.tiles_per_split = plan.tiles_per_split;
    a.tok_per_wg = plan.tok_per_wg;
    a.part_acc = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + prefill_part_acc_bytes(shape, n_new, plan));
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (rap::launch_prefill(a, s) != hipSuccess) return RAP_ERR_HIP;
  if (plan.n_ksplit > 1) {
    // the combining kernel of the decode path, one block per (b, token, query head), every slot read
    rap::DecodeArgs m;
    memset(&m, 0, sizeof(m));
    m.seq_lens = seq_lens;
    m.out = a.out;
    m.part_acc = a.part_acc;
    m.part_ml = a.part_ml;
    m.batch = a.batch;
    m.n_tok = n_new;
    m.n_q = a.n_q;
    m.n_kv = a.n_kv;
    m.group = a.group;
    m.d_k = a.d_k;
    m.d_v = a.d_v;
    m.max_len = a.max_len;
    m.rows_per_split = plan.tiles_per_split * 64;
    m.n_split = plan.n_ksplit;
    m.n_slots = plan.n_ksplit;
    m.all_slots = 1;
    if (rap::launch_merge(m, s) != hipSuccess) return RAP_ERR_HIP;
  }
  return RAP_OK;
}

}  // namespace

extern "C" {

rap_status_t rap_rope_append(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                             const int32_t* pos, const int32_t* keep_pair_idx, void* k_cache, void* v_cache,
                             void* stream) {
  AppendRequest r;
  r.shape = shape;
  r.n_new = n_new;
  r.k_new = k_new;
  r.v_new = v_new;
  r.pos = pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_cache;
  r.v_cache = v_cache;
  r.stream = stream;
  return append_impl(r);
}

rap_status_t rap_rope_append_paged(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                   const void* k_new, const void* v_new, const int32_t* pos,
                                   const int32_t* keep_pair_idx, void* k_pool, void* v_pool, void* stream) {
  if (!paging) return RAP_ERR_NULL;
  AppendRequest r;
  r.shape = shape;
  r.paging = paging;
  r.n_new = n_new;
  r.k_new = k_new;
  r.v_new = v_new;
  r.pos = pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_pool;
  r.v_cache = v_pool;
  r.stream = stream;
  return append_impl(r);
}

rap_status_t rap_rope_append_q8(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                                const int32_t* pos, const int32_t* keep_pair_idx, void* k_cache8, void* v_cache8,
                                const float* k_scale, const float* v_scale, void* stream) {
  AppendRequest r;
  r.shape = shape;
  r.n_new = n_new;
  r.k_new = k_new;
  r.v_new = v_new;
  r.pos = pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_cache8;
  r.v_cache = v_cache8;
  r.fp8 = true;
  r.k_scale = k_scale;
  r.v_scale = v_scale;
  r.stream = stream;
  return append_impl(r);
}

rap_status_t rap_rope_append_mx4(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                                 const int32_t* pos, const int32_t* keep_pair_idx, void* k_codes, void* k_scales,
                                 void* v_codes, void* v_scales, void* stream) {
  AppendRequest r;
  r.shape = shape;
  r.n_new = n_new;
  r.k_new = k_new;
  r.v_new = v_new;
  r.pos = pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_codes;
  r.v_cache = v_codes;
  r.mx4 = true;
  r.k_scales4 = k_scales;
  r.v_scales4 = v_scales;
  r.stream = stream;
  return append_impl(r);
}

rap_status_t rap_decode_attn_mx4(const rap_shape_t* shape, const void* q, const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales, const int32_t* seq_lens,
                                 int64_t max_seq_len, void* out, float scale, void* workspace, size_t workspace_bytes,
                                 const rap_tuning_t* tuning, void* stream) {
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.k_cache = k_codes;
  r.v_cache = v_codes;
  r.mx4 = true;
  r.k_scales4 = k_scales;
  r.v_scales4 = v_scales;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_rope_queries(const rap_shape_t* shape, int32_t n_new, const void* q, const int32_t* pos,
                              const int32_t* keep_pair_idx, void* q_out, void* stream) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  if (n_new < 0) return RAP_ERR_SHAPE;
  if (n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!q || !pos || no_rotation_rule(shape, keep_pair_idx) || !q_out) return RAP_ERR_NULL;
  if (static_cast<int64_t>(shape->batch) * n_new > kInt32Max) return RAP_ERR_UNSUPPORTED;
  if (misaligned(q, 4) || misaligned(q_out, 4)) return RAP_ERR_SHAPE;
  // the append kernel walking query rows: no V, no cache layout, G query heads per row of kept pairs
  rap::AppendArgs a;
  memset(&a, 0, sizeof(a));
  a.k_new = static_cast<const uint16_t*>(q);
  a.pos = pos;
  a.keep = keep_pair_idx;
  a.pair_freq = shape->pair_inv_freq;
  a.k_cache = static_cast<uint16_t*>(q_out);
  a.batch = shape->batch;
  a.n_new = n_new;
  a.n_kv = shape->n_q_heads;          // heads per token row of the input
  a.d_head = shape->d_head;
  a.n_pairs = shape->n_pairs;
  a.d_v = 0;
  a.group = shape->n_q_heads / shape->n_kv_heads;
  a.cap = shape->cache_cap;
  a.neg2_log2_theta_over_d = neg2_log2_theta_over_d(shape);
  return hip_status(rap::launch_rope_queries(a, static_cast<hipStream_t>(stream)));
}

size_t rap_decode_attn_workspace_bytes(const rap_shape_t* shape, int64_t max_seq_len, const rap_tuning_t* tuning) {
  if (check_shape(shape) != RAP_OK || max_seq_len < 1 || max_seq_len > shape->cache_cap) return 0;
  Plan p;
  if (make_plan(shape, max_seq_len, tuning, &p) != RAP_OK) return 0;
  return workspace_need(shape, p);
}

rap_status_t rap_decode_attn(const rap_shape_t* shape, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale, void* workspace,
                             size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.k_cache = k_cache;
  r.v_cache = v_cache;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_attn_static(const rap_shape_t* shape, const void* q, const void* k_cache, const void* v_cache,
                                    const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                    const rap_tuning_t* tuning, void* stream) {
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.k_cache = k_cache;
  r.v_cache = v_cache;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.tuning = tuning;
  r.stream = stream;
  // an invalid shape, length or tuning gives 0 here and its own error from decode_impl below
  const size_t need = rap_decode_attn_workspace_bytes(shape, max_seq_len, tuning);
  if (need > RAP_STATIC_SCRATCH_BYTES) return RAP_ERR_STATIC_LIMIT;
  if (need > 0 && shape->batch > 0) {
    void* ptr = nullptr;
    const rap_status_t st = static_scratch(&ptr);
    if (st != RAP_OK) return st;
    r.workspace = ptr;
    r.workspace_bytes = RAP_STATIC_SCRATCH_BYTES;
  }
  return decode_impl(r);
}

rap_status_t rap_decode_attn_rope(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                  const int32_t* keep_pair_idx, const void* k_cache, const void* v_cache,
                                  const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                  void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (live_call(shape, max_seq_len) && (!q_pos || no_rotation_rule(shape, keep_pair_idx))) return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.q_pos = q_pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_cache;
  r.v_cache = v_cache;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_step(const rap_shape_t* shape, const void* k_new, const void* v_new, const int32_t* pos,
                             const int32_t* keep_pair_idx, const void* q, int32_t q_is_rotated, void* k_cache,
                             void* v_cache, const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                             void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (live_call(shape, max_seq_len) && (!k_new || !v_new || !pos || no_rotation_rule(shape, keep_pair_idx)))
    return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.q_pos = q_is_rotated ? nullptr : pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_cache;
  r.v_cache = v_cache;
  r.k_new = k_new;
  r.v_new = v_new;
  r.new_pos = pos;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_step_ex(const rap_shape_t* shape, const rap_kv_cache_t* cache, const void* k_new,
                                const void* v_new, const int32_t* pos, const int32_t* keep_pair_idx, const void* q,
                                int32_t q_is_rotated, const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (!cache) return RAP_ERR_NULL;
  if ((cache->k_scale == nullptr) != (cache->v_scale == nullptr)) return null_after_shape(shape);
  if (live_call(shape, max_seq_len) && (!k_new || !v_new || !pos || no_rotation_rule(shape, keep_pair_idx)))
    return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.paging = cache->paging;
  r.q = q;
  r.q_pos = q_is_rotated ? nullptr : pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = cache->k;
  r.v_cache = cache->v;
  r.fp8 = cache->k_scale != nullptr;
  r.k_scale = cache->k_scale;
  r.v_scale = cache->v_scale;
  r.k_new = k_new;
  r.v_new = v_new;
  r.new_pos = pos;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_attn_multi(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_tok, const void* q,
                                   const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                   void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (!cache) return RAP_ERR_NULL;
  if ((cache->k_scale == nullptr) != (cache->v_scale == nullptr)) return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.paging = cache->paging;
  r.q = q;
  r.k_cache = cache->k;
  r.v_cache = cache->v;
  r.fp8 = cache->k_scale != nullptr;
  r.k_scale = cache->k_scale;
  r.v_scale = cache->v_scale;
  r.n_tok = n_tok;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_attn_q8(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                const int32_t* keep_pair_idx, const void* k_cache8, const void* v_cache8,
                                const float* k_scale, const float* v_scale, const int32_t* seq_lens,
                                int64_t max_seq_len, void* out, float scale, void* workspace, size_t workspace_bytes,
                                const rap_tuning_t* tuning, void* stream) {
  if (live_call(shape, max_seq_len) && q_pos && no_rotation_rule(shape, keep_pair_idx)) return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.q = q;
  r.q_pos = q_pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_cache8;
  r.v_cache = v_cache8;
  r.fp8 = true;
  r.k_scale = k_scale;
  r.v_scale = v_scale;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_decode_attn_paged(const rap_shape_t* shape, const rap_paging_t* paging, const void* q,
                                   const int32_t* q_pos, const int32_t* keep_pair_idx, const void* k_pool,
                                   const void* v_pool, const int32_t* seq_lens, int64_t max_seq_len, void* out,
                                   float scale, void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning,
                                   void* stream) {
  if (!paging) return RAP_ERR_NULL;
  if (live_call(shape, max_seq_len) && q_pos && no_rotation_rule(shape, keep_pair_idx)) return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.paging = paging;
  r.q = q;
  r.q_pos = q_pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_pool;
  r.v_cache = v_pool;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_rope_append_paged_q8(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                      const void* k_new, const void* v_new, const int32_t* pos,
                                      const int32_t* keep_pair_idx, void* k_pool8, void* v_pool8, const float* k_scale,
                                      const float* v_scale, void* stream) {
  if (!paging) return RAP_ERR_NULL;
  AppendRequest r;
  r.shape = shape;
  r.paging = paging;
  r.n_new = n_new;
  r.k_new = k_new;
  r.v_new = v_new;
  r.pos = pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_pool8;
  r.v_cache = v_pool8;
  r.fp8 = true;
  r.k_scale = k_scale;
  r.v_scale = v_scale;
  r.stream = stream;
  return append_impl(r);
}

rap_status_t rap_decode_attn_paged_q8(const rap_shape_t* shape, const rap_paging_t* paging, const void* q,
                                      const int32_t* q_pos, const int32_t* keep_pair_idx, const void* k_pool8,
                                      const void* v_pool8, const float* k_scale, const float* v_scale,
                                      const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                      void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (!paging) return RAP_ERR_NULL;
  if (live_call(shape, max_seq_len) && q_pos && no_rotation_rule(shape, keep_pair_idx)) return null_after_shape(shape);
  DecodeRequest r;
  r.shape = shape;
  r.paging = paging;
  r.q = q;
  r.q_pos = q_pos;
  r.keep_pair_idx = keep_pair_idx;
  r.k_cache = k_pool8;
  r.v_cache = v_pool8;
  r.fp8 = true;
  r.k_scale = k_scale;
  r.v_scale = v_scale;
  r.seq_lens = seq_lens;
  r.max_seq_len = max_seq_len;
  r.out = out;
  r.scale = scale;
  r.workspace = workspace;
  r.workspace_bytes = workspace_bytes;
  r.tuning = tuning;
  r.stream = stream;
  return decode_impl(r);
}

rap_status_t rap_prefill_attn(const rap_shape_t* shape, int32_t n_new, const void* q, const void* k_cache,
                              const void* v_cache, const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                              void* stream) {
  return prefill_impl(shape, nullptr, n_new, q, k_cache, v_cache, seq_lens, max_seq_len, out, scale, stream);
}

rap_status_t rap_prefill_attn_ex(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_new, const void* q,
                                 const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale, void* stream) {
  if (!cache) return RAP_ERR_NULL;
  return prefill_impl(shape, cache->paging, n_new, q, cache->k, cache->v, seq_lens, max_seq_len, out, scale, stream,
                      cache->k_scale, cache->v_scale);
}

size_t rap_prefill_attn_split_workspace_bytes(const rap_shape_t* shape, int32_t n_new, int64_t max_seq_len) {
  if (check_shape(shape) != RAP_OK || n_new < 1 || max_seq_len < 1 || max_seq_len > shape->cache_cap) return 0;
  if (shape->batch == 0) return 0;
  return prefill_workspace_need(shape, n_new, prefill_plan_of(shape, n_new, max_seq_len));
}

rap_status_t rap_prefill_attn_split(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_new, const void* q,
                                    const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!cache) return RAP_ERR_NULL;
  return prefill_impl(shape, cache->paging, n_new, q, cache->k, cache->v, seq_lens, max_seq_len, out, scale, stream,
                      cache->k_scale, cache->v_scale, true, workspace, workspace_bytes);
}

rap_status_t rap_prefill_attn_paged(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new, const void* q,
                                    const void* k_pool, const void* v_pool, const int32_t* seq_lens, int64_t max_seq_len,
                                    void* out, float scale, void* stream) {
  if (!paging) return RAP_ERR_NULL;
  return prefill_impl(shape, paging, n_new, q, k_pool, v_pool, seq_lens, max_seq_len, out, scale, stream);
}

rap_status_t rap_check_inputs(const rap_shape_t* shape, int32_t n_new, const int32_t* pos, const int32_t* keep_pair_idx,
                              const int32_t* seq_lens, int64_t max_seq_len, uint32_t* flags, void* stream) {
  const rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  if (!flags) return RAP_ERR_NULL;
  if (n_new < 0 || max_seq_len < 0 || max_seq_len > shape->cache_cap) return RAP_ERR_SHAPE;
  if (misaligned(flags, 4)) return RAP_ERR_SHAPE;
  const long long n_pos = pos ? static_cast<long long>(shape->batch) * n_new : 0;
  if (n_pos > kInt32Max) return RAP_ERR_UNSUPPORTED;
  return hip_status(rap::launch_validate(pos, n_pos, shape->cache_cap, keep_pair_idx, shape->n_kv_heads, shape->n_pairs,
                                         shape->d_head / 2, seq_lens, shape->batch, max_seq_len, flags,
                                         static_cast<hipStream_t>(stream)));
}

rap_status_t rap_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return RAP_ERR_NULL;
  if ((bytes & 15) || misaligned(src, 16) || misaligned(sink, 16)) return RAP_ERR_SHAPE;
  return hip_status(rap::launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

rap_status_t rap_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!src || !dst) return RAP_ERR_NULL;
  if ((bytes & 15) || misaligned(src, 16) || misaligned(dst, 16)) return RAP_ERR_SHAPE;
  return hip_status(rap::launch_stream_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

const char* rap_status_str(rap_status_t status) {
  switch (status) {
    case RAP_OK: return "ok";
    case RAP_ERR_NULL: return "null pointer";
    case RAP_ERR_SHAPE: return "inconsistent shape or argument";
    case RAP_ERR_UNSUPPORTED: return "shape outside the supported range";
    case RAP_ERR_CAPACITY: return "max_seq_len exceeds cache capacity";
    case RAP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RAP_ERR_HIP: return "HIP runtime error";
    case RAP_ERR_STATIC_LIMIT: return "shape needs more scratch than the static array of rap_decode_attn_static holds";
  }
  return "unknown status";
}

int32_t rap_version(void) { return 1000; }

}  // extern "C"
