// C ABI of librap: host-side validation, split planning and kernel dispatch.  See include/rap.h
// for the contract of every entry point.
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
int mfma_lds_wave_bytes(int d_k, int d_v, bool q8);
}  // namespace rap

namespace {

constexpr int kCUs = 256;   // MI355X

rap_status_t check_shape(const rap_shape_t* s) {
  if (!s) return RAP_ERR_NULL;
  if (s->batch < 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->d_head <= 0 || (s->d_head & 1) ||
      s->n_pairs <= 0 || s->d_v <= 0 || s->cache_cap <= 0 || !(s->rope_theta > 0.0))
    return RAP_ERR_SHAPE;
  if (s->n_q_heads % s->n_kv_heads != 0) return RAP_ERR_SHAPE;
  if (s->n_pairs > s->d_head / 2) return RAP_ERR_SHAPE;
  if (s->cache_cap % 8 != 0) return RAP_ERR_SHAPE;
  if (s->n_pairs > rap::kMaxPairs || s->d_v > rap::kMaxDv || s->n_q_heads / s->n_kv_heads > rap::kMaxGroup)
    return RAP_ERR_UNSUPPORTED;
  if (s->cache_cap > 0x7fffffffLL - 1024 || s->batch > 65535 || s->n_kv_heads > 65535) return RAP_ERR_UNSUPPORTED;
  return RAP_OK;
}

struct Plan {
  int rows_per_split;
  int n_split;
  int kernel;   // 1 vector ALU, 2 matrix core
};

// Row range per workgroup.  The grid is (n_split, H_kv, B); a workgroup whose range starts at or
// beyond its sequence's length exits at once, so ragged batches cost only empty launches.
// Measured on MI355X: a workgroup should stream for a long time (its fixed cost is a few
// microseconds), and when the whole job fits in one round of resident workgroups their number
// should be a multiple of the 256 compute units.  So: about 512 workgroups when the (b, h) count
// allows it, ranges never shorter than 512 rows nor longer than 4096 (longer ranges only lengthen
// the tail of a ragged batch).
rap_status_t make_plan(const rap_shape_t* s, int64_t max_seq_len, const rap_tuning_t* t, Plan* p) {
  int rps = t ? t->rows_per_split : 0;
  if (rps < 0 || (rps % rap::kSplitQuantum) != 0) return RAP_ERR_SHAPE;
  const int kernel = t ? t->kernel : 0;
  if (kernel < 0 || kernel > 2) return RAP_ERR_SHAPE;
  if (rps == 0) {
    const int64_t slabs = static_cast<int64_t>(s->batch) * s->n_kv_heads;
    int64_t per_slab = slabs > 0 ? (2LL * kCUs) / slabs : 1;            // ranges per (b, h)
    if (per_slab < 1) per_slab = 1;
    int64_t r = (max_seq_len + per_slab - 1) / per_slab;
    r = (r + rap::kSplitQuantum - 1) / rap::kSplitQuantum * rap::kSplitQuantum;
    if (r < 512) r = 512;
    if (r > 4096) r = 4096;
    rps = static_cast<int>(r);
  }
  p->rows_per_split = rps;
  p->n_split = static_cast<int>((max_seq_len + rps - 1) / rps);
  p->kernel = kernel == 0 ? 2 : kernel;
  return RAP_OK;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t part_acc_bytes(const rap_shape_t* s, const Plan& p) {
  return align_up(static_cast<size_t>(s->batch) * s->n_q_heads * (p.n_split + 1) * s->d_v * sizeof(float), 256);
}
size_t part_ml_bytes(const rap_shape_t* s, const Plan& p) {
  return align_up(static_cast<size_t>(s->batch) * s->n_q_heads * (p.n_split + 1) * 2 * sizeof(float), 256);
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

}  // namespace

extern "C" {

static rap_status_t append_impl(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new, const void* k_new,
                                const void* v_new, const int32_t* pos, const int32_t* keep_pair_idx, void* k_cache,
                                void* v_cache, void* stream, const float* k_scale = nullptr,
                                const float* v_scale = nullptr, bool q8 = false) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  int page_shift = 0;
  if (paging && (st = check_paging(shape, paging, &page_shift)) != RAP_OK) return st;
  if (n_new < 0) return RAP_ERR_SHAPE;
  if (n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!k_new || !v_new || !pos || (!keep_pair_idx && !shape->pair_inv_freq) || !k_cache || !v_cache) return RAP_ERR_NULL;
  if (static_cast<int64_t>(shape->batch) * n_new > 0x7fffffffLL) return RAP_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(k_new) & 3) || (reinterpret_cast<uintptr_t>(v_new) & 3) ||
      (reinterpret_cast<uintptr_t>(k_cache) & 3) || (reinterpret_cast<uintptr_t>(v_cache) & 3))
    return RAP_ERR_SHAPE;
  rap::AppendArgs a;
  memset(&a, 0, sizeof(a));
  if (paging) {
    a.block_table = paging->block_table;
    a.page_shift = page_shift;
    a.n_pages = paging->n_pages;
    a.max_pages = paging->max_pages;
  }
  if (q8) {
    if (!k_scale || !v_scale) return RAP_ERR_NULL;
    if (shape->cache_cap % 16 != 0) return RAP_ERR_SHAPE;
    a.k_scale = k_scale;
    a.v_scale = v_scale;
  }
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.pos = pos;
  a.keep = keep_pair_idx;
  a.pair_freq = shape->pair_inv_freq;
  a.k_cache = static_cast<uint16_t*>(k_cache);
  a.v_cache = static_cast<uint16_t*>(v_cache);
  a.batch = shape->batch;
  a.n_new = n_new;
  a.n_kv = shape->n_kv_heads;
  a.d_head = shape->d_head;
  a.n_pairs = shape->n_pairs;
  a.d_v = shape->d_v;
  a.group = 1;
  a.cap = shape->cache_cap;
  a.neg2_log2_theta_over_d = -2.0 * log2(shape->rope_theta) / static_cast<double>(shape->d_head);
  return rap::launch_append(a, static_cast<hipStream_t>(stream)) == hipSuccess ? RAP_OK : RAP_ERR_HIP;
}

rap_status_t rap_rope_append(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                             const int32_t* pos, const int32_t* keep_pair_idx, void* k_cache, void* v_cache,
                             void* stream) {
  return append_impl(shape, nullptr, n_new, k_new, v_new, pos, keep_pair_idx, k_cache, v_cache, stream);
}

rap_status_t rap_rope_append_paged(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                   const void* k_new, const void* v_new, const int32_t* pos,
                                   const int32_t* keep_pair_idx, void* k_pool, void* v_pool, void* stream) {
  if (!paging) return RAP_ERR_NULL;
  return append_impl(shape, paging, n_new, k_new, v_new, pos, keep_pair_idx, k_pool, v_pool, stream);
}

rap_status_t rap_rope_queries(const rap_shape_t* shape, int32_t n_new, const void* q, const int32_t* pos,
                              const int32_t* keep_pair_idx, void* q_out, void* stream) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  if (n_new < 0) return RAP_ERR_SHAPE;
  if (n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!q || !pos || (!keep_pair_idx && !shape->pair_inv_freq) || !q_out) return RAP_ERR_NULL;
  if (static_cast<int64_t>(shape->batch) * n_new > 0x7fffffffLL) return RAP_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(q) & 3) || (reinterpret_cast<uintptr_t>(q_out) & 3)) return RAP_ERR_SHAPE;
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
  a.neg2_log2_theta_over_d = -2.0 * log2(shape->rope_theta) / static_cast<double>(shape->d_head);
  return rap::launch_rope_queries(a, static_cast<hipStream_t>(stream)) == hipSuccess ? RAP_OK : RAP_ERR_HIP;
}

size_t rap_decode_attn_workspace_bytes(const rap_shape_t* shape, int64_t max_seq_len, const rap_tuning_t* tuning) {
  if (check_shape(shape) != RAP_OK || max_seq_len < 1 || max_seq_len > shape->cache_cap) return 0;
  Plan p;
  if (make_plan(shape, max_seq_len, tuning, &p) != RAP_OK) return 0;
  return part_acc_bytes(shape, p) + part_ml_bytes(shape, p) + 256;
}

}  // extern "C"

namespace {

struct Fp8Scales {         // fp8 caches: per-KV-head scales of the codes (device); null otherwise
  const float* k_scale;
  const float* v_scale;
};

struct NewToken {          // the append fused into rap_decode_step; all null otherwise
  const void* k_new = nullptr;
  const void* v_new = nullptr;
  const int32_t* pos = nullptr;
};

// Shared body of rap_decode_attn (q_pos == keep == null), rap_decode_attn_rope and rap_decode_step.
rap_status_t decode_impl(const rap_shape_t* shape, const void* q, const int32_t* q_pos, const int32_t* keep,
                         const void* k_cache, const void* v_cache, const int32_t* seq_lens, int64_t max_seq_len,
                         void* out, float scale, void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning,
                         void* stream, const NewToken& nt = NewToken(), const rap_paging_t* paging = nullptr,
                         const Fp8Scales* q8 = nullptr) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  int page_shift = 0;
  if (paging && (st = check_paging(shape, paging, &page_shift)) != RAP_OK) return st;
  if (max_seq_len < 1) return RAP_ERR_SHAPE;
  if (max_seq_len > shape->cache_cap) return RAP_ERR_CAPACITY;
  if (shape->batch == 0) return RAP_OK;
  if (!q || !k_cache || !v_cache || !seq_lens || !out) return RAP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(k_cache) & 15) || (reinterpret_cast<uintptr_t>(v_cache) & 15) ||
      (reinterpret_cast<uintptr_t>(q) & 3) || (reinterpret_cast<uintptr_t>(out) & 3))
    return RAP_ERR_SHAPE;
  Plan p;
  st = make_plan(shape, max_seq_len, tuning, &p);
  if (st != RAP_OK) return st;
  const size_t need = part_acc_bytes(shape, p) + part_ml_bytes(shape, p) + 256;
  // the one-call step on the matrix-core kernel hands the new token to the combining kernel, which
  // therefore always runs
  const bool fused_step = nt.k_new != nullptr && p.kernel == 2;
  if (p.n_split > 1 || fused_step) {
    if (!workspace || workspace_bytes < need) return RAP_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return RAP_ERR_WORKSPACE;
  }
  if (p.n_split > 65535 ||
      (static_cast<int64_t>(p.n_split) + 1) * shape->n_kv_heads * shape->batch > 0x7fffffffLL) return RAP_ERR_UNSUPPORTED;

  rap::DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.q = static_cast<const uint16_t*>(q);
  a.q_pos = q_pos;
  a.keep = keep;
  a.pair_freq = shape->pair_inv_freq;
  a.neg2_log2_theta_over_d = -2.0 * log2(shape->rope_theta) / static_cast<double>(shape->d_head);
  a.d_head = shape->d_head;
  a.k_cache = static_cast<const uint16_t*>(k_cache);
  a.v_cache = static_cast<const uint16_t*>(v_cache);
  a.seq_lens = seq_lens;
  a.out = static_cast<float*>(out);
  a.part_acc = static_cast<float*>(workspace);
  a.part_ml = workspace ? reinterpret_cast<float*>(static_cast<char*>(workspace) + part_acc_bytes(shape, p)) : nullptr;
  a.batch = shape->batch;
  a.n_q = shape->n_q_heads;
  a.n_kv = shape->n_kv_heads;
  a.group = shape->n_q_heads / shape->n_kv_heads;
  a.n_pairs = shape->n_pairs;
  a.d_k = 2 * shape->n_pairs;
  a.d_v = shape->d_v;
  a.max_len = static_cast<int32_t>(max_seq_len);
  a.rows_per_split = p.rows_per_split;
  a.n_split = p.n_split;
  a.n_slots = p.n_split;
  a.cap = shape->cache_cap;
  a.scale_log2e = scale * 1.4426950408889634f;
  a.lds_wave_bytes = rap::mfma_lds_wave_bytes(a.d_k, a.d_v, q8 != nullptr);
  if (q8) {
    if (p.kernel != 2 || paging || nt.k_new) return RAP_ERR_UNSUPPORTED;   // matrix-core kernel, dense cache, no fused step
    if (shape->cache_cap % 16 != 0) return RAP_ERR_SHAPE;
    if (!q8->k_scale || !q8->v_scale) return RAP_ERR_NULL;
    a.k_scale = q8->k_scale;
    a.v_scale = q8->v_scale;
  }
  if (paging) {
    if (p.kernel != 2) return RAP_ERR_UNSUPPORTED;      // the vector-ALU kernel reads dense caches only
    a.block_table = paging->block_table;
    a.page_shift = page_shift;
    a.n_pages = paging->n_pages;
    a.max_pages = paging->max_pages;
  }
  a.direct_out = (p.n_split == 1 && !fused_step) ? 1 : 0;
  if (fused_step) {
    a.k_new = static_cast<const uint16_t*>(nt.k_new);
    a.v_new = static_cast<const uint16_t*>(nt.v_new);
    a.new_pos = nt.pos;
    a.n_slots = p.n_split + 1;
    a.k_cache_w = static_cast<uint16_t*>(const_cast<void*>(k_cache));
    a.v_cache_w = static_cast<uint16_t*>(const_cast<void*>(v_cache));
  }

  hipStream_t s = static_cast<hipStream_t>(stream);
  if (nt.k_new && !fused_step) {
    // vector-ALU kernel: the append is a launch of its own ahead of the attention
    const rap_status_t ast = rap_rope_append(shape, 1, nt.k_new, nt.v_new, nt.pos, keep, const_cast<void*>(k_cache),
                                             const_cast<void*>(v_cache), stream);
    if (ast != RAP_OK) return ast;
  }
  if (tuning && tuning->ev_main_start && hipEventRecord(static_cast<hipEvent_t>(tuning->ev_main_start), s) != hipSuccess)
    return RAP_ERR_HIP;
  hipError_t e = p.kernel == 1 ? rap::launch_decode_valu(a, s) : rap::launch_decode_mfma(a, s);
  if (e != hipSuccess) return RAP_ERR_HIP;
  if (tuning && tuning->ev_main_stop && hipEventRecord(static_cast<hipEvent_t>(tuning->ev_main_stop), s) != hipSuccess)
    return RAP_ERR_HIP;
  if ((p.n_split > 1 || fused_step) && rap::launch_merge(a, s) != hipSuccess) return RAP_ERR_HIP;
  return RAP_OK;
}

}  // namespace

extern "C" {

rap_status_t rap_decode_attn(const rap_shape_t* shape, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale, void* workspace,
                             size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  return decode_impl(shape, q, nullptr, nullptr, k_cache, v_cache, seq_lens, max_seq_len, out, scale, workspace,
                     workspace_bytes, tuning, stream);
}

rap_status_t rap_decode_step(const rap_shape_t* shape, const void* k_new, const void* v_new, const int32_t* pos,
                             const int32_t* keep_pair_idx, const void* q, int32_t q_is_rotated, void* k_cache,
                             void* v_cache, const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                             void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (shape && shape->batch > 0 && max_seq_len >= 1 && (!k_new || !v_new || !pos || (!keep_pair_idx && !shape->pair_inv_freq))) {
    const rap_status_t st = check_shape(shape);
    return st != RAP_OK ? st : RAP_ERR_NULL;
  }
  NewToken nt;
  nt.k_new = k_new;
  nt.v_new = v_new;
  nt.pos = pos;
  return decode_impl(shape, q, q_is_rotated ? nullptr : pos, keep_pair_idx, k_cache, v_cache, seq_lens, max_seq_len, out,
                     scale, workspace, workspace_bytes, tuning, stream, nt);
}

rap_status_t rap_decode_attn_rope(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                  const int32_t* keep_pair_idx, const void* k_cache, const void* v_cache,
                                  const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                                  void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning, void* stream) {
  if (shape && shape->batch > 0 && max_seq_len >= 1 && (!q_pos || (!keep_pair_idx && !shape->pair_inv_freq))) {
    const rap_status_t st = check_shape(shape);
    return st != RAP_OK ? st : RAP_ERR_NULL;
  }
  return decode_impl(shape, q, q_pos, keep_pair_idx, k_cache, v_cache, seq_lens, max_seq_len, out, scale, workspace,
                     workspace_bytes, tuning, stream);
}

rap_status_t rap_prefill_attn(const rap_shape_t* shape, int32_t n_new, const void* q, const void* k_cache,
                              const void* v_cache, const int32_t* seq_lens, int64_t max_seq_len, void* out, float scale,
                              void* stream) {
  rap_status_t st = check_shape(shape);
  if (st != RAP_OK) return st;
  if (n_new < 0 || max_seq_len < 1) return RAP_ERR_SHAPE;
  if (max_seq_len > shape->cache_cap) return RAP_ERR_CAPACITY;
  if (n_new == 0 || shape->batch == 0) return RAP_OK;
  if (!q || !k_cache || !v_cache || !seq_lens || !out) return RAP_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(k_cache) & 15) || (reinterpret_cast<uintptr_t>(v_cache) & 15) ||
      (reinterpret_cast<uintptr_t>(q) & 3) || (reinterpret_cast<uintptr_t>(out) & 3))
    return RAP_ERR_SHAPE;
  if (static_cast<int64_t>(shape->batch) * n_new > 0x7fffffffLL) return RAP_ERR_UNSUPPORTED;
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
  a.scale_log2e = scale * 1.4426950408889634f;
  return rap::launch_prefill(a, static_cast<hipStream_t>(stream)) == hipSuccess ? RAP_OK : RAP_ERR_HIP;
}

rap_status_t rap_rope_append_q8(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                                const int32_t* pos, const int32_t* keep_pair_idx, void* k_cache8, void* v_cache8,
                                const float* k_scale, const float* v_scale, void* stream) {
  return append_impl(shape, nullptr, n_new, k_new, v_new, pos, keep_pair_idx, k_cache8, v_cache8, stream, k_scale, v_scale,
                     true);
}

rap_status_t rap_decode_attn_q8(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                const int32_t* keep_pair_idx, const void* k_cache8, const void* v_cache8,
                                const float* k_scale, const float* v_scale, const int32_t* seq_lens,
                                int64_t max_seq_len, void* out, float scale, void* workspace, size_t workspace_bytes,
                                const rap_tuning_t* tuning, void* stream) {
  if (shape && shape->batch > 0 && max_seq_len >= 1 && q_pos && !keep_pair_idx && !shape->pair_inv_freq) {
    const rap_status_t st = check_shape(shape);
    return st != RAP_OK ? st : RAP_ERR_NULL;
  }
  Fp8Scales sc{k_scale, v_scale};
  return decode_impl(shape, q, q_pos, keep_pair_idx, k_cache8, v_cache8, seq_lens, max_seq_len, out, scale, workspace,
                     workspace_bytes, tuning, stream, NewToken(), nullptr, &sc);
}

rap_status_t rap_decode_attn_paged(const rap_shape_t* shape, const rap_paging_t* paging, const void* q,
                                   const int32_t* q_pos, const int32_t* keep_pair_idx, const void* k_pool,
                                   const void* v_pool, const int32_t* seq_lens, int64_t max_seq_len, void* out,
                                   float scale, void* workspace, size_t workspace_bytes, const rap_tuning_t* tuning,
                                   void* stream) {
  if (!paging) return RAP_ERR_NULL;
  if (shape && shape->batch > 0 && max_seq_len >= 1 && q_pos && !keep_pair_idx && !shape->pair_inv_freq) {
    const rap_status_t st = check_shape(shape);
    return st != RAP_OK ? st : RAP_ERR_NULL;
  }
  return decode_impl(shape, q, q_pos, keep_pair_idx, k_pool, v_pool, seq_lens, max_seq_len, out, scale, workspace,
                     workspace_bytes, tuning, stream, NewToken(), paging);
}

rap_status_t rap_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return RAP_ERR_NULL;
  if ((bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(sink) & 15)) return RAP_ERR_SHAPE;
  return rap::launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? RAP_OK : RAP_ERR_HIP;
}

rap_status_t rap_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!src || !dst) return RAP_ERR_NULL;
  if ((bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15)) return RAP_ERR_SHAPE;
  return rap::launch_stream_copy(dst, src, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? RAP_OK : RAP_ERR_HIP;
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
  }
  return "unknown status";
}

int32_t rap_version(void) { return 100; }

}  // extern "C"
