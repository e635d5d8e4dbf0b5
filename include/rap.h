/* librap - decode-time attention over a RoPE-aligned-pruned KV cache, for AMD MI355X (gfx950).
 *
 * RAP (RoPE-Aligned Pruning) removes whole RoPE pairs from the key projection and whole channels
 * from the value projection, fuses the selection into W_q and W_o offline, and so leaves a KV
 * cache whose K rows have width d_k = 2 * P (P kept pairs) and whose V rows have width d_v.
 * This library is the online half: write a new token into that compact cache, and attend over it.
 *
 * All pointers marked "dev" are device (HBM) addresses valid on the current HIP device; "host"
 * pointers are ordinary process memory.  The caller owns every buffer.  The library allocates
 * nothing, keeps no state between calls, never synchronises the device and never throws: each
 * entry point validates what can be validated on the host, enqueues its kernels on `stream`
 * (a hipStream_t passed as void*, NULL = the default stream) and returns a status.  When a status
 * other than RAP_OK is returned, no kernel has been enqueued by that call (except RAP_ERR_HIP,
 * which reports a launch failure of the HIP runtime).
 *
 * Stream capture: the calls enqueue kernels only (no allocation, no memset, no copy), so a sequence
 * of them can be recorded into a HIP graph.  One thing happens outside the stream: the first launch
 * of a kernel variant that needs more than 64 KB of LDS raises that kernel's limit with
 * hipFuncSetAttribute (once per device and variant), so make every call once, directly, with the
 * shapes to be recorded, before recording it.
 *
 * Element type of q, k_new, v_new and both caches is bfloat16 (upper half of an IEEE binary32),
 * arithmetic is fp32 (fp64 for the rotation angle), `out` is fp32.
 */
#ifndef RAP_H_
#define RAP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rap_status {
  RAP_OK = 0,
  RAP_ERR_NULL = 1,        /* a required pointer is NULL                                        */
  RAP_ERR_SHAPE = 2,       /* inconsistent shape: G not integral, P > D/2, cap % 8 != 0, ...    */
  RAP_ERR_UNSUPPORTED = 3, /* consistent, but outside what the kernels are built for            */
  RAP_ERR_CAPACITY = 4,    /* max_seq_len exceeds cache_cap                                     */
  RAP_ERR_WORKSPACE = 5,   /* workspace missing or smaller than rap_decode_attn_workspace_bytes */
  RAP_ERR_HIP = 6,         /* the HIP runtime refused a launch                                  */
  RAP_ERR_STATIC_LIMIT = 7 /* rap_decode_attn_static: the shape needs more scratch than
                              RAP_STATIC_SCRATCH_BYTES                                          */
} rap_status_t;

/* Geometry of one attention layer and its compact cache.  Plain data, passed by const pointer.
 *
 * Layouts (row-major, innermost last, no padding anywhere):
 *   k_cache  bf16 [batch, n_kv_heads, cache_cap, 2 * n_pairs]
 *   v_cache  bf16 [batch, n_kv_heads, cache_cap, d_v]
 * A compact K (or q) row holds, for kept pair c in [0, P): element c = original dim
 * keep_pair_idx[h][c], element c + P = original dim keep_pair_idx[h][c] + d_head / 2
 * (the half-apart pairing of Eq. (rope), restricted to the kept pairs: the row order of the
 * selection matrix E_k of Eq. (pruned-decomposition)).
 * Limits: 1 <= n_pairs <= d_head / 2, n_pairs <= 64, 1 <= d_v <= 128, G = n_q_heads / n_kv_heads
 * integral and <= 16 (<= 8 for the vector-ALU kernel, the fused query rotation and the one-call
 * step: RAP_ERR_UNSUPPORTED otherwise), cache_cap a positive multiple of 8 (keeps every 8-row group of either
 * cache 16-byte aligned, whatever the row width).
 */
typedef struct rap_shape {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t d_head;     /* original head dim D: fixes theta_j = rope_theta^(-2j/D) */
  int32_t n_pairs;    /* P kept RoPE pairs; d_k = 2P                             */
  int32_t d_v;        /* kept V channels                                         */
  int64_t cache_cap;  /* rows per (batch, kv head) in both caches                */
  double rope_theta;  /* theta_base                                              */
  /* Optional frequency table, dev fp64 [n_kv_heads, P], or NULL.  When given it replaces both
   * rope_theta and keep_pair_idx (which may then be NULL) in every call that rotates: compact
   * pair c of KV head h turns by pair_inv_freq[h][c] radians per position.  This is how the RoPE
   * variants of Sec. "Practical Considerations" enter: a scaled table (YaRN and the like) is
   * gathered at the kept pairs by the caller, and an entry of 0 leaves a pair un-rotated, which
   * is the hybrid rule for partial-rotary heads and NoPE layers (App. "RoPE in Recent Open
   * LLMs"): channels kept by plain channel pruning ride along as frequency-0 pairs.           */
  const double* pair_inv_freq;
} rap_shape_t;

/* Optional knobs for rap_decode_attn; NULL or all-zero means "choose for me". */
typedef struct rap_tuning {
  int32_t kernel;          /* 0 auto, 1 plain vector-ALU kernel, 2 matrix-core (MFMA) kernel      */
  int32_t rows_per_split;  /* rows of one sequence handled by one workgroup; 0 auto; else a
                              positive multiple of 128                                            */
  int32_t reserved0;
  int32_t reserved1;
  void* ev_main_start;     /* host: optional hipEvent_t recorded on `stream` right before ...     */
  void* ev_main_stop;      /* ... and right after the partial-attention kernel (measurement aid) */
} rap_tuning_t;

/* Per-token cache append.
 *
 * Paper: Sec. "Background" (each new K_t, V_t is written into the cache); Sec. "RAP"
 * (index-aware rotation that uses the original indices of the retained pairs); Eq. (rope)
 * (block [[cos,-sin],[sin,cos]], angle t * theta_base^(-2j/D), pairing (j, j + D/2));
 * Eq. (latent-score) (the cache holds K_latent = RoPE(X W~_k), width 2m).
 *
 * For every b < batch, n < n_new, h < n_kv_heads, with t = pos[b][n] and j_c = keep_pair_idx[h][c]:
 *   phi = t * theta^(-2 j_c / D)                                  (fp64)
 *   k_cache[b][h][t][c]     = bf16( k_new[b][n][h][c] cos phi - k_new[b][n][h][c+P] sin phi )
 *   k_cache[b][h][t][c + P] = bf16( k_new[b][n][h][c] sin phi + k_new[b][n][h][c+P] cos phi )
 *   v_cache[b][h][t][:]     = v_new[b][n][h][:]                   (bit copy)
 * with one round-to-nearest-even to bf16.  Rows not named by pos are left untouched.
 * From n_new = 16 on, runs of 16 tokens whose positions go up by one take their first angle as
 * above and advance it by one fp64 rotation per position (a difference of order 1e-16 in the
 * sine and cosine, far below the rounding to bf16).
 *
 *   k_new          dev  bf16  [batch, n_new, n_kv_heads, 2P]  un-rotated, compact order
 *   v_new          dev  bf16  [batch, n_new, n_kv_heads, d_v]
 *   pos            dev  int32 [batch, n_new]   position of the token == destination row
 *   keep_pair_idx  dev  int32 [n_kv_heads, P]  original pair index in [0, D/2)
 *   k_cache/v_cache dev, updated in place
 * A token whose pos lies outside [0, cache_cap), and a pair whose index lies outside [0, D/2),
 * is skipped on the device (nothing is written for it); the host cannot see either.
 * n_new == 0 or batch == 0 is a no-op returning RAP_OK.
 */
rap_status_t rap_rope_append(const rap_shape_t* shape, int32_t n_new,
                             const void* k_new, const void* v_new,
                             const int32_t* pos, const int32_t* keep_pair_idx,
                             void* k_cache, void* v_cache, void* stream);

/* Bytes of device scratch rap_decode_attn needs for sequences up to max_seq_len rows with the
 * given tuning (NULL = auto).  Returns 0 for an invalid shape.  Never more than a few MB. */
size_t rap_decode_attn_workspace_bytes(const rap_shape_t* shape, int64_t max_seq_len,
                                       const rap_tuning_t* tuning);

/* GQA decode attention of one new token per sequence over the compact cache.
 *
 * Paper: Eq. (attn) and the GQA remark under it; Eq. (latent-score) (scores are taken between
 * the pruned, rotated query and K_latent); Sec. "Step 3" (the caller chooses the softmax scale;
 * the paper keeps 1/sqrt(D)).
 *
 * For every b, query head a (KV head h = a / G), over rows i < seq_lens[b]:
 *   s_i = scale * sum_c q[b][a][c] * k_cache[b][h][i][c]
 *   out[b][a][:] = sum_i softmax(s)_i * v_cache[b][h][i][:]
 * Long sequences are cut into row ranges handled by different workgroups (running max / sum /
 * accumulator per range) and combined by a second kernel; the result does not depend on the cut
 * beyond fp32 rounding.
 *
 *   q          dev  bf16  [batch, n_q_heads, 2P]  pruned and already rotated at its position
 *   seq_lens   dev  int32 [batch]  rows attended, includes the token just appended;
 *                                   0 gives a zero output row; values above max_seq_len are
 *                                   clamped to max_seq_len on the device
 *   max_seq_len host: upper bound on seq_lens, sizes the grid; 1 <= max_seq_len <= cache_cap
 *   out        dev  fp32  [batch, n_q_heads, d_v]
 *   workspace  dev, at least rap_decode_attn_workspace_bytes(shape, max_seq_len, tuning) bytes,
 *              256-byte aligned; contents before and after the call are unspecified (the size
 *              depends on the compute-unit count of the current device: ask on the device the
 *              call will run on)
 * Cache rows at or beyond seq_lens[b] are never used in the result, whatever bits they hold.
 */
rap_status_t rap_decode_attn(const rap_shape_t* shape, const void* q,
                             const void* k_cache, const void* v_cache,
                             const int32_t* seq_lens, int64_t max_seq_len,
                             void* out, float scale,
                             void* workspace, size_t workspace_bytes,
                             const rap_tuning_t* tuning, void* stream);

/* rap_decode_attn for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * per-range partials go to a fixed array of RAP_STATIC_SCRATCH_BYTES bytes that lives in the
 * library's device image (every GPU the library runs on holds its own copy until the process
 * ends); its address on the current device is looked up on the first call there
 * (hipGetSymbolAddress: make that first call outside any stream capture).  The call allocates
 * nothing and frees nothing.  Same kernels, same results, bit for bit, as rap_decode_attn with a
 * workspace of rap_decode_attn_workspace_bytes(shape, max_seq_len, tuning) bytes.
 *
 * A shape whose partials need more than the array holds is refused with RAP_ERR_STATIC_LIMIT and
 * nothing is launched (the five benchmark configurations need 0.8, 4.3, 1.4 and 13.5 MB).
 * Nothing in the array has to be zero beforehand and nothing is cleared: every slot that is read
 * was written by the same call.  All calls on one GPU share that GPU's array: two such calls
 * that overlap in time on one device (different streams, different host threads) race; calls on
 * one stream, or otherwise ordered, are fine.  Arguments as in rap_decode_attn. */
#define RAP_STATIC_SCRATCH_BYTES (16u << 20)
rap_status_t rap_decode_attn_static(const rap_shape_t* shape, const void* q,
                                    const void* k_cache, const void* v_cache,
                                    const int32_t* seq_lens, int64_t max_seq_len,
                                    void* out, float scale,
                                    const rap_tuning_t* tuning, void* stream);

/* The same attention with the query-side rotation fused in: q arrives pruned but UN-rotated and
 * is rotated at q_pos[b] by the index-aware RoPE of its KV head's kept pairs before the scores
 * are taken (Eq. (latent-score): RoPE(X W~_q) . RoPE(X W~_k)^T; Sec. "RAP", index-aware rotation).
 * The rotation uses the arithmetic of rap_rope_append (fp64 angle from the original pair index,
 * one rounding to bf16), so the result is bit-identical to rotating q into a bf16 buffer first
 * and calling rap_decode_attn; it saves that kernel and its launch.
 *
 *   q              dev  bf16  [batch, n_q_heads, 2P]  pruned, un-rotated, compact order
 *   q_pos          dev  int32 [batch]  position of the query token (normally seq_lens[b] - 1)
 *   keep_pair_idx  dev  int32 [n_kv_heads, P]  as for rap_rope_append; query head a uses the row
 *                                              of KV head a / G; a pair whose index lies outside
 *                                              [0, D/2) is taken as zero
 * Everything else as rap_decode_attn.
 */
rap_status_t rap_decode_attn_rope(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                  const int32_t* keep_pair_idx,
                                  const void* k_cache, const void* v_cache,
                                  const int32_t* seq_lens, int64_t max_seq_len,
                                  void* out, float scale,
                                  void* workspace, size_t workspace_bytes,
                                  const rap_tuning_t* tuning, void* stream);

/* Query-side index-aware RoPE for many tokens (the prefill counterpart of the rotation fused into
 * rap_decode_attn_rope): Eq. (latent-score), RoPE(X W~_q), with the arithmetic of rap_rope_append
 * (fp64 angle from the pair's original index or from pair_inv_freq, one rounding to bf16).
 *
 *   q              dev  bf16  [batch, n_new, n_q_heads, 2P]  pruned, un-rotated, compact order
 *   pos            dev  int32 [batch, n_new]  position of each token (any int32; no range rule)
 *   keep_pair_idx  dev  int32 [n_kv_heads, P]; query head a uses the row of KV head a / G; a pair
 *                                              whose index lies outside [0, D/2) is stored as zero
 *   q_out          dev  bf16  [batch, n_new, n_q_heads, 2P]  may be the same buffer as q
 */
rap_status_t rap_rope_queries(const rap_shape_t* shape, int32_t n_new, const void* q, const int32_t* pos,
                              const int32_t* keep_pair_idx, void* q_out, void* stream);

/* Causal attention of the last n_new tokens of every sequence over the compact cache: the prefill
 * (or chunked-prefill) counterpart of rap_decode_attn, Eq. (attn) with the GQA remark per query
 * token at the pruned widths of Eq. (latent-score).  Query i of sequence b sits at position
 * p = seq_lens[b] - n_new + i and attends cache rows [0, p] (itself included; the decoder-only
 * visibility rule).  The rows of the new tokens must already be in the cache (rap_rope_append).
 *
 *   q         dev  bf16  [batch, n_new, n_q_heads, 2P]  pruned, already rotated, compact order
 *   k_cache, v_cache, seq_lens, max_seq_len, scale      as for rap_decode_attn
 *   out       dev  fp32  [batch, n_new, n_q_heads, d_v] every row written; p < 0 (a sequence
 *                                                        shorter than n_new) gives a zero row
 * No workspace: a workgroup owns a block of query tokens and walks the rows they see.
 * Errors as rap_decode_attn; n_new < 0 is RAP_ERR_SHAPE, n_new == 0 returns RAP_OK at once.
 */
rap_status_t rap_prefill_attn(const rap_shape_t* shape, int32_t n_new, const void* q,
                              const void* k_cache, const void* v_cache,
                              const int32_t* seq_lens, int64_t max_seq_len,
                              void* out, float scale, void* stream);

/* One whole decode step of a layer in a single call: append the new token of every sequence
 * (the result of rap_rope_append with n_new = 1), rotate its query unless it already is, and
 * attend (the result of rap_decode_attn / rap_decode_attn_rope over the updated cache).
 * Paper: Sec. "Background" (decode step t: the new K_t, V_t enter the cache, attention runs over
 * the prefix 1:t), Eq. (rope) and Sec. "RAP" (index-aware rotation of the new K row and of the
 * query), Eq. (latent-score) and Eq. (attn) (scores against K_latent, softmax, weighted V).
 * On the matrix-core kernel the append is not a launch of its own: the attention kernel scans
 * the cache without row pos[b], one extra workgroup per (sequence, KV head) rotates the new K
 * row, writes it and the V row into the caches and scores the token straight from registers, and
 * the combining kernel folds that score in.  The caches end up bit-identical to the two-call
 * sequence and every value entering the sums is the same; only the order of fp32 additions
 * differs (outputs agree to fp32 rounding).  The workspace is required whatever the number of
 * row ranges.  With tuning->kernel = 1 (vector-ALU kernel) the call is the two launches.
 *
 *   k_new, v_new   dev  bf16  [batch, n_kv_heads, 2P] / [batch, n_kv_heads, d_v]  the new token
 *   pos            dev  int32 [batch]  its position == cache row (rules of rap_rope_append); also
 *                                      the query position
 *   keep_pair_idx  dev  int32 [n_kv_heads, P]
 *   q              dev  bf16  [batch, n_q_heads, 2P]; q_is_rotated != 0: used as is; 0: rotated at
 *                                      pos[b] first, as by rap_decode_attn_rope
 *   k_cache, v_cache  updated in place; seq_lens (normally pos + 1) and the rest as rap_decode_attn.
 */
rap_status_t rap_decode_step(const rap_shape_t* shape,
                             const void* k_new, const void* v_new, const int32_t* pos,
                             const int32_t* keep_pair_idx,
                             const void* q, int32_t q_is_rotated,
                             void* k_cache, void* v_cache,
                             const int32_t* seq_lens, int64_t max_seq_len,
                             void* out, float scale,
                             void* workspace, size_t workspace_bytes,
                             const rap_tuning_t* tuning, void* stream);

/* fp8 caches.  The paper names KV-cache quantisation as orthogonal to RAP and composable with it
 * (Sec. "Introduction", Sec. "Related Work") without fixing a format; here both caches hold
 * one-byte E4M3 codes (the finite-only 8-bit float of the OCP specification: 4 exponent bits,
 * bias 7, 3 mantissa bits, largest magnitude 448, S.1111.111 = NaN), and a code stands for its
 * value times the scale of its KV head:
 *   k_cache8  dev uint8 [batch, n_kv_heads, cache_cap, 2P],  v_cache8  dev uint8 [batch, n_kv_heads, cache_cap, d_v]
 *   k_scale, v_scale  dev fp32 [n_kv_heads], positive and finite (the caller's calibration)
 * cache_cap must be a multiple of 16 (keeps every 16-row group 16-byte aligned at any width).
 * The append rotates exactly as rap_rope_append, divides by the scale in fp64 and rounds once to
 * the nearest code (ties to the even mantissa, magnitudes above 448 saturate, NaN -> 0x7f); V
 * rows are divided and rounded the same way.  The attention is rap_decode_attn on the values the
 * codes stand for (q stays bf16; q_pos non-NULL fuses its rotation as rap_decode_attn_rope does):
 * the same matrix-core kernel at half the bytes per row.  tuning->kernel = 1 is
 * RAP_ERR_UNSUPPORTED.  Workspace size as for rap_decode_attn. */
rap_status_t rap_rope_append_q8(const rap_shape_t* shape, int32_t n_new,
                                const void* k_new, const void* v_new,
                                const int32_t* pos, const int32_t* keep_pair_idx,
                                void* k_cache8, void* v_cache8,
                                const float* k_scale, const float* v_scale, void* stream);

rap_status_t rap_decode_attn_q8(const rap_shape_t* shape, const void* q, const int32_t* q_pos,
                                const int32_t* keep_pair_idx,
                                const void* k_cache8, const void* v_cache8,
                                const float* k_scale, const float* v_scale,
                                const int32_t* seq_lens, int64_t max_seq_len,
                                void* out, float scale,
                                void* workspace, size_t workspace_bytes,
                                const rap_tuning_t* tuning, void* stream);

/* Paged caches, as batched serving stacks keep them (App. "Limitations", "Serving gains are
 * context-dependent": turning the smaller cache into throughput there needs a fused attention
 * kernel over the stack's own cache).  K and V live in pools of pages shared by all sequences,
 *   k_pool  dev bf16 [n_pages, n_kv_heads, page_rows, 2P],  v_pool  dev bf16 [n_pages, n_kv_heads, page_rows, d_v],
 * and row t of sequence b is row t % page_rows of page block_table[b][t / page_rows].
 *   page_rows        a power of two, 32 .. 65536 (a 32-row tile then never straddles two pages)
 *   n_pages          pages in the pools
 *   max_pages        columns of block_table; shape->cache_cap must equal max_pages * page_rows
 *   block_table      dev int32 [batch, max_pages]; only the entries that cover rows [0, seq_lens[b])
 *                    (and appended positions) are read; a page number outside [0, n_pages) is
 *                    clamped into the pool (wrong result for that sequence, no stray access)
 * Both pools 16-byte aligned.  Everything else is as for the dense calls of the same name:
 * the same kernels with another start address per 32-row tile. */
typedef struct rap_paging {
  int32_t page_rows;
  int32_t n_pages;
  int32_t max_pages;
  int32_t reserved;
  const int32_t* block_table;
} rap_paging_t;

rap_status_t rap_rope_append_paged(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                   const void* k_new, const void* v_new, const int32_t* pos,
                                   const int32_t* keep_pair_idx, void* k_pool, void* v_pool, void* stream);

/* rap_decode_attn over paged caches (matrix-core kernel only: tuning->kernel = 1 is
 * RAP_ERR_UNSUPPORTED); q_pos non-NULL fuses the query rotation as rap_decode_attn_rope does.
 * Workspace size: rap_decode_attn_workspace_bytes with the same shape. */
rap_status_t rap_decode_attn_paged(const rap_shape_t* shape, const rap_paging_t* paging, const void* q,
                                   const int32_t* q_pos, const int32_t* keep_pair_idx,
                                   const void* k_pool, const void* v_pool,
                                   const int32_t* seq_lens, int64_t max_seq_len,
                                   void* out, float scale,
                                   void* workspace, size_t workspace_bytes,
                                   const rap_tuning_t* tuning, void* stream);

/* rap_prefill_attn over paged bf16 pools; page_rows must be at least 64 (smaller pages are
 * RAP_ERR_UNSUPPORTED).  Everything else as in rap_prefill_attn. */
rap_status_t rap_prefill_attn_paged(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                    const void* q, const void* k_pool, const void* v_pool,
                                    const int32_t* seq_lens, int64_t max_seq_len,
                                    void* out, float scale, void* stream);

/* Both together: fp8 (E4M3) codes in paged pools, [n_pages, n_kv_heads, page_rows, d] bytes.
 * Arguments as in rap_rope_append_q8 / rap_decode_attn_q8 and rap_*_paged; page_rows being a
 * multiple of 32 keeps every page 16-byte aligned at one byte per element. */
rap_status_t rap_rope_append_paged_q8(const rap_shape_t* shape, const rap_paging_t* paging, int32_t n_new,
                                      const void* k_new, const void* v_new, const int32_t* pos,
                                      const int32_t* keep_pair_idx, void* k_pool8, void* v_pool8,
                                      const float* k_scale, const float* v_scale, void* stream);
rap_status_t rap_decode_attn_paged_q8(const rap_shape_t* shape, const rap_paging_t* paging, const void* q,
                                      const int32_t* q_pos, const int32_t* keep_pair_idx,
                                      const void* k_pool8, const void* v_pool8,
                                      const float* k_scale, const float* v_scale,
                                      const int32_t* seq_lens, int64_t max_seq_len,
                                      void* out, float scale,
                                      void* workspace, size_t workspace_bytes,
                                      const rap_tuning_t* tuning, void* stream);

/* 4-bit caches: the microscaling FP4 form of the compact cache.
 *
 * Paper: Sec. "Introduction" and Sec. "Related Work" (KV-cache quantisation composes with RAP; no
 * format is fixed there).  Format: the "MXFP4" of the OCP Microscaling Formats specification,
 * which gfx950 converts natively.  Elements are E2M1 codes (1 sign, 2 exponent bits with bias 1,
 * 1 mantissa bit: +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}); every block of 32 consecutive elements of a row
 * shares one scale byte e standing for 2^(e - 127).  With nb(d) = ceil(d / 32):
 *   k_codes  dev uint8 [batch, n_kv_heads, cache_cap, 16 * nb(2P)]   v_codes  [.., 16 * nb(d_v)]
 *            block j of a row holds elements 32 j .. 32 j + 31, element 2 i of the block in the low
 *            nibble of its byte i, element 2 i + 1 in the high nibble; elements at and beyond the
 *            row's width are code 0
 *   k_scales dev uint8 [batch, n_kv_heads, cache_cap, 4]             v_scales likewise
 *            byte j = scale of block j; bytes beyond the row's blocks hold 127
 * All four arrays 16-byte aligned (scales: 4).  A K row of d_k = 90 takes 48 + 4 bytes against 180
 * as bf16.
 *
 * rap_rope_append_mx4: as rap_rope_append (same rotation, Eq. (rope) at the pair's original index,
 * fp64), then each block of the rotated K row and of the V row gets the scale
 * 2^(floor(log2(largest magnitude in the block)) - 2), limited to 2^-126 .. 2^127 and 2^0 for a
 * block of zeros, and every element is divided by it and rounded once, from fp64, to the nearest
 * code (ties to the code with mantissa bit 0, magnitudes above 6 saturate).  A pair whose index
 * lies outside [0, D/2) counts as zero (a row is written as a whole); a token whose pos lies
 * outside [0, cache_cap) is skipped.  Any n_new.
 *
 * rap_decode_attn_mx4: rap_decode_attn with every cache element standing for its code's value
 * times its block's scale (all such values are bf16 numbers, so the arithmetic is that of the
 * bf16 call on the dequantised cache).  Matrix-core kernel only (tuning->kernel = 1 is
 * RAP_ERR_UNSUPPORTED); q arrives rotated.  Workspace and tuning as in rap_decode_attn.  Rows at
 * or beyond seq_lens[b] may hold any codes and scale bytes. */
rap_status_t rap_rope_append_mx4(const rap_shape_t* shape, int32_t n_new, const void* k_new, const void* v_new,
                                 const int32_t* pos, const int32_t* keep_pair_idx,
                                 void* k_codes, void* k_scales, void* v_codes, void* v_scales, void* stream);
rap_status_t rap_decode_attn_mx4(const rap_shape_t* shape, const void* q,
                                 const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales,
                                 const int32_t* seq_lens, int64_t max_seq_len,
                                 void* out, float scale,
                                 void* workspace, size_t workspace_bytes,
                                 const rap_tuning_t* tuning, void* stream);

/* The one-call decode step over any kind of cache.  k, v: the dense caches or, with paging, the
 * pools (dev, updated in place); k_scale, v_scale (dev fp32 [n_kv_heads]): both non-NULL when the
 * caches hold one-byte E4M3 codes, both NULL for bf16; paging: NULL for dense caches.  Everything
 * else as in rap_decode_step; matrix-core kernel only for paged or fp8 caches. */
typedef struct rap_kv_cache {
  void* k;
  void* v;
  const float* k_scale;
  const float* v_scale;
  const rap_paging_t* paging;
} rap_kv_cache_t;

rap_status_t rap_decode_step_ex(const rap_shape_t* shape, const rap_kv_cache_t* cache,
                                const void* k_new, const void* v_new, const int32_t* pos,
                                const int32_t* keep_pair_idx, const void* q, int32_t q_is_rotated,
                                const int32_t* seq_lens, int64_t max_seq_len,
                                void* out, float scale,
                                void* workspace, size_t workspace_bytes,
                                const rap_tuning_t* tuning, void* stream);

/* rap_prefill_attn over any kind of cache (bf16 or E4M3 codes with scales, dense or paged pools of
 * at least 64 rows per page), described as for rap_decode_step_ex; the caches are only read.
 * fp8 caches need cache_cap % 16 == 0. */
rap_status_t rap_prefill_attn_ex(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_new,
                                 const void* q, const int32_t* seq_lens, int64_t max_seq_len,
                                 void* out, float scale, void* stream);

/* rap_prefill_attn_ex for launches that would otherwise leave most of the chip idle (a short chunk
 * of new tokens at the end of long sequences, few sequences): with a workspace the rows a query
 * block sees are cut into key ranges as well, each range a workgroup of its own, and a combining
 * launch (the one of rap_decode_attn) follows.  Whether and how a launch is cut depends on the
 * shape, n_new and max_seq_len alone: rap_prefill_attn_split_workspace_bytes returns the bytes
 * needed, 0 when the launch is not cut (then workspace may be NULL and the call is
 * rap_prefill_attn_ex).  A missing, misaligned (256 bytes) or too small workspace is
 * RAP_ERR_WORKSPACE.  Results equal those of rap_prefill_attn_ex up to fp32 rounding. */
size_t rap_prefill_attn_split_workspace_bytes(const rap_shape_t* shape, int32_t n_new, int64_t max_seq_len);
rap_status_t rap_prefill_attn_split(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_new,
                                    const void* q, const int32_t* seq_lens, int64_t max_seq_len,
                                    void* out, float scale,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* Attention of a few query tokens per sequence at the speed of a decode step (verification of
 * drafted tokens, short chunks): the same result as rap_prefill_attn_ex with n_new = n_tok, i.e.
 * Eq. (attn) with the causal mask for the last n_tok rows of every sequence, which the append has
 * already written (token i sits at row seq_lens[b] - n_tok + i and attends rows 0 .. its own; a
 * token in front of the start of its sequence gives a zero row).  The cache in front of the new
 * rows is read once for all n_tok * (n_q_heads / n_kv_heads) query rows of a KV head, which ride
 * side by side through the matrix instruction: that product must not exceed 16, else
 * RAP_ERR_UNSUPPORTED (use rap_prefill_attn_ex).  n_tok = 1 is rap_decode_attn over `cache`.
 *   q   dev bf16 [batch, n_tok, n_q_heads, d_k] rotated;  out dev fp32 [batch, n_tok, n_q_heads, d_v]
 *   workspace: at least n_tok * rap_decode_attn_workspace_bytes(shape, max_seq_len, tuning) bytes,
 *   256-byte aligned, always needed when n_tok > 1; tuning->kernel must be 0 or 2.
 * Everything else as in rap_decode_attn / rap_decode_step_ex; the caches are only read. */
rap_status_t rap_decode_attn_multi(const rap_shape_t* shape, const rap_kv_cache_t* cache, int32_t n_tok,
                                   const void* q, const int32_t* seq_lens, int64_t max_seq_len,
                                   void* out, float scale,
                                   void* workspace, size_t workspace_bytes,
                                   const rap_tuning_t* tuning, void* stream);

/* A look at the device-side inputs whose values the host never sees, for callers who want to
 * know before trusting a result.  Not an operation of the paper: it checks the preconditions its
 * formulas put on the inputs (Sec. "RAP": the rotation uses the ORIGINAL indices of the retained
 * pairs, each in [0, D/2) and kept once; Sec. "Background": attention runs over a prefix that
 * lies inside the cache).  ORs into *flags (dev, one uint32 the caller has set to 0):
 *   RAP_FLAG_POS        a pos[b][n] outside [0, cache_cap): rap_rope_append skips that token
 *   RAP_FLAG_PAIR       a keep_pair_idx entry outside [0, d_head / 2): that pair is left alone
 *   RAP_FLAG_PAIR_ORDER a row of keep_pair_idx that is not strictly ascending (a pair kept twice)
 *   RAP_FLAG_SEQ_LEN    a seq_lens[b] outside [0, max_seq_len]: the attention clamps it
 * pos [batch, n_new], keep_pair_idx [n_kv_heads, P] and seq_lens [batch] may each be NULL (not
 * looked at).  One small launch on `stream`; nothing is synchronised. */
#define RAP_FLAG_POS 1u
#define RAP_FLAG_PAIR 2u
#define RAP_FLAG_PAIR_ORDER 4u
#define RAP_FLAG_SEQ_LEN 8u
rap_status_t rap_check_inputs(const rap_shape_t* shape, int32_t n_new, const int32_t* pos,
                              const int32_t* keep_pair_idx, const int32_t* seq_lens,
                              int64_t max_seq_len, uint32_t* flags, void* stream);

/* Measurement aids (not part of the method): a read-only streaming pass over `bytes` bytes of
 * `src` (16-byte aligned, bytes % 16 == 0) that folds everything into 16 bytes at `sink`, and a
 * plain copy of `bytes` bytes.  They give the bandwidth a trivial kernel reaches on the same
 * device and calibrate hardware byte counters.  Both are dev pointers. */
rap_status_t rap_stream_read(const void* src, size_t bytes, void* sink, void* stream);
rap_status_t rap_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Static string for a status code. */
const char* rap_status_str(rap_status_t status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t rap_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RAP_H_ */
