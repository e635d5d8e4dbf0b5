// Second stage of split decode attention: combine the per-range partials of one query head.
//
// A range s leaves (m_s, l_s, acc_s[d_v]) with m_s the running maximum of the scaled scores in
// log2 units, l_s = sum_i 2^(x_i - m_s) and acc_s = sum_i 2^(x_i - m_s) V[i].  Softmax over the
// whole sequence is then
//   out = sum_s 2^(m_s - m*) acc_s / sum_s 2^(m_s - m*) l_s,   m* = max_s m_s,
// which is Eq. (attn) regrouped by row ranges.  Only the ranges that hold rows of this sequence
// (ceil(len / rows_per_split) of them) were written by the first stage and only those are read.
// In the one-call decode step there is one more slot behind the ranges, always written: the new
// token on its own (m = its score, l = 1, acc = its V row, or m = -inf when it is not attended).
// MULTI, several query tokens per sequence: the ranges stop in front of the new tokens' rows, and
// the causal part among the tokens themselves (token t attends the new rows 0 .. t, at most 16) is
// worked out here, by the workgroup of the query row: each thread multiplies one element of the
// query row with the same element of the new K rows, the products are summed over the workgroup,
// and the weighted new V rows enter the combination like one more range.
#include "rap_device.h"

namespace rap {

constexpr int kMaxTok = 16;

template <bool MULTI>
__global__ __launch_bounds__(128) void merge_kernel(DecodeArgs a) {
  const long long hq = blockIdx.x;                 // query row: (b * n_tok + token) * n_q + query head
  const int b = static_cast<int>(hq / (static_cast<long long>(a.n_q) * a.n_tok));
  const int c = threadIdx.x;
  const bool live = c < a.d_v;
  const float* ml = a.part_ml + hq * a.n_slots * 2;
  const float* accc = a.part_acc + hq * a.n_slots * a.d_v + (live ? c : 0);
  const bool tok = a.n_slots > a.n_split;          // the slot behind the ranges is in use
  float m_tok = tok ? ml[2 * a.n_split] : -INFINITY;
  float l_tok = tok ? ml[2 * a.n_split + 1] : 0.f;
  float v_tok = tok ? accc[static_cast<long long>(a.n_split) * a.d_v] : 0.f;
  const int t_new = a.new_pos != nullptr ? a.new_pos[b] : -1;
  if constexpr (MULTI) {
    __shared__ float s_dot[2][kMaxTok];
    const int T = a.n_tok, G = a.group;
    const int t = static_cast<int>((hq / a.n_q) % T);           // this query row's token
    const int h = static_cast<int>(hq % a.n_q) / G;             // and KV head
    int len = a.seq_lens[b];
    len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
    const int p0 = len - T;                                     // position of new token 0, may be negative
    const bool q8 = a.k_scale != nullptr;
    // row of the cache (dense) or of the pool (paged) that holds position pos >= 0
    auto row_of = [&](int pos) -> long long {
      if (a.block_table == nullptr) return (static_cast<long long>(b) * a.n_kv + h) * a.cap + pos;
      int pg = a.block_table[static_cast<long long>(b) * a.max_pages + (pos >> a.page_shift)];
      pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);
      return ((static_cast<long long>(pg) * a.n_kv + h) << a.page_shift) + (pos & ((1 << a.page_shift) - 1));
    };
    const bool have_k = c < a.d_k;
    const float qv = have_k ? bf16_to_f32(a.q[hq * a.d_k + c]) : 0.f;
    float prod[kMaxTok], vnew[kMaxTok];
    // The loads of all n_tok slots are issued first and used afterwards, so that they travel
    // together: slot j beyond this token's own row repeats that row, a position in front of the
    // sequence reads row 0; what such a slot holds is dropped below by a select.
    const int ck = have_k ? c : 0, cv = live ? c : 0;
    uint32_t kraw[kMaxTok], vraw[kMaxTok];
#pragma unroll
    for (int j = 0; j < kMaxTok; ++j) {
      kraw[j] = 0;
      vraw[j] = 0;
      if (j < T) {
        const int pos = p0 + (j < t ? j : t);
        const long long row = row_of(pos < 0 ? 0 : pos);
        if (q8) {
          kraw[j] = reinterpret_cast<const uint8_t*>(a.k_cache)[row * a.d_k + ck];
          vraw[j] = reinterpret_cast<const uint8_t*>(a.v_cache)[row * a.d_v + cv];
        } else {
          kraw[j] = a.k_cache[row * a.d_k + ck];
          vraw[j] = a.v_cache[row * a.d_v + cv];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kMaxTok; ++j) {
      const float kf = q8 ? e4m3_to_f32(static_cast<uint8_t>(kraw[j])) : bf16_to_f32(static_cast<uint16_t>(kraw[j]));
      vnew[j] = q8 ? e4m3_to_f32(static_cast<uint8_t>(vraw[j])) : bf16_to_f32(static_cast<uint16_t>(vraw[j]));
      prod[j] = have_k ? qv * kf : 0.f;
    }
#pragma unroll
    for (int j = 0; j < kMaxTok; ++j) {
      if (j < T) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) prod[j] += __shfl_xor(prod[j], o);
      }
    }
    if ((c & 63) == 0) {
#pragma unroll
      for (int j = 0; j < kMaxTok; ++j) s_dot[c >> 6][j] = prod[j];
    }
    __syncthreads();
    const float sc = q8 ? a.scale_log2e * a.k_scale[h] : a.scale_log2e;
    float x[kMaxTok];
    m_tok = -INFINITY;
#pragma unroll
    for (int j = 0; j < kMaxTok; ++j) {
      x[j] = (j <= t && p0 + j >= 0) ? (s_dot[0][j] + s_dot[1][j]) * sc : -INFINITY;
      m_tok = fmaxf(m_tok, x[j]);
    }
    l_tok = 0.f;
    v_tok = 0.f;
    if (m_tok > -INFINITY) {
#pragma unroll
      for (int j = 0; j < kMaxTok; ++j) {
        const bool in = j <= t && p0 + j >= 0;
        const float pj = in ? exp2f(x[j] - m_tok) : 0.f;
        l_tok += pj;
        v_tok = fmaf(pj, in ? vnew[j] : 0.f, v_tok);            // a left-out slot may hold NaN or inf
      }
      if (q8) v_tok *= a.v_scale[h];
    }
  }
  // All slots of a query head are allocated, whatever they hold, so they are requested before the
  // sequence length is known, eight at a time: up to eight ranges cost one memory round trip (these
  // reads miss L2, the partials were written through other XCDs; wider groups were measured and
  // do not help: with 32 ranges the kernel takes 7.4 us either way).  Slots beyond the ranges that
  // hold rows are dropped by a select, not multiplied.
  constexpr int kGroup = 8;
  float mstar = m_tok, den = 0.f, num = 0.f;
  if (m_tok > -INFINITY) {
    den = l_tok;
    num = v_tok;
  }
  int n = 0;
  for (int s0 = 0; s0 < a.n_split; s0 += kGroup) {
    float m[kGroup], l[kGroup], v[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const bool have = s0 + u < a.n_split;
      m[u] = have ? ml[2 * (s0 + u)] : -INFINITY;
      l[u] = have ? ml[2 * (s0 + u) + 1] : 0.f;
      v[u] = have ? accc[static_cast<long long>(s0 + u) * a.d_v] : 0.f;
    }
    if (s0 == 0 && a.all_slots) {
      n = a.n_split;                               // prefill key ranges: every slot was written
    } else if (s0 == 0) {
      int len = a.seq_lens[b];
      len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
      if (len > 0 && t_new == len - 1) len -= 1;   // the first stage stopped before the new token's row
      if (a.n_tok > 1) len = len > a.n_tok ? len - a.n_tok : 0;   // or before the new tokens' rows
      n = (len + a.rows_per_split - 1) / a.rows_per_split;   // ranges that hold rows
    }
    if (s0 >= n) break;
    float gmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      if (s0 + u >= n) {                           // unwritten slot: any bits, NaN included
        m[u] = -INFINITY;
        l[u] = 0.f;
        v[u] = 0.f;
      }
      gmax = fmaxf(gmax, m[u]);
    }
    if (gmax > mstar) {                            // the reference follows the running maximum
      const float r = mstar > -INFINITY ? exp2f(mstar - gmax) : 0.f;
      den *= r;
      num *= r;
      mstar = gmax;
    }
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const bool has = m[u] > -INFINITY;           // an empty range leaves only its reference and sum
      const float w = has ? exp2f(m[u] - mstar) : 0.f;
      den = fmaf(w, l[u], den);
      num = fmaf(w, has ? v[u] : 0.f, num);
    }
  }
  if (live) a.out[hq * a.d_v + c] = den > 0.f ? num / den : 0.f;
}

hipError_t launch_merge(const DecodeArgs& a, hipStream_t stream) {
  dim3 grid(static_cast<unsigned>(a.batch) * a.n_tok * a.n_q), block(128);
  if (a.n_tok > 1 && !a.all_slots)
    hipLaunchKernelGGL(merge_kernel<true>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(merge_kernel<false>, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace rap
