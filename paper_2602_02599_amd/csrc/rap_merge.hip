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
#include "rap_device.h"

namespace rap {

__global__ __launch_bounds__(128) void merge_kernel(DecodeArgs a) {
  const long long hq = blockIdx.x;                 // b * n_q + query head
  const int b = static_cast<int>(hq / a.n_q);
  const int c = threadIdx.x;
  const bool live = c < a.d_v;
  const float* ml = a.part_ml + hq * a.n_slots * 2;
  const float* accc = a.part_acc + hq * a.n_slots * a.d_v + (live ? c : 0);
  const bool tok = a.new_pos != nullptr;
  const float m_tok = tok ? ml[2 * a.n_split] : -INFINITY;
  const float l_tok = tok ? ml[2 * a.n_split + 1] : 0.f;
  const float v_tok = tok ? accc[static_cast<long long>(a.n_split) * a.d_v] : 0.f;
  const int t_new = tok ? a.new_pos[b] : -1;
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
    if (s0 == 0) {
      int len = a.seq_lens[b];
      len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
      if (len > 0 && t_new == len - 1) len -= 1;   // the first stage stopped before the new token's row
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
      const float w = m[u] > -INFINITY ? exp2f(m[u] - mstar) : 0.f;
      den = fmaf(w, l[u], den);
      num = fmaf(w, v[u], num);
    }
  }
  if (live) a.out[hq * a.d_v + c] = den > 0.f ? num / den : 0.f;
}

hipError_t launch_merge(const DecodeArgs& a, hipStream_t stream) {
  dim3 grid(static_cast<unsigned>(a.batch) * a.n_q), block(128);
  hipLaunchKernelGGL(merge_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace rap
