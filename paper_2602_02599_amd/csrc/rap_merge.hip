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
  // The first four slots are requested before the sequence length is known (they are allocated,
  // whatever they hold), so the common case of a few ranges costs one memory round trip.
  float m[4], l[4], v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const bool have = u < a.n_split;
    m[u] = have ? ml[2 * u] : 0.f;
    l[u] = have ? ml[2 * u + 1] : 0.f;
    v[u] = have ? accc[static_cast<long long>(u) * a.d_v] : 0.f;
  }
  int len = a.seq_lens[b];
  len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
  if (len > 0 && t_new == len - 1) len -= 1;       // the first stage stopped before the new token's row
  const int n = (len + a.rows_per_split - 1) / a.rows_per_split;   // ranges that hold rows
  float mstar = m_tok;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (u >= n) { m[u] = -INFINITY; l[u] = 0.f; v[u] = 0.f; }      // unwritten slot: drop, do not multiply
    mstar = fmaxf(mstar, m[u]);
  }
  int s = 4;
  for (; s + 4 <= n; s += 4) {
    const float m0 = ml[2 * s], m1 = ml[2 * s + 2], m2 = ml[2 * s + 4], m3 = ml[2 * s + 6];
    mstar = fmaxf(fmaxf(mstar, fmaxf(m0, m1)), fmaxf(m2, m3));
  }
  for (; s < n; ++s) mstar = fmaxf(mstar, ml[2 * s]);
  float den = 0.f, num = 0.f;
  if (m_tok > -INFINITY) {
    den = exp2f(m_tok - mstar) * l_tok;
    num = exp2f(m_tok - mstar) * v_tok;
  }
  if (n > 0) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = exp2f(m[u] - mstar);                          // 2^-inf = 0 for dropped slots
      den = fmaf(w, l[u], den);
      num = fmaf(w, v[u], num);
    }
  }
  s = 4;
  for (; s + 4 <= n; s += 4) {
    float mm[4], ll[4], vv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      mm[u] = ml[2 * (s + u)];
      ll[u] = ml[2 * (s + u) + 1];
      vv[u] = accc[static_cast<long long>(s + u) * a.d_v];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = exp2f(mm[u] - mstar);
      den = fmaf(w, ll[u], den);
      num = fmaf(w, vv[u], num);
    }
  }
  for (; s < n; ++s) {
    const float w = exp2f(ml[2 * s] - mstar);
    den = fmaf(w, ml[2 * s + 1], den);
    num = fmaf(w, accc[static_cast<long long>(s) * a.d_v], num);
  }
  if (live) a.out[hq * a.d_v + c] = den > 0.f ? num / den : 0.f;
}

hipError_t launch_merge(const DecodeArgs& a, hipStream_t stream) {
  dim3 grid(static_cast<unsigned>(a.batch) * a.n_q), block(128);
  hipLaunchKernelGGL(merge_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace rap
