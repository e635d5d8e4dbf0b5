// Plain vector-ALU decode attention over the compact cache (no matrix cores).
//
// Eq. (attn) with the GQA remark: for the G query heads that share KV head h,
//   s[g][i] = scale * q[g] . K[i],   out[g] = softmax_i(s[g]) . V.
// One workgroup (4 wavefronts) owns a row range of one (sequence, KV head) and walks it in tiles of
// 64 rows with a running (max, sum, accumulator) per query head, i.e. online softmax.
//
//   scores   16 lanes per cache row, 4 rows per wavefront step; a lane reads dwords
//            sub, sub+16, ... of the row (two bf16 each; a compact K row is exactly P dwords), the
//            query fragment it needs lives in registers, and the 16 partial dots are folded with
//            lane shuffles.  The G heads reuse every unpacked K element.
//   softmax  one wavefront per query head over the 64 scores of the tile (lane = row).
//   P.V      lane = channel pair; every wavefront takes 16 rows of the tile, the probabilities are
//            broadcast reads from LDS; the four per-wave accumulators are summed at the end.
//
// This kernel is the simple, general one (any P <= 64, d_v <= 128, G <= 8).  It needs about
// (G + 1) vector instructions per cache element and two barriers per tile, which is why the
// matrix-core kernel, not this one, is the default.
#include "rap_device.h"

namespace rap {

namespace {

constexpr int kTile = 64;

template <int G, int NPL>
__global__ __launch_bounds__(256) void decode_valu_kernel(DecodeArgs a) {
  const int split = blockIdx.x;
  const int h = blockIdx.y;
  const int b = blockIdx.z;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;

  int len = a.seq_lens[b];
  len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
  const int r0 = split * a.rows_per_split;
  if (r0 >= len) {
    // no rows for this workgroup.  With a single range nobody else writes the output row of an
    // empty sequence; with several ranges the combining kernel does.
    if (a.direct_out)
      for (int e = tid; e < G * a.d_v; e += 256)
        a.out[(static_cast<long long>(b) * a.n_q + h * G) * a.d_v + e] = 0.f;
    return;
  }
  const int r1 = min(r0 + a.rows_per_split, len);

  const int P = a.n_pairs;
  const int dv = a.d_v;
  const long long slab = static_cast<long long>(b) * a.n_kv + h;
  const uint32_t* kbase = reinterpret_cast<const uint32_t*>(a.k_cache) + slab * a.cap * P;
  const uint16_t* vbase = a.v_cache + slab * a.cap * dv;

  __shared__ float s_sc[G][kTile];      // scaled scores of the tile (log2 units)
  __shared__ float s_p[G][kTile];       // exp2(score - running max)
  __shared__ float s_alpha[G];          // rescale factor of the accumulators for this tile
  __shared__ float s_m[G];
  __shared__ float s_l[G];
  __shared__ float s_red[4][G][kMaxDv];

  // query fragment: dwords sub + 16 n of each of the G query rows
  const int sub = lane & 15;
  const int rr = lane >> 4;
  __shared__ uint16_t s_q[kMaxGroup * 2 * kMaxPairs];
  const bool rope_q = a.q_pos != nullptr;     // un-rotated queries: rotate them into LDS first
  if (rope_q) {
    rotate_queries_to_lds(a, b, h, tid, 256, s_q);
    __syncthreads();
  }
  float qlo[G][NPL], qhi[G][NPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint32_t* qrow = rope_q ? reinterpret_cast<const uint32_t*>(s_q) + g * P
                                  : reinterpret_cast<const uint32_t*>(a.q) +
                                        (static_cast<long long>(b) * a.n_q + h * G + g) * P;
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int j = sub + 16 * n;
      const uint32_t w = j < P ? qrow[j] : 0u;
      qlo[g][n] = bf16_lo(w);
      qhi[g][n] = bf16_hi(w);
    }
  }
  if (tid < G) {
    s_m[tid] = -INFINITY;
    s_l[tid] = 0.f;
  }

  // P.V accumulators: this lane owns channels 2*lane and 2*lane+1
  float acc0[G], acc1[G];
#pragma unroll
  for (int g = 0; g < G; ++g) acc0[g] = acc1[g] = 0.f;
  const int c0 = 2 * lane;
  const bool c0_ok = c0 < dv;
  const bool c1_ok = c0 + 1 < dv;
  const bool v_dword = (dv & 1) == 0;
  __syncthreads();

  for (int base = r0; base < r1; base += kTile) {
    // ---- scores
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int rt = 16 * wave + 4 * st + rr;      // row inside the tile
      const int row = base + rt;
      const bool ok = row < r1;
      float d[G];
#pragma unroll
      for (int g = 0; g < G; ++g) d[g] = 0.f;
      const uint32_t* krow = kbase + static_cast<long long>(row) * P;
#pragma unroll
      for (int n = 0; n < NPL; ++n) {
        const int j = sub + 16 * n;
        const uint32_t w = (ok && j < P) ? krow[j] : 0u;
        const float lo = bf16_lo(w), hi = bf16_hi(w);
#pragma unroll
        for (int g = 0; g < G; ++g) d[g] = fmaf(hi, qhi[g][n], fmaf(lo, qlo[g][n], d[g]));
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float x = d[g];
        x += __shfl_xor(x, 1, 16);
        x += __shfl_xor(x, 2, 16);
        x += __shfl_xor(x, 4, 16);
        x += __shfl_xor(x, 8, 16);
        if (sub == 0) s_sc[g][rt] = ok ? x * a.scale_log2e : -INFINITY;
      }
    }
    __syncthreads();
    // ---- online softmax of the tile: wavefront w takes heads w, w+4, ...
    for (int g = wave; g < G; g += 4) {
      const float x = s_sc[g][lane];
      float mx = x;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float m_old = s_m[g];
      const float m_new = fmaxf(m_old, mx);            // finite: the tile holds >= 1 valid row
      const float p = exp2f(x - m_new);                // -inf row -> 0
      float sum = p;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
      s_p[g][lane] = p;
      if (lane == 0) {
        const float alpha = exp2f(m_old - m_new);      // first tile: exp2(-inf) = 0
        s_alpha[g] = alpha;
        s_l[g] = s_l[g] * alpha + sum;
        s_m[g] = m_new;
      }
    }
    __syncthreads();
    // ---- P.V: this wavefront takes rows 16*wave .. 16*wave+15 of the tile
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float al = s_alpha[g];
      acc0[g] *= al;
      acc1[g] *= al;
    }
    const int rows_here = min(kTile, r1 - base);
    for (int i = 16 * wave; i < min(16 * wave + 16, rows_here); ++i) {
      const uint16_t* vrow = vbase + static_cast<long long>(base + i) * dv;
      float v0 = 0.f, v1 = 0.f;
      if (v_dword) {
        if (c0_ok) {
          const uint32_t w = *reinterpret_cast<const uint32_t*>(vrow + c0);
          v0 = bf16_lo(w);
          v1 = bf16_hi(w);
        }
      } else {
        if (c0_ok) v0 = bf16_to_f32(vrow[c0]);
        if (c1_ok) v1 = bf16_to_f32(vrow[c0 + 1]);
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = s_p[g][i];
        acc0[g] = fmaf(p, v0, acc0[g]);
        acc1[g] = fmaf(p, v1, acc1[g]);
      }
    }
  }

  // ---- fold the four wavefronts, then write the result or the partial
#pragma unroll
  for (int g = 0; g < G; ++g) {
    if (c0_ok) s_red[wave][g][c0] = acc0[g];
    if (c1_ok) s_red[wave][g][c0 + 1] = acc1[g];
  }
  __syncthreads();
  for (int e = tid; e < G * dv; e += 256) {
    const int g = e / dv, c = e - g * dv;
    const float s = s_red[0][g][c] + s_red[1][g][c] + s_red[2][g][c] + s_red[3][g][c];
    const long long hq = static_cast<long long>(b) * a.n_q + h * G + g;
    if (a.direct_out) {
      const float l = s_l[g];
      a.out[hq * dv + c] = l > 0.f ? s / l : 0.f;
    } else {
      a.part_acc[(hq * a.n_slots + split) * dv + c] = s;
    }
  }
  if (a.n_split > 1 && tid < G) {
    const long long hq = static_cast<long long>(b) * a.n_q + h * G + tid;
    a.part_ml[(hq * a.n_slots + split) * 2 + 0] = s_m[tid];
    a.part_ml[(hq * a.n_slots + split) * 2 + 1] = s_l[tid];
  }
}

template <int G>
hipError_t launch_g(const DecodeArgs& a, hipStream_t stream) {
  dim3 grid(a.n_split, a.n_kv, a.batch), block(256);
  const int npl = (a.n_pairs + 15) / 16;
  switch (npl) {
    case 1: hipLaunchKernelGGL((decode_valu_kernel<G, 1>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((decode_valu_kernel<G, 2>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((decode_valu_kernel<G, 3>), grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((decode_valu_kernel<G, 4>), grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_valu(const DecodeArgs& a, hipStream_t stream) {
  switch (a.group) {
    case 1: return launch_g<1>(a, stream);
    case 2: return launch_g<2>(a, stream);
    case 3: return launch_g<3>(a, stream);
    case 4: return launch_g<4>(a, stream);
    case 5: return launch_g<5>(a, stream);
    case 6: return launch_g<6>(a, stream);
    case 7: return launch_g<7>(a, stream);
    case 8: return launch_g<8>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace rap
