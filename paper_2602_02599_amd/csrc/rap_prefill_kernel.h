// Causal prefill attention over the compact cache: rap_prefill_attn.  The kernel and its table of
// instantiations, included by one source file per score width (rap_prefill_k1.hip .. _k4.hip) so
// that they compile side by side.
//
// Eq. (attn) for the last n_new tokens of every sequence at once, each token seeing the cache rows
// up to and including its own (the decoder-only rule), at the pruned widths d_k = 2P and d_v.
// Unlike the decode step this is a dense contraction (n_new x len scores per head), so it is
// bound by the matrix cores, and the design is about feeding them:
//
//  * A workgroup takes a block of consecutive query tokens of one (sequence, KV head) together
//    with all G query heads of that KV head: its 64 NQ "columns" are (token, head) pairs, so a K
//    or V tile staged in LDS once serves G times as many scores as it would per head.
//  * Everything is computed transposed, as in the decode kernel: S^T[key][column] = K_tile . q on
//    v_mfma_f32_16x16x32_bf16 with the K tile as the A operand from LDS and the query columns,
//    resident in registers, as the B operand; in the result layout a lane holds eight keys of one
//    column, which are exactly the contraction slots of the P.V instruction when those are
//    numbered accordingly, so probabilities never leave the lane.  A K fragment read from LDS is
//    used for NQ column blocks, and so is the gathered V operand.
//  * Tiles of 64 keys are staged by the whole workgroup: 16-byte loads that write LDS themselves,
//    issued one tile ahead into the other buffer, one barrier per tile.
//  * Online softmax in the log2 domain against a per-column reference that moves only when a
//    score outgrows it by 2^64; the causal mask is applied only on the tiles that straddle the
//    diagonal of the wavefront's columns, later tiles are skipped by the wavefront, earlier ones
//    need no mask.
//
// Paged caches: with a block table the caches are pools of pages of at least 64 rows, a staged
// tile never straddles two pages, and only its start address changes (looked up a tile ahead).
//
// Garbage safety: rows at or beyond the sequence length may hold any bits; their scores are never
// visible (a select to -inf), their V rows are cleared on the way into LDS, K fragments are masked
// beyond d_k, and loads never touch rows >= round-up-8(len) <= cap.
#ifndef RAP_PREFILL_KERNEL_H_
#define RAP_PREFILL_KERNEL_H_

#include <utility>

#include "rap_device.h"

namespace rap {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(1))) const void* global_ptr_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// maximum of three floats in one instruction.  Written as the instruction because the compiler,
// asked for nested two-operand maxima of matrix-instruction results, first passes every operand
// through a max(x, x) of its own to quiet a possible signalling NaN: eleven instructions where
// three do (the instruction quiets NaNs by itself).
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

constexpr int kKeysPerTile = 64;     // staged per barrier
constexpr int kSub = 32;             // keys per matrix-instruction group (two 16-row fragments)
// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a
// constant inside the body (register arrays must never be indexed by a run-time value)
template <int... Is, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>()), ...);
}

constexpr float kHeadroomP = 64.f;   // log2 units a score may exceed the reference before a rescale

// Q8: the caches hold one-byte E4M3 codes (value = code value x the scale of the KV head): rows and
// tiles are half as long, a fragment is widened to bf16 (exactly) between LDS and the matrix
// instruction, k_scale folds into the softmax scale and v_scale into the final normalisation.
template <int KCH, int NT, bool VPAIR, int NQ, bool ONES, bool Q8, bool PADL>
__global__ __launch_bounds__(256, 2) void prefill_kernel(PrefillArgs a) {
  constexpr int EB = Q8 ? 1 : 2;                                      // bytes per cache element
  constexpr int NCK = (kKeysPerTile * 32 * EB * KCH + 4095) / 4096;   // 16-byte chunks per thread, K tile
  constexpr int NCV = (kKeysPerTile * 16 * EB * NT + 4095) / 4096;    // same, V tile
  // the same when every row is followed by a 16-byte gap in LDS (direct loads of padded rows)
  constexpr int NCKP = (kKeysPerTile * (32 * EB * KCH + 16) + 4095) / 4096;
  constexpr int NCVP = (kKeysPerTile * (16 * EB * NT + 16) + 4095) / 4096;
  extern __shared__ __align__(16) unsigned char smem[];

  int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15;
  const int lg = lane >> 4;

  // heaviest query blocks (the last tokens, which see the most rows) first
  // (with key ranges: consecutive workgroups are the ranges of one query block)
  const int slabs = a.n_kv * a.batch;
  const int ks = a.n_ksplit > 1 ? static_cast<int>(blockIdx.x % a.n_ksplit) : 0;
  const int wg = a.n_ksplit > 1 ? static_cast<int>(blockIdx.x / a.n_ksplit) : static_cast<int>(blockIdx.x);
  const int qb = a.n_qblk - 1 - wg / slabs;
  const int slab_id = wg - (wg / slabs) * slabs;
  const int h = slab_id % a.n_kv;
  const int b = slab_id / a.n_kv;

  int len = a.seq_lens[b];
  len = len < 0 ? 0 : (len > a.max_len ? a.max_len : len);
  const int G = a.group;
  const int dk = a.d_k, dv = a.d_v;
  const int BT = a.tok_per_wg;
  const int i0 = qb * BT;
  const int i_end = min(a.n_new, i0 + BT);
  const int shift = len - a.n_new;                 // position of token i is shift + i
  const int n_keys = min(len, shift + i_end);      // rows the block's last token sees
  const long long out_row0 = (static_cast<long long>(b) * a.n_new) * a.n_q + h * G;   // + i * n_q + g

  const int n_tiles_all = (n_keys + kKeysPerTile - 1) / kKeysPerTile;
  const int t_first = ks * a.tiles_per_split;                       // key range of this workgroup, in tiles
  const int n_tiles = a.n_ksplit > 1 ? min(n_tiles_all, t_first + a.tiles_per_split) : n_tiles_all;
  if (a.n_ksplit > 1 && t_first >= n_tiles) {
    // nothing of this range is visible to the block (or the block lies before the start of its
    // sequence): empty partials, which the combining kernel drops
    for (int r = tid; r < (i_end - i0) * G; r += 256) {
      const int g = r % G, i = i0 + r / G;
      const long long slot = (out_row0 + static_cast<long long>(i) * a.n_q + g) * a.n_ksplit + ks;
      a.part_ml[slot * 2 + 0] = -INFINITY;
      a.part_ml[slot * 2 + 1] = 0.f;
    }
    return;
  }
  if (n_keys <= 0) {
    // every token of this block lies before the start of its sequence: zero rows
    for (int e = tid; e < (i_end - i0) * G * dv; e += 256) {
      const int c = e % dv, r = e / dv;
      const int g = r % G, i = i0 + r / G;
      a.out[(out_row0 + static_cast<long long>(i) * a.n_q + g) * dv + c] = 0.f;
    }
    return;
  }

  // ---- this lane's columns: (token, head) pairs, and their positions
  int pos_col[NQ];
  bool col_valid[NQ];
  int wmin = 0x7fffffff, wmax = -1;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int cw = (wave * NQ + nq) * 16 + l16;
    const int tl = cw / G;
    const int i = i0 + tl;
    col_valid[nq] = tl < BT && i < a.n_new && shift + i >= 0;
    pos_col[nq] = col_valid[nq] ? shift + i : 0;
    wmin = min(wmin, col_valid[nq] ? pos_col[nq] : 0x7fffffff);
    wmax = max(wmax, col_valid[nq] ? pos_col[nq] : -1);
  }
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) {
    wmin = min(wmin, __shfl_xor(wmin, o));
    wmax = max(wmax, __shfl_xor(wmax, o));
  }
  wmin = __builtin_amdgcn_readfirstlane(wmin);
  wmax = __builtin_amdgcn_readfirstlane(wmax);

  // ---- query columns as the B operand: lane (l16 = column, lg = k sub-chunk)
  bf16x8 qf[NQ][KCH];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int cw = (wave * NQ + nq) * 16 + l16;
    const int tl = cw / G, g = cw - (cw / G) * G;
    const uint32_t* qrow = reinterpret_cast<const uint32_t*>(a.q) +
                           ((static_cast<long long>(b) * a.n_new + (col_valid[nq] ? i0 + tl : 0)) * a.n_q + h * G +
                            (col_valid[nq] ? g : 0)) * (dk / 2);
#pragma unroll
    for (int kk = 0; kk < KCH; ++kk) {
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = 32 * kk + 8 * lg + 2 * i;
        w[i] = (col_valid[nq] && e < dk) ? qrow[e >> 1] : 0u;
      }
      qf[nq][kk] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
  }

  const int pitch_k = EB * dk, pitch_v = EB * dv;  // bytes, in the cache
  const float scale_l2e = Q8 ? a.scale_log2e * a.k_scale[h] : a.scale_log2e;
  // In LDS a row pitch that is a multiple of 128 bytes gets 16 bytes of padding: otherwise the 16
  // rows a fragment read touches would all start in the same bank.
  const int lpk = pitch_k + a.pad_k, lpv = pitch_v + a.pad_v;
  const long long slab = static_cast<long long>(b) * a.n_kv + h;
  const bool paged = a.block_table != nullptr;
  const unsigned char* kslab = reinterpret_cast<const unsigned char*>(a.k_cache) + (paged ? 0 : slab * a.cap * pitch_k);
  const unsigned char* vslab = reinterpret_cast<const unsigned char*>(a.v_cache) + (paged ? 0 : slab * a.cap * pitch_v);
  // row of the (b, h) slab, or of the pool, where the tile that starts at logical row `row` lies
  // (a page number outside the pool is clamped into it)
  auto tile_row = [&](int row) -> long long {
    if (!paged) return row;
    int pg = a.block_table[static_cast<long long>(b) * a.max_pages + (row >> a.page_shift)];
    pg = pg < 0 ? 0 : (pg >= a.n_pages ? a.n_pages - 1 : pg);
    return ((static_cast<long long>(pg) * a.n_kv + h) << a.page_shift) + (row & ((1 << a.page_shift) - 1));
  };
  // rows below len8 are readable: <= cache_cap (a multiple of 8, of 16 for one-byte elements, which
  // keeps every such group of rows 16-byte aligned whatever the row width)
  const int len8 = Q8 ? (len + 15) & ~15 : (len + 7) & ~7;
  const int v_off = (kKeysPerTile * lpk + 64 + 127) & ~127;   // slack: the last K fragment read runs past the tile

  // The 16-byte global loads write LDS themselves (lane i of a wavefront lands at the wavefront's
  // LDS base + 16 i): no staging registers.  Without LDS padding the tile is a flat copy.  With
  // padded rows (PADL) where a lane's 16 bytes land is just as fixed, but where they come from is
  // not: the lane whose slot is piece p of padded row r loads piece p of cache row r, and the
  // lanes whose slot is a gap load nothing.  Offsets into the cache tile per lane and load are
  // worked out once (no load: an offset beyond any tile).
  constexpr int NDK = PADL ? NCKP : NCK, NDV = PADL ? NCVP : NCV;
  int kgo[PADL ? NCKP : 1], vgo[PADL ? NCVP : 1];
  if constexpr (PADL) {
    const int cprk = (pitch_k >> 4) + 1, cprv = (pitch_v >> 4) + 1;   // 16-byte slots per padded row
#pragma unroll
    for (int j = 0; j < NCKP; ++j) {
      const int c = j * 256 + tid, row = c / cprk, piece = c - row * cprk;
      kgo[j] = a.pad_k ? (piece < cprk - 1 ? row * pitch_k + piece * 16 : 0x7fffffff) : c * 16;
    }
#pragma unroll
    for (int j = 0; j < NCVP; ++j) {
      const int c = j * 256 + tid, row = c / cprv, piece = c - row * cprv;
      vgo[j] = a.pad_v ? (piece < cprv - 1 ? row * pitch_v + piece * 16 : 0x7fffffff) : c * 16;
    }
  }
  auto issue_direct = [&](int t, long long trow) {
    const int base = t * kKeysPerTile;
    const int rows = min(kKeysPerTile, len8 - base);
    const int kval = rows * pitch_k, vval = rows * pitch_v;
    const unsigned char* kg = kslab + trow * pitch_k;
    const unsigned char* vg = vslab + trow * pitch_v;
    unsigned char* kt = smem + (t & 1) * a.lds_buf_bytes;
    unsigned char* vt = kt + v_off;
#pragma unroll
    for (int j = 0; j < NDK; ++j) {
      const int off = PADL ? kgo[PADL ? j : 0] : (j * 256 + tid) * 16;
      if (off < kval)
        __builtin_amdgcn_global_load_lds((global_ptr_t)(kg + off), (lds_ptr_t)(kt + (j * 256 + wave * 64) * 16), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < NDV; ++j) {
      const int off = PADL ? vgo[PADL ? j : 0] : (j * 256 + tid) * 16;
      if (off < vval)
        __builtin_amdgcn_global_load_lds((global_ptr_t)(vg + off), (lds_ptr_t)(vt + (j * 256 + wave * 64) * 16), 16, 0, 0);
    }
  };

  f32x4 acc[NQ][NT];
  float m_run[NQ], l_run[NQ];
  float nref[NQ];      // minus the reference as the exponent's addend: kept beside m_run, 0 while that is -inf
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m_run[nq] = -INFINITY;
    nref[nq] = 0.f;
    l_run[nq] = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nq][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // A spare channel slot (d_v not a multiple of 16) carries the constant 1, so that the row sums
  // of the probabilities come out of the P.V product: slot l16 = 15 of the last channel tile.
  const int klim = dk - 32 * (KCH - 1) - 8 * lg;   // elements of this lane's last K fragment that exist
  // one-byte elements: the same limit as byte masks of the fragment's two words (d_k is even)
  uint32_t kmask8[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int left = klim - 4 * i;
    kmask8[i] = left >= 4 ? 0xffffffffu : (left >= 2 ? 0x0000ffffu : 0u);
  }
  int koff[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) koff[rt] = (16 * rt + l16) * lpk + 8 * EB * lg;
  int voff[2][4];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int r = 0; r < 4; ++r) voff[rt][r] = (16 * rt + 4 * lg + r) * lpv + (VPAIR ? 2 : 1) * EB * l16;

  // start row of the tile whose loads are issued next, looked up (paged) one tile ahead of them
  long long trow_next;
  auto row_of_tile = [&](int t) -> long long { return t < n_tiles ? tile_row(t * kKeysPerTile) : 0; };
  issue_direct(t_first, row_of_tile(t_first));
  trow_next = row_of_tile(t_first + 1);

  for (int t = t_first; t < n_tiles; ++t) {
    unsigned char* kt0 = smem + (t & 1) * a.lds_buf_bytes;
    unsigned char* vt0 = kt0 + v_off;
    __builtin_amdgcn_s_waitcnt(0);         // this wavefront's share of tile t has landed
    __syncthreads();                       // everybody's has, and nobody still reads the other buffer
    if (t + 1 < n_tiles) issue_direct(t + 1, trow_next);
    trow_next = row_of_tile(t + 2);
    if ((t + 1) * kKeysPerTile > len) {
      // The V rows at or beyond the sequence length may hold anything (NaN included) and a zero
      // probability does not silence a NaN: in the one tile that holds the end of the sequence
      // they are cleared in LDS before use.
      for (int o = (len - t * kKeysPerTile) * lpv + 2 * tid; o < kKeysPerTile * lpv; o += 512)
        *reinterpret_cast<uint16_t*>(vt0 + o) = 0;
      __syncthreads();
    }
#pragma unroll 1
    for (int sub = 0; sub < kKeysPerTile / kSub; ++sub) {
      const int sbase = t * kKeysPerTile + kSub * sub;
      if (sbase > wmax || sbase >= n_keys) break;   // nothing of this or any later key group is visible here
      const unsigned char* kt = kt0 + sub * kSub * lpk;
      const unsigned char* vt = vt0 + sub * kSub * lpv;
      const bool no_mask = sbase + kSub - 1 <= wmin;

      // ---- A. scores sc[nq][rt][r] = column (nq, l16) . K[sbase + 16 rt + 4 lg + r]
      f32x4 sc[NQ][2];
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) sc[nq][0] = sc[nq][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
        for (int kk = 0; kk < KCH; ++kk) {
          uint4 w;
          if constexpr (Q8) {
            const uint16_t* p = reinterpret_cast<const uint16_t*>(kt + koff[rt] + 32 * kk);   // rows are 2-byte aligned
            uint32_t c0 = p[0] | (static_cast<uint32_t>(p[1]) << 16), c1 = p[2] | (static_cast<uint32_t>(p[3]) << 16);
            if (kk == KCH - 1) {
              c0 &= kmask8[0];
              c1 &= kmask8[1];
            }
            w = widen_e4m3x8(c0, c1);
          } else {
            const uint32_t* p = reinterpret_cast<const uint32_t*>(kt + koff[rt] + 64 * kk);
            w = make_uint4(p[0], p[1], p[2], p[3]);
            if (kk == KCH - 1) {                      // beyond d_k lies the next row (or stale LDS)
              w.x = klim > 0 ? w.x : 0u;
              w.y = klim > 2 ? w.y : 0u;
              w.z = klim > 4 ? w.z : 0u;
              w.w = klim > 6 ? w.w : 0u;
            }
          }
          const bf16x8 kf = __builtin_bit_cast(bf16x8, w);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            sc[nq][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[nq][kk], sc[nq][rt], 0, 0, 0);
        }
      }
      // ---- B. the visibility test where the group straddles the diagonal of this wavefront's
      // columns, block maxima, and the rare move of a reference.  With all 32 keys visible and a
      // non-negative scale the raw scores stay as they are: scale and reference then fold into
      // one multiply-add per score (mul), and the maximum is scaled instead of the scores.
      bool grow = false;
      const bool raw = no_mask && scale_l2e >= 0.f;
      const float mul = raw ? scale_l2e : 1.f;
      if (!raw) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
          const int rel = no_mask ? kSub : pos_col[nq] - sbase;   // keys 0..rel of the group are visible to this column
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              sc[nq][rt][r] = (16 * rt + 4 * lg + r) <= rel ? sc[nq][rt][r] * scale_l2e : -INFINITY;
        }
      }
      float tmax[NQ];
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        tmax[nq] = max3(max3(sc[nq][0][0], sc[nq][0][1], sc[nq][0][2]), max3(sc[nq][0][3], sc[nq][1][0], sc[nq][1][1]),
                        max3(sc[nq][1][2], sc[nq][1][3], sc[nq][1][3])) * mul;
        grow = grow || tmax[nq] > m_run[nq] + kHeadroomP;
      }
      if (__any(grow)) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
          float tm = fmaxf(tmax[nq], __shfl_xor(tmax[nq], 16));
          tm = fmaxf(tm, __shfl_xor(tm, 32));
          const float m_new = fmaxf(m_run[nq], tm);
          // a column that has seen nothing yet and sees nothing here keeps its -inf reference
          const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_run[nq] - m_new) : 0.f;
          l_run[nq] *= alpha;
#pragma unroll
          for (int reg = 0; reg < 4; ++reg) {
            const float at = __shfl(alpha, 4 * lg + reg);   // the column this accumulator register holds
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nq][nt][reg] *= at;
          }
          m_run[nq] = m_new;
          nref[nq] = m_new > -INFINITY ? -m_new : 0.f;      // -inf - -inf would be NaN
        }
      }

      // ---- C. numerators, packed straight into the P.V operand: a bf16 head and a bf16 remainder
      // of every probability (16 significant bits).  The remainder is p minus the head widened
      // back (a shift or a mask, then a subtraction: exact).  A two-term dot instruction
      // (head . (-1, 0) + p) does the same in one instruction instead of two, but it runs on the
      // matrix pipeline: measured on this part, sixteen matrix instructions with two such dot
      // instructions after each take 254 ns against 120 ns with two multiply-adds, conversions or
      // permutes after each, which all hide completely; the one-instruction form made this kernel
      // slower, not faster.
      uint4 p_hi[NQ], p_lo[NQ];
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        float pr[2][4];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int r = 0; r < 4; ++r) pr[rt][r] = __builtin_amdgcn_exp2f(fmaf(sc[nq][rt][r], mul, nref[nq]));
        if constexpr (!ONES)                         // otherwise the sum comes out of the P.V product
          l_run[nq] += ((pr[0][0] + pr[0][1]) + (pr[0][2] + pr[0][3])) + ((pr[1][0] + pr[1][1]) + (pr[1][2] + pr[1][3]));
        uint32_t* ph = reinterpret_cast<uint32_t*>(&p_hi[nq]);
        uint32_t* pl = reinterpret_cast<uint32_t*>(&p_lo[nq]);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const float a0 = pr[d >> 1][2 * (d & 1)], a1 = pr[d >> 1][2 * (d & 1) + 1];
          const uint32_t hh = pack_bf16(a0, a1);
          ph[d] = hh;
          pl[d] = pack_bf16(a0 - bf16_lo(hh), a1 - bf16_hi(hh));
        }
      }

      // ---- D. P.V: acc[nq][nt][reg] (column 4 lg + reg of block nq, channel slot l16 of tile nt);
      // a gathered V operand serves all NQ blocks
      if constexpr (VPAIR) {
#pragma unroll
        for (int np = 0; np < NT / 2; ++np) {
          uint4 be, bo;   // even / odd channel of the pair, rows packed two by two
          if constexpr (Q8) {
            uint32_t hw[8];                // two adjacent channels of row j: even channel in the low byte
#pragma unroll
            for (int j = 0; j < 8; ++j) hw[j] = *reinterpret_cast<const uint16_t*>(vt + voff[j >> 2][j & 3] + 32 * np);
            // bytes of one channel over rows 0..3 and 4..7, then widened
            const uint32_t lo01 = __builtin_amdgcn_perm(hw[1], hw[0], 0x0c0c0400u), lo23 = __builtin_amdgcn_perm(hw[3], hw[2], 0x04000c0cu);
            const uint32_t lo45 = __builtin_amdgcn_perm(hw[5], hw[4], 0x0c0c0400u), lo67 = __builtin_amdgcn_perm(hw[7], hw[6], 0x04000c0cu);
            const uint32_t hi01 = __builtin_amdgcn_perm(hw[1], hw[0], 0x0c0c0501u), hi23 = __builtin_amdgcn_perm(hw[3], hw[2], 0x05010c0cu);
            const uint32_t hi45 = __builtin_amdgcn_perm(hw[5], hw[4], 0x0c0c0501u), hi67 = __builtin_amdgcn_perm(hw[7], hw[6], 0x05010c0cu);
            be = widen_e4m3x8(lo01 | lo23, lo45 | lo67);
            bo = widen_e4m3x8(hi01 | hi23, hi45 | hi67);
          } else {
            uint32_t w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = *reinterpret_cast<const uint32_t*>(vt + voff[j >> 2][j & 3] + 64 * np);
            be.x = __builtin_amdgcn_perm(w[1], w[0], 0x05040100u);
            be.y = __builtin_amdgcn_perm(w[3], w[2], 0x05040100u);
            be.z = __builtin_amdgcn_perm(w[5], w[4], 0x05040100u);
            be.w = __builtin_amdgcn_perm(w[7], w[6], 0x05040100u);
            bo.x = __builtin_amdgcn_perm(w[1], w[0], 0x07060302u);
            bo.y = __builtin_amdgcn_perm(w[3], w[2], 0x07060302u);
            bo.z = __builtin_amdgcn_perm(w[5], w[4], 0x07060302u);
            bo.w = __builtin_amdgcn_perm(w[7], w[6], 0x07060302u);
          }
          if (ONES && np == NT / 2 - 1 && l16 == 15) bo = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
          const bf16x8 vbe = __builtin_bit_cast(bf16x8, be), vbo = __builtin_bit_cast(bf16x8, bo);
          // heads of all column blocks first, remainders after: an accumulator's two instructions
          // then lie 2 NQ instructions apart, and the second never waits for the first
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            const bf16x8 pa_hi = __builtin_bit_cast(bf16x8, p_hi[nq]);
            acc[nq][2 * np] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vbe, acc[nq][2 * np], 0, 0, 0);
            acc[nq][2 * np + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vbo, acc[nq][2 * np + 1], 0, 0, 0);
          }
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            const bf16x8 pa_lo = __builtin_bit_cast(bf16x8, p_lo[nq]);
            acc[nq][2 * np] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vbe, acc[nq][2 * np], 0, 0, 0);
            acc[nq][2 * np + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vbo, acc[nq][2 * np + 1], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          uint32_t u[8];
          uint4 bv;
          if constexpr (Q8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) u[j] = *reinterpret_cast<const uint8_t*>(vt + voff[j >> 2][j & 3] + 16 * nt);
            bv = widen_e4m3x8(u[0] | (u[1] << 8) | (u[2] << 16) | (u[3] << 24), u[4] | (u[5] << 8) | (u[6] << 16) | (u[7] << 24));
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) u[j] = *reinterpret_cast<const uint16_t*>(vt + voff[j >> 2][j & 3] + 32 * nt);
            bv = make_uint4(u[0] | (u[1] << 16), u[2] | (u[3] << 16), u[4] | (u[5] << 16), u[6] | (u[7] << 16));
          }
          if (ONES && nt == NT - 1 && l16 == 15) bv = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
          const bf16x8 vb = __builtin_bit_cast(bf16x8, bv);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            acc[nq][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, p_hi[nq]), vb, acc[nq][nt], 0, 0, 0);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            acc[nq][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, p_lo[nq]), vb, acc[nq][nt], 0, 0, 0);
        }
      }
    }
  }

  // ---- normalise and store: accumulator register reg of lane (l16, lg) is column 4 lg + reg
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    float l = l_run[nq];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) {
      const int col = 4 * lg + reg;
      const float lc = ONES ? __shfl(acc[nq][NT - 1][reg], 16 * lg + 15) : __shfl(l, col);
      const int cw = (wave * NQ + nq) * 16 + col;
      const int tl = cw / G, g = cw - (cw / G) * G;
      const int i = i0 + tl;
      if (a.n_ksplit > 1) {
        // partial of this key range: reference (log2 units), sum, un-normalised accumulators
        const float mc = __shfl(m_run[nq], col);
        if (tl < BT && i < a.n_new) {
          const bool seen = shift + i >= 0 && mc > -INFINITY;
          const long long slot = (out_row0 + static_cast<long long>(i) * a.n_q + g) * a.n_ksplit + ks;
          if (l16 == 0) {
            a.part_ml[slot * 2 + 0] = seen ? mc : -INFINITY;
            a.part_ml[slot * 2 + 1] = seen ? lc : 0.f;
          }
          const float vsc = Q8 ? a.v_scale[h] : 1.f;      // codes -> values
          float* prow = a.part_acc + slot * dv;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int c = VPAIR ? 32 * (nt >> 1) + 2 * l16 + (nt & 1) : 16 * nt + l16;
            if (c < dv) prow[c] = seen ? acc[nq][nt][reg] * vsc : 0.f;
          }
        }
      } else if (tl < BT && i < a.n_new) {
        float inv = (shift + i >= 0 && lc > 0.f) ? 1.f / lc : 0.f;
        if constexpr (Q8) inv *= a.v_scale[h];       // codes -> values
        float* orow = a.out + (out_row0 + static_cast<long long>(i) * a.n_q + g) * dv;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const int c = VPAIR ? 32 * (nt >> 1) + 2 * l16 + (nt & 1) : 16 * nt + l16;
          if (c < dv) orow[c] = acc[nq][nt][reg] * inv;
        }
      }
    }
  }
}

template <int KCH, int NT, bool VPAIR, int NQ, bool ONES, bool Q8, bool PADL>
hipError_t launch_prefill_go3(const PrefillArgs& a, size_t lds, long long n_wg, hipStream_t stream) {
  if (lds > 64 * 1024) {
    const hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(&prefill_kernel<KCH, NT, VPAIR, NQ, ONES, Q8, PADL>), static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((prefill_kernel<KCH, NT, VPAIR, NQ, ONES, Q8, PADL>), dim3(static_cast<unsigned>(n_wg)), dim3(256), lds, stream, a);
  return hipGetLastError();
}

template <int KCH, int NT, bool VPAIR, int NQ, bool ONES, bool PADL>
hipError_t launch_prefill_go2(const PrefillArgs& a, size_t lds, long long n_wg, hipStream_t stream) {
  if (a.k_scale != nullptr) return launch_prefill_go3<KCH, NT, VPAIR, NQ, ONES, true, PADL>(a, lds, n_wg, stream);
  return launch_prefill_go3<KCH, NT, VPAIR, NQ, ONES, false, PADL>(a, lds, n_wg, stream);
}

// a spare channel slot exists exactly when d_v is not a multiple of 16
template <int KCH, int NT, bool VPAIR, int NQ, bool PADL>
hipError_t launch_prefill_go(const PrefillArgs& a, size_t lds, long long n_wg, hipStream_t stream) {
  if ((a.d_v & 15) != 0) return launch_prefill_go2<KCH, NT, VPAIR, NQ, true, PADL>(a, lds, n_wg, stream);
  return launch_prefill_go2<KCH, NT, VPAIR, NQ, false, PADL>(a, lds, n_wg, stream);
}

template <int KCH, int NT, bool VPAIR, int NQ>
hipError_t launch_prefill_inst(PrefillArgs a, hipStream_t stream) {
  // key ranges were planned for a block size: it has to be this instantiation's
  if (a.n_ksplit > 1 && a.tok_per_wg != (64 * NQ) / a.group) return hipErrorInvalidValue;
  a.tok_per_wg = (64 * NQ) / a.group;
  a.n_qblk = (a.n_new + a.tok_per_wg - 1) / a.tok_per_wg;
  // padded LDS rows for pitches of 128 or 256 bytes
  const int eb = a.k_scale != nullptr ? 1 : 2;        // bytes per cache element
  const int pk = eb * a.d_k, pv = eb * a.d_v;
  a.pad_k = (pk % 128 == 0) ? 16 : 0;
  a.pad_v = (pv % 128 == 0) ? 16 : 0;
  const int kbytes = kKeysPerTile * (pk + a.pad_k), vbytes = kKeysPerTile * (pv + a.pad_v);
  a.lds_buf_bytes = ((kbytes + 64 + 127) & ~127) + ((vbytes + 64 + 127) & ~127);
  const size_t lds = 2 * static_cast<size_t>(a.lds_buf_bytes);
  const long long n_wg = static_cast<long long>(a.n_qblk) * a.n_kv * a.batch * (a.n_ksplit > 1 ? a.n_ksplit : 1);
  if (n_wg > 0x7fffffffLL) return hipErrorInvalidValue;
  // padded rows only occur at 128- and 256-byte pitches (d = 64, 128; one-byte codes: d = 128)
  if constexpr ((KCH == 2 || KCH == 4) || (NT == 4 || NT == 8)) {
    if (a.pad_k || a.pad_v) return launch_prefill_go<KCH, NT, VPAIR, NQ, true>(a, lds, n_wg, stream);
  }
  return launch_prefill_go<KCH, NT, VPAIR, NQ, false>(a, lds, n_wg, stream);
}

template <int KCH, int NQ>
hipError_t launch_prefill_k(const PrefillArgs& a, hipStream_t stream) {
  const int nt = (a.d_v + 15) / 16;
  constexpr int NQW = NQ > kPrefillBlocksWide ? kPrefillBlocksWide : NQ;   // d_v > 96: four column blocks of accumulators do not fit the registers
  if ((a.d_v & 1) == 0 && (nt & 1) == 0) {
    switch (nt) {
      case 2: return launch_prefill_inst<KCH, 2, true, NQ>(a, stream);
      case 4: return launch_prefill_inst<KCH, 4, true, NQ>(a, stream);
      case 6: return launch_prefill_inst<KCH, 6, true, NQ>(a, stream);
      case 8: return launch_prefill_inst<KCH, 8, true, NQW>(a, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (nt) {
    case 1: return launch_prefill_inst<KCH, 1, false, NQ>(a, stream);
    case 2: return launch_prefill_inst<KCH, 2, false, NQ>(a, stream);
    case 3: return launch_prefill_inst<KCH, 3, false, NQ>(a, stream);
    case 4: return launch_prefill_inst<KCH, 4, false, NQ>(a, stream);
    case 5: return launch_prefill_inst<KCH, 5, false, NQ>(a, stream);
    case 6: return launch_prefill_inst<KCH, 6, false, NQ>(a, stream);
    case 7: return launch_prefill_inst<KCH, 7, false, NQW>(a, stream);
    case 8: return launch_prefill_inst<KCH, 8, false, NQW>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

}  // namespace rap

#endif  // RAP_PREFILL_KERNEL_H_
