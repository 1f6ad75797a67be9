// Forward kernel for rows whose support is small (the regime the paper's
// ASEntmax workloads live in: a handful of non-zero probabilities per row).
//
// alpha-entmax gives exact zeros below the threshold (Sec. 2.2, App. A), and the
// threshold is bounded below by any sub-problem: solving eq. (entmax) on a
// subset S of the row's scores gives tau_S <= tau, because dropping terms can
// only lower f(tau) = sum_j [(alpha-1) s_j - tau]_+^r - 1.  So after
//   1. a row-max sweep (Q K^T on the matrix cores) that also keeps the second
//      largest per-cell maximum, tau_lb = max(bracket's left end of App. A
//      eq. (bounds), two-element solution) is a valid lower bound, and
//   2. a second Q K^T sweep appends every key with (alpha-1) s_ij > tau_lb to
//      the row's candidate list (index + raw score) -- every key of the support
//      is on that list, nothing else of the row can matter --
// the rest is done on the lists alone, with no further sweep:
//   3. the threshold by the same safeguarded steps as the tiled kernel
//      (closed-form local-model root for alpha 1.5 / 2, Halley / Newton
//      otherwise), summing over the list instead of over key tiles,
//   4. O_i = sum over the list of p_ij v_j by gathering the few value rows.
// A workgroup that meets a row with more candidates than a list holds raises
// its flag and leaves the whole block to the tiled kernel (fwd.hip.h), which
// handles any density.
#pragma once
#include "fwd.hip.h"

namespace entmax {

constexpr int kCandCap = 32;  // candidates per lane = per half row; a row holds up to 2 * kCandCap

struct FwdSparseArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* tau;
  uint2* cand;          // [B*H*Nq][2][kCandCap] (key index, raw dot product bits)
  int* dense_flag;      // [B*H*nqb] 1: block left to the tiled kernel
  int* head_flag;       // [B*H] pre-zeroed; set to 1 when some block of the head is left to the tiled kernel
  unsigned long long* stats;
  int nqb;
};

template <typename T, int D, int AM>
__device__ __forceinline__ void fwd_sparse_block(const FwdSparseArgs& A, int bh_, int blk_, char* smem) {
  using C = QCtx<T, D, FwdTile<T>::value>;
  constexpr int KT = C::KT, NSB = C::NSB, TB = C::kTileBytes;
  const Geom& g = A.g;
  char* tiles = smem;  // 2 buffers x 1 slot
  int* ovf = reinterpret_cast<int*>(smem + 2 * TB);  // [2] sticky overflow flags, by tile parity

  C q;
  q.init(g, A.Q, bh_, blk_);
  const float r = 1.0f / (g.alpha - 1.0f);
  float* tau_out = A.tau + (long long)q.bh * g.Nq;
  const long long o_base = (long long)q.b * g.q_sb + (long long)q.h * g.q_sh;
  const int flag_idx = q.bh * A.nqb + q.qb;

  if (q.block_lim == 0) {  // no row of this workgroup sees any key
    for (int e = q.tid; e < kBlockRows * D; e += kThreads) {
      int row = q.qb * kBlockRows + e / D;
      if (row < g.Nq) Elem<T>::store(A.O, o_base + (long long)row * g.q_sn + e % D, 0.f);
    }
    if (q.tid < kBlockRows && q.qb * kBlockRows + q.tid < g.Nq) tau_out[q.qb * kBlockRows + q.tid] = 0.f;
    if (q.tid == 0) A.dense_flag[flag_idx] = 0;
    return;
  }
  if (q.tid < 2) ovf[q.tid] = 0;

  Slot slots[1];
  slots[0].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.K) + (long long)q.b * g.kv_sb +
                                                (long long)q.h * g.kv_sh);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);

  auto mask_block = [&](f32x16_t& acc, int j0) {
    int rel = q.lim - j0;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = (q.key_of(e) < rel) ? acc[e] : -kInf;
  };
  unsigned n_vis = 0, n_qk2 = 0, n_cand_tiles = 0;

  // ---------------------------------------------- 1. row max and runner-up
  // m1 >= m2 are the two largest per-cell maxima seen by this lane: two distinct scores of the row
  float m1 = -kInf, m2 = -kInf;
  sweep_tiles<C, T, D, 1, 0>(
      tiles, slots, q.ntiles, g.Nk, q.tid, [](int) { return true; },
      [&](int kt, const char* tl) {
        if ((kt + 1) * KT <= q.wave_lim_min) {
          f32x16_t acc[NSB];
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb) acc[sb] = q.scores(tl, sb);
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb) {
            float lm = max16(acc[sb]);
            m2 = fmaxf(m2, fminf(m1, lm));
            m1 = fmaxf(m1, lm);
          }
          n_vis += NSB;
          return;
        }
        const uint32_t act = q.visible_bits(kt);
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) {
          if (!(act & (1u << sb))) continue;
          int j0 = kt * KT + sb * 32;
          f32x16_t acc = q.scores(tl, sb);
          ++n_vis;
          if (j0 + 32 > q.wave_lim_min) mask_block(acc, j0);
          float lm = max16(acc);
          m2 = fmaxf(m2, fminf(m1, lm));
          m1 = fmaxf(m1, lm);
        }
      });
  {
    float p1 = __shfl_xor(m1, 32), p2 = __shfl_xor(m2, 32);
    float hi1 = fmaxf(m1, p1);
    m2 = fmaxf(fminf(m1, p1), fmaxf(m2, p2));
    m1 = hi1;
  }

  const bool live = q.valid && q.lim > 0;
  const float y1 = live ? q.a * m1 : 0.f;
  float lo = y1 - 1.0f;  // App. A eq. (bounds), left end
  float hi = live ? y1 - __builtin_amdgcn_exp2f(-(g.alpha - 1.0f) * __builtin_amdgcn_logf((float)q.lim)) : 0.f;
  if (live && m2 > -kInf) {
    // two-element sub-problem {y1, y2}: its threshold is a lower bound of the row's
    float dlt = y1 - q.a * m2;
    if (AM == 1 && dlt < 1.0f) lo = fmaxf(lo, 0.5f * (y1 + q.a * m2) - sqrtf(0.5f * (1.0f - 0.5f * dlt * dlt)));
    if (AM == 2 && dlt < 1.0f) lo = fmaxf(lo, 0.5f * (y1 + q.a * m2 - 1.0f));
  }
  lo = fminf(lo, hi);
  const float tau_lb = lo;

  // ---------------------------------------------- 2. candidate lists at tau_lb
  uint2* mylist = A.cand + (((long long)q.bh * g.Nq + (q.valid ? q.i : 0)) * 2 + q.hh) * kCandCap;
  int cnt = 0;
  sweep_tiles<C, T, D, 1, 0>(
      tiles, slots, q.ntiles, g.Nk, q.tid, [](int) { return true; },
      [&](int kt, const char* tl) {
        const bool interior = (kt + 1) * KT <= q.wave_lim_min;
        const uint32_t act = interior ? ((1u << NSB) - 1u) : q.visible_bits(kt);
        f32x16_t acc[NSB];
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb)
          if (act & (1u << sb)) acc[sb] = q.scores(tl, sb);
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) {
          if (!(act & (1u << sb))) continue;
          int j0 = kt * KT + sb * 32;
          ++n_qk2;
          if (!interior && j0 + 32 > q.wave_lim_min) mask_block(acc[sb], j0);
          float lm = max16(acc[sb]);
          bool cand = live && (lm > -kInf) && (fmaf(lm, q.a, -tau_lb) > 0.f);
          if (__ballot(cand) == 0ull) continue;
          ++n_cand_tiles;
          if (cand) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              float d = acc[sb][e];
              if ((d > -kInf) && (fmaf(d, q.a, -tau_lb) > 0.f)) {
                if (cnt < kCandCap) mylist[cnt] = make_uint2((unsigned)(j0 + q.key_of(e)), __float_as_uint(d));
                ++cnt;
              }
            }
          }
          if (__ballot(cnt > kCandCap) != 0ull && q.lane == 0) ovf[kt & 1] = 1;
        }
      },
      // flags of the previous tile's parity were final before the barrier that ended that tile
      [&](int kt) { return kt > 0 && ovf[(kt - 1) & 1] != 0; });
  // the sweep ended on a barrier: both flags are final
  const bool overflow = (ovf[0] | ovf[1]) != 0;
  if (overflow) {
    if (q.tid == 0) {
      A.dense_flag[flag_idx] = 1;
      A.head_flag[q.bh] = 1;
    }
    if (A.stats && q.lane == 0) {
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_TILES_VISIBLE], (unsigned long long)n_vis);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_LIST_QK], (unsigned long long)(n_vis + n_qk2));
    }
    return;
  }
  if (q.tid == 0) A.dense_flag[flag_idx] = 0;

  // ---------------------------------------------- 3 + 4. threshold and output from the lists
  // make this wave's own list stores visible to its own loads
  __threadfence_block();
  const T* Vbh = reinterpret_cast<const T*>(A.V) + (long long)q.b * g.kv_sb + (long long)q.h * g.kv_sh;
  unsigned n_support = 0;
  float tau = tau_lb;
  // NE: list entries per lane held in registers; chosen per wave from the longest list it holds
  auto finish = [&](auto ne_tag) {
    constexpr int NE = decltype(ne_tag)::value;
    float yv[NE];
    unsigned jv[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      uint2 en = (e < cnt) ? mylist[e] : make_uint2(0u, 0u);
      jv[e] = en.x;
      yv[e] = (e < cnt) ? q.a * __uint_as_float(en.y) : -kInf;  // -inf: never positive
    }
    bool done = !live;
    int iter = 0;
    while (__ballot(!done) != 0ull && iter < kMaxSolveIters) {
      RowSums sums;
      sums.clear();
#pragma unroll
      for (int e = 0; e < NE; ++e) accumulate<AM>(sums, yv[e] - tau, r);
      sums.combine_halves();
      if (!done) done = solve_step<AM>(sums, r, tau, lo, hi);
      ++iter;
    }
    // O = sum p_j v_j: each lane of a pair takes half of the features of every entry of the row
    constexpr int DH = D / 2;
    float oacc[DH];
#pragma unroll
    for (int t = 0; t < DH; ++t) oacc[t] = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int e = 0; e < NE; ++e) {
        float p_own = live ? pow_r<AM>(fmaxf(yv[e] - tau, 0.f), r) : 0.f;
        // half 0: the lane's own entry; half 1: its partner's entry
        float p = half == 0 ? p_own : __shfl_xor(p_own, 32);
        unsigned j = half == 0 ? jv[e] : (unsigned)__shfl_xor((int)jv[e], 32);
        if (__ballot(p > 0.f) == 0ull) continue;
        if (half == 0 && p > 0.f) ++n_support;
        if (p > 0.f) {
          const T* vrow = Vbh + (long long)j * g.kv_sn + q.hh * DH;
          if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int c8 = 0; c8 < DH / 8; ++c8) {
              u32x4_t w = *reinterpret_cast<const u32x4_t*>(vrow + 8 * c8);
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                oacc[8 * c8 + 2 * k] = fmaf(p, __uint_as_float(w[k] << 16), oacc[8 * c8 + 2 * k]);
                oacc[8 * c8 + 2 * k + 1] = fmaf(p, __uint_as_float(w[k] & 0xffff0000u), oacc[8 * c8 + 2 * k + 1]);
              }
            }
          } else {
#pragma unroll
            for (int c4 = 0; c4 < DH / 4; ++c4) {
              f32x4_t w = *reinterpret_cast<const f32x4_t*>(vrow + 4 * c4);
#pragma unroll
              for (int k = 0; k < 4; ++k) oacc[4 * c4 + k] = fmaf(p, w[k], oacc[4 * c4 + k]);
            }
          }
        }
      }
    }
    if (q.valid) {
      T* orow = reinterpret_cast<T*>(A.O) + o_base + (long long)q.i * g.q_sn + q.hh * DH;
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int c8 = 0; c8 < DH / 8; ++c8) *reinterpret_cast<u32x4_t*>(orow + 8 * c8) = Elem<T>::pack(oacc + 8 * c8).v;
      } else {
#pragma unroll
        for (int c4 = 0; c4 < DH / 4; ++c4)
          *reinterpret_cast<f32x4_t*>(orow + 4 * c4) =
              f32x4_t{oacc[4 * c4], oacc[4 * c4 + 1], oacc[4 * c4 + 2], oacc[4 * c4 + 3]};
      }
      if (q.hh == 0) tau_out[q.i] = live ? tau : 0.f;
    }
  };
  if (__ballot(cnt > 8) == 0ull)
    finish(std::integral_constant<int, 8>());
  else
    finish(std::integral_constant<int, kCandCap>());

  if (A.stats) {
    // per-wave totals of the per-lane counters
    unsigned sup = n_support, cands = (unsigned)cnt;
    for (int s = 32; s > 0; s >>= 1) {
      sup += __shfl_xor((int)sup, s);
      cands += __shfl_xor((int)cands, s);
    }
    if (q.lane == 0) {
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_TILES_VISIBLE], (unsigned long long)n_vis);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_LIST_QK], (unsigned long long)(n_vis + n_qk2));
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_CAND_TILES], (unsigned long long)n_cand_tiles);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_CANDIDATES], (unsigned long long)cands);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_SUPPORT], (unsigned long long)sup);
      if (q.wave == 0) atomicAdd(&A.stats[ENTMAX_STAT_FWD_SPARSE_BLOCKS], 1ull);
    }
  }
}

template <typename T, int D, int AM>
__global__ __launch_bounds__(kThreads, 3) void fwd_sparse_kernel(FwdSparseArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const PairItem it = pair_item(A.nqb);
  for (int part = 0; part < 2; ++part) {
    const int blk = part ? it.second : it.first;
    if (blk < 0) break;
    if (part) __syncthreads();
    fwd_sparse_block<T, D, AM>(A, it.bh, blk, smem);
  }
}

}  // namespace entmax
