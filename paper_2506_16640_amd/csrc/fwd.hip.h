// Forward kernel: alpha-entmax attention of Sec. 2.1 / eq. (entmax) on
// ASEntmax-scaled logits (eq. (asentmax)), one workgroup per 128 query rows of
// one (batch, head).
//
// Per workgroup, with every sweep recomputing Q K^T on the matrix cores from
// K tiles staged in LDS (the n x n scores are never stored):
//   1. row-max sweep                      -> bracket of App. A eq. (bounds):
//        (alpha-1) max - 1 <= tau <= (alpha-1) max - n_i^(1-alpha)
//   2. threshold sweeps: evaluate partial sums of
//        f(tau) = sum_j [(alpha-1) s_ij - tau]_+^r - 1,  r = 1/(alpha-1)
//      and take a safeguarded higher-order step inside the bracket (App. A,
//      "alpha-entmax computation": root finding with bisection as the fallback).
//      The first sweep runs at the lower bracket end, so the 32x32 tiles that
//      hold no positive term there can never hold one later (tau only grows
//      from that end): they are recorded per wave and skipped from then on.
//   3. P.V sweep: p = x^r, tiles whose p is all zero are skipped, the others
//      go through the matrix cores against the transposed V copy.
#pragma once
#include "qside.hip.h"

namespace entmax {

struct FwdArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* Vt;  // transposed, row-permuted copy of V: [B*H][D][npad_k]
  void* O;
  float* tau;
  unsigned long long* stats;
  int nqb;         // query blocks per head
  int mask_words;  // uint32 words of one wave's tile mask
  const int* dense_flag;  // NULL: run every block; else [B*H*nqb], run only the blocks whose flag is set
  const int* dense_count; // with dense_flag: the number of set flags, then the first kSplitMaxBlocks flagged blocks'
                          // numbers bh * nqb + qb in any order (decides how the blocks are shared out, see fwd_kernel)
  const float2* bounds;   // with dense_flag: [B*H*Nq]; for a block whose flag is kFlagWithBounds the list kernel left
                          // (lower bound of the threshold, (alpha-1) x largest score) of every row here
};

// values of a block's flag in dense_flag: left to the tiled kernel without / with the rows' bounds
constexpr int kFlagDense = 1;
constexpr int kFlagWithBounds = 2;

constexpr int kMaxSolveIters = 48;

// Partial sums of the threshold function over the lane's keys.
//   AM 1 (alpha 1.5, r 2): s0 = #positive, s1 = sum x,   s2 = sum x^2
//   AM 2 (alpha 2,   r 1): s0 = #positive, s1 = sum x
//   AM 3 (alpha 1.25,r 4): s0 = sum x^2,   s1 = sum x^3, s2 = sum x^4
//   AM 0 (generic)       : s0 = sum x^(r-1), s1 = sum x^r
// xmin is the smallest positive x (AM 1 and 2 only).
struct RowSums {
  float s0, s1, s2, xmin;
  __device__ __forceinline__ void clear() {
    s0 = s1 = s2 = 0.f;
    xmin = kInf;
  }
  __device__ __forceinline__ void combine_halves() {
    s0 += __shfl_xor(s0, 32);
    s1 += __shfl_xor(s1, 32);
    s2 += __shfl_xor(s2, 32);
    xmin = fminf(xmin, __shfl_xor(xmin, 32));
  }
};

template <int AM>
__device__ __forceinline__ void accumulate(RowSums& s, float xp, float r) {
  // xp = (alpha-1) s_ij - tau before clamping
  if (AM == 1) {
    bool pos = xp > 0.f;
    float x = fmaxf(xp, 0.f);
    s.s2 = fmaf(x, x, s.s2);
    s.s1 += x;
    s.s0 += pos ? 1.f : 0.f;
    s.xmin = pos ? fminf(s.xmin, xp) : s.xmin;
  } else if (AM == 2) {
    bool pos = xp > 0.f;
    float x = fmaxf(xp, 0.f);
    s.s1 += x;
    s.s0 += pos ? 1.f : 0.f;
    s.xmin = pos ? fminf(s.xmin, xp) : s.xmin;
  } else if (AM == 3) {
    float x = fmaxf(xp, 0.f);
    float x2 = x * x;
    s.s0 += x2;
    s.s1 = fmaf(x2, x, s.s1);
    s.s2 = fmaf(x2, x2, s.s2);
  } else {
    if (xp > 0.f) {
      float l = __builtin_amdgcn_logf(xp);
      s.s1 += __builtin_amdgcn_exp2f(r * l);
      s.s0 += __builtin_amdgcn_exp2f((r - 1.f) * l);
    }
  }
}

// accumulate() over the 16 scores a lane holds of one 32 x 32 block: xp_e = a acc_e - tau; with `masked`
// (wave-uniform) entries equal to -inf stand for keys the row does not see.
// AM 1 and 2 spend fewer instructions per score than 16 accumulate() calls: the sign bits are shifted into one
// word and counted once, and the smallest positive xp is an unsigned-integer minimum over the bit patterns
// (positive floats order like unsigned integers, and every negative one lies above them).  A score with
// xp = +0 counts as positive here; it then also makes xmin zero, which only ever withholds the `exact`
// verdict of solve_step().
template <int AM>
__device__ __forceinline__ void accumulate_block(RowSums& s, const f32x16_t& acc, float a, float tau, float r, bool masked) {
  if constexpr (AM == 1 || AM == 2) {
    uint32_t signs = 0u, xm = __float_as_uint(s.xmin);
    auto one = [&](float xp) {
      signs = __builtin_amdgcn_alignbit(signs, __float_as_uint(xp), 31);  // signs << 1 | sign of xp
      xm = min(xm, __float_as_uint(xp));
      float x = fmaxf(xp, 0.f);
      s.s1 += x;
      if (AM == 1) s.s2 = fmaf(x, x, s.s2);
    };
    if (masked) {
#pragma unroll
      for (int e = 0; e < 16; ++e) one(acc[e] == -kInf ? -1.f : fmaf(acc[e], a, -tau));
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) one(fmaf(acc[e], a, -tau));
    }
    s.s0 += (float)(16 - __popc(signs));
    s.xmin = __uint_as_float(xm);
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float xp = (masked && acc[e] == -kInf) ? -1.f : fmaf(acc[e], a, -tau);
      accumulate<AM>(s, xp, r);
    }
  }
}

// One safeguarded root-finding step for a row.  [lo,hi] brackets the root
// (f(lo) >= 0 >= f(hi)).  Returns true when the row is finished.
//   AM 1 / AM 2: f is piecewise quadratic / linear, so the root of the local
//     model is exact as soon as the support stops changing, which is the case
//     when the step stays below the smallest positive term (xmin).
//   AM 3: Halley step from f, f', f''.   AM 0: Newton step (f is convex and
//     decreasing for alpha <= 2, so Newton from the left is monotone).
template <int AM>
__device__ __forceinline__ bool solve_step(const RowSums& s, float r, float& tau, float& lo, float& hi) {
  float f, t;
  bool exact = false;
  if (AM == 1) {
    f = s.s2 - 1.f;
    float disc = fmaf(s.s1, s.s1, -s.s0 * f);
    t = f / (s.s1 + sqrtf(fmaxf(disc, 0.f)));  // = (s1 - sqrt(disc)) / s0 without cancellation
    exact = (f >= 0.f) && (t <= s.xmin);
  } else if (AM == 2) {
    f = s.s1 - 1.f;
    t = f / s.s0;
    exact = (f >= 0.f) && (t <= s.xmin);
  } else if (AM == 3) {
    f = s.s2 - 1.f;
    // f' = -4 s1, f'' = 12 s0;  Halley: t = -2 f f' / (2 f'^2 - f f'') = 2 f s1 / (8 s1^2 - 3 f s0)
    float den = 8.f * s.s1 * s.s1 - 3.f * f * s.s0;
    t = (den != 0.f) ? 2.f * f * s.s1 / den : -kInf;  // no positive term at all: leave the bracket (bisect)
  } else {
    f = s.s1 - 1.f;
    t = f / (r * s.s0);
  }
  if (f >= 0.f)
    lo = fmaxf(lo, tau);
  else
    hi = fminf(hi, tau);
  float tn = tau + t;
  if (exact) {
    tau = fminf(tn, hi);
    return true;
  }
  float tol = 2e-6f * fmaxf(1.f, fabsf(tau));
  bool in = (tn >= lo) && (tn <= hi);
  if (!in) tn = 0.5f * (lo + hi);
  bool fin = (fabsf(tn - tau) <= tol) || (hi - lo <= tol);
  tau = tn;
  return fin;
}

// Where the tiled forward starts its threshold search.  The closed-form / Halley steps converge in two or three
// sweeps from a nearby point but need five or six from the bracket's left end when a row keeps hundreds of keys
// (every sweep recomputes Q K^T).  The row-max sweep therefore also sums the scores and their squares over the
// key blocks the whole wave sees, and the row's threshold is estimated as if its n scores were normal with that
// mean and deviation: n sigma^r G_r(t) = 1 for t = (tau - mu) / sigma, with
//   G_r(t) = E[(z - t)_+^r], z ~ N(0,1):  G_1 = phi - t Q,  G_2 = (1 + t^2) Q - t phi,
//   G_4 = (t^4 + 6 t^2 + 3) Q - (t^3 + 5 t) phi        (Q = upper tail, phi = density),
// solved by bisection once per row.  Only a starting point: the search itself stays safeguarded inside the
// bracket of App. A, and a row whose estimate keeps fewer than kGaussMinSupport keys starts at the left end as before
// (there the top few scores decide, not the bulk).  Measured on dense-regime workloads (B 4, H 12, n 4096, delta 0,
// gamma -1/2): alpha 1.5: 5.3 -> 3.0 sweeps per block, 919 -> 650 us; alpha 1.25: 6.3 -> 2.9, 1120 -> 684 us; alpha 2:
// 8.2 -> 7.0.  At alpha 1.25 with supports of 10 to 60 keys the estimate cost a sweep (3.9 -> 4.4 to 5.2 per block,
// also when aimed to the left of the root), hence the larger minimum for the Halley steps.
constexpr float kGaussMinSupport = 8.f;
constexpr float kGaussMinSupportHalley = 100.f;
template <int AM>
__device__ __forceinline__ float gauss_mass(float t) {
  const float Qt = 0.5f * erfcf(t * 0.70710678f);
  const float ph = 0.39894228f * __expf(-0.5f * t * t);
  const float t2 = t * t;
  if (AM == 1) return fmaf(1.f + t2, Qt, -t * ph);
  if (AM == 2) return fmaf(-t, Qt, ph);
  return (t2 * t2 + 6.f * t2 + 3.f) * Qt - (t2 + 5.f) * t * ph;
}
// mu, sigma: of y = (alpha-1) s over the sample; n: keys the row sees.  Returns false when there is no usable estimate.
template <int AM>
__device__ __forceinline__ bool gauss_start(float mu, float sigma, float n, float& tau0) {
  if (AM == 0) return false;
  if (!(sigma > 0.f) || !(n >= 2.f * kGaussMinSupport)) return false;
  const float s2 = sigma * sigma;
  const float c = 1.0f / (n * (AM == 1 ? s2 : (AM == 2 ? sigma : s2 * s2)));  // G_r(t) = c
  float tl = -6.f, th = 4.f;  // beyond t = 4 the two terms of G_r cancel in single precision
  if (!(gauss_mass<AM>(tl) > c) || !(gauss_mass<AM>(th) < c)) return false;
  for (int it = 0; it < 18; ++it) {
    const float tm = 0.5f * (tl + th);
    if (gauss_mass<AM>(tm) > c) tl = tm; else th = tm;
  }
  const float t = 0.5f * (tl + th);
  if (n * 0.5f * erfcf(t * 0.70710678f) < (AM == 3 ? kGaussMinSupportHalley : kGaussMinSupport)) return false;
  tau0 = fmaf(sigma, t, mu);
  return true;
}

// Keys per LDS tile and waves per SIMD of the tiled forward kernel, as measured on a dense-regime workload
// (B 4, H 12, n 4096, every block on this kernel): at D = 64, 64-key tiles leave room for three workgroups per CU
// (168 registers, no spills) and run the threshold sweeps -- vector-ALU bound, so a third wave per SIMD fills the
// gaps -- a fifth faster than 128-key tiles with two (0.88 against 1.10 ms); at D = 128 three would spill badly
// (1.83 against 1.11 ms at n 16384), but 64-key tiles (64 KB of LDS) with two workgroups per CU (256 registers, a
// dozen spilled) beat 128-key tiles with one: B 2, H 16, n 8192, every block here: 3.87 -> 2.61 ms; 162 split
// blocks (alpha 1.25): 0.89 -> 0.70 ms.
template <typename T, int D>
struct FwdTile {
  static constexpr int value = sizeof(T) == 2 ? 64 : 32;
  static constexpr int kOcc = sizeof(T) == 2 ? (D == 64 ? 3 : 2) : 1;
};

// Keys per LDS tile and workgroups per CU of the list sweeps (fwd_sparse.hip.h, bwd_sparse.hip.h), as measured:
// at D = 64 four 32-key blocks per tile and three workgroups per CU; at D = 128 the query fragments take twice
// the registers, and two blocks per tile with four workgroups per CU run a quarter faster (no spills).
template <typename T, int D>
struct ListCfg {
  static constexpr int kTile = sizeof(T) == 2 ? (D == 64 ? 128 : 64) : 32;
  static constexpr int kOcc = (sizeof(T) == 2 && D == 128) ? 4 : 3;
  // key tiles in flight (sweep_tiles).  Measured at B 4, H 12, n 4096, D 64: two in flight cost registers
  // (spills at three workgroups per CU: 145 us against 139; no spills at two per CU: 188 us)
  static constexpr int kDepth = 1;
  // cells per thread that the collecting sweep keeps in LDS (20 bytes each)
  static constexpr int kLdsCells = kOcc == 4 ? 1 : 4;
  // Per wave, one bit per 32-key block of the head: set by the forward's first sweep where a key of the block can
  // still be a candidate (fwd_sparse.hip.h), so that the second sweep skips the others; blocks beyond the words'
  // range are always visited.  LDS is handed out in pieces of 1280 bytes (measured: 53760 bytes per workgroup run
  // three to a CU, 54080 only two, which costs the sweeps 40 %), so at D = 64 the words take what is left of the
  // 42nd piece: 30 per wave, 30720 keys.  At D = 128 (four workgroups of 32 pieces) there is room for 128.
  static constexpr int kFlagWords = (sizeof(T) == 2 && D == 64) ? 30 : 128;
  // sequences shorter than this do not keep the bits: nearly every block of a wave has some lane that passes
  // (measured at n = 4096: 97 %), so there is nothing to skip
  static constexpr int kFlagMinKeys = 16384;
  // dynamic LDS of a list-sweep kernel: two tile buffers, the overflow flags, the cells, the block bits
  static constexpr size_t kLdsBytes = 2 * (size_t)kTile * D * sizeof(T) + 16 + (size_t)kLdsCells * kThreads * 20 +
                                      (size_t)kWaves * kFlagWords * 4;
};

// SPLIT: the workgroup takes one 32-row group (rg_) of the block instead of four, and its four waves share out
// the 32-key blocks of every tile (block number mod 4 = wave); row maxima, the partial sums of the threshold
// function and the partial outputs are combined across the waves through LDS.  A block then runs as four
// workgroups with a quarter of the serial work each: for the case where only a few blocks need this kernel.
template <typename T, int D, int AM, bool BIAS, bool SPLIT>
__device__ __forceinline__ void fwd_block(const FwdArgs& A, int bh_, int blk_, int rg_, char* smem) {
  using C = QCtx<T, D, FwdTile<T, D>::value, BIAS>;
  constexpr int KT = C::KT, NSB = C::NSB, NM = C::NM, TB = C::kTileBytes;
  // key tiles in flight (sweep_tiles): a split block has its compute unit nearly to itself
  constexpr int kFwdDepth = SPLIT ? 2 : 1;
  const Geom& g = A.g;
  char* tiles = smem;  // 2 buffers x 2 slots
  WaveMask wm;
  wm.words = reinterpret_cast<uint32_t*>(smem + 4 * TB);
  wm.nwords = A.mask_words;
  float* xch = reinterpret_cast<float*>(wm.words + (kWaves + 1) * A.mask_words);  // SPLIT: [kWaves][64][4]

  C q;
  q.init(g, A.Q, bh_, blk_, SPLIT ? rg_ : -1);
  q.init_window(g);
  // SPLIT: 32-key block number (kt NSB + sb) mod 4 = wave is this wave's, which is block sb_own of every NSB-th,
  // or of every, tile; own_bits(kt): the blocks of tile kt that are this wave's (all of them unless SPLIT)
  static_assert(!SPLIT || NSB == 1 || NSB == 2 || NSB == 4, "the split shares out 4 consecutive blocks");
  const int sb_own = __builtin_amdgcn_readfirstlane(q.wave % NSB);
  auto own_bits = [&](int kt) -> uint32_t {
    if constexpr (!SPLIT) return (1u << NSB) - 1u;
    return (((kt * NSB + sb_own) & (kWaves - 1)) == q.wave) ? (1u << sb_own) : 0u;
  };
  // fn(acc, sb) on the score block of every set bit of act.  All of a tile's blocks are computed before the
  // first is used (the matrix pipeline stays busy); a split wave has at most one.
  auto each_block = [&](int kt, const char* tl, uint32_t act, auto&& fn) {
    if constexpr (SPLIT) {
      if (act == 0u) return;
      f32x16_t acc = q.scores(tl, sb_own, kt);
      fn(acc, sb_own);
    } else {
      f32x16_t acc[NSB];
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb)
        if (act & (1u << sb)) acc[sb] = q.scores(tl, sb, kt);
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb)
        if (act & (1u << sb)) fn(acc[sb], sb);
    }
  };
  const float r = 1.0f / (g.alpha - 1.0f);
  float* tau_out = A.tau + (long long)q.bh * g.Nq;
  const long long o_base = (long long)q.b * g.q_sb + (long long)q.h * g.q_sh;

  if (q.block_lim == 0) {  // no row of this workgroup sees any key
    const int row0 = SPLIT ? q.q0 : q.qb * kBlockRows, nrows = SPLIT ? 32 : kBlockRows;
    for (int e = q.tid; e < nrows * D; e += kThreads) {
      int row = row0 + e / D;
      if (row < g.Nq) Elem<T>::store(A.O, o_base + (long long)row * g.q_sn + e % D, 0.f);
    }
    if (q.tid < nrows && row0 + q.tid < g.Nq) tau_out[row0 + q.tid] = 0.f;
    return;
  }
  for (int w = q.tid; w < (kWaves + 1) * A.mask_words; w += kThreads) wm.words[w] = 0u;

  const T* Kbh = reinterpret_cast<const T*>(A.K) + (long long)q.b * g.kv_sb + (long long)q.h * g.kv_sh;
  Slot slots[2];
  slots[0].base = reinterpret_cast<const char*>(Kbh);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);
  slots[1].base = reinterpret_cast<const char*>(A.Vt) + (long long)q.bh * D * g.npad_k * (long long)sizeof(T);
  slots[1].row_bytes = (long long)g.npad_k * (long long)sizeof(T);

  unsigned n_vis = 0, n_qk_solve = 0, n_eval = 0, n_qk_pv = 0, n_pv = 0, n_sweeps = 0;
  // The sweeps over K alone (row maximum, threshold).  SPLIT with two 32-key blocks per tile (64-key tiles): two
  // key tiles between barriers -- with one, half of the waves have no block of their own in it, and every tile
  // costs a barrier and a wait for the staged copy whatever the work (B 4, H 12, n 4096, alpha 1.25, 183 flagged
  // blocks: 351 -> 275 us).  With four blocks per tile (128-key tiles, as D = 128 once had) every wave has one
  // already, and pairs were slower (B 2, H 16, n 8192: 1042 -> 1106 us).
  auto sweep_k = [&](auto needed, auto body) {
    if constexpr (SPLIT && NSB < kWaves) {
      Slot kk[2] = {slots[0], slots[0]};
      sweep_tiles<C, T, D, 2, 0, kFwdDepth, 2>(
          tiles, kk, q.ntiles, g.Nk, q.tid,
          [&](int kp) { return needed(2 * kp) || (2 * kp + 1 < q.ntiles && needed(2 * kp + 1)); },
          [&](int kp, const char* tl) {
            body(2 * kp, tl);
            if (2 * kp + 1 < q.ntiles) body(2 * kp + 1, tl + TB);
          });
    } else {
      sweep_tiles<C, T, D, 1, 0, kFwdDepth>(tiles, slots, q.ntiles, g.Nk, q.tid, needed, body);
    }
  };

  // mask of a 32-key block whose keys are not all visible to all rows of the wave
  auto mask_block = [&](f32x16_t& acc, int j0) {
    int rel = q.lim - j0;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = (q.key_of(e) < rel) ? acc[e] : -kInf;
  };

  // ------------------------------------------------------------ 1. row max
  float m = -kInf;
  // sums of the raw scores and of their squares over the blocks every row of the wave sees in full (gauss_start)
  float ms1 = 0.f, ms2 = 0.f, msn = 0.f;
  // A split block that the list kernel gave up only when its lists overflowed comes with every row's largest
  // score and the list kernel's lower bound of the threshold: no sweep for the maximum, and the search starts
  // from that bound (alpha 1.25; B 4, H 12, n 4096, D 64: 279 -> 246 us; B 2, H 16, n 8192, D 128: 1035 -> 883 us).
  bool have_bounds = false;
  float2 given = make_float2(0.f, 0.f);
  if constexpr (SPLIT) {
    have_bounds = A.bounds != nullptr && __builtin_amdgcn_readfirstlane(A.dense_flag[q.bh * A.nqb + q.qb]) == kFlagWithBounds;
    if (have_bounds && q.valid) given = A.bounds[(long long)q.bh * g.Nq + q.i];
  }
  if (!have_bounds) sweep_k(
      [&](int kt) { return q.tile_in_window(kt); },
      [&](int kt, const char* tl) {
        if (!q.tile_in_wave_window(kt)) return;
        each_block(kt, tl, q.visible_bits(kt) & own_bits(kt), [&](f32x16_t& acc, int sb) {
          int j0 = kt * KT + sb * 32;
          ++n_vis;
          if (j0 + 32 > q.wave_lim_min) {
            mask_block(acc, j0);
          } else if (AM != 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              ms1 += acc[e];
              ms2 = fmaf(acc[e], acc[e], ms2);
            }
            msn += 32.f;
          }
          m = fmaxf(m, max16(acc));
        });
      });
  m = fmaxf(m, __shfl_xor(m, 32));
  ms1 += __shfl_xor(ms1, 32);
  ms2 += __shfl_xor(ms2, 32);
  if (SPLIT && !have_bounds) {  // the row maximum and the sums over all waves' keys
    float* mine = xch + (q.wave * 64 + q.lane) * 4;
    mine[0] = m;
    mine[1] = ms1;
    mine[2] = ms2;
    mine[3] = msn;
    __syncthreads();
    ms1 = ms2 = msn = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float* o = xch + (w * 64 + q.lane) * 4;
      m = fmaxf(m, o[0]);
      ms1 += o[1];
      ms2 += o[2];
      msn += o[3];
    }
    __syncthreads();
  }

  // ------------------------------------------------------------ 2. threshold
  const bool live = q.valid && q.lim > 0;
  float my = live ? (have_bounds ? given.y : q.a * m) : 0.f;
  float lo = my - 1.0f;
  float hi = live ? my - __builtin_amdgcn_exp2f(-(g.alpha - 1.0f) * __builtin_amdgcn_logf((float)q.lim)) : 0.f;
  if (have_bounds && live) lo = fminf(fmaxf(lo, given.x), hi);
  const float lo0 = lo;  // the tiles without a positive term at the left end are zero for good
  float tau = lo;
  if (live && msn >= 64.f) {
    const float mean = ms1 / msn, var = ms2 / msn - mean * mean;
    float t0;
    if (var > 0.f && gauss_start<AM>(q.a * mean, q.a * sqrtf(var), (float)q.lim, t0)) tau = fminf(fmaxf(t0, lo), hi);
  }
  bool done = !live;
  int iter = 0;
  int more;
  do {
    const bool wave_on = __ballot(!done) != 0ull;
    RowSums sums;
    sums.clear();
    const bool first = (iter == 0);
    auto needed = [&](int kt) { return first ? q.tile_in_window(kt) : wm.tile_bits<NSB>(kWaves, kt) != 0u; };
    sweep_k(needed, [&](int kt, const char* tl) {
      if (!wave_on || !q.tile_in_wave_window(kt)) return;
      uint32_t act = q.visible_bits(kt) & own_bits(kt);
      if (!first) act &= wm.tile_bits<NSB>(q.wave, kt);
      each_block(kt, tl, act, [&](f32x16_t& acc, int sb) {
        int j0 = kt * KT + sb * 32;
        ++n_qk_solve;
        const bool masked = j0 + 32 > q.wave_lim_min;
        if (masked) mask_block(acc, j0);
        float lm = max16(acc);
        // masked entries are -inf: a = 0 (scale 0) must not turn them into NaN
        bool cand = (lm > -kInf) && (fmaf(lm, q.a, -tau) > 0.f) && !done;
        if (first) {
          // at the bracket's left end: a tile without a positive term here never gets one later
          bool cand_any = (lm > -kInf) && (fmaf(lm, q.a, -lo0) > 0.f) && live;
          if (__ballot(cand_any) != 0ull && q.lane == 0) wm.set(q.wave, kt * NSB + sb);
        }
        if (__ballot(cand) == 0ull) return;
        ++n_eval;
        accumulate_block<AM>(sums, acc, q.a, tau, r, masked);
      });
    });
    if (first) wm.merge(q.tid);
    sums.combine_halves();
    if constexpr (SPLIT) {  // the sums over all waves' keys, added in wave order: every wave then takes the same step
      float* mine = xch + (q.wave * 64 + q.lane) * 4;
      mine[0] = sums.s0;
      mine[1] = sums.s1;
      mine[2] = sums.s2;
      mine[3] = sums.xmin;
      __syncthreads();
      sums.clear();
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float* o = xch + (w * 64 + q.lane) * 4;
        sums.s0 += o[0];
        sums.s1 += o[1];
        sums.s2 += o[2];
        sums.xmin = fminf(sums.xmin, o[3]);
      }
      __syncthreads();
    }
    if (!done) done = solve_step<AM>(sums, r, tau, lo, hi);
    ++iter;
    ++n_sweeps;
    more = __syncthreads_or(done ? 0 : 1);
  } while (more && iter < kMaxSolveIters);

  // ------------------------------------------------------------ 3. P.V
  f32x16_t oacc[NM];
#pragma unroll
  for (int mm = 0; mm < NM; ++mm)
    oacc[mm] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // lane offsets of the V^T fragments: row (l%32) of a 32-feature block, key chunk 2 sb + cc
  // (a split wave keeps those of its one block)
  constexpr int NVB = SPLIT ? 1 : NSB;
  FragOff<T> voff[2 * NVB];
#pragma unroll
  for (int k = 0; k < 2 * NVB; ++k)
    voff[k] = FragOff<T>::template make<typename C::XtTile>(q.li, 2 * ((SPLIT ? 2 * sb_own : 0) + k) + q.hh);

  sweep_tiles<C, T, D, 2, 2, kFwdDepth>(
      tiles, slots, q.ntiles, g.Nk, q.tid, [&](int kt) { return wm.tile_bits<NSB>(kWaves, kt) != 0u; },
      [&](int kt, const char* tl) {
        const uint32_t act = q.visible_bits(kt) & wm.tile_bits<NSB>(q.wave, kt) & own_bits(kt);
        each_block(kt, tl, act, [&](f32x16_t& acc, int sb) {
          int j0 = kt * KT + sb * 32;
          ++n_qk_pv;
          const bool masked = j0 + 32 > q.wave_lim_min;
          if (masked) mask_block(acc, j0);
          float lm = max16(acc);
          bool cand = live && (lm > -kInf) && (fmaf(lm, q.a, -tau) > 0.f);
          if (__ballot(cand) == 0ull) return;  // every probability of this tile is exactly zero
          ++n_pv;
          float p[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float xp = (masked && acc[e] == -kInf) ? 0.f : fmaf(acc[e], q.a, -tau);
            p[e] = live ? pow_r<AM>(fmaxf(xp, 0.f), r) : 0.f;
          }
          const char* vt = tl + TB;
#pragma unroll
          for (int cc = 0; cc < 2; ++cc) {
            // bf16 probabilities would cost up to 2^-9 |v| of output error; the hi + lo split keeps
            // the product at fp32-level accuracy so that only the output rounding remains
            Frag<T> pf, pl;
            Elem<T>::pack_split(p + 8 * cc, pf, pl);
#pragma unroll
            for (int mm = 0; mm < NM; ++mm) {
              Frag<T> vfr = voff[(SPLIT ? 0 : 2 * sb) + cc].load(vt, mm * 32 * C::XtTile::kRowBytes);
              oacc[mm] = Elem<T>::mma(pf, vfr, oacc[mm]);
              if (Elem<T>::kSplit) oacc[mm] = Elem<T>::mma(pl, vfr, oacc[mm]);
            }
          }
        });
      });

  if constexpr (SPLIT) {
    // the waves' partial outputs, added in wave order by wave 0 (the tile buffers are free: the sweep ended on a
    // barrier)
    float* red = reinterpret_cast<float*>(smem);  // [kWaves][NM * 16][64]
#pragma unroll
    for (int mm = 0; mm < NM; ++mm)
#pragma unroll
      for (int e = 0; e < 16; ++e) red[(q.wave * NM * 16 + mm * 16 + e) * 64 + q.lane] = oacc[mm][e];
    __syncthreads();
    if (q.wave != 0) return;
#pragma unroll
    for (int mm = 0; mm < NM; ++mm)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += red[(w * NM * 16 + mm * 16 + e) * 64 + q.lane];
        oacc[mm][e] = v;
      }
  }
  // oacc[mm][4g + r] of lane l is O[q0 + 8g + 4*(l/32) + r][32 mm + l%32]
#pragma unroll
  for (int mm = 0; mm < NM; ++mm) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int row = q.q0 + q.key_of(e);
      if (row < g.Nq) Elem<T>::store(A.O, o_base + (long long)row * g.q_sn + mm * 32 + q.li, oacc[mm][e]);
    }
  }
  if (q.valid && q.hh == 0) tau_out[q.i] = live ? tau : 0.f;

  if (A.stats && q.lane == 0) {
    const unsigned n_win = q.window_skipped_blocks();
    if (!have_bounds) {  // (else the list kernel has counted this block's tiles)
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_TILES_VISIBLE], (unsigned long long)(n_vis + n_win));
      if (BIAS) atomicAdd(&A.stats[ENTMAX_STAT_FWD_WINDOW_SKIPPED], (unsigned long long)n_win);
    }
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_QK_MAX], (unsigned long long)n_vis);
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_QK_SOLVE], (unsigned long long)n_qk_solve);
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_QK_PV], (unsigned long long)n_qk_pv);
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_PV_TILES], (unsigned long long)n_pv);
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_EVAL_TILES], (unsigned long long)n_eval);
    if (q.wave == 0 && (!SPLIT || rg_ == 0)) {
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_SOLVE_SWEEPS], (unsigned long long)n_sweeps);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_BLOCKS], 1ull);
    }
  }
}

// workgroups that cover either way of sharing the blocks out
inline int fwd_workgroups(int nheads, int nqb, bool flags) {
  const int npairs = nheads * ((nqb + 1) >> 1);
  if (!flags) return npairs;
  // (split: the flagged blocks are dealt out in eights, one to each XCD -- see fwd_kernel)
  const long long nsplit = nheads * (long long)nqb < kSplitMaxBlocks ? nheads * (long long)nqb : kSplitMaxBlocks;
  const long long split = (long long)kWaves * ((nsplit + 7) / 8 * 8);
  return npairs > split ? npairs : (int)split;
}

template <typename T, int D, int AM, bool BIAS>
__global__ __launch_bounds__(kThreads, (FwdTile<T, D>::kOcc)) void fwd_kernel(FwdArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nheads = A.g.B * A.g.H, npairs = nheads * ((A.nqb + 1) >> 1);
  const int nflagged = A.dense_count ? __builtin_amdgcn_readfirstlane(A.dense_count[0]) : kSplitMaxBlocks + 1;
  if (nflagged <= kSplitMaxBlocks) {
    // one workgroup per (flagged block, 32-row group); the blocks' numbers follow the count.  Consecutive
    // workgroups go to the eight XCDs in turn: the four row groups of a block take four consecutive places on
    // one XCD, so that the block's key tiles pass through one L2 instead of four.
    const int xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
    const int slot = (place / kWaves) * 8 + xcd;
    if (slot >= nflagged) return;
    // (the list grows roughly in launch order of the finish kernel, a head's short early blocks first: taken from
    // its end, the long blocks start first)
    const int item = __builtin_amdgcn_readfirstlane(A.dense_count[nflagged - slot]);
    fwd_block<T, D, AM, BIAS, true>(A, item / A.nqb, item % A.nqb, place % kWaves, smem);
    return;
  }
  if ((int)blockIdx.x >= npairs) return;
  const PairItem it = pair_item(A.nqb, blockIdx.x, npairs);
  for (int part = 0; part < 2; ++part) {
    const int blk = part ? it.second : it.first;
    if (blk < 0) break;
    if (A.dense_flag && __builtin_amdgcn_readfirstlane(A.dense_flag[it.bh * A.nqb + blk]) == 0) continue;
    __syncthreads();
    fwd_block<T, D, AM, BIAS, false>(A, it.bh, blk, 0, smem);
  }
}

}  // namespace entmax
