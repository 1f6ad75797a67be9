// Backward kernels.  With x_ij = [(alpha-1) s_ij - tau_i]_+, r = 1/(alpha-1):
//   p = x^r,  g = p^(2-alpha) = x^(r-1)            (derivative of eq. (entmax) on the support)
//   dP_ij = <dO_i, v_j>,  mu_i = sum_j g dP / sum_j g,  dS_ij = g_ij (dP_ij - mu_i)
//   dV_j = sum_i p_ij dO_i,   dQ_i = c_i sum_j dS_ij k_j,   dK_j = sum_i c_i dS_ij q_i,
//   dscale_i = sum_j dS_ij z_ij,   c_i = scale_i / sqrt(D),  z_ij = <q_i,k_j>/sqrt(D)
// and d beta, d gamma by the chain rule through eq. (asentmax).
// Everything is multiplied by p or g, which vanish off the support, so only the
// 32x32 tiles that hold some positive x are visited:
//   bwd_dq_kernel    query-block outer loop: row scalars mu_i, dscale_i and dQ; records the tiles with some
//                    positive x (bit per tile) for the key-side kernel.
//                    dQ is linear in mu:  dQ_i = c_i (sum_j g dP k_j - mu_i sum_j g k_j),
//                    so both sums are accumulated in the same pass and combined
//                    once mu is known -- no second pass and no atomics;
//   bwd_dkv_kernel   key-block outer loop: dK and dV (needs mu from the above);
//   scale_grad_*     reduction of dscale into d beta, d gamma.
#pragma once
#include "qside.hip.h"

namespace entmax {

struct BwdArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* V;
  const void* dO;
  const void* Kt;   // transposed, row-permuted copies (see transpose.hip.h)
  const void* Qt;
  const void* dOt;
  const float* tau;
  void* dQ;
  void* dK;
  void* dV;
  float* mu;        // [B*H*Nq] row term, written by bwd_dq_kernel
  float* crow;      // [B*H*Nq] scale_i / sqrt(D)
  float* dscale;    // [B*H*Nq] gradient with respect to scale_i
  uint32_t* mask;   // [B*H][nqg][mask_words] bit jb of row ig: tile (ig, jb) holds some p > 0
  unsigned long long* stats;
  const int* head_flag;  // NULL: every head, whole; else [B*H]: 0 skip the head, 1 only its flagged query blocks,
                         // 2 the whole head
  const int* block_flag; // with head_flag: [B*H*nqb] the query blocks the list path left over
  int nqb, nkb, nqg, mask_words;
  int xcd_room;  // workgroups of the kernel being launched that one XCD holds at a time (see bwd_tiled_item)
  // whether query block qb of head bh is this path's (call only for heads whose flag is not 0)
  __device__ __forceinline__ bool block_is_ours(int bh, int qb) const {
    if (!head_flag) return true;
    return __builtin_amdgcn_readfirstlane(head_flag[bh]) == 2 || __builtin_amdgcn_readfirstlane(block_flag[bh * nqb + qb]) != 0;
  }
};

// ------------------------------------------------- row scalars, dscale and dQ

template <typename T, int D, int AM, bool BIAS>
__device__ __forceinline__ void bwd_dq_block(const BwdArgs& A, int bh_, int blk_, char* smem) {
  using C = QCtx<T, D, Elem<T>::kTile, BIAS>;
  constexpr int KT = C::KT, NSB = C::NSB, NC = C::NC, NM = C::NM, TB = C::kTileBytes;
  const Geom& g = A.g;
  char* tiles = smem;  // 2 buffers x 3 slots: K, V, Kt
  WaveMask wm;
  wm.words = reinterpret_cast<uint32_t*>(smem + 6 * TB);
  wm.nwords = A.mask_words;
  float* xch = reinterpret_cast<float*>(wm.words + (kWaves + 1) * A.mask_words);  // [kWaves][64]

  C q;
  q.init(g, A.Q, bh_, blk_);
  if (A.head_flag && __builtin_amdgcn_readfirstlane(A.head_flag[q.bh]) == 0) return;
  if (!A.block_is_ours(q.bh, q.qb)) {
    // dQ and the row scalars of this block come from the list path: none of its tiles is the key-side kernel's
    const int ig = q.q0 >> 5;
    if (ig < A.nqg) {
      uint32_t* dst = A.mask + ((long long)q.bh * A.nqg + ig) * A.mask_words;
      for (int w = q.lane; w < A.mask_words; w += 64) dst[w] = 0u;
    }
    return;
  }
  q.init_window(g);
  const float r = 1.0f / (g.alpha - 1.0f);
  const long long row_idx = (long long)q.bh * g.Nq + q.i;
  const float tau = q.valid ? A.tau[row_idx] : 0.f;
  const bool live = q.valid && q.lim > 0;
  const long long q_base = (long long)q.b * g.q_sb + (long long)q.h * g.q_sh;

  Frag<T> dof[NC];
  {
    const T* drow = reinterpret_cast<const T*>(A.dO) + q_base + (long long)q.i * g.q_sn;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) dof[cc] = q.valid ? Elem<T>::load(drow + 16 * cc + 8 * q.hh) : Elem<T>::zero();
  }
  // the map of the tiles that hold some p > 0 is a by-product of this pass (the key-side kernel reads it)
  for (int w = q.tid; w < kWaves * A.mask_words; w += kThreads) wm.words[w] = 0u;
  __syncthreads();

  const long long kv_base = (long long)q.b * g.kv_sb + (long long)q.h * g.kv_sh;
  Slot slots[3];
  slots[0].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.K) + kv_base);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);
  slots[1].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.V) + kv_base);
  slots[1].row_bytes = g.kv_sn * (long long)sizeof(T);
  slots[2].base = reinterpret_cast<const char*>(A.Kt) + (long long)q.bh * D * g.npad_k * (long long)sizeof(T);
  slots[2].row_bytes = (long long)g.npad_k * (long long)sizeof(T);

  f32x16_t acc1[NM], acc2[NM];
#pragma unroll
  for (int mm = 0; mm < NM; ++mm) {
    acc1[mm] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    acc2[mm] = acc1[mm];
  }
  float Z = 0.f, N = 0.f, Aq = 0.f, Cq = 0.f;
  unsigned n_tiles = 0, n_vis = 0;

  auto needed = [&](int kt) { return q.tile_in_window(kt); };
  const bool plain = __ballot(!live) == 0ull;  // every row of the wave exists and sees a key
  sweep_tiles<C, T, D, 3, 4>(tiles, slots, q.ntiles, g.Nk, q.tid, needed, [&](int kt, const char* tl) {
    if (!q.tile_in_wave_window(kt)) return;
    const uint32_t act = q.visible_bits(kt);
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      if (!(act & (1u << sb))) continue;
      int j0 = kt * KT + sb * 32;
      ++n_vis;
      f32x16_t acc = q.scores(tl, sb, kt);
      const bool masked = j0 + 32 > q.wave_lim_min;
      const int rel = q.lim - j0;
      float x[16];
      bool any;
      if (plain && !masked) {
        // every row of the wave sees every key of the block: no select per score
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = fmaxf(fmaf(acc[e], q.a, -tau), 0.f);
        float xm = fmaxf(x[0], x[1]);
#pragma unroll
        for (int e = 2; e < 16; e += 2) xm = fmaxf(fmaxf(xm, x[e]), x[e + 1]);
        any = xm > 0.f;
      } else {
        any = false;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          bool vis = live && (!masked || q.key_of(e) < rel);
          float xp = fmaf(acc[e], q.a, -tau);
          x[e] = vis ? fmaxf(xp, 0.f) : 0.f;
          acc[e] = vis ? acc[e] : 0.f;
          any = any || (x[e] > 0.f);
        }
      }
      if (__ballot(any) == 0ull) continue;
      ++n_tiles;
      if (q.lane == 0) wm.set(q.wave, kt * NSB + sb);
      // dP^T = V_tile dO^T, same lane layout as the scores
      f32x16_t dp = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cc = 0; cc < NC; ++cc)
        dp = Elem<T>::mma(C::KTile::frag(tl + TB, sb * 32 + q.li, 2 * cc + q.hh), dof[cc], dp);
      if constexpr (BIAS) {
        // bias outside the scale: dscale_i = sum_j dS_ij z_ij needs the scores without their bias term
        if (g.bias_mode == 1 && q.wave_bias) {
          f32x16_t bb;
          q.bias_block(bb, j0);
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[e] -= bb[e];
        }
      }
      float w1[16], w2[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float gg = pow_rm1<AM>(x[e], r);
        // (g = 0 where x = 0, except for alpha = 2 whose g is the support indicator)
        float gd = (AM == 2) ? ((x[e] > 0.f) ? dp[e] : 0.f) : gg * dp[e];
        Z += gg;
        N += gd;
        Aq = fmaf(gd, acc[e], Aq);
        Cq = fmaf(gg, acc[e], Cq);
        w1[e] = gd;
        w2[e] = gg;
      }
      const char* ktt = tl + 2 * TB;
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        Frag<T> f1 = Elem<T>::pack(w1 + 8 * cc);
        Frag<T> f2 = Elem<T>::pack(w2 + 8 * cc);
#pragma unroll
        for (int mm = 0; mm < NM; ++mm) {
          Frag<T> kf = C::XtTile::frag(ktt, mm * 32 + q.li, 2 * (2 * sb + cc) + q.hh);
          acc1[mm] = Elem<T>::mma(f1, kf, acc1[mm]);
          acc2[mm] = Elem<T>::mma(f2, kf, acc2[mm]);
        }
      }
    }
  });

  Z += __shfl_xor(Z, 32);
  N += __shfl_xor(N, 32);
  Aq += __shfl_xor(Aq, 32);
  Cq += __shfl_xor(Cq, 32);
  const float mu = (Z > 0.f) ? N / Z : 0.f;
  if (q.valid && q.hh == 0) {
    // the scores were formed with q negated when scale_i < 0: undo the sign for z_ij
    float sgn = (q.c < 0.f) ? -1.f : 1.f;
    A.mu[row_idx] = mu;
    A.crow[row_idx] = q.c;
    A.dscale[row_idx] = sgn * (Aq - mu * Cq) * (1.0f / sqrtf((float)D));
  }
  if (q.hh == 0) {
    xch[q.wave * 64 + q.li] = mu;
    xch[q.wave * 64 + 32 + q.li] = q.c;
  }
  __syncthreads();
  // acc[mm][4g + r] of lane l belongs to query row q0 + 8g + 4*(l/32) + r, feature 32 mm + l%32
#pragma unroll
  for (int mm = 0; mm < NM; ++mm) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int rl = q.key_of(e);
      int row = q.q0 + rl;
      float mur = xch[q.wave * 64 + rl], cr = xch[q.wave * 64 + 32 + rl];
      if (row < g.Nq)
        Elem<T>::store(A.dQ, q_base + (long long)row * g.q_sn + mm * 32 + q.li, cr * (acc1[mm][e] - mur * acc2[mm][e]));
    }
  }
  // (the sweep ended on a barrier: all bits are in LDS)
  {
    const int ig = q.q0 >> 5;
    if (ig < A.nqg) {
      uint32_t* dst = A.mask + ((long long)q.bh * A.nqg + ig) * A.mask_words;
      for (int w = q.lane; w < A.mask_words; w += 64) dst[w] = wm.words[q.wave * A.mask_words + w];
    }
  }
  if (A.stats && q.lane == 0) {
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_DQ_TILES], (unsigned long long)n_tiles);
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_TILES_VISIBLE], (unsigned long long)n_vis);
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_QK_MASK], (unsigned long long)n_vis);
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_ACTIVE_TILES], (unsigned long long)n_tiles);
  }
}

// ------------------------------------------------------------------ dK, dV

template <typename T, int D, int AM>
__device__ __forceinline__ void bwd_dkv_block(const BwdArgs& A, int bh_, int blk_, char* smem) {
  using C = QCtx<T, D>;
  constexpr int QT = C::KT, NSG = C::NSB, NC = C::NC, NM = C::NM, TB = C::kTileBytes;
  const Geom& g = A.g;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, li = lane & 31,
            hh = lane >> 5;
  const int bh = __builtin_amdgcn_readfirstlane(bh_), kb = __builtin_amdgcn_readfirstlane(blk_);
  const int b = __builtin_amdgcn_readfirstlane(bh / g.H), h = __builtin_amdgcn_readfirstlane(bh % g.H);
  if (A.head_flag && __builtin_amdgcn_readfirstlane(A.head_flag[bh]) == 0) return;
  const float r = 1.0f / (g.alpha - 1.0f);
  const float am1 = g.alpha - 1.0f;
  const int off = g.Nk - g.Nq;

  // smem: [2 buffers x 4 tiles: Q, dO, Qt, dOt][2 buffers x 3 row arrays x QT floats][need: nqg bytes]
  char* tiles = smem;
  float* rows = reinterpret_cast<float*>(smem + 8 * TB);
  unsigned char* need = reinterpret_cast<unsigned char*>(rows + 2 * 4 * QT);

  const int jw0 = kb * kBlockRows + wave * 32;  // first key of this wave
  const int j = jw0 + li;                       // this lane's key (as the B-operand column)
  const bool jvalid = j < g.Nk;
  const long long kv_base = (long long)b * g.kv_sb + (long long)h * g.kv_sh;
  const long long q_base = (long long)b * g.q_sb + (long long)h * g.q_sh;
  Frag<T> kf[NC], vf[NC];
  {
    const T* krow = reinterpret_cast<const T*>(A.K) + kv_base + (long long)j * g.kv_sn;
    const T* vrow = reinterpret_cast<const T*>(A.V) + kv_base + (long long)j * g.kv_sn;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) {
      kf[cc] = jvalid ? Elem<T>::load(krow + 16 * cc + 8 * hh) : Elem<T>::zero();
      vf[cc] = jvalid ? Elem<T>::load(vrow + 16 * cc + 8 * hh) : Elem<T>::zero();
    }
  }
  {
    int jb0 = kb * 4;  // the four 32-key blocks of this workgroup share one mask word
    for (int ig = tid; ig < A.nqg; ig += kThreads) {
      uint32_t w = A.mask[((long long)bh * A.nqg + ig) * A.mask_words + (jb0 >> 5)];
      need[ig] = (unsigned char)((w >> (jb0 & 31)) & 0xFu);
    }
  }
  __syncthreads();

  // query tiles that can see this key block: row i sees key j iff j <= i + off
  const int nqt = (g.Nq + QT - 1) / QT;
  int qt_first = 0;
  if (g.causal) {
    int imin = kb * kBlockRows - off;
    qt_first = imin > 0 ? imin / QT : 0;
  }

  f32x16_t dk[NM], dv[NM];
#pragma unroll
  for (int mm = 0; mm < NM; ++mm) {
    dk[mm] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    dv[mm] = dk[mm];
  }
  unsigned n_tiles = 0;

  using NTile = typename C::KTile;   // natural: rows = queries
  using TTile = typename C::XtTile;  // transposed: rows = features
  Stage<NTile> sq, sdo;
  Stage<TTile> sqt, sdot;
  float rv[4] = {0.f, 0.f, 0.f, 0.f};  // staged row values (threads < QT): tau, (alpha-1) c, mu, bias per unit distance
  const bool biased = g.slopes != nullptr && g.slopes[h] != 0.f;  // uniform

  const char* Qg = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.Q) + q_base);
  const char* dOg = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.dO) + q_base);
  const char* Qtg = reinterpret_cast<const char*>(A.Qt) + (long long)bh * D * g.npad_q * (long long)sizeof(T);
  const char* dOtg = reinterpret_cast<const char*>(A.dOt) + (long long)bh * D * g.npad_q * (long long)sizeof(T);
  const long long qrow_bytes = g.q_sn * (long long)sizeof(T);
  const long long trow_bytes = (long long)g.npad_q * (long long)sizeof(T);
  sq.init(qrow_bytes, tid);
  sdo.init(qrow_bytes, tid);
  sqt.init(trow_bytes, tid);
  sdot.init(trow_bytes, tid);

  auto tile_needed = [&](int qt) {
    bool n = false;
    for (int sg = 0; sg < NSG; ++sg) {
      int ig = qt * NSG + sg;
      if (ig < A.nqg) n = n || (need[ig] != 0);
    }
    return n;
  };
  auto next_needed = [&](int qt) {
    while (qt < nqt && !tile_needed(qt)) ++qt;
    return qt;
  };
  auto fetch = [&](int qt) {
    int rows_left = g.Nq - qt * QT;
    if (rows_left >= QT) {
      sq.fetch_full(Qg + (long long)qt * QT * qrow_bytes);
      sdo.fetch_full(dOg + (long long)qt * QT * qrow_bytes);
    } else {
      sq.fetch(Qg + (long long)qt * QT * qrow_bytes, rows_left, qrow_bytes);
      sdo.fetch(dOg + (long long)qt * QT * qrow_bytes, rows_left, qrow_bytes);
    }
    sqt.fetch_full(Qtg + (long long)qt * QT * (long long)sizeof(T));
    sdot.fetch_full(dOtg + (long long)qt * QT * (long long)sizeof(T));
    if (tid < QT) {
      int i = qt * QT + tid;
      if (i < g.Nq) {
        long long ri = (long long)bh * g.Nq + i;
        rv[0] = A.tau[ri];
        rv[1] = am1 * A.crow[ri];
        rv[2] = A.mu[ri];
        // (alpha-1) s_ij = rv[1] <q_i,k_j> + rv[3] dist_ij: the same product a w as on the query side
        if (biased) rv[3] = fabsf(rv[1]) * bias_w<D>(g, h, A.crow[ri], fabsf(rv[1]));
      } else {  // rows beyond Nq: x = -1 everywhere
        rv[0] = 1.f;
        rv[1] = 0.f;
        rv[2] = 0.f;
        rv[3] = 0.f;
      }
    }
  };
  auto commit = [&](int bufi) {
    char* bf = tiles + bufi * 4 * TB;
    sq.commit(bf);
    sdo.commit(bf + TB);
    sqt.commit(bf + 2 * TB);
    sdot.commit(bf + 3 * TB);
    if (tid < QT) {
      float* rw = rows + bufi * 4 * QT;
      rw[tid] = rv[0];
      rw[QT + tid] = rv[1];
      rw[2 * QT + tid] = rv[2];
      rw[3 * QT + tid] = rv[3];
    }
  };

  int qt = next_needed(qt_first);
  if (qt < nqt) {
    fetch(qt);
    commit(0);
  }
  __syncthreads();
  int cur = 0;
  while (qt < nqt) {
    int nxt = next_needed(qt + 1);
    if (nxt < nqt) fetch(nxt);
    const char* tl = tiles + cur * 4 * TB;
    const float* rw = rows + cur * 4 * QT;
#pragma unroll
    for (int sg = 0; sg < NSG; ++sg) {
      int ig = qt * NSG + sg;
      if (ig >= A.nqg) continue;
      if (!((__builtin_amdgcn_readfirstlane((int)need[ig]) >> wave) & 1)) continue;
      int i0 = ig * 32;
      // S block: rows = the 32 queries of the group, cols = the wave's 32 keys
      f32x16_t s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) s = Elem<T>::mma(NTile::frag(tl, sg * 32 + li, 2 * cc + hh), kf[cc], s);
      float x[16], mur[16], car[16];
      bool any;
      // every key of the wave exists and lies at or before the group's first query: no select per score
      const bool full = (jw0 + 32 <= g.Nk) && (!g.causal || jw0 + 31 <= i0 + off);
      if (full && !biased) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          int rl = sg * 32 + 8 * gq + 4 * hh;
          f32x4_t t4 = *reinterpret_cast<const f32x4_t*>(rw + rl);
          f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(rw + QT + rl);
          f32x4_t m4 = *reinterpret_cast<const f32x4_t*>(rw + 2 * QT + rl);
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            int e = 4 * gq + rr;
            x[e] = fmaxf(fmaf(s[e], a4[rr], -t4[rr]), 0.f);
            mur[e] = m4[rr];
            car[e] = a4[rr];
          }
        }
        float xm = fmaxf(x[0], x[1]);
#pragma unroll
        for (int e = 2; e < 16; e += 2) xm = fmaxf(fmaxf(xm, x[e]), x[e + 1]);
        any = xm > 0.f;
      } else {
        any = false;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          int rl = sg * 32 + 8 * gq + 4 * hh;
          f32x4_t t4 = *reinterpret_cast<const f32x4_t*>(rw + rl);
          f32x4_t a4 = *reinterpret_cast<const f32x4_t*>(rw + QT + rl);
          f32x4_t m4 = *reinterpret_cast<const f32x4_t*>(rw + 2 * QT + rl);
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            int e = 4 * gq + rr;
            int i = i0 + 8 * gq + 4 * hh + rr;
            bool vis = jvalid && (!g.causal || (j <= i + off));
            float xp = fmaf(s[e], a4[rr], -t4[rr]);
            if (biased) xp = fmaf(rw[3 * QT + rl + rr], (float)bias_dist(i + off, j), xp);
            x[e] = vis ? fmaxf(xp, 0.f) : 0.f;
            mur[e] = m4[rr];
            car[e] = a4[rr];
            any = any || (x[e] > 0.f);
          }
        }
      }
      if (__ballot(any) == 0ull) continue;
      ++n_tiles;
      f32x16_t dp = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) dp = Elem<T>::mma(NTile::frag(tl + TB, sg * 32 + li, 2 * cc + hh), vf[cc], dp);
      // ds = (alpha-1) dS: car holds (alpha-1) c_i; the factor goes into dK once, at the end.  g = 0 where x = 0,
      // except for alpha = 2 whose g is the support indicator.
      float pp[16], ds[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        pp[e] = pow_r<AM>(x[e], r);
        float gg = pow_rm1<AM>(x[e], r);
        ds[e] = gg * (dp[e] - mur[e]) * car[e];
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        Frag<T> pf = Elem<T>::pack(pp + 8 * cc);
        Frag<T> df = Elem<T>::pack(ds + 8 * cc);
#pragma unroll
        for (int mm = 0; mm < NM; ++mm) {
          int fidx = 2 * (2 * sg + cc) + hh;
          dv[mm] = Elem<T>::mma(pf, TTile::frag(tl + 3 * TB, mm * 32 + li, fidx), dv[mm]);
          dk[mm] = Elem<T>::mma(df, TTile::frag(tl + 2 * TB, mm * 32 + li, fidx), dk[mm]);
        }
      }
    }
    if (nxt < nqt) commit(cur ^ 1);
    __syncthreads();
    cur ^= 1;
    qt = nxt;
  }

  // dk/dv[mm][4g + r] of lane l belongs to key jw0 + 8g + 4*(l/32) + r, feature 32 mm + l%32
  const float inv_am1 = 1.0f / am1;
#pragma unroll
  for (int mm = 0; mm < NM; ++mm) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int row = jw0 + 8 * (e >> 2) + 4 * hh + (e & 3);
      if (row < g.Nk) {
        long long idx = kv_base + (long long)row * g.kv_sn + mm * 32 + li;
        Elem<T>::store(A.dK, idx, dk[mm][e] * inv_am1);
        Elem<T>::store(A.dV, idx, dv[mm][e]);
      }
    }
  }
  if (A.stats && lane == 0) atomicAdd(&A.stats[ENTMAX_STAT_BWD_DKV_TILES], (unsigned long long)n_tiles);
}

// Which (head, block) item a workgroup of the tiled backward kernels takes.  When most heads are here, a head's
// blocks share an XCD (xcd_remap: one L2 for the head's K and V).  When only a few heads are -- the others went
// down the list path -- that order would queue a whole head's long-running workgroups on one XCD's 32 CUs while
// seven XCDs idle (B 2, H 16, n 8192, D 128, two heads of 32 flagged: 64 workgroups at one per CU ran as two rounds,
// 0.79 ms for work that takes 0.40), so where a head has more blocks than an XCD holds at a time the items are then
// dealt out to the XCDs in turn (0.79 -> 0.59 ms, dK/dV 0.83 -> 0.70 ms).  Every workgroup makes the same choice
// from the heads' flags (up to 1024 heads are counted; more keep the head-per-XCD order).
__device__ __forceinline__ int bwd_tiled_item(const BwdArgs& A, int per_head) {
  const int nheads = A.g.B * A.g.H;
  if (A.head_flag == nullptr || nheads > 4 * kThreads || per_head <= A.xcd_room) return xcd_remap(blockIdx.x, gridDim.x);
  int flagged = 0;
  for (int k0 = 0; k0 < nheads; k0 += kThreads) {
    const int k = k0 + (int)threadIdx.x;
    flagged += __syncthreads_count(k < nheads && A.head_flag[k] != 0);
  }
  return 4 * flagged <= nheads ? (int)blockIdx.x : xcd_remap(blockIdx.x, gridDim.x);
}

// The register-heavy kernels hold two workgroups per CU; one block per workgroup, long blocks first.
template <typename T, int D, int AM, bool BIAS>
__global__ __launch_bounds__(kThreads) void bwd_dq_kernel(BwdArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int item = bwd_tiled_item(A, A.nqb);
  if (A.head_flag && __builtin_amdgcn_readfirstlane(A.head_flag[item / A.nqb]) == 0) return;
  bwd_dq_block<T, D, AM, BIAS>(A, item / A.nqb, A.nqb - 1 - item % A.nqb, smem);
}
template <typename T, int D, int AM>
__global__ __launch_bounds__(kThreads) void bwd_dkv_kernel(BwdArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int item = bwd_tiled_item(A, A.nkb);
  if (A.head_flag && __builtin_amdgcn_readfirstlane(A.head_flag[item / A.nkb]) == 0) return;
  bwd_dkv_block<T, D, AM>(A, item / A.nkb, item % A.nkb, smem);
}

// ------------------------------------------------------- d beta, d gamma

constexpr int kScaleGradThreads = 1024;

// Per-head parameters: dbeta_h = sum_{b,i} dscale L^gamma, dgamma_h = sum dscale beta L^gamma ln L,
// L = ln n (eq. (asentmax)); one workgroup per head, fixed summation order.
// NT threads of one workgroup; sb_, sg_: NT floats of LDS each.
template <int NT>
__device__ __forceinline__ void scale_grad_head_part(const Geom& g, const float* dscale, float* dbeta, float* dgamma, int h,
                                                     float* sb_, float* sg_) {
  const int tid = threadIdx.x;
  float ab = 0.f, ag = 0.f;
  if (g.logn_mode == 0) {
    // n = Nk for every row: (ln n)^gamma is one number per head, only dscale has to be summed
    float Lg, lnL, bt;
    row_scale(g, 0, h, 0, g.Nk, &Lg, &lnL, &bt);
    float s = 0.f;
    for (int b = 0; b < g.B; ++b) {
      const float* ds = dscale + ((long long)b * g.H + h) * g.Nq;
      for (int i = tid; i < g.Nq; i += NT) s += ds[i];
    }
    ab = s * Lg;
    ag = s * bt * Lg * lnL;
  } else {
    for (int b = 0; b < g.B; ++b) {
      for (int i = tid; i < g.Nq; i += NT) {
        float Lg, lnL, bt;
        row_scale(g, b, h, i, row_limit(g, i), &Lg, &lnL, &bt);
        float ds = dscale[((long long)b * g.H + h) * g.Nq + i];
        ab += ds * Lg;
        ag += ds * bt * Lg * lnL;
      }
    }
  }
  sb_[tid] = ab;
  sg_[tid] = ag;
  __syncthreads();
  for (int s = NT / 2; s > 0; s >>= 1) {
    if (tid < s) {
      sb_[tid] += sb_[tid + s];
      sg_[tid] += sg_[tid + s];
    }
    __syncthreads();
  }
  if (tid == 0) {
    dbeta[h] = sb_[0];
    dgamma[h] = sg_[0];
  }
}

static __global__ __launch_bounds__(kScaleGradThreads) void scale_grad_head_kernel(Geom g, const float* dscale, float* dbeta,
                                                                   float* dgamma) {
  __shared__ float sb_[kScaleGradThreads], sg_[kScaleGradThreads];
  scale_grad_head_part<kScaleGradThreads>(g, dscale, dbeta, dgamma, blockIdx.x, sb_, sg_);
}

// Per-query parameters: one value per row.
static __global__ void scale_grad_query_kernel(Geom g, const float* dscale, float* dbeta, float* dgamma) {
  long long row = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long rows = (long long)g.B * g.H * g.Nq;
  if (row >= rows) return;
  int i = (int)(row % g.Nq);
  int h = (int)((row / g.Nq) % g.H);
  int b = (int)(row / ((long long)g.Nq * g.H));
  float Lg, lnL, bt;
  row_scale(g, b, h, i, row_limit(g, i), &Lg, &lnL, &bt);
  float ds = dscale[row];
  dbeta[row] = ds * Lg;
  dgamma[row] = ds * bt * Lg * lnL;
}

}  // namespace entmax
