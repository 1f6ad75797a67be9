// Forward path for rows whose support is small (the regime the paper's
// ASEntmax workloads live in: a handful of non-zero probabilities per row).
//
// alpha-entmax gives exact zeros below the threshold (Sec. 2.2, App. A), and the
// threshold is bounded below by any sub-problem: solving eq. (entmax) on a
// subset S of the row's scores gives tau_S <= tau, because dropping terms can
// only lower f(tau) = sum_j [(alpha-1) s_j - tau]_+^r - 1.  So
//   fwd_lists_kernel (matrix cores, K tiles through LDS, two sweeps)
//     1. row-max sweep that also keeps the second largest per-cell maximum:
//        tau_lb = max(left end of the bracket of App. A eq. (bounds),
//                     solution of the two-element sub-problem) <= tau;
//     2. second Q K^T sweep: every key with (alpha-1) s_ij > tau_lb goes on the
//        row's candidate list (key index + raw score).  Every key of the
//        support is on that list; nothing else of the row can matter.
//   fwd_finish_kernel (no matrix work, one lane pair per row)
//     3. the threshold by the same safeguarded steps as the tiled kernel
//        (closed-form local-model root for alpha 1.5 / 2, Halley / Newton
//        otherwise), summing over the list instead of over key tiles;
//     4. O_i = sum over the list of p_ij v_j, gathering the few value rows; for the
//        backward, the entries with p_ij > 0 are written out as the row's support list.
// A workgroup that meets a row with more candidates than a list holds raises
// its flag and leaves the whole block to the tiled kernel (fwd.hip.h), which
// handles any density.
// Also here: what the other list kernels share (bwd_sparse.hip.h, decode.hip.h): the
// slot-major list layout, the collect sweep, row gather helpers.
#pragma once
#include "fwd.hip.h"
#include "transpose.hip.h"

namespace entmax {

// Row lists (candidates, supports, per-entry records) are stored per wave of 32 rows x 2 halves with
// entry s of all 64 lanes together: short lists then touch only the first few 512-byte groups of a
// wave's region instead of one cache line per half row.  Wave w = ((bh * nqb + qb) * 4 + wave in block);
// entry (lane, s) sits at list_entry<CAP>(w, lane) + s * kListStride.
template <int CAP>
__device__ __forceinline__ long long list_entry(int bh, int nqb, int qb, int wave, int lane) {
  return (((long long)bh * nqb + qb) * kWaves + wave) * CAP * kListStride + lane;
}


struct FwdSparseArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* tau;
  uint2* cand;      // [B*H*nqb*4 waves][kCandCap][64 lanes] (key index, raw dot product bits), see list_entry()
  uint2* list;      // NULL, or the pool of the `saved` buffer the rows' supports are packed into for the backward:
                    // every 32-row group takes one contiguous piece (lane after lane, entry after entry)
  char* pool_cursor;       // with list: the pool's parts each have a 64-bit cursor (entries handed out so far, zeroed
                           // by the list kernel), kSavedCursorStride bytes apart
  int pool_parts;          // with list: parts the pool is cut into (a power of two)
  long long pool_part_cap; // with list: entries a part holds
  int* slcnt;       // with list: [B*H*Nq][2] per half row: (place of its first entry in the pool) << 5 | entries
  int* bwd_flag;    // with list: [B*H*nqb] not 0: the backward cannot take its list path for this block
                    // (kBlockListsUnused, kBlockNoLists)
  int* kcount;      // with list: [B*H*Nk] support entries naming each key (zeroed by the list kernel, counted by
                    // the finish kernel): the sizes of the backward's key-major segments
  void* cells;      // sweep scratch: one CellBuf<kCandCap> per workgroup of the list sweep's grid
  int* lcnt;        // [B*H*Nq][2] list lengths
  float2* bounds;   // [B*H*Nq] (tau_lb, right end of the bracket)
  int* dense_flag;  // [B*H*nqb] 1: block left to the tiled kernel; behind them: how many are set (zeroed by the
                    // list kernel, counted by the finish kernel), then the first kSplitMaxBlocks flagged blocks' numbers
  unsigned long long* stats;
  int nqb;
  int force_long;      // run the long-sequence kernels whatever the sizes (params.path = 2: test aid)
  int unpaired;        // fwd_lists_kernel: one query block per workgroup (see fwd_lists_unpaired())
  TransposeRide ride;  // V^T copies for the tiled kernel, as extra workgroups of the finish launch
};

// A cell is a group of four consecutive accumulator registers of a lane (keys j, j+1, j+2, j+3 of
// one row).  During a sweep a lane appends whole cells
// -- all their raw scores and the first key index -- to a private strip of scratch memory whenever the
// cell maximum passes the cutoff: one short divergent region per cell instead of one per score.  After
// the sweep each lane walks its own cells and writes the scores above the cutoff to its list.
// The first LS cells of a thread stay in LDS (the common case: a row has a handful of candidates), the others go
// to a strip of global scratch.  Addresses are formed where they are used: the struct holds two registers.
template <int CAP, int LS>
struct CellBuf {
  static_assert(kCellGroups == 1, "a cell is one group of four accumulator registers");
  // cell s of the 256 threads of a workgroup together (s-major), for the same reason as the row lists:
  //   LDS:    scores of cell s at lds + (s * kThreads + tid) * 16, its first key at lds + LS * kThreads * 16 + (s * kThreads + tid) * 4
  //   global: the same with CAP in place of LS, in the workgroup's strip
  char* lds;
  char* strip;  // workgroup-uniform
  int tid;
  static constexpr size_t kBytesPerWorkgroup = cell_bytes_per_workgroup(CAP);
  static constexpr int kLdsBytes = LS * kThreads * 20;
  __device__ __forceinline__ void init(void* base, char* lds_, int tid_, int strip_no = blockIdx.x) {
    strip = reinterpret_cast<char*>(base) + (size_t)strip_no * kBytesPerWorkgroup;
    lds = lds_;
    tid = tid_;
  }
  // n: cells this thread stored before.  A strip that is full keeps overwriting its last cell (the caller
  // then discards the lists).
  __device__ __forceinline__ void store(int n, const f32x4_t& v, int key) {
    if (LS > 0 && n < LS) {
      const int e = n * kThreads + tid;
      *reinterpret_cast<f32x4_t*>(lds + e * 16) = v;
      *reinterpret_cast<int*>(lds + LS * kThreads * 16 + e * 4) = key;
    } else {
      const int e = min(n, CAP - 1) * kThreads + tid;
      *reinterpret_cast<f32x4_t*>(strip + (size_t)e * 16) = v;
      *reinterpret_cast<int*>(strip + (size_t)CAP * kThreads * 16 + (size_t)e * 4) = key;
    }
  }
  __device__ __forceinline__ void load(int n, f32x4_t& v, int& key) const {
    if (LS > 0 && n < LS) {
      const int e = n * kThreads + tid;
      v = *reinterpret_cast<const f32x4_t*>(lds + e * 16);
      key = *reinterpret_cast<const int*>(lds + LS * kThreads * 16 + e * 4);
    } else {
      const int e = n * kThreads + tid;
      v = *reinterpret_cast<const f32x4_t*>(strip + (size_t)e * 16);
      key = *reinterpret_cast<const int*>(strip + (size_t)CAP * kThreads * 16 + (size_t)e * 4);
    }
  }
};

// One sweep over the visible key tiles of the block: every key whose shifted score
// a * dot - thr is positive ends up in the lane's list.  Returns false (workgroup-uniform) if
// some list overflowed; the sweep is abandoned early in that case.  ovf: three ints of LDS;
// lds_cells: CellBuf<CAP, LS>::kLdsBytes bytes of LDS.  blockbits: NULL, or this wave's ListCfg::kFlagWords words
// of LDS with one bit per 32-key block of the head: a block whose bit is clear holds no candidate of any row of
// the wave and is not computed (blocks beyond the words' range always are).
template <typename C, typename T, int D, int CAP, int LS>
__device__ __forceinline__ bool collect_sweep(const C& q, const Geom& g, const void* K, char* tiles, int* ovf, char* lds_cells,
                                              bool live, float thr, void* cells, uint2* mylist, int& cnt, unsigned& n_qk,
                                              unsigned& n_cand_tiles, const uint32_t* blockbits = nullptr,
                                              int strip_no = -1) {
  constexpr int KT = C::KT, NSB = C::NSB;
  // candidates are the keys with a * dot > thr: in raw units, dot > cut.  Rounding may move a key that
  // sits on the threshold (probability ~ 0) in or out of the list; the consumers recompute its value.
  // Scale 0 (a = 0): every visible key ties; they all qualify iff thr < 0.
  const float cut = !live ? kInf : (q.a > 0.f ? thr / q.a : (thr < 0.f ? -3.0e38f : kInf));
  if (q.tid < 3) ovf[q.tid] = 0;
  CellBuf<CAP, LS> cb;
  cb.init(cells, lds_cells, q.tid, strip_no < 0 ? (int)blockIdx.x : strip_no);  // (which of the scratch strips is this workgroup's)
  int ncell = 0;
  Slot slots[1];
  slots[0].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(K) + (long long)q.b * g.kv_sb +
                                                (long long)q.h * g.kv_sh);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);
  sweep_tiles<C, T, D, 1, 0, ListCfg<T, D>::kDepth>(
      tiles, slots, q.ntiles, g.Nk, q.tid, [&](int kt) { return q.tile_in_window(kt); },
      [&](int kt, const char* tl) {
        if (!q.tile_in_wave_window(kt)) return;
        const bool interior = (kt + 1) * KT <= q.wave_lim_min;
        uint32_t act = interior ? ((1u << NSB) - 1u) : q.visible_bits(kt);
        if (blockbits && (kt + 1) * NSB <= ListCfg<T, D>::kFlagWords * 32) {
          const int jb = kt * NSB;
          act &= __builtin_amdgcn_readfirstlane(blockbits[jb >> 5]) >> (jb & 31);
          if (act == 0u) return;
        }
        f32x16_t acc[NSB];
        if (interior && act == (1u << NSB) - 1u) {
          q.scores_all(tl, acc, kt);
        } else {
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb)
            if (act & (1u << sb)) acc[sb] = q.scores(tl, sb, kt);
        }
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) {
          if (!(act & (1u << sb))) continue;
          int j0 = kt * KT + sb * 32;
          ++n_qk;
          if (j0 + 32 > q.wave_lim_min) {
            int rel = q.lim - j0;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[sb][e] = (q.key_of(e) < rel) ? acc[sb][e] : -kInf;
          }
          // maxima of the four 4-key groups of the lane, then of the block
          float gm[4];
#pragma unroll
          for (int gq = 0; gq < 4; ++gq)
            gm[gq] = fmaxf(fmaxf(acc[sb][4 * gq], acc[sb][4 * gq + 1]), fmaxf(acc[sb][4 * gq + 2], acc[sb][4 * gq + 3]));
          float lm = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
          // masked entries are -inf and never exceed the cutoff
          if (__ballot(lm > cut) == 0ull) continue;
          ++n_cand_tiles;
#pragma unroll
          for (int cl = 0; cl < 4; ++cl) {
            if (gm[cl] > cut) {
              cb.store(ncell, f32x4_t{acc[sb][4 * cl], acc[sb][4 * cl + 1], acc[sb][4 * cl + 2], acc[sb][4 * cl + 3]},
                       j0 + q.key_of(4 * cl));
              ++ncell;
            }
          }
        }
        // once per tile: a strip that overflowed (its last cell was overwritten: the lists are discarded)
        if (__ballot(ncell > CAP) != 0ull && q.lane == 0) ovf[kt & 1] = 1;
      },
      // flags of the previous tile's parity were final before the barrier that ended that tile
      [&](int kt) { return kt > 0 && ovf[(kt - 1) & 1] != 0; });
  // the sweep ended on a barrier: both flags are final
  bool fits = (ovf[0] | ovf[1]) == 0;
  if (fits) {
    // a cell holds at most four candidates, so there are at least as many candidates as cells.  One pass: the
    // scores above the cutoff go to the list; a list that would grow beyond CAP raises the third flag, and the
    // block's lists are then discarded as a whole.
    int total = 0;
    for (int k = 0; k < ncell; ++k) {
      f32x4_t dv;
      int jc;
      cb.load(k, dv, jc);
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        if (dv[rr] > cut) {
          if (cnt < CAP) {
            mylist[cnt * kListStride] = make_uint2((unsigned)(jc + rr), __float_as_uint(dv[rr]));
            ++cnt;
          }
          ++total;
        }
      }
    }
    if (total > CAP) ovf[2] = 1;
    __syncthreads();
    fits = ovf[2] == 0;
  }
  return fits;
}

// Lower bound of the threshold from the two-element sub-problem {y1 >= y2} (y = (alpha-1) s) and the left
// end y1 - 1 of the bracket of App. A eq. (bounds).  alpha 1.5 and 2: closed forms.  Other alpha: Newton steps
// on f(t) = (y1-t)^r + [y2-t]_+^r - 1 from t = y1 - 1, where f >= 0: f is convex and decreasing, so the
// iterates rise towards the root and stay on its left -- each of them is a valid bound.
template <int AM>
__device__ __forceinline__ float two_key_bound(float y1, float y2, float r) {
  float lo = y1 - 1.0f;
  const float dlt = y1 - y2;
  if (!(dlt < 1.0f)) return lo;  // y2 is zero already at the left end (also y2 = -inf)
  if (AM == 2) return fmaxf(lo, 0.5f * (y1 + y2 - 1.0f));
  float t = lo;
  if (AM == 1) {
    // closed form; the hardware square root is good to an ulp, which the step back below covers
    t = 0.5f * (y1 + y2) - __builtin_amdgcn_sqrtf(0.5f * (1.0f - 0.5f * dlt * dlt));
    return fmaxf(lo, t - 4e-6f * fmaxf(1.0f, fabsf(t)));
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const float x1 = y1 - t, x2 = fmaxf(y2 - t, 0.f);
    const float f = pow_r<AM>(x1, r) + pow_r<AM>(x2, r) - 1.0f;
    const float fp = r * (pow_rm1<AM>(x1, r) + pow_rm1<AM>(x2, r));
    t += fmaxf(f, 0.f) / fp;  // fp >= r x1^(r-1) > 0 while t < y1
  }
  // rounding may carry the last iterate a few ulps past the root: step back by more than that
  return fmaxf(lo, t - 4e-6f * fmaxf(1.0f, fabsf(t)));
}

// BITS: the kernel for long sequences (Nk >= ListCfg::kFlagMinKeys), which keeps the block bits described below
template <typename T, int D, int AM, bool BIAS, bool BITS>
__device__ __forceinline__ void fwd_lists_block(const FwdSparseArgs& A, int bh_, int blk_, char* smem, int strip_no = -1) {
  using C = QCtx<T, D, ListCfg<T, D>::kTile, BIAS>;
  constexpr int KT = C::KT, NSB = C::NSB, TB = C::kTileBytes;
  const Geom& g = A.g;
  char* tiles = smem;  // 2 buffers x 1 slot
  int* ovf = reinterpret_cast<int*>(smem + 2 * TB);  // sticky overflow flags: [0], [1] by tile parity, [2] list
  char* lds_cells = smem + 2 * TB + 16;
  using Cfg = ListCfg<T, D>;
  uint32_t* allbits = reinterpret_cast<uint32_t*>(lds_cells + (size_t)Cfg::kLdsCells * kThreads * 20);
  // Long sequences: the first sweep notes, per wave, the 32-key blocks in which some lane's largest score comes
  // within the bracket's width of that lane's running maximum.  The final cutoff is at least (final maximum) - 1/a
  // in raw units (App. A eq. (bounds), left end), and the running maximum never exceeds the final one: a block
  // that fails this test for every lane holds no candidate, and the second sweep does not compute it.
  // At n = 32768 (B 1, H 12) 44 % of the blocks keep their bit against 12 % that hold a candidate: a lane's
  // running maximum is beaten O(log n) times along the sweep, and a block stays if any of its 64 lanes passes.
  // Neither the running two-key bound as the cutoff (42 %) nor a first pass over every eighth tile to raise the
  // running maxima early (44 %) changed that.
  constexpr bool keep_bits = BITS;
  if (keep_bits)
    for (int w = threadIdx.x; w < kWaves * Cfg::kFlagWords; w += kThreads) allbits[w] = 0u;  // (first barrier: the sweep's)

  if (threadIdx.x < kWaves) ovf[threadIdx.x] = 0;  // during the first sweep: the waves' votes (see `votes` below)

  C q;
  q.init(g, A.Q, bh_, blk_);
  q.init_window(g);
  uint32_t* mybits = allbits + q.wave * Cfg::kFlagWords;
  const int flag_idx = q.bh * A.nqb + q.qb;
  const long long row_idx = (long long)q.bh * g.Nq + (q.valid ? q.i : 0);
  const bool live = q.valid && q.lim > 0;

  if (q.block_lim == 0) {  // no row of this workgroup sees any key: the finish kernel writes the zeros
    if (q.valid) {
      A.lcnt[row_idx * 2 + q.hh] = 0;
      if (q.hh == 0) A.bounds[row_idx] = make_float2(0.f, 0.f);
    }
    if (q.tid == 0) A.dense_flag[flag_idx] = 0;
    return;
  }

  Slot slots[1];
  slots[0].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.K) + (long long)q.b * g.kv_sb +
                                                (long long)q.h * g.kv_sh);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);
  unsigned n_vis = 0, n_qk2 = 0, n_cand_tiles = 0;

  // ---------------------------------------------- 1. row max and runner-up
  // m1 >= m2 are the two largest per-cell maxima seen by this lane: two distinct scores of the row
  float m1 = -kInf, m2 = -kInf;
  // BITS: the bracket's width in raw units, a little wider than needed (rounding); lanes without a live row never pass
  const float reach = (q.valid && q.lim > 0) ? (q.a > 0.f ? 1.0001f / q.a : 3.0e38f) : -kInf;
  // Dense rows are found out on the first tile: where, for three quarters of a wave's rows, half of the keys of
  // the tile's first block come within the bracket's width of the block's largest score, the lists would overflow anyway (a row of
  // the paper's sparse setting has a handful of such keys).  A block all of whose waves vote so is handed to the
  // tiled kernel after two tiles instead of after a full sweep (a matter of time only: the tiled kernel handles
  // any row).  votes: one word per wave in the overflow flags' place, which the second sweep zeroes again.
  int* votes = ovf;
  int kt_vote = 0;  // the first tile of the sweep
  if constexpr (BIAS) kt_vote = q.kt_first;
  auto max_body = [&](int kt, const char* tl) {
        if (!q.tile_in_wave_window(kt)) return;
        uint32_t bits = 0u;
        if ((kt + 1) * KT <= q.wave_lim_min) {
          f32x16_t acc[NSB];
          q.scores_all(tl, acc, kt);
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb) {
            float lm = max16(acc[sb]);
            if (sb == 0 && kt == kt_vote) {  // the vote, on the lane's 16 keys of the tile's first block
              int near = 0;
#pragma unroll
              for (int e = 0; e < 16; ++e) near += (acc[0][e] + reach > lm) ? 1 : 0;
              if (__popcll(__ballot(near >= 8)) >= 48 && q.lane == 0) votes[q.wave] = 1;
            }
            m2 = fmaxf(m2, fminf(m1, lm));
            m1 = fmaxf(m1, lm);
            if (keep_bits && __ballot(lm + reach > m1) != 0ull) bits |= 1u << sb;
          }
          n_vis += NSB;
        } else {
          const uint32_t act = q.visible_bits(kt);
#pragma unroll
          for (int sb = 0; sb < NSB; ++sb) {
            if (!(act & (1u << sb))) continue;
            int j0 = kt * KT + sb * 32;
            f32x16_t acc = q.scores(tl, sb, kt);
            ++n_vis;
            if (j0 + 32 > q.wave_lim_min) {
              int rel = q.lim - j0;
#pragma unroll
              for (int e = 0; e < 16; ++e) acc[e] = (q.key_of(e) < rel) ? acc[e] : -kInf;
            }
            float lm = max16(acc);
            m2 = fmaxf(m2, fminf(m1, lm));
            m1 = fmaxf(m1, lm);
            if (keep_bits && __ballot(lm + reach > m1) != 0ull) bits |= 1u << sb;
          }
        }
        // (each wave writes only its own words)
        if (bits != 0u && (kt + 1) * NSB <= Cfg::kFlagWords * 32 && q.lane == 0) mybits[(kt * NSB) >> 5] |= bits << ((kt * NSB) & 31);
      };
  auto all_dense = [&]() { return (votes[0] & votes[1] & votes[2] & votes[3]) != 0; };
  sweep_tiles<C, T, D, 1, 0, ListCfg<T, D>::kDepth>(
      tiles, slots, q.ntiles, g.Nk, q.tid, [&](int kt) { return q.tile_in_window(kt); }, max_body,
      // (the votes of a tile are final before the barrier that ends it)
      [&](int kt) { return kt == kt_vote + 1 && all_dense(); });
  if (all_dense()) {  // (the sweep ended on a barrier)
    __syncthreads();  // every thread has read the votes before the next block's zeroes them
    if (q.tid == 0) A.dense_flag[flag_idx] = kFlagDense;
    if (A.stats && q.lane == 0) atomicAdd(&A.stats[ENTMAX_STAT_FWD_LIST_QK], (unsigned long long)n_vis);
    return;
  }
  {
    float p1 = __shfl_xor(m1, 32), p2 = __shfl_xor(m2, 32);
    float hi1 = fmaxf(m1, p1);
    m2 = fmaxf(fminf(m1, p1), fmaxf(m2, p2));
    m1 = hi1;
  }
  const float y1 = live ? q.a * m1 : 0.f;
  float lo = y1 - 1.0f;  // App. A eq. (bounds), left end
  float hi = live ? y1 - __builtin_amdgcn_exp2f(-(g.alpha - 1.0f) * __builtin_amdgcn_logf((float)q.lim)) : 0.f;
  // two-element sub-problem {y1, y2}: its threshold is a lower bound of the row's
  if (live && m2 > -kInf) lo = two_key_bound<AM>(y1, q.a * m2, 1.0f / (g.alpha - 1.0f));
  lo = fminf(lo, hi);

  // ---------------------------------------------- 2. candidate lists at tau_lb
  uint2* mylist = A.cand + list_entry<kCandCap>(q.bh, A.nqb, q.qb, q.wave, q.lane);
  int cnt = 0;
  const bool fits = collect_sweep<C, T, D, kCandCap, ListCfg<T, D>::kLdsCells>(q, g, A.K, tiles, ovf, lds_cells, live, lo, A.cells, mylist, cnt, n_qk2, n_cand_tiles,
                                                                                     keep_bits ? mybits : nullptr, strip_no);
  if (!fits) {
    // the tiled kernel takes the block, and with it what the first sweep found out about every row
    if (q.tid == 0) A.dense_flag[flag_idx] = kFlagWithBounds;
    if (q.valid && q.hh == 0) A.bounds[row_idx] = make_float2(lo, y1);
  } else {
    if (q.tid == 0) A.dense_flag[flag_idx] = 0;
    if (q.valid) {
      A.lcnt[row_idx * 2 + q.hh] = cnt;
      if (q.hh == 0) A.bounds[row_idx] = make_float2(lo, hi);
    }
  }
  if (A.stats && q.lane == 0) {
    const unsigned n_win = q.window_skipped_blocks();
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_TILES_VISIBLE], (unsigned long long)(n_vis + n_win));
    if (BIAS) atomicAdd(&A.stats[ENTMAX_STAT_FWD_WINDOW_SKIPPED], (unsigned long long)n_win);
    atomicAdd(&A.stats[ENTMAX_STAT_FWD_LIST_QK], (unsigned long long)(n_vis + n_qk2));
    if (fits) {
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_CAND_TILES], (unsigned long long)n_cand_tiles);
      if (q.wave == 0) atomicAdd(&A.stats[ENTMAX_STAT_FWD_SPARSE_BLOCKS], 1ull);
    }
  }
}

template <typename T, int D, int AM, bool BIAS, bool BITS>
__global__ __launch_bounds__(kThreads, (ListCfg<T, D>::kOcc)) void fwd_lists_kernel(FwdSparseArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  PairItem it;
  if (A.unpaired) {  // a head's blocks on one XCD, the longest first
    const int item = xcd_remap(blockIdx.x, gridDim.x);
    it.bh = __builtin_amdgcn_readfirstlane(item / A.nqb);
    it.first = A.nqb - 1 - __builtin_amdgcn_readfirstlane(item % A.nqb);
    it.second = -1;
  } else {
    it = pair_item(A.nqb);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    A.dense_flag[A.g.B * A.g.H * A.nqb] = 0;
  }
  if (blockIdx.x == 0 && A.pool_cursor && (int)threadIdx.x < A.pool_parts)
    *reinterpret_cast<unsigned long long*>(A.pool_cursor + (size_t)threadIdx.x * kSavedCursorStride) = 0ull;
  if (A.kcount) {
    // this workgroup's share of its head's per-key counters starts at zero for the finish kernel
    const int npair = A.unpaired ? A.nqb : (A.nqb + 1) >> 1, pp = A.nqb - 1 - it.first;
    const int chunk = (A.g.Nk + npair - 1) / npair;
    int* dst = A.kcount + (long long)it.bh * A.g.Nk;
    for (int j = pp * chunk + (int)threadIdx.x; j < min(A.g.Nk, (pp + 1) * chunk); j += kThreads) dst[j] = 0;
  }
  for (int part = 0; part < 2; ++part) {
    const int blk = part ? it.second : it.first;
    if (blk < 0) break;
    if (part) __syncthreads();
    fwd_lists_block<T, D, AM, BIAS, BITS>(A, it.bh, blk, smem);
  }
}

// ------------------------------------------------- long sequences: two query blocks per workgroup
// The same two sweeps as fwd_lists_block<.., BITS = true> for the adjacent blocks 2 sblk and 2 sblk + 1 at once:
// every wave holds its 32-row group of both blocks (64 query rows), so that a K fragment read from LDS feeds two
// matrix instructions and a K tile staged through LDS serves 256 rows.  Each block keeps its own lists, flags,
// bounds and block bits, exactly as if it had run alone.  Used where the launch still fills the chip with half as
// many workgroups (Nk >= ListCfg::kFlagMinKeys).
template <typename T, int D>
struct PairCfg {
  using Cfg = ListCfg<T, D>;
  static constexpr int kLdsCells = 1;   // cells per thread and block kept in LDS
  static constexpr int kFlagWords = 64; // block bits per wave and block: 65536 keys
  static constexpr size_t kLdsBytes = 2 * (size_t)Cfg::kTile * D * sizeof(T) + 32 + 2 * (size_t)kLdsCells * kThreads * 20 +
                                      2 * (size_t)kWaves * kFlagWords * 4;
};

template <typename T, int D, int AM, bool BIAS>
__device__ __forceinline__ void fwd_lists_pair(const FwdSparseArgs& A, int bh_, int sblk, char* smem) {
  using C = QCtx<T, D, ListCfg<T, D>::kTile, BIAS>;
  using P = PairCfg<T, D>;
  using KTile = typename C::KTile;
  constexpr int KT = C::KT, NSB = C::NSB, NC = C::NC, TB = C::kTileBytes, LS = P::kLdsCells, W = P::kFlagWords;
  constexpr uint32_t kAll = (1u << NSB) - 1u;
  const Geom& g = A.g;
  char* tiles = smem;
  int* ovf = reinterpret_cast<int*>(smem + 2 * TB);  // [2 blocks][3], see collect_sweep
  char* lds_cells = smem + 2 * TB + 32;
  uint32_t* allbits = reinterpret_cast<uint32_t*>(lds_cells + 2 * (size_t)LS * kThreads * 20);  // [2][kWaves][W]
  for (int w = threadIdx.x; w < 2 * kWaves * W; w += kThreads) allbits[w] = 0u;
  if (threadIdx.x < 6) ovf[threadIdx.x] = 0;  // (first barrier: init_window's or the first sweep's)

  C q[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    q[k].init(g, A.Q, bh_, 2 * sblk + k);
    q[k].init_window(g);
  }
  const int tid = q[0].tid, wave = q[0].wave, lane = q[0].lane;
  uint32_t* mybits[2] = {allbits + wave * W, allbits + (kWaves + wave) * W};
  const int ntiles = q[1].ntiles;  // the later block sees at least the keys of the earlier one
  bool live[2];
  long long row_idx[2];
  int flag_idx[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    live[k] = q[k].valid && q[k].lim > 0;
    row_idx[k] = (long long)q[k].bh * g.Nq + (q[k].valid ? q[k].i : 0);
    flag_idx[k] = q[k].bh * A.nqb + q[k].qb;
  }
  if (q[1].block_lim == 0) {  // no row of either block sees any key: the finish kernel writes the zeros
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (q[k].valid) {
        A.lcnt[row_idx[k] * 2 + q[k].hh] = 0;
        if (q[k].hh == 0) A.bounds[row_idx[k]] = make_float2(0.f, 0.f);
      }
      if (tid == 0) A.dense_flag[flag_idx[k]] = 0;
    }
    return;
  }
  Slot slots[1];
  slots[0].base = reinterpret_cast<const char*>(reinterpret_cast<const T*>(A.K) + (long long)q[0].b * g.kv_sb +
                                                (long long)q[0].h * g.kv_sh);
  slots[0].row_bytes = g.kv_sn * (long long)sizeof(T);
  auto needed = [&](int kt) { return q[0].tile_in_window(kt) || q[1].tile_in_window(kt); };
  // 32-key blocks of tile kt some row of the wave's group of block k sees
  auto visible = [&](int k, int kt) -> uint32_t { return q[k].tile_in_wave_window(kt) ? q[k].visible_bits(kt) : 0u; };
  auto mask_block = [&](int k, f32x16_t& acc, int j0) {
    const int rel = q[k].lim - j0;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = (q[k].key_of(e) < rel) ? acc[e] : -kInf;
  };
  // the K fragments of a 32-key block, shared by both groups
  auto load_k = [&](const char* tl, int sb, Frag<T> (&kf)[NC]) {
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) kf[cc] = q[0].koff[cc].load(tl, sb * 32 * KTile::kRowBytes);
  };
  auto product = [&](int k, const Frag<T> (&kf)[NC], int j0) -> f32x16_t {
    f32x16_t acc = q[k].block_start(j0);
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) acc = Elem<T>::mma(kf[cc], q[k].qf[cc], acc);
    return acc;
  };
  unsigned n_vis[2] = {0u, 0u}, n_qk2[2] = {0u, 0u}, n_cand_tiles[2] = {0u, 0u};

  // ---------------------------------------------- 1. row maxima, runners-up and the block bits
  float m1[2] = {-kInf, -kInf}, m2[2] = {-kInf, -kInf}, reach[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) reach[k] = live[k] ? (q[k].a > 0.f ? 1.0001f / q[k].a : 3.0e38f) : -kInf;
  sweep_tiles<C, T, D, 1, 0, ListCfg<T, D>::kDepth>(tiles, slots, ntiles, g.Nk, tid, needed, [&](int kt, const char* tl) {
    uint32_t act[2] = {visible(0, kt), visible(1, kt)};
    if ((act[0] | act[1]) == 0u) return;
    uint32_t bits[2] = {0u, 0u};
    auto take = [&](int k, f32x16_t& acc, int sb) {
      const int j0 = kt * KT + sb * 32;
      ++n_vis[k];
      if (j0 + 32 > q[k].wave_lim_min) mask_block(k, acc, j0);
      const float lm = max16(acc);
      m2[k] = fmaxf(m2[k], fminf(m1[k], lm));
      m1[k] = fmaxf(m1[k], lm);
      if (__ballot(lm + reach[k] > m1[k]) != 0ull) bits[k] |= 1u << sb;
    };
    if (act[0] == kAll && act[1] == kAll) {
      // every block for both groups: the fragments of block sb + 1 are requested before the products of block sb
      Frag<T> kf[2][NC];
      load_k(tl, 0, kf[0]);
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
        if (sb + 1 < NSB) load_k(tl, sb + 1, kf[(sb + 1) & 1]);
        const int j0 = kt * KT + sb * 32;
        f32x16_t a0 = q[0].block_start(j0), a1 = q[1].block_start(j0);
#pragma unroll
        for (int cc = 0; cc < NC; ++cc) {
          a0 = Elem<T>::mma(kf[sb & 1][cc], q[0].qf[cc], a0);
          a1 = Elem<T>::mma(kf[sb & 1][cc], q[1].qf[cc], a1);
        }
        take(0, a0, sb);
        take(1, a1, sb);
      }
    } else {
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
        if (((act[0] | act[1]) & (1u << sb)) == 0u) continue;
        Frag<T> kf[NC];
        load_k(tl, sb, kf);
        f32x16_t acc[2];  // (both products before the vector work on either)
#pragma unroll
        for (int k = 0; k < 2; ++k)
          if ((act[k] & (1u << sb)) != 0u) acc[k] = product(k, kf, kt * KT + sb * 32);
#pragma unroll
        for (int k = 0; k < 2; ++k)
          if ((act[k] & (1u << sb)) != 0u) take(k, acc[k], sb);
      }
    }
    if ((kt + 1) * NSB <= W * 32 && lane == 0) {  // (each wave writes only its own words)
#pragma unroll
      for (int k = 0; k < 2; ++k)
        if (bits[k] != 0u) mybits[k][(kt * NSB) >> 5] |= bits[k] << ((kt * NSB) & 31);
    }
  });
  float lo[2], hi[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const float p1 = __shfl_xor(m1[k], 32), p2 = __shfl_xor(m2[k], 32);
    const float top = fmaxf(m1[k], p1);
    m2[k] = fmaxf(fminf(m1[k], p1), fmaxf(m2[k], p2));
    m1[k] = top;
    const float y1 = live[k] ? q[k].a * m1[k] : 0.f;
    lo[k] = y1 - 1.0f;  // App. A eq. (bounds), left end
    hi[k] = live[k] ? y1 - __builtin_amdgcn_exp2f(-(g.alpha - 1.0f) * __builtin_amdgcn_logf((float)q[k].lim)) : 0.f;
    if (live[k] && m2[k] > -kInf) lo[k] = two_key_bound<AM>(y1, q[k].a * m2[k], 1.0f / (g.alpha - 1.0f));
    lo[k] = fminf(lo[k], hi[k]);
  }

  // ---------------------------------------------- 2. candidate lists at tau_lb (see collect_sweep)
  float cut[2];
  CellBuf<kCandCap, LS> cb[2];
  int ncell[2] = {0, 0};
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    cut[k] = !live[k] ? kInf : (q[k].a > 0.f ? lo[k] / q[k].a : (lo[k] < 0.f ? -3.0e38f : kInf));
    cb[k].init(A.cells, lds_cells + k * CellBuf<kCandCap, LS>::kLdsBytes, tid, 2 * (int)blockIdx.x + k);
  }
  sweep_tiles<C, T, D, 1, 0, ListCfg<T, D>::kDepth>(
      tiles, slots, ntiles, g.Nk, tid, needed,
      [&](int kt, const char* tl) {
        uint32_t act[2] = {visible(0, kt), visible(1, kt)};
        if ((kt + 1) * NSB <= W * 32) {
          const int jb = kt * NSB;
#pragma unroll
          for (int k = 0; k < 2; ++k) act[k] &= __builtin_amdgcn_readfirstlane(mybits[k][jb >> 5]) >> (jb & 31);
        }
        // a block whose strip overflowed is lost to the tiled kernel anyway (flags of the previous tile's parity
        // were final before the barrier that ended that tile)
#pragma unroll
        for (int k = 0; k < 2; ++k)
          if (kt > 0 && ovf[3 * k + ((kt - 1) & 1)] != 0) act[k] = 0u;
        if ((act[0] | act[1]) == 0u) return;
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) {
          if (((act[0] | act[1]) & (1u << sb)) == 0u) continue;
          Frag<T> kf[NC];
          load_k(tl, sb, kf);
          const int j0 = kt * KT + sb * 32;
          f32x16_t accs[2];  // (both products before the vector work on either)
#pragma unroll
          for (int k = 0; k < 2; ++k)
            if ((act[k] & (1u << sb)) != 0u) accs[k] = product(k, kf, j0);
#pragma unroll
          for (int k = 0; k < 2; ++k) {
            if ((act[k] & (1u << sb)) == 0u) continue;
            f32x16_t& acc = accs[k];
            ++n_qk2[k];
            if (j0 + 32 > q[k].wave_lim_min) mask_block(k, acc, j0);
            float gm[4];
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
              gm[gq] = fmaxf(fmaxf(acc[4 * gq], acc[4 * gq + 1]), fmaxf(acc[4 * gq + 2], acc[4 * gq + 3]));
            const float lm = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
            if (__ballot(lm > cut[k]) == 0ull) continue;
            ++n_cand_tiles[k];
#pragma unroll
            for (int cl = 0; cl < 4; ++cl) {
              if (gm[cl] > cut[k]) {
                cb[k].store(ncell[k], f32x4_t{acc[4 * cl], acc[4 * cl + 1], acc[4 * cl + 2], acc[4 * cl + 3]},
                            j0 + q[k].key_of(4 * cl));
                ++ncell[k];
              }
            }
          }
        }
#pragma unroll
        for (int k = 0; k < 2; ++k)
          if (__ballot(ncell[k] > kCandCap) != 0ull && lane == 0) ovf[3 * k + (kt & 1)] = 1;
      },
      [&](int kt) { return kt > 0 && ovf[(kt - 1) & 1] != 0 && ovf[3 + ((kt - 1) & 1)] != 0; });
  // the sweep ended on a barrier: the strips' flags are final
  int cnt[2] = {0, 0};
  bool fits[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    fits[k] = (ovf[3 * k] | ovf[3 * k + 1]) == 0;
    if (fits[k]) {
      uint2* mylist = A.cand + list_entry<kCandCap>(q[k].bh, A.nqb, q[k].qb, wave, lane);
      int total = 0;
      for (int c = 0; c < ncell[k]; ++c) {
        f32x4_t dv;
        int jc;
        cb[k].load(c, dv, jc);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          if (dv[rr] > cut[k]) {
            if (cnt[k] < kCandCap) {
              mylist[cnt[k] * kListStride] = make_uint2((unsigned)(jc + rr), __float_as_uint(dv[rr]));
              ++cnt[k];
            }
            ++total;
          }
        }
      }
      if (total > kCandCap) ovf[3 * k + 2] = 1;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    fits[k] = fits[k] && ovf[3 * k + 2] == 0;
    if (tid == 0) A.dense_flag[flag_idx[k]] = fits[k] ? 0 : 1;
    if (fits[k] && q[k].valid) {
      A.lcnt[row_idx[k] * 2 + q[k].hh] = cnt[k];
      if (q[k].hh == 0) A.bounds[row_idx[k]] = make_float2(lo[k], hi[k]);
    }
    if (A.stats && lane == 0) {
      const unsigned n_win = q[k].window_skipped_blocks();
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_TILES_VISIBLE], (unsigned long long)(n_vis[k] + n_win));
      if (BIAS) atomicAdd(&A.stats[ENTMAX_STAT_FWD_WINDOW_SKIPPED], (unsigned long long)n_win);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_LIST_QK], (unsigned long long)(n_vis[k] + n_qk2[k]));
      if (fits[k]) {
        atomicAdd(&A.stats[ENTMAX_STAT_FWD_CAND_TILES], (unsigned long long)n_cand_tiles[k]);
        if (wave == 0) atomicAdd(&A.stats[ENTMAX_STAT_FWD_SPARSE_BLOCKS], 1ull);
      }
    }
  }
}

template <typename T, int D, int AM, bool BIAS>
__global__ __launch_bounds__(kThreads, (ListCfg<T, D>::kOcc)) void fwd_lists_pair_kernel(FwdSparseArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nsb = (A.nqb + 1) >> 1;  // pairs of adjacent blocks per head
  const PairItem it = pair_item(nsb);
  if (blockIdx.x == 0 && threadIdx.x == 0) A.dense_flag[A.g.B * A.g.H * A.nqb] = 0;
  if (blockIdx.x == 0 && A.pool_cursor && (int)threadIdx.x < A.pool_parts)
    *reinterpret_cast<unsigned long long*>(A.pool_cursor + (size_t)threadIdx.x * kSavedCursorStride) = 0ull;
  if (A.kcount) {
    // this workgroup's share of its head's per-key counters starts at zero for the finish kernel
    const int npair = (nsb + 1) >> 1, pp = nsb - 1 - it.first;
    const int chunk = (A.g.Nk + npair - 1) / npair;
    int* dst = A.kcount + (long long)it.bh * A.g.Nk;
    for (int j = pp * chunk + (int)threadIdx.x; j < min(A.g.Nk, (pp + 1) * chunk); j += kThreads) dst[j] = 0;
  }
  for (int part = 0; part < 2; ++part) {
    const int sblk = part ? it.second : it.first;
    if (sblk < 0) break;
    if (part) __syncthreads();
    if (2 * sblk + 1 < A.nqb)
      fwd_lists_pair<T, D, AM, BIAS>(A, it.bh, sblk, smem);
    else  // a head's odd last block
      fwd_lists_block<T, D, AM, BIAS, true>(A, it.bh, 2 * sblk, smem, 2 * (int)blockIdx.x);
  }
}

// widen 8 (bf16) or 4 (fp32) consecutive elements to fp32
template <typename T>
__device__ __forceinline__ void load_row_f32(const T* row, int n, float* out) {
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int c8 = 0; c8 < n / 8; ++c8) {
      u32x4_t w = *reinterpret_cast<const u32x4_t*>(row + 8 * c8);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        out[8 * c8 + 2 * k] = __uint_as_float(w[k] << 16);
        out[8 * c8 + 2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
      }
    }
  } else {
#pragma unroll
    for (int c4 = 0; c4 < n / 4; ++c4) {
      f32x4_t w = *reinterpret_cast<const f32x4_t*>(row + 4 * c4);
#pragma unroll
      for (int k = 0; k < 4; ++k) out[4 * c4 + k] = w[k];
    }
  }
}
// The same row kept as loaded (16-byte words) and widened only where it is used: a gather in flight
// costs half (bf16) of the registers of a widened row.
template <typename T, int N>
struct RawRow {
  static constexpr int kWords = N * (int)sizeof(T) / 16;
  u32x4_t w[kWords];
  __device__ __forceinline__ void load(const T* row) {
#pragma unroll
    for (int c = 0; c < kWords; ++c) w[c] = *reinterpret_cast<const u32x4_t*>(reinterpret_cast<const char*>(row) + 16 * c);
  }
  // element t (a compile-time index once the caller's loop is unrolled)
  __device__ __forceinline__ float get(int t) const {
    if constexpr (sizeof(T) == 2) {
      const uint32_t word = w[t >> 3][(t >> 1) & 3];
      return __uint_as_float((t & 1) ? (word & 0xffff0000u) : (word << 16));
    } else {
      return __uint_as_float(w[t >> 2][t & 3]);
    }
  }
};

template <typename T>
__device__ __forceinline__ void store_row(T* row, int n, const float* v) {
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int c8 = 0; c8 < n / 8; ++c8) *reinterpret_cast<u32x4_t*>(row + 8 * c8) = Elem<T>::pack(v + 8 * c8).v;
  } else {
#pragma unroll
    for (int c4 = 0; c4 < n / 4; ++c4)
      *reinterpret_cast<f32x4_t*>(row + 4 * c4) = f32x4_t{v[4 * c4], v[4 * c4 + 1], v[4 * c4 + 2], v[4 * c4 + 3]};
  }
}

// Row coordinates of a lane in the list kernels.  FH = 1: wave w of block qb owns rows qb*128 + 32 w .. + 31,
// lane l row (l % 32), list half hh = l / 32 -- the same assignment as in the sweeps that wrote the lists; a
// workgroup is one 128-row block.  FH = 2: two lanes per list half, each with half of that half's features
// (f = 0, 1): a wave owns 16 rows, lane l = 32 hh + 16 f + r, and two consecutive workgroups share a block.
// (li, w32): the row's lane and 32-row group in the sweeps' numbering, as list_entry() wants them.
// Where the heads divide evenly over the eight XCDs the workgroups are renumbered so that a head's rows all run on
// one XCD, the one whose L2 saw the head's keys and lists in the sweeps (finish kernel, measured on one box:
// B 4, H 12, n 4096: 54 -> 50 us; with 12 heads at n 32768, one and a half heads per XCD, it was 60 -> 73 us).
struct RowLane {
  int bh, b, h, qb, i, li, hh, f, w32;
  bool valid;
  template <int FH = 1>
  __device__ __forceinline__ void init(const Geom& g, int nqb) {
    static_assert(FH == 1 || FH == 2, "one or two lanes per list half");
    constexpr int R = 32 / FH;  // rows per wave
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int vb = (g.B * g.H) % 8 == 0 ? xcd_remap(blockIdx.x, g.B * g.H * nqb * FH) : (int)blockIdx.x;
    const int blk = vb / FH, sub = vb % FH;
    bh = blk / nqb;
    qb = blk % nqb;
    b = bh / g.H;
    h = bh % g.H;
    hh = lane >> 5;
    f = (lane & 31) / R;
    const int row_in_block = (sub * kWaves + wave) * R + (lane & (R - 1));
    li = row_in_block & 31;
    w32 = row_in_block >> 5;
    i = qb * kBlockRows + row_in_block;
    valid = i < g.Nq;
  }
};

template <typename T, int D, int AM>
__global__ __launch_bounds__(kThreads) void fwd_finish_kernel(FwdSparseArgs A) {
  const Geom& g = A.g;
  if ((int)blockIdx.x >= g.B * g.H * A.nqb) {  // riders behind the row workgroups
    transpose_ride<T, D>(A.ride, (int)blockIdx.x - g.B * g.H * A.nqb);
    return;
  }
  RowLane rl;
  rl.init(g, A.nqb);
  // (the flag is tested further down: every load that does not depend on another is issued first)
  const int block_dense = A.dense_flag[rl.bh * A.nqb + rl.qb];
  constexpr int DH = D / 2;
  const float r = 1.0f / (g.alpha - 1.0f);
  const long long row_idx = (long long)rl.bh * g.Nq + (rl.valid ? rl.i : 0);
  const int lim = rl.valid ? row_limit(g, rl.i) : 0;
  const bool live = rl.valid && lim > 0;
  const float scale = rl.valid ? row_scale(g, rl.b, rl.h, rl.i, lim, nullptr, nullptr, nullptr) : 0.f;
  const float c = scale * (1.0f / sqrtf((float)D));
  const float a = (g.alpha - 1.0f) * fabsf(c);  // same arithmetic as the sweeps that made the lists
  const int cnt_raw = A.lcnt[row_idx * 2 + rl.hh];
  const float2 bd_raw = A.bounds[row_idx];
  const int cnt = live ? cnt_raw : 0;
  const float2 bd = live ? bd_raw : make_float2(0.f, 0.f);
  const uint2* mylist = A.cand + list_entry<kCandCap>(rl.bh, A.nqb, rl.qb, threadIdx.x >> 6, threadIdx.x & 63);
  const T* Vbh = reinterpret_cast<const T*>(A.V) + (long long)rl.b * g.kv_sb + (long long)rl.h * g.kv_sh;
  float lo = bd.x, hi = bd.y, tau = bd.x;
  unsigned n_support = 0;
  // the first entries are requested before the list length is known (the slots exist whatever they hold):
  // one memory round trip less on the critical path of this latency-bound kernel
  constexpr int kEarly = 4;
  uint2 early[kEarly];
#pragma unroll
  for (int e = 0; e < kEarly; ++e) early[e] = mylist[e * kListStride];
  if (block_dense != 0) {  // the tiled kernel owns this block, and so do the backward's tiled kernels
    if (A.list && threadIdx.x == 0) A.bwd_flag[rl.bh * A.nqb + rl.qb] = kBlockNoLists;
    if (threadIdx.x == 0) {
      int* count = A.dense_flag + g.B * g.H * A.nqb;
      const int slot = atomicAdd(count, 1);
      if (slot < kSplitMaxBlocks) count[1 + slot] = rl.bh * A.nqb + rl.qb;
    }
    return;
  }
  // The 32-row group's piece of the pool, sized before the supports are known: a half row's support is part of
  // its candidate list, and a half row with more than kBwdCap support entries sends the block to the backward's
  // tiled kernels anyway.  One returning atomic per wave, in flight together with the first list entries.
  uint2* suplist = nullptr;
  int sup_off = 0;
  bool pool_full = false;
  if (A.list) {
    const int lane = threadIdx.x & 63;
    const int want = min(cnt, kBwdCap);
    int incl = want;  // inclusive running sum over the lanes
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) {
      const int up = __shfl_up(incl, sft);
      if (lane >= sft) incl += up;
    }
    const int total = __builtin_amdgcn_readlane(incl, 63);
    // the groups take the pool's parts in turn
    const int part = (int)(((unsigned)blockIdx.x * kWaves + (threadIdx.x >> 6)) & (unsigned)(A.pool_parts - 1));
    unsigned long long base = 0ull;
    if (lane == 0 && total > 0)
      base = atomicAdd(reinterpret_cast<unsigned long long*>(A.pool_cursor + (size_t)part * kSavedCursorStride),
                       (unsigned long long)total);
    base = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(base >> 32)) << 32) |
           (unsigned)__builtin_amdgcn_readfirstlane((int)base);
    pool_full = total > 0 && base + (unsigned long long)total > (unsigned long long)A.pool_part_cap;
    sup_off = pool_full ? 0 : (int)(part * A.pool_part_cap + (long long)base) + incl - want;
    if (!pool_full) suplist = A.list + sup_off;
  }
  int scnt = 0;  // support entries of this half row

  // NE: list entries per lane held in registers; chosen per wave from the longest list it holds.
  // (Same sums in the same order whichever NE is chosen: entry order.)
  auto finish = [&](auto ne_tag) {
    constexpr int NE = decltype(ne_tag)::value;
    float yv[NE], dvv[NE];
    unsigned jv[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      uint2 en = make_uint2(0u, 0u);
      if (e < kEarly)
        en = early[e];
      else if (e < cnt)
        en = mylist[e * kListStride];
      jv[e] = (e < cnt) ? en.x : 0u;
      dvv[e] = __uint_as_float(en.y);
      yv[e] = (e < cnt) ? a * dvv[e] : -kInf;  // -inf: never positive
    }
    // entries beyond the NE held in registers (few lanes) are read again wherever they are needed
    const bool has_tail = __ballot(cnt > NE) != 0ull;
    bool done = !live;
    int iter = 0;
    while (__ballot(!done) != 0ull && iter < kMaxSolveIters) {
      RowSums sums;
      sums.clear();
#pragma unroll
      for (int e = 0; e < NE; ++e) accumulate<AM>(sums, yv[e] - tau, r);
      if (has_tail)
        for (int e = NE; e < cnt; ++e) accumulate<AM>(sums, a * __uint_as_float(mylist[e * kListStride].y) - tau, r);
      sums.combine_halves();
      if (!done) done = solve_step<AM>(sums, r, tau, lo, hi);
      ++iter;
    }
    // O = sum p_j v_j: each lane of a pair takes half of the features of every entry of the row
    float oacc[DH];
#pragma unroll
    for (int t = 0; t < DH; ++t) oacc[t] = 0.f;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      // (the same expression as the backward's row kernel, so that both sides agree on the support)
      float p_own = (live && e < cnt) ? pow_r<AM>(fmaxf(fmaf(dvv[e], a, -tau), 0.f), r) : 0.f;
      float p_oth = __shfl_xor(p_own, 32);
      unsigned j_oth = (unsigned)__shfl_xor((int)jv[e], 32);
      if (p_own > 0.f) {
        ++n_support;
        if (suplist && scnt < kBwdCap) {
          // (writing the entries after the gathers, so that the counter's answer is not waited for here, gained nothing)
          const unsigned rank = (unsigned)atomicAdd(&A.kcount[(long long)rl.bh * g.Nk + jv[e]], 1);
          suplist[scnt] = make_uint2(jv[e] | (min(rank, kSavedRankMost) << kSavedKeyBits), __float_as_uint(dvv[e]));
        }
        ++scnt;
      }
#pragma unroll
      for (int src = 0; src < 2; ++src) {
        // both lanes of the pair take the same entry: entry e of the lane whose half index is src
        float p = (rl.hh == src) ? p_own : p_oth;
        unsigned j = (rl.hh == src) ? jv[e] : j_oth;
        if (__ballot(p > 0.f) == 0ull) continue;
        if (p > 0.f) {
          RawRow<T, DH> vv;
          vv.load(Vbh + (long long)j * g.kv_sn + rl.hh * DH);
#pragma unroll
          for (int t = 0; t < DH; ++t) oacc[t] = fmaf(p, vv.get(t), oacc[t]);
        }
      }
    }
    if (has_tail) {
      for (int e = NE; __ballot(e < cnt) != 0ull; ++e) {
        uint2 en = make_uint2(0u, 0u);
        if (e < cnt) en = mylist[e * kListStride];
        float p_own = (live && e < cnt) ? pow_r<AM>(fmaxf(fmaf(__uint_as_float(en.y), a, -tau), 0.f), r) : 0.f;
        float p_oth = __shfl_xor(p_own, 32);
        unsigned j_oth = (unsigned)__shfl_xor((int)en.x, 32);
        if (p_own > 0.f) {
          ++n_support;
          if (suplist && scnt < kBwdCap) {
            const unsigned rank = (unsigned)atomicAdd(&A.kcount[(long long)rl.bh * g.Nk + en.x], 1);
            suplist[scnt] = make_uint2(en.x | (min(rank, kSavedRankMost) << kSavedKeyBits), en.y);
          }
          ++scnt;
        }
#pragma unroll
        for (int src = 0; src < 2; ++src) {
          float p = (rl.hh == src) ? p_own : p_oth;
          unsigned j = (rl.hh == src) ? en.x : j_oth;
          if (p > 0.f) {
            RawRow<T, DH> vv;
            vv.load(Vbh + (long long)j * g.kv_sn + rl.hh * DH);
#pragma unroll
            for (int t = 0; t < DH; ++t) oacc[t] = fmaf(p, vv.get(t), oacc[t]);
          }
        }
      }
    }
    if (rl.valid) {
      T* orow = reinterpret_cast<T*>(A.O) + (long long)rl.b * g.q_sb + (long long)rl.h * g.q_sh +
                (long long)rl.i * g.q_sn + rl.hh * DH;
      store_row<T>(orow, DH, oacc);
      if (rl.hh == 0) A.tau[row_idx] = live ? tau : 0.f;
      if (A.list) A.slcnt[row_idx * 2 + rl.hh] = (int)(((unsigned)sup_off << 5) | (unsigned)(pool_full ? 0 : min(scnt, kBwdCap)));
    }
  };
  if (__ballot(cnt > 4) == 0ull)
    finish(std::integral_constant<int, 4>());
  else
    finish(std::integral_constant<int, 8>());

  if (A.list) {
    // a support longer than the backward's lists hold, or no room left in the pool, sends the block to the
    // backward's tiled kernels
    const int any_long = __syncthreads_or((scnt > kBwdCap || pool_full) ? 1 : 0);
    if (threadIdx.x == 0) A.bwd_flag[rl.bh * A.nqb + rl.qb] = any_long ? kBlockListsUnused : 0;
  }
  if (A.stats) {
    unsigned sup = n_support, cands = (unsigned)cnt;
    for (int s = 32; s > 0; s >>= 1) {
      sup += __shfl_xor((int)sup, s);
      cands += __shfl_xor((int)cands, s);
    }
    if ((threadIdx.x & 63) == 0) {
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_CANDIDATES], (unsigned long long)cands);
      atomicAdd(&A.stats[ENTMAX_STAT_FWD_SUPPORT], (unsigned long long)sup);
    }
  }
}

}  // namespace entmax
