// Query-side machinery shared by the kernels whose workgroups own 128 query
// rows and stream key tiles (forward, backward tile-mask, backward dQ):
//   - QCtx: the per-lane row state.  Scores are produced TRANSPOSED,
//     S^T = K_tile Q^T, so that lane l of a wave owns query row (l%32) and holds
//     16 of the 32 keys of a tile; every per-row quantity (max, threshold,
//     partial sums of the threshold function) is then a per-lane scalar and the
//     inner loops need no cross-lane reduction.  The two lane halves are
//     combined once per sweep.
//   - sweep_tiles: double-buffered LDS pipeline over the key tiles a
//     workgroup needs, with register-staged prefetch of the next tile.
#pragma once
#include "common.hip.h"

#include <type_traits>

namespace entmax {

// BIAS: the kernel was built for the linear distance bias (Sec. 4.2; App. B, ALiBi definition): the score
// blocks start from w_i dist_ij instead of zero (the matrix instruction adds its products to it), and the
// key tiles beyond every row's window (App. B, ALiBi proposition) are not visited.
template <typename T, int D, int KT_ = Elem<T>::kTile, bool BIAS_ = false>
struct QCtx {
  static constexpr bool BIAS = BIAS_;
  static constexpr int KT = KT_;             // keys per LDS tile
  static constexpr int NSB = KT / 32;        // 32-key MFMA blocks per tile
  static constexpr int NC = D / 16;          // 16-wide k chunks of a Q.K product
  static constexpr int NM = D / 32;          // 32-wide feature blocks of an output
  static constexpr int kTileBytes = KT * D * (int)sizeof(T);
  using KTile = LdsTile<T, KT, D>;   // natural tile: rows = keys, cols = features
  using XtTile = LdsTile<T, D, KT>;  // transposed tile: rows = features, cols = (permuted) keys

  int tid, wave, lane, li, hh;
  int b, h, bh, qb;
  int q0;             // first query row of this wave
  int i;              // this lane's query row
  int lim;            // keys visible to row i are j < lim (0 for rows beyond Nq)
  bool valid;         // i < Nq
  int wave_lim_min;   // smallest / largest limit among the wave's rows
  int wave_lim_max;
  int block_lim;      // largest limit in the workgroup
  int ntiles;         // key tiles the workgroup sweeps
  float a;            // (alpha-1) |scale_i| / sqrt(D): y_ij = a * dot_ij are the entmax inputs times (alpha-1)
  float c;            // scale_i / sqrt(D), signed
  Frag<T> qf[NC];     // the row's query fragments (negated when scale_i < 0 so that a >= 0)
  FragOff<T> koff[NC];  // lane offsets of the K-tile fragments of row (l%32)
  // BIAS only
  float w;            // d'_ij = d_ij + w dist_ij (see bias_w()); 0: this row has no bias
  int pos;            // the row's position in the key sequence, i + (Nk - Nq): dist_ij = max(pos - j, 0)
  int wave_pos_min;   // smallest pos of the wave
  bool wave_bias;     // some row of the wave has w != 0
  int kt_first;       // first key tile some row of the workgroup / of the wave can have a non-zero probability in
  int kt_first_wave;

  // rg >= 0: every wave of the workgroup takes row group rg (rows 32 rg .. 32 rg + 31) of the block -- the waves
  // then share out the keys (split mode of the tiled forward); rg < 0: wave w takes row group w
  __device__ __forceinline__ void init(const Geom& g, const void* Q, int bh_, int qb_, int rg = -1) {
    tid = threadIdx.x;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps everything derived from it scalar
    lane = tid & 63;
    li = lane & 31;
    hh = lane >> 5;
    // blockIdx-derived values are uniform; readfirstlane pins them (and everything computed from
    // them) to SGPRs even where the compiler merges them with per-lane code
    auto uni = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    bh = uni(bh_);
    qb = uni(qb_);
    b = uni(bh / g.H);
    h = uni(bh % g.H);
    q0 = uni(qb * kBlockRows + (rg >= 0 ? rg : wave) * 32);
    i = q0 + li;
    valid = i < g.Nq;
    lim = valid ? row_limit(g, i) : 0;
    int last_blk = min(g.Nq, rg >= 0 ? q0 + 32 : (qb + 1) * kBlockRows) - 1;
    block_lim = uni(last_blk >= q0 || rg < 0 ? row_limit(g, last_blk) : 0);
    ntiles = uni((block_lim + KT - 1) / KT);
    wave_lim_min = uni(q0 < g.Nq ? row_limit(g, q0) : 0);
    wave_lim_max = uni(q0 < g.Nq ? row_limit(g, min(g.Nq, q0 + 32) - 1) : 0);
    float scale = valid ? row_scale(g, b, h, i, lim, nullptr, nullptr, nullptr) : 0.f;
    float inv_sqrt_d = 1.0f / sqrtf((float)D);
    c = scale * inv_sqrt_d;
    a = (g.alpha - 1.0f) * fabsf(c);
    const T* qrow = reinterpret_cast<const T*>(Q) + (long long)b * g.q_sb + (long long)h * g.q_sh + (long long)i * g.q_sn;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) {
      Frag<T> f = valid ? Elem<T>::load(qrow + 16 * cc + 8 * hh) : Elem<T>::zero();
      qf[cc] = (c < 0.f) ? Elem<T>::negate(f) : f;
      koff[cc] = FragOff<T>::template make<KTile>(li, 2 * cc + hh);
    }
    if constexpr (BIAS) {
      w = valid ? bias_w<D>(g, h, c, a) : 0.f;
      pos = i + (g.Nk - g.Nq);
      wave_pos_min = uni(q0 + (g.Nk - g.Nq));
      wave_bias = __ballot(w != 0.f) != 0ull;
      kt_first = kt_first_wave = 0;
    }
  }

  // Window of the distance bias (App. B, ALiBi proposition, with the proposition's logit range taken per row
  // from |d_ij| <= |q_i| max_j |k_j|): y_ij <= a (|q||k|max + w dist) for a penalising bias (w < 0), and the
  // threshold is at least y_max - 1 >= -a |q||k|max - 1 (the key at distance 0 is visible to every live row).
  // So a key with dist >= (2 |q||k|max + 1/a) / |w| has probability exactly zero and cannot be the row maximum.
  // Sets kt_first / kt_first_wave: the key tiles before them are skipped by every sweep.
  // All threads of the workgroup call this together (two barriers).
  __device__ __forceinline__ void init_window(const Geom& g) {
    if constexpr (BIAS) {
      __shared__ int wg_first;
      float s2 = 0.f;
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) s2 += Elem<T>::sumsq(qf[cc]);
      s2 += __shfl_xor(s2, 32);
      int first = 0x7fffffff;  // rows beyond Nq, rows without visible keys: no constraint
      if (valid && lim > 0) {
        first = 0;
        if (w < 0.f && a > 0.f) {
          const float reach = (2.0002f * sqrtf(s2) * g.knorm[bh] + 1.0f / a) / (-w);
          if (reach < 1.0e9f) first = max(0, pos - (int)reach - 2);
        }
      }
#pragma unroll
      for (int sft = 32; sft >= 1; sft >>= 1) first = min(first, __shfl_xor(first, sft));
      __syncthreads();
      if (tid == 0) wg_first = 0x7fffffff;
      __syncthreads();
      if (lane == 0) atomicMin(&wg_first, first);
      __syncthreads();
      kt_first_wave = __builtin_amdgcn_readfirstlane(min(first / KT, ntiles));
      kt_first = __builtin_amdgcn_readfirstlane(min(wg_first / KT, ntiles));
    }
  }
  // blocks (32 x 32) of this wave that are visible but lie before its first visited tile
  __device__ __forceinline__ unsigned window_skipped_blocks() const {
    if constexpr (BIAS) return (unsigned)min(kt_first_wave * NSB, (wave_lim_max + 31) >> 5);
    return 0u;
  }
  // the sweeps' tile predicates: workgroup-uniform and wave-uniform
  __device__ __forceinline__ bool tile_in_window(int kt) const {
    if constexpr (BIAS) return kt >= kt_first;
    return true;
  }
  __device__ __forceinline__ bool tile_in_wave_window(int kt) const {
    if constexpr (BIAS) return kt >= kt_first_wave;
    return true;
  }

  // accumulator start of the 32-key block at key j0: zero, or w dist for the lane's 16 (row, key) pairs
  __device__ __forceinline__ f32x16_t block_start(int j0) const {
    f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (BIAS) {
      if (wave_bias) bias_block(acc, j0);
    }
    return acc;
  }
  __device__ __forceinline__ void bias_block(f32x16_t& acc, int j0) const {
    const int rel = pos - j0;
    if (j0 + 31 <= wave_pos_min) {
      // every key of the block is at or before every row's position: dist = rel - key_of(e) > = 0
      const float base = w * (float)(rel - 4 * hh);
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = fmaf(-w, (float)(8 * (e >> 2) + (e & 3)), base);
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = w * (float)max(rel - key_of(e), 0);
    }
  }

  // S^T block: rows = 32 keys of sub-block sb of the K tile, cols = the wave's 32 queries.
  // acc[4g + r] of lane l is the raw dot product with key 8g + 4*(l/32) + r of the block.
  // kt: index of the tile in the key sequence (the distance bias needs the keys' positions)
  __device__ __forceinline__ f32x16_t scores(const char* ktile, int sb, int kt) const {
    f32x16_t acc = block_start(kt * KT + sb * 32);
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) acc = Elem<T>::mma(koff[cc].load(ktile, sb * 32 * KTile::kRowBytes), qf[cc], acc);
    return acc;
  }

  // All NSB blocks of a tile.  The K fragments of block sb+1 are requested before the products of
  // block sb are issued, so that LDS latency overlaps the matrix pipeline inside one wave.
  __device__ __forceinline__ void scores_all(const char* ktile, f32x16_t (&acc)[NSB], int kt) const {
    if constexpr (NC > 4) {  // two fragment sets would not fit the register budget
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) acc[sb] = scores(ktile, sb, kt);
      return;
    }
    Frag<T> kf[2][NC];
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) kf[0][cc] = koff[cc].load(ktile, 0);
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      if (sb + 1 < NSB) {
#pragma unroll
        for (int cc = 0; cc < NC; ++cc) kf[(sb + 1) & 1][cc] = koff[cc].load(ktile, (sb + 1) * 32 * KTile::kRowBytes);
      }
      f32x16_t a0 = block_start(kt * KT + sb * 32);
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) a0 = Elem<T>::mma(kf[sb & 1][cc], qf[cc], a0);
      acc[sb] = a0;
    }
    // keep that order through instruction scheduling: one LDS read behind each matrix instruction
    if constexpr (sizeof(T) == 2) {
      __builtin_amdgcn_sched_group_barrier(0x100, NC, 0);
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
#pragma unroll
        for (int cc = 0; cc < NC; ++cc) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (sb + 1 < NSB) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    }
  }

  // bits sb of the result: 32-key block sb of tile kt holds a key some row of this wave may see
  __device__ __forceinline__ uint32_t visible_bits(int kt) const {
    int nvis = (wave_lim_max - kt * KT + 31) >> 5;  // blocks of the tile that start below the wave's largest limit
    nvis = nvis < 0 ? 0 : (nvis > NSB ? NSB : nvis);
    return (1u << nvis) - 1u;
  }

  // key index (relative to the sub-block start) of accumulator element e of this lane
  __device__ __forceinline__ int key_of(int e) const { return 8 * (e >> 2) + 4 * hh + (e & 3); }
};

// Causal work grows linearly with the block index, so a workgroup takes block (n-1-p) and then
// block p of the same head: every workgroup of a launch carries the same amount of work, whatever
// order the hardware starts them in.  `second` is -1 when the pair is the middle block alone.
struct PairItem {
  int bh, first, second;
};
__device__ __forceinline__ PairItem pair_item(int nblk, int block = blockIdx.x, int total = gridDim.x) {
  const int npair = (nblk + 1) >> 1;
  const int item = xcd_remap(block, total);
  PairItem it;
  it.bh = __builtin_amdgcn_readfirstlane(item / npair);
  const int pp = __builtin_amdgcn_readfirstlane(item % npair);
  it.first = nblk - 1 - pp;
  it.second = (pp == it.first) ? -1 : pp;
  return it;
}

struct Slot {
  const char* base;     // tensor of this (batch, head): natural [N][row], transposed [D][npad]
  long long row_bytes;  // bytes between consecutive rows in global memory
};

// Streams the tiles kt with needed(kt) (a workgroup-uniform predicate) through a
// double-buffered LDS ring and calls body(kt, tiles) on each; `tiles` points at
// NSLOT consecutive tiles.  Bit s of TMASK says slot s is a transposed copy.
// All threads of the workgroup must call this together.
template <int S>
using Set = std::integral_constant<int, S>;  // a register set of the staging (see Stage), as a compile-time argument

struct NeverAbort {
  __device__ __forceinline__ bool operator()(int) const { return false; }
};

// abort(kt), evaluated by every thread at the start of the iteration that processes tile kt, may end
// the sweep after that tile.  It must be workgroup-uniform: it may only read state that was complete
// before the barrier that ended the previous iteration.
// DEPTH: tiles in flight from global memory while one is computed on (register sets per thread).  One is
// enough where several workgroups share a compute unit and hide each other's waits; a workgroup that has a
// compute unit (nearly) to itself needs two, or every tile costs a full memory round trip.  With DEPTH 2 the
// tile already on its way when abort(kt) turns true is still processed.
// STEP 2: the slots are two copies of one natural-layout tensor and step kt brings its tiles 2 kt and 2 kt + 1 (slot
// 0 and slot 1) between the same two barriers; ntiles still counts single tiles, needed(kt) and body(kt, tiles) count
// pairs, and the second tile of the last pair may lie beyond the sweep (it is then a copy of the last tile, which the
// body leaves alone).  For a workgroup whose waves share out the keys of a tile: twice the work per barrier.
template <typename C, typename T, int D, int NSLOT, int TMASK, int DEPTH = 1, int STEP = 1, class Needed, class Body,
          class Abort = NeverAbort>
__device__ __forceinline__ void sweep_tiles(char* smem, const Slot* slots, int ntiles, int Nk, int tid, Needed needed,
                                            Body body, Abort abort = Abort()) {
  static_assert(DEPTH == 1 || DEPTH == 2, "one or two tiles in flight");
  static_assert(STEP == 1 || (STEP == 2 && NSLOT == 2 && TMASK == 0), "pairs of natural tiles of one tensor");
  constexpr int KT = C::KT;
  const int last_tile = ntiles - 1;
  ntiles = (ntiles + STEP - 1) / STEP;  // from here on: steps
  constexpr int TB = C::kTileBytes;
  using Tile0 = typename std::conditional<(TMASK & 1) != 0, typename C::XtTile, typename C::KTile>::type;
  using Tile1 = typename std::conditional<(TMASK & 2) != 0, typename C::XtTile, typename C::KTile>::type;
  using Tile2 = typename std::conditional<(TMASK & 4) != 0, typename C::XtTile, typename C::KTile>::type;
  Stage<Tile0, kThreads, DEPTH> s0;
  Stage<Tile1, kThreads, DEPTH> s1;
  Stage<Tile2, kThreads, DEPTH> s2;
  s0.init(slots[0].row_bytes, tid);
  if constexpr (NSLOT > 1) s1.init(slots[1].row_bytes, tid);
  if constexpr (NSLOT > 2) s2.init(slots[2].row_bytes, tid);

  // tile kt of slot s starts at: natural copy -> row kt*KT; transposed copy -> column kt*KT
  auto tile_ptr = [&](int s, bool tr, int kt) {
    return slots[s].base + (tr ? (long long)kt * KT * (long long)sizeof(T) : (long long)kt * KT * slots[s].row_bytes);
  };
  auto fetch = [&](int step, auto set_) {
    constexpr int set = decltype(set_)::value;
    const int kt = STEP == 1 ? step : min(STEP * step, last_tile);
    const int rows_left = Nk - kt * KT;
    const bool full = rows_left >= KT;  // uniform
    if constexpr ((TMASK & 1) != 0) {
      s0.fetch_full(tile_ptr(0, true, kt), set);
    } else {
      if (full) s0.fetch_full(tile_ptr(0, false, kt), set);
      else s0.fetch(tile_ptr(0, false, kt), rows_left, slots[0].row_bytes, set);
    }
    if constexpr (NSLOT > 1) {
      if constexpr (STEP == 2) {
        const int kt1 = min(STEP * step + 1, last_tile);
        const int rows_left1 = Nk - kt1 * KT;
        if (rows_left1 >= KT) s1.fetch_full(tile_ptr(1, false, kt1), set);
        else s1.fetch(tile_ptr(1, false, kt1), rows_left1, slots[1].row_bytes, set);
      } else if constexpr ((TMASK & 2) != 0) {
        s1.fetch_full(tile_ptr(1, true, kt), set);
      } else {
        if (full) s1.fetch_full(tile_ptr(1, false, kt), set);
        else s1.fetch(tile_ptr(1, false, kt), rows_left, slots[1].row_bytes, set);
      }
    }
    if constexpr (NSLOT > 2) {
      if constexpr ((TMASK & 4) != 0) {
        s2.fetch_full(tile_ptr(2, true, kt), set);
      } else {
        if (full) s2.fetch_full(tile_ptr(2, false, kt), set);
        else s2.fetch(tile_ptr(2, false, kt), rows_left, slots[2].row_bytes, set);
      }
    }
  };
  auto commit = [&](char* buf, auto set_) {
    constexpr int set = decltype(set_)::value;
    s0.commit(buf, set);
    if constexpr (NSLOT > 1) s1.commit(buf + TB, set);
    if constexpr (NSLOT > 2) s2.commit(buf + 2 * TB, set);
  };
  auto next_needed = [&](int kt) {
    while (kt < ntiles && !needed(kt)) ++kt;
    return kt;
  };

  int kt = next_needed(0);
  if constexpr (DEPTH == 1) {
    if (kt < ntiles) {
      fetch(kt, Set<0>());
      commit(smem, Set<0>());
    }
    __syncthreads();
    int cur = 0;
    while (kt < ntiles) {
      int nxt = abort(kt) ? ntiles : next_needed(kt + 1);
      if (nxt < ntiles) fetch(nxt, Set<0>());
      body(kt, smem + cur * (NSLOT * TB));
      if (nxt < ntiles) commit(smem + (cur ^ 1) * (NSLOT * TB), Set<0>());
      __syncthreads();
      cur ^= 1;
      kt = nxt;
    }
  } else {
    // tile kt is in LDS, tile nxt on its way in one register set; the other set takes the tile after that
    // before the work on kt starts, and set `arrived` goes to LDS when that work is done
    int nxt = ntiles;
    if (kt < ntiles) {
      fetch(kt, Set<0>());
      nxt = next_needed(kt + 1);
      if (nxt < ntiles) fetch(nxt, Set<1>());
      commit(smem, Set<0>());
    }
    __syncthreads();
    int cur = 0;
    auto step = [&](auto arrived, auto free_set) {
      const int nxt2 = (nxt < ntiles && !abort(kt)) ? next_needed(nxt + 1) : ntiles;
      if (nxt2 < ntiles) fetch(nxt2, free_set);
      body(kt, smem + cur * (NSLOT * TB));
      if (nxt < ntiles) commit(smem + (cur ^ 1) * (NSLOT * TB), arrived);
      __syncthreads();
      cur ^= 1;
      kt = nxt;
      nxt = nxt2;
    };
    while (kt < ntiles) {
      step(Set<1>(), Set<0>());
      if (kt >= ntiles) break;
      step(Set<0>(), Set<1>());
    }
  }
}

// Per-wave bit sets over the 32-key blocks of a head, kept in LDS: bit jb of
// wave w says the block can hold a non-zero probability for some row of the wave.
struct WaveMask {
  uint32_t* words;  // [kWaves + 1][nwords]; row kWaves is the OR over the waves (see merge())
  int nwords;
  __device__ __forceinline__ void set(int w, int jb) { words[w * nwords + (jb >> 5)] |= (1u << (jb & 31)); }
  // the NSB (<= 4, aligned) consecutive bits of row w that belong to key tile kt, as a wave-uniform scalar
  template <int NSB>
  __device__ __forceinline__ uint32_t tile_bits(int w, int kt) const {
    int jb = kt * NSB;
    uint32_t word = __builtin_amdgcn_readfirstlane(words[w * nwords + (jb >> 5)]);
    return (word >> (jb & 31)) & ((1u << NSB) - 1u);
  }
  // all threads of the workgroup: row kWaves = OR of the wave rows; ends on a barrier
  __device__ __forceinline__ void merge(int tid) {
    __syncthreads();
    for (int w = tid; w < nwords; w += kThreads) {
      uint32_t v = 0u;
      for (int k = 0; k < kWaves; ++k) v |= words[k * nwords + w];
      words[kWaves * nwords + w] = v;
    }
    __syncthreads();
  }
};

}  // namespace entmax
