// Backward kernels for rows with a small support (the regime of the paper's
// ASEntmax workloads: a few non-zero probabilities per row).  With
// x_ij = [(alpha-1) s_ij - tau_i]_+, r = 1/(alpha-1), on the support only:
//   p = x^r, g = x^(r-1), dP_ij = <dO_i, v_j>, mu_i = sum g dP / sum g,
//   dS_ij = g (dP - mu_i), dQ_i = c_i sum_j dS_ij k_j, dscale_i = sum_j dS_ij z_ij,
//   dV_j = sum_i p_ij dO_i,  dK_j = sum_i c_i dS_ij q_i.
// The Jacobian of eq. (entmax) vanishes off the support, so the whole backward
// is a sparse problem once the support is known:
//   bwd_lists_kernel   one Q K^T sweep on the matrix cores at the saved tau lists
//                      each row's support (key index + raw score) -- not launched when the forward
//                      handed its own support lists over (`saved` buffer);
//   key_offsets_kernel one workgroup per head: how many listed entries name each key, prefix sums
//                      of these counts (every key gets a segment that can hold all its entries), and
//                      the list of keys with long segments;
//   bwd_rows_kernel    everything row-wise (mu, dscale, dQ) from the lists, by
//                      gathering the few K and V rows (one lane pair per row).
//                      Each entry's (query, p, c dS) goes straight into its key's segment, at the
//                      place a returning atomic on the key's cursor hands out;
//   bwd_keys_kernel    eight lanes per key (one wave per key for long segments): dV_j and dK_j as
//                      sums over the key's entries, in query order.
// A 128-row query block in which some half row holds more than kBwdCap support entries is flagged and
// left to the tiled kernels of bwd.hip.h, which then run on the flagged blocks of that head only: dQ and the
// row scalars of a block come from one path or the other, and dK, dV of such a head are the tiled kernels'
// sums over the flagged blocks plus the key kernel's sums over the listed entries of the others.
#pragma once
#include "bwd.hip.h"
#include "fwd_sparse.hip.h"

namespace entmax {

constexpr int kHeadMixed = 1, kHeadTiled = 2;  // values of a head's flag, see BwdSparseArgs::head_flag
constexpr int kSortedKeyEntries = 8;        // a key with at most this many entries is summed by one lane pair

struct BwdSparseArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* V;
  const void* dO;
  const float* tau;
  void* dQ;
  void* dK;
  void* dV;
  float* dscale;       // [B*H*Nq]
  // The rows' support lists, their lengths and the block flags: written by bwd_lists_kernel into the workspace,
  // or the forward's (in the `saved` buffer, read only here).
  uint2* list;         // (key index, raw dot product bits) of the listed entries.  Workspace lists:
                       // [B*H*nqb*4 row groups][kBwdCap][64 lanes], see list_entry().  The forward's (packed = 1): the
                       // pool of the `saved` buffer, a half row's entries next to each other.
  int* lcnt;           // [B*H*Nq][2] entries per half row; packed: (place of the first entry in the pool) << 5 | entries
  int packed;
  long long pool_cap;  // packed: entries the pool holds (places beyond it are never followed)
  int* block_flag;     // [B*H*nqb] 1 when the block cannot take the list path (a list too long, or no lists)
  void* cells;         // sweep scratch: one CellBuf<kBwdCap> per workgroup of the list sweep's grid
  int* kcount;         // [B*H*Nk] listed entries per key = size of the key's segment (key_offsets_kernel)
  const int* precount; // NULL, or the same counts as the forward left them in the `saved` buffer
  int* kcursor;        // [B*H*Nk] entries placed so far; after bwd_rows_kernel: the key's entries with p > 0
  int* koffs;          // [B*H*Nk] exclusive prefix sums of kcount within the head: segment starts
  int* csc_i;          // [B*H][Nq*2*kBwdCap] query row of each entry, key-major
  float2* csc_pw;      // same order: (p, c dS)
  int* head_flag;      // [2*B*H], written by key_offsets_kernel: entry bh: 0 no block of the head needs the tiled
                       // kernels, 1 its flagged blocks do (kHeadMixed), 2 the whole head does (kHeadTiled);
                       // entry B*H + bh: number of the head's keys on the long-segment list
  int* long_keys;      // [B*H][Nk] per head: its keys whose segment holds more than kSortedKeyEntries entries
  float* dbeta;        // per-head scale gradients, reduced by extra workgroups of the keys launch
  float* dgamma;       //   (scale_heads = 0: not here)
  int scale_heads;     // H for per-head scale parameters, else 0
  unsigned long long* stats;
  int nqb;
  TransposeRide ride;  // operand copies for the tiled kernels, as extra workgroups of the row launch
};

// ------------------------------------------------------------------ rows

// One Q K^T sweep at the saved threshold: the lists it writes are the rows' exact supports.
template <typename T, int D, int AM, bool BIAS>
__device__ __forceinline__ void bwd_lists_block(const BwdSparseArgs& A, int bh_, int blk_, char* smem) {
  using C = QCtx<T, D, ListCfg<T, D>::kTile, BIAS>;
  constexpr int TB = C::kTileBytes;
  const Geom& g = A.g;
  int* ovf = reinterpret_cast<int*>(smem + 2 * TB);
  C q;
  q.init(g, A.Q, bh_, blk_);
  q.init_window(g);
  const long long row_idx = (long long)q.bh * g.Nq + (q.valid ? q.i : 0);
  const float tau = q.valid ? A.tau[row_idx] : 0.f;
  const bool live = q.valid && q.lim > 0;
  uint2* mylist = A.list + list_entry<kBwdCap>(q.bh, A.nqb, q.qb, q.wave, q.lane);
  int cnt = 0;
  unsigned n_qk = 0, n_cand_tiles = 0;
  bool fits = true;
  if (q.block_lim > 0) fits = collect_sweep<C, T, D, kBwdCap, ListCfg<T, D>::kLdsCells>(q, g, A.K, smem, ovf, smem + 2 * TB + 16, live, tau, A.cells, mylist, cnt, n_qk, n_cand_tiles);
  if (q.tid == 0) A.block_flag[q.bh * A.nqb + q.qb] = fits ? 0 : 1;
  if (fits && q.valid) A.lcnt[row_idx * 2 + q.hh] = cnt;
  if (A.stats && q.lane == 0) {
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_TILES_VISIBLE], (unsigned long long)n_qk);
    atomicAdd(&A.stats[ENTMAX_STAT_BWD_LIST_QK], (unsigned long long)n_qk);
  }
}

template <typename T, int D, int AM, bool BIAS>
__global__ __launch_bounds__(kThreads, (ListCfg<T, D>::kOcc)) void bwd_lists_kernel(BwdSparseArgs A) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const PairItem it = pair_item(A.nqb);
  for (int part = 0; part < 2; ++part) {
    const int blk = part ? it.second : it.first;
    if (blk < 0) break;
    if (part) __syncthreads();
    bwd_lists_block<T, D, AM, BIAS>(A, it.bh, blk, smem);
  }
}

// Everything row-wise from the lists: D / 32 lanes per row, each with 32 of the features (a lane pair per row at
// D = 64; at D = 128 two lanes per list half, which both read that half's entries -- with 64 features per lane the
// kernel needed 388 registers and ran one wave per SIMD: 234 against 174 us at B 2, H 16, n 8192).
// Measured and not kept: 16 features per lane (twice the waves at 146 registers: same time at both head
// dimensions), eight consecutive lanes per row so that a gathered row is one load instruction (D = 64: 78 -> 82 us),
// all gathers of a short row requested before the first is used (-> 101 us), a head's keys on its rows' XCD in the
// key kernel (no change).
template <int D>
struct RowsCfg {
  static constexpr int kFH = D / 64;  // lanes per list half
};
template <typename T, int D, int AM>
__global__ __launch_bounds__(kThreads, 2) void bwd_rows_kernel(BwdSparseArgs A) {
  const Geom& g = A.g;
  constexpr int FH = RowsCfg<D>::kFH;
  if ((int)blockIdx.x >= g.B * g.H * A.nqb * FH) {  // riders behind the row workgroups
    transpose_ride<T, D>(A.ride, (int)blockIdx.x - g.B * g.H * A.nqb * FH);
    return;
  }
  RowLane rl;
  rl.init<FH>(g, A.nqb);
  constexpr int DH = 32;  // features per lane
  const int feat0 = (rl.hh * FH + rl.f) * DH;  // the lane's first feature
  const bool owner_lane = rl.f == 0;           // the lane of its list half that places the entries and writes the row scalars
  const float r = 1.0f / (g.alpha - 1.0f);
  const long long row_idx = (long long)rl.bh * g.Nq + (rl.valid ? rl.i : 0);
  const int lim = rl.valid ? row_limit(g, rl.i) : 0;
  const bool live = rl.valid && lim > 0;
  const float scale = rl.valid ? row_scale(g, rl.b, rl.h, rl.i, lim, nullptr, nullptr, nullptr) : 0.f;
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const float c = scale * inv_sqrt_d;
  const float a = (g.alpha - 1.0f) * fabsf(c);  // same arithmetic as the sweep that made the lists
  const float sgn = (c < 0.f) ? -1.f : 1.f;
  // distance bias outside the scale: dscale_i = sum_j dS_ij z_ij needs the listed scores without their bias term
  const float w_out = (g.slopes && g.bias_mode == 1) ? bias_w<D>(g, rl.h, c, a) : 0.f;
  const int pos = rl.i + (g.Nk - g.Nq);
  // every load that does not depend on another is issued before the first wait (the head's flags included)
  const int head_dense = (A.head_flag[rl.bh] == kHeadTiled || A.block_flag[rl.bh * A.nqb + rl.qb] != 0) ? 1 : 0;
  const float tau_raw = A.tau[row_idx];
  const int cnt_raw = A.lcnt[row_idx * 2 + rl.hh];
  const float tau = live ? tau_raw : 0.f;
  const long long q_base = (long long)rl.b * g.q_sb + (long long)rl.h * g.q_sh;
  const long long kv_base = (long long)rl.b * g.kv_sb + (long long)rl.h * g.kv_sh;
  // where this half row's entries are, and how far apart
  const uint2* rdlist;
  int cnt_list, lstride;
  if (A.packed) {
    long long off = (long long)((unsigned)cnt_raw >> 5);
    cnt_list = cnt_raw & 31;
    if (off + cnt_list > A.pool_cap) {  // not a place the forward wrote (a flagged block's words hold anything)
      off = 0;
      cnt_list = 0;
    }
    rdlist = A.list + off;
    lstride = 1;
  } else {
    rdlist = A.list + list_entry<kBwdCap>(rl.bh, A.nqb, rl.qb, rl.w32, rl.hh * 32 + rl.li);
    cnt_list = cnt_raw;
    lstride = kListStride;
  }
  const int cnt = live ? min(cnt_list, kBwdCap) : 0;
  const T* Kbh = reinterpret_cast<const T*>(A.K) + kv_base;
  const T* Vbh = reinterpret_cast<const T*>(A.V) + kv_base;

  // the row's dO, this lane's half of the features, widened to fp32
  float dov[DH];
  if (rl.valid) {
    load_row_f32<T>(reinterpret_cast<const T*>(A.dO) + q_base + (long long)rl.i * g.q_sn + feat0, DH, dov);
  } else {
#pragma unroll
    for (int t = 0; t < DH; ++t) dov[t] = 0.f;
  }
  unsigned n_entries = 0;
  // the first entries are requested whatever the list length is (the slots exist whatever they hold; the
  // pool ends on kSavedPoolPad spare entries)
  constexpr int kEarly = 4;
  uint2 early[kEarly];
#pragma unroll
  for (int e = 0; e < kEarly; ++e) early[e] = rdlist[e * lstride];
  if (head_dense != 0) {  // the tiled kernels own this block
    // The forward numbered this block's entries among their keys' entries before it knew that the block would
    // not take the list path: in a head whose other blocks do, those places must not stay undefined.  They get
    // records that add nothing.
    if (A.packed && owner_lane && A.block_flag[rl.bh * A.nqb + rl.qb] == kBlockListsUnused && A.head_flag[rl.bh] == kHeadMixed) {
      const long long cap = (long long)g.Nq * 2 * kBwdCap;
      for (int e = 0; e < cnt; ++e) {
        const uint2 en = rdlist[e];
        const unsigned key = min(en.x & ((1u << kSavedKeyBits) - 1u), (unsigned)(g.Nk - 1)), rank = en.x >> kSavedKeyBits;
        const long long kidx = (long long)rl.bh * g.Nk + key;
        const int slot = A.koffs[kidx] + (rank < kSavedRankMost ? (int)rank : (int)kSavedRankMost + atomicAdd(&A.kcursor[kidx], 1));
        if (slot >= 0 && slot < cap) {
          A.csc_i[rl.bh * cap + slot] = min(rl.i, g.Nq - 1);
          A.csc_pw[rl.bh * cap + slot] = make_float2(0.f, 0.f);
        }
      }
    }
    return;
  }

  auto finish = [&](auto ne_tag) {
    constexpr int NE = decltype(ne_tag)::value;
    unsigned jv[NE], rkv[NE];
    float dv[NE];  // raw dot products (sign-folded), -inf for empty slots
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      uint2 en = make_uint2(0u, 0u);
      if (e < kEarly)
        en = early[e];
      else if (e < cnt)
        en = rdlist[e * lstride];
      // the forward's entries carry their arrival number among their key's entries above the key index
      rkv[e] = A.packed ? en.x >> kSavedKeyBits : kSavedRankMost;
      if (A.packed) en.x &= (1u << kSavedKeyBits) - 1u;
      // (a key index is never followed outside the tensors, whatever a stale or foreign `saved` buffer holds)
      jv[e] = (e < cnt) ? min(en.x, (unsigned)(g.Nk - 1)) : 0u;
      dv[e] = (e < cnt) ? __uint_as_float(en.y) : -kInf;
    }
    // One gather pass over the entries of the row (both halves): dP = <dO, v_j> and, because dQ and dscale
    // are linear in mu,
    //   dQ_i = c (sum_j g dP k_j - mu sum_j g k_j),   dscale_i = sum_j g dP d_j - mu sum_j g d_j,
    // the K rows are gathered in the same pass as the V rows: one memory round trip for both.
    float dpv[NE];  // dP of the lane's own entries
    float Z = 0.f, N = 0.f, sd1 = 0.f, sd0 = 0.f;
    float qa[DH], qb[DH];  // this lane's half of sum g dP k and of sum g k
#pragma unroll
    for (int t = 0; t < DH; ++t) qa[t] = qb[t] = 0.f;
    int slotv[NE];  // place in the key-major arrays of the lane's own entries; -1: not part of the support
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      slotv[e] = -1;
      dpv[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      unsigned pj = (unsigned)__shfl_xor((int)jv[e], 32);
      float pd = __shfl_xor(dv[e], 32);
#pragma unroll
      for (int src = 0; src < 2; ++src) {
        // both lanes of the pair look at the same entry: entry e of the lane whose half index is src
        unsigned j = (rl.hh == src) ? jv[e] : pj;
        float d = (rl.hh == src) ? dv[e] : pd;
        float x = (d > -kInf) ? fmaxf(fmaf(d, a, -tau), 0.f) : 0.f;
        if (__ballot(x > 0.f) == 0ull) continue;
        float part = 0.f;
        RawRow<T, DH> kk;
        if (x > 0.f) {
          RawRow<T, DH> vv;
          vv.load(Vbh + (long long)j * g.kv_sn + feat0);
          kk.load(Kbh + (long long)j * g.kv_sn + feat0);
          // the entry's owner takes its arrival number among the key's entries: its place in the key's segment
          if (rl.hh == src && owner_lane) {
            const long long kidx = (long long)rl.bh * g.Nk + j;
            // its arrival number: the forward's, or (lists made here, and a key's entries beyond the numbers
            // the forward can write) from the key's cursor
            slotv[e] = A.koffs[kidx] +
                       (rkv[e] < kSavedRankMost ? (int)rkv[e] : (A.packed ? (int)kSavedRankMost : 0) + atomicAdd(&A.kcursor[kidx], 1));
            ++n_entries;
          }
#pragma unroll
          for (int t = 0; t < DH; ++t) part = fmaf(dov[t], vv.get(t), part);
        }
        if (FH == 2) part += __shfl_xor(part, 16);
        float dp = part + __shfl_xor(part, 32);
        if (x > 0.f) {
          float gg = pow_rm1<AM>(x, r);
          float gdp = gg * dp;
          Z += gg;
          N += gdp;
          const float dz = (w_out != 0.f) ? fmaf(-w_out, (float)bias_dist(pos, (int)j), d) : d;
          sd1 = fmaf(gdp, dz, sd1);
          sd0 = fmaf(gg, dz, sd0);
#pragma unroll
          for (int t = 0; t < DH; ++t) {
            const float kt = kk.get(t);
            qa[t] = fmaf(gdp, kt, qa[t]);
            qb[t] = fmaf(gg, kt, qb[t]);
          }
          if (rl.hh == src) dpv[e] = dp;
        }
      }
    }
    const float mu = (Z > 0.f) ? N / Z : 0.f;
    float dq[DH];
#pragma unroll
    for (int t = 0; t < DH; ++t) dq[t] = c * fmaf(-mu, qb[t], qa[t]);
    const float dsc = fmaf(-mu, sd0, sd1);
    // the per-entry records (query, p, c dS) go straight to their place in the key-major arrays
    // (a listed key whose probability rounds to zero here has no place and is dropped)
    const long long cap = (long long)g.Nq * 2 * kBwdCap;  // entries a head can hold
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      if (slotv[e] >= 0 && slotv[e] < cap) {  // (key_offsets_kernel flags heads whose segments would not fit)
        float x = fmaxf(fmaf(dv[e], a, -tau), 0.f);
        float ds = pow_rm1<AM>(x, r) * (dpv[e] - mu);
        A.csc_i[rl.bh * cap + slotv[e]] = rl.i;
        A.csc_pw[rl.bh * cap + slotv[e]] = make_float2(pow_r<AM>(x, r), c * ds);
      }
    }
    if (rl.valid) {
      store_row<T>(reinterpret_cast<T*>(A.dQ) + q_base + (long long)rl.i * g.q_sn + feat0, DH, dq);
      // the scores were formed with q negated when scale_i < 0: undo the sign for z_ij
      if (rl.hh == 0 && owner_lane) A.dscale[row_idx] = sgn * dsc * inv_sqrt_d;
    }
  };
  if (__ballot(cnt > 4) == 0ull)
    finish(std::integral_constant<int, 4>());
  else
    finish(std::integral_constant<int, kBwdCap>());

  if (A.stats) {
    unsigned ent = n_entries;
    for (int s = 32; s > 0; s >>= 1) ent += __shfl_xor((int)ent, s);
    if ((threadIdx.x & 63) == 0) atomicAdd(&A.stats[ENTMAX_STAT_BWD_SUPPORT], (unsigned long long)ent);
  }
}

// ------------------------------------------------------------ key-major order

// One workgroup per head, before the row kernel.  Counts, per key, the list entries that name it (the
// entries with p > 0, and possibly a few whose p rounds to zero), and gives every key a segment of that size in the key-major
// arrays: koffs = exclusive prefix sums of the counts.  The row kernel then places an entry at
// koffs[key] + (arrival number from the key's cursor) -- no reordering pass.  Also: the head's flag (OR of
// its block flags), zeroed cursors, and the list of keys whose segment exceeds kSortedKeyEntries.
// counters: LDS when a head's keys fit (use_lds), else the kcount array itself.
constexpr int kOffsThreads = 1024;

static __global__ __launch_bounds__(kOffsThreads) void key_offsets_kernel(BwdSparseArgs A, int use_lds) {
  extern __shared__ int offs_lds[];
  int* part = offs_lds;                   // entries in the thread's range of keys
  int* partl = offs_lds + kOffsThreads;   // long segments in it
  const Geom& g = A.g;
  const int bh = blockIdx.x, tid = threadIdx.x, Nk = g.Nk;
  {
    int flagged = 0, unflagged = 0;
    for (int k = tid; k < A.nqb; k += kOffsThreads) {
      if (A.block_flag[bh * A.nqb + k] != 0)
        ++flagged;
      else
        ++unflagged;
    }
    const int any = __syncthreads_or(flagged);
    const int all = __syncthreads_and(unflagged == 0);
    const int nflag = !any ? 0 : (all ? kHeadTiled : kHeadMixed);
    if (tid == 0) {
      A.head_flag[bh] = nflag;          // 0, kHeadMixed, or kHeadTiled when every block is flagged
      A.head_flag[g.B * g.H + bh] = 0;  // no long keys yet
    }
    if (nflag == kHeadTiled) return;  // the tiled kernels own this head
  }
  int* gcount = A.kcount + (long long)bh * Nk;
  const int* cnt = A.precount ? A.precount + (long long)bh * Nk : (use_lds ? offs_lds + 2 * kOffsThreads : gcount);
  int* wcnt = use_lds ? offs_lds + 2 * kOffsThreads : gcount;  // counted here unless the forward did
  if (!A.precount) {
  for (int j = tid; j < Nk; j += kOffsThreads) wcnt[j] = 0;
  __syncthreads();
  // a lane of a row group per step: the 64 lanes of a slot are one 512-byte run of the list
  for (int hr = tid; hr < A.nqb * kThreads; hr += kOffsThreads) {
    const int qb = hr / kThreads, wave = (hr % kThreads) >> 6, lane = hr & 63;
    const int i = qb * kBlockRows + wave * 32 + (lane & 31), hh = lane >> 5;
    if (i >= g.Nq || A.block_flag[bh * A.nqb + qb] != 0) continue;  // (a flagged block has no lists)
    const int n = min(A.lcnt[((long long)bh * g.Nq + i) * 2 + hh], kBwdCap);
    const uint2* src = A.list + list_entry<kBwdCap>(bh, A.nqb, qb, wave, lane);
    for (int e = 0; e < n; ++e) {
      const unsigned key = src[e * kListStride].x;
      if (key < (unsigned)Nk) atomicAdd(&wcnt[key], 1);
    }
  }
  __syncthreads();
  }
  const int per = (Nk + kOffsThreads - 1) / kOffsThreads;
  const int beg = tid * per, end = min(Nk, beg + per);
  int s = 0, nl = 0;
  for (int j = beg; j < end; ++j) {
    const int cj = cnt[j];
    s += cj;
    nl += cj > kSortedKeyEntries ? 1 : 0;
  }
  part[tid] = s;
  partl[tid] = nl;
  __syncthreads();
  // Hillis-Steele inclusive scans over the partial sums
  for (int off = 1; off < kOffsThreads; off <<= 1) {
    int v = (tid >= off) ? part[tid - off] : 0;
    int vl = (tid >= off) ? partl[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    partl[tid] += vl;
    __syncthreads();
  }
  // The key-major arrays hold kBwdCap entries per half row and head, and every list holds at most that many:
  // the segments fit.  (Checked all the same: a head that would not fit is left to the tiled kernels.)
  if (part[kOffsThreads - 1] > g.Nq * 2 * kBwdCap) {
    if (tid == 0) A.head_flag[bh] = kHeadTiled;
    return;
  }
  if (tid == kOffsThreads - 1) A.head_flag[g.B * g.H + bh] = partl[tid];
  int run = part[tid] - s;
  long long lpos = (long long)bh * Nk + partl[tid] - nl;
  for (int j = beg; j < end; ++j) {
    const int cj = cnt[j];
    A.koffs[(long long)bh * Nk + j] = run;
    A.kcursor[(long long)bh * Nk + j] = 0;
    if (cnt != gcount) gcount[j] = cj;
    run += cj;
    if (cj > kSortedKeyEntries) A.long_keys[lpos++] = bh * Nk + j;
  }
}

// dV_j = sum_i p_ij dO_i,  dK_j = sum_i (c_i dS_ij) q_i  over the key's entries.
// Eight lanes per key, each lane an eighth of the features: a gathered dO or Q row is then one
// fully used cache line per load instruction and key, instead of four instructions that each touch a
// quarter of it.  A key's entries sit in arrival order; lane k of the eight takes entry k, the entries
// are ranked by query row inside the group and summed in that order, which makes the result independent
// of the arrival order.  Keys whose segment holds more than kSortedKeyEntries (= 8) entries are served
// by the first kLongKeyBlocks workgroups of the same launch (bwd_long_keys_part), which run alongside
// the others; scale_heads more workgroups reduce dscale to d beta, d gamma.
constexpr int kLongKeyBlocks = 1024;
constexpr int kKeysPerBlock = kThreads / kSortedKeyEntries;  // 32

template <typename T, int D>
__device__ __forceinline__ void bwd_long_keys_part(const BwdSparseArgs& A, int vblock, int vgrid);

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void bwd_keys_kernel(BwdSparseArgs A) {
  static_assert(kSortedKeyEntries == 8, "one entry per lane of a group of eight");
  constexpr int DL = D / 8;  // features per lane
  const Geom& g = A.g;
  if (blockIdx.x < kLongKeyBlocks) {
    bwd_long_keys_part<T, D>(A, blockIdx.x, kLongKeyBlocks);
    return;
  }
  if (blockIdx.x < kLongKeyBlocks + A.scale_heads) {
    // dscale is complete by now (row kernel, tiled dQ kernel): its reduction to d beta, d gamma rides along
    __shared__ float sb_[kThreads], sg_[kThreads];
    scale_grad_head_part<kThreads>(g, A.dscale, A.dbeta, A.dgamma, blockIdx.x - kLongKeyBlocks, sb_, sg_);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, k = tid & 7, group0 = lane & ~7;
  const long long nkeys = (long long)g.B * g.H * g.Nk;
  const long long key = (long long)(blockIdx.x - kLongKeyBlocks - A.scale_heads) * kKeysPerBlock + (tid >> 3);
  bool on = key < nkeys;
  const int bh = on ? (int)(key / g.Nk) : 0;
  const int j = on ? (int)(key % g.Nk) : 0;
  const int hflag = on ? A.head_flag[bh] : 0;
  on = on && hflag != kHeadTiled;
  const int b = bh / g.H, h = bh % g.H;
  const int seg = on ? A.kcount[key] : 0;            // size of the key's segment
  // entries with p > 0 placed in it: with the forward's numbers all of them, but for what the cursor counted beyond
  int n = on ? (A.packed ? min(seg, (int)kSavedRankMost + A.kcursor[key]) : min(A.kcursor[key], seg)) : 0;
  if (seg > kSortedKeyEntries) {  // on the long-key list
    on = false;
    n = 0;
  }
  const long long base = (long long)bh * g.Nq * 2 * kBwdCap + (on ? A.koffs[key] : 0);
  const long long q_base = (long long)b * g.q_sb + (long long)h * g.q_sh + k * DL;
  const T* dObh = reinterpret_cast<const T*>(A.dO) + q_base;
  const T* Qbh = reinterpret_cast<const T*>(A.Q) + q_base;
  // entry k of the key, then its rank by query row within the group (rows of a key are distinct;
  // empty slots rank last, among themselves by lane)
  const int ci = (k < n) ? A.csc_i[base + k] : 0x7fffffff;
  const float2 cpw = (k < n) ? A.csc_pw[base + k] : make_float2(0.f, 0.f);
  int rank = 0;
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const int cm = __shfl(ci, group0 + m);
    rank += (cm < ci || (cm == ci && m < k)) ? 1 : 0;
  }
  // lane t of the group then holds the entry with the t-th smallest row
  const int dst = (group0 + rank) << 2;
  const int si = __builtin_amdgcn_ds_permute(dst, ci);
  const float sp = __int_as_float(__builtin_amdgcn_ds_permute(dst, __float_as_int(cpw.x)));
  const float sw = __int_as_float(__builtin_amdgcn_ds_permute(dst, __float_as_int(cpw.y)));
  float dv[DL], dk[DL];
#pragma unroll
  for (int t = 0; t < DL; ++t) dv[t] = dk[t] = 0.f;
  // kB entries at a time: their rows are all requested before the first is used (one memory round trip for most
  // keys instead of one per entry); the sums still run in query order.  Four where a lane's share of a row is one
  // 16-byte word (B 4, H 12, n 4096, D 64: 47 -> 38 us); with 32 bytes per lane the registers of four cost more
  // than the round trips (B 2, H 16, n 8192, D 128: 83 -> 93 us), so one.
  constexpr int kB = DL * (int)sizeof(T) <= 16 ? 4 : 1;
#pragma unroll
  for (int t0 = 0; t0 < 8; t0 += kB) {
    if (__ballot(t0 < n) == 0ull) break;
    RawRow<T, DL> rd[kB], rq[kB];
    float pe[kB], we[kB];
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      const int t = t0 + u;
      int i = __shfl(si, group0 + t);
      pe[u] = __shfl(sp, group0 + t);
      we[u] = __shfl(sw, group0 + t);
      if (t < n) {
        i = min(max(i, 0), g.Nq - 1);  // a valid row by construction; never index outside the tensor
        rd[u].load(dObh + (long long)i * g.q_sn);
        rq[u].load(Qbh + (long long)i * g.q_sn);
      }
    }
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      if (t0 + u < n) {
#pragma unroll
        for (int f = 0; f < DL; ++f) {
          dv[f] = fmaf(pe[u], rd[u].get(f), dv[f]);
          dk[f] = fmaf(we[u], rq[u].get(f), dk[f]);
        }
      }
    }
  }
  if (on) {
    const long long o = (long long)b * g.kv_sb + (long long)h * g.kv_sh + (long long)j * g.kv_sn + k * DL;
    if (hflag == kHeadMixed) {  // the tiled kernels wrote the flagged blocks' share: add it
      float ev[DL], ek[DL];
      load_row_f32<T>(reinterpret_cast<const T*>(A.dV) + o, DL, ev);
      load_row_f32<T>(reinterpret_cast<const T*>(A.dK) + o, DL, ek);
#pragma unroll
      for (int t = 0; t < DL; ++t) {
        dv[t] += ev[t];
        dk[t] += ek[t];
      }
    }
    store_row<T>(reinterpret_cast<T*>(A.dV) + o, DL, dv);
    store_row<T>(reinterpret_cast<T*>(A.dK) + o, DL, dk);
  }
}

// Keys with more than kSortedKeyEntries entries: one wave per key, one (D = 64) or two (D = 128)
// features per lane, whole dO / Q rows per entry.  Within chunks of 64 entries the sum runs in
// query-row order (rank by comparison across the wave), so keys with up to 64 entries get an
// order-independent result; only longer segments depend on the arrival order of their chunks.
template <typename T, int D>
__device__ __forceinline__ void bwd_long_keys_part(const BwdSparseArgs& A, int vblock, int vgrid) {
  constexpr int PER = D / 64;
  const Geom& g = A.g;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  // Persistent workgroups: the waves share out the per-head lists key_offsets_kernel made.  The heads' list
  // lengths are fetched 64 at a time (one load per lane); their running sums number the long keys of these 64
  // heads consecutively, and the waves take those numbers in turn.
  const int nheads = g.B * g.H;
  for (int h0 = 0; h0 < nheads; h0 += 64) {
  const int my_count = (h0 + lane < nheads) ? A.head_flag[nheads + h0 + lane] : 0;
  int my_end = my_count;  // inclusive running sum over the lanes
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) {
    const int up = __shfl_up(my_end, sft);
    if (lane >= sft) my_end += up;
  }
  const int ntotal = __builtin_amdgcn_readlane(my_end, 63);
  for (int gidx = vblock * kWaves + wave; gidx < ntotal; gidx += vgrid * kWaves) {
  {
  // the head whose range holds gidx: the first lane whose running sum exceeds it
  const int hu = __builtin_amdgcn_readfirstlane(__builtin_popcountll(__ballot(my_end <= gidx)));
  const int lbh = h0 + hu;
  const int idx = gidx - (__builtin_amdgcn_readlane(my_end, hu) - __builtin_amdgcn_readlane(my_count, hu));
  const long long key = __builtin_amdgcn_readfirstlane(A.long_keys[(long long)lbh * g.Nk + idx]);
  const int n = __builtin_amdgcn_readfirstlane(
      A.packed ? min(A.kcount[key], (int)kSavedRankMost + A.kcursor[key]) : min(A.kcursor[key], A.kcount[key]));
  const int bh = (int)(key / g.Nk), j = (int)(key % g.Nk);
  const int b = bh / g.H, h = bh % g.H;
  const long long base = (long long)bh * g.Nq * 2 * kBwdCap + __builtin_amdgcn_readfirstlane(A.koffs[key]);
  const long long q_base = (long long)b * g.q_sb + (long long)h * g.q_sh;
  float av[PER], ak[PER];
#pragma unroll
  for (int t = 0; t < PER; ++t) av[t] = ak[t] = 0.f;
  for (int e0 = 0; e0 < n; e0 += 64) {
    const int m = min(64, n - e0);
    int ci = (lane < m) ? A.csc_i[base + e0 + lane] : 0x7fffffff;
    float2 cpw = (lane < m) ? A.csc_pw[base + e0 + lane] : make_float2(0.f, 0.f);
    int rank = 0;
    for (int k = 0; k < m; ++k) rank += (__shfl(ci, k) < ci) ? 1 : 0;
    // push every entry to the lane of its rank: lane k then holds the k-th smallest row
    int si = __builtin_amdgcn_ds_permute(rank << 2, ci);
    float sp = __int_as_float(__builtin_amdgcn_ds_permute(rank << 2, __float_as_int(cpw.x)));
    float sw = __int_as_float(__builtin_amdgcn_ds_permute(rank << 2, __float_as_int(cpw.y)));
    // rows, weights and addresses are wave-uniform (readlane): batches of 8 entries keep 16 row
    // loads in flight
    for (int k0 = 0; k0 < m; k0 += 8) {
      float dov[8][PER], qv[8][PER], pp[8], ww[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = min(k0 + u, m - 1);
        const int i = min(max(__builtin_amdgcn_readlane(si, k), 0), g.Nq - 1);
        pp[u] = (k0 + u < m) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sp), k)) : 0.f;
        ww[u] = (k0 + u < m) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sw), k)) : 0.f;
        const T* dorow = reinterpret_cast<const T*>(A.dO) + q_base + (long long)i * g.q_sn;
        const T* qrow = reinterpret_cast<const T*>(A.Q) + q_base + (long long)i * g.q_sn;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
          if constexpr (sizeof(T) == 2) {
            dov[u][t] = __uint_as_float((unsigned)reinterpret_cast<const unsigned short*>(dorow)[lane + 64 * t] << 16);
            qv[u][t] = __uint_as_float((unsigned)reinterpret_cast<const unsigned short*>(qrow)[lane + 64 * t] << 16);
          } else {
            dov[u][t] = reinterpret_cast<const float*>(dorow)[lane + 64 * t];
            qv[u][t] = reinterpret_cast<const float*>(qrow)[lane + 64 * t];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
#pragma unroll
        for (int t = 0; t < PER; ++t) {
          av[t] = fmaf(pp[u], dov[u][t], av[t]);
          ak[t] = fmaf(ww[u], qv[u][t], ak[t]);
        }
      }
    }
  }
  const long long o = (long long)b * g.kv_sb + (long long)h * g.kv_sh + (long long)j * g.kv_sn;
  const bool mixed = __builtin_amdgcn_readfirstlane(A.head_flag[bh]) == kHeadMixed;
#pragma unroll
  for (int t = 0; t < PER; ++t) {
    if (mixed) {  // the tiled kernels wrote the flagged blocks' share: add it
      av[t] += Elem<T>::load_one(A.dV, o + lane + 64 * t);
      ak[t] += Elem<T>::load_one(A.dK, o + lane + 64 * t);
    }
    Elem<T>::store(A.dV, o + lane + 64 * t, av[t]);
    Elem<T>::store(A.dK, o + lane + 64 * t, ak[t]);
  }
  }
  }
  }
}

}  // namespace entmax
