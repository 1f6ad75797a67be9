// Forward for a handful of query rows against a long key sequence (decoding:
// see decode_shape()).  The tiled and list kernels give a workgroup 128 query
// rows and one head's whole key sequence; with a few rows that is one
// workgroup per head streaming megabytes of K.  Here the keys are split
// instead, and the path is bound by reading K once from HBM:
//   decode_scores_kernel  grid (key chunks, heads): z_ij = (alpha-1) scale_i <q_i,k_j>/sqrt(d)
//                         (Sec. 2.1 scores, eq. (asentmax) scale) for the visible keys, fp32, to
//                         the workspace;
//   decode_solve_kernel   one workgroup per query row: row maximum, the keys that can be in the
//                         support (z > max - 1: everything else is zero already at the lowest
//                         possible threshold), the threshold of eq. (entmax) by Newton steps from
//                         that lowest threshold (sum_j [z_j - tau]_+^r - 1 is convex and decreasing
//                         in tau, so the steps rise to the root and never pass it), and
//                         O_i = sum_j p_ij v_j over the support.
#pragma once
#include "common.hip.h"
#include "fwd_sparse.hip.h"

namespace entmax {

// dynamic LDS of decode_scores_kernel: Q rows as in memory, the groups' maxima, a coefficient and a limit per row
inline size_t decode_scores_lds(int Nq, int D, size_t esize) { return (size_t)Nq * (D * esize + (kThreads / 8) * 4 + 12); }
constexpr int kDecodeSolveThreads = 1024;
constexpr int kDecodeListCap = 4096;    // support candidates kept in LDS; longer ones are re-read from the score row

struct DecodeArgs {
  Geom g;
  const void* Q;
  const void* K;
  const void* V;
  void* O;
  float* tau;     // [B*H*Nq]
  float* scores;  // [B*H*Nq][nks] workspace, entries j < row_limit(i) written; nks = Nk rounded up to 4
  float* cmax;    // [B*H*Nq][nchunks] largest score of each chunk of `chunk` keys (-inf: none visible)
  int nks, nchunks;
  int chunk;      // keys per workgroup of decode_scores_kernel, a multiple of 256
};

// x + (x of the lane that the DPP control CTRL pairs this lane with): one VALU instruction, no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
// Sum over each aligned group of eight lanes, in every lane of the group: lane k adds lane 7-k
// (row_half_mirror), then its neighbour in the pair (quad_perm [1,0,3,2]), then the other pair of its quad
// (quad_perm [2,3,0,1]).  The additions form the same tree in all eight lanes, so they agree to the bit.
__device__ __forceinline__ float sum8(float x) {
  x = dpp_add<0x141>(x);
  x = dpp_add<0xB1>(x);
  return dpp_add<0x4E>(x);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
// acc + a.lo * b.lo + a.hi * b.hi for two packed bf16 pairs, in fp32
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

// Eight lanes share a key row (each a contiguous eighth of its features), so a wave's load
// instruction covers eight whole rows; a thread keeps four rows in flight.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_scores_kernel(DecodeArgs A) {
  constexpr int kSlice = D / 8;
  extern __shared__ __align__(16) char decode_lds[];
  const Geom& g = A.g;
  constexpr int kRowWords = D * (int)sizeof(T) / 4;
  constexpr int kGroups = kThreads / 8;
  uint32_t* qw = reinterpret_cast<uint32_t*>(decode_lds);                  // [Nq][kRowWords]
  float* group_max = reinterpret_cast<float*>(qw + g.Nq * kRowWords);      // [Nq][kGroups]: entry [i][grp] is touched
                                                                           // by the group's first lane only
  float* coef = group_max + g.Nq * kGroups;                                // [Nq]
  int* limit = reinterpret_cast<int*>(coef + g.Nq);                        // [Nq]
  float* ybias = reinterpret_cast<float*>(limit + g.Nq);                   // [Nq] distance bias per unit distance, times (alpha-1)
  const int tid = threadIdx.x, bh = blockIdx.y, b = bh / g.H, h = bh % g.H;
  const int j0 = blockIdx.x * A.chunk;
  const T* Qh = reinterpret_cast<const T*>(A.Q) + (long long)b * g.q_sb + (long long)h * g.q_sh;
  const T* Kh = reinterpret_cast<const T*>(A.K) + (long long)b * g.kv_sb + (long long)h * g.kv_sh;
  // the first key rows are requested before anything else: their addresses need nothing from the queries
  const int grp = tid >> 3, sub = tid & 7;
  const int jend = min(j0 + A.chunk, g.Nk);
  RawRow<T, kSlice> nx[4];
  auto fetch = [&](RawRow<T, kSlice>* dst, int base) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = min(base + u * 32 + grp, g.Nk - 1);  // rows past the end repeat the last one and are not written
      dst[u].load(Kh + (long long)j * g.kv_sn + sub * kSlice);
    }
  };
  fetch(nx, j0);
  // Q in LDS as it is in memory: fp32, or bf16 pairs (then row i starts at word i * D/2)
  for (int e = tid; e < g.Nq * kRowWords; e += kThreads) {
    const int i = e / kRowWords, c = e % kRowWords;
    qw[e] = reinterpret_cast<const uint32_t*>(Qh + (long long)i * g.q_sn)[c];
  }
  if (tid < g.Nq) {
    const int lim = row_limit(g, tid);
    limit[tid] = lim;
    for (int w = 0; w < kGroups; ++w) group_max[tid * kGroups + w] = -kInf;
    const float cf = (g.alpha - 1.0f) * row_scale(g, b, h, tid, lim, nullptr, nullptr, nullptr) * (1.0f / sqrtf((float)D));
    coef[tid] = cf;
    // the same product a w as in the tiled kernels (bias_w(): sign taken from the scale)
    ybias[tid] = fabsf(cf) * bias_w<D>(g, h, cf, fabsf(cf));
  }
  __syncthreads();
  for (int base = j0; base < jend; base += 128) {
    RawRow<T, kSlice> kk[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) kk[u] = nx[u];
    if (base + 128 < jend) fetch(nx, base + 128);  // the next rows are on their way during the arithmetic
    for (int i = 0; i < g.Nq; ++i) {
      constexpr int kWords = RawRow<T, kSlice>::kWords;
      u32x4_t qv[kWords];  // the lane's slice of query row i
#pragma unroll
      for (int w = 0; w < kWords; ++w)
        qv[w] = *reinterpret_cast<const u32x4_t*>(&qw[i * kRowWords + sub * (kRowWords / 8) + 4 * w]);
      const float c = coef[i];
      const int lim = limit[i];
      const float yb = ybias[i];
      const int pos = i + (g.Nk - g.Nq);
      float best = -kInf;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float dot = 0.f;
#pragma unroll
        for (int w = 0; w < kWords; ++w) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            if constexpr (sizeof(T) == 2)
              dot = dot2_bf16(kk[u].w[w][k], qv[w][k], dot);  // two features per instruction, nothing to widen
            else
              dot = fmaf(__uint_as_float(kk[u].w[w][k]), __uint_as_float(qv[w][k]), dot);
          }
        }
        const int j = base + u * 32 + grp;
        const float zj = fmaf(yb, (float)bias_dist(pos, j), sum8(dot) * c);
        if (j < lim) best = fmaxf(best, zj);
        if (sub == u && j < lim) A.scores[((long long)bh * g.Nq + i) * A.nks + j] = zj;
      }
      if (sub == 0) group_max[i * kGroups + grp] = fmaxf(group_max[i * kGroups + grp], best);
    }
  }
  __syncthreads();
  for (int i0 = 0; i0 < g.Nq; i0 += 8) {
    // thread (i, grp) of an 8 x 32 arrangement: the row's maximum over the 32 groups
    const int i = i0 + (tid >> 5);
    float mx = i < g.Nq ? group_max[i * kGroups + (tid & 31)] : -kInf;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((tid & 31) == 0 && i < g.Nq) A.cmax[((long long)bh * g.Nq + i) * A.nchunks + blockIdx.x] = mx;
  }
}

// The same scores for 9 to 64 query rows, where the per-row dot products of the kernel above (about 5 us per
// row at Nk = 32768 and 48 heads) outweigh the read of K: S = Q K_chunk^T on the matrix cores, one or two
// 32-query blocks against 32-key blocks whose fragments come straight from global memory (every K row is read
// once by one lane pair, 16 bytes at a time along the row).  In the accumulator layout the 32 lanes of a half
// wave hold 32 consecutive keys of one query: the score rows are written in 128-byte runs.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_scores_mfma_kernel(DecodeArgs A) {
  constexpr int NC = D / 16;
  __shared__ f32x4_t rowinfo[64];  // per query row: coefficient, bias per unit distance, limit, position (as bits)
  __shared__ float wmax[kWaves][64];
  const Geom& g = A.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int bh = blockIdx.y, b = bh / g.H, h = bh % g.H;
  const int jc0 = blockIdx.x * A.chunk, jend = min(jc0 + A.chunk, g.Nk);
  const T* Qh = reinterpret_cast<const T*>(A.Q) + (long long)b * g.q_sb + (long long)h * g.q_sh;
  const T* Kh = reinterpret_cast<const T*>(A.K) + (long long)b * g.kv_sb + (long long)h * g.kv_sh;
  const int nqblk = (g.Nq + 31) >> 5;  // 1 or 2
  if (tid < 64) {
    const bool valid = tid < g.Nq;
    const int lim = valid ? row_limit(g, tid) : 0;
    const float cf = valid ? (g.alpha - 1.0f) * row_scale(g, b, h, tid, lim, nullptr, nullptr, nullptr) * (1.0f / sqrtf((float)D))
                           : 0.f;
    rowinfo[tid] = f32x4_t{cf, valid ? fabsf(cf) * bias_w<D>(g, h, cf, fabsf(cf)) : 0.f, __int_as_float(lim),
                           __int_as_float(tid + (g.Nk - g.Nq))};
  }
  // query fragments (A operand: row = query, 8 features per lane half)
  Frag<T> qf[2][NC];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int row = qb * 32 + li;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc)
      qf[qb][cc] = row < g.Nq ? Elem<T>::load(Qh + (long long)row * g.q_sn + 16 * cc + 8 * hh) : Elem<T>::zero();
  }
  __syncthreads();
  float rmax[2][16];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int e = 0; e < 16; ++e) rmax[qb][e] = -kInf;
  const int per_wave = A.chunk / kWaves;  // a multiple of 32 (the chunk is a multiple of 256)
  for (int j0 = jc0 + wave * per_wave; j0 < min(jc0 + (wave + 1) * per_wave, jend); j0 += 32) {
    const int key = j0 + li;  // this lane's key (B operand column, accumulator column)
    const bool kvalid = key < g.Nk;
    const T* krow = Kh + (long long)min(key, g.Nk - 1) * g.kv_sn;
    Frag<T> kf[NC];
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) kf[cc] = Elem<T>::load(krow + 16 * cc + 8 * hh);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      if (qb >= nqblk) break;
      f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) acc = Elem<T>::mma(qf[qb][cc], kf[cc], acc);
      // acc[4 q + r] of lane l: query qb*32 + 8 q + 4 (l/32) + r, key j0 + l%32
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int i = qb * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
        const f32x4_t ri = rowinfo[i];
        const int lim = __float_as_int(ri[2]), pos = __float_as_int(ri[3]);
        const float zj = fmaf(ri[1], (float)bias_dist(pos, key), acc[e] * ri[0]);
        if (kvalid && key < lim) {  // (lim = 0 for rows beyond Nq)
          A.scores[((long long)bh * g.Nq + i) * A.nks + key] = zj;
          rmax[qb][e] = fmaxf(rmax[qb][e], zj);
        }
      }
    }
  }
  // a query's maximum over the keys this wave saw: across the 32 lanes of its half wave
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float v = rmax[qb][e];
#pragma unroll
      for (int sft = 16; sft >= 1; sft >>= 1) v = fmaxf(v, __shfl_xor(v, sft));
      if (li == 0) wmax[wave][qb * 32 + 8 * (e >> 2) + 4 * hh + (e & 3)] = v;
    }
  }
  __syncthreads();
  if (tid < g.Nq) {
    float mx = wmax[0][tid];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, wmax[w][tid]);
    A.cmax[((long long)bh * g.Nq + tid) * A.nchunks + blockIdx.x] = mx;
  }
}

// Sum of two values over the workgroup; every thread gets the totals.  `buf` holds 2 * 2 * 16
// floats: calls alternate between its halves (parity), so one barrier per call is enough.
__device__ __forceinline__ float2 decode_block_sum(float a, float b, float* buf, int parity) {
  constexpr int kW = kDecodeSolveThreads / 64;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    a += __shfl_xor(a, off);
    b += __shfl_xor(b, off);
  }
  float* mine = buf + parity * 2 * kW;
  if ((threadIdx.x & 63) == 0) {
    mine[threadIdx.x >> 6] = a;
    mine[kW + (threadIdx.x >> 6)] = b;
  }
  __syncthreads();
  float sa = 0.f, sb = 0.f;
#pragma unroll
  for (int w = 0; w < kW; ++w) {
    sa += mine[w];
    sb += mine[kW + w];
  }
  return make_float2(sa, sb);
}

template <typename T, int D, int AM>
__global__ __launch_bounds__(kDecodeSolveThreads) void decode_solve_kernel(DecodeArgs A) {
  constexpr int kW = kDecodeSolveThreads / 64;
  constexpr int kSlots = kDecodeSolveThreads / D;  // threads with the same feature share out the support
  __shared__ float2 list[kDecodeListCap];          // (key index bits, z)
  __shared__ float red[2 * 2 * kW];
  __shared__ float wmax[kW];
  __shared__ int count;
  __shared__ float osum[kSlots * D];
  const Geom& g = A.g;
  const int tid = threadIdx.x;
  const int row = blockIdx.x, i = row % g.Nq, bh = row / g.Nq, b = bh / g.H, h = bh % g.H;
  const int lim = row_limit(g, i);
  const long long o_idx = (long long)b * g.q_sb + (long long)h * g.q_sh + (long long)i * g.q_sn;
  if (lim == 0) {  // no visible key: an empty sum
    if (tid < D) Elem<T>::store(A.O, o_idx + tid, 0.f);
    if (tid == 0) A.tau[row] = 0.f;
    return;
  }
  const float* z = A.scores + (long long)row * A.nks;
  const float* cmax = A.cmax + (long long)row * A.nchunks;
  const float r = 1.0f / (g.alpha - 1.0f);
  // row maximum from the chunks' maxima
  float m = -kInf;
  for (int c = tid; c < A.nchunks; c += kDecodeSolveThreads) m = fmaxf(m, cmax[c]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((tid & 63) == 0) wmax[tid >> 6] = m;
  if (tid == 0) count = 0;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kW; ++w) m = fmaxf(m, wmax[w]);
  // keys with a non-zero term at the lowest threshold tau_lo = max - 1 (there the maximum's own term is 1,
  // so the sum is >= 1 and the root is >= tau_lo); a wave takes a chunk at a time and skips those whose
  // maximum is out of reach
  const float tau_lo = m - 1.0f;
  for (int c = tid >> 6; c < A.nchunks; c += kW) {
    if (!(cmax[c] > tau_lo)) continue;
    for (int v = 0; v < A.chunk / 256; ++v) {
      const int j = c * A.chunk + (v * 64 + (tid & 63)) * 4;
      if (j >= lim) continue;
      const f32x4_t zv = *reinterpret_cast<const f32x4_t*>(z + j);  // nks is a multiple of 4: the word is inside the row
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (j + k < lim && zv[k] > tau_lo) {
          const int pos = atomicAdd(&count, 1);
          if (pos < kDecodeListCap) list[pos] = make_float2(__int_as_float(j + k), zv[k]);
        }
      }
    }
  }
  __syncthreads();
  const int total = count;
  const bool in_lds = total <= kDecodeListCap;
  const int n_items = in_lds ? total : lim;
  float tau = tau_lo;
  for (int it = 0; it < 96; ++it) {
    float F = 0.f, G = 0.f;
    for (int e = tid; e < n_items; e += kDecodeSolveThreads) {
      const float x = (in_lds ? list[e].y : z[e]) - tau;
      if (x > 0.f) {
        F += pow_r<AM>(x, r);
        G += pow_rm1<AM>(x, r);
      }
    }
    const float2 s = decode_block_sum(F, G, red, it & 1);
    if (!(s.y > 0.f)) break;
    const float step = (s.x - 1.0f) / (r * s.y);  // Newton: f = F - 1, f' = -r G; G > 0 while tau < max
    if (!(step > 0.f)) break;
    tau += step;
    if (step <= 1e-6f * fmaxf(1.0f, fabsf(tau))) break;  // what is left is a small multiple of the last step
  }
  if (tid == 0) A.tau[row] = tau;
  // O_i = sum_j p_ij v_j
  const T* Vh = reinterpret_cast<const T*>(A.V) + (long long)b * g.kv_sb + (long long)h * g.kv_sh;
  const int slot = tid / D, c = tid % D;
  float acc = 0.f;
  for (int e = slot; e < n_items; e += kSlots) {
    const float2 en = in_lds ? list[e] : make_float2(__int_as_float(e), z[e]);
    const float x = en.y - tau;
    if (x > 0.f) {
      const long long vi = (long long)__float_as_int(en.x) * g.kv_sn + c;
      float v;
      if constexpr (sizeof(T) == 2)
        v = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(Vh)[vi] << 16);
      else
        v = reinterpret_cast<const float*>(Vh)[vi];
      acc = fmaf(pow_r<AM>(x, r), v, acc);
    }
  }
  osum[slot * D + c] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
#pragma unroll
    for (int s = 0; s < kSlots; ++s) o += osum[s * D + tid];
    Elem<T>::store(A.O, o_idx + tid, o);
  }
}

}  // namespace entmax
