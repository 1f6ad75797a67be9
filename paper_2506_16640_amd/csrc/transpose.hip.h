// Transposed, row-permuted copies of a [B,H,N,D] tensor, written once per call
// into the workspace: Xt[bh][dc][16c + p] = X[bh][16c + perm(p)][dc] with
//   perm(p) = 8*((p%8)/4) + 4*(p/8) + p%4,
// zero beyond row N, N padded to a multiple of 64.  A lane of half hh then finds
// the 8 rows {16c + 8*(e/4) + 4*hh + e%4 : e = 0..7} -- the rows whose
// accumulator values it holds after a 32x32 MFMA -- contiguous at column
// 16c + 8*hh of row dc, i.e. as one MFMA fragment of the product that contracts
// over the rows of X (P.V, dS.K, P^T.dO, dS^T.Q).
#pragma once
#include "common.hip.h"

namespace entmax {

struct TransposeJob {
  const void* X;
  void* Xt;
  long long sb, sh, sn;
  int N, npad;
};
struct TransposeJobs {
  TransposeJob job[3];  // blockIdx.z picks one
};

// head_flag (one per head) or block_flag (nqb per head), when given, say whether any consumer needs the
// head's copies: without a set flag the workgroup returns at once.
// bx: 64-row tile of the tensor, bh: (batch, head), bz: job.  All 256 threads of a workgroup call this together.
template <typename T, int D>
__device__ __forceinline__ void transpose_perm_part(const TransposeJobs& jobs, int H, const int* head_flag,
                                                    const int* block_flag, int nqb, int bx, int bh, int bz) {
  constexpr int kPad = sizeof(T) == 2 ? 2 : 1;
  __shared__ T tile[64][D + kPad];
  const int tid = threadIdx.x;
  const int b = bh / H, h = bh % H;
  if (head_flag && head_flag[bh] == 0) return;  // no consumer for this head's copy
  if (block_flag) {
    int any = 0;
    for (int k = tid; k < nqb; k += kThreads) any |= block_flag[bh * nqb + k];
    if (__syncthreads_or(any) == 0) return;
  }
  const TransposeJob& jb = jobs.job[bz];
  const int N = jb.N, npad = jb.npad;
  const long long sn = jb.sn;
  const int j0 = bx * 64;
  if (j0 >= npad) return;  // the grid covers the longest job
  const T* src = reinterpret_cast<const T*>(jb.X) + (long long)b * jb.sb + (long long)h * jb.sh;
  T* Xt = reinterpret_cast<T*>(jb.Xt);
  // 16-byte chunks both ways: rows of X come in whole chunks (the strides are multiples of 16 bytes), and a chunk
  // of a row of Xt is kEpc consecutive positions, gathered from one column of the tile
  constexpr int kEpc = 16 / (int)sizeof(T), kCpr = D / kEpc, kCpo = 64 / kEpc;
  for (int c = tid; c < 64 * kCpr; c += kThreads) {
    const int row = c / kCpr, ch = c % kCpr;
    const int j = j0 + row;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (j < N) v = *reinterpret_cast<const u32x4_t*>(src + (long long)j * sn + ch * kEpc);
    uint32_t* t = reinterpret_cast<uint32_t*>(&tile[row][ch * kEpc]);  // rows are 4-byte, not 16-byte, aligned
    t[0] = v[0];
    t[1] = v[1];
    t[2] = v[2];
    t[3] = v[3];
  }
  __syncthreads();
  T* dst = Xt + (long long)bh * D * npad + j0;
  for (int c = tid; c < D * kCpo; c += kThreads) {
    const int dc = c / kCpo, pos0 = (c % kCpo) * kEpc;  // neighbouring lanes: neighbouring chunks of one row of Xt
    T vals[kEpc];
#pragma unroll
    for (int e = 0; e < kEpc; ++e) {
      const int pos = pos0 + e, p = pos & 15;
      const int srow = (pos & ~15) + 8 * ((p & 7) >> 2) + 4 * (p >> 3) + (p & 3);
      vals[e] = tile[srow][dc];
    }
    u32x4_t o;
    __builtin_memcpy(&o, vals, 16);
    *reinterpret_cast<u32x4_t*>(dst + (long long)dc * npad + pos0) = o;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void transpose_perm_kernel(TransposeJobs jobs, int H, const int* head_flag,
                                                                 const int* block_flag, int nqb) {
  transpose_perm_part<T, D>(jobs, H, head_flag, block_flag, nqb, blockIdx.x, blockIdx.y, blockIdx.z);
}

// The same work as extra workgroups of another kernel's launch (the copies are only needed by the tiled kernels
// that follow, and a launch of their own would cost more than the copies of the few heads that need them):
// workgroup `idx` of the nx * BH * njobs riders.
struct TransposeRide {
  TransposeJobs jobs;
  int njobs, nx, BH, H;     // nx: 64-row tiles of the longest job; njobs = 0: no riders
  const int* head_flag;
  const int* block_flag;
  int nqb;
  __host__ __device__ int workgroups() const { return njobs * nx * BH; }
};
template <typename T, int D>
__device__ __forceinline__ void transpose_ride(const TransposeRide& r, int idx) {
  const int bx = idx % r.nx, bh = (idx / r.nx) % r.BH, bz = idx / (r.nx * r.BH);
  transpose_perm_part<T, D>(r.jobs, r.H, r.head_flag, r.block_flag, r.nqb, bx, bh, bz);
}

// O = 0, tau = 0 for problems without keys (Nk = 0), or any plain fill.
static __global__ void fill_words_kernel(uint32_t* p, long long nwords, uint32_t value) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nwords) p[i] = value;
}

}  // namespace entmax
