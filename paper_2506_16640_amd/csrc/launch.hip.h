// Host-side launch helpers shared by the forward and backward launchers, and the
// declarations of the per-(element type, head dimension) launchers themselves.
// Each launcher is instantiated in a translation unit of its own (inst.hip) so that
// the kernels of the four (type, D) combinations compile in parallel.
#pragma once
#include <hip/hip_runtime.h>

#include "common.hip.h"
#include "host_layout.h"
#include "transpose.hip.h"

namespace entmax {

// Enqueues the forward / backward for validated parameters; returns an entmax_attn_status.
// BIAS: the kernels built for the linear distance bias (slopes must then be given); the entry points choose
// by whether the caller passed slopes, so calls without them run exactly the kernels without the bias code.
template <typename T, int D, bool BIAS>
int run_fwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V,
            const float* beta, const float* gamma, const float* slopes, void* O, float* tau, char* saved,
            size_t saved_bytes, uint64_t* stats, char* ws, hipStream_t st, void* const* ev);
template <typename T, int D, bool BIAS>
int run_bwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V, const void* dO,
            const float* tau, const char* saved, size_t saved_bytes, const float* beta, const float* gamma,
            const float* slopes, void* dQ, void* dK, void* dV, float* dbeta, float* dgamma, uint64_t* stats, char* ws,
            hipStream_t st, void* const* ev);

namespace {

Geom make_geom(const entmax_attn_params* p, const Layout& L, const float* beta, const float* gamma,
               const float* slopes, const float* knorm) {
  Geom g;
  g.B = p->B;
  g.H = p->H;
  g.Nq = p->Nq;
  g.Nk = p->Nk;
  g.causal = p->causal;
  g.scale_layout = p->scale_layout;
  g.logn_mode = p->logn_mode;
  g.alpha = p->alpha;
  g.delta = p->delta;
  g.q_sb = L.q_sb;
  g.q_sh = L.q_sh;
  g.q_sn = L.q_sn;
  g.kv_sb = L.kv_sb;
  g.kv_sh = L.kv_sh;
  g.kv_sn = L.kv_sn;
  g.npad_k = L.npad_k;
  g.npad_q = L.npad_q;
  g.beta = beta;
  g.gamma = gamma;
  g.slopes = slopes;
  g.bias_mode = p->bias_mode;
  g.knorm = knorm;
  return g;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int alpha_mode(float alpha) {
  if (alpha == 1.5f) return 1;
  if (alpha == 2.0f) return 2;
  if (alpha == 1.25f) return 3;
  return 0;
}

inline bool launch_ok() { return hipGetLastError() == hipSuccess; }

// Raises a kernel's dynamic-LDS limit to `bytes` on the current device, once: later calls that need no more than
// what was already granted make no runtime call.  One counter per kernel (KERN) and device.
template <auto KERN>
bool ensure_dynamic_lds(size_t bytes) {
  constexpr int kMaxDevices = 64;
  static int granted[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
  int have = __atomic_load_n(&granted[dev], __ATOMIC_ACQUIRE);
  if ((size_t)have >= bytes) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(KERN), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) !=
      hipSuccess)
    return false;
  // concurrent callers may both set the attribute; the larger request wins in the table
  while (have < (int)bytes && !__atomic_compare_exchange_n(&granted[dev], &have, (int)bytes, false, __ATOMIC_RELEASE,
                                                           __ATOMIC_ACQUIRE)) {
  }
  return true;
}

inline void record(void* const* ev, int k, hipStream_t st) {
  if (ev) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(ev[k]), st);
}

// writes zeros into every row of a [B,H,N,D] tensor given by strides
template <typename T>
__global__ void zero_rows_kernel(T* X, long long sb, long long sh, long long sn, int H, int N, int D) {
  long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long per = (long long)N * D;
  if (e >= per) return;
  int bh = blockIdx.y;
  T z{};
  X[(long long)(bh / H) * sb + (long long)(bh % H) * sh + (e / D) * sn + e % D] = z;
}

template <typename T>
bool zero_rows(void* X, long long sb, long long sh, long long sn, int B, int H, int N, int D, hipStream_t st) {
  if ((long long)B * H * N == 0) return true;
  long long per = (long long)N * D;
  dim3 grid((unsigned)((per + 255) / 256), (unsigned)(B * H));
  hipLaunchKernelGGL(zero_rows_kernel<T>, grid, dim3(256), 0, st, reinterpret_cast<T*>(X), sb, sh, sn, H, N, D);
  return launch_ok();
}

bool fill_words(void* p, size_t bytes, uint32_t value, hipStream_t st) {
  long long n = (long long)(bytes / 4);
  if (n == 0) return true;
  hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(p), n, value);
  return launch_ok();
}
bool zero_words(void* p, size_t bytes, hipStream_t st) { return fill_words(p, bytes, 0u, st); }

template <typename T, int D>
bool launch_transposes(const TransposeJobs& jobs, int njobs, int B, int H, hipStream_t st, const int* head_flag = nullptr,
                       const int* block_flag = nullptr, int nqb = 0) {
  int npad = 0;
  for (int k = 0; k < njobs; ++k) npad = jobs.job[k].npad > npad ? jobs.job[k].npad : npad;
  if (npad == 0) return true;
  dim3 grid((unsigned)(npad / 64), (unsigned)(B * H), (unsigned)njobs);
  hipLaunchKernelGGL((transpose_perm_kernel<T, D>), grid, dim3(kThreads), 0, st, jobs, H, head_flag, block_flag, nqb);
  return launch_ok();
}

// the same jobs as riders of another launch (see TransposeRide)
inline TransposeRide transpose_ride_of(const TransposeJobs& jobs, int njobs, int B, int H, const int* head_flag,
                                       const int* block_flag, int nqb) {
  TransposeRide r{};
  r.jobs = jobs;
  int npad = 0;
  for (int k = 0; k < njobs; ++k) npad = jobs.job[k].npad > npad ? jobs.job[k].npad : npad;
  r.njobs = npad > 0 ? njobs : 0;
  r.nx = npad / 64;
  r.BH = B * H;
  r.H = H;
  r.head_flag = head_flag;
  r.block_flag = block_flag;
  r.nqb = nqb;
  return r;
}

inline TransposeJob transpose_job(const void* X, long long sb, long long sh, long long sn, int N, int npad, void* Xt) {
  TransposeJob j;
  j.X = X;
  j.Xt = Xt;
  j.sb = sb;
  j.sh = sh;
  j.sn = sn;
  j.N = N;
  j.npad = npad;
  return j;
}

}  // namespace
}  // namespace entmax
