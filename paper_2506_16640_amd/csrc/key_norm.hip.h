// The heads' largest key norms: what the window of the linear distance bias (App. B, ALiBi proposition;
// QCtx::init_window) needs to bound a row's logits.
#pragma once
#include "fwd_sparse.hip.h"
#include "launch.hip.h"

namespace entmax {

// Largest key norm of every head, for the window of the distance bias (QCtx::init_window).  Eight lanes share
// a key row; knorm [B*H] must hold zeros before the launch (norms are >= 0, so their bit patterns order like
// unsigned integers).  grid (ceil(Nk / 256), B*H).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void key_norm_kernel(const void* K, long long sb, long long sh, long long sn, int H,
                                                            int Nk, float* knorm) {
  constexpr int kSlice = D / 8;
  const int bh = blockIdx.y, grp = threadIdx.x >> 3, sub = threadIdx.x & 7;
  const T* Kh = reinterpret_cast<const T*>(K) + (long long)(bh / H) * sb + (long long)(bh % H) * sh;
  float best = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int j = blockIdx.x * 256 + u * 32 + grp;
    RawRow<T, kSlice> kk;
    kk.load(Kh + (long long)min(j, Nk - 1) * sn + sub * kSlice);
    float s2 = 0.f;
#pragma unroll
    for (int t = 0; t < kSlice; ++t) s2 = fmaf(kk.get(t), kk.get(t), s2);
    s2 += __shfl_xor(s2, 1);
    s2 += __shfl_xor(s2, 2);
    s2 += __shfl_xor(s2, 4);
    best = fmaxf(best, s2);
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) best = fmaxf(best, __shfl_xor(best, sft));
  if ((threadIdx.x & 63) == 0) atomicMax(reinterpret_cast<unsigned*>(knorm) + bh, __float_as_uint(sqrtf(best)));
}

namespace {

// the heads' largest key norms into knorm (zero fill, then one pass over K)
template <typename T, int D>
bool launch_key_norms(const entmax_attn_params* p, const Layout& L, const void* K, float* knorm, hipStream_t st) {
  if (!zero_words(knorm, (size_t)p->B * p->H * sizeof(float), st)) return false;
  hipLaunchKernelGGL((key_norm_kernel<T, D>), dim3((unsigned)((p->Nk + 255) / 256), (unsigned)(p->B * p->H)),
                     dim3(kThreads), 0, st, K, L.kv_sb, L.kv_sh, L.kv_sn, p->H, p->Nk, knorm);
  return launch_ok();
}


}  // namespace
}  // namespace entmax
