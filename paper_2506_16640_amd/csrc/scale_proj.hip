// ASEntmax scale projections (Sec. 4.1, the equations after eq. (asentmax)): the step right before the
// attention.  For token embeddings X [B,N,E] and per-head projection vectors w_beta,h, w_gamma,h (rows of
// Wb, Wg [H,E], fp32)
//     beta[b,h,i] = softplus(<x_{b,i}, w_beta,h>),   gamma[b,h,i] = s tanh(<x_{b,i}, w_gamma,h>)
// in the per-query layout [B,H,N] the attention takes, and the gradients dX, dWb, dWg from d beta, d gamma.
//
//   scale_proj_fwd_kernel   the 2H inner products per token are a thin dense contraction over E: on the
//                           matrix cores, transposed (rows = the 2H outputs, columns = 32 tokens of a wave) so
//                           that a lane owns a token and stores run along the token axis.  W is split into
//                           bf16 hi + lo parts in registers (two products): the pre-activations carry fp32
//                           accuracy, which they need because beta multiplies every logit of the row.
//   scale_proj_bwd_kernel   bound by one read of X and one write of dX: plain fp32 FMAs, a thread per feature
//                           column, a workgroup per (64 tokens, 256 columns).  One pass over the tokens with the
//                           2H pre-activation gradients G of a token broadcast from LDS:
//                           dX_t[k] = sum_c G[t][c] W[c][k] (W[.][k] in registers) and this workgroup's share of
//                           dW[c][k] = sum_t G[t][c] x_t[k], written as a partial sum.
//   scale_proj_reduce_kernel  sums the workgroups' partial dW in a fixed order (no floating-point atomics).
// beta and gamma determine their own derivatives (sigmoid(u) = 1 - e^-beta, 1 - tanh^2 v = 1 - (gamma/s)^2), so
// the pre-activations are not stored.
#include "entmax_attn.h"

#include <hip/hip_runtime.h>

#include "common.hip.h"

using namespace entmax;

namespace {

constexpr int kProjTokens = 32;   // tokens per workgroup of the forward
constexpr int kBwdTokens = 64;    // tokens per workgroup of the backward

struct ProjGeom {
  int B, H, N, E;
  float s;
};

// 8 consecutive elements of a token row as bf16 hi (+ lo for fp32 inputs) fragments
template <typename T>
__device__ __forceinline__ void load_x_frag(const T* p, bool valid, Frag<bf16_t>& hi, Frag<bf16_t>& lo) {
  if constexpr (sizeof(T) == 2) {
    hi = valid ? Elem<bf16_t>::load(p) : Elem<bf16_t>::zero();
    lo = Elem<bf16_t>::zero();
  } else {
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = valid ? p[e] : 0.f;
    Elem<bf16_t>::pack_split(x, hi, lo);
  }
}

// A workgroup takes 32 tokens; its four waves split the contraction over E between them (16-wide chunks in
// turn), and the four partial products are added through LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(kThreads) void scale_proj_fwd_kernel(ProjGeom g, const T* X, const float* Wb, const float* Wg,
                                                                  float* beta, float* gamma) {
  __shared__ float part[kWaves][16][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, hh = lane >> 5;
  const int hg = blockIdx.y;  // group of 16 heads: output rows 0..15 = beta of heads 16 hg + r, 16..31 = gamma
  const long long T_total = (long long)g.B * g.N;
  const long long t = (long long)blockIdx.x * kProjTokens + li;  // this lane's token (B operand column)
  const bool tvalid = t < T_total;
  const T* xrow = X + (tvalid ? t : 0) * g.E;
  // this lane's output row of W (A operand row li): beta rows first
  const int wh = hg * 16 + (li & 15);
  const bool wvalid = wh < g.H;
  const float* wrow = ((li < 16) ? Wb : Wg) + (long long)(wvalid ? wh : 0) * g.E;

  f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int k0 = wave * 16; k0 < g.E; k0 += kWaves * 16) {
    const int k = k0 + 8 * hh;
    float w[8];
    const f32x4_t w0 = *reinterpret_cast<const f32x4_t*>(wrow + k), w1 = *reinterpret_cast<const f32x4_t*>(wrow + k + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[e] = wvalid ? w0[e] : 0.f;
      w[4 + e] = wvalid ? w1[e] : 0.f;
    }
    Frag<bf16_t> whi, wlo, xhi, xlo;
    Elem<bf16_t>::pack_split(w, whi, wlo);
    load_x_frag<T>(xrow + k, tvalid, xhi, xlo);
    acc = Elem<bf16_t>::mma(whi, xhi, acc);
    acc = Elem<bf16_t>::mma(wlo, xhi, acc);
    if constexpr (sizeof(T) == 4) {
      acc = Elem<bf16_t>::mma(whi, xlo, acc);
      acc = Elem<bf16_t>::mma(wlo, xlo, acc);
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) part[wave][e][lane] = acc[e];
  __syncthreads();
  if (!tvalid) return;
  const int b = (int)(t / g.N), i = (int)(t % g.N);
  // element e of lane l is output row 8 (e/4) + 4 (l/32) + e%4 for token l%32; wave w finishes e = 4w .. 4w+3
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int e = 4 * wave + r;
    const int row = 8 * wave + 4 * hh + r;
    const int head = hg * 16 + (row & 15);
    if (head >= g.H) continue;
    const float u = ((part[0][e][lane] + part[1][e][lane]) + part[2][e][lane]) + part[3][e][lane];
    const long long o = ((long long)b * g.H + head) * g.N + i;
    if (row < 16)
      beta[o] = fmaxf(u, 0.f) + log1pf(expf(-fabsf(u)));  // ln(1 + e^u) without overflow
    else
      gamma[o] = g.s * tanhf(u);
  }
}

// C2: rows of the stacked projection matrix handled per thread (2 H rounded up to a multiple of 8)
template <typename T, int C2>
__global__ __launch_bounds__(kThreads) void scale_proj_bwd_kernel(ProjGeom g, const T* X, const float* Wb, const float* Wg,
                                                                  const float* beta, const float* gamma, const float* dbeta,
                                                                  const float* dgamma, T* dX, float* partial) {
  __shared__ float G[kBwdTokens][C2];  // pre-activation gradients: columns 0..H-1 beta, H..2H-1 gamma
  const int tid = threadIdx.x;
  const long long T_total = (long long)g.B * g.N;
  const long long t0 = (long long)blockIdx.x * kBwdTokens;
  const int ntok = (int)min((long long)kBwdTokens, T_total - t0);
  const int H = g.H;
  // G: thread (c, token) with the token index fastest (beta, gamma are contiguous along tokens)
  for (int idx = tid; idx < C2 * kBwdTokens; idx += kThreads) {
    const int c = idx / kBwdTokens, tt = idx % kBwdTokens;
    float gval = 0.f;
    if (tt < ntok && c < 2 * H) {
      const long long t = t0 + tt;
      const int b = (int)(t / g.N), i = (int)(t % g.N), h = c < H ? c : c - H;
      const long long o = ((long long)b * H + h) * g.N + i;
      if (c < H) {
        gval = dbeta[o] * -expm1f(-beta[o]);  // d softplus / du = e^u / (1 + e^u) = 1 - e^-beta
      } else {
        const float ga = gamma[o];
        gval = dgamma[o] * (g.s - ga * ga / g.s);  // s (1 - tanh^2 v), tanh v = gamma / s
      }
    }
    G[tt][c] = gval;
  }
  __syncthreads();
  // a thread per feature column: W[.][k] and the partial dW[.][k] in registers, one pass over the tokens
  const int k = blockIdx.y * kThreads + tid;
  if (k >= g.E) return;
  float w[C2], acc[C2];
#pragma unroll
  for (int c = 0; c < C2; ++c) {
    acc[c] = 0.f;
    w[c] = 0.f;
    if (c < 2 * H) w[c] = (c < H ? Wb + (long long)c * g.E : Wg + (long long)(c - H) * g.E)[k];
  }
  auto widen = [](T v) {
    if constexpr (sizeof(T) == 2)
      return __uint_as_float((uint32_t)v.bits << 16);
    else
      return v;
  };
  constexpr int kUnroll = 8;  // token rows in flight
  for (int t8 = 0; t8 < ntok; t8 += kUnroll) {
    float x[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) x[u] = widen(X[(t0 + min(t8 + u, ntok - 1)) * g.E + k]);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int tt = t8 + u;
      if (tt >= ntok) break;  // uniform
      float a = 0.f;
#pragma unroll
      for (int c4 = 0; c4 < C2 / 4; ++c4) {
        const f32x4_t gv = *reinterpret_cast<const f32x4_t*>(&G[tt][4 * c4]);  // same address in all lanes: broadcast
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          a = fmaf(gv[r], w[4 * c4 + r], a);                               // dX_t[k] = sum_c G[t][c] W[c][k]
          acc[4 * c4 + r] = fmaf(gv[r], x[u], acc[4 * c4 + r]);            // dW[c][k] += G[t][c] x_t[k]
        }
      }
      Elem<T>::store(dX, (t0 + tt) * g.E + k, a);
    }
  }
  float* dst = partial + (long long)blockIdx.x * 2 * H * g.E;
#pragma unroll
  for (int c = 0; c < C2; ++c)
    if (c < 2 * H) dst[(long long)c * g.E + k] = acc[c];
}

// dWb | dWg [2H][E] = sum over the nblk workgroups' partial sums.  A workgroup takes 64 outputs; four groups of
// threads each sum every fourth partial (eight loads in flight), and the four sums are added in a fixed order.
__global__ __launch_bounds__(kThreads) void scale_proj_reduce_kernel(const float* partial, int nblk, int H, int E, float* dWb,
                                                                     float* dWg) {
  __shared__ float part[4][64];
  const int o = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const long long idx = (long long)blockIdx.x * 64 + o;
  const long long per = 2LL * H * E;
  float s = 0.f;
  if (idx < per) {
    int b = grp;
    for (; b + 28 < nblk; b += 32) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[(long long)(b + 4 * u) * per + idx];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; b < nblk; b += 4) s += partial[(long long)b * per + idx];
  }
  part[grp][o] = s;
  __syncthreads();
  if (grp == 0 && idx < per) {
    const float tot = ((part[0][o] + part[1][o]) + part[2][o]) + part[3][o];
    if (idx < (long long)H * E)
      dWb[idx] = tot;
    else
      dWg[idx - (long long)H * E] = tot;
  }
}

int check_proj(const entmax_scale_proj_params* p) {
  if (!p) return ENTMAX_ATTN_INVALID_ARG;
  if (p->B < 0 || p->H < 0 || p->N < 0 || p->E <= 0) return ENTMAX_ATTN_INVALID_ARG;
  if (p->dtype != ENTMAX_ATTN_BF16 && p->dtype != ENTMAX_ATTN_FP32) return ENTMAX_ATTN_INVALID_ARG;
  if (!(p->gamma_scale > 0.0f) || !(p->gamma_scale < 3.0e38f)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->E % 16 != 0 || p->E > 16384) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (p->H > 16) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;  // one 32-row product holds the 2 H stacked projections
  if ((long long)p->B * p->N > 0x7fffffffLL / 64) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  return ENTMAX_ATTN_OK;
}

inline long long bwd_blocks(const entmax_scale_proj_params* p) {
  return ((long long)p->B * p->N + kBwdTokens - 1) / kBwdTokens;
}

inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace

namespace {
template <typename T>
bool launch_proj_bwd(const ProjGeom& g, int nblk, const void* X, const float* Wb, const float* Wg, const float* beta,
                     const float* gamma, const float* dbeta, const float* dgamma, void* dX, float* partial, hipStream_t st) {
  const T* x = reinterpret_cast<const T*>(X);
  T* dx = reinterpret_cast<T*>(dX);
  const dim3 grid((unsigned)nblk, (unsigned)((g.E + kThreads - 1) / kThreads)), block(kThreads);
  const int c2 = (2 * g.H + 7) / 8 * 8;
  switch (c2) {
    case 8: hipLaunchKernelGGL((scale_proj_bwd_kernel<T, 8>), grid, block, 0, st, g, x, Wb, Wg, beta, gamma, dbeta, dgamma, dx, partial); break;
    case 16: hipLaunchKernelGGL((scale_proj_bwd_kernel<T, 16>), grid, block, 0, st, g, x, Wb, Wg, beta, gamma, dbeta, dgamma, dx, partial); break;
    case 24: hipLaunchKernelGGL((scale_proj_bwd_kernel<T, 24>), grid, block, 0, st, g, x, Wb, Wg, beta, gamma, dbeta, dgamma, dx, partial); break;
    default: hipLaunchKernelGGL((scale_proj_bwd_kernel<T, 32>), grid, block, 0, st, g, x, Wb, Wg, beta, gamma, dbeta, dgamma, dx, partial); break;
  }
  return hipGetLastError() == hipSuccess;
}
}  // namespace

extern "C" {

size_t entmax_scale_proj_workspace_bytes(const entmax_scale_proj_params* p) {
  if (check_proj(p) != ENTMAX_ATTN_OK) return 0;
  const size_t n = (size_t)bwd_blocks(p) * 2 * p->H * p->E * sizeof(float);
  return n < 256 ? 256 : n;
}

int entmax_scale_proj_fwd(const entmax_scale_proj_params* p, const void* X, const float* Wb, const float* Wg, float* beta,
                          float* gamma, void* hip_stream) {
  int rc = check_proj(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  if ((long long)p->B * p->N * p->H == 0) return ENTMAX_ATTN_OK;
  if (!X || !Wb || !Wg || !beta || !gamma) return ENTMAX_ATTN_INVALID_ARG;
  if (misaligned16(X) || misaligned16(Wb) || misaligned16(Wg) || (reinterpret_cast<uintptr_t>(beta) & 3u) ||
      (reinterpret_cast<uintptr_t>(gamma) & 3u))
    return ENTMAX_ATTN_MISALIGNED;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  ProjGeom g{p->B, p->H, p->N, p->E, p->gamma_scale};
  const dim3 grid((unsigned)(((long long)p->B * p->N + kProjTokens - 1) / kProjTokens), (unsigned)((p->H + 15) / 16));
  if (p->dtype == ENTMAX_ATTN_BF16)
    hipLaunchKernelGGL(scale_proj_fwd_kernel<bf16_t>, grid, dim3(kThreads), 0, st, g, reinterpret_cast<const bf16_t*>(X), Wb,
                       Wg, beta, gamma);
  else
    hipLaunchKernelGGL(scale_proj_fwd_kernel<float>, grid, dim3(kThreads), 0, st, g, reinterpret_cast<const float*>(X), Wb, Wg,
                       beta, gamma);
  return hipGetLastError() == hipSuccess ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED;
}

int entmax_scale_proj_bwd(const entmax_scale_proj_params* p, const void* X, const float* Wb, const float* Wg,
                          const float* beta, const float* gamma, const float* dbeta, const float* dgamma, void* dX,
                          float* dWb, float* dWg, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_proj(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  if (p->H == 0) return ENTMAX_ATTN_OK;
  if (!Wb || !Wg || !dWb || !dWg || !workspace) return ENTMAX_ATTN_INVALID_ARG;
  const long long tokens = (long long)p->B * p->N;
  if (tokens > 0 && (!X || !beta || !gamma || !dbeta || !dgamma || !dX)) return ENTMAX_ATTN_INVALID_ARG;
  if (misaligned16(X) || misaligned16(dX) || misaligned16(Wb) || misaligned16(Wg) || misaligned16(dWb) || misaligned16(dWg) ||
      misaligned16(workspace))
    return ENTMAX_ATTN_MISALIGNED;
  if (workspace_bytes < entmax_scale_proj_workspace_bytes(p)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  ProjGeom g{p->B, p->H, p->N, p->E, p->gamma_scale};
  const int nblk = (int)bwd_blocks(p);
  float* partial = reinterpret_cast<float*>(workspace);
  if (nblk > 0) {
    const bool ok = p->dtype == ENTMAX_ATTN_BF16
                        ? launch_proj_bwd<bf16_t>(g, nblk, X, Wb, Wg, beta, gamma, dbeta, dgamma, dX, partial, st)
                        : launch_proj_bwd<float>(g, nblk, X, Wb, Wg, beta, gamma, dbeta, dgamma, dX, partial, st);
    if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
  }
  const long long per = 2LL * p->H * p->E;
  hipLaunchKernelGGL(scale_proj_reduce_kernel, dim3((unsigned)((per + 63) / 64)), dim3(kThreads), 0, st, partial,
                     nblk, p->H, p->E, dWb, dWg);
  return hipGetLastError() == hipSuccess ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED;
}

}  // extern "C"
