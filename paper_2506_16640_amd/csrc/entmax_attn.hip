// Entry points of the C ABI declared in include/entmax_attn.h: argument validation
// and dispatch to the per-(element type, head dimension) launchers.  Nothing here
// allocates device memory or synchronises.
#include "entmax_attn.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "launch.hip.h"

using namespace entmax;

namespace entmax {
#define ENTMAX_FWD_SIG                                                                                                  \
  (const entmax_attn_params*, const Layout&, const void*, const void*, const void*, const float*, const float*,        \
   const float*, void*, float*, char*, size_t, uint64_t*, char*, hipStream_t, void* const*)
#define ENTMAX_BWD_SIG                                                                                                  \
  (const entmax_attn_params*, const Layout&, const void*, const void*, const void*, const void*, const float*,         \
   const char*, size_t, const float*, const float*, const float*, void*, void*, void*, float*, float*, uint64_t*,      \
   char*, hipStream_t, void* const*)
#define ENTMAX_EXTERN(T, D)                                   \
  extern template int run_fwd<T, D, false> ENTMAX_FWD_SIG;    \
  extern template int run_fwd<T, D, true> ENTMAX_FWD_SIG;     \
  extern template int run_bwd<T, D, false> ENTMAX_BWD_SIG;    \
  extern template int run_bwd<T, D, true> ENTMAX_BWD_SIG;
ENTMAX_EXTERN(bf16_t, 64)
ENTMAX_EXTERN(bf16_t, 128)
ENTMAX_EXTERN(float, 64)
ENTMAX_EXTERN(float, 128)
#undef ENTMAX_EXTERN
#undef ENTMAX_FWD_SIG
#undef ENTMAX_BWD_SIG
}  // namespace entmax

namespace {

// Built-in scratch of entmax_attn_fwd_noalloc.  Every device that loads the library holds its own copy of
// the array at its own address; in host code the array's name is only a handle for hipGetSymbolAddress.
constexpr size_t kNoallocScratchBytes = (size_t)32 << 20;
constexpr int kNoallocMaxDevices = 64;
static __device__ __align__(256) unsigned char noalloc_scratch[kNoallocScratchBytes];
void* noalloc_ptr[kNoallocMaxDevices] = {};  // device address per device ordinal, filled on first use
std::mutex noalloc_mutex;

// Device address of the current device's scratch array (NULL if the runtime cannot resolve it).
void* noalloc_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNoallocMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(noalloc_mutex);
  if (!noalloc_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(noalloc_scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    noalloc_ptr[dev] = ptr;
  }
  return noalloc_ptr[dev];
}

// Back-to-back matrix instructions on four independent accumulators per wave, nothing else: what the matrix
// pipeline of this chip sustains, for the benchmark's measured roofline.
__global__ __launch_bounds__(kThreads) void mfma_probe_kernel(int iters, float* sink) {
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, u32x4_t{0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
  const bf16x8_t b = __builtin_bit_cast(bf16x8_t, u32x4_t{0x3f803f80u, 0x3f803f80u + blockIdx.x, 0x3f803f80u, 0x3f803f80u});
  f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  const float s = c0[0] + c1[1] + c2[2] + c3[3];
  if (s == 12345.678f) sink[0] = s;  // never true for these operands; keeps the products alive
}

template <typename T, int D, typename... Args>
int fwd_dispatch(bool bias, Args... args) {
  return bias ? run_fwd<T, D, true>(args...) : run_fwd<T, D, false>(args...);
}
template <typename T, int D, typename... Args>
int bwd_dispatch(bool bias, Args... args) {
  return bias ? run_bwd<T, D, true>(args...) : run_bwd<T, D, false>(args...);
}

int fwd_checked(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const float* beta,
                const float* gamma, const float* slopes, void* O, float* tau, void* saved, size_t saved_bytes, uint64_t* stats,
                void* workspace, size_t workspace_bytes, hipStream_t st, void* const* phase_events) {
  int rc = check_params(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  if ((long long)p->B * p->H * p->Nq == 0) {
    for (int k = 0; k <= ENTMAX_FWD_NUM_PHASES; ++k) record(phase_events, k, st);
    return ENTMAX_ATTN_OK;
  }
  if (!Q || !O || !tau || !workspace) return ENTMAX_ATTN_INVALID_ARG;
  if (p->Nk > 0 && (!K || !V)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->scale_layout != 0 && (!beta || !gamma)) return ENTMAX_ATTN_INVALID_ARG;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(workspace) || misaligned(saved))
    return ENTMAX_ATTN_MISALIGNED;
  if ((reinterpret_cast<uintptr_t>(tau) & 3u) || (reinterpret_cast<uintptr_t>(stats) & 7u) ||
      (reinterpret_cast<uintptr_t>(slopes) & 3u))
    return ENTMAX_ATTN_MISALIGNED;
  if (workspace_bytes < workspace_bytes_of(p, 0)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  if (saved && saved_bytes < saved_bytes_of(p)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  Layout L = make_layout(p);
  char* ws = reinterpret_cast<char*>(workspace);
  char* sv = reinterpret_cast<char*>(saved);
  const bool bias = slopes != nullptr;
  if (p->dtype == ENTMAX_ATTN_BF16) {
    if (p->D == 64)
      return fwd_dispatch<bf16_t, 64>(bias, p, L, Q, K, V, beta, gamma, slopes, O, tau, sv, saved_bytes, stats, ws, st, phase_events);
    return fwd_dispatch<bf16_t, 128>(bias, p, L, Q, K, V, beta, gamma, slopes, O, tau, sv, saved_bytes, stats, ws, st, phase_events);
  }
  if (p->D == 64)
    return fwd_dispatch<float, 64>(bias, p, L, Q, K, V, beta, gamma, slopes, O, tau, sv, saved_bytes, stats, ws, st, phase_events);
  return fwd_dispatch<float, 128>(bias, p, L, Q, K, V, beta, gamma, slopes, O, tau, sv, saved_bytes, stats, ws, st, phase_events);
}

}  // namespace

extern "C" {

int entmax_attn_check_params(const entmax_attn_params* p) { return check_params(p); }

size_t entmax_attn_saved_bytes(const entmax_attn_params* p) { return saved_bytes_of(p); }

size_t entmax_attn_workspace_bytes(const entmax_attn_params* p, int is_bwd) { return workspace_bytes_of(p, is_bwd); }

const char* entmax_attn_strerror(int code) {
  switch (code) {
    case ENTMAX_ATTN_OK: return "success";
    case ENTMAX_ATTN_INVALID_ARG: return "invalid argument";
    case ENTMAX_ATTN_UNSUPPORTED_SHAPE: return "unsupported shape (D must be 64 or 128; sizes within index range)";
    case ENTMAX_ATTN_MISALIGNED: return "pointer or stride not 16-byte aligned";
    case ENTMAX_ATTN_WORKSPACE_TOO_SMALL: return "workspace or saved buffer too small";
    case ENTMAX_ATTN_LAUNCH_FAILED: return "kernel launch failed";
    case ENTMAX_ATTN_SCRATCH_LIMIT: return "problem needs more scratch than the built-in buffer of the no-allocation entry point";
    default: return "unknown status";
  }
}

int entmax_attn_fwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const float* beta,
                    const float* gamma, const float* alibi_slopes, void* O, float* tau, void* saved, size_t saved_bytes,
                    uint64_t* stats, void* workspace, size_t workspace_bytes, void* hip_stream,
                    void* const* phase_events) {
  return fwd_checked(p, Q, K, V, beta, gamma, alibi_slopes, O, tau, saved, saved_bytes, stats, workspace, workspace_bytes,
                     reinterpret_cast<hipStream_t>(hip_stream), phase_events);
}

int entmax_attn_mfma_probe(int iters, int blocks, float* sink, void* hip_stream) {
  if (iters <= 0 || blocks <= 0 || blocks > (1 << 20) || !sink) return ENTMAX_ATTN_INVALID_ARG;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3(kThreads), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), iters, sink);
  return launch_ok() ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED;
}

size_t entmax_attn_noalloc_scratch_bytes(void) { return kNoallocScratchBytes; }

int entmax_attn_noalloc_init(void) { return noalloc_scratch_ptr() ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED; }

int entmax_attn_fwd_noalloc(const entmax_attn_params* p, const void* Q, const void* K, const void* V,
                            const float* beta, const float* gamma, const float* alibi_slopes, void* O, float* tau,
                            uint64_t* stats, void* hip_stream) {
  int rc = check_params(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  if (workspace_bytes_of(p, 0) > kNoallocScratchBytes) return ENTMAX_ATTN_SCRATCH_LIMIT;
  void* ws = noalloc_scratch_ptr();
  if (!ws) return ENTMAX_ATTN_LAUNCH_FAILED;
  return fwd_checked(p, Q, K, V, beta, gamma, alibi_slopes, O, tau, nullptr, 0, stats, ws, kNoallocScratchBytes,
                     reinterpret_cast<hipStream_t>(hip_stream), nullptr);
}

int entmax_attn_bwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* tau, const void* saved, size_t saved_bytes, const float* beta,
                    const float* gamma, const float* alibi_slopes, void* dQ, void* dK, void* dV, float* dbeta,
                    float* dgamma, uint64_t* stats, void* workspace, size_t workspace_bytes, void* hip_stream,
                    void* const* phase_events) {
  (void)O;
  int rc = check_params(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if ((long long)p->B * p->H == 0 || (p->Nq == 0 && p->Nk == 0)) {
    for (int k = 0; k <= ENTMAX_BWD_NUM_PHASES; ++k) record(phase_events, k, st);
    return ENTMAX_ATTN_OK;
  }
  if (!workspace) return ENTMAX_ATTN_INVALID_ARG;
  if (p->Nq > 0 && (!Q || !dO || !tau || !dQ)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->Nk > 0 && (!K || !V || !dK || !dV)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->scale_layout != 0 && (!beta || !gamma || !dbeta || !dgamma)) return ENTMAX_ATTN_INVALID_ARG;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(dO) || misaligned(dQ) || misaligned(dK) ||
      misaligned(dV) || misaligned(workspace) || misaligned(saved))
    return ENTMAX_ATTN_MISALIGNED;
  if ((reinterpret_cast<uintptr_t>(tau) & 3u) || (reinterpret_cast<uintptr_t>(stats) & 7u)) return ENTMAX_ATTN_MISALIGNED;
  if (workspace_bytes < workspace_bytes_of(p, 1)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  if (saved && saved_bytes < saved_bytes_of(p)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  Layout L = make_layout(p);
  char* ws = reinterpret_cast<char*>(workspace);
  const char* sv = reinterpret_cast<const char*>(saved);
  const bool bias = alibi_slopes != nullptr;
  if (reinterpret_cast<uintptr_t>(alibi_slopes) & 3u) return ENTMAX_ATTN_MISALIGNED;
  if (p->dtype == ENTMAX_ATTN_BF16) {
    if (p->D == 64)
      return bwd_dispatch<bf16_t, 64>(bias, p, L, Q, K, V, dO, tau, sv, saved_bytes, beta, gamma, alibi_slopes, dQ, dK, dV, dbeta,
                                      dgamma, stats, ws, st, phase_events);
    return bwd_dispatch<bf16_t, 128>(bias, p, L, Q, K, V, dO, tau, sv, saved_bytes, beta, gamma, alibi_slopes, dQ, dK, dV, dbeta,
                                     dgamma, stats, ws, st, phase_events);
  }
  if (p->D == 64)
    return bwd_dispatch<float, 64>(bias, p, L, Q, K, V, dO, tau, sv, saved_bytes, beta, gamma, alibi_slopes, dQ, dK, dV, dbeta,
                                   dgamma, stats, ws, st, phase_events);
  return bwd_dispatch<float, 128>(bias, p, L, Q, K, V, dO, tau, sv, saved_bytes, beta, gamma, alibi_slopes, dQ, dK, dV, dbeta,
                                  dgamma, stats, ws, st, phase_events);
}

}  // extern "C"
