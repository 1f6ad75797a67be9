// Host side of the C ABI declared in include/entmax_attn.h: argument
// validation, workspace carving and kernel launches.  Nothing here allocates
// device memory or synchronises.
#include "entmax_attn.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include "bwd.hip.h"
#include "bwd_sparse.hip.h"
#include "decode.hip.h"
#include "fwd.hip.h"
#include "fwd_sparse.hip.h"
#include "transpose.hip.h"

using namespace entmax;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Layout {
  size_t esize;
  int npad_q, npad_k;
  int nqb, nkb;       // 128-row query / key blocks per head
  int nqg;            // 32-row query groups per head
  int mask_words;     // uint32 words covering the 32-key blocks of a head
  long long q_sb, q_sh, q_sn, kv_sb, kv_sh, kv_sn;
  // workspace offsets
  size_t off_vt, off_cand, off_flcnt, off_bounds, off_flags, off_kt, off_qt, off_dot, off_mu, off_crow, off_dscale, off_mask,
      off_jlist, off_lcnt, off_kcount, off_koffs, off_kcursor, off_csc_i, off_csc_pw, off_hflag, off_longkeys, off_fcells, off_bcells, sv_cand, sv_lcnt, sv_flags, sv_kcand, total_saved, total_fwd,
      total_bwd;
  size_t off_dec_cmax;  // decode kernels: score rows at offset 0, then the chunk maxima
  int dec_nks, dec_nchunks, dec_chunk;
};

int check(const entmax_attn_params* p) {
  if (!p) return ENTMAX_ATTN_INVALID_ARG;
  if (p->B < 0 || p->H < 0 || p->Nq < 0 || p->Nk < 0) return ENTMAX_ATTN_INVALID_ARG;
  if (p->dtype != ENTMAX_ATTN_BF16 && p->dtype != ENTMAX_ATTN_FP32) return ENTMAX_ATTN_INVALID_ARG;
  if (p->causal != 0 && p->causal != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (p->scale_layout < 0 || p->scale_layout > 2) return ENTMAX_ATTN_INVALID_ARG;
  if (p->logn_mode != 0 && p->logn_mode != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (p->path != 0 && p->path != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (!(p->alpha > 1.0f) || !(p->alpha <= 2.0f)) return ENTMAX_ATTN_INVALID_ARG;
  if (!isfinite(p->delta)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->D != 64 && p->D != 128) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (p->Nq > (1 << 22) || p->Nk > (1 << 22)) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;  // 32-bit offsets inside a tile
  long long bh = (long long)p->B * p->H;
  if (bh * (long long)ceil_div(p->Nq > p->Nk ? p->Nq : p->Nk, 32) > 0x7fffffffLL) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (bh > 65535) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  const int64_t s[6] = {p->q_stride_b, p->q_stride_h, p->q_stride_n, p->kv_stride_b, p->kv_stride_h, p->kv_stride_n};
  bool q_zero = s[0] == 0 && s[1] == 0 && s[2] == 0, kv_zero = s[3] == 0 && s[4] == 0 && s[5] == 0;
  size_t es = p->dtype == ENTMAX_ATTN_BF16 ? 2 : 4;
  for (int k = 0; k < 6; ++k) {
    if (s[k] < 0) return ENTMAX_ATTN_INVALID_ARG;
    if ((s[k] * (int64_t)es) % 16 != 0) return ENTMAX_ATTN_MISALIGNED;
  }
  if (s[2] * (int64_t)es > (1 << 24) || s[5] * (int64_t)es > (1 << 24)) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (!q_zero && s[2] < p->D) return ENTMAX_ATTN_INVALID_ARG;
  if (!kv_zero && s[5] < p->D) return ENTMAX_ATTN_INVALID_ARG;
  return ENTMAX_ATTN_OK;
}

Layout make_layout(const entmax_attn_params* p) {
  Layout L;
  L.esize = p->dtype == ENTMAX_ATTN_BF16 ? 2 : 4;
  L.npad_q = ceil_div(p->Nq, 128) * 128;
  L.npad_k = ceil_div(p->Nk, 128) * 128;
  L.nqb = ceil_div(p->Nq, kBlockRows);
  L.nkb = ceil_div(p->Nk, kBlockRows);
  L.nqg = ceil_div(p->Nq, 32);
  L.mask_words = ceil_div(ceil_div(p->Nk, 32), 32);
  if (L.mask_words < 1) L.mask_words = 1;
  bool q_zero = p->q_stride_b == 0 && p->q_stride_h == 0 && p->q_stride_n == 0;
  bool kv_zero = p->kv_stride_b == 0 && p->kv_stride_h == 0 && p->kv_stride_n == 0;
  L.q_sn = q_zero ? p->D : p->q_stride_n;
  L.q_sh = q_zero ? (long long)p->Nq * p->D : p->q_stride_h;
  L.q_sb = q_zero ? (long long)p->H * p->Nq * p->D : p->q_stride_b;
  L.kv_sn = kv_zero ? p->D : p->kv_stride_n;
  L.kv_sh = kv_zero ? (long long)p->Nk * p->D : p->kv_stride_h;
  L.kv_sb = kv_zero ? (long long)p->H * p->Nk * p->D : p->kv_stride_b;
  size_t bh = (size_t)p->B * p->H;
  size_t kt_bytes = align_up(bh * p->D * (size_t)L.npad_k * L.esize);
  size_t qt_bytes = align_up(bh * p->D * (size_t)L.npad_q * L.esize);
  size_t row_bytes = align_up(bh * (size_t)p->Nq * sizeof(float));
  size_t mask_bytes = align_up(bh * (size_t)L.nqg * L.mask_words * sizeof(uint32_t));
  // forward: V^T copy | candidate lists | per-workgroup and per-head fallback flags
  L.off_vt = 0;
  L.off_cand = kt_bytes;
  size_t cand_bytes = align_up(bh * (size_t)L.nqb * kThreads * kCandCap * sizeof(uint2));  // one list per lane of the list grid
  // the `saved` buffer: the same three arrays, for the backward
  L.sv_cand = 0;
  L.sv_lcnt = cand_bytes;
  L.sv_flags = L.sv_lcnt + align_up(bh * (size_t)p->Nq * 2 * sizeof(int));
  L.sv_kcand = L.sv_flags + align_up(bh * (size_t)L.nqb * sizeof(int));
  L.total_saved = L.sv_kcand + align_up(bh * (size_t)p->Nk * sizeof(int));
  L.off_flcnt = L.off_cand + cand_bytes;
  L.off_bounds = L.off_flcnt + align_up(bh * (size_t)p->Nq * 2 * sizeof(int));
  L.off_flags = L.off_bounds + align_up(bh * (size_t)p->Nq * sizeof(float2));
  L.off_fcells = L.off_flags + align_up((bh * (size_t)L.nqb + bh + 1) * sizeof(int));
  const size_t list_groups = bh * (size_t)((L.nqb + 1) / 2);  // workgroups of the list sweeps
  L.total_fwd = L.off_fcells + align_up(list_groups * CellBuf<kCandCap>::kBytesPerWorkgroup);
  // the decode kernels' score rows take the place of everything above
  if (decode_shape(p->Nq, p->Nk)) {
    L.dec_nks = (p->Nk + 3) / 4 * 4;
    L.dec_chunk = 512;  // 64 to 128 KB of K per workgroup; 256 to 2048 keys measured alike at Nk = 32768
    L.dec_nchunks = ceil_div(p->Nk, L.dec_chunk);
    L.off_dec_cmax = align_up(bh * (size_t)p->Nq * L.dec_nks * sizeof(float));
    const size_t dec_bytes = L.off_dec_cmax + align_up(bh * (size_t)p->Nq * L.dec_nchunks * sizeof(float));
    if (dec_bytes > L.total_fwd) L.total_fwd = dec_bytes;
  }
  size_t o = 0;
  L.off_kt = o;
  o += kt_bytes;
  L.off_qt = o;
  o += qt_bytes;
  L.off_dot = o;
  o += qt_bytes;
  L.off_mu = o;
  o += row_bytes;
  L.off_crow = o;
  o += row_bytes;
  L.off_dscale = o;
  o += row_bytes;
  L.off_mask = o;
  o += mask_bytes;
  // support-list backward
  size_t rows = bh * (size_t)p->Nq;
  L.off_jlist = o;
  o += align_up(bh * (size_t)L.nqb * kThreads * kBwdCap * sizeof(uint2));
  L.off_lcnt = o;
  o += align_up(rows * 2 * sizeof(int));
  size_t key_bytes = align_up(bh * (size_t)p->Nk * sizeof(int));
  L.off_kcount = o;
  o += key_bytes;
  L.off_koffs = o;
  o += key_bytes;
  L.off_kcursor = o;
  o += key_bytes;
  L.off_csc_i = o;
  o += align_up(rows * 2 * kBwdCap * sizeof(int));
  L.off_csc_pw = o;
  o += align_up(rows * 2 * kBwdCap * sizeof(float2));
  L.off_hflag = o;
  o += align_up((bh * (size_t)L.nqb + bh + kLongCountOffset + 1) * sizeof(int));  // block flags, head flags, counter
  L.off_longkeys = o;
  o += key_bytes;
  L.off_bcells = o;
  o += align_up(list_groups * CellBuf<kBwdCap>::kBytesPerWorkgroup);
  L.total_bwd = o;
  return L;
}

Geom make_geom(const entmax_attn_params* p, const Layout& L, const float* beta, const float* gamma) {
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
bool launch_transposes(const TransposeJobs& jobs, int njobs, int B, int H, hipStream_t st, const int* head_flag = nullptr) {
  int npad = 0;
  for (int k = 0; k < njobs; ++k) npad = jobs.job[k].npad > npad ? jobs.job[k].npad : npad;
  if (npad == 0) return true;
  dim3 grid((unsigned)(npad / 64), (unsigned)(B * H), (unsigned)njobs);
  hipLaunchKernelGGL((transpose_perm_kernel<T, D>), grid, dim3(kThreads), 0, st, jobs, H, head_flag);
  return launch_ok();
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

template <typename T, int D, int AM>
bool launch_fwd_main(const FwdArgs& a, int nblocks, hipStream_t st) {
  size_t smem = 4 * (size_t)QCtx<T, D, FwdTile<T>::value>::kTileBytes + (size_t)(kWaves + 1) * a.mask_words * 4 + 64;
  auto kern = fwd_kernel<T, D, AM>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) !=
      hipSuccess)
    return false;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  return launch_ok();
}

template <typename T, int D>
bool launch_fwd_am(const FwdArgs& a, int am, int nblocks, hipStream_t st) {
  switch (am) {
    case 1: return launch_fwd_main<T, D, 1>(a, nblocks, st);
    case 2: return launch_fwd_main<T, D, 2>(a, nblocks, st);
    case 3: return launch_fwd_main<T, D, 3>(a, nblocks, st);
    default: return launch_fwd_main<T, D, 0>(a, nblocks, st);
  }
}

template <typename T, int D, int AM>
bool launch_fwd_sparse(const FwdSparseArgs& a, int nblocks, hipStream_t st, void* const* ev) {
  size_t smem = 2 * (size_t)QCtx<T, D, FwdTile<T>::value>::kTileBytes + 64;
  hipLaunchKernelGGL((fwd_lists_kernel<T, D, AM>), dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
  hipLaunchKernelGGL((fwd_finish_kernel<T, D, AM>), dim3((unsigned)(a.g.B * a.g.H * a.nqb)), dim3(kThreads), 0, st, a);
  return launch_ok();
}

template <typename T, int D>
bool launch_fwd_sparse_am(const FwdSparseArgs& a, int am, int nblocks, hipStream_t st, void* const* ev) {
  switch (am) {
    case 1: return launch_fwd_sparse<T, D, 1>(a, nblocks, st, ev);
    case 2: return launch_fwd_sparse<T, D, 2>(a, nblocks, st, ev);
    case 3: return launch_fwd_sparse<T, D, 3>(a, nblocks, st, ev);
    default: return launch_fwd_sparse<T, D, 0>(a, nblocks, st, ev);
  }
}

template <typename T, int D>
bool launch_decode(const DecodeArgs& a, int am, hipStream_t st, void* const* ev) {
  const Geom& g = a.g;
  hipLaunchKernelGGL((decode_scores_kernel<T, D>), dim3((unsigned)a.nchunks, (unsigned)(g.B * g.H)),
                     dim3(kThreads), decode_scores_lds(g.Nq, D, sizeof(T)), st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
  const dim3 grid((unsigned)(g.B * g.H * g.Nq)), block(kDecodeSolveThreads);
  switch (am) {
    case 1: hipLaunchKernelGGL((decode_solve_kernel<T, D, 1>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((decode_solve_kernel<T, D, 2>), grid, block, 0, st, a); break;
    case 3: hipLaunchKernelGGL((decode_solve_kernel<T, D, 3>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((decode_solve_kernel<T, D, 0>), grid, block, 0, st, a); break;
  }
  return launch_ok();
}

template <typename T, int D>
int run_fwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V,
            const float* beta, const float* gamma, void* O, float* tau, char* saved, uint64_t* stats, char* ws,
            hipStream_t st, void* const* ev) {
  record(ev, 0, st);
  if (p->Nk == 0) {
    bool ok = zero_rows<T>(O, L.q_sb, L.q_sh, L.q_sn, p->B, p->H, p->Nq, p->D, st) &&
              zero_words(tau, (size_t)p->B * p->H * p->Nq * 4, st);
    for (int k = 1; k <= ENTMAX_FWD_NUM_PHASES; ++k) record(ev, k, st);
    return ok ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED;
  }
  if (p->path == 0 && decode_shape(p->Nq, p->Nk)) {
    // a few query rows against the whole key sequence: split the keys over the chip
    if (p->Nq > 0 && p->B * p->H > 0) {
      // no lists for the backward: every block belongs to its tiled kernels
      if (saved && !fill_words(saved + L.sv_flags, (size_t)p->B * p->H * L.nqb * sizeof(int), 1u, st))
        return ENTMAX_ATTN_LAUNCH_FAILED;
      record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
      DecodeArgs da;
      da.g = make_geom(p, L, beta, gamma);
      da.Q = Q;
      da.K = K;
      da.V = V;
      da.O = O;
      da.tau = tau;
      da.scores = reinterpret_cast<float*>(ws);
      da.cmax = reinterpret_cast<float*>(ws + L.off_dec_cmax);
      da.nks = L.dec_nks;
      da.nchunks = L.dec_nchunks;
      da.chunk = L.dec_chunk;
      if (!launch_decode<T, D>(da, alpha_mode(p->alpha), st, ev)) return ENTMAX_ATTN_LAUNCH_FAILED;
    } else {
      record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
      record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
    }
    for (int k = ENTMAX_FWD_PHASE_FINISH; k < ENTMAX_FWD_NUM_PHASES; ++k) record(ev, k + 1, st);
    return ENTMAX_ATTN_OK;
  }
  void* Vt = ws + L.off_vt;
  // with a `saved` buffer the lists, their lengths and the block flags are written there
  int* dense_flag = reinterpret_cast<int*>(saved ? saved + L.sv_flags : ws + L.off_flags);
  int* head_flag = reinterpret_cast<int*>(ws + L.off_flags) + (size_t)p->B * p->H * L.nqb;
  const int nblocks = p->B * p->H * ((L.nqb + 1) / 2);  // workgroups take query blocks in pairs
  const bool lists = p->path == 0;
  if (lists) {
    FwdSparseArgs sa;
    sa.g = make_geom(p, L, beta, gamma);
    sa.Q = Q;
    sa.K = K;
    sa.V = V;
    sa.O = O;
    sa.tau = tau;
    sa.cand = reinterpret_cast<uint2*>(saved ? saved + L.sv_cand : ws + L.off_cand);
    sa.cells = ws + L.off_fcells;
    sa.lcnt = reinterpret_cast<int*>(saved ? saved + L.sv_lcnt : ws + L.off_flcnt);
    sa.kcand = saved ? reinterpret_cast<int*>(saved + L.sv_kcand) : nullptr;
    if (sa.kcand && !zero_words(sa.kcand, (size_t)p->B * p->H * p->Nk * sizeof(int), st)) return ENTMAX_ATTN_LAUNCH_FAILED;
    record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
    sa.bounds = reinterpret_cast<float2*>(ws + L.off_bounds);
    sa.dense_flag = dense_flag;
    sa.head_flag = head_flag;
    sa.stats = reinterpret_cast<unsigned long long*>(stats);
    sa.nqb = L.nqb;
    if (!launch_fwd_sparse_am<T, D>(sa, alpha_mode(p->alpha), nblocks, st, ev)) return ENTMAX_ATTN_LAUNCH_FAILED;
  } else {
    // no lists: tell the backward that every block belongs to its tiled kernels
    if (saved && !fill_words(dense_flag, (size_t)p->B * p->H * L.nqb * sizeof(int), 1u, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
    record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
    record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
  }
  record(ev, ENTMAX_FWD_PHASE_FINISH + 1, st);
  {
    TransposeJobs jobs{};
    jobs.job[0] = transpose_job(V, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, Vt);
    if (!launch_transposes<T, D>(jobs, 1, p->B, p->H, st, lists ? head_flag : nullptr)) return ENTMAX_ATTN_LAUNCH_FAILED;
  }
  record(ev, ENTMAX_FWD_PHASE_TRANSPOSE + 1, st);
  FwdArgs a;
  a.g = make_geom(p, L, beta, gamma);
  a.Q = Q;
  a.K = K;
  a.Vt = Vt;
  a.O = O;
  a.tau = tau;
  a.stats = reinterpret_cast<unsigned long long*>(stats);
  a.nqb = L.nqb;
  a.mask_words = L.mask_words;
  a.dense_flag = lists ? dense_flag : nullptr;
  a.head_flag = lists ? head_flag : nullptr;
  if (!launch_fwd_am<T, D>(a, alpha_mode(p->alpha), nblocks, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
  record(ev, ENTMAX_FWD_PHASE_TILED + 1, st);
  return ENTMAX_ATTN_OK;
}

template <typename T, int D, int AM>
bool launch_bwd_kernels(const BwdArgs& a, const Layout& L, int B, int H, hipStream_t st, void* const* ev) {
  size_t smem_mask = 2 * (size_t)QCtx<T, D, MaskTile<T>::value>::kTileBytes + (size_t)(kWaves + 1) * a.mask_words * 4 + 64;
  size_t smem_dq = 6 * (size_t)QCtx<T, D>::kTileBytes + (size_t)(kWaves + 1) * a.mask_words * 4 + kWaves * 64 * 4 + 64;
  size_t smem_dkv = 8 * (size_t)QCtx<T, D>::kTileBytes + 2 * 4 * (size_t)QCtx<T, D>::KT * 4 + (size_t)a.nqg + 64;
  auto k_mask = bwd_mask_kernel<T, D, AM>;
  auto k_dq = bwd_dq_kernel<T, D, AM>;
  auto k_dkv = bwd_dkv_kernel<T, D, AM>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_dq), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)smem_dq) != hipSuccess)
    return false;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_dkv), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)smem_dkv) != hipSuccess)
    return false;
  hipLaunchKernelGGL(k_mask, dim3((unsigned)(B * H * ((L.nqb + 1) / 2))), dim3(kThreads), smem_mask, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_MASK + 1, st);
  hipLaunchKernelGGL(k_dq, dim3((unsigned)(B * H * L.nqb)), dim3(kThreads), smem_dq, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_DQ + 1, st);
  hipLaunchKernelGGL(k_dkv, dim3((unsigned)(B * H * L.nkb)), dim3(kThreads), smem_dkv, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_DKV + 1, st);
  return true;
}

template <typename T, int D, int AM>
bool launch_bwd_rows(const BwdSparseArgs& a, int nblocks, hipStream_t st, void* const* ev, bool from_saved) {
  const dim3 row_grid((unsigned)(a.g.B * a.g.H * a.nqb));
  if (from_saved) {
    hipLaunchKernelGGL(bwd_prepare_kernel<D>, row_grid, dim3(kThreads), 0, st, a);
  } else {
    size_t smem = 2 * (size_t)QCtx<T, D, FwdTile<T>::value>::kTileBytes + 64;
    hipLaunchKernelGGL((bwd_lists_kernel<T, D, AM>), dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  }
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_LISTS + 1, st);
  {
    // per-key counters in LDS when a head's keys fit beside the scan arrays
    const size_t scan_bytes = 2 * (size_t)kOffsThreads * sizeof(int);
    const bool use_lds = !from_saved && scan_bytes + (size_t)a.g.Nk * sizeof(int) <= 150 * 1024;
    const size_t smem = scan_bytes + (use_lds ? (size_t)a.g.Nk * sizeof(int) : 0);
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(key_offsets_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)smem) != hipSuccess)
      return false;
    hipLaunchKernelGGL(key_offsets_kernel, dim3((unsigned)(a.g.B * a.g.H)), dim3(kOffsThreads), smem, st, a,
                       from_saved ? kCandCap : kBwdCap, use_lds ? 1 : 0, from_saved ? 1 : 0);
    if (!launch_ok()) return false;
  }
  if (from_saved)
    hipLaunchKernelGGL((bwd_rows_kernel<T, D, AM, kCandCap>), row_grid, dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL((bwd_rows_kernel<T, D, AM, kBwdCap>), row_grid, dim3(kThreads), 0, st, a);
  return launch_ok();
}

template <typename T, int D>
bool launch_bwd_rows_am(const BwdSparseArgs& a, int am, int nblocks, hipStream_t st, void* const* ev, bool from_saved) {
  switch (am) {
    case 1: return launch_bwd_rows<T, D, 1>(a, nblocks, st, ev, from_saved);
    case 2: return launch_bwd_rows<T, D, 2>(a, nblocks, st, ev, from_saved);
    case 3: return launch_bwd_rows<T, D, 3>(a, nblocks, st, ev, from_saved);
    default: return launch_bwd_rows<T, D, 0>(a, nblocks, st, ev, from_saved);
  }
}

template <typename T, int D>
int run_bwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V, const void* dO,
            const float* tau, const char* saved, const float* beta, const float* gamma, void* dQ, void* dK, void* dV,
            float* dbeta, float* dgamma, uint64_t* stats, char* ws, hipStream_t st, void* const* ev) {
  record(ev, 0, st);
  const int B = p->B, H = p->H;
  Geom g = make_geom(p, L, beta, gamma);
  float* dscale = reinterpret_cast<float*>(ws + L.off_dscale);
  bool ok = true;
  if (p->Nk == 0 || p->Nq == 0) {
    ok = ok && zero_rows<T>(dQ, L.q_sb, L.q_sh, L.q_sn, B, H, p->Nq, p->D, st);
    ok = ok && zero_rows<T>(dK, L.kv_sb, L.kv_sh, L.kv_sn, B, H, p->Nk, p->D, st);
    ok = ok && zero_rows<T>(dV, L.kv_sb, L.kv_sh, L.kv_sn, B, H, p->Nk, p->D, st);
    ok = ok && zero_words(dscale, (size_t)B * H * p->Nq * 4, st);
    for (int k = 1; k <= ENTMAX_BWD_PHASE_KEYS + 1; ++k) record(ev, k, st);
  } else {
    const bool lists = p->path == 0;
    int* block_flag = reinterpret_cast<int*>(ws + L.off_hflag);
    int* head_flag = block_flag + (size_t)B * H * L.nqb;
    BwdSparseArgs sa;
    if (lists) {
      sa.g = g;
      sa.Q = Q;
      sa.K = K;
      sa.V = V;
      sa.dO = dO;
      sa.tau = tau;
      sa.dQ = dQ;
      sa.dK = dK;
      sa.dV = dV;
      sa.dscale = dscale;
      sa.jlist = reinterpret_cast<uint2*>(ws + L.off_jlist);
      sa.cells = ws + L.off_bcells;
      sa.kcursor = reinterpret_cast<int*>(ws + L.off_kcursor);
      sa.lcnt = reinterpret_cast<int*>(ws + L.off_lcnt);
      sa.src_list = saved ? reinterpret_cast<const uint2*>(saved + L.sv_cand) : sa.jlist;
      sa.src_lcnt = saved ? reinterpret_cast<const int*>(saved + L.sv_lcnt) : nullptr;
      sa.src_dense = saved ? reinterpret_cast<const int*>(saved + L.sv_flags) : nullptr;
      // with the forward's lists come the forward's per-key counts (read only here)
      sa.kcount = saved ? reinterpret_cast<int*>(const_cast<char*>(saved) + L.sv_kcand) : reinterpret_cast<int*>(ws + L.off_kcount);
      sa.koffs = reinterpret_cast<int*>(ws + L.off_koffs);
      sa.csc_i = reinterpret_cast<int*>(ws + L.off_csc_i);
      sa.csc_pw = reinterpret_cast<float2*>(ws + L.off_csc_pw);
      sa.block_flag = block_flag;
      sa.head_flag = head_flag;
      sa.long_keys = reinterpret_cast<int*>(ws + L.off_longkeys);
      sa.stats = reinterpret_cast<unsigned long long*>(stats);
      sa.nqb = L.nqb;
      sa.dbeta = dbeta;
      sa.dgamma = dgamma;
      sa.scale_heads = p->scale_layout == 1 ? H : 0;
      ok = ok && launch_bwd_rows_am<T, D>(sa, alpha_mode(p->alpha), B * H * ((L.nqb + 1) / 2), st, ev, saved != nullptr);
      if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
    } else {
      record(ev, ENTMAX_BWD_PHASE_LISTS + 1, st);
    }
    record(ev, ENTMAX_BWD_PHASE_ROWS + 1, st);
    const int* hf = lists ? head_flag : nullptr;
    void* Kt = ws + L.off_kt;
    void* Qt = ws + L.off_qt;
    void* dOt = ws + L.off_dot;
    {
      TransposeJobs jobs{};
      jobs.job[0] = transpose_job(K, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, Kt);
      jobs.job[1] = transpose_job(Q, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, Qt);
      jobs.job[2] = transpose_job(dO, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, dOt);
      ok = ok && launch_transposes<T, D>(jobs, 3, B, H, st, hf);
    }
    if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
    record(ev, ENTMAX_BWD_PHASE_TRANSPOSE + 1, st);
    BwdArgs a;
    a.g = g;
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.dO = dO;
    a.Kt = Kt;
    a.Qt = Qt;
    a.dOt = dOt;
    a.tau = tau;
    a.dQ = dQ;
    a.dK = dK;
    a.dV = dV;
    a.mu = reinterpret_cast<float*>(ws + L.off_mu);
    a.crow = reinterpret_cast<float*>(ws + L.off_crow);
    a.dscale = dscale;
    a.mask = reinterpret_cast<uint32_t*>(ws + L.off_mask);
    a.stats = reinterpret_cast<unsigned long long*>(stats);
    a.head_flag = hf;
    a.nqb = L.nqb;
    a.nkb = L.nkb;
    a.nqg = L.nqg;
    a.mask_words = L.mask_words;
    switch (alpha_mode(p->alpha)) {
      case 1: ok = launch_bwd_kernels<T, D, 1>(a, L, B, H, st, ev); break;
      case 2: ok = launch_bwd_kernels<T, D, 2>(a, L, B, H, st, ev); break;
      case 3: ok = launch_bwd_kernels<T, D, 3>(a, L, B, H, st, ev); break;
      default: ok = launch_bwd_kernels<T, D, 0>(a, L, B, H, st, ev); break;
    }
    if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
    if (lists) {
      long long keys = (long long)B * H * p->Nk;
      hipLaunchKernelGGL((bwd_keys_kernel<T, D>),
                         dim3((unsigned)(kLongKeyBlocks + sa.scale_heads + (keys + kKeysPerBlock - 1) / kKeysPerBlock)),
                         dim3(kThreads), 0, st, sa);
      ok = ok && launch_ok();
    }
    record(ev, ENTMAX_BWD_PHASE_KEYS + 1, st);
  }
  if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
  if (p->scale_layout == 1 && !(p->path == 0 && p->Nk > 0 && p->Nq > 0)) {  // (else done inside the keys launch)
    hipLaunchKernelGGL(scale_grad_head_kernel, dim3((unsigned)H), dim3(kScaleGradThreads), 0, st, g, dscale, dbeta,
                       dgamma);
    ok = launch_ok();
  } else if (p->scale_layout == 2) {
    long long rows = (long long)B * H * p->Nq;
    if (rows > 0) {
      hipLaunchKernelGGL(scale_grad_query_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, g, dscale,
                         dbeta, dgamma);
      ok = launch_ok();
    }
  }
  record(ev, ENTMAX_BWD_PHASE_SCALE_GRAD + 1, st);
  return ok ? ENTMAX_ATTN_OK : ENTMAX_ATTN_LAUNCH_FAILED;
}

}  // namespace

extern "C" {

int entmax_attn_check_params(const entmax_attn_params* p) { return check(p); }

size_t entmax_attn_saved_bytes(const entmax_attn_params* p) {
  if (check(p) != ENTMAX_ATTN_OK) return 0;
  Layout L = make_layout(p);
  return L.total_saved < kAlign ? kAlign : L.total_saved;
}

size_t entmax_attn_workspace_bytes(const entmax_attn_params* p, int is_bwd) {
  if (check(p) != ENTMAX_ATTN_OK) return 0;
  Layout L = make_layout(p);
  size_t n = is_bwd ? L.total_bwd : L.total_fwd;
  return n < kAlign ? kAlign : n;
}

const char* entmax_attn_strerror(int code) {
  switch (code) {
    case ENTMAX_ATTN_OK: return "success";
    case ENTMAX_ATTN_INVALID_ARG: return "invalid argument";
    case ENTMAX_ATTN_UNSUPPORTED_SHAPE: return "unsupported shape (D must be 64 or 128; sizes within index range)";
    case ENTMAX_ATTN_MISALIGNED: return "pointer or stride not 16-byte aligned";
    case ENTMAX_ATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case ENTMAX_ATTN_LAUNCH_FAILED: return "kernel launch failed";
    default: return "unknown status";
  }
}

int entmax_attn_fwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const float* beta,
                    const float* gamma, void* O, float* tau, void* saved, uint64_t* stats, void* workspace,
                    size_t workspace_bytes, void* hip_stream, void* const* phase_events) {
  int rc = check(p);
  if (rc != ENTMAX_ATTN_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if ((long long)p->B * p->H * p->Nq == 0) {
    for (int k = 0; k <= ENTMAX_FWD_NUM_PHASES; ++k) record(phase_events, k, st);
    return ENTMAX_ATTN_OK;
  }
  if (!Q || !O || !tau || !workspace) return ENTMAX_ATTN_INVALID_ARG;
  if (p->Nk > 0 && (!K || !V)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->scale_layout != 0 && (!beta || !gamma)) return ENTMAX_ATTN_INVALID_ARG;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(workspace) || misaligned(saved))
    return ENTMAX_ATTN_MISALIGNED;
  if ((reinterpret_cast<uintptr_t>(tau) & 3u) || (reinterpret_cast<uintptr_t>(stats) & 7u)) return ENTMAX_ATTN_MISALIGNED;
  if (workspace_bytes < entmax_attn_workspace_bytes(p, 0)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  Layout L = make_layout(p);
  char* ws = reinterpret_cast<char*>(workspace);
  char* sv = reinterpret_cast<char*>(saved);
  if (p->dtype == ENTMAX_ATTN_BF16) {
    if (p->D == 64) return run_fwd<bf16_t, 64>(p, L, Q, K, V, beta, gamma, O, tau, sv, stats, ws, st, phase_events);
    return run_fwd<bf16_t, 128>(p, L, Q, K, V, beta, gamma, O, tau, sv, stats, ws, st, phase_events);
  }
  if (p->D == 64) return run_fwd<float, 64>(p, L, Q, K, V, beta, gamma, O, tau, sv, stats, ws, st, phase_events);
  return run_fwd<float, 128>(p, L, Q, K, V, beta, gamma, O, tau, sv, stats, ws, st, phase_events);
}

int entmax_attn_bwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* tau, const void* saved, const float* beta, const float* gamma,
                    void* dQ, void* dK, void* dV, float* dbeta, float* dgamma, uint64_t* stats, void* workspace,
                    size_t workspace_bytes, void* hip_stream, void* const* phase_events) {
  (void)O;
  int rc = check(p);
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
  if (workspace_bytes < entmax_attn_workspace_bytes(p, 1)) return ENTMAX_ATTN_WORKSPACE_TOO_SMALL;
  Layout L = make_layout(p);
  char* ws = reinterpret_cast<char*>(workspace);
  const char* sv = reinterpret_cast<const char*>(saved);
  if (p->dtype == ENTMAX_ATTN_BF16) {
    if (p->D == 64)
      return run_bwd<bf16_t, 64>(p, L, Q, K, V, dO, tau, sv, beta, gamma, dQ, dK, dV, dbeta, dgamma, stats, ws, st,
                                 phase_events);
    return run_bwd<bf16_t, 128>(p, L, Q, K, V, dO, tau, sv, beta, gamma, dQ, dK, dV, dbeta, dgamma, stats, ws, st,
                                phase_events);
  }
  if (p->D == 64)
    return run_bwd<float, 64>(p, L, Q, K, V, dO, tau, sv, beta, gamma, dQ, dK, dV, dbeta, dgamma, stats, ws, st,
                              phase_events);
  return run_bwd<float, 128>(p, L, Q, K, V, dO, tau, sv, beta, gamma, dQ, dK, dV, dbeta, dgamma, stats, ws, st,
                             phase_events);
}

}  // extern "C"
