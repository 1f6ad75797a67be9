// Backward launcher: support-list kernels per head with the tiled kernels as fallback.
#pragma once
#include "bwd.hip.h"
#include "bwd_sparse.hip.h"
#include "key_norm.hip.h"
#include "launch.hip.h"

namespace entmax {
namespace {

template <typename T, int D, int AM, bool BIAS>
bool launch_bwd_kernels(const BwdArgs& a_in, const Layout& L, int B, int H, hipStream_t st, void* const* ev) {
  BwdArgs a = a_in;
  // workgroups one XCD (32 CUs, 160 KB of LDS each) holds at a time: the registers allow two per CU
  auto xcd_room = [](size_t smem) { return 32 * (int)(smem * 2 <= 160 * 1024 ? 2 : 1); };
  size_t smem_dq = 6 * (size_t)QCtx<T, D>::kTileBytes + (size_t)(kWaves + 1) * a.mask_words * 4 + kWaves * 64 * 4 + 64;
  size_t smem_dkv = 8 * (size_t)QCtx<T, D>::kTileBytes + 2 * 4 * (size_t)QCtx<T, D>::KT * 4 + (size_t)a.nqg + 64;
  constexpr auto k_dq = bwd_dq_kernel<T, D, AM, BIAS>;
  constexpr auto k_dkv = bwd_dkv_kernel<T, D, AM>;
  if (!ensure_dynamic_lds<k_dq>(smem_dq) || !ensure_dynamic_lds<k_dkv>(smem_dkv))
    return false;
  record(ev, ENTMAX_BWD_PHASE_MASK + 1, st);
  a.xcd_room = xcd_room(smem_dq);
  hipLaunchKernelGGL(k_dq, dim3((unsigned)(B * H * L.nqb)), dim3(kThreads), smem_dq, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_DQ + 1, st);
  a.xcd_room = xcd_room(smem_dkv);
  hipLaunchKernelGGL(k_dkv, dim3((unsigned)(B * H * L.nkb)), dim3(kThreads), smem_dkv, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_BWD_PHASE_DKV + 1, st);
  return true;
}

template <typename T, int D, int AM, bool BIAS>
bool launch_bwd_rows(const BwdSparseArgs& a, int nblocks, hipStream_t st, void* const* ev, bool from_saved) {
  const dim3 row_grid((unsigned)(a.g.B * a.g.H * a.nqb * RowsCfg<D>::kFH + a.ride.workgroups()));
  if (!from_saved) {
    // no lists from the forward: one Q K^T sweep at tau rebuilds the supports
    size_t smem = ListCfg<T, D>::kLdsBytes;
    hipLaunchKernelGGL((bwd_lists_kernel<T, D, AM, BIAS>), dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
    if (!launch_ok()) return false;
  }
  record(ev, ENTMAX_BWD_PHASE_LISTS + 1, st);
  {
    // per-key counters in LDS when a head's keys fit beside the scan arrays
    const size_t scan_bytes = 2 * (size_t)kOffsThreads * sizeof(int);
    const bool use_lds = !a.precount && scan_bytes + (size_t)a.g.Nk * sizeof(int) <= 150 * 1024;
    const size_t smem = scan_bytes + (use_lds ? (size_t)a.g.Nk * sizeof(int) : 0);
    if (!ensure_dynamic_lds<key_offsets_kernel>(smem)) return false;
    hipLaunchKernelGGL(key_offsets_kernel, dim3((unsigned)(a.g.B * a.g.H)), dim3(kOffsThreads), smem, st, a,
                       use_lds ? 1 : 0);
    if (!launch_ok()) return false;
  }
  hipLaunchKernelGGL((bwd_rows_kernel<T, D, AM>), row_grid, dim3(kThreads), 0, st, a);
  return launch_ok();
}

template <typename T, int D, bool BIAS>
bool launch_bwd_rows_am(const BwdSparseArgs& a, int am, int nblocks, hipStream_t st, void* const* ev, bool from_saved) {
  switch (am) {
    case 1: return launch_bwd_rows<T, D, 1, BIAS>(a, nblocks, st, ev, from_saved);
    case 2: return launch_bwd_rows<T, D, 2, BIAS>(a, nblocks, st, ev, from_saved);
    case 3: return launch_bwd_rows<T, D, 3, BIAS>(a, nblocks, st, ev, from_saved);
    default: return launch_bwd_rows<T, D, 0, BIAS>(a, nblocks, st, ev, from_saved);
  }
}

}  // namespace

template <typename T, int D, bool BIAS>
int run_bwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V, const void* dO,
            const float* tau, const char* saved, size_t saved_bytes, const float* beta, const float* gamma,
            const float* slopes, void* dQ, void* dK, void* dV, float* dbeta, float* dgamma, uint64_t* stats, char* ws,
            hipStream_t st, void* const* ev) {
  record(ev, 0, st);
  const int B = p->B, H = p->H;
  // the forward left the key norms in `saved`; without it they are computed again
  const float* knorm = !BIAS ? nullptr
                             : reinterpret_cast<const float*>(saved ? saved + L.sv_knorm : ws + L.off_bknorm);
  Geom g = make_geom(p, L, beta, gamma, slopes, knorm);
  float* dscale = reinterpret_cast<float*>(ws + L.off_dscale);
  bool ok = true;
  if (p->Nk == 0 || p->Nq == 0) {
    ok = ok && zero_rows<T>(dQ, L.q_sb, L.q_sh, L.q_sn, B, H, p->Nq, p->D, st);
    ok = ok && zero_rows<T>(dK, L.kv_sb, L.kv_sh, L.kv_sn, B, H, p->Nk, p->D, st);
    ok = ok && zero_rows<T>(dV, L.kv_sb, L.kv_sh, L.kv_sn, B, H, p->Nk, p->D, st);
    ok = ok && zero_words(dscale, (size_t)B * H * p->Nq * 4, st);
    for (int k = 1; k <= ENTMAX_BWD_PHASE_KEYS + 1; ++k) record(ev, k, st);
  } else {
    const bool lists = p->path != 1;
    if (BIAS && !saved && !launch_key_norms<T, D>(p, L, K, reinterpret_cast<float*>(ws + L.off_bknorm), st))
      return ENTMAX_ATTN_LAUNCH_FAILED;
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
      // the forward's lists, lengths and flags are only read (the list kernel that writes them is not launched)
      char* sv = const_cast<char*>(saved);
      sa.list = reinterpret_cast<uint2*>(saved ? sv + L.sv_pool : ws + L.off_jlist);
      sa.packed = saved ? 1 : 0;
      sa.pool_cap = saved ? saved_pool_entries(L, saved_bytes) : 0;
      sa.lcnt = reinterpret_cast<int*>(saved ? sv + L.sv_lcnt : ws + L.off_lcnt);
      sa.block_flag = saved ? reinterpret_cast<int*>(sv + L.sv_flags) : block_flag;
      sa.cells = ws + L.off_bcells;
      sa.kcursor = reinterpret_cast<int*>(ws + L.off_kcursor);
      sa.kcount = reinterpret_cast<int*>(ws + L.off_kcount);
      sa.precount = saved ? reinterpret_cast<const int*>(saved + L.sv_kcount) : nullptr;
      sa.koffs = reinterpret_cast<int*>(ws + L.off_koffs);
      sa.csc_i = reinterpret_cast<int*>(ws + L.off_csc_i);
      sa.csc_pw = reinterpret_cast<float2*>(ws + L.off_csc_pw);
      sa.head_flag = head_flag;
      sa.long_keys = reinterpret_cast<int*>(ws + L.off_longkeys);
      sa.stats = reinterpret_cast<unsigned long long*>(stats);
      sa.nqb = L.nqb;
      sa.dbeta = dbeta;
      sa.dgamma = dgamma;
      sa.scale_heads = p->scale_layout == 1 ? H : 0;
      {
        TransposeJobs jobs{};
        jobs.job[0] = transpose_job(K, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, ws + L.off_kt);
        jobs.job[1] = transpose_job(Q, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, ws + L.off_qt);
        jobs.job[2] = transpose_job(dO, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, ws + L.off_dot);
        sa.ride = transpose_ride_of(jobs, 3, B, H, head_flag, nullptr, 0);
      }
      ok = ok && launch_bwd_rows_am<T, D, BIAS>(sa, alpha_mode(p->alpha), B * H * ((L.nqb + 1) / 2), st, ev, saved != nullptr);
      if (!ok) return ENTMAX_ATTN_LAUNCH_FAILED;
    } else {
      record(ev, ENTMAX_BWD_PHASE_LISTS + 1, st);
    }
    record(ev, ENTMAX_BWD_PHASE_ROWS + 1, st);
    const int* hf = lists ? head_flag : nullptr;
    void* Kt = ws + L.off_kt;
    void* Qt = ws + L.off_qt;
    void* dOt = ws + L.off_dot;
    if (!lists) {  // (with lists the copies rode in the row launch)
      TransposeJobs jobs{};
      jobs.job[0] = transpose_job(K, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, Kt);
      jobs.job[1] = transpose_job(Q, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, Qt);
      jobs.job[2] = transpose_job(dO, L.q_sb, L.q_sh, L.q_sn, p->Nq, L.npad_q, dOt);
      ok = ok && launch_transposes<T, D>(jobs, 3, B, H, st);
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
    a.block_flag = lists ? sa.block_flag : nullptr;
    a.nqb = L.nqb;
    a.nkb = L.nkb;
    a.nqg = L.nqg;
    a.mask_words = L.mask_words;
    switch (alpha_mode(p->alpha)) {
      case 1: ok = launch_bwd_kernels<T, D, 1, BIAS>(a, L, B, H, st, ev); break;
      case 2: ok = launch_bwd_kernels<T, D, 2, BIAS>(a, L, B, H, st, ev); break;
      case 3: ok = launch_bwd_kernels<T, D, 3, BIAS>(a, L, B, H, st, ev); break;
      default: ok = launch_bwd_kernels<T, D, 0, BIAS>(a, L, B, H, st, ev); break;
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
  if (p->scale_layout == 1 && !(p->path != 1 && p->Nk > 0 && p->Nq > 0)) {  // (else done inside the keys launch)
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

}  // namespace entmax
