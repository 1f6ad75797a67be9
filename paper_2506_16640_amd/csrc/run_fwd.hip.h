// Forward launcher: candidate-list kernels with the tiled kernel as fallback, or the
// split-key kernels for decode shapes.
#pragma once
#include "decode.hip.h"
#include "fwd.hip.h"
#include "fwd_sparse.hip.h"
#include "key_norm.hip.h"
#include "launch.hip.h"

namespace entmax {
namespace {

template <typename T, int D, int AM, bool BIAS>
bool launch_fwd_main(const FwdArgs& a, int nblocks, hipStream_t st) {
  size_t smem = 4 * (size_t)QCtx<T, D, FwdTile<T, D>::value>::kTileBytes + (size_t)(kWaves + 1) * a.mask_words * 4 +
                kWaves * 64 * 4 * sizeof(float) + 64;
  constexpr auto kern = fwd_kernel<T, D, AM, BIAS>;
  if (!ensure_dynamic_lds<kern>(smem)) return false;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  return launch_ok();
}

template <typename T, int D, bool BIAS>
bool launch_fwd_am(const FwdArgs& a, int am, int nblocks, hipStream_t st) {
  switch (am) {
    case 1: return launch_fwd_main<T, D, 1, BIAS>(a, nblocks, st);
    case 2: return launch_fwd_main<T, D, 2, BIAS>(a, nblocks, st);
    case 3: return launch_fwd_main<T, D, 3, BIAS>(a, nblocks, st);
    default: return launch_fwd_main<T, D, 0, BIAS>(a, nblocks, st);
  }
}

template <typename T, int D, int AM, bool BIAS>
bool launch_fwd_sparse(const FwdSparseArgs& a, int nblocks, hipStream_t st, void* const* ev) {
  size_t smem = ListCfg<T, D>::kLdsBytes;
  const int nsb = (a.nqb + 1) / 2;
  const long long pair_grid = (long long)a.g.B * a.g.H * ((nsb + 1) / 2);
  const bool long_seq = a.g.Nk >= ListCfg<T, D>::kFlagMinKeys;
  bool launched = false;
  if constexpr (sizeof(T) == 2 && D == 64) {  // (the only combination the two-block kernel is built for)
    if (a.force_long || (long_seq && pair_grid >= kPairMinWorkgroups)) {
    // long sequences: the second sweep skips blocks the first cleared, and a workgroup takes two adjacent blocks
    // where that still leaves three workgroups for every CU (measured at B 4, H 12, n 4096, where it leaves 1.5:
    // 221 us against 139 us with one block per workgroup)
    const size_t smem2 = PairCfg<T, D>::kLdsBytes > smem ? PairCfg<T, D>::kLdsBytes : smem;
    hipLaunchKernelGGL((fwd_lists_pair_kernel<T, D, AM, BIAS>), dim3((unsigned)pair_grid), dim3(kThreads), smem2, st, a);
    launched = true;
    }
  }
  if (a.unpaired) nblocks = a.g.B * a.g.H * a.nqb;
  if (launched) {
  } else if (long_seq || a.force_long)
    hipLaunchKernelGGL((fwd_lists_kernel<T, D, AM, BIAS, true>), dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  else
    hipLaunchKernelGGL((fwd_lists_kernel<T, D, AM, BIAS, false>), dim3((unsigned)nblocks), dim3(kThreads), smem, st, a);
  if (!launch_ok()) return false;
  record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
  hipLaunchKernelGGL((fwd_finish_kernel<T, D, AM>), dim3((unsigned)(a.g.B * a.g.H * a.nqb + a.ride.workgroups())),
                     dim3(kThreads), 0, st, a);
  return launch_ok();
}

template <typename T, int D, bool BIAS>
bool launch_fwd_sparse_am(const FwdSparseArgs& a, int am, int nblocks, hipStream_t st, void* const* ev) {
  switch (am) {
    case 1: return launch_fwd_sparse<T, D, 1, BIAS>(a, nblocks, st, ev);
    case 2: return launch_fwd_sparse<T, D, 2, BIAS>(a, nblocks, st, ev);
    case 3: return launch_fwd_sparse<T, D, 3, BIAS>(a, nblocks, st, ev);
    default: return launch_fwd_sparse<T, D, 0, BIAS>(a, nblocks, st, ev);
  }
}

template <typename T, int D>
bool launch_decode(const DecodeArgs& a, int am, hipStream_t st, void* const* ev) {
  const Geom& g = a.g;
  const dim3 sgrid((unsigned)a.nchunks, (unsigned)(g.B * g.H));
  if (g.Nq >= kDecodeMfmaRows)  // more rows than the per-row dot products are worth: matrix cores
    hipLaunchKernelGGL((decode_scores_mfma_kernel<T, D>), sgrid, dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL((decode_scores_kernel<T, D>), sgrid, dim3(kThreads), decode_scores_lds(g.Nq, D, sizeof(T)), st, a);
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

}  // namespace

template <typename T, int D, bool BIAS>
int run_fwd(const entmax_attn_params* p, const Layout& L, const void* Q, const void* K, const void* V,
            const float* beta, const float* gamma, const float* slopes, void* O, float* tau, char* saved,
            size_t saved_bytes, uint64_t* stats, char* ws, hipStream_t st, void* const* ev) {
  record(ev, 0, st);
  // with a `saved` buffer the key norms are written there: the backward needs them too
  float* knorm = !BIAS ? nullptr : reinterpret_cast<float*>(saved ? saved + L.sv_knorm : ws + L.off_fknorm);
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
      if (saved && !fill_words(saved + L.sv_flags, (size_t)p->B * p->H * L.nqb * sizeof(int), (unsigned)kBlockNoLists, st))
        return ENTMAX_ATTN_LAUNCH_FAILED;
      if (BIAS && saved && !launch_key_norms<T, D>(p, L, K, knorm, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
      record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
      DecodeArgs da;
      da.g = make_geom(p, L, beta, gamma, slopes, nullptr);
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
  int* dense_flag = reinterpret_cast<int*>(ws + L.off_flags);  // [B*H*nqb] blocks left to the tiled kernel
  const int npairs = p->B * p->H * ((L.nqb + 1) / 2);  // workgroups that take query blocks in pairs
  const bool lists = p->path != 1;
  if (BIAS && !launch_key_norms<T, D>(p, L, K, knorm, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
  record(ev, ENTMAX_FWD_PHASE_PREPARE + 1, st);
  if (lists) {
    FwdSparseArgs sa;
    sa.g = make_geom(p, L, beta, gamma, slopes, knorm);
    sa.Q = Q;
    sa.K = K;
    sa.V = V;
    sa.O = O;
    sa.tau = tau;
    sa.cand = reinterpret_cast<uint2*>(ws + L.off_cand);
    sa.cells = ws + L.off_fcells;
    sa.lcnt = reinterpret_cast<int*>(ws + L.off_flcnt);
    sa.bounds = reinterpret_cast<float2*>(ws + L.off_bounds);
    // with a `saved` buffer the rows' supports are listed for the backward
    sa.list = saved ? reinterpret_cast<uint2*>(saved + L.sv_pool) : nullptr;
    sa.pool_cursor = saved ? saved + L.sv_cursor : nullptr;
    sa.pool_parts = saved_pool_parts((long long)p->B * p->H * L.nqg);
    sa.pool_part_cap = saved ? saved_pool_entries(L, saved_bytes) / sa.pool_parts : 0;
    sa.slcnt = saved ? reinterpret_cast<int*>(saved + L.sv_lcnt) : nullptr;
    sa.bwd_flag = saved ? reinterpret_cast<int*>(saved + L.sv_flags) : nullptr;
    sa.kcount = saved ? reinterpret_cast<int*>(saved + L.sv_kcount) : nullptr;
    sa.dense_flag = dense_flag;
    sa.stats = reinterpret_cast<unsigned long long*>(stats);
    sa.nqb = L.nqb;
    sa.force_long = p->path == 2;
    sa.unpaired = fwd_lists_unpaired((long long)p->B * p->H, L.nqb) ? 1 : 0;
    {
      TransposeJobs jobs{};
      jobs.job[0] = transpose_job(V, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, Vt);
      sa.ride = transpose_ride_of(jobs, 1, p->B, p->H, nullptr, dense_flag, L.nqb);
    }
    if (!launch_fwd_sparse_am<T, D, BIAS>(sa, alpha_mode(p->alpha), npairs, st, ev)) return ENTMAX_ATTN_LAUNCH_FAILED;
  } else {
    // no lists: tell the backward that every block belongs to its tiled kernels
    if (saved && !fill_words(saved + L.sv_flags, (size_t)p->B * p->H * L.nqb * sizeof(int), (unsigned)kBlockNoLists, st))
      return ENTMAX_ATTN_LAUNCH_FAILED;
    record(ev, ENTMAX_FWD_PHASE_LISTS + 1, st);
  }
  record(ev, ENTMAX_FWD_PHASE_FINISH + 1, st);
  if (!lists) {  // (with lists the copies rode in the finish launch)
    TransposeJobs jobs{};
    jobs.job[0] = transpose_job(V, L.kv_sb, L.kv_sh, L.kv_sn, p->Nk, L.npad_k, Vt);
    if (!launch_transposes<T, D>(jobs, 1, p->B, p->H, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
  }
  record(ev, ENTMAX_FWD_PHASE_TRANSPOSE + 1, st);
  FwdArgs a;
  a.g = make_geom(p, L, beta, gamma, slopes, knorm);
  a.Q = Q;
  a.K = K;
  a.Vt = Vt;
  a.O = O;
  a.tau = tau;
  a.stats = reinterpret_cast<unsigned long long*>(stats);
  a.nqb = L.nqb;
  a.mask_words = L.mask_words;
  a.dense_flag = lists ? dense_flag : nullptr;
  a.dense_count = lists ? dense_flag + (size_t)p->B * p->H * L.nqb : nullptr;
  a.bounds = lists ? reinterpret_cast<const float2*>(ws + L.off_bounds) : nullptr;
  const int nwg = fwd_workgroups(p->B * p->H, L.nqb, lists);
  if (!launch_fwd_am<T, D, BIAS>(a, alpha_mode(p->alpha), nwg, st)) return ENTMAX_ATTN_LAUNCH_FAILED;
  record(ev, ENTMAX_FWD_PHASE_TILED + 1, st);
  return ENTMAX_ATTN_OK;
}

}  // namespace entmax
