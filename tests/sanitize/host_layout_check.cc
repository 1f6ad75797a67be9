// Host-only check of the C ABI's argument validation and buffer carving
// (paper_2506_16640_amd/csrc/host_layout.h), meant to be built with
// -fsanitize=address,undefined: sweeps many parameter sets, including hostile ones,
// and verifies that every carved region is aligned, ordered and inside the size the
// library reports.  Prints "ok <number of parameter sets>" on success.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "host_layout.h"

using namespace entmax;

static int failures = 0;
#define CHECK(cond)                                                      \
  do {                                                                   \
    if (!(cond)) {                                                       \
      std::fprintf(stderr, "FAILED %s (line %d)\n", #cond, __LINE__);    \
      ++failures;                                                        \
    }                                                                    \
  } while (0)

static void check_valid(const entmax_attn_params& p) {
  const Layout L = make_layout(&p);
  const size_t fwd = workspace_bytes_of(&p, 0), bwd = workspace_bytes_of(&p, 1), sv = saved_bytes_of(&p);
  CHECK(fwd >= kAlign && bwd >= kAlign && sv >= kAlign);
  CHECK(L.total_fwd <= fwd && L.total_bwd <= bwd && L.total_saved <= sv);
  const size_t fo[] = {L.off_vt, L.off_cand, L.off_flcnt, L.off_bounds, L.off_flags, L.off_fcells, L.total_fwd};
  for (size_t k = 0; k + 1 < sizeof(fo) / sizeof(fo[0]); ++k) CHECK(fo[k] <= fo[k + 1] && fo[k] % kAlign == 0);
  const size_t bo[] = {L.off_kt, L.off_qt, L.off_dot, L.off_mu, L.off_crow, L.off_dscale, L.off_mask, L.off_jlist,
                       L.off_lcnt, L.off_kcount, L.off_koffs, L.off_kcursor, L.off_csc_i, L.off_csc_pw, L.off_hflag,
                       L.off_longkeys, L.off_bcells, L.total_bwd};
  for (size_t k = 0; k + 1 < sizeof(bo) / sizeof(bo[0]); ++k) CHECK(bo[k] <= bo[k + 1] && bo[k] % kAlign == 0);
  const size_t so[] = {L.sv_cursor, L.sv_lcnt, L.sv_flags, L.sv_knorm, L.sv_kcount, L.sv_pool, L.total_saved};
  for (size_t k = 0; k + 1 < sizeof(so) / sizeof(so[0]); ++k) CHECK(so[k] <= so[k + 1] && so[k] % kAlign == 0);
  const size_t bh = (size_t)p.B * p.H;
  // the key-major arrays hold kBwdCap entries per half row: that is the bound the kernels check segments against
  CHECK(L.csc_cap == (long long)p.Nq * 2 * kBwdCap);
  CHECK(L.off_csc_pw - L.off_csc_i >= bh * (size_t)L.csc_cap * sizeof(int));
  CHECK(L.off_hflag - L.off_csc_pw >= bh * (size_t)L.csc_cap * 2 * sizeof(float));
  // support lists: kBwdCap (key, score) slots per lane of every 128-row block in the workspace; in `saved` a pool
  // behind the cursors of its parts, cut into parts that each hold at least one 32-row group's worst case
  CHECK(L.sv_lcnt - L.sv_cursor >= (size_t)kSavedSubPools * kSavedCursorStride);
  CHECK(L.sv_pool - L.sv_kcount >= bh * (size_t)p.Nk * sizeof(int));
  {
    const long long cap = saved_pool_entries(L, sv);
    const int parts = saved_pool_parts((long long)bh * L.nqg);
    CHECK(parts >= 1 && parts <= kSavedSubPools && (parts & (parts - 1)) == 0);
    const long long want = (long long)bh * p.Nq * kSavedPerRow + kSavedPoolFloor;
    CHECK(cap >= (want < (long long)kSavedPoolMost ? want : (long long)kSavedPoolMost) && cap < (1ll << 27));
    CHECK(L.sv_pool + ((size_t)cap + kSavedPoolPad) * 8 <= sv);
    CHECK(cap / parts >= (p.Nq < 32 ? p.Nq : 32) * 2 * kBwdCap);  // one 32-row group's worst case
    CHECK(saved_pool_entries(L, 0) == 0 && saved_pool_entries(L, L.sv_pool) == 0);
  }
  CHECK(L.off_lcnt - L.off_jlist >= bh * (size_t)L.nqb * kThreads * kBwdCap * 8);
  CHECK(L.sv_flags - L.sv_lcnt >= bh * (size_t)p.Nq * 2 * sizeof(int));
  CHECK(L.total_saved - L.sv_flags >= bh * (size_t)L.nqb * sizeof(int));
  CHECK(L.off_fcells - L.off_flags >= bh * (size_t)L.nqb * sizeof(int));
  {  // a cell strip for every workgroup of whichever list launch the forward picks
    const size_t pairs = bh * (size_t)((L.nqb + 1) / 2), strips = fwd_lists_unpaired((long long)bh, L.nqb) ? bh * (size_t)L.nqb : pairs;
    CHECK(L.off_fknorm - L.off_fcells >= strips * cell_bytes_per_workgroup(kCandCap));
  }
  CHECK(L.off_flcnt - L.off_cand >= bh * (size_t)L.nqb * kThreads * kCandCap * 8);
  CHECK(L.off_bounds - L.off_flcnt >= bh * (size_t)p.Nq * 2 * sizeof(int));
  CHECK(L.off_flags - L.off_bounds >= bh * (size_t)p.Nq * 2 * sizeof(float));
  CHECK(L.off_longkeys - L.off_hflag >= (bh * (size_t)L.nqb + 2 * bh) * sizeof(int));
  if (decode_shape(p.Nq, p.Nk)) {
    CHECK(L.off_dec_cmax >= bh * (size_t)p.Nq * (size_t)p.Nk * sizeof(float));
    CHECK(L.total_fwd >= L.off_dec_cmax + bh * (size_t)p.Nq * L.dec_nchunks * sizeof(float));
  }
}

int main() {
  long n = 0;
  const int sizes[] = {0, 1, 2, 31, 32, 33, 127, 128, 129, 1000, 4096, 32768, (1 << 22), (1 << 22) + 1, -1};
  const int heads[] = {0, 1, 3, 12, 65535, 65536};
  for (int dtype = -1; dtype <= 2; ++dtype)
    for (int D : {0, 32, 64, 96, 128, 256})
      for (int Nq : sizes)
        for (int Nk : sizes)
          for (int H : heads)
            for (int B : {0, 1, 4}) {
              entmax_attn_params p{};
              p.B = B; p.H = H; p.Nq = Nq; p.Nk = Nk; p.D = D; p.dtype = dtype;
              p.causal = 1; p.scale_layout = 1; p.logn_mode = 0; p.path = 0; p.alpha = 1.5f; p.delta = 1.0f;
              const int rc = check_params(&p);
              ++n;
              if (rc == ENTMAX_ATTN_OK) {
                check_valid(p);
              } else {
                CHECK(workspace_bytes_of(&p, 0) == 0 && workspace_bytes_of(&p, 1) == 0 && saved_bytes_of(&p) == 0);
              }
            }
  // strides: negative, misaligned, overlapping rows, huge
  const int64_t strides[] = {0, 8, 64, 65, 128, 1 << 20, (int64_t)1 << 40, INT64_MAX, -64};
  for (int64_t sb : strides)
    for (int64_t sh : strides)
      for (int64_t sn : strides)
        for (int dtype = 0; dtype <= 1; ++dtype) {
          entmax_attn_params p{};
          p.B = 2; p.H = 3; p.Nq = 100; p.Nk = 70; p.D = 64; p.dtype = dtype;
          p.causal = 0; p.scale_layout = 2; p.logn_mode = 1; p.path = 1; p.alpha = 2.0f; p.delta = 0.0f;
          p.q_stride_b = sb; p.q_stride_h = sh; p.q_stride_n = sn;
          p.kv_stride_b = sn; p.kv_stride_h = sb; p.kv_stride_n = sh;
          ++n;
          if (check_params(&p) == ENTMAX_ATTN_OK) check_valid(p);
        }
  CHECK(check_params(nullptr) == ENTMAX_ATTN_INVALID_ARG);
  if (failures) return 1;
  std::printf("ok %ld\n", n);
  return 0;
}
