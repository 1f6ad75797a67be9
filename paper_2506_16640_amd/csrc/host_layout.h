// Host-side argument validation and buffer carving for the C ABI of
// include/entmax_attn.h.  Plain C++ (no HIP types): the entry points use it, and so does
// the host-only sanitizer build of the tests.
#pragma once
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "constants.h"
#include "entmax_attn.h"

namespace entmax {

constexpr size_t kAlign = 256;
constexpr unsigned long long kSavedPoolMost = (1ull << 27) - 1;  // entries a `saved` pool can address
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
  size_t off_vt, off_cand, off_flcnt, off_bounds, off_flags, off_fcells, off_kt, off_qt, off_dot, off_mu, off_crow, off_dscale, off_mask, off_jlist, off_lcnt,
      off_kcount, off_koffs, off_kcursor, off_csc_i, off_csc_pw, off_hflag, off_longkeys, off_bcells, off_fknorm, off_bknorm, sv_cursor, sv_lcnt,
      sv_flags, sv_knorm, sv_kcount, sv_pool, total_saved, total_fwd, total_bwd;
  size_t off_dec_cmax;  // decode kernels: score rows at offset 0, then the chunk maxima
  int dec_nks, dec_nchunks, dec_chunk;
  long long csc_cap;    // entries of the key-major arrays per head
};

inline int check_params(const entmax_attn_params* p) {
  if (!p) return ENTMAX_ATTN_INVALID_ARG;
  if (p->B < 0 || p->H < 0 || p->Nq < 0 || p->Nk < 0) return ENTMAX_ATTN_INVALID_ARG;
  if (p->dtype != ENTMAX_ATTN_BF16 && p->dtype != ENTMAX_ATTN_FP32) return ENTMAX_ATTN_INVALID_ARG;
  if (p->causal != 0 && p->causal != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (p->scale_layout < 0 || p->scale_layout > 2) return ENTMAX_ATTN_INVALID_ARG;
  if (p->logn_mode != 0 && p->logn_mode != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (p->bias_mode != 0 && p->bias_mode != 1) return ENTMAX_ATTN_INVALID_ARG;
  if (p->path < 0 || p->path > 2) return ENTMAX_ATTN_INVALID_ARG;
  if (!(p->alpha > 1.0f) || !(p->alpha <= 2.0f)) return ENTMAX_ATTN_INVALID_ARG;
  if (!isfinite(p->delta)) return ENTMAX_ATTN_INVALID_ARG;
  if (p->D != 64 && p->D != 128) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (p->Nq > (1 << 22) || p->Nk > (1 << 22)) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;  // 32-bit offsets inside a tile
  long long bh = (long long)p->B * p->H;
  if (bh * (long long)ceil_div(p->Nq > p->Nk ? p->Nq : p->Nk, 32) > 0x7fffffffLL) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (bh > 65535) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  const int64_t s[6] = {p->q_stride_b, p->q_stride_h, p->q_stride_n, p->kv_stride_b, p->kv_stride_h, p->kv_stride_n};
  bool q_zero = s[0] == 0 && s[1] == 0 && s[2] == 0, kv_zero = s[3] == 0 && s[4] == 0 && s[5] == 0;
  int64_t es = p->dtype == ENTMAX_ATTN_BF16 ? 2 : 4;
  for (int k = 0; k < 6; ++k) {
    if (s[k] < 0) return ENTMAX_ATTN_INVALID_ARG;
    if (s[k] > (INT64_MAX >> 3)) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;  // byte offsets must not wrap
    if ((s[k] * es) % 16 != 0) return ENTMAX_ATTN_MISALIGNED;
  }
  if (s[2] * es > (1 << 24) || s[5] * es > (1 << 24)) return ENTMAX_ATTN_UNSUPPORTED_SHAPE;
  if (!q_zero && s[2] < p->D) return ENTMAX_ATTN_INVALID_ARG;
  if (!kv_zero && s[5] < p->D) return ENTMAX_ATTN_INVALID_ARG;
  return ENTMAX_ATTN_OK;
}

inline Layout make_layout(const entmax_attn_params* p) {
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
  // forward: V^T copy (tiled kernel only) | candidate lists (one per lane of the list grid), their lengths, the
  // rows' brackets | per-block fallback flags | the list sweep's cell strips
  // cell strips of the list sweeps: one per workgroup (a pair of blocks), or two per workgroup of the
  // long-sequence kernel (two pairs of adjacent blocks)
  const size_t list_groups = bh * (size_t)(2 * ((L.nqb + 3) / 4));
  // (the forward's strips: one per block where its list kernel takes the blocks one by one)
  const size_t fwd_groups = fwd_lists_unpaired((long long)bh, L.nqb) ? bh * (size_t)L.nqb : list_groups;
  L.off_vt = 0;
  L.off_cand = kt_bytes;
  L.off_flcnt = L.off_cand + align_up(bh * (size_t)L.nqb * kThreads * kCandCap * 8);
  L.off_bounds = L.off_flcnt + align_up(bh * (size_t)p->Nq * 2 * sizeof(int));
  L.off_flags = L.off_bounds + align_up(bh * (size_t)p->Nq * 2 * sizeof(float));
  L.off_fcells = L.off_flags + align_up((bh * (size_t)L.nqb + 1 + kSplitMaxBlocks) * sizeof(int));  // flags, their count, flagged blocks
  L.off_fknorm = L.off_fcells + align_up(fwd_groups * cell_bytes_per_workgroup(kCandCap));
  L.total_fwd = L.off_fknorm + align_up(bh * sizeof(float));  // the heads' largest key norms (distance bias only)
  // the `saved` buffer: the pool's cursors, per half row (place, length) of its support list, one flag per block for the
  // backward, the heads' key norms, the number of support entries that name each key, and behind them the pool
  // the lists themselves are packed into (each 32-row group takes one contiguous piece, sized by its candidate
  // counts).  The pool runs to the end of the caller's buffer; the size asked for holds kSavedPerRow entries per
  // row on average.  A block whose group finds the pool used up is flagged and left to the backward's tiled kernels.
  const size_t list_bytes = align_up(bh * (size_t)L.nqb * kThreads * kBwdCap * 8);  // (fixed-slot lists of the workspace)
  L.sv_cursor = 0;
  L.sv_lcnt = align_up((size_t)kSavedSubPools * kSavedCursorStride);
  L.sv_flags = L.sv_lcnt + align_up(bh * (size_t)p->Nq * 2 * sizeof(int));
  L.sv_knorm = L.sv_flags + align_up(bh * (size_t)L.nqb * sizeof(int));
  L.sv_kcount = L.sv_knorm + align_up(bh * sizeof(float));  // (the heads' largest key norms: distance bias only)
  L.sv_pool = L.sv_kcount + align_up(bh * (size_t)p->Nk * sizeof(int));  // support entries per key
  size_t pool_entries = bh * (size_t)p->Nq * kSavedPerRow + kSavedPoolFloor;
  if (pool_entries > kSavedPoolMost) pool_entries = kSavedPoolMost;  // places are 27-bit numbers
  L.total_saved = L.sv_pool + align_up((pool_entries + kSavedPoolPad) * 8);
  // the decode kernels' score rows take the place of everything above
  L.dec_nks = L.dec_nchunks = L.dec_chunk = 0;
  L.off_dec_cmax = 0;
  if (decode_shape(p->Nq, p->Nk)) {
    L.dec_nks = (p->Nk + 3) / 4 * 4;
    L.dec_chunk = kDecodeChunk;
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
  o += list_bytes;
  L.off_lcnt = o;
  o += align_up(rows * 2 * sizeof(int));
  size_t key_bytes = align_up(bh * (size_t)p->Nk * sizeof(int));
  L.off_kcount = o;
  o += key_bytes;
  L.off_koffs = o;
  o += key_bytes;
  L.off_kcursor = o;
  o += key_bytes;
  // key-major arrays: a head holds at most kBwdCap support entries per half row on the list path
  L.csc_cap = (long long)p->Nq * 2 * kBwdCap;
  L.off_csc_i = o;
  o += align_up(rows * 2 * kBwdCap * sizeof(int));
  L.off_csc_pw = o;
  o += align_up(rows * 2 * kBwdCap * 2 * sizeof(float));
  L.off_hflag = o;
  o += align_up((bh * (size_t)L.nqb + 2 * bh) * sizeof(int));  // block flags, head flags, long-key counts per head
  L.off_longkeys = o;
  o += key_bytes;
  L.off_bcells = o;
  o += align_up(list_groups * cell_bytes_per_workgroup(kBwdCap));
  L.off_bknorm = o;
  o += align_up(bh * sizeof(float));
  L.total_bwd = o;
  return L;
}

// Entries the pool of a `saved` buffer of `bytes` bytes holds (beyond them: kSavedPoolPad entries that may be read
// but never hold anything).  Places are packed into 27 bits next to the 5-bit length.
inline long long saved_pool_entries(const Layout& L, size_t bytes) {
  if (bytes < L.sv_pool + (size_t)kSavedPoolPad * 8) return 0;
  const unsigned long long n = (bytes - L.sv_pool) / 8 - kSavedPoolPad;
  return (long long)(n < kSavedPoolMost ? n : kSavedPoolMost);
}

inline size_t saved_bytes_of(const entmax_attn_params* p) {
  if (check_params(p) != ENTMAX_ATTN_OK) return 0;
  Layout L = make_layout(p);
  return L.total_saved < kAlign ? kAlign : L.total_saved;
}

inline size_t workspace_bytes_of(const entmax_attn_params* p, int is_bwd) {
  if (check_params(p) != ENTMAX_ATTN_OK) return 0;
  Layout L = make_layout(p);
  size_t n = is_bwd ? L.total_bwd : L.total_fwd;
  return n < kAlign ? kAlign : n;
}

}  // namespace entmax
