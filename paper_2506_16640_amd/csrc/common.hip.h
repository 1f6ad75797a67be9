// Shared device-side building blocks for the gfx950 entmax attention kernels:
// MFMA fragments for bf16 and fp32 elements, swizzled LDS tiles with a
// register-staged global->LDS pipeline, and the per-row quantities of the
// method (visible-key limit, ASEntmax scale).
//
// MFMA conventions used throughout (v_mfma_f32_32x32x16_bf16, wave64):
//   A operand: lane l holds A[row = l%32][k = 8*(l/32) + e], e = 0..7
//   B operand: lane l holds B[k = 8*(l/32) + e][col = l%32]
//   C/D      : lane l holds D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32], v = 0..15
// A "fragment" is the 8 consecutive k-elements one lane feeds to one MFMA.
// Because the contraction index may be enumerated in any order as long as both
// operands agree, the 16 accumulator values of one lane (8 per 16-row chunk)
// can be fed straight back as an A fragment whose k runs over the rows of the
// previous product: chunk c uses v = 8c..8c+7, i.e. rows
//   16c + 8*(e/4) + 4*(l/32) + e%4.
// The other operand of such a product must list the same rows in the same
// order; the transposed copies built by transpose_perm_kernel do exactly that.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "constants.h"
#include "entmax_attn.h"

namespace entmax {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr float kInf = __builtin_inff();

struct bf16_t {
  uint16_t bits;
};

// ---------------------------------------------------------------- fragments

template <typename T>
struct Frag;

template <>
struct Frag<bf16_t> {
  u32x4_t v;
};
template <>
struct Frag<float> {
  f32x4_t lo, hi;
};

template <typename T>
struct Elem;

template <>
struct Elem<bf16_t> {
  static constexpr int kTile = 64;  // rows of the streamed operand per LDS tile
  static __device__ __forceinline__ Frag<bf16_t> zero() {
    Frag<bf16_t> f;
    f.v = u32x4_t{0u, 0u, 0u, 0u};
    return f;
  }
  static __device__ __forceinline__ Frag<bf16_t> load(const void* p) {
    Frag<bf16_t> f;
    f.v = *reinterpret_cast<const u32x4_t*>(p);
    return f;
  }
  static __device__ __forceinline__ Frag<bf16_t> negate(Frag<bf16_t> f) {
    f.v ^= u32x4_t{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
    return f;
  }
  // sum of the squares of the fragment's 8 elements
  static __device__ __forceinline__ float sumsq(const Frag<bf16_t>& f) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float lo = __uint_as_float(f.v[k] << 16), hi = __uint_as_float(f.v[k] & 0xffff0000u);
      s = fmaf(lo, lo, fmaf(hi, hi, s));
    }
    return s;
  }
  // 8 fp32 values -> one fragment (round to nearest even)
  static __device__ __forceinline__ Frag<bf16_t> pack(const float* x) {
    bf16x8_t b;
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = (__bf16)x[e];
    Frag<bf16_t> f;
    f.v = __builtin_bit_cast(u32x4_t, b);
    return f;
  }
  // x = hi + lo with both parts bf16: keeps ~16 mantissa bits of x through two products
  static constexpr bool kSplit = true;
  static __device__ __forceinline__ void pack_split(const float* x, Frag<bf16_t>& hi, Frag<bf16_t>& lo) {
    bf16x8_t bh, bl;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      bh[e] = (__bf16)x[e];
      bl[e] = (__bf16)(x[e] - (float)bh[e]);
    }
    hi.v = __builtin_bit_cast(u32x4_t, bh);
    lo.v = __builtin_bit_cast(u32x4_t, bl);
  }
  static __device__ __forceinline__ f32x16_t mma(const Frag<bf16_t>& a, const Frag<bf16_t>& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a.v), __builtin_bit_cast(bf16x8_t, b.v),
                                                   c, 0, 0, 0);
  }
  static __device__ __forceinline__ void store(void* base, long long idx, float v) {
    reinterpret_cast<__bf16*>(base)[idx] = (__bf16)v;
  }
  static __device__ __forceinline__ float load_one(const void* base, long long idx) {
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
  }
};

template <>
struct Elem<float> {
  static constexpr int kTile = 32;
  static __device__ __forceinline__ Frag<float> zero() {
    Frag<float> f;
    f.lo = f32x4_t{0.f, 0.f, 0.f, 0.f};
    f.hi = f.lo;
    return f;
  }
  static __device__ __forceinline__ Frag<float> load(const void* p) {
    Frag<float> f;
    f.lo = reinterpret_cast<const f32x4_t*>(p)[0];
    f.hi = reinterpret_cast<const f32x4_t*>(p)[1];
    return f;
  }
  static __device__ __forceinline__ Frag<float> negate(Frag<float> f) {
    f.lo = -f.lo;
    f.hi = -f.hi;
    return f;
  }
  static __device__ __forceinline__ float sumsq(const Frag<float>& f) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) s = fmaf(f.lo[k], f.lo[k], fmaf(f.hi[k], f.hi[k], s));
    return s;
  }
  static __device__ __forceinline__ Frag<float> pack(const float* x) {
    Frag<float> f;
    f.lo = f32x4_t{x[0], x[1], x[2], x[3]};
    f.hi = f32x4_t{x[4], x[5], x[6], x[7]};
    return f;
  }
  static constexpr bool kSplit = false;
  static __device__ __forceinline__ void pack_split(const float* x, Frag<float>& hi, Frag<float>& lo) {
    hi = pack(x);
    lo = zero();
  }
  // eight 32x32x2 products: the e-th one contracts element e of both lane halves
  static __device__ __forceinline__ f32x16_t mma(const Frag<float>& a, const Frag<float>& b, f32x16_t c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo[e], b.lo[e], c, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi[e], b.hi[e], c, 0, 0, 0);
    return c;
  }
  static __device__ __forceinline__ void store(void* base, long long idx, float v) {
    reinterpret_cast<float*>(base)[idx] = v;
  }
  static __device__ __forceinline__ float load_one(const void* base, long long idx) {
    return reinterpret_cast<const float*>(base)[idx];
  }
};

// ------------------------------------------------------------------ LDS tiles

// ROWS x COLS elements of T, stored row-major in 16-byte chunks whose position
// inside the row is XOR-swizzled with the row index so that the 16 lanes served
// together by a ds_read_b128 / ds_write_b128 hit distinct banks.
template <typename T, int ROWS, int COLS>
struct LdsTile {
  static constexpr int kRowBytes = COLS * (int)sizeof(T);
  static constexpr int kCpr = kRowBytes / 16;  // chunks per row: 8, 16 or 32
  static constexpr int kBytes = ROWS * kRowBytes;
  static constexpr int kChunks = ROWS * kCpr;
  static constexpr int kPerThread = (kChunks + kThreads - 1) / kThreads;
  static_assert(kCpr >= 8, "row must span at least 128 bytes");
  static __device__ __forceinline__ int swz(int row) { return kCpr == 8 ? ((row >> 1) & 7) : (row & 15); }
  static __device__ __forceinline__ int off(int row, int chunk) {
    return row * kRowBytes + ((chunk ^ swz(row)) << 4);
  }
  // fragment f (8 elements) of a row
  static __device__ __forceinline__ Frag<T> frag(const char* tile, int row, int f);
};

template <typename T, int ROWS, int COLS>
__device__ __forceinline__ Frag<T> LdsTile<T, ROWS, COLS>::frag(const char* tile, int row, int f) {
  if constexpr (sizeof(T) == 2) {
    Frag<T> r;
    r.v = *reinterpret_cast<const u32x4_t*>(tile + off(row, f));
    return r;
  } else {
    Frag<T> r;
    r.lo = *reinterpret_cast<const f32x4_t*>(tile + off(row, 2 * f));
    r.hi = *reinterpret_cast<const f32x4_t*>(tile + off(row, 2 * f + 1));
    return r;
  }
}

// Byte offset(s) of one fragment inside a tile, precomputed per lane so that the
// inner loops issue ds_read_b128 with an immediate for everything that is
// uniform (buffer, 32-row block).  Valid as long as the rows added later are
// multiples of 32 (they do not change the swizzle).
template <typename T>
struct FragOff;
template <>
struct FragOff<bf16_t> {
  int o;
  template <typename TileT>
  static __device__ __forceinline__ FragOff make(int row, int f) {
    FragOff r;
    r.o = TileT::off(row, f);
    return r;
  }
  __device__ __forceinline__ Frag<bf16_t> load(const char* tile, int extra) const {
    Frag<bf16_t> r;
    r.v = *reinterpret_cast<const u32x4_t*>(tile + o + extra);
    return r;
  }
};
template <>
struct FragOff<float> {
  int o0, o1;
  template <typename TileT>
  static __device__ __forceinline__ FragOff make(int row, int f) {
    FragOff r;
    r.o0 = TileT::off(row, 2 * f);
    r.o1 = TileT::off(row, 2 * f + 1);
    return r;
  }
  __device__ __forceinline__ Frag<float> load(const char* tile, int extra) const {
    Frag<float> r;
    r.lo = *reinterpret_cast<const f32x4_t*>(tile + o0 + extra);
    r.hi = *reinterpret_cast<const f32x4_t*>(tile + o1 + extra);
    return r;
  }
};

// Register staging for one tile: init() fixes, per thread, which 16-byte chunks
// it moves (global byte offset inside the tile, swizzled LDS offset); fetch()
// issues the global loads of a ragged tile (rows at or beyond valid_rows repeat the last valid row),
// fetch_full() does the same for a tile known to lie wholly inside the tensor,
// commit() writes the staged chunks to LDS.
// NSET register sets let that many tiles be in flight at once (`set` must be a compile-time constant
// after inlining).
template <typename TileT, int NT = kThreads, int NSET = 1>
struct Stage {
  static_assert(TileT::kChunks % NT == 0, "every thread must move the same number of chunks");
  static constexpr int kPer = TileT::kChunks / NT;
  u32x4_t r[NSET][kPer];
  uint32_t goff[kPer];
  int loff[kPer];
  int row0;  // row of the first chunk; chunk `it` sits NT / kCpr rows further per step
  __device__ __forceinline__ void init(long long grow_bytes, int tid) {
    row0 = tid / TileT::kCpr;
    int ch = tid % TileT::kCpr;
#pragma unroll
    for (int it = 0; it < kPer; ++it) {
      int row = row0 + it * (NT / TileT::kCpr);
      goff[it] = (uint32_t)row * (uint32_t)grow_bytes + (uint32_t)(ch * 16);
      loff[it] = TileT::off(row, ch);
    }
  }
  __device__ __forceinline__ void fetch_full(const char* gtile, int set = 0) {
#pragma unroll
    for (int it = 0; it < kPer; ++it) r[set][it] = *reinterpret_cast<const u32x4_t*>(gtile + goff[it]);
  }
  // Ragged last tile: rows at or beyond valid_rows re-read the last valid row instead of being
  // zero-filled.  Every consumer masks those rows (they lie beyond the tensor), and a finite
  // stand-in keeps "0 x value" products finite; above all the loads stay unconditional, so the
  // compiler has no reason to wait for them before the tile that is computed meanwhile.
  __device__ __forceinline__ void fetch(const char* gtile, int valid_rows, long long grow_bytes, int set = 0) {
#pragma unroll
    for (int it = 0; it < kPer; ++it) {
      int row = min(row0 + it * (NT / TileT::kCpr), valid_rows - 1);
      uint32_t off = (uint32_t)row * (uint32_t)grow_bytes + (goff[0] - (uint32_t)row0 * (uint32_t)grow_bytes);
      r[set][it] = *reinterpret_cast<const u32x4_t*>(gtile + off);
    }
  }
  __device__ __forceinline__ void commit(char* tile, int set = 0) const {
#pragma unroll
    for (int it = 0; it < kPer; ++it) *reinterpret_cast<u32x4_t*>(tile + loff[it]) = r[set][it];
  }
};

// ------------------------------------------------------------ problem geometry

struct Geom {
  int B, H, Nq, Nk;
  int causal, scale_layout, logn_mode;
  float alpha, delta;
  long long q_sb, q_sh, q_sn;     // element strides of Q-like tensors
  long long kv_sb, kv_sh, kv_sn;  // element strides of K-like tensors
  int npad_k, npad_q;             // padded lengths (multiples of 64) of the transposed copies
  const float* beta;
  const float* gamma;
  const float* slopes;  // NULL, or [H] slopes of the linear distance bias (Sec. 4.2, App. B ALiBi definition)
  int bias_mode;        // 0: the bias is inside the ASEntmax scale, 1: outside
  const float* knorm;   // with slopes: [B*H] largest key norm of the head (key_norm_kernel)
};

// Keys visible to query row i are j < row_limit(i) (Sec. 2.1: j <= i, shifted by
// Nk - Nq when the two lengths differ).
__device__ __forceinline__ int row_limit(const Geom& g, int i) {
  if (!g.causal) return g.Nk;
  int c = i + (g.Nk - g.Nq) + 1;
  return c < 0 ? 0 : (c > g.Nk ? g.Nk : c);
}

// ASEntmax multiplier of eq. (asentmax): delta + beta (ln n)^gamma, natural log;
// rows whose n is <= 1 use delta.  Lg receives (ln n)^gamma and lnL receives
// ln ln n (both 0 when unused) for the parameter gradients.
__device__ __forceinline__ float row_scale(const Geom& g, int b, int h, int i, int nvis, float* Lg, float* lnL,
                                           float* bt) {
  float scale = g.delta, lg = 0.f, ll = 0.f, be = 0.f;
  if (g.scale_layout != 0) {
    long long idx = (g.scale_layout == 1) ? (long long)h : ((long long)b * g.H + h) * g.Nq + i;
    int n = (g.logn_mode == 0) ? g.Nk : nvis;
    be = g.beta[idx];
    if (n > 1) {
      float L = logf((float)n);
      lg = powf(L, g.gamma[idx]);
      ll = logf(L);
      scale = g.delta + be * lg;
    }
  }
  if (Lg) *Lg = lg;
  if (lnL) *lnL = ll;
  if (bt) *bt = be;
  return scale;
}

// Distance of key j from the position of query row i in the key sequence (App. B, ALiBi definition: the bias is
// m_h (j - i) for keys at or before the query and 0 after it); pos = i + (Nk - Nq).
__device__ __forceinline__ int bias_dist(int pos, int j) { return max(pos - j, 0); }

// The kernels work on y_ij = a_i d_ij with a_i = (alpha-1) |scale_i| / sqrt(D) and d_ij the dot product with
// the query negated when scale_i < 0.  The distance bias enters as d'_ij = d_ij + w_i dist_ij:
//   bias_mode 0, s = scale (z + b):  (alpha-1) scale b = a w dist  =>  w = -sgn(scale) m sqrt(D)
//   bias_mode 1, s = scale z + b:    (alpha-1) b       = a w dist  =>  w = -(alpha-1) m / a   (a = 0: no bias)
// c = scale_i / sqrt(D).
template <int D>
__device__ __forceinline__ float bias_w(const Geom& g, int h, float c, float a) {
  if (!g.slopes) return 0.f;
  const float m = g.slopes[h];
  if (m == 0.f || a == 0.f) return 0.f;
  if (g.bias_mode == 0) return (c < 0.f ? m : -m) * sqrtf((float)D);
  return -(g.alpha - 1.0f) * m / a;
}

// x^r and x^(r-1) for x >= 0, r = 1/(alpha-1) (eq. (entmax): p = x^r; its
// derivative factor g = p^(2-alpha) = x^(r-1)).  AM selects the integer-power
// paths: 1 -> alpha 1.5 (r=2), 2 -> alpha 2 (r=1), 3 -> alpha 1.25 (r=4), 0 -> generic.
template <int AM>
__device__ __forceinline__ float pow_r(float x, float r) {
  if (AM == 1) return x * x;
  if (AM == 2) return x;
  if (AM == 3) {
    float x2 = x * x;
    return x2 * x2;
  }
  return x > 0.f ? __builtin_amdgcn_exp2f(r * __builtin_amdgcn_logf(x)) : 0.f;
}
template <int AM>
__device__ __forceinline__ float pow_rm1(float x, float r) {
  if (AM == 1) return x;
  if (AM == 2) return x > 0.f ? 1.f : 0.f;
  if (AM == 3) return x * x * x;
  return x > 0.f ? __builtin_amdgcn_exp2f((r - 1.f) * __builtin_amdgcn_logf(x)) : 0.f;
}

__device__ __forceinline__ float max16(const f32x16_t& a) {
  float m0 = fmaxf(fmaxf(a[0], a[1]), a[2]);
  float m1 = fmaxf(fmaxf(a[3], a[4]), a[5]);
  float m2 = fmaxf(fmaxf(a[6], a[7]), a[8]);
  float m3 = fmaxf(fmaxf(a[9], a[10]), a[11]);
  float m4 = fmaxf(fmaxf(a[12], a[13]), a[14]);
  return fmaxf(fmaxf(fmaxf(m0, m1), fmaxf(m2, m3)), fmaxf(m4, a[15]));
}

// XCD-aware work order: consecutive workgroup ids land on different XCDs (8 of
// them, each with its own L2), so give every XCD a contiguous range of work
// items; all query blocks of a head then share one L2 for that head's K and V.
__device__ __forceinline__ int xcd_remap(int block, int total) {
  if (total % 8 != 0) return block;
  return (block & 7) * (total >> 3) + (block >> 3);
}

}  // namespace entmax
