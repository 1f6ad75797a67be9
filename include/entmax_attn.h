/*
 * entmax_attn.h -- C ABI of the MI355X (gfx950) alpha-entmax / ASEntmax
 * attention library.
 *
 * The operation (paper Sec. 2.1, Sec. 2.2 eq. (entmax), Sec. 4.1 eq. (asentmax)):
 * for every batch b, head h and query row i
 *
 *     z_ij  = <q_i, k_j> / sqrt(D)                      visible keys j only
 *     s_ij  = scale_i * z_ij,   scale_i = delta + beta * (ln n)^gamma
 *             (with a positional bias, below: scale_i * (z_ij + b_ij) or scale_i * z_ij + b_ij)
 *     p_ij  = [ (alpha-1) s_ij - tau_i ]_+ ^ (1/(alpha-1)),   sum_j p_ij = 1
 *     o_i   = sum_j p_ij v_j
 *
 * tau_i is the entmax threshold of row i (App. A); keys with
 * (alpha-1) s_ij <= tau_i get exactly zero weight.  Under the causal flag key j
 * is visible to query i iff j <= i + (Nk - Nq).  The backward pass applies the
 * exact Jacobian of eq. (entmax): g = p^(2-alpha), dS = g * (dP - sum(g dP)/sum(g)),
 * and the chain rule through scale_i to beta and gamma.
 *
 * Conventions common to all entry points
 *   - Every pointer except `p` and `phase_events` is DEVICE memory owned by the
 *     caller; the library allocates and frees nothing and keeps no state.
 *   - All work is enqueued on `hip_stream` (a hipStream_t; NULL = default
 *     stream); no entry point synchronises.
 *   - Q, O, dO, dQ are [B,H,Nq,D]; K, V, dK, dV are [B,H,Nk,D]; the last
 *     dimension is contiguous; batch/head/row strides are given in elements
 *     (0 = contiguous default).  Element type per `dtype`.  Pointers and row
 *     strides must be 16-byte aligned.
 *   - tau is [B,H,Nq] fp32 contiguous, in the units of eq. (entmax).
 *   - beta, gamma: fp32, [H] (scale_layout 1) or [B,H,Nq] (scale_layout 2),
 *     ignored (may be NULL) for scale_layout 0 where scale_i = delta.
 *   - alibi_slopes: NULL (no positional bias, "NoPE"), or fp32 [H] slopes m_h >= 0 of the linear distance
 *     bias of Sec. 4.2 / App. B (ALiBi definition): b_ij = -m_h * max(0, i + (Nk - Nq) - j), i.e. m_h (j - i)
 *     for the keys at or before the query's position and 0 after it.  A head with m_h = 0 has no bias
 *     (NAPE, Sec. 4.2: half of the heads biased, the other half not).  `bias_mode` places b_ij inside or
 *     outside the ASEntmax scale.  The slopes are constants: no gradient is returned for them.  The
 *     backward must be given the same slopes and bias_mode as the forward.  With the bias, keys further
 *     from the query than the window of App. B (ALiBi proposition; evaluated per row from
 *     |z_ij| <= |q_i| max_j |k_j| / sqrt(D)) cannot be in the support, and the kernels do not visit their
 *     tiles.  bias_mode 1 needs scale_i != 0 (a row whose scale is exactly 0 is computed without bias).
 *   - Return value: 0 on success, a negative entmax_attn_status otherwise.
 *     Arguments are validated on the host before anything is launched: with
 *     INVALID_ARG, UNSUPPORTED_SHAPE, MISALIGNED or WORKSPACE_TOO_SMALL nothing has
 *     been enqueued.  LAUNCH_FAILED means the HIP runtime refused one of the
 *     call's launches: the kernels before it are already on the stream and will
 *     run, so the outputs, the workspace and `saved` are then undefined.
 *   - `stats`, `phase_events` and `params.path` are optional instrumentation for
 *     tests and measurement (NULL, NULL and 0 in production use).
 */
#ifndef ENTMAX_ATTN_H
#define ENTMAX_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ENTMAX_ATTN_OK = 0,
  ENTMAX_ATTN_INVALID_ARG = -1,       /* NULL where a pointer is required, bad enum, non-positive size, alpha outside (1,2] */
  ENTMAX_ATTN_UNSUPPORTED_SHAPE = -2, /* D not in {64,128}, sizes beyond the index range */
  ENTMAX_ATTN_MISALIGNED = -3,        /* pointer or stride not 16-byte aligned */
  ENTMAX_ATTN_WORKSPACE_TOO_SMALL = -4, /* workspace_bytes or saved_bytes below what the parameters need */
  ENTMAX_ATTN_LAUNCH_FAILED = -5,     /* the HIP runtime refused a launch */
  ENTMAX_ATTN_SCRATCH_LIMIT = -6      /* entmax_attn_fwd_noalloc: the problem needs more scratch than the library's
                                         built-in buffer holds (use entmax_attn_fwd with a workspace) */
} entmax_attn_status;

enum { ENTMAX_ATTN_BF16 = 0, ENTMAX_ATTN_FP32 = 1 };

typedef struct {
  int32_t B, H, Nq, Nk, D; /* D in {64, 128} */
  int32_t dtype;           /* ENTMAX_ATTN_BF16 or ENTMAX_ATTN_FP32: type of Q,K,V,O,dO,dQ,dK,dV */
  int32_t causal;          /* 1: key j visible to query i iff j <= i + (Nk - Nq); 0: all keys visible */
  int32_t scale_layout;    /* 0: scale = delta; 1: beta,gamma per head [H]; 2: per query [B,H,Nq] */
  int32_t logn_mode;       /* n in (ln n)^gamma: 0 = Nk for every row, 1 = number of keys visible to the row.
                              A row with n <= 1 uses scale = delta and contributes no beta/gamma gradient. */
  int32_t bias_mode;       /* with alibi_slopes: 0 = s_ij = scale_i (z_ij + b_ij), the bias is part of the logit that
                              eq. (asentmax) scales; 1 = s_ij = scale_i z_ij + b_ij.  Ignored without slopes. */
  int32_t path;            /* forward path: 0 = automatic (candidate-list kernel first; workgroups that meet a row
                              with too many candidates fall back to the tiled kernel; with Nq <= 8, or Nq <= 64 and
                              Nk >= 64 Nq -- the decoding shape -- kernels that split the keys instead),
                              1 = tiled kernel only, 2 = as 0 without the decoding-shape kernels and with the list
                              kernels for long sequences (Nk >= 16384) whatever the sizes: a test aid */
  float alpha;             /* 1 < alpha <= 2; 1.5, 2.0 and 1.25 run on integer-power fast paths */
  float delta;             /* ASEntmax delta (1.0 in the paper's experiments) */
  int64_t q_stride_b, q_stride_h, q_stride_n;    /* strides of Q,O,dO,dQ in elements; all 0 = contiguous */
  int64_t kv_stride_b, kv_stride_h, kv_stride_n; /* strides of K,V,dK,dV in elements; all 0 = contiguous */
} entmax_attn_params;

/* Indices into the optional device counter array `stats` (uint64, at least
 * ENTMAX_ATTN_NUM_STATS entries, zeroed by the caller; the kernels add to it).
 * A "tile" is one 32-query x 32-key block, the unit of one MFMA output block
 * and of the zero-tile test. */
enum {
  ENTMAX_STAT_FWD_TILES_VISIBLE = 0, /* tiles holding at least one unmasked (i,j) pair */
  ENTMAX_STAT_FWD_QK_MAX = 1,        /* score tiles computed by the row-max sweep */
  ENTMAX_STAT_FWD_QK_SOLVE = 2,      /* score tiles computed by all threshold sweeps together */
  ENTMAX_STAT_FWD_QK_PV = 3,         /* score tiles recomputed by the P.V sweep */
  ENTMAX_STAT_FWD_PV_TILES = 4,      /* tiles whose P.V product ran (the others were all zero: skipped) */
  ENTMAX_STAT_FWD_SOLVE_SWEEPS = 5,  /* threshold sweeps, summed over workgroups */
  ENTMAX_STAT_FWD_BLOCKS = 6,        /* workgroups */
  ENTMAX_STAT_FWD_EVAL_TILES = 7,    /* tiles on which the threshold function was evaluated element by element */
  ENTMAX_STAT_BWD_TILES_VISIBLE = 8,
  ENTMAX_STAT_BWD_QK_MASK = 9,       /* score tiles the dQ kernel computed (it finds the non-zero tiles on the way) */
  ENTMAX_STAT_BWD_ACTIVE_TILES = 10, /* tiles with some p_ij > 0 */
  ENTMAX_STAT_BWD_DQ_TILES = 11,     /* tiles processed by the dQ / row-scalar kernel */
  ENTMAX_STAT_BWD_DKV_TILES = 12,    /* tiles processed by the dK / dV kernel */
  ENTMAX_STAT_FWD_CAND_TILES = 13,   /* candidate-list kernel: tiles holding at least one candidate key */
  ENTMAX_STAT_FWD_CANDIDATES = 14,   /* candidate-list kernel: keys put on the lists */
  ENTMAX_STAT_FWD_SUPPORT = 15,      /* candidate-list kernel: non-zero probabilities (exact support size, summed) */
  ENTMAX_STAT_FWD_SPARSE_BLOCKS = 16, /* workgroups finished by the candidate-list kernel */
  ENTMAX_STAT_FWD_LIST_QK = 17,      /* candidate-list kernel: score tiles computed (both sweeps) */
  ENTMAX_STAT_BWD_LIST_QK = 18,      /* support-list backward: score tiles computed by its one sweep */
  ENTMAX_STAT_BWD_SUPPORT = 19,      /* support-list backward: (row, key) entries with p > 0 */
  ENTMAX_STAT_FWD_WINDOW_SKIPPED = 20, /* with alibi_slopes: visible tiles (counted in FWD_TILES_VISIBLE) that no sweep
                                          visited because they lie beyond the rows' distance window */
  ENTMAX_ATTN_NUM_STATS = 24
};

/* Phases of one call, for the optional profiling hook `phase_events`: when not
 * NULL it is a HOST array of hipEvent_t handles (created by the caller) with
 * one more entry than the call has phases; entry 0 is recorded on the stream
 * before the first kernel and entry k after the last kernel of phase k-1. */
enum {
  ENTMAX_FWD_PHASE_PREPARE = 0,   /* with alibi_slopes: the heads' largest key norms (else empty) */
  ENTMAX_FWD_PHASE_LISTS = 1,     /* candidate-list kernel: two Q K^T sweeps (row maximum, candidates);
                                     decoding shape: the score rows, one pass over K */
  ENTMAX_FWD_PHASE_FINISH = 2,    /* threshold and output from the candidate lists (decoding shape: from the
                                     score rows) */
  ENTMAX_FWD_PHASE_TRANSPOSE = 3, /* path 1: V^T copy for the tiled kernel (path 0: made by extra workgroups of the
                                     finish launch, for the heads that need it) */
  ENTMAX_FWD_PHASE_TILED = 4,     /* tiled kernel on the workgroups the list kernel left over */
  ENTMAX_FWD_NUM_PHASES = 5
};
enum {
  ENTMAX_BWD_PHASE_LISTS = 0,      /* without `saved`: one Q K^T sweep at the saved threshold, and with alibi_slopes
                                      the heads' largest key norms before it */
  ENTMAX_BWD_PHASE_ROWS = 1,       /* per-key segment offsets; mu, dscale, dQ and the per-entry (p, dS) from the lists */
  ENTMAX_BWD_PHASE_TRANSPOSE = 2,  /* path 1: operand copies for the tiled kernels (path 0: made by extra workgroups
                                      of the row launch, for the heads that need them) */
  ENTMAX_BWD_PHASE_MASK = 3,       /* (empty: the non-zero tile map is a by-product of the dQ kernel) */
  ENTMAX_BWD_PHASE_DQ = 4,         /* tiled path: row scalars, dQ and the non-zero tile map */
  ENTMAX_BWD_PHASE_DKV = 5,        /* tiled path: dK, dV */
  ENTMAX_BWD_PHASE_KEYS = 6,       /* support-list path: dK and dV per key (and d beta, d gamma per head) */
  ENTMAX_BWD_PHASE_SCALE_GRAD = 7,
  ENTMAX_BWD_NUM_PHASES = 8
};

/*
 * Forward (Sec. 2.1 with pi = alpha-entmax on ASEntmax-scaled logits).
 *   in : Q, K, V, beta, gamma, alibi_slopes
 *   out: O (dtype, written for every row), tau [B,H,Nq] fp32 (saved for the backward).
 *        A row with no visible key gets O = 0, tau = 0.
 *   stats: NULL or device uint64[ENTMAX_ATTN_NUM_STATS], added to.
 *   saved: NULL, or device memory of at least entmax_attn_saved_bytes(p) bytes, 256-byte aligned, owned by the
 *        caller: receives the rows' support lists (key, raw score) -- Sec. 2.2: the keys with non-zero
 *        probability -- for the backward, which then skips its own Q K^T sweep.  The lists are packed into a
 *        pool that runs to the end of the buffer; the size the library asks for holds six entries per row on
 *        average (under half the size of O at D = 64), and a larger buffer gives a larger pool.  A 128-row query
 *        block that finds the pool used up, or has a half row with more than 16 support entries, is marked for
 *        the backward's tiled kernels instead (same results up to rounding; slower).  When the pool runs out,
 *        which blocks are marked depends on the order the workgroups arrive in.  Needs Nk <= 2^22 (as everything).  Opaque; valid only together
 *        with this call's tau and the same params, inputs and saved_bytes.
 *   saved_bytes: size of `saved` (ignored when saved is NULL); less than entmax_attn_saved_bytes(p) is
 *        refused with WORKSPACE_TOO_SMALL before anything is launched.
 *   workspace: device scratch of at least entmax_attn_workspace_bytes(p, 0)
 *        bytes, 256-byte aligned; contents are undefined afterwards.
 * The row threshold is found from sweeps over the key tiles that recompute
 * Q K^T each time (row max, then safeguarded Newton/Halley steps on
 * f(tau) = sum_j [(alpha-1) s_ij - tau]_+^(1/(alpha-1)) - 1 inside the bracket of
 * App. A eq. (bounds)); the n x n score matrix is never stored.  Rows with few
 * candidates above a lower bound of tau are finished from a short per-row list
 * after two sweeps; denser rows run the tile-wise iteration and P.V on the
 * matrix cores with zero tiles skipped.
 * Decoding shape (path 0; Nq <= 8, or Nq <= 64 with Nk >= 64 Nq: a few query rows against a long key sequence, the regime of the
 * long-context evaluation of Sec. 4): the keys, not the queries, are split over the chip; K is
 * read once, the rows' scores (Nq x Nk fp32 per head) go to the workspace, and each row's
 * threshold and output come from its score row.  `saved` then only tells the backward to rebuild
 * the supports itself.
 */
int entmax_attn_fwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const float* beta,
                    const float* gamma, const float* alibi_slopes, void* O, float* tau, void* saved, size_t saved_bytes, uint64_t* stats,
                    void* workspace, size_t workspace_bytes, void* hip_stream, void* const* phase_events);

/*
 * Backward (exact derivative of the forward; Jacobian of eq. (entmax)).
 *   in : Q, K, V, dO, tau (as written by the forward), beta, gamma, alibi_slopes
 *   out: dQ, dK, dV (dtype; every element written);
 *        dbeta, dgamma fp32 in beta/gamma's layout, OVERWRITTEN (not
 *        accumulated); ignored (may be NULL) for scale_layout 0.
 *   O is accepted for symmetry with the usual attention backward and may be NULL
 *   (the row term is rebuilt from tau, not from O).
 *   saved: NULL, or the buffer the forward filled for these same inputs (read only).  With it the
 *        rows' supports are taken from the forward's lists; without it one Q K^T sweep at tau rebuilds them.  Same results either way up
 *        to the summation order inside a row.
 *   saved_bytes: size of `saved`, checked as in the forward; pass the value the forward was given.
 *   workspace: at least entmax_attn_workspace_bytes(p, 1) bytes, 256-byte aligned.
 * `path` selects as in the forward: 0 = support lists per row and per key for the 128-row query blocks
 * whose rows have few non-zero probabilities, tiled kernels for the other blocks; 1 = tiled kernels only.
 * No floating-point atomics touch the outputs.  The tiled path is bitwise reproducible; the
 * list path sums each key's entries in query order whenever a key has at most 64 of them.
 */
int entmax_attn_bwd(const entmax_attn_params* p, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* tau, const void* saved, size_t saved_bytes, const float* beta,
                    const float* gamma, const float* alibi_slopes, void* dQ, void* dK, void* dV, float* dbeta, float* dgamma, uint64_t* stats,
                    void* workspace, size_t workspace_bytes, void* hip_stream, void* const* phase_events);

/*
 * Forward for callers that cannot allocate device memory and have no workspace to hand over: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments
 * and results as entmax_attn_fwd without `saved`, `workspace` and `phase_events`: the scratch is a buffer
 * built into the library (device memory of entmax_attn_noalloc_scratch_bytes() bytes that every GPU the
 * library runs on holds until the process ends).  The call allocates and frees nothing.
 *   - Parameters with entmax_attn_workspace_bytes(p, 0) above that size are refused with
 *     ENTMAX_ATTN_SCRATCH_LIMIT before anything is launched.
 *   - All calls on one GPU share that GPU's buffer: calls that may overlap in time (different streams,
 *     different host threads) race; calls on one stream are ordered and safe.  The buffer keeps the previous
 *     call's contents; the kernels write every word they later read, so nothing needs clearing.
 *   - The buffer's address is looked up once per device, at the first call there or by
 *     entmax_attn_noalloc_init() (call it once per device, with that device current, before a capture).
 */
int entmax_attn_fwd_noalloc(const entmax_attn_params* p, const void* Q, const void* K, const void* V,
                            const float* beta, const float* gamma, const float* alibi_slopes, void* O, float* tau,
                            uint64_t* stats, void* hip_stream);
/* Looks up the built-in scratch buffer of the current device; 0 on success, ENTMAX_ATTN_LAUNCH_FAILED if the
 * runtime cannot resolve it. */
int entmax_attn_noalloc_init(void);
/* Size of the built-in scratch buffer, a compile-time constant of the library. Host-only. */
size_t entmax_attn_noalloc_scratch_bytes(void);

/* Measurement aid (the matrix-core roofline a benchmark reports beside the data-sheet figure): launches
 * `blocks` workgroups of four waves that each issue 4 * iters independent-chain v_mfma_f32_32x32x16_bf16
 * instructions (2 * 32 * 32 * 16 flops each) and nothing else.  `sink` is device memory for one float (never
 * written in practice).  The caller times the launch. */
int entmax_attn_mfma_probe(int iters, int blocks, float* sink, void* hip_stream);

/*
 * ASEntmax scale projections (Sec. 4.1, the two equations after eq. (asentmax)): the step that produces the
 * attention's per-query beta and gamma (scale_layout 2) from the layer's token embeddings.
 *     beta[b,h,i]  = softplus(<x_{b,i}, w_beta,h>)          > 0
 *     gamma[b,h,i] = gamma_scale * tanh(<x_{b,i}, w_gamma,h>)   in (-gamma_scale, gamma_scale)
 *   X, dX: [B,N,E] contiguous, element type `dtype`, device memory, 16-byte aligned; E a multiple of 16.
 *   Wb, Wg, dWb, dWg: [H,E] fp32 contiguous (row h = head h's projection vector), 16-byte aligned; H <= 16.
 *   beta, gamma, dbeta, dgamma: [B,H,N] fp32 contiguous -- the layout entmax_attn_fwd / entmax_attn_bwd use.
 *   gamma_scale: the constant the paper calls s and gives no value for; must be > 0.
 * Forward: writes beta and gamma.  Backward: from d beta, d gamma (as entmax_attn_bwd returns them) and the
 * forward's beta, gamma it OVERWRITES dX (the projections' contribution only: the caller adds the other paths
 * into X), dWb and dWg.  The backward needs entmax_scale_proj_workspace_bytes(p) bytes of 256-byte aligned
 * workspace (partial sums of dW, added in a fixed order: results are reproducible).
 * Errors as for the attention entry points; nothing is launched when an error is returned before LAUNCH_FAILED.
 */
typedef struct {
  int32_t B, H, N, E; /* batch, heads, tokens per sequence, embedding width */
  int32_t dtype;      /* ENTMAX_ATTN_BF16 or ENTMAX_ATTN_FP32: type of X and dX */
  float gamma_scale;  /* s in gamma = s tanh(.) */
} entmax_scale_proj_params;

int entmax_scale_proj_fwd(const entmax_scale_proj_params* p, const void* X, const float* Wb, const float* Wg, float* beta,
                          float* gamma, void* hip_stream);
int entmax_scale_proj_bwd(const entmax_scale_proj_params* p, const void* X, const float* Wb, const float* Wg,
                          const float* beta, const float* gamma, const float* dbeta, const float* dgamma, void* dX,
                          float* dWb, float* dWg, void* workspace, size_t workspace_bytes, void* hip_stream);
/* Workspace bytes of entmax_scale_proj_bwd; 0 if the parameters are invalid. Host-only. */
size_t entmax_scale_proj_workspace_bytes(const entmax_scale_proj_params* p);

/* Scratch bytes the forward (is_bwd = 0) or backward (is_bwd != 0) needs for
 * these parameters; 0 if the parameters are invalid. Host-only, no GPU call. */
size_t entmax_attn_workspace_bytes(const entmax_attn_params* p, int is_bwd);

/* Smallest size of the optional `saved` buffer that carries the forward's lists to the backward (a larger
 * one holds longer lists, see entmax_attn_fwd); 0 if the parameters are invalid. Host-only, no GPU call. */
size_t entmax_attn_saved_bytes(const entmax_attn_params* p);

/* Validates parameters without touching the GPU: returns the status the
 * entry points would return for them (pointer checks excluded). */
int entmax_attn_check_params(const entmax_attn_params* p);

/* Static, NUL-terminated description of a status code. */
const char* entmax_attn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ENTMAX_ATTN_H */
