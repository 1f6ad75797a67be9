// Sizes shared by the host-side layout code (plain C++, no HIP) and the kernels.
#pragma once
#include <stddef.h>

namespace entmax {

constexpr int kThreads = 256;    // 4 wave64 per workgroup
constexpr int kWaves = 4;
constexpr int kBlockRows = 128;  // rows (queries or keys) owned by a workgroup: 32 per wave

// The long-sequence list kernel that takes two adjacent query blocks per workgroup runs only where its launch has
// at least this many workgroups (three for each of the 256 CUs).
constexpr int kPairMinWorkgroups = 768;
// The forward's list kernel takes one query block per workgroup instead of a causal pair where the pairs would
// leave the chip short of workgroups (fewer than three per CU; B 8, H 12, n 1024: 51 -> 47 us).  Launches of less
// than half a workgroup per CU are as long as their longest block either way and keep the pairs.
constexpr int kUnpairedBelowWorkgroups = 768;
constexpr int kUnpairedFromWorkgroups = 128;
inline bool fwd_lists_unpaired(long long heads, int nqb) {
  const long long pairs = heads * ((nqb + 1) / 2);
  return nqb >= 2 && pairs >= kUnpairedFromWorkgroups && pairs < kUnpairedBelowWorkgroups;
}

constexpr int kCandCap = 32;     // candidate entries per lane = per half row (forward lists)
constexpr int kBwdCap = 16;      // support entries per lane = per half row (the lists the backward works from)
constexpr int kListStride = 64;  // lists are stored slot-major per wave: entry s of the 64 lanes together
// The `saved` buffer packs the rows' support lists into a pool: the size the library asks for holds this many
// entries per row on average (a larger buffer gives a larger pool), at least kSavedPoolFloor (one block's worst
// case), plus kSavedPoolPad entries behind the end that speculative reads may touch.
// A packed entry's first word is the key index (22 bits: Nk <= 2^22) with, above it, the entry's arrival number
// among its key's entries, so that the backward knows its place in the key's segment without asking; the largest
// value stands for "later than that" (those entries take their place from a cursor in the backward).
constexpr int kSavedKeyBits = 22;
constexpr unsigned kSavedRankMost = (1u << (32 - kSavedKeyBits)) - 1u;  // 1023
// Values of a block's flag in the `saved` buffer besides 0 (the backward takes its list path): the forward wrote
// lists for the block's rows and numbered their entries before it found a list too long (the backward's tiled
// kernels take the block, and the entries' places in the key-major arrays are filled with zeros), or it wrote none.
constexpr int kBlockListsUnused = 1;
constexpr int kBlockNoLists = 2;
constexpr int kSavedPerRow = 6;
constexpr int kSavedPoolFloor = kThreads * kBwdCap;
constexpr int kSavedPoolPad = 4;
// The pool is cut into up to kSavedSubPools equal parts with a cursor each, and the 32-row groups take their part
// in turn (group number modulo the number of parts): pieces are handed out by a returning atomic, and atomics on
// one address queue up behind each other (one cursor for the 6144 groups of a 4 x 12 x 4096 problem doubled the
// time of the kernel that fills the pool).  The cursors sit kSavedCursorStride bytes apart so that they do not
// share a memory channel either.  Every part serves at least kSavedGroupsPerPart groups.
constexpr int kSavedSubPools = 64;
constexpr int kSavedCursorStride = 4352;
constexpr int kSavedGroupsPerPart = 16;
inline int saved_pool_parts(long long groups) {
  int n = 1;
  while (n < kSavedSubPools && groups / (2 * n) >= kSavedGroupsPerPart) n *= 2;
  return n;
}

// Tiled forward behind the list kernels: up to this many flagged blocks run four workgroups to a block (a few long
// blocks alone on the chip are bound by their own serial length), more run as block pairs (bound by throughput).
constexpr int kSplitMaxBlocks = 256;

// Sweep scratch of the list kernels: CAP cells of (4 raw scores, first key) per thread.
constexpr int kCellGroups = 1;  // 4-key accumulator groups per cell
constexpr size_t cell_bytes_per_workgroup(int cap) { return (size_t)kThreads * cap * (16 * kCellGroups + 4); }

// Decode shapes: up to kDecodeRows query rows always take the split-key kernels, up to kDecodeRowsLong
// when the keys are at least kDecodeLongRatio times as many.
constexpr int kDecodeRows = 8;
constexpr int kDecodeRowsLong = 64;
constexpr int kDecodeMfmaRows = 16;  // from this many rows on the scores come from the matrix cores (measured: 9 rows
                                     // 91 us with per-row dot products against 114 us, 16 rows 131 against 121)
constexpr int kDecodeLongRatio = 64;
constexpr int kDecodeChunk = 512;  // keys per workgroup of the score kernel (64 to 128 KB of K); 256 to 2048 measured alike
inline bool decode_shape(int Nq, int Nk) {
  return Nq <= kDecodeRows || (Nq <= kDecodeRowsLong && (long long)Nk >= (long long)kDecodeLongRatio * Nq);
}

}  // namespace entmax
