// Work decomposition shared by the Q-stationary kernels (forward, dQ): block decode, KV tile schedule of
// a row block across the two KV regions, and the visibility predicates of the causal / window mask in
// the logical position space (prompt positions 0..P-1, then P + r; Sec. 3.1 and App. F of the paper).
#pragma once
#include "common.h"

namespace dkv {

// ---------------------------------------------------------------------------------------------
// block decode + KV tile schedule shared by fwd and dq
// ---------------------------------------------------------------------------------------------
struct QBlock {
  int hk, hc, mb, seq, row_begin, R, blk_row0;
  int P, ctx_off;   // prompt length and first prompt row of the sequence's group
  int c0, n_ctx, d0, n_dec, n_tiles;
};

template <int BN>
__device__ __forceinline__ bool decode_qblock(const AttnParams& p, QBlock& b) {
  int t = blockIdx.x;
  if (p.window > 0) {
    // Workgroups go to the eight XCDs round-robin by index, each XCD with an L2 of its own.  With a window a row block
    // reads only the K / V tiles of the W keys before it, nearly the same ones as the neighbouring row blocks of its
    // sequence: neighbours are therefore given to the same XCD (block i takes work item (i % 8) * n / 8 + i / 8).  All
    // items carry about the same work here; without a window the work grows with the row index and the round-robin
    // order is the balanced one.
    const int chunk = (int)gridDim.x / 8;
    if (t < chunk * 8) t = (t % 8) * chunk + t / 8;
  }
  b.hk = t % p.Hk; t /= p.Hk;
  b.hc = t % p.HC; t /= p.HC;
  b.mb = p.MB - 1 - (t % p.MB);   // late (long-horizon) row blocks first
  b.seq = t / p.MB;
  b.row_begin = p.cu ? p.cu[b.seq] : 0;
  b.R = p.cu ? (p.cu[b.seq + 1] - b.row_begin) : p.total;
  b.blk_row0 = b.mb * p.BMR;
  if (b.blk_row0 >= b.R) return false;
  b.P = p.seq_ctx ? p.seq_ctx[2 * b.seq + 1] : p.ctx_len;
  b.ctx_off = p.seq_ctx ? p.seq_ctx[2 * b.seq] : 0;
  const int P = b.P;
  const int last_row = min(b.R, b.blk_row0 + p.BMR) - 1;
  b.n_ctx = (P + BN - 1) / BN;
  b.n_dec = last_row / BN + 1;
  b.c0 = 0;
  b.d0 = 0;
  if (p.window > 0) {
    // lowest key any row of the block may see: logical (P + blk_row0) - W + 1
    const int lo = P + b.blk_row0 - p.window + 1;
    if (lo >= P) {
      b.c0 = b.n_ctx;
      b.d0 = (lo - P) / BN;
    } else if (lo > 0) {
      b.c0 = lo / BN;
    }
  }
  b.n_tiles = (b.n_ctx - b.c0) + (b.n_dec - b.d0);
  return true;
}

// Visibility of key `key` (index inside its region) for row `row` of the sequence.
template <bool LOCAL>
__device__ __forceinline__ bool visible(bool is_ctx, int key, int row, int P, int R, int W) {
  if (is_ctx) {
    bool ok = key < P;
    if (LOCAL) ok = ok && (key > P + row - W);
    return ok;
  }
  bool ok = (key <= row) && (key < R);
  if (LOCAL) ok = ok && (key > row - W);
  return ok;
}

// Does any (row, key) pair of a 32-row subtile x BN-key tile need masking?
template <bool LOCAL, int BN>
__device__ __forceinline__ bool tile_needs_mask(bool is_ctx, int key0, int row0, int P, int R, int W) {
  if (is_ctx) {
    bool need = key0 + BN > P;
    if (LOCAL) need = need || (key0 <= P + row0 + 31 - W);
    return need;
  }
  bool need = (key0 + BN - 1 > row0) || (key0 + BN > R);
  if (LOCAL) need = need || (key0 <= row0 + 31 - W);
  return need;
}

// Is any pair of rows [rmin, rmax] x the BN-key tile visible at all?
template <bool LOCAL, int BN>
__device__ __forceinline__ bool tile_active(bool is_ctx, int key0, int rmin, int rmax, int P, int W) {
  if (is_ctx) {
    if (LOCAL) return key0 + BN - 1 > P + rmin - W;
    return true;
  }
  bool act = key0 <= rmax;
  if (LOCAL) act = act && (key0 + BN - 1 > rmin - W);
  return act;
}


// Head packing of one workgroup that owns `nst` 32-row subtiles: GP query heads of the KV group share
// the staged K/V tiles, each with RSH consecutive subtiles (BMR rows).
static inline void fill_packing(AttnParams& p, int nst) {
  int a = p.G, b = nst;
  while (b) {
    const int t = a % b;
    a = b;
    b = t;
  }
  p.GP = a;
  p.RSH = nst / p.GP;
  p.BMR = p.RSH * 32;
  p.HC = p.G / p.GP;
  p.MB = (p.max_rows + p.BMR - 1) / p.BMR;
}

}  // namespace dkv
