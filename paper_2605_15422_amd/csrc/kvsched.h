// Row-block schedule of the KV-stationary backward kernels: the sequence of (sequence, row block, query
// head) steps whose rows can see at least one key of a workgroup's key tile.  Prompt tiles are visited
// by the rows of every sequence of the group (all of them without a window); response tiles only by the
// rows of their own sequence from the diagonal on (Alg. 1, "Q-row blocks in causal support of K_n").
#pragma once
#include "common.h"

namespace dkv {

// Block decode of the KV-stationary kernels: prompt tiles first (heavy), then response tiles.  With several prompt
// groups, the prompt tiles of group g are the blocks [g * n_ctx_tiles, (g + 1) * n_ctx_tiles) x Hk x n_split, where
// n_ctx_tiles covers the longest prompt; tiles past a shorter prompt have nothing to do.
struct KVBlock {
  bool is_ctx;
  int hk, key0, seq_lo, seq_hi;
  int P, ctx_off;   // prompt length and first prompt row of the block's group
};

// false: the block owns no key (beyond its prompt or its response)
__device__ __forceinline__ bool decode_kvblock(const AttnParams& p, int BN, KVBlock& b) {
  const int n_grp = p.grp ? p.n_groups : 1;
  const int ctx_blocks = n_grp * p.n_ctx_tiles * p.Hk * p.n_split;
  int bid = blockIdx.x;
  if (bid < ctx_blocks) {
    b.is_ctx = true;
    b.hk = bid % p.Hk;
    int t = bid / p.Hk;
    const int split = t % p.n_split;
    t /= p.n_split;
    b.key0 = (t % p.n_ctx_tiles) * BN;
    const int g = t / p.n_ctx_tiles;
    int s0 = 0, s1 = p.n_seqs;
    b.P = p.ctx_len;
    b.ctx_off = 0;
    if (p.grp) {
      b.ctx_off = p.grp[4 * g];
      b.P = p.grp[4 * g + 1];
      s0 = p.grp[4 * g + 2];
      s1 = p.grp[4 * g + 3];
    }
    if (b.key0 >= b.P) return false;
    const int n = s1 - s0;
    b.seq_lo = s0 + (int)((int64_t)n * split / p.n_split);
    b.seq_hi = s0 + (int)((int64_t)n * (split + 1) / p.n_split);
    // a part without sequences adds nothing to the accumulators; an unsplit tile still has to write its zeros
    if (p.n_split > 1 && b.seq_lo == b.seq_hi) return false;
    return true;
  }
  bid -= ctx_blocks;
  if (p.window > 0) {
    // Workgroups go to the eight XCDs round-robin by index, each XCD with an L2 of its own.  With a window a response
    // tile reads only the W + BN rows behind its keys, rows that its neighbours read as well: neighbouring tiles are
    // therefore given to the same XCD (block i takes tile (i % 8) * n / 8 + i / 8), where one fetch from memory then
    // serves many of them.  All tiles carry about the same work here, so the XCDs stay balanced; without a window the
    // work falls with the key index and the round-robin order is the balanced one.
    const int chunk = ((int)gridDim.x - ctx_blocks) / 8;
    if (bid < chunk * 8) bid = (bid % 8) * chunk + bid / 8;
  }
  b.is_ctx = false;
  b.hk = bid % p.Hk;
  const int t = bid / p.Hk;
  b.key0 = (t % p.n_dec_tiles) * BN;
  b.seq_lo = t / p.n_dec_tiles;
  b.seq_hi = b.seq_lo + 1;
  b.P = p.seq_ctx ? p.seq_ctx[2 * b.seq_lo + 1] : p.ctx_len;
  b.ctx_off = 0;
  const int rb0 = p.cu ? p.cu[b.seq_lo] : 0;
  const int Rs = p.cu ? (p.cu[b.seq_lo + 1] - rb0) : p.total;
  return b.key0 < Rs;
}

struct RowStep {
  int64_t grow;   // global row index of the block's first row
  int row0;       // first row of the block inside its sequence
  int nvalid;     // valid rows in the block
  int head;       // query head
};

template <int BM, int BN, bool LOCAL>
struct StepIter {
  const AttnParams& p;
  int hk, key0, key_hi, P;
  bool is_ctx;
  int seq, seq_end, rb, rb_end, g, row_begin, R;

  __device__ StepIter(const AttnParams& p_, int hk_, bool is_ctx_, int key0_, int seq_lo, int seq_hi, int P_)
      : p(p_), hk(hk_), key0(key0_), P(P_), is_ctx(is_ctx_), seq(seq_lo), seq_end(seq_hi), rb(0), rb_end(0), g(0) {
    if (seq < seq_end) init_seq();
  }
  __device__ void init_seq() {
    row_begin = p.cu ? p.cu[seq] : 0;
    R = p.cu ? (p.cu[seq + 1] - row_begin) : p.total;
    g = 0;
    if (is_ctx) {
      key_hi = min(P, key0 + BN) - 1;
      int rows = R;
      if (LOCAL) rows = min(R, key_hi + p.window - P);
      rb = 0;
      rb_end = rows > 0 ? (rows + BM - 1) / BM : 0;
    } else {
      key_hi = min(R, key0 + BN) - 1;
      int rows = R;
      if (LOCAL) rows = min(R, key_hi + p.window);
      rb = key0 / BM;
      rb_end = (rows + BM - 1) / BM;
    }
  }
  __device__ bool next(RowStep& s) {
    while (seq < seq_end) {
      if (rb < rb_end) {
        s.row0 = rb * BM;
        s.grow = (int64_t)row_begin + s.row0;
        s.nvalid = min(BM, R - s.row0);
        s.head = hk * p.G + g;
        if (++g == p.G) {
          g = 0;
          ++rb;
        }
        return true;
      }
      ++seq;
      if (seq < seq_end) init_seq();
    }
    return false;
  }
};

}  // namespace dkv
