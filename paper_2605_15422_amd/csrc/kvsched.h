// Row-block schedule of the KV-stationary backward kernels: the sequence of (sequence, row block, query
// head) steps whose rows can see at least one key of a workgroup's key tile.  Prompt tiles are visited
// by the rows of every sequence of the group (all of them without a window); response tiles only by the
// rows of their own sequence from the diagonal on (Alg. 1, "Q-row blocks in causal support of K_n").
#pragma once
#include "common.h"

namespace dkv {

struct RowStep {
  int64_t grow;   // global row index of the block's first row
  int row0;       // first row of the block inside its sequence
  int nvalid;     // valid rows in the block
  int head;       // query head
};

template <int BM, int BN, bool LOCAL>
struct StepIter {
  const AttnParams& p;
  int hk, key0, key_hi;
  bool is_ctx;
  int seq, seq_end, rb, rb_end, g, row_begin, R;

  __device__ StepIter(const AttnParams& p_, int hk_, bool is_ctx_, int key0_, int seq_lo, int seq_hi)
      : p(p_), hk(hk_), key0(key0_), is_ctx(is_ctx_), seq(seq_lo), seq_end(seq_hi), rb(0), rb_end(0), g(0) {
    if (seq < seq_end) init_seq();
  }
  __device__ void init_seq() {
    row_begin = p.cu ? p.cu[seq] : 0;
    R = p.cu ? (p.cu[seq + 1] - row_begin) : p.total;
    g = 0;
    if (is_ctx) {
      key_hi = min(p.ctx_len, key0 + BN) - 1;
      int rows = R;
      if (LOCAL) rows = min(R, key_hi + p.window - p.ctx_len);
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
