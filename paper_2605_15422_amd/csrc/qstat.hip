// Q-stationary kernels: forward (Alg. 3 of the paper, re-tiled for CDNA4) and the dQ half of the
// backward (the dQ line of Alg. 1 evaluated without atomics).
//
// One workgroup owns a block of BMR response rows of one sequence for GP query heads of one KV
// head ("GQA packing": the K/V tiles staged in LDS are shared by all packed heads) and walks the two
// KV regions in logical order: shared-prompt tiles [K_c, V_c] first, then the sequence's own tiles
// [K_d^(i), V_d^(i)] up to the causal horizon (Sec. 3.1: context phase, decoded phase).  Prompt tiles
// need no causal mask; only a partial last prompt tile, the diagonal tiles of the decoded phase and
// window edges are masked.
//
// The score tile is computed transposed, S^T = K Q^T, so that a lane owns one query row (column of
// the MFMA result): row max / row sum are reductions over the lane's own registers plus one exchange
// with lane^32, the per-row rescale factor is a per-lane scalar, and exp(S^T) is already laid out as
// the B operand of O^T += V^T P^T.
#include "common.h"
#include "launch.h"
#include "qsched.h"

namespace dkv {

template <int D, int DSPLIT, int QSUB, int BN, int NWAVES>
struct QCfg {
  static constexpr int NW = NWAVES;
  static constexpr int NT = NW * WAVE;
  static constexpr int RG = NW / DSPLIT;         // row groups (waves that own distinct rows)
  static constexpr int NST = RG * QSUB;          // 32-row subtiles per workgroup
  static constexpr int DC = D / DSPLIT;          // head-dim chunk of one wave
  static constexpr int KS = DC / 16;             // MFMA k-steps over the head-dim chunk
  static constexpr int KVSUB = BN / 32;
  static constexpr int DSUB = DC / 32;
  static constexpr int KPITCH = D + 8;           // row-major K / V image
  static constexpr int TPITCH = BN + 8;          // transposed image
  static_assert(DSPLIT == 1 || QSUB == 1, "head-dim split assumes one row subtile per wave");
};

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
template <int D, int DSPLIT, int QSUB, int BN, int NW, bool LOCAL>
__global__ __launch_bounds__(NW * 64) void fwd_kernel(const AttnParams p) {
  using C = QCfg<D, DSPLIT, QSUB, BN, NW>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  u16* Ks = reinterpret_cast<u16*>(smem_raw);                 // [BN][KPITCH]
  u16* VTs = Ks + BN * C::KPITCH;                             // [D][TPITCH]
  float* xch = reinterpret_cast<float*>(VTs + D * C::TPITCH); // [NW][KVSUB*16][64] (DSPLIT > 1)

  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int dp = wave % DSPLIT, rg = wave / DSPLIT;
  const int P = b.P, R = b.R, W = p.window;
  const float c = p.scale_log2;

  int head[QSUB], row0[QSUB];
  int rmin = 1 << 30, rmax = -1;
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int st = rg * QSUB + qs;
    head[qs] = b.hk * p.G + b.hc * p.GP + st / p.RSH;
    row0[qs] = b.blk_row0 + (st % p.RSH) * 32;
    rmin = min(rmin, row0[qs]);
    rmax = max(rmax, row0[qs] + 31);
  }
  const bool wave_valid = rmin < R;

  // Q fragments (B operand of S^T = K Q^T): lane -> its query row, 8 consecutive head-dim values
  bf16x8 qf[QSUB][C::KS];
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int r = min(row0[qs] + l32, R - 1);
    const u16* qp = p.q.ptr + (int64_t)(b.row_begin + r) * p.q.ts + (int64_t)head[qs] * p.q.hs + dp * C::DC + hi * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) qf[qs][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  f32x16 oacc[QSUB][C::DSUB];
  float m_ref[QSUB], l_sum[QSUB];
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    m_ref[qs] = NEG_BIG;
    l_sum[qs] = 0.f;
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qs][ds][r] = 0.f;
  }

  const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;

  TileRegs<BN, D, C::NT> kreg, vreg;
  auto issue_loads = [&](int it) {
    if (it < n_ctx_run) {
      const int key0 = (b.c0 + it) * BN;
      kreg.load(kc_base + (int64_t)key0 * p.kc.ts, p.kc.ts, P - key0, tid);
      vreg.load(vc_base + (int64_t)key0 * p.vc.ts, p.vc.ts, P - key0, tid);
    } else {
      const int key0 = (b.d0 + it - n_ctx_run) * BN;
      kreg.load(kd_base + (int64_t)key0 * p.kd.ts, p.kd.ts, R - key0, tid);
      vreg.load(vd_base + (int64_t)key0 * p.vd.ts, p.vd.ts, R - key0, tid);
    }
  };
  issue_loads(0);

  for (int it = 0; it < b.n_tiles; ++it) {
    kreg.store_rowmajor(Ks, C::KPITCH, tid);
    vreg.store_transposed(VTs, C::TPITCH, tid);
    __syncthreads();
    if (it + 1 < b.n_tiles) issue_loads(it + 1);

    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const bool active = wave_valid && tile_active<LOCAL, BN>(is_ctx, key0, rmin, rmax, P, W);

    f32x16 s[QSUB][C::KVSUB];
    if (active) {
#pragma unroll
      for (int qs = 0; qs < QSUB; ++qs)
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qs][kv][r] = 0.f;
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv) {
        const u16* ka = Ks + (kv * 32 + l32) * C::KPITCH + dp * C::DC + hi * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(ka + ks * 16);
#pragma unroll
          for (int qs = 0; qs < QSUB; ++qs) s[qs][kv] = mfma32(a, qf[qs][ks], s[qs][kv]);
        }
      }
    }
    if (DSPLIT > 1) {
      // sum the partial scores of the waves that split the head dim
      if (active) {
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) xch[(wave * C::KVSUB * 16 + kv * 16 + r) * 64 + lane] = s[0][kv][r];
      }
      __syncthreads();
      if (active) {
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < DSPLIT; ++w2)
              acc += xch[((rg * DSPLIT + w2) * C::KVSUB * 16 + kv * 16 + r) * 64 + lane];
            s[0][kv][r] = acc;
          }
      }
    }

    if (active) {
#pragma unroll
      for (int qs = 0; qs < QSUB; ++qs) {
        const int row = row0[qs] + l32;
        if (tile_needs_mask<LOCAL, BN>(is_ctx, key0, row0[qs], P, R, W)) {
#pragma unroll
          for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = key0 + kv * 32 + crow(r, hi);
              if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) s[qs][kv][r] = -INFINITY;
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qs][kv][r]);
        mx = xor32_max(mx) * c;
        // rescale lazily: keep the reference maximum until some row's maximum outgrows it by 2^8
        if (__any(mx > m_ref[qs] + 8.0f)) {
          const float mn = fmaxf(m_ref[qs], mx);
          const float alpha = __builtin_amdgcn_exp2f(m_ref[qs] - mn);
          m_ref[qs] = mn;
          l_sum[qs] *= alpha;
#pragma unroll
          for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qs][ds][r] *= alpha;
        }
        float ls = 0.f;
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(s[qs][kv][r] * c - m_ref[qs]);
            s[qs][kv][r] = e;
            ls += e;
          }
        l_sum[qs] += ls;
      }
      // O^T += V^T P^T
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          bf16x8 pb[QSUB];
#pragma unroll
          for (int qs = 0; qs < QSUB; ++qs) {
            float tmp[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) tmp[e] = s[qs][kv][t2 * 8 + e];
            pb[qs] = pack8_bf16(tmp);
          }
#pragma unroll
          for (int ds = 0; ds < C::DSUB; ++ds) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(
                VTs + (dp * C::DC + ds * 32 + l32) * C::TPITCH + kv * 32 + t2 * 16 + hi * 8);
#pragma unroll
            for (int qs = 0; qs < QSUB; ++qs) oacc[qs][ds] = mfma32(a, pb[qs], oacc[qs][ds]);
          }
        }
    }
    __syncthreads();
  }

  // epilogue: normalise, write O (bf16) and LSE (natural log)
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int row = row0[qs] + l32;
    const float l = xor32_sum(l_sum[qs]);
    if (row >= R) continue;
    const float inv = 1.0f / l;
    u16* op = p.out_o.ptr + (int64_t)(b.row_begin + row) * p.out_o.ts + (int64_t)head[qs] * p.out_o.hs + dp * C::DC;
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack2_bf16(oacc[qs][ds][r4 * 4 + 0] * inv, oacc[qs][ds][r4 * 4 + 1] * inv);
        w.y = pack2_bf16(oacc[qs][ds][r4 * 4 + 2] * inv, oacc[qs][ds][r4 * 4 + 3] * inv);
        *reinterpret_cast<u32x2*>(op + ds * 32 + r4 * 8 + hi * 4) = w;
      }
    if (hi == 0 && dp == 0)
      p.lse[(int64_t)head[qs] * p.total + b.row_begin + row] = (m_ref[qs] + log2f(l)) * LN2;
  }
}

// ---------------------------------------------------------------------------------------------
// backward, dQ:  dQ = scale * dS K with dS = P * (dP - D), P = exp(S*scale - LSE), dP = dO V^T
// (Alg. 1, inner loop), evaluated per query block over all its visible key tiles so that dQ is
// accumulated in registers and written once -- no fp32 dQ scratch, no atomics, no convert pass.
// ---------------------------------------------------------------------------------------------
template <int D, int DSPLIT, int QSUB, int BN, int NW, bool LOCAL>
__global__ __launch_bounds__(NW * 64) void dq_kernel(const AttnParams p) {
  using C = QCfg<D, DSPLIT, QSUB, BN, NW>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  u16* Ks = reinterpret_cast<u16*>(smem_raw);                 // [BN][KPITCH]
  u16* Vs = Ks + BN * C::KPITCH;                              // [BN][KPITCH]
  u16* KTs = Vs + BN * C::KPITCH;                             // [D][TPITCH]
  float* xch = reinterpret_cast<float*>(KTs + D * C::TPITCH); // [NW][KVSUB*16][64] (DSPLIT > 1)
  uint32_t* pbuf = reinterpret_cast<uint32_t*>(xch + C::NW * C::KVSUB * 16 * 64);   // [RG][KVSUB][64 lanes][8 words]

  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int dp = wave % DSPLIT, rg = wave / DSPLIT;
  const int P = b.P, R = b.R, W = p.window;
  const float c = p.scale_log2;

  int head[QSUB], row0[QSUB];
  int rmin = 1 << 30, rmax = -1;
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int st = rg * QSUB + qs;
    head[qs] = b.hk * p.G + b.hc * p.GP + st / p.RSH;
    row0[qs] = b.blk_row0 + (st % p.RSH) * 32;
    rmin = min(rmin, row0[qs]);
    rmax = max(rmax, row0[qs] + 31);
  }
  const bool wave_valid = rmin < R;

  bf16x8 qf[QSUB][C::KS], dof[QSUB][C::KS];
  float lse2[QSUB], dvec[QSUB];   // LSE * log2(e), D of the lane's row
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int r = min(row0[qs] + l32, R - 1);
    const int64_t grow = b.row_begin + r;
    const u16* qp = p.q.ptr + grow * p.q.ts + (int64_t)head[qs] * p.q.hs + dp * C::DC + hi * 8;
    const u16* dop = p.dout.ptr + grow * p.dout.ts + (int64_t)head[qs] * p.dout.hs + dp * C::DC + hi * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      qf[qs][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
      dof[qs][ks] = *reinterpret_cast<const bf16x8*>(dop + ks * 16);
    }
    lse2[qs] = p.lse[(int64_t)head[qs] * p.total + grow] * LOG2E;
    dvec[qs] = p.dvec[(int64_t)head[qs] * p.total + grow];
  }

  f32x16 dqacc[QSUB][C::DSUB];
#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs)
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
      for (int r = 0; r < 16; ++r) dqacc[qs][ds][r] = 0.f;

  const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;

  TileRegs<BN, D, C::NT> kreg, vreg;
  auto issue_loads = [&](int it) {
    if (it < n_ctx_run) {
      const int key0 = (b.c0 + it) * BN;
      kreg.load(kc_base + (int64_t)key0 * p.kc.ts, p.kc.ts, P - key0, tid);
      vreg.load(vc_base + (int64_t)key0 * p.vc.ts, p.vc.ts, P - key0, tid);
    } else {
      const int key0 = (b.d0 + it - n_ctx_run) * BN;
      kreg.load(kd_base + (int64_t)key0 * p.kd.ts, p.kd.ts, R - key0, tid);
      vreg.load(vd_base + (int64_t)key0 * p.vd.ts, p.vd.ts, R - key0, tid);
    }
  };
  issue_loads(0);

  for (int it = 0; it < b.n_tiles; ++it) {
    kreg.store_rowmajor(Ks, C::KPITCH, tid);
    kreg.store_transposed(KTs, C::TPITCH, tid);
    vreg.store_rowmajor(Vs, C::KPITCH, tid);
    __syncthreads();
    if (it + 1 < b.n_tiles) issue_loads(it + 1);

    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const bool active = wave_valid && tile_active<LOCAL, BN>(is_ctx, key0, rmin, rmax, P, W);

    f32x16 s[QSUB][C::KVSUB], dpt[QSUB][C::KVSUB];
    if (active) {
#pragma unroll
      for (int qs = 0; qs < QSUB; ++qs)
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            s[qs][kv][r] = 0.f;
            dpt[qs][kv][r] = 0.f;
          }
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv) {
        const u16* ka = Ks + (kv * 32 + l32) * C::KPITCH + dp * C::DC + hi * 8;
        const u16* va = Vs + (kv * 32 + l32) * C::KPITCH + dp * C::DC + hi * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(ka + ks * 16);
          const bf16x8 a2 = *reinterpret_cast<const bf16x8*>(va + ks * 16);
#pragma unroll
          for (int qs = 0; qs < QSUB; ++qs) {
            s[qs][kv] = mfma32(a, qf[qs][ks], s[qs][kv]);
            dpt[qs][kv] = mfma32(a2, dof[qs][ks], dpt[qs][kv]);
          }
        }
      }
    }
    uint32_t* img = pbuf + rg * (C::KVSUB * 64 * 8);   // dS^T operand image of the row group (DSPLIT > 1)
    if (DSPLIT > 1) {
      // The waves of a row group hold partial S and dP tiles (their part of the head dim).  Each of them sums RPW
      // of the 16 accumulator registers of every subtile over the group (S, then dP, through one buffer),
      // evaluates dS for those and publishes it as bf16 words of the operand image [lane][8 words]; every wave
      // then reads the whole image, and each exponential is evaluated once per row group.
      constexpr int PER = C::KVSUB * 16, RPW = 16 / DSPLIT;
      float ssum[C::KVSUB][RPW], dsum[C::KVSUB][RPW];
#pragma unroll
      for (int which = 0; which < 2; ++which) {
        if (which) __syncthreads();
        if (active) {
#pragma unroll
          for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              xch[(wave * PER + kv * 16 + r) * 64 + lane] = which ? dpt[0][kv][r] : s[0][kv][r];
        }
        __syncthreads();
        if (active) {
#pragma unroll
          for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
              float acc = 0.f;
#pragma unroll
              for (int w2 = 0; w2 < DSPLIT; ++w2)
                acc += xch[((rg * DSPLIT + w2) * PER + kv * 16 + dp * RPW + j) * 64 + lane];
              if (which) dsum[kv][j] = acc; else ssum[kv][j] = acc;
            }
        }
      }
      if (active) {
        const int row = row0[0] + l32;
        const bool need = tile_needs_mask<LOCAL, BN>(is_ctx, key0, row0[0], P, R, W);
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv) {
          float dsv[RPW];
#pragma unroll
          for (int j = 0; j < RPW; ++j) {
            float e = __builtin_amdgcn_exp2f(ssum[kv][j] * c - lse2[0]);
            if (need) {
              const int key = key0 + kv * 32 + crow(dp * RPW + j, hi);
              if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) e = 0.f;
            }
            dsv[j] = e * (dsum[kv][j] - dvec[0]);
          }
#pragma unroll
          for (int w = 0; w < RPW / 2; ++w)
            img[(kv * 64 + lane) * 8 + dp * (RPW / 2) + w] = pack2_bf16(dsv[2 * w], dsv[2 * w + 1]);
        }
      }
      __syncthreads();
    } else if (active) {
#pragma unroll
      for (int qs = 0; qs < QSUB; ++qs) {
        const int row = row0[qs] + l32;
        const bool need = tile_needs_mask<LOCAL, BN>(is_ctx, key0, row0[qs], P, R, W);
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float e = __builtin_amdgcn_exp2f(s[qs][kv][r] * c - lse2[qs]);
            if (need) {
              const int key = key0 + kv * 32 + crow(r, hi);
              if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) e = 0.f;
            }
            s[qs][kv][r] = e * (dpt[qs][kv][r] - dvec[qs]);   // dS^T
          }
        }
      }
    }

    if (active) {
      // dQ^T += K^T dS^T
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          bf16x8 pb[QSUB];
          if (DSPLIT > 1) {
            pb[0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(img + (kv * 64 + lane) * 8 + t2 * 4));
          } else {
#pragma unroll
            for (int qs = 0; qs < QSUB; ++qs) {
              float tmp[8];
#pragma unroll
              for (int e = 0; e < 8; ++e) tmp[e] = s[qs][kv][t2 * 8 + e];
              pb[qs] = pack8_bf16(tmp);
            }
          }
#pragma unroll
          for (int ds = 0; ds < C::DSUB; ++ds) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(
                KTs + (dp * C::DC + ds * 32 + l32) * C::TPITCH + kv * 32 + t2 * 16 + hi * 8);
#pragma unroll
            for (int qs = 0; qs < QSUB; ++qs) dqacc[qs][ds] = mfma32(a, pb[qs], dqacc[qs][ds]);
          }
        }
    }
    __syncthreads();
  }

#pragma unroll
  for (int qs = 0; qs < QSUB; ++qs) {
    const int row = row0[qs] + l32;
    if (row >= R) continue;
    u16* op = p.dq.ptr + (int64_t)(b.row_begin + row) * p.dq.ts + (int64_t)head[qs] * p.dq.hs + dp * C::DC;
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack2_bf16(dqacc[qs][ds][r4 * 4 + 0] * p.scale, dqacc[qs][ds][r4 * 4 + 1] * p.scale);
        w.y = pack2_bf16(dqacc[qs][ds][r4 * 4 + 2] * p.scale, dqacc[qs][ds][r4 * 4 + 3] * p.scale);
        *reinterpret_cast<u32x2*>(op + ds * 32 + r4 * 8 + hi * 4) = w;
      }
  }
}

// ---------------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------------
template <int D, int DSPLIT, int QSUB, int BN, int NW, bool LOCAL>
static hipError_t launch_fwd_t(AttnParams p, hipStream_t st) {
  using C = QCfg<D, DSPLIT, QSUB, BN, NW>;
  fill_packing(p, C::NST);
  size_t smem = (size_t)(BN * C::KPITCH + D * C::TPITCH) * 2;
  if (DSPLIT > 1) smem += (size_t)C::NW * C::KVSUB * 16 * 64 * 4;
  auto kern = fwd_kernel<D, DSPLIT, QSUB, BN, NW, LOCAL>;
  hipError_t e = ensure_dynamic_lds<fwd_kernel<D, DSPLIT, QSUB, BN, NW, LOCAL>>(smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(NW * 64), smem, st, p);
  return hipGetLastError();
}

template <int D, int DSPLIT, int QSUB, int BN, int NW, bool LOCAL>
static hipError_t launch_dq_t(AttnParams p, hipStream_t st) {
  using C = QCfg<D, DSPLIT, QSUB, BN, NW>;
  fill_packing(p, C::NST);
  size_t smem = (size_t)(2 * BN * C::KPITCH + D * C::TPITCH) * 2;
  if (DSPLIT > 1) smem += (size_t)C::NW * C::KVSUB * 16 * 64 * 4 + (size_t)C::RG * C::KVSUB * 64 * 8 * 4;
  auto kern = dq_kernel<D, DSPLIT, QSUB, BN, NW, LOCAL>;
  hipError_t e = ensure_dynamic_lds<dq_kernel<D, DSPLIT, QSUB, BN, NW, LOCAL>>(smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(NW * 64), smem, st, p);
  return hipGetLastError();
}

// Per head dim: <D, DSPLIT, QSUB, BN, NW>.  Head dims 256 (forward) and 512 split the head dim over the waves of
// a row group and run eight waves, two per SIMD: the per-wave state then fits 256 registers without spills, which
// more than pays for the exchange of partial scores through LDS (measured: forward 256 1.55x, dQ 512 1.9x faster
// than four waves with twice the registers each; dQ 256 is faster unsplit).
hipError_t launch_fwd(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_fwd_t<64, 1, 2, 64, 4, true>(p, st) : launch_fwd_t<64, 1, 2, 64, 4, false>(p, st);
    case 96:  return local ? launch_fwd_t<96, 1, 2, 64, 4, true>(p, st) : launch_fwd_t<96, 1, 2, 64, 4, false>(p, st);
    case 128: return local ? launch_fwd_t<128, 1, 2, 64, 4, true>(p, st) : launch_fwd_t<128, 1, 2, 64, 4, false>(p, st);
    case 192: return local ? launch_fwd_t<192, 1, 1, 64, 4, true>(p, st) : launch_fwd_t<192, 1, 1, 64, 4, false>(p, st);
    case 256: return local ? launch_fwd_t<256, 2, 1, 64, 8, true>(p, st) : launch_fwd_t<256, 2, 1, 64, 8, false>(p, st);
    case 512: return launch_fwd_t<512, 4, 1, 32, 8, false>(p, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_dq(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_dq_t<64, 1, 2, 64, 4, true>(p, st) : launch_dq_t<64, 1, 2, 64, 4, false>(p, st);
    case 96:  return local ? launch_dq_t<96, 1, 1, 64, 4, true>(p, st) : launch_dq_t<96, 1, 1, 64, 4, false>(p, st);
    case 128: return local ? launch_dq_t<128, 1, 1, 64, 4, true>(p, st) : launch_dq_t<128, 1, 1, 64, 4, false>(p, st);
    case 192: return local ? launch_dq_t<192, 1, 1, 32, 4, true>(p, st) : launch_dq_t<192, 1, 1, 32, 4, false>(p, st);
    case 256: return local ? launch_dq_t<256, 1, 1, 32, 4, true>(p, st) : launch_dq_t<256, 1, 1, 32, 4, false>(p, st);
    case 512: return launch_dq_t<512, 4, 1, 32, 8, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
