// KV-stationary backward kernel: dK and dV (Alg. 1 of the paper without its dQ line).
//
// A workgroup owns one tile of BN keys of one KV head and keeps K, V (MFMA operands) and the fp32
// dK / dV accumulators in registers while it streams query-row blocks through LDS:
//   S = Q K^T,  P = exp(S*scale - LSE),  dV += P^T dO,  dP = dO V^T,  dS = P * (dP - D),  dK += dS^T Q.
//
// Shared-prompt tiles (keys of K_c / V_c): the paper launches one block per (tile, sequence, head) and
// resolves the N-way write race on dK_c / dV_c with fp32 atomics into a scratch buffer (Sec. 3.2).  Here
// ONE workgroup per (prompt tile, KV head) walks the rows of ALL N sequences and all G heads of the
// group, so the N*G partial gradients are summed in fp32 registers and cast to bf16 exactly once -- the
// same "sum in fp32, cast at the end" precision profile with no race, no scratch and a deterministic
// result.  When there are too few prompt tiles to fill the chip the sequence loop is cut in n_split
// parts that add their fp32 partials atomically into an accumulator (the paper's Stage 1), followed by
// the cast kernel (Stage 2, Alg. 2); the same path serves callers that want the Call-1 + Call-2 sum in
// fp32.
//
// Response tiles (keys of K_d^(i) / V_d^(i)) belong to one sequence: the workgroup walks that sequence's
// rows from the diagonal on and writes bf16 directly (Alg. 1, "decoded block: no race").
#include "common.h"
#include "launch.h"
#include "kvsched.h"

namespace dkv {

template <int D, int DSPLIT, int NW, int BM, int TPAD>
struct KCfg {
  static constexpr int NT = NW * WAVE;
  static constexpr int KVS = NW / DSPLIT;        // 32-key subtiles per workgroup
  static constexpr int BN = 32 * KVS;
  static constexpr int DC = D / DSPLIT;
  static constexpr int KS = DC / 16;
  static constexpr int DSUB = DC / 32;
  static constexpr int QSUB = BM / 32;
  static constexpr int QPITCH = D + 8;
  static constexpr int TPITCH = BM + TPAD;
  // The exchange buffer of a head-dim split ([S | dP][NW][16][64] floats) lies over the row-major images, which are
  // dead by then (one row subtile per step), when it fits there; otherwise it gets LDS of its own.
  static_assert(DSPLIT == 1 || QSUB == 1, "a head-dim split takes one row subtile per step");
  static constexpr size_t XCH_BYTES = (size_t)2 * NW * 16 * 64 * 4;
  static constexpr bool XCH_OVERLAY = XCH_BYTES <= (size_t)2 * BM * QPITCH * 2;
  static constexpr size_t base_bytes() { return (size_t)(2 * BM * QPITCH + 2 * D * TPITCH) * 2 + 2 * BM * 4; }
  static constexpr size_t smem_bytes() {
    size_t s = base_bytes();
    if (DSPLIT > 1) s += (size_t)KVS * 2 * 64 * 8 * 4;   // bf16 operand images of P and dS per key group
    if (DSPLIT > 1 && !XCH_OVERLAY) s += XCH_BYTES;
    return s;
  }
};

template <int D, int DSPLIT, int NW, int BM, int TPAD, bool LOCAL>
__global__ __launch_bounds__(NW * 64) void dkdv_kernel(const AttnParams p) {
  using C = KCfg<D, DSPLIT, NW, BM, TPAD>;
  constexpr int BN = C::BN;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  u16* Qs = reinterpret_cast<u16*>(smem_raw);           // [BM][QPITCH]
  u16* dOs = Qs + BM * C::QPITCH;                       // [BM][QPITCH]
  u16* QTs = dOs + BM * C::QPITCH;                      // [D][TPITCH]
  u16* dOTs = QTs + D * C::TPITCH;                      // [D][TPITCH]
  float* lseL = reinterpret_cast<float*>(dOTs + D * C::TPITCH);  // [BM] LSE * log2(e)
  float* DL = lseL + BM;                                // [BM]
  uint32_t* pbuf = reinterpret_cast<uint32_t*>(DL + BM); // [KVS][P | dS][64 lanes][8 words] (DSPLIT > 1)
  float* xch = C::XCH_OVERLAY ? reinterpret_cast<float*>(smem_raw)      // [S | dP][NW][16][64] (DSPLIT > 1)
                              : reinterpret_cast<float*>(pbuf + C::KVS * 2 * 64 * 8);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int dp = wave % DSPLIT, kvs = wave / DSPLIT;
  const int W = p.window;
  const float c = p.scale_log2;

  KVBlock kb;
  if (!decode_kvblock(p, BN, kb)) return;
  const bool is_ctx = kb.is_ctx;
  const int hk = kb.hk, key0 = kb.key0, seq_lo = kb.seq_lo, seq_hi = kb.seq_hi, P = kb.P;

  // ---- stationary K, V fragments (B operands: lane -> key, 8 consecutive head-dim values)
  int region_len, key_row_begin = 0;
  const u16 *kbase, *vbase;
  int64_t kts, vts;
  if (is_ctx) {
    region_len = P;
    key_row_begin = kb.ctx_off;
    kbase = p.kc.ptr + (int64_t)kb.ctx_off * p.kc.ts + (int64_t)hk * p.kc.hs;
    vbase = p.vc.ptr + (int64_t)kb.ctx_off * p.vc.ts + (int64_t)hk * p.vc.hs;
    kts = p.kc.ts;
    vts = p.vc.ts;
  } else {
    key_row_begin = p.cu ? p.cu[seq_lo] : 0;
    region_len = p.cu ? (p.cu[seq_lo + 1] - key_row_begin) : p.total;
    kbase = p.kd.ptr + (int64_t)key_row_begin * p.kd.ts + (int64_t)hk * p.kd.hs;
    vbase = p.vd.ptr + (int64_t)key_row_begin * p.vd.ts + (int64_t)hk * p.vd.hs;
    kts = p.kd.ts;
    vts = p.vd.ts;
  }
  const int my_key = key0 + kvs * 32 + l32;
  bf16x8 kf[C::KS], vf[C::KS];
  {
    const int kr = min(my_key, region_len - 1);   // clamp: gradients of padded keys are never stored
    const u16* kp = kbase + (int64_t)kr * kts + dp * C::DC + hi * 8;
    const u16* vp = vbase + (int64_t)kr * vts + dp * C::DC + hi * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
      vf[ks] = *reinterpret_cast<const bf16x8*>(vp + ks * 16);
    }
  }

  f32x16 dk[C::DSUB], dv[C::DSUB];
#pragma unroll
  for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[ds][r] = 0.f;
      dv[ds][r] = 0.f;
    }

  StepIter<BM, BN, LOCAL> iter(p, hk, is_ctx, key0, seq_lo, seq_hi, P);
  TileRegs<BM, D, C::NT> qreg, doreg;
  float lse_pf = LSE_MASKED, d_pf = 0.f;
  auto issue_loads = [&](const RowStep& s) {
    qreg.load(p.q.ptr + s.grow * p.q.ts + (int64_t)s.head * p.q.hs, p.q.ts, s.nvalid, tid);
    doreg.load(p.dout.ptr + s.grow * p.dout.ts + (int64_t)s.head * p.dout.hs, p.dout.ts, s.nvalid, tid);
    if (tid < BM) {
      const bool ok = tid < s.nvalid;
      // (scaled by log2(e) when it is stored to LDS: arithmetic on the value here would wait for every load in flight)
      lse_pf = ok ? p.lse[(int64_t)s.head * p.total + s.grow + tid] : LSE_MASKED;
      d_pf = ok ? p.dvec[(int64_t)s.head * p.total + s.grow + tid] : 0.f;
    }
  };

  RowStep cur, nxt;
  bool has = iter.next(cur);
  if (has) issue_loads(cur);
  const int wave_key_lo = key0 + kvs * 32, wave_key_hi = wave_key_lo + 31;

  while (has) {
    qreg.store_rowmajor(Qs, C::QPITCH, tid);
    qreg.store_transposed(QTs, C::TPITCH, tid);
    doreg.store_rowmajor(dOs, C::QPITCH, tid);
    doreg.store_transposed(dOTs, C::TPITCH, tid);
    if (tid < BM) {
      lseL[tid] = lse_pf * LOG2E;
      DL[tid] = d_pf;
    }
    __syncthreads();
    const bool has_n = iter.next(nxt);
    if (has_n) issue_loads(nxt);

#pragma unroll
    for (int qs = 0; qs < C::QSUB; ++qs) {
      const int srow0 = cur.row0 + qs * 32;   // first row of the subtile inside its sequence
      // any visible (row, key) pair for this wave's 32 keys?
      bool active = srow0 < cur.row0 + cur.nvalid;
      bool need_mask = false;
      if (is_ctx) {
        if (LOCAL) {
          active = active && (wave_key_hi > P + srow0 - W);
          need_mask = wave_key_lo <= P + srow0 + 31 - W;
        }
      } else {
        active = active && (wave_key_lo <= srow0 + 31);
        need_mask = wave_key_hi > srow0;
        if (LOCAL) {
          active = active && (wave_key_hi > srow0 - W);
          need_mask = need_mask || (wave_key_lo <= srow0 + 31 - W);
        }
      }

      f32x16 s, dpv;
      if (active) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[r] = 0.f;
          dpv[r] = 0.f;
        }
        const u16* qa = Qs + (qs * 32 + l32) * C::QPITCH + dp * C::DC + hi * 8;
        const u16* da = dOs + (qs * 32 + l32) * C::QPITCH + dp * C::DC + hi * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
          s = mfma32(*reinterpret_cast<const bf16x8*>(qa + ks * 16), kf[ks], s);
          dpv = mfma32(*reinterpret_cast<const bf16x8*>(da + ks * 16), vf[ks], dpv);
        }
      }
      bf16x8 pa[2], dsa[2];   // P^T and dS^T of the subtile as MFMA operands (k-steps 0, 1 over the 32 rows)
      if (DSPLIT > 1) {
        // The waves of a key group hold partial S and dP tiles (their part of the head dim).  Each of them sums
        // RPW of the 16 accumulator registers over the group (S and dP), evaluates P and dS
        // for those, and publishes them as bf16 words of the operand image [lane][8 words]; every wave then
        // reads the whole image: 2 x 16 bytes per operand instead of DSPLIT x 16 partial values, and each
        // exponential is evaluated once per key group.
        constexpr int RPW = 16 / DSPLIT;
        float ssum[RPW], dsum[RPW];
        if (C::XCH_OVERLAY) __syncthreads();   // every wave has read its row-major operands: the buffer may overwrite them
        if (active) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            xch[(wave * 16 + r) * 64 + lane] = s[r];
            xch[((NW + wave) * 16 + r) * 64 + lane] = dpv[r];
          }
        }
        __syncthreads();
        if (active) {
#pragma unroll
          for (int j = 0; j < RPW; ++j) {
            float a0 = 0.f, a1 = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < DSPLIT; ++w2) {
              a0 += xch[((kvs * DSPLIT + w2) * 16 + dp * RPW + j) * 64 + lane];
              a1 += xch[((NW + kvs * DSPLIT + w2) * 16 + dp * RPW + j) * 64 + lane];
            }
            ssum[j] = a0;
            dsum[j] = a1;
          }
        }
        uint32_t* img = pbuf + kvs * (2 * 64 * 8);
        if (active) {
          float pv[RPW], dsv[RPW];
#pragma unroll
          for (int j = 0; j < RPW; ++j) {
            const int rl = crow(dp * RPW + j, hi);
            float e = __builtin_amdgcn_exp2f(ssum[j] * c - lseL[qs * 32 + rl]);
            if (need_mask) {
              const int row = srow0 + rl;
              bool ok;
              if (is_ctx) ok = !LOCAL || (my_key > P + row - W);
              else ok = (my_key <= row) && (!LOCAL || (my_key > row - W));
              if (!ok) e = 0.f;
            }
            pv[j] = e;
            dsv[j] = e * (dsum[j] - DL[qs * 32 + rl]);
          }
#pragma unroll
          for (int w = 0; w < RPW / 2; ++w) {
            img[lane * 8 + dp * (RPW / 2) + w] = pack2_bf16(pv[2 * w], pv[2 * w + 1]);
            img[64 * 8 + lane * 8 + dp * (RPW / 2) + w] = pack2_bf16(dsv[2 * w], dsv[2 * w + 1]);
          }
        }
        __syncthreads();
        if (active) {
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2) {
            pa[t2] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(img + lane * 8 + t2 * 4));
            dsa[t2] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(img + 64 * 8 + lane * 8 + t2 * 4));
          }
        }
      } else if (active) {
        float lr[16], dr[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 a = *reinterpret_cast<const f32x4*>(lseL + qs * 32 + r4 * 8 + hi * 4);
          const f32x4 b2 = *reinterpret_cast<const f32x4*>(DL + qs * 32 + r4 * 8 + hi * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            lr[r4 * 4 + e] = a[e];
            dr[r4 * 4 + e] = b2[e];
          }
        }
        float pv[16], dsv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float e = __builtin_amdgcn_exp2f(s[r] * c - lr[r]);
          if (need_mask) {
            const int row = srow0 + crow(r, hi);
            bool ok;
            if (is_ctx) ok = !LOCAL || (my_key > P + row - W);
            else ok = (my_key <= row) && (!LOCAL || (my_key > row - W));
            if (!ok) e = 0.f;
          }
          pv[r] = e;
          dsv[r] = e * (dpv[r] - dr[r]);
        }
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          pa[t2] = pack8_bf16(pv + t2 * 8);
          dsa[t2] = pack8_bf16(dsv + t2 * 8);
        }
      }
      if (active) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int ds = 0; ds < C::DSUB; ++ds) {
            const int off = (dp * C::DC + ds * 32 + l32) * C::TPITCH + qs * 32 + t2 * 16 + hi * 8;
            dv[ds] = mfma32(pa[t2], *reinterpret_cast<const bf16x8*>(dOTs + off), dv[ds]);
            dk[ds] = mfma32(dsa[t2], *reinterpret_cast<const bf16x8*>(QTs + off), dk[ds]);
          }
      }
    }
    __syncthreads();
    cur = nxt;
    has = has_n;
  }

  // ---- epilogue: C layout -> lane owns head-dim column, register r owns key crow(r)
  const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
  float* acc_k = is_ctx ? p.dkc_acc : p.dkd_acc;
  float* acc_v = is_ctx ? p.dvc_acc : p.dvd_acc;
#pragma unroll
  for (int ds = 0; ds < C::DSUB; ++ds) {
    const int dcol = dp * C::DC + ds * 32 + l32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = key0 + kvs * 32 + crow(r, hi);
      if (key >= region_len) continue;
      const float gk = dk[ds][r] * p.scale, gv = dv[ds][r];
      if (to_acc) {
        const int64_t off = ((int64_t)(key_row_begin + key) * p.Hk + hk) * D + dcol;
        unsafeAtomicAdd(acc_k + off, gk);
        unsafeAtomicAdd(acc_v + off, gv);
      } else if (is_ctx) {
        p.dkc.ptr[(int64_t)(key_row_begin + key) * p.dkc.ts + (int64_t)hk * p.dkc.hs + dcol] = (u16)(pack2_bf16(gk, 0.f) & 0xffffu);
        p.dvc.ptr[(int64_t)(key_row_begin + key) * p.dvc.ts + (int64_t)hk * p.dvc.hs + dcol] = (u16)(pack2_bf16(gv, 0.f) & 0xffffu);
      } else {
        const int64_t grow = key_row_begin + key;
        p.dkd.ptr[grow * p.dkd.ts + (int64_t)hk * p.dkd.hs + dcol] = (u16)(pack2_bf16(gk, 0.f) & 0xffffu);
        p.dvd.ptr[grow * p.dvd.ts + (int64_t)hk * p.dvd.hs + dcol] = (u16)(pack2_bf16(gv, 0.f) & 0xffffu);
      }
    }
  }
}

template <int D, int DSPLIT, int NW, int BM, int TPAD, bool LOCAL>
static hipError_t launch_dkdv_t(AttnParams p, hipStream_t st) {
  using C = KCfg<D, DSPLIT, NW, BM, TPAD>;
  p.n_ctx_tiles = (p.ctx_len + C::BN - 1) / C::BN;
  p.n_dec_tiles = (p.max_rows + C::BN - 1) / C::BN;
  if (p.n_split < 1) p.n_split = 1;
  const size_t smem = C::smem_bytes();
  auto kern = dkdv_kernel<D, DSPLIT, NW, BM, TPAD, LOCAL>;
  hipError_t e = ensure_dynamic_lds<dkdv_kernel<D, DSPLIT, NW, BM, TPAD, LOCAL>>(smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)(p.grp ? p.n_groups : 1) * p.n_ctx_tiles * p.Hk * p.n_split +
                       (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(NW * 64), smem, st, p);
  return hipGetLastError();
}

// Per head dim: <D, DSPLIT, NW, BM, TPAD>.  Head dims 256 and 512 run eight waves (two per SIMD) with the head dim
// split four and eight ways: no spills (measured at head dim 512: 1.4x faster than four waves with a four-way split).
int dkdv_key_tile(int head_dim) {
  switch (head_dim) {
    case 64:  return KCfg<64, 1, 4, 64, 8>::BN;
    case 96:  return KCfg<96, 1, 4, 64, 8>::BN;
    case 128: return KCfg<128, 1, 4, 64, 8>::BN;
    case 192: return KCfg<192, 2, 4, 32, 8>::BN;
    case 256: return KCfg<256, 4, 8, 32, 8>::BN;
    case 512: return KCfg<512, 8, 8, 32, 8>::BN;
  }
  return 0;
}

hipError_t launch_dkdv(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_dkdv_t<64, 1, 4, 64, 8, true>(p, st) : launch_dkdv_t<64, 1, 4, 64, 8, false>(p, st);
    case 96:  return local ? launch_dkdv_t<96, 1, 4, 64, 8, true>(p, st) : launch_dkdv_t<96, 1, 4, 64, 8, false>(p, st);
    case 128: return local ? launch_dkdv_t<128, 1, 4, 64, 8, true>(p, st) : launch_dkdv_t<128, 1, 4, 64, 8, false>(p, st);
    case 192: return local ? launch_dkdv_t<192, 2, 4, 32, 8, true>(p, st) : launch_dkdv_t<192, 2, 4, 32, 8, false>(p, st);
    case 256: return local ? launch_dkdv_t<256, 4, 8, 32, 8, true>(p, st) : launch_dkdv_t<256, 4, 8, 32, 8, false>(p, st);
    case 512: return launch_dkdv_t<512, 8, 8, 32, 8, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
