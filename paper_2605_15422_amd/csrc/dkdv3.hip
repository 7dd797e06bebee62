// dK / dV kernel for head dims 64 and 128, tuned variant (same mathematics and the same ownership rule
// as the generic dkdv_kernel: one workgroup owns a 128-key tile of one KV head; a shared-prompt tile
// sums the contributions of ALL sequences and heads of the group in fp32 registers and is cast once).
//
// Shape: 8 waves = 4 key subtiles (32 keys) x 2 partners, two waves per SIMD so that one wave's
// exponentials overlap the other's MFMAs.  Both partners keep the K, V fragments of their 32 keys
// (B operands of S = Q K^T and dP = dO V^T) in registers; partner h owns the fp32 dK, dV accumulators of
// head-dim half h.  Query-row blocks of 64 rows (Q and dO, one query head) stream through
// double-buffered, swizzled LDS tiles.  Per step:
//   phase 1  partner h computes S, dP, P = exp(S*scale - LSE) and dS = P * (dP - D) for row subtile h
//            (16-byte row reads of the Q / dO tiles) and publishes P, dS as bf16 MFMA operands in LDS;
//   phase 2  every wave accumulates its head-dim half of dV += P^T dO and dK += dS^T Q over both row
//            subtiles; dO^T / Q^T come from LDS transpose reads of the SAME tiles.
// No MFMA work is duplicated; the exchange costs 8 KB of LDS traffic per wave and step.
#include "common.h"
#include "kvsched.h"
#include "launch.h"
#include "tiles.h"

namespace dkv {

template <int D, bool LOCAL>
__global__ __launch_bounds__(512) void dkdv3_kernel(const AttnParams p) {
  constexpr int NT = 512, BN = 128, BM = 64;
  constexpr int KS = D / 16, DSUB = D / 32, DH = DSUB / 2, RB = 2 * D, CPR = D / 8;
  constexpr int TILE_BYTES = BM * RB, CPT = BM * CPR / NT;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES + 2 * BM * 4;   // Q | dO | lse[BM] | D[BM]
  constexpr int XCH_BYTES = 4 * 2 * 2 * 2 * 1024;            // [key subtile][row subtile][P|dS][k-step][lane] x 16 B
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int kvs = wave & 3, dh = wave >> 2;   // key subtile, partner index (row subtile in phase 1, head-dim half in phase 2)
  const int P = p.ctx_len, W = p.window;
  const float c = p.scale_log2;
  unsigned char* xch = smem + 2 * STAGE_BYTES;

  // ---- block decode: prompt tiles first (heavy), then response tiles
  const int ctx_blocks = p.n_ctx_tiles * p.Hk * p.n_split;
  int bid = blockIdx.x;
  bool is_ctx;
  int hk, key0, seq_lo, seq_hi;
  if (bid < ctx_blocks) {
    is_ctx = true;
    hk = bid % p.Hk;
    int t = bid / p.Hk;
    const int split = t % p.n_split;
    key0 = (t / p.n_split) * BN;
    seq_lo = (int)((int64_t)p.n_seqs * split / p.n_split);
    seq_hi = (int)((int64_t)p.n_seqs * (split + 1) / p.n_split);
  } else {
    bid -= ctx_blocks;
    is_ctx = false;
    hk = bid % p.Hk;
    int t = bid / p.Hk;
    key0 = (t % p.n_dec_tiles) * BN;
    seq_lo = t / p.n_dec_tiles;
    seq_hi = seq_lo + 1;
    const int rb0 = p.cu ? p.cu[seq_lo] : 0;
    const int Rs = p.cu ? (p.cu[seq_lo + 1] - rb0) : p.total;
    if (key0 >= Rs) return;
  }

  int region_len, key_row_begin = 0;
  const u16 *kbase, *vbase;
  int64_t kts, vts;
  if (is_ctx) {
    region_len = P;
    kbase = p.kc.ptr + (int64_t)hk * p.kc.hs;
    vbase = p.vc.ptr + (int64_t)hk * p.vc.hs;
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
  const int wave_key_lo = key0 + kvs * 32, wave_key_hi = wave_key_lo + 31;
  const int my_key = wave_key_lo + l32;
  bf16x8 kf[KS], vf[KS];
  {
    const int kr = min(my_key, region_len - 1);   // clamp: gradients of padded keys are never stored
    const u16* kp = kbase + (int64_t)kr * kts + hi * 8;
    const u16* vp = vbase + (int64_t)kr * vts + hi * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
      vf[ks] = *reinterpret_cast<const bf16x8*>(vp + ks * 16);
    }
  }

  f32x16 dk[DH], dv[DH];
#pragma unroll
  for (int ds = 0; ds < DH; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[ds][r] = 0.f;
      dv[ds][r] = 0.f;
    }

  // per-lane LDS offsets (bytes, relative to a 32-row aligned origin inside a tile)
  int roff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) roff[ks] = tile_off<D>(l32, 2 * ks + hi);
  int toff0[DH], toff1[DH];
#pragma unroll
  for (int ds = 0; ds < DH; ++ds) {
    toff0[ds] = tr_off<D>(lane, hi * 4, (dh * DH + ds) * 32);
    toff1[ds] = tr_off<D>(lane, hi * 4 + 8, (dh * DH + ds) * 32);
  }
  int st_row[CPT], st_col[CPT], st_off[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int id = tid + j * NT;
    st_row[j] = id / CPR;
    st_col[j] = (id % CPR) * 8;
    st_off[j] = tile_off<D>(st_row[j], id % CPR);
  }

  StepIter<BM, BN, LOCAL> iter(p, hk, is_ctx, key0, seq_lo, seq_hi);
  u32x4 qst[CPT], dost[CPT];
  float lse_pf = LSE_MASKED, d_pf = 0.f;
  auto issue_loads = [&](const RowStep& s) {
    const u16* qb = p.q.ptr + s.grow * p.q.ts + (int64_t)s.head * p.q.hs;
    const u16* db = p.dout.ptr + s.grow * p.dout.ts + (int64_t)s.head * p.dout.hs;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      u32x4 zq = {0u, 0u, 0u, 0u}, zd = {0u, 0u, 0u, 0u};
      if (st_row[j] < s.nvalid) {
        zq = *reinterpret_cast<const u32x4*>(qb + (int64_t)st_row[j] * p.q.ts + st_col[j]);
        zd = *reinterpret_cast<const u32x4*>(db + (int64_t)st_row[j] * p.dout.ts + st_col[j]);
      }
      qst[j] = zq;
      dost[j] = zd;
    }
    if (tid < BM) {
      const bool ok = tid < s.nvalid;
      lse_pf = ok ? p.lse[(int64_t)s.head * p.total + s.grow + tid] * LOG2E : LSE_MASKED;
      d_pf = ok ? p.dvec[(int64_t)s.head * p.total + s.grow + tid] : 0.f;
    }
  };
  auto store_stage = [&](int buf) {
    unsigned char* qb = smem + buf * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      *reinterpret_cast<u32x4*>(qb + st_off[j]) = qst[j];
      *reinterpret_cast<u32x4*>(qb + TILE_BYTES + st_off[j]) = dost[j];
    }
    if (tid < BM) {
      float* lp = reinterpret_cast<float*>(qb + 2 * TILE_BYTES);
      lp[tid] = lse_pf;
      lp[BM + tid] = d_pf;
    }
  };

  RowStep cur, nxt, nn;
  bool has = iter.next(cur), has_n = false;
  if (has) {
    issue_loads(cur);
    store_stage(0);
    has_n = iter.next(nxt);
    if (has_n) issue_loads(nxt);
  }
  __syncthreads();
  int buf = 0;

  while (has) {
    if (has_n) store_stage(buf ^ 1);
    const bool has_nn = has_n && iter.next(nn);
    if (has_nn) issue_loads(nn);

    const unsigned char* Qb = smem + buf * STAGE_BYTES;
    const unsigned char* dOb = Qb + TILE_BYTES;
    const float* lseL = reinterpret_cast<const float*>(Qb + 2 * TILE_BYTES);
    const float* DL = lseL + BM;

    // ---- phase 1: this wave's row subtile (qs = dh) against its 32 keys
    bool act[2];
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      const int srow0 = cur.row0 + qs * 32;
      bool a = qs * 32 < cur.nvalid;
      if (is_ctx) {
        if (LOCAL) a = a && (wave_key_hi > P + srow0 - W);
      } else {
        a = a && (wave_key_lo <= srow0 + 31);
        if (LOCAL) a = a && (wave_key_hi > srow0 - W);
      }
      act[qs] = a;
    }
    {
      const int qs = dh;
      const int srow0 = cur.row0 + qs * 32;   // first row of the subtile inside its sequence
      bool need_mask = false;
      if (is_ctx) {
        if (LOCAL) need_mask = wave_key_lo <= P + srow0 + 31 - W;
      } else {
        need_mask = wave_key_hi > srow0;
        if (LOCAL) need_mask = need_mask || (wave_key_lo <= srow0 + 31 - W);
      }
      if (dh == 0 ? act[0] : act[1]) {
        f32x16 s, dpv;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[r] = 0.f;
          dpv[r] = 0.f;
        }
        const unsigned char* qh = Qb + qs * 32 * RB;
        const unsigned char* dhp = dOb + qs * 32 * RB;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          s = mfma32(*reinterpret_cast<const bf16x8*>(qh + roff[ks]), kf[ks], s);
          dpv = mfma32(*reinterpret_cast<const bf16x8*>(dhp + roff[ks]), vf[ks], dpv);
        }
        float pv[16], dsv[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 lr = *reinterpret_cast<const f32x4*>(lseL + qs * 32 + r4 * 8 + hi * 4);
          const f32x4 dr = *reinterpret_cast<const f32x4*>(DL + qs * 32 + r4 * 8 + hi * 4);
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const int r = r4 * 4 + e4;
            float e = __builtin_amdgcn_exp2f(s[r] * c - lr[e4]);
            if (need_mask) {
              const int rw = srow0 + crow(r, hi);
              bool ok;
              if (is_ctx) ok = !LOCAL || (my_key > P + rw - W);
              else ok = (my_key <= rw) && (!LOCAL || (my_key > rw - W));
              if (!ok) e = 0.f;
            }
            pv[r] = e;
            dsv[r] = e * (dpv[r] - dr[e4]);
          }
        }
        unsigned char* xw = xch + ((kvs * 2 + qs) * 4) * 1024 + lane * 16;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          *reinterpret_cast<bf16x8*>(xw + t2 * 1024) = pack8_bf16(pv + t2 * 8);
          *reinterpret_cast<bf16x8*>(xw + (2 + t2) * 1024) = pack8_bf16(dsv + t2 * 8);
        }
      }
    }
    __syncthreads();
    // ---- phase 2: this wave's head-dim half of dV, dK over both row subtiles
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      if (!act[qs]) continue;
      const unsigned char* xr = xch + ((kvs * 2 + qs) * 4) * 1024 + lane * 16;
      const unsigned char* qh = Qb + qs * 32 * RB;
      const unsigned char* dhp = dOb + qs * 32 * RB;
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16x8 pa = *reinterpret_cast<const bf16x8*>(xr + t2 * 1024);
        const bf16x8 dsa = *reinterpret_cast<const bf16x8*>(xr + (2 + t2) * 1024);
        const unsigned char* qt = qh + t2 * 16 * RB;
        const unsigned char* dt = dhp + t2 * 16 * RB;
#pragma unroll
        for (int ds = 0; ds < DH; ++ds) {
          dv[ds] = mfma32(pa, tr_pair(dt + toff0[ds], dt + toff1[ds]), dv[ds]);
          dk[ds] = mfma32(dsa, tr_pair(qt + toff0[ds], qt + toff1[ds]), dk[ds]);
        }
      }
    }
    __syncthreads();
    cur = nxt;
    nxt = nn;
    has = has_n;
    has_n = has_nn;
    buf ^= 1;
  }

  // ---- epilogue: C layout -> lane owns head-dim column, register r owns key crow(r)
  const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
  float* acc_k = is_ctx ? p.dkc_acc : p.dkd_acc;
  float* acc_v = is_ctx ? p.dvc_acc : p.dvd_acc;
#pragma unroll
  for (int ds = 0; ds < DH; ++ds) {
    const int dcol = (dh * DH + ds) * 32 + l32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = wave_key_lo + crow(r, hi);
      if (key >= region_len) continue;
      const float gk = dk[ds][r] * p.scale, gv = dv[ds][r];
      if (to_acc) {
        const int64_t off = ((int64_t)(key_row_begin + key) * p.Hk + hk) * D + dcol;
        unsafeAtomicAdd(acc_k + off, gk);
        unsafeAtomicAdd(acc_v + off, gv);
      } else if (is_ctx) {
        p.dkc.ptr[(int64_t)key * p.dkc.ts + (int64_t)hk * p.dkc.hs + dcol] = (u16)(pack2_bf16(gk, 0.f) & 0xffffu);
        p.dvc.ptr[(int64_t)key * p.dvc.ts + (int64_t)hk * p.dvc.hs + dcol] = (u16)(pack2_bf16(gv, 0.f) & 0xffffu);
      } else {
        const int64_t grow = key_row_begin + key;
        p.dkd.ptr[grow * p.dkd.ts + (int64_t)hk * p.dkd.hs + dcol] = (u16)(pack2_bf16(gk, 0.f) & 0xffffu);
        p.dvd.ptr[grow * p.dvd.ts + (int64_t)hk * p.dvd.hs + dcol] = (u16)(pack2_bf16(gv, 0.f) & 0xffffu);
      }
    }
  }
}

template <int D, bool LOCAL>
static hipError_t launch_dkdv3_t(AttnParams p, hipStream_t st) {
  constexpr int BN = 128, BM = 64;
  p.n_ctx_tiles = (p.ctx_len + BN - 1) / BN;
  p.n_dec_tiles = (p.max_rows + BN - 1) / BN;
  if (p.n_split < 1) p.n_split = 1;
  const size_t smem = 2 * (2 * BM * 2 * D + 2 * BM * 4) + 32768;
  auto kern = dkdv3_kernel<D, LOCAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_ctx_tiles * p.Hk * p.n_split + (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(512), smem, st, p);
  return hipGetLastError();
}

hipError_t launch_dkdv3(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_dkdv3_t<64, true>(p, st) : launch_dkdv3_t<64, false>(p, st);
    case 128: return local ? launch_dkdv3_t<128, true>(p, st) : launch_dkdv3_t<128, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
