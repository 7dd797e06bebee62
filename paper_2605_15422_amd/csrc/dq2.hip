// dQ kernel for head dims 64 and 128, tuned variant (same mathematics as the generic dq_kernel):
//   dQ = scale * dS K,  dS = P * (dP - D),  P = exp(scale * Q K^T - LSE),  dP = dO V^T     (Alg. 1)
// evaluated per query block over all its visible key tiles (prompt tiles, then own-response tiles), so
// dQ is accumulated in registers and written once: no fp32 dQ scratch, no atomics, no convert pass.
//
// Shape: 8 waves (two per SIMD), each owning one 32-row subtile with Q, dO fragments and the dQ^T
// accumulator in registers; K and V tiles of 64 keys double-buffered in swizzled LDS.  S^T = K Q^T and
// dP^T = V dO^T take 16-byte row operands from LDS; dQ^T += K^T dS^T takes K^T through LDS transpose
// reads of the same row-major K tile.  A 64-key tile is consumed as two 32-key halves so only one
// 32x32 S and dP tile is live at a time.
#include "common.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {

template <int D, bool LOCAL>
__global__ __launch_bounds__(512) void dq2_kernel(const AttnParams p) {
  constexpr int NT = 512, BN = 64;
  constexpr int KS = D / 16, DSUB = D / 32, RB = 2 * D, CPR = D / 8;
  constexpr int TILE_BYTES = BN * RB, CPT = BN * CPR / NT;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][K tile | V tile]

  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int P = p.ctx_len, R = b.R, W = p.window;
  const float c = p.scale_log2;

  const int head = b.hk * p.G + b.hc * p.GP + wave / p.RSH;
  const int row0 = b.blk_row0 + (wave % p.RSH) * 32;
  const int row = row0 + l32;
  const bool wave_valid = row0 < R;

  bf16x8 qf[KS], dof[KS];
  float lse2, dvec;
  {
    const int64_t grow = b.row_begin + min(row, R - 1);
    const u16* qp = p.q.ptr + grow * p.q.ts + (int64_t)head * p.q.hs + hi * 8;
    const u16* dop = p.dout.ptr + grow * p.dout.ts + (int64_t)head * p.dout.hs + hi * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
      dof[ks] = *reinterpret_cast<const bf16x8*>(dop + ks * 16);
    }
    lse2 = p.lse[(int64_t)head * p.total + grow] * LOG2E;
    dvec = p.dvec[(int64_t)head * p.total + grow];
  }

  f32x16 dqacc[DSUB];
#pragma unroll
  for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[ds][r] = 0.f;

  // per-lane LDS offsets relative to a tile base (the swizzle has period 16 rows)
  int roff[KS];             // 16-byte row operand: row l32 (+32*half), chunk 2*ks+hi
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) roff[ks] = tile_off<D>(l32, 2 * ks + hi);
  int toff0[DSUB], toff1[DSUB];   // transpose reads: rows 4*hi + (lane%16)/4 and +8, head-dim block ds
#pragma unroll
  for (int ds = 0; ds < DSUB; ++ds) {
    toff0[ds] = tr_off<D>(lane, hi * 4, ds * 32);
    toff1[ds] = tr_off<D>(lane, hi * 4 + 8, ds * 32);
  }

  const u16* kc_base = p.kc.ptr + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;
  int st_row[CPT], st_col[CPT], st_off[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int id = tid + j * NT;
    st_row[j] = id / CPR;
    st_col[j] = (id % CPR) * 8;
    st_off[j] = tile_off<D>(st_row[j], id % CPR);
  }
  u32x4 kst[CPT], vst[CPT];
  auto issue_loads = [&](int it) {
    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const u16* kb = is_ctx ? kc_base : kd_base;
    const u16* vb = is_ctx ? vc_base : vd_base;
    const int64_t kts = is_ctx ? p.kc.ts : p.kd.ts, vts = is_ctx ? p.vc.ts : p.vd.ts;
    const int nvalid = (is_ctx ? P : R) - key0;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      u32x4 zk = {0u, 0u, 0u, 0u}, zv = {0u, 0u, 0u, 0u};
      if (st_row[j] < nvalid) {
        zk = *reinterpret_cast<const u32x4*>(kb + (int64_t)(key0 + st_row[j]) * kts + st_col[j]);
        zv = *reinterpret_cast<const u32x4*>(vb + (int64_t)(key0 + st_row[j]) * vts + st_col[j]);
      }
      kst[j] = zk;
      vst[j] = zv;
    }
  };
  auto store_stage = [&](int buf) {
    unsigned char* kb = smem + buf * 2 * TILE_BYTES;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      *reinterpret_cast<u32x4*>(kb + st_off[j]) = kst[j];
      *reinterpret_cast<u32x4*>(kb + TILE_BYTES + st_off[j]) = vst[j];
    }
  };

  issue_loads(0);
  store_stage(0);
  if (b.n_tiles > 1) issue_loads(1);
  __syncthreads();

  for (int it = 0; it < b.n_tiles; ++it) {
    if (it + 1 < b.n_tiles) store_stage((it + 1) & 1);
    if (it + 2 < b.n_tiles) issue_loads(it + 2);

    const unsigned char* Kb = smem + (it & 1) * 2 * TILE_BYTES;
    const unsigned char* Vb = Kb + TILE_BYTES;
    const bool is_ctx = it < n_ctx_run;
    const int tile_key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;

#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int key0 = tile_key0 + half * 32;
      const bool active = wave_valid && tile_active<LOCAL, 32>(is_ctx, key0, row0, row0 + 31, P, W) &&
                          key0 < (is_ctx ? P : R);
      if (!active) continue;
      f32x16 s, dpt;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = 0.f;
        dpt[r] = 0.f;
      }
      const unsigned char* kh = Kb + half * 32 * RB;
      const unsigned char* vh = Vb + half * 32 * RB;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = mfma32(*reinterpret_cast<const bf16x8*>(kh + roff[ks]), qf[ks], s);
        dpt = mfma32(*reinterpret_cast<const bf16x8*>(vh + roff[ks]), dof[ks], dpt);
      }
      const bool need = tile_needs_mask<LOCAL, 32>(is_ctx, key0, row0, P, R, W);
      float dsv[16];
      // two straight-line variants: a per-element test of a run-time flag costs three branches per element
      if (__builtin_expect(need, 0)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float e = __builtin_amdgcn_exp2f(s[r] * c - lse2);
          const int key = key0 + crow(r, hi);
          if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) e = 0.f;
          dsv[r] = e * (dpt[r] - dvec);   // dS^T
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) dsv[r] = __builtin_amdgcn_exp2f(s[r] * c - lse2) * (dpt[r] - dvec);
      }
      // dQ^T += K^T dS^T
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16x8 pb = pack8_bf16(dsv + t2 * 8);
        const unsigned char* kt = kh + t2 * 16 * RB;
#pragma unroll
        for (int ds = 0; ds < DSUB; ++ds)
          dqacc[ds] = mfma32(tr_pair(kt + toff0[ds], kt + toff1[ds]), pb, dqacc[ds]);
      }
    }
    __syncthreads();
  }

  if (row < R) {
    u16* op = p.dq.ptr + (int64_t)(b.row_begin + row) * p.dq.ts + (int64_t)head * p.dq.hs;
#pragma unroll
    for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack2_bf16(dqacc[ds][r4 * 4 + 0] * p.scale, dqacc[ds][r4 * 4 + 1] * p.scale);
        w.y = pack2_bf16(dqacc[ds][r4 * 4 + 2] * p.scale, dqacc[ds][r4 * 4 + 3] * p.scale);
        *reinterpret_cast<u32x2*>(op + ds * 32 + r4 * 8 + hi * 4) = w;
      }
  }
}

template <int D, bool LOCAL>
static hipError_t launch_dq2_t(AttnParams p, hipStream_t st) {
  fill_packing(p, 8);
  const size_t smem = 4 * 64 * 2 * D;
  auto kern = dq2_kernel<D, LOCAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(512), smem, st, p);
  return hipGetLastError();
}

hipError_t launch_dq2(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_dq2_t<64, true>(p, st) : launch_dq2_t<64, false>(p, st);
    case 128: return local ? launch_dq2_t<128, true>(p, st) : launch_dq2_t<128, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
