// dQ kernel for head dims 64 and 128, tuned variant (same mathematics as the generic dq_kernel):
//   dQ = scale * dS K,  dS = P * (dP - D),  P = exp(scale * Q K^T - LSE),  dP = dO V^T     (Alg. 1)
// evaluated per query block over all its visible key tiles (prompt tiles, then own-response tiles), so
// dQ is accumulated in registers and written once: no fp32 dQ scratch, no atomics, no convert pass.
//
// Shape: 8 waves (two per SIMD), each owning one 32-row subtile with Q, dO fragments and the dQ^T
// accumulator in registers; K and V tiles of 64 keys travel global -> LDS directly (global_load_lds, three
// stages, two tiles ahead: no staging registers, which pays for a deeper operand prefetch) into swizzled LDS.  S^T = K Q^T and
// dP^T = V dO^T take 16-byte row operands from LDS; dQ^T += K^T dS^T takes K^T through LDS transpose
// reads of the same row-major K tile.  A 64-key tile is consumed as two 32-key halves so only one
// 32x32 S and dP tile is live at a time.
#include "common.h"
#include "dma.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {

template <int D, bool LOCAL>
__global__ __launch_bounds__(512) void dq2_kernel(const AttnParams p) {
  constexpr int NT = 512, BN = 64;
  constexpr int KS = D / 16, DSUB = D / 32, RB = 2 * D, CPR = D / 8;
  constexpr int TILE_BYTES = BN * RB;
  constexpr int NSTAGE = 3, STAGE_BYTES = 2 * TILE_BYTES;
  constexpr int IPT = TILE_BYTES / 1024 / 8;   // 1 KB load instructions per wave, tile and tensor
  constexpr int RPI = 1024 / RB;               // rows per load instruction
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [NSTAGE][K tile | V tile]

  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int P = b.P, R = b.R, W = p.window;
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
    // consumed (and therefore waited for) here: no compiler-placed vector-memory wait inside the main loop
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : : "v"(qf[ks]), "v"(dof[ks]));
    asm volatile("" : : "v"(lse2), "v"(dvec));
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

  const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;
  // global -> LDS tile loads: instruction j = wave + 8 t of a tile covers RPI key rows; lane l lands at LDS
  // chunk position l % CPR of row l / CPR of the instruction and fetches the chunk the swizzle stores there
  // (the swizzle has period 16 rows, so one offset serves every t).  Keys past the end of the region re-read
  // the last key: their scores are masked like any invisible key.
  const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  const int ld_row0 = wave * RPI + lane / CPR;
  const int ld_coff = ((lane % CPR) ^ swz<D>(ld_row0)) * 16;
  // (token strides in bytes, read from the kernel arguments once: a scalar load inside the loop would make the
  // wave wait for every LDS read in flight as well)
  const int ktsb_c = (int)p.kc.ts * 2, ktsb_d = (int)p.kd.ts * 2, vtsb_c = (int)p.vc.ts * 2, vtsb_d = (int)p.vd.ts * 2;
  auto issue_loads = [&](int it, int stage) __attribute__((always_inline)) {
    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const int ktsb = is_ctx ? ktsb_c : ktsb_d, vtsb = is_ctx ? vtsb_c : vtsb_d;
    const u16* kb = uniform_ptr(reinterpret_cast<const u16*>(
        reinterpret_cast<const unsigned char*>(is_ctx ? kc_base : kd_base) + (int64_t)key0 * ktsb));
    const u16* vb = uniform_ptr(reinterpret_cast<const u16*>(
        reinterpret_cast<const unsigned char*>(is_ctx ? vc_base : vd_base) + (int64_t)key0 * vtsb));
    const int last = (is_ctx ? P : R) - key0 - 1;
    const uint32_t dst = smem_addr + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
      const unsigned row = (unsigned)min(ld_row0 + t * 8 * RPI, last);
      dma16(kb, __umul24(row, (unsigned)ktsb) + ld_coff, dst + t * 8192);
      dma16(vb, __umul24(row, (unsigned)vtsb) + ld_coff, dst + TILE_BYTES + t * 8192);
    }
  };
  // the tile consumed next must have landed; the 2 IPT loads of the tile after it may stay in flight
  auto wait_loads = [&](bool newer_in_flight) __attribute__((always_inline)) {
    wait_vm<2 * IPT>();
    if (__builtin_expect(!newer_in_flight, 0)) wait_vm<0>();
  };

  issue_loads(0, 0);
  if (b.n_tiles > 1) issue_loads(1, 1);
  wait_loads(b.n_tiles > 1);
  __syncthreads();

  f32x16 negd;   // accumulator image of -D: this lane's query row in all sixteen registers
#pragma unroll
  for (int r = 0; r < 16; ++r) negd[r] = -dvec;
  const bool never_plain = LOCAL || !wave_valid;
  const int ctx_masked = (P % BN) ? b.n_ctx - 1 : -1;   // the partial last prompt tile
  const int dec_masked = min(row0 + 1, R) / BN;         // response tiles from the diagonal (or the sequence end) on
  int stage = 0;
  for (int it = 0; it < b.n_tiles; ++it) {
    // tile it+2 goes into the stage that tile it-1 left at the last barrier
    const int stage2 = stage == 0 ? 2 : stage - 1;
    if (it + 2 < b.n_tiles) issue_loads(it + 2, stage2);

    const unsigned char* Kb = smem + stage * STAGE_BYTES;
    const unsigned char* Vb = Kb + TILE_BYTES;
    const bool is_ctx = it < n_ctx_run;
    const int kt = is_ctx ? b.c0 + it : b.d0 + it - n_ctx_run;
    const int tile_key0 = kt * BN;
    // most tiles are entirely visible to the 32 rows of this wave: no per-half tests for them
    const bool plain = !never_plain && (is_ctx ? kt != ctx_masked : kt < dec_masked);

#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int key0 = tile_key0 + half * 32;
      const bool active = plain || (wave_valid && tile_active<LOCAL, 32>(is_ctx, key0, row0, row0 + 31, P, W) &&
                                    key0 < (is_ctx ? P : R));
      if (!active) continue;
      const unsigned char* kh = Kb + half * 32 * RB;
      const unsigned char* vh = Vb + half * 32 * RB;
      // S^T = K Q^T first, complete, then dP^T - D = V dO^T - D (accumulator initialised to -D): the exponentials of
      // S^T issue in the shadow of the dP MFMAs (two per MFMA), only the products and the packing are left after them.
      // The K operands are requested before the V operands, so the S chain starts as soon as its own have landed.
      bf16x8 ko[KS], vo[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) ko[ks] = *reinterpret_cast<const bf16x8*>(kh + roff[ks]);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) vo[ks] = *reinterpret_cast<const bf16x8*>(vh + roff[ks]);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 s, dpt;
      // S chain first (complete before the dP chain starts) ...
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) s = mfma32(ko[ks], qf[ks], s);
      __builtin_amdgcn_sched_barrier(0);
      // ... so that the exponentials of S issue in the shadow of the dP MFMAs
      const bool need = !plain && tile_needs_mask<LOCAL, 32>(is_ctx, key0, row0, P, R, W);
      float ev[16], dsv[16];
      constexpr int EPM = 16 / KS;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        dpt = mfma32(vo[ks], dof[ks], ks == 0 ? negd : dpt);
#pragma unroll
        for (int e = ks * EPM; e < (ks + 1) * EPM; ++e) {
          ev[e] = __builtin_amdgcn_exp2f(s[e] * c - lse2);
          asm volatile("" : "+v"(ev[e]));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (__builtin_expect(need, 0)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + crow(r, hi);
          if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) ev[r] = 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) dsv[r] = ev[r] * dpt[r];   // dS^T
      // dQ^T += K^T dS^T
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const bf16x8 pb = pack8_bf16(dsv + t2 * 8);
        const unsigned char* kt2 = kh + t2 * 16 * RB;
#pragma unroll
        for (int ds = 0; ds < DSUB; ++ds)
          dqacc[ds] = mfma32(tr_pair(kt2 + toff0[ds], kt2 + toff1[ds]), pb, dqacc[ds]);
      }
    }
    wait_loads(it + 2 < b.n_tiles);
    __syncthreads();
    stage = stage == 2 ? 0 : stage + 1;
  }

  // ---- epilogue: lane owns a query row, register r the head-dim column crow(r) of a 32-column block.  Stored from
  // here a row would leave in 16-byte pieces, 32 rows per instruction.  The wave's scaled 32 x D tile goes through LDS
  // instead (all stages are free after the last barrier; 16-byte chunks XOR-swizzled by the row) and is read back as
  // whole rows.  Wave-private: no barrier.
  unsigned char* ot = smem + wave * 32 * RB;
#pragma unroll
  for (int ds = 0; ds < DSUB; ++ds)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      u32x2 w;
      w.x = pack2_bf16(dqacc[ds][r4 * 4 + 0] * p.scale, dqacc[ds][r4 * 4 + 1] * p.scale);
      w.y = pack2_bf16(dqacc[ds][r4 * 4 + 2] * p.scale, dqacc[ds][r4 * 4 + 3] * p.scale);
      *reinterpret_cast<u32x2*>(ot + l32 * RB + (((ds * 4 + r4) ^ (l32 & (CPR - 1))) << 4) + hi * 8) = w;
    }
  constexpr int RPS = 64 / CPR;   // rows per store instruction
  const int chunk = lane % CPR;
#pragma unroll
  for (int i = 0; i < 32 / RPS; ++i) {
    const int tr = i * RPS + lane / CPR;
    const u32x4 w = *reinterpret_cast<const u32x4*>(ot + tr * RB + ((chunk ^ (tr & (CPR - 1))) << 4));
    if (row0 + tr < R) {
      u16* op = p.dq.ptr + (int64_t)(b.row_begin + row0 + tr) * p.dq.ts + (int64_t)head * p.dq.hs;
      *reinterpret_cast<u32x4*>(op + chunk * 8) = w;
    }
  }
}

template <int D, bool LOCAL>
static hipError_t launch_dq2_t(AttnParams p, hipStream_t st) {
  fill_packing(p, 8);
  const size_t smem = 3 * 2 * 64 * 2 * D;
  auto kern = dq2_kernel<D, LOCAL>;
  hipError_t e = ensure_dynamic_lds<dq2_kernel<D, LOCAL>>(smem);
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
