// dQ kernel for head dim 512 with producer / consumer wave specialisation:
//   dQ = scale * dS K,  dS = P * (dP - D),  P = exp(scale * Q K^T - LSE),  dP = dO V^T     (Alg. 1)
// evaluated per query block over all its visible key tiles (prompt tiles, then own-response tiles), dQ
// accumulated in registers and written once, as in the narrower kernels.
//
// What this head dim dictates.  The fp32 dQ of one row fills 2 KB and the four consumer waves can give 128 of
// their 256 registers to accumulators: a workgroup owns 64 rows (two 32-row subtiles), each consumer wave
// holding four of the sixteen 32-wide head-dim blocks of dQ^T for both.  The Q and dO fragments of 16 rows
// already fill 128 registers, so each of the four producers takes 16 rows and works with the 16x16x32 MFMA:
// per 16-key tile it forms S^T = K Q^T, dP^T - D = V dO^T - D, P and dS^T in fp32 and publishes dS^T as the
// bf16 B operand of the consumers' 32x32x16 product (32 small MFMAs per tile); the consumers, one tile behind,
// add K^T dS^T with K^T from LDS transpose reads (8 MFMAs per tile).  K / V tiles of 16 keys (16 KB + 16 KB)
// travel global -> LDS three tiles ahead into four stages, issued by the consumers, which read their K^T
// operands one interval early so that a stage is free again after one interval.  One barrier per tile.
#include "common.h"
#include "dma.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {
namespace {

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

constexpr int D = 512;
constexpr int BN = 16, NSUB = 2;                 // keys per tile, 32-row subtiles per workgroup (consumers' view)
constexpr int NDB = D / 128;                     // head-dim blocks per consumer wave
constexpr int KS = D / 32, RB = 2 * D;           // k-steps of the 16x16x32 MFMA
constexpr int TILE_BYTES = BN * RB;
constexpr int NSTAGE = 4, STAGE_BYTES = 2 * TILE_BYTES;   // K tile | V tile
constexpr int XCH_OFF = NSTAGE * STAGE_BYTES;
constexpr int XCH_BYTES = NSUB * 1024;           // [subtile][lane] x 16 B
constexpr int SMEM_BYTES = XCH_OFF + 2 * XCH_BYTES;
constexpr int IPT = TILE_BYTES / 1024 / 4;       // 1 KB load instructions per consumer wave, tile and tensor

template <bool LOCAL>
__global__ __launch_bounds__(512) void dq512_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int P = b.P, R = b.R, W = p.window;
  const int n_ctx_run = b.n_ctx - b.c0;
  const int n_tiles = b.n_tiles;

  if (wave < 4) {
    // ================================= producer ==============================================
    // 16x16x32 operands: lane = (l16, g): A row / B column l16, eight contraction indices of the k-step;
    // accumulator: column l16, register r <-> row 4 g + r.  Here A = K or V (LDS, row = key), B = Q or dO
    // (registers, column = query row): the lane owns a query row and the keys 4 g + r of the tile.  Lane group g
    // takes chunk cg = (0, 3, 1, 2)[g] of a 64-byte k-step (both operands agree on it), which keeps the 16-byte
    // LDS reads of the sixteen-lane groups the hardware serves together on different bank groups.
    const float c = p.scale_log2;
    const int l16 = lane & 15, g = lane >> 4;
    const int cg = (0x9C >> (2 * g)) & 3;
    const int sub = wave >> 1;
    const int head = b.hk * p.G + b.hc * p.GP + sub / p.RSH;
    const int row0 = b.blk_row0 + (sub % p.RSH) * 32 + (wave & 1) * 16;
    const int row = row0 + l16;
    const bool wave_valid = row0 < R;

    bf16x8 qf[KS], dof[KS];
    float lse2, negd;
    {
      const int64_t grow = b.row_begin + min(row, R - 1);
      const u16* qp = p.q.ptr + grow * p.q.ts + (int64_t)head * p.q.hs + cg * 8;
      const u16* dop = p.dout.ptr + grow * p.dout.ts + (int64_t)head * p.dout.hs + cg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
        dof[ks] = *reinterpret_cast<const bf16x8*>(dop + ks * 32);
      }
      lse2 = p.lse[(int64_t)head * p.total + grow] * LOG2E;
      negd = -p.dvec[(int64_t)head * p.total + grow];
      // consumed (and therefore waited for) here: no compiler-placed vector-memory wait inside the main loop
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : : "v"(qf[ks]), "v"(dof[ks]));
      asm volatile("" : : "v"(lse2), "v"(negd));
    }
    // K / V operand of k-step ks: key row l16, chunk 4 ks + cg; with the tile swizzle its position is
    // 4 ((ks % 4) ^ (row % 4)) + (cg ^ (row / 4 % 4)) + 16 (ks / 4): four per-lane offsets serve all k-steps.
    int roff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) roff[j] = l16 * RB + 64 * (j ^ (l16 & 3)) + 16 * (cg ^ ((l16 >> 2) & 3));
    // consumer B operand (32x32x16): lane (row of the subtile, hi'), element e <-> key 4 hi' + 8 (e / 4) + e % 4 of
    // the tile.  This lane holds keys 4 g + r: hi' = g % 2, elements 4 (g / 2) .. + 3.
    unsigned char* xw = smem + XCH_OFF + sub * 1024 + ((g & 1) * 32 + (wave & 1) * 16 + l16) * 16 + (g >> 1) * 8;

    const int ctx_masked = (P % BN) ? b.n_ctx - 1 : -1;   // the partial last prompt tile
    const int dec_masked = min(row0 + 1, R) / BN;         // response tiles from the diagonal (or the sequence end) on

    __syncthreads();   // tile 0 is in LDS
    for (int it = 0; it < n_tiles; ++it) {
      const unsigned char* kh = smem + (it & (NSTAGE - 1)) * STAGE_BYTES;
      const unsigned char* vh = kh + TILE_BYTES;
      const bool is_ctx = it < n_ctx_run;
      const int kt = is_ctx ? b.c0 + it : b.d0 + it - n_ctx_run;
      const int key0 = kt * BN;
      // most tiles are entirely visible to the 16 rows of this wave: no tests for them
      const bool plain = wave_valid && (is_ctx ? kt != ctx_masked : kt < dec_masked);
      const bool active = plain || (wave_valid && (is_ctx || key0 <= row0 + 15) && key0 < (is_ctx ? P : R));
      unsigned char* xo = xw + (it & 1) * XCH_BYTES;
      if (__builtin_expect(active, 1)) {
        // operands in groups of four, the next group requested before the MFMAs of the current one
        constexpr int GRP = 4, NG = 2 * KS / GRP;
        bf16x8 op[2][GRP];
        auto request = [&](int gi, bf16x8* out) __attribute__((always_inline)) {
#pragma unroll
          for (int q = 0; q < GRP; ++q) {
            const int ks = (gi * GRP + q) % KS;
            const unsigned char* base = gi * GRP < KS ? kh : vh;
            out[q] = *reinterpret_cast<const bf16x8*>(base + roff[ks & 3] + (ks >> 2) * 256);
          }
        };
        request(0, op[0]);
        f32x4 s = {0.f, 0.f, 0.f, 0.f}, dpt = {negd, negd, negd, negd};
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
          if (gi + 1 < NG) request(gi + 1, op[(gi + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int q = 0; q < GRP; ++q) {
            const int i = gi * GRP + q;
            if (i < KS) s = mfma16(op[gi & 1][q], qf[i], s);               // S^T = K Q^T
            else dpt = mfma16(op[gi & 1][q], dof[i - KS], dpt);           // dP^T - D = V dO^T - D
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        float dsv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float e = __builtin_amdgcn_exp2f(s[r] * c - lse2);
          if (!plain && !visible<LOCAL>(is_ctx, key0 + 4 * g + r, row, P, R, W)) e = 0.f;
          dsv[r] = e * dpt[r];   // dS^T
        }
        u32x2 w;
        w.x = pack2_bf16(dsv[0], dsv[1]);
        w.y = pack2_bf16(dsv[2], dsv[3]);
        *reinterpret_cast<u32x2*>(xo) = w;
      } else {
        // nothing visible: the consumers do not branch, they add a product with dS = 0
        const u32x2 z = {0u, 0u};
        *reinterpret_cast<u32x2*>(xo) = z;
      }
      __syncthreads();
    }
    __syncthreads();   // the consumers' last interval
  } else {
    // ================================= consumer ==============================================
    const int jb = wave - 4;
    const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
    const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
    const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
    const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
    // global -> LDS tile loads: one instruction per 1 KB key row; this wave takes rows jb, jb + 4, jb + 8, jb + 12 of
    // K and of V.  Lane l lands at chunk position l of the row and fetches the chunk the swizzle stores there.  Keys
    // past the end of the region re-read the last key: their scores are masked like any invisible key.
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    const int ktsb_c = (int)p.kc.ts * 2, ktsb_d = (int)p.kd.ts * 2, vtsb_c = (int)p.vc.ts * 2, vtsb_d = (int)p.vd.ts * 2;
    auto issue_loads = [&](int it) __attribute__((always_inline)) {
      const bool is_ctx = it < n_ctx_run;
      const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
      const int ktsb = is_ctx ? ktsb_c : ktsb_d, vtsb = is_ctx ? vtsb_c : vtsb_d;
      const u16* kb = uniform_ptr(reinterpret_cast<const u16*>(
          reinterpret_cast<const unsigned char*>(is_ctx ? kc_base : kd_base) + (int64_t)key0 * ktsb));
      const u16* vb = uniform_ptr(reinterpret_cast<const u16*>(
          reinterpret_cast<const unsigned char*>(is_ctx ? vc_base : vd_base) + (int64_t)key0 * vtsb));
      const int last = (is_ctx ? P : R) - key0 - 1;
      const uint32_t dst = smem_addr + (it & (NSTAGE - 1)) * STAGE_BYTES + jb * 1024;
#pragma unroll
      for (int t = 0; t < IPT; ++t) {
        const unsigned row = (unsigned)min(jb + t * 4, last);
        const uint32_t coff = (uint32_t)((lane ^ swz<D>(jb + t * 4)) * 16);
        dma16(kb, __umul24(row, (unsigned)ktsb) + coff, dst + t * 4096);
        dma16(vb, __umul24(row, (unsigned)vtsb) + coff, dst + TILE_BYTES + t * 4096);
      }
    };
    issue_loads(0);
    if (n_tiles > 1) issue_loads(1);
    if (n_tiles > 2) issue_loads(2);
    // tile 0 must have landed; younger tiles may stay in flight
    if (n_tiles > 2) wait_vm<4 * IPT>();
    else if (n_tiles > 1) wait_vm<2 * IPT>();
    else wait_vm<0>();

    f32x16 dq[NSUB][NDB];
#pragma unroll
    for (int s = 0; s < NSUB; ++s)
#pragma unroll
      for (int e = 0; e < NDB; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[s][e][r] = 0.f;
    // transpose reads: rows 4 hi + (lane % 16) / 4 and + 8 of the 16-key tile, head-dim block jb (blocks jb + 4,
    // jb + 8, jb + 12 lie 256, 512, 768 bytes further: the chunk index bits the swizzle leaves alone)
    const int toff0 = tr_off<D>(lane, hi * 4, jb * 32), toff1 = tr_off<D>(lane, hi * 4 + 8, jb * 32);
    const unsigned char* xr = smem + XCH_OFF + lane * 16;
    bf16x8 kt[NDB];   // K^T operands (one per head-dim block) of the tile accumulated next interval

    __syncthreads();   // tile 0 is in LDS
    for (int it = 0; it <= n_tiles; ++it) {
      // tile it+3 goes into the stage of tile it-1: the producers read it during the last interval, and its
      // K^T operands are in this wave's registers since then
      if (it + 3 < n_tiles) issue_loads(it + 3);
      if (it > 0) {
        const unsigned char* xi = xr + ((it - 1) & 1) * XCH_BYTES;
        bf16x8 ds[NSUB];
#pragma unroll
        for (int s = 0; s < NSUB; ++s) ds[s] = *reinterpret_cast<const bf16x8*>(xi + s * 1024);
        __builtin_amdgcn_sched_barrier(0);
        // dQ^T += K^T dS^T
#pragma unroll
        for (int e = 0; e < NDB; ++e)
#pragma unroll
          for (int s = 0; s < NSUB; ++s) dq[s][e] = mfma32(kt[e], ds[s], dq[s][e]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (it < n_tiles) {
        const unsigned char* kh = smem + (it & (NSTAGE - 1)) * STAGE_BYTES;
#pragma unroll
        for (int e = 0; e < NDB; ++e) kt[e] = tr_pair(kh + e * 256 + toff0, kh + e * 256 + toff1);
      }
      // tile it+1 must have landed before the barrier; tiles it+2 and it+3 may stay in flight
      if (it + 3 < n_tiles) wait_vm<4 * IPT>();
      else if (it + 2 < n_tiles) wait_vm<2 * IPT>();
      else wait_vm<0>();
      __syncthreads();
    }

    // ---- epilogue: lane owns a query row, register r the head-dim column crow(r) of a block
#pragma unroll
    for (int s = 0; s < NSUB; ++s) {
      const int head = b.hk * p.G + b.hc * p.GP + s / p.RSH;
      const int row = b.blk_row0 + (s % p.RSH) * 32 + l32;
      if (row >= R) continue;
      u16* op = p.dq.ptr + (int64_t)(b.row_begin + row) * p.dq.ts + (int64_t)head * p.dq.hs;
#pragma unroll
      for (int e = 0; e < NDB; ++e)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 w;
          w.x = pack2_bf16(dq[s][e][r4 * 4 + 0] * p.scale, dq[s][e][r4 * 4 + 1] * p.scale);
          w.y = pack2_bf16(dq[s][e][r4 * 4 + 2] * p.scale, dq[s][e][r4 * 4 + 3] * p.scale);
          *reinterpret_cast<u32x2*>(op + (jb + 4 * e) * 32 + r4 * 8 + hi * 4) = w;
        }
    }
  }
}

template <bool LOCAL>
hipError_t launch_t(AttnParams p, hipStream_t st) {
  fill_packing(p, NSUB);
  hipError_t e = ensure_dynamic_lds<dq512_kernel<LOCAL>>(SMEM_BYTES);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(dq512_kernel<LOCAL>, dim3((unsigned)nblk), dim3(512), SMEM_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_dq512(const AttnParams& p, hipStream_t st) {
  if (p.window > 0) return hipErrorInvalidValue;   // (the interface offers no window at this head dim)
  return launch_t<false>(p, st);
}

}  // namespace dkv
