// Forward kernel for head dim 512 (Alg. 3 of the paper re-tiled for CDNA4; the "split tiling for head_dim 512")
// with producer / consumer wave specialisation.  Same work decomposition as the other Q-stationary kernels.
//
// What this head dim dictates.  The fp32 O of one row fills 2 KB and the four consumer waves can give 128 of their
// 256 registers to accumulators: a workgroup owns 64 rows (two 32-row subtiles), each consumer wave holding four
// of the sixteen 32-wide head-dim blocks of O^T for both.  Each of the four producers keeps the Q fragments of 16
// rows (64 registers) and works with the 16x16x32 MFMA: per 16-key tile it forms S^T = K Q^T and the online
// softmax (reference maximum moved lazily, row sum) and publishes P^T as the bf16 B operand of the consumers'
// 32x32x16 product, with the rescaling factor of every row (1 unless the maximum moved) and a flag; the
// consumers, one tile behind, add V^T P^T with V^T from LDS transpose reads.  K / V tiles of 16 keys (16 KB +
// 16 KB) travel global -> LDS three tiles ahead into four stages, issued by the consumers, which read their V^T
// operands one interval early.  Per tile a producer issues 16 small MFMAs, a consumer 8; one barrier per tile.
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
constexpr int FAC_OFF = NSUB * 1024;             // [subtile][lane] x 16 B, then the factors
constexpr int FLAG_OFF = FAC_OFF + NSUB * 128;   // [subtile][32 rows] fp32, then one flag word per producer wave
constexpr int XCH_BYTES = FLAG_OFF + 256;
constexpr int SMEM_BYTES = XCH_OFF + 2 * XCH_BYTES;
constexpr int IPT = TILE_BYTES / 1024 / 4;       // 1 KB load instructions per consumer wave, tile and tensor

template <bool LOCAL>
__global__ __launch_bounds__(512) void fwd512_kernel(const AttnParams p) {
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
    // accumulator: column l16, register r <-> row 4 g + r.  Here A = K (LDS, row = key), B = Q (registers, column =
    // query row): the lane owns a query row and the keys 4 g + r of the tile; the four lanes l16 + 16 g' share a row.
    // Lane group g takes chunk cg = (0, 3, 1, 2)[g] of a 64-byte k-step (both operands agree on it), which keeps
    // the 16-byte LDS reads of the sixteen-lane groups the hardware serves together on different bank groups.
    const float c = p.scale_log2;
    const int l16 = lane & 15, g = lane >> 4;
    const int cg = (0x9C >> (2 * g)) & 3;
    const int sub = wave >> 1;
    const int head = b.hk * p.G + b.hc * p.GP + sub / p.RSH;
    const int row0 = b.blk_row0 + (sub % p.RSH) * 32 + (wave & 1) * 16;
    const int row = row0 + l16;
    const bool wave_valid = row0 < R;

    bf16x8 qf[KS];
    {
      const int r = min(row, R - 1);
      const u16* qp = p.q.ptr + (int64_t)(b.row_begin + r) * p.q.ts + (int64_t)head * p.q.hs + cg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
      // consumed (and therefore waited for) here: no compiler-placed vector-memory wait inside the main loop
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : : "v"(qf[ks]));
    }
    // K operand of k-step ks: key row l16, chunk 4 ks + cg; with the tile swizzle its position is
    // 4 ((ks % 4) ^ (row % 4)) + (cg ^ (row / 4 % 4)) + 16 (ks / 4): four per-lane offsets serve all k-steps.
    int roff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) roff[j] = l16 * RB + 64 * (j ^ (l16 & 3)) + 16 * (cg ^ ((l16 >> 2) & 3));
    unsigned char* xbase = smem + XCH_OFF;
    // consumer B operand (32x32x16): lane (row of the subtile, hi'), element e <-> key 4 hi' + 8 (e / 4) + e % 4 of
    // the tile.  This lane holds keys 4 g + r: hi' = g % 2, elements 4 (g / 2) .. + 3.
    const int xw_off = sub * 1024 + ((g & 1) * 32 + (wave & 1) * 16 + l16) * 16 + (g >> 1) * 8;
    const int fac_off = FAC_OFF + sub * 128 + ((wave & 1) * 16 + l16) * 4;
    const int flag_off = FLAG_OFF + wave * 4;

    const int ctx_masked = (P % BN) ? b.n_ctx - 1 : -1;   // the partial last prompt tile
    const int dec_masked = min(row0 + 1, R) / BN;         // response tiles from the diagonal (or the sequence end) on
    float m_ref = NEG_BIG, l_sum = 0.f;
    float thr = (m_ref + 8.0f) / c;   // an (unscaled) row maximum above this moves the reference

    __syncthreads();   // tile 0 is in LDS
    for (int it = 0; it < n_tiles; ++it) {
      const unsigned char* kh = smem + (it & (NSTAGE - 1)) * STAGE_BYTES;
      const bool is_ctx = it < n_ctx_run;
      const int kt = is_ctx ? b.c0 + it : b.d0 + it - n_ctx_run;
      const int key0 = kt * BN;
      // most tiles are entirely visible to the 16 rows of this wave: no tests for them
      const bool plain = wave_valid && (is_ctx ? kt != ctx_masked : kt < dec_masked);
      const bool active = plain || (wave_valid && (is_ctx || key0 <= row0 + 15) && key0 < (is_ctx ? P : R));
      unsigned char* xo = xbase + (it & 1) * XCH_BYTES;
      uint32_t moved = 0u;
      float alpha = 1.0f;
      if (__builtin_expect(active, 1)) {
        // S^T = K Q^T: operands in groups of four, the next group requested before the MFMAs of the current one
        constexpr int GRP = 4, NG = KS / GRP;
        bf16x8 op[2][GRP];
        auto request = [&](int gi, bf16x8* out) __attribute__((always_inline)) {
#pragma unroll
          for (int q = 0; q < GRP; ++q) {
            const int ks = gi * GRP + q;
            out[q] = *reinterpret_cast<const bf16x8*>(kh + roff[ks & 3] + (ks >> 2) * 256);
          }
        };
        request(0, op[0]);
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
          if (gi + 1 < NG) request(gi + 1, op[(gi + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int q = 0; q < GRP; ++q) s = mfma16(op[gi & 1][q], qf[gi * GRP + q], s);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (!plain) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (!visible<LOCAL>(is_ctx, key0 + 4 * g + r, row, P, R, W)) s[r] = -INFINITY;
        }
        // This lane's four scores of the row (the lanes l16 + 16 g' hold the other twelve; their own tests cover them:
        // the branch is taken if ANY lane exceeds the threshold).  The reference maximum is kept until some row's
        // maximum outgrows it by 2^8 (lazy rescaling); the row maximum itself is only formed then.
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        if (__any(mx > thr)) {
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32)) * c;
          const float mn = fmaxf(m_ref, mx);
          alpha = __builtin_amdgcn_exp2f(m_ref - mn);
          m_ref = mn;
          thr = (m_ref + 8.0f) / c;
          l_sum *= alpha;
          moved = 1u;
        }
        float ev[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) ev[r] = __builtin_amdgcn_exp2f(s[r] * c - m_ref);
        l_sum += (ev[0] + ev[1]) + (ev[2] + ev[3]);
        u32x2 w;
        w.x = pack2_bf16(ev[0], ev[1]);
        w.y = pack2_bf16(ev[2], ev[3]);
        *reinterpret_cast<u32x2*>(xo + xw_off) = w;
      } else {
        // nothing visible: the consumers do not branch on activity, they add a product with P = 0
        const u32x2 z = {0u, 0u};
        *reinterpret_cast<u32x2*>(xo + xw_off) = z;
      }
      // the factor of this lane's row (the four lanes of a row store the same value), the flag of this wave
      *reinterpret_cast<float*>(xo + fac_off) = alpha;
      if (lane == 0) *reinterpret_cast<uint32_t*>(xo + flag_off) = moved;
      __syncthreads();
    }
    // the row sums: 1 / l for the consumers (in the factor slots of the buffer the last tile did not use), LSE
    float l = l_sum + __shfl_xor(l_sum, 16);
    l += __shfl_xor(l, 32);
    *reinterpret_cast<float*>(xbase + (n_tiles & 1) * XCH_BYTES + fac_off) = 1.0f / l;
    if (g == 0 && row < R) p.lse[(int64_t)head * p.total + b.row_begin + row] = (m_ref + log2f(l)) * LN2;
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

    f32x16 o[NSUB][NDB];
#pragma unroll
    for (int s = 0; s < NSUB; ++s)
#pragma unroll
      for (int e = 0; e < NDB; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[s][e][r] = 0.f;
    // transpose reads: rows 4 hi + (lane % 16) / 4 and + 8 of the 16-key tile, head-dim block jb (blocks jb + 4,
    // jb + 8, jb + 12 lie 256, 512, 768 bytes further: the chunk index bits the swizzle leaves alone)
    const int toff0 = tr_off<D>(lane, hi * 4, jb * 32), toff1 = tr_off<D>(lane, hi * 4 + 8, jb * 32);
    const unsigned char* xbase = smem + XCH_OFF;
    bf16x8 vt[NDB];   // V^T operands (one per head-dim block) of the tile accumulated next interval

    __syncthreads();   // tile 0 is in LDS
    for (int it = 0; it <= n_tiles; ++it) {
      // tile it+3 goes into the stage of tile it-1: the producers read its K during the last interval, and its
      // V^T operands are in this wave's registers since then
      if (it + 3 < n_tiles) issue_loads(it + 3);
      if (it > 0) {
        const unsigned char* xi = xbase + ((it - 1) & 1) * XCH_BYTES;
        bf16x8 pp[NSUB];
        const u32x4 fl = *reinterpret_cast<const u32x4*>(xi + FLAG_OFF);   // one word per producer wave
#pragma unroll
        for (int s = 0; s < NSUB; ++s) pp[s] = *reinterpret_cast<const bf16x8*>(xi + s * 1024 + lane * 16);
        // subtiles whose reference maximum moved with this tile: rescale what was accumulated before it
        if (__builtin_expect(__builtin_amdgcn_readfirstlane((int)(fl.x | fl.y | fl.z | fl.w)) != 0, 0)) {
#pragma unroll
          for (int s = 0; s < NSUB; ++s) {
            if (__builtin_amdgcn_readfirstlane((int)(fl[2 * s] | fl[2 * s + 1])) == 0) continue;
            const float a = *reinterpret_cast<const float*>(xi + FAC_OFF + s * 128 + l32 * 4);
#pragma unroll
            for (int e = 0; e < NDB; ++e)
#pragma unroll
              for (int r = 0; r < 16; ++r) o[s][e][r] *= a;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T
#pragma unroll
        for (int e = 0; e < NDB; ++e)
#pragma unroll
          for (int s = 0; s < NSUB; ++s) o[s][e] = mfma32(vt[e], pp[s], o[s][e]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (it < n_tiles) {
        const unsigned char* vh = smem + (it & (NSTAGE - 1)) * STAGE_BYTES + TILE_BYTES;
#pragma unroll
        for (int e = 0; e < NDB; ++e) vt[e] = tr_pair(vh + e * 256 + toff0, vh + e * 256 + toff1);
      }
      // tile it+1 must have landed before the barrier; tiles it+2 and it+3 may stay in flight
      if (it + 3 < n_tiles) wait_vm<4 * IPT>();
      else if (it + 2 < n_tiles) wait_vm<2 * IPT>();
      else wait_vm<0>();
      __syncthreads();
    }

    // ---- epilogue: lane owns a query row, register r the head-dim column crow(r) of a block
    const unsigned char* xl = xbase + (n_tiles & 1) * XCH_BYTES;
#pragma unroll
    for (int s = 0; s < NSUB; ++s) {
      const int head = b.hk * p.G + b.hc * p.GP + s / p.RSH;
      const int row = b.blk_row0 + (s % p.RSH) * 32 + l32;
      if (row >= R) continue;
      const float inv = *reinterpret_cast<const float*>(xl + FAC_OFF + s * 128 + l32 * 4);
      u16* op = p.out_o.ptr + (int64_t)(b.row_begin + row) * p.out_o.ts + (int64_t)head * p.out_o.hs;
#pragma unroll
      for (int e = 0; e < NDB; ++e)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 w;
          w.x = pack2_bf16(o[s][e][r4 * 4 + 0] * inv, o[s][e][r4 * 4 + 1] * inv);
          w.y = pack2_bf16(o[s][e][r4 * 4 + 2] * inv, o[s][e][r4 * 4 + 3] * inv);
          *reinterpret_cast<u32x2*>(op + (jb + 4 * e) * 32 + r4 * 8 + hi * 4) = w;
        }
    }
  }
}

template <bool LOCAL>
hipError_t launch_t(AttnParams p, hipStream_t st) {
  fill_packing(p, NSUB);
  hipError_t e = ensure_dynamic_lds<fwd512_kernel<LOCAL>>(SMEM_BYTES);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(fwd512_kernel<LOCAL>, dim3((unsigned)nblk), dim3(512), SMEM_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd512(const AttnParams& p, hipStream_t st) {
  if (p.window > 0) return hipErrorInvalidValue;   // (the interface offers no window at this head dim)
  return launch_t<false>(p, st);
}

}  // namespace dkv
