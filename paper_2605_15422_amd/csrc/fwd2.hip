// Forward kernel for head dims 64 and 128 (Alg. 3 of the paper re-tiled for CDNA4), tuned variant.
//
// Same work decomposition as the generic Q-stationary kernel (one workgroup = BMR rows x GP packed
// query heads of one KV head, prompt tiles then own-response tiles):
//   * 8 waves (two per SIMD), each owning ONE 32-row subtile: Q fragments (B operands) and the O^T
//     accumulator stay in registers (~200 VGPRs, no spills);
//   * K and V tiles (64 keys) are staged row-major, un-padded, XOR-swizzled by row so that both the
//     16-byte K operand reads and the transposing V reads are bank-conflict free; V^T operands come
//     from ds_read_b64_tr_b16 (LDS transpose read), so nothing is transposed on the way into LDS;
//   * the tiles travel global -> LDS directly (global_load_lds) into two rings of four slots, K three
//     tiles ahead (requested by waves 0-3) and V two (waves 4-7): no staging registers, no LDS stores, one
//     barrier per tile;
//   * each wave runs a software pipeline over 32-key half tiles: while the VALU does the softmax of
//     half g, the matrix pipe computes the scores of half g+1 and the P V product of half g-1.  Two
//     waves per SIMD do not hide a wave's own MFMA -> softmax -> MFMA dependency chain on this chip
//     (their phases drift together at every barrier); interleaving independent work inside one
//     instruction stream does.
#include <type_traits>
#include "common.h"
#include "dma.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {

constexpr int kFwdWaves = 8;   // the K / V loader split below assumes eight waves

template <int D>
struct F2Cfg {
  static constexpr int NW = kFwdWaves, NT = NW * 64, BN = 64;
  static constexpr int KS = D / 16, DSUB = D / 32;
  static constexpr int RB = 2 * D;                 // row bytes
  static constexpr int CPR = D / 8;                // 16-byte chunks per row
  static constexpr int RPL = CPR < 16 ? 16 / CPR : 1;   // rows per 256-byte bank line
  static constexpr int TILE_BYTES = BN * RB;
  __device__ static __forceinline__ int fK(int row) { return (row / RPL) % CPR; }
  __device__ static __forceinline__ int fV(int row) { return 4 * ((row / RPL) % (CPR / 4)); }
};

template <int D, bool LOCAL>
__global__ __launch_bounds__(kFwdWaves * 64) void fwd2_kernel(const AttnParams p) {
  using C = F2Cfg<D>;
  constexpr int BN = C::BN;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // K ring [4 tiles] | V ring [4 tiles]
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

  bf16x8 qf[C::KS];
  {
    const int r = min(row, R - 1);
    const u16* qp = p.q.ptr + (int64_t)(b.row_begin + r) * p.q.ts + (int64_t)head * p.q.hs + hi * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    // consumed (and therefore waited for) here: no compiler-placed vector-memory wait inside the main loop
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : : "v"(qf[ks]));
  }

  f32x16 oacc[C::DSUB];
#pragma unroll
  for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[ds][r] = 0.f;
  float m_ref = NEG_BIG, l_sum = 0.f;

  // ---- per-lane LDS offsets (bytes, relative to a tile base)
  int koff[C::KS];          // K operand: row l32 (+32*half), chunk 2*ks+hi
#pragma unroll
  for (int ks = 0; ks < C::KS; ++ks) koff[ks] = l32 * C::RB + (((2 * ks + hi) ^ C::fK(l32)) << 4);
  int voff[C::DSUB];        // V transpose read: row (lane%16)/4 (+ key base), 4 head-dim values at 16*((lane/16)%2)+4*(lane%4)
  {
    const int r16 = lane & 15, g = (lane >> 4) & 1;
    const int vrow = hi * 4 + (r16 >> 2);
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds) {
      const int dcol = ds * 32 + g * 16 + (r16 & 3) * 4;
      voff[ds] = vrow * C::RB + ((((dcol >> 3)) ^ C::fV(vrow)) << 4) + ((dcol >> 2) & 1) * 8;
    }
  }

  // ---- global -> LDS tile loads: instruction j = lwave + LW t of a tile covers RPI key rows; lane l lands at
  // LDS chunk position l % CPR of row l / CPR of the instruction and fetches the chunk the swizzle stores
  // there (both swizzles have a period that divides LW RPI rows, so one offset per tensor serves every t).
  // Keys past the end of the region re-read the last key: their scores are masked like any invisible key.
  const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;
  constexpr int NSTAGE = 4;                           // ring slots per tensor: K ring, then V ring
  constexpr int V_RING = NSTAGE * C::TILE_BYTES;
  // the K tiles are requested by waves 0-3, the V tiles by waves 4-7: one address computation per wave and tile
  constexpr int LW = C::NW / 2;                       // waves per tensor
  constexpr int IPT = C::TILE_BYTES / 1024 / LW;      // 1 KB load instructions per wave and tile
  constexpr int RPI = 1024 / C::RB;                   // rows per load instruction
  static_assert(IPT >= 1, "tile must split evenly over the waves");
  const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  const int lwave = wave % LW;
  const bool v_loader = wave >= LW;
  const int ld_row0 = lwave * RPI + lane / C::CPR;
  const int ld_kcoff = ((lane % C::CPR) ^ C::fK(ld_row0)) * 16;
  const int ld_vcoff = ((lane % C::CPR) ^ C::fV(ld_row0)) * 16;
  // which = 0: K tile `it` into the K ring, 1: V tile `it` into the V ring (slot it % 4)
  const int tsb_c[2] = {(int)p.kc.ts * 2, (int)p.vc.ts * 2}, tsb_d[2] = {(int)p.kd.ts * 2, (int)p.vd.ts * 2};
  auto issue_tile = [&](int it, int which) __attribute__((always_inline)) {
    const bool is_ctx = it < n_ctx_run;
    const int kt = is_ctx ? b.c0 + it : b.d0 + it - n_ctx_run;
    const int tsb = is_ctx ? tsb_c[which] : tsb_d[which];   // bytes per token
    const u16* base = is_ctx ? (which ? vc_base : kc_base) : (which ? vd_base : kd_base);
    const unsigned char* tb = reinterpret_cast<const unsigned char*>(base) + (int64_t)(kt * BN) * tsb;
    const int last = (is_ctx ? P : R) - kt * BN - 1;
    const uint32_t dst = smem_addr + which * V_RING + (it & (NSTAGE - 1)) * C::TILE_BYTES + lwave * 1024;
    const int coff = which ? ld_vcoff : ld_kcoff;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
      const int r = min(ld_row0 + t * LW * RPI, last);
      dma16(uniform_ptr(reinterpret_cast<const u16*>(tb)), (uint32_t)(__umul24((unsigned)r, (unsigned)tsb) + coff),
            dst + t * LW * 1024);
    }
  };

  // ---- the three pieces of work of a 32-key half tile
  // S^T half = K_half Q^T
  auto s_half = [&](const unsigned char* Kh, f32x16& s) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kh + koff[ks]);
      s = mfma32(a, qf[ks], s);
    }
  };
  // O^T += V_half^T P_half^T
  auto pv_half = [&](const unsigned char* Vh, const bf16x8 (&pp)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      const unsigned char* vrow = Vh + t2 * 16 * C::RB;
#pragma unroll
      for (int ds = 0; ds < C::DSUB; ++ds) {
        const bf16x8 a = tr_pair(vrow + voff[ds], vrow + 8 * C::RB + voff[ds]);
        oacc[ds] = mfma32(a, pp[t2], oacc[ds]);
      }
    }
  };
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  // One step of the software pipeline: the softmax of half tile g (scores in `sc`) runs on the VALU while the
  // matrix pipe computes the scores of half g+1 (into `sn`) and accumulates the P V product of half g-1
  // (`pprev`); the three are independent.  Measured on this chip, a SIMD issues one VALU-class instruction
  // (MFMA included) per ~5 cycles over all its waves, so a 32-cycle MFMA hides about six of them if independent
  // ones are next in the stream; the softmax needs 4.5 per MFMA at d = 128.  The step consists of
  // NSLOT slots of {one MFMA, the softmax of 16 / NSLOT scores} in groups of four.  All operand reads of a
  // group are requested at the start of the previous group, and a group's MFMAs consume their operands in the
  // reverse of the request order, so one wait per group covers them all; the softmax of a score is spread
  // over three slots so that no instruction of a slot depends on another one of the same slot.  Fences keep
  // the compiler from regrouping.  The operands of the first group are requested by the previous step
  // (`pre`), those of the next step's first group here.
  constexpr int NS = C::KS, NPV = 2 * C::DSUB, NSLOT = NS + NPV, EPS = 16 / NSLOT, LEAD = 4, NG = NSLOT / LEAD;
  static_assert(NS == NPV && 16 % NSLOT == 0 && NSLOT % LEAD == 0, "slot layout");
  auto k_operand = [&](const unsigned char* Kh, int ks) __attribute__((always_inline)) {
    return *reinterpret_cast<const bf16x8*>(Kh + koff[ks]);
  };
  auto v_operand = [&](const unsigned char* Vh, int j) __attribute__((always_inline)) {
    const unsigned char* vrow = Vh + (j / C::DSUB) * 16 * C::RB;
    return tr_pair(vrow + voff[j % C::DSUB], vrow + 8 * C::RB + voff[j % C::DSUB]);
  };
  // slot i < NS: score MFMA of k-step i; slot NS + j: product MFMA j
  auto operand = [&](const unsigned char* Kh, const unsigned char* Vh, int i) __attribute__((always_inline)) {
    return i < NS ? k_operand(Kh, i) : v_operand(Vh, i - NS);
  };
  float thr = (m_ref + 8.0f) / c;   // an (unscaled) row maximum above this moves the reference
  // (plain C: the compiler must see these reads of MFMA results to place the wait states they need)
  auto lane_max = [&](const f32x16& v) __attribute__((always_inline)) {
    float m = fmaxf(fmaxf(v[0], v[1]), v[2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) m = fmaxf(fmaxf(m, v[r]), v[r + 1]);
    return fmaxf(m, v[15]);
  };
  // mx: on entry the maximum of this lane's 16 scores in `sc` before masking, on exit that of `sn`
  auto step = [&](bool masked, float& mx, f32x16& sc, f32x16& sn, bf16x8 (&pprev)[2], bf16x8 (&pcur)[2], bf16x8 (&pre)[LEAD],
                  const unsigned char* Kn, const unsigned char* Vp, const unsigned char* Kn2, const unsigned char* Vn2,
                  bool is_ctx, int keyh0) __attribute__((always_inline)) {
    if (masked) {
      // visible keys of this lane's row: lo < key < lim (indices inside the region)
      int lim, lo = -1;
      if (is_ctx) {
        lim = P;
        if (LOCAL) lo = P + row - W;
      } else {
        lim = min(row + 1, R);
        if (LOCAL) lo = row - W;
      }
      lim -= keyh0 + 4 * hi;
      lo -= keyh0 + 4 * hi;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int k = 8 * (r >> 2) + (r & 3);
        const bool vis = LOCAL ? (k < lim && k > lo) : (k < lim);
        sc[r] = vis ? sc[r] : -INFINITY;
      }
    }
    // Row maximum of this lane's 16 scores (the partner lane l ^ 32 holds the other 16 of the row; its own
    // test below covers them: the branch is taken if ANY lane exceeds the threshold).  It was formed in the
    // shadow of the previous step's last MFMAs; only a masked half tile has to form it again.
    if (masked) mx = lane_max(sc);
    // rescale lazily: keep the reference maximum until some row's maximum outgrows it by 2^8.  The product of
    // the previous half was formed against the old reference, so it is accumulated before the rescale (and
    // the slots below then add a product with P = 0).
    if (__any(mx > thr)) {
      mx = xor32_max(mx) * c;
      pv_half(Vp, pprev);
      pprev[0] = __builtin_bit_cast(bf16x8, zero4);
      pprev[1] = __builtin_bit_cast(bf16x8, zero4);
      const float mn = fmaxf(m_ref, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
      m_ref = mn;
      thr = (m_ref + 8.0f) / c;
      l_sum *= alpha;
#pragma unroll
      for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[ds][r] *= alpha;
    }
    // (the exponentials below must not be computed ahead of the branch above)
    asm volatile("" : "+v"(m_ref));
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 ob[NSLOT];
#pragma unroll
    for (int i = 0; i < LEAD; ++i) ob[i] = pre[i];
    uint32_t pw[8];
    float tv[16 + 2 * EPS], ev[16 + EPS];
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int e = 0; e < 2 * EPS; ++e) tv[e] = sc[e] * c - m_ref;
#pragma unroll
    for (int e = 0; e < EPS; ++e) ev[e] = __builtin_amdgcn_exp2f(tv[e]);
    bool first_s = true;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
#pragma unroll
      for (int q = 0; q < LEAD; ++q) {
        const int i = g * LEAD + (LEAD - 1 - q);   // reverse of the request order
        if (i >= NS) {
          const int j = i - NS;
          oacc[j % C::DSUB] = mfma32(ob[i], pprev[j / C::DSUB], oacc[j % C::DSUB]);
        } else if (first_s) {
          f32x16 z;
#pragma unroll
          for (int r = 0; r < 16; ++r) z[r] = 0.f;
          sn = mfma32(ob[i], qf[i], z);
          first_s = false;
        } else {
          sn = mfma32(ob[i], qf[i], sn);
        }
        if (q == 0) {
          // request the next group's operands (the next step's first group at the end)
#pragma unroll
          for (int n = 0; n < LEAD; ++n) {
            const int i2 = (g + 1) * LEAD + n;
            if (i2 < NSLOT) ob[i2] = operand(Kn, Vp, i2);
            else pre[n] = operand(Kn2, Vn2, n);
          }
        }
#pragma unroll
        for (int e = (g * LEAD + q) * EPS; e < (g * LEAD + q + 1) * EPS; ++e) {
          if (e + 2 * EPS < 16) {
            tv[e + 2 * EPS] = sc[e + 2 * EPS] * c - m_ref;
            asm volatile("" : "+v"(tv[e + 2 * EPS]));   // (keeps this slot's softmax work inside the slot)
          }
          if (e + EPS < 16) {
            ev[e + EPS] = __builtin_amdgcn_exp2f(tv[e + EPS]);
            asm volatile("" : "+v"(ev[e + EPS]));
          }
          if (e & 1) {
            ls1 += ev[e];
            pw[e >> 1] = pack2_bf16(ev[e - 1], ev[e]);
            asm volatile("" : "+v"(pw[e >> 1]), "+v"(ls1));
          } else {
            ls0 += ev[e];
            asm volatile("" : "+v"(ls0));
          }
        }
        if (g == NG - 1 && q == 1) {
          // the scores of the next half are complete: their maximum, needed at the top of the next step
          mx = lane_max(sn);
          asm volatile("" : "+v"(mx));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    l_sum += ls0 + ls1;
    u32x4 w0 = {pw[0], pw[1], pw[2], pw[3]}, w1 = {pw[4], pw[5], pw[6], pw[7]};
    pcur[0] = __builtin_bit_cast(bf16x8, w0);
    pcur[1] = __builtin_bit_cast(bf16x8, w1);
  };

  // ---- prologue: K0 V0 K1 V1 K2 requested, everything landed and published, scores of the first half
  if (v_loader) {
    issue_tile(0, 1);
    if (b.n_tiles > 1) issue_tile(1, 1);
  } else {
    issue_tile(0, 0);
    if (b.n_tiles > 1) issue_tile(1, 0);
    if (b.n_tiles > 2) issue_tile(2, 0);
  }
  wait_vm<0>();
  __syncthreads();

  const bool always_masked = LOCAL || !wave_valid;
  const int ctx_masked = (P % BN) ? b.n_ctx - 1 : -1;
  const int dec_masked = min(row0 + 1, R) / BN;
  f32x16 sA, sB;
  bf16x8 pA[2], pB[2];
  pB[0] = __builtin_bit_cast(bf16x8, zero4);
  pB[1] = __builtin_bit_cast(bf16x8, zero4);
  s_half(smem, sA);
  float mxs = lane_max(sA);
  bf16x8 pre[LEAD];   // operands of the first four slots of step (tile 0, half 0): K half 1 of tile 0, V with P = 0
#pragma unroll
  for (int i = 0; i < LEAD; ++i) pre[i] = operand(smem + 32 * C::RB, smem + V_RING + 32 * C::RB, i);

  for (int it = 0; it < b.n_tiles; ++it) {
    // K tile it+3 replaces K tile it-1, V tile it+2 replaces V tile it-2: both were last read before the
    // barrier that ended tile it-1
    const bool more = it + 3 < b.n_tiles;
    bool issued;
    if (v_loader) {
      issued = it + 2 < b.n_tiles;
      if (issued) issue_tile(it + 2, 1);
    } else {
      issued = more;
      if (issued) issue_tile(it + 3, 0);
    }

    const int slot = it & (NSTAGE - 1), slot_n = (it + 1) & (NSTAGE - 1), slot_p = (it > 0 ? it - 1 : 0) & (NSTAGE - 1);
    const unsigned char* Kt = smem + slot * C::TILE_BYTES;
    const unsigned char* Kn = smem + slot_n * C::TILE_BYTES;
    const unsigned char* Vt = smem + V_RING + slot * C::TILE_BYTES;
    const unsigned char* Vp = smem + V_RING + slot_p * C::TILE_BYTES + 32 * C::RB;
    const bool is_ctx = it < n_ctx_run;
    const int kt = is_ctx ? b.c0 + it : b.d0 + it - n_ctx_run;
    const int key0 = kt * BN;
    // tiles that can hold an invisible (row, key) pair for this wave: the partial last prompt tile, response
    // tiles from the diagonal (or the end of the sequence) on; windowed runs mask every tile
    const bool masked = always_masked || (is_ctx ? kt == ctx_masked : kt >= dec_masked);
    step(masked, mxs, sA, sB, pB, pA, pre, Kt + 32 * C::RB, Vp, Kn, Vt, is_ctx, key0);
    step(masked, mxs, sB, sA, pA, pB, pre, Kn, Vt, Kn + 32 * C::RB, Vt + 32 * C::RB, is_ctx, key0 + 32);
    // tiles it+2 (K) and it+1 (V) must have landed; the loads requested at the top of this tile may stay in flight
    if (issued) wait_vm<IPT>();
    else wait_vm<0>();
    __syncthreads();
  }
  // the product of the last half tile
  pv_half(smem + V_RING + ((b.n_tiles - 1) & (NSTAGE - 1)) * C::TILE_BYTES + 32 * C::RB, pB);

  // ---- epilogue: lane owns a query row, register r the head-dim column crow(r) of a 32-column block.  Stored from
  // here a row would leave in 16-byte pieces, 32 rows per instruction.  The wave's normalised 32 x D tile goes through
  // LDS instead: its own 32 rows of the K ring (free since the last barrier: only V is read after it; 16-byte chunks
  // XOR-swizzled by the row), read back as whole rows.  Wave-private: no barrier.
  const float l = xor32_sum(l_sum);
  const float inv = 1.0f / l;
  unsigned char* ot = smem + wave * 32 * C::RB;
#pragma unroll
  for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      u32x2 w;
      w.x = pack2_bf16(oacc[ds][r4 * 4 + 0] * inv, oacc[ds][r4 * 4 + 1] * inv);
      w.y = pack2_bf16(oacc[ds][r4 * 4 + 2] * inv, oacc[ds][r4 * 4 + 3] * inv);
      *reinterpret_cast<u32x2*>(ot + l32 * C::RB + (((ds * 4 + r4) ^ (l32 & (C::CPR - 1))) << 4) + hi * 8) = w;
    }
  if (hi == 0 && row < R) p.lse[(int64_t)head * p.total + b.row_begin + row] = (m_ref + log2f(l)) * LN2;
  constexpr int RPS = 64 / C::CPR;   // rows per store instruction
  const int chunk = lane % C::CPR;
#pragma unroll
  for (int i = 0; i < 32 / RPS; ++i) {
    const int tr = i * RPS + lane / C::CPR;
    const u32x4 w = *reinterpret_cast<const u32x4*>(ot + tr * C::RB + ((chunk ^ (tr & (C::CPR - 1))) << 4));
    if (row0 + tr < R) {
      u16* op = p.out_o.ptr + (int64_t)(b.row_begin + row0 + tr) * p.out_o.ts + (int64_t)head * p.out_o.hs;
      *reinterpret_cast<u32x4*>(op + chunk * 8) = w;
    }
  }
}

template <int D, bool LOCAL>
static hipError_t launch_fwd2_t(AttnParams p, hipStream_t st) {
  using C = F2Cfg<D>;
  fill_packing(p, C::NW);
  const size_t smem = 4 * 2 * C::TILE_BYTES;
  auto kern = fwd2_kernel<D, LOCAL>;
  hipError_t e = ensure_dynamic_lds<fwd2_kernel<D, LOCAL>>(smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(C::NT), smem, st, p);
  return hipGetLastError();
}

hipError_t launch_fwd2(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_fwd2_t<64, true>(p, st) : launch_fwd2_t<64, false>(p, st);
    case 128: return local ? launch_fwd2_t<128, true>(p, st) : launch_fwd2_t<128, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
