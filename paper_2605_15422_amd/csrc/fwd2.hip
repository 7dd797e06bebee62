// Forward kernel for head dims 64 and 128 (Alg. 3 of the paper re-tiled for CDNA4), tuned variant.
//
// Same work decomposition as the generic Q-stationary kernel (one workgroup = BMR rows x GP packed
// query heads of one KV head, prompt tiles then own-response tiles), but shaped for two waves per
// SIMD so that one wave's softmax (VALU / transcendental) overlaps the other wave's MFMAs:
//   * 8 waves, each owning ONE 32-row subtile: Q fragments (B operands) and the O^T accumulator stay
//     in registers (~200 VGPRs, no AGPR shuffling, no spills);
//   * K and V tiles (64 keys) are staged row-major, un-padded, XOR-swizzled by row so that both the
//     16-byte K operand reads and the transposing V reads are bank-conflict free; V^T operands come
//     from ds_read_b64_tr_b16 (LDS transpose read), so nothing is transposed on the way into LDS;
//   * the tiles travel global -> LDS directly (global_load_lds, three stages, two tiles ahead): no
//     staging registers, no LDS stores, one barrier per tile.
#include "common.h"
#include "dma.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {

#ifndef DKV_FWD_NW
#define DKV_FWD_NW 8
#endif

template <int D>
struct F2Cfg {
  static constexpr int NW = DKV_FWD_NW, NT = NW * 64, BN = 64;
  static constexpr int KS = D / 16, DSUB = D / 32, KVSUB = BN / 32;
  static constexpr int RB = 2 * D;                 // row bytes
  static constexpr int CPR = D / 8;                // 16-byte chunks per row
  static constexpr int RPL = CPR < 16 ? 16 / CPR : 1;   // rows per 256-byte bank line
  static constexpr int TILE_BYTES = BN * RB;
  static constexpr int CHUNKS = BN * CPR;
  static constexpr int CPT = CHUNKS / NT;          // chunks per thread (1 or 2)
  static_assert(CHUNKS % NT == 0, "tile must split evenly over the threads");
  __device__ static __forceinline__ int fK(int row) { return (row / RPL) % CPR; }
  __device__ static __forceinline__ int fV(int row) { return 4 * ((row / RPL) % (CPR / 4)); }
};

template <int D, bool LOCAL>
__global__ __launch_bounds__(DKV_FWD_NW * 64) void fwd2_kernel(const AttnParams p) {
  using C = F2Cfg<D>;
  constexpr int BN = C::BN;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // [2][K tile | V tile]
  QBlock b;
  if (!decode_qblock<BN>(p, b)) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int P = p.ctx_len, R = b.R, W = p.window;
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
  int koff[C::KS];          // K operand: row l32 (+32*kv), chunk 2*ks+hi
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

  // ---- global -> LDS tile loads: instruction j = wave + 8 t of a tile covers RPI key rows; lane l lands at
  // LDS chunk position l % CPR of row l / CPR of the instruction and fetches the chunk the swizzle stores
  // there (both swizzles have a period that divides 8 RPI rows, so one offset per tensor serves every t).
  // Keys past the end of the region re-read the last key: their scores are masked like any invisible key.
  const u16* kc_base = p.kc.ptr + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;
  constexpr int NSTAGE = 3, STAGE_BYTES = 2 * C::TILE_BYTES;
  constexpr int IPT = C::TILE_BYTES / 1024 / C::NW;   // 1 KB load instructions per wave, tile and tensor
  constexpr int RPI = 1024 / C::RB;                   // rows per load instruction
  static_assert(IPT >= 1 && NSTAGE == 3, "tile must split evenly over the waves");
  const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  const int ld_row0 = wave * RPI + lane / C::CPR;
  const int ld_kcoff = ((lane % C::CPR) ^ C::fK(ld_row0)) * 16;
  const int ld_vcoff = ((lane % C::CPR) ^ C::fV(ld_row0)) * 16;
  auto issue_loads = [&](int it, int stage) __attribute__((always_inline)) {
    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const int kts = (int)(is_ctx ? p.kc.ts : p.kd.ts), vts = (int)(is_ctx ? p.vc.ts : p.vd.ts);
    const u16* kb = uniform_ptr((is_ctx ? kc_base : kd_base) + (int64_t)key0 * kts);
    const u16* vb = uniform_ptr((is_ctx ? vc_base : vd_base) + (int64_t)key0 * vts);
    const int last = (is_ctx ? P : R) - key0 - 1;
    const uint32_t dst = smem_addr + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
    for (int t = 0; t < IPT; ++t) {
      const int r = min(ld_row0 + t * C::NW * RPI, last);
      dma16(kb, (uint32_t)(r * kts * 2 + ld_kcoff), dst + t * C::NW * 1024);
      dma16(vb, (uint32_t)(r * vts * 2 + ld_vcoff), dst + C::TILE_BYTES + t * C::NW * 1024);
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

  int stage = 0;
  for (int it = 0; it < b.n_tiles; ++it) {
    // tile it+2 goes into the stage that tile it-1 left at the last barrier
    if (it + 2 < b.n_tiles) issue_loads(it + 2, stage == 0 ? 2 : stage - 1);

    const unsigned char* Kb = smem + stage * STAGE_BYTES;
    const unsigned char* Vb = Kb + C::TILE_BYTES;
    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const bool active = wave_valid && tile_active<LOCAL, BN>(is_ctx, key0, row0, row0 + 31, P, W);

    if (active) {
      f32x16 s[C::KVSUB];
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kv][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kb + kv * 32 * C::RB + koff[ks]);
          s[kv] = mfma32(a, qf[ks], s[kv]);
        }
      }
      // instruction order: keep four K-operand reads in flight ahead of the MFMA that consumes them
      constexpr int DEPTH = 4;
      __builtin_amdgcn_sched_group_barrier(0x100, DEPTH, 0);
#pragma unroll
      for (int i = 0; i < C::KVSUB * C::KS - DEPTH; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, DEPTH, 0);
      if (tile_needs_mask<LOCAL, BN>(is_ctx, key0, row0, P, R, W)) {
#pragma unroll
        for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kv * 32 + crow(r, hi);
            if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) s[kv][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kv][r]);
      mx = xor32_max(mx) * c;
      // rescale lazily: keep the reference maximum until some row's maximum outgrows it by 2^8
      if (__any(mx > m_ref + 8.0f)) {
        const float mn = fmaxf(m_ref, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
        m_ref = mn;
        l_sum *= alpha;
#pragma unroll
        for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[ds][r] *= alpha;
      }
      float ls = 0.f;
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(s[kv][r] * c - m_ref);
          s[kv][r] = e;
          ls += e;
        }
      l_sum += ls;
      // O^T += V^T P^T
#pragma unroll
      for (int kv = 0; kv < C::KVSUB; ++kv)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          float tmp[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) tmp[e] = s[kv][t2 * 8 + e];
          const bf16x8 pb = pack8_bf16(tmp);
          const unsigned char* vrow = Vb + (kv * 32 + t2 * 16) * C::RB;
#pragma unroll
          for (int ds = 0; ds < C::DSUB; ++ds) {
            const bf16x8 a = tr_pair(vrow + voff[ds], vrow + 8 * C::RB + voff[ds]);
            oacc[ds] = mfma32(a, pb, oacc[ds]);
          }
        }
    }
    wait_loads(it + 2 < b.n_tiles);
    __syncthreads();
    stage = stage == 2 ? 0 : stage + 1;
  }

  const float l = xor32_sum(l_sum);
  if (row < R) {
    const float inv = 1.0f / l;
    u16* op = p.out_o.ptr + (int64_t)(b.row_begin + row) * p.out_o.ts + (int64_t)head * p.out_o.hs;
#pragma unroll
    for (int ds = 0; ds < C::DSUB; ++ds)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack2_bf16(oacc[ds][r4 * 4 + 0] * inv, oacc[ds][r4 * 4 + 1] * inv);
        w.y = pack2_bf16(oacc[ds][r4 * 4 + 2] * inv, oacc[ds][r4 * 4 + 3] * inv);
        *reinterpret_cast<u32x2*>(op + ds * 32 + r4 * 8 + hi * 4) = w;
      }
    if (hi == 0) p.lse[(int64_t)head * p.total + b.row_begin + row] = (m_ref + log2f(l)) * LN2;
  }
}

template <int D, bool LOCAL>
static hipError_t launch_fwd2_t(AttnParams p, hipStream_t st) {
  using C = F2Cfg<D>;
  fill_packing(p, C::NW);
  const size_t smem = 3 * 2 * C::TILE_BYTES;
  auto kern = fwd2_kernel<D, LOCAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
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
