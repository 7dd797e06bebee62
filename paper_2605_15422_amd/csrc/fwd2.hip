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
//   * LDS is double-buffered: global loads for tile t+2 are in flight and tile t+1 is written to the
//     other buffer while tile t is consumed; one barrier per tile.
#include "common.h"
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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

  // ---- staging: thread -> CPT chunks of K and of V
  const u16* kc_base = p.kc.ptr + (int64_t)b.hk * p.kc.hs;
  const u16* vc_base = p.vc.ptr + (int64_t)b.hk * p.vc.hs;
  const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
  const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
  const int n_ctx_run = b.n_ctx - b.c0;
  int st_row[C::CPT], st_col[C::CPT], st_koff[C::CPT], st_voff[C::CPT];
#pragma unroll
  for (int j = 0; j < C::CPT; ++j) {
    const int id = tid + j * C::NT;
    st_row[j] = id / C::CPR;
    st_col[j] = (id % C::CPR) * 8;
    st_koff[j] = st_row[j] * C::RB + (((id % C::CPR) ^ C::fK(st_row[j])) << 4);
    st_voff[j] = st_row[j] * C::RB + (((id % C::CPR) ^ C::fV(st_row[j])) << 4);
  }
  u32x4 kst[C::CPT], vst[C::CPT];
  auto issue_loads = [&](int it) {
    const bool is_ctx = it < n_ctx_run;
    const int key0 = is_ctx ? (b.c0 + it) * BN : (b.d0 + it - n_ctx_run) * BN;
    const u16* kb = is_ctx ? kc_base : kd_base;
    const u16* vb = is_ctx ? vc_base : vd_base;
    const int64_t kts = is_ctx ? p.kc.ts : p.kd.ts, vts = is_ctx ? p.vc.ts : p.vd.ts;
    const int nvalid = (is_ctx ? P : R) - key0;
#pragma unroll
    for (int j = 0; j < C::CPT; ++j) {
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
    unsigned char* kb = smem + buf * 2 * C::TILE_BYTES;
    unsigned char* vb = kb + C::TILE_BYTES;
#pragma unroll
    for (int j = 0; j < C::CPT; ++j) {
      *reinterpret_cast<u32x4*>(kb + st_koff[j]) = kst[j];
      *reinterpret_cast<u32x4*>(vb + st_voff[j]) = vst[j];
    }
  };

  issue_loads(0);
  store_stage(0);
  if (b.n_tiles > 1) issue_loads(1);
  __syncthreads();

  for (int it = 0; it < b.n_tiles; ++it) {
    if (it + 1 < b.n_tiles) store_stage((it + 1) & 1);
    if (it + 2 < b.n_tiles) issue_loads(it + 2);

    const unsigned char* Kb = smem + (it & 1) * 2 * C::TILE_BYTES;
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
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int i = 0; i < C::KVSUB * C::KS - 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
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
    __syncthreads();
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
  const size_t smem = 4 * C::TILE_BYTES;
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
