// Forward kernel for head dim 256 (Alg. 3 of the paper re-tiled for CDNA4) with producer / consumer wave
// specialisation.  Same work decomposition as the other Q-stationary kernels (a workgroup owns row subtiles of
// the packed query heads of one KV head and walks the prompt tiles, then the own-response tiles).
//
// At this head dim the Q fragments (64 registers) and the O accumulator (128 registers) of a 32-row subtile do
// not fit one wave of 256 registers next to the score tile and the operands, so they live in different waves.
// A workgroup owns four 32-row subtiles (128 rows sharing the staged K / V tiles):
//   * producer wave w (0-3) keeps Q of subtile w in registers and forms, per 32-key tile, S^T = K Q^T and the
//     online softmax (running reference maximum moved lazily, row sum), and publishes P^T as the bf16 B operand
//     of the product through a double-buffered exchange area; when it moves the reference maximum it also
//     leaves the rescaling factor of every row and raises a flag;
//   * consumer wave c (4-7) owns the head-dim blocks c and c + 4 of O^T for ALL four subtiles (128 accumulator
//     registers) and, one tile behind, adds V^T P^T with V^T from LDS transpose reads of the row-major V tile
//     (every transposed operand feeds four MFMAs), after rescaling the subtiles whose flag is up.  The consumers
//     also issue the global -> LDS loads of K and V, three tiles ahead, into four stages, and read their V^T
//     operands one interval early, so that a stage is free again after one interval.
// Each SIMD runs one producer (16 MFMAs and the softmax per tile) and one consumer (16 MFMAs), one barrier per tile.
// LDS: 4 x (16 KB K + 16 KB V) + 2 x (8 KB P + factors and flags) = 146 KB.
#include "common.h"
#include "dma.h"
#include "launch.h"
#include "qsched.h"
#include "tiles.h"

namespace dkv {
namespace {

constexpr int D = 256;
constexpr int BN = 32, NSUB = 4;                 // keys per tile, 32-row subtiles per workgroup
constexpr int KS = D / 16, RB = 2 * D, CPR = D / 8;
constexpr int TILE_BYTES = BN * RB;
constexpr int NSTAGE = 4, STAGE_BYTES = 2 * TILE_BYTES;   // K tile | V tile
constexpr int XCH_OFF = NSTAGE * STAGE_BYTES;
constexpr int FAC_OFF = NSUB * 2048;             // [subtile][k-step 0,1][lane] x 16 B, then the factors
constexpr int FLAG_OFF = FAC_OFF + NSUB * 128;   // [subtile][32 rows] fp32, then one flag word per subtile
constexpr int XCH_BYTES = FLAG_OFF + 256;
constexpr int SMEM_BYTES = XCH_OFF + 2 * XCH_BYTES;
constexpr int OUT_RS = RB + 16;                  // row stride of the output tile staged in LDS (rows 4 banks apart)
static_assert(NSUB * 32 * OUT_RS <= XCH_OFF, "the output tile fits the stages");
constexpr int IPT = TILE_BYTES / 1024 / 4;       // 1 KB load instructions per consumer wave, tile and tensor
constexpr int RPI = 1024 / RB;                   // rows per load instruction

template <bool LOCAL>
__global__ __launch_bounds__(512) void fwd256_kernel(const AttnParams p) {
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
    const float c = p.scale_log2;
    const int head = b.hk * p.G + b.hc * p.GP + wave / p.RSH;
    const int row0 = b.blk_row0 + (wave % p.RSH) * 32;
    const int row = row0 + l32;
    const bool wave_valid = row0 < R;

    bf16x8 qf[KS];
    {
      const int r = min(row, R - 1);
      const u16* qp = p.q.ptr + (int64_t)(b.row_begin + r) * p.q.ts + (int64_t)head * p.q.hs + hi * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
      // consumed (and therefore waited for) here: no compiler-placed vector-memory wait inside the main loop
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : : "v"(qf[ks]));
    }
    // 16-byte row operand of k-step ks: row l32, chunk 2 ks + hi.  The swizzle (four bits) leaves bit 4 of the
    // chunk index alone: eight per-lane offsets serve the sixteen k-steps, the upper eight 256 bytes further.
    int roff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) roff[j] = tile_off<D>(l32, 2 * j + hi);
    unsigned char* xbase = smem + XCH_OFF;
    const int xw_off = wave * 2048 + lane * 16;
    const int fac_off = FAC_OFF + wave * 128 + l32 * 4;
    const int flag_off = FLAG_OFF + wave * 4;

    const bool never_plain = LOCAL || !wave_valid;
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
      // most tiles are entirely visible to the 32 rows of this wave: no tests for them
      const bool plain = !never_plain && (is_ctx ? kt != ctx_masked : kt < dec_masked);
      const bool active = plain || (wave_valid && tile_active<LOCAL, 32>(is_ctx, key0, row0, row0 + 31, P, W) &&
                                    key0 < (is_ctx ? P : R));
      unsigned char* xo = xbase + (it & 1) * XCH_BYTES;
      uint32_t moved = 0u;
      if (__builtin_expect(active, 1)) {
        // S^T = K Q^T: operands in groups of four, the next group requested before the MFMAs of the current one
        constexpr int GRP = 4, NG = KS / GRP;
        bf16x8 op[2][GRP];
        auto request = [&](int gi, bf16x8* out) __attribute__((always_inline)) {
#pragma unroll
          for (int q = 0; q < GRP; ++q) {
            const int ks = gi * GRP + q;
            out[q] = *reinterpret_cast<const bf16x8*>(kh + roff[ks & 7] + (ks >> 3) * 256);
          }
        };
        request(0, op[0]);
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
          if (gi + 1 < NG) request(gi + 1, op[(gi + 1) & 1]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int q = 0; q < GRP; ++q) s = mfma32(op[gi & 1][q], qf[gi * GRP + q], s);
          __builtin_amdgcn_sched_barrier(0);
        }
        const bool need = !plain && tile_needs_mask<LOCAL, 32>(is_ctx, key0, row0, P, R, W);
        if (__builtin_expect(need, 0)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + crow(r, hi);
            if (!visible<LOCAL>(is_ctx, key, row, P, R, W)) s[r] = -INFINITY;
          }
        }
        // Row maximum of this lane's 16 scores (the partner lane l ^ 32 holds the other 16 of the row; its own test
        // covers them: the branch is taken if ANY lane exceeds the threshold).  The reference maximum is kept until
        // some row's maximum outgrows it by 2^8 (lazy rescaling).
        float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
        for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
        mx = fmaxf(mx, s[15]);
        if (__any(mx > thr)) {
          mx = xor32_max(mx) * c;
          const float mn = fmaxf(m_ref, mx);
          const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
          m_ref = mn;
          thr = (m_ref + 8.0f) / c;
          l_sum *= alpha;
          if (hi == 0) *reinterpret_cast<float*>(xo + fac_off) = alpha;
          moved = 1u;
        }
        float ev[16];
        float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          ev[r] = __builtin_amdgcn_exp2f(s[r] * c - m_ref);
          ev[r + 1] = __builtin_amdgcn_exp2f(s[r + 1] * c - m_ref);
          ls0 += ev[r];
          ls1 += ev[r + 1];
        }
        l_sum += ls0 + ls1;
        *reinterpret_cast<bf16x8*>(xo + xw_off) = pack8_bf16(ev);
        *reinterpret_cast<bf16x8*>(xo + xw_off + 1024) = pack8_bf16(ev + 8);
      } else {
        // nothing visible: the consumers do not branch on activity, they add a product with P = 0
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(xo + xw_off) = z;
        *reinterpret_cast<u32x4*>(xo + xw_off + 1024) = z;
      }
      if (lane == 0) *reinterpret_cast<uint32_t*>(xo + flag_off) = moved;
      __syncthreads();
    }
    // the row sums: 1 / l for the consumers (in the factor slots of the buffer the last tile did not use), LSE
    const float l = xor32_sum(l_sum);
    if (hi == 0) *reinterpret_cast<float*>(xbase + (n_tiles & 1) * XCH_BYTES + fac_off) = 1.0f / l;
    if (hi == 0 && row < R) p.lse[(int64_t)head * p.total + b.row_begin + row] = (m_ref + log2f(l)) * LN2;
    __syncthreads();   // the consumers' last interval
  } else {
    // ================================= consumer ==============================================
    const int jb = wave - 4;
    const u16* kc_base = p.kc.ptr + (int64_t)b.ctx_off * p.kc.ts + (int64_t)b.hk * p.kc.hs;
    const u16* vc_base = p.vc.ptr + (int64_t)b.ctx_off * p.vc.ts + (int64_t)b.hk * p.vc.hs;
    const u16* kd_base = p.kd.ptr + (int64_t)b.row_begin * p.kd.ts + (int64_t)b.hk * p.kd.hs;
    const u16* vd_base = p.vd.ptr + (int64_t)b.row_begin * p.vd.ts + (int64_t)b.hk * p.vd.hs;
    // global -> LDS tile loads: instruction i = jb + 4 t of a tile covers RPI key rows; lane l lands at LDS chunk
    // position l % CPR of row l / CPR of the instruction and fetches the chunk the swizzle stores there.  The
    // swizzle has a period of 16 rows and the instructions of a wave are 8 rows apart: odd t flip bit 1 of the
    // chunk index.  Keys past the end of the region re-read the last key: their scores are masked like any
    // invisible key.
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    const int ld_row0 = jb * RPI + lane / CPR;
    const int ld_coff = ((lane % CPR) ^ swz<D>(ld_row0)) * 16;
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
        const unsigned row = (unsigned)min(ld_row0 + t * 4 * RPI, last);
        const uint32_t coff = (uint32_t)(ld_coff ^ ((t & 1) * 32));
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

    f32x16 o[NSUB][2];
#pragma unroll
    for (int s = 0; s < NSUB; ++s)
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[s][e][r] = 0.f;
    // transpose reads: rows 4 hi + (lane % 16) / 4 and + 8 of a 16-key group, head-dim block jb (block jb + 4 lies
    // 256 bytes further: bit 4 of the chunk index)
    const int toff0 = tr_off<D>(lane, hi * 4, jb * 32), toff1 = tr_off<D>(lane, hi * 4 + 8, jb * 32);
    const unsigned char* xbase = smem + XCH_OFF;
    bf16x8 vt[2][2];   // [16-key group][head-dim block]: V^T operands of the tile accumulated next interval

    __syncthreads();   // tile 0 is in LDS
    for (int it = 0; it <= n_tiles; ++it) {
      // tile it+3 goes into the stage of tile it-1: the producers read its K during the last interval, and its
      // V^T operands are in this wave's registers since then
      if (it + 3 < n_tiles) issue_loads(it + 3);
      if (it > 0) {
        const unsigned char* xi = xbase + ((it - 1) & 1) * XCH_BYTES;
        bf16x8 pp[2][NSUB];
        const u32x4 fl = *reinterpret_cast<const u32x4*>(xi + FLAG_OFF);
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int s = 0; s < NSUB; ++s)
            pp[t2][s] = *reinterpret_cast<const bf16x8*>(xi + s * 2048 + t2 * 1024 + lane * 16);
        // subtiles whose reference maximum moved with this tile: rescale what was accumulated before it
        if (__builtin_expect(__builtin_amdgcn_readfirstlane((int)(fl.x | fl.y | fl.z | fl.w)) != 0, 0)) {
#pragma unroll
          for (int s = 0; s < NSUB; ++s) {
            if (__builtin_amdgcn_readfirstlane((int)fl[s]) == 0) continue;
            const float a = *reinterpret_cast<const float*>(xi + FAC_OFF + s * 128 + l32 * 4);
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
              for (int r = 0; r < 16; ++r) o[s][e][r] *= a;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int s = 0; s < NSUB; ++s) o[s][e] = mfma32(vt[t2][e], pp[t2][s], o[s][e]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (it < n_tiles) {
        const unsigned char* vh = smem + (it & (NSTAGE - 1)) * STAGE_BYTES + TILE_BYTES;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int e = 0; e < 2; ++e)
            vt[t2][e] = tr_pair(vh + t2 * 16 * RB + e * 256 + toff0, vh + t2 * 16 * RB + e * 256 + toff1);
      }
      // tile it+1 must have landed before the barrier; tiles it+2 and it+3 may stay in flight
      if (it + 3 < n_tiles) wait_vm<4 * IPT>();
      else if (it + 2 < n_tiles) wait_vm<2 * IPT>();
      else wait_vm<0>();
      __syncthreads();
    }

    // ---- epilogue: lane owns a query row, register r the head-dim column crow(r) of a block.  Stored from here a
    // row would leave in 16-byte pieces, 32 rows per instruction; the normalised tile goes through LDS instead (the
    // stages are free now) and leaves as whole 512-byte rows, written by all eight waves.
    const unsigned char* xl = xbase + (n_tiles & 1) * XCH_BYTES;
#pragma unroll
    for (int s = 0; s < NSUB; ++s) {
      const float inv = *reinterpret_cast<const float*>(xl + FAC_OFF + s * 128 + l32 * 4);
      unsigned char* orow = smem + (s * 32 + l32) * OUT_RS;
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 w;
          w.x = pack2_bf16(o[s][e][r4 * 4 + 0] * inv, o[s][e][r4 * 4 + 1] * inv);
          w.y = pack2_bf16(o[s][e][r4 * 4 + 2] * inv, o[s][e][r4 * 4 + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + ((jb + 4 * e) * 32 + r4 * 8 + hi * 4) * 2) = w;
        }
    }
  }
  __syncthreads();   // the normalised tile is in LDS
  {
    // thread t: 16-byte piece t % 32 of tile rows t / 32, + 16, ...
    const int piece = tid & 31;
#pragma unroll
    for (int i = 0; i < NSUB * 32 / 16; ++i) {
      const int tr = i * 16 + (tid >> 5), s = tr >> 5;
      const int head = b.hk * p.G + b.hc * p.GP + s / p.RSH;
      const int row = b.blk_row0 + (s % p.RSH) * 32 + (tr & 31);
      if (row >= R) continue;
      const u32x4 w = *reinterpret_cast<const u32x4*>(smem + tr * OUT_RS + piece * 16);
      u16* op = p.out_o.ptr + (int64_t)(b.row_begin + row) * p.out_o.ts + (int64_t)head * p.out_o.hs;
      *reinterpret_cast<u32x4*>(op + piece * 8) = w;
    }
  }
}

template <bool LOCAL>
hipError_t launch_t(AttnParams p, hipStream_t st) {
  fill_packing(p, NSUB);
  hipError_t e = ensure_dynamic_lds<fwd256_kernel<LOCAL>>(SMEM_BYTES);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_seqs * p.MB * p.HC * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(fwd256_kernel<LOCAL>, dim3((unsigned)nblk), dim3(512), SMEM_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd256(const AttnParams& p, hipStream_t st) {
  return p.window > 0 ? launch_t<true>(p, st) : launch_t<false>(p, st);
}

}  // namespace dkv
