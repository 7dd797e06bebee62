// dK / dV kernel for head dim 512 with producer / consumer wave specialisation (the mathematics, the
// ownership rule and the row-block schedule of the narrower kernels: one workgroup owns a key tile of one KV
// head; a shared-prompt tile sums the contributions of ALL sequences and heads of the group in fp32 registers
// and is cast once -- Alg. 1 with the race of the shared prompt gradients removed by ownership).
//
// What this head dim dictates.  The fp32 dK and dV of one key fill 4 KB, and the four consumer waves can give
// 128 of their 256 registers to accumulators: the key tile is 32 keys, each consumer wave owning four of the
// sixteen 32-wide head-dim blocks of dK and dV.  A row block of Q and dO is 2 KB per row, so the LDS stages
// hold 16 rows (16 KB + 16 KB, four stages).  The K and -V fragments of 16 keys already fill 128 registers
// of a producer; the four producers are therefore two per 16-key half, and the two of a half take the row
// blocks in turn: a producer spends one interval on S = Q K^T of its block and the next one on D - dP, P and
// dS (16x16x32 MFMAs, everything of a block in the registers of one wave, in fp32), while its partner is one
// block behind.  Per interval every wave issues 8 MFMA-equivalents, one producer and one consumer per SIMD.
//
//   * producers (waves 0-3): Q / dO fragments are read from LDS as they are needed; P and -dS leave as bf16
//     MFMA operands through two exchange buffers (one per block parity), laid out as the consumers' 32x32x16
//     A operands; after their MFMAs they request the dO rows and the row statistics of the next block;
//   * consumers (waves 4-7): two row blocks behind, dV += P^T dO and -dK += (-dS)^T Q with dO^T / Q^T from LDS
//     transpose reads (taken one interval early); they walk the schedule, request the Q rows two row blocks
//     ahead and leave a header per stage (flags, rows, and where the block's dO rows and statistics are);
//   * the main loop is unrolled over the four stages (immediate LDS offsets), one barrier per row block.
#include <type_traits>
#include "common.h"
#include "dma.h"
#include "kvsched.h"
#include "launch.h"
#include "tiles.h"

namespace dkv {
namespace {

enum : int { HDR_VALID = 1, HDR_ACTIVE = 2, HDR_MASK = 4 };
template <int V>
using IC = std::integral_constant<int, V>;

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

constexpr int D = 512;
constexpr int BN = 32, HB = 16;                  // keys per workgroup, query rows per block
constexpr int KS = D / 32;                       // k-steps of the 16x16x32 MFMA
constexpr int NDB = D / 128;                     // head-dim blocks per consumer wave
constexpr int RB = 2 * D;
constexpr int HT_BYTES = HB * RB;                // one Q or dO row block
constexpr int STAT_OFF = 2 * HT_BYTES;           // lse2[16] | D[16]
constexpr int HDR_OFF = STAT_OFF + 256;          // {flags, row0, nvalid, end marks so far}, {dO address, statistics address}
constexpr int STAGE_BYTES = HDR_OFF + 64;
constexpr int NBUF = 4;
constexpr int XCH_OFF = NBUF * STAGE_BYTES;
constexpr int XCH_BYTES = 2048;                  // [P | dS][lane] x 16 B
constexpr int SMEM_BYTES = XCH_OFF + 2 * XCH_BYTES;
constexpr int IPB = HB / 4;                      // 1 KB load instructions (one row each) per wave, block and tensor
constexpr int HALF = (NBUF / 2) * STAGE_BYTES;   // second base register of every LDS operand (16-bit offset field)
static_assert(STAGE_BYTES + HT_BYTES + 1024 < 65536, "immediate offsets");

__global__ __launch_bounds__(512) void dkdv512_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;

  KVBlock kb;
  if (!decode_kvblock(p, BN, kb)) return;
  const bool is_ctx = kb.is_ctx;
  const int hk = kb.hk, key0 = kb.key0, seq_lo = kb.seq_lo, seq_hi = kb.seq_hi, P = kb.P;
  int region_len, key_row_begin;
  if (is_ctx) {
    region_len = P;
    key_row_begin = kb.ctx_off;
  } else {
    key_row_begin = p.cu ? p.cu[seq_lo] : 0;
    region_len = p.cu ? (p.cu[seq_lo + 1] - key_row_begin) : p.total;
  }

  if (wave < 4) {
    // ================================= producer ==============================================
    // 16x16x32 operands: lane = (l16, g): A row / B column l16, eight contraction indices of the k-step;
    // accumulator: column l16, register r <-> row 4 g + r.  Lane group g takes chunk cg = (0, 3, 1, 2)[g] of a
    // 64-byte k-step (both operands agree on it): a 16-byte LDS read is served in groups of sixteen lanes that
    // are not contiguous (lanes 0-3, 12-15, 20-23, 24-27 form the first one), and with this assignment the
    // fragment reads of such a group fall on sixteen different bank groups.
    const int kh = wave & 1, pb = wave >> 1;   // key half, parity of the row blocks this wave takes
    const int l16 = lane & 15, g = lane >> 4;
    const int cg = (0x9C >> (2 * g)) & 3;
    const float c = p.scale_log2;
    const int my_key = key0 + kh * 16 + l16;
    const u16 *kbase, *vbase;
    int64_t kts, vts;
    if (is_ctx) {
      kbase = p.kc.ptr + (int64_t)key_row_begin * p.kc.ts + (int64_t)hk * p.kc.hs;
      vbase = p.vc.ptr + (int64_t)key_row_begin * p.vc.ts + (int64_t)hk * p.vc.hs;
      kts = p.kc.ts;
      vts = p.vc.ts;
    } else {
      kbase = p.kd.ptr + (int64_t)key_row_begin * p.kd.ts + (int64_t)hk * p.kd.hs;
      vbase = p.vd.ptr + (int64_t)key_row_begin * p.vd.ts + (int64_t)hk * p.vd.hs;
      kts = p.kd.ts;
      vts = p.vd.ts;
    }
    bf16x8 kf[KS], vfn[KS];   // K and -V (sign bits flipped: exact)
    {
      const int kr = min(my_key, region_len - 1);   // clamp: gradients of padded keys are never stored
      const u16* kp = kbase + (int64_t)kr * kts + cg * 8;
      const u16* vp = vbase + (int64_t)kr * vts + cg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 32);
        u32x4 v = *reinterpret_cast<const u32x4*>(vp + ks * 32);
        v.x ^= 0x80008000u;
        v.y ^= 0x80008000u;
        v.z ^= 0x80008000u;
        v.w ^= 0x80008000u;
        vfn[ks] = __builtin_bit_cast(bf16x8, v);
      }
      // the loads are consumed (and therefore waited for) here, before the main loop
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : : "v"(kf[ks]), "v"(vfn[ks]));
    }
    // Q / dO fragment of k-step ks: row l16, chunk 4 ks + cg; with the tile swizzle its position is
    // 4 ((ks % 4) ^ (row % 4)) + (cg ^ (row / 4 % 4)) + 16 (ks / 4): four base registers serve all k-steps.
    const unsigned char* fr_lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) fr_lo[j] = smem + l16 * RB + 64 * (j ^ (l16 & 3)) + 16 * (cg ^ ((l16 >> 2) & 3));
    const unsigned char* fr_hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) fr_hi[j] = fr_lo[j] + HALF;
    const unsigned char* stat_lo = smem + STAT_OFF + 4 * g * 4;   // this lane's rows 4 g + r
    const unsigned char* stat_hi = stat_lo + HALF;
    // consumer A operand (32x32x16): lane (key, hi'), element e <-> row 4 hi' + 8 (e / 4) + e % 4 of the block.
    // This lane holds rows 4 g + r: hi' = g % 2, elements 4 (g / 2) .. + 3.
    unsigned char* xw = smem + XCH_OFF + pb * XCH_BYTES + ((g & 1) * 32 + kh * 16 + l16) * 16 + (g >> 1) * 8;

    // ---- the producers request the dO rows and the row statistics of a block (the consumers its Q rows).  A CU takes one
    // 1 KB request per ~17 cycles, and a wave waits at each request until it is taken: the 33 requests of a block keep
    // the memory pipeline busy for about as long as the block's MFMAs keep the matrix pipes busy.  The consumers make
    // theirs at the start of an interval, while the producers' MFMAs run, the producers after their MFMAs, while the
    // consumers' run.  dO and the statistics are first read one interval later than Q.  In interval t: block t + 1, whose header (with the
    // addresses) the consumers wrote in interval t - 1; this wave takes rows wave, wave + 4, ... as the consumers do for Q.
    // Row statistics: lanes 0-15 fetch LSE*log2e, lanes 16-31 fetch D (lanes 32-63 repeat them into the unused half
    // of the 256-byte area); both arrays live in one workspace, D first and LSE*log2e less than 4 GB behind it
    // (checked by the launcher), so one scalar base plus an unsigned 32-bit lane offset addresses both.
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    const uint32_t ld_lds = smem_addr + wave * 1024;
    const int do_neg = own_sgpr(-(int)p.dout.ts * 2);
    uint32_t voff_do[IPB];
#pragma unroll
    for (int t = 0; t < IPB; ++t) {
      const int row = wave + t * 4;
      voff_do[t] = (uint32_t)(-row * do_neg + ((lane ^ swz<D>(row)) * 16));
    }
    const uint32_t stat_lane_off = (lane & 16) ? 0u : (uint32_t)((const char*)p.lse2 - (const char*)p.dvec);
    bool issued = false;   // requests made in the current interval
    auto request_do = [&](auto NSc) __attribute__((always_inline)) {
      constexpr int NS = decltype(NSc)::value;
      const u32x4 h = *reinterpret_cast<const u32x4*>(smem + NS * STAGE_BYTES + HDR_OFF);
      const u32x4 a = *reinterpret_cast<const u32x4*>(smem + NS * STAGE_BYTES + HDR_OFF + 16);
      if (!(__builtin_amdgcn_readfirstlane((int)h.x) & HDR_VALID)) return;
      const int last = __builtin_amdgcn_readfirstlane((int)h.z) - 1;   // rows past the end re-read the last row
      const u16* dob = reinterpret_cast<const u16*>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)a.y) << 32) |
                                                    (uint32_t)__builtin_amdgcn_readfirstlane((int)a.x));
      static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
        constexpr int t = decltype(Tc)::value;
        const int over = max(wave + t * 4 - last, 0);
        dma16_at<NS * STAGE_BYTES + HT_BYTES + t * 4096>(dob, (uint32_t)__mul24(over, do_neg) + voff_do[t], ld_lds);
      });
      if (wave == 1) {
        const u16* stp = reinterpret_cast<const u16*>(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)a.w) << 32) |
                                                      (uint32_t)__builtin_amdgcn_readfirstlane((int)a.z));
        dma4_at<NS * STAGE_BYTES + STAT_OFF>(stp, stat_lane_off + (uint32_t)min(lane & 15, last) * 4u, smem_addr);
      }
      issued = true;
    };
    // end of an interval: the requests of the interval before this one have landed (in the next interval their first
    // readers start), this interval's may stay in flight
    auto end_interval = [&]() __attribute__((always_inline)) {
      if (__builtin_expect(issued, 1)) {
        if (wave == 1) wait_vm<IPB + 1>();
        else wait_vm<IPB>();
      } else {
        wait_vm<0>();
      }
      issued = false;
      __syncthreads();
    };

    int flags = 0, row0 = 0, nvalid = 0;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};   // scores of the block in flight, times scale * log2(e)
    // fragments of one tensor in groups of four k-steps, the next group requested before the MFMAs of the current one
    auto chain = [&](auto Uc, auto which, const bf16x8 (&kv)[KS], f32x4 acc) __attribute__((always_inline)) -> f32x4 {
      constexpr int U = decltype(Uc)::value;
      constexpr int GRP = 4, NG = KS / GRP;
      bf16x8 op[2][GRP];
      auto request = [&](int gi, bf16x8* out) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < GRP; ++q) {
          const int ks = gi * GRP + q;
          const unsigned char* b = U >= NBUF / 2 ? fr_hi[ks & 3] : fr_lo[ks & 3];
          out[q] = *reinterpret_cast<const bf16x8*>(b + (U % (NBUF / 2)) * STAGE_BYTES + decltype(which)::value * HT_BYTES +
                                                    (ks >> 2) * 256);
        }
      };
      request(0, op[0]);
#pragma unroll
      for (int gi = 0; gi < NG; ++gi) {
        if (gi + 1 < NG) request(gi + 1, op[(gi + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < GRP; ++q) acc = mfma16(op[gi & 1][q], kv[gi * GRP + q], acc);
        __builtin_amdgcn_sched_barrier(0);
      }
      return acc;
    };
    // First interval of a block (stage U): its header, S = Q K^T.  Returns 0 to go on, else the number of intervals
    // left including this one (1 or 2: the end marks are numbered).
    auto s_phase = [&](auto Uc) __attribute__((always_inline)) -> int {
      constexpr int U = decltype(Uc)::value;
      const u32x4 h = *reinterpret_cast<const u32x4*>(smem + U * STAGE_BYTES + HDR_OFF);
      flags = __builtin_amdgcn_readfirstlane((int)h.x);
      row0 = __builtin_amdgcn_readfirstlane((int)h.y);
      nvalid = __builtin_amdgcn_readfirstlane((int)h.z);
      const int ends = __builtin_amdgcn_readfirstlane((int)h.w);
      if (__builtin_expect(!(flags & HDR_VALID), 0)) return ends == 1 ? 2 : 1;
      if (__builtin_expect(flags & HDR_ACTIVE, 1)) {
        // The scores wait in registers for the next interval.  They are scaled here, in the basic block of the MFMAs:
        // what crosses the branches and the barrier is then the result of a vector ALU instruction.  (Carried as
        // they came from the matrix pipe, the compiler copied them in another block without the wait states an
        // MFMA result needs before it is read, and the copies held partial sums.)
        s = chain(Uc, IC<0>{}, kf, f32x4{0.f, 0.f, 0.f, 0.f}) * c;
      }
      return 0;
    };
    // Second interval of the block in stage U: D - dP = D + dO (-V)^T, P, -dS, published for the consumers.
    auto dp_phase = [&](auto Uc) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
      if (!(flags & HDR_VALID)) return;
      if (__builtin_expect(flags & HDR_ACTIVE, 1)) {
        const unsigned char* st = (U < NBUF / 2 ? stat_lo : stat_hi) + (U % (NBUF / 2)) * STAGE_BYTES;
        const f32x4 dinit = *reinterpret_cast<const f32x4*>(st + 64);
        const f32x4 l2 = *reinterpret_cast<const f32x4*>(st);
        const f32x4 dpv = chain(Uc, IC<1>{}, vfn, dinit);
        float pv[4], dsv[4];
        const bool masked = flags & HDR_MASK;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float e = __builtin_amdgcn_exp2f(s[r] - l2[r]);
          if (masked) {
            // rows past the end of the sequence hold copies of its last row: masked like invisible keys
            const int rl = 4 * g + r;
            bool ok = rl < nvalid;
            if (!is_ctx) ok = ok && (my_key <= row0 + rl);
            if (!ok) e = 0.f;
          }
          pv[r] = e;
          dsv[r] = e * dpv[r];   // -dS
        }
        u32x2 wp, wd;
        wp.x = pack2_bf16(pv[0], pv[1]);
        wp.y = pack2_bf16(pv[2], pv[3]);
        wd.x = pack2_bf16(dsv[0], dsv[1]);
        wd.y = pack2_bf16(dsv[2], dsv[3]);
        *reinterpret_cast<u32x2*>(xw) = wp;
        *reinterpret_cast<u32x2*>(xw + 1024) = wd;
      } else {
        // no visible (row, key) pair in this block: publish zero operands, the consumers do not branch
        const u32x2 z = {0u, 0u};
        *reinterpret_cast<u32x2*>(xw) = z;
        *reinterpret_cast<u32x2*>(xw + 1024) = z;
      }
    };

    __syncthreads();   // row block 0 and its header are in LDS
    // interval t works on stage t % 4: the wave of parity pb starts the blocks t = pb (mod 2) and finishes them in
    // the following interval.  `left` counts down the intervals after the end mark.
    int left = 0;
    auto first = [&](auto Uc) __attribute__((always_inline)) -> bool {   // interval of an S phase; false: stop
      constexpr int U = decltype(Uc)::value;
      if (left == 0) {
        left = s_phase(Uc);
        if (left == 0) request_do(IC<(U + 1) % NBUF>{});
      }
      end_interval();
      return left == 0 || --left > 0;
    };
    auto second = [&](auto Uc) __attribute__((always_inline)) -> bool {   // interval of a dP phase (block in stage U)
      constexpr int U = decltype(Uc)::value;
      if (left == 0) {
        dp_phase(Uc);
        request_do(IC<(U + 2) % NBUF>{});
      }
      end_interval();
      return left == 0 || --left > 0;
    };
    // (interval 0 requests blocks 0 and 1; `issued` stands for block 1 alone: block 0 must land in this interval)
    request_do(IC<0>{});
    issued = false;
    if (pb == 0) {
      while (true) {
        if (!first(IC<0>{})) break;
        if (!second(IC<0>{})) break;
        if (!first(IC<2>{})) break;
        if (!second(IC<2>{})) break;
      }
    } else {
      flags = 0;   // interval 0: no block to finish
      while (true) {
        if (!second(IC<3>{})) break;
        if (!first(IC<1>{})) break;
        if (!second(IC<1>{})) break;
        if (!first(IC<3>{})) break;
      }
    }
  } else {
    // ================================= consumer ==============================================
    const int jb = wave - 4;
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    // ---- global -> LDS loads: one instruction per 1 KB row; this wave takes rows jb, jb + 4, jb + 8, jb + 12 of Q and
    // of dO.  Lane l lands at chunk position l of the row and fetches the chunk that the tile swizzle stores there.
    const int G = own_sgpr(p.G);
    const int q_ts = own_sgpr((int)p.q.ts), do_ts = own_sgpr((int)p.dout.ts);
    const int64_t q_hs = own_sgpr(p.q.hs), do_hs = own_sgpr(p.dout.hs), total = own_sgpr((int64_t)p.total);
    // per-lane global offsets of this wave's load instructions for a block of 16 valid rows (a partial last
    // block clamps its rows instead: rare, computed on the spot)
    uint32_t voff_full[IPB];
#pragma unroll
    for (int t = 0; t < IPB; ++t) {
      const int row = jb + t * 4;
      voff_full[t] = (uint32_t)(row * q_ts * 2 + ((lane ^ swz<D>(row)) * 16));
    }
    const uint32_t ld_lds = smem_addr + jb * 1024;
    const float* stat_ptr = p.dvec;

    // ---- row-block schedule (Alg. 1, "Q-row blocks in causal support of K_n"): sequences of the tile, row
    // blocks of 16 that see at least one key of the tile, query heads of the group innermost.  All state is
    // wave-uniform and advanced incrementally.
    int seq = seq_lo, rb = 0, rb_end = 0, g = 0, R = 0, row_begin = 0, row0 = 0, nvalid = 0;
    const u16 *q_row = nullptr, *do_row = nullptr, *q_cur = nullptr, *do_cur = nullptr;
    int64_t st_row = 0, st_cur = 0;
    bool more = false;
    uint32_t gflags = 0;
    auto enter_group = [&]() __attribute__((always_inline)) {
      row0 = rb * HB;
      nvalid = min(HB, R - row0);
      q_cur = q_row;
      do_cur = do_row;
      st_cur = st_row;
      g = 0;
      const int k_lo = key0, k_hi = k_lo + BN - 1;
      bool a = true, m = false;
      if (!is_ctx) {
        a = k_lo <= row0 + HB - 1;
        m = k_hi > row0;
      }
      m = m || nvalid < HB;
      gflags = HDR_VALID | (a ? HDR_ACTIVE : 0) | (m ? HDR_MASK : 0);
    };
    auto init_seq = [&]() __attribute__((always_inline)) {
      // the offsets are loaded through the vector path: make their uniformity explicit
      row_begin = p.cu ? __builtin_amdgcn_readfirstlane(p.cu[seq]) : 0;
      R = p.cu ? (__builtin_amdgcn_readfirstlane(p.cu[seq + 1]) - row_begin) : p.total;
      if (is_ctx) {
        rb = 0;
        rb_end = R > 0 ? (R + HB - 1) / HB : 0;
      } else {
        rb = key0 / HB;
        rb_end = (R + HB - 1) / HB;
      }
      const int64_t grow = (int64_t)row_begin + rb * HB;
      q_row = uniform_ptr(p.q.ptr + grow * q_ts + (int64_t)hk * G * q_hs);
      do_row = uniform_ptr(p.dout.ptr + grow * do_ts + (int64_t)hk * G * do_hs);
      st_row = (int64_t)hk * G * total + grow;
    };
    auto next_group = [&]() __attribute__((always_inline)) {
      if (++rb < rb_end) {
        q_row += (int64_t)HB * q_ts;
        do_row += (int64_t)HB * do_ts;
        st_row += HB;
        enter_group();
        return;
      }
      more = false;
      while (++seq < seq_hi) {
        init_seq();
        if (rb < rb_end) {
          more = true;
          enter_group();
          return;
        }
      }
    };
    uint32_t vbits = 0;   // bit i: block (request position - 1 - i) exists
    uint32_t ends = 0;    // end marks written so far
    // requests the next block of the schedule (or marks the end) in stage IS and advances the schedule
    auto issue_block = [&](auto ISc) __attribute__((always_inline)) {
      constexpr int IS = decltype(ISc)::value;
      if (!more) ++ends;
      if (wave == 4 && lane < 2) {
        // lane 0: the block's header; lane 1: where its dO rows and row statistics are (the producers request those)
        const uint64_t dop = reinterpret_cast<uint64_t>(do_cur), stp = reinterpret_cast<uint64_t>(stat_ptr + st_cur);
        u32x4 h;
        h.x = lane == 0 ? (more ? gflags : 0u) : (uint32_t)dop;
        h.y = lane == 0 ? (uint32_t)row0 : (uint32_t)(dop >> 32);
        h.z = lane == 0 ? (uint32_t)nvalid : (uint32_t)stp;
        h.w = lane == 0 ? ends : (uint32_t)(stp >> 32);
        *reinterpret_cast<u32x4*>(smem + IS * STAGE_BYTES + HDR_OFF + lane * 16) = h;
      }
      vbits = (vbits << 1) | (more ? 1u : 0u);
      if (__builtin_expect(more, 1)) {
        const int last = nvalid - 1;   // rows past the end of the sequence re-read its last row
        const u16* q_base = uniform_ptr(q_cur);
        // (one branch for the whole block, not one per load)
        if (__builtin_expect(nvalid == HB, 1)) {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            dma16_at<IS * STAGE_BYTES + t * 4096>(q_base, voff_full[t], ld_lds);
          });
        } else {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            const int row = jb + t * 4;
            const uint32_t voff = __umul24((unsigned)min(row, last), (unsigned)(q_ts * 2)) + (uint32_t)((lane ^ swz<D>(row)) * 16);
            dma16_at<IS * STAGE_BYTES + t * 4096>(q_base, voff, ld_lds);
          });
        }
        if (__builtin_expect(++g < G, 1)) {
          q_cur += q_hs;
          do_cur += do_hs;
          st_cur += total;
        } else {
          next_group();
        }
      }
    };
    // The block requested in an interval may stay in flight at its end, the one before it must have landed (its
    // first readers start in the next interval).  If the newest request was an end mark, fewer loads are
    // outstanding: wait for all of them.
    auto wait_loads = [&]() __attribute__((always_inline)) {
      wait_vm<IPB>();
      if (__builtin_expect(!(vbits & 1u), 0)) wait_vm<0>();
    };

    for (; seq < seq_hi; ++seq) {
      init_seq();
      if (rb < rb_end) {
        more = true;
        enter_group();
        break;
      }
    }
    issue_block(IC<0>{});
    issue_block(IC<1>{});
    wait_loads();

    // Each consumer wave owns the head-dim blocks jb, jb + 4, jb + 8, jb + 12 (128 columns apart: the same
    // swizzled chunk position, 256 bytes further).
    f32x16 dk[NDB], dv[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dk[db][r] = 0.f;
        dv[db][r] = 0.f;
      }
    const unsigned char* tr0_lo = smem + tr_off<D>(lane, hi * 4, jb * 32);
    const unsigned char* tr1_lo = smem + tr_off<D>(lane, hi * 4 + 8, jb * 32);
    const unsigned char* tr0_hi = tr0_lo + HALF;
    const unsigned char* tr1_hi = tr1_lo + HALF;
    const unsigned char* xr_lane = smem + XCH_OFF + lane * 16;
    bf16x8 tq[NDB], tdo[NDB];   // Q^T, dO^T operands of the row block accumulated next interval

    // interval t (stage U = t % 4 holds block t): requests block t + 2, accumulates block t - 2, reads the
    // transposed operands of block t - 1; returns false after the last interval
    auto interval = [&](auto Uc) __attribute__((always_inline)) -> bool {
      constexpr int U = decltype(Uc)::value, IS = (U + 2) % NBUF, UP = (U + NBUF - 1) % NBUF, XB = U & 1;
      issue_block(IC<IS>{});
      if (vbits & (1u << 4)) {
        const unsigned char* xr = xr_lane + XB * XCH_BYTES;   // block t - 2 has the parity of t
        const bf16x8 pa = *reinterpret_cast<const bf16x8*>(xr);
        const bf16x8 dsa = *reinterpret_cast<const bf16x8*>(xr + 1024);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          dv[db] = mfma32(pa, tdo[db], dv[db]);
          dk[db] = mfma32(dsa, tq[db], dk[db]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      const bool prev = vbits & (1u << 3);
      if (__builtin_expect(prev, 1)) {
        const unsigned char* t0 = (UP < NBUF / 2 ? tr0_lo : tr0_hi) + (UP % (NBUF / 2)) * STAGE_BYTES;
        const unsigned char* t1 = (UP < NBUF / 2 ? tr1_lo : tr1_hi) + (UP % (NBUF / 2)) * STAGE_BYTES;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          tdo[db] = tr_pair(t0 + HT_BYTES + db * 256, t1 + HT_BYTES + db * 256);
          tq[db] = tr_pair(t0 + db * 256, t1 + db * 256);
        }
      }
      wait_loads();
      __syncthreads();
      return prev;
    };

    __syncthreads();   // row block 0 and its header are in LDS
    {
      // interval 0 always runs, interval t > 0 runs if block t - 1 exists: NB + 2 intervals for NB blocks
      bool go = true;
      interval(IC<0>{});
      while (go) {
        if (!interval(IC<1>{})) break;
        if (!interval(IC<2>{})) break;
        if (!interval(IC<3>{})) break;
        go = interval(IC<0>{});
      }
    }

    // ---- epilogue: C layout -> lane owns head-dim column, register r owns key crow(r); the dK
    // accumulator holds -dK / scale
    const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
    float* acc_k = is_ctx ? p.dkc_acc : p.dkd_acc;
    float* acc_v = is_ctx ? p.dvc_acc : p.dvd_acc;
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const int dcol = (jb + 4 * db) * 32 + l32;
      const f32x16 gks = dk[db], gvs = dv[db];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + crow(r, hi);
        if (key >= region_len) continue;
        const float gk = -gks[r] * p.scale, gv = gvs[r];
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
}

}  // namespace

hipError_t launch_dkdv512(const AttnParams& p0, hipStream_t st) {
  AttnParams p = p0;
  p.n_ctx_tiles = (p.ctx_len + BN - 1) / BN;
  p.n_dec_tiles = (p.max_rows + BN - 1) / BN;
  if (p.n_split < 1) p.n_split = 1;
  // the kernel addresses LSE*log2e as D + 32-bit unsigned byte offset
  if (reinterpret_cast<uintptr_t>(p.lse2) < reinterpret_cast<uintptr_t>(p.dvec) ||
      reinterpret_cast<uintptr_t>(p.lse2) - reinterpret_cast<uintptr_t>(p.dvec) >= (1ull << 32))
    return hipErrorInvalidValue;
  hipError_t e = ensure_dynamic_lds<dkdv512_kernel>(SMEM_BYTES);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)(p.grp ? p.n_groups : 1) * p.n_ctx_tiles * p.Hk * p.n_split +
                       (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(dkdv512_kernel, dim3((unsigned)nblk), dim3(512), SMEM_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace dkv
