// dK / dV kernel for head dims 64 and 128 with producer / consumer wave specialisation (same mathematics
// and the same ownership rule as the other dK/dV kernels: one workgroup owns a 128-key tile of one KV
// head; a shared-prompt tile sums the contributions of ALL sequences and heads of the group in fp32
// registers and is cast once -- Alg. 1 with the race of the shared prompt gradients removed by ownership).
//
// Measured on gfx950 with two waves per SIMD: a wave issues about one instruction every 4-5 cycles, a taken
// branch costs ~25 cycles, a VGPR -> SGPR round trip ~35, an LDS round trip ~130.  At 32 query rows per
// step the MFMA work of a SIMD is only ~1050 cycles, so the kernel is bound by the instruction stream of
// its busiest wave unless control flow, address arithmetic and waiting are kept out of it.  Hence:
//   * two roles share each SIMD.  A producer wave (0-3, one per 32-key subtile) keeps K and -V fragments in
//     registers and computes S = Q K^T, D - dP = D + dO (-V)^T (accumulator initialised to D),
//     P = exp2(S*scale*log2e - LSE*log2e) and -dS = P * (D - dP), publishing P and -dS as bf16 MFMA
//     operands in LDS.  A consumer wave (4-7) owns one 32-wide head-dim block of dK, dV for all 128 keys
//     and, one row block behind, accumulates dV += P^T dO and -dK += (-dS)^T Q with dO^T / Q^T from LDS
//     transpose reads.  The producers' exponentials overlap the consumers' MFMAs.
//   * the consumers also walk the row-block schedule (a few scalar operations per block) and issue the
//     global -> LDS loads (global_load_lds: Q, dO, LSE*log2e, D never pass through registers) five row
//     blocks ahead; wave 4 leaves a 16-byte header per key subtile in the stage (valid / active / mask flags,
//     first row, row count), which is all a producer needs to know about the schedule.
//   * the main loop is unrolled over the six LDS stages, so every LDS address is an immediate offset;
//     every LDS operand is read one interval before its use, across the single barrier per row block.
//
// The compiler does not know about the global -> LDS loads: the consumers count them themselves
// (s_waitcnt vmcnt) before the barrier that publishes a row block, and no compiler-visible vector memory
// load is issued inside the main loop (a compiler-placed wait would also wait for all blocks in flight).
#include <type_traits>
#include "common.h"
#include "dma.h"
#include "kvsched.h"
#include "launch.h"
#include "tiles.h"

namespace dkv {

enum : int { HDR_VALID = 1, HDR_ACTIVE = 2, HDR_MASK = 4 };
template <int V>
using IC = std::integral_constant<int, V>;

template <int D, bool LOCAL>
__global__ __launch_bounds__(512) void dkdv4_kernel(const AttnParams p) {
  constexpr int BN = 128, HB = 32;                 // keys per workgroup, query rows per block
  constexpr int KS = D / 16, DSUB = D / 32, RB = 2 * D, CPR = D / 8;
  constexpr int HT_BYTES = HB * RB;                // one Q or dO row block
  constexpr int STAT_OFF = 2 * HT_BYTES;           // lse2[32] | D[32]
  constexpr int HDR_OFF = STAT_OFF + 256;          // 4 x {flags, row0, nvalid, -}
  constexpr int STAGE_BYTES = HDR_OFF + 64;
  constexpr int NBUF = 6, AHEAD = NBUF - 1;        // row blocks requested ahead of the one being computed
  constexpr int XCH_OFF = NBUF * STAGE_BYTES;
  constexpr int XCH_BYTES = 16384;                 // [key subtile][P k-step 0,1 | dS k-step 0,1][lane] x 16 B
  constexpr int NIT = HT_BYTES / 1024;             // 1 KB load instructions per row block and tensor
  constexpr int IPB = 2 * NIT / 4;                 // per consumer wave (Q and dO)
  constexpr int RPI = 1024 / RB;                   // rows per load instruction
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int kvs = wave & 3;
  const int W = p.window;

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
    const float c = p.scale_log2;
    const int my_key = key0 + kvs * 32 + l32;
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
      const u16* kp = kbase + (int64_t)kr * kts + hi * 8;
      const u16* vp = vbase + (int64_t)kr * vts + hi * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
        u32x4 v = *reinterpret_cast<const u32x4*>(vp + ks * 16);
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
    // LDS addresses: two base registers per operand (stages 0-2 and 3-5) so that every access of the
    // unrolled loop is base + immediate offset (the offset field has 16 bits)
    constexpr int HALF = (NBUF / 2) * STAGE_BYTES;
    const unsigned char* frag_lo[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) frag_lo[ks] = smem + tile_off<D>(l32, 2 * ks + hi);
    const unsigned char* frag_hi[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) frag_hi[ks] = frag_lo[ks] + HALF;
    const unsigned char* stat_lo = smem + STAT_OFF + hi * 16;   // this lane's rows 8*(r/4) + 4*hi + r%4
    const unsigned char* stat_hi = stat_lo + HALF;
    const unsigned char* hdr_lo = smem + HDR_OFF + kvs * 16;
    const unsigned char* hdr_hi = hdr_lo + HALF;
    unsigned char* xw_lane = smem + XCH_OFF + kvs * 4096 + lane * 16;

    bf16x8 qfr[KS];
    int flags, row0, nvalid;
    auto read_header = [&](auto Uc, u32x4& h) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
      h = *reinterpret_cast<const u32x4*>((U < NBUF / 2 ? hdr_lo : hdr_hi) + (U % (NBUF / 2)) * STAGE_BYTES);
    };
    // which = 0: Q fragments (read one interval early), 1: dO fragments (read at the start of their interval,
    // behind the S chain: keeping both sets across the barrier does not fit next to the K / V fragments)
    auto load_frags = [&](auto Uc, auto which, bf16x8* out) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const unsigned char* b = U >= NBUF / 2 ? frag_hi[ks] : frag_lo[ks];
        out[ks] = *reinterpret_cast<const bf16x8*>(b + (U % (NBUF / 2)) * STAGE_BYTES + decltype(which)::value * HT_BYTES);
      }
    };
    // row statistics of this lane's 16 rows (register r <-> row crow(r, hi)): which = 0 LSE*log2e, 1 D
    auto load_stat = [&](auto Uc, int which, float* out) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
      const unsigned char* b = (U < NBUF / 2 ? stat_lo : stat_hi) + (U % (NBUF / 2)) * STAGE_BYTES + which * 128;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(b + r4 * 32);
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) out[r4 * 4 + e4] = v[e4];
      }
    };

    // one interval: block h in stage U; returns false after the end of the schedule
    auto interval = [&](auto Uc) __attribute__((always_inline)) -> bool {
      constexpr int U = decltype(Uc)::value, NU = (U + 1) % NBUF, XB = U & 1;
      if (__builtin_expect(!(flags & HDR_VALID), 0)) {
        __syncthreads();
        return false;
      }
      u32x4 hn;
      read_header(IC<NU>{}, hn);
      const bool act = flags & HDR_ACTIVE;
      f32x16 s, dpv;
      float l2[16];
      if (__builtin_expect(act, 1)) {
        float dinit[16];
        bf16x8 dofr[KS];
        load_stat(Uc, 1, dinit);   // their latency hides behind the S chain
        load_frags(Uc, IC<1>{}, dofr);
        __builtin_amdgcn_sched_barrier(0);   // all reads requested before the first MFMA, not trickled in between
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s = mfma32(qfr[ks], kf[ks], s);
#pragma unroll
        for (int r = 0; r < 16; ++r) dpv[r] = dinit[r];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dpv = mfma32(dofr[ks], vfn[ks], dpv);   // D - dP
        load_stat(Uc, 0, l2);
      }
      // keep the operand reads of block h+1 behind the MFMAs of block h: issued earlier they would need a
      // second set of 64 fragment registers and push the K / V fragments out of the register file
      __builtin_amdgcn_sched_barrier(0);
      const int nflags = __builtin_amdgcn_readfirstlane((int)hn.x);
      const int nrow0 = __builtin_amdgcn_readfirstlane((int)hn.y);
      const int nnvalid = __builtin_amdgcn_readfirstlane((int)hn.z);
      // unconditional: a load that depends on the next header would make the compiler keep the old fragments in
      // a second register set (sixteen moves per block); an inactive or invalid block's fragments are never used
      load_frags(IC<NU>{}, IC<0>{}, qfr);
      __builtin_amdgcn_sched_barrier(0);
      unsigned char* xw = xw_lane + XB * XCH_BYTES;
      if (__builtin_expect(act, 1)) {
        float pv[16], dsv[16];
        auto softmax_part = [&](auto masked) __attribute__((always_inline)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float e = __builtin_amdgcn_exp2f(s[r] * c - l2[r]);
            if (decltype(masked)::value) {
              // rows past the end of the sequence hold copies of its last row: masked like invisible keys
              const int rl = crow(r, hi), rw = row0 + rl;
              bool ok = rl < nvalid;
              if (is_ctx) ok = ok && (!LOCAL || (my_key > P + rw - W));
              else ok = ok && (my_key <= rw) && (!LOCAL || (my_key > rw - W));
              if (!ok) e = 0.f;
            }
            pv[r] = e;
            dsv[r] = e * dpv[r];   // -dS
          }
        };
        if (__builtin_expect(flags & HDR_MASK, 0)) softmax_part(std::true_type{});
        else softmax_part(std::false_type{});
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          *reinterpret_cast<bf16x8*>(xw + t2 * 1024) = pack8_bf16(pv + t2 * 8);
          *reinterpret_cast<bf16x8*>(xw + (2 + t2) * 1024) = pack8_bf16(dsv + t2 * 8);
        }
      } else {
        // no visible (row, key) pair in this block: publish zero operands, the consumers do not branch
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < 4; ++t) *reinterpret_cast<u32x4*>(xw + t * 1024) = z;
      }
      __syncthreads();
      flags = nflags;
      row0 = nrow0;
      nvalid = nnvalid;
      return true;
    };

    __syncthreads();   // row blocks 0 and 1 and their headers are in LDS
    {
      u32x4 h0;
      read_header(IC<0>{}, h0);
      flags = __builtin_amdgcn_readfirstlane((int)h0.x);
      row0 = __builtin_amdgcn_readfirstlane((int)h0.y);
      nvalid = __builtin_amdgcn_readfirstlane((int)h0.z);
    }
    if (flags & HDR_ACTIVE) load_frags(IC<0>{}, IC<0>{}, qfr);
    while (true) {
      if (!interval(IC<0>{})) break;
      if (!interval(IC<1>{})) break;
      if (!interval(IC<2>{})) break;
      if (!interval(IC<3>{})) break;
      if (!interval(IC<4>{})) break;
      if (!interval(IC<5>{})) break;
    }
  } else {
    // ================================= consumer ==============================================
    const int jb = wave - 4;
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    // ---- global -> LDS loads: instruction i = jb + 4 t of a row block covers RPI rows of Q (t < IPB/2) or
    // dO; lane l lands at LDS chunk position l % CPR of row (l / CPR) of the instruction, so it fetches the
    // chunk that the tile swizzle stores there (the swizzle has period 4 RPI rows: one offset serves all t).
    const int G = own_sgpr(p.G);
    const int q_ts = own_sgpr((int)p.q.ts), do_ts = own_sgpr((int)p.dout.ts);
    const int64_t q_hs = own_sgpr(p.q.hs), do_hs = own_sgpr(p.dout.hs), total = own_sgpr((int64_t)p.total);
    const int ld_row0 = jb * RPI + lane / CPR;
    const int ld_coff = ((lane % CPR) ^ swz<D>(ld_row0)) * 16;
    const uint32_t ld_lds = smem_addr + jb * 1024;
    // per-lane global offsets of this wave's load instructions for a block of 32 valid rows (a partial last
    // block clamps its rows instead: rare, computed on the spot)
    uint32_t voff_full[IPB];
#pragma unroll
    for (int t = 0; t < IPB; ++t)
      voff_full[t] = LOCAL ? 0u : (uint32_t)((ld_row0 + (t % (IPB / 2)) * 4 * RPI) * (t < IPB / 2 ? q_ts : do_ts) * 2 + ld_coff);
    // row statistics: lanes 0-31 fetch LSE*log2e, lanes 32-63 fetch D; both arrays live in one workspace, D
    // first and LSE*log2e less than 4 GB behind it (checked by the launcher), so one scalar base plus an
    // unsigned 32-bit lane offset addresses both
    const float* stat_ptr = p.dvec;
    const uint32_t stat_lane_off = hi ? 0u : (uint32_t)((const char*)p.lse2 - (const char*)p.dvec);

    // ---- row-block schedule (Alg. 1, "Q-row blocks in causal support of K_n"): sequences of the tile, row
    // blocks of 32 that see at least one key of the tile, query heads of the group innermost.  All state is
    // wave-uniform and advanced incrementally.
    int seq = seq_lo, rb = 0, rb_end = 0, g = 0, R = 0, row_begin = 0, row0 = 0, nvalid = 0;
    const u16 *q_row = nullptr, *do_row = nullptr, *q_cur = nullptr, *do_cur = nullptr;
    int64_t st_row = 0, st_cur = 0;
    bool more = false;
    uint32_t gflags = 0;   // wave 4, lanes 0-3: flags of key subtile `lane` for the current row group
    auto enter_group = [&]() __attribute__((always_inline)) {
      row0 = rb * HB;
      nvalid = min(HB, R - row0);
      q_cur = q_row;
      do_cur = do_row;
      st_cur = st_row;
      g = 0;
      if (wave == 4) {
        const int k_lo = key0 + (lane & 3) * 32, k_hi = k_lo + 31;
        bool a, m;
        if (is_ctx) {
          a = !LOCAL || (k_hi > P + row0 - W);
          m = LOCAL && (k_lo <= P + row0 + 31 - W);
        } else {
          a = k_lo <= row0 + 31;
          m = k_hi > row0;
          if (LOCAL) {
            a = a && (k_hi > row0 - W);
            m = m || (k_lo <= row0 + 31 - W);
          }
        }
        m = m || nvalid < HB;
        gflags = HDR_VALID | (a ? HDR_ACTIVE : 0) | (m ? HDR_MASK : 0);
      }
    };
    auto init_seq = [&]() __attribute__((always_inline)) {
      // the offsets are loaded through the vector path: make their uniformity explicit
      row_begin = p.cu ? __builtin_amdgcn_readfirstlane(p.cu[seq]) : 0;
      R = p.cu ? (__builtin_amdgcn_readfirstlane(p.cu[seq + 1]) - row_begin) : p.total;
      int rows = R;
      if (is_ctx) {
        const int key_hi = min(P, key0 + BN) - 1;
        if (LOCAL) rows = min(R, key_hi + W - P);
        rb = 0;
        rb_end = rows > 0 ? (rows + HB - 1) / HB : 0;
      } else {
        const int key_hi = min(R, key0 + BN) - 1;
        if (LOCAL) rows = min(R, key_hi + W);
        rb = key0 / HB;
        rb_end = (rows + HB - 1) / HB;
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
    // requests the next block of the schedule (or marks the end) in stage IS and advances the schedule
    auto issue_block = [&](auto ISc) __attribute__((always_inline)) {
      constexpr int IS = decltype(ISc)::value;
      if (wave == 4 && lane < 4) {
        u32x4 h;
        h.x = more ? gflags : 0u;
        h.y = (uint32_t)row0;
        h.z = (uint32_t)nvalid;
        h.w = 0u;
        *reinterpret_cast<u32x4*>(smem + IS * STAGE_BYTES + HDR_OFF + lane * 16) = h;
      }
      vbits = (vbits << 1) | (more ? 1u : 0u);
      if (__builtin_expect(more, 1)) {
        const int last = nvalid - 1;   // rows past the end of the sequence re-read its last row
        const u16* q_base = uniform_ptr(q_cur);
        const u16* do_base = uniform_ptr(do_cur);
        // (one branch for the whole block, not one per load)
        if (__builtin_expect(!LOCAL && nvalid == HB, 1)) {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            dma16_at<IS * STAGE_BYTES + (t < IPB / 2 ? 0 : HT_BYTES) + (t % (IPB / 2)) * 4096>(
                t < IPB / 2 ? q_base : do_base, voff_full[t], ld_lds);
          });
        } else {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            constexpr bool is_q = t < IPB / 2;
            const int row = ld_row0 + (t % (IPB / 2)) * 4 * RPI;
            const uint32_t voff = __umul24((unsigned)min(row, last), (unsigned)((is_q ? q_ts : do_ts) * 2)) + ld_coff;
            dma16_at<IS * STAGE_BYTES + (is_q ? 0 : HT_BYTES) + (t % (IPB / 2)) * 4096>(is_q ? q_base : do_base, voff, ld_lds);
          });
        }
        if (wave == 5) {
          dma4_at<IS * STAGE_BYTES + STAT_OFF>(uniform_ptr(reinterpret_cast<const u16*>(stat_ptr + st_cur)),
                                               stat_lane_off + (uint32_t)min(l32, last) * 4u, smem_addr);
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
    // Block b is requested AHEAD blocks early and must have landed by the end of interval b - 2 (the
    // producer reads its operands one interval early): the three youngest blocks (IPB loads each per
    // wave; wave 5 issues one more, for it the bound is a little stricter) may stay in flight.  If the
    // newest request was the end mark, fewer loads are outstanding: wait for all of them.
    auto wait_loads = [&]() __attribute__((always_inline)) {
      wait_vm<(AHEAD - 2) * IPB>();
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
    issue_block(IC<2>{});
    issue_block(IC<3>{});
    issue_block(IC<4>{});
    wait_loads();

    // Each consumer wave owns one 32-wide head-dim block (dblk) of the gradients of NK key subtiles: the
    // transposed Q / dO operands of its head-dim block are shared by all its key subtiles, which keeps the
    // (slow) LDS transpose reads at 8 per row block.
    constexpr int NK = DSUB;                       // key subtiles per wave: 4 (d = 128) or 2 (d = 64)
    const int dblk = jb % DSUB, k0 = (jb / DSUB) * NK;
    f32x16 dk[NK], dv[NK];
#pragma unroll
    for (int i = 0; i < NK; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dk[i][r] = 0.f;
        dv[i][r] = 0.f;
      }
    const unsigned char* tr0 = smem + tr_off<D>(lane, hi * 4, dblk * 32);
    const unsigned char* tr1 = smem + tr_off<D>(lane, hi * 4 + 8, dblk * 32);
    const unsigned char* xr_lane = smem + XCH_OFF + k0 * 4096 + lane * 16;
    bf16x8 tq[2], tdo[2];   // Q^T, dO^T operands of the row block accumulated next interval

    // one interval: accumulates block h-1, reads the transposed operands of block h (stage U), requests
    // block h + AHEAD; returns false after the end of the schedule
    auto interval = [&](auto Uc) __attribute__((always_inline)) -> bool {
      constexpr int U = decltype(Uc)::value, IS = (U + AHEAD) % NBUF, XB = (U + 1) & 1;
      // requests first: the producers' MFMAs run meanwhile, the consumers' follow them
      issue_block(IC<IS>{});
      if (vbits & (1u << (AHEAD + 1))) {
        const unsigned char* xr = xr_lane + XB * XCH_BYTES;
        // all P / -dS operands are requested before the first MFMA (left alone, the compiler reads one operand,
        // waits for it and issues one MFMA, sixteen LDS latencies in a row)
        bf16x8 pa[2][NK], dsa[2][NK];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int i = 0; i < NK; ++i) {
            pa[t2][i] = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + t2 * 1024);
            dsa[t2][i] = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + (2 + t2) * 1024);
          }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int i = 0; i < NK; ++i) {
            dv[i] = mfma32(pa[t2][i], tdo[t2], dv[i]);
            dk[i] = mfma32(dsa[t2][i], tq[t2], dk[i]);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
      const bool cur = vbits & (1u << AHEAD);
      if (__builtin_expect(cur, 1)) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          tdo[t2] = tr_pair(tr0 + U * STAGE_BYTES + HT_BYTES + t2 * 16 * RB, tr1 + U * STAGE_BYTES + HT_BYTES + t2 * 16 * RB);
          tq[t2] = tr_pair(tr0 + U * STAGE_BYTES + t2 * 16 * RB, tr1 + U * STAGE_BYTES + t2 * 16 * RB);
        }
      }
      wait_loads();
      __syncthreads();
      return cur;
    };

    __syncthreads();   // row blocks 0 and 1 and their headers are in LDS
    while (true) {
      if (!interval(IC<0>{})) break;
      if (!interval(IC<1>{})) break;
      if (!interval(IC<2>{})) break;
      if (!interval(IC<3>{})) break;
      if (!interval(IC<4>{})) break;
      if (!interval(IC<5>{})) break;
    }

    // ---- epilogue: C layout -> lane owns head-dim column, register r owns key crow(r); the dK
    // accumulator holds -dK / scale
    const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
    float* acc_k = is_ctx ? p.dkc_acc : p.dkd_acc;
    float* acc_v = is_ctx ? p.dvc_acc : p.dvd_acc;
    const int dcol = dblk * 32 + l32;
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      const f32x16 gks = dk[i], gvs = dv[i];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + (k0 + i) * 32 + crow(r, hi);
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

template <int D, bool LOCAL>
static hipError_t launch_dkdv4_t(AttnParams p, hipStream_t st) {
  constexpr int BN = 128;
  p.n_ctx_tiles = (p.ctx_len + BN - 1) / BN;
  p.n_dec_tiles = (p.max_rows + BN - 1) / BN;
  if (p.n_split < 1) p.n_split = 1;
  // the kernel addresses LSE*log2e as D + 32-bit unsigned byte offset
  if (reinterpret_cast<uintptr_t>(p.lse2) < reinterpret_cast<uintptr_t>(p.dvec) ||
      reinterpret_cast<uintptr_t>(p.lse2) - reinterpret_cast<uintptr_t>(p.dvec) >= (1ull << 32))
    return hipErrorInvalidValue;
  const size_t smem = 6 * (2 * 32 * 2 * D + 256 + 64) + 2 * 16384;
  auto kern = dkdv4_kernel<D, LOCAL>;
  hipError_t e = ensure_dynamic_lds<dkdv4_kernel<D, LOCAL>>(smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)(p.grp ? p.n_groups : 1) * p.n_ctx_tiles * p.Hk * p.n_split +
                       (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(512), smem, st, p);
  return hipGetLastError();
}

hipError_t launch_dkdv4(const AttnParams& p, int head_dim, hipStream_t st) {
  const bool local = p.window > 0;
  switch (head_dim) {
    case 64:  return local ? launch_dkdv4_t<64, true>(p, st) : launch_dkdv4_t<64, false>(p, st);
    case 128: return local ? launch_dkdv4_t<128, true>(p, st) : launch_dkdv4_t<128, false>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
