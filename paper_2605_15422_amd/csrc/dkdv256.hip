// dK / dV kernel for head dim 256 with producer / consumer wave specialisation (the mathematics, the
// ownership rule and the row-block schedule of the head-dim 64 / 128 kernel: one workgroup owns a key tile of
// one KV head; a shared-prompt tile sums the contributions of ALL sequences and heads of the group in fp32
// registers and is cast once -- Alg. 1 with the race of the shared prompt gradients removed by ownership).
//
// What the wider head changes.  The fp32 dK and dV of one key fill 2 KB, and the four consumer waves can give
// 128 of their 256 registers to accumulators: the key tile is 64 keys (two 32-key subtiles), each consumer wave
// owning two of the eight 32-wide head-dim blocks of both subtiles.  A producer that kept the K and V
// fragments of a 32-key subtile (128 registers) next to the Q and dO fragments of 32 rows (128 more) would not
// fit either, so the four producers split the 32-row block by ROW HALVES: producer (subtile k, half h) forms
// S, D - dP, P and dS of 16 rows x 32 keys with the 16x16x32 MFMA (two 16-key accumulators of four registers
// each), entirely in its own registers and in fp32, as the narrower kernel does.  The MFMA work of a row block
// is then spread evenly: 16 MFMA-equivalents per wave, one producer and one consumer per SIMD.
//
//   * producers (waves 0-3): K and -V fragments in registers; Q fragments are read one interval early, dO
//     fragments at the start of their interval; P and -dS leave as bf16 MFMA operands through a double-buffered
//     exchange area, laid out exactly as the consumers' 32x32x16 A operands expect them;
//   * consumers (waves 4-7): one row block behind, dV += P^T dO and -dK += (-dS)^T Q with dO^T / Q^T from LDS
//     transpose reads; they walk the schedule, issue the global -> LDS loads (Q, dO, LSE*log2e, D) three row
//     blocks ahead into four stages of 32 rows and leave a 16-byte header per key subtile and stage;
//   * the main loop is unrolled over the four stages (immediate LDS offsets), one barrier per row block.
// LDS: 4 x (16 KB Q + 16 KB dO + statistics + headers) + 2 x 8 KB exchange = 145 KB.
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

constexpr int D = 256;
constexpr int BN = 64, HB = 32, NKS = BN / 32;   // keys per workgroup, query rows per block, key subtiles
static_assert(NKS == 2, "the header store selects between two subtiles");
constexpr int KS = D / 32;                       // k-steps of the 16x16x32 MFMA
constexpr int RB = 2 * D, CPR = D / 8;
constexpr int HT_BYTES = HB * RB;                // one Q or dO row block
constexpr int STAT_OFF = 2 * HT_BYTES;           // lse2[32] | D[32]
constexpr int HDR_OFF = STAT_OFF + 256;          // NKS x {flags, row0, nvalid, -}
constexpr int STAGE_BYTES = HDR_OFF + 64;
constexpr int NBUF = 4, AHEAD = NBUF - 1;        // row blocks requested ahead of the one being computed
constexpr int XCH_OFF = NBUF * STAGE_BYTES;
constexpr int XCH_BYTES = NKS * 4096;            // [key subtile][P k-step 0,1 | dS k-step 0,1][lane] x 16 B
constexpr int SMEM_BYTES = XCH_OFF + 2 * XCH_BYTES;
constexpr int NIT = HT_BYTES / 1024;             // 1 KB load instructions per row block and tensor
constexpr int IPB = 2 * NIT / 4;                 // per consumer wave (Q and dO)
constexpr int RPI = 1024 / RB;                   // rows per load instruction
constexpr int HALF = (NBUF / 2) * STAGE_BYTES;   // second base register of every LDS operand (16-bit offset field)
static_assert(NBUF % 2 == 0 && STAGE_BYTES + HT_BYTES + 16 * RB + 512 < 65536, "immediate offsets");

template <bool LOCAL>
__global__ __launch_bounds__(512) void dkdv256_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
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

  if (LOCAL && is_ctx && min(P, key0 + BN) - 1 + W - P <= 0) {
    // With a window only the last W prompt keys are visible to response rows: the other prompt tiles (most of them)
    // have no row block at all.  Their gradient is zero: nothing to add to fp32 accumulators, zeros to write otherwise.
    if (p.dkc_acc == nullptr) {
      const int nkeys = min(P, key0 + BN) - key0;
      for (int i = tid; i < nkeys * D; i += 512) {
        const int key = key0 + i / D, col = i % D;
        p.dkc.ptr[(int64_t)(key_row_begin + key) * p.dkc.ts + (int64_t)hk * p.dkc.hs + col] = 0;
        p.dvc.ptr[(int64_t)(key_row_begin + key) * p.dvc.ts + (int64_t)hk * p.dvc.hs + col] = 0;
      }
    }
    return;
  }

  if (wave < 4) {
    // ================================= producer ==============================================
    // 16x16x32 operands: lane = (l16, g): A row / B column l16, contraction indices 8 g .. 8 g + 7 of the k-step;
    // accumulator: column l16, register r <-> row 4 g + r.
    const int kvs = wave & 1, rh = wave >> 1;
    const int l16 = lane & 15, g = lane >> 4;
    // Which eight contraction indices of a k-step lane group g supplies is free as long as both operands agree:
    // group g takes chunk cg = (0, 3, 1, 2)[g] of the 64-byte k-step.  A 16-byte LDS read is served in groups of
    // sixteen lanes that are not contiguous (lanes 0-3, 12-15, 20-23, 24-27 form the first one); with cg = g the
    // fragment reads below collide two ways in every group, with this assignment they do not.
    const int cg = (0x9C >> (2 * g)) & 3;
    const float c = p.scale_log2;
    const int my_key[2] = {key0 + kvs * 32 + l16, key0 + kvs * 32 + 16 + l16};
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
    bf16x8 kf[KS][2], vfn[KS][2];   // K and -V (sign bits flipped: exact) of the two 16-key halves
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kr = min(my_key[h], region_len - 1);   // clamp: gradients of padded keys are never stored
      const u16* kp = kbase + (int64_t)kr * kts + cg * 8;
      const u16* vp = vbase + (int64_t)kr * vts + cg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[ks][h] = *reinterpret_cast<const bf16x8*>(kp + ks * 32);
        u32x4 v = *reinterpret_cast<const u32x4*>(vp + ks * 32);
        v.x ^= 0x80008000u;
        v.y ^= 0x80008000u;
        v.z ^= 0x80008000u;
        v.w ^= 0x80008000u;
        vfn[ks][h] = __builtin_bit_cast(bf16x8, v);
      }
    }
    // the loads are consumed (and therefore waited for) here, before the main loop
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      asm volatile("" : : "v"(kf[ks][0]), "v"(kf[ks][1]), "v"(vfn[ks][0]), "v"(vfn[ks][1]));

    // Q / dO fragment of k-step ks: row rh*16 + l16, chunk 4 ks + cg.  With the tile swizzle (low two row bits
    // into chunk bits 2-3, row bits 2-3 into chunk bits 0-1) the chunk position is
    // 4 ((ks % 4) ^ (row % 4)) + (cg ^ (row / 4 % 4)) + 16 (ks / 4): four base registers serve all eight k-steps.
    const int frow = rh * 16 + l16;
    const unsigned char* fr_lo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) fr_lo[j] = smem + frow * RB + 64 * (j ^ (frow & 3)) + 16 * (cg ^ ((frow >> 2) & 3));
    const unsigned char* fr_hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) fr_hi[j] = fr_lo[j] + HALF;
    const unsigned char* stat_lo = smem + STAT_OFF + (rh * 16 + 4 * g) * 4;   // this lane's rows rh*16 + 4 g + r
    const unsigned char* stat_hi = stat_lo + HALF;
    const unsigned char* hdr_lo = smem + HDR_OFF + kvs * 16;
    const unsigned char* hdr_hi = hdr_lo + HALF;
    // consumer A operand (32x32x16): lane (key, hi'), element e <-> row 4 hi' + 8 (e / 4) + e % 4 of the k-step.
    // This lane holds rows 4 g + r of k-step rh: hi' = g % 2, elements 4 (g / 2) .. + 3.
    unsigned char* xw_lane = smem + XCH_OFF + kvs * 4096 + rh * 1024 + ((g & 1) * 32 + l16) * 16 + (g >> 1) * 8;

    bf16x8 qfr[KS];
    int flags, row0, nvalid;
    auto read_header = [&](auto Uc, u32x4& h) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
      h = *reinterpret_cast<const u32x4*>((U < NBUF / 2 ? hdr_lo : hdr_hi) + (U % (NBUF / 2)) * STAGE_BYTES);
    };
    // which = 0: Q fragments (read one interval early), 1: dO fragments (read at the start of their interval)
    auto load_frags = [&](auto Uc, auto which, bf16x8* out) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const unsigned char* b = U >= NBUF / 2 ? fr_hi[ks & 3] : fr_lo[ks & 3];
        out[ks] = *reinterpret_cast<const bf16x8*>(b + (U % (NBUF / 2)) * STAGE_BYTES + decltype(which)::value * HT_BYTES +
                                                   (ks >> 2) * 256);
      }
    };
    auto load_stat = [&](auto Uc, int which) __attribute__((always_inline)) {
      constexpr int U = decltype(Uc)::value;
      return *reinterpret_cast<const f32x4*>((U < NBUF / 2 ? stat_lo : stat_hi) + (U % (NBUF / 2)) * STAGE_BYTES + which * 128);
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
      f32x4 s[2], dpv[2], l2;
      if (__builtin_expect(act, 1)) {
        bf16x8 dofr[KS];
        const f32x4 dinit = load_stat(Uc, 1);   // its latency hides behind the S chain
        load_frags(Uc, IC<1>{}, dofr);
        __builtin_amdgcn_sched_barrier(0);   // all reads requested before the first MFMA
        s[0] = f32x4{0.f, 0.f, 0.f, 0.f};
        s[1] = s[0];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          s[0] = mfma16(qfr[ks], kf[ks][0], s[0]);
          s[1] = mfma16(qfr[ks], kf[ks][1], s[1]);
        }
        dpv[0] = dinit;
        dpv[1] = dinit;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          dpv[0] = mfma16(dofr[ks], vfn[ks][0], dpv[0]);   // D - dP
          dpv[1] = mfma16(dofr[ks], vfn[ks][1], dpv[1]);
        }
        l2 = load_stat(Uc, 0);
      }
      // the operand reads of block h+1 stay behind the MFMAs of block h (a second set of fragment registers
      // would push the K / V fragments out of the register file)
      __builtin_amdgcn_sched_barrier(0);
      const int nflags = __builtin_amdgcn_readfirstlane((int)hn.x);
      const int nrow0 = __builtin_amdgcn_readfirstlane((int)hn.y);
      const int nnvalid = __builtin_amdgcn_readfirstlane((int)hn.z);
      // unconditional (an inactive or invalid block's fragments are never used)
      load_frags(IC<NU>{}, IC<0>{}, qfr);
      __builtin_amdgcn_sched_barrier(0);
      unsigned char* xw = xw_lane + XB * XCH_BYTES;
      if (__builtin_expect(act, 1)) {
        float pv[2][4], dsv[2][4];
        auto softmax_part = [&](auto masked) __attribute__((always_inline)) {
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float e = __builtin_amdgcn_exp2f(s[h][r] * c - l2[r]);
              if (decltype(masked)::value) {
                // rows past the end of the sequence hold copies of its last row: masked like invisible keys
                const int rl = rh * 16 + 4 * g + r, rw = row0 + rl;
                bool ok = rl < nvalid;
                if (is_ctx) ok = ok && (!LOCAL || (my_key[h] > P + rw - W));
                else ok = ok && (my_key[h] <= rw) && (!LOCAL || (my_key[h] > rw - W));
                if (!ok) e = 0.f;
              }
              pv[h][r] = e;
              dsv[h][r] = e * dpv[h][r];   // -dS
            }
        };
        if (__builtin_expect(flags & HDR_MASK, 0)) softmax_part(std::true_type{});
        else softmax_part(std::false_type{});
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          u32x2 wp, wd;
          wp.x = pack2_bf16(pv[h][0], pv[h][1]);
          wp.y = pack2_bf16(pv[h][2], pv[h][3]);
          wd.x = pack2_bf16(dsv[h][0], dsv[h][1]);
          wd.y = pack2_bf16(dsv[h][2], dsv[h][3]);
          *reinterpret_cast<u32x2*>(xw + h * 256) = wp;
          *reinterpret_cast<u32x2*>(xw + h * 256 + 2048) = wd;
        }
      } else {
        // no visible (row, key) pair in this block: publish zero operands, the consumers do not branch
        const u32x2 z = {0u, 0u};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          *reinterpret_cast<u32x2*>(xw + h * 256) = z;
          *reinterpret_cast<u32x2*>(xw + h * 256 + 2048) = z;
        }
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
    }
  } else {
    // ================================= consumer ==============================================
    const int jb = wave - 4;
    const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);
    // ---- global -> LDS loads: instruction i = jb + 4 t of a row block covers RPI rows of Q (t < IPB/2) or
    // dO; lane l lands at LDS chunk position l % CPR of row (l / CPR) of the instruction, so it fetches the
    // chunk that the tile swizzle stores there.  The swizzle has a period of 16 rows and the instructions of a
    // wave are 8 rows apart: odd t flip bit 1 of the chunk index.
    // (registers of their own for the loop's scalar inputs: measured faster without a window, slower with one)
    auto keep = [](auto v) __attribute__((always_inline)) {
      if constexpr (LOCAL) return v;
      else return own_sgpr(v);
    };
    const int G = keep(p.G);
    const int q_ts = keep((int)p.q.ts), do_ts = keep((int)p.dout.ts);
    const int64_t q_hs = keep(p.q.hs), do_hs = keep(p.dout.hs), total = keep((int64_t)p.total);
    const int ld_row0 = jb * RPI + lane / CPR;
    const int ld_coff = ((lane % CPR) ^ swz<D>(ld_row0)) * 16;
    const uint32_t ld_lds = smem_addr + jb * 1024;
    // per-lane global offsets of this wave's load instructions for a block of 32 valid rows (a partial last
    // block clamps its rows instead: rare, computed on the spot)
    uint32_t voff_full[IPB];
#pragma unroll
    for (int t = 0; t < IPB; ++t) {
      const int tt = t % (IPB / 2);
      voff_full[t] = (uint32_t)((ld_row0 + tt * 4 * RPI) * (t < IPB / 2 ? q_ts : do_ts) * 2 + (ld_coff ^ ((tt & 1) * 32)));
    }
    // row statistics: lanes 0-31 fetch LSE*log2e, lanes 32-63 fetch D; both arrays live in one workspace, D
    // first and LSE*log2e less than 4 GB behind it (checked by the launcher), so one scalar base plus an
    // unsigned 32-bit lane offset addresses both
    const float* stat_ptr = p.dvec;
    const uint32_t stat_lane_off = hi ? 0u : (uint32_t)((const char*)p.lse2 - (const char*)p.dvec);

    // ---- row-block schedule (Alg. 1, "Q-row blocks in causal support of K_n"): sequences of the tile, row
    // blocks of 32 that see at least one key of the tile, query heads of the group innermost.  All state is
    // wave-uniform and advanced incrementally.
    // With a window the order is sequences, heads, row blocks: neighbouring key tiles then read a given (head, row
    // block) two intervals apart instead of 2 G, close enough for the second one to find it in the L2 (a tile reads
    // only the W + BN rows behind its keys, and without that reuse every tile fetches them from memory again).
    int seq = seq_lo, rb = 0, rb_lo = 0, rb_end = 0, g = 0, R = 0, row_begin = 0, row0 = 0, nvalid = 0;
    const u16 *q_row = nullptr, *do_row = nullptr, *q_cur = nullptr, *do_cur = nullptr;
    int64_t st_row = 0, st_cur = 0;
    bool more = false;
    uint32_t gflags[NKS] = {};   // wave 4: flags of the key subtiles for the current row group
    // Row blocks [plain_lo, plain_hi) (first rows) of a windowed run see every key of the tile, none masked: in the response
    // region those whose first row is at or past the tile's last key and whose last row is still inside the window of its
    // first key; in the prompt region (every response row is past every prompt key) only the window bounds them.
    const int plain_lo = is_ctx ? INT_MIN : key0 + BN - 1;
    const int plain_hi = is_ctx ? key0 + W - 31 - P : key0 + W - 31;
    // (formed per subtile with scalar operations: comparing the schedule state with a lane-dependent key makes the
    // compiler keep that state, and everything derived from it, in vector registers, with spills and with
    // execution masks for the schedule's branches)
    auto enter_group = [&]() __attribute__((always_inline)) {
      row0 = rb * HB;
      nvalid = min(HB, R - row0);
      if (!LOCAL) {
        q_cur = q_row;
        do_cur = do_row;
        st_cur = st_row;
        g = 0;
      }
      if (wave == 4) {
        // most row blocks see every key of the tile: two comparisons settle them
        if (LOCAL && row0 >= plain_lo && row0 < plain_hi && nvalid == HB) {
#pragma unroll
          for (int i = 0; i < NKS; ++i) gflags[i] = HDR_VALID | HDR_ACTIVE;
          return;
        }
#pragma unroll
        for (int i = 0; i < NKS; ++i) {
          const int k_lo = key0 + i * 32, k_hi = k_lo + 31;
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
          gflags[i] = HDR_VALID | (a ? HDR_ACTIVE : 0) | (m ? HDR_MASK : 0);
        }
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
      if (LOCAL) {
        rb_lo = rb;
        g = 0;
        q_cur = q_row;
        do_cur = do_row;
        st_cur = st_row;
      }
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
    // what the loads of the block requested last need (the windowed kernel issues them one by one, see below)
    const u16 *ib_q = nullptr, *ib_do = nullptr, *ib_stat = nullptr;
    int ib_last = 0;
    // requests the next block of the schedule (or marks the end) in stage IS and advances the schedule; without its
    // loads if the caller issues them itself (issue_one)
    auto issue_block = [&](auto ISc, auto with_loads) __attribute__((always_inline)) {
      constexpr int IS = decltype(ISc)::value;
      constexpr bool LOADS = decltype(with_loads)::value;
      if (wave == 4 && lane < NKS) {
        u32x4 h;
        h.x = more ? (lane == 0 ? gflags[0] : gflags[1]) : 0u;
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
        if constexpr (LOCAL) {
          ib_last = last;
          ib_q = q_base;
          ib_do = do_base;
          ib_stat = uniform_ptr(reinterpret_cast<const u16*>(stat_ptr + st_cur));
        }
        // (one branch for the whole block, not one per load)
        if constexpr (!LOADS) {
        } else if (__builtin_expect(nvalid == HB, 1)) {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            dma16_at<IS * STAGE_BYTES + (t < IPB / 2 ? 0 : HT_BYTES) + (t % (IPB / 2)) * 4096>(
                t < IPB / 2 ? q_base : do_base, voff_full[t], ld_lds);
          });
        } else {
          static_for<IPB>([&](auto Tc) __attribute__((always_inline)) {
            constexpr int t = decltype(Tc)::value;
            constexpr bool is_q = t < IPB / 2;
            constexpr int tt = t % (IPB / 2);
            const int row = ld_row0 + tt * 4 * RPI;
            const uint32_t voff = __umul24((unsigned)min(row, last), (unsigned)((is_q ? q_ts : do_ts) * 2)) +
                                  (uint32_t)(ld_coff ^ ((tt & 1) * 32));
            dma16_at<IS * STAGE_BYTES + (is_q ? 0 : HT_BYTES) + tt * 4096>(is_q ? q_base : do_base, voff, ld_lds);
          });
        }
        if (LOADS && wave == 5) {
          dma4_at<IS * STAGE_BYTES + STAT_OFF>(uniform_ptr(reinterpret_cast<const u16*>(stat_ptr + st_cur)),
                                               stat_lane_off + (uint32_t)min(l32, last) * 4u, smem_addr);
        }
        if constexpr (LOCAL) {
          if (__builtin_expect(++rb < rb_end, 1)) {
            q_cur += (int64_t)HB * q_ts;
            do_cur += (int64_t)HB * do_ts;
            st_cur += HB;
            enter_group();
          } else if (++g < G) {
            rb = rb_lo;
            q_row += q_hs;
            do_row += do_hs;
            st_row += total;
            q_cur = q_row;
            do_cur = do_row;
            st_cur = st_row;
            enter_group();
          } else {
            rb = rb_end - 1;   // (next_group steps past the last row block: on to the next sequence)
            next_group();
          }
        } else {
          if (__builtin_expect(++g < G, 1)) {
            q_cur += q_hs;
            do_cur += do_hs;
            st_cur += total;
          } else {
            next_group();
          }
        }
      }
    };
    // Load instruction t of the block requested last, without a branch: the rows of a partial last block are clamped with
    // three vector operations, and after the end of the schedule the loads repeat the last block's, into a stage whose
    // header says that it holds nothing.
    const int q_neg = -q_ts * 2, do_neg = -do_ts * 2;
    auto issue_one = [&](auto ISc, auto Tc) __attribute__((always_inline)) {
      constexpr int IS = decltype(ISc)::value, t = decltype(Tc)::value;
      constexpr bool is_q = t < IPB / 2;
      constexpr int tt = t % (IPB / 2);
      const int over = max(ld_row0 + tt * 4 * RPI - ib_last, 0);   // rows past the last valid one step back to it
      const uint32_t voff = (uint32_t)__mul24(over, is_q ? q_neg : do_neg) + voff_full[t];
      dma16_at<IS * STAGE_BYTES + (is_q ? 0 : HT_BYTES) + tt * 4096>(is_q ? ib_q : ib_do, voff, ld_lds);
      if (t == IPB - 1 && wave == 5)
        dma4_at<IS * STAGE_BYTES + STAT_OFF>(ib_stat, stat_lane_off + (uint32_t)min(l32, ib_last) * 4u, smem_addr);
    };
    // Block b is requested AHEAD blocks early and must have landed by the end of interval b - 2 (the
    // producer reads its operands one interval early): the youngest block (IPB loads per wave; wave 5
    // issues one more, for it the bound is a little stricter) may stay in flight.  If the newest request was
    // the end mark, fewer loads are outstanding: wait for all of them.
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
    if (LOCAL && !more) {
      // No row block at all: the windowed main loop issues its loads unconditionally and would have no valid address.
      // One empty header ends the producers' schedule after one interval; the gradient of these keys is zero.
      if (wave == 4 && lane < NKS) *reinterpret_cast<u32x4*>(smem + HDR_OFF + lane * 16) = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
      __syncthreads();   // the producers' only interval
      const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
      if (!to_acc) {
        const TViewOut& gk = is_ctx ? p.dkc : p.dkd;
        const TViewOut& gv = is_ctx ? p.dvc : p.dvd;
        const int nkeys = min(region_len, key0 + BN) - key0;
        for (int i = tid - 256; i < nkeys * D; i += 256) {
          const int64_t grow = key_row_begin + key0 + i / D;
          const int col = i % D;
          gk.ptr[grow * gk.ts + (int64_t)hk * gk.hs + col] = 0;
          gv.ptr[grow * gv.ts + (int64_t)hk * gv.hs + col] = 0;
        }
      }
      return;
    }
    issue_block(IC<0>{}, std::true_type{});
    issue_block(IC<1>{}, std::true_type{});
    issue_block(IC<2>{}, std::true_type{});
    wait_loads();

    // Each consumer wave owns the head-dim blocks jb and jb + 4 (128 columns apart: the same swizzled chunk
    // position, 256 bytes further) of both key subtiles; the transposed Q / dO operands of a head-dim block are
    // shared by the two subtiles.
    f32x16 dk[NKS][2], dv[NKS][2];
#pragma unroll
    for (int i = 0; i < NKS; ++i)
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          dk[i][db][r] = 0.f;
          dv[i][db][r] = 0.f;
        }
    const unsigned char* tr0_lo = smem + tr_off<D>(lane, hi * 4, jb * 32);
    const unsigned char* tr1_lo = smem + tr_off<D>(lane, hi * 4 + 8, jb * 32);
    const unsigned char* tr0_hi = tr0_lo + HALF;
    const unsigned char* tr1_hi = tr1_lo + HALF;
    const unsigned char* xr_lane = smem + XCH_OFF + lane * 16;
    bf16x8 tq[2][2], tdo[2][2];   // [k-step][head-dim block]: Q^T, dO^T operands of the row block accumulated next interval
    if constexpr (LOCAL) {
      // The windowed loop accumulates in every interval, also in the first one, where there is no block yet: zero operands,
      // in the registers and in the exchange buffer that the producers fill in the second interval (every consumer clears
      // exactly the bytes it reads: no barrier needed)
      const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          tq[t2][db] = __builtin_bit_cast(bf16x8, z);
          tdo[t2][db] = __builtin_bit_cast(bf16x8, z);
        }
#pragma unroll
      for (int j = 0; j < XCH_BYTES / 1024; ++j)
        *reinterpret_cast<u32x4*>(smem + XCH_OFF + XCH_BYTES + j * 1024 + lane * 16) = z;
    }

    // one interval: accumulates block h-1, reads the transposed operands of block h (stage U), requests
    // block h + AHEAD; returns false after the end of the schedule
    auto interval = [&](auto Uc) __attribute__((always_inline)) -> bool {
      constexpr int U = decltype(Uc)::value, IS = (U + AHEAD) % NBUF, XB = (U + 1) & 1;
      // Without a window the requests go first: the producers' MFMAs run meanwhile, the consumers' follow them.  With a
      // window, where the schedule costs more scalar work per block, one request behind each MFMA pair measured faster
      // (a wave waits at a load until the memory pipeline takes it, and the MFMAs run meanwhile); the MFMAs are then not
      // conditional (a branch around them and the loads makes the compiler copy the accumulators).
      issue_block(IC<IS>{}, std::integral_constant<bool, !LOCAL>{});
      if (LOCAL || (vbits & (1u << (AHEAD + 1)))) {
        const unsigned char* xr = xr_lane + XB * XCH_BYTES;
        // all P / -dS operands are requested before the first MFMA
        bf16x8 pa[2][NKS], dsa[2][NKS];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int i = 0; i < NKS; ++i) {
            pa[t2][i] = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + t2 * 1024);
            dsa[t2][i] = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + (2 + t2) * 1024);
          }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (LOCAL) {
          static_assert(IPB == 4 * NKS, "one load instruction per MFMA pair");
          static_for<IPB>([&](auto Nc) __attribute__((always_inline)) {
            constexpr int n = decltype(Nc)::value, t2 = n / (2 * NKS), db = (n / NKS) % 2, i = n % NKS;
            dv[i][db] = mfma32(pa[t2][i], tdo[t2][db], dv[i][db]);
            dk[i][db] = mfma32(dsa[t2][i], tq[t2][db], dk[i][db]);
            __builtin_amdgcn_sched_barrier(0);
            issue_one(IC<IS>{}, Nc);
            __builtin_amdgcn_sched_barrier(0);
          });
        } else {
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
              for (int i = 0; i < NKS; ++i) {
                dv[i][db] = mfma32(pa[t2][i], tdo[t2][db], dv[i][db]);
                dk[i][db] = mfma32(dsa[t2][i], tq[t2][db], dk[i][db]);
              }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      const bool cur = vbits & (1u << AHEAD);
      if (__builtin_expect(cur, 1)) {
        const unsigned char* t0 = (U < NBUF / 2 ? tr0_lo : tr0_hi) + (U % (NBUF / 2)) * STAGE_BYTES;
        const unsigned char* t1 = (U < NBUF / 2 ? tr1_lo : tr1_hi) + (U % (NBUF / 2)) * STAGE_BYTES;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            tdo[t2][db] = tr_pair(t0 + HT_BYTES + t2 * 16 * RB + db * 256, t1 + HT_BYTES + t2 * 16 * RB + db * 256);
            tq[t2][db] = tr_pair(t0 + t2 * 16 * RB + db * 256, t1 + t2 * 16 * RB + db * 256);
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
    }

    // ---- epilogue: C layout -> lane owns head-dim column, register r owns key crow(r); the dK
    // accumulator holds -dK / scale
    const bool to_acc = is_ctx ? (p.dkc_acc != nullptr) : (p.dkd_acc != nullptr);
    float* acc_k = is_ctx ? p.dkc_acc : p.dkd_acc;
    float* acc_v = is_ctx ? p.dvc_acc : p.dvd_acc;
#pragma unroll
    for (int i = 0; i < NKS; ++i)
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int dcol = (jb + 4 * db) * 32 + l32;
        const f32x16 gks = dk[i][db], gvs = dv[i][db];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + i * 32 + crow(r, hi);
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

template <bool LOCAL>
hipError_t launch_t(AttnParams p, hipStream_t st) {
  p.n_ctx_tiles = (p.ctx_len + BN - 1) / BN;
  p.n_dec_tiles = (p.max_rows + BN - 1) / BN;
  if (p.n_split < 1) p.n_split = 1;
  // the kernel addresses LSE*log2e as D + 32-bit unsigned byte offset
  if (reinterpret_cast<uintptr_t>(p.lse2) < reinterpret_cast<uintptr_t>(p.dvec) ||
      reinterpret_cast<uintptr_t>(p.lse2) - reinterpret_cast<uintptr_t>(p.dvec) >= (1ull << 32))
    return hipErrorInvalidValue;
  hipError_t e = ensure_dynamic_lds<dkdv256_kernel<LOCAL>>(SMEM_BYTES);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)(p.grp ? p.n_groups : 1) * p.n_ctx_tiles * p.Hk * p.n_split +
                       (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
  if (nblk == 0) return hipSuccess;
  hipLaunchKernelGGL(dkdv256_kernel<LOCAL>, dim3((unsigned)nblk), dim3(512), SMEM_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_dkdv256(const AttnParams& p, hipStream_t st) {
  return p.window > 0 ? launch_t<true>(p, st) : launch_t<false>(p, st);
}

}  // namespace dkv
