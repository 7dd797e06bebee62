// dK / dV kernel for head dims 64 and 128 with producer / consumer wave specialisation (same mathematics
// and the same ownership rule as the other dK/dV kernels: one workgroup owns a 128-key tile of one KV
// head; a shared-prompt tile sums the contributions of ALL sequences and heads of the group in fp32
// registers and is cast once -- Alg. 1 with the race of the shared prompt gradients removed by ownership).
//
// A wave issues at most one instruction every four cycles, so with two waves per SIMD the kernel is bound
// by the instruction count of its busiest wave, not by MFMA or LDS throughput.  The work of one block of 32
// query rows is therefore cut into two roles of about equal, small instruction count that share a SIMD:
//   producer (waves 0-3, one per 32-key subtile) keeps its K and -V fragments in registers, computes
//             S = Q K^T and D - dP = D + dO (-V)^T with the MFMA accumulator initialised to D, then
//             P = exp2(S*scale*log2e - LSE*log2e) and -dS = P * (D - dP), and publishes P, -dS as bf16
//             MFMA operands in LDS.  Nothing else: no address arithmetic, no schedule, no global loads.
//   consumer (waves 4-7) owns the fp32 dK, dV accumulators of the same 32 keys (all of the head dim) and,
//             one row block behind the producer, accumulates dV += P^T dO and -dK += (-dS)^T Q with
//             dO^T / Q^T from LDS transpose reads of the same tiles.  The consumers also walk the row-block
//             schedule, issue the global -> LDS loads (global_load_lds: Q, dO, LSE*log2e, D land in LDS
//             without passing through registers, several row blocks ahead) and write a small per-block
//             header (valid / active / needs-mask flags per key subtile, first row, row count) that is all
//             the producers need to know about the schedule.
// Every LDS operand is read into registers one interval before it is used, across the single workgroup
// barrier per row block, so LDS latency is hidden although each role has only one wave per SIMD.
//
// The compiler does not know about the global -> LDS loads; the consumers count them themselves
// (s_waitcnt vmcnt) before the barrier that publishes a row block, and no other vector memory load is
// issued inside the main loop (a compiler-placed wait would also wait for every row block in flight).
#include <cstdlib>
#include <type_traits>
#include "common.h"
#include "kvsched.h"
#include "launch.h"
#include "tiles.h"

namespace dkv {

// 64 lanes x 16 bytes: global address = sbase + voff (per lane), LDS address = lds_addr + 16 * lane.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory");
}
// 64 lanes x 4 bytes from per-lane 64-bit addresses, LDS address = lds_addr + 4 * lane.
__device__ __forceinline__ void dma4(const void* vaddr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               :
               : "s"(lds_addr), "v"(vaddr)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ const u16* uniform_ptr(const u16* ptr) {
  const uint64_t v = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const u16*>(((uint64_t)hi << 32) | lo);
}

#ifdef DKV_PROF
__device__ unsigned long long g_prof[32];
#define PROF_INIT long long pbusy = 0, pwait = 0, pmid = 0, tprev = clock64();
#define PT_MID { const long long t_ = clock64(); pmid += t_ - tprev; tprev = t_; }
#define PT_BUSY { const long long t_ = clock64(); pbusy += t_ - tprev; tprev = t_; }
#define PT_WAIT { const long long t_ = clock64(); pwait += t_ - tprev; tprev = t_; }
#define PROF_END(slot) if (lane == 0 && is_ctx) { atomicAdd(&g_prof[slot], (unsigned long long)pbusy); atomicAdd(&g_prof[slot + 1], (unsigned long long)pwait); atomicAdd(&g_prof[slot + 2], (unsigned long long)pmid); }
#else
#define PROF_INIT
#define PT_MID
#define PT_BUSY
#define PT_WAIT
#define PROF_END(slot)
#endif
enum : int { HDR_VALID = 1, HDR_ACTIVE = 2, HDR_MASK = 4 };

template <int D, bool LOCAL>
__global__ __launch_bounds__(512) void dkdv4_kernel(const AttnParams p) {
  constexpr int BN = 128, HB = 32;                 // keys per workgroup, query rows per block
  constexpr int KS = D / 16, DSUB = D / 32, RB = 2 * D, CPR = D / 8;
  constexpr int HT_BYTES = HB * RB;                // one Q or dO row block
  constexpr int STAT_OFF = 2 * HT_BYTES;           // lse2[32] | D[32]
  constexpr int STAGE_BYTES = STAT_OFF + 256;
  constexpr int NBUF = 6, AHEAD = NBUF - 1;        // row blocks requested ahead of the one being computed
  constexpr int XCH_BYTES = 16384;                 // [key subtile][P k-step 0,1 | dS k-step 0,1][lane] x 16 B
  constexpr int HDR_SLOTS = 16, HDR_BYTES = 128;    // per block: 4 flag chunks | Q chunk | dO chunk | stat chunk
  constexpr int NIT = HT_BYTES / 1024;             // 1 KB load instructions per row block and tensor
  constexpr int IPW = NIT / 4;                     // per wave (producers load Q, consumers dO)
  constexpr int RPI = 1024 / RB;                   // rows per load instruction
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int kvs = wave & 3;
  const bool producer = wave < 4;
  const int P = p.ctx_len, W = p.window;
  unsigned char* xch = smem + NBUF * STAGE_BYTES;
  unsigned char* hdr = xch + 2 * XCH_BYTES;
  const uint32_t smem_addr = (uint32_t)reinterpret_cast<uintptr_t>(smem);

  // ---- block decode: prompt tiles first (heavy), then response tiles
  const int ctx_blocks = p.n_ctx_tiles * p.Hk * p.n_split;
  int bid = blockIdx.x;
  bool is_ctx;
  int hk, key0, seq_lo, seq_hi;
  if (bid < ctx_blocks) {
    is_ctx = true;
    hk = bid % p.Hk;
    int t = bid / p.Hk;
    const int split = t % p.n_split;
    key0 = (t / p.n_split) * BN;
    seq_lo = (int)((int64_t)p.n_seqs * split / p.n_split);
    seq_hi = (int)((int64_t)p.n_seqs * (split + 1) / p.n_split);
  } else {
    bid -= ctx_blocks;
    is_ctx = false;
    hk = bid % p.Hk;
    int t = bid / p.Hk;
    key0 = (t % p.n_dec_tiles) * BN;
    seq_lo = t / p.n_dec_tiles;
    seq_hi = seq_lo + 1;
    const int rb0 = p.cu ? p.cu[seq_lo] : 0;
    const int Rs = p.cu ? (p.cu[seq_lo + 1] - rb0) : p.total;
    if (key0 >= Rs) return;
  }

  int region_len, key_row_begin = 0;
  if (is_ctx) {
    region_len = P;
  } else {
    key_row_begin = p.cu ? p.cu[seq_lo] : 0;
    region_len = p.cu ? (p.cu[seq_lo + 1] - key_row_begin) : p.total;
  }
  const int wave_key_lo = key0 + kvs * 32;
  const int my_key = wave_key_lo + l32;

  // ---- global -> LDS loads of this wave: instructions j = kvs + 4 t of its tensor (producers Q, consumers
  // dO), RPI rows each; lane l lands at LDS chunk position l % CPR of row (l / CPR) of the instruction, so it
  // fetches the chunk that the tile swizzle stores there.
  const int G = p.G;
  const int ld_ts = producer ? (int)p.q.ts : (int)p.dout.ts;
  const int64_t ld_hs2 = (producer ? p.q.hs : p.dout.hs) * 2;   // bytes between heads
  const int ld_row0 = kvs * RPI + lane / CPR;
  const int ld_coff = ((lane % CPR) ^ swz<D>(ld_row0)) * 16;   // same for every t: the swizzle has period 4 RPI
  const uint32_t ld_lds = smem_addr + (producer ? 0 : HT_BYTES) + kvs * 1024;
  const float* lse2_ptr = p.lse2;
  const float* dvec_ptr = p.dvec;
  const int64_t total = p.total;

  // ---- row-block schedule (Alg. 1, "Q-row blocks in causal support of K_n"): sequences of the tile, row
  // blocks of 32 that see at least one key of the tile, query heads of the group innermost.  A "row group"
  // is one row block for all G heads: its G blocks share everything but the head.  Wave 4 walks the row
  // groups and writes one header per group into a small LDS ring: per key subtile the valid / active /
  // needs-mask flags, first row and row count, and the base pointers (head 0 of the group) of Q, dO and
  // the row statistics.  Every wave follows the block sequence with a head counter and reads a header only
  // when it enters a new group, so the per-block control cost is a few scalar operations.
  auto hdr_at = [&](int grp) { return hdr + (grp & (HDR_SLOTS - 1)) * HDR_BYTES; };
  struct Flags {
    int flags, row0, nvalid;
  };
  auto read_flags = [&](int grp) {
    const u32x4 h = *reinterpret_cast<const u32x4*>(hdr_at(grp) + kvs * 16);
    Flags f;
    f.flags = __builtin_amdgcn_readfirstlane((int)h.x);
    f.row0 = __builtin_amdgcn_readfirstlane((int)h.y);
    f.nvalid = __builtin_amdgcn_readfirstlane((int)h.z);
    return f;
  };
  // request position: block `blk + AHEAD` of the schedule
  int gd = 0, grp_d = 0, nvalid_d = 0;
  const unsigned char* base_d = nullptr;
  int64_t st_d = 0;
  auto read_request_header = [&]() {
    const u32x4 h = *reinterpret_cast<const u32x4*>(hdr_at(grp_d) + (producer ? 64 : 80));
    nvalid_d = __builtin_amdgcn_readfirstlane((int)h.z);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(h.x), hi32 = __builtin_amdgcn_readfirstlane(h.y);
    base_d = reinterpret_cast<const unsigned char*>(((uint64_t)hi32 << 32) | lo);
    if (wave == 5) {
      const u32x4 hs = *reinterpret_cast<const u32x4*>(hdr_at(grp_d) + 96);
      st_d = (int64_t)(((uint64_t)__builtin_amdgcn_readfirstlane(hs.y) << 32) | __builtin_amdgcn_readfirstlane(hs.x));
    }
  };
  // requests this wave's share of the block at the request position into stage `buf` and advances the
  // position; false if the block is past the end of the schedule
  auto issue_block = [&](int buf) -> bool {
    const bool valid = nvalid_d != 0;
    if (__builtin_expect(valid && !(p.dbg & 4), 1)) {
      const uint32_t dst = ld_lds + buf * STAGE_BYTES;
      const int last = nvalid_d - 1;   // rows past the end of the sequence re-read its last row
#pragma unroll
      for (int t = 0; t < IPW; ++t)
        dma16(base_d, (uint32_t)(min(ld_row0 + t * 4 * RPI, last) * ld_ts * 2 + ld_coff), dst + t * 4096);
      if (wave == 5) {
        // lanes 0-31 fetch LSE*log2e, lanes 32-63 fetch D of the block's rows
        const int64_t off = st_d + min(l32, last);
        const float* a0 = lse2_ptr + off;
        const float* a1 = dvec_ptr + off;
        dma4(hi ? a1 : a0, smem_addr + buf * STAGE_BYTES + STAT_OFF);
      }
    }
    if (__builtin_expect(++gd == G, 0)) {
      gd = 0;
      ++grp_d;
      read_request_header();
    } else {
      base_d += ld_hs2;
      st_d += total;
    }
    return valid;
  };
  // Row block g is requested AHEAD blocks early and must have landed by the end of interval g - 2 (the
  // producer reads its operands one interval early): up to AHEAD-2 younger row blocks (each IPW loads per
  // wave, one more in wave 5) may stay in flight.
  auto wait_loads = [&](bool full) {
    wait_vm<(AHEAD - 2) * IPW>();   // wave 5 issues one more load per block: for it the bound is a little stricter
    if (__builtin_expect(!full, 0)) wait_vm<0>();
  };

  // wave 4: schedule state (wave-uniform) and header writer
  const int q_ts = (int)p.q.ts, do_ts = (int)p.dout.ts;
  int seq = seq_lo, rb = 0, rb_end = 0, R = 0, row_begin = 0, hdr_written = 0;
  const u16 *q_row = nullptr, *do_row = nullptr;
  int64_t st_row = 0;
  bool more = false;
  auto init_seq = [&]() {
    row_begin = p.cu ? p.cu[seq] : 0;
    R = p.cu ? (p.cu[seq + 1] - row_begin) : p.total;
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
    q_row = p.q.ptr + grow * q_ts + (int64_t)hk * G * p.q.hs;
    do_row = p.dout.ptr + grow * do_ts + (int64_t)hk * G * p.dout.hs;
    st_row = (int64_t)hk * G * p.total + grow;
  };
  auto advance_group = [&]() {
    if (++rb < rb_end) {
      q_row += (int64_t)HB * q_ts;
      do_row += (int64_t)HB * do_ts;
      st_row += HB;
      return;
    }
    more = false;
    while (++seq < seq_hi) {
      init_seq();
      if (rb < rb_end) {
        more = true;
        return;
      }
    }
  };
  // writes the header of the next row group (or an end mark) and advances the schedule
  auto write_header = [&]() {
    const int row0 = rb * HB;
    const int nvalid = more ? min(HB, R - row0) : 0;
    // lanes 0-3: flag chunk of key subtile `lane`
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
    const uint32_t flags = more ? (HDR_VALID | (a ? HDR_ACTIVE : 0) | (m ? HDR_MASK : 0)) : 0;
    // lanes 4, 5, 6: 64-bit base of Q, dO (head 0 of the group), statistics offset
    const uint64_t pq = reinterpret_cast<uint64_t>(q_row), pd = reinterpret_cast<uint64_t>(do_row);
    const uint64_t ps = (uint64_t)st_row;
    const uint64_t pv = lane == 4 ? pq : (lane == 5 ? pd : ps);
    u32x4 h;
    h.x = lane < 4 ? flags : (uint32_t)pv;
    h.y = lane < 4 ? (uint32_t)row0 : (uint32_t)(pv >> 32);
    h.z = (uint32_t)nvalid;
    h.w = 0;
    if (lane < 7) *reinterpret_cast<u32x4*>(hdr_at(hdr_written) + lane * 16) = h;
    ++hdr_written;
    if (more) advance_group();
  };

  // ---- prologue: headers of the first row groups, requests of blocks 0 .. AHEAD-1
  constexpr int HDR_AHEAD = 3;   // headers kept ahead of the group of the request position
  if (wave == 4) {
    for (; seq < seq_hi; ++seq) {
      init_seq();
      if (rb < rb_end) {
        more = true;
        break;
      }
    }
#pragma unroll 1
    for (int i = 0; i < AHEAD + HDR_AHEAD; ++i) write_header();   // covers block AHEAD's group even when G = 1
  }
  __syncthreads();
  read_request_header();
  bool issued = false;   // the most recent request was a row block (not past the end)
#pragma unroll 1
  for (int b = 0; b < AHEAD; ++b) issued = issue_block(b);

  if (producer) {
    // =========================================================================================
    const float c = p.scale_log2;
    const u16 *kbase, *vbase;
    int64_t kts, vts;
    if (is_ctx) {
      kbase = p.kc.ptr + (int64_t)hk * p.kc.hs;
      vbase = p.vc.ptr + (int64_t)hk * p.vc.hs;
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
    int roff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) roff[ks] = tile_off<D>(l32, 2 * ks + hi);
    const int stat_off = STAT_OFF + hi * 16;   // this lane's rows 8*(r/4) + 4*hi + r%4: four 16-byte groups

    bf16x8 qfr[KS], dofr[KS];
    auto load_frags = [&](int buf) {
      const unsigned char* Qb = smem + buf * STAGE_BYTES;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        qfr[ks] = *reinterpret_cast<const bf16x8*>(Qb + roff[ks]);
        dofr[ks] = *reinterpret_cast<const bf16x8*>(Qb + HT_BYTES + roff[ks]);
      }
    };
    // row statistics of this lane's 16 rows (register r <-> row crow(r, hi)) from stage `buf`
    auto load_stat = [&](int buf, int which, float* out) {
      const unsigned char* Sb = smem + buf * STAGE_BYTES + stat_off + which * 128;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(Sb + r4 * 32);
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) out[r4 * 4 + e4] = v[e4];
      }
    };

    wait_loads(issued);
    __syncthreads();   // row blocks 0 and 1 are in LDS
    // compute position (block h) and operand-prefetch position (block h + 1)
    Flags cur = read_flags(0), pre = cur;
    int gp = 0, grp_p = 0;
    auto advance_prefetch = [&]() {
      if (__builtin_expect(++gp == G, 0)) {
        gp = 0;
        pre = read_flags(++grp_p);
      }
    };
    advance_prefetch();
    if ((cur.flags & HDR_ACTIVE) && !(p.dbg & 1)) load_frags(0);
    int hbuf = 0, ibuf = AHEAD, xb = 0;
    PROF_INIT
    while (true) {
      if (!(cur.flags & HDR_VALID)) {
        __syncthreads();
        break;
      }
      const int nbuf = hbuf + 1 == NBUF ? 0 : hbuf + 1;
      const int flags = cur.flags, row0 = cur.row0, nvalid = cur.nvalid;
      const bool act = (flags & HDR_ACTIVE) && !(p.dbg & 1), nact = (pre.flags & HDR_ACTIVE) && !(p.dbg & 1);

      f32x16 s, dpv;
      float l2[16];
      if (act) {
        float dinit[16];
        load_stat(hbuf, 1, dinit);   // its latency hides behind the S chain
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s = mfma32(qfr[ks], kf[ks], s);
#pragma unroll
        for (int r = 0; r < 16; ++r) dpv[r] = dinit[r];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dpv = mfma32(dofr[ks], vfn[ks], dpv);   // D - dP
        load_stat(hbuf, 0, l2);
      }
      if (nact) load_frags(nbuf);
      issued = issue_block(ibuf);
      PT_MID
      if (act) {
        float pv[16], dsv[16];
        auto softmax_part = [&](auto masked) {
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
        unsigned char* xw = xch + xb * XCH_BYTES + kvs * 4096 + lane * 16;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          *reinterpret_cast<bf16x8*>(xw + t2 * 1024) = pack8_bf16(pv + t2 * 8);
          *reinterpret_cast<bf16x8*>(xw + (2 + t2) * 1024) = pack8_bf16(dsv + t2 * 8);
        }
      } else {
        // no visible (row, key) pair in this block: publish zero operands, the consumers do not branch
        unsigned char* xw = xch + xb * XCH_BYTES + kvs * 4096 + lane * 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < 4; ++t) *reinterpret_cast<u32x4*>(xw + t * 1024) = z;
      }
      PT_BUSY
      wait_loads(issued);
      __syncthreads();
      PT_WAIT
      cur = pre;
      advance_prefetch();
      hbuf = nbuf;
      ibuf = ibuf + 1 == NBUF ? 0 : ibuf + 1;
      xb ^= 1;
    }
    PROF_END(wave * 4)
  } else {
    // =========================================================================================
    // Each consumer wave owns one 32-wide head-dim block (dblk) of the gradients of NK key subtiles: the
    // transposed Q / dO operands of its head-dim block are shared by all its key subtiles, which keeps the
    // (slow) LDS transpose reads at 8 per row block.
    constexpr int NK = DSUB;                       // key subtiles per wave: 4 (d = 128) or 2 (d = 64)
    const int jb = wave - 4, dblk = jb % DSUB, k0 = (jb / DSUB) * NK;
    f32x16 dk[NK], dv[NK];
#pragma unroll
    for (int i = 0; i < NK; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dk[i][r] = 0.f;
        dv[i][r] = 0.f;
      }
    const int toff0 = tr_off<D>(lane, hi * 4, dblk * 32), toff1 = tr_off<D>(lane, hi * 4 + 8, dblk * 32);
    bf16x8 tq[2], tdo[2];   // Q^T, dO^T operands of the row block accumulated next interval
    wait_loads(issued);
    __syncthreads();   // row blocks 0 and 1 are in LDS
    int hbuf = 0, ibuf = AHEAD, xb = 1;   // xb: exchange buffer written during the previous interval
    int flags = read_flags(0).flags, flags_prev = 0;   // only the valid bit matters: inactive subtiles publish zeros
    int gc = 0, grp_c = 0;
    PROF_INIT
    while (true) {
      // requests and schedule first: the producers' MFMAs run meanwhile, the consumers' follow them
      issued = issue_block(ibuf);
      if (wave == 4 && hdr_written < grp_d + HDR_AHEAD) write_header();

      if (!(p.dbg & 2)) {
        const unsigned char* xr = xch + xb * XCH_BYTES + k0 * 4096 + lane * 16;
        if (flags_prev & HDR_VALID) {
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int i = 0; i < NK; ++i) {
              const bf16x8 pa = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + t2 * 1024);
              const bf16x8 dsa = *reinterpret_cast<const bf16x8*>(xr + i * 4096 + (2 + t2) * 1024);
              dv[i] = mfma32(pa, tdo[t2], dv[i]);
              dk[i] = mfma32(dsa, tq[t2], dk[i]);
            }
        }
        if (flags & HDR_VALID) {
          const unsigned char* Qb = smem + hbuf * STAGE_BYTES;
          const unsigned char* dOb = Qb + HT_BYTES;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2) {
            tdo[t2] = tr_pair(dOb + t2 * 16 * RB + toff0, dOb + t2 * 16 * RB + toff1);
            tq[t2] = tr_pair(Qb + t2 * 16 * RB + toff0, Qb + t2 * 16 * RB + toff1);
          }
        }
      }
      PT_MID
      PT_BUSY
      wait_loads(issued);
      __syncthreads();
      PT_WAIT
      if (!(flags & HDR_VALID)) break;
      flags_prev = flags;
      if (__builtin_expect(++gc == G, 0)) {
        gc = 0;
        flags = read_flags(++grp_c).flags;
      }
      hbuf = hbuf + 1 == NBUF ? 0 : hbuf + 1;
      ibuf = ibuf + 1 == NBUF ? 0 : ibuf + 1;
      xb ^= 1;
    }
    PROF_END(wave * 4)

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
          p.dkc.ptr[(int64_t)key * p.dkc.ts + (int64_t)hk * p.dkc.hs + dcol] = (u16)(pack2_bf16(gk, 0.f) & 0xffffu);
          p.dvc.ptr[(int64_t)key * p.dvc.ts + (int64_t)hk * p.dvc.hs + dcol] = (u16)(pack2_bf16(gv, 0.f) & 0xffffu);
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
  p.dbg = getenv("DKV_DBG") ? atoi(getenv("DKV_DBG")) : 0;
  const size_t smem = 6 * (2 * 32 * 2 * D + 256) + 2 * 16384 + 16 * 128;
  auto kern = dkdv4_kernel<D, LOCAL>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  const int64_t nblk = (int64_t)p.n_ctx_tiles * p.Hk * p.n_split + (int64_t)p.n_seqs * p.n_dec_tiles * p.Hk;
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
#ifdef DKV_PROF
extern "C" int dualkv_debug_prof(unsigned long long* out, int reset) {
  hipDeviceSynchronize();
  hipMemcpyFromSymbol(out, HIP_SYMBOL(dkv::g_prof), sizeof(dkv::g_prof));
  if (reset) { unsigned long long z[32] = {}; hipMemcpyToSymbol(HIP_SYMBOL(dkv::g_prof), z, sizeof(z)); }
  return 0;
}
#endif
