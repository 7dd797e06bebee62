// Shared device helpers for the gfx950 shared-prompt attention kernels.
//
// MFMA conventions used everywhere (v_mfma_f32_32x32x16_bf16, wave64):
//   A operand (M x K = 32 x 16): lane l holds row  i = l % 32, k = 8*(l/32) .. 8*(l/32)+7
//   B operand (K x N = 16 x 32): lane l holds col  j = l % 32, k = 8*(l/32) .. 8*(l/32)+7
//   C/D       (M x N = 32 x 32): lane l holds col  j = l % 32, and register r (0..15) holds
//                                row i = 8*(r/4) + 4*(l/32) + r%4
// Because the contraction index only has to agree between A and B, an accumulator tile can be fed
// back as the K-indexed operand of the next MFMA without leaving registers: registers 8t..8t+7 of a
// C tile are 16 distinct rows {16t + 8a + 4*(l/32) + c}, and the matching operand of the other
// matrix is stored in LDS with the same permutation of the contraction index ("kperm" below).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dkv {

typedef unsigned short u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float NEG_BIG = -1.0e30f;      // finite "minus infinity" for running maxima
constexpr float LSE_MASKED = 1.0e30f;    // LSE given to padded rows so that exp2(s - lse) == 0

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// eight consecutive fp32 values of an accumulator tile -> one MFMA operand
__device__ __forceinline__ bf16x8 pack8_bf16(const float* v) {
  u32x4 r;
  r.x = pack2_bf16(v[0], v[1]);
  r.y = pack2_bf16(v[2], v[3]);
  r.z = pack2_bf16(v[4], v[5]);
  r.w = pack2_bf16(v[6], v[7]);
  return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// Combine a value with the one held by lane ^ 32.  v_permlane32_swap exchanges, in place, the upper
// 32 lanes of its first operand with the lower 32 lanes of its second; fed two copies of the same value,
// every lane ends up with its own value in one register and its partner's in the other (no LDS round
// trip).  Written as inline asm with both registers as read-write operands; the leading s_nop covers
// the VALU-write -> permlane-read hazard the compiler cannot see.
// NEVER feed an MFMA result straight into an inline-asm VALU instruction: the wait states between an MFMA and
// a VALU read of its destination are inserted by the compiler, and it does not insert them for inline asm (the
// instruction then reads the registers before the MFMA has written them; seen as run-to-run differences).
__device__ __forceinline__ void swap32(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float xor32_max(float x) {
  float a = x, b = x;
  swap32(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float xor32_sum(float x) {
  float a = x, b = x;
  swap32(a, b);
  return a + b;
}

// Row of a C tile held in register r by this lane.
__device__ __forceinline__ int crow(int r, int hi) { return 8 * (r >> 2) + 4 * hi + (r & 3); }

// Position of contraction index k (0..ROWS-1) inside a "kperm" LDS row: within every group of 16 the
// two middle groups of four are swapped, so that the eight indices one lane needs are contiguous.
__device__ __forceinline__ int kperm4(int k4) {  // k4 = k / 4
  return (k4 & ~3) | ((k4 & 1) << 1) | ((k4 >> 1) & 1);
}

// ---------------------------------------------------------------------------------------------
// Cooperative global -> register -> LDS tile staging.
// A tile is ROWS x D bf16 taken from `ROWS` consecutive token rows of one head.  Thread t owns
// "units" of 4 rows x 8 columns (four 16-byte loads), so it can write both the row-major image
// (4 x 16 B) and the transposed, kperm-ordered image (8 x 8 B) without any cross-lane traffic.
// Consecutive threads take consecutive row quads of one 8-column chunk: their 8-byte writes into the
// transposed image are then contiguous within an image row (with consecutive chunks per thread they land
// eight image rows apart, on two banks: the transposed stores then cost 40 % of the head-dim-512 dK/dV kernel).
// ---------------------------------------------------------------------------------------------
template <int ROWS, int D, int NT>
struct TileRegs {
  static constexpr int CH = D / 8;                       // 16-byte chunks per row
  static constexpr int RQ = ROWS / 4;                    // row quads; consecutive threads take consecutive quads
  static constexpr int NUNITS = (ROWS / 4) * CH;
  static constexpr int UPT = (NUNITS + NT - 1) / NT;     // units per thread
  u32x4 v[UPT][4];

  // base: pointer to (row 0, column 0) of the tile (the same for every thread); rows >= nvalid are zero-filled.
  // Addresses are the uniform base plus a 32-bit byte offset per thread (token strides are bounded by the API),
  // one register per load instead of a 64-bit pointer pair: with pointer pairs the d = 512 dQ kernel spilled them
  // and waited for each load before it could issue the next.
  __device__ __forceinline__ void load(const u16* base, int64_t tok_stride, int nvalid, int tid) {
    const unsigned char* b8 = reinterpret_cast<const unsigned char*>(base);
    const uint32_t sb = (uint32_t)tok_stride * 2u;
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * NT;
      const int rq = unit % RQ, ch = unit / RQ;
      uint32_t off0 = (uint32_t)(rq * 4) * sb + (uint32_t)(ch * 16);
      asm volatile("" : "+v"(off0));   // keeps the zero extension next to the load (base + 32-bit offset form)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = rq * 4 + j;
        u32x4 z = {0u, 0u, 0u, 0u};
        if ((NUNITS % NT == 0 || unit < NUNITS) && row < nvalid)
          z = *reinterpret_cast<const u32x4*>(b8 + (off0 + (uint32_t)j * sb));
        v[u][j] = z;
      }
    }
  }

  // row-major image: lds[row][col], pitch in elements (multiple of 8)
  __device__ __forceinline__ void store_rowmajor(u16* lds, int pitch, int tid) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * NT;
      if (NUNITS % NT != 0 && unit >= NUNITS) continue;
      const int rq = unit % RQ, ch = unit / RQ;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<u32x4*>(lds + (rq * 4 + j) * pitch + ch * 8) = v[u][j];
    }
  }

  // transposed image: lds[col][kperm(row)], pitch in elements (multiple of 4)
  __device__ __forceinline__ void store_transposed(u16* lds, int pitch, int tid) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = tid + u * NT;
      if (NUNITS % NT != 0 && unit >= NUNITS) continue;
      const int rq = unit % RQ, ch = unit / RQ;
      const int pos = kperm4(rq) * 4;
      const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&v[u][0]);
      const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&v[u][1]);
      const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&v[u][2]);
      const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&v[u][3]);
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        u32x2 lo, hi;
        lo.x = (w0[m] & 0xffffu) | (w1[m] << 16);
        lo.y = (w2[m] & 0xffffu) | (w3[m] << 16);
        hi.x = (w0[m] >> 16) | (w1[m] & 0xffff0000u);
        hi.y = (w2[m] >> 16) | (w3[m] & 0xffff0000u);
        *reinterpret_cast<u32x2*>(lds + (ch * 8 + 2 * m) * pitch + pos) = lo;
        *reinterpret_cast<u32x2*>(lds + (ch * 8 + 2 * m + 1) * pitch + pos) = hi;
      }
    }
  }
};

// A bf16 tensor view: element strides.
struct TView {
  const u16* ptr;
  int64_t ts, hs;
};
struct TViewOut {
  u16* ptr;
  int64_t ts, hs;
};

// Parameters shared by the three attention kernels.  "rows" are response rows (Call 2) or prompt
// rows (Call 1, run as N = 1, ctx_len = 0).
struct AttnParams {
  TView q, kc, vc, kd, vd, o, dout;     // o / dout only used by the backward kernels
  TViewOut out_o;                        // fwd: O
  TViewOut dq, dkc, dvc, dkd, dvd;       // bwd outputs (bf16)
  float* lse;                            // (H, total) fwd: written, bwd: read
  float* dvec;                           // (H, total) D = rowsum(dO * O), bwd only
  float* lse2;                           // (H, total) LSE * log2(e), written with D by the preprocess
  float* dkc_acc;                        // optional fp32 (P, Hk, d) accumulators (atomic adds)
  float* dvc_acc;
  float* dkd_acc;                        // optional fp32 (rows, Hk, d) accumulators for response-region keys
  float* dvd_acc;
  const int32_t* cu;                     // (N+1) or nullptr => one sequence [0, total)
  // Several prompt groups in one launch (Sec. 2.2): grp = n_groups x {first prompt row, P_g, first sequence, end
  // sequence} (device), seq_ctx = per sequence {first prompt row, P_g} expanded from it; both nullptr for one group,
  // whose prompt is rows [0, ctx_len) of kc / vc.  With groups, ctx_len is the largest P_g (grid sizing only).
  const int32_t* grp;
  const int32_t* seq_ctx;
  int n_groups;
  int n_seqs, ctx_len, total, max_rows;
  int H, Hk, G;
  int window;                            // > 0: sliding window
  float scale;                           // softmax scale
  float scale_log2;                      // scale * log2(e)
  // Q-stationary kernels: head packing of one workgroup
  int GP, RSH, BMR, MB, HC;              // heads packed, row-subtiles per head, rows per block, blocks, head chunks
  // KV-stationary kernel
  int n_ctx_tiles, n_dec_tiles;          // per sequence upper bound for dec
  int n_split;                           // ctx tiles: the sequence loop is cut in n_split parts
};

// A scalar kernel argument in scalar registers of its own.  The arguments arrive in blocks of up to sixteen registers;
// a value used inside a loop keeps its whole block alive, and when scalar registers run short the block is spilled and
// reloaded as a whole for it.  The copy ends the block's life here.
__device__ __forceinline__ int own_sgpr(int v) {
  int r;
  asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "s"(v));
  return r;
}
__device__ __forceinline__ int64_t own_sgpr(int64_t v) {
  int64_t r;
  asm volatile("s_mov_b64 %0, %1" : "=s"(r) : "s"(v));
  return r;
}

}  // namespace dkv
