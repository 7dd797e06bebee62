// Bandwidth-bound helper kernels: D = rowsum(dO * O) (the "dot_do_o" preprocess of Alg. 1), fp32 fill,
// fp32 -> bf16 cast of the accumulated shared-prompt gradients (Alg. 2) and the layout gathers between
// the standard packing (Eq. 1) and the single-prompt packing (Eq. 5).
#include "common.h"
#include "launch.h"

namespace dkv {

// ---------------------------------------------------------------------------------------------
// D[h][row] = sum_d dO[row,h,d] * O[row,h,d].  One group of D/8 lanes per (row, head); each lane reads
// 16 bytes of dO and of O, so a wave reads whole contiguous rows.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void dot_do_o_kernel(TView dout, TView o, const float* __restrict__ lse,
                                                       float* __restrict__ dvec, float* __restrict__ lse2,
                                                       int total, int H) {
  // lanes per (row, head): D / 8 of them carry data, rounded up to a power of two for the butterfly (d = 96, 192)
  constexpr int LPR = D / 8 <= 8 ? 8 : D / 8 <= 16 ? 16 : D / 8 <= 32 ? 32 : 64;
  constexpr int RPB = 256 / LPR;      // (row, head) pairs per block
  const int tid = threadIdx.x;
  const int64_t pair = (int64_t)blockIdx.x * RPB + tid / LPR;
  const int sub = tid % LPR;
  float acc = 0.f;
  const bool ok = pair < (int64_t)total * H;
  const int64_t row = ok ? pair / H : 0;
  const int h = ok ? (int)(pair % H) : 0;
  if (ok && sub < D / 8) {
    const u32x4 a = *reinterpret_cast<const u32x4*>(dout.ptr + row * dout.ts + (int64_t)h * dout.hs + sub * 8);
    const u32x4 b = *reinterpret_cast<const u32x4*>(o.ptr + row * o.ts + (int64_t)h * o.hs + sub * 8);
    const uint32_t* aw = reinterpret_cast<const uint32_t*>(&a);
    const uint32_t* bw = reinterpret_cast<const uint32_t*>(&b);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc += bf16_lo(aw[i]) * bf16_lo(bw[i]) + bf16_hi(aw[i]) * bf16_hi(bw[i]);
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (ok && sub == 0) {
    dvec[(int64_t)h * total + row] = acc;
    lse2[(int64_t)h * total + row] = lse[(int64_t)h * total + row] * LOG2E;   // exponent offset in base-2 units
  }
}

hipError_t launch_dot_do_o(const TView& dout, const TView& o, const float* lse, float* dvec, float* lse2, int total,
                           int H, int head_dim, hipStream_t st) {
  const int64_t pairs = (int64_t)total * H;
  if (pairs == 0) return hipSuccess;
  const int lanes = head_dim / 8, lpr = lanes <= 8 ? 8 : lanes <= 16 ? 16 : lanes <= 32 ? 32 : 64, rpb = 256 / lpr;
  const unsigned grid = (unsigned)((pairs + rpb - 1) / rpb);
  switch (head_dim) {
    case 64:  hipLaunchKernelGGL(dot_do_o_kernel<64>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    case 96:  hipLaunchKernelGGL(dot_do_o_kernel<96>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    case 128: hipLaunchKernelGGL(dot_do_o_kernel<128>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    case 192: hipLaunchKernelGGL(dot_do_o_kernel<192>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    case 256: hipLaunchKernelGGL(dot_do_o_kernel<256>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    case 512: hipLaunchKernelGGL(dot_do_o_kernel<512>, dim3(grid), dim3(256), 0, st, dout, o, lse, dvec, lse2, total, H); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_f32_kernel(float* __restrict__ ptr, int64_t n, float value) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      f32x4 v = {value, value, value, value};
      *reinterpret_cast<f32x4*>(ptr + i) = v;
    } else {
      for (int64_t j = i; j < n; ++j) ptr[j] = value;
    }
  }
}

hipError_t launch_fill_f32(float* ptr, int64_t n, float value, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 1023) / 1024;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, ptr, n, value);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Several prompt groups in one launch: per-sequence {first prompt row, prompt length} from the group table
// {first prompt row, P_g, first sequence, end sequence}; one thread per (group, sequence slot).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void expand_groups_kernel(const int32_t* __restrict__ grp, int n_groups,
                                                            int32_t* __restrict__ seq_ctx) {
  const int g = blockIdx.y;
  if (g >= n_groups) return;
  const int s0 = grp[4 * g + 2], s1 = grp[4 * g + 3];
  for (int s = s0 + blockIdx.x * 256 + threadIdx.x; s < s1; s += gridDim.x * 256) {
    seq_ctx[2 * s] = grp[4 * g];
    seq_ctx[2 * s + 1] = grp[4 * g + 1];
  }
}

// prompt offsets (n + 1) of groups packed back to back: the groups' first rows, then the total
__global__ __launch_bounds__(256) void group_offsets_kernel(const int32_t* __restrict__ grp, int n_groups, int total_ctx,
                                                            int32_t* __restrict__ cu) {
  for (int g = blockIdx.x * 256 + threadIdx.x; g <= n_groups; g += gridDim.x * 256) cu[g] = g < n_groups ? grp[4 * g] : total_ctx;
}

hipError_t launch_group_offsets(const int32_t* grp, int n_groups, int total_ctx, int32_t* cu, hipStream_t st) {
  hipLaunchKernelGGL(group_offsets_kernel, dim3((unsigned)min(64, (n_groups + 256) / 256)), dim3(256), 0, st, grp, n_groups,
                     total_ctx, cu);
  return hipGetLastError();
}

hipError_t launch_expand_groups(const int32_t* grp, int n_groups, int n_seqs, int32_t* seq_ctx, hipStream_t st) {
  if (n_groups <= 0 || n_seqs <= 0) return hipSuccess;
  const int bx = min(64, (n_seqs + 255) / 256);
  hipLaunchKernelGGL(expand_groups_kernel, dim3((unsigned)bx, (unsigned)n_groups), dim3(256), 0, st, grp, n_groups,
                     seq_ctx);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// acc (P, Hk, D) fp32 contiguous -> out (P, Hk, D) bf16 strided, multiplied by `mul`
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void convert_ctx_kernel(const float* __restrict__ acc, TViewOut out, int64_t n8,
                                                          int Hk, int D, float mul) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  const int cpr = D / 8;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
    const int ch = (int)(i % cpr);
    const int64_t rh = i / cpr;
    const int h = (int)(rh % Hk);
    const int64_t row = rh / Hk;
    const f32x4 a = *reinterpret_cast<const f32x4*>(acc + i * 8);
    const f32x4 b = *reinterpret_cast<const f32x4*>(acc + i * 8 + 4);
    u32x4 w;
    w.x = pack2_bf16(a[0] * mul, a[1] * mul);
    w.y = pack2_bf16(a[2] * mul, a[3] * mul);
    w.z = pack2_bf16(b[0] * mul, b[1] * mul);
    w.w = pack2_bf16(b[2] * mul, b[3] * mul);
    *reinterpret_cast<u32x4*>(out.ptr + row * out.ts + (int64_t)h * out.hs + ch * 8) = w;
  }
}

hipError_t launch_convert_ctx(const float* acc, const TViewOut& out, int P, int Hk, int head_dim, float mul,
                              hipStream_t st) {
  const int64_t n8 = (int64_t)P * Hk * head_dim / 8;
  if (n8 == 0) return hipSuccess;
  int64_t blocks = (n8 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(convert_ctx_kernel, dim3((unsigned)blocks), dim3(256), 0, st, acc, out, n8, Hk, head_dim, mul);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Layout gathers.  Destination-row driven: one workgroup per destination row finds its source row
// (binary search in cu_seqlens) and copies row_bytes.
//   to_packed : dst = single-prompt packing, src = standard packing
//   !to_packed: dst = standard packing,      src = single-prompt packing
// ---------------------------------------------------------------------------------------------
template <typename VEC>
__global__ __launch_bounds__(256) void rows_copy_kernel(bool to_packed, int n_seqs, int P, int total_resp,
                                                        const int32_t* __restrict__ cu, int64_t row_vecs,
                                                        const VEC* __restrict__ src, VEC* __restrict__ dst,
                                                        int32_t* __restrict__ pos_ids) {
  const int64_t drow = blockIdx.x;
  int64_t srow;
  int pos;
  if (to_packed) {
    if (drow < P) {
      srow = drow;   // prompt copy of sequence 0 (cu[0] == 0)
      pos = (int)drow;
    } else {
      const int x = (int)(drow - P);   // packed response row
      int lo = 0, hi = n_seqs;         // find i with cu[i] <= x < cu[i+1]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= x) lo = mid; else hi = mid;
      }
      srow = (int64_t)(lo + 1) * P + x;
      pos = P + (x - cu[lo]);
    }
  } else {
    // standard row: sequence i starts at i*P + cu[i]
    int lo = 0, hi = n_seqs;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if ((int64_t)mid * P + cu[mid] <= drow) lo = mid; else hi = mid;
    }
    const int64_t off = drow - ((int64_t)lo * P + cu[lo]);
    pos = (int)off;
    srow = off < P ? off : (int64_t)P + cu[lo] + (off - P);
  }
  const VEC* s = src + srow * row_vecs;
  VEC* d = dst + drow * row_vecs;
  for (int64_t i = threadIdx.x; i < row_vecs; i += 256) d[i] = s[i];
  if (pos_ids != nullptr && threadIdx.x == 0) pos_ids[drow] = pos;
}

hipError_t launch_rows_copy(bool to_packed, int n_seqs, int ctx_len, int total_resp, const int32_t* cu,
                            int64_t row_bytes, const void* src, void* dst, int32_t* pos_ids, hipStream_t st) {
  const int64_t drows = to_packed ? (int64_t)ctx_len + total_resp : (int64_t)n_seqs * ctx_len + total_resp;
  if (drows == 0) return hipSuccess;
  const bool v16 = (row_bytes % 16 == 0) && (((uintptr_t)src | (uintptr_t)dst) % 16 == 0);
  if (v16) {
    hipLaunchKernelGGL(rows_copy_kernel<u32x4>, dim3((unsigned)drows), dim3(256), 0, st, to_packed, n_seqs, ctx_len,
                       total_resp, cu, row_bytes / 16, static_cast<const u32x4*>(src), static_cast<u32x4*>(dst),
                       pos_ids);
  } else {
    hipLaunchKernelGGL(rows_copy_kernel<uint32_t>, dim3((unsigned)drows), dim3(256), 0, st, to_packed, n_seqs, ctx_len,
                       total_resp, cu, row_bytes / 4, static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst),
                       pos_ids);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Next-token map of the single-prompt packing (Sec. 2.3 "shared prompt logits"): packed row t predicts the
// token at packed row next_index[t] (-1: nothing).  Prompt rows and response rows shift by one inside their own
// segment; the row of the last prompt token predicts the FIRST token of every response, which cannot be
// expressed per row: first_token_index[i] (row P + cu[i], or -1 for an empty response or P = 0) lists them, all
// read from row P - 1.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void label_map_kernel(int n_seqs, int P, int total_resp,
                                                        const int32_t* __restrict__ cu, int32_t* __restrict__ next_index,
                                                        int32_t* __restrict__ first_token_index) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t T = (int64_t)P + total_resp;
  if (next_index != nullptr && t < T) {
    int nxt;
    if (t < P) {
      nxt = t + 1 < P ? (int)(t + 1) : -1;
    } else {
      const int x = (int)(t - P);
      int lo = 0, hi = n_seqs;   // find i with cu[i] <= x < cu[i+1]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= x) lo = mid; else hi = mid;
      }
      nxt = x + 1 < cu[lo + 1] ? (int)(t + 1) : -1;
    }
    next_index[t] = nxt;
  }
  if (first_token_index != nullptr && t < n_seqs) {
    const int i = (int)t;
    first_token_index[i] = (P > 0 && cu[i + 1] > cu[i]) ? P + cu[i] : -1;
  }
}

hipError_t launch_label_map(int n_seqs, int ctx_len, int total_resp, const int32_t* cu, int32_t* next_index,
                            int32_t* first_token_index, hipStream_t st) {
  const int64_t n = max((int64_t)ctx_len + total_resp, (int64_t)n_seqs);
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(label_map_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n_seqs, ctx_len,
                     total_resp, cu, next_index, first_token_index);
  return hipGetLastError();
}

}  // namespace dkv
