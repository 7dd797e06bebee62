// Host-side launch entry points of the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "common.h"

namespace dkv {

hipError_t launch_fwd(const AttnParams& p, int head_dim, hipStream_t st);
// tuned forward for head dims 64 / 128
hipError_t launch_fwd2(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_dq(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_dkdv(const AttnParams& p, int head_dim, hipStream_t st);
// tuned backward kernels for head dims 64 / 128
hipError_t launch_dq2(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_dkdv4(const AttnParams& p, int head_dim, hipStream_t st);
// tuned kernels for head dim 256 (forward, dQ: 128 rows per workgroup; dK/dV: 64-key tile)
hipError_t launch_fwd256(const AttnParams& p, hipStream_t st);
hipError_t launch_dq256(const AttnParams& p, hipStream_t st);
hipError_t launch_dkdv256(const AttnParams& p, hipStream_t st);
// tuned dK/dV kernel for head dim 512 (32-key tile, 16-row blocks)
hipError_t launch_dkdv512(const AttnParams& p, hipStream_t st);
// tuned dQ kernel for head dim 512 (64 rows per workgroup, 16-key tiles)
hipError_t launch_dq512(const AttnParams& p, hipStream_t st);
hipError_t launch_fwd512(const AttnParams& p, hipStream_t st);
// key tile (rows of K/V owned by one workgroup) of the dK/dV kernel for a head dim
int dkdv_key_tile(int head_dim);

hipError_t launch_dot_do_o(const TView& dout, const TView& o, const float* lse, float* dvec, float* lse2, int total,
                           int H, int head_dim, hipStream_t st);
hipError_t launch_group_offsets(const int32_t* grp, int n_groups, int total_ctx, int32_t* cu, hipStream_t st);
hipError_t launch_expand_groups(const int32_t* grp, int n_groups, int n_seqs, int32_t* seq_ctx, hipStream_t st);
hipError_t launch_fill_f32(float* ptr, int64_t n, float value, hipStream_t st);
hipError_t launch_convert_ctx(const float* acc, const TViewOut& out, int P, int Hk, int head_dim, float mul,
                              hipStream_t st);
hipError_t launch_rows_copy(bool to_packed, int n_seqs, int ctx_len, int total_resp, const int32_t* cu,
                            int64_t row_bytes, const void* src, void* dst, int32_t* pos_ids, hipStream_t st);
hipError_t launch_label_map(int n_seqs, int ctx_len, int total_resp, const int32_t* cu, int32_t* next_index,
                            int32_t* first_token_index, hipStream_t st);

// Raises the dynamic-LDS limit of a kernel instantiation once per process (a host API call; not repeated on
// every launch, so that nothing but kernel launches is issued on a stream under capture after the first use).
template <auto Kern>
inline hipError_t ensure_dynamic_lds(size_t bytes) {
  static hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  return once;
}

}  // namespace dkv
