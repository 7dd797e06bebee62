// C ABI of the library (include/dualkv.h): host-side validation, workspace carving and dispatch.
// Nothing here touches device memory except through kernel launches on the caller's stream.
#include <cstdlib>
#include <mutex>
#include "../../include/dualkv.h"

#include "common.h"
#include "launch.h"

// Scratch of dualkv_bwd_noalloc (see static_scratch below).  Host code never passes this name to a kernel.
static __device__ __align__(256) unsigned char scratch[DUALKV_STATIC_SCRATCH_BYTES];

namespace {

using dkv::AttnParams;
using dkv::TView;
using dkv::TViewOut;

constexpr int kTargetBlocks = 512;   // prompt-tile workgroups wanted before the sequence loop is split

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_shape(const dualkv_shape* s, bool ctx_call) {
  if (s == nullptr) return DUALKV_E_INVALID;
  if (s->ctx_len < 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0) return DUALKV_E_INVALID;
  if (s->n_q_heads % s->n_kv_heads != 0) return DUALKV_E_INVALID;
  if (!ctx_call) {
    if (s->n_seqs < 1 || s->total_resp < 0 || s->max_resp < 0 || s->max_resp > s->total_resp) return DUALKV_E_INVALID;
    if (s->total_resp > 0 && s->max_resp == 0) return DUALKV_E_INVALID;
  }
  const int d = s->head_dim;
  if (d != 64 && d != 96 && d != 128 && d != 192 && d != 256 && d != 512) return DUALKV_E_UNSUPPORTED;
  if (s->window > 0 && d == 512) return DUALKV_E_UNSUPPORTED;
  // the backward statistics (D, then LSE in base-2 units) are two (H, rows) fp32 arrays carved from one workspace;
  // the d = 64 / 128 dK/dV kernel addresses the second as the first plus a 32-bit byte offset
  const int64_t rows = ctx_call ? s->ctx_len : s->total_resp;
  if ((d == 64 || d == 128) && rows * s->n_q_heads >= (int64_t(1) << 30) - 64) return DUALKV_E_UNSUPPORTED;
  return DUALKV_OK;
}

int check_view(const void* ptr, int64_t ts, int64_t hs, int64_t rows, int d) {
  if (rows == 0) return DUALKV_OK;
  if (ptr == nullptr) return DUALKV_E_INVALID;
  if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return DUALKV_E_ALIGN;
  if (ts % 8 != 0 || hs % 8 != 0) return DUALKV_E_ALIGN;
  if (ts < d || hs < d) return DUALKV_E_INVALID;
  if (ts > DUALKV_MAX_TOK_STRIDE) return DUALKV_E_UNSUPPORTED;   // the kernels form row offsets in 32 bits
  return DUALKV_OK;
}
int check_in(const dualkv_tin& t, int64_t rows, int d) { return check_view(t.ptr, t.tok_stride, t.head_stride, rows, d); }
int check_out(const dualkv_tout& t, int64_t rows, int d) { return check_view(t.ptr, t.tok_stride, t.head_stride, rows, d); }

TView view(const dualkv_tin& t) { return TView{static_cast<const dkv::u16*>(t.ptr), t.tok_stride, t.head_stride}; }
TViewOut view(const dualkv_tout& t) { return TViewOut{static_cast<dkv::u16*>(t.ptr), t.tok_stride, t.head_stride}; }

int check_cu_host(const dualkv_shape* s, const int32_t* cu) {
  if (cu == nullptr) return DUALKV_OK;
  if (cu[0] != 0) return DUALKV_E_INVALID;
  int mx = 0;
  for (int i = 0; i < s->n_seqs; ++i) {
    const int r = cu[i + 1] - cu[i];
    if (r < 0) return DUALKV_E_INVALID;
    if (r > mx) mx = r;
  }
  if (cu[s->n_seqs] != s->total_resp) return DUALKV_E_INVALID;
  if (mx > s->max_resp) return DUALKV_E_INVALID;
  return DUALKV_OK;
}

float resolve_scale(const dualkv_shape* s) {
  return s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
}

// Several prompt groups in one call (n == 0: the single group of the plain entry points).
struct Groups {
  int n = 0;
  const dualkv_group* dev = nullptr;
  const dualkv_group* host = nullptr;
  int total_ctx = 0;   // rows of the packed prompt tensors = sum of the prompt lengths
};

// rows of the prompt-side tensors (k_c, v_c and their gradients)
int64_t ctx_rows(const dualkv_shape* s, const Groups& g) { return g.n > 0 ? g.total_ctx : s->ctx_len; }

int check_groups(const dualkv_shape* s, const Groups& g) {
  if (g.n == 0) return DUALKV_OK;
  if (g.n < 0 || g.total_ctx < 0 || g.dev == nullptr) return DUALKV_E_INVALID;
  if (reinterpret_cast<uintptr_t>(g.dev) % 16) return DUALKV_E_ALIGN;
  if (g.host == nullptr) return DUALKV_OK;
  // the sequences of the groups partition [0, n_seqs) in order; every prompt lies inside the packed prompt tensors
  int next = 0;
  for (int i = 0; i < g.n; ++i) {
    const dualkv_group& x = g.host[i];
    if (x.seq_begin != next || x.seq_end < x.seq_begin) return DUALKV_E_INVALID;
    next = x.seq_end;
    if (x.ctx_len < 0 || x.ctx_len > s->ctx_len || x.ctx_offset < 0 ||
        (int64_t)x.ctx_offset + x.ctx_len > g.total_ctx)
      return DUALKV_E_INVALID;
  }
  return next == s->n_seqs ? DUALKV_OK : DUALKV_E_INVALID;
}

// number of parts the sequence loop of a prompt-tile workgroup is cut into
int ctx_split(const dualkv_shape* s, const Groups& g = Groups()) {
  if (s->ctx_len == 0) return 1;
  const int bn = dkv::dkdv_key_tile(s->head_dim);
  const int n_grp = g.n > 0 ? g.n : 1;
  const int64_t blocks = (int64_t)n_grp * ((s->ctx_len + bn - 1) / bn) * s->n_kv_heads;
  if (blocks >= kTargetBlocks) return 1;
  int64_t want = (kTargetBlocks + blocks - 1) / blocks;
  const int64_t seqs_per_group = (s->n_seqs + n_grp - 1) / n_grp;
  if (want > seqs_per_group) want = seqs_per_group;
  return (int)(want < 1 ? 1 : want);
}

struct BwdWorkspace {
  size_t dvec_off, dvec_bytes, lse2_off, acc_off, acc_bytes, seqctx_off, seqctx_bytes, total;
};

BwdWorkspace bwd_workspace(const dualkv_shape* s, bool ctx_call, const Groups& g = Groups()) {
  BwdWorkspace w{};
  const int64_t rows = ctx_call ? ctx_rows(s, g) : s->total_resp;
  w.dvec_off = 0;
  w.dvec_bytes = align_up((size_t)rows * s->n_q_heads * sizeof(float), 256);
  w.lse2_off = w.dvec_bytes;
  w.acc_off = 2 * w.dvec_bytes;
  w.acc_bytes = 0;
  if (!ctx_call && !(s->flags & DUALKV_FLAG_ACCUM_CTX_F32) && ctx_split(s, g) > 1)
    w.acc_bytes = align_up((size_t)ctx_rows(s, g) * s->n_kv_heads * s->head_dim * sizeof(float), 256);
  w.seqctx_off = w.acc_off + 2 * w.acc_bytes;
  w.seqctx_bytes = (!ctx_call && g.n > 0) ? align_up((size_t)s->n_seqs * 2 * sizeof(int32_t), 256) : 0;
  w.total = w.seqctx_off + w.seqctx_bytes;
  return w;
}

// per-sequence {first prompt row, prompt length} in the workspace, and the group fields of the kernel parameters
int bind_groups(AttnParams& p, const Groups& g, int n_seqs, void* seqctx, hipStream_t st) {
  if (g.n == 0) return DUALKV_OK;
  p.grp = reinterpret_cast<const int32_t*>(g.dev);
  p.n_groups = g.n;
  p.seq_ctx = static_cast<const int32_t*>(seqctx);
  return dkv::launch_expand_groups(p.grp, g.n, n_seqs, static_cast<int32_t*>(seqctx), st) == hipSuccess ? DUALKV_OK
                                                                                                         : DUALKV_E_HIP;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? DUALKV_OK : DUALKV_E_HIP; }

hipError_t run_fwd(const AttnParams& p, int d, hipStream_t st) {
  if (d == 64 || d == 128) return dkv::launch_fwd2(p, d, st);
  if (d == 256) return dkv::launch_fwd256(p, st);
  if (d == 512) return dkv::launch_fwd512(p, st);
  return dkv::launch_fwd(p, d, st);
}
hipError_t run_dq(const AttnParams& p, int d, hipStream_t st) {
  if (d == 64 || d == 128) return dkv::launch_dq2(p, d, st);
  if (d == 256) return dkv::launch_dq256(p, st);
  if (d == 512) return dkv::launch_dq512(p, st);
  return dkv::launch_dq(p, d, st);
}
hipError_t run_dkdv(const AttnParams& p, int d, hipStream_t st) {
  if (d == 64 || d == 128) return dkv::launch_dkdv4(p, d, st);
  if (d == 256) return dkv::launch_dkdv256(p, st);
  if (d == 512) return dkv::launch_dkdv512(p, st);
  return dkv::launch_dkdv(p, d, st);
}

void base_params(AttnParams& p, const dualkv_shape* s) {
  p = AttnParams{};
  p.H = s->n_q_heads;
  p.Hk = s->n_kv_heads;
  p.G = s->n_q_heads / s->n_kv_heads;
  p.window = s->window > 0 ? s->window : 0;
  p.scale = resolve_scale(s);
  p.scale_log2 = p.scale * dkv::LOG2E;
  p.n_split = 1;
}


// Prompt offsets of the Call-1 kernels with several groups: the prompts are packed back to back in group order, so
// the (n + 1) offsets are the groups' first rows followed by the total; written into the workspace by a tiny kernel.
int bind_ctx_groups(AttnParams& p, const dualkv_shape* shape, const Groups& g, void* cu_ws, hipStream_t st) {
  p.cu = nullptr;
  p.n_seqs = 1;
  p.ctx_len = 0;
  p.total = shape->ctx_len;
  p.max_rows = shape->ctx_len;
  if (g.n == 0) return DUALKV_OK;
  if (g.host != nullptr) {
    int64_t off = 0;
    for (int i = 0; i < g.n; ++i) {
      if (g.host[i].ctx_offset != off) return DUALKV_E_INVALID;   // not packed back to back
      off += g.host[i].ctx_len;
    }
    if (off != g.total_ctx) return DUALKV_E_INVALID;
  }
  if (dkv::launch_group_offsets(reinterpret_cast<const int32_t*>(g.dev), g.n, g.total_ctx, static_cast<int32_t*>(cu_ws),
                                st) != hipSuccess)
    return DUALKV_E_HIP;
  p.cu = static_cast<const int32_t*>(cu_ws);
  p.n_seqs = g.n;
  p.total = g.total_ctx;
  return DUALKV_OK;
}

int ctx_fwd_impl(const dualkv_shape* shape, dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c, dualkv_tout o_c,
                 float* lse_c, void* workspace, size_t workspace_bytes, void* stream, const Groups& groups) {
  int rc = check_shape(shape, true);
  if (rc != DUALKV_OK) return rc;
  if ((rc = check_groups(shape, groups))) return rc;
  const int d = shape->head_dim;
  const int P = (int)ctx_rows(shape, groups);
  if (P == 0) return DUALKV_OK;
  if ((rc = check_in(q_c, P, d)) || (rc = check_in(k_c, P, d)) || (rc = check_in(v_c, P, d)) ||
      (rc = check_out(o_c, P, d)))
    return rc;
  if (lse_c == nullptr) return DUALKV_E_INVALID;
  const size_t cu_bytes = groups.n > 0 ? align_up((size_t)(groups.n + 1) * sizeof(int32_t), 256) : 0;
  if (cu_bytes > 0 && (workspace == nullptr || workspace_bytes < cu_bytes)) return DUALKV_E_WORKSPACE;
  if (cu_bytes > 0 && reinterpret_cast<uintptr_t>(workspace) % 16) return DUALKV_E_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  AttnParams p;
  base_params(p, shape);
  p.q = view(q_c);
  p.kd = view(k_c);
  p.vd = view(v_c);
  p.kc = p.kd;   // unused (ctx_len = 0)
  p.vc = p.vd;
  p.out_o = view(o_c);
  p.lse = lse_c;
  if ((rc = bind_ctx_groups(p, shape, groups, workspace, st))) return rc;
  return hip_rc(run_fwd(p, d, st));
}

int fwd_impl(const dualkv_shape* shape, dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d,
             dualkv_tin v_d, const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host, dualkv_tout o_d,
             float* lse_d, void* workspace, size_t workspace_bytes, void* stream, const Groups& groups) {
  int rc = check_shape(shape, false);
  if (rc != DUALKV_OK) return rc;
  if ((rc = check_cu_host(shape, cu_seqlens_host))) return rc;
  if ((rc = check_groups(shape, groups))) return rc;
  const int T = shape->total_resp, d = shape->head_dim;
  const int P = (int)ctx_rows(shape, groups);
  if (T == 0) return DUALKV_OK;
  if (cu_seqlens_dev == nullptr || lse_d == nullptr) return DUALKV_E_INVALID;
  if ((rc = check_in(q_d, T, d)) || (rc = check_in(k_c, P, d)) || (rc = check_in(v_c, P, d)) ||
      (rc = check_in(k_d, T, d)) || (rc = check_in(v_d, T, d)) || (rc = check_out(o_d, T, d)))
    return rc;
  const size_t seqctx_bytes = groups.n > 0 ? align_up((size_t)shape->n_seqs * 2 * sizeof(int32_t), 256) : 0;
  if (seqctx_bytes > 0 && (workspace == nullptr || workspace_bytes < seqctx_bytes)) return DUALKV_E_WORKSPACE;
  if (seqctx_bytes > 0 && reinterpret_cast<uintptr_t>(workspace) % 16) return DUALKV_E_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  AttnParams p;
  base_params(p, shape);
  p.q = view(q_d);
  p.kc = view(k_c);
  p.vc = view(v_c);
  p.kd = view(k_d);
  p.vd = view(v_d);
  p.out_o = view(o_d);
  p.lse = lse_d;
  p.cu = cu_seqlens_dev;
  p.n_seqs = shape->n_seqs;
  p.ctx_len = shape->ctx_len;
  p.total = T;
  p.max_rows = shape->max_resp;
  if ((rc = bind_groups(p, groups, shape->n_seqs, workspace, st))) return rc;
  return hip_rc(run_fwd(p, d, st));
}

int ctx_bwd_impl(const dualkv_shape* shape, dualkv_tin do_c, dualkv_tin o_c, const float* lse_c, dualkv_tin q_c,
                   dualkv_tin k_c, dualkv_tin v_c, dualkv_tout dq_c, dualkv_tout dk_c, dualkv_tout dv_c,
                   float* dk_c_acc32, float* dv_c_acc32, void* workspace, size_t workspace_bytes, void* stream,
                 const Groups& groups) {
  int rc = check_shape(shape, true);
  if (rc != DUALKV_OK) return rc;
  if ((rc = check_groups(shape, groups))) return rc;
  const int d = shape->head_dim;
  const int P = (int)ctx_rows(shape, groups);
  if (P == 0) return DUALKV_OK;
  const bool accum = (shape->flags & DUALKV_FLAG_ACCUM_CTX_F32) != 0;
  if ((rc = check_in(do_c, P, d)) || (rc = check_in(o_c, P, d)) || (rc = check_in(q_c, P, d)) ||
      (rc = check_in(k_c, P, d)) || (rc = check_in(v_c, P, d)) || (rc = check_out(dq_c, P, d)))
    return rc;
  if (lse_c == nullptr) return DUALKV_E_INVALID;
  if (accum) {
    if (dk_c_acc32 == nullptr || dv_c_acc32 == nullptr) return DUALKV_E_INVALID;
    if ((reinterpret_cast<uintptr_t>(dk_c_acc32) | reinterpret_cast<uintptr_t>(dv_c_acc32)) % 16) return DUALKV_E_ALIGN;
  } else if ((rc = check_out(dk_c, P, d)) || (rc = check_out(dv_c, P, d))) {
    return rc;
  }
  const BwdWorkspace w = bwd_workspace(shape, true, groups);
  const size_t cu_bytes = groups.n > 0 ? align_up((size_t)(groups.n + 1) * sizeof(int32_t), 256) : 0;
  if (workspace == nullptr || workspace_bytes < w.total + cu_bytes) return DUALKV_E_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 16) return DUALKV_E_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);

  AttnParams p;
  base_params(p, shape);
  p.q = view(q_c);
  p.kd = view(k_c);
  p.vd = view(v_c);
  p.kc = p.kd;
  p.vc = p.vd;
  p.o = view(o_c);
  p.dout = view(do_c);
  p.dq = view(dq_c);
  if (!accum) {
    p.dkd = view(dk_c);
    p.dvd = view(dv_c);
  } else {
    p.dkd_acc = dk_c_acc32;
    p.dvd_acc = dv_c_acc32;
  }
  p.lse = const_cast<float*>(lse_c);
  p.dvec = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.dvec_off);
  p.lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.lse2_off);
  if ((rc = bind_ctx_groups(p, shape, groups, static_cast<char*>(workspace) + w.total, st))) return rc;
  const bool do_dq = !(shape->flags & DUALKV_FLAG_SKIP_DQ), do_dkdv = !(shape->flags & DUALKV_FLAG_SKIP_DKDV);
  if (!(shape->flags & DUALKV_FLAG_SKIP_PRE) && (rc = hip_rc(dkv::launch_dot_do_o(p.dout, p.o, p.lse, p.dvec, p.lse2, P, p.H, d, st))))
    return rc;
  if (do_dkdv && (rc = hip_rc(run_dkdv(p, d, st)))) return rc;
  if (do_dq) return hip_rc(run_dq(p, d, st));
  return DUALKV_OK;
}


// ---- the Call-2 backward, shared by dualkv_bwd (caller's workspace) and dualkv_bwd_noalloc (static scratch)
int bwd_impl(const dualkv_shape* shape, dualkv_tin do_d, dualkv_tin o_d, const float* lse_d, dualkv_tin q_d,
               dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d, const int32_t* cu_seqlens_dev,
               const int32_t* cu_seqlens_host, dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d,
               dualkv_tout dv_d, float* dk_c_acc32, float* dv_c_acc32, void* workspace, size_t workspace_bytes,
               void* stream, const Groups& groups = Groups()) {
  int rc = check_shape(shape, false);
  if (rc != DUALKV_OK) return rc;
  if ((rc = check_cu_host(shape, cu_seqlens_host))) return rc;
  if ((rc = check_groups(shape, groups))) return rc;
  const int T = shape->total_resp, d = shape->head_dim;
  const int P = (int)ctx_rows(shape, groups);   // rows of the prompt-side tensors
  const bool accum = (shape->flags & DUALKV_FLAG_ACCUM_CTX_F32) != 0;
  if (T > 0) {
    if (cu_seqlens_dev == nullptr || lse_d == nullptr) return DUALKV_E_INVALID;
    if ((rc = check_in(do_d, T, d)) || (rc = check_in(o_d, T, d)) || (rc = check_in(q_d, T, d)) ||
        (rc = check_in(k_d, T, d)) || (rc = check_in(v_d, T, d)) || (rc = check_out(dq_d, T, d)) ||
        (rc = check_out(dk_d, T, d)) || (rc = check_out(dv_d, T, d)))
      return rc;
  }
  if ((rc = check_in(k_c, P, d)) || (rc = check_in(v_c, P, d))) return rc;
  if (accum) {
    if (P > 0 && (dk_c_acc32 == nullptr || dv_c_acc32 == nullptr)) return DUALKV_E_INVALID;
    if ((reinterpret_cast<uintptr_t>(dk_c_acc32) | reinterpret_cast<uintptr_t>(dv_c_acc32)) % 16) return DUALKV_E_ALIGN;
  } else if ((rc = check_out(dk_c, P, d)) || (rc = check_out(dv_c, P, d))) {
    return rc;
  }
  const BwdWorkspace w = bwd_workspace(shape, false, groups);
  if (w.total > 0 && (workspace == nullptr || workspace_bytes < w.total)) return DUALKV_E_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 16) return DUALKV_E_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t n_acc = (int64_t)P * shape->n_kv_heads * d;

  AttnParams p;
  base_params(p, shape);
  p.q = view(q_d);
  p.kc = view(k_c);
  p.vc = view(v_c);
  p.kd = view(k_d);
  p.vd = view(v_d);
  p.o = view(o_d);
  p.dout = view(do_d);
  p.dq = view(dq_d);
  p.dkd = view(dk_d);
  p.dvd = view(dv_d);
  p.lse = const_cast<float*>(lse_d);
  p.dvec = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.dvec_off);
  p.lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.lse2_off);
  p.cu = cu_seqlens_dev;
  p.n_seqs = shape->n_seqs;
  p.ctx_len = shape->ctx_len;
  p.total = T;
  p.max_rows = shape->max_resp;
  if ((rc = bind_groups(p, groups, shape->n_seqs, static_cast<char*>(workspace) + w.seqctx_off, st))) return rc;

  const bool scratch = !accum && w.acc_bytes > 0;
  if (accum) {
    p.dkc_acc = dk_c_acc32;
    p.dvc_acc = dv_c_acc32;
    p.n_split = ctx_split(shape, groups);
  } else if (scratch) {
    p.dkc_acc = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.acc_off);
    p.dvc_acc = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.acc_off + w.acc_bytes);
    p.n_split = ctx_split(shape, groups);
    // zero-initialise the fp32 scratch (Alg. 1, "Require: zero-initialized")
    if (!(shape->flags & DUALKV_FLAG_SKIP_DKDV)) {
      if ((rc = hip_rc(dkv::launch_fill_f32(p.dkc_acc, n_acc, 0.f, st)))) return rc;
      if ((rc = hip_rc(dkv::launch_fill_f32(p.dvc_acc, n_acc, 0.f, st)))) return rc;
    }
  } else {
    p.dkc = view(dk_c);
    p.dvc = view(dv_c);
  }
  const bool do_dq = !(shape->flags & DUALKV_FLAG_SKIP_DQ), do_dkdv = !(shape->flags & DUALKV_FLAG_SKIP_DKDV);
  if (T > 0 && !(shape->flags & DUALKV_FLAG_SKIP_PRE) &&
      (rc = hip_rc(dkv::launch_dot_do_o(p.dout, p.o, p.lse, p.dvec, p.lse2, T, p.H, d, st))))
    return rc;
  if (do_dkdv && (rc = hip_rc(run_dkdv(p, d, st)))) return rc;
  if (scratch && do_dkdv) {
    // Stage 2 (Alg. 2): cast the accumulated prompt gradients once
    if ((rc = hip_rc(dkv::launch_convert_ctx(p.dkc_acc, view(dk_c), P, p.Hk, d, 1.0f, st)))) return rc;
    if ((rc = hip_rc(dkv::launch_convert_ctx(p.dvc_acc, view(dv_c), P, p.Hk, d, 1.0f, st)))) return rc;
  }
  if (T > 0 && do_dq) return hip_rc(run_dq(p, d, st));
  return DUALKV_OK;
}


// ---- static scratch of dualkv_bwd_noalloc: one array per GPU the library is loaded on, held until the process
// ends.  The array's name is only a host-side handle: its device address is looked up once per device (with that
// device current) and only that address is ever handed to kernels.
constexpr size_t kStaticScratchBytes = DUALKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DUALKV_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return DUALKV_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DUALKV_OK;
}

}  // namespace

extern "C" {

int dualkv_version(void) { return 200; }

const char* dualkv_strerror(int code) {
  switch (code) {
    case DUALKV_OK: return "ok";
    case DUALKV_E_INVALID: return "invalid argument";
    case DUALKV_E_UNSUPPORTED: return "unsupported head_dim / window combination";
    case DUALKV_E_WORKSPACE: return "workspace missing or too small";
    case DUALKV_E_ALIGN: return "pointer not 16-byte aligned or stride not a multiple of 8 elements";
    case DUALKV_E_HIP: return "HIP runtime error";
    case DUALKV_E_SCRATCH: return "shape needs more than the library's static scratch (DUALKV_STATIC_SCRATCH_BYTES)";
  }
  return "unknown error";
}

int dualkv_workspace_bytes(const dualkv_shape* shape, int op, size_t* out_bytes) {
  if (out_bytes == nullptr) return DUALKV_E_INVALID;
  const bool ctx_call = (op == DUALKV_OP_CTX_FWD || op == DUALKV_OP_CTX_BWD);
  if (op < DUALKV_OP_CTX_FWD || op > DUALKV_OP_BWD) return DUALKV_E_INVALID;
  const int rc = check_shape(shape, ctx_call);
  if (rc != DUALKV_OK) return rc;
  if (op == DUALKV_OP_CTX_FWD || op == DUALKV_OP_FWD) {
    *out_bytes = 0;
    return DUALKV_OK;
  }
  *out_bytes = bwd_workspace(shape, ctx_call).total;
  return DUALKV_OK;
}

int dualkv_groups_workspace_bytes(const dualkv_shape* shape, int32_t n_groups, int32_t total_ctx, int op,
                                  size_t* out_bytes) {
  if (out_bytes == nullptr || n_groups < 1 || total_ctx < 0) return DUALKV_E_INVALID;
  if (op < DUALKV_OP_CTX_FWD || op > DUALKV_OP_BWD) return DUALKV_E_INVALID;
  const bool ctx_call = (op == DUALKV_OP_CTX_FWD || op == DUALKV_OP_CTX_BWD);
  const int rc = check_shape(shape, ctx_call);
  if (rc != DUALKV_OK) return rc;
  Groups g;
  g.n = n_groups;
  g.total_ctx = total_ctx;
  const size_t cu_bytes = align_up((size_t)(n_groups + 1) * sizeof(int32_t), 256);   // prompt offsets of the ctx calls
  const size_t seqctx_bytes = align_up((size_t)shape->n_seqs * 2 * sizeof(int32_t), 256);
  switch (op) {
    case DUALKV_OP_CTX_FWD: *out_bytes = cu_bytes; break;
    case DUALKV_OP_FWD: *out_bytes = seqctx_bytes; break;
    case DUALKV_OP_CTX_BWD: *out_bytes = bwd_workspace(shape, true, g).total + cu_bytes; break;
    default: *out_bytes = bwd_workspace(shape, false, g).total; break;
  }
  return DUALKV_OK;
}

int dualkv_ctx_fwd(const dualkv_shape* shape, dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c, dualkv_tout o_c,
                   float* lse_c, void* workspace, size_t workspace_bytes, void* stream) {
  return ctx_fwd_impl(shape, q_c, k_c, v_c, o_c, lse_c, workspace, workspace_bytes, stream, Groups());
}

int dualkv_fwd(const dualkv_shape* shape, dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d,
               dualkv_tin v_d, const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host, dualkv_tout o_d,
               float* lse_d, void* workspace, size_t workspace_bytes, void* stream) {
  return fwd_impl(shape, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, o_d, lse_d, workspace,
                  workspace_bytes, stream, Groups());
}

int dualkv_ctx_bwd(const dualkv_shape* shape, dualkv_tin do_c, dualkv_tin o_c, const float* lse_c, dualkv_tin q_c,
                   dualkv_tin k_c, dualkv_tin v_c, dualkv_tout dq_c, dualkv_tout dk_c, dualkv_tout dv_c,
                   float* dk_c_acc32, float* dv_c_acc32, void* workspace, size_t workspace_bytes, void* stream) {
  return ctx_bwd_impl(shape, do_c, o_c, lse_c, q_c, k_c, v_c, dq_c, dk_c, dv_c, dk_c_acc32, dv_c_acc32, workspace,
                      workspace_bytes, stream, Groups());
}

int dualkv_bwd(const dualkv_shape* shape, dualkv_tin do_d, dualkv_tin o_d, const float* lse_d, dualkv_tin q_d,
               dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d, const int32_t* cu_seqlens_dev,
               const int32_t* cu_seqlens_host, dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d,
               dualkv_tout dv_d, float* dk_c_acc32, float* dv_c_acc32, void* workspace, size_t workspace_bytes,
               void* stream) {
  return bwd_impl(shape, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, dq_d, dk_c, dv_c,
                  dk_d, dv_d, dk_c_acc32, dv_c_acc32, workspace, workspace_bytes, stream);
}

int dualkv_bwd_noalloc(const dualkv_shape* shape, dualkv_tin do_d, dualkv_tin o_d, const float* lse_d, dualkv_tin q_d,
                       dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d, const int32_t* cu_seqlens_dev,
                       const int32_t* cu_seqlens_host, dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c,
                       dualkv_tout dk_d, dualkv_tout dv_d, float* dk_c_acc32, float* dv_c_acc32, void* stream) {
  int rc = check_shape(shape, false);
  if (rc != DUALKV_OK) return rc;
  if (bwd_workspace(shape, false).total > kStaticScratchBytes) return DUALKV_E_SCRATCH;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  return bwd_impl(shape, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, dq_d, dk_c, dv_c,
                  dk_d, dv_d, dk_c_acc32, dv_c_acc32, ws, kStaticScratchBytes, stream);
}

// ---- several prompt groups in one call (Sec. 2.2)
static Groups make_groups(int32_t n_groups, const dualkv_group* dev, const dualkv_group* host, int32_t total_ctx) {
  Groups g;
  g.n = n_groups;
  g.dev = dev;
  g.host = host;
  g.total_ctx = total_ctx;
  return g;
}

int dualkv_ctx_fwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                          const dualkv_group* groups_host, int32_t total_ctx, dualkv_tin q_c, dualkv_tin k_c,
                          dualkv_tin v_c, dualkv_tout o_c, float* lse_c, void* workspace, size_t workspace_bytes,
                          void* stream) {
  if (n_groups < 1) return DUALKV_E_INVALID;
  return ctx_fwd_impl(shape, q_c, k_c, v_c, o_c, lse_c, workspace, workspace_bytes, stream,
                      make_groups(n_groups, groups_dev, groups_host, total_ctx));
}

int dualkv_fwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                      const dualkv_group* groups_host, int32_t total_ctx, dualkv_tin q_d, dualkv_tin k_c,
                      dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d, const int32_t* cu_seqlens_dev,
                      const int32_t* cu_seqlens_host, dualkv_tout o_d, float* lse_d, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (n_groups < 1) return DUALKV_E_INVALID;
  return fwd_impl(shape, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, o_d, lse_d, workspace,
                  workspace_bytes, stream, make_groups(n_groups, groups_dev, groups_host, total_ctx));
}

int dualkv_ctx_bwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                          const dualkv_group* groups_host, int32_t total_ctx, dualkv_tin do_c, dualkv_tin o_c,
                          const float* lse_c, dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c, dualkv_tout dq_c,
                          dualkv_tout dk_c, dualkv_tout dv_c, float* dk_c_acc32, float* dv_c_acc32, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (n_groups < 1) return DUALKV_E_INVALID;
  return ctx_bwd_impl(shape, do_c, o_c, lse_c, q_c, k_c, v_c, dq_c, dk_c, dv_c, dk_c_acc32, dv_c_acc32, workspace,
                      workspace_bytes, stream, make_groups(n_groups, groups_dev, groups_host, total_ctx));
}

int dualkv_bwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                      const dualkv_group* groups_host, int32_t total_ctx, dualkv_tin do_d, dualkv_tin o_d,
                      const float* lse_d, dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d,
                      dualkv_tin v_d, const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host, dualkv_tout dq_d,
                      dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d, dualkv_tout dv_d, float* dk_c_acc32,
                      float* dv_c_acc32, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_groups < 1) return DUALKV_E_INVALID;
  return bwd_impl(shape, do_d, o_d, lse_d, q_d, k_c, v_c, k_d, v_d, cu_seqlens_dev, cu_seqlens_host, dq_d, dk_c, dv_c,
                  dk_d, dv_d, dk_c_acc32, dv_c_acc32, workspace, workspace_bytes, stream,
                  make_groups(n_groups, groups_dev, groups_host, total_ctx));
}

int dualkv_finalize_ctx_grads(const dualkv_shape* shape, const float* dk_c_acc32, const float* dv_c_acc32,
                              dualkv_tout dk_c, dualkv_tout dv_c, void* stream) {
  int rc = check_shape(shape, true);
  if (rc != DUALKV_OK) return rc;
  const int P = shape->ctx_len, d = shape->head_dim;
  if (P == 0) return DUALKV_OK;
  if (dk_c_acc32 == nullptr || dv_c_acc32 == nullptr) return DUALKV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(dk_c_acc32) | reinterpret_cast<uintptr_t>(dv_c_acc32)) % 16) return DUALKV_E_ALIGN;
  if ((rc = check_out(dk_c, P, d)) || (rc = check_out(dv_c, P, d))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = hip_rc(dkv::launch_convert_ctx(dk_c_acc32, view(dk_c), P, shape->n_kv_heads, d, 1.0f, st)))) return rc;
  return hip_rc(dkv::launch_convert_ctx(dv_c_acc32, view(dv_c), P, shape->n_kv_heads, d, 1.0f, st));
}

int dualkv_zero_ctx_grads(const dualkv_shape* shape, float* dk_c_acc32, float* dv_c_acc32, void* stream) {
  int rc = check_shape(shape, true);
  if (rc != DUALKV_OK) return rc;
  if (shape->ctx_len == 0) return DUALKV_OK;
  if (dk_c_acc32 == nullptr || dv_c_acc32 == nullptr) return DUALKV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(dk_c_acc32) | reinterpret_cast<uintptr_t>(dv_c_acc32)) % 16) return DUALKV_E_ALIGN;
  const int64_t n = (int64_t)shape->ctx_len * shape->n_kv_heads * shape->head_dim;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = hip_rc(dkv::launch_fill_f32(dk_c_acc32, n, 0.f, st)))) return rc;
  return hip_rc(dkv::launch_fill_f32(dv_c_acc32, n, 0.f, st));
}

static int rows_copy_common(bool to_packed, int32_t n_seqs, int32_t ctx_len, int32_t total_resp,
                            const int32_t* cu, int64_t row_bytes, const void* src, void* dst, int32_t* pos,
                            void* stream) {
  if (n_seqs < 1 || ctx_len < 0 || total_resp < 0 || row_bytes <= 0) return DUALKV_E_INVALID;
  if (row_bytes % 4 != 0) return DUALKV_E_ALIGN;
  if ((int64_t)ctx_len + total_resp == 0) return DUALKV_OK;
  if (cu == nullptr || src == nullptr || dst == nullptr) return DUALKV_E_INVALID;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) % 4) return DUALKV_E_ALIGN;
  return hip_rc(dkv::launch_rows_copy(to_packed, n_seqs, ctx_len, total_resp, cu, row_bytes, src, dst, pos,
                                      static_cast<hipStream_t>(stream)));
}

int dualkv_repack(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                  int64_t row_bytes, const void* standard, void* packed, int32_t* position_ids, void* stream) {
  return rows_copy_common(true, n_seqs, ctx_len, total_resp, cu_seqlens_dev, row_bytes, standard, packed,
                          position_ids, stream);
}

int dualkv_replicate(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                     int64_t row_bytes, const void* packed, void* standard, int32_t* position_ids, void* stream) {
  return rows_copy_common(false, n_seqs, ctx_len, total_resp, cu_seqlens_dev, row_bytes, packed, standard,
                          position_ids, stream);
}

int dualkv_label_map(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                     int32_t* next_index, int32_t* first_token_index, void* stream) {
  if (n_seqs < 1 || ctx_len < 0 || total_resp < 0 || cu_seqlens_dev == nullptr) return DUALKV_E_INVALID;
  if ((int64_t)ctx_len + total_resp > 0x7fffffff) return DUALKV_E_INVALID;
  return hip_rc(dkv::launch_label_map(n_seqs, ctx_len, total_resp, cu_seqlens_dev, next_index, first_token_index,
                                      static_cast<hipStream_t>(stream)));
}

}  // extern "C"
