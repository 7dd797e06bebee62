/*
 * dualkv.h -- C ABI of the MI355X (gfx950) shared-prompt attention library.
 *
 * The library evaluates exact softmax attention for a group of N responses that
 * share one P-token prompt, in the single-prompt packing [P | R_1 | ... | R_N]
 * (paper Eq. 5).  Attention is split in two calls (paper Sec. 2.2, "two-call
 * decomposition"):
 *
 *   Call 1  dualkv_ctx_fwd / dualkv_ctx_bwd   causal self-attention over the
 *           prompt alone (Eq. 3, App. A.3 "Call 1");
 *   Call 2  dualkv_fwd / dualkv_bwd           every response row r of sequence i
 *           attends to the shared prompt keys K_c (all visible) followed by its
 *           own response keys K_d^(i)[0..r] (causal at logical position P + r)
 *           (Eq. 4, App. A.3 "Call 2", Alg. 3; backward Alg. 1 + Alg. 2).
 *
 * General rules
 *   - Every tensor pointer is a DEVICE pointer.  Activations and gradients are
 *     bf16 (16-bit storage), LSE and the optional fp32 accumulators are fp32,
 *     cu_seqlens is int32.  The innermost (head_dim) axis is contiguous; the
 *     token and head strides are given in ELEMENTS, so the prompt / response
 *     halves of one packed QKV buffer can be passed as zero-copy views
 *     (App. A.3 "QKV split").  Base pointers must be 16-byte aligned and strides
 *     multiples of 8 elements.
 *   - The caller owns every buffer, including the workspace; the library never
 *     allocates device memory, keeps no mutable global state and never
 *     synchronises: all work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL is the default stream).  The enqueued work consists of kernel
 *     launches only (no memset or copy nodes), so the calls may be issued on a
 *     stream under capture.  Several prompt groups (Sec. 2.2) are either one call of
 *     the *_groups entry points, or one call sequence per group captured in a HIP graph.
 *   - Outputs are fully overwritten.  The only exception are the fp32
 *     accumulators in DUALKV_FLAG_ACCUM_CTX_F32 mode, which are added into.
 *   - Every entry point returns DUALKV_OK or a negative error code; arguments are
 *     validated on the host before anything is launched.  No exceptions, no abort.
 *   - Semantics fixed here: diagonal inclusive; GQA map kv_head = q_head / (H/H_k);
 *     LSE = natural log of sum_j exp(softmax_scale * q.k_j) over visible keys, laid
 *     out (H, rows); window W > 0 means row t sees keys j with t-W < j <= t in the
 *     logical position space (prompt positions 0..P-1, then P + r), App. F.
 */
#ifndef DUALKV_H_
#define DUALKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DUALKV_OK             0
#define DUALKV_E_INVALID     (-1)  /* NULL pointer, negative size, H % H_k != 0, bad cu_seqlens ... */
#define DUALKV_E_UNSUPPORTED (-2)  /* head_dim not in {64,96,128,192,256,512}; window with head_dim 512;
                                      tok_stride > DUALKV_MAX_TOK_STRIDE; rows * H >= 2^30 at head_dim 64/128 */
#define DUALKV_E_WORKSPACE   (-3)  /* workspace pointer NULL or smaller than dualkv_workspace_bytes  */
#define DUALKV_E_ALIGN       (-4)  /* pointer not 16-byte aligned or stride not a multiple of 8      */
#define DUALKV_E_HIP         (-5)  /* a HIP runtime call (launch) failed                             */
#define DUALKV_E_SCRATCH     (-6)  /* dualkv_bwd_noalloc: the shape needs more than DUALKV_STATIC_SCRATCH_BYTES */

#define DUALKV_OP_CTX_FWD 0
#define DUALKV_OP_CTX_BWD 1
#define DUALKV_OP_FWD     2
#define DUALKV_OP_BWD     3

/* dK_c / dV_c of this call are ADDED into caller-provided fp32 buffers (P, H_k, d), contiguous,
 * instead of being written as bf16; both backward calls may add into the same buffers so that the
 * Call-1 + Call-2 sum (Eq. 6; App. A.4, total gradient of the shared keys and values) is formed in fp32 and cast once by
 * dualkv_finalize_ctx_grads.  The caller zeroes the buffers before the first call. */
#define DUALKV_FLAG_ACCUM_CTX_F32 1u
/* Backward calls only: run a subset of the three backward stages (preprocess: D = rowsum(dO*O) and
 * LSE in base-2 units; dK/dV; dQ).  Outputs of a skipped stage are left untouched.  The dK/dV and dQ
 * stages read the preprocess results from the workspace, so DUALKV_FLAG_SKIP_PRE requires that an earlier call with the same inputs and the
 * same workspace has run the preprocess.  For callers that need only some gradients, and for timing
 * the stages separately. */
#define DUALKV_FLAG_SKIP_DQ   2u
#define DUALKV_FLAG_SKIP_DKDV 4u
#define DUALKV_FLAG_SKIP_PRE  8u

typedef struct dualkv_shape {
  int32_t n_seqs;        /* N >= 1 responses in the group (ignored by the ctx calls)            */
  int32_t ctx_len;       /* P >= 0 prompt tokens (context_seqlen); 0 => plain varlen causal     */
  int32_t total_resp;    /* sum_i R_i == cu_seqlens[N]                                          */
  int32_t max_resp;      /* max_i R_i                                                           */
  int32_t n_q_heads;     /* H                                                                   */
  int32_t n_kv_heads;    /* H_k, H % H_k == 0                                                   */
  int32_t head_dim;      /* d in {64, 96, 128, 192, 256, 512}                                   */
  int32_t window;        /* W > 0: sliding window of W keys incl. self; <= 0: none              */
  float   softmax_scale; /* <= 0 => 1/sqrt(d)                                                   */
  uint32_t flags;        /* DUALKV_FLAG_*                                                       */
} dualkv_shape;

/* A tensor view: device pointer (16-byte aligned) to element (token 0, head 0, 0) of a bf16 tensor whose head_dim
 * axis is contiguous; strides in ELEMENTS, multiples of 8 and >= head_dim.  tok_stride may not exceed
 * DUALKV_MAX_TOK_STRIDE (the kernels form the byte offset of a row inside a tile in 32 bits); larger strides are
 * rejected with DUALKV_E_UNSUPPORTED. */
#define DUALKV_MAX_TOK_STRIDE (1 << 22)
typedef struct dualkv_tin  { const void* ptr; int64_t tok_stride; int64_t head_stride; } dualkv_tin;
typedef struct dualkv_tout { void*       ptr; int64_t tok_stride; int64_t head_stride; } dualkv_tout;

/* Workspace (device bytes) an operation needs for `shape`; 0 is a valid answer. */
int dualkv_workspace_bytes(const dualkv_shape* shape, int op, size_t* out_bytes);

/* Call 1 forward (Eq. 3): O_c = causal softmax(Q_c K_c^T * scale) V_c over the P prompt tokens.
 * q_c, o_c: (P, H, d); k_c, v_c: (P, H_k, d); lse_c: (H, P) fp32 contiguous.
 * The window, if any, applies exactly as in Call 2 (windowed attention over the contiguous
 * sequence, App. F). */
int dualkv_ctx_fwd(const dualkv_shape* shape, dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c,
                   dualkv_tout o_c, float* lse_c, void* workspace, size_t workspace_bytes,
                   void* stream);

/* Call 1 backward (App. A.4 "Call 1 backward"): given dO_c (the upstream gradient of the prompt
 * rows, already aggregated over the N branches, App. A.5), O_c and LSE_c from dualkv_ctx_fwd,
 * returns dQ_c (P,H,d) and the Call-1 terms of dK_c, dV_c (P,H_k,d) as bf16, or adds the latter
 * into dk_c_acc32 / dv_c_acc32 (then dk_c / dv_c pointers are ignored) under
 * DUALKV_FLAG_ACCUM_CTX_F32. */
int dualkv_ctx_bwd(const dualkv_shape* shape, dualkv_tin do_c, dualkv_tin o_c, const float* lse_c,
                   dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c,
                   dualkv_tout dq_c, dualkv_tout dk_c, dualkv_tout dv_c,
                   float* dk_c_acc32, float* dv_c_acc32,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Call 2 forward (Eq. 4, Alg. 3): q_d, o_d: (total_resp, H, d); k_c, v_c: (P, H_k, d) stored ONCE;
 * k_d, v_d: (total_resp, H_k, d); cu_seqlens_dev: (N+1) int32 offsets of the responses in the packed
 * response tensors (one array serves q and k_d, App. E); lse_d: (H, total_resp) fp32.
 * cu_seqlens_host (optional, may be NULL): host copy of the same array, used only to validate it
 * (monotone, last == total_resp) before launch.  The device array itself cannot be checked without a
 * synchronisation: it must start at 0, be non-decreasing, end at total_resp and have no response longer than
 * max_resp; the kernels index the response tensors with it and do not test it. */
int dualkv_fwd(const dualkv_shape* shape, dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c,
               dualkv_tin k_d, dualkv_tin v_d,
               const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
               dualkv_tout o_d, float* lse_d, void* workspace, size_t workspace_bytes, void* stream);

/* Call 2 backward (Alg. 1 + Alg. 2; App. A.4 "Call 2 backward", the response-branch terms of dK_c and
 * dV_c): returns dQ_d (total_resp,H,d),
 * dK_d, dV_d (total_resp,H_k,d) and the Call-2 terms of dK_c, dV_c (P,H_k,d): the sum over all N
 * sequences and the H/H_k heads of each group, accumulated in fp32 and cast to bf16 once, or added
 * into dk_c_acc32 / dv_c_acc32 under DUALKV_FLAG_ACCUM_CTX_F32. */
int dualkv_bwd(const dualkv_shape* shape, dualkv_tin do_d, dualkv_tin o_d, const float* lse_d,
               dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d,
               const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
               dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d, dualkv_tout dv_d,
               float* dk_c_acc32, float* dv_c_acc32,
               void* workspace, size_t workspace_bytes, void* stream);

/* dualkv_bwd for callers that cannot allocate device memory and have no workspace to hand over: code under HIP
 * graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * error codes as dualkv_bwd, without the workspace pair: the scratch (D, LSE in base-2 units, and the fp32
 * accumulators of the split shared-prompt path) lives in a static device array of DUALKV_STATIC_SCRATCH_BYTES inside
 * the library, one per GPU the library is loaded on, held until the process ends.  The call allocates nothing and
 * frees nothing; its first use on a device looks the array's address up (make that first call outside a capture).
 * A shape whose dualkv_workspace_bytes(shape, DUALKV_OP_BWD) exceeds DUALKV_STATIC_SCRATCH_BYTES is rejected with
 * DUALKV_E_SCRATCH before anything is launched.  Every call on a GPU uses that GPU's one array: what must start
 * at zero is cleared by the call itself, but two calls that overlap in time on one GPU (different streams,
 * different threads) race -- serialise them.  The DUALKV_FLAG_SKIP_* flags work as in dualkv_bwd, provided no other
 * call used the scratch in between. */
#define DUALKV_STATIC_SCRATCH_BYTES (32u << 20)
int dualkv_bwd_noalloc(const dualkv_shape* shape, dualkv_tin do_d, dualkv_tin o_d, const float* lse_d,
                       dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d,
                       const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                       dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d, dualkv_tout dv_d,
                       float* dk_c_acc32, float* dv_c_acc32, void* stream);

/* fp32 -> bf16 cast of the accumulated shared-prompt gradients (Alg. 2), acc32: (P,H_k,d) contiguous. */
int dualkv_finalize_ctx_grads(const dualkv_shape* shape, const float* dk_c_acc32, const float* dv_c_acc32,
                              dualkv_tout dk_c, dualkv_tout dv_c, void* stream);

/* ---- Several prompt groups in one call (Sec. 2.2: a micro-batch holds the response groups of several prompts) ----
 *
 * All groups share H, H_k, head_dim, window and scale.  Packing: the prompts of the groups back to back in one set of
 * prompt tensors (q_c, k_c, v_c, ...: total_ctx = sum_g P_g rows), the responses of all groups back to back in one set
 * of response tensors with ONE cu_seqlens over all n_seqs sequences (sequences of group 0 first, then group 1, ...).
 * A group is {first prompt row, P_g, first sequence, end sequence}; P_g = 0 and groups without sequences are allowed.
 * In `shape`: n_seqs = all sequences, total_resp / max_resp over all of them, ctx_len = the LARGEST P_g (an upper bound
 * is enough; it sizes the launch).  groups_dev: device array of n_groups entries, 16-byte aligned; groups_host
 * (optional, may be NULL): host copy, used only to validate (sequence ranges partition [0, n_seqs) in order, prompts
 * inside [0, total_ctx) and, for the ctx calls, packed back to back in group order).  Layouts of the other arguments
 * as in the single-group calls with P replaced by total_ctx: lse_c is (H, total_ctx), dk_c / dv_c and the fp32
 * accumulators are (total_ctx, H_k, d).  Each call runs the kernels of its single-group counterpart once for all
 * groups (plus one tiny index kernel), instead of once per group.  Workspace: dualkv_groups_workspace_bytes (the forward calls need a small one too).
 * dualkv_zero_ctx_grads / dualkv_finalize_ctx_grads serve the accumulators of all groups when given a shape whose
 * ctx_len is total_ctx. */
typedef struct dualkv_group {
  int32_t ctx_offset;   /* first row of the group's prompt in the prompt tensors            */
  int32_t ctx_len;      /* P_g >= 0                                                          */
  int32_t seq_begin;    /* the group's sequences are [seq_begin, seq_end) of cu_seqlens      */
  int32_t seq_end;
} dualkv_group;

int dualkv_groups_workspace_bytes(const dualkv_shape* shape, int32_t n_groups, int32_t total_ctx, int op,
                                  size_t* out_bytes);
int dualkv_ctx_fwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                          const dualkv_group* groups_host, int32_t total_ctx,
                          dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c, dualkv_tout o_c, float* lse_c,
                          void* workspace, size_t workspace_bytes, void* stream);
int dualkv_fwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                      const dualkv_group* groups_host, int32_t total_ctx,
                      dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d,
                      const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                      dualkv_tout o_d, float* lse_d, void* workspace, size_t workspace_bytes, void* stream);
int dualkv_ctx_bwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                          const dualkv_group* groups_host, int32_t total_ctx,
                          dualkv_tin do_c, dualkv_tin o_c, const float* lse_c,
                          dualkv_tin q_c, dualkv_tin k_c, dualkv_tin v_c,
                          dualkv_tout dq_c, dualkv_tout dk_c, dualkv_tout dv_c,
                          float* dk_c_acc32, float* dv_c_acc32,
                          void* workspace, size_t workspace_bytes, void* stream);
int dualkv_bwd_groups(const dualkv_shape* shape, int32_t n_groups, const dualkv_group* groups_dev,
                      const dualkv_group* groups_host, int32_t total_ctx,
                      dualkv_tin do_d, dualkv_tin o_d, const float* lse_d,
                      dualkv_tin q_d, dualkv_tin k_c, dualkv_tin v_c, dualkv_tin k_d, dualkv_tin v_d,
                      const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                      dualkv_tout dq_d, dualkv_tout dk_c, dualkv_tout dv_c, dualkv_tout dk_d, dualkv_tout dv_d,
                      float* dk_c_acc32, float* dv_c_acc32,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Clears the fp32 accumulators of DUALKV_FLAG_ACCUM_CTX_F32 mode ((P, H_k, d) contiguous each) with a fill kernel on
 * `stream` (Alg. 1 "Require: zero-initialised accumulators"; no memset node, so it may be captured in a graph). */
int dualkv_zero_ctx_grads(const dualkv_shape* shape, float* dk_c_acc32, float* dv_c_acc32, void* stream);

/* Layout kernels (Eq. 1 <-> Eq. 5).  Rows are opaque records of row_bytes (multiple of 4) bytes.
 * Standard packing: sequence i occupies rows [i*P + cu[i], (i+1)*P + cu[i+1]) = prompt then response i.
 * Single-prompt packing: rows [0,P) prompt, row P + cu[i] + r = response i row r.
 * dualkv_repack    : standard -> single-prompt (the prompt is taken from sequence 0's copy).
 * dualkv_replicate : single-prompt -> standard (the prompt is written N times); used to build the
 *                    N-copy baseline input.
 * position_ids (optional, may be NULL): int32 logical position of every destination row
 * (prompt j -> j, response row r -> P + r; App. A.2 RoPE positions). */
int dualkv_repack(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                  int64_t row_bytes, const void* standard, void* packed, int32_t* position_ids,
                  void* stream);
int dualkv_replicate(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                     int64_t row_bytes, const void* packed, void* standard, int32_t* position_ids,
                     void* stream);

/* Next-token map of the single-prompt packing (Sec. 2.3, "shared prompt logits"; the rolled labels and other
 * per-token side tensors of the packed sequence are gathered with it).  Device outputs, either may be NULL:
 *   next_index        (P + total_resp) int32: packed row t predicts the token at packed row next_index[t];
 *                     -1 where it predicts nothing through this map (last prompt row, last row of a response).
 *                     Prompt rows and response rows shift by one inside their own segment.
 *   first_token_index (N) int32: the first token of response i sits at packed row P + cu[i] and is predicted
 *                     by the logits of the LAST PROMPT ROW P - 1, shared by all N responses; -1 for an empty
 *                     response or when there is no prompt.
 * Errors: DUALKV_E_INVALID for n_seqs < 1, negative sizes, a NULL cu_seqlens_dev or more than 2^31 - 1 rows. */
int dualkv_label_map(int32_t n_seqs, int32_t ctx_len, int32_t total_resp, const int32_t* cu_seqlens_dev,
                     int32_t* next_index, int32_t* first_token_index, void* stream);

const char* dualkv_strerror(int code);
int dualkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DUALKV_H_ */
