/*
 * linattn.h -- C ABI of the MI355X (gfx950) library for causal kernelised
 * linear attention fused with a causal depthwise convolution on V.
 *
 * The operation (per batch row b and head h, independently):
 *
 *   Phi_q = phi(Q), Phi_k = phi(K), phi(x) = elu(x) + 1 (or max(x, 0), see linattn_phi), elementwise.
 *   Y_t   = ( Phi_q[t]^T S_t ) / ( Phi_q[t] . z_t + eps )
 *   S_t   = S_in + sum_{i<=t} Phi_k[i] V[i]^T      (d x d)
 *   z_t   = z_in + sum_{i<=t} Phi_k[i]             (d)
 *   U_t[c]= sum_{j<Kc} conv_w[h][c][j] * Vext[t-j][c]
 *   out_t = Y_t + U_t
 *
 * Sec. 3 ("Linear Attentions") of the paper gives the factorisation
 * Sim(Q,K) ~ phi(Q) phi(K)^T and its re-association phi(Q)(phi(K)^T V);
 * Sec. 4.1 gives the causal form (query t meets the cumulative sum over
 * i <= t of the key/value products), the partition of the sequence into
 * groups with group-level cumulative sums between them (here: `chunk`), and
 * the causally masked depthwise convolution on the V branch; Sec. 4.2 gives
 * speculative verification, where several draft tokens are scored in one call
 * and each may see the verified past and earlier drafts only, the convolution
 * window of draft j being the verified history followed by drafts <= j.
 * The row normaliser z, eps, and out = Y + U are this library's reading where
 * the paper leaves them open.
 *
 * linattn_prefill_grouped / linattn_verify_grouped compute the block in the
 * other form that Sec. 4.1 describes (group-level sums only in the linear
 * branch, softmax attention inside each group, the same convolution); see
 * their declarations.
 *
 * Vext is V extended to the left by `hist` (the last Kc-1 value rows seen so
 * far, oldest first), or by zeros at the start of a sequence.  Tap j of the
 * convolution multiplies the value row j positions back (j = 0: the current
 * token).  No output for token t depends on any token after t.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers, 16-byte aligned.  The descriptor
 *     and the scalar arguments are host values.  `n_commit` is a device pointer.
 *   - The caller owns every buffer.  The library allocates no device memory,
 *     keeps no state between calls (linattn_set_wait_limit apart) and may be
 *     called from several host threads.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without waiting for it.
 *   - The return value reports argument validation and launch errors only.
 *     Validation happens before anything is enqueued: on any error other than
 *     LINATTN_ERR_HIP nothing has been launched and no buffer was touched.
 *   - q, k, v, out are addressed as  base + b*stride_b + h*stride_h +
 *     t*stride_t + c  (element units; the last axis, length d, is contiguous;
 *     every stride is a multiple of 8 elements).  The same strides apply to all
 *     four.  State tensors are dense: S [B,H,d,d] float (row = key feature i,
 *     column = value channel c, c contiguous), z [B,H,d] float,
 *     hist [B,H,Kc-1,d] in the i/o dtype, conv_w [H,d,Kc] float.  (With value
 *     rows wider than key rows -- linattn_desc.d_v -- every "d" that counts
 *     value channels reads d_v, and v, out take strides of their own.)
 *   - Buffers must not overlap except where an alias is explicitly allowed.
 */
#ifndef LINATTN_H
#define LINATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LINATTN_OK = 0,
  LINATTN_ERR_NULL = 1,        /* a required pointer is NULL                          */
  LINATTN_ERR_SHAPE = 2,       /* B, H, L, k, d, conv_k, chunk or a stride is invalid  */
  LINATTN_ERR_DTYPE = 3,       /* unknown io_dtype or phi                              */
  LINATTN_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                     */
  LINATTN_ERR_UNSUPPORTED = 5, /* valid request this build has no kernel for           */
  LINATTN_ERR_WORKSPACE = 6,   /* workspace missing or smaller than required           */
  LINATTN_ERR_HIP = 7          /* the HIP runtime refused a launch                     */
} linattn_status;

typedef enum { LINATTN_F32 = 0, LINATTN_BF16 = 1 } linattn_dtype;
/* Feature map on Q and K (Sec. 3: "kernel embeddings").  ELU1: phi(x) = elu(x) + 1, the default of
 * every workload here.  RELU: phi(x) = max(x, 0), the ReLU linear attention the paper lists among the
 * existing ones (Sec. 3, "Comprehensive Evaluation"); its denominator can vanish, so pass eps > 0. */
typedef enum { LINATTN_PHI_ELU1 = 0, LINATTN_PHI_RELU = 1 } linattn_phi;

#define LINATTN_MAX_CONV_K 8   /* taps t, t-1, ..., t-Kc+1: verify, decode, tree            */
#define LINATTN_MAX_CONV_K_PREFILL 63  /* ... and of the prefill entry points (Sec. 4.1: the
                                  FLASH experiment uses a masked DWConv of kernel size 63) */
#define LINATTN_MAX_DRAFT 16   /* draft tokens per verify call                          */
#define LINATTN_MAX_TREE 64    /* candidate tokens per tree-verify call                 */
#define LINATTN_MAX_DV 2048    /* widest value row (a multiple of d)                       */

typedef struct {
  int32_t B, H;            /* batch rows, heads                                        */
  int32_t d;               /* head dimension d_k = d_v: 64 or 128                       */
  int32_t conv_k;          /* Kc, 1..LINATTN_MAX_CONV_K; the prefill entry points take
                              up to LINATTN_MAX_CONV_K_PREFILL (kernels of more than 8
                              taps run as a pass of their own behind the attention)     */
  int32_t chunk;           /* tokens per group in prefill: 64, 128 or 256 (ignored by
                              verify/decode).  The result of linattn_prefill does not
                              depend on it; that of the three-branch form does.         */
  int32_t io_dtype;        /* linattn_dtype of q, k, v, out, hist                       */
  int32_t phi;             /* linattn_phi                                               */
  float eps;               /* added to every denominator; >= 0                          */
  int64_t stride_b, stride_h, stride_t; /* element strides of q, k, v, out: multiples of
                              8, stride_t >= d and <= 2^22                           */
  /* Value rows wider than key rows (Sec. 3, Eq. 1: Q, K of width d_k, V of width d_v).  */
  int32_t d_v;             /* 0 or d: d_v = d_k = d.  Otherwise a multiple of d, at most
                              LINATTN_MAX_DV: v, out and hist rows have d_v elements,
                              S is [B,H,d,d_v], conv_w [H,d_v,Kc]; q, k, z keep d.
                              linattn_prefill, _noalloc, linattn_verify and
                              linattn_decode only (LINATTN_ERR_UNSUPPORTED elsewhere);
                              z_out must then not be z_in in the prefill calls.        */
  int32_t reserved;        /* 0                                                        */
  int64_t stride_b_v, stride_h_v, stride_t_v; /* element strides of v and out when
                              d_v differs from d (q and k keep stride_b/h/t); all 0
                              when d_v is 0 or d: v and out then share q's strides     */
} linattn_desc;

/* Bytes of device scratch `linattn_prefill` needs for this descriptor and L
 * (0 if none).  Depends on B, H, d and on how the sequence axis is split over
 * workgroups, never on L beyond that split: it is bounded by a constant for
 * fixed B, H, d.  Returns 0 for an invalid descriptor. */
size_t linattn_workspace_bytes(const linattn_desc *desc, int32_t L);

/* Prefill (Sec. 4.1): all L tokens of every (b, h) at once, processed in
 * groups of `chunk` tokens; inside a group the masked phi(Q)phi(K)^T V product,
 * between groups the running (S, z) carry.
 *   q, k, v      in   [B,H,L,d] by strides, i/o dtype
 *   conv_w       in   [H,d,Kc] float
 *   S_in, z_in, hist_in   in, optional: all three NULL = start of a sequence
 *                (zeros), or all three given = continue from that state
 *   out          out  [B,H,L,d] by strides, i/o dtype
 *   S_out, z_out, hist_out  out, optional (each may be NULL = not wanted);
 *                each may alias its *_in counterpart
 *   workspace    device scratch of at least linattn_workspace_bytes(desc, L)
 *                bytes (may be NULL when that is 0); contents are undefined
 *                before and after
 * L >= 0; L need not be a multiple of chunk.  L == 0 copies the state through. */
linattn_status linattn_prefill(const linattn_desc *desc, int32_t L,
                               const void *q, const void *k, const void *v,
                               const float *conv_w,
                               const float *S_in, const float *z_in, const void *hist_in,
                               void *out,
                               float *S_out, float *z_out, void *hist_out,
                               void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* linattn_prefill for callers that cannot allocate or pass device scratch (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments minus the workspace, same kernels, same
 * results bit for bit.  The scratch of a segmented prefill lives in a static device array inside the library,
 * linattn_noalloc_scratch_bytes() = 17 432 576 bytes, which every GPU the library runs on holds until the
 * process ends; that is enough for every descriptor linattn_prefill accepts (LINATTN_ERR_WORKSPACE if a request
 * ever needed more).  The call allocates and frees nothing; its first use on a device asks the runtime once for the
 * array's address there (with that device current, which is also the device `hip_stream` must belong to).
 * All calls on one GPU share the one array: two such calls that overlap in time on the same GPU (different
 * streams, or a captured graph replayed concurrently with itself) race; calls in stream order are safe, and
 * nothing in the array needs to be cleared between calls. */
linattn_status linattn_prefill_noalloc(const linattn_desc *desc, int32_t L,
                                       const void *q, const void *k, const void *v,
                                       const float *conv_w,
                                       const float *S_in, const float *z_in, const void *hist_in,
                                       void *out,
                                       float *S_out, float *z_out, void *hist_out,
                                       void *hip_stream);

/* Size in bytes of the static device scratch behind linattn_prefill_noalloc. */
size_t linattn_noalloc_scratch_bytes(void);

/* Prefill in the three-branch form of Sec. 4.1 (the text around the figure of the
 * augmented attention): the sequence is cut into consecutive groups of `chunk`
 * tokens, counted from the first token of the call, and every token gets
 *   alpha * phi(q)^T S / (phi(q).z + eps)    with S, z as they stood BEFORE the
 *                                            token's group (grouped linear attention:
 *                                            the sums advance once per group; a
 *                                            denominator of exactly 0 gives 0)
 * + causal softmax attention over the tokens of its own group, logits
 *   q.k / sqrt(d) on the raw rows (local attention)
 * + the masked depthwise convolution of V, as in linattn_prefill.
 * Unlike linattn_prefill the result depends on the group size.  Arguments,
 * layouts, state handling, workspace and L as for linattn_prefill (same
 * linattn_workspace_bytes); the state handed back is the same running sum.  To
 * continue a sequence with the same grouping, cut it at multiples of `chunk`.
 *   alpha        finite (LINATTN_ERR_SHAPE otherwise)
 * chunk must be 64 (the paper's group size for LLaMA) or 256 (its group size for
 * FLASH, Sec. 5 "Settings"); LINATTN_ERR_UNSUPPORTED otherwise, and for fp32 rows
 * of 128 elements in groups of 256.  bf16 rows run on the matrix cores (groups of
 * 256 keep their running state in the workspace, which they need for every L > 0);
 * fp32 rows on a plain fp32 kernel that is exact to fp32 rounding but not built
 * for speed (one workgroup per (b, h), no workspace). */
linattn_status linattn_prefill_grouped(const linattn_desc *desc, int32_t L, float alpha,
                                       const void *q, const void *k, const void *v,
                                       const float *conv_w,
                                       const float *S_in, const float *z_in, const void *hist_in,
                                       void *out,
                                       float *S_out, float *z_out, void *hist_out,
                                       void *workspace, size_t workspace_bytes,
                                       void *hip_stream);

/* Gradient of linattn_prefill_grouped (Sec. 5.3: the paper times a training step,
 * forward and backward, of FLASH with this block in groups of 256 tokens), for a
 * sequence that starts from nothing (no incoming state or history: training).
 * With out = linattn_prefill_grouped(q, k, v, conv_w) and dout = d loss / d out, it
 * writes the derivatives of the loss with respect to q, k, v and the conv weights:
 *   grouped branch   through phi(q)^T S / (phi(q).z + eps) into the queries, and
 *                    through the group-level sums S, z into every key and value
 *                    of the earlier groups (phi'(x) = 1 for x > 0, else exp(x); for
 *                    the map max(x, 0): 1 for x > 0, else 0);
 *   local branch     the gradient of causal softmax attention inside each group;
 *   conv             dv[s] += sum_j conv_w[h][c][j] dout[s+j], and
 *                    dconv_w[h][c][j] = sum over batch rows and tokens of
 *                    dout[b,h,t,c] * v[b,h,t-j,c].
 *   desc         in      as for the forward call; bf16 rows, d_v = d, chunk 64 or
 *                        256 (LINATTN_ERR_UNSUPPORTED otherwise); conv_k <= 63
 *   L            in      tokens per sequence, any L >= 0
 *   q, k, v, dout in     device, bf16, addressed by the descriptor's strides
 *   conv_w       in      device float [H,d,Kc]
 *   dq, dk, dv   out     device, bf16, same strides; must not alias the inputs
 *   dconv_w      out     device float [H,d,Kc], written (not added to); NULL = not wanted
 *   workspace    scratch device, >= linattn_backward_workspace_bytes(desc, L), 16-byte
 *                        aligned: the sums before every group and the gradients with
 *                        respect to them ((d*d+d) floats per group and head, twice),
 *                        five floats per token and head, and the partial conv-weight
 *                        sums.  Contents on entry are ignored.
 * Arithmetic: bf16 operands on the matrix cores, fp32 accumulation; the conv's
 * share of dv is rounded to bf16 before the rest is added to it (a second rounding).
 * The result does not depend on the launch configuration (no atomics: fixed
 * summation order).
 * Asynchronous on hip_stream; every argument is validated before anything is
 * enqueued.  Part of the work (the conv's share of dv, the conv-weight sums) runs on
 * a second stream that the library creates at the first such call of a host thread
 * on a device (default priority; it is forked from hip_stream and joined back into
 * it with events inside the call, so work enqueued on hip_stream after the call
 * sees all of the call's results, and a graph capture of hip_stream captures all of
 * it).  If hip_stream is being captured at that first call, or the stream cannot be
 * made, everything runs on hip_stream. */
size_t linattn_backward_workspace_bytes(const linattn_desc *desc, int32_t L);

linattn_status linattn_prefill_grouped_backward(const linattn_desc *desc, int32_t L, float alpha,
                                                const void *q, const void *k, const void *v,
                                                const float *conv_w, const void *dout,
                                                void *dq, void *dk, void *dv, float *dconv_w,
                                                void *workspace, size_t workspace_bytes,
                                                void *hip_stream);

/* Speculative verification (Sec. 4.2): scores kk draft tokens per (b, h) from
 * one running state.  Output j equals what kk single decode steps would give
 * at step j.  Afterwards the state has advanced over the first n_commit[b]
 * drafts of batch row b (the accepted ones); n_commit == NULL keeps all kk;
 * n_commit[b] == 0 leaves that row's state bit-unchanged.
 *   q, k, v      in      [B,H,kk,d] dense, i/o dtype (desc strides are ignored)
 *   conv_w       in      [H,d,Kc] float
 *   S, z, hist   in/out  updated in place (hist may be NULL only if Kc == 1)
 *   n_commit     in      device int32 [B], each in 0..kk, or NULL.  Values
 *                        outside 0..kk are clamped into that range.
 *   out          out     [B,H,kk,d] dense, i/o dtype
 * 1 <= kk <= LINATTN_MAX_DRAFT. */
linattn_status linattn_verify(const linattn_desc *desc, int32_t kk,
                              const void *q, const void *k, const void *v,
                              const float *conv_w,
                              float *S, float *z, void *hist,
                              const int32_t *n_commit,
                              void *out, void *hip_stream);

/* Generation with the three-branch form (the block of linattn_prefill_grouped in the
 * decode phase of Sec. 3; kk > 1: the verification step of Sec. 4.2): kk draft
 * tokens per (b, h), each scored as linattn_prefill_grouped would score it at
 * the end of the sequence so far.  The state between calls is
 *   S, z         in/out  sums over the COMPLETED groups of `chunk` tokens only
 *   hist         in/out  last Kc-1 value rows (may be NULL only if Kc == 1)
 *   kwin, vwin   in/out  [B,H,chunk,d] dense, i/o dtype: raw key / value rows of
 *                        the open group; rows 0 .. fill[b][h]-1 are in use, the
 *                        rest is neither read nor (unless a kept draft lands
 *                        there) written
 *   fill         in/out  device int32 [B,H], rows of the open group in use,
 *                        0 .. chunk-1 (values outside are clamped into it); the
 *                        heads of a batch row carry equal values -- one count per
 *                        head so that each is read and advanced by one owner
 * A new sequence starts from zeros with fill = 0; after linattn_prefill_grouped
 * over a multiple of `chunk` tokens its S, z, hist are this state with fill = 0
 * (a remainder of the prompt goes through this call).  Afterwards the state has
 * advanced over the first n_commit[b] drafts (NULL: all kk; 0: bit-unchanged);
 * when they fill the group, its rows enter S and z and the next group opens.
 *   q, k, v, out [B,H,kk,d] dense, i/o dtype; conv_w [H,d,Kc] float
 *   n_commit     device int32 [B] or NULL, clamped into 0..kk
 * 1 <= kk <= LINATTN_MAX_DRAFT; chunk must be 64 (LINATTN_ERR_UNSUPPORTED
 * otherwise); fp32 and bf16 rows.  Arithmetic is fp32 throughout. */
linattn_status linattn_verify_grouped(const linattn_desc *desc, int32_t kk, float alpha,
                                      const void *q, const void *k, const void *v,
                                      const float *conv_w,
                                      float *S, float *z, void *hist,
                                      void *kwin, void *vwin, int32_t *fill,
                                      const int32_t *n_commit,
                                      void *out, void *hip_stream);

/* Tree-structured speculative verification (Sec. 4.2, "Proposed Solution": the
 * candidates of a speculation step follow Medusa's tree-based attention
 * pattern; Sec. 5.3 / Tab. 9 use 64 speculated tokens).  n candidate tokens per
 * (b, h) hang off the verified sequence as a tree: parent[i] < i is the
 * candidate that precedes candidate i in time, -1 if candidate i follows the
 * verified sequence directly.  Candidate i is scored from the verified state
 * and the candidates on its own root path (its ancestors and itself), never
 * from a sibling or another branch, and its convolution window is that path
 * read backwards, continuing into the verified history; output i is what
 * linattn_verify would give for the last token of that path.  A common prefix
 * of several candidates is computed once and the state is read once for all
 * of them.  Afterwards the state of batch row b has advanced over the root
 * path of candidate accept[b], oldest token first.
 *   q, k, v      in      [B,H,n,d] dense, i/o dtype (desc strides are ignored)
 *   parent       in      device int32 [n], shared by all (b, h); an entry outside
 *                        -1..i-1 is read as -1
 *   conv_w       in      [H,d,Kc] float
 *   S, z, hist   in/out  updated in place (hist may be NULL only if Kc == 1)
 *   accept       in      device int32 [B] or NULL; -1, NULL or an entry outside
 *                        0..n-1 accepts nothing and leaves that row's state
 *                        bit-unchanged
 *   out          out     [B,H,n,d] dense, i/o dtype
 * 1 <= n <= LINATTN_MAX_TREE.  bf16 candidates run on the matrix cores (bf16
 * operands, fp32 accumulation), fp32 candidates in exact fp32 multiply-adds on the
 * vector ALUs; d_v = d only (LINATTN_ERR_UNSUPPORTED otherwise). */
linattn_status linattn_verify_tree(const linattn_desc *desc, int32_t n,
                                   const void *q, const void *k, const void *v,
                                   const int32_t *parent,
                                   const float *conv_w,
                                   float *S, float *z, void *hist,
                                   const int32_t *accept,
                                   void *out, void *hip_stream);

/* One generated token per (b, h) (Sec. 3, decode phase; Sec. 4.1 recurrence):
 * linattn_verify with kk = 1 whose draft is always kept.
 *   q, k, v, out  [B,H,d] dense (equivalently [B,H,1,d]). */
linattn_status linattn_decode(const linattn_desc *desc,
                              const void *q, const void *k, const void *v,
                              const float *conv_w,
                              float *S, float *z, void *hist,
                              void *out, void *hip_stream);

/* What happens when the kernels' own synchronisation fails.  The waves of a bf16 prefill workgroup hand each
 * other data through LDS and wait for one another with bounded polling, so that a logic error or an extreme
 * slowdown cannot hang the GPU.  A wait that gives up does not go unnoticed: from then on every output row
 * that workgroup stores, and the S_out and z_out it hands back, are NaN (never finite numbers computed from
 * operands that were not ready).  The call itself still returns LINATTN_OK, since it returned before the
 * kernel ran; callers that must know check their outputs for NaN.
 * linattn_set_wait_limit sets the number of polls (about 64 clock cycles each) after which a wait gives up,
 * for all later prefill calls of this process, and returns the previous value.  spins == 0 restores the
 * default (2^20); spins < 0 makes every wait give up without looking, which is how the tests reach the NaN
 * path with kernels that still run to their end.  The only setting the library keeps; thread-safe. */
int32_t linattn_set_wait_limit(int32_t spins);

/* Static, NUL-terminated description of a status code (never NULL). */
const char *linattn_status_string(linattn_status status);

/* Library version as major*10000 + minor*100 + patch. */
int32_t linattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LINATTN_H */
