// Internal launch interfaces between the C-ABI layer (api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace linattn {

// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per kernel and device instead of once per launch: the call
// costs host time that a call made of a dozen short launches cannot hide.  `done` is the call site's own mask of the
// devices that have been served (a site names one kernel instantiation).
inline hipError_t set_max_lds_once(const void* kern, int bytes, std::atomic<uint64_t>& done) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t(1) << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
  return e;
}
#define LINATTN_MAX_LDS_ONCE(kern, bytes)                                             \
  ([&]() -> hipError_t {                                                              \
    static std::atomic<uint64_t> done_{0};                                            \
    return ::linattn::set_max_lds_once(reinterpret_cast<const void*>(kern), (bytes), done_); \
  }())

struct VerifyArgs {
  const void* q;
  const void* k;
  const void* v;            // [B,H,kk,d] dense, i/o dtype
  const float* conv_w;      // [H,d,Kc]
  float* S;                 // [B,H,d,d] in/out
  float* z;                 // [B,H,d]   in/out
  void* hist;               // [B,H,Kc-1,d] in/out, i/o dtype
  const int32_t* n_commit;  // device [B] or null
  void* out;                // [B,H,kk,d]
  int B, H, kk, Kc;
  float eps;
  int relu;                 // feature map: 0 = elu + 1, 1 = max(x, 0)
  int dv;                   // width of the value rows (v, out, hist, the rows of S, conv_w): a multiple of d
};

struct VerifyTreeArgs {
  const void* q;
  const void* k;
  const void* v;            // [B,H,n,d] dense, i/o dtype
  const float* conv_w;      // [H,d,Kc]
  float* S;                 // [B,H,d,d] in/out
  float* z;                 // [B,H,d]   in/out
  void* hist;               // [B,H,Kc-1,d] in/out, i/o dtype
  const int32_t* parent;    // device [n]
  const int32_t* accept;    // device [B] or null
  void* out;                // [B,H,n,d]
  int B, H, n, Kc;
  float eps;
  int relu;
};

struct VerifyGroupedArgs {
  const void* q;
  const void* k;
  const void* v;            // [B,H,kk,d] dense, i/o dtype
  const float* conv_w;      // [H,d,Kc]
  float* S;                 // [B,H,d,d] in/out: completed groups only
  float* z;                 // [B,H,d]   in/out
  void* hist;               // [B,H,Kc-1,d] in/out, i/o dtype
  void* kwin;               // [B,H,64,d] in/out, i/o dtype: raw key rows of the open group
  void* vwin;               // [B,H,64,d] in/out: its value rows
  int32_t* fill;            // device [B,H] in/out: rows of the open group in use, 0..63 (equal over the heads of a row)
  const int32_t* n_commit;  // device [B] or null
  void* out;                // [B,H,kk,d]
  int B, H, kk, Kc;
  float eps, alpha;
  int relu;
};

struct PrefillArgs {
  const void* q;
  const void* k;
  const void* v;            // [B,H,L,d] by strides
  const float* conv_w;      // [H,d,Kc]
  const float* S_in;        // null = zeros
  const float* z_in;
  const void* hist_in;
  void* out;
  float* S_out;             // null = not wanted
  float* z_out;
  void* hist_out;
  float* ws;                // [B*H][nseg][d*d + d] floats (segment start states), then staged history rows
  int B, H, L, Kc;
  float eps;
  int relu;                 // feature map: 0 = elu + 1, 1 = max(x, 0)
  float alpha;              // three-branch form only: weight of the grouped linear branch
  int64_t sb, sh, st;       // element strides of q, k, v, out
  int nseg;                 // workgroups along the sequence axis per (b, h)
  int seg_len;              // tokens per segment (multiple of the chunk size)
  int wait_spins;           // polls before a wait between the waves of a workgroup gives up; < 0: give up at once
  int no_conv;              // the taps are taken as zero: a convolution with more than 8 taps runs as a pass of its own
  int group;                // three-branch form: tokens per group (64 or 256)
  // Value rows wider than key rows: d_v = m d.  The kernels then see B*H*m heads of d value channels each, head
  // (b, h, block) sharing q, k, z with its siblings and owning channels block*d .. block*d + d - 1 of v, out, hist,
  // conv_w and of the rows of S.  m = 1: nothing changes.
  int m;
  int64_t sb_v, sh_v, st_v; // element strides of v and out
};

// (b, h, value block) of a prefill workgroup and what follows from it
struct HeadIndex {
  int bhs;                  // index over B*H*m: workspace slots
  int bh;                   // index over B*H: q, k, z
  int b, h, blk;
  int dvt;                  // m * d: row length of v, out, hist, S
};
__device__ __forceinline__ HeadIndex head_index(const PrefillArgs& a, int bhs, int d) {
  HeadIndex x;
  x.bhs = bhs; x.bh = bhs / a.m; x.blk = bhs % a.m;
  x.b = x.bh / a.H; x.h = x.bh % a.H; x.dvt = a.m * d;
  return x;
}


struct ConvLongArgs {
  const void* v;            // [B,H,L,d] by strides
  const float* conv_w;      // [H,d,Kc]
  const void* hist_in;      // [B,H,Kc-1,d] or null
  void* out;                // [B,H,L,d] by strides: out += conv
  void* hist_out;           // [B,H,Kc-1,d] or null; may be hist_in
  int B, H, L, Kc;
  int64_t sb, sh, st;       // strides of v and out
  int m;                    // value blocks of d channels per head (d_v = m d)
  int rev;                  // the token axis runs backwards (out[t] += sum_j w[j] v[t + j]): the conv's share of the
                            // gradient with respect to its input; no history then
  int hist_fused;           // set by the launcher: the conv kernel writes hist_out itself (no launch of its own)
  int assign;               // out = conv instead of out += conv (bf16 rows only): the pass then runs ahead of the
                            // kernel that adds the rest, and needs nothing from it
};

// Gradient of the three-branch form for a sequence that starts from nothing (training): bf16 rows, one set of strides
struct GroupedBwdArgs {
  const void* q; const void* k; const void* v;   // [B,H,L,d] by strides
  const void* dout;         // gradient with respect to the outputs, same layout
  void* dq; void* dk; void* dv;                  // same layout
  const float* conv_w;      // [H,d,Kc]
  float* dconv_w;           // [H,d,Kc], summed over the batch rows; null = not wanted
  float* P;                 // [B*H][ng][d*d + d]: the sums before every group
  float* Dg;                // [B*H][ng][d*d + d]: what a group's queries add to the gradient of the sums before it; after
                            // the suffix sum: the gradient with respect to the sums after the group
  float* stats;             // [5][B*H*L]: per token, largest logit (log2 units), 1 / sum of weights, pbar, alpha / den, d den
  float* dw_part;           // [H][B*nwb][d*Kc]: conv-weight gradient of one block of tokens; as much again behind it
                            // for the stages of the sum over them
  int B, H, L, Kc;
  float eps;
  int relu;
  float alpha;
  int64_t sb, sh, st;
  int group, ng;            // tokens per group (64 or 256), groups per sequence
  int nwb;                  // token blocks of the conv-weight pass per sequence
};

// verify.hip
int verify_pick_split(int BH);
hipError_t launch_verify(const VerifyArgs& a, bool bf16, int d, int nsplit, hipStream_t st);
hipError_t launch_verify_z(const VerifyArgs& a, bool bf16, int d, hipStream_t st);   // z += accepted phi(k), all heads

// verify_mfma.hip : the same step as one 16-token group on the matrix cores (bf16 drafts, whole heads)
bool verify_mfma_available(bool bf16, int d, int nsplit, int kk);
hipError_t launch_verify_mfma(const VerifyArgs& a, int d, hipStream_t st);

// verify_grouped.hip : generation with the three-branch form (state of the completed groups + the open group's rows)
hipError_t launch_verify_grouped(const VerifyGroupedArgs& a, bool bf16, int d, hipStream_t st);

// verify_grouped_mfma.hip : the same step on the matrix cores (bf16 drafts, four or more of them)
bool verify_grouped_mfma_available(bool bf16, int d, int kk);
hipError_t launch_verify_grouped_mfma(const VerifyGroupedArgs& a, int d, hipStream_t st);

// verify_tree.hip : candidates arranged as a tree, scored from one read of the state
hipError_t launch_verify_tree(const VerifyTreeArgs& a, int d, hipStream_t st);
// verify_tree_simt.hip : the same for fp32 candidates, exact fp32 multiply-adds on the vector ALUs
hipError_t launch_verify_tree_simt(const VerifyTreeArgs& a, int d, hipStream_t st);

// prefill_simt.hip : fp32 arithmetic on the vector ALUs, one workgroup per (b, h)
hipError_t launch_prefill_simt(const PrefillArgs& a, bool bf16, int d, hipStream_t st);
// ... and the three-branch form (a.group tokens per group, a.alpha): fp32 rows, and any rows in groups of 256
bool prefill_grouped_simt_available(bool bf16, int d, int group);
hipError_t launch_prefill_grouped_simt(const PrefillArgs& a, bool bf16, int d, hipStream_t st);

// conv_long.hip : out += causal depthwise conv with 9..63 taps, and the history that goes with it
hipError_t launch_conv_long(const ConvLongArgs& a, bool bf16, int d, hipStream_t st);

// prefill_grouped_bwd.hip : gradient of the three-branch form (bf16 rows, groups of 64 or 256)
int grouped_bwd_dw_blocks(int L);
// ... in two parts that need nothing from each other: everything but the conv-weight sums (dv is added to what it
// holds: the conv's share is written first; `before_dkdv`, if not null, is waited for ahead of the kernel that does
// so), and the conv-weight sums
hipError_t launch_grouped_bwd_core(const GroupedBwdArgs& a, int d, hipStream_t st, hipEvent_t before_dkdv);
hipError_t launch_grouped_bwd_dw(const GroupedBwdArgs& a, int d, hipStream_t st);

// prefill_mfma.hip : launch plan of the bf16 prefill (segments, prefix sum over segment states)
hipError_t launch_segment_scan(const PrefillArgs& a, int d, hipStream_t st);   // the prefix sum alone
int prefill_mfma_pick_segments(int BH, int L, int chunk, int d);
size_t prefill_mfma_workspace_bytes(int BH, int d, int nseg);
hipError_t launch_prefill_mfma(const PrefillArgs& a, int d, int chunk, bool grouped, hipStream_t st);

// prefill_grouped256.hip : the three-branch form in groups of 256 tokens on the matrix cores (bf16 rows); one
// workspace slot per (b, h, segment) also without segments
int prefill_grouped256_pick_segments(int BH, int L);
size_t prefill_grouped256_workspace_bytes(int BH, int d, int nseg);
hipError_t launch_prefill_grouped256(const PrefillArgs& a, int d, hipStream_t st);

// prefill_mfma_ws.hip : the matrix-core kernel, with front-end waves (HBM traffic, feature map, scores)
// and state waves (everything that touches S and z) working side by side
hipError_t launch_prefill_mfma_ws(const PrefillArgs& a, int d, bool state_only, bool grouped, hipStream_t st);

}  // namespace linattn
