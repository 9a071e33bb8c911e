// C ABI (include/linattn.h): argument validation, launch planning, dispatch.
// No device memory is allocated here.  What is kept between calls: the wait limit (linattn_set_wait_limit), the
// device address of the static scratch of linattn_prefill_noalloc, and the gradient's side stream with its events
// (one per host thread and device); no results, no buffers.
#include "../../include/linattn.h"

#include <hip/hip_runtime.h>

#include <atomic>

#include "kernels.h"
#include "mfma_util.h"

using namespace linattn;

namespace {

// Polls before a wait between the waves of a prefill workgroup gives up (linattn_set_wait_limit).
constexpr int32_t kDefaultWaitSpins = 1 << 20;
std::atomic<int32_t> g_wait_spins{kDefaultWaitSpins};

// Scratch of linattn_prefill_noalloc: the workspace of a segmented prefill, held by every GPU the library runs
// on until the process ends.  Sized for the largest workspace any descriptor can ask for: the launch plan never
// puts more than 256 (b, h, segment) slots of d*d + d floats on the chip, plus 8 staged history rows per (b, h)
// for fewer than 256 of those.
constexpr size_t kScratchBytes = 256 * (128 * 128 + 128) * sizeof(float) + 256 * HALO * 128 * sizeof(uint16_t);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for the symbol: the array's device address is asked for once per device
// (each GPU has its own copy at its own address) and kept here.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

hipError_t scratch_for_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the same answer from every thread that gets here first
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return hipSuccess;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// chunk: the group size takes part in the call; strides: q, k, v, out are addressed by the descriptor's strides
// (the verify entry points take dense tensors and ignore them).
// Value blocks of d channels per head: d_v = m d (m = 1 when d_v is 0 or d).
int value_blocks(const linattn_desc* d) { return d->d_v == 0 ? 1 : d->d_v / d->d; }

linattn_status check_desc(const linattn_desc* d, bool chunk, bool strides, int max_conv_k = LINATTN_MAX_CONV_K) {
  if (!d) return LINATTN_ERR_NULL;
  if (d->io_dtype != LINATTN_F32 && d->io_dtype != LINATTN_BF16) return LINATTN_ERR_DTYPE;
  if (d->phi != LINATTN_PHI_ELU1 && d->phi != LINATTN_PHI_RELU) return LINATTN_ERR_DTYPE;
  if (d->B < 1 || d->H < 1) return LINATTN_ERR_SHAPE;
  if ((int64_t)d->B * d->H > (int64_t)1 << 24) return LINATTN_ERR_SHAPE;
  if (d->d != 64 && d->d != 128) return LINATTN_ERR_SHAPE;
  if (d->conv_k < 1 || d->conv_k > max_conv_k) return LINATTN_ERR_SHAPE;
  if (!(d->eps >= 0.f)) return LINATTN_ERR_SHAPE;
  if (chunk && d->chunk != 64 && d->chunk != 128 && d->chunk != 256) return LINATTN_ERR_SHAPE;
  if (d->d_v < 0 || d->d_v > LINATTN_MAX_DV || d->d_v % d->d != 0 || d->reserved != 0) return LINATTN_ERR_SHAPE;
  const bool wide = d->d_v != 0 && d->d_v != d->d;
  if (strides) {
    if (d->stride_t < d->d || d->stride_h < 0 || d->stride_b < 0) return LINATTN_ERR_SHAPE;
    if ((d->stride_t | d->stride_h | d->stride_b) & 7) return LINATTN_ERR_SHAPE;
    if (d->stride_t > (int64_t)1 << 22) return LINATTN_ERR_SHAPE;   // the kernels index inside a group with 32 bits
    if (wide) {
      if (d->stride_t_v < d->d_v || d->stride_h_v < 0 || d->stride_b_v < 0) return LINATTN_ERR_SHAPE;
      if ((d->stride_t_v | d->stride_h_v | d->stride_b_v) & 7) return LINATTN_ERR_SHAPE;
      if (d->stride_t_v > (int64_t)1 << 22) return LINATTN_ERR_SHAPE;
    } else if (d->stride_t_v != 0 || d->stride_h_v != 0 || d->stride_b_v != 0) {
      return LINATTN_ERR_SHAPE;                                     // v and out share q's strides when d_v = d
    }
  }
  return LINATTN_OK;
}

struct PrefillPlan {
  bool mfma;
  int nseg, seg_len;
  size_t ws_bytes;
};

// How a prefill call is laid out on the chip.  fp32 inputs go to the vector-ALU
// kernel (exact fp32 products).  bf16 inputs go to the matrix-core kernel; when
// B*H alone cannot fill the 256 compute units the sequence axis is cut into
// segments whose start states come from a first pass over K, V and a scan.
PrefillPlan plan_prefill(const linattn_desc* d, int32_t L, bool grouped = false) {
  PrefillPlan p{};
  p.mfma = d->io_dtype == LINATTN_BF16;
  const bool g256 = p.mfma && grouped && d->chunk == 256;   // three-branch form in groups of 256: its own full pass
  p.nseg = 1;
  p.seg_len = L;
  const int heads = d->B * d->H * value_blocks(d);      // what the kernels see as heads: one per value block
  if (p.mfma && L > 0) {
    p.nseg = g256 ? prefill_grouped256_pick_segments(heads, L) : prefill_mfma_pick_segments(heads, L, d->chunk, d->d);
    const int chunks = (L + d->chunk - 1) / d->chunk;
    const int cps = (chunks + p.nseg - 1) / p.nseg;
    p.seg_len = cps * d->chunk;
    p.nseg = (L + p.seg_len - 1) / p.seg_len;
  }
  p.ws_bytes = !p.mfma ? 0 : g256 ? prefill_grouped256_workspace_bytes(heads, d->d, p.nseg)
                                  : prefill_mfma_workspace_bytes(heads, d->d, p.nseg);
  return p;
}

// A second stream of the library's own for work that needs nothing from the kernels beside it (the conv's share of dv
// and the conv-weight sums next to the gradient kernels): forked from the caller's
// stream and joined back into it with events, so that for the caller everything still happens on its stream --
// also under graph capture, where the side stream becomes part of the capture.  One per host thread and device,
// made at the first call that wants it (never while the caller's stream is being captured: then, and if anything
// cannot be made, the work simply stays on the caller's stream, in the same order).  Default priority.
struct SideLane {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, mid = nullptr, join = nullptr;
  bool ok = false;
};
SideLane* side_lane(hipStream_t caller) {
  static thread_local SideLane lanes[16];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
  SideLane& l = lanes[dev];
  if (l.ok) return &l;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(caller, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return nullptr;
  }
  bool made = hipStreamCreateWithFlags(&l.s, hipStreamNonBlocking) == hipSuccess &&
              hipEventCreateWithFlags(&l.fork, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&l.mid, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&l.join, hipEventDisableTiming) == hipSuccess;
  if (!made) {
    (void)hipGetLastError();
    if (l.join) (void)hipEventDestroy(l.join);
    if (l.mid) (void)hipEventDestroy(l.mid);
    if (l.fork) (void)hipEventDestroy(l.fork);
    if (l.s) (void)hipStreamDestroy(l.s);
    l = SideLane{};
    return nullptr;
  }
  l.ok = true;
  return &l;
}
// the side stream starts behind everything the caller's stream holds so far
hipError_t fork_side(SideLane* l, hipStream_t caller) {
  hipError_t e = hipEventRecord(l->fork, caller);
  return e != hipSuccess ? e : hipStreamWaitEvent(l->s, l->fork, 0);
}
// the caller's stream goes on behind everything the side stream holds so far
hipError_t join_side(SideLane* l, hipStream_t caller) {
  hipError_t e = hipEventRecord(l->join, l->s);
  return e != hipSuccess ? e : hipStreamWaitEvent(caller, l->join, 0);
}

linattn_status prefill_any(const linattn_desc* desc, int32_t L, bool grouped, float alpha, const void* q, const void* k,
                           const void* v, const float* conv_w, const float* S_in, const float* z_in, const void* hist_in,
                           void* out, float* S_out, float* z_out, void* hist_out, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  linattn_status st = check_desc(desc, true, true, LINATTN_MAX_CONV_K_PREFILL);
  if (st != LINATTN_OK) return st;
  if (L < 0) return LINATTN_ERR_SHAPE;
  const int m = value_blocks(desc);
  if (m > 1) {
    if (grouped) return LINATTN_ERR_UNSUPPORTED;                      // the three-branch kernels take d_v = d only
    // the value blocks of a head all read z_in and the first of them writes z_out
    if (z_in != nullptr && z_out == z_in) return LINATTN_ERR_UNSUPPORTED;
  }
  if (grouped) {
    if (!(alpha == alpha) || alpha - alpha != 0.f) return LINATTN_ERR_SHAPE;   // NaN, infinity
    // the groups are part of the result here: 64 tokens (the paper's size for LLaMA) or 256 (its size for FLASH)
    if (!prefill_grouped_simt_available(desc->io_dtype == LINATTN_BF16, desc->d, desc->chunk)) return LINATTN_ERR_UNSUPPORTED;
  }
  if (!conv_w) return LINATTN_ERR_NULL;
  if (L > 0 && (!q || !k || !v || !out)) return LINATTN_ERR_NULL;
  const bool has_hist = desc->conv_k > 1;
  const int given = (S_in != nullptr) + (z_in != nullptr) + ((hist_in != nullptr) || !has_hist);
  const bool cont = S_in != nullptr || z_in != nullptr || hist_in != nullptr;
  if (cont && given != 3) return LINATTN_ERR_NULL;   // all of the incoming state, or none of it
  const void* ptrs[] = {q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out, workspace};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LINATTN_ERR_ALIGN;
  // the last token of the last (b, h) must be addressable with 64-bit offsets
  if ((double)desc->stride_b * desc->B + (double)desc->stride_h * desc->H + (double)desc->stride_t * L > 9.0e18 ||
      (double)desc->stride_b_v * desc->B + (double)desc->stride_h_v * desc->H + (double)desc->stride_t_v * L > 9.0e18)
    return LINATTN_ERR_SHAPE;
  const PrefillPlan plan = plan_prefill(desc, L, grouped);
  if (plan.ws_bytes > 0 && (!workspace || workspace_bytes < plan.ws_bytes)) return LINATTN_ERR_WORKSPACE;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  PrefillArgs a{};
  // More than 8 taps: the attention kernels run without the convolution (one tap, taken as zero, no history) and
  // a pass of its own adds it to the outputs and hands the history on.
  const bool long_conv = desc->conv_k > LINATTN_MAX_CONV_K;
  const bool kernel_hist = has_hist && !long_conv;
  a.q = q; a.k = k; a.v = v; a.conv_w = conv_w;
  a.S_in = S_in; a.z_in = z_in; a.hist_in = kernel_hist ? hist_in : nullptr;
  a.out = out; a.S_out = S_out; a.z_out = z_out; a.hist_out = kernel_hist ? hist_out : nullptr;
  a.ws = static_cast<float*>(workspace);
  a.B = desc->B; a.H = desc->H; a.L = L; a.Kc = long_conv ? 1 : desc->conv_k; a.no_conv = long_conv;
  a.eps = desc->eps; a.relu = desc->phi == LINATTN_PHI_RELU; a.group = desc->chunk;
  a.sb = desc->stride_b; a.sh = desc->stride_h; a.st = desc->stride_t;
  a.m = m;
  a.sb_v = m > 1 ? desc->stride_b_v : desc->stride_b;
  a.sh_v = m > 1 ? desc->stride_h_v : desc->stride_h;
  a.st_v = m > 1 ? desc->stride_t_v : desc->stride_t;
  a.nseg = plan.nseg; a.seg_len = plan.seg_len;
  a.alpha = alpha;
  a.wait_spins = g_wait_spins.load(std::memory_order_relaxed);
  hipError_t e;
  const bool bf16 = desc->io_dtype == LINATTN_BF16;
  if (plan.mfma && L > 0 && grouped && desc->chunk == 256 && long_conv) {
    // Groups of 256 with a long conv: the conv pass writes out first and the full pass adds the rest to it (one
    // rounding of the sum, and the conv pass reads only V).  On the caller's stream: beside the first pass on the
    // side stream the call took 9 to 14 us longer -- the fork and the join cost more than the two short kernels
    // they would overlap.
    {
      ConvLongArgs c{};
      c.v = v; c.conv_w = conv_w; c.hist_in = hist_in; c.out = out; c.hist_out = hist_out;
      c.B = desc->B; c.H = desc->H; c.L = L; c.Kc = desc->conv_k;
      c.sb = a.sb_v; c.sh = a.sh_v; c.st = a.st_v; c.m = m; c.assign = 1;
      e = launch_conv_long(c, true, desc->d, stream);
    }
    if (e == hipSuccess && a.nseg > 1) {
      e = launch_prefill_mfma_ws(a, desc->d, true, false, stream);
      if (e == hipSuccess) e = launch_segment_scan(a, desc->d, stream);
    }
    if (e == hipSuccess) e = launch_prefill_grouped256(a, desc->d, stream);
    return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
  }
  if (plan.mfma && L > 0) e = launch_prefill_mfma(a, desc->d, desc->chunk, grouped, stream);
  else if (grouped && L > 0) e = launch_prefill_grouped_simt(a, bf16, desc->d, stream);   // fp32 rows; groups of 256
  else e = launch_prefill_simt(a, bf16, desc->d, stream);                                 // L = 0: the state is handed through
  if (e == hipSuccess && long_conv) {
    ConvLongArgs c{};
    c.v = v; c.conv_w = conv_w; c.hist_in = hist_in; c.out = out; c.hist_out = hist_out;
    c.B = desc->B; c.H = desc->H; c.L = L; c.Kc = desc->conv_k;
    c.sb = a.sb_v; c.sh = a.sh_v; c.st = a.st_v; c.m = m;
    e = launch_conv_long(c, bf16, desc->d, stream);
  }
  return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
}

}  // namespace

extern "C" {

const char* linattn_status_string(linattn_status s) {
  switch (s) {
    case LINATTN_OK: return "ok";
    case LINATTN_ERR_NULL: return "a required pointer is NULL";
    case LINATTN_ERR_SHAPE: return "invalid shape, size or stride";
    case LINATTN_ERR_DTYPE: return "unknown dtype or feature map";
    case LINATTN_ERR_ALIGN: return "pointer not 16-byte aligned";
    case LINATTN_ERR_UNSUPPORTED: return "no kernel for this request";
    case LINATTN_ERR_WORKSPACE: return "workspace missing or too small";
    case LINATTN_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

int32_t linattn_version(void) { return 210; }

int32_t linattn_set_wait_limit(int32_t spins) {
  return g_wait_spins.exchange(spins == 0 ? kDefaultWaitSpins : spins, std::memory_order_relaxed);
}

size_t linattn_workspace_bytes(const linattn_desc* desc, int32_t L) {
  if (check_desc(desc, true, true, LINATTN_MAX_CONV_K_PREFILL) != LINATTN_OK || L < 0) return 0;
  // the descriptor does not say which prefill form will be called: enough for either
  const size_t a = plan_prefill(desc, L, false).ws_bytes;
  const size_t b = desc->chunk == 256 && value_blocks(desc) == 1 ? plan_prefill(desc, L, true).ws_bytes : 0;
  return a > b ? a : b;
}

linattn_status linattn_prefill(const linattn_desc* desc, int32_t L, const void* q, const void* k, const void* v,
                               const float* conv_w, const float* S_in, const float* z_in, const void* hist_in,
                               void* out, float* S_out, float* z_out, void* hist_out, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  return prefill_any(desc, L, false, 0.f, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out, workspace,
                     workspace_bytes, hip_stream);
}

linattn_status linattn_prefill_noalloc(const linattn_desc* desc, int32_t L, const void* q, const void* k, const void* v,
                                       const float* conv_w, const float* S_in, const float* z_in, const void* hist_in,
                                       void* out, float* S_out, float* z_out, void* hist_out, void* hip_stream) {
  linattn_status st = check_desc(desc, true, true, LINATTN_MAX_CONV_K_PREFILL);
  if (st != LINATTN_OK) return st;
  if (L < 0) return LINATTN_ERR_SHAPE;
  const size_t need = plan_prefill(desc, L).ws_bytes;
  if (need > kScratchBytes) return LINATTN_ERR_WORKSPACE;     // beyond what the static scratch holds
  void* ws = nullptr;
  if (need > 0 && scratch_for_current_device(&ws) != hipSuccess) return LINATTN_ERR_HIP;
  return prefill_any(desc, L, false, 0.f, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out, ws, need,
                     hip_stream);
}

size_t linattn_noalloc_scratch_bytes(void) { return kScratchBytes; }

linattn_status linattn_prefill_grouped(const linattn_desc* desc, int32_t L, float alpha, const void* q, const void* k,
                                       const void* v, const float* conv_w, const float* S_in, const float* z_in,
                                       const void* hist_in, void* out, float* S_out, float* z_out, void* hist_out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  return prefill_any(desc, L, true, alpha, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out, workspace,
                     workspace_bytes, hip_stream);
}

namespace {
struct BackwardPlan {
  int ng, nwb;
  size_t off_P, off_D, off_stats, off_dw, bytes;   // byte offsets of the pieces of the workspace
};
size_t round256(size_t x) { return (x + 255) / 256 * 256; }
BackwardPlan plan_backward(const linattn_desc* d, int32_t L) {
  BackwardPlan p{};
  const size_t BH = (size_t)d->B * d->H, slot = (size_t)d->d * d->d + d->d;
  p.ng = L > 0 ? (L + d->chunk - 1) / d->chunk : 0;
  p.nwb = grouped_bwd_dw_blocks(L);
  p.off_P = 0;
  p.off_D = round256(BH * (p.ng > 0 ? p.ng : 1) * slot * sizeof(float));
  p.off_stats = p.off_D + round256(BH * (p.ng > 0 ? p.ng : 1) * slot * sizeof(float));
  p.off_dw = p.off_stats + round256(5 * BH * (size_t)(L > 0 ? L : 1) * sizeof(float));
  // partial conv-weight sums, and as much again for the stages of their reduction
  p.bytes = p.off_dw + 2 * round256(BH * (size_t)(p.nwb > 0 ? p.nwb : 1) * d->d * d->conv_k * sizeof(float));
  return p;
}
linattn_status check_backward(const linattn_desc* desc, int32_t L) {
  linattn_status st = check_desc(desc, true, true, LINATTN_MAX_CONV_K_PREFILL);
  if (st != LINATTN_OK) return st;
  if (L < 0) return LINATTN_ERR_SHAPE;
  if (desc->io_dtype != LINATTN_BF16 || value_blocks(desc) > 1) return LINATTN_ERR_UNSUPPORTED;
  if (desc->chunk != 64 && desc->chunk != 256) return LINATTN_ERR_UNSUPPORTED;
  return LINATTN_OK;
}
}  // namespace

size_t linattn_backward_workspace_bytes(const linattn_desc* desc, int32_t L) {
  if (check_backward(desc, L) != LINATTN_OK) return 0;
  return plan_backward(desc, L).bytes;
}

linattn_status linattn_prefill_grouped_backward(const linattn_desc* desc, int32_t L, float alpha, const void* q,
                                                const void* k, const void* v, const float* conv_w, const void* dout,
                                                void* dq, void* dk, void* dv, float* dconv_w, void* workspace,
                                                size_t workspace_bytes, void* hip_stream) {
  linattn_status st = check_backward(desc, L);
  if (st != LINATTN_OK) return st;
  if (!(alpha == alpha) || alpha - alpha != 0.f) return LINATTN_ERR_SHAPE;   // NaN, infinity
  if (!conv_w) return LINATTN_ERR_NULL;
  if (L > 0 && (!q || !k || !v || !dout || !dq || !dk || !dv)) return LINATTN_ERR_NULL;
  const void* ptrs[] = {q, k, v, conv_w, dout, dq, dk, dv, dconv_w, workspace};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LINATTN_ERR_ALIGN;
  if ((double)desc->stride_b * desc->B + (double)desc->stride_h * desc->H + (double)desc->stride_t * L > 9.0e18)
    return LINATTN_ERR_SHAPE;
  const BackwardPlan plan = plan_backward(desc, L);
  if (!workspace || workspace_bytes < plan.bytes) return LINATTN_ERR_WORKSPACE;
  if ((int64_t)desc->B * desc->H > 65535 || (int64_t)2 * plan.ng > 0x7fffffff) return LINATTN_ERR_SHAPE;   // grid limits

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  GroupedBwdArgs a{};
  a.q = q; a.k = k; a.v = v; a.dout = dout; a.dq = dq; a.dk = dk; a.dv = dv; a.conv_w = conv_w; a.dconv_w = dconv_w;
  a.P = reinterpret_cast<float*>(ws + plan.off_P);
  a.Dg = reinterpret_cast<float*>(ws + plan.off_D);
  a.stats = reinterpret_cast<float*>(ws + plan.off_stats);
  a.dw_part = reinterpret_cast<float*>(ws + plan.off_dw);
  a.B = desc->B; a.H = desc->H; a.L = L; a.Kc = desc->conv_k; a.eps = desc->eps; a.relu = desc->phi == LINATTN_PHI_RELU;
  a.alpha = alpha;
  a.sb = desc->stride_b; a.sh = desc->stride_h; a.st = desc->stride_t;
  a.group = desc->chunk; a.ng = plan.ng; a.nwb = plan.nwb;
  // The conv's share of dv (the same taps met from the other side, dv[s] = sum_j w[j] dout[s + j]) is written first
  // and the conv-weight sums need nothing from the other kernels: both run on the side stream; the kernel that adds
  // the rest of dv waits for the first, the end of the call for the second.
  hipError_t e = hipSuccess;
  SideLane* lane = (L > 0) ? side_lane(stream) : nullptr;
  hipStream_t cs = lane ? lane->s : stream;
  if (lane) e = fork_side(lane, stream);
  if (e == hipSuccess && L > 0) {
    ConvLongArgs c{};
    c.v = dout; c.conv_w = conv_w; c.out = dv;
    c.B = a.B; c.H = a.H; c.L = L; c.Kc = a.Kc; c.sb = a.sb; c.sh = a.sh; c.st = a.st; c.m = 1; c.rev = 1; c.assign = 1;
    e = launch_conv_long(c, true, desc->d, cs);
    if (e == hipSuccess && lane) e = hipEventRecord(lane->mid, cs);
  }
  if (e == hipSuccess) e = launch_grouped_bwd_dw(a, desc->d, cs);            // no tokens: the sums over nothing
  if (e == hipSuccess) e = launch_grouped_bwd_core(a, desc->d, stream, lane ? lane->mid : nullptr);
  if (lane) {                                              // joined whatever happened, so that nothing stays forked
    const hipError_t ej = join_side(lane, stream);
    if (e == hipSuccess) e = ej;
  }
  return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
}

linattn_status linattn_verify(const linattn_desc* desc, int32_t kk, const void* q, const void* k, const void* v,
                              const float* conv_w, float* S, float* z, void* hist, const int32_t* n_commit,
                              void* out, void* hip_stream) {
  linattn_status st = check_desc(desc, false, false);
  if (st != LINATTN_OK) return st;
  if (kk < 1 || kk > LINATTN_MAX_DRAFT) return LINATTN_ERR_SHAPE;
  if (!q || !k || !v || !conv_w || !S || !z || !out) return LINATTN_ERR_NULL;
  if (desc->conv_k > 1 && !hist) return LINATTN_ERR_NULL;
  const void* ptrs[] = {q, k, v, conv_w, S, z, hist, out};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LINATTN_ERR_ALIGN;
  if (n_commit && (reinterpret_cast<uintptr_t>(n_commit) & 3u)) return LINATTN_ERR_ALIGN;

  VerifyArgs a{};
  a.q = q; a.k = k; a.v = v; a.conv_w = conv_w; a.S = S; a.z = z; a.hist = hist;
  a.n_commit = n_commit; a.out = out;
  a.B = desc->B; a.H = desc->H; a.kk = kk; a.Kc = desc->conv_k; a.eps = desc->eps; a.relu = desc->phi == LINATTN_PHI_RELU;
  const int m = value_blocks(desc);
  a.dv = m * desc->d;
  const int nsplit = verify_pick_split(desc->B * desc->H * m);
  const bool bf16 = desc->io_dtype == LINATTN_BF16;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // whole blocks of d value channels per workgroup on the matrix cores when there are enough of them to fill the
  // chip (B H m >= 768), column slices of a head's state on the streaming kernel otherwise
  const hipError_t e = verify_mfma_available(bf16, desc->d, nsplit, kk) ? launch_verify_mfma(a, desc->d, stream)
                                                                        : launch_verify(a, bf16, desc->d, nsplit, stream);
  return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
}

linattn_status linattn_verify_grouped(const linattn_desc* desc, int32_t kk, float alpha, const void* q, const void* k,
                                      const void* v, const float* conv_w, float* S, float* z, void* hist, void* kwin,
                                      void* vwin, int32_t* fill, const int32_t* n_commit, void* out, void* hip_stream) {
  linattn_status st = check_desc(desc, true, false);     // the group size is part of the result; the tensors are dense
  if (st != LINATTN_OK) return st;
  if (kk < 1 || kk > LINATTN_MAX_DRAFT) return LINATTN_ERR_SHAPE;
  if (!(alpha == alpha) || alpha - alpha != 0.f) return LINATTN_ERR_SHAPE;   // NaN, infinity
  if (!q || !k || !v || !conv_w || !S || !z || !kwin || !vwin || !fill || !out) return LINATTN_ERR_NULL;
  if (desc->conv_k > 1 && !hist) return LINATTN_ERR_NULL;
  const void* ptrs[] = {q, k, v, conv_w, S, z, hist, kwin, vwin, out};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LINATTN_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(fill) & 3u) || (reinterpret_cast<uintptr_t>(n_commit) & 3u)) return LINATTN_ERR_ALIGN;
  if (desc->chunk != 64) return LINATTN_ERR_UNSUPPORTED;
  if (value_blocks(desc) > 1) return LINATTN_ERR_UNSUPPORTED;

  VerifyGroupedArgs a{};
  a.q = q; a.k = k; a.v = v; a.conv_w = conv_w; a.S = S; a.z = z; a.hist = hist;
  a.kwin = kwin; a.vwin = vwin; a.fill = fill; a.n_commit = n_commit; a.out = out;
  a.B = desc->B; a.H = desc->H; a.kk = kk; a.Kc = desc->conv_k; a.eps = desc->eps; a.alpha = alpha;
  a.relu = desc->phi == LINATTN_PHI_RELU;
  const bool bf16 = desc->io_dtype == LINATTN_BF16;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = verify_grouped_mfma_available(bf16, desc->d, kk) ? launch_verify_grouped_mfma(a, desc->d, stream)
                                                                        : launch_verify_grouped(a, bf16, desc->d, stream);
  return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
}

linattn_status linattn_verify_tree(const linattn_desc* desc, int32_t n, const void* q, const void* k, const void* v,
                                   const int32_t* parent, const float* conv_w, float* S, float* z, void* hist,
                                   const int32_t* accept, void* out, void* hip_stream) {
  linattn_status st = check_desc(desc, false, false);
  if (st != LINATTN_OK) return st;
  if (n < 1 || n > LINATTN_MAX_TREE) return LINATTN_ERR_SHAPE;
  if (!q || !k || !v || !parent || !conv_w || !S || !z || !out) return LINATTN_ERR_NULL;
  if (desc->conv_k > 1 && !hist) return LINATTN_ERR_NULL;
  const void* ptrs[] = {q, k, v, conv_w, S, z, hist, out};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LINATTN_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(parent) & 3u) || (reinterpret_cast<uintptr_t>(accept) & 3u)) return LINATTN_ERR_ALIGN;
  if (value_blocks(desc) > 1) return LINATTN_ERR_UNSUPPORTED;

  VerifyTreeArgs a{};
  a.q = q; a.k = k; a.v = v; a.conv_w = conv_w; a.S = S; a.z = z; a.hist = hist;
  a.parent = parent; a.accept = accept; a.out = out;
  a.B = desc->B; a.H = desc->H; a.n = n; a.Kc = desc->conv_k; a.eps = desc->eps; a.relu = desc->phi == LINATTN_PHI_RELU;
  // bf16 candidates on the matrix cores; fp32 candidates in exact fp32 on the vector ALUs
  const hipError_t e = desc->io_dtype == LINATTN_BF16 ? launch_verify_tree(a, desc->d, static_cast<hipStream_t>(hip_stream))
                                                      : launch_verify_tree_simt(a, desc->d, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? LINATTN_OK : LINATTN_ERR_HIP;
}

linattn_status linattn_decode(const linattn_desc* desc, const void* q, const void* k, const void* v,
                              const float* conv_w, float* S, float* z, void* hist, void* out, void* hip_stream) {
  return linattn_verify(desc, 1, q, k, v, conv_w, S, z, hist, nullptr, out, hip_stream);
}

}  // extern "C"
