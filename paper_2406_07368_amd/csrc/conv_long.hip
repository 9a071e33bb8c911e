// Causal depthwise convolution on V with more than 8 taps (Sec. 4.1: the FLASH experiment runs the masked
// DWConv with kernel size 63), as a pass of its own behind the attention kernels:
//
//   out[t][c] += sum_{j < Kc} w[h][c][j] * Vext[t - j][c]        Vext = hist_in ++ V, zeros before that
//   (or out = ..., when the pass runs ahead of the kernel that adds the rest)
//
// The attention kernels keep an 8-row halo of V in LDS and gather the taps per token; a 62-row halo does not
// fit next to their row buffers, and 63 taps per output are a vector-ALU workload of the size of the attention
// itself.  So long kernels are register-blocked here instead: a thread owns one channel, holds its taps in
// registers and slides over 16 (adding to out: 8) outputs at a time, every value row read from LDS feeding that many
// multiply-adds.
// One workgroup = 64 (or 32) tokens of one (b, h); rows t0-62 .. t0+63 of V are staged in LDS as they lie in memory.
#include "common.h"
#include "kernels.h"

namespace linattn {

namespace {
constexpr int CL_TOK = 64;        // tokens per workgroup (32 when that still leaves compute units without one: a
                                  // workgroup's time is one thread's chain over its tokens, and half the chain is
                                  // worth more then than the halo rows it reads twice)
constexpr int CL_HALO = 62;       // rows before them that the longest kernel reaches
constexpr int CL_MAXK = 63;
constexpr int CL_BLK = 16;        // outputs a thread carries at once (fewer if it has fewer tokens; half when adding to out)
}  // namespace

// KMAX: tap capacity of the instantiation (taps beyond Kc are zeros; the loops below are straight-line code for
// exactly KMAX taps: a branch per tap would put every LDS read into a basic block of its own, with a full wait
// behind it).
static __device__ __forceinline__ float elem_to_f32(float x) { return x; }
static __device__ __forceinline__ float elem_to_f32(uint16_t x) { return bf16_bits_to_f32(x); }

template <typename Io, int D, int KMAX, bool ASSIGN, int TOK>
__global__ __launch_bounds__(256) void conv_long_kernel(ConvLongArgs a) {
  // the value rows [CL_HALO + TOK][D] as they lie in memory (bf16 rows stay bf16: half the LDS of fp32 rows, so
  // twice the workgroups per compute unit); before them, for a moment, the taps as fp32
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_cl[];
  float* xs = reinterpret_cast<float*>(smem_cl);
  typename Io::elem* xe = reinterpret_cast<typename Io::elem*>(smem_cl);
  constexpr int NG = 256 / D;                 // token groups of threads
  constexpr int TPT = TOK / NG;            // tokens per thread
  // (adding to out, a block also holds its own and the next block's elements of out: with sixteen the registers allow
  // two workgroups per compute unit instead of three, which costs 13 % at a chip-filling size)
  constexpr int BLK_MAX = ASSIGN ? CL_BLK : CL_BLK / 2;
  constexpr int BLK = TPT < BLK_MAX ? TPT : BLK_MAX;
  const int tid = threadIdx.x;
  // one (b, h, value block of D channels); d_v = D: one block per head
  const int bh = blockIdx.y / a.m, blk = blockIdx.y % a.m, b = bh / a.H, h = bh % a.H;
  const int DVT = a.m * D;
  // Neighbouring token blocks share 62 of their rows: block indices 8 apart land on the same chiplet, so they get
  // neighbouring token blocks, and the shared rows come from that chiplet's L2 (when the count is a multiple of 8).
  const int nblk = gridDim.x;
  const int tblk = nblk % 8 == 0 ? (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3) : (int)blockIdx.x;
  const int t0 = tblk * TOK;
  const int Kc = a.Kc, L = a.L;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh + (int64_t)blk * D;
  const int64_t hist_base = (int64_t)bh * (Kc - 1) * DVT + (int64_t)blk * D;
  const int c = tid % D, tg = tid / D;

  // this channel's taps; beyond Kc they are zero, so the unrolled loop below needs no tap count.  The D * Kc taps of
  // the block are contiguous in memory: they come in through LDS with whole-row requests (a thread reading its own
  // Kc consecutive floats would touch 64 cache lines per request), then each thread picks its own (stride Kc floats
  // between lanes; Kc odd or not, at most a 2-way bank conflict, once per workgroup).
  // Every request of the workgroup -- taps, value rows, the 32 elements of out that the thread adds to -- is issued
  // before the first wait: one trip to memory per workgroup instead of one per stage.
  constexpr int RIT = ((CL_HALO + TOK) * (D / 8) + 255) / 256;
  typename Io::raw8 raw[RIT];
  bool have[RIT];
  auto issue_rows = [&]() __attribute__((always_inline)) {
    // rows t0 - 62 .. t0 + 63: the sequence, before it the incoming history, before that (and past the end) zeros
#pragma unroll
    for (int i = 0; i < RIT; ++i) {
      const int e = tid + 256 * i;
      const int row = e / (D / 8), i0 = 8 * (e % (D / 8));
      const int tok = t0 - CL_HALO + row;
      // unconditional requests (a row that does not exist reads row 0 of the sequence instead and is dropped):
      // every branch around a request would end in a full wait
      const bool in_seq = tok >= 0 && tok < L;
      const bool in_hist = tok < 0 && a.hist_in != nullptr && Kc - 1 + tok >= 0;
      const void* src = in_hist ? a.hist_in : a.v;
      const int mt = in_seq ? (a.rev ? L - 1 - tok : tok) : 0;     // where the token lies in memory
      const int64_t idx = in_hist ? hist_base + (int64_t)(Kc - 1 + tok) * DVT + i0 : base + (int64_t)mt * a.st + i0;
      raw[i] = Io::load_raw8(src, idx);
      have[i] = in_seq || in_hist;
    }
  };
  // what the attention kernels left in out, as it lies in memory (converted where it is added to), a block of tokens at a
  // time: the first block with the first requests, the next while the current ones are being computed (all 32
  // at once would cost the registers that let a second and third workgroup share the compute unit).  Past the end: the
  // first token's element, never stored.
  [[maybe_unused]] typename Io::elem prev[BLK];
  auto issue_prev = [&](int blk8, typename Io::elem (&dst)[BLK]) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < BLK; ++e) {
      const int tok = t0 + tg * TPT + blk8 * BLK + e;
      const int mt = tok < L ? (a.rev ? L - 1 - tok : tok) : 0;
      dst[e] = static_cast<const typename Io::elem*>(a.out)[base + (int64_t)mt * a.st + c];
    }
  };
  float wreg[KMAX];
  {
    // (16 bytes per request, every request of the thread issued before the first value is stored)
    const f32x4* wsrc = reinterpret_cast<const f32x4*>(a.conv_w + ((size_t)h * DVT + blk * D) * Kc);
    constexpr int WIT = (D * KMAX / 4 + 255) / 256;
    f32x4 wt[WIT];
#pragma unroll
    for (int i = 0; i < WIT; ++i) {
      const int e = tid + 256 * i;
      wt[i] = wsrc[e < D * Kc / 4 ? e : D * Kc / 4 - 1];   // unconditional: a branch would end in a full wait
    }
    issue_rows();                             // the value rows are on their way while the taps make their trip through LDS
#pragma unroll
    for (int i = 0; i < WIT; ++i) {
      const int e = tid + 256 * i;
      if (e < D * Kc / 4) *reinterpret_cast<f32x4*>(xs + 4 * e) = wt[i];
    }
    if constexpr (!ASSIGN) issue_prev(0, prev);   // ... and the first of what is already in out
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KMAX; ++j) wreg[j] = j < Kc ? xs[c * Kc + j] : 0.f;
    __syncthreads();                          // the staging area is about to take the value rows
  }

  {
#pragma unroll
    for (int i = 0; i < RIT; ++i) {
      const int e = tid + 256 * i;
      const int row = e / (D / 8), i0 = 8 * (e % (D / 8));
      if (e < (CL_HALO + TOK) * (D / 8)) {
        typename Io::raw8 y = raw[i];
        if (!have[i]) y = typename Io::raw8{};
        *reinterpret_cast<typename Io::raw8*>(xe + row * D + i0) = y;
      }
    }
  }
  __syncthreads();

  // The history handed on (the last Kc - 1 rows of history ++ sequence), when the launcher asked for it here: every
  // workgroup writes the rows whose tokens it owns (t0 <= token < t0 + 64; the first one also the rows that stay
  // history rows), straight from its LDS copy.  Asked for only when no other workgroup can still have hist_in to read.
  if (a.hist_fused) {
    const int R = Kc - 1;
    for (int e = tid; e < R * (D / 8); e += 256) {
      const int r = e / (D / 8), i0 = 8 * (e % (D / 8));
      const int tok = L - R + r;                           // the token (negative: a row of the old history) that becomes row r
      const bool mine = tok < L && ((tok >= t0 && tok < t0 + TOK) || (tok < 0 && t0 == 0));
      const int row = tok - t0 + CL_HALO;                  // its row in the LDS copy
      if (mine && row >= 0)
        *reinterpret_cast<typename Io::raw8*>(static_cast<typename Io::elem*>(a.hist_out) + hist_base + (int64_t)r * DVT + i0) =
            *reinterpret_cast<const typename Io::raw8*>(xe + row * D + i0);
    }
  }

  // (one copy of the 500 multiply-adds in the instruction stream: the loop over the thread's blocks stays a loop)
#pragma unroll 1
  for (int blk8 = 0; blk8 < TPT / BLK; ++blk8) {
    const int tb0 = tg * TPT + blk8 * BLK;
    float acc[BLK];
    [[maybe_unused]] typename Io::elem next[BLK];
    if constexpr (!ASSIGN) issue_prev(blk8 + 1 < TPT / BLK ? blk8 + 1 : blk8, next);
#pragma unroll
    for (int e = 0; e < BLK; ++e) acc[e] = 0.f;
    // value rows from the newest output's own row backwards: row m feeds output e through tap e - 7 + m
    const typename Io::elem* newest = xe + (CL_HALO + tb0 + BLK - 1) * D + c;
    // (fully unrolled, so that every tap index is a constant and the taps stay in registers)
#pragma unroll
    for (int m = 0; m < KMAX + BLK - 1; ++m) {
      const float x = elem_to_f32(newest[-m * D]);
#pragma unroll
      for (int e = 0; e < BLK; ++e) {
        constexpr int J0 = -(BLK - 1);
        const int j = e + J0 + m;
        if (j >= 0 && j < KMAX) acc[e] = fmaf(wreg[j], x, acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < BLK; ++e) {
      const int tok = t0 + tb0 + e;
      if (tok < L)
        Io::store1(a.out, base + (int64_t)(a.rev ? L - 1 - tok : tok) * a.st + c, ASSIGN ? acc[e] : elem_to_f32(prev[e]) + acc[e]);
    }
    if constexpr (!ASSIGN) {
#pragma unroll
      for (int e = 0; e < BLK; ++e) prev[e] = next[e];
    }
  }
}

// New history = the last Kc-1 rows of (incoming history ++ sequence), for the cases the conv kernel cannot do on the
// way (hist_out is hist_in on a sequence of several workgroups; no tokens).  Runs behind conv_long_kernel, which is the
// last reader of hist_in before this.  One workgroup per (b, h, value block): every element is read (all requests in
// flight at once) before, behind a barrier, any is written, so hist_out may be hist_in.
template <typename Io, int D>
__global__ __launch_bounds__(256) void conv_long_hist_kernel(ConvLongArgs a) {
  const int bh = blockIdx.x / a.m, blk = blockIdx.x % a.m, b = bh / a.H, h = bh % a.H;
  const int tid = threadIdx.x;
  const int R = a.Kc - 1, DVT = a.m * D;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh + (int64_t)blk * D;
  const int64_t hist_base = (int64_t)bh * R * DVT + (int64_t)blk * D;
  // whole vectors of 8 channels, as they lie in memory (history and value rows share their element type); every
  // request is unconditional -- a vector that does not exist reads the first one of hist_out instead and is
  // replaced by zeros -- so that all of them are in flight together
  using raw8 = typename Io::raw8;
  using elem = typename Io::elem;
  constexpr int VPR = D / 8;
  constexpr int EIT = (CL_HALO * VPR + 255) / 256;
  raw8 x[EIT];
  bool have[EIT];
#pragma unroll
  for (int i = 0; i < EIT; ++i) {
    const int el = tid + 256 * i;
    const int r = el / VPR, c = 8 * (el % VPR);
    const int e = a.L + r;                    // row of (history ++ sequence), the history being rows 0 .. R-1
    const bool from_v = r < R && e >= R;
    const bool from_h = r < R && e < R && a.hist_in != nullptr;
    const void* src = from_v ? a.v : from_h ? a.hist_in : a.hist_out;
    const int64_t idx = from_v ? base + (int64_t)(e - R) * a.st + c : from_h ? hist_base + (int64_t)e * DVT + c : hist_base;
    x[i] = Io::load_raw8(src, idx);
    have[i] = from_v || from_h;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < EIT; ++i) {
    const int el = tid + 256 * i;
    const int r = el / VPR, c = 8 * (el % VPR);
    if (r < R) {
      raw8 y = x[i];
      if (!have[i]) y = raw8{};
      *reinterpret_cast<raw8*>(static_cast<elem*>(a.hist_out) + hist_base + (int64_t)r * DVT + c) = y;
    }
  }
}

template <typename Io, int D, int KMAX, bool ASSIGN, int TOK>
static hipError_t launch_cl_t(const ConvLongArgs& a, hipStream_t st) {
  constexpr int LDS_ROWS = (CL_HALO + TOK) * D * (int)sizeof(typename Io::elem), LDS_TAPS = D * KMAX * (int)sizeof(float);
  constexpr int LDS = LDS_ROWS > LDS_TAPS ? LDS_ROWS : LDS_TAPS;
  auto kern = conv_long_kernel<Io, D, KMAX, ASSIGN, TOK>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, LDS);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)((a.L + TOK - 1) / TOK), (unsigned)(a.B * a.H * a.m)), dim3(256), LDS, st, a);
  return hipGetLastError();
}

template <typename Io, int D, int KMAX, bool ASSIGN>
static hipError_t launch_cl_k(const ConvLongArgs& a, hipStream_t st) {
  // fewer 64-token workgroups than compute units: 32 tokens each
  const int64_t wgs = (int64_t)((a.L + CL_TOK - 1) / CL_TOK) * a.B * a.H * a.m;
  return wgs < 256 ? launch_cl_t<Io, D, KMAX, ASSIGN, CL_TOK / 2>(a, st) : launch_cl_t<Io, D, KMAX, ASSIGN, CL_TOK>(a, st);
}

template <typename Io, int D, bool ASSIGN>
static hipError_t launch_cl(const ConvLongArgs& a_in, hipStream_t st) {
  hipError_t e = hipSuccess;
  // The history can be handed on by the conv kernel itself unless hist_out is hist_in and several workgroups share a
  // head: the first of them reads the old rows, the last would overwrite them, and nothing orders the two.
  ConvLongArgs a = a_in;
  a.hist_fused = a.hist_out != nullptr && !a.rev && a.L > 0 && (a.hist_out != a.hist_in || a.L <= CL_TOK / 2);
  if (a.L > 0) {
    e = a.Kc <= 16   ? launch_cl_k<Io, D, 16, ASSIGN>(a, st)
        : a.Kc <= 32 ? launch_cl_k<Io, D, 32, ASSIGN>(a, st)
                     : launch_cl_k<Io, D, CL_MAXK, ASSIGN>(a, st);
    if (e != hipSuccess) return e;
  }
  if (a.hist_out && !a.hist_fused) {
    hipLaunchKernelGGL((conv_long_hist_kernel<Io, D>), dim3((unsigned)(a.B * a.H * a.m)), dim3(256), 0, st, a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_conv_long(const ConvLongArgs& a, bool bf16, int d, hipStream_t st) {
  if (a.assign) {
    if (!bf16) return hipErrorInvalidValue;
    return d == 128 ? launch_cl<IoBf16, 128, true>(a, st) : launch_cl<IoBf16, 64, true>(a, st);
  }
  if (bf16) return d == 128 ? launch_cl<IoBf16, 128, false>(a, st) : launch_cl<IoBf16, 64, false>(a, st);
  return d == 128 ? launch_cl<IoF32, 128, false>(a, st) : launch_cl<IoF32, 64, false>(a, st);
}

}  // namespace linattn
