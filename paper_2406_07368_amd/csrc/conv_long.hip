// Causal depthwise convolution on V with more than 8 taps (Sec. 4.1: the FLASH experiment runs the masked
// DWConv with kernel size 63), as a pass of its own behind the attention kernels:
//
//   out[t][c] += sum_{j < Kc} w[h][c][j] * Vext[t - j][c]        Vext = hist_in ++ V, zeros before that
//
// The attention kernels keep an 8-row halo of V in LDS and gather the taps per token; a 62-row halo does not
// fit next to their row buffers, and 63 taps per output are a vector-ALU workload of the size of the attention
// itself.  So long kernels are register-blocked here instead: a thread owns one channel, holds its taps in
// registers and slides over 8 outputs at a time, every value row read from LDS feeding up to 8 multiply-adds.
// One workgroup = 64 tokens of one (b, h); rows t0-62 .. t0+63 of V are staged in LDS as fp32.
#include "common.h"
#include "kernels.h"

namespace linattn {

namespace {
constexpr int CL_TOK = 64;        // tokens per workgroup
constexpr int CL_HALO = 62;       // rows before them that the longest kernel reaches
constexpr int CL_MAXK = 63;
constexpr int CL_BLK = 8;         // outputs a thread carries at once
}  // namespace

template <typename Io, int D>
__global__ __launch_bounds__(256) void conv_long_kernel(ConvLongArgs a) {
  extern __shared__ float xs[];   // [CL_HALO + CL_TOK][D]
  constexpr int NG = 256 / D;                 // token groups of threads
  constexpr int TPT = CL_TOK / NG;            // tokens per thread
  const int tid = threadIdx.x;
  // one (b, h, value block of D channels); d_v = D: one block per head
  const int bh = blockIdx.y / a.m, blk = blockIdx.y % a.m, b = bh / a.H, h = bh % a.H;
  const int DVT = a.m * D;
  const int t0 = blockIdx.x * CL_TOK;
  const int Kc = a.Kc, L = a.L;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh + (int64_t)blk * D;
  const int64_t hist_base = (int64_t)bh * (Kc - 1) * DVT + (int64_t)blk * D;
  const int c = tid % D, tg = tid / D;

  // this channel's taps; beyond Kc they are zero, so the unrolled loop below needs no tap count
  float wreg[CL_MAXK];
#pragma unroll
  for (int j = 0; j < CL_MAXK; ++j) wreg[j] = j < Kc ? a.conv_w[((size_t)h * DVT + blk * D + c) * Kc + j] : 0.f;

  // rows t0 - 62 .. t0 + 63: the sequence, before it the incoming history, before that (and past the end) zeros
  for (int e = tid; e < (CL_HALO + CL_TOK) * (D / 8); e += 256) {
    const int row = e / (D / 8), i0 = 8 * (e % (D / 8));
    const int tok = t0 - CL_HALO + row;
    float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (tok >= 0 && tok < L) Io::load8(a.v, base + (int64_t)tok * a.st + i0, x);
    else if (tok < 0 && a.hist_in && Kc - 1 + tok >= 0) Io::load8(a.hist_in, hist_base + (int64_t)(Kc - 1 + tok) * DVT + i0, x);
#pragma unroll
    for (int i = 0; i < 8; ++i) xs[row * D + i0 + i] = x[i];
  }
  __syncthreads();

  for (int tb0 = tg * TPT; tb0 < (tg + 1) * TPT; tb0 += CL_BLK) {
    if (t0 + tb0 >= L) break;                 // uniform per wave: D >= 64 channels share tb0
    float acc[CL_BLK];
#pragma unroll
    for (int e = 0; e < CL_BLK; ++e) acc[e] = 0.f;
    // value rows from the newest output's own row backwards: row m feeds output e through tap e - 7 + m
    const float* newest = xs + (CL_HALO + tb0 + CL_BLK - 1) * D + c;
    // (fully unrolled, so that every tap index is a constant and the taps stay in registers)
#pragma unroll
    for (int m = 0; m < CL_MAXK + CL_BLK - 1; ++m) {
      if (m - (CL_BLK - 1) < Kc) {            // uniform: beyond that no output of the block reaches this far back
        const float x = newest[-m * D];
#pragma unroll
        for (int e = 0; e < CL_BLK; ++e) {
          constexpr int J0 = -(CL_BLK - 1);
          const int j = e + J0 + m;
          if (j >= 0 && j < CL_MAXK) acc[e] = fmaf(wreg[j], x, acc[e]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < CL_BLK; ++e) {
      const int tok = t0 + tb0 + e;
      if (tok < L) {
        const int64_t o = base + (int64_t)tok * a.st + c;
        Io::store1(a.out, o, Io::load1(a.out, o) + acc[e]);
      }
    }
  }
}

// New history = the last Kc-1 rows of (incoming history ++ sequence).  Runs behind conv_long_kernel, which is the
// last reader of hist_in; one thread per channel writes its rows in ascending order and reads row L + r >= r of
// the extended sequence for row r, so hist_out may be hist_in.
template <typename Io>
__global__ void conv_long_hist_kernel(ConvLongArgs a, int D) {
  const int bh = blockIdx.x / a.m, blk = blockIdx.x % a.m, b = bh / a.H, h = bh % a.H;
  const int c = threadIdx.x;
  if (c >= D) return;
  const int R = a.Kc - 1, DVT = a.m * D;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh + (int64_t)blk * D;
  const int64_t hist_base = (int64_t)bh * R * DVT + (int64_t)blk * D;
  for (int r = 0; r < R; ++r) {
    const int e = a.L + r;                    // row of (history ++ sequence), the history being rows 0 .. R-1
    float x = 0.f;
    if (e >= R) x = Io::load1(a.v, base + (int64_t)(e - R) * a.st + c);
    else if (a.hist_in) x = Io::load1(a.hist_in, hist_base + (int64_t)e * DVT + c);
    Io::store1(a.hist_out, hist_base + (int64_t)r * DVT + c, x);
  }
}

template <typename Io, int D>
static hipError_t launch_cl(const ConvLongArgs& a, hipStream_t st) {
  constexpr int LDS = (CL_HALO + CL_TOK) * D * (int)sizeof(float);
  hipError_t e = hipSuccess;
  if (a.L > 0) {
    auto kern = conv_long_kernel<Io, D>;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((a.L + CL_TOK - 1) / CL_TOK), (unsigned)(a.B * a.H * a.m)), dim3(256), LDS, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (a.hist_out) {
    hipLaunchKernelGGL((conv_long_hist_kernel<Io>), dim3((unsigned)(a.B * a.H * a.m)), dim3(D), 0, st, a, D);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_conv_long(const ConvLongArgs& a, bool bf16, int d, hipStream_t st) {
  if (bf16) return d == 128 ? launch_cl<IoBf16, 128>(a, st) : launch_cl<IoBf16, 64>(a, st);
  return d == 128 ? launch_cl<IoF32, 128>(a, st) : launch_cl<IoF32, 64>(a, st);
}

}  // namespace linattn
