// Prefill with fp32 arithmetic on the vector ALUs (Sec. 4.1: groups of tokens,
// masked in-group product, running (S, z) between groups).  One workgroup of 256
// threads walks one (b, h) in steps of 32 tokens with the whole d x d state in
// LDS.  This is the path for fp32 inputs, where every product has to be an exact
// fp32 multiply-add to meet a 1e-4 bound; it is not tuned for throughput.
#include "common.h"
#include "kernels.h"

namespace linattn {

namespace {
constexpr int TC = 32;     // tokens per step (the result does not depend on the grouping)
constexpr int HMAX = 7;    // history rows kept in LDS: enough for the largest conv kernel (8 taps)

template <int D>
struct SimtLayout {
  static constexpr int S = 0;                         // [D][D]
  static constexpr int FQ = S + D * D;                // [TC][D+1]
  static constexpr int FK = FQ + TC * (D + 1);        // [TC][D+1]
  static constexpr int VV = FK + TC * (D + 1);        // [HMAX+TC][D]: history rows, then the step's rows
  static constexpr int P = VV + (HMAX + TC) * D;      // [TC][TC+1]
  static constexpr int DEN = P + TC * (TC + 1);       // [TC]
  static constexpr int ZZ = DEN + TC;                 // [D]
  static constexpr int TOTAL = ZZ + D;
};
}  // namespace

template <typename Io, int D>
__global__ __launch_bounds__(256) void prefill_simt_kernel(PrefillArgs a) {
  using Lay = SimtLayout<D>;
  constexpr int NG = 256 / D;
  extern __shared__ float sm[];
  float* S = sm + Lay::S;
  float* fq = sm + Lay::FQ;
  float* fk = sm + Lay::FK;
  float* vv = sm + Lay::VV;
  float* P = sm + Lay::P;
  float* den = sm + Lay::DEN;
  float* zz = sm + Lay::ZZ;

  const int tid = threadIdx.x;
  const HeadIndex hx = head_index(a, blockIdx.x, D);      // one (b, h, value block)
  const int bh = hx.bh, h = hx.h, DVT = hx.dvt;
  const int Kc = a.Kc, L = a.L;
  const int64_t base = (int64_t)hx.b * a.sb + (int64_t)h * a.sh;
  const int64_t base_v = (int64_t)hx.b * a.sb_v + (int64_t)h * a.sh_v + (int64_t)hx.blk * D;
  const int64_t hist_base = (int64_t)bh * (Kc - 1) * DVT + (int64_t)hx.blk * D;
  const int64_t S_base = (int64_t)bh * D * DVT + (int64_t)hx.blk * D;
  const int c = tid % D, tg = tid / D;

  float wreg[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) wreg[j] = (j < Kc && !a.no_conv) ? a.conv_w[((size_t)h * DVT + hx.blk * D + c) * Kc + j] : 0.f;

  for (int e = tid; e < D * D; e += 256) S[e] = a.S_in ? a.S_in[S_base + (int64_t)(e / D) * DVT + e % D] : 0.f;
  if (tid < D) zz[tid] = a.z_in ? a.z_in[(size_t)bh * D + tid] : 0.f;
  for (int e = tid; e < HMAX * D; e += 256) {
    const int row = e / D, cc = e % D;
    const int r = row - (HMAX - (Kc - 1));   // row of the incoming history, oldest first
    vv[e] = (r >= 0 && a.hist_in) ? Io::load1(a.hist_in, hist_base + (int64_t)r * DVT + cc) : 0.f;
  }
  __syncthreads();

  for (int t0 = 0; t0 < L; t0 += TC) {
    const int nt = (L - t0) < TC ? (L - t0) : TC;
    // a. rows of this step, feature map applied; rows past the end are zeros
    for (int c8 = tid; c8 < TC * (D / 8); c8 += 256) {
      const int t = c8 / (D / 8), i0 = (c8 % (D / 8)) * 8;
      float xq[8], xk[8], xv[8];
      if (t < nt) {
        const int64_t off = base + (int64_t)(t0 + t) * a.st + i0;
        Io::load8(a.q, off, xq);
        Io::load8(a.k, off, xk);
        Io::load8(a.v, base_v + (int64_t)(t0 + t) * a.st_v + i0, xv);
#pragma unroll
        for (int e = 0; e < 8; ++e) { xq[e] = phi_any(xq[e], a.relu); xk[e] = phi_any(xk[e], a.relu); }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) { xq[e] = 0.f; xk[e] = 0.f; xv[e] = 0.f; }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        fq[t * (D + 1) + i0 + e] = xq[e];
        fk[t * (D + 1) + i0 + e] = xk[e];
        vv[(HMAX + t) * D + i0 + e] = xv[e];
      }
    }
    __syncthreads();
    // b. masked in-step scores P[t][s] = phi(q_t).phi(k_s), s <= t
    for (int p = tid; p < TC * TC; p += 256) {
      const int t = p / TC, s = p % TC;
      float acc = 0.f;
      if (s <= t && t < nt) {
        const float* x = fq + t * (D + 1);
        const float* y = fk + s * (D + 1);
#pragma unroll 8
        for (int i = 0; i < D; ++i) acc = fmaf(x[i], y[i], acc);
      }
      P[t * (TC + 1) + s] = acc;
    }
    __syncthreads();
    if (tid < nt) {
      float dsum = a.eps;
      for (int s = 0; s <= tid; ++s) dsum += P[tid * (TC + 1) + s];
      const float* x = fq + tid * (D + 1);
      float dz = 0.f;
      for (int i = 0; i < D; ++i) dz = fmaf(x[i], zz[i], dz);
      den[tid] = dsum + dz;
    }
    __syncthreads();
    // c. outputs: in-step part + carried state, normalised, plus the causal conv
    for (int t = tg; t < nt; t += NG) {
      float num = 0.f;
      for (int s = 0; s <= t; ++s) num = fmaf(P[t * (TC + 1) + s], vv[(HMAX + s) * D + c], num);
      const float* x = fq + t * (D + 1);
#pragma unroll 8
      for (int i = 0; i < D; ++i) num = fmaf(x[i], S[i * D + c], num);
      float u = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (j < Kc) u = fmaf(wreg[j], vv[(HMAX + t - j) * D + c], u);
      Io::store1(a.out, base_v + (int64_t)(t0 + t) * a.st_v + c, num / den[t] + u);
    }
    __syncthreads();
    // d. carry: S += phi(K)^T V, z += colsum phi(K); history slides forward by nt rows
    for (int i = tg; i < D; i += NG) {
      float acc = S[i * D + c];
      for (int s = 0; s < nt; ++s) acc = fmaf(fk[s * (D + 1) + i], vv[(HMAX + s) * D + c], acc);
      S[i * D + c] = acc;
    }
    if (tid < D) {
      float zs = zz[tid];
      for (int s = 0; s < nt; ++s) zs += fk[s * (D + 1) + tid];
      zz[tid] = zs;
      for (int r = 0; r < HMAX; ++r) vv[r * D + tid] = vv[(r + nt) * D + tid];
    }
    __syncthreads();
  }

  if (a.S_out)
    for (int e = tid; e < D * D; e += 256) a.S_out[S_base + (int64_t)(e / D) * DVT + e % D] = S[e];
  if (a.z_out && tid < D && hx.blk == 0) a.z_out[(size_t)bh * D + tid] = zz[tid];   // the same in every value block
  if (a.hist_out)
    for (int e = tid; e < (Kc - 1) * D; e += 256) {
      const int r = e / D, cc = e % D;
      Io::store1(a.hist_out, hist_base + (int64_t)r * DVT + cc, vv[(HMAX - (Kc - 1) + r) * D + cc]);
    }
}

// The three-branch form (grouped linear attention over the groups before a token's own, weight alpha + causal
// softmax attention inside its group + masked conv) with fp32 arithmetic: the path for fp32 rows, and for
// groups of 256 tokens (the group size of the paper's FLASH experiment, Sec. 5 "Settings") whatever the rows.
// One workgroup walks one (b, h) group by group and, inside a group, token by token; S and z are only advanced
// at the end of a group, which is exactly what the linear branch is defined on.  The state sits in registers
// (thread (c, tg) holds S[i][c] for i = tg, tg + NG, ...), the group's raw key rows and value rows in LDS in
// the i/o dtype.  Exact to fp32 rounding; not built for speed.
namespace {
template <typename Io, int D, int GCT>
struct GroupedSimtLayout {
  typedef typename Io::elem elem;
  static constexpr int KSTR = D + 4 / (int)sizeof(elem);                  // key row stride: one 4-byte word of padding
  static constexpr int KR = 0;                                             // [GCT][KSTR] raw key rows of the group (elem)
  static constexpr int VV = KR + GCT * KSTR * (int)sizeof(elem);           // [HMAX+GCT][D]: history rows, then the group's value rows (elem)
  static constexpr int F0 = (VV + (HMAX + GCT) * D * (int)sizeof(elem) + 15) / 16 * 16;   // floats from here
  static constexpr int QR = 0;                        // [D] raw q_t
  static constexpr int FQ = QR + D;                   // [D] phi(q_t)
  static constexpr int LG = FQ + D;                   // [GCT] logits, then weights
  static constexpr int PART = LG + GCT;               // [256 / D][D] partial outputs
  static constexpr int ZZ = PART + 256;               // [D]
  static constexpr int SCAL = ZZ + D;                 // [16]: alpha / denominator; per-wave maxima and sums
  static constexpr int NFLOAT = SCAL + 16;
  static constexpr int TOTAL = F0 + NFLOAT * (int)sizeof(float);
};
__device__ __forceinline__ float elem_to_f32(float x) { return x; }
__device__ __forceinline__ float elem_to_f32(uint16_t x) { return bf16_bits_to_f32(x); }
}  // namespace

template <typename Io, int D, int GCT>
__global__ __launch_bounds__(256) void prefill_grouped_simt_kernel(PrefillArgs a) {
  using Lay = GroupedSimtLayout<Io, D, GCT>;
  typedef typename Io::elem elem;
  constexpr int NG = 256 / D;
  constexpr int NS = D / NG;                           // state rows per thread
  constexpr int KSTR = Lay::KSTR;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  elem* kr = reinterpret_cast<elem*>(smem + Lay::KR);
  elem* vv = reinterpret_cast<elem*>(smem + Lay::VV);
  float* fl = reinterpret_cast<float*>(smem + Lay::F0);
  float* qr = fl + Lay::QR;
  float* fq = fl + Lay::FQ;
  float* lg = fl + Lay::LG;
  float* part = fl + Lay::PART;
  float* zz = fl + Lay::ZZ;
  float* scal = fl + Lay::SCAL;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bh = blockIdx.x, b = bh / a.H, h = bh % a.H;
  const int Kc = a.Kc, L = a.L;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const int c = tid % D, tg = tid / D;
  static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
  constexpr float inv_sqrt_d = D == 64 ? 0.125f : 0.08838834764831845f;

  float wreg[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) wreg[j] = (j < Kc && !a.no_conv) ? a.conv_w[((size_t)h * D + c) * Kc + j] : 0.f;
  float Sreg[NS];                                      // S[tg + NG m][c]
#pragma unroll
  for (int m = 0; m < NS; ++m) Sreg[m] = a.S_in ? a.S_in[(size_t)bh * D * D + (size_t)(tg + NG * m) * D + c] : 0.f;
  if (tid < D) zz[tid] = a.z_in ? a.z_in[(size_t)bh * D + tid] : 0.f;
  for (int e = tid; e < HMAX * D; e += 256) {
    const int row = e / D, cc = e % D;
    const int r = row - (HMAX - (Kc - 1));   // row of the incoming history, oldest first
    if (r >= 0 && a.hist_in) vv[e] = static_cast<const elem*>(a.hist_in)[((int64_t)bh * (Kc - 1) + r) * D + cc];
    else vv[e] = (elem)0;
  }
  __syncthreads();

  for (int t0 = 0; t0 < L; t0 += GCT) {
    const int nt = (L - t0) < GCT ? (L - t0) : GCT;
    // a. the group's raw key and value rows, as they are
    for (int e = tid; e < nt * D; e += 256) {
      const int t = e / D, i = e % D;
      const int64_t off = base + (int64_t)(t0 + t) * a.st + i;
      kr[t * KSTR + i] = static_cast<const elem*>(a.k)[off];
      vv[(HMAX + t) * D + i] = static_cast<const elem*>(a.v)[off];
    }
    __syncthreads();
    for (int t = 0; t < nt; ++t) {
      // b. the token's query, raw and under the feature map
      if (tid < D) {
        const float x = Io::load1(a.q, base + (int64_t)(t0 + t) * a.st + tid);
        qr[tid] = x;
        fq[tid] = phi_any(x, a.relu);
      }
      __syncthreads();
      // c. logits against the group's rows up to the token (four lanes per row); the linear normaliser
      for (int i0 = 0; i0 <= t; i0 += 64) {
        const int i = i0 + tid / 4, sub = tid % 4;
        float acc = 0.f;
        if (i <= t) {
          const elem* y = kr + i * KSTR + sub * (D / 4);
          const float* x = qr + sub * (D / 4);
#pragma unroll 8
          for (int f = 0; f < D / 4; ++f) acc = fmaf(x[f], elem_to_f32(y[f]), acc);
        }
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        if (sub == 0 && i < GCT) lg[i] = acc * inv_sqrt_d;
      }
      if (wave == 3) {                          // the last wave: phi(q_t).z
        float dz = 0.f;
        for (int f = lane; f < D; f += 64) dz = fmaf(fq[f], zz[f], dz);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) dz += __shfl_xor(dz, off);
        if (lane == 0) {
          const float gden = dz + a.eps;
          scal[0] = gden != 0.f ? a.alpha / gden : 0.f;
        }
      }
      __syncthreads();
      // d. softmax over rows 0..t, one row per thread: largest logit and mass over the workgroup
      {
        const bool seen = tid < GCT && tid <= t;
        const float x = seen ? lg[tid] : -INFINITY;
        float top = x;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) top = fmaxf(top, __shfl_xor(top, off));
        if (lane == 0) scal[4 + wave] = top;
        __syncthreads();
        top = fmaxf(fmaxf(scal[4], scal[5]), fmaxf(scal[6], scal[7]));   // row 0 is always seen: finite
        const float p = seen ? __expf(x - top) : 0.f;
        float mass = p;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mass += __shfl_xor(mass, off);
        if (lane == 0) scal[8 + wave] = mass;
        __syncthreads();
        mass = (scal[8] + scal[9]) + (scal[10] + scal[11]);
        if (tid < GCT) lg[tid] = p / mass;
      }
      __syncthreads();
      // e. both branches for channel c, the features / rows dealt out over the NG thread groups
      {
        float lin = 0.f, loc = 0.f;
#pragma unroll
        for (int m = 0; m < NS; ++m) lin = fmaf(fq[tg + NG * m], Sreg[m], lin);
        for (int s2 = tg; s2 <= t; s2 += NG) loc = fmaf(lg[s2], elem_to_f32(vv[(HMAX + s2) * D + c]), loc);
        part[tg * D + c] = fmaf(scal[0], lin, loc);
      }
      __syncthreads();
      if (tid < D) {
        float y = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) y += part[g * D + tid];
        float u = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (j < Kc) u = fmaf(wreg[j], elem_to_f32(vv[(HMAX + t - j) * D + tid]), u);
        Io::store1(a.out, base + (int64_t)(t0 + t) * a.st + tid, y + u);
      }
      // the next token's step b writes qr, fq (read in c, e: both behind barriers by then); lg, part and scal are
      // written by the next token's c, d, e after barriers of their own
    }
    __syncthreads();
    // f. the group enters the sums: S += phi(K)^T V, z += colsum phi(K); the history slides forward by nt rows
    for (int s2 = 0; s2 < nt; ++s2) {
      const float x = elem_to_f32(vv[(HMAX + s2) * D + c]);
#pragma unroll
      for (int m = 0; m < NS; ++m) Sreg[m] = fmaf(phi_any(elem_to_f32(kr[s2 * KSTR + tg + NG * m]), a.relu), x, Sreg[m]);
    }
    if (tid < D) {
      float zs = zz[tid];
      for (int s2 = 0; s2 < nt; ++s2) zs += phi_any(elem_to_f32(kr[s2 * KSTR + tid]), a.relu);
      zz[tid] = zs;
      for (int r = 0; r < HMAX; ++r) vv[r * D + tid] = vv[(r + nt) * D + tid];
    }
    __syncthreads();
  }

  if (a.S_out) {
#pragma unroll
    for (int m = 0; m < NS; ++m) a.S_out[(size_t)bh * D * D + (size_t)(tg + NG * m) * D + c] = Sreg[m];
  }
  if (a.z_out && tid < D) a.z_out[(size_t)bh * D + tid] = zz[tid];
  if (a.hist_out)
    for (int e = tid; e < (Kc - 1) * D; e += 256) {
      const int r = e / D, cc = e % D;
      static_cast<elem*>(a.hist_out)[((int64_t)bh * (Kc - 1) + r) * D + cc] = vv[(HMAX - (Kc - 1) + r) * D + cc];
    }
}

template <typename Io, int D, int GCT>
static hipError_t launch_grouped_one(const PrefillArgs& a, hipStream_t st) {
  constexpr int bytes = GroupedSimtLayout<Io, D, GCT>::TOTAL;
  static_assert(bytes <= 160 * 1024, "LDS");
  auto kern = prefill_grouped_simt_kernel<Io, D, GCT>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H)), dim3(256), bytes, st, a);
  return hipGetLastError();
}

// fp32 rows of 128 elements in groups of 256 would need 266 KB of LDS for the group's rows: no kernel.
bool prefill_grouped_simt_available(bool bf16, int d, int group) {
  return (group == 64 || group == 256) && (d == 64 || d == 128) && (bf16 || d == 64 || group == 64);
}

hipError_t launch_prefill_grouped_simt(const PrefillArgs& a, bool bf16, int d, hipStream_t st) {
  if (a.group == 256) {
    if (bf16) return d == 128 ? launch_grouped_one<IoBf16, 128, 256>(a, st) : launch_grouped_one<IoBf16, 64, 256>(a, st);
    if (d == 64) return launch_grouped_one<IoF32, 64, 256>(a, st);
    return hipErrorInvalidValue;
  }
  if (bf16) return d == 128 ? launch_grouped_one<IoBf16, 128, 64>(a, st) : launch_grouped_one<IoBf16, 64, 64>(a, st);
  return d == 128 ? launch_grouped_one<IoF32, 128, 64>(a, st) : launch_grouped_one<IoF32, 64, 64>(a, st);
}

template <typename Io, int D>
static hipError_t launch_one(const PrefillArgs& a, hipStream_t st) {
  constexpr size_t bytes = sizeof(float) * SimtLayout<D>::TOTAL;
  auto kern = prefill_simt_kernel<Io, D>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, (int)bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H * a.m)), dim3(256), bytes, st, a);
  return hipGetLastError();
}

hipError_t launch_prefill_simt(const PrefillArgs& a, bool bf16, int d, hipStream_t st) {
  if (bf16) return d == 128 ? launch_one<IoBf16, 128>(a, st) : launch_one<IoBf16, 64>(a, st);
  return d == 128 ? launch_one<IoF32, 128>(a, st) : launch_one<IoF32, 64>(a, st);
}

}  // namespace linattn
