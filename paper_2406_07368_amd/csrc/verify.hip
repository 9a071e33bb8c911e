// Speculative verification / decode step (Sec. 4.2; decode = one draft that is
// always kept).  Memory-bound: every head's fp32 state S (d x d) is read once
// and, if any draft is accepted, written once; everything else is tiny.
//
// One workgroup of 256 threads owns the column slice S[:, c0 : c0+CW] of one
// (b, h).  The slice streams through registers in row passes with 16-byte loads
// (rows are contiguous, so a wave reads whole 128..512 B row segments; nontemporal:
// the state is touched once per step), a few
// passes in flight at a time: each row adds its term to the kk read-outs
// phi(q_j)^T S, receives the accepted rank-1 updates and is written straight back.
// The read-outs are then reduced across the threads that share a column group,
// completed with the causal in-block term, normalised, and joined with the
// convolution over (history ++ drafts <= j).
#include "common.h"
#include "kernels.h"

namespace linattn {

template <int D, int CW, int KP>
struct VerifySmem {
  float fq[D][KP];          // phi(q_j)[i], feature-major so one thread reads all drafts of its row
  float fk[D][KP];          // phi(k_j)[i]
  float vv[KP][CW];         // v_j[c0 + c]
  float red[4][KP][CW];     // per-wave partial read-outs
  float amat[KP][KP];       // phi(q_j).phi(k_j') for j' <= j, else 0
  float den[KP];            // phi(q_j).z + sum_j' amat + eps
  float zz[D];
  float wt[8][CW];          // conv taps of the slice's channels, tap-major (taps >= Kc are 0)
  float hh[8][CW];          // hh[t]: the value row t+1 positions before the first draft (t < Kc-1)
};

template <int KP>
__device__ __forceinline__ void load_row(const float* row, float (&f)[KP]) {
  if constexpr (KP >= 4) {
#pragma unroll
    for (int g = 0; g < KP / 4; ++g) {
      f32x4 t = *reinterpret_cast<const f32x4*>(row + 4 * g);
      f[4 * g] = t[0]; f[4 * g + 1] = t[1]; f[4 * g + 2] = t[2]; f[4 * g + 3] = t[3];
    }
  } else {
#pragma unroll
    for (int j = 0; j < KP; ++j) f[j] = row[j];
  }
}

// At most 128 registers per thread for up to 8 drafts, so that four workgroups fit on a compute unit
// and B*H = 1024 heads are all resident at once (a partial second round would run at a fraction of
// the bandwidth).
template <typename Io, int D, int CW, int KP>
__global__ __launch_bounds__(256, (KP <= 8 ? 4 : 2)) void verify_kernel(VerifyArgs a) {
  constexpr int CG = CW / 4;          // float4 column groups per row slice
  constexpr int RPP = 256 / CG;       // rows covered per pass
  constexpr int NPASS = D / RPP;
  static_assert(NPASS >= 1 && RPP * NPASS == D, "tile shape");
  __shared__ VerifySmem<D, CW, KP> sm;

  const int tid = threadIdx.x;
  // value rows of DV = a.dv elements (a multiple of D; DV == D: d_v = d_k): DV / CW column slices per head, and
  // DV is the row length of v, out, hist, conv_w and S
  const int DV = a.dv, nslice = DV / CW;
  const int bh = blockIdx.x / nslice;
  const int c0 = (blockIdx.x % nslice) * CW;
  const int b = bh / a.H, h = bh % a.H;
  const int kk = a.kk, Kc = a.Kc;
  const int cg = tid % CG, r0 = tid / CG;

  // ---- 0. every request of the step is issued before anything waits, the small inputs FIRST: every workgroup of
  //         the launch is about to ask for its state at the same moment, and anything requested after that waits
  //         behind it.  All requests unconditional -- indices past the end are clamped, what they bring is dropped --:
  //         under conditions on the thread index every one of them sat in a block of its own with a full wait at its
  //         end, a dozen trips to memory in a row before the state was asked for. ------------------------------------
  const int64_t tok0 = (int64_t)bh * kk * D;              // q, k
  const int64_t vtok0 = (int64_t)bh * kk * DV;            // v, out
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * DV;
  constexpr int QK_IT = (KP * (D / 8) + 255) / 256;   // 8-element pieces of q and k per thread
  constexpr int V_IT = (KP * (CW / 8) + 255) / 256;
  typename Io::raw8 rq[QK_IT], rk[QK_IT], rv[V_IT];
#pragma unroll
  for (int m = 0; m < QK_IT; ++m) {
    const int c8 = tid + 256 * m;
    const int j = c8 / (D / 8), i0 = (c8 % (D / 8)) * 8;
    const int64_t off = tok0 + (int64_t)(j < kk ? j : kk - 1) * D + i0;
    rq[m] = Io::load_raw8(a.q, off);
    rk[m] = Io::load_raw8(a.k, off);
  }
#pragma unroll
  for (int m = 0; m < V_IT; ++m) {
    const int c8 = tid + 256 * m;
    const int j = c8 / (CW / 8), cc = (c8 % (CW / 8)) * 8;
    rv[m] = Io::load_raw8(a.v, vtok0 + (int64_t)(j < kk ? j : kk - 1) * DV + c0 + cc);
  }
  const float zreg = a.z[(size_t)bh * D + tid % D];
  // taps and history rows of the slice's channels: element e = tid + 256 m of the [8][CW] arrays in LDS
  constexpr int TAP_IT = (8 * CW + 255) / 256;
  float tap_reg[TAP_IT], hist_reg[TAP_IT];
  // (one tap: no history; the request then reads a draft's value row, which is dropped)
  const void* hsrc = Kc > 1 ? a.hist : a.v;
  const int64_t hbase = (Kc > 1 ? hist0 : vtok0) + c0;
#pragma unroll
  for (int m = 0; m < TAP_IT; ++m) {
    const int e = (tid + 256 * m) % (8 * CW);
    const int t = e / CW, cc = e % CW;
    tap_reg[m] = a.conv_w[((size_t)h * DV + c0 + cc) * Kc + (t < Kc ? t : 0)];
    hist_reg[m] = Io::load1(hsrc, hbase + (int64_t)(t < Kc - 1 ? Kc - 2 - t : 0) * DV + cc);
  }
  int n = kk;
  if (a.n_commit) { n = a.n_commit[b]; n = n < 0 ? 0 : (n > kk ? kk : n); }

  // ---- 0. the state slice streams through a window of PD row passes: the first PD loads are
  //         in flight before anything else, each later one is issued when its slot frees up ----
  constexpr int PDW = KP >= 8 ? 2 : 4;        // fewer passes in flight when the read-outs need the registers
  constexpr int PD = NPASS < PDW ? NPASS : PDW;
  float* Sg = a.S + (size_t)bh * D * DV + c0 + 4 * cg;
  f32x4 s[PD];
#pragma unroll
  for (int p = 0; p < PD; ++p) s[p] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Sg + (size_t)(p * RPP + r0) * DV));
  // (values that only some threads use: kept ahead of the state's requests, or the compiler moves their requests down
  // to the uses, behind the state's)
#pragma unroll
  for (int m = 0; m < QK_IT; ++m) { Io::needed_here(rq[m]); Io::needed_here(rk[m]); }
#pragma unroll
  for (int m = 0; m < V_IT; ++m) Io::needed_here(rv[m]);

  // ---- 1. drafts -> LDS (phi applied), normaliser, taps and history -> LDS -----------------------
#pragma unroll
  for (int m = 0; m < QK_IT; ++m) {
    const int c8 = tid + 256 * m;
    const int j = c8 / (D / 8), i0 = (c8 % (D / 8)) * 8;
    if (c8 < KP * (D / 8)) {
      float xq[8], xk[8];
      Io::unpack8(rq[m], xq);
      Io::unpack8(rk[m], xk);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sm.fq[i0 + e][j] = j < kk ? phi_any(xq[e], a.relu) : 0.f;
        sm.fk[i0 + e][j] = j < kk ? phi_any(xk[e], a.relu) : 0.f;
      }
    }
  }
#pragma unroll
  for (int m = 0; m < V_IT; ++m) {
    const int c8 = tid + 256 * m;
    const int j = c8 / (CW / 8), cc = (c8 % (CW / 8)) * 8;
    if (c8 < KP * (CW / 8)) {
      float xv[8];
      Io::unpack8(rv[m], xv);
#pragma unroll
      for (int e = 0; e < 8; ++e) sm.vv[j][cc + e] = j < kk ? xv[e] : 0.f;
    }
  }
  if (tid < D) sm.zz[tid] = zreg;
#pragma unroll
  for (int m = 0; m < TAP_IT; ++m) {
    const int e = tid + 256 * m;
    if (e < 8 * CW) {
      const int t = e / CW, cc = e % CW;
      sm.wt[t][cc] = t < Kc ? tap_reg[m] : 0.f;
      sm.hh[t][cc] = t < Kc - 1 ? hist_reg[m] : 0.f;
    }
  }
  __syncthreads();

  // ---- 2. in-block scores and denominators ----------------------------------------
  {
    constexpr int NPAIR = KP * KP;
    constexpr int TPP = (256 / NPAIR) > 64 ? 64 : (256 / NPAIR);   // threads per (j, j') pair
    if (tid < NPAIR * TPP) {
      const int pair = tid / TPP, sub = tid % TPP;
      const int j = pair / KP, jp = pair % KP;
      float acc = 0.f, dz = 0.f;
      for (int i = sub; i < D; i += TPP) {
        const float fqv = sm.fq[i][j];
        acc += fqv * sm.fk[i][jp];
        dz += fqv * sm.zz[i];
      }
#pragma unroll
      for (int off = TPP / 2; off >= 1; off >>= 1) {
        acc += __shfl_xor(acc, off);
        dz += __shfl_xor(dz, off);
      }
      if (sub == 0) {
        sm.amat[j][jp] = (jp <= j && j < kk) ? acc : 0.f;
        if (jp == 0) sm.den[j] = dz;     // completed below
      }
    }
  }

  // ---- 3. read-outs phi(q_j)^T S from registers; accepted drafts folded in and the row
  //         streamed back as soon as it has been used (reads of later rows are still in flight)
  float acc[KP][4];
#pragma unroll
  for (int j = 0; j < KP; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
  float vr[KP][4];
#pragma unroll
  for (int j = 0; j < KP; ++j) {
    f32x4 t = *reinterpret_cast<const f32x4*>(&sm.vv[j][4 * cg]);
    const bool keep = j < n;
    vr[j][0] = keep ? t[0] : 0.f; vr[j][1] = keep ? t[1] : 0.f;
    vr[j][2] = keep ? t[2] : 0.f; vr[j][3] = keep ? t[3] : 0.f;
  }
#pragma unroll 1
  for (int pb = 0; pb < NPASS; pb += PD) {
#pragma unroll
    for (int q = 0; q < PD; ++q) {
      const int p = pb + q;
      const int i = p * RPP + r0;
      float f[KP], g[KP];
      f32x4 cur = s[q];
      load_row<KP>(&sm.fq[i][0], f);
#pragma unroll
      for (int j = 0; j < KP; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] = fmaf(f[j], cur[e], acc[j][e]);
      if (n > 0) {   // uniform per workgroup; n == 0 leaves the state untouched
        load_row<KP>(&sm.fk[i][0], g);
#pragma unroll
        for (int j = 0; j < KP; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) cur[e] = fmaf(g[j], vr[j][e], cur[e]);
        __builtin_nontemporal_store(cur, reinterpret_cast<f32x4*>(Sg + (size_t)i * DV));
      }
      if (p + PD < NPASS) s[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Sg + (size_t)((p + PD) * RPP + r0) * DV));
    }
  }
  // threads that share a column group sit CG lanes apart inside a wave
#pragma unroll
  for (int off = CG; off < kWave; off <<= 1)
#pragma unroll
    for (int j = 0; j < KP; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[j][e] += __shfl_xor(acc[j][e], off);
  if ((tid % kWave) < CG) {
    const int wv = tid / kWave;
#pragma unroll
    for (int j = 0; j < KP; ++j)
      *reinterpret_cast<f32x4*>(&sm.red[wv][j][4 * cg]) = f32x4{acc[j][0], acc[j][1], acc[j][2], acc[j][3]};
  }
  __syncthreads();
  if (tid < kk) {
    float dsum = sm.den[tid] + a.eps;
    for (int jp = 0; jp <= tid; ++jp) dsum += sm.amat[tid][jp];
    sm.den[tid] = dsum;
  }
  __syncthreads();

  // ---- 4. outputs: normalise, add the causal convolution -------------------------------
  for (int idx = tid; idx < kk * CW; idx += 256) {
    const int j = idx / CW, c = idx % CW;
    float num = sm.red[0][j][c] + sm.red[1][j][c] + sm.red[2][j][c] + sm.red[3][j][c];
    for (int jp = 0; jp <= j; ++jp) num = fmaf(sm.amat[j][jp], sm.vv[jp][c], num);
    float u = 0.f;
    for (int t = 0; t < Kc; ++t) {
      // tap t looks t rows back from draft j: another draft if t <= j, else history row (t - j) back
      const float x = t <= j ? sm.vv[j - t][c] : sm.hh[t - j - 1][c];
      u = fmaf(sm.wt[t][c], x, u);
    }
    Io::store1(a.out, vtok0 + (int64_t)j * DV + c0 + c, num / sm.den[j] + u);
  }

  // ---- 5. the rest of the state: normaliser and history ----------------------------------
  if (n == 0) return;   // uniform per workgroup: nothing accepted, state untouched
  if (nslice == 1 && tid < D) {   // with several slices per head a separate launch updates z
    float zs = sm.zz[tid];
    for (int j = 0; j < n; ++j) zs += sm.fk[tid][j];
    a.z[(size_t)bh * D + tid] = zs;
  }
  if (Kc > 1) {
    __syncthreads();   // every conv read of the old history is done
    for (int c = tid; c < CW; c += 256) {
      for (int r = 0; r < Kc - 1; ++r) {
        const int sidx = n - (Kc - 1) + r;   // position in (history ++ accepted drafts)
        const int64_t dst = hist0 + (int64_t)r * DV + c0 + c;
        if (sidx >= 0) Io::store1(a.hist, dst, sm.vv[sidx][c]);
        else Io::store1(a.hist, dst, sm.hh[-sidx - 1][c]);   // an old history row, -sidx positions back
      }
    }
  }
}

// z += sum of the accepted phi(k_j); used when a head's columns are split over
// several workgroups (they all read the old z, so it cannot be updated by one of them).
template <typename Io, int D>
__global__ __launch_bounds__(256) void verify_z_kernel(VerifyArgs a) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  if (gid >= a.B * a.H * D) return;
  const int bh = gid / D, i = gid % D;
  const int b = bh / a.H;
  // every draft's element requested at once, whatever the count says (a loop up to the count was one trip to memory
  // per draft, one after the other); kept or dropped by select
  constexpr int KMAX = 16;   // drafts per call at most (the entry point refuses more)
  float x[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) x[j] = Io::load1(a.k, ((int64_t)bh * a.kk + (j < a.kk ? j : a.kk - 1)) * D + i);
  float zs = a.z[gid];
  int n = a.kk;
  if (a.n_commit) { n = a.n_commit[b]; n = n < 0 ? 0 : (n > a.kk ? a.kk : n); }
  if (n == 0) return;
#pragma unroll
  for (int j = 0; j < KMAX; ++j) zs += j < n ? phi_any(x[j], a.relu) : 0.f;
  a.z[gid] = zs;
}

// z += sum of the accepted phi(k_j) for every head, as a launch of its own (fp32 sums of fp32 feature maps).
hipError_t launch_verify_z(const VerifyArgs& a, bool bf16, int d, hipStream_t st) {
  const int total = a.B * a.H * d;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (bf16) {
    if (d == 128) hipLaunchKernelGGL((verify_z_kernel<IoBf16, 128>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((verify_z_kernel<IoBf16, 64>), grid, block, 0, st, a);
  } else {
    if (d == 128) hipLaunchKernelGGL((verify_z_kernel<IoF32, 128>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((verify_z_kernel<IoF32, 64>), grid, block, 0, st, a);
  }
  return hipGetLastError();
}

template <typename Io, int D, int CW>
static hipError_t launch_kp(const VerifyArgs& a, hipStream_t st) {
  const dim3 grid((unsigned)(a.B * a.H * (a.dv / CW))), block(256);
  if (a.kk <= 1) hipLaunchKernelGGL((verify_kernel<Io, D, CW, 1>), grid, block, 0, st, a);
  else if (a.kk <= 4) hipLaunchKernelGGL((verify_kernel<Io, D, CW, 4>), grid, block, 0, st, a);
  else if (a.kk <= 8) hipLaunchKernelGGL((verify_kernel<Io, D, CW, 8>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((verify_kernel<Io, D, CW, 16>), grid, block, 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.dv / CW > 1) {
    const int total = a.B * a.H * D;
    hipLaunchKernelGGL((verify_z_kernel<Io, D>), dim3((total + 255) / 256), block, 0, st, a);
    e = hipGetLastError();
  }
  return e;
}

template <typename Io, int D>
static hipError_t launch_split(const VerifyArgs& a, int nsplit, hipStream_t st) {
  if (nsplit <= 1) return launch_kp<Io, D, D>(a, st);
  if (nsplit == 2) return launch_kp<Io, D, D / 2>(a, st);
  return launch_kp<Io, D, D / 4>(a, st);
}

// Columns of a head are split over 1, 2 or 4 workgroups so that small B*H still
// puts enough workgroups on the 256 compute units.
int verify_pick_split(int BH) {
  if (BH >= 768) return 1;
  if (BH >= 384) return 2;
  return 4;
}

hipError_t launch_verify(const VerifyArgs& a, bool bf16, int d, int nsplit, hipStream_t st) {
  if (bf16) return d == 128 ? launch_split<IoBf16, 128>(a, nsplit, st) : launch_split<IoBf16, 64>(a, nsplit, st);
  return d == 128 ? launch_split<IoF32, 128>(a, nsplit, st) : launch_split<IoF32, 64>(a, nsplit, st);
}

}  // namespace linattn
