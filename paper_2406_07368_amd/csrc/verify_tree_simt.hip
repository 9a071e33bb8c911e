// Tree-structured verification (Sec. 4.2, "Proposed Solution") for fp32 candidates: the same function as
// verify_tree.hip -- candidate i is scored from the verified state and the candidates on its own root path, its
// conv window is that path read backwards, then the history; the state moves along the root path of the accepted
// candidate -- in exact fp32 multiply-adds on the vector ALUs, so that fp32 rows meet the fp32 bar.  One workgroup of
// 256 threads per (b, h); a thread owns one value channel and one of 256 / d runs of key features, holds that part
// of its state column in registers from the one read of the state to the one write, and the parts are added up through
// LDS in a fixed order.  The parity path for fp32, not built for speed.
#include "common.h"
#include "kernels.h"

namespace linattn {

namespace {

constexpr int TS_HALO = 8;   // value rows before the candidates that the taps can reach (Kc - 1 <= 7)
constexpr int TS_KT = 64;    // candidates per call at most

template <int D>
struct VtsCfg {
  static constexpr int NF = 256 / D;          // runs of key features (parts of a state column) per channel
  static constexpr int RPP = D / NF;          // state rows per part
  static constexpr int FS = D + 4;            // rows of phi(Q), phi(K): 16-byte reads
  static constexpr int AS = TS_KT + 2;        // rows of the scores: column 64 is phi(q).z
};

template <int D>
struct VtsSmem {
  using G = VtsCfg<D>;
  float fq[TS_KT * G::FS];                    // later: partial read-outs of the parts above the first
  float fk[TS_KT * G::FS];
  float v[(TS_HALO + TS_KT) * D];             // row r: history (r < 8: the row 8 - r positions back), then candidate r - 8
  float A[TS_KT * G::AS];                     // A[i][a] = phi(q_i).phi(k_a) for a on the root path of i, else 0
  float w[8 * D];                             // taps, tap-major; zeros beyond Kc
  float z[D];
  float den[TS_KT];
  unsigned long long onpath[TS_KT];
  int parent[TS_KT];
  uint8_t taprow[TS_KT][8];
};

}  // namespace

template <typename Io, int D>
__global__ __launch_bounds__(256) void verify_tree_simt_kernel(VerifyTreeArgs a) {
  using G = VtsCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  VtsSmem<D>& sm = *reinterpret_cast<VtsSmem<D>*>(smem);
  const int tid = threadIdx.x;
  const int bh = blockIdx.x, b = bh / a.H, h = bh % a.H;
  const int n = a.n, Kc = a.Kc;
  const int c = tid % D, part = tid / D;
  const int64_t tok0 = (int64_t)bh * n * D;
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * D;

  // ---- candidates -> LDS: phi(Q), phi(K), V (rows >= n are zero rows); history, taps, z -------------------------
  for (int piece = tid; piece < TS_KT * (D / 8); piece += 256) {
    const int dj = piece / (D / 8), i0 = 8 * (piece % (D / 8));
    float xq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, xk[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float xv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (dj < n) {
      Io::load8(a.q, tok0 + (int64_t)dj * D + i0, xq);
      Io::load8(a.k, tok0 + (int64_t)dj * D + i0, xk);
      Io::load8(a.v, tok0 + (int64_t)dj * D + i0, xv);
#pragma unroll
      for (int e = 0; e < 8; ++e) { xq[e] = phi_any(xq[e], a.relu); xk[e] = phi_any(xk[e], a.relu); }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sm.fq[dj * G::FS + i0 + e] = xq[e];
      sm.fk[dj * G::FS + i0 + e] = xk[e];
      sm.v[(TS_HALO + dj) * D + i0 + e] = xv[e];
    }
  }
  if (part == 0) {
    sm.z[c] = a.z[(size_t)bh * D + c];
#pragma unroll
    for (int t = 0; t < 8; ++t) sm.w[t * D + c] = t < Kc ? a.conv_w[((size_t)h * D + c) * Kc + t] : 0.f;
  } else if (part == 1) {
#pragma unroll
    for (int r = 0; r < TS_HALO; ++r) {
      const int back = TS_HALO - r;             // 1 .. 8
      sm.v[r * D + c] = back <= Kc - 1 ? Io::load1(a.hist, hist0 + (int64_t)(Kc - 1 - back) * D + c) : 0.f;
    }
  }
  if (tid < TS_KT) {
    int par = -1;
    if (tid < n) { par = a.parent[tid]; par = (par < -1 || par >= tid) ? -1 : par; }   // a malformed entry starts a new root
    sm.parent[tid] = par;
  }
  int acc_node = -1;
  if (a.accept) { acc_node = a.accept[b]; acc_node = (acc_node < 0 || acc_node >= n) ? -1 : acc_node; }
  // this thread's part of its state column: requested now, needed after the scores
  float Sreg[G::RPP];
  {
    const float* Sp = a.S + (size_t)bh * D * D + (size_t)part * G::RPP * D + c;
#pragma unroll
    for (int j = 0; j < G::RPP; ++j) Sreg[j] = __builtin_nontemporal_load(Sp + (size_t)j * D);
  }
  __syncthreads();

  // ---- the tree: root paths as bit sets, and tap by tap the row a candidate's convolution reads ---------------------
  if (tid < TS_KT) {
    unsigned long long bits = 0ull;
    int steps = 0;
    if (tid < n) {
      for (int x = tid; x >= 0; x = sm.parent[x]) {      // at most n steps: parents have smaller indices
        bits |= 1ull << x;
        if (steps < 8) sm.taprow[tid][steps] = (uint8_t)(TS_HALO + x);
        ++steps;
      }
    }
    for (int t = steps; t < 8; ++t) {
      const int back = t - steps + 1;                    // rows into the history
      sm.taprow[tid][t] = (uint8_t)(back <= TS_HALO ? TS_HALO - back : 0);
    }
    sm.onpath[tid] = bits;
  }
  __syncthreads();

  // ---- scores of the pairs on a root path, and phi(q).z as column 64 --------------------------------------------------
  for (int idx = tid; idx < TS_KT * (TS_KT + 1); idx += 256) {
    const int i = idx / (TS_KT + 1), x = idx % (TS_KT + 1);
    float s = 0.f;
    if (i < n && (x == TS_KT || ((sm.onpath[i] >> x) & 1ull))) {
      const float* qa = sm.fq + i * G::FS;
      const float* kb = x == TS_KT ? sm.z : sm.fk + x * G::FS;
      for (int f = 0; f < D; f += 4) {
        const f32x4 qv = *reinterpret_cast<const f32x4*>(qa + f), kv = *reinterpret_cast<const f32x4*>(kb + f);
        s = fmaf(qv[0], kv[0], s); s = fmaf(qv[1], kv[1], s); s = fmaf(qv[2], kv[2], s); s = fmaf(qv[3], kv[3], s);
      }
    }
    sm.A[i * G::AS + x] = s;
  }
  __syncthreads();
  if (tid < TS_KT) {
    float den = a.eps;
    for (int x = 0; x <= TS_KT; ++x) den += sm.A[tid * G::AS + x];
    sm.den[tid] = den;
  }

  // ---- read-out: this thread's part of  phi(q_i)^T S[:, c]  for all candidates, plus its share of the path's own rows --
  float acc[TS_KT];
#pragma unroll
  for (int i = 0; i < TS_KT; ++i) {
    const float* qa = sm.fq + i * G::FS + part * G::RPP;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < G::RPP; j += 4) {
      const f32x4 qv = *reinterpret_cast<const f32x4*>(qa + j);
      s = fmaf(qv[0], Sreg[j], s); s = fmaf(qv[1], Sreg[j + 1], s); s = fmaf(qv[2], Sreg[j + 2], s); s = fmaf(qv[3], Sreg[j + 3], s);
    }
    acc[i] = s;
  }
  {
    constexpr int APP = TS_KT / G::NF;                   // path rows per part
    for (int x = part * APP; x < (part + 1) * APP; ++x) {
      if (x >= n) break;                                 // uniform per wave (a wave lies in one part)
      const float va = sm.v[(TS_HALO + x) * D + c];
#pragma unroll
      for (int i = 0; i < TS_KT; ++i) acc[i] = fmaf(sm.A[i * G::AS + x], va, acc[i]);
    }
  }
  // the parts add up in a fixed order through the memory of phi(Q), which nobody reads any more
  float* R = sm.fq;
  for (int p = 1; p < G::NF; ++p) {
    __syncthreads();
    if (part == p) {
#pragma unroll
      for (int i = 0; i < TS_KT; ++i) R[i * D + c] = acc[i];
    }
    __syncthreads();
    if (part == 0) {
#pragma unroll
      for (int i = 0; i < TS_KT; ++i) acc[i] += R[i * D + c];
    }
  }
  static_assert(TS_KT * D <= TS_KT * VtsCfg<D>::FS, "the partial read-outs fit in the memory of phi(Q)");

  // ---- outputs: normalise, add the convolution gathered along the root path ---------------------------------------------
  if (part == 0) {
#pragma unroll
    for (int i = 0; i < TS_KT; ++i) {
      if (i < n) {
        float u = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) u = fmaf(sm.w[t * D + c], sm.v[sm.taprow[i][t] * D + c], u);
        Io::store1(a.out, tok0 + (int64_t)i * D + c, acc[i] / sm.den[i] + u);
      }
    }
  }

  // ---- the state moves along the accepted root path ---------------------------------------------------------------------
  if (acc_node < 0) return;                              // uniform per workgroup: the state stays bit-unchanged
  const unsigned long long commit = sm.onpath[acc_node];
  for (int x = 0; x < n; ++x) {
    if (!((commit >> x) & 1ull)) continue;               // uniform
    const float va = sm.v[(TS_HALO + x) * D + c];
    const float* kb = sm.fk + x * G::FS + part * G::RPP;
#pragma unroll
    for (int j = 0; j < G::RPP; j += 4) {
      const f32x4 kv = *reinterpret_cast<const f32x4*>(kb + j);
      Sreg[j] = fmaf(kv[0], va, Sreg[j]); Sreg[j + 1] = fmaf(kv[1], va, Sreg[j + 1]);
      Sreg[j + 2] = fmaf(kv[2], va, Sreg[j + 2]); Sreg[j + 3] = fmaf(kv[3], va, Sreg[j + 3]);
    }
  }
  {
    float* Sp = a.S + (size_t)bh * D * D + (size_t)part * G::RPP * D + c;
#pragma unroll
    for (int j = 0; j < G::RPP; ++j) __builtin_nontemporal_store(Sreg[j], Sp + (size_t)j * D);
  }
  if (part == 0) {
    float zs = sm.z[c];
    for (int x = 0; x < n; ++x)
      if ((commit >> x) & 1ull) zs += sm.fk[x * G::FS + c];
    a.z[(size_t)bh * D + c] = zs;
  } else if (part == 1) {
    // the last Kc-1 rows of (history ++ accepted path) are what the taps 0..Kc-2 of the accepted candidate read
    for (int r = 0; r < Kc - 1; ++r)
      Io::store1(a.hist, hist0 + (int64_t)r * D + c, sm.v[sm.taprow[acc_node][Kc - 2 - r] * D + c]);
  }
}

template <typename Io, int D>
static hipError_t launch_vts(const VerifyTreeArgs& a, hipStream_t st) {
  auto kern = verify_tree_simt_kernel<Io, D>;
  constexpr int LDS = (int)sizeof(VtsSmem<D>);
  static_assert(LDS <= 160 * 1024, "LDS");
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, LDS);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H)), dim3(256), LDS, st, a);
  return hipGetLastError();
}

hipError_t launch_verify_tree_simt(const VerifyTreeArgs& a, int d, hipStream_t st) {
  return d == 128 ? launch_vts<IoF32, 128>(a, st) : launch_vts<IoF32, 64>(a, st);
}

}  // namespace linattn
