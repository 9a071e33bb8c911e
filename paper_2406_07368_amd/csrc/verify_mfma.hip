// Speculative verification / decode step on the matrix cores (Sec. 4.2), for bf16
// drafts and a head that is not split over workgroups.
//
// The step is one group of the chunked form with at most 16 tokens: with the drafts'
// phi(Q), phi(K), V as bf16 rows in LDS and the fp32 state S of the head as MFMA accumulators,
//
//   O^T  = S0^T phi(Q)^T + V^T P^T        P^T = causal(phi(K) phi(Q)^T)  (select mask)
//   S   += phi(K_acc)^T V                 K_acc: rows of the accepted drafts, the others zero
//
// exactly as in the prefill kernel, with bf16 operands and fp32 accumulation; S is rounded to
// bf16 for the read-out only, the stored state stays fp32.  Unlike the prefill, the state update
// takes phi(k) as the sum of two bf16 terms (two MFMAs per tile): the state lives on through
// thousands of such steps, the matrix cores are idle most of the step, and this way every
// product that enters S carries sixteen significant bits of phi(k) -- the same state, to 1e-5,
// as the streaming kernel's fp32 products.
// The work on the vector ALUs no longer grows with the number of drafts, which is what
// held the streaming form back at k = 4 and k = 8.
//
// One workgroup per (b, h), D/32 waves; wave w owns value channels 32w..32w+31, i.e. the
// column block S[:, 32w:32w+32] as D/32 accumulator tiles (lane <-> channel, register <->
// feature).  Every lane requests its 4 D/32 state words first thing (a half wave reads one
// whole 128-byte row segment per request), then the drafts are prepared and scored while
// the state is on its way; the updated tiles go straight back.  n_commit == 0 writes nothing.
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D>
struct VmCfg {
  static constexpr int NW = D / 32;
  static constexpr int NT = NW * 64;
  static constexpr int KT = 16;              // draft rows in LDS (LINATTN_MAX_DRAFT)
  static constexpr int IB = D / 32;
  static constexpr int KSD = D / 16;
  static constexpr int QS = D + 4;           // phi(Q): 8-byte row reads
  static constexpr int KS = D + 8;           // phi(K): 16-byte row reads, transpose reads
  static constexpr int VS = D + 4;           // history ++ drafts: transpose reads, 8-byte row reads
  static constexpr int PS = 24;              // P[j][i], 16-byte row reads
};

template <int D>
struct VmSmem {
  using G = VmCfg<D>;
  __attribute__((aligned(16))) uint16_t q[G::KT * G::QS];
  __attribute__((aligned(16))) uint16_t k[G::KT * G::KS];            // phi(K) rounded to bf16
  __attribute__((aligned(16))) uint16_t klo[G::KT * G::KS];          // what the rounding dropped, as bf16
  __attribute__((aligned(16))) uint16_t v[(HALO + G::KT) * G::VS];   // row r = draft r - HALO
  __attribute__((aligned(16))) uint16_t p[G::NW][G::KT * G::PS];     // each wave's own copy of the scores
  __attribute__((aligned(16))) float w[8 * D];                       // conv taps, tap-major
  __attribute__((aligned(16))) float z[D];
};

}  // namespace

template <int D>
__global__ __launch_bounds__(D * 2, 4) void verify_mfma_kernel(VerifyArgs a) {
  using G = VmCfg<D>;
  __shared__ VmSmem<D> sm;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  // Value rows of DV = a.dv = m D elements: one workgroup per (b, h, block of D value channels).  The blocks of a head
  // share q, k and z (each computes the feature maps and scores for itself: the matrix cores are idle most of the
  // step) and own their channels of v, out, hist, conv_w and of the rows of S.  DV == D: one block per head.
  const int DV = a.dv, nblk = DV / D;
  const int bh = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int b = bh / a.H, h = bh % a.H;
  const int kk = a.kk, Kc = a.Kc;
  const int cw = 32 * w + l32;               // the channel this lane owns in the state tiles

  // ---- the drafts and the other small inputs are requested first, then the state ---------------
  const int64_t tok0 = (int64_t)bh * kk * D;                                    // q, k
  const int64_t vtok0 = (int64_t)bh * kk * DV + (int64_t)blk * D;               // v, out: rows of DV elements
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * DV + (int64_t)blk * D;
  const int dj = tid / (D / 8), di0 = 8 * (tid % (D / 8));   // one 8-element piece of q, k, v per thread
  u32x4 rq = {0, 0, 0, 0}, rk = {0, 0, 0, 0}, rv = {0, 0, 0, 0};
  if (dj < kk) {
    rq = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.q) + tok0 + (int64_t)dj * D + di0);
    rk = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.k) + tok0 + (int64_t)dj * D + di0);
    rv = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.v) + vtok0 + (int64_t)dj * DV + di0);
  }
  // taps, history and z: channel tid % D; the lower D threads take the taps and z, the upper D the history
  const int cc = tid % D, upper = tid / D;
  float zreg = 0.f;
  uint32_t aux[8];
  if (!upper) {
    zreg = a.z[(size_t)bh * D + cc];
#pragma unroll
    for (int t = 0; t < 8; ++t) aux[t] = t < Kc ? __float_as_uint(a.conv_w[((size_t)h * DV + blk * D + cc) * Kc + t]) : 0u;
  } else {
#pragma unroll
    for (int r = 0; r < HALO; ++r) {          // LDS row r holds the value row HALO - r positions before the drafts
      const int back = HALO - r;              // 1 .. HALO
      aux[r] = back <= Kc - 1 ? static_cast<const uint16_t*>(a.hist)[hist0 + (int64_t)(Kc - 1 - back) * DV + cc] : 0u;
    }
  }
  int n = kk;
  if (a.n_commit) { n = a.n_commit[b]; n = n < 0 ? 0 : (n > kk ? kk : n); }

  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw]
  // Buffer addressing (descriptor of this head's 4 d^2 bytes in scalar registers + one 32-bit lane
  // offset + a constant per request), so that the 4 D/32 requests need no address registers of their own.
  // The state is touched once per step: the requests carry the nontemporal policy (last argument 2),
  // which on this chip is worth 13 % of the step time.
  const __amdgpu_buffer_rsrc_t Srs =
      __builtin_amdgcn_make_buffer_rsrc(a.S + (size_t)bh * D * DV + (size_t)blk * D, 0, (D * DV - blk * D) * 4, 0x00020000);
  const int row_bytes = DV * 4;              // D * 4 when the value rows are as wide as the key rows: a constant then
  const int so = 4 * hi * row_bytes + cw * 4;
  f32x16 Sacc[G::IB];
#pragma unroll
  for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      Sacc[ib][r] = __builtin_bit_cast(
          float, __builtin_amdgcn_raw_buffer_load_b32(Srs, so, (32 * ib + 8 * (r >> 2) + (r & 3)) * row_bytes, 2));

  // ---- drafts -> LDS: phi(Q), phi(K) as bf16 rows (rows >= kk are zero rows), V, history, z, taps --
  {
    u32x4 qp = phi_pack8(rq, a.relu), kp, kl;
    phi_split8(rk, a.relu, kp, kl);
    if (dj >= kk) { qp = u32x4{0, 0, 0, 0}; kp = u32x4{0, 0, 0, 0}; kl = u32x4{0, 0, 0, 0}; }
    u32x2* qrow = reinterpret_cast<u32x2*>(sm.q + dj * G::QS + di0);
    qrow[0] = u32x2{qp[0], qp[1]};
    qrow[1] = u32x2{qp[2], qp[3]};
    *reinterpret_cast<u32x4*>(sm.k + dj * G::KS + di0) = kp;
    *reinterpret_cast<u32x4*>(sm.klo + dj * G::KS + di0) = kl;
    u32x2* vrow = reinterpret_cast<u32x2*>(sm.v + (HALO + dj) * G::VS + di0);
    vrow[0] = u32x2{rv[0], rv[1]};
    vrow[1] = u32x2{rv[2], rv[3]};
    if (!upper) {
      sm.z[cc] = zreg;
#pragma unroll
      for (int t = 0; t < 8; ++t) sm.w[t * D + cc] = __uint_as_float(aux[t]);
    } else {
#pragma unroll
      for (int r = 0; r < HALO; ++r) sm.v[r * G::VS + cc] = (uint16_t)aux[r];
    }
  }
  __syncthreads();

  const int jr = l32 & 15;                   // the draft a lane stands for where lanes are tokens (lanes 16..31 repeat)
  // ---- scores: P^T = phi(K) phi(Q)^T, causal by select; every wave computes its own copy ---------
  float rs = 0.f;
  {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const uint16_t* ka = sm.k + jr * G::KS + 8 * hi;
    const uint16_t* qb = sm.q + jr * G::QS + 8 * hi;
    constexpr int QB = 2;                    // feature steps per batch of LDS reads (the state tiles hold half the registers)
#pragma unroll
    for (int k0 = 0; k0 < G::KSD; k0 += QB) {
      bf16x8 ak[QB], bq[QB];
#pragma unroll
      for (int k2 = 0; k2 < QB; ++k2) {
        ak[k2] = lds_row8(ka + 16 * (k0 + k2));
        bq[k2] = cat4(lds_row4(qb + 16 * (k0 + k2)), lds_row4(qb + 16 * (k0 + k2) + 4));
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k2 = 0; k2 < QB; ++k2) acc = mfma(ak[k2], bq[k2], acc);
      __builtin_amdgcn_sched_barrier(0);
    }
    // acc[r]: source draft i = 8(r/4) + 4hi + r%4 (rows 16..31 of the tile repeat 0..15), query draft j = l32
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      float x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 8 * g + 4 * hi + e;
        x[e] = (i <= l32 && l32 < kk) ? acc[4 * g + e] : 0.f;   // select, never multiply: later drafts cannot leak
        rs += x[e];
      }
      if (l32 < G::KT)
        *reinterpret_cast<u32x2*>(sm.p[w] + l32 * G::PS + 8 * g + 4 * hi) = u32x2{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
    }
    rs += __shfl_xor(rs, 32);
  }
  // ---- phi(q_j).z: lane (j = lane % 16, quarter = lane / 16) sums a quarter of the features --------
  float dq = 0.f;
  {
    const int quarter = lane >> 4;
    const uint16_t* qrow = sm.q + (lane & 15) * G::QS + quarter * (D / 4);
    const float* zrow = sm.z + quarter * (D / 4);
#pragma unroll
    for (int x = 0; x < D / 16; ++x) {
      const u32x2 pk = *reinterpret_cast<const u32x2*>(qrow + 4 * x);
      const f32x4 zv = *reinterpret_cast<const f32x4*>(zrow + 4 * x);
      dq = fmaf(bf16_lo_to_f32(pk[0]), zv[0], dq);
      dq = fmaf(bf16_hi_to_f32(pk[0]), zv[1], dq);
      dq = fmaf(bf16_lo_to_f32(pk[1]), zv[2], dq);
      dq = fmaf(bf16_hi_to_f32(pk[1]), zv[3], dq);
    }
    dq += __shfl_xor(dq, 16);
    dq += __shfl_xor(dq, 32);                // every lane now holds the value of draft lane % 16
  }

  // ---- operands that do not involve the state ----------------------------------------------------
  // vf: lanes <-> channels 32w + l32, registers <-> drafts 8hi + 0..7
  const bf16x8 vf = tr_operand(sm.v + HALO * G::VS, G::VS, 0, 32 * w, lane);
  const bf16x8 pB = lds_row8(sm.p[w] + jr * G::PS + 8 * hi);
  // register r of S holds feature 32ib + 8(r/4) + 4hi + r%4, so the phi(Q) operand takes features
  // {16h2 + 4hi + 0..3, 16h2 + 8 + 4hi + 0..3} of block ib for MFMA step h2
  const uint16_t* qb = sm.q + jr * G::QS + 4 * hi;
  // accepted drafts only: draft 8hi + e of the phi(K)^T operand is kept when it is below n
  u32x4 keep;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    keep[i] = (8 * hi + 2 * i < n ? 0x0000ffffu : 0u) | (8 * hi + 2 * i + 1 < n ? 0xffff0000u : 0u);

  // ---- read-out from the state as it was, then the state update, tile by tile --------------------
  // o[r] = O[draft l32][channel 32w + 8(r/4) + 4hi + r%4]
  f32x16 o;
#pragma unroll
  for (int r = 0; r < 16; ++r) o[r] = 0.f;
  o = mfma(vf, pB, o);
#pragma unroll
  for (int ib = 0; ib < G::IB; ++ib) {
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int x = 2 * ib + h2;
      o = mfma(pack8(Sacc[ib], 8 * h2), cat4(lds_row4(qb + 16 * x), lds_row4(qb + 16 * x + 8)), o);
    }
    if (n > 0) {   // uniform per workgroup; n == 0 leaves the state untouched
      const u32x4 kt = __builtin_bit_cast(u32x4, tr_operand(sm.k, G::KS, 0, 32 * ib, lane)) & keep;
      const u32x4 ktl = __builtin_bit_cast(u32x4, tr_operand(sm.klo, G::KS, 0, 32 * ib, lane)) & keep;
      Sacc[ib] = mfma(__builtin_bit_cast(bf16x8, ktl), vf, Sacc[ib]);
      Sacc[ib] = mfma(__builtin_bit_cast(bf16x8, kt), vf, Sacc[ib]);
#pragma unroll
      for (int r = 0; r < 16; ++r)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(Sacc[ib][r]), Srs, so,
                                              (32 * ib + 8 * (r >> 2) + (r & 3)) * row_bytes, 2);
    }
  }

  // ---- outputs: normalise, add the causal convolution over (history ++ drafts <= j) ---------------
  if (l32 < kk) {
    const float inv = __builtin_amdgcn_rcpf(a.eps + dq + rs);
    const uint16_t* vrow = sm.v + (HALO + l32) * G::VS + 32 * w + 4 * hi;
    const float* wrow = sm.w + 32 * w + 4 * hi;
    uint16_t* orow = static_cast<uint16_t*>(a.out) + vtok0 + (int64_t)l32 * DV + 32 * w + 4 * hi;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float u[4] = {0.f, 0.f, 0.f, 0.f};
      for (int t = 0; t < Kc; ++t) {
        const f32x4 wv4 = *reinterpret_cast<const f32x4*>(wrow + t * D + 8 * g);
        const u32x2 x = *reinterpret_cast<const u32x2*>(vrow - t * G::VS + 8 * g);
        u[0] = fmaf(wv4[0], bf16_lo_to_f32(x[0]), u[0]);
        u[1] = fmaf(wv4[1], bf16_hi_to_f32(x[0]), u[1]);
        u[2] = fmaf(wv4[2], bf16_lo_to_f32(x[1]), u[2]);
        u[3] = fmaf(wv4[3], bf16_hi_to_f32(x[1]), u[3]);
      }
      *reinterpret_cast<u32x2*>(orow + 8 * g) =
          u32x2{pack_bf16x2(fmaf(o[4 * g], inv, u[0]), fmaf(o[4 * g + 1], inv, u[1])),
                pack_bf16x2(fmaf(o[4 * g + 2], inv, u[2]), fmaf(o[4 * g + 3], inv, u[3]))};
    }
  }

  // ---- the rest of the state: normaliser and history ----------------------------------------------
  if (n == 0) return;   // uniform per workgroup: nothing accepted, state untouched
  if (tid < D) {
    if (nblk == 1) {                         // several blocks per head all read the old z: a launch of its own updates it
      float zs = zreg;
      for (int j = 0; j < n; ++j) zs += bf16_bits_to_f32(sm.k[j * G::KS + tid]) + bf16_bits_to_f32(sm.klo[j * G::KS + tid]);
      a.z[(size_t)bh * D + tid] = zs;
    }
    // the last Kc-1 rows of (history ++ accepted drafts); all of them are rows of the LDS copy
    for (int r = 0; r < Kc - 1; ++r)
      static_cast<uint16_t*>(a.hist)[hist0 + (int64_t)r * DV + tid] = sm.v[(HALO + n - (Kc - 1) + r) * G::VS + tid];
  }
}

bool verify_mfma_available(bool bf16, int d, int nsplit, int kk) {
  return bf16 && nsplit == 1 && kk <= VmCfg<128>::KT && (d == 128 || d == 64);
}

hipError_t launch_verify_mfma(const VerifyArgs& a, int d, hipStream_t st) {
  const dim3 grid((unsigned)(a.B * a.H * (a.dv / d)));
  if (d == 128) hipLaunchKernelGGL((verify_mfma_kernel<128>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((verify_mfma_kernel<64>), grid, dim3(128), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && a.dv != d) e = launch_verify_z(a, true, d, st);   // z of a head with several value blocks
  return e;
}

}  // namespace linattn
