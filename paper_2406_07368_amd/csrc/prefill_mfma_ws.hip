// Prefill on the matrix cores with specialised waves (Sec. 4.1), the kernel used
// whenever two copies of a group's rows fit in LDS.
//
// A workgroup walks one (b, h) -- or one segment of it -- in groups of C tokens and
// is split into two halves that run at the same time on every SIMD:
//
//   loader waves   bring the next group's Q, K, V rows from HBM (loads issued one whole
//                  group ahead), apply the feature map on the vector ALUs, and write
//                  phi(Q), phi(K), V as bf16 rows into the LDS buffer that is not in use;
//   compute waves  run the matrix-core work of the current group from the other buffer:
//                  the causal tiles of P^T = phi(K) phi(Q)^T (masked by select), then for
//                  their 32 value channels O^T = V^T P^T + S^T phi(Q)^T, the row
//                  normaliser, the causal convolution over V, the store, and finally
//                  S += phi(K)^T V.
//
// The state never leaves the compute waves' accumulator registers: wave w holds
// S[:, 32w:32w+32] and the 32 entries z[32w:32w+32] of the normaliser.  z is carried as
// the state column of a virtual value channel that is constantly one, so that both its
// update (phi(K)^T 1) and its read-out (phi(Q) z) are MFMAs as well; the read-out is split
// over the waves by feature block and summed through LDS.
//
// Two workgroup barriers per group keep the halves in step: B (scores and normaliser
// partials are in LDS) and C (the current buffer is free, the next one is full).
#include <type_traits>

#include "common.cuh"
#include "kernels.h"
#include "mfma_util.cuh"

namespace linattn {

namespace {

template <int D, int C>
struct WsCfg {
  static constexpr int NW = D / 32;          // compute waves (and as many loader waves)
  static constexpr int NT = 2 * NW * 64;
  static constexpr int NLT = NW * 64;        // loader threads
  static constexpr int TB = C / 32;
  static constexpr int IB = D / 32;
  static constexpr int KSD = D / 16;
  static constexpr int KSC = C / 16;
  static constexpr int NP = C / 16;          // loader passes: 16 tokens x all columns per pass
  static constexpr int QS = D + 4;           // phi(Q): 8-byte row reads, one row per lane
  static constexpr int KS = D + 16;          // phi(K): transpose reads and 16-byte row reads
  static constexpr int VS = D + 4;           // V: 8-byte row reads by the conv, some transpose reads
  static constexpr int PS = C + 8;           // P: 16-byte row reads
  static constexpr int NTILE = TB * (TB + 1) / 2;
  static constexpr int MAXT = (NTILE + NW - 1) / NW;
  static constexpr int KCMAX = 8;
  static constexpr int BQ = 0;
  static constexpr int BK = BQ + C * QS * 2;
  static constexpr int BV = BK + C * KS * 2;
  static constexpr int BUF = (BV + (HALO + C) * VS * 2 + 15) / 16 * 16;   // bytes of one row buffer
  static constexpr int OFF_PN = 2 * BUF;
  static constexpr int OFF_DENQ = OFF_PN + C * PS * 2;     // [NW][C] float
  static constexpr int OFF_DENP = OFF_DENQ + NW * C * 4;   // [TB][C] float
  static constexpr int OFF_WL = OFF_DENP + TB * C * 4;     // [KCMAX][D] float, tap-major
  static constexpr int TOTAL = OFF_WL + KCMAX * D * 4;
  static constexpr bool FITS = TOTAL <= 160 * 1024;
};

}  // namespace

template <int D, int C, int KCM>
__global__ __launch_bounds__(D * 4) void prefill_mfma_ws_kernel(PrefillArgs a) {
  using G = WsCfg<D, C>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Pn = reinterpret_cast<uint16_t*>(smem + G::OFF_PN);
  float* denq = reinterpret_cast<float*>(smem + G::OFF_DENQ);
  float* denp = reinterpret_cast<float*>(smem + G::OFF_DENP);
  float* wl = reinterpret_cast<float*>(smem + G::OFF_WL);
  auto bufQ = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + bi * G::BUF + G::BQ); };
  auto bufK = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + bi * G::BUF + G::BK); };
  auto bufV = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + bi * G::BUF + G::BV); };   // row r = token r - HALO

  const int tid = threadIdx.x;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;

  const int bh = blockIdx.x / a.nseg, seg = blockIdx.x % a.nseg;
  const int b = bh / a.H, h = bh % a.H;
  const int t_begin = seg * a.seg_len;
  const int t_end = (t_begin + a.seg_len) < a.L ? (t_begin + a.seg_len) : a.L;
  const int nchunks = (t_end - t_begin + C - 1) / C;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  uint16_t* gout = static_cast<uint16_t*>(a.out) + base;
  constexpr int SLOT = D * D + D;
  const float* ws_bh = a.ws + (size_t)bh * a.nseg * SLOT;
  const uint16_t* staged_hist =
      reinterpret_cast<const uint16_t*>(a.ws + (size_t)a.B * a.H * a.nseg * SLOT) + (size_t)bh * HALO * D;

  if (wv >= G::NW) {
    // =============================== loader waves ===============================================
    const int lt = tid - G::NLT;                       // 0 .. NLT-1
    const int lw = wv - G::NW;
    const int r16 = lane & 15;                         // token within a 16-token pass
    const int c0 = 8 * (4 * lw + (lane >> 4));         // first of the 8 columns this thread carries
    const int loff = r16 * (int)a.st + c0;             // this thread's offset inside a pass (elements)

    u32x4 rq[G::NP], rk[G::NP], rv[G::NP];
    auto load_pass = [&](int ci, int p) {              // rows past the end of the segment read as zero
      const int tok = t_begin + ci * C + 16 * p;       // uniform
      const bool ok = tok + r16 < t_end;
      const int64_t off = (int64_t)tok * a.st;         // uniform
      const u32x4 zero = {0, 0, 0, 0};
      rk[p] = ok ? *reinterpret_cast<const u32x4*>(gk + off + loff) : zero;
      rv[p] = ok ? *reinterpret_cast<const u32x4*>(gv + off + loff) : zero;
      rq[p] = ok ? *reinterpret_cast<const u32x4*>(gq + off + loff) : zero;
    };
    auto fill_pass = [&](int bi, int p, int nt, auto tail_tag) {
      constexpr bool TAIL = decltype(tail_tag)::value;
      const int t = 16 * p + r16;
      const bool ok = !TAIL || t < nt;
      u32x4 kp, qp;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float k0 = phi_elu1_max(bf16_lo_to_f32(rk[p][i])), k1 = phi_elu1_max(bf16_hi_to_f32(rk[p][i]));
        float q0 = phi_elu1_max(bf16_lo_to_f32(rq[p][i])), q1 = phi_elu1_max(bf16_hi_to_f32(rq[p][i]));
        kp[i] = pack_bf16x2(k0, k1);
        qp[i] = pack_bf16x2(q0, q1);
        if (TAIL) { kp[i] = ok ? kp[i] : 0u; qp[i] = ok ? qp[i] : 0u; }   // phi(0) = 1, so zero after the map
      }
      *reinterpret_cast<u32x4*>(bufK(bi) + t * G::KS + c0) = kp;
      u32x2* vrow = reinterpret_cast<u32x2*>(bufV(bi) + (HALO + t) * G::VS + c0);
      vrow[0] = u32x2{rv[p][0], rv[p][1]};
      vrow[1] = u32x2{rv[p][2], rv[p][3]};
      u32x2* qrow = reinterpret_cast<u32x2*>(bufQ(bi) + t * G::QS + c0);
      qrow[0] = u32x2{qp[0], qp[1]};
      qrow[1] = u32x2{qp[2], qp[3]};
    };
    // group ci -> buffer ci & 1; afterwards the registers hold group ci + 1.  `split` passes are
    // done before barrier B, the rest after it.
    auto fill_group = [&](int ci, bool with_barrier) {
      const int bi = ci & 1;
      const int nt = (t_end - (t_begin + ci * C)) < C ? (t_end - (t_begin + ci * C)) : C;
      const bool more = ci + 1 < nchunks;
      constexpr int SPLIT = G::NP / 4 > 0 ? G::NP / 4 : 1;
#pragma unroll
      for (int p = 0; p < G::NP; ++p) {
        if (p == SPLIT && with_barrier) __syncthreads();            // barrier B
        if (nt == C) fill_pass(bi, p, nt, std::false_type{});
        else fill_pass(bi, p, nt, std::true_type{});
        if (more) load_pass(ci + 1, p);
      }
    };

    for (int e = lt; e < KCM * D; e += G::NLT) {
      const int j = e / D, cc = e % D;
      wl[e] = j < a.Kc ? a.conv_w[((size_t)h * D + cc) * a.Kc + j] : 0.f;
    }
    // value rows just before this segment: earlier tokens, else the incoming history, else zeros
    for (int e = lt; e < HALO * D; e += G::NLT) {
      const int r = e / D, cc = e % D;
      const int tok = t_begin - HALO + r;
      uint16_t x = 0;
      if (tok >= 0) x = gv[(int64_t)tok * a.st + cc];
      else if (a.hist_in) {
        if (a.nseg > 1) x = staged_hist[(size_t)(HALO + tok) * D + cc];
        else if (a.Kc - 1 + tok >= 0)
          x = static_cast<const uint16_t*>(a.hist_in)[((size_t)bh * (a.Kc - 1) + (a.Kc - 1 + tok)) * D + cc];
      }
      bufV(0)[r * G::VS + cc] = x;
    }
    if (nchunks > 0) {
#pragma unroll
      for (int p = 0; p < G::NP; ++p) load_pass(0, p);
      fill_group(0, false);
    }
    __syncthreads();                                   // buffer 0 is full
    for (int ci = 0; ci < nchunks; ++ci) {
      if (ci + 1 < nchunks) {
        // the last HALO value rows of group ci become the rows before group ci + 1
        if (lt < HALO * D / 8) {
          const int r = lt / (D / 8), piece = 8 * (lt % (D / 8));
          const u32x2* src = reinterpret_cast<const u32x2*>(bufV(ci & 1) + (C + r) * G::VS + piece);
          u32x2* dst = reinterpret_cast<u32x2*>(bufV((ci + 1) & 1) + r * G::VS + piece);
          const u32x2 t0 = src[0], t1 = src[1];
          dst[0] = t0; dst[1] = t1;
        }
        fill_group(ci + 1, true);                      // contains barrier B
      } else {
        __syncthreads();                               // barrier B
      }
      __syncthreads();                                 // barrier C
    }
    return;
  }

  // ================================= compute waves =================================================
  const int w = wv;
  const int cw = 32 * w + l32;             // the channel this lane owns in the state accumulators

  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw];  Zacc[r] = z[32w + 8(r/4) + 4hi + r%4] (every lane)
  f32x16 Sacc[G::IB], Zacc;
  {
    const float* Ssrc = nullptr;
    const float* zsrc = nullptr;
    if (a.nseg > 1) { Ssrc = ws_bh + (size_t)seg * SLOT; zsrc = Ssrc + D * D; }
    else if (a.S_in) { Ssrc = a.S_in + (size_t)bh * D * D; zsrc = a.z_in + (size_t)bh * D; }
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
        Sacc[ib][r] = Ssrc ? Ssrc[(size_t)i * D + cw] : 0.f;
      }
#pragma unroll
    for (int r = 0; r < 16; ++r) Zacc[r] = zsrc ? zsrc[32 * w + 8 * (r >> 2) + 4 * hi + (r & 3)] : 0.f;
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  __syncthreads();                                     // buffer 0 is full, conv taps are in LDS

  // conv taps of this lane's 16 output channels (32w + 8g + 4hi + e), kept in registers when few
  constexpr bool W_REGS = KCM <= 3;
  f32x4 wreg[W_REGS ? KCM : 1][4];
  if (W_REGS) {
#pragma unroll
    for (int j = 0; j < (W_REGS ? KCM : 1); ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) wreg[j][g] = *reinterpret_cast<const f32x4*>(wl + j * D + 32 * w + 8 * g + 4 * hi);
  }

  auto group = [&](int ci, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int tok0 = t_begin + ci * C;
    const int nt = TAIL ? (t_end - tok0) : C;
    const uint16_t* Qn = bufQ(ci & 1);
    const uint16_t* Kn = bufK(ci & 1);
    const uint16_t* Vn = bufV(ci & 1);

    // ---- scores: causal tiles of P^T = phi(K) phi(Q)^T, masked, to LDS as P[t][s] ---------------------
#pragma unroll
    for (int s = 0; s < G::MAXT; ++s) {
      const int idx = w + s * G::NW;
      if (idx < G::NTILE) {
        int tb = 0;
        while ((tb + 1) * (tb + 2) / 2 <= idx) ++tb;
        const int sb = idx - tb * (tb + 1) / 2;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const uint16_t* ka = Kn + (32 * sb + l32) * G::KS + 8 * hi;
        const uint16_t* qb = Qn + (32 * tb + l32) * G::QS + 8 * hi;
#pragma unroll
        for (int ks = 0; ks < G::KSD; ++ks)
          acc = mfma(lds_row8(ka + 16 * ks), cat4(lds_row4(qb + 16 * ks), lds_row4(qb + 16 * ks + 4)), acc);
        // acc[r]: source token s = 32sb + 8(r/4) + 4hi + r%4, query token t = 32tb + l32
        float rs = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int sl = 8 * g + 4 * hi + e;
            const float v0 = acc[4 * g + e];
            x[e] = (sb < tb || sl <= l32) ? v0 : 0.f;   // select, never multiply: later tokens cannot leak
            rs += x[e];
          }
          u32x2 pk = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
          *reinterpret_cast<u32x2*>(Pn + (32 * tb + l32) * G::PS + 32 * sb + 8 * g + 4 * hi) = pk;
        }
        rs += __shfl_xor(rs, 32);
        if (lane < 32) denp[sb * C + 32 * tb + l32] = rs;
      }
    }
    // ---- phi(q_t).z over this wave's 32 features, for every token of the group -------------------------
    {
      const bf16x8 zb0 = pack8(Zacc, 0), zb1 = pack8(Zacc, 8);
#pragma unroll
      for (int tb = 0; tb < G::TB; ++tb) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const uint16_t* p = Qn + (32 * tb + l32) * G::QS + 32 * w + 4 * hi;
        acc = mfma(zb0, cat4(lds_row4(p), lds_row4(p + 8)), acc);
        acc = mfma(zb1, cat4(lds_row4(p + 16), lds_row4(p + 24)), acc);
        if (lane < 32) denq[w * C + 32 * tb + l32] = acc[0];   // every row of the product is the same
      }
    }
    __syncthreads();   // B: P and the normaliser partials are in LDS

    // ---- this wave's channels ------------------------------------------------------------------------
    // vf[ks]: lanes <-> channels 32w + l32, registers <-> tokens 16ks + 8hi + 0..7
    bf16x8 vf[G::KSC];
#pragma unroll
    for (int ks = 0; ks < G::KSC; ++ks) vf[ks] = tr_operand(Vn + HALO * G::VS, G::VS, 16 * ks, 32 * w, lane);
    bf16x8 sbf[G::IB][2];
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib) { sbf[ib][0] = pack8(Sacc[ib], 0); sbf[ib][1] = pack8(Sacc[ib], 8); }
#pragma unroll
    for (int tb = 0; tb < G::TB; ++tb) {
      // o[r] = O[token 32tb + l32][channel 32w + 8(r/4) + 4hi + r%4]
      f32x16 o;
#pragma unroll
      for (int r = 0; r < 16; ++r) o[r] = 0.f;
      const uint16_t* pb = Pn + (32 * tb + l32) * G::PS + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < 2 * (tb + 1); ++ks) o = mfma(vf[ks], lds_row8(pb + 16 * ks), o);
      // S^T phi(Q)^T: register r of S holds feature 32ib + 8(r/4) + 4hi + r%4, so the phi(Q) operand
      // takes features {16h2 + 4hi + 0..3, 16h2 + 8 + 4hi + 0..3} of block ib for MFMA step h2
      const uint16_t* qb = Qn + (32 * tb + l32) * G::QS + 4 * hi;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const uint16_t* p = qb + 32 * ib + 16 * h2;
          o = mfma(sbf[ib][h2], cat4(lds_row4(p), lds_row4(p + 8)), o);
        }
      // normalise, add the causal conv, store
      const int t = 32 * tb + l32;
      float den = a.eps;
#pragma unroll
      for (int ww = 0; ww < G::NW; ++ww) den += denq[ww * C + t];
#pragma unroll
      for (int sb = 0; sb <= tb; ++sb) den += denp[sb * C + t];
      const float inv = __builtin_amdgcn_rcpf(den);
      const uint16_t* vrow = Vn + (HALO + t) * G::VS + 32 * w + 4 * hi;
      uint16_t* orow = gout + (int64_t)(tok0 + t) * a.st + 32 * w + 4 * hi;
      const float* wrow = wl + 32 * w + 4 * hi;
      const bool live = !TAIL || t < nt;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KCM; ++j) {
          const u32x2 xv = *reinterpret_cast<const u32x2*>(vrow - j * G::VS + 8 * g);
          const f32x4 wv4 = W_REGS ? wreg[W_REGS ? j : 0][g] : *reinterpret_cast<const f32x4*>(wrow + j * D + 8 * g);
          u[0] = fmaf(wv4[0], bf16_lo_to_f32(xv[0]), u[0]);
          u[1] = fmaf(wv4[1], bf16_hi_to_f32(xv[0]), u[1]);
          u[2] = fmaf(wv4[2], bf16_lo_to_f32(xv[1]), u[2]);
          u[3] = fmaf(wv4[3], bf16_hi_to_f32(xv[1]), u[3]);
        }
        const u32x2 y = {pack_bf16x2(fmaf(o[4 * g], inv, u[0]), fmaf(o[4 * g + 1], inv, u[1])),
                         pack_bf16x2(fmaf(o[4 * g + 2], inv, u[2]), fmaf(o[4 * g + 3], inv, u[3]))};
        if (live) *reinterpret_cast<u32x2*>(orow + 8 * g) = y;
      }
    }
    // S += phi(K)^T V for this wave's channels, z += phi(K)^T 1 for this wave's features
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int ks = 0; ks < G::KSC; ++ks) {
        const bf16x8 kt = tr_operand(Kn, G::KS, 16 * ks, 32 * ib, lane);
        Sacc[ib] = mfma(kt, vf[ks], Sacc[ib]);
        if (ib == w) Zacc = mfma(kt, ones, Zacc);
      }
    __syncthreads();   // C: this buffer may be refilled, the other one is complete
  };

  for (int ci = 0; ci < nchunks; ++ci) {
    if (t_begin + (ci + 1) * C <= t_end) group(ci, std::false_type{});
    else group(ci, std::true_type{});
  }

  // ---- hand the state over ---------------------------------------------------------------------------
  if (seg == a.nseg - 1) {
    if (a.S_out) {
      float* Sdst = a.S_out + (size_t)bh * D * D;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
          Sdst[(size_t)i * D + cw] = Sacc[ib][r];
        }
    }
    if (a.z_out && l32 == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) a.z_out[(size_t)bh * D + 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3)] = Zacc[r];
    }
    if (a.hist_out && tid < D) {
      // last Kc-1 value rows of (history ++ sequence); one thread per channel, rows in ascending order,
      // so an aliased hist_in is read before it is overwritten (with segments the staged copy is read)
      const uint16_t* hin = static_cast<const uint16_t*>(a.hist_in);
      uint16_t* hout = static_cast<uint16_t*>(a.hist_out) + (size_t)bh * (a.Kc - 1) * D;
      for (int r = 0; r < a.Kc - 1; ++r) {
        const int tok = a.L - (a.Kc - 1) + r;
        uint16_t x = 0;
        if (tok >= 0) x = gv[(int64_t)tok * a.st + tid];
        else if (hin) x = a.nseg > 1 ? staged_hist[(size_t)(HALO + tok) * D + tid]
                                     : hin[((size_t)bh * (a.Kc - 1) + (a.Kc - 1 + tok)) * D + tid];
        hout[(size_t)r * D + tid] = x;
      }
    }
  }
}

template <int D, int C>
bool ws_fits() { return WsCfg<D, C>::FITS; }

template <int D, int C, int KCM>
static hipError_t launch_ws(const PrefillArgs& a, hipStream_t st) {
  using G = WsCfg<D, C>;
  if constexpr (!G::FITS) {
    return hipErrorInvalidConfiguration;
  } else {
    auto kern = prefill_mfma_ws_kernel<D, C, KCM>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, G::TOTAL);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H * a.nseg)), dim3(G::NT), G::TOTAL, st, a);
    return hipGetLastError();
  }
}

template <int D, int C>
static hipError_t launch_ws_k(const PrefillArgs& a, hipStream_t st) {
  if (a.Kc <= 3) return launch_ws<D, C, 3>(a, st);
  if (a.Kc <= 5) return launch_ws<D, C, 5>(a, st);
  return launch_ws<D, C, 8>(a, st);
}

// True when the specialised kernel exists for this shape (two row buffers fit in 160 KB of LDS).
bool prefill_mfma_ws_available(int d, int chunk) {
  if (d == 128) return chunk == 64 ? ws_fits<128, 64>() : ws_fits<128, 128>();
  return chunk == 64 ? ws_fits<64, 64>() : ws_fits<64, 128>();
}

// The full pass of one prefill call (all segments); segment start states must already be in a.ws.
hipError_t launch_prefill_mfma_ws(const PrefillArgs& a, int d, int chunk, hipStream_t st) {
  if (d == 128) return chunk == 64 ? launch_ws_k<128, 64>(a, st) : launch_ws_k<128, 128>(a, st);
  return chunk == 64 ? launch_ws_k<64, 64>(a, st) : launch_ws_k<64, 128>(a, st);
}

}  // namespace linattn
