// Prefill on the matrix cores (Sec. 4.1): bf16 operands, fp32 accumulation.
//
// One workgroup walks one (b, h) -- or one segment of its sequence -- group by
// group (C tokens).  Wave w owns value channels [32w, 32w+32): its slice of the
// running state S[:, 32w:32w+32] lives in MFMA accumulator registers for the whole
// walk and never goes to LDS or HBM in between.  Per group:
//   1. the prefetched Q, K, V rows get the feature map and go to LDS in their
//      natural [token][feature] layout (bf16);
//   2. the causal tiles of P^T = phi(K) phi(Q)^T are computed (32x32x16 MFMA),
//      masked by select, rounded to bf16 and written to LDS as P[t][s];
//   3. each wave forms O^T[its channels, :] = V^T P^T + S^T phi(Q)^T, where S^T is fed
//      to the MFMA straight from the accumulator registers (the accumulator layout
//      of S[i][c] is, up to a fixed permutation of i that is also applied to the
//      phi(Q) operand, the A-operand layout), then S += phi(K)^T V; operands that
//      need the token axis in registers (V, phi(K)^T) are fetched from the natural
//      layout with the LDS transpose loads of gfx950;
//   4. in the O^T accumulator a lane holds one token and 16 of the wave's channels,
//      so the row normaliser is one reciprocal per lane; the causal convolution
//      over V is added from LDS rows and the result is stored 8 bytes at a time.
// The state is carried from group to group in registers; between segments of one
// sequence (used when B*H alone cannot fill the chip) it is carried by a first pass
// that reduces each segment's K, V to its state increment, a prefix sum over the
// segments, and a second pass that starts every segment from its prefix.
#include <type_traits>

#include "common.cuh"
#include "kernels.h"
#include "mfma_util.cuh"

namespace linattn {

namespace {

template <int D, int C>
struct Cfg {
  static constexpr int NW = D / 32;          // waves; wave w owns channels 32w..32w+31
  static constexpr int NT = NW * 64;
  static constexpr int TB = C / 32;          // 32-token blocks per group
  static constexpr int IB = D / 32;          // 32-feature blocks
  static constexpr int KSD = D / 16;         // MFMA K steps over the feature axis
  static constexpr int KSC = C / 16;         // MFMA K steps over the token axis
  static constexpr int NP = C / 16;          // load passes: 16 tokens x (NW*4) column groups per pass
  // LDS row strides in bf16 elements, chosen per array for the way it is read most:
  static constexpr int QS = D + 4;           // phi(Q): 8-byte row reads, one row per lane
  static constexpr int KS = D + 16;          // phi(K): transpose reads (4 rows x 32 B per 16 lanes)
  static constexpr int VS = D + 4;           // V: 8-byte row reads by the conv, some transpose reads
  static constexpr int PS = C + 8;           // P: 16-byte row reads
  static constexpr int KCMAX = 8;            // conv weight rows kept in LDS
  static constexpr int NTILE = TB * (TB + 1) / 2;
  static constexpr int MAXT = (NTILE + NW - 1) / NW;
  // byte offsets into dynamic LDS
  static constexpr int OFF_QN = 0;
  static constexpr int OFF_KN = OFF_QN + C * QS * 2;
  static constexpr int OFF_VN = OFF_KN + C * KS * 2;
  static constexpr int OFF_PN = (OFF_VN + (HALO + C) * VS * 2 + 15) / 16 * 16;
  static constexpr int OFF_DENQ = OFF_PN + C * PS * 2;       // [NW][C] float: phi(q_t).z over each wave's features
  static constexpr int OFF_DENP = OFF_DENQ + NW * C * 4;     // [TB][C] float: row sums of P per source block
  static constexpr int OFF_ZZ = OFF_DENP + TB * C * 4;       // [2][D] float: normaliser, double-buffered
  static constexpr int OFF_WL = OFF_ZZ + 2 * D * 4;          // [KCMAX][D] float: conv taps, tap-major
  static constexpr int TOTAL = OFF_WL + KCMAX * D * 4;
  static_assert(TOTAL <= 160 * 1024, "LDS budget");
};

}  // namespace

// STATE_ONLY: reduce a segment's K, V to its state increment (first pass of the
// segmented form); otherwise the full path.  KCM: number of conv taps evaluated
// (taps >= Kc have zero weight).
template <int D, int C, int KCM, bool STATE_ONLY>
__global__ __launch_bounds__(D * 2) void prefill_mfma_kernel(PrefillArgs a) {
  using G = Cfg<D, C>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Qn = reinterpret_cast<uint16_t*>(smem + G::OFF_QN);
  uint16_t* Kn = reinterpret_cast<uint16_t*>(smem + G::OFF_KN);
  uint16_t* Vn = reinterpret_cast<uint16_t*>(smem + G::OFF_VN);   // row r holds token r - HALO of the group
  uint16_t* Pn = reinterpret_cast<uint16_t*>(smem + G::OFF_PN);
  float* denq = reinterpret_cast<float*>(smem + G::OFF_DENQ);
  float* denp = reinterpret_cast<float*>(smem + G::OFF_DENP);
  float* zz = reinterpret_cast<float*>(smem + G::OFF_ZZ);
  float* wl = reinterpret_cast<float*>(smem + G::OFF_WL);

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  const int r16 = lane & 15;               // token within a 16-token load pass
  const int c0 = 8 * (4 * w + (lane >> 4));  // first of the 8 features/channels this thread loads
  const int cw = 32 * w + l32;             // the channel this lane owns in the state accumulators

  const int nseg_grid = STATE_ONLY ? a.nseg - 1 : a.nseg;
  const int bh = blockIdx.x / nseg_grid, seg = blockIdx.x % nseg_grid;
  const int b = bh / a.H, h = bh % a.H;
  const int t_begin = seg * a.seg_len;
  const int t_end = (t_begin + a.seg_len) < a.L ? (t_begin + a.seg_len) : a.L;
  const int nchunks = (t_end - t_begin + C - 1) / C;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  uint16_t* gout = static_cast<uint16_t*>(a.out) + base;
  constexpr int SLOT = D * D + D;          // floats per stored state (S then z)
  float* ws_bh = a.ws + (size_t)bh * a.nseg * SLOT;
  const uint16_t* staged_hist =
      reinterpret_cast<const uint16_t*>(a.ws + (size_t)a.B * a.H * a.nseg * SLOT) + (size_t)bh * HALO * D;

  // ---- start state -------------------------------------------------------------------------
  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw]
  f32x16 Sacc[G::IB];
  {
    const float* Ssrc = nullptr;
    const float* zsrc = nullptr;
    if (!STATE_ONLY) {
      if (a.nseg > 1) { Ssrc = ws_bh + (size_t)seg * SLOT; zsrc = Ssrc + D * D; }
      else if (a.S_in) { Ssrc = a.S_in + (size_t)bh * D * D; zsrc = a.z_in + (size_t)bh * D; }
    }
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
        Sacc[ib][r] = Ssrc ? Ssrc[(size_t)i * D + cw] : 0.f;
      }
    if (tid < D) zz[tid] = zsrc ? zsrc[tid] : 0.f;
  }

  if (!STATE_ONLY) {
    for (int e = tid; e < KCM * D; e += G::NT) {
      const int j = e / D, cc = e % D;
      wl[e] = j < a.Kc ? a.conv_w[((size_t)h * D + cc) * a.Kc + j] : 0.f;
    }
    // value rows just before this segment: earlier tokens, else the incoming history, else zeros
    for (int e = tid; e < HALO * D; e += G::NT) {
      const int r = e / D, cc = e % D;
      const int tok = t_begin - HALO + r;
      uint16_t x = 0;
      if (tok >= 0) x = gv[(int64_t)tok * a.st + cc];
      else if (a.hist_in) {
        // history rows are oldest first and end right before token 0
        if (a.nseg > 1) x = staged_hist[(size_t)(HALO + tok) * D + cc];     // staged copy: always HALO rows
        else if (a.Kc - 1 + tok >= 0)
          x = static_cast<const uint16_t*>(a.hist_in)[((size_t)bh * (a.Kc - 1) + (a.Kc - 1 + tok)) * D + cc];
      }
      Vn[r * G::VS + cc] = x;
    }
  }

  // ---- prefetch registers ---------------------------------------------------------------------
  u32x4 rq[G::NP], rk[G::NP], rv[G::NP];
  auto prefetch = [&](int ci) {
    const int tok0 = t_begin + ci * C;
#pragma unroll
    for (int p = 0; p < G::NP; ++p) {
      const int tok = tok0 + 16 * p + r16;
      const bool ok = tok < t_end;
      const int64_t off = (int64_t)tok * a.st + c0;
      const u32x4 zero = {0, 0, 0, 0};
      rk[p] = ok ? *reinterpret_cast<const u32x4*>(gk + off) : zero;
      rv[p] = ok ? *reinterpret_cast<const u32x4*>(gv + off) : zero;
      if (!STATE_ONLY) rq[p] = ok ? *reinterpret_cast<const u32x4*>(gq + off) : zero;
    }
  };
  if (nchunks > 0) prefetch(0);
  __syncthreads();

  // One group of C tokens.  TAIL: the group may be short (rows past the end are zero-filled and
  // their outputs are not stored); full groups skip those checks.
  auto group = [&](int ci, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int tok0 = t_begin + ci * C;
    const int nt = TAIL ? (t_end - tok0) : C;
    float* zc = zz + (ci & 1) * D;
    float* zn = zz + ((ci + 1) & 1) * D;

    // ---- 1. feature map, rows to LDS ---------------------------------------------------------------
    {
      float zsum[8], zcur[8], dq[G::NP];
#pragma unroll
      for (int e = 0; e < 8; ++e) { zsum[e] = 0.f; zcur[e] = zc[c0 + e]; }
#pragma unroll
      for (int p = 0; p < G::NP; ++p) {
        const int t = 16 * p + r16;
        const bool ok = !TAIL || t < nt;
        u32x4 kp, qp;
        float dsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float k0 = phi_elu1_fast(bf16_lo_to_f32(rk[p][i])), k1 = phi_elu1_fast(bf16_hi_to_f32(rk[p][i]));
          if (TAIL) { k0 = ok ? k0 : 0.f; k1 = ok ? k1 : 0.f; }
          kp[i] = pack_bf16x2(k0, k1);
          zsum[2 * i] += k0; zsum[2 * i + 1] += k1;
          if (!STATE_ONLY) {
            float q0 = phi_elu1_fast(bf16_lo_to_f32(rq[p][i])), q1 = phi_elu1_fast(bf16_hi_to_f32(rq[p][i]));
            if (TAIL) { q0 = ok ? q0 : 0.f; q1 = ok ? q1 : 0.f; }
            qp[i] = pack_bf16x2(q0, q1);
            dsum = fmaf(q0, zcur[2 * i], dsum);
            dsum = fmaf(q1, zcur[2 * i + 1], dsum);
          }
        }
        *reinterpret_cast<u32x4*>(Kn + t * G::KS + c0) = kp;
        u32x2* vrow = reinterpret_cast<u32x2*>(Vn + (HALO + t) * G::VS + c0);
        vrow[0] = u32x2{rv[p][0], rv[p][1]};
        vrow[1] = u32x2{rv[p][2], rv[p][3]};
        if (!STATE_ONLY) {
          u32x2* qrow = reinterpret_cast<u32x2*>(Qn + t * G::QS + c0);
          qrow[0] = u32x2{qp[0], qp[1]};
          qrow[1] = u32x2{qp[2], qp[3]};
          dq[p] = dsum;
        }
      }
      if (!STATE_ONLY) {
        // phi(q_t).z over this wave's 32 features: the 4 column groups of a token sit 16 lanes apart
#pragma unroll
        for (int p = 0; p < G::NP; ++p) {
          float x = dq[p];
          x += __shfl_xor(x, 16);
          x += __shfl_xor(x, 32);
          if (lane < 16) denq[w * C + 16 * p + r16] = x;
        }
      }
      // z += column sums of phi(K): the 16 tokens of a pass sit in the low 4 lane bits
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = zsum[e];
        x += __shfl_xor(x, 1); x += __shfl_xor(x, 2); x += __shfl_xor(x, 4); x += __shfl_xor(x, 8);
        zsum[e] = x;
      }
      if (r16 == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) zn[c0 + e] = zcur[e] + zsum[e];
      }
    }
    if (ci + 1 < nchunks) prefetch(ci + 1);
    __syncthreads();   // A: rows of this group are in LDS

    if (!STATE_ONLY) {
      // ---- 2. causal tiles of P^T = phi(K) phi(Q)^T, masked, to LDS as P[t][s] -------------------------
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
      __syncthreads();   // B: P and the row sums are in LDS
    }

    // ---- 3. this wave's channels ---------------------------------------------------------------------
    // vf[ks]: lanes <-> channels 32w + l32, registers <-> tokens 16ks + 8hi + 0..7
    bf16x8 vf[G::KSC];
#pragma unroll
    for (int ks = 0; ks < G::KSC; ++ks) vf[ks] = tr_operand(Vn + HALO * G::VS, G::VS, 16 * ks, 32 * w, lane);

    if (!STATE_ONLY) {
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
        // ---- 4. normalise, add the causal conv, store ---------------------------------------------------
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
            const f32x4 wv = *reinterpret_cast<const f32x4*>(wrow + j * D + 8 * g);
            u[0] = fmaf(wv[0], bf16_lo_to_f32(xv[0]), u[0]);
            u[1] = fmaf(wv[1], bf16_hi_to_f32(xv[0]), u[1]);
            u[2] = fmaf(wv[2], bf16_lo_to_f32(xv[1]), u[2]);
            u[3] = fmaf(wv[3], bf16_hi_to_f32(xv[1]), u[3]);
          }
          const u32x2 y = {pack_bf16x2(fmaf(o[4 * g], inv, u[0]), fmaf(o[4 * g + 1], inv, u[1])),
                           pack_bf16x2(fmaf(o[4 * g + 2], inv, u[2]), fmaf(o[4 * g + 3], inv, u[3]))};
          if (live) *reinterpret_cast<u32x2*>(orow + 8 * g) = y;
        }
      }
    }

    // S += phi(K)^T V for this wave's channels; both operands come through transpose loads
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int ks = 0; ks < G::KSC; ++ks)
        Sacc[ib] = mfma(tr_operand(Kn, G::KS, 16 * ks, 32 * ib, lane), vf[ks], Sacc[ib]);

    __syncthreads();   // C: every read of this group's rows is done
    if (!STATE_ONLY && tid < HALO * D / 8) {
      // keep the last HALO value rows for the next group's conv taps
      const int r = tid / (D / 8), piece = 8 * (tid % (D / 8));
      const u32x2* src = reinterpret_cast<const u32x2*>(Vn + (C + r) * G::VS + piece);
      u32x2* dst = reinterpret_cast<u32x2*>(Vn + r * G::VS + piece);
      const u32x2 t0 = src[0], t1 = src[1];
      dst[0] = t0; dst[1] = t1;
    }
  };

  for (int ci = 0; ci < nchunks; ++ci) {
    if (t_begin + (ci + 1) * C <= t_end) group(ci, std::false_type{});
    else group(ci, std::true_type{});
  }

  // ---- hand the state over -------------------------------------------------------------------------------
  const float* zfin = zz + (nchunks & 1) * D;
  float* Sdst = nullptr;
  float* zdst = nullptr;
  if (STATE_ONLY) { Sdst = ws_bh + (size_t)(seg + 1) * SLOT; zdst = Sdst + D * D; }
  else if (seg == a.nseg - 1 && a.S_out) { Sdst = a.S_out + (size_t)bh * D * D; }
  if (!STATE_ONLY && seg == a.nseg - 1 && a.z_out) zdst = a.z_out + (size_t)bh * D;
  if (Sdst) {
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
        Sdst[(size_t)i * D + cw] = Sacc[ib][r];
      }
  }
  if (zdst && tid < D) zdst[tid] = zfin[tid];
  if (!STATE_ONLY && seg == a.nseg - 1 && a.hist_out && tid < D) {
    // last Kc-1 value rows of (history ++ sequence); one thread per channel, rows in ascending
    // order, so an aliased hist_in is read before it is overwritten (with segments the copy
    // staged by the scan kernel is read instead of hist_in)
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

// Prefix sum over the segments of one (b, h): slot 0 <- incoming state, slot g <- slot g-1 +
// increment of segment g-1.  Also stages the incoming history so that the second pass never
// reads hist_in (which hist_out may alias).  One thread per state element walks the segments.
template <int D>
__global__ __launch_bounds__(256) void segment_scan_kernel(PrefillArgs a) {
  constexpr int SLOT = D * D + D;
  const int bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  float* ws_bh = a.ws + (size_t)bh * a.nseg * SLOT;
  if (e < SLOT) {
    float run = 0.f;
    if (a.S_in) run = e < D * D ? a.S_in[(size_t)bh * D * D + e] : a.z_in[(size_t)bh * D + (e - D * D)];
    ws_bh[e] = run;
    for (int g = 1; g < a.nseg; ++g) {
      run += ws_bh[(size_t)g * SLOT + e];
      ws_bh[(size_t)g * SLOT + e] = run;
    }
  }
  if (a.hist_in && e < HALO * D) {
    uint16_t* staged = reinterpret_cast<uint16_t*>(a.ws + (size_t)a.B * a.H * a.nseg * SLOT) + (size_t)bh * HALO * D;
    const int r = e / D, cc = e % D;           // staged row r holds token r - HALO
    const int hr = (a.Kc - 1) - HALO + r;      // row of the incoming history
    staged[e] = hr >= 0 ? static_cast<const uint16_t*>(a.hist_in)[((size_t)bh * (a.Kc - 1) + hr) * D + cc] : (uint16_t)0;
  }
}

// Segments per (b, h): enough workgroups to cover the 256 compute units about once,
// but at least 4 groups per segment so the first pass stays a small fraction.
int prefill_mfma_pick_segments(int BH, int L, int chunk) {
  const int chunks = (L + chunk - 1) / chunk;
  int want = (256 + BH - 1) / BH;
  int most = chunks / 4;
  if (most < 1) most = 1;
  if (want > most) want = most;
  if (want > 64) want = 64;
  return want < 1 ? 1 : want;
}

size_t prefill_mfma_workspace_bytes(int BH, int d, int nseg) {
  if (nseg <= 1) return 0;
  return (size_t)BH * nseg * ((size_t)d * d + d) * sizeof(float) + (size_t)BH * HALO * d * sizeof(uint16_t);
}

template <int D, int C, int KCM>
static hipError_t launch_dc(const PrefillArgs& a, hipStream_t st) {
  using G = Cfg<D, C>;
  const int BH = a.B * a.H;
  const bool ws = prefill_mfma_ws_available(D, C);   // specialised front-end/state waves: two row buffers fit in LDS
  hipError_t e;
  if (a.nseg > 1) {
    if (ws) {
      if ((e = launch_prefill_mfma_ws(a, D, C, true, st)) != hipSuccess) return e;
    } else {
      auto first = prefill_mfma_kernel<D, C, KCM, true>;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(first), hipFuncAttributeMaxDynamicSharedMemorySize, G::TOTAL);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(first, dim3((unsigned)(BH * (a.nseg - 1))), dim3(G::NT), G::TOTAL, st, a);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    constexpr int SLOT = D * D + D;
    hipLaunchKernelGGL((segment_scan_kernel<D>), dim3((SLOT + 255) / 256, (unsigned)BH), dim3(256), 0, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (ws) return launch_prefill_mfma_ws(a, D, C, false, st);
  auto full = prefill_mfma_kernel<D, C, KCM, false>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(full), hipFuncAttributeMaxDynamicSharedMemorySize, G::TOTAL);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(full, dim3((unsigned)(BH * a.nseg)), dim3(G::NT), G::TOTAL, st, a);
  return hipGetLastError();
}

template <int D, int C>
static hipError_t launch_k(const PrefillArgs& a, hipStream_t st) {
  if (a.Kc <= 3) return launch_dc<D, C, 3>(a, st);
  if (a.Kc <= 5) return launch_dc<D, C, 5>(a, st);
  return launch_dc<D, C, 8>(a, st);
}

// The group size only blocks the computation; the result does not depend on it (the in-group
// part is the exact masked product).  At d = 128 a requested group of 128 tokens is walked as two
// steps of 64: two 128-token row buffers do not fit in LDS, and larger groups only add in-group
// MFMA work per token on this design.  Segment boundaries stay multiples of the requested size.
hipError_t launch_prefill_mfma(const PrefillArgs& a, int d, int chunk, hipStream_t st) {
  if (d == 128) return launch_k<128, 64>(a, st);
  return chunk == 64 ? launch_k<64, 64>(a, st) : launch_k<64, 128>(a, st);
}

}  // namespace linattn
