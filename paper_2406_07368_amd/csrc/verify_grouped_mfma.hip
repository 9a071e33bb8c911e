// Generation with the three-branch form on the matrix cores: k >= 4 bf16 drafts per head (Sec. 4.1 block,
// Sec. 4.2 verification).  Same function as verify_grouped.hip, whose vector-ALU arithmetic is the bound
// from a few drafts on; here the three contractions are MFMAs:
//
//   logits      P^T tiles = K Q^T over the rows of (open group ++ drafts), raw rows   (32 keys x drafts)
//   read-out    O^T  = S^T phi(Q)^T, the state tiles fed from accumulator registers
//   values      O^T += V^T W^T, W the softmax weights (and, for a draft beyond the end of the group,
//               the linear weights f_j phi(q_j).phi(k_r) of the group that has just been completed)
//
// One workgroup per (b, h), D/32 waves; wave w owns value channels 32w..32w+31, i.e. the column block
// S[:, 32w:32w+32] as D/32 accumulator tiles, requested first thing (nontemporal buffer loads) and only
// written when the kept drafts complete the group: then S += phi(K)^T V over the 64 rows, again by MFMA.
// Up to 96 rows (63 of the open group + 16 drafts, padded with zero rows) and 16 query rows live in LDS.
// Arithmetic: bf16 operands (the logits are exact products of bf16 inputs), fp32 accumulation, S rounded
// to bf16 for the read-out only; the stored state stays fp32, and when a group enters it phi(k) is taken as
// the sum of two bf16 terms (two MFMAs per tile: sixteen significant bits of phi(k) in every product).
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D>
struct VgmCfg {
  static constexpr int NW = D / 32;
  static constexpr int NT = NW * 64;
  static constexpr int GC = 64;              // tokens per group
  static constexpr int RK = 96;              // rows of (open group ++ drafts) in LDS: 63 + 16, padded to three tiles
  static constexpr int NQ = 16;              // query rows (LINATTN_MAX_DRAFT)
  static constexpr int KTL = RK / 32;        // key tiles
  static constexpr int IB = D / 32;
  static constexpr int KSD = D / 16;
  static constexpr int KSR = RK / 16;
  static constexpr int QS = D + 4;           // Q rows: 8-byte row reads
  static constexpr int KS = D + 8;           // K rows: 16-byte row reads, transpose reads
  static constexpr int VS = D + 4;           // history ++ rows: transpose reads, 8-byte row reads
  static constexpr int PS = RK + 8;          // W[j][r], 16-byte row reads
  static constexpr int RP = RK * (D / 8) / NT;   // 8-element pieces of the K (V) rows per thread
};

template <int D>
struct VgmSmem {
  using G = VgmCfg<D>;
  __attribute__((aligned(16))) uint16_t kr[G::RK * G::KS];           // raw key rows; rows < 64 become phi(k) when the group is completed
  __attribute__((aligned(16))) uint16_t v[(HALO + G::RK) * G::VS];    // row HALO + r = value row r; rows < HALO: the history
  __attribute__((aligned(16))) uint16_t qr[G::NQ * G::QS];            // raw q_j
  __attribute__((aligned(16))) uint16_t q[G::NQ * G::QS];             // phi(q_j)
  __attribute__((aligned(16))) uint16_t p[G::NQ * G::PS];             // the weight of value row r in the output of draft j
  __attribute__((aligned(16))) float W[G::NQ][G::RK];                 // logits q_j.k_r
  __attribute__((aligned(16))) float lin[G::NQ][G::GC];               // phi(q_j).phi(k_r), rows of a group being completed
  __attribute__((aligned(16))) float w[8 * D];                        // conv taps, tap-major
  __attribute__((aligned(16))) float z[D];
  float fscale[G::NQ];                                                 // alpha / (phi(q_j).z [+ completed group] + eps), 0 if that is 0
  // qr .. lin are dead once the outputs are complete; when the group is then completed their memory holds
  // the low-order term of phi(k) of its 64 rows
  __device__ uint16_t* klo() { return qr; }                            // [GC][KS]
};
static_assert(offsetof(VgmSmem<128>, w) - offsetof(VgmSmem<128>, qr) >= VgmCfg<128>::GC * VgmCfg<128>::KS * 2 &&
              offsetof(VgmSmem<64>, w) - offsetof(VgmSmem<64>, qr) >= VgmCfg<64>::GC * VgmCfg<64>::KS * 2,
              "the low-order term of phi(K) takes the place of qr, q, p, W and lin");

}  // namespace

// KCM: tap capacity of the instantiation (3, 5 or 8; taps beyond Kc are zeros in LDS and their rows are valid rows), so
// that the output loop over the taps is straight-line code.
template <int D, int KCM>
__global__ __launch_bounds__(D * 2, 2) void verify_grouped_mfma_kernel(VerifyGroupedArgs a) {
  using G = VgmCfg<D>;
  constexpr int GC = G::GC;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  VgmSmem<D>& sm = *reinterpret_cast<VgmSmem<D>*>(smem);
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  const int bh = blockIdx.x;
  const int b = bh / a.H, h = bh % a.H;
  const int kk = a.kk, Kc = a.Kc;
  const int cw = 32 * w + l32;               // the channel this lane owns in the state tiles

  const int64_t tok0 = (int64_t)bh * kk * D;
  const int64_t win0 = (int64_t)bh * GC * D;
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * D;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + tok0;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + tok0;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + tok0;
  uint16_t* wk = static_cast<uint16_t*>(a.kwin) + win0;
  uint16_t* wvp = static_cast<uint16_t*>(a.vwin) + win0;

  // ---- every request first.  The count of rows in use is itself a trip to memory that the rows' addresses have to
  //      wait for: whatever does not need it -- the drafts' q, the small inputs, the first tile of the state -- is
  //      requested ahead of that wait, then the rows (clamped past the end, the data then not used), then the rest
  //      of the state. -------------------------------------------------------------------------------------------
  // q: NQ * D / 8 pieces, at most one per thread
  const int qj = tid / (D / 8), qi0 = 8 * (tid % (D / 8));
  const u32x4 rq = *reinterpret_cast<const u32x4*>(gq + (size_t)(qj < kk ? qj : kk - 1) * D + qi0);
  // taps and history rows: element e = tid + NT m of the [8][D] arrays in LDS; z: one element per thread.  Unconditional,
  // like every request here: a request under a condition that depends on the lane ends in a wait for the requests
  // before it.
  const int cc = tid % D, upper = tid / D;
  constexpr int TAP_IT = 8 * D / G::NT;
  uint32_t tap_reg[TAP_IT], hist_reg[TAP_IT];
  // (one tap: no history, and any address that can be read serves)
  const uint16_t* hsrc = Kc > 1 ? static_cast<const uint16_t*>(a.hist) + hist0 : gq;
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + G::NT * mth;
    const int t = e / D, c = e % D;
    tap_reg[mth] = __float_as_uint(a.conv_w[((size_t)h * D + c) * Kc + (t < Kc ? t : 0)]);
    const int back = HALO - t;                // LDS row t holds the value row HALO - t positions before the first draft
    hist_reg[mth] = hsrc[(size_t)(back <= Kc - 1 ? Kc - 1 - back : 0) * D + c];
  }
  const float zreg = a.z[(size_t)bh * D + cc];
  // (the fences keep the small requests ahead of the state's and every use behind all requests: a use scheduled
  // between two requests is a wait between them)
  __builtin_amdgcn_sched_barrier(0);
  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw]
  const __amdgpu_buffer_rsrc_t Srs =
      __builtin_amdgcn_make_buffer_rsrc(a.S + (size_t)bh * D * D, 0, D * D * 4, 0x00020000);
  const int so = (4 * hi * D + cw) * 4;
  f32x16 Sacc[G::IB];
#pragma unroll
  for (int r = 0; r < 16; ++r)
    Sacc[0][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(Srs, so, (8 * (r >> 2) + (r & 3)) * (D * 4), 2));
  __builtin_amdgcn_sched_barrier(0);
  int n = a.fill[bh];                        // every head carries its own copy of the count
  n = n < 0 ? 0 : (n > GC - 1 ? GC - 1 : n);
  int m = kk;
  if (a.n_commit) { m = a.n_commit[b]; m = m < 0 ? 0 : (m > kk ? kk : m); }
  const int rows = n + kk;                   // rows of (open group ++ drafts)
  const bool crossing = rows > GC;           // some draft belongs to the next group
  u32x4 rk[G::RP], rv[G::RP];
#pragma unroll
  for (int mth = 0; mth < G::RP; ++mth) {
    const int piece = tid + G::NT * mth;
    int r = piece / (D / 8);
    const int i0 = 8 * (piece % (D / 8));
    r = r < rows ? r : rows - 1;
    const uint16_t* ks = r < n ? wk + (size_t)r * D : gk + (size_t)(r - n) * D;
    const uint16_t* vs = r < n ? wvp + (size_t)r * D : gv + (size_t)(r - n) * D;
    rk[mth] = *reinterpret_cast<const u32x4*>(ks + i0);
    rv[mth] = *reinterpret_cast<const u32x4*>(vs + i0);
  }
#pragma unroll
  for (int ib = 1; ib < G::IB; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      Sacc[ib][r] = __builtin_bit_cast(
          float, __builtin_amdgcn_raw_buffer_load_b32(Srs, so, (32 * ib + 8 * (r >> 2) + (r & 3)) * (D * 4), 2));
  __builtin_amdgcn_sched_barrier(0);

  // ---- rows -> LDS (rows past the end are zero rows), q raw and phi(q), history, z, taps -------------
#pragma unroll
  for (int mth = 0; mth < G::RP; ++mth) {
    const int piece = tid + G::NT * mth;
    const int r = piece / (D / 8), i0 = 8 * (piece % (D / 8));
    u32x4 kp = rk[mth], vp = rv[mth];
    if (r >= rows) { kp = u32x4{0, 0, 0, 0}; vp = u32x4{0, 0, 0, 0}; }
    *reinterpret_cast<u32x4*>(sm.kr + r * G::KS + i0) = kp;
    u32x2* vrow = reinterpret_cast<u32x2*>(sm.v + (HALO + r) * G::VS + i0);
    vrow[0] = u32x2{vp[0], vp[1]};
    vrow[1] = u32x2{vp[2], vp[3]};
  }
  static_assert(G::NT / (D / 8) == G::NQ, "every thread has a piece of a query row");
  {
    u32x4 raw = rq, fq = phi_pack8(rq, a.relu);
    if (qj >= kk) { raw = u32x4{0, 0, 0, 0}; fq = u32x4{0, 0, 0, 0}; }
    u32x2* r0 = reinterpret_cast<u32x2*>(sm.qr + qj * G::QS + qi0);
    r0[0] = u32x2{raw[0], raw[1]};
    r0[1] = u32x2{raw[2], raw[3]};
    u32x2* f0 = reinterpret_cast<u32x2*>(sm.q + qj * G::QS + qi0);
    f0[0] = u32x2{fq[0], fq[1]};
    f0[1] = u32x2{fq[2], fq[3]};
  }
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + G::NT * mth;
    const int t = e / D, c = e % D;
    sm.w[t * D + c] = t < Kc ? __uint_as_float(tap_reg[mth]) : 0.f;
    sm.v[t * G::VS + c] = HALO - t <= Kc - 1 ? (uint16_t)hist_reg[mth] : (uint16_t)0;
  }
  if (!upper) sm.z[cc] = zreg;
  __syncthreads();

  // ---- 1. logits: the 32-key tiles of K Q^T (and, for a group being completed, phi(K) phi(Q)^T), dealt out
  //         over the waves; lanes <-> drafts (16 of the 32 columns exist) --------------------------------
  const int qrow = l32 < G::NQ ? l32 : G::NQ - 1;        // lanes beyond the query rows repeat the last one; never kept
#pragma unroll
  for (int s = 0; s < (G::KTL + G::NW - 1) / G::NW; ++s) {
    const int sb = w + s * G::NW;
    if (sb < G::KTL && 32 * sb < rows) {                 // uniform
      f32x16 acc, accl;
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[r] = 0.f; accl[r] = 0.f; }
      const uint16_t* ka = sm.kr + (32 * sb + l32) * G::KS + 8 * hi;
      const uint16_t* qb = sm.qr + qrow * G::QS + 8 * hi;
      const uint16_t* fb = sm.q + qrow * G::QS + 8 * hi;
      const bool need_lin = crossing && 32 * sb < GC;    // uniform
      constexpr int QB = 4;
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
        if (need_lin) {
#pragma unroll
          for (int k2 = 0; k2 < QB; ++k2) {
            const bf16x8 fk = __builtin_bit_cast(bf16x8, phi_pack8(__builtin_bit_cast(u32x4, ak[k2]), a.relu));
            accl = mfma(fk, cat4(lds_row4(fb + 16 * (k0 + k2)), lds_row4(fb + 16 * (k0 + k2) + 4)), accl);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // acc[r]: key row 32sb + 8(r/4) + 4hi + r%4, draft l32
      if (l32 < G::NQ) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 32 * sb + 8 * (r >> 2) + 4 * hi + (r & 3);
          sm.W[l32][row] = acc[r];
          if (need_lin) sm.lin[l32][row] = accl[r];
        }
      }
    }
  }
  __syncthreads();

  // ---- 2. per draft: softmax over its rows, the linear normaliser, the weights of the value rows (bf16) ----
  static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
  constexpr float to_log2 = 1.44269504088896340736f * (D == 64 ? 0.125f : 0.08838834764831845f);
  // Sixteen lanes per draft, four drafts per wave at once, every sum and maximum inside a row of sixteen lanes with
  // DPP modifiers (a wave per draft with the sums across 64 lanes through the LDS crossbar was 18 dependent shuffles
  // per draft: 2.5 us of a workgroup's 10).
  constexpr int RPL = G::RK / 16;                        // rows per lane
#pragma unroll
  for (int j0 = 0; j0 < G::NQ; j0 += 4 * G::NW) {
    const int j = j0 + 4 * w + (lane >> 4), sub = lane & 15;
    const bool live = j < kk;                            // a draft that does not exist has no weights
    const int P = n + j;                                 // position of the draft
    const int g0 = P < GC ? 0 : GC;                      // first row of its group
    float xr[RPL];
    float top = -INFINITY;
#pragma unroll
    for (int t = 0; t < RPL; ++t) {
      const int r = sub + 16 * t;
      const float x = sm.W[j][r];
      xr[t] = (live && r >= g0 && r <= P) ? x : -INFINITY;
      top = fmaxf(top, xr[t]);
    }
    top = max_lanes<16>(top);
    top = live ? top : 0.f;                              // (the draft itself is always seen: finite for a live draft)
    float mass = 0.f;
#pragma unroll
    for (int t = 0; t < RPL; ++t) {
      xr[t] = __builtin_amdgcn_exp2f((xr[t] - top) * to_log2);   // exp2(-inf) = 0: rows that are not seen
      mass += xr[t];
    }
    float dz = 0.f;
#pragma unroll
    for (int e = 0; e < D / 16; ++e) dz = fmaf(bf16_bits_to_f32(sm.q[j * G::QS + sub + 16 * e]), sm.z[sub + 16 * e], dz);
    float lin[GC / 16];
#pragma unroll
    for (int t = 0; t < GC / 16; ++t) lin[t] = sm.lin[j][sub + 16 * t];
    if (g0 > 0) {
#pragma unroll
      for (int t = 0; t < GC / 16; ++t) dz += lin[t];
    }
    mass = sum_lanes<16>(mass);
    dz = sum_lanes<16>(dz);
    const float gden = dz + a.eps;
    const float f = (live && gden != 0.f) ? a.alpha / gden : 0.f;
    const float inv_mass = live ? 1.f / mass : 0.f;      // the draft itself is always seen: mass >= 1
#pragma unroll
    for (int t = 0; t < RPL; ++t) {
      const int r = sub + 16 * t;
      float wgt = xr[t] * inv_mass;
      if (t < GC / 16) wgt = g0 > 0 ? f * lin[t] : wgt;  // the completed group, through the linear branch
      sm.p[j * G::PS + r] = f32_to_bf16_bits(wgt);
    }
    if (sub == 0) sm.fscale[j] = f;
  }
  __syncthreads();

  // ---- 3. this wave's channels: read-out from the state, scaled per draft, plus the value rows ----------
  // vf[ks]: lanes <-> channels 32w + l32, registers <-> rows 16ks + 8hi + 0..7
  bf16x8 vf[G::KSR];
#pragma unroll
  for (int ks = 0; ks < G::KSR; ++ks) vf[ks] = tr_operand(sm.v + HALO * G::VS, G::VS, 16 * ks, 32 * w, lane);
  // o[r] = O[draft l32][channel 32w + 8(r/4) + 4hi + r%4]
  f32x16 o;
#pragma unroll
  for (int r = 0; r < 16; ++r) o[r] = 0.f;
  {
    // register r of S holds feature 32ib + 8(r/4) + 4hi + r%4, so the phi(Q) operand takes features
    // {16h2 + 4hi + 0..3, 16h2 + 8 + 4hi + 0..3} of block ib for MFMA step h2
    const uint16_t* qb = sm.q + qrow * G::QS + 4 * hi;
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const int x = 2 * ib + h2;
        o = mfma(pack8(Sacc[ib], 8 * h2), cat4(lds_row4(qb + 16 * x), lds_row4(qb + 16 * x + 8)), o);
      }
    const float f = sm.fscale[qrow];
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] *= f;
    const uint16_t* pb = sm.p + qrow * G::PS + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSR; ++ks)
      if (16 * ks < rows) o = mfma(vf[ks], lds_row8(pb + 16 * ks), o);   // uniform
  }

  // ---- 4. outputs: add the convolution over (history ++ drafts <= j) -----------------------------------
  if (l32 < kk) {
    const int j = l32;
    const float* wrow = sm.w + 32 * w + 4 * hi;
    uint16_t* orow = static_cast<uint16_t*>(a.out) + tok0 + (int64_t)j * D + 32 * w + 4 * hi;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < KCM; ++t) {
        // tap t looks t rows back from draft j: another draft if t <= j, else history row (t - j) back
        const int row = t <= j ? HALO + n + j - t : HALO - (t - j);
        const f32x4 wv4 = *reinterpret_cast<const f32x4*>(wrow + t * D + 8 * g);
        const u32x2 x = *reinterpret_cast<const u32x2*>(sm.v + row * G::VS + 32 * w + 4 * hi + 8 * g);
        u[0] = fmaf(wv4[0], bf16_lo_to_f32(x[0]), u[0]);
        u[1] = fmaf(wv4[1], bf16_hi_to_f32(x[0]), u[1]);
        u[2] = fmaf(wv4[2], bf16_lo_to_f32(x[1]), u[2]);
        u[3] = fmaf(wv4[3], bf16_hi_to_f32(x[1]), u[3]);
      }
      *reinterpret_cast<u32x2*>(orow + 8 * g) =
          u32x2{pack_bf16x2(o[4 * g] + u[0], o[4 * g + 1] + u[1]), pack_bf16x2(o[4 * g + 2] + u[2], o[4 * g + 3] + u[3])};
    }
  }

  // ---- 5. the kept drafts join the state --------------------------------------------------------------
  if (m == 0) return;                                    // uniform: nothing kept, nothing changes
  if (tid == 0) a.fill[bh] = (n + m) % GC;
  if (upper) {
    // the last Kc-1 rows of (history ++ kept drafts): position sidx is a draft row or, if negative, -sidx rows back
    for (int r = 0; r < Kc - 1; ++r) {
      const int sidx = m - (Kc - 1) + r;
      const int row = sidx >= 0 ? HALO + n + sidx : HALO + sidx;
      static_cast<uint16_t*>(a.hist)[hist0 + (int64_t)r * D + cc] = sm.v[row * G::VS + cc];
    }
  }
  if (n + m < GC) {
    // the group stays open: drafts 0..m-1 become rows n..n+m-1
    for (int e = tid; e < m * (D / 8); e += G::NT) {
      const int r = n + e / (D / 8), i0 = 8 * (e % (D / 8));
      *reinterpret_cast<u32x4*>(wk + (size_t)r * D + i0) = *reinterpret_cast<const u32x4*>(sm.kr + r * G::KS + i0);
      const u32x2* vrow = reinterpret_cast<const u32x2*>(sm.v + (HALO + r) * G::VS + i0);
      const u32x2 v0 = vrow[0], v1 = vrow[1];
      *reinterpret_cast<u32x4*>(wvp + (size_t)r * D + i0) = u32x4{v0[0], v0[1], v1[0], v1[1]};
    }
    return;
  }
  // the group is complete: rows 0..63 enter S and z.  Their keys get the feature map in place first.
  __syncthreads();                                       // every wave is done with the raw rows, the queries and the weights
  for (int e = tid; e < GC * (D / 8); e += G::NT) {
    const int r = e / (D / 8), i0 = 8 * (e % (D / 8));
    u32x4* p8 = reinterpret_cast<u32x4*>(sm.kr + r * G::KS + i0);
    u32x4 fh, fl;
    phi_split8(*p8, a.relu, fh, fl);
    *p8 = fh;
    *reinterpret_cast<u32x4*>(sm.klo() + r * G::KS + i0) = fl;
  }
  __syncthreads();
#pragma unroll
  for (int ib = 0; ib < G::IB; ++ib) {
#pragma unroll
    for (int ks = 0; ks < GC / 16; ++ks) {
      Sacc[ib] = mfma(tr_operand(sm.klo(), G::KS, 16 * ks, 32 * ib, lane), vf[ks], Sacc[ib]);
      Sacc[ib] = mfma(tr_operand(sm.kr, G::KS, 16 * ks, 32 * ib, lane), vf[ks], Sacc[ib]);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r)
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(Sacc[ib][r]), Srs, so,
                                            (32 * ib + 8 * (r >> 2) + (r & 3)) * (D * 4), 2);
  }
  if (!upper) {
    float zs = zreg;
    for (int r = 0; r < GC; ++r) zs += bf16_bits_to_f32(sm.kr[r * G::KS + cc]) + bf16_bits_to_f32(sm.klo()[r * G::KS + cc]);
    a.z[(size_t)bh * D + cc] = zs;
  }
  // the next group opens with the kept drafts beyond the completed one: rows 64 .. n+m-1 -> rows 0 ..
  for (int e = tid; e < (n + m - GC) * (D / 8); e += G::NT) {
    const int r = e / (D / 8), i0 = 8 * (e % (D / 8));
    *reinterpret_cast<u32x4*>(wk + (size_t)r * D + i0) = *reinterpret_cast<const u32x4*>(sm.kr + (GC + r) * G::KS + i0);
    const u32x2* vrow = reinterpret_cast<const u32x2*>(sm.v + (HALO + GC + r) * G::VS + i0);
    const u32x2 v0 = vrow[0], v1 = vrow[1];
    *reinterpret_cast<u32x4*>(wvp + (size_t)r * D + i0) = u32x4{v0[0], v0[1], v1[0], v1[1]};
  }
}

template <int D, int KCM>
static hipError_t launch_vgm(const VerifyGroupedArgs& a, hipStream_t st) {
  auto kern = verify_grouped_mfma_kernel<D, KCM>;
  constexpr int LDS = (int)sizeof(VgmSmem<D>);
  static_assert(LDS <= 80 * 1024, "two workgroups per compute unit");
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, LDS);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H)), dim3(VgmCfg<D>::NT), LDS, st, a);
  return hipGetLastError();
}

// bf16 drafts, from four of them on; below that the vector-ALU kernel is as fast or faster (fewer fixed steps, four
// workgroups per CU instead of two).
bool verify_grouped_mfma_available(bool bf16, int d, int kk) { return bf16 && kk >= 4 && kk <= 16 && (d == 64 || d == 128); }

hipError_t launch_verify_grouped_mfma(const VerifyGroupedArgs& a, int d, hipStream_t st) {
  if (d == 128) return a.Kc <= 3 ? launch_vgm<128, 3>(a, st) : a.Kc <= 5 ? launch_vgm<128, 5>(a, st) : launch_vgm<128, 8>(a, st);
  return a.Kc <= 3 ? launch_vgm<64, 3>(a, st) : a.Kc <= 5 ? launch_vgm<64, 5>(a, st) : launch_vgm<64, 8>(a, st);
}

}  // namespace linattn
