// Tree-structured speculative verification (Sec. 4.2, "Proposed Solution").
//
// The n <= 64 candidate tokens of a speculation step hang off the verified sequence as a
// tree (parent[i] < i, or -1 for a candidate that follows the verified sequence
// directly).  Candidate i is scored from the verified state and from the candidates on
// its own root path only, and its convolution window is that path read backwards,
// continuing into the verified history.  That is one 64-token group of the chunked form
// with the causal mask replaced by the ancestor-or-self relation of the tree (which is
// still lower triangular, because parents come first) and the conv taps gathered along
// the path (the "unfolded" convolution of the paper): all candidates share one read of the
// state, and a common prefix of several candidates is scored once.
//
//   O^T  = S0^T phi(Q)^T + V^T P^T        P^T = on_path(phi(K) phi(Q)^T)   (select mask)
//   S   += phi(K_acc)^T V                 K_acc: the rows on the accepted root path, else zero
//
// One workgroup per (b, h), D/32 waves; wave w owns value channels 32w..32w+31, i.e. the
// column block S[:, 32w:32w+32] as D/32 MFMA accumulator tiles, requested first thing and
// written straight back (nontemporal, buffer addressing), as in the chain kernel.  The
// score tiles are shared through LDS.  Arithmetic: bf16 operands, fp32 accumulation; the
// stored state stays fp32, and the state update takes phi(k) as the sum of two bf16 terms (two
// MFMAs per tile), so that every product entering S carries sixteen significant bits of phi(k).
// Nothing accepted = nothing written.
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D>
struct VtCfg {
  static constexpr int NW = D / 32;
  static constexpr int NT = NW * 64;
  static constexpr int KT = 64;              // candidate rows in LDS (LINATTN_MAX_TREE)
  static constexpr int TB = KT / 32;
  static constexpr int IB = D / 32;
  static constexpr int KSD = D / 16;
  static constexpr int KSC = KT / 16;
  static constexpr int QS = D + 4;           // phi(Q): 8-byte row reads
  static constexpr int KS = D + 8;           // phi(K): 16-byte row reads, transpose reads
  static constexpr int VS = D + 4;           // history ++ candidates: transpose reads, 8-byte row reads
  static constexpr int PS = KT + 8;          // P[i][a], 16-byte row reads
  static constexpr int NTILE = TB * (TB + 1) / 2;
  static constexpr int QP = KT * (D / 8) / NT;   // 8-element pieces of q (k, v) per thread
};

template <int D>
struct VtSmem {
  using G = VtCfg<D>;
  // q and p are only read until the outputs' accumulators are complete; after that their memory holds the
  // low-order term of phi(K) for the state update (klo() below)
  __attribute__((aligned(16))) uint16_t q[G::KT * G::QS];
  __attribute__((aligned(16))) uint16_t p[G::KT * G::PS];
  __attribute__((aligned(16))) uint16_t k[G::KT * G::KS];            // phi(K) rounded to bf16
  __attribute__((aligned(16))) uint16_t v[(HALO + G::KT) * G::VS];   // row r = candidate r - HALO
  __attribute__((aligned(16))) float w[8 * D];                       // conv taps, tap-major
  __attribute__((aligned(16))) float z[D];
  __attribute__((aligned(16))) float denq[4][G::KT];                 // phi(q).z, one part per quarter of the features
  __attribute__((aligned(16))) float denp[G::TB][G::KT];             // row sums of the score tiles
  __attribute__((aligned(16))) unsigned long long onpath[G::KT];     // bit a of row i: candidate a is on the root path of i
  __attribute__((aligned(16))) uint8_t taprow[G::KT][8];             // row of sm.v that tap t of candidate i reads
  int parent[G::KT];
  __device__ uint16_t* klo() { return q; }                           // [KT][KS], over q and p
};
static_assert(sizeof(VtSmem<128>::q) + sizeof(VtSmem<128>::p) >= sizeof(VtSmem<128>::k) &&
              sizeof(VtSmem<64>::q) + sizeof(VtSmem<64>::p) >= sizeof(VtSmem<64>::k) &&
              offsetof(VtSmem<128>, p) == sizeof(VtSmem<128>::q) && offsetof(VtSmem<64>, p) == sizeof(VtSmem<64>::q),
              "the low-order term of phi(K) takes the place of q and p");

}  // namespace

// KCM: tap capacity of the instantiation (3, 5 or 8; taps beyond Kc are zeros in LDS and their rows are valid rows):
// the epilogue's loops over the taps are straight-line code -- a test of the tap count per tap and channel group cut
// them into sixty basic blocks, each with a full wait at its end.
template <int D, int KCM>
__global__ __launch_bounds__(D * 2, 2) void verify_tree_kernel(VerifyTreeArgs a) {
  using G = VtCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  VtSmem<D>& sm = *reinterpret_cast<VtSmem<D>*>(smem);
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  const int bh = blockIdx.x;
  const int b = bh / a.H, h = bh % a.H;
  const int n = a.n, Kc = a.Kc;
  const int cw = 32 * w + l32;               // the channel this lane owns in the state tiles

  // ---- every request of the call is issued before anything waits: the candidates and the small inputs first (they
  //      are needed first), then the state.  All of them unconditional -- a request under a condition that depends on
  //      the lane ends in a wait for everything before it, and three of those in a row kept the state requests back
  //      for three trips to memory --: indices past the end are clamped and what they bring is dropped. ------------
  const int64_t tok0 = (int64_t)bh * n * D;
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * D;
  u32x4 rq[G::QP], rk[G::QP], rv[G::QP];
#pragma unroll
  for (int m = 0; m < G::QP; ++m) {
    const int piece = tid + G::NT * m;
    const int dj = piece / (D / 8), di0 = 8 * (piece % (D / 8));
    const int64_t off = tok0 + (int64_t)(dj < n ? dj : n - 1) * D + di0;
    rq[m] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.q) + off);
    rk[m] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.k) + off);
    rv[m] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.v) + off);
  }
  // taps and history rows: element e = tid + NT m of the [8][D] arrays in LDS; z and parent: one element per thread
  constexpr int TAP_IT = 8 * D / G::NT;
  uint32_t tap_reg[TAP_IT], hist_reg[TAP_IT];
  // (one tap: no history, and any address that can be read serves)
  const uint16_t* hsrc = Kc > 1 ? static_cast<const uint16_t*>(a.hist) + hist0 : static_cast<const uint16_t*>(a.v) + tok0;
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + G::NT * mth;
    const int t = e / D, c = e % D;
    tap_reg[mth] = __float_as_uint(a.conv_w[((size_t)h * D + c) * Kc + (t < Kc ? t : 0)]);
    const int back = HALO - t;                // LDS row t holds the value row HALO - t positions before the candidates
    hist_reg[mth] = hsrc[(size_t)(back <= Kc - 1 ? Kc - 1 - back : 0) * D + c];
  }
  const int cc = tid % D, upper = tid / D;
  const float zreg = a.z[(size_t)bh * D + cc];
  const int par_raw = a.parent[tid < n ? tid : 0];
  int acc_node = -1;
  if (a.accept) { acc_node = a.accept[b]; acc_node = (acc_node < 0 || acc_node >= n) ? -1 : acc_node; }

  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw]; nontemporal buffer requests (descriptor in scalar
  // registers + one lane offset + a constant each).  A wave can have 63 requests under way: the first half of the
  // tiles goes out here, the second when the candidates have arrived, so that no request has to wait for a free slot.
  const __amdgpu_buffer_rsrc_t Srs =
      __builtin_amdgcn_make_buffer_rsrc(a.S + (size_t)bh * D * D, 0, D * D * 4, 0x00020000);
  const int so = (4 * hi * D + cw) * 4;
  f32x16 Sacc[G::IB];
  constexpr int IB0 = G::IB > 2 ? G::IB / 2 : G::IB;
#pragma unroll
  for (int ib = 0; ib < IB0; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      Sacc[ib][r] = __builtin_bit_cast(
          float, __builtin_amdgcn_raw_buffer_load_b32(Srs, so, (32 * ib + 8 * (r >> 2) + (r & 3)) * (D * 4), 2));
  __builtin_amdgcn_sched_barrier(0);

  // ---- candidates -> LDS: phi(Q), phi(K) as bf16 rows (rows >= n are zero rows), V, history, z, taps --
  u32x4 kl[G::QP];                                       // phi(K) - bf16(phi(K)): stays in registers until q and p are free
#pragma unroll
  for (int m = 0; m < G::QP; ++m) {
    const int piece = tid + G::NT * m;
    const int dj = piece / (D / 8), di0 = 8 * (piece % (D / 8));
    u32x4 qp = phi_pack8_nb(rq[m], a.relu ? 0.f : 1.f), kp, vp = rv[m];
    phi_split8_nb(rk[m], a.relu ? 0.f : 1.f, kp, kl[m]);
    if (dj >= n) { qp = u32x4{0, 0, 0, 0}; kp = u32x4{0, 0, 0, 0}; kl[m] = u32x4{0, 0, 0, 0}; vp = u32x4{0, 0, 0, 0}; }
    u32x2* qrow = reinterpret_cast<u32x2*>(sm.q + dj * G::QS + di0);
    qrow[0] = u32x2{qp[0], qp[1]};
    qrow[1] = u32x2{qp[2], qp[3]};
    *reinterpret_cast<u32x4*>(sm.k + dj * G::KS + di0) = kp;
    u32x2* vrow = reinterpret_cast<u32x2*>(sm.v + (HALO + dj) * G::VS + di0);
    vrow[0] = u32x2{vp[0], vp[1]};
    vrow[1] = u32x2{vp[2], vp[3]};
  }
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + G::NT * mth;
    const int t = e / D, c = e % D;
    sm.w[t * D + c] = t < Kc ? __uint_as_float(tap_reg[mth]) : 0.f;
    sm.v[t * G::VS + c] = HALO - t <= Kc - 1 ? (uint16_t)hist_reg[mth] : (uint16_t)0;
  }
  if (!upper) sm.z[cc] = zreg;
  if (tid < G::KT) sm.parent[tid] = (tid < n && par_raw >= -1 && par_raw < tid) ? par_raw : -1;   // a malformed entry starts a new root
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int ib = IB0; ib < G::IB; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      Sacc[ib][r] = __builtin_bit_cast(
          float, __builtin_amdgcn_raw_buffer_load_b32(Srs, so, (32 * ib + 8 * (r >> 2) + (r & 3)) * (D * 4), 2));
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();

  // ---- the tree: for every candidate the set of candidates on its root path and, tap by tap, the
  //      row its convolution reads (the path backwards, then the history) -----------------------------
  if (tid < G::KT) {
    unsigned long long bits = 0ull;
    int steps = 0;
    if (tid < n) {
      for (int c = tid; c >= 0; c = sm.parent[c]) {   // at most n steps: parents have smaller indices
        bits |= 1ull << c;
        if (steps < 8) sm.taprow[tid][steps] = (uint8_t)(HALO + c);
        ++steps;
      }
    }
    for (int t = steps; t < 8; ++t) {
      const int back = t - steps + 1;                  // rows into the history
      sm.taprow[tid][t] = (uint8_t)(back <= HALO ? HALO - back : 0);
    }
    sm.onpath[tid] = bits;
  }
  // phi(q_i).z: thread (i = tid % 64, part = tid / 64) sums its share of the features
  {
    constexpr int NPART = G::NT / G::KT;               // 4 at D = 128, 2 at D = 64
    constexpr int FPP = D / NPART;                     // features per part
    const int i = tid % G::KT, part = tid / G::KT;
    const uint16_t* qrow = sm.q + i * G::QS + part * FPP;
    const float* zrow = sm.z + part * FPP;
    float dq = 0.f;
#pragma unroll
    for (int x = 0; x < FPP / 4; ++x) {
      const u32x2 pk = *reinterpret_cast<const u32x2*>(qrow + 4 * x);
      const f32x4 zv = *reinterpret_cast<const f32x4*>(zrow + 4 * x);
      dq = fmaf(bf16_lo_to_f32(pk[0]), zv[0], dq);
      dq = fmaf(bf16_hi_to_f32(pk[0]), zv[1], dq);
      dq = fmaf(bf16_lo_to_f32(pk[1]), zv[2], dq);
      dq = fmaf(bf16_hi_to_f32(pk[1]), zv[3], dq);
    }
    sm.denq[part][i] = dq;
    if (NPART < 4) { sm.denq[2][i] = 0.f; sm.denq[3][i] = 0.f; }
  }
  __syncthreads();

  // ---- scores: the lower-triangular 32 x 32 tiles of P^T = phi(K) phi(Q)^T, kept where the source
  //      candidate is on the query candidate's root path; tiles are dealt out over the waves -----------
#pragma unroll
  for (int s = 0; s < (G::NTILE + G::NW - 1) / G::NW; ++s) {
    const int idx = w + s * G::NW;
    if (idx < G::NTILE) {
      int tb = 0;
      while ((tb + 1) * (tb + 2) / 2 <= idx) ++tb;
      const int sb = idx - tb * (tb + 1) / 2;
      const int qi = 32 * tb + l32;                      // the query candidate of this lane
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      if (32 * tb < n) {                                 // uniform: a tile of rows that do not exist stays zero
        const uint16_t* ka = sm.k + (32 * sb + l32) * G::KS + 8 * hi;
        const uint16_t* qb = sm.q + qi * G::QS + 8 * hi;
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
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // acc[r]: source candidate 32sb + 8(r/4) + 4hi + r%4, query candidate qi
      const unsigned long long vis = sm.onpath[qi];
      float rs = 0.f;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int src = 32 * sb + 8 * g + 4 * hi + e;
          x[e] = ((vis >> src) & 1ull) ? acc[4 * g + e] : 0.f;   // select, never multiply: nothing off the path can leak
          rs += x[e];
        }
        *reinterpret_cast<u32x2*>(sm.p + qi * G::PS + 32 * sb + 8 * g + 4 * hi) =
            u32x2{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
      }
      rs += __shfl_xor(rs, 32);
      if (lane < 32) sm.denp[sb][qi] = rs;
    }
  }
  __syncthreads();

  // ---- this wave's channels: read-out from the state as it was, plus the path's own contribution ----
  // vf[ks]: lanes <-> channels 32w + l32, registers <-> candidates 16ks + 8hi + 0..7
  bf16x8 vf[G::KSC];
#pragma unroll
  for (int ks = 0; ks < G::KSC; ++ks) vf[ks] = tr_operand(sm.v + HALO * G::VS, G::VS, 16 * ks, 32 * w, lane);
  // o[tb][r] = O[candidate 32tb + l32][channel 32w + 8(r/4) + 4hi + r%4]
  f32x16 o[G::TB];
#pragma unroll
  for (int tb = 0; tb < G::TB; ++tb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) o[tb][r] = 0.f;
    if (32 * tb < n) {                                   // uniform
      const int qi = 32 * tb + l32;
      const uint16_t* pb = sm.p + qi * G::PS + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < 2 * (tb + 1); ++ks) o[tb] = mfma(vf[ks], lds_row8(pb + 16 * ks), o[tb]);
      // register r of S holds feature 32ib + 8(r/4) + 4hi + r%4, so the phi(Q) operand takes features
      // {16h2 + 4hi + 0..3, 16h2 + 8 + 4hi + 0..3} of block ib for MFMA step h2
      const uint16_t* qb = sm.q + qi * G::QS + 4 * hi;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const int x = 2 * ib + h2;
          o[tb] = mfma(pack8(Sacc[ib], 8 * h2), cat4(lds_row4(qb + 16 * x), lds_row4(qb + 16 * x + 8)), o[tb]);
        }
    }
  }

  // ---- the state moves along the accepted root path (rows off the path are masked out of phi(K)^T) ---
  const unsigned long long commit = acc_node >= 0 ? sm.onpath[acc_node] : 0ull;
  if (acc_node >= 0) {   // uniform per workgroup; nothing accepted leaves the state untouched
    __syncthreads();     // every wave has read q and p for the last time
#pragma unroll
    for (int m = 0; m < G::QP; ++m) {
      const int piece = tid + G::NT * m;
      *reinterpret_cast<u32x4*>(sm.klo() + (piece / (D / 8)) * G::KS + 8 * (piece % (D / 8))) = kl[m];
    }
    __syncthreads();
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib) {
#pragma unroll
      for (int ks = 0; ks < G::KSC; ++ks) {
        {                                                // (candidates that do not exist are not on the path: masked)
          u32x4 keep;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int c0 = 16 * ks + 8 * hi + 2 * i;     // candidates c0 (low half) and c0 + 1 (high half)
            keep[i] = (((commit >> c0) & 1ull) ? 0x0000ffffu : 0u) | (((commit >> (c0 + 1)) & 1ull) ? 0xffff0000u : 0u);
          }
          const u32x4 kt = __builtin_bit_cast(u32x4, tr_operand(sm.k, G::KS, 16 * ks, 32 * ib, lane)) & keep;
          const u32x4 ktl = __builtin_bit_cast(u32x4, tr_operand(sm.klo(), G::KS, 16 * ks, 32 * ib, lane)) & keep;
          Sacc[ib] = mfma(__builtin_bit_cast(bf16x8, ktl), vf[ks], Sacc[ib]);
          Sacc[ib] = mfma(__builtin_bit_cast(bf16x8, kt), vf[ks], Sacc[ib]);
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(Sacc[ib][r]), Srs, so,
                                              (32 * ib + 8 * (r >> 2) + (r & 3)) * (D * 4), 2);
    }
  }

  // ---- outputs: normalise, add the convolution gathered along the root path ---------------------------
#pragma unroll
  for (int tb = 0; tb < G::TB; ++tb) {
    const int qi = 32 * tb + l32;
    if (qi < n) {
      float den = a.eps + (sm.denq[0][qi] + sm.denq[1][qi]) + (sm.denq[2][qi] + sm.denq[3][qi]);
#pragma unroll
      for (int sb = 0; sb <= tb; ++sb) den += sm.denp[sb][qi];
      const float inv = __builtin_amdgcn_rcpf(den);
      const float* wrow = sm.w + 32 * w + 4 * hi;
      uint16_t* orow = static_cast<uint16_t*>(a.out) + tok0 + (int64_t)qi * D + 32 * w + 4 * hi;
      int rows[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) rows[t] = sm.taprow[qi][t];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < KCM; ++t) {
          const f32x4 wv4 = *reinterpret_cast<const f32x4*>(wrow + t * D + 8 * g);
          const u32x2 x = *reinterpret_cast<const u32x2*>(sm.v + rows[t] * G::VS + 32 * w + 4 * hi + 8 * g);
          u[0] = fmaf(wv4[0], bf16_lo_to_f32(x[0]), u[0]);
          u[1] = fmaf(wv4[1], bf16_hi_to_f32(x[0]), u[1]);
          u[2] = fmaf(wv4[2], bf16_lo_to_f32(x[1]), u[2]);
          u[3] = fmaf(wv4[3], bf16_hi_to_f32(x[1]), u[3]);
        }
        *reinterpret_cast<u32x2*>(orow + 8 * g) =
            u32x2{pack_bf16x2(fmaf(o[tb][4 * g], inv, u[0]), fmaf(o[tb][4 * g + 1], inv, u[1])),
                  pack_bf16x2(fmaf(o[tb][4 * g + 2], inv, u[2]), fmaf(o[tb][4 * g + 3], inv, u[3]))};
      }
    }
  }

  // ---- the rest of the state: normaliser and history ----------------------------------------------------
  if (acc_node < 0) return;   // uniform per workgroup
  {
    // z += the sum of phi(k) over the accepted path, both terms: this wave's 32 features as one more tile against an
    // all-ones operand (as a loop over the rows it was 64 dependent trips to LDS on half of the waves, at the very end
    // of the workgroup).  Zacc[r] = the increment of z[32w + 8(r/4) + 4hi + r%4], the same in every lane of a half wave.
    f32x16 Zacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) Zacc[r] = 0.f;
    const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
#pragma unroll
    for (int ks = 0; ks < G::KSC; ++ks) {
      u32x4 keep;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c0 = 16 * ks + 8 * hi + 2 * i;
        keep[i] = (((commit >> c0) & 1ull) ? 0x0000ffffu : 0u) | (((commit >> (c0 + 1)) & 1ull) ? 0xffff0000u : 0u);
      }
      const u32x4 kt = __builtin_bit_cast(u32x4, tr_operand(sm.k, G::KS, 16 * ks, 32 * w, lane)) & keep;
      const u32x4 ktl = __builtin_bit_cast(u32x4, tr_operand(sm.klo(), G::KS, 16 * ks, 32 * w, lane)) & keep;
      Zacc = mfma(__builtin_bit_cast(bf16x8, ktl), ones, Zacc);
      Zacc = mfma(__builtin_bit_cast(bf16x8, kt), ones, Zacc);
    }
    float inc = Zacc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) inc = l32 == r ? Zacc[r] : inc;
    if (l32 < 16) {
      const int f = 32 * w + 8 * (l32 >> 2) + 4 * hi + (l32 & 3);
      a.z[(size_t)bh * D + f] = sm.z[f] + inc;
    }
  }
  if (upper) {
    // the last Kc-1 rows of (history ++ accepted path) are what the taps 0..Kc-2 of the accepted candidate read
    for (int r = 0; r < Kc - 1; ++r)
      static_cast<uint16_t*>(a.hist)[hist0 + (int64_t)r * D + cc] = sm.v[sm.taprow[acc_node][Kc - 2 - r] * G::VS + cc];
  }
}

template <int D, int KCM>
static hipError_t launch_vt(const VerifyTreeArgs& a, hipStream_t st) {
  auto kern = verify_tree_kernel<D, KCM>;
  constexpr int LDS = (int)sizeof(VtSmem<D>);
  static_assert(LDS <= 80 * 1024, "two workgroups per compute unit");
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, LDS);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H)), dim3(VtCfg<D>::NT), LDS, st, a);
  return hipGetLastError();
}

hipError_t launch_verify_tree(const VerifyTreeArgs& a, int d, hipStream_t st) {
  if (d == 128) return a.Kc <= 3 ? launch_vt<128, 3>(a, st) : a.Kc <= 5 ? launch_vt<128, 5>(a, st) : launch_vt<128, 8>(a, st);
  return a.Kc <= 3 ? launch_vt<64, 3>(a, st) : a.Kc <= 5 ? launch_vt<64, 5>(a, st) : launch_vt<64, 8>(a, st);
}

}  // namespace linattn
