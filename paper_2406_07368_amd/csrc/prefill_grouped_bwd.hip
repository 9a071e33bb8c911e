// Gradient of the three-branch form of Sec. 4.1 on the matrix cores (bf16 rows): the training direction of the
// paper's FLASH experiment (Sec. 5.3 times a training step, forward and backward, in groups of 256 tokens).
//
// With P_g = (S_g, z_g) the sums over everything before group g and D_g the gradient with respect to the sums after
// group g, for a token t of group g and the incoming gradient dO = d loss / d out:
//
//   grouped branch   N = S_g^T phi(q_t),  den = phi(q_t).z_g + eps,  f = alpha / den:
//                    W = S_g dO_t,  nd = phi(q_t).W,  dden = -f nd / den,
//                    dq_t += (f W + z_g dden) * phi'(q_t),   G_g += phi(q_t) (f dO_t)^T,   gz_g += phi(q_t) dden
//   local branch     p = softmax over the keys i <= t of the group of q_t.k_i / sqrt(d),  dp_i = dO_t.v_i,
//                    pbar = sum_i p_i dp_i,  ds_i = p_i (dp_i - pbar) / sqrt(d):
//                    dq_t += sum_i ds_i k_i,   dk_i += ds_i q_t,   dv_i += p_i dO_t
//   the sums         D_g = sum_{g' > g} (G_g', gz_g'):  dk_i += (D_g.S v_i + D_g.z) * phi'(k_i),  dv_i += D_g.S^T phi(k_i)
//   conv             dv_s += sum_j w[c][j] dO[s + j][c],   dw[c][j] = sum_t dO[t][c] v[t - j][c]   (conv_long.hip)
//
// One workgroup per (b, h, group), GT / 32 waves, everything a 32 x 32 x 16 bf16 MFMA with fp32 accumulation:
//   grouped_bwd_dq_kernel     wave = 32 queries; the group's K and V rows in LDS.  Pass 1 over the key tiles up to the
//                             diagonal: scores, running maximum and sum, and the running sum of e_i dp_i (so pbar needs
//                             no pass of its own).  Pass 2: scores and dp again, ds from the accumulators as the MFMA
//                             operand (accumulator order applied to the transposed reads of K), dQ^T += K^T ds^T.  Then
//                             the grouped branch with S_g in LDS as bf16.  Hands the per-token scalars on.
//   grouped_bwd_gs_kernel     G_g = (f phi(Q))^T dO and gz_g, contraction over the group's tokens.
//   grouped_bwd_suffix_kernel D_g = sum over the later groups, in place.
//   grouped_bwd_dkdv_kernel   wave = 32 keys; the group's Q and dO rows in LDS; one workgroup for dV, one for dK (the
//                             accumulators of both do not fit next to the operands of both).
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D, int GT>
struct BwdCfg {
  static constexpr int NW = GT / 32;         // waves: one 32-row tile each
  static constexpr int NT = NW * 64;
  static constexpr int KSD = D / 16;         // contraction steps over features / channels
  static constexpr int CT = D / 32;          // 32-wide tiles of features / channels
  static constexpr int KS = D + 8;           // token rows: 16-byte row reads and transposed reads
  static constexpr int SS = D + 8;           // rows of a d x d operand [feature][channel]
  static constexpr int OS = D + 4;           // staged fp32 output rows
  static constexpr int RP = GT < 128 ? GT : 128;   // rows per staging pass
  static constexpr int OFF_A = 0;                  // K rows (dq kernel), Q rows (the others)
  static constexpr int OFF_B = GT * KS * 2;        // V rows, dO rows
  // the d x d operand (as two bf16 terms, hi and lo) and the staged outputs take the place of the token rows
  static constexpr int ROWS = 2 * GT * KS * 2, SREG = 2 * D * SS * 2, STG = RP * OS * 4;
  static constexpr int REGION = ((ROWS > SREG ? (ROWS > STG ? ROWS : STG) : (SREG > STG ? SREG : STG)) + 15) / 16 * 16;
  static constexpr int OFF_Z = REGION;             // [D] float
  static constexpr int OFF_ST = OFF_Z + D * 4;     // [3][GT] float: per-token scalars
  static constexpr int OFF_RED = OFF_ST + 3 * GT * 4;   // [NT] float: partial sums of the z passes
  static constexpr int TOTAL = OFF_RED + NT * 4;
  static constexpr int SLOT = D * D + D;
  static_assert(TOTAL <= 160 * 1024, "LDS");
  static_assert(NT >= D, "one thread per feature in the z passes");
};

// phi(x) and phi'(x) without a branch on the feature map (a branch per element would cut the unrolled loops into
// pieces): with one = 1 for elu + 1 and 0 for max(x, 0), phi = max(x + one, one * min(exp(x), 1)) and
// phi' = 1 above zero, one * exp(x) below.
__device__ __forceinline__ float phi_f(float x, int relu) {
  const float one = relu ? 0.f : 1.f;
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(x * 1.44269504088896340736f), 0.f, 1.f);
  return fmaxf(x + one, one * e);
}
__device__ __forceinline__ float dphi_f(float x, int relu) {
  const float one = relu ? 0.f : 1.f;
  return x > 0.f ? 1.f : one * __builtin_amdgcn_exp2f(x * 1.44269504088896340736f);
}

// rows tok0 .. tok0 + GT - 1 of two tensors -> LDS (rows past the end are zero rows); every request before the first store
template <int D, int GT>
__device__ __forceinline__ void load_rows2(const uint16_t* ga, const uint16_t* gb, int64_t st, int tok0, int nt,
                                           uint16_t* La, uint16_t* Lb, int tid) {
  using G = BwdCfg<D, GT>;
  constexpr int NPC = GT * (D / 8) / G::NT;
  u32x4 ax[NPC], bx[NPC];
#pragma unroll
  for (int i = 0; i < NPC; ++i) {
    const int e = tid + G::NT * i;
    const int r = e / (D / 8), c0 = 8 * (e % (D / 8));
    const int rr = r < nt ? r : nt - 1;        // unconditional requests; a row that does not exist is replaced by zeros
    ax[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ga + (int64_t)(tok0 + rr) * st + c0));
    bx[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gb + (int64_t)(tok0 + rr) * st + c0));
  }
#pragma unroll
  for (int i = 0; i < NPC; ++i) {
    const int e = tid + G::NT * i;
    const int r = e / (D / 8), c0 = 8 * (e % (D / 8));
    const u32x4 zero = {0, 0, 0, 0};
    *reinterpret_cast<u32x4*>(La + r * G::KS + c0) = r < nt ? ax[i] : zero;
    *reinterpret_cast<u32x4*>(Lb + r * G::KS + c0) = r < nt ? bx[i] : zero;
  }
}

// a slot's d x d part -> LDS as two bf16 arrays [feature][channel] (row stride SS), hi = bf16(x) at Sl and
// lo = bf16(x - hi) at Sl + D * SS; its d-vector -> LDS as fp32.  Two terms because what is computed from these sums is
// a difference of two nearly equal parts (the derivative of a ratio: numerator part minus denominator part), which the
// rounding of one bf16 term (2^-9 of the common part) would swamp.
template <int D, int GT>
__device__ __forceinline__ void load_slot(const float* slot, uint16_t* Sl, float* zl, int tid) {
  using G = BwdCfg<D, GT>;
  constexpr int SIT = D * D / 4 / G::NT;
  f32x4 sx[SIT];
#pragma unroll
  for (int i = 0; i < SIT; ++i) sx[i] = reinterpret_cast<const f32x4*>(slot)[tid + G::NT * i];
  const float zx = tid < D ? slot[D * D + tid] : 0.f;
#pragma unroll
  for (int i = 0; i < SIT; ++i) {
    const int e = 4 * (tid + G::NT * i);
    const u32x2 h = {pack_bf16x2(sx[i][0], sx[i][1]), pack_bf16x2(sx[i][2], sx[i][3])};
    const u32x2 l = {pack_bf16x2(sx[i][0] - bf16_lo_to_f32(h[0]), sx[i][1] - bf16_hi_to_f32(h[0])),
                     pack_bf16x2(sx[i][2] - bf16_lo_to_f32(h[1]), sx[i][3] - bf16_hi_to_f32(h[1]))};
    *reinterpret_cast<u32x2*>(Sl + (e / D) * G::SS + e % D) = h;
    *reinterpret_cast<u32x2*>(Sl + D * G::SS + (e / D) * G::SS + e % D) = l;
  }
  if (tid < D) zl[tid] = zx;
}

// acc[ct][r] = X[row 32w + l32][column 32ct + 8(r/4) + 4hi + r%4] (w: the wave's row tile) -> global bf16 rows, staged
// through LDS in fp32, RP rows at a time (the waves of one pass write, all threads store whole rows).  add (uniform):
// the rows are added to what gout holds (requested ahead of the staging; one rounding).  Ends with a barrier.
template <int D, int GT>
__device__ __forceinline__ void store_rows(const f32x16 (&acc)[D / 32], float* Ol, uint16_t* gout, int64_t st, int tok0,
                                           int nt, int tid, int w, int l32, int hi, bool add = false) {
  using G = BwdCfg<D, GT>;
  constexpr int PPT = G::RP * (D / 8) / G::NT;
  static_assert(PPT * G::NT == G::RP * (D / 8), "whole pieces per thread");
#pragma unroll 1
  for (int pass = 0; pass < GT / G::RP; ++pass) {
    u32x4 held[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) held[i] = u32x4{0, 0, 0, 0};
    if (add) {
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const int e = tid + G::NT * i;
        const int r = G::RP * pass + e / (D / 8), c0 = 8 * (e % (D / 8));
        held[i] = *reinterpret_cast<const u32x4*>(gout + (int64_t)(tok0 + (r < nt ? r : nt - 1)) * st + c0);
      }
    }
    if ((32 * w) / G::RP == pass) {                          // uniform per wave
      float* orow = Ol + (32 * w + l32 - G::RP * pass) * G::OS + 4 * hi;
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<f32x4*>(orow + 32 * ct + 8 * g) = f32x4{acc[ct][4 * g], acc[ct][4 * g + 1], acc[ct][4 * g + 2], acc[ct][4 * g + 3]};
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int e = tid + G::NT * i;
      const int r = G::RP * pass + e / (D / 8), c0 = 8 * (e % (D / 8));
      if (r < nt) {
        const float* src = Ol + (r - G::RP * pass) * G::OS + c0;
        const f32x4 y0 = *reinterpret_cast<const f32x4*>(src), y1 = *reinterpret_cast<const f32x4*>(src + 4);
        const u32x4 h4 = held[i];
        *reinterpret_cast<u32x4*>(gout + (int64_t)(tok0 + r) * st + c0) =
            u32x4{pack_bf16x2(y0[0] + bf16_lo_to_f32(h4[0]), y0[1] + bf16_hi_to_f32(h4[0])),
                  pack_bf16x2(y0[2] + bf16_lo_to_f32(h4[1]), y0[3] + bf16_hi_to_f32(h4[1])),
                  pack_bf16x2(y1[0] + bf16_lo_to_f32(h4[2]), y1[1] + bf16_hi_to_f32(h4[2])),
                  pack_bf16x2(y1[2] + bf16_lo_to_f32(h4[3]), y1[3] + bf16_hi_to_f32(h4[3]))};
      }
    }
    __syncthreads();
  }
}

// a row of a tensor in the accumulator's column order: x[4g + j] = row[32 ft + 8g + 4hi + j]
__device__ __forceinline__ void row_in_acc_order(const uint16_t* row, int ft, int hi, float (&x)[16]) {
  u32x2 raw[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) raw[g] = *reinterpret_cast<const u32x2*>(row + 32 * ft + 8 * g + 4 * hi);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    x[4 * g] = bf16_lo_to_f32(raw[g][0]);
    x[4 * g + 1] = bf16_hi_to_f32(raw[g][0]);
    x[4 * g + 2] = bf16_lo_to_f32(raw[g][1]);
    x[4 * g + 3] = bf16_hi_to_f32(raw[g][1]);
  }
}

}  // namespace

// ---- dq and the per-token scalars ---------------------------------------------------------------------------------
template <int D, int GT>
__global__ __launch_bounds__(GT * 2) void grouped_bwd_dq_kernel(GroupedBwdArgs a) {
  using G = BwdCfg<D, GT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Kl = reinterpret_cast<uint16_t*>(smem + G::OFF_A);
  uint16_t* Vl = reinterpret_cast<uint16_t*>(smem + G::OFF_B);
  float* zl = reinterpret_cast<float*>(smem + G::OFF_Z);
  uint16_t* Sl = Kl;                                       // S_g as bf16, once the key rows are done with
  float* Ol = reinterpret_cast<float*>(smem);

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  const int g = blockIdx.x, bh = blockIdx.y;
  const int b = bh / a.H, h = bh % a.H;
  const int tok0 = g * GT;
  const int nt = (a.L - tok0) < GT ? (a.L - tok0) : GT;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  const uint16_t* gdo = static_cast<const uint16_t*>(a.dout) + base;
  uint16_t* gdq = static_cast<uint16_t*>(a.dq) + base;
  const float* slot = a.P + ((size_t)bh * a.ng + g) * G::SLOT;
  static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
  constexpr float inv_sqrt_d = D == 64 ? 0.125f : 0.08838834764831845f;
  constexpr float to_log2 = 1.44269504088896340736f * inv_sqrt_d;

  // Query tile j meets j + 1 key tiles.  Waves w and w + NW/2 share a SIMD: the tiles (w, NW - 1 - w) give every SIMD
  // the same number of key tiles.
  const int qtile = w < G::NW / 2 ? w : G::NW + G::NW / 2 - 1 - w;
  // this wave's queries and their incoming gradients, straight into MFMA operand registers: lane = query
  // 32 qtile + l32, registers = features / channels 16ks + 8hi + 0..7.  A query past the end reads the last row; it is
  // never stored.
  const int qt = 32 * qtile + l32;
  const int qrow = qt < nt ? qt : nt - 1;
  u32x4 qraw[G::KSD], draw[G::KSD];
  {
    const uint16_t* qp = gq + (int64_t)(tok0 + qrow) * a.st + 8 * hi;
    const uint16_t* dp = gdo + (int64_t)(tok0 + qrow) * a.st + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) {
      qraw[ks] = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
      draw[ks] = *reinterpret_cast<const u32x4*>(dp + 16 * ks);
    }
  }
  load_rows2<D, GT>(gk, gv, a.st, tok0, nt, Kl, Vl, tid);
  __syncthreads();

  auto scores = [&](int kt, f32x16& acc, f32x16& dpa) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = dpa[r] = 0.f;
    const uint16_t* ka = Kl + (32 * kt + l32) * G::KS + 8 * hi;
    const uint16_t* va = Vl + (32 * kt + l32) * G::KS + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) {
      acc = mfma(lds_row8(ka + 16 * ks), __builtin_bit_cast(bf16x8, qraw[ks]), acc);
      dpa = mfma(lds_row8(va + 16 * ks), __builtin_bit_cast(bf16x8, draw[ks]), dpa);
    }
  };

  // ---- pass 1: largest logit, sum of the weights and sum of e_i dp_i per query ---------------------------------
  float mtop = -INFINITY, mass = 0.f, racc = 0.f;
  for (int kt = 0; kt <= qtile; ++kt) {
    f32x16 acc, dpa;
    scores(kt, acc, dpa);
    // acc[r], dpa[r]: key 32kt + 8(r/4) + 4hi + r%4, query 32 qtile + l32; keys later than the query do not exist for it
    float top = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kl = 8 * (r >> 2) + 4 * hi + (r & 3);
      acc[r] = (kt < qtile || kl <= l32) ? acc[r] : -INFINITY;
      top = fmaxf(top, acc[r]);
    }
    top = fmaxf(top, __shfl_xor(top, 32));
    const float mnew = fmaxf(mtop, top);
    const float corr = __builtin_amdgcn_exp2f((mtop - mnew) * to_log2);
    const float shift = -mnew * to_log2;
    float rs = 0.f, rd = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float e = __builtin_amdgcn_exp2f(fmaf(acc[r], to_log2, shift));
      rs += e;
      rd = fmaf(e, dpa[r], rd);
    }
    mass = fmaf(mass, corr, rs);
    racc = fmaf(racc, corr, rd);
    mtop = mnew;
  }
  mass += __shfl_xor(mass, 32);
  racc += __shfl_xor(racc, 32);
  const float inv_mass = 1.f / mass;                       // the token itself is always seen: mass >= 1
  const float pbar = racc * inv_mass;
  const float mlog2 = mtop * to_log2;

  // ---- pass 2: ds = p (dp - pbar) / sqrt(d), dQ^T += K^T ds^T --------------------------------------------------
  // dqa[ft][r] = dQ[query 32 qtile + l32][feature 32ft + 8(r/4) + 4hi + r%4]
  f32x16 dqa[G::CT];
#pragma unroll
  for (int ft = 0; ft < G::CT; ++ft)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqa[ft][r] = 0.f;
  for (int kt = 0; kt <= qtile; ++kt) {
    f32x16 acc, dpa;
    scores(kt, acc, dpa);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kl = 8 * (r >> 2) + 4 * hi + (r & 3);
      // (the mask as a select on the exponent, exp2(-inf) = 0: a branch per element would cut the loop into pieces)
      const float arg = (kt < qtile || kl <= l32) ? fmaf(acc[r], to_log2, -mlog2) : -INFINITY;
      const float p = __builtin_amdgcn_exp2f(arg) * inv_mass;
      acc[r] = p * (dpa[r] - pbar) * inv_sqrt_d;
    }
    // ds enters as hi + lo (two bf16 terms): with one term its rounding, met by cancelling products, is the largest
    // error of dq; the matrix cores are idle most of the time here
    bf16x8 d0, d0l, d1, d1l;
    split8(acc, 0, d0, d0l);
    split8(acc, 8, d1, d1l);
#pragma unroll
    for (int ft = 0; ft < G::CT; ++ft) {
      const bf16x8 k0 = tr_operand_acc_order(Kl, G::KS, 32 * kt, 32 * ft, lane);
      const bf16x8 k1 = tr_operand_acc_order(Kl, G::KS, 32 * kt + 16, 32 * ft, lane);
      dqa[ft] = mfma(k0, d0, dqa[ft]);
      dqa[ft] = mfma(k0, d0l, dqa[ft]);
      dqa[ft] = mfma(k1, d1, dqa[ft]);
      dqa[ft] = mfma(k1, d1l, dqa[ft]);
    }
  }
  __syncthreads();                                         // every wave is done with the key and value rows

  // ---- the grouped branch: S_g -> LDS as bf16 [feature][channel], z_g -> LDS ------------------------------------
  load_slot<D, GT>(slot, Sl, zl, tid);
  __syncthreads();
  const uint16_t* qrow_p = gq + (int64_t)(tok0 + qrow) * a.st;
  // W[f][t] = sum_c S_g[f][c] dO[t][c], one 32-feature tile at a time; nd = phi(q).W first, then the tiles' own use
  auto w_tile = [&](int ft, f32x16& wt) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) wt[r] = 0.f;
    const uint16_t* sa = Sl + (32 * ft + l32) * G::SS + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) {
      wt = mfma(lds_row8(sa + 16 * ks), __builtin_bit_cast(bf16x8, draw[ks]), wt);
      wt = mfma(lds_row8(sa + D * G::SS + 16 * ks), __builtin_bit_cast(bf16x8, draw[ks]), wt);
    }
  };
  // den = phi(q).z + eps and nd = phi(q).W, both with phi(q) in fp32: f W and z dden nearly cancel, so neither may
  // carry the rounding of a bf16 phi(q)
  float nd = 0.f, dz = 0.f;
  f32x16 wt[G::CT];                                        // kept for the second use below (the raw q rows' registers are free)
#pragma unroll
  for (int ft = 0; ft < G::CT; ++ft) {
    w_tile(ft, wt[ft]);
    float qv[16];
    row_in_acc_order(qrow_p, ft, hi, qv);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float fqv = phi_f(qv[r], a.relu);
      nd = fmaf(fqv, wt[ft][r], nd);
      dz = fmaf(fqv, zl[32 * ft + 8 * (r >> 2) + 4 * hi + (r & 3)], dz);
    }
  }
  nd += __shfl_xor(nd, 32);
  dz += __shfl_xor(dz, 32);
  const float gden = dz + a.eps;
  const float fscale = gden != 0.f ? a.alpha / gden : 0.f; // nothing before the group: no branch
  const float dden = gden != 0.f ? -fscale * nd / gden : 0.f;
#pragma unroll
  for (int ft = 0; ft < G::CT; ++ft) {
    float qv[16];
    row_in_acc_order(qrow_p, ft, hi, qv);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int f = 32 * ft + 8 * (r >> 2) + 4 * hi + (r & 3);
      dqa[ft][r] = fmaf(fmaf(fscale, wt[ft][r], zl[f] * dden), dphi_f(qv[r], a.relu), dqa[ft][r]);
    }
  }
  // the per-token scalars for the kernels that follow
  if (hi == 0 && qt < nt) {
    const size_t n = (size_t)a.B * a.H * a.L, e = (size_t)bh * a.L + tok0 + qt;
    a.stats[e] = mlog2;
    a.stats[n + e] = inv_mass;
    a.stats[2 * n + e] = pbar;
    a.stats[3 * n + e] = fscale;
    a.stats[4 * n + e] = dden;
  }
  __syncthreads();                                         // every wave is done with the state operand
  store_rows<D, GT>(dqa, Ol, gdq, a.st, tok0, nt, tid, qtile, l32, hi);
}

// ---- what the queries of a group add to the gradient of the sums before it; and those sums themselves -----------------
// SUMS: the same contraction over a group's tokens with (K, V) in the place of (Q, dO) and weights of one: the group's
// own phi(K)^T V and sum of phi(K), written to the slot of the group after it (the prefix sum follows).  The forward's
// first pass is not used for this: it rounds phi(k) to one bf16, and with keys of the size 1/sqrt(d) most of what the
// keys say sits below that rounding, while the gradient of the grouped branch is a difference that lives on it.
template <int D, int GT, bool SUMS>
__global__ __launch_bounds__(GT * 2) void grouped_bwd_gs_kernel(GroupedBwdArgs a) {
  using G = BwdCfg<D, GT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ql = reinterpret_cast<uint16_t*>(smem + G::OFF_A);
  uint16_t* Dl = reinterpret_cast<uint16_t*>(smem + G::OFF_B);
  float* fs = reinterpret_cast<float*>(smem + G::OFF_ST);  // alpha / den per token
  float* dd = fs + GT;                                     // d den per token
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  // gradients: groups 1 .. ng-1 (group 0 has nothing before it); sums: groups 0 .. ng-2 (nothing follows the last)
  const int g = SUMS ? blockIdx.x : blockIdx.x + 1, bh = blockIdx.y;
  const int b = bh / a.H, h = bh % a.H;
  const int tok0 = g * GT;
  const int nt = (a.L - tok0) < GT ? (a.L - tok0) : GT;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(SUMS ? a.k : a.q) + base;
  const uint16_t* gdo = static_cast<const uint16_t*>(SUMS ? a.v : a.dout) + base;
  float* slot = SUMS ? a.P + ((size_t)bh * a.ng + g + 1) * G::SLOT : a.Dg + ((size_t)bh * a.ng + g) * G::SLOT;
  const size_t n = (size_t)a.B * a.H * a.L, e0 = (size_t)bh * a.L + tok0;

  float f3 = 0.f, d4 = 0.f;
  if (tid < GT && tid < nt) {
    if (SUMS) f3 = d4 = 1.f;
    else { f3 = a.stats[3 * n + e0 + tid]; d4 = a.stats[4 * n + e0 + tid]; }
  }
  load_rows2<D, GT>(gq, gdo, a.st, tok0, nt, Ql, Dl, tid);
  if (tid < GT) { fs[tid] = f3; dd[tid] = d4; }
  __syncthreads();
  // gz[f] = sum_t phi(q_t[f]) dden_t: thread = (feature, one of NT / D runs of tokens), eight independent terms in
  // flight (one by one, every term would wait for its own LDS reads and exponential), the runs added up through LDS
  {
    constexpr int NP = G::NT / D, TPP = GT / NP;           // runs per feature, tokens per run
    float* zp = reinterpret_cast<float*>(smem + G::OFF_RED);   // [NP][D]
    const int f = tid % D, part = tid / D;
    float gz = 0.f;
#pragma unroll 8
    for (int i = 0; i < TPP; ++i) {
      const int t = part * TPP + i;                        // rows past the end are zero rows with weight 0
      gz = fmaf(phi_f(bf16_bits_to_f32(Ql[t * G::KS + f]), a.relu), dd[t], gz);
    }
    zp[part * D + f] = gz;
  }
  __syncthreads();
  if (tid < D) {
    const float* zp = reinterpret_cast<const float*>(smem + G::OFF_RED);
    float gz = 0.f;
#pragma unroll
    for (int p = 0; p < G::NT / D; ++p) gz += zp[p * D + tid];
    slot[D * D + tid] = gz;
  }
  // the tiles (feature block ib, channel block cb) over the waves; lanes = channels, registers = features.  The
  // operand (alpha / den_t) phi(q_t) is made from the raw rows as they are read (lane = feature, registers = tokens
  // 16ks + 8hi + 0..7) and enters as hi + lo: D.S v + D.z is again a difference of nearly equal parts.
  // A wave takes a feature block and CBG channel blocks at a time, so that the operand made above serves several tiles.
  constexpr int CBG = (G::CT * G::CT / G::NW) < 1 ? 1 : ((G::CT * G::CT / G::NW) > G::CT ? G::CT : (G::CT * G::CT / G::NW));
  constexpr int UPB = G::CT / CBG;                         // units per feature block
#pragma unroll 1
  for (int unit = w; unit < G::CT * UPB; unit += G::NW) {
    const int ib = unit / UPB, cb0 = (unit % UPB) * CBG;
    f32x16 sacc[CBG];
#pragma unroll
    for (int j = 0; j < CBG; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[j][r] = 0.f;
    for (int ks = 0; ks < GT / 16; ++ks) {
      const u32x4 raw = __builtin_bit_cast(u32x4, tr_operand(Ql, G::KS, 16 * ks, 32 * ib, lane));
      const float* fsp = fs + 16 * ks + 8 * hi;            // 0 for rows past the end
      u32x4 ah, al;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float x0 = fsp[2 * i] * phi_f(bf16_lo_to_f32(raw[i]), a.relu);
        const float x1 = fsp[2 * i + 1] * phi_f(bf16_hi_to_f32(raw[i]), a.relu);
        ah[i] = pack_bf16x2(x0, x1);
        al[i] = pack_bf16x2(x0 - bf16_lo_to_f32(ah[i]), x1 - bf16_hi_to_f32(ah[i]));
      }
#pragma unroll
      for (int j = 0; j < CBG; ++j) {
        const bf16x8 dop = tr_operand(Dl, G::KS, 16 * ks, 32 * (cb0 + j), lane);
        sacc[j] = mfma(__builtin_bit_cast(bf16x8, ah), dop, sacc[j]);
        sacc[j] = mfma(__builtin_bit_cast(bf16x8, al), dop, sacc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < CBG; ++j) {
      float* so = slot + (32 * ib + 4 * hi) * D + 32 * (cb0 + j) + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) so[(8 * (r >> 2) + (r & 3)) * D] = sacc[j][r];
    }
  }
}

// ---- D_g = sum over the later groups of what their queries added, in place (one thread per element) ----------------
__global__ __launch_bounds__(256) void grouped_bwd_suffix_kernel(GroupedBwdArgs a, int slot_elems) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= slot_elems) return;
  float* ws = a.Dg + (size_t)blockIdx.y * a.ng * slot_elems + e;
  float run = 0.f;
  // sixteen groups at a time, every request before the first store; slot 0 was never written and is not read
  for (int g1 = a.ng - 1; g1 >= 0; g1 -= 16) {
    float inc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int g = g1 - i;
      inc[i] = ws[(size_t)(g >= 1 ? g : 1) * slot_elems];     // (launched for two groups or more: slot 1 exists)
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int g = g1 - i;
      if (g >= 0) ws[(size_t)g * slot_elems] = run;
      if (g >= 1) run += inc[i];
    }
  }
}

// ---- dk, dv ---------------------------------------------------------------------------------------------------------
template <int D, int GT>
__global__ __launch_bounds__(GT * 2) void grouped_bwd_dkdv_kernel(GroupedBwdArgs a) {
  using G = BwdCfg<D, GT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ql = reinterpret_cast<uint16_t*>(smem + G::OFF_A);
  uint16_t* Dl = reinterpret_cast<uint16_t*>(smem + G::OFF_B);
  float* zl = reinterpret_cast<float*>(smem + G::OFF_Z);
  float* ml = reinterpret_cast<float*>(smem + G::OFF_ST);  // largest logit (log2 units), 1 / sum, pbar per query
  float* il = ml + GT;
  float* pl = il + GT;
  uint16_t* Sl = Ql;                                       // D_g as bf16, once the token rows are done with
  float* Ol = reinterpret_cast<float*>(smem);

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  // The two workgroups of a group (0: dv, 1: dk) read the same Q and dO rows: they get block indices 8 apart, which
  // the dispatcher places on the same chiplet, so that the second of them finds the rows in that chiplet's L2 (blocks
  // 0..7 = groups 0..7 for dv, 8..15 = the same groups for dk, and so on; a remainder of fewer than 8 groups alternates).
  const int full = (a.ng >> 3) << 3, bx = blockIdx.x;
  const int role = bx < 2 * full ? (bx >> 3) & 1 : (bx - 2 * full) & 1;
  const int g = bx < 2 * full ? ((bx >> 4) << 3) | (bx & 7) : full + ((bx - 2 * full) >> 1);
  const int bh = blockIdx.y;
  const int b = bh / a.H, h = bh % a.H;
  const int tok0 = g * GT;
  const int nt = (a.L - tok0) < GT ? (a.L - tok0) : GT;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  const uint16_t* gdo = static_cast<const uint16_t*>(a.dout) + base;
  uint16_t* gout = static_cast<uint16_t*>(role ? a.dk : a.dv) + base;
  const float* slot = a.Dg + ((size_t)bh * a.ng + g) * G::SLOT;
  const size_t n = (size_t)a.B * a.H * a.L, e0 = (size_t)bh * a.L + tok0;
  constexpr float inv_sqrt_d = D == 64 ? 0.125f : 0.08838834764831845f;
  constexpr float to_log2 = 1.44269504088896340736f * inv_sqrt_d;

  // this wave's keys (and their values) as MFMA operands: lane = key 32 ktile + l32, registers = features 16ks + 8hi + 0..7
  // key tile j meets the query tiles j .. NW - 1: mirrored over the waves as in the query-side kernel
  const int ktile = w < G::NW / 2 ? w : G::NW + G::NW / 2 - 1 - w;
  const int kt_own = 32 * ktile + l32;
  const int krow = kt_own < nt ? kt_own : nt - 1;
  u32x4 kop[G::KSD], vop[G::KSD];
  {
    const uint16_t* kp = gk + (int64_t)(tok0 + krow) * a.st + 8 * hi;
    const uint16_t* vp = gv + (int64_t)(tok0 + krow) * a.st + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) {
      kop[ks] = *reinterpret_cast<const u32x4*>(kp + 16 * ks);
      vop[ks] = *reinterpret_cast<const u32x4*>(vp + 16 * ks);
    }
  }
  float s0 = 0.f, s1 = 0.f, s2 = 0.f;                      // queries past the end weigh nothing
  if (tid < GT && tid < nt) { s0 = a.stats[e0 + tid]; s1 = a.stats[n + e0 + tid]; s2 = a.stats[2 * n + e0 + tid]; }
  load_rows2<D, GT>(gq, gdo, a.st, tok0, nt, Ql, Dl, tid);
  if (tid < GT) { ml[tid] = s0; il[tid] = s1; pl[tid] = s2; }
  __syncthreads();

  // acc4[ct][r] = dV or dK [key 32 ktile + l32][column 32ct + 8(r/4) + 4hi + r%4]
  f32x16 acc4[G::CT];
#pragma unroll
  for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc4[ct][r] = 0.f;
  const int nqt = (nt + 31) / 32;
  for (int qt = ktile; qt < nqt; ++qt) {
    // sc[r]: query 32qt + 8(r/4) + 4hi + r%4 (registers), key 32 ktile + l32 (lane)
    f32x16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
    const uint16_t* qa = Ql + (32 * qt + l32) * G::KS + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) sc = mfma(lds_row8(qa + 16 * ks), __builtin_bit_cast(bf16x8, kop[ks]), sc);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int tl = 8 * (r >> 2) + 4 * hi + (r & 3);
      const int t = 32 * qt + tl;
      // (the scalars are read whatever the mask says: a read under the condition would make it a branch per element)
      const float mt = ml[t], it = il[t];
      const float x = fmaf(sc[r], to_log2, -mt);
      sc[r] = __builtin_amdgcn_exp2f((qt > ktile || tl >= l32) ? x : -INFINITY) * it;
    }
    if (role == 0) {                                       // dV^T += dO^T P
      bf16x8 p0, p0l, p1, p1l;                             // the weights as hi + lo too
      split8(sc, 0, p0, p0l);
      split8(sc, 8, p1, p1l);
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct) {
        const bf16x8 g0 = tr_operand_acc_order(Dl, G::KS, 32 * qt, 32 * ct, lane);
        const bf16x8 g1 = tr_operand_acc_order(Dl, G::KS, 32 * qt + 16, 32 * ct, lane);
        acc4[ct] = mfma(g0, p0, acc4[ct]);
        acc4[ct] = mfma(g0, p0l, acc4[ct]);
        acc4[ct] = mfma(g1, p1, acc4[ct]);
        acc4[ct] = mfma(g1, p1l, acc4[ct]);
      }
    } else {                                               // dK^T += Q^T ds,  ds = p (dp - pbar) / sqrt(d)
      f32x16 dpa;
#pragma unroll
      for (int r = 0; r < 16; ++r) dpa[r] = 0.f;
      const uint16_t* da = Dl + (32 * qt + l32) * G::KS + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < G::KSD; ++ks) dpa = mfma(lds_row8(da + 16 * ks), __builtin_bit_cast(bf16x8, vop[ks]), dpa);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = 32 * qt + 8 * (r >> 2) + 4 * hi + (r & 3);
        sc[r] = sc[r] * (dpa[r] - pl[t]) * inv_sqrt_d;
      }
      bf16x8 d0, d0l, d1, d1l;                             // hi + lo, as in the dq kernel
      split8(sc, 0, d0, d0l);
      split8(sc, 8, d1, d1l);
#pragma unroll
      for (int ft = 0; ft < G::CT; ++ft) {
        const bf16x8 q0 = tr_operand_acc_order(Ql, G::KS, 32 * qt, 32 * ft, lane);
        const bf16x8 q1 = tr_operand_acc_order(Ql, G::KS, 32 * qt + 16, 32 * ft, lane);
        acc4[ft] = mfma(q0, d0, acc4[ft]);
        acc4[ft] = mfma(q0, d0l, acc4[ft]);
        acc4[ft] = mfma(q1, d1, acc4[ft]);
        acc4[ft] = mfma(q1, d1l, acc4[ft]);
      }
    }
  }
  __syncthreads();                                         // every wave is done with the query and gradient rows

  // ---- the group's keys and values entered the sums every later group read ---------------------------------------
  if (g + 1 < a.ng) {                                      // uniform; after the last group nothing reads the sums
    load_slot<D, GT>(slot, Sl, zl, tid);
    __syncthreads();
    if (role == 0) {                                       // dV^T += D.S^T phi(K)^T
      bf16x8 fko[G::KSD];
#pragma unroll
      for (int ks = 0; ks < G::KSD; ++ks) fko[ks] = __builtin_bit_cast(bf16x8, phi_pack8(kop[ks], a.relu));
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct) {
        f32x16 lin;
#pragma unroll
        for (int r = 0; r < 16; ++r) lin[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < G::KSD; ++ks) {
          lin = mfma(tr_operand(Sl, G::SS, 16 * ks, 32 * ct, lane), fko[ks], lin);
          lin = mfma(tr_operand(Sl + D * G::SS, G::SS, 16 * ks, 32 * ct, lane), fko[ks], lin);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc4[ct][r] += lin[r];
      }
    } else {                                               // dK += (D.S V^T + D.z) * phi'(K)
      const uint16_t* krow_p = gk + (int64_t)(tok0 + krow) * a.st;
#pragma unroll
      for (int ft = 0; ft < G::CT; ++ft) {
        f32x16 lin;
#pragma unroll
        for (int r = 0; r < 16; ++r) lin[r] = 0.f;
        const uint16_t* sa = Sl + (32 * ft + l32) * G::SS + 8 * hi;
#pragma unroll
        for (int ks = 0; ks < G::KSD; ++ks) {
          lin = mfma(lds_row8(sa + 16 * ks), __builtin_bit_cast(bf16x8, vop[ks]), lin);
          lin = mfma(lds_row8(sa + D * G::SS + 16 * ks), __builtin_bit_cast(bf16x8, vop[ks]), lin);
        }
        float kv[16];
        row_in_acc_order(krow_p, ft, hi, kv);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int f = 32 * ft + 8 * (r >> 2) + 4 * hi + (r & 3);
          acc4[ft][r] = fmaf(lin[r] + zl[f], dphi_f(kv[r], a.relu), acc4[ft][r]);
        }
      }
    }
    __syncthreads();                                       // every wave is done with the d x d operand
  }
  // dv is added to what the conv's share left there (written ahead of this kernel); dk is written
  store_rows<D, GT>(acc4, Ol, gout, a.st, tok0, nt, tid, ktile, l32, hi, role == 0);
}

// ---- dw: per workgroup the products of its tokens, then one sum over batch rows and token blocks --------------------
// dw[h][c][j] = sum_b sum_t dO[b,h,t,c] v[b,h,t-j,c].  One workgroup = DW_TOK tokens of one (b, h); a thread owns one
// channel and a quarter (d = 64) or half (d = 128) of the tokens, holds the sums of all taps in registers and walks its
// tokens sixteen at a time.  Both factors are bf16, so two products per instruction come for free: the gradients of
// tokens (t, t+1) and the values of tokens (s, s+1), each pair in one register, meet in one v_dot2 (exact products,
// fp32 sum) and both products belong to tap t - s.  The value pairs of all alignments are made on the way: every
// value read from LDS joins the one read before it.  (The loops are straight-line code for the tap capacity of the
// instantiation, as in the forward long conv.)
namespace {
constexpr int DW_TOK = 128;
constexpr int DW_HALO = 62;
constexpr int DW_BLK = 16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
}  // namespace

template <int D, int KMAX>
__global__ __launch_bounds__(256) void grouped_bwd_dw_kernel(GroupedBwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dw_smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(dw_smem);     // [DW_HALO + DW_TOK][D] value rows (bf16) ...
  float* red = reinterpret_cast<float*>(dw_smem);          // ... then [NG - 1][D][KMAX] sums
  constexpr int NG = 256 / D, TPT = DW_TOK / NG;
  static_assert(TPT % DW_BLK == 0, "whole blocks of gradients per thread");
  const int tid = threadIdx.x;
  const int bh = blockIdx.y, b = bh / a.H, h = bh % a.H;
  // (neighbouring token blocks share 62 value rows: block indices 8 apart, which land on the same chiplet, get
  // neighbouring token blocks when the count is a multiple of 8)
  const int nblk = gridDim.x;
  const int tblk = nblk % 8 == 0 ? (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3) : (int)blockIdx.x;
  const int t0 = tblk * DW_TOK;
  const int L = a.L, Kc = a.Kc;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  const uint16_t* gdo = static_cast<const uint16_t*>(a.dout) + base;
  const int c = tid % D, tg = tid / D;
  // this thread's gradients (a token past the end: zero), two tokens per register, and the value rows
  // t0 - 62 .. t0 + DW_TOK - 1, all requested first
  uint32_t gp[TPT / 2];
  {
    uint16_t go_raw[TPT];
#pragma unroll
    for (int e = 0; e < TPT; ++e) {
      const int tok = t0 + tg * TPT + e;
      go_raw[e] = gdo[(int64_t)(tok < L ? tok : L - 1) * a.st + c];
    }
    constexpr int RIT = ((DW_HALO + DW_TOK) * (D / 8) + 255) / 256;
    u32x4 raw[RIT];
#pragma unroll
    for (int i = 0; i < RIT; ++i) {
      const int e = tid + 256 * i;
      const int row = e / (D / 8), i0 = 8 * (e % (D / 8));
      const int tok = t0 - DW_HALO + row;
      raw[i] = *reinterpret_cast<const u32x4*>(gv + (int64_t)((tok >= 0 && tok < L) ? tok : 0) * a.st + i0);
    }
#pragma unroll
    for (int i = 0; i < RIT; ++i) {
      const int e = tid + 256 * i;
      const int row = e / (D / 8), i0 = 8 * (e % (D / 8));
      const int tok = t0 - DW_HALO + row;
      if (e < (DW_HALO + DW_TOK) * (D / 8))
        *reinterpret_cast<u32x4*>(xs + row * D + i0) = (tok >= 0 && tok < L) ? raw[i] : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int e = 0; e < TPT; e += 2) {
      const int tok = t0 + tg * TPT + e;
      const uint32_t lo = tok < L ? go_raw[e] : 0u, hi = tok + 1 < L ? go_raw[e + 1] : 0u;
      gp[e / 2] = lo | (hi << 16);
    }
  }
  __syncthreads();
  float acc[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) acc[j] = 0.f;
#pragma unroll 1
  for (int blk = 0; blk < TPT / DW_BLK; ++blk) {
    const int tb0 = tg * TPT + blk * DW_BLK;
    // value rows from the block's newest token backwards: x(m) = v[newest - m].  The pair (x(m), x(m-1)) = tokens
    // (s, s+1) meets the gradients of tokens (tb0 + e, tb0 + e + 1), e even, through tap e - (DW_BLK - 1) + m.
    const uint16_t* newest = xs + (DW_HALO + tb0 + DW_BLK - 1) * D + c;
    uint32_t newer = newest[0];
#pragma unroll
    for (int m = 1; m < KMAX + DW_BLK - 1; ++m) {
      const uint32_t x = newest[-m * D];
      const uint32_t pair = x | (newer << 16);
      newer = x;
#pragma unroll
      for (int e = 0; e < DW_BLK; e += 2) {
        const int j = e - (DW_BLK - 1) + m;
        if (j >= 0 && j < KMAX) acc[j] = dot2_bf16(gp[e / 2], pair, acc[j]);
      }
    }
#pragma unroll
    for (int e = 0; e + DW_BLK / 2 < TPT / 2; ++e) gp[e] = gp[e + DW_BLK / 2];
  }
  // the token groups of threads add up through LDS (fixed order), then one row of partial sums per workgroup
  __syncthreads();
  if (tg > 0) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) red[((tg - 1) * D + c) * KMAX + j] = acc[j];
  }
  __syncthreads();
  if (tg == 0) {
#pragma unroll
    for (int q = 0; q < NG - 1; ++q)
#pragma unroll
      for (int j = 0; j < KMAX; ++j) acc[j] += red[(q * D + c) * KMAX + j];
  }
  __syncthreads();
  if (tg == 0) {
#pragma unroll
    for (int j = 0; j < KMAX; ++j) red[c * KMAX + j] = acc[j];
  }
  __syncthreads();
  // partial sums of a head lie together: [H][B * nwb][D * Kc]
  float* part = a.dw_part + (((size_t)h * a.B + b) * a.nwb + tblk) * D * Kc;
  for (int e = tid; e < D * Kc; e += 256) part[e] = red[(e / Kc) * KMAX + e % Kc];
}

// Sums over batch rows and token blocks in a fixed order, DW_RED partial sums at a time: in [H][n][per_head] ->
// out [H][ceil(n / DW_RED)][per_head]; the last stage writes dconv_w (n = 0: zeros).
namespace { constexpr int DW_RED = 32; }
__global__ __launch_bounds__(256) void grouped_bwd_dw_reduce_kernel(const float* in, float* out, int n, int per_head) {
  const int e = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y, c = blockIdx.z;
  if (e >= per_head) return;
  const int nout = (n + DW_RED - 1) / DW_RED;
  const int i0 = c * DW_RED, i1 = (i0 + DW_RED) < n ? (i0 + DW_RED) : n;
  const float* p = in + ((size_t)h * n + i0) * per_head + e;
  float s = 0.f;
#pragma unroll 8
  for (int i = i0; i < i1; ++i, p += per_head) s += *p;
  out[((size_t)h * (nout > 0 ? nout : 1) + c) * per_head + e] = s;
}

int grouped_bwd_dw_blocks(int L) { return (L + DW_TOK - 1) / DW_TOK; }

template <int D, int GT>
static hipError_t launch_bwd_core(const GroupedBwdArgs& a, hipStream_t st, hipEvent_t before_dkdv) {
  using G = BwdCfg<D, GT>;
  const int BH = a.B * a.H;
  hipError_t e;
  auto kq = grouped_bwd_dq_kernel<D, GT>;
  auto kg = grouped_bwd_gs_kernel<D, GT, false>;
  auto ks = grouped_bwd_gs_kernel<D, GT, true>;
  auto kk = grouped_bwd_dkdv_kernel<D, GT>;
  if ((e = LINATTN_MAX_LDS_ONCE(kq, G::TOTAL)) != hipSuccess) return e;
  if ((e = LINATTN_MAX_LDS_ONCE(kg, G::TOTAL)) != hipSuccess) return e;
  if ((e = LINATTN_MAX_LDS_ONCE(kk, G::TOTAL)) != hipSuccess) return e;
  if ((e = LINATTN_MAX_LDS_ONCE(ks, G::TOTAL)) != hipSuccess) return e;
  // the sums before every group: every group's own sums, then the prefix sum (which also writes the zeros before group 0)
  if (a.ng > 1) {
    hipLaunchKernelGGL(ks, dim3((unsigned)(a.ng - 1), (unsigned)BH), dim3(G::NT), G::TOTAL, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    PrefillArgs f{};
    f.ws = a.P; f.B = a.B; f.H = a.H; f.m = 1; f.nseg = a.ng;
    if ((e = launch_segment_scan(f, D, st)) != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kq, dim3((unsigned)a.ng, (unsigned)BH), dim3(G::NT), G::TOTAL, st, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (a.ng > 1) {
    hipLaunchKernelGGL(kg, dim3((unsigned)(a.ng - 1), (unsigned)BH), dim3(G::NT), G::TOTAL, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(grouped_bwd_suffix_kernel, dim3((unsigned)((G::SLOT + 255) / 256), (unsigned)BH), dim3(256), 0, st, a, (int)G::SLOT);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (before_dkdv && (e = hipStreamWaitEvent(st, before_dkdv, 0)) != hipSuccess) return e;
  hipLaunchKernelGGL(kk, dim3((unsigned)(2 * a.ng), (unsigned)BH), dim3(G::NT), G::TOTAL, st, a);
  return hipGetLastError();
}

template <int D, int KMAX>
static hipError_t launch_bwd_dw(const GroupedBwdArgs& a, hipStream_t st) {
  constexpr int LDS_ROWS = (DW_HALO + DW_TOK) * D * (int)sizeof(uint16_t);
  constexpr int LDS_RED = (256 / D > 2 ? 256 / D - 1 : 1) * D * KMAX * (int)sizeof(float);
  constexpr int LDS = LDS_ROWS > LDS_RED ? LDS_ROWS : LDS_RED;
  auto kern = grouped_bwd_dw_kernel<D, KMAX>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, LDS);
  if (e != hipSuccess) return e;
  if (a.nwb > 0) hipLaunchKernelGGL(kern, dim3((unsigned)a.nwb, (unsigned)(a.B * a.H)), dim3(256), LDS, st, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int per_head = D * a.Kc;
  // stages of 32: the partial sums ping-pong between the two halves of the buffer until one row per head is left
  const float* in = a.dw_part;
  float* other = a.dw_part + (size_t)a.B * a.H * (a.nwb > 0 ? a.nwb : 1) * per_head;
  int n = a.B * a.nwb;
  for (;;) {
    const int nout = (n + DW_RED - 1) / DW_RED;
    float* out = nout <= 1 ? a.dconv_w : other;
    hipLaunchKernelGGL(grouped_bwd_dw_reduce_kernel, dim3((unsigned)((per_head + 255) / 256), (unsigned)a.H, (unsigned)(nout > 0 ? nout : 1)),
                       dim3(256), 0, st, in, out, n, per_head);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (nout <= 1) break;
    other = const_cast<float*>(in);
    in = out;
    n = nout;
  }
  return hipSuccess;
}

// Everything but the conv-weight sums, in order.
hipError_t launch_grouped_bwd_core(const GroupedBwdArgs& a, int d, hipStream_t st, hipEvent_t before_dkdv) {
  if (a.L <= 0) return hipSuccess;
  if (d == 128) return a.group == 256 ? launch_bwd_core<128, 256>(a, st, before_dkdv) : launch_bwd_core<128, 64>(a, st, before_dkdv);
  return a.group == 256 ? launch_bwd_core<64, 256>(a, st, before_dkdv) : launch_bwd_core<64, 64>(a, st, before_dkdv);
}

// The conv-weight sums (no tokens: zeros).
hipError_t launch_grouped_bwd_dw(const GroupedBwdArgs& a, int d, hipStream_t st) {
  if (!a.dconv_w) return hipSuccess;
  if (d == 128) return a.Kc <= 16 ? launch_bwd_dw<128, 16>(a, st) : a.Kc <= 32 ? launch_bwd_dw<128, 32>(a, st) : launch_bwd_dw<128, 63>(a, st);
  return a.Kc <= 16 ? launch_bwd_dw<64, 16>(a, st) : a.Kc <= 32 ? launch_bwd_dw<64, 32>(a, st) : launch_bwd_dw<64, 63>(a, st);
}

}  // namespace linattn
