// Generation with the three-branch form (Sec. 4.1 block in the decode phase of Sec. 3; with k > 1 the
// verification step of Sec. 4.2): k draft tokens of one (b, h) are scored from one state, which is
//   S, z        sums of phi(k) v^T and phi(k) over the COMPLETED groups of 64 tokens (fp32),
//   hist        the last Kc-1 value rows (conv),
//   kwin, vwin  the raw key / value rows of the open group, rows 0 .. fill[b][h]-1 in use.
// Draft j sits at position P = fill + j of the open group.  Its output is
//   alpha * phi(q)^T S / (phi(q).z + eps)  +  softmax over the group's rows 0..P of q.k/sqrt(d), times V  +  conv.
// A draft beyond the end of the group (P >= 64) belongs to the next group: its local branch starts at
// row 64 and its linear branch sees the group that has just been completed, which is added in the
// quadratic form (weights phi(q).phi(k_r) on the value rows r < 64) instead of forming S + that group.
// Memory-bound on the read of S (64 KB per head at d = 128); S is only written when the kept drafts
// complete the group (once in 64 tokens), so a step moves about half the bytes of the token-level form.
//
// One workgroup of 256 threads per (b, h), fp32 arithmetic on the vector ALUs throughout:
//   1. logits: one wave per row of (window ++ drafts), lanes over features, wave reduction;
//   2. per draft: softmax over its rows, the linear normaliser, one weight per row in LDS;
//   3. the state streams through registers once (16-byte nontemporal loads, a few row passes in
//      flight) for the read-outs phi(q_j)^T S; the value rows are combined with the weights;
//   4. outputs; 5. the kept drafts join the window, or complete the group and enter S and z.
// The count of rows in use is kept per head ([B,H], equal over the heads of a batch row), so that every
// workgroup owns the one it reads and advances.
#include "common.h"
#include "kernels.h"

namespace linattn {

namespace {

constexpr int GC = 64;         // tokens per group
constexpr int GROWS = GC + 16; // rows of (window ++ drafts) at most (63 + 16), rounded up

template <int D, int KP>
struct VgScore {
  float rq[KP][D];            // q_j as it came
  float fq[D][KP];            // phi(q_j), feature-major: one thread reads all drafts of its state row
  float red[KP][D];           // phi(q_j)^T S
  float loc[KP][D];           // sum_r W[j][r] v_r
};
template <int D>
struct VgStage {              // completion of a group: 16 rows of phi(k) and of v at a time
  float k[16][D];
  float v[16][D];
};
template <int D, int KP>
struct VgSmem {
  union {                     // the completion runs when the outputs are done
    VgScore<D, KP> sc;
    VgStage<D> st;
  };
  float W[KP][GROWS];         // first the logits, then the weight of value row r in the output of draft j
  float lin[KP][GC];          // phi(q_j).phi(k_r) for the rows of the group being completed
  float vv[KP][D];            // v_j (conv)
  float fscale[KP];           // alpha / (phi(q_j).z [+ completed group] + eps), 0 if that denominator is 0
  float zz[D];
  float wt[8][D];             // conv taps, tap-major (taps >= Kc are 0)
  float hh[8][D];             // hh[t]: the value row t+1 positions before the first draft
};

// x[l] + x[l ^ 8] (rotation by 8 inside a row of 16)
__device__ __forceinline__ float add_xor8(float x) { return dpp_add<0x128>(x); }
// x[l] + x[l ^ 16]: rows 0,1 and rows 2,3 of the wave are swapped against each other
__device__ __forceinline__ float add_xor16(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// x[l] + x[l ^ 32]
__device__ __forceinline__ float add_xor32(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// x[l] + x[l ^ off] for the strides that occur here
template <int OFF>
__device__ __forceinline__ float add_xor(float x) {
  static_assert(OFF == 8 || OFF == 16 || OFF == 32, "stride");
  return OFF == 8 ? add_xor8(x) : OFF == 16 ? add_xor16(x) : add_xor32(x);
}

__device__ __forceinline__ const void* row_of(const void* win, const void* drafts, int64_t win0, int64_t tok0, int D, int n, int r,
                                              int64_t* idx) {
  // virtual row r of (window ++ drafts): which array, and the element index of its first element
  if (r < n) { *idx = win0 + (int64_t)r * D; return win; }
  *idx = tok0 + (int64_t)(r - n) * D;
  return drafts;
}

}  // namespace

// At most 128 registers per thread for up to 8 bf16 drafts: four workgroups per compute unit, so that 1024
// heads are all resident at once.
template <typename Io, int D, int KP>
__global__ __launch_bounds__(256, (sizeof(typename Io::elem) != 2 ? 2 : KP <= 8 ? 4 : 2)) void verify_grouped_kernel(VerifyGroupedArgs a) {
  constexpr int CG = D / 4;          // float4 column groups per state row
  constexpr int RPP = 256 / CG;      // state rows per pass
  constexpr int NPASS = D / RPP;
  constexpr int EPL = D / 64;        // features per lane where a wave walks a feature vector
  __shared__ VgSmem<D, KP> sm;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int bh = blockIdx.x;
  const int b = bh / a.H, h = bh % a.H;
  const int kk = a.kk, Kc = a.Kc;
  const int cg = tid % CG, r0 = tid / CG;

  const int64_t tok0 = (int64_t)bh * kk * D;
  const int64_t win0 = (int64_t)bh * GC * D;
  const int64_t hist0 = (int64_t)bh * (Kc - 1) * D;

  // ---- 0. every request of the step is issued before anything waits: the small inputs first (they are
  //         needed first), then this thread's rows of the open group and of the drafts, then the first passes
  //         of the state.  All of them unconditional (indices past the end are clamped, the data not used),
  //         so that nothing serialises on a round trip to memory.  The count of rows in use is itself a trip to
  //         memory that the rows' addresses have to wait for: whatever does not need it -- the small inputs and the
  //         first passes of the state -- is requested ahead of that wait (behind it, every workgroup of the launch
  //         spent its first microseconds with nothing requested). ----
  constexpr int CG8 = D / 8;                       // 8-feature pieces per row
  constexpr int NPART = 256 / CG8;                 // row partitions
  constexpr int RT = (GROWS + NPART - 1) / NPART;  // rows per thread
  const int c8 = tid % CG8, part = tid / CG8;
  // drafts: at most one 8-element piece of q and of v per thread (KP * D / 8 <= 256 pieces)
  const int pj = tid / CG8;                        // draft of this thread's piece (== part)
  const int64_t piece = tok0 + (int64_t)(pj < kk ? pj : kk - 1) * D + 8 * c8;
  const typename Io::raw8 q_raw = Io::load_raw8(a.q, piece);
  const typename Io::raw8 v_raw = Io::load_raw8(a.v, piece);
  const float z_reg = a.z[(size_t)bh * D + (tid < D ? tid : 0)];
  constexpr int TAP_IT = 8 * D / 256;
  float tap_reg[TAP_IT], hist_reg[TAP_IT];
  // (one tap: no history; the request then reads a draft's value row, which is dropped.  As `Kc > 1 ? load : 0` every
  // one of these requests sat in a branch of its own with a full wait behind it: four trips to memory in a row ahead
  // of the state's requests)
  const void* hsrc = Kc > 1 ? a.hist : a.v;
  const int64_t hbase = Kc > 1 ? hist0 : tok0;
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + 256 * mth;
    const int t = e / D, cc = e % D;
    tap_reg[mth] = a.conv_w[((size_t)h * D + cc) * Kc + (t < Kc ? t : 0)];
    hist_reg[mth] = Io::load1(hsrc, hbase + (int64_t)(t < Kc - 1 ? Kc - 2 - t : 0) * D + cc);
  }
  constexpr int PDW = KP <= 1 ? 8 : 4;             // row passes in flight (more when the read-outs leave registers free)
  constexpr int PD = NPASS < PDW ? NPASS : PDW;
  const float* Sg = a.S + (size_t)bh * D * D + 4 * cg;
  f32x4 s[PD];
  constexpr int PD0 = PD < 2 ? PD : 2;            // passes requested ahead of the rows (which are needed first and come in behind them)
#pragma unroll
  for (int p = 0; p < PD0; ++p) s[p] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Sg + (size_t)(p * RPP + r0) * D));
  __builtin_amdgcn_sched_barrier(0);
  int n = a.fill[bh];                                               // every head carries its own copy of the count
  n = n < 0 ? 0 : (n > GC - 1 ? GC - 1 : n);                       // rows of the open group
  int m = kk;
  if (a.n_commit) { m = a.n_commit[b]; m = m < 0 ? 0 : (m > kk ? kk : m); }
  const int rows = n + kk;                                          // rows of (window ++ drafts)
  const bool crossing = rows > GC;                                  // some draft belongs to the next group
  typename Io::raw8 rk[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int r = part + NPART * t;
    int64_t idx;
    const void* src = row_of(a.kwin, a.k, win0, tok0, D, n, r < rows ? r : rows - 1, &idx);
    rk[t] = Io::load_raw8(src, idx + 8 * c8);
  }
#pragma unroll
  for (int p = PD0; p < PD; ++p) s[p] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Sg + (size_t)(p * RPP + r0) * D));
  Io::needed_here(q_raw);                          // (used by a few threads only: kept ahead of the state's requests)
  Io::needed_here(v_raw);

  if (pj < KP) {
    float xq[8], xv[8];
    Io::unpack8(q_raw, xq);
    Io::unpack8(v_raw, xv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = 8 * c8 + e;
      const bool live = pj < kk;
      sm.sc.rq[pj][i] = live ? xq[e] : 0.f;
      sm.sc.fq[i][pj] = live ? phi_any(xq[e], a.relu) : 0.f;
      sm.vv[pj][i] = live ? xv[e] : 0.f;
      sm.sc.red[pj][i] = 0.f;
      sm.sc.loc[pj][i] = live ? phi_any(xq[e], a.relu) : 0.f;   // phi(q_j) once more, draft-major, until step 2 clears it
    }
  }
  if (tid < D) sm.zz[tid] = z_reg;
#pragma unroll
  for (int mth = 0; mth < TAP_IT; ++mth) {
    const int e = tid + 256 * mth;
    const int t = e / D, cc = e % D;
    sm.wt[t][cc] = t < Kc ? tap_reg[mth] : 0.f;
    sm.hh[t][cc] = t < Kc - 1 ? hist_reg[mth] : 0.f;
  }
  __syncthreads();

  // ---- 1. logits q_j.k_r (raw rows), and phi(q_j).phi(k_r) for the rows of a group being completed.
  //         Thread = (8 consecutive features, every NPART-th row) ----
#pragma unroll
  for (int jj = 0; jj < KP; ++jj) {
    if (jj >= kk) continue;                                         // uniform
    float q8[8];
    {
      const f32x4 q0 = *reinterpret_cast<const f32x4*>(&sm.sc.rq[jj][8 * c8]);
      const f32x4 q1 = *reinterpret_cast<const f32x4*>(&sm.sc.rq[jj][8 * c8 + 4]);
      q8[0] = q0[0]; q8[1] = q0[1]; q8[2] = q0[2]; q8[3] = q0[3];
      q8[4] = q1[0]; q8[5] = q1[1]; q8[6] = q1[2]; q8[7] = q1[3];
    }
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      const int r = part + NPART * t;
      float xk[8];
      Io::unpack8(rk[t], xk);
      float dotv = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dotv = fmaf(q8[e], xk[e], dotv);
      dotv = sum_lanes<CG8>(dotv);
      if (c8 == 0 && r < rows) sm.W[jj][r] = dotv;
    }
    if (crossing) {                                                 // uniform
      {
        const f32x4 q0 = *reinterpret_cast<const f32x4*>(&sm.sc.loc[jj][8 * c8]);
        const f32x4 q1 = *reinterpret_cast<const f32x4*>(&sm.sc.loc[jj][8 * c8 + 4]);
        q8[0] = q0[0]; q8[1] = q0[1]; q8[2] = q0[2]; q8[3] = q0[3];
        q8[4] = q1[0]; q8[5] = q1[1]; q8[6] = q1[2]; q8[7] = q1[3];
      }
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        const int r = part + NPART * t;
        float xk[8];
        Io::unpack8(rk[t], xk);
        float lin = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) lin = fmaf(q8[e], phi_any(xk[e], a.relu), lin);
        lin = sum_lanes<CG8>(lin);
        if (c8 == 0 && r < GC) sm.lin[jj][r] = lin;
      }
    }
  }
  // the value rows, in the arrangement of step 1, are needed after the state has streamed: requested now, into the
  // registers that the key rows leave
  typename Io::raw8 rv[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int r = part + NPART * t;
    int64_t idx;
    const void* src = row_of(a.vwin, a.v, win0, tok0, D, n, r < rows ? r : rows - 1, &idx);
    rv[t] = Io::load_raw8(src, idx + 8 * c8);
  }
  __syncthreads();

  // ---- 2. per draft: softmax over its rows, the linear normaliser, the weights of the value rows ----
  for (int e = tid; e < KP * D; e += 256) sm.sc.loc[e / D][e % D] = 0.f;   // step 1 is done with its copy of phi(q)
  static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
  constexpr float to_log2 = 1.44269504088896340736f * (D == 64 ? 0.125f : 0.08838834764831845f);
  {
    // Sixteen lanes per draft, four drafts per wave, every sum and maximum inside a row of sixteen lanes with DPP
    // modifiers (a wave per draft with sums across its 64 lanes through the LDS crossbar was 18 dependent shuffles).
    constexpr int RPL = GROWS / 16;                                 // rows per lane
    static_assert(KP <= 16, "one pass of four waves");
    const int j = 4 * wv + (lane >> 4), sub = lane & 15;
    const bool live = j < kk;
    const int jj = live ? j : 0;                                    // lanes without a draft follow the first and write nothing
    const int P = n + jj;                                           // position of the draft
    const int g0 = P < GC ? 0 : GC;                                 // first row of its group
    float xr[RPL];
    float top = -INFINITY;
#pragma unroll
    for (int t = 0; t < RPL; ++t) {
      const int r = sub + 16 * t;
      const float x = sm.W[jj][r];
      xr[t] = (r >= g0 && r <= P) ? x : -INFINITY;
      top = fmaxf(top, xr[t]);
    }
    top = max_lanes<16>(top);                                       // the draft itself is always seen: finite
    float mass = 0.f;
#pragma unroll
    for (int t = 0; t < RPL; ++t) {
      xr[t] = __builtin_amdgcn_exp2f((xr[t] - top) * to_log2);      // exp2(-inf) = 0: rows that are not seen
      mass += xr[t];
    }
    // phi(q_j).z, plus the completed group for a draft of the next group
    float dz = 0.f;
#pragma unroll
    for (int e = 0; e < D / 16; ++e) dz = fmaf(sm.sc.fq[sub + 16 * e][jj], sm.zz[sub + 16 * e], dz);
    float lin[GC / 16];
#pragma unroll
    for (int t = 0; t < GC / 16; ++t) lin[t] = sm.lin[jj][sub + 16 * t];
    if (g0 > 0) {
#pragma unroll
      for (int t = 0; t < GC / 16; ++t) dz += lin[t];
    }
    mass = sum_lanes<16>(mass);
    dz = sum_lanes<16>(dz);
    const float gden = dz + a.eps;
    const float f = gden != 0.f ? a.alpha / gden : 0.f;
    const float inv_mass = 1.f / mass;                              // the draft itself is always seen: mass >= 1
    if (live) {
#pragma unroll
      for (int t = 0; t < RPL; ++t) {
        const int r = sub + 16 * t;
        float wgt = xr[t] * inv_mass;
        if (t < GC / 16) wgt = g0 > 0 ? f * lin[t] : wgt;           // the completed group, through the linear branch
        sm.W[j][r] = wgt;
      }
      if (sub == 0) sm.fscale[j] = f;
    }
  }
  __syncthreads();

  // ---- 3a. read-outs phi(q_j)^T S: the state streams through registers once ---------------------
  {
    float acc[KP][4];
#pragma unroll
    for (int j = 0; j < KP; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
#pragma unroll 1
    for (int pb = 0; pb < NPASS; pb += PD) {
#pragma unroll
      for (int q = 0; q < PD; ++q) {
        const int p = pb + q;
        const int i = p * RPP + r0;
        const f32x4 cur = s[q];
#pragma unroll
        for (int j = 0; j < KP; ++j) {
          const float f = sm.sc.fq[i][j];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[j][e] = fmaf(f, cur[e], acc[j][e]);
        }
        if (p + PD < NPASS) s[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Sg + (size_t)((p + PD) * RPP + r0) * D));
      }
    }
    // threads that share a column group sit CG lanes apart inside a wave; the four waves add up in LDS,
#pragma unroll
    for (int j = 0; j < KP; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (CG <= 16) acc[j][e] = add_xor<16>(acc[j][e]);
        acc[j][e] = add_xor<32>(acc[j][e]);
      }
    // ... one after the other, so that the sum does not depend on which wave arrives first
    for (int turn = 0; turn < 4; ++turn) {
      if (wv == turn && lane < CG) {
#pragma unroll
        for (int j = 0; j < KP; ++j) {
          if (j < kk) {
#pragma unroll
            for (int e = 0; e < 4; ++e) sm.sc.red[j][4 * cg + e] += acc[j][e];
          }
        }
      }
      __syncthreads();
    }
  }
  // ---- 3b. value rows times their weights, in the arrangement of step 1 (a row past the end has weight 0);
  //          the partitions of a wave are CG8 lanes apart, the waves add up in LDS in turn ----------------
  {
    constexpr int JB = KP < 4 ? KP : 4;            // drafts at a time
#pragma unroll
    for (int jb = 0; jb < KP; jb += JB) {
      float accl[JB][8];
#pragma unroll
      for (int j = 0; j < JB; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) accl[j][e] = 0.f;
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        const int r = part + NPART * t;
        float xv[8];
        Io::unpack8(rv[t], xv);
#pragma unroll
        for (int j = 0; j < JB; ++j) {
          const float wgt = r < GROWS ? sm.W[jb + j][r < GROWS ? r : GROWS - 1] : 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) accl[j][e] = fmaf(wgt, xv[e], accl[j][e]);
        }
      }
#pragma unroll
      for (int j = 0; j < JB; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (CG8 <= 8) accl[j][e] = add_xor<8>(accl[j][e]);
          accl[j][e] = add_xor<16>(accl[j][e]);
          accl[j][e] = add_xor<32>(accl[j][e]);
        }
      for (int turn = 0; turn < 4; ++turn) {
        if (wv == turn && lane < CG8) {
#pragma unroll
          for (int j = 0; j < JB; ++j)
            if (jb + j < kk) {
#pragma unroll
              for (int e = 0; e < 8; ++e) sm.sc.loc[jb + j][8 * c8 + e] += accl[j][e];
            }
        }
        __syncthreads();
      }
    }
  }

  // ---- 4. outputs ---------------------------------------------------------------------------------
  for (int idx = tid; idx < kk * D; idx += 256) {
    const int j = idx / D, c = idx % D;
    float u = 0.f;
    for (int t = 0; t < Kc; ++t) {
      // tap t looks t rows back from draft j: another draft if t <= j, else history row (t - j) back
      const float x = t <= j ? sm.vv[j - t][c] : sm.hh[t - j - 1][c];
      u = fmaf(sm.wt[t][c], x, u);
    }
    Io::store1(a.out, tok0 + idx, fmaf(sm.fscale[j], sm.sc.red[j][c], sm.sc.loc[j][c]) + u);
  }

  // ---- 5. the kept drafts join the state ----------------------------------------------------------
  if (m == 0) return;                                               // uniform: nothing kept, nothing changes
  if (tid == 0) a.fill[bh] = (n + m) % GC;                          // read at the top by this workgroup only
  if (Kc > 1) {
    for (int c = tid; c < D; c += 256) {
      for (int r = 0; r < Kc - 1; ++r) {
        const int sidx = m - (Kc - 1) + r;                          // position in (history ++ kept drafts)
        const int64_t dst = hist0 + (int64_t)r * D + c;
        if (sidx >= 0) Io::store1(a.hist, dst, sm.vv[sidx][c]);
        else Io::store1(a.hist, dst, sm.hh[-sidx - 1][c]);
      }
    }
  }
  typedef typename Io::elem elem_t;
  const elem_t* dk = static_cast<const elem_t*>(a.k) + tok0;
  const elem_t* dv = static_cast<const elem_t*>(a.v) + tok0;
  elem_t* wk = static_cast<elem_t*>(a.kwin) + win0;
  elem_t* wvp = static_cast<elem_t*>(a.vwin) + win0;
  if (n + m < GC) {
    // the group stays open: drafts 0..m-1 become rows n..n+m-1
    for (int e = tid; e < m * D; e += 256) {
      wk[(size_t)n * D + e] = dk[e];
      wvp[(size_t)n * D + e] = dv[e];
    }
    return;
  }
  // the group is complete: rows 0..63 of (window ++ drafts) enter S and z, 16 rows at a time through LDS.
  // Once in 64 tokens: the state slice is walked once per 16 rows (through the cache) rather than held in
  // registers, which would cost the common path its occupancy.
  float* Sw = a.S + (size_t)bh * D * D + 4 * cg;
  float zsum = tid < D ? sm.zz[tid] : 0.f;
  for (int rb = 0; rb < GC; rb += 16) {
    __syncthreads();                                                // the previous 16 rows have been used (first turn: the outputs are done)
    for (int e = tid; e < 16 * D; e += 256) {
      const int r = rb + e / D, i = e % D;
      int64_t ik, iv;
      const void* ksrc = row_of(a.kwin, a.k, win0, tok0, D, n, r, &ik);
      const void* vsrc = row_of(a.vwin, a.v, win0, tok0, D, n, r, &iv);
      sm.st.k[e / D][i] = phi_any(Io::load1(ksrc, ik + i), a.relu);
      sm.st.v[e / D][i] = Io::load1(vsrc, iv + i);
    }
    __syncthreads();
#pragma unroll 1
    for (int p = 0; p < NPASS; ++p) {
      const int i = p * RPP + r0;
      f32x4 cur = *reinterpret_cast<const f32x4*>(Sw + (size_t)i * D);
#pragma unroll 4
      for (int r = 0; r < 16; ++r) {
        const f32x4 v4 = *reinterpret_cast<const f32x4*>(&sm.st.v[r][4 * cg]);
        const float kf = sm.st.k[r][i];
#pragma unroll
        for (int e = 0; e < 4; ++e) cur[e] = fmaf(kf, v4[e], cur[e]);
      }
      *reinterpret_cast<f32x4*>(Sw + (size_t)i * D) = cur;
    }
    if (tid < D) {
#pragma unroll
      for (int r = 0; r < 16; ++r) zsum += sm.st.k[r][tid];
    }
  }
  if (tid < D) a.z[(size_t)bh * D + tid] = zsum;
  __syncthreads();                                                  // every read of the old window rows is done
  // the next group opens with the kept drafts beyond the completed one: drafts 64-n .. m-1 -> rows 0 ..
  const int first = GC - n;
  for (int e = tid; e < (m - first) * D; e += 256) {
    wk[e] = dk[(size_t)first * D + e];
    wvp[e] = dv[(size_t)first * D + e];
  }
}

template <typename Io, int D>
static hipError_t launch_kp(const VerifyGroupedArgs& a, hipStream_t st) {
  const dim3 grid((unsigned)(a.B * a.H)), block(256);
  if (a.kk <= 1) hipLaunchKernelGGL((verify_grouped_kernel<Io, D, 1>), grid, block, 0, st, a);
  else if (a.kk <= 4) hipLaunchKernelGGL((verify_grouped_kernel<Io, D, 4>), grid, block, 0, st, a);
  else if (a.kk <= 8) hipLaunchKernelGGL((verify_grouped_kernel<Io, D, 8>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((verify_grouped_kernel<Io, D, 16>), grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t launch_verify_grouped(const VerifyGroupedArgs& a, bool bf16, int d, hipStream_t st) {
  if (bf16) return d == 128 ? launch_kp<IoBf16, 128>(a, st) : launch_kp<IoBf16, 64>(a, st);
  return d == 128 ? launch_kp<IoF32, 128>(a, st) : launch_kp<IoF32, 64>(a, st);
}

}  // namespace linattn
