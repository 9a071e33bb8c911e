// The three-branch form of Sec. 4.1 in groups of 256 tokens on the matrix cores (bf16 rows): the group size of the
// paper's FLASH experiment (Sec. 5 "Settings", Sec. 5.3).  Per token t of a group g
//
//   out_t = alpha * phi(q_t)^T S_g / (phi(q_t).z_g + eps)            S_g, z_g: the sums over everything before the group
//         + sum_{i in g, i <= t} softmax_i(q_t.k_i / sqrt(d)) v_i     causal softmax attention inside the group (Eq. 1)
//         + causal depthwise conv of V
//
// A group of 256 tokens is four times what the 64-token kernel keeps in LDS, and its running state cannot both stay
// frozen for the group and take the group's own products in the same registers.  So this kernel is built the other
// way round: one workgroup of eight waves per (b, h, segment) walks its groups with the whole group's raw key and
// value rows in LDS (139 KB at d = 128) and the running state in its workspace slot in global memory (fp32; it stays
// in the L2 cache between the group's read-out and its update).  Every wave owns one 32-query tile of the
// group and all value channels:
//
//   local branch    for each 32-key tile up to the diagonal: S^T tile = K Q^T (keys in registers, queries in lanes),
//                   online softmax per lane (running maximum, running sum), and O^T += V^T P^T with P taken
//                   straight from the score accumulators as the MFMA operand -- the accumulator layout is the
//                   operand layout up to a permutation of the key index, which is applied to the transposed reads
//                   of V instead, so the weights never touch LDS;
//   linear branch   O_lin^T = S_g^T phi(Q)^T, one 32-channel tile at a time, the state before the group as the MFMA
//                   operand (bf16 in LDS, rounded for the read-out only, as in the other matrix-core kernels);
//   epilogue        O / l + alpha O_lin / (phi(q).z_g + eps), staged through LDS in fp32 (the key rows' memory); the
//                   store loop adds the causal conv over V (up to 8 taps; with more, what the long-conv pass left in
//                   out) and writes whole rows.
//
// Then, unless nothing after the group needs it, the group enters the state: phi is applied to the key rows in
// place and every wave adds phi(K)^T V to its two 32 x 32 tiles of the state -- the tiles it read for the linear
// branch -- and writes them back to the slot.  Segments along the sequence start on group
// boundaries; their start states come from the same first pass and prefix sum as in the 64-token kernels.
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D>
struct G256Cfg {
  static constexpr int GT = 256;             // tokens per group
  static constexpr int NW = 8;               // waves: one 32-query tile each
  static constexpr int NT = NW * 64;
  static constexpr int KSD = D / 16;         // feature steps of a 32 x 32 x 16 MFMA
  static constexpr int CT = D / 32;          // 32-channel tiles
  static constexpr int KS = D + 8;           // key rows: 16-byte row reads, transpose reads
  static constexpr int VS = D + 4;           // value rows: transpose reads, 8-byte row reads
  static constexpr int OS = D + 4;           // staged output rows, fp32, 128 at a time (in the key rows' memory)
  static constexpr int OFF_K = 0;
  static constexpr int OFF_V = OFF_K + GT * KS * 2;                   // row r = token r - HALO
  static constexpr int OFF_W = (OFF_V + (HALO + GT) * VS * 2 + 15) / 16 * 16;   // [8][D] float conv taps, tap-major
  static constexpr int OFF_Z = OFF_W + 8 * D * 4;                     // [D] float: z before the group
  static constexpr int OFF_R = OFF_Z + D * 4;                         // [NW][D] float: per-wave column sums of phi(K)
  static constexpr int TOTAL = OFF_R + NW * D * 4;
  static_assert(128 * OS * 4 <= GT * KS * 2, "the staged outputs take the place of the key rows");
  static_assert(TOTAL <= 160 * 1024, "LDS");
};

}  // namespace

// Keeps the compiler from moving memory operations across this point: the unrolled epilogue would otherwise
// request every tap, value row and state word of a group at once and spill hundreds of registers.
#define LINATTN_ORDER() __asm__ volatile("" ::: "memory")

template <int D, int KCM>
__global__ __launch_bounds__(512) void prefill_grouped256_kernel(PrefillArgs a) {
  using G = G256Cfg<D>;
  constexpr int GT = G::GT;
  constexpr int SLOT = D * D + D;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Kl = reinterpret_cast<uint16_t*>(smem + G::OFF_K);
  uint16_t* Vl = reinterpret_cast<uint16_t*>(smem + G::OFF_V);
  float* wl = reinterpret_cast<float*>(smem + G::OFF_W);
  float* zl = reinterpret_cast<float*>(smem + G::OFF_Z);
  float* redl = reinterpret_cast<float*>(smem + G::OFF_R);
  float* Ol = reinterpret_cast<float*>(smem + G::OFF_K);   // staged output rows, once the key rows are done with

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
  // Query tile j meets j + 1 key tiles.  Waves w and w + 4 share a SIMD: tiles (w, 7 - w) give every SIMD nine.
  const int qtile = w < 4 ? w : 11 - w;
  const int bh = blockIdx.x / a.nseg, seg = blockIdx.x % a.nseg;
  const int b = bh / a.H, h = bh % a.H;
  const int t_begin = seg * a.seg_len;
  const int t_end = (t_begin + a.seg_len) < a.L ? (t_begin + a.seg_len) : a.L;
  const int ngroups = (t_end - t_begin + GT - 1) / GT;
  const int64_t base = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base;
  uint16_t* gout = static_cast<uint16_t*>(a.out) + base;
  // this workgroup's slot: the state before its current group, S [D][D] then z [D], fp32
  float* slot = a.ws + ((size_t)bh * a.nseg + seg) * SLOT;
  const uint16_t* staged_hist =
      reinterpret_cast<const uint16_t*>(a.ws + (size_t)a.B * a.H * a.nseg * SLOT) + (size_t)bh * HALO * D;
  const bool last_seg = seg == a.nseg - 1;
  // The slot through buffer addressing (descriptor in scalar registers + one lane offset + a constant per request):
  // the several hundred requests of a group then need no address registers of their own.
  const __amdgpu_buffer_rsrc_t slot_rs = __builtin_amdgcn_make_buffer_rsrc(slot, 0, SLOT * 4, 0x00020000);
  static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
  constexpr float to_log2 = 1.44269504088896340736f * (D == 64 ? 0.125f : 0.08838834764831845f);

  // ---- once: the conv taps; without segments nobody has written the slot yet -----------------------------------
  for (int e = tid; e < 8 * D; e += G::NT) {
    const int j = e / D, cc = e % D;
    wl[e] = (j < a.Kc && !a.no_conv) ? a.conv_w[((size_t)h * D + cc) * a.Kc + j] : 0.f;
  }
  if (a.nseg == 1) {
    for (int e = tid; e < SLOT; e += G::NT) {
      float x = 0.f;
      if (a.S_in) x = e < D * D ? a.S_in[(size_t)bh * D * D + e] : a.z_in[(size_t)bh * D + (e - D * D)];
      slot[e] = x;
    }
  }
  // The slot is written and read by this workgroup only, but by different waves: a fence of workgroup scope (the
  // waves of a workgroup share their compute unit's vector cache, so completed stores are seen by all of them; a
  // fence of device scope would write back and invalidate the whole L2 of the chiplet, tens of microseconds) and
  // the barrier.
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __syncthreads();

  for (int gi = 0; gi < ngroups; ++gi) {
    const int tok0 = t_begin + gi * GT;
    const int nt = (t_end - tok0) < GT ? (t_end - tok0) : GT;
    // ---- 1. this wave's queries, straight into MFMA operand registers: lane = query 32 qtile + l32, registers =
    //         features 16ks + 8hi + 0..7.  A query past the end reads the last row that exists; it is never stored.
    const int qt = 32 * qtile + l32;
    const int qrow = qt < nt ? qt : nt - 1;
    u32x4 qraw[G::KSD];
    {
      const uint16_t* qp = gq + (int64_t)(tok0 + qrow) * a.st + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < G::KSD; ++ks) qraw[ks] = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
    }
    // ---- 2. the group's raw key rows and value rows -> LDS (rows past the end are zero rows), the 8 value rows
    //         before the group (earlier tokens, else the incoming history, else zeros), z before the group.
    //         Every request is issued without a condition -- a row past the end re-reads the last row that exists,
    //         a history row that does not exist re-reads a row that does; the values are dropped afterwards --
    //         because a load under a lane-dependent branch makes the compiler wait for all earlier ones first, and
    //         the rows then arrive one round trip after the other.
    {
      constexpr int NPC = GT * (D / 8) / G::NT;            // 16-byte pieces of K (and of V) per thread
      constexpr int NHL = HALO * D / G::NT;                // elements of the 8 rows before the group per thread
      u32x4 kx[NPC], vx[NPC];
      uint16_t hx[NHL];
#pragma unroll
      for (int i = 0; i < NPC; ++i) {
        const int e = tid + G::NT * i;
        const int r = e / (D / 8), c0 = 8 * (e % (D / 8));
        const int64_t off = (int64_t)(tok0 + (r < nt ? r : nt - 1)) * a.st + c0;
        kx[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gk + off));
        vx[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gv + off));
      }
      if constexpr (KCM > 0) {
        const uint16_t* hin = static_cast<const uint16_t*>(a.hist_in);
#pragma unroll
        for (int i = 0; i < NHL; ++i) {
          const int e = tid + G::NT * i;
          const int r = e / D, cc = e % D;
          const int tok = tok0 - HALO + r;
          // (selects only: the load below has no condition)
          const bool staged = tok < 0 && hin != nullptr && a.nseg > 1;
          const bool given = tok < 0 && hin != nullptr && a.nseg <= 1 && a.Kc - 1 + tok >= 0;
          const uint16_t* base_p = staged ? staged_hist : given ? hin : gv;
          const int64_t off = staged ? (int64_t)(HALO + tok) * D + cc
                              : given ? ((int64_t)bh * (a.Kc - 1) + (a.Kc - 1 + tok)) * D + cc
                                      : (int64_t)(tok >= 0 ? tok : 0) * a.st + cc;
          const uint16_t* src = base_p + off;
          const bool have = tok >= 0 || staged || given;
          const uint16_t x = *src;
          hx[i] = have ? x : (uint16_t)0;
        }
      }
      const float zx = slot[D * D + (tid < D ? tid : 0)];
      const bool ragged = nt < GT;                         // uniform
#pragma unroll
      for (int i = 0; i < NPC; ++i) {
        const int e = tid + G::NT * i;
        const int r = e / (D / 8), c0 = 8 * (e % (D / 8));
        if (ragged && r >= nt) kx[i] = vx[i] = u32x4{0, 0, 0, 0};
        *reinterpret_cast<u32x4*>(Kl + r * G::KS + c0) = kx[i];
        u32x2* vrow = reinterpret_cast<u32x2*>(Vl + (HALO + r) * G::VS + c0);
        vrow[0] = u32x2{vx[i][0], vx[i][1]};
        vrow[1] = u32x2{vx[i][2], vx[i][3]};
      }
      if constexpr (KCM > 0) {
#pragma unroll
        for (int i = 0; i < NHL; ++i) {
          const int e = tid + G::NT * i;
          Vl[(e / D) * G::VS + e % D] = hx[i];
        }
      }
      if (tid < D) zl[tid] = zx;
    }
    __syncthreads();                                       // A: the group is in LDS

    // ---- 3. local branch: key tiles 0 .. qtile, online softmax per lane, O^T += V^T P^T -----------------------
    // o[ct][r] = O[query 32 qtile + l32][channel 32ct + 8(r/4) + 4hi + r%4]
    // The products of key tile kt + 1 are issued before the softmax of tile kt, so that the matrix cores work while
    // the vector ALUs do: a wave alone is a chain of LDS read -> MFMA -> exp -> MFMA that nothing else fills (two
    // waves per SIMD).  After the last tile the look-ahead repeats that tile; its result is dropped.
    f32x16 o[G::CT];
#pragma unroll
    for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ct][r] = 0.f;
    float mtop = -INFINITY, mass = 0.f;                    // largest raw product so far; this lane's share of the sum
    auto scores = [&](int kt) {
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
      const uint16_t* ka = Kl + (32 * kt + l32) * G::KS + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < G::KSD; ++ks) s = mfma(lds_row8(ka + 16 * ks), __builtin_bit_cast(bf16x8, qraw[ks]), s);
      return s;
    };
    f32x16 ahead = scores(0);
    for (int kt = 0; kt <= qtile; ++kt) {
      f32x16 acc = ahead;
      ahead = scores(kt < qtile ? kt + 1 : qtile);
      // acc[r]: key 32kt + 8(r/4) + 4hi + r%4, query 32 qtile + l32.  Keys later than the query (diagonal tile
      // only) become -inf: their weight is an exact zero, nothing of a later token leaks.
      float top = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kl = 8 * (r >> 2) + 4 * hi + (r & 3);
        acc[r] = (kt < qtile || kl <= l32) ? acc[r] : -INFINITY;
        top = fmaxf(top, acc[r]);
      }
      top = fmaxf(top, __shfl_xor(top, 32));               // lanes l and l + 32 hold the same query
      const float mnew = fmaxf(mtop, top);                 // finite from the first tile on: key 0 is seen by every query
      const float corr = __builtin_amdgcn_exp2f((mtop - mnew) * to_log2);   // exp2(-inf) = 0 the first time
      const float shift = -mnew * to_log2;
      float rs = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[r] = __builtin_amdgcn_exp2f(fmaf(acc[r], to_log2, shift));
        rs += acc[r];
      }
      mass = fmaf(mass, corr, rs);
      mtop = mnew;
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ct][r] *= corr;
      const bf16x8 p0 = pack8(acc, 0), p1 = pack8(acc, 8);
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct) {
        o[ct] = mfma(tr_operand_acc_order(Vl + HALO * G::VS, G::VS, 32 * kt, 32 * ct, lane), p0, o[ct]);
        o[ct] = mfma(tr_operand_acc_order(Vl + HALO * G::VS, G::VS, 32 * kt + 16, 32 * ct, lane), p1, o[ct]);
      }
    }
    // ---- 4. this wave's tiles of the state before the group (feature block ib, channel block cb; lanes = channels,
    //         registers = features): requested here, so that they travel while the feature map runs.  They are the
    //         linear branch's operand and, with the group's own products added, the state after the group -- the slot
    //         is read once.
    constexpr int TPW = (G::CT * G::CT + G::NW - 1) / G::NW;
    f32x16 sold[TPW];
#pragma unroll
    for (int s2 = 0; s2 < TPW; ++s2) {
      const int tile = w + G::NW * s2;
      if (tile < G::CT * G::CT) {                          // uniform
        const int so = ((32 * (tile / G::CT) + 4 * hi) * D + 32 * (tile % G::CT) + l32) * 4;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sold[s2][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(slot_rs, so, (8 * (r >> 2) + (r & 3)) * (D * 4), 0));
      }
    }
    mass += __shfl_xor(mass, 32);
    const float inv_mass = __builtin_amdgcn_rcpf(mass);    // the token itself is always seen: mass >= 1
#pragma unroll
    for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ct][r] *= inv_mass;

    // ---- 5. for the linear branch: phi(Q) as the MFMA operand (in place of the raw rows) and phi(q).z -----------
    bf16x8 fq[G::KSD];
    float dz = 0.f;
#pragma unroll
    for (int ks = 0; ks < G::KSD; ++ks) {
      const u32x4 f = phi_pack8_nb(qraw[ks], a.relu ? 0.f : 1.f);
      fq[ks] = __builtin_bit_cast(bf16x8, f);
      const float* zp = zl + 16 * ks + 8 * hi;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        dz = fmaf(bf16_lo_to_f32(f[i]), zp[2 * i], dz);
        dz = fmaf(bf16_hi_to_f32(f[i]), zp[2 * i + 1], dz);
      }
    }
    dz += __shfl_xor(dz, 32);
    const float gden = dz + a.eps;
    const float fscale = gden != 0.f ? a.alpha * __builtin_amdgcn_rcpf(gden) : 0.f;   // nothing before the group: no branch

    // ---- 6. the group enters the state, if anything after it needs that -----------------------------------------
    const bool more = gi + 1 < ngroups;
    const bool update = more || (last_seg && (a.S_out != nullptr || a.z_out != nullptr));   // uniform
    __syncthreads();                                       // B: every wave is done with the raw key rows
    if (update) {
      // phi in place on the key rows (a thread meets the same eight features in every row it maps: their sums over
      // the rows, for z, on the way)
      static_assert(G::NT % (D / 8) == 0 && 64 % (D / 8) == 0, "a thread's feature block is fixed");
      float zp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < GT * (D / 8) / G::NT; ++i) {
        const int e = tid + G::NT * i;
        const int r = e / (D / 8), c0 = 8 * (e % (D / 8));
        u32x4* p8 = reinterpret_cast<u32x4*>(Kl + r * G::KS + c0);
        u32x4 f = phi_pack8_nb(*p8, a.relu ? 0.f : 1.f);
        if (r >= nt) f = u32x4{0, 0, 0, 0};                // phi(0) = 1: rows that do not exist stay zero rows
        *p8 = f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          zp[2 * j] += bf16_lo_to_f32(f[j]);
          zp[2 * j + 1] += bf16_hi_to_f32(f[j]);
        }
      }
      // the lanes of a wave that share a feature block (lane % (D/8) equal) add up; one row of sums per wave
#pragma unroll
      for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int m = D / 8; m < 64; m *= 2) zp[j] += __shfl_xor(zp[j], m);
      }
      if (lane < D / 8) {
        *reinterpret_cast<f32x4*>(redl + w * D + 8 * lane) = f32x4{zp[0], zp[1], zp[2], zp[3]};
        *reinterpret_cast<f32x4*>(redl + w * D + 8 * lane + 4) = f32x4{zp[4], zp[5], zp[6], zp[7]};
      }
      __syncthreads();
      // S += phi(K)^T V on this wave's tiles: they share their channel block, so one value operand serves both
      static_assert(G::NW % G::CT == 0, "a wave's tiles lie in one channel block");
      if (w < G::CT * G::CT) {                             // uniform
        const int cb = w % G::CT;
        f32x16 snew[TPW];
#pragma unroll
        for (int s2 = 0; s2 < TPW; ++s2) snew[s2] = sold[s2];
#pragma unroll 8
        for (int ks = 0; ks < GT / 16; ++ks) {
          const bf16x8 vb = tr_operand(Vl + HALO * G::VS, G::VS, 16 * ks, 32 * cb, lane);
#pragma unroll
          for (int s2 = 0; s2 < TPW; ++s2)
            if (w + G::NW * s2 < G::CT * G::CT)
              snew[s2] = mfma(tr_operand(Kl, G::KS, 16 * ks, 32 * ((w + G::NW * s2) / G::CT), lane), vb, snew[s2]);
        }
#pragma unroll
        for (int s2 = 0; s2 < TPW; ++s2) {
          const int tile = w + G::NW * s2;
          if (tile < G::CT * G::CT) {
            const int so = ((32 * (tile / G::CT) + 4 * hi) * D + 32 * cb + l32) * 4;
#pragma unroll
            for (int r = 0; r < 16; ++r)
              __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(snew[s2][r]), slot_rs, so, (8 * (r >> 2) + (r & 3)) * (D * 4), 0);
          }
        }
      }
      if (tid < D) {
        float zs = zl[tid];
#pragma unroll
        for (int i = 0; i < G::NW; ++i) zs += redl[i * D + tid];
        slot[D * D + tid] = zs;
      }
      // (No fence: from here to the end of the walk every lane re-reads from the slot only what it stored itself --
      // the tile layout and the tile-to-wave map are the same in every group, and z is one thread per feature.)
      __syncthreads();                                     // the key rows' memory is free
    }

    // ---- 6b. linear branch: the state before the group goes to the key rows' memory as bf16 [channel][feature]
    //          (rounded for the read-out only), every wave its own tiles; O^T += (alpha / (phi(q).z + eps))
    //          S_g^T phi(Q)^T with the state operand read row-wise (lanes = channels, registers = features
    //          16ks + 8hi + 0..7)
    {
      uint16_t* Sl = Kl;
      constexpr int SS = D + 8;
#pragma unroll
      for (int s2 = 0; s2 < TPW; ++s2) {
        const int tile = w + G::NW * s2;
        if (tile < G::CT * G::CT) {                        // uniform
          uint16_t* srow = Sl + (32 * (tile % G::CT) + l32) * SS + 32 * (tile / G::CT) + 4 * hi;
#pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<u32x2*>(srow + 8 * g) =
                u32x2{pack_bf16x2(sold[s2][4 * g], sold[s2][4 * g + 1]), pack_bf16x2(sold[s2][4 * g + 2], sold[s2][4 * g + 3])};
        }
      }
      __syncthreads();
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct) {
        f32x16 lin;
#pragma unroll
        for (int r = 0; r < 16; ++r) lin[r] = 0.f;
        const uint16_t* sa = Sl + (32 * ct + l32) * SS + 8 * hi;
#pragma unroll
        for (int ks = 0; ks < G::KSD; ++ks) lin = mfma(lds_row8(sa + 16 * ks), fq[ks], lin);
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ct][r] = fmaf(lin[r], fscale, o[ct][r]);
      }
      __syncthreads();                                     // every wave is done with the state operand
    }

    // ---- 7. outputs: staged as fp32 rows in the key rows' memory, 128 tokens at a time (waves 0..3, then 4..7);
    //         the store loop adds the causal conv over V (taps and value rows from LDS), rounds once and writes
    //         whole rows
    if constexpr (KCM == 0) {
      // No conv in this kernel (more than 8 taps): the pass that computes it ran first and left it in out, which is
      // added to here -- the requests for this thread's pieces of out go ahead of the staging, the sum is formed in
      // fp32 and rounded once.  128 tokens at a time (waves 0..3, then 4..7), as below.
      constexpr int PPT = 128 * (D / 8) / G::NT;
#pragma unroll 1
      for (int half = 0; half < 2; ++half) {
        u32x4 held[PPT];
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
          const int e = tid + G::NT * i;
          const int r = 128 * half + e / (D / 8), c0 = 8 * (e % (D / 8));
          held[i] = *reinterpret_cast<const u32x4*>(gout + (int64_t)(tok0 + (r < nt ? r : nt - 1)) * a.st + c0);
        }
        if ((w >> 2) == half) {                            // uniform per wave
          float* orow = Ol + (qt - 128 * half) * G::OS + 4 * hi;
#pragma unroll
          for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *reinterpret_cast<f32x4*>(orow + 32 * ct + 8 * g) = f32x4{o[ct][4 * g], o[ct][4 * g + 1], o[ct][4 * g + 2], o[ct][4 * g + 3]};
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
          const int e = tid + G::NT * i;
          const int r = 128 * half + e / (D / 8), c0 = 8 * (e % (D / 8));
          if (r < nt) {
            const float* src = Ol + (r - 128 * half) * G::OS + c0;
            const f32x4 y0 = *reinterpret_cast<const f32x4*>(src), y1 = *reinterpret_cast<const f32x4*>(src + 4);
            const u32x4 h4 = held[i];
            __builtin_nontemporal_store(u32x4{pack_bf16x2(y0[0] + bf16_lo_to_f32(h4[0]), y0[1] + bf16_hi_to_f32(h4[0])),
                                              pack_bf16x2(y0[2] + bf16_lo_to_f32(h4[1]), y0[3] + bf16_hi_to_f32(h4[1])),
                                              pack_bf16x2(y1[0] + bf16_lo_to_f32(h4[2]), y1[1] + bf16_hi_to_f32(h4[2])),
                                              pack_bf16x2(y1[2] + bf16_lo_to_f32(h4[3]), y1[3] + bf16_hi_to_f32(h4[3]))},
                                        reinterpret_cast<u32x4*>(gout + (int64_t)(tok0 + r) * a.st + c0));
          }
        }
        __syncthreads();                                   // the staging rows are free again; after the second half, all of LDS
      }
    } else
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
      if ((w >> 2) == half) {                              // uniform per wave
        float* orow = Ol + (qt - 128 * half) * G::OS + 4 * hi;
#pragma unroll
        for (int ct = 0; ct < G::CT; ++ct)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<f32x4*>(orow + 32 * ct + 8 * g) = f32x4{o[ct][4 * g], o[ct][4 * g + 1], o[ct][4 * g + 2], o[ct][4 * g + 3]};
      }
      __syncthreads();
      for (int e = tid; e < 128 * (D / 8); e += G::NT) {
        const int r = 128 * half + e / (D / 8), c0 = 8 * (e % (D / 8));
        if (r < nt) {
          const float* src = Ol + (r - 128 * half) * G::OS + c0;
          const f32x4 y0 = *reinterpret_cast<const f32x4*>(src), y1 = *reinterpret_cast<const f32x4*>(src + 4);
          float y[8] = {y0[0], y0[1], y0[2], y0[3], y1[0], y1[1], y1[2], y1[3]};
#pragma unroll
          for (int j = 0; j < KCM; ++j) {
            const f32x4 w0 = *reinterpret_cast<const f32x4*>(wl + j * D + c0), w1 = *reinterpret_cast<const f32x4*>(wl + j * D + c0 + 4);
            const u32x2* vp = reinterpret_cast<const u32x2*>(Vl + (HALO + r - j) * G::VS + c0);
            const u32x2 x0 = vp[0], x1 = vp[1];
            y[0] = fmaf(w0[0], bf16_lo_to_f32(x0[0]), y[0]);
            y[1] = fmaf(w0[1], bf16_hi_to_f32(x0[0]), y[1]);
            y[2] = fmaf(w0[2], bf16_lo_to_f32(x0[1]), y[2]);
            y[3] = fmaf(w0[3], bf16_hi_to_f32(x0[1]), y[3]);
            y[4] = fmaf(w1[0], bf16_lo_to_f32(x1[0]), y[4]);
            y[5] = fmaf(w1[1], bf16_hi_to_f32(x1[0]), y[5]);
            y[6] = fmaf(w1[2], bf16_lo_to_f32(x1[1]), y[6]);
            y[7] = fmaf(w1[3], bf16_hi_to_f32(x1[1]), y[7]);
          }
          __builtin_nontemporal_store(u32x4{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])},
                                      reinterpret_cast<u32x4*>(gout + (int64_t)(tok0 + r) * a.st + c0));
        }
      }
      __syncthreads();                                     // the staging rows are free again; after the second half, all of LDS
    }
  }

  // ---- the state after the last token, handed over by the last segment ----------------------------------------------
  if (!last_seg) return;
  // other lanes than the ones that stored it read the slot from here on
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __syncthreads();
  if (ngroups > 0 && (a.S_out || a.z_out)) {
    if (a.S_out) {
      // (every request of the thread in flight before the first store: a loop of load, wait, store would pay one
      // round trip to memory per iteration)
      constexpr int SIT = D * D / 4 / G::NT;
      f32x4 sx[SIT];
#pragma unroll
      for (int i = 0; i < SIT; ++i) sx[i] = reinterpret_cast<const f32x4*>(slot)[tid + G::NT * i];
#pragma unroll
      for (int i = 0; i < SIT; ++i) reinterpret_cast<f32x4*>(a.S_out + (size_t)bh * D * D)[tid + G::NT * i] = sx[i];
    }
    if (a.z_out && tid < D) a.z_out[(size_t)bh * D + tid] = slot[D * D + tid];
  }
  if (a.hist_out && tid < D) {
    // last Kc-1 value rows of (history ++ sequence); one thread per channel reads all its rows before it writes
    // any, so an aliased hist_in is read before it is overwritten (with segments the staged copy is read)
    const uint16_t* hin = static_cast<const uint16_t*>(a.hist_in);
    uint16_t* hout = static_cast<uint16_t*>(a.hist_out) + (size_t)bh * (a.Kc - 1) * D;
    uint16_t hx[HALO];
#pragma unroll
    for (int r = 0; r < HALO; ++r) {
      const int tok = a.L - (a.Kc - 1) + r;
      hx[r] = 0;
      if (r < a.Kc - 1) {
        if (tok >= 0) hx[r] = gv[(int64_t)tok * a.st + tid];
        else if (hin) hx[r] = a.nseg > 1 ? staged_hist[(size_t)(HALO + tok) * D + tid]
                                         : hin[((size_t)bh * (a.Kc - 1) + (a.Kc - 1 + tok)) * D + tid];
      }
    }
#pragma unroll
    for (int r = 0; r < HALO; ++r)
      if (r < a.Kc - 1) hout[(size_t)r * D + tid] = hx[r];
  }
}

#undef LINATTN_ORDER

template <int D, int KCM>
static hipError_t launch_g256(const PrefillArgs& a, hipStream_t st) {
  using G = G256Cfg<D>;
  auto kern = prefill_grouped256_kernel<D, KCM>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, G::TOTAL);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H * a.nseg)), dim3(G::NT), G::TOTAL, st, a);
  return hipGetLastError();
}

// The full pass of the three-branch form in groups of 256 tokens.  a.ws holds one slot per (b, h, segment) -- with
// segments, filled by the first pass and the prefix sum; without, initialised here -- and the staged history rows.
hipError_t launch_prefill_grouped256(const PrefillArgs& a, int d, hipStream_t st) {
  if (d == 128) {
    if (a.no_conv) return launch_g256<128, 0>(a, st);
    if (a.Kc <= 3) return launch_g256<128, 3>(a, st);
    if (a.Kc <= 5) return launch_g256<128, 5>(a, st);
    return launch_g256<128, 8>(a, st);
  }
  if (a.no_conv) return launch_g256<64, 0>(a, st);
  if (a.Kc <= 3) return launch_g256<64, 3>(a, st);
  if (a.Kc <= 5) return launch_g256<64, 5>(a, st);
  return launch_g256<64, 8>(a, st);
}

}  // namespace linattn
