// Prefill on the matrix cores with specialised waves (Sec. 4.1): the kernel of every bf16
// prefill (bf16 operands, fp32 accumulation).
//
// A workgroup walks one (b, h) -- or one segment of it -- in groups of C tokens and
// is split into two halves that run at the same time, one wave of each on every SIMD:
//
//   front-end waves  do all HBM traffic with whole 16-byte-per-lane rows and everything that
//                    needs no state.  Per step: the causal tiles of P^T = phi(K) phi(Q)^T of the
//                    current group (masked by select) with their row sums, and phi(q).z, from
//                    the rows in LDS; then the next group's rows (requested two groups ahead,
//                    the requests in a fixed sequence so that the hardware counter can be waited
//                    on pass by pass) get the feature map on the vector ALUs and go to the LDS
//                    buffer that is not in use; half-way through, the previous group's finished
//                    output rows (staged in LDS by the state waves) are written back out.
//   state waves      hold the state in accumulator registers for the whole sequence: wave w owns
//                    S[:, 32w:32w+32] and z[32w:32w+32].  Per group, for their 32 value channels:
//                    O^T = S^T phi(Q)^T, then S += phi(K)^T V (neither needs the front end), then
//                    O^T += V^T P^T once the scores are there, the row normaliser, the causal
//                    convolution over V, and the result to the LDS staging buffer.
//
// z is carried as the state column of a virtual value channel that is constantly one, so that its
// update (phi(K)^T 1) and its read-out (phi(Q) z) are MFMAs as well; after each update the state
// waves leave z in LDS in operand form for the front end.
//
// Synchronisation per group: one workgroup barrier (C: the current buffer is free, the next one is
// full) and one LDS counter on which the state waves wait for the front end's scores.
//
// GROUPED: the three-branch form of Sec. 4.1 on the same machinery.  The linear branch of a token
// only meets the state as it stood before the token's group (S^T phi(Q)^T over its own normaliser
// phi(q).z + eps, weighted by alpha); inside the group the scores are causal softmax attention on
// the raw rows (logits q.k / sqrt(d)).  The front end therefore also keeps the raw Q and K rows of
// the current group in LDS; to make room, everything that is only read at the start of a group
// (phi(Q), raw Q, raw K) and the output staging exist once instead of twice, and a second LDS
// counter tells the front end when the state waves are done with phi(Q).
#include <type_traits>

#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

namespace {

template <int D, int C, bool GROUPED = false>
struct WsCfg {
  static constexpr int NW = D / 32;          // state waves (and as many front-end waves)
  static constexpr int NT = 2 * NW * 64;
  static constexpr int NLT = NW * 64;        // front-end threads (the upper half of the workgroup)
  static constexpr int TB = C / 32;
  static constexpr int IB = D / 32;
  static constexpr int KSD = D / 16;
  static constexpr int KSC = C / 16;
  static constexpr int NP = C / 16;          // front-end passes: 16 tokens x all columns per pass
  static constexpr int QS = D + 4;           // phi(Q): 8-byte row reads, one row per lane
  static constexpr int KS = D + 16;          // phi(K): transpose reads and 16-byte row reads
  static constexpr int VS = D + 4;           // V: 8-byte row reads by the conv, some transpose reads
  static constexpr int PS = C + 8;           // P: 16-byte row reads
  static constexpr int NTILE = TB * (TB + 1) / 2;
  static constexpr int MAXT = (NTILE + NW - 1) / NW;
  static constexpr int KCMAX = 8;
  static constexpr int SZQ = C * QS * 2, SZK = C * KS * 2;
  static constexpr int BQ = 0;                               // GROUPED: phi(Q) is not part of the row buffers
  static constexpr int BK = GROUPED ? 0 : BQ + SZQ;
  static constexpr int BV = BK + SZK;
  static constexpr int BUF = (BV + (HALO + C) * VS * 2 + 15) / 16 * 16;   // bytes of one row buffer
  static constexpr int OFF_FQ = 2 * BUF;                     // GROUPED: phi(Q), raw Q, raw K of the current group
  static constexpr int OFF_RQ = OFF_FQ + (GROUPED ? SZQ : 0);
  static constexpr int OFF_RK = OFF_RQ + (GROUPED ? SZQ : 0);
  static constexpr int OFF_PN = OFF_RK + (GROUPED ? SZK : 0);
  static constexpr int OFF_DENQ = OFF_PN + C * PS * 2;     // [C] float (room for [NW][C])
  static constexpr int OFF_DENP = OFF_DENQ + NW * C * 4;   // [TB][C] float
  static constexpr int OFF_WL = OFF_DENP + TB * C * 4;     // [KCMAX][D] float, tap-major
  static constexpr int OS = D + 4;           // output staging rows: 8-byte writes, one row per lane
  static constexpr int OFF_OST = OFF_WL + KCMAX * D * 4;   // [2][C][OS] bf16: finished output rows of a group
  static constexpr int OST = C * OS * 2;
  // One staging buffer (emptied at the start of a step, before the signal the state waves wait for) or two (emptied
  // half-way through the fill).  The three-branch form has no room for two; at d = 64 one buffer brings the
  // workgroup under half of a compute unit's LDS, and two workgroups per unit are worth more than the later store.
  static constexpr bool ONE_STAGE = GROUPED || D == 64;
  static constexpr int NOST = ONE_STAGE ? 1 : 2;           // staging buffers
  static constexpr int OFF_ZOP = OFF_OST + NOST * OST;     // [NW][2][16] bf16: z as the MFMA operand of each feature block
  static constexpr int OFF_SYNC = OFF_ZOP + NW * 64;       // the counters of the front-end waves' and the state waves' signals
  static constexpr int TOTAL = OFF_SYNC + 16;
  static constexpr bool FITS = TOTAL <= 160 * 1024;
};

}  // namespace

// STATE_ONLY: the first pass of the segmented form -- a segment's K, V are reduced to its state
// increment (S, z) only: no Q, no scores, no output.
template <int D, int C, int KCM, bool STATE_ONLY, bool GROUPED = false>
__global__ __launch_bounds__(D * 4) void prefill_mfma_ws_kernel(PrefillArgs a) {
  static_assert(!(STATE_ONLY && GROUPED), "the state does not depend on the form");
  using G = WsCfg<D, C, GROUPED>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, hi = lane >> 5;

  uint16_t* Pn = reinterpret_cast<uint16_t*>(smem + G::OFF_PN);
  float* denq = reinterpret_cast<float*>(smem + G::OFF_DENQ);
  float* denp = reinterpret_cast<float*>(smem + G::OFF_DENP);
  float* wl = reinterpret_cast<float*>(smem + G::OFF_WL);
  uint16_t* zop = reinterpret_cast<uint16_t*>(smem + G::OFF_ZOP);
  // A counter that only ever grows: every front-end wave adds one per group once its share of the
  // group's scores, their row sums and phi(q).z is in LDS.
  unsigned* sync_q = reinterpret_cast<unsigned*>(smem + G::OFF_SYNC);
  // GROUPED only: every state wave adds one per group once it has read phi(Q) for the last time.
  unsigned* sync_s = sync_q + 1;
  // GROUPED with eight waves: the two waves that share a query block add one each per group once their
  // largest logits are in LDS.
  unsigned* sync_m = sync_q + 2;
  auto signal = [&](unsigned* ctr) __attribute__((always_inline)) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  };
  // Bounded wait: the signalling waves never wait for anything that depends on the waiting ones
  // before they signal, so the count is always reached; the bound only keeps a logic error from
  // hanging the GPU.  A wait that gives up raises the workgroup's `gave_up` word, and from then on
  // everything the workgroup hands back -- output rows, S, z -- is NaN instead of numbers computed
  // from operands that were not ready: an error shows as such, never as a finite wrong result.
  // a.wait_spins < 0 gives up without looking (the host's way to exercise this path).
  unsigned* gave_up = sync_q + 3;
  auto wait_for = [&](unsigned* ctr, unsigned want) __attribute__((always_inline)) {
    bool reached = false;
    for (int spin = 0; spin <= a.wait_spins; ++spin) {
      if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= want) { reached = true; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    if (!reached && lane == 0) __hip_atomic_store(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };
  auto bufQ = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + (GROUPED ? G::OFF_FQ : bi * G::BUF + G::BQ)); };
  uint16_t* rawQ = reinterpret_cast<uint16_t*>(smem + G::OFF_RQ);   // GROUPED: the current group's rows as they came
  uint16_t* rawK = reinterpret_cast<uint16_t*>(smem + G::OFF_RK);
  auto bufK = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + bi * G::BUF + G::BK); };
  auto bufV = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + bi * G::BUF + G::BV); };   // row r = token r - HALO
  auto bufO = [&](int bi) { return reinterpret_cast<uint16_t*>(smem + G::OFF_OST + (G::ONE_STAGE ? 0 : bi) * G::OST); };

  const int nseg_grid = STATE_ONLY ? a.nseg - 1 : a.nseg;
  // a workgroup is one (b, h, value block) -- or one segment of it; with d_v = d there is one block per head
  // The value blocks of a head read the same q and k rows: without segments they get block indices 8 apart, which
  // the dispatcher places on the same chiplet, so that all but the first of them find the rows in that chiplet's L2
  // (blocks 0..7 = heads 0..7, value block 0; 8..15 = the same heads, value block 1; ...).
  int bhs_idx = blockIdx.x / nseg_grid;
  if (a.m > 1 && nseg_grid == 1 && (a.B * a.H) % 8 == 0) {
    const int bx = blockIdx.x;
    bhs_idx = ((bx / (8 * a.m)) * 8 + (bx & 7)) * a.m + (bx >> 3) % a.m;
  }
  const HeadIndex hx = head_index(a, bhs_idx, D);
  const int seg = blockIdx.x % nseg_grid;
  const int bh = hx.bh, h = hx.h, DVT = hx.dvt;
  const int t_begin = seg * a.seg_len;
  const int t_end = (t_begin + a.seg_len) < a.L ? (t_begin + a.seg_len) : a.L;
  const int nchunks = (t_end - t_begin + C - 1) / C;
  const int64_t base = (int64_t)hx.b * a.sb + (int64_t)h * a.sh;
  const int64_t base_v = (int64_t)hx.b * a.sb_v + (int64_t)h * a.sh_v + (int64_t)hx.blk * D;
  const uint16_t* gq = static_cast<const uint16_t*>(a.q) + base;
  const uint16_t* gk = static_cast<const uint16_t*>(a.k) + base;
  const uint16_t* gv = static_cast<const uint16_t*>(a.v) + base_v;
  uint16_t* gout = static_cast<uint16_t*>(a.out) + base_v;
  constexpr int SLOT = D * D + D;
  float* ws_bh = a.ws + (size_t)hx.bhs * a.nseg * SLOT;
  const uint16_t* staged_hist =
      reinterpret_cast<const uint16_t*>(a.ws + (size_t)a.B * a.H * a.m * a.nseg * SLOT) + (size_t)hx.bhs * HALO * D;
  // this block's corner of the tensors whose rows count value channels
  const int64_t hist_base = (int64_t)bh * (a.Kc - 1) * DVT + (int64_t)hx.blk * D;   // + r * DVT + c
  const int64_t S_base = (int64_t)bh * D * DVT + (int64_t)hx.blk * D;               // + i * DVT + c

  if (tid == 0) { *sync_q = 0u; *sync_s = 0u; *sync_m = 0u; *gave_up = 0u; }
  __syncthreads();                                     // the counters are used before the next barrier

  if (wv >= G::NW) {
    // =============================== front-end waves ============================================
    const int lt = tid - G::NLT;                       // 0 .. NLT-1
    const int lw = wv - G::NW;
    // a pass is 16 tokens; D/8 consecutive lanes carry one whole row (8 columns each), so every
    // load instruction of a wave covers complete rows and every LDS row is written contiguously
    constexpr int LPR = D / 8;                         // lanes per row
    const int r16 = (64 / LPR) * lw + lane / LPR;      // token within a 16-token pass
    const int c0 = 8 * (lane % LPR);                   // first of the 8 columns this thread carries

    const uint32_t loff_b = (uint32_t)(r16 * (int)a.st + c0) * 2u;   // this thread's byte offset inside a pass: q, k
    const uint32_t loff_v = (uint32_t)(r16 * (int)a.st_v + c0) * 2u; // ... v, out

    // Two register sets: group g lives in set g & 1 from the moment it is requested (two groups
    // ahead of its use) until it has been written to LDS.
    //
    // Every load below is issued unconditionally (requests for groups or rows past the end re-read
    // one row that exists; the data is not used), and the main loop is unrolled by two so
    // that the set of each step is fixed at compile time.  The compiler counts outstanding memory
    // operations statically: only with a fixed sequence of them can it wait for exactly the pass
    // that is needed while the requests of the following two groups stay in flight.
    u32x4 rq[2][G::NP], rk[2][G::NP], rv[2][G::NP];
    using Full = std::false_type;
    using Part = std::true_type;
    // Only the last group of a segment can be short; everything about it takes the PARTIAL paths.
    const bool last_partial = (t_end - t_begin) % C != 0;
    // 16 rows of group g: uniform base + 32-bit lane offset
    // part_tag: 0 = K, V and Q; GROUPED fills in two parts and requests with them: 1 = V only, 2 = K and Q
    auto load_pass = [&](int g, int p, auto set_tag, auto partial_tag, auto part_tag) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_tag)::value;
      constexpr bool PARTIAL = decltype(partial_tag)::value;
      constexpr int PART = decltype(part_tag)::value;
      constexpr bool LK = PART != 1, LV = PART != 2, LQ = PART != 1 && !STATE_ONLY;
      const int gc = g < nchunks ? g : nchunks - 1;    // uniform
      const int tok = t_begin + gc * C + 16 * p;       // uniform
      const int64_t off = (int64_t)tok * a.st;
      const char* bk = reinterpret_cast<const char*>(gk + off);
      const char* bv = reinterpret_cast<const char*>(gv + (int64_t)tok * a.st_v);
      const char* bq = reinterpret_cast<const char*>(gq + off);
      // past the last group every lane of a row group re-reads row 0 of the last group: one cache line
      // per request instead of 16 fresh rows
      uint32_t lo = g < nchunks ? loff_b : (uint32_t)c0 * 2u;
      uint32_t lv = g < nchunks ? loff_v : (uint32_t)c0 * 2u;
      if (PARTIAL) {
        const int last = t_end - 1 - tok;              // last row of the segment, relative to this pass
        const int r = (g < nchunks && r16 <= last) ? r16 : (last < 0 ? last : 0);   // a row that exists
        lo = (uint32_t)(r * (int)a.st + c0) * 2u;      // byte offset, may be negative: wraps with the base
        lv = (uint32_t)(r * (int)a.st_v + c0) * 2u;
        if (LK) rk[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bk + (int32_t)lo));
        if (LV) rv[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bv + (int32_t)lv));
        if (LQ) rq[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bq + (int32_t)lo));
      } else {
        if (LK) rk[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bk + lo));
        if (LV) rv[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bv + lv));
        if (LQ) rq[SET][p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(bq + lo));
      }
    };
    // feature map on the 16 rows held in registers, then to buffer bi.  PARTIAL: rows >= nt become
    // zero rows (phi(0) = 1, so they are cleared after the map).
    auto fill_pass = [&](int bi, int p, int nt, auto set_tag, auto partial_tag, auto relu_tag, auto part_tag) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_tag)::value;
      constexpr bool PARTIAL = decltype(partial_tag)::value;
      constexpr bool RELU = decltype(relu_tag)::value;
      constexpr int PART = decltype(part_tag)::value;    // 0: everything; GROUPED: 1 = phi(K) and V, 2 = the rest
      constexpr bool DO_KV = PART != 2, DO_Q = PART != 1 && !STATE_ONLY, DO_RAW = GROUPED && PART != 1;
      const int t = 16 * p + r16;
      const bool ok = !PARTIAL || t < nt;
      auto phi2 = [&](uint32_t x) __attribute__((always_inline)) {
        return RELU ? pack_bf16x2(fmaxf(bf16_lo_to_f32(x), 0.f), fmaxf(bf16_hi_to_f32(x), 0.f))
                    : pack_bf16x2(phi_elu1_max(bf16_lo_to_f32(x)), phi_elu1_max(bf16_hi_to_f32(x)));
      };
      if constexpr (DO_KV) {
        u32x4 kp, vp = rv[SET][p];
#pragma unroll
        for (int i = 0; i < 4; ++i) kp[i] = phi2(rk[SET][p][i]);
        if (PARTIAL) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            kp[i] = ok ? kp[i] : 0u;
            vp[i] = ok ? vp[i] : 0u;
          }
        }
        *reinterpret_cast<u32x4*>(bufK(bi) + t * G::KS + c0) = kp;
        u32x2* vrow = reinterpret_cast<u32x2*>(bufV(bi) + (HALO + t) * G::VS + c0);
        vrow[0] = u32x2{vp[0], vp[1]};
        vrow[1] = u32x2{vp[2], vp[3]};
      }
      if constexpr (DO_Q) {
        u32x4 qp;
#pragma unroll
        for (int i = 0; i < 4; ++i) qp[i] = phi2(rq[SET][p][i]);
        if (PARTIAL) {
#pragma unroll
          for (int i = 0; i < 4; ++i) qp[i] = ok ? qp[i] : 0u;
        }
        u32x2* qrow = reinterpret_cast<u32x2*>(bufQ(bi) + t * G::QS + c0);
        qrow[0] = u32x2{qp[0], qp[1]};
        qrow[1] = u32x2{qp[2], qp[3]};
      }
      if constexpr (DO_RAW) {
        u32x4 rq0 = rq[SET][p], rk0 = rk[SET][p];
        if (PARTIAL) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            rq0[i] = ok ? rq0[i] : 0u;
            rk0[i] = ok ? rk0[i] : 0u;
          }
        }
        u32x2* rqrow = reinterpret_cast<u32x2*>(rawQ + t * G::QS + c0);
        rqrow[0] = u32x2{rq0[0], rq0[1]};
        rqrow[1] = u32x2{rq0[2], rq0[3]};
        *reinterpret_cast<u32x4*>(rawK + t * G::KS + c0) = rk0;
      }
    };
    // finished output rows of group g (left in LDS by the state waves) -> HBM, whole rows per
    // D/8 consecutive lanes, 16 bytes per lane.  PARTIAL: only the rows that exist.
    auto store_group = [&](int g, auto partial_tag) __attribute__((always_inline)) {
      constexpr bool PARTIAL = decltype(partial_tag)::value;
      const int tok0 = t_begin + g * C;
      const int nt = (t_end - tok0) < C ? (t_end - tok0) : C;
      const uint16_t* ost = bufO(g & 1);
      char* bo = reinterpret_cast<char*>(gout + (int64_t)tok0 * a.st_v);
      // a wait of this workgroup gave up (the word was written before the barrier that precedes this store):
      // the rows become NaN.  One uniform branch per group; the path is never taken in a correct run.
      if (__builtin_amdgcn_readfirstlane(*gave_up)) {
#pragma unroll
        for (int p = 0; p < G::NP; ++p) {
          const int t = 16 * p + r16;
          if (!PARTIAL || t < nt)
            __builtin_nontemporal_store(u32x4{0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u, 0x7fc07fc0u},
                                        reinterpret_cast<u32x4*>(bo + (uint32_t)(16 * p) * (uint32_t)a.st_v * 2u + loff_v));
        }
        return;
      }
#pragma unroll
      for (int p = 0; p < G::NP; ++p) {
        const int t = 16 * p + r16;
        const u32x2* src = reinterpret_cast<const u32x2*>(ost + t * G::OS + c0);
        const u32x2 lo = src[0], hi2 = src[1];
        if (!PARTIAL || t < nt)
          __builtin_nontemporal_store(u32x4{lo[0], lo[1], hi2[0], hi2[1]}, reinterpret_cast<u32x4*>(bo + (uint32_t)(16 * p) * (uint32_t)a.st_v * 2u + loff_v));
      }
    };
    // Group g (held in set g & 1) -> buffer g & 1; as each pass leaves the registers, the same pass
    // of group g + 2 is requested from HBM into the freed registers.  STORE: the finished output
    // rows of group g - 2 (always a full group) are written out half-way through, so that no HBM
    // request is younger than half a group when the next fill starts waiting for its rows.
    //
    // GROUPED (STORE means something else there: "wait"): first everything that goes to the row buffer not in
    // use (phi(K), V); then, once every front-end wave has its scores of group g - 1 and every state wave its
    // products with phi(Q) -- normally long since --, the arrays that exist once (phi(Q), raw Q, raw K).
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    auto fill_group = [&](int g, auto set_tag, auto store_tag, auto relu_tag) __attribute__((always_inline)) {
      constexpr bool STORE = decltype(store_tag)::value;
      const int bi = g & 1;
      const int nt = (t_end - (t_begin + g * C)) < C ? (t_end - (t_begin + g * C)) : C;
      const bool fill_part = last_partial && g == nchunks - 1;
      const bool load_part = last_partial && g + 2 >= nchunks - 1;
      if constexpr (GROUPED) {
#pragma unroll
        for (int p = 0; p < G::NP; ++p) {
          if (!fill_part) fill_pass(bi, p, nt, set_tag, Full{}, relu_tag, P1{});
          else fill_pass(bi, p, nt, set_tag, Part{}, relu_tag, P1{});
          if (!load_part) load_pass(g + 2, p, set_tag, Full{}, P1{});
          else load_pass(g + 2, p, set_tag, Part{}, P1{});
        }
        if (STORE) {
          wait_for(sync_q, (unsigned)G::NW * (unsigned)g);
          wait_for(sync_s, (unsigned)G::NW * (unsigned)g);
        }
#pragma unroll
        for (int p = 0; p < G::NP; ++p) {
          if (!fill_part) fill_pass(bi, p, nt, set_tag, Full{}, relu_tag, P2{});
          else fill_pass(bi, p, nt, set_tag, Part{}, relu_tag, P2{});
          if (!load_part) load_pass(g + 2, p, set_tag, Full{}, P2{});
          else load_pass(g + 2, p, set_tag, Part{}, P2{});
        }
      } else {
#pragma unroll
        for (int p = 0; p < G::NP; ++p) {
          if (!STATE_ONLY && STORE && p == G::NP / 2) store_group(g - 2, Full{});
          if (!fill_part) fill_pass(bi, p, nt, set_tag, Full{}, relu_tag, P0{});
          else fill_pass(bi, p, nt, set_tag, Part{}, relu_tag, P0{});
          if (!load_part) load_pass(g + 2, p, set_tag, Full{}, P0{});
          else load_pass(g + 2, p, set_tag, Part{}, P0{});
        }
      }
    };
    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;

    // Scores of group ci from its rows in LDS: the causal 32 x 32 tiles of P^T = phi(K) phi(Q)^T,
    // masked by select, to LDS as P[t][s] in bf16, and the row sums of each tile (of the fp32
    // values) as the scores' part of the normaliser.  Tiles are dealt out over the waves.
    auto scores = [&](int ci) __attribute__((always_inline)) {
      const uint16_t* Qn = bufQ(ci & 1);
      const uint16_t* Kn = bufK(ci & 1);
#pragma unroll
      for (int s = 0; s < G::MAXT; ++s) {
        const int idx = lw + s * G::NW;
        if (idx < G::NTILE) {
          int tb = 0;
          while ((tb + 1) * (tb + 2) / 2 <= idx) ++tb;
          const int sb = idx - tb * (tb + 1) / 2;
          f32x16 acc;
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[r] = 0.f;
          const uint16_t* ka = Kn + (32 * sb + l32) * G::KS + 8 * hi;
          const uint16_t* qb = Qn + (32 * tb + l32) * G::QS + 8 * hi;
          constexpr int HB = G::KSD / 2;   // two batches of K steps
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            bf16x8 ak[HB], bq[HB];
#pragma unroll
            for (int k2 = 0; k2 < HB; ++k2) {
              const int ks = half * HB + k2;
              ak[k2] = lds_row8(ka + 16 * ks);
              bq[k2] = cat4(lds_row4(qb + 16 * ks), lds_row4(qb + 16 * ks + 4));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k2 = 0; k2 < HB; ++k2) acc = mfma(ak[k2], bq[k2], acc);
          }
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
    };
    // GROUPED: the local branch.  Causal softmax weights of the group's raw rows, logits q.k / sqrt(d)
    // (Sec. 3, Eq. 1), in base 2, left in LDS like the other form's scores: unnormalised weights
    // exp2(x - top) as P[t][s] in bf16 and their sums (of the fp32 values) per key tile.  top is the
    // largest logit of the query: lanes l and l + 32 of a tile hold the same query; with eight waves
    // the two key tiles of the second query block are on two waves, which pass each other their
    // largest logits through LDS (a counter of their own tells when both are there), with four waves
    // one wave has both tiles.
    auto scores_local = [&](int ci) __attribute__((always_inline)) {
      static_assert(!GROUPED || G::TB == 2, "two query blocks per group");
      constexpr bool SPLIT = G::NW >= 4;
      constexpr int NA = SPLIT ? 1 : 2;                  // tiles per wave at most
      // SPLIT: wave 0 -> tile (1, 0), wave 1 -> (1, 1), wave 2 -> (0, 0); the last wave has phi(q).z.
      // otherwise: wave 0 -> (1, 0) and (1, 1), wave 1 -> (0, 0) (and phi(q).z)
      const int tb = SPLIT ? (lw <= 1 ? 1 : 0) : (lw == 0 ? 1 : 0);
      const int sb0 = SPLIT && lw == 1 ? 1 : 0;
      const int nsb = SPLIT ? (lw <= 2 ? 1 : 0) : (lw == 0 ? 2 : 1);
      if (nsb == 0) return;
      static_assert(D == 64 || D == 128, "1 / sqrt(d) below");
      constexpr float to_log2 = 1.44269504088896340736f * (D == 64 ? 0.125f : 0.08838834764831845f);
      f32x16 acc[NA];
#pragma unroll
      for (int j = 0; j < NA; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
      const uint16_t* qb = rawQ + (32 * tb + l32) * G::QS + 8 * hi;
      constexpr int HB = G::KSD / 2;   // two batches of K steps
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        bf16x8 ak[NA][HB], bq[HB];
#pragma unroll
        for (int k2 = 0; k2 < HB; ++k2) {
          const int ks = half * HB + k2;
          bq[k2] = cat4(lds_row4(qb + 16 * ks), lds_row4(qb + 16 * ks + 4));
#pragma unroll
          for (int j = 0; j < NA; ++j)
            if (j < nsb) ak[j][k2] = lds_row8(rawK + (32 * (sb0 + j) + l32) * G::KS + 8 * hi + 16 * ks);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k2 = 0; k2 < HB; ++k2)
#pragma unroll
          for (int j = 0; j < NA; ++j)
            if (j < nsb) acc[j] = mfma(ak[j][k2], bq[k2], acc[j]);
      }
      // acc[j][r]: key token s = 32(sb0 + j) + 8(r/4) + 4hi + r%4, query token t = 32tb + l32.
      // Only the diagonal tile has keys later than the query: they become -inf, exp2 of which is 0
      // (later tokens cannot leak).  The scale is positive, so the largest raw product is the largest logit.
      float top = -INFINITY;
#pragma unroll
      for (int j = 0; j < NA; ++j) {
        if (j >= nsb) continue;
        const bool diag = sb0 + j == tb;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int sl = 8 * (r >> 2) + 4 * hi + (r & 3);
          acc[j][r] = (!diag || sl <= l32) ? acc[j][r] : -INFINITY;
          top = fmaxf(top, acc[j][r]);
        }
      }
      top = fmaxf(top, __shfl_xor(top, 32));
      if (SPLIT && tb == 1) {
        float* mx = denq + C;                            // [2][32], behind phi(q).z
        if (lane < 32) mx[32 * sb0 + l32] = top;
        signal(sync_m);
        wait_for(sync_m, 2u * (unsigned)(ci + 1));
        top = fmaxf(top, mx[32 * (1 - sb0) + l32]);
      }
      const float shift = -top * to_log2;                // the diagonal is always seen: top is finite
#pragma unroll
      for (int j = 0; j < NA; ++j) {
        if (j >= nsb) continue;
        const int sb = sb0 + j;
        float rs = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x[e] = __builtin_amdgcn_exp2f(fmaf(acc[j][4 * g + e], to_log2, shift));
            rs += x[e];
          }
          u32x2 pk = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
          *reinterpret_cast<u32x2*>(Pn + (32 * tb + l32) * G::PS + 32 * sb + 8 * g + 4 * hi) = pk;
        }
        rs += __shfl_xor(rs, 32);
        if (lane < 32) denp[sb * C + 32 * tb + l32] = rs;
      }
    };
    // phi(q_t).z for every token of group ci, by the last front-end wave alone (it has the fewest
    // score tiles); z (the state before the group) is read from LDS in operand form, where the
    // state waves left it
    auto q_dot_z = [&](int ci) __attribute__((always_inline)) {
      if (lw != G::NW - 1) return;
      const uint16_t* Qn = bufQ(ci & 1);
      f32x16 acc[G::TB];
#pragma unroll
      for (int tb = 0; tb < G::TB; ++tb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib) {
        bf16x8 bq[G::TB][2];
#pragma unroll
        for (int tb = 0; tb < G::TB; ++tb) {
          const uint16_t* p = Qn + (32 * tb + l32) * G::QS + 32 * ib + 4 * hi;
          bq[tb][0] = cat4(lds_row4(p), lds_row4(p + 8));
          bq[tb][1] = cat4(lds_row4(p + 16), lds_row4(p + 24));
        }
        const uint16_t* zp = zop + (2 * ib + hi) * 16;
        const bf16x8 zb0 = lds_row8(zp), zb1 = lds_row8(zp + 8);
#pragma unroll
        for (int tb = 0; tb < G::TB; ++tb) {
          acc[tb] = mfma(zb0, bq[tb][0], acc[tb]);
          acc[tb] = mfma(zb1, bq[tb][1], acc[tb]);
        }
      }
#pragma unroll
      for (int tb = 0; tb < G::TB; ++tb)
        if (lane < 32) denq[32 * tb + l32] = acc[tb][0];   // every row of the product is the same
    };

    // The conv taps and the value rows just before this segment (earlier tokens, else the incoming history, else
    // zeros) are requested ahead of the first two groups and stored behind those requests: unconditional loads
    // (an address that exists where there is nothing to read), so that a short sequence does not pay one round
    // trip to memory per loop iteration before its first group is even asked for.
    constexpr int TAP_IT = (KCM * D + G::NLT - 1) / G::NLT;
    constexpr int HALO_IT = HALO * D / G::NLT;
    float tap_reg[TAP_IT];
    uint16_t halo_reg[HALO_IT];
    bool halo_ok[HALO_IT];
    auto small_inputs_request = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int mth = 0; mth < TAP_IT; ++mth) {
        const int e = lt + G::NLT * mth;
        const int j = e / D, cc = e % D;
        tap_reg[mth] = a.conv_w[((size_t)h * DVT + hx.blk * D + cc) * a.Kc + (j < a.Kc ? j : 0)];
      }
#pragma unroll
      for (int mth = 0; mth < HALO_IT; ++mth) {
        const int e = lt + G::NLT * mth;
        const int r = e / D, cc = e % D;
        const int tok = t_begin - HALO + r;
        const uint16_t* src = gv + (int64_t)t_begin * a.st_v + cc;   // exists: the segment is not empty
        bool ok = false;
        if (tok >= 0) { src = gv + (int64_t)tok * a.st_v + cc; ok = true; }
        else if (a.hist_in && a.nseg > 1) { src = staged_hist + (size_t)(HALO + tok) * D + cc; ok = true; }
        else if (a.hist_in && a.Kc - 1 + tok >= 0) {
          src = static_cast<const uint16_t*>(a.hist_in) + hist_base + (int64_t)(a.Kc - 1 + tok) * DVT + cc;
          ok = true;
        }
        halo_reg[mth] = *src;
        halo_ok[mth] = ok;
      }
    };
    auto small_inputs_store = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int mth = 0; mth < TAP_IT; ++mth) {
        const int e = lt + G::NLT * mth;
        if (e < KCM * D) wl[e] = (e / D < a.Kc && !a.no_conv) ? tap_reg[mth] : 0.f;
      }
#pragma unroll
      for (int mth = 0; mth < HALO_IT; ++mth) {
        const int e = lt + G::NLT * mth;
        bufV(0)[(e / D) * G::VS + e % D] = halo_ok[mth] ? halo_reg[mth] : (uint16_t)0;
      }
    };
    // The whole walk, once per feature map: the map is a property of the launch, and choosing it out here
    // keeps the loop of either map free of selects and branches on it.
    auto walk = [&](auto relu_tag) __attribute__((always_inline)) {
      if (nchunks > 0) {
        if (!STATE_ONLY) small_inputs_request();
#pragma unroll
        for (int p = 0; p < G::NP; ++p) load_pass(0, p, Set0{}, Part{}, P0{});
#pragma unroll
        for (int p = 0; p < G::NP; ++p) load_pass(1, p, Set1{}, Part{}, P0{});
        if (!STATE_ONLY) small_inputs_store();
        fill_group(0, Set0{}, std::false_type{}, relu_tag);
      }
      __syncthreads();                                   // buffer 0 is full, z is in LDS

      // One step of the front end.  First the scores and phi(q).z of group ci, which the state waves
      // need a little later (they start with the products that involve the state only); then, while
      // the state waves work on group ci, group ci + 1 is filled, group ci + 3 requested and group
      // ci - 1 stored.
      auto step = [&](int ci, auto set_tag, auto store_tag) __attribute__((always_inline)) {
        if (!STATE_ONLY) {
          // the one staging buffer: group ci - 1 leaves before the state waves may write group ci
          // (they wait for this step's signal first)
          if constexpr (G::ONE_STAGE) {
            if (decltype(store_tag)::value) store_group(ci - 1, Full{});
          }
          if constexpr (GROUPED) scores_local(ci);
          else scores(ci);
          q_dot_z(ci);
          signal(sync_q);
          // the last HALO value rows of group ci become the rows before group ci + 1
          if (lt < HALO * D / 8) {
            const int r = lt / (D / 8), piece = 8 * (lt % (D / 8));
            const u32x2* src = reinterpret_cast<const u32x2*>(bufV(ci & 1) + (C + r) * G::VS + piece);
            u32x2* dst = reinterpret_cast<u32x2*>(bufV((ci + 1) & 1) + r * G::VS + piece);
            const u32x2 t0 = src[0], t1 = src[1];
            dst[0] = t0; dst[1] = t1;
          }
        }
        if constexpr (GROUPED) {
          // phi(Q), raw Q and raw K exist once: group ci + 1 may replace them when every front-end wave
          // has its scores of group ci and every state wave its products with phi(Q) (the fill waits)
          fill_group(ci + 1, set_tag, std::true_type{}, relu_tag);
        } else if constexpr (G::ONE_STAGE) {
          fill_group(ci + 1, set_tag, std::false_type{}, relu_tag);   // the store has happened already
        } else {
          fill_group(ci + 1, set_tag, store_tag, relu_tag);
        }
        __syncthreads();                                 // barrier C
      };
      // store_tag of a step: GROUPED, group ci - 1 exists (ci > 0); otherwise, group ci - 1 exists and
      // is stored half-way through the fill (ci > 0, too)
      int ci = 0;
      if (nchunks > 1) { step(0, Set1{}, std::false_type{}); ci = 1; }
      for (; ci + 2 < nchunks; ci += 2) {                // ci is odd here: group ci + 1 is even
        step(ci, Set0{}, std::true_type{});
        step(ci + 1, Set1{}, std::true_type{});
      }
      if (ci >= 1 && ci + 1 < nchunks) { step(ci, Set0{}, std::true_type{}); ++ci; }
      if (nchunks > 0) {                                 // ci == nchunks - 1: nothing left to fill
        if (!STATE_ONLY) {
          if constexpr (G::ONE_STAGE) {
            if (ci > 0) store_group(ci - 1, Full{});
          }
          if constexpr (GROUPED) scores_local(ci);
          else scores(ci);
          q_dot_z(ci);
          signal(sync_q);
          if (!G::ONE_STAGE && ci > 0) store_group(ci - 1, Full{});
        }
        __syncthreads();                                 // barrier C
      }
      if (!STATE_ONLY && nchunks > 0) {
        if (last_partial) store_group(nchunks - 1, Part{});
        else store_group(nchunks - 1, Full{});
      }
    };
    if (a.relu) walk(std::true_type{});
    else walk(std::false_type{});
    return;
  }

  // ================================= state waves ===================================================
  const int w = wv;
  const int cw = 32 * w + l32;             // the channel this lane owns in the state accumulators

  // Sacc[ib][r] = S[32ib + 8(r/4) + 4hi + r%4][cw];  Zacc[r] = z[32w + 8(r/4) + 4hi + r%4] (every lane)
  f32x16 Sacc[G::IB], Zacc;
  {
    const float* Ssrc = nullptr;
    const float* zsrc = nullptr;
    int srow = D;                                      // row length of the source: a workspace slot, or the caller's S
    if (STATE_ONLY) {}
    else if (a.nseg > 1) { Ssrc = ws_bh + (size_t)seg * SLOT; zsrc = Ssrc + D * D; }
    else if (a.S_in) { Ssrc = a.S_in + S_base; zsrc = a.z_in + (size_t)bh * D; srow = DVT; }
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
        Sacc[ib][r] = Ssrc ? Ssrc[(size_t)i * srow + cw] : 0.f;
      }
#pragma unroll
    for (int r = 0; r < 16; ++r) Zacc[r] = zsrc ? zsrc[32 * w + 8 * (r >> 2) + 4 * hi + (r & 3)] : 0.f;
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  // z of the state as it stands, as the bf16 MFMA operand of this wave's feature block, for the
  // front-end waves' phi(q).z of the next group
  auto publish_z = [&]() __attribute__((always_inline)) {
    if (l32 == 0) {
      uint16_t* zp = zop + (2 * w + hi) * 16;
      *reinterpret_cast<bf16x8*>(zp) = pack8(Zacc, 0);
      *reinterpret_cast<bf16x8*>(zp + 8) = pack8(Zacc, 8);
    }
  };
  if (!STATE_ONLY) publish_z();

  __syncthreads();                                     // buffer 0 is full, the conv taps and z are in LDS

  // conv taps of this lane's 16 output channels (32w + 8g + 4hi + e), kept in registers when few
  constexpr bool W_REGS = KCM <= 3 && D == 64;   // D = 128: the registers do not suffice
  f32x4 wreg[W_REGS ? KCM : 1][4];
  if (W_REGS) {
#pragma unroll
    for (int j = 0; j < (W_REGS ? KCM : 1); ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) wreg[j][g] = *reinterpret_cast<const f32x4*>(wl + j * D + 32 * w + 8 * g + 4 * hi);
  }

  // LDS reads are issued in batches ahead of the MFMAs that consume them (the fences keep the
  // compiler from sinking each read next to its use, which would expose the full LDS latency
  // once per MFMA).
#define LINATTN_FENCE() __builtin_amdgcn_sched_barrier(0)

  // One group of C tokens.  A short last group needs no special case here: its missing rows are
  // zero rows in LDS, and the front-end waves do not store their outputs.
  auto group = [&](int ci) __attribute__((always_inline)) {
    const uint16_t* Qn = bufQ(ci & 1);
    const uint16_t* Kn = bufK(ci & 1);
    const uint16_t* Vn = bufV(ci & 1);
    // ---- this wave's channels ------------------------------------------------------------------------
    // vf[ks]: lanes <-> channels 32w + l32, registers <-> tokens 16ks + 8hi + 0..7
    bf16x8 vf[G::KSC];
#pragma unroll
    for (int ks = 0; ks < G::KSC; ++ks) vf[ks] = tr_operand(Vn + HALO * G::VS, G::VS, 16 * ks, 32 * w, lane);
    auto update_state = [&]() __attribute__((always_inline)) {
    // S += phi(K)^T V for this wave's channels, z += phi(K)^T 1 for this wave's features;
    // the phi(K)^T operands of feature block ib + 1 are requested while block ib is multiplied
    {
      bf16x8 kt[2][G::KSC];
#pragma unroll
      for (int ks = 0; ks < G::KSC; ++ks) kt[0][ks] = tr_operand(Kn, G::KS, 16 * ks, 0, lane);
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib) {
        if (ib + 1 < G::IB) {
#pragma unroll
          for (int ks = 0; ks < G::KSC; ++ks) kt[(ib + 1) & 1][ks] = tr_operand(Kn, G::KS, 16 * ks, 32 * (ib + 1), lane);
        }
        LINATTN_FENCE();
#pragma unroll
        for (int ks = 0; ks < G::KSC; ++ks) {
          Sacc[ib] = mfma(kt[ib & 1][ks], vf[ks], Sacc[ib]);
          if (ib == w) Zacc = mfma(kt[ib & 1][ks], ones, Zacc);
        }
      }
    }
    };
    if constexpr (!STATE_ONLY) {
    // First the part that needs the state only, S^T phi(Q)^T, for every token block; the front-end
    // waves compute the scores of this group meanwhile.
    // o[tb][r] = O[token 32tb + l32][channel 32w + 8(r/4) + 4hi + r%4]
    f32x16 o[G::TB];
#pragma unroll
    for (int tb = 0; tb < G::TB; ++tb) {
      // register r of S holds feature 32ib + 8(r/4) + 4hi + r%4, so the phi(Q) operand takes
      // features {16h2 + 4hi + 0..3, 16h2 + 8 + 4hi + 0..3} of block ib for MFMA step h2
      bf16x8 qB[2 * G::IB];
      const uint16_t* qb = Qn + (32 * tb + l32) * G::QS + 4 * hi;
#pragma unroll
      for (int x = 0; x < 2 * G::IB; ++x) qB[x] = cat4(lds_row4(qb + 16 * x), lds_row4(qb + 16 * x + 8));
      LINATTN_FENCE();
#pragma unroll
      for (int r = 0; r < 16; ++r) o[tb][r] = 0.f;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) o[tb] = mfma(pack8(Sacc[ib], 8 * h2), qB[2 * ib + h2], o[tb]);
    }
    if constexpr (GROUPED) signal(sync_s);   // phi(Q) of this group has been read for the last time
    // the state update needs nothing from the front end either: it goes before the wait for the scores
    update_state();
    wait_for(sync_q, (unsigned)G::NW * (unsigned)(ci + 1));   // scores, their row sums and phi(q).z are in LDS
    publish_z();   // only now: the front end has read the previous z by the time it signals
#pragma unroll
    for (int tb = 0; tb < G::TB; ++tb) {
      const int t = 32 * tb + l32;
      // the scores of this token block (lane <-> query token) and the parts of the normaliser
      bf16x8 pB[2 * G::TB];
      const uint16_t* pb = Pn + t * G::PS + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < 2 * (tb + 1); ++ks) pB[ks] = lds_row8(pb + 16 * ks);
      float dpart[1 + G::TB];
      dpart[0] = denq[t];
#pragma unroll
      for (int sb = 0; sb <= tb; ++sb) dpart[1 + sb] = denp[sb * C + t];
      const uint16_t* vrow = Vn + (HALO + t) * G::VS + 32 * w + 4 * hi;
      const float* wrow = wl + 32 * w + 4 * hi;
      // conv inputs of channel group g are requested one group ahead of their use (with many
      // taps the registers for that do not suffice: then just before)
      constexpr int CB = KCM > 5 ? 1 : 2;
      u32x2 xv[CB][KCM];
      f32x4 wv[CB][W_REGS ? 1 : KCM];
      auto conv_request = [&](int g) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < KCM; ++j) {
          xv[g % CB][j] = *reinterpret_cast<const u32x2*>(vrow - j * G::VS + 8 * g);
          if (!W_REGS) wv[g % CB][j] = *reinterpret_cast<const f32x4*>(wrow + j * D + 8 * g);
        }
      };
      conv_request(0);
      LINATTN_FENCE();
      float den;
      if constexpr (GROUPED) {
        // two normalisers: the linear branch (so far alone in o) over eps + phi(q).z, the local branch
        // over the sum of its weights.  The first is applied here, times the second, so that one
        // division by the second at the end serves both.  A linear branch with nothing before it
        // (denominator exactly zero) contributes nothing.
        den = 0.f;
#pragma unroll
        for (int sb = 0; sb <= tb; ++sb) den += dpart[1 + sb];
        const float gden = a.eps + dpart[0];
        const float f = gden != 0.f ? a.alpha * den * __builtin_amdgcn_rcpf(gden) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) o[tb][r] = gden != 0.f ? o[tb][r] * f : 0.f;
      }
#pragma unroll
      for (int ks = 0; ks < 2 * (tb + 1); ++ks) o[tb] = mfma(vf[ks], pB[ks], o[tb]);
      if constexpr (!GROUPED) {
        // the normaliser: eps + phi(q).z + the scores' row sums
        den = a.eps + dpart[0];
#pragma unroll
        for (int sb = 0; sb <= tb; ++sb) den += dpart[1 + sb];
      }
      const float inv = __builtin_amdgcn_rcpf(den);
      // normalise, add the causal conv, stage the row for the front-end waves to store
      uint16_t* orow = bufO(ci & 1) + t * G::OS + 32 * w + 4 * hi;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (CB == 2 && g + 1 < 4) conv_request(g + 1);
        if (CB == 1 && g > 0) conv_request(g);
        float u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KCM; ++j) {
          const f32x4 wv4 = W_REGS ? wreg[W_REGS ? j : 0][g] : wv[g % CB][W_REGS ? 0 : j];
          const u32x2 x = xv[g % CB][j];
          u[0] = fmaf(wv4[0], bf16_lo_to_f32(x[0]), u[0]);
          u[1] = fmaf(wv4[1], bf16_hi_to_f32(x[0]), u[1]);
          u[2] = fmaf(wv4[2], bf16_lo_to_f32(x[1]), u[2]);
          u[3] = fmaf(wv4[3], bf16_hi_to_f32(x[1]), u[3]);
        }
        const u32x2 y = {pack_bf16x2(fmaf(o[tb][4 * g], inv, u[0]), fmaf(o[tb][4 * g + 1], inv, u[1])),
                         pack_bf16x2(fmaf(o[tb][4 * g + 2], inv, u[2]), fmaf(o[tb][4 * g + 3], inv, u[3]))};
        *reinterpret_cast<u32x2*>(orow + 8 * g) = y;
      }
    }
    } else {
      update_state();
    }
    __syncthreads();   // C: this buffer may be refilled, the other one is complete
  };

  for (int ci = 0; ci < nchunks; ++ci) group(ci);
#undef LINATTN_FENCE

  // ---- hand the state over ---------------------------------------------------------------------------
  if (STATE_ONLY) {
    // this segment's increment goes to the slot that the prefix sum turns into the next segment's start
    float* Sdst = ws_bh + (size_t)(seg + 1) * SLOT;
#pragma unroll
    for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
        Sdst[(size_t)i * D + cw] = Sacc[ib][r];
      }
    if (l32 == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) Sdst[D * D + 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3)] = Zacc[r];
    }
  } else if (seg == a.nseg - 1) {
    if (__builtin_amdgcn_readfirstlane(*gave_up)) {      // a wait gave up (written before the last barrier): no numbers
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) Sacc[ib][r] = __builtin_nanf("");
#pragma unroll
      for (int r = 0; r < 16; ++r) Zacc[r] = __builtin_nanf("");
    }
    if (a.S_out) {
      float* Sdst = a.S_out + S_base;
#pragma unroll
      for (int ib = 0; ib < G::IB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 32 * ib + 8 * (r >> 2) + 4 * hi + (r & 3);
          Sdst[(size_t)i * DVT + cw] = Sacc[ib][r];
        }
    }
    if (a.z_out && l32 == 0 && hx.blk == 0) {           // z is the same in every value block: the first one hands it back
#pragma unroll
      for (int r = 0; r < 16; ++r) a.z_out[(size_t)bh * D + 32 * w + 8 * (r >> 2) + 4 * hi + (r & 3)] = Zacc[r];
    }
    if (a.hist_out && tid < D) {
      // last Kc-1 value rows of (history ++ sequence); one thread per channel reads all its rows before it
      // writes any, so an aliased hist_in is read before it is overwritten (with segments the staged copy is read)
      const uint16_t* hin = static_cast<const uint16_t*>(a.hist_in);
      uint16_t* hout = static_cast<uint16_t*>(a.hist_out) + hist_base;
      uint16_t hrow[HALO];                                 // all rows requested before the first one is stored
#pragma unroll
      for (int r = 0; r < HALO; ++r) {
        const int tok = a.L - (a.Kc - 1) + r;
        hrow[r] = 0;
        if (r < a.Kc - 1) {
          if (tok >= 0) hrow[r] = gv[(int64_t)tok * a.st_v + tid];
          else if (hin) hrow[r] = a.nseg > 1 ? staged_hist[(size_t)(HALO + tok) * D + tid]
                                             : hin[hist_base + (int64_t)(a.Kc - 1 + tok) * DVT + tid];
        }
      }
#pragma unroll
      for (int r = 0; r < HALO; ++r)
        if (r < a.Kc - 1) hout[(size_t)r * DVT + tid] = hrow[r];
    }
  }
}

template <int D, int C, int KCM, bool STATE_ONLY, bool GROUPED = false>
static hipError_t launch_ws(const PrefillArgs& a, hipStream_t st) {
  using G = WsCfg<D, C, GROUPED>;
  static_assert(G::FITS, "two row buffers must fit in the 160 KB of LDS");
  auto kern = prefill_mfma_ws_kernel<D, C, KCM, STATE_ONLY, GROUPED>;
  hipError_t e = LINATTN_MAX_LDS_ONCE(kern, G::TOTAL);
  if (e != hipSuccess) return e;
  const int segs = STATE_ONLY ? a.nseg - 1 : a.nseg;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.B * a.H * a.m * segs)), dim3(G::NT), G::TOTAL, st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_ws_k(const PrefillArgs& a, bool state_only, bool grouped, hipStream_t st) {
  constexpr int C = 64;   // tokens per group
  if (state_only) return launch_ws<D, C, 3, true>(a, st);   // the conv taps play no part in the state
  if (grouped) {
    if (a.Kc <= 3) return launch_ws<D, C, 3, false, true>(a, st);
    if (a.Kc <= 5) return launch_ws<D, C, 5, false, true>(a, st);
    return launch_ws<D, C, 8, false, true>(a, st);
  }
  if (a.Kc <= 3) return launch_ws<D, C, 3, false>(a, st);
  if (a.Kc <= 5) return launch_ws<D, C, 5, false>(a, st);
  return launch_ws<D, C, 8, false>(a, st);
}

// One pass of a prefill call over all its segments.  state_only: the first pass of the segmented
// form (segment increments into a.ws); otherwise the full pass (segment start states must be in a.ws).
// grouped: the three-branch form with 64-token groups (a.alpha weighs its linear branch).
hipError_t launch_prefill_mfma_ws(const PrefillArgs& a, int d, bool state_only, bool grouped, hipStream_t st) {
  return d == 128 ? launch_ws_k<128>(a, state_only, grouped, st) : launch_ws_k<64>(a, state_only, grouped, st);
}

}  // namespace linattn
