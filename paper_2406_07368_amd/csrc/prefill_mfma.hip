// Prefill of bf16 inputs (Sec. 4.1): the launch plan around the matrix-core kernel.
//
// The kernel itself (prefill_mfma_ws.hip) walks one (b, h) -- or one segment of its
// sequence -- group by group with the state in registers.  When B*H alone cannot fill
// the chip the sequence axis is cut into segments: a first pass reduces each segment's
// K, V to its state increment, a prefix sum over the segments (here) turns the
// increments into segment start states, and the full pass starts every segment from its
// prefix.
#include "common.h"
#include "kernels.h"
#include "mfma_util.h"

namespace linattn {

// Prefix sum over the segments of one (b, h): slot 0 <- incoming state, slot g <- slot g-1 +
// increment of segment g-1.  Also stages the incoming history so that the second pass never
// reads hist_in (which hist_out may alias).  One thread per state element walks the segments.
template <int D>
__global__ __launch_bounds__(256) void segment_scan_kernel(PrefillArgs a) {
  constexpr int SLOT = D * D + D;
  const HeadIndex hx = head_index(a, blockIdx.y, D);      // one (b, h, value block)
  const int bh = hx.bh;
  const int e = blockIdx.x * 256 + threadIdx.x;
  float* ws_bh = a.ws + (size_t)hx.bhs * a.nseg * SLOT;
  if (e < SLOT) {
    float run = 0.f;
    if (a.S_in) run = e < D * D ? a.S_in[(size_t)bh * D * hx.dvt + (size_t)(e / D) * hx.dvt + hx.blk * D + e % D]
                                : a.z_in[(size_t)bh * D + (e - D * D)];
    ws_bh[e] = run;
    // sixteen segments at a time: all their increments are requested before the first is added (read, add and
    // write back one by one, every segment would pay a trip to memory of its own: the compiler may not move a
    // load across the store before it)
    for (int g0 = 1; g0 < a.nseg; g0 += 16) {
      float inc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int g = g0 + i < a.nseg ? g0 + i : a.nseg - 1;   // past the end: the last one again, not used
        inc[i] = ws_bh[(size_t)g * SLOT + e];
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        run += inc[i];
        if (g0 + i < a.nseg) ws_bh[(size_t)(g0 + i) * SLOT + e] = run;
      }
    }
  }
  if (a.hist_in && e < HALO * D) {
    uint16_t* staged = reinterpret_cast<uint16_t*>(a.ws + (size_t)a.B * a.H * a.m * a.nseg * SLOT) + (size_t)hx.bhs * HALO * D;
    const int r = e / D, cc = e % D;           // staged row r holds token r - HALO
    const int hr = (a.Kc - 1) - HALO + r;      // row of the incoming history
    staged[e] = hr >= 0 ? static_cast<const uint16_t*>(a.hist_in)[((size_t)bh * (a.Kc - 1) + hr) * hx.dvt + hx.blk * D + cc] : (uint16_t)0;
  }
}

// Segments per (b, h): as many as keep all workgroups of the second pass resident at once (at d = 128 one per compute
// unit: a workgroup takes most of a unit's LDS, so the 257th would wait for a whole segment; at d = 64 two), with at
// least 2 groups per segment, and no segments at all for sequences of fewer than 8 groups, where a second launch costs
// more than it saves.
int prefill_mfma_pick_segments(int BH, int L, int chunk, int d) {
  const int groups = (L + 63) / 64;            // the kernel walks groups of 64 tokens whatever `chunk` says
  const int chunks = (L + chunk - 1) / chunk;  // segments start on multiples of `chunk`
  int want = (d == 64 ? 512 : 256) / BH;
  int most = groups >= 8 ? groups / 2 : 1;
  if (most > chunks) most = chunks;
  if (want > most) want = most;
  if (want > 64) want = 64;
  return want < 1 ? 1 : want;
}

size_t prefill_mfma_workspace_bytes(int BH, int d, int nseg) {
  if (nseg <= 1) return 0;
  return (size_t)BH * nseg * ((size_t)d * d + d) * sizeof(float) + (size_t)BH * HALO * d * sizeof(uint16_t);
}

// Segments of the 256-token three-branch kernel: a workgroup takes all of a compute unit, so as many as fill the
// chip, down to one group per segment (the groups of a segment are walked one after the other).
int prefill_grouped256_pick_segments(int BH, int L) {
  const int groups = (L + 255) / 256;
  int want = 256 / BH;
  if (want > groups) want = groups;
  if (want > 64) want = 64;
  return want < 1 ? 1 : want;
}

// ... whose running state lives in its workspace slot: one slot per (b, h, segment) even without segments
size_t prefill_grouped256_workspace_bytes(int BH, int d, int nseg) {
  return (size_t)BH * nseg * ((size_t)d * d + d) * sizeof(float) + (size_t)BH * HALO * d * sizeof(uint16_t);
}

// The group size only blocks the computation; the result does not depend on it (the in-group
// part is the exact masked product).  A requested group of 128 tokens is walked as two steps of
// 64: two 128-token row buffers do not fit in LDS, and larger groups only add in-group MFMA work
// per token on this design.  Segment boundaries stay multiples of the requested size.
// grouped: the three-branch form, whose groups are exactly `chunk` tokens, 64 or 256 (segments start on
// group boundaries, so the first pass and the prefix sum are the same for both forms; groups of 256 have a
// kernel of their own for the full pass).
hipError_t launch_segment_scan(const PrefillArgs& a, int d, hipStream_t st) {
  const int BH = a.B * a.H * a.m;             // heads the kernels see: one per value block
  const int slot = d * d + d;
  const dim3 grid((unsigned)((slot + 255) / 256), (unsigned)BH);
  if (d == 128) hipLaunchKernelGGL((segment_scan_kernel<128>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((segment_scan_kernel<64>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_prefill_mfma(const PrefillArgs& a, int d, int chunk, bool grouped, hipStream_t st) {
  hipError_t e;
  if (a.nseg > 1) {
    if ((e = launch_prefill_mfma_ws(a, d, true, false, st)) != hipSuccess) return e;
    if ((e = launch_segment_scan(a, d, st)) != hipSuccess) return e;
  }
  if (grouped && chunk == 256) return launch_prefill_grouped256(a, d, st);
  return launch_prefill_mfma_ws(a, d, false, grouped, st);
}

}  // namespace linattn
