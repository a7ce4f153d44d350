// The two streaming passes over every element: the fused neighbour-averaging +
// momentum-SGD update (Section 3, Eq. 2 with the last received neighbour values
// of Section 4), which also accumulates the squared drift || x - xhat ||^2 that the
// next iteration's trigger test needs, and a stand-alone drift-norm pass.
//
// One workgroup (256 threads, one float4 per thread) owns one 1024-element sweep of
// one chunk of one worker: the launch shape that streams best on MI355X; with Top-K
// messages to apply it owns two consecutive sweeps, which halves the per-workgroup
// cost of that work.  HBM-bound: 5 reads + 2 writes of 4 bytes per element.
//
// Top-K messages are applied here, where the dense arrays pass through registers
// anyway: the sender's own message patches xhat (only the sent entries count as
// communicated), the left and right neighbours' messages patch the two mailboxes
// (the receiving end of the put, Section 6).  A message slice is scattered into an
// LDS window first, so that global accesses stay 16-byte wide and coalesced, and a
// float4 is written back only if its 64-byte group changed.
#include "trigger_device.h"

// Build-time variants of the Top-K message handling, kept so that the measurements behind the
// defaults can be repeated (EVG_EXTRA_FLAGS="-DEVG_PATCH_WINDOWS=2" python -m paper_2103_07454_amd.build):
//   EVG_PATCH_WINDOWS  LDS windows the three messages of a workgroup are scattered into: 3 = one each
//                      (default: one barrier pair), 2 = two used in turn, 1 = one after the other
//                      (less LDS, more barriers; measured 1-2 % slower);
//   EVG_UPDATE_SPW     sweeps per workgroup when messages are applied: 2 (default) or 1 (5-7 % slower).
// Results are identical in every variant.
#ifndef EVG_PATCH_WINDOWS
#define EVG_PATCH_WINDOWS 3
#endif
#ifndef EVG_UPDATE_SPW
#define EVG_UPDATE_SPW 2
#endif

namespace evg {

__device__ __forceinline__ float4 ld4(const float* p) { return ld4s(p); }

// Squared drift of the first nv lanes of a float4 pair, added in lane order.
__device__ __forceinline__ void drift_acc(double& acc, const float x[4], const float h[4], uint32_t nv) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if ((uint32_t)i < nv) {
      const float e = x[i] - h[i];
      acc += (double)e * (double)e;
    }
  }
}

// Sum of squares of the first nv lanes, added in lane order.
__device__ __forceinline__ void square_acc(double& acc, const float x[4], uint32_t nv) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if ((uint32_t)i < nv) acc += (double)x[i] * (double)x[i];
}

// NORMDIFF: the trigger compares ||x|| with ||xhat||: two sums instead of the drift's.
template <bool NORMDIFF>
__global__ __launch_bounds__(kThreads) void k_norm(Tables T) {
  __shared__ double ws[4];
  const uint32_t c = blockIdx.x / T.SW, sub = blockIdx.x % T.SW, r = blockIdx.y;
  const ChunkDesc cd = T.chunks[c];
  const size_t base = (size_t)r * T.Npad + cd.off;
  const uint32_t e = sub * kSweep + threadIdx.x * kLaneElems;
  double acc = 0.0, acc_hat = 0.0;
  if (e < cd.len) {
    const float4 x4 = ld4(T.x + base + e), h4 = ld4(T.xhat + base + e);
    const float xa[4] = {x4.x, x4.y, x4.z, x4.w}, ha[4] = {h4.x, h4.y, h4.z, h4.w};
    const uint32_t nv = cd.len - e < 4u ? cd.len - e : 4u;
    if (NORMDIFF) { square_acc(acc, xa, nv); square_acc(acc_hat, ha, nv); }
    else drift_acc(acc, xa, ha, nv);
  }
  const size_t slot = ((size_t)r * T.C + c) * T.SW + sub;
  const double total = block_sum(acc, ws);
  if (threadIdx.x == 0) T.partials_out[slot] = total;
  if (NORMDIFF) {
    const double total_hat = block_sum(acc_hat, ws);
    if (threadIdx.x == 0) T.partials_hat_out[slot] = total_hat;
  }
}

// One source of a sparse patch for this workgroup's window of SPW sweeps: the slice
// of worker `src`'s message that chunk c, sweeps sub0 .. sub0+SPW-1 produced (empty if
// `src` sent no Top-K message for this tensor in this iteration).
struct Slice { uint32_t at; uint32_t n; };   // P*Ktot and P*C*(SW+1) fit 32 bits (checked at init)

template <int SPW>
__device__ __forceinline__ Slice message_slice(const Tables& T, uint32_t src, uint32_t layer, uint32_t c,
                                               uint32_t sub0, uint32_t msg_off) {
  Slice s;
  const uint32_t w = (src * T.C + c) * (T.SW + 1) + sub0;
  const uint32_t lo = T.chunk_sub[w], hi = T.chunk_sub[w + SPW];
  s.at = src * T.Ktot + msg_off + lo;
  s.n = T.fired[src * T.L + layer] == 2 ? hi - lo : 0u;
  return s;
}

// Scatters a slice into its LDS window (values + one bit per element).
template <int SPW>
__device__ __forceinline__ void scatter_slice(const Tables& T, const Slice& s, uint32_t j_lo, float* pv,
                                              uint32_t* pm) {
  for (uint32_t q = threadIdx.x; q < s.n; q += kThreads) {
    const uint32_t loc = T.msg_idx[s.at + q] - j_lo;
    if (loc < (uint32_t)(SPW * kSweep)) {
      pv[loc] = T.msg_val[s.at + q];
      atomicOr(&pm[loc >> 5], 1u << (loc & 31u));
    }
  }
}

// Replaces the lanes of this thread's float4 in sweep u of the window by the window's
// entries.  Returns the change mask of the aligned 64-byte group (4 neighbouring float4s)
// the float4 belongs to: write-back is decided per group, because scattered 16-byte
// writes cost far more in HBM than the few unchanged bytes a full 64-byte line carries.
__device__ __forceinline__ uint32_t take_patch(const float* pv, const uint32_t* pm, uint32_t u, float a[4]) {
  const uint32_t l0 = u * kSweep + threadIdx.x * kLaneElems;   // first element of the float4
  const uint32_t g0 = l0 & ~15u;                               // first element of its 64-byte group
  const uint32_t group = (pm[g0 >> 5] >> (g0 & 31u)) & 0xFFFFu;   // (32-byte groups measured 19 % slower)
  const uint32_t bits = (group >> (l0 & 15u)) & 0xFu;
  const float4 v = *reinterpret_cast<const float4*>(pv + l0);   // unwritten lanes hold garbage: masked
  a[0] = (bits & 1u) ? v.x : a[0];
  a[1] = (bits & 2u) ? v.y : a[1];
  a[2] = (bits & 4u) ? v.z : a[2];
  a[3] = (bits & 8u) ? v.w : a[3];
  return group;
}

// Workgroup sums of SPW values at once (one barrier pair); each in the association
// order of block_sum.  `ws` is 4 * SPW doubles of LDS.
template <int SPW>
__device__ __forceinline__ void block_sums(const double v[SPW], double* ws, double total[SPW]) {
#pragma unroll
  for (int u = 0; u < SPW; ++u) {
    const double s = wave_sum(v[u]);
    if (lane_id() == 0) ws[u * 4 + wave_id()] = s;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < SPW; ++u) total[u] = ((ws[u * 4] + ws[u * 4 + 1]) + ws[u * 4 + 2]) + ws[u * 4 + 3];
  __syncthreads();
}

// DIST: 0 normal (one Philox block per float4), 1 Student-t(3) (two blocks per float4).
// GRADBUF: gradients come from a caller buffer.
// NORM: what the pass accumulates for the next trigger test: 0 nothing, 1 the sweep's squared
// drift, 2 its squared x (xhat is then not read at all), 3 its squared x and squared xhat.
// TOPK: messages of this iteration may have to be applied.
// HISTA: also histogram the top 11 bits of the new rank keys per tensor, the first
// radix pass of the next iteration's Top-K selection, while the values are in registers.
// SPW: consecutive sweeps of a chunk per workgroup (one float4 per thread and sweep).  One
// streams best; two halve the per-workgroup costs of the Top-K work (message look-up,
// barriers, clearing and merging the histogram).
// STREAM: non-temporal accesses to the arenas (rings larger than the last-level cache).
// PULL: whole-tensor sends of this iteration have NOT been copied into the mailboxes: where a
// neighbour sent, its values are fetched from the copy of x that the previous update pass left
// (x itself is being overwritten by its owner in this very launch), used, and written into the
// mailbox here; and the new x is also written to the other of the two copies for the next
// iteration (two copies in turn: the one read now is written by nobody in this launch).  Fewer
// launches per iteration for rings that live in the cache, where launches are what costs.
// TESTS (with PULL): no kernel has run the trigger tests of this iteration.  Every workgroup
// runs the three it depends on itself (its own tensor's and that tensor's of the two
// neighbours: three wavefronts, one each, from the sweep sums the previous pass left), and the
// first workgroup of each tensor books its tensor's outcome.  What the tests read is not
// written by this launch (Tables: the _out arrays), so every workgroup decides alike.  One
// launch per iteration.
template <int DIST, bool GRADBUF, int NORM, bool TOPK, bool HISTA, int SPW, bool STREAM, bool PULL = false,
          bool TESTS = false>
__global__ __launch_bounds__(kThreads) void k_update(Tables T, StepArgs A) {
  static_assert(!TESTS || (PULL && !TOPK && SPW == 1), "the tests ride in the pass of rings whose receivers fetch the sends");
  __shared__ double ws[4 * SPW];
  __shared__ uint32_t outcome[3];
  // LDS: the windows of the three patches; once those are consumed the same
  // storage holds the key histogram
  constexpr int NWIN = EVG_PATCH_WINDOWS;
  constexpr int kWinFloats = NWIN * SPW * kSweep > (HISTA ? kHistBins : 0) ? NWIN * SPW * kSweep : kHistBins;
  __shared__ __attribute__((aligned(16))) float pv[TOPK ? kWinFloats : 4];
  __shared__ uint32_t pm[3 * 32 * SPW];
  constexpr uint32_t kWin = SPW * kSweep, kWinWords = 32 * SPW;
  uint32_t* hA = reinterpret_cast<uint32_t*>(pv);
  static_assert(!HISTA || TOPK, "the histogram shares the patch windows' storage");
  static_assert(NWIN >= 1 && NWIN <= 3, "EVG_PATCH_WINDOWS is 1, 2 or 3");
  const uint32_t groups = T.SW / SPW;      // workgroups per chunk (SW is a multiple of SPW)
  const uint32_t c = blockIdx.x / groups, sub0 = (blockIdx.x % groups) * SPW, r = blockIdx.y;
  const ChunkDesc cd = T.chunks[c];
  const uint32_t seg = r * T.L + cd.layer;
  bool vl = T.valid_l[seg] != 0, vr = T.valid_r[seg] != 0;
  const uint32_t lw = (r + T.P - 1) % T.P, rw = (r + 1) % T.P;
  uint32_t my_event;
  bool from_l = false, from_r = false;
  if (TESTS) {
    const uint32_t segs[3] = {seg, lw * T.L + cd.layer, rw * T.L + cd.layer};
    const bool books = blockIdx.x == T.layers[cd.layer].chunk0 * groups;    // the tensor's first workgroup
    if (wave_id() < 3) {
      const uint32_t sg = segs[wave_id()];
      double acc, acc_hat;
      bool hat_sums;
      segment_sums(T, A, sg, &acc, &acc_hat, &hat_sums);
      if (lane_id() == 0)
        outcome[wave_id()] = (books && wave_id() == 0) ? segment_test<true, false>(T, A, sg, acc, acc_hat, hat_sums)
                                                       : segment_test<false, false>(T, A, sg, acc, acc_hat, hat_sums);
    }
    __syncthreads();
    my_event = outcome[0];
    from_l = outcome[1] == 1;
    from_r = outcome[2] == 1;
    // a neighbour's send fills my mailbox slot for good (the flags only ever go from 0 to 1, so
    // a workgroup that reads one after the booking below sees what it would have computed)
    vl = vl || from_l;
    vr = vr || from_r;
    if (books && threadIdx.x == 0) {
      if (from_l) T.valid_l[seg] = 1;
      if (from_r) T.valid_r[seg] = 1;
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) close_step(T, A);
  } else {
    my_event = T.fired[seg];
    // PULL: did my neighbours send this tensor whole in this iteration? (then vl / vr are set)
    from_l = PULL && T.fired[lw * T.L + cd.layer] == 1;
    from_r = PULL && T.fired[rw * T.L + cd.layer] == 1;
  }
  // step n reads copy (n-1) & 1 of x and writes copy n & 1; where a kernel ahead of this one ran
  // the tests it has counted this step already
  const size_t arena = (size_t)T.P * T.Npad;
  const uint64_t step_no = !PULL ? 0 : TESTS ? (uint64_t)A.step_no + 1 : T.it->iters;
  const float* snap_in = PULL ? T.xsnap + ((step_no + 1) & 1) * arena : nullptr;
  float* snap_out = PULL ? T.xsnap + (step_no & 1) * arena : nullptr;
  // xhat := x for the whole tensor: after a whole send, or after any event when a Top-K
  // event is read as resetting the tensor's xhat
  const bool sent_whole = my_event == 1 || (TOPK && A.xhat_reset && my_event == 2);
  const size_t base = (size_t)r * T.Npad + cd.off;
  const float third = 0.333333343f;   // (float)(1/3): the ring's mixing weight
  const uint32_t k_iter = step_k(T, A);
  uint32_t e[SPW];
  bool live[SPW];
#pragma unroll
  for (int u = 0; u < SPW; ++u) {
    e[u] = (sub0 + u) * kSweep + threadIdx.x * kLaneElems;
    live[u] = e[u] < cd.len;
  }
  double acc[SPW], acc_hat[SPW];
#pragma unroll
  for (int u = 0; u < SPW; ++u) { acc[u] = 0.0; acc_hat[u] = 0.0; }
  if (sub0 * kSweep < cd.len) {        // uniform: the window holds elements
    float xa[SPW][4], va[SPW][4], la[SPW][4], ra[SPW][4], ha[SPW][4], g[SPW][4];
#pragma unroll
    for (int u = 0; u < SPW; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) { xa[u][i] = 0.f; va[u][i] = 0.f; la[u][i] = 0.f; ra[u][i] = 0.f; ha[u][i] = 0.f; g[u][i] = 0.f; }
      if (live[u]) {
        const float4 x4 = ld4t<STREAM>(T.x + base + e[u]);
        float4 v4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!A.plain_sgd) v4 = ld4t<STREAM>(T.vel + base + e[u]);   // uniform
        xa[u][0] = x4.x; xa[u][1] = x4.y; xa[u][2] = x4.z; xa[u][3] = x4.w;
        va[u][0] = v4.x; va[u][1] = v4.y; va[u][2] = v4.z; va[u][3] = v4.w;
        if (from_l) {        // the put of my left neighbour, carried out by its receiver
          const float4 t = ld4t<STREAM>(snap_in + (size_t)lw * T.Npad + cd.off + e[u]);
          la[u][0] = t.x; la[u][1] = t.y; la[u][2] = t.z; la[u][3] = t.w;
          st4t<STREAM>(T.mbox_l + base + e[u], t);
        } else if (vl) { const float4 t = ld4t<STREAM>(T.mbox_l + base + e[u]); la[u][0] = t.x; la[u][1] = t.y; la[u][2] = t.z; la[u][3] = t.w; }
        if (from_r) {
          const float4 t = ld4t<STREAM>(snap_in + (size_t)rw * T.Npad + cd.off + e[u]);
          ra[u][0] = t.x; ra[u][1] = t.y; ra[u][2] = t.z; ra[u][3] = t.w;
          st4t<STREAM>(T.mbox_r + base + e[u], t);
        } else if (vr) { const float4 t = ld4t<STREAM>(T.mbox_r + base + e[u]); ra[u][0] = t.x; ra[u][1] = t.y; ra[u][2] = t.z; ra[u][3] = t.w; }
        if (sent_whole) {
          // the whole tensor was sent in this iteration: xhat becomes the x just read
          ha[u][0] = xa[u][0]; ha[u][1] = xa[u][1]; ha[u][2] = xa[u][2]; ha[u][3] = xa[u][3];
          st4t<STREAM>(T.xhat + base + e[u], x4);
        } else if (NORM == 1 || NORM == 3 || TOPK) {
          const float4 t = ld4t<STREAM>(T.xhat + base + e[u]); ha[u][0] = t.x; ha[u][1] = t.y; ha[u][2] = t.z; ha[u][3] = t.w;
        }
        if (GRADBUF) { const float4 t = ld4t<STREAM>(A.grad + base + e[u]); g[u][0] = t.x; g[u][1] = t.y; g[u][2] = t.z; g[u][3] = t.w; }
      }
    }
    if (TOPK) {
      // three sparse patches of this iteration: my own message (what xhat must now
      // hold) and the two messages that arrive in my mailboxes
      const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
      const uint32_t moff = T.layers[cd.layer].msg_off, j_lo = cd.j0 + sub0 * kSweep;
      const Slice s0m = message_slice<SPW>(T, r, cd.layer, c, sub0, moff);
      Slice s1 = message_slice<SPW>(T, left, cd.layer, c, sub0, moff);
      Slice s2 = message_slice<SPW>(T, right, cd.layer, c, sub0, moff);
      Slice s0 = s0m;
      if (sent_whole) s0.n = 0;              // xhat has just been written from registers
      if (A.delay) { s1.n = 0; s2.n = 0; }   // the neighbours' messages land after this pass
      if (s0.n | s1.n | s2.n) {          // uniform
        for (uint32_t q = threadIdx.x; q < 3 * kWinWords; q += kThreads) pm[q] = 0;
        __syncthreads();
        // applies window w (values) / mask m to array a of every sweep and writes changed groups back
        auto apply = [&](const float* w, const uint32_t* m, float (*a)[4], float* arena) {
#pragma unroll
          for (int u = 0; u < SPW; ++u) {
            const uint32_t b = take_patch(w, m, u, a[u]);
            if (live[u] && b) st4t<STREAM>(arena + base + e[u], make_float4(a[u][0], a[u][1], a[u][2], a[u][3]));
          }
        };
        if (NWIN == 3) {
          scatter_slice<SPW>(T, s0, j_lo, pv, pm);
          scatter_slice<SPW>(T, s1, j_lo, pv + kWin, pm + kWinWords);
          scatter_slice<SPW>(T, s2, j_lo, pv + 2 * kWin, pm + 2 * kWinWords);
          __syncthreads();
          apply(pv, pm, ha, T.xhat);
          apply(pv + kWin, pm + kWinWords, la, T.mbox_l);
          apply(pv + 2 * kWin, pm + 2 * kWinWords, ra, T.mbox_r);
        } else if (NWIN == 2) {
          // two windows in turn: while one is read the next message is scattered into the other
          scatter_slice<SPW>(T, s0, j_lo, pv, pm);
          __syncthreads();
          scatter_slice<SPW>(T, s1, j_lo, pv + kWin, pm + kWinWords);
          apply(pv, pm, ha, T.xhat);
          __syncthreads();
          scatter_slice<SPW>(T, s2, j_lo, pv, pm + 2 * kWinWords);
          apply(pv + kWin, pm + kWinWords, la, T.mbox_l);
          __syncthreads();
          apply(pv, pm + 2 * kWinWords, ra, T.mbox_r);
        } else {
          // one window, the three messages one after the other (empty ones skipped: uniform)
          if (s0.n) {
            scatter_slice<SPW>(T, s0, j_lo, pv, pm);
            __syncthreads();
            apply(pv, pm, ha, T.xhat);
            __syncthreads();
          }
          if (s1.n) {
            scatter_slice<SPW>(T, s1, j_lo, pv, pm + kWinWords);
            __syncthreads();
            apply(pv, pm + kWinWords, la, T.mbox_l);
            __syncthreads();
          }
          if (s2.n) {
            scatter_slice<SPW>(T, s2, j_lo, pv, pm + 2 * kWinWords);
            __syncthreads();
            apply(pv, pm + 2 * kWinWords, ra, T.mbox_r);
          }
        }
      }
    }
    if (HISTA) {
      __syncthreads();                 // patches consumed by every thread
      for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) hA[b] = 0;
      __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < SPW; ++u) {
      if (live[u]) {
        if (!GRADBUF) {
          const float sg = (float)(T.layers[cd.layer].sig_base * step_decay(T, A));
          if (DIST == 0) {
            float z[4];
            normals4(philox((cd.j0 + e[u]) >> 2, cd.layer, k_iter, r, A.key0, A.key1), z);
#pragma unroll
            for (int i = 0; i < 4; ++i) g[u][i] = sg * z[i];
          } else {
            // four variates from the two Philox blocks 2g, 2g+1 of this float4 (g = index / 4):
            // variate i takes words 2i (radius) and 2i+1 (angle) of the eight
            const uint32_t b0 = ((cd.j0 + e[u]) >> 2) << 1;
            const Rand4 ra = philox(b0, cd.layer, k_iter, r, A.key0, A.key1);
            const Rand4 rb = philox(b0 + 1u, cd.layer, k_iter, r, A.key0, A.key1);
            g[u][0] = sg * student_t3(ra.w[0], ra.w[1]);
            g[u][1] = sg * student_t3(ra.w[2], ra.w[3]);
            g[u][2] = sg * student_t3(rb.w[0], rb.w[1]);
            g[u][3] = sg * student_t3(rb.w[2], rb.w[3]);
          }
          if (A.spike_prob > 0.0f) {
            const Rand4 sp = philox(0u, 0xFFFFFFFFu, k_iter, r, A.key0, A.key1);
            if (unit_open(sp.w[0]) < A.spike_prob) {
#pragma unroll
              for (int i = 0; i < 4; ++i) g[u][i] = g[u][i] * A.spike_gain;
            }
          }
        }
        const uint32_t nv = cd.len - e[u] < 4u ? cd.len - e[u] : 4u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if ((uint32_t)i < nv) {   // lanes past the tensor's end are padding: left as they are
            // momentum 0 is the paper's plain SGD: the velocity is the gradient, and the
            // velocity arena is neither read nor written
            const float vn = A.plain_sgd ? g[u][i] : __builtin_fmaf(A.mu, va[u][i], g[u][i]);
            const float a = (vl ? (la[u][i] - xa[u][i]) : 0.0f) + (vr ? (ra[u][i] - xa[u][i]) : 0.0f);
            const float cns = __builtin_fmaf(a, third, xa[u][i]);
            xa[u][i] = __builtin_fmaf(-A.lr, vn, cns);
            va[u][i] = vn;
          }
        }
        st4t<STREAM>(T.x + base + e[u], make_float4(xa[u][0], xa[u][1], xa[u][2], xa[u][3]));
        if (PULL) st4t<STREAM>(snap_out + base + e[u], make_float4(xa[u][0], xa[u][1], xa[u][2], xa[u][3]));
        if (!A.plain_sgd) st4t<STREAM>(T.vel + base + e[u], make_float4(va[u][0], va[u][1], va[u][2], va[u][3]));
        if (NORM == 1) drift_acc(acc[u], xa[u], ha[u], nv);
        if (NORM >= 2) square_acc(acc[u], xa[u], nv);
        if (NORM == 3) square_acc(acc_hat[u], ha[u], nv);
        if (HISTA) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if ((uint32_t)i < nv) atomicAdd(&hA[rank_key(xa[u][i], ha[u][i], A.topk_key) >> 20], 1u);
        }
      }
    }
  }
  if (HISTA && sub0 * kSweep < cd.len) {     // uniform
    __syncthreads();
    uint32_t* gh = T.hist + (size_t)seg * kHistBins;
    for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) {
      const uint32_t v = hA[b];
      if (v) atomicAdd(&gh[b], v);
    }
  }
  if (NORM) {
    const size_t slot = ((size_t)r * T.C + c) * T.SW + sub0;
    double total[SPW];
    block_sums<SPW>(acc, ws, total);
    if (threadIdx.x == 0) {
#pragma unroll
      for (int u = 0; u < SPW; ++u) T.partials_out[slot + u] = total[u];
    }
    if (NORM == 3) {
      block_sums<SPW>(acc_hat, ws, total);
      if (threadIdx.x == 0) {
#pragma unroll
        for (int u = 0; u < SPW; ++u) T.partials_hat_out[slot + u] = total[u];
      }
    }
  }
}

// Mean over workers, one thread per float4 of a slice (last line of Algorithm B).
__global__ __launch_bounds__(kThreads) void k_average(Tables T, float* out) {
  const size_t q = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (q * 4 >= T.Npad) return;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (uint32_t r = 0; r < T.P; ++r) {
    const float4 v = ld4(T.x + (size_t)r * T.Npad + q * 4);
    a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
  }
  const double p = (double)T.P;
  st4s(out + q * 4, make_float4((float)(a0 / p), (float)(a1 / p), (float)(a2 / p), (float)(a3 / p)));
}

hipError_t launch_norm(const Tables& t, bool norm_diff, hipStream_t s) {
  const dim3 grid(t.C * t.SW, t.P), block(kThreads);
  if (norm_diff) k_norm<true><<<grid, block, 0, s>>>(t);
  else k_norm<false><<<grid, block, 0, s>>>(t);
  return hipGetLastError();
}

template <int NORM, bool TOPK, bool HISTA, int SPW>
static void launch_update_w(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                            hipStream_t s) {
  const dim3 grid(t.C * (t.SW / SPW), t.P), block(kThreads);
  if (!TOPK && a.pull) {     // the host sets pull only for cache-resident rings with whole-tensor sends
    constexpr bool NT = false, NH = false;
    if (a.one_launch) {      // ... and one_launch only where the pass accumulates the norms (NORM != 0)
      constexpr bool TS = NORM != 0;
      if (grad_mode == 1) k_update<0, true, NORM, NT, NH, 1, false, true, TS><<<grid, block, 0, s>>>(t, a);
      else if (dist == 0) k_update<0, false, NORM, NT, NH, 1, false, true, TS><<<grid, block, 0, s>>>(t, a);
      else k_update<1, false, NORM, NT, NH, 1, false, true, TS><<<grid, block, 0, s>>>(t, a);
      return;
    }
    if (grad_mode == 1) k_update<0, true, NORM, NT, NH, 1, false, true><<<grid, block, 0, s>>>(t, a);
    else if (dist == 0) k_update<0, false, NORM, NT, NH, 1, false, true><<<grid, block, 0, s>>>(t, a);
    else k_update<1, false, NORM, NT, NH, 1, false, true><<<grid, block, 0, s>>>(t, a);
    return;
  }
  if (a.cached) {
    if (grad_mode == 1) k_update<0, true, NORM, TOPK, HISTA, SPW, false><<<grid, block, 0, s>>>(t, a);
    else if (dist == 0) k_update<0, false, NORM, TOPK, HISTA, SPW, false><<<grid, block, 0, s>>>(t, a);
    else k_update<1, false, NORM, TOPK, HISTA, SPW, false><<<grid, block, 0, s>>>(t, a);
    return;
  }
  if (grad_mode == 1) k_update<0, true, NORM, TOPK, HISTA, SPW, true><<<grid, block, 0, s>>>(t, a);
  else if (dist == 0) k_update<0, false, NORM, TOPK, HISTA, SPW, true><<<grid, block, 0, s>>>(t, a);
  else k_update<1, false, NORM, TOPK, HISTA, SPW, true><<<grid, block, 0, s>>>(t, a);
}

template <int NORM, bool TOPK, bool HISTA>
static void launch_update_v(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                            hipStream_t s) {
  // two sweeps per workgroup where the pass carries the Top-K extras and a chunk has them
  // (measured: four are slower again, LDS and registers then hold occupancy down)
  if (TOPK && HISTA && t.SW % 2 == 0)
    launch_update_w<NORM, TOPK, HISTA, (TOPK && HISTA) ? EVG_UPDATE_SPW : 1>(t, a, dist, grad_mode, s);
  else
    launch_update_w<NORM, TOPK, HISTA, 1>(t, a, dist, grad_mode, s);
}

hipError_t launch_update(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                         int norm, hipStream_t s) {
  if (a.topk_on) {
    if (norm == 1 && a.hist_fused) launch_update_v<1, true, true>(t, a, dist, grad_mode, s);
    else if (norm == 3 && a.hist_fused) launch_update_v<3, true, true>(t, a, dist, grad_mode, s);
    else if (norm == 0) launch_update_v<0, true, false>(t, a, dist, grad_mode, s);
    else return hipErrorInvalidValue;
  } else {
    if (norm == 0) launch_update_v<0, false, false>(t, a, dist, grad_mode, s);
    else if (norm == 1) launch_update_v<1, false, false>(t, a, dist, grad_mode, s);
    else if (norm == 2) launch_update_v<2, false, false>(t, a, dist, grad_mode, s);
    else return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_average(const Tables& t, float* out, hipStream_t s) {
  const uint64_t quads = t.Npad / 4;
  const uint32_t grid = (uint32_t)((quads + kThreads - 1) / kThreads);
  k_average<<<dim3(grid), dim3(kThreads), 0, s>>>(t, out);
  return hipGetLastError();
}

}  // namespace evg
