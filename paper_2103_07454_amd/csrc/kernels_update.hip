// The two streaming passes over every element: the fused neighbour-averaging +
// momentum-SGD update (Section 3, Eq. 2 with the last received neighbour values
// of Section 4), which also accumulates the squared drift || x - xhat ||^2 that the
// next iteration's trigger test needs, and a stand-alone drift-norm pass.
//
// One workgroup (256 threads, one float4 per thread) owns one 1024-element sweep of
// one chunk of one worker: the launch shape that streams best on MI355X.  HBM-bound:
// 5 reads + 2 writes of 4 bytes per element.
//
// Top-K messages are applied here, where the dense arrays pass through registers
// anyway: the sender's own message patches xhat (only the sent entries count as
// communicated), the left and right neighbours' messages patch the two mailboxes
// (the receiving end of the put, Section 6).  A message slice is scattered into an
// LDS window first, so that global accesses stay 16-byte wide and coalesced, and a
// float4 is written back only if it changed.
#include "evg_device.h"

namespace evg {

__device__ __forceinline__ float4 ld4(const float* p) { return ld4s(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { st4s(p, v); }

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
  if (threadIdx.x == 0) T.partials[slot] = total;
  if (NORMDIFF) {
    const double total_hat = block_sum(acc_hat, ws);
    if (threadIdx.x == 0) T.partials_hat[slot] = total_hat;
  }
}

// One source of a sparse patch for this workgroup's 1024-element window: the slice
// of worker `src`'s message that chunk c, sweep sub produced (empty if `src` sent no
// Top-K message for this tensor in this iteration).
struct Slice { uint32_t at; uint32_t n; };   // P*Ktot and P*C*(SW+1) fit 32 bits (checked at init)

__device__ __forceinline__ Slice message_slice(const Tables& T, uint32_t src, uint32_t layer, uint32_t c,
                                               uint32_t sub, uint32_t msg_off) {
  Slice s;
  const uint32_t w = (src * T.C + c) * (T.SW + 1) + sub;
  const uint32_t lo = T.chunk_sub[w], hi = T.chunk_sub[w + 1];
  s.at = src * T.Ktot + msg_off + lo;
  s.n = T.fired[src * T.L + layer] == 2 ? hi - lo : 0u;
  return s;
}

// Scatters a slice into its LDS window (values + one bit per element).
__device__ __forceinline__ void scatter_slice(const Tables& T, const Slice& s, uint32_t j_lo, float* pv,
                                              uint32_t* pm) {
  for (uint32_t q = threadIdx.x; q < s.n; q += kThreads) {
    const uint32_t loc = T.msg_idx[s.at + q] - j_lo;
    if (loc < (uint32_t)kSweep) {
      pv[loc] = T.msg_val[s.at + q];
      atomicOr(&pm[loc >> 5], 1u << (loc & 31u));
    }
  }
}

// Replaces this thread's lanes by the window's entries.  Returns the change mask of
// the aligned 64-byte group (4 neighbouring float4s) this thread's float4 belongs to:
// write-back is decided per group, because scattered 16-byte writes cost far more in
// HBM than the few unchanged bytes a full 64-byte line carries.
__device__ __forceinline__ uint32_t take_patch(const float* pv, const uint32_t* pm, float a[4]) {
  const uint32_t l0 = threadIdx.x * kLaneElems;          // first element of this thread
  const uint32_t g0 = l0 & ~15u;                         // first element of its 64-byte group
  const uint32_t group = (pm[g0 >> 5] >> (g0 & 31u)) & 0xFFFFu;   // (32-byte groups measured 19 % slower)
  const uint32_t bits = (group >> (l0 & 15u)) & 0xFu;
  const float4 v = *reinterpret_cast<const float4*>(pv + l0);   // unwritten lanes hold garbage: masked
  a[0] = (bits & 1u) ? v.x : a[0];
  a[1] = (bits & 2u) ? v.y : a[1];
  a[2] = (bits & 4u) ? v.z : a[2];
  a[3] = (bits & 8u) ? v.w : a[3];
  return group;
}

// DIST: 0 normal (one Philox block per float4), 1 Student-t(3) (one block per element).
// GRADBUF: gradients come from a caller buffer.
// NORM: what the pass accumulates for the next trigger test: 0 nothing, 1 the sweep's squared
// drift, 2 its squared x (xhat is then not read at all), 3 its squared x and squared xhat.
// TOPK: messages of this iteration may have to be applied.
// HISTA: also histogram the top 11 bits of the new rank keys per tensor, the first
// radix pass of the next iteration's Top-K selection, while the values are in registers.
template <int DIST, bool GRADBUF, int NORM, bool TOPK, bool HISTA>
__global__ __launch_bounds__(kThreads) void k_update(Tables T, StepArgs A) {
  __shared__ double ws[4];
  // LDS: the windows of the three patches; once those are consumed the same
  // storage holds the key histogram
  __shared__ __attribute__((aligned(16))) float pv[TOPK ? 3 * kSweep : 4];
  __shared__ uint32_t pm[96];
  uint32_t* hA = reinterpret_cast<uint32_t*>(pv);
  static_assert(!HISTA || (TOPK && 3 * kSweep >= kHistBins), "histogram must fit the patch windows");
  const uint32_t c = blockIdx.x / T.SW, sub = blockIdx.x % T.SW, r = blockIdx.y;
  const ChunkDesc cd = T.chunks[c];
  const uint32_t seg = r * T.L + cd.layer;
  const bool vl = T.valid_l[seg] != 0, vr = T.valid_r[seg] != 0;
  const bool sent_whole = T.fired[seg] == 1;
  const size_t base = (size_t)r * T.Npad + cd.off;
  const float third = 0.333333343f;   // (float)(1/3): the ring's mixing weight
  const uint32_t e = sub * kSweep + threadIdx.x * kLaneElems;
  const bool live = e < cd.len;
  double acc = 0.0, acc_hat = 0.0;
  if (sub * kSweep < cd.len) {        // uniform: this sweep holds elements
    float xa[4] = {0.f, 0.f, 0.f, 0.f}, va[4] = {0.f, 0.f, 0.f, 0.f};
    float la[4] = {0.f, 0.f, 0.f, 0.f}, ra[4] = {0.f, 0.f, 0.f, 0.f}, ha[4] = {0.f, 0.f, 0.f, 0.f};
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (live) {
      const float4 x4 = ld4(T.x + base + e), v4 = ld4(T.vel + base + e);
      xa[0] = x4.x; xa[1] = x4.y; xa[2] = x4.z; xa[3] = x4.w;
      va[0] = v4.x; va[1] = v4.y; va[2] = v4.z; va[3] = v4.w;
      if (vl) { const float4 t = ld4(T.mbox_l + base + e); la[0] = t.x; la[1] = t.y; la[2] = t.z; la[3] = t.w; }
      if (vr) { const float4 t = ld4(T.mbox_r + base + e); ra[0] = t.x; ra[1] = t.y; ra[2] = t.z; ra[3] = t.w; }
      if (sent_whole) {
        // the whole tensor was sent in this iteration: xhat becomes the x just read
        ha[0] = xa[0]; ha[1] = xa[1]; ha[2] = xa[2]; ha[3] = xa[3];
        st4(T.xhat + base + e, x4);
      } else if (NORM == 1 || NORM == 3 || TOPK) {
        const float4 t = ld4(T.xhat + base + e); ha[0] = t.x; ha[1] = t.y; ha[2] = t.z; ha[3] = t.w;
      }
      if (GRADBUF) { const float4 t = ld4(A.grad + base + e); g[0] = t.x; g[1] = t.y; g[2] = t.z; g[3] = t.w; }
    }
    if (TOPK) {
      // three sparse patches of this iteration: my own message (what xhat must now
      // hold) and the two messages that arrive in my mailboxes
      const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
      const uint32_t moff = T.layers[cd.layer].msg_off, j_lo = cd.j0 + sub * kSweep;
      const Slice s0 = message_slice(T, r, cd.layer, c, sub, moff);
      Slice s1 = message_slice(T, left, cd.layer, c, sub, moff);
      Slice s2 = message_slice(T, right, cd.layer, c, sub, moff);
      if (A.delay) { s1.n = 0; s2.n = 0; }   // the neighbours' messages land after this pass
      if (s0.n | s1.n | s2.n) {          // uniform
        if (threadIdx.x < 96) pm[threadIdx.x] = 0;
        __syncthreads();
        scatter_slice(T, s0, j_lo, pv, pm);
        scatter_slice(T, s1, j_lo, pv + kSweep, pm + 32);
        scatter_slice(T, s2, j_lo, pv + 2 * kSweep, pm + 64);
        __syncthreads();
        const uint32_t b0 = take_patch(pv, pm, ha);
        const uint32_t b1 = take_patch(pv + kSweep, pm + 32, la);
        const uint32_t b2 = take_patch(pv + 2 * kSweep, pm + 64, ra);
        if (live && b0) st4(T.xhat + base + e, make_float4(ha[0], ha[1], ha[2], ha[3]));
        if (live && b1) st4(T.mbox_l + base + e, make_float4(la[0], la[1], la[2], la[3]));
        if (live && b2) st4(T.mbox_r + base + e, make_float4(ra[0], ra[1], ra[2], ra[3]));
      }
    }
    if (HISTA) {
      __syncthreads();                 // patches consumed by every thread
      for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) hA[b] = 0;
      __syncthreads();
    }
    if (live) {
      if (!GRADBUF) {
        const float sg = (float)(T.layers[cd.layer].sig_base * A.decay_pow);
        if (DIST == 0) {
          float z[4];
          normals4(philox((cd.j0 + e) >> 2, cd.layer, A.k, r, A.key0, A.key1), z);
#pragma unroll
          for (int i = 0; i < 4; ++i) g[i] = sg * z[i];
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float z[4];
            normals4(philox(cd.j0 + e + i, cd.layer, A.k, r, A.key0, A.key1), z);
            g[i] = sg * student_t3(z);
          }
        }
        if (A.spike_prob > 0.0f) {
          const Rand4 sp = philox(0u, 0xFFFFFFFFu, A.k, r, A.key0, A.key1);
          if (unit_open(sp.w[0]) < A.spike_prob) {
#pragma unroll
            for (int i = 0; i < 4; ++i) g[i] = g[i] * A.spike_gain;
          }
        }
      }
      const uint32_t nv = cd.len - e < 4u ? cd.len - e : 4u;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if ((uint32_t)i < nv) {   // lanes past the tensor's end are padding: left as they are
          const float vn = __builtin_fmaf(A.mu, va[i], g[i]);
          const float a = (vl ? (la[i] - xa[i]) : 0.0f) + (vr ? (ra[i] - xa[i]) : 0.0f);
          const float cns = __builtin_fmaf(a, third, xa[i]);
          xa[i] = __builtin_fmaf(-A.lr, vn, cns);
          va[i] = vn;
        }
      }
      st4(T.x + base + e, make_float4(xa[0], xa[1], xa[2], xa[3]));
      st4(T.vel + base + e, make_float4(va[0], va[1], va[2], va[3]));
      if (NORM == 1) drift_acc(acc, xa, ha, nv);
      if (NORM >= 2) square_acc(acc, xa, nv);
      if (NORM == 3) square_acc(acc_hat, ha, nv);
      if (HISTA) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if ((uint32_t)i < nv) atomicAdd(&hA[rank_key(xa[i], ha[i], A.topk_key) >> 20], 1u);
      }
    }
  }
  if (HISTA && sub * kSweep < cd.len) {     // uniform
    __syncthreads();
    uint32_t* gh = T.hist + (size_t)seg * kHistBins;
    for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) {
      const uint32_t v = hA[b];
      if (v) atomicAdd(&gh[b], v);
    }
  }
  if (NORM) {
    const size_t slot = ((size_t)r * T.C + c) * T.SW + sub;
    const double total = block_sum(acc, ws);
    if (threadIdx.x == 0) T.partials[slot] = total;
    if (NORM == 3) {
      const double total_hat = block_sum(acc_hat, ws);
      if (threadIdx.x == 0) T.partials_hat[slot] = total_hat;
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
  st4(out + q * 4, make_float4((float)(a0 / p), (float)(a1 / p), (float)(a2 / p), (float)(a3 / p)));
}

hipError_t launch_norm(const Tables& t, bool norm_diff, hipStream_t s) {
  const dim3 grid(t.C * t.SW, t.P), block(kThreads);
  if (norm_diff) k_norm<true><<<grid, block, 0, s>>>(t);
  else k_norm<false><<<grid, block, 0, s>>>(t);
  return hipGetLastError();
}

template <int NORM, bool TOPK, bool HISTA>
static void launch_update_v(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                            hipStream_t s) {
  const dim3 grid(t.C * t.SW, t.P), block(kThreads);
  if (grad_mode == 1) k_update<0, true, NORM, TOPK, HISTA><<<grid, block, 0, s>>>(t, a);
  else if (dist == 0) k_update<0, false, NORM, TOPK, HISTA><<<grid, block, 0, s>>>(t, a);
  else k_update<1, false, NORM, TOPK, HISTA><<<grid, block, 0, s>>>(t, a);
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
