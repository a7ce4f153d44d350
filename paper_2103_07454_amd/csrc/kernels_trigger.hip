// Trigger test and whole-tensor sends.
//   k_trigger  one wavefront per (worker, tensor): finishes the drift norm from the
//              per-chunk partial sums in a fixed order, applies the event condition
//              || xhat - x || >= delta (Section 4), recomputes the adaptive threshold
//              at events (Eq. 3), marks the neighbours' mailbox slots as filled.
//   k_scan     exclusive prefix sums of the fired flags weighted by chunk counts.
//   k_expand   writes the compact lists of chunks to copy / to Top-K select.
//   k_copy     x -> left neighbour's right mailbox, right neighbour's left mailbox for
//              every listed chunk: the stand-in for the one-sided puts of Section 6.
#include "trigger_device.h"

namespace evg {

// The trigger test of one (worker, tensor), by one whole wavefront.
__device__ __forceinline__ void trigger_segment(const Tables& T, const StepArgs& A, uint32_t seg) {
  double acc, acc_hat;
  bool hat_sums;
  segment_sums(T, A, seg, &acc, &acc_hat, &hat_sums);
  if (lane_id() == 0) (void)segment_test<true, true>(T, A, seg, acc, acc_hat, hat_sums);
}

__global__ __launch_bounds__(kThreads) void k_trigger(Tables T, StepArgs A) {
  const uint32_t seg = blockIdx.x * (kThreads / 64) + wave_id();
  if (seg >= T.S) return;           // whole wavefront leaves; no workgroup barrier below
  trigger_segment(T, A, seg);
  // receivers fetch the sends themselves: no chunk lists, so no scan kernel follows
  if (A.pull && seg == 0 && lane_id() == 0) close_step(T, A);
}

// First kernel of a replayable step: one thread moves the device's iteration on.
__global__ void k_begin(Tables T) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const uint32_t k = T.it->k_next;
  T.it->k = k;
  if (k >= T.decay_len) T.it->overflow = 1;
  T.it->decay_pow = T.decay_tab[k < T.decay_len ? k : T.decay_len - 1];
}

// One workgroup of 1024 threads scans all P*L flags.  It runs once per step, after the
// trigger tests: its first thread also closes the step's bookkeeping.
// EXPAND: each thread also writes the chunk lists of its own tensors (small rings: one
// dependent launch less; large rings leave that to k_expand's many wavefronts).
template <bool EXPAND>
__device__ __forceinline__ void scan_segments(const Tables& T, const StepArgs& A, uint32_t* ws) {
  const uint32_t per = (T.S + 1023u) / 1024u;
  const uint32_t lo = threadIdx.x * per;
  const uint32_t hi = lo + per < T.S ? lo + per : T.S;
  uint32_t nf = 0, nt = 0, ns = 0;
  for (uint32_t s = lo; s < hi; ++s) {
    const uint32_t f = T.fired[s], nc = T.layers[s % T.L].nchunks;
    if (f == 1) nf += nc;
    if (f == 2) { nt += nc; ns += 1; }
  }
  uint32_t tf, tt, ts;
  uint32_t of = block_excl_scan<16>(nf, ws, &tf);
  uint32_t ot = block_excl_scan<16>(nt, ws, &tt);
  (void)block_excl_scan<16>(ns, ws, &ts);
  for (uint32_t s = lo; s < hi; ++s) {
    const uint32_t f = T.fired[s], nc = T.layers[s % T.L].nchunks;
    T.seg_woff_full[s] = of;
    T.seg_woff_topk[s] = ot;
    if (EXPAND && f) {
      uint32_t* dst = f == 1 ? T.work_full + of : T.work_topk + ot;
      const uint32_t first = (s / T.L) * T.C + T.layers[s % T.L].chunk0;
      for (uint32_t i = 0; i < nc; ++i) dst[i] = first + i;
    }
    if (f == 1) of += nc;
    if (f == 2) ot += nc;
  }
  if (threadIdx.x == 0) {
    T.counts[0] = tf; T.counts[1] = tt; T.counts[2] = ts;
    close_step(T, A);
  }
}

template <bool EXPAND>
__global__ __launch_bounds__(1024) void k_scan(Tables T, StepArgs A) {
  __shared__ uint32_t ws[16];
  scan_segments<EXPAND>(T, A, ws);
}

// Rings of a few tensors in all: the sixteen wavefronts of one workgroup run the trigger
// tests, then the same workgroup scans and writes the lists -- one launch instead of two.
__global__ __launch_bounds__(1024) void k_front(Tables T, StepArgs A) {
  __shared__ uint32_t ws[16];
  for (uint32_t seg = wave_id(); seg < T.S; seg += 16) trigger_segment(T, A, seg);
  if (A.pull) {                     // uniform: no lists are needed
    if (threadIdx.x == 0) close_step(T, A);
    return;
  }
  __syncthreads();                  // the flags written above are read below by other wavefronts
  scan_segments<true>(T, A, ws);
}

__global__ __launch_bounds__(kThreads) void k_expand(Tables T) {
  const uint32_t seg = blockIdx.x * (kThreads / 64) + wave_id();
  if (seg >= T.S) return;
  const uint32_t f = T.fired[seg];
  if (f == 0) return;
  const uint32_t r = seg / T.L;
  const LayerDesc ld = T.layers[seg % T.L];
  uint32_t* dst = f == 1 ? T.work_full + T.seg_woff_full[seg] : T.work_topk + T.seg_woff_topk[seg];
  const uint32_t first = r * T.C + ld.chunk0;
  for (uint32_t i = lane_id(); i < ld.nchunks; i += 64) dst[i] = first + i;
}

// (xhat takes the sent values in the update pass, which has them in registers.)
template <int SWEEPS, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_copy(Tables T) {
  const uint32_t n = T.counts[0];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = T.work_full[i];
    const uint32_t r = w / T.C, c = w % T.C;
    const ChunkDesc cd = T.chunks[c];
    const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
    const float* src = T.x + (size_t)r * T.Npad + cd.off;
    float* d1 = T.mbox_r + (size_t)left * T.Npad + cd.off;
    float* d2 = T.mbox_l + (size_t)right * T.Npad + cd.off;
#pragma unroll
    for (int it = 0; it < SWEEPS; ++it) {
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      if (e < cd.len) {
        const float4 v = ld4t<STREAM>(src + e);
        st4t<STREAM>(d1 + e, v);
        st4t<STREAM>(d2 + e, v);
      }
    }
  }
}

// Rings with at most this many chunks in all have their lists written by the scan itself.
static bool scan_expands(const Tables& t) { return (uint64_t)t.P * t.C <= 8192; }
// ... and those with at most 64 tensors in all run trigger, scan and lists as one workgroup.
static bool one_front(const Tables& t) { return t.S <= 64 && scan_expands(t); }

hipError_t launch_trigger(const Tables& t, const StepArgs& a, hipStream_t s) {
  if (one_front(t)) {
    k_front<<<dim3(1), dim3(1024), 0, s>>>(t, a);
    return hipGetLastError();
  }
  const uint32_t grid = (t.S + 3) / 4;
  k_trigger<<<dim3(grid), dim3(kThreads), 0, s>>>(t, a);
  return hipGetLastError();
}

hipError_t launch_begin(const Tables& t, hipStream_t s) {
  k_begin<<<dim3(1), dim3(64), 0, s>>>(t);
  return hipGetLastError();
}

hipError_t launch_scan(const Tables& t, const StepArgs& a, hipStream_t s) {
  if (one_front(t) || a.pull) return hipSuccess;
  if (scan_expands(t)) k_scan<true><<<dim3(1), dim3(1024), 0, s>>>(t, a);
  else k_scan<false><<<dim3(1), dim3(1024), 0, s>>>(t, a);
  return hipGetLastError();
}

hipError_t launch_expand(const Tables& t, const StepArgs& a, hipStream_t s) {
  if (scan_expands(t) || a.pull) return hipSuccess;
  const uint32_t grid = (t.S + 3) / 4;
  k_expand<<<dim3(grid), dim3(kThreads), 0, s>>>(t);
  return hipGetLastError();
}

// Delayed delivery: after the updates, every tensor that sent in this iteration (whole
// or Top-K) lands in its neighbours' mailboxes.  What a neighbour must hold afterwards is
// exactly the sender's xhat (entries that were not sent are equal already), so each listed
// chunk of xhat is copied, and the receivers' slots are marked as filled.
template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_deliver(Tables T) {
  const uint32_t n_full = T.counts[0], n = n_full + T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = i < n_full ? T.work_full[i] : T.work_topk[i - n_full];
    const uint32_t r = w / T.C, c = w % T.C;
    const ChunkDesc cd = T.chunks[c];
    const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
    const float* src = T.xhat + (size_t)r * T.Npad + cd.off;
    float* d1 = T.mbox_r + (size_t)left * T.Npad + cd.off;
    float* d2 = T.mbox_l + (size_t)right * T.Npad + cd.off;
#pragma unroll
    for (int it = 0; it < SWEEPS; ++it) {
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      if (e < cd.len) {
        const float4 v = ld4s(src + e);
        st4s(d1 + e, v);
        st4s(d2 + e, v);
      }
    }
    if (threadIdx.x == 0 && cd.j0 == 0) {     // the tensor's first chunk speaks for the tensor
      T.valid_r[left * T.L + cd.layer] = 1;
      T.valid_l[right * T.L + cd.layer] = 1;
    }
  }
}

template <bool STREAM>
static hipError_t launch_copy_v(const Tables& t, uint32_t chunk_elems, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kThreads);
  switch (chunk_elems / kSweep) {
    case 1: k_copy<1, STREAM><<<g, b, 0, s>>>(t); break;
    case 2: k_copy<2, STREAM><<<g, b, 0, s>>>(t); break;
    case 4: k_copy<4, STREAM><<<g, b, 0, s>>>(t); break;
    case 8: k_copy<8, STREAM><<<g, b, 0, s>>>(t); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_copy(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid, hipStream_t s) {
  return a.cached ? launch_copy_v<false>(t, chunk_elems, grid, s) : launch_copy_v<true>(t, chunk_elems, grid, s);
}

hipError_t launch_deliver(const Tables& t, uint32_t chunk_elems, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kThreads);
  switch (chunk_elems / kSweep) {
    case 1: k_deliver<1><<<g, b, 0, s>>>(t); break;
    case 2: k_deliver<2><<<g, b, 0, s>>>(t); break;
    case 4: k_deliver<4><<<g, b, 0, s>>>(t); break;
    case 8: k_deliver<8><<<g, b, 0, s>>>(t); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace evg
