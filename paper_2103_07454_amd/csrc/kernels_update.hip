// The two streaming passes over every element: the fused neighbour-averaging +
// momentum-SGD update (Section 3, Eq. 2 with the last received neighbour values
// of Section 4), which also accumulates the squared drift || x - xhat ||^2 that the
// next iteration's trigger test needs, and a stand-alone drift-norm pass.
//
// One workgroup (256 threads) owns one chunk of one tensor of one worker and sweeps
// it in float4 steps; HBM-bound: 5 reads + 2 writes of 4 bytes per element.
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

template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_norm(Tables T) {
  __shared__ double ws[4];
  const uint32_t c = blockIdx.x, r = blockIdx.y;
  const ChunkDesc cd = T.chunks[c];
  const size_t base = (size_t)r * T.Npad + cd.off;
  double acc = 0.0;
#pragma unroll
  for (int it = 0; it < SWEEPS; ++it) {
    const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
    if (e < cd.len) {
      const float4 x4 = ld4(T.x + base + e), h4 = ld4(T.xhat + base + e);
      const float xa[4] = {x4.x, x4.y, x4.z, x4.w}, ha[4] = {h4.x, h4.y, h4.z, h4.w};
      const uint32_t nv = cd.len - e < 4u ? cd.len - e : 4u;
      drift_acc(acc, xa, ha, nv);
    }
  }
  const double total = block_sum(acc, ws);
  if (threadIdx.x == 0) T.partials[(size_t)r * T.C + c] = total;
}

// DIST: 0 normal (one Philox block per float4), 1 Student-t(3) (one block per element).
// GRADBUF: gradients come from a caller buffer.  NORM: also write the chunk's squared drift.
template <int SWEEPS, int DIST, bool GRADBUF, bool NORM>
__global__ __launch_bounds__(kThreads) void k_update(Tables T, StepArgs A) {
  __shared__ double ws[4];
  const uint32_t c = blockIdx.x, r = blockIdx.y;
  const ChunkDesc cd = T.chunks[c];
  const uint32_t seg = r * T.L + cd.layer;
  const bool vl = T.valid_l[seg] != 0, vr = T.valid_r[seg] != 0;
  const size_t base = (size_t)r * T.Npad + cd.off;
  const float third = 0.333333343f;   // (float)(1/3): the ring's mixing weight
  float sg = 0.0f;
  bool spike = false;
  if (!GRADBUF) {
    sg = (float)(T.layers[cd.layer].sig_base * A.decay_pow);
    if (A.spike_prob > 0.0f) {
      const Rand4 sp = philox(0u, 0xFFFFFFFFu, A.k, r, A.key0, A.key1);
      spike = unit_open(sp.w[0]) < A.spike_prob;
    }
  }
  double acc = 0.0;
#pragma unroll
  for (int it = 0; it < SWEEPS; ++it) {
    const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
    if (e < cd.len) {
      const float4 x4 = ld4(T.x + base + e), v4 = ld4(T.vel + base + e);
      float4 l4 = make_float4(0.f, 0.f, 0.f, 0.f), r4 = l4, h4 = l4;
      if (vl) l4 = ld4(T.mbox_l + base + e);
      if (vr) r4 = ld4(T.mbox_r + base + e);
      if (NORM) h4 = ld4(T.xhat + base + e);
      float g[4];
      if (GRADBUF) {
        const float4 g4 = ld4(A.grad + base + e);
        g[0] = g4.x; g[1] = g4.y; g[2] = g4.z; g[3] = g4.w;
      } else if (DIST == 0) {
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
      if (!GRADBUF && spike) {
#pragma unroll
        for (int i = 0; i < 4; ++i) g[i] = g[i] * A.spike_gain;
      }
      float xa[4] = {x4.x, x4.y, x4.z, x4.w}, va[4] = {v4.x, v4.y, v4.z, v4.w};
      const float la[4] = {l4.x, l4.y, l4.z, l4.w}, ra[4] = {r4.x, r4.y, r4.z, r4.w};
      const float ha[4] = {h4.x, h4.y, h4.z, h4.w};
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
      if (NORM) drift_acc(acc, xa, ha, nv);
    }
  }
  if (NORM) {
    const double total = block_sum(acc, ws);
    if (threadIdx.x == 0) T.partials[(size_t)r * T.C + c] = total;
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

hipError_t launch_norm(const Tables& t, uint32_t chunk_elems, hipStream_t s) {
  const dim3 grid(t.C, t.P), block(kThreads);
  switch (chunk_elems / kSweep) {
    case 1: k_norm<1><<<grid, block, 0, s>>>(t); break;
    case 2: k_norm<2><<<grid, block, 0, s>>>(t); break;
    case 4: k_norm<4><<<grid, block, 0, s>>>(t); break;
    case 8: k_norm<8><<<grid, block, 0, s>>>(t); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int SWEEPS>
static void launch_update_s(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                            bool norm, hipStream_t s) {
  const dim3 grid(t.C, t.P), block(kThreads);
  if (grad_mode == 1) {
    if (norm) k_update<SWEEPS, 0, true, true><<<grid, block, 0, s>>>(t, a);
    else k_update<SWEEPS, 0, true, false><<<grid, block, 0, s>>>(t, a);
  } else if (dist == 0) {
    if (norm) k_update<SWEEPS, 0, false, true><<<grid, block, 0, s>>>(t, a);
    else k_update<SWEEPS, 0, false, false><<<grid, block, 0, s>>>(t, a);
  } else {
    if (norm) k_update<SWEEPS, 1, false, true><<<grid, block, 0, s>>>(t, a);
    else k_update<SWEEPS, 1, false, false><<<grid, block, 0, s>>>(t, a);
  }
}

hipError_t launch_update(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t dist,
                         uint32_t grad_mode, bool fused_norm, hipStream_t s) {
  switch (chunk_elems / kSweep) {
    case 1: launch_update_s<1>(t, a, dist, grad_mode, fused_norm, s); break;
    case 2: launch_update_s<2>(t, a, dist, grad_mode, fused_norm, s); break;
    case 4: launch_update_s<4>(t, a, dist, grad_mode, fused_norm, s); break;
    case 8: launch_update_s<8>(t, a, dist, grad_mode, fused_norm, s); break;
    default: return hipErrorInvalidValue;
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
