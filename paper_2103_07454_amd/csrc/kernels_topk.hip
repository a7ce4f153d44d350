// Top-K sparsified sends (Section 7): on an event only the K elements of largest
// rank key travel, with their indices.  The winning set is unique: keys descending,
// ties to the lower index.  Everything here is integer work on 31-bit keys (bit
// patterns of non-negative floats), so results are exact and repeatable.
//
//   select   radix search for the K-th largest key t of every fired tensor in three
//            passes of 11 + 11 + 9 bits: per-chunk LDS histograms, merged into the
//            tensor's global histogram with integer atomics; one workgroup per
//            tensor then walks the histogram from the top.
//            Then per chunk the number of keys > t and == t, and per tensor the
//            running totals over its chunks.
//   send     per chunk a stable compaction of the winners (key > t, or key == t
//            while fewer than T equal keys precede it in the tensor) into the
//            tensor's (index, value) message in ascending index order, updating
//            xhat at the same entries; then the put: the message is read back and
//            scattered into the two neighbours' dense mailboxes.
#include "evg_device.h"

namespace evg {

__device__ __forceinline__ float4 ld4c(const float* p) { return *reinterpret_cast<const float4*>(p); }

// PASS 0: bits 30..20, PASS 1: bits 19..9 under the prefix found so far, PASS 2: bits 8..0.
template <int PASS, int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_topk_hist(Tables T, StepArgs A) {
  constexpr int NB = PASS == 2 ? 512 : kHistBins;
  __shared__ uint32_t h[NB];
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = T.work_topk[i];
    const uint32_t r = w / T.C, c = w % T.C;
    const ChunkDesc cd = T.chunks[c];
    const uint32_t seg = r * T.L + cd.layer;
    const uint32_t prefix = PASS == 0 ? 0u : T.sel_prefix[seg];
    const size_t base = (size_t)r * T.Npad + cd.off;
    for (uint32_t b = threadIdx.x; b < (uint32_t)NB; b += kThreads) h[b] = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SWEEPS; ++it) {
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      if (e < cd.len) {
        const float4 x4 = ld4c(T.x + base + e);
        float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!A.topk_key) h4 = ld4c(T.xhat + base + e);
        const float xa[4] = {x4.x, x4.y, x4.z, x4.w}, ha[4] = {h4.x, h4.y, h4.z, h4.w};
        const uint32_t nv = cd.len - e < 4u ? cd.len - e : 4u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((uint32_t)q < nv) {
            const uint32_t key = rank_key(xa[q], ha[q], A.topk_key);
            if (PASS == 0) atomicAdd(&h[key >> 20], 1u);
            else if (PASS == 1) { if ((key >> 20) == prefix) atomicAdd(&h[(key >> 9) & 2047u], 1u); }
            else { if ((key >> 9) == prefix) atomicAdd(&h[key & 511u], 1u); }
          }
        }
      }
    }
    __syncthreads();
    uint32_t* gh = T.hist + (size_t)seg * kHistBins;
    for (uint32_t b = threadIdx.x; b < (uint32_t)NB; b += kThreads) {
      const uint32_t v = h[b];
      if (v) atomicAdd(&gh[b], v);
    }
    __syncthreads();
  }
}

// One workgroup per tensor that sends a Top-K message: find the bin that holds the
// krem-th largest key, append it to the prefix, keep what is still to be taken
// inside that bin, and clear the histogram for the next pass.
template <int PASS>
__global__ __launch_bounds__(kThreads) void k_topk_pick(Tables T) {
  constexpr int NB = PASS == 2 ? 512 : kHistBins;
  constexpr int PER = NB / kThreads;
  __shared__ uint32_t ws[4];
  const uint32_t seg = blockIdx.x;
  if (T.fired[seg] != 2) return;    // uniform for the workgroup
  const uint32_t krem = PASS == 0 ? T.layers[seg % T.L].K : T.sel_krem[seg];
  uint32_t* gh = T.hist + (size_t)seg * kHistBins;
  const uint32_t top = NB - 1 - threadIdx.x * PER;   // this thread's highest bin
  uint32_t cnt[PER], local = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    cnt[j] = gh[top - j];
    gh[top - j] = 0;
    local += cnt[j];
  }
  uint32_t total;
  const uint32_t above = block_excl_scan<4>(local, ws, &total);   // keys in higher bins
  if (above < krem && krem <= above + local) {    // exactly one thread
    uint32_t run = above, bin = top, rem = krem - above;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (run < krem && krem <= run + cnt[j]) { bin = top - j; rem = krem - run; }
      run += cnt[j];
    }
    const uint32_t prefix = PASS == 0 ? 0u : T.sel_prefix[seg];
    T.sel_prefix[seg] = PASS == 0 ? bin : PASS == 1 ? ((prefix << 11) | bin) : ((prefix << 9) | bin);
    T.sel_krem[seg] = rem;
  }
}

// Per chunk: how many keys exceed / equal the threshold key.
template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_topk_count(Tables T, StepArgs A) {
  __shared__ uint32_t ws[4];
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = T.work_topk[i];
    const uint32_t r = w / T.C, c = w % T.C;
    const ChunkDesc cd = T.chunks[c];
    const uint32_t t = T.sel_prefix[r * T.L + cd.layer];
    const size_t base = (size_t)r * T.Npad + cd.off;
    uint32_t packed = 0;    // greater in the low half, equal in the high half (both <= 8192)
#pragma unroll
    for (int it = 0; it < SWEEPS; ++it) {
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      if (e < cd.len) {
        const float4 x4 = ld4c(T.x + base + e);
        float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!A.topk_key) h4 = ld4c(T.xhat + base + e);
        const float xa[4] = {x4.x, x4.y, x4.z, x4.w}, ha[4] = {h4.x, h4.y, h4.z, h4.w};
        const uint32_t nv = cd.len - e < 4u ? cd.len - e : 4u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((uint32_t)q < nv) {
            const uint32_t key = rank_key(xa[q], ha[q], A.topk_key);
            packed += (key > t ? 1u : 0u) + (key == t ? 0x10000u : 0u);
          }
        }
      }
    }
    uint32_t total;
    (void)block_excl_scan<4>(packed, ws, &total);
    if (threadIdx.x == 0) T.chunk_cnt[w] = make_uint2(total & 0xFFFFu, total >> 16);
  }
}

// One wavefront per Top-K tensor: running totals over its chunks, in chunk order.
__global__ __launch_bounds__(64) void k_topk_chunkscan(Tables T) {
  const uint32_t seg = blockIdx.x;
  if (T.fired[seg] != 2) return;
  const uint32_t r = seg / T.L;
  const LayerDesc ld = T.layers[seg % T.L];
  const uint32_t ties = T.sel_krem[seg];
  const uint32_t first = r * T.C + ld.chunk0;
  uint32_t carry_g = 0, carry_e = 0;
  for (uint32_t b = 0; b < ld.nchunks; b += 64) {
    const uint32_t i = b + threadIdx.x;
    uint2 ce = make_uint2(0, 0);
    if (i < ld.nchunks) ce = T.chunk_cnt[first + i];
    const uint32_t ig = wave_incl_scan(ce.x), ie = wave_incl_scan(ce.y);
    const uint32_t gb = carry_g + ig - ce.x, eb = carry_e + ie - ce.y;
    if (i < ld.nchunks) {
      const uint32_t take_e = eb >= ties ? 0u : (ties - eb < ce.y ? ties - eb : ce.y);
      T.chunk_before[first + i] = make_uint2(gb, eb);
      T.chunk_out[first + i] = make_uint2(gb + (eb < ties ? eb : ties), ce.x + take_e);
    }
    carry_g += __shfl(ig, 63, 64);
    carry_e += __shfl(ie, 63, 64);
  }
}

// Stable compaction of a chunk's winners into the tensor's message; xhat takes the
// sent values (only those entries were communicated).
template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_topk_pack(Tables T, StepArgs A) {
  __shared__ uint32_t ws[4];
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = T.work_topk[i];
    const uint32_t r = w / T.C, c = w % T.C;
    const ChunkDesc cd = T.chunks[c];
    const uint32_t seg = r * T.L + cd.layer;
    const uint32_t t = T.sel_prefix[seg], ties = T.sel_krem[seg];
    const uint2 before = T.chunk_before[w];
    const size_t base = (size_t)r * T.Npad + cd.off;
    const size_t mbase = (size_t)r * T.Ktot + T.layers[cd.layer].msg_off;
    uint32_t run_g = before.x, run_e = before.y;
    for (int it = 0; it < SWEEPS; ++it) {          // uniform trip count: scans need every thread
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      float xa[4] = {0.f, 0.f, 0.f, 0.f}, ha[4] = {0.f, 0.f, 0.f, 0.f};
      uint32_t isg = 0, ise = 0, nv = 0;
      if (e < cd.len) {
        const float4 x4 = ld4c(T.x + base + e), h4 = ld4c(T.xhat + base + e);
        xa[0] = x4.x; xa[1] = x4.y; xa[2] = x4.z; xa[3] = x4.w;
        ha[0] = h4.x; ha[1] = h4.y; ha[2] = h4.z; ha[3] = h4.w;
        nv = cd.len - e < 4u ? cd.len - e : 4u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((uint32_t)q < nv) {
            const uint32_t key = rank_key(xa[q], ha[q], A.topk_key);
            isg |= (key > t ? 1u : 0u) << q;
            ise |= (key == t ? 1u : 0u) << q;
          }
        }
      }
      const uint32_t mine = __popc(isg) + (__popc(ise) << 16);
      uint32_t total;
      const uint32_t ex = block_excl_scan<4>(mine, ws, &total);
      uint32_t g = run_g + (ex & 0xFFFFu), q_e = run_e + (ex >> 16);
      bool any = false;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const bool bg = (isg >> q) & 1u, be = (ise >> q) & 1u;
        const bool win = bg || (be && q_e < ties);
        if (win) {
          const uint32_t pos = g + (q_e < ties ? q_e : ties);
          T.msg_idx[mbase + pos] = cd.j0 + e + q;
          T.msg_val[mbase + pos] = xa[q];
          ha[q] = xa[q];
          any = true;
        }
        g += bg ? 1u : 0u;
        q_e += be ? 1u : 0u;
      }
      if (any) *reinterpret_cast<float4*>(T.xhat + base + e) = make_float4(ha[0], ha[1], ha[2], ha[3]);
      run_g += total & 0xFFFFu;
      run_e += total >> 16;
    }
  }
}

// The put: each chunk's slice of the message is scattered into the receivers' dense copies.
__global__ __launch_bounds__(kThreads) void k_topk_put(Tables T) {
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const uint32_t w = T.work_topk[i];
    const uint32_t r = w / T.C, c = w % T.C;
    const LayerDesc ld = T.layers[T.chunks[c].layer];
    const uint2 out = T.chunk_out[w];
    const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
    const size_t mbase = (size_t)r * T.Ktot + ld.msg_off + out.x;
    float* toR = T.mbox_r + (size_t)left * T.Npad + ld.off;
    float* toL = T.mbox_l + (size_t)right * T.Npad + ld.off;
    for (uint32_t q = threadIdx.x; q < out.y; q += kThreads) {
      const uint32_t j = T.msg_idx[mbase + q];
      const float v = T.msg_val[mbase + q];
      toR[j] = v;
      toL[j] = v;
    }
  }
}

template <int SWEEPS>
static void select_s(const Tables& t, const StepArgs& a, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kThreads), segs(t.S);
  k_topk_hist<0, SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_pick<0><<<segs, b, 0, s>>>(t);
  k_topk_hist<1, SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_pick<1><<<segs, b, 0, s>>>(t);
  k_topk_hist<2, SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_pick<2><<<segs, b, 0, s>>>(t);
  k_topk_count<SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_chunkscan<<<segs, dim3(64), 0, s>>>(t);
}

hipError_t launch_topk_select(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid,
                              hipStream_t s) {
  switch (chunk_elems / kSweep) {
    case 1: select_s<1>(t, a, grid, s); break;
    case 2: select_s<2>(t, a, grid, s); break;
    case 4: select_s<4>(t, a, grid, s); break;
    case 8: select_s<8>(t, a, grid, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_topk_send(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid,
                            hipStream_t s) {
  const dim3 g(grid), b(kThreads);
  switch (chunk_elems / kSweep) {
    case 1: k_topk_pack<1><<<g, b, 0, s>>>(t, a); break;
    case 2: k_topk_pack<2><<<g, b, 0, s>>>(t, a); break;
    case 4: k_topk_pack<4><<<g, b, 0, s>>>(t, a); break;
    case 8: k_topk_pack<8><<<g, b, 0, s>>>(t, a); break;
    default: return hipErrorInvalidValue;
  }
  k_topk_put<<<g, b, 0, s>>>(t);
  return hipGetLastError();
}

}  // namespace evg
