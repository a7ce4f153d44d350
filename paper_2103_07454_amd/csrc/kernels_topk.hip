// Top-K sparsified sends (Section 7): on an event only the K elements of largest
// rank key travel, with their indices.  The winning set is unique: keys descending,
// ties to the lower index.  Everything here is integer work on 31-bit keys (bit
// patterns of non-negative floats), so results are exact and repeatable.
//
// Only two kernels read the fired tensors themselves (x and xhat):
//   k_topk_hist   pass A: per-chunk LDS histogram of key bits 30..20, merged into the
//                 tensor's histogram with integer atomics; k_topk_pick<0> then finds
//                 the bin b that holds the K-th largest key.
//   k_topk_stage  copies every element whose bin is >= b ("staged": all possible
//                 winners, roughly K plus one bin's worth) as (index, value) into
//                 the chunk's staging slot in ascending index order, marks those IN bin b
//                 (bit 31 of the index), keeps the keys of the marked ones in a list of
//                 their own, and histograms bits 19..9 of those keys.  Entries above bin b
//                 win whatever the exact threshold turns out to be, so their keys are dropped.
// The rest works on the staged entries only, a small fraction of the tensor:
//   k_topk_hist_low   bits 8..0 of the in-bin keys under the 22-bit prefix -> threshold key t
//                     and T = how many keys equal to t are still needed
//   k_topk_count      per chunk: staged entries above bin b + in-bin keys > t, and in-bin keys == t
//   k_topk_chunkscan  running totals over a tensor's chunks (one wavefront per tensor)
//   k_topk_pack       stable compaction of the winners (key > t, or key == t while fewer
//                     than T equal keys precede it in the tensor) into the tensor's
//                     (index, value) message, ascending indices.
// The message is applied to xhat and to the neighbours' mailboxes by the update pass.
#include "evg_device.h"

namespace evg {

struct WorkItem {
  uint32_t w, r, c, seg;
  ChunkDesc cd;
  size_t base;   // arena offset of the chunk
  size_t slot;   // where the chunk's staged entries start in the staging arrays
  uint32_t cap;  // how many entries the slot holds
};

// A chunk whose possible winners do not fit its staging slot is marked with this count and
// staged not at all: the kernels that would read its staged entries read the chunk's elements
// from the arenas instead (exact all the same; it takes massive ties or a large Top-K share).
constexpr uint32_t kNotStaged = 0xFFFFFFFFu;

__device__ __forceinline__ WorkItem work_item(const Tables& T, uint32_t i) {
  WorkItem it;
  it.w = T.work_topk[i];
  it.r = it.w / T.C;
  it.c = it.w % T.C;
  it.cd = T.chunks[it.c];
  it.seg = it.r * T.L + it.cd.layer;
  it.base = (size_t)it.r * T.Npad + it.cd.off;
  // a slot holds stage_num of every 16 elements of the chunk's range; slots of neighbouring
  // chunks cannot overlap (floor(a/16) + floor(len/16) <= floor((a + len)/16)) and start on
  // multiples of 4 entries (stage_num is 4, 8, 12 or 16), i.e. 16-byte aligned
  it.slot = (size_t)it.r * T.stage_stride + (size_t)(it.cd.off >> 4) * T.stage_num;
  it.cap = (it.cd.len >> 4) * T.stage_num;
  return it;
}

// Adds the non-empty bins of a workgroup's LDS histogram to the tensor's histogram.
template <int NB>
__device__ __forceinline__ void flush_hist(const uint32_t* h, uint32_t* gh) {
  for (uint32_t b = threadIdx.x; b < (uint32_t)NB; b += kThreads) {
    const uint32_t v = h[b];
    if (v) atomicAdd(&gh[b], v);
  }
}

template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_topk_hist(Tables T, StepArgs A) {
  __shared__ uint32_t h[kHistBins];
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const WorkItem wi = work_item(T, i);
    for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) h[b] = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < SWEEPS; ++it) {
      const uint32_t e = it * kSweep + threadIdx.x * kLaneElems;
      if (e < wi.cd.len) {
        const float4 x4 = ld4s(T.x + wi.base + e);
        float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!A.topk_key) h4 = ld4s(T.xhat + wi.base + e);
        const float xa[4] = {x4.x, x4.y, x4.z, x4.w}, ha[4] = {h4.x, h4.y, h4.z, h4.w};
        const uint32_t nv = wi.cd.len - e < 4u ? wi.cd.len - e : 4u;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if ((uint32_t)q < nv) atomicAdd(&h[rank_key(xa[q], ha[q], A.topk_key) >> 20], 1u);
      }
    }
    __syncthreads();
    flush_hist<kHistBins>(h, T.hist + (size_t)wi.seg * kHistBins);
    __syncthreads();
  }
}

// One workgroup per tensor that sends a Top-K message: find the bin that holds the
// krem-th largest key, append it to the prefix, keep what is still to be taken
// inside that bin, and clear the histogram for the next pass.
// PASS 0: bits 30..20, PASS 1: bits 19..9, PASS 2: bits 8..0.
template <int PASS>
__global__ __launch_bounds__(kThreads) void k_topk_pick(Tables T) {
  constexpr int NB = PASS == 2 ? 512 : kHistBins;
  constexpr int PER = NB / kThreads;
  __shared__ uint32_t ws[4];
  const uint32_t seg = blockIdx.x;
  uint32_t* gh = T.hist + (size_t)seg * kHistBins;
  if (T.fired[seg] != 2) {          // uniform for the workgroup
    // pass A histograms are built for every tensor when the update pass makes them:
    // those of tensors that stay silent are simply dropped
    if (PASS == 0)
      for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) gh[b] = 0;
    return;
  }
  const uint32_t krem = PASS == 0 ? T.layers[seg % T.L].K : T.sel_krem[seg];
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

// Up to four sweeps (16 elements per thread) share one workgroup scan, so that more
// loads are in flight between barriers: the four per-sweep counts travel as 16-bit
// fields of one 64-bit word (a sweep stages at most 1024 entries).  The entries are
// compacted in LDS and written out once per chunk.
//
// What is staged per chunk, both lists in ascending index order in the chunk's staging slot
// (a share of the chunk's length; a chunk with more possible winners than that is marked and
// left to the arena paths of the kernels below):
//   (index | in-bin flag in bit 31, value)  for every element whose bin is >= b: all possible winners;
//   key                                     for those of them whose bin IS b (flag set): only they
//                                           still have to be compared with the exact threshold,
//                                           everything above bin b wins whatever the threshold is.
template <int SWEEPS>
__global__ __launch_bounds__(kThreads) void k_topk_stage(Tables T, StepArgs A) {
  constexpr int STEP = SWEEPS >= 4 ? 4 : SWEEPS;
  __shared__ uint32_t h[kHistBins];
  __shared__ uint64_t ws[8];
  // a chunk's staged entries are gathered here and leave as whole 16-byte streaming stores
  // (scattered 4-byte stores straight to memory measured 12 % slower for the kernel); a chunk
  // that stages more than the buffers hold falls back to direct stores
  constexpr uint32_t kCap = kStageCap, kCapB = kStageCapBin;
  __shared__ __attribute__((aligned(16))) uint32_t li[kCap], lb[kCapB];
  __shared__ __attribute__((aligned(16))) float lv[kCap];
  const uint32_t n = T.counts[1];
  for (uint32_t i = blockIdx.x; i < n; i += gridDim.x) {
    const WorkItem wi = work_item(T, i);
    const uint32_t bin = T.sel_prefix[wi.seg];
    for (uint32_t b = threadIdx.x; b < (uint32_t)kHistBins; b += kThreads) h[b] = 0;
    __syncthreads();
    uint32_t run = 0, runb = 0;   // staged so far: all entries, in-bin entries
    bool direct = false;          // uniform: this chunk overflowed an LDS buffer
    bool over = false;            // uniform: this chunk overflowed its staging slot, nothing more is staged
    for (int it = 0; it < SWEEPS; it += STEP) {   // uniform trip count: the scan needs every thread
      float xa[STEP][4];
      uint32_t key[STEP][4], take[STEP], inb[STEP], e[STEP];
      float4 x4[STEP], h4[STEP];
#pragma unroll
      for (int u = 0; u < STEP; ++u) {
        e[u] = (it + u) * kSweep + threadIdx.x * kLaneElems;
        x4[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        h4[u] = x4[u];
        if (e[u] < wi.cd.len) {
          x4[u] = ld4s(T.x + wi.base + e[u]);
          if (!A.topk_key) h4[u] = ld4s(T.xhat + wi.base + e[u]);
        }
      }
      uint64_t mine = 0, mineb = 0;
#pragma unroll
      for (int u = 0; u < STEP; ++u) {
        take[u] = 0;
        inb[u] = 0;
        xa[u][0] = x4[u].x; xa[u][1] = x4[u].y; xa[u][2] = x4[u].z; xa[u][3] = x4[u].w;
        const float ha[4] = {h4[u].x, h4[u].y, h4[u].z, h4[u].w};
        const uint32_t nv = e[u] >= wi.cd.len ? 0u : (wi.cd.len - e[u] < 4u ? wi.cd.len - e[u] : 4u);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          key[u][q] = 0;
          if ((uint32_t)q < nv) {
            key[u][q] = rank_key(xa[u][q], ha[q], A.topk_key);
            const uint32_t kb = key[u][q] >> 20;
            if (kb >= bin) take[u] |= 1u << q;
            if (kb == bin) {
              inb[u] |= 1u << q;
              atomicAdd(&h[(key[u][q] >> 9) & 2047u], 1u);
            }
          }
        }
        mine |= (uint64_t)__popc(take[u]) << (16 * u);
        mineb |= (uint64_t)__popc(inb[u]) << (16 * u);
      }
      // staged order = index order: all of sweep `it` precedes sweep `it + 1`
      uint64_t total, totalb, ex, exb;
      block_excl_scan64x2<4>(mine, mineb, ws, &ex, &exb, &total, &totalb);
      uint32_t before = run, beforeb = runb;   // entries of this chunk's earlier sweeps
      uint32_t all = 0, allb = 0;
#pragma unroll
      for (int u = 0; u < STEP; ++u) {
        all += (uint32_t)((total >> (16 * u)) & 0xFFFFu);
        allb += (uint32_t)((totalb >> (16 * u)) & 0xFFFFu);
      }
      if (run + all > wi.cap) over = true;      // uniform (in-bin entries are among them: they fit if these do)
      if (over) continue;                       // only the histogram above still matters for this chunk
      if (!direct && (run + all > kCap || runb + allb > kCapB)) {   // uniform: empty the buffers and go direct
        __syncthreads();
        for (uint32_t q = threadIdx.x; q < run; q += kThreads) {
          T.stage_idx[wi.slot + q] = li[q];
          T.stage_val[wi.slot + q] = lv[q];
        }
        for (uint32_t q = threadIdx.x; q < runb; q += kThreads) T.stage_key[wi.slot + q] = lb[q];
        direct = true;
      }
#pragma unroll
      for (int u = 0; u < STEP; ++u) {
        uint32_t pos = before + (uint32_t)((ex >> (16 * u)) & 0xFFFFu);
        uint32_t posb = beforeb + (uint32_t)((exb >> (16 * u)) & 0xFFFFu);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((take[u] >> q) & 1u) {
            const uint32_t flag = (inb[u] >> q) & 1u;
            const uint32_t jf = (wi.cd.j0 + e[u] + q) | (flag << 31);
            if (!direct) {
              li[pos] = jf;
              lv[pos] = xa[u][q];
              if (flag) lb[posb] = key[u][q];
            } else {
              T.stage_idx[wi.slot + pos] = jf;
              T.stage_val[wi.slot + pos] = xa[u][q];
              if (flag) T.stage_key[wi.slot + posb] = key[u][q];
            }
            ++pos;
            posb += flag;
          }
        }
        before += (uint32_t)((total >> (16 * u)) & 0xFFFFu);
        beforeb += (uint32_t)((totalb >> (16 * u)) & 0xFFFFu);
      }
      run = before;
      runb = beforeb;
    }
    if (threadIdx.x == 0) {
      T.stage_n[wi.w] = over ? make_uint2(kNotStaged, 0u) : make_uint2(run, runb);
      if (over) atomicAdd(&T.counts[3], 1u);     // running count, reported by evg_stats
    }
    __syncthreads();
    if (!direct && !over) {
      // the chunk's slot starts 16-byte aligned: whole quads stream out, the tail goes singly
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      const uint32_t quads = run / 4, quadsb = runb / 4;
      for (uint32_t q = threadIdx.x; q < quads; q += kThreads) {
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(li + 4 * q),
                                    reinterpret_cast<u32x4*>(T.stage_idx + wi.slot) + q);
        __builtin_nontemporal_store(*reinterpret_cast<const f32x4*>(lv + 4 * q),
                                    reinterpret_cast<f32x4*>(T.stage_val + wi.slot) + q);
      }
      for (uint32_t q = threadIdx.x; q < quadsb; q += kThreads)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(lb + 4 * q),
                                    reinterpret_cast<u32x4*>(T.stage_key + wi.slot) + q);
      for (uint32_t q = 4 * quads + threadIdx.x; q < run; q += kThreads) {
        T.stage_idx[wi.slot + q] = li[q];
        T.stage_val[wi.slot + q] = lv[q];
      }
      for (uint32_t q = 4 * quadsb + threadIdx.x; q < runb; q += kThreads) T.stage_key[wi.slot + q] = lb[q];
    }

    flush_hist<kHistBins>(h, T.hist + (size_t)wi.seg * kHistBins);
    __syncthreads();
  }
}

// The three kernels below walk a chunk's staged entries, a thousand or so, so
// one wavefront per chunk does it without LDS or workgroup barriers: ballots give
// counts and ranks.  Four independent wavefronts share a workgroup.

__device__ __forceinline__ uint32_t wave_slot() { return blockIdx.x * (kThreads / 64) + wave_id(); }
__device__ __forceinline__ uint32_t wave_slots() { return gridDim.x * (kThreads / 64); }
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
  return __popcll(mask & ((1ull << lane_id()) - 1ull));
}

// Finaliser of the SplitMix64 generator (Steele, Lea, Flood, OOPSLA'14): used to turn a
// message entry into 64 well-mixed bits, so that the sum over a message's entries is a
// fingerprint of the message that does not depend on the order of summation.
__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Rank key and value of element q of a chunk, straight from the arenas (chunks that were not staged).
__device__ __forceinline__ uint32_t arena_key(const Tables& T, const WorkItem& wi, uint32_t q, uint32_t by_value,
                                              float* xv) {
  const float x = T.x[wi.base + q];
  const float h = by_value ? 0.0f : T.xhat[wi.base + q];
  *xv = x;
  return rank_key(x, h, by_value);
}

constexpr int kBatch = 8;    // 64-entry groups loaded together by a wavefront, to overlap their latency

// Bits 8..0 of the in-bin keys that carry the 22-bit prefix found so far.  Matches are
// rare (a 2^-22 slice of the key range), so they go straight to the tensor's histogram,
// one atomic per distinct value per 64 entries.
__global__ __launch_bounds__(kThreads) void k_topk_hist_low(Tables T, StepArgs A) {
  const uint32_t n = T.counts[1];
  for (uint32_t i = wave_slot(); i < n; i += wave_slots()) {
    const WorkItem wi = work_item(T, i);
    const uint2 sn = T.stage_n[wi.w];
    const bool staged = sn.x != kNotStaged;             // wave-uniform
    const uint32_t prefix = T.sel_prefix[wi.seg], ns = staged ? sn.y : wi.cd.len;
    uint32_t* gh = T.hist + (size_t)wi.seg * kHistBins;
    for (uint32_t q0 = 0; q0 < ns; q0 += 64 * kBatch) {
      uint32_t key[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint32_t q = q0 + u * 64 + lane_id();
        key[u] = 0xFFFFFFFFu;                           // no key has bit 31: never matches
        float unused;
        if (q < ns) key[u] = staged ? T.stage_key[wi.slot + q] : arena_key(T, wi, q, A.topk_key, &unused);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        bool pending = (key[u] >> 9) == prefix;
        uint64_t todo = __ballot(pending);
        while (todo) {                                  // uniform: every lane sees the same mask
          const uint32_t leader = __ffsll((unsigned long long)todo) - 1;
          const uint32_t v = __shfl(key[u] & 511u, leader, 64);
          const uint64_t same = __ballot(pending && (key[u] & 511u) == v);
          if (lane_id() == leader) atomicAdd(&gh[v], (uint32_t)__popcll(same));
          if ((same >> lane_id()) & 1ull) pending = false;
          todo &= ~same;
        }
      }
    }
  }
}

// Per chunk: how many staged keys exceed / equal the threshold key.  Every key above
// the threshold is staged (its bin is >= the threshold's), so these are the chunk's counts;
// entries staged without a key lie above the threshold's bin and exceed it.
__global__ __launch_bounds__(kThreads) void k_topk_count(Tables T, StepArgs A) {
  const uint32_t n = T.counts[1];
  for (uint32_t i = wave_slot(); i < n; i += wave_slots()) {
    const WorkItem wi = work_item(T, i);
    const uint32_t t = T.sel_prefix[wi.seg];
    const uint2 sn = T.stage_n[wi.w];
    const bool staged = sn.x != kNotStaged;             // wave-uniform
    const uint32_t ns = staged ? sn.y : wi.cd.len;
    uint32_t g = staged ? sn.x - sn.y : 0u, e = 0;
    for (uint32_t q0 = 0; q0 < ns; q0 += 64 * kBatch) {
      uint32_t key[kBatch];
      bool in[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const uint32_t q = q0 + u * 64 + lane_id();
        in[u] = q < ns;
        key[u] = 0u;
        float unused;
        if (in[u]) key[u] = staged ? T.stage_key[wi.slot + q] : arena_key(T, wi, q, A.topk_key, &unused);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        g += __popcll(__ballot(in[u] && key[u] > t));
        e += __popcll(__ballot(in[u] && key[u] == t));
      }
    }
    if (lane_id() == 0) T.chunk_cnt[wi.w] = make_uint2(g, e);
  }
}

// One wavefront per Top-K tensor: running totals over its chunks, in chunk order.
__global__ __launch_bounds__(64) void k_topk_chunkscan(Tables T) {
  const uint32_t seg = blockIdx.x;
  if (T.fired[seg] != 2) return;
  const uint32_t r = seg / T.L;
  const LayerDesc ld = T.layers[seg % T.L];
  const uint32_t first = r * T.C + ld.chunk0;
  uint32_t carry_g = 0, carry_e = 0;
  for (uint32_t b = 0; b < ld.nchunks; b += 64) {
    const uint32_t i = b + threadIdx.x;
    uint2 ce = make_uint2(0, 0);
    if (i < ld.nchunks) ce = T.chunk_cnt[first + i];
    const uint32_t ig = wave_incl_scan(ce.x), ie = wave_incl_scan(ce.y);
    const uint32_t gb = carry_g + ig - ce.x, eb = carry_e + ie - ce.y;
    if (i < ld.nchunks) T.chunk_before[first + i] = make_uint2(gb, eb);
    carry_g += __shfl(ig, 63, 64);
    carry_e += __shfl(ie, 63, 64);
  }
}

// Stable compaction of a chunk's winners from its staged entries into the tensor's
// message.  Also records where each 1024-element sweep of the chunk starts in the
// message, so that the update pass can fetch exactly its part.
__global__ __launch_bounds__(kThreads) void k_topk_pack(Tables T, StepArgs A) {
  const uint32_t n = T.counts[1];
  for (uint32_t i = wave_slot(); i < n; i += wave_slots()) {
    const WorkItem wi = work_item(T, i);
    const uint32_t t = T.sel_prefix[wi.seg], ties = T.sel_krem[wi.seg];
    const bool staged = T.stage_n[wi.w].x != kNotStaged;           // wave-uniform
    const uint32_t ns = staged ? T.stage_n[wi.w].x : wi.cd.len;
    const uint2 before = T.chunk_before[wi.w];
    const size_t mbase = (size_t)wi.r * T.Ktot + T.layers[wi.cd.layer].msg_off;
    uint32_t* sub = T.chunk_sub + (size_t)wi.w * (T.SW + 1);
    const uint32_t first = before.x + (before.y < ties ? before.y : ties);   // the chunk's first slot
    uint32_t run_g = before.x, run_e = before.y;
    uint32_t run_b = 0;                                 // in-bin entries of this chunk met so far
    uint32_t per_sweep[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // winners per sweep (wave-uniform)
    for (uint32_t q0 = 0; q0 < ns; q0 += 64 * kBatch) {
      uint32_t key[kBatch], j[kBatch];
      float val[kBatch];
      bool in[kBatch], flag[kBatch];
      if (staged) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const uint32_t q = q0 + u * 64 + lane_id();
          in[u] = q < ns;
          j[u] = in[u] ? T.stage_idx[wi.slot + q] : wi.cd.j0;
          val[u] = in[u] ? T.stage_val[wi.slot + q] : 0.0f;   // most staged entries win: fetch with the indices
        }
        // an entry with the in-bin flag finds its key in the chunk's key list, at its rank among
        // the flagged entries; the others lie above the threshold's bin (any key above t will do)
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          flag[u] = (j[u] >> 31) != 0u;
          j[u] &= 0x7FFFFFFFu;
          const uint64_t mf = __ballot(flag[u]);
          key[u] = 0xFFFFFFFFu;
          if (flag[u]) key[u] = T.stage_key[wi.slot + run_b + lanes_below(mf)];
          run_b += __popcll(mf);
        }
      } else {
        // not staged: every element of the chunk, keys recomputed from the arenas
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const uint32_t q = q0 + u * 64 + lane_id();
          in[u] = q < ns;
          j[u] = wi.cd.j0 + (in[u] ? q : 0u);
          val[u] = 0.0f;
          key[u] = 0u;
          if (in[u]) key[u] = arena_key(T, wi, q, A.topk_key, &val[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {                // groups in index order
        const bool isg = in[u] && key[u] > t, ise = in[u] && key[u] == t;
        const uint64_t mg = __ballot(isg), me = __ballot(ise);
        const uint32_t g = run_g + lanes_below(mg), eq = run_e + lanes_below(me);
        const bool win = isg || (ise && eq < ties);
        if (win) {
          const uint32_t pos = g + (eq < ties ? eq : ties);
          T.msg_idx[mbase + pos] = j[u];
          T.msg_val[mbase + pos] = val[u];
        }
        // entries ascend, so a group of 64 touches only the sweeps between its first and its last
        // entry's (all three values below are wave-uniform)
        const uint32_t sw = (j[u] - wi.cd.j0) / (uint32_t)kSweep;
        const uint64_t mi = __ballot(in[u]);
        const uint32_t last = mi ? 63u - (uint32_t)__builtin_clzll(mi) : 0u;
        const uint32_t sw_lo = __shfl(sw, 0, 64), sw_hi = __shfl(sw, last, 64);
#pragma unroll
        for (uint32_t s2 = 0; s2 < 8; ++s2)
          if (s2 >= sw_lo && s2 <= sw_hi) per_sweep[s2] += __popcll(__ballot(win && sw == s2));
        run_g += __popcll(mg);
        run_e += __popcll(me);
      }
    }
    if (lane_id() == 0) {
      uint32_t at = first;
#pragma unroll
      for (uint32_t s2 = 0; s2 < 8; ++s2)
        if (s2 < T.SW) { sub[s2] = at; at += per_sweep[s2]; }
      sub[T.SW] = at;
    }
  }
}

// Fingerprints of the messages of the last step, computed when asked for (evg_message_hashes):
// one workgroup per (worker, tensor) walks the packed message.  Integer sums: the order of
// summation does not change the result.
__global__ __launch_bounds__(kThreads) void k_message_hashes(Tables T) {
  __shared__ unsigned long long ws[2 * (kThreads / 64)];
  const uint32_t seg = blockIdx.x;
  unsigned long long hi = 0ull, hm = 0ull;
  if (T.fired[seg] == 2) {          // uniform for the workgroup
    const LayerDesc ld = T.layers[seg % T.L];
    const size_t mbase = (size_t)(seg / T.L) * T.Ktot + ld.msg_off;
    for (uint32_t q = threadIdx.x; q < ld.K; q += kThreads) {
      const unsigned long long j = T.msg_idx[mbase + q];
      hi += mix64(j);
      hm += mix64(((unsigned long long)__float_as_uint(T.msg_val[mbase + q]) << 32) | j);
    }
  }
  hi = wave_sum_u64(hi);
  hm = wave_sum_u64(hm);
  if (lane_id() == 0) { ws[wave_id()] = hi; ws[kThreads / 64 + wave_id()] = hm; }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long a = 0ull, b = 0ull;
    for (int w = 0; w < kThreads / 64; ++w) { a += ws[w]; b += ws[kThreads / 64 + w]; }
    T.idx_hash[seg] = a;
    T.msg_hash[seg] = b;
  }
}

hipError_t launch_message_hashes(const Tables& t, hipStream_t s) {
  k_message_hashes<<<dim3(t.S), dim3(kThreads), 0, s>>>(t);
  return hipGetLastError();
}

template <int SWEEPS>
static void select_s(const Tables& t, const StepArgs& a, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kThreads), segs(t.S);
  if (!a.hist_fused) k_topk_hist<SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_pick<0><<<segs, b, 0, s>>>(t);
  k_topk_stage<SWEEPS><<<g, b, 0, s>>>(t, a);
  k_topk_pick<1><<<segs, b, 0, s>>>(t);
  k_topk_hist_low<<<g, b, 0, s>>>(t, a);
  k_topk_pick<2><<<segs, b, 0, s>>>(t);
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

hipError_t launch_topk_send(const Tables& t, const StepArgs& a, uint32_t, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kThreads);
  k_topk_count<<<g, b, 0, s>>>(t, a);
  k_topk_chunkscan<<<dim3(t.S), dim3(64), 0, s>>>(t);
  k_topk_pack<<<g, b, 0, s>>>(t, a);
  return hipGetLastError();
}

}  // namespace evg
