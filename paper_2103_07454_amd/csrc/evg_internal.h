// Internal types shared by the host side of libevg and its gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evg {

constexpr int kThreads = 256;          // 4 wavefronts of 64 lanes
constexpr int kLaneElems = 4;          // one float4 per lane and sweep
constexpr int kSweep = kThreads * kLaneElems;   // elements one workgroup covers per sweep
constexpr int kHistBins = 2048;        // 11 key bits per selection pass (passes A, B); pass C uses 512
constexpr uint32_t kStageCap = 2048;   // staged entries / in-bin keys of a chunk that the staging kernel
constexpr uint32_t kStageCapBin = 1024;   // gathers in LDS before writing them out (more: direct stores)

// A chunk is a run of one tensor's elements that one workgroup handles; it never
// straddles tensors, starts at a multiple of 4 elements and is at most chunk_elems long.
struct ChunkDesc {
  uint32_t off;    // start inside a worker's arena slice (floats, multiple of 4)
  uint32_t len;    // elements (multiple of 4 except a tensor's last chunk)
  uint32_t layer;  // tensor index
  uint32_t j0;     // start inside the tensor (multiple of 4)
};

struct LayerDesc {
  uint32_t off;      // start inside a worker's slice
  uint32_t numel;
  uint32_t chunk0;   // first chunk
  uint32_t nchunks;
  uint32_t K;        // Top-K message length (0 when Top-K is off)
  uint32_t msg_off;  // start of this tensor's message slot inside a worker's staging slice
  double sig_base;   // sigma0 [/ sqrt(fan_in)]
};

// The iteration as the device knows it.  evg_step passes the iteration by value; a step
// that must be replayable from a captured graph (evg_step_next) reads it from here instead.
struct IterState {
  uint32_t k;          // iteration of the step in flight (set by k_begin in replayable steps)
  uint32_t k_next;     // the iteration after the last completed step
  uint64_t iters;      // steps completed
  double decay_pow;    // decay^k for the step in flight (replayable steps)
  uint32_t overflow;   // a replayable step ran past the decay table
  uint32_t pad;
};

// Device pointers and sizes, passed to kernels by value.
struct Tables {
  const ChunkDesc* chunks;
  const LayerDesc* layers;
  float* x; float* xhat; float* mbox_l; float* mbox_r; float* vel;
  float* xsnap;            // [2][P*Npad] or null: copies of x that the update pass of one iteration leaves
                           // for the next one, two in turn (cache-resident rings with whole-tensor
                           // sends: the receivers then fetch what a neighbour sends, no copy kernel)
  double* partials;        // [P*C*SW] per 1024-element sweep of a chunk: sum of squared drift, or
                           // of squared x when the trigger compares norms
  double* partials_hat;    // [P*C*SW] sum of squared xhat (norm-difference trigger only)
  double* xhat_sq;         // [S] squared norm of what was last sent, kept as a scalar when whole
                           // tensors are sent (norm-difference trigger only)
  float* delta; float* last_norm; float* delta_before;
  int32_t* last_event;
  // Where a step WRITES the sweep sums, and an event the threshold, its iteration and the squared
  // norm of what was sent.  The same arrays as partials, partials_hat, delta, last_event, xhat_sq
  // (which a step reads), except in a single-launch step, whose workgroups must all still see the
  // values from before the step: there the two sets alternate from step to step.
  double* partials_out; double* partials_hat_out; double* xhat_sq_out;
  float* delta_out; int32_t* last_event_out;
  uint8_t* valid_l; uint8_t* valid_r; uint8_t* fired; uint8_t* near_tie;
  uint32_t* ev_full; uint32_t* ev_topk; uint32_t* near_cnt; uint32_t* nonfinite_cnt;
  float* slope_hist; uint32_t* slope_cnt;   // [S*hist_len], [S]
  uint32_t* seg_woff_full; uint32_t* seg_woff_topk;   // [S] exclusive scans
  uint32_t* counts;        // [0] chunks to copy whole, [1] chunks of Top-K tensors, [2] Top-K tensors,
                           // [3] chunks so far whose possible winners did not fit their staging slot
  uint32_t* work_full; uint32_t* work_topk;   // [P*C] compact chunk lists (r*C + c)
  uint32_t* hist;          // [S*kHistBins]
  uint32_t* sel_prefix; uint32_t* sel_krem;   // [S]
  uint2* stage_n;          // [P*C] per chunk: staged entries (bin >= the threshold bin), and how many
                           // of them lie IN the threshold bin; x = 0xFFFFFFFF: more than the chunk's
                           // slot holds, nothing staged (its elements are then read from the arenas)
  uint32_t* stage_idx; float* stage_val;   // [P*stage_stride] a chunk's staged entries, in ascending index
                           // order; bit 31 of the index = in the threshold bin.  The chunk at arena
                           // offset `off` owns entries (off/16)*stage_num .. +(len/16)*stage_num
  uint32_t* stage_key;     // [P*stage_stride] the keys of the chunk's in-bin entries, same place, same order
  uint32_t stage_num;      // staging entries per 16 elements: 4, 8, 12 or 16
  uint64_t stage_stride;   // staging entries per worker
  uint2* chunk_cnt;        // [P*C] (keys above threshold, keys equal) per chunk
  uint2* chunk_before;     // [P*C] the same, summed over the tensor's earlier chunks
  uint32_t* chunk_sub;     // [P*C*(SW+1)] winners before each 1024-element sweep of a chunk,
                           // as message slots (entry 0 = the chunk's first slot)
  uint32_t* msg_idx; float* msg_val;          // [P*Ktot]
  unsigned long long* idx_hash;               // [S] fingerprints of the last step's Top-K messages (sums of
  unsigned long long* msg_hash;               // mixed indices / mixed (value, index) pairs), filled on request
  IterState* it;
  const double* decay_tab;   // decay^k for k < decay_len (replayable steps only)
  uint32_t decay_len;
  uint32_t P, L, C, S;
  uint32_t SW;             // 1024-element sweeps per chunk
  uint32_t hist_len;
  uint32_t Ktot;           // sum of K over tensors
  uint64_t Npad;
};

struct StepArgs {
  uint32_t k;
  float lr, mu;
  uint32_t thr_mode;
  float horizon;
  uint32_t force_first;
  uint32_t topk_on;
  uint32_t topk_key;
  uint32_t norm_src;       // what k_trigger finds: 0 squared drift in partials; 1 squared x in
                           // partials, squared xhat in xhat_sq once a tensor has sent; 2 squared x
                           // and squared xhat in partials / partials_hat
  uint32_t delay;          // messages of this iteration land after its updates
  uint32_t hist_fused;     // the update pass of the previous iteration already built pass A's histograms
  uint32_t plain_sgd;      // momentum == 0: the velocity arena is not touched
  uint32_t from_device;    // take k and decay^k from IterState instead of the two fields here
  uint32_t xhat_reset;     // a Top-K event resets the whole tensor's xhat to x
  uint32_t cached;         // the arenas fit the last-level cache: ordinary instead of streaming accesses
  uint32_t pull;           // whole-tensor sends are fetched by the receivers inside the update pass
  uint32_t one_launch;     // ... and the update pass also runs the trigger tests (no other kernel in the step)
  uint32_t step_no;        // one_launch: steps completed before this one (picks the copy of x to read)
  uint32_t key0, key1;
  double decay_pow;        // decay^k
  float spike_prob, spike_gain;
  const float* grad;       // buffer mode only
};

// launchers (each enqueues on the stream and returns the launch status)
hipError_t launch_norm(const Tables& t, bool norm_diff, hipStream_t s);
// norm: 0 no norm work, 1 squared drift, 2 squared x, 3 squared x and squared xhat
hipError_t launch_update(const Tables& t, const StepArgs& a, uint32_t dist, uint32_t grad_mode,
                         int norm, hipStream_t s);
hipError_t launch_trigger(const Tables& t, const StepArgs& a, hipStream_t s);
hipError_t launch_begin(const Tables& t, hipStream_t s);
hipError_t launch_scan(const Tables& t, const StepArgs& a, hipStream_t s);
hipError_t launch_expand(const Tables& t, const StepArgs& a, hipStream_t s);
hipError_t launch_copy(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid, hipStream_t s);
hipError_t launch_deliver(const Tables& t, uint32_t chunk_elems, uint32_t grid, hipStream_t s);
hipError_t launch_topk_select(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid,
                              hipStream_t s);
hipError_t launch_topk_send(const Tables& t, const StepArgs& a, uint32_t chunk_elems, uint32_t grid,
                            hipStream_t s);
hipError_t launch_average(const Tables& t, float* out, hipStream_t s);
hipError_t launch_message_hashes(const Tables& t, hipStream_t s);

}  // namespace evg
