// The trigger test of one (worker, tensor) as device functions, shared by the kernels that
// run it: k_trigger / k_front (one wavefront per tensor, ahead of the update pass) and the
// update pass of rings that take a single launch per iteration (every workgroup repeats the
// tests it depends on; the tensor's first workgroup records the outcome).
//
// What a test READS (sweep sums, delta, last_event, xhat_sq) and what an event WRITES of the
// same (delta, last_event, xhat_sq; the sweep sums are written by the update pass) go through
// two sets of pointers, T.name and T.name_out.  Normally both name the same array.  The
// single-launch step gives them different arrays, because there other workgroups of the same
// launch still have to read the values from before the event.
#pragma once
#include "evg_device.h"

namespace evg {

// Sums of the tensor's sweep partials in a fixed order, by one whole wavefront; valid in every lane.
// *hat_sums: the squared norm of xhat comes from the arena sums (norm-difference trigger with
// Top-K, or before the tensor's first event) rather than from the scalar kept at its last event.
__device__ __forceinline__ void segment_sums(const Tables& T, const StepArgs& A, uint32_t seg, double* acc_out,
                                             double* acc_hat_out, bool* hat_sums_out) {
  const uint32_t r = seg / T.L, l = seg % T.L;
  const LayerDesc ld = T.layers[l];
  const double* part = T.partials + ((size_t)r * T.C + ld.chunk0) * T.SW;
  const uint32_t np = ld.nchunks * T.SW;
  double acc = 0.0, acc_hat = 0.0;
  for (uint32_t i = lane_id(); i < np; i += 64) acc += part[i];
  acc = wave_sum(acc);
  const bool hat_sums = A.norm_src == 2 || (A.norm_src == 1 && T.last_event[seg] < 0);
  if (hat_sums) {
    const double* ph = T.partials_hat + ((size_t)r * T.C + ld.chunk0) * T.SW;
    for (uint32_t i = lane_id(); i < np; i += 64) acc_hat += ph[i];
    acc_hat = wave_sum(acc_hat);
  }
  *acc_out = acc;
  *acc_hat_out = acc_hat;
  *hat_sums_out = hat_sums;
}

// The event condition || xhat - x || >= delta (Section 4) on those sums, for ONE lane.  Returns
// 0 silent, 1 the whole tensor is sent, 2 a Top-K message is sent.
// RECORD: also book the outcome: norm, threshold before, near-tie flag, counters, and at an
// event the adaptive threshold (Eq. 3), the event's iteration and the event counters.
// MARK: at an event also mark the two neighbours' mailbox slots as filled.
template <bool RECORD, bool MARK>
__device__ __forceinline__ uint8_t segment_test(const Tables& T, const StepArgs& A, uint32_t seg, double acc,
                                                double acc_hat, bool hat_sums) {
  const uint32_t r = seg / T.L, l = seg % T.L;
  const uint32_t k = step_k(T, A);
  float d;
  if (A.norm_src == 0) {
    d = (float)sqrt(acc);
  } else {
    if (!hat_sums) acc_hat = T.xhat_sq[seg];
    d = __builtin_fabsf((float)sqrt(acc) - (float)sqrt(acc_hat));
  }
  const float dl = T.delta[seg];
  const int32_t khat = T.last_event[seg];
  const bool fire = (A.force_first && k == 0) || (d >= dl);   // NaN never fires
  // a tensor's first message has nothing to patch on the receiving side: send it whole
  const uint8_t code = !fire ? 0 : (!A.topk_on || khat < 0) ? 1 : 2;
  if (!RECORD) return code;

  T.last_norm[seg] = d;
  T.delta_before[seg] = dl;
  if (!(__builtin_fabsf(d) <= 3.402823466e+38f)) T.nonfinite_cnt[seg] += 1;   // NaN or inf
  const bool near = __builtin_fabsf(d - dl) < 1e-6f * dl;
  T.near_tie[seg] = near ? 1 : 0;
  if (near) T.near_cnt[seg] += 1;
  float dl_new = dl;
  if (fire) {
    if (A.thr_mode == 1) {
      const float slope = d / (float)((int32_t)k - khat);
      if (T.hist_len <= 1) {
        dl_new = A.horizon * slope;
      } else {
        // mean of the slopes between the last hist_len consecutive events (Section 7)
        float* hs = T.slope_hist + (size_t)seg * T.hist_len;
        uint32_t cnt = T.slope_cnt[seg];
        if (cnt == T.hist_len) {
          for (uint32_t i = 1; i < cnt; ++i) hs[i - 1] = hs[i];
          cnt -= 1;
        }
        hs[cnt++] = slope;
        T.slope_cnt[seg] = cnt;
        float sum = 0.0f;
        for (uint32_t i = 0; i < cnt; ++i) sum += hs[i];
        dl_new = A.horizon * (sum / (float)cnt);
      }
    }
    if (code == 1) T.ev_full[seg] += 1;
    else T.ev_topk[seg] += 1;
    if (MARK && !A.delay) {             // with delayed delivery: set when the put lands (k_deliver)
      const uint32_t left = (r + T.P - 1) % T.P, right = (r + 1) % T.P;
      T.valid_r[left * T.L + l] = 1;    // I am my left neighbour's right-hand source
      T.valid_l[right * T.L + l] = 1;
    }
  }
  T.delta_out[seg] = dl_new;
  T.last_event_out[seg] = fire ? (int32_t)k : khat;
  // the whole tensor is sent: xhat becomes x, and so does its squared norm
  if (A.norm_src == 1) T.xhat_sq_out[seg] = fire ? acc : T.xhat_sq[seg];
  T.fired[seg] = code;
  return code;
}

// The step's bookkeeping, once per step.
__device__ __forceinline__ void close_step(const Tables& T, const StepArgs& A) {
  T.it->k_next = step_k(T, A) + 1;
  T.it->iters += 1;
}

}  // namespace evg
