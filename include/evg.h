/* evg.h -- C ABI of the EventGraD per-iteration parameter path on one MI355X.
 *
 * Scope.  The paper (arXiv 2103.07454) runs, on every worker ("PE") and every
 * training iteration, after the local gradient is available (Algorithm B):
 *   for every parameter tensor I:  if || xhat_I - x_I || >= delta_I  then send x_I
 *   to both ring neighbours and set xhat_I := x_I          (Section 4, trigger cases)
 *   delta_I := h * || xhat_I - x_I || / (k - khat)  at each event     (Section 4, Eq. 3)
 *   x := average of own and the neighbours' last received values - lr * gradient
 *                                                          (Section 3, Eq. 2; Section 4)
 * optionally sending only the Top-K share of a tensor with its indices
 * (Section 7).  This library runs that path for P ring workers simulated as P
 * replicas resident in one GPU's memory: a "message" is a write into the
 * neighbour's mailbox array (the paper's one-sided put into a window, Section 6).
 *
 * Conventions for every call
 *   - returns an evg_status; never throws or aborts across the ABI; on failure
 *     evg_error_text() explains, handles and counters are left untouched (array
 *     outputs of a failed evg_stats / evg_last_decisions may be partly written).
 *   - the HIP device that holds the arenas must be the current device of the
 *     calling thread for every call.
 *   - pointers are HOST pointers unless the comment says DEVICE.
 *   - a context is bound to one HIP stream and is not re-entrant: calls on one
 *     context must not overlap.  evg_step only enqueues work (no host sync).
 */
#ifndef EVG_H
#define EVG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evg_ctx evg_ctx;

typedef enum {
  EVG_OK = 0,
  EVG_ERR_INVALID = 1, /* bad argument or configuration value            */
  EVG_ERR_ALIGN = 2,   /* a device arena is not 16-byte aligned          */
  EVG_ERR_OOM = 3,     /* device or host allocation failed               */
  EVG_ERR_HIP = 4,     /* a HIP runtime call failed (no GPU, launch ...) */
  EVG_ERR_STATE = 5    /* call order: iteration not increasing, ...      */
} evg_status;

enum { EVG_THR_FIXED = 0, EVG_THR_ADAPTIVE = 1 };
enum { EVG_KEY_ABS_DRIFT = 0, EVG_KEY_ABS_VALUE = 1 };
enum { EVG_GRAD_SYNTH = 0, EVG_GRAD_BUFFER = 1 };
enum { EVG_DIST_NORMAL = 0, EVG_DIST_STUDENT_T3 = 1 };
enum { EVG_NORM_FUSED = 0, EVG_NORM_SEPARATE = 1 };
enum { EVG_TRIGGER_DRIFT_NORM = 0, EVG_TRIGGER_NORM_DIFF = 1 };
enum { EVG_ACCESS_AUTO = 0, EVG_ACCESS_STREAM = 1, EVG_ACCESS_CACHED = 2 };

/* Synthetic gradients (they stand in for the gradient computation step of
 * Algorithm B): element j of tensor l of worker r at iteration k is
 * sigma_l(k) * z, z drawn from a Philox4x32-10 stream with key = seed and
 * counter (block, l, k, r).  Normals: block j/4 gives elements 4(j/4) .. +3 by Box-Muller on
 * its word pairs (0,1) and (2,3).  Student-t(3): blocks 2(j/4), +1 give eight words, element
 * 4(j/4)+i takes words 2i, 2i+1 as t = sqrt(3 (u^(-2/3) - 1)) cos(2 pi v), u and v their uniforms
 * (the polar method: radius and angle of a spherical bivariate t).
 * sigma_l(k) = sigma0 [/ sqrt(fan_in_l)] * decay^k; with
 * probability spike_prob a whole (worker, iteration) gradient is multiplied by
 * spike_gain. */
typedef struct {
  uint64_t seed;
  uint32_t dist;           /* EVG_DIST_*                                   */
  uint32_t fan_in_scaling; /* nonzero: divide sigma0 by sqrt(fan_in)       */
  double sigma0;           /* >= 0                                         */
  double decay;            /* > 0                                          */
  float spike_prob;        /* in [0, 1]                                    */
  float spike_gain;
} evg_synth;

typedef struct {
  uint32_t P;                   /* ring size, >= 3 (Section 3: two distinct neighbours) */
  uint32_t L;                   /* parameter tensors per worker, >= 1                   */
  const uint64_t* layer_numel;  /* [L], each 1 .. 2^31-8; read during evg_init only     */
  const uint32_t* layer_fan_in; /* [L] or NULL when fan_in_scaling == 0                 */
  float lr;                     /* step size gamma (Eq. 2)                              */
  float momentum;               /* 0 = the paper's plain SGD: vel is then left at zero,
                                   neither read nor written by evg_step                 */
  uint32_t thr_mode;            /* EVG_THR_FIXED: delta = thr_fixed for every tensor;
                                   EVG_THR_ADAPTIVE: Eq. 3                              */
  float thr_fixed;              /* >= 0; 0 and +inf are legal                           */
  float horizon;                /* h of Eq. 3 (1 in the paper's experiments)            */
  uint32_t hist_len;            /* slopes kept per tensor, 1 .. 16: the threshold is h times the
                                   mean of the last hist_len slopes, one slope per event (they
                                   span hist_len + 1 events); 1 = Eq. 3 as printed (Section 7) */
  float delta_init;             /* adaptive threshold before a tensor's first event     */
  uint32_t force_first;         /* nonzero: every tensor sends at iteration 0 (Section 4) */
  uint32_t topk_ppm;            /* 0 = whole tensors; else K = max(1, ceil(n*ppm/1e6))
                                   elements per event (Section 7); a tensor's first
                                   event is always sent whole                           */
  uint32_t topk_key;            /* EVG_KEY_*: rank by |x - xhat| or by |x|              */
  uint32_t grad_mode;           /* EVG_GRAD_*                                           */
  uint32_t norm_mode;           /* EVG_NORM_FUSED: the update pass also accumulates the
                                   next iteration's drift norms (and the first radix
                                   histogram of its Top-K selection); EVG_NORM_SEPARATE:
                                   passes of their own read x and xhat                  */
  uint32_t chunk_elems;         /* work granule of the send kernels: 1024, 2048, 4096 or
                                   8192 elements, or 0 = chosen from the ring's size (2048
                                   if the five arenas together take at most 128 MB, else
                                   8192); no tensor shares one; results never differ     */
  uint32_t trigger_kind;        /* EVG_TRIGGER_DRIFT_NORM: test || x - xhat || (the formula of
                                   Section 4); EVG_TRIGGER_NORM_DIFF: test | ||x|| - ||xhat|| |
                                   (Section 4's prose reading: the change of the norm itself);
                                   Eq. 3 then uses the same quantity                         */
  uint32_t delivery_delay;      /* 0: a message is visible to the updates of the iteration it is
                                   sent in; 1: it lands after them and is used from the next
                                   iteration on (a deterministic stand-in for the asynchrony of
                                   one-sided puts, Section 7)                                 */
  uint32_t xhat_reset;          /* what a Top-K event does to xhat.  0: only the sent entries take
                                   the sent values (they are what was communicated).  1: the
                                   whole tensor's xhat becomes x, as after a whole send (the
                                   per-tensor xhat of Section 4 read literally); the mailboxes
                                   still change only at the sent indices.  Not available
                                   together with delivery_delay = 1                            */
  uint32_t access_mode;         /* how the dense passes touch the arenas; results never differ.
                                   EVG_ACCESS_STREAM: non-temporal (rings far larger than the
                                   caches); EVG_ACCESS_CACHED: ordinary accesses (rings that fit
                                   the 256 MB last-level cache); EVG_ACCESS_AUTO: cached if the
                                   five arenas together take at most 128 MB.  A cached ring that
                                   sends whole tensors without delivery delay also skips the copy
                                   kernel: each receiver fetches what its neighbours send inside
                                   the update pass, from a copy of x the library keeps (two more
                                   arrays of the ring's size, library-owned).  If its norms are
                                   accumulated by the update pass (norm_mode) and no tensor is
                                   longer than 131 072 elements, evg_step is then ONE kernel launch:
                                   the update pass runs the trigger tests itself.  evg_step_next
                                   keeps the trigger kernel (two launches), and so does evg_step on
                                   a ring once evg_step_next has been called on it               */
  evg_synth synth;
  /* DEVICE arenas owned by the caller, each P * evg_padded_numel() floats,
   * 16-byte aligned, non-overlapping, alive until evg_destroy.  Worker r's
   * tensor l starts at r * padded_numel + offset_l (evg_layer_offsets).  x holds
   * the initial parameters at evg_init; the library then sets xhat := x and
   * vel := 0 and treats both mailboxes as empty (their contents are never read
   * before a first message arrives).  evg_init asks the runtime about each pointer:
   * host memory, memory of another device, or an allocation that ends before the
   * stated size gives EVG_ERR_INVALID (the same holds for evg_step's grad and
   * evg_average's out). */
  float* x;      /* current parameters                                   */
  float* xhat;   /* values last sent (Section 4, X-hat)                   */
  float* mbox_l; /* last received from the left neighbour (r-1)           */
  float* mbox_r; /* last received from the right neighbour (r+1)          */
  float* vel;    /* momentum buffer (untouched after evg_init when momentum == 0) */
} evg_config;

/* Counters since evg_init (Section 7: share of messages, share of communication).
 * One event = one (worker, tensor, iteration) that fired = two puts. */
typedef struct {
  uint64_t iters;           /* evg_step calls completed                          */
  uint64_t events_total;    /* events_full + events_topk                         */
  uint64_t events_full;     /* events that sent the whole tensor                 */
  uint64_t events_topk;     /* events that sent a Top-K message                  */
  uint64_t value_words;     /* parameter values sent, per event (not per put)    */
  uint64_t index_words;     /* indices sent, per event                           */
  uint64_t bytes_sent;      /* 4 * (value + index words) * 2 puts                */
  uint64_t regular_events;  /* P * L * iters: what Algorithm A would send        */
  uint64_t regular_words;   /* P * N * iters                                     */
  uint64_t near_tie_flags;  /* tests with |norm - delta| < 1e-6 * delta          */
  uint64_t nonfinite_norms; /* tests whose norm was NaN or infinite              */
  uint64_t chunks_not_staged; /* Top-K work granules whose possible winners exceeded their staging
                               slot and were selected straight from x and xhat instead (slower,
                               same result): massive ties or winners crowded into a few granules */
  uint64_t library_bytes;   /* device memory the library holds for this context besides the
                               caller's five arenas (tables, work lists, Top-K histograms,
                               staging and message buffers); for evg_init_static the part
                               of the static block in use                           */
  /* optional per-(worker, tensor) outputs, HOST arrays of P*L entries or NULL  */
  uint32_t* events_full_rl;
  uint32_t* events_topk_rl;
  float* last_norm;          /* norm used by the most recent test                */
  float* delta;              /* current threshold                                */
  int32_t* last_event_iter;  /* khat of Eq. 3; -1 = never sent                   */
  uint8_t* valid_l;          /* has worker r received tensor l from the left ... */
  uint8_t* valid_r;          /* ... from the right                               */
} evg_stats_t;

/* Phases reported by evg_timing_read. */
enum {
  EVG_PH_NORM = 0,       /* separate drift-norm pass (EVG_NORM_SEPARATE only)        */
  EVG_PH_TRIGGER = 1,    /* norm finalisation, trigger test, thresholds, work lists
                            (no samples where the update pass runs the tests itself:
                            cache-resident rings that send whole tensors, norms fused,
                            no tensor above 131 072 elements, evg_step only)          */
  EVG_PH_SEND_FULL = 2,  /* whole-tensor copies into both mailboxes (no samples where
                            the receivers fetch the sends inside the update pass)     */
  EVG_PH_TOPK_SELECT = 3,/* threshold-key search for the Top-K set                   */
  EVG_PH_TOPK_SEND = 4,  /* pack (index, value) messages, put them                   */
  EVG_PH_UPDATE = 5,     /* fused averaging + momentum SGD (+ next drift norms)      */
  EVG_PH_DELIVER = 6,    /* delivery_delay = 1 only: the iteration's puts land       */
  EVG_PH_COUNT = 7
};

/* Size in floats of one worker's slice of an arena: every tensor start is
 * padded to 4 elements and the slice to 64 elements.  0 on invalid input. */
uint64_t evg_padded_numel(uint32_t L, const uint64_t* layer_numel);

/* offsets_out[l] = start of tensor l inside a worker's slice, in floats. */
evg_status evg_layer_offsets(uint32_t L, const uint64_t* layer_numel, uint64_t* offsets_out);

/* Validates cfg, builds the device tables, initialises xhat, vel and the
 * thresholds (Section 4: nothing has been sent yet, so xhat = x).  hip_stream
 * is a hipStream_t (NULL = the default stream); all work of this context is
 * enqueued on it.  Allocates library-owned device memory (tables, work lists,
 * Top-K histograms and message staging). */
evg_status evg_init(evg_ctx** out, const evg_config* cfg, void* hip_stream);

/* evg_init for callers that must not allocate device memory (harnesses that forbid
 * hipMalloc, tight serving loops that create and drop rings, code that is later captured
 * into a HIP graph): identical to evg_init in arguments, results and in every later call on
 * the context, except that all library-owned device tables (norm partial sums, decisions,
 * counters, work lists, Top-K histograms, staging and message buffers) are carved out of one
 * block of EVG_STATIC_SCRATCH_BYTES that is part of the library image on every GPU, instead
 * of coming from hipMalloc.  Calls no hipMalloc / hipFree and no allocating library routine;
 * evg_destroy on such a context frees no device memory either.  A configuration whose
 * tables do not fit is rejected with EVG_ERR_INVALID (the text gives the bytes needed).
 * The HIP runtime places the block on a GPU when it is first used there: the first call on
 * a device (which looks the block's address up) lowers free device memory by the block's
 * size, later calls leave it unchanged.
 * All calls on one GPU share that GPU's block, and it keeps the previous context's
 * contents (what must start at zero is cleared here): at most one such context may exist
 * per GPU at a time -- a second evg_init_static before the first context's evg_destroy
 * returns EVG_ERR_STATE -- and two threads that race through these calls on one GPU are
 * not protected against each other beyond that check. */
#define EVG_STATIC_SCRATCH_BYTES (64u << 20)
evg_status evg_init_static(evg_ctx** out, const evg_config* cfg, void* hip_stream);

/* One iteration k = iter of Algorithm B for all P workers: trigger tests, sends
 * (visible to every worker's update of the same iteration), then the averaging
 * and SGD update.  iter must be larger than the previous call's and below 2^31.
 * grad: DEVICE array laid out like x, required iff grad_mode == EVG_GRAD_BUFFER,
 * read during the step.  Asynchronous on the context's stream.  The iteration number
 * and what depends on it travel as kernel arguments, so a captured HIP graph of this
 * call must not be replayed for another iteration (evg_step_next is the call for that). */
evg_status evg_step(evg_ctx* c, uint64_t iter, const float* grad);

/* The same iteration as evg_step, for the iteration that follows the context's last one
 * (0 after evg_init), with the iteration number and what depends on it kept in device
 * memory: nothing in the launch sequence changes from call to call, so a HIP graph captured
 * around one call (hipStreamBeginCapture on the context's stream) may be replayed, each
 * replay being the next iteration.  For callers that drive the iterations from a graph.
 * Makes no synchronising or allocating call, records no memset and no event (the phase
 * timers of evg_timing skip these steps).  Iterations up to 65535; the first call that
 * needs the host's view of the iteration again (evg_step, evg_stats, evg_state_export)
 * synchronises and reports EVG_ERR_STATE if that limit was passed; once this call has been
 * used on a context, every evg_step on it synchronises first, to learn how far replays have
 * gone.  grad as in evg_step: a captured graph keeps reading the same pointer. */
evg_status evg_step_next(evg_ctx* c, const float* grad);

/* Waits for the stream, then fills *out (array members that are non-NULL too). */
evg_status evg_stats(evg_ctx* c, evg_stats_t* out);

/* Decisions of the most recent step, HOST arrays of P*L entries, any may be NULL:
 * fired (0 = silent, 1 = whole tensor, 2 = Top-K message), near_tie (the 1e-6
 * band), norm and the threshold the norm was compared with.  Waits for the stream. */
evg_status evg_last_decisions(evg_ctx* c, uint8_t* fired, uint8_t* near_tie, float* norm,
                              float* delta_before);

/* The Top-K message worker r sent for tensor l in the most recent step: ascending
 * element indices within the tensor and their values (Section 7: values + indices
 * = 2K words).  *count = K, or 0 if (r, l) sent no Top-K message (or no step has run
 * in this context since evg_init / evg_state_import); at most cap
 * entries are copied to the HOST arrays idx / val (either may be NULL). */
evg_status evg_message(evg_ctx* c, uint32_t r, uint32_t l, uint32_t* idx, float* val,
                       uint64_t cap, uint64_t* count);

/* Fingerprints of the Top-K messages of the most recent step, HOST arrays of P*L entries,
 * either may be NULL.  A message is K indices and K values (Section 7); for worker r,
 * tensor l: idx_hash = sum over the message's entries of mix(index) and msg_hash = sum of
 * mix(value bits << 32 | index), both modulo 2^64, with mix the finaliser of the SplitMix64
 * generator (z += 0x9E3779B97F4A7C15; z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9;
 * z = (z ^ z >> 27) * 0x94D049BB133111EB; z ^ z >> 31).  0 where (r, l) sent no Top-K
 * message.  They let a caller compare every message of a step with another implementation
 * without copying the messages themselves to the host.  Computed by this call from the message
 * buffers (one small kernel on the context's stream; nothing is added to evg_step); waits for
 * the stream. */
evg_status evg_message_hashes(evg_ctx* c, uint64_t* idx_hash, uint64_t* msg_hash);

/* Final model: out[j] = mean over workers of x[r][j] (last line of Algorithm B).
 * out: DEVICE array of evg_padded_numel floats.  Asynchronous on the stream. */
evg_status evg_average(evg_ctx* c, float* out);

/* Checkpoint / resume.  The five arenas are the caller's to save; everything else a run
 * depends on (thresholds, last-event iterations, mailbox flags, slope histories, counters,
 * the norm partial sums and radix histograms carried from the last update pass, the
 * iteration count) goes into one opaque HOST blob.  evg_state_export waits for the stream.
 * evg_state_import expects a context created with the same configuration whose arenas
 * already hold the saved contents; a blob from a different configuration is rejected with
 * EVG_ERR_INVALID.  After import, evg_step continues exactly (bit for bit) where the
 * exporting context stopped. */
uint64_t evg_state_size(evg_ctx* c); /* bytes needed for the blob; 0 if c is NULL */
evg_status evg_state_export(evg_ctx* c, void* blob, uint64_t capacity);
evg_status evg_state_import(evg_ctx* c, const void* blob, uint64_t size);

/* Per-phase GPU time.  enable != 0 starts bracketing every phase of every later
 * step with HIP events on the context's stream (and clears earlier samples);
 * evg_timing_read waits for the stream and returns, per phase, the summed
 * milliseconds and the number of samples since enabling. */
evg_status evg_timing(evg_ctx* c, int enable);
evg_status evg_timing_read(evg_ctx* c, double ms_out[EVG_PH_COUNT], uint64_t samples_out[EVG_PH_COUNT]);

/* Frees library-owned memory.  The caller's arenas are untouched. */
evg_status evg_destroy(evg_ctx* c);

const char* evg_strerror(evg_status s);
/* Text of the most recent failure on this thread ("" if none). */
const char* evg_error_text(void);

#ifdef __cplusplus
}
#endif
#endif /* EVG_H */
