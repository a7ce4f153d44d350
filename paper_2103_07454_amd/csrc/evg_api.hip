// Host side of libevg: argument checking, table construction, the per-iteration
// launch sequence and the counters.  See include/evg.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/evg.h"
#include "evg_internal.h"

using namespace evg;

namespace {

thread_local std::string g_err;

evg_status fail(evg_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return s;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return fail(e_ == hipErrorOutOfMemory ? EVG_ERR_OOM : EVG_ERR_HIP, "%s: %s", #expr, \
                  hipGetErrorString(e_));                                               \
  } while (0)

inline uint64_t pad_to(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

struct TimerPair { hipEvent_t a, b; int phase; };

constexpr uint32_t kDecayTable = 1u << 16;   // iterations a replayable step can reach

// ---- the one block of device memory that evg_init_static hands out -------------------
// Every GPU the library runs on holds its own copy of this array from the moment the
// library is loaded until the process ends.  In host code the array's NAME is only a
// handle for hipGetSymbolAddress: the device address differs per GPU and is looked up
// once per device (scratch_base), and only that address is ever passed to kernels,
// memsets or copies.
constexpr size_t kScratchBytes = EVG_STATIC_SCRATCH_BYTES;
constexpr size_t kScratchAlign = 256;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mu;
unsigned char* g_scratch_base[kMaxDevices] = {nullptr};   // per device: where its copy lives
evg_ctx* g_scratch_user[kMaxDevices] = {nullptr};         // per device: the context living in it

}  // namespace

struct evg_ctx {
  evg_config cfg{};
  hipStream_t stream = nullptr;
  Tables t{};
  uint32_t chunk_elems = 8192;
  uint32_t work_grid = 1;
  std::vector<uint64_t> numel;      // per tensor
  std::vector<uint32_t> K;          // per tensor Top-K message length
  std::vector<uint32_t> msg_off;
  std::vector<void*> owned;         // device allocations to free
  uint64_t N = 0;                   // unpadded elements per worker
  uint64_t iters = 0;
  int64_t last_iter = -1;
  bool messages_live = false;       // the message buffers hold the last step's messages
  bool cached = false;              // the five arenas together fit the last-level cache
  bool device_ahead = false;        // evg_step_next has been used: replays of a captured graph
                                    // advance the device's iteration without the host seeing
                                    // it, so iters / last_iter are re-read whenever needed
  // Single-launch steps (cache-resident rings, whole-tensor sends, norms accumulated by the update
  // pass, no tensor longer than 128 sweeps): the update pass runs the trigger tests itself.  What the
  // tests read must then not be written in the same launch, so these arrays exist twice and a step
  // writes the set it does not read; c->t always names the set that holds the current state.
  struct SecondSet { double* partials; double* xhat_sq; float* delta; int32_t* last_event; };
  // (the sums of squared xhat are not among them: such a ring's steps only read those)
  SecondSet second{};
  bool one_launch = false;          // the ring qualifies
  bool replayable_used = false;     // evg_step_next has been called: a captured graph may hold the pointers
                                    // of c->t, so the sets must not change places any more
  // evg_init_static: the tables are carved out of the device's static scratch block
  unsigned char* arena_base = nullptr;   // null = tables come from hipMalloc
  size_t arena_used = 0;
  int arena_dev = -1;
  uint64_t owned_bytes = 0;              // device memory handed out by dalloc
  // timing
  bool timing = false;
  std::vector<TimerPair> pending;
  std::vector<hipEvent_t> pool;
  double ms[EVG_PH_COUNT] = {0};
  uint64_t samples[EVG_PH_COUNT] = {0};

  template <typename T>
  evg_status dalloc(T** p, size_t count, bool zero) {
    void* d = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(T);
    if (arena_base) {
      const size_t at = (arena_used + kScratchAlign - 1) / kScratchAlign * kScratchAlign;
      if (at + bytes > kScratchBytes)
        return fail(EVG_ERR_INVALID, "the static scratch block holds %zu bytes; this configuration needs more",
                    kScratchBytes);
      d = arena_base + at;
      arena_used = at + bytes;
    } else {
      hipError_t e = hipMalloc(&d, bytes);
      if (e != hipSuccess) return fail(EVG_ERR_OOM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e));
      owned.push_back(d);
    }
    owned_bytes += bytes;
    if (zero) HIP_TRY(hipMemsetAsync(d, 0, bytes, stream));
    *p = static_cast<T*>(d);
    return EVG_OK;
  }

  evg_status drain_timers() {
    if (pending.empty()) return EVG_OK;
    HIP_TRY(hipStreamSynchronize(stream));
    for (const TimerPair& p : pending) {
      float m = 0.f;
      HIP_TRY(hipEventElapsedTime(&m, p.a, p.b));
      ms[p.phase] += (double)m;
      samples[p.phase] += 1;
      pool.push_back(p.a);
      pool.push_back(p.b);
    }
    pending.clear();
    return EVG_OK;
  }

  evg_status mark(hipEvent_t* ev) {
    if (pool.empty()) {
      HIP_TRY(hipEventCreate(ev));
    } else {
      *ev = pool.back();
      pool.pop_back();
    }
    HIP_TRY(hipEventRecord(*ev, stream));
    return EVG_OK;
  }
};

namespace {

// Brackets one phase with events when timing is on.
struct Phase {
  evg_ctx* c;
  int phase;
  hipEvent_t a{};
  evg_status st = EVG_OK;
  Phase(evg_ctx* c_, int ph) : c(c_), phase(ph) {
    if (c->timing) st = c->mark(&a);
  }
  evg_status end() {
    if (!c->timing || st != EVG_OK) return st;
    hipEvent_t b;
    st = c->mark(&b);
    if (st == EVG_OK) c->pending.push_back({a, b, phase});
    return st;
  }
};

evg_status check_layers(uint32_t L, const uint64_t* layer_numel) {
  if (L < 1 || !layer_numel) return fail(EVG_ERR_INVALID, "need L >= 1 tensors and their sizes");
  uint64_t total = 0;
  for (uint32_t l = 0; l < L; ++l) {
    if (layer_numel[l] < 1 || layer_numel[l] > 0x7FFFFFF8ull)
      return fail(EVG_ERR_INVALID, "tensor %u has %llu elements (1 .. 2^31-8 allowed)", l,
                  (unsigned long long)layer_numel[l]);
    total += pad_to(layer_numel[l], 4);
    if (total > 0xFFFFFF00ull) return fail(EVG_ERR_INVALID, "a worker's slice exceeds 2^32 floats");
  }
  return EVG_OK;
}

bool finite_f(float v) { return std::isfinite(v); }

// A kernel that is handed host memory, or an array shorter than the sizes say, faults
// the GPU; so ask the runtime what `p` is.  The range test sees the whole allocation
// `p` lies in (a sub-allocator's pool block counts as one), so it catches what runs
// past that; where the runtime cannot name the range the test is skipped.
evg_status check_device_array(const void* p, uint64_t bytes, const char* what) {
  hipPointerAttribute_t at;
  hipError_t e = hipPointerGetAttributes(&at, p);
  if (e != hipSuccess || (at.type != hipMemoryTypeDevice && at.type != hipMemoryTypeManaged)) {
    (void)hipGetLastError();   // a failed query must not surface after the next launch
    return fail(EVG_ERR_INVALID, "%s does not point to device memory", what);
  }
  int dev = -1;
  if (hipGetDevice(&dev) == hipSuccess && at.device != dev)
    return fail(EVG_ERR_INVALID, "%s lives on device %d, the current device is %d", what, at.device, dev);
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  e = hipMemGetAddressRange(&base, &size, const_cast<void*>(p));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return EVG_OK;
  }
  const uintptr_t end = (uintptr_t)base + size;
  if ((uintptr_t)p < (uintptr_t)base || (uintptr_t)p + bytes > end)
    return fail(EVG_ERR_INVALID, "%s needs %llu bytes, its allocation ends after %llu", what,
                (unsigned long long)bytes, (unsigned long long)(end - (uintptr_t)p));
  return EVG_OK;
}

}  // namespace

extern "C" {

const char* evg_strerror(evg_status s) {
  switch (s) {
    case EVG_OK: return "ok";
    case EVG_ERR_INVALID: return "invalid argument";
    case EVG_ERR_ALIGN: return "misaligned device pointer";
    case EVG_ERR_OOM: return "out of memory";
    case EVG_ERR_HIP: return "HIP runtime error";
    case EVG_ERR_STATE: return "call out of order";
  }
  return "unknown status";
}

const char* evg_error_text(void) { return g_err.c_str(); }

uint64_t evg_padded_numel(uint32_t L, const uint64_t* layer_numel) {
  if (check_layers(L, layer_numel) != EVG_OK) return 0;
  uint64_t total = 0;
  for (uint32_t l = 0; l < L; ++l) total += pad_to(layer_numel[l], 4);
  return pad_to(total, 64);
}

evg_status evg_layer_offsets(uint32_t L, const uint64_t* layer_numel, uint64_t* offsets_out) {
  if (!offsets_out) return fail(EVG_ERR_INVALID, "offsets_out is NULL");
  evg_status st = check_layers(L, layer_numel);
  if (st != EVG_OK) return st;
  uint64_t total = 0;
  for (uint32_t l = 0; l < L; ++l) {
    offsets_out[l] = total;
    total += pad_to(layer_numel[l], 4);
  }
  return EVG_OK;
}

evg_status evg_destroy(evg_ctx* c) {
  if (!c) return EVG_OK;
  (void)hipStreamSynchronize(c->stream);
  if (c->arena_base) {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (c->arena_dev >= 0 && g_scratch_user[c->arena_dev] == c) g_scratch_user[c->arena_dev] = nullptr;
  }
  for (void* p : c->owned) (void)hipFree(p);
  for (const TimerPair& p : c->pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (hipEvent_t e : c->pool) (void)hipEventDestroy(e);
  delete c;
  return EVG_OK;
}

// Bytes of library-owned device tables a configuration needs, with every table rounded up to
// the scratch block's alignment: the same list as the allocations of init_common.
// Staging entries reserved per 16 elements of a chunk.  The possible winners of a Top-K event are
// its K winners plus the rest of the threshold bin (a 9 % wide slice of the key range: a few per
// cent of the tensor): one and a half times the Top-K share plus a sixteenth covers that with room
// to spare, and a chunk that needs more is handled from the arenas.
static uint32_t stage_num_for(uint32_t topk_ppm) {
  const uint64_t want = (3ull * topk_ppm * 8ull + 999999ull) / 1000000ull + 1ull;   // in sixteenths
  return want <= 4 ? 4u : want <= 8 ? 8u : want <= 12 ? 12u : 16u;
}

static uint64_t table_bytes(uint64_t P, uint64_t L, uint64_t C, uint64_t SW, uint64_t hist_len, uint64_t Npad,
                            uint64_t ktot, uint64_t stage_num, bool topk, bool norm_diff, bool pull, bool one_launch) {
  const uint64_t S = P * L, PC = P * C;
  uint64_t total = 0;
  auto add = [&total](uint64_t count, uint64_t elem) {
    total = (total + kScratchAlign - 1) / kScratchAlign * kScratchAlign + (count ? count : 1) * elem;
  };
  add(C, sizeof(ChunkDesc)); add(L, sizeof(LayerDesc));
  add(PC * SW, 8);
  if (norm_diff) { add(PC * SW, 8); add(S, 8); }
  add(S, 4); add(S, 4); add(S, 4); add(S, 4);            // delta, last_norm, delta_before, last_event
  add(S, 1); add(S, 1); add(S, 1); add(S, 1);            // valid_l, valid_r, fired, near_tie
  add(S, 4); add(S, 4); add(S, 4); add(S, 4);            // ev_full, ev_topk, near_cnt, nonfinite_cnt
  add(S * hist_len, 4); add(S, 4); add(S, 4); add(S, 4); // slope_hist, slope_cnt, seg_woff_full/topk
  add(4, 4); add(1, sizeof(IterState)); add(kDecayTable, 8);
  add(PC, 4);                                            // work_full
  if (pull) add(2 * P * Npad, 4);                        // xsnap
  if (one_launch) {                                      // the second set of what the trigger tests read
    add(PC * SW, 8); add(S, 4); add(S, 4);
    if (norm_diff) add(S, 8);
  }
  if (topk) {
    add(PC, 4); add(S * kHistBins, 4); add(S, 4); add(S, 4); add(PC, 8);
    const uint64_t stage = P * (Npad / 16 * stage_num);
    add(stage, 4); add(stage, 4); add(stage, 4);
    add(PC, 8); add(PC, 8); add(PC * (SW + 1), 4);
    add(P * ktot, 4); add(P * ktot, 4); add(S, 8); add(S, 8);
  }
  return total;
}

static evg_status init_common(evg_ctx** out, const evg_config* cfg, void* hip_stream, bool use_scratch) {
  if (!out || !cfg) return fail(EVG_ERR_INVALID, "out and cfg must be non-NULL");
  evg_status st = check_layers(cfg->L, cfg->layer_numel);
  if (st != EVG_OK) return st;
  if (cfg->P < 3 || cfg->P > 65535)
    return fail(EVG_ERR_INVALID, "ring size P = %u (3 .. 65535: a worker needs two distinct neighbours)", cfg->P);
  if (!finite_f(cfg->lr) || !finite_f(cfg->momentum)) return fail(EVG_ERR_INVALID, "lr and momentum must be finite");
  if (cfg->thr_mode > EVG_THR_ADAPTIVE) return fail(EVG_ERR_INVALID, "unknown thr_mode %u", cfg->thr_mode);
  if (cfg->thr_mode == EVG_THR_FIXED && !(cfg->thr_fixed >= 0.0f))
    return fail(EVG_ERR_INVALID, "thr_fixed must be >= 0 (+inf allowed)");
  if (cfg->thr_mode == EVG_THR_ADAPTIVE) {
    if (!finite_f(cfg->horizon) || cfg->horizon < 0.0f) return fail(EVG_ERR_INVALID, "horizon must be finite and >= 0");
    if (!(cfg->delta_init >= 0.0f)) return fail(EVG_ERR_INVALID, "delta_init must be >= 0");
    if (cfg->hist_len < 1 || cfg->hist_len > 16) return fail(EVG_ERR_INVALID, "hist_len must be 1 .. 16");
  }
  if (cfg->topk_ppm > 1000000u) return fail(EVG_ERR_INVALID, "topk_ppm must be <= 1000000");
  if (cfg->topk_key > EVG_KEY_ABS_VALUE) return fail(EVG_ERR_INVALID, "unknown topk_key %u", cfg->topk_key);
  if (cfg->grad_mode > EVG_GRAD_BUFFER) return fail(EVG_ERR_INVALID, "unknown grad_mode %u", cfg->grad_mode);
  if (cfg->norm_mode > EVG_NORM_SEPARATE) return fail(EVG_ERR_INVALID, "unknown norm_mode %u", cfg->norm_mode);
  if (cfg->trigger_kind > EVG_TRIGGER_NORM_DIFF) return fail(EVG_ERR_INVALID, "unknown trigger_kind %u", cfg->trigger_kind);
  if (cfg->delivery_delay > 1) return fail(EVG_ERR_INVALID, "delivery_delay must be 0 or 1");
  if (cfg->xhat_reset > 1) return fail(EVG_ERR_INVALID, "xhat_reset must be 0 or 1");
  if (cfg->xhat_reset && cfg->delivery_delay)
    return fail(EVG_ERR_INVALID, "xhat_reset = 1 is not available with delivery_delay = 1");
  if (cfg->access_mode > EVG_ACCESS_CACHED) return fail(EVG_ERR_INVALID, "unknown access_mode %u", cfg->access_mode);
  if (cfg->chunk_elems != 0 && cfg->chunk_elems != 1024 && cfg->chunk_elems != 2048 &&
      cfg->chunk_elems != 4096 && cfg->chunk_elems != 8192)
    return fail(EVG_ERR_INVALID, "chunk_elems must be 0, 1024, 2048, 4096 or 8192");
  if (cfg->grad_mode == EVG_GRAD_SYNTH) {
    const evg_synth& s = cfg->synth;
    if (s.dist > EVG_DIST_STUDENT_T3) return fail(EVG_ERR_INVALID, "unknown synth.dist %u", s.dist);
    if (!std::isfinite(s.sigma0) || s.sigma0 < 0) return fail(EVG_ERR_INVALID, "synth.sigma0 must be finite and >= 0");
    if (!std::isfinite(s.decay) || s.decay <= 0) return fail(EVG_ERR_INVALID, "synth.decay must be finite and > 0");
    if (!(s.spike_prob >= 0.0f && s.spike_prob <= 1.0f)) return fail(EVG_ERR_INVALID, "synth.spike_prob must be in [0,1]");
    if (!finite_f(s.spike_gain)) return fail(EVG_ERR_INVALID, "synth.spike_gain must be finite");
    if (s.fan_in_scaling) {
      if (!cfg->layer_fan_in) return fail(EVG_ERR_INVALID, "fan_in_scaling needs layer_fan_in");
      for (uint32_t l = 0; l < cfg->L; ++l)
        if (cfg->layer_fan_in[l] < 1) return fail(EVG_ERR_INVALID, "layer_fan_in[%u] must be >= 1", l);
    }
  }
  const uint64_t Npad = evg_padded_numel(cfg->L, cfg->layer_numel);
  const uint64_t arena_bytes = (uint64_t)cfg->P * Npad * 4;
  // rings that live in the last-level cache are bound by launch and workgroup counts, not by
  // HBM: small granules leave fewer empty sweeps behind their many short tensors (measured)
  const bool small_ring = 5 * arena_bytes <= (128ull << 20);
  const uint32_t ce = cfg->chunk_elems ? cfg->chunk_elems : small_ring ? 2048u : 8192u;
  const float* arenas[5] = {cfg->x, cfg->xhat, cfg->mbox_l, cfg->mbox_r, cfg->vel};
  static const char* names[5] = {"x", "xhat", "mbox_l", "mbox_r", "vel"};
  for (int i = 0; i < 5; ++i) {
    if (!arenas[i]) return fail(EVG_ERR_INVALID, "arena %s is NULL", names[i]);
    if ((uintptr_t)arenas[i] % 16) return fail(EVG_ERR_ALIGN, "arena %s is not 16-byte aligned", names[i]);
  }
  for (int i = 0; i < 5; ++i)
    for (int j = i + 1; j < 5; ++j) {
      const uintptr_t a = (uintptr_t)arenas[i], b = (uintptr_t)arenas[j];
      if (a < b + arena_bytes && b < a + arena_bytes)
        return fail(EVG_ERR_INVALID, "arenas %s and %s overlap", names[i], names[j]);
    }
  // everything above is plain arithmetic; from here on the HIP runtime is involved
  for (int i = 0; i < 5; ++i)
    if ((st = check_device_array(arenas[i], arena_bytes, names[i])) != EVG_OK) return st;

  // ---- host tables --------------------------------------------------------
  evg_ctx* c = new (std::nothrow) evg_ctx();
  if (!c) return fail(EVG_ERR_OOM, "host allocation failed");
  c->cfg = *cfg;
  c->cfg.layer_numel = nullptr;
  c->cfg.layer_fan_in = nullptr;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->chunk_elems = ce;
  // 256 MB of last-level cache on MI355X; a ring whose arenas take at most half of it is
  // served from there and does better with ordinary than with streaming accesses
  c->cached = cfg->access_mode == EVG_ACCESS_CACHED || (cfg->access_mode == EVG_ACCESS_AUTO && small_ring);
  const uint32_t P = cfg->P, L = cfg->L;
  std::vector<LayerDesc> layers(L);
  std::vector<ChunkDesc> chunks;
  uint64_t off = 0, ktot = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const uint64_t n = cfg->layer_numel[l];
    LayerDesc& d = layers[l];
    d.off = (uint32_t)off;
    d.numel = (uint32_t)n;
    d.chunk0 = (uint32_t)chunks.size();
    d.nchunks = (uint32_t)((n + ce - 1) / ce);
    uint64_t k = 0;
    if (cfg->topk_ppm) {
      k = (n * (uint64_t)cfg->topk_ppm + 999999ull) / 1000000ull;
      if (k < 1) k = 1;
      if (k > n) k = n;
    }
    d.K = (uint32_t)k;
    d.msg_off = (uint32_t)ktot;
    ktot += k;
    d.sig_base = cfg->synth.sigma0;
    if (cfg->grad_mode == EVG_GRAD_SYNTH && cfg->synth.fan_in_scaling)
      d.sig_base = cfg->synth.sigma0 / std::sqrt((double)cfg->layer_fan_in[l]);
    for (uint32_t i = 0; i < d.nchunks; ++i) {
      ChunkDesc cd;
      cd.j0 = i * ce;
      cd.off = d.off + cd.j0;
      cd.len = (uint32_t)(n - cd.j0 < ce ? n - cd.j0 : ce);
      cd.layer = l;
      chunks.push_back(cd);
    }
    c->numel.push_back(n);
    c->K.push_back(d.K);
    c->msg_off.push_back(d.msg_off);
    c->N += n;
    off += pad_to(n, 4);
  }
  const uint64_t C = chunks.size();
  if ((uint64_t)P * C * (ce / 1024 + 1) > 0xFFFFFFF0ull || (uint64_t)P * ktot > 0xFFFFFFF0ull) {
    delete c;
    return fail(EVG_ERR_INVALID, "configuration too large: work lists and message slots are indexed with 32 bits");
  }
  const uint64_t S = (uint64_t)P * L;

  // ---- device tables ------------------------------------------------------
  Tables& t = c->t;
  t.P = P; t.L = L; t.C = (uint32_t)C; t.S = (uint32_t)S;
  t.SW = ce / (uint32_t)kSweep;
  t.hist_len = cfg->thr_mode == EVG_THR_ADAPTIVE ? cfg->hist_len : 1;
  t.Ktot = (uint32_t)ktot;
  t.Npad = Npad;
  t.stage_num = stage_num_for(cfg->topk_ppm);
  t.stage_stride = Npad / 16 * t.stage_num;
  t.x = cfg->x; t.xhat = cfg->xhat; t.mbox_l = cfg->mbox_l; t.mbox_r = cfg->mbox_r; t.vel = cfg->vel;
  // one launch per iteration: the ring's receivers fetch the sends (see `pull` below), the update pass
  // accumulates the norms, and one wavefront sums a tensor's sweep partials with two loads per lane
  uint32_t most_sweeps = 0;
  for (const LayerDesc& d : layers) most_sweeps = std::max(most_sweeps, d.nchunks * t.SW);
  const bool one_launch = c->cached && !cfg->topk_ppm && !cfg->delivery_delay &&
                          cfg->norm_mode == EVG_NORM_FUSED && most_sweeps <= 128;
  int dev = 0, cus = 256;
  ChunkDesc* d_chunks = nullptr;
  LayerDesc* d_layers = nullptr;
#define TRY_OR_FREE(expr)              \
  do {                                 \
    evg_status s_ = (expr);            \
    if (s_ != EVG_OK) {                \
      evg_destroy(c);                  \
      return s_;                       \
    }                                  \
  } while (0)
#define HIP_OR_FREE(expr)                                                            \
  do {                                                                               \
    hipError_t e_ = (expr);                                                          \
    if (e_ != hipSuccess) {                                                          \
      evg_destroy(c);                                                                \
      return fail(EVG_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));              \
    }                                                                                \
  } while (0)
  HIP_OR_FREE(hipGetDevice(&dev));
  HIP_OR_FREE(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (use_scratch) {
    const uint64_t need = table_bytes(P, L, C, t.SW, t.hist_len, Npad, ktot, t.stage_num, cfg->topk_ppm != 0,
                                      cfg->trigger_kind == EVG_TRIGGER_NORM_DIFF,
                                      c->cached && !cfg->topk_ppm && !cfg->delivery_delay, one_launch);
    if (need > kScratchBytes) {
      evg_destroy(c);
      return fail(EVG_ERR_INVALID, "this configuration needs %llu bytes of tables; the static scratch block "
                  "holds %llu (use evg_init)", (unsigned long long)need, (unsigned long long)kScratchBytes);
    }
    if (dev < 0 || dev >= kMaxDevices) {
      evg_destroy(c);
      return fail(EVG_ERR_INVALID, "device %d is beyond the %d devices evg_init_static keeps track of", dev, kMaxDevices);
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_base[dev]) {
      // once per device, with that device current: where this GPU's copy of the array lives
      void* base = nullptr;
      hipError_t e = hipGetSymbolAddress(&base, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !base) {
        delete c;
        return fail(EVG_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      }
      g_scratch_base[dev] = static_cast<unsigned char*>(base);
    }
    if (g_scratch_user[dev]) {
      delete c;
      return fail(EVG_ERR_STATE, "the static scratch block of device %d is in use by another context: "
                  "destroy that context first", dev);
    }
    g_scratch_user[dev] = c;
    c->arena_base = g_scratch_base[dev];
    c->arena_dev = dev;
  }
  const uint64_t full_grid = (uint64_t)P * C;
  c->work_grid = (uint32_t)(full_grid < (uint64_t)cus * 8 ? full_grid : (uint64_t)cus * 8);
  TRY_OR_FREE(c->dalloc(&d_chunks, C, false));
  TRY_OR_FREE(c->dalloc(&d_layers, L, false));
  HIP_OR_FREE(hipMemcpyAsync(d_chunks, chunks.data(), C * sizeof(ChunkDesc), hipMemcpyHostToDevice, c->stream));
  HIP_OR_FREE(hipMemcpyAsync(d_layers, layers.data(), L * sizeof(LayerDesc), hipMemcpyHostToDevice, c->stream));
  t.chunks = d_chunks;
  t.layers = d_layers;
  TRY_OR_FREE(c->dalloc(&t.partials, P * C * t.SW, true));
  if (cfg->trigger_kind == EVG_TRIGGER_NORM_DIFF) {
    TRY_OR_FREE(c->dalloc(&t.partials_hat, P * C * t.SW, true));
    TRY_OR_FREE(c->dalloc(&t.xhat_sq, S, true));
  }
  TRY_OR_FREE(c->dalloc(&t.delta, S, false));
  TRY_OR_FREE(c->dalloc(&t.last_norm, S, true));
  TRY_OR_FREE(c->dalloc(&t.delta_before, S, true));
  TRY_OR_FREE(c->dalloc(&t.last_event, S, false));
  TRY_OR_FREE(c->dalloc(&t.valid_l, S, true));
  TRY_OR_FREE(c->dalloc(&t.valid_r, S, true));
  TRY_OR_FREE(c->dalloc(&t.fired, S, true));
  TRY_OR_FREE(c->dalloc(&t.near_tie, S, true));
  TRY_OR_FREE(c->dalloc(&t.ev_full, S, true));
  TRY_OR_FREE(c->dalloc(&t.ev_topk, S, true));
  TRY_OR_FREE(c->dalloc(&t.near_cnt, S, true));
  TRY_OR_FREE(c->dalloc(&t.nonfinite_cnt, S, true));
  TRY_OR_FREE(c->dalloc(&t.slope_hist, S * t.hist_len, true));
  TRY_OR_FREE(c->dalloc(&t.slope_cnt, S, true));
  TRY_OR_FREE(c->dalloc(&t.seg_woff_full, S, true));
  TRY_OR_FREE(c->dalloc(&t.seg_woff_topk, S, true));
  TRY_OR_FREE(c->dalloc(&t.counts, 4, true));
  TRY_OR_FREE(c->dalloc(&t.it, 1, true));
  {
    // decay^k as evg_step computes it, for the steps that take k from the device
    std::vector<double> tab(kDecayTable);
    for (uint32_t k = 0; k < kDecayTable; ++k) tab[k] = std::pow(cfg->synth.decay, (double)k);
    double* d_tab = nullptr;
    TRY_OR_FREE(c->dalloc(&d_tab, kDecayTable, false));
    HIP_OR_FREE(hipMemcpy(d_tab, tab.data(), kDecayTable * sizeof(double), hipMemcpyHostToDevice));
    t.decay_tab = d_tab;
    t.decay_len = kDecayTable;
  }
  TRY_OR_FREE(c->dalloc(&t.work_full, P * C, true));
  // cache-resident ring, whole tensors, same-iteration delivery: the update pass fetches the sends
  // itself from a copy of x it keeps (one more array of the ring's size, library-owned)
  const bool pull = c->cached && !cfg->topk_ppm && !cfg->delivery_delay;
  if (pull) TRY_OR_FREE(c->dalloc(&t.xsnap, 2 * (uint64_t)P * Npad, false));
  if (one_launch) {
    TRY_OR_FREE(c->dalloc(&c->second.partials, P * C * t.SW, true));
    TRY_OR_FREE(c->dalloc(&c->second.delta, S, true));
    TRY_OR_FREE(c->dalloc(&c->second.last_event, S, true));
    if (cfg->trigger_kind == EVG_TRIGGER_NORM_DIFF) TRY_OR_FREE(c->dalloc(&c->second.xhat_sq, S, true));
    c->one_launch = true;
  }
  // a step writes where it reads, unless it is a single-launch step (enqueue_step)
  t.partials_out = t.partials; t.partials_hat_out = t.partials_hat; t.xhat_sq_out = t.xhat_sq;
  t.delta_out = t.delta; t.last_event_out = t.last_event;
  if (cfg->topk_ppm) {
    TRY_OR_FREE(c->dalloc(&t.work_topk, P * C, true));
    TRY_OR_FREE(c->dalloc(&t.hist, S * kHistBins, true));
    TRY_OR_FREE(c->dalloc(&t.sel_prefix, S, true));
    TRY_OR_FREE(c->dalloc(&t.sel_krem, S, true));
    TRY_OR_FREE(c->dalloc(&t.stage_n, P * C, true));
    TRY_OR_FREE(c->dalloc(&t.stage_key, (uint64_t)P * t.stage_stride, false));
    TRY_OR_FREE(c->dalloc(&t.stage_idx, (uint64_t)P * t.stage_stride, false));
    TRY_OR_FREE(c->dalloc(&t.stage_val, (uint64_t)P * t.stage_stride, false));
    TRY_OR_FREE(c->dalloc(&t.chunk_cnt, P * C, true));
    TRY_OR_FREE(c->dalloc(&t.chunk_before, P * C, true));
    TRY_OR_FREE(c->dalloc(&t.chunk_sub, P * C * (t.SW + 1), true));
    TRY_OR_FREE(c->dalloc(&t.msg_idx, (uint64_t)P * ktot, true));
    TRY_OR_FREE(c->dalloc(&t.msg_val, (uint64_t)P * ktot, true));
    TRY_OR_FREE(c->dalloc(&t.idx_hash, S, true));
    TRY_OR_FREE(c->dalloc(&t.msg_hash, S, true));
  } else {
    t.work_topk = t.work_full;   // never listed: k_expand only writes it for Top-K events
  }
  // nothing sent yet: xhat = x, khat = -1, delta = its starting value, v = 0
  const float d0 = cfg->thr_mode == EVG_THR_FIXED ? cfg->thr_fixed : cfg->delta_init;
  std::vector<float> dinit(S, d0);
  HIP_OR_FREE(hipMemcpyAsync(t.delta, dinit.data(), S * sizeof(float), hipMemcpyHostToDevice, c->stream));
  HIP_OR_FREE(hipMemsetAsync(t.last_event, 0xFF, S * sizeof(int32_t), c->stream));
  HIP_OR_FREE(hipMemcpyAsync(t.xhat, t.x, arena_bytes, hipMemcpyDeviceToDevice, c->stream));
  if (t.xsnap) {     // step 1 reads copy 0; both are set so that either parity finds x
    HIP_OR_FREE(hipMemcpyAsync(t.xsnap, t.x, arena_bytes, hipMemcpyDeviceToDevice, c->stream));
    HIP_OR_FREE(hipMemcpyAsync(t.xsnap + (uint64_t)P * Npad, t.x, arena_bytes, hipMemcpyDeviceToDevice, c->stream));
  }
  HIP_OR_FREE(hipMemsetAsync(t.vel, 0, arena_bytes, c->stream));
  HIP_OR_FREE(launch_norm(t, cfg->trigger_kind == EVG_TRIGGER_NORM_DIFF, c->stream));
  HIP_OR_FREE(hipStreamSynchronize(c->stream));   // host staging buffers above go out of scope
#undef TRY_OR_FREE
#undef HIP_OR_FREE
  *out = c;
  return EVG_OK;
}

evg_status evg_init(evg_ctx** out, const evg_config* cfg, void* hip_stream) {
  return init_common(out, cfg, hip_stream, false);
}

evg_status evg_init_static(evg_ctx** out, const evg_config* cfg, void* hip_stream) {
  return init_common(out, cfg, hip_stream, true);
}

// Brings iters / last_iter up to date with the device after replayable steps.
static evg_status refresh_iteration(evg_ctx* c) {
  if (!c->device_ahead) return EVG_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  IterState it{};
  HIP_TRY(hipMemcpy(&it, c->t.it, sizeof it, hipMemcpyDeviceToHost));
  if (it.overflow)
    return fail(EVG_ERR_STATE, "evg_step_next ran past iteration %u, the end of its decay table", kDecayTable - 1);
  c->iters = it.iters;
  c->last_iter = (int64_t)it.k_next - 1;
  return EVG_OK;
}

// The launch sequence of one iteration.  `timed`: bracket the phases with events.
static evg_status enqueue_step(evg_ctx* c, const StepArgs& args, bool timed) {
  const evg_config& g = c->cfg;
  Tables t = c->t;
  StepArgs a = args;
  const bool fused = g.norm_mode == EVG_NORM_FUSED;
  const bool norm_diff = g.trigger_kind == EVG_TRIGGER_NORM_DIFF;
  const bool was_timing = c->timing;
  c->timing = was_timing && timed;
  struct Restore { evg_ctx* c; bool v; ~Restore() { c->timing = v; } } restore{c, was_timing};
  evg_status st;
  // single launch: the update pass runs the trigger tests on the current set of arrays and writes
  // the other set, which is the current one from then on.  Not once evg_step_next has been used:
  // a captured graph holds c->t's pointers.
  const bool single = c->one_launch && !c->replayable_used && !a.from_device;
  if (single) {
    a.one_launch = 1;
    a.step_no = (uint32_t)c->iters;
    t.partials_out = c->second.partials;
    t.xhat_sq_out = c->second.xhat_sq; t.delta_out = c->second.delta; t.last_event_out = c->second.last_event;
  }
  if (a.from_device) HIP_TRY(launch_begin(t, c->stream));
  if (!fused) {
    Phase ph(c, EVG_PH_NORM);
    HIP_TRY(launch_norm(t, norm_diff, c->stream));
    if ((st = ph.end()) != EVG_OK) return st;
  }
  if (!single) {
    Phase ph(c, EVG_PH_TRIGGER);
    HIP_TRY(launch_trigger(t, a, c->stream));
    HIP_TRY(launch_scan(t, a, c->stream));
    HIP_TRY(launch_expand(t, a, c->stream));
    if ((st = ph.end()) != EVG_OK) return st;
  }
  if (!a.delay && !a.pull) {      // with delayed delivery the mailboxes are written after the update;
                                  // a cache-resident ring's receivers fetch the sends in the update pass
    Phase ph(c, EVG_PH_SEND_FULL);
    HIP_TRY(launch_copy(t, a, c->chunk_elems, c->work_grid, c->stream));
    if ((st = ph.end()) != EVG_OK) return st;
  }
  if (a.topk_on) {
    {
      Phase ph(c, EVG_PH_TOPK_SELECT);
      HIP_TRY(launch_topk_select(t, a, c->chunk_elems, c->work_grid, c->stream));
      if ((st = ph.end()) != EVG_OK) return st;
    }
    {
      Phase ph(c, EVG_PH_TOPK_SEND);
      HIP_TRY(launch_topk_send(t, a, c->chunk_elems, c->work_grid, c->stream));
      if ((st = ph.end()) != EVG_OK) return st;
    }
  }
  {
    Phase ph(c, EVG_PH_UPDATE);
    const int norm = !fused ? 0 : !norm_diff ? 1 : g.topk_ppm ? 3 : 2;
    HIP_TRY(launch_update(t, a, g.synth.dist, g.grad_mode, norm, c->stream));
    if ((st = ph.end()) != EVG_OK) return st;
  }
  if (single) {
    Tables& ct = c->t;
    std::swap(ct.partials, c->second.partials);
    std::swap(ct.xhat_sq, c->second.xhat_sq); std::swap(ct.delta, c->second.delta);
    std::swap(ct.last_event, c->second.last_event);
    ct.partials_out = ct.partials; ct.partials_hat_out = ct.partials_hat; ct.xhat_sq_out = ct.xhat_sq;
    ct.delta_out = ct.delta; ct.last_event_out = ct.last_event;
  }
  if (a.delay) {
    Phase ph(c, EVG_PH_DELIVER);
    HIP_TRY(launch_deliver(t, c->chunk_elems, c->work_grid, c->stream));
    if ((st = ph.end()) != EVG_OK) return st;
  }
  c->messages_live = true;
  return EVG_OK;
}

// Everything of StepArgs that does not depend on the iteration.
static evg_status fixed_args(evg_ctx* c, const float* grad, StepArgs* out) {
  const evg_config& g = c->cfg;
  if (g.grad_mode == EVG_GRAD_BUFFER) {
    if (!grad) return fail(EVG_ERR_INVALID, "grad_mode is EVG_GRAD_BUFFER but grad is NULL");
    if ((uintptr_t)grad % 16) return fail(EVG_ERR_ALIGN, "grad is not 16-byte aligned");
    evg_status gs = check_device_array(grad, (uint64_t)c->t.P * c->t.Npad * 4, "grad");
    if (gs != EVG_OK) return gs;
  }
  StepArgs a{};
  a.lr = g.lr;
  a.mu = g.momentum;
  a.plain_sgd = g.momentum == 0.0f ? 1u : 0u;
  a.thr_mode = g.thr_mode;
  a.horizon = g.horizon;
  a.force_first = g.force_first ? 1u : 0u;
  a.topk_on = g.topk_ppm ? 1u : 0u;
  a.topk_key = g.topk_key;
  a.delay = g.delivery_delay;
  a.hist_fused = (g.topk_ppm && g.norm_mode == EVG_NORM_FUSED) ? 1u : 0u;
  a.cached = c->cached ? 1u : 0u;
  a.pull = c->t.xsnap ? 1u : 0u;
  a.xhat_reset = (g.xhat_reset && g.topk_ppm) ? 1u : 0u;
  const bool norm_diff = g.trigger_kind == EVG_TRIGGER_NORM_DIFF;
  // fused + whole-tensor sends: xhat's norm is a scalar per tensor and xhat is never read
  a.norm_src = !norm_diff ? 0u : (g.norm_mode == EVG_NORM_FUSED && !g.topk_ppm) ? 1u : 2u;
  a.key0 = (uint32_t)g.synth.seed;
  a.key1 = (uint32_t)(g.synth.seed >> 32);
  a.spike_prob = g.synth.spike_prob;
  a.spike_gain = g.synth.spike_gain;
  a.grad = grad;
  *out = a;
  return EVG_OK;
}

evg_status evg_step(evg_ctx* c, uint64_t iter, const float* grad) {
  if (!c) return fail(EVG_ERR_INVALID, "context is NULL");
  evg_status st = refresh_iteration(c);
  if (st != EVG_OK) return st;
  if ((int64_t)iter <= c->last_iter || iter >= 0x7FFFFFFFull)
    return fail(EVG_ERR_STATE, "iteration %llu does not follow %lld", (unsigned long long)iter,
                (long long)c->last_iter);
  StepArgs a{};
  if ((st = fixed_args(c, grad, &a)) != EVG_OK) return st;
  a.k = (uint32_t)iter;
  a.decay_pow = std::pow(c->cfg.synth.decay, (double)iter);
  if (c->timing && c->pending.size() > 4096 && (st = c->drain_timers()) != EVG_OK) return st;
  if ((st = enqueue_step(c, a, true)) != EVG_OK) return st;
  c->last_iter = (int64_t)iter;
  c->iters += 1;
  return EVG_OK;
}

evg_status evg_step_next(evg_ctx* c, const float* grad) {
  if (!c) return fail(EVG_ERR_INVALID, "context is NULL");
  StepArgs a{};
  evg_status st = fixed_args(c, grad, &a);
  if (st != EVG_OK) return st;
  a.from_device = 1;
  c->replayable_used = true;
  if ((st = enqueue_step(c, a, false)) != EVG_OK) return st;
  c->device_ahead = true;
  return EVG_OK;
}

evg_status evg_stats(evg_ctx* c, evg_stats_t* out) {
  if (!c || !out) return fail(EVG_ERR_INVALID, "context and out must be non-NULL");
  const Tables& t = c->t;
  const size_t S = t.S;
  HIP_TRY(hipStreamSynchronize(c->stream));
  evg_status rs = refresh_iteration(c);
  if (rs != EVG_OK) return rs;
  std::vector<uint32_t> ef(S), et(S), nt(S), nf(S);
  HIP_TRY(hipMemcpy(ef.data(), t.ev_full, S * 4, hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(et.data(), t.ev_topk, S * 4, hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(nt.data(), t.near_cnt, S * 4, hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(nf.data(), t.nonfinite_cnt, S * 4, hipMemcpyDeviceToHost));
  if (out->last_norm) HIP_TRY(hipMemcpy(out->last_norm, t.last_norm, S * 4, hipMemcpyDeviceToHost));
  if (out->delta) HIP_TRY(hipMemcpy(out->delta, t.delta, S * 4, hipMemcpyDeviceToHost));
  if (out->last_event_iter) HIP_TRY(hipMemcpy(out->last_event_iter, t.last_event, S * 4, hipMemcpyDeviceToHost));
  if (out->valid_l) HIP_TRY(hipMemcpy(out->valid_l, t.valid_l, S, hipMemcpyDeviceToHost));
  if (out->valid_r) HIP_TRY(hipMemcpy(out->valid_r, t.valid_r, S, hipMemcpyDeviceToHost));
  if (out->events_full_rl) std::memcpy(out->events_full_rl, ef.data(), S * 4);
  if (out->events_topk_rl) std::memcpy(out->events_topk_rl, et.data(), S * 4);
  uint64_t e_full = 0, e_topk = 0, vw = 0, iw = 0, near = 0, nonf = 0;
  for (uint32_t r = 0; r < t.P; ++r)
    for (uint32_t l = 0; l < t.L; ++l) {
      const size_t s = (size_t)r * t.L + l;
      e_full += ef[s];
      e_topk += et[s];
      vw += (uint64_t)ef[s] * c->numel[l] + (uint64_t)et[s] * c->K[l];
      iw += (uint64_t)et[s] * c->K[l];
      near += nt[s];
      nonf += nf[s];
    }
  out->iters = c->iters;
  out->events_full = e_full;
  out->events_topk = e_topk;
  out->events_total = e_full + e_topk;
  out->value_words = vw;
  out->index_words = iw;
  out->bytes_sent = 2ull * 4ull * (vw + iw);
  out->regular_events = (uint64_t)t.P * t.L * c->iters;
  out->regular_words = (uint64_t)t.P * c->N * c->iters;
  out->near_tie_flags = near;
  out->nonfinite_norms = nonf;
  uint32_t not_staged = 0;
  HIP_TRY(hipMemcpy(&not_staged, t.counts + 3, 4, hipMemcpyDeviceToHost));
  out->chunks_not_staged = not_staged;
  out->library_bytes = c->owned_bytes;
  return EVG_OK;
}

evg_status evg_last_decisions(evg_ctx* c, uint8_t* fired, uint8_t* near_tie, float* norm, float* delta_before) {
  if (!c) return fail(EVG_ERR_INVALID, "context is NULL");
  const Tables& t = c->t;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (fired) HIP_TRY(hipMemcpy(fired, t.fired, t.S, hipMemcpyDeviceToHost));
  if (near_tie) HIP_TRY(hipMemcpy(near_tie, t.near_tie, t.S, hipMemcpyDeviceToHost));
  if (norm) HIP_TRY(hipMemcpy(norm, t.last_norm, t.S * 4, hipMemcpyDeviceToHost));
  if (delta_before) HIP_TRY(hipMemcpy(delta_before, t.delta_before, t.S * 4, hipMemcpyDeviceToHost));
  return EVG_OK;
}

evg_status evg_message(evg_ctx* c, uint32_t r, uint32_t l, uint32_t* idx, float* val, uint64_t cap,
                       uint64_t* count) {
  if (!c || !count) return fail(EVG_ERR_INVALID, "context and count must be non-NULL");
  const Tables& t = c->t;
  if (r >= t.P || l >= t.L) return fail(EVG_ERR_INVALID, "no worker %u / tensor %u", r, l);
  HIP_TRY(hipStreamSynchronize(c->stream));
  uint8_t code = 0;
  HIP_TRY(hipMemcpy(&code, t.fired + (size_t)r * t.L + l, 1, hipMemcpyDeviceToHost));
  if (code != 2 || !c->cfg.topk_ppm || !c->messages_live) {
    *count = 0;
    return EVG_OK;
  }
  const uint64_t K = c->K[l], n = K < cap ? K : cap;
  const size_t base = (size_t)r * t.Ktot + c->msg_off[l];
  if (idx && n) HIP_TRY(hipMemcpy(idx, t.msg_idx + base, n * 4, hipMemcpyDeviceToHost));
  if (val && n) HIP_TRY(hipMemcpy(val, t.msg_val + base, n * 4, hipMemcpyDeviceToHost));
  *count = K;
  return EVG_OK;
}

evg_status evg_message_hashes(evg_ctx* c, uint64_t* idx_hash, uint64_t* msg_hash) {
  if (!c) return fail(EVG_ERR_INVALID, "context is NULL");
  const Tables& t = c->t;
  const bool live = c->cfg.topk_ppm && c->messages_live;
  if (live) HIP_TRY(launch_message_hashes(t, c->stream));    // from the message buffers of the last step
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (idx_hash) {
    if (live) HIP_TRY(hipMemcpy(idx_hash, t.idx_hash, (size_t)t.S * 8, hipMemcpyDeviceToHost));
    else std::memset(idx_hash, 0, (size_t)t.S * 8);
  }
  if (msg_hash) {
    if (live) HIP_TRY(hipMemcpy(msg_hash, t.msg_hash, (size_t)t.S * 8, hipMemcpyDeviceToHost));
    else std::memset(msg_hash, 0, (size_t)t.S * 8);
  }
  return EVG_OK;
}

evg_status evg_average(evg_ctx* c, float* out) {
  if (!c || !out) return fail(EVG_ERR_INVALID, "context and out must be non-NULL");
  if ((uintptr_t)out % 16) return fail(EVG_ERR_ALIGN, "out is not 16-byte aligned");
  evg_status st = check_device_array(out, c->t.Npad * 4, "out");
  if (st != EVG_OK) return st;
  HIP_TRY(launch_average(c->t, out, c->stream));
  return EVG_OK;
}

}  // extern "C"

namespace {

struct StateHeader {
  char magic[8];
  uint32_t version, P, L, C, SW, S, hist_len, topk_ppm, trigger_kind, norm_mode, thr_mode, pad;
  uint64_t Npad, iters;
  int64_t last_iter;
};

struct Piece { void* dev; size_t bytes; };

// Every library-owned array a later step reads before writing it.
std::vector<Piece> state_pieces(evg_ctx* c) {
  const Tables& t = c->t;
  const size_t S = t.S, sweeps = (size_t)t.P * t.C * t.SW;
  std::vector<Piece> v = {
      {t.delta, S * 4}, {t.last_norm, S * 4}, {t.delta_before, S * 4}, {t.last_event, S * 4},
      {t.valid_l, S}, {t.valid_r, S}, {t.fired, S}, {t.near_tie, S},
      {t.ev_full, S * 4}, {t.ev_topk, S * 4}, {t.near_cnt, S * 4}, {t.nonfinite_cnt, S * 4},
      {t.slope_hist, S * t.hist_len * 4}, {t.slope_cnt, S * 4}, {t.partials, sweeps * 8},
      {t.it, sizeof(IterState)}, {t.counts, 4 * sizeof(uint32_t)}};   // counts[3] is a running counter
  if (t.partials_hat) { v.push_back({t.partials_hat, sweeps * 8}); v.push_back({t.xhat_sq, S * 8}); }
  if (t.hist) v.push_back({t.hist, S * kHistBins * 4});
  return v;
}

StateHeader state_header(evg_ctx* c) {
  StateHeader h{};
  std::memcpy(h.magic, "EVGSTATE", 8);
  h.version = 3;
  h.P = c->t.P; h.L = c->t.L; h.C = c->t.C; h.SW = c->t.SW; h.S = c->t.S;
  h.hist_len = c->t.hist_len;
  h.topk_ppm = c->cfg.topk_ppm;
  h.trigger_kind = c->cfg.trigger_kind;
  h.norm_mode = c->cfg.norm_mode;
  h.thr_mode = c->cfg.thr_mode;
  h.pad = c->cfg.delivery_delay | (c->cfg.xhat_reset << 8);
  h.Npad = c->t.Npad;
  h.iters = c->iters;
  h.last_iter = c->last_iter;
  return h;
}

}  // namespace

extern "C" {

uint64_t evg_state_size(evg_ctx* c) {
  if (!c) return 0;
  uint64_t n = sizeof(StateHeader);
  for (const Piece& p : state_pieces(c)) n += p.bytes;
  return n;
}

evg_status evg_state_export(evg_ctx* c, void* blob, uint64_t capacity) {
  if (!c || !blob) return fail(EVG_ERR_INVALID, "context and blob must be non-NULL");
  if (capacity < evg_state_size(c))
    return fail(EVG_ERR_INVALID, "blob holds %llu bytes, %llu needed", (unsigned long long)capacity,
                (unsigned long long)evg_state_size(c));
  HIP_TRY(hipStreamSynchronize(c->stream));
  evg_status rs = refresh_iteration(c);
  if (rs != EVG_OK) return rs;
  const StateHeader h = state_header(c);
  char* out = static_cast<char*>(blob);
  std::memcpy(out, &h, sizeof h);
  out += sizeof h;
  for (const Piece& p : state_pieces(c)) {
    HIP_TRY(hipMemcpy(out, p.dev, p.bytes, hipMemcpyDeviceToHost));
    out += p.bytes;
  }
  return EVG_OK;
}

evg_status evg_state_import(evg_ctx* c, const void* blob, uint64_t size) {
  if (!c || !blob) return fail(EVG_ERR_INVALID, "context and blob must be non-NULL");
  if (size != evg_state_size(c)) return fail(EVG_ERR_INVALID, "blob size does not match this configuration");
  StateHeader got;
  std::memcpy(&got, blob, sizeof got);
  StateHeader want = state_header(c);
  want.iters = got.iters;
  want.last_iter = got.last_iter;
  if (std::memcmp(&got, &want, sizeof got) != 0)
    return fail(EVG_ERR_INVALID, "blob was exported from a different configuration or version");
  HIP_TRY(hipStreamSynchronize(c->stream));
  const char* in = static_cast<const char*>(blob) + sizeof got;
  for (const Piece& p : state_pieces(c)) {
    HIP_TRY(hipMemcpy(p.dev, in, p.bytes, hipMemcpyHostToDevice));
    in += p.bytes;
  }
  // the library's copy of x follows the caller's arena, which holds the saved parameters again
  if (c->t.xsnap) {
    const size_t arena = (size_t)c->t.P * c->t.Npad;
    HIP_TRY(hipMemcpy(c->t.xsnap, c->t.x, arena * 4, hipMemcpyDeviceToDevice));
    HIP_TRY(hipMemcpy(c->t.xsnap + arena, c->t.x, arena * 4, hipMemcpyDeviceToDevice));
  }
  c->iters = got.iters;
  c->last_iter = got.last_iter;
  c->messages_live = false;         // message buffers are scratch and are not part of the blob
  return EVG_OK;
}

evg_status evg_timing(evg_ctx* c, int enable) {
  if (!c) return fail(EVG_ERR_INVALID, "context is NULL");
  evg_status st = c->drain_timers();
  if (st != EVG_OK) return st;
  for (int i = 0; i < EVG_PH_COUNT; ++i) { c->ms[i] = 0; c->samples[i] = 0; }
  c->timing = enable != 0;
  return EVG_OK;
}

evg_status evg_timing_read(evg_ctx* c, double ms_out[EVG_PH_COUNT], uint64_t samples_out[EVG_PH_COUNT]) {
  if (!c || !ms_out || !samples_out) return fail(EVG_ERR_INVALID, "NULL argument");
  evg_status st = c->drain_timers();
  if (st != EVG_OK) return st;
  for (int i = 0; i < EVG_PH_COUNT; ++i) { ms_out[i] = c->ms[i]; samples_out[i] = c->samples[i]; }
  return EVG_OK;
}

}  // extern "C"
