// Context, CU partition controller, per-phase streams, staging buffers.
//
// Paper, "Computational Resource Controller": the (x, y) split is realised with MPS and can
// only change by replacing the worker processes; the cost is hidden by (1) keeping weights and
// KV cache in a resident owner, (2) preparing the new workers first and switching late, and
// (3) letting each worker switch at its own iteration boundary.  On this GPU a stream's CU
// mask is likewise fixed at creation, so the same three ideas apply to streams: the pool is
// owned outside any stream, spd_set_partition prepares (or re-uses) the new masked streams and
// only stages them, and each phase adopts its staged stream at its next step entry.
#include "internal.h"

#include <string.h>

#include <algorithm>
#include <new>
#include <chrono>
#include <set>
#include <thread>

using namespace spd;

static int round_cus(int x, int gran, int total) {
  if (x < gran) x = gran;
  int r = (x + gran / 2) / gran * gran;
  if (r > total) r = total / gran * gran;
  if (r < gran) r = gran;
  return r;
}

extern "C" int spd_partition_masks(int total_cus, int granularity, int prefill_cus, int decode_cus,
                                   uint32_t* prefill_words, uint32_t* decode_words, int* p_out, int* d_out) {
  if (total_cus <= 0 || granularity <= 0 || total_cus % granularity != 0 || total_cus > 1024) return SPD_EINVAL;
  if (prefill_cus <= 0 || decode_cus <= 0 || !prefill_words || !decode_words) return SPD_EINVAL;
  int p = round_cus(prefill_cus, granularity, total_cus);
  int d = round_cus(decode_cus, granularity, total_cus);
  // a request for disjoint shares stays disjoint after the rounding
  if ((int64_t)prefill_cus + decode_cus <= total_cus && p + d > total_cus) {
    if (p > total_cus - granularity) p = total_cus - granularity;
    d = total_cus - p;
  }
  int words = (total_cus + 31) / 32;
  memset(prefill_words, 0, sizeof(uint32_t) * words);
  memset(decode_words, 0, sizeof(uint32_t) * words);
  for (int i = 0; i < p; ++i) prefill_words[i / 32] |= 1u << (i % 32);
  for (int i = total_cus - d; i < total_cus; ++i) decode_words[i / 32] |= 1u << (i % 32);
  if (p_out) *p_out = p;
  if (d_out) *d_out = d;
  return SPD_OK;
}

static int get_masked_stream(spd_ctx* ctx, int phase, const std::vector<uint32_t>& mask, hipStream_t* out) {
  std::vector<uint32_t> key = mask;
  key.push_back((uint32_t)phase);   // the two phases never share a stream, even with equal masks
  auto it = ctx->stream_cache.find(key);
  if (it != ctx->stream_cache.end()) { *out = it->second; return SPD_OK; }
  hipStream_t s = nullptr;
  SPD_HIP(hipExtStreamCreateWithCUMask(&s, (uint32_t)mask.size(), mask.data()));
  ctx->stream_cache[key] = s;
  *out = s;
  return SPD_OK;
}

extern "C" int spd_ctx_create(int device, spd_ctx** out) {
  if (!out || device < -1) return SPD_EINVAL;
  spd_ctx* c = new (std::nothrow) spd_ctx();
  if (!c) return SPD_EINVAL;
  c->device = device;
  // the two measurement overrides are read here, once: the steps never touch the environment
  if (const char* env = getenv("SPD_PREFILL_PERSISTENT")) c->env_prefill_persistent = atoi(env) != 0;
  if (const char* env = getenv("SPD_DECODE_CHUNK_TILES")) c->env_decode_chunk_tiles = std::max(0, atoi(env));
  if (device >= 0) {
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) { delete c; return hip_fail(e); }
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) { delete c; return SPD_ESTATE; }
    c->total_cus = prop.multiProcessorCount;
    c->xcds = 8;
    if (c->total_cus % c->xcds != 0) c->xcds = 1;
    // An XCD hands its workgroups to its four shader arrays in turn, whatever each array has left of
    // the mask, so a share is only as fast as four times its smallest per-array count (measured: 64, 72
    // and 80 compute units give the same prefill time, 96 and 112 too): whole rows of one compute
    // unit per shader array and XCD.
    c->granularity = c->xcds * 4;
    if (c->total_cus % c->granularity != 0) c->granularity = c->xcds;
    e = hipSetDevice(device);
    if (e != hipSuccess) { delete c; return hip_fail(e); }
  }
  int words = (c->total_cus + 31) / 32;
  std::vector<uint32_t> full(words, 0);
  for (int i = 0; i < c->total_cus; ++i) full[i / 32] |= 1u << (i % 32);
  for (int ph = 0; ph < 2; ++ph) {
    spd_phase_state& s = c->phase[ph];
    s.active_cus = s.pending_cus = c->total_cus;
    s.active_mask = s.pending_mask = full;
    if (device >= 0) {
      int rc = get_masked_stream(c, ph, full, &s.stream);
      hipError_t e = hipSuccess;
      if (rc == SPD_OK) e = hipEventCreate(&s.ev_start);
      if (rc == SPD_OK && e == hipSuccess) e = hipEventCreate(&s.ev_end);
      if (rc == SPD_OK && e == hipSuccess) e = hipEventCreateWithFlags(&s.ev_switch, hipEventDisableTiming);
      if (rc == SPD_OK && e == hipSuccess) e = hipEventCreateWithFlags(&s.ev_cross, hipEventDisableTiming);
      // The decode phase's staging ring exists from the start, with the capacity the entry point that
      // allocates nothing works with; each slot has a device twin of its own and one in the scratch array.
      if (rc == SPD_OK && e == hipSuccess && ph == SPD_PHASE_DECODE) {
        rc = scratch_resolve(device, &c->scratch);
        for (int i = 0; rc == SPD_OK && e == hipSuccess && i < 4; ++i) {
          spd_stage& st = s.ring[i];
          e = hipHostMalloc((void**)&st.host, NOALLOC_STAGE_BYTES, hipHostMallocDefault);
          if (e == hipSuccess) e = hipMalloc((void**)&st.dev, NOALLOC_STAGE_BYTES);
          if (e == hipSuccess) e = hipEventCreateWithFlags(&st.done, hipEventDisableTiming);
          st.cap = NOALLOC_STAGE_BYTES;
          st.dev_static = c->scratch + (size_t)i * NOALLOC_STAGE_BYTES;
        }
      }
      if (rc != SPD_OK || e != hipSuccess) {
        if (e != hipSuccess) hip_fail(e);
        spd_ctx_destroy(c);
        return rc != SPD_OK && rc != SPD_EHIP ? rc : SPD_EHIP;
      }
    }
  }
  *out = c;
  return SPD_OK;
}

extern "C" int spd_ctx_destroy(spd_ctx* ctx) {
  if (!ctx) return SPD_EINVAL;
  if (ctx->device >= 0) {
    (void)hipSetDevice(ctx->device);
    for (auto& kv : ctx->stream_cache) (void)hipStreamSynchronize(kv.second);
    for (int ph = 0; ph < 2; ++ph) {
      spd_phase_state& s = ctx->phase[ph];
      for (spd_stage& st : s.ring) {
        if (st.host) (void)hipHostFree(st.host);
        if (st.dev) (void)hipFree(st.dev);
        if (st.done) (void)hipEventDestroy(st.done);
      }
      if (s.workspace) (void)hipFree(s.workspace);
      for (auto& r : s.ws_retired) (void)hipFree(r.first);
      for (hipEvent_t e : {s.ev_start, s.ev_end, s.ev_switch, s.ev_cross})
        if (e) (void)hipEventDestroy(e);
      for (auto& pair : s.kev)
        for (hipEvent_t e : pair)
          if (e) (void)hipEventDestroy(e);
    }
    for (auto& kv : ctx->stream_cache) (void)hipStreamDestroy(kv.second);
  }
  delete ctx;
  return SPD_OK;
}

extern "C" int spd_device_info(spd_ctx* ctx, int* total_cus, int* xcds, int* cu_granularity) {
  if (!ctx) return SPD_EINVAL;
  if (total_cus) *total_cus = ctx->total_cus;
  if (xcds) *xcds = ctx->xcds;
  if (cu_granularity) *cu_granularity = ctx->granularity;
  return SPD_OK;
}

extern "C" int spd_set_partition(spd_ctx* ctx, int prefill_cus, int decode_cus) {
  if (!ctx) return SPD_EINVAL;
  int words = (ctx->total_cus + 31) / 32;
  std::vector<uint32_t> pm(words), dm(words);
  int p = 0, d = 0;
  int rc = spd_partition_masks(ctx->total_cus, ctx->granularity, prefill_cus, decode_cus, pm.data(), dm.data(), &p, &d);
  if (rc != SPD_OK) return rc;
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  hipStream_t ps = nullptr, ds = nullptr;
  if (ctx->device >= 0) {
    (void)hipSetDevice(ctx->device);
    // preparation: both streams exist before anything is staged, so a failure changes nothing
    if ((rc = get_masked_stream(ctx, SPD_PHASE_PREFILL, pm, &ps)) != SPD_OK) return rc;
    if ((rc = get_masked_stream(ctx, SPD_PHASE_DECODE, dm, &ds)) != SPD_OK) return rc;
  }
  spd_phase_state& P = ctx->phase[SPD_PHASE_PREFILL];
  spd_phase_state& D = ctx->phase[SPD_PHASE_DECODE];
  P.pending_stream = ps; P.pending_cus = p; P.pending_mask = pm; P.has_pending = true;
  D.pending_stream = ds; D.pending_cus = d; D.pending_mask = dm; D.has_pending = true;
  return SPD_OK;
}

extern "C" int spd_get_partition(spd_ctx* ctx, int* prefill_active, int* decode_active, int* prefill_pending,
                                 int* decode_pending) {
  if (!ctx) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  if (prefill_active) *prefill_active = ctx->phase[0].active_cus;
  if (decode_active) *decode_active = ctx->phase[1].active_cus;
  if (prefill_pending) *prefill_pending = ctx->phase[0].has_pending ? ctx->phase[0].pending_cus : ctx->phase[0].active_cus;
  if (decode_pending) *decode_pending = ctx->phase[1].has_pending ? ctx->phase[1].pending_cus : ctx->phase[1].active_cus;
  return SPD_OK;
}

extern "C" int spd_phase_cu_mask(spd_ctx* ctx, int phase, uint32_t* words, int32_t cap, int32_t* n_words) {
  if (!ctx || phase < 0 || phase > 1 || !n_words || cap < 0 || (cap > 0 && !words)) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  const std::vector<uint32_t>& m = ctx->phase[phase].active_mask;
  *n_words = (int32_t)m.size();
  if ((size_t)cap < m.size()) return SPD_EINVAL;
  memcpy(words, m.data(), m.size() * sizeof(uint32_t));
  return SPD_OK;
}

namespace spd {

// Step entry of one phase: adopt the staged partition, if any (asynchronous switching: the
// other phase is not consulted).  The new stream first waits, on the GPU, for the old
// stream's last work, so that the phase's own steps stay ordered across the switch.
int phase_enter(spd_ctx* ctx, int phase, hipStream_t* stream_out) {
  if (ctx->device < 0) return SPD_ESTATE;
  SPD_HIP(hipSetDevice(ctx->device));
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  spd_phase_state& s = ctx->phase[phase];
  if (s.has_pending) {
    if (s.pending_stream != s.stream) {
      SPD_HIP(hipEventRecord(s.ev_switch, s.stream));
      SPD_HIP(hipStreamWaitEvent(s.pending_stream, s.ev_switch, 0));
      s.stream = s.pending_stream;
    }
    s.active_cus = s.pending_cus;
    s.active_mask = s.pending_mask;
    s.has_pending = false;
  }
  *stream_out = s.stream;
  return SPD_OK;
}

static void raise_done_seq(spd_phase_state& s, uint64_t seq) {
  uint64_t cur = s.done_seq.load(std::memory_order_relaxed);
  while (cur < seq && !s.done_seq.compare_exchange_weak(cur, seq, std::memory_order_release)) {
  }
}

int stage_acquire(spd_ctx* ctx, int phase, size_t bytes, spd_stage** out, bool may_alloc) {
  spd_phase_state& s = ctx->phase[phase];
  spd_stage& st = s.ring[s.ring_pos];
  if (st.in_flight) {
    // Poll, with pauses, instead of hipEventSynchronize: a blocking wait inside the runtime (and a
    // tight polling loop as well) keeps the other phase's thread from launching meanwhile.
    hipError_t e;
    while ((e = hipEventQuery(st.done)) == hipErrorNotReady) std::this_thread::sleep_for(std::chrono::microseconds(20));
    if (e != hipSuccess) return hip_fail(e);
    st.in_flight = false;
    raise_done_seq(s, st.seq.load(std::memory_order_relaxed));
  }
  if (!may_alloc && (!st.done || st.cap < bytes || !st.dev_static)) return SPD_ETOOBIG;
  if (!st.done) SPD_HIP(hipEventCreateWithFlags(&st.done, hipEventDisableTiming));
  if (st.cap < bytes) {
    size_t cap = std::max<size_t>(256 * 1024, st.cap);
    while (cap < bytes) cap *= 2;
    char *h = nullptr, *d = nullptr;
    SPD_HIP(hipHostMalloc((void**)&h, cap, hipHostMallocDefault));
    hipError_t e = hipMalloc((void**)&d, cap);
    if (e != hipSuccess) { (void)hipHostFree(h); return hip_fail(e); }
    if (st.host) (void)hipHostFree(st.host);
    if (st.dev) (void)hipFree(st.dev);
    st.host = h; st.dev = d; st.cap = cap;
  }
  *out = &st;
  return SPD_OK;
}

int stage_host_as_device(spd_stage* st, void** out) {
  SPD_HIP(hipHostGetDevicePointer(out, st->host, 0));
  return SPD_OK;
}

int stage_copy(spd_stage* st, size_t bytes, hipStream_t stream, char* dev) {
  // The step's metadata crosses to the device with a small copy kernel on the phase's own stream
  // (pinned host memory is device-readable).  hipMemcpyAsync would put it on a copy path that the
  // two phases share: with each phase driven by its own thread the copies then wait for each
  // other's predecessors and one phase starves the other.
  void* host_dev = nullptr;
  SPD_HIP(hipHostGetDevicePointer(&host_dev, st->host, 0));
  SPD_HIP(launch_copy(dev ? dev : st->dev, host_dev, (bytes + 15) & ~(size_t)15, 1, stream));
  return SPD_OK;
}

// Called behind the step's last kernel: the slot's event then also says that the step has finished, which is
// what spd_kv_free asks about.
int stage_commit(spd_ctx* ctx, int phase, spd_stage* st, size_t bytes, hipStream_t stream, bool copy, char* dev) {
  spd_phase_state& s = ctx->phase[phase];
  if (copy) {
    int rc = stage_copy(st, bytes, stream, dev);
    if (rc != SPD_OK) return rc;
  }
  SPD_HIP(hipEventRecord(st->done, stream));
  st->seq.store(s.issue_seq.load(std::memory_order_relaxed) + 1, std::memory_order_release);   // after the record
  s.issue_seq.fetch_add(1, std::memory_order_release);
  st->in_flight = true;
  s.ring_pos = (s.ring_pos + 1) % 4;
  return SPD_OK;
}

bool phase_step_done(spd_ctx* ctx, int phase, uint64_t seq) {
  if (seq == 0 || ctx->device < 0) return true;
  spd_phase_state& s = ctx->phase[phase];
  if (s.done_seq.load(std::memory_order_acquire) >= seq) return true;
  (void)hipSetDevice(ctx->device);
  // A slot whose number is `seq` or later carries an event recorded behind that step's last kernel (the number is
  // stored after the record, so reading it first means the event is at least that recent).
  for (spd_stage& st : s.ring) {
    const uint64_t q = st.seq.load(std::memory_order_acquire);
    if (q >= seq && st.done && hipEventQuery(st.done) == hipSuccess) {
      raise_done_seq(s, q);
      return true;
    }
  }
  (void)hipGetLastError();      // hipErrorNotReady is not an error to keep
  return false;
}

static void workspace_release_retired(spd_ctx* ctx, int phase) {
  spd_phase_state& s = ctx->phase[phase];
  std::lock_guard<std::mutex> lk(s.ws_mu);
  size_t keep = 0;
  for (auto& r : s.ws_retired) {
    if (phase_step_done(ctx, phase, r.second)) (void)hipFree(r.first);
    else s.ws_retired[keep++] = r;
  }
  s.ws_retired.resize(keep);
}

int workspace_reserve(spd_ctx* ctx, int phase, size_t bytes, char** out) {
  spd_phase_state& s = ctx->phase[phase];
  if (s.ws_cap < bytes) {
    size_t cap = std::max<size_t>(16u << 20, s.ws_cap);
    while (cap < bytes) cap *= 2;
    char* d = nullptr;
    SPD_HIP(hipMalloc((void**)&d, cap));
    // Earlier steps of this phase may still read the old buffer: it is kept until the last of them (the step
    // issued most recently; the one being built takes the new buffer) is known to have finished.  No wait here.
    if (s.workspace) {
      std::lock_guard<std::mutex> lk(s.ws_mu);
      s.ws_retired.emplace_back(s.workspace, s.issue_seq.load(std::memory_order_acquire));
    }
    s.workspace = d;
    s.ws_cap = cap;
    workspace_release_retired(ctx, phase);
  }
  *out = s.workspace;
  return SPD_OK;
}

int kernel_timing_mark(spd_ctx* ctx, int phase, int which, hipStream_t stream) {
  if (!ctx->kernel_timing) return SPD_OK;
  spd_phase_state& s = ctx->phase[phase];
  hipEvent_t& e = s.kev[s.kev_count % 256][which];
  if (!e) SPD_HIP(hipEventCreate(&e));
  SPD_HIP(hipEventRecord(e, stream));
  if (which == 1) ++s.kev_count;
  return SPD_OK;
}

}  // namespace spd

extern "C" int spd_set_kernel_timing(spd_ctx* ctx, int on) {
  if (!ctx) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  ctx->kernel_timing = on != 0;
  return SPD_OK;
}

extern "C" int spd_phase_kernel_ms(spd_ctx* ctx, int phase, float* out, int32_t cap, int32_t* n_out) {
  if (!ctx || phase < 0 || phase > 1 || !n_out || cap < 0 || (cap > 0 && !out)) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  int rc = spd_phase_sync(ctx, phase);
  if (rc != SPD_OK) return rc;
  spd_phase_state& s = ctx->phase[phase];
  uint64_t first = s.kev_count > 256 ? s.kev_count - 256 : 0;
  if (first < s.kev_read) first = s.kev_read;
  int32_t n = 0;
  for (uint64_t i = first; i < s.kev_count && n < cap; ++i, ++n)
    SPD_HIP(hipEventElapsedTime(&out[n], s.kev[i % 256][0], s.kev[i % 256][1]));
  s.kev_read = first + (uint64_t)n;
  *n_out = n;
  return SPD_OK;
}

extern "C" int spd_phase_sync(spd_ctx* ctx, int phase) {
  if (!ctx || phase < 0 || phase > 1) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  hipStream_t s;
  { std::lock_guard<std::mutex> lk(ctx->part_mu); s = ctx->phase[phase].stream; }
  const uint64_t issued = ctx->phase[phase].issue_seq.load(std::memory_order_acquire);
  SPD_HIP(hipStreamSynchronize(s));
  raise_done_seq(ctx->phase[phase], issued);
  workspace_release_retired(ctx, phase);
  return SPD_OK;
}

extern "C" int spd_phase_query(spd_ctx* ctx, int phase, int* done) {
  if (!ctx || phase < 0 || phase > 1 || !done) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  hipStream_t s;
  { std::lock_guard<std::mutex> lk(ctx->part_mu); s = ctx->phase[phase].stream; }
  const uint64_t issued = ctx->phase[phase].issue_seq.load(std::memory_order_acquire);
  hipError_t e = hipStreamQuery(s);
  if (e == hipSuccess) { raise_done_seq(ctx->phase[phase], issued); *done = 1; return SPD_OK; }
  if (e == hipErrorNotReady) { *done = 0; return SPD_OK; }
  return hip_fail(e);
}

extern "C" int spd_phase_wait_for(spd_ctx* ctx, int phase, int other) {
  if (!ctx || phase < 0 || phase > 1 || other < 0 || other > 1 || phase == other) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  spd_phase_state& me = ctx->phase[phase];
  SPD_HIP(hipEventRecord(me.ev_cross, ctx->phase[other].stream));
  SPD_HIP(hipStreamWaitEvent(me.stream, me.ev_cross, 0));
  return SPD_OK;
}

extern "C" int spd_phase_stream(spd_ctx* ctx, int phase, void** hip_stream_out) {
  if (!ctx || phase < 0 || phase > 1 || !hip_stream_out) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  std::lock_guard<std::mutex> lk(ctx->part_mu);
  *hip_stream_out = (void*)ctx->phase[phase].stream;
  return SPD_OK;
}

extern "C" int spd_phase_last_ms(spd_ctx* ctx, int phase, float* ms) {
  if (!ctx || phase < 0 || phase > 1 || !ms) return SPD_EINVAL;
  if (ctx->device < 0 || !ctx->phase[phase].timed) return SPD_ESTATE;
  SPD_HIP(hipEventSynchronize(ctx->phase[phase].ev_end));
  SPD_HIP(hipEventElapsedTime(ms, ctx->phase[phase].ev_start, ctx->phase[phase].ev_end));
  return SPD_OK;
}

extern "C" int spd_phase_copy(spd_ctx* ctx, int phase, void* dst, const void* src, uint64_t bytes) {
  if (!ctx || phase < 0 || phase > 1 || !dst || !src || bytes == 0 || bytes % 16 != 0) return SPD_EINVAL;
  if (((uintptr_t)dst | (uintptr_t)src) & 15) return SPD_EINVAL;
  hipStream_t stream;
  int rc = phase_enter(ctx, phase, &stream);
  if (rc != SPD_OK) return rc;
  SPD_HIP(launch_copy(dst, src, bytes, ctx->phase[phase].active_cus, stream));
  return SPD_OK;
}

extern "C" int spd_phase_read(spd_ctx* ctx, int phase, const void* src, uint64_t bytes) {
  if (!ctx || phase < 0 || phase > 1 || !src || bytes == 0 || bytes % 16 != 0) return SPD_EINVAL;
  if ((uintptr_t)src & 15) return SPD_EINVAL;
  hipStream_t stream;
  int rc = phase_enter(ctx, phase, &stream);
  if (rc != SPD_OK) return rc;
  SPD_HIP(launch_read(src, bytes, ctx->phase[phase].active_cus, nullptr, stream));
  return SPD_OK;
}

extern "C" int spd_phase_read_lds(spd_ctx* ctx, int phase, const void* src, uint64_t bytes) {
  if (!ctx || phase < 0 || phase > 1 || !src || bytes == 0 || bytes % 16 != 0) return SPD_EINVAL;
  if ((uintptr_t)src & 15) return SPD_EINVAL;
  hipStream_t stream;
  int rc = phase_enter(ctx, phase, &stream);
  if (rc != SPD_OK) return rc;
  SPD_HIP(launch_read_lds(src, bytes, ctx->phase[phase].active_cus, nullptr, stream));
  return SPD_OK;
}

extern "C" int spd_clock_probe(spd_ctx* ctx, void* hip_stream, uint64_t iters, uint64_t* dev_out) {
  if (!ctx || !dev_out || iters == 0 || iters > (1ull << 32)) return SPD_EINVAL;
  if ((uintptr_t)dev_out & 7) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  SPD_HIP(hipSetDevice(ctx->device));
  SPD_HIP(launch_clock_probe(iters, dev_out, (hipStream_t)hip_stream));
  return SPD_OK;
}

extern "C" int spd_issue_probe(spd_ctx* ctx, void* hip_stream, uint64_t* dev_out) {
  if (!ctx || !dev_out || ((uintptr_t)dev_out & 7)) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  SPD_HIP(hipSetDevice(ctx->device));
  SPD_HIP(launch_issue_probe(dev_out, (hipStream_t)hip_stream));
  return SPD_OK;
}

extern "C" int spd_phase_probe_cus(spd_ctx* ctx, int phase, int32_t n_blocks, int32_t* ids, int32_t cap,
                                   int32_t* n_ids) {
  if (!ctx || phase < 0 || phase > 1 || n_blocks <= 0 || n_blocks > (1 << 20) || !ids || cap <= 0 || !n_ids)
    return SPD_EINVAL;
  hipStream_t stream;
  int rc = phase_enter(ctx, phase, &stream);
  if (rc != SPD_OK) return rc;
  char* ws = nullptr;
  if ((rc = workspace_reserve(ctx, phase, sizeof(int32_t) * (size_t)n_blocks, &ws)) != SPD_OK) return rc;
  SPD_HIP(launch_probe((int32_t*)ws, n_blocks, stream));
  std::vector<int32_t> host((size_t)n_blocks);
  SPD_HIP(hipMemcpyAsync(host.data(), ws, sizeof(int32_t) * (size_t)n_blocks, hipMemcpyDeviceToHost, stream));
  SPD_HIP(hipStreamSynchronize(stream));
  std::set<int32_t> uniq(host.begin(), host.end());
  *n_ids = (int32_t)uniq.size();
  if ((size_t)cap < uniq.size()) return SPD_EINVAL;
  std::copy(uniq.begin(), uniq.end(), ids);
  return SPD_OK;
}
