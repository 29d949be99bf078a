// Host side of the two steps and of the page write / gather: validation, atomic block
// reservation, block-table staging, launch geometry.  All arithmetic of the method runs in
// the kernels (kernels_*.hip).
#include "internal.h"
#include "prefill_work.h"

#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <functional>
#include <new>
#include <thread>
#include <cmath>

using namespace spd;

namespace spd {
int64_t blocks_missing_locked(spd_pool* pool, uint64_t req, int64_t n_tokens);
uint64_t reserve_locked(spd_pool* pool, uint64_t req, int64_t n_tokens);
}  // namespace spd

static inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// Tile descriptors covering logical positions [start, start + n) of a request whose block
// table is `bt`; dense row src_row0 maps to position `start`.
static void build_tile_descs(const PoolGeom& g, const int32_t* bt, int32_t start, int32_t n, int32_t src_row0,
                             std::vector<TileDesc>& out) {
  int32_t pos = start, end = start + n;
  while (pos < end) {
    int32_t tile = pos / TILE_T, t_begin = pos % TILE_T;
    int32_t t_end = std::min<int32_t>(TILE_T, t_begin + (end - pos));
    TileDesc d{};
    d.src_row = src_row0 + (pos - start);
    d.page = bt[tile / g.tiles_per_page];
    d.sub = tile % g.tiles_per_page;
    d.t_begin = t_begin;
    d.t_end = t_end;
    d.pad[0] = tile * TILE_T;
    out.push_back(d);
    pos += t_end - t_begin;
  }
}

// The kernels move 16 bytes per lane: every tensor a step is given must start on a 16-byte boundary.
static bool misaligned16(const void* a, const void* b = nullptr, const void* c = nullptr, const void* d = nullptr,
                         const void* e = nullptr) {
  return (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)d | (uintptr_t)e) & 15) != 0;
}

// The number the phase's step now being prepared will carry (its staging slot's commit assigns it).
static uint64_t next_step_number(spd_ctx* ctx, int phase) {
  return ctx->phase[phase].issue_seq.load(std::memory_order_relaxed) + 1;
}

static int kv_copy(spd_ctx* ctx, spd_pool* pool, int phase, uint64_t req_id, int32_t start_pos, int32_t n_tokens,
                   const void* k, const void* v, bool write) {
  if (!ctx || !pool || pool->ctx != ctx || phase < 0 || phase > 1 || start_pos < 0 || n_tokens <= 0 || !k)
    return SPD_EINVAL;
  const PoolGeom& g = pool->geom;
  if ((g.kind == SPD_KV_GQA) != (v != nullptr)) return SPD_EINVAL;
  if (misaligned16(k, v)) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  std::vector<TileDesc> descs;
  {
    std::lock_guard<std::mutex> lk(pool->mu);
    auto it = pool->tables.find(req_id);
    if (it == pool->tables.end()) return SPD_ENOENT;
    int64_t need = ((int64_t)start_pos + n_tokens + g.P - 1) / g.P;
    if ((int64_t)it->second.size() < need) return SPD_EINVAL;
    build_tile_descs(g, it->second.data(), start_pos, n_tokens, 0, descs);
    it->second.last_use[phase] = next_step_number(ctx, phase);
  }
  hipStream_t stream;
  int rc = phase_enter(ctx, phase, &stream);
  if (rc != SPD_OK) return rc;
  size_t bytes = descs.size() * sizeof(TileDesc);
  spd_stage* st;
  if ((rc = stage_acquire(ctx, phase, bytes, &st)) != SPD_OK) return rc;
  memcpy(st->host, descs.data(), bytes);
  if ((rc = stage_copy(st, bytes, stream)) != SPD_OK) return rc;
  const bool fp8 = g.kind == SPD_KV_MLA_LATENT_FP8;
  if (write && fp8)
    SPD_HIP(launch_kv_write_fp8(g, pool->base, (const TileDesc*)st->dev, (int)descs.size(), k, stream));
  else if (write)
    SPD_HIP(launch_kv_write(g, pool->base, (const TileDesc*)st->dev, (int)descs.size(), k, v, stream));
  else if (fp8)
    SPD_HIP(launch_kv_gather_fp8(g, pool->base, (const TileDesc*)st->dev, (int)descs.size(), (void*)k, stream));
  else
    SPD_HIP(launch_kv_gather(g, pool->base, (const TileDesc*)st->dev, (int)descs.size(), (void*)k, (void*)v, stream));
  return stage_commit(ctx, phase, st, bytes, stream, false);
}

extern "C" int spd_kv_write(spd_ctx* ctx, spd_pool* pool, int phase, uint64_t req_id, int32_t start_pos,
                            int32_t n_tokens, const void* k, const void* v) {
  return kv_copy(ctx, pool, phase, req_id, start_pos, n_tokens, k, v, true);
}

extern "C" int spd_kv_gather(spd_ctx* ctx, spd_pool* pool, int phase, uint64_t req_id, int32_t n_tokens,
                             void* k_out, void* v_out) {
  return kv_copy(ctx, pool, phase, req_id, 0, n_tokens, k_out, v_out, false);
}

// ------------------------------------------------------------------------------------------ prefill
extern "C" int spd_prefill_step(spd_ctx* ctx, spd_pool* pool, const spd_prefill_batch* b) {
  if (!ctx || !pool || pool->ctx != ctx || !b || b->n_req <= 0 || !b->req_ids || !b->cu_seqlens) return SPD_EINVAL;
  if (!b->q || !b->k || !b->v || !b->out || b->n_q_heads <= 0 || b->n_kv_heads <= 0) return SPD_EINVAL;
  const PoolGeom& g = pool->geom;
  if (b->n_q_heads % b->n_kv_heads != 0 || b->cu_seqlens[0] != 0) return SPD_EINVAL;
  if (!(b->scale > 0.f) || !std::isfinite(b->scale)) return SPD_EINVAL;
  if (g.kind == SPD_KV_GQA) {
    if (b->latent || b->n_kv_heads != g.Hkv || b->dim_qk != g.dk || b->dim_v != g.dv) return SPD_EINVAL;
  } else {
    if (!b->latent || b->n_kv_heads != b->n_q_heads) return SPD_EINVAL;
  }
  if (!prefill_shape_supported(b->dim_qk, b->dim_v)) return SPD_EINVAL;
  if (misaligned16(b->q, b->k, b->v, b->out, b->latent)) return SPD_EINVAL;
  if (b->rope) {
    if (g.kind != SPD_KV_GQA) return SPD_EINVAL;
    int rrc = rope_config_check(b->rope);
    if (rrc != SPD_OK) return rrc;
    if (b->rope->rotary_dim % 16 || b->rope->rotary_offset % 8 || b->rope->rotary_offset + b->rope->rotary_dim > b->dim_qk)
      return SPD_EINVAL;
  }
  for (int r = 0; r < b->n_req; ++r) {
    if (b->cu_seqlens[r + 1] <= b->cu_seqlens[r]) return SPD_EINVAL;     // zero-length prompt
    for (int r2 = 0; r2 < r; ++r2)
      if (b->req_ids[r2] == b->req_ids[r]) return SPD_EINVAL;
  }
  if (ctx->device < 0) return SPD_ESTATE;

  // chunked prefill: some request continues a prompt whose first prefix_lens[r] tokens are cached
  bool chunked = false;
  if (b->prefix_lens) {
    if (g.kind != SPD_KV_GQA) return SPD_EINVAL;
    for (int r = 0; r < b->n_req; ++r) {
      if (b->prefix_lens[r] < 0) return SPD_EINVAL;
      chunked = chunked || b->prefix_lens[r] > 0;
    }
  }
  // rows of each request in the gathered K, V (prefix + this step's rows)
  std::vector<int32_t> kv_cu;
  if (chunked) {
    kv_cu.resize((size_t)b->n_req + 1, 0);
    for (int r = 0; r < b->n_req; ++r) {
      const int64_t rows = (int64_t)kv_cu[(size_t)r] + b->prefix_lens[r] + (b->cu_seqlens[r + 1] - b->cu_seqlens[r]);
      if (rows > INT32_MAX) return SPD_EINVAL;
      kv_cu[(size_t)r + 1] = (int32_t)rows;
    }
  }

  int rc;
  // One persistent workgroup per compute unit of the prefill share, each with its chain of work
  // items, where such a launch gets one compute unit per workgroup: an XCD deals its workgroups to
  // its four shader arrays in turn, so every XCD must contribute a multiple of 4 compute units (the
  // partition granularity sees to that; with 10 per XCD some workgroups wait for others to finish,
  // and the step takes up to twice as long).  Elsewhere: one workgroup per item, handed out by the
  // hardware as compute units free up.
  // Nor where the two phases' masks overlap: a persistent workgroup keeps its compute unit for the
  // whole kernel, and decode workgroups that are allowed nowhere else would wait that long.
  // The share is the one this step will run on: a staged partition is adopted below, once nothing but a HIP
  // call can fail any more, so a step that returns an error of its own leaves the partition as it was.
  int share;
  bool persistent;
  {
    std::lock_guard<std::mutex> lk(ctx->part_mu);
    const spd_phase_state& psx = ctx->phase[SPD_PHASE_PREFILL];
    share = std::max(1, psx.has_pending ? psx.pending_cus : psx.active_cus);
    persistent = share % ctx->xcds == 0 && (share / ctx->xcds) % 4 == 0;
    const std::vector<uint32_t>& pm = psx.has_pending ? psx.pending_mask : psx.active_mask;
    const spd_phase_state& dsx = ctx->phase[SPD_PHASE_DECODE];
    const std::vector<uint32_t>& dm = dsx.has_pending ? dsx.pending_mask : dsx.active_mask;
    for (size_t i = 0; i < pm.size() && i < dm.size(); ++i)
      if (pm[i] & dm[i]) persistent = false;
    if (dsx.has_pending)
      for (size_t i = 0; i < pm.size() && i < dsx.active_mask.size(); ++i)
        if (pm[i] & dsx.active_mask[i]) persistent = false;
  }
  if (ctx->env_prefill_persistent >= 0) persistent = ctx->env_prefill_persistent != 0;   // experiment switch
  std::vector<PrefillWork> work;
  std::vector<int32_t> chain;
  build_prefill_chains(b->cu_seqlens, chunked ? b->prefix_lens : nullptr, chunked ? kv_cu.data() : nullptr, b->n_req,
                       b->n_q_heads, b->n_kv_heads, ctx->xcds, persistent ? share : 0, work, chain);
  const int n_blocks = (int)chain.size() - 1;

  size_t n_descs = 0, n_gather = 0;
  for (int r = 0; r < b->n_req; ++r) {
    const int32_t len = b->cu_seqlens[r + 1] - b->cu_seqlens[r], pre = chunked ? b->prefix_lens[r] : 0;
    n_descs += (size_t)((pre % TILE_T) + len + TILE_T - 1) / TILE_T;
    if (chunked) n_gather += (size_t)(pre + len + TILE_T - 1) / TILE_T;
  }
  size_t off_chain = align16(work.size() * sizeof(PrefillWork));
  size_t off_desc = align16(off_chain + chain.size() * sizeof(int32_t));
  size_t off_gather = align16(off_desc + n_descs * sizeof(TileDesc));
  // RoPE inside the step: the frequency table, and every row's position for the rotation of q
  const int32_t n_rows = b->cu_seqlens[b->n_req];
  size_t off_w = align16(off_gather + n_gather * sizeof(TileDesc));
  size_t off_pos = align16(off_w + (b->rope ? sizeof(double) * (size_t)(b->rope->rotary_dim / 2) : 0));
  size_t bytes = off_pos + (b->rope ? sizeof(int32_t) * (size_t)n_rows : 0);
  spd_stage* st;
  if ((rc = stage_acquire(ctx, SPD_PHASE_PREFILL, bytes, &st)) != SPD_OK) return rc;
  char* ws = nullptr;
  size_t ws_k_bytes = 0;
  if (chunked) {
    ws_k_bytes = align16((size_t)kv_cu.back() * g.Hkv * g.dk * 2);
    const size_t ws_v_bytes = (size_t)kv_cu.back() * g.Hkv * g.dv * 2;
    if ((rc = workspace_reserve(ctx, SPD_PHASE_PREFILL, ws_k_bytes + ws_v_bytes, &ws)) != SPD_OK) return rc;
  }
  std::vector<TileDesc> descs, gdescs;
  descs.reserve(n_descs);
  gdescs.reserve(n_gather);
  {
    std::lock_guard<std::mutex> lk(pool->mu);                       // atomic: query, get, update
    int64_t need = 0;
    for (int r = 0; r < b->n_req; ++r) {
      const int32_t len = b->cu_seqlens[r + 1] - b->cu_seqlens[r], pre = chunked ? b->prefix_lens[r] : 0;
      if (pre > 0) {                                                // the cached prefix must be there
        auto it = pool->tables.find(b->req_ids[r]);
        if (it == pool->tables.end()) return SPD_ENOENT;
        if ((int64_t)it->second.size() * g.P < pre) return SPD_EINVAL;
      }
      need += blocks_missing_locked(pool, b->req_ids[r], pre + len);
    }
    if (need > (int64_t)pool->free_stack.size()) return SPD_ENOMEM;
    for (int r = 0; r < b->n_req; ++r) {
      const int32_t row0 = b->cu_seqlens[r], len = b->cu_seqlens[r + 1] - row0, pre = chunked ? b->prefix_lens[r] : 0;
      reserve_locked(pool, b->req_ids[r], pre + len);
      spd_req_table& entry = pool->tables[b->req_ids[r]];
      entry.last_use[SPD_PHASE_PREFILL] = next_step_number(ctx, SPD_PHASE_PREFILL);
      const int32_t* table = entry.data();
      build_tile_descs(g, table, pre, len, row0, descs);
      if (chunked) build_tile_descs(g, table, 0, pre + len, kv_cu[(size_t)r], gdescs);
    }
  }
  hipStream_t stream;
  if ((rc = phase_enter(ctx, SPD_PHASE_PREFILL, &stream)) != SPD_OK) return rc;
  memcpy(st->host, work.data(), work.size() * sizeof(PrefillWork));
  memcpy(st->host + off_chain, chain.data(), chain.size() * sizeof(int32_t));
  memcpy(st->host + off_desc, descs.data(), descs.size() * sizeof(TileDesc));
  if (chunked) memcpy(st->host + off_gather, gdescs.data(), gdescs.size() * sizeof(TileDesc));
  if (b->rope) {
    rope_frequencies(b->rope, (double*)(st->host + off_w));
    int32_t* pos = (int32_t*)(st->host + off_pos);
    for (int r = 0; r < b->n_req; ++r)
      for (int32_t i = b->cu_seqlens[r]; i < b->cu_seqlens[r + 1]; ++i)
        pos[i] = (chunked ? b->prefix_lens[r] : 0) + (i - b->cu_seqlens[r]);
  }
  spd_phase_state& ps = ctx->phase[SPD_PHASE_PREFILL];
  if (ctx->kernel_timing) SPD_HIP(hipEventRecord(ps.ev_start, stream));
  const void* page_src_k = g.kind == SPD_KV_GQA ? b->k : b->latent;
  const void* page_src_v = g.kind == SPD_KV_GQA ? b->v : nullptr;
  // one launch: the page write reads its descriptors straight out of the pinned staging buffer,
  // and extra workgroups of the same kernel copy the whole staging buffer to its device twin,
  // where the attention kernel (and the gather of a chunked step) find their lists
  void* host_dev = nullptr;
  if ((rc = stage_host_as_device(st, &host_dev)) != SPD_OK) return rc;
  const spd_rope_config* rc_ = b->rope;
  const bool fused = rc_ && kv_write_can_rotate(g);
  if (rc_ && !fused)        // no fused form for this pool shape: q and k in one pass of their own, before the page write
    SPD_HIP(launch_rope((void*)b->q, b->n_q_heads, (void*)b->k, b->n_kv_heads, b->dim_qk, rc_->rotary_dim, rc_->rotary_offset,
                        rc_->interleaved != 0, n_rows, (const int32_t*)((const char*)host_dev + off_pos),
                        (const double*)((const char*)host_dev + off_w), stream));
  if (g.kind == SPD_KV_MLA_LATENT_FP8)
    SPD_HIP(launch_kv_write_fp8(g, pool->base, (const TileDesc*)((const char*)host_dev + off_desc), (int)descs.size(), page_src_k,
                                stream, st->dev, host_dev, bytes));
  else
    SPD_HIP(launch_kv_write(g, pool->base, (const TileDesc*)((const char*)host_dev + off_desc), (int)descs.size(), page_src_k,
                            page_src_v, stream, st->dev, host_dev, bytes,
                            fused ? (const double*)((const char*)host_dev + off_w) : nullptr, fused ? rc_->rotary_dim : 0,
                            fused ? rc_->rotary_offset : 0, fused && rc_->interleaved != 0));
  if (fused)                // the keys were rotated on their way into the pages (and in place); the queries here
    SPD_HIP(launch_rope((void*)b->q, b->n_q_heads, nullptr, 0, b->dim_qk, rc_->rotary_dim, rc_->rotary_offset,
                        rc_->interleaved != 0, n_rows, (const int32_t*)(st->dev + off_pos), (const double*)(st->dev + off_w),
                        stream));
  const void *att_k = b->k, *att_v = b->v;
  if (chunked) {
    // every request's rows 0 .. prefix+len-1, the new ones included, back out of the pages
    SPD_HIP(launch_kv_gather(g, pool->base, (const TileDesc*)(st->dev + off_gather), (int)gdescs.size(), ws,
                             ws + ws_k_bytes, stream));
    att_k = ws;
    att_v = ws + ws_k_bytes;
  }
  if ((rc = kernel_timing_mark(ctx, SPD_PHASE_PREFILL, 0, stream)) != SPD_OK) return rc;
  SPD_HIP(launch_prefill(b->q, att_k, att_v, b->out, (const PrefillWork*)st->dev, (const int32_t*)(st->dev + off_chain),
                         n_blocks, b->n_q_heads, b->n_kv_heads, b->dim_qk, b->dim_v, b->scale, stream));
  if ((rc = kernel_timing_mark(ctx, SPD_PHASE_PREFILL, 1, stream)) != SPD_OK) return rc;
  // the staging buffer is free again once the kernels above have run; its event goes behind the
  // attention kernel so that nothing sits between the page write and the attention launch
  if ((rc = stage_commit(ctx, SPD_PHASE_PREFILL, st, bytes, stream, false)) != SPD_OK) return rc;
  if (ctx->kernel_timing) {
    SPD_HIP(hipEventRecord(ps.ev_end, stream));
    ps.timed = true;
  }
  return SPD_OK;
}

// ------------------------------------------------------------------------------------------ decode
// Split-K chunk length in units (16-token tiles for GQA, 16-token steps for MLA).
static int decode_chunk_units(spd_phase_state& ps, const int32_t* ctx_lens, int B, int unit_t, int64_t sum_units, int Hkv,
                              int cus, bool mla, int override_tiles) {
  const int64_t round = mla ? 1 : 8;              // GQA: 4 waves x 2 tiles per step
  if (override_tiles > 0) return (int)((override_tiles + round - 1) / round * round);   // tuning override
  if (mla) {
    // Two workgroups are resident per CU (slots); items are issued longest first and a slot takes
    // the next item when it is done, so a chunk length is judged by replaying exactly that: the
    // candidate with the shortest finish time wins.  An item costs its steps plus a pipeline
    // fill.  The choice is kept while the batch stays about the same.
    if (ps.ck_chunk > 0 && ps.ck_B == B && ps.ck_cus == cus && llabs(sum_units - ps.ck_sum) * 32 <= ps.ck_sum)
      return ps.ck_chunk;
    const int slots = std::max(1, 2 * cus);
    const int64_t fill = 6;
    const int64_t c_min = std::max<int64_t>(8, (sum_units + slots - 1) / slots);
    int64_t best_c = c_min, best_t = INT64_MAX;
    std::vector<int32_t> sizes;
    std::vector<int64_t> heap;
    for (int k = 0; k < 16; ++k) {
      const int64_t c = c_min + c_min * k / 6;    // c_min .. 3.5 c_min
      sizes.clear();
      for (int r = 0; r < B; ++r) {
        int32_t u = (ctx_lens[r] + unit_t - 1) / unit_t;
        for (; u > 0; u -= (int32_t)c) sizes.push_back((int32_t)std::min<int64_t>(u, c));
      }
      std::sort(sizes.begin(), sizes.end(), std::greater<int32_t>());
      heap.assign((size_t)slots, 0);              // min-heap of slot finish times
      auto cmp = std::greater<int64_t>();
      int64_t finish = 0;
      for (int32_t sz : sizes) {
        std::pop_heap(heap.begin(), heap.end(), cmp);
        heap.back() += sz + fill;
        finish = std::max(finish, heap.back());
        std::push_heap(heap.begin(), heap.end(), cmp);
      }
      if (finish < best_t) { best_t = finish; best_c = c; }
    }
    ps.ck_B = B; ps.ck_cus = cus; ps.ck_sum = sum_units; ps.ck_chunk = (int)std::min<int64_t>(best_c, 1 << 20);
    return ps.ck_chunk;
  }
  // GQA: aim at ~6 workgroups per CU of the decode share: enough to balance unequal contexts
  // (items are issued longest first), few enough to keep the split-K partials small
  int64_t target_wgs = (int64_t)cus * 6;
  int64_t per_head_chunks = std::max<int64_t>(1, target_wgs / std::max(1, Hkv));
  int64_t c = (sum_units + per_head_chunks - 1) / per_head_chunks;
  c = (c + round - 1) / round * round;
  return (int)std::min<int64_t>(std::max<int64_t>(c, 16), 1 << 20);
}

// noalloc: the variant that allocates nothing.  Metadata twins and workspace lie in the static scratch
// array, the staging ring is used as spd_ctx_create made it, no timing events are recorded.
static int decode_step_impl(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* b, bool noalloc) {
  if (!ctx || !pool || pool->ctx != ctx || !b || b->n_req <= 0 || !b->req_ids || !b->ctx_lens) return SPD_EINVAL;
  if (!b->q || !b->out || b->n_q_heads <= 0) return SPD_EINVAL;
  const PoolGeom& g = pool->geom;
  if (b->n_q_heads % g.Hkv != 0 || b->n_q_heads / g.Hkv > 16) return SPD_EINVAL;
  if (!(b->scale > 0.f) || !std::isfinite(b->scale)) return SPD_EINVAL;
  const bool append = b->k_new != nullptr;
  if (append && (g.kind == SPD_KV_GQA) != (b->v_new != nullptr)) return SPD_EINVAL;
  if (!append && b->v_new) return SPD_EINVAL;
  if (misaligned16(b->q, b->out, b->k_new, b->v_new)) return SPD_EINVAL;
  for (int r = 0; r < b->n_req; ++r) {
    if (b->ctx_lens[r] <= 0) return SPD_EINVAL;                            // empty context
    if (append)
      for (int r2 = 0; r2 < r; ++r2)
        if (b->req_ids[r2] == b->req_ids[r]) return SPD_EINVAL;
  }
  if (b->rope) {
    if (g.kind == SPD_KV_MLA_LATENT_FP8) return SPD_EINVAL;
    int rrc = rope_config_check(b->rope);
    if (rrc != SPD_OK) return rrc;
    if (b->rope->rotary_dim % 16 || b->rope->rotary_dim > 256 || b->rope->rotary_offset % 8 ||
        b->rope->rotary_offset + b->rope->rotary_dim > g.dk)
      return SPD_EINVAL;
  }
  if (ctx->device < 0) return SPD_ESTATE;

  const int B = b->n_req;
  const bool fp8 = g.kind == SPD_KV_MLA_LATENT_FP8;
  const bool mla = g.kind == SPD_KV_MLA_LATENT || fp8;
  const int unit_t = mla ? decode_mla_step_tokens() : TILE_T;     // tokens per split-K unit
  int64_t sum_tiles = 0;
  int32_t max_tiles = 0, max_pages = 0;
  for (int r = 0; r < B; ++r) {
    int32_t tiles = (b->ctx_lens[r] + unit_t - 1) / unit_t;
    sum_tiles += tiles;
    max_tiles = std::max(max_tiles, tiles);
    max_pages = std::max(max_pages, (b->ctx_lens[r] + g.P - 1) / g.P);
  }
  const int bt_stride = max_pages;

  // the share this step will run on: a staged partition is adopted further down, once nothing but a HIP call can
  // fail any more, so a step that returns an error of its own leaves the partition as it was
  int rc;
  spd_phase_state& ds = ctx->phase[SPD_PHASE_DECODE];
  int share;
  {
    std::lock_guard<std::mutex> lk(ctx->part_mu);
    share = ds.has_pending ? ds.pending_cus : ds.active_cus;
  }
  int chunk_tiles = decode_chunk_units(ds, b->ctx_lens, B, unit_t, sum_tiles, g.Hkv, share, mla,
                                       ctx->env_decode_chunk_tiles);
  // the MLA kernel keeps the page ids of a chunk in the 64 lanes of one register: at most 63 pages per chunk
  // (a chunk that starts inside a page touches one more than it holds)
  if (mla) chunk_tiles = std::min(chunk_tiles, 62 * (g.P / unit_t));
  const int max_chunks = (max_tiles + chunk_tiles - 1) / chunk_tiles;

  // work items (request, chunk), longest first: only chunks that exist are launched
  struct Item { int32_t req, chunk, units; };
  std::vector<Item> items;
  for (int r = 0; r < B; ++r) {
    const int32_t units = (b->ctx_lens[r] + unit_t - 1) / unit_t;
    for (int32_t ck = 0; ck * chunk_tiles < units; ++ck)
      items.push_back(Item{r, ck, std::min<int32_t>(chunk_tiles, units - ck * chunk_tiles)});
  }
  std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& c) { return a.units > c.units; });
  const int n_items = (int)items.size();

  size_t off_bt = align16(sizeof(int32_t) * (size_t)B);
  size_t off_items = align16(off_bt + sizeof(int32_t) * (size_t)B * bt_stride);
  size_t off_desc = align16(off_items + sizeof(int32_t) * 2 * (size_t)n_items);
  size_t off_w = align16(off_desc + (append ? sizeof(TileDesc) * (size_t)B : 0));
  size_t bytes = off_w + (b->rope ? sizeof(double) * (size_t)(b->rope->rotary_dim / 2) : 0);
  spd_stage* st;
  if (noalloc && bytes > NOALLOC_STAGE_BYTES) return SPD_ETOOBIG;
  if ((rc = stage_acquire(ctx, SPD_PHASE_DECODE, bytes, &st, !noalloc)) != SPD_OK) return rc;
  char* const sdev = noalloc ? st->dev_static : st->dev;          // device twin of the step's metadata
  const bool timing = ctx->kernel_timing && !noalloc;
  char* ws = nullptr;
  size_t ws_o_bytes = max_chunks > 1 ? align16(sizeof(float) * (size_t)B * b->n_q_heads * max_chunks * g.dv) : 0;
  size_t ws_ml_bytes = max_chunks > 1 ? align16(sizeof(float) * (size_t)B * b->n_q_heads * max_chunks * 2) : 0;
  size_t ws_q_bytes = b->rope ? (size_t)B * b->n_q_heads * g.dk * 2 : 0;      // the rotated query
  if (noalloc) {
    if (ws_o_bytes + ws_ml_bytes + ws_q_bytes > NOALLOC_WS_BYTES) return SPD_ETOOBIG;
    ws = ctx->scratch + 4 * NOALLOC_STAGE_BYTES;
  } else if (ws_o_bytes + ws_ml_bytes + ws_q_bytes > 0 &&
             (rc = workspace_reserve(ctx, SPD_PHASE_DECODE, ws_o_bytes + ws_ml_bytes + ws_q_bytes, &ws)) != SPD_OK) {
    return rc;
  }
  char* ws_q = b->rope ? ws + ws_o_bytes + ws_ml_bytes : nullptr;
  if (b->rope) rope_frequencies(b->rope, (double*)(st->host + off_w));

  int32_t* h_ctx = (int32_t*)st->host;
  int32_t* h_bt = (int32_t*)(st->host + off_bt);
  int32_t* h_items = (int32_t*)(st->host + off_items);
  for (int i = 0; i < n_items; ++i) {
    h_items[2 * i] = items[(size_t)i].req;
    h_items[2 * i + 1] = items[(size_t)i].chunk;
  }
  TileDesc* h_desc = (TileDesc*)(st->host + off_desc);
  {
    std::lock_guard<std::mutex> lk(pool->mu);                       // atomic: query, get, update
    if (append) {
      int64_t need = 0;
      for (int r = 0; r < B; ++r) need += blocks_missing_locked(pool, b->req_ids[r], b->ctx_lens[r]);
      if (need > (int64_t)pool->free_stack.size()) return SPD_ENOMEM;
    } else {
      for (int r = 0; r < B; ++r) {
        auto it = pool->tables.find(b->req_ids[r]);
        if (it == pool->tables.end()) return SPD_ENOENT;
        if ((int64_t)it->second.size() * g.P < b->ctx_lens[r]) return SPD_EINVAL;
      }
    }
    for (int r = 0; r < B; ++r) {
      if (append) reserve_locked(pool, b->req_ids[r], b->ctx_lens[r]);
      spd_req_table& t = pool->tables[b->req_ids[r]];
      t.last_use[SPD_PHASE_DECODE] = next_step_number(ctx, SPD_PHASE_DECODE);
      int32_t pages = (b->ctx_lens[r] + g.P - 1) / g.P;
      h_ctx[r] = b->ctx_lens[r];
      memcpy(h_bt + (size_t)r * bt_stride, t.data(), sizeof(int32_t) * pages);
      for (int32_t p = pages; p < bt_stride; ++p) h_bt[(size_t)r * bt_stride + p] = t[0];
      if (append) {
        std::vector<TileDesc> one;
        build_tile_descs(g, t.data(), b->ctx_lens[r] - 1, 1, r, one);
        h_desc[r] = one[0];
      }
    }
  }
  hipStream_t stream;
  if ((rc = phase_enter(ctx, SPD_PHASE_DECODE, &stream)) != SPD_OK) return rc;
  if (timing) SPD_HIP(hipEventRecord(ds.ev_start, stream));
  if ((rc = stage_copy(st, bytes, stream, sdev)) != SPD_OK) return rc;
  const void* att_q = b->q;
  if (b->rope) {
    SPD_HIP(launch_rope_append(g, pool->base, (const TileDesc*)(sdev + off_desc), (const int32_t*)sdev, B, b->q, ws_q,
                               b->n_q_heads, g.dk, append ? b->k_new : nullptr, append ? b->v_new : nullptr,
                               b->rope->rotary_dim, b->rope->rotary_offset, b->rope->interleaved != 0,
                               (const double*)(sdev + off_w), stream));
    att_q = ws_q;
  } else if (append && fp8) {
    SPD_HIP(launch_kv_write_fp8(g, pool->base, (const TileDesc*)(sdev + off_desc), B, b->k_new, stream));
  } else if (append) {
    SPD_HIP(launch_kv_write(g, pool->base, (const TileDesc*)(sdev + off_desc), B, b->k_new, b->v_new, stream));
  }
  if (timing && (rc = kernel_timing_mark(ctx, SPD_PHASE_DECODE, 0, stream)) != SPD_OK) return rc;
  if (mla)
    SPD_HIP(launch_decode_mla(g, pool->base, att_q, b->out, (const int32_t*)sdev, (const int32_t*)(sdev + off_bt),
                              bt_stride, sdev + off_items, n_items, B, b->n_q_heads, b->scale, chunk_tiles, max_chunks,
                              (float*)(max_chunks > 1 ? ws : nullptr), (float*)(max_chunks > 1 ? ws + ws_o_bytes : nullptr), stream,
                              fp8));
  else
    SPD_HIP(launch_decode_gqa(g, pool->base, att_q, b->out, (const int32_t*)sdev, (const int32_t*)(sdev + off_bt),
                              bt_stride, sdev + off_items, n_items, B, b->n_q_heads, b->scale, chunk_tiles, max_chunks,
                              (float*)(max_chunks > 1 ? ws : nullptr), (float*)(max_chunks > 1 ? ws + ws_o_bytes : nullptr), stream));
  if (timing && (rc = kernel_timing_mark(ctx, SPD_PHASE_DECODE, 1, stream)) != SPD_OK) return rc;
  // the slot's event goes behind the attention kernels: it frees the staging slot and tells spd_kv_free that
  // the step no longer reads its requests' pages
  if ((rc = stage_commit(ctx, SPD_PHASE_DECODE, st, bytes, stream, false)) != SPD_OK) return rc;
  if (timing) {
    SPD_HIP(hipEventRecord(ds.ev_end, stream));
    ds.timed = true;
  }
  return SPD_OK;
}

extern "C" int spd_decode_step(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* b) {
  return decode_step_impl(ctx, pool, b, false);
}

extern "C" int spd_decode_step_noalloc(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* b) {
  return decode_step_impl(ctx, pool, b, true);
}

extern "C" int spd_noalloc_limits(uint64_t* metadata_bytes, uint64_t* workspace_bytes) {
  if (metadata_bytes) *metadata_bytes = NOALLOC_STAGE_BYTES;
  if (workspace_bytes) *workspace_bytes = NOALLOC_WS_BYTES;
  return SPD_OK;
}


// ------------------------------------------------------------------------------------------ decode worker
struct spd_worker {
  std::thread th;
  std::atomic<bool> stop{false};
  std::atomic<int64_t> issued{0};
  std::atomic<int> status{SPD_OK};
};

extern "C" int spd_decode_worker_start(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* const* batches,
                                       int32_t n_batches, spd_worker** out) {
  if (!ctx || !pool || pool->ctx != ctx || !batches || n_batches <= 0 || !out) return SPD_EINVAL;
  for (int i = 0; i < n_batches; ++i)
    if (!batches[i]) return SPD_EINVAL;
  if (ctx->device < 0) return SPD_ESTATE;
  spd_worker* w = new (std::nothrow) spd_worker();
  if (!w) return SPD_EINVAL;
  std::vector<const spd_decode_batch*> list(batches, batches + n_batches);
  w->th = std::thread([w, ctx, pool, list]() {
    if (hipSetDevice(ctx->device) != hipSuccess) {
      w->status.store(SPD_EHIP);
      return;
    }
    size_t i = 0;
    do {                                          // at least one step, however early the stop comes
      const int rc = spd_decode_step(ctx, pool, list[i]);
      if (rc != SPD_OK) {
        w->status.store(rc);
        return;
      }
      w->issued.fetch_add(1, std::memory_order_relaxed);
      i = (i + 1) % list.size();
    } while (!w->stop.load(std::memory_order_relaxed));
  });
  *out = w;
  return SPD_OK;
}

extern "C" int spd_decode_worker_steps(spd_worker* w, int64_t* steps_issued) {
  if (!w || !steps_issued) return SPD_EINVAL;
  *steps_issued = w->issued.load(std::memory_order_relaxed);
  return SPD_OK;
}

extern "C" int spd_decode_worker_stop(spd_worker* w, int64_t* steps_issued, int* status) {
  if (!w) return SPD_EINVAL;
  w->stop.store(true);
  if (w->th.joinable()) w->th.join();
  if (steps_issued) *steps_issued = w->issued.load();
  if (status) *status = w->status.load();
  delete w;
  return SPD_OK;
}
