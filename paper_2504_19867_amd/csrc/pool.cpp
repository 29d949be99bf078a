// Unified KV pool: geometry, block allocator and block tables (host side, no GPU work).
//
// Paper, "Unified Memory Manager": both workers allocate from one paged pool; the
// query / get / update of the memory utilisation happens under one lock.  Every
// mutating entry point below holds pool->mu for the whole operation.
#include "internal.h"

#include <string.h>

#include <new>

namespace spd {
thread_local int g_last_hip_error = 0;

static bool desc_ok(const spd_pool_desc* d) {
  if (!d || d->num_pages <= 0 || d->num_pages > INT32_MAX) return false;
  if (d->page_tokens <= 0 || d->page_tokens % TILE_T != 0 || d->page_tokens > 1024) return false;
  if (d->kind == SPD_KV_GQA) {
    if (d->n_kv_heads <= 0 || d->n_kv_heads > 1024) return false;
    if (d->dim_k != d->dim_v) return false;
    return d->dim_k == 64 || d->dim_k == 128;
  }
  if (d->kind == SPD_KV_MLA_LATENT || d->kind == SPD_KV_MLA_LATENT_FP8)
    return d->n_kv_heads == 1 && d->dim_k == 576 && d->dim_v == 512 && d->page_tokens % 32 == 0;
  return false;
}
}  // namespace spd

using namespace spd;

extern "C" int spd_pool_bytes(const spd_pool_desc* desc, uint64_t* bytes_out) {
  if (!desc_ok(desc) || !bytes_out) return SPD_EINVAL;
  *bytes_out = make_geom(*desc).page_bytes * (uint64_t)desc->num_pages;
  return SPD_OK;
}

extern "C" int spd_pool_create(spd_ctx* ctx, void* dev_mem, uint64_t bytes, const spd_pool_desc* desc,
                               spd_pool** out) {
  if (!ctx || !out || !desc_ok(desc)) return SPD_EINVAL;
  PoolGeom g = make_geom(*desc);
  if (ctx->device >= 0) {
    if (!dev_mem || ((uintptr_t)dev_mem & 255) != 0) return SPD_EINVAL;
    if (bytes < g.page_bytes * (uint64_t)desc->num_pages) return SPD_EINVAL;
  }
  spd_pool* p = new (std::nothrow) spd_pool();
  if (!p) return SPD_EINVAL;
  p->ctx = ctx;
  p->desc = *desc;
  p->geom = g;
  p->base = (char*)dev_mem;
  p->bytes = bytes;
  p->free_stack.resize((size_t)desc->num_pages);
  for (int64_t i = 0; i < desc->num_pages; ++i) p->free_stack[(size_t)i] = (int32_t)(desc->num_pages - 1 - i);
  *out = p;
  return SPD_OK;
}

extern "C" int spd_pool_destroy(spd_pool* pool) {
  if (!pool) return SPD_EINVAL;
  delete pool;
  return SPD_OK;
}

extern "C" int spd_pool_stats(spd_pool* pool, int64_t* total, int64_t* free_pages, int64_t* live_reqs,
                              uint64_t* op_seq) {
  if (!pool) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(pool->mu);
  if (total) *total = pool->desc.num_pages;
  if (free_pages) *free_pages = (int64_t)pool->free_stack.size();
  if (live_reqs) *live_reqs = (int64_t)pool->tables.size();
  if (op_seq) *op_seq = pool->op_seq;
  return SPD_OK;
}

namespace spd {
// Caller holds pool->mu.  Blocks still missing for `n_tokens` tokens of request `req`.
int64_t blocks_missing_locked(spd_pool* pool, uint64_t req, int64_t n_tokens) {
  int64_t want = (n_tokens + pool->desc.page_tokens - 1) / pool->desc.page_tokens;
  auto it = pool->tables.find(req);
  int64_t have = it == pool->tables.end() ? 0 : (int64_t)it->second.size();
  return want > have ? want - have : 0;
}

// Caller holds pool->mu and has checked that enough blocks are free.
uint64_t reserve_locked(spd_pool* pool, uint64_t req, int64_t n_tokens) {
  int64_t need = blocks_missing_locked(pool, req, n_tokens);
  std::vector<int32_t>& t = pool->tables[req];
  for (int64_t i = 0; i < need; ++i) {
    t.push_back(pool->free_stack.back());
    pool->free_stack.pop_back();
  }
  pool->used += need;
  return ++pool->op_seq;
}
}  // namespace spd

extern "C" int spd_kv_reserve(spd_pool* pool, uint64_t req_id, int32_t n_tokens_total, uint64_t* op_seq_out) {
  if (!pool || n_tokens_total <= 0) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(pool->mu);
  int64_t need = blocks_missing_locked(pool, req_id, n_tokens_total);          // query
  if (need > (int64_t)pool->free_stack.size()) return SPD_ENOMEM;
  uint64_t seq = reserve_locked(pool, req_id, n_tokens_total);                 // get + update
  if (op_seq_out) *op_seq_out = seq;
  return SPD_OK;
}

extern "C" int spd_kv_free(spd_pool* pool, uint64_t req_id, uint64_t* op_seq_out) {
  if (!pool) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(pool->mu);
  auto it = pool->tables.find(req_id);
  if (it == pool->tables.end()) return SPD_ENOENT;
  spd_req_table& t = it->second;
  // pages go back on the free stack at once, so no step that took this table may still be running
  for (int ph = 0; ph < 2; ++ph)
    if (!spd::phase_step_done(pool->ctx, ph, t.last_use[ph])) return SPD_ESTATE;
  for (size_t i = t.size(); i-- > 0;) pool->free_stack.push_back(t[i]);
  pool->used -= (int64_t)t.size();
  pool->tables.erase(it);
  uint64_t seq = ++pool->op_seq;
  if (op_seq_out) *op_seq_out = seq;
  return SPD_OK;
}

extern "C" int spd_kv_block_table(spd_pool* pool, uint64_t req_id, int32_t* out, int32_t cap, int32_t* n_out) {
  if (!pool || !n_out || cap < 0 || (cap > 0 && !out)) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(pool->mu);
  auto it = pool->tables.find(req_id);
  if (it == pool->tables.end()) return SPD_ENOENT;
  *n_out = (int32_t)it->second.size();
  if ((size_t)cap < it->second.size()) return SPD_EINVAL;
  if (!it->second.empty()) memcpy(out, it->second.data(), it->second.size() * sizeof(int32_t));
  return SPD_OK;
}

extern "C" int spd_kv_free_list(spd_pool* pool, int32_t* out, int64_t cap, int64_t* n_out) {
  if (!pool || !n_out || cap < 0 || (cap > 0 && !out)) return SPD_EINVAL;
  std::lock_guard<std::mutex> lk(pool->mu);
  *n_out = (int64_t)pool->free_stack.size();
  if ((size_t)cap < pool->free_stack.size()) return SPD_EINVAL;
  if (!pool->free_stack.empty()) memcpy(out, pool->free_stack.data(), pool->free_stack.size() * sizeof(int32_t));
  return SPD_OK;
}

extern "C" const char* spd_strerror(int status) {
  switch (status) {
    case SPD_OK: return "ok";
    case SPD_EINVAL: return "invalid argument";
    case SPD_ENOMEM: return "KV pool exhausted";
    case SPD_ENOENT: return "unknown request id";
    case SPD_EHIP: return "HIP call failed";
    case SPD_ESTATE: return "call not valid in this state";
    case SPD_ETOOBIG: return "batch exceeds the fixed scratch memory of the entry point that allocates nothing";
    default: return "unknown status";
  }
}

extern "C" int spd_last_hip_error(void) { return g_last_hip_error; }
