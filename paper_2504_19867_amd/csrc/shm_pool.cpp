// The block allocator of the unified KV pool in POSIX shared memory, for workers that are processes.
//
// Paper, "Unified Memory Manager": the prefill and the decode worker are two processes that allocate from one
// KV cache; query / get / update of the memory utilisation are one atomic operation under a lock, so the two
// asynchronous workers cannot both take the last blocks.  Here the whole allocator state - free stack, block
// tables, utilisation, operation counter - lies in one shared-memory segment that every worker process maps, under
// a process-shared mutex in the segment itself.  Policy and results are those of the in-process allocator
// (pool.cpp): the free list is a stack whose first pops are 0, 1, 2, ...; reserve grows a request's table one block
// at a time, all or nothing; free pushes the blocks back last to first; every successful mutating call gets the
// next operation number.
//
// Layout of the segment (all offsets from its start; no pointers are stored, each process maps it where it likes):
//   Header | free_stack[num_pages] | next[num_pages] | prev[num_pages] | slots[n_slots]
// A request's block table is a doubly linked list through next[] / prev[] (page -> the request's next / previous
// page), so tables of any length share the one array; slots[] is an open-addressing hash table req_id -> (first
// page, last page, number of pages) with linear probing and tombstones.
#include <errno.h>
#include <fcntl.h>
#include <pthread.h>
#include <stdint.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#include <new>
#include <string>
#include <vector>

#include "semipd.h"

namespace {

constexpr uint64_t MAGIC = 0x53454d4950443031ull;   // "SEMIPD01"
enum : int32_t { SLOT_EMPTY = 0, SLOT_LIVE = 1, SLOT_DEAD = 2 };

struct Slot {
  uint64_t req;
  int32_t state, first, last, count;
};

struct Header {
  uint64_t magic;
  uint64_t bytes;
  int64_t num_pages;
  int32_t page_tokens;
  int32_t n_slots;              // power of two
  int32_t max_requests;
  int32_t damaged;              // a process died inside a mutation: the state can no longer be trusted
  int64_t n_free, used, live, tombstones;
  uint64_t op_seq;
  pthread_mutex_t mu;
};

size_t align64(size_t x) { return (x + 63) & ~(size_t)63; }
size_t off_free(const Header*) { return align64(sizeof(Header)); }
size_t off_next(const Header* h) { return align64(off_free(h) + sizeof(int32_t) * (size_t)h->num_pages); }
size_t off_prev(const Header* h) { return align64(off_next(h) + sizeof(int32_t) * (size_t)h->num_pages); }
size_t off_slots(const Header* h) { return align64(off_prev(h) + sizeof(int32_t) * (size_t)h->num_pages); }
size_t total_bytes(const Header* h) { return off_slots(h) + sizeof(Slot) * (size_t)h->n_slots; }

}  // namespace

struct spd_shm_pool {
  Header* h = nullptr;
  int32_t *free_stack = nullptr, *next = nullptr, *prev = nullptr;
  Slot* slots = nullptr;
  size_t bytes = 0;
  std::string name;
};

namespace {

void bind(spd_shm_pool* p) {
  char* b = (char*)p->h;
  p->free_stack = (int32_t*)(b + off_free(p->h));
  p->next = (int32_t*)(b + off_next(p->h));
  p->prev = (int32_t*)(b + off_prev(p->h));
  p->slots = (Slot*)(b + off_slots(p->h));
}

uint64_t mix(uint64_t x) {                       // splitmix64 finaliser
  x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27; x *= 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

// the request's slot, or the slot to create it in (null if the table is full)
Slot* find(spd_shm_pool* p, uint64_t req, bool create) {
  const uint32_t mask = (uint32_t)p->h->n_slots - 1;
  Slot* grave = nullptr;
  for (uint32_t i = (uint32_t)mix(req) & mask, n = 0; n <= mask; i = (i + 1) & mask, ++n) {
    Slot& s = p->slots[i];
    if (s.state == SLOT_LIVE && s.req == req) return &s;
    if (s.state == SLOT_DEAD && !grave) grave = &s;
    if (s.state == SLOT_EMPTY) return create ? (grave ? grave : &s) : nullptr;
  }
  return create ? grave : nullptr;
}

// Too many tombstones lengthen every probe: rebuild the table in place (under the lock).
void rehash(spd_shm_pool* p) {
  const int32_t n = p->h->n_slots;
  std::vector<Slot> live;                         // in this process's own memory, for the duration of the rebuild
  live.reserve((size_t)p->h->live);
  for (int32_t i = 0; i < n; ++i) {
    if (p->slots[i].state == SLOT_LIVE) live.push_back(p->slots[i]);
    p->slots[i].state = SLOT_EMPTY;
  }
  p->h->tombstones = 0;
  for (const Slot& s : live) *find(p, s.req, true) = s;
}

struct Lock {
  Header* h;
  int rc;
  explicit Lock(Header* hh) : h(hh) {
    int e = pthread_mutex_lock(&h->mu);
    if (e == EOWNERDEAD) {                        // a worker died holding the lock
      h->damaged = 1;
      pthread_mutex_consistent(&h->mu);
      e = 0;
    }
    rc = e == 0 ? (h->damaged ? SPD_ESTATE : SPD_OK) : SPD_ESTATE;
    if (e == 0 && rc != SPD_OK) { pthread_mutex_unlock(&h->mu); locked = false; } else locked = e == 0;
  }
  ~Lock() { if (locked) pthread_mutex_unlock(&h->mu); }
  bool locked = false;
};

}  // namespace

extern "C" int spd_shm_pool_create(const char* name, int64_t num_pages, int32_t page_tokens, int32_t max_requests,
                                   spd_shm_pool** out) {
  if (!name || name[0] != '/' || !out || num_pages <= 0 || num_pages > INT32_MAX || page_tokens <= 0 || max_requests <= 0)
    return SPD_EINVAL;
  Header tmp{};
  tmp.num_pages = num_pages;
  int32_t n_slots = 16;
  while (n_slots < 2 * (int64_t)max_requests && n_slots < (1 << 30)) n_slots <<= 1;
  tmp.n_slots = n_slots;
  const size_t bytes = total_bytes(&tmp);
  int fd = shm_open(name, O_CREAT | O_EXCL | O_RDWR, 0600);
  if (fd < 0) return errno == EEXIST ? SPD_ESTATE : SPD_EINVAL;
  if (ftruncate(fd, (off_t)bytes) != 0) { close(fd); shm_unlink(name); return SPD_ENOMEM; }
  void* m = mmap(nullptr, bytes, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (m == MAP_FAILED) { shm_unlink(name); return SPD_ENOMEM; }
  Header* h = (Header*)m;                        // fresh shared memory is zero: all slots empty
  h->bytes = bytes;
  h->num_pages = num_pages;
  h->page_tokens = page_tokens;
  h->n_slots = n_slots;
  h->max_requests = max_requests;
  h->n_free = num_pages;
  pthread_mutexattr_t a;
  pthread_mutexattr_init(&a);
  pthread_mutexattr_setpshared(&a, PTHREAD_PROCESS_SHARED);
  pthread_mutexattr_setrobust(&a, PTHREAD_MUTEX_ROBUST);
  const int e = pthread_mutex_init(&h->mu, &a);
  pthread_mutexattr_destroy(&a);
  if (e != 0) { munmap(m, bytes); shm_unlink(name); return SPD_ESTATE; }
  spd_shm_pool* p = new (std::nothrow) spd_shm_pool();
  if (!p) { munmap(m, bytes); shm_unlink(name); return SPD_EINVAL; }
  p->h = h; p->bytes = bytes; p->name = name;
  bind(p);
  for (int64_t i = 0; i < num_pages; ++i) p->free_stack[i] = (int32_t)(num_pages - 1 - i);   // top = back(): pops 0, 1, 2, ...
  __atomic_store_n(&h->magic, MAGIC, __ATOMIC_RELEASE);   // last: an opener that sees it sees a complete segment
  *out = p;
  return SPD_OK;
}

extern "C" int spd_shm_pool_open(const char* name, spd_shm_pool** out) {
  if (!name || name[0] != '/' || !out) return SPD_EINVAL;
  int fd = shm_open(name, O_RDWR, 0600);
  if (fd < 0) return SPD_ENOENT;
  struct stat st;
  if (fstat(fd, &st) != 0 || (size_t)st.st_size < sizeof(Header)) { close(fd); return SPD_ESTATE; }
  void* m = mmap(nullptr, (size_t)st.st_size, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
  close(fd);
  if (m == MAP_FAILED) return SPD_ENOMEM;
  Header* h = (Header*)m;
  if (__atomic_load_n(&h->magic, __ATOMIC_ACQUIRE) != MAGIC || h->bytes != (uint64_t)st.st_size || total_bytes(h) != h->bytes) {
    munmap(m, (size_t)st.st_size);
    return SPD_ESTATE;                            // not (yet) a pool segment
  }
  spd_shm_pool* p = new (std::nothrow) spd_shm_pool();
  if (!p) { munmap(m, (size_t)st.st_size); return SPD_EINVAL; }
  p->h = h; p->bytes = (size_t)st.st_size; p->name = name;
  bind(p);
  *out = p;
  return SPD_OK;
}

extern "C" int spd_shm_pool_close(spd_shm_pool* p) {
  if (!p) return SPD_EINVAL;
  munmap((void*)p->h, p->bytes);
  delete p;
  return SPD_OK;
}

extern "C" int spd_shm_pool_unlink(const char* name) {
  if (!name || name[0] != '/') return SPD_EINVAL;
  return shm_unlink(name) == 0 ? SPD_OK : SPD_ENOENT;
}

extern "C" int spd_shm_pool_stats(spd_shm_pool* p, int64_t* total, int64_t* free_pages, int64_t* live_reqs, uint64_t* op_seq) {
  if (!p) return SPD_EINVAL;
  Lock lk(p->h);
  if (lk.rc != SPD_OK) return lk.rc;
  if (total) *total = p->h->num_pages;
  if (free_pages) *free_pages = p->h->n_free;
  if (live_reqs) *live_reqs = p->h->live;
  if (op_seq) *op_seq = p->h->op_seq;
  return SPD_OK;
}

extern "C" int spd_shm_kv_reserve(spd_shm_pool* p, uint64_t req_id, int32_t n_tokens_total, uint64_t* op_seq_out) {
  if (!p || n_tokens_total <= 0) return SPD_EINVAL;
  Lock lk(p->h);
  if (lk.rc != SPD_OK) return lk.rc;
  Header* h = p->h;
  Slot* s = find(p, req_id, false);
  const int64_t want = ((int64_t)n_tokens_total + h->page_tokens - 1) / h->page_tokens;
  const int64_t have = s ? s->count : 0;
  const int64_t need = want > have ? want - have : 0;
  if (need > h->n_free) return SPD_ENOMEM;                          // query
  if (!s) {
    if (h->live >= h->max_requests) return SPD_ENOMEM;              // the request table is as much a resource as the pages
    if (h->tombstones > h->n_slots / 4) rehash(p);
    s = find(p, req_id, true);
    if (!s) return SPD_ENOMEM;
    if (s->state == SLOT_DEAD) --h->tombstones;
    *s = Slot{req_id, SLOT_LIVE, -1, -1, 0};
    ++h->live;
  }
  for (int64_t i = 0; i < need; ++i) {                               // get
    const int32_t page = p->free_stack[--h->n_free];
    p->next[page] = -1;
    p->prev[page] = s->last;
    if (s->last >= 0) p->next[s->last] = page; else s->first = page;
    s->last = page;
    ++s->count;
  }
  h->used += need;                                                   // update
  const uint64_t seq = ++h->op_seq;
  if (op_seq_out) *op_seq_out = seq;
  return SPD_OK;
}

extern "C" int spd_shm_kv_free(spd_shm_pool* p, uint64_t req_id, uint64_t* op_seq_out) {
  if (!p) return SPD_EINVAL;
  Lock lk(p->h);
  if (lk.rc != SPD_OK) return lk.rc;
  Header* h = p->h;
  Slot* s = find(p, req_id, false);
  if (!s) return SPD_ENOENT;
  for (int32_t page = s->last; page >= 0; page = p->prev[page]) p->free_stack[h->n_free++] = page;   // last to first
  h->used -= s->count;
  s->state = SLOT_DEAD;
  ++h->tombstones;
  --h->live;
  const uint64_t seq = ++h->op_seq;
  if (op_seq_out) *op_seq_out = seq;
  return SPD_OK;
}

extern "C" int spd_shm_kv_block_table(spd_shm_pool* p, uint64_t req_id, int32_t* out, int32_t cap, int32_t* n_out) {
  if (!p || !n_out || cap < 0 || (cap > 0 && !out)) return SPD_EINVAL;
  Lock lk(p->h);
  if (lk.rc != SPD_OK) return lk.rc;
  Slot* s = find(p, req_id, false);
  if (!s) return SPD_ENOENT;
  *n_out = s->count;
  if (cap < s->count) return SPD_EINVAL;
  int32_t i = 0;
  for (int32_t page = s->first; page >= 0; page = p->next[page]) out[i++] = page;
  return SPD_OK;
}

extern "C" int spd_shm_kv_free_list(spd_shm_pool* p, int32_t* out, int64_t cap, int64_t* n_out) {
  if (!p || !n_out || cap < 0 || (cap > 0 && !out)) return SPD_EINVAL;
  Lock lk(p->h);
  if (lk.rc != SPD_OK) return lk.rc;
  *n_out = p->h->n_free;
  if (cap < p->h->n_free) return SPD_EINVAL;
  if (p->h->n_free) memcpy(out, p->free_stack, sizeof(int32_t) * (size_t)p->h->n_free);
  return SPD_OK;
}
