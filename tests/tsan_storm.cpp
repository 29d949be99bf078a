// Two-thread storm over the host logic of the library, for a ThreadSanitizer build on the CPU
// (tests/test_tsan_host.py compiles pool.cpp, ctx.cpp and controller.cpp with -fsanitize=thread and runs this).
// A "prefill worker" and a "decode worker" thread reserve and free on one pool at once, as the two asynchronous
// workers do, and both feed one SLO adjuster; afterwards the logged operations are replayed in the order of their
// operation numbers on a second pool by one thread, and the two pools must agree block for block.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "semipd.h"

// the kernel launchers that ctx.cpp refers to: a host-only context never reaches them
namespace spd {
hipError_t launch_probe(int32_t*, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_copy(void*, const void*, uint64_t, int, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_read(const void*, uint64_t, int, uint32_t*, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_read_lds(const void*, uint64_t, int, uint32_t*, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_clock_probe(uint64_t, uint64_t*, hipStream_t) { return hipErrorUnknown; }
hipError_t launch_issue_probe(uint64_t*, hipStream_t) { return hipErrorUnknown; }
int scratch_resolve(int, char**) { return SPD_ESTATE; }
}  // namespace spd

struct Op { uint64_t seq; int kind; uint64_t req; int32_t n; };   // kind 0 reserve, 1 free

#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); exit(1); } } while (0)

static void worker(spd_pool* pool, spd_ctrl* ctrl, int who, std::vector<Op>* log) {
  uint32_t s = 12345u + 977u * (uint32_t)who;
  auto rnd = [&]() { s = s * 1664525u + 1013904223u; return s >> 8; };
  std::vector<std::pair<uint64_t, int32_t>> live;                // (request, tokens)
  uint64_t next_id = (uint64_t)(who + 1) << 32;
  for (int i = 0; i < 20000; ++i) {
    const uint32_t r = rnd() % 100;
    uint64_t seq = 0;
    if (live.empty() || r < 35) {                                // a new request
      const int32_t n = 1 + (int32_t)(rnd() % (who == 0 ? 600 : 60));
      const int rc = spd_kv_reserve(pool, next_id, n, &seq);
      CHECK(rc == SPD_OK || rc == SPD_ENOMEM);
      if (rc == SPD_OK) { log->push_back(Op{seq, 0, next_id, n}); live.emplace_back(next_id, n); }
      ++next_id;
    } else if (r < 75) {                                         // a live request grows (decode appends)
      auto& e = live[rnd() % live.size()];
      const int32_t n = e.second + 1 + (int32_t)(rnd() % 20);
      const int rc = spd_kv_reserve(pool, e.first, n, &seq);
      CHECK(rc == SPD_OK || rc == SPD_ENOMEM);
      if (rc == SPD_OK) { log->push_back(Op{seq, 0, e.first, n}); e.second = n; }
    } else {                                                     // a request finishes
      const size_t j = rnd() % live.size();
      CHECK(spd_kv_free(pool, live[j].first, &seq) == SPD_OK);
      log->push_back(Op{seq, 1, live[j].first, 0});
      live[j] = live.back();
      live.pop_back();
    }
    if (who == 0) CHECK(spd_ctrl_observe_ttft(ctrl, 0.05 + (rnd() % 100) * 1e-3) == SPD_OK);
    else CHECK(spd_ctrl_observe_tpot(ctrl, 0.01 + (rnd() % 100) * 1e-4) == SPD_OK);
    if (who == 1 && i % 64 == 0) {
      int32_t x, y;
      CHECK(spd_ctrl_step(ctrl, i, 50, 50, &x, &y) == SPD_OK);
    }
    if (i % 97 == 0) {                                           // readers beside the writers
      int64_t total, free_pages, live_reqs;
      uint64_t ops;
      CHECK(spd_pool_stats(pool, &total, &free_pages, &live_reqs, &ops) == SPD_OK);
      CHECK(free_pages >= 0 && free_pages <= total);
    }
  }
}

int main() {
  spd_ctx* ctx = nullptr;
  CHECK(spd_ctx_create(-1, &ctx) == SPD_OK);
  spd_pool_desc d{SPD_KV_GQA, 16, 2, 64, 64, 4096};
  spd_pool *pool = nullptr, *replay = nullptr;
  CHECK(spd_pool_create(ctx, nullptr, 0, &d, &pool) == SPD_OK);
  CHECK(spd_pool_create(ctx, nullptr, 0, &d, &replay) == SPD_OK);
  spd_ctrl_config cc{0.2, 0.02, 90.0, 64, 4, 10, 16};
  spd_ctrl* ctrl = nullptr;
  CHECK(spd_ctrl_create(&cc, &ctrl) == SPD_OK);
  // a partition staged from a third thread meanwhile (the adjuster's caller)
  std::vector<Op> logs[2];
  std::thread a(worker, pool, ctrl, 0, &logs[0]), b(worker, pool, ctrl, 1, &logs[1]);
  for (int i = 0; i < 200; ++i) {
    CHECK(spd_set_partition(ctx, 32 + 32 * (i % 6), 224 - 32 * (i % 6)) == SPD_OK);
    int pa, da, pp, dp;
    CHECK(spd_get_partition(ctx, &pa, &da, &pp, &dp) == SPD_OK);
  }
  a.join();
  b.join();
  std::vector<Op> all(logs[0]);
  all.insert(all.end(), logs[1].begin(), logs[1].end());
  std::sort(all.begin(), all.end(), [](const Op& x, const Op& y) { return x.seq < y.seq; });
  for (size_t i = 0; i < all.size(); ++i) CHECK(all[i].seq == i + 1);       // every operation number handed out once
  for (const Op& o : all) {
    uint64_t seq = 0;
    CHECK((o.kind == 0 ? spd_kv_reserve(replay, o.req, o.n, &seq) : spd_kv_free(replay, o.req, &seq)) == SPD_OK);
    CHECK(seq == o.seq);
  }
  std::vector<int32_t> f1(4096), f2(4096);
  int64_t n1 = 0, n2 = 0;
  CHECK(spd_kv_free_list(pool, f1.data(), 4096, &n1) == SPD_OK && spd_kv_free_list(replay, f2.data(), 4096, &n2) == SPD_OK);
  CHECK(n1 == n2 && std::equal(f1.begin(), f1.begin() + n1, f2.begin()));
  printf("storm ok: %zu operations, %lld pages free at the end\n", all.size(), (long long)n1);
  spd_ctrl_destroy(ctrl);
  spd_pool_destroy(pool);
  spd_pool_destroy(replay);
  spd_ctx_destroy(ctx);
  return 0;
}
