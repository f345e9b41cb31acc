// Host-only driver for the paged activation store, meant to be built with
// -fsanitize=address,undefined: random sequences of every call of daf_store.h on two stores,
// one per index kind.  After every call both stores must pass daf_store_validate and must have
// made the same decision (Sec. 3.4: the red-black trees and the re-sorting index are two ways
// to find the same victim).  Exit status 0 = no difference and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "daf.h"
#include "daf_store.h"

namespace {
uint64_t rng_state = 1;
uint64_t rnd() {                                    // splitmix64
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
int64_t below(int64_t n) { return (int64_t)(rnd() % (uint64_t)n); }
long n_not_stored = 0, n_narrowed = 0, n_moves = 0, n_evicted = 0, n_release_gone = 0;

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "line %d: %s (seed %d, op %d)\n", __LINE__, #cond, seed, op); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

void run(int seed, int n_ops) {
  int op = 0;
  rng_state = (uint64_t)seed * 7919u + 1;
  const int64_t page = 256 << below(3);
  const int64_t budget = page * (8 + below(200));
  const int64_t time_budget = below(3) == 0 ? 0 : 1000 + below(200000);
  daf_store_t* st[2] = {nullptr, nullptr};
  for (int k = 0; k < 2; ++k) CHECK(daf_store_create(page, budget, time_budget, page * (1 + below(4)), k, &st[k]) == DAF_OK || k == 1);
  // (the step differs between the two on purpose only if the first create consumed other random
  // numbers; keep them equal: re-create the second with the first's parameters)
  daf_store_destroy(st[1]);
  daf_store_destroy(st[0]);
  const int64_t step = page * (1 + below(4));
  for (int k = 0; k < 2; ++k) CHECK(daf_store_create(page, budget, time_budget, step, k, &st[k]) == DAF_OK);

  std::vector<int64_t> planned, allocated;
  int64_t next_id = 0;
  const int32_t widths[4] = {8, 4, 2, 1};
  for (op = 0; op < n_ops; ++op) {
    const int what = (int)below(100);
    int rc[2] = {0, 0};
    if (what < 35) {                                // add
      const int64_t id = next_id++;
      const int32_t nw = 1 + (int32_t)below(4);
      int64_t bytes[4], ns[4];
      const int64_t base = 64 + below(20 * page);
      for (int i = 0; i < nw; ++i) {
        bytes[i] = base * widths[i] / 8 + 8;
        ns[i] = 10 + below(5000);
      }
      const double imp = (double)below(1000000) / 1000.0;
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_add(st[k], id, widths, bytes, ns, nw, imp);
      CHECK(rc[0] == rc[1] && rc[0] == DAF_OK);
      planned.push_back(id);
    } else if (what < 65 && !planned.empty()) {     // receive
      const size_t i = (size_t)below((int64_t)planned.size());
      const int64_t id = planned[i];
      planned[i] = planned.back();
      planned.pop_back();
      const double imp = (double)below(1000000) / 1000.0;
      int32_t b[2];
      int64_t o[2], s[2];
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_receive(st[k], id, imp, &b[k], &o[k], &s[k]);
      CHECK(rc[0] == rc[1] && rc[0] == DAF_OK);
      CHECK(b[0] == b[1] && o[0] == o[1] && s[0] == s[1]);
      if (b[0] != 0) allocated.push_back(id);
      if (b[0] == 0) ++n_not_stored;
      if (b[0] != 0 && b[0] != 8) ++n_narrowed;
    } else if (what < 80 && !allocated.empty()) {   // release (it may have been evicted meanwhile)
      const size_t i = (size_t)below((int64_t)allocated.size());
      const int64_t id = allocated[i];
      allocated[i] = allocated.back();
      allocated.pop_back();
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_release(st[k], id);
      CHECK(rc[0] == rc[1]);
      if (rc[0] != DAF_OK) ++n_release_gone;
    } else if (what < 88) {                         // new memory budget
      const int64_t nb = page * (4 + below(220));
      std::vector<daf_store_move_t> mv[2];
      int32_t n[2] = {0, 0};
      for (int k = 0; k < 2; ++k) {
        mv[k].resize(allocated.size() + planned.size() + 4);
        rc[k] = daf_store_set_mem_budget(st[k], nb, mv[k].data(), (int32_t)mv[k].size(), &n[k]);
      }
      CHECK(rc[0] == rc[1] && rc[0] == DAF_OK && n[0] == n[1]);
      n_moves += n[0];
      for (int32_t i = 0; i < n[0]; ++i)
        CHECK(mv[0][i].id == mv[1][i].id && mv[0][i].from_offset_bytes == mv[1][i].from_offset_bytes &&
              mv[0][i].to_offset_bytes == mv[1][i].to_offset_bytes && mv[0][i].size_bytes == mv[1][i].size_bytes);
    } else if (what < 92) {                         // new time budget
      const int64_t nt = below(4) == 0 ? 0 : 500 + below(300000);
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_set_time_budget(st[k], nt);
      CHECK(rc[0] == rc[1] && rc[0] == DAF_OK);
    } else if (what < 97) {                         // evicted ids, a few at a time
      int64_t ids[2][3];
      int32_t n[2];
      for (int k = 0; k < 2; ++k) n[k] = daf_store_pop_evicted(st[k], ids[k], 3);
      CHECK(n[0] == n[1]);
      n_evicted += n[0];
      for (int32_t i = 0; i < n[0]; ++i) CHECK(ids[0][i] == ids[1][i]);
    } else if (what < 98) {                         // new iteration
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_reset(st[k]);
      CHECK(rc[0] == rc[1] && rc[0] == DAF_OK);
      planned.clear();
      allocated.clear();
    } else {                                        // queries, also of ids that do not exist
      const int64_t id = below(next_id + 3);
      int32_t stt[2], b[2];
      int64_t o[2], s[2];
      for (int k = 0; k < 2; ++k) rc[k] = daf_store_query(st[k], id, &stt[k], &b[k], &o[k], &s[k]);
      CHECK(rc[0] == rc[1]);
      if (rc[0] == DAF_OK) CHECK(stt[0] == stt[1] && b[0] == b[1] && o[0] == o[1] && s[0] == s[1]);
    }
    for (int k = 0; k < 2; ++k) CHECK(daf_store_validate(st[k]) == DAF_OK);
    CHECK(daf_store_used_bytes(st[0]) == daf_store_used_bytes(st[1]));
    CHECK(daf_store_used_time_ns(st[0]) == daf_store_used_time_ns(st[1]));
    CHECK(daf_store_capacity_bytes(st[0]) == daf_store_capacity_bytes(st[1]));
    CHECK(daf_store_num_selections(st[0]) == daf_store_num_selections(st[1]));
  }
  for (int k = 0; k < 2; ++k) daf_store_destroy(st[k]);
}
}  // namespace

int main(int argc, char** argv) {
  const int seeds = argc > 1 ? std::atoi(argv[1]) : 20;
  const int n_ops = argc > 2 ? std::atoi(argv[2]) : 3000;
  for (int seed = 0; seed < seeds; ++seed) run(seed, n_ops);
  std::printf("ok: %d seeds x %d calls; not stored %ld, stored narrower %ld, moved %ld, evicted after storing %ld, released after eviction %ld\n",
              seeds, n_ops, n_not_stored, n_narrowed, n_moves, n_evicted, n_release_gone);
  return 0;
}
