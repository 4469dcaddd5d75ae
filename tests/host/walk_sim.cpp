// Host-only check of the work decomposition in csrc/dppf_walk.h, meant to be built with
// g++ -fsanitize=address,undefined -pthread.  One host thread stands in for each thread block and
// runs the very walk_items() the kernels run, with an atomic counter in place of the device's:
// for many random shapes every work item must be visited exactly once, every row of partial sums
// written exactly once, and the hand-out counter must be back at zero afterwards.  The tile lists
// are checked for exact coverage of every tensor.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

#include "dppf_walk.h"

using namespace dppf_walk;

namespace {

int g_failures = 0;
#define CHECK(cond, ...)                        \
  do {                                          \
    if (!(cond)) {                              \
      ++g_failures;                             \
      std::fprintf(stderr, "FAILED %s: ", #cond); \
      std::fprintf(stderr, __VA_ARGS__);        \
      std::fprintf(stderr, "\n");               \
    }                                           \
  } while (0)

// One simulated thread block (its thread 0 is the only thread).
struct HostEnv {
  int block_index, grid_size;
  int block() const { return block_index; }
  int grid() const { return grid_size; }
  unsigned int request(Sched* s) { return __atomic_fetch_add(&s->next, 1u, __ATOMIC_RELAXED); }
  int share(unsigned int v) { return static_cast<int>(v); }
  void leave(Sched* s, int gfull) {
    if (__atomic_fetch_add(&s->done, 1u, __ATOMIC_ACQ_REL) == static_cast<unsigned int>(gfull) - 1u) {
      __atomic_store_n(&s->next, 0u, __ATOMIC_RELEASE);
      __atomic_store_n(&s->done, 0u, __ATOMIC_RELEASE);
    }
  }
};

template <bool REVERSE>
void run_launch(const Walk& w, int grid, int per_tile, std::vector<std::atomic<int>>& full_seen,
                std::vector<std::atomic<int>>& part_seen, std::vector<std::atomic<int>>& rows) {
  std::vector<std::thread> blocks;
  for (int b = 0; b < grid; ++b)
    blocks.emplace_back([&, b] {
      HostEnv env{b, grid};
      walk_items<REVERSE>(
          env, w, per_tile, [&](int item) { full_seen.at(static_cast<size_t>(item)).fetch_add(1); },
          [&](int item) { part_seen.at(static_cast<size_t>(item)).fetch_add(1); },
          [&](int row) { rows.at(static_cast<size_t>(row)).fetch_add(1); });
    });
  for (auto& t : blocks) t.join();
}

void check_walk(int nfull, int npart, int num_cu, int per_cu, int workers_per_tile, int tiles_per_item, OnDemand policy,
                double bytes_per_elem, int forced_static, bool reverse, const char* what) {
  Sched sched{0u, 0u};
  const int ntiles = nfull + npart;
  const long long full_items = static_cast<long long>(worker_item_groups(nfull, tiles_per_item)) * workers_per_tile;
  const long long part_items = static_cast<long long>(npart) * workers_per_tile;
  int gfull = 0, grid = 0;
  grid_shape(num_cu, per_cu, full_items, part_items, &gfull, &grid);
  CHECK(gfull <= full_items && grid - gfull <= part_items && grid <= num_cu * (per_cu + 1), "%s", what);
  Walk w = make_walk(nfull, ntiles, 4096, gfull, workers_per_tile, tiles_per_item, policy, bytes_per_elem, &sched);
  CHECK(w.nitems == full_items, "%s: nitems", what);
  CHECK(w.nstatic >= 0 && w.nstatic <= w.nitems, "%s: nstatic %d of %d", what, w.nstatic, w.nitems);
  if (forced_static >= 0 && forced_static <= w.nitems && gfull > 0) {   // any split must work, not only make_walk's
    w.nstatic = forced_static;
    w.sched = w.nstatic < w.nitems ? &sched : nullptr;
  }
  const int ndyn = w.nitems - w.nstatic;
  std::vector<std::atomic<int>> full_seen(static_cast<size_t>(w.nitems)), part_seen(static_cast<size_t>(part_items)),
      rows(static_cast<size_t>(grid + ndyn));
  for (auto& a : full_seen) a = 0;
  for (auto& a : part_seen) a = 0;
  for (auto& a : rows) a = 0;
  if (grid == 0) return;
  if (reverse) run_launch<true>(w, grid, workers_per_tile, full_seen, part_seen, rows);
  else run_launch<false>(w, grid, workers_per_tile, full_seen, part_seen, rows);
  for (size_t i = 0; i < full_seen.size(); ++i)
    CHECK(full_seen[i] == 1, "%s: full item %zu visited %d times (nfull %d gfull %d nstatic %d rev %d)", what, i,
          full_seen[i].load(), nfull, gfull, w.nstatic, reverse);
  for (size_t i = 0; i < part_seen.size(); ++i)
    CHECK(part_seen[i] == 1, "%s: partial item %zu visited %d times", what, i, part_seen[i].load());
  for (size_t i = 0; i < rows.size(); ++i)
    CHECK(rows[i] == 1, "%s: row %zu written %d times (grid %d ndyn %d)", what, i, rows[i].load(), grid, ndyn);
  CHECK(sched.next == 0u && sched.done == 0u, "%s: counter left at %u/%u", what, sched.next, sched.done);
  // worker items cover every (worker, tile) pair exactly once
  if (workers_per_tile > 1) {
    std::vector<int> cover(static_cast<size_t>(nfull) * workers_per_tile, 0);
    for (int item = 0; item < w.nitems; ++item) {
      const WorkerItem wi = worker_item(item, nfull, tiles_per_item);
      CHECK(wi.worker >= 0 && wi.worker < workers_per_tile, "%s: worker %d", what, wi.worker);
      for (int t = wi.first_tile; t < wi.end_tile; ++t) {
        CHECK(t >= 0 && t < nfull, "%s: tile %d", what, t);
        if (t >= 0 && t < nfull && wi.worker >= 0 && wi.worker < workers_per_tile)
          ++cover[static_cast<size_t>(wi.worker) * nfull + t];
      }
    }
    for (int c : cover) CHECK(c == 1, "%s: a (worker, tile) pair is covered %d times", what, c);
  }
}

void check_tile_list(const std::vector<int64_t>& numel, int tile) {
  std::vector<Tile> tiles;
  std::vector<long long> offs;
  int nfull = 0;
  long long d = 0;
  const int rc = build_tile_list(static_cast<int>(numel.size()), numel.data(), tile, &tiles, &nfull, &d, &offs);
  CHECK(rc == 0, "build_tile_list rc %d", rc);
  long long total = 0;
  for (int64_t n : numel) total += n;
  CHECK(d == total, "d");
  std::vector<std::vector<char>> seen(numel.size());
  for (size_t t = 0; t < numel.size(); ++t) seen[t].assign(static_cast<size_t>(numel[t]), 0);
  for (size_t i = 0; i < tiles.size(); ++i) {
    const Tile& tl = tiles[i];
    CHECK(tl.tensor >= 0 && tl.tensor < static_cast<int>(numel.size()), "tensor index");
    CHECK(tl.count >= 1 && tl.count <= tile, "count");
    CHECK((static_cast<int>(i) < nfull) == (tl.count == tile), "full tiles come first");
    CHECK(tl.offset >= 0 && tl.offset + tl.count <= numel[static_cast<size_t>(tl.tensor)], "range");
    for (int k = 0; k < tl.count; ++k) ++seen[static_cast<size_t>(tl.tensor)][static_cast<size_t>(tl.offset + k)];
  }
  for (auto& s : seen)
    for (char c : s) CHECK(c == 1, "element covered %d times", c);
  const int64_t bad[2] = {5, -1};
  CHECK(build_tile_list(2, bad, tile, &tiles, &nfull, &d, &offs) == -1, "negative size is rejected");
}

}  // namespace

int main(int argc, char** argv) {
  const int rounds = argc > 1 ? std::atoi(argv[1]) : 300;
  std::mt19937 rng(12345);
  auto pick = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };
  // tile lists
  for (int tile : {4096, 2048, 1024}) {
    check_tile_list({}, tile);
    check_tile_list({0}, tile);
    check_tile_list({1, 0, tile - 1, tile, tile + 1, 3 * tile, 3 * tile + 5, 7}, tile);
    for (int k = 0; k < 20; ++k) {
      std::vector<int64_t> numel(static_cast<size_t>(pick(1, 12)));
      for (auto& n : numel) n = pick(0, 4) == 0 ? pick(0, 9) : pick(0, 5 * tile);
      check_tile_list(numel, tile);
    }
  }
  // evenly_split_items: the documented policy
  CHECK(evenly_split_items(1000, 10, kEvenSplit, 1e9) == 1000, "even split keeps everything");
  CHECK(evenly_split_items(39, 10, kOnDemand, 1e9) == 39, "fewer than four items per block: even split");
  CHECK(evenly_split_items(1000, 10, kOnDemand, 1e3) == 500, "short launch: second half on demand");
  CHECK(evenly_split_items(1000, 10, kOnDemand, 1e9) == 0, "long launch: everything on demand");
  CHECK(evenly_split_items(310, 10, kOnDemandReducing, 1e9) == 150, "reducing sweep below 32 rounds: half");
  CHECK(evenly_split_items(320, 10, kOnDemandReducing, 1e9) == 0, "reducing sweep from 32 rounds: everything");
  // walks: edge shapes first, then random ones
  const OnDemand policies[3] = {kEvenSplit, kOnDemand, kOnDemandReducing};
  for (bool rev : {false, true}) {
    check_walk(0, 0, 4, 1, 1, 1, kOnDemand, 1e9, -1, rev, "empty");
    check_walk(0, 5, 4, 1, 1, 1, kOnDemand, 1e9, -1, rev, "only partial tiles");
    check_walk(1, 0, 4, 1, 1, 1, kOnDemand, 1e9, -1, rev, "one tile");
    check_walk(100, 3, 4, 2, 1, 1, kOnDemand, 1e9, 0, rev, "all on demand");
    check_walk(100, 3, 4, 2, 1, 1, kOnDemand, 1e9, 1, rev, "one fixed item");
    check_walk(100, 3, 4, 2, 1, 1, kOnDemand, 1e9, 99, rev, "one on-demand item");
    check_walk(101, 0, 4, 1, 3, 2, kOnDemand, 1e9, -1, rev, "odd number of full tiles in pairs");
    check_walk(7, 9, 8, 1, 5, 2, kOnDemand, 1e9, 3, rev, "more blocks than items");
  }
  for (int k = 0; k < rounds; ++k) {
    const int nfull = pick(0, 3) == 0 ? pick(0, 6) : pick(0, 400);
    const int npart = pick(0, 2) == 0 ? 0 : pick(0, 40);
    const int num_cu = pick(1, 12), per_cu = pick(1, 2);
    const int workers = pick(0, 1) ? 1 : pick(2, 6);
    const int tiles_per_item = workers == 1 ? 1 : pick(1, 3);
    const OnDemand policy = policies[pick(0, 2)];
    const double bytes = pick(0, 1) ? 1e9 : 100.0;
    const int groups = worker_item_groups(nfull, tiles_per_item) * workers;
    const int forced = pick(0, 2) == 0 ? pick(0, groups) : -1;
    check_walk(nfull, npart, num_cu, per_cu, workers, tiles_per_item, policy, bytes, forced, pick(0, 1) == 1, "random");
  }
  if (g_failures) {
    std::fprintf(stderr, "%d checks failed\n", g_failures);
    return 1;
  }
  std::printf("walk simulation: all checks passed (%d random launches)\n", rounds);
  return 0;
}
