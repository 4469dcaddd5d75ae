// Work decomposition of the DPPF kernels: the tile list of a tensor list, the split of the tiles
// over thread blocks, and the walk a block makes over its share.  Nothing here touches HIP: the
// same code runs inside the kernels (dppf_kernels.h supplies the block's view of the machine) and,
// compiled with a host compiler and sanitizers, inside a plain C++ test that runs one host thread
// per simulated block.
#ifndef DPPF_WALK_H_
#define DPPF_WALK_H_

#include <cstdint>
#include <new>
#include <vector>

#if defined(__HIPCC__)
#define DPPF_HD __host__ __device__
#else
#define DPPF_HD
#endif

namespace dppf_walk {

struct Tile {
  long long offset;   // first element inside the tensor
  int tensor;         // index into the tensor list
  int count;          // 1..tile_elems elements
};

// The counter behind the on-demand part of a walk.  It resets itself: the last block to leave puts
// it back to zero, so every launch finds it clean and nothing has to be cleared between launches
// (also inside a captured graph).
struct Sched {
  unsigned int next;   // next on-demand item to hand out
  unsigned int done;   // full-tile blocks that have left the kernel
};

// The tile list holds all full tiles first, then the partial ones (tensor tails and tensors
// smaller than a tile).  Blocks [0, gfull) take the full tiles, the remaining blocks the partial
// ones, so a list of many small tensors does not put short, latency-bound tiles into the streaming
// blocks' loops.
//
// Full tiles are work ITEMS (one per tile, or one per (group of tiles, worker) pair).  Items
// [0, nstatic) go to the blocks with a fixed stride; items [nstatic, nitems) are handed out on
// demand from a counter in device memory.  The compute dies of the chip do not stream at the same
// rate (blocks on some finish a fixed share about 10 % earlier than on others), and with a fixed
// split the early ones idle while the late ones finish; handing out the tail on demand keeps every
// CU busy to the end.
struct Walk {
  int nfull, ntiles;   // tiles [0, nfull) are full, [nfull, ntiles) partial
  int gfull;           // blocks [0, gfull) take full tiles
  int nitems;          // full-tile work items
  int nstatic;         // full-tile items with a fixed owner; the rest are handed out on demand
  Sched* sched;        // used only when nstatic < nitems
};

// Calls full_body(item) for every full-tile item and part_body(item) for every partial-tile item
// of this block.  `item` counts within the full tiles or within the partial tiles.  A block
// owns the items congruent to its index (modulo the number of blocks on that part of the list) in
// the forward and in the REVERSE walk alike, so on a small model sweep 2 finds in its die's L2 what
// sweep 1 left there.  REVERSE walks from the far end: the fixed shares are the upper items and the
// on-demand ones run down to item 0, so sweep 2 starts where sweep 1 stopped, whose data are still
// in the last-level cache.  flush(row) is called with row = block index once the block's fixed
// share (or its partial tiles) is done, and with row = grid size + k after the k-th on-demand item:
// kernels that reduce store their partial sums there, so that the set of rows and what each row
// holds never depend on which block took which item -- results stay bit-reproducible.
//
// Env is the block's view of the machine:
//   int block(), int grid()                    this block's index and the number of blocks
//   unsigned request(Sched*)                   hand-out counter += 1 (one caller per block; the value
//                                              is meaningful in that caller only)
//   int share(unsigned v)                      the requesting caller's v, seen by the whole block
//                                              (the only block-wide synchronisation of the walk)
//   void leave(Sched*, int gfull)              count this block out; the last one resets the counter
template <bool REVERSE, typename Env, typename FullBody, typename PartBody, typename Flush>
DPPF_HD inline void walk_items(Env& env, const Walk& w, int per_tile, FullBody&& full_body, PartBody&& part_body,
                               Flush&& flush) {
  const bool full = env.block() < w.gfull;
  const int me = full ? env.block() : env.block() - w.gfull;
  const int lanes = full ? w.gfull : env.grid() - w.gfull;
  const int count = full ? w.nitems : (w.ntiles - w.nfull) * per_tile;
  // last item this block owns (below `me` if it owns none)
  const int last_owned = count > me ? me + ((count - 1 - me) / lanes) * lanes : me - lanes;
  if (!full) {
    if (REVERSE) {
      for (int j = last_owned; j >= me; j -= lanes) part_body(j);
    } else {
      for (int j = me; j < count; j += lanes) part_body(j);
    }
    flush(env.block());
    return;
  }
  const int ndyn = count - w.nstatic;            // items handed out on demand
  const int lo = REVERSE ? ndyn : 0;             // fixed shares are the items [lo, lo + nstatic)
  // The first on-demand item is requested right away: the answer is there long before it is needed.
  unsigned int fetched = 0;
  if (ndyn > 0) fetched = env.request(w.sched);
  int j = REVERSE ? last_owned : me;
  bool on_demand = false;
  for (;;) {
    if (!on_demand && (REVERSE ? j < lo : j >= lo + w.nstatic)) {
      flush(env.block());
      if (ndyn <= 0) break;
      on_demand = true;
    }
    int k = 0;
    if (on_demand) {
      k = env.share(fetched);
      if (k >= ndyn) break;              // every block gets here: the counter only grows
      fetched = env.request(w.sched);    // the one after, while this one runs
      j = REVERSE ? ndyn - 1 - k : w.nstatic + k;
    }
    full_body(j);
    if (on_demand) flush(env.grid() + k);
    else j += REVERSE ? -lanes : lanes;
  }
  // A block counts itself out only after its last request has been answered, so when the count is
  // complete nobody will touch the counter again in this launch.
  if (ndyn > 0) env.leave(w.sched, w.gfull);
}

// Kernels that handle one worker at a time number their items worker-major: item = worker *
// groups + group, a group being `tiles_per_item` consecutive tiles (the last group may be short).
struct WorkerItem {
  int worker;
  int first_tile;   // within the full tiles, or within the partial tiles
  int end_tile;     // one past the last tile of the item
};

DPPF_HD inline int worker_item_groups(int ntile, int tiles_per_item) {
  return (ntile + tiles_per_item - 1) / tiles_per_item;
}

DPPF_HD inline WorkerItem worker_item(int item, int ntile, int tiles_per_item) {
  const int groups = worker_item_groups(ntile, tiles_per_item);
  WorkerItem it;
  it.worker = item / groups;
  it.first_tile = (item - it.worker * groups) * tiles_per_item;
  it.end_tile = it.first_tile + tiles_per_item < ntile ? it.first_tile + tiles_per_item : ntile;
  return it;
}

// ------------------------------------------------------------------------------ host side

// The tile list of a tensor list: every tensor cut into pieces of tile_elems elements, full
// pieces first (list order kept), then the partial ones.  Returns 0, -1 (a negative size) or
// -4 (more tiles than an int can index safely); throws std::bad_alloc like any container code.
inline int build_tile_list(int T, const int64_t* numel, int tile_elems, std::vector<Tile>* tiles, int* nfull,
                           long long* d, std::vector<long long>* tensor_offset) {
  std::vector<Tile> all;
  tensor_offset->assign(static_cast<size_t>(T) + 1, 0);
  long long total = 0;
  for (int t = 0; t < T; ++t) {
    if (numel[t] < 0) return -1;
    (*tensor_offset)[t] = total;
    total += numel[t];
    for (long long off = 0; off < numel[t]; off += tile_elems) {
      const long long left = numel[t] - off;
      all.push_back(Tile{off, t, static_cast<int>(left < tile_elems ? left : tile_elems)});
    }
    if (all.size() > static_cast<size_t>(INT32_MAX / 2)) return -4;
  }
  (*tensor_offset)[T] = total;
  tiles->clear();
  tiles->reserve(all.size());
  for (const Tile& t : all)
    if (t.count == tile_elems) tiles->push_back(t);
  *nfull = static_cast<int>(tiles->size());
  for (const Tile& t : all)
    if (t.count != tile_elems) tiles->push_back(t);
  *d = total;
  return 0;
}

// How much of a kernel's full-tile work is handed out on demand instead of being split evenly.
// Measured on the five parameter lists:
//  * with an even split the blocks of the slower dies finish last, and on the way there the
//    blocks drift apart, so the part of the tile list (and of DRAM) the chip is working on at one
//    moment widens; on demand the blocks stay on one compact window of consecutive tiles.
//  * short launches lose a little per on-demand item (a barrier per item, per-tile partial sums
//    in the reducing sweeps), long ones gain more than that from the compact window.
// So: launches that move more than kAllOnDemandBytes hand out everything, shorter ones the second
// half; the pure-read reducing sweeps (a few microseconds per tile, per-tile sums too dear) and
// lists with fewer than kMinRoundsOnDemand items per block keep the even split.  The kernels that
// take one worker at a time (items of two tiles of one worker) gain from handing out everything
// earlier: the stand-alone step on a 2.0 GB launch -3.4 %, while sweep 2 of 5..7 workers on
// 1.5..2.2 GB launches loses 2..6 % that way.
enum OnDemand { kEvenSplit, kOnDemand, kOnDemandReducing };
constexpr int kMinRoundsOnDemand = 4;
constexpr int kMinRoundsAllOnDemandReducing = 32;     // per-tile sums: only worth it on long lists
constexpr double kAllOnDemandBytes = 2.2e9;           // about 0.4 ms of traffic
constexpr double kAllOnDemandBytesWorkerItems = 1.5e9;

// Items [0, returned value) of `count` are split evenly over `blocks` blocks, the rest handed out
// on demand; returns count when nothing is.  bytes_per_item: what one item moves.
inline long long evenly_split_items(long long count, int blocks, OnDemand policy, double bytes_per_item,
                                    double all_from_bytes = kAllOnDemandBytes) {
  if (policy == kEvenSplit || blocks <= 0) return count;
  const long long rounds = count / blocks;
  if (rounds < kMinRoundsOnDemand) return count;
  const bool all = static_cast<double>(count) * bytes_per_item >= all_from_bytes &&
                   (policy != kOnDemandReducing || rounds >= kMinRoundsAllOnDemandReducing);
  return all ? 0 : (rounds - (rounds + 1) / 2) * blocks;
}

// Kernels that take all workers of a tile together: one item per full tile (workers_per_tile = 1,
// tiles_per_item = 1).  Kernels that take one worker at a time: one item per worker and group of
// tiles_per_item full tiles (workers_per_tile = M), numbered as worker_item() reads them.
// bytes_per_elem: what the kernel moves per tile element.
inline Walk make_walk(int nfull, int ntiles, int tile_elems, int gfull, int workers_per_tile, int tiles_per_item,
                      OnDemand policy, double bytes_per_elem, Sched* sched) {
  Walk w;
  w.nfull = nfull;
  w.ntiles = ntiles;
  w.gfull = gfull;
  const long long count = static_cast<long long>(worker_item_groups(nfull, tiles_per_item)) * workers_per_tile;
  w.nitems = static_cast<int>(count);
  w.nstatic = static_cast<int>(
      evenly_split_items(count, gfull, policy, bytes_per_elem * tile_elems * tiles_per_item,
                         tiles_per_item > 1 ? kAllOnDemandBytesWorkerItems : kAllOnDemandBytes));
  w.sched = w.nstatic < count ? sched : nullptr;
  return w;
}

// Grid of a launch: `want_per_cu` streaming blocks per CU for the full tiles (never more blocks
// than items) plus up to one more block per CU for the partial tiles.
inline void grid_shape(int num_cu, int per_cu, long long full_items, long long part_items, int* gfull, int* grid) {
  long long gf = static_cast<long long>(num_cu) * per_cu;
  if (gf > full_items) gf = full_items;
  long long gp = num_cu;
  if (gp > part_items) gp = part_items;
  *gfull = static_cast<int>(gf);
  *grid = static_cast<int>(gf + gp);
}

}  // namespace dppf_walk

#endif  // DPPF_WALK_H_
