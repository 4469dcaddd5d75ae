// DPPF consensus round and local step for MI355X (gfx950, wave64).
//
// The work is bandwidth-bound streaming over the M workers' parameter tensors, so the design
// is about bytes and about what the memory system likes, not about flops:
//   * the round is two sweeps over x, because the per-worker coefficient alpha - lambda/r_m
//     (Sec. 5, Eq. 5) needs r_m, a reduction over the whole model, before any element moves:
//     sweep 1 reads x once (average kept in registers, squared distances accumulated into
//     per-block partial sums), sweep 2 turns the partial sums into the coefficients, reads x
//     again, recomputes the average from the same M loads and writes x.  12 bytes per
//     replica-parameter.
//   * the fused form folds the last local step (Alg. 1, SGD line) into sweep 1 and never stores
//     the stepped x: sweep 1 reads x, v, g and writes only v; sweep 2 reads the OLD x and the NEW
//     v, rebuilds x - lr v with the same fused multiply-add (same bits) and applies Eq. 5.
//     28 bytes instead of 32, and 20 of them reads (reads stream faster than writes here).
//   * a tensor list is cut into tiles of kTileElems consecutive elements of one tensor; a fixed
//     number of thread blocks (one or two per CU) walks the tile list, so one launch covers any
//     number of tensors of any size.  Full tiles and partial ones (tensor tails, small tensors)
//     are walked by different blocks.  Loads are 16-byte vectors with 4-byte alignment (legal for
//     global memory on gfx9), so no tensor needs 16-byte alignment; only the last, partial vector
//     of a tensor is handled element by element.
//   * the chip's compute dies do not stream at the same rate, so an even split of the tiles leaves
//     the faster ones idle at the end: the read-write sweeps split only the first part of their
//     tiles evenly and hand the rest out on demand from a counter (see walk_items).  Partial sums
//     are kept per block for the even part and per tile for the on-demand part, so the result does
//     not depend on which block took which tile.
//   * the gap of a worker to the average is formed relative to worker 0 (see mean_offset), so it
//     keeps full relative precision and is exactly zero for identical replicas.
//   * squared distances: fp32 inside a tile (16 values per lane), fp64 across tiles, lanes,
//     waves and blocks, in a fixed order -- results are bit-reproducible run to run.
//   * sweep 2 walks the tiles in the opposite order to sweep 1, so that the part of x that
//     sweep 1 touched last is still in the last-level cache when sweep 2 starts.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "dppf.h"
#include "dppf_kernels.h"

static_assert(kTileElems == DPPF_TILE_ELEMS, "the header documents the tile size");

namespace {

// =========================================================================== host side
thread_local int g_last_hip_error = 0;

#define HIP_TRY(expr)                                  \
  do {                                                 \
    hipError_t e__ = (expr);                           \
    if (e__ != hipSuccess) {                           \
      g_last_hip_error = static_cast<int>(e__);        \
      return DPPF_EHIP;                                \
    }                                                  \
  } while (0)

// A device copy of a host pointer table, refreshed only when the host contents change.
struct PtrTable {
  std::vector<const void*> host;   // what the device copy currently holds
  const void** staging = nullptr;  // pinned, source of the async upload
  const void** dev = nullptr;
  hipEvent_t uploaded = nullptr;   // marks the end of the last upload from `staging`
  size_t cap = 0;
  bool valid = false;
};

struct TimingRec {
  int id;
  hipEvent_t start, stop;
};

// What the library remembers per device for the life of the process, in fixed-size storage (the
// entry point that must not allocate uses it too): resident blocks per CU of every kernel that has
// been launched there, and the address of that device's copy of the static scratch array.
constexpr int kMaxDevices = 64;
constexpr int kOccupancySlots = 1024;
struct DeviceState {
  int num_cu = 0;
  int nocc = 0;
  const void* occ_kernel[kOccupancySlots];
  int occ_per_cu[kOccupancySlots];
  unsigned char* static_scratch = nullptr;
};
DeviceState g_device[kMaxDevices];
std::mutex g_device_mutex;

// Scratch memory of dppf_pull_push_round_flat_static, the entry point for callers that may not
// allocate: a file-scope device array (every GPU the library runs on holds its own copy until the
// process ends).  Host code never uses the array's name as an address; it asks the runtime for
// this device's copy once (static_scratch_base) and passes that pointer to the kernels.
constexpr long long kStaticMaxDim = 1ll << 27;              // elements per worker
constexpr int kStaticMaxWorkers = kMaxTemplM;
constexpr int kStaticMaxTiles = static_cast<int>(kStaticMaxDim / kTileElems) + 1;
constexpr int kStaticMaxRows = 2048;                        // rows of partial sums (one per block)
constexpr size_t round_up_256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t kStaticOffSched = 0;
constexpr size_t kStaticOffCoef = kStaticOffSched + round_up_256(sizeof(Sched));
constexpr size_t kStaticOffPtrs = kStaticOffCoef + round_up_256(sizeof(Coef) * kStaticMaxWorkers);
constexpr size_t kStaticOffTiles = kStaticOffPtrs + round_up_256(sizeof(float*) * kStaticMaxWorkers);
constexpr size_t kStaticOffPartials = kStaticOffTiles + round_up_256(sizeof(Tile) * (kStaticMaxTiles + 1));
constexpr size_t kStaticBytes =
    kStaticOffPartials + round_up_256(sizeof(double) * kStaticMaxRows * kStaticMaxWorkers);
static_assert(kStaticBytes == DPPF_STATIC_SCRATCH_BYTES, "the header documents the size of the static scratch");
static __device__ __align__(256) unsigned char g_static_scratch[kStaticBytes];

}  // namespace

struct dppf_plan {
  int M = 0, T = 0;
  int device = 0;
  int num_cu = 0;
  long long d = 0;
  std::vector<long long> numel;
  int ntiles = 0;
  int nfull = 0;                // tiles [0, nfull) are full, [nfull, ntiles) partial
  Tile* tiles_dev = nullptr;
  double* partials = nullptr;   // [partials_rows][M]: one row per block, then one per on-demand tile
  int partials_rows = 0;
  Sched* sched = nullptr;       // the counter behind the on-demand part of a kernel's tile walk
  Coef* coef = nullptr;         // [M]
  float* xbar_scratch = nullptr;            // d floats, only when M > kMaxTemplM
  float* usum_scratch = nullptr;            // d floats, only when M > kMaxTemplM (exact update)
  std::vector<long long> tensor_offset;     // start of tensor t inside xbar_scratch
  enum Role { RX = 0, RV, RG, RM1, RM2, RXBAR, RXBAR_SCRATCH, RUSUM_SCRATCH, RXC, NROLES };
  PtrTable tab[NROLES];
  // timing
  bool timing = false;
  std::vector<TimingRec> recs;
  std::vector<hipEvent_t> event_pool;
};

namespace {

int table_upload(dppf_plan* p, int role, const void* const* host, size_t n, hipStream_t s,
                 const void*** dev_out) {
  PtrTable& t = p->tab[role];
  // Every entry point that takes a plan comes through here first: its buffers live on one device.
  int current = -1;
  HIP_TRY(hipGetDevice(&current));
  if (current != p->device) return DPPF_EINVAL;
  if (n == 0) {
    *dev_out = t.dev;   // never dereferenced: no tiles
    return DPPF_OK;
  }
  if (t.valid && t.host.size() == n && std::memcmp(t.host.data(), host, n * sizeof(void*)) == 0) {
    *dev_out = t.dev;
    return DPPF_OK;
  }
  // validate before touching anything
  const size_t per_row = static_cast<size_t>(p->T);
  for (size_t i = 0; i < n; ++i) {
    const long long ne = p->numel[i % per_row];
    if (ne > 0 && host[i] == nullptr) return DPPF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(host[i]) & 3u) != 0) return DPPF_EINVAL;
  }
  HIP_TRY(hipEventSynchronize(t.uploaded));   // the previous upload has left the staging buffer
  t.valid = false;                            // until the new contents are on their way
  std::memcpy(t.staging, host, n * sizeof(void*));
  HIP_TRY(hipMemcpyAsync(t.dev, t.staging, n * sizeof(void*), hipMemcpyHostToDevice, s));
  HIP_TRY(hipEventRecord(t.uploaded, s));
  t.host.assign(host, host + n);
  t.valid = true;
  *dev_out = t.dev;
  return DPPF_OK;
}

int table_alloc(PtrTable& t, size_t n) {
  t.cap = n;
  if (n == 0) n = 1;
  HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&t.staging), n * sizeof(void*), hipHostMallocDefault));
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&t.dev), n * sizeof(void*)));
  HIP_TRY(hipEventCreateWithFlags(&t.uploaded, hipEventDisableTiming));
  return DPPF_OK;
}

void table_free(PtrTable& t) {
  if (t.staging) (void)hipHostFree(t.staging);
  if (t.dev) (void)hipFree(t.dev);
  if (t.uploaded) (void)hipEventDestroy(t.uploaded);
  t = PtrTable();
}

// ---- timing brackets
int timing_begin(dppf_plan* p, int id, hipStream_t s) {
  if (!p->timing) return DPPF_OK;
  hipEvent_t ev[2];
  for (int i = 0; i < 2; ++i) {
    if (!p->event_pool.empty()) {
      ev[i] = p->event_pool.back();
      p->event_pool.pop_back();
    } else {
      HIP_TRY(hipEventCreate(&ev[i]));
    }
  }
  p->recs.push_back(TimingRec{id, ev[0], ev[1]});
  HIP_TRY(hipEventRecord(ev[0], s));
  return DPPF_OK;
}

int timing_end(dppf_plan* p, hipStream_t s) {
  if (!p->timing) return DPPF_OK;
  HIP_TRY(hipEventRecord(p->recs.back().stop, s));
  return DPPF_OK;
}

// ---- grid sizes: enough resident blocks to fill every CU, never more blocks than tiles
template <typename K>
int grid_for(dppf_plan* p, K kernel, int per_tile_items, int want_per_cu, int* gfull_out, int* grid_out) {
  int per_cu = 0;
  const void* key = reinterpret_cast<const void*>(kernel);
  if (p->device < 0 || p->device >= kMaxDevices) return DPPF_ELIMIT;
  {
    std::lock_guard<std::mutex> lock(g_device_mutex);
    DeviceState& dev = g_device[p->device];
    for (int i = 0; i < dev.nocc; ++i)
      if (dev.occ_kernel[i] == key) per_cu = dev.occ_per_cu[i];
    if (per_cu == 0) {
      HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kBlock, 0));
      if (per_cu < 1) per_cu = 1;
      if (dev.nocc < kOccupancySlots) {      // a full table only means the query is repeated
        dev.occ_kernel[dev.nocc] = key;
        dev.occ_per_cu[dev.nocc] = per_cu;
        ++dev.nocc;
      }
    }
  }
  if (per_cu < 1) per_cu = 1;
  if (per_cu > want_per_cu) per_cu = want_per_cu;
  if (per_cu > kMaxBlocksPerCU - 1) per_cu = kMaxBlocksPerCU - 1;
  // streaming blocks for the full tiles ...
  long long gfull = static_cast<long long>(p->num_cu) * per_cu;
  const long long full_items = static_cast<long long>(p->nfull) * per_tile_items;
  if (gfull > full_items) gfull = full_items;
  // ... plus up to one more block per CU for the partial tiles
  long long gpart = p->num_cu;
  const long long part_items = static_cast<long long>(p->ntiles - p->nfull) * per_tile_items;
  if (gpart > part_items) gpart = part_items;
  *gfull_out = static_cast<int>(gfull);
  *grid_out = static_cast<int>(gfull + gpart);   // <= num_cu * kMaxBlocksPerCU
  return DPPF_OK;
}

// How much of a kernel's full-tile work is handed out on demand instead of being split evenly
// (see walk_items).  Measured on the five lists:
//  * with an even split the blocks of the slower dies finish last, and on the way there the
//    blocks drift apart, so the part of the tile list (and of DRAM) the chip is working on at one
//    moment widens; on demand the blocks stay on one compact window of consecutive tiles.
//  * short launches lose a little per on-demand item (a barrier per item, per-tile partial sums
//    in the reducing sweeps), long ones gain more than that from the compact window.
// So: launches that move more than kAllOnDemandBytes hand out everything, shorter ones the second
// half; the pure-read reducing sweeps (a few microseconds per tile, per-tile sums too dear) and
// lists with fewer than kMinRoundsOnDemand items per block keep the even split.
enum OnDemand { kEvenSplit, kOnDemand, kOnDemandReducing };
constexpr int kMinRoundsOnDemand = 4;
constexpr int kMinRoundsAllOnDemandReducing = 32;     // per-tile sums: only worth it on long lists
constexpr double kAllOnDemandBytes = 2.2e9;           // about 0.4 ms of traffic

// Items [0, returned value) of `count` are split evenly over `blocks` blocks, the rest handed out
// on demand; returns count when nothing is.  bytes_per_item: what one item moves.
long long evenly_split_items(long long count, int blocks, OnDemand policy, double bytes_per_item) {
  if (policy == kEvenSplit || blocks <= 0) return count;
  const long long rounds = count / blocks;
  if (rounds < kMinRoundsOnDemand) return count;
  const bool all = static_cast<double>(count) * bytes_per_item >= kAllOnDemandBytes &&
                   (policy != kOnDemandReducing || rounds >= kMinRoundsAllOnDemandReducing);
  return all ? 0 : (rounds - (rounds + 1) / 2) * blocks;
}

// Kernels that take all workers of a tile together: one item per full tile (workers_per_tile = 1,
// tiles_per_item = 1).  Kernels that take one worker at a time: one item per worker and
// kTilesPerWorkerItem full tiles (workers_per_tile = M) -- the kernel's own arithmetic on item
// numbers assumes exactly that, whatever M is.  bytes_per_elem: what a kernel moves per tile element.
Walk make_walk(const dppf_plan* p, int gfull, int workers_per_tile, int tiles_per_item, OnDemand policy,
               double bytes_per_elem) {
  Walk w;
  w.nfull = p->nfull;
  w.ntiles = p->ntiles;
  w.gfull = gfull;
  const long long count =
      static_cast<long long>((p->nfull + tiles_per_item - 1) / tiles_per_item) * workers_per_tile;
  w.nitems = static_cast<int>(count);
  w.nstatic = static_cast<int>(
      evenly_split_items(count, gfull, policy, bytes_per_elem * kTileElems * tiles_per_item));
  w.sched = w.nstatic < count ? p->sched : nullptr;
  return w;
}

// The launch shape of a reducing sweep: later launches that add to the same rows of partial
// sums (worker groups) and the launch that reads them must agree on it.
struct GridShape {
  int grid = 0;
  Walk walk{};
  int nparts() const { return grid + (walk.nitems - walk.nstatic); }
};

// Which of sweep 1's x loads go through the caches (see k_sweep1).
enum KeepPolicy {
  kKeepTail,     // only the tiles touched last, as many as fit the last-level cache budget
  kKeepNone      // nothing reads x again soon
};
constexpr long long kLastLevelCacheBudget = 256ll << 20;   // bytes of x worth keeping (the cache is 256 MB)

int keep_from_tile(const dppf_plan* p, int workers, KeepPolicy keep) {
  if (keep == kKeepNone) return p->nfull;
  const long long per_tile = static_cast<long long>(workers) * kTileElems * sizeof(float);
  const long long tiles = kLastLevelCacheBudget / per_tile;
  return tiles >= p->nfull ? 0 : p->nfull - static_cast<int>(tiles);
}

// U = 16-byte vectors of one worker that a lane handles per pass over a tile (a tile is four).  A
// lane keeps M*U vectors of x; the fused sweeps add one worker's v and g (or AdamW's three) at a
// time.  With one block per CU a lane may use the whole 512-entry register file; the values are
// the fastest measured per range of M.
constexpr int unroll_plain(int M) { return M <= 4 ? 4 : (M <= 8 ? 2 : 1); }
constexpr int unroll_step_update(int M) { return M <= 4 ? 4 : (M <= 8 ? 2 : 1); }
constexpr int unroll_fused(int M) { return M <= 8 ? 4 : 2; }

#define DPPF_SWITCH_M(m_value, ...)                                \
  switch (m_value) {                                               \
    case 1: { constexpr int kM = 1; __VA_ARGS__ } break;           \
    case 2: { constexpr int kM = 2; __VA_ARGS__ } break;           \
    case 3: { constexpr int kM = 3; __VA_ARGS__ } break;           \
    case 4: { constexpr int kM = 4; __VA_ARGS__ } break;           \
    case 5: { constexpr int kM = 5; __VA_ARGS__ } break;           \
    case 6: { constexpr int kM = 6; __VA_ARGS__ } break;           \
    case 7: { constexpr int kM = 7; __VA_ARGS__ } break;           \
    case 8: { constexpr int kM = 8; __VA_ARGS__ } break;           \
    case 9: { constexpr int kM = 9; __VA_ARGS__ } break;           \
    case 10: { constexpr int kM = 10; __VA_ARGS__ } break;           \
    case 11: { constexpr int kM = 11; __VA_ARGS__ } break;           \
    case 12: { constexpr int kM = 12; __VA_ARGS__ } break;           \
    case 13: { constexpr int kM = 13; __VA_ARGS__ } break;           \
    case 14: { constexpr int kM = 14; __VA_ARGS__ } break;           \
    case 15: { constexpr int kM = 15; __VA_ARGS__ } break;           \
    case 16: { constexpr int kM = 16; __VA_ARGS__ } break;           \
    default: return DPPF_ELIMIT;                                   \
  }

// Launch sweep 1 over workers [m0, m0+mg) of the table (mg <= kMaxTemplM).
template <bool SGD, int XBAR, bool NORMS>
int launch_sweep1(dppf_plan* p, int mg, const void** xp, const void** vp, const void** gp,
                  const void** xbarp, float lr, float mu, float wd, int m0, KeepPolicy keep, GridShape* shape,
                  hipStream_t s) {
  float* const* x = (float* const*)(xp) + static_cast<size_t>(m0) * p->T;
  float* const* v = vp ? (float* const*)(vp) + static_cast<size_t>(m0) * p->T : nullptr;
  const float* const* g = gp ? (const float* const*)(gp) + static_cast<size_t>(m0) * p->T : nullptr;
  float* const* xb = (float* const*)(xbarp);
  DPPF_SWITCH_M(mg, {
    constexpr int kU = SGD ? unroll_fused(kM) : unroll_plain(kM);
    auto kern = k_sweep1<kM, kU, SGD, XBAR, NORMS>;
    int grid = 0;
    Walk walk;
    if (shape && shape->grid > 0) {   // later worker groups must fill the same rows of the partial sums
      grid = shape->grid;
      walk = shape->walk;
    } else {
      int gfull = 0;
      int rc = grid_for(p, kern, 1, (SGD || XBAR == 1) ? kBlocksPerCUReadWrite : kBlocksPerCUReadOnly, &gfull,
                        &grid);
      if (rc) return rc;
      walk = make_walk(p, gfull, 1, 1, SGD ? kOnDemandReducing : kEvenSplit, 16.0 * mg);
      if (shape) {
        shape->grid = grid;
        shape->walk = walk;
      }
    }
    if (grid + (walk.nitems - walk.nstatic) > p->partials_rows) return DPPF_ELIMIT;   // rows of partial sums
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, walk, p->T, x, v, g, xb,
                       lr, mu, wd, p->partials + m0, p->M, keep_from_tile(p, mg, keep));
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

template <int XBAR, bool STEP, bool FOLD>
int launch_sweep2(dppf_plan* p, int mg, const void** xp, const void** vp, const void** xbarp, float lr,
                  int m0, int nparts, float pull, float push, float* r_out, float* c_out, hipStream_t s) {
  float* const* x = (float* const*)(xp) + static_cast<size_t>(m0) * p->T;
  const float* const* v = vp ? (const float* const*)(vp) + static_cast<size_t>(m0) * p->T : nullptr;
  const float* const* xb = (const float* const*)(xbarp);
  DPPF_SWITCH_M(mg, {
    constexpr int kU = STEP ? unroll_step_update(kM) : unroll_plain(kM);
    auto kern = k_sweep2<kM, kU, XBAR, STEP, FOLD>;
    int grid = 0, gfull = 0;
    int rc = grid_for(p, kern, 1, kBlocksPerCUReadWrite, &gfull, &grid);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kOnDemand, (STEP ? 12.0 : 8.0) * mg), p->T, x, v, xb, lr,
                       p->coef + m0, 1.0f / static_cast<float>(kM), p->partials, nparts, p->M, pull, push,
                       r_out, c_out);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_finalize(dppf_plan* p, int nparts, float pull, float push, bool want_coef, float* r_out,
                    float* c_out, hipStream_t s) {
  int rc = timing_begin(p, DPPF_K_FINALIZE, s);
  if (rc) return rc;
  hipLaunchKernelGGL(k_finalize, dim3(p->M), dim3(kBlock), 0, s, p->partials, nparts, p->M, pull, push,
                     want_coef ? p->coef : nullptr, r_out, c_out);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_local_step(dppf_plan* p, const void** xp, const void** vp, const void** gp, float lr,
                      float mu, float wd, hipStream_t s) {
  auto kern = k_local_step<4>;
  int grid = 0, gfull = 0;
  int rc = grid_for(p, kern, p->M, kBlocksPerCUReadWrite, &gfull, &grid);
  if (rc) return rc;
  rc = timing_begin(p, DPPF_K_LOCAL_STEP, s);
  if (rc) return rc;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, p->M, kTilesPerWorkerItem, kOnDemand, 20.0), p->M,
                     p->T, (float* const*)(xp), (float* const*)(vp), (const float* const*)(gp), lr, mu, wd);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_mean_any(dppf_plan* p, const void** xp, const void** xbarp, hipStream_t s) {
  int grid = 0, gfull = 0;
  int rc = grid_for(p, k_mean_any, 1, kBlocksPerCUReadOnly, &gfull, &grid);
  if (rc) return rc;
  hipLaunchKernelGGL(k_mean_any, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kEvenSplit, 0.0),
                     p->M, p->T, (float* const*)(xp), (float* const*)(xbarp));
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_update_exact(dppf_plan* p, const void** xp, int nparts, float pull, float push_r, float* r_out,
                        float* c_out, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float mf = static_cast<float>(p->M);
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_plain(kM);
    auto kern = k_update_exact<kM, kU>;
    int grid = 0, gfull = 0;
    int rc = grid_for(p, kern, 1, kBlocksPerCUReadWrite, &gfull, &grid);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kOnDemand, 8.0 * p->M), p->T, x,
                       p->partials, nparts, p->M, pull, push_r / mf, push_r / (mf * mf), r_out, c_out);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

// Sweep 1 (WRITE = false) or sweep 2 (WRITE = true) of dppf_pull_then_push over workers
// [m0, m0+mg).  REF as in seq_tile; refp is the stored average for REF == 2.
template <int REF, bool WRITE>
int launch_seq(dppf_plan* p, int mg, int m0, const void** xp, const void** xcp, const void** refp, float pull,
               float push, int nparts, float* r_post_out, GridShape* shape, hipStream_t s) {
  float* const* x = (float* const*)(xp) + static_cast<size_t>(m0) * p->T;
  const float* const* xc = (const float* const*)(xcp);
  const float* const* rf = (const float* const*)(refp);
  const float keep = static_cast<float>(1.0 - static_cast<double>(pull));
  int rc;
  DPPF_SWITCH_M(mg, {
    constexpr int kU = unroll_plain(kM) > 2 ? 2 : unroll_plain(kM);
    int grid = 0, gfull = 0;
    if (WRITE) {
      auto kern = k_seq2<kM, kU, REF>;
      if ((rc = grid_for(p, kern, 1, kBlocksPerCUReadWrite, &gfull, &grid))) return rc;
      hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kOnDemand, 8.0 * mg + 4.0), p->T, x,
                         xc, rf, pull, keep, push, p->partials + m0, nparts, p->M,
                         r_post_out ? r_post_out + m0 : nullptr);
    } else {
      auto kern = k_seq1<kM, kU, REF>;
      if (shape->grid == 0) {     // later worker groups fill the same rows of the partial sums
        if ((rc = grid_for(p, kern, 1, kBlocksPerCUReadOnly, &gfull, &grid))) return rc;
        shape->grid = grid;
        shape->walk = make_walk(p, gfull, 1, 1, kEvenSplit, 0.0);
      }
      hipLaunchKernelGGL(kern, dim3(shape->grid), dim3(kBlock), 0, s, p->tiles_dev, shape->walk, p->T, x, xc,
                         rf, pull, keep, p->partials + m0, p->M);
    }
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

template <int REF>
int run_seq(dppf_plan* p, const void** xp, const void** xcp, const void** refp, float pull, float push,
            float* r_post_out, hipStream_t s) {
  GridShape shape;
  int rc;
  if ((rc = timing_begin(p, DPPF_K_SEQ_REDUCE, s))) return rc;
  for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
    const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
    if ((rc = launch_seq<REF, false>(p, mg, m0, xp, xcp, refp, pull, push, 0, nullptr, &shape, s))) return rc;
  }
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_SEQ_UPDATE, s))) return rc;
  for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
    const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
    if ((rc = launch_seq<REF, true>(p, mg, m0, xp, xcp, refp, pull, push, shape.nparts(), r_post_out, nullptr, s)))
      return rc;
  }
  return timing_end(p, s);
}

// The scratch average used when M > kMaxTemplM: a pointer table into the plan's own d-vector.
int scratch_xbar_table(dppf_plan* p, hipStream_t s, const void*** dev_out) {
  std::vector<const void*> host(static_cast<size_t>(p->T));
  for (int t = 0; t < p->T; ++t) host[t] = p->xbar_scratch + p->tensor_offset[t];
  return table_upload(p, dppf_plan::RXBAR_SCRATCH, host.data(), host.size(), s, dev_out);
}

// The second scratch vector (sum of unit gap vectors of the exact update), M > kMaxTemplM only.
int scratch_usum_table(dppf_plan* p, hipStream_t s, const void*** dev_out) {
  std::vector<const void*> host(static_cast<size_t>(p->T));
  for (int t = 0; t < p->T; ++t) host[t] = p->usum_scratch + p->tensor_offset[t];
  return table_upload(p, dppf_plan::RUSUM_SCRATCH, host.data(), host.size(), s, dev_out);
}

// The tile list of a tensor list: every tensor cut into pieces of kTileElems elements, full
// pieces first (list order kept), then the partial ones.  Pure host code.
int build_tile_list(int T, const int64_t* numel, std::vector<Tile>* tiles, int* nfull, long long* d,
                    std::vector<long long>* tensor_offset) {
  try {
    std::vector<Tile> all;
    tensor_offset->assign(static_cast<size_t>(T) + 1, 0);
    long long total = 0;
    for (int t = 0; t < T; ++t) {
      if (numel[t] < 0) return DPPF_EINVAL;
      (*tensor_offset)[t] = total;
      total += numel[t];
      for (long long off = 0; off < numel[t]; off += kTileElems) {
        const long long left = numel[t] - off;
        all.push_back(Tile{off, t, static_cast<int>(left < kTileElems ? left : kTileElems)});
      }
      if (all.size() > static_cast<size_t>(INT32_MAX / 2)) return DPPF_ELIMIT;
    }
    (*tensor_offset)[T] = total;
    tiles->clear();
    tiles->reserve(all.size());
    for (const Tile& t : all)
      if (t.count == kTileElems) tiles->push_back(t);
    *nfull = static_cast<int>(tiles->size());
    for (const Tile& t : all)
      if (t.count != kTileElems) tiles->push_back(t);
    *d = total;
  } catch (const std::bad_alloc&) {
    return DPPF_ENOMEM;
  }
  return DPPF_OK;
}

// Adam's hyper-parameters as the kernels take them; the bias corrections 1 - beta^t are formed in
// double on the host.
AdamHyper adam_hyper(float lr, float beta1, float beta2, float eps, float wd, long long step) {
  const double bc1 = 1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step));
  return AdamHyper{lr, beta1, beta2, eps, wd, static_cast<float>(1.0 / bc1), static_cast<float>(1.0 / bc2)};
}

int launch_adamw_step(dppf_plan* p, const void** xd, const void** ad, const void** sd, const void** gd,
                      const AdamHyper hp, hipStream_t s) {
  auto kern = k_adamw_step<2>;
  int grid = 0, gfull = 0, rc;
  if ((rc = grid_for(p, kern, p->M, kBlocksPerCUReadWrite, &gfull, &grid))) return rc;
  if ((rc = timing_begin(p, DPPF_K_ADAMW_STEP, s))) return rc;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, p->M, kTilesPerWorkerItem, kOnDemand, 28.0), p->M,
                     p->T, (float* const*)(xd), (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

// Shared body of dppf_pull_push_round and dppf_round (with_step).
int round_impl(dppf_plan* p, bool with_step, float* const* x, float* const* v, const float* const* g,
               float lr, float mu, float wd, float pull, float push, float* r_out, float* c_out,
               float* const* xbar_out, hipStream_t s) {
  if (!p || !x) return DPPF_EINVAL;
  if (with_step && (!v || !g)) return DPPF_EINVAL;
  const size_t n = static_cast<size_t>(p->M) * p->T;
  const void **xd = nullptr, **vd = nullptr, **gd = nullptr, **xbd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x), n, s, &xd))) return rc;
  if (with_step) {
    if ((rc = table_upload(p, dppf_plan::RV, reinterpret_cast<const void* const*>(v), n, s, &vd))) return rc;
    if ((rc = table_upload(p, dppf_plan::RG, reinterpret_cast<const void* const*>(g), n, s, &gd))) return rc;
  }
  if (xbar_out) {
    if ((rc = table_upload(p, dppf_plan::RXBAR, reinterpret_cast<const void* const*>(xbar_out),
                           static_cast<size_t>(p->T), s, &xbd)))
      return rc;
  }
  if (p->ntiles == 0) {   // d == 0: every distance is zero, nothing moves
    return launch_finalize(p, 0, pull, push, true, r_out, c_out, s);
  }
  GridShape shape;
  if (p->M <= kMaxTemplM) {
    if ((rc = timing_begin(p, with_step ? DPPF_K_STEP_REDUCE : DPPF_K_REDUCE, s))) return rc;
    if (with_step) {
      rc = xbar_out ? launch_sweep1<true, 1, true>(p, p->M, xd, vd, gd, xbd, lr, mu, wd, 0, kKeepTail, &shape, s)
                    : launch_sweep1<true, 0, true>(p, p->M, xd, vd, gd, nullptr, lr, mu, wd, 0, kKeepTail, &shape, s);
    } else {
      rc = xbar_out ? launch_sweep1<false, 1, true>(p, p->M, xd, nullptr, nullptr, xbd, 0, 0, 0, 0, kKeepTail, &shape, s)
                    : launch_sweep1<false, 0, true>(p, p->M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepTail, &shape, s);
    }
    if (rc) return rc;
    if ((rc = timing_end(p, s))) return rc;
    if ((rc = timing_begin(p, with_step ? DPPF_K_STEP_UPDATE : DPPF_K_UPDATE, s))) return rc;
    if (with_step)
      rc = launch_sweep2<0, true, true>(p, p->M, xd, vd, nullptr, lr, 0, shape.nparts(), pull, push, r_out, c_out, s);
    else
      rc = launch_sweep2<0, false, true>(p, p->M, xd, nullptr, nullptr, 0.f, 0, shape.nparts(), pull, push, r_out, c_out, s);
    if (rc) return rc;
    return timing_end(p, s);
  }
  // More workers than the register-resident kernels take: materialise the average once, then run
  // those kernels over groups of up to kMaxTemplM workers that read it back.
  if (with_step && (rc = launch_local_step(p, xd, vd, gd, lr, mu, wd, s))) return rc;
  const void** avg = xbd;
  if (!avg && (rc = scratch_xbar_table(p, s, &avg))) return rc;
  if ((rc = timing_begin(p, DPPF_K_MEAN, s))) return rc;
  if ((rc = launch_mean_any(p, xd, avg, s))) return rc;
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
  for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
    const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
    if ((rc = launch_sweep1<false, 2, true>(p, mg, xd, nullptr, nullptr, avg, 0, 0, 0, m0, kKeepNone, &shape, s))) return rc;
  }
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = launch_finalize(p, shape.nparts(), pull, push, true, r_out, c_out, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_UPDATE, s))) return rc;
  for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
    const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
    if ((rc = launch_sweep2<2, false, false>(p, mg, xd, nullptr, avg, 0.f, m0, 0, 0.f, 0.f, nullptr, nullptr, s)))
      return rc;
  }
  return timing_end(p, s);
}

}  // namespace

// =============================================================================== C ABI
// No C++ exception may cross the boundary: entry points that can allocate on the host are
// function-try-blocks ending in this.
#define DPPF_CATCH                                        \
  catch (const std::bad_alloc&) { return DPPF_ENOMEM; }   \
  catch (...) { return DPPF_EINVAL; }

extern "C" {

const char* dppf_strerror(int code) {
  switch (code) {
    case DPPF_OK: return "ok";
    case DPPF_EINVAL: return "invalid argument";
    case DPPF_EHIP: return "HIP runtime call failed";
    case DPPF_ENOMEM: return "out of memory";
    case DPPF_ELIMIT: return "size exceeds a library limit";
    default: return "unknown dppf error code";
  }
}

int dppf_last_hip_error(void) { return g_last_hip_error; }

int dppf_plan_destroy(dppf_plan* p) {
  if (!p) return DPPF_OK;
  for (int r = 0; r < dppf_plan::NROLES; ++r) table_free(p->tab[r]);
  if (p->tiles_dev) (void)hipFree(p->tiles_dev);
  if (p->partials) (void)hipFree(p->partials);
  if (p->coef) (void)hipFree(p->coef);
  if (p->sched) (void)hipFree(p->sched);
  if (p->xbar_scratch) (void)hipFree(p->xbar_scratch);
  if (p->usum_scratch) (void)hipFree(p->usum_scratch);
  for (auto& r : p->recs) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  for (auto e : p->event_pool) (void)hipEventDestroy(e);
  delete p;
  return DPPF_OK;
}

int dppf_plan_create(dppf_plan** out, int M, int T, const int64_t* numel) {
  if (!out) return DPPF_EINVAL;
  *out = nullptr;
  if (M < 1 || T < 0 || (T > 0 && !numel)) return DPPF_EINVAL;
  if (M > DPPF_MAX_WORKERS) return DPPF_ELIMIT;
  dppf_plan* p = new (std::nothrow) dppf_plan();
  if (!p) return DPPF_ENOMEM;
  std::vector<Tile> tiles;
  p->M = M;
  p->T = T;
  {
    const int rc = build_tile_list(T, numel, &tiles, &p->nfull, &p->d, &p->tensor_offset);
    if (rc != DPPF_OK) {
      delete p;
      return rc;
    }
    p->numel.assign(numel, numel + T);
  }
  p->ntiles = static_cast<int>(tiles.size());

#define PLAN_TRY(expr)                                                             \
  do {                                                                             \
    hipError_t e__ = (expr);                                                       \
    if (e__ != hipSuccess) {                                                       \
      g_last_hip_error = static_cast<int>(e__);                                    \
      dppf_plan_destroy(p);                                                        \
      return e__ == hipErrorOutOfMemory ? DPPF_ENOMEM : DPPF_EHIP;                 \
    }                                                                              \
  } while (0)

  PLAN_TRY(hipGetDevice(&p->device));
  hipDeviceProp_t prop;
  PLAN_TRY(hipGetDeviceProperties(&prop, p->device));
  p->num_cu = prop.multiProcessorCount;
  p->partials_rows = p->num_cu * kMaxBlocksPerCU + p->nfull;   // one per block + at most one per full tile
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->tiles_dev), (tiles.size() + 1) * sizeof(Tile)));
  if (!tiles.empty())
    PLAN_TRY(hipMemcpy(p->tiles_dev, tiles.data(), tiles.size() * sizeof(Tile), hipMemcpyHostToDevice));
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->partials),
                     static_cast<size_t>(p->partials_rows) * M * sizeof(double)));
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->coef), static_cast<size_t>(M) * sizeof(Coef)));
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->sched), sizeof(Sched)));
  PLAN_TRY(hipMemset(p->sched, 0, sizeof(Sched)));
  if (M > kMaxTemplM && p->d > 0) {
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->xbar_scratch), static_cast<size_t>(p->d) * sizeof(float)));
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->usum_scratch), static_cast<size_t>(p->d) * sizeof(float)));
  }
  const size_t n = static_cast<size_t>(M) * T;
  for (int r = 0; r < dppf_plan::NROLES; ++r) {
    const bool per_model = (r == dppf_plan::RXBAR || r == dppf_plan::RXBAR_SCRATCH ||
                            r == dppf_plan::RUSUM_SCRATCH || r == dppf_plan::RXC);
    if (table_alloc(p->tab[r], per_model ? static_cast<size_t>(T) : n) != DPPF_OK) {
      dppf_plan_destroy(p);
      return DPPF_EHIP;
    }
  }
  PLAN_TRY(hipDeviceSynchronize());
#undef PLAN_TRY
  *out = p;
  return DPPF_OK;
}

int64_t dppf_plan_dim(const dppf_plan* p) { return p ? p->d : 0; }

int dppf_layout_tiles(int T, const int64_t* numel, int64_t* d, int64_t* nfull, int64_t* ntiles, int64_t cap,
                      int32_t* tile_tensor, int64_t* tile_offset, int32_t* tile_count) {
  if (T < 0 || (T > 0 && !numel) || !d || !nfull || !ntiles || cap < 0) return DPPF_EINVAL;
  std::vector<Tile> tiles;
  std::vector<long long> offsets;
  int full = 0;
  long long total = 0;
  const int rc = build_tile_list(T, numel, &tiles, &full, &total, &offsets);
  if (rc != DPPF_OK) return rc;
  *d = total;
  *nfull = full;
  *ntiles = static_cast<int64_t>(tiles.size());
  if (tile_tensor && tile_offset && tile_count) {
    if (cap < static_cast<int64_t>(tiles.size())) return DPPF_ELIMIT;
    for (size_t i = 0; i < tiles.size(); ++i) {
      tile_tensor[i] = tiles[i].tensor;
      tile_offset[i] = tiles[i].offset;
      tile_count[i] = tiles[i].count;
    }
  }
  return DPPF_OK;
}

int dppf_replica_mean(dppf_plan* p, const float* const* x, float* const* xbar, void* stream) try {
  if (!p || !x || !xbar) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const void **xd = nullptr, **xbd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x),
                         static_cast<size_t>(p->M) * p->T, s, &xd)))
    return rc;
  if ((rc = table_upload(p, dppf_plan::RXBAR, reinterpret_cast<const void* const*>(xbar),
                         static_cast<size_t>(p->T), s, &xbd)))
    return rc;
  if (p->ntiles == 0) return DPPF_OK;
  if ((rc = timing_begin(p, DPPF_K_MEAN, s))) return rc;
  if (p->M <= kMaxTemplM)
    rc = launch_sweep1<false, 1, false>(p, p->M, xd, nullptr, nullptr, xbd, 0, 0, 0, 0, kKeepNone, nullptr, s);
  else
    rc = launch_mean_any(p, xd, xbd, s);
  if (rc) return rc;
  return timing_end(p, s);
} DPPF_CATCH

int dppf_dist_norms(dppf_plan* p, const float* const* x, const float* const* xbar, float* r_out,
                    void* stream) try {
  if (!p || !x || !r_out) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const void **xd = nullptr, **xbd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x),
                         static_cast<size_t>(p->M) * p->T, s, &xd)))
    return rc;
  if (xbar && (rc = table_upload(p, dppf_plan::RXBAR, reinterpret_cast<const void* const*>(xbar),
                                 static_cast<size_t>(p->T), s, &xbd)))
    return rc;
  if (p->ntiles == 0) return launch_finalize(p, 0, 0.f, 0.f, false, r_out, nullptr, s);
  GridShape shape;
  if (p->M <= kMaxTemplM) {
    if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
    rc = xbar ? launch_sweep1<false, 2, true>(p, p->M, xd, nullptr, nullptr, xbd, 0, 0, 0, 0, kKeepNone, &shape, s)
              : launch_sweep1<false, 0, true>(p, p->M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepNone, &shape, s);
    if (rc) return rc;
    if ((rc = timing_end(p, s))) return rc;
  } else {
    const void** avg = xbd;
    if (!avg) {
      if ((rc = scratch_xbar_table(p, s, &avg))) return rc;
      if ((rc = timing_begin(p, DPPF_K_MEAN, s))) return rc;
      if ((rc = launch_mean_any(p, xd, avg, s))) return rc;
      if ((rc = timing_end(p, s))) return rc;
    }
    if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
    for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
      const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
      if ((rc = launch_sweep1<false, 2, true>(p, mg, xd, nullptr, nullptr, avg, 0, 0, 0, m0, kKeepNone, &shape, s))) return rc;
    }
    if ((rc = timing_end(p, s))) return rc;
  }
  return launch_finalize(p, shape.nparts(), 0.f, 0.f, false, r_out, nullptr, s);
} DPPF_CATCH

int dppf_pull_push_round(dppf_plan* p, float* const* x, float pull, float push, float* r_out,
                         float* c_out, float* const* xbar_out, void* stream) try {
  return round_impl(p, false, x, nullptr, nullptr, 0.f, 0.f, 0.f, pull, push, r_out, c_out, xbar_out,
                    static_cast<hipStream_t>(stream));
} DPPF_CATCH

int dppf_local_sgd_step(dppf_plan* p, float* const* x, float* const* v, const float* const* g, float lr,
                        float momentum, float weight_decay, void* stream) try {
  if (!p || !x || !v || !g) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = static_cast<size_t>(p->M) * p->T;
  const void **xd = nullptr, **vd = nullptr, **gd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x), n, s, &xd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RV, reinterpret_cast<const void* const*>(v), n, s, &vd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RG, reinterpret_cast<const void* const*>(g), n, s, &gd))) return rc;
  if (p->ntiles == 0) return DPPF_OK;
  return launch_local_step(p, xd, vd, gd, lr, momentum, weight_decay, s);
} DPPF_CATCH

int dppf_round(dppf_plan* p, float* const* x, float* const* v, const float* const* g, float lr,
               float momentum, float weight_decay, float pull, float push, float* r_out, float* c_out,
               float* const* xbar_out, void* stream) try {
  return round_impl(p, true, x, v, g, lr, momentum, weight_decay, pull, push, r_out, c_out, xbar_out,
                    static_cast<hipStream_t>(stream));
} DPPF_CATCH

int dppf_pull_push_round_exact(dppf_plan* p, float* const* x, float pull, float push_r, float* r_out,
                               float* c_out, void* stream) try {
  if (!p || !x) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const void** xd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x),
                         static_cast<size_t>(p->M) * p->T, s, &xd)))
    return rc;
  if (p->ntiles == 0) return launch_finalize(p, 0, pull, push_r / static_cast<float>(p->M), false, r_out, c_out, s);
  GridShape shape;
  if (p->M > kMaxTemplM) {
    // stored average -> distances per group -> coefficients and 1/r -> stored sum of unit gap
    // vectors -> update per group
    const float mf = static_cast<float>(p->M);
    const void **avg = nullptr, **usum = nullptr;
    if ((rc = scratch_xbar_table(p, s, &avg))) return rc;
    if ((rc = scratch_usum_table(p, s, &usum))) return rc;
    if ((rc = timing_begin(p, DPPF_K_MEAN, s))) return rc;
    if ((rc = launch_mean_any(p, xd, avg, s))) return rc;
    if ((rc = timing_end(p, s))) return rc;
    if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
    for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
      const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
      if ((rc = launch_sweep1<false, 2, true>(p, mg, xd, nullptr, nullptr, avg, 0, 0, 0, m0, kKeepNone, &shape, s)))
        return rc;
    }
    if ((rc = timing_end(p, s))) return rc;
    if ((rc = launch_finalize(p, shape.nparts(), pull, push_r / mf, true, r_out, c_out, s))) return rc;
    if ((rc = timing_begin(p, DPPF_K_UPDATE_EXACT, s))) return rc;
    int grid = 0, gfull = 0;
    if ((rc = grid_for(p, k_unit_sum_any, 1, kBlocksPerCUReadOnly, &gfull, &grid))) return rc;
    hipLaunchKernelGGL(k_unit_sum_any, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kEvenSplit, 0.0),
                       p->M, p->T, (float* const*)(xd), (const float* const*)(avg), p->coef, (float* const*)(usum));
    HIP_TRY(hipGetLastError());
    for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
      const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
      float* const* xg = (float* const*)(xd) + static_cast<size_t>(m0) * p->T;
      DPPF_SWITCH_M(mg, {
        constexpr int kU = unroll_plain(kM) > 2 ? 2 : unroll_plain(kM);
        auto kern = k_update_exact_given<kM, kU>;
        if ((rc = grid_for(p, kern, 1, kBlocksPerCUReadWrite, &gfull, &grid))) return rc;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, make_walk(p, gfull, 1, 1, kOnDemand, 8.0 * mg + 8.0), p->T, xg,
                           (const float* const*)(avg), (const float* const*)(usum), p->coef + m0, push_r / (mf * mf));
      })
      HIP_TRY(hipGetLastError());
    }
    return timing_end(p, s);
  }
  if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
  if ((rc = launch_sweep1<false, 0, true>(p, p->M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepTail, &shape, s))) return rc;
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_UPDATE_EXACT, s))) return rc;
  if ((rc = launch_update_exact(p, xd, shape.nparts(), pull, push_r, r_out, c_out, s))) return rc;
  return timing_end(p, s);
} DPPF_CATCH

int dppf_pull_then_push(dppf_plan* p, float* const* x, const float* const* x_c, float pull, float push,
                        int push_from, float* r_post_out, void* stream) try {
  if (!p || !x || !x_c || (push_from != DPPF_PUSH_FROM_AVERAGE && push_from != DPPF_PUSH_FROM_CONSENSUS))
    return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const void **xd = nullptr, **xcd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x),
                         static_cast<size_t>(p->M) * p->T, s, &xd)))
    return rc;
  if ((rc = table_upload(p, dppf_plan::RXC, reinterpret_cast<const void* const*>(x_c),
                         static_cast<size_t>(p->T), s, &xcd)))
    return rc;
  if (p->ntiles == 0) return launch_finalize(p, 0, 0.f, 0.f, false, r_post_out, nullptr, s);
  if (push_from == DPPF_PUSH_FROM_CONSENSUS) return run_seq<1>(p, xd, xcd, nullptr, pull, push, r_post_out, s);
  if (p->M <= kMaxTemplM) return run_seq<0>(p, xd, xcd, nullptr, pull, push, r_post_out, s);
  // more workers than one kernel sees at once: the pre-round average is stored first
  const void** avg = nullptr;
  if ((rc = scratch_xbar_table(p, s, &avg))) return rc;
  if ((rc = timing_begin(p, DPPF_K_MEAN, s))) return rc;
  if ((rc = launch_mean_any(p, xd, avg, s))) return rc;
  if ((rc = timing_end(p, s))) return rc;
  return run_seq<2>(p, xd, xcd, avg, pull, push, r_post_out, s);
} DPPF_CATCH

int dppf_local_adamw_step(dppf_plan* p, float* const* x, float* const* m1, float* const* m2,
                          const float* const* g, float lr, float beta1, float beta2, float eps,
                          float weight_decay, int64_t step, void* stream) try {
  if (!p || !x || !m1 || !m2 || !g || step < 1) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = static_cast<size_t>(p->M) * p->T;
  const void **xd = nullptr, **ad = nullptr, **sd = nullptr, **gd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x), n, s, &xd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RM1, reinterpret_cast<const void* const*>(m1), n, s, &ad))) return rc;
  if ((rc = table_upload(p, dppf_plan::RM2, reinterpret_cast<const void* const*>(m2), n, s, &sd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RG, reinterpret_cast<const void* const*>(g), n, s, &gd))) return rc;
  if (p->ntiles == 0) return DPPF_OK;
  const AdamHyper hp = adam_hyper(lr, beta1, beta2, eps, weight_decay, step);
  return launch_adamw_step(p, xd, ad, sd, gd, hp, s);
} DPPF_CATCH

int dppf_round_adamw(dppf_plan* p, float* const* x, float* const* m1, float* const* m2, const float* const* g,
                     float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step, float pull,
                     float push, float* r_out, float* c_out, void* stream) try {
  if (!p || !x || !m1 || !m2 || !g || step < 1) return DPPF_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = static_cast<size_t>(p->M) * p->T;
  const void **xd = nullptr, **ad = nullptr, **sd = nullptr, **gd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x), n, s, &xd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RM1, reinterpret_cast<const void* const*>(m1), n, s, &ad))) return rc;
  if ((rc = table_upload(p, dppf_plan::RM2, reinterpret_cast<const void* const*>(m2), n, s, &sd))) return rc;
  if ((rc = table_upload(p, dppf_plan::RG, reinterpret_cast<const void* const*>(g), n, s, &gd))) return rc;
  if (p->ntiles == 0) return launch_finalize(p, 0, pull, push, true, r_out, c_out, s);
  const AdamHyper hp = adam_hyper(lr, beta1, beta2, eps, weight_decay, step);
  if (p->M > kMaxTemplM) {   // no register-resident kernel for this many workers: step, then the round
    if ((rc = launch_adamw_step(p, xd, ad, sd, gd, hp, s))) return rc;
    return round_impl(p, false, x, nullptr, nullptr, 0.f, 0.f, 0.f, pull, push, r_out, c_out, nullptr, s);
  }
  GridShape shape;
  if ((rc = timing_begin(p, DPPF_K_ADAMW_REDUCE, s))) return rc;
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_fused(kM);
    auto kern = k_adamw_reduce<kM, kU>;
    int gfull = 0;
    if ((rc = grid_for(p, kern, 1, kBlocksPerCUReadWrite, &gfull, &shape.grid))) return rc;
    shape.walk = make_walk(p, gfull, 1, 1, kOnDemandReducing, 28.0 * p->M);
    hipLaunchKernelGGL(kern, dim3(shape.grid), dim3(kBlock), 0, s, p->tiles_dev, shape.walk, p->T,
                       (float* const*)(xd), (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp,
                       p->partials, p->M);
  })
  HIP_TRY(hipGetLastError());
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_UPDATE, s))) return rc;
  if ((rc = launch_sweep2<0, false, true>(p, p->M, xd, nullptr, nullptr, 0.f, 0, shape.nparts(), pull, push, r_out,
                                          c_out, s)))
    return rc;
  return timing_end(p, s);
} DPPF_CATCH

int dppf_round_statistics(const float* r, int M, float pull, float push, float* out, void* stream) {
  if (!r || !out || M < 1 || M > DPPF_MAX_WORKERS) return DPPF_EINVAL;
  hipLaunchKernelGGL(k_round_stats, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), r, M, pull, push, out);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

float dppf_push_schedule(int kind, float push, int64_t t, int64_t t_total) {
  const double kPi = 3.14159265358979323846;
  const double frac = (t_total > 0) ? static_cast<double>(t) / static_cast<double>(t_total) : 0.0;
  switch (kind) {
    case DPPF_SCHEDULE_DECREASING: return static_cast<float>(0.5 * push * (1.0 + std::cos(kPi * frac)));
    case DPPF_SCHEDULE_INCREASING: return static_cast<float>(0.5 * push * (1.0 - std::cos(kPi * frac)));
    default: return push;
  }
}

// ---- flat forms (T == 1): build the M-entry tables on the stack of the call
static int flat_check(const dppf_plan* p, const void* base, int64_t ld) {
  if (!p || p->T != 1 || !base || ld < p->d) return DPPF_EINVAL;
  return DPPF_OK;
}

int dppf_pull_push_round_flat(dppf_plan* p, float* x, int64_t ld, float pull, float push, float* r_out,
                              float* c_out, float* xbar_out, void* stream) try {
  int rc = flat_check(p, x, ld);
  if (rc) return rc;
  std::vector<float*> xt(static_cast<size_t>(p->M));
  for (int m = 0; m < p->M; ++m) xt[m] = x + static_cast<long long>(m) * ld;
  float* xb[1] = {xbar_out};
  return dppf_pull_push_round(p, xt.data(), pull, push, r_out, c_out, xbar_out ? xb : nullptr, stream);
} DPPF_CATCH

int dppf_local_sgd_step_flat(dppf_plan* p, float* x, float* v, const float* g, int64_t ld, float lr,
                             float momentum, float weight_decay, void* stream) try {
  int rc = flat_check(p, x, ld);
  if (rc) return rc;
  if (!v || !g) return DPPF_EINVAL;
  std::vector<float*> xt(p->M), vt(p->M);
  std::vector<const float*> gt(p->M);
  for (int m = 0; m < p->M; ++m) {
    xt[m] = x + static_cast<long long>(m) * ld;
    vt[m] = v + static_cast<long long>(m) * ld;
    gt[m] = g + static_cast<long long>(m) * ld;
  }
  return dppf_local_sgd_step(p, xt.data(), vt.data(), gt.data(), lr, momentum, weight_decay, stream);
} DPPF_CATCH

int dppf_round_flat(dppf_plan* p, float* x, float* v, const float* g, int64_t ld, float lr, float momentum,
                    float weight_decay, float pull, float push, float* r_out, float* c_out, float* xbar_out,
                    void* stream) try {
  int rc = flat_check(p, x, ld);
  if (rc) return rc;
  if (!v || !g) return DPPF_EINVAL;
  std::vector<float*> xt(p->M), vt(p->M);
  std::vector<const float*> gt(p->M);
  for (int m = 0; m < p->M; ++m) {
    xt[m] = x + static_cast<long long>(m) * ld;
    vt[m] = v + static_cast<long long>(m) * ld;
    gt[m] = g + static_cast<long long>(m) * ld;
  }
  float* xb[1] = {xbar_out};
  return dppf_round(p, xt.data(), vt.data(), gt.data(), lr, momentum, weight_decay, pull, push, r_out,
                    c_out, xbar_out ? xb : nullptr, stream);
} DPPF_CATCH

// ---- the plain round on one flat buffer, for callers that may not allocate
// This device's copy of the static scratch array and its CU count, looked up once per device.
static int static_scratch_base(int device, unsigned char** base, int* num_cu) {
  if (device < 0 || device >= kMaxDevices) return DPPF_ELIMIT;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  DeviceState& dev = g_device[device];
  if (!dev.static_scratch) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)));   // of the CURRENT device
    if (!ptr) return DPPF_EHIP;
    dev.static_scratch = static_cast<unsigned char*>(ptr);
  }
  if (dev.num_cu == 0)
    HIP_TRY(hipDeviceGetAttribute(&dev.num_cu, hipDeviceAttributeMultiprocessorCount, device));
  *base = dev.static_scratch;
  *num_cu = dev.num_cu;
  return DPPF_OK;
}

int dppf_pull_push_round_flat_static(float* x, int M, int64_t d, int64_t ld, float pull, float push,
                                     float* r_out, float* c_out, void* stream) try {
  if (M < 1 || d < 0 || ld < d || (d > 0 && !x)) return DPPF_EINVAL;
  if (reinterpret_cast<uintptr_t>(x) & 3u) return DPPF_EINVAL;
  if (M > kStaticMaxWorkers || d > kStaticMaxDim) return DPPF_ELIMIT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int device = -1, num_cu = 0, rc;
  HIP_TRY(hipGetDevice(&device));
  unsigned char* base = nullptr;
  if ((rc = static_scratch_base(device, &base, &num_cu))) return rc;
  if (num_cu < 1 || num_cu * kMaxBlocksPerCU > kStaticMaxRows) return DPPF_ELIMIT;
  // a plan-shaped view of the static scratch: nothing in it is owned, nothing is allocated
  dppf_plan view;
  view.M = M;
  view.T = 1;
  view.device = device;
  view.num_cu = num_cu;
  view.d = d;
  view.nfull = static_cast<int>(d / kTileElems);
  view.ntiles = view.nfull + (d % kTileElems ? 1 : 0);
  view.tiles_dev = reinterpret_cast<Tile*>(base + kStaticOffTiles);
  view.partials = reinterpret_cast<double*>(base + kStaticOffPartials);
  view.partials_rows = kStaticMaxRows * kStaticMaxWorkers / M;
  view.sched = reinterpret_cast<Sched*>(base + kStaticOffSched);
  view.coef = reinterpret_cast<Coef*>(base + kStaticOffCoef);
  const void** xd = reinterpret_cast<const void**>(base + kStaticOffPtrs);
  // the tile list, the pointer table and a clean counter are written by a kernel (no copy from
  // host memory, no memset: both would be foreign bodies in a captured graph)
  int setup_blocks = (view.ntiles + kBlock - 1) / kBlock;
  if (setup_blocks < 1) setup_blocks = 1;
  if (setup_blocks > num_cu) setup_blocks = num_cu;
  hipLaunchKernelGGL(k_flat_setup, dim3(setup_blocks), dim3(kBlock), 0, s, view.tiles_dev, static_cast<long long>(d),
                     (float**)(xd), x, static_cast<long long>(ld), M, view.sched);
  HIP_TRY(hipGetLastError());
  if (view.ntiles == 0) return launch_finalize(&view, 0, pull, push, true, r_out, c_out, s);
  GridShape shape;
  if ((rc = launch_sweep1<false, 0, true>(&view, M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepTail, &shape, s)))
    return rc;
  return launch_sweep2<0, false, true>(&view, M, xd, nullptr, nullptr, 0.f, 0, shape.nparts(), pull, push, r_out,
                                       c_out, s);
} DPPF_CATCH

// ---- plain device-to-device copy of n floats with the library's own load/store path
int dppf_util_copy(float* dst, const float* src, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!dst || !src))) return DPPF_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dst) & 3u) || (reinterpret_cast<uintptr_t>(src) & 3u)) return DPPF_EINVAL;
  if (n == 0) return DPPF_OK;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  int cus = 0;
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  long long blocks = (n / 4 + kBlock - 1) / kBlock;
  const long long cap = static_cast<long long>(cus) * kBlocksPerCUReadWrite;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_copy, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), dst, src, static_cast<long long>(n));
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

// ---- streaming probe (measurement aid)
int dppf_util_stream_probe(float* base, int64_t stride, int64_t n, int reads, int writes, int inplace,
                           int blocks_per_cu, int on_demand, void* stream) {
  if (!base || n < 0 || stride < n || blocks_per_cu < 1 || blocks_per_cu > 16) return DPPF_EINVAL;
  if (reinterpret_cast<uintptr_t>(base) & 15u || (stride & 3)) return DPPF_EINVAL;
  if (n / 1024 >= INT32_MAX) return DPPF_ELIMIT;
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  Sched* sched = nullptr;   // this device's copy of the probe's counter
  HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&sched), HIP_SYMBOL(g_probe_sched)));
  const dim3 grid(static_cast<unsigned>(cus * blocks_per_cu)), block(kBlock);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* sink = base;   // never written unless a sum hits one magic value
#define DPPF_PROBE(R_, W_, U_, IP_)                                                              \
  if (reads == R_ && writes == W_ && (inplace != 0) == IP_) {                                    \
    const long long tiles_ = n / (static_cast<long long>(kBlock) * U_ * 4);                      \
    const long long items_ = (tiles_ + kProbeItemTiles - 1) / kProbeItemTiles;                   \
    Walk walk_;                                                                                  \
    walk_.nfull = walk_.ntiles = walk_.nitems = static_cast<int>(items_);                        \
    walk_.gfull = static_cast<int>(grid.x);                                                      \
    walk_.nstatic = static_cast<int>(                                                            \
        evenly_split_items(items_, walk_.gfull, on_demand ? kOnDemand : kEvenSplit,              \
                           4.0 * kProbeItemTiles * kBlock * U_ * 4 * (R_ + W_)));                \
    walk_.sched = walk_.nstatic < items_ ? sched : nullptr;                                      \
    hipLaunchKernelGGL((k_probe<R_, W_, U_, IP_>), grid, block, 0, s, base, static_cast<long long>(stride), \
                       static_cast<long long>(n), sink, walk_);                                  \
    HIP_TRY(hipGetLastError());                                                                  \
    return DPPF_OK;                                                                              \
  }
  DPPF_PROBE(1, 0, 4, false)
  DPPF_PROBE(4, 0, 4, false)
  DPPF_PROBE(12, 0, 1, false)
  DPPF_PROBE(0, 1, 4, false)
  DPPF_PROBE(0, 4, 4, false)
  DPPF_PROBE(1, 1, 4, false)
  DPPF_PROBE(2, 1, 4, false)
  DPPF_PROBE(4, 4, 2, false)
  DPPF_PROBE(4, 4, 2, true)
  DPPF_PROBE(8, 4, 1, false)
  DPPF_PROBE(8, 4, 1, true)
  DPPF_PROBE(12, 4, 1, false)
  DPPF_PROBE(12, 4, 1, true)
  DPPF_PROBE(12, 8, 1, false)
  DPPF_PROBE(12, 8, 1, true)
  DPPF_PROBE(16, 8, 1, true)
  DPPF_PROBE(24, 8, 1, true)
#undef DPPF_PROBE
  return DPPF_EINVAL;   // this read/write mix is not instantiated
}

// ---- timing
int dppf_plan_timing_enable(dppf_plan* p, int enable) {
  if (!p) return DPPF_EINVAL;
  p->timing = enable != 0;
  return DPPF_OK;
}

int dppf_plan_timing_read(dppf_plan* p, int* kernel_id, float* ms, int cap) try {
  if (!p || cap < 0 || (cap > 0 && (!kernel_id || !ms))) return DPPF_EINVAL;
  // A bracket whose launch failed half way has no recorded stop event: such a record is dropped.
  // Every record leaves the list whatever happens, so no event is ever handed out twice.
  int n = 0, failed = 0;
  for (auto& r : p->recs) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
    if (e != hipSuccess) {
      g_last_hip_error = static_cast<int>(e);
      ++failed;
    } else if (n < cap) {
      kernel_id[n] = r.id;
      ms[n] = t;
      ++n;
    }
    p->event_pool.push_back(r.start);
    p->event_pool.push_back(r.stop);
  }
  p->recs.clear();
  if (failed) (void)hipGetLastError();   // the unreadable records are gone; leave no sticky error behind
  return n;
} DPPF_CATCH

}  // extern "C"
