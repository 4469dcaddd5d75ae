// Host-side internals shared by the translation units of the DPPF library: the plan, the
// per-device state, and the launchers each unit exports for the C ABI in dppf_api.hip.
#ifndef DPPF_INTERNAL_H_
#define DPPF_INTERNAL_H_

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "dppf.h"
#include "dppf_kernels.h"

namespace dppf_detail {

extern thread_local int g_last_hip_error;

#define HIP_TRY(expr)                                               \
  do {                                                              \
    hipError_t e__ = (expr);                                        \
    if (e__ != hipSuccess) {                                        \
      dppf_detail::g_last_hip_error = static_cast<int>(e__);        \
      return DPPF_EHIP;                                             \
    }                                                               \
  } while (0)

// A device copy of a host pointer table, refreshed only when the host contents change.
struct PtrTable {
  std::vector<const void*> host;   // what the device copy currently holds
  const void** staging = nullptr;  // pinned, source of the async upload
  const void** dev = nullptr;
  hipEvent_t uploaded = nullptr;   // marks the end of the last upload from `staging`
  hipStream_t upload_stream = nullptr;   // the stream that upload was enqueued on
  size_t cap = 0;
  bool valid = false;
};

struct TimingRec {
  int id;
  hipEvent_t start, stop;
};

// A tensor list cut into tiles of one size, in device memory.
struct TileList {
  Tile* dev = nullptr;
  int nfull = 0;        // tiles [0, nfull) are full, [nfull, ntiles) partial
  int ntiles = 0;
  int tile_elems = 0;
};

// What the library remembers per device for the life of the process, in fixed-size storage (the
// entry point that must not allocate uses it too): resident blocks per CU of every kernel that has
// been launched there, the kernels whose dynamic-LDS limit has been raised, and the address of that
// device's copy of the static scratch array.
constexpr int kMaxDevices = 64;
constexpr int kOccupancySlots = 1024;
struct DeviceState {
  int num_cu = 0;
  int nocc = 0;
  const void* occ_kernel[kOccupancySlots];   // key: kernel, block size, dynamic LDS bytes
  int occ_threads[kOccupancySlots];
  size_t occ_lds[kOccupancySlots];
  int occ_per_cu[kOccupancySlots];
  unsigned char* static_scratch = nullptr;
};
extern DeviceState g_device[kMaxDevices];
extern std::mutex g_device_mutex;

}  // namespace dppf_detail

struct dppf_plan {
  int M = 0, T = 0;
  int device = 0;
  int num_cu = 0;
  long long d = 0;
  std::vector<long long> numel;
  // `step` holds tiles of kStepTileElems elements (kernels that take one worker at a time, any-M
  // streaming kernels); `sweep` holds tiles of sweep_tile_elems(M) elements (the sweeps that take
  // all workers of a tile together).  They are the same list when the two sizes agree.
  dppf_detail::TileList step, sweep;
  // partial sums, stored column by column: [M + 1][partials_rows]; one row per block, then one per
  // on-demand item of the reducing launch
  double* partials = nullptr;
  int partials_rows = 0;
  dppf_walk::Sched* sched = nullptr;   // the counter behind the on-demand part of a kernel's tile walk
  dppf_detail::Coef* coef = nullptr;   // [M]
  float* avg_norm = nullptr;           // ||x_A|| of the most recent round
  float* xbar_scratch = nullptr;            // d floats, only when M > kMaxTemplM
  float* usum_scratch = nullptr;            // d floats, only when M > kMaxLdsM (exact update)
  std::vector<long long> tensor_offset;     // start of tensor t inside xbar_scratch
  enum Role { RX = 0, RV, RG, RM1, RM2, RXBAR, RXBAR_SCRATCH, RUSUM_SCRATCH, RXC, NROLES };
  dppf_detail::PtrTable tab[NROLES];
  // timing
  bool timing = false;
  std::vector<dppf_detail::TimingRec> recs;
  std::vector<hipEvent_t> event_pool;

  int cols() const { return M + 1; }   // columns of the partial sums: the M squared distances, ||x_A||^2
};

namespace dppf_detail {

using dppf_walk::OnDemand;

int timing_begin(dppf_plan* p, int id, hipStream_t s);
int timing_end(dppf_plan* p, hipStream_t s);

// The launch shape of a reducing sweep: the launch that reads the partial sums must know how many
// rows the reducing launch filled.
struct GridShape {
  int grid = 0;
  Walk walk{};
  int nparts() const { return grid + (walk.nitems - walk.nstatic); }
};

// Resident blocks per CU of a kernel on the plan's device (queried once per device and kernel).
int blocks_per_cu(int device, const void* kernel, int block_threads, size_t dynamic_lds, int* per_cu);

// ---- grid sizes: enough resident blocks to fill every CU, never more blocks than items
template <typename K>
int grid_for(dppf_plan* p, const TileList& list, K kernel, int per_tile_items, int tiles_per_item, int want_per_cu,
             size_t dynamic_lds, int* gfull_out, int* grid_out, int block_threads = kBlock) {
  int per_cu = 0;
  const int rc =
      blocks_per_cu(p->device, reinterpret_cast<const void*>(kernel), block_threads, dynamic_lds, &per_cu);
  if (rc) return rc;
  if (per_cu > want_per_cu) per_cu = want_per_cu;
  if (per_cu > kMaxBlocksPerCU - 1) per_cu = kMaxBlocksPerCU - 1;
  const long long full_items =
      static_cast<long long>(dppf_walk::worker_item_groups(list.nfull, tiles_per_item)) * per_tile_items;
  const long long part_items = static_cast<long long>(list.ntiles - list.nfull) * per_tile_items;
  dppf_walk::grid_shape(p->num_cu, per_cu, full_items, part_items, gfull_out, grid_out);   // <= num_cu * kMaxBlocksPerCU
  return DPPF_OK;
}

inline Walk plan_walk(const dppf_plan* p, const TileList& list, int gfull, int workers_per_tile, int tiles_per_item,
                      OnDemand policy, double bytes_per_elem) {
  return dppf_walk::make_walk(list.nfull, list.ntiles, list.tile_elems, gfull, workers_per_tile, tiles_per_item,
                              policy, bytes_per_elem, p->sched);
}

// Which of sweep 1's x loads go through the caches (see k_sweep1).
enum KeepPolicy {
  kKeepTail,     // only the tiles touched last, as many as fit the last-level cache budget
  kKeepNone      // nothing reads x again soon
};

constexpr long long kLastLevelCacheBudget = 256ll << 20;   // bytes of x worth keeping (the cache is 256 MB)

// First tile of the sweep list whose x loads go through the caches in sweep 1.
inline int keep_from_tile(const dppf_plan* p, KeepPolicy keep) {
  if (keep == kKeepNone) return p->sweep.nfull;
  const long long per_tile = static_cast<long long>(p->M) * p->sweep.tile_elems * sizeof(float);
  const long long tiles = kLastLevelCacheBudget / per_tile;
  return tiles >= p->sweep.nfull ? 0 : p->sweep.nfull - static_cast<int>(tiles);
}

// Rows of partial sums a reducing launch of this shape fills; they must fit the plan's buffer.
inline bool rows_fit(const dppf_plan* p, int grid, const Walk& walk) {
  return grid + (walk.nitems - walk.nstatic) <= p->partials_rows;
}

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
    case 10: { constexpr int kM = 10; __VA_ARGS__ } break;         \
    case 11: { constexpr int kM = 11; __VA_ARGS__ } break;         \
    case 12: { constexpr int kM = 12; __VA_ARGS__ } break;         \
    case 13: { constexpr int kM = 13; __VA_ARGS__ } break;         \
    case 14: { constexpr int kM = 14; __VA_ARGS__ } break;         \
    case 15: { constexpr int kM = 15; __VA_ARGS__ } break;         \
    case 16: { constexpr int kM = 16; __VA_ARGS__ } break;         \
    default: return DPPF_ELIMIT;                                   \
  }

// U = 16-byte vectors of one worker that a lane handles per pass over a tile.  A lane keeps M*U
// vectors of x; the fused sweeps add one worker's v and g (or AdamW's three) at a time.  With one
// block per CU a lane may use the whole 512-entry register file; the values are the fastest
// measured per range of M (never more than a tile holds per lane).
constexpr int at_most_tile(int u, int M) {
  return u < vectors_per_lane(sweep_tile_elems(M)) ? u : vectors_per_lane(sweep_tile_elems(M));
}
constexpr int unroll_plain(int M) { return at_most_tile(M <= 4 ? 4 : 2, M); }
constexpr int unroll_step_update(int M) { return at_most_tile(M <= 4 ? 4 : 2, M); }
constexpr int unroll_fused(int M) { return at_most_tile(M <= 8 ? 4 : 2, M); }
constexpr int unroll_seq(int M) { return at_most_tile(unroll_plain(M) > 2 ? 2 : unroll_plain(M), M); }

// ------------------------------------------------------------------ launchers, by unit
// All take DEVICE pointer tables (the plan's copies).  Every launcher returns DPPF_OK or an error
// code and has enqueued nothing on error.

// dppf_launch_reduce.hip -- M <= 16, sweep 1 without a folded step
//   store_avg: also write x_A to xbarp; norms: accumulate the squared distances (rows of partial sums)
int launch_reduce(dppf_plan* p, const void** xp, const void** xbarp, bool store_avg, bool norms, KeepPolicy keep,
                  GridShape* shape, hipStream_t s);
// dppf_launch_step_reduce.hip -- M <= 16, sweep 1 with the momentum-SGD step folded in
int launch_step_reduce(dppf_plan* p, const void** xp, const void** vp, const void** gp, const void** xbarp,
                       bool store_avg, float lr, float mu, float wd, GridShape* shape, hipStream_t s);
// dppf_launch_update.hip -- M <= 16, sweep 2 (coefficients folded from `nparts` rows of partial sums)
//   fold: every block derives the coefficients itself from the rows of partial sums (and block 0
//   writes r_out, c_out and the norm of the average); otherwise they are read from the plan's
//   coefficient buffer, which a finalize launch has filled
int launch_update(dppf_plan* p, const void** xp, const void** vp, bool step, bool fold, float lr, int nparts,
                  float pull, float push, float* r_out, float* c_out, hipStream_t s);
// whether reading `nparts` rows in every block of sweep 2 is still cheaper than a finalize launch
bool fold_pays(int nparts);
int launch_update_exact(dppf_plan* p, const void** xp, int nparts, float pull, float push_r, float* r_out,
                        float* c_out, hipStream_t s);
// dppf_launch_seq.hip -- M <= 16, Alg. 1 literally; from_consensus: push away from x_C, else from x_A
int launch_seq_reduce(dppf_plan* p, const void** xp, const void** xcp, bool from_consensus, float pull,
                      GridShape* shape, hipStream_t s);
int launch_seq_update(dppf_plan* p, const void** xp, const void** xcp, bool from_consensus, float pull, float push,
                      int nparts, float* r_post_out, hipStream_t s);
// dppf_launch_adamw.hip
int launch_adamw_step(dppf_plan* p, const void** xd, const void** ad, const void** sd, const void** gd,
                      const AdamHyper hp, hipStream_t s);
int launch_adamw_reduce(dppf_plan* p, const void** xd, const void** ad, const void** sd, const void** gd,
                        const AdamHyper hp, GridShape* shape, hipStream_t s);
// dppf_launch_misc.hip
int launch_local_step(dppf_plan* p, const void** xp, const void** vp, const void** gp, float lr, float mu, float wd,
                      hipStream_t s);
//   want_avg_norm: column M of the partial sums holds the squared norm of the average; its root goes
//   to the plan's slot for ||x_A||
int launch_finalize(dppf_plan* p, int nparts, float pull, float push, bool want_coef, bool want_avg_norm,
                    float* r_out, float* c_out, hipStream_t s);
int launch_round_stats(const float* r, int M, float pull, float push, const float* avg_norm, float* out,
                       hipStream_t s);
int launch_copy_scalar(const float* src, float* dst, hipStream_t s);
int launch_flat_setup(Tile* tiles, long long d, int tile_elems, int ntiles, int num_cu, float** ptrs, float* x,
                      long long ld, int M, Sched* sched, hipStream_t s);
int launch_copy(float* dst, const float* src, int64_t n, hipStream_t s);
int launch_stream_probe(float* base, int64_t stride, int64_t n, int reads, int writes, int inplace,
                        int blocks_per_cu, int on_demand, hipStream_t s);
int launch_stream_probe_grouped(float* base, int64_t stride, int64_t n, int groups, int reads_per_group,
                                int vectors, int ahead, int blocks_per_cu, int on_demand, hipStream_t s);
// dppf_launch_any.hip -- any M, stored average
int launch_mean_any(dppf_plan* p, const void** xp, const void** xbarp, hipStream_t s);
int launch_norms_any(dppf_plan* p, const void** xp, const void** xbarp, GridShape* shape, hipStream_t s);
int launch_update_any(dppf_plan* p, const void** xp, const void** xbarp, const void** sump, bool exact, float k2,
                      hipStream_t s);
int launch_unit_sum_any(dppf_plan* p, const void** xp, const void** xbarp, const void** sump, hipStream_t s);
//   ref_is_consensus: push away from x_C, else away from the stored average refp
int launch_seq_any(dppf_plan* p, const void** xp, const void** xcp, const void** refp, bool ref_is_consensus,
                   bool write, float pull, GridShape* shape, hipStream_t s);
// dppf_launch_lds.hip -- 17 <= M <= 39, staged in LDS
//   opt: 0 none, 1 momentum SGD (o.vp, o.gp, lr, mu, wd), 2 AdamW (o.vp, o.sp, o.gp, o.adam)
int launch_sweep1_lds(dppf_plan* p, const void** xp, int opt, const LdsOptArgs& o, const void** xbarp,
                      bool store_avg, GridShape* shape, hipStream_t s);
//   mode: 0 Eq. 5, 1 Eq. 5 on x - lr v, 2 the exact two-term update (k2 = lambda_r / M^2)
int launch_sweep2_lds(dppf_plan* p, const void** xp, const void** vp, int mode, float lr, float k2, hipStream_t s);

}  // namespace dppf_detail

#endif  // DPPF_INTERNAL_H_
