// DPPF consensus round and local step for MI355X (gfx950, wave64): the plan and the C ABI.
//
// The work is bandwidth-bound streaming over the M workers' parameter tensors, so the design
// is about bytes and about what the memory system likes, not about flops:
//   * the round is two sweeps over x, because the per-worker coefficient alpha - lambda/r_m
//     (Sec. 5, Eq. 5) needs r_m, a reduction over the whole model, before any element moves:
//     sweep 1 reads x once (average kept on chip, squared distances accumulated into partial
//     sums), sweep 2 turns the partial sums into the coefficients, reads x again, recomputes the
//     average from the same M loads and writes x.  12 bytes per replica-parameter.
//   * the fused form folds the last local step (Alg. 1, SGD line) into sweep 1 and never stores
//     the stepped x: sweep 1 reads x, v, g and writes only v; sweep 2 reads the OLD x and the NEW
//     v, rebuilds x - lr v with the same fused multiply-add (same bits) and applies Eq. 5.
//     28 bytes instead of 32, and 20 of them reads (reads stream faster than writes here).
//   * a tensor list is cut into tiles of consecutive elements of one tensor; a fixed number of
//     thread blocks (one or two per CU) walks the tile list, so one launch covers any number of
//     tensors of any size.  Full tiles and partial ones (tensor tails, small tensors) are walked
//     by different blocks.  Loads are 16-byte vectors with 4-byte alignment (legal for global
//     memory on gfx9), so no tensor needs 16-byte alignment; only the last, partial vector of a
//     tensor is handled element by element.
//   * up to 16 workers all replicas of a lane's elements sit in registers; up to 39 they are staged
//     in LDS; beyond that the average is stored once and streamed back (see dppf_kernels.h).
//   * the chip's compute dies do not stream at the same rate, so an even split of the tiles leaves
//     the faster ones idle at the end: the read-write sweeps hand part or all of their tiles out on
//     demand from a counter (see dppf_walk.h).  Partial sums are kept per block for the even part
//     and per tile for the on-demand part, so the result does not depend on which block took which
//     tile.
//   * the gap of a worker to the average is formed relative to worker 0 (see mean_offset), so it
//     keeps full relative precision and is exactly zero for identical replicas.
//   * squared distances: fp32 inside a tile, fp64 across tiles, lanes, waves and blocks, in a
//     fixed order -- results are bit-reproducible run to run.
//   * sweep 2 walks the tiles in the opposite order to sweep 1, so that the part of x that
//     sweep 1 touched last is still in the last-level cache when sweep 2 starts.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <utility>

#include "dppf_internal.h"
#include "dppf_util.h"

static_assert(dppf_detail::kMaxTemplM == DPPF_STATIC_MAX_WORKERS, "the header documents the static entry point's limit");

namespace dppf_detail {

thread_local int g_last_hip_error = 0;
DeviceState g_device[kMaxDevices];
std::mutex g_device_mutex;

// The LDS-staged kernels ask for more dynamic LDS than the default limit allows; the limit is
// raised once per kernel and device, to the most any worker count needs.
constexpr size_t kRaiseLdsLimitFrom = 32 * 1024;
constexpr size_t kLdsLimitBytes =
    static_cast<size_t>(kMaxLdsM) * kBlock * sizeof(f4) + sizeof(double) * kWaves * (kMaxLdsM + 1);

int blocks_per_cu(int device, const void* kernel, int block_threads, size_t dynamic_lds, int* per_cu_out) {
  if (device < 0 || device >= kMaxDevices) return DPPF_ELIMIT;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  DeviceState& dev = g_device[device];
  for (int i = 0; i < dev.nocc; ++i)
    if (dev.occ_kernel[i] == kernel && dev.occ_threads[i] == block_threads && dev.occ_lds[i] == dynamic_lds) {
      *per_cu_out = dev.occ_per_cu[i];
      return DPPF_OK;
    }
  if (dynamic_lds >= kRaiseLdsLimitFrom)
    HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kLdsLimitBytes)));
  int per_cu = 0;
  HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, block_threads, dynamic_lds));
  if (per_cu < 1) per_cu = 1;
  if (dev.nocc < kOccupancySlots) {      // a full table only means the query is repeated
    dev.occ_kernel[dev.nocc] = kernel;
    dev.occ_threads[dev.nocc] = block_threads;
    dev.occ_lds[dev.nocc] = dynamic_lds;
    dev.occ_per_cu[dev.nocc] = per_cu;
    ++dev.nocc;
  }
  *per_cu_out = per_cu;
  return DPPF_OK;
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
    // Same table as last time.  If this call runs on another stream than the one that carried the
    // upload, that stream must not start before the copy has landed.  (Inside a stream capture the
    // wait would be illegal; there the header's rule applies: one eager call first, on any stream,
    // and the table is long there.)
    if (s != t.upload_stream) {
      hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
      (void)hipStreamIsCapturing(s, &capturing);
      if (capturing == hipStreamCaptureStatusNone) HIP_TRY(hipStreamWaitEvent(s, t.uploaded, 0));
    }
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
  t.upload_stream = s;
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

// Pointer tables into the plan's own d-vectors (the stored average; the stored sum of unit gap
// vectors of the exact update).
int scratch_table(dppf_plan* p, int role, float* base, hipStream_t s, const void*** dev_out) {
  if (!base) return DPPF_EINVAL;
  std::vector<const void*> host(static_cast<size_t>(p->T));
  for (int t = 0; t < p->T; ++t) host[t] = base + p->tensor_offset[t];
  return table_upload(p, role, host.data(), host.size(), s, dev_out);
}

enum Family { kRegisters, kLds, kStoredAverage };
Family family(const dppf_plan* p) {
  return p->M <= kMaxTemplM ? kRegisters : (p->M <= kMaxLdsM ? kLds : kStoredAverage);
}

// Adam's hyper-parameters as the kernels take them; the bias corrections 1 - beta^t are formed in
// double on the host.
AdamHyper adam_hyper(float lr, float beta1, float beta2, float eps, float wd, long long step) {
  const double bc1 = 1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step));
  const double bc2 = 1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step));
  return AdamHyper{lr, beta1, beta2, eps, wd, static_cast<float>(1.0 / bc1), static_cast<float>(1.0 / bc2)};
}

#define DPPF_TIMED(plan_, id_, stream_, call_)                         \
  do {                                                                 \
    int rc__;                                                          \
    if ((rc__ = timing_begin(plan_, id_, stream_))) return rc__;       \
    if ((rc__ = (call_))) return rc__;                                 \
    if ((rc__ = timing_end(plan_, stream_))) return rc__;              \
  } while (0)

// Sweep 2 of the register-resident round, with a finalize launch in front of it when the rows of
// partial sums are too many for every block to re-reduce them itself.
int update_in_registers(dppf_plan* p, int timing_id, const void** xd, const void** vd, bool step, float lr,
                        int nparts, float pull, float push, float* r_out, float* c_out, hipStream_t s) {
  const bool fold = fold_pays(nparts);
  int rc;
  if (!fold && (rc = launch_finalize(p, nparts, pull, push, true, true, r_out, c_out, s))) return rc;
  DPPF_TIMED(p, timing_id, s, launch_update(p, xd, vd, step, fold, lr, nparts, pull, push, r_out, c_out, s));
  return DPPF_OK;
}

// The stored-average path of the round, any M: [x_A stored] -> distances -> coefficients -> update.
// avg: table of the average's tensors (the caller's xbar_out or the plan's scratch).
int round_with_stored_average(dppf_plan* p, const void** xd, const void** avg, float pull, float push, float* r_out,
                              float* c_out, hipStream_t s) {
  GridShape shape;
  int rc;
  DPPF_TIMED(p, DPPF_K_MEAN, s, launch_mean_any(p, xd, avg, s));
  DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_norms_any(p, xd, avg, &shape, s));
  if ((rc = launch_finalize(p, shape.nparts(), pull, push, true, true, r_out, c_out, s))) return rc;
  DPPF_TIMED(p, DPPF_K_UPDATE, s, launch_update_any(p, xd, avg, nullptr, false, 0.f, s));
  return DPPF_OK;
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
  if (p->sweep.ntiles == 0)   // d == 0: every distance is zero, nothing moves
    return launch_finalize(p, 0, pull, push, true, true, r_out, c_out, s);
  GridShape shape;
  switch (family(p)) {
    case kRegisters:
      if (with_step) {
        DPPF_TIMED(p, DPPF_K_STEP_REDUCE, s,
                   launch_step_reduce(p, xd, vd, gd, xbd, xbd != nullptr, lr, mu, wd, &shape, s));
        if ((rc = update_in_registers(p, DPPF_K_STEP_UPDATE, xd, vd, true, lr, shape.nparts(), pull, push, r_out,
                                      c_out, s)))
          return rc;
      } else {
        DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_reduce(p, xd, xbd, xbd != nullptr, true, kKeepTail, &shape, s));
        if ((rc = update_in_registers(p, DPPF_K_UPDATE, xd, nullptr, false, 0.f, shape.nparts(), pull, push, r_out,
                                      c_out, s)))
          return rc;
      }
      return DPPF_OK;
    case kLds: {
      LdsOptArgs o{};
      o.vp = (float* const*)(vd);
      o.gp = (const float* const*)(gd);
      o.lr = lr;
      o.mu = mu;
      o.wd = wd;
      DPPF_TIMED(p, with_step ? DPPF_K_STEP_REDUCE : DPPF_K_REDUCE, s,
                 launch_sweep1_lds(p, xd, with_step ? 1 : 0, o, xbd, xbd != nullptr, &shape, s));
      if ((rc = launch_finalize(p, shape.nparts(), pull, push, true, true, r_out, c_out, s))) return rc;
      DPPF_TIMED(p, with_step ? DPPF_K_STEP_UPDATE : DPPF_K_UPDATE, s,
                 launch_sweep2_lds(p, xd, vd, with_step ? 1 : 0, lr, 0.f, s));
      return DPPF_OK;
    }
    case kStoredAverage: {
      if (with_step && (rc = launch_local_step(p, xd, vd, gd, lr, mu, wd, s))) return rc;
      const void** avg = xbd;
      if (!avg && (rc = scratch_table(p, dppf_plan::RXBAR_SCRATCH, p->xbar_scratch, s, &avg))) return rc;
      return round_with_stored_average(p, xd, avg, pull, push, r_out, c_out, s);
    }
  }
  return DPPF_EINVAL;
}

// ---- the static scratch of dppf_pull_push_round_flat_static, the entry point for callers that may
// not allocate: a file-scope device array (every GPU the library runs on holds its own copy until
// the process ends).  Host code never uses the array's name as an address; it asks the runtime for
// this device's copy once (static_scratch_base) and passes that pointer to the kernels.
constexpr long long kStaticMaxDim = DPPF_STATIC_MAX_DIM;              // elements per worker
constexpr int kStaticMaxWorkers = kMaxTemplM;
constexpr int kStaticMaxTiles = static_cast<int>(kStaticMaxDim / sweep_tile_elems(kMaxTemplM)) + 1;
constexpr int kStaticMaxRows = 2048;                        // rows of partial sums (one per block)
constexpr size_t round_up_256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t kStaticOffSched = 0;
constexpr size_t kStaticOffCoef = kStaticOffSched + round_up_256(sizeof(Sched));
constexpr size_t kStaticOffAvgNorm = kStaticOffCoef + round_up_256(sizeof(Coef) * kStaticMaxWorkers);
constexpr size_t kStaticOffPtrs = kStaticOffAvgNorm + round_up_256(sizeof(float));
constexpr size_t kStaticOffTiles = kStaticOffPtrs + round_up_256(sizeof(float*) * kStaticMaxWorkers);
constexpr size_t kStaticOffPartials = kStaticOffTiles + round_up_256(sizeof(Tile) * (kStaticMaxTiles + 1));
constexpr size_t kStaticBytes =
    kStaticOffPartials + round_up_256(sizeof(double) * kStaticMaxRows * (kStaticMaxWorkers + 1));
static_assert(kStaticBytes == DPPF_STATIC_SCRATCH_BYTES, "the header documents the size of the static scratch");
static __device__ __align__(256) unsigned char g_static_scratch[kStaticBytes];

// This device's copy of the static scratch array and its CU count, looked up once per device.
int static_scratch_base(int device, unsigned char** base, int* num_cu) {
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

}  // namespace
}  // namespace dppf_detail

using namespace dppf_detail;

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
  if (p->sweep.dev && p->sweep.dev != p->step.dev) (void)hipFree(p->sweep.dev);
  if (p->step.dev) (void)hipFree(p->step.dev);
  if (p->partials) (void)hipFree(p->partials);
  if (p->coef) (void)hipFree(p->coef);
  if (p->avg_norm) (void)hipFree(p->avg_norm);
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
  try {
    std::vector<Tile> step_tiles, sweep_tiles;
    p->M = M;
    p->T = T;
    p->step.tile_elems = kStepTileElems;
    p->sweep.tile_elems = sweep_tile_elems(M);
    int rc = dppf_walk::build_tile_list(T, numel, p->step.tile_elems, &step_tiles, &p->step.nfull, &p->d,
                                        &p->tensor_offset);
    if (rc == 0 && p->sweep.tile_elems != p->step.tile_elems)
      rc = dppf_walk::build_tile_list(T, numel, p->sweep.tile_elems, &sweep_tiles, &p->sweep.nfull, &p->d,
                                      &p->tensor_offset);
    if (rc != 0) {
      delete p;
      return rc;     // build_tile_list's codes are DPPF_EINVAL / DPPF_ELIMIT
    }
    p->numel.assign(numel, numel + T);
    p->step.ntiles = static_cast<int>(step_tiles.size());
    const bool shared_list = p->sweep.tile_elems == p->step.tile_elems;
    if (shared_list) p->sweep = p->step;
    else p->sweep.ntiles = static_cast<int>(sweep_tiles.size());

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
    // one row per block + at most one per full tile of the sweep list
    p->partials_rows = p->num_cu * kMaxBlocksPerCU + p->sweep.nfull;
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->step.dev), (step_tiles.size() + 1) * sizeof(Tile)));
    if (!step_tiles.empty())
      PLAN_TRY(hipMemcpy(p->step.dev, step_tiles.data(), step_tiles.size() * sizeof(Tile), hipMemcpyHostToDevice));
    if (shared_list) {
      p->sweep.dev = p->step.dev;
    } else {
      PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->sweep.dev), (sweep_tiles.size() + 1) * sizeof(Tile)));
      if (!sweep_tiles.empty())
        PLAN_TRY(hipMemcpy(p->sweep.dev, sweep_tiles.data(), sweep_tiles.size() * sizeof(Tile),
                           hipMemcpyHostToDevice));
    }
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->partials),
                       static_cast<size_t>(p->partials_rows) * p->cols() * sizeof(double)));
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->coef), static_cast<size_t>(M) * sizeof(Coef)));
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->avg_norm), sizeof(float)));
    PLAN_TRY(hipMemset(p->avg_norm, 0, sizeof(float)));
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->sched), sizeof(Sched)));
    PLAN_TRY(hipMemset(p->sched, 0, sizeof(Sched)));
    if (M > kMaxTemplM && p->d > 0)
      PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->xbar_scratch), static_cast<size_t>(p->d) * sizeof(float)));
    if (M > kMaxLdsM && p->d > 0)
      PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->usum_scratch), static_cast<size_t>(p->d) * sizeof(float)));
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
  } catch (const std::bad_alloc&) {
    dppf_plan_destroy(p);
    return DPPF_ENOMEM;
  } catch (...) {
    dppf_plan_destroy(p);
    return DPPF_EINVAL;
  }
  *out = p;
  return DPPF_OK;
}

int64_t dppf_plan_dim(const dppf_plan* p) { return p ? p->d : 0; }

int dppf_sweep_tile_elems(int M) {
  if (M < 1 || M > DPPF_MAX_WORKERS) return DPPF_EINVAL;
  return sweep_tile_elems(M);
}

int dppf_layout_tiles(int tile_elems, int T, const int64_t* numel, int64_t* d, int64_t* nfull, int64_t* ntiles,
                      int64_t cap, int32_t* tile_tensor, int64_t* tile_offset, int32_t* tile_count) try {
  if (tile_elems < 1 || T < 0 || (T > 0 && !numel) || !d || !nfull || !ntiles || cap < 0) return DPPF_EINVAL;
  std::vector<Tile> tiles;
  std::vector<long long> offsets;
  int full = 0;
  long long total = 0;
  const int rc = dppf_walk::build_tile_list(T, numel, tile_elems, &tiles, &full, &total, &offsets);
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
} DPPF_CATCH

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
  if (p->step.ntiles == 0) return DPPF_OK;
  if (family(p) == kRegisters)
    DPPF_TIMED(p, DPPF_K_MEAN, s, launch_reduce(p, xd, xbd, true, false, kKeepNone, nullptr, s));
  else
    DPPF_TIMED(p, DPPF_K_MEAN, s, launch_mean_any(p, xd, xbd, s));
  return DPPF_OK;
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
  if (p->step.ntiles == 0) return launch_finalize(p, 0, 0.f, 0.f, false, false, r_out, nullptr, s);
  GridShape shape;
  if (xbd) {
    DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_norms_any(p, xd, xbd, &shape, s));
  } else if (family(p) == kRegisters) {
    DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_reduce(p, xd, nullptr, false, true, kKeepNone, &shape, s));
  } else if (family(p) == kLds) {
    DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_sweep1_lds(p, xd, 0, LdsOptArgs{}, nullptr, false, &shape, s));
  } else {
    const void** avg = nullptr;
    if ((rc = scratch_table(p, dppf_plan::RXBAR_SCRATCH, p->xbar_scratch, s, &avg))) return rc;
    DPPF_TIMED(p, DPPF_K_MEAN, s, launch_mean_any(p, xd, avg, s));
    DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_norms_any(p, xd, avg, &shape, s));
  }
  return launch_finalize(p, shape.nparts(), 0.f, 0.f, false, false, r_out, nullptr, s);
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
  if (p->step.ntiles == 0) return DPPF_OK;
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
  const float mf = static_cast<float>(p->M);
  if (p->sweep.ntiles == 0) return launch_finalize(p, 0, pull, push_r / mf, false, true, r_out, c_out, s);
  GridShape shape;
  switch (family(p)) {
    case kRegisters:
      DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_reduce(p, xd, nullptr, false, true, kKeepTail, &shape, s));
      DPPF_TIMED(p, DPPF_K_UPDATE_EXACT, s,
                 launch_update_exact(p, xd, shape.nparts(), pull, push_r, r_out, c_out, s));
      return DPPF_OK;
    case kLds:
      DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_sweep1_lds(p, xd, 0, LdsOptArgs{}, nullptr, false, &shape, s));
      if ((rc = launch_finalize(p, shape.nparts(), pull, push_r / mf, true, true, r_out, c_out, s))) return rc;
      DPPF_TIMED(p, DPPF_K_UPDATE_EXACT, s, launch_sweep2_lds(p, xd, nullptr, 2, 0.f, push_r / (mf * mf), s));
      return DPPF_OK;
    case kStoredAverage: {
      // stored average -> distances -> coefficients and 1/r -> stored sum of unit gap vectors -> update
      const void **avg = nullptr, **usum = nullptr;
      if ((rc = scratch_table(p, dppf_plan::RXBAR_SCRATCH, p->xbar_scratch, s, &avg))) return rc;
      if ((rc = scratch_table(p, dppf_plan::RUSUM_SCRATCH, p->usum_scratch, s, &usum))) return rc;
      DPPF_TIMED(p, DPPF_K_MEAN, s, launch_mean_any(p, xd, avg, s));
      DPPF_TIMED(p, DPPF_K_REDUCE, s, launch_norms_any(p, xd, avg, &shape, s));
      if ((rc = launch_finalize(p, shape.nparts(), pull, push_r / mf, true, true, r_out, c_out, s))) return rc;
      if ((rc = timing_begin(p, DPPF_K_UPDATE_EXACT, s))) return rc;
      if ((rc = launch_unit_sum_any(p, xd, avg, usum, s))) return rc;
      if ((rc = launch_update_any(p, xd, avg, usum, true, push_r / (mf * mf), s))) return rc;
      return timing_end(p, s);
    }
  }
  return DPPF_EINVAL;
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
  if (p->sweep.ntiles == 0) return launch_finalize(p, 0, 0.f, 0.f, false, false, r_post_out, nullptr, s);
  const bool from_consensus = push_from == DPPF_PUSH_FROM_CONSENSUS;
  GridShape shape;
  if (family(p) == kRegisters) {
    DPPF_TIMED(p, DPPF_K_SEQ_REDUCE, s, launch_seq_reduce(p, xd, xcd, from_consensus, pull, &shape, s));
    DPPF_TIMED(p, DPPF_K_SEQ_UPDATE, s,
               launch_seq_update(p, xd, xcd, from_consensus, pull, push, shape.nparts(), r_post_out, s));
    return DPPF_OK;
  }
  // more workers than one lane holds in registers: the pre-round average (when the push refers to
  // it) is stored first, then the workers stream past it
  const void** avg = nullptr;
  if (!from_consensus) {
    if ((rc = scratch_table(p, dppf_plan::RXBAR_SCRATCH, p->xbar_scratch, s, &avg))) return rc;
    DPPF_TIMED(p, DPPF_K_MEAN, s, launch_mean_any(p, xd, avg, s));
  }
  DPPF_TIMED(p, DPPF_K_SEQ_REDUCE, s, launch_seq_any(p, xd, xcd, avg, from_consensus, false, pull, &shape, s));
  // lambda / r_m = -(0 - push / r_m): the coefficients of a round with pull 0
  if ((rc = launch_finalize(p, shape.nparts(), 0.f, push, true, false, r_post_out, nullptr, s))) return rc;
  DPPF_TIMED(p, DPPF_K_SEQ_UPDATE, s, launch_seq_any(p, xd, xcd, avg, from_consensus, true, pull, nullptr, s));
  return DPPF_OK;
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
  if (p->step.ntiles == 0) return DPPF_OK;
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
  if (p->sweep.ntiles == 0) return launch_finalize(p, 0, pull, push, true, true, r_out, c_out, s);
  const AdamHyper hp = adam_hyper(lr, beta1, beta2, eps, weight_decay, step);
  GridShape shape;
  switch (family(p)) {
    case kRegisters:
      DPPF_TIMED(p, DPPF_K_ADAMW_REDUCE, s, launch_adamw_reduce(p, xd, ad, sd, gd, hp, &shape, s));
      return update_in_registers(p, DPPF_K_UPDATE, xd, nullptr, false, 0.f, shape.nparts(), pull, push, r_out, c_out,
                                 s);
    case kLds: {
      LdsOptArgs o{};
      o.vp = (float* const*)(ad);
      o.sp = (float* const*)(sd);
      o.gp = (const float* const*)(gd);
      o.adam = hp;
      DPPF_TIMED(p, DPPF_K_ADAMW_REDUCE, s, launch_sweep1_lds(p, xd, 2, o, nullptr, false, &shape, s));
      if ((rc = launch_finalize(p, shape.nparts(), pull, push, true, true, r_out, c_out, s))) return rc;
      DPPF_TIMED(p, DPPF_K_UPDATE, s, launch_sweep2_lds(p, xd, nullptr, 0, 0.f, 0.f, s));
      return DPPF_OK;
    }
    case kStoredAverage:   // step, then the round
      if ((rc = launch_adamw_step(p, xd, ad, sd, gd, hp, s))) return rc;
      return round_impl(p, false, x, nullptr, nullptr, 0.f, 0.f, 0.f, pull, push, r_out, c_out, nullptr, s);
  }
  return DPPF_EINVAL;
} DPPF_CATCH

int dppf_plan_average_norm(dppf_plan* p, float* out, void* stream) {
  if (!p || !out) return DPPF_EINVAL;
  return launch_copy_scalar(p->avg_norm, out, static_cast<hipStream_t>(stream));
}

int dppf_round_statistics(const float* r, int M, float pull, float push, const float* avg_norm, float* out,
                          void* stream) {
  if (!r || !out || M < 1 || M > DPPF_MAX_WORKERS) return DPPF_EINVAL;
  return launch_round_stats(r, M, pull, push, avg_norm, out, static_cast<hipStream_t>(stream));
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
  view.sweep.tile_elems = sweep_tile_elems(M);
  view.sweep.nfull = static_cast<int>(d / view.sweep.tile_elems);
  view.sweep.ntiles = view.sweep.nfull + (d % view.sweep.tile_elems ? 1 : 0);
  view.sweep.dev = reinterpret_cast<Tile*>(base + kStaticOffTiles);
  view.partials = reinterpret_cast<double*>(base + kStaticOffPartials);
  view.partials_rows = kStaticMaxRows;
  view.sched = reinterpret_cast<Sched*>(base + kStaticOffSched);
  view.coef = reinterpret_cast<Coef*>(base + kStaticOffCoef);
  view.avg_norm = reinterpret_cast<float*>(base + kStaticOffAvgNorm);
  const void** xd = reinterpret_cast<const void**>(base + kStaticOffPtrs);
  // the tile list, the pointer table and a clean counter are written by a kernel (no copy from
  // host memory, no memset: both would be foreign bodies in a captured graph)
  if ((rc = launch_flat_setup(view.sweep.dev, static_cast<long long>(d), view.sweep.tile_elems, view.sweep.ntiles,
                              num_cu, (float**)(xd), x, static_cast<long long>(ld), M, view.sched, s)))
    return rc;
  if (view.sweep.ntiles == 0) return launch_finalize(&view, 0, pull, push, true, true, r_out, c_out, s);
  GridShape shape;
  if ((rc = launch_reduce(&view, xd, nullptr, false, true, kKeepTail, &shape, s))) return rc;
  return update_in_registers(&view, DPPF_K_UPDATE, xd, nullptr, false, 0.f, shape.nparts(), pull, push, r_out, c_out,
                             s);
} DPPF_CATCH

// ---- measurement aids (dppf_util.h)
int dppf_util_copy(float* dst, const float* src, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!dst || !src))) return DPPF_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dst) & 3u) || (reinterpret_cast<uintptr_t>(src) & 3u)) return DPPF_EINVAL;
  if (n == 0) return DPPF_OK;
  return launch_copy(dst, src, n, static_cast<hipStream_t>(stream));
}

int dppf_util_stream_probe(float* base, int64_t stride, int64_t n, int reads, int writes, int inplace,
                           int blocks_per_cu, int on_demand, void* stream) {
  if (!base || n < 0 || stride < n || blocks_per_cu < 1 || blocks_per_cu > 16) return DPPF_EINVAL;
  if (reinterpret_cast<uintptr_t>(base) & 15u || (stride & 3)) return DPPF_EINVAL;
  if (n / 1024 >= INT32_MAX) return DPPF_ELIMIT;
  return launch_stream_probe(base, stride, n, reads, writes, inplace, blocks_per_cu, on_demand,
                             static_cast<hipStream_t>(stream));
}

int dppf_util_stream_probe_grouped(float* base, int64_t stride, int64_t n, int groups, int reads_per_group,
                                   int vectors, int ahead, int blocks_per_cu, int on_demand, void* stream) {
  if (!base || n < 0 || stride < n || blocks_per_cu < 1 || blocks_per_cu > 16) return DPPF_EINVAL;
  if (reinterpret_cast<uintptr_t>(base) & 15u || (stride & 3)) return DPPF_EINVAL;
  if (n / 1024 >= INT32_MAX) return DPPF_ELIMIT;
  return launch_stream_probe_grouped(base, stride, n, groups, reads_per_group, vectors, ahead, blocks_per_cu,
                                     on_demand, static_cast<hipStream_t>(stream));
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
