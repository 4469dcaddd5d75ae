// The two sweeps of the round for 17..39 workers: every worker's vector of a lane is staged in
// LDS, so x is read once per sweep whatever M is (the register-resident kernels stop at 16).
#include "dppf_internal.h"

namespace dppf_detail {
namespace {

size_t stage_bytes(int M) { return static_cast<size_t>(M) * kBlock * sizeof(f4); }

template <typename K, typename... Args>
int launch_on(dppf_plan* p, K kern, int want_per_cu, size_t lds, OnDemand policy, double bytes_per_elem,
              GridShape* shape, hipStream_t s, Args... args) {
  int grid = 0, gfull = 0;
  const int rc = grid_for(p, p->sweep, kern, 1, 1, want_per_cu, lds, &gfull, &grid);
  if (rc) return rc;
  const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, policy, bytes_per_elem);
  if (shape) {
    if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    shape->grid = grid;
    shape->walk = walk;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), lds, s, p->sweep.dev, walk, p->M, p->T, args...);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace

int launch_sweep1_lds(dppf_plan* p, const void** xp, int opt, const LdsOptArgs& o, const void** xbarp,
                      bool store_avg, GridShape* shape, hipStream_t s) {
  if (p->M <= kMaxTemplM || p->M > kMaxLdsM || p->sweep.tile_elems != kLdsTileElems) return DPPF_EINVAL;
  const size_t lds = stage_bytes(p->M) + sizeof(double) * kWaves * (static_cast<size_t>(p->M) + 1);
  float* const* x = (float* const*)(xp);
  float* const* xb = (float* const*)(xbarp);
  double* parts = p->partials;
  const int ps = p->partials_rows;
  const double bytes = (opt == 0 ? 4.0 : (opt == 1 ? 16.0 : 28.0)) * p->M;
  // a pure read keeps the even split (per-tile sums would cost more than they win), see make_walk's policy
  const OnDemand policy = opt == 0 && !store_avg ? dppf_walk::kEvenSplit : dppf_walk::kOnDemandReducing;
  // Like the register-resident sweeps: a sweep that only reads streams best from two resident
  // blocks per CU (M = 17: -38 %; the LDS holds two stages up to 19 workers), one that also writes
  // from one.  Smaller blocks that would fit twice for any M were slower than one block of 256
  // threads (128 threads x 2: +10 %): each start of the load pipeline costs a memory latency, and
  // they start it twice per tile.
  const int want_per_cu = opt == 0 && !store_avg ? kBlocksPerCUReadOnly : kBlocksPerCUReadWrite;
#define DPPF_LDS1(OPT_, XBAR_) \
  return launch_on(p, k_sweep1_lds<OPT_, XBAR_>, want_per_cu, lds, policy, bytes, shape, s, x, o, xb, parts, ps)
  if (store_avg) {
    if (opt == 0) DPPF_LDS1(0, 1);
    if (opt == 1) DPPF_LDS1(1, 1);
    if (opt == 2) DPPF_LDS1(2, 1);
  } else {
    if (opt == 0) DPPF_LDS1(0, 0);
    if (opt == 1) DPPF_LDS1(1, 0);
    if (opt == 2) DPPF_LDS1(2, 0);
  }
#undef DPPF_LDS1
  return DPPF_EINVAL;
}

int launch_sweep2_lds(dppf_plan* p, const void** xp, const void** vp, int mode, float lr, float k2, hipStream_t s) {
  if (p->M <= kMaxTemplM || p->M > kMaxLdsM || p->sweep.tile_elems != kLdsTileElems) return DPPF_EINVAL;
  const size_t lds = stage_bytes(p->M);
  float* const* x = (float* const*)(xp);
  const float* const* v = (const float* const*)(vp);
  const double bytes = (mode == 1 ? 12.0 : 8.0) * p->M;
#define DPPF_LDS2(MODE_) \
  return launch_on(p, k_sweep2_lds<MODE_>, kBlocksPerCUReadWrite, lds, dppf_walk::kOnDemand, bytes, nullptr, s, x, v, lr, p->coef, k2)
  if (mode == 0) DPPF_LDS2(0);
  if (mode == 1) DPPF_LDS2(1);
  if (mode == 2) DPPF_LDS2(2);
#undef DPPF_LDS2
  return DPPF_EINVAL;
}

}  // namespace dppf_detail
