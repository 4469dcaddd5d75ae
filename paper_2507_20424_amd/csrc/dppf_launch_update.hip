// Sweep 2 of the round for M <= 16: Eq. 5 (optionally on x - lr v of the fused round), and the
// exact two-term form of Eq. 4 (a).
#include "dppf_internal.h"

namespace dppf_detail {
namespace {

// Every block of sweep 2 re-reduces the rows of partial sums itself (no finalize launch on the
// round's critical path) as long as there are few of them -- an evenly split reducing sweep leaves
// one row per block.  A sweep that took its tiles on demand leaves a row per tile; re-reading
// twenty thousand rows in every block costs more than the extra launch (ViT-B-sized list, M = 4:
// 27 against 8 microseconds).
constexpr int kFoldMaxRows = 4096;

template <bool STEP, bool FOLD>
int launch(dppf_plan* p, const void** xp, const void** vp, float lr, int nparts, float pull, float push,
           float* r_out, float* c_out, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float* const* v = (const float* const*)(vp);
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = STEP ? unroll_step_update(kM) : unroll_plain(kM);
    auto kern = k_sweep2<kM, kU, STEP, FOLD>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kOnDemand, (STEP ? 12.0 : 8.0) * kM);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, v, lr, p->coef,
                       p->partials, nparts, p->partials_rows, pull, push, r_out, c_out, p->avg_norm);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace

bool fold_pays(int nparts) { return nparts <= kFoldMaxRows; }

int launch_update(dppf_plan* p, const void** xp, const void** vp, bool step, bool fold, float lr, int nparts,
                  float pull, float push, float* r_out, float* c_out, hipStream_t s) {
  if (!fold)
    return step ? launch<true, false>(p, xp, vp, lr, 0, pull, push, nullptr, nullptr, s)
                : launch<false, false>(p, xp, nullptr, 0.f, 0, pull, push, nullptr, nullptr, s);
  return step ? launch<true, true>(p, xp, vp, lr, nparts, pull, push, r_out, c_out, s)
              : launch<false, true>(p, xp, nullptr, 0.f, nparts, pull, push, r_out, c_out, s);
}

int launch_update_exact(dppf_plan* p, const void** xp, int nparts, float pull, float push_r, float* r_out,
                        float* c_out, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float mf = static_cast<float>(p->M);
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_plain(kM);
    auto kern = k_update_exact<kM, kU>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kOnDemand, 8.0 * kM);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, p->partials, nparts,
                       p->partials_rows, pull, push_r / mf, push_r / (mf * mf), r_out, c_out, p->avg_norm);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace dppf_detail
