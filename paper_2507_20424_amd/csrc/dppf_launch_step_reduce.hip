// Sweep 1 of the fused round for M <= 16: the momentum-SGD step of Alg. 1 folded in (v stored, the
// stepped x kept in registers only), the average and the squared distances of the stepped x.
#include "dppf_internal.h"

namespace dppf_detail {
namespace {

template <int XBAR>
int launch(dppf_plan* p, const void** xp, const void** vp, const void** gp, const void** xbarp, float lr, float mu,
           float wd, GridShape* shape, hipStream_t s) {
  float* const* x = (float* const*)(xp);
  float* const* v = (float* const*)(vp);
  const float* const* g = (const float* const*)(gp);
  float* const* xb = (float* const*)(xbarp);
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_fused(kM);
    auto kern = k_sweep1<kM, kU, true, XBAR, true>;
    int grid = 0, gfull = 0;
    const int rc = grid_for(p, p->sweep, kern, 1, 1, kBlocksPerCUReadWrite, 0, &gfull, &grid);
    if (rc) return rc;
    const Walk walk = plan_walk(p, p->sweep, gfull, 1, 1, dppf_walk::kOnDemandReducing, 16.0 * kM);
    if (!rows_fit(p, grid, walk)) return DPPF_ELIMIT;
    shape->grid = grid;
    shape->walk = walk;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->sweep.dev, walk, p->T, x, v, g, xb, lr, mu, wd,
                       p->partials, p->partials_rows, keep_from_tile(p, kKeepTail));
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

}  // namespace

int launch_step_reduce(dppf_plan* p, const void** xp, const void** vp, const void** gp, const void** xbarp,
                       bool store_avg, float lr, float mu, float wd, GridShape* shape, hipStream_t s) {
  return store_avg ? launch<1>(p, xp, vp, gp, xbarp, lr, mu, wd, shape, s)
                   : launch<0>(p, xp, vp, gp, nullptr, lr, mu, wd, shape, s);
}

}  // namespace dppf_detail
