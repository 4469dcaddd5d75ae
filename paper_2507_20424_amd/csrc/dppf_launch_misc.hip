// The stand-alone momentum-SGD step, the small kernels (finalize, logged by-products, flat-tensor
// setup) and the two measurement aids (plain copy, streaming probe).
#include "dppf_internal.h"

namespace dppf_detail {

int launch_local_step(dppf_plan* p, const void** xp, const void** vp, const void** gp, float lr, float mu, float wd,
                      hipStream_t s) {
  auto kern = k_local_step<4>;
  int grid = 0, gfull = 0;
  int rc = grid_for(p, p->step, kern, p->M, kTilesPerWorkerItem, kBlocksPerCUReadWrite, 0, &gfull, &grid);
  if (rc) return rc;
  if ((rc = timing_begin(p, DPPF_K_LOCAL_STEP, s))) return rc;
  const Walk walk = plan_walk(p, p->step, gfull, p->M, kTilesPerWorkerItem, dppf_walk::kOnDemand, 20.0);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->step.dev, walk, p->M, p->T, (float* const*)(xp),
                     (float* const*)(vp), (const float* const*)(gp), lr, mu, wd);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_finalize(dppf_plan* p, int nparts, float pull, float push, bool want_coef, bool want_avg_norm,
                    float* r_out, float* c_out, hipStream_t s) {
  int rc = timing_begin(p, DPPF_K_FINALIZE, s);
  if (rc) return rc;
  hipLaunchKernelGGL(k_finalize, dim3(p->M + (want_avg_norm ? 1 : 0)), dim3(kFinalizeThreads), 0, s, p->partials, nparts,
                     p->partials_rows, p->M, pull, push, want_coef ? p->coef : nullptr, r_out, c_out, p->avg_norm);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_round_stats(const float* r, int M, float pull, float push, const float* avg_norm, float* out,
                       hipStream_t s) {
  hipLaunchKernelGGL(k_round_stats, dim3(1), dim3(64), 0, s, r, M, pull, push, avg_norm, out);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_copy_scalar(const float* src, float* dst, hipStream_t s) {
  hipLaunchKernelGGL(k_copy_scalar, dim3(1), dim3(64), 0, s, src, dst);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_flat_setup(Tile* tiles, long long d, int tile_elems, int ntiles, int num_cu, float** ptrs, float* x,
                      long long ld, int M, Sched* sched, hipStream_t s) {
  int blocks = (ntiles + kBlock - 1) / kBlock;
  if (blocks < 1) blocks = 1;
  if (blocks > num_cu) blocks = num_cu;
  hipLaunchKernelGGL(k_flat_setup, dim3(blocks), dim3(kBlock), 0, s, tiles, d, tile_elems, ptrs, x, ld, M, sched);
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

// ---------------------------------------------- plain copy (bandwidth / counter calibration)
namespace {

__global__ __launch_bounds__(kBlock) void k_copy(float* __restrict__ dst, const float* __restrict__ src,
                                                 long long n) {
  const long long nvec = n / 4;
  const long long stride = static_cast<long long>(gridDim.x) * kBlock;
  for (long long i = static_cast<long long>(blockIdx.x) * kBlock + threadIdx.x; i < nvec; i += stride)
    store4_stream<true>(dst + 4 * i, load4_stream<true>(src + 4 * i, 4), 4);
  if (blockIdx.x == 0 && threadIdx.x < n - 4 * nvec) dst[4 * nvec + threadIdx.x] = src[4 * nvec + threadIdx.x];
}

// ------------------------------------ streaming probe: R read streams, W write streams
// Stream k is the n floats at base + k*stride.  Each element's R values are added and the sum
// (times w+1) is stored to W streams: streams R..R+W-1, or, with INPLACE, streams 0..W-1 (read
// and written by the same lane).  Gives the device's bandwidth for a given read/write mix when
// every stream is touched at once.  The blocks walk items of kProbeItemTiles tiles the way the
// DPPF kernels walk their tiles: an even split, or an even split with the tail handed out on demand.
constexpr int kProbeItemTiles = 16;
__device__ Sched g_probe_sched;

template <int R, int W, int U, bool INPLACE>
__global__ __launch_bounds__(kBlock) void k_probe(float* __restrict__ base, long long stride, long long n,
                                                  float* __restrict__ sink, const Walk wk) {
  const long long tile = static_cast<long long>(kBlock) * U * 4;
  const long long ntiles = n / tile;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  walk<false>(
      wk, 1,
      [&](int item) {
        const long long t0 = static_cast<long long>(item) * kProbeItemTiles;
        const long long t1 = t0 + kProbeItemTiles < ntiles ? t0 + kProbeItemTiles : ntiles;
#pragma unroll 1
        for (long long t = t0; t < t1; ++t) {
          f4 v[U];
#pragma unroll
          for (int k = 0; k < U; ++k)
            v[k] = (R > 0) ? (f4){0.f, 0.f, 0.f, 0.f} : (f4){1.f, 2.f, 3.f, static_cast<float>(t)};
          if (R > 0) {
            f4 tmp[R > 0 ? R : 1][U];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
              for (int k = 0; k < U; ++k)
                tmp[r][k] = load4_stream<true>(base + r * stride + t * tile + 4 * (k * kBlock + threadIdx.x), 4);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
              for (int k = 0; k < U; ++k) v[k] += tmp[r][k];
          }
          if (W > 0) {
#pragma unroll
            for (int w = 0; w < W; ++w)
#pragma unroll
              for (int k = 0; k < U; ++k)
                store4_stream<true>(base + (INPLACE ? w : R + w) * stride + t * tile + 4 * (k * kBlock + threadIdx.x),
                                    v[k] * static_cast<float>(w + 1), 4);
          } else {
#pragma unroll
            for (int k = 0; k < U; ++k) acc += v[k];
          }
        }
      },
      [](int) {}, [](int) {});
  if (W == 0 && acc.x + acc.y + acc.z + acc.w == 123.456f) sink[0] = acc.x;   // keeps the loads alive
}


// ------------------------------------ the same traffic in the order the sweeps use
// NG groups of GR streams each (group j: streams j*GR .. j*GR+GR-1), taken one group after the
// other inside a tile of kBlock*U vectors, the way the fused sweeps take one worker after the
// other: a lane loads the group's GR*U vectors, adds them and overwrites the group's first stream
// with the sum (half the value when the group is a single stream): GR reads and 1 write in place
// per group and element, with the loads of the next AHEAD groups requested before the current
// group's are waited for.  One tile per work item, handed out like the sweeps' tiles.  The memory
// traffic of a sweep with none of its arithmetic, reductions or pointer tables.
template <int NG, int GR, int U, int AHEAD>
__global__ __launch_bounds__(kBlock) void k_probe_grouped(float* __restrict__ base, long long stride, const Walk wk) {
  constexpr long long kTile = static_cast<long long>(kBlock) * U * 4;
  walk<false>(
      wk, 1,
      [&](int item) {
        float* at = base + item * kTile + 4 * threadIdx.x;
        f4 buf[NG][GR][U];
        auto request = [&](int j) {
#pragma unroll
          for (int r = 0; r < GR; ++r)
#pragma unroll
            for (int k = 0; k < U; ++k)
              buf[j][r][k] = load4_stream<true>(at + (j * GR + r) * stride + 4 * k * kBlock, 4);
        };
#pragma unroll
        for (int j = 0; j < AHEAD && j < NG; ++j) request(j);
#pragma unroll
        for (int j = 0; j < NG; ++j) {
          if (j + AHEAD < NG) request(j + AHEAD);
#pragma unroll
          for (int k = 0; k < U; ++k) {
            f4 sum = buf[j][0][k];
#pragma unroll
            for (int r = 1; r < GR; ++r) sum += buf[j][r][k];
            if (GR == 1) sum = sum * 0.5f;   // storing back the very value loaded would be dropped as a dead store
            store4_stream<true>(at + (j * GR) * stride + 4 * k * kBlock, sum, 4);
          }
        }
      },
      [](int) {}, [](int) {});
}

}  // namespace

int launch_copy(float* dst, const float* src, int64_t n, hipStream_t s) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  int cus = 0;
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  long long blocks = (n / 4 + kBlock - 1) / kBlock;
  const long long cap = static_cast<long long>(cus) * kBlocksPerCUReadWrite;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_copy, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, s, dst, src,
                     static_cast<long long>(n));
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

int launch_stream_probe(float* base, int64_t stride, int64_t n, int reads, int writes, int inplace,
                        int blocks_per_cu, int on_demand, hipStream_t s) {
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  Sched* sched = nullptr;   // this device's copy of the probe's counter
  HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&sched), HIP_SYMBOL(g_probe_sched)));
  const dim3 grid(static_cast<unsigned>(cus * blocks_per_cu)), block(kBlock);
  float* sink = base;   // never written unless a sum hits one magic value
#define DPPF_PROBE(R_, W_, U_, IP_)                                                                        \
  if (reads == R_ && writes == W_ && (inplace != 0) == IP_) {                                              \
    const long long tiles_ = n / (static_cast<long long>(kBlock) * U_ * 4);                                \
    const long long items_ = (tiles_ + kProbeItemTiles - 1) / kProbeItemTiles;                             \
    const Walk walk_ = dppf_walk::make_walk(static_cast<int>(items_), static_cast<int>(items_),            \
                                            kProbeItemTiles * kBlock * U_ * 4, static_cast<int>(grid.x), 1, 1, \
                                            on_demand ? dppf_walk::kOnDemand : dppf_walk::kEvenSplit,      \
                                            4.0 * (R_ + W_), sched);                                       \
    hipLaunchKernelGGL((k_probe<R_, W_, U_, IP_>), grid, block, 0, s, base, static_cast<long long>(stride), \
                       static_cast<long long>(n), sink, walk_);                                            \
    HIP_TRY(hipGetLastError());                                                                            \
    return DPPF_OK;                                                                                        \
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

int launch_stream_probe_grouped(float* base, int64_t stride, int64_t n, int groups, int reads_per_group,
                                int vectors, int ahead, int blocks_per_cu, int on_demand, hipStream_t s) {
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  Sched* sched = nullptr;
  HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&sched), HIP_SYMBOL(g_probe_sched)));
  const dim3 block(kBlock);
#define DPPF_PROBE_G(NG_, GR_, U_, A_)                                                                        \
  if (groups == NG_ && reads_per_group == GR_ && vectors == U_ && ahead == A_) {                              \
    const long long tiles_ = n / (static_cast<long long>(kBlock) * U_ * 4);                                   \
    if (tiles_ < 1 || tiles_ > INT32_MAX) return DPPF_EINVAL;                                                 \
    long long grid_ = static_cast<long long>(cus) * blocks_per_cu;                                            \
    if (grid_ > tiles_) grid_ = tiles_;                                                                       \
    const Walk walk_ = dppf_walk::make_walk(static_cast<int>(tiles_), static_cast<int>(tiles_), kBlock * U_ * 4, \
                                            static_cast<int>(grid_), 1, 1,                                    \
                                            on_demand ? dppf_walk::kOnDemand : dppf_walk::kEvenSplit,         \
                                            4.0 * NG_ * (GR_ + 1), sched);                                    \
    hipLaunchKernelGGL((k_probe_grouped<NG_, GR_, U_, A_>), dim3(static_cast<unsigned>(grid_)), block, 0, s,  \
                       base, static_cast<long long>(stride), walk_);                                          \
    HIP_TRY(hipGetLastError());                                                                               \
    return DPPF_OK;                                                                                           \
  }
  DPPF_PROBE_G(2, 3, 4, 0)    // two workers
  DPPF_PROBE_G(4, 3, 4, 0)    // sweep 1 of the fused round, 4 workers
  DPPF_PROBE_G(4, 3, 4, 3)
  DPPF_PROBE_G(4, 3, 2, 0)
  DPPF_PROBE_G(4, 3, 8, 0)
  DPPF_PROBE_G(4, 2, 4, 0)    // sweep 2 of the fused round, 4 workers
  DPPF_PROBE_G(4, 2, 4, 3)
  DPPF_PROBE_G(4, 2, 8, 0)
  DPPF_PROBE_G(8, 3, 2, 0)    // 8 workers
  DPPF_PROBE_G(8, 3, 2, 7)
  DPPF_PROBE_G(8, 2, 2, 0)
  DPPF_PROBE_G(8, 2, 2, 7)
  DPPF_PROBE_G(16, 3, 2, 0)   // 16 workers
  DPPF_PROBE_G(16, 3, 2, 7)
  DPPF_PROBE_G(16, 2, 2, 7)
  DPPF_PROBE_G(4, 1, 4, 0)    // the plain round's sweep 2 (read x, write x)
#undef DPPF_PROBE_G
  return DPPF_EINVAL;   // this shape is not instantiated
}

}  // namespace dppf_detail
