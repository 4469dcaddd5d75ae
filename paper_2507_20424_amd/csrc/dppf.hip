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
//   * a tensor list is cut into tiles of kTileElems consecutive elements of one tensor; thread
//     blocks walk the tile list with a grid stride, so one launch covers any number of tensors
//     of any size.  Full tiles and partial ones (tensor tails, small tensors) are walked by
//     different blocks.  Loads are 16-byte vectors with 4-byte alignment (legal for global
//     memory on gfx9), so no tensor needs 16-byte alignment; only the last, partial vector of a
//     tensor is handled element by element.
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
#include <new>
#include <utility>
#include <vector>

#include "dppf.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));   // 16-byte vector that may sit on any 4-byte boundary

constexpr int kBlock = 256;                   // threads per block (4 waves)
constexpr int kTileElems = 4096;              // elements of ONE worker's tensor per tile
constexpr int kVecPerThread = kTileElems / (4 * kBlock);   // 16-byte vectors per thread per tile
constexpr int kMaxTemplM = 8;                 // worker counts with a register-resident kernel
constexpr int kMaxBlocksPerCU = 8;             // upper bound on resident blocks per CU (sizes buffers)
// Resident blocks per CU by traffic pattern (measured): kernels that mix reads and writes run
// fastest with ONE block per CU -- fewer concurrently open DRAM rows and longer same-direction
// bursts outweigh the lost latency hiding; kernels that only read do best with two.
constexpr int kBlocksPerCUReadOnly = 2;
constexpr int kBlocksPerCUReadWrite = 1;
// The fused AdamW sweep does a division and a square root per element between its loads and its
// stores; one wave per SIMD cannot hide that, so it gets more resident blocks.
constexpr int kBlocksPerCUHeavyMath = 3;

struct Tile {
  long long offset;   // first element inside the tensor
  int tensor;         // index into the tensor list
  int count;          // 1..kTileElems elements
};

struct Coef {
  float c;            // alpha - lambda / r_m
  int skip;           // r_m == 0: leave the worker untouched
};

// ------------------------------------------------------------------------------- helpers
template <bool FULL>
__device__ __forceinline__ f4 load4(const float* p, int n) {
  if (FULL || n >= 4) return *reinterpret_cast<const f4u*>(p);
  f4 r = {0.f, 0.f, 0.f, 0.f};
  if (n > 0) r.x = p[0];
  if (n > 1) r.y = p[1];
  if (n > 2) r.z = p[2];
  return r;
}

template <bool FULL>
__device__ __forceinline__ f4 load4_stream(const float* p, int n) {   // data not needed again soon
  if (FULL || n >= 4) return __builtin_nontemporal_load(reinterpret_cast<const f4u*>(p));
  return load4<false>(p, n);
}

template <bool FULL>
__device__ __forceinline__ void store4(float* p, f4 v, int n) {
  if (FULL || n >= 4) { *reinterpret_cast<f4u*>(p) = v; return; }
  if (n > 0) p[0] = v.x;
  if (n > 1) p[1] = v.y;
  if (n > 2) p[2] = v.z;
}

template <bool FULL>
__device__ __forceinline__ void store4_stream(float* p, f4 v, int n) {
  if (FULL || n >= 4) { __builtin_nontemporal_store(v, reinterpret_cast<f4u*>(p)); return; }
  store4<false>(p, v, n);
}

__device__ __forceinline__ f4 fma4(f4 a, float b, f4 c) {
  f4 r;
  r.x = __builtin_fmaf(a.x, b, c.x);
  r.y = __builtin_fmaf(a.y, b, c.y);
  r.z = __builtin_fmaf(a.z, b, c.z);
  r.w = __builtin_fmaf(a.w, b, c.w);
  return r;
}

__device__ __forceinline__ float sumsq4(f4 d, float acc) {
  acc = __builtin_fmaf(d.x, d.x, acc);
  acc = __builtin_fmaf(d.y, d.y, acc);
  acc = __builtin_fmaf(d.z, d.z, acc);
  acc = __builtin_fmaf(d.w, d.w, acc);
  return acc;
}

// The average is handled in coordinates relative to worker 0:  mu = (sum_j (x_j - x_0)) / M is
// the average minus x_0, and worker m's gap to the average is  x_A - x_m = mu - (x_m - x_0).
// The differences x_j - x_0 of nearby replicas are exact or nearly so, so the gap keeps its full
// relative precision instead of inheriting the rounding of x_A (an ulp of x, which the
// coefficient alpha - lambda/r multiplies -- by hundreds for a strong push).  For identical
// replicas every difference is exactly zero, so every gap is exactly zero for ANY M.  A
// power-of-two M multiplies by the exact reciprocal; any other M divides (correctly rounded), so
// a worker that sits exactly on a representable average gets an exactly zero gap as well.
__device__ __forceinline__ f4 scale_by_inverse_count(f4 s, int m_total, float inv_m) {
  if ((m_total & (m_total - 1)) == 0) return s * inv_m;
  const float mf = static_cast<float>(m_total);
  f4 q;
  q.x = s.x / mf;
  q.y = s.y / mf;
  q.z = s.z / mf;
  q.w = s.w / mf;
  return q;
}

template <int M>
__device__ __forceinline__ f4 mean_offset(const f4 (&x)[M], float inv_m) {
  f4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int m = 1; m < M; ++m) s += x[m] - x[0];
  return scale_by_inverse_count(s, M, inv_m);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Block-wide sums of M per-lane doubles; thread m < M writes the m-th sum to out[m].
template <int M>
__device__ __forceinline__ void block_sums_store(const double (&acc)[M], double* out) {
  __shared__ double lds[kBlock / 64][M];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int m = 0; m < M; ++m) {
    double s = wave_sum(acc[m]);
    if (lane == 0) lds[wave][m] = s;
  }
  __syncthreads();
  if (threadIdx.x < M) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) s += lds[w][threadIdx.x];
    out[threadIdx.x] = s;
  }
}

// The tile list holds all full tiles first, then the partial ones (tensor tails and tensors
// smaller than a tile).  Blocks [0, gfull) walk the full tiles with a stride of gfull; the
// remaining blocks walk the partial tiles.  A list of many small tensors therefore does not put
// short, latency-bound tiles into the streaming blocks' loops.
struct TileWalk {
  int first, end, stride;
  bool full;
};

__device__ __forceinline__ TileWalk tile_walk(int nfull, int ntiles, int gfull) {
  TileWalk w;
  if (static_cast<int>(blockIdx.x) < gfull) {
    w.first = blockIdx.x;
    w.end = nfull;
    w.stride = gfull;
    w.full = true;
  } else {
    w.first = nfull + static_cast<int>(blockIdx.x) - gfull;
    w.end = ntiles;
    w.stride = static_cast<int>(gridDim.x) - gfull;
    w.full = false;
  }
  return w;
}

// --------------------------------------------------------------------- sweep 1 of the round
// XBAR: 0 = average stays in registers, 1 = also written out, 2 = read from memory instead of
// being recomputed (dppf_dist_norms with a given x_A).
// KEEPX: load x through the caches (it is read again soon) instead of streaming it past them.
template <int M, int U, bool SGD, int XBAR, bool NORMS, bool FULL, bool KEEPX>
__device__ __forceinline__ void sweep1_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                            float* const* __restrict__ vp,
                                            const float* const* __restrict__ gp,
                                            float* const* __restrict__ xbarp, float lr, float mu,
                                            float wd, float inv_m, double (&acc)[M]) {
  float* x[M];
  float* v[M];
  const float* g[M];
#pragma unroll
  for (int m = 0; m < M; ++m) {
    x[m] = xp[m * T + tl.tensor] + tl.offset;
    if (SGD) {
      v[m] = vp[m * T + tl.tensor] + tl.offset;
      g[m] = gp[m * T + tl.tensor] + tl.offset;
    }
  }
  float* xb = (XBAR != 0) ? xbarp[tl.tensor] + tl.offset : nullptr;

  float part[M];
#pragma unroll
  for (int m = 0; m < M; ++m) part[m] = 0.f;

#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
    }
    f4 xv[U][M];
    if (SGD) {
      f4 vv[U][M], gv[U][M];
#pragma unroll
      for (int k = 0; k < U; ++k)
#pragma unroll
        for (int m = 0; m < M; ++m) {
          xv[k][m] = KEEPX ? load4<FULL>(x[m] + e[k], n[k]) : load4_stream<FULL>(x[m] + e[k], n[k]);
          vv[k][m] = load4_stream<FULL>(v[m] + e[k], n[k]);
          gv[k][m] = load4_stream<FULL>(g[m] + e[k], n[k]);
        }
#pragma unroll
      for (int k = 0; k < U; ++k)
#pragma unroll
        for (int m = 0; m < M; ++m) {
          // Alg. 1 local step with heavy-ball momentum: g' = g + wd x; v <- mu v + g'; x <- x - lr v
          f4 ge = fma4(xv[k][m], wd, gv[k][m]);
          f4 vn = fma4(vv[k][m], mu, ge);
          f4 xn = fma4(vn, -lr, xv[k][m]);
          store4_stream<FULL>(v[m] + e[k], vn, n[k]);
          // The stepped x is not written: sweep 2 re-derives it from the old x and the new v with
          // the same fused multiply-add (same bits), which trades 4 written bytes for 4 read bytes
          // per element -- reads are the cheaper direction.
          xv[k][m] = xn;
        }
    } else {
#pragma unroll
      for (int k = 0; k < U; ++k)
#pragma unroll
        for (int m = 0; m < M; ++m)
          xv[k][m] = KEEPX ? load4<FULL>(x[m] + e[k], n[k]) : load4_stream<FULL>(x[m] + e[k], n[k]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      if (XBAR == 2) {
        const f4 xbar = load4<FULL>(xb + e[k], n[k]);
        if (NORMS) {
#pragma unroll
          for (int m = 0; m < M; ++m) part[m] = sumsq4(xv[k][m] - xbar, part[m]);
        }
      } else {
        const f4 mu = mean_offset<M>(xv[k], inv_m);
        if (XBAR == 1) store4_stream<FULL>(xb + e[k], xv[k][0] + mu, n[k]);
        if (NORMS) {
#pragma unroll
          for (int m = 0; m < M; ++m) part[m] = sumsq4((xv[k][m] - xv[k][0]) - mu, part[m]);
        }
      }
    }
  }
  if (NORMS) {
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] += static_cast<double>(part[m]);
  }
}

template <int M, int U, bool SGD, int XBAR, bool NORMS>
__global__ __launch_bounds__(kBlock) void k_sweep1(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                   int gfull, int T,
                                                   float* const* __restrict__ xp,
                                                   float* const* __restrict__ vp,
                                                   const float* const* __restrict__ gp,
                                                   float* const* __restrict__ xbarp, float lr,
                                                   float mu, float wd, double* __restrict__ partials,
                                                   int pstride, int keep_from) {
  double acc[M];
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.full) {
    // Pure reads stream fastest when they bypass the last-level cache, but the tiles this sweep
    // touches last are the ones sweep 2 (which walks backwards) reads first: those, from
    // keep_from on, go through the cache so that sweep 2 finds them there.
    int t = w.first;
    for (; t < w.end && t < keep_from; t += w.stride)
      sweep1_tile<M, U, SGD, XBAR, NORMS, true, false>(tiles[t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m, acc);
    for (; t < w.end; t += w.stride)
      sweep1_tile<M, U, SGD, XBAR, NORMS, true, true>(tiles[t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m, acc);
  } else {
    for (int t = w.first; t < w.end; t += w.stride)
      sweep1_tile<M, U, SGD, XBAR, NORMS, false, true>(tiles[t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m, acc);
  }
  if (NORMS) block_sums_store<M>(acc, partials + static_cast<size_t>(blockIdx.x) * pstride);
}

// ------------------------------------------------------- partial sums -> r_m and c_m (Eq. 5)
// One block per worker; fixed summation order, fp64.
__global__ __launch_bounds__(kBlock) void k_finalize(const double* __restrict__ partials, int nparts,
                                                     int pstride, float pull, float push,
                                                     Coef* __restrict__ coef, float* __restrict__ r_out,
                                                     float* __restrict__ c_out) {
  __shared__ double lds[kBlock];
  const int m = blockIdx.x;
  double s = 0.0;
  for (int b = threadIdx.x; b < nparts; b += kBlock) s += partials[static_cast<size_t>(b) * pstride + m];
  lds[threadIdx.x] = s;
  __syncthreads();
  for (int off = kBlock / 2; off > 0; off >>= 1) {
    if (threadIdx.x < off) lds[threadIdx.x] += lds[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double r = sqrt(lds[0]);
    const bool zero = !(r > 0.0);
    // a worker sitting exactly on the average has no push direction: coefficient alpha, no move
    const double c = zero ? static_cast<double>(pull)
                          : static_cast<double>(pull) - static_cast<double>(push) / r;
    if (coef) {
      coef[m].c = static_cast<float>(c);
      coef[m].skip = zero ? 1 : 0;
    }
    if (r_out) r_out[m] = static_cast<float>(r);
    if (c_out) c_out[m] = static_cast<float>(c);
  }
}

// The same reduction done by every block of sweep 2 on its own (saves a launch): all blocks
// add the per-block partial sums of sweep 1 in the same fixed order, so all get the same bits.
template <int M>
__device__ __forceinline__ void coefficients_from_partials(const double* __restrict__ partials, int nparts,
                                                           int pstride, float pull, float push,
                                                           float (&c)[M], bool (&skip)[M],
                                                           float (&inv_r)[M],
                                                           float* __restrict__ r_out,
                                                           float* __restrict__ c_out) {
  __shared__ double lds[kBlock / 64][M];
  __shared__ float c_sh[M];
  __shared__ float inv_sh[M];
  __shared__ int skip_sh[M];
  double acc[M];
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] = 0.0;
  for (int b = threadIdx.x; b < nparts; b += kBlock) {
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] += partials[static_cast<size_t>(b) * pstride + m];
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int m = 0; m < M; ++m) {
    const double s = wave_sum(acc[m]);
    if (lane == 0) lds[wave][m] = s;
  }
  __syncthreads();
  if (threadIdx.x < M) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) s += lds[w][threadIdx.x];
    const double r = sqrt(s);
    const bool zero = !(r > 0.0);
    const double cc = zero ? static_cast<double>(pull)
                           : static_cast<double>(pull) - static_cast<double>(push) / r;
    c_sh[threadIdx.x] = static_cast<float>(cc);
    inv_sh[threadIdx.x] = zero ? 0.f : static_cast<float>(1.0 / r);
    skip_sh[threadIdx.x] = zero ? 1 : 0;
    if (blockIdx.x == 0) {
      if (r_out) r_out[threadIdx.x] = static_cast<float>(r);
      if (c_out) c_out[threadIdx.x] = static_cast<float>(cc);
    }
  }
  __syncthreads();
#pragma unroll
  for (int m = 0; m < M; ++m) {
    c[m] = c_sh[m];
    inv_r[m] = inv_sh[m];
    skip[m] = skip_sh[m] != 0;
  }
}

// --------------------------------------------------------------------- sweep 2 of the round
// Eq. 5: x_m <- x_m + (x_A - x_m) c_m, with x_A recomputed from the same M loads (XBAR == 0)
// or read from memory (XBAR == 2).
// STEP: x in memory is still the value from before the fused local step and v is already the
// new momentum; the stepped x is rebuilt as x - lr v before the update.
template <int M, int U, int XBAR, bool STEP, bool FULL>
__device__ __forceinline__ void sweep2_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                            const float* const* __restrict__ vp,
                                            const float* const* __restrict__ xbarp, float lr,
                                            const float (&c)[M], const bool (&skip)[M], float inv_m) {
  float* x[M];
  const float* v[M];
#pragma unroll
  for (int m = 0; m < M; ++m) {
    x[m] = xp[m * T + tl.tensor] + tl.offset;
    if (STEP) v[m] = vp[m * T + tl.tensor] + tl.offset;
  }
  const float* xb = (XBAR == 2) ? xbarp[tl.tensor] + tl.offset : nullptr;
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U][M];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
#pragma unroll
      for (int m = 0; m < M; ++m) xv[k][m] = load4_stream<FULL>(x[m] + e[k], n[k]);
    }
    if (STEP) {
      f4 vv[U][M];
#pragma unroll
      for (int k = 0; k < U; ++k)
#pragma unroll
        for (int m = 0; m < M; ++m) vv[k][m] = load4_stream<FULL>(v[m] + e[k], n[k]);
#pragma unroll
      for (int k = 0; k < U; ++k)
#pragma unroll
        for (int m = 0; m < M; ++m) xv[k][m] = fma4(vv[k][m], -lr, xv[k][m]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      // ref - (x_m - base) is the gap x_A - x_m: base = 0, ref = x_A when the average is given,
      // base = x_0, ref = mu otherwise
      const f4 ref = (XBAR == 2) ? load4_stream<FULL>(xb + e[k], n[k]) : mean_offset<M>(xv[k], inv_m);
      const f4 base = (XBAR == 2) ? (f4){0.f, 0.f, 0.f, 0.f} : xv[k][0];
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const f4 moved = fma4(ref - (xv[k][m] - base), c[m], xv[k][m]);
        store4_stream<FULL>(x[m] + e[k], skip[m] ? xv[k][m] : moved, n[k]);
      }
    }
  }
}

// FOLD: the coefficients are derived here from sweep 1's partial sums (no finalize launch);
// otherwise they are read from `coef`.
template <int M, int U, int XBAR, bool STEP, bool FOLD>
__global__ __launch_bounds__(kBlock) void k_sweep2(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                   int gfull, int T,
                                                   float* const* __restrict__ xp,
                                                   const float* const* __restrict__ vp,
                                                   const float* const* __restrict__ xbarp, float lr,
                                                   const Coef* __restrict__ coef, float inv_m_total,
                                                   const double* __restrict__ partials, int nparts,
                                                   int pstride, float pull, float push,
                                                   float* __restrict__ r_out, float* __restrict__ c_out) {
  float c[M];
  bool skip[M];
  if (FOLD) {
    float inv_r[M];
    coefficients_from_partials<M>(partials, nparts, pstride, pull, push, c, skip, inv_r, r_out, c_out);
  } else {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      c[m] = coef[m].c;
      skip[m] = coef[m].skip != 0;
    }
  }
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.first >= w.end) return;
  // opposite walk order to sweep 1
  const int last = (w.end - 1 - w.first) / w.stride;
  if (w.full) {
    for (int j = last; j >= 0; --j)
      sweep2_tile<M, U, XBAR, STEP, true>(tiles[w.first + j * w.stride], T, xp, vp, xbarp, lr, c, skip,
                                          inv_m_total);
  } else {
    for (int j = last; j >= 0; --j)
      sweep2_tile<M, U, XBAR, STEP, false>(tiles[w.first + j * w.stride], T, xp, vp, xbarp, lr, c, skip,
                                           inv_m_total);
  }
}

// ------------------------------------------------ sweep 2 with the exact two-term gradient
// Eq. 4 (a): x_m <- x_m - alpha d_m + (lambda_r / M^2) (M d_m/r_m - sum_j d_j/r_j), d = x - x_A.
// With gap = x_A - x (= -d):  x_m + gap_m (alpha - (lambda_r/M)/r_m) + (lambda_r/M^2) sum_j gap_j/r_j.
// All M replicas of an element are in registers here, so the sum over j costs no memory traffic.
// Workers at zero distance contribute a zero unit vector (1/r_j := 0) but still receive the sum.
template <int M, int U, bool FULL>
__device__ __forceinline__ void exact_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                           const float (&c)[M], const float (&inv_r)[M], float k2,
                                           float inv_m) {
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U][M];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
#pragma unroll
      for (int m = 0; m < M; ++m) xv[k][m] = load4_stream<FULL>(x[m] + e[k], n[k]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const f4 mu = mean_offset<M>(xv[k], inv_m);
      f4 usum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < M; ++m) usum = fma4(mu - (xv[k][m] - xv[k][0]), inv_r[m], usum);
#pragma unroll
      for (int m = 0; m < M; ++m) {
        f4 moved = fma4(mu - (xv[k][m] - xv[k][0]), c[m], xv[k][m]);
        moved = fma4(usum, k2, moved);
        store4_stream<FULL>(x[m] + e[k], moved, n[k]);
      }
    }
  }
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_update_exact(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                         int gfull, int T, float* const* __restrict__ xp,
                                                         const double* __restrict__ partials, int nparts,
                                                         int pstride, float pull, float push_over_m, float k2,
                                                         float* __restrict__ r_out, float* __restrict__ c_out) {
  float c[M], inv_r[M];
  bool skip[M];
  coefficients_from_partials<M>(partials, nparts, pstride, pull, push_over_m, c, skip, inv_r, r_out, c_out);
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.first >= w.end) return;
  const int last = (w.end - 1 - w.first) / w.stride;
  if (w.full) {
    for (int j = last; j >= 0; --j) exact_tile<M, U, true>(tiles[w.first + j * w.stride], T, xp, c, inv_r, k2, inv_m);
  } else {
    for (int j = last; j >= 0; --j) exact_tile<M, U, false>(tiles[w.first + j * w.stride], T, xp, c, inv_r, k2, inv_m);
  }
}

// ------------------------------------------- Alg. 1 written literally, any consensus variable
// pulled_m = (1 - alpha) x_m + alpha x_C; gap_m = pulled_m - ref (ref = x_A before the round, or x_C);
// r_m = ||gap_m||; x_m <- pulled_m + lambda gap_m / r_m  (no push where r_m = 0).
// REF: 0 = push away from the average, 1 = push away from the consensus variable.
template <int M, int U, int REF, bool WRITE, bool FULL>
__device__ __forceinline__ void seq_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                         const float* const* __restrict__ xcp, float pull, float keep,
                                         const float (&scale)[M], float inv_m, double (&acc)[M]) {
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
  const float* xc = xcp[tl.tensor] + tl.offset;
  float part[M];
#pragma unroll
  for (int m = 0; m < M; ++m) part[m] = 0.f;
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U][M], cv[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
      cv[k] = load4<FULL>(xc + e[k], n[k]);
#pragma unroll
      for (int m = 0; m < M; ++m)
        xv[k][m] = WRITE ? load4_stream<FULL>(x[m] + e[k], n[k]) : load4<FULL>(x[m] + e[k], n[k]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const f4 ref = (REF == 0) ? xv[k][0] + mean_offset<M>(xv[k], inv_m) : cv[k];
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const f4 pulled = fma4(cv[k], pull, xv[k][m] * keep);   // (1-alpha) x + alpha x_C: exactly x_C at alpha = 1
        const f4 gap = pulled - ref;
        if (WRITE) store4_stream<FULL>(x[m] + e[k], fma4(gap, scale[m], pulled), n[k]);
        else part[m] = sumsq4(gap, part[m]);
      }
    }
  }
  if (!WRITE) {
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] += static_cast<double>(part[m]);
  }
}

template <int M, int U, int REF>
__global__ __launch_bounds__(kBlock) void k_seq1(const Tile* __restrict__ tiles, int nfull, int ntiles, int gfull,
                                                 int T, float* const* __restrict__ xp,
                                                 const float* const* __restrict__ xcp, float pull, float keep,
                                                 double* __restrict__ partials, int pstride) {
  double acc[M];
  float scale[M];
#pragma unroll
  for (int m = 0; m < M; ++m) {
    acc[m] = 0.0;
    scale[m] = 0.f;
  }
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.full) {
    for (int t = w.first; t < w.end; t += w.stride)
      seq_tile<M, U, REF, false, true>(tiles[t], T, xp, xcp, pull, keep, scale, inv_m, acc);
  } else {
    for (int t = w.first; t < w.end; t += w.stride)
      seq_tile<M, U, REF, false, false>(tiles[t], T, xp, xcp, pull, keep, scale, inv_m, acc);
  }
  block_sums_store<M>(acc, partials + static_cast<size_t>(blockIdx.x) * pstride);
}

template <int M, int U, int REF>
__global__ __launch_bounds__(kBlock) void k_seq2(const Tile* __restrict__ tiles, int nfull, int ntiles, int gfull,
                                                 int T, float* const* __restrict__ xp,
                                                 const float* const* __restrict__ xcp, float pull, float keep,
                                                 float push, const double* __restrict__ partials, int nparts,
                                                 int pstride, float* __restrict__ r_post_out) {
  // lambda / r_m from the partial sums (c = 0 - push/r, so scale = -c; zero distance: no push)
  float c[M], scale[M], inv_r[M];
  bool skip[M];
  coefficients_from_partials<M>(partials, nparts, pstride, 0.f, push, c, skip, inv_r, r_post_out, nullptr);
#pragma unroll
  for (int m = 0; m < M; ++m) scale[m] = skip[m] ? 0.f : -c[m];
  double unused[M];
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.first >= w.end) return;
  const int last = (w.end - 1 - w.first) / w.stride;
  if (w.full) {
    for (int j = last; j >= 0; --j)
      seq_tile<M, U, REF, true, true>(tiles[w.first + j * w.stride], T, xp, xcp, pull, keep, scale, inv_m, unused);
  } else {
    for (int j = last; j >= 0; --j)
      seq_tile<M, U, REF, true, false>(tiles[w.first + j * w.stride], T, xp, xcp, pull, keep, scale, inv_m, unused);
  }
}

// ------------------------------------------------------------------ AdamW local step
// Decoupled weight decay Adam: x <- x (1 - lr wd); m <- b1 m + (1-b1) g; s <- b2 s + (1-b2) g^2;
// x <- x - lr (m / bc1) / (sqrt(s / bc2) + eps), bc_i = 1 - b_i^t computed on the host.
struct AdamHyper {
  float lr, b1, b2, eps, wd, inv_bc1, inv_bc2;
};

__device__ __forceinline__ void adamw_vec(const f4& xv, const f4& av, const f4& sv, const f4& gv,
                                          const AdamHyper& hp, f4& xn, f4& an, f4& sn) {
  const float* xs = reinterpret_cast<const float*>(&xv);
  const float* as = reinterpret_cast<const float*>(&av);
  const float* ss = reinterpret_cast<const float*>(&sv);
  const float* gs = reinterpret_cast<const float*>(&gv);
  float* xo = reinterpret_cast<float*>(&xn);
  float* ao = reinterpret_cast<float*>(&an);
  float* so = reinterpret_cast<float*>(&sn);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float xd = __builtin_fmaf(-hp.lr * hp.wd, xs[i], xs[i]);
    const float a = __builtin_fmaf(hp.b1, as[i], (1.0f - hp.b1) * gs[i]);
    const float q = __builtin_fmaf(hp.b2, ss[i], (1.0f - hp.b2) * gs[i] * gs[i]);
    const float denom = __builtin_sqrtf(q * hp.inv_bc2) + hp.eps;
    xo[i] = xd - hp.lr * (a * hp.inv_bc1) / denom;
    ao[i] = a;
    so[i] = q;
  }
}

template <int U, bool FULL>
__device__ __forceinline__ void adamw_tile(float* x, float* m1, float* m2, const float* g, int count,
                                           const AdamHyper hp) {
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U], av[U], sv[U], gv[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : count - e[k];
      xv[k] = load4_stream<FULL>(x + e[k], n[k]);
      av[k] = load4_stream<FULL>(m1 + e[k], n[k]);
      sv[k] = load4_stream<FULL>(m2 + e[k], n[k]);
      gv[k] = load4_stream<FULL>(g + e[k], n[k]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      f4 xn, an, sn;
      adamw_vec(xv[k], av[k], sv[k], gv[k], hp, xn, an, sn);
      store4_stream<FULL>(m1 + e[k], an, n[k]);
      store4_stream<FULL>(m2 + e[k], sn, n[k]);
      store4_stream<FULL>(x + e[k], xn, n[k]);
    }
  }
}

template <int U>
__global__ __launch_bounds__(kBlock) void k_adamw_step(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                       int gfull, int M, int T, float* const* __restrict__ xp,
                                                       float* const* __restrict__ ap, float* const* __restrict__ sp,
                                                       const float* const* __restrict__ gp, const AdamHyper hp) {
  const bool full = static_cast<int>(blockIdx.x) < gfull;
  const long long base = full ? 0 : nfull;
  const long long count = full ? nfull : ntiles - nfull;
  const long long first = full ? blockIdx.x : static_cast<long long>(blockIdx.x) - gfull;
  const long long stride = full ? gfull : static_cast<long long>(gridDim.x) - gfull;
  for (long long j = first; j < count * M; j += stride) {
    const int m = static_cast<int>(j / count);
    const Tile tl = tiles[base + (j - static_cast<long long>(m) * count)];
    const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
    float* x = xp[slot] + tl.offset;
    float* a = ap[slot] + tl.offset;
    float* q = sp[slot] + tl.offset;
    const float* g = gp[slot] + tl.offset;
    if (full) adamw_tile<U, true>(x, a, q, g, tl.count, hp);
    else adamw_tile<U, false>(x, a, q, g, tl.count, hp);
  }
}

// Sweep 1 of the round with the AdamW step folded in: read x, m1, m2, g of all M workers, step,
// write m1, m2 and the stepped x (unlike SGD it cannot be rebuilt later from one extra read),
// accumulate the squared distances of the stepped x.  28 bytes per replica-parameter; the plain
// sweep 2 follows (8 bytes): 36 instead of 40.
template <int M, int U, bool FULL>
__device__ __forceinline__ void adamw_reduce_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                                  float* const* __restrict__ ap, float* const* __restrict__ sp,
                                                  const float* const* __restrict__ gp, const AdamHyper hp,
                                                  float inv_m, double (&acc)[M]) {
  float part[M];
#pragma unroll
  for (int m = 0; m < M; ++m) part[m] = 0.f;
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U][M], av[U][M], sv[U][M], gv[U][M];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
        xv[k][m] = load4_stream<FULL>(xp[slot] + tl.offset + e[k], n[k]);
        av[k][m] = load4_stream<FULL>(ap[slot] + tl.offset + e[k], n[k]);
        sv[k][m] = load4_stream<FULL>(sp[slot] + tl.offset + e[k], n[k]);
        gv[k][m] = load4_stream<FULL>(gp[slot] + tl.offset + e[k], n[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
#pragma unroll
      for (int m = 0; m < M; ++m) {
        const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
        f4 xn, an, sn;
        adamw_vec(xv[k][m], av[k][m], sv[k][m], gv[k][m], hp, xn, an, sn);
        store4_stream<FULL>(ap[slot] + tl.offset + e[k], an, n[k]);
        store4_stream<FULL>(sp[slot] + tl.offset + e[k], sn, n[k]);
        store4<FULL>(xp[slot] + tl.offset + e[k], xn, n[k]);     // read again by sweep 2
        xv[k][m] = xn;
      }
      const f4 mo = mean_offset<M>(xv[k], inv_m);
#pragma unroll
      for (int m = 0; m < M; ++m) part[m] = sumsq4((xv[k][m] - xv[k][0]) - mo, part[m]);
    }
  }
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] += static_cast<double>(part[m]);
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_adamw_reduce(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                         int gfull, int T, float* const* __restrict__ xp,
                                                         float* const* __restrict__ ap,
                                                         float* const* __restrict__ sp,
                                                         const float* const* __restrict__ gp, const AdamHyper hp,
                                                         double* __restrict__ partials, int pstride) {
  double acc[M];
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  if (w.full) {
    for (int t = w.first; t < w.end; t += w.stride)
      adamw_reduce_tile<M, U, true>(tiles[t], T, xp, ap, sp, gp, hp, inv_m, acc);
  } else {
    for (int t = w.first; t < w.end; t += w.stride)
      adamw_reduce_tile<M, U, false>(tiles[t], T, xp, ap, sp, gp, hp, inv_m, acc);
  }
  block_sums_store<M>(acc, partials + static_cast<size_t>(blockIdx.x) * pstride);
}

// ------------------------------------------------ by-products the paper logs every round
// out[0] = relaxed MV = (1/M) sum r_m; out[1..M] = pull strength alpha r_m; out[M+1..2M] = lambda.
__global__ void k_round_stats(const float* __restrict__ r, int M, float pull, float push, float* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double s = 0.0;
    for (int m = 0; m < M; ++m) s += static_cast<double>(r[m]);
    out[0] = static_cast<float>(s / M);
  }
  for (int m = threadIdx.x; m < M; m += blockDim.x) {
    out[1 + m] = pull * r[m];
    out[1 + M + m] = push;
  }
}

// ----------------------------------------------------------------- stand-alone local step
template <int U, bool FULL>
__device__ __forceinline__ void local_tile(float* x, float* v, const float* g, int count, float lr,
                                           float mu, float wd) {
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
    int e[U], n[U];
    f4 xv[U], vv[U], gv[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : count - e[k];
      xv[k] = load4_stream<FULL>(x + e[k], n[k]);
      vv[k] = load4_stream<FULL>(v + e[k], n[k]);
      gv[k] = load4_stream<FULL>(g + e[k], n[k]);
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const f4 ge = fma4(xv[k], wd, gv[k]);
      const f4 vn = fma4(vv[k], mu, ge);
      const f4 xn = fma4(vn, -lr, xv[k]);
      store4_stream<FULL>(v + e[k], vn, n[k]);
      store4_stream<FULL>(x + e[k], xn, n[k]);
    }
  }
}

template <int U>
__global__ __launch_bounds__(kBlock) void k_local_step(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                       int gfull, int M, int T,
                                                       float* const* __restrict__ xp,
                                                       float* const* __restrict__ vp,
                                                       const float* const* __restrict__ gp, float lr,
                                                       float mu, float wd) {
  // work items are (tile, worker) pairs; blocks [0, gfull) take the full tiles
  const bool full = static_cast<int>(blockIdx.x) < gfull;
  const long long base = full ? 0 : nfull;
  const long long count = full ? nfull : ntiles - nfull;
  const long long first = full ? blockIdx.x : static_cast<long long>(blockIdx.x) - gfull;
  const long long stride = full ? gfull : static_cast<long long>(gridDim.x) - gfull;
  for (long long j = first; j < count * M; j += stride) {
    const int m = static_cast<int>(j / count);
    const Tile tl = tiles[base + (j - static_cast<long long>(m) * count)];
    const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
    float* x = xp[slot] + tl.offset;
    float* v = vp[slot] + tl.offset;
    const float* g = gp[slot] + tl.offset;
    if (full)
      local_tile<U, true>(x, v, g, tl.count, lr, mu, wd);
    else
      local_tile<U, false>(x, v, g, tl.count, lr, mu, wd);
  }
}

// ------------------------------------------- average over a runtime number of workers (M > 8)
template <bool FULL>
__device__ __forceinline__ void mean_any_tile(const Tile tl, int M, int T,
                                              float* const* __restrict__ xp, float* xb, float inv_m) {
#pragma unroll 1
  for (int it = 0; it < kVecPerThread; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    const int n = FULL ? 4 : tl.count - e;
    const f4 x0 = load4<FULL>(xp[tl.tensor] + tl.offset + e, n);
    f4 s = {0.f, 0.f, 0.f, 0.f};
    for (int m = 1; m < M; ++m) s += load4<FULL>(xp[static_cast<size_t>(m) * T + tl.tensor] + tl.offset + e, n) - x0;
    store4<FULL>(xb + e, x0 + scale_by_inverse_count(s, M, inv_m), n);
  }
}

__global__ __launch_bounds__(kBlock) void k_mean_any(const Tile* __restrict__ tiles, int nfull, int ntiles,
                                                     int gfull, int M, int T,
                                                     float* const* __restrict__ xp,
                                                     float* const* __restrict__ xbarp) {
  const float inv_m = 1.0f / static_cast<float>(M);
  const TileWalk w = tile_walk(nfull, ntiles, gfull);
  for (int t = w.first; t < w.end; t += w.stride) {
    const Tile tl = tiles[t];
    float* xb = xbarp[tl.tensor] + tl.offset;
    if (w.full) mean_any_tile<true>(tl, M, T, xp, xb, inv_m);
    else mean_any_tile<false>(tl, M, T, xp, xb, inv_m);
  }
}

// ---------------------------------------------- plain copy (bandwidth / counter calibration)
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
// and written by the same lane).  Gives the device's practical bandwidth for a given read/write
// mix, the ceiling the DPPF kernels are compared with.
template <int R, int W, int U, bool INPLACE>
__global__ __launch_bounds__(kBlock) void k_probe(float* __restrict__ base, long long stride, long long n,
                                                  float* __restrict__ sink) {
  const long long tile = static_cast<long long>(kBlock) * U * 4;
  const long long ntiles = n / tile;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  for (long long t = blockIdx.x; t < ntiles; t += gridDim.x) {
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
  if (W == 0 && acc.x + acc.y + acc.z + acc.w == 123.456f) sink[0] = acc.x;   // keeps the loads alive
}

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
  double* partials = nullptr;   // [max blocks][M]
  int partials_rows = 0;
  Coef* coef = nullptr;         // [M]
  float* xbar_scratch = nullptr;            // d floats, only when M > kMaxTemplM
  std::vector<long long> tensor_offset;     // start of tensor t inside xbar_scratch
  enum Role { RX = 0, RV, RG, RM1, RM2, RXBAR, RXBAR_SCRATCH, RXC, NROLES };
  PtrTable tab[NROLES];
  // resident blocks per CU of each kernel that has been launched (queried once)
  std::vector<std::pair<const void*, int>> occupancy;
  // timing
  bool timing = false;
  std::vector<TimingRec> recs;
  std::vector<hipEvent_t> event_pool;
};

namespace {

int table_upload(dppf_plan* p, int role, const void* const* host, size_t n, hipStream_t s,
                 const void*** dev_out) {
  PtrTable& t = p->tab[role];
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
  for (const auto& kv : p->occupancy)
    if (kv.first == key) per_cu = kv.second;
  if (per_cu == 0) {
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kBlock, 0));
    if (per_cu < 1) per_cu = 1;
    p->occupancy.emplace_back(key, per_cu);
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
  *grid_out = static_cast<int>(gfull + gpart);   // <= num_cu * kMaxBlocksPerCU = partials_rows
  return DPPF_OK;
}

struct GridShape {
  int gfull = 0, grid = 0;
};

// Which of sweep 1's x loads go through the caches (see k_sweep1).
enum KeepPolicy {
  kKeepAll,      // every tile: sweep 2 follows and the loads are not the bottleneck (fused sweep 1)
  kKeepTail,     // only the tiles touched last, as many as fit the last-level cache budget
  kKeepNone      // nothing reads x again soon
};
constexpr long long kLastLevelCacheBudget = 256ll << 20;   // bytes of x worth keeping (the cache is 256 MB)

int keep_from_tile(const dppf_plan* p, int workers, KeepPolicy keep) {
  if (keep == kKeepAll) return 0;
  if (keep == kKeepNone) return p->nfull;
  const long long per_tile = static_cast<long long>(workers) * kTileElems * sizeof(float);
  const long long tiles = kLastLevelCacheBudget / per_tile;
  return tiles >= p->nfull ? 0 : p->nfull - static_cast<int>(tiles);
}

constexpr int unroll_plain(int M) { return M <= 4 ? 4 : (M <= 8 ? 2 : 1); }   // M*U <= 16 vectors
constexpr int unroll_step_update(int M) { return M <= 2 ? 4 : (M <= 4 ? 2 : 1); }   // 2*M*U <= 16 vectors
constexpr int unroll_fused(int M) { return M <= 2 ? 4 : (M <= 4 ? 2 : 1); }   // 3*M*U <= 24 vectors

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
    default: return DPPF_ELIMIT;                                   \
  }

// Launch sweep 1 over workers [m0, m0+mg) of the table (mg <= 8).
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
    int grid = 0, gfull = 0;
    if (shape && shape->grid > 0) {   // later worker groups must fill the same rows of the partial sums
      gfull = shape->gfull;
      grid = shape->grid;
    } else {
      int rc = grid_for(p, kern, 1, (SGD || XBAR == 1) ? kBlocksPerCUReadWrite : kBlocksPerCUReadOnly, &gfull,
                        &grid);
      if (rc) return rc;
      if (shape) {
        shape->gfull = gfull;
        shape->grid = grid;
      }
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T, x, v, g, xb,
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
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T, x, v, xb, lr,
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
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->M, p->T,
                     (float* const*)(xp), (float* const*)(vp),
                     (const float* const*)(gp), lr, mu, wd);
  HIP_TRY(hipGetLastError());
  return timing_end(p, s);
}

int launch_mean_any(dppf_plan* p, const void** xp, const void** xbarp, hipStream_t s) {
  int grid = 0, gfull = 0;
  int rc = grid_for(p, k_mean_any, 1, kBlocksPerCUReadWrite, &gfull, &grid);
  if (rc) return rc;
  hipLaunchKernelGGL(k_mean_any, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->M, p->T,
                     (float* const*)(xp), (float* const*)(xbarp));
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
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T, x,
                       p->partials, nparts, p->M, pull, push_r / mf, push_r / (mf * mf), r_out, c_out);
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

template <int REF>
int launch_seq(dppf_plan* p, const void** xp, const void** xcp, float pull, float push, float* r_post_out,
               hipStream_t s) {
  float* const* x = (float* const*)(xp);
  const float* const* xc = (const float* const*)(xcp);
  const float keep = static_cast<float>(1.0 - static_cast<double>(pull));
  int rc;
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = unroll_plain(kM) > 2 ? 2 : unroll_plain(kM);
    auto k1 = k_seq1<kM, kU, REF>;
    auto k2 = k_seq2<kM, kU, REF>;
    int grid = 0, gfull = 0;
    if ((rc = grid_for(p, k1, 1, kBlocksPerCUReadOnly, &gfull, &grid))) return rc;
    if ((rc = timing_begin(p, DPPF_K_SEQ_REDUCE, s))) return rc;
    hipLaunchKernelGGL(k1, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T, x, xc,
                       pull, keep, p->partials, p->M);
    if ((rc = timing_end(p, s))) return rc;
    const int nparts = grid;
    if ((rc = grid_for(p, k2, 1, kBlocksPerCUReadWrite, &gfull, &grid))) return rc;
    if ((rc = timing_begin(p, DPPF_K_SEQ_UPDATE, s))) return rc;
    hipLaunchKernelGGL(k2, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T, x, xc,
                       pull, keep, push, p->partials, nparts, p->M, r_post_out);
    if ((rc = timing_end(p, s))) return rc;
  })
  HIP_TRY(hipGetLastError());
  return DPPF_OK;
}

// The scratch average used when M > 8: a pointer table into the plan's own d-vector.
int scratch_xbar_table(dppf_plan* p, hipStream_t s, const void*** dev_out) {
  std::vector<const void*> host(static_cast<size_t>(p->T));
  for (int t = 0; t < p->T; ++t) host[t] = p->xbar_scratch + p->tensor_offset[t];
  return table_upload(p, dppf_plan::RXBAR_SCRATCH, host.data(), host.size(), s, dev_out);
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
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->M, p->T,
                     (float* const*)(xd), (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp);
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
      rc = xbar_out ? launch_sweep1<true, 1, true>(p, p->M, xd, vd, gd, xbd, lr, mu, wd, 0, kKeepAll, &shape, s)
                    : launch_sweep1<true, 0, true>(p, p->M, xd, vd, gd, nullptr, lr, mu, wd, 0, kKeepAll, &shape, s);
    } else {
      rc = xbar_out ? launch_sweep1<false, 1, true>(p, p->M, xd, nullptr, nullptr, xbd, 0, 0, 0, 0, kKeepTail, &shape, s)
                    : launch_sweep1<false, 0, true>(p, p->M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepTail, &shape, s);
    }
    if (rc) return rc;
    if ((rc = timing_end(p, s))) return rc;
    if ((rc = timing_begin(p, with_step ? DPPF_K_STEP_UPDATE : DPPF_K_UPDATE, s))) return rc;
    if (with_step)
      rc = launch_sweep2<0, true, true>(p, p->M, xd, vd, nullptr, lr, 0, shape.grid, pull, push, r_out, c_out, s);
    else
      rc = launch_sweep2<0, false, true>(p, p->M, xd, nullptr, nullptr, 0.f, 0, shape.grid, pull, push, r_out, c_out, s);
    if (rc) return rc;
    return timing_end(p, s);
  }
  // M > 8: materialise the average once, then run the register-resident kernels over groups
  // of up to 8 workers that read it back.
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
  if ((rc = launch_finalize(p, shape.grid, pull, push, true, r_out, c_out, s))) return rc;
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
  if (p->xbar_scratch) (void)hipFree(p->xbar_scratch);
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
  try {
    p->numel.resize(static_cast<size_t>(T));
    p->tensor_offset.resize(static_cast<size_t>(T) + 1, 0);
    for (int t = 0; t < T; ++t) {
      if (numel[t] < 0) { delete p; return DPPF_EINVAL; }
      p->numel[t] = numel[t];
      p->tensor_offset[t] = p->d;
      p->d += numel[t];
      for (long long off = 0; off < numel[t]; off += kTileElems) {
        const long long left = numel[t] - off;
        tiles.push_back(Tile{off, t, static_cast<int>(left < kTileElems ? left : kTileElems)});
      }
      if (tiles.size() > static_cast<size_t>(INT32_MAX / 2)) { delete p; return DPPF_ELIMIT; }
    }
    p->tensor_offset[T] = p->d;
  } catch (const std::bad_alloc&) {
    delete p;
    return DPPF_ENOMEM;
  }
  {   // full tiles first (list order kept inside each group)
    std::vector<Tile> ordered;
    try {
      ordered.reserve(tiles.size());
      for (const Tile& t : tiles) if (t.count == kTileElems) ordered.push_back(t);
      p->nfull = static_cast<int>(ordered.size());
      for (const Tile& t : tiles) if (t.count != kTileElems) ordered.push_back(t);
    } catch (const std::bad_alloc&) {
      delete p;
      return DPPF_ENOMEM;
    }
    tiles.swap(ordered);
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
  p->partials_rows = p->num_cu * kMaxBlocksPerCU;
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->tiles_dev), (tiles.size() + 1) * sizeof(Tile)));
  if (!tiles.empty())
    PLAN_TRY(hipMemcpy(p->tiles_dev, tiles.data(), tiles.size() * sizeof(Tile), hipMemcpyHostToDevice));
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->partials),
                     static_cast<size_t>(p->partials_rows) * M * sizeof(double)));
  PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->coef), static_cast<size_t>(M) * sizeof(Coef)));
  if (M > kMaxTemplM && p->d > 0)
    PLAN_TRY(hipMalloc(reinterpret_cast<void**>(&p->xbar_scratch), static_cast<size_t>(p->d) * sizeof(float)));
  const size_t n = static_cast<size_t>(M) * T;
  for (int r = 0; r < dppf_plan::NROLES; ++r) {
    const bool per_model = (r == dppf_plan::RXBAR || r == dppf_plan::RXBAR_SCRATCH || r == dppf_plan::RXC);
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
      if ((rc = launch_mean_any(p, xd, avg, s))) return rc;
    }
    if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
    for (int m0 = 0; m0 < p->M; m0 += kMaxTemplM) {
      const int mg = (p->M - m0 < kMaxTemplM) ? p->M - m0 : kMaxTemplM;
      if ((rc = launch_sweep1<false, 2, true>(p, mg, xd, nullptr, nullptr, avg, 0, 0, 0, m0, kKeepNone, &shape, s))) return rc;
    }
    if ((rc = timing_end(p, s))) return rc;
  }
  return launch_finalize(p, shape.grid, 0.f, 0.f, false, r_out, nullptr, s);
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
  if (p->M > kMaxTemplM) return DPPF_ELIMIT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const void** xd = nullptr;
  int rc;
  if ((rc = table_upload(p, dppf_plan::RX, reinterpret_cast<const void* const*>(x),
                         static_cast<size_t>(p->M) * p->T, s, &xd)))
    return rc;
  if (p->ntiles == 0) return launch_finalize(p, 0, pull, push_r / static_cast<float>(p->M), false, r_out, c_out, s);
  GridShape shape;
  if ((rc = timing_begin(p, DPPF_K_REDUCE, s))) return rc;
  if ((rc = launch_sweep1<false, 0, true>(p, p->M, xd, nullptr, nullptr, nullptr, 0, 0, 0, 0, kKeepTail, &shape, s))) return rc;
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_UPDATE_EXACT, s))) return rc;
  if ((rc = launch_update_exact(p, xd, shape.grid, pull, push_r, r_out, c_out, s))) return rc;
  return timing_end(p, s);
} DPPF_CATCH

int dppf_pull_then_push(dppf_plan* p, float* const* x, const float* const* x_c, float pull, float push,
                        int push_from, float* r_post_out, void* stream) try {
  if (!p || !x || !x_c || (push_from != DPPF_PUSH_FROM_AVERAGE && push_from != DPPF_PUSH_FROM_CONSENSUS))
    return DPPF_EINVAL;
  if (p->M > kMaxTemplM) return DPPF_ELIMIT;
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
  return push_from == DPPF_PUSH_FROM_AVERAGE ? launch_seq<0>(p, xd, xcd, pull, push, r_post_out, s)
                                             : launch_seq<1>(p, xd, xcd, pull, push, r_post_out, s);
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
  int grid = 0, gfull = 0;
  if ((rc = timing_begin(p, DPPF_K_ADAMW_REDUCE, s))) return rc;
  DPPF_SWITCH_M(p->M, {
    constexpr int kU = kM <= 2 ? 2 : 1;     // 4*M*U <= 32 vectors in flight
    auto kern = k_adamw_reduce<kM, kU>;
    if ((rc = grid_for(p, kern, 1, kBlocksPerCUHeavyMath, &gfull, &grid))) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, s, p->tiles_dev, p->nfull, p->ntiles, gfull, p->T,
                       (float* const*)(xd), (float* const*)(ad), (float* const*)(sd), (const float* const*)(gd), hp,
                       p->partials, p->M);
  })
  HIP_TRY(hipGetLastError());
  if ((rc = timing_end(p, s))) return rc;
  if ((rc = timing_begin(p, DPPF_K_UPDATE, s))) return rc;
  if ((rc = launch_sweep2<0, false, true>(p, p->M, xd, nullptr, nullptr, 0.f, 0, grid, pull, push, r_out, c_out, s)))
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
                           int blocks_per_cu, void* stream) {
  if (!base || n < 0 || stride < n || blocks_per_cu < 1 || blocks_per_cu > 16) return DPPF_EINVAL;
  if (reinterpret_cast<uintptr_t>(base) & 15u || (stride & 3)) return DPPF_EINVAL;
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const dim3 grid(static_cast<unsigned>(cus * blocks_per_cu)), block(kBlock);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* sink = base;   // never written unless a sum hits one magic value
#define DPPF_PROBE(R_, W_, U_, IP_)                                                              \
  if (reads == R_ && writes == W_ && (inplace != 0) == IP_) {                                    \
    hipLaunchKernelGGL((k_probe<R_, W_, U_, IP_>), grid, block, 0, s, base, static_cast<long long>(stride), \
                       static_cast<long long>(n), sink);                                         \
    HIP_TRY(hipGetLastError());                                                                  \
    return DPPF_OK;                                                                              \
  }
  DPPF_PROBE(1, 0, 4, false)
  DPPF_PROBE(4, 0, 4, false)
  DPPF_PROBE(12, 0, 1, false)
  DPPF_PROBE(0, 1, 4, false)
  DPPF_PROBE(0, 4, 4, false)
  DPPF_PROBE(1, 1, 4, false)
  DPPF_PROBE(4, 4, 2, false)
  DPPF_PROBE(4, 4, 2, true)
  DPPF_PROBE(8, 4, 1, false)
  DPPF_PROBE(8, 4, 1, true)
  DPPF_PROBE(12, 4, 1, false)
  DPPF_PROBE(12, 4, 1, true)
  DPPF_PROBE(12, 8, 1, false)
  DPPF_PROBE(12, 8, 1, true)
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
  int n = 0;
  for (auto& r : p->recs) {
    HIP_TRY(hipEventSynchronize(r.stop));
    if (n < cap) {
      float t = 0.f;
      HIP_TRY(hipEventElapsedTime(&t, r.start, r.stop));
      kernel_id[n] = r.id;
      ms[n] = t;
      ++n;
    }
    p->event_pool.push_back(r.start);
    p->event_pool.push_back(r.stop);
  }
  p->recs.clear();
  return n;
} DPPF_CATCH

}  // extern "C"
