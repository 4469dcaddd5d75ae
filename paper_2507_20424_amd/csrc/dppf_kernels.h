// Device code of the DPPF library: tile walk, load/store helpers and every kernel.
// Included once, by dppf.hip (which holds the plan, the launchers and the C ABI).
#ifndef DPPF_KERNELS_H_
#define DPPF_KERNELS_H_

#include <hip/hip_runtime.h>

#include <type_traits>

namespace {


typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));   // 16-byte vector that may sit on any 4-byte boundary

constexpr int kBlock = 256;                   // threads per block (4 waves)
constexpr int kTileElems = 4096;              // elements of ONE worker's tensor per tile (DPPF_TILE_ELEMS)
constexpr int kVecPerThread = kTileElems / (4 * kBlock);   // 16-byte vectors per thread per tile
constexpr int kMaxTemplM = 16;                 // worker counts with a register-resident kernel
constexpr int kAnyChunk = 4;                   // workers whose loads the any-M kernels keep in flight together
constexpr int kMaxBlocksPerCU = 8;             // upper bound on resident blocks per CU (sizes buffers)
// Resident blocks per CU by traffic pattern (measured): kernels that mix reads and writes run
// fastest with ONE block per CU -- fewer concurrently open DRAM rows and longer same-direction
// bursts outweigh the lost latency hiding; kernels that only read do best with two.
constexpr int kBlocksPerCUReadOnly = 2;
constexpr int kBlocksPerCUReadWrite = 1;
struct Tile {
  long long offset;   // first element inside the tensor
  int tensor;         // index into the tensor list
  int count;          // 1..kTileElems elements
};

struct Coef {
  float c;            // alpha - lambda / r_m
  int skip;           // r_m == 0: leave the worker untouched
  float inv_r;        // 1 / r_m, 0 where r_m == 0
};

// ------------------------------------------------------------------------------- helpers
// Tensor data always live in device (global) memory.  The pointers come out of pointer tables, so
// the compiler cannot know that and would use flat addressing; these types tell it.
typedef __attribute__((address_space(1))) const f4u* gvec_in;
typedef __attribute__((address_space(1))) f4u* gvec_out;
typedef __attribute__((address_space(1))) const float* gf_in;
typedef __attribute__((address_space(1))) float* gf_out;

template <bool FULL>
__device__ __forceinline__ f4 load4(const float* p, int n) {
  if (FULL || n >= 4) return *(gvec_in)(p);
  gf_in q = (gf_in)(p);
  f4 r = {0.f, 0.f, 0.f, 0.f};
  if (n > 0) r.x = q[0];
  if (n > 1) r.y = q[1];
  if (n > 2) r.z = q[2];
  return r;
}

template <bool FULL>
__device__ __forceinline__ f4 load4_stream(const float* p, int n) {   // data not needed again soon
  if (FULL || n >= 4) return __builtin_nontemporal_load((gvec_in)(p));
  return load4<false>(p, n);
}

template <bool FULL>
__device__ __forceinline__ void store4(float* p, f4 v, int n) {
  if (FULL || n >= 4) { *(gvec_out)(p) = v; return; }
  gf_out q = (gf_out)(p);
  if (n > 0) q[0] = v.x;
  if (n > 1) q[1] = v.y;
  if (n > 2) q[2] = v.z;
}

template <bool FULL>
__device__ __forceinline__ void store4_stream(float* p, f4 v, int n) {
  if (FULL || n >= 4) { __builtin_nontemporal_store(v, (gvec_out)(p)); return; }
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

// Block-wide sums of M per-lane doubles; thread m < M writes the m-th sum to out[m].  The per-lane
// values are set back to zero.  May be called repeatedly by a block, with at least one barrier
// between two calls (the loop of walk_items has them).
template <int M>
__device__ __forceinline__ void block_sums_flush(double (&acc)[M], double* out) {
  __shared__ double lds[kBlock / 64][M];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int m = 0; m < M; ++m) {
    double s = wave_sum(acc[m]);
    if (lane == 0) lds[wave][m] = s;
    acc[m] = 0.0;
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
// smaller than a tile).  Blocks [0, gfull) take the full tiles, the remaining blocks the partial
// ones, so a list of many small tensors does not put short, latency-bound tiles into the streaming
// blocks' loops.
//
// Full tiles are work ITEMS (one per tile, or one per (two tiles, worker) pair).  Items [0, nstatic) go
// to the blocks with a fixed stride; items [nstatic, count) are handed out on demand from a counter
// in device memory.  The compute dies of the chip do not stream at the same rate (blocks on some
// finish a fixed share about 10 % earlier than on others), and with a fixed split the early ones
// idle while the late ones finish; handing out the tail on demand keeps every CU busy to the end.
// The counter resets itself: the last block to leave puts it back to zero, so every launch finds
// it clean and nothing has to be cleared between launches (also inside a captured graph).
struct Sched {
  unsigned int next;   // next on-demand item to hand out
  unsigned int done;   // full-tile blocks that have left the kernel
};

struct Walk {
  int nfull, ntiles;   // tiles [0, nfull) are full, [nfull, ntiles) partial
  int gfull;           // blocks [0, gfull) take full tiles
  int nitems;          // full-tile work items: one per tile, or one per (pair of tiles, worker)
  int nstatic;         // full-tile items with a fixed owner; the rest are handed out on demand
  Sched* sched;        // used only when nstatic < nitems
};

// The kernels that handle one worker at a time (local steps) take two full tiles per item: one
// tile of one worker is only about 3 microseconds of traffic, too little to hide the request for
// the next item behind (measured: two tiles 3-6 % faster than one, three or four slower again;
// the sweeps that take all workers of a tile together are fastest with one tile per item).
constexpr int kTilesPerWorkerItem = 2;

using FullTile = std::integral_constant<bool, true>;
using PartialTile = std::integral_constant<bool, false>;

// Calls body(item, FullTile{} or PartialTile{}) for every item of this block, all threads of the
// block together.  item counts within the full tiles or within the partial tiles.  A block owns
// the items congruent to its index (modulo the number of blocks on that part of the list) in the
// forward and in the REVERSE walk alike, so on a small model sweep 2 finds in its die's L2 what
// sweep 1 left there.  REVERSE walks from the far end: the fixed shares are the upper items and the
// on-demand ones run down to item 0, so sweep 2 starts where sweep 1 stopped, whose data are still
// in the last-level cache.  flush(row) is called with row = blockIdx.x once the block's fixed share
// (or its partial tiles) is done, and with row = gridDim.x + k after the k-th on-demand item:
// kernels that reduce store their partial sums there, so that the set of rows and what each row
// holds never depend on which block took which item -- results stay bit-reproducible.
template <bool REVERSE, typename Body, typename Flush>
__device__ __forceinline__ void walk_items(const Walk& w, int per_tile, Body&& body, Flush&& flush) {
  __shared__ int s_next[2];
  const bool full = static_cast<int>(blockIdx.x) < w.gfull;
  const int me = full ? static_cast<int>(blockIdx.x) : static_cast<int>(blockIdx.x) - w.gfull;
  const int lanes = full ? w.gfull : static_cast<int>(gridDim.x) - w.gfull;
  const int count = full ? w.nitems : (w.ntiles - w.nfull) * per_tile;
  // last item this block owns (below `me` if it owns none)
  const int last_owned = count > me ? me + ((count - 1 - me) / lanes) * lanes : me - lanes;
  if (!full) {
    if (REVERSE) {
      for (int j = last_owned; j >= me; j -= lanes) body(j, PartialTile{});
    } else {
      for (int j = me; j < count; j += lanes) body(j, PartialTile{});
    }
    flush(static_cast<int>(blockIdx.x));
    return;
  }
  const int ndyn = count - w.nstatic;            // items handed out on demand
  const int lo = REVERSE ? ndyn : 0;             // fixed shares are the items [lo, lo + nstatic)
  // The first on-demand item is requested right away: the answer is there long before it is needed.
  unsigned int fetched = 0;
  if (ndyn > 0 && threadIdx.x == 0) fetched = atomicAdd(&w.sched->next, 1u);
  int j = REVERSE ? last_owned : me;
  bool on_demand = false;
  int slot = 0;   // the item number travels from thread 0 to the block through two alternating words:
                  // one barrier per item is enough, the next write goes to the other word
  for (;;) {
    if (!on_demand && (REVERSE ? j < lo : j >= lo + w.nstatic)) {
      flush(static_cast<int>(blockIdx.x));
      if (ndyn <= 0) break;
      on_demand = true;
    }
    int k = 0;
    if (on_demand) {
      if (threadIdx.x == 0) s_next[slot] = static_cast<int>(fetched);
      __syncthreads();
      k = s_next[slot];
      slot ^= 1;
      if (k >= ndyn) break;            // every block gets here: the counter only grows
      if (threadIdx.x == 0) fetched = atomicAdd(&w.sched->next, 1u);   // the one after, while this one runs
      j = REVERSE ? ndyn - 1 - k : w.nstatic + k;
    }
    body(j, FullTile{});
    if (on_demand) flush(static_cast<int>(gridDim.x) + k);
    else j += REVERSE ? -lanes : lanes;
  }
  // A block counts itself out only after its last request has been answered, so when the count is
  // complete nobody will touch the counter again in this launch.
  if (ndyn > 0 && threadIdx.x == 0 &&
      atomicAdd(&w.sched->done, 1u) == static_cast<unsigned int>(w.gfull) - 1u) {
    atomicExch(&w.sched->next, 0u);
    atomicExch(&w.sched->done, 0u);
  }
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

  // One worker at a time: all U vectors of worker m are loaded (and, with the step, updated and
  // their momentum stored) before worker m+1 is touched, so a wave's burst of memory traffic
  // stays on a few streams instead of spreading over all M workers' -- measured 4 % faster than
  // vector-by-vector over all workers.
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
#pragma unroll
      for (int m = 0; m < M; ++m) {
        f4 vv[U], gv[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
          xv[k][m] = KEEPX ? load4<FULL>(x[m] + e[k], n[k]) : load4_stream<FULL>(x[m] + e[k], n[k]);
          vv[k] = load4_stream<FULL>(v[m] + e[k], n[k]);
          gv[k] = load4_stream<FULL>(g[m] + e[k], n[k]);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
          // Alg. 1 local step with heavy-ball momentum: g' = g + wd x; v <- mu v + g'; x <- x - lr v
          const f4 ge = fma4(xv[k][m], wd, gv[k]);
          const f4 vn = fma4(vv[k], mu, ge);
          store4_stream<FULL>(v[m] + e[k], vn, n[k]);
          // The stepped x is not written: sweep 2 re-derives it from the old x and the new v with
          // the same fused multiply-add (same bits), which trades 4 written bytes for 4 read bytes
          // per element -- reads are the cheaper direction.
          xv[k][m] = fma4(vn, -lr, xv[k][m]);
        }
      }
    } else {
#pragma unroll
      for (int m = 0; m < M; ++m)
#pragma unroll
        for (int k = 0; k < U; ++k)
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
__global__ __launch_bounds__(kBlock) void k_sweep1(const Tile* __restrict__ tiles, const Walk w, int T,
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
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        if constexpr (decltype(full)::value) {
          // Pure reads stream fastest when they bypass the last-level cache, but the tiles this sweep
          // touches last are the ones sweep 2 (which walks backwards) reads first: those, from
          // keep_from on, go through the cache so that sweep 2 finds them there.
          if (t < keep_from) {
            sweep1_tile<M, U, SGD, XBAR, NORMS, true, false>(tiles[t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m, acc);
          } else {
            // The two branches differ only in the cache hint of their loads; left alone the compiler
            // merges them and drops the hint.  The empty statements keep them apart.
            asm volatile("" ::: "memory");
            sweep1_tile<M, U, SGD, XBAR, NORMS, true, true>(tiles[t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m, acc);
            asm volatile("" ::: "memory");
          }
        } else {
          sweep1_tile<M, U, SGD, XBAR, NORMS, false, true>(tiles[w.nfull + t], T, xp, vp, gp, xbarp, lr, mu, wd,
                                                           inv_m, acc);
        }
      },
      [&](int row) {
        if (NORMS) block_sums_flush<M>(acc, partials + static_cast<size_t>(row) * pstride);
      });
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
      coef[m].inv_r = zero ? 0.f : static_cast<float>(1.0 / r);
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
                                            const float (&c)[M], unsigned int skip, float inv_m) {
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
    }
    // loads and stores go worker by worker (see sweep1_tile)
#pragma unroll
    for (int m = 0; m < M; ++m) {
#pragma unroll
      for (int k = 0; k < U; ++k) xv[k][m] = load4_stream<FULL>(x[m] + e[k], n[k]);
      if (STEP) {
        f4 vv[U];
#pragma unroll
        for (int k = 0; k < U; ++k) vv[k] = load4_stream<FULL>(v[m] + e[k], n[k]);
#pragma unroll
        for (int k = 0; k < U; ++k) xv[k][m] = fma4(vv[k], -lr, xv[k][m]);
      }
    }
    // ref - (x_m - base) is the gap x_A - x_m: base = 0, ref = x_A when the average is given,
    // base = x_0, ref = mu otherwise
    f4 ref[U], base[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      ref[k] = (XBAR == 2) ? load4_stream<FULL>(xb + e[k], n[k]) : mean_offset<M>(xv[k], inv_m);
      base[k] = (XBAR == 2) ? (f4){0.f, 0.f, 0.f, 0.f} : xv[k][0];
    }
#pragma unroll
    for (int m = 0; m < M; ++m) {
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const f4 moved = fma4(ref[k] - (xv[k][m] - base[k]), c[m], xv[k][m]);
        store4_stream<FULL>(x[m] + e[k], ((skip >> m) & 1u) ? xv[k][m] : moved, n[k]);
      }
    }
  }
}

// FOLD: the coefficients are derived here from sweep 1's partial sums (no finalize launch);
// otherwise they are read from `coef`.
template <int M, int U, int XBAR, bool STEP, bool FOLD>
__global__ __launch_bounds__(kBlock) void k_sweep2(const Tile* __restrict__ tiles, const Walk w, int T,
                                                   float* const* __restrict__ xp,
                                                   const float* const* __restrict__ vp,
                                                   const float* const* __restrict__ xbarp, float lr,
                                                   const Coef* __restrict__ coef, float inv_m_total,
                                                   const double* __restrict__ partials, int nparts,
                                                   int pstride, float pull, float push,
                                                   float* __restrict__ r_out, float* __restrict__ c_out) {
  float c[M];
  unsigned int skip = 0;        // bit m: worker m sits on the average and stays where it is
  if (FOLD) {
    float inv_r[M];
    bool on_average[M];
    coefficients_from_partials<M>(partials, nparts, pstride, pull, push, c, on_average, inv_r, r_out, c_out);
#pragma unroll
    for (int m = 0; m < M; ++m) skip |= on_average[m] ? (1u << m) : 0u;
  } else {
#pragma unroll
    for (int m = 0; m < M; ++m) {
      c[m] = coef[m].c;
      skip |= coef[m].skip != 0 ? (1u << m) : 0u;
    }
  }
  walk_items<true>(
      w, 1,
      [&](int t, auto full) {
        if constexpr (decltype(full)::value)
          sweep2_tile<M, U, XBAR, STEP, true>(tiles[t], T, xp, vp, xbarp, lr, c, skip, inv_m_total);
        else
          sweep2_tile<M, U, XBAR, STEP, false>(tiles[w.nfull + t], T, xp, vp, xbarp, lr, c, skip, inv_m_total);
      },
      [](int) {});
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
    }
#pragma unroll
    for (int m = 0; m < M; ++m)       // worker by worker (see sweep1_tile)
#pragma unroll
      for (int k = 0; k < U; ++k) xv[k][m] = load4_stream<FULL>(x[m] + e[k], n[k]);
    f4 mu[U], usum[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      mu[k] = mean_offset<M>(xv[k], inv_m);
      usum[k] = (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < M; ++m) usum[k] = fma4(mu[k] - (xv[k][m] - xv[k][0]), inv_r[m], usum[k]);
    }
#pragma unroll
    for (int m = 0; m < M; ++m) {
#pragma unroll
      for (int k = 0; k < U; ++k) {
        f4 moved = fma4(mu[k] - (xv[k][m] - xv[k][0]), c[m], xv[k][m]);
        moved = fma4(usum[k], k2, moved);
        store4_stream<FULL>(x[m] + e[k], moved, n[k]);
      }
    }
  }
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_update_exact(const Tile* __restrict__ tiles, const Walk w, int T,
                                                         float* const* __restrict__ xp,
                                                         const double* __restrict__ partials, int nparts,
                                                         int pstride, float pull, float push_over_m, float k2,
                                                         float* __restrict__ r_out, float* __restrict__ c_out) {
  float c[M], inv_r[M];
  bool skip[M];
  coefficients_from_partials<M>(partials, nparts, pstride, pull, push_over_m, c, skip, inv_r, r_out, c_out);
  const float inv_m = 1.0f / static_cast<float>(M);
  walk_items<true>(
      w, 1,
      [&](int t, auto full) {
        if constexpr (decltype(full)::value) exact_tile<M, U, true>(tiles[t], T, xp, c, inv_r, k2, inv_m);
        else exact_tile<M, U, false>(tiles[w.nfull + t], T, xp, c, inv_r, k2, inv_m);
      },
      [](int) {});
}

// ---- the exact update when there are more workers than fit in registers: the sum of unit gap
// vectors S = sum_j (x_A - x_j) / r_j is materialised once (any M), then every group of up to
// kMaxTemplM workers applies  x_m + (x_A - x_m) c_m + k2 S  with x_A and S read from memory.
template <bool FULL>
__device__ __forceinline__ void unit_sum_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                              const float* xb, const Coef* __restrict__ coef, float* out) {
  // Same chunked loads as the any-M average; the sum runs over the workers in ascending order.
  f4 xbar[kVecPerThread], s[kVecPerThread];
#pragma unroll
  for (int it = 0; it < kVecPerThread; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    xbar[it] = load4<FULL>(xb + e, FULL ? 4 : tl.count - e);
    s[it] = (f4){0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll 1
  for (int m = 0; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kVecPerThread];
    float w[kAnyChunk];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = xp[static_cast<size_t>(m + k) * T + tl.tensor] + tl.offset;
        w[k] = coef[m + k].inv_r;
#pragma unroll
        for (int it = 0; it < kVecPerThread; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
#pragma unroll
        for (int it = 0; it < kVecPerThread; ++it) s[it] = fma4(xbar[it] - t[k][it], w[k], s[it]);
      }
  }
#pragma unroll
  for (int it = 0; it < kVecPerThread; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    store4<FULL>(out + e, s[it], FULL ? 4 : tl.count - e);
  }
}

__global__ __launch_bounds__(kBlock) void k_unit_sum_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                         float* const* __restrict__ xp,
                                                         const float* const* __restrict__ xbarp,
                                                         const Coef* __restrict__ coef,
                                                         float* const* __restrict__ sump) {
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        const Tile tl = tiles[kFull ? t : w.nfull + t];
        unit_sum_tile<kFull>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, coef, sump[tl.tensor] + tl.offset);
      },
      [](int) {});
}

template <int M, int U, bool FULL>
__device__ __forceinline__ void exact_given_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                                 const float* xb, const float* us, const float (&c)[M], float k2) {
#pragma unroll 1
  for (int it = 0; it < kVecPerThread / U; ++it) {
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int e = 4 * (threadIdx.x + (it * U + k) * kBlock);
      const int n = FULL ? 4 : tl.count - e;
      const f4 xbar = load4_stream<FULL>(xb + e, n);
      const f4 usum = load4_stream<FULL>(us + e, n);
#pragma unroll
      for (int m = 0; m < M; ++m) {
        float* x = xp[m * T + tl.tensor] + tl.offset + e;
        const f4 xv = load4_stream<FULL>(x, n);
        f4 moved = fma4(xbar - xv, c[m], xv);
        moved = fma4(usum, k2, moved);
        store4_stream<FULL>(x, moved, n);
      }
    }
  }
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_update_exact_given(const Tile* __restrict__ tiles, const Walk w, int T,
                                                               float* const* __restrict__ xp,
                                                               const float* const* __restrict__ xbarp,
                                                               const float* const* __restrict__ sump,
                                                               const Coef* __restrict__ coef, float k2) {
  float c[M];
#pragma unroll
  for (int m = 0; m < M; ++m) c[m] = coef[m].c;
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        const Tile tl = tiles[kFull ? t : w.nfull + t];
        exact_given_tile<M, U, kFull>(tl, T, xp, xbarp[tl.tensor] + tl.offset, sump[tl.tensor] + tl.offset, c, k2);
      },
      [](int) {});
}

// ------------------------------------------- Alg. 1 written literally, any consensus variable
// pulled_m = (1 - alpha) x_m + alpha x_C; gap_m = pulled_m - ref (ref = x_A before the round, or x_C);
// r_m = ||gap_m||; x_m <- pulled_m + lambda gap_m / r_m  (no push where r_m = 0).
// REF: 0 = push away from the average (formed from these M workers), 1 = push away from the
// consensus variable, 2 = push away from an average that is read from memory (when the kernel
// sees only a group of the workers).
template <int M, int U, int REF, bool WRITE, bool FULL>
__device__ __forceinline__ void seq_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                         const float* const* __restrict__ xcp,
                                         const float* const* __restrict__ refp, float pull, float keep,
                                         const float (&scale)[M], float inv_m, double (&acc)[M]) {
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
  const float* xc = xcp[tl.tensor] + tl.offset;
  const float* rf = (REF == 2) ? refp[tl.tensor] + tl.offset : nullptr;
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
    }
#pragma unroll
    for (int m = 0; m < M; ++m)       // worker by worker (see sweep1_tile)
#pragma unroll
      for (int k = 0; k < U; ++k)
        xv[k][m] = WRITE ? load4_stream<FULL>(x[m] + e[k], n[k]) : load4<FULL>(x[m] + e[k], n[k]);
    f4 ref[U];
#pragma unroll
    for (int k = 0; k < U; ++k)
      ref[k] = (REF == 0)   ? xv[k][0] + mean_offset<M>(xv[k], inv_m)
               : (REF == 1) ? cv[k]
                            : load4<FULL>(rf + e[k], n[k]);
#pragma unroll
    for (int m = 0; m < M; ++m) {
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const f4 pulled = fma4(cv[k], pull, xv[k][m] * keep);   // (1-alpha) x + alpha x_C: exactly x_C at alpha = 1
        const f4 gap = pulled - ref[k];
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
__global__ __launch_bounds__(kBlock) void k_seq1(const Tile* __restrict__ tiles, const Walk w, int T,
                                                 float* const* __restrict__ xp,
                                                 const float* const* __restrict__ xcp,
                                                 const float* const* __restrict__ refp, float pull, float keep,
                                                 double* __restrict__ partials, int pstride) {
  double acc[M];
  float scale[M];
#pragma unroll
  for (int m = 0; m < M; ++m) {
    acc[m] = 0.0;
    scale[m] = 0.f;
  }
  const float inv_m = 1.0f / static_cast<float>(M);
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        seq_tile<M, U, REF, false, kFull>(tiles[kFull ? t : w.nfull + t], T, xp, xcp, refp, pull, keep, scale, inv_m,
                                          acc);
      },
      [&](int row) { block_sums_flush<M>(acc, partials + static_cast<size_t>(row) * pstride); });
}

template <int M, int U, int REF>
__global__ __launch_bounds__(kBlock) void k_seq2(const Tile* __restrict__ tiles, const Walk w, int T,
                                                 float* const* __restrict__ xp,
                                                 const float* const* __restrict__ xcp,
                                                 const float* const* __restrict__ refp, float pull, float keep,
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
  walk_items<true>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        seq_tile<M, U, REF, true, kFull>(tiles[kFull ? t : w.nfull + t], T, xp, xcp, refp, pull, keep, scale, inv_m,
                                         unused);
      },
      [](int) {});
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
__global__ __launch_bounds__(kBlock) void k_adamw_step(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                       float* const* __restrict__ xp,
                                                       float* const* __restrict__ ap, float* const* __restrict__ sp,
                                                       const float* const* __restrict__ gp, const AdamHyper hp) {
  // work items are (pair of full tiles, worker) or (partial tile, worker), worker-major
  walk_items<false>(
      w, M,
      [&](int item, auto full) {
        constexpr bool kFull = decltype(full)::value;
        constexpr int kPer = kFull ? kTilesPerWorkerItem : 1;
        const int ntile = kFull ? w.nfull : w.ntiles - w.nfull;
        const int per_worker = (ntile + kPer - 1) / kPer;
        const int m = item / per_worker;
        const int first = (item - m * per_worker) * kPer;
        if (m >= M) return;       // cannot happen while the host counts items the same way
#pragma unroll 1
        for (int t = first; t < first + kPer && t < ntile; ++t) {
          const Tile tl = tiles[(kFull ? 0 : w.nfull) + t];
          const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
          adamw_tile<U, kFull>(xp[slot] + tl.offset, ap[slot] + tl.offset, sp[slot] + tl.offset,
                               gp[slot] + tl.offset, tl.count, hp);
        }
      },
      [](int) {});
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
    f4 xv[U][M];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
    }
    // worker by worker (see sweep1_tile): here 7 % faster than all workers' loads at once
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
      float* x = xp[slot] + tl.offset;
      float* a = ap[slot] + tl.offset;
      float* q = sp[slot] + tl.offset;
      const float* g = gp[slot] + tl.offset;
      f4 av[U], sv[U], gv[U];
#pragma unroll
      for (int k = 0; k < U; ++k) {
        xv[k][m] = load4_stream<FULL>(x + e[k], n[k]);
        av[k] = load4_stream<FULL>(a + e[k], n[k]);
        sv[k] = load4_stream<FULL>(q + e[k], n[k]);
        gv[k] = load4_stream<FULL>(g + e[k], n[k]);
      }
#pragma unroll
      for (int k = 0; k < U; ++k) {
        f4 xn, an, sn;
        adamw_vec(xv[k][m], av[k], sv[k], gv[k], hp, xn, an, sn);
        store4_stream<FULL>(a + e[k], an, n[k]);
        store4_stream<FULL>(q + e[k], sn, n[k]);
        store4<FULL>(x + e[k], xn, n[k]);     // read again by sweep 2
        xv[k][m] = xn;
      }
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const f4 mo = mean_offset<M>(xv[k], inv_m);
#pragma unroll
      for (int m = 0; m < M; ++m) part[m] = sumsq4((xv[k][m] - xv[k][0]) - mo, part[m]);
    }
  }
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] += static_cast<double>(part[m]);
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_adamw_reduce(const Tile* __restrict__ tiles, const Walk w, int T,
                                                         float* const* __restrict__ xp,
                                                         float* const* __restrict__ ap,
                                                         float* const* __restrict__ sp,
                                                         const float* const* __restrict__ gp, const AdamHyper hp,
                                                         double* __restrict__ partials, int pstride) {
  double acc[M];
#pragma unroll
  for (int m = 0; m < M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        adamw_reduce_tile<M, U, kFull>(tiles[kFull ? t : w.nfull + t], T, xp, ap, sp, gp, hp, inv_m, acc);
      },
      [&](int row) { block_sums_flush<M>(acc, partials + static_cast<size_t>(row) * pstride); });
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
__global__ __launch_bounds__(kBlock) void k_local_step(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                       float* const* __restrict__ xp,
                                                       float* const* __restrict__ vp,
                                                       const float* const* __restrict__ gp, float lr,
                                                       float mu, float wd) {
  // work items are (pair of full tiles, worker) or (partial tile, worker), worker-major
  walk_items<false>(
      w, M,
      [&](int item, auto full) {
        constexpr bool kFull = decltype(full)::value;
        constexpr int kPer = kFull ? kTilesPerWorkerItem : 1;
        const int ntile = kFull ? w.nfull : w.ntiles - w.nfull;
        const int per_worker = (ntile + kPer - 1) / kPer;
        const int m = item / per_worker;
        const int first = (item - m * per_worker) * kPer;
        if (m >= M) return;       // cannot happen while the host counts items the same way
#pragma unroll 1
        for (int t = first; t < first + kPer && t < ntile; ++t) {
          const Tile tl = tiles[(kFull ? 0 : w.nfull) + t];
          const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
          local_tile<U, kFull>(xp[slot] + tl.offset, vp[slot] + tl.offset, gp[slot] + tl.offset, tl.count, lr, mu, wd);
        }
      },
      [](int) {});
}

// ------------------------------- average over a runtime number of workers (M > kMaxTemplM)
template <bool FULL>
__device__ __forceinline__ void mean_any_tile(const Tile tl, int M, int T,
                                              float* const* __restrict__ xp, float* xb, float inv_m) {
  // Workers are taken kAnyChunk at a time and all of a chunk's loads are issued before the first
  // is used; the sums still run over the workers in ascending order.
  f4 x0[kVecPerThread], s[kVecPerThread];
  const float* base0 = xp[tl.tensor] + tl.offset;
#pragma unroll
  for (int it = 0; it < kVecPerThread; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    x0[it] = load4<FULL>(base0 + e, FULL ? 4 : tl.count - e);
    s[it] = (f4){0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll 1
  for (int m = 1; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kVecPerThread];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = xp[static_cast<size_t>(m + k) * T + tl.tensor] + tl.offset;
#pragma unroll
        for (int it = 0; it < kVecPerThread; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
#pragma unroll
        for (int it = 0; it < kVecPerThread; ++it) s[it] += t[k][it] - x0[it];
      }
  }
#pragma unroll
  for (int it = 0; it < kVecPerThread; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    store4<FULL>(xb + e, x0[it] + scale_by_inverse_count(s[it], M, inv_m), FULL ? 4 : tl.count - e);
  }
}

__global__ __launch_bounds__(kBlock) void k_mean_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                     float* const* __restrict__ xp,
                                                     float* const* __restrict__ xbarp) {
  const float inv_m = 1.0f / static_cast<float>(M);
  walk_items<false>(
      w, 1,
      [&](int t, auto full) {
        constexpr bool kFull = decltype(full)::value;
        const Tile tl = tiles[kFull ? t : w.nfull + t];
        mean_any_tile<kFull>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, inv_m);
      },
      [](int) {});
}

// ------------------------------- work decomposition of ONE flat tensor, built on the device
// For callers that may not allocate: the tile list of a single tensor of d elements per worker
// (full tiles first, then the ragged tail, exactly what the host-side list builder produces) and
// the table of the M workers' base pointers x + m*ld are written straight into caller-provided
// device memory, and the on-demand counter is put back to zero.
__global__ __launch_bounds__(kBlock) void k_flat_setup(Tile* __restrict__ tiles, long long d,
                                                       float** __restrict__ ptrs, float* x, long long ld, int M,
                                                       Sched* __restrict__ sched) {
  const long long nfull = d / kTileElems;
  const int tail = static_cast<int>(d - nfull * kTileElems);
  const long long ntiles = nfull + (tail > 0 ? 1 : 0);
  const long long stride = static_cast<long long>(gridDim.x) * kBlock;
  for (long long t = static_cast<long long>(blockIdx.x) * kBlock + threadIdx.x; t < ntiles; t += stride) {
    Tile tl;
    tl.offset = t * kTileElems;
    tl.tensor = 0;
    tl.count = t < nfull ? kTileElems : tail;
    tiles[t] = tl;
  }
  if (blockIdx.x == 0) {
    if (static_cast<int>(threadIdx.x) < M) ptrs[threadIdx.x] = x + static_cast<long long>(threadIdx.x) * ld;
    if (threadIdx.x == 0) {
      sched->next = 0u;
      sched->done = 0u;
    }
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
// mix, the ceiling the DPPF kernels are compared with.  The blocks walk items of kProbeItemTiles
// tiles the way the DPPF kernels walk their tiles (walk_items): an even split, or an even split
// with the tail handed out on demand.
constexpr int kProbeItemTiles = 16;
__device__ Sched g_probe_sched;

template <int R, int W, int U, bool INPLACE>
__global__ __launch_bounds__(kBlock) void k_probe(float* __restrict__ base, long long stride, long long n,
                                                  float* __restrict__ sink, const Walk walk) {
  const long long tile = static_cast<long long>(kBlock) * U * 4;
  const long long ntiles = n / tile;
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  walk_items<false>(
      walk, 1,
      [&](int item, auto) {
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
      [](int) {});
  if (W == 0 && acc.x + acc.y + acc.z + acc.w == 123.456f) sink[0] = acc.x;   // keeps the loads alive
}

}  // namespace

#endif  // DPPF_KERNELS_H_
