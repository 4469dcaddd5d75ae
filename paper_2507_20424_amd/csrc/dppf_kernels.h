// Device code of the DPPF library: load/store helpers and every kernel template.  Included by the
// translation units that launch them (each instantiates only the kernels it launches).
//
// Three families of kernels cover the worker counts:
//   * M <= 16: all M replicas of a lane's elements sit in registers (M is a template parameter);
//   * 17 <= M <= 39: one 16-byte vector per lane and worker is staged in LDS (M is a run-time value;
//     39 workers x 256 lanes x 16 bytes fill the CU's 160 KB), so the traffic stays at the algorithmic
//     bytes;
//   * any M: streaming kernels that read a STORED average instead of forming it (used beyond 39
//     workers and by the variants that have no LDS form).
#ifndef DPPF_KERNELS_H_
#define DPPF_KERNELS_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "dppf_walk.h"

// Types and constants that the host side shares with the kernels.
namespace dppf_detail {

using dppf_walk::Sched;
using dppf_walk::Tile;
using dppf_walk::Walk;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4u __attribute__((aligned(4)));   // 16-byte vector that may sit on any 4-byte boundary

constexpr int kBlock = 256;                   // threads per block (4 waves)
constexpr int kWaves = kBlock / 64;
constexpr int kMaxTemplM = 16;                // worker counts with a register-resident kernel
constexpr int kMaxLdsM = 39;                  // worker counts with an LDS-staged kernel
constexpr int kAnyChunk = 4;                  // workers whose loads the any-M kernels keep in flight together
constexpr int kMaxBlocksPerCU = 8;            // upper bound on resident blocks per CU (sizes buffers)

// Elements of ONE worker's tensor per tile.  What a block holds of a tile grows with M, and from 5
// workers on half-size tiles are faster (fused round, M = 5: +1 %, 7: +4 %, 8: +6 %, 12: +6 %,
// 16: +7 %; sweep 2 gains most); up to 4 workers they are slower (M = 4: -7 %, M = 2: -16 %).
// The LDS-staged kernels hold one vector per lane.  The kernels that take one worker at a time and
// the any-M streaming kernels use kStepTileElems.
constexpr int kStepTileElems = 4096;
constexpr int kLdsTileElems = 4 * kBlock;
constexpr int kSmallTileFromM = 5;
constexpr int sweep_tile_elems(int M) {
  return M < kSmallTileFromM ? 4096 : (M <= kMaxTemplM ? 2048 : (M <= kMaxLdsM ? kLdsTileElems : kStepTileElems));
}
constexpr int vectors_per_lane(int tile_elems) { return tile_elems / (4 * kBlock); }
// Workers whose loads the fused sweeps 1 keep in flight ahead of the worker they work on (`arrays`
// = streams per worker: x, v, g or x, m1, m2, g).  With two vectors per lane and worker (5 workers
// and more) a single worker's requests are too few to cover the latency, and as many workers as 48
// vectors per lane allow are requested ahead (M = 8: sweep 1 of the fused round -4 %); with four
// vectors per worker the look-ahead gains nothing (M = 4: +1 %) and is left out.
constexpr int lookahead(int M, int U, int arrays) {
  return U >= 4 ? 0 : (48 / (arrays * U) - 1 > M ? M : 48 / (arrays * U) - 1);
}

// Resident blocks per CU by traffic pattern (measured): kernels that mix reads and writes run
// fastest with ONE block per CU -- fewer concurrently open DRAM rows and longer same-direction
// bursts outweigh the lost latency hiding; kernels that only read do best with two.
constexpr int kBlocksPerCUReadOnly = 2;
constexpr int kBlocksPerCUReadWrite = 1;

struct Coef {
  float c;            // alpha - lambda / r_m
  int skip;           // r_m == 0: leave the worker untouched
  float inv_r;        // 1 / r_m, 0 where r_m == 0
};

// Adam's hyper-parameters as the kernels take them: bc_i = 1 - beta_i^t is formed on the host.
struct AdamHyper {
  float lr, b1, b2, eps, wd, inv_bc1, inv_bc2;
};

// The kernels that handle one worker at a time (local steps) take two full tiles per item: one
// tile of one worker is only about 3 microseconds of traffic, too little to hide the request for
// the next item behind (measured: two tiles 3-6 % faster than one, three or four slower again;
// the sweeps that take all workers of a tile together are fastest with one tile per item).
constexpr int kTilesPerWorkerItem = 2;

// What the LDS-staged first sweep folds in.  OPT: 0 = x as it is, 1 = momentum-SGD step (v stored,
// stepped x kept only on chip), 2 = AdamW step (m1, m2 and the stepped x stored).
constexpr int kLdsChunk = 4;                  // workers per register chunk of the LDS-staged kernels (8 is no
                                              // faster and wastes more load slots when M is not a multiple)
struct LdsOptArgs {
  float* const* vp;          // SGD: momentum; AdamW: first moment
  float* const* sp;          // AdamW: second moment
  const float* const* gp;
  float lr, mu, wd;          // SGD
  AdamHyper adam;
};

}  // namespace dppf_detail

namespace {

using namespace dppf_detail;

// ------------------------------------------------------------------------------- helpers
// Tensor data always live in device (global) memory.  The pointers come out of pointer tables, so
// the compiler cannot know that and would use flat addressing; these types tell it.
typedef __attribute__((address_space(1))) const f4u* gvec_in;
typedef __attribute__((address_space(1))) f4u* gvec_out;
typedef __attribute__((address_space(1))) const float* gf_in;
typedef __attribute__((address_space(1))) float* gf_out;

// Entry `slot` of a pointer table (slot the same for every lane), fetched through the scalar path.
// The tables are written before the launch and never during it, but a kernel that also stores
// through the pointers it fetched gives the compiler no way to know that; left to itself it fetches
// entries inside a loop over the workers with vector loads, and those share the in-order counter
// of the data loads: waiting for the next workers' pointers then means waiting for every data load
// issued before them, and the overlap between one group of workers and the next is gone.
template <typename P>
__device__ __forceinline__ P* table_entry(P* const* table, size_t slot) {
  typedef P* entry;
  typedef __attribute__((address_space(4))) const entry* constant_table;   // the ENTRIES sit in constant memory
  return ((constant_table)(table))[slot];
}

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

// The first n components of v, zeros after them (n >= 4: v itself).  Lanes that reach past the end
// of a partial tile compute on zeros; where a formula does not map zeros to zero (AdamW with
// eps = 0 divides 0 by 0) its result is cut back before it enters a sum.
template <bool FULL>
__device__ __forceinline__ f4 first_components(f4 v, int n) {
  if (FULL || n >= 4) return v;
  f4 r = {0.f, 0.f, 0.f, 0.f};
  if (n > 0) r.x = v.x;
  if (n > 1) r.y = v.y;
  if (n > 2) r.z = v.z;
  return r;
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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Block-wide sums of C per-lane doubles; thread c < C writes the c-th sum to out[c * stride] (the
// partial sums are stored column by column: column c of row r sits at [c * rows + r], so that the
// readers, which add up one column over all rows, read consecutive addresses).  The per-lane
// values are set back to zero.  May be called repeatedly by a block, with at least one barrier
// between two calls (the on-demand part of a walk has one per item).
template <int C>
__device__ __forceinline__ void block_sums_flush(double (&acc)[C], double* out, int stride) {
  __shared__ double lds[kWaves][C];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int c = 0; c < C; ++c) {
    double s = wave_sum(acc[c]);
    if (lane == 0) lds[wave][c] = s;
    acc[c] = 0.0;
  }
  __syncthreads();
  if (threadIdx.x < C) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds[w][threadIdx.x];
    out[static_cast<size_t>(threadIdx.x) * stride] = s;
  }
}

// The same for a run-time number of columns: per-wave running sums in LDS (`acc`, kWaves x cols
// doubles, the caller's memory).  add() folds one value per lane into column `col` -- all lanes of
// a wave must call it together; flush() writes the block's sums and clears them.
struct ColumnSums {
  double* acc;
  int cols;
  __device__ __forceinline__ void init(double* lds, int ncols) {
    acc = lds;
    cols = ncols;
    for (int i = threadIdx.x; i < kWaves * cols; i += kBlock) acc[i] = 0.0;
    __syncthreads();
  }
  __device__ __forceinline__ void add(float v, int col) {
    const float s = wave_sum(v);
    if ((threadIdx.x & 63) == 0) acc[(threadIdx.x >> 6) * cols + col] += static_cast<double>(s);
  }
  // G values per lane for the columns col0 .. col0+G-1 (those below `limit` are kept): the wave
  // sums of all G columns in log2(G) + ... exchanges instead of G full butterflies.  Each exchange
  // halves the number of columns a lane is responsible for -- the lanes with the exchanged lane bit
  // set keep the upper half -- until every lane holds one column; three more exchanges finish the
  // sum over the lanes that share it.  G = 4 or 8.
  template <int G>
  __device__ __forceinline__ void add_group(float (&p)[G], int col0, int limit) {
    static_assert(kAnyChunk == 4 && (G == 4 || G == 8), "group of 4 or 8 columns");
    const int lane = threadIdx.x & 63;
    float q[4], r[2], t;
    if (G == 8) {
      const bool up = (lane & 32) != 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float mine = up ? p[k + 4] : p[k];
        const float theirs = up ? p[k] : p[k + 4];
        q[k] = mine + __shfl_xor(theirs, 32, 64);
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) q[k] = p[k] + __shfl_xor(p[k], 32, 64);
    }
    {
      const bool up = (lane & 16) != 0;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const float mine = up ? q[k + 2] : q[k];
        const float theirs = up ? q[k] : q[k + 2];
        r[k] = mine + __shfl_xor(theirs, 16, 64);
      }
    }
    {
      const bool up = (lane & 8) != 0;
      const float mine = up ? r[1] : r[0];
      const float theirs = up ? r[0] : r[1];
      t = mine + __shfl_xor(theirs, 8, 64);
    }
    t += __shfl_xor(t, 4, 64);
    t += __shfl_xor(t, 2, 64);
    t += __shfl_xor(t, 1, 64);
    // the column this lane ended up with: lane bit 5 chose between halves of 8, bit 4 of 4, bit 3 of 2
    const int col = col0 + (G == 8 ? ((lane >> 5) & 1) * 4 : 0) + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
    const bool writer = (lane & 7) == 0 && (G == 8 || (lane & 32) == 0);
    if (writer && col < limit) acc[(threadIdx.x >> 6) * cols + col] += static_cast<double>(t);
  }
  __device__ __forceinline__ void flush(double* out, int stride) {
    __syncthreads();
    for (int c = threadIdx.x; c < cols; c += kBlock) {
      double s = 0.0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        s += acc[w * cols + c];
        acc[w * cols + c] = 0.0;
      }
      out[static_cast<size_t>(c) * stride] = s;
    }
    __syncthreads();
  }
};

// A thread block's view of the machine for dppf_walk::walk_items.
struct BlockEnv {
  int slot = 0;   // the item number travels from thread 0 to the block through two alternating words:
                  // one barrier per item is enough, the next write goes to the other word
  __device__ __forceinline__ int block() const { return static_cast<int>(blockIdx.x); }
  __device__ __forceinline__ int grid() const { return static_cast<int>(gridDim.x); }
  __device__ __forceinline__ unsigned int request(Sched* s) {
    return threadIdx.x == 0 ? atomicAdd(&s->next, 1u) : 0u;
  }
  __device__ __forceinline__ int share(unsigned int v) {
    __shared__ int s_next[2];
    if (threadIdx.x == 0) s_next[slot] = static_cast<int>(v);
    __syncthreads();
    const int k = s_next[slot];
    slot ^= 1;
    return k;
  }
  __device__ __forceinline__ void leave(Sched* s, int gfull) {
    if (threadIdx.x == 0 && atomicAdd(&s->done, 1u) == static_cast<unsigned int>(gfull) - 1u) {
      atomicExch(&s->next, 0u);
      atomicExch(&s->done, 0u);
    }
  }
};

template <bool REVERSE, typename FullBody, typename PartBody, typename Flush>
__device__ __forceinline__ void walk(const Walk& w, int per_tile, FullBody&& full_body, PartBody&& part_body,
                                     Flush&& flush) {
  BlockEnv env;
  dppf_walk::walk_items<REVERSE>(env, w, per_tile, full_body, part_body, flush);
}

// ===================================================================== M <= 16: in registers
// --------------------------------------------------------------------- sweep 1 of the round
// XBAR: 0 = average stays in registers, 1 = also written out.
// KEEPX: load x through the caches (it is read again soon) instead of streaming it past them.
// acc[0..M-1]: squared distances; acc[M]: squared norm of the average (the appendix section on
// hyper-parameter sensitivity tracks ||x_A||; it rides along for four multiply-adds per vector).
template <int M, int U, bool SGD, int XBAR, bool NORMS, bool FULL, bool KEEPX>
__device__ __forceinline__ void sweep1_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                            float* const* __restrict__ vp,
                                            const float* const* __restrict__ gp,
                                            float* const* __restrict__ xbarp, float lr, float mu,
                                            float wd, float inv_m, double (&acc)[M + 1]) {
  constexpr int kVec = vectors_per_lane(sweep_tile_elems(M));
  static_assert(kVec % U == 0, "a lane's vectors of a tile are taken U at a time");
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

  float part[M + 1];
#pragma unroll
  for (int m = 0; m <= M; ++m) part[m] = 0.f;

  // One worker at a time: all U vectors of worker m are loaded (and, with the step, updated and
  // their momentum stored) before worker m+1 is touched, so a wave's burst of memory traffic
  // stays on a few streams instead of spreading over all M workers' -- measured 4 % faster than
  // vector-by-vector over all workers.
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
    int e[U], n[U];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
    }
    f4 xv[U][M];
    if (SGD) {
      // The loads of the next kAhead workers are issued before worker m's data are waited for, so a
      // wave has several workers' worth of requests in flight; written as one worker after the
      // other, each wave drains its loads before it issues the stores and the next worker's loads
      // (the compiler cannot move loads above stores of possibly overlapping memory).
      constexpr int kAhead = lookahead(M, U, 3);
      f4 vv[M][U], gv[M][U];
      auto request = [&](int m) {
#pragma unroll
        for (int k = 0; k < U; ++k) {
          xv[k][m] = KEEPX ? load4<FULL>(x[m] + e[k], n[k]) : load4_stream<FULL>(x[m] + e[k], n[k]);
          vv[m][k] = load4_stream<FULL>(v[m] + e[k], n[k]);
          gv[m][k] = load4_stream<FULL>(g[m] + e[k], n[k]);
        }
      };
#pragma unroll
      for (int m = 0; m < kAhead && m < M; ++m) request(m);
#pragma unroll
      for (int m = 0; m < M; ++m) {
        if (m + kAhead < M) request(m + kAhead);
#pragma unroll
        for (int k = 0; k < U; ++k) {
          // Alg. 1 local step with heavy-ball momentum: g' = g + wd x; v <- mu v + g'; x <- x - lr v
          const f4 ge = fma4(xv[k][m], wd, gv[m][k]);
          const f4 vn = fma4(vv[m][k], mu, ge);
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
      const f4 mo = mean_offset<M>(xv[k], inv_m);
      const f4 xa = xv[k][0] + mo;
      if (XBAR == 1) store4_stream<FULL>(xb + e[k], xa, n[k]);
      if (NORMS) {
#pragma unroll
        for (int m = 0; m < M; ++m) part[m] = sumsq4((xv[k][m] - xv[k][0]) - mo, part[m]);
        part[M] = sumsq4(xa, part[M]);
      }
    }
  }
  if (NORMS) {
#pragma unroll
    for (int m = 0; m <= M; ++m) acc[m] += static_cast<double>(part[m]);
  }
}

template <int M, int U, bool SGD, int XBAR, bool NORMS>
__global__ __launch_bounds__(kBlock) void k_sweep1(const Tile* __restrict__ tiles, const Walk w, int T,
                                                   float* const* __restrict__ xp,
                                                   float* const* __restrict__ vp,
                                                   const float* const* __restrict__ gp,
                                                   float* const* __restrict__ xbarp, float lr,
                                                   float mu, float wd, double* __restrict__ partials,
                                                   int prows, int keep_from) {
  double acc[M + 1];
#pragma unroll
  for (int m = 0; m <= M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<false>(
      w, 1,
      [&](int t) {
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
      },
      [&](int t) {
        sweep1_tile<M, U, SGD, XBAR, NORMS, false, true>(tiles[w.nfull + t], T, xp, vp, gp, xbarp, lr, mu, wd, inv_m,
                                                         acc);
      },
      [&](int row) {
        if (NORMS) block_sums_flush<M + 1>(acc, partials + row, prows);
      });
}

// ------------------------------------------------------- partial sums -> r_m and c_m (Eq. 5)
// One block per column of the partial sums; fixed summation order, fp64.  Columns 0..M-1 are the
// workers' squared distances, column M is the squared norm of the average.
constexpr int kFinalizeThreads = 1024;
__global__ __launch_bounds__(kFinalizeThreads) void k_finalize(const double* __restrict__ partials, int nparts,
                                                               int prows, int M, float pull, float push,
                                                               Coef* __restrict__ coef, float* __restrict__ r_out,
                                                               float* __restrict__ c_out,
                                                               float* __restrict__ avg_norm_out) {
  __shared__ double lds[kFinalizeThreads];
  const int m = blockIdx.x;
  const double* column = partials + static_cast<size_t>(m) * prows;
  double s = 0.0;
  // a column is contiguous; eight loads are in flight per thread, the additions keep their order
#pragma unroll 8
  for (int b = threadIdx.x; b < nparts; b += kFinalizeThreads) s += column[b];
  lds[threadIdx.x] = s;
  __syncthreads();
  for (int off = kFinalizeThreads / 2; off > 0; off >>= 1) {
    if (threadIdx.x < off) lds[threadIdx.x] += lds[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double r = sqrt(lds[0]);
    if (m == M) {
      if (avg_norm_out) avg_norm_out[0] = static_cast<float>(r);
      return;
    }
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
                                                           int prows, float pull, float push,
                                                           float (&c)[M], bool (&skip)[M],
                                                           float (&inv_r)[M],
                                                           float* __restrict__ r_out,
                                                           float* __restrict__ c_out,
                                                           float* __restrict__ avg_norm_out) {
  __shared__ double lds[kWaves][M + 1];
  __shared__ float c_sh[M];
  __shared__ float inv_sh[M];
  __shared__ int skip_sh[M];
  const bool want_avg = blockIdx.x == 0 && avg_norm_out != nullptr;   // only one block needs column M
  double acc[M + 1];
#pragma unroll
  for (int m = 0; m <= M; ++m) acc[m] = 0.0;
  // columns are contiguous; four rows' loads are in flight per thread, the additions keep their order
#pragma unroll 4
  for (int b = threadIdx.x; b < nparts; b += kBlock) {
#pragma unroll
    for (int m = 0; m < M; ++m) acc[m] += partials[static_cast<size_t>(m) * prows + b];
    if (want_avg) acc[M] += partials[static_cast<size_t>(M) * prows + b];
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int m = 0; m <= M; ++m) {
    const double s = wave_sum(acc[m]);
    if (lane == 0) lds[wave][m] = s;
  }
  __syncthreads();
  if (threadIdx.x <= M) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += lds[w][threadIdx.x];
    const double r = sqrt(s);
    if (threadIdx.x == M) {
      if (want_avg) avg_norm_out[0] = static_cast<float>(r);
    } else {
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
// Eq. 5: x_m <- x_m + (x_A - x_m) c_m, with x_A recomputed from the same M loads.
// STEP: x in memory is still the value from before the fused local step and v is already the
// new momentum; the stepped x is rebuilt as x - lr v before the update.
template <int M, int U, bool STEP, bool FULL>
__device__ __forceinline__ void sweep2_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                            const float* const* __restrict__ vp, float lr,
                                            const float (&c)[M], unsigned int skip, float inv_m) {
  constexpr int kVec = vectors_per_lane(sweep_tile_elems(M));
  static_assert(kVec % U == 0, "a lane's vectors of a tile are taken U at a time");
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
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
        // v is read once: its pointer is fetched where it is used (kept in an array beside x's, the
        // 2M pointers ran one instantiation out of scalar registers)
        const float* vm = vp[m * T + tl.tensor] + tl.offset;
        f4 vv[U];
#pragma unroll
        for (int k = 0; k < U; ++k) vv[k] = load4_stream<FULL>(vm + e[k], n[k]);
#pragma unroll
        for (int k = 0; k < U; ++k) xv[k][m] = fma4(vv[k], -lr, xv[k][m]);
      }
    }
    // mu - (x_m - x_0) is the gap x_A - x_m
    f4 mo[U];
#pragma unroll
    for (int k = 0; k < U; ++k) mo[k] = mean_offset<M>(xv[k], inv_m);
#pragma unroll
    for (int m = 0; m < M; ++m) {
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const f4 moved = fma4(mo[k] - (xv[k][m] - xv[k][0]), c[m], xv[k][m]);
        store4_stream<FULL>(x[m] + e[k], ((skip >> m) & 1u) ? xv[k][m] : moved, n[k]);
      }
    }
  }
}

// FOLD: the coefficients are derived here from sweep 1's partial sums (no finalize launch);
// otherwise they are read from `coef`.
template <int M, int U, bool STEP, bool FOLD>
__global__ __launch_bounds__(kBlock) void k_sweep2(const Tile* __restrict__ tiles, const Walk w, int T,
                                                   float* const* __restrict__ xp,
                                                   const float* const* __restrict__ vp, float lr,
                                                   const Coef* __restrict__ coef,
                                                   const double* __restrict__ partials, int nparts,
                                                   int prows, float pull, float push,
                                                   float* __restrict__ r_out, float* __restrict__ c_out,
                                                   float* __restrict__ avg_norm_out) {
  float c[M];
  unsigned int skip = 0;        // bit m: worker m sits on the average and stays where it is
  if (FOLD) {
    float inv_r[M];
    bool on_average[M];
    coefficients_from_partials<M>(partials, nparts, prows, pull, push, c, on_average, inv_r, r_out, c_out,
                                  avg_norm_out);
#pragma unroll
    for (int m = 0; m < M; ++m) skip |= on_average[m] ? (1u << m) : 0u;
  } else {
    // through LDS, like the folded form: read straight into scalar registers the M coefficients
    // compete with the tile's 2M pointers and one instantiation (M = 12) spilled
    __shared__ float c_sh[M];
    __shared__ int skip_sh[M];
    if (threadIdx.x < M) {
      c_sh[threadIdx.x] = coef[threadIdx.x].c;
      skip_sh[threadIdx.x] = coef[threadIdx.x].skip;
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < M; ++m) {
      c[m] = c_sh[m];
      skip |= skip_sh[m] != 0 ? (1u << m) : 0u;
    }
  }
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<true>(
      w, 1, [&](int t) { sweep2_tile<M, U, STEP, true>(tiles[t], T, xp, vp, lr, c, skip, inv_m); },
      [&](int t) { sweep2_tile<M, U, STEP, false>(tiles[w.nfull + t], T, xp, vp, lr, c, skip, inv_m); },
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
  constexpr int kVec = vectors_per_lane(sweep_tile_elems(M));
  static_assert(kVec % U == 0, "a lane's vectors of a tile are taken U at a time");
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
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
                                                         int prows, float pull, float push_over_m, float k2,
                                                         float* __restrict__ r_out, float* __restrict__ c_out,
                                                         float* __restrict__ avg_norm_out) {
  float c[M], inv_r[M];
  bool skip[M];
  coefficients_from_partials<M>(partials, nparts, prows, pull, push_over_m, c, skip, inv_r, r_out, c_out,
                                avg_norm_out);
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<true>(
      w, 1, [&](int t) { exact_tile<M, U, true>(tiles[t], T, xp, c, inv_r, k2, inv_m); },
      [&](int t) { exact_tile<M, U, false>(tiles[w.nfull + t], T, xp, c, inv_r, k2, inv_m); }, [](int) {});
}

// ------------------------------------------- Alg. 1 written literally, any consensus variable
// pulled_m = (1 - alpha) x_m + alpha x_C; gap_m = pulled_m - ref (ref = x_A before the round, or x_C);
// r_m = ||gap_m||; x_m <- pulled_m + lambda gap_m / r_m  (no push where r_m = 0).
// REF: 0 = push away from the average (formed from these M workers), 1 = push away from the
// consensus variable.
template <int M, int U, int REF, bool WRITE, bool FULL>
__device__ __forceinline__ void seq_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                         const float* const* __restrict__ xcp, float pull, float keep,
                                         const float (&scale)[M], float inv_m, double (&acc)[M + 1]) {
  constexpr int kVec = vectors_per_lane(sweep_tile_elems(M));
  static_assert(kVec % U == 0, "a lane's vectors of a tile are taken U at a time");
  float* x[M];
#pragma unroll
  for (int m = 0; m < M; ++m) x[m] = xp[m * T + tl.tensor] + tl.offset;
  const float* xc = xcp[tl.tensor] + tl.offset;
  float part[M];
#pragma unroll
  for (int m = 0; m < M; ++m) part[m] = 0.f;
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
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
    for (int k = 0; k < U; ++k) ref[k] = (REF == 0) ? xv[k][0] + mean_offset<M>(xv[k], inv_m) : cv[k];
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
                                                 const float* const* __restrict__ xcp, float pull, float keep,
                                                 double* __restrict__ partials, int prows) {
  double acc[M + 1];          // column M (the norm of the average) is not formed here: stays zero
  float scale[M];
#pragma unroll
  for (int m = 0; m < M; ++m) scale[m] = 0.f;
#pragma unroll
  for (int m = 0; m <= M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<false>(
      w, 1, [&](int t) { seq_tile<M, U, REF, false, true>(tiles[t], T, xp, xcp, pull, keep, scale, inv_m, acc); },
      [&](int t) {
        seq_tile<M, U, REF, false, false>(tiles[w.nfull + t], T, xp, xcp, pull, keep, scale, inv_m, acc);
      },
      [&](int row) { block_sums_flush<M + 1>(acc, partials + row, prows); });
}

template <int M, int U, int REF>
__global__ __launch_bounds__(kBlock) void k_seq2(const Tile* __restrict__ tiles, const Walk w, int T,
                                                 float* const* __restrict__ xp,
                                                 const float* const* __restrict__ xcp, float pull, float keep,
                                                 float push, const double* __restrict__ partials, int nparts,
                                                 int prows, float* __restrict__ r_post_out) {
  // lambda / r_m from the partial sums (c = 0 - push/r, so scale = -c; zero distance: no push)
  float c[M], scale[M], inv_r[M];
  bool skip[M];
  coefficients_from_partials<M>(partials, nparts, prows, 0.f, push, c, skip, inv_r, r_post_out, nullptr, nullptr);
#pragma unroll
  for (int m = 0; m < M; ++m) scale[m] = skip[m] ? 0.f : -c[m];
  double unused[M + 1];
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<true>(
      w, 1, [&](int t) { seq_tile<M, U, REF, true, true>(tiles[t], T, xp, xcp, pull, keep, scale, inv_m, unused); },
      [&](int t) {
        seq_tile<M, U, REF, true, false>(tiles[w.nfull + t], T, xp, xcp, pull, keep, scale, inv_m, unused);
      },
      [](int) {});
}

// ------------------------------------------------------------------ AdamW local step
// Decoupled weight decay Adam: x <- x (1 - lr wd); m <- b1 m + (1-b1) g; s <- b2 s + (1-b2) g^2;
// x <- x - lr (m / bc1) / (sqrt(s / bc2) + eps), bc_i = 1 - b_i^t computed on the host.

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
  constexpr int kVec = vectors_per_lane(kStepTileElems);
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
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
  auto item_tiles = [&](int item, int ntile, int per, int first_tile, auto full) {
    constexpr bool kFull = decltype(full)::value;
    const dppf_walk::WorkerItem wi = dppf_walk::worker_item(item, ntile, per);
    if (wi.worker >= M) return;       // cannot happen while the host counts items the same way
#pragma unroll 1
    for (int t = wi.first_tile; t < wi.end_tile; ++t) {
      const Tile tl = tiles[first_tile + t];
      const size_t slot = static_cast<size_t>(wi.worker) * T + tl.tensor;
      adamw_tile<U, kFull>(xp[slot] + tl.offset, ap[slot] + tl.offset, sp[slot] + tl.offset, gp[slot] + tl.offset,
                           tl.count, hp);
    }
  };
  walk<false>(
      w, M, [&](int item) { item_tiles(item, w.nfull, kTilesPerWorkerItem, 0, std::true_type{}); },
      [&](int item) { item_tiles(item, w.ntiles - w.nfull, 1, w.nfull, std::false_type{}); }, [](int) {});
}

// Sweep 1 of the round with the AdamW step folded in: read x, m1, m2, g of all M workers, step,
// write m1, m2 and the stepped x (unlike SGD it cannot be rebuilt later from one extra read),
// accumulate the squared distances of the stepped x.  28 bytes per replica-parameter; the plain
// sweep 2 follows (8 bytes): 36 instead of 40.
template <int M, int U, bool FULL>
__device__ __forceinline__ void adamw_reduce_tile(const Tile tl, int T, float* const* __restrict__ xp,
                                                  float* const* __restrict__ ap, float* const* __restrict__ sp,
                                                  const float* const* __restrict__ gp, const AdamHyper hp,
                                                  float inv_m, double (&acc)[M + 1]) {
  constexpr int kVec = vectors_per_lane(sweep_tile_elems(M));
  static_assert(kVec % U == 0, "a lane's vectors of a tile are taken U at a time");
  float part[M + 1];
#pragma unroll
  for (int m = 0; m <= M; ++m) part[m] = 0.f;
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
    int e[U], n[U];
    f4 xv[U][M];
#pragma unroll
    for (int k = 0; k < U; ++k) {
      e[k] = 4 * (threadIdx.x + (it * U + k) * kBlock);
      n[k] = FULL ? 4 : tl.count - e[k];
    }
    // worker by worker (see sweep1_tile: 7 % faster here than all workers' loads at once), the next
    // workers' loads requested ahead
    constexpr int kAhead = lookahead(M, U, 4);
    f4 av[M][U], sv[M][U], gv[M][U];
    auto request = [&](int m) {
      const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
#pragma unroll
      for (int k = 0; k < U; ++k) {
        xv[k][m] = load4_stream<FULL>(xp[slot] + tl.offset + e[k], n[k]);
        av[m][k] = load4_stream<FULL>(ap[slot] + tl.offset + e[k], n[k]);
        sv[m][k] = load4_stream<FULL>(sp[slot] + tl.offset + e[k], n[k]);
        gv[m][k] = load4_stream<FULL>(gp[slot] + tl.offset + e[k], n[k]);
      }
    };
#pragma unroll
    for (int m = 0; m < kAhead && m < M; ++m) request(m);
#pragma unroll
    for (int m = 0; m < M; ++m) {
      if (m + kAhead < M) request(m + kAhead);
      const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
      float* x = xp[slot] + tl.offset;
      float* a = ap[slot] + tl.offset;
      float* q = sp[slot] + tl.offset;
#pragma unroll
      for (int k = 0; k < U; ++k) {
        f4 xn, an, sn;
        adamw_vec(xv[k][m], av[m][k], sv[m][k], gv[m][k], hp, xn, an, sn);
        store4_stream<FULL>(a + e[k], an, n[k]);
        store4_stream<FULL>(q + e[k], sn, n[k]);
        store4<FULL>(x + e[k], xn, n[k]);     // read again by sweep 2
        xv[k][m] = first_components<FULL>(xn, n[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const f4 mo = mean_offset<M>(xv[k], inv_m);
#pragma unroll
      for (int m = 0; m < M; ++m) part[m] = sumsq4((xv[k][m] - xv[k][0]) - mo, part[m]);
      part[M] = sumsq4(xv[k][0] + mo, part[M]);
    }
  }
#pragma unroll
  for (int m = 0; m <= M; ++m) acc[m] += static_cast<double>(part[m]);
}

template <int M, int U>
__global__ __launch_bounds__(kBlock) void k_adamw_reduce(const Tile* __restrict__ tiles, const Walk w, int T,
                                                         float* const* __restrict__ xp,
                                                         float* const* __restrict__ ap,
                                                         float* const* __restrict__ sp,
                                                         const float* const* __restrict__ gp, const AdamHyper hp,
                                                         double* __restrict__ partials, int prows) {
  double acc[M + 1];
#pragma unroll
  for (int m = 0; m <= M; ++m) acc[m] = 0.0;
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<false>(
      w, 1, [&](int t) { adamw_reduce_tile<M, U, true>(tiles[t], T, xp, ap, sp, gp, hp, inv_m, acc); },
      [&](int t) { adamw_reduce_tile<M, U, false>(tiles[w.nfull + t], T, xp, ap, sp, gp, hp, inv_m, acc); },
      [&](int row) { block_sums_flush<M + 1>(acc, partials + row, prows); });
}

// ------------------------------------------------ by-products the paper logs every round
// out[0] = relaxed MV = (1/M) sum r_m; out[1..M] = pull strength alpha r_m; out[M+1..2M] = lambda;
// with the norm of the average given: out[2M+1] = ||x_A||, out[2M+2] = relaxed MV / ||x_A||.
__global__ void k_round_stats(const float* __restrict__ r, int M, float pull, float push,
                              const float* __restrict__ avg_norm, float* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double s = 0.0;
    for (int m = 0; m < M; ++m) s += static_cast<double>(r[m]);
    const double mv = s / M;
    out[0] = static_cast<float>(mv);
    if (avg_norm) {
      const double na = static_cast<double>(avg_norm[0]);
      out[2 * M + 1] = static_cast<float>(na);
      out[2 * M + 2] = static_cast<float>(mv / na);
    }
  }
  for (int m = threadIdx.x; m < M; m += blockDim.x) {
    out[1 + m] = pull * r[m];
    out[1 + M + m] = push;
  }
}

__global__ void k_copy_scalar(const float* __restrict__ src, float* __restrict__ dst) {
  if (threadIdx.x == 0 && blockIdx.x == 0) dst[0] = src[0];
}

// ----------------------------------------------------------------- stand-alone local step
template <int U, bool FULL>
__device__ __forceinline__ void local_tile(float* x, float* v, const float* g, int count, float lr,
                                           float mu, float wd) {
  constexpr int kVec = vectors_per_lane(kStepTileElems);
#pragma unroll 1
  for (int it = 0; it < kVec / U; ++it) {
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
  auto item_tiles = [&](int item, int ntile, int per, int first_tile, auto full) {
    constexpr bool kFull = decltype(full)::value;
    const dppf_walk::WorkerItem wi = dppf_walk::worker_item(item, ntile, per);
    if (wi.worker >= M) return;       // cannot happen while the host counts items the same way
#pragma unroll 1
    for (int t = wi.first_tile; t < wi.end_tile; ++t) {
      const Tile tl = tiles[first_tile + t];
      const size_t slot = static_cast<size_t>(wi.worker) * T + tl.tensor;
      local_tile<U, kFull>(xp[slot] + tl.offset, vp[slot] + tl.offset, gp[slot] + tl.offset, tl.count, lr, mu, wd);
    }
  };
  walk<false>(
      w, M, [&](int item) { item_tiles(item, w.nfull, kTilesPerWorkerItem, 0, std::true_type{}); },
      [&](int item) { item_tiles(item, w.ntiles - w.nfull, 1, w.nfull, std::false_type{}); }, [](int) {});
}

// ============================================================ any M: a STORED average is read
// These kernels walk the tile list of kStepTileElems-element tiles.  A lane holds its four vectors
// of the average (and of whatever else is per element) and streams the workers past them,
// kAnyChunk workers' loads in flight at a time.
constexpr int kAnyVec = vectors_per_lane(kStepTileElems);

// ------------------------------- average over a runtime number of workers
template <bool FULL>
__device__ __forceinline__ void mean_any_tile(const Tile tl, int M, int T,
                                              float* const* __restrict__ xp, float* xb, float inv_m) {
  // The sums run over the workers in ascending order.
  f4 x0[kAnyVec], s[kAnyVec];
  const float* base0 = xp[tl.tensor] + tl.offset;
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    x0[it] = load4<FULL>(base0 + e, FULL ? 4 : tl.count - e);
    s[it] = (f4){0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll 1
  for (int m = 1; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kAnyVec];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) s[it] += t[k][it] - x0[it];
      }
  }
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    store4<FULL>(xb + e, x0[it] + scale_by_inverse_count(s[it], M, inv_m), FULL ? 4 : tl.count - e);
  }
}

__global__ __launch_bounds__(kBlock) void k_mean_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                     float* const* __restrict__ xp,
                                                     float* const* __restrict__ xbarp) {
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<false>(
      w, 1,
      [&](int t) {
        const Tile tl = tiles[t];
        mean_any_tile<true>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, inv_m);
      },
      [&](int t) {
        const Tile tl = tiles[w.nfull + t];
        mean_any_tile<false>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, inv_m);
      },
      [](int) {});
}

// ------------------------------- squared distances to a stored average (columns 0..M-1) and the
// squared norm of that average (column M)
template <bool FULL>
__device__ __forceinline__ void norms_any_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                               const float* xb, ColumnSums& sums) {
  f4 xbar[kAnyVec];
  float pa = 0.f;
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    xbar[it] = load4<FULL>(xb + e, FULL ? 4 : tl.count - e);
    pa = sumsq4(xbar[it], pa);
  }
  sums.add(pa, M);
#pragma unroll 1
  for (int m = 0; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kAnyVec];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4_stream<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
    float p[kAnyChunk];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k) {
      p[k] = 0.f;
      if (m + k < M) {
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) p[k] = sumsq4(t[k][it] - xbar[it], p[k]);   // past a partial tile's end: 0 - 0
      }
    }
    sums.add_group<kAnyChunk>(p, m, M);
  }
}

__global__ __launch_bounds__(kBlock) void k_norms_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                      float* const* __restrict__ xp,
                                                      const float* const* __restrict__ xbarp,
                                                      double* __restrict__ partials, int prows) {
  extern __shared__ double lds_cols[];
  ColumnSums sums;
  sums.init(lds_cols, M + 1);
  walk<false>(
      w, 1,
      [&](int t) {
        const Tile tl = tiles[t];
        norms_any_tile<true>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, sums);
      },
      [&](int t) {
        const Tile tl = tiles[w.nfull + t];
        norms_any_tile<false>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, sums);
      },
      [&](int row) { sums.flush(partials + row, prows); });
}

// ------------------------------- Eq. 5 (EXACT = false) or Eq. 4 (a) (EXACT = true) with the average
// (and, for the exact form, the sum of unit gap vectors S = sum_j (x_A - x_j)/r_j) read from memory:
//   x_m + (x_A - x_m) c_m [+ k2 S]
template <bool EXACT, bool FULL>
__device__ __forceinline__ void update_any_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                                const float* xb, const float* us, const Coef* __restrict__ coef,
                                                float k2) {
  f4 xbar[kAnyVec], usum[kAnyVec];
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    xbar[it] = load4_stream<FULL>(xb + e, FULL ? 4 : tl.count - e);
    if (EXACT) usum[it] = load4_stream<FULL>(us + e, FULL ? 4 : tl.count - e);
  }
#pragma unroll 1
  for (int m = 0; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kAnyVec];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4_stream<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
        const float c = coef[m + k].c;
        const bool stay = !EXACT && coef[m + k].skip != 0;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          f4 moved = fma4(xbar[it] - t[k][it], c, t[k][it]);
          if (EXACT) moved = fma4(usum[it], k2, moved);
          store4_stream<FULL>(base + e, stay ? t[k][it] : moved, FULL ? 4 : tl.count - e);
        }
      }
  }
}

template <bool EXACT>
__global__ __launch_bounds__(kBlock) void k_update_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                       float* const* __restrict__ xp,
                                                       const float* const* __restrict__ xbarp,
                                                       const float* const* __restrict__ sump,
                                                       const Coef* __restrict__ coef, float k2) {
  walk<false>(
      w, 1,
      [&](int t) {
        const Tile tl = tiles[t];
        update_any_tile<EXACT, true>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset,
                                     EXACT ? sump[tl.tensor] + tl.offset : nullptr, coef, k2);
      },
      [&](int t) {
        const Tile tl = tiles[w.nfull + t];
        update_any_tile<EXACT, false>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset,
                                      EXACT ? sump[tl.tensor] + tl.offset : nullptr, coef, k2);
      },
      [](int) {});
}

// ------------------------------- S = sum_j (x_A - x_j) / r_j of the exact update, stored
template <bool FULL>
__device__ __forceinline__ void unit_sum_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                              const float* xb, const Coef* __restrict__ coef, float* out) {
  // the sum runs over the workers in ascending order
  f4 xbar[kAnyVec], s[kAnyVec];
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    xbar[it] = load4<FULL>(xb + e, FULL ? 4 : tl.count - e);
    s[it] = (f4){0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll 1
  for (int m = 0; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kAnyVec];
    float wgt[kAnyChunk];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
        wgt[k] = coef[m + k].inv_r;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = load4<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) s[it] = fma4(xbar[it] - t[k][it], wgt[k], s[it]);
      }
  }
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    store4<FULL>(out + e, s[it], FULL ? 4 : tl.count - e);
  }
}

__global__ __launch_bounds__(kBlock) void k_unit_sum_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                         float* const* __restrict__ xp,
                                                         const float* const* __restrict__ xbarp,
                                                         const Coef* __restrict__ coef,
                                                         float* const* __restrict__ sump) {
  walk<false>(
      w, 1,
      [&](int t) {
        const Tile tl = tiles[t];
        unit_sum_tile<true>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, coef, sump[tl.tensor] + tl.offset);
      },
      [&](int t) {
        const Tile tl = tiles[w.nfull + t];
        unit_sum_tile<false>(tl, M, T, xp, xbarp[tl.tensor] + tl.offset, coef, sump[tl.tensor] + tl.offset);
      },
      [](int) {});
}

// ------------------------------- Alg. 1 literally for any M: the reference point of the push is x_C
// (REF = 1) or a stored average (REF = 2).  WRITE = false accumulates the squared norms of the
// pulled gaps, WRITE = true applies pull and push with lambda / r_m = -coef[m].c.
template <int REF, bool WRITE, bool FULL>
__device__ __forceinline__ void seq_any_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                             const float* xc, const float* rf, float pull, float keep,
                                             const Coef* __restrict__ coef, ColumnSums& sums) {
  f4 cv[kAnyVec], ref[kAnyVec];
#pragma unroll
  for (int it = 0; it < kAnyVec; ++it) {
    const int e = 4 * (threadIdx.x + it * kBlock);
    cv[it] = load4<FULL>(xc + e, FULL ? 4 : tl.count - e);
    ref[it] = (REF == 1) ? cv[it] : load4<FULL>(rf + e, FULL ? 4 : tl.count - e);
  }
#pragma unroll 1
  for (int m = 0; m < M; m += kAnyChunk) {
    f4 t[kAnyChunk][kAnyVec];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k)
      if (m + k < M) {
        const float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          t[k][it] = WRITE ? load4_stream<FULL>(base + e, FULL ? 4 : tl.count - e)
                           : load4<FULL>(base + e, FULL ? 4 : tl.count - e);
        }
      }
    float p[kAnyChunk];
#pragma unroll
    for (int k = 0; k < kAnyChunk; ++k) {
      p[k] = 0.f;
      if (m + k < M) {
        float* base = table_entry(xp, static_cast<size_t>(m + k) * T + tl.tensor) + tl.offset;
        const float scale = WRITE ? (coef[m + k].skip != 0 ? 0.f : -coef[m + k].c) : 0.f;
#pragma unroll
        for (int it = 0; it < kAnyVec; ++it) {
          const int e = 4 * (threadIdx.x + it * kBlock);
          const f4 pulled = fma4(cv[it], pull, t[k][it] * keep);
          const f4 gap = pulled - ref[it];
          if (WRITE) store4_stream<FULL>(base + e, fma4(gap, scale, pulled), FULL ? 4 : tl.count - e);
          else p[k] = sumsq4(gap, p[k]);       // lanes past a partial tile's end hold zeros throughout
        }
      }
    }
    if (!WRITE) sums.add_group<kAnyChunk>(p, m, M);
  }
}

template <int REF, bool WRITE>
__global__ __launch_bounds__(kBlock) void k_seq_any(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                    float* const* __restrict__ xp,
                                                    const float* const* __restrict__ xcp,
                                                    const float* const* __restrict__ refp, float pull, float keep,
                                                    const Coef* __restrict__ coef, double* __restrict__ partials,
                                                    int prows) {
  extern __shared__ double lds_cols[];
  ColumnSums sums;
  if (!WRITE) sums.init(lds_cols, M + 1);
  walk<false>(
      w, 1,
      [&](int t) {
        const Tile tl = tiles[t];
        seq_any_tile<REF, WRITE, true>(tl, M, T, xp, xcp[tl.tensor] + tl.offset,
                                       REF == 2 ? refp[tl.tensor] + tl.offset : nullptr, pull, keep, coef, sums);
      },
      [&](int t) {
        const Tile tl = tiles[w.nfull + t];
        seq_any_tile<REF, WRITE, false>(tl, M, T, xp, xcp[tl.tensor] + tl.offset,
                                        REF == 2 ? refp[tl.tensor] + tl.offset : nullptr, pull, keep, coef, sums);
      },
      [&](int row) {
        if (!WRITE) sums.flush(partials + row, prows);
      });
}

// ======================================================= 17 <= M <= 39: staged in LDS
// A tile is kLdsTileElems elements: one 16-byte vector per lane.  A lane streams the workers
// through registers kLdsChunk at a time (the next chunk's loads are issued before the current
// chunk is processed), parks every worker's vector in its own LDS column, and once the average is
// known reads them back.  LDS holds M x 256 vectors (4 KB per worker) and, for the reducing
// sweep, the per-wave running sums.
//
// Two things about the chunk pipeline were measured, not guessed.  (1) Every slot of a chunk
// issues its loads, also the slots past the last worker (they re-read the last worker and are never
// consumed): with a fixed number of loads per chunk the compiler can wait for exactly this chunk's
// data while the next chunk's loads stay in flight; loads under a condition make it wait for
// everything (the sweep ran 1.5 times longer).  (2) Carrying a chunk across tiles, to request the
// next tile's first workers before the current tile's second phase, made the generated code slower,
// not faster (+36 %), with items of one, two or four tiles alike: each tile starts its own pipeline.

// OPT: 0 = x as it is, 1 = momentum-SGD step folded in (v stored, stepped x kept only on chip),
// 2 = AdamW step folded in (m1, m2 and the stepped x stored); see LdsOptArgs.
template <int OPT, bool FULL>
struct LdsChunk {
  f4 x[kLdsChunk], a[kLdsChunk], s[kLdsChunk], g[kLdsChunk];
  __device__ __forceinline__ void load(int m0, int M, int T, const Tile& tl, int e, int n, float* const* xp,
                                       const LdsOptArgs& o) {
#pragma unroll
    for (int k = 0; k < kLdsChunk; ++k) {
      const int m = m0 + k < M ? m0 + k : M - 1;
      const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
      x[k] = load4_stream<FULL>(table_entry(xp, slot) + tl.offset + e, n);
      if (OPT != 0) {
        a[k] = load4_stream<FULL>(table_entry(o.vp, slot) + tl.offset + e, n);
        g[k] = load4_stream<FULL>(table_entry(o.gp, slot) + tl.offset + e, n);
      }
      if (OPT == 2) s[k] = load4_stream<FULL>(table_entry(o.sp, slot) + tl.offset + e, n);
    }
  }
  __device__ __forceinline__ f4 stepped(int k, int m, int T, const Tile& tl, int e, int n, float* const* xp,
                                        const LdsOptArgs& o) {
    if (OPT == 0) return x[k];
    const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
    if (OPT == 1) {
      const f4 ge = fma4(x[k], o.wd, g[k]);
      const f4 vn = fma4(a[k], o.mu, ge);
      store4_stream<FULL>(table_entry(o.vp, slot) + tl.offset + e, vn, n);
      return fma4(vn, -o.lr, x[k]);
    }
    f4 xn, an, sn;
    adamw_vec(x[k], a[k], s[k], g[k], o.adam, xn, an, sn);
    store4_stream<FULL>(table_entry(o.vp, slot) + tl.offset + e, an, n);
    store4_stream<FULL>(table_entry(o.sp, slot) + tl.offset + e, sn, n);
    store4<FULL>(table_entry(xp, slot) + tl.offset + e, xn, n);
    return first_components<FULL>(xn, n);
  }
};

template <int OPT, int XBAR, bool FULL>
__device__ __forceinline__ void sweep1_lds_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                                const LdsOptArgs& o, float* const* __restrict__ xbarp, float inv_m,
                                                f4* stage, ColumnSums& sums) {
  const int e = 4 * threadIdx.x;
  const int n = FULL ? 4 : tl.count - e;
  f4 x0 = {0.f, 0.f, 0.f, 0.f}, s = {0.f, 0.f, 0.f, 0.f};
  LdsChunk<OPT, FULL> ca, cb;
  auto consume = [&](LdsChunk<OPT, FULL>& c, int m0) {
#pragma unroll
    for (int k = 0; k < kLdsChunk; ++k)
      if (m0 + k < M) {
        const f4 xn = c.stepped(k, m0 + k, T, tl, e, n, xp, o);
        stage[(m0 + k) * kBlock + threadIdx.x] = xn;
        if (m0 + k == 0) x0 = xn;
        else s += xn - x0;
      }
  };
  int m0 = 0;
  ca.load(0, M, T, tl, e, n, xp, o);
#pragma unroll 1
  for (; m0 + 2 * kLdsChunk < M; m0 += 2 * kLdsChunk) {
    cb.load(m0 + kLdsChunk, M, T, tl, e, n, xp, o);
    consume(ca, m0);
    ca.load(m0 + 2 * kLdsChunk, M, T, tl, e, n, xp, o);
    consume(cb, m0 + kLdsChunk);
  }
  if (M - m0 > kLdsChunk) {
    cb.load(m0 + kLdsChunk, M, T, tl, e, n, xp, o);
    consume(ca, m0);
    consume(cb, m0 + kLdsChunk);
  } else {
    consume(ca, m0);
  }
  const f4 mo = scale_by_inverse_count(s, M, inv_m);
  const f4 xa = x0 + mo;
  if (XBAR == 1) store4_stream<FULL>(xbarp[tl.tensor] + tl.offset + e, xa, n);
  sums.add(sumsq4(xa, 0.f), M);
#pragma unroll 1
  for (int g0 = 0; g0 < M; g0 += 8) {
    float p[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      p[k] = 0.f;
      if (g0 + k < M) p[k] = sumsq4((stage[(g0 + k) * kBlock + threadIdx.x] - x0) - mo, 0.f);
    }
    sums.add_group<8>(p, g0, M);
  }
}

template <int OPT, int XBAR>
__global__ __launch_bounds__(kBlock) void k_sweep1_lds(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                       float* const* __restrict__ xp, const LdsOptArgs o,
                                                       float* const* __restrict__ xbarp,
                                                       double* __restrict__ partials, int prows) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  f4* stage = reinterpret_cast<f4*>(lds_raw);
  ColumnSums sums;
  sums.init(reinterpret_cast<double*>(lds_raw + static_cast<size_t>(M) * kBlock * sizeof(f4)), M + 1);
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<false>(
      w, 1, [&](int t) { sweep1_lds_tile<OPT, XBAR, true>(tiles[t], M, T, xp, o, xbarp, inv_m, stage, sums); },
      [&](int t) { sweep1_lds_tile<OPT, XBAR, false>(tiles[w.nfull + t], M, T, xp, o, xbarp, inv_m, stage, sums); },
      [&](int row) { sums.flush(partials + row, prows); });
}

// MODE: 0 = Eq. 5; 1 = Eq. 5 on x - lr v (fused momentum-SGD round: x in memory is still the old
// value, v already the new momentum); 2 = the exact two-term update of Eq. 4 (a).
template <int MODE, bool FULL>
__device__ __forceinline__ void sweep2_lds_tile(const Tile tl, int M, int T, float* const* __restrict__ xp,
                                                const float* const* __restrict__ vp, float lr,
                                                const Coef* __restrict__ coef, float k2, float inv_m, f4* stage) {
  const int e = 4 * threadIdx.x;
  const int n = FULL ? 4 : tl.count - e;
  f4 x0 = {0.f, 0.f, 0.f, 0.f}, s = {0.f, 0.f, 0.f, 0.f};
  f4 ax[kLdsChunk], av[kLdsChunk], bx[kLdsChunk], bv[kLdsChunk];
  auto load = [&](f4 (&cx)[kLdsChunk], f4 (&cv)[kLdsChunk], int m0) {   // unconditional, see above
#pragma unroll
    for (int k = 0; k < kLdsChunk; ++k) {
      const int m = m0 + k < M ? m0 + k : M - 1;
      const size_t slot = static_cast<size_t>(m) * T + tl.tensor;
      cx[k] = load4_stream<FULL>(table_entry(xp, slot) + tl.offset + e, n);
      if (MODE == 1) cv[k] = load4_stream<FULL>(table_entry(vp, slot) + tl.offset + e, n);
    }
  };
  auto consume = [&](f4 (&cx)[kLdsChunk], f4 (&cv)[kLdsChunk], int m0) {
#pragma unroll
    for (int k = 0; k < kLdsChunk; ++k)
      if (m0 + k < M) {
        const f4 xn = (MODE == 1) ? fma4(cv[k], -lr, cx[k]) : cx[k];
        stage[(m0 + k) * kBlock + threadIdx.x] = xn;
        if (m0 + k == 0) x0 = xn;
        else s += xn - x0;
      }
  };
  int m0 = 0;                // two alternating chunks, see sweep1_lds_tile
  load(ax, av, 0);
#pragma unroll 1
  for (; m0 + 2 * kLdsChunk < M; m0 += 2 * kLdsChunk) {
    load(bx, bv, m0 + kLdsChunk);
    consume(ax, av, m0);
    load(ax, av, m0 + 2 * kLdsChunk);
    consume(bx, bv, m0 + kLdsChunk);
  }
  if (M - m0 > kLdsChunk) {
    load(bx, bv, m0 + kLdsChunk);
    consume(ax, av, m0);
    consume(bx, bv, m0 + kLdsChunk);
  } else {
    consume(ax, av, m0);
  }
  const f4 mo = scale_by_inverse_count(s, M, inv_m);
  f4 usum = {0.f, 0.f, 0.f, 0.f};
  if (MODE == 2) {
#pragma unroll 4
    for (int m = 0; m < M; ++m)
      usum = fma4(mo - (stage[m * kBlock + threadIdx.x] - x0), coef[m].inv_r, usum);
  }
#pragma unroll 4
  for (int m = 0; m < M; ++m) {
    const f4 xm = stage[m * kBlock + threadIdx.x];
    f4 moved = fma4(mo - (xm - x0), coef[m].c, xm);
    if (MODE == 2) moved = fma4(usum, k2, moved);
    const bool stay = MODE != 2 && coef[m].skip != 0;
    store4_stream<FULL>(table_entry(xp, static_cast<size_t>(m) * T + tl.tensor) + tl.offset + e, stay ? xm : moved, n);
  }
}

template <int MODE>
__global__ __launch_bounds__(kBlock) void k_sweep2_lds(const Tile* __restrict__ tiles, const Walk w, int M, int T,
                                                       float* const* __restrict__ xp,
                                                       const float* const* __restrict__ vp, float lr,
                                                       const Coef* __restrict__ coef, float k2) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  f4* stage = reinterpret_cast<f4*>(lds_raw);
  const float inv_m = 1.0f / static_cast<float>(M);
  walk<true>(
      w, 1, [&](int t) { sweep2_lds_tile<MODE, true>(tiles[t], M, T, xp, vp, lr, coef, k2, inv_m, stage); },
      [&](int t) { sweep2_lds_tile<MODE, false>(tiles[w.nfull + t], M, T, xp, vp, lr, coef, k2, inv_m, stage); },
      [](int) {});
}

// ------------------------------- work decomposition of ONE flat tensor, built on the device
// For callers that may not allocate: the tile list of a single tensor of d elements per worker
// (full tiles first, then the ragged tail, exactly what the host-side list builder produces) and
// the table of the M workers' base pointers x + m*ld are written straight into caller-provided
// device memory, and the on-demand counter is put back to zero.
__global__ __launch_bounds__(kBlock) void k_flat_setup(Tile* __restrict__ tiles, long long d, int tile_elems,
                                                       float** __restrict__ ptrs, float* x, long long ld, int M,
                                                       Sched* __restrict__ sched) {
  const long long nfull = d / tile_elems;
  const int tail = static_cast<int>(d - nfull * tile_elems);
  const long long ntiles = nfull + (tail > 0 ? 1 : 0);
  const long long stride = static_cast<long long>(gridDim.x) * kBlock;
  for (long long t = static_cast<long long>(blockIdx.x) * kBlock + threadIdx.x; t < ntiles; t += stride) {
    Tile tl;
    tl.offset = t * tile_elems;
    tl.tensor = 0;
    tl.count = t < nfull ? tile_elems : tail;
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

}  // namespace

#endif  // DPPF_KERNELS_H_
