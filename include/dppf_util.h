/*
 * dppf_util.h -- measurement aids that ship with the DPPF library but are no part of the method:
 * a plain copy of known size (bandwidth reference, and the launch against which hardware byte
 * counters are scaled) and a streaming probe for a given mix of read and written arrays.
 * Conventions (device pointers, stream as void*, return codes) are those of dppf.h.
 */
#ifndef DPPF_UTIL_H_
#define DPPF_UTIL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A plain copy dst[i] = src[i] of n floats (device pointers, 4-byte aligned, non-overlapping)
 * using the same 16-byte load/store path as the library's kernels: a launch of known size (4n
 * bytes read, 4n written) against which hardware counters can be scaled.  */
int dppf_util_copy(float* dst, const float* src, int64_t n, void* stream);

/* Measurement aid: streams `reads` arrays and writes `writes` arrays of n floats each; array k
 * starts at base + k*stride floats (base 16-byte aligned, stride >= n, multiple of 4).  Written
 * arrays are k = reads..reads+writes-1, or k = 0..writes-1 when inplace != 0 (the lane that read
 * an element overwrites it).  Only elements below the largest multiple of the probe's tile are
 * touched.  Supported (reads, writes): (1,0) (4,0) (12,0) (0,1) (0,4) (1,1) (2,1) and, with or without
 * inplace, (4,4) (8,4) (12,4) (12,8), and in place only (16,8) (24,8); anything else returns
 * DPPF_EINVAL.  blocks_per_cu in 1..16.  on_demand = 0: the blocks split the work evenly;
 * on_demand != 0: they take work on demand the way the library's read-write sweeps do (the second
 * half of it, or all of it when the launch moves more than about 2 GB).  The probe keeps one
 * counter per device: calls that could overlap on one device (different streams) must not both
 * use on_demand.
 * Timing is the caller's job (events around the call).  */
int dppf_util_stream_probe(float* base, int64_t stride, int64_t n, int reads, int writes, int inplace,
                           int blocks_per_cu, int on_demand, void* stream);

/* Measurement aid: the same kind of traffic in the order the library's sweeps produce it.  The
 * arrays (array k at base + k*stride floats, as above) form `groups` groups of `reads_per_group`
 * arrays each.  Inside a tile of 256*vectors 16-byte vectors a lane takes one group after the
 * other: it loads the group's reads_per_group*vectors vectors, adds them and overwrites the group's
 * first array with the sum (with half the value when reads_per_group is 1) -- per group and
 * element reads_per_group reads and one write in place, the pattern of a sweep that handles one
 * worker after the other.  `ahead` = how many groups' loads are requested before the current
 * group's data are waited for.  One tile per work item; on_demand and blocks_per_cu as above (same
 * per-device counter, same rule about overlapping calls); only elements below the largest multiple
 * of the tile are touched.  Supported (groups, reads_per_group, vectors, ahead): (2,3,4,0) (4,3,4,0)
 * (4,3,4,3) (4,3,2,0) (4,3,8,0) (4,2,4,0) (4,2,4,3) (4,2,8,0) (8,3,2,0) (8,3,2,7) (8,2,2,0) (8,2,2,7)
 * (16,3,2,0) (16,3,2,7) (16,2,2,7) (4,1,4,0); anything else returns DPPF_EINVAL.  */
int dppf_util_stream_probe_grouped(float* base, int64_t stride, int64_t n, int groups, int reads_per_group,
                                   int vectors, int ahead, int blocks_per_cu, int on_demand, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DPPF_UTIL_H_ */
