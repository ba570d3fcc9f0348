// Stand-in for <hip/hip_runtime.h> that lets the per-rank device functions of
// the HIP library be compiled by g++ and run on the CPU, one "lane" at a time.
// Only what bcast_device.hpp uses is provided.
#pragma once
#include <stdint.h>

#define __device__
#define __forceinline__ inline
#define __host__

static inline int __ffs(int x) { return x == 0 ? 0 : __builtin_ctz((unsigned)x) + 1; }
static inline int __clz(int x) { return x == 0 ? 32 : __builtin_clz((unsigned)x); }
static inline int __popc(unsigned x) { return __builtin_popcount(x); }
// cross-lane operations for a wavefront of one lane
static inline int __any(int pred) { return pred != 0; }
static inline int __shfl_xor(int v, int, int) { return v; }
static inline int __builtin_amdgcn_readfirstlane(int v) { return v; }
