// Stand-in for <hip/hip_runtime.h> that lets the per-rank device functions of
// the HIP library be compiled by g++ and run on the CPU.  Only what
// bcast_device.hpp uses is provided.
//
// Cross-lane operations go through shim_wave::cross_lane.  Inside
// shim_wave::run the lanes of a wavefront are coroutines that meet at every
// such operation, so __any, readfirstlane and the shuffles see the values of
// all lanes that take part, as on the GPU; outside of it they are those of a
// wavefront of one lane.
#pragma once
#include <stdint.h>

#define BCAST_DEVICE_CODE_ON_HOST 1   // the one instruction written in assembly has a C form for this
#define __device__
#define __forceinline__ inline
#define __host__

struct uint4 { unsigned x, y, z, w; };

static inline int __ffs(int x) { return x == 0 ? 0 : __builtin_ctz((unsigned)x) + 1; }
static inline int __clz(int x) { return x == 0 ? 32 : __builtin_clz((unsigned)x); }
static inline int __popc(unsigned x) { return __builtin_popcount(x); }

namespace shim_wave {
enum Op : int { kAny = 0, kShflXor = 1, kFirstLane = 2 };
// `site` names the place in the source: lanes that meet must all come from the same one.
int cross_lane(Op op, int value, int arg, int site);
}  // namespace shim_wave

#define __any(pred) shim_wave::cross_lane(shim_wave::kAny, (pred) ? 1 : 0, 0, __LINE__)
#define __shfl_xor(v, mask, width) shim_wave::cross_lane(shim_wave::kShflXor, (v), (mask), __LINE__)
#define __builtin_amdgcn_readfirstlane(v) shim_wave::cross_lane(shim_wave::kFirstLane, (v), 0, __LINE__)
