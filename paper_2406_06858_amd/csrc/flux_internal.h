// Host-side declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include "flux.h"
#include "flux_device.h"

namespace flux {

// One entry per compiled tile configuration (index = public id - 1).
struct CfgInfo {
  int bm, bn, bk;
  int occupancy;   // workgroups per CU the kernel is built for
  int stages;      // LDS stages of the direct-to-LDS kernel (more than two: the deep pipeline)
  hipError_t (*launch)(int epi, int wait, int edge, const GemmArgs& a, int grid, hipStream_t s);
};

constexpr int NUM_CFGS = 10;
extern CfgInfo g_cfgs[NUM_CFGS];

#define FLUX_DECLARE_CFG(ID) \
  hipError_t launch_cfg##ID(int epi, int wait, int edge, const GemmArgs& a, int grid, hipStream_t s); \
  void info_cfg##ID(int* bm, int* bn, int* bk);
FLUX_DECLARE_CFG(1)
FLUX_DECLARE_CFG(2)
FLUX_DECLARE_CFG(3)
FLUX_DECLARE_CFG(4)
FLUX_DECLARE_CFG(5)
FLUX_DECLARE_CFG(6)
FLUX_DECLARE_CFG(7)
FLUX_DECLARE_CFG(8)
FLUX_DECLARE_CFG(9)
FLUX_DECLARE_CFG(10)

}  // namespace flux
