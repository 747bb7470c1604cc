// Instantiates the GEMM kernel family for ONE tile configuration; compiled once per
// configuration with -DFLUX_CFG_ID=<id> so the configurations build in parallel.
#include "flux_internal.h"

namespace flux {

#if FLUX_CFG_ID == 1
#define FLUX_CFG_PARAMS 256, 256, 64, 2, 2, 2, 1   // 128x128 per wave, one workgroup per CU
#elif FLUX_CFG_ID == 2
#define FLUX_CFG_PARAMS 256, 128, 64, 2, 2, 3, 1   // 128x64 per wave: twice the tiles of 256x256; three LDS stages
#elif FLUX_CFG_ID == 3
#define FLUX_CFG_PARAMS 128, 128, 64, 2, 2, 2, 2   // 64x64 per wave
#elif FLUX_CFG_ID == 4
#define FLUX_CFG_PARAMS 64, 64, 64, 2, 2, 2, 2     // 32x32 per wave, small problems
#elif FLUX_CFG_ID == 5
#define FLUX_CFG_PARAMS 64, 128, 64, 2, 2, 2, 2    // decode, M <= 64
#elif FLUX_CFG_ID == 6
#define FLUX_CFG_PARAMS 32, 128, 64, 1, 4, 2, 2    // decode, M <= 32
#elif FLUX_CFG_ID == 7
#define FLUX_CFG_PARAMS 64, 64, 64, 2, 2, 6, 1     // decode, M <= 64: six LDS stages, one workgroup per CU
#elif FLUX_CFG_ID == 8
#define FLUX_CFG_PARAMS 32, 128, 64, 1, 4, 6, 1    // decode, M <= 32: six LDS stages
#elif FLUX_CFG_ID == 9
#define FLUX_CFG_PARAMS 64, 128, 64, 2, 2, 4, 1    // M <= 256: four LDS stages
#elif FLUX_CFG_ID == 10
#define FLUX_CFG_PARAMS 64, 128, 64, 2, 2, 3, 2    // EXPERIMENT: 64x128, three stages, two workgroups per CU
#else
#error "FLUX_CFG_ID must be 1..10"
#endif
typedef TileCfg<FLUX_CFG_PARAMS> Cfg;            // B as [K,N]
typedef TileCfg<FLUX_CFG_PARAMS, true> CfgNK;    // B as [N,K]

// Shapes the tile divides take a direct-to-LDS kernel (two stages, or the deep pipeline for
// configurations with more); ragged shapes the register-staged one, which masks rows, columns
// and the K tail.  The deep pipeline also takes shapes where only M is ragged (edge = 2).
enum : int { EDGE_NONE = 0, EDGE_ANY = 1, EDGE_ROWS = 2 };

template <class Cfg, int EPI, bool WAIT, int EDGE>
static hipError_t launch_one(const GemmArgs& a, int grid, hipStream_t s) {
  if constexpr (EDGE == EDGE_NONE && Cfg::NSTAGE == 2) {
    if constexpr (!WAIT && Cfg::OCC == 1) {
      if (a.persist_blocks > 0) {
        hipLaunchKernelGGL((gemm_kernel_dma_resident<Cfg, EPI>), dim3(grid), dim3(Cfg::NT), 0, s, a);
        return hipGetLastError();
      }
    }
    hipLaunchKernelGGL((gemm_kernel_dma<Cfg, EPI, WAIT>), dim3(grid), dim3(Cfg::NT), 0, s, a);
    return hipGetLastError();
  } else if constexpr (EDGE != EDGE_ANY && Cfg::NSTAGE >= 3) {
    hipLaunchKernelGGL((gemm_kernel_dma_deep<Cfg, EPI, WAIT, EDGE == EDGE_ROWS>), dim3(grid), dim3(Cfg::NT), 0, s, a);
    return hipGetLastError();
  } else if constexpr (EDGE == EDGE_ROWS) {
    return hipErrorInvalidValue;     // only asked of the deep pipeline
  } else {
    auto k = gemm_kernel<Cfg, EPI, WAIT, EDGE == EDGE_ANY>;
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(Cfg::NT), Cfg::LDS_BYTES, s, a);
    return hipGetLastError();
  }
}

template <class Cfg, int EPI, bool WAIT>
static hipError_t launch_edge(int edge, const GemmArgs& a, int grid, hipStream_t s) {
  if (edge == EDGE_ANY) return launch_one<Cfg, EPI, WAIT, EDGE_ANY>(a, grid, s);
  if (edge == EDGE_ROWS) return launch_one<Cfg, EPI, WAIT, EDGE_ROWS>(a, grid, s);
  return launch_one<Cfg, EPI, WAIT, EDGE_NONE>(a, grid, s);
}

template <class Cfg>
static hipError_t launch_layout(int epi, int wait, int edge, const GemmArgs& a, int grid, hipStream_t s) {
  if (epi == EPI_RS) return launch_edge<Cfg, EPI_RS, false>(edge, a, grid, s);
  if (wait) return launch_edge<Cfg, EPI_PLAIN, true>(edge, a, grid, s);
  return launch_edge<Cfg, EPI_PLAIN, false>(edge, a, grid, s);
}

#define FLUX_CAT2(a, b) a##b
#define FLUX_CAT(a, b) FLUX_CAT2(a, b)

hipError_t FLUX_CAT(launch_cfg, FLUX_CFG_ID)(int epi, int wait, int edge, const GemmArgs& a, int grid, hipStream_t s) {
  // one set of kernels per layout of B
  if (a.b_is_nk) return launch_layout<CfgNK>(epi, wait, edge, a, grid, s);
  return launch_layout<Cfg>(epi, wait, edge, a, grid, s);
}

void FLUX_CAT(info_cfg, FLUX_CFG_ID)(int* bm, int* bn, int* bk) {
  *bm = Cfg::BM; *bn = Cfg::BN; *bk = Cfg::BK;
}

}  // namespace flux
