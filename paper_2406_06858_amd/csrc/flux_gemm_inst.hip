// Instantiates the GEMM kernel family for ONE tile configuration; compiled once per
// configuration with -DFLUX_CFG_ID=<id> so the configurations build in parallel.
#include "flux_internal.h"

namespace flux {

#if FLUX_CFG_ID == 1
typedef TileCfg<256, 256, 64, 2, 2, 2, 1> Cfg;   // 128x128 per wave, one workgroup per CU
#elif FLUX_CFG_ID == 2
typedef TileCfg<256, 128, 64, 2, 2, 2, 1> Cfg;   // 128x64 per wave: twice the tiles of 256x256
#elif FLUX_CFG_ID == 3
typedef TileCfg<128, 128, 64, 2, 2, 2, 2> Cfg;   // 64x64 per wave
#elif FLUX_CFG_ID == 4
typedef TileCfg<64, 64, 64, 2, 2, 2, 2> Cfg;     // 32x32 per wave, small problems
#elif FLUX_CFG_ID == 5
typedef TileCfg<64, 128, 64, 2, 2, 2, 2> Cfg;    // decode, M <= 64
#elif FLUX_CFG_ID == 6
typedef TileCfg<32, 128, 64, 1, 4, 2, 2> Cfg;    // decode, M <= 32
#else
#error "FLUX_CFG_ID must be 1..6"
#endif

// Shapes the tile divides take the direct-to-LDS kernel; ragged shapes the register-staged one,
// which masks rows, columns and the K tail.
template <int EPI, bool WAIT, bool EDGE>
static hipError_t launch_one(const GemmArgs& a, int grid, hipStream_t s) {
  if constexpr (!EDGE && Cfg::NSTAGE == 2) {
    hipLaunchKernelGGL((gemm_kernel_dma<Cfg, EPI, WAIT>), dim3(grid), dim3(Cfg::NT), 0, s, a);
    return hipGetLastError();
  } else {
    auto k = gemm_kernel<Cfg, EPI, WAIT, EDGE>;
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

#define FLUX_CAT2(a, b) a##b
#define FLUX_CAT(a, b) FLUX_CAT2(a, b)

hipError_t FLUX_CAT(launch_cfg, FLUX_CFG_ID)(int epi, int wait, int edge, const GemmArgs& a, int grid, hipStream_t s) {
  if (epi == EPI_RS) return edge ? launch_one<EPI_RS, false, true>(a, grid, s) : launch_one<EPI_RS, false, false>(a, grid, s);
  if (wait) return edge ? launch_one<EPI_PLAIN, true, true>(a, grid, s) : launch_one<EPI_PLAIN, true, false>(a, grid, s);
  return edge ? launch_one<EPI_PLAIN, false, true>(a, grid, s) : launch_one<EPI_PLAIN, false, false>(a, grid, s);
}

void FLUX_CAT(info_cfg, FLUX_CFG_ID)(int* bm, int* bn, int* bk) {
  *bm = Cfg::BM; *bn = Cfg::BN; *bk = Cfg::BK;
}

}  // namespace flux
