// Instantiations and launch dispatch of the grouped bf16 shard GEMM (kernel template in caat_gemm_kernel.h).
#include "caat_gemm_kernel.h"

namespace caat {

// Measured choices (C2/C3 shard shapes, warm clocks): operands that are K-contiguous in memory go global -> LDS
// directly and run best with 8 waves (2 x 4) per 256 x 256 tile; the weight-gradient layout (both operands
// transposed through registers) needs the registers of the 4-wave (2 x 2) arrangement.
typedef TileCfg<256, 256, 2, 4, 2, true> CfgDma8;
typedef TileCfg<256, 256, 2, 2, 2, false> CfgReg4;
// Decode (at most 64 token rows per rank): the GEMM is a weight stream, so small tiles that put one workgroup on
// every 64 weight rows (several per CU) replace the big tile, which would leave most CUs idle.
typedef TileCfg<64, 64, 2, 2, 2, true> CfgSkinny;
typedef TileCfg<64, 128, 2, 2, 2, true> CfgSkinnySwi;

hipError_t launch_gemm(const GemmParams& p, int layout, int epilogue, hipStream_t s) {
  // buffer-load offsets are 32-bit and relative to the tile origin: the farthest row a tile touches times the
  // row stride must stay below 2 GiB
  const long long far_rows = (epilogue == EPI_SWIGLU_FWD ? (long long)p.half : 0) + 256 + 64;
  if (far_rows * p.lda * 2 >= 0x7FFFFFFFLL || far_rows * p.ldb * 2 >= 0x7FFFFFFFLL) return hipErrorInvalidValue;
  if (layout == 0 && p.M <= 64) {
    switch (epilogue) {
      case EPI_PLAIN: return launch_one<CfgSkinny, false, false, EPI_PLAIN>(p, s);
      case EPI_GELU_FWD: return launch_one<CfgSkinny, false, false, EPI_GELU_FWD>(p, s);
      case EPI_SWIGLU_FWD: return launch_one<CfgSkinnySwi, false, false, EPI_SWIGLU_FWD>(p, s);
      case EPI_ROWPAR: return launch_one<CfgSkinny, false, false, EPI_ROWPAR>(p, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (layout) {
    case 0:  // NT
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<CfgDma8, false, false, EPI_PLAIN>(p, s);
        case EPI_GELU_FWD: return launch_one<CfgDma8, false, false, EPI_GELU_FWD>(p, s);
        case EPI_SWIGLU_FWD: return launch_one<CfgDma8, false, false, EPI_SWIGLU_FWD>(p, s);
        case EPI_ROWPAR: return launch_one<CfgDma8, false, false, EPI_ROWPAR>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 1:  // NN
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<CfgDma8, false, true, EPI_PLAIN>(p, s);
        case EPI_GELU_BWD: return launch_one<CfgDma8, false, true, EPI_GELU_BWD>(p, s);
        case EPI_SWIGLU_BWD: return launch_one<CfgDma8, false, true, EPI_SWIGLU_BWD>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 2:  // TN
      if (epilogue == EPI_PLAIN) return launch_one<CfgReg4, true, true, EPI_PLAIN>(p, s);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace caat
