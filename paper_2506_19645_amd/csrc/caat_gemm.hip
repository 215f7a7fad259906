// Instantiations and launch dispatch of the grouped bf16 shard GEMM (kernel template in caat_gemm_kernel.h).
#include <algorithm>
#include "caat_gemm_kernel.h"

namespace caat {

// Tile choices: 256 x 256 tiles with 8 waves (2 x 4) and 2 LDS stages of 64 k for the block-sized GEMMs of every
// layout (with 4 stages of 32 k an operand that is contiguous along K was fetched in 64-byte pieces of rows that lie
// kilobytes apart, which cost the NT GEMMs 12 %; 64-k stages fetch whole 128-byte lines).  For decode (at most 64 token rows per rank) the GEMM is a weight stream, so small tiles that put a
// workgroup on every 64 (or, for wide outputs, 128) weight rows replace the big tile; their stages are 64 k deep so
// that a weight row is fetched 128 contiguous bytes at a time (64-byte pieces of rows that lie kilobytes apart cost
// about a fifth of the HBM rate), 4 stages, two workgroups per CU.
typedef TileCfg<256, 256, 2, 4, 2, 2, true, 64> CfgBig;
typedef TileCfg<128, 128, 2, 2, 2, 2, false, 64> CfgMid;   // problems with too few 256 x 256 tiles to fill the chip
typedef TileCfg<64, 64, 2, 2, 4, 2, false, 64> CfgSkinny;
typedef TileCfg<64, 128, 2, 2, 4, 2, false, 64> CfgSkinnyWide;
typedef CfgSkinnyWide CfgSkinnySwi;

// every (layout, epilogue) pair that exists, for one block-sized tile shape
template <class CFG>
static hipError_t launch_block_sized(const GemmParams& p, int layout, int epilogue, hipStream_t s) {
  switch (layout) {
    case 0:  // NT
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<CFG, false, false, EPI_PLAIN>(p, s);
        case EPI_GELU_FWD: return launch_one<CFG, false, false, EPI_GELU_FWD>(p, s);
        case EPI_SWIGLU_FWD: return launch_one<CFG, false, false, EPI_SWIGLU_FWD>(p, s);
        case EPI_ROWPAR: return launch_one<CFG, false, false, EPI_ROWPAR>(p, s);
        case EPI_SHARED_BCAST: return launch_one<CFG, false, false, EPI_SHARED_BCAST>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 1:  // NN
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<CFG, false, true, EPI_PLAIN>(p, s);
        case EPI_GELU_BWD: return launch_one<CFG, false, true, EPI_GELU_BWD>(p, s);
        case EPI_SWIGLU_BWD: return launch_one<CFG, false, true, EPI_SWIGLU_BWD>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 2:  // TN
      if (epilogue == EPI_PLAIN) return launch_one<CFG, true, true, EPI_PLAIN>(p, s);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

static int compute_units() {
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
      n_cu = v;
    if (n_cu <= 0) n_cu = 256;
  }
  return n_cu;
}

// Decode (at most 64 token rows per rank): the launch streams N weight rows per rank, and what a compute unit can have
// in flight is bounded, so its time is set by the bytes it has to pull: per tile the weight rows the tile covers (from
// HBM) plus the 64 activation rows every tile re-reads (from L2, at about a third of the latency: counted as 20 rows),
// times the tiles a compute unit gets.  Among the widths a tile may cover (multiples of 8 up to the MFMA tile's), take
// the one that minimises this, the widest on a tie.  Example: 8 ranks x 1536 rows in tiles of 64 are 192 tiles (a
// quarter of the chip idle), in tiles of 48 they are 256.
struct DecodeTile {
  bool wide;   // 64 x 128 tile (CfgSkinnyWide) instead of 64 x 64; SwiGLU always takes its own 64 x 128 tile
  int bn_out;  // output columns one tile covers
};
static DecodeTile choose_decode_tile(int G, int N, int epilogue) {
  DecodeTile t;
  t.wide = (N >= 2048) && (epilogue == EPI_PLAIN || epilogue == EPI_ROWPAR || epilogue == EPI_SHARED_BCAST);
  const int full = epilogue == EPI_SWIGLU_FWD ? CfgSkinnySwi::BN / 2 : (t.wide ? CfgSkinnyWide::BN : CfgSkinny::BN);
  const int n_cu = compute_units();
  t.bn_out = full;
  long long best = -1;
  for (int bn = full; bn >= 16; bn -= 8) {
    const long long tiles = (long long)((N + bn - 1) / bn) * G;
    const long long cost = ((tiles + n_cu - 1) / n_cu) * ((epilogue == EPI_SWIGLU_FWD ? 2 : 1) * bn + 20);
    if (best < 0 || cost < best) {
      best = cost;
      t.bn_out = bn;
    }
  }
  return t;
}

hipError_t launch_gemm(const GemmParams& p, int layout, int epilogue, hipStream_t s) {
  // buffer-load offsets are 32-bit and relative to the tile origin: the farthest row a tile touches times the
  // row stride must stay below 2 GiB
  const long long far_rows = (epilogue == EPI_SWIGLU_FWD ? (long long)p.half : 0) + 256 + 64;  // rows or k-rows
  if (far_rows * p.lda * 2 >= 0x7FFFF000LL || far_rows * p.ldb * 2 >= 0x7FFFF000LL) return hipErrorInvalidValue;
  // the epilogue's buffer offsets are relative to a wave's first row: up to 256 rows of any output / second operand
  const long long ldmax = std::max(std::max(p.ldc, p.ldc2), p.ldaux);
  if ((256 * ldmax + 2 * (long long)p.half + (long long)p.N) * 2 >= 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const int n_cu = compute_units();
  if (layout == 0 && p.M <= 64) {
    const DecodeTile t = choose_decode_tile(p.G, p.N, epilogue);
    GemmParams q = p;
    q.bn_out = t.bn_out;
    if (t.wide) {
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<CfgSkinnyWide, false, false, EPI_PLAIN>(q, s);
        case EPI_ROWPAR: return launch_one<CfgSkinnyWide, false, false, EPI_ROWPAR>(q, s);
        default: return launch_one<CfgSkinnyWide, false, false, EPI_SHARED_BCAST>(q, s);
      }
    }
    switch (epilogue) {
      case EPI_PLAIN: return launch_one<CfgSkinny, false, false, EPI_PLAIN>(q, s);
      case EPI_GELU_FWD: return launch_one<CfgSkinny, false, false, EPI_GELU_FWD>(q, s);
      case EPI_SWIGLU_FWD: return launch_one<CfgSkinnySwi, false, false, EPI_SWIGLU_FWD>(q, s);
      case EPI_ROWPAR: return launch_one<CfgSkinny, false, false, EPI_ROWPAR>(q, s);
      case EPI_SHARED_BCAST: return launch_one<CfgSkinny, false, false, EPI_SHARED_BCAST>(q, s);
      default: return hipErrorInvalidValue;
    }
  }
  // 256 x 256 tiles (one workgroup per CU) unless they would leave much of the chip idle: then 128 x 128 tiles, two
  // workgroups per CU (measured 17 % less efficient per tile at full occupancy, hence the factor).  Occupancy of a launch =
  // tiles / (rounds x slots), times the fraction of the tiles' area that lies inside the matrix.
  auto occupancy = [&](long long bm, long long bn, long long slots) {
    const long long bn_out = epilogue == EPI_SWIGLU_FWD ? bn / 2 : bn;
    const long long tm = (p.M + bm - 1) / bm, tn = (p.N + bn_out - 1) / bn_out;
    const long long tiles = tm * tn * p.G;
    const long long rounds = (tiles + slots - 1) / slots;
    const double filled = ((double)p.M * (double)p.N) / ((double)(tm * bm) * (double)(tn * bn_out));  // ragged edge tiles
    return filled * (double)tiles / (double)(rounds * slots);
  };
  GemmParams q = p;
  q.bn_out = 0;  // block-sized tiles always cover their full width
  if (0.83 * occupancy(128, 128, 2LL * n_cu) > occupancy(256, 256, n_cu)) return launch_block_sized<CfgMid>(q, layout, epilogue, s);
  return launch_block_sized<CfgBig>(q, layout, epilogue, s);
}

}  // namespace caat
