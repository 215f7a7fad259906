// Grouped bf16 shard GEMM for gfx950 (CDNA4): MFMA 32x32x16 bf16, fp32 accumulation, LDS-staged tiles.
//
// One launch covers all T emulated tensor-parallel ranks (group index g).  It implements the two
// contractions of Eq. A3 (column-parallel X_m A_m with the activation fused, row-parallel Y_m B_m with the
// private-column part of the partial channel-reduce + residual fused) and their data / weight gradients.
//
// Tiling: a workgroup owns a BM x BN tile of C and walks K in steps of BK = 64.  Both operand tiles live in
// LDS as [rows][64] bf16, K-contiguous, 16-byte chunks XOR-swizzled so that the MFMA fragment reads
// (32 consecutive rows x one chunk) and the tile writes are bank-conflict free.  Operands whose contiguous
// memory dimension is NOT K (layouts NN / TN) are transposed in registers (8x8 blocks of 16-bit values) on
// their way from global memory to LDS, so the MFMA inner loop is the same for the three layouts.
// Global loads of tile kt+1 are issued before the MFMAs of tile kt (register prefetch), LDS is double
// buffered: one barrier per K step.
//
// The accumulator is computed transposed (operands swapped in the MFMA) so that each lane ends up with 4
// consecutive columns of one row of C: the epilogue works on 8-byte bf16x4 vectors.
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

static constexpr int BK = 64;  // K step: 8 chunks of 8 bf16 per tile row

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wave
  static constexpr int STAGE_CHUNKS = (BM + BN) * 8;  // uint4 per LDS stage
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(TN % 2 == 0, "SwiGLU pairing needs an even number of N tiles per wave");
};

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_index(int row, int chunk) { return row * 8 + (chunk ^ swz(row)); }

// ---- K-contiguous source: tile rows x 64 k, thread moves 16-byte chunks straight through registers
template <int ROWS, int THREADS>
struct DirectLoader {
  static constexpr int NCH = (ROWS * 8 + THREADS - 1) / THREADS;
  const bf16_t* ptr[NCH];  // row base + kc*8, nullptr if the row is outside the matrix (or the chunk is idle)
  uint4 reg[NCH];
  int kc;

  // rowmap(rr) gives the source row of tile row rr, or -1 if it does not exist
  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* base, long long ld, RowMap rowmap) {
    const int tid = threadIdx.x;
    kc = tid & 7;
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      const int rr = it * (THREADS / 8) + (tid >> 3);
      long long srow = (rr < ROWS) ? rowmap(rr) : -1;
      ptr[it] = (srow >= 0) ? base + srow * ld + kc * 8 : nullptr;
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const bool kin = (k0 + kc * 8) < K;
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (kin && ptr[it] != nullptr) v = *reinterpret_cast<const uint4*>(ptr[it] + k0);
      reg[it] = v;
    }
  }
  __device__ __forceinline__ void store(uint4* tile) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      const int rr = it * (THREADS / 8) + (tid >> 3);
      if (rr < ROWS) tile[lds_index(rr, kc)] = reg[it];
    }
  }
};

// ---- row-contiguous source ([K][rows]): thread loads an 8(k) x 8(rows) block, transposes it in registers
template <int ROWS, int THREADS>
struct TransLoader {
  static constexpr int NBLK = ROWS;  // (ROWS/8) row blocks x 8 k groups
  static constexpr int NB = (NBLK + THREADS - 1) / THREADS;
  const bf16_t* ptr[NB];  // base + src_row0 (column of the source), nullptr if outside / idle
  long long ld;
  uint4 reg[NB][8];

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* base, long long ld_, RowMap rowmap) {
    ld = ld_;
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int blk = it * THREADS + tid;
      const int rb = blk % (ROWS / 8);
      long long srow = (blk < NBLK) ? rowmap(rb * 8) : -1;  // 8 consecutive rows share validity (dims % 8 == 0)
      ptr[it] = (srow >= 0) ? base + srow : nullptr;
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int blk = it * THREADS + tid;
      const int kg = blk / (ROWS / 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + kg * 8 + j;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (ptr[it] != nullptr && k < K) v = *reinterpret_cast<const uint4*>(ptr[it] + (long long)k * ld);
        reg[it][j] = v;
      }
    }
  }
  __device__ __forceinline__ void store(uint4* tile) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int blk = it * THREADS + tid;
      if (blk >= NBLK) continue;
      const int rb = blk % (ROWS / 8);
      const int kg = blk / (ROWS / 8);
      const unsigned* in = reinterpret_cast<const unsigned*>(&reg[it][0]);  // in[j*4 + q]: k=j, rows 2q (lo), 2q+1 (hi)
#pragma unroll
      for (int i = 0; i < 8; ++i) {  // output row rb*8+i gets k = 0..7
        unsigned o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const unsigned a = in[(2 * d) * 4 + (i >> 1)];
          const unsigned b = in[(2 * d + 1) * 4 + (i >> 1)];
          o[d] = (i & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
        tile[lds_index(rb * 8 + i, kg)] = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  }
};

template <bool TRANS, int ROWS, int THREADS>
struct LoaderSel { typedef DirectLoader<ROWS, THREADS> type; };
template <int ROWS, int THREADS>
struct LoaderSel<true, ROWS, THREADS> { typedef TransLoader<ROWS, THREADS> type; };

__device__ __forceinline__ void store4(bf16_t* dst, float v0, float v1, float v2, float v3) {
  uint2 w;
  w.x = pack2bf(v0, v1);
  w.y = pack2bf(v2, v3);
  *reinterpret_cast<uint2*>(dst) = w;
}

template <class CFG, bool AT, bool BT, int EPI>
__global__ __launch_bounds__(CFG::THREADS) void gemm_kernel(const GemmParams p) {
  constexpr int BM = CFG::BM, BN = CFG::BN, THREADS = CFG::THREADS;
  constexpr int TM = CFG::TM, TN = CFG::TN, WTM = CFG::WTM, WTN = CFG::WTN;
  constexpr bool SWI = (EPI == EPI_SWIGLU_FWD);
  constexpr int BN_OUT = SWI ? BN / 2 : BN;  // output columns covered by one tile

  __shared__ uint4 smem[2 * CFG::STAGE_CHUNKS];

  // ---- which tile: spread consecutive tile ids over the 8 XCDs' L2s, then a grouped (8 tile rows) order
  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = (p.N + BN_OUT - 1) / BN_OUT;
  const int tiles = tiles_m * tiles_n;
  const int total = tiles * p.G;
  int pid;
  {
    const int bid = blockIdx.x;
    const int q = total >> 3, rem = total & 7, x = bid & 7;
    pid = x * q + (x < rem ? x : rem) + (bid >> 3);
  }
  const int g = pid / tiles;
  const int t = pid - g * tiles;
  int tm, tn;
  {
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int grp = t / width;
    const int first = grp * GROUP;
    const int gsize = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
    const int r = t - grp * width;
    tm = first + r % gsize;
    tn = r / gsize;
  }
  const int m0 = tm * BM;
  const int n0 = tn * BN_OUT;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / CFG::WN;
  const int wn = wave - wm * CFG::WN;

  const bf16_t* ag = p.a + (long long)g * p.stride_a;
  const bf16_t* bg = p.b + (long long)g * p.stride_b;

  typename LoaderSel<AT, BM, THREADS>::type la;
  typename LoaderSel<BT, BN, THREADS>::type lb;
  {
    const int M = p.M;
    la.init(ag, p.lda, [=](int rr) -> long long { return (m0 + rr < M) ? (long long)(m0 + rr) : -1; });
    if constexpr (SWI) {
      const int half = p.half;
      lb.init(bg, p.ldb, [=](int rr) -> long long {
        const int w = rr / WTN, rw = rr - w * WTN;
        const int j = rw >> 5, c = rw & 31;
        const int col = n0 + (w * (TN / 2) + (j >> 1)) * 32 + c;
        if (col >= half) return -1;
        return (long long)col + ((j & 1) ? half : 0);
      });
    } else {
      const int N = p.N;
      lb.init(bg, p.ldb, [=](int rr) -> long long { return (n0 + rr < N) ? (long long)(n0 + rr) : -1; });
    }
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int K = p.K;
  const int nk = (K + BK - 1) / BK;

  la.load(0, K);
  lb.load(0, K);
  la.store(smem);
  lb.store(smem + BM * 8);
  __syncthreads();

  const int frow = lane & 31;  // fragment row within a 32-row MFMA tile
  const int fk = lane >> 5;    // which 8-wide half of a 16-wide k step

  for (int kt = 0; kt < nk; ++kt) {
    const uint4* As = smem + (kt & 1) * CFG::STAGE_CHUNKS;
    const uint4* Bs = As + BM * 8;
    uint4* An = smem + ((kt + 1) & 1) * CFG::STAGE_CHUNKS;
    uint4* Bn = An + BM * 8;
    const bool more = (kt + 1) < nk;
    if (more) {
      la.load((kt + 1) * BK, K);
      lb.load((kt + 1) * BK, K);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * WTM + i * 32 + frow;
        af[i] = __builtin_bit_cast(bf16x8_t, As[lds_index(row, ks * 2 + fk)]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * WTN + j * 32 + frow;
        bfr[j] = __builtin_bit_cast(bf16x8_t, Bs[lds_index(row, ks * 2 + fk)]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // operands swapped: the accumulator holds C^T, i.e. lane = row of C, registers = columns of C
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    if (more) {
      la.store(An);
      lb.store(Bn);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds C[row = m + lane%32][col = n + 8*q + 4*(lane/32) + 0..3] in acc[..][4q..4q+3]
  const long long M = p.M;
  bf16_t* cg = p.c + (long long)g * p.stride_c;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const long long row = (long long)m0 + wm * WTM + i * 32 + frow;
    if (row >= M) continue;
    if constexpr (SWI) {
      bf16_t* yg = p.c2 + (long long)g * p.stride_c2;
#pragma unroll
      for (int jj = 0; jj < TN / 2; ++jj) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = n0 + (wn * (TN / 2) + jj) * 32 + q * 8 + fk * 4;
          if (col >= p.half) continue;
          float gt[4], up[4], y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            gt[e] = acc[i][2 * jj][q * 4 + e];
            up[e] = acc[i][2 * jj + 1][q * 4 + e];
            y[e] = gt[e] * sigmoid_f(gt[e]) * up[e];
          }
          store4(cg + row * p.ldc + col, gt[0], gt[1], gt[2], gt[3]);
          store4(cg + row * p.ldc + p.half + col, up[0], up[1], up[2], up[3]);
          store4(yg + row * p.ldc2 + col, y[0], y[1], y[2], y[3]);
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = n0 + wn * WTN + j * 32 + q * 8 + fk * 4;
          if (col >= p.N) continue;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
          if constexpr (EPI == EPI_PLAIN) {
            store4(cg + row * p.ldc + col, v[0], v[1], v[2], v[3]);
          } else if constexpr (EPI == EPI_GELU_FWD) {
            bf16_t* yg = p.c2 + (long long)g * p.stride_c2;
            store4(cg + row * p.ldc + col, v[0], v[1], v[2], v[3]);
            store4(yg + row * p.ldc2 + col, gelu_f(v[0]), gelu_f(v[1]), gelu_f(v[2]), gelu_f(v[3]));
          } else if constexpr (EPI == EPI_ROWPAR) {
            // Eq. A3 case split, private side: columns >= hs are final here (scale, + residual);
            // columns < hs are stored as this rank's partial sum for the reduce kernel.
            if (col + 3 >= p.hs) {
              const bf16_t* rg = p.aux + (long long)g * p.stride_aux + row * p.ldaux + col;
              const uint2 rw = *reinterpret_cast<const uint2*>(rg);
              const float r0 = lo_bf(rw.x), r1 = hi_bf(rw.x), r2 = lo_bf(rw.y), r3 = hi_bf(rw.y);
              if (col + 0 >= p.hs) v[0] = p.scale * v[0] + r0;
              if (col + 1 >= p.hs) v[1] = p.scale * v[1] + r1;
              if (col + 2 >= p.hs) v[2] = p.scale * v[2] + r2;
              if (col + 3 >= p.hs) v[3] = p.scale * v[3] + r3;
            }
            store4(cg + row * p.ldc + col, v[0], v[1], v[2], v[3]);
          } else if constexpr (EPI == EPI_GELU_BWD) {
            const bf16_t* pg = p.aux + (long long)g * p.stride_aux + row * p.ldaux + col;
            const uint2 pw = *reinterpret_cast<const uint2*>(pg);
            store4(cg + row * p.ldc + col, v[0] * gelu_grad_f(lo_bf(pw.x)), v[1] * gelu_grad_f(hi_bf(pw.x)),
                   v[2] * gelu_grad_f(lo_bf(pw.y)), v[3] * gelu_grad_f(hi_bf(pw.y)));
          } else if constexpr (EPI == EPI_SWIGLU_BWD) {
            const bf16_t* pg = p.aux + (long long)g * p.stride_aux + row * p.ldaux + col;
            const uint2 gw = *reinterpret_cast<const uint2*>(pg);
            const uint2 uw = *reinterpret_cast<const uint2*>(pg + p.half);
            const float gt[4] = {lo_bf(gw.x), hi_bf(gw.x), lo_bf(gw.y), hi_bf(gw.y)};
            const float up[4] = {lo_bf(uw.x), hi_bf(uw.x), lo_bf(uw.y), hi_bf(uw.y)};
            float dg[4], du[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float s = sigmoid_f(gt[e]);
              dg[e] = v[e] * up[e] * s * (1.0f + gt[e] * (1.0f - s));
              du[e] = v[e] * gt[e] * s;
            }
            store4(cg + row * p.ldc + col, dg[0], dg[1], dg[2], dg[3]);
            store4(cg + row * p.ldc + p.half + col, du[0], du[1], du[2], du[3]);
          }
        }
      }
    }
  }
}

template <class CFG, bool AT, bool BT, int EPI>
static hipError_t launch_one(const GemmParams& p, hipStream_t s) {
  constexpr int BN_OUT = (EPI == EPI_SWIGLU_FWD) ? CFG::BN / 2 : CFG::BN;
  const long long tiles_m = (p.M + CFG::BM - 1) / CFG::BM;
  const long long tiles_n = (p.N + BN_OUT - 1) / BN_OUT;
  const long long total = tiles_m * tiles_n * p.G;
  if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gemm_kernel<CFG, AT, BT, EPI>), dim3((unsigned)total), dim3(CFG::THREADS), 0, s, p);
  return hipGetLastError();
}

typedef TileCfg<256, 256, 2, 2> CfgBig;

hipError_t launch_gemm(const GemmParams& p, int layout, int epilogue, hipStream_t s) {
  typedef CfgBig C;
  switch (layout) {
    case 0:  // NT
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<C, false, false, EPI_PLAIN>(p, s);
        case EPI_GELU_FWD: return launch_one<C, false, false, EPI_GELU_FWD>(p, s);
        case EPI_SWIGLU_FWD: return launch_one<C, false, false, EPI_SWIGLU_FWD>(p, s);
        case EPI_ROWPAR: return launch_one<C, false, false, EPI_ROWPAR>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 1:  // NN
      switch (epilogue) {
        case EPI_PLAIN: return launch_one<C, false, true, EPI_PLAIN>(p, s);
        case EPI_GELU_BWD: return launch_one<C, false, true, EPI_GELU_BWD>(p, s);
        case EPI_SWIGLU_BWD: return launch_one<C, false, true, EPI_SWIGLU_BWD>(p, s);
        default: return hipErrorInvalidValue;
      }
    case 2:  // TN
      if (epilogue == EPI_PLAIN) return launch_one<C, true, true, EPI_PLAIN>(p, s);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace caat
