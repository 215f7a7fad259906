// Grouped bf16 shard GEMM kernel template for gfx950 (CDNA4): MFMA 32x32x16 bf16, fp32 accumulation.
//
// One launch covers all T emulated tensor-parallel ranks (group index g).  It implements the two contractions
// of Eq. A3 (column-parallel X_m A_m with the activation fused, row-parallel Y_m B_m with the private-column
// half of the partial channel-reduce + residual fused) and their data / weight gradients.
//
// Tiling: a workgroup owns a BM x BN tile of C and walks K in steps of BK = 64.  Both operand tiles live in
// LDS as [rows][64] bf16, K-contiguous, 16-byte chunks XOR-swizzled so that MFMA fragment reads (32
// consecutive rows x one chunk) and tile writes are bank-conflict free.  Operands whose contiguous memory
// dimension is NOT K (layouts NN / TN) are transposed in registers (8x8 blocks of 16-bit values) on their way
// from global memory to LDS, so the MFMA inner loop is the same for the three layouts.
//
// Global memory is read with buffer loads: rows / k positions outside the matrix get an out-of-range offset
// and come back as zeros, so the main loop has no branches.  Tile kt+1 is fetched into registers while the
// MFMAs of tile kt run; LDS is double buffered (one barrier per K step); MFMA fragments are double buffered
// in registers across the four 16-wide k sub-steps.
//
// The accumulator is computed transposed (operands swapped in the MFMA) so that each lane ends up with 4
// consecutive columns of one row of C: the epilogue works on 8-byte bf16x4 vectors.
#pragma once
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

static constexpr int BK = 64;                 // K step: 8 chunks of 8 bf16 per tile row
static constexpr unsigned OOB = 0x80000000u;  // buffer offset that is always out of range -> load returns 0

template <int BM_, int BN_, int WM_, int WN_, int SCHED_ = 2>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int SCHED = SCHED_;  // 0: compiler's order, 1: phase fences, 2: fences + MFMA/LDS/VMEM interleave
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wave
  static constexpr int STAGE_CHUNKS = (BM + BN) * 8;  // uint4 per LDS stage
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "tile chunks must divide over the threads");
};

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_index(int row, int chunk) { return row * 8 + (chunk ^ swz(row)); }

// raw buffer descriptor over [p, p + 2 GiB): offsets >= 0x80000000 are out of range and read as zero
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)0x80000000, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned voff) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- K-contiguous source: tile rows x 64 k; a thread moves 16-byte chunks straight through registers.
// `origin` points at the tile's first row (uniform); rowmap(rr) gives the row of tile row rr RELATIVE to the
// origin, or -1 if that row does not exist.
template <int ROWS, int THREADS>
struct DirectLoader {
  static constexpr int NCH = ROWS * 8 / THREADS;
  const bf16_t* origin;
  unsigned voff[NCH];  // byte offset of (row, kc) from origin, OOB for missing rows
  uint4 reg[NCH];
  int kc;

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* origin_, long long ld, RowMap rowmap) {
    origin = origin_;
    const int tid = threadIdx.x;
    kc = tid & 7;
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      const int rr = it * (THREADS / 8) + (tid >> 3);
      const long long r = rowmap(rr);
      voff[it] = (r >= 0) ? (unsigned)((r * ld + kc * 8) * 2) : OOB;
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(origin + k0);
    const bool kin = (k0 + kc * 8) < K;
#pragma unroll
    for (int it = 0; it < NCH; ++it) reg[it] = buf_load16(rs, kin ? voff[it] : OOB);
  }
  __device__ __forceinline__ void store(uint4* tile) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      const int rr = it * (THREADS / 8) + (tid >> 3);
      tile[lds_index(rr, kc)] = reg[it];
    }
  }
};

// ---- row-contiguous source ([K][rows]): thread loads an 8(k) x 8(rows) block, transposes it in registers.
// `origin` points at (k = 0, first row of the tile); rowmap as above (8 consecutive rows share validity).
template <int ROWS, int THREADS>
struct TransLoader {
  static constexpr int NBLK = ROWS;  // (ROWS/8) row blocks x 8 k groups
  static constexpr int NB = (NBLK + THREADS - 1) / THREADS;
  const bf16_t* origin;
  long long ld;
  unsigned voff[NB];  // byte offset of (k = kg*8, row block) from origin + k0*ld, OOB if missing / idle
  unsigned ld2;
  uint4 reg[NB][8];

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* origin_, long long ld_, RowMap rowmap) {
    origin = origin_;
    ld = ld_;
    ld2 = (unsigned)(ld_ * 2);
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int blk = it * THREADS + tid;
      const int rb = blk % (ROWS / 8);
      const int kg = blk / (ROWS / 8);
      const long long r = (blk < NBLK) ? rowmap(rb * 8) : -1;
      voff[it] = (r >= 0) ? (unsigned)(((long long)kg * 8 * ld_ + r) * 2) : OOB;
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(origin + (long long)k0 * ld);
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int kg = (it * THREADS + tid) / (ROWS / 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool in = (voff[it] != OOB) && (k0 + kg * 8 + j < K);
        reg[it][j] = buf_load16(rs, in ? voff[it] + (unsigned)j * ld2 : OOB);
      }
    }
  }
  __device__ __forceinline__ void store(uint4* tile) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int blk = it * THREADS + tid;
      if (NBLK % THREADS != 0 && blk >= NBLK) continue;
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

template <int TM, int TN>
struct Frags {
  bf16x8_t a[TM], b[TN];
};

template <class CFG, bool AT, bool BT, int EPI>
__global__ __launch_bounds__(CFG::THREADS) void gemm_kernel(const GemmParams p) {
  constexpr int BM = CFG::BM, BN = CFG::BN, THREADS = CFG::THREADS;
  constexpr int TM = CFG::TM, TN = CFG::TN, WTM = CFG::WTM, WTN = CFG::WTN;
  constexpr bool SWI = (EPI == EPI_SWIGLU_FWD);
  constexpr int BN_OUT = SWI ? BN / 2 : BN;  // output columns covered by one tile
  static_assert(!SWI || TN % 2 == 0, "SwiGLU pairing needs an even number of N tiles per wave");

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
    const int mrem = p.M - m0;
    la.init(AT ? ag + m0 : ag + (long long)m0 * p.lda, p.lda,
            [=](int rr) -> long long { return (rr < mrem) ? (long long)rr : -1; });
    if constexpr (SWI) {
      const int half = p.half;
      lb.init(bg + (long long)n0 * p.ldb, p.ldb, [=](int rr) -> long long {
        const int w = rr / WTN, rw = rr - w * WTN;
        const int j = rw >> 5, c = rw & 31;
        const int col = (w * (TN / 2) + (j >> 1)) * 32 + c;  // output column relative to n0
        if (n0 + col >= half) return -1;
        return (long long)col + ((j & 1) ? half : 0);
      });
    } else {
      const int nrem = p.N - n0;
      lb.init(BT ? bg + n0 : bg + (long long)n0 * p.ldb, p.ldb,
              [=](int rr) -> long long { return (rr < nrem) ? (long long)rr : -1; });
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
  const int frow = lane & 31;  // fragment row within a 32-row MFMA tile
  const int fk = lane >> 5;    // which 8-wide half of a 16-wide k step

  auto load_frags = [&](const uint4* As, const uint4* Bs, int ks, Frags<TM, TN>& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      f.a[i] = __builtin_bit_cast(bf16x8_t, As[lds_index(wm * WTM + i * 32 + frow, ks * 2 + fk)]);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      f.b[j] = __builtin_bit_cast(bf16x8_t, Bs[lds_index(wn * WTN + j * 32 + frow, ks * 2 + fk)]);
  };
  auto mfma_all = [&](const Frags<TM, TN>& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        // operands swapped: the accumulator holds C^T, i.e. lane = row of C, registers = columns of C
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
  };

  la.load(0, K);
  lb.load(0, K);
  la.store(smem);
  lb.store(smem + BM * 8);
  __syncthreads();

  Frags<TM, TN> f0, f1;
  load_frags(smem, smem + BM * 8, 0, f0);

  // Instruction-order control.  fence(): nothing may be moved across.  interleave<n_mfma, n_other>(mask):
  // ask for n_other instructions of class `mask` after every MFMA (classes: 0x100 LDS read, 0x200 LDS write,
  // 0x020 VMEM read), so that the next sub-step's fragment reads, the next tile's global loads and its LDS
  // writes are spread between the MFMAs of the current sub-step instead of bunching up in front of a wait.
  constexpr int SCHED = CFG::SCHED;
  constexpr int NMFMA = TM * TN;
  constexpr int NFRAG = TM + TN;
  auto fence = [&]() {
    if constexpr (SCHED >= 1) __builtin_amdgcn_sched_barrier(0);
  };

  for (int kt = 0; kt < nk; ++kt) {
    const uint4* As = smem + (kt & 1) * CFG::STAGE_CHUNKS;
    const uint4* Bs = As + BM * 8;
    uint4* An = smem + ((kt + 1) & 1) * CFG::STAGE_CHUNKS;
    uint4* Bn = An + BM * 8;
    // tile kt+1 (past the end of K: every offset is out of range, zeros come back, nobody uses them)
    la.load((kt + 1) * BK, K);
    lb.load((kt + 1) * BK, K);
    fence();
    load_frags(As, Bs, 1, f1);
    mfma_all(f0);
    if constexpr (SCHED >= 2) {
#pragma unroll
      for (int i = 0; i < NFRAG; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
    }
    fence();
    load_frags(As, Bs, 2, f0);
    mfma_all(f1);
    if constexpr (SCHED >= 2) {
#pragma unroll
      for (int i = 0; i < NFRAG; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
    }
    fence();
    load_frags(As, Bs, 3, f1);
    mfma_all(f0);
    if constexpr (SCHED >= 2) {
#pragma unroll
      for (int i = 0; i < NFRAG; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
    }
    fence();
    la.store(An);
    lb.store(Bn);
    __syncthreads();
    fence();
    load_frags(An, Bn, 0, f0);
    mfma_all(f1);
    if constexpr (SCHED >= 2) {
#pragma unroll
      for (int i = 0; i < NFRAG; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
    }
    fence();
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

}  // namespace caat
