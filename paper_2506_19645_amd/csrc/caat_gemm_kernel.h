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
// consecutive columns of one row of C; the epilogue stages the bf16 tile through LDS and stores whole rows.
#pragma once
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

static constexpr int BK = 64;                 // K step: 8 chunks of 8 bf16 per tile row
static constexpr unsigned OOB = 0x80000000u;  // buffer offset that is always out of range -> load returns 0

template <int BM_, int BN_, int WM_, int WN_, int SCHED_ = 2, bool LDSD_ = false>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int SCHED = SCHED_;  // 0: compiler's order, 1: phase fences, 2: fences + MFMA/LDS/VMEM interleave
  static constexpr bool LDSD = LDSD_;   // K-contiguous operands go global -> LDS directly (no register staging)
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

// ---- K-contiguous source, global -> LDS without passing through registers (buffer_load ... lds): one wave
// instruction fills 8 consecutive tile rows (64 lanes x 16 B = 1 KiB of LDS, lane order); the XOR swizzle is
// applied on the global side (lane L fetches the chunk that belongs at LDS position L).
template <int ROWS, int THREADS>
struct DirectLdsLoader {
  static constexpr int NWAVES = THREADS / 64;
  static constexpr int NI = ROWS / 8 / NWAVES;
  static constexpr int N_VMEM = NI, N_DSWRITE = 0;
  const bf16_t* origin;
  unsigned voff[NI];
  int wave, lane;

  __device__ __forceinline__ int kc_of(int it) const { return (lane & 7) ^ (((lane >> 3) ^ (it * NWAVES + wave)) & 7); }

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* origin_, long long ld, RowMap rowmap) {
    origin = origin_;
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      const int row = (it * NWAVES + wave) * 8 + (lane >> 3);
      const long long r = rowmap(row);
      voff[it] = (r >= 0) ? (unsigned)((r * ld + kc_of(it) * 8) * 2) : OOB;
    }
  }
  __device__ __forceinline__ void load(int k0, int K, uint4* tile) {
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(origin + k0);
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      const bool kin = (k0 + kc_of(it) * 8) < K;
      uint4* dst = tile + (it * NWAVES + wave) * 64;  // wave-uniform
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)dst, 16,
                                               (int)(kin ? voff[it] : OOB), 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(uint4*) const {}
};

template <int ROWS, int THREADS>
struct DirectRegLoader : DirectLoader<ROWS, THREADS> {
  static constexpr int N_VMEM = DirectLoader<ROWS, THREADS>::NCH, N_DSWRITE = DirectLoader<ROWS, THREADS>::NCH;
  __device__ __forceinline__ void load(int k0, int K, uint4*) { DirectLoader<ROWS, THREADS>::load(k0, K); }
};
template <int ROWS, int THREADS>
struct TransRegLoader : TransLoader<ROWS, THREADS> {
  static constexpr int N_VMEM = 8 * TransLoader<ROWS, THREADS>::NB, N_DSWRITE = 8 * TransLoader<ROWS, THREADS>::NB;
  __device__ __forceinline__ void load(int k0, int K, uint4*) { TransLoader<ROWS, THREADS>::load(k0, K); }
};

template <bool TRANS, bool LDSD, int ROWS, int THREADS>
struct LoaderSel { typedef DirectRegLoader<ROWS, THREADS> type; };
template <int ROWS, int THREADS>
struct LoaderSel<false, true, ROWS, THREADS> { typedef DirectLdsLoader<ROWS, THREADS> type; };
template <bool LDSD, int ROWS, int THREADS>
struct LoaderSel<true, LDSD, ROWS, THREADS> { typedef TransRegLoader<ROWS, THREADS> type; };

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

// Instruction-order request for one k sub-step (between two scheduling fences): after every MFMA place this
// MFMA's share of the NR LDS reads (front-loaded: one per MFMA), NV global loads and NW LDS writes.
template <int I, int NM, int NR, int NV, int NW>
struct Pipe {
  static __device__ __forceinline__ void run() {
    if constexpr (I < NM) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      constexpr int r = (NR <= NM) ? (I < NR ? 1 : 0) : ((NR * (I + 1)) / NM - (NR * I) / NM);
      constexpr int v = (NV * (I + 1)) / NM - (NV * I) / NM;
      constexpr int w = (NW * (I + 1)) / NM - (NW * I) / NM;
      if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
      if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
      if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
      Pipe<I + 1, NM, NR, NV, NW>::run();
    }
  }
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

  typedef typename LoaderSel<AT, CFG::LDSD, BM, THREADS>::type LoaderA;
  typedef typename LoaderSel<BT, CFG::LDSD, BN, THREADS>::type LoaderB;
  LoaderA la;
  LoaderB lb;
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
  // LDS-direct loads are counted by vmcnt: they must have landed before the barrier that publishes the tile
  auto wait_lds_dma = [&]() {
    if constexpr (CFG::LDSD && (!AT || !BT)) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  la.load(0, K, smem);
  lb.load(0, K, smem + BM * 8);
  la.store(smem);
  lb.store(smem + BM * 8);
  wait_lds_dma();
  __syncthreads();

  Frags<TM, TN> f0, f1;
  load_frags(smem, smem + BM * 8, 0, f0);

  // Instruction-order control: fence() = nothing moves across; Pipe<> spreads the next sub-step's fragment
  // reads, the next tile's global loads and its LDS writes between the MFMAs of the current sub-step.
  constexpr int SCHED = CFG::SCHED;
  constexpr int NM = TM * TN, NR = TM + TN;
  constexpr int NV = LoaderA::N_VMEM + LoaderB::N_VMEM, NW = LoaderA::N_DSWRITE + LoaderB::N_DSWRITE;
  auto fence = [&]() {
    if constexpr (SCHED >= 1) __builtin_amdgcn_sched_barrier(0);
  };

  for (int kt = 0; kt < nk; ++kt) {
    const uint4* As = smem + (kt & 1) * CFG::STAGE_CHUNKS;
    const uint4* Bs = As + BM * 8;
    uint4* An = smem + ((kt + 1) & 1) * CFG::STAGE_CHUNKS;
    uint4* Bn = An + BM * 8;
    // k sub-step 0, and the fetch of tile kt+1 (past the end of K every offset is out of range: zeros come
    // back and nobody uses them, so the loop needs no branch)
    la.load((kt + 1) * BK, K, An);
    lb.load((kt + 1) * BK, K, Bn);
    if constexpr (SCHED == 1) fence();
    load_frags(As, Bs, 1, f1);
    mfma_all(f0);
    if constexpr (SCHED >= 2) Pipe<0, NM, NR, NV, 0>::run();
    fence();
    load_frags(As, Bs, 2, f0);
    mfma_all(f1);
    if constexpr (SCHED >= 2) Pipe<0, NM, NR, 0, 0>::run();
    fence();
    load_frags(As, Bs, 3, f1);
    mfma_all(f0);
    if constexpr (SCHED == 1) fence();
    la.store(An);
    lb.store(Bn);
    if constexpr (SCHED >= 2) Pipe<0, NM, NR, 0, NW>::run();
    fence();
    wait_lds_dma();
    __syncthreads();
    fence();
    load_frags(An, Bn, 0, f0);
    mfma_all(f1);
    if constexpr (SCHED >= 2) Pipe<0, NM, NR, 0, 0>::run();
    fence();
  }

  // ---- epilogue.  Each lane holds C[row = lane%32][col = 8*q + 4*(lane/32) + 0..3] of every 32x32 tile in
  // acc[..][4q..4q+3].  Writing that to global memory directly would scatter 8-byte pieces over 32 rows per
  // instruction, so the tile is first rounded to bf16 and parked in LDS (the operand buffers are free now) as
  // [BM][BN/8] 16-byte chunks, chunk index XOR-swizzled by the row (conflict-free for the column-of-rows
  // writes and for the row-wise reads); then every wave instruction stores whole rows: 16 bytes per lane,
  // consecutive lanes = consecutive columns.  The fused element-wise work (activation, its derivative, the
  // private half of the partial channel-reduce + residual) is done in this second phase on 8 values per lane.
  constexpr int CH = BN / 8;  // chunks per staged row
  __syncthreads();            // every wave is done reading the operand tiles
  {
    char* stage = reinterpret_cast<char*>(smem);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = wm * WTM + i * 32 + frow;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = (wn * WTN + j * 32) / 8 + q;
          uint2 w;
          w.x = pack2bf(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1]);
          w.y = pack2bf(acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
          *reinterpret_cast<uint2*>(stage + ((row * CH + (c ^ (row & (CH - 1)))) * 16 + fk * 8)) = w;
        }
      }
    }
  }
  __syncthreads();

  const int M = p.M;
  bf16_t* cg = p.c + (long long)g * p.stride_c;
  auto staged = [&](int row, int c) -> uint4 { return smem[row * CH + (c ^ (row & (CH - 1)))]; };
  auto unpack = [](const uint4& v, float* f) {
    f[0] = lo_bf(v.x); f[1] = hi_bf(v.x); f[2] = lo_bf(v.y); f[3] = hi_bf(v.y);
    f[4] = lo_bf(v.z); f[5] = hi_bf(v.z); f[6] = lo_bf(v.w); f[7] = hi_bf(v.w);
  };
  auto pack = [](const float* f) -> uint4 {
    return make_uint4(pack2bf(f[0], f[1]), pack2bf(f[2], f[3]), pack2bf(f[4], f[5]), pack2bf(f[6], f[7]));
  };
  constexpr int OCH = BN_OUT / 8;  // output chunks per row
  constexpr int STEPS = BM * OCH / THREADS;
  static_assert((BM * OCH) % THREADS == 0, "epilogue chunks must divide over the threads");
#pragma unroll 4
  for (int st = 0; st < STEPS; ++st) {
    const int idx = st * THREADS + tid;
    const int row = idx / OCH, oc = idx - row * OCH;
    const long long grow = (long long)m0 + row;
    const int gcol = n0 + oc * 8;
    if (grow >= M || gcol >= p.N) continue;
    if constexpr (SWI) {
      // staged columns: per wave [gate 32 | up 32] pairs; output column -> its gate chunk, up chunk = +4
      const int ocol = oc * 8;
      const int w = ocol / (WTN / 2), rw = ocol - w * (WTN / 2);
      const int gc = (w * WTN + (rw >> 5) * 64 + (rw & 31)) / 8;
      float gt[8], up[8], y[8];
      unpack(staged(row, gc), gt);
      unpack(staged(row, gc + 4), up);
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = gt[e] * sigmoid_f(gt[e]) * up[e];
      bf16_t* yg = p.c2 + (long long)g * p.stride_c2;
      *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = staged(row, gc);
      *reinterpret_cast<uint4*>(cg + grow * p.ldc + p.half + gcol) = staged(row, gc + 4);
      *reinterpret_cast<uint4*>(yg + grow * p.ldc2 + gcol) = pack(y);
    } else {
      const uint4 raw = staged(row, oc);
      if constexpr (EPI == EPI_PLAIN) {
        *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = raw;
      } else if constexpr (EPI == EPI_GELU_FWD) {
        // the activation is taken of the bf16-rounded pre-activation, the value the backward pass sees too
        float v[8], y[8];
        unpack(raw, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = gelu_f(v[e]);
        bf16_t* yg = p.c2 + (long long)g * p.stride_c2;
        *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = raw;
        *reinterpret_cast<uint4*>(yg + grow * p.ldc2 + gcol) = pack(y);
      } else if constexpr (EPI == EPI_ROWPAR) {
        // Eq. A3 case split, private side: columns >= hs are final here (scale, + residual); columns < hs are
        // stored as this rank's partial sum for the reduce kernel.  NOTE: the private value is scaled from the
        // bf16-rounded partial.
        if (gcol + 7 >= p.hs) {
          float v[8], r[8];
          unpack(raw, v);
          unpack(*reinterpret_cast<const uint4*>(p.aux + (long long)g * p.stride_aux + grow * p.ldaux + gcol), r);
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (gcol + e >= p.hs) v[e] = p.scale * v[e] + r[e];
          *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = pack(v);
        } else {
          *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = raw;
        }
      } else if constexpr (EPI == EPI_GELU_BWD) {
        float v[8], pr[8];
        unpack(raw, v);
        unpack(*reinterpret_cast<const uint4*>(p.aux + (long long)g * p.stride_aux + grow * p.ldaux + gcol), pr);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(pr[e]);
        *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = pack(v);
      } else if constexpr (EPI == EPI_SWIGLU_BWD) {
        const bf16_t* pg = p.aux + (long long)g * p.stride_aux + grow * p.ldaux + gcol;
        float v[8], gt[8], up[8], dg[8], du[8];
        unpack(raw, v);
        unpack(*reinterpret_cast<const uint4*>(pg), gt);
        unpack(*reinterpret_cast<const uint4*>(pg + p.half), up);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float sg = sigmoid_f(gt[e]);
          dg[e] = v[e] * up[e] * sg * (1.0f + gt[e] * (1.0f - sg));
          du[e] = v[e] * gt[e] * sg;
        }
        *reinterpret_cast<uint4*>(cg + grow * p.ldc + gcol) = pack(dg);
        *reinterpret_cast<uint4*>(cg + grow * p.ldc + p.half + gcol) = pack(du);
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
