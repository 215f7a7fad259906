// Grouped bf16 shard GEMM kernel template for gfx950 (CDNA4): MFMA 32x32x16 bf16, fp32 accumulation.
//
// One launch covers all T emulated tensor-parallel ranks (group index g).  It implements the two contractions
// of Eq. A3 (column-parallel X_m A_m with the activation fused, row-parallel Y_m B_m with the private-column
// half of the partial channel-reduce + residual fused) and their data / weight gradients.
//
// Tiling: a workgroup owns a BM x BN tile of C and walks K in stages of BKS (64 in every tile shape in use).  NSTAGE
// stages of both operand tiles live in LDS and every operand goes global -> LDS directly (buffer_load ... lds, no
// register staging), NSTAGE-1 stages ahead of the MFMAs, so a global / L2 round trip is hidden.
//   * operand contiguous along K in memory (NT's a and b, NN's a): stage = [rows][BKS k], fragment reads are
//     ds_read_b128 (32 consecutive rows x one 16-byte chunk);
//   * operand contiguous along its row index in memory (NN's b, TN's a and b): stage = [BKS k][rows], the memory
//     layout as it is, and the MFMA fragments (8 consecutive k of one row per lane) are gathered by the LDS
//     transpose read ds_read_b64_tr_b16 (16 lanes fetch 4 k-rows x 16 rows and lane j receives row j's 4 k).
// 16-byte chunks are XOR-swizzled (applied on the global side of the copy) so that both kinds of reads are
// bank-conflict free.  Rows / k outside the matrix get an out-of-range buffer offset and arrive as zeros, so
// the main loop has no branch.  MFMA fragments are double buffered over the 16-wide k sub-steps of a stage.
//
// The accumulator is computed transposed (operands swapped in the MFMA) so that each lane ends up with 4
// consecutive columns of one row of C; in the epilogue every wave passes its sub-tile, 32 rows at a time, through a
// private LDS scratch and stores row segments of 16 bytes per lane (no workgroup barrier).  With PERSIST a workgroup
// walks several tiles, the first NSTAGE-1 stages of the next tile are already in flight during the epilogue, and
// only half of its waves issue copies (NLOAD below), so that the other half's stores can drain under the next tile.
// Decode-sized tiles (BM <= 64) may cover fewer output columns than the MFMA tile is wide (bn_out).
#pragma once
#include <type_traits>
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));

static constexpr int BKS = 32;                // default k extent of one LDS stage
static constexpr unsigned OOB = 0x80000000u;  // buffer offset that is always out of range -> load returns 0
static constexpr int DMA_SHIFT = 3072;        // operand windows start this many bytes early (see dma16_group's offsets)

template <int BM_, int BN_, int WM_, int WN_, int NSTAGE_ = 4, int SCHED_ = 2, bool PERSIST_ = true, int BKS_ = 32>
struct TileCfg {
  static constexpr int BKS = BKS_;              // k extent of one LDS stage (multiple of 32; K-contiguous operands only if > 32)
  // PERSIST: one workgroup per CU walks several tiles and fetches the next tile's first stages under the epilogue
  static constexpr bool PERSIST = PERSIST_;
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NSTAGE = NSTAGE_;
  static constexpr int SCHED = SCHED_;  // 0: compiler's order, 1: fences between sub-steps, 2: + LDS reads spread 1:1 between
                                        // the MFMAs, 3: + all LDS reads of a sub-step issued ahead of its MFMAs
  static constexpr int THREADS = 64 * WM * WN;
  static constexpr int NWAVES = WM * WN;
  static constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wave
  static constexpr int STAGE_CHUNKS = (BM + BN) * (BKS / 8);  // uint4 per LDS stage
  static constexpr int SMEM_CHUNKS = NSTAGE * STAGE_CHUNKS;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
  // epilogue scratch: every wave parks 32 rows x its WTN columns of bf16 at a time, at the tail of the LDS buffer
  static constexpr int SCRATCH_BYTES = NWAVES * 32 * WTN * 2;
  static_assert(SCRATCH_BYTES <= SMEM_CHUNKS * 16, "epilogue scratch must fit");
  static_assert(!PERSIST || SCRATCH_BYTES <= STAGE_CHUNKS * 16, "persistent tiles keep NSTAGE-1 stages free of the scratch");
  static_assert(SMEM_CHUNKS * 16 <= 160 * 1024, "LDS capacity");
  // workgroups that fit on one compute unit: LDS (160 KB) and at most 8 waves (2 per SIMD, 256 registers each)
  static constexpr int WGS_PER_CU = ((160 * 1024) / (SMEM_CHUNKS * 16)) < (8 / NWAVES) ? ((160 * 1024) / (SMEM_CHUNKS * 16))
                                                                                        : (8 / NWAVES);
  static constexpr int MIN_WAVES_PER_EU = (NWAVES * WGS_PER_CU) / 4 > 0 ? (NWAVES * WGS_PER_CU) / 4 : 1;
};

// ---- operand contiguous along K: stage [ROWS][BKS k], row = BKS*2 bytes = CPR chunks of 16 bytes; 16 chunks make
// up the 64 LDS banks, so chunk c of row r sits at c ^ ((r >> SWZ_SHIFT) & (CPR-1)) (for 64-byte rows: c ^ ((r>>2)&3)):
// 16 consecutive rows then read the same logical chunk from 16 different bank groups.
// One wave instruction fills 64/CPR rows (64 lanes x 16 B, lane order).  `origin` points at the tile's first row;
// rowmap(rr) gives the row of tile row rr RELATIVE to the origin, or -1 if that row does not exist.
template <int ROWS, int NWAVES, int BKS_ = 32, bool GROUPED = true>
struct KContigOperand {
  static constexpr int CPR = BKS_ / 8;           // chunks per row: 4, 8 or 16
  static constexpr int RPI = 64 / CPR;           // rows per copy instruction
  static constexpr int SWZ_SHIFT = CPR == 4 ? 2 : (CPR == 8 ? 1 : 0);
  static constexpr int NI = ROWS / RPI / NWAVES;  // copy instructions per wave per stage
  // copies that share one LDS base (see dma16_group).  GROUPED: a wave's NI copies fill consecutive 1 KB groups of the
  // stage; otherwise the waves' copies interleave (copy `it` of wave w fills group it*NWAVES + w), which keeps the
  // rows a wave instruction touches in memory next to those of its neighbours: the decode-sized weight streams
  // measured 1-1.5 % faster that way, the block-sized tiles with the grouped issue.
  static constexpr int GRP = GROUPED ? (NI >= 4 ? 4 : NI) : 1;
  static __device__ __forceinline__ int group_of(int wave, int it) { return GROUPED ? wave * NI + it : it * NWAVES + wave; }
  static constexpr int N_VMEM = NI;
  static constexpr int READS_PER_FRAG = 1;
  static_assert(NI % GRP == 0, "whole groups of copies");
  static_assert(CPR == 4 || CPR == 8 || CPR == 16, "stage depth must be 32, 64 or 128");
  static_assert(ROWS % (RPI * NWAVES) == 0, "rows must divide over the waves");
  static __device__ __forceinline__ int swz(int row) { return (row >> SWZ_SHIFT) & (CPR - 1); }
  const bf16_t* origin;
  unsigned voff[NI];
  int wave;
  int kc[NI];  // logical chunk this lane fetches in copy instruction `it` (the same for all `it` when RPI == 16)

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* origin_, long long ld, RowMap rowmap) {
    origin = origin_;
    const int lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      // a wave's NI copies fill consecutive groups of RPI rows (1 KB of LDS each).  Physical slot lane % CPR of row
      // (wave*NI + it)*RPI + lane / CPR holds logical chunk slot ^ swz(row); the swizzle has a period of 16 rows, so
      // with 16 rows per instruction it does not depend on `it`
      const int row = group_of(wave, it) * RPI + lane / CPR;
      kc[it] = (lane & (CPR - 1)) ^ swz(RPI == 16 ? lane / CPR : row);
      const long long r = rowmap(row);
      // memory-side offsets are relative to a base DMA_SHIFT bytes in front of the operand, less the immediate offset
      // the copy carries as member it % GRP of its group (dma16_group)
      voff[it] = (r >= 0) ? (unsigned)((r * ld + kc[it] * 8) * 2 + DMA_SHIFT - (it % GRP) * 1024) : OOB;
    }
  }
  // koff: element offset of the K-group the stage belongs to (0 unless the contraction runs over several buffers)
  template <bool STREAM = false>
  __device__ __forceinline__ void issue(int k0, int K, uint4* tile, long long koff) const {
    const i32x4_t rs = make_rsrc(reinterpret_cast<const char*>(origin + koff + k0) - DMA_SHIFT);
    if (k0 + BKS_ <= K) {  // a whole stage inside the contraction (all but the last one or two): no per-lane test
#pragma unroll
      for (int gi = 0; gi < NI / GRP; ++gi) dma16_group<STREAM, GRP>(rs, voff + gi * GRP, tile + group_of(wave, gi * GRP) * 64);
      return;
    }
#pragma unroll
    for (int gi = 0; gi < NI / GRP; ++gi) {
      unsigned v[GRP];
#pragma unroll
      for (int j = 0; j < GRP; ++j) v[j] = (k0 + kc[RPI == 16 ? 0 : gi * GRP + j] * 8) < K ? voff[gi * GRP + j] : OOB;
      dma16_group<STREAM, GRP>(rs, v, tile + group_of(wave, gi * GRP) * 64);
    }
  }
  // fragment for MFMA rows row0 .. row0+31, k sub-step ks (16 wide): lane (row0 + lane%32, k = 16 ks + 8 (lane/32) ..+7)
  static __device__ __forceinline__ bf16x8_t frag(const uint4* tile, int row0, int ks, int lane) {
    const int row = row0 + (lane & 31);
    const int c = ks * 2 + (lane >> 5);
    return __builtin_bit_cast(bf16x8_t, tile[row * CPR + (c ^ swz(row))]);
  }
};

// ---- operand contiguous along its row index ([K][rows] in memory): stage [BKS k][ROWS] as in memory, k-row =
// ROWS*2 bytes; chunk c of k-row k sits at c ^ ((k&3)<<2).  One wave instruction fills 512/ROWS k-rows.
// `origin` points at (k = 0, first row of the tile); rows_valid = rows of the tile that exist (multiple of 8).
template <int ROWS, int NWAVES, int BKS_ = 32, bool GROUPED = true>
struct RowContigOperand {
  static constexpr int CPR = ROWS / 8;       // chunks per k-row
  static constexpr int KPI = 64 / CPR;       // k-rows per copy instruction
  static constexpr int NI = BKS_ / KPI / NWAVES;
  static constexpr int GRP = GROUPED ? (NI >= 4 ? 4 : NI) : 1;  // as in KContigOperand
  static __device__ __forceinline__ int group_of(int wave, int it) { return GROUPED ? wave * NI + it : it * NWAVES + wave; }
  static constexpr int N_VMEM = NI;
  static constexpr int READS_PER_FRAG = 2;
  static_assert(NI % GRP == 0, "whole groups of copies");
  static_assert(ROWS >= 128 && ROWS <= 512 && BKS_ % (KPI * NWAVES) == 0, "unsupported tile shape for a transposed operand");
  const bf16_t* origin;
  long long ld;
  unsigned voff[NI];
  int wave, klocal;  // klocal: k-row inside an instruction's group

  template <class RowMap>
  __device__ __forceinline__ void init(const bf16_t* origin_, long long ld_, RowMap rowmap) {
    origin = origin_;
    ld = ld_;
    const int lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    klocal = lane / CPR;
    const int phys = lane % CPR;
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      const int k = group_of(wave, it) * KPI + klocal;
      const int c = phys ^ ((k & 3) << 2);
      const long long r = rowmap(c * 8);  // 8 consecutive rows share validity (dims % 8 == 0)
      voff[it] = (r >= 0) ? (unsigned)(((long long)k * ld_ + r) * 2 + DMA_SHIFT - (it % GRP) * 1024) : OOB;
    }
  }
  template <bool STREAM = false>
  __device__ __forceinline__ void issue(int k0, int K, uint4* tile, long long koff) const {
    const i32x4_t rs = make_rsrc(reinterpret_cast<const char*>(origin + koff + (long long)k0 * ld) - DMA_SHIFT);
    if (k0 + BKS_ <= K) {  // a whole stage inside the contraction: no per-lane test
#pragma unroll
      for (int gi = 0; gi < NI / GRP; ++gi) dma16_group<STREAM, GRP>(rs, voff + gi * GRP, tile + group_of(wave, gi * GRP) * 64);
      return;
    }
#pragma unroll
    for (int gi = 0; gi < NI / GRP; ++gi) {
      unsigned v[GRP];
#pragma unroll
      for (int j = 0; j < GRP; ++j) {
        const int k = group_of(wave, gi * GRP + j) * KPI + klocal;
        v[j] = (k0 + k < K) ? voff[gi * GRP + j] : OOB;
      }
      dma16_group<STREAM, GRP>(rs, v, tile + group_of(wave, gi * GRP) * 64);
    }
  }
  // same fragment as KContigOperand::frag, gathered by two transpose reads of 4 k each
  static __device__ __forceinline__ bf16x8_t frag(const uint4* tile, int row0, int ks, int lane) {
    const int i16 = lane & 15;
    const int m = row0 + ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;  // the 4 rows this lane's 8 bytes cover
    const int kq = i16 >> 2;                                      // which of the 4 k-rows this lane fetches
    const int kb = ks * 16 + (lane >> 5) * 8;
    const char* base = reinterpret_cast<const char*>(tile);
    const int coff = (((m >> 3) ^ (kq << 2)) << 4) + ((m & 7) << 1);  // (k & 3) == kq for both reads
    const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4_t*)(base + (kb + kq) * (ROWS * 2) + coff));
    const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4_t*)(base + (kb + 4 + kq) * (ROWS * 2) + coff));
    const short8_t v = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  }
};

template <bool ROWCONTIG, int ROWS, int NWAVES, int BKS_, bool GROUPED>
struct OperandSel { typedef KContigOperand<ROWS, NWAVES, BKS_, GROUPED> type; };
template <int ROWS, int NWAVES, int BKS_, bool GROUPED>
struct OperandSel<true, ROWS, NWAVES, BKS_, GROUPED> { typedef RowContigOperand<ROWS, NWAVES, BKS_, GROUPED> type; };

// Which weight row (relative to the tile's first row n0) lies in row rr of the B tile in LDS, or -1 for none.  Plain
// epilogues: rows in order, as many as the tile covers (bn_out) and the matrix has.  SwiGLU: each wave's WTN tile rows
// are 32 gate rows, then the 32 up rows of the same output columns (`half` rows further down), and so on, so that an
// accumulator pair of a wave holds gate and up of the same 32 outputs.
template <class CFG, bool SWI>
__device__ __forceinline__ long long b_tile_row(int rr, int n0, int bn_out, int N, int half) {
  if constexpr (SWI) {
    const int w = rr / CFG::WTN, rw = rr - w * CFG::WTN;
    const int j = rw >> 5, c = rw & 31;
    const int col = (w * (CFG::TN / 2) + (j >> 1)) * 32 + c;  // output column relative to n0
    if (col >= bn_out || n0 + col >= half) return -1;
    return (long long)col + ((j & 1) ? half : 0);
  } else {
    const int nrem = (N - n0) < bn_out ? (N - n0) : bn_out;
    return rr < nrem ? (long long)rr : -1;
  }
}

template <int TM, int TN>
struct Frags {
  bf16x8_t a[TM], b[TN];
};

// Instruction-order request for one k sub-step (between two scheduling fences): after every MFMA place this
// MFMA's share of the NR LDS reads and NV global->LDS copies.
template <int I, int NM, int NR, int NV>
struct Pipe {
  static __device__ __forceinline__ void run() {
    if constexpr (I < NM) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      constexpr int r = (NR * (I + 1)) / NM - (NR * I) / NM;
      constexpr int v = (NV * (I + 1)) / NM - (NV * I) / NM;
      if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
      if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
      Pipe<I + 1, NM, NR, NV>::run();
    }
  }
};

template <class CFG, bool AT, bool BT, int EPI>
__global__ __launch_bounds__(CFG::THREADS, CFG::MIN_WAVES_PER_EU) void gemm_kernel(const GemmParams p) {
  constexpr int BM = CFG::BM, BN = CFG::BN, NSTAGE = CFG::NSTAGE;
  constexpr int TM = CFG::TM, TN = CFG::TN, WTM = CFG::WTM, WTN = CFG::WTN;
  constexpr bool SWI = (EPI == EPI_SWIGLU_FWD);
  constexpr int BN_OUT = SWI ? BN / 2 : BN;  // output columns covered by one tile
  static_assert(!SWI || TN % 2 == 0, "SwiGLU pairing needs an even number of N tiles per wave");

  __shared__ uint4 smem[CFG::SMEM_CHUNKS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / CFG::WN;
  const int wn = wave - wm * CFG::WN;
  const int frow = lane & 31;  // accumulator row within a 32-row MFMA tile
  const int fk = lane >> 5;    // which half of the tile's columns / k this lane holds

  // ---- tiles of this workgroup.  Tile ids are cut into 8 contiguous ranges, one per XCD (workgroup b runs on XCD
  // b % 8), so that the workgroups sharing an L2 work on neighbouring tiles; inside a range the workgroups of the XCD
  // take tiles round-robin.  A tile id maps to (rank g, tile row, tile column) in a grouped (8 tile rows) order.
  // Decode-sized tiles may be told to cover fewer output columns than the MFMA tile is wide (bn_out, a multiple of
  // 8): the kernel is then a weight stream, and what counts is that every compute unit gets the same number of weight
  // rows.  The rows beyond bn_out are not fetched (out-of-range copy offsets) and their columns are not stored.
  constexpr bool NARROW = (BM <= 64);
  const int bn_out = (NARROW && p.bn_out > 0) ? p.bn_out : BN_OUT;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = (p.N + bn_out - 1) / bn_out;
  const int tiles = tiles_m * tiles_n;
  const int total = tiles * p.G;
  int pid, pid_end, pid_step;
  {
    const int bid = blockIdx.x, nb = gridDim.x;
    const int q = total >> 3, rem = total & 7, x = bid & 7;
    const int start = x * q + (x < rem ? x : rem);
    pid_end = start + q + (x < rem ? 1 : 0);
    pid = start + (bid >> 3);
    pid_step = (nb - x + 7) >> 3;  // workgroups on this XCD
  }

  constexpr int BKS = CFG::BKS;         // this instantiation's stage depth (hides the namespace default)
  constexpr int NSUB = BKS / 16;        // 16-wide k sub-steps (one MFMA deep) per stage
  // Waves that issue the global -> LDS copies.  A wave's copies and its epilogue stores complete in issue order on one
  // counter, so a wave that copies has to let its stores drain before it can wait for the next tile's second stage,
  // and the stores of all compute units come as one chip-wide burst (the workgroups run in lockstep) that takes
  // several k steps when a tile has several outputs.  In the persistent eight-wave tiles only the first four waves
  // copy (twice the instructions each, one such wave per SIMD next to a wave that only computes): the other four never
  // wait on that counter in the main loop, and their half of the stores drains under the next tile.  Measured: forward
  // SwiGLU GEMM -5 %, GELU' GEMM -5 %, weight gradients -2.4 %, QKV -3 %; nothing lost anywhere.
  constexpr int NLOAD = (CFG::PERSIST && CFG::NWAVES == 8) ? 4 : CFG::NWAVES;
  const bool loader = wave < NLOAD;
  typedef typename OperandSel<AT, BM, NLOAD, BKS, (BM > 64)>::type OpA;
  typedef typename OperandSel<BT, BN, NLOAD, BKS, (BM > 64)>::type OpB;
  OpA la;
  OpB lb;
  int g = 0, m0 = 0, n0 = 0;
  int ik0 = 0, ikg = 0;  // k position and K-group of the next stage to be copied
  auto setup_tile = [&](int id) {
    ik0 = 0;
    ikg = 0;
    g = id / tiles;
    const int t = id - g * tiles;
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int grp = t / width;
    const int first = grp * GROUP;
    const int gsize = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
    const int r = t - grp * width;
    m0 = (first + r % gsize) * BM;
    n0 = (r / gsize) * bn_out;
    const bf16_t* ag = p.a + (long long)g * p.stride_a;
    const bf16_t* bg = p.b + (long long)g * p.stride_b;
    const int mrem = p.M - m0;
    la.init(AT ? ag + m0 : ag + (long long)m0 * p.lda, p.lda,
            [=](int rr) -> long long { return (rr < mrem) ? (long long)rr : -1; });
    if constexpr (!BT) {
      const int n0c = n0, bnc = bn_out, Nc = p.N, halfc = p.half;
      auto rowmap = [=](int rr) -> long long { return b_tile_row<CFG, SWI>(rr, n0c, bnc, Nc, halfc); };
      lb.init(bg + (long long)n0 * p.ldb, p.ldb, rowmap);
    } else {
      const int nrem = p.N - n0;
      lb.init(bg + n0, p.ldb, [=](int rr) -> long long { return (rr < nrem) ? (long long)rr : -1; });
    }
  };

  // With the broadcast epilogue the contraction index runs over kcat buffers of K each (operand g' of both a and b lies
  // kstride elements after operand g'-1): that is how the sum over ranks of Eq. A3's shared channels is taken inside
  // the accumulator.  Every other instantiation keeps the single-buffer code (no per-stage bookkeeping).
  constexpr bool KCAT = (EPI == EPI_SHARED_BCAST);
  const int K = p.K;
  const int kcat = KCAT ? (p.kcat > 1 ? p.kcat : 1) : 1;
  const int nk = ((K + BKS - 1) / BKS) * kcat;
  constexpr int A_CHUNKS = BM * (BKS / 8);
  // decode-sized tiles (at most 64 token rows per rank: one tile row) read every weight row exactly once
  constexpr bool B_STREAM = (BM <= 64);
  auto stage_a = [&](int s) -> uint4* { return smem + (s % NSTAGE) * CFG::STAGE_CHUNKS; };
  // stages are issued in order; past the end every offset is out of range: zeros land in a slot nobody reads
  auto issue_stage = [&](int s) {
    if (!loader) return;
    uint4* As = stage_a(s);
    if constexpr (KCAT) {
      const int kk = ikg < kcat ? K : 0;
      la.issue(ik0, kk, As, (long long)ikg * p.kstride_a);
      lb.template issue<B_STREAM>(ik0, kk, As + A_CHUNKS, (long long)ikg * p.kstride_b);
      ik0 += BKS;
      if (ik0 >= K) {
        ik0 = 0;
        ++ikg;
      }
    } else {
      la.issue(s * BKS, K, As, 0);
      lb.template issue<B_STREAM>(s * BKS, K, As + A_CHUNKS, 0);
    }
  };

  constexpr int SCHED = CFG::SCHED;
  constexpr int NM = TM * TN;
  constexpr int NR = TM * OpA::READS_PER_FRAG + TN * OpB::READS_PER_FRAG;
  constexpr int NV = OpA::N_VMEM + OpB::N_VMEM;  // copies per wave per stage
  auto fence = [&]() {
    if constexpr (SCHED >= 1) __builtin_amdgcn_sched_barrier(0);
  };

  // epilogue stores per wave and tile (known at compile time except for the broadcast epilogue's loop over ranks)
  constexpr int EPI_STORES =
      (EPI == EPI_SHARED_BCAST)
          ? 1000
          : TM * (32 * (SWI ? WTN / 16 : WTN / 8) / 64) *
                (EPI == EPI_SWIGLU_FWD ? 3 : ((EPI == EPI_GELU_FWD || EPI == EPI_SWIGLU_BWD) ? 2 : 1));
  bool first_tile = true;

  if (pid >= pid_end) return;
  setup_tile(pid);
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s) issue_stage(s);

  while (true) {
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto load_frags = [&](int s, int ks, Frags<TM, TN>& f) {
      const uint4* As = stage_a(s);
      const uint4* Bs = As + A_CHUNKS;
#pragma unroll
      for (int i = 0; i < TM; ++i) f.a[i] = OpA::frag(As, wm * WTM + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) f.b[j] = OpB::frag(Bs, wn * WTN + j * 32, ks, lane);
    };
    auto mfma_all = [&](const Frags<TM, TN>& f) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          // operands swapped: the accumulator holds C^T, i.e. lane = row of C, registers = columns of C
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
    };

    // copies complete in order: with at most the two newest stages outstanding, stage 0 has landed.  After a
    // previous tile, the wave's newest vector-memory instructions are that tile's epilogue stores (a fixed number,
    // all issued after this tile's first copies): they may stay in flight under the first stage's MFMAs.  The
    // barrier also separates the previous tile's epilogue scratch from the copies that will reuse its LDS slot.
    if (loader) {
      if (first_tile || EPI_STORES + (NSTAGE - 2) * NV > 63)
        wait_vmcnt<(NSTAGE - 2) * NV>();
      else
        wait_vmcnt<(EPI_STORES + (NSTAGE - 2) * NV > 63) ? 0 : EPI_STORES + (NSTAGE - 2) * NV>();
    }
    first_tile = false;
    __syncthreads();
    // fragments are double buffered over the NSUB 16-wide k sub-steps of a stage (NSUB is even)
    Frags<TM, TN> fr[2];
    load_frags(0, 0, fr[0]);
    fence();

    for (int kt = 0; kt < nk; ++kt) {
      // the slot of stage kt-1 is free (everyone passed the barrier below in the previous iteration)
      issue_stage(kt + NSTAGE - 1);
#pragma unroll
      for (int ss = 0; ss < NSUB; ++ss) {
        if (ss + 1 < NSUB) {
          load_frags(kt, ss + 1, fr[(ss + 1) & 1]);
        } else {
          // last sub-step: stage kt+1 must have landed (the two newest stages may still be in flight) and be visible
          if (loader) wait_vmcnt<(NSTAGE - 2) * NV>();
          __syncthreads();
          fence();
          load_frags(kt + 1, 0, fr[0]);
        }
        mfma_all(fr[ss & 1]);
        if constexpr (SCHED == 2) Pipe<0, NM, NR, 0>::run();
        if constexpr (SCHED == 3) {
          __builtin_amdgcn_sched_group_barrier(0x100, NR, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
        }
        fence();
      }
    }
    // the zero-filled stages past K still target LDS: let them land, and let every wave finish its fragment reads,
    // before the buffers are reused
    if (loader) wait_vmcnt<0>();
    __syncthreads();

    // ---- the finished tile's coordinates; then start on the next tile's data before the epilogue
    const int eg = g, em0 = m0, en0 = n0;
    const int next = pid + pid_step;
    const bool has_next = CFG::PERSIST && next < pid_end;
    if (has_next) {
      setup_tile(next);
#pragma unroll
      for (int s = 0; s < NSTAGE - 1; ++s) issue_stage(s);  // slots 0 .. NSTAGE-2; the scratch below is in the last slot
    }

    // ---- epilogue.  Each lane holds C[row = lane%32][col = 8*q + 4*(lane/32) + 0..3] of every 32x32 tile in
    // acc[..][4q..4q+3].  Stored as they are, these 8-byte pieces would scatter over 32 rows per instruction; so each
    // wave rounds 32 rows x WTN columns to bf16 into its own LDS scratch (chunk index XOR-swizzled by the row) and
    // reads them back row-wise: 16 bytes per lane, consecutive lanes = consecutive columns.  The fused element-wise
    // work (activation, its derivative, the private half of the partial channel-reduce + residual) happens there.
    //
    // Every global access of the epilogue is a raw buffer load / store whose offset is replaced by an out-of-range
    // one where the row or column does not exist (the load then returns zero, the store is dropped): the code has no
    // branch, so the number of vector-memory instructions per tile is fixed (the wait at the top of the next tile
    // counts on it) and the compiler's own waits for the prefetched second operand stay exact (vmcnt(n), not
    // vmcnt(0), which would also wait for the stores and the prefetch issued just before).
    constexpr int CHW = WTN / 8;  // 16-byte chunks per scratch row
    char* scratch = reinterpret_cast<char*>(smem) + (CFG::SMEM_CHUNKS * 16 - CFG::SCRATCH_BYTES) + wave * (32 * WTN * 2);
    const uint4* scr4 = reinterpret_cast<const uint4*>(scratch);
    auto staged = [&](int row, int c) -> uint4 { return scr4[row * CHW + (c ^ (row & (CHW - 1)))]; };
    auto unpack = [](const uint4& v, float* f) {
      f[0] = lo_bf(v.x); f[1] = hi_bf(v.x); f[2] = lo_bf(v.y); f[3] = hi_bf(v.y);
      f[4] = lo_bf(v.z); f[5] = hi_bf(v.z); f[6] = lo_bf(v.w); f[7] = hi_bf(v.w);
    };
    auto pack = [](const float* f) -> uint4 {
      return make_uint4(pack2bf(f[0], f[1]), pack2bf(f[2], f[3]), pack2bf(f[4], f[5]), pack2bf(f[6], f[7]));
    };
    constexpr int OCW = SWI ? CHW / 2 : CHW;      // 16-byte chunks per output row of the wave
    constexpr int STEPS = 32 * OCW / 64;          // vectors per lane per 32-row slab
    static_assert(STEPS >= 1, "a slab must give every lane at least one vector");
    constexpr bool HAS_AUX = (EPI == EPI_ROWPAR || EPI == EPI_GELU_BWD || EPI == EPI_SWIGLU_BWD);
    constexpr int AUXV = (EPI == EPI_SWIGLU_BWD) ? 2 : 1;
    const int wrow0 = em0 + wm * WTM;             // first row of the wave's sub-tile
    const int wcol0 = en0 + wn * (SWI ? WTN / 2 : WTN);  // first output column of the wave's sub-tile
    const int ncols = SWI ? p.half : p.N;
    // buffer windows start at the wave's first row, so that offsets stay small: (row in slab) * ld + column, in
    // bytes; the slab's 32 * i rows go into the scalar offset
    const rsrc_t rc = make_rsrc_t(p.c + (long long)eg * p.stride_c + (long long)wrow0 * p.ldc);
    const rsrc_t rc2 = make_rsrc_t((EPI == EPI_GELU_FWD || SWI) ? p.c2 + (long long)eg * p.stride_c2 + (long long)wrow0 * p.ldc2 : p.c);
    const rsrc_t raux = make_rsrc_t(HAS_AUX ? p.aux + (long long)eg * p.stride_aux + (long long)wrow0 * p.ldaux : p.c);
    int erow[STEPS], ecol[STEPS];                 // slab row and output column of the lane's vector in step st
    unsigned voff_c[STEPS], voff_c2[STEPS], voff_aux[STEPS];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      const int idx = st * 64 + lane;
      erow[st] = idx / OCW;
      const int oc = idx - erow[st] * OCW;
      ecol[st] = wcol0 + oc * 8;
      const bool colok = ecol[st] < ncols && ecol[st] - en0 < bn_out;
      voff_c[st] = colok ? (unsigned)((erow[st] * p.ldc + ecol[st]) * 2) : OOB;
      voff_c2[st] = colok ? (unsigned)((erow[st] * p.ldc2 + ecol[st]) * 2) : OOB;
      // the residual is only needed where the vector has a private channel (Eq. A3)
      const bool auxok = colok && (EPI != EPI_ROWPAR || ecol[st] + 7 >= p.hs);
      voff_aux[st] = auxok ? (unsigned)((erow[st] * p.ldaux + ecol[st]) * 2) : OOB;
    }
    auto rows_left = [&](int i) { return p.M - wrow0 - i * 32; };
    // epilogues that read a second tensor (residual, saved pre-activations) fetch it AUXD 32-row slabs ahead: a slab's
    // conversion, LDS round trip and stores take less time than one trip to memory.  The residual epilogue, light on
    // registers, fetches all of the wave's slabs at once; the activation-derivative epilogues (whose NN main loop
    // already needs nearly every register) measured faster with two.
    constexpr int AUXD = !HAS_AUX ? 1 : (TM < 2 ? 1 : (EPI == EPI_ROWPAR && STEPS * 4 * TM <= 64 ? TM : 2));
    u32x4_t auxbuf[AUXD][HAS_AUX ? STEPS * AUXV : 1];
    auto aux_fetch = [&](int i, u32x4_t* buf) {
      const int rl = rows_left(i);
      const int so = i * 32 * (int)p.ldaux * 2;
#pragma unroll
      for (int st = 0; st < STEPS; ++st) {
        const unsigned vo = erow[st] < rl ? voff_aux[st] : OOB;
        // read once by this tile only: non-temporal hint (cache policy bit 1)
        buf[st * AUXV] = __builtin_amdgcn_raw_buffer_load_b128(raux, vo, so, 2);
        if constexpr (AUXV == 2) buf[st * AUXV + 1] = __builtin_amdgcn_raw_buffer_load_b128(raux, vo, so + p.half * 2, 2);
      }
    };
    auto to_u4 = [](const u32x4_t& v) -> uint4 { return make_uint4(v[0], v[1], v[2], v[3]); };
    // Stores keep the slab offset in the vector offset and pass no scalar offset register: the 16-byte store reads
    // its data registers a few cycles after it issues, and the compiler only keeps the following instructions from
    // overwriting them (the documented store-data hazard) for the form without a scalar offset register; with one,
    // the first data register was now and then overwritten by the next vector's arithmetic before the store had
    // read it (seen as a wrong first dword in a few lanes at full problem sizes).  The two idle cycles after the
    // store restate that requirement where the store is issued.
    auto put = [&](const rsrc_t& r, const uint4& v, bool ok, unsigned vo, int so) {
      const u32x4_t w = {v.x, v.y, v.z, v.w};
      __builtin_amdgcn_raw_buffer_store_b128(w, r, ok ? vo + (unsigned)so : OOB, 0, 0);
      asm volatile("s_nop 1" ::: "memory");
    };
    // the same for a tensor that nothing reads before the backward pass (saved pre-activations): non-temporal hint,
    // so that it does not push the activation the next GEMM is about to read out of the caches
    auto put_late = [&](const rsrc_t& r, const uint4& v, bool ok, unsigned vo, int so) {
      const u32x4_t w = {v.x, v.y, v.z, v.w};
      __builtin_amdgcn_raw_buffer_store_b128(w, r, ok ? vo + (unsigned)so : OOB, 0, 2);
      asm volatile("s_nop 1" ::: "memory");
    };
    // The slab loop exists three times for the row-parallel epilogue: a tile that lies entirely left of hs holds
    // shared channels only (Eq. A3: every rank's partial sum goes out as it is, the reduce adds the residual), so it
    // needs neither the residual fetch nor the case split and runs the plain store path; a tile entirely right of hs
    // needs no case split; only a tile that contains hs takes the general code.  All versions issue the same number
    // of stores, and each is free of branches in itself.
    auto slabs = [&](auto tile_kind) {
      constexpr bool SH = decltype(tile_kind)::value == 1;    // shared channels only
      constexpr bool PRIV = decltype(tile_kind)::value == 2;  // private channels only
      if constexpr (HAS_AUX && !SH) {
#pragma unroll
        for (int i = 0; i < AUXD && i < TM; ++i) aux_fetch(i, auxbuf[i]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int c = j * 4 + q;
            uint2 w;
            w.x = pack2bf(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1]);
            w.y = pack2bf(acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
            *reinterpret_cast<uint2*>(scratch + ((frow * CHW + (c ^ (frow & (CHW - 1)))) * 16 + fk * 8)) = w;
          }
        // the wave reads back what its other lanes wrote: LDS executes a wave's operations in order; the compiler
        // must not reorder across this point either
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int rl = rows_left(i);
        const int so_c = i * 32 * (int)p.ldc * 2;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
          const bool rowok = erow[st] < rl;
          const unsigned vo = voff_c[st];
          if constexpr (SWI) {
            // scratch columns: [gate 32 | up 32] pairs; output chunk oc -> gate chunk (oc/4)*8 + oc%4, up chunk = +4
            const int oc = (st * 64 + lane) - erow[st] * OCW;
            const int gc = (oc >> 2) * 8 + (oc & 3);
            const uint4 gw = staged(erow[st], gc), uw = staged(erow[st], gc + 4);
            float gt[8], up[8], y[8];
            unpack(gw, gt);
            unpack(uw, up);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = gt[e] * sigmoid_f(gt[e]) * up[e];
            put_late(rc, gw, rowok, vo, so_c);
            put_late(rc, uw, rowok, vo, so_c + p.half * 2);
            put(rc2, pack(y), rowok, voff_c2[st], i * 32 * (int)p.ldc2 * 2);
          } else {
            const int c = (st * 64 + lane) - erow[st] * CHW;
            const uint4 raw = staged(erow[st], c);
            if constexpr (EPI == EPI_PLAIN) {
              if (p.late_c) put_late(rc, raw, rowok, vo, so_c);
              else put(rc, raw, rowok, vo, so_c);
            } else if constexpr (EPI == EPI_GELU_FWD) {
              // the activation is taken of the bf16-rounded pre-activation, the value the backward pass sees too
              float v[8], y[8];
              unpack(raw, v);
#pragma unroll
              for (int e = 0; e < 8; ++e) y[e] = gelu_f(v[e]);
              put_late(rc, raw, rowok, vo, so_c);
              put(rc2, pack(y), rowok, voff_c2[st], i * 32 * (int)p.ldc2 * 2);
            } else if constexpr (EPI == EPI_ROWPAR && SH) {
              put(rc, raw, rowok, vo, so_c);  // a tile of shared channels only: this rank's partial sums as they are
            } else if constexpr (EPI == EPI_ROWPAR) {
              // Eq. A3 case split, private side: columns >= hs are final here (scale, + residual); columns < hs are
              // stored as this rank's partial sum for the reduce kernel (rounding a bf16 value to bf16 again leaves
              // its bits as they are).  The private value is scaled from the bf16-rounded partial.
              float v[8], r[8];
              unpack(raw, v);
              unpack(to_u4(auxbuf[i % AUXD][st]), r);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] = (PRIV || ecol[st] + e >= p.hs) ? p.scale * v[e] + r[e] : v[e];
              put(rc, pack(v), rowok, vo, so_c);
            } else if constexpr (EPI == EPI_SHARED_BCAST) {
              // Eq. A3, shared channels with the sum over ranks already in the accumulator: every rank's output gets
              // the same sum plus that rank's residual
              float v[8];
              unpack(raw, v);
              for (int m = 0; m < p.bcast; ++m) {
                const rsrc_t rr = make_rsrc_t(p.aux + (long long)m * p.stride_aux + (long long)wrow0 * p.ldaux);
                const rsrc_t rw = make_rsrc_t(p.c + (long long)m * p.stride_c + (long long)wrow0 * p.ldc);
                const unsigned va = (rowok && ecol[st] < ncols) ? (unsigned)((erow[st] * p.ldaux + ecol[st]) * 2) : OOB;
                float r[8], o[8];
                unpack(to_u4(__builtin_amdgcn_raw_buffer_load_b128(rr, va, i * 32 * (int)p.ldaux * 2, 0)), r);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = v[e] + r[e];
                put(rw, pack(o), rowok, vo, so_c);
              }
            } else if constexpr (EPI == EPI_GELU_BWD) {
              float v[8], pr[8];
              unpack(raw, v);
              unpack(to_u4(auxbuf[i % AUXD][st]), pr);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(pr[e]);
              put(rc, pack(v), rowok, vo, so_c);
            } else if constexpr (EPI == EPI_SWIGLU_BWD) {
              float v[8], gt[8], up[8], dg[8], du[8];
              unpack(raw, v);
              unpack(to_u4(auxbuf[i % AUXD][st * AUXV]), gt);
              unpack(to_u4(auxbuf[i % AUXD][st * AUXV + (AUXV - 1)]), up);
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const float sg = sigmoid_f(gt[e]);
                dg[e] = v[e] * up[e] * sg * (1.0f + gt[e] * (1.0f - sg));
                du[e] = v[e] * gt[e] * sg;
              }
              put(rc, pack(dg), rowok, vo, so_c);
              put(rc, pack(du), rowok, vo, so_c + p.half * 2);
            }
          }
        }
        asm volatile("" ::: "memory");  // keep the next 32 rows' scratch writes behind these reads
        if constexpr (HAS_AUX && !SH) {
          if (i + AUXD < TM) aux_fetch(i + AUXD, auxbuf[i % AUXD]);  // this slab's registers are free again
        }
      }
    };
    if constexpr (EPI == EPI_ROWPAR) {
      if (en0 + bn_out <= p.hs) slabs(std::integral_constant<int, 1>{});
      else if (en0 >= p.hs) slabs(std::integral_constant<int, 2>{});
      else slabs(std::integral_constant<int, 0>{});
    } else {
      slabs(std::integral_constant<int, 0>{});
    }
    if (!has_next) break;
    pid = next;
  }
}

template <class CFG, bool AT, bool BT, int EPI>
static hipError_t launch_one(const GemmParams& p, hipStream_t s) {
  constexpr int BN_OUT = (EPI == EPI_SWIGLU_FWD) ? CFG::BN / 2 : CFG::BN;
  if (p.bn_out < 0 || p.bn_out > BN_OUT || (p.bn_out & 7)) return hipErrorInvalidValue;
  const long long bn_out = (CFG::BM <= 64 && p.bn_out > 0) ? p.bn_out : BN_OUT;  // as in the kernel
  const long long tiles_m = (p.M + CFG::BM - 1) / CFG::BM;
  const long long tiles_n = (p.N + bn_out - 1) / bn_out;
  const long long total = tiles_m * tiles_n * p.G;
  if (total <= 0 || total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  long long blocks = total;
  if (CFG::PERSIST) {
    static int n_cu = 0;  // as many workgroups as the compute units hold at once
    if (n_cu == 0) {
      int dev = 0, v = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return hipErrorInvalidValue;
      n_cu = v > 0 ? v : 256;
    }
    if (blocks > (long long)n_cu * CFG::WGS_PER_CU) blocks = (long long)n_cu * CFG::WGS_PER_CU;
  }
  hipLaunchKernelGGL((gemm_kernel<CFG, AT, BT, EPI>), dim3((unsigned)blocks), dim3(CFG::THREADS), 0, s, p);
  return hipGetLastError();
}

}  // namespace caat
