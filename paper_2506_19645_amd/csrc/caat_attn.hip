// Attention core of the partial-sync attention sub-block (Eq. A5, first line) for gfx950: rotary embedding of
// q and k in place, and causal softmax(q k^T / sqrt(d)) v per head with an online softmax (one pass over the keys,
// MFMA 32x32x16 bf16 for both contractions, fp32 scores / statistics / accumulators).  head_dim = 128.
//
// Work split: a workgroup of 4 waves owns 128 consecutive queries of one (rank, sequence, head); each wave owns
// 32 of them.  Keys / values are walked in blocks of 64: the K and V blocks go global -> LDS directly (double
// buffered), chunk-swizzled on the global side.  The forward kernel is software-pipelined inside a wave: the K ring
// runs one block ahead of the V ring, and the score MFMAs of block b+1 are issued interleaved, one per step, with the
// softmax arithmetic of block b (a wave issues in order, so what should run under an MFMA stands right behind it).  Scores are computed transposed (S^T = K q^T) so that a lane owns
// one query row: lane l holds, for query l%32, the keys 8*(r/4) + 4*(l/32) + r%4 of each 32-key tile in register r.
// Those registers, exponentiated and rounded to bf16, ARE the k-slices the second MFMA needs for P (the order
// of the contraction index inside an MFMA is free as long as both operands agree), and the matching V operand
// (4 consecutive keys of one head-dim column per read) comes from the LDS transpose read ds_read_b64_tr_b16.
#include <type_traits>
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// LDS pointers with a type (address space 3): reads through them are single ds_read instructions with immediate offsets
typedef __attribute__((address_space(3))) const u32x4_t* lds_u4_t;
typedef __attribute__((address_space(3))) const char* lds_c_t;
typedef __attribute__((address_space(3))) short4_t* lds_s4_t;

static constexpr unsigned OOB_OFF = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t attn_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)0x80000000, 0x00020000);
}

// ---------------------------------------------------------------------------------------------------------
// RoPE in place on the q and k column blocks of qkv [rows, ld] (row = rank*tokens + batch*seq + pos; the first
// n_rot heads of a row, i.e. the q heads then the k heads, are rotated, the v heads after them are not):
// pairs (j, j + d/2), angle pos * base^(-2j/d).  One thread owns 8 pairs (j = 8 grp .. 8 grp + 7) of one row and
// rotates them in every head: the angles depend on the position and on j, not on the head, so the 8 sines and cosines
// are computed once per thread (with a thread per head they were what the kernel spent its time on).
// sign = +1 rotates forward; sign = -1 applies the transpose of that rotation (its inverse), which is what the
// gradients of the rotated q and k need on their way back to the projection outputs.
__global__ __launch_bounds__(256) void rope_kernel(bf16_t* qkv, long long rows, int seq, int ld, int n_rot, int d,
                                                   float log2_base, long long pos0, float sign) {
  const int half = d >> 1;
  const int groups = half >> 3;                     // 8 pairs per thread
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * groups) return;
  const long long row = idx / groups;
  const int grp = (int)(idx - row * groups);
  const float pos = (float)(pos0 + row % seq);
  float sn[8], cs[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int j = grp * 8 + e;
    const float inv = exp2f(-2.0f * (float)j / (float)d * log2_base);
    sincosf(pos * inv, &sn[e], &cs[e]);
    sn[e] *= sign;
  }
  bf16_t* p = qkv + row * (long long)ld + grp * 8;  // q heads first, k heads right after them
  for (int head = 0; head < n_rot; ++head, p += d) {
    const uint4 lo = *reinterpret_cast<const uint4*>(p);
    const uint4 hi = *reinterpret_cast<const uint4*>(p + half);
    const unsigned lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
    unsigned ol[4], oh[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float x1[2] = {lo_bf(lw[w]), hi_bf(lw[w])}, x2[2] = {lo_bf(hw[w]), hi_bf(hw[w])};
      float y1[2], y2[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        y1[e] = x1[e] * cs[w * 2 + e] - x2[e] * sn[w * 2 + e];
        y2[e] = x2[e] * cs[w * 2 + e] + x1[e] * sn[w * 2 + e];
      }
      ol[w] = pack2bf(y1[0], y1[1]);
      oh[w] = pack2bf(y2[0], y2[1]);
    }
    *reinterpret_cast<uint4*>(p) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    *reinterpret_cast<uint4*>(p + half) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
  }
}

hipError_t launch_rope(bf16_t* qkv, long long rows, int seq, int ld, int n_rot, int d, float base, long long pos0,
                       bool inverse, hipStream_t s) {
  if (n_rot == 0) return hipSuccess;
  const long long work = rows * (long long)(d / 16);
  if (work == 0) return hipSuccess;
  const long long blocks = (work + 255) / 256;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, rows, seq, ld, n_rot, d, log2f(base),
                     pos0, inverse ? -1.0f : 1.0f);
  return hipGetLastError();
}

// RoPE on q and k in place and, in the same pass, the store of the rotated k and of v into the KV caches
// [n_seq][kvpr][cap][128] at positions pos0 .. pos0+seq-1 (the prompts of a prefill; a decode step does the same for
// its one token inside the attention kernel).  One thread
// rotates 8 pairs (j, j + d/2) of one q or k head of one token; the threads of a k head also write their two rotated
// chunks to the key cache and copy the matching two chunks of v to the value cache, so a k / v head is covered by
// its 8 threads.  d = 128 only (the cache rows are 128 wide).
__global__ __launch_bounds__(256) void rope_append_kernel(bf16_t* qkv, bf16_t* __restrict__ kc, bf16_t* __restrict__ vc,
                                                          long long rows, int seq, int hpr, int kvpr, float log2_base,
                                                          long long cap, long long pos0) {
  constexpr int d = 128, half = 64, groups_per_head = 8;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long per_row = (long long)(hpr + kvpr) * groups_per_head;
  if (idx >= rows * per_row) return;
  const long long row = idx / per_row;                 // sequence * seq + token
  const int rem = (int)(idx - row * per_row);
  const int head = rem / groups_per_head, grp = rem - head * groups_per_head;
  const long long sq = row / seq;
  const long long t = row - sq * seq;
  const float pos = (float)(pos0 + t);
  const long long ld = (long long)(hpr + 2 * kvpr) * d;
  bf16_t* p = qkv + row * ld + (long long)head * d + grp * 8;   // q heads first, k heads right after them
  const uint4 lo = *reinterpret_cast<const uint4*>(p);
  const uint4 hi = *reinterpret_cast<const uint4*>(p + half);
  const bool is_k = head >= hpr;
  uint4 vlo = make_uint4(0u, 0u, 0u, 0u), vhi = vlo;
  if (is_k) {                                                   // the v head sits kvpr heads after its k head
    vlo = *reinterpret_cast<const uint4*>(p + (long long)kvpr * d);
    vhi = *reinterpret_cast<const uint4*>(p + (long long)kvpr * d + half);
  }
  const unsigned lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
  unsigned ol[4], oh[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float x1[2] = {lo_bf(lw[w]), hi_bf(lw[w])}, x2[2] = {lo_bf(hw[w]), hi_bf(hw[w])}, y1[2], y2[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int j = grp * 8 + w * 2 + e;
      const float inv = exp2f(-2.0f * (float)j / (float)d * log2_base);
      float sn, cs;
      sincosf(pos * inv, &sn, &cs);
      y1[e] = x1[e] * cs - x2[e] * sn;
      y2[e] = x2[e] * cs + x1[e] * sn;
    }
    ol[w] = pack2bf(y1[0], y1[1]);
    oh[w] = pack2bf(y2[0], y2[1]);
  }
  const uint4 rlo = make_uint4(ol[0], ol[1], ol[2], ol[3]), rhi = make_uint4(oh[0], oh[1], oh[2], oh[3]);
  *reinterpret_cast<uint4*>(p) = rlo;
  *reinterpret_cast<uint4*>(p + half) = rhi;
  if (is_k) {
    const long long dst = ((sq * kvpr + (head - hpr)) * cap + pos0 + t) * d + grp * 8;
    // the caches are read by later decode steps, not by this layer's attention (which reads qkv): non-temporal stores
    st_stream(kc + dst, rlo);
    st_stream(kc + dst + half, rhi);
    st_stream(vc + dst, vlo);
    st_stream(vc + dst + half, vhi);
  }
}

hipError_t launch_rope_append(bf16_t* qkv, bf16_t* kc, bf16_t* vc, long long n_seq, int seq, int hpr, int kvpr, int d,
                              float base, long long cap, long long pos0, hipStream_t s) {
  if (d != 128 || pos0 < 0 || pos0 + seq > cap) return hipErrorInvalidValue;
  const long long work = n_seq * seq * (long long)(hpr + kvpr) * 8;
  if (work == 0) return hipSuccess;
  const long long blocks = (work + 255) / 256;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, kc, vc, n_seq * seq, seq, hpr, kvpr,
                     log2f(base), cap, pos0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
static constexpr int HD = 128;    // head dim
static constexpr int BQ = 128;    // queries per workgroup (32 per wave)
static constexpr int BKV = 64;    // keys per step
static constexpr int KCH = HD / 8;  // 16-byte chunks per K/V row

// Per-query attention statistics, fp32 [n_seq*heads][2][seq_pad] with seq_pad = seq rounded up to 64: row 0 of a
// (sequence, head) holds the forward's log2-domain log-sum-exp of the scaled scores, row 1 the backward's
// D = sum_d dO*O.  Entries seq .. seq_pad-1 are written as 0.
long long attn_seq_pad(int seq) { return ((long long)seq + 63) / 64 * 64; }
size_t attn_stats_bytes(long long n_seq, int heads, int seq) { return (size_t)(n_seq * heads * 2 * attn_seq_pad(seq)) * 4; }

// maximum of three finite-or-infinite values in one instruction (the scores are MFMA results or -inf, never NaN: no
// quieting of the inputs needed, which the generic fmaxf costs one extra instruction per operand)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// LDS chunk swizzles (chunk = 16 bytes of a 256-byte row): K is read as MFMA fragments (32 consecutive rows, one
// chunk) -> spread by row & 15; V is read by the transpose read (4 consecutive rows x 64 bytes) -> spread by row & 3.
__device__ __forceinline__ int kswz(int row, int c) { return c ^ (row & 15); }
__device__ __forceinline__ int vswz(int row, int c) { return c ^ ((row & 3) << 2); }

// Workgroup order of the attention kernels.  A launch covers n_bh (sequence, head) pairs x n_blk blocks whose cost grows
// with the block index (causal).  Heaviest blocks should start first, but the blocks of one head re-read that head's
// K / V (or Q / dO) rows, so all blocks of a head should also run close together in time: heads are taken in chunks of
// `chunk` (a multiple of 8, so that a head's blocks also land on one XCD and share its L2: workgroup b runs on XCD
// b % 8), and inside a chunk the order is heaviest block first, heads innermost.
// Returns the head index; `rank` = 0 for the heaviest block .. n_blk-1 for the lightest.
__device__ __forceinline__ int attn_block_order(int bid, int n_bh, int n_blk, int chunk, int& rank) {
  const int per_chunk = chunk * n_blk;
  const int c = bid / per_chunk;
  const int r = bid - c * per_chunk;
  const int first = c * chunk;
  const int size = min(chunk, n_bh - first);      // the last chunk may hold fewer heads
  rank = r / size;
  return first + (r - rank * size);
}
// chunk size: about 32 MB of K + V rows (seq x 512 bytes per head) per chunk, a multiple of 8, at least 8
static int attn_chunk_heads(int seq) {
  long long c = (32LL << 20) / ((long long)seq * 512);
  c = c / 8 * 8;
  if (c < 8) c = 8;
  if (c > 1024) c = 1024;
  return (int)c;
}

// qkv: [T*tokens, (heads + 2*kv_heads)*128] with q | k | v column blocks (q, k already rotated); out: [T*tokens, hd],
// hd = heads*128.  Query head a reads key / value head a / (heads / kv_heads) (grouped-query attention).
// stats (may be null): the forward fills the log-sum-exp rows (what the backward needs to rebuild the probabilities).
__global__ __launch_bounds__(256, 2) void flash_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                        float* __restrict__ stats, int seq, int seq_pad, int hd, int heads,
                                                        int kv_heads, int n_qblk, float scale_log2, int chunk) {
  __shared__ uint4 smem[4 * BKV * KCH];  // K slot 0, K slot 1, V slot 0, V slot 1: 64 rows x 16 chunks each = 64 KB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, hf = lane >> 5;
  // longest-first over the whole launch: the last (heaviest, causal) query blocks of every head come first
  const int n_bh = gridDim.x / n_qblk;
  int lpt_rank;
  const int bh = attn_block_order(blockIdx.x, n_bh, n_qblk, chunk, lpt_rank);   // (rank*batch + b) * heads + head
  const int qb = n_qblk - 1 - lpt_rank;          // the last (heaviest, causal) query blocks first
  const int head = bh % heads;
  const long long seq_row0 = (long long)(bh / heads) * seq;   // first row of this sequence in qkv
  const long long ld = (long long)(heads + 2 * kv_heads) * HD;
  const int q0 = qb * BQ;
  const bf16_t* qbase = qkv + seq_row0 * ld + (long long)head * HD;
  const bf16_t* kbase = qkv + seq_row0 * ld + hd + (long long)(head / (heads / kv_heads)) * HD;
  const bf16_t* vbase = kbase + kv_heads * HD;

  // ---- Q fragments: B operand of S^T = K q^T: lane (query frow, k-half hf) holds q[16*ks + 8*hf .. +7]
  bf16x8_t qf[HD / 16];
  const int qrow = q0 + wave * 32 + frow;
  {
    const __amdgpu_buffer_rsrc_t rs = attn_rsrc(qbase);
    const unsigned base_off = (qrow < seq) ? (unsigned)((long long)qrow * ld * 2 + hf * 16) : OOB_OFF;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
      const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(base_off == OOB_OFF ? OOB_OFF : base_off + ks * 32), 0, 0);
      qf[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
  }

  f32x16_t oacc[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[t][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;   // running max (raw score units) and this lane's share of the row sum

  const int kv_end = min(seq, q0 + BQ);                 // causal: keys 0 .. last query of the block
  const int nblk = (kv_end + BKV - 1) / BKV;

  // global -> LDS: a wave instruction fills 4 rows (64 lanes x 16 B); 64 rows = 16 instructions per tile, 4 per wave.
  // LDS: two K slots, then two V slots (one 64-row tile each).  The K ring runs one block ahead of the V ring: the
  // scores of block b+1 are computed while block b goes through the softmax (see the loop below).
  constexpr int TILE_BYTES = BKV * KCH * 16;
  unsigned dko[4], dvo[4];   // per-lane memory-side offsets of this wave's 4 copies of a tile (row, swizzled chunk)
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int rg = it * 4 + wave;                      // group of 4 rows
    const int row = rg * 4 + (lane >> 4), phys = lane & 15;
    dko[it] = (unsigned)((long long)row * ld * 2 + kswz(row, phys) * 16);
    dvo[it] = (unsigned)((long long)row * ld * 2 + vswz(row, phys) * 16);
  }
  auto issue_rows = [&](const bf16_t* base, const unsigned* off, int blk, int slot_tile) {
    const int kv0 = blk * BKV;
    const i32x4_t rs = make_rsrc(base + (long long)kv0 * ld);
    uint4* t = smem + slot_tile * (BKV * KCH);
    const bool whole = kv0 + BKV <= seq;               // all 64 rows exist (every block but the last of a ragged sequence)
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int rg = it * 4 + wave;
      const unsigned o = (whole || kv0 + rg * 4 + (lane >> 4) < seq) ? off[it] : OOB_OFF;
      dma16(rs, o, t + rg * 64);
    }
  };
  auto issue_k = [&](int blk) { issue_rows(kbase, dko, blk, blk & 1); };
  auto issue_v = [&](int blk) { issue_rows(vbase, dvo, blk, 2 + (blk & 1)); };

  // Per-lane LDS addresses of the fragment reads, fixed for the whole kernel: what changes from read to read (slot,
  // key tile, 16-key slice) is a compile-time constant that goes into the instruction's immediate offset, so the key loop
  // spends no vector ALU work on addresses (they were about a third of its vector instructions).
  //   K fragment (32 rows x one 16-byte chunk): row = 32 j + frow, logical chunk 2 ks + hf  -> koff[ks] + (slot, j) constant
  //   V transpose read: row = 16 u + 4 hf + (i16 >> 2) (+ 8), head-dim column 32 dt + 16 grp + 4 (i16 & 3) -> voff[dt] + constant
  lds_u4_t koff[HD / 16];
  lds_c_t voff[HD / 32];
  {
    const lds_c_t lds0 = (lds_c_t)smem;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) koff[ks] = (lds_u4_t)(lds0 + (frow * KCH + kswz(frow, ks * 2 + hf)) * 16);
    const int i16 = lane & 15, grp = (lane >> 4) & 1;
    const int vrow = 4 * hf + (i16 >> 2);
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt) {
      const int col = dt * 32 + grp * 16 + (i16 & 3) * 4;
      voff[dt] = lds0 + ((vrow * KCH + vswz(vrow, col >> 3)) * 16 + (col & 7) * 2);
    }
  }
  const f32x16_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t ones2 = {(__bf16)1.0f, (__bf16)1.0f};

  // S^T = K q^T for the 64 keys in K slot SLOT: 2 key tiles of 32, contraction over the head dim in 8 steps of 16 (the
  // first step starts from zero instead of clearing the accumulator first)
  auto scores = [&](f32x16_t* sacc, auto slot_c) {
    constexpr int SLOT = decltype(slot_c)::value;
#pragma unroll
    for (int j = 0; j < BKV / 32; ++j)
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) {
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, koff[ks][(SLOT * TILE_BYTES + j * 32 * KCH * 16) / 16]);
        sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? zero16 : sacc[j], 0, 0, 0);
      }
  };

  // One key block, software-pipelined inside the wave: the scores of block blk are already in `scur`; the matrix unit
  // works on the scores of block blk+1 (`snext`, from the other K slot) while the vector ALU takes block blk through the
  // online softmax; then the second product of block blk.  SLOT = blk & 1 (compile-time: the loop alternates two
  // instantiations, which also swaps the roles of the two score register sets without a copy).
  auto key_block = [&](int blk, f32x16_t* scur, f32x16_t* snext, auto slot_c, auto last_c) {
    constexpr int SLOT = decltype(slot_c)::value;
    constexpr bool LAST = decltype(last_c)::value;
    wait_vmcnt<0>();
    __syncthreads();                 // K(blk+1) and V(blk) have landed; everyone is done with K(blk) and V(blk-1)
    if (blk + 2 < nblk) issue_k(blk + 2);
    if (blk + 1 < nblk) issue_v(blk + 1);
    const int kv0 = blk * BKV;
    // ---- causal mask for query qrow (keys of register r: kv0 + 32j + 8(r/4) + 4hf + r%4); wave-uniform test: does
    // some key of this block exceed some query of this wave?  (only the last blocks of a tile)
    if ((kv0 + BKV - 1) > (q0 + wave * 32)) {
#pragma unroll
      for (int j = 0; j < BKV / 32; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + j * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key > qrow) scur[j][r] = -INFINITY;
        }
    }
    // ---- The instruction stream of the block is laid out by hand, one MFMA per step, with a scheduling fence after
    // every step (the compiler keeps the order of the steps and only arranges the few instructions inside one):
    // a wave issues in order, so whatever should run under an MFMA has to stand right behind it in the stream.
    //   steps 0-15 : score MFMAs of block blk+1 (fragments read three steps ahead); underneath: the row maximum of
    //                block blk (steps 0-3), its exchange with the other half-row (4-5), the exponentials of keys 0-31 (6-13)
    //   (rescale of the output accumulators, only if some row's maximum moved)
    //   steps 16-31: second-product MFMAs, 16-key slice by slice (V fragments read three steps ahead); underneath: the
    //                exponentials of keys 32-63 (steps 16-23), which only slices 2 and 3 need
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    auto kread = [&](int idx) -> u32x4_t {
      return koff[idx & 7][((SLOT ^ 1) * TILE_BYTES + (idx >> 3) * 32 * KCH * 16) / 16];
    };
    float mx = -INFINITY, mxo = 0.0f, m_new = 0.0f, alpha = 1.0f, mb = 0.0f, psum = 0.0f;
    unsigned pw[BKV / 2];               // the block's probabilities, bf16 pairs: pw[4 i .. 4 i + 3] = slice i's B operand
    auto prob_pair = [&](int i) {       // pair i: registers 2 i, 2 i + 1 of the 32 scores of this lane
      const int j = i >> 3, r = (i & 7) * 2;
      // arguments <= 0; tiny results flush to 0
      const float p0 = __builtin_amdgcn_exp2f(scur[j][r] * scale_log2 - mb);
      const float p1 = __builtin_amdgcn_exp2f(scur[j][r + 1] * scale_log2 - mb);
      pw[i] = pack2bf(p0, p1);
      // the row sum takes the probabilities as the second product sees them (rounded to bf16), two per instruction
      psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pw[i]), ones2, psum, false);
      // pins the pair to this place in the stream (the optimiser would otherwise sink it to its first use)
      asm volatile("" : "+v"(pw[i]), "+v"(psum));
    };
    u32x4_t kr[3];
    if constexpr (!LAST) {
      kr[0] = kread(0);
      kr[1] = kread(1);
      kr[2] = kread(2);
    }
    fence();
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) {
      if constexpr (!LAST) {
        const int j = idx >> 3, ks = idx & 7;
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, kr[idx % 3]);
        snext[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? zero16 : snext[j], 0, 0, 0);
        if (idx + 3 < 16) kr[idx % 3] = kread(idx + 3);
      }
      if (idx < 4) {                                    // row maximum: 8 of the lane's 32 scores per step
        const int j = idx >> 1, r0 = (idx & 1) * 8;
#pragma unroll
        for (int r = 0; r < 8; r += 2) mx = max3(mx, scur[j][r0 + r], scur[j][r0 + r + 1]);
        if (idx == 3) mxo = __shfl_xor(mx, 32, 64);    // the other half of the row lives in lane ^ 32
      } else if (idx == 5) {
        m_new = fmaxf(m_run, fmaxf(mx, mxo));           // finite: key 0 is visible to every query
        alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
        mb = m_new * scale_log2;
      } else if (idx >= 6 && idx < 14) {
        prob_pair(idx - 6);                             // keys 0-31 of the block: pairs 0-7; pairs 8-15 under the second product
      }
      fence();
    }
    // the running maximum settles after the first blocks: rescale the accumulators only if some row's maximum moved
    if (__any(m_new != m_run)) {
#pragma unroll
      for (int t = 0; t < HD / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
    }
    m_run = m_new;

    // ---- O^T += V^T P^T : A operand = V columns (head-dim index frow of tile dt), B operand = P (query frow).
    // k-slice u (16 keys) of the block: lane half hf contributes keys 16u + 4hf + {0..3} and 16u + 8 + 4hf + {0..3};
    // transpose read: input lane i of a 16-lane group supplies row (i/4), 8-byte column group (i%4); output lane j
    // receives column j of those 4 rows.  Step st: slice u = st / 4, head-dim tile dt = st % 4.
    typedef short short8_t __attribute__((ext_vector_type(8)));
    auto vread = [&](int st, short4_t& v0, short4_t& v1) {
      const lds_c_t a0 = voff[st & 3] + ((2 + SLOT) * TILE_BYTES + (st >> 2) * 16 * KCH * 16);
      v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)a0);
      v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)(a0 + 8 * KCH * 16));
    };
    short4_t va[3], vb[3];
    vread(0, va[0], vb[0]);
    vread(1, va[1], vb[1]);
    vread(2, va[2], vb[2]);
    fence();
#pragma unroll
    for (int st = 0; st < 16; ++st) {
      const int u = st >> 2, dt = st & 3;
      const short8_t vv = {va[st % 3][0], va[st % 3][1], va[st % 3][2], va[st % 3][3],
                           vb[st % 3][0], vb[st % 3][1], vb[st % 3][2], vb[st % 3][3]};
      const bf16x8_t pfu = __builtin_bit_cast(bf16x8_t, make_uint4(pw[4 * u], pw[4 * u + 1], pw[4 * u + 2], pw[4 * u + 3]));
      oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv), pfu, oacc[dt], 0, 0, 0);
      if (st + 3 < 16) vread(st + 3, va[st % 3], vb[st % 3]);
      if (st < 8) prob_pair(8 + st);                    // keys 32-63: needed from step 8 (slice 2) on
      fence();
    }
    l_run = l_run * alpha + psum;
  };

  // prologue: K(0) alone first (its scores open the pipeline), then K(1) and V(0) for the first loop iteration
  f32x16_t sa[BKV / 32], sb[BKV / 32];
  issue_k(0);
  wait_vmcnt<0>();
  __syncthreads();
  if (1 < nblk) issue_k(1);
  issue_v(0);
  scores(sa, std::integral_constant<int, 0>{});
  int blk = 0;
  for (; blk + 2 < nblk; blk += 2) {
    key_block(blk, sa, sb, std::integral_constant<int, 0>{}, std::false_type{});
    key_block(blk + 1, sb, sa, std::integral_constant<int, 1>{}, std::false_type{});
  }
  if (blk + 1 < nblk) {       // two blocks left
    key_block(blk, sa, sb, std::integral_constant<int, 0>{}, std::false_type{});
    key_block(blk + 1, sb, sa, std::integral_constant<int, 1>{}, std::true_type{});
  } else {                    // one block left
    key_block(blk, sa, sb, std::integral_constant<int, 0>{}, std::true_type{});
  }

  // ---- normalise and store: lane holds out[qrow][32dt + 8(r/4) + 4hf + r%4]
  l_run += __shfl_xor(l_run, 32, 64);
  if (stats != nullptr && hf == 0 && qrow < seq_pad)
    stats[(long long)bh * 2 * seq_pad + qrow] = qrow < seq ? m_run * scale_log2 + __log2f(l_run) : 0.0f;
  if (qrow < seq) {
    const float inv = 1.0f / l_run;
    bf16_t* o = out + (seq_row0 + qrow) * (long long)hd + (long long)head * HD;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 w;
        w.x = pack2bf(oacc[dt][q * 4 + 0] * inv, oacc[dt][q * 4 + 1] * inv);
        w.y = pack2bf(oacc[dt][q * 4 + 2] * inv, oacc[dt][q * 4 + 3] * inv);
        *reinterpret_cast<uint2*>(o + dt * 32 + q * 8 + hf * 4) = w;
      }
  }
}

// qkv [n_seq*seq, 3*hd] (q|k|v, rotated) -> out [n_seq*seq, hd]; n_seq = T*batch sequences, heads = hd / 128 per rank
hipError_t launch_flash_fwd(const bf16_t* qkv, bf16_t* out, float* stats, long long n_seq, int seq, int heads, int kv_heads,
                            int d, hipStream_t s) {
  if (d != HD || kv_heads < 1 || heads % kv_heads != 0) return hipErrorInvalidValue;
  const int hd = heads * HD;
  const int n_qblk = (seq + BQ - 1) / BQ;
  const long long blocks = n_seq * heads * n_qblk;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFLL || (long long)(seq + BKV) * (heads + 2 * kv_heads) * HD * 2 >= 0x7FFFFFFFLL)
    return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  hipLaunchKernelGGL(flash_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, out, stats, seq, (int)attn_seq_pad(seq), hd,
                     heads, kv_heads, n_qblk, scale_log2, attn_chunk_heads(seq));
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------
// Backward of the attention core (chain rule of Eq. A5's Attention(.)): with S = q k^T / sqrt(d) (causal),
// P = softmax(S), O = P v and D_i = sum_d dO_id O_id:
//   dV = P^T dO;  dP = dO V^T;  dS = P o (dP - D);  dQ = dS K / sqrt(d);  dK = dS^T Q / sqrt(d).
// P is rebuilt from the forward's log-sum-exp, never stored.  Two kernels, each without atomics so that every
// output element is summed in one fixed order: one owns a block of keys and walks the queries (dK, dV), the other
// owns a block of queries and walks the keys (dQ).  Both keep the "lane owns one row" register layout of the
// forward so that the exponentiated score registers are directly the k-slices of the next MFMA.
//
// LDS tiles here are read both as row fragments (32 consecutive rows, one 16-byte chunk) and through the transpose
// read (4 consecutive rows x 64 bytes), so the chunk swizzle spreads 16 consecutive rows over all 16 chunks AND 4
// consecutive rows over the four 64-byte groups.
__device__ __forceinline__ int fswz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// 8 consecutive bf16 of a tile row: chunk index c of row `row` ([rows][16 chunks], swizzled)
__device__ __forceinline__ bf16x8_t frag_rows(const uint4* tile, int row, int c) {
  return __builtin_bit_cast(bf16x8_t, tile[row * KCH + (c ^ fswz(row))]);
}
// A operand of X^T (X = tile [rows][128]): lane (l%32 = column 32*dt + l%32 of X) receives the 8 rows
// r16 + 4hf + {0..3} and r16 + 8 + 4hf + {0..3}, the order in which a lane's score registers run over rows
__device__ __forceinline__ bf16x8_t frag_cols(const uint4* tile, int dt, int r16, int lane) {
  const int i16 = lane & 15, grp = (lane >> 4) & 1, hf = lane >> 5;
  const int col = dt * 32 + grp * 16 + (i16 & 3) * 4;
  const char* base = reinterpret_cast<const char*>(tile);
  const int row0 = r16 + 4 * hf + (i16 >> 2), row1 = row0 + 8;
  const char* a0 = base + (row0 * KCH + ((col >> 3) ^ fswz(row0))) * 16 + (col & 7) * 2;
  const char* a1 = base + (row1 * KCH + ((col >> 3) ^ fswz(row1))) * 16 + (col & 7) * 2;
  const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)a0);
  const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)a1);
  typedef short short8_t __attribute__((ext_vector_type(8)));
  const short8_t vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
  return __builtin_bit_cast(bf16x8_t, vv);
}
// global -> LDS copy of a 64-row x 128-column tile (rows of `ld` elements starting at `src`, rows >= valid read
// as zero): a wave instruction fills 4 rows, 16 instructions per tile, 4 per wave
__device__ __forceinline__ void issue_tile64(const bf16_t* src, long long ld, int valid, uint4* tile, int wave, int lane) {
  const i32x4_t rs = make_rsrc(src);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int rg = it * 4 + wave;
    const int row = rg * 4 + (lane >> 4), phys = lane & 15;
    const unsigned off = row < valid ? (unsigned)((long long)row * ld * 2 + ((phys ^ fswz(row)) * 16)) : OOB_OFF;
    dma16(rs, off, tile + rg * 64);
  }
}
// 8 fragments (one row of 128, this lane's k-half) straight from global memory
__device__ __forceinline__ void load_row_frags(const bf16_t* base, long long ld, int row, bool valid, int hf, bf16x8_t* f) {
  const __amdgpu_buffer_rsrc_t rs = attn_rsrc(base);
  const unsigned base_off = valid ? (unsigned)((long long)row * ld * 2 + hf * 16) : OOB_OFF;
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(valid ? base_off + ks * 32 : OOB_OFF), 0, 0);
    f[ks] = __builtin_bit_cast(bf16x8_t, v);
  }
}
// Makes the compiler wait for these register loads HERE.  It counts the loads it knows of, not the global -> LDS copies
// issued from inline assembly: left alone it puts its waits (down to vmcnt(0)) in front of the first use of each
// fragment inside the key / query loop, where they wait in every iteration for the copies just issued for the next
// block -- the prefetch then covers nothing.
__device__ __forceinline__ void settle_row_frags(bf16x8_t* f) {
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks) asm volatile("" : "+v"(f[ks]));
}
__device__ __forceinline__ bf16x8_t pack8(const float* v) {
  const uint4 w = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
  return __builtin_bit_cast(bf16x8_t, w);
}

// Per-lane LDS addresses of the fragment reads of a [64 rows][16 chunks] tile at LDS offset 0, fixed for a whole
// kernel: which tile, which 32-row group or 16-row slice and which stage a read means is a constant added in the
// read's immediate offset (or, for the stage, one add per address register and block), so the loops over key / query
// blocks spend no vector ALU work on swizzled addresses.
//   row fragment (frag_rows): row 32 j + frow, logical chunk 2 ks + hf             -> rows[ks] + constant
//   transpose read (frag_cols): rows 16 u + 4 hf + (i16 >> 2) and + 8, column 32 dt + 16 grp + 4 (i16 & 3) -> cols0/1[dt] + constant
struct FragAddr {
  lds_u4_t rows[HD / 16];
  lds_c_t cols0[HD / 32], cols1[HD / 32];
  __device__ __forceinline__ void init(const uint4* smem, int lane) {
    const lds_c_t lds0 = (lds_c_t)smem;
    const int frow = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) rows[ks] = (lds_u4_t)(lds0 + (frow * KCH + ((ks * 2 + hf) ^ fswz(frow))) * 16);
    const int i16 = lane & 15, grp = (lane >> 4) & 1;
    const int row0 = 4 * hf + (i16 >> 2), row1 = row0 + 8;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt) {
      const int col = dt * 32 + grp * 16 + (i16 & 3) * 4;
      cols0[dt] = lds0 + ((row0 * KCH + ((col >> 3) ^ fswz(row0))) * 16 + (col & 7) * 2);
      cols1[dt] = lds0 + ((row1 * KCH + ((col >> 3) ^ fswz(row1))) * 16 + (col & 7) * 2);
    }
  }
  // the same addresses moved by `bytes` (a stage's offset)
  __device__ __forceinline__ FragAddr at(int bytes) const {
    FragAddr f;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) f.rows[ks] = (lds_u4_t)((lds_c_t)rows[ks] + bytes);
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt) f.cols0[dt] = cols0[dt] + bytes, f.cols1[dt] = cols1[dt] + bytes;
    return f;
  }
  // row fragment ks of the 32-row group whose first row lies `c` bytes into the addressed stage (c: compile-time)
  __device__ __forceinline__ bf16x8_t row_frag(int ks, int c) const { return __builtin_bit_cast(bf16x8_t, rows[ks][c / 16]); }
  // transposed fragment of head-dim tile dt of the 16-row slice whose first row lies `c` bytes into the stage
  __device__ __forceinline__ bf16x8_t col_frag(int dt, int c) const {
    typedef short short8_t __attribute__((ext_vector_type(8)));
    const short4_t v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)(cols0[dt] + c));
    const short4_t v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)(cols1[dt] + c));
    const short8_t vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    return __builtin_bit_cast(bf16x8_t, vv);
  }
};

// D rows of the statistics: D[query] = sum_d dO * O, fp32; 16 lanes per (row, head).
__global__ __launch_bounds__(256) void attn_bwd_prep_kernel(const bf16_t* __restrict__ dout, const bf16_t* __restrict__ out,
                                                            float* __restrict__ stats, long long n_seq, int seq, int seq_pad,
                                                            int hd, int heads) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int c = (int)(idx & 15);
  const long long item = idx >> 4;                         // (sequence * heads + head) * seq_pad + pos
  if (item >= n_seq * heads * seq_pad) return;
  const int pos = (int)(item % seq_pad);
  const long long sh = item / seq_pad;
  const int head = (int)(sh % heads);
  const long long sq = sh / heads;
  float acc = 0.0f;
  if (pos < seq) {
    const long long o = (sq * seq + pos) * (long long)hd + (long long)head * HD + c * 8;
    const uint4 a = *reinterpret_cast<const uint4*>(dout + o);
    const uint4 b = *reinterpret_cast<const uint4*>(out + o);
    acc = lo_bf(a.x) * lo_bf(b.x) + hi_bf(a.x) * hi_bf(b.x) + lo_bf(a.y) * lo_bf(b.y) + hi_bf(a.y) * hi_bf(b.y) +
          lo_bf(a.z) * lo_bf(b.z) + hi_bf(a.z) * hi_bf(b.z) + lo_bf(a.w) * lo_bf(b.w) + hi_bf(a.w) * hi_bf(b.w);
  }
  acc += __shfl_xor(acc, 1, 64);
  acc += __shfl_xor(acc, 2, 64);
  acc += __shfl_xor(acc, 4, 64);
  acc += __shfl_xor(acc, 8, 64);
  if (c == 0) stats[(sh * 2 + 1) * seq_pad + pos] = acc;
}

// ---- dQ: a workgroup owns 128 queries of one (sequence, head), a wave 32 of them (lane = query), keys in blocks of 64.
//   S^T = K q^T and dP^T = V dO^T (A operand = K / V row fragments from LDS, B operand = q / dO registers);
//   dS^T registers, rounded to bf16, are the B operand of dQ^T += K^T dS^T (A operand = transpose reads of K).
__global__ __launch_bounds__(256, 2) void flash_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                           const float* __restrict__ stats, bf16_t* __restrict__ dqkv, int seq,
                                                           int seq_pad, int hd, int heads, int kv_heads, int n_qblk,
                                                           float scale_log2, float scale, int chunk) {
  __shared__ uint4 smem[4 * BKV * KCH];  // K slot 0, K slot 1, V slot 0, V slot 1: 64 rows x 16 chunks each = 64 KB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, hf = lane >> 5;
  const int n_bh = gridDim.x / n_qblk;
  int lpt_rank;
  const int bh = attn_block_order(blockIdx.x, n_bh, n_qblk, chunk, lpt_rank);
  const int qb = n_qblk - 1 - lpt_rank;                      // heaviest (last) query blocks first
  const int head = bh % heads;
  const long long seq_row0 = (long long)(bh / heads) * seq;
  const long long ld = (long long)(heads + 2 * kv_heads) * HD;
  const int q0 = qb * BQ;
  const bf16_t* qbase = qkv + seq_row0 * ld + (long long)head * HD;
  const bf16_t* kbase = qkv + seq_row0 * ld + hd + (long long)(head / (heads / kv_heads)) * HD;
  const bf16_t* vbase = kbase + kv_heads * HD;
  const bf16_t* dobase = dout + seq_row0 * (long long)hd + (long long)head * HD;
  const int qrow = q0 + wave * 32 + frow;
  const bool qvalid = qrow < seq;

  bf16x8_t qf[HD / 16], dof[HD / 16];
  load_row_frags(qbase, ld, qrow, qvalid, hf, qf);
  load_row_frags(dobase, hd, qrow, qvalid, hf, dof);
  float my_lse = qvalid ? stats[(long long)bh * 2 * seq_pad + qrow] : 0.0f;
  float my_d = qvalid ? stats[((long long)bh * 2 + 1) * seq_pad + qrow] : 0.0f;
  settle_row_frags(qf);
  settle_row_frags(dof);
  asm volatile("" : "+v"(my_lse), "+v"(my_d));

  f32x16_t acc[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

  const int kv_end = min(seq, q0 + BQ);
  const int nblk = (kv_end + BKV - 1) / BKV;
  auto issue = [&](int blk, int stage) {
    const int kv0 = blk * BKV;
    uint4* kt = smem + stage * (2 * BKV * KCH);
    issue_tile64(kbase + (long long)kv0 * ld, ld, seq - kv0, kt, wave, lane);
    issue_tile64(vbase + (long long)kv0 * ld, ld, seq - kv0, kt + BKV * KCH, wave, lane);
  };
  FragAddr fa0;
  fa0.init(smem, lane);
  constexpr int TILE_BYTES = BKV * KCH * 16;               // stage = K tile, V tile
  const f32x16_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  issue(0, 0);
  for (int blk = 0; blk < nblk; ++blk) {
    const int stage = blk & 1;
    wait_vmcnt<0>();
    __syncthreads();
    if (blk + 1 < nblk) issue(blk + 1, stage ^ 1);
    const int kv0 = blk * BKV;
    if (kv0 > q0 + wave * 32 + 31) continue;               // wave-uniform: every key of the block is masked for this wave
    const bool diag = (kv0 + BKV - 1) > (q0 + wave * 32);  // wave-uniform: some key exceeds some query
    const FragAddr fa = fa0.at(stage * 2 * TILE_BYTES);
    // two instantiations: the compare-and-select per score exists only in the blocks at the diagonal
    auto key_block = [&](auto diag_c) {
      constexpr bool DIAG = decltype(diag_c)::value;
      bf16x8_t dsf[BKV / 16];
#pragma unroll
      for (int j = 0; j < BKV / 32; ++j) {
        f32x16_t sacc = zero16, pacc = zero16;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.row_frag(ks, j * 32 * KCH * 16), qf[ks], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.row_frag(ks, TILE_BYTES + j * 32 * KCH * 16), dof[ks], pacc, 0, 0, 0);
        }
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(sacc[r] * scale_log2 - my_lse);
          if constexpr (DIAG) {
            const int key = kv0 + j * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
            p = key > qrow ? 0.0f : p;
          }
          ds[r] = p * (pacc[r] - my_d);
        }
        dsf[j * 2 + 0] = pack8(ds);
        dsf[j * 2 + 1] = pack8(ds + 8);
      }
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int u = 0; u < BKV / 16; ++u)
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.col_frag(dt, u * 16 * KCH * 16), dsf[u], acc[dt], 0, 0, 0);
    };
    if (diag) key_block(std::true_type{});
    else key_block(std::false_type{});
  }
  // lane holds dQ[qrow][32dt + 8(r/4) + 4hf + r%4]
  if (qvalid) {
    bf16_t* o = dqkv + (seq_row0 + qrow) * ld + (long long)head * HD;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 w;
        w.x = pack2bf(acc[dt][q * 4 + 0] * scale, acc[dt][q * 4 + 1] * scale);
        w.y = pack2bf(acc[dt][q * 4 + 2] * scale, acc[dt][q * 4 + 3] * scale);
        *reinterpret_cast<uint2*>(o + dt * 32 + q * 8 + hf * 4) = w;
      }
  }
}

// ---- dK, dV: a workgroup owns 128 keys of one (sequence, head), a wave 32 of them (lane = key), queries in blocks of 64
// from the diagonal to the end of the sequence.  S = Q k^T and dP = dO v^T (A operand = Q / dO row fragments from LDS,
// B operand = k / v registers); the P and dS registers, rounded to bf16, are the B operands of dV^T += dO^T P and
// dK^T += Q^T dS (A operands = transpose reads of the same dO and Q tiles).  The per-query lse and D of the block sit
// next to the tiles in LDS: lane registers run over queries here.
static constexpr int BQB = 64;                              // queries per step of the dK/dV kernel
static constexpr int DKV_STAGE = 2 * BQB * KCH + 64;        // uint4 per stage: Q tile, dO tile, 1 KB of statistics

__global__ __launch_bounds__(256) void flash_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                            const float* __restrict__ stats, bf16_t* __restrict__ dqkv, int seq,
                                                            int seq_pad, int hd, int heads, int kv_heads, int n_kblk,
                                                            float scale_log2, float scale, int chunk) {
  __shared__ uint4 smem[2 * DKV_STAGE];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, hf = lane >> 5;
  const int n_bh = gridDim.x / n_kblk;                        // sequences x key/value heads
  int kb;                                                     // heaviest (first) key blocks first
  const int bh = attn_block_order(blockIdx.x, n_bh, n_kblk, chunk, kb);
  const int kvh = bh % kv_heads;
  const int grp = heads / kv_heads;                           // query heads that read this key / value head
  const long long sq = bh / kv_heads;
  const long long seq_row0 = sq * seq;
  const long long ld = (long long)(heads + 2 * kv_heads) * HD;
  const int k0 = kb * 128;
  const int kw0 = k0 + wave * 32;
  const int krow = kw0 + frow;
  const bool kvalid = krow < seq;
  const bf16_t* qbase = qkv + seq_row0 * ld + (long long)(kvh * grp) * HD;             // first query head of the group
  const bf16_t* kbase = qkv + seq_row0 * ld + hd + (long long)kvh * HD;
  const bf16_t* vbase = kbase + kv_heads * HD;
  const bf16_t* dobase = dout + seq_row0 * (long long)hd + (long long)(kvh * grp) * HD;
  const float* stats_bh = stats + (sq * heads + kvh * grp) * 2 * seq_pad;              // lse row, then D row, per query head

  bf16x8_t kf[HD / 16], vf[HD / 16];
  load_row_frags(kbase, ld, krow, kvalid, hf, kf);
  load_row_frags(vbase, ld, krow, kvalid, hf, vf);
  settle_row_frags(kf);
  settle_row_frags(vf);

  f32x16_t dk[HD / 32], dv[HD / 32];
#pragma unroll
  for (int t = 0; t < HD / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[t][r] = 0.0f, dv[t][r] = 0.0f;

  const int nqb = (seq + BQB - 1) / BQB;
  const int qb0 = k0 / BQB;
  const int nq = nqb - qb0;                                  // query blocks per query head (>= 1: k0 < seq)
  // walk: query head of the group (outer), query block (inner)
  // global -> LDS copies of a block (query head g of the group, query block qblk): per-lane memory-side offsets are
  // fixed for the kernel, a block only moves the two base addresses
  unsigned qo[4], doo[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int row = (c * 4 + wave) * 4 + (lane >> 4), phys = lane & 15;
    qo[c] = (unsigned)((long long)row * ld * 2 + ((phys ^ fswz(row)) * 16));
    doo[c] = (unsigned)((long long)row * hd * 2 + ((phys ^ fswz(row)) * 16));
  }
  const unsigned so = lane < 32 ? (unsigned)(((lane >> 4) * seq_pad + 4 * (lane & 15)) * 4) : OOB_OFF;
  auto issue = [&](int g, int qblk, int stage) {
    const int q0 = qblk * BQB;
    const bool whole = q0 + BQB <= seq;                      // all 64 query rows exist (every block but a ragged last one)
    const i32x4_t rq = make_rsrc(qbase + (long long)g * HD + (long long)q0 * ld);
    const i32x4_t rd = make_rsrc(dobase + (long long)g * HD + (long long)q0 * hd);
    uint4* qt = smem + stage * DKV_STAGE;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int rg = c * 4 + wave;
      const bool ok = whole || q0 + rg * 4 + (lane >> 4) < seq;   // rows past the sequence read as zero
      dma16(rq, ok ? qo[c] : OOB_OFF, qt + rg * 64);
      dma16(rd, ok ? doo[c] : OOB_OFF, qt + BQB * KCH + rg * 64);
    }
    if (wave == 0) {
      // lanes 0..15: lse of queries q0 + 4*lane .. +3; lanes 16..31: D likewise; the rest reads zeros.
      // q0 + 63 < seq_pad always, so the 16-byte pieces stay inside this (sequence, head)'s rows of statistics.
      const i32x4_t rs = make_rsrc(stats_bh + (long long)g * 2 * seq_pad + q0);
      dma16(rs, so, qt + 2 * BQB * KCH);
    }
  };
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) const f32x4_t* lds_f4_t;
  constexpr int TILE_BYTES = BQB * KCH * 16, STAGE_BYTES = DKV_STAGE * 16;   // stage = Q tile, dO tile, statistics
  FragAddr fa0;
  fa0.init(smem, lane);
  const lds_f4_t soff = (lds_f4_t)((lds_c_t)smem + 2 * TILE_BYTES + hf * 16);
  const f32x16_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  // A block of 64 queries none of which is masked for this wave (every block of the walk but the one or two at the
  // diagonal), both 32-query tiles in one hand-laid instruction stream: a wave issues in order and is alone on its
  // SIMD here, so the vector work of one tile has to stand right behind the MFMAs of the other to run under them.
  //   steps  0-15: S and dP of tile 0 (row fragments read three steps ahead)
  //   steps 16-31: S and dP of tile 1; underneath: P and dS of tile 0, one query per step
  //   steps 32-47: dV += dO^T P, dK += Q^T dS of tile 0 (transpose reads three steps ahead); underneath: P, dS of tile 1
  //   steps 48-63: the same products of tile 1
  // Every accumulator sees its MFMAs in the order of the tile-by-tile code below, so the two give the same bits.
  auto full_block = [&](int stage) {
    const FragAddr fa = fa0.at(stage * STAGE_BYTES);       // one add per address register and block
    const lds_f4_t scur = (lds_f4_t)((lds_c_t)soff + stage * STAGE_BYTES);
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    auto rread = [&](int idx) -> u32x4_t {   // idx 0..31: tile idx / 16, head-dim slice (idx % 16) / 2, Q (even) or dO (odd)
      return fa.rows[(idx & 15) >> 1][((idx & 1) * TILE_BYTES + (idx >> 4) * 32 * KCH * 16) / 16];
    };
    // idx 0..31: tile idx / 16, 16-query slice (idx % 16) / 8, head-dim tile (idx % 8) / 2, dO (even) or Q (odd)
    auto cread = [&](int idx, short4_t& v0, short4_t& v1) {
      const int dt = (idx & 7) >> 1;
      const int c = ((idx & 1) ? 0 : TILE_BYTES) + ((idx >> 4) * 32 + ((idx & 15) >> 3) * 16) * KCH * 16;
      v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)(fa.cols0[dt] + c));
      v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_t)(fa.cols1[dt] + c));
    };
    f32x16_t sc[2], dp[2];
    unsigned pw[2][8], dw[2][8];      // P and dS of the two tiles as bf16 pairs: words 4 t .. 4 t + 3 = slice t's B operand
    f32x4_t l4[4], d4[4];             // lse and D of the 16 queries of this lane's registers
    auto stats = [&](int j, int i) {  // query group i of tile j
      l4[i] = scur[8 * j + 2 * i];
      d4[i] = scur[16 + 8 * j + 2 * i];
    };
    // P and dS of registers 2k, 2k+1 of tile j over two steps, so that the two chains of a step are independent of each
    // other and a step's results are first used a step later (nothing waits on the exponential it has just issued)
    float e0 = 0.0f, e1 = 0.0f, t0 = 0.0f, t1 = 0.0f;
    auto prob = [&](int j, int step) {
      const int k = step >> 1, r = 2 * k;
      if ((step & 1) == 0) {
        e0 = __builtin_amdgcn_exp2f(sc[j][r] * scale_log2 - l4[r >> 2][r & 3]);
        e1 = __builtin_amdgcn_exp2f(sc[j][r + 1] * scale_log2 - l4[r >> 2][(r & 3) + 1]);
        t0 = dp[j][r] - d4[r >> 2][r & 3];
        t1 = dp[j][r + 1] - d4[r >> 2][(r & 3) + 1];
        asm volatile("" : "+v"(e0), "+v"(e1), "+v"(t0), "+v"(t1));      // pins the work to this step
      } else {
        pw[j][k] = pack2bf(e0, e1);
        dw[j][k] = pack2bf(e0 * t0, e1 * t1);
        asm volatile("" : "+v"(pw[j][k]), "+v"(dw[j][k]));
      }
    };
    u32x4_t fr[3];
    fr[0] = rread(0);
    fr[1] = rread(1);
    fr[2] = rread(2);
    fence();
    short4_t va[3], vb[3];
#pragma unroll
    for (int idx = 0; idx < 32; ++idx) {
      const int j = idx >> 4, ks = (idx & 15) >> 1;
      const bf16x8_t f = __builtin_bit_cast(bf16x8_t, fr[idx % 3]);
      if (idx & 1)
        dp[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, vf[ks], ks == 0 ? zero16 : dp[j], 0, 0, 0);
      else
        sc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, kf[ks], ks == 0 ? zero16 : sc[j], 0, 0, 0);
      if (idx + 3 < 32) fr[idx % 3] = rread(idx + 3);
      else cread(idx + 3 - 32, va[(idx + 3) % 3], vb[(idx + 3) % 3]);   // the ring goes on into the transpose reads
      if (idx >= 12 && idx < 16) stats(0, idx - 12);
      if (idx >= 16) prob(0, idx - 16);
      fence();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) stats(1, i);
    fence();
    typedef short short8_t __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int idx = 0; idx < 32; ++idx) {
      const int j = idx >> 4, t = (idx & 15) >> 3, dt = (idx & 7) >> 1;
      const int sl = (idx + 32) % 3;
      const short8_t vv = {va[sl][0], va[sl][1], va[sl][2], va[sl][3], vb[sl][0], vb[sl][1], vb[sl][2], vb[sl][3]};
      const bf16x8_t a = __builtin_bit_cast(bf16x8_t, vv);
      if (idx & 1) {
        const bf16x8_t b = __builtin_bit_cast(bf16x8_t, make_uint4(dw[j][4 * t], dw[j][4 * t + 1], dw[j][4 * t + 2], dw[j][4 * t + 3]));
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, dk[dt], 0, 0, 0);
      } else {
        const bf16x8_t b = __builtin_bit_cast(bf16x8_t, make_uint4(pw[j][4 * t], pw[j][4 * t + 1], pw[j][4 * t + 2], pw[j][4 * t + 3]));
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, dv[dt], 0, 0, 0);
      }
      if (idx + 3 < 32) cread(idx + 3, va[sl], vb[sl]);
      if (idx < 16) prob(1, idx);
      fence();
    }
  };

  // a block at the diagonal, tile by tile: a tile may be skipped (all its queries precede this wave's keys) or masked
  auto diag_block = [&](int q0, int stage) {
    const uint4* qt = smem + stage * DKV_STAGE;
    const uint4* dot = qt + BQB * KCH;
    const float4* st = reinterpret_cast<const float4*>(qt + 2 * BQB * KCH);
    // scores and dP of one 32-query tile: 16 MFMAs over the head dim
    auto scores = [&](int j, f32x16_t& sacc, f32x16_t& pacc) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.0f, pacc[r] = 0.0f;
      const int row = j * 32 + frow;
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(qt, row, ks * 2 + hf), kf[ks], sacc, 0, 0, 0);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(dot, row, ks * 2 + hf), vf[ks], pacc, 0, 0, 0);
      }
    };
    // P = exp2(S*c - lse), dS = P o (dP - D), both rounded to bf16 as the next MFMAs' B operands.
    // register r <-> query qs + 8(r/4) + 4hf + r%4, lane <-> key krow; masked (key > query) only where MASK
    auto probs = [&](int j, bool mask, const f32x16_t& sacc, const f32x16_t& pacc, bf16x8_t* pf, bf16x8_t* df) {
      const int qs = q0 + j * 32;
      float pv[16], ds[16];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 l4 = st[8 * j + 2 * i + hf];
        const float4 d4 = st[16 + 8 * j + 2 * i + hf];
        const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * i + e;
          float p = __builtin_amdgcn_exp2f(sacc[r] * scale_log2 - ls[e]);
          if (mask) {
            const int q = qs + 8 * i + 4 * hf + e;
            p = krow > q ? 0.0f : p;
          }
          pv[r] = p;
          ds[r] = p * (pacc[r] - dd[e]);
        }
      }
      pf[0] = pack8(pv);
      pf[1] = pack8(pv + 8);
      df[0] = pack8(ds);
      df[1] = pack8(ds + 8);
    };
    // dV^T += dO^T P and dK^T += Q^T dS for one 32-query tile: 16 MFMAs, A operands by transpose reads
    auto accumulate = [&](int j, const bf16x8_t* pf, const bf16x8_t* df) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int dt = 0; dt < HD / 32; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(dot, dt, j * 32 + t * 16, lane), pf[t], dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(qt, dt, j * 32 + t * 16, lane), df[t], dk[dt], 0, 0, 0);
        }
    };
#pragma unroll
    for (int j = 0; j < BQB / 32; ++j) {
      const int qs = q0 + j * 32;
      if (qs + 31 < kw0) continue;                           // wave-uniform: all 32 queries precede this wave's keys
      f32x16_t sacc, pacc;
      bf16x8_t pf[2], df[2];
      scores(j, sacc, pacc);
      probs(j, qs < kw0 + 31, sacc, pacc, pf, df);           // wave-uniform: some key exceeds some query
      accumulate(j, pf, df);
    }
  };
  // block it has landed and everyone is done with block it - 1: fetch block it + 1 = (query head ng, query block nb)
  auto next_stage = [&](int it, int ng, int nb) {
    wait_vmcnt<0>();
    __syncthreads();
    if (ng < grp) issue(ng, nb, (it + 1) & 1);
  };
  issue(0, qb0, 0);
  int it = 0;
  for (int g = 0; g < grp; ++g) {
    // the first two blocks of a query head's walk (128 queries = the workgroup's keys) touch the diagonal for some wave;
    // from the third on no wave has a masked or skipped query, and every wave takes the fused two-tile stream
    int b = 0;
    for (; b < 2 && b < nq; ++b, ++it) {
      const bool last = b + 1 == nq;
      next_stage(it, last ? g + 1 : g, last ? qb0 : qb0 + b + 1);
      diag_block((qb0 + b) * BQB, it & 1);
    }
    for (; b < nq; ++b, ++it) {
      const bool last = b + 1 == nq;
      next_stage(it, last ? g + 1 : g, last ? qb0 : qb0 + b + 1);
      full_block(it & 1);
    }
  }
  // lane holds dK[krow][32dt + 8(r/4) + 4hf + r%4] and dV likewise
  if (kvalid) {
    bf16_t* ok = dqkv + (seq_row0 + krow) * ld + hd + (long long)kvh * HD;
    bf16_t* ov = ok + kv_heads * HD;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 w;
        w.x = pack2bf(dk[dt][q * 4 + 0] * scale, dk[dt][q * 4 + 1] * scale);
        w.y = pack2bf(dk[dt][q * 4 + 2] * scale, dk[dt][q * 4 + 3] * scale);
        *reinterpret_cast<uint2*>(ok + dt * 32 + q * 8 + hf * 4) = w;
        w.x = pack2bf(dv[dt][q * 4 + 0], dv[dt][q * 4 + 1]);
        w.y = pack2bf(dv[dt][q * 4 + 2], dv[dt][q * 4 + 3]);
        *reinterpret_cast<uint2*>(ov + dt * 32 + q * 8 + hf * 4) = w;
      }
  }
}

// Backward of the attention core for every (sequence, head): qkv (rotated q | k | v), out = forward output, dout its
// gradient, stats with the forward's lse rows -> dqkv (gradients w.r.t. the ROTATED q, k and w.r.t. v, same layout
// as qkv).  The D rows of stats are filled here.
hipError_t launch_flash_bwd(const bf16_t* qkv, const bf16_t* out, const bf16_t* dout, float* stats, bf16_t* dqkv,
                            long long n_seq, int seq, int heads, int kv_heads, int d, hipStream_t s) {
  if (d != HD || kv_heads < 1 || heads % kv_heads != 0) return hipErrorInvalidValue;
  const int hd = heads * HD;
  const long long n_bh = n_seq * heads;
  if (n_bh == 0 || seq == 0) return hipSuccess;
  const int seq_pad = (int)attn_seq_pad(seq);
  const int n_qblk = (seq + BQ - 1) / BQ;
  if (n_bh * n_qblk > 0x7FFFFFFFLL || (long long)(seq + 128) * (heads + 2 * kv_heads) * HD * 2 >= 0x7FFFFFFFLL)
    return hipErrorInvalidValue;
  const float inv_sqrt_d = 1.0f / sqrtf((float)d);
  const float scale_log2 = 1.4426950408889634f * inv_sqrt_d;
  const long long prep_threads = n_bh * seq_pad * 16;
  if ((prep_threads + 255) / 256 > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_bwd_prep_kernel, dim3((unsigned)((prep_threads + 255) / 256)), dim3(256), 0, s, dout, out, stats, n_seq,
                     seq, seq_pad, hd, heads);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(flash_bwd_dkv_kernel, dim3((unsigned)(n_seq * kv_heads * n_qblk)), dim3(256), 0, s, qkv, dout, stats, dqkv,
                     seq, seq_pad, hd, heads, kv_heads, n_qblk, scale_log2, inv_sqrt_d, attn_chunk_heads(seq));
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(flash_bwd_dq_kernel, dim3((unsigned)(n_bh * n_qblk)), dim3(256), 0, s, qkv, dout, stats, dqkv, seq, seq_pad,
                     hd, heads, kv_heads, n_qblk, scale_log2, inv_sqrt_d, attn_chunk_heads(seq));
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------
// Decode: one new token per sequence at position kv_len: attention of its single query over the kv_len cached keys
// and its own.  Pure streaming (the KV read is the layer's dominant HBM traffic), so there is no MFMA here: a workgroup
// owns one (rank, sequence, head); 16 lanes own one key row (256 B), a wave takes 4 consecutive keys per step, the 4
// waves 16; every 16-lane group runs its own online softmax and the 16 partial results are merged through LDS in a
// fixed order.
// ROPE: the kernel also does what the RoPE + append kernel would have done for this token (one launch less per decode
// step): qkv holds the UN-rotated projections; q and the new k are rotated here for position nkeys - 1 (rounded to
// bf16 exactly as that kernel stores them), the new k and v take part in the attention from registers, keys
// 0 .. nkeys-2 are streamed from the caches, and the first query head of every key / value group writes the new rows
// into the caches for later steps.  Nobody reads cache row nkeys - 1 in this launch.
template <bool ROPE>
__global__ __launch_bounds__(256) void decode_attn_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ kc,
                                                          bf16_t* __restrict__ vc, bf16_t* __restrict__ out, int hpr,
                                                          int kvpr, long long cap, int nkeys, float scale_log2,
                                                          float log2_base) {
  __shared__ float s_acc[16][128];
  __shared__ float s_m[16], s_l[16];
  __shared__ float s_cs[64], s_sn[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  const long long sh = blockIdx.x;                 // seq * hpr + head
  const long long sq = sh / hpr;
  const int head = (int)(sh - sq * hpr);
  const int grp = hpr / kvpr;
  const long long kvh = sq * kvpr + head / grp;    // grouped-query attention: the group's cache rows
  const __amdgpu_buffer_rsrc_t rk = attn_rsrc(kc + kvh * cap * 128);
  const __amdgpu_buffer_rsrc_t rv = attn_rsrc(vc + kvh * cap * 128);
  const int ncache = ROPE ? nkeys - 1 : nkeys;     // keys that come from the caches
  constexpr int UN = 4;   // loads per lane and stream in flight; 2 and 8 measured the same (319 - 321 us at batch 64, 2048 keys)
  u32x4_t kv[UN], vv[UN];
  auto fetch = [&](int key0) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int key = key0 + 16 * u;
      const unsigned off = key < ncache ? (unsigned)key * 256u + c * 16 : OOB_OFF;
      // read-once stream: the non-temporal hint (cache policy bit 1) measured 7.1 TB/s against 6.2 TB/s for plain
      // loads on a 2 GiB read with this access pattern
      kv[u] = __builtin_amdgcn_raw_buffer_load_b128(rk, (int)off, 0, 2);
      vv[u] = __builtin_amdgcn_raw_buffer_load_b128(rv, (int)off, 0, 2);
    }
  };
  int key0 = wave * 4 + g;
  fetch(key0);                                     // the first keys are on their way while q is prepared
  const bf16_t* row = qkv + sq * (long long)(hpr + 2 * kvpr) * 128;
  float q[8];
  uint4 knew = make_uint4(0u, 0u, 0u, 0u), vnew = knew;   // the token's own key (rotated) and value, 8 dims per lane
  {
    uint4 w = *reinterpret_cast<const uint4*>(row + (long long)head * 128 + c * 8);
    if constexpr (ROPE) {
      const uint4 kw = *reinterpret_cast<const uint4*>(row + (long long)(hpr + head / grp) * 128 + c * 8);
      vnew = *reinterpret_cast<const uint4*>(row + (long long)(hpr + kvpr + head / grp) * 128 + c * 8);
      // angle j of the position, j = 0 .. 63, once per workgroup (the same expressions as the RoPE + append kernel)
      if (tid < 64) {
        const float inv = exp2f(-2.0f * (float)tid / 128.0f * log2_base);
        float sn, cs;
        sincosf((float)(nkeys - 1) * inv, &sn, &cs);
        s_cs[tid] = cs;
        s_sn[tid] = sn;
      }
      __syncthreads();
      // lanes c < 8 hold dims 8c .. 8c+7 (x1 of the pairs), lanes c >= 8 the dims 64 further on (x2): partner = lane ^ 8
      auto rotate = [&](const uint4& v) -> uint4 {
        const unsigned own[4] = {v.x, v.y, v.z, v.w};
        unsigned res[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned oth = (unsigned)__shfl_xor((int)own[i], 8, 64);
          float y[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int j = (c & 7) * 8 + i * 2 + e;
            const float mine = e ? hi_bf(own[i]) : lo_bf(own[i]), theirs = e ? hi_bf(oth) : lo_bf(oth);
            const float cs = s_cs[j], sn = s_sn[j];
            y[e] = c < 8 ? mine * cs - theirs * sn : mine * cs + theirs * sn;
          }
          res[i] = pack2bf(y[0], y[1]);
        }
        return make_uint4(res[0], res[1], res[2], res[3]);
      };
      w = rotate(w);
      knew = rotate(kw);
      if (head % grp == 0 && wave == 0 && g == 0) {          // one 16-lane group writes the 256-byte rows
        const long long dst = (kvh * cap + (nkeys - 1)) * 128 + c * 8;
        st_stream(kc + dst, knew);
        st_stream(vc + dst, vnew);
      }
    }
    q[0] = lo_bf(w.x); q[1] = hi_bf(w.x); q[2] = lo_bf(w.y); q[3] = hi_bf(w.y);
    q[4] = lo_bf(w.z); q[5] = hi_bf(w.z); q[6] = lo_bf(w.w); q[7] = hi_bf(w.w);
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] *= scale_log2;
  }
  float m = -INFINITY, l = 0.0f, acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  // one key: score of the 16-lane group, online-softmax update with its value row
  auto take = [&](const u32x4_t& kx, const u32x4_t& vx, bool valid) {
    float s = q[0] * lo_bf(kx.x) + q[1] * hi_bf(kx.x) + q[2] * lo_bf(kx.y) + q[3] * hi_bf(kx.y) +
              q[4] * lo_bf(kx.z) + q[5] * hi_bf(kx.z) + q[6] * lo_bf(kx.w) + q[7] * hi_bf(kx.w);
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    s += __shfl_xor(s, 4, 64);
    s += __shfl_xor(s, 8, 64);
    const float m_new = valid ? fmaxf(m, s) : m;
    const float alpha = valid ? exp2f(m - m_new) : 1.0f;     // m = -inf on the first key: exp2(-inf) = 0
    const float p = valid ? exp2f(s - m_new) : 0.0f;
    l = l * alpha + p;
    const unsigned w[4] = {vx.x, vx.y, vx.z, vx.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] = acc[2 * e] * alpha + p * lo_bf(w[e]);
      acc[2 * e + 1] = acc[2 * e + 1] * alpha + p * hi_bf(w[e]);
    }
    m = m_new;
  };
  while (key0 < ncache) {
    u32x4_t kcur[UN], vcur[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) kcur[u] = kv[u], vcur[u] = vv[u];
    const int k0 = key0;
    key0 += 16 * UN;
    if (key0 < ncache) fetch(key0);
#pragma unroll
    for (int u = 0; u < UN; ++u) take(kcur[u], vcur[u], (k0 + 16 * u) < ncache);
  }
  if constexpr (ROPE) {
    // the token's own key and value: one stream takes them (the same for every workgroup: a fixed order of summation)
    const u32x4_t kx = {knew.x, knew.y, knew.z, knew.w}, vx = {vnew.x, vnew.y, vnew.z, vnew.w};
    take(kx, vx, wave == 0 && g == 0);
  }
  const int stream = wave * 4 + g;
#pragma unroll
  for (int e = 0; e < 8; ++e) s_acc[stream][c * 8 + e] = acc[e];
  if (c == 0) {
    s_m[stream] = m;
    s_l[stream] = l;
  }
  __syncthreads();
  if (tid < 128) {
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) M = fmaxf(M, s_m[i]);
    float num = 0.0f, den = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float w = (s_m[i] == -INFINITY) ? 0.0f : exp2f(s_m[i] - M);
      num += s_acc[i][tid] * w;
      den += s_l[i] * w;
    }
    out[sh * 128 + tid] = f2bf(num / den);
  }
}

// out [n_seq, hpr*128] = softmax(q K^T / sqrt(d)) V over keys 0 .. nkeys-1 of caches [n_seq][kvpr][cap][128].
// rope_base > 0: qkv holds the un-rotated projections of the token at position nkeys - 1; the kernel rotates q and k,
// uses the new key / value from registers and stores them at cache row nkeys - 1 (no RoPE + append launch needed).
// rope_base = 0: q is rotated already and all nkeys keys are in the caches.
hipError_t launch_decode_attn(const bf16_t* qkv, bf16_t* kc, bf16_t* vc, bf16_t* out, long long n_seq, int hpr,
                              int kvpr, int d, long long cap, long long nkeys, float rope_base, hipStream_t s) {
  if (d != HD || kvpr < 1 || hpr % kvpr != 0 || nkeys < 1 || nkeys > cap || cap * 256 >= 0x7FFFFFFFLL)
    return hipErrorInvalidValue;
  const long long blocks = n_seq * hpr;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  if (rope_base > 0.0f)
    hipLaunchKernelGGL(decode_attn_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, qkv, kc, vc, out, hpr, kvpr, cap,
                       (int)nkeys, scale_log2, log2f(rope_base));
  else
    hipLaunchKernelGGL(decode_attn_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, qkv, kc, vc, out, hpr, kvpr, cap,
                       (int)nkeys, scale_log2, 0.0f);
  return hipGetLastError();
}

}  // namespace caat
