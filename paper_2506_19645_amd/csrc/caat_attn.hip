// Attention core of the partial-sync attention sub-block (Eq. A5, first line) for gfx950: rotary embedding of
// q and k in place, and causal softmax(q k^T / sqrt(d)) v per head with an online softmax (one pass over the keys,
// MFMA 32x32x16 bf16 for both contractions, fp32 scores / statistics / accumulators).  head_dim = 128.
//
// Work split: a workgroup of 4 waves owns 128 consecutive queries of one (rank, sequence, head); each wave owns
// 32 of them.  Keys / values are walked in blocks of 64: the K and V blocks go global -> LDS directly (double
// buffered), chunk-swizzled on the global side.  Scores are computed transposed (S^T = K q^T) so that a lane owns
// one query row: lane l holds, for query l%32, the keys 8*(r/4) + 4*(l/32) + r%4 of each 32-key tile in register r.
// Those registers, exponentiated and rounded to bf16, ARE the k-slices the second MFMA needs for P (the order
// of the contraction index inside an MFMA is free as long as both operands agree), and the matching V operand
// (4 consecutive keys of one head-dim column per read) comes from the LDS transpose read ds_read_b64_tr_b16.
#include "caat_internal.h"

namespace caat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

static constexpr unsigned OOB_OFF = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t attn_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)0x80000000, 0x00020000);
}

// ---------------------------------------------------------------------------------------------------------
// RoPE in place on the q and k column blocks of qkv [rows, 3*hd] (row = rank*tokens + batch*seq + pos):
// pairs (j, j + d/2), angle pos * base^(-2j/d).  One thread rotates 8 pairs of one head of one row.
__global__ __launch_bounds__(256) void rope_kernel(bf16_t* qkv, long long rows, int seq, int hd, int d, float log2_base,
                                                   long long pos0) {
  const int half = d >> 1;
  const int groups_per_head = half >> 3;            // 8 pairs per thread
  const int heads2 = 2 * (hd / d);                  // q heads then k heads
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long per_row = (long long)heads2 * groups_per_head;
  if (idx >= rows * per_row) return;
  const long long row = idx / per_row;
  const int rem = (int)(idx - row * per_row);
  const int head = rem / groups_per_head, grp = rem - head * groups_per_head;
  const float pos = (float)(pos0 + row % seq);
  bf16_t* p = qkv + row * 3LL * hd + (long long)head * d + grp * 8;   // q heads occupy [0,hd), k heads [hd,2hd)
  const uint4 lo = *reinterpret_cast<const uint4*>(p);
  const uint4 hi = *reinterpret_cast<const uint4*>(p + half);
  const unsigned lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
  unsigned ol[4], oh[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float x1[2] = {lo_bf(lw[w]), hi_bf(lw[w])}, x2[2] = {lo_bf(hw[w]), hi_bf(hw[w])}, y1[2], y2[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int j = grp * 8 + w * 2 + e;
      const float inv = exp2f(-2.0f * (float)j / (float)d * log2_base);
      float s, c;
      sincosf(pos * inv, &s, &c);
      y1[e] = x1[e] * c - x2[e] * s;
      y2[e] = x2[e] * c + x1[e] * s;
    }
    ol[w] = pack2bf(y1[0], y1[1]);
    oh[w] = pack2bf(y2[0], y2[1]);
  }
  *reinterpret_cast<uint4*>(p) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
  *reinterpret_cast<uint4*>(p + half) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
}

hipError_t launch_rope(bf16_t* qkv, long long rows, int seq, int hd, int d, float base, long long pos0, hipStream_t s) {
  const long long work = rows * 2LL * (hd / d) * (d / 16);
  if (work == 0) return hipSuccess;
  const long long blocks = (work + 255) / 256;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, rows, seq, hd, d, log2f(base), pos0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
static constexpr int HD = 128;    // head dim
static constexpr int BQ = 128;    // queries per workgroup (32 per wave)
static constexpr int BKV = 64;    // keys per step
static constexpr int KCH = HD / 8;  // 16-byte chunks per K/V row

// LDS chunk swizzles (chunk = 16 bytes of a 256-byte row): K is read as MFMA fragments (32 consecutive rows, one
// chunk) -> spread by row & 15; V is read by the transpose read (4 consecutive rows x 64 bytes) -> spread by row & 3.
__device__ __forceinline__ int kswz(int row, int c) { return c ^ (row & 15); }
__device__ __forceinline__ int vswz(int row, int c) { return c ^ ((row & 3) << 2); }

// qkv: [T*tokens, 3*hd] with q | k | v column blocks (q, k already rotated); out: [T*tokens, hd]
__global__ __launch_bounds__(256) void flash_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out, int seq,
                                                        int hd, int heads, int n_qblk, float scale_log2) {
  __shared__ uint4 smem[2 * 2 * BKV * KCH];  // [stage][K|V][64 rows][16 chunks] = 64 KB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int frow = lane & 31, hf = lane >> 5;
  // longest-first over the whole launch: the last (heaviest, causal) query blocks of every head come first
  const int n_bh = gridDim.x / n_qblk;
  const int qb = n_qblk - 1 - (int)(blockIdx.x / n_bh);
  const int bh = blockIdx.x % n_bh;              // (rank*batch + b) * heads + head
  const int head = bh % heads;
  const long long seq_row0 = (long long)(bh / heads) * seq;   // first row of this sequence in qkv
  const long long ld = 3LL * hd;
  const int q0 = qb * BQ;
  const bf16_t* qbase = qkv + seq_row0 * ld + (long long)head * HD;
  const bf16_t* kbase = qbase + hd;
  const bf16_t* vbase = qbase + 2 * hd;

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

  // global -> LDS: a wave instruction fills 4 rows (64 lanes x 16 B); 64 rows = 16 instructions per tile, 4 per wave
  auto issue_tile = [&](int blk, int stage) {
    const int kv0 = blk * BKV;
    const i32x4_t rk = make_rsrc(kbase + (long long)kv0 * ld);
    const i32x4_t rv = make_rsrc(vbase + (long long)kv0 * ld);
    uint4* kt = smem + stage * (2 * BKV * KCH);
    uint4* vt = kt + BKV * KCH;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int rg = it * 4 + wave;                    // group of 4 rows
      const int row = rg * 4 + (lane >> 4), phys = lane & 15;
      const bool in = (kv0 + row) < seq;
      const unsigned ko = in ? (unsigned)((long long)row * ld * 2 + kswz(row, phys) * 16) : OOB_OFF;
      const unsigned vo = in ? (unsigned)((long long)row * ld * 2 + vswz(row, phys) * 16) : OOB_OFF;
      dma16(rk, ko, kt + rg * 64);
      dma16(rv, vo, vt + rg * 64);
    }
  };

  issue_tile(0, 0);
  for (int blk = 0; blk < nblk; ++blk) {
    const int stage = blk & 1;
    wait_vmcnt<0>();
    __syncthreads();                                   // tile blk landed; everyone is done with the other stage
    if (blk + 1 < nblk) issue_tile(blk + 1, stage ^ 1);
    const uint4* kt = smem + stage * (2 * BKV * KCH);
    const char* vt = reinterpret_cast<const char*>(kt + BKV * KCH);
    const int kv0 = blk * BKV;

    // ---- S^T tiles: 2 key tiles of 32; contraction over head dim in 8 steps of 16
    f32x16_t sacc[BKV / 32];
#pragma unroll
    for (int j = 0; j < BKV / 32; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[j][r] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) {
        const int row = j * 32 + frow;
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, kt[row * KCH + kswz(row, ks * 2 + hf)]);
        sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[j], 0, 0, 0);
      }
    }
    // ---- causal mask + online softmax for query qrow (keys of register r: kv0 + 32j + 8(r/4) + 4hf + r%4)
    float mx = -INFINITY;
    // wave-uniform: does some key of this block exceed some query of this wave?  (only the last blocks of a tile)
    if ((kv0 + BKV - 1) > (q0 + wave * 32)) {
#pragma unroll
      for (int j = 0; j < BKV / 32; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + j * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key > qrow) sacc[j][r] = -INFINITY;
        }
    }
#pragma unroll
    for (int j = 0; j < BKV / 32; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[j][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));            // the other half of the row lives in lane ^ 32
    const float m_new = fmaxf(m_run, mx);               // finite: key 0 is visible to every query
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
    const float mb = m_new * scale_log2;
    float psum = 0.0f;
    bf16x8_t pf[BKV / 16];
#pragma unroll
    for (int j = 0; j < BKV / 32; ++j)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float pv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pv[e] = __builtin_amdgcn_exp2f(sacc[j][t * 8 + e] * scale_log2 - mb);   // arguments <= 0; tiny results flush to 0
          psum += pv[e];
        }
        const uint4 w = make_uint4(pack2bf(pv[0], pv[1]), pack2bf(pv[2], pv[3]), pack2bf(pv[4], pv[5]), pack2bf(pv[6], pv[7]));
        pf[j * 2 + t] = __builtin_bit_cast(bf16x8_t, w);
      }
    l_run = l_run * alpha + psum;
    // the running maximum settles after the first blocks: rescale the accumulators only if some row's maximum moved
    if (__any(m_new != m_run)) {
#pragma unroll
      for (int t = 0; t < HD / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
    }
    m_run = m_new;

    // ---- O^T += V^T P^T : A operand = V columns (head-dim index frow of tile dt), B operand = P (query frow).
    // k-slice u (16 keys) of the block: lane half hf contributes keys 16u + 4hf + {0..3} and 16u + 8 + 4hf + {0..3}
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt) {
#pragma unroll
      for (int u = 0; u < BKV / 16; ++u) {
        // transpose read: input lane i of a 16-lane group supplies row (i/4), 8-byte column group (i%4);
        // output lane j receives column j of those 4 rows
        const int i16 = lane & 15, grp = (lane >> 4) & 1;
        const int col = dt * 32 + grp * 16 + (i16 & 3) * 4;      // head-dim column of the 8-byte piece
        short4_t v0, v1;
        {
          const int row = u * 16 + 4 * hf + (i16 >> 2);
          const char* a0 = vt + (row * KCH + vswz(row, col >> 3)) * 16 + (col & 7) * 2;
          v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)a0);
          const int row1 = row + 8;
          const char* a1 = vt + (row1 * KCH + vswz(row1, col >> 3)) * 16 + (col & 7) * 2;
          v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)a1);
        }
        typedef short short8_t __attribute__((ext_vector_type(8)));
        const short8_t vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv), pf[u], oacc[dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise and store: lane holds out[qrow][32dt + 8(r/4) + 4hf + r%4]
  l_run += __shfl_xor(l_run, 32, 64);
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
hipError_t launch_flash_fwd(const bf16_t* qkv, bf16_t* out, long long n_seq, int seq, int hd, int d, hipStream_t s) {
  if (d != HD) return hipErrorInvalidValue;
  const int heads = hd / HD;
  const int n_qblk = (seq + BQ - 1) / BQ;
  const long long blocks = n_seq * heads * n_qblk;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFLL || (long long)(seq + BKV) * 3 * hd * 2 >= 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  hipLaunchKernelGGL(flash_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, out, seq, hd, heads, n_qblk, scale_log2);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------
// Decode: one new token per sequence.  (a) append the token's rotated k and its v to the caches at position
// kv_len; (b) attention of the single query over kv_len + 1 cached keys.  Both are pure streaming (the KV read is
// the layer's dominant HBM traffic), so there is no MFMA here: a workgroup owns one (rank, sequence, head);
// 16 lanes own one key row (256 B), a wave takes 4 consecutive keys per step, the 4 waves 16; every 16-lane group
// runs its own online softmax and the 16 partial results are merged through LDS in a fixed order.
__global__ __launch_bounds__(256) void kv_append_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ kc,
                                                        bf16_t* __restrict__ vc, long long n_seq, int hpr, int hd,
                                                        long long cap, long long pos) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;   // (seq, head, chunk of 8)
  if (idx >= n_seq * hpr * 16) return;
  const int c = (int)(idx & 15);
  const long long sh = idx >> 4;                                      // seq * hpr + head
  const long long sq = sh / hpr;
  const int head = (int)(sh - sq * hpr);
  const bf16_t* src = qkv + sq * 3LL * hd + (long long)head * 128 + c * 8;
  const long long dst = (sh * cap + pos) * 128 + c * 8;
  *reinterpret_cast<uint4*>(kc + dst) = *reinterpret_cast<const uint4*>(src + hd);
  *reinterpret_cast<uint4*>(vc + dst) = *reinterpret_cast<const uint4*>(src + 2 * hd);
}

__global__ __launch_bounds__(256) void decode_attn_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ kc,
                                                          const bf16_t* __restrict__ vc, bf16_t* __restrict__ out, int hpr,
                                                          int hd, long long cap, int nkeys, float scale_log2) {
  __shared__ float s_acc[16][128];
  __shared__ float s_m[16], s_l[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, c = lane & 15;
  const long long sh = blockIdx.x;                 // seq * hpr + head
  const long long sq = sh / hpr;
  const int head = (int)(sh - sq * hpr);
  float q[8];
  {
    const uint4 w = *reinterpret_cast<const uint4*>(qkv + sq * 3LL * hd + (long long)head * 128 + c * 8);
    q[0] = lo_bf(w.x); q[1] = hi_bf(w.x); q[2] = lo_bf(w.y); q[3] = hi_bf(w.y);
    q[4] = lo_bf(w.z); q[5] = hi_bf(w.z); q[6] = lo_bf(w.w); q[7] = hi_bf(w.w);
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] *= scale_log2;
  }
  const __amdgpu_buffer_rsrc_t rk = attn_rsrc(kc + sh * cap * 128);
  const __amdgpu_buffer_rsrc_t rv = attn_rsrc(vc + sh * cap * 128);
  float m = -INFINITY, l = 0.0f, acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  constexpr int UN = 4;
  for (int key0 = wave * 4 + g; key0 < nkeys; key0 += 16 * UN) {
    u32x4_t kv[UN], vv[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int key = key0 + 16 * u;
      const unsigned off = key < nkeys ? (unsigned)key * 256u + c * 16 : OOB_OFF;
      kv[u] = __builtin_amdgcn_raw_buffer_load_b128(rk, (int)off, 0, 0);
      vv[u] = __builtin_amdgcn_raw_buffer_load_b128(rv, (int)off, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const bool valid = (key0 + 16 * u) < nkeys;
      float s = q[0] * lo_bf(kv[u].x) + q[1] * hi_bf(kv[u].x) + q[2] * lo_bf(kv[u].y) + q[3] * hi_bf(kv[u].y) +
                q[4] * lo_bf(kv[u].z) + q[5] * hi_bf(kv[u].z) + q[6] * lo_bf(kv[u].w) + q[7] * hi_bf(kv[u].w);
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      s += __shfl_xor(s, 4, 64);
      s += __shfl_xor(s, 8, 64);
      const float m_new = valid ? fmaxf(m, s) : m;
      const float alpha = valid ? exp2f(m - m_new) : 1.0f;     // m = -inf on the first key: exp2(-inf) = 0
      const float p = valid ? exp2f(s - m_new) : 0.0f;
      l = l * alpha + p;
      const unsigned w[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] = acc[2 * e] * alpha + p * lo_bf(w[e]);
        acc[2 * e + 1] = acc[2 * e + 1] * alpha + p * hi_bf(w[e]);
      }
      m = m_new;
    }
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
    out[sq * (long long)hd + (long long)head * 128 + tid] = f2bf(num / den);
  }
}

hipError_t launch_kv_append(const bf16_t* qkv, bf16_t* kc, bf16_t* vc, long long n_seq, int hpr, int hd, long long cap,
                            long long pos, hipStream_t s) {
  const long long work = n_seq * hpr * 16;
  if (work == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, qkv, kc, vc, n_seq, hpr, hd,
                     cap, pos);
  return hipGetLastError();
}

// out [n_seq, hd] = softmax(q K^T / sqrt(d)) V over keys 0 .. nkeys-1 of caches [n_seq][hpr][cap][128]
hipError_t launch_decode_attn(const bf16_t* qkv, const bf16_t* kc, const bf16_t* vc, bf16_t* out, long long n_seq, int hpr,
                              int hd, int d, long long cap, long long nkeys, hipStream_t s) {
  if (d != HD || nkeys < 1 || nkeys > cap || cap * 256 >= 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const long long blocks = n_seq * hpr;
  if (blocks == 0) return hipSuccess;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  hipLaunchKernelGGL(decode_attn_kernel, dim3((unsigned)blocks), dim3(256), 0, s, qkv, kc, vc, out, hpr, hd, cap, (int)nkeys,
                     scale_log2);
  return hipGetLastError();
}

}  // namespace caat
