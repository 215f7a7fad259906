// HBM-bound streaming kernels of the partial-sync block (gfx950): the partial channel-reduce of Eq. A3/A5 with
// the residual add of Sec. 4, and the per-rank LayerNorm / RMSNorm forward and backward (Sec. 4, Fig. 2b).
// All of them move 16-byte vectors (8 bf16), keep arithmetic in fp32 and round once.
#include "caat_internal.h"

namespace caat {

__device__ __forceinline__ void unpack8(const uint4& v, float* f) {
  f[0] = lo_bf(v.x); f[1] = hi_bf(v.x); f[2] = lo_bf(v.y); f[3] = hi_bf(v.y);
  f[4] = lo_bf(v.z); f[5] = hi_bf(v.z); f[6] = lo_bf(v.w); f[7] = hi_bf(v.w);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 v;
  v.x = pack2bf(f[0], f[1]); v.y = pack2bf(f[2], f[3]); v.z = pack2bf(f[4], f[5]); v.w = pack2bf(f[6], f[7]);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// ---------------------------------------------------------------------------------------------------------
// Partial channel-reduce.  One thread owns one group of 8 channels of one token for ALL ranks: it reads the T
// partial vectors, sums them in ascending rank order in fp32, and writes the T outputs.  Because a thread
// reads every input of its group before it writes, out may alias y.  `ncg` = number of 8-channel groups per
// row that are processed: ceil(hs/8) when the private channels need no work, h/8 otherwise.
// TT > 0: compile-time rank count (loads fully unrolled and in flight together); TT == 0: any T.
// The partial sums were written by the kernel just before and mostly still sit in the caches: plain loads.  The
// residual is older data read once: non-temporal loads (with the hint on both, small problems whose partials are
// cache-resident lost 7 %, large ones gained 14 %).  `big`: the shared part of one tensor is too large to stay in the
// caches between kernels (more than 96 MiB): its partial sums are streamed too, and so are the results.
template <int TT, bool HAS_RES>
__device__ __forceinline__ void partial_sync_item(const bf16_t* y, const bf16_t* resid, bf16_t* out, int T_, long long n,
                                                  int h, int hs, float scale, int shared_only, int big, long long i,
                                                  int col) {
  const int T = TT > 0 ? TT : T_;
  const long long plane = n * (long long)h;  // elements per rank
  const long long off = i * h + col;

  if (col + 8 <= hs) {  // all 8 channels shared
    float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (TT > 0) {
      uint4 v[TT > 0 ? TT : 1];
#pragma unroll
      for (int m = 0; m < TT; ++m)
        v[m] = big ? ld_stream(y + m * plane + off) : *reinterpret_cast<const uint4*>(y + m * plane + off);
#pragma unroll
      for (int m = 0; m < TT; ++m) {
        float f[8];
        unpack8(v[m], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum[e] += f[e];
      }
    } else {
      for (int m = 0; m < T; ++m) {
        float f[8];
        unpack8(*reinterpret_cast<const uint4*>(y + m * plane + off), f);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum[e] += f[e];
      }
    }
    if constexpr (HAS_RES) {
#pragma unroll 4
      for (int m = 0; m < T; ++m) {
        float r[8], o[8];
        unpack8(ld_stream(resid + m * plane + off), r);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = sum[e] + r[e];
        if (big) st_stream(out + m * plane + off, pack8(o));
        else *reinterpret_cast<uint4*>(out + m * plane + off) = pack8(o);
      }
    } else {
      const uint4 o = pack8(sum);  // one rounding, the same bits on every rank
#pragma unroll 4
      for (int m = 0; m < T; ++m) {
        if (big) st_stream(out + m * plane + off, o);
        else *reinterpret_cast<uint4*>(out + m * plane + off) = o;
      }
    }
    return;
  }

  // group straddles hs or is entirely private: channel-wise case split of Eq. A3
  float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < hs) {
    for (int m = 0; m < T; ++m) {
      float f[8];
      unpack8(*reinterpret_cast<const uint4*>(y + m * plane + off), f);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum[e] += f[e];
    }
  }
  for (int m = 0; m < T; ++m) {
    float f[8], r[8], o[8];
    unpack8(*reinterpret_cast<const uint4*>(y + m * plane + off), f);  // rank m's own values (not yet overwritten)
    if constexpr (HAS_RES) {
      unpack8(ld_stream(resid + m * plane + off), r);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = 0.0f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (col + e < hs) o[e] = sum[e] + r[e];
      else o[e] = shared_only ? f[e] : scale * f[e] + r[e];  // shared_only: private channels are already final
    }
    *reinterpret_cast<uint4*>(out + m * plane + off) = pack8(o);
  }
}


// Flat mode (tok_per_wg == 0): one thread per (token, 8-channel group).  Chunked mode: a workgroup walks a contiguous
// range of tok_per_wg tokens.  With 512 such workgroups and the non-temporal hint on every access, a reduce whose
// shared part of a row is at least 4 KB long (whole rows at p = 1, half rows at h = 4096) measured 65 - 68 % of the
// 8 TB/s peak cold, against 54 - 62 % for the flat grid; with shorter runs per row (2 KB at 4 KB stride: h = 2048,
// p = 0.5) every variant stays near 50 % -- half of each DRAM interleave unit is skipped -- and the flat grid is best.
template <int TT, bool HAS_RES>
__global__ __launch_bounds__(256) void partial_sync_kernel(const bf16_t* y, const bf16_t* resid,
                                                           bf16_t* out, int T_, long long n, int h, int hs,
                                                           float scale, int ncg, int shared_only, int big,
                                                           long long tok_per_wg) {
  if (tok_per_wg == 0) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * (long long)ncg) return;
    const long long i = idx / ncg;
    partial_sync_item<TT, HAS_RES>(y, resid, out, T_, n, h, hs, scale, shared_only, big, i, (int)(idx - i * ncg) * 8);
    return;
  }
  const long long t0 = (long long)blockIdx.x * tok_per_wg;
  const long long t1 = t0 + tok_per_wg < n ? t0 + tok_per_wg : n;
  const long long total = (t1 - t0) * ncg;
  for (long long idx = threadIdx.x; idx < total; idx += 256) {
    const long long i = idx / ncg;
    partial_sync_item<TT, HAS_RES>(y, resid, out, T_, n, h, hs, scale, shared_only, big, t0 + i, (int)(idx - i * ncg) * 8);
  }
}

template <int TT>
static hipError_t sync_dispatch(const bf16_t* y, const bf16_t* resid, bf16_t* out, int T, long long n, int h, int hs,
                                float scale, int ncg, int shared_only, hipStream_t s) {
  const long long work = n * (long long)ncg;
  long long blocks = (work + 255) / 256;
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  const int big = ((double)T * (double)n * (double)hs * 2.0 > 96.0 * 1048576.0) ? 1 : 0;
  // chunked walk for large reduces with long contiguous runs per row (see the kernel's comment)
  long long tok_per_wg = 0;
  if (big && (long long)ncg * 16 >= 4096 && n >= 1024) {
    tok_per_wg = (n + 511) / 512;
    blocks = (n + tok_per_wg - 1) / tok_per_wg;
  }
  if (resid)
    hipLaunchKernelGGL((partial_sync_kernel<TT, true>), dim3((unsigned)blocks), dim3(256), 0, s, y, resid, out, T, n,
                       h, hs, scale, ncg, shared_only, big, tok_per_wg);
  else
    hipLaunchKernelGGL((partial_sync_kernel<TT, false>), dim3((unsigned)blocks), dim3(256), 0, s, y, resid, out, T, n,
                       h, hs, scale, ncg, shared_only, big, tok_per_wg);
  return hipGetLastError();
}

static hipError_t sync_any(const bf16_t* y, const bf16_t* resid, bf16_t* out, int T, long long tokens, int h, int hs,
                           float private_scale, int shared_only, hipStream_t s) {
  const bool private_work = !shared_only && ((out != y) || (resid != nullptr) || (private_scale != 1.0f));
  const int ncg = private_work ? h / 8 : (hs + 7) / 8;
  if (ncg == 0 || tokens == 0) return hipSuccess;  // p = 0 in place: nothing moves
  switch (T) {
    case 2: return sync_dispatch<2>(y, resid, out, T, tokens, h, hs, private_scale, ncg, shared_only, s);
    case 4: return sync_dispatch<4>(y, resid, out, T, tokens, h, hs, private_scale, ncg, shared_only, s);
    case 8: return sync_dispatch<8>(y, resid, out, T, tokens, h, hs, private_scale, ncg, shared_only, s);
    case 16: return sync_dispatch<16>(y, resid, out, T, tokens, h, hs, private_scale, ncg, shared_only, s);
    default: return sync_dispatch<0>(y, resid, out, T, tokens, h, hs, private_scale, ncg, shared_only, s);
  }
}

hipError_t launch_partial_sync(const bf16_t* y, const bf16_t* resid, bf16_t* out, int T, long long tokens, int h,
                               int hs, float private_scale, hipStream_t s) {
  return sync_any(y, resid, out, T, tokens, h, hs, private_scale, 0, s);
}

// In place on the shared channels only, with the residual added there; private channels are left as they are
// (the row-parallel GEMM's epilogue has already finished them).
hipError_t launch_partial_sync_shared(bf16_t* io, const bf16_t* resid, int T, long long tokens, int h, int hs,
                                      hipStream_t s) {
  return sync_any(io, resid, io, T, tokens, h, hs, 1.0f, 1, s);
}

// The reduce of the backward pass, shared channels only, from one buffer into another: dst[m][:, l < hs] = sum over
// ranks of src[m'][:, l]; nothing else of dst is touched.  hs must be a multiple of 8 (no vector straddles it).
hipError_t launch_partial_sync_shared_from(const bf16_t* src, bf16_t* dst, int T, long long tokens, int h, int hs,
                                           hipStream_t s) {
  if (hs % 8 != 0) return hipErrorInvalidValue;
  return sync_any(src, nullptr, dst, T, tokens, h, hs, 1.0f, 1, s);
}

// ---------------------------------------------------------------------------------------------------------
// Norm forward: one wavefront per row, the row stays in registers (VPL 16-byte vectors per lane), statistics
// by wave reduction in fp32 (two passes over registers: mean, then centred second moment).
// Split source (xs != null): the first hs_split channels of every rank's row are stored once, xs [tokens, hs_split]
// (row = rank*tokens + token reads token's shared row), and x holds only the private channels [rows, h - hs_split].
template <int VPL, bool LN, bool STREAM>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
                                                       const bf16_t* __restrict__ beta, bf16_t* __restrict__ y,
                                                       float* __restrict__ mean, float* __restrict__ rstd,
                                                       long long rows, int h, float eps, const bf16_t* __restrict__ xs,
                                                       int hs_split, long long tokens) {
  const int lane = threadIdx.x & 63;
  const long long wave0 = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long nwaves = (long long)gridDim.x * 4;
  const int nvec = h >> 3;
  const float inv_h = 1.0f / (float)h;
  for (long long row = wave0; row < rows; row += nwaves) {
    const bf16_t* xr = x + row * h;
    const bf16_t* xsr = nullptr;
    if (xs != nullptr) {
      xr = x + row * (h - hs_split) - hs_split;       // column c >= hs_split of this row sits at xr[c]
      xsr = xs + (row % tokens) * hs_split;
    }
    float f[VPL][8];
    float s = 0.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 64 + lane;
      uint4 w = make_uint4(0u, 0u, 0u, 0u);
      if (vi < nvec) {
        const bf16_t* src = (xsr != nullptr && vi * 8 < hs_split ? xsr : xr) + vi * 8;
        w = STREAM ? ld_stream(src) : *reinterpret_cast<const uint4*>(src);
      }
      unpack8(w, f[v]);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += LN ? f[v][e] : f[v][e] * f[v][e];
    }
    s = wave_sum(s);
    float mu = 0.0f, var;
    if constexpr (LN) {
      mu = s * inv_h;
      float q = 0.0f;
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        if (v * 64 + lane < nvec) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float d = f[v][e] - mu;
            q += d * d;
          }
        }
      }
      var = wave_sum(q) * inv_h;
    } else {
      var = s * inv_h;
    }
    const float rs = rsqrtf(var + eps);
    if (lane == 0) {
      if (LN && mean) mean[row] = mu;
      rstd[row] = rs;
    }
    bf16_t* yr = y + row * h;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 64 + lane;
      if (vi < nvec) {
        float g[8], b[8], o[8];
        unpack8(*reinterpret_cast<const uint4*>(gamma + vi * 8), g);
        if constexpr (LN) unpack8(*reinterpret_cast<const uint4*>(beta + vi * 8), b);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = LN ? ((f[v][e] - mu) * rs * g[e] + b[e]) : (f[v][e] * rs * g[e]);
        if (STREAM) st_stream(yr + vi * 8, pack8(o));   // an output this large is out of the caches before it is read
        else *reinterpret_cast<uint4*>(yr + vi * 8) = pack8(o);
      }
    }
  }
}

template <int VPL>
static hipError_t norm_fwd_dispatch(const bf16_t* x, const bf16_t* gamma, const bf16_t* beta, bf16_t* y, float* mean,
                                    float* rstd, int norm, long long rows, int h, float eps, const bf16_t* xs,
                                    int hs_split, long long tokens, hipStream_t s) {
  long long blocks = (rows + 3) / 4;
  if (blocks > 65536) blocks = 65536;
  if (blocks == 0) return hipSuccess;
  // An input of about the size of the 256 MB memory-side cache or more cannot still be there from the kernel that wrote it: it is
  // read with the non-temporal hint (h = 4096, T = 8, 4096 tokens: -15 %); a smaller one mostly is, and the hint cost
  // 4 % there.
  const bool stream = (double)rows * h * 2.0 > 192.0 * 1048576.0;
#define CAAT_NORM_FWD(LN_, ST_) hipLaunchKernelGGL((norm_fwd_kernel<VPL, LN_, ST_>), dim3((unsigned)blocks), dim3(256), 0, s, x, gamma, beta, y, mean, rstd, rows, h, eps, xs, hs_split, tokens)
  if (norm == 0) {
    if (stream) CAAT_NORM_FWD(true, true); else CAAT_NORM_FWD(true, false);
  } else {
    if (stream) CAAT_NORM_FWD(false, true); else CAAT_NORM_FWD(false, false);
  }
#undef CAAT_NORM_FWD
  return hipGetLastError();
}

// dedup_hs > 0: x is a residual stream that stores its first dedup_hs channels once: [tokens, dedup_hs] followed by the
// private channels [T, tokens, h - dedup_hs] (dedup_hs a multiple of 8)
hipError_t launch_norm_fwd(const bf16_t* x, const bf16_t* gamma, const bf16_t* beta, bf16_t* y, float* mean,
                           float* rstd, int norm, int T, long long tokens, int h, float eps, hipStream_t s,
                           int dedup_hs) {
  const long long rows = (long long)T * tokens;
  const int vpl = (h / 8 + 63) / 64;
  const bf16_t* xs = nullptr;
  if (dedup_hs > 0) {
    if (dedup_hs % 8 != 0 || dedup_hs > h) return hipErrorInvalidValue;
    xs = x;
    x = x + tokens * dedup_hs;
  }
  if (vpl <= 1) return norm_fwd_dispatch<1>(x, gamma, beta, y, mean, rstd, norm, rows, h, eps, xs, dedup_hs, tokens, s);
  if (vpl <= 2) return norm_fwd_dispatch<2>(x, gamma, beta, y, mean, rstd, norm, rows, h, eps, xs, dedup_hs, tokens, s);
  if (vpl <= 4) return norm_fwd_dispatch<4>(x, gamma, beta, y, mean, rstd, norm, rows, h, eps, xs, dedup_hs, tokens, s);
  if (vpl <= 8) return norm_fwd_dispatch<8>(x, gamma, beta, y, mean, rstd, norm, rows, h, eps, xs, dedup_hs, tokens, s);
  if (vpl <= 16) return norm_fwd_dispatch<16>(x, gamma, beta, y, mean, rstd, norm, rows, h, eps, xs, dedup_hs, tokens, s);
  return hipErrorInvalidValue;  // h > 8192
}

// ---------------------------------------------------------------------------------------------------------
// The reduce and the norm that follows it in one launch (Eq. A3 / A5 second line + Sec. 4: X'_m = Norm(R_m + Z_m)).
// For decode-sized batches (a few dozen tokens) the two launches are start-up latency, not traffic; for prompts and
// training batches the fused kernel saves reading the reduced shared channels back.  One workgroup owns one token of
// ALL ranks: it sums the T partial vectors of the shared channels in ascending rank order, adds each rank's residual,
// rounds once and stores R' (exactly what partial_sync_kernel does), keeps every rank's row (rounded values, packed)
// in registers, and then normalises each rank's row with its own statistics (what norm_fwd_kernel does on R':
// RMSNorm, or LayerNorm with the two-pass variance).  hs % 8 == 0; a thread holds NG 16-byte column groups of every
// rank's row (h <= 2048 NG), so the register budget is NG*TT*4: T = 16 is taken up to h = 4096.
template <int TT, int NG, bool LN>
__global__ __launch_bounds__(256) void sync_norm_kernel(bf16_t* io, const bf16_t* __restrict__ resid,
                                                        const bf16_t* __restrict__ gamma,
                                                        const bf16_t* __restrict__ beta, bf16_t* __restrict__ xout,
                                                        float* __restrict__ mean, float* __restrict__ rstd,
                                                        long long n, int h, int hs, float eps, int big) {
  __shared__ float red[2][4][TT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long i = blockIdx.x;                        // token
  const long long plane = n * (long long)h;
  const int nvec = h >> 3;
  uint4 val[NG][TT];
  float ss[TT];
#pragma unroll
  for (int m = 0; m < TT; ++m) ss[m] = 0.0f;
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int vi = g * 256 + tid;
    if (vi < nvec) {
      const int col = vi * 8;
      const long long off = i * h + col;
      if (col < hs) {                                     // shared channels (hs is a multiple of 8)
        float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        {
          uint4 pv[TT];   // the T partials and the T residual vectors are requested together
#pragma unroll
          for (int m = 0; m < TT; ++m) {
            pv[m] = big ? ld_stream(io + m * plane + off) : *reinterpret_cast<const uint4*>(io + m * plane + off);
            val[g][m] = ld_stream(resid + m * plane + off);          // read once
          }
#pragma unroll
          for (int m = 0; m < TT; ++m) {
            float f[8];
            unpack8(pv[m], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] += f[e];
          }
        }
#pragma unroll
        for (int m = 0; m < TT; ++m) {
          float r[8], o[8];
          unpack8(val[g][m], r);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = sum[e] + r[e];
          val[g][m] = pack8(o);
          if (big) st_stream(io + m * plane + off, val[g][m]);
          else *reinterpret_cast<uint4*>(io + m * plane + off) = val[g][m];
        }
      } else {                                            // private channels: final since the GEMM epilogue
#pragma unroll
        for (int m = 0; m < TT; ++m)
          val[g][m] = big ? ld_stream(io + m * plane + off) : *reinterpret_cast<const uint4*>(io + m * plane + off);
      }
#pragma unroll
      for (int m = 0; m < TT; ++m) {
        float f[8];
        unpack8(val[g][m], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) ss[m] += LN ? f[e] : f[e] * f[e];
      }
    } else {
#pragma unroll
      for (int m = 0; m < TT; ++m) val[g][m] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
  // workgroup sums of the T rows: wave sums, then the four waves in a fixed order
  auto block_sums = [&](float* v, int slot) {
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      const float w = wave_sum(v[m]);
      if (lane == 0) red[slot][wave][m] = w;
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < TT; ++m) v[m] = ((red[slot][0][m] + red[slot][1][m]) + red[slot][2][m]) + red[slot][3][m];
  };
  const float inv_h = 1.0f / (float)h;
  block_sums(ss, 0);
  float mu[TT], rs[TT];
  if constexpr (LN) {
    float q[TT];
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      mu[m] = ss[m] * inv_h;
      q[m] = 0.0f;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if (g * 256 + tid < nvec) {
#pragma unroll
        for (int m = 0; m < TT; ++m) {
          float f[8];
          unpack8(val[g][m], f);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float d = f[e] - mu[m];
            q[m] += d * d;
          }
        }
      }
    }
    block_sums(q, 1);
#pragma unroll
    for (int m = 0; m < TT; ++m) rs[m] = rsqrtf(q[m] * inv_h + eps);
  } else {
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      mu[m] = 0.0f;
      rs[m] = rsqrtf(ss[m] * inv_h + eps);
    }
  }
  if (tid == 0) {
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      if (LN && mean) mean[m * n + i] = mu[m];
      rstd[m * n + i] = rs[m];
    }
  }
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int vi = g * 256 + tid;
    if (vi < nvec) {
      float gm[8], bt[8];
      unpack8(*reinterpret_cast<const uint4*>(gamma + vi * 8), gm);
      if constexpr (LN) unpack8(*reinterpret_cast<const uint4*>(beta + vi * 8), bt);
      const long long off = i * h + vi * 8;
#pragma unroll
      for (int m = 0; m < TT; ++m) {
        float f[8], o[8];
        unpack8(val[g][m], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = LN ? ((f[e] - mu[m]) * rs[m] * gm[e] + bt[e]) : (f[e] * rs[m] * gm[e]);
        if (big) st_stream(xout + m * plane + off, pack8(o));
        else *reinterpret_cast<uint4*>(xout + m * plane + off) = pack8(o);
      }
    }
  }
}

// Measured per launch, hint on every access against hint on the residual only: 134 MB per tensor (h = 2048, T = 4, 8192
// tokens) 76 against 72 us; 268 MB (h = 4096, T = 8, 4096 tokens) 153 against 165 us; 2.1 GB 1.24 against 1.30 ms.
static constexpr double SYNC_NORM_STREAM_BYTES = 192.0 * 1048576.0;
template <int TT, int NG>
static hipError_t sync_norm_dispatch(bf16_t* io, const bf16_t* resid, const bf16_t* gamma, const bf16_t* beta, bf16_t* xout,
                                     float* mean, float* rstd, int norm, long long tokens, int h, int hs, float eps,
                                     hipStream_t s) {
  // tensors too large to survive in the caches until their consumer runs (as in the norm forward kernel): every access
  // carries the non-temporal hint; smaller ones only the residual, which nothing has read before
  const int big = ((double)TT * (double)tokens * (double)h * 2.0 >= SYNC_NORM_STREAM_BYTES) ? 1 : 0;
  if (norm == 0)
    hipLaunchKernelGGL((sync_norm_kernel<TT, NG, true>), dim3((unsigned)tokens), dim3(256), 0, s, io, resid, gamma, beta, xout,
                       mean, rstd, tokens, h, hs, eps, big);
  else
    hipLaunchKernelGGL((sync_norm_kernel<TT, NG, false>), dim3((unsigned)tokens), dim3(256), 0, s, io, resid, gamma, beta, xout,
                       mean, rstd, tokens, h, hs, eps, big);
  return hipGetLastError();
}

// shapes the fused reduce + norm kernel takes: whole 16-byte groups of shared channels, T in {2, 4, 8} up to h = 8192 and
// T = 16 up to h = 4096 (a thread keeps its columns of all T rows in registers)
bool sync_norm_takes(int T, long long tokens, int h, int hs) {
  if (hs <= 0 || hs % 8 != 0 || hs > h || h % 8 != 0 || h > 8192 || tokens <= 0 || tokens > 0x7FFFFFFFLL) return false;
  if (T == 2 || T == 4 || T == 8) return true;
  return T == 16 && h <= 4096;
}

// io [T,n,h]: partial sums on the shared channels, final values on the private ones -> R' in place; xout = Norm(R');
// returns hipErrorInvalidValue for shapes the fused kernel does not take (the caller then runs the two kernels)
hipError_t launch_sync_norm(bf16_t* io, const bf16_t* resid, const bf16_t* gamma, const bf16_t* beta, bf16_t* xout,
                            float* mean, float* rstd, int norm, int T, long long tokens, int h, int hs, float eps,
                            hipStream_t s) {
  if (!sync_norm_takes(T, tokens, h, hs)) return hipErrorInvalidValue;
  const int ng = (h / 8 + 255) / 256;   // 1 .. 4
#define CAAT_SN(TT_, NG_) return sync_norm_dispatch<TT_, NG_>(io, resid, gamma, beta, xout, mean, rstd, norm, tokens, h, hs, eps, s)
#define CAAT_SN_T(TT_) \
  if (ng <= 1) CAAT_SN(TT_, 1); \
  if (ng <= 2) CAAT_SN(TT_, 2); \
  CAAT_SN(TT_, 4);
  switch (T) {
    case 2: CAAT_SN_T(2)
    case 4: CAAT_SN_T(4)
    case 8: CAAT_SN_T(8)
    case 16:
      if (ng <= 1) CAAT_SN(16, 1);
      CAAT_SN(16, 2);
    default: return hipErrorInvalidValue;
  }
#undef CAAT_SN_T
#undef CAAT_SN
}

// ---------------------------------------------------------------------------------------------------------
// Norm backward, placed before the reduce (Fig. 2b): g = dres + NormBwd(dy).  Each wave walks a contiguous
// range of rows and keeps its lanes' columns of dgamma / dbeta in registers; a workgroup combines its 4 waves
// through LDS and writes one partial row [2][h] to the workspace; a second kernel sums the partials in order.
static constexpr int NORM_BWD_MAX_BLOCKS = 512;

template <int VPL, bool LN>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ dres,
                                                       const bf16_t* __restrict__ x,
                                                       const bf16_t* __restrict__ gamma,
                                                       const float* __restrict__ mean, const float* __restrict__ rstd,
                                                       bf16_t* __restrict__ g_out, bf16_t* __restrict__ g_scaled,
                                                       float* __restrict__ partial, long long rows, int h, int hs,
                                                       float scale, long long rows_per_block, int skip_shared) {
  __shared__ float red[4][64 * 8];  // one vector column group at a time
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nvec = h >> 3;
  const float inv_h = 1.0f / (float)h;
  // per-lane column accumulators; gamma and the row's raw vectors stay packed (bf16) to save registers
  float dgam[VPL][8], dbet[LN ? VPL : 1][8];
  uint4 gam[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int vi = v * 64 + lane;
    gam[v] = make_uint4(0u, 0u, 0u, 0u);
    if (vi < nvec) gam[v] = *reinterpret_cast<const uint4*>(gamma + vi * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dgam[v][e] = 0.0f;
      if constexpr (LN) dbet[v][e] = 0.0f;
    }
  }
  const long long r0 = (long long)blockIdx.x * rows_per_block;
  long long r1 = r0 + rows_per_block;
  if (r1 > rows) r1 = rows;
  for (long long row = r0 + wave; row < r1; row += 4) {
    const float mu = LN ? mean[row] : 0.0f;
    const float rs = rstd[row];
    // all three inputs of the row are requested together: fetching the residual gradient only after the row sums
    // put a second trip to memory into every row.  They are read once: non-temporal loads (-10 % at h = 2048; in the
    // wide-row kernel below the hint gained 3 % and cost the reduce kernel that follows more than that)
    uint4 wx[VPL], wd[VPL], wr[VPL];
    float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 64 + lane;
      wx[v] = make_uint4(0u, 0u, 0u, 0u);
      wd[v] = wx[v];
      wr[v] = wx[v];
      if (vi < nvec) {
        wx[v] = ld_stream(x + row * h + vi * 8);
        wd[v] = ld_stream(dy + row * h + vi * 8);
        if (dres) wr[v] = ld_stream(dres + row * h + vi * 8);
      }
    }
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      float fx[8], fd[8], g[8];
      unpack8(wx[v], fx);
      unpack8(wd[v], fd);
      unpack8(gam[v], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xh = (fx[e] - mu) * rs;  // idle lanes: fd = 0 and gamma = 0, so they add nothing
        const float dxh = fd[e] * g[e];
        c1 += dxh;
        c2 += dxh * xh;
        dgam[v][e] += fd[e] * xh;
        if constexpr (LN) dbet[v][e] += fd[e];
      }
    }
    if constexpr (LN) c1 = wave_sum(c1) * inv_h;
    c2 = wave_sum(c2) * inv_h;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 64 + lane;
      if (vi < nvec) {
        float fx[8], fd[8], g[8], r[8], o[8];
        unpack8(wx[v], fx);
        unpack8(wd[v], fd);
        unpack8(gam[v], g);
        unpack8(wr[v], r);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (fx[e] - mu) * rs;
          const float dxh = fd[e] * g[e];
          o[e] = r[e] + rs * (LN ? (dxh - c1 - xh * c2) : (dxh - xh * c2));
        }
        // the private channels of g_out are not read again by the backward pass (the reduce reads the shared ones)
        if (skip_shared && vi * 8 >= hs) st_stream(g_out + row * h + vi * 8, pack8(o));
        else *reinterpret_cast<uint4*>(g_out + row * h + vi * 8) = pack8(o);
        // skip_shared: the reduce that follows writes the shared channels of g_scaled itself (from g_out)
        if (g_scaled && !(skip_shared && vi * 8 + 8 <= hs)) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (vi * 8 + e >= hs) o[e] *= scale;
          *reinterpret_cast<uint4*>(g_scaled + row * h + vi * 8) = pack8(o);
        }
      }
    }
  }
  // combine the 4 waves of the block in a fixed order, one 512-column slab at a time
  float* prow = partial + (long long)blockIdx.x * 2 * h;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
#pragma unroll
    for (int which = 0; which < (LN ? 2 : 1); ++which) {
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = (LN && which) ? dbet[LN ? v : 0][e] : dgam[v][e];
      __syncthreads();
      for (int c = threadIdx.x; c < 512; c += 256) {
        const int colg = v * 512 + c;
        if (colg < h) prow[which * h + colg] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
      }
    }
  }
}

// Wide rows (h > 4096; up to there the kernel above, at h = 4096 with every register of a one-wave-per-SIMD
// budget, measured 8 % faster than this one): the per-lane column accumulators would not fit, so here a whole
// workgroup owns one row at a time: thread t holds the 16-byte vectors v*256 + t (v < VPL) of the row, the two row
// sums go wave -> LDS -> all waves (slot chosen by row parity, one barrier per row), and the next row's x, dy and
// residual gradient are already in flight while the current row is reduced and written.  A thread's dgamma / dbeta
// columns are its own, so the partial row is written without any cross-wave combination.  Workgroup b walks rows
// [b*rpb, (b+1)*rpb).
template <int VPL, bool LN>
__global__ __launch_bounds__(256) void norm_bwd_wide_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ dres,
                                                            const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            bf16_t* __restrict__ g_out, bf16_t* __restrict__ g_scaled,
                                                            float* __restrict__ partial, long long rows, int h, int hs,
                                                            float scale, long long rows_per_block, int skip_shared) {
  __shared__ float red[2][2][4];  // [row parity][c1 | c2][wave]
  const int tid = threadIdx.x, wave = tid >> 6;
  const int nvec = h >> 3;
  const float inv_h = 1.0f / (float)h;
  float dgam[VPL][8], dbet[LN ? VPL : 1][8];
  uint4 gam[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int vi = v * 256 + tid;
    gam[v] = make_uint4(0u, 0u, 0u, 0u);
    if (vi < nvec) gam[v] = *reinterpret_cast<const uint4*>(gamma + vi * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dgam[v][e] = 0.0f;
      if constexpr (LN) dbet[v][e] = 0.0f;
    }
  }
  const long long r0 = (long long)blockIdx.x * rows_per_block;
  long long r1 = r0 + rows_per_block;
  if (r1 > rows) r1 = rows;
  uint4 nx[VPL], nd[VPL], nr[VPL];
  auto fetch = [&](long long row) {
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 256 + tid;
      nx[v] = make_uint4(0u, 0u, 0u, 0u);
      nd[v] = nx[v];
      nr[v] = nx[v];
      if (vi < nvec && row < r1) {
        nx[v] = *reinterpret_cast<const uint4*>(x + row * h + vi * 8);
        nd[v] = *reinterpret_cast<const uint4*>(dy + row * h + vi * 8);
        if (dres) nr[v] = *reinterpret_cast<const uint4*>(dres + row * h + vi * 8);
      }
    }
  };
  if (r0 < r1) fetch(r0);
  for (long long row = r0; row < r1; ++row) {
    const int par = (int)((row - r0) & 1);
    const float mu = LN ? mean[row] : 0.0f;
    const float rs = rstd[row];
    uint4 wx[VPL], wd[VPL], wr[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      wx[v] = nx[v];
      wd[v] = nd[v];
      wr[v] = nr[v];
    }
    fetch(row + 1);
    float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      float fx[8], fd[8], g[8];
      unpack8(wx[v], fx);
      unpack8(wd[v], fd);
      unpack8(gam[v], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xh = (fx[e] - mu) * rs;  // idle threads: fd = 0 and gamma = 0, so they add nothing
        const float dxh = fd[e] * g[e];
        c1 += dxh;
        c2 += dxh * xh;
        dgam[v][e] += fd[e] * xh;
        if constexpr (LN) dbet[v][e] += fd[e];
      }
    }
    if constexpr (LN) c1 = wave_sum(c1);
    c2 = wave_sum(c2);
    if ((tid & 63) == 0) {
      red[par][0][wave] = c1;
      red[par][1][wave] = c2;
    }
    __syncthreads();
    if constexpr (LN) c1 = (((red[par][0][0] + red[par][0][1]) + red[par][0][2]) + red[par][0][3]) * inv_h;
    c2 = (((red[par][1][0] + red[par][1][1]) + red[par][1][2]) + red[par][1][3]) * inv_h;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int vi = v * 256 + tid;
      if (vi < nvec) {
        float fx[8], fd[8], g[8], r[8], o[8];
        unpack8(wx[v], fx);
        unpack8(wd[v], fd);
        unpack8(gam[v], g);
        unpack8(wr[v], r);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (fx[e] - mu) * rs;
          const float dxh = fd[e] * g[e];
          o[e] = r[e] + rs * (LN ? (dxh - c1 - xh * c2) : (dxh - xh * c2));
        }
        // the private channels of g_out are not read again by the backward pass (the reduce reads the shared ones)
        if (skip_shared && vi * 8 >= hs) st_stream(g_out + row * h + vi * 8, pack8(o));
        else *reinterpret_cast<uint4*>(g_out + row * h + vi * 8) = pack8(o);
        // skip_shared: the reduce that follows writes the shared channels of g_scaled itself (from g_out)
        if (g_scaled && !(skip_shared && vi * 8 + 8 <= hs)) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (vi * 8 + e >= hs) o[e] *= scale;
          *reinterpret_cast<uint4*>(g_scaled + row * h + vi * 8) = pack8(o);
        }
      }
    }
  }
  float* prow = partial + (long long)blockIdx.x * 2 * h;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int vi = v * 256 + tid;
    if (vi < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        prow[vi * 8 + e] = dgam[v][e];
        if constexpr (LN) prow[h + vi * 8 + e] = dbet[v][e];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Norm backward and the backward partial channel-reduce in one launch (Fig. 2b: norm backward per rank first, the same
// reduce `h` on the result; Sec. 4: fp32 accumulation of values that travel as bf16).  One workgroup owns one token of
// ALL ranks at a time (thread t of NT holds the 16-byte column groups t, t+NT, ... of every rank's row, as in the
// forward sync_norm_kernel): it computes g_m = dres_m + NormBwd(dy_m) for the T rows, stores them rounded to bf16 as the
// un-reduced residual gradient (App. B), keeps those rounded values in registers, sums the shared channels over the
// ranks in ascending order in fp32 -- exactly the values and the order the stand-alone reduce would read back from
// g_out -- rounds once and stores the result to every rank's row of g_red; private channels of g_red get scale * g_m.
// A workgroup walks a contiguous range of tokens and keeps its threads' columns of dgamma / dbeta in registers over
// all of them (summed over tokens AND ranks), one partial row per workgroup; norm_bwd_finalize_kernel adds them up.
// hs % 8 == 0.  Saves, against the two kernels, the read-back of the shared channels and one launch.
template <int TT, int NG, bool LN, int NT>
__global__ __launch_bounds__(NT) void norm_bwd_sync_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ dres,
                                                            const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            bf16_t* __restrict__ g_out, bf16_t* __restrict__ g_red,
                                                            float* __restrict__ partial, long long n, int h, int hs,
                                                            float scale, long long tokens_per_block) {
  constexpr int NW = NT / 64;
  __shared__ float red[2][2][NW][TT];   // [token parity][c1 | c2][wave][rank]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nvec = h >> 3;
  const float inv_h = 1.0f / (float)h;
  const long long plane = n * (long long)h;
  float dgam[NG][8], dbet[LN ? NG : 1][8];
  uint4 gam[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int vi = g * NT + tid;
    gam[g] = make_uint4(0u, 0u, 0u, 0u);
    if (vi < nvec) gam[g] = *reinterpret_cast<const uint4*>(gamma + vi * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dgam[g][e] = 0.0f;
      if constexpr (LN) dbet[g][e] = 0.0f;
    }
  }
  const long long t0 = (long long)blockIdx.x * tokens_per_block;
  long long t1 = t0 + tokens_per_block;
  if (t1 > n) t1 = n;
  for (long long i = t0; i < t1; ++i) {
    const int par = (int)((i - t0) & 1);
    // the three inputs of all T rows of the token are requested together (read once: non-temporal)
    uint4 wx[NG][TT], wd[NG][TT], wr[NG][TT];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int vi = g * NT + tid;
#pragma unroll
      for (int m = 0; m < TT; ++m) {
        wx[g][m] = make_uint4(0u, 0u, 0u, 0u);
        wd[g][m] = wx[g][m];
        wr[g][m] = wx[g][m];
        if (vi < nvec) {
          const long long off = m * plane + i * h + vi * 8;
          wx[g][m] = ld_stream(x + off);
          wd[g][m] = ld_stream(dy + off);
          if (dres) wr[g][m] = ld_stream(dres + off);
        }
      }
    }
    float mu[TT], rs[TT], c1[TT], c2[TT];
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      mu[m] = LN ? mean[m * n + i] : 0.0f;
      rs[m] = rstd[m * n + i];
      c1[m] = 0.0f;
      c2[m] = 0.0f;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float gm[8];
      unpack8(gam[g], gm);
#pragma unroll
      for (int m = 0; m < TT; ++m) {
        float fx[8], fd[8];
        unpack8(wx[g][m], fx);
        unpack8(wd[g][m], fd);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (fx[e] - mu[m]) * rs[m];   // idle threads: fd = 0 and gamma = 0, so they add nothing
          const float dxh = fd[e] * gm[e];
          c1[m] += dxh;
          c2[m] += dxh * xh;
          dgam[g][e] += fd[e] * xh;
          if constexpr (LN) dbet[g][e] += fd[e];
        }
      }
    }
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      if constexpr (LN) c1[m] = wave_sum(c1[m]);
      c2[m] = wave_sum(c2[m]);
      if (lane == 0) {
        if constexpr (LN) red[par][0][wave][m] = c1[m];
        red[par][1][wave][m] = c2[m];
      }
    }
    __syncthreads();   // one barrier per token: the slot of the token before last is free again by then
#pragma unroll
    for (int m = 0; m < TT; ++m) {
      float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {     // the waves' sums in ascending order
        if constexpr (LN) s1 += red[par][0][w][m];
        s2 += red[par][1][w][m];
      }
      if constexpr (LN) c1[m] = s1 * inv_h;
      c2[m] = s2 * inv_h;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int vi = g * NT + tid;
      if (vi < nvec) {
        const int col = vi * 8;
        float gm[8];
        unpack8(gam[g], gm);
        float sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int m = 0; m < TT; ++m) {
          float fx[8], fd[8], r[8], o[8];
          unpack8(wx[g][m], fx);
          unpack8(wd[g][m], fd);
          unpack8(wr[g][m], r);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float xh = (fx[e] - mu[m]) * rs[m];
            const float dxh = fd[e] * gm[e];
            o[e] = r[e] + rs[m] * (LN ? (dxh - c1[m] - xh * c2[m]) : (dxh - xh * c2[m]));
          }
          const long long off = m * plane + i * h + col;
          const uint4 gb = pack8(o);
          if (col < hs) {                 // shared channels: the reduce runs on the ROUNDED residual gradient
            *reinterpret_cast<uint4*>(g_out + off) = gb;
            float f[8];
            unpack8(gb, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] += f[e];
          } else {                        // private channels: nothing reads g_out again in the backward pass
            st_stream(g_out + off, gb);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] *= scale;
            *reinterpret_cast<uint4*>(g_red + off) = pack8(o);
          }
        }
        if (col < hs) {
          const uint4 sb = pack8(sum);    // one rounding, the same bits on every rank
#pragma unroll
          for (int m = 0; m < TT; ++m) *reinterpret_cast<uint4*>(g_red + m * plane + i * h + col) = sb;
        }
      }
    }
  }
  float* prow = partial + (long long)blockIdx.x * 2 * h;
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int vi = g * NT + tid;
    if (vi < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        prow[vi * 8 + e] = dgam[g][e];
        if constexpr (LN) prow[h + vi * 8 + e] = dbet[g][e];
      }
    }
  }
}

// sums partial[nb][2][h] over nb in a fixed order: a workgroup owns 64 columns (a thread 4 of them, one 16-byte
// load per partial row), its 16 row groups each add every 16th partial row (4 independent chains), and the 16 group
// sums are combined in ascending order through LDS.  h % 8 == 0, so 2h is a multiple of 4.  Only the first `ncols`
// columns of a partial row are read and reduced: 2h for LayerNorm (dgamma | dbeta), h for RMSNorm, whose backward
// kernels never write the dbeta half of a partial row (and whose dbeta is never stored).
__global__ __launch_bounds__(256) void norm_bwd_finalize_kernel(const float* __restrict__ partial, int nb, int h,
                                                                int ncols, float* __restrict__ dgamma,
                                                                float* __restrict__ dbeta) {
  __shared__ float4 red[16][16];
  const int cl = threadIdx.x & 15, rg = threadIdx.x >> 4;
  const int c = (blockIdx.x * 16 + cl) * 4;
  const long long w = 2LL * h;
  float4 s[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) s[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  auto add = [](float4& a, const float4& b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; };
  if (c < ncols) {
    int b = rg;
    for (; b + 48 < nb; b += 64) {
      float4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const float4*>(partial + (long long)(b + 16 * k) * w + c);
#pragma unroll
      for (int k = 0; k < 4; ++k) add(s[k], v[k]);
    }
    for (; b < nb; b += 16) add(s[0], *reinterpret_cast<const float4*>(partial + (long long)b * w + c));
  }
  add(s[0], s[1]);
  add(s[2], s[3]);
  add(s[0], s[2]);
  red[rg][cl] = s[0];
  __syncthreads();
  if (rg == 0 && c < ncols) {
    float4 t = red[0][cl];
#pragma unroll
    for (int k = 1; k < 16; ++k) add(t, red[k][cl]);
    const float o[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c + e < h) dgamma[c + e] = o[e];
      else if (dbeta) dbeta[c + e - h] = o[e];
    }
  }
}

static constexpr int NORM_BWD_WIDE_H = 4096;          // rows wider than this take the workgroup-per-row kernel
static constexpr int NORM_BWD_WIDE_MAX_BLOCKS = 1024;
static long long norm_bwd_blocks(long long rows, int h) {
  long long nb;
  if (h > NORM_BWD_WIDE_H) {
    nb = (rows + 7) / 8;                             // at least 8 rows per workgroup
    if (nb > NORM_BWD_WIDE_MAX_BLOCKS) nb = NORM_BWD_WIDE_MAX_BLOCKS;
  } else {
    nb = (rows + 3) / 4;
    if (nb > NORM_BWD_MAX_BLOCKS) nb = NORM_BWD_MAX_BLOCKS;
  }
  if (nb < 1) nb = 1;
  return nb;
}

size_t norm_bwd_workspace_bytes(int T, long long tokens, int h) {
  return (size_t)norm_bwd_blocks((long long)T * tokens, h) * 2 * (size_t)h * sizeof(float);
}

template <int VPL>
static hipError_t norm_bwd_wide_dispatch(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                                         const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_scaled,
                                         float* partial, int norm, long long rows, int h, int hs, float scale,
                                         long long nb, long long rpb, int skip_shared, hipStream_t s) {
  if (norm == 0)
    hipLaunchKernelGGL((norm_bwd_wide_kernel<VPL, true>), dim3((unsigned)nb), dim3(256), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_scaled, partial, rows, h, hs, scale, rpb, skip_shared);
  else
    hipLaunchKernelGGL((norm_bwd_wide_kernel<VPL, false>), dim3((unsigned)nb), dim3(256), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_scaled, partial, rows, h, hs, scale, rpb, skip_shared);
  return hipGetLastError();
}

template <int VPL>
static hipError_t norm_bwd_dispatch(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                                    const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_scaled,
                                    float* partial, int norm, long long rows, int h, int hs, float scale, long long nb,
                                    long long rpb, int skip_shared, hipStream_t s) {
  if (norm == 0)
    hipLaunchKernelGGL((norm_bwd_kernel<VPL, true>), dim3((unsigned)nb), dim3(256), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_scaled, partial, rows, h, hs, scale, rpb, skip_shared);
  else
    hipLaunchKernelGGL((norm_bwd_kernel<VPL, false>), dim3((unsigned)nb), dim3(256), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_scaled, partial, rows, h, hs, scale, rpb, skip_shared);
  return hipGetLastError();
}

hipError_t launch_norm_bwd(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                           const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_scaled, float* dgamma,
                           float* dbeta, int norm, int T, long long tokens, int h, int hs, float private_scale,
                           void* workspace, hipStream_t s, bool skip_shared_scaled) {
  const long long rows = (long long)T * tokens;
  const int skip_shared = (skip_shared_scaled && g_scaled != nullptr && hs % 8 == 0) ? 1 : 0;
  if (rows == 0) return hipSuccess;
  long long nb = norm_bwd_blocks(rows, h);
  const long long rpb = (rows + nb - 1) / nb;
  nb = (rows + rpb - 1) / rpb;                       // no empty workgroups: every partial row is written
  float* partial = reinterpret_cast<float*>(workspace);
  const int vpl = (h / 8 + 63) / 64;
  hipError_t e;
  if (h > NORM_BWD_WIDE_H) {
    const int vw = (h / 8 + 255) / 256;
    if (vw <= 2) e = norm_bwd_wide_dispatch<2>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
    else if (vw <= 4) e = norm_bwd_wide_dispatch<4>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
    else return hipErrorInvalidValue;
  } else if (vpl <= 1) e = norm_bwd_dispatch<1>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
  else if (vpl <= 2) e = norm_bwd_dispatch<2>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
  else if (vpl <= 4) e = norm_bwd_dispatch<4>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
  else if (vpl <= 8) e = norm_bwd_dispatch<8>(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, partial, norm, rows, h, hs, private_scale, nb, rpb, skip_shared, s);
  else return hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  const int ncols = norm == 0 ? 2 * h : h;           // RMSNorm has no dbeta: that half of a partial row is never written
  hipLaunchKernelGGL(norm_bwd_finalize_kernel, dim3((unsigned)((ncols + 63) / 64)), dim3(256), 0, s, partial, (int)nb,
                     h, ncols, dgamma, norm == 0 ? dbeta : nullptr);
  return hipGetLastError();
}

// Shapes the fused norm backward + reduce takes: a thread (of 256) holds x, dy and dres of its column groups for all T
// rows of a token, and the kernel only beats the two separate kernels while that is at most 4 (rank, column group)
// pairs per input (T = 4 up to h = 2048, T = 2 up to h = 4096).  Measured beyond that budget, T = 8 and h = 4096 with
// 256, 512 or 1024 threads: 327 - 354 us against 279 us for the two kernels (every register of a one-wave-per-SIMD
// budget, or spills), so those shapes keep the two kernels.
static int norm_bwd_sync_groups(int T, int h) {
  const int ng = (h / 8 + 255) / 256;
  return ((T == 2 || T == 4) && T * ng <= 4) ? ng : 0;
}
bool norm_bwd_sync_takes(int T, long long tokens, int h, int hs) {
  if (hs <= 0 || hs % 8 != 0 || hs > h || h % 8 != 0 || h > 8192 || tokens <= 0) return false;
  return norm_bwd_sync_groups(T, h) != 0;
}

template <int TT, int NG, int NT>
static hipError_t norm_bwd_sync_dispatch(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                                         const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_red, float* partial,
                                         int norm, long long tokens, int h, int hs, float scale, long long nb, long long tpb,
                                         hipStream_t s) {
  if (norm == 0)
    hipLaunchKernelGGL((norm_bwd_sync_kernel<TT, NG, true, NT>), dim3((unsigned)nb), dim3(NT), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_red, partial, tokens, h, hs, scale, tpb);
  else
    hipLaunchKernelGGL((norm_bwd_sync_kernel<TT, NG, false, NT>), dim3((unsigned)nb), dim3(NT), 0, s, dy, dres, x, gamma, mean,
                       rstd, g_out, g_red, partial, tokens, h, hs, scale, tpb);
  return hipGetLastError();
}

// g_out = dres + NormBwd(dy) per rank (un-reduced); g_red = the partial channel-reduce of g_out (shared channels summed
// over ranks, private channels scaled); dgamma / dbeta summed over tokens and ranks.  The workspace is the one
// launch_norm_bwd takes (at most 512 partial rows are used).  hipErrorInvalidValue for shapes not taken.
hipError_t launch_norm_bwd_sync(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                                const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_red, float* dgamma,
                                float* dbeta, int norm, int T, long long tokens, int h, int hs, float private_scale,
                                void* workspace, hipStream_t s) {
  if (!norm_bwd_sync_takes(T, tokens, h, hs)) return hipErrorInvalidValue;
  // as many partial rows as the row-wise kernels would use for this shape at most, so that the same workspace serves
  long long nb = norm_bwd_blocks((long long)T * tokens, h);
  if (nb > NORM_BWD_MAX_BLOCKS) nb = NORM_BWD_MAX_BLOCKS;
  if (nb > tokens) nb = tokens;
  const long long tpb = (tokens + nb - 1) / nb;
  nb = (tokens + tpb - 1) / tpb;                     // no empty workgroups: every partial row is written
  float* partial = reinterpret_cast<float*>(workspace);
  const int ng = norm_bwd_sync_groups(T, h);
  hipError_t e = hipErrorInvalidValue;
#define CAAT_NBS(TT_, NG_) e = norm_bwd_sync_dispatch<TT_, NG_, 256>(dy, dres, x, gamma, mean, rstd, g_out, g_red, partial, norm, tokens, h, hs, private_scale, nb, tpb, s)
  if (T == 2 && ng == 1) CAAT_NBS(2, 1);
  else if (T == 2 && ng == 2) CAAT_NBS(2, 2);
  else if (T == 4 && ng == 1) CAAT_NBS(4, 1);
#undef CAAT_NBS
  if (e != hipSuccess) return e;
  const int ncols = norm == 0 ? 2 * h : h;
  hipLaunchKernelGGL(norm_bwd_finalize_kernel, dim3((unsigned)((ncols + 63) / 64)), dim3(256), 0, s, partial, (int)nb,
                     h, ncols, dgamma, norm == 0 ? dbeta : nullptr);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// HBM streaming probe (measuring tool): read or copy a buffer with a chosen access pattern and cache hint.
template <bool CHUNK, bool NTL, bool COPY, bool NTS>
__global__ __launch_bounds__(256) void hbm_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                        long long nvec, long long vec_per_wg) {
  constexpr int U = 4;   // 16-byte loads in flight per thread
  const long long begin = CHUNK ? (long long)blockIdx.x * vec_per_wg : 0;
  const long long end = CHUNK ? (begin + vec_per_wg < nvec ? begin + vec_per_wg : nvec) : nvec;
  const long long first = CHUNK ? begin + threadIdx.x : (long long)blockIdx.x * 256 + threadIdx.x;
  const long long step = CHUNK ? 256 : (long long)gridDim.x * 256;
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  for (long long i = first; i < end; i += step * U) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long j = i + u * step;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (j < end) v[u] = NTL ? ld_stream(src + j) : src[j];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long j = i + u * step;
      if (COPY) {
        if (j < end) {
          if (NTS) st_stream(dst + j, v[u]);
          else dst[j] = v[u];
        }
      } else {
        acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
      }
    }
  }
  if (!COPY && dst != nullptr && acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u) dst[0] = acc;   // keeps the loads alive
}

hipError_t launch_hbm_probe(const void* src, void* dst, size_t bytes, int mode, hipStream_t s) {
  const long long nvec = (long long)(bytes / 16);
  if (nvec == 0) return hipSuccess;
  const uint4* a = reinterpret_cast<const uint4*>(src);
  uint4* b = reinterpret_cast<uint4*>(dst);
  long long wgs = 8192;
  if (wgs > (nvec + 255) / 256) wgs = (nvec + 255) / 256;
  const long long vpw = (nvec + wgs - 1) / wgs;
  switch (mode) {
    case 0: hipLaunchKernelGGL((hbm_probe_kernel<true, false, false, false>), dim3((unsigned)wgs), dim3(256), 0, s, a, b, nvec, vpw); break;
    case 1: hipLaunchKernelGGL((hbm_probe_kernel<true, true, false, false>), dim3((unsigned)wgs), dim3(256), 0, s, a, b, nvec, vpw); break;
    case 2: hipLaunchKernelGGL((hbm_probe_kernel<false, false, false, false>), dim3(4096), dim3(256), 0, s, a, b, nvec, vpw); break;
    case 3: hipLaunchKernelGGL((hbm_probe_kernel<true, false, true, false>), dim3((unsigned)wgs), dim3(256), 0, s, a, b, nvec, vpw); break;
    case 4: hipLaunchKernelGGL((hbm_probe_kernel<true, true, true, true>), dim3((unsigned)wgs), dim3(256), 0, s, a, b, nvec, vpw); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace caat
