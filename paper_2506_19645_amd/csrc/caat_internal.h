// Internal declarations shared by the HIP translation units of libcaat (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace caat {

typedef unsigned short bf16_t;  // raw bfloat16 bit pattern in memory

__device__ __forceinline__ float bf2f(bf16_t u) { return __uint_as_float(((unsigned)u) << 16); }

// fp32 -> bf16, round-to-nearest-even: gfx950's v_cvt_pk_bf16_f32 (two values per instruction)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack2bf(float lo, float hi) {
  const bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack2bf(f, 0.0f) & 0xFFFFu); }
__device__ __forceinline__ float lo_bf(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

// Exact (erf-form) GELU x*Phi(x) and its derivative Phi(x) + x*phi(x), evaluated with one hardware exponential
// and a short polynomial each (the activation runs in the GEMM epilogues, where every VALU cycle is exposed).
// With a = |x|: the lower tail is Phi(-a) = 2^r(a), r a degree-5 minimax fit of log2 Phi(-a) on [0, 5.5]
// (relative error of the tail <= 2.5e-4, an eighth of bf16's rounding step, also where the tail is tiny);
// gelu(x) = x*Phi(-a) for x <= 0 and x - x*Phi(-a) for x > 0, i.e. max(x, 0) - a*Phi(-a) for both signs (one
// maximum and one fused multiply-add instead of a product, a difference, a comparison and a select).  Beyond 5.5
// the polynomial keeps falling (its leading coefficient is negative), so the tail runs smoothly into 0 (absolute
// error of gelu there < 1e-7).
__device__ __forceinline__ float gelu_f(float x) {
  const float a = fabsf(x);
  float r = -0.000233251485f;
  r = r * a + 0.00486977212f;
  r = r * a - 0.0445989817f;
  r = r * a - 0.469681203f;
  r = r * a - 1.14626062f;
  r = r * a - 1.00035918f;
  return __builtin_fmaf(-a, __builtin_amdgcn_exp2f(r), fmaxf(x, 0.0f));
}
// The derivative on the negative side is u(a) = Phi(-a) - a*phi(a) = phi(a)*(m(a) - a) with Mills' ratio
// m = Phi(-a)/phi(a); (m(a) - a)/sqrt(2 pi) is a smooth function fitted by a degree-6 polynomial weighted with
// phi (absolute error of the derivative <= 1.6e-5); gelu'(x) = u(a) for x <= 0 and 1 - u(a) for x > 0.
__device__ __forceinline__ float gelu_grad_f(float x) {
  const float a = fminf(fabsf(x), 14.0f);  // exp(-a^2/2) is 0 in fp32 from here on; keeps a^2 and m finite
  float m = 0.000704242266f;
  m = m * a - 0.00804199837f;
  m = m * a + 0.0396726206f;
  m = m * a - 0.116941683f;
  m = m * a + 0.244423941f;
  m = m * a - 0.797151923f;
  m = m * a + 0.499984324f;
  const float u = __builtin_amdgcn_exp2f(-0.72134752f * (a * a)) * m;  // exp(-a^2/2) * (m(a) - a)/sqrt(2 pi)
  return x > 0.0f ? 1.0f - u : u;
}
__device__ __forceinline__ float sigmoid_f(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// ---------------------------------------------------------------- global -> LDS copies
// Raw buffer descriptor over [p, p + 2 GiB): offsets >= 0x80000000 are out of range and read as zero.
typedef int i32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4_t make_rsrc(const void* p) {
  const unsigned long long a = (unsigned long long)p;
  i32x4_t r;
  r.x = (int)(unsigned)a;
  r.y = (int)((unsigned)(a >> 32) & 0xFFFFu);
  r.z = (int)0x80000000;
  r.w = 0x00020000;
  return r;
}
// The same window as a compiler-level buffer resource, for raw buffer loads / stores issued through builtins.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_t make_rsrc_t(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)0x80000000, 0x00020000);
}
__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const char*)p;
}
// One global -> LDS copy instruction: lane L's 16 bytes from rs[voff] land at lds_wave_uniform + 16*L.
// Written as inline assembly on purpose: the compiler then does not know that LDS is written by a vector-memory
// operation and does not force "wait for every outstanding copy" in front of each later LDS read; the kernel
// orders copies and reads itself (wait_vmcnt + barrier), which is what lets NSTAGE-1 stages stay in flight.
// The copy takes its LDS base from M0.  M0 is a reserved register for this compiler (it cannot be named in a clobber
// list), so every statement saves M0 into a scalar temporary first and puts it back after its last copy: from the
// compiler's point of view M0 is unchanged, whatever it keeps there (indirect register indexing, lane reads).  The
// copies read M0 when they issue, in order, so the restoring move right behind them is safe.
// STREAM: non-temporal hint, for bytes that no other workgroup will ask for (a read-once stream keeps 7.1 TB/s
// against 6.2 TB/s without the hint); operands that several workgroups share stay cacheable.
template <bool STREAM = false>
__device__ __forceinline__ void dma16(i32x4_t rs, unsigned voff, const uint4* lds_wave_uniform) {
  unsigned keep;  // M0 as the compiler left it
  if constexpr (STREAM)
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(keep)
                 : "v"(voff), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                 : "memory");
  else
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(keep)
                 : "v"(voff), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                 : "memory");
}

// G copies (1, 2 or 4) whose LDS destinations lie 1 KB apart, written with one LDS base: the instruction's immediate
// offset o moves BOTH sides of a copy (memory address and LDS address) by o bytes, so copy number i of the group
// takes offset 1024 i, and its memory-side offset v[i] must have those 1024 i bytes taken off beforehand.  Saves
// the M0 write and its wait state on all but the first copy of a group.
template <bool STREAM, int G>
__device__ __forceinline__ void dma16_group(i32x4_t rs, const unsigned* v, const uint4* lds_wave_uniform) {
  static_assert(G == 1 || G == 2 || G == 4, "group of 1, 2 or 4 copies");
  unsigned keep;
  if constexpr (G == 1) {
    dma16<STREAM>(rs, v[0], lds_wave_uniform);
  } else if constexpr (G == 2) {
    if constexpr (STREAM)
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %3, 0 offen nt lds\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 nt lds\n\t"
                   "s_mov_b32 m0, %0"
                   : "=&s"(keep)
                   : "v"(v[0]), "v"(v[1]), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                   : "memory");
    else
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 lds\n\t"
                   "s_mov_b32 m0, %0"
                   : "=&s"(keep)
                   : "v"(v[0]), "v"(v[1]), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                   : "memory");
  } else {
    if constexpr (STREAM)
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %6\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %5, 0 offen nt lds\n\t"
                   "buffer_load_dwordx4 %2, %5, 0 offen offset:1024 nt lds\n\t"
                   "buffer_load_dwordx4 %3, %5, 0 offen offset:2048 nt lds\n\t"
                   "buffer_load_dwordx4 %4, %5, 0 offen offset:3072 nt lds\n\t"
                   "s_mov_b32 m0, %0"
                   : "=&s"(keep)
                   : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                   : "memory");
    else
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %6\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %5, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %5, 0 offen offset:1024 lds\n\t"
                   "buffer_load_dwordx4 %3, %5, 0 offen offset:2048 lds\n\t"
                   "buffer_load_dwordx4 %4, %5, 0 offen offset:3072 lds\n\t"
                   "s_mov_b32 m0, %0"
                   : "=&s"(keep)
                   : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "s"(rs), "s"(lds_addr(lds_wave_uniform))
                   : "memory");
  }
}

// 16-byte load of data that this kernel reads once (non-temporal hint: see dma16)
__device__ __forceinline__ uint4 ld_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}

// 16-byte store of data that nothing reads again soon
__device__ __forceinline__ void st_stream(void* p, const uint4& v) {
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(p));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---------------------------------------------------------------- GEMM
enum GemmEpilogue {
  EPI_PLAIN = 0,       // c = acc
  EPI_GELU_FWD = 1,    // c = acc (pre-activation P), c2 = gelu(acc)
  EPI_SWIGLU_FWD = 2,  // b holds gate rows then up rows; c = [gate|up] pre-activations, c2 = silu(gate)*up
  EPI_ROWPAR = 3,      // col < hs: c = acc (partial sum);  col >= hs: c = scale*acc + resid
  EPI_GELU_BWD = 4,    // c = acc * gelu'(aux)
  EPI_SWIGLU_BWD = 5,  // c[:, col] = acc*up*silu'(gate), c[:, half+col] = acc*silu(gate); aux = [gate|up]
  EPI_SHARED_BCAST = 6 // for m in [0, bcast): c[m] = round_bf16(acc) + aux[m]   (c, aux advance by stride_c / stride_aux)
};

struct GemmParams {
  const bf16_t* a;
  const bf16_t* b;
  bf16_t* c;
  bf16_t* c2;          // second output (EPI_*_FWD)
  const bf16_t* aux;   // saved pre-activations (EPI_*_BWD) or residual (EPI_ROWPAR)
  long long lda, ldb, ldc, ldc2, ldaux;
  long long stride_a, stride_b, stride_c, stride_c2, stride_aux;  // per group, elements
  int G;
  int M, N, K;         // N = number of output columns of the accumulator tile grid (for SWIGLU_FWD: ffn/T)
  int half;            // SWIGLU: ffn/T (offset between gate and up columns / rows)
  int hs;              // EPI_ROWPAR
  float scale;         // EPI_ROWPAR private scale
  int kcat;            // > 1: the contraction runs over kcat operand pairs, K each, kstride_* elements apart
  long long kstride_a, kstride_b;
  int bcast;           // EPI_SHARED_BCAST: number of output copies (ranks)
  int late_c;          // EPI_PLAIN: c is not read again soon (weight / input gradients): store it with the non-temporal hint
  int bn_out;          // decode-sized tiles: output columns one tile covers (0 = the tile's full width); set by launch_gemm
};

// layout: 0 NT, 1 NN, 2 TN (see caat_gemm_layout).  Returns hipError_t of the launch.
hipError_t launch_gemm(const GemmParams& p, int layout, int epilogue, hipStream_t s);

// ---------------------------------------------------------------- streaming kernels
hipError_t launch_partial_sync(const bf16_t* y, const bf16_t* resid, bf16_t* out, int T, long long tokens, int h,
                               int hs, float private_scale, hipStream_t s);
hipError_t launch_partial_sync_shared(bf16_t* io, const bf16_t* resid, int T, long long tokens, int h, int hs,
                                      hipStream_t s);
hipError_t launch_norm_fwd(const bf16_t* x, const bf16_t* gamma, const bf16_t* beta, bf16_t* y, float* mean,
                           float* rstd, int norm, int T, long long tokens, int h, float eps, hipStream_t s,
                           int dedup_hs = 0);
// reduce on the shared channels + residual + norm in one launch (hs % 8 == 0; T in {2,4,8} with h <= 8192, T = 16 with
// h <= 4096: sync_norm_takes); hipErrorInvalidValue if the shape is not taken
bool sync_norm_takes(int T, long long tokens, int h, int hs);
hipError_t launch_sync_norm(bf16_t* io, const bf16_t* resid, const bf16_t* gamma, const bf16_t* beta, bf16_t* xout,
                            float* mean, float* rstd, int norm, int T, long long tokens, int h, int hs, float eps,
                            hipStream_t s);
size_t norm_bwd_workspace_bytes(int T, long long tokens, int h);
hipError_t launch_norm_bwd(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                           const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_scaled, float* dgamma,
                           float* dbeta, int norm, int T, long long tokens, int h, int hs, float private_scale,
                           void* workspace, hipStream_t s, bool skip_shared_scaled = false);
// norm backward + the backward partial channel-reduce in one launch (hs % 8 == 0; T = 4 up to h = 2048, T = 2 up to
// h = 4096: norm_bwd_sync_takes); hipErrorInvalidValue if the shape is not taken.  Same workspace as launch_norm_bwd.
bool norm_bwd_sync_takes(int T, long long tokens, int h, int hs);
hipError_t launch_norm_bwd_sync(const bf16_t* dy, const bf16_t* dres, const bf16_t* x, const bf16_t* gamma,
                                const float* mean, const float* rstd, bf16_t* g_out, bf16_t* g_red, float* dgamma,
                                float* dbeta, int norm, int T, long long tokens, int h, int hs, float private_scale,
                                void* workspace, hipStream_t s);
// shared channels of dst = sum over ranks of src's; dst's other channels are not touched (hs % 8 == 0)
hipError_t launch_partial_sync_shared_from(const bf16_t* src, bf16_t* dst, int T, long long tokens, int h, int hs,
                                           hipStream_t s);

hipError_t launch_hbm_probe(const void* src, void* dst, size_t bytes, int mode, hipStream_t s);   // measuring tool

// ---------------------------------------------------------------- attention core
// Projections of one rank-row: [heads*128 q | kv_heads*128 k | kv_heads*128 v] (grouped-query attention when
// kv_heads < heads; heads, kv_heads are per rank); ld = (heads + 2*kv_heads)*128.
hipError_t launch_rope(bf16_t* qkv, long long rows, int seq, int ld, int n_rot, int d, float base, long long pos0,
                       bool inverse, hipStream_t s);
hipError_t launch_rope_append(bf16_t* qkv, bf16_t* kc, bf16_t* vc, long long n_seq, int seq, int hpr, int kvpr, int d,
                              float base, long long cap, long long pos0, hipStream_t s);   // RoPE + KV cache store in one pass
size_t attn_stats_bytes(long long n_seq, int heads, int seq);   // fp32 [n_seq*heads][2][seq rounded up to 64]: lse, D
hipError_t launch_flash_fwd(const bf16_t* qkv, bf16_t* out, float* stats, long long n_seq, int seq, int heads, int kv_heads,
                            int d, hipStream_t s);
hipError_t launch_flash_bwd(const bf16_t* qkv, const bf16_t* out, const bf16_t* dout, float* stats, bf16_t* dqkv,
                            long long n_seq, int seq, int heads, int kv_heads, int d, hipStream_t s);
hipError_t launch_decode_attn(const bf16_t* qkv, bf16_t* kc, bf16_t* vc, bf16_t* out, long long n_seq, int hpr,
                              int kvpr, int d, long long cap, long long nkeys, float rope_base, hipStream_t s);

}  // namespace caat
