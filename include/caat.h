/*
 * caat.h -- C ABI of the MI355X (gfx950) partial-sync tensor-parallel block library.
 *
 * The library computes the hot path of CAAT-Net ("Tensor-Parallelism with Partially Synchronized
 * Activations"): a tensor-parallel transformer sub-block whose row-parallel outputs are summed over
 * the T tensor-parallel ranks only on the first hs = floor(h*p) hidden channels ("shared" channels)
 * and stay rank-local on the others ("private" channels) -- Sec. 3, Eq. A3 (MLP) and Eq. A5
 * (attention) -- followed by the residual add and the per-rank normalisation of Sec. 4, forward and
 * backward.  All T ranks live on ONE GPU (the "logical devices" of Sec. 3.2), so the reduce over
 * ranks is a reduction in HBM.
 *
 * Conventions that hold for every entry point
 *  - Every pointer is a DEVICE pointer unless it is said to be a host pointer.  The caller owns
 *    every buffer; the library never allocates or frees device memory.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *    on that stream and return without waiting for it.
 *  - The return value is a caat_status.  Argument errors are detected on the host before anything
 *    is launched and leave all outputs untouched.
 *  - Storage is bf16 (IEEE bfloat16 bit patterns, 2 bytes) unless stated; accumulation is fp32;
 *    results are rounded to bf16 once, round-to-nearest-even.
 *  - Tensors are row-major with the rank index outermost: an activation is [T, tokens, h].
 *    Weight shards use the [out_features, in_features] convention per rank.
 *  - Device pointers must be 16-byte aligned; h, ffn/T and (n_heads/T)*head_dim must be multiples
 *    of 8.  hs may be any integer in [0, h].
 *  - Calls that overlap in time must not share output or workspace buffers.
 */
#ifndef CAAT_H
#define CAAT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum caat_status {
  CAAT_OK = 0,
  CAAT_EINVAL = 1,      /* null pointer, T < 1, p outside [0,1] or NaN, unknown enum value */
  CAAT_ESHAPE = 2,      /* ffn % T, n_heads % T, hs > h, a dimension that is not a multiple of 8 ... */
  CAAT_EALIGN = 3,      /* a device pointer is not 16-byte aligned */
  CAAT_EWORKSPACE = 4,  /* workspace smaller than caat_workspace_bytes() */
  CAAT_EHIP = 5,        /* a HIP runtime call (kernel launch) reported an error */
  CAAT_EUNSUPPORTED = 6,/* valid request that this build does not implement */
  CAAT_ESCRATCH = 7     /* caat_norm_bwd_static only: the problem needs more than the library's fixed device scratch */
} caat_status;

typedef enum caat_kind {
  CAAT_MLP_GELU = 0,    /* Y = gelu(X A),               LayerNorm or RMSNorm after the residual */
  CAAT_MLP_SWIGLU = 1,  /* Y = silu(X Wg) * (X Wu) */
  CAAT_ATTN = 2,        /* causal multi-head attention with RoPE, prefill / training forward and backward */
  CAAT_ATTN_DECODE = 3, /* full decoder layer (attention + SwiGLU MLP), one new token per sequence */
  CAAT_LAYER_PREFILL = 4 /* the same decoder layer over a whole prompt (batch x seq tokens) that fills the KV cache:
                            the time-to-first-token workload of Sec. 5.2; forward only */
} caat_kind;

typedef enum caat_norm { CAAT_LAYERNORM = 0, CAAT_RMSNORM = 1 } caat_norm;

/* Operand layouts of caat_gemm_bf16: which index of each operand is contiguous in memory. */
typedef enum caat_gemm_layout {
  CAAT_GEMM_NT = 0, /* a[M][K], b[N][K]  (forward GEMMs: activation x weight[out,in]^T)          */
  CAAT_GEMM_NN = 1, /* a[M][K], b[K][N]  (data gradients: grad x weight[out,in])                 */
  CAAT_GEMM_TN = 2  /* a[K][M], b[K][N]  (weight gradients: reduction over tokens)               */
} caat_gemm_layout;

/*
 * Problem statement of one block call, following the paper's notation: hidden size h, tensor-
 * parallel degree T (the paper's r), synchronisation factor p entering only through
 * hs = floor(h*p) (Eq. A3), tokens = batch*seq.
 */
typedef struct caat_desc {
  int kind;             /* caat_kind */
  int norm;             /* caat_norm */
  int h;                /* hidden size */
  int ffn;              /* FFN size f over ALL ranks (each rank owns ffn/T columns); 0 for CAAT_ATTN */
  int T;                /* number of emulated tensor-parallel ranks */
  int hs;               /* number of shared channels, 0 <= hs <= h; see caat_shared_channels() */
  long long tokens;     /* batch*seq */
  int batch, seq;       /* attention kinds need both; MLP kinds only use tokens */
  int n_heads, head_dim;/* attention kinds; each rank owns n_heads/T heads */
  long long kv_len;     /* decode: number of filled cache positions; the new token sits at kv_len.  prefill: 0 */
  long long kv_cap;     /* decode: capacity (positions) of the cache buffers, > kv_len; prefill: >= seq */
  float eps;            /* norm epsilon */
  float private_scale;  /* factor applied to private channels (Sec. 4 private channel scaling,
                           sqrt(T) in the paper); 1.0f switches it off */
  float rope_base;      /* RoPE base (10000) */
  int n_kv_heads;       /* grouped-query attention: key / value heads over all ranks; 0 = n_heads (multi-head).
                           n_heads % n_kv_heads == 0 and n_kv_heads % T == 0 (each rank owns whole groups) */
  int reduce_in_gemm;   /* forward only.  0: every rank's partial sum on the shared channels is written out and a reduce
                           pass sums them (the in-HBM stand-in for the tensor-parallel collective).  1: single-device
                           serving with logical ranks (Sec. 3.2, the reduce becomes a local summation): the shared
                           channels come from one GEMM whose contraction runs over all T ranks, so the sum is taken in
                           the accumulator, no partial sum reaches memory and no reduce pass runs.  Needs hs % 8 == 0
                           and more than 64 tokens (otherwise the default path is taken: a decode-sized GEMM has too few
                           tiles once the ranks are folded into the contraction).  Same result up to the rounding of the partials. */
  int dedup_shared;     /* forward only, needs reduce_in_gemm = 1, hs % 8 == 0, more than 64 tokens, not the decode kind
                           (CAAT_EUNSUPPORTED otherwise).  1: the residual-stream tensors r and r_out (and the layer
                           kinds' internal residual) store the shared channels ONCE instead of T identical copies:
                           [tokens, hs] followed by the private channels [T, tokens, h - hs], one contiguous buffer of
                           tokens*hs + T*tokens*(h-hs) elements.  x / x_out keep the [T, tokens, h] layout. */
  int separate_reduce;  /* 0: where the shape allows (see caat_partial_sync_norm_fwd) the reduce over ranks, the residual
                           add and the norm that follows run as ONE kernel, which does not read the reduced channels
                           back from memory.  1: the reduce stays a kernel of its own (caat_partial_sync's kernel, the
                           in-HBM stand-in for the tensor-parallel collective, whose time against p is what the
                           benchmark's sweep reports) followed by the norm kernel.  Same values either way.  The
                           backward pass does likewise: norm backward and the reduce on its result are one kernel
                           (0, for T = 4 up to h = 2048 and T = 2 up to h = 4096 with hs % 8 == 0) or two (1, and
                           every other shape). */
} caat_desc;

/* Byte offsets of the tensors caat_block_fwd leaves in the workspace (0 size = not present).  For tests
 * and for callers that want the saved activations; everything else in the workspace is scratch. */
typedef struct caat_ws_layout {
  size_t total_bytes;
  size_t off_P, bytes_P;       /* pre-activations: [T,tokens,ffn/T] (GELU) or [T,tokens,2*ffn/T] gate|up (SwiGLU) */
  size_t off_Y, bytes_Y;       /* sigma output [T,tokens,ffn/T]; attention kinds: heads output H [T,tokens,hd_r] */
  size_t off_mean, bytes_mean; /* fp32 [T,tokens] (LayerNorm only) */
  size_t off_rstd, bytes_rstd; /* fp32 [T,tokens] */
  size_t off_dZt, bytes_dZt;   /* backward: reduced gradient [T,tokens,h] */
  size_t off_dP, bytes_dP;     /* backward: gradient of the pre-activations, same shape as P; CAAT_ATTN: gradient of the
                                  un-rotated projections [T,tokens,hd_r+2*kvd_r], column blocks dq | dk | dv */
  size_t off_Q, bytes_Q;       /* attention: projections [T,tokens,hd_r+2*kvd_r], column blocks q | k | v, q and k rotated (RoPE) */
  size_t off_scratch, bytes_scratch;
  /* decode and prefill layers only: attention heads output [T,tokens,hd_r]; first norm output X1, residual after the
   * attention half R1 and second norm output X2, each [T,tokens,h] */
  size_t off_H, bytes_H;
  size_t off_X1, bytes_X1;
  size_t off_R1, bytes_R1;
  size_t off_X2, bytes_X2;
  /* CAAT_ATTN only: fp32 per-query softmax statistics [T*batch*n_heads/T][2][seq rounded up to 64] (row 0: log2-domain
   * log-sum-exp of the scaled scores, saved by the forward; row 1: sum_d dH*H, written by the backward), and the
   * backward's gradient of the heads output dH [T,tokens,hd_r] */
  size_t off_stats, bytes_stats;
  size_t off_dH, bytes_dH;
} caat_ws_layout;

/* Sec. 3 / Eq. A3: number of shared channels floor(h*p), evaluated in IEEE double.  Host function.
 * Returns -1 if h < 0 or p is NaN or outside [0,1]. */
int caat_shared_channels(int h, double p);

/* Static, NUL-terminated description of a caat_status; never freed by the caller.  Host function. */
const char* caat_status_string(int status);

/* Workspace (bytes) that caat_block_fwd / caat_block_bwd need for `d` (host pointer).  0 on an invalid
 * descriptor.  caat_workspace_layout fills `out` (host pointer) and returns a caat_status. */
size_t caat_workspace_bytes(const caat_desc* d);
int caat_workspace_layout(const caat_desc* d, caat_ws_layout* out);

/*
 * Partial channel-reduce (Eq. A3 / A5, second line) plus optional residual (Sec. 4):
 *   out[m,i,l] = sum_{m'} y[m',i,l]            + resid[m,i,l]   for l <  hs   (shared)
 *   out[m,i,l] = private_scale * y[m,i,l]      + resid[m,i,l]   for l >= hs   (private)
 * y, resid, out: [T, tokens, h] bf16.  resid may be NULL (no residual; this is the backward reduce
 * of Fig. 2b, accumulated in fp32).  out may alias y exactly (in place); then, if resid is NULL and
 * private_scale == 1, only the hs shared columns are read and written, so HBM traffic is
 * 4*T*hs bytes per token, proportional to p.  The sum runs over ranks in ascending order in fp32 and
 * is rounded once, so the shared channels are bit-identical on all ranks.
 */
int caat_partial_sync(const void* y, const void* resid, void* out, int T, long long tokens, int h, int hs,
                      float private_scale, void* hip_stream);

/*
 * Per-rank, per-token normalisation (the Norm of Sec. 4): x, y [T,tokens,h] bf16; gamma, beta [h] bf16
 * (beta NULL for RMSNorm); mean (LayerNorm only, may be NULL for RMSNorm) and rstd: [T,tokens] fp32 outputs.
 */
int caat_norm_fwd(const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                  int norm, int T, long long tokens, int h, float eps, void* hip_stream);

/*
 * The shared half of the partial channel-reduce, the residual add and the norm in one launch (Eq. A3 / A5 second
 * line + Sec. 4: X'_m = Norm(R_m + Z_m)), the unit the block calls use after a row-parallel GEMM whose epilogue has
 * already finished the private channels:
 *   io [T,tokens,h] on entry : channels l <  hs: rank m's partial sum Zt_m[:,l];  l >= hs: the final R'_m[:,l]
 *   io on return             : R'_m everywhere: for l < hs  sum_{m'} Zt_m'[:,l] + resid[m,:,l] (fp32 sum in ascending
 *                              rank order, residual added, rounded once)
 *   x_out [T,tokens,h]       : Norm(R'_m) with gamma (and beta for LayerNorm, NULL for RMSNorm)
 *   mean (LayerNorm; may be NULL), rstd : [T,tokens] fp32
 * resid [T,tokens,h] is read on the shared channels only.  Shapes taken: hs > 0 and hs % 8 == 0, T in {2,4,8} with
 * h <= 8192, or T = 16 with h <= 4096 (a thread keeps its columns of all T rows in registers); anything else
 * returns CAAT_EUNSUPPORTED and the caller runs caat_partial_sync and caat_norm_fwd instead.
 */
int caat_partial_sync_norm_fwd(void* io, const void* resid, const void* gamma, const void* beta, void* x_out,
                               float* mean, float* rstd, int norm, int T, long long tokens, int h, int hs, float eps,
                               void* hip_stream);

/*
 * Backward of the norm placed BEFORE the reduce (Sec. 4, Fig. 2b):
 *   g[m] = dres[m] + NormBwd(dy[m]; x[m], gamma)                (dres may be NULL)
 * g is written to `g_out` (the un-reduced residual gradient, App. B) and, if `g_scaled` is not NULL,
 * also to `g_scaled` with its private columns (l >= hs) multiplied by private_scale -- the buffer the
 * backward partial channel-reduce then runs on in place.  dgamma/dbeta: [h] fp32, summed over tokens AND
 * over ranks in a fixed order (Sec. 4: norm parameters are replicated, their gradients reduced).
 * dbeta is neither read nor written for RMSNorm (may be NULL).  workspace: at least caat_norm_bwd_workspace_bytes() bytes.
 */
size_t caat_norm_bwd_workspace_bytes(int T, long long tokens, int h);
int caat_norm_bwd(const void* dy, const void* dres, const void* x, const void* gamma, const float* mean,
                  const float* rstd, void* g_out, void* g_scaled, float* dgamma, float* dbeta, int norm, int T,
                  long long tokens, int h, int hs, float private_scale, void* workspace, size_t ws_bytes,
                  void* hip_stream);

/*
 * caat_norm_bwd for callers that cannot allocate device memory or size a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * caat_norm_bwd, minus `workspace` / `ws_bytes`: the per-workgroup partial sums of dgamma / dbeta go to a fixed
 * 16 MiB device array inside the library (one copy per GPU, held until the process ends).  The call allocates and
 * frees nothing.  Limit: caat_norm_bwd_workspace_bytes(T, tokens, h) <= 16 MiB, i.e. every shape with h <= 4096 and,
 * for 4096 < h <= 8192, at most 16 MiB / (8 h) partial rows of 8 token rows each (T*tokens <= 2048 at h = 8192);
 * beyond that the call returns CAAT_ESCRATCH before anything is launched and leaves every output untouched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams, or
 * different host threads) race on it -- serialise them, or use caat_norm_bwd with separate workspaces.  The array
 * keeps the last call's contents; nothing in it needs clearing between calls (the kernels write every partial row
 * that the final sum reads).
 */
int caat_norm_bwd_static(const void* dy, const void* dres, const void* x, const void* gamma, const float* mean,
                         const float* rstd, void* g_out, void* g_scaled, float* dgamma, float* dbeta, int norm, int T,
                         long long tokens, int h, int hs, float private_scale, void* hip_stream);

/*
 * Grouped bf16 shard GEMM with fp32 accumulation, the building block of Eq. A3's two contractions and of
 * their gradients: for g in [0,G): c_g[M,N] = op(a_g) op(b_g), layouts per caat_gemm_layout.
 * lda/ldb/ldc are row strides in elements, stride_* the distance between groups in elements.
 * M,N,K >= 1 arbitrary except: the contiguous dimension of every operand and N must be multiples of 8.
 */
int caat_gemm_bf16(const void* a, const void* b, void* c, int layout, int G, long long M, long long N, long long K,
                   long long lda, long long ldb, long long ldc, long long stride_a, long long stride_b,
                   long long stride_c, void* hip_stream);

/*
 * Forward of one sub-block (Eq. A3 / A5 + Sec. 4):  Zt_m = SubLayer_m(x_m);  r_out_m = r_m + PCR(Zt)_m;
 * x_out_m = Norm(r_out_m).
 *   weights (host array of device pointers), by kind:
 *     CAAT_MLP_GELU   : {A [T][ffn/T][h], B [T][h][ffn/T], gamma [h], beta [h] or NULL}
 *     CAAT_MLP_SWIGLU : {Wgu [T][2*ffn/T][h] (gate rows then up rows), B [T][h][ffn/T], gamma, beta or NULL}
 *     CAAT_ATTN       : {Wqkv [T][hd_r + 2*kvd_r][h] (q rows, k rows, v rows; heads contiguous), Wo [T][h][hd_r],
 *                        gamma, beta or NULL},  hd_r = (n_heads/T)*head_dim, kvd_r = (n_kv_heads/T)*head_dim
 *     CAAT_ATTN_DECODE, CAAT_LAYER_PREFILL: {gamma_attn [h], Wqkv, Wo, gamma_mlp [h], Wgu, B}; RMSNorm only
 *   x, r       : [T,tokens,h] inputs (x already normalised; the layer kinds ignore x and normalise r themselves)
 *   r_out      : [T,tokens,h] new residual stream R'
 *   x_out      : [T,tokens,h] Norm(R'); layer kinds: may be NULL (not produced)
 *   kv_k, kv_v : layer kinds only, [T][batch][n_kv_heads/T][kv_cap][head_dim]; decode writes row kv_len, prefill
 *                rows 0 .. seq-1 (rotated keys, values)
 *   workspace  : caat_workspace_bytes(d) bytes; keeps what caat_block_bwd needs
 */
int caat_block_fwd(const caat_desc* d, const void* const* weights, const void* x, const void* r, void* r_out,
                   void* x_out, void* kv_k, void* kv_v, void* workspace, size_t ws_bytes, void* hip_stream);

/*
 * Backward of caat_block_fwd for the MLP kinds and CAAT_ATTN (Fig. 2b): norm backward per rank, residual
 * gradient dr_m = g_m un-reduced, the SAME partial channel-reduce on g (fp32 accumulation), then the chain
 * rule of Eq. A3 / A5 per rank (for CAAT_ATTN: o_proj, the causal attention core rebuilt from the saved
 * softmax statistics, the inverse RoPE rotation, the q/k/v projections); dx_m is NOT reduced over ranks.
 * The layer kinds have no backward (CAAT_EUNSUPPORTED).
 *   x, r_out           : the forward's input x and output r_out
 *   workspace          : the forward's workspace (also used as scratch here)
 *   dx_out, dr_out     : [T,tokens,h] gradients w.r.t. x_out and r_out
 *   dx, dr             : [T,tokens,h] outputs
 *   dweights           : host array of device pointers, bf16, same shapes/order as the weight matrices
 *                        ({dA, dB}, {dWgu, dB} or {dWqkv, dWo})
 *   dgamma, dbeta      : [h] fp32, summed over ranks; dbeta NULL for RMSNorm
 */
int caat_block_bwd(const caat_desc* d, const void* const* weights, const void* x, const void* r_out,
                   void* workspace, size_t ws_bytes, const void* dx_out, const void* dr_out, void* dx, void* dr,
                   void* const* dweights, float* dgamma, float* dbeta, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CAAT_H */
