// C ABI of libcaat: host-side argument validation and the launch sequences of the block forward / backward.
// No device memory is allocated here; everything is enqueued on the caller's stream.
#include "../../include/caat.h"
#include "caat_tools.h"
#include "caat_internal.h"

#include <cmath>
#include <cstring>
#include <vector>

using namespace caat;

static __device__ __align__(256) unsigned char caat_static_scratch[(size_t)16 << 20];

namespace {

// ---- the one entry point that allocates nothing (caat_norm_bwd_static) keeps its partial sums here instead of in a
// caller-supplied workspace.  Every GPU the library runs on holds its own copy of the array until the process ends.
// In host code the array's name is only a stand-in for the symbol: the device address comes from
// hipGetSymbolAddress, once per device with that device current, and only that pointer is ever passed to a kernel.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
void* g_static_scratch[STATIC_SCRATCH_MAX_DEVICES] = {};   // device address of caat_static_scratch, per device id

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int hip_status(hipError_t e) { return e == hipSuccess ? CAAT_OK : CAAT_EHIP; }

// ---- optional per-launch timing (host-side tool): hipEvent pairs around every kernel of the block calls
struct ProfRec {
  const char* name;
  hipEvent_t e0, e1;
};
bool g_prof_on = false;
std::vector<ProfRec> g_prof;   // event pool, reused after caat_profile_reset
size_t g_prof_used = 0;

struct ProfScope {
  hipStream_t s;
  ProfRec* rec;
  ProfScope(hipStream_t stream, const char* name) : s(stream), rec(nullptr) {
    if (!g_prof_on) return;
    if (g_prof_used == g_prof.size()) {
      ProfRec r;
      r.name = name;
      if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
      g_prof.push_back(r);
    }
    rec = &g_prof[g_prof_used++];
    rec->name = name;
    (void)hipEventRecord(rec->e0, s);
  }
  ~ProfScope() {
    if (rec) (void)hipEventRecord(rec->e1, s);
  }
};

bool is_mlp(int kind) { return kind == CAAT_MLP_GELU || kind == CAAT_MLP_SWIGLU; }
bool is_layer(int kind) { return kind == CAAT_ATTN_DECODE || kind == CAAT_LAYER_PREFILL; }
// key / value heads over all ranks (n_kv_heads = 0 means one per query head) and the width of a rank's fused
// q | k | v projection
// the residual stream stores its shared channels once (only together with the reduce inside the GEMM)
bool dedup_on(const caat_desc* d) { return d->dedup_shared != 0; }
int dedup_hs(const caat_desc* d) { return dedup_on(d) ? d->hs : 0; }
int kv_heads_of(const caat_desc* d) { return d->n_kv_heads > 0 ? d->n_kv_heads : d->n_heads; }
long long qkv_width(const caat_desc* d) {
  return (long long)(d->n_heads / d->T + 2 * (kv_heads_of(d) / d->T)) * d->head_dim;
}

int validate_desc(const caat_desc* d) {
  if (!d) return CAAT_EINVAL;
  if (d->kind < CAAT_MLP_GELU || d->kind > CAAT_LAYER_PREFILL) return CAAT_EINVAL;
  if (d->norm != CAAT_LAYERNORM && d->norm != CAAT_RMSNORM) return CAAT_EINVAL;
  if (d->T < 1 || d->h < 1 || d->tokens < 0) return CAAT_EINVAL;
  if (!(d->eps >= 0.0f) || std::isnan(d->private_scale)) return CAAT_EINVAL;
  if (d->reduce_in_gemm != 0 && d->reduce_in_gemm != 1) return CAAT_EINVAL;
  if (d->dedup_shared != 0 && d->dedup_shared != 1) return CAAT_EINVAL;
  if (d->separate_reduce != 0 && d->separate_reduce != 1) return CAAT_EINVAL;
  // the de-duplicated layout exists only where the shared channels are produced once: reduce inside the GEMM, whole
  // 16-byte groups of shared channels, more than 64 tokens, and not for the decode step
  if (d->dedup_shared && (!d->reduce_in_gemm || d->hs % 8 != 0 || d->tokens <= 64 || d->kind == CAAT_ATTN_DECODE))
    return CAAT_EUNSUPPORTED;
  if (d->hs < 0 || d->hs > d->h) return CAAT_ESHAPE;
  if (d->h % 8 != 0 || d->h > 8192) return CAAT_ESHAPE;
  if (d->tokens > 0x7FFFFFFFLL) return CAAT_ESHAPE;
  if (is_mlp(d->kind) || is_layer(d->kind)) {
    if (d->ffn < 1 || d->ffn % d->T != 0 || (d->ffn / d->T) % 8 != 0) return CAAT_ESHAPE;
  }
  if (d->kind == CAAT_ATTN || is_layer(d->kind)) {
    if (d->n_heads < 1 || d->head_dim < 1 || d->n_heads % d->T != 0) return CAAT_ESHAPE;
    if (d->n_kv_heads < 0 || d->n_heads % kv_heads_of(d) != 0 || kv_heads_of(d) % d->T != 0) return CAAT_ESHAPE;
    if (d->batch < 1 || d->seq < 1 || (long long)d->batch * d->seq != d->tokens) return CAAT_ESHAPE;
    if (((d->n_heads / d->T) * d->head_dim) % 8 != 0) return CAAT_ESHAPE;
  }
  return CAAT_OK;
}

int layout_of(const caat_desc* d, caat_ws_layout* L) {
  std::memset(L, 0, sizeof(*L));
  int st = validate_desc(d);
  if (st != CAAT_OK) return st;
  const size_t T = d->T, n = (size_t)d->tokens, h = d->h;
  size_t off = 0;
  auto take = [&](size_t bytes, size_t* o, size_t* b) {
    *o = off;
    *b = bytes;
    off += align256(bytes);
  };
  if (is_mlp(d->kind)) {
    const size_t fr = d->ffn / d->T;
    const size_t pw = d->kind == CAAT_MLP_SWIGLU ? 2 * fr : fr;
    take(T * n * pw * 2, &L->off_P, &L->bytes_P);
    take(T * n * fr * 2, &L->off_Y, &L->bytes_Y);
    if (d->norm == CAAT_LAYERNORM) take(T * n * 4, &L->off_mean, &L->bytes_mean);
    take(T * n * 4, &L->off_rstd, &L->bytes_rstd);
    take(T * n * h * 2, &L->off_dZt, &L->bytes_dZt);
    take(T * n * pw * 2, &L->off_dP, &L->bytes_dP);
    take(norm_bwd_workspace_bytes(d->T, d->tokens, d->h), &L->off_scratch, &L->bytes_scratch);
  } else if (d->kind == CAAT_ATTN) {
    const size_t hd = (size_t)(d->n_heads / d->T) * d->head_dim, qw = (size_t)qkv_width(d);
    take(T * n * qw * 2, &L->off_Q, &L->bytes_Q);
    take(T * n * hd * 2, &L->off_Y, &L->bytes_Y);
    if (d->norm == CAAT_LAYERNORM) take(T * n * 4, &L->off_mean, &L->bytes_mean);
    take(T * n * 4, &L->off_rstd, &L->bytes_rstd);
    take(attn_stats_bytes((long long)T * d->batch, d->n_heads / d->T, d->seq), &L->off_stats, &L->bytes_stats);
    take(T * n * h * 2, &L->off_dZt, &L->bytes_dZt);
    take(T * n * hd * 2, &L->off_dH, &L->bytes_dH);
    take(T * n * qw * 2, &L->off_dP, &L->bytes_dP);
    take(norm_bwd_workspace_bytes(d->T, d->tokens, d->h), &L->off_scratch, &L->bytes_scratch);
  } else if (is_layer(d->kind)) {
    const size_t hd = (size_t)(d->n_heads / d->T) * d->head_dim, fr = d->ffn / d->T;
    take(T * n * h * 2, &L->off_X1, &L->bytes_X1);
    take(T * n * (size_t)qkv_width(d) * 2, &L->off_Q, &L->bytes_Q);
    take(T * n * hd * 2, &L->off_H, &L->bytes_H);
    take(T * n * h * 2, &L->off_R1, &L->bytes_R1);
    take(T * n * h * 2, &L->off_X2, &L->bytes_X2);
    take(T * n * 2 * fr * 2, &L->off_P, &L->bytes_P);
    take(T * n * fr * 2, &L->off_Y, &L->bytes_Y);
    take(T * n * 4, &L->off_rstd, &L->bytes_rstd);
  } else {
    return CAAT_EUNSUPPORTED;
  }
  L->total_bytes = off;
  return CAAT_OK;
}

// The reduce over ranks, the residual add and the norm run as one kernel where its shape is taken and the caller has
// not asked for the reduce as a kernel of its own; the folded-into-the-GEMM serving modes have no reduce pass at all.
bool fuse_reduce_norm(const caat_desc* d) {
  return !d->separate_reduce && !d->reduce_in_gemm && !d->dedup_shared && sync_norm_takes(d->T, d->tokens, d->h, d->hs);
}

// the same for the backward pass: norm backward + the reduce on its result
bool fuse_norm_bwd_reduce(const caat_desc* d) {
  return !d->separate_reduce && norm_bwd_sync_takes(d->T, d->tokens, d->h, d->hs);
}

// Row-parallel projection closed by the partial channel-reduce and the residual add (Eq. A3 / A5, second line + Sec. 4):
//   out_m = PCR_p(a_m W_m^T)_m + resid_m,   a [T,n,kdim], W [T][h][kdim], resid / out [T,n,h].
// Default: one grouped GEMM whose epilogue finishes the private channels and leaves each rank's partial sum on the
// shared ones, then the reduce kernel over the T partials (the stand-in for the tensor-parallel collective).
// reduce_in_gemm (single-device serving with logical ranks, Sec. 3.2: the reduce becomes a local summation): the
// private channels come from a grouped GEMM over columns hs..h-1, the shared channels from ONE GEMM whose contraction
// index runs over all T ranks' inputs and weight rows, so the sum over ranks is taken in the accumulator and no partial
// sum ever reaches memory.
int rowpar_pcr(const caat_desc* d, const bf16_t* a, long long kdim, const bf16_t* w, const bf16_t* resid, bf16_t* out,
               hipStream_t s, bool leave_reduce_to_caller = false) {
  const long long T = d->T, n = d->tokens, h = d->h;
  const int hs = d->hs;
  hipError_t e = hipSuccess;
  GemmParams q;
  // (Not for skinny problems: with at most 64 token rows per rank the GEMM is a weight stream whose only parallelism
  // is the number of tiles, and folding the ranks into the contraction would leave hs/64 workgroups for 256 CUs.)
  if (d->reduce_in_gemm && hs % 8 == 0 && n > 64) {
    // residual stream layouts: [T,n,h] (shared columns in every rank's rows), or de-duplicated: [n,hs] once, then the
    // private columns [T,n,h-hs]
    const bool dd = dedup_on(d);
    const long long ldp = dd ? h - hs : h, ldsh = dd ? hs : h;
    const bf16_t* resid_p = dd ? resid + n * hs : resid + hs;
    bf16_t* out_p = dd ? out + n * hs : out + hs;
    if (hs < h) {
      std::memset(&q, 0, sizeof(q));
      q.a = a; q.lda = kdim; q.stride_a = n * kdim;
      q.b = w + (long long)hs * kdim; q.ldb = kdim; q.stride_b = h * kdim;
      q.c = out_p; q.ldc = ldp; q.stride_c = n * ldp;
      q.aux = resid_p; q.ldaux = ldp; q.stride_aux = n * ldp;
      q.G = (int)T; q.M = (int)n; q.N = (int)(h - hs); q.K = (int)kdim;
      q.hs = 0; q.scale = d->private_scale;
      {
        ProfScope ps(s, "gemm_nt_rowpar_private");
        e = launch_gemm(q, 0, EPI_ROWPAR, s);
      }
      if (e != hipSuccess) return CAAT_EHIP;
    }
    if (hs > 0) {
      std::memset(&q, 0, sizeof(q));
      q.a = a; q.lda = kdim; q.kstride_a = n * kdim;
      q.b = w; q.ldb = kdim; q.kstride_b = h * kdim;
      q.c = out; q.ldc = ldsh; q.stride_c = n * h;
      q.aux = resid; q.ldaux = ldsh; q.stride_aux = n * h;
      q.G = 1; q.M = (int)n; q.N = hs; q.K = (int)kdim; q.kcat = (int)T; q.bcast = dd ? 1 : (int)T;
      {
        ProfScope ps(s, "gemm_nt_shared_kcat");
        e = launch_gemm(q, 0, EPI_SHARED_BCAST, s);
      }
      if (e != hipSuccess) return CAAT_EHIP;
    }
    return CAAT_OK;
  }
  std::memset(&q, 0, sizeof(q));
  q.a = a; q.lda = kdim; q.stride_a = n * kdim;
  q.b = w; q.ldb = kdim; q.stride_b = h * kdim;
  q.c = out; q.ldc = h; q.stride_c = n * h;
  q.aux = resid; q.ldaux = h; q.stride_aux = n * h;
  q.G = (int)T; q.M = (int)n; q.N = (int)h; q.K = (int)kdim;
  q.hs = hs; q.scale = d->private_scale;
  {
    ProfScope ps(s, "gemm_nt_rowpar");
    e = launch_gemm(q, 0, EPI_ROWPAR, s);
  }
  if (e != hipSuccess) return CAAT_EHIP;
  if (hs > 0 && !leave_reduce_to_caller) {
    ProfScope ps(s, "partial_sync_fwd");
    e = launch_partial_sync_shared(out, resid, (int)T, n, (int)h, hs, s);
    if (e != hipSuccess) return CAAT_EHIP;
  }
  return CAAT_OK;
}

// Attention sub-block forward (Eq. A5 + Sec. 4): per rank q,k,v = X_m Wqkv_m^T; RoPE(q,k); causal attention per head;
// Zt_m = H_m Wo_m^T with the private half of the partial channel-reduce in the epilogue; shared half; norm.
int attn_block_fwd(const caat_desc* d, const caat_ws_layout& L, const void* const* weights, const void* x, const void* r,
                   void* r_out, void* x_out, void* workspace, size_t ws_bytes, void* hip_stream) {
  const void* wqkv = weights[0]; const void* wo = weights[1]; const void* gamma = weights[2]; const void* beta = weights[3];
  if (!wqkv || !wo || !gamma || (d->norm == CAAT_LAYERNORM && !beta)) return CAAT_EINVAL;
  if (d->head_dim != 128) return CAAT_EUNSUPPORTED;
  if (misaligned(wqkv) || misaligned(wo) || misaligned(gamma) || (beta && misaligned(beta)) || misaligned(x) ||
      misaligned(r) || misaligned(r_out) || misaligned(x_out) || misaligned(workspace))
    return CAAT_EALIGN;
  if (ws_bytes < L.total_bytes) return CAAT_EWORKSPACE;
  if (d->tokens == 0) return CAAT_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const long long T = d->T, n = d->tokens, h = d->h, hd = (long long)(d->n_heads / d->T) * d->head_dim, qw = qkv_width(d);
  const int hpr = d->n_heads / d->T, kvpr = kv_heads_of(d) / d->T;
  bf16_t* QKV = (bf16_t*)(ws + L.off_Q);
  bf16_t* H = (bf16_t*)(ws + L.off_Y);
  float* mean = d->norm == CAAT_LAYERNORM ? (float*)(ws + L.off_mean) : nullptr;
  float* rstd = (float*)(ws + L.off_rstd);
  float* stats = (float*)(ws + L.off_stats);
  hipError_t e;
  GemmParams g1;
  std::memset(&g1, 0, sizeof(g1));
  g1.a = (const bf16_t*)x; g1.lda = h; g1.stride_a = n * h;
  g1.b = (const bf16_t*)wqkv; g1.ldb = h; g1.stride_b = qw * h;
  g1.c = QKV; g1.ldc = qw; g1.stride_c = n * qw;
  g1.G = (int)T; g1.M = (int)n; g1.N = (int)qw; g1.K = (int)h;
  {
    ProfScope ps(s, "gemm_nt_qkv");
    e = launch_gemm(g1, 0, EPI_PLAIN, s);
  }
  if (e != hipSuccess) return CAAT_EHIP;
  {
    ProfScope ps(s, "rope");
    e = launch_rope(QKV, T * n, d->seq, (int)qw, hpr + kvpr, d->head_dim, d->rope_base, 0, false, s);
  }
  if (e != hipSuccess) return CAAT_EHIP;
  {
    ProfScope ps(s, "flash_attn_fwd");
    e = launch_flash_fwd(QKV, H, stats, T * d->batch, d->seq, hpr, kvpr, d->head_dim, s);
  }
  if (e != hipSuccess) return CAAT_EHIP;
  const bool fuse = fuse_reduce_norm(d);
  {
    const int st = rowpar_pcr(d, H, hd, (const bf16_t*)wo, (const bf16_t*)r, (bf16_t*)r_out, s, fuse);
    if (st != CAAT_OK) return st;
  }
  if (fuse) {
    ProfScope ps(s, "partial_sync_norm_fwd");
    e = launch_sync_norm((bf16_t*)r_out, (const bf16_t*)r, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x_out, mean, rstd,
                         d->norm, (int)T, n, (int)h, d->hs, d->eps, s);
  } else {
    ProfScope ps(s, "norm_fwd");
    e = launch_norm_fwd((const bf16_t*)r_out, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x_out, mean, rstd, d->norm,
                        (int)T, n, (int)h, d->eps, s, dedup_hs(d));
  }
  return hip_status(e);
}

// Attention sub-block backward (Fig. 2b applied to Eq. A5): norm backward per rank first, dr_m = g_m un-reduced, the
// partial channel-reduce on g, then per rank dH = dZt Wo, dWo = dZt^T H, the attention-core gradient w.r.t. the rotated
// q, k and v, the inverse rotation of dq and dk, dX = dqkv Wqkv (never reduced over ranks) and dWqkv = dqkv^T X.
int attn_block_bwd(const caat_desc* d, const caat_ws_layout& L, const void* const* weights, const void* x, const void* r_out,
                   void* workspace, size_t ws_bytes, const void* dx_out, const void* dr_out, void* dx, void* dr,
                   void* const* dweights, float* dgamma, float* dbeta, void* hip_stream) {
  const void* wqkv = weights[0]; const void* wo = weights[1]; const void* gamma = weights[2];
  void* dwqkv = dweights[0]; void* dwo = dweights[1];
  if (!wqkv || !wo || !gamma || !dwqkv || !dwo || (d->norm == CAAT_LAYERNORM && !dbeta)) return CAAT_EINVAL;
  if (d->head_dim != 128) return CAAT_EUNSUPPORTED;
  if (misaligned(wqkv) || misaligned(wo) || misaligned(gamma) || misaligned(dwqkv) || misaligned(dwo) || misaligned(x) ||
      misaligned(r_out) || misaligned(workspace) || misaligned(dx_out) || misaligned(dr_out) || misaligned(dx) ||
      misaligned(dr))
    return CAAT_EALIGN;
  if (ws_bytes < L.total_bytes) return CAAT_EWORKSPACE;
  if (d->tokens == 0) return CAAT_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const long long T = d->T, n = d->tokens, h = d->h, hd = (long long)(d->n_heads / d->T) * d->head_dim, qw = qkv_width(d);
  const int hpr = d->n_heads / d->T, kvpr = kv_heads_of(d) / d->T;
  const bf16_t* QKV = (const bf16_t*)(ws + L.off_Q);
  const bf16_t* H = (const bf16_t*)(ws + L.off_Y);
  const float* mean = d->norm == CAAT_LAYERNORM ? (const float*)(ws + L.off_mean) : nullptr;
  const float* rstd = (const float*)(ws + L.off_rstd);
  float* stats = (float*)(ws + L.off_stats);
  bf16_t* dZt = (bf16_t*)(ws + L.off_dZt);
  bf16_t* dH = (bf16_t*)(ws + L.off_dH);
  bf16_t* dQKV = (bf16_t*)(ws + L.off_dP);
  hipError_t e;
  GemmParams q;
#define CAAT_STEP(name, call) { ProfScope ps(s, name); e = (call); } if (e != hipSuccess) return CAAT_EHIP;
  if (fuse_norm_bwd_reduce(d)) {
    // norm backward and the reduce on its result in one launch (the shared channels are not read back from memory)
    CAAT_STEP("norm_bwd_sync", launch_norm_bwd_sync((const bf16_t*)dx_out, (const bf16_t*)dr_out, (const bf16_t*)r_out,
                                                    (const bf16_t*)gamma, mean, rstd, (bf16_t*)dr, dZt, dgamma, dbeta, d->norm,
                                                    (int)T, n, (int)h, d->hs, d->private_scale, ws + L.off_scratch, s))
  } else {
    CAAT_STEP("norm_bwd", launch_norm_bwd((const bf16_t*)dx_out, (const bf16_t*)dr_out, (const bf16_t*)r_out, (const bf16_t*)gamma,
                                          mean, rstd, (bf16_t*)dr, dZt, dgamma, dbeta, d->norm, (int)T, n, (int)h, d->hs,
                                          d->private_scale, ws + L.off_scratch, s, true))
    // when no 8-channel vector straddles hs, the norm backward leaves the shared channels of dZt to the reduce, which
    // reads them from dr (the same values) instead of reading them back from dZt: one write of T*n*hs values less
    CAAT_STEP("partial_sync_bwd", d->hs % 8 == 0
                                      ? launch_partial_sync_shared_from((const bf16_t*)dr, dZt, (int)T, n, (int)h, d->hs, s)
                                      : launch_partial_sync(dZt, nullptr, dZt, (int)T, n, (int)h, d->hs, 1.0f, s))
  }
  // dH_m = dZt_m Wo_m (NN): [n,h] x [h,hd]
  std::memset(&q, 0, sizeof(q));
  q.a = dZt; q.lda = h; q.stride_a = n * h;
  q.b = (const bf16_t*)wo; q.ldb = hd; q.stride_b = h * hd;
  q.c = dH; q.ldc = hd; q.stride_c = n * hd;
  q.G = (int)T; q.M = (int)n; q.N = (int)hd; q.K = (int)h;
  CAAT_STEP("gemm_nn_dgrad", launch_gemm(q, 1, EPI_PLAIN, s))
  // dWo_m [h,hd] = dZt_m^T H_m (TN, reduction over tokens)
  std::memset(&q, 0, sizeof(q));
  q.a = dZt; q.lda = h; q.stride_a = n * h;
  q.b = H; q.ldb = hd; q.stride_b = n * hd;
  q.c = (bf16_t*)dwo; q.ldc = hd; q.stride_c = h * hd; q.late_c = 1;   // gradients leave the block: not read again here
  q.G = (int)T; q.M = (int)h; q.N = (int)hd; q.K = (int)n;
  CAAT_STEP("gemm_tn_wgrad", launch_gemm(q, 2, EPI_PLAIN, s))
  CAAT_STEP("flash_attn_bwd", launch_flash_bwd(QKV, H, dH, stats, dQKV, T * d->batch, d->seq, hpr, kvpr, d->head_dim, s))
  CAAT_STEP("rope_bwd", launch_rope(dQKV, T * n, d->seq, (int)qw, hpr + kvpr, d->head_dim, d->rope_base, 0, true, s))
  // dX_m = dqkv_m Wqkv_m (NN): [n,qw] x [qw,h]; not reduced over ranks
  std::memset(&q, 0, sizeof(q));
  q.a = dQKV; q.lda = qw; q.stride_a = n * qw;
  q.b = (const bf16_t*)wqkv; q.ldb = h; q.stride_b = qw * h;
  q.c = (bf16_t*)dx; q.ldc = h; q.stride_c = n * h; q.late_c = 1;
  q.G = (int)T; q.M = (int)n; q.N = (int)h; q.K = (int)qw;
  CAAT_STEP("gemm_nn_dgrad", launch_gemm(q, 1, EPI_PLAIN, s))
  // dWqkv_m [qw,h] = dqkv_m^T X_m (TN)
  std::memset(&q, 0, sizeof(q));
  q.a = dQKV; q.lda = qw; q.stride_a = n * qw;
  q.b = (const bf16_t*)x; q.ldb = h; q.stride_b = n * h;
  q.c = (bf16_t*)dwqkv; q.ldc = h; q.stride_c = qw * h; q.late_c = 1;
  q.G = (int)T; q.M = (int)qw; q.N = (int)h; q.K = (int)n;
  CAAT_STEP("gemm_tn_wgrad", launch_gemm(q, 2, EPI_PLAIN, s))
#undef CAAT_STEP
  return CAAT_OK;
}

// One Llama-style decoder layer at inference (which uses the partial channel-reduce too, Sec. 3.2), either for one
// new token per sequence over a KV cache (decode) or for a whole prompt that fills the cache (prefill, the
// time-to-first-token workload of Sec. 5.2): RMSNorm -> q,k,v -> RoPE -> store k,v in the cache -> attention
// (streaming over kv_len+1 keys / causal flash attention over the prompt) -> o_proj -> PCR + residual -> RMSNorm ->
// SwiGLU MLP -> PCR + residual.
int layer_fwd(const caat_desc* d, const caat_ws_layout& L, const void* const* weights, const void* r, void* r_out,
              void* kv_k, void* kv_v, void* workspace, size_t ws_bytes, void* hip_stream) {
  const bool prefill = d->kind == CAAT_LAYER_PREFILL;
  if (!weights || !r || !r_out || !kv_k || !kv_v || !workspace) return CAAT_EINVAL;
  const void* g_attn = weights[0]; const void* wqkv = weights[1]; const void* wo = weights[2];
  const void* g_mlp = weights[3]; const void* wgu = weights[4]; const void* wb = weights[5];
  if (!g_attn || !wqkv || !wo || !g_mlp || !wgu || !wb) return CAAT_EINVAL;
  if (d->norm != CAAT_RMSNORM || d->head_dim != 128) return CAAT_EUNSUPPORTED;
  if (prefill) {
    if (d->kv_len != 0 || d->kv_cap < d->seq) return CAAT_ESHAPE;     // the prompt starts an empty cache
  } else {
    if (d->seq != 1 || d->kv_len < 0 || d->kv_cap <= d->kv_len) return CAAT_ESHAPE;
  }
  if (d->kv_cap * 256 >= 0x7FFFFFFFLL) return CAAT_ESHAPE;
  if (misaligned(g_attn) || misaligned(wqkv) || misaligned(wo) || misaligned(g_mlp) || misaligned(wgu) || misaligned(wb) ||
      misaligned(r) || misaligned(r_out) || misaligned(kv_k) || misaligned(kv_v) || misaligned(workspace))
    return CAAT_EALIGN;
  if (ws_bytes < L.total_bytes) return CAAT_EWORKSPACE;
  if (d->tokens == 0) return CAAT_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const long long T = d->T, n = d->tokens, h = d->h, hpr = d->n_heads / d->T, hd = hpr * d->head_dim, fr = d->ffn / d->T;
  const long long kvpr = kv_heads_of(d) / d->T, qw = qkv_width(d);
  bf16_t* X1 = (bf16_t*)(ws + L.off_X1);
  bf16_t* QKV = (bf16_t*)(ws + L.off_Q);
  bf16_t* H = (bf16_t*)(ws + L.off_H);
  bf16_t* R1 = (bf16_t*)(ws + L.off_R1);
  bf16_t* X2 = (bf16_t*)(ws + L.off_X2);
  bf16_t* P = (bf16_t*)(ws + L.off_P);
  bf16_t* Y = (bf16_t*)(ws + L.off_Y);
  float* rstd = (float*)(ws + L.off_rstd);
  hipError_t e;
  GemmParams q;
#define CAAT_STEP(name, call) { ProfScope ps(s, name); e = (call); } if (e != hipSuccess) return CAAT_EHIP;
  CAAT_STEP("norm_fwd", launch_norm_fwd((const bf16_t*)r, (const bf16_t*)g_attn, nullptr, X1, nullptr, rstd, CAAT_RMSNORM, (int)T,
                                        n, (int)h, d->eps, s, dedup_hs(d)))
  std::memset(&q, 0, sizeof(q));
  q.a = X1; q.lda = h; q.stride_a = n * h;
  q.b = (const bf16_t*)wqkv; q.ldb = h; q.stride_b = qw * h;
  q.c = QKV; q.ldc = qw; q.stride_c = n * qw;
  q.G = (int)T; q.M = (int)n; q.N = (int)qw; q.K = (int)h;
  CAAT_STEP("gemm_nt_qkv", launch_gemm(q, 0, EPI_PLAIN, s))
  if (prefill) {
    CAAT_STEP("rope_kv_append", launch_rope_append(QKV, (bf16_t*)kv_k, (bf16_t*)kv_v, T * d->batch, d->seq, (int)hpr, (int)kvpr,
                                                   d->head_dim, d->rope_base, d->kv_cap, d->kv_len, s))
    CAAT_STEP("flash_attn_fwd", launch_flash_fwd(QKV, H, nullptr, T * d->batch, d->seq, (int)hpr, (int)kvpr, d->head_dim, s))
  } else {
    // decode: the attention kernel rotates q and the new k itself, appends k, v to the caches and attends to
    // kv_len cached keys plus the new one
    CAAT_STEP("decode_attn", launch_decode_attn(QKV, (bf16_t*)kv_k, (bf16_t*)kv_v, H, T * n, (int)hpr, (int)kvpr,
                                                d->head_dim, d->kv_cap, d->kv_len + 1, d->rope_base, s))
  }
  // the reduce after o_proj and the RMSNorm in front of the MLP run as one launch where the fused kernel takes the
  // shape: for decode-sized batches both are start-up latency, for prompts the fused kernel does not read the
  // reduced shared channels back from memory (measured 1.28 ms instead of 0.61 + 0.78 ms on 16 prompts of 2048)
  const bool fuse_mid = fuse_reduce_norm(d);
  {
    const int st = rowpar_pcr(d, H, hd, (const bf16_t*)wo, (const bf16_t*)r, R1, s, fuse_mid);
    if (st != CAAT_OK) return st;
  }
  if (fuse_mid) {
    CAAT_STEP("partial_sync_norm_fwd", launch_sync_norm(R1, (const bf16_t*)r, (const bf16_t*)g_mlp, nullptr, X2, nullptr, rstd,
                                                        CAAT_RMSNORM, (int)T, n, (int)h, d->hs, d->eps, s))
  } else {
    CAAT_STEP("norm_fwd", launch_norm_fwd(R1, (const bf16_t*)g_mlp, nullptr, X2, nullptr, rstd, CAAT_RMSNORM, (int)T, n, (int)h,
                                          d->eps, s, dedup_hs(d)))
  }
  std::memset(&q, 0, sizeof(q));
  q.a = X2; q.lda = h; q.stride_a = n * h;
  q.b = (const bf16_t*)wgu; q.ldb = h; q.stride_b = 2 * fr * h;
  q.c = P; q.ldc = 2 * fr; q.stride_c = n * 2 * fr;
  q.c2 = Y; q.ldc2 = fr; q.stride_c2 = n * fr;
  q.G = (int)T; q.M = (int)n; q.N = (int)fr; q.K = (int)h; q.half = (int)fr;
  CAAT_STEP("gemm_nt_swiglu_fwd", launch_gemm(q, 0, EPI_SWIGLU_FWD, s))
  {
    const int st = rowpar_pcr(d, Y, fr, (const bf16_t*)wb, R1, (bf16_t*)r_out, s);
    if (st != CAAT_OK) return st;
  }
#undef CAAT_STEP
  return CAAT_OK;
}

}  // namespace

extern "C" {

int caat_shared_channels(int h, double p) {
  if (h < 0 || !(p >= 0.0 && p <= 1.0)) return -1;
  double v = std::floor((double)h * p);
  if (v < 0) v = 0;
  if (v > h) v = h;
  return (int)v;
}

const char* caat_status_string(int status) {
  switch (status) {
    case CAAT_OK: return "ok";
    case CAAT_EINVAL: return "invalid argument (null pointer, bad T / p / enum)";
    case CAAT_ESHAPE: return "unsupported shape (divisibility by T or 8, hs > h, h > 8192)";
    case CAAT_EALIGN: return "device pointer not 16-byte aligned";
    case CAAT_EWORKSPACE: return "workspace too small";
    case CAAT_EHIP: return "HIP runtime error at kernel launch";
    case CAAT_EUNSUPPORTED: return "valid request not implemented in this build";
    case CAAT_ESCRATCH: return "problem needs more scratch than the library's fixed 16 MiB device array (use the entry point that takes a workspace)";
    default: return "unknown status";
  }
}

size_t caat_workspace_bytes(const caat_desc* d) {
  caat_ws_layout L;
  if (layout_of(d, &L) != CAAT_OK) return 0;
  return L.total_bytes;
}

int caat_workspace_layout(const caat_desc* d, caat_ws_layout* out) {
  if (!out) return CAAT_EINVAL;
  return layout_of(d, out);
}

int caat_hbm_probe(const void* src, void* dst, size_t bytes, int mode, void* hip_stream) {
  if (!src || mode < 0 || mode > 4 || (mode >= 3 && !dst)) return CAAT_EINVAL;
  if (bytes % 16 != 0) return CAAT_ESHAPE;
  if (misaligned(src) || (dst && misaligned(dst))) return CAAT_EALIGN;
  return hip_status(launch_hbm_probe(src, dst, bytes, mode, (hipStream_t)hip_stream));
}

int caat_profile_enable(int on) {
  g_prof_on = on != 0;
  return CAAT_OK;
}

int caat_profile_reset(void) {
  g_prof_used = 0;
  return CAAT_OK;
}

int caat_profile_count(void) { return (int)g_prof_used; }

int caat_profile_get(int index, const char** name, float* ms) {
  if (index < 0 || (size_t)index >= g_prof_used || !name || !ms) return CAAT_EINVAL;
  ProfRec& r = g_prof[(size_t)index];
  if (hipEventSynchronize(r.e1) != hipSuccess) return CAAT_EHIP;
  if (hipEventElapsedTime(ms, r.e0, r.e1) != hipSuccess) return CAAT_EHIP;
  *name = r.name;
  return CAAT_OK;
}

int caat_partial_sync(const void* y, const void* resid, void* out, int T, long long tokens, int h, int hs,
                      float private_scale, void* hip_stream) {
  if (!y || !out || T < 1 || tokens < 0 || h < 1 || std::isnan(private_scale)) return CAAT_EINVAL;
  if (hs < 0 || hs > h || h % 8 != 0) return CAAT_ESHAPE;
  if (misaligned(y) || misaligned(out) || (resid && misaligned(resid))) return CAAT_EALIGN;
  return hip_status(launch_partial_sync((const bf16_t*)y, (const bf16_t*)resid, (bf16_t*)out, T, tokens, h, hs,
                                        private_scale, (hipStream_t)hip_stream));
}

int caat_norm_fwd(const void* x, const void* gamma, const void* beta, void* y, float* mean, float* rstd, int norm,
                  int T, long long tokens, int h, float eps, void* hip_stream) {
  if (!x || !gamma || !y || !rstd || T < 1 || tokens < 0 || h < 1) return CAAT_EINVAL;
  if (norm != CAAT_LAYERNORM && norm != CAAT_RMSNORM) return CAAT_EINVAL;
  if (norm == CAAT_LAYERNORM && (!beta || !mean)) return CAAT_EINVAL;
  if (h % 8 != 0 || h > 8192) return CAAT_ESHAPE;
  if (misaligned(x) || misaligned(gamma) || misaligned(y) || (beta && misaligned(beta))) return CAAT_EALIGN;
  return hip_status(launch_norm_fwd((const bf16_t*)x, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, mean, rstd,
                                    norm, T, tokens, h, eps, (hipStream_t)hip_stream));
}

int caat_partial_sync_norm_fwd(void* io, const void* resid, const void* gamma, const void* beta, void* x_out, float* mean,
                               float* rstd, int norm, int T, long long tokens, int h, int hs, float eps, void* hip_stream) {
  if (!io || !resid || !gamma || !x_out || !rstd || T < 1 || tokens < 0 || h < 1 || !(eps >= 0.0f)) return CAAT_EINVAL;
  if (norm != CAAT_LAYERNORM && norm != CAAT_RMSNORM) return CAAT_EINVAL;
  if (norm == CAAT_LAYERNORM && !beta) return CAAT_EINVAL;
  if (h % 8 != 0 || h > 8192 || hs < 0 || hs > h) return CAAT_ESHAPE;
  if (misaligned(io) || misaligned(resid) || misaligned(gamma) || misaligned(x_out) || (beta && misaligned(beta)))
    return CAAT_EALIGN;
  if (tokens == 0) return CAAT_OK;
  if (!sync_norm_takes(T, tokens, h, hs)) return CAAT_EUNSUPPORTED;
  return hip_status(launch_sync_norm((bf16_t*)io, (const bf16_t*)resid, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x_out,
                                     mean, rstd, norm, T, tokens, h, hs, eps, (hipStream_t)hip_stream));
}

size_t caat_norm_bwd_workspace_bytes(int T, long long tokens, int h) {
  if (T < 1 || tokens < 0 || h < 1) return 0;
  return norm_bwd_workspace_bytes(T, tokens, h);
}

int caat_norm_bwd(const void* dy, const void* dres, const void* x, const void* gamma, const float* mean,
                  const float* rstd, void* g_out, void* g_scaled, float* dgamma, float* dbeta, int norm, int T,
                  long long tokens, int h, int hs, float private_scale, void* workspace, size_t ws_bytes,
                  void* hip_stream) {
  if (!dy || !x || !gamma || !rstd || !g_out || !dgamma || !workspace || T < 1 || tokens < 0 || h < 1)
    return CAAT_EINVAL;
  if (norm != CAAT_LAYERNORM && norm != CAAT_RMSNORM) return CAAT_EINVAL;
  if (norm == CAAT_LAYERNORM && (!mean || !dbeta)) return CAAT_EINVAL;
  if (h % 8 != 0 || h > 8192 || hs < 0 || hs > h) return CAAT_ESHAPE;
  if (misaligned(dy) || misaligned(x) || misaligned(gamma) || misaligned(g_out) || (dres && misaligned(dres)) ||
      (g_scaled && misaligned(g_scaled)) || misaligned(workspace))
    return CAAT_EALIGN;
  if (ws_bytes < norm_bwd_workspace_bytes(T, tokens, h)) return CAAT_EWORKSPACE;
  return hip_status(launch_norm_bwd((const bf16_t*)dy, (const bf16_t*)dres, (const bf16_t*)x, (const bf16_t*)gamma, mean,
                                    rstd, (bf16_t*)g_out, (bf16_t*)g_scaled, dgamma, dbeta, norm, T, tokens, h, hs,
                                    private_scale, workspace, (hipStream_t)hip_stream));
}

int caat_norm_bwd_static(const void* dy, const void* dres, const void* x, const void* gamma, const float* mean,
                         const float* rstd, void* g_out, void* g_scaled, float* dgamma, float* dbeta, int norm, int T,
                         long long tokens, int h, int hs, float private_scale, void* hip_stream) {
  if (!dy || !x || !gamma || !rstd || !g_out || !dgamma || T < 1 || tokens < 0 || h < 1) return CAAT_EINVAL;
  if (norm != CAAT_LAYERNORM && norm != CAAT_RMSNORM) return CAAT_EINVAL;
  if (norm == CAAT_LAYERNORM && (!mean || !dbeta)) return CAAT_EINVAL;
  if (h % 8 != 0 || h > 8192 || hs < 0 || hs > h) return CAAT_ESHAPE;
  if (misaligned(dy) || misaligned(x) || misaligned(gamma) || misaligned(g_out) || (dres && misaligned(dres)) ||
      (g_scaled && misaligned(g_scaled)))
    return CAAT_EALIGN;
  if (norm_bwd_workspace_bytes(T, tokens, h) > STATIC_SCRATCH_BYTES) return CAAT_ESCRATCH;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return CAAT_EHIP;
  void* scratch = g_static_scratch[dev];
  if (!scratch) {   // first call on this device (it is the current one): look the array's device address up, once
    if (hipGetSymbolAddress(&scratch, HIP_SYMBOL(caat_static_scratch)) != hipSuccess || !scratch) return CAAT_EHIP;
    g_static_scratch[dev] = scratch;
  }
  // nothing in the array has to start at zero: the backward kernels write every partial row that the final sum reads
  return hip_status(launch_norm_bwd((const bf16_t*)dy, (const bf16_t*)dres, (const bf16_t*)x, (const bf16_t*)gamma, mean,
                                    rstd, (bf16_t*)g_out, (bf16_t*)g_scaled, dgamma, dbeta, norm, T, tokens, h, hs,
                                    private_scale, scratch, (hipStream_t)hip_stream));
}

int caat_gemm_bf16(const void* a, const void* b, void* c, int layout, int G, long long M, long long N, long long K,
                   long long lda, long long ldb, long long ldc, long long stride_a, long long stride_b,
                   long long stride_c, void* hip_stream) {
  if (!a || !b || !c || G < 1 || M < 1 || N < 1 || K < 1) return CAAT_EINVAL;
  if (layout < CAAT_GEMM_NT || layout > CAAT_GEMM_TN) return CAAT_EINVAL;
  if (M > 0x7FFFFFFFLL || N > 0x7FFFFFFFLL || K > 0x7FFFFFFFLL) return CAAT_ESHAPE;
  if (N % 8 != 0 || ldc % 8 != 0 || lda % 8 != 0 || ldb % 8 != 0) return CAAT_ESHAPE;
  if (stride_a % 8 != 0 || stride_b % 8 != 0 || stride_c % 8 != 0) return CAAT_ESHAPE;
  const bool a_kcontig = layout != CAAT_GEMM_TN, b_kcontig = layout == CAAT_GEMM_NT;
  if ((a_kcontig || b_kcontig) && K % 8 != 0) return CAAT_ESHAPE;
  if (!a_kcontig && M % 8 != 0) return CAAT_ESHAPE;
  if (lda < (a_kcontig ? K : M) || ldb < (b_kcontig ? K : N) || ldc < N) return CAAT_ESHAPE;
  if (misaligned(a) || misaligned(b) || misaligned(c)) return CAAT_EALIGN;
  GemmParams p;
  std::memset(&p, 0, sizeof(p));
  p.a = (const bf16_t*)a;
  p.b = (const bf16_t*)b;
  p.c = (bf16_t*)c;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.stride_a = stride_a; p.stride_b = stride_b; p.stride_c = stride_c;
  p.G = G; p.M = (int)M; p.N = (int)N; p.K = (int)K;
  return hip_status(launch_gemm(p, layout, EPI_PLAIN, (hipStream_t)hip_stream));
}

int caat_block_fwd(const caat_desc* d, const void* const* weights, const void* x, const void* r, void* r_out,
                   void* x_out, void* kv_k, void* kv_v, void* workspace, size_t ws_bytes, void* hip_stream) {
  caat_ws_layout L;
  int st = layout_of(d, &L);
  if (st != CAAT_OK) return st;
  if (is_layer(d->kind)) return layer_fwd(d, L, weights, r, r_out, kv_k, kv_v, workspace, ws_bytes, hip_stream);
  if (!weights || !x || !r || !r_out || !x_out || !workspace) return CAAT_EINVAL;
  if (d->kind == CAAT_ATTN) return attn_block_fwd(d, L, weights, x, r, r_out, x_out, workspace, ws_bytes, hip_stream);
  if (!is_mlp(d->kind)) return CAAT_EUNSUPPORTED;
  const void* w0 = weights[0]; const void* w1 = weights[1]; const void* gamma = weights[2]; const void* beta = weights[3];
  if (!w0 || !w1 || !gamma || (d->norm == CAAT_LAYERNORM && !beta)) return CAAT_EINVAL;
  if (misaligned(w0) || misaligned(w1) || misaligned(gamma) || (beta && misaligned(beta)) || misaligned(x) ||
      misaligned(r) || misaligned(r_out) || misaligned(x_out) || misaligned(workspace))
    return CAAT_EALIGN;
  if (ws_bytes < L.total_bytes) return CAAT_EWORKSPACE;
  if (d->tokens == 0) return CAAT_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const long long T = d->T, n = d->tokens, h = d->h, fr = d->ffn / d->T;
  const bool swi = d->kind == CAAT_MLP_SWIGLU;
  const long long pw = swi ? 2 * fr : fr;
  bf16_t* P = (bf16_t*)(ws + L.off_P);
  bf16_t* Y = (bf16_t*)(ws + L.off_Y);
  float* mean = d->norm == CAAT_LAYERNORM ? (float*)(ws + L.off_mean) : nullptr;
  float* rstd = (float*)(ws + L.off_rstd);

  // a1: column-parallel GEMM + activation (Eq. A3, inner sum and sigma): P_m = X_m A_m^T, Y_m = sigma(P_m)
  GemmParams g1;
  std::memset(&g1, 0, sizeof(g1));
  g1.a = (const bf16_t*)x; g1.lda = h; g1.stride_a = n * h;
  g1.b = (const bf16_t*)w0; g1.ldb = h; g1.stride_b = pw * h;
  g1.c = P; g1.ldc = pw; g1.stride_c = n * pw;
  g1.c2 = Y; g1.ldc2 = fr; g1.stride_c2 = n * fr;
  g1.G = (int)T; g1.M = (int)n; g1.N = (int)fr; g1.K = (int)h; g1.half = (int)fr;
  hipError_t e;
  {
    ProfScope ps(s, swi ? "gemm_nt_swiglu_fwd" : "gemm_nt_gelu_fwd");
    e = launch_gemm(g1, 0, swi ? EPI_SWIGLU_FWD : EPI_GELU_FWD, s);
  }
  if (e != hipSuccess) return CAAT_EHIP;

  // a2 + a3/a4: Zt_m = Y_m B_m^T closed by the partial channel-reduce and the residual.  Default: columns >= hs
  // become scale*Zt + R in the GEMM epilogue (final), columns < hs hold the rank's partial sum inside r_out until the
  // reduce kernel sums the T partials on the hs shared channels and adds each rank's residual, in place.
  // a5: per-rank norm on the now rank-divergent residual stream; where the shape allows (and unless the caller wants
  // the reduce as a kernel of its own) the shared half of the reduce, the residual add and the norm are one launch
  const bool fuse = fuse_reduce_norm(d);
  {
    const int st2 = rowpar_pcr(d, Y, fr, (const bf16_t*)w1, (const bf16_t*)r, (bf16_t*)r_out, s, fuse);
    if (st2 != CAAT_OK) return st2;
  }
  if (fuse) {
    ProfScope ps(s, "partial_sync_norm_fwd");
    e = launch_sync_norm((bf16_t*)r_out, (const bf16_t*)r, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x_out, mean, rstd,
                         d->norm, (int)T, n, (int)h, d->hs, d->eps, s);
  } else {
    ProfScope ps(s, "norm_fwd");
    e = launch_norm_fwd((const bf16_t*)r_out, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)x_out, mean, rstd,
                        d->norm, (int)T, n, (int)h, d->eps, s, dedup_hs(d));
  }
  return hip_status(e);
}

int caat_block_bwd(const caat_desc* d, const void* const* weights, const void* x, const void* r_out, void* workspace,
                   size_t ws_bytes, const void* dx_out, const void* dr_out, void* dx, void* dr, void* const* dweights,
                   float* dgamma, float* dbeta, void* hip_stream) {
  caat_ws_layout L;
  int st = layout_of(d, &L);
  if (st != CAAT_OK) return st;
  if (!weights || !dweights || !x || !r_out || !workspace || !dx_out || !dr_out || !dx || !dr || !dgamma)
    return CAAT_EINVAL;
  if (d->dedup_shared) return CAAT_EUNSUPPORTED;   // serving-only layout
  if (d->kind == CAAT_ATTN)
    return attn_block_bwd(d, L, weights, x, r_out, workspace, ws_bytes, dx_out, dr_out, dx, dr, dweights, dgamma, dbeta,
                          hip_stream);
  if (!is_mlp(d->kind)) return CAAT_EUNSUPPORTED;
  const void* w0 = weights[0]; const void* w1 = weights[1]; const void* gamma = weights[2];
  void* dw0 = dweights[0]; void* dw1 = dweights[1];
  if (!w0 || !w1 || !gamma || !dw0 || !dw1 || (d->norm == CAAT_LAYERNORM && !dbeta)) return CAAT_EINVAL;
  if (misaligned(w0) || misaligned(w1) || misaligned(gamma) || misaligned(dw0) || misaligned(dw1) || misaligned(x) ||
      misaligned(r_out) || misaligned(workspace) || misaligned(dx_out) || misaligned(dr_out) || misaligned(dx) ||
      misaligned(dr))
    return CAAT_EALIGN;
  if (ws_bytes < L.total_bytes) return CAAT_EWORKSPACE;
  if (d->tokens == 0) return CAAT_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  const long long T = d->T, n = d->tokens, h = d->h, fr = d->ffn / d->T;
  const bool swi = d->kind == CAAT_MLP_SWIGLU;
  const long long pw = swi ? 2 * fr : fr;
  const bf16_t* P = (const bf16_t*)(ws + L.off_P);
  const bf16_t* Y = (const bf16_t*)(ws + L.off_Y);
  const float* mean = d->norm == CAAT_LAYERNORM ? (const float*)(ws + L.off_mean) : nullptr;
  const float* rstd = (const float*)(ws + L.off_rstd);
  bf16_t* dZt = (bf16_t*)(ws + L.off_dZt);
  bf16_t* dP = (bf16_t*)(ws + L.off_dP);

  // a6/a7: norm backward per rank FIRST (Fig. 2b): g_m = dr_out_m + NormBwd(dx_out_m); dr_m = g_m un-reduced;
  // a copy with scaled private channels goes to dZt; dgamma/dbeta summed over tokens and ranks
  hipError_t e;
  if (fuse_norm_bwd_reduce(d)) {
    // ... as one launch where the shape allows: the reduce sums the rounded residual gradients straight from the
    // registers of the norm backward instead of reading them back
    ProfScope ps(s, "norm_bwd_sync");
    e = launch_norm_bwd_sync((const bf16_t*)dx_out, (const bf16_t*)dr_out, (const bf16_t*)r_out, (const bf16_t*)gamma, mean,
                             rstd, (bf16_t*)dr, dZt, dgamma, dbeta, d->norm, (int)T, n, (int)h, d->hs, d->private_scale,
                             ws + L.off_scratch, s);
    if (e != hipSuccess) return CAAT_EHIP;
  } else {
    {
      ProfScope ps(s, "norm_bwd");
      e = launch_norm_bwd((const bf16_t*)dx_out, (const bf16_t*)dr_out, (const bf16_t*)r_out, (const bf16_t*)gamma,
                          mean, rstd, (bf16_t*)dr, dZt, dgamma, dbeta, d->norm, (int)T, n, (int)h, d->hs,
                          d->private_scale, ws + L.off_scratch, s, true);
    }
    if (e != hipSuccess) return CAAT_EHIP;
    // a8: the same partial channel-reduce on the gradients, shared channels only, fp32 accumulation.  When no 8-channel
    // vector straddles hs, the norm backward has left dZt's shared channels unwritten and the reduce reads them from dr
    // (the same values) and writes the sums into dZt; otherwise it runs in place on dZt.
    {
      ProfScope ps(s, "partial_sync_bwd");
      e = d->hs % 8 == 0 ? launch_partial_sync_shared_from((const bf16_t*)dr, dZt, (int)T, n, (int)h, d->hs, s)
                         : launch_partial_sync(dZt, nullptr, dZt, (int)T, n, (int)h, d->hs, 1.0f, s);
    }
    if (e != hipSuccess) return CAAT_EHIP;
  }

  // The four GEMMs of the backward pass, in the order G (activation-derivative GEMM), B (dB), X (dX), A (dA).
  // Whichever GEMM runs right behind the streaming norm-backward kernel measured about 20 us slower than elsewhere in
  // the sequence (that kernel's fresh writes are still draining).  The six admissible orders (h = 2048, T = 4, 8192
  // tokens): B G X A 1.637 ms per step, G B X A 1.645, the rest 1.645 - 1.679; B first only moves the slow slot from G
  // to the weight-gradient GEMM (213 -> 221 us averaged over its two launches), so the plain order stays.
  GemmParams q;
  auto run_B = [&]() {
    std::memset(&q, 0, sizeof(q));
    q.a = dZt; q.lda = h; q.stride_a = n * h;
    q.b = Y; q.ldb = fr; q.stride_b = n * fr;
    q.c = (bf16_t*)dw1; q.ldc = fr; q.stride_c = h * fr; q.late_c = 1;
    q.G = (int)T; q.M = (int)h; q.N = (int)fr; q.K = (int)n;
    ProfScope ps(s, "gemm_tn_wgrad");
    return launch_gemm(q, 2, EPI_PLAIN, s);
  };
  auto run_G = [&]() {
    std::memset(&q, 0, sizeof(q));
    q.a = dZt; q.lda = h; q.stride_a = n * h;
    q.b = (const bf16_t*)w1; q.ldb = fr; q.stride_b = h * fr;
    q.c = dP; q.ldc = pw; q.stride_c = n * pw;
    q.aux = P; q.ldaux = pw; q.stride_aux = n * pw;
    q.G = (int)T; q.M = (int)n; q.N = (int)fr; q.K = (int)h; q.half = (int)fr;
    ProfScope ps(s, swi ? "gemm_nn_swiglu_bwd" : "gemm_nn_gelu_bwd");
    return launch_gemm(q, 1, swi ? EPI_SWIGLU_BWD : EPI_GELU_BWD, s);
  };
  auto run_X = [&]() {
    std::memset(&q, 0, sizeof(q));
    q.a = dP; q.lda = pw; q.stride_a = n * pw;
    q.b = (const bf16_t*)w0; q.ldb = h; q.stride_b = pw * h;
    q.c = (bf16_t*)dx; q.ldc = h; q.stride_c = n * h; q.late_c = 1;
    q.G = (int)T; q.M = (int)n; q.N = (int)h; q.K = (int)pw;
    ProfScope ps(s, "gemm_nn_dgrad");
    return launch_gemm(q, 1, EPI_PLAIN, s);
  };
  auto run_A = [&]() {
    std::memset(&q, 0, sizeof(q));
    q.a = dP; q.lda = pw; q.stride_a = n * pw;
    q.b = (const bf16_t*)x; q.ldb = h; q.stride_b = n * h;
    q.c = (bf16_t*)dw0; q.ldc = h; q.stride_c = pw * h; q.late_c = 1;
    q.G = (int)T; q.M = (int)pw; q.N = (int)h; q.K = (int)n;
    ProfScope ps(s, "gemm_tn_wgrad");
    return launch_gemm(q, 2, EPI_PLAIN, s);
  };
  e = run_G();   // a9 + a10: dY_m = dZt_m B_m (NN), fused with the activation derivative -> dP_m
  if (e != hipSuccess) return CAAT_EHIP;
  e = run_B();   // a9: dB_m [h, f/T] = dZt_m^T Y_m (TN, reduction over tokens)
  if (e != hipSuccess) return CAAT_EHIP;
  e = run_X();   // a11: dX_m = dP_m A_m (NN); NOT reduced over ranks (Sec. 4: the only reduce sits at the row-parallel output)
  if (e != hipSuccess) return CAAT_EHIP;
  e = run_A();   // a11: dA_m [pw, h] = dP_m^T X_m (TN)
  return hip_status(e);
}

}  // extern "C"
