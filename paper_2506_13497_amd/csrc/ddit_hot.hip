// C ABI of libddit_hot: argument validation, workspace carving and the sequencing of the
// kernels of one STDiT layer / block / denoising step on the caller's HIP stream.
// Nothing here allocates device memory or synchronises with the host.
#include "../../include/ddit_hot.h"

#include <stdarg.h>
#include <algorithm>
#include <stdio.h>
#include <string.h>

#include "ddit_common.hpp"

namespace ddit {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
  if (e == hipSuccess) return DDIT_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return DDIT_ERR_HIP;
}

int device_cus() {
  static int cus = 0;   // benign race: every thread computes the same value
  if (cus == 0) {
    int dev = 0, n = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
    cus = n > 0 ? n : 256;
  }
  return cus;
}

namespace {

#define DDIT_HIP_TRY(expr, what) do { int rc_ = hip_fail((expr), (what)); if (rc_ != DDIT_OK) return rc_; } while (0)

// Scratch of the entry point that allocates nothing (ddit_stdit_block_fwd_static): the block's
// workspace lives in this file-scope device array.  Every GPU the library runs on holds its own copy
// at its own address until the process ends; host code never passes the array's name to a kernel, only
// the address hipGetSymbolAddress returns for the current device (kept per device below).
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)DDIT_STATIC_SCRATCH_BYTES;
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static void *g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];   // benign race: every thread stores the same address

// device address of `scratch` on the current device, looked up once per device
int static_scratch(void **ptr_out) {
  int dev = -1;
  DDIT_HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) {
    set_error("device index %d outside the %d this library keeps scratch for", dev, STATIC_SCRATCH_MAX_DEVICES);
    return DDIT_ERR_UNSUPPORTED;
  }
  void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    DDIT_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (!p) { set_error("hipGetSymbolAddress(scratch) returned a null address"); return DDIT_ERR_HIP; }
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
  }
  *ptr_out = p;
  return DDIT_OK;
}

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Dims {
  int64_t B, T, S, L, N, D, H, dh, A, M, Ly, n_blocks;
};

struct Layout {
  size_t x, xh, qkv, o, kvc, h, c6, cond, rope, taps, total;
  size_t tap_off[2][DDIT_TAP_COUNT], tap_bytes[DDIT_TAP_COUNT];
};

int check_shape(const ddit_shape *sh, Dims *d) {
  if (!sh) { set_error("shape is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (sh->struct_size != sizeof(ddit_shape)) {
    set_error("shape->struct_size=%u, this library expects %zu", sh->struct_size, sizeof(ddit_shape));
    return DDIT_ERR_INVALID_ARG;
  }
  if (sh->B < 1 || sh->T < 1 || sh->Hp < 1 || sh->Wp < 1 || sh->D < 1 || sh->H < 1 || sh->dh < 1 || sh->M < 1 ||
      sh->Ly < 1 || sh->n_blocks < 0) {
    set_error("shape: every extent must be positive (B=%d T=%d Hp=%d Wp=%d D=%d H=%d dh=%d M=%d Ly=%d n_blocks=%d)",
              sh->B, sh->T, sh->Hp, sh->Wp, sh->D, sh->H, sh->dh, sh->M, sh->Ly, sh->n_blocks);
    return DDIT_ERR_INVALID_ARG;
  }
  if (!(sh->ln_eps > 0.f)) { set_error("shape->ln_eps must be positive"); return DDIT_ERR_INVALID_ARG; }
  if (sh->dh != 64 && sh->dh != 72) { set_error("dh=%d: supported head dims are 64 and 72", sh->dh); return DDIT_ERR_UNSUPPORTED; }
  if (sh->B > 64) { set_error("B=%d: at most 64 samples per call", sh->B); return DDIT_ERR_UNSUPPORTED; }
  const int64_t A = (int64_t)sh->H * sh->dh;
  if (A > sh->D) { set_error("H*dh=%lld exceeds D=%d", (long long)A, sh->D); return DDIT_ERR_UNSUPPORTED; }
  if (sh->D % 8 || sh->M % 8) { set_error("D=%d and M=%d must be multiples of 8", sh->D, sh->M); return DDIT_ERR_UNSUPPORTED; }
  if (sh->D > 4096) { set_error("D=%d: hidden size above 4096 is not supported", sh->D); return DDIT_ERR_UNSUPPORTED; }
  d->B = sh->B; d->T = sh->T; d->S = (int64_t)sh->Hp * sh->Wp; d->L = d->T * d->S; d->N = d->B * d->L;
  d->D = sh->D; d->H = sh->H; d->dh = sh->dh; d->A = A; d->M = sh->M; d->Ly = sh->Ly; d->n_blocks = sh->n_blocks;
  if (d->N > (int64_t)1 << 30) { set_error("B*T*S=%lld tokens: too many", (long long)d->N); return DDIT_ERR_UNSUPPORTED; }
  // The linears index activations and weights with 31 bits; refuse here, before anything is enqueued, every
  // shape one of a layer's launches would refuse later (activation rows of width D, 3A, M; the text rows; the
  // largest weights).
  const int64_t widest = std::max<int64_t>(std::max<int64_t>(3 * A, sh->M), sh->D), lim = (int64_t)1 << 31;
  if (d->N * widest >= lim) {
    set_error("B*T*S * max(3*H*dh, M, D) = %lld x %lld exceeds the 31-bit index range of the linears: split the batch",
              (long long)d->N, (long long)widest);
    return DDIT_ERR_UNSUPPORTED;
  }
  if (d->B * d->Ly * d->D >= lim) { set_error("B*Ly*D=%lld exceeds the 31-bit index range of the linears", (long long)(d->B * d->Ly * d->D)); return DDIT_ERR_UNSUPPORTED; }
  if ((int64_t)sh->M * sh->D >= lim) { set_error("M*D=%lld exceeds the 31-bit weight index range", (long long)sh->M * sh->D); return DDIT_ERR_UNSUPPORTED; }
  return DDIT_OK;
}

void make_layout(const Dims &d, uint32_t flags, Layout *lo) {
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  lo->x = take((size_t)d.N * d.D * 4);
  lo->xh = take((size_t)d.N * d.D * 2);
  lo->qkv = take((size_t)d.N * 3 * d.A * 2);
  lo->o = take((size_t)d.N * d.A * 2);
  // text k|v of every layer of a step (one layer's worth at least: the single-block call uses it layer by layer)
  lo->kvc = take((size_t)(d.n_blocks > 0 ? 2 * d.n_blocks : 1) * d.B * d.Ly * 2 * d.A * 2);
  lo->h = take((size_t)d.N * d.M * 2);
  lo->c6 = take((size_t)d.B * 6 * d.D * 4);
  lo->cond = take((size_t)d.B * (256 + 2 * d.D) * 4);
  lo->rope = (flags & DDIT_FLAG_ROPE_TEMPORAL) ? take((size_t)d.T * d.dh * 4) : 0;
  lo->taps = off;
  const size_t ND = (size_t)d.N * d.D, NA = (size_t)d.N * d.A;
  const size_t tb[DDIT_TAP_COUNT] = {ND * 2, 3 * NA * 2, NA * 2, ND * 4, NA * 2, (size_t)d.B * d.Ly * 2 * d.A * 2,
                                     NA * 2, ND * 4, ND * 2, (size_t)d.N * d.M * 2, ND * 4};
  for (int t = 0; t < DDIT_TAP_COUNT; ++t) lo->tap_bytes[t] = tb[t];
  if (flags & DDIT_FLAG_TAPS) {
    for (int l = 0; l < 2; ++l)
      for (int t = 0; t < DDIT_TAP_COUNT; ++t) lo->tap_off[l][t] = take(tb[t]);
  }
  lo->total = off;
}

int check_valid_len(const int32_t *vl, const Dims &d) {
  if (!vl) return DDIT_OK;
  for (int b = 0; b < d.B; ++b)
    if (vl[b] < 1 || vl[b] > d.Ly) {
      set_error("valid_len[%d]=%d outside [1,%lld]", b, vl[b], (long long)d.Ly);
      return DDIT_ERR_INVALID_ARG;
    }
  return DDIT_OK;
}

int check_layer_weights(const ddit_layer_weights &w, const char *which, uint32_t flags) {
  if (flags & DDIT_FLAG_QK_NORM) {
    if (!w.g_q || !w.g_k) { set_error("%s: DDIT_FLAG_QK_NORM needs g_q and g_k", which); return DDIT_ERR_INVALID_ARG; }
    if (!aligned16(w.g_q) || !aligned16(w.g_k)) { set_error("%s: g_q / g_k not 16-byte aligned", which); return DDIT_ERR_ALIGNMENT; }
  }
  const void *req[] = {w.w_qkv, w.w_o, w.w_cq, w.w_ckv, w.w_co, w.w_fc1, w.w_fc2, w.ada_table};
  const char *names[] = {"w_qkv", "w_o", "w_cq", "w_ckv", "w_co", "w_fc1", "w_fc2", "ada_table"};
  for (int i = 0; i < 8; ++i)
    if (!req[i]) { set_error("%s.%s is NULL", which, names[i]); return DDIT_ERR_INVALID_ARG; }
  const void *all[] = {w.w_qkv, w.b_qkv, w.w_o, w.b_o, w.w_cq, w.b_cq, w.w_ckv, w.b_ckv,
                       w.w_co, w.b_co, w.w_fc1, w.b_fc1, w.w_fc2, w.b_fc2, w.ada_table};
  for (const void *p : all)
    if (p && !aligned16(p)) { set_error("%s: a weight pointer is not 16-byte aligned", which); return DDIT_ERR_ALIGNMENT; }
  return DDIT_OK;
}

// q_norm_g (bf16 [dh] or null): the streaming kernel RMS-normalises the queries with these scales as it
// loads them (spatial layers with the q/k normalisation option)
int run_attention(ddit_attn_kind kind, const Dims &d, const void *q, const void *k, const void *v, int64_t ld_q,
                  int64_t ld_kv, const int32_t *valid_len, void *o, int64_t ld_o, float *lse, hipStream_t s,
                  const void *q_norm_g = nullptr, float q_norm_eps = 0.f) {
  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
  a.q_norm_g = q_norm_g; a.q_norm_eps = q_norm_eps;
  a.ld_q = ld_q; a.ld_kv = ld_kv; a.ld_o = ld_o;
  a.H = (int)d.H; a.dh = (int)d.dh;
  switch (kind) {
    case DDIT_ATTN_SPATIAL:
      a.n_groups = (int)(d.B * d.T); a.g_inner = 1;
      a.q_outer = a.kv_outer = d.S; a.q_inner = a.kv_inner = 0;
      a.q_tok_step = a.kv_tok_step = 1;
      a.Lq = a.Lk_max = (int)d.S;
      break;
    case DDIT_ATTN_TEMPORAL:
      // short sequences (one matrix-core tile of frames): the dedicated kernel; longer ones take
      // the generic streaming kernel with strided groups
      if (d.T <= temporal_attn_max_T())
        return launch_temporal_attn(q, k, v, o, lse, ld_q, ld_kv, ld_o, (int)d.B, (int)d.T, (int)d.S, (int)d.H,
                                    (int)d.dh, nullptr, nullptr, 0.f, nullptr, s);
      a.n_groups = (int)(d.B * d.S); a.g_inner = (int)d.S;
      a.q_outer = a.kv_outer = d.T * d.S; a.q_inner = a.kv_inner = 1;
      a.q_tok_step = a.kv_tok_step = d.S;
      a.Lq = a.Lk_max = (int)d.T;
      break;
    case DDIT_ATTN_CROSS:
      a.n_groups = (int)d.B; a.g_inner = 1;
      a.q_outer = d.L; a.kv_outer = d.Ly; a.q_inner = a.kv_inner = 0;
      a.q_tok_step = a.kv_tok_step = 1;
      a.Lq = (int)d.L; a.Lk_max = (int)d.Ly;
      if (valid_len) {
        a.use_kv_len = 1;
        for (int b = 0; b < d.B; ++b) a.kv_len[b] = valid_len[b];
      }
      break;
    default:
      set_error("unknown attention kind %d", (int)kind);
      return DDIT_ERR_INVALID_ARG;
  }
  return launch_flash_attn(a, s);
}

// Self-attention with the two optional treatments of q and k (per-head RMS normalisation with scales g_q,
// g_k, both or neither; rotation by rope_table, temporal only), done where it costs least:
//   temporal, T within the dedicated kernel: inside that kernel, after the operands have landed in LDS;
//   spatial: the queries inside the attention kernel as they are loaded, the keys (which every query tile
//            re-reads) once, in place, by the streaming kernel;
//   otherwise, or with fuse == false: q and k in place by the streaming kernel, then the plain attention.
// q and k may therefore be overwritten with their treated values.
int run_self_attention(ddit_attn_kind kind, const Dims &d, void *q, void *k, const void *v, int64_t ld_q, int64_t ld_kv,
                       const void *g_q, const void *g_k, float eps, const float *rope_table, bool fuse, void *o,
                       int64_t ld_o, float *lse, hipStream_t s) {
  const float *rope = kind == DDIT_ATTN_TEMPORAL ? rope_table : nullptr;
  if (!g_q && !rope) return run_attention(kind, d, q, k, v, ld_q, ld_kv, nullptr, o, ld_o, lse, s);
  const int H = (int)d.H, dh = (int)d.dh;
  if (fuse && kind == DDIT_ATTN_TEMPORAL && d.T <= temporal_attn_max_T())
    return launch_temporal_attn(q, k, v, o, lse, ld_q, ld_kv, ld_o, (int)d.B, (int)d.T, (int)d.S, H, dh, g_q, g_k, eps,
                                rope, s);
  if (fuse && kind == DDIT_ATTN_SPATIAL) {
    int rc = launch_qk_norm_rope(k, ld_kv, d.N, H, 0, dh, g_q, g_k, eps, nullptr, d.S, (int)d.T, s);
    if (rc != DDIT_OK) return rc;
    return run_attention(kind, d, q, k, v, ld_q, ld_kv, nullptr, o, ld_o, lse, s, g_q, eps);
  }
  int rc;
  if (ld_q == ld_kv && reinterpret_cast<unsigned char *>(k) == reinterpret_cast<unsigned char *>(q) + d.A * 2) {
    rc = launch_qk_norm_rope(q, ld_q, d.N, 2 * H, H, dh, g_q, g_k, eps, rope, d.S, (int)d.T, s);   // q | k side by side
  } else {
    rc = launch_qk_norm_rope(q, ld_q, d.N, H, H, dh, g_q, g_k, eps, rope, d.S, (int)d.T, s);
    if (rc == DDIT_OK) rc = launch_qk_norm_rope(k, ld_kv, d.N, H, 0, dh, g_q, g_k, eps, rope, d.S, (int)d.T, s);
  }
  if (rc != DDIT_OK) return rc;
  return run_attention(kind, d, q, k, v, ld_q, ld_kv, nullptr, o, ld_o, lse, s);
}

struct Taps {
  bool on; unsigned char *ws; const Layout *lo; int layer; hipStream_t s;
  int keep(int tap, const void *src) const {
    if (!on) return DDIT_OK;
    return hip_fail(hipMemcpyAsync(ws + lo->tap_off[layer][tap], src, lo->tap_bytes[tap], hipMemcpyDeviceToDevice, s),
                    "tap copy");
  }
};

#define DDIT_TRY(expr) do { int rc_ = (expr); if (rc_ != DDIT_OK) return rc_; } while (0)

// One layer on the fp32 stream x (in the workspace).
// kvc_cached: this layer's cross-attention k|v [B*Ly, 2A] formed earlier, or null (then y is projected here)
int run_layer(ddit_attn_kind kind, const Dims &d, const ddit_layer_weights &w, const void *y, const void *kvc_cached,
              const int32_t *valid_len, const float *c6, float eps, uint32_t flags, unsigned char *ws,
              const Layout &lo, const Taps &tp, hipStream_t s) {
  float *x = reinterpret_cast<float *>(ws + lo.x);
  void *xh = ws + lo.xh;
  unsigned char *qkv = ws + lo.qkv;
  void *o = ws + lo.o;
  const unsigned char *kvc = kvc_cached ? reinterpret_cast<const unsigned char *>(kvc_cached) : ws + lo.kvc;
  void *h = ws + lo.h;
  const int64_t N = d.N, D = d.D, A = d.A, M = d.M;

  GemmArgs g;
  auto base = [&](const void *u, int64_t ld_u, const void *W, const void *b, int64_t rows, int n, int k) {
    memset(&g, 0, sizeof(g)); g.tile = -1;
    g.u = u; g.ld_u = ld_u; g.W = W; g.bias = b; g.N = rows; g.n = n; g.k = k; g.tokens_per_sample = d.L;
  };
  auto gated = [&](int row) {
    g.resid = x;
    if (row >= 0) { g.gate_tab = w.ada_table + (int64_t)row * D; g.gate_c6 = c6 + (int64_t)row * D; g.gate_c6_stride = 6 * D; }
  };

  // self-attention branch
  DDIT_TRY(launch_modulated_layernorm(x, w.ada_table, c6, 0, N, d.L, (int)D, eps, xh, s));
  DDIT_TRY(tp.keep(DDIT_TAP_XH_MSA, xh));
  base(xh, D, w.w_qkv, w.b_qkv, N, (int)(3 * A), (int)D); g.out = qkv; g.ld_out = 3 * A;
  DDIT_TRY(launch_gemm(DDIT_EPI_BF16, g, s));
  {
    // With taps the treated q | k must be visible in memory (the tap shows what the attention reads), so
    // the treatment then runs as a pass of its own; otherwise it is folded into the attention kernels.
    const bool norm = (flags & DDIT_FLAG_QK_NORM) != 0, rope = (flags & DDIT_FLAG_ROPE_TEMPORAL) != 0;
    const void *gq = norm ? w.g_q : nullptr, *gk = norm ? w.g_k : nullptr;
    const float *tab = rope ? reinterpret_cast<const float *>(ws + lo.rope) : nullptr;
    if (tp.on) {
      DDIT_TRY(launch_qk_norm_rope(qkv, 3 * A, N, 2 * (int)d.H, (int)d.H, (int)d.dh, gq, gk, eps,
                                   kind == DDIT_ATTN_TEMPORAL ? tab : nullptr, d.S, (int)d.T, s));
      DDIT_TRY(tp.keep(DDIT_TAP_QKV, qkv));
      DDIT_TRY(run_attention(kind, d, qkv, qkv + A * 2, qkv + 2 * A * 2, 3 * A, 3 * A, nullptr, o, A, nullptr, s));
    } else {
      DDIT_TRY(run_self_attention(kind, d, qkv, qkv + A * 2, qkv + 2 * A * 2, 3 * A, 3 * A, gq, gk, eps, tab, true, o, A,
                                  nullptr, s));
    }
  }
  DDIT_TRY(tp.keep(DDIT_TAP_O, o));
  base(o, A, w.w_o, w.b_o, N, (int)D, (int)A); gated(2); g.out = xh; g.ld_out = D;   // also xh := bf16(x)
  DDIT_TRY(launch_gemm(DDIT_EPI_RESIDUAL_F32, g, s));
  DDIT_TRY(tp.keep(DDIT_TAP_X_AFTER_ATTN, x));

  // cross-attention branch (reads the stream itself; ungated)
  base(xh, D, w.w_cq, w.b_cq, N, (int)A, (int)D); g.out = qkv; g.ld_out = 3 * A;
  DDIT_TRY(launch_gemm(DDIT_EPI_BF16, g, s));
  if (!kvc_cached) {
    base(y, D, w.w_ckv, w.b_ckv, d.B * d.Ly, (int)(2 * A), (int)D); g.out = ws + lo.kvc; g.ld_out = 2 * A;
    DDIT_TRY(launch_gemm(DDIT_EPI_BF16, g, s));
  }
  if (tp.on) {  // q_c lives strided inside the qkv buffer: copy it out row by row
    DDIT_TRY(hip_fail(hipMemcpy2DAsync(tp.ws + lo.tap_off[tp.layer][DDIT_TAP_QC], A * 2, qkv, 3 * A * 2, A * 2, N,
                                       hipMemcpyDeviceToDevice, s), "tap copy"));
  }
  DDIT_TRY(tp.keep(DDIT_TAP_KVC, kvc));
  DDIT_TRY(run_attention(DDIT_ATTN_CROSS, d, qkv, kvc, kvc + A * 2, 3 * A, 2 * A, valid_len, o, A, nullptr, s));
  DDIT_TRY(tp.keep(DDIT_TAP_OC, o));
  base(o, A, w.w_co, w.b_co, N, (int)D, (int)A); gated(-1);
  DDIT_TRY(launch_gemm(DDIT_EPI_RESIDUAL_F32, g, s));
  DDIT_TRY(tp.keep(DDIT_TAP_X_AFTER_CROSS, x));

  // MLP branch
  DDIT_TRY(launch_modulated_layernorm(x, w.ada_table, c6, 1, N, d.L, (int)D, eps, xh, s));
  DDIT_TRY(tp.keep(DDIT_TAP_XH_MLP, xh));
  base(xh, D, w.w_fc1, w.b_fc1, N, (int)M, (int)D); g.out = h; g.ld_out = M;
  DDIT_TRY(launch_gemm(DDIT_EPI_GELU_BF16, g, s));
  DDIT_TRY(tp.keep(DDIT_TAP_H, h));
  base(h, M, w.w_fc2, w.b_fc2, N, (int)D, (int)M); gated(5);
  DDIT_TRY(launch_gemm(DDIT_EPI_RESIDUAL_F32, g, s));
  DDIT_TRY(tp.keep(DDIT_TAP_X_OUT, x));
  return DDIT_OK;
}

// Text k|v projections of all 2 * n_blocks layers: y [B*Ly, D] against every layer's w_ckv, layer l's result at
// out + l * (B*Ly*2A*2 bytes).  One grouped launch where the shape allows it (the projections share y and are
// far too small, one by one, for the chip), else layer by layer.
int project_text_kv(const Dims &d, const ddit_step_weights *weights, const void *y, unsigned char *out, hipStream_t s) {
  const size_t per_layer = (size_t)d.B * d.Ly * 2 * d.A * 2;
  const int layers = (int)(2 * d.n_blocks);
  GemmArgs g;
  memset(&g, 0, sizeof(g)); g.tile = -1;
  g.u = y; g.ld_u = d.D; g.N = d.B * d.Ly; g.n = (int)(2 * d.A); g.k = (int)d.D; g.ld_out = 2 * d.A; g.tokens_per_sample = d.Ly;
  constexpr int CHUNK = 128;
  for (int l0 = 0; l0 < layers; l0 += CHUNK) {
    const int G = layers - l0 < CHUNK ? layers - l0 : CHUNK;
    const void *W[CHUNK], *bias[CHUNK];
    void *o[CHUNK];
    for (int j = 0; j < G; ++j) {
      const int l = l0 + j;
      const ddit_layer_weights &w = (l & 1) ? weights->blocks[l >> 1].temporal : weights->blocks[l >> 1].spatial;
      W[j] = w.w_ckv; bias[j] = w.b_ckv; o[j] = out + (size_t)l * per_layer;
    }
    int rc = launch_gemm_grouped(g, G, W, bias, o, s);
    if (rc == 1) {
      for (int j = 0; j < G; ++j) {
        g.W = W[j]; g.bias = bias[j]; g.out = o[j];
        DDIT_TRY(launch_gemm(DDIT_EPI_BF16, g, s));
      }
    } else if (rc != 0) {
      return rc;
    }
  }
  return DDIT_OK;
}

int check_common(const Dims &d, const Layout &lo, const void *x_in, const void *y, const void *x_out, void *ws,
                 size_t ws_bytes) {
  if (!x_in || !y || !x_out) { set_error("x_in, y and x_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(x_in) || !aligned16(y) || !aligned16(x_out)) {
    set_error("x_in, y and x_out must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  if (!ws || ws_bytes < lo.total) {
    set_error("workspace of %zu bytes given, %zu required", ws ? ws_bytes : (size_t)0, lo.total);
    return DDIT_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(ws) & 255u) { set_error("workspace must be 256-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  (void)d;
  return DDIT_OK;
}

// ---- latent in / latent out ----------------------------------------------------------------
struct IoLayout {
  size_t step;      // the step's own workspace starts at 0
  size_t pos, x_tok, x_res, cap, cond, total;
};

int check_io(const ddit_shape *sh, const Dims &d, const ddit_io_weights *io) {
  if (!io) { set_error("io weights are NULL"); return DDIT_ERR_INVALID_ARG; }
  if (io->struct_size != sizeof(ddit_io_weights)) {
    set_error("io->struct_size=%u, this library expects %zu", io->struct_size, sizeof(ddit_io_weights));
    return DDIT_ERR_INVALID_ARG;
  }
  if (io->C_in < 1 || io->C_out < 1 || io->C_text < 1) {
    set_error("io: C_in=%d C_out=%d C_text=%d must be positive", io->C_in, io->C_out, io->C_text);
    return DDIT_ERR_INVALID_ARG;
  }
  if (4 * io->C_in > 64 || 4 * io->C_out > 64) {
    set_error("io: C_in=%d, C_out=%d: at most 16 latent channels", io->C_in, io->C_out); return DDIT_ERR_UNSUPPORTED;
  }
  if (io->C_text % 8) { set_error("io: C_text=%d must be a multiple of 8", io->C_text); return DDIT_ERR_UNSUPPORTED; }
  if (d.D % 4) { set_error("D=%lld must be a multiple of 4 for the position code", (long long)d.D); return DDIT_ERR_UNSUPPORTED; }
  (void)sh;
  return DDIT_OK;
}

void make_io_layout(const Dims &d, uint32_t flags, IoLayout *lo) {
  Layout st;
  make_layout(d, flags, &st);
  size_t off = st.total;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  lo->step = 0;
  lo->pos = take((size_t)d.S * d.D * 4);
  lo->x_tok = take((size_t)d.N * d.D * 2);
  lo->x_res = take((size_t)d.N * d.D * 2);
  lo->cap = take((size_t)d.B * d.Ly * d.D * 2);
  lo->cond = take((size_t)d.B * (256 + 2 * d.D) * 4 + (size_t)d.B * 6 * d.D * 4);
  lo->total = off;
}

int check_ws(void *ws, size_t ws_bytes, size_t need) {
  if (!ws || ws_bytes < need) {
    set_error("workspace of %zu bytes given, %zu required", ws ? ws_bytes : (size_t)0, need);
    return DDIT_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(ws) & 255u) { set_error("workspace must be 256-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  return DDIT_OK;
}

}  // namespace
}  // namespace ddit

using namespace ddit;

extern "C" {

uint32_t ddit_abi_version(void) { return DDIT_ABI_VERSION; }

const char *ddit_status_string(int status) {
  switch (status) {
    case DDIT_OK: return "ok";
    case DDIT_ERR_INVALID_ARG: return "invalid argument";
    case DDIT_ERR_UNSUPPORTED: return "unsupported shape";
    case DDIT_ERR_WORKSPACE: return "workspace missing or too small";
    case DDIT_ERR_ALIGNMENT: return "misaligned pointer or leading dimension";
    case DDIT_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

const char *ddit_last_error(void) { return g_err; }

int ddit_workspace_bytes(const ddit_shape *shape, size_t *bytes_out) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (!bytes_out) { set_error("bytes_out is NULL"); return DDIT_ERR_INVALID_ARG; }
  Layout lo;
  make_layout(d, shape->flags, &lo);
  *bytes_out = lo.total;
  return DDIT_OK;
}

int ddit_tap_region(const ddit_shape *shape, int layer, int tap, size_t *offset_out, size_t *bytes_out) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (!(shape->flags & DDIT_FLAG_TAPS)) { set_error("DDIT_FLAG_TAPS is not set in shape->flags"); return DDIT_ERR_INVALID_ARG; }
  if (layer < 0 || layer > 1 || tap < 0 || tap >= DDIT_TAP_COUNT || !offset_out || !bytes_out) {
    set_error("tap_region: layer=%d tap=%d out of range or NULL output", layer, tap);
    return DDIT_ERR_INVALID_ARG;
  }
  Layout lo;
  make_layout(d, shape->flags, &lo);
  *offset_out = lo.tap_off[layer][tap];
  *bytes_out = lo.tap_bytes[tap];
  return DDIT_OK;
}

int ddit_attn_fwd(ddit_attn_kind kind, const ddit_shape *shape, const void *q, const void *k, const void *v,
                  int64_t ld_q, int64_t ld_kv, const int32_t *kv_valid_len_host, void *o, int64_t ld_o,
                  float *lse_or_null, void *workspace, size_t workspace_bytes, void *hip_stream) {
  (void)workspace; (void)workspace_bytes;
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (kind != DDIT_ATTN_SPATIAL && kind != DDIT_ATTN_TEMPORAL && kind != DDIT_ATTN_CROSS) {
    set_error("unknown attention kind %d", (int)kind); return DDIT_ERR_INVALID_ARG;
  }
  if (!q || !k || !v || !o) { set_error("q, k, v and o must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) {
    set_error("q, k, v and o must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  if (ld_q < d.A || ld_kv < d.A || ld_o < d.A) {
    set_error("leading dimensions (%lld,%lld,%lld) must be at least H*dh=%lld", (long long)ld_q, (long long)ld_kv,
              (long long)ld_o, (long long)d.A);
    return DDIT_ERR_INVALID_ARG;
  }
  if (ld_q % 8 || ld_kv % 8 || ld_o % 8) { set_error("leading dimensions must be multiples of 8"); return DDIT_ERR_ALIGNMENT; }
  if (kind == DDIT_ATTN_CROSS) DDIT_TRY(check_valid_len(kv_valid_len_host, d));
  return run_attention(kind, d, q, k, v, ld_q, ld_kv, kind == DDIT_ATTN_CROSS ? kv_valid_len_host : nullptr, o, ld_o,
                       lse_or_null, reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_stdit_block_fwd(const ddit_shape *shape, const ddit_block_weights *weights, const void *x_in,
                         const void *y, const int32_t *y_valid_len_host, const float *c6, void *x_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  Layout lo;
  make_layout(d, shape->flags, &lo);
  if (!weights || !c6) { set_error("weights and c6 must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(c6)) { set_error("c6 must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  DDIT_TRY(check_common(d, lo, x_in, y, x_out, workspace, workspace_bytes));
  DDIT_TRY(check_valid_len(y_valid_len_host, d));
  DDIT_TRY(check_layer_weights(weights->spatial, "spatial", shape->flags));
  DDIT_TRY(check_layer_weights(weights->temporal, "temporal", shape->flags));
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  float *x = reinterpret_cast<float *>(ws + lo.x);
  Taps tp{(shape->flags & DDIT_FLAG_TAPS) != 0, ws, &lo, 0, s};
  DDIT_TRY(launch_cast_bf16_to_f32(x_in, x, d.N * d.D, s));
  if (shape->flags & DDIT_FLAG_ROPE_TEMPORAL)
    DDIT_TRY(launch_rope_table(reinterpret_cast<float *>(ws + lo.rope), (int)d.T, (int)d.dh, s));
  DDIT_TRY(run_layer(DDIT_ATTN_SPATIAL, d, weights->spatial, y, nullptr, y_valid_len_host, c6, shape->ln_eps, shape->flags, ws, lo, tp, s));
  tp.layer = 1;
  DDIT_TRY(run_layer(DDIT_ATTN_TEMPORAL, d, weights->temporal, y, nullptr, y_valid_len_host, c6, shape->ln_eps, shape->flags, ws, lo, tp, s));
  return launch_cast_f32_to_bf16(x, x_out, d.N * d.D, s);
}

int ddit_stdit_block_fwd_static(const ddit_shape *shape, const ddit_block_weights *weights, const void *x_in,
                                const void *y, const int32_t *y_valid_len_host, const float *c6, void *x_out,
                                void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (shape->flags & DDIT_FLAG_TAPS) {
    set_error("ddit_stdit_block_fwd_static keeps no taps: clear DDIT_FLAG_TAPS"); return DDIT_ERR_UNSUPPORTED;
  }
  Layout lo;
  make_layout(d, shape->flags, &lo);
  if (lo.total > STATIC_SCRATCH_BYTES) {
    set_error("this shape needs %zu bytes of workspace; the built-in scratch of ddit_stdit_block_fwd_static holds %zu "
              "(use ddit_stdit_block_fwd with a caller-owned workspace)", lo.total, STATIC_SCRATCH_BYTES);
    return DDIT_ERR_WORKSPACE;
  }
  void *ws = nullptr;
  DDIT_TRY(static_scratch(&ws));
  // nothing in the block's workspace has to start at zero: every region is written before it is read
  return ddit_stdit_block_fwd(shape, weights, x_in, y, y_valid_len_host, c6, x_out, ws, STATIC_SCRATCH_BYTES, hip_stream);
}

int ddit_timestep_conditioning(const ddit_shape *shape, const ddit_step_weights *weights,
                               const float *timesteps_host, const float *temb_or_null, float *c6_out,
                               float *scratch, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (!weights || !c6_out || !weights->w_ada) { set_error("weights, w_ada and c6_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!temb_or_null) {
    if (!timesteps_host || !weights->w_t1 || !weights->w_t2 || !scratch) {
      set_error("timesteps_host, w_t1, w_t2 and scratch are required when no temb is given");
      return DDIT_ERR_INVALID_ARG;
    }
    if (!aligned16(weights->w_t1) || !aligned16(weights->w_t2)) { set_error("w_t1/w_t2 not 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  }
  if (!aligned16(weights->w_ada)) { set_error("w_ada not 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  CondArgs c;
  memset(&c, 0, sizeof(c));
  c.B = (int)d.B; c.D = (int)d.D;
  if (!temb_or_null)
    for (int b = 0; b < d.B; ++b) c.t[b] = timesteps_host[b];
  return launch_timestep_conditioning(c, weights->w_t1, weights->b_t1, weights->w_t2, weights->b_t2, weights->w_ada,
                                      weights->b_ada, temb_or_null, c6_out, scratch,
                                      reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_cross_kv_bytes(const ddit_shape *shape, size_t *bytes_out) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (!bytes_out) { set_error("bytes_out is NULL"); return DDIT_ERR_INVALID_ARG; }
  *bytes_out = (size_t)2 * shape->n_blocks * d.B * d.Ly * 2 * d.A * 2;
  return DDIT_OK;
}

int ddit_cross_kv_precompute(const ddit_shape *shape, const ddit_step_weights *weights, const void *y,
                             void *cross_kv_out, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (!weights || !y || !cross_kv_out) { set_error("weights, y and cross_kv_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (shape->n_blocks > 0 && !weights->blocks) { set_error("weights->blocks is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(y) || !aligned16(cross_kv_out)) { set_error("y and cross_kv_out must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  for (int i = 0; i < shape->n_blocks; ++i)
    for (const ddit_layer_weights *w : {&weights->blocks[i].spatial, &weights->blocks[i].temporal}) {
      if (!w->w_ckv) { set_error("block %d: w_ckv is NULL", i); return DDIT_ERR_INVALID_ARG; }
      if (!aligned16(w->w_ckv) || (w->b_ckv && !aligned16(w->b_ckv))) { set_error("block %d: w_ckv/b_ckv not 16-byte aligned", i); return DDIT_ERR_ALIGNMENT; }
    }
  return project_text_kv(d, weights, y, reinterpret_cast<unsigned char *>(cross_kv_out), reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_denoise_step(const ddit_shape *shape, const ddit_step_weights *weights, const void *x_in,
                      const void *y, const int32_t *y_valid_len_host, const float *timesteps_host,
                      const float *temb_or_null, void *x_out, void *workspace, size_t workspace_bytes,
                      void *hip_stream) {
  return ddit_denoise_step_cached(shape, weights, x_in, y, nullptr, y_valid_len_host, timesteps_host, temb_or_null,
                                  x_out, workspace, workspace_bytes, hip_stream);
}

int ddit_denoise_step_cached(const ddit_shape *shape, const ddit_step_weights *weights, const void *x_in,
                             const void *y, const void *cross_kv_or_null, const int32_t *y_valid_len_host,
                             const float *timesteps_host, const float *temb_or_null, void *x_out,
                             void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  Layout lo;
  make_layout(d, shape->flags, &lo);
  if (!weights) { set_error("weights is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (cross_kv_or_null) {
    if (!aligned16(cross_kv_or_null)) { set_error("cross_kv must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
    if (!y) y = cross_kv_or_null;   // y is not read when every layer's k|v is cached; keep the checks below uniform
  }
  if (shape->n_blocks > 0 && !weights->blocks) { set_error("weights->blocks is NULL"); return DDIT_ERR_INVALID_ARG; }
  DDIT_TRY(check_common(d, lo, x_in, y, x_out, workspace, workspace_bytes));
  DDIT_TRY(check_valid_len(y_valid_len_host, d));
  for (int i = 0; i < shape->n_blocks; ++i) {
    DDIT_TRY(check_layer_weights(weights->blocks[i].spatial, "spatial", shape->flags));
    DDIT_TRY(check_layer_weights(weights->blocks[i].temporal, "temporal", shape->flags));
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  float *x = reinterpret_cast<float *>(ws + lo.x);
  float *c6 = reinterpret_cast<float *>(ws + lo.c6);
  DDIT_TRY(ddit_timestep_conditioning(shape, weights, timesteps_host, temb_or_null, c6,
                                      reinterpret_cast<float *>(ws + lo.cond), hip_stream));
  Taps tp{(shape->flags & DDIT_FLAG_TAPS) != 0, ws, &lo, 0, s};
  DDIT_TRY(launch_cast_bf16_to_f32(x_in, x, d.N * d.D, s));
  if (shape->flags & DDIT_FLAG_ROPE_TEMPORAL)
    DDIT_TRY(launch_rope_table(reinterpret_cast<float *>(ws + lo.rope), (int)d.T, (int)d.dh, s));
  const size_t kv_layer = (size_t)d.B * d.Ly * 2 * d.A * 2;
  const unsigned char *kv = reinterpret_cast<const unsigned char *>(cross_kv_or_null);
  if (!kv && shape->n_blocks > 0) {
    // no cache given: the text k|v of every layer are formed here, in one grouped launch, into the workspace
    for (int i = 0; i < shape->n_blocks; ++i)
      for (const ddit_layer_weights *w : {&weights->blocks[i].spatial, &weights->blocks[i].temporal})
        if (!w->w_ckv) { set_error("block %d: w_ckv is NULL", i); return DDIT_ERR_INVALID_ARG; }
    DDIT_TRY(project_text_kv(d, weights, y, ws + lo.kvc, s));
    kv = ws + lo.kvc;
  }
  for (int i = 0; i < shape->n_blocks; ++i) {
    tp.layer = 0;
    DDIT_TRY(run_layer(DDIT_ATTN_SPATIAL, d, weights->blocks[i].spatial, y, kv ? kv + (size_t)(2 * i) * kv_layer : nullptr,
                       y_valid_len_host, c6, shape->ln_eps, shape->flags, ws, lo, tp, s));
    tp.layer = 1;
    DDIT_TRY(run_layer(DDIT_ATTN_TEMPORAL, d, weights->blocks[i].temporal, y,
                       kv ? kv + (size_t)(2 * i + 1) * kv_layer : nullptr, y_valid_len_host, c6, shape->ln_eps, shape->flags, ws, lo, tp, s));
  }
  return launch_cast_f32_to_bf16(x, x_out, d.N * d.D, s);
}

int ddit_modulated_layernorm_fwd(const float *x, const float *ada_table, const float *c6, int which,
                                 int64_t N, int64_t tokens_per_sample, int32_t D, float eps, void *out,
                                 void *hip_stream) {
  if (!x || !ada_table || !c6 || !out) { set_error("x, ada_table, c6 and out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (which < 0 || which > 1 || N < 0 || tokens_per_sample < 1 || D < 1 || !(eps > 0.f)) {
    set_error("modulated_layernorm: which=%d N=%lld tokens_per_sample=%lld D=%d", which, (long long)N,
              (long long)tokens_per_sample, D);
    return DDIT_ERR_INVALID_ARG;
  }
  if (D % 8) { set_error("D=%d must be a multiple of 8", D); return DDIT_ERR_UNSUPPORTED; }
  if (!aligned16(x) || !aligned16(ada_table) || !aligned16(c6) || !aligned16(out)) {
    set_error("pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  return launch_modulated_layernorm(x, ada_table, c6, which, N, tokens_per_sample, D, eps, out,
                                    reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_qk_norm_rope_fwd(void *qk, int64_t ld, int64_t N, int32_t H, int32_t dh, const void *g_q, const void *g_k,
                          float eps, int64_t S, int32_t T, float *rope_table_or_null, void *hip_stream) {
  if (!qk) { set_error("qk must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (N < 0 || H < 1 || S < 1 || T < 1 || !(eps > 0.f)) {
    set_error("qk_norm_rope: N=%lld H=%d S=%lld T=%d eps=%g", (long long)N, H, (long long)S, T, (double)eps);
    return DDIT_ERR_INVALID_ARG;
  }
  if (dh != 64 && dh != 72) { set_error("dh=%d: supported head dims are 64 and 72", dh); return DDIT_ERR_UNSUPPORTED; }
  if ((g_q == nullptr) != (g_k == nullptr)) { set_error("g_q and g_k must be given together"); return DDIT_ERR_INVALID_ARG; }
  if (ld < 2 * (int64_t)H * dh || ld % 8) { set_error("ld=%lld invalid for 2*H*dh=%lld", (long long)ld, 2LL * H * dh); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(qk) || (g_q && (!aligned16(g_q) || !aligned16(g_k))) || (rope_table_or_null && !aligned16(rope_table_or_null))) {
    set_error("pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (rope_table_or_null) DDIT_TRY(launch_rope_table(rope_table_or_null, T, dh, s));
  return launch_qk_norm_rope(qk, ld, N, 2 * H, H, dh, g_q, g_k, eps, rope_table_or_null, S, T, s);
}

int ddit_self_attn_fwd(ddit_attn_kind kind, const ddit_shape *shape, void *q, void *k, const void *v, int64_t ld_q,
                       int64_t ld_kv, const void *g_q, const void *g_k, float *rope_table_or_null, int fuse, void *o,
                       int64_t ld_o, float *lse_or_null, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  if (kind != DDIT_ATTN_SPATIAL && kind != DDIT_ATTN_TEMPORAL) { set_error("self-attention kind must be spatial or temporal"); return DDIT_ERR_INVALID_ARG; }
  if (!q || !k || !v || !o) { set_error("q, k, v and o must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if ((g_q == nullptr) != (g_k == nullptr)) { set_error("g_q and g_k must be given together"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (g_q && (!aligned16(g_q) || !aligned16(g_k))) ||
      (rope_table_or_null && !aligned16(rope_table_or_null))) {
    set_error("pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  if (ld_q < d.A || ld_kv < d.A || ld_o < d.A) { set_error("leading dimensions must be at least H*dh=%lld", (long long)d.A); return DDIT_ERR_INVALID_ARG; }
  if (ld_q % 8 || ld_kv % 8 || ld_o % 8) { set_error("leading dimensions must be multiples of 8"); return DDIT_ERR_ALIGNMENT; }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const float *tab = nullptr;
  if (rope_table_or_null && kind == DDIT_ATTN_TEMPORAL) {
    DDIT_TRY(launch_rope_table(rope_table_or_null, (int)d.T, (int)d.dh, s));
    tab = rope_table_or_null;
  }
  return run_self_attention(kind, d, q, k, v, ld_q, ld_kv, g_q, g_k, shape->ln_eps, tab, fuse != 0, o, ld_o, lse_or_null, s);
}

int ddit_linear_tile_count(void) { return gemm_tile_count(); }

int ddit_linear_tile_info(int tile, int32_t *rows, int32_t *cols, int32_t *wavefronts, int32_t *workgroups_per_cu) {
  int r, c, w, g;
  if (gemm_tile_info(tile, &r, &c, &w, &g) != 0) {
    set_error("no tile %d (there are %d)", tile, gemm_tile_count());
    return DDIT_ERR_INVALID_ARG;
  }
  if (rows) *rows = r;
  if (cols) *cols = c;
  if (wavefronts) *wavefronts = w;
  if (workgroups_per_cu) *workgroups_per_cu = g;
  return DDIT_OK;
}

int ddit_linear_tile_choice(int epilogue, int64_t N, int32_t n, int32_t k, int32_t compute_units, int32_t *tile_out,
                            float *predicted_us_host) {
  if (epilogue < 0 || epilogue > 2) { set_error("unknown epilogue %d", epilogue); return DDIT_ERR_INVALID_ARG; }
  if (N < 0 || n < 1 || k < 1) { set_error("linear: N=%lld n=%d k=%d", (long long)N, n, k); return DDIT_ERR_INVALID_ARG; }
  if (!tile_out) { set_error("tile_out is NULL"); return DDIT_ERR_INVALID_ARG; }
  *tile_out = gemm_tile_choice(epilogue, N, n, k, compute_units, predicted_us_host);
  return DDIT_OK;
}

int ddit_linear_fwd(int epilogue, const void *u, int64_t ld_u, const void *W, const void *bias, int64_t N,
                    int32_t n, int32_t k, void *out, int64_t ld_out, float *resid, const float *ada_table,
                    const float *c6, int gate_row, int64_t tokens_per_sample, void *hip_stream) {
  return ddit_linear_fwd_tile(-1, epilogue, u, ld_u, W, bias, N, n, k, out, ld_out, resid, ada_table, c6, gate_row,
                              tokens_per_sample, hip_stream);
}

int ddit_linear_fwd_tile(int tile, int epilogue, const void *u, int64_t ld_u, const void *W, const void *bias,
                         int64_t N, int32_t n, int32_t k, void *out, int64_t ld_out, float *resid,
                         const float *ada_table, const float *c6, int gate_row, int64_t tokens_per_sample,
                         void *hip_stream) {
  if (tile >= gemm_tile_count()) { set_error("no tile %d (there are %d)", tile, gemm_tile_count()); return DDIT_ERR_INVALID_ARG; }
  if (epilogue < 0 || epilogue > 2) { set_error("unknown epilogue %d", epilogue); return DDIT_ERR_INVALID_ARG; }
  if (!u || !W) { set_error("u and W must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (N < 0 || n < 1 || k < 1 || ld_u < k) { set_error("linear: N=%lld n=%d k=%d ld_u=%lld", (long long)N, n, k, (long long)ld_u); return DDIT_ERR_INVALID_ARG; }
  if (n % 8 || k % 8 || ld_u % 8) { set_error("n, k and ld_u must be multiples of 8"); return DDIT_ERR_UNSUPPORTED; }
  if (!aligned16(u) || !aligned16(W) || (bias && !aligned16(bias)) || (out && !aligned16(out)) ||
      (resid && !aligned16(resid))) {
    set_error("pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  GemmArgs g;
  memset(&g, 0, sizeof(g)); g.tile = -1;
  g.u = u; g.ld_u = ld_u; g.W = W; g.bias = bias; g.N = N; g.n = n; g.k = k;
  g.tokens_per_sample = tokens_per_sample > 0 ? tokens_per_sample : 1;
  if (epilogue == DDIT_EPI_RESIDUAL_F32) {
    if (!resid) { set_error("resid must not be NULL for the residual epilogue"); return DDIT_ERR_INVALID_ARG; }
    g.resid = resid;
    if (gate_row >= 0) {
      if (gate_row > 5 || !ada_table || !c6) { set_error("gate_row=%d needs ada_table and c6, and must be < 6", gate_row); return DDIT_ERR_INVALID_ARG; }
      if (!aligned16(ada_table) || !aligned16(c6)) { set_error("ada_table and c6 must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
      g.gate_tab = ada_table + (int64_t)gate_row * n;
      g.gate_c6 = c6 + (int64_t)gate_row * n;
      g.gate_c6_stride = 6 * (int64_t)n;
    }
    if (out) { if (ld_out < n || ld_out % 8) { set_error("ld_out=%lld invalid", (long long)ld_out); return DDIT_ERR_INVALID_ARG; } }
  } else {
    if (!out) { set_error("out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
    if (ld_out < n || ld_out % 8) { set_error("ld_out=%lld invalid", (long long)ld_out); return DDIT_ERR_INVALID_ARG; }
  }
  g.out = out; g.ld_out = ld_out;
  g.tile = tile < 0 ? -1 : tile;
  return launch_gemm(epilogue, g, reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_io_workspace_bytes(const ddit_shape *shape, const ddit_io_weights *io, size_t *bytes_out) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (!bytes_out) { set_error("bytes_out is NULL"); return DDIT_ERR_INVALID_ARG; }
  IoLayout lo;
  make_io_layout(d, shape->flags, &lo);
  *bytes_out = lo.total;
  return DDIT_OK;
}

int ddit_embed_latent(const ddit_shape *shape, const ddit_io_weights *io, const float *z, void *x_out,
                      void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (!z || !x_out || !io->w_patch) { set_error("z, x_out and w_patch must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(z) || !aligned16(x_out) || !aligned16(io->w_patch)) {
    set_error("z, x_out and w_patch must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  IoLayout lo;
  make_io_layout(d, shape->flags, &lo);
  DDIT_TRY(check_ws(workspace, workspace_bytes, lo.total));
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  float *pos = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(workspace) + lo.pos);
  DDIT_TRY(launch_position_code(pos, shape->Hp, shape->Wp, shape->D, s));
  return launch_patch_embed(z, io->w_patch, io->b_patch, pos, x_out, shape->B, io->C_in, shape->T, shape->Hp,
                            shape->Wp, shape->D, s);
}

int ddit_embed_caption(const ddit_shape *shape, const ddit_io_weights *io, const void *c_text, void *y_out,
                       void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (!c_text || !y_out || !io->w_y1 || !io->w_y2) { set_error("c_text, y_out, w_y1 and w_y2 must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!aligned16(c_text) || !aligned16(y_out) || !aligned16(io->w_y1) || !aligned16(io->w_y2) ||
      (io->b_y1 && !aligned16(io->b_y1)) || (io->b_y2 && !aligned16(io->b_y2))) {
    set_error("caption embedder: pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT;
  }
  IoLayout lo;
  make_io_layout(d, shape->flags, &lo);
  DDIT_TRY(check_ws(workspace, workspace_bytes, lo.total));
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  void *tmp = reinterpret_cast<unsigned char *>(workspace) + lo.cap;
  GemmArgs g;
  memset(&g, 0, sizeof(g)); g.tile = -1;
  g.u = c_text; g.ld_u = io->C_text; g.W = io->w_y1; g.bias = io->b_y1; g.N = d.B * d.Ly; g.n = (int)d.D;
  g.k = io->C_text; g.out = tmp; g.ld_out = d.D; g.tokens_per_sample = d.Ly;
  DDIT_TRY(launch_gemm(DDIT_EPI_GELU_BF16, g, s));
  g.u = tmp; g.ld_u = d.D; g.W = io->w_y2; g.bias = io->b_y2; g.k = (int)d.D; g.out = y_out;
  return launch_gemm(DDIT_EPI_BF16, g, s);
}

int ddit_output_head(const ddit_shape *shape, const ddit_io_weights *io, const void *x, const float *temb,
                     float *eps_out, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (!x || !temb || !eps_out || !io->final_table || !io->w_final) {
    set_error("x, temb, eps_out, final_table and w_final must not be NULL"); return DDIT_ERR_INVALID_ARG;
  }
  if (!aligned16(x) || !aligned16(io->w_final)) { set_error("x and w_final must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  return launch_output_head(x, temb, io->final_table, io->w_final, io->b_final, eps_out, shape->B, io->C_out, shape->T,
                            shape->Hp, shape->Wp, shape->D, shape->ln_eps, reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_eps_theta(const ddit_shape *shape, const ddit_step_weights *weights, const ddit_io_weights *io,
                   const float *z, const void *y, const void *cross_kv_or_null, const int32_t *y_valid_len_host,
                   const float *timesteps_host, float *eps_out, void *workspace, size_t workspace_bytes,
                   void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (!weights || !timesteps_host || !eps_out) { set_error("weights, timesteps_host and eps_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  IoLayout lo;
  make_io_layout(d, shape->flags, &lo);
  DDIT_TRY(check_ws(workspace, workspace_bytes, lo.total));
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  void *x_tok = ws + lo.x_tok, *x_res = ws + lo.x_res;
  float *cond = reinterpret_cast<float *>(ws + lo.cond);
  float *c6_tmp = cond + d.B * (256 + 2 * d.D);
  const float *temb = cond + d.B * 256 + d.B * d.D;   // where the conditioning stage leaves the timestep embedding
  DDIT_TRY(ddit_embed_latent(shape, io, z, x_tok, workspace, workspace_bytes, hip_stream));
  DDIT_TRY(ddit_timestep_conditioning(shape, weights, timesteps_host, nullptr, c6_tmp, cond, hip_stream));
  DDIT_TRY(ddit_denoise_step_cached(shape, weights, x_tok, y, cross_kv_or_null, y_valid_len_host, nullptr, temb, x_res,
                                    workspace, workspace_bytes, hip_stream));
  return ddit_output_head(shape, io, x_res, temb, eps_out, hip_stream);
}

int ddit_solver_step(float *z, const float *eps_c, const float *eps_u_or_null, float guidance,
                     const float *t_host, const float *t_next_host, int32_t B, int64_t per_sample,
                     void *hip_stream) {
  if (!z || !eps_c || !t_host || !t_next_host) { set_error("z, eps_c, t_host and t_next_host must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (B < 1 || B > 64 || per_sample < 0) { set_error("solver step: B=%d per_sample=%lld", B, (long long)per_sample); return DDIT_ERR_INVALID_ARG; }
  float dt[64];
  for (int b = 0; b < B; ++b) dt[b] = (t_next_host[b] - t_host[b]) / 1000.0f;
  return launch_solver_step(z, eps_c, eps_u_or_null, guidance, dt, B, per_sample, reinterpret_cast<hipStream_t>(hip_stream));
}

int ddit_sample(const ddit_shape *shape, const ddit_step_weights *weights, const ddit_io_weights *io, float *z,
                const void *y, const int32_t *y_valid_len_host, const void *y_uncond_or_null,
                const void *cross_kv_or_null, const void *cross_kv_uncond_or_null, float guidance,
                int32_t n_steps, int32_t first_step, int32_t last_step, float *eps_scratch, void *workspace,
                size_t workspace_bytes, void *hip_stream) {
  Dims d;
  DDIT_TRY(check_shape(shape, &d));
  DDIT_TRY(check_io(shape, d, io));
  if (n_steps < 1 || first_step < 0 || last_step < first_step || last_step > n_steps) {
    set_error("sample: n_steps=%d first_step=%d last_step=%d", n_steps, first_step, last_step);
    return DDIT_ERR_INVALID_ARG;
  }
  if (!z || !eps_scratch) { set_error("z and eps_scratch must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (y_uncond_or_null && ((cross_kv_or_null != nullptr) != (cross_kv_uncond_or_null != nullptr))) {
    set_error("sample: with guidance give both cross-attention caches or none"); return DDIT_ERR_INVALID_ARG;
  }
  const int64_t per_sample = (int64_t)io->C_out * d.T * 4 * d.S;
  if (io->C_out != io->C_in) { set_error("sample: the prediction must have the latent's channels (C_out=%d, C_in=%d)", io->C_out, io->C_in); return DDIT_ERR_UNSUPPORTED; }
  float *eps_c = eps_scratch, *eps_u = eps_scratch + d.B * per_sample;
  for (int i = first_step; i < last_step; ++i) {
    float t[64], tn[64];
    for (int b = 0; b < d.B; ++b) {
      t[b] = 1000.0f * (1.0f - (float)i / (float)n_steps);
      tn[b] = 1000.0f * (1.0f - (float)(i + 1) / (float)n_steps);
    }
    DDIT_TRY(ddit_eps_theta(shape, weights, io, z, y, cross_kv_or_null, y_valid_len_host, t, eps_c, workspace,
                            workspace_bytes, hip_stream));
    if (y_uncond_or_null)
      DDIT_TRY(ddit_eps_theta(shape, weights, io, z, y_uncond_or_null, cross_kv_uncond_or_null, nullptr, t, eps_u,
                              workspace, workspace_bytes, hip_stream));
    DDIT_TRY(ddit_solver_step(z, eps_c, y_uncond_or_null ? eps_u : nullptr, guidance, t, tn, (int)d.B, per_sample, hip_stream));
  }
  return DDIT_OK;
}

}  // extern "C"
