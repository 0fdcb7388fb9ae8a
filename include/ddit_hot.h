/*
 * libddit_hot - the DiT denoising step eps_theta(x_t, t, c) of a text-to-video
 * diffusion transformer (paper eq. 1), as hand-written HIP kernels for gfx950.
 *
 * The model is the spatial-temporal DiT of the paper's section 2.2: three kinds of
 * Transformer blocks, "spatial" (tokens sharing a temporal index attend to each
 * other), "temporal" (tokens sharing a spatial location attend across time) and
 * "cross-attention" (every token attends to the text condition).  Table 1 names it
 * (STDiT-v3, 1.1 B parameters).  One *layer* here is
 *     x += gate_msa * Wo . SelfAttn(QKV(modulate(LN(x), shift_msa, scale_msa)))
 *     x +=            Wco . CrossAttn(Wcq x, Wckv y, valid_len)
 *     x += gate_mlp * W2 . GELU_tanh(W1 modulate(LN(x), shift_mlp, scale_mlp))
 * with SelfAttn spatial or temporal; one *block* is a spatial layer followed by a
 * temporal layer; a denoising step is the timestep conditioning followed by
 * n_blocks blocks.  (shift, scale, gate) x (msa, mlp) are the six D-vectors of
 * table_l[6,D] + c6[b], c6 = W_ada SiLU(temb) + b_ada (adaLN-single).
 *
 * Conventions for every entry point
 *  - Token order: x[B,T,S,D], token n = (b*T + t)*S + s, S = Hp*Wp.  Text y[B,Ly,D].
 *  - All data pointers are DEVICE pointers unless the name ends in _host.
 *    Activations and weights are bf16 (the upper 16 bits of an IEEE fp32), row
 *    major; a Linear's weight is [out,in] and computes u W^T + b.  The adaLN table,
 *    c6 and lse are fp32.  Every device pointer must be 16-byte aligned and every
 *    leading dimension a multiple of 8 elements.
 *  - Ownership: the caller owns every buffer including the workspace; the library
 *    allocates and frees no device memory.  Between calls it keeps no data of a call; what it does keep
 *    per process is set once and never changes results: the compute-unit count of the device, a
 *    "dynamic LDS size attribute set" flag per kernel, and the address of the built-in scratch of
 *    ddit_stdit_block_fwd_static per device.
 *    Buffers must stay alive until `hip_stream` has run past the call.
 *  - Asynchrony: all work is enqueued on `hip_stream` (a hipStream_t, NULL = the
 *    default stream); no call synchronises with the host.  *_host arrays are read
 *    before the call returns.
 *  - Errors: the return value is DDIT_OK (0) or a negative ddit_status.  Arguments
 *    are validated before anything is enqueued; on error nothing has been launched
 *    (except DDIT_ERR_HIP, raised by a failing launch).  ddit_last_error() gives a
 *    thread-local description.  Nothing throws or aborts across this boundary.
 *  - Sizes: a ddit_shape has every dimension >= 1.  The single-stage calls that take a
 *    token count N of their own (ddit_linear_fwd*, ddit_modulated_layernorm_fwd,
 *    ddit_qk_norm_rope_fwd) accept N = 0: arguments are validated, nothing is enqueued,
 *    DDIT_OK is returned.
 *  - Arithmetic: bf16 storage, fp32 accumulation; the residual stream is fp32
 *    inside ddit_stdit_block_fwd and ddit_denoise_step and is rounded to bf16 once,
 *    at the output.
 */
#ifndef DDIT_HOT_H
#define DDIT_HOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DDIT_ABI_VERSION 7u

typedef enum {
  DDIT_OK = 0,
  DDIT_ERR_INVALID_ARG = -1, /* NULL required pointer, non-positive size, valid_len outside [1,Ly] */
  DDIT_ERR_UNSUPPORTED = -2, /* a shape the kernels do not cover (message names the field) */
  DDIT_ERR_WORKSPACE = -3,   /* workspace NULL or smaller than ddit_workspace_bytes() */
  DDIT_ERR_ALIGNMENT = -4,   /* pointer not 16-byte aligned / leading dimension not a multiple of 8 */
  DDIT_ERR_HIP = -5          /* a HIP launch failed; message carries hipGetErrorString() */
} ddit_status;

typedef enum { DDIT_ATTN_SPATIAL = 0, DDIT_ATTN_TEMPORAL = 1, DDIT_ATTN_CROSS = 2 } ddit_attn_kind;

/* flags of ddit_shape */
#define DDIT_FLAG_TAPS 1u /* block/step: keep per-branch intermediates of the LAST layer pair run
                             (see ddit_tap_region) in the tail of the workspace, for tests */
/* Two options of the self-attention that the paper's section 2.2 does not mention and the
 * released model of its Table 1 has; both off by default.  They act on q and k between the
 * q|k|v projection and the attention, in fp32, with one rounding to bf16: */
#define DDIT_FLAG_QK_NORM 2u /* per-head RMS normalisation of the spatial and temporal self-attention's
                                q and k:  u / sqrt(mean_d(u^2) + ln_eps) * g  over the dh elements of a
                                head, g = the layer's g_q (queries) or g_k (keys).  Cross-attention is
                                not normalised. */
#define DDIT_FLAG_ROPE_TEMPORAL 4u /* rotary position embedding of the TEMPORAL self-attention's q and k
                                (after the normalisation): the pair (u[2i], u[2i+1]) of every head is
                                rotated by the angle t * 10000^(-2i/dh), t = the token's frame index */

/* Problem shape.  Supported: dh in {64, 72}; D, A = H*dh, M, multiples of 8; A <= D
 * (A < D is one rank's share of a head-split sequence-parallel run); B <= 64. */
typedef struct {
  uint32_t struct_size; /* sizeof(ddit_shape): versions the struct */
  uint32_t flags;
  int32_t B, T, Hp, Wp;              /* S = Hp*Wp tokens per frame, L = T*S per sample */
  int32_t D, H, dh, M, Ly, n_blocks; /* hidden, heads, head dim, MLP width, text tokens, blocks */
  float ln_eps;                      /* LayerNorm epsilon (1e-6) */
} ddit_shape;

/* One layer's parameters.  bf16 [out,in] weights; a bias may be NULL (= zero).
 * w_qkv rows are ordered q (all heads) | k | v, head h owning rows h*dh..(h+1)*dh-1 of
 * each group; w_ckv rows are k | v.  ada_table is fp32 [6,D] in the order shift_msa,
 * scale_msa, gate_msa, shift_mlp, scale_mlp, gate_mlp. */
typedef struct {
  const void *w_qkv, *b_qkv; /* [3A,D], [3A] */
  const void *w_o, *b_o;     /* [D,A],  [D]  */
  const void *w_cq, *b_cq;   /* [A,D],  [A]  */
  const void *w_ckv, *b_ckv; /* [2A,D], [2A] */
  const void *w_co, *b_co;   /* [D,A],  [D]  */
  const void *w_fc1, *b_fc1; /* [M,D],  [M]  */
  const void *w_fc2, *b_fc2; /* [D,M],  [D]  */
  const float *ada_table;    /* [6,D] fp32 */
  const void *g_q, *g_k;     /* [dh] bf16 each; read only with DDIT_FLAG_QK_NORM (else may be NULL) */
} ddit_layer_weights;

typedef struct {
  ddit_layer_weights spatial, temporal;
} ddit_block_weights;

/* Timestep conditioning: e = [cos(t f_i), sin(t f_i)], f_i = 10000^(-i/128), i < 128;
 * temb = W_t2 SiLU(W_t1 e + b_t1) + b_t2;  c6 = W_ada SiLU(temb) + b_ada. */
typedef struct {
  const void *w_t1, *b_t1;          /* [D,256], [D] */
  const void *w_t2, *b_t2;          /* [D,D],   [D] */
  const void *w_ada, *b_ada;        /* [6D,D],  [6D] */
  const ddit_block_weights *blocks; /* HOST array of n_blocks entries (holding device pointers) */
} ddit_step_weights;

uint32_t ddit_abi_version(void);
const char *ddit_status_string(int status);
const char *ddit_last_error(void); /* thread-local, never NULL */

/* Bytes of workspace ddit_stdit_block_fwd / ddit_denoise_step / ddit_attn_fwd need for
 * this shape (with DDIT_FLAG_TAPS: including the tap area). */
int ddit_workspace_bytes(const ddit_shape *shape, size_t *bytes_out);

/* Where a tap lives, when DDIT_FLAG_TAPS is set: offset from the start of the workspace
 * and size in bytes.  layer: 0 = spatial layer, 1 = temporal layer of the last block run.
 * tap ids: */
typedef enum {
  DDIT_TAP_XH_MSA = 0,      /* bf16 [N,D]  modulate(LN(x)) feeding QKV            */
  DDIT_TAP_QKV = 1,         /* bf16 [N,3A] q | k | v as the attention reads them   */
  DDIT_TAP_O = 2,           /* bf16 [N,A]  self-attention output                   */
  DDIT_TAP_X_AFTER_ATTN = 3,  /* fp32 [N,D] stream after the gated attention add   */
  DDIT_TAP_QC = 4,          /* bf16 [N,A]  cross-attention queries                 */
  DDIT_TAP_KVC = 5,         /* bf16 [B*Ly,2A] cross-attention k | v                */
  DDIT_TAP_OC = 6,          /* bf16 [N,A]  cross-attention output                  */
  DDIT_TAP_X_AFTER_CROSS = 7, /* fp32 [N,D]                                        */
  DDIT_TAP_XH_MLP = 8,      /* bf16 [N,D]                                          */
  DDIT_TAP_H = 9,           /* bf16 [N,M]  GELU(fc1)                               */
  DDIT_TAP_X_OUT = 10,      /* fp32 [N,D]  stream after the layer                  */
  DDIT_TAP_COUNT = 11
} ddit_tap_id;
int ddit_tap_region(const ddit_shape *shape, int layer, int tap, size_t *offset_out, size_t *bytes_out);

/* Exact softmax attention, O = softmax(Q K^T / sqrt(dh)) V (section 2.2: which tokens
 * attend to which is fixed by `kind`).
 *   SPATIAL : q,k,v,o are [B,T,S,H,dh]; for each (b,t,h) the S tokens of frame t.
 *   TEMPORAL: same tensors; for each (b,s,h) the T tokens at location s.
 *   CROSS   : q,o [B,L,H,dh], k,v [B,Ly,H,dh]; keys j >= kv_valid_len_host[b] take no part.
 * ld_* are the row (token) strides in elements, >= H*dh: q, k and v may be column
 * slices of one fused projection buffer.  kv_valid_len_host: HOST int32[B] or NULL
 * (= Ly), CROSS only, each in [1,Ly].  lse_or_null: optional fp32 [tokens,H] receiving
 * log(sum_j exp(score_ij)) of the scaled scores.  Uses no workspace today; the
 * arguments are reserved (may be NULL/0). */
int ddit_attn_fwd(ddit_attn_kind kind, const ddit_shape *shape, const void *q, const void *k, const void *v,
                  int64_t ld_q, int64_t ld_kv, const int32_t *kv_valid_len_host, void *o, int64_t ld_o,
                  float *lse_or_null, void *workspace, size_t workspace_bytes, void *hip_stream);

/* One block of the model of section 2.2 (a "spatial" Transformer layer, which mixes the tokens of one temporal
 * index, followed by a "temporal" one, which mixes the tokens of one spatial location; each with its
 * "cross-attention" to the conditioning text): spatial layer then temporal layer on x_in bf16 [B,T,S,D] with text y bf16
 * [B,Ly,D], valid lengths (HOST int32[B] or NULL = Ly) and conditioning c6 (device fp32
 * [B,6D]).  x_out bf16 [B,T,S,D] may alias x_in.  shape->n_blocks is ignored. */
int ddit_stdit_block_fwd(const ddit_shape *shape, const ddit_block_weights *weights, const void *x_in,
                         const void *y, const int32_t *y_valid_len_host, const float *c6, void *x_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* ddit_stdit_block_fwd for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * block's workspace is a device array built into the library, DDIT_STATIC_SCRATCH_BYTES per GPU,
 * held from the library's load until the process ends.  The call allocates and frees nothing.
 * Same arguments and results as ddit_stdit_block_fwd, less the workspace.  Shapes whose
 * ddit_workspace_bytes() exceeds DDIT_STATIC_SCRATCH_BYTES are refused with DDIT_ERR_WORKSPACE
 * (64 MiB holds a block of the 144p latent: T=16, 9x16 tokens per frame, hidden 1152);
 * DDIT_FLAG_TAPS is refused with DDIT_ERR_UNSUPPORTED.  Every call on one GPU uses that GPU's one
 * array: calls that overlap in time on the same GPU (different streams or threads) race on it;
 * calls on one stream, or ordered by the caller, are safe.  The array keeps the previous call's
 * contents; no region of it has to start at zero. */
#define DDIT_STATIC_SCRATCH_BYTES (64u << 20)
int ddit_stdit_block_fwd_static(const ddit_shape *shape, const ddit_block_weights *weights, const void *x_in,
                                const void *y, const int32_t *y_valid_len_host, const float *c6, void *x_out,
                                void *hip_stream);

/* One evaluation of eps_theta(x_t, t, c) of eq. 1 in token space (x_t = x_in, t = timesteps_host, c = y; the
 * model of section 2.2 and Table 1): conditioning from timesteps_host (HOST fp32[B]),
 * then shape->n_blocks blocks with an fp32 residual stream, rounded to bf16 at x_out.
 * If temb_or_null (device fp32 [B,D]) is given it replaces the timestep embedder's
 * output (timesteps_host may then be NULL). */
int ddit_denoise_step(const ddit_shape *shape, const ddit_step_weights *weights, const void *x_in,
                      const void *y, const int32_t *y_valid_len_host, const float *timesteps_host,
                      const float *temb_or_null, void *x_out, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/* The text condition is constant over a request's steps (section 2.1: every step is called with
 * the same c), so the cross-attention keys and values of every layer, k|v = y W_ckv^T + b_ckv,
 * can be formed once per request instead of once per step.
 * ddit_cross_kv_bytes: size of that cache, bf16 [2*n_blocks, B*Ly, 2A] in layer order (block 0
 * spatial, block 0 temporal, block 1 spatial, ...).  ddit_cross_kv_precompute fills it.
 * ddit_denoise_step_cached is ddit_denoise_step reading the cache instead of projecting y
 * (y is then unused and may be NULL; cross_kv NULL = project y as usual). */
int ddit_cross_kv_bytes(const ddit_shape *shape, size_t *bytes_out);
int ddit_cross_kv_precompute(const ddit_shape *shape, const ddit_step_weights *weights, const void *y,
                             void *cross_kv_out, void *hip_stream);
int ddit_denoise_step_cached(const ddit_shape *shape, const ddit_step_weights *weights, const void *x_in,
                             const void *y, const void *cross_kv_or_null, const int32_t *y_valid_len_host,
                             const float *timesteps_host, const float *temb_or_null, void *x_out,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- single stages of the path, exported for kernel-level parity tests and profiling ---- */

/* out[n,:] = bf16( LN(x[n,:]) * (1 + scale_b) + shift_b ), LN without affine over D with
 * biased variance; (shift_b, scale_b) = rows (3*which, 3*which+1) of ada_table + c6[b],
 * which = 0 (msa) or 1 (mlp), b = n / tokens_per_sample.  x fp32 [N,D], out bf16 [N,D]. */
int ddit_modulated_layernorm_fwd(const float *x, const float *ada_table, const float *c6, int which,
                                 int64_t N, int64_t tokens_per_sample, int32_t D, float eps, void *out,
                                 void *hip_stream);

typedef enum {
  DDIT_EPI_BF16 = 0,          /* out bf16 [N,n] = u W^T + b                                        */
  DDIT_EPI_GELU_BF16 = 1,     /* out bf16 = GELU_tanh(u W^T + b)                                    */
  DDIT_EPI_RESIDUAL_F32 = 2   /* resid fp32 [N,n] += gate_b * (u W^T + b); gate_b = row gate_row of
                                 ada_table + c6[b] (gate_row < 0: no gate); if out != NULL it also
                                 receives bf16(resid)                                               */
} ddit_epilogue;

/* u bf16 [N,k] (row stride ld_u), W bf16 [n,k], bias bf16 [n] or NULL. */
int ddit_linear_fwd(int epilogue, const void *u, int64_t ld_u, const void *W, const void *bias, int64_t N,
                    int32_t n, int32_t k, void *out, int64_t ld_out, float *resid, const float *ada_table,
                    const float *c6, int gate_row, int64_t tokens_per_sample, void *hip_stream);

/* In place on q | k, the first 2*H*dh columns of the rows of qk (bf16, row stride ld elements,
 * N rows): per-head RMS normalisation with scales g_q, g_k (bf16 [dh]; both NULL = none) and,
 * if rope_table_or_null is given, rotary embedding with frame index t = (row / S) % T
 * (DDIT_FLAG_QK_NORM / DDIT_FLAG_ROPE_TEMPORAL above).  rope_table_or_null: device scratch of
 * T*dh floats that the call fills with the (cos, sin) table first; NULL = no rotation. */
int ddit_qk_norm_rope_fwd(void *qk, int64_t ld, int64_t N, int32_t H, int32_t dh, const void *g_q,
                          const void *g_k, float eps, int64_t S, int32_t T, float *rope_table_or_null,
                          void *hip_stream);

/* Spatial or temporal self-attention with those two options applied to q and k on the way (what a
 * layer does between its q|k|v projection and its out-projection): per-head RMS normalisation iff
 * g_q and g_k (bf16 [dh]) are given, with shape->ln_eps; rotation by the frame index iff kind is
 * TEMPORAL and rope_table_or_null is given (device scratch of T*dh floats, filled by the call).
 * fuse != 0 folds the treatment into the attention kernels where that is possible (temporal with
 * T <= 32: wholly; spatial: the queries, while the keys are treated in place first); fuse == 0 treats
 * q and k in place first and then runs the plain attention.  Either way q and k may be overwritten
 * with their treated values; v is only read.  Tensors and strides as in ddit_attn_fwd. */
int ddit_self_attn_fwd(ddit_attn_kind kind, const ddit_shape *shape, void *q, void *k, const void *v, int64_t ld_q,
                       int64_t ld_kv, const void *g_q, const void *g_k, float *rope_table_or_null, int fuse, void *o,
                       int64_t ld_o, float *lse_or_null, void *hip_stream);

/* ---- output tiles of the linear: for tuning and for parity tests of every compiled tile ----
 * The linear is compiled for a short list of output tiles (rows x cols of out per workgroup) and
 * ddit_linear_fwd takes, per call, the one that a cost model of the kernel prices cheapest for
 * (epilogue, N, n, k) on the current device.  None of the three calls below is on the hot path. */

/* Number of compiled tiles; tile indices are 0 .. count-1. */
int ddit_linear_tile_count(void);

/* Geometry of one tile: out rows and columns per workgroup, wavefronts per workgroup, and how
 * many workgroups the launcher keeps resident per CU (a tile shape may be listed twice, once per
 * depth of its operand pipeline: the shallower form lets one more workgroup share the CU).
 * The list is ordered by tile area, largest first.  Any pointer may be NULL.
 * DDIT_ERR_INVALID_ARG if tile is out of range.  Host only; needs no GPU. */
int ddit_linear_tile_info(int tile, int32_t *rows, int32_t *cols, int32_t *wavefronts,
                          int32_t *workgroups_per_cu);

/* The tile ddit_linear_fwd would take for this problem on a device of compute_units CUs
 * (compute_units <= 0: the current device's count, 256 if there is no device) -> *tile_out.
 * predicted_us_host, if not NULL, is a HOST array of ddit_linear_tile_count() floats that
 * receives the model's time for every tile, in microseconds.  Host only; needs no GPU. */
int ddit_linear_tile_choice(int epilogue, int64_t N, int32_t n, int32_t k, int32_t compute_units,
                            int32_t *tile_out, float *predicted_us_host);

/* ddit_linear_fwd with the tile fixed (tile < 0: the model's choice, i.e. ddit_linear_fwd itself).
 * Every tile computes the same function for every valid shape; only the time differs. */
int ddit_linear_fwd_tile(int tile, int epilogue, const void *u, int64_t ld_u, const void *W, const void *bias,
                         int64_t N, int32_t n, int32_t k, void *out, int64_t ld_out, float *resid,
                         const float *ada_table, const float *c6, int gate_row, int64_t tokens_per_sample,
                         void *hip_stream);

/* c6 fp32 [B,6D] from timesteps (HOST fp32[B]) or from a given temb (device fp32 [B,D]).
 * scratch: device fp32, at least B*(256 + 2*D) floats. */
int ddit_timestep_conditioning(const ddit_shape *shape, const ddit_step_weights *weights,
                               const float *timesteps_host, const float *temb_or_null, float *c6_out,
                               float *scratch, void *hip_stream);

/* ---- measurement probes: the denominators the kernels are held against, reproducible on any box ----
 * None is on the hot path; the benchmark times them beside the step.
 * ddit_probe_mfma_bf16: a register-resident loop of the bf16 matrix-core instruction the linears and the
 *   attention use, 2 workgroups of 4 wavefronts per compute unit, 12 independent accumulators each, `iters`
 *   rounds; `operands` = 64 KiB of bf16 the fragments are taken from (the sustained clock depends on the data:
 *   constant data runs faster than random data), `sink` = device fp32, 512 floats per compute unit;
 *   *flop_out (HOST, optional) receives the floating-point operations of the launch.
 * ddit_probe_stream_copy: out[0..bytes) = in[0..bytes) with streaming 16-byte loads and stores.
 * ddit_probe_stream_read: reads in[0..bytes) with streaming 16-byte loads; sink: device fp32, 4096 floats per compute unit.
 * ddit_probe_residual_stream: the memory traffic of an out-projection with gated residual update and none of
 *   its matrix work: per token row reads A bf16 of o and D fp32 of x, writes D fp32 of x and D bf16 of xh_out
 *   (x += gate * f(o) with a cheap f; the result has no meaning).  gate: device fp32 [D]. */
int ddit_probe_mfma_bf16(const void *operands, float *sink, int32_t iters, double *flop_out, void *hip_stream);
int ddit_probe_stream_copy(const void *in, void *out, int64_t bytes, void *hip_stream);
int ddit_probe_stream_read(const void *in, int64_t bytes, float *sink, void *hip_stream);
int ddit_probe_residual_stream(float *x, void *xh_out, const void *o, const float *gate, int64_t N, int32_t D,
                               int32_t A, void *hip_stream);

/* ---- latent in, latent out, and the sampling loop of eq. 1 -------------------------------
 *
 * Section 2.1 states the reverse process: from Gaussian noise x_T, each step calls the model on
 * (x_t, t, c) and a solver Phi turns its prediction into x_{t-1}; section 2.2 places the DiT
 * between the text encoder and the VAE, working on a latent video.  The paper gives neither the
 * embedding of the latent into tokens, nor the output head, nor Phi; the forms below are this
 * library's reading of the public spatial-temporal DiT design:
 *   latent z fp32 [B, C, T, 2Hp, 2Wp]; token (b,t,i,j), s = i*Wp + j, is the 1x2x2 patch
 *   z[b, :, t, 2i:2i+2, 2j:2j+2] flattened as (c, di, dj), embedded by Linear(4C -> D), plus a
 *   fixed 2-D sine/cosine position code (quarters of D: sin(j w_m), cos(j w_m), sin(i w_m),
 *   cos(i w_m), w_m = 10000^(-m/(D/4)));
 *   text c bf16 [B, Ly, C_text] -> y = W_y2 GELU_tanh(W_y1 c + b_y1) + b_y2;
 *   head: LN(x) (1 + scale_b) + shift_b with (shift_b, scale_b) = final_table[2,D] + temb_b,
 *   then Linear(D -> 4 C_out) ordered (di, dj, c), scattered back to [B, C_out, T, 2Hp, 2Wp];
 *   Phi: z += (t_next - t) / 1000 * eps, eps = eps_u + guidance (eps_c - eps_u) when an
 *   unconditional text input is given, else eps_c; a run of n steps visits t_i = 1000 (1 - i/n).
 * Latents and predictions are fp32 (a latent is a few MB); D must be a multiple of 8 and of 4,
 * 4 C_in <= 64, 4 C_out <= 64, C_text a multiple of 8. */
typedef struct {
  uint32_t struct_size;          /* sizeof(ddit_io_weights) */
  int32_t C_in, C_out, C_text;
  const void *w_patch, *b_patch; /* bf16 [D, 4 C_in], [D]   */
  const void *w_y1, *b_y1;       /* bf16 [D, C_text], [D]   */
  const void *w_y2, *b_y2;       /* bf16 [D, D], [D]        */
  const float *final_table;      /* fp32 [2, D]: shift, scale */
  const void *w_final, *b_final; /* bf16 [4 C_out, D], [4 C_out] */
} ddit_io_weights;

/* Bytes of workspace for ddit_embed_latent / ddit_embed_caption / ddit_eps_theta / ddit_sample
 * (it contains ddit_workspace_bytes(shape)). */
int ddit_io_workspace_bytes(const ddit_shape *shape, const ddit_io_weights *io, size_t *bytes_out);

/* x_out bf16 [B,T,S,D] = patch embedding of z + position code. */
int ddit_embed_latent(const ddit_shape *shape, const ddit_io_weights *io, const float *z, void *x_out,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* y_out bf16 [B,Ly,D] from the text encoder's output c_text bf16 [B,Ly,C_text]. */
int ddit_embed_caption(const ddit_shape *shape, const ddit_io_weights *io, const void *c_text, void *y_out,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* eps_out fp32 [B,C_out,T,2Hp,2Wp] from tokens x bf16 [B,T,S,D] and temb (device fp32 [B,D]). */
int ddit_output_head(const ddit_shape *shape, const ddit_io_weights *io, const void *x, const float *temb,
                     float *eps_out, void *hip_stream);

/* The whole model on a latent: embed z, run ddit_denoise_step at timesteps_host (HOST fp32 [B])
 * with the embedded text y bf16 [B,Ly,D] (valid lengths HOST int32[B] or NULL), apply the head.
 * cross_kv_or_null: a cache from ddit_cross_kv_precompute for this y (then y may be NULL). */
int ddit_eps_theta(const ddit_shape *shape, const ddit_step_weights *weights, const ddit_io_weights *io,
                   const float *z, const void *y, const void *cross_kv_or_null, const int32_t *y_valid_len_host,
                   const float *timesteps_host, float *eps_out, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/* z[b] += (t_next_host[b] - t_host[b]) / 1000 * (eps_u + guidance (eps_c - eps_u)); eps_u may be
 * NULL (then eps = eps_c).  z, eps_* fp32 with `per_sample` elements per sample, B samples. */
int ddit_solver_step(float *z, const float *eps_c, const float *eps_u_or_null, float guidance,
                     const float *t_host, const float *t_next_host, int32_t B, int64_t per_sample,
                     void *hip_stream);

/* Steps first_step .. last_step-1 of an n_steps run, in place on z.  A caller that schedules at
 * step granularity (the paper's sections 4.2-4.3 change a request's resources between steps)
 * calls this with one step, or a few, at a time; nothing is kept between calls but z.
 * y_uncond_or_null bf16 [B,Ly,D]: unconditional text input for guidance (its valid length is Ly).
 * cross_kv_or_null / cross_kv_uncond_or_null: caches from ddit_cross_kv_precompute for y and
 * y_uncond (kept by the caller across calls); with guidance either both or none are given.
 * eps_scratch: device fp32, 2 * B * C_out * T * 2Hp * 2Wp floats. */
int ddit_sample(const ddit_shape *shape, const ddit_step_weights *weights, const ddit_io_weights *io, float *z,
                const void *y, const int32_t *y_valid_len_host, const void *y_uncond_or_null,
                const void *cross_kv_or_null, const void *cross_kv_uncond_or_null, float guidance,
                int32_t n_steps, int32_t first_step, int32_t last_step, float *eps_scratch, void *workspace,
                size_t workspace_bytes, void *hip_stream);

/* ---- what the paper builds on top of the step: choosing and changing a request's GPUs ----
 * Host only (no GPU, no HIP call, host pointers throughout): the optimal degree of parallelism
 * from a table of measured step times (section 4.2.3), a buddy allocator of GPUs (section 5) and
 * the greedy step-granular scheduler (section 4.2.3 and the scheduling algorithm of the appendix)
 * run as an event simulation over such a table.  All times are integer microseconds, so results
 * are exact.  bench.py --dop-table measures the table for this library on one MI355X. */

/* B for one resolution: step_us_row_host[k] = time of one step on 2^k GPUs, k < n_dop.
 * z(2^k) = 1 - t_k / t_{k-1} (the paper's change rate); B = the parallel size with the largest z
 * (the smaller size on ties), or 1 if no z exceeds z_min = z_min_num / z_min_den (the paper
 * reports B = 1 for its lowest resolution; with 0/1 that is "no doubling gains anything").
 * Exact integer comparisons.  Step times in [1, 2^40]. */
int ddit_optimal_dop(const int64_t *step_us_row_host, int32_t n_dop, int64_t z_min_num, int64_t z_min_den,
                     int32_t *dop_out);

/* Buddy system over GPUs 0 .. n_gpus-1 (a power of two, at most 4096): blocks are aligned runs of
 * 2^k GPUs.  alloc takes the SMALLEST free block that is large enough, the lowest-numbered of
 * that size, and splits it keeping the lower half each time; *start_out = -1 when nothing fits
 * (that is not an error).  release merges a block with its buddy as long as the buddy is free;
 * it refuses a range that is not an aligned block or not allocated as a whole.  The pool is host
 * memory owned by the library between create and destroy; calls on one pool must not overlap. */
int ddit_buddy_create(int32_t n_gpus, void **pool_out);
int ddit_buddy_alloc(void *pool, int32_t size, int32_t *start_out);
int ddit_buddy_release(void *pool, int32_t start, int32_t size);
int ddit_buddy_free_gpus(void *pool, int32_t *free_out);
int ddit_buddy_destroy(void *pool);

typedef struct {
  uint32_t struct_size;   /* sizeof(ddit_sched_config) */
  int32_t n_gpus;         /* power of two, at most 4096 */
  int32_t n_steps;        /* denoising steps per request (30 in the paper's evaluation) */
  int32_t n_resolutions;  /* R */
  int32_t n_dop;          /* parallel sizes in the table: 1, 2, ..., 2^(n_dop-1) <= n_gpus */
  int32_t vae_gpus;       /* GPUs a request keeps for the decoder (power of two) */
  const int64_t *step_us; /* HOST [R, n_dop]: DiT_step_time(parallel size, resolution), each in [1, 2^40] */
  const int32_t *opt_dop; /* HOST [R]: B(r), a power of two inside the table */
  const int64_t *vae_us;  /* HOST [R] or NULL: time of the decoder phase; 0 = none */
} ddit_sched_config;

typedef struct { int64_t arrival_us; int32_t resolution; int32_t reserved; } ddit_sched_request;

typedef struct {
  int64_t start_us, dit_end_us, end_us; /* first step starts / last step ends / GPUs all given back */
  int64_t starvation;                   /* the priority value when last brought up to date */
  int32_t first_dop, final_dop;         /* GPUs at the start / during the last step */
  int32_t promotions, reserved;         /* scheduling passes that gave the request more GPUs */
} ddit_sched_record;

typedef enum { DDIT_SCHED_START = 0, DDIT_SCHED_PROMOTE = 1, DDIT_SCHED_DIT_DONE = 2, DDIT_SCHED_RELEASE = 3 } ddit_sched_event_kind;
typedef struct { int64_t time_us; int32_t kind, request, gpu_start, gpu_count; } ddit_sched_event;
typedef struct { int64_t occupancy_gpu_us, makespan_us; } ddit_sched_totals;

/* Serves requests_host[0 .. n_requests-1] (ordered by arrival, at most 2^22 of them) and reports what happened.
 * Host memory that runs out is reported as DDIT_ERR_UNSUPPORTED ("out of host memory"), never thrown.
 * Rules (the first four are the paper's, the rest are this library's readings of what it leaves open):
 *  - first come, first served; a waiting request asks for B(r) GPUs and goes down (B, B/2, .., 1)
 *    until the allocator has a block; below B it is "hungry";
 *  - whenever GPUs were released, every hungry request's starvation grows by
 *    (steps done since its last update) x (its step time now - its step time at B), and hungry
 *    requests are promoted in descending order of starvation, before the waiting queue is served;
 *  - a promotion takes effect between two denoising steps: the step in flight ends at the old
 *    rate, later steps run at the new one; the new GPUs count as occupied from the grant;
 *  - after the last step the request keeps the vae_gpus lowest-numbered GPUs of its
 *    lowest-numbered block (at most that block) for vae_us[r], and gives back the rest at once;
 *  - a promotion from p to 2p GPUs takes ANY free block of p GPUs from the allocator, and repeats
 *    until B or until none is free; a request thus holds a list of blocks;
 *  - within one microsecond: step ends and decoder ends (by request index), then arrivals, then one
 *    scheduling pass; equal starvation goes to the earlier request;
 *  - blocks are given back in the order they were granted (the decoder's block: upper halves first).
 * records_out: n_requests entries.  events_out_or_null: up to max_events entries are written in
 * the order they happen (START / PROMOTE / RELEASE carry one block each; DIT_DONE carries the
 * request's lowest GPU and its parallel size); *n_events_out is the number that occurred, which
 * may exceed max_events.  totals: sum over GPUs of occupied time, and the time of the last event. */
int ddit_sched_simulate(const ddit_sched_config *config, const ddit_sched_request *requests_host, int32_t n_requests,
                        ddit_sched_record *records_out, ddit_sched_event *events_out_or_null, int64_t max_events,
                        int64_t *n_events_out, ddit_sched_totals *totals_out);

#ifdef __cplusplus
}
#endif
#endif /* DDIT_HOT_H */
