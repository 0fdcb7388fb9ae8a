// Shared device/host helpers of libddit_hot (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define DDIT_WAVE 64

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] B[16x32].
//   A operand: lane l holds A[l%32][8*(l/32) .. 8*(l/32)+7]
//   B operand: lane l holds B[8*(l/32) .. +7][l%32]
//   D: lane l, register 4*g+e holds D[8*g + 4*(l/32) + e][l%32], g,e in 0..3
__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// host side ---------------------------------------------------------------
namespace ddit {
void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);
int device_cus();   // compute units of the current device (cached per process; 256 if there is no device)

// kernel launchers (each validates nothing: callers have validated shapes)
int launch_modulated_layernorm(const float *x, const float *ada_table, const float *c6, int which, int64_t N,
                               int64_t tokens_per_sample, int D, float eps, void *out, hipStream_t s);

struct GemmArgs {
  const void *u; int64_t ld_u;      // bf16 [N,k]
  const void *W;                    // bf16 [n,k]
  const void *bias;                 // bf16 [n] or null
  int64_t N; int n; int k;
  void *out; int64_t ld_out;        // bf16 [N,n] (may be null for RESIDUAL)
  float *resid;                     // fp32 [N,n] updated in place (RESIDUAL)
  const float *gate_tab;            // fp32 [n] table row or null
  const float *gate_c6;             // fp32, element (b, col) at gate_c6[b*gate_c6_stride + col], or null
  int64_t gate_c6_stride;
  int64_t tokens_per_sample;
  int tile;                         // index into the tile list, or negative: the launcher's own choice
};
int launch_gemm(int epilogue, const GemmArgs &a, hipStream_t s);
// G problems that share u (a.W, a.bias, a.out are ignored; a.n is one problem's out-features): 0 = launched,
// 1 = this shape cannot be grouped (nothing launched: launch them one by one), negative = error
int launch_gemm_grouped(const GemmArgs &a, int G, const void *const *W, const void *const *bias, void *const *out,
                        hipStream_t s);
int gemm_tile_count();
int gemm_tile_info(int tile, int *rows, int *cols, int *wavefronts, int *wg_per_cu);
// the tile the launcher would take (cus <= 0: the current device's CU count); us_per_tile, if not
// null, receives the model's time for each of the gemm_tile_count() tiles
int gemm_tile_choice(int epilogue, int64_t N, int n, int k, int cus, float *us_per_tile);

struct AttnArgs {
  const void *q, *k, *v; void *o; float *lse;
  int64_t ld_q, ld_kv, ld_o;       // token (row) strides in elements
  int n_groups;                     // independent sequences' groups (per head): spatial B*T, temporal B*S, cross B
  int g_inner;                      // group g -> (g / g_inner, g % g_inner)
  int64_t q_outer, q_inner;         // first query token of group = outer*(g/g_inner) + inner*(g%g_inner)
  int64_t kv_outer, kv_inner;
  int64_t q_tok_step, kv_tok_step;  // distance in tokens between consecutive sequence elements
  int Lq;                           // queries per group
  int Lk_max;                       // keys per group when kv_len is null
  int kv_len[64];                   // per OUTER index (batch) valid key count, used if use_kv_len
  int use_kv_len;
  int H, dh;
  const void *q_norm_g;             // bf16 [dh] or null: RMS-normalise every query with these scales as it is loaded
  float q_norm_eps;
};
int launch_flash_attn(const AttnArgs &a, hipStream_t s);
int temporal_attn_max_T();   // longest sequence the dedicated temporal kernel takes
// g_q/g_k (per-head RMS-norm scales, both or neither) and rope_table ([T, dh/2] (cos, sin)) may be null:
// when given, q and k are normalised / rotated inside the kernel on their way in
int launch_temporal_attn(const void *q, const void *k, const void *v, void *o, float *lse, int64_t ld_q,
                         int64_t ld_kv, int64_t ld_o, int B, int T, int S, int H, int dh, const void *g_q,
                         const void *g_k, float norm_eps, const float *rope_table, hipStream_t s);

// per-head RMS normalisation and rotary embedding, in place (qk_norm_rope.hip), of `slots` consecutive heads
// per token row starting at qk: the first q_slots of them take the scales g_q, the others g_k (q | k of a
// fused projection: slots = 2H, q_slots = H; one operand alone: slots = H, q_slots = H or 0).
// g_q/g_k null: no normalisation; rope_table null: no rotation
int launch_rope_table(float *table, int T, int dh, hipStream_t s);   // [T, dh/2] (cos, sin)
int launch_qk_norm_rope(void *qk, int64_t ld, int64_t N, int slots, int q_slots, int dh, const void *g_q,
                        const void *g_k, float eps, const float *rope_table, int64_t S, int T, hipStream_t s);

int launch_cast_bf16_to_f32(const void *in, float *out, int64_t n, hipStream_t s);
int launch_cast_f32_to_bf16(const float *in, void *out, int64_t n, hipStream_t s);
struct CondArgs {
  int B, D;
  float t[64];
};
int launch_timestep_conditioning(const CondArgs &c, const void *w_t1, const void *b_t1, const void *w_t2,
                                 const void *b_t2, const void *w_ada, const void *b_ada, const float *temb_in,
                                 float *c6_out, float *scratch, hipStream_t s);

// layers around the token-space step, solver
int launch_position_code(float *pos, int Hp, int Wp, int D, hipStream_t s);
int launch_patch_embed(const float *z, const void *W, const void *bias, const float *pos, void *x, int B, int C,
                       int T, int Hp, int Wp, int D, hipStream_t s);
int launch_output_head(const void *x, const float *temb, const float *table, const void *W, const void *bias,
                       float *out, int B, int C_out, int T, int Hp, int Wp, int D, float eps, hipStream_t s);
int launch_solver_step(float *z, const float *ec, const float *eu, float guidance, const float *dt, int B,
                       int64_t per_sample, hipStream_t s);
}  // namespace ddit
