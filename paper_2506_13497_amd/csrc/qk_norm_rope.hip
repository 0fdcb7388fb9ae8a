// Optional treatment of the self-attention queries and keys between the q|k|v projection and
// the attention kernel (the paper's section 2.2 does not write the block down; these are the
// two pieces the released model of its Table 1 has on top of the plain block):
//
//   * per-head RMS normalisation:  u <- u / sqrt(mean_d(u^2) + eps) * g,  u the d_h elements of one
//     head of q (scales g_q) or of k (scales g_k);
//   * rotary position embedding (temporal layers only): with t the token's frame index, the element
//     pair (u[2i], u[2i+1]) is rotated by the angle t * 10000^(-2i/d_h).
//
// In place on the q and k columns of the fused projection buffer (q | k are 2A contiguous columns
// of a token row), fp32 arithmetic, one rounding to bf16 at the end.
//
// Bound: HBM.  Algorithmic bytes: 2 * (2A * 2) per token (q and k read and written once); at 480p
// 448 MB per call.  One thread owns one 16-byte piece (8 elements = 4 rotation pairs) of one head;
// the d_h/8 threads of a head add their partial sums of squares through LDS (d_h/8 is 8 or 9, so
// the groups do not line up with wavefronts); the block size is a multiple of both, so a head's
// group never straddles a block.  The angles come from a table [T, d_h/2] of (cos, sin) built once
// per call by k_rope_table with the accurate sincosf (the angle reaches t itself for the first pair).
#include "ddit_common.hpp"

namespace {

constexpr int BLOCK = 576;   // 64 * 9: a multiple of d_h/8 for d_h = 64 and 72

__global__ void k_rope_table(float2 *__restrict__ tab, int T, int half) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * half) return;
  const int t = i / half, p = i % half;
  // 10000^(-2p/d_h) = 2^(-p * log2(10000) / half)
  const float w = exp2f(-(float)p * 13.287712379549449f / (float)half);
  float s, c;
  sincosf((float)t * w, &s, &c);
  tab[i] = make_float2(c, s);
}

struct QkArgs {
  bf16_t *qk;              // first treated column of token 0
  int64_t ld;              // row stride in elements
  int64_t pieces;          // N * pieces_per_token
  int pieces_per_token;    // slots * (DH / 8), slots = heads treated per token (q heads first, then k heads)
  int q_slots;             // the first q_slots heads take g_q, the rest g_k
  const bf16_t *g_q, *g_k; // [DH] or null: no normalisation
  float eps;
  const float2 *rope;      // [T, DH/2] or null: no rotation
  int64_t S; int T;
};

__device__ __forceinline__ unsigned short f32_to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                                  // round to nearest even
  return (unsigned short)(u >> 16);
}

template <int DH>
__global__ __launch_bounds__(BLOCK) void k_qk_norm_rope(QkArgs a) {
  constexpr int PIECES = DH / 8;
  static_assert(DH % 8 == 0 && BLOCK % PIECES == 0, "a head's pieces must not straddle a block");
  __shared__ float part[BLOCK];
  const int tid = threadIdx.x;
  const int64_t f = (int64_t)blockIdx.x * BLOCK + tid;
  const bool live = f < a.pieces;
  const int64_t n = live ? f / a.pieces_per_token : 0;
  const int r = live ? (int)(f - n * a.pieces_per_token) : 0;
  const int slot = r / PIECES, piece = r - slot * PIECES;   // slot < q_slots: a q head, else a k head
  float v[8];
  uint4 raw = make_uint4(0, 0, 0, 0);
  bf16_t *ptr = a.qk + n * a.ld + (int64_t)r * 8;
  if (live) raw = *reinterpret_cast<const uint4 *>(ptr);
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[2 * j] = __uint_as_float(w[j] << 16);
    v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
  if (a.g_q) {
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
    part[tid] = ss;
    __syncthreads();
    const int g0 = tid - piece;   // first thread of this head's group (same block by construction)
    float tot = 0.f;
#pragma unroll
    for (int j = 0; j < PIECES; ++j) tot += part[g0 + j];
    const float rinv = rsqrtf(tot * (1.0f / DH) + a.eps);
    const uint4 graw = *reinterpret_cast<const uint4 *>((slot < a.q_slots ? a.g_q : a.g_k) + piece * 8);
    const unsigned gw[4] = {graw.x, graw.y, graw.z, graw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] = v[2 * j] * rinv * __uint_as_float(gw[j] << 16);
      v[2 * j + 1] = v[2 * j + 1] * rinv * __uint_as_float(gw[j] & 0xffff0000u);
    }
  }
  if (a.rope) {
    const int t = (int)((n / a.S) % a.T);
    const float2 *cs = a.rope + (int64_t)t * (DH / 2) + piece * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float2 c = cs[j];
      const float x0 = v[2 * j], x1 = v[2 * j + 1];
      v[2 * j] = x0 * c.x - x1 * c.y;
      v[2 * j + 1] = x1 * c.x + x0 * c.y;
    }
  }
  if (live) {
    uint4 out;
    out.x = (unsigned)f32_to_bf16(v[0]) | ((unsigned)f32_to_bf16(v[1]) << 16);
    out.y = (unsigned)f32_to_bf16(v[2]) | ((unsigned)f32_to_bf16(v[3]) << 16);
    out.z = (unsigned)f32_to_bf16(v[4]) | ((unsigned)f32_to_bf16(v[5]) << 16);
    out.w = (unsigned)f32_to_bf16(v[6]) | ((unsigned)f32_to_bf16(v[7]) << 16);
    *reinterpret_cast<uint4 *>(ptr) = out;
  }
}

}  // namespace

namespace ddit {

int launch_rope_table(float *table, int T, int dh, hipStream_t s) {
  const int half = dh / 2, total = T * half;
  if (total <= 0) return 0;
  hipLaunchKernelGGL(k_rope_table, dim3((total + 255) / 256), dim3(256), 0, s, reinterpret_cast<float2 *>(table), T, half);
  return hip_fail(hipGetLastError(), "rope table launch");
}

int launch_qk_norm_rope(void *qk, int64_t ld, int64_t N, int slots, int q_slots, int dh, const void *g_q,
                        const void *g_k, float eps, const float *rope_table, int64_t S, int T, hipStream_t s) {
  if (N == 0 || slots == 0 || (!g_q && !rope_table)) return 0;
  QkArgs a;
  a.qk = reinterpret_cast<bf16_t *>(qk); a.ld = ld;
  a.pieces_per_token = slots * (dh / 8);
  a.pieces = N * a.pieces_per_token;
  a.q_slots = q_slots;
  a.g_q = reinterpret_cast<const bf16_t *>(g_q); a.g_k = reinterpret_cast<const bf16_t *>(g_k);
  a.eps = eps;
  a.rope = reinterpret_cast<const float2 *>(rope_table);
  a.S = S > 0 ? S : 1; a.T = T > 0 ? T : 1;
  const int64_t blocks = (a.pieces + BLOCK - 1) / BLOCK;
  if (blocks > 0x7fffffff) { set_error("qk_norm_rope: %lld blocks: too many", (long long)blocks); return -2; }
  if (dh == 72) hipLaunchKernelGGL(k_qk_norm_rope<72>, dim3((unsigned)blocks), dim3(BLOCK), 0, s, a);
  else if (dh == 64) hipLaunchKernelGGL(k_qk_norm_rope<64>, dim3((unsigned)blocks), dim3(BLOCK), 0, s, a);
  else { set_error("qk_norm_rope: dh=%d not supported", dh); return -2; }
  return hip_fail(hipGetLastError(), "qk_norm_rope launch");
}

}  // namespace ddit
