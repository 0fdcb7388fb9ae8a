// Fused adaLN-single modulation + LayerNorm:  out = bf16( LN(x) * (1 + scale_b) + shift_b ).
//
// LN is taken over the hidden axis without affine parameters and with the biased
// variance; (shift_b, scale_b) are two rows of the per-layer table plus the sample's
// conditioning vector.  The stage is HBM-bound (reads 4 B, writes 2 B per element), so
// the kernel keeps one token row per wavefront entirely in registers: one pass over
// HBM, 16-byte loads, 8-byte stores, mean and variance by two wave reductions (the
// variance from the deviations, not from E[x^2]).
#include "ddit_common.hpp"

namespace {

template <int CHUNKS>  // float4 chunks per lane; D <= 256*CHUNKS
__global__ __launch_bounds__(256) void k_modulated_layernorm(const float *__restrict__ x,
                                                             const float *__restrict__ tab,
                                                             const float *__restrict__ c6, int which, int64_t N,
                                                             int64_t tokens_per_sample, int D, float eps,
                                                             bf16_t *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= N) return;
  const int nchunk = D >> 2;
  const float4 *xr = reinterpret_cast<const float4 *>(x + row * (int64_t)D);
  float4 v[CHUNKS];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunk) {
      v[j] = xr[c];
      s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
    } else {
      v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const float mean = wave_sum(s) / (float)D;
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunk) {
      const float a = v[j].x - mean, b = v[j].y - mean, cc = v[j].z - mean, d = v[j].w - mean;
      ss += (a * a + b * b) + (cc * cc + d * d);
    }
  }
  const float rstd = rsqrtf(wave_sum(ss) / (float)D + eps);
  const int64_t b = row / tokens_per_sample;
  const float4 *t_shift = reinterpret_cast<const float4 *>(tab + (int64_t)(3 * which) * D);
  const float4 *t_scale = reinterpret_cast<const float4 *>(tab + (int64_t)(3 * which + 1) * D);
  const float4 *c_shift = reinterpret_cast<const float4 *>(c6 + b * 6 * (int64_t)D + (int64_t)(3 * which) * D);
  const float4 *c_scale = reinterpret_cast<const float4 *>(c6 + b * 6 * (int64_t)D + (int64_t)(3 * which + 1) * D);
  bf16x4 *orow = reinterpret_cast<bf16x4 *>(out + row * (int64_t)D);
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunk) {
      const float4 ts = t_shift[c], tc = t_scale[c], cs = c_shift[c], cc = c_scale[c];
      bf16x4 o;
      o[0] = (bf16_t)((v[j].x - mean) * rstd * (1.f + (tc.x + cc.x)) + (ts.x + cs.x));
      o[1] = (bf16_t)((v[j].y - mean) * rstd * (1.f + (tc.y + cc.y)) + (ts.y + cs.y));
      o[2] = (bf16_t)((v[j].z - mean) * rstd * (1.f + (tc.z + cc.z)) + (ts.z + cs.z));
      o[3] = (bf16_t)((v[j].w - mean) * rstd * (1.f + (tc.w + cc.w)) + (ts.w + cs.w));
      orow[c] = o;
    }
  }
}

}  // namespace

namespace ddit {

int launch_modulated_layernorm(const float *x, const float *ada_table, const float *c6, int which, int64_t N,
                               int64_t tokens_per_sample, int D, float eps, void *out, hipStream_t s) {
  if (N == 0) return 0;
  const unsigned grid = (unsigned)((N + 3) / 4);
  bf16_t *o = reinterpret_cast<bf16_t *>(out);
  if (D <= 256 * 2)
    hipLaunchKernelGGL(k_modulated_layernorm<2>, dim3(grid), dim3(256), 0, s, x, ada_table, c6, which, N,
                       tokens_per_sample, D, eps, o);
  else if (D <= 256 * 5)
    hipLaunchKernelGGL(k_modulated_layernorm<5>, dim3(grid), dim3(256), 0, s, x, ada_table, c6, which, N,
                       tokens_per_sample, D, eps, o);
  else if (D <= 256 * 16)
    hipLaunchKernelGGL(k_modulated_layernorm<16>, dim3(grid), dim3(256), 0, s, x, ada_table, c6, which, N,
                       tokens_per_sample, D, eps, o);
  else {
    set_error("D=%d: hidden size above 4096 is not supported by the LayerNorm kernel", D);
    return -2;
  }
  return hip_fail(hipGetLastError(), "modulated_layernorm launch");
}

}  // namespace ddit
