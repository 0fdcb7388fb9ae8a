// Fused adaLN-single modulation + LayerNorm:  out = bf16( LN(x) * (1 + scale_b) + shift_b ).
//
// LN is taken over the hidden axis without affine parameters and with the biased
// variance; (shift_b, scale_b) are two rows of the per-layer table plus the sample's
// conditioning vector.  The stage is HBM-bound (reads 4 B, writes 2 B per element), so
// the kernel keeps a token row of a wavefront entirely in registers: one pass over
// HBM, 16-byte loads, 8-byte stores, mean and variance by two wave reductions (the
// variance from the deviations, not from E[x^2]).
#include "ddit_common.hpp"

namespace {

constexpr int ROWS_PER_WAVE = 4;

// CHUNKS = float4 chunks per lane; D <= 256*CHUNKS.  A wavefront takes ROWS_PER_WAVE consecutive
// token rows and keeps the sample's (1 + scale) and shift vectors in registers across them: read
// per row they would be four more vectors of D floats against one row of x, and although they come
// from cache, that traffic through the CU's vector cache then costs as much time as the HBM side.
template <int CHUNKS>
__global__ __launch_bounds__(256) void k_modulated_layernorm(const float *__restrict__ x,
                                                             const float *__restrict__ tab,
                                                             const float *__restrict__ c6, int which, int64_t N,
                                                             int64_t tokens_per_sample, int D, float eps,
                                                             bf16_t *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * ROWS_PER_WAVE;
  if (row0 >= N) return;
  const int nchunk = D >> 2;
  const float4 *t_shift = reinterpret_cast<const float4 *>(tab + (int64_t)(3 * which) * D);
  const float4 *t_scale = reinterpret_cast<const float4 *>(tab + (int64_t)(3 * which + 1) * D);
  float4 sc1[CHUNKS], sh[CHUNKS];   // 1 + scale, shift of sample b_cur
  int64_t b_cur = -1;
  const int64_t row_end = row0 + ROWS_PER_WAVE < N ? row0 + ROWS_PER_WAVE : N;
  // the first row's loads are issued before the modulation vectors are fetched
  float4 v[CHUNKS];
  auto load_row = [&](int64_t row) {
    const floatx4 *xr = reinterpret_cast<const floatx4 *>(x + row * (int64_t)D);
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      const int c = lane + 64 * j;
      v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (c < nchunk) {   // each row is read once and written once: streaming accesses
        const floatx4 t = __builtin_nontemporal_load(xr + c);
        v[j] = make_float4(t[0], t[1], t[2], t[3]);
      }
    }
  };
  load_row(row0);
  for (int64_t row = row0; row < row_end; ++row) {
    const int64_t b = row / tokens_per_sample;
    if (b != b_cur) {
      b_cur = b;
      const float4 *c_shift = reinterpret_cast<const float4 *>(c6 + b * 6 * (int64_t)D + (int64_t)(3 * which) * D);
      const float4 *c_scale = reinterpret_cast<const float4 *>(c6 + b * 6 * (int64_t)D + (int64_t)(3 * which + 1) * D);
#pragma unroll
      for (int j = 0; j < CHUNKS; ++j) {
        const int c = lane + 64 * j;
        if (c < nchunk) {
          const float4 ts = t_shift[c], tc = t_scale[c], cs = c_shift[c], cc = c_scale[c];
          sh[j] = make_float4(ts.x + cs.x, ts.y + cs.y, ts.z + cs.z, ts.w + cs.w);
          sc1[j] = make_float4(1.f + (tc.x + cc.x), 1.f + (tc.y + cc.y), 1.f + (tc.z + cc.z), 1.f + (tc.w + cc.w));
        }
      }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) s += (v[j].x + v[j].y) + (v[j].z + v[j].w);   // chunks past D hold zeros
    const float mean = wave_sum(s) / (float)D;
    float ss = 0.f;
    float4 dv[CHUNKS];
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      dv[j] = make_float4(v[j].x - mean, v[j].y - mean, v[j].z - mean, v[j].w - mean);
      if (lane + 64 * j < nchunk) ss += (dv[j].x * dv[j].x + dv[j].y * dv[j].y) + (dv[j].z * dv[j].z + dv[j].w * dv[j].w);
    }
    // the next row is on its way while this one is reduced and written
    if (row + 1 < row_end) load_row(row + 1);
    const float rstd = rsqrtf(wave_sum(ss) / (float)D + eps);
    bf16x4 *orow = reinterpret_cast<bf16x4 *>(out + row * (int64_t)D);
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      const int c = lane + 64 * j;
      if (c < nchunk) {
        bf16x4 o;
        o[0] = (bf16_t)(dv[j].x * rstd * sc1[j].x + sh[j].x);
        o[1] = (bf16_t)(dv[j].y * rstd * sc1[j].y + sh[j].y);
        o[2] = (bf16_t)(dv[j].z * rstd * sc1[j].z + sh[j].z);
        o[3] = (bf16_t)(dv[j].w * rstd * sc1[j].w + sh[j].w);
        __builtin_nontemporal_store(o, orow + c);
      }
    }
  }
}

}  // namespace

namespace ddit {

int launch_modulated_layernorm(const float *x, const float *ada_table, const float *c6, int which, int64_t N,
                               int64_t tokens_per_sample, int D, float eps, void *out, hipStream_t s) {
  if (N == 0) return 0;
  const unsigned grid = (unsigned)((N + 4 * ROWS_PER_WAVE - 1) / (4 * ROWS_PER_WAVE));
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
