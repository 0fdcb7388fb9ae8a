// The layers around the token-space step and the solver of the sampling loop (eq. 1):
//   patch embedding of the latent + position code, output head (modulated LayerNorm + small
//   Linear + scatter back to the latent grid), Euler update with optional guidance.
// All of them are bound by memory traffic or launch latency (well under 0.1 % of a step's
// arithmetic), so they are plain vector-ALU kernels with coalesced token rows.
#include "ddit_common.hpp"

namespace {

constexpr int PATCH_MAX = 64;   // 4 * channels at most
constexpr int TOK_PER_WG = 32;

// pos[s, :] for s = i*Wp + j: quarters sin(j w_m), cos(j w_m), sin(i w_m), cos(i w_m),
// w_m = 10000^(-m/Q), Q = D/4.  Arguments stay below a few hundred radians; evaluated in fp64
// like the timestep features (once per call, S*D values).
__global__ void k_position_code(float *__restrict__ pos, int Hp, int Wp, int D) {
  const int s = blockIdx.x;
  const int i = s / Wp, j = s - i * Wp;
  const int Q = D / 4;
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    const int quarter = d / Q, m = d - quarter * Q;
    const double w = exp(-log(10000.0) * (double)m / (double)Q);
    const double arg = (double)(quarter < 2 ? j : i) * w;
    pos[(int64_t)s * D + d] = (float)((quarter & 1) ? cos(arg) : sin(arg));
  }
}

// x[token, d] = bf16( sum_p patch[token, p] W[d, p] + bias[d] + pos[s, d] ), patch order (c, di, dj).
// A workgroup takes TOK_PER_WG consecutive tokens: their patches go to LDS, then every thread
// owns output features d = tid, tid + 256, ... and keeps that feature's weight row in registers
// across the tokens.  PC = compile-time channel count (weight rows fetched as 16-byte pieces,
// patches read from LDS four values at a time), or 0 for any channel count.
template <int PC>
__global__ __launch_bounds__(256) void k_patch_embed(const float *__restrict__ z, const bf16_t *__restrict__ W,
                                                     const bf16_t *__restrict__ bias, const float *__restrict__ pos,
                                                     bf16_t *__restrict__ x, int B, int C, int T, int Hp, int Wp,
                                                     int D) {
  __shared__ __attribute__((aligned(16))) float patch[TOK_PER_WG][PATCH_MAX];
  const int P = PC > 0 ? 4 * PC : 4 * C;
  const int64_t S = (int64_t)Hp * Wp, N = (int64_t)B * T * S;
  const int64_t tok0 = (int64_t)blockIdx.x * TOK_PER_WG;
  for (int e = threadIdx.x; e < TOK_PER_WG * P; e += blockDim.x) {
    const int k = e / P, p = e - k * P;
    const int64_t tok = tok0 + k;
    float v = 0.f;
    if (tok < N) {
      const int64_t bt = tok / S, s = tok - bt * S;
      const int b = (int)(bt / T), t = (int)(bt - (int64_t)b * T);
      const int i = (int)(s / Wp), j = (int)(s - (int64_t)i * Wp);
      const int c = p >> 2, di = (p >> 1) & 1, dj = p & 1;
      v = z[((((int64_t)b * C + c) * T + t) * (2 * Hp) + (2 * i + di)) * (2 * Wp) + (2 * j + dj)];
    }
    patch[k][p] = v;
  }
  __syncthreads();
  const int ntok = N - tok0 < TOK_PER_WG ? (int)(N - tok0) : TOK_PER_WG;
  const int64_t s0 = tok0 % S;
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    constexpr int PW = PC > 0 ? 4 * PC : PATCH_MAX;
    float w[PW];
    if constexpr (PC > 0 && PC % 2 == 0) {
#pragma unroll
      for (int p8 = 0; p8 < PW / 8; ++p8) {
        const bf16x8 v = *reinterpret_cast<const bf16x8 *>(W + (int64_t)d * P + 8 * p8);
#pragma unroll
        for (int e = 0; e < 8; ++e) w[8 * p8 + e] = (float)v[e];
      }
    } else {
#pragma unroll
      for (int p = 0; p < PW; ++p) w[p] = p < P ? (float)W[(int64_t)d * P + p] : 0.f;
    }
    const float bd = bias ? (float)bias[d] : 0.f;
    int64_t s = s0;
    for (int k = 0; k < ntok; ++k) {
      float acc = 0.f;
#pragma unroll
      for (int p4 = 0; p4 < PW / 4; ++p4) {
        if (4 * p4 < P) {
          const float4 pv = *reinterpret_cast<const float4 *>(&patch[k][4 * p4]);
          acc += pv.x * w[4 * p4] + pv.y * w[4 * p4 + 1] + pv.z * w[4 * p4 + 2] + pv.w * w[4 * p4 + 3];
        }
      }
      x[(tok0 + k) * D + d] = (bf16_t)(acc + bd + pos[s * D + d]);
      if (++s == S) s = 0;
    }
  }
}

// Output head, one wavefront per token: LayerNorm of the bf16 token row (biased variance, the
// variance from the deviations), modulation by final_table + temb_b, F = 4*C_out dot products
// of length D with the head's weight rows, each reduced over the wavefront; lane f stores
// output f = (di*2 + dj)*C_out + c at z_out[b, c, t, 2i+di, 2j+dj].
template <int CHUNKS>   // 8-element chunks per lane; D <= 512 * CHUNKS
__global__ __launch_bounds__(256) void k_output_head(const bf16_t *__restrict__ x, const float *__restrict__ temb,
                                                     const float *__restrict__ table, const bf16_t *__restrict__ W,
                                                     const bf16_t *__restrict__ bias, float *__restrict__ out, int B,
                                                     int C_out, int T, int Hp, int Wp, int D, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t S = (int64_t)Hp * Wp, N = (int64_t)B * T * S;
  const int64_t tok = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= N) return;
  const int nchunk = D >> 3;
  const bf16x8 *xr = reinterpret_cast<const bf16x8 *>(x + tok * D);
  float v[CHUNKS][8];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunk) {
      const bf16x8 r = xr[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) { v[j][e] = (float)r[e]; s += v[j][e]; }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[j][e] = 0.f;
    }
  }
  const float mean = wave_sum(s) / (float)D;
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j)
    if (lane + 64 * j < nchunk) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float dlt = v[j][e] - mean; ss += dlt * dlt; }
    }
  const float rstd = rsqrtf(wave_sum(ss) / (float)D + eps);
  const int64_t bt = tok / S, sidx = tok - bt * S;
  const int b = (int)(bt / T), t = (int)(bt - (int64_t)b * T);
  const float *tb = temb + (int64_t)b * D;
#pragma unroll
  for (int j = 0; j < CHUNKS; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunk) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int d = 8 * c + e;
        v[j][e] = (v[j][e] - mean) * rstd * (1.f + (table[D + d] + tb[d])) + (table[d] + tb[d]);
      }
    }
  }
  const int F = 4 * C_out;
  float mine = 0.f;
  for (int f = 0; f < F; ++f) {
    const bf16x8 *wr = reinterpret_cast<const bf16x8 *>(W + (int64_t)f * D);
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < CHUNKS; ++j) {
      const int c = lane + 64 * j;
      if (c < nchunk) {
        const bf16x8 wv = wr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += v[j][e] * (float)wv[e];
      }
    }
    acc = wave_sum(acc);
    if (lane == f) mine = acc + (bias ? (float)bias[f] : 0.f);
  }
  if (lane < F) {
    const int i = (int)(sidx / Wp), jj = (int)(sidx - (int64_t)i * Wp);
    const int pq = lane / C_out, c = lane - pq * C_out, di = pq >> 1, dj = pq & 1;
    out[((((int64_t)b * C_out + c) * T + t) * (2 * Hp) + (2 * i + di)) * (2 * Wp) + (2 * jj + dj)] = mine;
  }
}

struct SolverArgs { float dt[64]; };   // (t_next - t) / 1000 per sample

__global__ void k_solver_step(float *__restrict__ z, const float *__restrict__ ec, const float *__restrict__ eu,
                              float guidance, SolverArgs a, int64_t per_sample, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int b = (int)(idx / per_sample);
  float e = ec[idx];
  if (eu) { const float u = eu[idx]; e = u + guidance * (e - u); }
  z[idx] += a.dt[b] * e;
}

}  // namespace

namespace ddit {

int launch_position_code(float *pos, int Hp, int Wp, int D, hipStream_t s) {
  hipLaunchKernelGGL(k_position_code, dim3((unsigned)(Hp * Wp)), dim3(256), 0, s, pos, Hp, Wp, D);
  return hip_fail(hipGetLastError(), "position code launch");
}

int launch_patch_embed(const float *z, const void *W, const void *bias, const float *pos, void *x, int B, int C,
                       int T, int Hp, int Wp, int D, hipStream_t s) {
  const int64_t N = (int64_t)B * T * Hp * Wp;
  if (N == 0) return 0;
  if (4 * C > PATCH_MAX) { set_error("patch embedding: 4*C_in=%d exceeds %d", 4 * C, PATCH_MAX); return -2; }
  const dim3 grid((unsigned)((N + TOK_PER_WG - 1) / TOK_PER_WG));
  const bf16_t *w = reinterpret_cast<const bf16_t *>(W), *bb = reinterpret_cast<const bf16_t *>(bias);
  bf16_t *xo = reinterpret_cast<bf16_t *>(x);
  // weight rows of 4*C bf16 are fetched as 16-byte pieces when that keeps them aligned
  if (C == 4) hipLaunchKernelGGL(k_patch_embed<4>, grid, dim3(256), 0, s, z, w, bb, pos, xo, B, C, T, Hp, Wp, D);
  else if (C == 8) hipLaunchKernelGGL(k_patch_embed<8>, grid, dim3(256), 0, s, z, w, bb, pos, xo, B, C, T, Hp, Wp, D);
  else if (C == 16) hipLaunchKernelGGL(k_patch_embed<16>, grid, dim3(256), 0, s, z, w, bb, pos, xo, B, C, T, Hp, Wp, D);
  else hipLaunchKernelGGL(k_patch_embed<0>, grid, dim3(256), 0, s, z, w, bb, pos, xo, B, C, T, Hp, Wp, D);
  return hip_fail(hipGetLastError(), "patch embedding launch");
}

int launch_output_head(const void *x, const float *temb, const float *table, const void *W, const void *bias,
                       float *out, int B, int C_out, int T, int Hp, int Wp, int D, float eps, hipStream_t s) {
  const int64_t N = (int64_t)B * T * Hp * Wp;
  if (N == 0) return 0;
  if (4 * C_out > 64) { set_error("output head: 4*C_out=%d exceeds 64", 4 * C_out); return -2; }
  const unsigned grid = (unsigned)((N + 3) / 4);
  const bf16_t *xx = reinterpret_cast<const bf16_t *>(x), *ww = reinterpret_cast<const bf16_t *>(W),
               *bb = reinterpret_cast<const bf16_t *>(bias);
  if (D <= 512)
    hipLaunchKernelGGL(k_output_head<1>, dim3(grid), dim3(256), 0, s, xx, temb, table, ww, bb, out, B, C_out, T, Hp, Wp, D, eps);
  else if (D <= 512 * 3)
    hipLaunchKernelGGL(k_output_head<3>, dim3(grid), dim3(256), 0, s, xx, temb, table, ww, bb, out, B, C_out, T, Hp, Wp, D, eps);
  else if (D <= 512 * 8)
    hipLaunchKernelGGL(k_output_head<8>, dim3(grid), dim3(256), 0, s, xx, temb, table, ww, bb, out, B, C_out, T, Hp, Wp, D, eps);
  else { set_error("D=%d: hidden size above 4096 is not supported by the output head", D); return -2; }
  return hip_fail(hipGetLastError(), "output head launch");
}

int launch_solver_step(float *z, const float *ec, const float *eu, float guidance, const float *dt, int B,
                       int64_t per_sample, hipStream_t s) {
  const int64_t total = (int64_t)B * per_sample;
  if (total == 0) return 0;
  SolverArgs a;
  for (int i = 0; i < 64; ++i) a.dt[i] = i < B ? dt[i] : 0.f;
  hipLaunchKernelGGL(k_solver_step, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, z, ec, eu, guidance, a,
                     per_sample, total);
  return hip_fail(hipGetLastError(), "solver step launch");
}

}  // namespace ddit
