// Measurement probes: the denominators the step's kernels are held against, as kernels of this
// library so that the benchmark reproduces them on the box it runs on.
//   ddit_probe_mfma_bf16       - a register-resident loop of v_mfma_f32_32x32x16_bf16 on operand data the
//                                caller supplies (the chip's clock under matrix load depends on the data)
//   ddit_probe_stream_copy     - a plain streaming copy of n bytes (16 bytes per lane, grid-stride)
//   ddit_probe_stream_read     - the same bytes read only
//   ddit_probe_residual_stream - the memory traffic of a k = A out-projection with gated residual update
//                                (fp32 stream read and written, bf16 copy written, bf16 operand rows and a
//                                gate vector read) and none of its matrix work: the floor such a launch
//                                cannot go below
// None of them is on the hot path.
#include "../../include/ddit_hot.h"
#include "ddit_common.hpp"

namespace {

// 12 independent accumulators per wavefront (the linear's 3 x 4 wave tile), two wavefronts per SIMD
__global__ __launch_bounds__(256, 2) void k_probe_mfma(const bf16x8 *__restrict__ src, float *out, int iters) {
  bf16x8 a[4], b[3];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = src[(threadIdx.x + 256 * i) & 4095];
#pragma unroll
  for (int i = 0; i < 3; ++i) b[i] = src[(threadIdx.x + 256 * (i + 4)) & 4095];
  floatx16 acc[12];
#pragma unroll
  for (int j = 0; j < 12; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < 3; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) acc[x * 4 + y] = mfma32(b[x], a[y], acc[x * 4 + y]);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 12; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// grid-stride over 16-byte pieces, four independent pieces in flight per thread
__global__ __launch_bounds__(256) void k_probe_copy(const floatx4 *__restrict__ in, floatx4 *__restrict__ out, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const floatx4 a = __builtin_nontemporal_load(in + i), b = __builtin_nontemporal_load(in + i + stride),
                  c = __builtin_nontemporal_load(in + i + 2 * stride), d = __builtin_nontemporal_load(in + i + 3 * stride);
    __builtin_nontemporal_store(a, out + i);
    __builtin_nontemporal_store(b, out + i + stride);
    __builtin_nontemporal_store(c, out + i + 2 * stride);
    __builtin_nontemporal_store(d, out + i + 3 * stride);
  }
  for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(in + i), out + i);
}

// read-only stream: every thread adds up its pieces and leaves one float
__global__ __launch_bounds__(256) void k_probe_read(const floatx4 *__restrict__ in, float *__restrict__ sink, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  floatx4 s = {0.f, 0.f, 0.f, 0.f};
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const floatx4 a = __builtin_nontemporal_load(in + i), b = __builtin_nontemporal_load(in + i + stride),
                  c = __builtin_nontemporal_load(in + i + 2 * stride), d = __builtin_nontemporal_load(in + i + 3 * stride);
    s += (a + b) + (c + d);
  }
  for (; i < n16; i += stride) s += __builtin_nontemporal_load(in + i);
  sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = (s[0] + s[1]) + (s[2] + s[3]);
}

// One wavefront per token row, rows dealt to wavefronts in consecutive runs of four; per row: read A bf16 of
// the operand row `o`, read D fp32 of the stream, add gate * (a value derived from the operand row), write D fp32
// and D bf16.  Streaming loads and stores, like the epilogue it stands for.
__global__ __launch_bounds__(256) void k_probe_residual_stream(float *__restrict__ x, bf16_t *__restrict__ xh,
                                                               const bf16_t *__restrict__ o, const float *__restrict__ gate,
                                                               int64_t N, int D, int A) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t row0 = wave * 4; row0 < N; row0 += n_waves * 4) {
    for (int r = 0; r < 4 && row0 + r < N; ++r) {
      const int64_t row = row0 + r;
      float s = 0.f;
      for (int c = lane * 8; c < A; c += 64 * 8) {
        const bf16x8 v = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(o + row * A + c));
        s += (float)v[0] + (float)v[7];
      }
      s = wave_sum(s) * 1e-3f;
      for (int c = lane * 4; c < D; c += 64 * 4) {
        floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(x + row * D + c));
        const floatx4 g = *reinterpret_cast<const floatx4 *>(gate + c);
        bf16x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] += g[e] * s;
          h[e] = (bf16_t)v[e];
        }
        __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(x + row * D + c));
        __builtin_nontemporal_store(h, reinterpret_cast<bf16x4 *>(xh + row * D + c));
      }
    }
  }
}

inline bool al16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

using ddit::set_error;

extern "C" {

int ddit_probe_mfma_bf16(const void *operands, float *sink, int32_t iters, double *flop_out, void *hip_stream) {
  if (!operands || !sink || iters < 1 || iters > (1 << 24)) { set_error("probe_mfma: operands, sink and 1 <= iters <= 2^24 required"); return DDIT_ERR_INVALID_ARG; }
  if (!al16(operands) || !al16(sink)) { set_error("probe_mfma: pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  const int blocks = 2 * ddit::device_cus();
  if (flop_out) *flop_out = (double)blocks * 4 * iters * 12 * (2.0 * 32 * 32 * 16);
  hipLaunchKernelGGL(k_probe_mfma, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<const bf16x8 *>(operands), sink, iters);
  return ddit::hip_fail(hipGetLastError(), "probe_mfma launch");
}

int ddit_probe_stream_copy(const void *in, void *out, int64_t bytes, void *hip_stream) {
  if (!in || !out || bytes < 0 || bytes % 16) { set_error("probe_copy: in, out and a multiple of 16 bytes required"); return DDIT_ERR_INVALID_ARG; }
  if (!al16(in) || !al16(out)) { set_error("probe_copy: pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  if (bytes == 0) return DDIT_OK;
  const int blocks = 16 * ddit::device_cus();
  hipLaunchKernelGGL(k_probe_copy, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<const floatx4 *>(in), reinterpret_cast<floatx4 *>(out), bytes / 16);
  return ddit::hip_fail(hipGetLastError(), "probe_copy launch");
}

int ddit_probe_stream_read(const void *in, int64_t bytes, float *sink, void *hip_stream) {
  if (!in || !sink || bytes < 0 || bytes % 16) { set_error("probe_read: in, sink and a multiple of 16 bytes required"); return DDIT_ERR_INVALID_ARG; }
  if (!al16(in) || !al16(sink)) { set_error("probe_read: pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  const int blocks = 16 * ddit::device_cus();
  hipLaunchKernelGGL(k_probe_read, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<const floatx4 *>(in), sink, bytes / 16);
  return ddit::hip_fail(hipGetLastError(), "probe_read launch");
}

int ddit_probe_residual_stream(float *x, void *xh_out, const void *o, const float *gate, int64_t N, int32_t D, int32_t A,
                               void *hip_stream) {
  if (!x || !xh_out || !o || !gate || N < 0 || D < 8 || A < 8 || D % 8 || A % 8) {
    set_error("probe_residual_stream: x, xh_out, o, gate, N >= 0 and D, A multiples of 8 required"); return DDIT_ERR_INVALID_ARG;
  }
  if (!al16(x) || !al16(xh_out) || !al16(o) || !al16(gate)) { set_error("probe_residual_stream: pointers must be 16-byte aligned"); return DDIT_ERR_ALIGNMENT; }
  if (N == 0) return DDIT_OK;
  const int blocks = 8 * ddit::device_cus();
  hipLaunchKernelGGL(k_probe_residual_stream, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), x,
                     reinterpret_cast<bf16_t *>(xh_out), reinterpret_cast<const bf16_t *>(o), gate, N, (int)D, (int)A);
  return ddit::hip_fail(hipGetLastError(), "probe_residual_stream launch");
}

}  // extern "C"
