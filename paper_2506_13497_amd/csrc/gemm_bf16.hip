// bf16 Linear  out = u W^T + b  on the CDNA4 matrix cores, with fused epilogues.
//
// u is [N,k] tokens x in-features, W is [n,k]: both operands have the contraction axis
// contiguous, which is exactly what v_mfma_f32_32x32x16_bf16 wants in its registers
// (8 consecutive k per lane), so tiles go global -> LDS -> registers as 16-byte pieces
// with no transposition anywhere.
//
// Tiling.  One workgroup of 4 wavefronts owns a BM x BN tile of the output (BM tokens,
// BN out-features) and walks k in steps of 64.  The wavefronts form a 2x2 grid; each
// owns (BM/2) x (BN/2), i.e. (BM/64)*(BN/64) MFMA tiles of 32x32 with fp32 accumulators
// in registers.  The MFMA is issued with W as its first operand and u as its second, so
// a lane ends up holding, for one token, 4 consecutive out-features per accumulator
// group: the epilogue reads/writes 8-byte (bf16) or 16-byte (fp32) pieces per lane.
// LDS holds two stages of (BM + BN) rows x 128 B.  A row's eight 16-byte chunks are
// stored at chunk position c ^ (row & 7): the ds_read_b128 of 8 consecutive rows at the
// same k then touches all 32 banks once.  Global loads for step i+2 are in flight while
// step i is multiplied; one barrier per step.
//
// Workgroup -> tile map.  Workgroups are dealt round-robin to the 8 XCDs, each with its
// own L2, so ids are re-numbered to give every XCD a contiguous run of tiles, ordered
// with the out-feature tile fastest: the CUs of one XCD share a token panel of u.
//
// Epilogues: bf16 store; GELU(tanh form) + bf16 store; gated residual update of the
// fp32 stream (x += gate_b * (acc + bias)), optionally also storing bf16(x).
#include "ddit_common.hpp"

namespace {

constexpr int BK = 64;          // k per pipeline step (bf16 elements); one LDS row = 128 B
constexpr int ROW_BYTES = 128;

struct GemmParams {
  const bf16_t *u; int64_t ld_u;
  const bf16_t *W;
  const bf16_t *bias;
  int64_t N; int n; int k;
  bf16_t *out; int64_t ld_out;
  float *resid;
  const float *gate_tab;
  const float *gate_c6; int64_t gate_c6_stride;
  int64_t tokens_per_sample;
  int tiles_n; int64_t total_tiles;
};

__device__ __forceinline__ float gelu_tanh_f(float u) {
  // 0.5 u (1 + tanh(z)) == u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3)
  const float kA = -2.0f * 0.7978845608028654f * 1.4426950408889634f;  // -2 sqrt(2/pi) log2(e)
  const float t = u * u;
  const float z2 = u * (kA + (kA * 0.044715f) * t);                    // -2 z log2(e)
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z2));
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmParams p) {
  constexpr int TM = BM / 64;  // 32-token MFMA tiles per wave
  constexpr int TN = BN / 64;  // 32-feature MFMA tiles per wave
  constexpr int U_CH = BM * 8 / 256;  // 16-byte chunks per thread per stage
  constexpr int W_CH = BN * 8 / 256;
  constexpr int STAGE = (BM + BN) * ROW_BYTES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- XCD-aware tile id
  const int64_t pid = blockIdx.x;
  const int64_t q8 = p.total_tiles >> 3, r8 = p.total_tiles & 7;
  const int64_t xcd = pid & 7, loc = pid >> 3;
  const int64_t tile = xcd * q8 + (xcd < r8 ? xcd : r8) + loc;
  const int64_t tile_m = tile / p.tiles_n;
  const int tile_n = (int)(tile - tile_m * p.tiles_n);
  const int64_t row0 = tile_m * BM;
  const int col0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  // ---- global -> register staging: chunk idx -> (row r, 16-byte chunk c)
  const int ld_r = tid >> 3, ld_c = tid & 7;  // + 32 rows per extra chunk
  const bf16_t *u_ptr[U_CH];
  const bf16_t *w_ptr[W_CH];
#pragma unroll
  for (int i = 0; i < U_CH; ++i) {
    int64_t r = row0 + ld_r + 32 * i;
    if (r > p.N - 1) r = p.N - 1;  // overhanging rows re-read the last token; never stored
    u_ptr[i] = p.u + r * p.ld_u + ld_c * 8;
  }
#pragma unroll
  for (int i = 0; i < W_CH; ++i) {
    int r = col0 + ld_r + 32 * i;
    if (r > p.n - 1) r = p.n - 1;
    w_ptr[i] = p.W + (int64_t)r * p.k + ld_c * 8;
  }
  uint4 u_reg[U_CH], w_reg[W_CH];
  const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

  auto g_load = [&](int k0) {
    const bool ok = (k0 + ld_c * 8) < p.k;  // k tail: zero-fill both operands
#pragma unroll
    for (int i = 0; i < U_CH; ++i) u_reg[i] = ok ? *reinterpret_cast<const uint4 *>(u_ptr[i] + k0) : zero4;
#pragma unroll
    for (int i = 0; i < W_CH; ++i) w_reg[i] = ok ? *reinterpret_cast<const uint4 *>(w_ptr[i] + k0) : zero4;
  };
  auto s_store = [&](int stage) {
    unsigned char *su = smem + stage * STAGE;
    unsigned char *sw = su + BM * ROW_BYTES;
#pragma unroll
    for (int i = 0; i < U_CH; ++i) {
      const int r = ld_r + 32 * i;
      *reinterpret_cast<uint4 *>(su + r * ROW_BYTES + ((ld_c ^ (r & 7)) << 4)) = u_reg[i];
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
      const int r = ld_r + 32 * i;
      *reinterpret_cast<uint4 *>(sw + r * ROW_BYTES + ((ld_c ^ (r & 7)) << 4)) = w_reg[i];
    }
  };

  floatx16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  const int nk = (p.k + BK - 1) / BK;
  g_load(0);
  s_store(0);
  if (nk > 1) g_load(BK);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) s_store(cur ^ 1);         // registers hold step kt+1
    if (kt + 2 < nk) g_load((kt + 2) * BK);    // in flight during the multiply below
    const unsigned char *su = smem + cur * STAGE + (wm * (BM / 2)) * ROW_BYTES;
    const unsigned char *sw = smem + cur * STAGE + BM * ROW_BYTES + (wn * (BN / 2)) * ROW_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int c = kk * 2 + lh;
      bf16x8 uf[TM], wf[TN];
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const int r = b * 32 + l32;
        uf[b] = *reinterpret_cast<const bf16x8 *>(su + r * ROW_BYTES + ((c ^ (r & 7)) << 4));
      }
#pragma unroll
      for (int a = 0; a < TN; ++a) {
        const int r = a * 32 + l32;
        wf[a] = *reinterpret_cast<const bf16x8 *>(sw + r * ROW_BYTES + ((c ^ (r & 7)) << 4));
      }
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = mfma32(wf[a], uf[b], acc[a][b]);
    }
    __syncthreads();
  }

  // ---- epilogue: acc[a][b][4g+e] = C[token = tb + l32][feature = fb + 8g + 4 lh + e]
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int64_t tok = row0 + wm * (BM / 2) + b * 32 + l32;
    if (tok >= p.N) continue;
    int64_t sample = 0;
    if (EPI == 2 && p.gate_c6) sample = tok / p.tokens_per_sample;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int f = col0 + wn * (BN / 2) + a * 32 + 8 * g + 4 * lh;
        if (f >= p.n) continue;
        float v0 = acc[a][b][4 * g + 0], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
              v3 = acc[a][b][4 * g + 3];
        if (p.bias) {
          const bf16x4 bb = *reinterpret_cast<const bf16x4 *>(p.bias + f);
          v0 += (float)bb[0]; v1 += (float)bb[1]; v2 += (float)bb[2]; v3 += (float)bb[3];
        }
        if (EPI == 1) {
          v0 = gelu_tanh_f(v0); v1 = gelu_tanh_f(v1); v2 = gelu_tanh_f(v2); v3 = gelu_tanh_f(v3);
        }
        if (EPI == 2) {
          if (p.gate_tab) {
            float4 gt = *reinterpret_cast<const float4 *>(p.gate_tab + f);
            if (p.gate_c6) {
              const float4 gc = *reinterpret_cast<const float4 *>(p.gate_c6 + sample * p.gate_c6_stride + f);
              gt.x += gc.x; gt.y += gc.y; gt.z += gc.z; gt.w += gc.w;
            }
            v0 *= gt.x; v1 *= gt.y; v2 *= gt.z; v3 *= gt.w;
          }
          float4 *rp = reinterpret_cast<float4 *>(p.resid + tok * (int64_t)p.n + f);
          float4 r = *rp;
          r.x += v0; r.y += v1; r.z += v2; r.w += v3;
          *rp = r;
          v0 = r.x; v1 = r.y; v2 = r.z; v3 = r.w;
          if (!p.out) continue;
        }
        bf16x4 o;
        o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
        *reinterpret_cast<bf16x4 *>(p.out + tok * p.ld_out + f) = o;
      }
    }
  }
}

template <int BM, int BN, int EPI>
int launch_one(const GemmParams &p0, hipStream_t s) {
  GemmParams p = p0;
  const int64_t tiles_m = (p.N + BM - 1) / BM;
  p.tiles_n = (p.n + BN - 1) / BN;
  p.total_tiles = tiles_m * p.tiles_n;
  constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
  static bool attr_set = false;  // benign race: the attribute is idempotent
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<BM, BN, EPI>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return ddit::hip_fail(e, "gemm hipFuncSetAttribute");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_gemm_bf16<BM, BN, EPI>), dim3((unsigned)p.total_tiles), dim3(256), smem, s, p);
  return ddit::hip_fail(hipGetLastError(), "gemm launch");
}

template <int EPI>
int launch_epi(const GemmParams &p, hipStream_t s) {
  // 192-wide feature tiles divide 1152, 3456, 4608 and 2304 exactly; narrow outputs and
  // short token counts take the smaller tile so more than a handful of CUs get work.
  const int64_t big_tiles = ((p.N + 255) / 256) * ((p.n + 191) / 192);
  if (big_tiles >= 128 && (p.n % 192 == 0 || p.n > 1024)) return launch_one<256, 192, EPI>(p, s);
  return launch_one<128, 128, EPI>(p, s);
}

}  // namespace

namespace ddit {

int launch_gemm(int epilogue, const GemmArgs &a, hipStream_t s) {
  if (a.N == 0 || a.n == 0) return 0;
  GemmParams p;
  p.u = reinterpret_cast<const bf16_t *>(a.u); p.ld_u = a.ld_u;
  p.W = reinterpret_cast<const bf16_t *>(a.W);
  p.bias = reinterpret_cast<const bf16_t *>(a.bias);
  p.N = a.N; p.n = a.n; p.k = a.k;
  p.out = reinterpret_cast<bf16_t *>(a.out); p.ld_out = a.ld_out;
  p.resid = a.resid;
  p.gate_tab = a.gate_tab; p.gate_c6 = a.gate_c6; p.gate_c6_stride = a.gate_c6_stride;
  p.tokens_per_sample = a.tokens_per_sample > 0 ? a.tokens_per_sample : 1;
  p.tiles_n = 0; p.total_tiles = 0;
  switch (epilogue) {
    case 0: return launch_epi<0>(p, s);
    case 1: return launch_epi<1>(p, s);
    case 2: return launch_epi<2>(p, s);
  }
  set_error("unknown epilogue %d", epilogue);
  return -1;
}

}  // namespace ddit
