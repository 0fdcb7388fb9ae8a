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
// a lane ends up holding, for one token, 4 consecutive out-features per accumulator group.
// LDS holds two stages of (BM + BN) rows x 128 B.  A row's eight 16-byte chunks are
// stored at chunk position c ^ (row & 7): the ds_read_b128 of 8 consecutive rows at the
// same k then touches all 32 banks once.
//
// Pipeline.  A k-step is four sub-steps of 16.  The fragments of sub-step s+1 are read
// from LDS while the MFMAs of sub-step s run (register double buffer); the LDS writes of
// k-step i+1 and the global loads of k-step i+2 are slotted between the MFMAs of
// sub-steps 0 and 1; the last sub-step prefetches the first fragments of the next stage.
// One barrier per k-step.  The issue order inside a sub-step is pinned with
// sched_group_barrier, since with one wavefront per SIMD nothing else hides LDS latency.
//
// Persistent workgroups.  The grid is one workgroup per CU; each loops over output
// tiles.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so in
// every round the 32 workgroups of an XCD take 32 consecutive tiles, out-feature tile
// fastest: they share a token panel of u.  The next tile's first global loads are issued
// before the epilogue, and the epilogue's stores drain while the next tile is multiplied.
//
// Epilogue.  The accumulators are staged through LDS (free once the k loop is done) so
// that global memory is written in whole-row pieces, 16 bytes per lane, instead of 8-byte
// pieces scattered over 32 rows: bf16 store; GELU(tanh form) + bf16 store; gated residual
// update of the fp32 stream (x += gate_b * (acc + bias)), optionally also storing bf16(x).
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
  int tiles_m; int tiles_n; int group_w; int total_tiles; int rounds;
};

__device__ __forceinline__ float gelu_tanh_f(float u) {
  // 0.5 u (1 + tanh(z)) == u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3)
  const float kA = -2.0f * 0.7978845608028654f * 1.4426950408889634f;  // -2 sqrt(2/pi) log2(e)
  const float t = u * u;
  const float z2 = u * (kA + (kA * 0.044715f) * t);                    // -2 z log2(e)
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z2));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for the
// epilogue's global stores of the previous tile to be acknowledged, which is exactly the
// overlap the persistent loop is after; nothing in this kernel communicates through global
// memory inside a workgroup.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
#define SG_MFMA 0x008
#define SG_VMEM_RD 0x020
#define SG_DS_RD 0x100
#define SG_DS_WR 0x200

// Issue order for one sub-step: NM MFMAs with NS instructions of class OTHER spread between them.
template <int OTHER, int I, int NM, int NS>
__device__ __forceinline__ void sched_interleave() {
  if constexpr (I < NM) {
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
    constexpr int cnt = (I < NS % NM ? 1 : 0) + NS / NM;
    if constexpr (cnt > 0) __builtin_amdgcn_sched_group_barrier(OTHER, cnt, 0);
    sched_interleave<OTHER, I + 1, NM, NS>();
  }
}

// Order of the output tiles.  Tiles are enumerated in groups of `group_w` out-feature tiles and,
// inside a group, token-panel major; that sequence is cut into 8 contiguous parts, one per XCD
// (workgroups are dealt round-robin to the XCDs, each with its own L2), and in every round the
// workgroups of an XCD take the next consecutive tiles of its part.  An XCD therefore works for
// many rounds on the same few W tiles (they stay in its L2) while it streams token panels of u,
// each of which is shared by the group_w workgroups next to each other.
__device__ __forceinline__ int tile_sequence_index(const GemmParams &p, int round) {
  const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3, per = gridDim.x >> 3;
  const int q8 = p.total_tiles >> 3, r8 = p.total_tiles & 7;
  const int cnt = q8 + (xcd < r8 ? 1 : 0);
  const int idx = round * per + loc;
  if (idx >= cnt) return -1;
  return xcd * q8 + (xcd < r8 ? xcd : r8) + idx;
}
__device__ __forceinline__ void decode_tile(const GemmParams &p, int L, int &tile_m, int &tile_n) {
  const int gsz = p.tiles_m * p.group_w;
  int g = L / gsz;
  const int full = p.tiles_n / p.group_w;
  int bw = p.group_w;
  if (g >= full) { g = full; bw = p.tiles_n - full * p.group_w; }
  const int r = L - g * gsz;
  tile_m = r / bw;
  tile_n = g * p.group_w + (r - tile_m * bw);
}

template <int BM, int BN>
struct GemmCfg {
  static constexpr int STAGE = (BM + BN) * ROW_BYTES;
  static constexpr int PITCH_BF16 = BN * 2 + 16;             // epilogue staging row pitches: +16 B keeps the
  static constexpr int PITCH_F32 = BN * 4 + 16;              // 8 lanes of a 16-byte access on distinct banks
  static constexpr int EPI_BF16_BYTES = BM * PITCH_BF16;
  static constexpr int EPI_F32_BYTES = (BM / 2) * PITCH_F32;  // fp32 staging goes in two halves of BM/2 rows
  static constexpr int MAIN_BYTES = 2 * STAGE;
  static constexpr int SMEM = MAIN_BYTES > EPI_BF16_BYTES ? (MAIN_BYTES > EPI_F32_BYTES ? MAIN_BYTES : EPI_F32_BYTES)
                                                          : (EPI_BF16_BYTES > EPI_F32_BYTES ? EPI_BF16_BYTES : EPI_F32_BYTES);
};

// Epilogue of one output tile.  acc[a][b][4g+e] = C[token tb + l32][feature fb + 8g + 4 lh + e]
// (bias already inside).  The accumulators are staged through LDS (`smem`, free once the k loop is
// done; the caller guarantees no read of it is pending) so that global memory sees whole-row pieces.
// Ends with every thread past a barrier after its last read of the staging area when EPI == 2;
// for the bf16 epilogues the caller places that barrier before reusing `smem`.
template <int BM, int BN, int EPI>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[BN / 64][BM / 64], unsigned char *smem,
                                              const float *smem_gate, const GemmParams &p, int64_t my_row0,
                                              int my_col0, int64_t my_sample0, int tid, int wm, int wn, int l32,
                                              int lh) {
  using C = GemmCfg<BM, BN>;
  constexpr int TM = BM / 64;
  constexpr int TN = BN / 64;
  if constexpr (EPI != 2) {
    // bias (+ GELU), round to bf16, stage the whole BM x BN tile, then store whole rows
#pragma unroll
    for (int a = 0; a < TN; ++a) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int fl = wn * (BN / 2) + a * 32 + 8 * g + 4 * lh;   // feature inside the tile
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          float v0 = acc[a][b][4 * g + 0], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                v3 = acc[a][b][4 * g + 3];
          if (EPI == 1) {
            v0 = gelu_tanh_f(v0); v1 = gelu_tanh_f(v1); v2 = gelu_tanh_f(v2); v3 = gelu_tanh_f(v3);
          }
          bf16x4 o;
          o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
          const int rl = wm * (BM / 2) + b * 32 + l32;             // token inside the tile
          *reinterpret_cast<bf16x4 *>(smem + rl * C::PITCH_BF16 + fl * 2) = o;
        }
      }
    }
    lds_barrier();
    constexpr int CPR = BN / 8;   // 16-byte chunks per tile row
#pragma unroll 8
    for (int idx = tid; idx < BM * CPR; idx += 256) {
      const int rl = idx / CPR, c = idx - rl * CPR;
      const int64_t tok = my_row0 + rl;
      const int f = my_col0 + c * 8;
      if (tok < p.N && f < p.n)
        *reinterpret_cast<uint4 *>(p.out + tok * p.ld_out + f) =
            *reinterpret_cast<const uint4 *>(smem + rl * C::PITCH_BF16 + c * 16);
    }
  } else {
    // gated residual: the raw accumulators are staged in two halves of BM/2 rows (an fp32
    // tile does not fit LDS in one piece); bias, gate and the update of x happen on the way
    // out, on whole-row pieces
    constexpr int HB = TM / 2;        // token tiles per wave per half
    constexpr int HROWS = BM / 2;     // rows per half: wave-row wm owns HB*32 of them
    constexpr int CPR = BN / 4;       // float4 chunks per tile row
    const int64_t sample1_tok = (my_sample0 + 1) * p.tokens_per_sample;   // first token of the tile's second sample
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int bb = 0; bb < HB; ++bb) {
        const int b = half * HB + bb;
        const int rl = wm * (HB * 32) + bb * 32 + l32;             // row inside the half
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int fl = wn * (BN / 2) + a * 32 + 8 * g + 4 * lh;
            *reinterpret_cast<float4 *>(smem + rl * C::PITCH_F32 + fl * 4) =
                make_float4(acc[a][b][4 * g + 0], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]);
          }
      }
      lds_barrier();
      // Loads of x are batched ahead of the stores (the compiler must assume that a store to
      // the stream may alias a later load from it, so it would serialise them one by one).
      constexpr int ITERS = HROWS * CPR / 256;
      constexpr int UB = ITERS % 8 == 0 ? 8 : (ITERS % 6 == 0 ? 6 : (ITERS % 4 == 0 ? 4 : 1));
      static_assert(HROWS * CPR % 256 == 0, "row pieces must divide evenly over the threads");
#pragma unroll 1
      for (int it0 = 0; it0 < ITERS; it0 += UB) {
        float4 xr[UB];
        int64_t off[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int idx = tid + 256 * (it0 + u);
          const int rl = idx / CPR, c = idx - rl * CPR;
          const int wrow = rl / (HB * 32), within = rl - wrow * (HB * 32);
          const int64_t tok = my_row0 + wrow * (BM / 2) + half * (HB * 32) + within;
          const int f = my_col0 + c * 4;
          const bool ok = tok < p.N && f < p.n;
          off[u] = ok ? tok * (int64_t)p.n + f : -1;
          xr[u] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (ok) xr[u] = *reinterpret_cast<const float4 *>(p.resid + off[u]);
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          if (off[u] >= 0) {
            const int idx = tid + 256 * (it0 + u);
            const int rl = idx / CPR, c = idx - rl * CPR;
            const int wrow = rl / (HB * 32), within = rl - wrow * (HB * 32);
            const int64_t tok = my_row0 + wrow * (BM / 2) + half * (HB * 32) + within;
            const float4 v = *reinterpret_cast<const float4 *>(smem + rl * C::PITCH_F32 + c * 16);
            float4 gt = make_float4(1.f, 1.f, 1.f, 1.f);
            if (p.gate_tab) {
              const int64_t ds = tok - sample1_tok;   // >= 0: second sample of the tile (or beyond)
              if (ds < p.tokens_per_sample) {
                gt = *reinterpret_cast<const float4 *>(smem_gate + (ds >= 0 ? BN : 0) + c * 4);
              } else {   // a tile over more than two samples (tiny shapes only): fetch the gate directly
                const int f = my_col0 + c * 4;
                gt = *reinterpret_cast<const float4 *>(p.gate_tab + f);
                if (p.gate_c6) {
                  const float4 gc = *reinterpret_cast<const float4 *>(
                      p.gate_c6 + (tok / p.tokens_per_sample) * p.gate_c6_stride + f);
                  gt.x += gc.x; gt.y += gc.y; gt.z += gc.z; gt.w += gc.w;
                }
              }
            }
            float4 r = xr[u];
            r.x += v.x * gt.x; r.y += v.y * gt.y; r.z += v.z * gt.z; r.w += v.w * gt.w;
            *reinterpret_cast<float4 *>(p.resid + off[u]) = r;
            if (p.out) {
              bf16x4 o;
              o[0] = (bf16_t)r.x; o[1] = (bf16_t)r.y; o[2] = (bf16_t)r.z; o[3] = (bf16_t)r.w;
              *reinterpret_cast<bf16x4 *>(p.out + tok * p.ld_out + my_col0 + c * 4) = o;
            }
          }
        }
      }
      lds_barrier();   // the staging area is rewritten by the next half / the next tile's prologue
    }
  }
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmParams p) {
  using C = GemmCfg<BM, BN>;
  constexpr int TM = BM / 64;  // 32-token MFMA tiles per wave
  constexpr int TN = BN / 64;  // 32-feature MFMA tiles per wave
  constexpr int U_CH = BM * 8 / 256;  // 16-byte chunks per thread per stage
  constexpr int W_CH = BN * 8 / 256;
  constexpr int STAGE = C::STAGE;
  constexpr int NFRAG = TM + TN;
  constexpr int NMFMA = TM * TN;
  constexpr int NST = U_CH + W_CH;  // staging chunks per thread = ds_writes = global loads per k-step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int ld_r = tid >> 3, ld_c = tid & 7;  // staging: row ld_r (+32 per extra chunk), 16-byte chunk ld_c
  const bf16_t *u_base = p.u + ld_c * 8;
  const bf16_t *w_base = p.W + ld_c * 8;
  // LDS byte offset of this thread's staging chunk (row ld_r + 32 i keeps (row & 7) == (ld_r & 7))
  const int st_off = ld_r * ROW_BYTES + ((ld_c ^ (ld_r & 7)) << 4);
  // fragment read offsets: row (tile*32 + l32), chunk (2 kk + lh) swizzled by (row & 7) == (l32 & 7)
  const int frag_u = (wm * (BM / 2) + l32) * ROW_BYTES;
  const int frag_w = BM * ROW_BYTES + (wn * (BN / 2) + l32) * ROW_BYTES;
  int coff[BK / 16];
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) coff[kk] = ((kk * 2 + lh) ^ (l32 & 7)) << 4;
  const int nk = (p.k + BK - 1) / BK;
  const int n_steady = (p.k / BK) - 2;  // k-steps kt with kt+2 a full step

  auto tile_of = [&](int r) -> int {   // position in the tile sequence, or total_tiles when there is none
    const int t = tile_sequence_index(p, r);
    return t < 0 ? p.total_tiles : t;
  };

  int u_off[U_CH];   // element offsets; the host checks that they fit 31 bits
  int w_off[W_CH];
  uint4 u_reg[U_CH], w_reg[W_CH];
  // bias of this lane's out-features; the accumulators START from it (so no epilogue load)
  bf16x4 bias_r[TN][4];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int e = 0; e < 4; ++e) bias_r[a][g][e] = (bf16_t)0.f;

#define GEMM_SET_TILE(TILE)                                                                        \
  do {                                                                                             \
    int tile_m_, tile_n_;                                                                          \
    decode_tile(p, (TILE), tile_m_, tile_n_);                                                      \
    row0 = (int64_t)tile_m_ * BM;                                                                  \
    col0 = tile_n_ * BN;                                                                           \
    _Pragma("unroll") for (int i = 0; i < U_CH; ++i) {                                             \
      int64_t r_ = row0 + ld_r + 32 * i;                                                           \
      if (r_ > p.N - 1) r_ = p.N - 1; /* overhanging rows re-read the last row; never stored */    \
      u_off[i] = (int)(r_ * p.ld_u);                                                               \
    }                                                                                              \
    _Pragma("unroll") for (int i = 0; i < W_CH; ++i) {                                             \
      int r_ = col0 + ld_r + 32 * i;                                                               \
      if (r_ > p.n - 1) r_ = p.n - 1;                                                              \
      w_off[i] = r_ * p.k;                                                                         \
    }                                                                                              \
  } while (0)

  // Gate vectors of the tile's out-features for the (at most two) samples its rows belong to, kept
  // in LDS past the stages: slot 0 = sample of the tile's first row, slot 1 = the next sample.
  float4 gate_reg = make_float4(1.f, 1.f, 1.f, 1.f);
  float *smem_gate = reinterpret_cast<float *>(smem + C::SMEM);
  int64_t tile_sample0 = 0;      // sample of the first row of the tile whose gate is in gate_reg
#define GEMM_GATE_LOAD()                                                                           \
  do {                                                                                             \
    if (EPI == 2 && p.gate_tab) {                                                                  \
      tile_sample0 = row0 / p.tokens_per_sample;                                                   \
      if (tid < 2 * (BN / 4)) {                                                                    \
        const int which_ = tid / (BN / 4), c_ = tid - which_ * (BN / 4);                           \
        int f_ = col0 + 4 * c_;                                                                    \
        if (f_ > p.n - 4) f_ = p.n - 4;                                                            \
        gate_reg = *reinterpret_cast<const float4 *>(p.gate_tab + f_);                             \
        if (p.gate_c6) {                                                                           \
          int64_t smp_ = tile_sample0 + which_;                                                    \
          const int64_t last_ = (p.N - 1) / p.tokens_per_sample;                                   \
          if (smp_ > last_) smp_ = last_;                                                          \
          const float4 gc_ = *reinterpret_cast<const float4 *>(p.gate_c6 + smp_ * p.gate_c6_stride + f_); \
          gate_reg.x += gc_.x; gate_reg.y += gc_.y; gate_reg.z += gc_.z; gate_reg.w += gc_.w;      \
        }                                                                                          \
      }                                                                                            \
    }                                                                                              \
  } while (0)

#define GEMM_BIAS_LOAD()                                                                           \
  do {                                                                                             \
    if (p.bias) {                                                                                  \
      _Pragma("unroll") for (int a = 0; a < TN; ++a)                                               \
          _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                          \
        int f_ = col0 + wn * (BN / 2) + a * 32 + 8 * g + 4 * lh;                                   \
        if (f_ > p.n - 4) f_ = p.n - 4; /* overhanging features: a valid address, never stored */  \
        bias_r[a][g] = *reinterpret_cast<const bf16x4 *>(p.bias + f_);                             \
      }                                                                                            \
    }                                                                                              \
  } while (0)

#define GEMM_G_LOAD(K0)                                                                            \
  do {                                                                                             \
    const int k0_ = (K0);                                                                          \
    if (k0_ + ld_c * 8 < p.k) {                                                                    \
      _Pragma("unroll") for (int i = 0; i < U_CH; ++i)                                             \
          u_reg[i] = *reinterpret_cast<const uint4 *>(u_base + u_off[i] + k0_);                    \
      _Pragma("unroll") for (int i = 0; i < W_CH; ++i)                                             \
          w_reg[i] = *reinterpret_cast<const uint4 *>(w_base + w_off[i] + k0_);                    \
    } else { /* k tail: zero-fill both operands */                                                 \
      _Pragma("unroll") for (int i = 0; i < U_CH; ++i) u_reg[i] = make_uint4(0u, 0u, 0u, 0u);      \
      _Pragma("unroll") for (int i = 0; i < W_CH; ++i) w_reg[i] = make_uint4(0u, 0u, 0u, 0u);      \
    }                                                                                              \
  } while (0)

#define GEMM_G_LOAD_FULL(K0)                                                                       \
  do {                                                                                             \
    const int k0_ = (K0);                                                                          \
    _Pragma("unroll") for (int i = 0; i < U_CH; ++i)                                               \
        u_reg[i] = *reinterpret_cast<const uint4 *>(u_base + u_off[i] + k0_);                      \
    _Pragma("unroll") for (int i = 0; i < W_CH; ++i)                                               \
        w_reg[i] = *reinterpret_cast<const uint4 *>(w_base + w_off[i] + k0_);                      \
  } while (0)

#define GEMM_S_STORE(STAGE_IDX)                                                                    \
  do {                                                                                             \
    unsigned char *su_ = smem + (STAGE_IDX) * STAGE + st_off;                                      \
    unsigned char *sw_ = su_ + BM * ROW_BYTES;                                                     \
    _Pragma("unroll") for (int i = 0; i < U_CH; ++i)                                               \
        *reinterpret_cast<uint4 *>(su_ + i * 32 * ROW_BYTES) = u_reg[i];                           \
    _Pragma("unroll") for (int i = 0; i < W_CH; ++i)                                               \
        *reinterpret_cast<uint4 *>(sw_ + i * 32 * ROW_BYTES) = w_reg[i];                           \
  } while (0)

#define GEMM_READ_FRAGS(BUF, STAGE_IDX, KK)                                                        \
  do {                                                                                             \
    const unsigned char *sb_ = smem + (STAGE_IDX) * STAGE + coff[KK];                              \
    _Pragma("unroll") for (int b = 0; b < TM; ++b)                                                 \
        uf[BUF][b] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_u + b * 32 * ROW_BYTES);         \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        wf[BUF][a] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_w + a * 32 * ROW_BYTES);         \
  } while (0)

#define GEMM_MFMAS(BUF)                                                                            \
  do {                                                                                             \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        _Pragma("unroll") for (int b = 0; b < TM; ++b)                                             \
            acc[a][b] = mfma32(wf[BUF][a], uf[BUF][b], acc[a][b]);                                 \
  } while (0)

  int64_t row0 = 0;
  int col0 = 0;
  int tile = tile_of(0);
  if (tile >= p.total_tiles) return;
  GEMM_SET_TILE(tile);
  GEMM_BIAS_LOAD();
  GEMM_GATE_LOAD();
  GEMM_G_LOAD(0);

  for (int round = 0;; ++round) {
    // ---- prologue: the registers hold k-step 0 of this tile
    const int64_t my_row0 = row0;
    const int my_col0 = col0;
    const int64_t my_sample0 = tile_sample0;
    GEMM_S_STORE(0);
    if (EPI == 2 && tid < 2 * (BN / 4)) *reinterpret_cast<float4 *>(smem_gate + tid * 4) = gate_reg;
    if (nk > 1) GEMM_G_LOAD(BK);
    floatx16 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
      for (int b = 0; b < TM; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][b][e] = (float)bias_r[a][e >> 2][e & 3];
    lds_barrier();

    bf16x8 uf[2][TM], wf[2][TN];
    GEMM_READ_FRAGS(0, 0, 0);
    int kt = 0;
    // ---- steady state: k-steps kt+1 and kt+2 exist and kt+2 is a full step; no branches inside,
    // so each sub-step is one scheduling region with an explicit issue order
    for (; kt < n_steady; ++kt) {
      const int cur = kt & 1;
      // sub-step 0: stage k-step kt+1 into the other buffer
      GEMM_READ_FRAGS(1, cur, 1);
      GEMM_S_STORE(cur ^ 1);
      GEMM_MFMAS(0);
      __builtin_amdgcn_sched_group_barrier(SG_DS_RD, NFRAG, 0);
      sched_interleave<SG_DS_WR, 0, NMFMA, NST>();
      __builtin_amdgcn_sched_barrier(0);
      // sub-step 1: issue the global loads of k-step kt+2
      GEMM_READ_FRAGS(0, cur, 2);
      GEMM_G_LOAD_FULL((kt + 2) * BK);
      GEMM_MFMAS(1);
      __builtin_amdgcn_sched_group_barrier(SG_DS_RD, NFRAG, 0);
      sched_interleave<SG_VMEM_RD, 0, NMFMA, NST>();
      __builtin_amdgcn_sched_barrier(0);
      // sub-step 2
      GEMM_READ_FRAGS(1, cur, 3);
      __builtin_amdgcn_sched_barrier(0);
      GEMM_MFMAS(0);
      __builtin_amdgcn_sched_barrier(0);
      // Past this barrier every wave's last read of the current stage has returned and its
      // writes of the next stage are done: the next stage may be read, and the following
      // k-step may overwrite the current one.
      lds_barrier();
      // sub-step 3: first fragments of the next stage
      GEMM_READ_FRAGS(0, cur ^ 1, 0);
      __builtin_amdgcn_sched_barrier(0);
      GEMM_MFMAS(1);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- the last k-steps (and the k tail, zero-filled)
    for (; kt < nk; ++kt) {
      const int cur = kt & 1;
      const bool has_next = kt + 1 < nk;
      if (has_next) GEMM_S_STORE(cur ^ 1);
      GEMM_READ_FRAGS(1, cur, 1);
      GEMM_MFMAS(0);
      if (kt + 2 < nk) GEMM_G_LOAD((kt + 2) * BK);
      GEMM_READ_FRAGS(0, cur, 2);
      GEMM_MFMAS(1);
      GEMM_READ_FRAGS(1, cur, 3);
      GEMM_MFMAS(0);
      lds_barrier();
      if (has_next) GEMM_READ_FRAGS(0, cur ^ 1, 0);
      GEMM_MFMAS(1);
    }
    // every wave is past the last barrier of the k loop: no LDS read of the stages is pending

    // ---- epilogue.  acc[a][b][4g+e] = C[token tb + l32][feature fb + 8g + 4 lh + e]
    // ---- next tile: start its first global loads now, they land during the epilogue
    const int next_tile = (round + 1 < p.rounds) ? tile_of(round + 1) : p.total_tiles;
    const bool more = next_tile < p.total_tiles;
    if (more) {
      GEMM_SET_TILE(next_tile);
      GEMM_BIAS_LOAD();
      GEMM_GATE_LOAD();
      GEMM_G_LOAD(0);
    }

    gemm_epilogue<BM, BN, EPI>(acc, smem, smem_gate, p, my_row0, my_col0, my_sample0, tid, wm, wn, l32, lh);
    if (!more) break;
    if constexpr (EPI != 2) lds_barrier();   // staged rows are read by other waves until here
    tile = next_tile;
  }
#undef GEMM_SET_TILE
#undef GEMM_BIAS_LOAD
#undef GEMM_GATE_LOAD
#undef GEMM_G_LOAD
#undef GEMM_G_LOAD_FULL
#undef GEMM_S_STORE
#undef GEMM_READ_FRAGS
#undef GEMM_MFMAS
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS variant (k a multiple of 32).  Operand tiles go global -> LDS with 16-byte
// global_load_lds: no staging registers, no ds_write, and the loads of k-step i+3 are in flight
// while k-step i is multiplied (four LDS stages of (BM+BN) rows x 64 B).  A wave-wide load places
// lane l's piece at LDS base + 16 l, i.e. 16 consecutive 64-byte rows; the XOR swizzle that keeps
// the fragment reads conflict-free (chunk slot = chunk ^ ((row >> 1) & 3)) is therefore applied
// to the GLOBAL address each lane fetches from.  Completion is tracked with the vector-memory
// counter, which retires in order: before the barrier of k-step i each wave waits until at most
// the loads of k-steps i+2 and i+3 are outstanding, so past the barrier stage i+1 is complete.
// ---------------------------------------------------------------------------------------------
constexpr int DL_BK = 32;
constexpr int DL_ROW = 64;   // bytes per LDS row
constexpr int DL_NS = 4;     // stages

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(1))) const void *gbl_ptr_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if constexpr (N == 7) asm volatile("s_waitcnt vmcnt(7)" ::: "memory");
  else if constexpr (N == 14) asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
  else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else static_assert(N == 0, "unsupported count");
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void k_gemm_dl(GemmParams p) {
  using C = GemmCfg<BM, BN>;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int STAGE = (BM + BN) * DL_ROW;
  constexpr int NI = (BM + BN) / 16;   // wave-wide loads per k-step (16 rows each)
  constexpr int NJ = NI / 4;           // per wave
  constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
  static_assert(NI % 4 == 0, "loads must divide over the four waves");
  static_assert(DL_NS * STAGE <= C::SMEM, "stages must fit the shared allocation");
  static_assert(NJ == 7 || NJ == 4, "wait_vmcnt covers these counts");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *smem_gate = reinterpret_cast<float *>(smem + C::SMEM);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int nk = p.k / DL_BK;

  // fragment reads: row (tile*32 + l32) of 64 B, chunk (2 kk + lh) at slot chunk ^ ((row >> 1) & 3)
  const int frag_u = (wm * (BM / 2) + l32) * DL_ROW;
  const int frag_w = BM * DL_ROW + (wn * (BN / 2) + l32) * DL_ROW;
  int coff[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) coff[kk] = ((kk * 2 + lh) ^ ((l32 >> 1) & 3)) << 4;
  // loads: instruction g = wave*NJ + j covers tile rows 16 g .. 16 g + 15; this lane: row lane/4, slot lane%4
  const int ld_row = lane >> 2;
  const int ld_chunk = ((lane & 3) ^ ((ld_row >> 1) & 3)) * 8;   // element offset of the global chunk to fetch

  int src_off[NJ];   // element offset of this lane's piece at k = 0 (u or W, by instruction)

#define DL_ISSUE(KT)                                                                               \
  do {                                                                                             \
    const int k0_ = (KT) * DL_BK;                                                                  \
    unsigned char *sb_ = smem + ((KT) & (DL_NS - 1)) * STAGE + wave * NJ * 1024;                   \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                               \
      const bf16_t *src_ = ((wave * NJ + j) * 16 < BM ? p.u : p.W) + src_off[j] + k0_;             \
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src_, (lds_ptr_t)(sb_ + j * 1024), 16, 0, 0);    \
    }                                                                                              \
  } while (0)

#define DL_READ_FRAGS(BUF, KT, KK)                                                                 \
  do {                                                                                             \
    const unsigned char *sb_ = smem + ((KT) & (DL_NS - 1)) * STAGE + coff[KK];                     \
    _Pragma("unroll") for (int b = 0; b < TM; ++b)                                                 \
        uf[BUF][b] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_u + b * 32 * DL_ROW);            \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        wf[BUF][a] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_w + a * 32 * DL_ROW);            \
  } while (0)

#define DL_MFMAS(BUF)                                                                              \
  do {                                                                                             \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        _Pragma("unroll") for (int b = 0; b < TM; ++b)                                             \
            acc[a][b] = mfma32(wf[BUF][a], uf[BUF][b], acc[a][b]);                                 \
  } while (0)

  for (int round = 0; round < p.rounds; ++round) {
    const int tile = tile_sequence_index(p, round);
    if (tile < 0) break;
    int tile_m, tile_n;
    decode_tile(p, tile, tile_m, tile_n);
    const int64_t row0 = (int64_t)tile_m * BM;
    const int col0 = tile_n * BN;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int R = (wave * NJ + j) * 16 + ld_row;
      if (R < BM) {
        int64_t t = row0 + R;
        if (t > p.N - 1) t = p.N - 1;           // overhanging rows re-read the last row; never stored
        src_off[j] = (int)(t * p.ld_u) + ld_chunk;
      } else {
        int f = col0 + R - BM;
        if (f > p.n - 1) f = p.n - 1;
        src_off[j] = f * p.k + ld_chunk;
      }
    }
    // bias and gate first: the memory counter retires in order, so what is needed first is issued first
    bf16x4 bias_r[TN][4];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) bias_r[a][g][e] = (bf16_t)0.f;
        if (p.bias) {
          int f = col0 + wn * (BN / 2) + a * 32 + 8 * g + 4 * lh;
          if (f > p.n - 4) f = p.n - 4;
          bias_r[a][g] = *reinterpret_cast<const bf16x4 *>(p.bias + f);
        }
      }
    int64_t sample0 = 0;
    if (EPI == 2 && p.gate_tab) {
      sample0 = row0 / p.tokens_per_sample;
      if (tid < 2 * (BN / 4)) {
        const int which = tid / (BN / 4), c = tid - which * (BN / 4);
        int f = col0 + 4 * c;
        if (f > p.n - 4) f = p.n - 4;
        float4 gt = *reinterpret_cast<const float4 *>(p.gate_tab + f);
        if (p.gate_c6) {
          int64_t smp = sample0 + which;
          const int64_t last = (p.N - 1) / p.tokens_per_sample;
          if (smp > last) smp = last;
          const float4 gc = *reinterpret_cast<const float4 *>(p.gate_c6 + smp * p.gate_c6_stride + f);
          gt.x += gc.x; gt.y += gc.y; gt.z += gc.z; gt.w += gc.w;
        }
        *reinterpret_cast<float4 *>(smem_gate + tid * 4) = gt;
      }
    }
    DL_ISSUE(0);
    if (nk > 1) DL_ISSUE(1);
    if (nk > 2) DL_ISSUE(2);

    floatx16 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
      for (int b = 0; b < TM; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][b][e] = (float)bias_r[a][e >> 2][e & 3];

    if (nk > 2) wait_vmcnt<2 * NJ>();
    else if (nk > 1) wait_vmcnt<NJ>();
    else wait_vmcnt<0>();
    lds_barrier();

    bf16x8 uf[2][TM], wf[2][TN];
    DL_READ_FRAGS(0, 0, 0);
    int kt = 0;
    // ---- steady state: k-steps kt+1 .. kt+3 exist; no branches, issue order pinned
    for (; kt + 3 < nk; ++kt) {
      DL_READ_FRAGS(1, kt, 1);
      DL_ISSUE(kt + 3);
      DL_MFMAS(0);
      __builtin_amdgcn_sched_group_barrier(SG_DS_RD, NFRAG, 0);
      sched_interleave<SG_VMEM_RD, 0, NMFMA, NJ>();
      __builtin_amdgcn_sched_barrier(0);
      wait_vmcnt<2 * NJ>();   // k-step kt+1 has landed (this wave's part)
      lds_barrier();          // ... everyone's part; and every wave is done reading stage kt
      DL_READ_FRAGS(0, kt + 1, 0);
      __builtin_amdgcn_sched_barrier(0);
      DL_MFMAS(1);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- last k-steps
    for (; kt < nk; ++kt) {
      DL_READ_FRAGS(1, kt, 1);
      DL_MFMAS(0);
      if (kt + 2 < nk) wait_vmcnt<NJ>();
      else wait_vmcnt<0>();
      lds_barrier();
      if (kt + 1 < nk) DL_READ_FRAGS(0, kt + 1, 0);
      DL_MFMAS(1);
    }
    // every wave is past the last barrier of the k loop: no LDS read of the stages is pending
    gemm_epilogue<BM, BN, EPI>(acc, smem, smem_gate, p, row0, col0, sample0, tid, wm, wn, l32, lh);
    if constexpr (EPI != 2) lds_barrier();   // staged rows are read by other waves until here
  }
#undef DL_ISSUE
#undef DL_READ_FRAGS
#undef DL_MFMAS
}

int num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

template <int BM, int BN, int EPI, bool DIRECT>
int launch_one(const GemmParams &p0, hipStream_t s) {
  using C = GemmCfg<BM, BN>;
  GemmParams p = p0;
  const int64_t tiles_m = (p.N + BM - 1) / BM;
  p.tiles_m = (int)tiles_m;
  p.tiles_n = (p.n + BN - 1) / BN;
  // width of an out-feature group: at most 8 tiles, as even as the tile count allows
  const int n_groups = (p.tiles_n + 7) / 8;
  p.group_w = (p.tiles_n + n_groups - 1) / n_groups;
  const int64_t total = tiles_m * p.tiles_n;
  if (total > (int64_t)1 << 30) {
    ddit::set_error("linear: %lld output tiles: too many", (long long)total);
    return -2;
  }
  p.total_tiles = (int)total;
  // one workgroup per CU (the LDS stages leave room for one); a multiple of 8 so that every
  // round gives each XCD a contiguous run of tiles
  int grid = num_cus() & ~7;
  if (grid < 8) grid = 8;
  if (total <= grid) grid = (int)((total + 7) & ~(int64_t)7);
  p.rounds = (int)(((total + 7) / 8 + grid / 8 - 1) / (grid / 8));
  static bool attr_set = false;  // benign race: the attribute is idempotent
  if (!attr_set) {
    const void *fn = DIRECT ? reinterpret_cast<const void *>(&k_gemm_dl<BM, BN, EPI>)
                            : reinterpret_cast<const void *>(&k_gemm_bf16<BM, BN, EPI>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM + 2 * BN * 4);
    if (e != hipSuccess) return ddit::hip_fail(e, "gemm hipFuncSetAttribute");
    attr_set = true;
  }
  if (DIRECT)
    hipLaunchKernelGGL((k_gemm_dl<BM, BN, EPI>), dim3((unsigned)grid), dim3(256), C::SMEM + 2 * BN * 4, s, p);
  else
    hipLaunchKernelGGL((k_gemm_bf16<BM, BN, EPI>), dim3((unsigned)grid), dim3(256), C::SMEM + 2 * BN * 4, s, p);
  return ddit::hip_fail(hipGetLastError(), "gemm launch");
}

template <int EPI>
int launch_epi(const GemmParams &p, hipStream_t s) {
  // 192-wide feature tiles divide 1152, 3456, 4608 and 2304 exactly; narrow outputs and
  // short token counts take the smaller tile so more than a handful of CUs get work.
  const int64_t big_tiles = ((p.N + 255) / 256) * ((p.n + 191) / 192);
  const bool big = big_tiles >= 128 && (p.n % 192 == 0 || p.n > 1024);
  // the direct-to-LDS kernel cannot zero-fill a k tail
  if (p.k % DL_BK == 0) return big ? launch_one<256, 192, EPI, true>(p, s) : launch_one<128, 128, EPI, true>(p, s);
  return big ? launch_one<256, 192, EPI, false>(p, s) : launch_one<128, 128, EPI, false>(p, s);
}

}  // namespace

namespace ddit {

int launch_gemm(int epilogue, const GemmArgs &a, hipStream_t s) {
  if (a.N == 0 || a.n == 0) return 0;
  if ((int64_t)a.n * a.k >= (int64_t)1 << 31) {
    set_error("linear: n*k = %lld exceeds the 32-bit weight index range", (long long)a.n * a.k);
    return -2;
  }
  if (a.N * a.ld_u >= (int64_t)1 << 31) {
    set_error("linear: N*ld_u = %lld exceeds the 31-bit activation index range", (long long)(a.N * a.ld_u));
    return -2;
  }
  GemmParams p;
  p.u = reinterpret_cast<const bf16_t *>(a.u); p.ld_u = a.ld_u;
  p.W = reinterpret_cast<const bf16_t *>(a.W);
  p.bias = reinterpret_cast<const bf16_t *>(a.bias);
  p.N = a.N; p.n = a.n; p.k = a.k;
  p.out = reinterpret_cast<bf16_t *>(a.out); p.ld_out = a.ld_out;
  p.resid = a.resid;
  p.gate_tab = a.gate_tab; p.gate_c6 = a.gate_c6; p.gate_c6_stride = a.gate_c6_stride;
  p.tokens_per_sample = a.tokens_per_sample > 0 ? a.tokens_per_sample : 1;
  p.tiles_m = 0; p.tiles_n = 0; p.group_w = 1; p.total_tiles = 0; p.rounds = 0;
  switch (epilogue) {
    case 0: return launch_epi<0>(p, s);
    case 1: return launch_epi<1>(p, s);
    case 2: return launch_epi<2>(p, s);
  }
  set_error("unknown epilogue %d", epilogue);
  return -1;
}

}  // namespace ddit
