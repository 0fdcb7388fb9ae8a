// Exact softmax attention  O = softmax(Q K^T / sqrt(dh)) V  without ever forming the
// score matrix in memory: K/V are streamed through LDS in tiles of 64 keys and the
// softmax is carried online (running row maximum and running sum).
//
// One kernel serves the three attention kinds of the spatial-temporal DiT; they differ
// only in which tokens form a sequence, which the host expresses as strides:
//   spatial  - group = (b,t): the S tokens of one frame, consecutive rows
//   cross    - group = b: the L video tokens query the (valid prefix of the) text tokens
//   temporal - group = (b,s): T rows a frame apart (generic fallback; the dedicated
//              kernel in temporal_attn.hip is the fast path for short T)
//
// Work split.  grid = (query tiles of 128, heads, groups); 4 wavefronts per workgroup,
// each owning 32 queries against all keys of the group.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-wide wavefronts).  Scores are
// computed transposed, S^T = K Q^T: the K tile is the first operand (read from LDS, 16
// bytes per lane), the wave's Q fragment the second (held in registers for the whole
// kernel).  In the result layout a lane owns ONE query (column l%32) and 16 of every 32
// keys, so the row maximum is a register reduction plus one exchange with lane l^32.
// The probabilities P^T, rounded to bf16, are then already laid out as the second
// operand of O^T = V^T P^T, provided V^T's key axis is enumerated in the same order:
// V is transposed on its way into LDS (two keys packed per 32-bit write) with the keys
// of each group of 16 stored in the order the accumulator registers enumerate them.
// The head dim 72 is padded to 80 for Q K^T (zeros in LDS, never in HBM) and to 96 rows
// for V^T; one of the spare V^T rows is set to 1 so that the same MFMAs that form O also
// accumulate the softmax denominator (of the bf16-rounded probabilities actually used).
//
// LDS rows are padded by 16 bytes (K: 176 B, V^T: 144 B) so that a 16-byte read of 8
// consecutive rows covers all 32 banks once.  Two stages; the next tile's global loads
// are in flight during the current tile's MFMAs; one barrier per tile.
#include "ddit_common.hpp"

namespace {

constexpr int QT = 128;   // queries per workgroup
constexpr int KT = 64;    // keys per LDS tile

struct FlashParams {
  const bf16_t *q, *k, *v;
  bf16_t *o;
  float *lse;
  int64_t ld_q, ld_kv, ld_o;
  int g_inner;
  int64_t q_outer, q_inner, kv_outer, kv_inner;
  int64_t q_tok_step, kv_tok_step;
  int Lq, Lk_max, H;
  int use_kv_len;
  int kv_len[64];
  float scale_log2;  // log2(e) / sqrt(dh)
  float scale;       // 1 / sqrt(dh)
};

template <int DH>
struct Cfg {
  static constexpr int KS = (DH + 15) / 16;        // k-steps of Q K^T
  static constexpr int DCH = DH / 8;               // 16-byte chunks per row in HBM
  static constexpr int KROW = KS * 32 + 16;        // K row stride in LDS (bytes)
  static constexpr bool ONES = (DH % 32) != 0;     // a spare V^T row exists for the row sum
  static constexpr int DT = (DH + 31) / 32;        // 32-row tiles of V^T
  static constexpr int VROW = KT * 2 + 16;         // V^T row stride (bytes)
  static constexpr int K_BYTES = KT * KROW;
  static constexpr int V_BYTES = DT * 32 * VROW;
  static constexpr int STAGE = K_BYTES + V_BYTES;
};

// position of key offset o (0..15) inside its group of 16 in the V^T rows:
// o = 8 g + 4 h + e  ->  8 h + 4 g + e   (h: lane half, g: accumulator group parity)
__device__ __forceinline__ int key_pos16(int o) { return ((o & 4) << 1) | ((o & 8) >> 1) | (o & 3); }

template <int DH>
__global__ __launch_bounds__(256) void k_flash_attn(FlashParams p) {
  using C = Cfg<DH>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int h = blockIdx.y, g = blockIdx.z;
  const int g_out = g / p.g_inner, g_in = g - g_out * p.g_inner;
  const int Lk = p.use_kv_len ? p.kv_len[g_out] : p.Lk_max;
  const int64_t q_tok0 = p.q_outer * g_out + p.q_inner * g_in;
  const int64_t kv_tok0 = p.kv_outer * g_out + p.kv_inner * g_in;
  const int q0 = blockIdx.x * QT + wave * 32;

  // ---- Q fragment: lane holds query l32, d = 16 ks + 8 lh .. +7
  bf16x8 qf[C::KS];
  {
    int qi = q0 + l32;
    if (qi > p.Lq - 1) qi = p.Lq - 1;
    const bf16_t *qrow = p.q + (q_tok0 + (int64_t)qi * p.q_tok_step) * p.ld_q + h * DH;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int d0 = 16 * ks + 8 * lh;
      if (d0 < DH) {
        qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + d0);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16_t)0.f;
      }
    }
  }

  // ---- zero the padding of both stages once (K chunk DH/8.., V^T rows DH..), set the ones row
  for (int i = tid; i < 2 * KT; i += 256) {
    unsigned char *kr = smem + (i / KT) * C::STAGE + (i % KT) * C::KROW;
    for (int c = C::DCH; c < C::KS * 2; ++c) *reinterpret_cast<uint4 *>(kr + c * 16) = make_uint4(0, 0, 0, 0);
  }
  if constexpr (C::DT * 32 > DH) {
    constexpr int PER_STAGE = (C::DT * 32 - DH) * (KT / 2);   // 32-bit words of V^T padding
    for (int i = tid; i < 2 * PER_STAGE; i += 256) {
      const int st = i / PER_STAGE, rem = i % PER_STAGE;
      const int row = DH + rem / (KT / 2), w = rem % (KT / 2);
      const uint32_t val = (C::ONES && row == DH) ? 0x3F803F80u : 0u;  // bf16 1.0 twice
      *reinterpret_cast<uint32_t *>(smem + st * C::STAGE + C::K_BYTES + row * C::VROW + w * 4) = val;
    }
  }

  // ---- global -> register staging of one K/V tile
  constexpr int K_TASKS = KT * C::DCH;            // 16-byte chunks of K
  constexpr int V_TASKS = (KT / 2) * C::DCH;      // key pairs x chunks
  constexpr int K_PER = (K_TASKS + 255) / 256;
  constexpr int V_PER = (V_TASKS + 255) / 256;
  uint4 k_reg[K_PER], v_reg[V_PER][2];

  auto g_load = [&](int key0) {
#pragma unroll
    for (int i = 0; i < K_PER; ++i) {
      const int t = tid + 256 * i;
      if (t < K_TASKS) {
        int key = key0 + t / C::DCH;
        if (key > Lk - 1) key = Lk - 1;   // tail keys re-read the last valid key; masked below
        k_reg[i] = *reinterpret_cast<const uint4 *>(p.k + (kv_tok0 + (int64_t)key * p.kv_tok_step) * p.ld_kv +
                                                    h * DH + (t % C::DCH) * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < V_PER; ++i) {
      const int t = tid + 256 * i;
      if (t < V_TASKS) {
        const int kp = t % (KT / 2), dc = t / (KT / 2);
        int key_a = key0 + 2 * kp, key_b = key_a + 1;
        if (key_a > Lk - 1) key_a = Lk - 1;
        if (key_b > Lk - 1) key_b = Lk - 1;
        v_reg[i][0] = *reinterpret_cast<const uint4 *>(p.v + (kv_tok0 + (int64_t)key_a * p.kv_tok_step) * p.ld_kv +
                                                       h * DH + dc * 8);
        v_reg[i][1] = *reinterpret_cast<const uint4 *>(p.v + (kv_tok0 + (int64_t)key_b * p.kv_tok_step) * p.ld_kv +
                                                       h * DH + dc * 8);
      }
    }
  };
  auto s_store = [&](int stage) {
    unsigned char *sk = smem + stage * C::STAGE;
    unsigned char *sv = sk + C::K_BYTES;
#pragma unroll
    for (int i = 0; i < K_PER; ++i) {
      const int t = tid + 256 * i;
      if (t < K_TASKS) *reinterpret_cast<uint4 *>(sk + (t / C::DCH) * C::KROW + (t % C::DCH) * 16) = k_reg[i];
    }
#pragma unroll
    for (int i = 0; i < V_PER; ++i) {
      const int t = tid + 256 * i;
      if (t < V_TASKS) {
        const int kp = t % (KT / 2), dc = t / (KT / 2);
        const int ko = 2 * kp;                                   // even key offset in the tile
        const int pos = (ko & ~15) | key_pos16(ko & 15);         // even: the pair stays adjacent
        const uint32_t a[4] = {v_reg[i][0].x, v_reg[i][0].y, v_reg[i][0].z, v_reg[i][0].w};
        const uint32_t b[4] = {v_reg[i][1].x, v_reg[i][1].y, v_reg[i][1].z, v_reg[i][1].w};
        unsigned char *dst = sv + (dc * 8) * C::VROW + pos * 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          // d = 8 dc + 2j: low halves; d = 8 dc + 2j + 1: high halves
          *reinterpret_cast<uint32_t *>(dst + (2 * j) * C::VROW) = (a[j] & 0xFFFFu) | (b[j] << 16);
          *reinterpret_cast<uint32_t *>(dst + (2 * j + 1) * C::VROW) = (a[j] >> 16) | (b[j] & 0xFFFF0000u);
        }
      }
    }
  };

  floatx16 oacc[C::DT];
#pragma unroll
  for (int d = 0; d < C::DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
  float m_run = -INFINITY;   // running maximum of the raw (unscaled) scores of this lane's query
  float l_run = 0.f;         // running sum (only used when there is no ones row)

  const int n_tiles = (Lk + KT - 1) / KT;
  g_load(0);
  __syncthreads();           // padding writes done before tile data lands next to them
  s_store(0);
  if (n_tiles > 1) g_load(KT);
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const int cur = it & 1;
    const unsigned char *sk = smem + cur * C::STAGE;
    const unsigned char *sv = sk + C::K_BYTES;

    // ---- S^T = K Q^T for the 64 keys of this tile
    floatx16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[kt][e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(sk + (kt * 32 + l32) * C::KROW + (2 * ks + lh) * 16);
        s[kt] = mfma32(kf, qf[ks], s[kt]);
      }
    }
    // ---- mask the keys past the end (last tile only)
    const int key0 = it * KT;
    if (key0 + KT > Lk) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (key >= Lk) s[kt][r] = -INFINITY;
        }
    }
    // ---- online softmax for this lane's query
    float mx = s[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2);
    const float mb = m_new * p.scale_log2;
    m_run = m_new;
    bf16x8 pf[4];
    float psum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = __builtin_amdgcn_exp2f(s[kt][r] * p.scale_log2 - mb);
        const bf16_t pb = (bf16_t)pv;
        pf[kt * 2 + (r >> 3)][r & 7] = pb;
        if (!C::ONES) psum += (float)pb;
      }
#pragma unroll
    for (int d = 0; d < C::DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[d][e] *= alpha;
    if (!C::ONES) l_run = l_run * alpha + psum;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
#pragma unroll
      for (int d = 0; d < C::DT; ++d) {
        const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(sv + (d * 32 + l32) * C::VROW + (2 * kc + lh) * 16);
        oacc[d] = mfma32(vf, pf[kc], oacc[d]);
      }
    }

    if (it + 1 < n_tiles) s_store(cur ^ 1);
    if (it + 2 < n_tiles) g_load((it + 2) * KT);
    __syncthreads();
  }

  // ---- row sum
  float l_tot;
  if (C::ONES) {
    // V^T row DH lives in tile DH/32, accumulator register 4*((DH%32)/8) of the lanes with lh == 0
    constexpr int dt = DH / 32, reg = 4 * ((DH % 32) / 8);
    l_tot = __shfl(oacc[dt][reg], l32, 64);
  } else {
    l_tot = l_run + __shfl_xor(l_run, 32, 64);
  }
  const float inv = 1.0f / l_tot;
  const int qi = q0 + l32;
  if (qi < p.Lq) {
    const int64_t tok = q_tok0 + (int64_t)qi * p.q_tok_step;
    bf16_t *orow = p.o + tok * p.ld_o + h * DH;
#pragma unroll
    for (int d = 0; d < C::DT; ++d)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const int d0 = 32 * d + 8 * gq + 4 * lh;
        if (d0 < DH) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[d][4 * gq + e] * inv);
          *reinterpret_cast<bf16x4 *>(orow + d0) = ov;
        }
      }
    if (p.lse && lh == 0) p.lse[tok * p.H + h] = m_run * p.scale + __logf(l_tot);
  }
}

template <int DH>
int launch_dh(const FlashParams &p, int n_groups, hipStream_t s) {
  using C = Cfg<DH>;
  constexpr int smem = 2 * C::STAGE;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_flash_attn<DH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return ddit::hip_fail(e, "flash hipFuncSetAttribute");
    attr_set = true;
  }
  dim3 grid((unsigned)((p.Lq + QT - 1) / QT), (unsigned)p.H, (unsigned)n_groups);
  hipLaunchKernelGGL(k_flash_attn<DH>, grid, dim3(256), smem, s, p);
  return ddit::hip_fail(hipGetLastError(), "flash attention launch");
}

}  // namespace

namespace ddit {

int launch_flash_attn(const AttnArgs &a, hipStream_t s) {
  if (a.n_groups == 0 || a.Lq == 0) return 0;
  FlashParams p;
  p.q = reinterpret_cast<const bf16_t *>(a.q);
  p.k = reinterpret_cast<const bf16_t *>(a.k);
  p.v = reinterpret_cast<const bf16_t *>(a.v);
  p.o = reinterpret_cast<bf16_t *>(a.o);
  p.lse = a.lse;
  p.ld_q = a.ld_q; p.ld_kv = a.ld_kv; p.ld_o = a.ld_o;
  p.g_inner = a.g_inner;
  p.q_outer = a.q_outer; p.q_inner = a.q_inner; p.kv_outer = a.kv_outer; p.kv_inner = a.kv_inner;
  p.q_tok_step = a.q_tok_step; p.kv_tok_step = a.kv_tok_step;
  p.Lq = a.Lq; p.Lk_max = a.Lk_max; p.H = a.H;
  p.use_kv_len = a.use_kv_len;
  for (int i = 0; i < 64; ++i) p.kv_len[i] = a.kv_len[i];
  p.scale = 1.0f / sqrtf((float)a.dh);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  if (a.n_groups > 65535 || a.H > 65535) {
    set_error("attention grid too large (groups=%d heads=%d)", a.n_groups, a.H);
    return -2;
  }
  if (a.dh == 72) return launch_dh<72>(p, a.n_groups, s);
  if (a.dh == 64) return launch_dh<64>(p, a.n_groups, s);
  set_error("dh=%d: supported head dims are 64 and 72", a.dh);
  return -2;
}

}  // namespace ddit
