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
// The head dim 72 is padded to 80 for Q K^T (zeros in registers, never in memory) and to
// 96 rows for V^T; one of the spare V^T rows is set to 1 so that the same MFMAs that form
// O also accumulate the softmax denominator (of the bf16-rounded probabilities used).
//
// Data movement.  K tiles go global -> LDS directly (16 bytes per lane, no registers),
// packed at a 144-byte row pitch for dh 72 (16-byte reads of 8 consecutive rows then
// cover all 32 banks once) or at 128 bytes with an XOR chunk swizzle for dh 64.  V goes
// through registers for the transposition.  Two stages; the next tile's loads are in
// flight during the current tile's MFMAs; one barrier per tile.
#include "ddit_common.hpp"

namespace {

constexpr int QT = 128;   // queries per workgroup
constexpr int KT = 64;    // keys per LDS tile

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(1))) const void *gbl_ptr_t;

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
  static constexpr int DCH = DH / 8;               // 16-byte chunks per K/V row
  static constexpr int KROW = DCH * 16;            // K row pitch in LDS: packed
  static constexpr bool SWZ = (KROW % 128) == 0;   // packed pitch would alias banks: swizzle chunks
  static constexpr bool ONES = (DH % 32) != 0;     // a spare V^T row exists for the row sum
  static constexpr int DT = (DH + 31) / 32;        // 32-row tiles of V^T
  static constexpr int VROW = KT * 2 + 16;         // V^T row pitch (bytes)
  static constexpr int K_BYTES = KT * KROW;
  static constexpr int V_BYTES = DT * 32 * VROW;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int K_INSTR = K_BYTES / 1024;   // wave-wide 16-byte direct loads per K tile
  static_assert(K_BYTES % 1024 == 0, "K tile must be a whole number of wave loads");
};

// position of key offset o (0..15) inside its group of 16 in the V^T rows:
// o = 8 g + 4 h + e  ->  8 h + 4 g + e   (h: lane half, g: accumulator group parity)
__device__ __forceinline__ int key_pos16(int o) { return ((o & 4) << 1) | ((o & 8) >> 1) | (o & 3); }

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int DH>
__global__ __launch_bounds__(256, 2) void k_flash_attn(FlashParams p) {
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
  const bf16_t *kbase = p.k + kv_tok0 * p.ld_kv + h * DH;
  const bf16_t *vbase = p.v + kv_tok0 * p.ld_kv + h * DH;
  const int64_t kv_row = p.kv_tok_step * p.ld_kv;   // elements between consecutive keys

  // ---- Q fragment: lane holds query l32, d = 16 ks + 8 lh .. +7 (zeros past DH)
  bf16x8 qf[C::KS];
  {
    int qi = q0 + l32;
    if (qi > p.Lq - 1) qi = p.Lq - 1;
    const bf16_t *qrow = p.q + (q_tok0 + (int64_t)qi * p.q_tok_step) * p.ld_q + h * DH;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int d0 = 16 * ks + 8 * lh;
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16_t)0.f;
      if (d0 < DH) qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + d0);
    }
  }

  // ---- V^T padding rows (DH .. 32 DT - 1) of both stages: zero, except the row of ones
  if constexpr (C::DT * 32 > DH) {
    constexpr int PER_STAGE = (C::DT * 32 - DH) * (KT / 2);   // 32-bit words
    for (int i = tid; i < 2 * PER_STAGE; i += 256) {
      const int st = i / PER_STAGE, rem = i % PER_STAGE;
      const int row = DH + rem / (KT / 2), w = rem % (KT / 2);
      const uint32_t val = (C::ONES && row == DH) ? 0x3F803F80u : 0u;  // bf16 1.0 twice
      *reinterpret_cast<uint32_t *>(smem + st * C::STAGE + C::K_BYTES + row * C::VROW + w * 4) = val;
    }
  }

  // ---- K tile, global -> LDS: wave-wide load j fills LDS bytes [1024 j, 1024 j + 1024) of the tile;
  // this lane's piece is LDS chunk m = 64 j + lane = (key m / DCH, chunk slot m % DCH)
  constexpr int KJ = (C::K_INSTR + 3) / 4;   // loads per wave (the last one only on some waves)
  int k_key[KJ], k_col[KJ];
#pragma unroll
  for (int i = 0; i < KJ; ++i) {
    const int m = 64 * (wave + 4 * i) + lane;
    const int key = m / C::DCH, slot = m - key * C::DCH;
    k_key[i] = key;
    k_col[i] = (C::SWZ ? (slot ^ (key & 7)) : slot) * 8;
  }
  // ---- V tile through registers: task A (every lane): key pair kp = l32, chunk 2 wave + lh;
  // task B (dh 72 only: the 9th chunk): lanes 0..31 of wave (tile & 3)
  constexpr bool VB = (C::DCH % 8) != 0;
  const int v_pos = ((2 * l32) & ~15) | key_pos16((2 * l32) & 15);   // even: the pair stays adjacent
  uint4 va0, va1, vb0, vb1;
  va0 = va1 = vb0 = vb1 = make_uint4(0u, 0u, 0u, 0u);

#define FA_LOAD_TILE(KEY0, STAGE_IDX, TILE_IDX)                                                         \
  do {                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < KJ; ++i) {                                                    \
      if (wave + 4 * i < C::K_INSTR) {                                                                  \
        int key_ = (KEY0) + k_key[i];                                                                   \
        if (key_ > Lk - 1) key_ = Lk - 1; /* tail keys re-read the last valid key; masked below */      \
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(kbase + key_ * kv_row + k_col[i]),                 \
                                         (lds_ptr_t)(smem + (STAGE_IDX) * C::STAGE + (wave + 4 * i) * 1024), \
                                         16, 0, 0);                                                     \
      }                                                                                                 \
    }                                                                                                   \
    {                                                                                                   \
      int ka_ = (KEY0) + 2 * l32, kb_ = ka_ + 1;                                                        \
      if (ka_ > Lk - 1) ka_ = Lk - 1;                                                                   \
      if (kb_ > Lk - 1) kb_ = Lk - 1;                                                                   \
      const int dc_ = 2 * wave + lh;                                                                    \
      va0 = *reinterpret_cast<const uint4 *>(vbase + ka_ * kv_row + dc_ * 8);                           \
      va1 = *reinterpret_cast<const uint4 *>(vbase + kb_ * kv_row + dc_ * 8);                           \
      if (VB && wave == ((TILE_IDX) & 3) && lh == 0) {                                                  \
        vb0 = *reinterpret_cast<const uint4 *>(vbase + ka_ * kv_row + 64);                              \
        vb1 = *reinterpret_cast<const uint4 *>(vbase + kb_ * kv_row + 64);                              \
      }                                                                                                 \
    }                                                                                                   \
  } while (0)

#define FA_VT_WRITE(DST, A, B)                                                                          \
  do {                                                                                                  \
    unsigned char *d_ = (DST);                                                                          \
    *reinterpret_cast<uint32_t *>(d_ + 0 * C::VROW) = ((A).x & 0xFFFFu) | ((B).x << 16);               \
    *reinterpret_cast<uint32_t *>(d_ + 1 * C::VROW) = ((A).x >> 16) | ((B).x & 0xFFFF0000u);           \
    *reinterpret_cast<uint32_t *>(d_ + 2 * C::VROW) = ((A).y & 0xFFFFu) | ((B).y << 16);               \
    *reinterpret_cast<uint32_t *>(d_ + 3 * C::VROW) = ((A).y >> 16) | ((B).y & 0xFFFF0000u);           \
    *reinterpret_cast<uint32_t *>(d_ + 4 * C::VROW) = ((A).z & 0xFFFFu) | ((B).z << 16);               \
    *reinterpret_cast<uint32_t *>(d_ + 5 * C::VROW) = ((A).z >> 16) | ((B).z & 0xFFFF0000u);           \
    *reinterpret_cast<uint32_t *>(d_ + 6 * C::VROW) = ((A).w & 0xFFFFu) | ((B).w << 16);               \
    *reinterpret_cast<uint32_t *>(d_ + 7 * C::VROW) = ((A).w >> 16) | ((B).w & 0xFFFF0000u);           \
  } while (0)

#define FA_STORE_V(STAGE_IDX, TILE_IDX)                                                                 \
  do {                                                                                                  \
    unsigned char *sv_ = smem + (STAGE_IDX) * C::STAGE + C::K_BYTES + v_pos * 2;                        \
    FA_VT_WRITE(sv_ + (2 * wave + lh) * 8 * C::VROW, va0, va1);                                         \
    if (VB && wave == ((TILE_IDX) & 3) && lh == 0) FA_VT_WRITE(sv_ + 64 * C::VROW, vb0, vb1);           \
  } while (0)

  floatx16 oacc[C::DT];
#pragma unroll
  for (int d = 0; d < C::DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
  float m_run = -INFINITY;   // running maximum of the raw (unscaled) scores of this lane's query
  float l_run = 0.f;         // running sum (only used when there is no ones row)

  const int n_tiles = (Lk + KT - 1) / KT;
  FA_LOAD_TILE(0, 0, 0);
  FA_STORE_V(0, 0);
  if (n_tiles > 1) FA_LOAD_TILE(KT, 1, 1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // K of tile 0 has landed (once per kernel: also waits tile 1)
  lds_barrier();

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
      const int row = kt * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const int c = 2 * ks + lh;
        bf16x8 kf;
#pragma unroll
        for (int e = 0; e < 8; ++e) kf[e] = (bf16_t)0.f;
        if (c < C::DCH)
          kf = *reinterpret_cast<const bf16x8 *>(sk + row * C::KROW + (C::SWZ ? (c ^ (row & 7)) : c) * 16);
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
    const float mb = m_new * p.scale_log2;
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
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // some query of the wave has a new maximum
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2);
#pragma unroll
      for (int d = 0; d < C::DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[d][e] *= alpha;
      if (!C::ONES) l_run *= alpha;
      m_run = m_new;
    }
    if (!C::ONES) l_run += psum;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
#pragma unroll
      for (int d = 0; d < C::DT; ++d) {
        const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(sv + (d * 32 + l32) * C::VROW + (2 * kc + lh) * 16);
        oacc[d] = mfma32(vf, pf[kc], oacc[d]);
      }
    }

    if (it + 1 < n_tiles) FA_STORE_V(cur ^ 1, it + 1);           // registers hold V of tile it+1
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // K of tile it+1 has landed
    lds_barrier();                                               // stage cur is free, stage cur^1 complete
    if (it + 2 < n_tiles) FA_LOAD_TILE((it + 2) * KT, cur, it + 2);
  }
#undef FA_LOAD_TILE
#undef FA_VT_WRITE
#undef FA_STORE_V

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
