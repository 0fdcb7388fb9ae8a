// Temporal self-attention: for every (sample, location, head) the T frames attend to each other,
//   O = softmax(Q K^T / sqrt(dh)) V  over T <= 32 rows that lie a whole frame (S tokens) apart.
//
// The arithmetic is tiny (4 T A flop per token against 8 A bytes); what matters is how memory is
// touched: a (location, head) sequence is T pieces of 2 dh bytes, S rows apart.  A workgroup
// therefore takes FOUR neighbouring heads of one location, so that every row contributes one
// contiguous piece of 8 dh bytes per operand, fetched as 16-byte chunks, and the four workgroups
// of a location (16 heads) are dealt to the same XCD so that cache lines straddling two head
// groups are served from its L2.
//
// Each wavefront then owns one head.  T <= 32 fits a single 32x32 matrix-core tile:
// S^T = K Q^T (keys x queries; a lane owns one query, so the softmax is a register reduction
// plus one lane exchange), P^T rounded to bf16 is the second operand of O^T = V^T P^T as it
// stands, with V^T gathered from LDS in the key order the accumulator registers enumerate.
// The head dim is padded with zeros in registers only.  O is staged in LDS (over Q, which is
// dead by then) and written out as 16-byte chunks of whole rows.
#include "ddit_common.hpp"

namespace {

constexpr int HG = 4;      // heads per workgroup, one per wavefront
constexpr int TP = 32;     // rows of the matrix-core tile

struct TemporalParams {
  const bf16_t *q, *k, *v;
  bf16_t *o;
  float *lse;
  int64_t ld_q, ld_kv, ld_o;
  int B, T, S, H;
  int n_hg;            // head groups per location
  float scale_log2;    // log2(e) / sqrt(dh)
  float scale;         // 1 / sqrt(dh)
  // optional treatment of q and k on their way in (OPTS form of the kernel):
  const bf16_t *g_q, *g_k;   // per-head RMS-norm scales [dh], or null
  const float2 *rope;        // (cos, sin) of frame t, pair i at [t * dh/2 + i], or null
  float norm_eps;
};

template <int DH>
struct TCfg {
  static constexpr int DCH = DH / 8;                 // 16-byte chunks per head row
  static constexpr int RCH = HG * DCH;               // chunks per LDS row (four heads)
  static constexpr int PITCH = RCH * 16 + 16;        // +16 B: 16 consecutive rows hit 16 different bank groups
  static constexpr int MAT = TP * PITCH;             // one operand
  static constexpr int KS = (DH + 15) / 16;          // k-steps of Q K^T
  static constexpr int DT = (DH + 31) / 32;          // 32-row tiles of V^T
  static_assert((PITCH / 16) % 2 == 1, "odd pitch in 16-byte units keeps the reads conflict-free");
};

__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// OPTS: q and k are RMS-normalised per head and rotated by their frame's angles after they have
// landed in LDS (every sequence is loaded exactly once here, so this costs no memory traffic):
// one thread per (operand, frame, head) row, two passes over its d_h elements, fp32 arithmetic,
// one rounding back to bf16; scales and the (cos, sin) rows of the T frames sit in LDS beside the operands.
template <int DH, bool OPTS>
__global__ __launch_bounds__(256) void k_temporal_attn(TemporalParams p) {
  using C = TCfg<DH>;
  constexpr int OPT_BYTES = OPTS ? TP * (DH / 2) * 8 + 2 * DH * 4 : 0;
  __shared__ __attribute__((aligned(16))) unsigned char smem[3 * C::MAT + OPT_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;

  // block -> (location, head group): the head groups of a location are 8 blocks apart (same XCD)
  const int xcd = blockIdx.x & 7;
  const int rest = blockIdx.x >> 3;
  const int hg = rest % p.n_hg;
  const int64_t loc = (int64_t)(rest / p.n_hg) * 8 + xcd;     // b * S + s
  if (loc >= (int64_t)p.B * p.S) return;
  const int b = (int)(loc / p.S), s = (int)(loc - (int64_t)b * p.S);
  const int h0 = hg * HG;
  const int nh = p.H - h0 < HG ? p.H - h0 : HG;               // heads of this group that exist
  const int64_t tok0 = (int64_t)b * p.T * p.S + s;            // token of frame 0; frame t is t*S further

  // ---- operands -> LDS: rows t < T, the chunks of the existing heads; V rows T..31 are zeroed.
  // All of a thread's loads are issued before the first one is used.
  {
    constexpr int NCH = (3 * TP * C::RCH + 255) / 256;
    uint4 val[NCH];
    int dst[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int m = tid + 256 * i;
      const int rr = m / C::RCH, ch = m - rr * C::RCH;           // rr = operand * T + frame
      const int mat = (rr >= p.T) + (rr >= 2 * p.T);
      const int r = rr - mat * p.T;
      dst[i] = rr < 3 * p.T ? mat * C::MAT + r * C::PITCH + ch * 16 : -1;
      val[i] = make_uint4(0u, 0u, 0u, 0u);
      if (rr < 3 * p.T && ch < nh * C::DCH) {
        const int64_t tok = tok0 + (int64_t)r * p.S;
        const bf16_t *src = mat == 0 ? p.q + tok * p.ld_q : (mat == 1 ? p.k + tok * p.ld_kv : p.v + tok * p.ld_kv);
        val[i] = *reinterpret_cast<const uint4 *>(src + h0 * DH + ch * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < NCH; ++i)
      if (dst[i] >= 0) *reinterpret_cast<uint4 *>(smem + dst[i]) = val[i];
    const int pad_rows = TP - p.T;
    for (int m = tid; m < pad_rows * C::RCH; m += 256) {
      const int r = p.T + m / C::RCH, ch = m % C::RCH;
      *reinterpret_cast<uint4 *>(smem + 2 * C::MAT + r * C::PITCH + ch * 16) = make_uint4(0u, 0u, 0u, 0u);
    }
  }
  if constexpr (OPTS) {
    float2 *tab = reinterpret_cast<float2 *>(smem + 3 * C::MAT);
    float *gs = reinterpret_cast<float *>(smem + 3 * C::MAT + TP * (DH / 2) * 8);
    if (p.rope)
      for (int m = tid; m < p.T * (DH / 2); m += 256) tab[m] = p.rope[m];
    if (tid < 2 * DH) gs[tid] = p.g_q ? (float)(tid < DH ? p.g_q[tid] : p.g_k[tid - DH]) : 1.0f;
    wg_barrier();
    // row (operand, frame, head) -> thread; T <= 32 and four heads: at most 256 rows
    const int hh = tid & 3, r = (tid >> 2) % TP, mat = tid / (4 * TP);
    if (mat < 2 && r < p.T && hh < nh) {
      unsigned char *row = smem + mat * C::MAT + r * C::PITCH + hh * (DH * 2);
      float rinv = 1.0f;
      if (p.g_q) {
        float ss = 0.f;
#pragma unroll
        for (int c = 0; c < C::DCH; ++c) {
          const bf16x8 v = *reinterpret_cast<const bf16x8 *>(row + c * 16);
#pragma unroll
          for (int e = 0; e < 8; ++e) ss += (float)v[e] * (float)v[e];
        }
        rinv = rsqrtf(ss * (1.0f / DH) + p.norm_eps);
      }
      const float *g = gs + mat * DH;
      const float2 *cs = tab + r * (DH / 2);
#pragma unroll
      for (int c = 0; c < C::DCH; ++c) {
        bf16x8 v = *reinterpret_cast<const bf16x8 *>(row + c * 16);
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)v[e] * rinv * g[c * 8 + e];
        if (p.rope) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float2 a = cs[c * 4 + j];
            const float x0 = f[2 * j], x1 = f[2 * j + 1];
            f[2 * j] = x0 * a.x - x1 * a.y;
            f[2 * j + 1] = x1 * a.x + x0 * a.y;
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)f[e];
        *reinterpret_cast<bf16x8 *>(row + c * 16) = v;
      }
    }
  }
  wg_barrier();

  const int h = h0 + wave;
  floatx16 oacc[C::DT];
  float m_q = 0.f, l_q = 1.f;
  if (wave < nh) {
    // ---- S^T = K Q^T: lane holds key/query l32, d = 16 ks + 8 lh .. +7 (zeros past DH; rows >= T clamp)
    const int row = l32 < p.T ? l32 : p.T - 1;
    const unsigned char *qrow = smem + row * C::PITCH + wave * (DH * 2);
    const unsigned char *krow = qrow + C::MAT;
    floatx16 sc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int c = 2 * ks + lh;
      bf16x8 qf, kf;
#pragma unroll
      for (int e = 0; e < 8; ++e) { qf[e] = (bf16_t)0.f; kf[e] = (bf16_t)0.f; }
      if (c < C::DCH) {
        qf = *reinterpret_cast<const bf16x8 *>(qrow + c * 16);
        kf = *reinterpret_cast<const bf16x8 *>(krow + c * 16);
      }
      sc = mfma32(kf, qf, sc);
    }
    // register r of this lane: key 8 (r >> 2) + 4 lh + (r & 3), query l32
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = 8 * (r >> 2) + 4 * lh + (r & 3);
      if (key >= p.T) sc[r] = -INFINITY;
      mx = fmaxf(mx, sc[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mb = mx * p.scale_log2;
    bf16x8 pf[2];
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const bf16_t pb = (bf16_t)__builtin_amdgcn_exp2f(sc[r] * p.scale_log2 - mb);
      pf[r >> 3][r & 7] = pb;
      psum += (float)pb;      // the sum of what the matrix core will use
    }
    psum += __shfl_xor(psum, 32, 64);
    m_q = mx;
    l_q = psum;

    // ---- O^T = V^T P^T: first operand V^T[d = 32 dt + l32][key]; contraction index (kc, lh, j)
    // stands for key 16 kc + 8 (j >> 2) + 4 lh + (j & 3), the order of the accumulator registers
    const unsigned char *vcol = smem + 2 * C::MAT + wave * (DH * 2);
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
      const int d = 32 * dt + l32;
#pragma unroll
      for (int kc = 0; kc < 2; ++kc) {
        bf16x8 vf;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int key = 16 * kc + 8 * (j >> 2) + 4 * lh + (j & 3);
          uint16_t bits = 0;
          if (d < DH) bits = *reinterpret_cast<const uint16_t *>(vcol + key * C::PITCH + d * 2);
          vf[j] = __builtin_bit_cast(bf16_t, bits);
        }
        oacc[dt] = mfma32(vf, pf[kc], oacc[dt]);
      }
    }
  }
  wg_barrier();   // every wavefront is done with Q: its place takes O

  if (wave < nh) {
    // register r of tile dt: d = 32 dt + 8 (r >> 2) + 4 lh + (r & 3), query l32
    const float inv = 1.0f / l_q;
    unsigned char *orow = smem + l32 * C::PITCH + wave * (DH * 2);
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d0 = 32 * dt + 8 * g + 4 * lh;
        if (d0 < DH) {
          bf16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[dt][4 * g + e] * inv);
          *reinterpret_cast<bf16x4 *>(orow + d0 * 2) = ov;
        }
      }
    if (p.lse && lh == 0 && l32 < p.T)
      p.lse[(tok0 + (int64_t)l32 * p.S) * p.H + h] = m_q * p.scale + __logf(l_q);
  }
  wg_barrier();
  {
    const int row_ch = nh * C::DCH;   // chunks of a row that hold existing heads
#pragma unroll 4
    for (int m = tid; m < p.T * row_ch; m += 256) {
      const int r = m / row_ch, ch = m - r * row_ch;
      const uint4 val = *reinterpret_cast<const uint4 *>(smem + r * C::PITCH + ch * 16);
      *reinterpret_cast<uint4 *>(p.o + (tok0 + (int64_t)r * p.S) * p.ld_o + h0 * DH + ch * 8) = val;
    }
  }
}

template <int DH>
int launch_t(const TemporalParams &p, hipStream_t s) {
  const bool opts = p.g_q != nullptr || p.rope != nullptr;
  const int64_t locs = (int64_t)p.B * p.S;
  const int64_t blocks = ((locs + 7) / 8) * p.n_hg * 8;
  if (blocks > 0x7fffffff) { ddit::set_error("temporal attention: too many workgroups"); return -2; }
  if (opts) hipLaunchKernelGGL((k_temporal_attn<DH, true>), dim3((unsigned)blocks), dim3(256), 0, s, p);
  else hipLaunchKernelGGL((k_temporal_attn<DH, false>), dim3((unsigned)blocks), dim3(256), 0, s, p);
  return ddit::hip_fail(hipGetLastError(), "temporal attention launch");
}

}  // namespace

namespace ddit {

int temporal_attn_max_T() { return TP; }

int launch_temporal_attn(const void *q, const void *k, const void *v, void *o, float *lse, int64_t ld_q,
                         int64_t ld_kv, int64_t ld_o, int B, int T, int S, int H, int dh, const void *g_q,
                         const void *g_k, float norm_eps, const float *rope_table, hipStream_t s) {
  if (B == 0 || S == 0 || T == 0) return 0;
  if (T > TP) { set_error("temporal attention kernel: T=%d exceeds %d", T, TP); return -2; }
  TemporalParams p;
  p.q = reinterpret_cast<const bf16_t *>(q);
  p.k = reinterpret_cast<const bf16_t *>(k);
  p.v = reinterpret_cast<const bf16_t *>(v);
  p.o = reinterpret_cast<bf16_t *>(o);
  p.lse = lse;
  p.ld_q = ld_q; p.ld_kv = ld_kv; p.ld_o = ld_o;
  p.B = B; p.T = T; p.S = S; p.H = H;
  p.n_hg = (H + HG - 1) / HG;
  p.scale = 1.0f / sqrtf((float)dh);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  p.g_q = reinterpret_cast<const bf16_t *>(g_q);
  p.g_k = reinterpret_cast<const bf16_t *>(g_k);
  p.rope = reinterpret_cast<const float2 *>(rope_table);
  p.norm_eps = norm_eps;
  if (dh == 72) return launch_t<72>(p, s);
  if (dh == 64) return launch_t<64>(p, s);
  set_error("dh=%d: supported head dims are 64 and 72", dh);
  return -2;
}

}  // namespace ddit
