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
// Work split.  Streaming form: grid = (query tiles of 128, heads, groups); 4 wavefronts per
// workgroup, each owning 32 queries against all keys of the group, K/V tiles through a two-stage
// LDS ring.  Resident form (key sequences of at most 320 shared by thousands of queries: the text
// tokens of cross-attention): 8 wavefronts, one workgroup per CU; the unit's whole K and V are
// fetched into LDS once and the workgroup walks over a run of 256-query tiles with no further tile
// load and no barrier (480p cross-attention: 0.149 -> 0.109 ms; each further key tile then costs
// what its MFMAs cost).
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-wide wavefronts).  Scores are
// computed transposed, S^T = K Q^T: the K tile is the first operand (read from LDS, 16
// bytes per lane), the wave's Q fragment the second (held in registers for the whole
// kernel).  In the result layout a lane owns ONE query (column l%32) and 16 of every 32
// keys, so the row maximum is a register reduction plus one exchange with lane l^32.
// The probabilities P^T, rounded to bf16, are then already laid out as the second
// operand of O^T = V^T P^T, provided the first operand V^T enumerates the keys in the
// order of the accumulator registers.  V stays row-major [key][d] in LDS, exactly as it
// comes from memory; the transposition happens in the LDS read: ds_read_b64_tr_b16 hands
// each lane of a 16-lane block four KEYS' values of its own d (lane i of the block
// supplies the address of the 8-byte piece "key i/4, d-group i%4"; it receives element i%4
// of the pieces of lanes i/4, 4+i/4, 8+i/4, 12+i/4), two such reads per operand.
// The head dim is padded to the next multiple of 16 above it for Q K^T and to 96 rows for V^T
// (rows past the head dim read neighbouring data and produce rows of O^T that are never
// stored); row 72 of V^T reads constant pieces holding ones, so that the same MFMAs that form O
// also accumulate the softmax denominator (of the bf16-rounded probabilities used).
//
// Online softmax without per-score bookkeeping.  The first padding column of the contraction
// (index dh) is put to work: K holds a one there (a constant 16-byte piece in LDS that the lanes
// of that column read instead of tile data) and Q holds minus the query's reference score, so the
// matrix core delivers s - m_ref directly and a probability is one multiply (by log2(e)/sqrt(dh))
// and one exponential.  m_ref is set from the first key tile and moved later only if a score
// exceeds it by 8 binary orders of magnitude; only then are O and the pending scores rescaled.
// Any reference gives the same softmax as long as every term uses the same one.
//
// Data movement.  K and V tiles go global -> LDS directly (16 bytes per lane, no
// registers), packed at a 144-byte row pitch for dh 72 or at 128 bytes with an XOR chunk
// swizzle for dh 64.  Two stages; the next tile's loads are in flight during the current
// tile's arithmetic; one barrier per tile.
//
// Instruction order.  Per key tile a wavefront has about as many vector-ALU clocks (one
// exponential per score is a half-rate instruction) as matrix-core clocks, so the MFMAs are
// threaded through the exponentials by hand: see tile_step.
#include "ddit_common.hpp"

namespace {

constexpr int STREAM_NW = 4;   // wavefronts per workgroup of the streaming form (two workgroups per CU)
constexpr int RES_NW = 8;      // ... of the resident form (one workgroup per CU)
constexpr int RES_TILES = 5;   // key tiles the resident form keeps in LDS: sequences of up to 320 keys
constexpr int KT = 64;         // keys per LDS tile

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(1))) const void *gbl_ptr_t;
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) shortx4 *lds_s4_ptr_t;

struct FlashParams {
  const bf16_t *q, *k, *v;
  bf16_t *o;
  float *lse;
  int64_t ld_q, ld_kv, ld_o;
  int g_inner;
  int64_t q_outer, q_inner, kv_outer, kv_inner;
  int64_t q_tok_step, kv_tok_step;
  int Lq, Lk_max, H;
  int n_qtiles, n_units;   // query tiles per (group, head) unit; units = groups * heads
  int n_chunks, qtiles_per_chunk;   // resident form: workgroups per unit, consecutive query tiles per workgroup
  int spread;              // few units: spread a unit's query tiles over the XCDs
  int use_kv_len;
  int kv_len[64];
  float scale_log2;  // log2(e) / sqrt(dh)
  float scale;       // 1 / sqrt(dh)
  float rebase;      // 8 / scale_log2: a score this far above its query's reference moves the reference
  const bf16_t *q_norm_g;   // per-head RMS-norm scales of the queries [dh], or null
  float q_norm_eps;
};

template <int DH>
struct Cfg {
  static constexpr int KS = DH / 16 + 1;           // k-steps of Q K^T: the head dim plus the reference column (index DH)
  static constexpr int DCH = DH / 8;               // 16-byte chunks per K/V row
  static constexpr int KROW = DCH * 16;            // K/V row pitch in LDS: packed
  static constexpr bool SWZ = (KROW % 128) == 0;   // packed pitch would alias banks: swizzle chunks
  static constexpr bool ONES = (DH % 32) != 0;     // a spare V^T row exists for the row sum
  static constexpr int DT = (DH + 31) / 32;        // 32-row tiles of V^T
  static constexpr int T_BYTES = KT * KROW;        // one K or V tile
  static constexpr int KCONST = 2 * T_BYTES;       // offset of the constant K piece (1, 0, ..., 0) in a stage
  static constexpr int OVERRUN = 64;               // V^T rows past the head dim read up to this far past a tile
  // After the K piece come, when the head dim leaves a spare V^T row, four 8-byte pieces (1, 0, 0, 0),
  // 16 keys apart like the contraction chunks of the V reads: the lanes that supply the pieces of row
  // DH of V^T point there, so the row of ones needs no substitution in registers.
  static constexpr int VONE = KCONST + 16;
  static constexpr int TAIL = ONES ? 3 * 16 * KROW : 0;
  static constexpr int STAGE = 2 * T_BYTES + OVERRUN + TAIL;   // K tile, V tile, constant pieces (the rest is slack)
  static constexpr int T_INSTR = T_BYTES / 1024;   // wave-wide 16-byte direct loads per tile
  static_assert(T_BYTES % 1024 == 0, "a tile must be a whole number of wave loads");
  static_assert((DT * 32 - DH) * 2 <= OVERRUN, "overrun of the padded V^T rows");
  static_assert(DH % 8 == 0, "the reference column starts a 16-byte chunk");
};

__device__ __forceinline__ unsigned lds_addr(const void *p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
// Transposing 8-byte LDS read (see the V^T operand below), issued WITHOUT a wait: the result may
// be used only after lds_wait_* on it.  Written as inline assembly because the compiler, when it
// sees an LDS read while direct-to-LDS loads are in flight, first waits for ALL of them (it cannot
// tell that they fill a different stage), which would expose the whole fetch latency every tile.
template <int IMM>
__device__ __forceinline__ shortx4 lds_read_tr_nowait(unsigned addr) {
  shortx4 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(IMM));
  return r;
}

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <bool V>
struct BoolTag { static constexpr bool value = V; };

// RES = false, the streaming form: one query tile per workgroup, K/V tiles through a two-stage ring.
// RES = true, the resident form, for short key sequences shared by many queries (the text tokens of
// cross-attention): the whole K and V of the unit are fetched into LDS once (stage t = key tile t),
// then the workgroup walks over its run of query tiles with no further tile load and no barrier;
// what it saves is the per-query-tile prologue (with five key tiles that is a third of the time)
// and four fifths of the K/V traffic.
template <int DH, int NW, bool RES>
__global__ __launch_bounds__(64 * NW, 2) void k_flash_attn(FlashParams p) {
  using C = Cfg<DH>;
  constexpr int QT = 32 * NW;              // queries per workgroup and query tile
  constexpr int NST = RES ? RES_TILES : 2; // LDS stages
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  // The scalar arguments of the set-up are fetched in ONE batch: left to itself the compiler
  // fetches each where it is first used, one memory latency after the other.
  {
    const int a0 = p.spread, a1 = p.n_qtiles, a2 = p.n_units, a3 = p.H, a4 = p.g_inner, a5 = p.use_kv_len,
              a6 = p.Lk_max, a7 = p.Lq;
    const int64_t b0 = p.q_outer, b1 = p.q_inner, b2 = p.kv_outer, b3 = p.kv_inner, b4 = p.q_tok_step,
                  b5 = p.kv_tok_step, b6 = p.ld_q, b7 = p.ld_kv;
    const void *c0 = p.q, *c1 = p.k, *c2 = p.v;
    asm volatile("" ::"s"(a0), "s"(a1), "s"(a2), "s"(a3), "s"(a4), "s"(a5), "s"(a6), "s"(a7), "s"(b0), "s"(b1),
                 "s"(b2), "s"(b3), "s"(b4), "s"(b5), "s"(b6), "s"(b7), "s"(c0), "s"(c1), "s"(c2));
  }
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  All query tiles of a
  // (group, head) unit read the same K/V, so a unit lives on ONE XCD: unit u on XCD u % 8, its
  // query tiles consecutive there.
  // (With only a few units that would leave XCDs idle; their K/V are then small enough for every
  // L2, and consecutive workgroups simply take consecutive query tiles.)
  int unit, qtile, qt_end;
  if constexpr (RES) {
    unit = blockIdx.x / p.n_chunks;
    qtile = (blockIdx.x - unit * p.n_chunks) * p.qtiles_per_chunk;
    qt_end = qtile + p.qtiles_per_chunk < p.n_qtiles ? qtile + p.qtiles_per_chunk : p.n_qtiles;
  } else if (p.spread) {
    unit = blockIdx.x / p.n_qtiles;
    qtile = blockIdx.x - unit * p.n_qtiles;
  } else {
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    unit = (idx / p.n_qtiles) * 8 + xcd;
    qtile = idx % p.n_qtiles;
  }
  if constexpr (!RES) qt_end = qtile + 1;
  if (unit >= p.n_units || qtile >= qt_end) return;
  const int h = unit % p.H, g = unit / p.H;
  const int g_out = g / p.g_inner, g_in = g - g_out * p.g_inner;
  const int Lk = p.use_kv_len ? p.kv_len[g_out] : p.Lk_max;
  const int64_t q_tok0 = p.q_outer * g_out + p.q_inner * g_in;
  const int64_t kv_tok0 = p.kv_outer * g_out + p.kv_inner * g_in;
  const bf16_t *kbase = p.k + kv_tok0 * p.ld_kv + h * DH;
  const bf16_t *vbase = p.v + kv_tok0 * p.ld_kv + h * DH;
  const int64_t kv_row = p.kv_tok_step * p.ld_kv;   // elements between consecutive keys

  // ---- Q fragment: lane holds query l32, d = 16 ks + 8 lh .. +7.  Column DH (zero for now) will
  // carry minus the query's reference score, against a K column of ones; the columns past it stay
  // zero.
  bf16x8 qf[C::KS];
  auto load_q = [&](int q0_) {
    int qi = q0_ + l32;
    if (qi > p.Lq - 1) qi = p.Lq - 1;
    const bf16_t *qrow = p.q + (q_tok0 + (int64_t)qi * p.q_tok_step) * p.ld_q + h * DH;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int d0 = 16 * ks + 8 * lh;
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16_t)0.f;
      if (d0 < DH) qf[ks] = *reinterpret_cast<const bf16x8 *>(qrow + d0);
    }
    if (p.q_norm_g) {
      // per-head RMS normalisation of the query on its way in: lanes l and l ^ 32 hold the two halves
      // of every 16 elements of one query; fp32 arithmetic, one rounding back to bf16
      float ss = 0.f;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += (float)qf[ks][e] * (float)qf[ks][e];   // columns past the head dim are zero
      ss += __shfl_xor(ss, 32, 64);
      const float rinv = rsqrtf(ss * (1.0f / DH) + p.q_norm_eps);
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const int d0 = 16 * ks + 8 * lh;
        if (d0 < DH) {
          const bf16x8 g = *reinterpret_cast<const bf16x8 *>(p.q_norm_g + d0);
#pragma unroll
          for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16_t)((float)qf[ks][e] * rinv * (float)g[e]);
        }
      }
    }
  };
  load_q(qtile * QT + wave * 32);
  constexpr int KS_REF = DH / 16;                       // k-step of the reference column
  const bool ref_lane = (8 * lh == DH - 16 * KS_REF);   // lanes whose fragment of that k-step starts at column DH

  // K fragment addressing inside a stage: key (half * 32 + l32), 16-byte chunk 2 ks + lh; the lanes
  // whose columns lie past the head dim read the constant piece (1, 0, ..., 0) instead
  int k_off[C::KS][2];
#pragma unroll
  for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int row = hf * 32 + l32, c = 2 * ks + lh;
      k_off[ks][hf] = c < C::DCH ? row * C::KROW + (C::SWZ ? (c ^ (row & 7)) : c) * 16 : C::KCONST;
    }
  static_assert(C::VONE == C::KCONST + 16 && C::OVERRUN >= 24, "the first piece of ones lies in the slack after the K piece");
  static_assert(NST * (C::OVERRUN / 4) + NST * 6 <= 64 * NW, "one thread per constant word");
  if (tid < NST * (C::OVERRUN / 4)) {
    // per stage, the 64 bytes after the V tile: the constant K piece (1, 0, ..., 0), the first
    // (1, 0, 0, 0) piece of V^T's row of ones, zeros in the rest (padded V^T rows read it); every
    // word has exactly one writer
    const int st = tid / (C::OVERRUN / 4), w = tid - st * (C::OVERRUN / 4);
    *reinterpret_cast<unsigned *>(smem + st * C::STAGE + C::KCONST + 4 * w) =
        (w == 0 || (C::ONES && w == 4)) ? 0x00003F80u : 0u;
  } else if (C::ONES && tid >= NST * (C::OVERRUN / 4) && tid < NST * (C::OVERRUN / 4) + NST * 6) {
    // the other three pieces of ones, 16 keys apart
    const int e = tid - NST * (C::OVERRUN / 4), st = e / 6, kc = 1 + (e % 6) / 2, w = e & 1;
    *reinterpret_cast<unsigned *>(smem + st * C::STAGE + C::VONE + kc * 16 * C::KROW + 4 * w) = w == 0 ? 0x00003F80u : 0u;
  }

  // ---- K and V tiles, global -> LDS: wave-wide load j fills LDS bytes [1024 j, 1024 j + 1024) of a
  // tile; this lane's piece is LDS chunk m = 64 j + lane = (key m / DCH, chunk slot m % DCH)
  constexpr int TJ = (C::T_INSTR + NW - 1) / NW;   // loads per wave and tile (the last one only on some waves)
  int t_key[TJ], t_col[TJ];
#pragma unroll
  for (int i = 0; i < TJ; ++i) {
    const int m = 64 * (wave + NW * i) + lane;
    const int key = m / C::DCH, slot = m - key * C::DCH;
    t_key[i] = key;
    t_col[i] = (C::SWZ ? (slot ^ (key & 7)) : slot) * 8;
  }
  // offsets of this lane's pieces in tile 0; a full tile t is fetched at + t * KT keys, a tile that
  // overhangs the sequence takes the slow path (its keys are clamped, and masked later)
  int64_t t_off[TJ];
#pragma unroll
  for (int i = 0; i < TJ; ++i) t_off[i] = t_key[i] * kv_row + t_col[i];

  // one operand (K: WHICH = 0, V: WHICH = 1) of the tile starting at key KEY0 -> stage STAGE_IDX
#define FA_LOAD(WHICH, KEY0, STAGE_IDX, TILE_IDX)                                                       \
  do {                                                                                                  \
    unsigned char *dst_ = smem + (STAGE_IDX) * C::STAGE + (WHICH) * C::T_BYTES;                         \
    const bf16_t *src_ = (WHICH) ? vbase : kbase;                                                       \
    if ((KEY0) + KT <= Lk) {                                                                            \
      const int64_t toff_ = (int64_t)(TILE_IDX) * KT * kv_row;                                          \
      _Pragma("unroll") for (int i = 0; i < TJ; ++i) {                                                  \
        if (wave + NW * i < C::T_INSTR)                                                                 \
          __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src_ + t_off[i] + toff_),                        \
                                           (lds_ptr_t)(dst_ + (wave + NW * i) * 1024), 16, 0, 0);       \
      }                                                                                                 \
    } else {                                                                                            \
      _Pragma("unroll") for (int i = 0; i < TJ; ++i) {                                                  \
        if (wave + NW * i < C::T_INSTR) {                                                               \
          int key_ = (KEY0) + t_key[i];                                                                 \
          if (key_ > Lk - 1) key_ = Lk - 1; /* tail keys re-read the last valid key; masked below */    \
          __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src_ + key_ * kv_row + t_col[i]),                \
                                           (lds_ptr_t)(dst_ + (wave + NW * i) * 1024), 16, 0, 0);       \
        }                                                                                               \
      }                                                                                                 \
    }                                                                                                   \
  } while (0)

  // ---- V^T operand addressing (ds_read_b64_tr_b16).  For contraction chunk kc and row tile dt this
  // lane (d = 32 dt + l32, key half lh) needs keys 16 kc + 4 lh + {0..3} and 16 kc + 8 + 4 lh + {0..3}.
  // Inside its 16-lane block (d base 32 dt + 16 (l32 / 16)) lane i supplies the piece of key
  // (i / 4) at d-group (i % 4).
  const int tr_key = 4 * lh + ((lane & 15) >> 2);                 // + 16 kc (+ 8 for the second read)
  const int tr_d = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);       // + 32 dt
  int tr_off[C::DT][2];   // byte offset inside a V tile for kc = 0, first / second read
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int key = tr_key + 8 * hf, d = 32 * dt + tr_d;
      const int chunk = d >> 3;
      // past the packed row (d >= DH) the address simply runs on into the next key's row
      tr_off[dt][hf] = C::SWZ ? key * C::KROW + (((chunk ^ (key & 7)) << 4) | ((d & 7) << 1)) : key * C::KROW + d * 2;
      // the piece that holds row DH of V^T (element 0 of d-group DH%16/4 in block DH%32/16 of tile DH/32)
      if (C::ONES && dt == DH / 32 && tr_d == DH % 32) tr_off[dt][hf] = C::VONE - C::T_BYTES;
    }

  floatx16 oacc[C::DT];
#pragma unroll
  for (int d = 0; d < C::DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
  // Scores are taken relative to a per-query reference m_ref (a bf16 value): they come out of the
  // matrix core as s - m_ref, because column DH of Q holds -m_ref.  The reference is set from the
  // first tile and afterwards moved only when a score exceeds it by more than p.rebase
  // (probabilities up to 2^8 are harmless in bf16 and in the fp32 sums), so the common tile needs
  // neither a subtraction per score nor a rescaling of O.
  float m_ref = 0.f;
  float l_run = 0.f;         // running sum (only used when there is no ones row)

  // S^T = K Q^T for the 64 keys of the tile in stage STAGE_IDX (prologue only)
#define FA_QK(SREG, STAGE_IDX)                                                                          \
  do {                                                                                                  \
    const unsigned char *sk_ = smem + (STAGE_IDX) * C::STAGE;                                           \
    _Pragma("unroll") for (int kt = 0; kt < 2; ++kt) {                                                  \
      _Pragma("unroll") for (int e = 0; e < 16; ++e) SREG[kt][e] = 0.f;                                 \
      _Pragma("unroll") for (int ks = 0; ks < C::KS; ++ks) {                                            \
        const bf16x8 kf_ = *reinterpret_cast<const bf16x8 *>(sk_ + k_off[ks][kt]);                      \
        SREG[kt] = mfma32(kf_, qf[ks], SREG[kt]);                                                       \
      }                                                                                                 \
    }                                                                                                   \
  } while (0)

#define FENCE() __builtin_amdgcn_sched_barrier(0)

  floatx16 s_a[2], s_b[2];   // scores of the current / next tile, swapping roles every tile

  // One key tile: online softmax of s_cur (tile it) and O^T += V^T P^T, with -- when there is a next
  // tile -- the MFMAs of its scores s_nxt = K Q^T threaded through the softmax arithmetic.  The
  // instruction order is written out by hand and fenced: a wavefront issues in order, so each MFMA
  // (32 clocks in the matrix core, dependent on the one two slots earlier) is followed by a slice
  // of VALU work that does not depend on it; the exponentials of tile it and the MFMAs of both
  // products then run side by side instead of one after the other.
  auto tile_step = [&](auto next_tag, bool first, int k_stage, int v_stage, floatx16 (&s_cur)[2], floatx16 (&s_nxt)[2]) {
    constexpr bool NEXT = decltype(next_tag)::value;
    constexpr int NQ = NEXT ? 2 * C::KS : 0;      // MFMAs of the next tile's scores
    constexpr int NPV = 4 * C::DT;                // MFMAs of this tile's O update
    constexpr int M = NQ + NPV;
    const unsigned char *sk = smem + k_stage * C::STAGE;              // K of tile it+1
    const unsigned char *sv = smem + v_stage * C::STAGE + C::T_BYTES; // V of tile it
    bf16x8 kf[NEXT ? NQ : 1];
    if constexpr (NEXT) {
#pragma unroll
      for (int q = 0; q < NQ; ++q) {              // slot q: key half q & 1, k-step q >> 1
        kf[q] = *reinterpret_cast<const bf16x8 *>(sk + k_off[q >> 1][q & 1]);
      }
    }
    FENCE();
    floatx16 zero16;
#pragma unroll
    for (int e = 0; e < 16; ++e) zero16[e] = 0.f;
#define FA_SLOT_QK(Q)                                                                                   \
  do {                                                                                                  \
    if constexpr (NEXT) s_nxt[(Q) & 1] = mfma32(kf[Q], qf[(Q) >> 1], (Q) < 2 ? zero16 : s_nxt[(Q) & 1]); \
  } while (0)
    // ---- largest exponent of the tile (this lane's half of the keys)
    FA_SLOT_QK(0);
    FENCE();
    float mx = s_cur[0][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_cur[0][r]);
    FENCE();
    FA_SLOT_QK(1);
    FENCE();
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_cur[1][r]);
    FENCE();
    FA_SLOT_QK(2);
    FENCE();
    FA_SLOT_QK(3);
    FENCE();
    // ---- new reference for the queries that need one (always on the first tile): O, the running
    // sum and this tile's exponents move to it here; the scores of the next tile pick it up from
    // the Q fragment, whose k-step KS_REF has not been issued yet (slots 2 KS_REF and 2 KS_REF + 1)
    static_assert(2 * KS_REF >= 4, "the reference column's k-step is issued after the decision");
    if (__builtin_amdgcn_ballot_w64(first || mx > p.rebase) != 0) {
      const float mq = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = (first || mq > p.rebase) ? (float)(bf16_t)(m_ref + mq) : m_ref;
      const float delta = m_new - m_ref;
      // (the first tile moves the reference from 0, possibly far down: O and the sum are still zero)
      const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta * p.scale_log2);
#pragma unroll
      for (int d = 0; d < C::DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[d][e] *= alpha;
      if (!C::ONES) l_run *= alpha;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) s_cur[kt][e] -= delta;
      m_ref = m_new;
      if (ref_lane) qf[KS_REF][0] = (bf16_t)(-m_new);
    }
    bf16x8 vf[NPV];   // V^T fragments, slot v = kc * DT + d; read three pairs ahead of their first use
    FENCE();
    // ---- exponentials two at a time; after each pair the next MFMA slot: the rest of the next
    // tile's scores first, then the O update, whose slot (kc, d) needs the 8 kc + 8 first
    // probabilities, i.e. pair 4 kc + 3
    shortx4 vlo[NPV], vhi[NPV];
    const unsigned sv_addr = lds_addr(sv);
    auto vt_issue = [&](int kc) {      // the six reads of contraction chunk kc (16 keys)
#pragma unroll
      for (int d = 0; d < C::DT; ++d) {
        const int v = kc * C::DT + d;
        switch (kc) {                  // the key offset is an immediate of the instruction
          case 0: vlo[v] = lds_read_tr_nowait<0 * 16 * C::KROW>(sv_addr + tr_off[d][0]);
                  vhi[v] = lds_read_tr_nowait<0 * 16 * C::KROW>(sv_addr + tr_off[d][1]); break;
          case 1: vlo[v] = lds_read_tr_nowait<1 * 16 * C::KROW>(sv_addr + tr_off[d][0]);
                  vhi[v] = lds_read_tr_nowait<1 * 16 * C::KROW>(sv_addr + tr_off[d][1]); break;
          case 2: vlo[v] = lds_read_tr_nowait<2 * 16 * C::KROW>(sv_addr + tr_off[d][0]);
                  vhi[v] = lds_read_tr_nowait<2 * 16 * C::KROW>(sv_addr + tr_off[d][1]); break;
          default: vlo[v] = lds_read_tr_nowait<3 * 16 * C::KROW>(sv_addr + tr_off[d][0]);
                   vhi[v] = lds_read_tr_nowait<3 * 16 * C::KROW>(sv_addr + tr_off[d][1]); break;
        }
      }
    };
    // Chunk kc has arrived once at most the reads of ONE later chunk are outstanding (LDS reads
    // return in order; chunk kc + 2 is never issued before chunk kc is used).  The wait names the
    // registers, so nothing that uses them can move above it.
    auto vt_ready = [&](int kc) {
      static_assert(C::DT == 3 || C::DT == 2, "register list of the wait");
      const int v = kc * C::DT;
      if (C::DT == 3) {
        if (kc == 3)
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vlo[v]), "+v"(vhi[v]), "+v"(vlo[v + 1]), "+v"(vhi[v + 1]),
                       "+v"(vlo[v + C::DT - 1]), "+v"(vhi[v + C::DT - 1]));
        else
          asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(vlo[v]), "+v"(vhi[v]), "+v"(vlo[v + 1]), "+v"(vhi[v + 1]),
                       "+v"(vlo[v + C::DT - 1]), "+v"(vhi[v + C::DT - 1]));
      } else {
        if (kc == 3)
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vlo[v]), "+v"(vhi[v]), "+v"(vlo[v + 1]), "+v"(vhi[v + 1]));
        else
          asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(vlo[v]), "+v"(vhi[v]), "+v"(vlo[v + 1]), "+v"(vhi[v + 1]));
      }
#pragma unroll
      for (int d = 0; d < C::DT; ++d) {
        typedef short shortx8 __attribute__((ext_vector_type(8)));
        const shortx8 both = __builtin_shufflevector(vlo[v + d], vhi[v + d], 0, 1, 2, 3, 4, 5, 6, 7);
        vf[v + d] = __builtin_bit_cast(bf16x8, both);
      }
    };
    bf16x8 pf[4];
    float psum = 0.f;
    int slot = NEXT ? 4 : 0;
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      if (g % 3 == 0 && g / 3 < 4) vt_issue(g / 3);
#pragma unroll
      for (int e = 2 * g; e < 2 * g + 2; ++e) {
        const bf16_t pb = (bf16_t)__builtin_amdgcn_exp2f(s_cur[e >> 4][e & 15] * p.scale_log2);
        pf[e >> 3][e & 7] = pb;
        if (!C::ONES) psum += (float)pb;
      }
      FENCE();
      if (slot < NQ) {
        FA_SLOT_QK(slot);
        ++slot;
      } else if (slot < M) {
        const int v = slot - NQ, kc = v / C::DT, d = v - kc * C::DT;
        if (g >= 4 * kc + 3) {
          if (d == 0) vt_ready(kc);
          oacc[d] = mfma32(vf[v], pf[kc], oacc[d]);
          ++slot;
        }
      }
      FENCE();
    }
#pragma unroll
    for (int sl = 0; sl < M; ++sl) {
      if (sl >= slot) {
        if (sl < NQ) {
          FA_SLOT_QK(sl);
        } else {
          const int v = sl - NQ, kc = v / C::DT, d = v - kc * C::DT;
          if (d == 0) vt_ready(kc);
          oacc[d] = mfma32(vf[v], pf[kc], oacc[d]);
        }
      }
    }
    if (!C::ONES) l_run += psum;
#undef FA_SLOT_QK
  };

  // Software pipeline over the key tiles (streaming form).  Stage it & 1 holds K and V of tile it.  K
  // of tile it is dead once its scores exist (formed during tile it-1), so K of tile it+2 is fetched at
  // the start of tile it; V of tile it is used until the end of tile it, so V of tile it+2 follows
  // after the barrier that ends tile it.  Both have a whole tile's time to land.
  // Resident form: every tile is fetched here, once, and stays.
  const int n_tiles = (Lk + KT - 1) / KT;
  if constexpr (RES) {
    for (int t = 0; t < n_tiles; ++t) {
      FA_LOAD(0, t * KT, t, t);
      FA_LOAD(1, t * KT, t, t);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
  }

#define FA_ITER(HAS_NEXT, S_CUR, S_NXT)                                                                 \
  do {                                                                                                  \
    const int cur_ = RES ? it : (it & 1);                                                               \
    if constexpr (!RES) {                                                                               \
      if (it + 2 < n_tiles) FA_LOAD(0, (it + 2) * KT, cur_, it + 2);                                    \
    }                                                                                                   \
    FENCE();                                                                                            \
    tile_step(BoolTag<HAS_NEXT>{}, it == 0, RES ? it + 1 : (cur_ ^ 1), cur_, S_CUR, S_NXT);             \
    FENCE();                                                                                            \
    if constexpr (!RES) {                                                                               \
      if (HAS_NEXT) {                                                                                   \
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); /* K of tile it+2 (and V of tile it+1) has landed */ \
        lds_barrier(); /* V of tile it, K of tile it+1 are free; tile it+1's V and tile it+2's K complete */ \
        if (it + 2 < n_tiles) FA_LOAD(1, (it + 2) * KT, cur_, it + 2);                                  \
      }                                                                                                 \
    }                                                                                                   \
  } while (0)

  for (;;) {   // over this workgroup's query tiles (the streaming form has one)
    const int q0 = qtile * QT + wave * 32;
    if constexpr (!RES) {
      FA_LOAD(0, 0, 0, 0);
      FA_LOAD(1, 0, 0, 0);
      if (n_tiles > 1) {
        FA_LOAD(0, KT, 1, 1);
        FA_LOAD(1, KT, 1, 1);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // tile 0 has landed (once per kernel: also waits tile 1)
      lds_barrier();
    }
    FA_QK(s_a, 0);
    if constexpr (!RES) lds_barrier();                    // K of tile 0 may now be overwritten (by tile 2)

    int it = 0;
    for (; it + 2 < n_tiles; it += 2) {
      FA_ITER(true, s_a, s_b);
      ++it;
      FA_ITER(true, s_b, s_a);
      --it;
    }
    // ---- one or two tiles left; the last one masks the keys past the end
    auto mask_tail = [&](floatx16 (&sc)[2]) {
      const int key0 = it * KT;
      if (key0 + KT > Lk) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (key >= Lk) sc[kt][r] = -INFINITY;
          }
      }
    };
    if (it + 1 < n_tiles) {
      FA_ITER(true, s_a, s_b);
      ++it;
      mask_tail(s_b);
      FA_ITER(false, s_b, s_a);
    } else {
      mask_tail(s_a);
      FA_ITER(false, s_a, s_b);
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
      if (p.lse && lh == 0) p.lse[tok * p.H + h] = m_ref * p.scale + __logf(l_tot);
    }
    if constexpr (!RES) {
      break;
    } else {
      if (++qtile >= qt_end) break;
      // next query tile of the run: fresh queries (their reference column is zero again), empty sums
      // (fetching them earlier, under the last key tile, costs 20 registers the kernel does not have:
      // measured with the spills it causes, 0.131 ms against 0.109 ms; the second wavefront of the
      // SIMD covers the wait instead)
      load_q(qtile * QT + wave * 32);
#pragma unroll
      for (int d = 0; d < C::DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
      m_ref = 0.f;
      l_run = 0.f;
    }
  }
#undef FA_ITER
#undef FENCE
#undef FA_QK
#undef FA_LOAD
}

template <int DH, int NW, bool RES>
int launch_dh(const FlashParams &p, int64_t blocks, hipStream_t s) {
  using C = Cfg<DH>;
  constexpr int smem = (RES ? RES_TILES : 2) * C::STAGE;
  static_assert(smem <= 160 * 1024, "the stages must fit the LDS");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_flash_attn<DH, NW, RES>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return ddit::hip_fail(e, "flash hipFuncSetAttribute");
    attr_set = true;
  }
  if (blocks > 0x7fffffff) { ddit::set_error("attention: too many workgroups"); return -2; }
  hipLaunchKernelGGL((k_flash_attn<DH, NW, RES>), dim3((unsigned)blocks), dim3(64 * NW), smem, s, p);
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
  p.rebase = 8.0f / p.scale_log2;
  p.q_norm_g = reinterpret_cast<const bf16_t *>(a.q_norm_g);
  p.q_norm_eps = a.q_norm_eps;
  if ((int64_t)a.n_groups * a.H > 0x3fffffff) {
    set_error("attention grid too large (groups=%d heads=%d)", a.n_groups, a.H);
    return -2;
  }
  p.n_units = a.n_groups * a.H;
  p.n_chunks = 1; p.qtiles_per_chunk = 1;
  // Short key sequences shared by long query sequences (cross-attention to the text): the resident
  // form, when every workgroup gets a run of at least four query tiles to spread the one-off K/V
  // fetch over.  One workgroup per CU: as many chunks per unit as that allows.
  const int res_qtiles = (a.Lq + 32 * RES_NW - 1) / (32 * RES_NW);
  int chunks = ddit::device_cus() / (p.n_units > 0 ? p.n_units : 1);
  if (chunks < 1) chunks = 1;
  if (a.Lk_max <= RES_TILES * KT && res_qtiles >= 4 * chunks) {
    p.n_qtiles = res_qtiles;
    p.qtiles_per_chunk = (res_qtiles + chunks - 1) / chunks;
    p.n_chunks = (res_qtiles + p.qtiles_per_chunk - 1) / p.qtiles_per_chunk;
    p.spread = 0;
    const int64_t blocks = (int64_t)p.n_units * p.n_chunks;
    if (a.dh == 72) return launch_dh<72, RES_NW, true>(p, blocks, s);
    if (a.dh == 64) return launch_dh<64, RES_NW, true>(p, blocks, s);
  }
  p.n_qtiles = (a.Lq + 32 * STREAM_NW - 1) / (32 * STREAM_NW);
  p.spread = p.n_units < 64;
  const int64_t blocks = (p.spread ? (int64_t)p.n_units : (int64_t)((p.n_units + 7) / 8) * 8) * p.n_qtiles;
  if (a.dh == 72) return launch_dh<72, STREAM_NW, false>(p, blocks, s);
  if (a.dh == 64) return launch_dh<64, STREAM_NW, false>(p, blocks, s);
  set_error("dh=%d: supported head dims are 64 and 72", a.dh);
  return -2;
}

}  // namespace ddit
