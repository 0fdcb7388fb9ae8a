// bf16 Linear  out = u W^T + b  on the CDNA4 matrix cores, with fused epilogues.
//
// u is [N,k] tokens x in-features, W is [n,k]: both operands have the contraction axis
// contiguous, which is exactly what v_mfma_f32_32x32x16_bf16 wants in its registers
// (8 consecutive k per lane), so tiles go global -> LDS -> registers as 16-byte pieces
// with no transposition anywhere.
//
// Tiling.  A workgroup of WGM x WGN wavefronts owns a BM x BN tile of the output (BM tokens,
// BN out-features); a wavefront owns TM x TN MFMA tiles of 32x32 with fp32 accumulators in
// registers.  The MFMA is issued with W as its first operand and u as its second, so a lane
// ends up holding, for one token, 4 consecutive out-features per accumulator group.
// The main configuration is 192 x 384 with eight wavefronts (2 x 4, each 96 x 96): the
// accumulators fill half of the compute unit's register file.  What sets the tile size is the
// path from L2 into the compute units: it delivers well under 100 bytes per clock to a CU, so a
// tile has to do about 128 flop per byte fetched, which 192 x 384 does (and 384 divides the
// model's widths 1152, 3456 and 4608).  Two wavefronts share a SIMD: one wavefront alone can draw
// only about 30 B/clk from the LDS, less than its matrix core eats.
//
// Operand path.  k is walked in steps of 32.  Tiles go global -> LDS with 16-byte
// global_load_lds: no staging registers, no ds_write, and the loads of k-step i+NS-1 are in
// flight while k-step i is multiplied (NS LDS stages of (BM+BN) rows x 64 B).  A wave-wide
// load places lane l's piece at LDS base + 16 l, i.e. 16 consecutive 64-byte rows.  The LDS
// of this chip has 64 banks (256 B per clock): the four 16-byte chunks of row r are stored
// at slot chunk ^ ((r >> 2) & 3), so the 16 lanes that a ds_read_b128 serves per clock (16
// consecutive rows, same chunk) touch 16 different 16-byte bank groups.  Since the load
// instruction fixes where each lane's piece lands, the swizzle is applied to the GLOBAL
// address each lane fetches from.  The (BM+BN)/16 loads of a k-step are dealt to the wavefronts
// round-robin; when they do not divide evenly the first wavefronts issue one more, and the k
// loop is compiled once per count, because completion is tracked with the vector-memory
// counter, which retires loads in order: before the barrier of k-step i each wave waits until
// at most its loads of the later k-steps are outstanding, so past the barrier stage i+1 is
// complete.  A k tail (k not a multiple of 32) is zero-filled by pointing the lanes past
// the end of the row at a block of zeros.
//
// Tile order.  Persistent workgroups; see tile_sequence_index.
//
// Epilogue.  The accumulators are staged through LDS (free once the k loop is done), 32 rows
// per wavefront at a time, so that global memory is written in whole-row pieces, 16 bytes per
// lane, instead of 8-byte pieces scattered over 32 rows: bf16 store; GELU(tanh form) + bf16
// store; gated residual update of the fp32 stream (x += gate_b * (acc + bias)), optionally
// also storing bf16(x).
#include "ddit_common.hpp"

#include <cmath>
#include <type_traits>

namespace {

constexpr int BK = 32;        // k per pipeline step (bf16 elements)
constexpr int ROW = 64;       // bytes per LDS row

__device__ __attribute__((aligned(16))) const unsigned int k_zero_block[4] = {0u, 0u, 0u, 0u};

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

// A grouped launch: one token matrix u against G weight matrices of the same shape [group_n, k], each
// with its own bias and its own output (the text k|v projections of all layers of a step).  To the
// tile loop it is one problem with G * group_n out-features; a tile lies inside one group
// (group_n is a multiple of the tile's columns), whose pointers it takes from this table.
constexpr int MAX_GROUPS = 128;
struct GroupTable {
  int group_n;
  const bf16_t *W[MAX_GROUPS];
  const bf16_t *bias[MAX_GROUPS];
  bf16_t *out[MAX_GROUPS];
};
struct NoGroups {};

__device__ __forceinline__ float gelu_tanh_f(float u) {
  // 0.5 u (1 + tanh(z)) == u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3)
  const float kA = -2.0f * 0.7978845608028654f * 1.4426950408889634f;  // -2 sqrt(2/pi) log2(e)
  const float t = u * u;
  const float z2 = u * (kA + (kA * 0.044715f) * t);                    // -2 z log2(e)
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z2));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for the
// epilogue's global stores of the previous tile to be acknowledged; nothing in this kernel
// communicates through global memory inside a workgroup.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// 16-byte LDS reads that the compiler does not see as LDS reads.  It guards every LDS read it
// knows of with a wait for ALL outstanding vector-memory operations (it cannot tell the
// direct-to-LDS loads from stores), which in the epilogues would make each read wait for the round
// trip of the stores issued just before it.  The epilogues read only what the workgroup itself
// staged behind a barrier, so no vector-memory wait is needed there.
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ unsigned lds_offset(const void *p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ void lds_read2_b128(uintx4 (&v)[2], unsigned a0, unsigned a1) {
  asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(v[0]), "=&v"(v[1])
               : "v"(a0), "v"(a1)
               : "memory");
}
__device__ __forceinline__ void lds_read3_b128(uintx4 (&v)[3], unsigned a0, unsigned a1, unsigned a2) {
  asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %4\n\tds_read_b128 %2, %5\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2])
               : "v"(a0), "v"(a1), "v"(a2)
               : "memory");
}
// the tile's bias for this lane: 4 consecutive features (8 bytes) at each of four 8-feature steps
__device__ __forceinline__ void lds_read4_b64(uint2 (&v)[4], unsigned a) {
  asm volatile(
      "ds_read_b64 %0, %4\n\tds_read_b64 %1, %4 offset:16\n\tds_read_b64 %2, %4 offset:32\n\t"
      "ds_read_b64 %3, %4 offset:48\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
      : "v"(a)
      : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "the counter has 6 bits");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
#define SG_MFMA 0x008
#define SG_VMEM_RD 0x020
#define SG_DS_RD 0x100

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

template <int WGM, int WGN, int TM, int TN, int NS>
struct GemmCfg {
  static constexpr int WGM_ = WGM;
  static constexpr int NW = WGM * WGN;                       // wavefronts per workgroup
  static constexpr int NT = 64 * NW;
  static constexpr int BM = WGM * TM * 32;
  static constexpr int BN = WGN * TN * 32;
  static constexpr int STAGE = (BM + BN) * ROW;
  static constexpr int MAIN_BYTES = NS * STAGE;
  static constexpr int PASS_ROWS = WGM * 32;                 // rows staged per pass of the fp32 epilogue
  static constexpr int PITCH_BF16 = BN * 2 + 16;             // epilogue staging row pitches
  static constexpr int PITCH_F32 = BN * 4 + 16;
  static constexpr int EPI_BYTES = PASS_ROWS * PITCH_F32;
  static constexpr int SMEM = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
  static constexpr int GATE_BYTES = 2 * BN * 4;              // gate vectors of two samples, past the stages
  static constexpr int BIAS_BYTES = BN * 2;                  // the tile's bias, past the gates
  static constexpr int EXTRA_BYTES = GATE_BYTES + BIAS_BYTES;
  // the bf16 epilogues stage one row-tile of every wavefront at a time inside the LAST TWO stages,
  // so that the first stages can already receive the next tile's operands
  static constexpr int EARLY_STEPS = NS - 2;                 // k-steps of the next tile fetched before the epilogue
  static constexpr int BF16_STAGING = EARLY_STEPS * STAGE;
  static_assert(PASS_ROWS * PITCH_BF16 <= 2 * STAGE, "a pass of the bf16 epilogue must fit two stages");
  static_assert(BN / 8 <= 64, "one wavefront fetches the tile's bias");
  static constexpr int NI = (BM + BN) / 16;                  // wave-wide loads per k-step (16 rows each)
  static constexpr int NJ_LO = NI / NW;                      // loads per wavefront per k-step ...
  static constexpr int N_HI = NI % NW;                       // ... one more for the first N_HI wavefronts
  static constexpr int NJ_HI = NJ_LO + (N_HI ? 1 : 0);
  static_assert(BM % 16 == 0 && BN % 16 == 0, "tile rows come in sixteens");
  static_assert((NS - 2) * NJ_HI < 64 && NS >= 3, "pipeline depth");
};

// Epilogue of one output tile.  acc[a][b][4g+e] = C[token tb + l32][feature fb + 8g + 4 lh + e]
// (bias already inside).  Pass b stages accumulator row-tile b of every wavefront (32 rows per
// wavefront row) and writes those rows out.  `smem` is free once the k loop is done; the caller
// guarantees no read of it is pending.  Ends with every thread past a barrier after its last read
// of the staging area.
template <class C, int TM, int TN, int EPI>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[TN][TM], unsigned char *smem, const float *smem_gate,
                                              const GemmParams &p, int64_t my_row0, int my_col0, int64_t my_sample0,
                                              int tid, int wm, int wn, int l32, int lh, bf16_t *my_out, int my_shift) {
  constexpr int BN = C::BN, NT = C::NT, PR = C::PASS_ROWS;
  const unsigned stage_base = lds_offset(smem);
  const int rl_stage = wm * 32 + l32;   // this lane's row inside a pass
  if constexpr (EPI != 2) {
    // Pass b: every wavefront stages its row-tile b (32 token rows x its features); everyone writes
    // those WGM*32 rows out.
    constexpr int CPR = BN / 8;   // 16-byte chunks per tile row
    constexpr int ITERS = PR * CPR / NT;
    static_assert(PR * CPR % NT == 0 && (ITERS == 4 || ITERS == 6), "row pieces per thread and pass");
    constexpr int G = ITERS / 2;  // pieces per LDS read group
    unsigned char *const stg = smem + C::BF16_STAGING;
    const unsigned stg_base = lds_offset(stg);
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      // bias is inside; (+ GELU), round to bf16, stage
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int fl = wn * (TN * 32) + a * 32 + 8 * g + 4 * lh;   // feature inside the tile
          float v0 = acc[a][b][4 * g + 0], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2],
                v3 = acc[a][b][4 * g + 3];
          if (EPI == 1) {
            v0 = gelu_tanh_f(v0); v1 = gelu_tanh_f(v1); v2 = gelu_tanh_f(v2); v3 = gelu_tanh_f(v3);
          }
          bf16x4 o;
          o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
          *reinterpret_cast<bf16x4 *>(stg + rl_stage * C::PITCH_BF16 + fl * 2) = o;
        }
      lds_barrier();
#pragma unroll
      for (int it0 = 0; it0 < ITERS; it0 += G) {
        uintx4 piece[G];
        unsigned la[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const int idx = tid + NT * (it0 + j);
          const int rl = idx / CPR, c = idx - rl * CPR;
          la[j] = stg_base + rl * C::PITCH_BF16 + c * 16;
        }
        if constexpr (G == 2) lds_read2_b128(piece, la[0], la[1]);
        else lds_read3_b128(piece, la[0], la[1], la[2]);
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const int idx = tid + NT * (it0 + j);
          const int rl = idx / CPR, c = idx - rl * CPR;          // rl = 32 * wave-row + row
          const int64_t tok = my_row0 + (rl >> 5) * (TM * 32) + b * 32 + (rl & 31);
          const int f = my_col0 + c * 8;
          // streaming store: the output is not read again by this launch, and a plain store would push
          // the operand lines that other workgroups still re-read out of the L2
          if (tok < p.N && f < p.n)
            __builtin_nontemporal_store(piece[j], reinterpret_cast<uintx4 *>(my_out + tok * p.ld_out + (f - my_shift)));
        }
      }
      lds_barrier();   // staged rows are read by other waves until here
    }
  } else {
    // gated residual: gate * (acc + bias) is staged; the update of x happens on the way out, on
    // whole-row pieces
    constexpr int CPR = BN / 4;       // float4 chunks per tile row
    constexpr int ITERS = PR * CPR / NT;
    static_assert(PR * CPR % NT == 0 && ITERS % 2 == 0, "row pieces must divide evenly over the threads, in pairs");
    const int64_t sample1_tok = (my_sample0 + 1) * p.tokens_per_sample;   // first token of the tile's second sample
    float *const x_tile = p.resid + my_row0 * (int64_t)p.n + my_col0;
    // The reads of x run DEPTH groups (of G row pieces per thread) ahead of their use, across the
    // passes: memory requests complete in order, loads and stores alike, so a group's loads are
    // issued BEFORE the stores of the groups processed while they are in flight, and waiting for
    // them never waits for a store.  The piece indices start from an opaque copy of the thread
    // index: otherwise the compiler hoists every address out of the tile loop and keeps them in
    // registers across the k loop.
    constexpr int G = ITERS % 4 == 0 ? 4 : 2;
    constexpr int GP = ITERS / G;            // groups per pass
    constexpr int NG = TM * GP;              // groups per tile
    constexpr int DEPTH = NG < 3 ? NG : 3;
    int tq = tid;
    asm volatile("" : "+v"(tq));
    float4 xr[DEPTH][G];
    auto issue_x = [&](int g, int slot) {
      const int b = g / GP, u0 = (g - b * GP) * G;
      int tg = tq;
      asm volatile("" : "+v"(tg));   // per group: nothing of its index arithmetic is shared or kept
#pragma unroll
      for (int j = 0; j < G; ++j) {
        const int idx = tg + NT * (u0 + j);
        const int rl = idx / CPR, c = idx - rl * CPR;
        const int trow = (rl >> 5) * (TM * 32) + b * 32 + (rl & 31);   // row inside the tile
        const bool ok = my_row0 + trow < p.N && my_col0 + c * 4 < p.n;
        xr[slot][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok) {   // x is touched once per launch: streaming load and store keep it out of the operands' way
          const floatx4 t = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(x_tile + (trow * p.n + c * 4)));
          xr[slot][j] = make_float4(t[0], t[1], t[2], t[3]);
        }
      }
    };
#pragma unroll
    for (int g = 0; g < DEPTH; ++g) issue_x(g, g);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      {
        const int64_t tok = my_row0 + wm * (TM * 32) + b * 32 + l32;
        const int64_t ds = tok - sample1_tok;                      // >= 0: second sample of the tile (or beyond)
        const bool far = p.gate_tab && ds >= p.tokens_per_sample;  // tile over more than two samples (tiny shapes)
        const float *grow = smem_gate + (ds >= 0 ? BN : 0);
        const float *gfar = nullptr;                               // this row's c6 gate vector when `far`
        if (far && p.gate_c6) {
          int64_t smp = my_sample0 + 1, t = sample1_tok + p.tokens_per_sample;
          const int64_t tk = tok < p.N ? tok : p.N - 1;
          while (t <= tk) { ++smp; t += p.tokens_per_sample; }
          // rows past the end of a problem that ends inside the tile's first sample would name a
          // sample that does not exist (their result is never stored, but the read must stay inside c6)
          const int64_t last = (p.N - 1) / p.tokens_per_sample;
          if (smp > last) smp = last;
          gfar = p.gate_c6 + smp * p.gate_c6_stride;
        }
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int fl = wn * (TN * 32) + a * 32 + 8 * g + 4 * lh;
            float4 gt = make_float4(1.f, 1.f, 1.f, 1.f);
            if (p.gate_tab) {
              gt = *reinterpret_cast<const float4 *>(grow + fl);
              if (far) {
                int f = my_col0 + fl;
                if (f > p.n - 4) f = p.n - 4;
                gt = *reinterpret_cast<const float4 *>(p.gate_tab + f);
                if (gfar) {
                  const float4 gc = *reinterpret_cast<const float4 *>(gfar + f);
                  gt.x += gc.x; gt.y += gc.y; gt.z += gc.z; gt.w += gc.w;
                }
              }
            }
            *reinterpret_cast<float4 *>(smem + rl_stage * C::PITCH_F32 + fl * 4) =
                make_float4(acc[a][b][4 * g + 0] * gt.x, acc[a][b][4 * g + 1] * gt.y, acc[a][b][4 * g + 2] * gt.z,
                            acc[a][b][4 * g + 3] * gt.w);
            __builtin_amdgcn_sched_barrier(0);   // keeps the gate reads from piling up in registers
          }
      }
      lds_barrier();
      // update of x on whole-row pieces
#pragma unroll
      for (int i = 0; i < GP; ++i) {
        const int g = b * GP + i, slot = g % DEPTH, u0 = i * G;
        uintx4 piece[G];
        int tg = tq;
        asm volatile("" : "+v"(tg));
#pragma unroll
        for (int j = 0; j < G; j += 2) {
          uintx4 two[2];
          unsigned la[2];
#pragma unroll
          for (int e2 = 0; e2 < 2; ++e2) {
            const int idx = tg + NT * (u0 + j + e2);
            const int rl = idx / CPR, c = idx - rl * CPR;
            la[e2] = stage_base + rl * C::PITCH_F32 + c * 16;
          }
          lds_read2_b128(two, la[0], la[1]);
          piece[j] = two[0];
          piece[j + 1] = two[1];
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const int idx = tg + NT * (u0 + j);
          const int rl = idx / CPR, c = idx - rl * CPR;
          const int trow = (rl >> 5) * (TM * 32) + b * 32 + (rl & 31);   // row inside the tile
          if (my_row0 + trow < p.N && my_col0 + c * 4 < p.n) {
            float4 r = xr[slot][j];
            r.x += __uint_as_float(piece[j][0]); r.y += __uint_as_float(piece[j][1]);
            r.z += __uint_as_float(piece[j][2]); r.w += __uint_as_float(piece[j][3]);
            floatx4 rv;
            rv[0] = r.x; rv[1] = r.y; rv[2] = r.z; rv[3] = r.w;
            __builtin_nontemporal_store(rv, reinterpret_cast<floatx4 *>(x_tile + (trow * p.n + c * 4)));
            if (p.out) {
              bf16x4 o;
              o[0] = (bf16_t)r.x; o[1] = (bf16_t)r.y; o[2] = (bf16_t)r.z; o[3] = (bf16_t)r.w;
              __builtin_nontemporal_store(o, reinterpret_cast<bf16x4 *>(p.out + (my_row0 + trow) * p.ld_out + my_col0 + c * 4));
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (g + DEPTH < NG) issue_x(g + DEPTH, slot);
        __builtin_amdgcn_sched_barrier(0);
      }
      lds_barrier();   // the staging area is rewritten by the next pass / the next tile's loads
    }
  }
}

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef __attribute__((address_space(1))) const void *gbl_ptr_t;

template <int NJ_>
struct LoadCount { static constexpr int value = NJ_; };

template <int WGM, int WGN, int TM, int TN, int NS, int EPI, class GT>
__global__ __launch_bounds__(WGM *WGN * 64, 2) void k_gemm_bf16(GemmParams p, GT gt) {
  using C = GemmCfg<WGM, WGN, TM, TN, NS>;
  constexpr bool GROUPED = !std::is_same<GT, NoGroups>::value;
  static_assert(!GROUPED || EPI != 2, "grouped launches write bf16 outputs");
  constexpr int BM = C::BM, BN = C::BN, STAGE = C::STAGE, NW = C::NW;
  constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
  constexpr int AHEAD = NS - 1;          // k-steps in flight ahead of the one being multiplied
  // The bf16 epilogues stage in the last two LDS stages only, so the next tile's first k-steps are
  // fetched while the current tile is written out; the fp32 epilogue needs the whole LDS.
  constexpr bool EARLY_FETCH = EPI != 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *smem_gate = reinterpret_cast<float *>(smem + C::SMEM);
  unsigned char *smem_bias = smem + C::SMEM + C::GATE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave - wm * WGN;
  const int l32 = lane & 31, lh = lane >> 5;
  const int nk = (p.k + BK - 1) / BK;
  const int nk_full = p.k / BK;

  // fragment reads: row (tile*32 + l32) of 64 B, chunk (2 kk + lh) at slot chunk ^ ((row >> 2) & 3)
  const int frag_u = (wm * (TM * 32) + l32) * ROW;
  const int frag_w = BM * ROW + (wn * (TN * 32) + l32) * ROW;
  int coff[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) coff[kk] = ((kk * 2 + lh) ^ ((l32 >> 2) & 3)) << 4;
  // loads: this wave's j-th instruction is number g = wave + NW j of the k-step and covers tile rows
  // 16 g .. 16 g + 15 (token rows first, then W rows); this lane: row lane/4, slot lane%4
  const int ld_row = lane >> 2;
  const int ld_chunk = ((lane & 3) ^ ((ld_row >> 2) & 3)) * 8;   // element offset of the global chunk to fetch
  const unsigned bias_lds = lds_offset(smem_bias) + (wn * (TN * 32) + 4 * lh) * 2;

  // W, bias, output and first out-feature of the problem that the tile being FETCHED belongs to
  const bf16_t *W_tile = p.W, *bias_tile = p.bias;
  bf16_t *out_tile = p.out;
  int shift_tile = 0;

  // The whole tile loop, compiled per NJ = this wavefront's loads per k-step.
  auto run = [&](auto nj_tag) {
    constexpr int NJ = decltype(nj_tag)::value;
    constexpr int PENDING = (NS - 2) * NJ;   // loads that may still be outstanding when k-step i+1 is needed
    int src_off[NJ];                         // element offset of this lane's piece at k = 0 (u or W, by instruction)

#define DL_ISSUE(KT, ST)                                                                           \
  do {                                                                                             \
    const int k0_ = (KT) * BK;                                                                     \
    unsigned char *sb_ = smem + (ST) * STAGE + wave * 1024;                                        \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                               \
      const bf16_t *src_ = ((wave + NW * j) * 16 < BM ? p.u : W_tile) + src_off[j] + k0_;          \
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src_, (lds_ptr_t)(sb_ + j * (NW * 1024)), 16, 0, 0); \
    }                                                                                              \
  } while (0)

    // the last, partial k-step: lanes whose chunk starts at or past k fetch zeros instead
#define DL_ISSUE_TAIL(KT, ST)                                                                      \
  do {                                                                                             \
    const int k0_ = (KT) * BK;                                                                     \
    const bool in_ = k0_ + ld_chunk < p.k;                                                         \
    unsigned char *sb_ = smem + (ST) * STAGE + wave * 1024;                                        \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                               \
      const bf16_t *src_ = ((wave + NW * j) * 16 < BM ? p.u : W_tile) + src_off[j] + k0_;          \
      if (!in_) src_ = reinterpret_cast<const bf16_t *>(k_zero_block);                             \
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)src_, (lds_ptr_t)(sb_ + j * (NW * 1024)), 16, 0, 0); \
    }                                                                                              \
  } while (0)

#define DL_READ_FRAGS(BUF, ST, KK)                                                                 \
  do {                                                                                             \
    const unsigned char *sb_ = smem + (ST) * STAGE + coff[KK];                                     \
    _Pragma("unroll") for (int b = 0; b < TM; ++b)                                                 \
        uf[BUF][b] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_u + b * 32 * ROW);               \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        wf[BUF][a] = *reinterpret_cast<const bf16x8 *>(sb_ + frag_w + a * 32 * ROW);               \
  } while (0)

#define DL_MFMAS(BUF)                                                                              \
  do {                                                                                             \
    _Pragma("unroll") for (int a = 0; a < TN; ++a)                                                 \
        _Pragma("unroll") for (int b = 0; b < TM; ++b)                                             \
            acc[a][b] = mfma32(wf[BUF][a], uf[BUF][b], acc[a][b]);                                 \
  } while (0)

#define NEXT_STAGE(S) ((S) + 1 == NS ? 0 : (S) + 1)

    // Start of a tile's operand stream: source offsets, the tile's bias (one wavefront fetches it,
    // ahead of everything else, so it has landed when k-step 0 has), k-steps 0 .. AHEAD-1.
    auto begin_tile = [&](int64_t row0, int col0, int first_steps) {
      int n_lim = p.n;             // out-features of the tile's problem
      if constexpr (GROUPED) {
        const int g = col0 / gt.group_n;
        W_tile = gt.W[g]; bias_tile = gt.bias[g]; out_tile = gt.out[g];
        shift_tile = g * gt.group_n;
        n_lim = gt.group_n;
      }
      const int lcol0 = col0 - shift_tile;   // the tile's first out-feature inside its problem
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int R = (wave + NW * j) * 16 + ld_row;
        if (R < BM) {
          int64_t t = row0 + R;
          if (t > p.N - 1) t = p.N - 1;           // overhanging rows re-read the last row; never stored
          src_off[j] = (int)(t * p.ld_u) + ld_chunk;
        } else {
          int f = lcol0 + R - BM;
          if (f > n_lim - 1) f = n_lim - 1;
          src_off[j] = f * p.k + ld_chunk;
        }
      }
      if (bias_tile && wave == 0 && lane < BN / 8) {
        int f = lcol0 + lane * 8;
        if (f > n_lim - 8) f = n_lim - 8;         // overhanging features: a valid address, never stored
        __builtin_amdgcn_global_load_lds((gbl_ptr_t)(bias_tile + f), (lds_ptr_t)smem_bias, 16, 0, 0);
      }
#pragma unroll
      for (int s = 0; s < AHEAD; ++s) {
        if (s >= first_steps) break;
        if (s < nk_full) DL_ISSUE(s, s);
        else if (s < nk) DL_ISSUE_TAIL(s, s);
      }
    };
    // the remaining k-steps of the first AHEAD, once the epilogue has left the last stages
    auto finish_begin = [&](int first_steps) {
#pragma unroll
      for (int s = 0; s < AHEAD; ++s) {
        if (s < first_steps) continue;
        if (s < nk_full) DL_ISSUE(s, s);
        else if (s < nk) DL_ISSUE_TAIL(s, s);
      }
    };

    int tile = tile_sequence_index(p, 0);
    if (tile < 0) return;
    int tile_m, tile_n;
    decode_tile(p, tile, tile_m, tile_n);
    int64_t row0 = (int64_t)tile_m * BM;
    int col0 = tile_n * BN;
    begin_tile(row0, col0, AHEAD);

    for (int round = 0;; ++round) {
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
      // k-step 0 (and the bias) must have landed; up to AHEAD-1 later steps may be pending
      if (nk >= AHEAD) wait_vmcnt<PENDING>();
      else wait_vmcnt<0>();
      lds_barrier();

      // the accumulators start from the bias
      floatx16 acc[TN][TM];
#pragma unroll
      for (int a = 0; a < TN; ++a) {
        uint2 bq[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) bq[g] = make_uint2(0u, 0u);
        if (GROUPED ? bias_tile != nullptr : p.bias != nullptr) lds_read4_b64(bq, bias_lds + a * 64);
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            acc[a][b][4 * g + 0] = __uint_as_float(bq[g].x << 16);
            acc[a][b][4 * g + 1] = __uint_as_float(bq[g].x & 0xffff0000u);
            acc[a][b][4 * g + 2] = __uint_as_float(bq[g].y << 16);
            acc[a][b][4 * g + 3] = __uint_as_float(bq[g].y & 0xffff0000u);
          }
      }

      bf16x8 uf[2][TM], wf[2][TN];
      DL_READ_FRAGS(0, 0, 0);
      int kt = 0;
      int st = 0;                 // stage of k-step kt
      int st_new = AHEAD;         // stage that k-step kt + AHEAD goes to (== stage of kt-1)
      // ---- steady state: k-step kt + AHEAD exists and is a full step; no branches, issue order pinned.
      // Each half issues one MFMA first, then the LDS reads of the NEXT half's fragments, then the
      // rest: the wait that the compiler places before the first MFMA (it always waits for every
      // LDS read issued so far) then covers only reads issued a whole half earlier.
      for (; kt + AHEAD < nk_full; ++kt) {
        const int st_next = NEXT_STAGE(st);
        DL_READ_FRAGS(1, st, 1);
        DL_ISSUE(kt + AHEAD, st_new);
        DL_MFMAS(0);
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
        __builtin_amdgcn_sched_group_barrier(SG_DS_RD, NFRAG, 0);
        sched_interleave<SG_VMEM_RD, 0, NMFMA - 1, NJ>();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<PENDING>();        // k-step kt+1 has landed (this wave's part); kt+2 .. kt+AHEAD may be pending
        lds_barrier();                // ... everyone's part; and every wave is done reading stage kt
        DL_READ_FRAGS(0, st_next, 0);
        DL_MFMAS(1);
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
        __builtin_amdgcn_sched_group_barrier(SG_DS_RD, NFRAG, 0);
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, NMFMA - 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        st_new = st;
        st = st_next;
      }
      // ---- last k-steps: at most one more load (the partial step), then drain
      for (; kt < nk; ++kt) {
        const int st_next = NEXT_STAGE(st);
        DL_READ_FRAGS(1, st, 1);
        if (kt + AHEAD < nk) DL_ISSUE_TAIL(kt + AHEAD, st_new);
        DL_MFMAS(0);
        wait_vmcnt<0>();
        lds_barrier();
        if (kt + 1 < nk) DL_READ_FRAGS(0, st_next, 0);
        DL_MFMAS(1);
        st_new = st;
        st = st_next;
      }
      // every wave is past the last barrier of the k loop: no LDS read of the stages is pending

      const int64_t my_row0 = row0;
      const int my_col0 = col0;
      bf16_t *const my_out = out_tile;
      const int my_shift = GROUPED ? shift_tile : 0;
      const int next = round + 1 < p.rounds ? tile_sequence_index(p, round + 1) : -1;
      if (next >= 0) {
        decode_tile(p, next, tile_m, tile_n);
        row0 = (int64_t)tile_m * BM;
        col0 = tile_n * BN;
        if (EARLY_FETCH) begin_tile(row0, col0, C::EARLY_STEPS);
      }
      gemm_epilogue<C, TM, TN, EPI>(acc, smem, smem_gate, p, my_row0, my_col0, sample0, tid, wm, wn, l32, lh, my_out, my_shift);
      if (next < 0) break;
      if (EARLY_FETCH) finish_begin(C::EARLY_STEPS);
      else begin_tile(row0, col0, AHEAD);
    }
#undef DL_ISSUE
#undef DL_ISSUE_TAIL
#undef DL_READ_FRAGS
#undef DL_MFMAS
#undef NEXT_STAGE
  };

  if constexpr (C::N_HI == 0) {
    run(LoadCount<C::NJ_LO>{});
  } else {
    if (wave < C::N_HI) run(LoadCount<C::NJ_HI>{});
    else run(LoadCount<C::NJ_LO>{});
  }
}

template <int WGM, int WGN, int TM, int TN, int NS, int EPI, class GT = NoGroups>
int launch_one(const GemmParams &p0, hipStream_t s, const GT &gt = GT()) {
  using C = GemmCfg<WGM, WGN, TM, TN, NS>;
  constexpr int LDS_BYTES = C::SMEM + C::EXTRA_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "the tile's stages must fit the LDS");
  // workgroups resident per CU: what the LDS holds, at most three of the four-wavefront tiles
  constexpr int LDS_FIT = (160 * 1024) / LDS_BYTES;
  constexpr int WG_PER_CU = C::NW > 4 ? 1 : (LDS_FIT > 3 ? 3 : (LDS_FIT < 1 ? 1 : LDS_FIT));
  GemmParams p = p0;
  const int64_t tiles_m = (p.N + C::BM - 1) / C::BM;
  p.tiles_m = (int)tiles_m;
  p.tiles_n = (p.n + C::BN - 1) / C::BN;
  // width of an out-feature group: at most 4 tiles (their W, about 3.5 MB at k = 1152, stays in an
  // XCD's 4 MB L2 next to the token panels streaming through), as even as the tile count allows
  const int max_w = 4;
  const int n_groups = (p.tiles_n + max_w - 1) / max_w;
  p.group_w = (p.tiles_n + n_groups - 1) / n_groups;
  const int64_t total = tiles_m * p.tiles_n;
  if (total > (int64_t)1 << 30) {
    ddit::set_error("linear: %lld output tiles: too many", (long long)total);
    return -2;
  }
  p.total_tiles = (int)total;
  // as many workgroups as the chip holds at once; a multiple of 8 so that every round gives
  // each XCD a contiguous run of tiles
  int grid = (ddit::device_cus() * WG_PER_CU) & ~7;
  if (grid < 8) grid = 8;
  if (total <= grid) grid = (int)((total + 7) & ~(int64_t)7);
  p.rounds = (int)(((total + 7) / 8 + grid / 8 - 1) / (grid / 8));
  static bool attr_set = false;  // benign race: the attribute is idempotent
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_bf16<WGM, WGN, TM, TN, NS, EPI, GT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return ddit::hip_fail(e, "gemm hipFuncSetAttribute");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_gemm_bf16<WGM, WGN, TM, TN, NS, EPI, GT>), dim3((unsigned)grid), dim3(C::NT), LDS_BYTES, s, p, gt);
  return ddit::hip_fail(hipGetLastError(), "gemm launch");
}

// ---------------------------------------------------------------------------------------------
// Tile choice.  Nine forms of the kernel are compiled: seven output tiles, and for 192 x 192 and
// 128 x 192 two depths of the operand ring.  With three stages two workgroups of these tiles fit a
// CU's LDS and one's epilogue runs under the other's k loop (192 x 192 at 48600 tokens: fc1 0.62 ->
// 0.52 ms); with four a workgroup that has the CU to itself hides more of the fetch latency (128 x
// 192 at 3680 tokens, k = 4608: 63 against 69 microseconds).  Which form is fastest depends on how the tile grid
// divides over the CUs far more than on the tile's own efficiency (a 192 x 384 tile runs its k
// loop at about twice the rate per flop of a 128 x 128 one, but 60 of them leave 196 CUs idle).
// The launcher therefore prices every tile with a small model of the kernel and takes the
// cheapest.  With  tiles = ceil(N / rows) * ceil(n / cols)  and  q = ceil(tiles / CUs)  tiles on
// the busiest CU,
//     t = (a * k / 1152 + e[epilogue]) * q / gain[min(q, workgroups per CU)]
//         * (1 + 0.29 * min(1, tiles / CUs)) + 0.63      [microseconds]
// a: one workgroup's k-loop time per 1152 of k with a CU to itself; e: its epilogue and set-up;
// gain: what sharing a CU between two or three resident workgroups returns; the load term is the
// clock and memory slow-down of a full chip against a single busy CU.  The constants are a
// least-squares fit (in log time) to a sweep of the model's five linears over 23 token counts
// from 288 to 48600 with every tile forced in turn (ddit_linear_fwd_tile): over that sweep the
// model's picks are within 0.4 % of the best tile's total time.  (The load term and the launch
// constant trade against each other in the fit and differ between machines of one type: 0.29 / 0.63
// and 0.40 / 0 fit equally well; the picks do not change.)
// ---------------------------------------------------------------------------------------------
struct TileModel {
  int rows, cols, wavefronts, stages, wg_per_cu;   // stages: depth of the operand ring in LDS
  float a;        // k-loop microseconds per 1152 of k, alone on a CU
  float e[3];     // epilogue + set-up microseconds: bf16 / GELU / gated residual
};
constexpr int N_TILES = 9;
constexpr TileModel TILES[N_TILES] = {
    {192, 384, 8, 4, 1, 22.07f, {4.65f, 7.82f, 18.53f}},
    {192, 288, 6, 4, 1, 18.75f, {4.28f, 6.87f, 15.69f}},
    {192, 256, 8, 4, 1, 15.69f, {3.24f, 5.16f, 12.01f}},
    {192, 192, 4, 3, 2, 15.24f, {2.74f, 4.34f, 11.08f}},
    {192, 192, 4, 4, 1, 13.11f, {4.12f, 5.94f, 12.41f}},
    {128, 192, 4, 3, 2, 12.84f, {0.67f, 1.71f, 6.39f}},
    {128, 192, 4, 4, 1, 10.97f, {1.40f, 2.71f, 7.46f}},
    {128, 128, 4, 4, 2, 8.91f, {1.20f, 1.75f, 5.35f}},
    {64, 128, 4, 4, 3, 6.59f, {0.36f, 0.62f, 2.33f}},
};
constexpr float CU_SHARE_GAIN[3] = {1.0f, 1.21f, 1.22f};
constexpr float FULL_CHIP_SLOWDOWN = 0.29f, LAUNCH_US = 0.63f;

float predicted_us(int tile, int epilogue, int64_t N, int n, int k, int cus) {
  const TileModel &t = TILES[tile];
  const double tiles = (double)((N + t.rows - 1) / t.rows) * (double)((n + t.cols - 1) / t.cols);
  const double q = std::ceil(tiles / cus);
  const int sharing = q < t.wg_per_cu ? (int)q : t.wg_per_cu;
  const double one = t.a * (double)k / 1152.0 + t.e[epilogue];
  const double load = 1.0 + FULL_CHIP_SLOWDOWN * (tiles < cus ? tiles / cus : 1.0);
  return (float)(one * q / CU_SHARE_GAIN[sharing > 0 ? sharing - 1 : 0] * load + LAUNCH_US);
}

int cheapest_tile(int epilogue, int64_t N, int n, int k, int cus) {
  int best = 0;
  float best_us = predicted_us(0, epilogue, N, n, k, cus);
  for (int t = 1; t < N_TILES; ++t) {
    const float us = predicted_us(t, epilogue, N, n, k, cus);
    if (us < best_us) { best_us = us; best = t; }
  }
  return best;
}

template <int WGM, int WGN, int TM, int TN, int NS, int EPI>
int launch_checked(int tile, const GemmParams &p, hipStream_t s) {
  using C = GemmCfg<WGM, WGN, TM, TN, NS>;
  // the model's table and the compiled tile must describe the same thing
  if (TILES[tile].rows != C::BM || TILES[tile].cols != C::BN || TILES[tile].wavefronts != C::NW ||
      TILES[tile].stages != NS) {
    ddit::set_error("linear: tile table entry %d does not match its kernel", tile);
    return -2;
  }
  return launch_one<WGM, WGN, TM, TN, NS, EPI>(p, s);
}

template <int EPI>
int launch_epi(int tile, const GemmParams &p, hipStream_t s) {
  if (tile < 0) tile = cheapest_tile(EPI, p.N, p.n, p.k, ddit::device_cus());
  switch (tile) {
    case 0: return launch_checked<2, 4, 3, 3, 4, EPI>(tile, p, s);
    case 1: return launch_checked<2, 3, 3, 3, 4, EPI>(tile, p, s);
    case 2: return launch_checked<2, 4, 3, 2, 4, EPI>(tile, p, s);
    case 3: return launch_checked<2, 2, 3, 3, 3, EPI>(tile, p, s);
    case 4: return launch_checked<2, 2, 3, 3, 4, EPI>(tile, p, s);
    case 5: return launch_checked<2, 2, 2, 3, 3, EPI>(tile, p, s);
    case 6: return launch_checked<2, 2, 2, 3, 4, EPI>(tile, p, s);
    case 7: return launch_checked<2, 2, 2, 2, 4, EPI>(tile, p, s);
    case 8: return launch_checked<2, 2, 1, 2, 4, EPI>(tile, p, s);
  }
  ddit::set_error("linear: no tile %d (there are %d)", tile, N_TILES);
  return -1;
}

}  // namespace

namespace ddit {

int gemm_tile_count() { return N_TILES; }

int gemm_tile_info(int tile, int *rows, int *cols, int *wavefronts, int *wg_per_cu) {
  if (tile < 0 || tile >= N_TILES) return -1;
  *rows = TILES[tile].rows; *cols = TILES[tile].cols;
  *wavefronts = TILES[tile].wavefronts; *wg_per_cu = TILES[tile].wg_per_cu;
  return 0;
}

int gemm_tile_choice(int epilogue, int64_t N, int n, int k, int cus, float *us_per_tile) {
  if (cus <= 0) cus = ddit::device_cus();
  if (us_per_tile)
    for (int t = 0; t < N_TILES; ++t) us_per_tile[t] = predicted_us(t, epilogue, N, n, k, cus);
  return cheapest_tile(epilogue, N, n, k, cus);
}

template <int WGM, int WGN, int TM, int TN, int NS>
int launch_grouped_tile(const GemmParams &p, const GroupTable &gt, hipStream_t s) {
  return launch_one<WGM, WGN, TM, TN, NS, 0, GroupTable>(p, s, gt);
}

// One launch for G problems that share u: out[g] = u W[g]^T + bias[g], every W[g] of shape [a.n, a.k].
// Returns 1 (nothing launched) when the shape cannot be grouped: the caller then launches them one by one.
int launch_gemm_grouped(const GemmArgs &a, int G, const void *const *W, const void *const *bias, void *const *out,
                        hipStream_t s) {
  if (a.N == 0 || a.n == 0 || G == 0) return 0;
  if (G < 2 || G > MAX_GROUPS || (int64_t)G * a.n >= (int64_t)1 << 30) return 1;
  if ((int64_t)a.n * a.k >= (int64_t)1 << 31 || a.N * a.ld_u >= (int64_t)1 << 31) return 1;
  // cheapest tile whose columns divide a problem's out-features (a tile must lie inside one problem)
  const int n_all = G * a.n, cus = device_cus();
  int tile = -1;
  float best = 0.f;
  for (int t = 0; t < N_TILES; ++t) {
    if (a.n % TILES[t].cols) continue;
    const float us = predicted_us(t, 0, a.N, n_all, a.k, cus);
    if (tile < 0 || us < best) { tile = t; best = us; }
  }
  if (tile < 0) return 1;
  GroupTable gt;
  gt.group_n = a.n;
  for (int g = 0; g < G; ++g) {
    gt.W[g] = reinterpret_cast<const bf16_t *>(W[g]);
    gt.bias[g] = bias ? reinterpret_cast<const bf16_t *>(bias[g]) : nullptr;
    gt.out[g] = reinterpret_cast<bf16_t *>(out[g]);
  }
  GemmParams p;
  p.u = reinterpret_cast<const bf16_t *>(a.u); p.ld_u = a.ld_u;
  p.W = gt.W[0]; p.bias = gt.bias[0];
  p.N = a.N; p.n = n_all; p.k = a.k;
  p.out = gt.out[0]; p.ld_out = a.ld_out;
  p.resid = nullptr; p.gate_tab = nullptr; p.gate_c6 = nullptr; p.gate_c6_stride = 0;
  p.tokens_per_sample = a.tokens_per_sample > 0 ? a.tokens_per_sample : 1;
  p.tiles_m = 0; p.tiles_n = 0; p.group_w = 1; p.total_tiles = 0; p.rounds = 0;
  switch (tile) {
    case 0: return launch_grouped_tile<2, 4, 3, 3, 4>(p, gt, s);
    case 1: return launch_grouped_tile<2, 3, 3, 3, 4>(p, gt, s);
    case 2: return launch_grouped_tile<2, 4, 3, 2, 4>(p, gt, s);
    case 3: return launch_grouped_tile<2, 2, 3, 3, 3>(p, gt, s);
    case 4: return launch_grouped_tile<2, 2, 3, 3, 4>(p, gt, s);
    case 5: return launch_grouped_tile<2, 2, 2, 3, 3>(p, gt, s);
    case 6: return launch_grouped_tile<2, 2, 2, 3, 4>(p, gt, s);
    case 7: return launch_grouped_tile<2, 2, 2, 2, 4>(p, gt, s);
    default: return launch_grouped_tile<2, 2, 1, 2, 4>(p, gt, s);
  }
}

int launch_gemm(int epilogue, const GemmArgs &a, hipStream_t s) {
  if (a.N == 0 || a.n == 0) return 0;
  if (a.tile >= N_TILES) {
    set_error("linear: no tile %d (there are %d)", a.tile, N_TILES);
    return -1;
  }
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
    case 0: return launch_epi<0>(a.tile, p, s);
    case 1: return launch_epi<1>(a.tile, p, s);
    case 2: return launch_epi<2>(a.tile, p, s);
  }
  set_error("unknown epilogue %d", epilogue);
  return -1;
}

}  // namespace ddit
