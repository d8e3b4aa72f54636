// Device-side building blocks shared by the block kernels: matrix-core (MFMA) tile
// primitives for gfx950, the register layout they imply, and the weight stream.
//
// Register-resident transposed chain
// ----------------------------------
// A wave owns tiles of 32 tokens.  Every activation of a transformer block
// (Section 3.4 / 3.5 of the paper: LayerNorm, Q/K/V projection, attention, output
// projection, FFN) stays in that wave's registers in one layout, the accumulator layout
// of a 32x32 MFMA computing OUT^T = W^T * X^T:
//
//     lane l = (j, hi) with j = l % 32 the token, hi = l / 32;
//     register r of feature tile t holds feature 32 t + 8 (r / 4) + 4 hi + (r % 4).
//
// An accumulator tile becomes the next GEMM's B operand without leaving registers: a
// "group" is 16 bytes per lane (8 bf16 or 4 fp32 = registers [EPL g, EPL (g+1)) of a
// tile), and since A and B of an MFMA only have to agree on which contraction slot means
// which k, the weights are packed on the host side of the launch (pack kernel) with the
// same slot -> feature permutation.  V is produced with the operands swapped
// (OUT = X * W, lane = feature, registers = tokens), which is exactly the A operand that
// O^T = V^T P^T needs, and S^T = K Q^T leaves the probabilities with lane = query,
// registers = keys, the B operand of that product.  Nothing is transposed through LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace longer {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;   // 4 waves, one per SIMD
constexpr int kWaves = 4;
constexpr float kNegBig = -1.0e30f;

// Element traits: one operand group = 16 bytes per lane.
template <typename T> struct ET;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// bf16 mode, second FFN GEMM: the activated hidden chunk and the W2 fragments are fp16 (same
// matrix-core rate as bf16, 11 significand bits instead of 8), so that the activation can be
// evaluated two elements per instruction in packed fp16.  The pack kernel stores W1 and b1
// divided by kFfnScale and W2 multiplied by it (powers of two: exact), which keeps the
// polynomial's argument and coefficients of order 1 in fp16:
//   act(x) W2 = (act(4 y) / 4) (4 W2),  y = x / 4 = LN2(.) (W1 / 4) + b1 / 4.
constexpr float kFfnScale = 4.0f;

template <> struct ET<float> {
  typedef f32x4 grp;
  static constexpr int EPL = 4;   // elements per lane per group
  static constexpr int GPT = 4;   // groups per 32-wide tile (16 accumulator registers)
  static constexpr int GF = 8;    // contraction features covered by one group (both lane halves)
  static __device__ __forceinline__ f32x16 mma(grp a, grp b, f32x16 c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[i], c, 0, 0, 0);
    return c;
  }
  static __device__ __forceinline__ grp pack(const f32x16& c, int g) {
    grp o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = c[4 * g + e];
    return o;
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
  // the second FFN GEMM's activated operand: the same fp32 groups
  static constexpr bool HALF_FFN = false;
  typedef grp hgrp;
  static __device__ __forceinline__ f32x16 mma_h(grp a, hgrp b, f32x16 c) { return mma(a, b, c); }
};

template <> struct ET<__bf16> {
  typedef bf16x8 grp;
  static constexpr int EPL = 8;
  static constexpr int GPT = 2;
  static constexpr int GF = 16;
  static __device__ __forceinline__ f32x16 mma(grp a, grp b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ grp pack(const f32x16& c, int g) {
    grp o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)c[8 * g + e];   // round to nearest even
    return o;
  }
  static __device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }
  static __device__ __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }
  // the second FFN GEMM runs on fp16 operands (see kFfnScale): `a` holds fp16 bits
  static constexpr bool HALF_FFN = true;
  typedef f16x8 hgrp;
  static __device__ __forceinline__ f32x16 mma_h(grp a, hgrp b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), b, c, 0, 0, 0);
  }
};

// feature (inside a 32-wide tile) held by accumulator register r of lane half hi
__host__ __device__ __forceinline__ constexpr int tile_row(int r, int hi) {
  return 8 * (r / 4) + 4 * hi + (r % 4);
}

// Lane l and lane l ^ 32 hold the two feature halves of one token.  Their values are
// combined with the cross-half register swap (v_permlane32_swap: the upper 32 lanes of one
// operand trade places with the lower 32 lanes of the other), no LDS round trip: with both
// operands = v, one result is v's lower half in every lane, the other v's upper half.
__device__ __forceinline__ void both_halves(float v, float& lo, float& up) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const unsigned b = __builtin_bit_cast(unsigned, v);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0); up = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float sum_halves(float v) { float a, b; both_halves(v, a, b); return a + b; }
__device__ __forceinline__ float max_halves(float v) { float a, b; both_halves(v, a, b); return fmaxf(a, b); }

// ------------------------------------------------------------------------------------
// Packed parameters of one block (written by the pack kernel, read by the block kernels)
//   segments: [Q: NT][K: NT][V: NT][O: NT][FFN: (W1 chunk c, W2 chunk c) for c < NC]
//   each segment = D/GF fragments of 1 KiB (64 lanes x 16 B), then the fp32 vectors.
struct VecLayout {
  int D, FF;
  __host__ __device__ int ln1_g() const { return 0; }
  __host__ __device__ int ln1_b() const { return D; }
  __host__ __device__ int bq() const { return 2 * D; }
  __host__ __device__ int bk() const { return 3 * D; }
  __host__ __device__ int bv() const { return 4 * D; }
  __host__ __device__ int bo() const { return 5 * D; }
  __host__ __device__ int ln2_g() const { return 6 * D; }
  __host__ __device__ int ln2_b() const { return 7 * D; }
  __host__ __device__ int b2() const { return 8 * D; }
  __host__ __device__ int b1() const { return 9 * D; }
  __host__ __device__ int total() const { return 9 * D + FF; }
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Packed parameters of one block travel as "segments" of D/GF fragments (1 KiB each: 64
// lanes x 16 B).  Layouts, all in exactly the order a kernel consumes them so that a launch
// reads one linear stream ("ffn" = the FFN part, see below; "vec" = one segment holding the
// block's fp32 vectors (VecLayout), zero padded):
//   FUSED  [vec][q0 k0 v0 q1 k1 v1 ...][o0 ..][ffn]                     (merge, scoring)
//   SPLIT  [vec][k0 v0 k1 v1 ...] then [vec][q0 q1 ..][o0 ..][ffn]      (K/V projection, attention)
//   MLP    [vec][ffn]                                (input generation: biases b1, b2 only)
// Pair layouts, for the kernels that give a 32-row tile to a pair of waves which split every GEMM
// by output tile (even tiles to one wave, odd tiles to the other): the same segments, each
// consecutive two being one even and one odd tile of the same matrix, after [vec][unused]:
//   PAIR_FUSED  [vec][unused][q0 q1][k0 k1][v0 v1][q2 q3][k2 k3][v2 v3] ... [o0 o1][o2 o3] ...
//               [w1(0) w1(1)][w2(0) w2(1)][w1(2) w1(3)][w2(2) w2(3)] ...
//   PAIR_ATTN   [vec][unused][q0 q1][q2 q3] ... [o0 o1] ... then the FFN part as above
// (as many segments as FUSED and the attention half of SPLIT; the weight stream's panels hold two
// segments there, so each panel has one segment of work for either wave).
// The FFN part holds the NC = FF/32 chunk pairs (W1 chunk c: d x 32, W2 chunk c: 32 x d) and one
// unused segment, 2 NC + 1 in all, in one of two orders:
//   plain   w1(0) w2(0) w1(1) w2(1) ... w1(NC-1) w2(NC-1) [unused]
//   skewed  w1(0) w1(1) [unused] {w2(0) w1(2)} {w2(1) w1(3)} ... {w2(NC-3) w1(NC-1)} {w2(NC-2) w2(NC-1)}
// The skewed order serves the software-pipelined FFN loop (bf16 kernels up to d = 128): iteration
// i runs the second GEMM of chunk i-1 and the first GEMM of chunk i+1 under the activation of
// chunk i, so it reads the pair {w2(i-1), w1(i+1)} at once.  The FFN part starts at an odd
// segment index of every stream (after vec and an even number of projection segments), so the
// unused segment puts each pair at an even index: both of its segments lie in one panel of the
// weight stream.
enum PackLayout { LAYOUT_FUSED = 0, LAYOUT_SPLIT = 1, LAYOUT_MLP = 3, LAYOUT_PAIR_FUSED = 4, LAYOUT_PAIR_ATTN = 5 };
__host__ __device__ constexpr bool ffn_skewed(int es, int D) { return es == 2 && D <= 128; }
__host__ __device__ inline int ffn_segs(int FF) { return 2 * (FF / 32) + 1; }
// which matrix chunk sits at index q of the FFN part: kind 5 = W1, 6 = W2, 7 = the unused segment
__host__ __device__ inline void ffn_seg_decode(int q, int NC, bool skewed, int& kind, int& chunk) {
  if (!skewed) {
    if (q == 2 * NC) { kind = 7; chunk = 0; }
    else { kind = 5 + (q & 1); chunk = q >> 1; }
    return;
  }
  if (q < 2) { kind = 5; chunk = q; return; }
  if (q == 2) { kind = 7; chunk = 0; return; }
  const int r = q - 3, i = 1 + r / 2;          // pair of iteration i
  if ((r & 1) == 0) { kind = 6; chunk = i - 1; }
  else if (i + 1 < NC) { kind = 5; chunk = i + 1; }
  else { kind = 6; chunk = NC - 1; }
}
__host__ __device__ inline int mlp_segs(int FF) { return 1 + ffn_segs(FF); }
__host__ __device__ inline size_t packed_seg_bytes(int D, int es) { return (size_t)D * 32 * es; }   // D/GF KiB, GF = 32/es
__host__ __device__ inline int fused_segs(int D, int FF) { return 1 + 4 * (D / 32) + ffn_segs(FF); }
__host__ __device__ inline int kv_segs(int D) { return 1 + 2 * (D / 32); }
__host__ __device__ inline int attn_segs(int D, int FF) { return 1 + 2 * (D / 32) + ffn_segs(FF); }
// room for either layout (the split one is the longer)
__host__ __device__ inline size_t packed_block_bytes(int D, int FF, int es) {
  return (size_t)(kv_segs(D) + attn_segs(D, FF)) * packed_seg_bytes(D, es);
}

enum Mode { MODE_MERGE = 0, MODE_KVPROJ = 1, MODE_ATTN = 2, MODE_SCORE = 3, MODE_STACK = 4, MODE_INPUT = 5, MODE_MERGE_IN = 6 };

// 16 bytes per lane from global memory straight into LDS (no VGPR round trip):
// lane i of the wave writes LDS bytes [lds_wave_base + 16 i, +16).  lds_wave_base must be
// wave-uniform.  Completion is tracked by the wave's vector-memory counter.
// The LDS base travels in M0, which the statement overwrites: it is declared clobbered so that
// the compiler never keeps a value of its own there across a load (it uses M0 for indirect
// register indexing and LDS-direct operations).
__device__ __forceinline__ void gload_lds16(const void* g, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %1\n\t"
               "s_nop 0\n\t"
               "global_load_lds_dwordx4 %0, off\n\t"
               :: "v"(g), "s"(lds_wave_base) : "memory", "m0");
}
// The same with the global address given as a wave-uniform base (scalar registers) plus a 32-bit
// per-lane byte offset, so that advancing the base costs scalar instructions only.
__device__ __forceinline__ void gload_lds16(const void* g_uniform, unsigned lane_off, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %2\n\t"
               "s_nop 0\n\t"
               "global_load_lds_dwordx4 %0, %1\n\t"
               :: "v"(lane_off), "s"(g_uniform), "s"(lds_wave_base) : "memory", "m0");
}

// wait until at most N vector-memory operations of this wave are outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// ------------------------------------------------------------------------------------
// Weight stream: all waves of a workgroup consume the same linear sequence of segments.
// Segments travel global -> LDS directly, in panels of PSEG segments, into a ring of NB
// panel buffers, NB-1 panels ahead of the consumer, so that L2/HBM latency is covered by
// the MFMA work of several panels; one barrier per panel.  The stream's length is rounded
// up to whole panels: the packed buffer must hold PSEG-1 readable segments past its end.
//
// Ordering invariant behind the hand-counted waits.  The stream's loads are inline assembly, so
// the compiler's own wait-count bookkeeping does not see them; this struct counts them itself.
// Vector-memory LOADS of a wave return in issue order, and the counter a wait tests (vmcnt) counts
// the wave's outstanding loads, the compiler's ordinary global loads included.  "At most N
// outstanding" therefore proves that everything issued before the last N loads has landed.  An
// ordinary load that the compiler issues between two panels only makes the count larger than the
// stream assumes, so a wait for N can only wait longer than needed, never too little; and the
// compiler's own waits for its loads (which it believes are the only ones) are waits for a count
// that the stream's younger loads can only push up, so they too err on the strict side.  What
// breaks the argument is a global STORE inside the loop: stores also count in vmcnt on this
// target but may retire out of order with respect to loads.  A mode that stores inside its loop
// (the K/V projection) sets DRAIN and always waits for zero.  Every other mode stores only after
// its last advance() and a wait for zero.
template <int SEGV, int PSEG, int NB, bool DRAIN, int NTHR = kThreads>
struct WStream {
  static constexpr int PANV = SEGV * PSEG;              // 16-byte vectors per panel
  static constexpr int NSTAGE = PANV / NTHR;
  static constexpr int NPRE = NB - 1;
  static_assert(PANV % NTHR == 0 && NSTAGE >= 1, "panel must cover all threads");
  uint4* lds;
  const char* gnext;     // the next panel to fetch (wave-uniform); this thread takes the 16 bytes at lane_off
  unsigned lane_off;
  unsigned lds_wave;     // LDS byte address of this wave's first 16-byte slot in ring buffer 0
  int total, step, sub, issued, slot_issue, slot_cur, lane;   // total / step / issued count panels

  __device__ __forceinline__ void issue() {
    if (issued < total) {
      const unsigned dst = lds_wave + (unsigned)slot_issue * (PANV * 16);
#pragma unroll
      for (int i = 0; i < NSTAGE; ++i) {
        // multi-segment panels (d <= 128, two waves per SIMD): scalar base + lane offset keeps the
        // address arithmetic off the VALU (-2.6 % on the merge kernel); the single-segment panels of
        // the one-wave d = 256 kernels were 1 % faster with per-lane 64-bit addresses
        if (PSEG > 1) gload_lds16(gnext + NTHR * 16 * i, lane_off, dst + NTHR * 16 * i);
        else gload_lds16(gnext + NTHR * 16 * i + lane_off, dst + NTHR * 16 * i);
      }
      gnext += PANV * 16;
      ++issued;
      slot_issue = slot_issue + 1 == NB ? 0 : slot_issue + 1;
    }
  }
  // DRAIN: a mode that stores to global memory inside its loop (loads and stores may
  // retire out of order with respect to each other) always waits for everything.
  __device__ __forceinline__ void init(uint4* lds_, const void* gbase, int total_segments) {
    lds = lds_; total = (total_segments + PSEG - 1) / PSEG; step = 0; sub = 0; issued = 0; slot_issue = 0; slot_cur = 0;
    const int tid = threadIdx.x;
    lane = tid & 63;
    gnext = reinterpret_cast<const char*>(gbase);
    lane_off = (unsigned)tid * 16u;
    lds_wave = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)lds_ + (unsigned)(tid >> 6) * 1024u);
#pragma unroll
    for (int s = 0; s < NB; ++s) issue();
    // panels 0 .. NB-1 are in flight; the oldest must have landed
    if (!DRAIN && NB <= total) wait_vmcnt<(NB - 1) * NSTAGE>();
    else wait_vmcnt<0>();
    __syncthreads();
  }
  // the current segment has been consumed by this wave: move to the next one
  __device__ __forceinline__ void advance() {
    if (PSEG > 1 && ++sub < PSEG) return;      // still inside the panel: nothing to wait for
    sub = 0;
    ++step;
    slot_cur = slot_cur + 1 == NB ? 0 : slot_cur + 1;
    // panels step .. step+NPRE-1 are in flight (when that many remain): the oldest must have landed
    if (!DRAIN && step + NPRE <= total) wait_vmcnt<(NPRE - 1) * NSTAGE>();
    else wait_vmcnt<0>();
    __syncthreads();               // everyone sees panel `step`; everyone is done with `step - 1`
    issue();                       // into the buffer that held panel step - 1
  }
  template <typename G>
  __device__ __forceinline__ G frag(int f) const {
    return *reinterpret_cast<const G*>(&lds[slot_cur * PANV + sub * SEGV + f * 64 + lane]);
  }
  // fragment f of the segment `ahead` places after the current one, which must lie in the same panel
  template <typename G>
  __device__ __forceinline__ G frag_at(int ahead, int f) const {
    return *reinterpret_cast<const G*>(&lds[slot_cur * PANV + (sub + ahead) * SEGV + f * 64 + lane]);
  }
  __device__ __forceinline__ const uint4* cur() const { return &lds[slot_cur * PANV + sub * SEGV]; }
};

}  // namespace longer
