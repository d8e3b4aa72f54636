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

constexpr int kThreads = 256;   // 4 waves, one per SIMD
constexpr int kWaves = 4;
constexpr float kNegBig = -1.0e30f;

// Element traits: one operand group = 16 bytes per lane.
template <typename T> struct ET;

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
};

// feature (inside a 32-wide tile) held by accumulator register r of lane half hi
__host__ __device__ __forceinline__ constexpr int tile_row(int r, int hi) {
  return 8 * (r / 4) + 4 * hi + (r % 4);
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

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

// bytes of one packed block for element size es: all weight segments, then the fp32
// vectors padded to one more segment (they travel through the weight stream as well)
__host__ __device__ inline size_t packed_seg_bytes(int D, int es) { return (size_t)D * 32 * es; }   // D/GF KiB, GF = 32/es
__host__ __device__ inline int packed_num_segs(int D, int FF) { return 4 * (D / 32) + 2 * (FF / 32); }
__host__ __device__ inline size_t packed_vec_offset(int D, int FF, int es) {
  return (size_t)packed_num_segs(D, FF) * packed_seg_bytes(D, es);
}
__host__ __device__ inline size_t packed_block_bytes(int D, int FF, int es) {
  return (size_t)(packed_num_segs(D, FF) + 1) * packed_seg_bytes(D, es);
}

enum Mode { MODE_MERGE = 0, MODE_KVPROJ = 1, MODE_ATTN = 2, MODE_SCORE = 3 };

// 16 bytes per lane from global memory straight into LDS (no VGPR round trip):
// lane i of the wave writes LDS bytes [lds_wave_base + 16 i, +16).  lds_wave_base must be
// wave-uniform.  Completion is tracked by the wave's vector-memory counter.
__device__ __forceinline__ void gload_lds16(const void* g, unsigned lds_wave_base) {
  asm volatile("s_mov_b32 m0, %1\n\t"
               "s_nop 0\n\t"
               "global_load_lds_dwordx4 %0, off\n\t"
               :: "v"(g), "s"(lds_wave_base) : "memory");
}

// wait until at most N vector-memory operations of this wave are outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// ------------------------------------------------------------------------------------
// Weight stream: all waves of a workgroup consume the same sequence of 16-byte-per-lane
// segments.  Segments travel global -> LDS directly into a ring of NB buffers, NB-1
// segments ahead of the consumer, so that L2/HBM latency is covered by the MFMA work of
// several segments; one barrier per segment.  The first segment of every block carries
// the block's fp32 vectors (LayerNorm gain/bias, biases).
template <int SEGV, int MODE, int NT, int NB>
struct WStream {
  static constexpr int NSTAGE = SEGV / kThreads;
  static constexpr int NPRE = NB - 1;
  // K/V projection stores fragments inside its loop; loads and stores may retire out of
  // order with respect to each other, so that mode always drains the counter.
  static constexpr bool DRAIN = (MODE == MODE_KVPROJ);
  static_assert(SEGV % kThreads == 0 && NSTAGE >= 1, "segment must cover all threads");
  uint4* lds;
  const char* wbase;
  size_t bstride;
  unsigned lds_wave;     // LDS byte address of this wave's first 16-byte slot in ring buffer 0
  int steps_per_block, total_steps, step, tid;

  __device__ __forceinline__ const uint4* seg_ptr(int s) const {
    int blk = s / steps_per_block;
    int r = s - blk * steps_per_block - 1;
    int idx;
    if (r < 0) idx = steps_segs();                    // the vector segment sits after the weights
    else if (MODE == MODE_MERGE || MODE == MODE_SCORE) idx = r < 3 * NT ? (r % 3) * NT + r / 3 : r;
    else if (MODE == MODE_ATTN) idx = r < NT ? r : r + 2 * NT;
    else idx = (1 + (r & 1)) * NT + (r >> 1);
    return reinterpret_cast<const uint4*>(wbase + (size_t)blk * bstride) + (size_t)idx * SEGV;
  }
  __device__ __forceinline__ int steps_segs() const { return nsegs; }
  int nsegs;
  __device__ __forceinline__ void issue(int s) {
    if (s < total_steps) {
      const uint4* g = seg_ptr(s);
      const unsigned dst = lds_wave + (unsigned)(s % NB) * (SEGV * 16);
#pragma unroll
      for (int i = 0; i < NSTAGE; ++i) gload_lds16(g + tid + kThreads * i, dst + kThreads * 16 * i);
    }
  }
  __device__ __forceinline__ void init(uint4* lds_, const char* wbase_, size_t bstride_, int spb, int nblocks, int nsegs_) {
    lds = lds_; wbase = wbase_; bstride = bstride_; steps_per_block = spb; total_steps = spb * nblocks; nsegs = nsegs_;
    tid = threadIdx.x; step = 0;
    lds_wave = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)lds_ + (unsigned)(tid >> 6) * 1024u);
#pragma unroll
    for (int s = 0; s < NB; ++s) issue(s);
    // segments 0 .. NB-1 are in flight; the oldest must have landed
    if (!DRAIN && NB <= total_steps) wait_vmcnt<(NB - 1) * NSTAGE>();
    else wait_vmcnt<0>();
    __syncthreads();
  }
  // the current segment has been consumed by this wave: move to the next one
  __device__ __forceinline__ void advance() {
    ++step;
    // segments step .. step+NPRE-1 are in flight (when that many remain): the oldest must have landed
    if (!DRAIN && step + NPRE <= total_steps) wait_vmcnt<(NPRE - 1) * NSTAGE>();
    else wait_vmcnt<0>();
    __syncthreads();               // everyone sees segment `step`; everyone is done with `step - 1`
    issue(step + NPRE);            // into the buffer that held segment step - 1
  }
  template <typename G>
  __device__ __forceinline__ G frag(int f) const {
    return *reinterpret_cast<const G*>(&lds[(step % NB) * SEGV + f * 64 + (tid & 63)]);
  }
  __device__ __forceinline__ const uint4* cur() const { return &lds[(step % NB) * SEGV]; }
};

}  // namespace longer
