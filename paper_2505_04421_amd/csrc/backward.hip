// Backward pass with activation recomputation and mixed precision (Section 3.6.2):
// longer_token_merge_backward (the token merge of Section 3.4 alone), longer_forward_backward
// (the whole model: loss of Eq. 1-2 and the gradient of every input and parameter),
// longer_input_generation_backward (the stage of Section 3.5.1 in front of the merge) and their
// size queries.
//
// Token merge: nothing is kept from a forward call.  The pass reads the raw tokens H, gets every
// block's input rows (fp32) from the fused forward kernel, then walks the InnerTrans blocks from
// the last to the first; for each block it recomputes the block's intermediates from the block's
// input and takes the gradients.  Reduced stack (cross-causal and self-causal layers on B (m + k)
// query rows): its intermediates are a twentieth of the merge's and are kept.
// Precision policy: every GEMM runs on the matrix cores with bf16 operands and fp32
// accumulation; the residual stream, its gradient, LayerNorm and softmax statistics and every
// parameter gradient are fp32; activations and activation gradients between two GEMMs are
// stored as bf16.
//
// Unlike the forward kernels this pass is not fused per tile: a parameter gradient is a sum
// over every token of the batch, i.e. a GEMM whose contraction runs over the tokens, so the
// activations it contracts have to exist for the whole batch.  They are row-major
// [token, feature] tensors in the workspace, and three kinds of kernels work on them:
//   * one bf16 MFMA GEMM (bw_gemm_kernel) whose operands may each be stored with the
//     contraction index contiguous or strided, which covers y = x W (+ epilogues),
//     dx = dy W^T and dW = x^T dy (the tokens dealt to slices whose partial results a second
//     kernel sums; the bias gradient, a column sum, rides along as one more product with ones),
//     and the middle of the merge's FFN backward as two products under one epilogue (the hidden
//     pre-activation is formed again there and never stored);
//   * row kernels: LayerNorm forward / backward (+ gain / shift gradients), the merge's
//     backward, the reduced stack's row build, masks, head and loss, gradient routing;
//   * attention, forward and backward, one thread per (row, head), heads kept as packed bf16
//     (two-feature dot products, fp32 sums): inside a group of K tokens (InnerTrans: K x K scores
//     per head), and over a user's own rows under the mask of Eq. 8 (reduced stack).
// Padded token rows are never read and cost only the zeros written for them.
#include "../../include/longer.h"
#include "device.h"

#include <cstdio>

namespace longer {

int api_error(int code, const char* fmt, ...);   // longer_api.hip
int inner_chain_f32(const longer_config* cfg, const longer_block* inner, int layers, const void* H, const int32_t* lens,
                    int B, int L, float* Z_out, void* ws, size_t ws_bytes, void* stream);   // longer_api.hip

namespace bw {

constexpr int kMaxGroup = 32;   // K <= 32
constexpr int kComputeUnits = 256;

// ------------------------------------------------------------------------------------
// GEMM  C[M, N] = A[M, Kc] B[Kc, N]  (bf16 operands, fp32 accumulation)
//   A_KC: A is stored [M][Kc] (contraction contiguous), else [Kc][M];
//   B_KC: B is stored [N][Kc] (contraction contiguous), else [Kc][N].
// Workgroup tile 128 x 128, contraction step 32, four waves in 2 x 2, each 64 x 64 (2 x 2 MFMA
// tiles of 32 x 32).  Requirements checked by the host: strides multiples of 8 elements,
// 16-byte aligned bases; a contiguous contraction dimension is a multiple of 32; the
// non-contracted extent of a strided operand is a multiple of 8.  Rows / columns / contraction
// slices past the extents read as zeros.
enum Epilogue {
  EPI_BF16 = 0,      // out[m][n] = bf16(acc + bias[n])
  EPI_RES_F32 = 1,   // outf[m][n] = res[m][n] + acc + bias[n]
  EPI_ACT = 2,       // out[m][n] = bf16(v), out2[m][n] = bf16(act(v)), v = acc + bias[n]
  EPI_DACT = 3,      // out[m][n] = bf16(acc * act'(pre[m][n]))
  EPI_F32 = 5,       // outf[m][n] = acc + bias[n]
  EPI_FFN_MID = 6,   // two products in one launch, v = A B + bias and g = A2 B2 (same shapes):
                     // out[m][n] = bf16(g * act'(v)), out2[m][n] = bf16(act(v)); v itself is not stored
  EPI_PARTIAL = 4    // parameter gradients: the contraction (over the tokens) is dealt to slices, one workgroup per
                     // tile and slice; outf[slice][m][n] = acc, summed afterwards by bw_reduce_kernel (out2, if
                     // given: [slice][n] column sums of B, the bias gradient's partials)
};

// Padded token rows (row r = u L + pos with pos >= the user's length) carry no gradient.  With the
// batch's geometry at hand a kernel leaves them out: row GEMMs skip tiles without a valid row, the
// gradient GEMMs read them as zeros and pass over steps that hold nothing else, the LayerNorm kernels
// write zeros for them.  L = 0: every row counts (the reduced stack's rows).
struct RowsValid { const int32_t* lens; int L; };
__device__ __forceinline__ bool row_valid(const RowsValid& v, int r) {
  if (v.L == 0 || v.lens == nullptr) return true;
  const int u = r / v.L;
  return r - u * v.L < v.lens[u];
}
// any valid row in [r0, r1)?
__device__ __forceinline__ bool rows_any_valid(const RowsValid& v, int r0, int r1) {
  if (v.L == 0 || v.lens == nullptr) return true;
  for (int u = r0 / v.L; u * v.L < r1; ++u) {
    const int first = max(r0, u * v.L) - u * v.L;
    if (first < v.lens[u]) return true;
  }
  return false;
}

struct GemmArgs {
  RowsValid rows;             // of the token dimension (M of a row GEMM, the contraction of a gradient GEMM)
  const __bf16* A; const __bf16* B;
  int lda, ldb;
  int M, N, Kc;
  int nsplit;                 // gradient GEMM: number of slices the contraction steps are dealt to
  int epi, act;
  void* out; void* out2; int ldo;
  const __bf16* bias; const float* res; const __bf16* pre;
  const __bf16* A2; const __bf16* B2; int lda2, ldb2;   // the second product of a two-product launch (EPI_FFN_MID)
  int pstride, pstride2;      // EPI_PARTIAL: floats from one slice's partial result to the next (matrix, bias)
};

// Phi(v) = (1 + erf(v / sqrt 2)) / 2 and exp(-v^2 / 2) from one exponential: for z >= 0,
// erf(z) = 1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-z^2), t = 1 / (1 + p z), absolute error
// below 1.5e-7 (the classic five-term approximation; odd extension for z < 0).
__device__ __forceinline__ void gauss_cdf(float v, float* cdf, float* ex) {
  const float z = fabsf(v) * 0.70710678118654752f;
  const float e = __expf(-z * z);
  const float t = __frcp_rn(1.f + 0.3275911f * z);
  const float poly = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
  const float half_erfc = 0.5f * poly * e;                 // (1 - erf(|z|)) / 2
  *cdf = v >= 0.f ? 1.f - half_erfc : half_erfc;
  *ex = e;
}
__device__ __forceinline__ float act_fwd(float v, int act) {
  if (act == LONGER_ACT_RELU) return v > 0.f ? v : 0.f;
  float c, e;
  gauss_cdf(v, &c, &e);
  return v * c;
}
__device__ __forceinline__ float act_grad(float v, int act) {
  if (act == LONGER_ACT_RELU) return v > 0.f ? 1.f : 0.f;
  float c, e;
  gauss_cdf(v, &c, &e);
  return c + v * 0.39894228040143268f * e;
}

// The activation and its derivative at once, for the launch that rounds both to bf16 right away.
// GELU: Phi(v) - 1/2 as v times an even polynomial of degree 8 (minimax fit on [-3.5, 3.5] that reaches 1/2
// at the interval's end, clamped to [0, 1] beyond it; absolute error below 1.3e-3, under the bf16
// rounding step of the values it produces) and the density from one exponential.
__device__ __forceinline__ void act_both(float v, int act, float* a, float* da) {
  if (act == LONGER_ACT_RELU) { *a = v > 0.f ? v : 0.f; *da = v > 0.f ? 1.f : 0.f; return; }
  const float u = v * v;
  float pl = 9.366767568843253e-06f;
  pl = fmaf(pl, u, -0.0003847714538096606f);
  pl = fmaf(pl, u, 0.0064495445928312006f);
  pl = fmaf(pl, u, -0.05893596715178192f);
  pl = fmaf(pl, u, 0.3934098519357524f);
  const float c = __builtin_amdgcn_fmed3f(fmaf(v, pl, 0.5f), 0.f, 1.f);
  const float e = __expf(-0.5f * u);
  *a = v * c;
  *da = fmaf(v * e, 0.39894228040143268f, c);
}

constexpr int kStagePitch = 68;         // floats per row of the epilogue's staging area (64 + 4 pad)

// KS: contraction elements per step.  Every launch uses 32: steps of 64 and 128 (one LDS buffer per operand
// at 128) were measured for the two-product launch, whose contraction is only the model width, and
// changed nothing (6.49 - 6.56 ms per merge backward at the headline shape for the three widths).
template <bool A_KC, bool B_KC, bool DUAL = false, int KS = 32>
__global__ __launch_bounds__(256, DUAL ? 2 : (A_KC ? 4 : 3)) void bw_gemm_kernel(GemmArgs g) {
  static_assert(KS == 32 || (A_KC && B_KC), "wide steps: contraction-contiguous operands only");
  constexpr int kPitchKC = KS + 8;            // elements per row of a contraction-contiguous LDS tile (8 pad)
  constexpr int kTileElems = 128 * kPitchKC;  // >= KS * 128 of the strided form
  constexpr int CPR = KS / 8;                 // 16-byte chunks per tile row (contraction-contiguous form)
  constexpr int NCH = KS / 16;                // chunks per thread and operand tile
  constexpr int NBUF = KS >= 128 ? 1 : 2;
  __shared__ __attribute__((aligned(16))) __bf16 smem[2 * NBUF * kTileElems];
  auto sA = [&](int buf) { return smem + buf * kTileElems; };          // NBUF buffers per operand
  auto sB = [&](int buf) { return smem + (NBUF + buf) * kTileElems; };
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w & 1, wn = w >> 1, hi = lane >> 5, l32 = lane & 31;
  // Tile order.  Workgroups go to the 8 accelerator dies round-robin by index, each die with an L2 of
  // its own.  Row GEMMs: the N tiles of one M tile (which share the A rows) get consecutive slots
  // on one die.  Split GEMMs (parameter gradients): all tiles of one slice of the contraction
  // (which share both operands' rows) do, and the slices are spread over the dies.
  const int ntn = (g.N + 127) / 128, ntm = (g.M + 127) / 128;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const bool split = g.epi == EPI_PARTIAL;
  const int inner = split ? ntm * ntn : ntn;
  const int outer = (slot / inner) * 8 + xcd, in = slot % inner;
  if (outer >= (split ? g.nsplit : ntm)) return;
  const int mt = split ? in / ntn : outer, nt_ = in % ntn;
  const int m0 = mt * 128, n0 = nt_ * 128;
  // contraction steps of 32: a row GEMM takes them all; slice `outer` of a gradient GEMM takes every
  // nsplit-th step, so that every slice samples the whole batch (long and short users alike)
  const int kstride = split ? g.nsplit : 1, kfirst = split ? outer : 0;
  const int ksteps = (g.Kc + KS - 1) / KS;
  const int kend = g.Kc;
  if (!split && !rows_any_valid(g.rows, m0, min(g.M, m0 + 128))) return;   // a tile of padded rows: nobody reads its result
  const int nk = ksteps > kfirst ? (ksteps - kfirst + kstride - 1) / kstride : 0;

  constexpr int NPH = DUAL ? 2 : 1;     // products of the launch
  f32x16 accs[NPH][2][2];
#pragma unroll
  for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) accs[ph][a][b][r] = 0.f;
  const __bf16* opA = g.A; const __bf16* opB = g.B;
  int ldA = g.lda, ldB = g.ldb;

  // Split GEMM with a bias gradient asked for (out2): the column sums of B over the slice are one more
  // product, ones[32, Kc] B, taken by the waves that hold the first 32 rows of the first M tile;
  // every row of its result is the column sum.
  const bool bias_sum = split && g.out2 != nullptr && mt == 0 && wm == 0;
  f32x16 accb[2];
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.f;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) accb[b][r] = 0.f;

  // Operand tiles travel global -> registers -> LDS.  One tile = 512 chunks of 16 bytes, two per
  // thread.  (Keeping the loads of four steps in flight was measured: 188 registers, two waves per
  // SIMD instead of four, every GEMM slower.)
  bf16x8 ra[1][NCH], rb[1][NCH];
  auto gload = [&](int kt, bf16x8* pa, bf16x8* pb) {
    const int k0 = (kfirst + kt * kstride) * KS;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i;
      bf16x8 z;
#pragma unroll
      for (int e = 0; e < 8; ++e) z[e] = (__bf16)0.f;
      pa[i] = z; pb[i] = z;
      if (A_KC) {
        const int row = c / CPR, kc = c % CPR;
        const int gr = m0 + row, gk = k0 + 8 * kc;
        if (gr < g.M && gk < kend) pa[i] = *(const bf16x8*)(opA + (size_t)gr * ldA + gk);
      } else {
        const int kr = c >> 4, xc = c & 15;
        const int gk = k0 + kr, gx = m0 + 8 * xc;
        if (gk < kend && gx < g.M && (!split || row_valid(g.rows, gk))) pa[i] = *(const bf16x8*)(opA + (size_t)gk * ldA + gx);
      }
      if (B_KC) {
        const int row = c / CPR, kc = c % CPR;
        const int gr = n0 + row, gk = k0 + 8 * kc;
        if (gr < g.N && gk < kend) pb[i] = *(const bf16x8*)(opB + (size_t)gr * ldB + gk);
      } else {
        const int kr = c >> 4, xc = c & 15;
        const int gk = k0 + kr, gx = n0 + 8 * xc;
        if (gk < kend && gx < g.N && (!split || row_valid(g.rows, gk))) pb[i] = *(const bf16x8*)(opB + (size_t)gk * ldB + gx);
      }
    }
  };
  auto sstore = [&](int buf, const bf16x8* pa, const bf16x8* pb) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 256 * i;
      if (A_KC) *(bf16x8*)&sA(buf)[(c / CPR) * kPitchKC + 8 * (c % CPR)] = pa[i];
      else      *(bf16x8*)&sA(buf)[(c >> 4) * 128 + 8 * (c & 15)] = pa[i];
      if (B_KC) *(bf16x8*)&sB(buf)[(c / CPR) * kPitchKC + 8 * (c % CPR)] = pb[i];
      else      *(bf16x8*)&sB(buf)[(c >> 4) * 128 + 8 * (c & 15)] = pb[i];
    }
  };
  // fragment of the 32 x 16 operand slice: lane (x = l32, hi) holds contraction slots 8 hi .. 8 hi + 7
  auto frag = [&](const __bf16* s, bool kc, int x, int ks) -> bf16x8 {
    bf16x8 f;
    if (kc) {
      f = *(const bf16x8*)&s[x * kPitchKC + 16 * ks + 8 * hi];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = s[(16 * ks + 8 * hi + e) * 128 + x];
    }
    return f;
  };

  // Contraction steps, two LDS buffers: step's tile goes to LDS (the buffer was last read two steps ago,
  // which every thread left before the previous step's barrier), the registers are refilled with the
  // next step's tile, barrier, MFMAs.  A gradient GEMM passes over steps whose 32 token rows are all
  // padding (the test is the same for the whole workgroup).
  auto next_step = [&](int kt) {
    if (split)
      while (kt < nk && !rows_any_valid(g.rows, (kfirst + kt * kstride) * KS, min(kend, (kfirst + kt * kstride) * KS + KS))) ++kt;
    return kt;
  };
  int buf = 0;
#pragma unroll
  for (int ph = 0; ph < NPH; ++ph) {
  f32x16 (&acc)[2][2] = accs[ph];
  int kt = next_step(0);
  if (kt < nk && !(DUAL && ph == 1)) gload(kt, ra[0], rb[0]);   // (the second product's first tile is on its way already)
  while (kt < nk) {
    if (NBUF == 1) __syncthreads();          // the one buffer is still being read by the step before
    sstore(buf, ra[0], rb[0]);
    const int kn = next_step(kt + 1);
    if (kn < nk) {
      gload(kn, ra[0], rb[0]);
    } else if (DUAL && ph == 0) {            // last step of the first product: request the second product's first tile
      opA = g.A2; opB = g.B2; ldA = g.lda2; ldB = g.ldb2;
      gload(0, ra[0], rb[0]);
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS / 16; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = frag(sA(buf), A_KC, 64 * wm + 32 * t + l32, ks);
        fb[t] = frag(sB(buf), B_KC, 64 * wn + 32 * t + l32, ks);
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
      if (!A_KC && !B_KC && bias_sum) {
#pragma unroll
        for (int b = 0; b < 2; ++b) accb[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, fb[b], accb[b], 0, 0, 0);
      }
    }
    buf ^= NBUF - 1;
    kt = kn;
  }
  }
  f32x16 (&acc)[2][2] = accs[0];

  if (!A_KC && !B_KC && bias_sum && hi == 0) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int n = n0 + 64 * wn + 32 * b + l32;
      if (n < g.N) ((float*)g.out2)[(size_t)outer * g.pstride2 + n] = accb[b][0];     // row 0 of the ones product
    }
  }
  float* stage = (float*)smem + w * (32 * kStagePitch);
  static_assert(4 * 32 * kStagePitch * 4 <= 2 * NBUF * kTileElems * 2, "staging area fits the operand buffers");
  // Loads and stores leave one in-order queue: a load that follows a store is not back before the store
  // has been acknowledged.  What the epilogue reads from memory is therefore requested ahead of its
  // stores: the bias chunk once (a thread's chunks all lie in the same eight columns), the residual /
  // pre-activation rows of a 32-row slab before the slab's first store.
  const int ecc = lane & 7, en = n0 + 64 * wn + 8 * ecc;
  float biasv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) biasv[e] = 0.f;
  if (g.bias && en < g.N) {
    const bf16x8 bv = *(const bf16x8*)(g.bias + en);
#pragma unroll
    for (int e = 0; e < 8; ++e) biasv[e] = (float)bv[e];
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    f32x4 ld[4][2];                   // EPI_RES_F32: the chunk's residual values; EPI_DACT: its pre-activations (first 16 bytes)
    if (g.epi == EPI_RES_F32 || g.epi == EPI_DACT) {
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int m = m0 + 64 * wm + 32 * a + it * 8 + (lane >> 3);
        ld[it][0] = f32x4{0.f, 0.f, 0.f, 0.f}; ld[it][1] = ld[it][0];
        if (m >= g.M || en >= g.N) continue;
        const size_t o = (size_t)m * g.ldo + en;
        if (g.epi == EPI_RES_F32) { ld[it][0] = *(const f32x4*)(g.res + o); ld[it][1] = *(const f32x4*)(g.res + o + 4); }
        else ld[it][0] = *(const f32x4*)(g.pre + o);
      }
    }
    float v2[DUAL ? 4 : 1][8];        // two-product launch: the second product's values of this thread's chunks
    if constexpr (DUAL) {
      __syncthreads();
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) stage[tile_row(r, hi) * kStagePitch + 32 * b + l32] = accs[NPH - 1][a][b][r];
      __syncthreads();
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int id = it * 64 + lane, row = id >> 3, cc = id & 7;
        *(f32x4*)&v2[it][0] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc];
        *(f32x4*)&v2[it][4] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc + 4];
      }
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[tile_row(r, hi) * kStagePitch + 32 * b + l32] = acc[a][b][r];
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int id = it * 64 + lane, row = id >> 3, cc = id & 7;
      const int m = m0 + 64 * wm + 32 * a + row, n = n0 + 64 * wn + 8 * cc;
      if (m >= g.M || n >= g.N) continue;
      float v[8];
      *(f32x4*)&v[0] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc];
      *(f32x4*)&v[4] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc + 4];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += biasv[e];
      const size_t o = (size_t)m * g.ldo + n;
      bf16x8 ob;
      if (g.epi == EPI_BF16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ob[e] = (__bf16)v[e];
        *(bf16x8*)((__bf16*)g.out + o) = ob;
      } else if (g.epi == EPI_RES_F32) {
        const f32x4 r0 = ld[it][0], r1 = ld[it][1];
        f32x4 o0, o1;
#pragma unroll
        for (int e = 0; e < 4; ++e) { o0[e] = r0[e] + v[e]; o1[e] = r1[e] + v[4 + e]; }
        *(f32x4*)((float*)g.out + o) = o0;
        *(f32x4*)((float*)g.out + o + 4) = o1;
      } else if (g.epi == EPI_ACT) {
        bf16x8 oa;
#pragma unroll
        for (int e = 0; e < 8; ++e) { ob[e] = (__bf16)v[e]; oa[e] = (__bf16)act_fwd(v[e], g.act); }
        *(bf16x8*)((__bf16*)g.out + o) = ob;
        *(bf16x8*)((__bf16*)g.out2 + o) = oa;
      } else if (g.epi == EPI_DACT) {
        const bf16x8 pv = __builtin_bit_cast(bf16x8, ld[it][0]);
#pragma unroll
        for (int e = 0; e < 8; ++e) ob[e] = (__bf16)(v[e] * act_grad((float)pv[e], g.act));
        *(bf16x8*)((__bf16*)g.out + o) = ob;
      } else if (DUAL && g.epi == EPI_FFN_MID) {
        bf16x8 oa;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float av, dv;
          act_both(v[e], g.act, &av, &dv);
          oa[e] = (__bf16)av;
          ob[e] = (__bf16)(v2[DUAL ? it : 0][e] * dv);
        }
        *(bf16x8*)((__bf16*)g.out + o) = ob;
        *(bf16x8*)((__bf16*)g.out2 + o) = oa;
      } else if (g.epi == EPI_F32) {
        *(f32x4*)((float*)g.out + o) = *(const f32x4*)&v[0];
        *(f32x4*)((float*)g.out + o + 4) = *(const f32x4*)&v[4];
      } else {
        float* po = (float*)g.out + (size_t)outer * g.pstride + o;
        *(f32x4*)po = *(const f32x4*)&v[0];
        *(f32x4*)(po + 4) = *(const f32x4*)&v[4];
      }
    }
  }
}

// ------------------------------------------------------------------------------------
// Row GEMM with a short contraction (Kc = K <= 128, the model width): y = x W (+ epilogue) or dx = dy W^T,
// both operands with the contraction index contiguous (the caller hands W transposed where needed).
// With so short a contraction a tile per workgroup spends its time on the way from L2 to the compute unit:
// the weights tile weighs as much as the activation tile and is fetched again by every workgroup, and a
// step's loads are not back before the previous step's few MFMAs are done.  Here a workgroup stays: it
// loads its 128 columns of W (both matrices of the two-product launch) into LDS once, then walks over
// row tiles; the next row tile's activations travel to registers while the current one is multiplied
// and stored.  512 threads: wave w works on rows 32 (w & 3) .. + 31, columns 64 (w >> 2) .. + 63 of
// the 128 x 128 tile; the epilogue turns a wave's result through LDS for 16-byte stores.
// Epilogues: EPI_BF16, EPI_RES_F32, EPI_F32, and with DUAL EPI_FFN_MID.
template <int K, bool DUAL>
__global__ __launch_bounds__(512, 1) void bw_rowgemm_kernel(GemmArgs g, int P) {
  constexpr int PITCH = K + 8, TILE = 128 * PITCH, NPH = DUAL ? 2 : 1, CPR = K / 8;
  constexpr int NCH = (128 * CPR + 511) / 512;              // 16-byte chunks per thread and operand tile
  constexpr int STAGE_BYTES = 8 * 32 * kStagePitch * 4;
  constexpr int A_BYTES = NPH * TILE * 2 > STAGE_BYTES ? NPH * TILE * 2 : STAGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem_a[A_BYTES];   // activation tile(s); the epilogue's staging area
  __shared__ __attribute__((aligned(16))) __bf16 sB[NPH * TILE];           // weights, resident
  __bf16* sA = (__bf16*)smem_a;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w & 3, wn = w >> 2, hi = lane >> 5, l32 = lane & 31;
  float* stage = (float*)smem_a + w * (32 * kStagePitch);
  const int ntn = (g.N + 127) / 128, ntm = (g.M + 127) / 128;
  // workgroups of one row-tile sequence (they read the same activations) sit on one die
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int p = (slot / ntn) * 8 + xcd, nt_ = slot % ntn;
  if (p >= P) return;
  const int n0 = nt_ * 128;

  const __bf16* opA[2] = {g.A, DUAL ? g.A2 : g.A};
  const __bf16* opB[2] = {g.B, DUAL ? g.B2 : g.B};
  const int ldA[2] = {g.lda, DUAL ? g.lda2 : g.lda}, ldB[2] = {g.ldb, DUAL ? g.ldb2 : g.ldb};

#pragma unroll
  for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + 512 * i;
      if (c >= 128 * CPR) continue;
      const int row = c / CPR, kc = c % CPR, gr = n0 + row;
      bf16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.f;
      if (gr < g.N) v = *(const bf16x8*)(opB[ph] + (size_t)gr * ldB[ph] + 8 * kc);
      *(bf16x8*)&sB[ph * TILE + row * PITCH + 8 * kc] = v;
    }
  const int ecc = lane & 7, en = n0 + 64 * wn + 8 * ecc;
  float biasv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) biasv[e] = 0.f;
  if (g.bias && en < g.N) {
    const bf16x8 bv = *(const bf16x8*)(g.bias + en);
#pragma unroll
    for (int e = 0; e < 8; ++e) biasv[e] = (float)bv[e];
  }

  bf16x8 ra[NPH][NCH];
  auto gload = [&](int mt) {
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + 512 * i;
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.f;
        const int row = c / CPR, kc = c % CPR, gr = mt * 128 + row;
        if (c < 128 * CPR && gr < g.M) v = *(const bf16x8*)(opA[ph] + (size_t)gr * ldA[ph] + 8 * kc);
        ra[ph][i] = v;
      }
  };
  auto next_tile = [&](int mt) {      // row tiles without a valid row are passed over: nobody reads their result
    while (mt < ntm && !rows_any_valid(g.rows, mt * 128, min(g.M, mt * 128 + 128))) mt += P;
    return mt;
  };
  auto frag = [&](const __bf16* s_, int x, int ks) -> bf16x8 { return *(const bf16x8*)&s_[x * PITCH + 16 * ks + 8 * hi]; };

  int mt = next_tile(p);
  if (mt < ntm) gload(mt);
  while (mt < ntm) {
    __syncthreads();                  // the staging area of the tile before is read out (and, first time, sB is written)
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + 512 * i;
        if (c < 128 * CPR) *(bf16x8*)&sA[ph * TILE + (c / CPR) * PITCH + 8 * (c % CPR)] = ra[ph][i];
      }
    const int mn = next_tile(mt + P);
    if (mn < ntm) gload(mn);          // on its way during the products and the epilogue below
    __syncthreads();
    f32x16 acc[NPH][2];
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ph][t][r] = 0.f;
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph)
#pragma unroll
      for (int ks = 0; ks < K / 16; ++ks) {
        const bf16x8 fa = frag(sA + ph * TILE, 32 * wm + l32, ks);
#pragma unroll
        for (int t = 0; t < 2; ++t)
          acc[ph][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, frag(sB + ph * TILE, 64 * wn + 32 * t + l32, ks), acc[ph][t], 0, 0, 0);
      }
    __syncthreads();                  // every wave is done with the activation tile: its place becomes the staging area

    const int m0 = mt * 128 + 32 * wm;
    f32x4 ld[4][2];                   // EPI_RES_F32: the chunks' residual values, requested ahead of the stores
    if (g.epi == EPI_RES_F32) {
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int m = m0 + it * 8 + (lane >> 3);
        ld[it][0] = f32x4{0.f, 0.f, 0.f, 0.f}; ld[it][1] = ld[it][0];
        if (m >= g.M || en >= g.N) continue;
        const size_t o = (size_t)m * g.ldo + en;
        ld[it][0] = *(const f32x4*)(g.res + o); ld[it][1] = *(const f32x4*)(g.res + o + 4);
      }
    }
    float v2[DUAL ? 4 : 1][8];
    if constexpr (DUAL) {             // (a wave's staging area is its own: LDS keeps a wave's accesses in order)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) stage[tile_row(r, hi) * kStagePitch + 32 * t + l32] = acc[1][t][r];
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int id = it * 64 + lane, row = id >> 3, cc = id & 7;
        *(f32x4*)&v2[it][0] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc];
        *(f32x4*)&v2[it][4] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc + 4];
      }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[tile_row(r, hi) * kStagePitch + 32 * t + l32] = acc[0][t][r];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int id = it * 64 + lane, row = id >> 3, cc = id & 7;
      const int m = m0 + row, n = n0 + 64 * wn + 8 * cc;
      float v[8];
      *(f32x4*)&v[0] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc];
      *(f32x4*)&v[4] = *(const f32x4*)&stage[row * kStagePitch + 8 * cc + 4];
      if (m >= g.M || n >= g.N) continue;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += biasv[e];
      const size_t o = (size_t)m * g.ldo + n;
      bf16x8 ob;
      if (DUAL) {
        bf16x8 oa;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float av, dv;
          act_both(v[e], g.act, &av, &dv);
          oa[e] = (__bf16)av;
          ob[e] = (__bf16)(v2[DUAL ? it : 0][e] * dv);
        }
        *(bf16x8*)((__bf16*)g.out + o) = ob;
        *(bf16x8*)((__bf16*)g.out2 + o) = oa;
      } else if (g.epi == EPI_BF16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ob[e] = (__bf16)v[e];
        *(bf16x8*)((__bf16*)g.out + o) = ob;
      } else if (g.epi == EPI_RES_F32) {
        f32x4 o0, o1;
#pragma unroll
        for (int e = 0; e < 4; ++e) { o0[e] = ld[it][0][e] + v[e]; o1[e] = ld[it][1][e] + v[4 + e]; }
        *(f32x4*)((float*)g.out + o) = o0;
        *(f32x4*)((float*)g.out + o + 4) = o1;
      } else {
        *(f32x4*)((float*)g.out + o) = *(const f32x4*)&v[0];
        *(f32x4*)((float*)g.out + o + 4) = *(const f32x4*)&v[4];
      }
    }
    mt = mn;
  }
}

// ------------------------------------------------------------------------------------
// Row kernels.  A token row r = u L + pos is valid when pos < min(lens[u], L).
struct RowGeom { const int32_t* lens; int L, K, ntok; };

__device__ __forceinline__ int row_len(const RowGeom& q, int u) {
  int l = q.lens ? q.lens[u] : q.L;
  return l < 0 ? 0 : (l > q.L ? q.L : l);
}

// x0[r][:] = valid ? H[r][:] : 0   (fp32 copy of the raw tokens: the first block's input); four
// features per thread (d is a multiple of 4)
__global__ __launch_bounds__(256) void bw_load_x0_kernel(const __bf16* __restrict__ H, float* __restrict__ x0, RowGeom q, int d) {
  const size_t n = (size_t)q.ntok * d / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i * 4 / d);
    const int u = r / q.L, pos = r - u * q.L;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (pos < row_len(q, u)) {
      const bf16x4 t = *(const bf16x4*)(H + i * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (float)t[e];
    }
    *(f32x4*)(x0 + i * 4) = v;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// LayerNorm kernels: a row of width D = 4 LPR is held by LPR adjacent lanes, four consecutive
// features each (16-byte loads), so a wave works on 64 / LPR rows at a time.
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ f32x4 load_bf16x4(const __bf16* p) {
  const bf16x4 t = *(const bf16x4*)p;
  f32x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (float)t[e];
  return o;
}
__device__ __forceinline__ void store_bf16x4(__bf16* p, f32x4 v) {
  bf16x4 t;
#pragma unroll
  for (int e = 0; e < 4; ++e) t[e] = (__bf16)v[e];
  *(bf16x4*)p = t;
}

// n[r][:] = bf16(LN(x[r][:]) g + b)
template <int LPR>
__global__ __launch_bounds__(256) void bw_ln_fwd_kernel(const float* __restrict__ x, const __bf16* __restrict__ gam,
                                                        const __bf16* __restrict__ bet, __bf16* __restrict__ out,
                                                        int ntok, float eps, RowsValid rows) {
  constexpr int RPW = 64 / LPR, D = 4 * LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, rsub = lane / LPR;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const f32x4 gv = load_bf16x4(gam + 4 * sub), bv = load_bf16x4(bet + 4 * sub);
  const int ngroups = (ntok + RPW - 1) / RPW;
#pragma unroll 2
  for (int grp = wave; grp < ngroups; grp += nw) {
    const int r = grp * RPW + rsub;
    const bool ok = r < ntok;
    const bool live = ok && row_valid(rows, r);       // a padded row is written as zeros and not read
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (live) v = *(const f32x4*)(x + (size_t)r * D + 4 * sub);
    const float mean = row_sum<LPR>(v[0] + v[1] + v[2] + v[3]) * (1.f / D);
    v -= mean;
    const float rstd = 1.f / sqrtf(row_sum<LPR>(v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3]) * (1.f / D) + eps);
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    if (ok) store_bf16x4(out + (size_t)r * D + 4 * sub, live ? v * rstd * gv + bv : zero);
  }
}

// LayerNorm backward for y = LN(x) g + b with upstream dn = dL/dy (bf16) and the gradient dres that
// reaches x through the residual connection (NULL: none): dx_out = dres + dLN, also stored as bf16 (dxb, may be
// NULL); the block's share of dg[e] = sum_r dn xhat and db[e] = sum_r dn goes to part[block][2][D]
// (bw_reduce_kernel sums the blocks).
template <int LPR>
__global__ __launch_bounds__(256) void bw_ln_bwd_kernel(const __bf16* __restrict__ dn, const float* __restrict__ x,
                                                        const __bf16* __restrict__ gam, const float* __restrict__ dres,
                                                        float* __restrict__ dx_out, __bf16* __restrict__ dxb,
                                                        float* __restrict__ part, int ntok, float eps, RowsValid rows) {
  constexpr int RPW = 64 / LPR, D = 4 * LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, rsub = lane / LPR;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const f32x4 gv = load_bf16x4(gam + 4 * sub);
  f32x4 ag = {0.f, 0.f, 0.f, 0.f}, ab = {0.f, 0.f, 0.f, 0.f};
  const int ngroups = (ntok + RPW - 1) / RPW;
#pragma unroll 2
  for (int grp = wave; grp < ngroups; grp += nw) {
    const int r = grp * RPW + rsub;
    const bool ok = r < ntok;
    const bool live = ok && row_valid(rows, r);       // a padded row: zero gradient, nothing read
    const size_t o = (size_t)r * D + 4 * sub;
    f32x4 v = {0.f, 0.f, 0.f, 0.f}, t = v, res = v;
    if (live) {
      v = *(const f32x4*)(x + o);
      t = load_bf16x4(dn + o);
      if (dres) res = *(const f32x4*)(dres + o);
    }
    const float mean = row_sum<LPR>(v[0] + v[1] + v[2] + v[3]) * (1.f / D);
    v -= mean;
    const float rstd = 1.f / sqrtf(row_sum<LPR>(v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3]) * (1.f / D) + eps);
    v *= rstd;                                   // xhat
    ab += t;
    ag += t * v;
    t *= gv;                                     // dL/dxhat
    const float c1 = row_sum<LPR>(t[0] + t[1] + t[2] + t[3]) * (1.f / D);
    const float c2 = row_sum<LPR>(t[0] * v[0] + t[1] * v[1] + t[2] * v[2] + t[3] * v[3]) * (1.f / D);
    if (ok) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const f32x4 dx = live ? res + rstd * (t - c1 - v * c2) : zero;
      *(f32x4*)(dx_out + o) = dx;
      if (dxb) store_bf16x4(dxb + o, dx);
    }
  }
  // rows handled side by side in the wave, then the block's four waves (LDS)
#pragma unroll
  for (int e = 0; e < 4; ++e) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      ag[e] += __shfl_xor(ag[e], o, 64);
      ab[e] += __shfl_xor(ab[e], o, 64);
    }
  }
  __shared__ f32x4 red[2][4][LPR];
  const int wv = threadIdx.x >> 6;
  if (rsub == 0) {
    red[0][wv][sub] = ag;
    red[1][wv][sub] = ab;
  }
  __syncthreads();
  if (threadIdx.x < 2 * LPR) {
    const int which = threadIdx.x / LPR, c = threadIdx.x % LPR;
    *(f32x4*)(part + (size_t)blockIdx.x * 2 * D + which * D + 4 * c) =
        red[which][0][c] + red[which][1][c] + red[which][2][c] + red[which][3][c];
  }
}

// Gradient of the merge (Section 3.4) into the last block's output rows:
//   mean:   dZ[r][:] = dM[u][t][:] / n_{u,t} for the group's n valid tokens;
//   concat: dZ[r][:] = dM[u][t][j d : (j + 1) d] for the token in slot j of its group;
// zeros for padded tokens.  Written as fp32 and as bf16.
__global__ __launch_bounds__(256) void bw_merge_bwd_kernel(const float* __restrict__ dM, float* __restrict__ dy,
                                                           __bf16* __restrict__ dyb, RowGeom q, int d, int T, int concat) {
  const size_t n = (size_t)q.ntok * d / 4;      // four features per thread
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i * 4 / d), e = (int)(i * 4 - (size_t)r * d);
    const int u = r / q.L, pos = r - u * q.L;
    const int len = row_len(q, u);
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (pos < len) {
      const int t = pos / q.K, j = pos - t * q.K;
      if (concat) {
        v = *(const f32x4*)(dM + ((size_t)u * T + t) * ((size_t)q.K * d) + (size_t)j * d + e);
      } else {
        const int cnt = min(q.K, len - t * q.K);
        v = *(const f32x4*)(dM + ((size_t)u * T + t) * d + e) / (float)cnt;
      }
    }
    *(f32x4*)(dy + i * 4) = v;
    store_bf16x4(dyb + i * 4, v);
  }
}

// ------------------------------------------------------------------------------------
// Attention inside a group of K adjacent tokens (InnerTrans, Section 3.4): bidirectional, keys
// masked by validity.  qkv [ntok][3 d] = [q | k | v]; one thread per (row, head).
struct GroupOf {
  int first;      // first row of the group
  int n;          // valid tokens in it (they are its first n rows)
};
__device__ __forceinline__ bool group_of(const RowGeom& q, int r, GroupOf* g) {
  const int u = r / q.L, pos = r - u * q.L;
  const int len = row_len(q, u);
  const int t = pos / q.K;
  g->first = u * q.L + t * q.K;
  g->n = max(0, min(q.K, len - t * q.K));
  return pos < len;
}

// A head's DH features as stored (packed bf16): dot products take them two at a time
// (v_dot2_f32_bf16: fp32 sum of two bf16 products and the accumulator), sums weighted by a
// scalar widen them one by one.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int DH> struct HeadVec { bf16x8 c[DH / 8]; };
template <int DH>
__device__ __forceinline__ HeadVec<DH> load_head(const __bf16* p) {
  HeadVec<DH> v;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) v.c[c] = *(const bf16x8*)(p + 8 * c);
  return v;
}
template <int DH>
__device__ __forceinline__ void store_head(__bf16* p, const float* v) {
#pragma unroll
  for (int c = 0; c < DH; c += 8) {
    bf16x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = (__bf16)v[c + e];
    *(bf16x8*)(p + c) = t;
  }
}
template <int DH>
__device__ __forceinline__ float dot(const HeadVec<DH>& a, const HeadVec<DH>& b) {
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) {
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a.c[c], a.c[c], 0, 1), __builtin_shufflevector(b.c[c], b.c[c], 0, 1), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a.c[c], a.c[c], 2, 3), __builtin_shufflevector(b.c[c], b.c[c], 2, 3), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a.c[c], a.c[c], 4, 5), __builtin_shufflevector(b.c[c], b.c[c], 4, 5), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a.c[c], a.c[c], 6, 7), __builtin_shufflevector(b.c[c], b.c[c], 6, 7), s, false);
  }
  return s;
}
// acc[:] += w v[:]
template <int DH>
__device__ __forceinline__ void axpy(float* acc, float w, const HeadVec<DH>& v) {
#pragma unroll
  for (int c = 0; c < DH / 8; ++c)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[8 * c + e] = fmaf(w, (float)v.c[c][e], acc[8 * c + e]);
}

// The same with the weight rounded to bf16: acc[2i] and acc[2i + 1] each take one two-feature product
// against (w, 0) or (0, w), so the packed features need no widening (half the instructions of axpy).
// For the long loops of the reduced stack's attention, where the weight is a probability or a
// score gradient that multiplies bf16 values anyway.
template <int DH>
__device__ __forceinline__ void axpy_packed(float* acc, float w, const HeadVec<DH>& v) {
  const __bf16 wb = (__bf16)w;
  const bf16x2 w0 = {wb, (__bf16)0.f}, w1 = {(__bf16)0.f, wb};
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) {
    const bf16x2 pr[4] = {__builtin_shufflevector(v.c[c], v.c[c], 0, 1), __builtin_shufflevector(v.c[c], v.c[c], 2, 3),
                          __builtin_shufflevector(v.c[c], v.c[c], 4, 5), __builtin_shufflevector(v.c[c], v.c[c], 6, 7)};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[8 * c + 2 * e] = __builtin_amdgcn_fdot2_f32_bf16(pr[e], w0, acc[8 * c + 2 * e], false);
      acc[8 * c + 2 * e + 1] = __builtin_amdgcn_fdot2_f32_bf16(pr[e], w1, acc[8 * c + 2 * e + 1], false);
    }
  }
}

// KG: the loops over a group's tokens are unrolled KG times (K <= KG) so that the per-token values
// stay in registers; tokens past the group's valid count are predicated off.
template <int DH, int KG>
__global__ __launch_bounds__(256) void bw_attn_fwd_kernel(const __bf16* qkv, __bf16* o, RowGeom q, int d, int heads) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)q.ntok * heads) return;
  const int r = (int)(idx / heads), h = (int)(idx - (long long)r * heads);
  GroupOf g;
  float acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) acc[c] = 0.f;
  if (group_of(q, r, &g)) {
    const float scale = rsqrtf((float)DH);
    const HeadVec<DH> qv = load_head<DH>(qkv + (size_t)r * 3 * d + h * DH);
    const __bf16* kbase = qkv + (size_t)g.first * 3 * d + d + h * DH;
    float s[KG];
    float mx = -3.0e38f;
#pragma unroll
    for (int j = 0; j < KG; ++j) {
      s[j] = -3.0e38f;
      if (j < g.n) {
        s[j] = scale * dot<DH>(qv, load_head<DH>(kbase + (size_t)j * 3 * d));
        mx = fmaxf(mx, s[j]);
      }
    }
    float l = 0.f;
#pragma unroll
    for (int j = 0; j < KG; ++j) {
      s[j] = j < g.n ? __expf(s[j] - mx) : 0.f;
      l += s[j];
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int j = 0; j < KG; ++j)
      if (j < g.n) axpy<DH>(acc, s[j] * inv, load_head<DH>(kbase + (size_t)j * 3 * d + d));
  }
  store_head<DH>(o + (size_t)r * d + h * DH, acc);
}

// Query side of the attention backward: for query row i, P_i. is recomputed, dP_ij = do_i . v_j,
// D_i = sum_j P_ij dP_ij, dS_ij = P_ij (dP_ij - D_i), dq_i = scale sum_j dS_ij k_j.  Writes dq into
// dqkv[:, 0:d) and the row's softmax statistics (log-sum-exp of the scaled scores, D_i) into stat.
template <int DH, int KG>
__global__ __launch_bounds__(256) void bw_attn_bwd_q_kernel(const __bf16* qkv, const __bf16* dob, __bf16* dqkv,
                                                            float2* stat, RowGeom q, int d, int heads) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)q.ntok * heads) return;
  const int r = (int)(idx / heads), h = (int)(idx - (long long)r * heads);
  GroupOf g;
  float acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) acc[c] = 0.f;
  float2 st = make_float2(0.f, 0.f);
  if (group_of(q, r, &g)) {
    const float scale = rsqrtf((float)DH);
    const HeadVec<DH> qv = load_head<DH>(qkv + (size_t)r * 3 * d + h * DH);
    const HeadVec<DH> dov = load_head<DH>(dob + (size_t)r * d + h * DH);
    const __bf16* kbase = qkv + (size_t)g.first * 3 * d + d + h * DH;
    float s[KG], dp[KG];
    float mx = -3.0e38f;
#pragma unroll
    for (int j = 0; j < KG; ++j) {
      s[j] = -3.0e38f; dp[j] = 0.f;
      if (j < g.n) {
        s[j] = scale * dot<DH>(qv, load_head<DH>(kbase + (size_t)j * 3 * d));
        dp[j] = dot<DH>(dov, load_head<DH>(kbase + (size_t)j * 3 * d + d));
        mx = fmaxf(mx, s[j]);
      }
    }
    float l = 0.f, Dn = 0.f;
#pragma unroll
    for (int j = 0; j < KG; ++j) {
      s[j] = j < g.n ? __expf(s[j] - mx) : 0.f;
      l += s[j];
      Dn = fmaf(s[j], dp[j], Dn);
    }
    const float inv = 1.f / l;
    const float D = Dn * inv;
#pragma unroll
    for (int j = 0; j < KG; ++j)
      if (j < g.n) axpy<DH>(acc, scale * inv * s[j] * (dp[j] - D), load_head<DH>(kbase + (size_t)j * 3 * d));
    st = make_float2(mx + __logf(l), D);
  }
  store_head<DH>(dqkv + (size_t)r * 3 * d + h * DH, acc);
  stat[(size_t)r * heads + h] = st;
}

// Key side: for key row j, over the group's valid queries i: P_ij = exp(s_ij - lse_i),
// dv_j = sum_i P_ij do_i, dk_j = scale sum_i P_ij (do_i . v_j - D_i) q_i.  Writes dqkv[:, d:3d).
template <int DH, int KG>
__global__ __launch_bounds__(256) void bw_attn_bwd_kv_kernel(const __bf16* qkv, const __bf16* dob, __bf16* dqkv,
                                                             const float2* stat, RowGeom q, int d, int heads) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)q.ntok * heads) return;
  const int r = (int)(idx / heads), h = (int)(idx - (long long)r * heads);
  GroupOf g;
  float dk[DH], dv[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { dk[c] = 0.f; dv[c] = 0.f; }
  if (group_of(q, r, &g)) {
    const float scale = rsqrtf((float)DH);
    const HeadVec<DH> kv = load_head<DH>(qkv + (size_t)r * 3 * d + d + h * DH);
    const HeadVec<DH> vv = load_head<DH>(qkv + (size_t)r * 3 * d + 2 * d + h * DH);
#pragma unroll
    for (int i = 0; i < KG; ++i) {
      if (i < g.n) {
        const int ri = g.first + i;
        const HeadVec<DH> qi = load_head<DH>(qkv + (size_t)ri * 3 * d + h * DH);
        const HeadVec<DH> doi = load_head<DH>(dob + (size_t)ri * d + h * DH);
        const float2 st = stat[(size_t)ri * heads + h];
        const float p = __expf(scale * dot<DH>(qi, kv) - st.x);
        const float ds = scale * p * (dot<DH>(doi, vv) - st.y);
        axpy<DH>(dv, p, doi);
        axpy<DH>(dk, ds, qi);
      }
    }
  }
  store_head<DH>(dqkv + (size_t)r * 3 * d + d + h * DH, dk);
  store_head<DH>(dqkv + (size_t)r * 3 * d + 2 * d + h * DH, dv);
}

// Both sides in one launch, when every group lies inside one workgroup's rows (L a multiple of K, and K a divisor
// of the 256 / heads rows a workgroup holds): the query side first, its statistics to LDS, then the key side from
// there.  The second pass finds the group's rows in the cache that the first pass filled, so the pair reads
// q, k, v and the output gradient from memory once instead of twice.
template <int DH, int KG>
__global__ __launch_bounds__(256) void bw_attn_bwd_fused_kernel(const __bf16* qkv, const __bf16* dob, __bf16* dqkv,
                                                                RowGeom q, int d, int heads) {
  __shared__ float2 sst[256];
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const bool inside = idx < (long long)q.ntok * heads;
  const int r = inside ? (int)(idx / heads) : 0, h = inside ? (int)(idx - (long long)r * heads) : 0;
  const int r0 = (int)(((long long)blockIdx.x * 256) / heads);
  GroupOf g;
  const bool valid = inside && group_of(q, r, &g);
  const float scale = rsqrtf((float)DH);
  float2 st = make_float2(0.f, 0.f);
  {
    float acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.f;
    if (valid) {
      const HeadVec<DH> qv = load_head<DH>(qkv + (size_t)r * 3 * d + h * DH);
      const HeadVec<DH> dov = load_head<DH>(dob + (size_t)r * d + h * DH);
      const __bf16* kbase = qkv + (size_t)g.first * 3 * d + d + h * DH;
      float s[KG], dp[KG];
      float mx = -3.0e38f;
#pragma unroll
      for (int j = 0; j < KG; ++j) {
        s[j] = -3.0e38f; dp[j] = 0.f;
        if (j < g.n) {
          s[j] = scale * dot<DH>(qv, load_head<DH>(kbase + (size_t)j * 3 * d));
          dp[j] = dot<DH>(dov, load_head<DH>(kbase + (size_t)j * 3 * d + d));
          mx = fmaxf(mx, s[j]);
        }
      }
      float l = 0.f, Dn = 0.f;
#pragma unroll
      for (int j = 0; j < KG; ++j) {
        s[j] = j < g.n ? __expf(s[j] - mx) : 0.f;
        l += s[j];
        Dn = fmaf(s[j], dp[j], Dn);
      }
      const float inv = 1.f / l;
      const float D = Dn * inv;
#pragma unroll
      for (int j = 0; j < KG; ++j)
        if (j < g.n) axpy<DH>(acc, scale * inv * s[j] * (dp[j] - D), load_head<DH>(kbase + (size_t)j * 3 * d));
      st = make_float2(mx + __logf(l), D);
    }
    if (inside) store_head<DH>(dqkv + (size_t)r * 3 * d + h * DH, acc);
  }
  sst[threadIdx.x] = st;
  __syncthreads();
  float dk[DH], dv[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { dk[c] = 0.f; dv[c] = 0.f; }
  if (valid) {
    const HeadVec<DH> kv = load_head<DH>(qkv + (size_t)r * 3 * d + d + h * DH);
    const HeadVec<DH> vv = load_head<DH>(qkv + (size_t)r * 3 * d + 2 * d + h * DH);
#pragma unroll
    for (int i = 0; i < KG; ++i) {
      if (i < g.n) {
        const int ri = g.first + i;
        const HeadVec<DH> qi = load_head<DH>(qkv + (size_t)ri * 3 * d + h * DH);
        const HeadVec<DH> doi = load_head<DH>(dob + (size_t)ri * d + h * DH);
        const float2 si = sst[(ri - r0) * heads + h];
        const float p = __expf(scale * dot<DH>(qi, kv) - si.x);
        const float ds = scale * p * (dot<DH>(doi, vv) - si.y);
        axpy<DH>(dv, p, doi);
        axpy<DH>(dk, ds, qi);
      }
    }
  }
  if (inside) {
    store_head<DH>(dqkv + (size_t)r * 3 * d + d + h * DH, dk);
    store_head<DH>(dqkv + (size_t)r * 3 * d + 2 * d + h * DH, dv);
  }
}

// launchers by head width and group size
template <int DH, int KG>
static void attn_launch(int which, unsigned grid, hipStream_t st, const __bf16* qkv, const __bf16* dob, __bf16* out, float2* stat,
                        RowGeom q, int d, int heads) {
  if (which == 0) bw_attn_fwd_kernel<DH, KG><<<grid, 256, 0, st>>>(qkv, out, q, d, heads);
  else if (which == 3) bw_attn_bwd_fused_kernel<DH, KG><<<grid, 256, 0, st>>>(qkv, dob, out, q, d, heads);
  else if (which == 1) bw_attn_bwd_q_kernel<DH, KG><<<grid, 256, 0, st>>>(qkv, dob, out, stat, q, d, heads);
  else bw_attn_bwd_kv_kernel<DH, KG><<<grid, 256, 0, st>>>(qkv, dob, out, stat, q, d, heads);
}
// which: 0 forward (out = o), 1 backward, query side, 2 backward, key side (out = dqkv), 3 both sides in one launch
static void group_attn(int which, int dh, int K, unsigned grid, hipStream_t st, const __bf16* qkv, const __bf16* dob, __bf16* out,
                       float2* stat, RowGeom q, int d, int heads) {
#define LONGER_BW_ATTN(DH, KG) attn_launch<DH, KG>(which, grid, st, qkv, dob, out, stat, q, d, heads)
  if (dh == 16) {
    if (K <= 4) LONGER_BW_ATTN(16, 4); else if (K <= 8) LONGER_BW_ATTN(16, 8); else if (K <= 16) LONGER_BW_ATTN(16, 16); else LONGER_BW_ATTN(16, 32);
  } else {
    if (K <= 4) LONGER_BW_ATTN(32, 4); else if (K <= 8) LONGER_BW_ATTN(32, 8); else if (K <= 16) LONGER_BW_ATTN(32, 16); else LONGER_BW_ATTN(32, 32);
  }
#undef LONGER_BW_ATTN
}

// [wq | wk | wv] side by side: cat[i][j d + c] = w_j[i][c]; biases the same way
__global__ __launch_bounds__(256) void bw_concat_qkv_kernel(const __bf16* wq, const __bf16* wk, const __bf16* wv,
                                                            const __bf16* bq, const __bf16* bk, const __bf16* bv,
                                                            __bf16* cat, __bf16* bcat, int d) {
  const int n = d * 3 * d;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n + 3 * d; i += gridDim.x * 256) {
    if (i < n) {
      const int row = i / (3 * d), col = i - row * 3 * d;
      const int j = col / d, c = col - j * d;
      const __bf16* w = j == 0 ? wq : (j == 1 ? wk : wv);
      cat[i] = w[row * d + c];
    } else {
      const int col = i - n;
      const int j = col / d, c = col - j * d;
      const __bf16* b = j == 0 ? bq : (j == 1 ? bk : bv);
      bcat[col] = b[c];
    }
  }
}

// out[i] += sum over the slices s of part[s][i], i < count (count a multiple of 4; out starts at zero).
// Thread (x, y) of a 64 x 4 block sums every fourth slice of four adjacent outputs inside the block's
// share of the slices (blockIdx.y of gridDim.y shares), the four partial sums meet in LDS, and the
// block adds its sum with one atomic per output (a plain store when there is one share and the result
// is not to be added to what out holds).
__global__ __launch_bounds__(256) void bw_reduce_kernel(const float* __restrict__ part, int nsplit, int count, float* out,
                                                        int accumulate) {
  __shared__ f32x4 red[4][64];
  const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
  const int i = (blockIdx.x * 64 + x) * 4;
  const int per = (nsplit + gridDim.y - 1) / gridDim.y;
  const int s0 = blockIdx.y * per, s1 = min(nsplit, s0 + per);
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  if (i < count) {
#pragma unroll 4
    for (int sl = s0 + y; sl < s1; sl += 4) s += *(const f32x4*)(part + (size_t)sl * count + i);
  }
  red[y][x] = s;
  __syncthreads();
  if (y == 0 && i < count) {
    const f32x4 t = red[0][x] + red[1][x] + red[2][x] + red[3][x];
    if (gridDim.y == 1 && !accumulate) {
      *(f32x4*)(out + i) = t;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) unsafeAtomicAdd(out + i + e, t[e]);
    }
  }
}

// rows [B][T K][d] -> [B][L][d] (the first L rows of every user)
__global__ __launch_bounds__(256) void bw_take_rows_kernel(const float* __restrict__ src, float* __restrict__ dst, int B, int L,
                                                           int TK, int d) {
  const size_t per = (size_t)L * d / 4, total = per * B;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t u = i / per, r = i - u * per;
    *(f32x4*)(dst + (u * L * d + r * 4)) = *(const f32x4*)(src + (u * TK * d + r * 4));
  }
}

__global__ __launch_bounds__(256) void bw_zero_kernel(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}


// ------------------------------------------------------------------------------------
// The reduced stack (Section 3.5): cross-causal layer over R = [G; M] with the query set O of Eq. 5,
// self-causal layers over O's rows.  Every row carries a descriptor of its token: -1 invalid, a for
// global token a, kSeq + t for the sequence token with merged index t; visibility is the rule of
// Eq. 8 on those descriptors.
constexpr int kSeq = 1 << 24;

__device__ __forceinline__ bool visible(int qd, int kd, int gmask) {
  if (qd < 0 || kd < 0) return false;
  if (qd >= kSeq) return kd >= kSeq && kd <= qd;          // a sequence query: sequence keys not newer than itself
  if (kd >= kSeq) return true;                            // a global query: every valid sequence key
  return gmask == LONGER_GMASK_FULL || kd >= qd;          // and the global keys of its set
}

// merged index held by query slot i of a user with tu merged tokens (Section 3.5.1): the last
// k - k_uniform slots the most recent tokens, the first k_uniform spread evenly over the older ones
// (each the newest token of its share); negative: the slot is empty
__device__ __forceinline__ int slot_merged_index(int i, int k, int tu, int k_uniform) {
  if (tu <= k || i >= k_uniform) return tu - k + i;
  const int rest = tu - (k - k_uniform);
  return (int)(((long long)(i + 1) * rest) / k_uniform) - 1;
}

struct StackGeom { const int32_t* lens; int L, K, T, m, k, k_uniform, B, learn; };   // learn: the slots hold learnable query tokens

__device__ __forceinline__ int merged_len(const StackGeom& g, int u) {
  int l = g.lens ? g.lens[u] : g.L;
  l = l < 0 ? 0 : (l > g.L ? g.L : l);
  return (l + g.K - 1) / g.K;
}

// descriptors of the query rows [B][m + k] and of the cross layer's key rows [B][m + T]
__global__ __launch_bounds__(256) void bw_desc_kernel(StackGeom g, int* qdesc, int* kdesc) {
  const int n = g.m + g.k, nk = g.m + g.T;
  const int total = g.B * (n + nk);
  for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    if (i < g.B * n) {
      const int u = i / n, r = i - u * n;
      int dsc = r;
      if (r >= g.m) {
        const int tu = merged_len(g, u);
        // a learnable query token stands after the user's newest token, in slot order (it sees every valid
        // merged token in the cross layer and the slots up to itself in the self layers); no token, no slot
        const int t = g.learn ? (tu > 0 ? tu + (r - g.m) : -1) : slot_merged_index(r - g.m, g.k, tu, g.k_uniform);
        dsc = t >= 0 ? kSeq + t : -1;
      }
      qdesc[i] = dsc;
    } else {
      const int j = i - g.B * n;
      const int u = j / nk, r = j - u * nk;
      kdesc[j] = r < g.m ? r : (r - g.m < merged_len(g, u) ? kSeq + (r - g.m) : -1);
    }
  }
}

// R = [G; M] (merged tokens past T_u as zeros) and O = [G; the slots' merged tokens] as fp32 rows
__global__ __launch_bounds__(256) void bw_build_rows_kernel(StackGeom g, int d, const __bf16* __restrict__ G,
                                                            const __bf16* __restrict__ M, const __bf16* __restrict__ qlearn,
                                                            const int* __restrict__ qdesc,
                                                            const int* __restrict__ kdesc, float* __restrict__ Ox,
                                                            float* __restrict__ Rx) {
  const int n = g.m + g.k, nk = g.m + g.T, d4 = d / 4;
  const size_t total = (size_t)g.B * (n + nk) * d4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int c = (int)(i % d4) * 4;
    size_t row = i / d4;
    const bool isq = row < (size_t)g.B * n;
    if (!isq) row -= (size_t)g.B * n;
    const int per = isq ? n : nk;
    const int u = (int)(row / per), r = (int)(row - (size_t)u * per);
    const int dsc = isq ? qdesc[row] : kdesc[row];
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (dsc >= 0) {
      const __bf16* src = dsc < kSeq ? G + ((size_t)u * g.m + dsc) * d
                        : (isq && g.learn) ? qlearn + (size_t)(r - g.m) * d       // slot i: row i of the parameter
                                           : M + ((size_t)u * g.T + (dsc - kSeq)) * d;
      v = load_bf16x4(src + c);
    }
    *(f32x4*)((isq ? Ox : Rx) + row * d + c) = v;
  }
}

// x[row][:] = valid(row) ? x[row][:] : 0, and its bf16 copy (xb may be NULL)
__global__ __launch_bounds__(256) void bw_mask_rows_kernel(float* __restrict__ x, __bf16* __restrict__ xb,
                                                           const int* __restrict__ desc, size_t rows, int d) {
  const int d4 = d / 4;
  const size_t total = rows * d4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t row = i / d4;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (desc[row] >= 0) v = *(const f32x4*)(x + i * 4);
    *(f32x4*)(x + i * 4) = v;
    if (xb) store_bf16x4(xb + i * 4, v);
  }
}

struct SetAttn {
  const __bf16* q; int qpitch;          // [B nq][..]
  const __bf16* k; const __bf16* v; int kvpitch;   // [B nk][..]
  const int* qdesc; const int* kdesc;
  int nq, nk, B, heads, gmask;
  int m, self;                          // global rows come first in both sets; self: the key rows are the query rows
};

// Keys a query row can see at all lie in [lo, hi) of its user's key rows: a sequence query sees no global
// row and nothing newer than itself (its own row in a self layer, its merged token's row in the cross
// layer); the visibility test inside the loops still decides each pair.
__device__ __forceinline__ void key_range(const SetAttn& a, int qd, int i, int* lo, int* hi) {
  *lo = 0; *hi = a.nk;
  if (qd >= kSeq) {
    *lo = a.m;
    *hi = min(a.nk, a.self ? i + 1 : a.m + (qd - kSeq) + 1);
  }
}

// Row-per-thread set-attention kernels, reading keys (queries) from global memory: the ones that run when a
// user's rows do not fit the LDS-staged kernels further down.  They give a (row, head) pair to kSplit adjacent
// lanes, each taking every kSplit-th key (query) of the loop, and combine the lanes' partial results with
// cross-lane shuffles.
constexpr int kSplit = 1;   // measured at the headline batch: with the keys in global memory 8 lanes per pair were no
                            // faster, and slower in the two backward kernels
__device__ __forceinline__ float split_sum(float v) {
#pragma unroll
  for (int o = 1; o < kSplit; o <<= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float split_max(float v) {
#pragma unroll
  for (int o = 1; o < kSplit; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// o[row][h] = softmax over the visible keys of the row's user (q . k / sqrt(dh)) v; stat[row][h].x = the
// log-sum-exp of the scaled scores.  One pass with a running maximum per lane.
template <int DH>
__global__ __launch_bounds__(256) void bw_set_attn_fwd_kernel(SetAttn a, __bf16* __restrict__ o, int d, float2* __restrict__ stat) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) / kSplit;
  const int sub = threadIdx.x % kSplit;
  if (idx >= (long long)a.B * a.nq * a.heads) return;
  const int row = (int)(idx / a.heads), h = (int)(idx - (long long)row * a.heads);
  const int u = row / a.nq, qd = a.qdesc[row];
  float acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) acc[c] = 0.f;
  float mx = -3.0e38f, l = 0.f;
  if (qd >= 0) {
    const float scale = rsqrtf((float)DH);
    const HeadVec<DH> qv = load_head<DH>(a.q + (size_t)row * a.qpitch + h * DH);
    int lo, hi;
    key_range(a, qd, row - u * a.nq, &lo, &hi);
    // every row of the range is loaded, a hidden key weighs nothing: no branch in the loop, so that the
    // loads of several keys are in flight at once
#pragma unroll(DH == 16 ? 4 : 2)
    for (int j = lo + sub; j < hi; j += kSplit) {
      const size_t kr = (size_t)u * a.nk + j;
      const bool vis = visible(qd, a.kdesc[kr], a.gmask);
      const HeadVec<DH> kv = load_head<DH>(a.k + kr * a.kvpitch + h * DH);
      const HeadVec<DH> vv = load_head<DH>(a.v + kr * a.kvpitch + h * DH);
      const float sc = vis ? scale * dot<DH>(qv, kv) : -3.0e38f;
      const float mn = fmaxf(mx, sc);
      const float corr = __expf(mx - mn), p = vis ? __expf(sc - mn) : 0.f;
      l = l * corr + p;
#pragma unroll
      for (int c = 0; c < DH; ++c) acc[c] *= corr;
      axpy<DH>(acc, p, vv);
      mx = mn;
    }
  }
  const float mall = split_max(mx);
  const float corr = __expf(mx - mall);          // a lane without a visible key: l = 0, acc = 0
  l = split_sum(l * corr);
  const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
  for (int c = 0; c < DH; ++c) acc[c] = split_sum(acc[c] * corr) * inv;
  if (sub == 0) {
    store_head<DH>(o + (size_t)row * d + h * DH, acc);
    stat[(size_t)row * a.heads + h] = make_float2(l > 0.f ? mall + __logf(l) : 0.f, 0.f);
  }
}

// Query side of the backward: with P_ij = exp(s_ij - lse_i) and dP_ij = do_i . v_j,
// D_i = sum_j P_ij dP_ij and dq_i = scale (sum_j P_ij dP_ij k_j - D_i sum_j P_ij k_j), one pass.
template <int DH>
__global__ __launch_bounds__(256) void bw_set_attn_bwd_q_kernel(SetAttn a, const __bf16* __restrict__ dob, int d,
                                                                __bf16* __restrict__ dq, int dqpitch, float2* __restrict__ stat) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) / kSplit;
  const int sub = threadIdx.x % kSplit;
  if (idx >= (long long)a.B * a.nq * a.heads) return;
  const int row = (int)(idx / a.heads), h = (int)(idx - (long long)row * a.heads);
  const int u = row / a.nq, qd = a.qdesc[row];
  float A[DH], Bv[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { A[c] = 0.f; Bv[c] = 0.f; }
  float D = 0.f;
  const float scale = rsqrtf((float)DH);
  const float lse = stat[(size_t)row * a.heads + h].x;
  if (qd >= 0) {
    const HeadVec<DH> qv = load_head<DH>(a.q + (size_t)row * a.qpitch + h * DH);
    const HeadVec<DH> dov = load_head<DH>(dob + (size_t)row * d + h * DH);
    int lo, hi;
    key_range(a, qd, row - u * a.nq, &lo, &hi);
    // (branch-free, unrolled loops as in the forward kernel were slower here: more live registers)
    for (int j = lo + sub; j < hi; j += kSplit) {
      const size_t kr = (size_t)u * a.nk + j;
      if (!visible(qd, a.kdesc[kr], a.gmask)) continue;
      const HeadVec<DH> kv = load_head<DH>(a.k + kr * a.kvpitch + h * DH);
      const HeadVec<DH> vv = load_head<DH>(a.v + kr * a.kvpitch + h * DH);
      const float p = __expf(scale * dot<DH>(qv, kv) - lse);
      const float pd = p * dot<DH>(dov, vv);
      D += pd;
      axpy<DH>(A, pd, kv);
      axpy<DH>(Bv, p, kv);
    }
  }
  D = split_sum(D);
#pragma unroll
  for (int c = 0; c < DH; ++c) A[c] = scale * (split_sum(A[c]) - D * split_sum(Bv[c]));
  if (sub == 0) {
    store_head<DH>(dq + (size_t)row * dqpitch + h * DH, A);
    stat[(size_t)row * a.heads + h].y = D;
  }
}

// Key side: dv_j = sum_i P_ij do_i, dk_j = scale sum_i P_ij (do_i . v_j - D_i) q_i over the user's query
// rows that see key j.
template <int DH>
__global__ __launch_bounds__(256) void bw_set_attn_bwd_kv_kernel(SetAttn a, const __bf16* __restrict__ dob, int d,
                                                                 __bf16* __restrict__ dk, __bf16* __restrict__ dv, int dkvpitch,
                                                                 const float2* __restrict__ stat) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) / kSplit;
  const int sub = threadIdx.x % kSplit;
  if (idx >= (long long)a.B * a.nk * a.heads) return;
  const int kr = (int)(idx / a.heads), h = (int)(idx - (long long)kr * a.heads);
  const int u = kr / a.nk, kd = a.kdesc[kr];
  float gk[DH], gv[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { gk[c] = 0.f; gv[c] = 0.f; }
  if (kd >= 0) {
    const float scale = rsqrtf((float)DH);
    const HeadVec<DH> kv = load_head<DH>(a.k + (size_t)kr * a.kvpitch + h * DH);
    const HeadVec<DH> vv = load_head<DH>(a.v + (size_t)kr * a.kvpitch + h * DH);
    // a sequence key of a self layer is seen by the global rows and by the slots from its own on
    const int own = kr - u * a.nk;
    const int skip_lo = a.m, skip_hi = (a.self && kd >= kSeq) ? max(a.m, own) : a.m;
    for (int i0 = sub; i0 < a.nq - (skip_hi - skip_lo); i0 += kSplit) {
      const int i = i0 < skip_lo ? i0 : i0 + (skip_hi - skip_lo);      // the rows outside [skip_lo, skip_hi)
      const size_t qr = (size_t)u * a.nq + i;
      if (!visible(a.qdesc[qr], kd, a.gmask)) continue;
      const HeadVec<DH> qi = load_head<DH>(a.q + qr * a.qpitch + h * DH);
      const HeadVec<DH> doi = load_head<DH>(dob + qr * d + h * DH);
      const float2 st = stat[qr * a.heads + h];
      const float p = __expf(scale * dot<DH>(qi, kv) - st.x);
      const float ds = scale * p * (dot<DH>(doi, vv) - st.y);
      axpy<DH>(gv, p, doi);
      axpy<DH>(gk, ds, qi);
    }
  }
#pragma unroll
  for (int c = 0; c < DH; ++c) { gk[c] = split_sum(gk[c]); gv[c] = split_sum(gv[c]); }
  if (sub == 0) {
    store_head<DH>(dk + (size_t)kr * dkvpitch + h * DH, gk);
    store_head<DH>(dv + (size_t)kr * dkvpitch + h * DH, gv);
  }
}

// The same three kernels with one workgroup per (user, head): the rows every thread of the loop reads
// (the user's keys and values; for the key side its queries, output gradients and their statistics)
// are copied to LDS once, together with their descriptors, and the loops read them from there (all
// lanes the same address: a broadcast).  One thread per query row (key row), strided by the workgroup.
// Dynamic LDS: n rows x (2 DH bf16 + extras), see set_attn_lds_bytes.
template <int DH>
__device__ __forceinline__ HeadVec<DH> lds_head(const uint4* s, int row) {
  HeadVec<DH> v;
#pragma unroll
  for (int c = 0; c < DH / 8; ++c) v.c[c] = __builtin_bit_cast(bf16x8, s[row * (DH / 8) + c]);
  return v;
}
template <int DH>
__device__ __forceinline__ void stage_heads(uint4* dst, const __bf16* src, size_t pitch, int n, int h) {
  constexpr int CP = DH / 8;
  for (int c = threadIdx.x; c < n * CP; c += blockDim.x)
    dst[c] = *(const uint4*)(src + (size_t)(c / CP) * pitch + h * DH + 8 * (c % CP));
}

// S adjacent lanes share a row: lane s of them takes every S-th key (query) of the loop, and the partial
// results meet through cross-lane shuffles.  The loops are chains of dependent LDS reads and arithmetic,
// and a workgroup has only as many rows as a user has queries (keys): more lanes per row hide the latency.
template <int S>
__device__ __forceinline__ float lanes_sum(float v) {
#pragma unroll
  for (int o = 1; o < S; o <<= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <int S>
__device__ __forceinline__ float lanes_max(float v) {
#pragma unroll
  for (int o = 1; o < S; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

template <int DH, int S>
__global__ __launch_bounds__(512) void bw_set_attn_fwd_lds_kernel(SetAttn a, __bf16* __restrict__ o, int d, float2* __restrict__ stat) {
  extern __shared__ uint4 sm[];
  uint4* sK = sm; uint4* sV = sm + (size_t)a.nk * (DH / 8);
  int* sD = (int*)(sV + (size_t)a.nk * (DH / 8));
  const int u = blockIdx.x / a.heads, h = blockIdx.x - u * a.heads;
  stage_heads<DH>(sK, a.k + (size_t)u * a.nk * a.kvpitch, a.kvpitch, a.nk, h);
  stage_heads<DH>(sV, a.v + (size_t)u * a.nk * a.kvpitch, a.kvpitch, a.nk, h);
  for (int j = threadIdx.x; j < a.nk; j += blockDim.x) sD[j] = a.kdesc[(size_t)u * a.nk + j];
  __syncthreads();
  const float scale = rsqrtf((float)DH);
  const int sub = threadIdx.x % S;
  for (int base = 0; base < a.nq * S; base += blockDim.x) {        // (blockDim.x is a multiple of 64: a row's lanes share a wave)
    const int i = (base + threadIdx.x) / S;
    const bool live = i < a.nq;
    const size_t row = (size_t)u * a.nq + (live ? i : 0);
    const int qd = live ? a.qdesc[row] : -1;
    float acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.f;
    float mx = -3.0e38f, l = 0.f;
    if (qd >= 0) {
      const HeadVec<DH> qv = load_head<DH>(a.q + row * a.qpitch + h * DH);
      int lo, hi;
      key_range(a, qd, i, &lo, &hi);
#pragma unroll 2
      for (int j = lo + sub; j < hi; j += S) {
        const bool vis = visible(qd, sD[j], a.gmask);
        const float sc = vis ? scale * dot<DH>(qv, lds_head<DH>(sK, j)) : -3.0e38f;
        const float mn = fmaxf(mx, sc);
        const float corr = __expf(mx - mn), p = vis ? __expf(sc - mn) : 0.f;
        l = l * corr + p;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] *= corr;
        axpy_packed<DH>(acc, p, lds_head<DH>(sV, j));
        mx = mn;
      }
    }
    const float mall = lanes_max<S>(mx);
    const float corr = __expf(mx - mall);          // a lane without a visible key: l = 0, acc = 0
    l = lanes_sum<S>(l * corr);
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = lanes_sum<S>(acc[c] * corr) * inv;
    if (live && sub == 0) {
      store_head<DH>(o + row * d + h * DH, acc);
      stat[row * a.heads + h] = make_float2(l > 0.f ? mall + __logf(l) : 0.f, 0.f);
    }
  }
}

template <int DH, int S>
__global__ __launch_bounds__(512) void bw_set_attn_bwd_q_lds_kernel(SetAttn a, const __bf16* __restrict__ dob, int d,
                                                                   __bf16* __restrict__ dq, int dqpitch, float2* __restrict__ stat) {
  extern __shared__ uint4 sm[];
  uint4* sK = sm; uint4* sV = sm + (size_t)a.nk * (DH / 8);
  int* sD = (int*)(sV + (size_t)a.nk * (DH / 8));
  const int u = blockIdx.x / a.heads, h = blockIdx.x - u * a.heads;
  stage_heads<DH>(sK, a.k + (size_t)u * a.nk * a.kvpitch, a.kvpitch, a.nk, h);
  stage_heads<DH>(sV, a.v + (size_t)u * a.nk * a.kvpitch, a.kvpitch, a.nk, h);
  for (int j = threadIdx.x; j < a.nk; j += blockDim.x) sD[j] = a.kdesc[(size_t)u * a.nk + j];
  __syncthreads();
  const float scale = rsqrtf((float)DH);
  const int sub = threadIdx.x % S;
  for (int base = 0; base < a.nq * S; base += blockDim.x) {
    const int i = (base + threadIdx.x) / S;
    const bool live = i < a.nq;
    const size_t row = (size_t)u * a.nq + (live ? i : 0);
    const int qd = live ? a.qdesc[row] : -1;
    float A[DH], Bv[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) { A[c] = 0.f; Bv[c] = 0.f; }
    float D = 0.f;
    if (qd >= 0) {
      const float lse = stat[row * a.heads + h].x;
      const HeadVec<DH> qv = load_head<DH>(a.q + row * a.qpitch + h * DH);
      const HeadVec<DH> dov = load_head<DH>(dob + row * d + h * DH);
      int lo, hi;
      key_range(a, qd, i, &lo, &hi);
      for (int j = lo + sub; j < hi; j += S) {
        if (!visible(qd, sD[j], a.gmask)) continue;
        const HeadVec<DH> kv = lds_head<DH>(sK, j);
        const float p = __expf(scale * dot<DH>(qv, kv) - lse);
        const float pd = p * dot<DH>(dov, lds_head<DH>(sV, j));
        D += pd;
        axpy_packed<DH>(A, pd, kv);
        axpy_packed<DH>(Bv, p, kv);
      }
    }
    D = lanes_sum<S>(D);
#pragma unroll
    for (int c = 0; c < DH; ++c) A[c] = scale * (lanes_sum<S>(A[c]) - D * lanes_sum<S>(Bv[c]));
    if (live && sub == 0) {
      store_head<DH>(dq + row * dqpitch + h * DH, A);
      stat[row * a.heads + h].y = D;
    }
  }
}

template <int DH, int S>
__global__ __launch_bounds__(512) void bw_set_attn_bwd_kv_lds_kernel(SetAttn a, const __bf16* __restrict__ dob, int d,
                                                                    __bf16* __restrict__ dk, __bf16* __restrict__ dv, int dkvpitch,
                                                                    const float2* __restrict__ stat) {
  extern __shared__ uint4 sm[];
  uint4* sQ = sm; uint4* sO = sm + (size_t)a.nq * (DH / 8);
  float2* sS = (float2*)(sO + (size_t)a.nq * (DH / 8));
  int* sD = (int*)(sS + a.nq);
  const int u = blockIdx.x / a.heads, h = blockIdx.x - u * a.heads;
  stage_heads<DH>(sQ, a.q + (size_t)u * a.nq * a.qpitch, a.qpitch, a.nq, h);
  stage_heads<DH>(sO, dob + (size_t)u * a.nq * d, d, a.nq, h);
  for (int i = threadIdx.x; i < a.nq; i += blockDim.x) {
    sS[i] = stat[((size_t)u * a.nq + i) * a.heads + h];
    sD[i] = a.qdesc[(size_t)u * a.nq + i];
  }
  __syncthreads();
  const float scale = rsqrtf((float)DH);
  const int sub = threadIdx.x % S;
  for (int base = 0; base < a.nk * S; base += blockDim.x) {
    const int own = (base + threadIdx.x) / S;
    const bool live = own < a.nk;
    const size_t kr = (size_t)u * a.nk + (live ? own : 0);
    const int kd = live ? a.kdesc[kr] : -1;
    float gk[DH], gv[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) { gk[c] = 0.f; gv[c] = 0.f; }
    if (kd >= 0) {
      const HeadVec<DH> kv = load_head<DH>(a.k + kr * a.kvpitch + h * DH);
      const HeadVec<DH> vv = load_head<DH>(a.v + kr * a.kvpitch + h * DH);
      // a sequence key of a self layer is seen by the global rows and by the slots from its own on
      const int skip_lo = a.m, skip_hi = (a.self && kd >= kSeq) ? max(a.m, own) : a.m;
      for (int i0 = sub; i0 < a.nq - (skip_hi - skip_lo); i0 += S) {
        const int i = i0 < skip_lo ? i0 : i0 + (skip_hi - skip_lo);      // the rows outside [skip_lo, skip_hi)
        if (!visible(sD[i], kd, a.gmask)) continue;
        const HeadVec<DH> qi = lds_head<DH>(sQ, i);
        const HeadVec<DH> doi = lds_head<DH>(sO, i);
        const float2 st = sS[i];
        const float p = __expf(scale * dot<DH>(qi, kv) - st.x);
        const float ds = scale * p * (dot<DH>(doi, vv) - st.y);
        axpy_packed<DH>(gv, p, doi);
        axpy_packed<DH>(gk, ds, qi);
      }
    }
#pragma unroll
    for (int c = 0; c < DH; ++c) { gk[c] = lanes_sum<S>(gk[c]); gv[c] = lanes_sum<S>(gv[c]); }
    if (live && sub == 0) {
      store_head<DH>(dk + kr * dkvpitch + h * DH, gk);
      store_head<DH>(dv + kr * dkvpitch + h * DH, gv);
    }
  }
}

// Head and loss (Eq. 1-2) for one user per block: logit = <head_w, the m global rows of Y> + head_b,
// loss += (softplus form of the cross-entropy) / B, dlogit = (sigmoid(logit) - label) / B, and the
// gradients that follow: dY (global rows dlogit head_w, the other rows zero; fp32 and bf16), head_w, head_b.
__global__ __launch_bounds__(256) void bw_head_kernel(const float* __restrict__ Y, const __bf16* __restrict__ hw,
                                                      const __bf16* __restrict__ hb, const float* __restrict__ labels,
                                                      int B, int n, int m, int d, float* __restrict__ logits,
                                                      float* loss, float* __restrict__ dY, __bf16* __restrict__ dYb,
                                                      float* dhw, float* dhb) {
  __shared__ float red[4];
  __shared__ float dl_s;
  const int u = blockIdx.x;
  const float* y = Y + (size_t)u * n * d;
  float s = 0.f;
  for (int j = threadIdx.x; j < m * d; j += 256) s += y[j] * (float)hw[j];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float z = red[0] + red[1] + red[2] + red[3] + (float)hb[0];
    const float lab = labels[u];
    const float e = __expf(-fabsf(z));
    const float sig = z >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
    const float dl = (sig - lab) / (float)B;
    if (logits) logits[u] = z;
    unsafeAtomicAdd(loss, (fmaxf(z, 0.f) - z * lab + log1pf(e)) / (float)B);
    unsafeAtomicAdd(dhb, dl);
    dl_s = dl;
  }
  __syncthreads();
  const float dl = dl_s;
  for (int j = threadIdx.x; j < n * d; j += 256) {
    const float g = j < m * d ? dl * (float)hw[j] : 0.f;
    dY[(size_t)u * n * d + j] = g;
    dYb[(size_t)u * n * d + j] = (__bf16)g;
    if (j < m * d) unsafeAtomicAdd(dhw + j, dl * y[j]);
  }
}

// dG = the global rows of dO + the global rows of dR; dM[u][t] = dR's row of merged token t (zeros past T_u)
__global__ __launch_bounds__(256) void bw_split_grad_kernel(StackGeom g, int d, const float* __restrict__ dO,
                                                            const float* __restrict__ dR, float* __restrict__ dG,
                                                            float* __restrict__ dM) {
  const int n = g.m + g.k, nk = g.m + g.T, d4 = d / 4;
  const size_t total = (size_t)g.B * nk * d4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int c = (int)(i % d4) * 4;
    const size_t row = i / d4;
    const int u = (int)(row / nk), r = (int)(row - (size_t)u * nk);
    const f32x4 v = *(const f32x4*)(dR + row * d + c);
    if (r < g.m) {
      *(f32x4*)(dG + ((size_t)u * g.m + r) * d + c) = v + *(const f32x4*)(dO + ((size_t)u * n + r) * d + c);
    } else {
      const int t = r - g.m;
      f32x4 z = {0.f, 0.f, 0.f, 0.f};
      *(f32x4*)(dM + ((size_t)u * g.T + t) * d + c) = t < merged_len(g, u) ? v : z;
    }
  }
}
// dM[u][t_i] += dO's row of query slot i (each slot of a user holds a different merged token)
// (learnable query tokens: the slot's gradient belongs to row sl of the parameter instead, summed over the users)
__global__ __launch_bounds__(256) void bw_slot_grad_kernel(StackGeom g, int d, const float* __restrict__ dO,
                                                           const int* __restrict__ qdesc, float* __restrict__ dM,
                                                           float* dql) {
  const int n = g.m + g.k, d4 = d / 4;
  const size_t total = (size_t)g.B * g.k * d4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int c = (int)(i % d4) * 4;
    const size_t s = i / d4;
    const int u = (int)(s / g.k), sl = (int)(s - (size_t)u * g.k);
    const int dsc = qdesc[(size_t)u * n + g.m + sl];
    if (dsc < kSeq) continue;
    const f32x4 v = *(const f32x4*)(dO + ((size_t)u * n + g.m + sl) * d + c);
    if (g.learn) {
#pragma unroll
      for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dql + (size_t)sl * d + c + e, v[e]);
    } else {
      float* dst = dM + ((size_t)u * g.T + (dsc - kSeq)) * d + c;
      *(f32x4*)dst = *(const f32x4*)dst + v;
    }
  }
}


// ------------------------------------------------------------------------------------
// Input generation (Section 3.5.1): x = [E + pos ; tdiff] per valid token, H = act(x w1 + b1) w2 + b2.
// x[r][:] as bf16, zeros for padded tokens
__global__ __launch_bounds__(256) void bw_input_rows_kernel(const __bf16* __restrict__ E, const __bf16* __restrict__ pos,
                                                            const __bf16* __restrict__ td, __bf16* __restrict__ x,
                                                            RowGeom q, int d, int de) {
  const size_t n = (size_t)q.ntok * d / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i * 4 / d), c = (int)(i * 4 - (size_t)r * d);
    const int u = r / q.L, p = r - u * q.L;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (p < row_len(q, u)) {
      if (c < de) v = load_bf16x4(E + (size_t)r * de + c) + load_bf16x4(pos + (size_t)p * de + c);
      else v = load_bf16x4(td + (size_t)r * (d - de) + (c - de));
    }
    store_bf16x4(x + i * 4, v);
  }
}
// the upstream gradient as bf16, zeros for padded tokens
__global__ __launch_bounds__(256) void bw_cast_rows_kernel(const float* __restrict__ g, __bf16* __restrict__ gb, RowGeom q, int d) {
  const size_t n = (size_t)q.ntok * d / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i * 4 / d);
    const int u = r / q.L, p = r - u * q.L;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (p < row_len(q, u)) v = *(const f32x4*)(g + i * 4);
    store_bf16x4(gb + i * 4, v);
  }
}
// dx [ntok][d] -> dE [ntok][de] and dtdiff [ntok][d - de], zeros for padded tokens
__global__ __launch_bounds__(256) void bw_split_input_grad_kernel(const float* __restrict__ dx, float* __restrict__ dE,
                                                                  float* __restrict__ dtd, RowGeom q, int d, int de) {
  const size_t n = (size_t)q.ntok * d / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i * 4 / d), c = (int)(i * 4 - (size_t)r * d);
    const int u = r / q.L, p = r - u * q.L;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (p < row_len(q, u)) v = *(const f32x4*)(dx + i * 4);
    if (c < de) *(f32x4*)(dE + (size_t)r * de + c) = v;
    else *(f32x4*)(dtd + (size_t)r * (d - de) + (c - de)) = v;
  }
}
// dpos[p][c] = sum over the users whose sequence reaches position p of dx[u L + p][c], c < de
__global__ __launch_bounds__(256) void bw_pos_grad_kernel(const float* __restrict__ dx, float* __restrict__ dpos, RowGeom q,
                                                          int B, int d, int de) {
  const size_t n = (size_t)q.L * de / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int p = (int)(i * 4 / de), c = (int)(i * 4 - (size_t)p * de);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int u = 0; u < B; ++u)
      if (p < row_len(q, u)) s += *(const f32x4*)(dx + ((size_t)u * q.L + p) * d + c);
    *(f32x4*)(dpos + i * 4) = s;
  }
}

// out[c][r] = in[r][c]  (bf16, small parameter matrices; 32 x 32 tiles through LDS)
__global__ __launch_bounds__(256) void bw_transpose_kernel(const __bf16* __restrict__ in, __bf16* __restrict__ out, int rows, int cols) {
  __shared__ __bf16 t[32][33];
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32, x = threadIdx.x & 31, y = threadIdx.x >> 5;
  for (int i = y; i < 32; i += 8)
    if (r0 + i < rows && c0 + x < cols) t[i][x] = in[(size_t)(r0 + i) * cols + c0 + x];
  __syncthreads();
  for (int i = y; i < 32; i += 8)
    if (c0 + i < cols && r0 + x < rows) out[(size_t)(c0 + i) * rows + r0 + x] = t[x][i];
}

// ------------------------------------------------------------------------------------ host side
static inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// Parameter gradients of one block: fp32, in the order of the longer_block members.
struct GradLayout { size_t ln1_g, ln1_b, wq, bq, wk, bk, wv, bv, wo, bo, ln2_g, ln2_b, w1, b1, w2, b2, total; };
static GradLayout grad_layout(int d, int f) {
  GradLayout g;
  size_t o = 0;
  auto take = [&](size_t n) { size_t at = o; o += n; return at; };
  g.ln1_g = take(d); g.ln1_b = take(d);
  g.wq = take((size_t)d * d); g.bq = take(d);
  g.wk = take((size_t)d * d); g.bk = take(d);
  g.wv = take((size_t)d * d); g.bv = take(d);
  g.wo = take((size_t)d * d); g.bo = take(d);
  g.ln2_g = take(d); g.ln2_b = take(d);
  g.w1 = take((size_t)d * f); g.b1 = take(f);
  g.w2 = take((size_t)f * d); g.b2 = take(d);
  g.total = o;
  return g;      // ln*_b follows ln*_g directly: ln_bwd writes the two as one vector
}

// tiles x slices of a split GEMM <= kMaxPartials, each a 128 x 128 fp32 tile
constexpr int kMaxPartials = 512;
constexpr size_t kPartialBytes = (size_t)kMaxPartials * 128 * 128 * 4;

struct Workspace {
  size_t wcat, bcat;                       // per layer: [d][3d] bf16, [3d] bf16
  size_t xin;                              // per layer: fp32 [ntok][d]
  size_t w1t, wcatt, wot;                  // per layer, transposed: W1 [f][d], [wq | wk | wv] [3d][d], W_O [d][d] (bf16)
  size_t n1, qkv, o, xmid, n2, a;          // one block's recomputed intermediates
  size_t dy, dyb, dh, dn, dxm, dxmb, dob, dqkv, stat;
  size_t part, bpart;                      // partial parameter gradients of one split GEMM (matrix, bias)
  size_t fwd, fwd_bytes, ztmp;             // the fused forward kernel's scratch and output when it recomputes block inputs
  size_t total;
};
static Workspace workspace(int layers, size_t ntok, int d, int f, int heads, size_t fwd_bytes, size_t ztmp_bytes) {
  Workspace w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
  w.wcat = take((size_t)layers * d * 3 * d * 2);
  w.bcat = take((size_t)layers * up256((size_t)3 * d * 2));
  w.w1t = take((size_t)layers * d * f * 2);
  w.wcatt = take((size_t)layers * d * 3 * d * 2);
  w.wot = take((size_t)layers * d * d * 2);
  w.xin = take((size_t)layers * ntok * d * 4);
  w.n1 = take(ntok * d * 2);
  w.qkv = take(ntok * 3 * d * 2);
  w.o = take(ntok * d * 2);
  w.xmid = take(ntok * d * 4);
  w.n2 = take(ntok * d * 2);
  w.a = take(ntok * f * 2);
  w.dy = take(ntok * d * 4);
  w.dyb = take(ntok * d * 2);
  w.dh = take(ntok * f * 2);
  w.dn = take(ntok * d * 2);
  w.dxm = take(ntok * d * 4);
  w.dxmb = take(ntok * d * 2);
  w.dob = take(ntok * d * 2);
  w.dqkv = take(ntok * 3 * d * 2);
  w.stat = take(ntok * heads * 8);
  w.part = take(kPartialBytes);
  w.bpart = take((size_t)kMaxPartials * 2048 * 4);
  w.fwd = take(fwd_bytes);
  w.fwd_bytes = fwd_bytes;
  w.ztmp = take(ztmp_bytes);
  w.total = o;
  return w;
}

struct Dims { int d, f, heads, dh, layers, K, T; size_t ntok; };

// the merge backward's workspace for a batch: with more than one block the fused forward kernel
// recomputes the block inputs (its scratch; a staging copy when L is not a multiple of K, whose rows
// then sit at [B, T K] instead of [B, L])
static Workspace merge_workspace(const longer_config* c, const Dims& s, int B, int L) {
  size_t fwd = 0, zt = 0;
  if (s.layers > 1) {
    fwd = longer_workspace_bytes(c, B, L);
    if (L % s.K) zt = (size_t)B * s.T * s.K * s.d * 4;
  }
  return workspace(s.layers, s.ntok, s.d, s.f, s.heads, fwd, zt);
}

static int check(const longer_config* c, int B, int L, Dims* s) {
  if (!c) return api_error(LONGER_ERR_ARG, "config is NULL");
  if (c->dtype != LONGER_BF16) return api_error(LONGER_ERR_ARG, "the backward pass is mixed precision: dtype must be LONGER_BF16");
  if (c->act != LONGER_ACT_GELU_ERF && c->act != LONGER_ACT_RELU) return api_error(LONGER_ERR_ARG, "act %d unknown", c->act);
  if (c->merge != LONGER_MERGE_MEAN && c->merge != LONGER_MERGE_CONCAT) return api_error(LONGER_ERR_ARG, "merge %d unknown", c->merge);
  if (c->K <= 0 || c->K > kMaxGroup || 32 % c->K) return api_error(LONGER_ERR_ARG, "K=%d must divide 32", c->K);
  if (c->d <= 0 || c->d % 32) return api_error(LONGER_ERR_ARG, "d=%d must be a positive multiple of 32", c->d);
  int d = c->d;
  if (c->merge == LONGER_MERGE_CONCAT) {
    if (d % c->K) return api_error(LONGER_ERR_ARG, "concat merge: K=%d must divide d=%d", c->K, d);
    d /= c->K;
  }
  if (d != 32 && d != 64 && d != 128 && d != 256) return api_error(LONGER_ERR_ARG, "InnerTrans width %d unsupported (32, 64, 128 or 256)", d);
  if (c->inner_layers <= 0 || c->inner_layers > 32) return api_error(LONGER_ERR_ARG, "inner_layers=%d out of range", c->inner_layers);
  if (c->inner_heads <= 0 || d % c->inner_heads) return api_error(LONGER_ERR_ARG, "inner_heads=%d must divide the InnerTrans width %d", c->inner_heads, d);
  const int dh = d / c->inner_heads;
  if (dh != 16 && dh != 32) return api_error(LONGER_ERR_ARG, "head width %d unsupported (16 or 32)", dh);
  if (c->ffn_mult <= 0 || c->ffn_mult * d > 2048) return api_error(LONGER_ERR_ARG, "ffn_mult=%d: the FFN hidden width must be at most 2048", c->ffn_mult);
  if (!(c->ln_eps > 0.f)) return api_error(LONGER_ERR_ARG, "ln_eps must be positive");
  if (B <= 0 || L <= 0) return api_error(LONGER_ERR_ARG, "B=%d, L=%d must be positive", B, L);
  const long long ntok = (long long)B * L;
  if (ntok * c->inner_heads >= (1ll << 31) - 256 || ntok * d * c->ffn_mult >= (1ll << 40))
    return api_error(LONGER_ERR_ARG, "B * L = %lld token rows are too many for one call; split the batch", ntok);
  s->d = d; s->f = c->ffn_mult * d; s->heads = c->inner_heads; s->dh = dh; s->layers = c->inner_layers;
  s->K = c->K; s->T = (L + c->K - 1) / c->K; s->ntok = (size_t)ntok;
  return 0;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int launched(const char* what) {
  return hipGetLastError() == hipSuccess ? 0 : api_error(LONGER_ERR_HIP, "%s launch failed", what);
}

static int reduce(hipStream_t st, const float* part, int nsplit, int count, float* out, bool accumulate = false) {
  int shares = nsplit / 32;                 // at least 32 slices per block
  shares = shares < 1 ? 1 : (shares > 64 ? 64 : shares);
  bw_reduce_kernel<<<dim3((count / 4 + 63) / 64, shares), 256, 0, st>>>(part, nsplit, count, out, accumulate ? 1 : 0);
  return launched("gradient reduction");
}

static int gemm(hipStream_t st, bool a_kc, bool b_kc, GemmArgs g, int splits) {
  if (!aligned16(g.A) || !aligned16(g.B) || g.lda % 8 || g.ldb % 8) return api_error(LONGER_ERR_ARG, "backward GEMM operand misaligned");
  const int ntm = (g.M + 127) / 128, ntn = (g.N + 127) / 128;
  g.nsplit = splits;
  const int outer = g.epi == EPI_PARTIAL ? splits : ntm, inner = g.epi == EPI_PARTIAL ? ntm * ntn : ntn;
  dim3 grid((unsigned)(((outer + 7) / 8) * 8 * inner));            // see the tile order in the kernel
  if (a_kc && b_kc && splits == 1 && (g.Kc == 32 || g.Kc == 64 || g.Kc == 128) &&
      (g.epi == EPI_FFN_MID || g.epi == EPI_BF16 || g.epi == EPI_RES_F32 || g.epi == EPI_F32)) {
    if (g.epi == EPI_FFN_MID && (!aligned16(g.A2) || !aligned16(g.B2) || g.lda2 % 8 || g.ldb2 % 8))
      return api_error(LONGER_ERR_ARG, "backward GEMM operand misaligned");
    // one workgroup per compute unit, each walking over row tiles for its 128 columns
    int P = (kComputeUnits / ntn) / 8 * 8;
    if (P < 8) P = 8;
    if (P > ((ntm + 7) / 8) * 8) P = ((ntm + 7) / 8) * 8;
    dim3 pg((unsigned)(P * ntn));
    const bool dual = g.epi == EPI_FFN_MID;
#define LONGER_ROWGEMM(KK) (dual ? bw_rowgemm_kernel<KK, true><<<pg, 512, 0, st>>>(g, P) : bw_rowgemm_kernel<KK, false><<<pg, 512, 0, st>>>(g, P))
    if (g.Kc == 128) LONGER_ROWGEMM(128); else if (g.Kc == 64) LONGER_ROWGEMM(64); else LONGER_ROWGEMM(32);
#undef LONGER_ROWGEMM
    return launched("backward row GEMM");
  }
  if (g.epi == EPI_FFN_MID) {
    if (!(a_kc && b_kc) || !aligned16(g.A2) || !aligned16(g.B2) || g.lda2 % 8 || g.ldb2 % 8)
      return api_error(LONGER_ERR_ARG, "backward GEMM operand misaligned");
    bw_gemm_kernel<true, true, true><<<grid, 256, 0, st>>>(g);
  } else if (a_kc && b_kc) bw_gemm_kernel<true, true><<<grid, 256, 0, st>>>(g);
  else if (a_kc && !b_kc) bw_gemm_kernel<true, false><<<grid, 256, 0, st>>>(g);
  else if (!a_kc && !b_kc) bw_gemm_kernel<false, false><<<grid, 256, 0, st>>>(g);
  else return api_error(LONGER_ERR_ARG, "backward GEMM form not built");
  return launched("backward GEMM");
}

// y = x W (+ epilogue): x [ntok][kc] row-major, W [kc][.. n columns, pitch ldb] row-major; outputs,
// residual and pre-activation [ntok][n]
static int gemm_rows(hipStream_t st, const __bf16* x, int kc, const __bf16* W, int n, size_t ntok, int epi, int act,
                     void* out, void* out2, const __bf16* bias, const float* res, const __bf16* pre, int ldb = 0,
                     RowsValid rows = RowsValid{nullptr, 0}) {
  GemmArgs g = {};
  g.rows = rows;
  g.A = x; g.lda = kc; g.B = W; g.ldb = ldb ? ldb : n; g.M = (int)ntok; g.N = n; g.Kc = kc;
  g.epi = epi; g.act = act; g.out = out; g.out2 = out2; g.ldo = n; g.bias = bias; g.res = res; g.pre = pre;
  return gemm(st, true, false, g, 1);
}
// y = x W (+ epilogue) with W handed over transposed, wt [n][kc]: both operands contraction-contiguous
static int gemm_rows_wt(hipStream_t st, const __bf16* x, int kc, const __bf16* wt, int n, size_t ntok, int epi,
                        void* out, const __bf16* bias, const float* res, RowsValid rows) {
  GemmArgs g = {};
  g.rows = rows;
  g.A = x; g.lda = kc; g.B = wt; g.ldb = kc; g.M = (int)ntok; g.N = n; g.Kc = kc;
  g.epi = epi; g.out = out; g.ldo = n; g.bias = bias; g.res = res;
  return gemm(st, true, true, g, 1);
}
// dx = dy W^T: dy [ntok][kc], W [n][.. kc columns, pitch ldb] row-major (the forward's [in = n][out = kc])
static int gemm_rows_t(hipStream_t st, const __bf16* dy, int kc, const __bf16* W, int n, size_t ntok, int epi, int act,
                       void* out, const __bf16* pre, int ldb = 0, RowsValid rows = RowsValid{nullptr, 0}) {
  GemmArgs g = {};
  g.rows = rows;
  g.A = dy; g.lda = kc; g.B = W; g.ldb = ldb ? ldb : kc; g.M = (int)ntok; g.N = n; g.Kc = kc;
  g.epi = epi; g.act = act; g.out = out; g.ldo = n; g.pre = pre;
  return gemm(st, true, true, g, 1);
}
// The middle of the FFN's backward in one launch: v = x W1 + b1 (recomputed, not stored), g = dy W2^T,
// a_out = bf16(act(v)), dh_out = bf16(g act'(v)).  x, dy [ntok][d]; w1t = W1 transposed, [f][d]; w2 [f][d].
static int gemm_ffn_mid(hipStream_t st, const __bf16* x, const __bf16* dy, int d, const __bf16* w1t, const __bf16* w2, int f,
                        const __bf16* b1, size_t ntok, int act, __bf16* dh_out, __bf16* a_out, RowsValid rows) {
  GemmArgs g = {};
  g.rows = rows;
  g.A = x; g.lda = d; g.B = w1t; g.ldb = d; g.A2 = dy; g.lda2 = d; g.B2 = w2; g.ldb2 = d;
  g.M = (int)ntok; g.N = f; g.Kc = d;
  g.epi = EPI_FFN_MID; g.act = act; g.out = dh_out; g.out2 = a_out; g.ldo = f; g.bias = b1;
  return gemm(st, true, true, g, 1);
}
static int transpose(hipStream_t st, const __bf16* in, __bf16* out, int rows, int cols) {
  bw_transpose_kernel<<<dim3((cols + 31) / 32, (rows + 31) / 32), 256, 0, st>>>(in, out, rows, cols);
  return launched("transpose");
}
// dW [m][n] = x^T dy: x [ntok][.. m columns, pitch lda], dy [ntok][.. n columns, pitch ldb]
// and db [n] = column sums of dy
static int gemm_wgrad(hipStream_t st, const __bf16* x, int lda, int m, const __bf16* dy, int ldb, int n, size_t ntok,
                      float* part, float* bpart, float* dW, float* db, RowsValid rows = RowsValid{nullptr, 0}) {
  GemmArgs g = {};
  g.rows = rows;
  g.A = x; g.lda = lda; g.B = dy; g.ldb = ldb; g.M = m; g.N = n; g.Kc = (int)ntok;
  const int tiles = ((m + 127) / 128) * ((n + 127) / 128);
  if (tiles > kMaxPartials) return api_error(LONGER_ERR_ARG, "parameter matrix %d x %d too large for the backward pass", m, n);
  int splits = kMaxPartials / tiles;
  const int most = (int)((ntok + 255) / 256);
  if (splits > most) splits = most;
  const int steps = (int)((ntok + 31) / 32);
  if (splits > steps) splits = steps;
  g.epi = EPI_PARTIAL; g.out = part; g.ldo = n;
  // The bias gradient follows its matrix in every gradient buffer, and `bpart` follows `part` in every
  // workspace: a slice's bias partial then goes right behind its matrix partial, and one reduction
  // launch sums both.
  const bool together = db == dW + (size_t)m * n && bpart == part + kPartialBytes / 4;
  g.pstride = together ? m * n + n : m * n;
  g.pstride2 = together ? m * n + n : n;
  g.out2 = together ? part + (size_t)m * n : bpart;
  int rc = gemm(st, false, false, g, splits);
  if (rc) return rc;
  if (together) return reduce(st, part, splits, m * n + n, dW);
  rc = reduce(st, part, splits, m * n, dW);
  if (rc) return rc;
  return reduce(st, bpart, splits, n, db);
}

static void ln_fwd(hipStream_t st, unsigned grid, int d, const float* x, const __bf16* g, const __bf16* b, __bf16* out,
                   int ntok, float eps, RowsValid rows = RowsValid{nullptr, 0}) {
  switch (d) {
    case 32: bw_ln_fwd_kernel<8><<<grid, 256, 0, st>>>(x, g, b, out, ntok, eps, rows); break;
    case 64: bw_ln_fwd_kernel<16><<<grid, 256, 0, st>>>(x, g, b, out, ntok, eps, rows); break;
    case 128: bw_ln_fwd_kernel<32><<<grid, 256, 0, st>>>(x, g, b, out, ntok, eps, rows); break;
    default: bw_ln_fwd_kernel<64><<<grid, 256, 0, st>>>(x, g, b, out, ntok, eps, rows); break;
  }
}
// dgb: the gain gradient [d] followed directly by the shift gradient [d]
static int ln_bwd(hipStream_t st, unsigned grid, int d, const __bf16* dn, const float* x, const __bf16* g, const float* dres,
                  float* dx, __bf16* dxb, float* part, float* dgb, int ntok, float eps, bool accumulate = false,
                  RowsValid rows = RowsValid{nullptr, 0}) {
  switch (d) {
    case 32: bw_ln_bwd_kernel<8><<<grid, 256, 0, st>>>(dn, x, g, dres, dx, dxb, part, ntok, eps, rows); break;
    case 64: bw_ln_bwd_kernel<16><<<grid, 256, 0, st>>>(dn, x, g, dres, dx, dxb, part, ntok, eps, rows); break;
    case 128: bw_ln_bwd_kernel<32><<<grid, 256, 0, st>>>(dn, x, g, dres, dx, dxb, part, ntok, eps, rows); break;
    default: bw_ln_bwd_kernel<64><<<grid, 256, 0, st>>>(dn, x, g, dres, dx, dxb, part, ntok, eps, rows); break;
  }
  if (hipGetLastError() != hipSuccess) return api_error(LONGER_ERR_HIP, "LayerNorm backward launch failed");
  return reduce(st, part, (int)grid, 2 * d, dgb, accumulate);
}

static unsigned flat_grid(size_t n) {
  size_t b = (n + 255) / 256;
  return (unsigned)(b > 65536 ? 65536 : (b ? b : 1));
}

#define BW_TRY(x) do { int rc_ = (x); if (rc_) return rc_; } while (0)

static int run(const longer_config* c, const longer_block* inner, const void* H, const int32_t* lens, int B, int L,
               const float* dM, float* dH, float* grads, char* ws, hipStream_t st, const Dims& s) {
  const int d = s.d, f = s.f;
  const size_t nt = s.ntok;
  const Workspace w = merge_workspace(c, s, B, L);
  const GradLayout gl = grad_layout(d, f);
  const RowGeom q = {lens, L, s.K, (int)nt};
  const RowsValid rv = {lens, L};            // padded token rows are left out (lens NULL: there are none)
  auto xin = [&](int l) { return (float*)(ws + w.xin) + (size_t)l * nt * d; };
  auto wcat = [&](int l) { return (__bf16*)(ws + w.wcat) + (size_t)l * d * 3 * d; };
  auto bcat = [&](int l) { return (__bf16*)(ws + w.bcat + (size_t)l * up256((size_t)3 * d * 2)); };
  __bf16* n1 = (__bf16*)(ws + w.n1);   __bf16* qkv = (__bf16*)(ws + w.qkv); __bf16* o = (__bf16*)(ws + w.o);
  float* xmid = (float*)(ws + w.xmid); __bf16* n2 = (__bf16*)(ws + w.n2);
  auto w1t = [&](int l) { return (__bf16*)(ws + w.w1t) + (size_t)l * d * f; };
  auto wcatt = [&](int l) { return (__bf16*)(ws + w.wcatt) + (size_t)l * d * 3 * d; };
  auto wot = [&](int l) { return (__bf16*)(ws + w.wot) + (size_t)l * d * d; };
  __bf16* a = (__bf16*)(ws + w.a);     float* dy = (float*)(ws + w.dy);     __bf16* dyb = (__bf16*)(ws + w.dyb);
  __bf16* dh = (__bf16*)(ws + w.dh);   __bf16* dn = (__bf16*)(ws + w.dn);   float* dxm = (float*)(ws + w.dxm);
  __bf16* dxmb = (__bf16*)(ws + w.dxmb); __bf16* dob = (__bf16*)(ws + w.dob); __bf16* dqkv = (__bf16*)(ws + w.dqkv);
  float2* stat = (float2*)(ws + w.stat);
  float* part = (float*)(ws + w.part);
  float* bpart = (float*)(ws + w.bpart);
  const unsigned ln_grid = (unsigned)((nt + 3) / 4 > 4096 ? 4096 : (nt + 3) / 4);   // 4096 x 2 x 256 floats fit `part`
  const unsigned ah_grid = (unsigned)((nt * s.heads + 255) / 256);

  bw_zero_kernel<<<flat_grid(gl.total * s.layers), 256, 0, st>>>(grads, gl.total * s.layers);
  BW_TRY(launched("zero fill"));
  for (int l = 0; l < s.layers; ++l) {
    const longer_block& b = inner[l];
    bw_concat_qkv_kernel<<<64, 256, 0, st>>>((const __bf16*)b.wq, (const __bf16*)b.wk, (const __bf16*)b.wv, (const __bf16*)b.bq,
                                             (const __bf16*)b.bk, (const __bf16*)b.bv, wcat(l), bcat(l), d);
    BW_TRY(launched("weight concatenation"));
    BW_TRY(transpose(st, (const __bf16*)b.w1, w1t(l), d, f));
    BW_TRY(transpose(st, wcat(l), wcatt(l), d, 3 * d));
    BW_TRY(transpose(st, (const __bf16*)b.wo, wot(l), d, d));
  }
  bw_load_x0_kernel<<<flat_grid(nt * d / 4), 256, 0, st>>>((const __bf16*)H, xin(0), q, d);
  BW_TRY(launched("input load"));

  // one block forward from its input x, up to the FFN's input: intermediates into the workspace
  auto forward = [&](int l) -> int {
    const longer_block& b = inner[l];
    const float* x = xin(l);
    ln_fwd(st, ln_grid, d, x, (const __bf16*)b.ln1_g, (const __bf16*)b.ln1_b, n1, (int)nt, c->ln_eps, rv);
    BW_TRY(launched("LayerNorm"));
    BW_TRY(gemm_rows_wt(st, n1, d, wcatt(l), 3 * d, nt, EPI_BF16, qkv, bcat(l), nullptr, rv));
    group_attn(0, s.dh, s.K, ah_grid, st, qkv, nullptr, o, nullptr, q, d, s.heads);
    BW_TRY(launched("group attention"));
    BW_TRY(gemm_rows_wt(st, o, d, wot(l), d, nt, EPI_RES_F32, xmid, (const __bf16*)b.bo, x, rv));
    ln_fwd(st, ln_grid, d, xmid, (const __bf16*)b.ln2_g, (const __bf16*)b.ln2_b, n2, (int)nt, c->ln_eps, rv);
    return launched("LayerNorm");
  };

  // the chain of block inputs (recomputed: nothing is kept from a forward call), by the fused forward
  // kernel: its fp32 residual stream after l + 1 blocks is block l + 1's input
  for (int l = 0; l + 1 < s.layers; ++l) {
    const bool direct = L % s.K == 0;
    float* z = direct ? xin(l + 1) : (float*)(ws + w.ztmp);
    BW_TRY(inner_chain_f32(c, inner, l + 1, H, lens, B, L, z, ws + w.fwd, w.fwd_bytes, st));
    if (!direct) {
      bw_take_rows_kernel<<<flat_grid(nt * d / 4), 256, 0, st>>>(z, xin(l + 1), B, L, s.T * s.K, d);
      BW_TRY(launched("row copy"));
    }
  }

  bw_merge_bwd_kernel<<<flat_grid(nt * d / 4), 256, 0, st>>>(dM, dy, dyb, q, d, s.T, c->merge == LONGER_MERGE_CONCAT);
  BW_TRY(launched("merge gradient"));

  for (int l = s.layers - 1; l >= 0; --l) {
    const longer_block& b = inner[l];
    float* g = grads + (size_t)l * gl.total;
    BW_TRY(forward(l));                          // this block's intermediates, from its input alone
    // FFN: y = xmid + act(n2 W1 + b1) W2 + b2; the hidden pre-activation is formed inside the launch
    // that takes its gradient, and only the activated values and the hidden gradient reach memory
    BW_TRY(gemm_ffn_mid(st, n2, dyb, d, w1t(l), (const __bf16*)b.w2, f, (const __bf16*)b.b1, nt, c->act, dh, a, rv));
    BW_TRY(gemm_wgrad(st, a, f, f, dyb, d, d, nt, part, bpart, g + gl.w2, g + gl.b2, rv));
    BW_TRY(gemm_wgrad(st, n2, d, d, dh, f, f, nt, part, bpart, g + gl.w1, g + gl.b1, rv));
    BW_TRY(gemm_rows_t(st, dh, f, (const __bf16*)b.w1, d, nt, EPI_BF16, 0, dn, nullptr, 0, rv));
    BW_TRY(ln_bwd(st, ln_grid, d, dn, xmid, (const __bf16*)b.ln2_g, dy, dxm, dxmb, part, g + gl.ln2_g, (int)nt, c->ln_eps, false, rv));
    // attention: xmid = x + att W_O + b_O
    BW_TRY(gemm_wgrad(st, o, d, d, dxmb, d, d, nt, part, bpart, g + gl.wo, g + gl.bo, rv));
    BW_TRY(gemm_rows_t(st, dxmb, d, (const __bf16*)b.wo, d, nt, EPI_BF16, 0, dob, nullptr, 0, rv));
    if (L % s.K == 0 && 256 % s.heads == 0 && (256 / s.heads) % s.K == 0) {     // every group inside one workgroup's rows
      group_attn(3, s.dh, s.K, ah_grid, st, qkv, dob, dqkv, stat, q, d, s.heads);
    } else {
      group_attn(1, s.dh, s.K, ah_grid, st, qkv, dob, dqkv, stat, q, d, s.heads);
      group_attn(2, s.dh, s.K, ah_grid, st, qkv, dob, dqkv, stat, q, d, s.heads);
    }
    BW_TRY(launched("group attention backward"));
    const size_t wofs[3] = {gl.wq, gl.wk, gl.wv}, bofs[3] = {gl.bq, gl.bk, gl.bv};
    for (int j = 0; j < 3; ++j) {
      BW_TRY(gemm_wgrad(st, n1, d, d, dqkv + (size_t)j * d, 3 * d, d, nt, part, bpart, g + wofs[j], g + bofs[j], rv));
    }
    BW_TRY(gemm_rows_t(st, dqkv, 3 * d, wcat(l), d, nt, EPI_BF16, 0, dn, nullptr, 0, rv));
    // the gradient of this block's input is the upstream gradient of the block before it
    float* dx = l ? dy : dH;
    BW_TRY(ln_bwd(st, ln_grid, d, dn, xin(l), (const __bf16*)b.ln1_g, dxm, dx, l ? dyb : nullptr, part, g + gl.ln1_g,
                  (int)nt, c->ln_eps, false, rv));
  }
  return 0;
}


// ------------------------------------------------------------------------------------
// Whole model: loss and every gradient (longer_forward_backward)
struct StackDims { int d, f, heads, dh, m, k, n, T, B, layers; size_t rq, rk; };   // layers = 1 + n_self

struct StackWs {
  size_t fwd_ws, Mb, dM;                  // forward token merge: its scratch, M (bf16), and the gradient handed to the merge
  size_t qdesc, kdesc, wcat, bcat;
  size_t Rx, xs;                          // cross-layer key rows; the layers' input rows ([layers + 1][rq][d], [0] = O)
  size_t n1q, n1k, qkv, kv, o, xmid, n2, h, a, stat;    // every layer's intermediates are kept (per_layer bytes apart):
  size_t per_layer;                                     // the reduced stack is small, only the merge is recomputed
  size_t dy, dyb, dh, dnq, dnk, dxm, dxmb, dob, dqkv, dkv, dR, part, bpart;
  size_t total;
};
static StackWs stack_ws(const StackDims& s, size_t fwd_bytes) {
  StackWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
  const size_t rq = s.rq, rk = s.rk, d = s.d, f = s.f;
  w.fwd_ws = take(fwd_bytes);
  w.Mb = take((size_t)s.B * s.T * d * 2);
  w.dM = take((size_t)s.B * s.T * d * 4);
  w.qdesc = take(rq * 4);
  w.kdesc = take(rk * 4);
  w.wcat = take((size_t)s.layers * d * 3 * d * 2);
  w.bcat = take((size_t)s.layers * up256(3 * d * 2));
  w.Rx = take(rk * d * 4);
  w.xs = take((size_t)(s.layers + 1) * rq * d * 4);
  const size_t layer0 = o;
  w.n1q = take(rq * d * 2);
  w.n1k = take(rk * d * 2);
  w.qkv = take(rq * 3 * d * 2);
  w.kv = take(rk * 2 * d * 2);
  w.o = take(rq * d * 2);
  w.xmid = take(rq * d * 4);
  w.n2 = take(rq * d * 2);
  w.h = take(rq * f * 2);
  w.a = take(rq * f * 2);
  w.stat = take(rq * s.heads * 8);
  w.per_layer = o - layer0;
  o += (size_t)(s.layers - 1) * w.per_layer;
  w.dy = take(rq * d * 4);
  w.dyb = take(rq * d * 2);
  w.dh = take(rq * f * 2);
  w.dnq = take(rq * d * 2);
  w.dnk = take(rk * d * 2);
  w.dxm = take(rq * d * 4);
  w.dxmb = take(rq * d * 2);
  w.dob = take(rq * d * 2);
  w.dqkv = take(rq * 3 * d * 2);
  w.dkv = take(rk * 2 * d * 2);
  w.dR = take(rk * d * 4);
  w.part = take(kPartialBytes);
  w.bpart = take((size_t)kMaxPartials * 2048 * 4);
  w.total = o;
  return w;
}

static int check_stack(const longer_config* c, int B, int L, StackDims* s) {
  if (c->q_learn && (c->k_uniform || ((uintptr_t)c->q_learn & 15))) return api_error(LONGER_ERR_ARG, "q_learn needs k_uniform = 0 and 16-byte alignment");
  if (c->gmask != LONGER_GMASK_FULL && c->gmask != LONGER_GMASK_CAUSAL) return api_error(LONGER_ERR_ARG, "gmask %d unknown", c->gmask);
  const int d = c->d;
  if (d != 32 && d != 64 && d != 128 && d != 256) return api_error(LONGER_ERR_ARG, "width %d unsupported (32, 64, 128 or 256)", d);
  if (c->heads <= 0 || d % c->heads || (d / c->heads != 16 && d / c->heads != 32))
    return api_error(LONGER_ERR_ARG, "heads=%d: head width must be 16 or 32", c->heads);
  if (c->ffn_mult * d > 2048) return api_error(LONGER_ERR_ARG, "ffn_mult=%d: the FFN hidden width must be at most 2048", c->ffn_mult);
  if (c->m <= 0 || c->k_recent <= 0 || c->n_self < 0 || c->n_self > 30) return api_error(LONGER_ERR_ARG, "m, k_recent, n_self out of range");
  if (c->k_uniform < 0 || c->k_uniform > c->k_recent) return api_error(LONGER_ERR_ARG, "k_uniform=%d must lie in [0, k_recent]", c->k_uniform);
  s->d = d; s->f = c->ffn_mult * d; s->heads = c->heads; s->dh = d / c->heads; s->m = c->m; s->k = c->k_recent;
  s->n = c->m + c->k_recent; s->T = (L + c->K - 1) / c->K; s->B = B; s->layers = 1 + c->n_self;
  s->rq = (size_t)B * s->n; s->rk = (size_t)B * (c->m + s->T);
  if (s->rk * (size_t)s->heads * kSplit >= ((size_t)1 << 31) - 256) return api_error(LONGER_ERR_ARG, "too many key rows for one call; split the batch");
  return 0;
}

// layout of the gradient buffer: [InnerTrans blocks][cross block][self blocks][head_w (m d)][head_b (1), padded to 4]
// [learnable query tokens (k d), if the configuration has them]
struct ModelGrads { size_t inner, cross, self0, head_w, head_b, q_learn, total, per_main; };
static ModelGrads model_grads(const Dims& mi, const StackDims& s, bool learn) {
  ModelGrads g;
  g.inner = 0;
  g.cross = (size_t)mi.layers * grad_layout(mi.d, mi.f).total;
  g.per_main = grad_layout(s.d, s.f).total;
  g.self0 = g.cross + g.per_main;
  g.head_w = g.self0 + (size_t)(s.layers - 1) * g.per_main;
  g.head_b = g.head_w + (size_t)s.m * s.d;
  g.q_learn = (g.head_b + 1 + 3) & ~(size_t)3;
  g.total = g.q_learn + (learn ? (size_t)s.k * s.d : 0);
  return g;
}

// bytes of LDS the staged kernels need for n rows (two head vectors per row, its descriptor, and on the
// key side the query's two statistics)
static size_t set_attn_lds_bytes(int n, int dh, bool key_side) { return (size_t)n * (2 * dh * 2 + 4 + (key_side ? 8 : 0)); }
constexpr size_t kSetAttnLdsMax = 64 * 1024;     // what a workgroup may take without an opt-in

template <int DH>
static void set_attn_launch(hipStream_t st, int which, const SetAttn& a, const __bf16* dob, int d, __bf16* o_or_dq, int pitch,
                            __bf16* dk, __bf16* dv, float2* stat) {
  const unsigned gq = (unsigned)(((size_t)a.B * a.nq * a.heads * kSplit + 255) / 256);
  const unsigned gk = (unsigned)(((size_t)a.B * a.nk * a.heads * kSplit + 255) / 256);
  const size_t lq = set_attn_lds_bytes(a.nk, DH, false), lk = set_attn_lds_bytes(a.nq, DH, true);
  auto threads = [](int n) { int t = (n + 63) / 64 * 64; return t > 512 ? 512 : t; };
  const unsigned wgs = (unsigned)a.B * a.heads;
  // lanes per row: 1 / 2 / 4 / 8 measured at the headline batch (forward, query side, key side, four layers each):
  // 429 + 511 + 399, 324 + 367 + 336, 276 + 322 + 336, 274 + 324 + 380 us
  constexpr int kLanes = 4;
  if ((which == 2 ? lk : lq) <= kSetAttnLdsMax) {
    if (which == 0) bw_set_attn_fwd_lds_kernel<DH, kLanes><<<wgs, threads(a.nq * kLanes), lq, st>>>(a, o_or_dq, d, stat);
    else if (which == 1) bw_set_attn_bwd_q_lds_kernel<DH, kLanes><<<wgs, threads(a.nq * kLanes), lq, st>>>(a, dob, d, o_or_dq, pitch, stat);
    else bw_set_attn_bwd_kv_lds_kernel<DH, kLanes><<<wgs, threads(a.nk * kLanes), lk, st>>>(a, dob, d, dk, dv, pitch, stat);
  } else if (which == 0) bw_set_attn_fwd_kernel<DH><<<gq, 256, 0, st>>>(a, o_or_dq, d, stat);
  else if (which == 1) bw_set_attn_bwd_q_kernel<DH><<<gq, 256, 0, st>>>(a, dob, d, o_or_dq, pitch, stat);
  else bw_set_attn_bwd_kv_kernel<DH><<<gk, 256, 0, st>>>(a, dob, d, dk, dv, pitch, stat);
}

static int run_model(const longer_config* c, const longer_weights* wts, const void* H, const void* G, const int32_t* lens,
                     int B, int L, const float* labels, float* loss, float* logits, float* dH, float* dG, float* grads,
                     char* ws, size_t fwd_bytes, hipStream_t st, const Dims& mi, const StackDims& s) {
  const int d = s.d, f = s.f;
  const size_t rq = s.rq, rk = s.rk;
  const StackWs w = stack_ws(s, fwd_bytes);
  const ModelGrads mg = model_grads(mi, s, c->q_learn != nullptr);
  const GradLayout gl = grad_layout(d, f);
  const StackGeom geo = {lens, L, c->K, s.T, s.m, s.k, c->k_uniform, B, c->q_learn != nullptr};
  int* qdesc = (int*)(ws + w.qdesc);   int* kdesc = (int*)(ws + w.kdesc);
  __bf16* Mb = (__bf16*)(ws + w.Mb);   float* dM = (float*)(ws + w.dM);     float* Rx = (float*)(ws + w.Rx);
  auto xs = [&](int l) { return (float*)(ws + w.xs) + (size_t)l * rq * d; };
  auto wcat = [&](int l) { return (__bf16*)(ws + w.wcat) + (size_t)l * d * 3 * d; };
  auto bcat = [&](int l) { return (__bf16*)(ws + w.bcat + (size_t)l * up256((size_t)3 * d * 2)); };
  auto blk = [&](int l) -> const longer_block& { return l == 0 ? wts->cross[0] : wts->self[l - 1]; };
  __bf16 *n1q, *n1k, *qkv, *kv, *o, *n2, *h, *a;      // the current layer's intermediates
  float* xmid;
  float2* stat;
  auto use_layer = [&](int l) {
    char* base = ws + (size_t)l * w.per_layer;
    n1q = (__bf16*)(base + w.n1q); n1k = (__bf16*)(base + w.n1k); qkv = (__bf16*)(base + w.qkv); kv = (__bf16*)(base + w.kv);
    o = (__bf16*)(base + w.o); xmid = (float*)(base + w.xmid); n2 = (__bf16*)(base + w.n2); h = (__bf16*)(base + w.h);
    a = (__bf16*)(base + w.a); stat = (float2*)(base + w.stat);
  };
  float* dy = (float*)(ws + w.dy);     __bf16* dyb = (__bf16*)(ws + w.dyb); __bf16* dh = (__bf16*)(ws + w.dh);
  __bf16* dnq = (__bf16*)(ws + w.dnq); __bf16* dnk = (__bf16*)(ws + w.dnk); float* dxm = (float*)(ws + w.dxm);
  __bf16* dxmb = (__bf16*)(ws + w.dxmb); __bf16* dob = (__bf16*)(ws + w.dob); __bf16* dqkv = (__bf16*)(ws + w.dqkv);
  __bf16* dkv = (__bf16*)(ws + w.dkv); float* dR = (float*)(ws + w.dR);
  float* part = (float*)(ws + w.part); float* bpart = (float*)(ws + w.bpart);
  auto ln_grid = [&](size_t rows) { return (unsigned)((rows + 3) / 4 > 4096 ? 4096 : (rows + 3) / 4); };

  bw_zero_kernel<<<flat_grid(mg.total + 1), 256, 0, st>>>(grads, mg.total);
  bw_zero_kernel<<<1, 256, 0, st>>>(loss, 1);
  BW_TRY(launched("zero fill"));

  // ---- forward from the inputs: merged tokens (the fused forward kernel; the merge's intermediates are
  // recomputed later by its own backward pass), then the stack, keeping every layer's intermediates
  int rc = longer_token_merge(c, wts->inner, H, lens, B, L, Mb, ws + w.fwd_ws, fwd_bytes, st);
  if (rc) return rc;
  bw_desc_kernel<<<flat_grid(rq + rk), 256, 0, st>>>(geo, qdesc, kdesc);
  bw_build_rows_kernel<<<flat_grid((rq + rk) * d / 4), 256, 0, st>>>(geo, d, (const __bf16*)G, Mb, (const __bf16*)c->q_learn, qdesc, kdesc, xs(0), Rx);
  BW_TRY(launched("row build"));
  for (int l = 0; l < s.layers; ++l) {
    const longer_block& b = blk(l);
    bw_concat_qkv_kernel<<<64, 256, 0, st>>>((const __bf16*)b.wq, (const __bf16*)b.wk, (const __bf16*)b.wv, (const __bf16*)b.bq,
                                             (const __bf16*)b.bk, (const __bf16*)b.bv, wcat(l), bcat(l), d);
    BW_TRY(launched("weight concatenation"));
  }

  auto attn = [&](int l) {
    SetAttn t;
    t.qdesc = qdesc; t.nq = s.n; t.B = B; t.heads = s.heads; t.gmask = c->gmask; t.m = s.m; t.self = l != 0;
    if (l == 0) { t.q = qkv; t.qpitch = d; t.k = kv; t.v = kv + d; t.kvpitch = 2 * d; t.kdesc = kdesc; t.nk = s.m + s.T; }
    else { t.q = qkv; t.qpitch = 3 * d; t.k = qkv + d; t.v = qkv + 2 * d; t.kvpitch = 3 * d; t.kdesc = qdesc; t.nk = s.n; }
    return t;
  };
  // layer l forward from its input rows xs(l) (layer 0: and the key rows Rx), intermediates into the
  // layer's own buffers; output into y_out (masked to the valid rows)
  auto forward = [&](int l, float* y_out) -> int {
    const longer_block& b = blk(l);
    const float* x = xs(l);
    use_layer(l);
    ln_fwd(st, ln_grid(rq), d, x, (const __bf16*)b.ln1_g, (const __bf16*)b.ln1_b, n1q, (int)rq, c->ln_eps);
    if (l == 0) {
      ln_fwd(st, ln_grid(rk), d, Rx, (const __bf16*)b.ln1_g, (const __bf16*)b.ln1_b, n1k, (int)rk, c->ln_eps);
      BW_TRY(launched("LayerNorm"));
      BW_TRY(gemm_rows(st, n1q, d, wcat(l), d, rq, EPI_BF16, 0, qkv, nullptr, bcat(l), nullptr, nullptr, 3 * d));
      BW_TRY(gemm_rows(st, n1k, d, wcat(l) + d, 2 * d, rk, EPI_BF16, 0, kv, nullptr, bcat(l) + d, nullptr, nullptr, 3 * d));
    } else {
      BW_TRY(launched("LayerNorm"));
      BW_TRY(gemm_rows(st, n1q, d, wcat(l), 3 * d, rq, EPI_BF16, 0, qkv, nullptr, bcat(l), nullptr, nullptr));
    }
    const SetAttn t = attn(l);
    if (s.dh == 16) set_attn_launch<16>(st, 0, t, nullptr, d, o, 0, nullptr, nullptr, stat);
    else set_attn_launch<32>(st, 0, t, nullptr, d, o, 0, nullptr, nullptr, stat);
    BW_TRY(launched("attention"));
    BW_TRY(gemm_rows(st, o, d, (const __bf16*)b.wo, d, rq, EPI_RES_F32, 0, xmid, nullptr, (const __bf16*)b.bo, x, nullptr));
    ln_fwd(st, ln_grid(rq), d, xmid, (const __bf16*)b.ln2_g, (const __bf16*)b.ln2_b, n2, (int)rq, c->ln_eps);
    BW_TRY(launched("LayerNorm"));
    BW_TRY(gemm_rows(st, n2, d, (const __bf16*)b.w1, f, rq, EPI_ACT, c->act, h, a, (const __bf16*)b.b1, nullptr, nullptr));
    if (y_out) {
      BW_TRY(gemm_rows(st, a, f, (const __bf16*)b.w2, d, rq, EPI_RES_F32, 0, y_out, nullptr, (const __bf16*)b.b2, xmid, nullptr));
      bw_mask_rows_kernel<<<flat_grid(rq * d / 4), 256, 0, st>>>(y_out, nullptr, qdesc, rq, d);
      BW_TRY(launched("row mask"));
    }
    return 0;
  };
  for (int l = 0; l < s.layers; ++l) BW_TRY(forward(l, xs(l + 1)));

  // ---- head and loss (Eq. 1-2), and the gradient of the stack's output
  bw_head_kernel<<<B, 256, 0, st>>>(xs(s.layers), (const __bf16*)wts->head_w, (const __bf16*)wts->head_b, labels, B, s.n, s.m, d,
                                    logits, loss, dy, dyb, grads + mg.head_w, grads + mg.head_b);
  BW_TRY(launched("head"));

  // ---- back through the layers
  for (int l = s.layers - 1; l >= 0; --l) {
    const longer_block& b = blk(l);
    float* g = grads + (l == 0 ? mg.cross : mg.self0 + (size_t)(l - 1) * mg.per_main);
    // rows that were written as zeros pass no gradient
    bw_mask_rows_kernel<<<flat_grid(rq * d / 4), 256, 0, st>>>(dy, dyb, qdesc, rq, d);
    BW_TRY(launched("row mask"));
    use_layer(l);                                  // kept by the forward pass above
    BW_TRY(gemm_wgrad(st, a, f, f, dyb, d, d, rq, part, bpart, g + gl.w2, g + gl.b2));
    BW_TRY(gemm_rows_t(st, dyb, d, (const __bf16*)b.w2, f, rq, EPI_DACT, c->act, dh, h));
    BW_TRY(gemm_wgrad(st, n2, d, d, dh, f, f, rq, part, bpart, g + gl.w1, g + gl.b1));
    BW_TRY(gemm_rows_t(st, dh, f, (const __bf16*)b.w1, d, rq, EPI_BF16, 0, dnq, nullptr));
    BW_TRY(ln_bwd(st, ln_grid(rq), d, dnq, xmid, (const __bf16*)b.ln2_g, dy, dxm, dxmb, part, g + gl.ln2_g, (int)rq, c->ln_eps));
    BW_TRY(gemm_wgrad(st, o, d, d, dxmb, d, d, rq, part, bpart, g + gl.wo, g + gl.bo));
    BW_TRY(gemm_rows_t(st, dxmb, d, (const __bf16*)b.wo, d, rq, EPI_BF16, 0, dob, nullptr));
    const SetAttn t = attn(l);
    if (l == 0) {
      if (s.dh == 16) {
        set_attn_launch<16>(st, 1, t, dob, d, dqkv, d, nullptr, nullptr, stat);
        set_attn_launch<16>(st, 2, t, dob, d, nullptr, 2 * d, dkv, dkv + d, stat);
      } else {
        set_attn_launch<32>(st, 1, t, dob, d, dqkv, d, nullptr, nullptr, stat);
        set_attn_launch<32>(st, 2, t, dob, d, nullptr, 2 * d, dkv, dkv + d, stat);
      }
      BW_TRY(launched("attention backward"));
      BW_TRY(gemm_wgrad(st, n1q, d, d, dqkv, d, d, rq, part, bpart, g + gl.wq, g + gl.bq));
      BW_TRY(gemm_wgrad(st, n1k, d, d, dkv, 2 * d, d, rk, part, bpart, g + gl.wk, g + gl.bk));
      BW_TRY(gemm_wgrad(st, n1k, d, d, dkv + d, 2 * d, d, rk, part, bpart, g + gl.wv, g + gl.bv));
      BW_TRY(gemm_rows_t(st, dqkv, d, wcat(l), d, rq, EPI_BF16, 0, dnq, nullptr, 3 * d));
      BW_TRY(gemm_rows_t(st, dkv, 2 * d, wcat(l) + d, d, rk, EPI_BF16, 0, dnk, nullptr, 3 * d));
      // LN1 normalises the query rows and the key rows: its gain / shift gradient is the sum of both;
      // dO goes to dy (the query rows' gradient), dR to its own buffer
      BW_TRY(ln_bwd(st, ln_grid(rq), d, dnq, xs(0), (const __bf16*)b.ln1_g, dxm, dy, nullptr, part, g + gl.ln1_g, (int)rq, c->ln_eps, true));
      BW_TRY(ln_bwd(st, ln_grid(rk), d, dnk, Rx, (const __bf16*)b.ln1_g, nullptr, dR, nullptr, part, g + gl.ln1_g, (int)rk, c->ln_eps, true));
    } else {
      if (s.dh == 16) {
        set_attn_launch<16>(st, 1, t, dob, d, dqkv, 3 * d, nullptr, nullptr, stat);
        set_attn_launch<16>(st, 2, t, dob, d, nullptr, 3 * d, dqkv + d, dqkv + 2 * d, stat);
      } else {
        set_attn_launch<32>(st, 1, t, dob, d, dqkv, 3 * d, nullptr, nullptr, stat);
        set_attn_launch<32>(st, 2, t, dob, d, nullptr, 3 * d, dqkv + d, dqkv + 2 * d, stat);
      }
      BW_TRY(launched("attention backward"));
      const size_t wofs[3] = {gl.wq, gl.wk, gl.wv}, bofs[3] = {gl.bq, gl.bk, gl.bv};
      for (int j = 0; j < 3; ++j)
        BW_TRY(gemm_wgrad(st, n1q, d, d, dqkv + (size_t)j * d, 3 * d, d, rq, part, bpart, g + wofs[j], g + bofs[j]));
      BW_TRY(gemm_rows_t(st, dqkv, 3 * d, wcat(l), d, rq, EPI_BF16, 0, dnq, nullptr));
      BW_TRY(ln_bwd(st, ln_grid(rq), d, dnq, xs(l), (const __bf16*)b.ln1_g, dxm, dy, dyb, part, g + gl.ln1_g, (int)rq, c->ln_eps));
    }
  }
  // ---- gradients of the stack's inputs: global tokens (query rows and key rows), merged tokens (key
  // rows, plus the query slots that hold them)
  bw_split_grad_kernel<<<flat_grid(rk * d / 4), 256, 0, st>>>(geo, d, dy, dR, dG, dM);
  bw_slot_grad_kernel<<<flat_grid((size_t)B * s.k * d / 4), 256, 0, st>>>(geo, d, dy, qdesc, dM, grads + mg.q_learn);
  BW_TRY(launched("gradient routing"));
  return 0;
}


// ------------------------------------------------------------------------------------
// Input generation backward (longer_input_generation_backward)
struct InputWs { size_t w1t, x, a, dyb, dh, dx, part, bpart, total; };
static InputWs input_ws(size_t ntok, int d, int f) {
  InputWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
  w.w1t = take((size_t)d * f * 2);
  w.x = take(ntok * d * 2);
  w.a = take(ntok * f * 2);
  w.dyb = take(ntok * d * 2);
  w.dh = take(ntok * f * 2);
  w.dx = take(ntok * d * 4);
  w.part = take(kPartialBytes);
  w.bpart = take((size_t)kMaxPartials * 2048 * 4);
  w.total = o;
  return w;
}
// gradient buffer: [pos L de][w1 d f][b1 f][w2 f d][b2 d]
struct InputGrads { size_t pos, w1, b1, w2, b2, total; };
static InputGrads input_grads(int L, int d, int f, int de) {
  InputGrads g;
  g.pos = 0; g.w1 = (size_t)L * de; g.b1 = g.w1 + (size_t)d * f; g.w2 = g.b1 + f; g.b2 = g.w2 + (size_t)f * d;
  g.total = g.b2 + d;
  return g;
}
static int check_input_bw(const longer_config* c, int B, int L, int de, int* d, int* f) {
  if (!c) return api_error(LONGER_ERR_ARG, "config is NULL");
  if (c->dtype != LONGER_BF16) return api_error(LONGER_ERR_ARG, "the backward pass is mixed precision: dtype must be LONGER_BF16");
  if (c->merge != LONGER_MERGE_MEAN) return api_error(LONGER_ERR_ARG, "input generation feeds the mean merge (H of width d)");
  if (c->act != LONGER_ACT_GELU_ERF && c->act != LONGER_ACT_RELU) return api_error(LONGER_ERR_ARG, "act %d unknown", c->act);
  if (c->d <= 0 || c->d % 32 || c->d > 512) return api_error(LONGER_ERR_ARG, "d=%d must be a multiple of 32, at most 512", c->d);
  if (c->ffn_mult <= 0 || c->ffn_mult * c->d > 2048) return api_error(LONGER_ERR_ARG, "ffn_mult=%d: the hidden width must be at most 2048", c->ffn_mult);
  if (de <= 0 || de >= c->d || de % 32) return api_error(LONGER_ERR_ARG, "d_e=%d must be a multiple of 32 below d=%d", de, c->d);
  if (B <= 0 || L <= 0 || (long long)B * L >= (1ll << 31) / 8) return api_error(LONGER_ERR_ARG, "B=%d, L=%d out of range", B, L);
  *d = c->d; *f = c->ffn_mult * c->d;
  return 0;
}

}  // namespace bw
}  // namespace longer

using namespace longer;

extern "C" {

size_t longer_backward_workspace_bytes(const longer_config* cfg, int B, int L) {
  bw::Dims s;
  if (bw::check(cfg, B, L, &s)) return 0;
  return bw::merge_workspace(cfg, s, B, L).total;
}

size_t longer_block_grad_floats(const longer_config* cfg) {
  bw::Dims s;
  if (bw::check(cfg, 1, 1, &s)) return 0;
  return bw::grad_layout(s.d, s.f).total;
}

int longer_token_merge_backward(const longer_config* cfg, const longer_block* inner, const void* H,
                                const int32_t* lens, int B, int L, const float* dM,
                                float* dH_out, float* grads_out,
                                void* ws, size_t ws_bytes, void* stream) {
  bw::Dims s;
  int rc = bw::check(cfg, B, L, &s);
  if (rc) return rc;
  if (!inner || !H || !dM || !dH_out || !grads_out || !ws) return api_error(LONGER_ERR_ARG, "null pointer argument");
  if (!bw::aligned16(H) || !bw::aligned16(dM) || !bw::aligned16(dH_out) || !bw::aligned16(grads_out) || ((uintptr_t)ws & 255))
    return api_error(LONGER_ERR_ARG, "H, dM, dH_out, grads_out must be 16-byte aligned and ws 256-byte aligned");
  for (int l = 0; l < s.layers; ++l) {
    const void* const* p = (const void* const*)&inner[l];
    for (int i = 0; i < 16; ++i)
      if (!p[i] || !bw::aligned16(p[i])) return api_error(LONGER_ERR_ARG, "InnerTrans block %d: parameter %d is NULL or not 16-byte aligned", l, i);
  }
  const size_t need = bw::merge_workspace(cfg, s, B, L).total;
  if (ws_bytes < need) return api_error(LONGER_ERR_WS, "workspace too small: %zu < %zu bytes", ws_bytes, need);
  return bw::run(cfg, inner, H, lens, B, L, dM, dH_out, grads_out, (char*)ws, (hipStream_t)stream, s);
}

size_t longer_model_grad_floats(const longer_config* cfg) {
  bw::Dims mi;
  bw::StackDims s;
  if (bw::check(cfg, 1, 1, &mi) || bw::check_stack(cfg, 1, 1, &s)) return 0;
  return bw::model_grads(mi, s, cfg->q_learn != nullptr).total;
}

size_t longer_forward_backward_workspace_bytes(const longer_config* cfg, int B, int L) {
  bw::Dims mi;
  bw::StackDims s;
  if (bw::check(cfg, B, L, &mi) || bw::check_stack(cfg, B, L, &s)) return 0;
  const size_t fwd = longer_workspace_bytes(cfg, B, L);
  if (fwd == 0) return 0;
  return bw::stack_ws(s, fwd).total + bw::merge_workspace(cfg, mi, B, L).total;
}

int longer_forward_backward(const longer_config* cfg, const longer_weights* w, const void* H, const void* G,
                            const int32_t* lens, int B, int L, const float* labels,
                            float* loss_out, float* logits_out, float* dH_out, float* dG_out, float* grads_out,
                            void* ws, size_t ws_bytes, void* stream) {
  bw::Dims mi;
  bw::StackDims s;
  int rc = bw::check(cfg, B, L, &mi);
  if (rc) return rc;
  rc = bw::check_stack(cfg, B, L, &s);
  if (rc) return rc;
  if (!w || !w->inner || !w->cross || (cfg->n_self && !w->self) || !w->head_w || !w->head_b || !H || !G || !labels || !loss_out ||
      !dH_out || !dG_out || !grads_out || !ws)
    return api_error(LONGER_ERR_ARG, "null pointer argument");
  const void* ptrs[] = {H, G, labels, loss_out, dH_out, dG_out, grads_out, w->head_w};
  for (const void* p : ptrs)
    if (!bw::aligned16(p)) return api_error(LONGER_ERR_ARG, "H, G, labels, loss_out, dH_out, dG_out, grads_out, head_w must be 16-byte aligned");
  if ((uintptr_t)ws & 255) return api_error(LONGER_ERR_ARG, "ws must be 256-byte aligned");
  for (int l = 0; l < mi.layers + s.layers; ++l) {
    const longer_block* b = l < mi.layers ? &w->inner[l] : (l == mi.layers ? &w->cross[0] : &w->self[l - mi.layers - 1]);
    const void* const* p = (const void* const*)b;
    for (int i = 0; i < 16; ++i)
      if (!p[i] || !bw::aligned16(p[i])) return api_error(LONGER_ERR_ARG, "block %d: parameter %d is NULL or not 16-byte aligned", l, i);
  }
  const size_t fwd = longer_workspace_bytes(cfg, B, L);
  if (fwd == 0) return LONGER_ERR_ARG;
  const size_t stack_bytes = bw::stack_ws(s, fwd).total;
  const size_t need = stack_bytes + bw::merge_workspace(cfg, mi, B, L).total;
  if (ws_bytes < need) return api_error(LONGER_ERR_WS, "workspace too small: %zu < %zu bytes", ws_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  rc = bw::run_model(cfg, w, H, G, lens, B, L, labels, loss_out, logits_out, dH_out, dG_out, grads_out, (char*)ws, fwd, st, mi, s);
  if (rc) return rc;
  // the merge's gradients: dM was left in the stack's workspace; the InnerTrans blocks come first in grads_out
  const float* dM = (const float*)((char*)ws + bw::stack_ws(s, fwd).dM);
  return bw::run(cfg, w->inner, H, lens, B, L, dM, dH_out, grads_out, (char*)ws + stack_bytes, st, mi);
}

size_t longer_input_backward_workspace_bytes(const longer_config* cfg, int B, int L, int d_e) {
  int d, f;
  if (bw::check_input_bw(cfg, B, L, d_e, &d, &f)) return 0;
  return bw::input_ws((size_t)B * L, d, f).total;
}

size_t longer_input_grad_floats(const longer_config* cfg, int L, int d_e) {
  int d, f;
  if (bw::check_input_bw(cfg, 1, L, d_e, &d, &f)) return 0;
  return bw::input_grads(L, d, f, d_e).total;
}

int longer_input_generation_backward(const longer_config* cfg, const longer_input_weights* w, const void* E,
                                     const void* tdiff, const int32_t* lens, int B, int L, int d_e, const float* dH,
                                     float* dE_out, float* dtdiff_out, float* grads_out,
                                     void* ws, size_t ws_bytes, void* stream) {
  int d, f;
  int rc = bw::check_input_bw(cfg, B, L, d_e, &d, &f);
  if (rc) return rc;
  if (!w || !w->pos || !w->w1 || !w->b1 || !w->w2 || !w->b2 || !E || !tdiff || !dH || !dE_out || !dtdiff_out || !grads_out || !ws)
    return api_error(LONGER_ERR_ARG, "null pointer argument");
  const void* ptrs[] = {w->pos, w->w1, w->b1, w->w2, w->b2, E, tdiff, dH, dE_out, dtdiff_out, grads_out};
  for (const void* p : ptrs)
    if (!bw::aligned16(p)) return api_error(LONGER_ERR_ARG, "every pointer must be 16-byte aligned");
  if ((uintptr_t)ws & 255) return api_error(LONGER_ERR_ARG, "ws must be 256-byte aligned");
  const size_t nt = (size_t)B * L;
  const bw::InputWs l = bw::input_ws(nt, d, f);
  if (ws_bytes < l.total) return api_error(LONGER_ERR_WS, "workspace too small: %zu < %zu bytes", ws_bytes, l.total);
  const bw::InputGrads gl = bw::input_grads(L, d, f, d_e);
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  __bf16* x = (__bf16*)(w8 + l.x);   __bf16* w1t = (__bf16*)(w8 + l.w1t); __bf16* a = (__bf16*)(w8 + l.a);
  __bf16* dyb = (__bf16*)(w8 + l.dyb); __bf16* dh = (__bf16*)(w8 + l.dh); float* dx = (float*)(w8 + l.dx);
  float* part = (float*)(w8 + l.part); float* bpart = (float*)(w8 + l.bpart);
  const bw::RowGeom q = {lens, L, 1, (int)nt};
  const bw::RowsValid rv = {lens, L};
  const unsigned eg = bw::flat_grid(nt * d / 4);
  bw::bw_zero_kernel<<<bw::flat_grid(gl.total), 256, 0, st>>>(grads_out, gl.total);
  bw::bw_input_rows_kernel<<<eg, 256, 0, st>>>((const __bf16*)E, (const __bf16*)w->pos, (const __bf16*)tdiff, x, q, d, d_e);
  bw::bw_cast_rows_kernel<<<eg, 256, 0, st>>>(dH, dyb, q, d);
  if ((rc = bw::launched("input rows"))) return rc;
  // the hidden pre-activation is formed again inside the launch that takes its gradient (as in the merge's FFN)
  if ((rc = bw::transpose(st, (const __bf16*)w->w1, w1t, d, f))) return rc;
  if ((rc = bw::gemm_ffn_mid(st, x, dyb, d, w1t, (const __bf16*)w->w2, f, (const __bf16*)w->b1, nt, cfg->act, dh, a, rv))) return rc;
  // H = a w2 + b2
  if ((rc = bw::gemm_wgrad(st, a, f, f, dyb, d, d, nt, part, bpart, grads_out + gl.w2, grads_out + gl.b2, rv))) return rc;
  if ((rc = bw::gemm_wgrad(st, x, d, d, dh, f, f, nt, part, bpart, grads_out + gl.w1, grads_out + gl.b1, rv))) return rc;
  if ((rc = bw::gemm_rows_t(st, dh, f, (const __bf16*)w->w1, d, nt, bw::EPI_F32, 0, dx, nullptr, 0, rv))) return rc;
  bw::bw_split_input_grad_kernel<<<eg, 256, 0, st>>>(dx, dE_out, dtdiff_out, q, d, d_e);
  bw::bw_pos_grad_kernel<<<bw::flat_grid((size_t)L * d_e / 4), 256, 0, st>>>(dx, grads_out + gl.pos, q, B, d, d_e);
  return bw::launched("input gradient");
}

}  // extern "C"
