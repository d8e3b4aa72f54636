// The transformer-block kernel of the LONGER hot path and its modes:
//
//   MODE_MERGE   token merge (Section 3.4): gather K-groups of raw tokens, run the
//                InnerTrans blocks on them with attention inside each group, mean-pool
//                each group to one token (or write the un-pooled rows);
//   MODE_KVPROJ  key/value side of an attention layer (Eq. 6): K, V = LN1(rows) W + b,
//                stored as ready-made MFMA operand fragments;
//   MODE_ATTN    query side of the cross-causal layer (Eq. 5-8) or of a self-causal
//                layer (Eq. 9): Q projection, masked online-softmax attention over the
//                stored K/V fragments, output projection, FFN;
//   MODE_STACK   the whole reduced stack of one user in one workgroup (Eq. 10): the query side
//                of the cross-causal layer as in MODE_ATTN, then every self-causal layer
//                with its K/V projected in place and handed between the workgroup's waves
//                through LDS - no launch and no global round trip between the layers
//                (needs m + k <= 128 rows);
//   MODE_SCORE   candidate scoring of the KV-cache serving path (Section 3.6.3): the m
//                global tokens of each candidate through all 1 + N layers, attending to
//                their own globals (inside the tile) and the cached sequence K/V;
//   MODE_INPUT   input generation (Section 3.5.1): the FFN stage alone, as a two-layer MLP
//                over rows built from item embedding + positional embedding and the
//                time-difference features;
//   MODE_MERGE_IN  MODE_INPUT and MODE_MERGE in one pass: the MLP's result stays in the
//                registers as the rows the InnerTrans blocks start from.
//
// Every mode runs the same register-resident chain (see device.h); they differ in where
// rows come from, which attention sources exist and what is written.
#pragma once
#include "device.h"
#include <type_traits>

namespace longer {

struct RowSrc {
  const void* p;        // base of rows (element type T, or fp32 when f32 != 0)
  long long ustride;    // elements between consecutive users
  int f32;
};

struct BlockParams {
  // packed parameters: the linear segment stream this launch consumes (all its layers)
  const char* wbase;
  int n_layers, FF;
  float eps, scale_l2e;
  int act, gmask_causal;
  const int32_t* lens;
  int B, L, K, T, m, k;
  // MODE_MERGE
  const void* H;
  void* M_out; int M_f32;
  void* Z_out; int Z_f32;
  // MODE_KVPROJ / MODE_ATTN rows: rows [0, m0) of a user come from src0, the rest from src1
  RowSrc src0, src1;
  int m0;
  int rows_per_user, tiles_per_user;
  int gather_recent;    // src1 row of slot i is its sampled merged token (cross layer) instead of i
  int k_uni;            // the first k_uni of the k slots hold uniformly sampled older tokens
  int q_learn;          // the k slots hold learnable query tokens (rows of src1, the same for every user)
  int q0;               // MODE_ATTN: first query row (0: globals + slots, m: slots only)
  // stored K/V fragments: per user kt_per_user key tiles of NT*GPT fragments each
  char* kst; char* vst;
  size_t kv_ustride;
  int kt_per_user;
  int KG;               // number of global keys in front of the sequence keys
  int key_self;         // 1: sequence keys are the k recent slots, 0: all T merged tokens
  // MODE_ATTN / MODE_SCORE outputs
  void* X_out; int X_f32; long long X_ustride;
  float* logits; const float* head;   // head: fp32 [m*D] weights then the bias
  // MODE_INPUT / MODE_MERGE_IN: item embeddings [B, L, de], positional embedding [L, de],
  // time-difference features [B, L, D - de] (element type T); MODE_INPUT writes the result to
  // X_out [B, L, D]
  const void* in_e; const void* in_pos; const void* in_td; int de;
  // MODE_SCORE
  int xcds, wg_per_user;   // workgroup index -> (user, group of tiles), see the kernel
  const void* Gc; int C;
  const char* cache;    // layer 0 K then V, then layers 1..N
  size_t c0_ustride, c0_voff, c1_off, c1_lstride, c1_ustride, c1_voff;
  int kt0, kt1;
};

// ---------------------------------------------------------------------------- helpers
template <typename T, int NT>
__device__ __forceinline__ void load_rows(f32x16 (&x)[NT], const void* base, int is_f32, long long off,
                                          bool valid, int hi) {
#pragma unroll
  for (int t = 0; t < NT; ++t) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        long long o = off + 32 * t + 8 * q + 4 * hi;
        if (is_f32 || sizeof(T) == 4) {
          v = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(base) + o);
        } else {
          bf16x4 b = *reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(base) + o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (float)b[e];
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) x[t][4 * q + e] = v[e];
    }
  }
}

template <typename T, int NT>
__device__ __forceinline__ void store_rows(const f32x16 (&x)[NT], void* base, int is_f32, long long off,
                                           bool nonzero, int hi) {
#pragma unroll
  for (int t = 0; t < NT; ++t) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = nonzero ? x[t][4 * q + e] : 0.f;
      long long o = off + 32 * t + 8 * q + 4 * hi;
      if (is_f32 || sizeof(T) == 4) {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(base) + o) = v;
      } else {
        bf16x4 b;
#pragma unroll
        for (int e = 0; e < 4; ++e) b[e] = (__bf16)v[e];
        *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(base) + o) = b;
      }
    }
  }
}

// accumulator tile initialised with a per-feature bias (transposed layout)
__device__ __forceinline__ f32x16 bias_tile(const float* b, int tile, int hi) {
  f32x16 a;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    f32x4 v = *reinterpret_cast<const f32x4*>(b + 32 * tile + 8 * q + 4 * hi);
#pragma unroll
    for (int e = 0; e < 4; ++e) a[4 * q + e] = v[e];
  }
  return a;
}

__device__ __forceinline__ f32x16 splat16(float v) {
  f32x16 a;
#pragma unroll
  for (int r = 0; r < 16; ++r) a[r] = v;
  return a;
}

// x += x of the lane that the DPP control CTRL pairs this lane with (within rows of 16 lanes)
template <int CTRL, int NT>
__device__ __forceinline__ void lane_sum(f32x16 (&x)[NT]) {
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float v = x[t][r];   // (a bit cast straight from the vector element reads element 0)
      const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true);
      x[t][r] = v + __builtin_bit_cast(float, o);
    }
}

// bits b in [0,32) set iff base + b lies in [lo, hi)
__device__ __forceinline__ uint32_t range_bits(int lo, int hi, int base) {
  int a = max(lo - base, 0), b = min(hi - base, 32);
  if (b <= a) return 0u;
  uint32_t upper = b >= 32 ? 0xffffffffu : ((1u << b) - 1u);
  return upper & ~((1u << a) - 1u);
}

// GELU.  EXACT (fp32 mode): the erf form.  Otherwise (bf16 mode, where the result is rounded
// to bf16 right away): GELU(x) = x * Phi(x) with Phi - 1/2 replaced by an odd polynomial of
// degree 9 (minimax fit on [-3.5, 3.5], constrained to reach 1 at the interval end; it keeps
// growing beyond it) and Phi clamped to [0, 1] by the output modifier of the last fma;
// max abs error 1.3e-3, below the bf16 rounding step of the values it produces.
// The same polynomial in packed fp16, two elements per instruction, on y = x / kFfnScale;
// returns GELU(x) / kFfnScale.  Phi(4 y) - 1/2 = y (k0 + k1 v + ... + k4 v^4), v = y^2, with
// k_i = 4 * 16^i * c_i of the fp32 coefficients below (all of order 1).  A square that
// overflows gives an infinite polynomial of the right sign, which the clamp turns into 0 or 1.
// A whole operand group (8 elements, 4 register pairs) goes through each step together, so that
// an instruction never uses the result of the one right before it (which costs a wait state).
__device__ __forceinline__ f16x8 gelu_quarter_h8(f16x8 y) {
  const f16x8 v = y * y;
  f16x8 pl = (f16x8)((_Float16)2.4554419175668456f);
  pl = __builtin_elementwise_fma(pl, v, (f16x8)((_Float16)-6.304095499217479f));
  pl = __builtin_elementwise_fma(pl, v, (f16x8)((_Float16)6.604333663059149f));
  pl = __builtin_elementwise_fma(pl, v, (f16x8)((_Float16)-3.771901897714043f));
  pl = __builtin_elementwise_fma(pl, v, (f16x8)((_Float16)1.5736394077430096f));
  f16x8 phi = __builtin_elementwise_fma(y, pl, (f16x8)((_Float16)0.5f));
  phi = __builtin_elementwise_min(__builtin_elementwise_max(phi, (f16x8)((_Float16)0.f)), (f16x8)((_Float16)1.f));
  return y * phi;
}

template <bool EXACT>
__device__ __forceinline__ float gelu_fn(float x) {
  if (EXACT) return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
  const float u = x * x;
  float pl = 9.366767568843253e-06f;
  pl = fmaf(pl, u, -0.0003847714538096606f);
  pl = fmaf(pl, u, 0.0064495445928312006f);
  pl = fmaf(pl, u, -0.05893596715178192f);
  pl = fmaf(pl, u, 0.3934098519357524f);
  // (the compiler folds the median with 0 and 1 into the FMA's clamp modifier)
  const float phi = __builtin_amdgcn_fmed3f(fmaf(x, pl, 0.5f), 0.f, 1.f);
  return x * phi;
}

// First valid one of a user's k query slots: sampled tokens are right-aligned; learnable query
// tokens (Section 3.5.1) are all valid as soon as the user has a token to attend to.
__device__ __forceinline__ int first_slot(int k, int tu, int q_learn) {
  return q_learn ? (tu > 0 ? 0 : k) : max(k - tu, 0);
}

// Merged token held by slot i of the k sampled sequence queries of a user with tu merged tokens
// (Section 3.5.1): the last k - k_uni slots hold the most recent tokens, the first k_uni slots the
// newest token of each of k_uni equal shares of the older ones; a user with no more than k tokens
// gets all of them, right-aligned (negative = invalid slot).
__device__ __forceinline__ int slot_token(int i, int k, int tu, int k_uni) {
  if (tu <= k || i >= k_uni) return tu - k + i;
  const long long rest = tu - (k - k_uni);
  return (int)(((long long)(i + 1) * rest) / k_uni) - 1;
}

// Scheduling hint for a stretch of N MFMAs that each consume one weight fragment read from LDS
// (plus EXTRA other LDS reads ahead of them, e.g. a bias tile): the first AHEAD fragment reads go
// out together, then one read per MFMA, so that an MFMA never waits out the LDS latency of its
// own fragment.  Used by the kernels that run one wave per SIMD, where no other wave hides it.
template <int N, int EXTRA>
__device__ __forceinline__ void frag_pipeline_hint() {
  constexpr int AHEAD = N < 6 ? N : 6;
  __builtin_amdgcn_sched_group_barrier(0x100, EXTRA + AHEAD, 0);
#pragma unroll
  for (int i = 0; i < N - AHEAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
}

// LayerNorm over the feature dimension of TT token tiles, result as B-operand groups.
// fp32 mode takes the variance in a second pass over the centred values; bf16 mode uses
// E[x^2] - mean^2 in one pass (the result is rounded to bf16 anyway).
template <typename T, int D, int TT>
__device__ __forceinline__ void layer_norm(const f32x16 (&x)[TT][D / 32], const float* gam, const float* bet,
                                           float eps, int hi, typename ET<T>::grp (&out)[TT][D / ET<T>::GF]) {
  using E = ET<T>;
  constexpr int NT = D / 32;
  constexpr bool EXACT = sizeof(T) == 4;
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    float s = 0.f, q = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) { s += x[tt][t][r]; if (!EXACT) q = fmaf(x[tt][t][r], x[tt][t][r], q); }
    s = sum_halves(s);
    const float mean = s * (1.0f / D);
    float var;
    if (EXACT) {
      float v = 0.f;
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) { float dlt = x[tt][t][r] - mean; v += dlt * dlt; }
      v = sum_halves(v);
      var = v * (1.0f / D);
    } else {
      q = sum_halves(q);
      var = fmaxf(q * (1.0f / D) - mean * mean, 0.f);
    }
    // (bf16 mode: the hardware reciprocal square root, 1 ulp, instead of the exact division)
    const float rstd = EXACT ? 1.0f / sqrtf(var + eps) : __builtin_amdgcn_rsqf(var + eps);
    const float shift = -mean * rstd;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x16 g = bias_tile(gam, t, hi), b = bias_tile(bet, t, hi), y;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float nrm = EXACT ? (x[tt][t][r] - mean) * rstd : fmaf(x[tt][t][r], rstd, shift);
        y[r] = fmaf(nrm, g[r], b[r]);
      }
#pragma unroll
      for (int gg = 0; gg < E::GPT; ++gg) out[tt][t * E::GPT + gg] = E::pack(y, gg);
    }
  }
}

// bits of a tile's visibility word that correspond to accumulator registers
constexpr uint32_t kTileBits = 0x0F0F0F0Fu;

// Visibility of a 32-key tile as an additive score tile: 0 for a visible key, -infinity for a
// hidden one (bit 8 (r/4) + r%4 of `ab` belongs to accumulator register r).  The score MFMA
// starts from it, so masking costs nothing per head.
__device__ __forceinline__ f32x16 mask_tile(uint32_t ab) {
  f32x16 b;
#pragma unroll
  for (int r = 0; r < 16; ++r) b[r] = ((ab >> (8 * (r / 4) + (r % 4))) & 1u) ? 0.f : -__builtin_inff();
  return b;
}

// One online-softmax step over a 32-key tile.  S holds, for this lane's query, the scores of
// keys tile_row(r, hi), already in units of log2(e) / sqrt(head width) (the factor rides on
// Q); with MASKED, `ab` has bit (8 (r/4) + r%4) set iff that key is visible, and a hidden
// key gets the score -infinity (below the running maximum's start value, so its probability
// is an exact zero without a second test).  Updates the running maximum m and sum l,
// rescales the accumulator and writes the probabilities as B-operand groups.
template <typename T, bool MASKED>
__device__ __forceinline__ void softmax_step(const f32x16& S, uint32_t ab, float& m, float& l, f32x16& acc,
                                             typename ET<T>::grp (&pop)[ET<T>::GPT]) {
  float sc[16];
  float mt = kNegBig;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const bool ok = !MASKED || ((ab >> (8 * (r / 4) + (r % 4))) & 1u);
    sc[r] = ok ? S[r] : -__builtin_inff();
    mt = fmaxf(mt, sc[r]);
  }
  mt = max_halves(mt);
  const float mnew = fmaxf(m, mt);
  const float alpha = __builtin_amdgcn_exp2f(m - mnew);
  m = mnew;
  acc *= alpha;
  f32x16 pv;
  float lt = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pv[r] = __builtin_amdgcn_exp2f(sc[r] - mnew);
    lt += pv[r];
  }
  l = fmaf(l, alpha, sum_halves(lt));
#pragma unroll
  for (int g = 0; g < ET<T>::GPT; ++g) pop[g] = ET<T>::pack(pv, g);
}

// Softmax over the keys of the lane's own tile when only a window of W accumulator
// registers can be visible (groups of at most 2 W adjacent tokens: register window
// [W widx, W widx + W) with widx = (lane % 32) / (2 W)).  `wb` holds the visibility bits of
// the window (bit 8 (c/4) + c%4 for window register c).  It is the first step of a query's
// softmax (m, l, acc at their start values); with W = 16 it is softmax_step.
template <typename T, int W>
__device__ __forceinline__ void softmax_window(const f32x16& S, int widx, const uint32_t (&wmask)[16 / W], uint32_t wb,
                                               float& m, float& l, f32x16& acc,
                                               typename ET<T>::grp (&pop)[ET<T>::GPT]) {
  if (W == 16) { softmax_step<T, true>(S, wb, m, l, acc, pop); return; }
  float x[W];
  const bool b0 = widx & 1, b1 = widx & 2;
  // each score goes through an opaque register copy so that the choice below stays a
  // two-way select per value (not a variable-index extract from the 16-wide vector)
  float sv[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) { float t = S[r]; asm("" : "+v"(t)); sv[r] = t; }
#pragma unroll
  for (int c = 0; c < W; ++c) {
    if (W == 8) {
      const float a0 = sv[c], a1 = sv[8 + c];
      x[c] = b0 ? a1 : a0;
    } else {
      const float a0 = sv[c], a1 = sv[4 + c], a2 = sv[8 + c], a3 = sv[12 + c];
      const float lo = b0 ? a1 : a0, up = b0 ? a3 : a2;
      x[c] = b1 ? up : lo;
    }
  }
  float mt = kNegBig;
#pragma unroll
  for (int c = 0; c < W; ++c) {
    const bool ok = (wb >> (8 * (c / 4) + (c % 4))) & 1u;
    x[c] = ok ? x[c] : -__builtin_inff();
    mt = fmaxf(mt, x[c]);
  }
  mt = max_halves(mt);
  const float mnew = fmaxf(m, mt);
  const float alpha = __builtin_amdgcn_exp2f(m - mnew);
  float lt = 0.f;
#pragma unroll
  for (int c = 0; c < W; ++c) {
    x[c] = __builtin_amdgcn_exp2f(x[c] - mnew);
    lt += x[c];
  }
  lt = sum_halves(lt);
  l = l * alpha + lt;
  m = mnew;
  if (sizeof(T) == 2) {
    // pairs of probabilities -> packed bf16, dropped into the window's slots of the 8 pair slots
    uint32_t pk[W / 2];
#pragma unroll
    for (int c = 0; c < W / 2; ++c) {
      const bf16x2 t2 = {(__bf16)x[2 * c], (__bf16)x[2 * c + 1]};
      pk[c] = __builtin_bit_cast(uint32_t, t2);
    }
    uint32_t slot[8];     // wmask[w] is all ones in the lanes whose window is w, else zero
#pragma unroll
    for (int ps = 0; ps < 8; ++ps) slot[ps] = pk[ps % (W / 2)] & wmask[ps / (W / 2)];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const u32x4 v = {slot[4 * g], slot[4 * g + 1], slot[4 * g + 2], slot[4 * g + 3]};
      pop[g] = __builtin_bit_cast(typename ET<T>::grp, v);
    }
  } else {
    f32x16 pv;
#pragma unroll
    for (int r = 0; r < 16; ++r) pv[r] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x[r % W]) & wmask[r / W]);
#pragma unroll
    for (int g = 0; g < ET<T>::GPT; ++g) pop[g] = ET<T>::pack(pv, g);
  }
}

// Row `r` = (user, position) of the input-generation stage (Section 3.5.1): feature tiles below
// de hold item embedding + positional embedding, the others the time-difference features.
template <typename T, int NT>
__device__ __forceinline__ void input_rows(f32x16 (&x)[NT], const BlockParams& p, long long r, int pos, bool valid, int hi) {
  const int nte = p.de / 32, dt = NT * 32 - p.de;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    f32x16 a[1], b[1];
    if (t < nte) {
      load_rows<T, 1>(a, p.in_e, 0, r * p.de + 32 * t, valid, hi);
      load_rows<T, 1>(b, p.in_pos, 0, (long long)pos * p.de + 32 * t, valid, hi);
      x[t] = a[0] + b[0];
    } else {
      load_rows<T, 1>(a, p.in_td, 0, r * dt + 32 * (t - nte), valid, hi);
      x[t] = a[0];
    }
  }
}

// ---------------------------------------------------------------------------- the kernel
// RELU: the FFN activation (a template parameter: with both activations' loops in one kernel the
// compiler copies the residual registers in front of one of them)
// NW: waves (= tiles) per workgroup.  (One workgroup of 8 waves per compute unit instead of two of 4
// was measured for the d = 128 merge kernels, so that the two waves of a SIMD move through the
// block's phases together: 0.475-0.482 against 0.473-0.476 ms on one box, not kept.)
template <typename T, int D, int DH, int TT, int MODE, int W, bool RELU, int NW = kWaves>
__global__ void __launch_bounds__(64 * NW, (NW == kWaves && D <= 128 && TT == 1 && MODE != MODE_STACK) ? 2 : 1) block_kernel(const BlockParams p) {
  constexpr int kThreads = 64 * NW, kWaves = NW;   // (shadow the namespace-wide defaults)
  using E = ET<T>;
  using grp = typename E::grp;
  constexpr int NT = D / 32, NG = D / E::GF, GPT = E::GPT;
  constexpr int SEGV = NG * 64;
  constexpr int HPT = 32 / DH;        // heads per 32-feature tile
  constexpr int GPH = DH / E::GF;     // operand groups per head
  constexpr bool MERGE = MODE == MODE_MERGE || MODE == MODE_MERGE_IN;
  constexpr bool FUSED = (MERGE || MODE == MODE_SCORE);
  constexpr bool EXT = (MODE == MODE_ATTN || MODE == MODE_SCORE);
  constexpr bool STACK = MODE == MODE_STACK;
  constexpr bool ATTNLIKE = MODE == MODE_ATTN || STACK;   // rows are [globals; recent slots] of a user
  // kernels that run one wave per SIMD, where no other wave hides the LDS latency of a weight
  // fragment: the d <= 128 stack kernel takes scheduling hints (frag_pipeline_hint); at d = 256 the
  // compiler ignores them under its register pressure and the reads are placed ahead by hand.
  // The two-wave merge kernel takes the hints too (1 % faster)
  constexpr bool PIPE = sizeof(T) == 2 && TT == 1 && (STACK || MERGE) && D < 256;
  constexpr bool MANUAL = sizeof(T) == 2 && TT == 1 && D >= 256;
  constexpr bool BIGSEG = SEGV * 16 >= 16384;
  // bf16 kernels up to d = 128: the FFN loop is software pipelined over its hidden chunks and reads
  // the packed stream's FFN part in the skewed order (device.h)
  constexpr bool SKEW = ffn_skewed((int)sizeof(T), D);
  static_assert(!SKEW || TT == 1, "the pipelined FFN loop handles one tile per wave");
  constexpr int PSEG = BIGSEG ? 1 : 4;              // segments per panel of the weight stream (one barrier per panel)
  constexpr int NB = BIGSEG ? 6 : 2;                // ring depth in panels
  static_assert(DH == 16 || DH == 32, "head width");
  __shared__ uint4 lds[NB * PSEG * SEGV];
  __shared__ uint4 vecl[SEGV];          // the current block's fp32 vectors
  // MODE_STACK: K and V fragments of the current feature tile, [parity of ft][wave = key tile][K, V][group][lane]
  __shared__ uint4 kvl[STACK ? 2 * kWaves * 2 * GPT * 64 : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j = lane & 31, hi = lane >> 5;
  const int NC = p.FF / 32;

  // ------------------------------------------------------------------ rows of this wave
  bool valid[TT];          // the lane's token exists and takes part
  bool inrange[TT];        // the lane's row exists in the output tensor
  int usr[TT], Tu[TT];
  long long out_off[TT];   // element offset of the lane's output row
  uint32_t tilebits[TT];   // MODE_MERGE / MODE_SCORE: in-tile keys visible to this lane (window bits)
  const int widx = W == 16 ? 0 : j / (2 * W);
  uint32_t wmask[16 / W];
#pragma unroll
  for (int w = 0; w < 16 / W; ++w) { wmask[w] = widx == w ? 0xffffffffu : 0u; asm("" : "+v"(wmask[w])); }
  int lo1[TT], hi1[TT], lo2[TT], hi2[TT], kthi[TT];   // EXT: visible key ranges, key tile count
  int slo1[TT], shi1[TT], slo2[TT], shi2[TT];         // MODE_STACK: the same for the self-causal layers
  f32x16 resid[TT][NT];

  // Which group of 4 x TT tiles this workgroup takes.  Scoring: workgroups are dealt to the
  // chip's XCDs (each with its own L2) round-robin by their index, so the index is decoded
  // such that all candidate tiles of a user run on one XCD and its L2 holds that user's
  // cached K/V.
  int wg = blockIdx.x, su = 0;
  if (MODE == MODE_SCORE) {
    const int x = (int)blockIdx.x % p.xcds, sq = (int)blockIdx.x / p.xcds;
    su = x + p.xcds * (sq / p.wg_per_user);
    wg = sq % p.wg_per_user;
    if (su >= p.B) return;     // the grid is rounded up to whole XCD rows
  }

#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int tile = (wg * kWaves + wave) * TT + tt;
    valid[tt] = false; inrange[tt] = false; usr[tt] = 0; Tu[tt] = 0; out_off[tt] = 0; tilebits[tt] = 0;
    lo1[tt] = hi1[tt] = lo2[tt] = hi2[tt] = kthi[tt] = 0;
    slo1[tt] = shi1[tt] = slo2[tt] = shi2[tt] = 0;
    if (MERGE) {
      // K divides 32, so it is a power of two; the launcher keeps the slot count below 2^31
      const uint32_t slot = (uint32_t)tile * 32u + (uint32_t)j;
      const uint32_t gidx = slot >> __builtin_ctz(p.K);
      const int jj = (int)(slot & (uint32_t)(p.K - 1));
      const int u = (int)(gidx / (uint32_t)p.T), t = (int)(gidx - (uint32_t)u * (uint32_t)p.T);
      inrange[tt] = u < p.B;
      int len = 0;
      if (inrange[tt]) { len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L); }
      const int pos = t * p.K + jj;
      valid[tt] = inrange[tt] && pos < len;
      usr[tt] = u; Tu[tt] = len;             // Tu holds the raw length here
      out_off[tt] = slot;                    // group-slot index; scaled when writing
      if (MODE == MODE_MERGE_IN) input_rows<T, NT>(resid[tt], p, (long long)u * p.L + pos, pos, valid[tt], hi);
      else load_rows<T, NT>(resid[tt], p.H, 0, ((long long)u * p.L + pos) * D, valid[tt], hi);
      const uint32_t vb = (uint32_t)__ballot(valid[tt]);
      const uint32_t gb = (p.K >= 32 ? 0xffffffffu : ((1u << p.K) - 1u)) << (p.K * (j / p.K));
      tilebits[tt] = ((gb & vb) >> (4 * hi)) >> (2 * W * widx);
    } else if (MODE == MODE_KVPROJ) {
      const int u = tile / p.tiles_per_user, kt = tile - u * p.tiles_per_user;
      const int c = 32 * kt + j;
      inrange[tt] = u < p.B;
      const bool first = c < p.m0;
      // a row takes part only if its token exists: a merged token below T_u (cross layer), a valid
      // query slot (self layers).  Rows of other tokens are never read (they may hold anything) and
      // are projected from zeros; every query hides their keys.
      int len = 0;
      if (inrange[tt]) { len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L); }
      const int tu = (len + p.K - 1) / p.K, i = c - p.m0;
      const bool exists = first || (p.key_self ? i >= first_slot(p.k, tu, p.q_learn) : i < tu);
      valid[tt] = inrange[tt] && c < p.rows_per_user && exists;
      usr[tt] = u; Tu[tt] = kt;              // Tu holds the key tile index here
      const void* sp = first ? p.src0.p : p.src1.p;
      const int sf = first ? p.src0.f32 : p.src1.f32;
      const long long su = first ? p.src0.ustride : p.src1.ustride;
      load_rows<T, NT>(resid[tt], sp, sf, su * u + (long long)(first ? c : c - p.m0) * D, valid[tt], hi);
    } else if (ATTNLIKE) {
      const int u = tile / p.tiles_per_user, qt = tile - u * p.tiles_per_user;
      const int a = p.q0 + 32 * qt + j;
      inrange[tt] = u < p.B && (32 * qt + j) < p.rows_per_user;
      int len = 0;
      if (u < p.B) { len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L); }
      const int tu = (len + p.K - 1) / p.K;
      const bool glob = a < p.m;
      const int i = a - p.m, i0 = first_slot(p.k, tu, p.q_learn);
      valid[tt] = inrange[tt] && (glob || i >= i0);
      usr[tt] = u; Tu[tt] = tu;
      out_off[tt] = p.X_ustride * u + (long long)a * D;
      const void* sp = glob ? p.src0.p : p.src1.p;
      const int sf = glob ? p.src0.f32 : p.src1.f32;
      const long long su = glob ? p.src0.ustride : p.src1.ustride;
      // a learnable query token stands after the user's newest token: it sees all of them
      const int tok = glob ? 0 : (p.q_learn ? tu - 1 : slot_token(i, p.k, tu, p.k_uni));
      const int row = glob ? a : (p.gather_recent ? tok : i);
      load_rows<T, NT>(resid[tt], sp, sf, su * u + (long long)row * D, valid[tt], hi);
      // visible key ranges (Eq. 8 by token type)
      const int s0 = p.key_self ? i0 : 0;
      if (glob) {
        lo1[tt] = p.gmask_causal ? a : 0; hi1[tt] = p.KG;
        lo2[tt] = p.KG + s0; hi2[tt] = p.KG + (p.key_self ? p.k : tu);
      } else {
        lo1[tt] = 0; hi1[tt] = 0;
        lo2[tt] = p.KG + s0; hi2[tt] = p.KG + (p.key_self ? i : tok) + 1;
      }
      if (!valid[tt]) { hi1[tt] = lo1[tt]; hi2[tt] = lo2[tt]; }
      kthi[tt] = (p.KG + (p.key_self ? p.k : tu) + 31) / 32;
      if (u >= p.B) kthi[tt] = 0;
      if (STACK && valid[tt]) {   // keys of a self-causal layer: the user's own rows, key index = row index
        if (glob) { slo1[tt] = p.gmask_causal ? a : 0; shi1[tt] = p.m; slo2[tt] = p.m + i0; shi2[tt] = p.m + p.k; }
        else { slo2[tt] = p.m + i0; shi2[tt] = p.m + i + 1; }
      }
    } else if (MODE == MODE_INPUT) {
      // row = one raw token; x = [item embedding + positional embedding ; time-difference feature]
      const long long r = (long long)tile * 32 + j;
      const int u = (int)(r / p.L), pos = (int)(r - (long long)u * p.L);
      inrange[tt] = u < p.B;
      int len = 0;
      if (inrange[tt]) { len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L); }
      valid[tt] = inrange[tt] && pos < len;
      usr[tt] = u; out_off[tt] = r * D;
      input_rows<T, NT>(resid[tt], p, r, pos, valid[tt], hi);
    } else {  // MODE_SCORE
      const int u = su;
      const int a = 32 * tile + j;
      const int cand = a / p.m, gi = a - cand * p.m;
      inrange[tt] = cand < p.C;
      valid[tt] = inrange[tt];
      int len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L);
      usr[tt] = u; Tu[tt] = (len + p.K - 1) / p.K;
      out_off[tt] = ((long long)u * p.C * p.m + a) * D;
      load_rows<T, NT>(resid[tt], p.Gc, 0, out_off[tt], valid[tt], hi);
      const uint32_t vb = (uint32_t)__ballot(valid[tt]);
      const int gbase = p.m * (j / p.m);
      tilebits[tt] = ((range_bits(gbase + (p.gmask_causal ? gi : 0), gbase + p.m, 0) & vb) >> (4 * hi)) >> (2 * W * widx);
    }
  }

  if (MERGE) {
    // a workgroup whose tokens are all padding writes zeros and leaves
    bool any = false;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) any |= valid[tt];
    if (!__syncthreads_or(any ? 1 : 0)) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        if (!inrange[tt]) continue;
        if (p.Z_out) store_rows<T, NT>(resid[tt], p.Z_out, p.Z_f32, out_off[tt] * D, false, hi);
        if (p.M_out && (out_off[tt] & (p.K - 1)) == 0)
          store_rows<T, NT>(resid[tt], p.M_out, p.M_f32, (out_off[tt] >> __builtin_ctz(p.K)) * D, false, hi);
      }
      return;
    }
  }

  WStream<SEGV, PSEG, NB, MODE == MODE_KVPROJ, kThreads> ws;
  const int NF = 2 * NC + 1;     // segments of a block's FFN part (device.h)
  const int steps = 1 + (MODE == MODE_KVPROJ ? 2 * NT : MODE == MODE_INPUT ? NF : (ATTNLIKE ? 2 * NT + NF : 4 * NT + NF));
  // MODE_STACK: the cross block's attention sub-stream, then the self blocks in the fused
  // layout, back to back (every part has an even number of segments).
  // MODE_MERGE_IN: the input MLP's segments, then the InnerTrans blocks (n_layers counts both)
  ws.init(lds, p.wbase, STACK ? steps + (p.n_layers - 1) * (1 + 4 * NT + NF)
                              : MODE == MODE_MERGE_IN ? 1 + NF + (p.n_layers - 1) * steps : steps * p.n_layers);

  // hands the NG weight fragments of the current segment to use(s, w) one by one; MANUAL keeps
  // AH reads in flight in front of the MFMA that is being issued (the order is pinned)
  auto for_frags = [&](auto&& use) {
    if constexpr (!MANUAL) {
#pragma unroll
      for (int s = 0; s < NG; ++s) use(s, ws.template frag<grp>(s));
    } else {
      constexpr int AH = 4;
      grp ring[AH];
#pragma unroll
      for (int s = 0; s < AH; ++s) ring[s] = ws.template frag<grp>(s);
#pragma unroll
      for (int s = 0; s < NG; ++s) {
        __builtin_amdgcn_sched_barrier(0);
        use(s, ring[s % AH]);
        __builtin_amdgcn_sched_barrier(0);
        if (s + AH < NG) ring[s % AH] = ws.template frag<grp>(s + AH);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  for (int layer = 0; layer < p.n_layers; ++layer) {
    // the block's first segment holds its fp32 vectors: keep a copy for the whole layer
    // (barriers: nobody still reads the previous block's copy; everybody sees the new one)
    if (layer > 0) __syncthreads();
    if (SEGV < kThreads) {     // bf16 at d = 32: the segment is smaller than the workgroup
      if (tid < SEGV) vecl[tid] = ws.cur()[tid];
    }
#pragma unroll
    for (int i = 0; i < SEGV / kThreads; ++i) vecl[tid + kThreads * i] = ws.cur()[tid + kThreads * i];
    __syncthreads();
    ws.advance();
    const float* vec = reinterpret_cast<const float*>(vecl);
    const VecLayout vl{D, p.FF};
    grp xn[TT][NG];
    const bool selfl = STACK && layer > 0;   // a self-causal layer of the stack: K/V made here
    // input generation (alone, or as the pass in front of the InnerTrans blocks): no norm, no
    // attention, no residual -- the rows themselves are the first GEMM's operand and the result
    // starts from the output bias
    const bool mlp_only = MODE == MODE_INPUT || (MODE == MODE_MERGE_IN && layer == 0);
    if (mlp_only) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int g = 0; g < GPT; ++g) xn[tt][t * GPT + g] = E::pack(resid[tt][t], g);
          resid[tt][t] = splat16(0.f);
        }
    } else {
    layer_norm<T, D, TT>(resid, vec + vl.ln1_g(), vec + vl.ln1_b(), p.eps, hi, xn);
    grp oop[TT][NG];

#pragma unroll
    for (int ft = 0; ft < NT; ++ft) {
      f32x16 aq[TT], ak[TT], av[TT];
      if (MODE != MODE_KVPROJ) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) aq[tt] = bias_tile(vec + vl.bq(), ft, hi);
        for_frags([&](int s, const grp w) {
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) aq[tt] = E::mma(w, xn[tt][s], aq[tt]);
        });
        if (PIPE) frag_pipeline_hint<NG, 4>();
        ws.advance();
      }
      if (FUSED || MODE == MODE_KVPROJ || selfl) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) ak[tt] = splat16(0.f);   // no b_K: a per-query constant in the scores, softmax drops it
        for_frags([&](int s, const grp w) {
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) ak[tt] = E::mma(w, xn[tt][s], ak[tt]);
        });
        if (PIPE) frag_pipeline_hint<NG, 0>();
        ws.advance();
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) av[tt] = splat16(0.f);   // no b_V: probabilities sum to 1, so the pack kernel folds it into the output bias
        for_frags([&](int s, const grp w) {
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) av[tt] = E::mma(xn[tt][s], w, av[tt]);   // operands swapped: lane = feature
        });
        if (PIPE) frag_pipeline_hint<NG, 0>();
        ws.advance();
      }
      if (selfl) {
        // this wave's rows are key tile `wave`: hand its K and V fragments to the other waves.
        // One barrier per feature tile is enough with two buffers: nobody can be two tiles
        // ahead of a wave that still reads.
        static_assert(!STACK || TT == 1, "one tile per wave in the stack kernel");
        uint4* dstk = kvl + (size_t)(((ft & 1) * kWaves + wave) * 2) * GPT * 64 + lane;
#pragma unroll
        for (int g = 0; g < GPT; ++g) {
          *reinterpret_cast<grp*>(dstk + g * 64) = E::pack(ak[0], g);
          *reinterpret_cast<grp*>(dstk + (GPT + g) * 64) = E::pack(av[0], g);
        }
        __syncthreads();
      }
      if (MODE == MODE_KVPROJ) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          if (!inrange[tt]) continue;
          const size_t fo = (size_t)usr[tt] * p.kv_ustride + ((size_t)(Tu[tt] * NT + ft) * GPT) * 1024 + lane * 16;
#pragma unroll
          for (int g = 0; g < GPT; ++g) {
            *reinterpret_cast<grp*>(p.kst + fo + g * 1024) = E::pack(ak[tt], g);
            *reinterpret_cast<grp*>(p.vst + fo + g * 1024) = E::pack(av[tt], g);
          }
        }
        continue;
      }

#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        grp qop[GPT];   // Q carries log2(e) / sqrt(head width): the scores come out ready for exp2
        aq[tt] *= p.scale_l2e;
#pragma unroll
        for (int g = 0; g < GPT; ++g) qop[g] = E::pack(aq[tt], g);
        float mrun[HPT], lrun[HPT];
        f32x16 acc[HPT];
#pragma unroll
        for (int hh = 0; hh < HPT; ++hh) { mrun[hh] = kNegBig; lrun[hh] = 0.f; acc[hh] = splat16(0.f); }

        if (FUSED) {   // keys of the lane's own tile (group attention / the candidate's own globals)
          grp kop[GPT], vop[GPT];
#pragma unroll
          for (int g = 0; g < GPT; ++g) { kop[g] = E::pack(ak[tt], g); vop[g] = E::pack(av[tt], g); }
#pragma unroll
          for (int hh = 0; hh < HPT; ++hh) {
            f32x16 S = splat16(0.f);
#pragma unroll
            for (int g2 = 0; g2 < GPH; ++g2) S = E::mma(kop[hh * GPH + g2], qop[hh * GPH + g2], S);
            grp pop[GPT];
            softmax_window<T, W>(S, widx, wmask, tilebits[tt], mrun[hh], lrun[hh], acc[hh], pop);
#pragma unroll
            for (int g = 0; g < GPT; ++g) acc[hh] = E::mma(vop[g], pop[g], acc[hh]);
          }
        }
        if (selfl) {   // K/V fragments of the user's own rows, from LDS
          const int nkt = (p.m + p.k + 31) / 32;
          for (int kt = 0; kt < nkt; ++kt) {
            const uint32_t bits = range_bits(slo1[tt], shi1[tt], 32 * kt) | range_bits(slo2[tt], shi2[tt], 32 * kt);
            const uint32_t ab = (bits >> (4 * hi)) & kTileBits;
            if (__builtin_amdgcn_ballot_w64(ab != 0) == 0) continue;      // no query of the tile sees any of these keys
            const bool full = __builtin_amdgcn_ballot_w64(ab != kTileBits) == 0;   // every query sees all of them
            const f32x16 vis = full ? splat16(0.f) : mask_tile(ab);
            const uint4* srck = kvl + (size_t)(((ft & 1) * kWaves + kt) * 2) * GPT * 64 + lane;
            grp kfr[GPT], vfr[GPT];
#pragma unroll
            for (int g = 0; g < GPT; ++g) {
              kfr[g] = *reinterpret_cast<const grp*>(srck + g * 64);
              vfr[g] = *reinterpret_cast<const grp*>(srck + (GPT + g) * 64);
            }
#pragma unroll
            for (int hh = 0; hh < HPT; ++hh) {
              f32x16 S = vis;
#pragma unroll
              for (int g2 = 0; g2 < GPH; ++g2) S = E::mma(kfr[hh * GPH + g2], qop[hh * GPH + g2], S);
              grp pop[GPT];
              softmax_step<T, false>(S, 0u, mrun[hh], lrun[hh], acc[hh], pop);
#pragma unroll
              for (int g = 0; g < GPT; ++g) acc[hh] = E::mma(vfr[g], pop[g], acc[hh]);
            }
          }
        }
        if (EXT || (STACK && !selfl)) {     // stored K/V fragments (all waves of a tile's user read the same ones)
          // all rows of a tile belong to one user in these modes: user, key tile count and the
          // fragment base addresses are wave-uniform (scalar registers, scalar loop control)
          const int uu = __builtin_amdgcn_readfirstlane(usr[tt]);
          const int tuu = __builtin_amdgcn_readfirstlane(Tu[tt]);
          const char* kb; const char* vb; int nkt, rlo, rhi;
          if (ATTNLIKE) {
            kb = p.kst + (size_t)uu * p.kv_ustride; vb = p.vst + (size_t)uu * p.kv_ustride;
            nkt = __builtin_amdgcn_readfirstlane(kthi[tt]); rlo = 0; rhi = 0;
          } else {
            const int i0 = first_slot(p.k, tuu, p.q_learn);
            if (layer == 0) {
              kb = p.cache + (size_t)uu * p.c0_ustride; vb = kb + p.c0_voff;
              nkt = min(p.kt0, (tuu + 31) / 32); rlo = 0; rhi = tuu;
            } else {
              kb = p.cache + p.c1_off + (size_t)(layer - 1) * p.c1_lstride + (size_t)uu * p.c1_ustride;
              vb = kb + p.c1_voff;
              nkt = tuu > 0 ? p.kt1 : 0; rlo = i0; rhi = p.k;
            }
            if (!valid[tt]) rhi = rlo;
          }
          // scoring (long key sequences, one candidate tile per wave): the fragments of key
          // tile kt + 1 are requested before tile kt is worked on
          constexpr bool AHEAD = MODE == MODE_SCORE;
          grp knx[GPT], vnx[GPT];
          if (AHEAD && nkt > 0) {
            const size_t fo = ((size_t)ft * GPT) * 1024 + lane * 16;
#pragma unroll
            for (int g = 0; g < GPT; ++g) {
              knx[g] = *reinterpret_cast<const grp*>(kb + fo + g * 1024);
              vnx[g] = *reinterpret_cast<const grp*>(vb + fo + g * 1024);
            }
          }
          for (int kt = 0; kt < nkt; ++kt) {
            uint32_t bits;
            if (ATTNLIKE) bits = range_bits(lo1[tt], hi1[tt], 32 * kt) | range_bits(lo2[tt], hi2[tt], 32 * kt);
            else bits = range_bits(rlo, rhi, 32 * kt);
            const uint32_t ab = (bits >> (4 * hi)) & kTileBits;
            const bool none = __builtin_amdgcn_ballot_w64(ab != 0) == 0;           // nobody sees any of these keys
            const bool full = __builtin_amdgcn_ballot_w64(ab != kTileBits) == 0;   // everybody sees all of them
            if (!AHEAD && none) continue;
            grp kfr[GPT], vfr[GPT];
            if (AHEAD) {
#pragma unroll
              for (int g = 0; g < GPT; ++g) { kfr[g] = knx[g]; vfr[g] = vnx[g]; }
            } else {
              const size_t fo = ((size_t)(kt * NT + ft) * GPT) * 1024 + lane * 16;
#pragma unroll
              for (int g = 0; g < GPT; ++g) {
                kfr[g] = *reinterpret_cast<const grp*>(kb + fo + g * 1024);
                vfr[g] = *reinterpret_cast<const grp*>(vb + fo + g * 1024);
              }
            }
            if (AHEAD && kt + 1 < nkt) {
              const size_t fo = ((size_t)((kt + 1) * NT + ft) * GPT) * 1024 + lane * 16;
#pragma unroll
              for (int g = 0; g < GPT; ++g) {
                knx[g] = *reinterpret_cast<const grp*>(kb + fo + g * 1024);
                vnx[g] = *reinterpret_cast<const grp*>(vb + fo + g * 1024);
              }
            }
            if (AHEAD && none) continue;
            const f32x16 vis = full ? splat16(0.f) : mask_tile(ab);
#pragma unroll
            for (int hh = 0; hh < HPT; ++hh) {
              f32x16 S = vis;
#pragma unroll
              for (int g2 = 0; g2 < GPH; ++g2) S = E::mma(kfr[hh * GPH + g2], qop[hh * GPH + g2], S);
              grp pop[GPT];
              softmax_step<T, false>(S, 0u, mrun[hh], lrun[hh], acc[hh], pop);
#pragma unroll
              for (int g = 0; g < GPT; ++g) acc[hh] = E::mma(vfr[g], pop[g], acc[hh]);
            }
          }
        }
        // normalise; with two heads per tile each head owns half of the accumulator rows
        f32x16 o;
        float inv[HPT];
#pragma unroll
        for (int hh = 0; hh < HPT; ++hh)   // (bf16 mode: the hardware reciprocal, 1 ulp, instead of the exact division)
          inv[hh] = lrun[hh] > 0.f ? (sizeof(T) == 4 ? 1.0f / lrun[hh] : __builtin_amdgcn_rcpf(lrun[hh])) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int hh = HPT == 1 ? 0 : r / 8;
          o[r] = acc[hh][r] * inv[hh];
        }
#pragma unroll
        for (int g = 0; g < GPT; ++g) oop[tt][ft * GPT + g] = E::pack(o, g);
      }
    }
    if (MODE == MODE_KVPROJ) { wait_vmcnt<0>(); return; }

    // output projection + residual
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const f32x16 bo = bias_tile(vec + vl.bo(), nt, hi);
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) resid[tt][nt] += bo;
      for_frags([&](int s, const grp w) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) resid[tt][nt] = E::mma(w, oop[tt][s], resid[tt][nt]);
      });
      if (PIPE) frag_pipeline_hint<NG, 4>();
      ws.advance();
    }

    // FFN, 32 hidden features at a time: hidden chunk never leaves registers
    layer_norm<T, D, TT>(resid, vec + vl.ln2_g(), vec + vl.ln2_b(), p.eps, hi, xn);
    }   // !mlp_only
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {      // FFN output bias goes in first: the vectors may be
      const f32x16 b2 = bias_tile(vec + vl.b2(), nt, hi);   // replaced right after the last segment
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) resid[tt][nt] += b2;
    }
    if constexpr (SKEW) {
      // Software-pipelined FFN.  The matrix pipe and the vector ALU overlap only inside one wave's
      // instruction stream, at about four VALU instructions per MFMA (an MFMA followed by another
      // MFMA keeps the issue port until the pipe is free, and another wave's VALU work waits with
      // it).  The activation of chunk i is therefore issued between the MFMAs of two GEMMs that do
      // not depend on it, the first GEMM of chunk i + 1 and the second GEMM of chunk i - 1, one
      // stage of its polynomial (four packed instructions that do not depend on each other) behind
      // each MFMA.  ah[i & 1] holds chunk i's hidden pre-activations, hop[i & 1] its activated
      // operand groups; the packed stream brings the pair {W2(i-1), W1(i+1)} side by side (device.h).
      // The order is written out and pinned (sched_barrier): under this kernel's register pressure
      // the compiler's scheduler does not follow group hints here.
      f32x16 ah[2];
      typename E::hgrp hop[2][GPT];
      constexpr int NS = RELU ? 2 : 8;          // stages of one operand group's activation
      constexpr int NP = GPT * NS;              // stages of a chunk
      f16x8 ay, av, ap;                         // the group in flight: y = x / kFfnScale, y^2, the polynomial
      // stage st of operand group gg of the chunk in `a`; the last stage delivers the group
      // A stage's first operand passes through an empty volatile asm statement: the stage then
      // cannot be moved ahead of the MFMA it is written behind (pure arithmetic is otherwise free
      // to move across the pinned points, and the compiler gathers it in front of the MFMAs).
      auto pin = [&](f16x8& x) {
        u32x4 t = __builtin_bit_cast(u32x4, x);
        asm volatile("" : "+v"(t));
        x = __builtin_bit_cast(f16x8, t);
      };
      auto act_stage = [&](const f32x16& a, int gg, int st, typename E::hgrp& out) {
        if (st == 0) {          // pairs of elements to fp16 (toward zero: never to infinity)
#pragma unroll
          for (int e = 0; e < E::EPL / 2; ++e) {
            float lo = a[E::EPL * gg + 2 * e], up = a[E::EPL * gg + 2 * e + 1];
            asm volatile("" : "+v"(lo), "+v"(up));
            const f16x2 y2 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(lo, up));
            ay[2 * e] = y2[0]; ay[2 * e + 1] = y2[1];
          }
          return;
        }
        if (st == 1 || RELU) pin(ay); else if (st == 2) pin(av); else pin(ap);
        if (RELU) {
          out = __builtin_elementwise_max(ay, (f16x8)((_Float16)0.f));
        } else if (st == 1) {   // the polynomial of gelu_quarter_h8, one Horner step per stage
          av = ay * ay;
        } else if (st == 2) {
          ap = __builtin_elementwise_fma((f16x8)((_Float16)2.4554419175668456f), av, (f16x8)((_Float16)-6.304095499217479f));
        } else if (st == 3) {
          ap = __builtin_elementwise_fma(ap, av, (f16x8)((_Float16)6.604333663059149f));
        } else if (st == 4) {
          ap = __builtin_elementwise_fma(ap, av, (f16x8)((_Float16)-3.771901897714043f));
        } else if (st == 5) {
          ap = __builtin_elementwise_fma(ap, av, (f16x8)((_Float16)1.5736394077430096f));
        } else if (st == 6) {
          ap = __builtin_elementwise_fma(ay, ap, (f16x8)((_Float16)0.5f));
          ap = __builtin_elementwise_min(__builtin_elementwise_max(ap, (f16x8)((_Float16)0.f)), (f16x8)((_Float16)1.f));
        } else {
          out = ay * ap;
        }
      };
      // One pipeline step on chunk i (PA = i & 1).  F2: the second GEMM of chunk i - 1 from the
      // pair's first segment; F1: the first GEMM of chunk i + 1 from its second segment (the first,
      // without F2); ACT: the activation of chunk i.  The MFMAs of the two GEMMs alternate.
      auto step = [&](auto pa_, auto f1_, auto f2_, auto act_, int i) {
        constexpr int PA = decltype(pa_)::value, PB = PA ^ 1;
        constexpr bool F1 = decltype(f1_)::value, F2 = decltype(f2_)::value, ACT = decltype(act_)::value;
        constexpr int NM = (F1 ? NG : 0) + (F2 ? NG : 0);      // GPT * NT = NG MFMAs in either GEMM
        constexpr int AH = 3;                                    // fragment reads in flight
        if constexpr (F1) ah[PB] = bias_tile(vec + vl.b1(), i + 1, hi);
        // MFMA q of the step: which GEMM, which fragment
        auto is_f2 = [&](int q) { return F2 && (!F1 || (q & 1) == 0); };
        auto load = [&](int q) -> grp {
          const int j = (F1 && F2) ? q / 2 : q;
          if (is_f2(q)) return ws.template frag_at<grp>(0, (j % NT) * GPT + j / NT);   // output tile j % NT, operand group j / NT
          return ws.template frag_at<grp>(F2 ? 1 : 0, j);
        };
        grp fr[AH];
#pragma unroll
        for (int q = 0; q < AH && q < NM; ++q) fr[q] = load(q);
#pragma unroll
        for (int q = 0; q < NM; ++q) {
          __builtin_amdgcn_sched_barrier(0);
          const int j = (F1 && F2) ? q / 2 : q;
          if (is_f2(q)) resid[0][j % NT] = E::mma_h(fr[q % AH], hop[PB][j / NT], resid[0][j % NT]);
          else ah[PB] = E::mma(fr[q % AH], xn[0][j], ah[PB]);
          if (q + AH < NM) fr[q % AH] = load(q + AH);
          if constexpr (ACT) {
#pragma unroll
            for (int pc = q * NP / NM; pc < (q + 1) * NP / NM; ++pc) act_stage(ah[PA], pc / NS, pc % NS, hop[PA][pc / NS]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        ws.advance();
        ws.advance();
      };
      using std::integral_constant;
      typedef integral_constant<int, 0> I0; typedef integral_constant<int, 1> I1;
      typedef integral_constant<bool, true> Yes; typedef integral_constant<bool, false> No;
      // chunk 0's first GEMM alone
      ah[0] = bias_tile(vec + vl.b1(), 0, hi);
      for_frags([&](int sg, const grp w) { ah[0] = E::mma(w, xn[0][sg], ah[0]); });
      if (PIPE) frag_pipeline_hint<NG, 4>();
      ws.advance();
      step(I0{}, Yes{}, No{}, Yes{}, 0);                    // {W1(1), unused}: activation of chunk 0 under chunk 1's first GEMM
      int i = 1;
#pragma unroll 1
      for (; i + 1 <= NC - 2; i += 2) {
        step(I1{}, Yes{}, Yes{}, Yes{}, i);
        step(I0{}, Yes{}, Yes{}, Yes{}, i + 1);
      }
      // the last pair {W2(NC-2), W2(NC-1)}: second GEMM of chunk NC - 2 under the activation of
      // chunk NC - 1, then the second GEMM of chunk NC - 1 alone
      auto last = [&](auto pa_) {
        constexpr int PA = decltype(pa_)::value;
        constexpr int AH = 3;
        grp fr[AH];
        auto load = [&](int q) -> grp { const int j = q % NG; return ws.template frag_at<grp>(q / NG, (j % NT) * GPT + j / NT); };
#pragma unroll
        for (int q = 0; q < AH; ++q) fr[q] = load(q);
#pragma unroll
        for (int q = 0; q < 2 * NG; ++q) {
          __builtin_amdgcn_sched_barrier(0);
          const int j = q % NG;
          resid[0][j % NT] = E::mma_h(fr[q % AH], hop[q < NG ? (PA ^ 1) : PA][j / NT], resid[0][j % NT]);
          if (q + AH < 2 * NG) fr[q % AH] = load(q + AH);
          if (q < NG) {
#pragma unroll
            for (int pc = q * NP / NG; pc < (q + 1) * NP / NG; ++pc) act_stage(ah[PA], pc / NS, pc % NS, hop[PA][pc / NS]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        ws.advance();
        ws.advance();
      };
      if (i <= NC - 2) {                                    // an odd number of middle steps: chunk NC - 1 is even
        step(I1{}, Yes{}, Yes{}, Yes{}, i);
        last(I0{});
      } else {
        last(I1{});
      }
    } else {
#pragma unroll 1
    for (int c = 0; c < NC; ++c) {
      f32x16 ah[TT];
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) ah[tt] = bias_tile(vec + vl.b1(), c, hi);
      for_frags([&](int s, const grp w) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) ah[tt] = E::mma(w, xn[tt][s], ah[tt]);
      });
      if (PIPE) frag_pipeline_hint<NG, 4>();
      ws.advance();
      // operand group by operand group: the second GEMM's MFMAs that use group g (one per
      // output tile, independent accumulators) only need the activation of that group's
      // registers, so the rest of the activation's VALU work can run under them
#pragma unroll
      for (int g = 0; g < GPT; ++g) {
        typename E::hgrp hop[TT];
        auto act_group = [&](int gg) {
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) {
            if constexpr (E::HALF_FFN) {
              // ah holds x / kFfnScale; pairs of elements go to fp16 (toward zero: never to
              // infinity) and through the packed activation
              f16x8 y;
#pragma unroll
              for (int e = 0; e < E::EPL / 2; ++e) {
                const f16x2 y2 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(ah[tt][E::EPL * gg + 2 * e],
                                                                                      ah[tt][E::EPL * gg + 2 * e + 1]));
                y[2 * e] = y2[0]; y[2 * e + 1] = y2[1];
              }
              hop[tt] = RELU ? __builtin_elementwise_max(y, (f16x8)((_Float16)0.f)) : gelu_quarter_h8(y);
            } else {
#pragma unroll
              for (int e = 0; e < E::EPL; ++e) {
                const float v = ah[tt][E::EPL * gg + e];
                ah[tt][E::EPL * gg + e] = RELU ? fmaxf(v, 0.f) : gelu_fn<true>(v);
              }
              hop[tt] = E::pack(ah[tt], gg);
            }
          }
        };
        if constexpr (MANUAL) {
          // the wide kernels: the group's first fragments are requested before its activation
          // (their latency passes under the VALU work), the rest a fixed distance ahead
          constexpr int AH = 4;
          grp ring[AH];
#pragma unroll
          for (int nt = 0; nt < AH; ++nt) ring[nt] = ws.template frag<grp>(nt * GPT + g);
          __builtin_amdgcn_sched_barrier(0);
          act_group(g);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            __builtin_amdgcn_sched_barrier(0);
            resid[0][nt] = E::mma_h(ring[nt % AH], hop[0], resid[0][nt]);
            __builtin_amdgcn_sched_barrier(0);
            if (nt + AH < NT) ring[nt % AH] = ws.template frag<grp>((nt + AH) * GPT + g);
          }
          __builtin_amdgcn_sched_barrier(0);
          continue;
        }
        act_group(g);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const grp w = ws.template frag<grp>(nt * GPT + g);
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) resid[tt][nt] = E::mma_h(w, hop[tt], resid[tt][nt]);
        }
      }
      if (sizeof(T) == 2 && TT == 1 && !RELU && !MANUAL) {
        // order within this stretch: activation of group 0, the weight fragments, then each
        // MFMA of group 0 followed by a quarter of group 1's activation, then group 1's MFMAs
        constexpr int VG = 32;   // VALU instructions of one group's activation (4 conversions + 7 x 4 packed ops)
        __builtin_amdgcn_sched_group_barrier(0x002, VG, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * NT, 0);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, VG / NT, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);
      }
      ws.advance();
    }
    ws.advance();   // the unused segment that ends the FFN part
    }
  }

  wait_vmcnt<0>();   // nothing of the weight stream may still be in flight when the wave ends
  // ------------------------------------------------------------------ epilogues
  if (MERGE) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      if (p.Z_out && inrange[tt]) store_rows<T, NT>(resid[tt], p.Z_out, p.Z_f32, out_off[tt] * D, valid[tt], hi);
      if (p.M_out) {
        // mean over the valid tokens of each group: tokens of a group sit on K adjacent lanes
        const uint32_t gidx = (uint32_t)out_off[tt] >> __builtin_ctz(p.K);
        const int jj = (int)((uint32_t)out_off[tt] & (uint32_t)(p.K - 1));
        const int t = (int)(gidx % (uint32_t)p.T);
        const int nv = min(max(Tu[tt] - t * p.K, 0), p.K);
        const float wgt = valid[tt] ? 1.0f / (float)nv : 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) resid[tt][nt] *= wgt;
        // butterfly over the K lanes of a group, one level for all values at a time; the
        // mirrors serve as the xor-4 / xor-8 exchanges because the partial sums are already
        // uniform inside each block of 4 / 8 lanes
        if (p.K >= 2) lane_sum<0xB1, NT>(resid[tt]);     // quad_perm [1,0,3,2]
        if (p.K >= 4) lane_sum<0x4E, NT>(resid[tt]);     // quad_perm [2,3,0,1]
        if (p.K >= 8) lane_sum<0x141, NT>(resid[tt]);    // row_half_mirror
        if (p.K >= 16) lane_sum<0x140, NT>(resid[tt]);   // row_mirror
        if (p.K >= 32) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) resid[tt][nt][r] += __shfl_xor(resid[tt][nt][r], 16, 64);
        }
        if (inrange[tt] && jj == 0)
          store_rows<T, NT>(resid[tt], p.M_out, p.M_f32, (long long)gidx * D, true, hi);
      }
    }
  } else if (MODE == MODE_INPUT) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
      if (inrange[tt]) store_rows<T, NT>(resid[tt], p.X_out, 0, out_off[tt], valid[tt], hi);
  } else if (ATTNLIKE || MODE == MODE_SCORE) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      if (p.X_out && inrange[tt]) store_rows<T, NT>(resid[tt], p.X_out, p.X_f32, out_off[tt], valid[tt], hi);
      if (p.logits) {
        // logit = <head_w, flatten(global rows)> + head_b
        const int tile = (wg * kWaves + wave) * TT + tt;
        int a, width;       // row inside the head's m rows; lanes per logit
        bool take;
        if (ATTNLIKE) {
          const int qt = tile % p.tiles_per_user;
          a = p.q0 + 32 * qt + j; take = valid[tt] && a < p.m; width = 32;
        } else {
          a = (32 * tile + j) % p.m; take = valid[tt]; width = p.m;
        }
        float part = 0.f;
        if (take) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const f32x16 hw = bias_tile(p.head + (size_t)a * D, nt, hi);
#pragma unroll
            for (int r = 0; r < 16; ++r) part += resid[tt][nt][r] * hw[r];
          }
        }
        part = sum_halves(part);
        for (int sft = 1; sft < width; sft <<= 1) part += __shfl_xor(part, sft, 64);
        part += p.head[(size_t)p.m * D];
        if (ATTNLIKE) {
          if (lane == 0 && usr[tt] < p.B && (tile % p.tiles_per_user) == 0 && p.q0 == 0) p.logits[usr[tt]] = part;
        } else {
          const int cand = (32 * tile + j) / p.m;
          if (hi == 0 && (j % p.m) == 0 && cand < p.C) p.logits[(size_t)usr[tt] * p.C + cand] = part;
        }
      }
    }
  }
}

// Host-side launcher, one definition per (T, D, DH) instantiation file.  `win` is the
// register window of the in-tile softmax (4, 8 or 16; merge and scoring modes only).
template <typename T, int D, int DH>
int launch_block(int mode, int tt, int win, const BlockParams& p, dim3 grid, hipStream_t stream);

#define LONGER_LAUNCH(T, D, DH, TTV, MODEV, WV) \
  do {                                                                                                \
    constexpr int NWV = kWaves;                                                                       \
    if (p.act == 1 && MODEV != MODE_KVPROJ)                                                           \
      hipLaunchKernelGGL((block_kernel<T, D, DH, TTV, MODEV, WV, MODEV != MODE_KVPROJ, NWV>), grid, dim3(64 * NWV), 0, stream, p); \
    else                                                                                              \
      hipLaunchKernelGGL((block_kernel<T, D, DH, TTV, MODEV, WV, false, NWV>), grid, dim3(64 * NWV), 0, stream, p); \
  } while (0)

// The one-launch stack keeps a user's K/V hand-over area in LDS beside the weight ring; in fp32 at
// d >= 128 the two do not fit, and the layers run one launch pair each (the caller's plan knows:
// stack_in_one_launch in longer_api.hip).
template <typename T, int D>
constexpr bool kHasStackKernel = !(sizeof(T) == 4 && D >= 128);

template <typename T, int D, int DH>
static int launch_stack_mode(const BlockParams& p, dim3 grid, hipStream_t stream) {
  if constexpr (kHasStackKernel<T, D>) {
    LONGER_LAUNCH(T, D, DH, 1, MODE_STACK, 16);
    return 0;
  } else {
    return -1;
  }
}

#define LONGER_INSTANTIATE(T, D, DH)                                                                  \
  template <>                                                                                         \
  int launch_block<T, D, DH>(int mode, int tt, int win, const BlockParams& p, dim3 grid, hipStream_t stream) { \
    if (tt != 1) return -1;                                                                           \
    switch (mode) {                                                                                   \
      case MODE_MERGE:                                                                                \
        if (win == 4) LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE, 4);                                      \
        else if (win == 8) LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE, 8);                                 \
        else LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE, 16);                                              \
        break;                                                                                        \
      case MODE_KVPROJ: LONGER_LAUNCH(T, D, DH, 1, MODE_KVPROJ, 16); break;                           \
      case MODE_ATTN: LONGER_LAUNCH(T, D, DH, 1, MODE_ATTN, 16); break;                               \
      case MODE_STACK: if (launch_stack_mode<T, D, DH>(p, grid, stream)) return -1; break;           \
      case MODE_INPUT: LONGER_LAUNCH(T, D, DH, 1, MODE_INPUT, 16); break;                             \
      case MODE_MERGE_IN:                                                                             \
        if (win == 4) LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE_IN, 4);                                   \
        else if (win == 8) LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE_IN, 8);                              \
        else LONGER_LAUNCH(T, D, DH, 1, MODE_MERGE_IN, 16);                                           \
        break;                                                                                        \
      case MODE_SCORE:                                                                                \
        if (win == 4) LONGER_LAUNCH(T, D, DH, 1, MODE_SCORE, 4);                                      \
        else if (win == 8) LONGER_LAUNCH(T, D, DH, 1, MODE_SCORE, 8);                                 \
        else LONGER_LAUNCH(T, D, DH, 1, MODE_SCORE, 16);                                              \
        break;                                                                                        \
      default: return -1;                                                                             \
    }                                                                                                 \
    return hipGetLastError() == hipSuccess ? 0 : -3;                                                  \
  }

}  // namespace longer
