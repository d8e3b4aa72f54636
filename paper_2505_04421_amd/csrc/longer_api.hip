// C ABI of the library (declared in include/longer.h): argument checks, workspace
// layout, parameter packing and the launch sequence of each entry point.
#include "../../include/longer.h"
#include "pair_kernel.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <initializer_list>
#include <mutex>
#include <cstring>
#include <cstdlib>

namespace longer {

// explicit specialisations defined in the inst_*.hip files
template <> int launch_block<__bf16, 32, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 64, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 128, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 256, 32>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 64, 32>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 128, 32>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<__bf16, 256, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<float, 32, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<float, 64, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_block<float, 128, 16>(int, int, int, const BlockParams&, dim3, hipStream_t);

template <> int launch_pair<128, 16>(int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_pair<128, 32>(int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_pair<256, 16>(int, int, const BlockParams&, dim3, hipStream_t);
template <> int launch_pair<256, 32>(int, int, const BlockParams&, dim3, hipStream_t);

typedef int (*launch_fn)(int, int, int, const BlockParams&, dim3, hipStream_t);
typedef int (*pair_fn)(int, int, const BlockParams&, dim3, hipStream_t);

// The kernels that give a tile to a pair of waves (pair_kernel.h): bf16, d = 128 / 256.  The
// environment variable LONGER_DISABLE_PAIR_KERNELS=1 (read once) keeps every launch on the
// one-wave-per-tile kernels: a measurement aid for comparing the two.
static pair_fn find_pair(int dtype, int D, int DH) {
  static const bool off = [] { const char* e = getenv("LONGER_DISABLE_PAIR_KERNELS"); return e && e[0] == '1'; }();
  if (off || dtype != LONGER_BF16) return nullptr;
  if (D == 128 && DH == 16) return &launch_pair<128, 16>;
  if (D == 128 && DH == 32) return &launch_pair<128, 32>;
  if (D == 256 && DH == 16) return &launch_pair<256, 16>;
  if (D == 256 && DH == 32) return &launch_pair<256, 32>;
  return nullptr;
}

static launch_fn find_launch(int dtype, int D, int DH) {
  if (dtype == LONGER_BF16) {
    if (D == 32 && DH == 16) return &launch_block<__bf16, 32, 16>;
    if (D == 64 && DH == 16) return &launch_block<__bf16, 64, 16>;
    if (D == 128 && DH == 16) return &launch_block<__bf16, 128, 16>;
    if (D == 256 && DH == 32) return &launch_block<__bf16, 256, 32>;
    if (D == 64 && DH == 32) return &launch_block<__bf16, 64, 32>;
    if (D == 128 && DH == 32) return &launch_block<__bf16, 128, 32>;
    if (D == 256 && DH == 16) return &launch_block<__bf16, 256, 16>;
  } else if (dtype == LONGER_F32) {
    if (D == 32 && DH == 16) return &launch_block<float, 32, 16>;
    if (D == 64 && DH == 16) return &launch_block<float, 64, 16>;
    if (D == 128 && DH == 16) return &launch_block<float, 128, 16>;   // every mode but the one-launch stack
  }
  return nullptr;
}

static thread_local char g_err[256] = "";

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// the same for the library's other translation units (backward.hip): sets the thread's message
__attribute__((visibility("hidden"))) int api_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// ------------------------------------------------------------------------------------
// Optional per-stage timing with HIP events on the caller's stream (measurement aid).
enum Stage { ST_PACK = 0, ST_MERGE = 1, ST_KVPROJ = 2, ST_ATTN = 3, ST_SCORE = 4 };
static_assert(LONGER_NUM_STAGES == 5, "stage table");
struct StageTimer {
  static constexpr int kMaxPairs = 4096;
  unsigned mask = 0;             // bit s: stage s is timed
  int n = 0;
  int created = 0;               // events that exist (made pair by pair on first use, never destroyed)
  hipEvent_t ev[2 * kMaxPairs];  // fixed storage: the aid allocates no host memory either
  unsigned char stage[kMaxPairs];
};
static StageTimer g_timer;

struct StageScope {
  hipStream_t st; int idx;
  StageScope(int stage, hipStream_t s) : st(s), idx(-1) {
    if ((g_timer.mask >> stage & 1u) && g_timer.n < StageTimer::kMaxPairs) {
      if (2 * g_timer.n + 2 > g_timer.created) {
        if (hipEventCreate(&g_timer.ev[g_timer.created]) != hipSuccess) return;
        if (hipEventCreate(&g_timer.ev[g_timer.created + 1]) != hipSuccess) { (void)hipEventDestroy(g_timer.ev[g_timer.created]); return; }
        g_timer.created += 2;
      }
      idx = g_timer.n++;
      g_timer.stage[idx] = (unsigned char)stage;
      (void)hipEventRecord(g_timer.ev[2 * idx], st);
    }
  }
  ~StageScope() { if (idx >= 0) (void)hipEventRecord(g_timer.ev[2 * idx + 1], st); }
};

// ------------------------------------------------------------------------------------
// Pack kernel: raw [in, out] matrices of one block -> MFMA A/B fragments in the order
// the block kernels stream them (see PackLayout in device.h), the small vectors as fp32.
struct RawBlock { longer_block b; };

// One launch packs up to kMaxPackJobs blocks: blockIdx.y picks the job.
constexpr int kMaxPackJobs = 16;
constexpr int kLayoutHead = 2;     // a job that converts the head's weights instead of packing a block
struct PackJob { RawBlock raw; char* dst; int layout; int pad_; };
struct PackArgs { PackJob job[kMaxPackJobs]; };

template <typename T>
__global__ void pack_block_kernel(const PackArgs args, int D, int FF) {
  using E = ET<T>;
  // the job is picked with compile-time offsets into the kernel arguments and scalar selects
  // (a run-time index made the compiler select between addresses inside the argument block,
  // and the O-projection segment came out wrong)
  PackJob jb = args.job[0];
#pragma unroll
  for (int i = 1; i < kMaxPackJobs; ++i)
    if ((int)blockIdx.y == i) jb = args.job[i];
  const RawBlock& raw = jb.raw;
  char* dst = jb.dst;
  const int layout = jb.layout;
  if (layout == kLayoutHead) {   // the scoring head: pad_ weights (ln1_g) then the bias (ln1_b), as fp32
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < jb.pad_) reinterpret_cast<float*>(dst)[i] = (float)reinterpret_cast<const T*>(raw.b.ln1_g)[i];
    else if (i == jb.pad_) reinterpret_cast<float*>(dst)[i] = (float)reinterpret_cast<const T*>(raw.b.ln1_b)[0];
    return;
  }
  const int NT = D / 32, NC = FF / 32, NG = D / E::GF, SEGV = NG * 64;
  const int nseg = (layout == LAYOUT_FUSED || layout == LAYOUT_PAIR_FUSED) ? fused_segs(D, FF)
                 : layout == LAYOUT_MLP ? mlp_segs(FF) : layout == LAYOUT_PAIR_ATTN ? attn_segs(D, FF) : kv_segs(D) + attn_segs(D, FF);
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)nseg * SEGV) return;
  int seg = (int)(idx / SEGV);
  const int within = (int)(idx - (long long)seg * SEGV);
  // decode the destination segment: kind 0 vec, 1 q, 2 k, 3 v, 4 o, 5 w1, 6 w2, 7 unused; tile/chunk index
  int kind, ti;
  const bool skewed = ffn_skewed((int)sizeof(T), D);
  if (layout == LAYOUT_PAIR_FUSED || layout == LAYOUT_PAIR_ATTN) {     // two-wave kernels (device.h)
    const int nqkv = layout == LAYOUT_PAIR_FUSED ? 3 * NT : NT;
    const int q = seg - 2;
    if (seg == 0) { kind = 0; ti = 0; }
    else if (seg == 1) { kind = 7; ti = 0; }
    else if (q < nqkv) {
      if (layout == LAYOUT_PAIR_FUSED) { kind = 1 + (q % 6) / 2; ti = 2 * (q / 6) + (q & 1); }
      else { kind = 1; ti = q; }
    } else if (q < nqkv + NT) { kind = 4; ti = q - nqkv; }
    else { const int f = q - nqkv - NT; kind = 5 + (f % 4) / 2; ti = 2 * (f / 4) + (f & 1); }
  } else if (layout == LAYOUT_MLP) {          // the input-generation MLP: biases, then the FFN part
    if (seg == 0) { kind = 0; ti = 0; }
    else ffn_seg_decode(seg - 1, NC, skewed, kind, ti);
  } else if (layout == LAYOUT_FUSED) {
    if (seg == 0) { kind = 0; ti = 0; }
    else if (seg <= 3 * NT) { kind = 1 + (seg - 1) % 3; ti = (seg - 1) / 3; }
    else if (seg <= 4 * NT) { kind = 4; ti = seg - 1 - 3 * NT; }
    else ffn_seg_decode(seg - 1 - 4 * NT, NC, skewed, kind, ti);
  } else {
    if (seg < kv_segs(D)) {
      if (seg == 0) { kind = 0; ti = 0; }
      else { kind = 2 + ((seg - 1) & 1); ti = (seg - 1) >> 1; }
    } else {
      seg -= kv_segs(D);
      if (seg == 0) { kind = 0; ti = 0; }
      else if (seg <= NT) { kind = 1; ti = seg - 1; }
      else if (seg <= 2 * NT) { kind = 4; ti = seg - 1 - NT; }
      else ffn_seg_decode(seg - 1 - 2 * NT, NC, skewed, kind, ti);
    }
  }
  if (kind == 7) {                     // the unused segment of the FFN part
    reinterpret_cast<uint4*>(dst)[idx] = make_uint4(0u, 0u, 0u, 0u);
    return;
  }
  if (kind == 0 && layout == LAYOUT_MLP) {
    const VecLayout vl{D, FF};
    f32x4 out;
    for (int e = 0; e < 4; ++e) {
      const int i = within * 4 + e;
      float v = 0.f;
      if (i >= vl.b2() && i < vl.b1()) v = (float)((const T*)raw.b.b2)[i - vl.b2()];
      else if (i >= vl.b1() && i < vl.total()) v = (float)((const T*)raw.b.b1)[i - vl.b1()] * (E::HALF_FFN ? 1.0f / kFfnScale : 1.0f);
      out[e] = v;
    }
    reinterpret_cast<f32x4*>(dst)[idx] = out;
    return;
  }
  if (kind == 0) {
    const VecLayout vl{D, FF};
    f32x4 out;
    for (int e = 0; e < 4; ++e) {
      const int i = within * 4 + e;
      float v = 0.f;
      if (i < vl.total()) {
        const T* src;
        int off;
        if (i < vl.ln1_b()) { src = (const T*)raw.b.ln1_g; off = i; }
        else if (i < vl.bq()) { src = (const T*)raw.b.ln1_b; off = i - vl.ln1_b(); }
        else if (i < vl.bk()) { src = (const T*)raw.b.bq; off = i - vl.bq(); }
        else if (i < vl.bv()) { src = (const T*)raw.b.bk; off = i - vl.bk(); }
        else if (i < vl.bo()) { src = (const T*)raw.b.bv; off = i - vl.bv(); }
        else if (i < vl.ln2_g()) { src = (const T*)raw.b.bo; off = i - vl.bo(); }   // replaced below
        else if (i < vl.ln2_b()) { src = (const T*)raw.b.ln2_g; off = i - vl.ln2_g(); }
        else if (i < vl.b2()) { src = (const T*)raw.b.ln2_b; off = i - vl.ln2_b(); }
        else if (i < vl.b1()) { src = (const T*)raw.b.b2; off = i - vl.b2(); }
        else { src = (const T*)raw.b.b1; off = i - vl.b1(); }
        v = (float)src[off];
        if (E::HALF_FFN && i >= vl.b1()) v *= 1.0f / kFfnScale;     // the hidden pre-activation is kept as x / kFfnScale
      }
      out[e] = v;
    }
    // (the output bias slot is written by the fold below, possibly from another workgroup)
    if (within * 4 < vl.bo() || within * 4 >= vl.ln2_g()) reinterpret_cast<f32x4*>(dst)[idx] = out;
    // The block kernels apply no value bias: softmax rows sum to 1, so
    //   softmax(.)(V + 1 b_V^T) W_O + b_O = softmax(.) V W_O + (b_V W_O + b_O),
    // and the output bias slot gets b_O + b_V W_O.  (The key bias only adds a per-query
    // constant to the scores, which softmax drops.)  A workgroup folds 64 outputs: wave kp
    // sums a quarter of the rows of W_O (coalesced along the row), LDS adds the four up.
    // All threads of a workgroup belong to the same segment (the launch uses workgroups no
    // larger than a segment), so the barrier is uniform.
    __shared__ float red[4][64];
    const int nw = (int)blockDim.x >> 6;           // waves that split the rows: 4, or 2 for bf16 at d = 32
    const int wg_in_seg = within / (int)blockDim.x;
    if (wg_in_seg < (D + 63) / 64) {
      const int t = threadIdx.x, o = 64 * wg_in_seg + (t & 63), kp = t >> 6;
      float acc = 0.f;
      if (o < D) {
        const T* bvp = (const T*)raw.b.bv + kp * (D / nw);
        const T* wop = (const T*)raw.b.wo + (size_t)kp * (D / nw) * D + o;
#pragma unroll 8
        for (int k = 0; k < D / nw; ++k) acc += (float)bvp[k] * (float)wop[(size_t)k * D];
      }
      red[kp][t & 63] = acc;
      __syncthreads();
      if (kp == 0 && o < D) {
        float sum = red[0][t];
        for (int i = 1; i < nw; ++i) sum += red[i][t];
        reinterpret_cast<float*>(dst)[(idx - within) * 4 + vl.bo() + o] = (float)((const T*)raw.b.bo)[o] + sum;
      }
    }
    return;
  }
  const int f = within / 64, lane = within % 64, n_in = lane & 31, hi = lane >> 5;
  const T* W;
  int ncols, nt, sg;
  if (kind <= 4) {
    W = reinterpret_cast<const T*>(kind == 1 ? raw.b.wq : kind == 2 ? raw.b.wk : kind == 3 ? raw.b.wv : raw.b.wo);
    ncols = D; nt = ti; sg = f;
  } else if (kind == 5) {
    W = reinterpret_cast<const T*>(raw.b.w1); ncols = FF; nt = ti; sg = f;
  } else {
    W = reinterpret_cast<const T*>(raw.b.w2); ncols = D; nt = f / E::GPT; sg = ti * E::GPT + (f % E::GPT);
  }
  const int t = sg / E::GPT, g = sg % E::GPT;
  typename E::grp out;
  typename E::hgrp outh;
  for (int e = 0; e < E::EPL; ++e) {
    const int k = 32 * t + tile_row(E::EPL * g + e, hi);
    const T w = W[(size_t)k * ncols + 32 * nt + n_in];
    out[e] = w;
    if constexpr (E::HALF_FFN) {
      // bf16 mode: W1 / kFfnScale (exact), W2 * kFfnScale as fp16 (exact for 1.6e-5 <= |w| < 16376;
      // smaller weights lose low bits as fp16 subnormals, larger ones saturate)
      if (kind == 5) out[e] = (T)((float)w * (1.0f / kFfnScale));
      outh[e] = (_Float16)fminf(fmaxf((float)w * kFfnScale, -65504.f), 65504.f);
    }
  }
  if constexpr (E::HALF_FFN) {
    if (kind == 6) out = __builtin_bit_cast(typename E::grp, outh);
  }
  reinterpret_cast<typename E::grp*>(dst)[idx] = out;
}

__global__ void probe_kernel(int32_t* out) {
  const int lane = threadIdx.x & 63, j = lane & 31, hi = lane >> 5;
  // one contraction slot (hi = 0, element 0) carries a value, all others are zero
  bf16x8 a_row = {0, 0, 0, 0, 0, 0, 0, 0}, a_one = a_row, b_col = a_row, b_one = a_row;
  if (hi == 0) { a_row[0] = (__bf16)(float)j; a_one[0] = (__bf16)1.0f; b_col[0] = (__bf16)(float)j; b_one[0] = (__bf16)1.0f; }
  f32x16 z = splat16(0.f);
  f32x16 rows = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_row, b_one, z, 0, 0, 0);
  f32x16 cols = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_one, b_col, z, 0, 0, 0);
  for (int r = 0; r < 16; ++r) out[lane * 16 + r] = (int)rows[r] * 32 + (int)cols[r];
  const float fa_row = hi == 0 ? (float)j : 0.f, f_one = hi == 0 ? 1.f : 0.f;
  rows = __builtin_amdgcn_mfma_f32_32x32x2f32(fa_row, f_one, z, 0, 0, 0);
  cols = __builtin_amdgcn_mfma_f32_32x32x2f32(f_one, fa_row, z, 0, 0, 0);
  for (int r = 0; r < 16; ++r) out[1024 + lane * 16 + r] = (int)rows[r] * 32 + (int)cols[r];
}

// ------------------------------------------------------------------------------------
struct Shape {
  int D, DH, DHi, FF, es, n, NT, GPT;
  int Di;             // width of the raw tokens and the InnerTrans blocks (D, or D / K for a concat merge)
  size_t pb;          // bytes reserved per packed block (either layout)
  size_t seg;         // bytes of one stream segment
  launch_fn main_fn, inner_fn;
  pair_fn pair;       // the main stack's two-wave kernels, or NULL
};

static int check_cfg(const longer_config* c, Shape* s, bool need_inner, bool need_main) {
  if (!c) return fail(LONGER_ERR_ARG, "config is NULL");
  if (c->dtype != LONGER_F32 && c->dtype != LONGER_BF16) return fail(LONGER_ERR_ARG, "dtype %d unknown", c->dtype);
  if (c->act != LONGER_ACT_GELU_ERF && c->act != LONGER_ACT_RELU) return fail(LONGER_ERR_ARG, "act %d unknown", c->act);
  if (c->gmask != LONGER_GMASK_FULL && c->gmask != LONGER_GMASK_CAUSAL) return fail(LONGER_ERR_ARG, "gmask %d unknown", c->gmask);
  if (c->merge != LONGER_MERGE_MEAN && c->merge != LONGER_MERGE_CONCAT) return fail(LONGER_ERR_ARG, "merge %d unknown", c->merge);
  if (c->d <= 0 || c->d % 32) return fail(LONGER_ERR_ARG, "d=%d must be a positive multiple of 32", c->d);
  if (c->ffn_mult <= 0) return fail(LONGER_ERR_ARG, "ffn_mult=%d", c->ffn_mult);
  if (!(c->ln_eps > 0.f)) return fail(LONGER_ERR_ARG, "ln_eps must be positive");
  if (c->K <= 0 || 32 % c->K) return fail(LONGER_ERR_ARG, "K=%d must divide 32", c->K);
  if (c->m <= 0 || 32 % c->m) return fail(LONGER_ERR_ARG, "m=%d must divide 32", c->m);
  if (c->k_recent <= 0) return fail(LONGER_ERR_ARG, "k_recent=%d", c->k_recent);
  if (c->k_uniform < 0 || c->k_uniform > c->k_recent) return fail(LONGER_ERR_ARG, "k_uniform=%d must lie in [0, k_recent]", c->k_uniform);
  if (c->q_learn && c->k_uniform) return fail(LONGER_ERR_ARG, "learnable query tokens exclude k_uniform=%d", c->k_uniform);
  if (((uintptr_t)c->q_learn & 15) != 0) return fail(LONGER_ERR_ARG, "q_learn must be 16-byte aligned");
  if (c->n_self < 0 || c->inner_layers < 0 || c->n_self + c->inner_layers + 1 > 32)
    return fail(LONGER_ERR_ARG, "layer counts out of range");
  s->D = c->d; s->FF = c->ffn_mult * c->d; s->es = c->dtype == LONGER_BF16 ? 2 : 4;
  s->n = c->m + c->k_recent; s->NT = c->d / 32; s->GPT = c->dtype == LONGER_BF16 ? 2 : 4;
  s->pb = packed_block_bytes(s->D, s->FF, s->es);
  s->seg = packed_seg_bytes(s->D, s->es);
  if ((size_t)(9 * s->D + s->FF) * 4 > s->seg) return fail(LONGER_ERR_ARG, "ffn_mult=%d too large for d=%d", c->ffn_mult, c->d);
  if (ffn_skewed(s->es, s->D) && s->FF < 64) return fail(LONGER_ERR_ARG, "ffn_mult * d = %d: the bf16 FFN needs a hidden width of at least 64", s->FF);
  s->main_fn = s->inner_fn = nullptr; s->pair = nullptr; s->DH = s->DHi = 0;
  s->Di = c->d;
  if (c->merge == LONGER_MERGE_CONCAT) {
    if (c->d % c->K || (c->d / c->K) % 32)
      return fail(LONGER_ERR_ARG, "concat merge: d / K = %d / %d must be a multiple of 32", c->d, c->K);
    s->Di = c->d / c->K;
  }
  if (need_main) {
    if (c->heads <= 0 || c->d % c->heads) return fail(LONGER_ERR_ARG, "heads=%d does not divide d=%d", c->heads, c->d);
    s->DH = c->d / c->heads;
    s->main_fn = find_launch(c->dtype, c->d, s->DH);
    if (!s->main_fn) return fail(LONGER_ERR_ARG, "unsupported shape: dtype=%d d=%d head width=%d", c->dtype, c->d, s->DH);
    s->pair = find_pair(c->dtype, c->d, s->DH);
  }
  if (need_inner) {
    if (c->inner_layers < 1) return fail(LONGER_ERR_ARG, "inner_layers=%d", c->inner_layers);
    if (c->inner_heads <= 0 || s->Di % c->inner_heads) return fail(LONGER_ERR_ARG, "inner_heads=%d does not divide the InnerTrans width %d", c->inner_heads, s->Di);
    s->DHi = s->Di / c->inner_heads;
    s->inner_fn = find_launch(c->dtype, s->Di, s->DHi);
    if (!s->inner_fn) return fail(LONGER_ERR_ARG, "unsupported shape: dtype=%d InnerTrans width=%d inner head width=%d", c->dtype, s->Di, s->DHi);
    if ((size_t)(9 * s->Di + c->ffn_mult * s->Di) * 4 > packed_seg_bytes(s->Di, s->es))
      return fail(LONGER_ERR_ARG, "ffn_mult=%d too large for the InnerTrans width %d", c->ffn_mult, s->Di);
    if (ffn_skewed(s->es, s->Di) && c->ffn_mult * s->Di < 64)
      return fail(LONGER_ERR_ARG, "ffn_mult * InnerTrans width = %d: the bf16 FFN needs a hidden width of at least 64", c->ffn_mult * s->Di);
  }
  return 0;
}

// the same shape record seen from the InnerTrans side: its width, FFN width and segment size
static Shape inner_view(const longer_config* c, const Shape& s) {
  Shape si = s;
  si.D = s.Di; si.FF = c->ffn_mult * s.Di; si.NT = s.Di / 32;
  si.pb = packed_block_bytes(si.D, si.FF, s.es);
  si.seg = packed_seg_bytes(si.D, s.es);
  si.main_fn = nullptr;
  return si;
}

static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// MI355X: 8 accelerator dies (XCDs) of 32 compute units, each with its own L2; workgroups of a
// launch are dealt to them round-robin
constexpr int kXcds = 8;

// Packed parameters of a whole model, in the order the launches stream them.  The layout is a
// function of the configuration alone, so a buffer written once by longer_pack_weights serves
// every later call; without one, each entry point packs what it needs into the same places of
// its workspace.
//   merge stream   [input MLP][InnerTrans blocks, fused layout, back to back]
//   reduced stack  [cross block, split layout]([its attention half, pair layout])[self blocks, fused layout, back to back]
//                  (one stream: the stack kernel; the two-wave stack kernel starts at the pair copy and
//                  its self blocks are in the pair layout)
//   per-layer plan [self blocks, split layout]                              (m + k > 128, cache build)
//   scoring        [cross block, fused][self blocks, fused], back to back
//   head           fp32 weights and bias
struct PackedLayout {
  size_t mlp, inner, cross, cross_pair, self_fused, self_split, score, head, total;
  size_t inner_stride, score_stride;
};

// a user's reduced rows fit one workgroup, and the stack kernel exists for the shape (block_kernel.h: kHasStackKernel)
static bool stack_in_one_launch(const Shape& s) { return s.n <= 32 * kWaves && !(s.es == 4 && s.D >= 128); }
// which launches run on the two-wave kernels (their parts of the packed parameters are in the pair layouts)
static bool pair_stack(const Shape& s) { return s.pair && s.D == 128 && stack_in_one_launch(s); }   // (LDS: the K/V hand-over area fits at d = 128)
static bool pair_score(const Shape& s) { return s.pair != nullptr; }

static PackedLayout packed_layout(const longer_config* c, const Shape& s) {
  PackedLayout pl;
  const Shape si = inner_view(c, s);
  size_t o = 0;
  pl.mlp = o; o += (size_t)mlp_segs(s.FF) * s.seg;
  pl.inner = o; pl.inner_stride = (size_t)fused_segs(si.D, si.FF) * si.seg;
  o += (size_t)c->inner_layers * pl.inner_stride;
  o = align256(o + 4 * (s.seg > si.seg ? s.seg : si.seg));   // a stream may read whole panels past its end
  pl.score_stride = (size_t)fused_segs(s.D, s.FF) * s.seg;
  pl.cross = o; o += s.pb;                                  // the split layout fills its slot exactly:
  // (two-wave stack kernel: a copy of the cross block's attention half in the pair layout heads the stream)
  pl.cross_pair = o; if (pair_stack(s)) o += (size_t)attn_segs(s.D, s.FF) * s.seg;
  pl.self_fused = o; o += (size_t)c->n_self * pl.score_stride;   // the stack kernel's stream runs on into these
  pl.self_split = o; o += (size_t)c->n_self * s.pb;
  pl.score = o;
  o += (size_t)(1 + c->n_self) * pl.score_stride + 4 * s.seg;
  pl.head = align256(o); o = pl.head + align256(((size_t)c->m * s.D + 1) * 4);
  pl.total = o;
  return pl;
}

// workspace layout shared by all entry points
struct Layout {
  size_t packed, M, kst, vst, xa, xb, total;
  size_t kv_ustride;
  int ktmax;
};

static Layout make_layout(const longer_config* c, const Shape& s, int B, int L) {
  Layout l;
  const int T = cdiv(L, c->K);
  size_t o = 0;
  l.packed = o; o += packed_layout(c, s).total;
  l.M = o; o += align256((size_t)B * T * s.D * 4);
  l.ktmax = cdiv((long long)c->m + T, 32) > cdiv(s.n, 32) ? cdiv((long long)c->m + T, 32) : cdiv(s.n, 32);
  l.kv_ustride = (size_t)l.ktmax * s.NT * s.GPT * 1024;
  l.kst = o; o += (size_t)B * l.kv_ustride;
  l.vst = o; o += (size_t)B * l.kv_ustride;
  l.xa = o; o += align256((size_t)B * s.n * s.D * 4);
  l.xb = o; o += align256((size_t)B * s.n * s.D * 4);
  l.total = o;
  return l;
}

struct CacheLayout {
  int kt0, kt1;
  size_t c0_ustride, c0_voff, c1_off, c1_lstride, c1_ustride, c1_voff, total;
};

static CacheLayout make_cache_layout(const longer_config* c, const Shape& s, int U, int L) {
  CacheLayout cl;
  const int T = cdiv(L, c->K);
  cl.kt0 = cdiv(T, 32); cl.kt1 = cdiv(c->k_recent, 32);
  const size_t tile = (size_t)s.NT * s.GPT * 1024;
  cl.c0_voff = (size_t)cl.kt0 * tile; cl.c0_ustride = 2 * cl.c0_voff;
  cl.c1_off = (size_t)U * cl.c0_ustride;
  cl.c1_voff = (size_t)cl.kt1 * tile; cl.c1_ustride = 2 * cl.c1_voff;
  cl.c1_lstride = (size_t)U * cl.c1_ustride;
  cl.total = cl.c1_off + (size_t)c->n_self * cl.c1_lstride;
  return cl;
}

// Collects the blocks an entry point has to pack and packs them with one launch (per
// kMaxPackJobs blocks) when flushed.
struct PackBatch {
  const longer_config* c; const Shape& s; hipStream_t st;
  PackArgs a; int n = 0;
  PackBatch(const longer_config* c_, const Shape& s_, hipStream_t st_) : c(c_), s(s_), st(st_) { memset(&a, 0, sizeof(a)); }
  int add(const longer_block* blocks, int nb, int layout, char* dst, size_t stride) {
    for (int i = 0; i < nb; ++i) {
      const longer_block& b = blocks[i];
      const void* ptrs[16] = {b.ln1_g, b.ln1_b, b.wq, b.bq, b.wk, b.bk, b.wv, b.bv, b.wo, b.bo, b.ln2_g, b.ln2_b, b.w1, b.b1, b.w2, b.b2};
      for (int j = 0; j < 16; ++j)
        if (!ptrs[j]) return fail(LONGER_ERR_ARG, "block %d: parameter pointer %d is NULL", i, j);
      if (n == kMaxPackJobs) { int rc = flush(); if (rc) return rc; }
      a.job[n].raw.b = b; a.job[n].dst = dst + (size_t)i * stride; a.job[n].layout = layout;
      ++n;
    }
    return 0;
  }
  int add_head(const longer_weights* w, float* dst) {
    if (!w->head_w || !w->head_b) return fail(LONGER_ERR_ARG, "head_w / head_b is NULL but logits were asked for");
    if (n == kMaxPackJobs) { int rc = flush(); if (rc) return rc; }
    a.job[n].raw.b.ln1_g = w->head_w; a.job[n].raw.b.ln1_b = w->head_b;
    a.job[n].dst = (char*)dst; a.job[n].layout = kLayoutHead; a.job[n].pad_ = c->m * s.D;
    ++n;
    return 0;
  }
  // the two-layer MLP of the input-generation stage (weights [d, f], [f, d] and their biases)
  int add_mlp(const void* w1, const void* b1, const void* w2, const void* b2, void* dst) {
    if (!w1 || !b1 || !w2 || !b2) return fail(LONGER_ERR_ARG, "input MLP has NULL members");
    if (n == kMaxPackJobs) { int rc = flush(); if (rc) return rc; }
    memset(&a.job[n], 0, sizeof(a.job[n]));
    a.job[n].raw.b.w1 = w1; a.job[n].raw.b.b1 = b1; a.job[n].raw.b.w2 = w2; a.job[n].raw.b.b2 = b2;
    a.job[n].dst = (char*)dst; a.job[n].layout = LAYOUT_MLP;
    ++n;
    return 0;
  }
  int flush() {
    if (n == 0) return 0;
    StageScope scope(ST_PACK, st);
    // the split layout has the most segments; threads past a job's own count return at once
    const long long items = (long long)(kv_segs(s.D) + attn_segs(s.D, s.FF)) * (long long)(s.seg / 16);
    // a workgroup never straddles two segments (its bias fold has a barrier): 256 threads, or the
    // 128 sixteen-byte items of a bf16 segment at d = 32
    const int threads = s.seg / 16 < 256 ? (int)(s.seg / 16) : 256;
    const dim3 grid(cdiv(items, threads), n);
    if (c->dtype == LONGER_BF16) hipLaunchKernelGGL(pack_block_kernel<__bf16>, grid, dim3(threads), 0, st, a, s.D, s.FF);
    else hipLaunchKernelGGL(pack_block_kernel<float>, grid, dim3(threads), 0, st, a, s.D, s.FF);
    n = 0;
    return hipGetLastError() == hipSuccess ? 0 : fail(LONGER_ERR_HIP, "pack kernel launch failed");
  }
};

static BlockParams base_params(const longer_config* c, const Shape& s, const int32_t* lens, int B, int L, int DH) {
  BlockParams p;
  memset(&p, 0, sizeof(p));
  p.n_layers = 1; p.FF = s.FF; p.eps = c->ln_eps;
  p.scale_l2e = (float)(1.4426950408889634 / std::sqrt((double)DH));
  p.act = c->act; p.gmask_causal = c->gmask == LONGER_GMASK_CAUSAL;
  p.lens = lens; p.B = B; p.L = L; p.K = c->K; p.T = cdiv(L, c->K); p.m = c->m; p.k = c->k_recent; p.k_uni = c->k_uniform;
  p.q_learn = c->q_learn != nullptr;
  return p;
}

// rows are read and written with 8- and 16-byte vector accesses
static int check_aligned(std::initializer_list<const void*> ptrs) {
  for (const void* q : ptrs)
    if (((uintptr_t)q & 15) != 0) return fail(LONGER_ERR_ARG, "tensor pointers must be 16-byte aligned");
  return 0;
}

static int check_common(const void* ws, size_t ws_bytes, size_t need, int B, int L) {
  if (B <= 0 || L <= 0) return fail(LONGER_ERR_ARG, "B=%d, L=%d must be positive", B, L);
  if (!ws) return fail(LONGER_ERR_ARG, "workspace is NULL");
  if (((uintptr_t)ws & 255) != 0) return fail(LONGER_ERR_ARG, "workspace must be 256-byte aligned");
  if (ws_bytes < need) return fail(LONGER_ERR_WS, "workspace too small: %zu < %zu bytes", ws_bytes, need);
  return 0;
}

// the merge kernel numbers its token slots (B * ceil(L / K) * K, rounded up to whole workgroups) in 32 bits
static int check_slots(const longer_config* c, int B, int L) {
  const long long slots = (long long)B * cdiv(L, c->K) * c->K;
  if (slots + 32LL * 8 >= (1LL << 31))
    return fail(LONGER_ERR_ARG, "B*ceil(L/K)*K = %lld token slots: at most 2^31 per call", slots);
  return 0;
}

// -- stage launchers (packed parameters already in place) -----------------------------
// Raw inputs of the input-generation stage when it runs inside the merge kernel
struct MergeInput { const longer_input_weights* w; const void* E; const void* tdiff; int d_e; };

static int check_input(const longer_config* cfg, const longer_input_weights* w, const void* E, const void* tdiff, int d_e) {
  if (!w || !w->pos || !E || !tdiff) return fail(LONGER_ERR_ARG, "NULL argument");
  if (d_e <= 0 || d_e >= cfg->d || d_e % 32)
    return fail(LONGER_ERR_ARG, "d_e=%d must be a multiple of 32 below d=%d (the rest is the time-difference width)", d_e, cfg->d);
  return check_aligned({E, tdiff, w->pos});
}

// `packed`: the InnerTrans blocks in the fused layout; with `in`, the input MLP's segments
// followed directly by them, and the rows come from the raw inputs instead of H
static int run_merge(const longer_config* c, const Shape& s, const char* packed, const void* H, const int32_t* lens,
                     int B, int L, void* M_out, int M_f32, void* Z_out, int Z_f32, hipStream_t st,
                     const MergeInput* in = nullptr) {
  BlockParams p = base_params(c, s, lens, B, L, s.DHi);
  p.wbase = packed; p.n_layers = c->inner_layers;
  p.H = H; p.M_out = M_out; p.M_f32 = M_f32; p.Z_out = Z_out; p.Z_f32 = Z_f32;
  if (in) {
    p.in_e = in->E; p.in_pos = in->w->pos; p.in_td = in->tdiff; p.de = in->d_e;
    p.n_layers = c->inner_layers + 1;
  }
  const int tt = 1;
  const int win = c->K <= 8 ? 4 : (c->K <= 16 ? 8 : 16);
  const long long slots = (long long)B * p.T * c->K;
  if (slots + 32LL * tt * kWaves >= (1LL << 31)) return fail(LONGER_ERR_ARG, "B*ceil(L/K)*K = %lld token slots: at most 2^31 per call", slots);
  const int grid = cdiv(slots, 32LL * tt * kWaves);
  StageScope scope(ST_MERGE, st);
  int rc = s.inner_fn(in ? MODE_MERGE_IN : MODE_MERGE, tt, win, p, dim3(grid), st);
  return rc ? fail(LONGER_ERR_HIP, "merge kernel launch failed") : 0;
}

struct AttnIO {
  RowSrc src0, src1;     // rows of a user: [0, m0) from src0, rest from src1
  int m0;
  int key_rows;          // rows projected to K/V per user
  int KG, key_self, gather_recent, q0, q_rows;
  char* kst; char* vst; size_t kv_ustride;
  RowSrc q0src, q1src;   // query rows: globals from q0src, slots from q1src
  void* X_out; int X_f32; long long X_ustride;
  float* logits; const float* head;
};

static int run_layer(const longer_config* c, const Shape& s, const char* packed_blk, const int32_t* lens, int B, int L,
                     const AttnIO& io, bool do_attn, hipStream_t st) {
  {
    BlockParams p = base_params(c, s, lens, B, L, s.DH);
    p.wbase = packed_blk;
    p.src0 = io.src0; p.src1 = io.src1; p.m0 = io.m0;
    p.rows_per_user = io.key_rows; p.tiles_per_user = cdiv(io.key_rows, 32);
    p.kst = io.kst; p.vst = io.vst; p.kv_ustride = io.kv_ustride; p.kt_per_user = p.tiles_per_user;
    p.key_self = io.key_self;
    const int grid = cdiv((long long)B * p.tiles_per_user, kWaves);
    StageScope scope(ST_KVPROJ, st);
    if (s.main_fn(MODE_KVPROJ, 1, 16, p, dim3(grid), st)) return fail(LONGER_ERR_HIP, "kv projection launch failed");
  }
  if (!do_attn) return 0;
  BlockParams p = base_params(c, s, lens, B, L, s.DH);
  p.wbase = packed_blk + (size_t)kv_segs(s.D) * s.seg;     // the attention sub-stream follows the K/V one
  p.src0 = io.q0src; p.src1 = io.q1src;
  p.rows_per_user = io.q_rows; p.tiles_per_user = cdiv(io.q_rows, 32);
  p.gather_recent = io.gather_recent; p.q0 = io.q0;
  p.kst = io.kst; p.vst = io.vst; p.kv_ustride = io.kv_ustride;
  p.KG = io.KG; p.key_self = io.key_self;
  p.X_out = io.X_out; p.X_f32 = io.X_f32; p.X_ustride = io.X_ustride;
  p.logits = io.logits; p.head = io.head;
  const int grid = cdiv((long long)B * p.tiles_per_user, kWaves);
  StageScope scope(ST_ATTN, st);
  if (s.main_fn(MODE_ATTN, 1, 16, p, dim3(grid), st)) return fail(LONGER_ERR_HIP, "attention launch failed");
  return 0;
}

// The reduced stack of every user in one launch (one workgroup per user): the query side of
// the cross layer over the K/V fragments that run_layer(.., do_attn = false) stored, then
// all self layers.  `packed_cross` holds the cross block in the split layout, followed directly
// by the self blocks in the fused layout, back to back.  Needs m + k <= 128.
static int run_stack(const longer_config* c, const Shape& s, const char* packed_cross, const char* packed_pair,
                     const int32_t* lens, int B, int L, const AttnIO& io, hipStream_t st) {
  BlockParams p = base_params(c, s, lens, B, L, s.DH);
  p.wbase = pair_stack(s) ? packed_pair : packed_cross + (size_t)kv_segs(s.D) * s.seg;
  p.n_layers = 1 + c->n_self;
  p.src0 = io.q0src; p.src1 = io.q1src;
  p.rows_per_user = s.n; p.tiles_per_user = kWaves;
  p.gather_recent = io.gather_recent; p.q0 = 0;
  p.kst = io.kst; p.vst = io.vst; p.kv_ustride = io.kv_ustride;
  p.KG = io.KG; p.key_self = 0;
  p.X_out = io.X_out; p.X_f32 = io.X_f32; p.X_ustride = io.X_ustride;
  p.logits = io.logits; p.head = io.head;
  StageScope scope(ST_ATTN, st);
  if (pair_stack(s) ? s.pair(MODE_STACK, 16, p, dim3(B), st) : s.main_fn(MODE_STACK, 1, 16, p, dim3(B), st))
    return fail(LONGER_ERR_HIP, "stack launch failed");
  return 0;
}


// ------------------------------------------------------------------------------------
// Packing a model's parameters: which parts an entry point streams
enum : unsigned { PK_MERGE = 1, PK_STACK = 2, PK_LAYERS = 4, PK_SCORE = 8, PK_HEAD = 16 };

static int pack_model(const longer_config* cfg, const Shape& s, const longer_weights* w, const longer_input_weights* iw,
                      char* base, unsigned what, hipStream_t st) {
  const PackedLayout pl = packed_layout(cfg, s);
  const Shape si = inner_view(cfg, s);
  PackBatch pk_main(cfg, s, st);
  int rc;
  if (what & PK_MERGE) {
    if (!w->inner) return fail(LONGER_ERR_ARG, "weights struct has NULL members");
    if (iw && (rc = pk_main.add_mlp(iw->w1, iw->b1, iw->w2, iw->b2, base + pl.mlp))) return rc;
    // InnerTrans blocks of another width than the main stack's are packed by a launch of their own
    PackBatch pk_inner(cfg, si, st);
    PackBatch& pb = cfg->merge == LONGER_MERGE_CONCAT ? pk_inner : pk_main;
    if ((rc = pb.add(w->inner, cfg->inner_layers, LAYOUT_FUSED, base + pl.inner, pl.inner_stride))) return rc;
    if ((rc = pk_inner.flush())) return rc;
  }
  if (what & (PK_STACK | PK_LAYERS | PK_SCORE)) {
    if (!w->cross || (cfg->n_self > 0 && !w->self)) return fail(LONGER_ERR_ARG, "weights struct has NULL members");
  }
  if ((what & (PK_STACK | PK_LAYERS)) && (rc = pk_main.add(w->cross, 1, LAYOUT_SPLIT, base + pl.cross, s.pb))) return rc;
  if ((what & PK_STACK) && pair_stack(s) && (rc = pk_main.add(w->cross, 1, LAYOUT_PAIR_ATTN, base + pl.cross_pair, s.pb))) return rc;
  if ((what & PK_STACK) && cfg->n_self &&
      (rc = pk_main.add(w->self, cfg->n_self, pair_stack(s) ? LAYOUT_PAIR_FUSED : LAYOUT_FUSED, base + pl.self_fused, pl.score_stride))) return rc;
  if ((what & PK_LAYERS) && cfg->n_self && (rc = pk_main.add(w->self, cfg->n_self, LAYOUT_SPLIT, base + pl.self_split, s.pb))) return rc;
  if (what & PK_SCORE) {
    const int lay = pair_score(s) ? LAYOUT_PAIR_FUSED : LAYOUT_FUSED;
    if ((rc = pk_main.add(w->cross, 1, lay, base + pl.score, pl.score_stride))) return rc;
    if (cfg->n_self && (rc = pk_main.add(w->self, cfg->n_self, lay, base + pl.score + pl.score_stride, pl.score_stride))) return rc;
  }
  if ((what & PK_HEAD) && (rc = pk_main.add_head(w, (float*)(base + pl.head)))) return rc;
  return pk_main.flush();
}

// Where a call streams its parameters from: the caller's pre-packed buffer, or the workspace's
// packed region after packing the parts `what` into it.
static int packed_source(const longer_config* cfg, const Shape& s, const longer_weights* w, const longer_input_weights* iw,
                         char* ws_packed, unsigned what, hipStream_t st, char** base) {
  if (!w) return fail(LONGER_ERR_ARG, "weights struct is NULL");
  if (w->packed) {
    if (((uintptr_t)w->packed & 255) != 0) return fail(LONGER_ERR_ARG, "packed weights must be 256-byte aligned");
    *base = (char*)w->packed;
    return 0;
  }
  *base = ws_packed;
  return pack_model(cfg, s, w, iw, ws_packed, what, st);
}

}  // namespace longer

using namespace longer;

// ------------------------------------------------------------------------------------
// Device memory of the entry point that takes no workspace (longer_score_candidates_static): the
// packed parameters of the scoring launch.  Every device the library runs on holds its own copy at
// its own address; host code uses the address hipGetSymbolAddress returns for the current device,
// never the symbol itself.
static constexpr size_t kScratchBytes = (size_t)LONGER_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static constexpr int kMaxDevices = 64;
static char* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static int scratch_of_current_device(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(LONGER_ERR_HIP, "hipGetDevice failed or device index %d beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> guard(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(LONGER_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = (char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

extern "C" {

const char* longer_last_error(void) { return g_err; }

size_t longer_workspace_bytes(const longer_config* cfg, int B, int L) {
  g_err[0] = 0;
  Shape s;
  if (check_cfg(cfg, &s, cfg && cfg->inner_layers > 0, true) || B <= 0 || L <= 0) return 0;
  return make_layout(cfg, s, B, L).total;
}

size_t longer_kv_cache_bytes(const longer_config* cfg, int U, int L) {
  g_err[0] = 0;
  Shape s;
  if (check_cfg(cfg, &s, false, true) || U <= 0 || L <= 0) return 0;
  return make_cache_layout(cfg, s, U, L).total;
}

size_t longer_packed_weights_bytes(const longer_config* cfg) {
  g_err[0] = 0;
  Shape s;
  if (check_cfg(cfg, &s, cfg && cfg->inner_layers > 0, true)) return 0;
  return packed_layout(cfg, s).total;
}

int longer_pack_weights(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                        void* packed_out, size_t bytes, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_cfg(cfg, &s, cfg && cfg->inner_layers > 0, true);
  if (rc) return rc;
  if (!w || !packed_out) return fail(LONGER_ERR_ARG, "NULL argument");
  if (((uintptr_t)packed_out & 255) != 0) return fail(LONGER_ERR_ARG, "packed_out must be 256-byte aligned");
  const PackedLayout pl = packed_layout(cfg, s);
  if (bytes < pl.total) return fail(LONGER_ERR_WS, "packed buffer too small: %zu < %zu bytes", bytes, pl.total);
  if (iw && (!iw->w1 || !iw->b1 || !iw->w2 || !iw->b2)) return fail(LONGER_ERR_ARG, "input MLP has NULL members");
  unsigned what = PK_LAYERS | PK_SCORE;
  if (cfg->inner_layers > 0 && w->inner) what |= PK_MERGE;
  if (stack_in_one_launch(s)) what |= PK_STACK;
  if (w->head_w && w->head_b) what |= PK_HEAD;
  return pack_model(cfg, s, w, iw, (char*)packed_out, what, (hipStream_t)stream);
}

static int merge_entry(const longer_config* cfg, const longer_block* inner, const void* H, const int32_t* lens,
                       int B, int L, void* M_out, void* Z_out, void* ws, size_t ws_bytes, void* stream, int z_f32 = 0) {
  Shape s;
  int rc = check_cfg(cfg, &s, true, false);
  if (rc) return rc;
  if (!inner || !H || (!M_out && !Z_out)) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_aligned({H, M_out, Z_out}))) return rc;
  const Layout l = make_layout(cfg, s, B, L);
  if ((rc = check_common(ws, ws_bytes, l.total, B, L))) return rc;
  if ((rc = check_slots(cfg, B, L))) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  const Shape si = inner_view(cfg, s);
  PackBatch pk_batch(cfg, si, st);
  if ((rc = pk_batch.add(inner, cfg->inner_layers, LAYOUT_FUSED, w8 + l.packed, (size_t)fused_segs(si.D, si.FF) * si.seg))) return rc;
  if ((rc = pk_batch.flush())) return rc;
  // a concat merge is the un-pooled output [B, T, K, d / K] read as [B, T, d]
  if (cfg->merge == LONGER_MERGE_CONCAT && M_out) { Z_out = M_out; M_out = nullptr; }
  return run_merge(cfg, si, w8 + l.packed, H, lens, B, L, M_out, 0, Z_out, z_f32, st);
}

int longer_inner_transformer(const longer_config* cfg, const longer_block* inner, const void* H, const int32_t* lens,
                             int B, int L, void* Z_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  return merge_entry(cfg, inner, H, lens, B, L, nullptr, Z_out, ws, ws_bytes, stream);
}

int longer_token_merge(const longer_config* cfg, const longer_block* inner, const void* H, const int32_t* lens,
                       int B, int L, void* M_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  return merge_entry(cfg, inner, H, lens, B, L, M_out, nullptr, ws, ws_bytes, stream);
}

// K/V and query wiring of the cross layer over R = [G; M]
static AttnIO cross_io(const longer_config* cfg, const Shape& s, const Layout& l, char* w8, const void* G, const void* M,
                       int M_f32, int B, int L, void* X_out, int X_f32) {
  const int T = cdiv(L, cfg->K);
  AttnIO io;
  memset(&io, 0, sizeof(io));
  io.src0 = RowSrc{G, (long long)cfg->m * s.D, 0};
  io.src1 = RowSrc{M, (long long)T * s.D, M_f32};
  io.m0 = cfg->m; io.key_rows = cfg->m + T; io.KG = cfg->m; io.key_self = 0; io.gather_recent = 1;
  io.q0 = 0; io.q_rows = s.n;
  io.kst = w8 + l.kst; io.vst = w8 + l.vst; io.kv_ustride = l.kv_ustride;
  io.q0src = io.src0; io.q1src = io.src1;
  if (cfg->q_learn) { io.q1src = RowSrc{cfg->q_learn, 0, 0}; io.gather_recent = 0; }   // slot i = row i, every user
  io.X_out = X_out; io.X_f32 = X_f32; io.X_ustride = (long long)s.n * s.D;
  return io;
}

// a self layer over X [B, n, d]
static AttnIO self_io(const longer_config* cfg, const Shape& s, const Layout& l, char* w8, const void* X, int X_in_f32,
                      void* X_out, int X_f32) {
  AttnIO io;
  memset(&io, 0, sizeof(io));
  const size_t es_in = X_in_f32 ? 4 : s.es;
  io.src0 = RowSrc{X, (long long)s.n * s.D, X_in_f32};
  io.src1 = RowSrc{(const char*)X + (size_t)cfg->m * s.D * es_in, (long long)s.n * s.D, X_in_f32};
  io.m0 = cfg->m; io.key_rows = s.n; io.KG = cfg->m; io.key_self = 1; io.gather_recent = 0;
  io.q0 = 0; io.q_rows = s.n;
  io.kst = w8 + l.kst; io.vst = w8 + l.vst; io.kv_ustride = l.kv_ustride;
  io.q0src = io.src0; io.q1src = io.src1;
  io.X_out = X_out; io.X_f32 = X_f32; io.X_ustride = (long long)s.n * s.D;
  return io;
}

int longer_hybrid_cross_attn(const longer_config* cfg, const longer_block* cross, const void* G, const void* M,
                             const int32_t* lens, int B, int L, void* X_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_cfg(cfg, &s, false, true);
  if (rc) return rc;
  if (!cross || !G || !M || !X_out) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_aligned({G, M, X_out}))) return rc;
  const Layout l = make_layout(cfg, s, B, L);
  if ((rc = check_common(ws, ws_bytes, l.total, B, L))) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  PackBatch pk_batch(cfg, s, st);
  if ((rc = pk_batch.add(cross, 1, LAYOUT_SPLIT, w8 + l.packed, s.pb))) return rc;
  if ((rc = pk_batch.flush())) return rc;
  AttnIO io = cross_io(cfg, s, l, w8, G, M, 0, B, L, X_out, 0);
  return run_layer(cfg, s, w8 + l.packed, lens, B, L, io, true, st);
}

int longer_self_attn_layer(const longer_config* cfg, const longer_block* blk, const void* X_in, const int32_t* lens,
                           int B, int L, void* X_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_cfg(cfg, &s, false, true);
  if (rc) return rc;
  if (!blk || !X_in || !X_out || X_in == X_out) return fail(LONGER_ERR_ARG, "NULL or aliased argument");
  if ((rc = check_aligned({X_in, X_out}))) return rc;
  const Layout l = make_layout(cfg, s, B, L);
  if ((rc = check_common(ws, ws_bytes, l.total, B, L))) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  PackBatch pk_batch(cfg, s, st);
  if ((rc = pk_batch.add(blk, 1, LAYOUT_SPLIT, w8 + l.packed, s.pb))) return rc;
  if ((rc = pk_batch.flush())) return rc;
  AttnIO io = self_io(cfg, s, l, w8, X_in, 0, X_out, 0);
  return run_layer(cfg, s, w8 + l.packed, lens, B, L, io, true, st);
}

// longer_forward, on H or (in != NULL) on the raw inputs of the input-generation stage
static int forward_impl(const longer_config* cfg, const longer_weights* w, const void* H, const MergeInput* in,
                        const void* G, const int32_t* lens, int B, int L, void* Y_out, float* logits_out,
                        void* ws, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = check_cfg(cfg, &s, true, true);
  if (rc) return rc;
  if ((!H && !in) || !G || !Y_out) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_aligned({H, G, Y_out}))) return rc;
  if (in) {
    if (cfg->merge != LONGER_MERGE_MEAN) return fail(LONGER_ERR_ARG, "input generation produces tokens of width d: merge must be LONGER_MERGE_MEAN");
    if ((rc = check_input(cfg, in->w, in->E, in->tdiff, in->d_e))) return rc;
  }
  const Layout l = make_layout(cfg, s, B, L);
  if ((rc = check_common(ws, ws_bytes, l.total, B, L))) return rc;
  if ((rc = check_slots(cfg, B, L))) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  const Shape si = inner_view(cfg, s);
  const bool concat = cfg->merge == LONGER_MERGE_CONCAT;
  const bool one_launch = stack_in_one_launch(s);
  const PackedLayout pl = packed_layout(cfg, s);
  char* pk = nullptr;
  if ((rc = packed_source(cfg, s, w, in ? in->w : nullptr, w8 + l.packed,
                          PK_MERGE | (one_launch ? PK_STACK : PK_LAYERS) | (logits_out ? PK_HEAD : 0u), st, &pk))) return rc;
  char* pk_cross = pk + pl.cross;
  float* head = (float*)(pk + pl.head);

  // the merge kernel's stream: (the input MLP,) then the InnerTrans blocks, back to back
  if ((rc = run_merge(cfg, si, pk + (in ? pl.mlp : pl.inner), H, lens, B, L, concat ? nullptr : w8 + l.M, 1,
                      concat ? w8 + l.M : nullptr, 1, st, in))) return rc;
  if (one_launch) {
    AttnIO io = cross_io(cfg, s, l, w8, G, w8 + l.M, 1, B, L, Y_out, 0);
    if (logits_out) { io.logits = logits_out; io.head = head; }
    if ((rc = run_layer(cfg, s, pk_cross, lens, B, L, io, false, st))) return rc;
    return run_stack(cfg, s, pk_cross, pk + pl.cross_pair, lens, B, L, io, st);
  }
  void* xbuf[2] = {w8 + l.xa, w8 + l.xb};
  const bool last0 = cfg->n_self == 0;
  AttnIO io = cross_io(cfg, s, l, w8, G, w8 + l.M, 1, B, L, last0 ? Y_out : xbuf[0], last0 ? 0 : 1);
  if (last0 && logits_out) { io.logits = logits_out; io.head = head; }
  if ((rc = run_layer(cfg, s, pk_cross, lens, B, L, io, true, st))) return rc;
  for (int i = 0; i < cfg->n_self; ++i) {
    const bool last = i + 1 == cfg->n_self;
    AttnIO sio = self_io(cfg, s, l, w8, xbuf[i & 1], 1, last ? Y_out : xbuf[(i + 1) & 1], last ? 0 : 1);
    if (last && logits_out) { sio.logits = logits_out; sio.head = head; }
    if ((rc = run_layer(cfg, s, pk + pl.self_split + (size_t)i * s.pb, lens, B, L, sio, true, st))) return rc;
  }
  return 0;
}

int longer_forward(const longer_config* cfg, const longer_weights* w, const void* H, const void* G, const int32_t* lens,
                   int B, int L, void* Y_out, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  if (!H) return fail(LONGER_ERR_ARG, "NULL argument");
  return forward_impl(cfg, w, H, nullptr, G, lens, B, L, Y_out, logits_out, ws, ws_bytes, stream);
}

int longer_forward_from_inputs(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                               const void* E, const void* tdiff, int d_e, const void* G, const int32_t* lens,
                               int B, int L, void* Y_out, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  if (!iw) return fail(LONGER_ERR_ARG, "NULL argument");
  const MergeInput in{iw, E, tdiff, d_e};
  return forward_impl(cfg, w, nullptr, &in, G, lens, B, L, Y_out, logits_out, ws, ws_bytes, stream);
}

// longer_kv_cache_build, on H or (in != NULL) on the raw inputs of the input-generation stage
static int cache_build_impl(const longer_config* cfg, const longer_weights* w, const void* H, const MergeInput* in,
                            const int32_t* lens, int U, int L, void* cache, void* ws, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = check_cfg(cfg, &s, true, true);
  if (rc) return rc;
  if ((!H && !in) || !cache) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_aligned({H}))) return rc;
  if (in) {
    if (cfg->merge != LONGER_MERGE_MEAN) return fail(LONGER_ERR_ARG, "input generation produces tokens of width d: merge must be LONGER_MERGE_MEAN");
    if ((rc = check_input(cfg, in->w, in->E, in->tdiff, in->d_e))) return rc;
  }
  if (((uintptr_t)cache & 255) != 0) return fail(LONGER_ERR_ARG, "cache must be 256-byte aligned");
  const Layout l = make_layout(cfg, s, U, L);
  if ((rc = check_common(ws, ws_bytes, l.total, U, L))) return rc;
  if ((rc = check_slots(cfg, U, L))) return rc;
  const CacheLayout cl = make_cache_layout(cfg, s, U, L);
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  const Shape si = inner_view(cfg, s);
  const bool concat = cfg->merge == LONGER_MERGE_CONCAT;
  const PackedLayout pl = packed_layout(cfg, s);
  char* pk = nullptr;
  if ((rc = packed_source(cfg, s, w, in ? in->w : nullptr, w8 + l.packed, PK_MERGE | PK_LAYERS, st, &pk))) return rc;
  if ((rc = run_merge(cfg, si, pk + (in ? pl.mlp : pl.inner), H, lens, U, L, concat ? nullptr : w8 + l.M, 1,
                      concat ? w8 + l.M : nullptr, 1, st, in))) return rc;

  const int T = cdiv(L, cfg->K);
  char* c8 = (char*)cache;
  void* xbuf[2] = {w8 + l.xa, w8 + l.xb};
  // layer 0: keys = merged tokens only; queries = the k recent slots
  AttnIO io;
  memset(&io, 0, sizeof(io));
  io.src0 = RowSrc{nullptr, 0, 0};
  io.src1 = RowSrc{w8 + l.M, (long long)T * s.D, 1};
  io.m0 = 0; io.key_rows = T; io.KG = 0; io.key_self = 0; io.gather_recent = 1;
  io.q0 = cfg->m; io.q_rows = cfg->k_recent;
  io.kst = c8; io.vst = c8 + cl.c0_voff; io.kv_ustride = cl.c0_ustride;
  io.q0src = io.src0; io.q1src = io.src1;
  if (cfg->q_learn) { io.q1src = RowSrc{cfg->q_learn, 0, 0}; io.gather_recent = 0; }
  io.X_out = xbuf[0]; io.X_f32 = 1; io.X_ustride = (long long)s.n * s.D;
  if ((rc = run_layer(cfg, s, pk + pl.cross, lens, U, L, io, cfg->n_self > 0, st))) return rc;
  for (int i = 0; i < cfg->n_self; ++i) {
    const char* xin = (const char*)xbuf[i & 1];
    AttnIO sio;
    memset(&sio, 0, sizeof(sio));
    sio.src0 = RowSrc{nullptr, 0, 0};
    sio.src1 = RowSrc{xin + (size_t)cfg->m * s.D * 4, (long long)s.n * s.D, 1};
    sio.m0 = 0; sio.key_rows = cfg->k_recent; sio.KG = 0; sio.key_self = 1; sio.gather_recent = 0;
    sio.q0 = cfg->m; sio.q_rows = cfg->k_recent;
    sio.kst = c8 + cl.c1_off + (size_t)i * cl.c1_lstride; sio.vst = sio.kst + cl.c1_voff; sio.kv_ustride = cl.c1_ustride;
    sio.q0src = sio.src0; sio.q1src = sio.src1;
    sio.X_out = xbuf[(i + 1) & 1]; sio.X_f32 = 1; sio.X_ustride = (long long)s.n * s.D;
    // the last layer's sequence rows feed nothing: only its K/V are needed
    if ((rc = run_layer(cfg, s, pk + pl.self_split + (size_t)i * s.pb, lens, U, L, sio, i + 1 < cfg->n_self, st))) return rc;
  }
  return 0;
}

int longer_kv_cache_build(const longer_config* cfg, const longer_weights* w, const void* H, const int32_t* lens,
                          int U, int L, void* cache, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  if (!H) return fail(LONGER_ERR_ARG, "NULL argument");
  return cache_build_impl(cfg, w, H, nullptr, lens, U, L, cache, ws, ws_bytes, stream);
}

int longer_kv_cache_build_from_inputs(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                                      const void* E, const void* tdiff, int d_e, const int32_t* lens, int U, int L,
                                      void* cache, void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  if (!iw) return fail(LONGER_ERR_ARG, "NULL argument");
  const MergeInput in{iw, E, tdiff, d_e};
  return cache_build_impl(cfg, w, nullptr, &in, lens, U, L, cache, ws, ws_bytes, stream);
}

// argument checks shared by the two scoring entry points
static int check_score_args(const longer_config* cfg, Shape* s, const longer_weights* w, const void* cache, const void* G_cand,
                            int U, int L, int C, const void* Yg_out, const float* logits_out) {
  int rc = check_cfg(cfg, s, false, true);
  if (rc) return rc;
  if (!w) return fail(LONGER_ERR_ARG, "weights struct is NULL");
  if (!cache || !G_cand || (!Yg_out && !logits_out)) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_aligned({G_cand, Yg_out}))) return rc;
  if (U <= 0 || L <= 0) return fail(LONGER_ERR_ARG, "U=%d, L=%d must be positive", U, L);
  if (C <= 0) return fail(LONGER_ERR_ARG, "C=%d must be positive", C);
  return 0;
}

// the scoring launch: `stream_base` = cross block then self blocks, fused layout, back to back
static int run_score(const longer_config* cfg, const Shape& s, const char* stream_base, const float* head, const void* cache,
                     const int32_t* lens, int U, int L, const void* G_cand, int C, void* Yg_out, float* logits_out,
                     hipStream_t st) {
  const CacheLayout cl = make_cache_layout(cfg, s, U, L);
  BlockParams p = base_params(cfg, s, lens, U, L, s.DH);
  p.wbase = stream_base; p.n_layers = 1 + cfg->n_self;
  p.Gc = G_cand; p.C = C; p.cache = (const char*)cache;
  p.c0_ustride = cl.c0_ustride; p.c0_voff = cl.c0_voff; p.c1_off = cl.c1_off; p.c1_lstride = cl.c1_lstride;
  p.c1_ustride = cl.c1_ustride; p.c1_voff = cl.c1_voff; p.kt0 = cl.kt0; p.kt1 = cl.kt1;
  p.X_out = Yg_out; p.X_f32 = 0;
  p.logits = logits_out; p.head = head;
  const int tiles = cdiv((long long)C * cfg->m, 32);
  p.xcds = kXcds; p.wg_per_user = cdiv(tiles, kWaves);
  dim3 grid((unsigned)(kXcds * cdiv(U, kXcds) * p.wg_per_user));
  StageScope scope(ST_SCORE, st);
  const int win = cfg->m <= 8 ? 4 : (cfg->m <= 16 ? 8 : 16);
  if (pair_score(s) ? s.pair(MODE_SCORE, win, p, grid, st) : s.main_fn(MODE_SCORE, 1, win, p, grid, st))
    return fail(LONGER_ERR_HIP, "score kernel launch failed");
  return 0;
}

int longer_score_candidates(const longer_config* cfg, const longer_weights* w, const void* cache, const int32_t* lens,
                            int U, int L, const void* G_cand, int C, void* Yg_out, float* logits_out,
                            void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_score_args(cfg, &s, w, cache, G_cand, U, L, C, Yg_out, logits_out);
  if (rc) return rc;
  const Layout l = make_layout(cfg, s, U, L);
  if ((rc = check_common(ws, ws_bytes, l.total, U, L))) return rc;
  hipStream_t st = (hipStream_t)stream;
  const PackedLayout pl = packed_layout(cfg, s);
  char* pk = nullptr;
  if ((rc = packed_source(cfg, s, w, nullptr, (char*)ws + l.packed, PK_SCORE | (logits_out ? PK_HEAD : 0u), st, &pk))) return rc;
  return run_score(cfg, s, pk + pl.score, (const float*)(pk + pl.head), cache, lens, U, L, G_cand, C, Yg_out, logits_out, st);
}

int longer_score_candidates_static(const longer_config* cfg, const longer_weights* w, const void* cache, const int32_t* lens,
                                   int U, int L, const void* G_cand, int C, void* Yg_out, float* logits_out, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_score_args(cfg, &s, w, cache, G_cand, U, L, C, Yg_out, logits_out);
  if (rc) return rc;
  // the scratch holds what the scoring launch streams: [cross, self blocks (fused)][panel overrun][head]
  const size_t stride = (size_t)fused_segs(s.D, s.FF) * s.seg;
  const size_t head_off = align256((size_t)(1 + cfg->n_self) * stride + 4 * s.seg);
  const size_t need = head_off + align256(((size_t)cfg->m * s.D + 1) * 4);
  if (need > kScratchBytes)
    return fail(LONGER_ERR_WS, "model too large for the static scratch: %zu > %zu bytes (use longer_score_candidates)", need, kScratchBytes);
  char* base = nullptr;
  if ((rc = scratch_of_current_device(&base))) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (!w->cross || (cfg->n_self > 0 && !w->self)) return fail(LONGER_ERR_ARG, "weights struct has NULL members");
  PackBatch pk(cfg, s, st);
  const int lay = pair_score(s) ? LAYOUT_PAIR_FUSED : LAYOUT_FUSED;
  if ((rc = pk.add(w->cross, 1, lay, base, stride))) return rc;
  if (cfg->n_self && (rc = pk.add(w->self, cfg->n_self, lay, base + stride, stride))) return rc;
  if (logits_out && (rc = pk.add_head(w, (float*)(base + head_off)))) return rc;
  if ((rc = pk.flush())) return rc;
  return run_score(cfg, s, base, (const float*)(base + head_off), cache, lens, U, L, G_cand, C, Yg_out, logits_out, st);
}

int longer_input_generation(const longer_config* cfg, const longer_input_weights* w, const void* E, const void* tdiff,
                            const int32_t* lens, int B, int L, int d_e, void* H_out,
                            void* ws, size_t ws_bytes, void* stream) {
  g_err[0] = 0;
  Shape s;
  int rc = check_cfg(cfg, &s, false, true);
  if (rc) return rc;
  if (!H_out) return fail(LONGER_ERR_ARG, "NULL argument");
  if ((rc = check_input(cfg, w, E, tdiff, d_e))) return rc;
  if ((rc = check_aligned({H_out}))) return rc;
  const Layout l = make_layout(cfg, s, B, L);
  if ((rc = check_common(ws, ws_bytes, l.total, B, L))) return rc;
  if ((long long)B * L + 32LL * kWaves >= (1LL << 31)) return fail(LONGER_ERR_ARG, "B*L = %lld rows: at most 2^31 per call", (long long)B * L);
  hipStream_t st = (hipStream_t)stream;
  char* w8 = (char*)ws;
  PackBatch pk_batch(cfg, s, st);
  if ((rc = pk_batch.add_mlp(w->w1, w->b1, w->w2, w->b2, w8 + l.packed))) return rc;
  if ((rc = pk_batch.flush())) return rc;
  BlockParams p = base_params(cfg, s, lens, B, L, s.DH);
  p.wbase = w8 + l.packed;
  p.in_e = E; p.in_pos = w->pos; p.in_td = tdiff; p.de = d_e;
  p.X_out = H_out;
  const int grid = cdiv((long long)B * L, 32LL * kWaves);
  StageScope scope(ST_MERGE, st);
  if (s.main_fn(MODE_INPUT, 1, 16, p, dim3(grid), st)) return fail(LONGER_ERR_HIP, "input generation launch failed");
  return 0;
}

int longer_stage_timing(int enable) {
  g_err[0] = 0;
  // 1 = every stage; any other non-zero value = bit (s + 1) selects stage s
  g_timer.mask = enable == 1 ? ~0u : (unsigned)enable >> 1;
  g_timer.n = 0;
  return 0;
}

int longer_stage_timing_read(double* ms_out, int32_t* launches_out) {
  g_err[0] = 0;
  if (!ms_out || !launches_out) return fail(LONGER_ERR_ARG, "NULL argument");
  for (int i = 0; i < LONGER_NUM_STAGES; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
  for (int i = 0; i < g_timer.n; ++i) {
    if (hipEventSynchronize(g_timer.ev[2 * i + 1]) != hipSuccess) return fail(LONGER_ERR_HIP, "hipEventSynchronize failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_timer.ev[2 * i], g_timer.ev[2 * i + 1]) != hipSuccess)
      return fail(LONGER_ERR_HIP, "hipEventElapsedTime failed");
    ms_out[g_timer.stage[i]] += ms;
    launches_out[g_timer.stage[i]] += 1;
  }
  g_timer.n = 0;
  return 0;
}

int longer_probe_mfma_layout(int32_t* out, void* stream) {
  g_err[0] = 0;
  if (!out) return fail(LONGER_ERR_ARG, "out is NULL");
  hipLaunchKernelGGL(probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, out);
  return hipGetLastError() == hipSuccess ? 0 : fail(LONGER_ERR_HIP, "probe launch failed");
}

}  // extern "C"

namespace longer {
// For the backward pass (backward.hip): the output rows of the first `layers` InnerTrans blocks as fp32,
// Z [B, T, K, w] (the fp32 residual stream of the fused kernel, zeros for padded tokens): the input rows
// of block `layers`, recomputed by the forward kernel.
__attribute__((visibility("hidden"))) int inner_chain_f32(const longer_config* cfg, const longer_block* inner, int layers,
                                                          const void* H, const int32_t* lens, int B, int L, float* Z_out,
                                                          void* ws, size_t ws_bytes, void* stream) {
  longer_config c = *cfg;
  c.inner_layers = layers;
  return merge_entry(&c, inner, H, lens, B, L, nullptr, Z_out, ws, ws_bytes, stream, 1);
}
}  // namespace longer
