// The transformer-block kernel with a 32-row tile given to a PAIR of waves (bf16, d = 128 / 256):
//
//   MODE_STACK  the whole reduced stack of one user in one workgroup (Eq. 10), as in block_kernel.h;
//   MODE_SCORE  candidate scoring of the KV-cache serving path (Section 3.6.3).
//
// Why.  In these modes the number of tiles is fixed by the work (a user's m + k rows, or registers at
// d = 256 allow one tile-wave per SIMD only), and a single wave per SIMD is bound by its own
// instruction issue and dependency latencies.  Here a workgroup has 8 waves, two per SIMD: waves t
// and t + 4 share tile t.  They split every GEMM by output feature tile (wave half h owns tiles
// 2 i + h), so neither holds fp32 partial sums of the other:
//   - the fp32 residual rows are split by feature tile; LayerNorm exchanges two partial sums per row,
//     then each wave normalises its own tiles and the pair swaps the bf16 results through LDS (each
//     wave then holds all of LN(x), the B operand of Q / K / V and of the first FFN GEMM);
//   - Q, K, V and the attention heads of a wave's own tiles are private to it; the attention output
//     is swapped like the normalised rows and the output projection produces the own residual tiles;
//   - FFN: hidden chunks alternate between the two waves (first GEMM + activation), the activated
//     chunk goes through LDS, and each wave runs the second GEMM for its own output tiles over both;
//   - the packed stream brings the even and the odd tile of a matrix side by side (pair layouts,
//     device.h) in panels of two segments: one segment of work for either wave in every panel.
// Register indices never depend on the half (only LDS / global addresses do): a wave keeps its own
// operand groups and its partner's in separate arrays.
#pragma once
#include "block_kernel.h"

namespace longer {

constexpr int kPairThreads = 512;   // 8 waves: tile t is shared by waves t and t + 4 (the same SIMD)

template <int NTH>
__device__ __forceinline__ void load_rows_half(f32x16 (&x)[NTH], const void* base, int is_f32, long long off,
                                               bool valid, int hi, int h) {
#pragma unroll
  for (int i = 0; i < NTH; ++i) {
    f32x16 one[1];
    load_rows<__bf16, 1>(one, base, is_f32, off + 32 * (2 * i + h), valid, hi);
    x[i] = one[0];
  }
}

template <int NTH>
__device__ __forceinline__ void store_rows_half(const f32x16 (&x)[NTH], void* base, int is_f32, long long off,
                                                bool nonzero, int hi, int h) {
#pragma unroll
  for (int i = 0; i < NTH; ++i) {
    f32x16 one[1];
    one[0] = x[i];
    store_rows<__bf16, 1>(one, base, is_f32, off + 32 * (2 * i + h), nonzero, hi);
  }
}

template <int D, int DH, int MODE, int W, bool RELU>
__global__ void __launch_bounds__(kPairThreads, 1) pair_kernel(const BlockParams p) {
  using T = __bf16;
  using E = ET<T>;
  using grp = typename E::grp;
  constexpr int NT = D / 32, NTH = NT / 2, NG = D / E::GF, GPT = E::GPT, NGH = NG / 2;
  constexpr int SEGV = NG * 64;
  constexpr int HPT = 32 / DH;        // heads per 32-feature tile
  constexpr int GPH = DH / E::GF;     // operand groups per head
  constexpr bool STACK = MODE == MODE_STACK, SCORE = MODE == MODE_SCORE;
  static_assert(STACK || SCORE, "pair kernel modes");
  static_assert(NT % 2 == 0 && (DH == 16 || DH == 32), "shape");
  constexpr int PSEG = 2;                           // a panel = the even and the odd tile's segment
  constexpr int NB = D >= 256 ? 2 : 3;              // ring depth in panels
  __shared__ uint4 lds[NB * PSEG * SEGV];
  __shared__ uint4 vecl[SEGV];                      // the current block's fp32 vectors
  __shared__ uint4 xch[4 * NG * 64];                // per tile: operand groups swapped inside the pair
  __shared__ float stat[4][2][2][32];               // per tile, half: LayerNorm partial sums / logit parts per row
  // MODE_STACK: K and V fragments of the feature tile a half works on, [half][parity][key tile][K, V][group][lane]
  __shared__ uint4 kvl[STACK ? 2 * 2 * 4 * 2 * GPT * 64 : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j = lane & 31, hi = lane >> 5;
  const int ts = wave & 3, h = wave >> 2;           // tile slot in the workgroup; which half of the pair
  const int NC = p.FF / 32;

  // ------------------------------------------------------------------ rows of this wave's tile
  bool valid, inrange;
  int usr = 0, Tu = 0;
  long long out_off = 0;
  uint32_t tilebits = 0;
  const int widx = W == 16 ? 0 : j / (2 * W);
  uint32_t wmask[16 / W];
#pragma unroll
  for (int w = 0; w < 16 / W; ++w) { wmask[w] = widx == w ? 0xffffffffu : 0u; asm("" : "+v"(wmask[w])); }
  int lo1 = 0, hi1 = 0, lo2 = 0, hi2 = 0, kthi = 0;     // cross layer: visible key ranges, key tile count
  int slo1 = 0, shi1 = 0, slo2 = 0, shi2 = 0;           // self-causal layers of the stack
  f32x16 resid[NTH];

  int wg = blockIdx.x, su = 0;
  if (SCORE) {      // all candidate tiles of a user on one XCD (see block_kernel.h)
    const int x = (int)blockIdx.x % p.xcds, sq = (int)blockIdx.x / p.xcds;
    su = x + p.xcds * (sq / p.wg_per_user);
    wg = sq % p.wg_per_user;
    if (su >= p.B) return;
  }
  const int tile = wg * 4 + ts;
  if (STACK) {
    const int u = tile / p.tiles_per_user, qt = tile - u * p.tiles_per_user;
    const int a = p.q0 + 32 * qt + j;
    inrange = u < p.B && (32 * qt + j) < p.rows_per_user;
    int len = 0;
    if (u < p.B) { len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L); }
    const int tu = (len + p.K - 1) / p.K;
    const bool glob = a < p.m;
    const int i = a - p.m, i0 = first_slot(p.k, tu, p.q_learn);
    valid = inrange && (glob || i >= i0);
    usr = u; Tu = tu;
    out_off = p.X_ustride * u + (long long)a * D;
    const void* sp = glob ? p.src0.p : p.src1.p;
    const int sf = glob ? p.src0.f32 : p.src1.f32;
    const long long sus = glob ? p.src0.ustride : p.src1.ustride;
    const int tok = glob ? 0 : (p.q_learn ? tu - 1 : slot_token(i, p.k, tu, p.k_uni));
    const int row = glob ? a : (p.gather_recent ? tok : i);
    load_rows_half<NTH>(resid, sp, sf, sus * u + (long long)row * D, valid, hi, h);
    // visible key ranges (Eq. 8 by token type); keys of the cross layer are all T merged tokens
    if (glob) {
      lo1 = p.gmask_causal ? a : 0; hi1 = p.KG;
      lo2 = p.KG; hi2 = p.KG + tu;
    } else {
      lo2 = p.KG; hi2 = p.KG + tok + 1;
    }
    if (!valid) { hi1 = lo1; hi2 = lo2; }
    kthi = (p.KG + tu + 31) / 32;
    if (u >= p.B) kthi = 0;
    if (valid) {   // keys of a self-causal layer: the user's own rows, key index = row index
      if (glob) { slo1 = p.gmask_causal ? a : 0; shi1 = p.m; slo2 = p.m + i0; shi2 = p.m + p.k; }
      else { slo2 = p.m + i0; shi2 = p.m + i + 1; }
    }
  } else {  // MODE_SCORE
    const int u = su;
    const int a = 32 * tile + j;
    const int cand = a / p.m, gi = a - cand * p.m;
    inrange = cand < p.C;
    valid = inrange;
    int len = p.lens ? p.lens[u] : p.L; len = min(max(len, 0), p.L);
    usr = u; Tu = (len + p.K - 1) / p.K;
    out_off = ((long long)u * p.C * p.m + a) * D;
    load_rows_half<NTH>(resid, p.Gc, 0, out_off, valid, hi, h);
    const uint32_t vb = (uint32_t)__ballot(valid);
    const int gbase = p.m * (j / p.m);
    tilebits = ((range_bits(gbase + (p.gmask_causal ? gi : 0), gbase + p.m, 0) & vb) >> (4 * hi)) >> (2 * W * widx);
  }

  WStream<SEGV, PSEG, NB, false, kPairThreads> ws;
  const int segs_fused = 2 + 4 * NT + 2 * NC, segs_attn = 2 + 2 * NT + 2 * NC;
  ws.init(lds, p.wbase, STACK ? segs_attn + (p.n_layers - 1) * segs_fused : segs_fused * p.n_layers);

  uint4* const xt = xch + (size_t)ts * NG * 64 + lane;      // this tile's exchange area, this lane's 16 bytes of a group
  // operand groups of own tiles go to the exchange area, the partner's come back
  auto swap_groups = [&](const grp (&own)[NGH], grp (&oth)[NGH]) {
#pragma unroll
    for (int i = 0; i < NTH; ++i)
#pragma unroll
      for (int g = 0; g < GPT; ++g) *reinterpret_cast<grp*>(xt + ((2 * i + h) * GPT + g) * 64) = own[i * GPT + g];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NTH; ++i)
#pragma unroll
      for (int g = 0; g < GPT; ++g) oth[i * GPT + g] = *reinterpret_cast<const grp*>(xt + ((2 * i + (h ^ 1)) * GPT + g) * 64);
  };
  // one 32-wide output tile of a GEMM over all of the pair's operand groups; `which` = the segment
  // of the current panel (0 / 1) that holds the weights
  auto gemm_tile = [&](f32x16 acc, int which, const grp (&own)[NGH], const grp (&oth)[NGH]) -> f32x16 {
#pragma unroll
    for (int i = 0; i < NTH; ++i)
#pragma unroll
      for (int g = 0; g < GPT; ++g) {
        acc = E::mma(ws.template frag_at<grp>(which, (2 * i + h) * GPT + g), own[i * GPT + g], acc);
        acc = E::mma(ws.template frag_at<grp>(which, (2 * i + (h ^ 1)) * GPT + g), oth[i * GPT + g], acc);
      }
    return acc;
  };
  const VecLayout vl{D, p.FF};
  const float* vec = reinterpret_cast<const float*>(vecl);
  // the tile's operand groups back from the exchange area: own[] = this wave's tiles, oth[] = the partner's
  auto load_groups = [&](grp (&own)[NGH], grp (&oth)[NGH]) {
#pragma unroll
    for (int i = 0; i < NTH; ++i)
#pragma unroll
      for (int g = 0; g < GPT; ++g) {
        own[i * GPT + g] = *reinterpret_cast<const grp*>(xt + ((2 * i + h) * GPT + g) * 64);
        oth[i * GPT + g] = *reinterpret_cast<const grp*>(xt + ((2 * i + (h ^ 1)) * GPT + g) * 64);
      }
  };
  // LayerNorm of the pair's rows, as B-operand groups in the exchange area (each wave writes its tiles)
  auto layer_norm_pair = [&](const float* gam, const float* bet) {
    float s = 0.f, q = 0.f;
#pragma unroll
    for (int i = 0; i < NTH; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) { s += resid[i][r]; q = fmaf(resid[i][r], resid[i][r], q); }
    s = sum_halves(s); q = sum_halves(q);
    if (hi == 0) { stat[ts][h][0][j] = s; stat[ts][h][1][j] = q; }
    __syncthreads();
    s += stat[ts][h ^ 1][0][j]; q += stat[ts][h ^ 1][1][j];
    const float mean = s * (1.0f / D);
    const float var = fmaxf(q * (1.0f / D) - mean * mean, 0.f);
    const float rstd = __builtin_amdgcn_rsqf(var + p.eps);
    const float shift = -mean * rstd;
#pragma unroll
    for (int i = 0; i < NTH; ++i) {
      const f32x16 gt = bias_tile(gam, 2 * i + h, hi), bt = bias_tile(bet, 2 * i + h, hi);
      f32x16 y;
#pragma unroll
      for (int r = 0; r < 16; ++r) y[r] = fmaf(fmaf(resid[i][r], rstd, shift), gt[r], bt[r]);
#pragma unroll
      for (int g = 0; g < GPT; ++g) *reinterpret_cast<grp*>(xt + ((2 * i + h) * GPT + g) * 64) = E::pack(y, g);
    }
    __syncthreads();
  };

  for (int layer = 0; layer < p.n_layers; ++layer) {
    // the block's first segment holds its fp32 vectors: keep a copy for the whole layer
    // (barriers: nobody still reads the previous block's copy; everybody sees the new one)
    if (layer > 0) __syncthreads();
#pragma unroll
    for (int i = 0; i < SEGV / kPairThreads; ++i) vecl[tid + kPairThreads * i] = ws.cur()[tid + kPairThreads * i];
    __syncthreads();
    ws.advance();
    ws.advance();            // [vec][unused]
    const bool selfl = STACK && layer > 0;   // a self-causal layer of the stack: K/V made here
    const bool own_kv = SCORE || selfl;      // K and V of this tile's rows are projected here
    layer_norm_pair(vec + vl.ln1_g(), vec + vl.ln1_b());
    grp oo[NGH], op[NGH];     // attention output of the own tiles / the partner's

#pragma unroll
    for (int i = 0; i < NTH; ++i) {
      const int ft = 2 * i + h;               // the feature tile (= its heads) this wave works on
      // the normalised rows are read again for every feature tile instead of being held through
      // the attention in between (registers: two waves per SIMD have 256 each)
      grp xo[NGH], xp[NGH];
      load_groups(xo, xp);
      f32x16 aq = gemm_tile(bias_tile(vec + vl.bq(), ft, hi), h, xo, xp);
      ws.advance();
      ws.advance();
      f32x16 ak, av;
      if (own_kv) {
        ak = gemm_tile(splat16(0.f), h, xo, xp);   // no b_K: a per-query constant in the scores, softmax drops it
        ws.advance();
        ws.advance();
        // no b_V (folded into the output bias); operands swapped: lane = feature
        av = splat16(0.f);
#pragma unroll
        for (int i2 = 0; i2 < NTH; ++i2)
#pragma unroll
          for (int g = 0; g < GPT; ++g) {
            av = E::mma(xo[i2 * GPT + g], ws.template frag_at<grp>(h, (2 * i2 + h) * GPT + g), av);
            av = E::mma(xp[i2 * GPT + g], ws.template frag_at<grp>(h, (2 * i2 + (h ^ 1)) * GPT + g), av);
          }
        ws.advance();
        ws.advance();
      }
      if (selfl) {
        // this wave's rows are key tile ts of feature tile ft: hand K and V to the waves of the same half.
        // Two buffers per half: one barrier per feature tile is enough (nobody can be two tiles ahead
        // of a wave that still reads).
        uint4* dstk = kvl + (size_t)((((h * 2 + (i & 1)) * 4 + ts) * 2) * GPT) * 64 + lane;
#pragma unroll
        for (int g = 0; g < GPT; ++g) {
          *reinterpret_cast<grp*>(dstk + g * 64) = E::pack(ak, g);
          *reinterpret_cast<grp*>(dstk + (GPT + g) * 64) = E::pack(av, g);
        }
        __syncthreads();
      }

      grp qop[GPT];   // Q carries log2(e) / sqrt(head width): the scores come out ready for exp2
      aq *= p.scale_l2e;
#pragma unroll
      for (int g = 0; g < GPT; ++g) qop[g] = E::pack(aq, g);
      float mrun[HPT], lrun[HPT];
      f32x16 acc[HPT];
#pragma unroll
      for (int hh = 0; hh < HPT; ++hh) { mrun[hh] = kNegBig; lrun[hh] = 0.f; acc[hh] = splat16(0.f); }

      if (SCORE) {   // keys of the lane's own tile: the candidate's own globals
        grp kop[GPT], vop[GPT];
#pragma unroll
        for (int g = 0; g < GPT; ++g) { kop[g] = E::pack(ak, g); vop[g] = E::pack(av, g); }
#pragma unroll
        for (int hh = 0; hh < HPT; ++hh) {
          f32x16 S = splat16(0.f);
#pragma unroll
          for (int g2 = 0; g2 < GPH; ++g2) S = E::mma(kop[hh * GPH + g2], qop[hh * GPH + g2], S);
          grp pop[GPT];
          softmax_window<T, W>(S, widx, wmask, tilebits, mrun[hh], lrun[hh], acc[hh], pop);
#pragma unroll
          for (int g = 0; g < GPT; ++g) acc[hh] = E::mma(vop[g], pop[g], acc[hh]);
        }
      }
      if (selfl) {   // K/V fragments of the user's own rows, from LDS
        const int nkt = (p.m + p.k + 31) / 32;
        for (int kt = 0; kt < nkt; ++kt) {
          const uint32_t bits = range_bits(slo1, shi1, 32 * kt) | range_bits(slo2, shi2, 32 * kt);
          const uint32_t ab = (bits >> (4 * hi)) & kTileBits;
          if (__builtin_amdgcn_ballot_w64(ab != 0) == 0) continue;      // no query of the tile sees any of these keys
          const bool full = __builtin_amdgcn_ballot_w64(ab != kTileBits) == 0;
          const f32x16 vis = full ? splat16(0.f) : mask_tile(ab);
          const uint4* srck = kvl + (size_t)((((h * 2 + (i & 1)) * 4 + kt) * 2) * GPT) * 64 + lane;
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
      if (SCORE || (STACK && !selfl)) {     // stored K/V fragments (wave-uniform user, scalar loop control)
        const int uu = __builtin_amdgcn_readfirstlane(usr);
        const int tuu = __builtin_amdgcn_readfirstlane(Tu);
        const char* kb; const char* vb; int nkt, rlo, rhi;
        if (STACK) {
          kb = p.kst + (size_t)uu * p.kv_ustride; vb = p.vst + (size_t)uu * p.kv_ustride;
          nkt = __builtin_amdgcn_readfirstlane(kthi); rlo = 0; rhi = 0;
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
          if (!valid) rhi = rlo;
        }
        // the fragments of key tile kt + 1 are requested before tile kt is worked on (d = 128; at
        // d = 256 the registers for that are not there, and the SIMD's other wave covers the latency)
        constexpr bool AHEAD = D < 256;
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
          if (STACK) bits = range_bits(lo1, hi1, 32 * kt) | range_bits(lo2, hi2, 32 * kt);
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
          if (none) continue;
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
      for (int hh = 0; hh < HPT; ++hh) inv[hh] = lrun[hh] > 0.f ? __builtin_amdgcn_rcpf(lrun[hh]) : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int hh = HPT == 1 ? 0 : r / 8;
        o[r] = acc[hh][r] * inv[hh];
      }
#pragma unroll
      for (int g = 0; g < GPT; ++g) oo[i * GPT + g] = E::pack(o, g);
    }
    swap_groups(oo, op);

    // output projection + residual: own output tiles
#pragma unroll
    for (int i = 0; i < NTH; ++i) {
      resid[i] += bias_tile(vec + vl.bo(), 2 * i + h, hi);
      resid[i] = gemm_tile(resid[i], h, oo, op);
      ws.advance();
      ws.advance();
    }

    // FFN: hidden chunks 2 c2 + h are this wave's; the activated chunks go through the exchange area
    layer_norm_pair(vec + vl.ln2_g(), vec + vl.ln2_b());
    grp xo[NGH], xp[NGH];
    load_groups(xo, xp);
    __syncthreads();          // everybody has its copy: the exchange area is free for the activated chunks
#pragma unroll
    for (int i = 0; i < NTH; ++i) resid[i] += bias_tile(vec + vl.b2(), 2 * i + h, hi);
#pragma unroll 1
    for (int c2 = 0; c2 < NC / 2; ++c2) {
      // panel [w1(2 c2) w1(2 c2 + 1)]: first GEMM + activation of the own chunk
      f32x16 ah = gemm_tile(bias_tile(vec + vl.b1(), 2 * c2 + h, hi), h, xo, xp);
      typename E::hgrp hown[GPT], hoth[GPT];
#pragma unroll
      for (int g = 0; g < GPT; ++g) {
        f16x8 y;     // ah holds x / kFfnScale; to fp16 toward zero, then the packed activation
#pragma unroll
        for (int e = 0; e < E::EPL / 2; ++e) {
          const f16x2 y2 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(ah[E::EPL * g + 2 * e], ah[E::EPL * g + 2 * e + 1]));
          y[2 * e] = y2[0]; y[2 * e + 1] = y2[1];
        }
        hown[g] = RELU ? __builtin_elementwise_max(y, (f16x8)((_Float16)0.f)) : gelu_quarter_h8(y);
        *reinterpret_cast<typename E::hgrp*>(xt + (h * GPT + g) * 64) = hown[g];
      }
      ws.advance();
      ws.advance();          // (the panel switch's barrier also orders the exchange: written above, read below)
#pragma unroll
      for (int g = 0; g < GPT; ++g) hoth[g] = *reinterpret_cast<const typename E::hgrp*>(xt + ((h ^ 1) * GPT + g) * 64);
      // panel [w2(2 c2) w2(2 c2 + 1)]: second GEMM of both chunks for the own output tiles
#pragma unroll
      for (int g = 0; g < GPT; ++g)
#pragma unroll
        for (int i = 0; i < NTH; ++i) {
          resid[i] = E::mma_h(ws.template frag_at<grp>(h, (2 * i + h) * GPT + g), hown[g], resid[i]);
          resid[i] = E::mma_h(ws.template frag_at<grp>(h ^ 1, (2 * i + h) * GPT + g), hoth[g], resid[i]);
        }
      ws.advance();
      ws.advance();          // (its barrier: the partner has read this chunk pair before the next one is written)
    }
  }

  wait_vmcnt<0>();   // nothing of the weight stream may still be in flight when the wave ends
  // ------------------------------------------------------------------ epilogue
  if (p.X_out && inrange) store_rows_half<NTH>(resid, p.X_out, p.X_f32, out_off, valid, hi, h);
  if (p.logits) {
    // logit = <head_w, flatten(global rows)> + head_b: each wave sums over its own feature tiles
    int a, width;       // row inside the head's m rows; lanes per logit
    bool take;
    if (STACK) {
      const int qt = tile % p.tiles_per_user;
      a = p.q0 + 32 * qt + j; take = valid && a < p.m; width = 32;
    } else {
      a = (32 * tile + j) % p.m; take = valid; width = p.m;
    }
    float part = 0.f;
    if (take) {
#pragma unroll
      for (int i = 0; i < NTH; ++i) {
        const f32x16 hw = bias_tile(p.head + (size_t)a * D, 2 * i + h, hi);
#pragma unroll
        for (int r = 0; r < 16; ++r) part += resid[i][r] * hw[r];
      }
    }
    part = sum_halves(part);
    __syncthreads();                       // the LayerNorm sums in `stat` have been read by everybody
    if (hi == 0) stat[ts][h][0][j] = part;
    __syncthreads();
    part = stat[ts][0][0][j] + stat[ts][1][0][j];
    for (int sft = 1; sft < width; sft <<= 1) part += __shfl_xor(part, sft, 64);
    part += p.head[(size_t)p.m * D];
    if (h == 0) {
      if (STACK) {
        if (lane == 0 && usr < p.B && (tile % p.tiles_per_user) == 0 && p.q0 == 0) p.logits[usr] = part;
      } else {
        const int cand = (32 * tile + j) / p.m;
        if (hi == 0 && (j % p.m) == 0 && cand < p.C) p.logits[(size_t)usr * p.C + cand] = part;
      }
    }
  }
}

// Host-side launcher, one definition per (D, DH) instantiation file.
template <int D, int DH>
int launch_pair(int mode, int win, const BlockParams& p, dim3 grid, hipStream_t stream);

#define LONGER_PAIR_LAUNCH(D, DH, MODEV, WV) \
  do {                                                                                                \
    if (p.act == 1)                                                                                   \
      hipLaunchKernelGGL((pair_kernel<D, DH, MODEV, WV, true>), grid, dim3(kPairThreads), 0, stream, p); \
    else                                                                                              \
      hipLaunchKernelGGL((pair_kernel<D, DH, MODEV, WV, false>), grid, dim3(kPairThreads), 0, stream, p); \
  } while (0)

#define LONGER_PAIR_INSTANTIATE(D, DH)                                                                \
  template <>                                                                                         \
  int launch_pair<D, DH>(int mode, int win, const BlockParams& p, dim3 grid, hipStream_t stream) {    \
    switch (mode) {                                                                                   \
      case MODE_STACK:       /* (the K/V hand-over area fits the LDS at d = 128 only) */            \
        if constexpr (D <= 128) LONGER_PAIR_LAUNCH(D, DH, MODE_STACK, 16); else return -1;            \
        break;                                                                                        \
      case MODE_SCORE:                                                                                \
        if (win == 4) LONGER_PAIR_LAUNCH(D, DH, MODE_SCORE, 4);                                       \
        else if (win == 8) LONGER_PAIR_LAUNCH(D, DH, MODE_SCORE, 8);                                  \
        else LONGER_PAIR_LAUNCH(D, DH, MODE_SCORE, 16);                                               \
        break;                                                                                        \
      default: return -1;                                                                             \
    }                                                                                                 \
    return hipGetLastError() == hipSuccess ? 0 : -3;                                                  \
  }

}  // namespace longer
