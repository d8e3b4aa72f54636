// In-bounds instruction-rate probes (measurement aids, declared in include/longer.h): how fast
// this chip issues the 32x32x16 bf16 MFMA the block kernels are built from, alone and next to
// plain fp32 VALU work, in the arrangements a kernel can choose between.  The figures price the
// kernels against what the matrix pipe sustains under load, beside the vendor peak.
#include "../../include/longer.h"
#include "device.h"

namespace longer {

// One iteration per wave: an "M" phase of 16 MFMAs on four independent accumulators and / or a
// "V" phase of 128 independent fp32 FMAs.  512-thread workgroups: two waves on each SIMD.
//   mode 0  M in all 8 waves                           (the attainable MFMA rate)
//   mode 1  V in all 8 waves
//   mode 2  M then V in every wave                     (phases, as a kernel's GEMM / softmax stretches)
//   mode 3  waves 0-3 only M, waves 4-7 only V         (one wave of each kind per SIMD)
//   mode 4  as 3, each MFMA followed by idle cycles (s_nop) in its own wave
//   mode 5  every wave: each MFMA followed by 4 FMAs   (fine interleave inside a wave)
//   mode 6  every wave: each MFMA followed by 8 FMAs
//   mode 7  M in waves 0-3, waves 4-7 leave at once    (one wave per SIMD)
//   mode 8  M with the idle cycles of mode 4 in all 8 waves
//   mode 9  as 3 with the M waves at raised priority
//   mode 10 every wave: each MFMA followed by 4 packed fp16 FMAs    mode 11 packed fp16 FMAs alone (128)
//   mode 12 every wave: each MFMA followed by 2 packed fp16 FMAs    mode 13 each MFMA followed by 2 v_exp_f32
//   mode 14 v_exp_f32 alone (128)        mode 15 each MFMA followed by one 16-byte LDS read per lane
//   mode 16 each MFMA followed by 4 v_cvt_pk_bf16_f32               mode 17 each MFMA followed by 6 FMAs
//   modes 18-21, 128 instructions alone: packed fp16 FMA with a scalar-register constant / with the
//   clamp modifier and an inline constant / packed fp16 multiply / v_cvt_pkrtz_f16_f32
__device__ __forceinline__ void mm(f32x16& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ void ff(float& x, float m, float ad) {
  asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x) : "v"(m), "v"(ad));
}
__device__ __forceinline__ void pk(float& x, float m, float ad) {      // two fp16 FMAs per lane
  asm volatile("v_pk_fma_f16 %0, %0, %1, %2" : "+v"(x) : "v"(m), "v"(ad));
}
__device__ __forceinline__ void pks(float& x, float m) {               // with a scalar-register constant, low half broadcast
  asm volatile("v_pk_fma_f16 %0, %0, %1, s8 op_sel_hi:[1,1,0]" : "+v"(x) : "v"(m));
}
__device__ __forceinline__ void pkc(float& x, float m) {               // with the clamp modifier and an inline constant
  asm volatile("v_pk_fma_f16 %0, %0, %1, 0.5 op_sel_hi:[1,1,0] clamp" : "+v"(x) : "v"(m));
}
__device__ __forceinline__ void pkm(float& x, float m) { asm volatile("v_pk_mul_f16 %0, %0, %1" : "+v"(x) : "v"(m)); }
__device__ __forceinline__ void rtz(float& x, float y) { asm volatile("v_cvt_pkrtz_f16_f32 %0, %0, %1" : "+v"(x) : "v"(y)); }
__device__ __forceinline__ void ex(float& x) { asm volatile("v_exp_f32 %0, %0" : "+v"(x)); }
__device__ __forceinline__ void cv(float& x, float y) { asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x) : "v"(y)); }

template <int MODE>
__global__ void __launch_bounds__(512, 1) rate_kernel(float* out, int iters) {
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((lane + e) & 7); b[e] = (__bf16)(float)((lane * e) & 3); }
  f32x16 c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
  float v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = lane * 0.001f + i;
  const float m = 1.0001f, ad = 0.0001f;
  const bool first4 = wave < 4;
  if (MODE == 7 && !first4) return;
  if (MODE == 9 && first4) __builtin_amdgcn_s_setprio(3);
  for (int it = 0; it < iters; ++it) {
    const bool do_m = MODE == 0 || MODE == 2 || MODE == 7 || MODE == 8 || ((MODE == 3 || MODE == 4 || MODE == 9) && first4);
    const bool do_v = MODE == 1 || MODE == 2 || ((MODE == 3 || MODE == 4 || MODE == 9) && !first4);
    if (MODE >= 10) {
      __shared__ uint4 lbuf[512];
      if (MODE == 11 || MODE == 14 || MODE >= 18) {
#pragma unroll
        for (int sidx = 0; sidx < 128; ++sidx) {
          if (MODE == 11) pk(v[sidx & 15], m, ad);
          else if (MODE == 14) ex(v[sidx & 15]);
          else if (MODE == 18) pks(v[sidx & 15], m);
          else if (MODE == 19) pkc(v[sidx & 15], m);
          else if (MODE == 20) pkm(v[sidx & 15], m);
          else rtz(v[sidx & 15], ad);
        }
        continue;
      }
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        mm(c[s & 3], a, b);
        if (MODE == 10) { for (int i2 = 0; i2 < 4; ++i2) pk(v[(s * 4 + i2) & 15], m, ad); }
        if (MODE == 12) { for (int i2 = 0; i2 < 2; ++i2) pk(v[(s * 2 + i2) & 15], m, ad); }
        if (MODE == 13) { for (int i2 = 0; i2 < 2; ++i2) ex(v[(s * 2 + i2) & 15]); }
        if (MODE == 15) {     // one 16-byte LDS read per lane and MFMA (the shape of a weight-fragment read)
          const unsigned addr = (unsigned)(unsigned long long)&lbuf[0] + (unsigned)tid * 16u;
          u32x4 t;
          asm volatile("ds_read_b128 %0, %1" : "=v"(t) : "v"(addr));
          if ((s & 3) == 3) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        if (MODE == 16) { for (int i2 = 0; i2 < 4; ++i2) cv(v[(s * 4 + i2) & 15], ad); }
        if (MODE == 17) { for (int i2 = 0; i2 < 6; ++i2) ff(v[(s * 6 + i2) & 15], m, ad); }
      }
      continue;
    }
    if (MODE == 5 || MODE == 6) {
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        mm(c[s & 3], a, b);
#pragma unroll
        for (int i = 0; i < (MODE == 5 ? 4 : 8); ++i) ff(v[(s * (MODE == 5 ? 4 : 8) + i) & 15], m, ad);
      }
      continue;
    }
    if (do_m) {
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        mm(c[s & 3], a, b);
        if (MODE == 4 || MODE == 8) asm volatile("s_nop 15\n\ts_nop 7");
      }
    }
    if (do_v) {
#pragma unroll
      for (int s = 0; s < 128; ++s) ff(v[s & 15], m, ad);
    }
  }
  // (the MFMAs are opaque to the compiler's hazard tracking: let the last ones retire before their
  // results are read)
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) r += c[0][i] + c[1][i] + c[2][i] + c[3][i] + v[i];
  out[(size_t)blockIdx.x * 512 + tid] = r;
}

}  // namespace longer

using namespace longer;

extern "C" int longer_probe_rate(int mode, int iters, int workgroups, float* out, void* stream) {
  if (!out || iters <= 0 || workgroups <= 0 || workgroups > 65536 || mode < 0 || mode > 21) return LONGER_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const dim3 g(workgroups), t(512);
  switch (mode) {
    case 0: hipLaunchKernelGGL(rate_kernel<0>, g, t, 0, st, out, iters); break;
    case 1: hipLaunchKernelGGL(rate_kernel<1>, g, t, 0, st, out, iters); break;
    case 2: hipLaunchKernelGGL(rate_kernel<2>, g, t, 0, st, out, iters); break;
    case 3: hipLaunchKernelGGL(rate_kernel<3>, g, t, 0, st, out, iters); break;
    case 4: hipLaunchKernelGGL(rate_kernel<4>, g, t, 0, st, out, iters); break;
    case 5: hipLaunchKernelGGL(rate_kernel<5>, g, t, 0, st, out, iters); break;
    case 6: hipLaunchKernelGGL(rate_kernel<6>, g, t, 0, st, out, iters); break;
    case 7: hipLaunchKernelGGL(rate_kernel<7>, g, t, 0, st, out, iters); break;
    case 8: hipLaunchKernelGGL(rate_kernel<8>, g, t, 0, st, out, iters); break;
    case 9: hipLaunchKernelGGL(rate_kernel<9>, g, t, 0, st, out, iters); break;
    case 10: hipLaunchKernelGGL(rate_kernel<10>, g, t, 0, st, out, iters); break;
    case 11: hipLaunchKernelGGL(rate_kernel<11>, g, t, 0, st, out, iters); break;
    case 12: hipLaunchKernelGGL(rate_kernel<12>, g, t, 0, st, out, iters); break;
    case 13: hipLaunchKernelGGL(rate_kernel<13>, g, t, 0, st, out, iters); break;
    case 14: hipLaunchKernelGGL(rate_kernel<14>, g, t, 0, st, out, iters); break;
    case 15: hipLaunchKernelGGL(rate_kernel<15>, g, t, 0, st, out, iters); break;
    case 16: hipLaunchKernelGGL(rate_kernel<16>, g, t, 0, st, out, iters); break;
    case 17: hipLaunchKernelGGL(rate_kernel<17>, g, t, 0, st, out, iters); break;
    case 18: hipLaunchKernelGGL(rate_kernel<18>, g, t, 0, st, out, iters); break;
    case 19: hipLaunchKernelGGL(rate_kernel<19>, g, t, 0, st, out, iters); break;
    case 20: hipLaunchKernelGGL(rate_kernel<20>, g, t, 0, st, out, iters); break;
    default: hipLaunchKernelGGL(rate_kernel<21>, g, t, 0, st, out, iters); break;
  }
  return hipGetLastError() == hipSuccess ? LONGER_OK : LONGER_ERR_HIP;
}
