// Fast-transform realisation of the low-pass projection and deviation score (Eq. 6-10).
//
// The orthonormal DCT-II / DCT-III pair of Eq. 6 and Eq. 9 with the mask of Eq. 8 in between is a
// projection, so its scale factors cancel and it can be carried out on an unnormalised complex FFT:
//   * two adjacent feature columns ride as the real and imaginary part of one complex sequence;
//   * tokens are permuted (even tokens ascending, then odd tokens descending), w[j];
//   * W = DFT_N(w);  keeping DCT modes m < r of both columns is, in terms of W,
//       W^[0] = W[0],  W^[m] = (W[m] + e^{+i pi m/N} W[N-m]) / 2,  W^[N-m] = e^{-i pi m/N} W^[m]
//     for 1 <= m < r and zero elsewhere;
//   * w_base = IDFT_N(W^) un-permuted is the Base KV of both columns.
//
// The N-point transform is split N = N1*N2 with N1 = 1024 (j = N2*j1 + j2, m = m1 + N1*m2).  One
// workgroup owns CP column pairs of one tensor of one unit for all tokens and streams over j2:
// it loads the N1 rows {N2*j1 + j2}, runs a register-resident 1024-point FFT (radix 16 x 16 x 4:
// two in-register radix-16 passes around one LDS exchange, the radix-4 across four lanes with
// DPP), and folds the result into the only 2*Q blocks of m2 that the low-pass keeps
// (Q = ceil(r/N1)), which live in registers for the whole stream.  After the filter it streams
// again, expands the kept blocks back (the transposed network), subtracts from the re-read rows,
// and writes one partial squared-residual sum per token; nothing but K/V (twice) and those
// partial sums ever touches HBM.  A small second kernel adds the partial sums of the column
// groups in a fixed order, un-permutes them into scores and reduces the energies in fp64.
//
// This file is compiled once per lane radix R = FC_FFT_R in {16, 8, 4, 2, 1}: the register-resident
// transform has N1 = 256*R points (radix 16 x 16 x R).  R = 2 and 1 let token counts that are
// multiples of 512 or 256 only take the fast path (the smaller N1, the more passes a given cut-off
// needs); R = 8 and 16 (4 and 2 column pairs per workgroup) cover 4096 and 8192 modes per pass and
// are chosen when that saves passes.  The R = 4 unit also holds everything that does not depend on R.
#include <algorithm>
#include <atomic>

#include "fc_common.h"

#ifndef FC_FFT_R
#define FC_FFT_R 4
#endif
#define FC_CAT2(a, b) a##b
#define FC_CAT(a, b) FC_CAT2(a, b)

namespace fc {

namespace {

constexpr int kR = FC_FFT_R;       // radix of the stage that runs across lanes
constexpr int kN1 = 256 * kR;      // points of the register-resident FFT
constexpr int kA = kN1 / 16;       // rows a thread group strides over in the first radix-16
constexpr int kMaxQ = 2;           // kept low blocks: r <= 2048
constexpr size_t kLdsLimit = 160 * 1024 - 256;   // dynamic LDS per workgroup: a compute unit's, minus the static reduction scratch
constexpr bool kTeInLds = kR >= 4; // the smaller transforms read w_N^(j2*e2) from the global table: more workgroups per CU
// float2 per row of the first twiddle table (16 used): a wave reads 64/CP rows at once, and the row
// stride keeps them on distinct banks - 18 for 8 rows (8 column pairs), 17 for 16 or 32 rows
constexpr int kT1Row = kR >= 8 ? 17 : 18;
constexpr int kT2Skew = kR == 16 ? 1 : 2;
// R >= 4: the stage across lanes returns its result times the lane's sign (-1)^popcount(a_lo) (both
// directions); the kernel multiplies that sign into a per-thread factor it applies afterwards anyway:
// w_N^(j2*m1base) of the fold (forward), the 1/N of the residual (inverse)
// (only where the written-out instructions leave the register allocation without spills: bf16
// storage, single or first pass; elsewhere the plain form runs)
template <typename T, int MODE> constexpr bool lane_signed() { return kR >= 4 && sizeof(T) == 2 && MODE <= 1; }   // float2 between the a_lo blocks of the second table: distinct banks

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
// a * w
__device__ __forceinline__ float2 cmul(float2 a, float2 w) {
  return make_float2(a.x * w.x - a.y * w.y, a.x * w.y + a.y * w.x);
}
// a * conj(w)
__device__ __forceinline__ float2 cmulc(float2 a, float2 w) {
  return make_float2(a.x * w.x + a.y * w.y, a.y * w.x - a.x * w.y);
}
template <bool CONJ> __device__ __forceinline__ float2 cmul_t(float2 a, float2 w) {
  return CONJ ? cmulc(a, w) : cmul(a, w);
}

// 4-point DFT in place (natural order in and out); forward uses exp(-i..), INV exp(+i..).
template <bool INV>
__device__ __forceinline__ void bfly4(float2& x0, float2& x1, float2& x2, float2& x3) {
  float2 t0 = cadd(x0, x2), t1 = csub(x0, x2), t2 = cadd(x1, x3), t3 = csub(x1, x3);
  x0 = cadd(t0, t2);
  x2 = csub(t0, t2);
  if (!INV) {
    x1 = make_float2(t1.x + t3.y, t1.y - t3.x);   // t1 - i t3
    x3 = make_float2(t1.x - t3.y, t1.y + t3.x);   // t1 + i t3
  } else {
    x1 = make_float2(t1.x - t3.y, t1.y + t3.x);
    x3 = make_float2(t1.x + t3.y, t1.y - t3.x);
  }
}

// 4-point DFT of (x0, w1*x1, w2*x2, w3*x3) in place, the factors folded into the first butterflies:
// a + w*b costs four FMAs and a - w*b = 2a - (a + w*b) two more, so a pair of twiddled butterflies
// takes 6 (one factor) or 10 (two factors) instructions instead of 8 or 12.  CW = the factors are
// to be conjugated (w given for the forward direction).
template <bool CW> __device__ __forceinline__ float2 cmul_w(float2 a, float2 w) { return CW ? cmulc(a, w) : cmul(a, w); }
// a + w*b  (w conjugated if CW)
template <bool CW> __device__ __forceinline__ float2 cfma_w(float2 a, float2 b, float2 w) {
  return CW ? make_float2(fmaf(w.y, b.y, fmaf(w.x, b.x, a.x)), fmaf(-w.y, b.x, fmaf(w.x, b.y, a.y)))
            : make_float2(fmaf(-w.y, b.y, fmaf(w.x, b.x, a.x)), fmaf(w.y, b.x, fmaf(w.x, b.y, a.y)));
}
__device__ __forceinline__ float2 twice_minus(float2 a, float2 t) {      // 2a - t
  return make_float2(fmaf(2.f, a.x, -t.x), fmaf(2.f, a.y, -t.y));
}
template <bool INV>
__device__ __forceinline__ void bfly4_tail(float2 t0, float2 t1, float2 t2, float2 t3, float2& x0, float2& x1,
                                           float2& x2, float2& x3) {
  x0 = cadd(t0, t2);
  x2 = csub(t0, t2);
  if (!INV) {
    x1 = make_float2(t1.x + t3.y, t1.y - t3.x);   // t1 - i t3
    x3 = make_float2(t1.x - t3.y, t1.y + t3.x);   // t1 + i t3
  } else {
    x1 = make_float2(t1.x - t3.y, t1.y + t3.x);
    x3 = make_float2(t1.x + t3.y, t1.y - t3.x);
  }
}
// x0 plain, x1..x3 with factors
template <bool INV, bool CW>
__device__ __forceinline__ void bfly4_w3(float2& x0, float2& x1, float2& x2, float2& x3, float2 w1, float2 w2,
                                         float2 w3) {
  const float2 t0 = cfma_w<CW>(x0, x2, w2), t1 = twice_minus(x0, t0);
  const float2 q = cmul_w<CW>(x1, w1);
  const float2 t2 = cfma_w<CW>(q, x3, w3), t3 = twice_minus(q, t2);
  bfly4_tail<INV>(t0, t1, t2, t3, x0, x1, x2, x3);
}
// all four with factors
template <bool INV, bool CW>
__device__ __forceinline__ void bfly4_w4(float2& x0, float2& x1, float2& x2, float2& x3, float2 w0, float2 w1,
                                         float2 w2, float2 w3) {
  const float2 p = cmul_w<CW>(x0, w0);
  const float2 t0 = cfma_w<CW>(p, x2, w2), t1 = twice_minus(p, t0);
  const float2 q = cmul_w<CW>(x1, w1);
  const float2 t2 = cfma_w<CW>(q, x3, w3), t3 = twice_minus(q, t2);
  bfly4_tail<INV>(t0, t1, t2, t3, x0, x1, x2, x3);
}

// Second half of the 16-point DFT: the factors w16^(n0*k0) and the 4-point DFTs over n0 for each
// k0 (elements 4*k0 + n0), then the transposition to natural order.
template <bool INV>
__device__ __forceinline__ void fft16_second_half(float2 (&x)[16]) {
  constexpr float C1 = 0.92387953251128673848f;   // cos(pi/8)
  constexpr float S1 = 0.38268343236508978178f;   // sin(pi/8)
  constexpr float H = 0.70710678118654752440f;    // sqrt(1/2)
  const float2 w1 = make_float2(C1, -S1), w2 = make_float2(H, -H), w3 = make_float2(S1, -C1),
               w6 = make_float2(-H, -H), w9 = make_float2(-C1, S1);
  bfly4<INV>(x[0], x[1], x[2], x[3]);
  bfly4_w3<INV, INV>(x[4], x[5], x[6], x[7], w1, w2, w3);
  {  // k0 = 2: factors w16^2, w16^4 = -i (+i inverse), w16^6
    const float2 x0 = x[8], xb = x[10];
    const float2 t0 = INV ? make_float2(x0.x - xb.y, x0.y + xb.x) : make_float2(x0.x + xb.y, x0.y - xb.x);
    const float2 t1 = INV ? make_float2(x0.x + xb.y, x0.y - xb.x) : make_float2(x0.x - xb.y, x0.y + xb.x);
    const float2 q = cmul_w<INV>(x[9], w2);
    const float2 t2 = cfma_w<INV>(q, x[11], w6), t3 = twice_minus(q, t2);
    bfly4_tail<INV>(t0, t1, t2, t3, x[8], x[9], x[10], x[11]);
  }
  bfly4_w3<INV, INV>(x[12], x[13], x[14], x[15], w3, w6, w9);
  // X[k0 + 4*k1] sits at 4*k0 + k1: transpose to natural order
  float2 y[16];
#pragma unroll
  for (int k0 = 0; k0 < 4; ++k0)
#pragma unroll
    for (int k1 = 0; k1 < 4; ++k1) y[k0 + 4 * k1] = x[4 * k0 + k1];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = y[i];
}

// 16-point DFT, natural order in and out, fully in registers (4 x 4 Cooley-Tukey).
template <bool INV>
__device__ __forceinline__ void fft16(float2 (&x)[16]) {
  // 4-point DFTs over n1 for each n0 (inputs n0, n0+4, n0+8, n0+12); result k0 at n0+4*k0
#pragma unroll
  for (int n0 = 0; n0 < 4; ++n0) bfly4<INV>(x[n0], x[n0 + 4], x[n0 + 8], x[n0 + 12]);
  fft16_second_half<INV>(x);
}

// The same transform of (x[0], tw[1]*x[1], ..., tw[15]*x[15]) - or, with W0, of tw[i]*x[i] for all
// i - with the factors folded into the first butterflies.  `tw` may sit in LDS with stride TS
// between entries; CW: the factors are conjugated first.
template <bool INV, bool CW, bool W0, int TS>
__device__ __forceinline__ void fft16_tw(float2 (&x)[16], const float2* tw) {
  if (W0) bfly4_w4<INV, CW>(x[0], x[4], x[8], x[12], tw[0], tw[4 * TS], tw[8 * TS], tw[12 * TS]);
  else bfly4_w3<INV, CW>(x[0], x[4], x[8], x[12], tw[4 * TS], tw[8 * TS], tw[12 * TS]);
#pragma unroll
  for (int n0 = 1; n0 < 4; ++n0)
    bfly4_w4<INV, CW>(x[n0], x[n0 + 4], x[n0 + 8], x[n0 + 12], tw[n0 * TS], tw[(n0 + 4) * TS],
                      tw[(n0 + 8) * TS], tw[(n0 + 12) * TS]);
  fft16_second_half<INV>(x);
}

template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kQuadXor1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int kQuadXor2 = 0x4E;   // quad_perm:[2,3,0,1]

// 4-point DFT across the four lanes of a quad.  Forward: lane a holds input a, afterwards lane l
// holds output bitrev2(l).  Inverse: lane l holds input bitrev2(l), afterwards lane a holds output a.
template <bool INV>
__device__ __forceinline__ float2 quad_dft4(float2 v, float sgn_hi, float sgn_lo, bool lane3) {
  if (!INV) {
    float2 t = make_float2(fmaf(v.x, sgn_hi, dpp_f<kQuadXor2>(v.x)), fmaf(v.y, sgn_hi, dpp_f<kQuadXor2>(v.y)));
    if (lane3) t = make_float2(t.y, -t.x);                       // -i t
    return make_float2(fmaf(t.x, sgn_lo, dpp_f<kQuadXor1>(t.x)), fmaf(t.y, sgn_lo, dpp_f<kQuadXor1>(t.y)));
  } else {
    float2 t = make_float2(fmaf(v.x, sgn_lo, dpp_f<kQuadXor1>(v.x)), fmaf(v.y, sgn_lo, dpp_f<kQuadXor1>(v.y)));
    if (lane3) t = make_float2(-t.y, t.x);                       // +i t
    return make_float2(fmaf(t.x, sgn_hi, dpp_f<kQuadXor2>(t.x)), fmaf(t.y, sgn_hi, dpp_f<kQuadXor2>(t.y)));
  }
}

// x[i] += partner(x[i]) * sgn for 16 registers, the partner lane read through DPP: one v_fmac each.
// (The compiler keeps a DPP move and an FMA apart when it is given the same expression, so the
// instruction is written out.  The leading s_nop covers the two wait states a DPP read needs after
// a vector write of its source register, which the compiler's hazard pass cannot see in here.)
#define FC_DPP_FMAC16(PERM)                                                                             \
  asm volatile("s_nop 1\n\t"                                                                            \
               "v_fmac_f32_dpp %0, %0, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %1, %1, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %2, %2, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %3, %3, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %4, %4, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %5, %5, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %6, %6, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %7, %7, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %8, %8, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %9, %9, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %10, %10, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
               "v_fmac_f32_dpp %11, %11, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
               "v_fmac_f32_dpp %12, %12, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
               "v_fmac_f32_dpp %13, %13, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
               "v_fmac_f32_dpp %14, %14, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"      \
               "v_fmac_f32_dpp %15, %15, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1"            \
               : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(x4), "+v"(x5), "+v"(x6), "+v"(x7), "+v"(x8),  \
                 "+v"(x9), "+v"(x10), "+v"(x11), "+v"(x12), "+v"(x13), "+v"(x14), "+v"(x15)                  \
               : "v"(sgn))
template <int KIND>        // partner lane: 0 = xor 1, 1 = xor 2 (inside a quad), 2 = 8 away inside a row of 16
__device__ __forceinline__ void dpp_fmac16(float& x0, float& x1, float& x2, float& x3, float& x4, float& x5,
                                           float& x6, float& x7, float& x8, float& x9, float& x10, float& x11,
                                           float& x12, float& x13, float& x14, float& x15, float sgn) {
  if (KIND == 1) FC_DPP_FMAC16("quad_perm:[2,3,0,1]");
  else if (KIND == 0) FC_DPP_FMAC16("quad_perm:[1,0,3,2]");
  else FC_DPP_FMAC16("row_ror:8");
}
#undef FC_DPP_FMAC16
// x[i] += dpp(y[i]) * sgn for 8 registers, source and destination apart (for butterflies whose partner
// needs two permutations: the first is an ordinary DPP move, the second rides in the v_fmac)
#define FC_DPP_FMAC8_SRC(PERM)                                                                          \
  asm volatile("s_nop 1\n\t"                                                                            \
               "v_fmac_f32_dpp %0, %8, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %1, %9, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"        \
               "v_fmac_f32_dpp %2, %10, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"       \
               "v_fmac_f32_dpp %3, %11, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"       \
               "v_fmac_f32_dpp %4, %12, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"       \
               "v_fmac_f32_dpp %5, %13, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"       \
               "v_fmac_f32_dpp %6, %14, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"       \
               "v_fmac_f32_dpp %7, %15, %16 " PERM " row_mask:0xf bank_mask:0xf bound_ctrl:1"            \
               : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(x4), "+v"(x5), "+v"(x6), "+v"(x7)             \
               : "v"(y0), "v"(y1), "v"(y2), "v"(y3), "v"(y4), "v"(y5), "v"(y6), "v"(y7), "v"(sgn))
// x[i] += (value of x[i] in the lane 4 away inside a group of 8) * sgn
__device__ __forceinline__ void xor4_fmac8(float& x0, float& x1, float& x2, float& x3, float& x4, float& x5,
                                           float& x6, float& x7, float sgn) {
  const float y0 = dpp_f<0x141>(x0), y1 = dpp_f<0x141>(x1), y2 = dpp_f<0x141>(x2), y3 = dpp_f<0x141>(x3),
              y4 = dpp_f<0x141>(x4), y5 = dpp_f<0x141>(x5), y6 = dpp_f<0x141>(x6), y7 = dpp_f<0x141>(x7);
  FC_DPP_FMAC8_SRC("quad_perm:[3,2,1,0]");
}
#undef FC_DPP_FMAC8_SRC
#define FC_X16(v, m) v[0].m, v[1].m, v[2].m, v[3].m, v[4].m, v[5].m, v[6].m, v[7].m, v[8].m, v[9].m, v[10].m, \
                     v[11].m, v[12].m, v[13].m, v[14].m, v[15].m

// The 4-point DFT across the four lanes of a quad for 16 values at once, up to a per-lane sign: the
// result is sgn_hi*sgn_lo times quad_dft4's.  A butterfly v*sgn + partner needs the partner moved
// in and then an FMA; written as v + partner*sgn (= sgn times the former, sgn = +-1) it is one
// v_fmac reading the partner through DPP.  Both partners of the second butterfly carry the same
// sign from the first, so the signs multiply through; the caller folds the product into a factor
// it applies anyway.
//
// The factor -i (forward) / +i (inverse) that lane 3 of a quad takes between the two butterflies is a
// swap of its real and imaginary registers plus one negation.  The negation is not executed: lane 3
// keeps its imaginary part negated on the side of the swap that faces the caller (the output of the
// forward transform, the input of the inverse one), and the butterfly with lane 2 that lies on that
// side multiplies the imaginary parts by -sgn_lo on both lanes (sgn_lo_y), which keeps lane 2 exact
// and lane 3 negated.  The caller accounts for it in the complex multiplication it performs next to
// the transform anyway (kConjLane3 at the kernel).  The swap is one v_swap_b32 per value under the
// lane mask.
__device__ __forceinline__ void swap16(float2 (&v)[16]) {
#pragma unroll
  for (int i = 0; i < 16; ++i) asm volatile("v_swap_b32 %0, %1" : "+v"(v[i].x), "+v"(v[i].y));
}
template <bool INV>
__device__ __forceinline__ void quad_dft4_signed16(float2 (&v)[16], float sgn_hi, float sgn_lo, float sgn_lo_y,
                                                   bool lane3) {
  if (!INV) {
    dpp_fmac16<1>(FC_X16(v, x), sgn_hi);
    dpp_fmac16<1>(FC_X16(v, y), sgn_hi);
    if (lane3) swap16(v);                                        // (y, x) = -i t with the imaginary part negated
    dpp_fmac16<0>(FC_X16(v, x), sgn_lo);
    dpp_fmac16<0>(FC_X16(v, y), sgn_lo_y);
  } else {
    dpp_fmac16<0>(FC_X16(v, x), sgn_lo);
    dpp_fmac16<0>(FC_X16(v, y), sgn_lo_y);
    if (lane3) swap16(v);                                        // (-y, x) = +i t, exact
    dpp_fmac16<1>(FC_X16(v, x), sgn_hi);
    dpp_fmac16<1>(FC_X16(v, y), sgn_hi);
  }
}

// value of the lane 4 away inside a group of 8 lanes: mirror of the 8 lanes, then reversal of each quad
constexpr int kQuadReverse = 0x1B;   // quad_perm:[3,2,1,0]
__device__ __forceinline__ float lane_xor4(float v) { return dpp_f<kQuadReverse>(dpp_f<0x141>(v)); }

// value of the lane 8 away inside a row of 16 lanes
__device__ __forceinline__ float lane_xor8(float v) { return dpp_f<0x128>(v); }   // row_ror:8

// Per-lane constants of the stage that runs across R lanes.
struct LaneConsts {
  float sgn_hex, sgn_oct, sgn_hi, sgn_lo;   // -1 on the lanes whose bit 3 / 2 / 1 / 0 of a_lo is set
  float sgn_lo_y;                  // sgn_lo, negated on the lanes 2 and 3 of a quad (signed form only)
  bool lane3;                      // (a_lo & 3) == 3: takes the factor -i between the two quad stages
  float2 tw8;                      // R >= 8: w_8^(a_lo & 3) on the lanes with bit 2 set, 1 elsewhere
  float2 tw16;                     // R = 16: w_16^(a_lo & 7) on the lanes with bit 3 set, 1 elsewhere
};

// The R-point DFT across R adjacent lanes.  R = 4: the quad transform above.  R = 8: one butterfly
// across the lanes 4 apart with the factor w_8^(a & 3) on its lower outputs, then the quad
// transform on each half (forward: lane a holds input a, afterwards lane l holds output bitrev3(l);
// the inverse is the transposed network).  R = 2: one butterfly across a lane pair.  R = 1: nothing.
template <bool INV>
__device__ __forceinline__ float2 lane_dft(float2 v, const LaneConsts& lc) {
  const float sgn_hi = lc.sgn_hi, sgn_lo = lc.sgn_lo;
  const bool lane3 = lc.lane3;
  if (kR >= 8) {                   // R = 16: one more butterfly, across the lanes 8 apart, outside
    if (!INV) {
      if (kR == 16) {
        v = make_float2(fmaf(v.x, lc.sgn_hex, lane_xor8(v.x)), fmaf(v.y, lc.sgn_hex, lane_xor8(v.y)));
        v = cmul(v, lc.tw16);
      }
      float2 t = make_float2(fmaf(v.x, lc.sgn_oct, lane_xor4(v.x)), fmaf(v.y, lc.sgn_oct, lane_xor4(v.y)));
      t = cmul(t, lc.tw8);
      return quad_dft4<false>(t, sgn_hi, sgn_lo, lane3);
    } else {
      float2 t = quad_dft4<true>(v, sgn_hi, sgn_lo, lane3);
      t = cmulc(t, lc.tw8);
      t = make_float2(fmaf(t.x, lc.sgn_oct, lane_xor4(t.x)), fmaf(t.y, lc.sgn_oct, lane_xor4(t.y)));
      if (kR == 16) {
        t = cmulc(t, lc.tw16);
        t = make_float2(fmaf(t.x, lc.sgn_hex, lane_xor8(t.x)), fmaf(t.y, lc.sgn_hex, lane_xor8(t.y)));
      }
      return t;
    }
  }
  if (kR == 4) return quad_dft4<INV>(v, sgn_hi, sgn_lo, lane3);
  if (kR == 2) return make_float2(fmaf(v.x, sgn_lo, dpp_f<kQuadXor1>(v.x)), fmaf(v.y, sgn_lo, dpp_f<kQuadXor1>(v.y)));
  return v;
}

// The stage across lanes for a thread's 16 values.  R >= 4: the signed form (see kLaneSigned), every
// butterfly v + partner*sgn; the per-lane factors w_8^., w_16^. between the butterflies commute with
// the signs, and both partners of every later butterfly carry equal signs from the earlier ones,
// so the result is the transform times (-1)^popcount(a_lo).
template <bool INV, bool SIGNED>
__device__ __forceinline__ void lane_dft16(float2 (&v)[16], const LaneConsts& lc) {
  if (SIGNED) {
    if (!INV) {
      if (kR == 16) {
        dpp_fmac16<2>(FC_X16(v, x), lc.sgn_hex);
        dpp_fmac16<2>(FC_X16(v, y), lc.sgn_hex);
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = cmul(v[i], lc.tw16);
      }
      if (kR >= 8) {
        xor4_fmac8(v[0].x, v[1].x, v[2].x, v[3].x, v[4].x, v[5].x, v[6].x, v[7].x, lc.sgn_oct);
        xor4_fmac8(v[8].x, v[9].x, v[10].x, v[11].x, v[12].x, v[13].x, v[14].x, v[15].x, lc.sgn_oct);
        xor4_fmac8(v[0].y, v[1].y, v[2].y, v[3].y, v[4].y, v[5].y, v[6].y, v[7].y, lc.sgn_oct);
        xor4_fmac8(v[8].y, v[9].y, v[10].y, v[11].y, v[12].y, v[13].y, v[14].y, v[15].y, lc.sgn_oct);
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = cmul(v[i], lc.tw8);
      }
      quad_dft4_signed16<false>(v, lc.sgn_hi, lc.sgn_lo, lc.sgn_lo_y, lc.lane3);
    } else {
      quad_dft4_signed16<true>(v, lc.sgn_hi, lc.sgn_lo, lc.sgn_lo_y, lc.lane3);
      if (kR >= 8) {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = cmulc(v[i], lc.tw8);
        xor4_fmac8(v[0].x, v[1].x, v[2].x, v[3].x, v[4].x, v[5].x, v[6].x, v[7].x, lc.sgn_oct);
        xor4_fmac8(v[8].x, v[9].x, v[10].x, v[11].x, v[12].x, v[13].x, v[14].x, v[15].x, lc.sgn_oct);
        xor4_fmac8(v[0].y, v[1].y, v[2].y, v[3].y, v[4].y, v[5].y, v[6].y, v[7].y, lc.sgn_oct);
        xor4_fmac8(v[8].y, v[9].y, v[10].y, v[11].y, v[12].y, v[13].y, v[14].y, v[15].y, lc.sgn_oct);
      }
      if (kR == 16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = cmulc(v[i], lc.tw16);
        dpp_fmac16<2>(FC_X16(v, x), lc.sgn_hex);
        dpp_fmac16<2>(FC_X16(v, y), lc.sgn_hex);
      }
    }
  } else {
#pragma unroll
    for (int bh = 0; bh < 16; ++bh) v[bh] = lane_dft<INV>(v[bh], lc);
  }
}

// One row element of a thread: two adjacent feature columns, as stored.
template <typename T> struct RawPair;
template <> struct RawPair<uint16_t> {
  typedef uint32_t type;
  static __device__ __forceinline__ float2 unpack(uint32_t u) {
    return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xFFFF0000u));
  }
  static __device__ __forceinline__ uint32_t zero() { return 0u; }
  // acc + a^2 + b^2 of the two stored values: one packed-bf16 dot product (the products of bf16
  // values are exact in fp32)
  static __device__ __forceinline__ float sumsq(uint32_t u, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    union { uint32_t u; bf16x2 v; } c;
    c.u = u;
    return __builtin_amdgcn_fdot2_f32_bf16(c.v, c.v, acc, false);
  }
};
template <> struct RawPair<float> {
  typedef float2 type;
  static __device__ __forceinline__ float2 unpack(float2 u) { return u; }
  static __device__ __forceinline__ float2 zero() { return make_float2(0.f, 0.f); }
  static __device__ __forceinline__ float sumsq(float2 u, float acc) { return fmaf(u.y, u.y, fmaf(u.x, u.x, acc)); }
};

template <int CTRL> __device__ __forceinline__ float dpp_add(float v) { return v + dpp_f<CTRL>(v); }

// u[i] = s[i] + (s[i] of lane 7-c) on the lanes c < 4 of every eight, s[i+8] + (s[i+8] of lane 7-c) on
// the lanes c >= 4: the first add runs on all lanes and is right for the lower four, the second is
// written by the banks of the upper four only (a DPP bank is four lanes).
__device__ __forceinline__ void half_mirror_fold8(const float (&s)[16], float (&u)[8]) {
#define FC_HM(i, a, b)                                                                         \
  "v_add_f32_dpp %" #i ", %" #a ", %" #a " row_half_mirror row_mask:0xf bank_mask:0xf\n\t"    \
  "v_add_f32_dpp %" #i ", %" #b ", %" #b " row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
  asm volatile("s_nop 1\n\t"
               FC_HM(0, 8, 16) FC_HM(1, 9, 17) FC_HM(2, 10, 18) FC_HM(3, 11, 19)
               FC_HM(4, 12, 20) FC_HM(5, 13, 21) FC_HM(6, 14, 22) FC_HM(7, 15, 23)
               : "=&v"(u[0]), "=&v"(u[1]), "=&v"(u[2]), "=&v"(u[3]), "=&v"(u[4]), "=&v"(u[5]), "=&v"(u[6]),
                 "=&v"(u[7])
               : "v"(s[0]), "v"(s[1]), "v"(s[2]), "v"(s[3]), "v"(s[4]), "v"(s[5]), "v"(s[6]), "v"(s[7]),
                 "v"(s[8]), "v"(s[9]), "v"(s[10]), "v"(s[11]), "v"(s[12]), "v"(s[13]), "v"(s[14]), "v"(s[15]));
#undef FC_HM
}

constexpr int kRowHalfMirror = 0x141;

#if FC_FFT_R == 4
// ------------------------------------------------------------------ tables (step A1)
// twn[k] = exp(-2 pi i k / N), k < N;  phase[m] = exp(+i pi m / N), m < N
__global__ void fft_table_kernel(WsHeader* hdr, float2* __restrict__ twn, float2* __restrict__ phase, int n,
                                 int r, int d, int dtype) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx == 0) {
    hdr->magic = kWsMagic; hdr->path = FC_PATH_FFT; hdr->n = n; hdr->r = r; hdr->d = d;
    hdr->dtype = dtype; hdr->error = 0;
  }
  if (idx < n) {
    double s, c;
    sincospi(2.0 * (double)idx / (double)n, &s, &c);
    twn[idx] = make_float2((float)c, (float)(-s));
  }
  if (idx < n) {
    double s, c;
    sincospi((double)idx / (double)n, &s, &c);
    phase[idx] = make_float2((float)c, (float)s);
  }
}

#endif  // FC_FFT_R == 4

// w_8^k, k < 4, and w_16^k, k < 8 (read once per thread; in memory rather than built on the stack)
__device__ const float2 kW8[4] = {{1.f, 0.f}, {0.70710678118654752440f, -0.70710678118654752440f}, {0.f, -1.f},
                                  {-0.70710678118654752440f, -0.70710678118654752440f}};
__device__ const float2 kW16[8] = {{1.f, 0.f},
                                   {0.92387953251128673848f, -0.38268343236508978178f},
                                   {0.70710678118654752440f, -0.70710678118654752440f},
                                   {0.38268343236508978178f, -0.92387953251128673848f},
                                   {0.f, -1.f},
                                   {-0.38268343236508978178f, -0.92387953251128673848f},
                                   {-0.70710678118654752440f, -0.70710678118654752440f},
                                   {-0.92387953251128673848f, -0.38268343236508978178f}};

// ------------------------------------------------------------------ main kernel
// (N1 = 256*R points per register-resident transform, n2 = N / N1; "1024" below is the R = 4 case.)
// LDS: the twiddle tables, each laid out so that a thread reads its 15 factors of a stage from one
// base address with constant offsets, then one or two exchange buffers (two: they alternate per
// FFT, so one barrier per FFT suffices):
//   T1[a][e]            = w_N1^(a*e)                   after the first radix-16   (rows padded to 18)
//   T2[a_lo][j2][b_hi]  = w_N^(16*b_hi*(n2*a_lo + j2)) before the radix-R stage   (a_lo blocks 2 apart)
//   TE[j2][e2] * TF[j2][b_lo] = w_N^(j2*m1base)        the fold multiplier of the thread's modes
//                                                      (TE only for R >= 4; else read from the global table)
// The factor w_n2^(j2*blk) that distinguishes the kept blocks is uniform and comes from the global
// table through scalar loads.
//
// Cut-offs above 2*N1 modes are handled in passes of at most two low blocks each (q0 = first low
// block of the pass).  The projections of the passes are onto disjoint mode sets, so every pass
// transforms the stored input itself and the parts add up in an fp32 buffer [unit][K|V][N][d]:
//   MODE 0  only pass: squared-residual partial sums straight from the registers
//   MODE 1  first of several: buffer = part            (a workgroup owns its columns for all
//   MODE 2  middle:           buffer += part            tokens, so the update is race-free)
//   MODE 3  last:             partial sums of (input - buffer - part)^2
// The frequency N1*q0 pairs with N - N1*q0, which lies one block above this pass's high
// blocks; one extra accumulator per thread (meaningful only in the thread that owns m1 = 0)
// carries it when q0 > 0.
//
// Cut-offs above N/2 (cmode = 1).  A frequency pair (m, N-m) of the packed transform carries the
// DCT modes m and N-m of both columns.  For r <= N/2 the filter keeps mode m of the pairs m < r and
// drops everything else.  For r > N/2 only the modes N-m with 1 <= m <= N-r are dropped, so the
// kernel computes that high-pass part directly: the same blocks with cut-off rcut = N-r+1 and the
// complementary in-pair projector  R[m] = 1/2 (W[m] - e^{+i pi m/N} W[N-m]),  R[N-m] = -e^{-i pi m/N} R[m],
// R[0] = 0; its inverse transform is input - base itself, so the last stage squares the summed
// parts without subtracting them from the input.
//
// The first pass with two low blocks (FIRST, Q = 2: blocks 0, 1 and their mirrors -1, -2) shares
// the per-thread multiplier t = v * w_N^(j2*m1) between the blocks: the block factors w_n2^(j2*blk)
// are uniform, and after half a block step is taken out of t (one complex multiplication per step)
// the blocks 0 / -1 and +1 / -2 carry conjugate factors, so the sum and the difference of each pair
// are accumulated with one real multiplier each (PAIR below): 12 instead of 16 instructions per
// point, in both directions.
template <typename T, int CP, int Q, int MODE, int NBUF>
__global__ __launch_bounds__(kA * CP) __attribute__((amdgpu_waves_per_eu(2, 2))) void fft_score_kernel(
    const T* K, const T* V, KvStrides st, int n, int n2, int r, int rcut, int cmode, int d, int dtype,
    int q0, int n_ut, int slabs, int n_items, int ph_lds, WsHeader* hdr, const float2* __restrict__ twn,
    const float2* __restrict__ phase_arg, float* partial, double* __restrict__ etot_part, float* resid) {
  typedef typename RawPair<T>::type Raw;
  constexpr int NT = kA * CP;
  constexpr int PAD = (CP < 8) ? 16 : 0;
  constexpr int S = kA * CP + PAD;          // float2 stride between e-planes of an exchange buffer
  constexpr int XB = 16 * S;                // float2 per exchange buffer (>= kN1*CP)
  constexpr int NB = 2 * Q;                 // kept blocks: low q0+q, high n2-1-(q0+q), q < Q
  constexpr bool FIRST = MODE <= 1;         // the pass with q0 = 0
  constexpr bool SCORE = MODE == 0 || MODE == 3;
#ifdef FC_FFT_NOPIPE                          // experiment build: the two halves of a step never overlap
  constexpr bool PIPE = false;
#else
  // (not for the passes that also carry the fp32 parts of earlier passes, nor for fp32 storage:
  // the extra 32 live registers of the overlapped half would spill there)
  constexpr bool PIPE = NBUF == 2 && MODE <= 1 && sizeof(T) == 2;
#endif
#ifdef FC_FFT_NOPAIR                          // experiment build: the generic fold everywhere
  constexpr bool PAIR = false;
#else
  constexpr bool PAIR = FIRST && Q == 2;
#endif
  constexpr bool kLaneSigned = lane_signed<T, MODE>();
  if (ws_mismatch(hdr, FC_PATH_FFT, n, r, d, dtype)) return;

  extern __shared__ float2 smem[];
  // tables first: their reads then fit the 16-bit offset field of the LDS instructions
  float2* T1 = smem;
  float2* T2 = T1 + kA * kT1Row;
  float2* TE = T2 + kR * (n2 * 16 + kT2Skew);
  float2* TF = TE + (kTeInLds ? n2 * 16 : 0);
  float2* xchg = TF + n2 * kR;             // NBUF = 2: exchange buffers alternate, one barrier per FFT
  __shared__ double red[NT / 64];

  const int tid0 = threadIdx.x;
  {
    const int tid = tid0;
  for (int i = tid; i < kA * 16; i += NT) T1[(i >> 4) * kT1Row + (i & 15)] = twn[(i >> 4) * (i & 15) * n2];
  for (int i = tid; i < 16 * kR * n2; i += NT) {
    const int al = i / (16 * n2), rem = i - al * 16 * n2;         // rem = 16*j2 + b_hi
    T2[al * (n2 * 16 + kT2Skew) + rem] = twn[16 * (rem & 15) * (n2 * al + (rem >> 4))];
  }
  if (kTeInLds)
    for (int i = tid; i < 16 * n2; i += NT) TE[i] = twn[(i >> 4) * (i & 15)];
  for (int i = tid; i < kR * n2; i += NT) TF[i] = twn[256 * (i / kR) * (i % kR)];
  }

  // Persistent workgroups: the grid is what the device holds at once, and every workgroup walks the
  // column groups bid = blockIdx.x, blockIdx.x + gridDim.x, ... with its tables built once (a new
  // workgroup per column group would leave the compute unit empty while it is set up: the kept
  // blocks and the exchange buffers take all registers and LDS, so no second one can wait beside it).
  // XCD-aware placement: the `slabs` column groups of one tensor go to consecutive slots of one XCD;
  // gridDim.x is a multiple of 8, so a workgroup's column groups all belong to its own XCD.
  for (int bid = blockIdx.x; bid < n_items; bid += gridDim.x) {
  // (the thread index and the pointer to the filter's table are made opaque per column group:
  // everything derived from them - coordinates, the filter's per-thread table reads and conditions -
  // would otherwise be hoisted out of this loop and held in registers the streams need.  The
  // twiddle table keeps its declared pointer: its uniform reads stay scalar loads only as long as
  // the compiler knows that nothing writes there.)
  const float2* phase = phase_arg;
  int tid = tid0;
  asm volatile("" : "+s"(phase), "+v"(tid));
  __builtin_assume(tid >= 0 && tid < NT);
  // phase-1 coordinates (loads, first radix-16): rows j1 = a + kA*k, column pair c
  const int a = tid / CP, c = tid % CP;
  // phase-2 coordinates (second radix-16, radix R across lanes, kept blocks)
  const int a_lo = tid & (kR - 1), c2 = (tid / kR) % CP, e2 = tid / (kR * CP);
  const int b_lo = kR == 16  ? (((a_lo & 1) << 3) | ((a_lo & 2) << 1) | ((a_lo & 4) >> 1) | (a_lo >> 3))
                   : kR == 8 ? (((a_lo & 1) << 2) | (a_lo & 2) | (a_lo >> 2))
                   : kR == 4 ? (((a_lo & 1) << 1) | (a_lo >> 1))
                             : a_lo;
  const int m1base = e2 + 256 * b_lo;       // m1 = m1base + 16*b_hi
  LaneConsts lc;
  lc.sgn_hex = (a_lo & 8) ? -1.f : 1.f;
  lc.sgn_oct = (a_lo & 4) ? -1.f : 1.f;
  lc.sgn_hi = (a_lo & 2) ? -1.f : 1.f;
  lc.sgn_lo = (a_lo & 1) ? -1.f : 1.f;
  lc.sgn_lo_y = (a_lo & 2) ? -lc.sgn_lo : lc.sgn_lo;
  lc.lane3 = (a_lo & 3) == 3;
  const float lane_sign = (__popc(a_lo) & 1) ? -1.f : 1.f;
  // signed form: lane 3 of every quad hands over / expects its values with the imaginary part negated
  // (see quad_dft4_signed16); where conj3 holds, the factors that meet those imaginary parts change sign
  const bool conj3 = kLaneSigned && lc.lane3;
  lc.tw8 = (a_lo & 4) ? kW8[a_lo & 3] : make_float2(1.f, 0.f);
  lc.tw16 = (a_lo & 8) ? kW16[a_lo & 7] : make_float2(1.f, 0.f);
  const int buf_t = a * CP + c;             // + kA*CP*k within a step
  const int lds_w1 = a * CP + c;                                  // + e*S
  const int lds_r1 = e2 * S + a_lo * CP + c2;                     // + kR*CP*a_hi
  const float2* t1 = T1 + a * kT1Row;                              // w_N1^(a*e), e = 0..15 (writer side)
  const float2* t1r = T1 + a_lo * kT1Row + e2;                     // w_N1^((a_lo + R*ah)*e2), stride R rows
  const float2* t2base = T2 + a_lo * (n2 * 16 + kT2Skew);
  const float2* te = TE + e2;
  const float2* tf = TF + b_lo;

  const int xcd = bid & 7, kk = bid >> 3;
  const int slab = kk % slabs;
  const int ut = (kk / slabs) * 8 + xcd;
  if (ut >= n_ut) continue;                 // (uniform: the whole workgroup skips)
  const int unit = ut >> 1, tensor = ut & 1;
  const T* x = (tensor ? V : K) + unit_offset(st, unit);
  const int col = 2 * (slab * CP + c);      // first of this thread's two feature columns (phase 1)

  // This thread's rows: k < 8 are even tokens 2*(n2*(a+kA*k)+j2), k >= 8 odd tokens
  // 2n-1-2*(n2*(a+kA*k)+j2).  With D = 2*kA*n2 tokens, row k < 8 lies k*D above the thread's first even
  // row and, because 2n = 16*D, row k >= 8 lies (15-k)*D above its lowest odd row: the 16 loads of a
  // step share 8 uniform base pointers and two per-thread 32-bit byte offsets, one rising and one
  // falling in j2.
  const char* xbytes = reinterpret_cast<const char*>(x);
  const uint32_t esz = (uint32_t)sizeof(T), sn = (uint32_t)st.sn;
  const uint32_t jstep = 2u * sn * esz;
  const uint32_t even0 = (2u * (uint32_t)(n2 * a) * sn + (uint32_t)col) * esz;
  const uint32_t odd0 = ((uint32_t)(2 * kA * n2 - 1 - 2 * n2 * a) * sn + (uint32_t)col) * esz;
  const int64_t row_bytes = (int64_t)st.sn * (int64_t)sizeof(T);
  const char* xk[8];
  // (set once per stream: the eight pointers then need no register between the streams, where the
  // filter wants the scalar registers for itself)
  auto set_row_pointers = [&]() {
    int64_t step = (int64_t)(2 * kA * n2) * row_bytes;
    asm volatile("" : "+s"(step));            // keeps the two computations apart
#pragma unroll
    for (int k = 0; k < 8; ++k) xk[k] = xbytes + step * k;
  };
  set_row_pointers();
#define FC_ROW_PTR(k, j2v) ((k) < 8 ? xk[k] + (size_t)(even0 + (uint32_t)(j2v) * jstep) \
                                    : xk[15 - (k)] + (size_t)(odd0 - (uint32_t)(j2v) * jstep))
  // the fp32 buffer of MODE 1-3 is private to the passes, so it is laid out the way this kernel
  // walks it: [tensor][column group][j2][j1][column pair] float2 - a step is one contiguous 8*1024*CP
  // bytes, every access a full line
  float2* buf = reinterpret_cast<float2*>(resid) + ((size_t)ut * slabs + slab) * (size_t)n * CP;
  // The 4096-point transform owns only 8 bytes of every row, so a wave-load touches 32 cache lines;
  // its forward stream (single pass) therefore leaves the rows it read in the same private region,
  // in walking order, and the inverse stream re-reads them from there as full lines (measured at
  // 32768 tokens: 4.12 -> 3.96 ms; for the 2048-point transform the same costs more than it saves).
#ifdef FC_FFT_STAGEREAD                       // timing experiment: both streams read a staged copy nobody wrote
  constexpr bool kStage = kR >= 8 && MODE == 0;
  constexpr bool kPre = true;
#else
  constexpr bool kStage = kR == 16 && MODE == 0;
  constexpr bool kPre = false;
#endif
  Raw* stage = reinterpret_cast<Raw*>(resid) + ((size_t)ut * slabs + slab) * (size_t)n * CP;

  float2 acc[NB][16];
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[q][i] = make_float2(0.f, 0.f);
  float etot_f = 0.f;                       // this thread's share of the input energy (fp32; fp64 from the wave sum on)

  Raw raw[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) raw[k] = *reinterpret_cast<const Raw*>(FC_ROW_PTR(k, 0));
  // block q of this pass and its uniform factor index: jb[q] = j2*blk mod n2, kept incrementally
  int blk[NB], jb[NB];
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    blk[q] = (q < Q) ? (q0 + q) : (n2 - 1 - (q0 + q - Q));
    jb[q] = 0;
  }
  // the extra entry: block n2 - q0 at m1 = 0, used by the m1 = 0 thread when q0 > 0
  const int blkx = (q0 > 0) ? n2 - q0 : 0;
  int jbx = 0;
  float2 accx = make_float2(0.f, 0.f);
  __syncthreads();

  // ================================================================ forward stream
  // A step has two halves around the exchange through LDS.  Head: this step's rows -> first
  // radix-16 -> twiddle -> exchange buffer.  Tail: exchange buffer -> second radix-16 -> twiddle ->
  // radix-R across lanes -> fold into the kept blocks.  With two exchange buffers (PIPE) the loop is
  // software-pipelined: an iteration issues the LDS reads of step j2's tail, runs the head of step
  // j2 + 1 (which is independent of them) while they arrive, then the tail, so that the LDS
  // transfers of both halves overlap vector-ALU work of the same wave; one barrier per iteration.
  auto fwd_head = [&](int j2) {
    float2* xb = xchg + (j2 & (NBUF - 1)) * XB;
    float2 v[16];
    float ss = 0.f;
    if (kStage && !cmode && !kPre) {
      Raw* sstep = stage + (size_t)j2 * (kN1 * CP) + buf_t;
#pragma unroll
      for (int k = 0; k < 16; ++k) sstep[kA * CP * k] = raw[k];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      v[k] = RawPair<T>::unpack(raw[k]);
      if (FIRST) ss = RawPair<T>::sumsq(raw[k], ss);   // the input's energy: recorded by the first pass only
    }
    etot_f += ss;
    // the stored rows are unpacked before the next ones are requested, so that those land in the same
    // registers (left to itself the scheduler requests them earlier and copies all sixteen)
    // (not for the 4096-point transform, whose narrow row segments want their loads as early as possible)
    if (kR < 16) {
#pragma unroll
      for (int k = 0; k < 16; ++k) asm volatile("" : "+v"(v[k].x), "+v"(v[k].y));
      __builtin_amdgcn_sched_barrier(0);
    }
#ifndef FC_FFT_NOLOAD                         // (timing experiment: every step re-uses the first rows)
    // rows of the next step fly during this step's arithmetic.  (The last step loads its own rows
    // again: without a condition the loads land in the registers the loop carries, with one the
    // compiler copies all sixteen twice per step.  The 4096-point transform, which has few steps and
    // waits on its loads, keeps the condition.)
    if (kR < 16 || j2 + 1 < n2) {
      const int jn = j2 + 1 < n2 ? j2 + 1 : j2;
      if (kStage && kPre) {
        const Raw* sstep = stage + (size_t)jn * (kN1 * CP) + buf_t;
#pragma unroll
        for (int k = 0; k < 16; ++k) raw[k] = sstep[kA * CP * k];
      } else {
#pragma unroll
        for (int k = 0; k < 16; ++k)
          raw[k] = *reinterpret_cast<const Raw*>(FC_ROW_PTR(k, jn));
      }
    }
#endif
    fft16<false>(v);                        // (its twiddle w_N1^(a*e) is applied by the reading side)
#pragma unroll
    for (int e = 0; e < 16; ++e) xb[lds_w1 + e * S] = v[e];
  };
  auto fwd_tail = [&](int j2, float2 (&v)[16]) {
    // v[ah] is element (e2, a = a_lo + R*ah) of the first radix-16's output: its factor w_N1^(a*e2)
    // is folded into the first butterflies of the second one
    fft16_tw<false, false, true, kR * kT1Row>(v, t1r);
    const float2* t2 = t2base + 16 * j2;
#pragma unroll
    for (int bh = 1; bh < 16; ++bh) v[bh] = cmul(v[bh], t2[bh]);
    lane_dft16<false, kLaneSigned>(v, lc);
    // fold into the kept blocks: W[m1 + N1*blk] += v * w_N^(j2*(m1base + N1*blk))
    float2 tq = cmul(kTeInLds ? te[16 * j2] : twn[j2 * e2], tf[kR * j2]);         // w_N^(j2*m1base)
    if (kLaneSigned) tq = make_float2(tq.x * lane_sign, tq.y * lane_sign);
    // factors applied to v.y (v.y is the negated imaginary part on the lanes with conj3)
    const float2 tqy = conj3 ? make_float2(-tq.x, -tq.y) : tq;
    if constexpr (PAIR) {
      // with u = w_(2*n2)^j2 (u^2 = w_n2^j2) and t' = t*conj(u), the blocks 0, -1, +1, -2 receive
      // t'*u, t'*conj(u), t'*u^3, t'*conj(u^3): two conjugate pairs, each accumulated as its sum
      // (real multiplier 2 Re) and its difference (imaginary multiplier 2i Im):
      // acc[0] = block 0 + block -1, acc[2] = block 0 - block -1, acc[1] = block 1 + block -2,
      // acc[3] = block 1 - block -2
      const float2 u1 = twn[j2 * (kN1 / 2)];                                   // uniform
      const int j3 = 3 * j2 * (kN1 / 2);
      const float2 u3 = twn[j3 >= n ? j3 - n : j3];
      const float c0 = 2.f * u1.x, d0 = 2.f * u1.y, c1 = 2.f * u3.x, d1 = 2.f * u3.y;
      const float2 tp = cmulc(tq, u1), tpy = cmulc(tqy, u1);                  // tq * conj(u)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float2 t = make_float2(fmaf(v[i].x, tp.x, -v[i].y * tpy.y), fmaf(v[i].x, tp.y, v[i].y * tpy.x));
        acc[0][i].x = fmaf(t.x, c0, acc[0][i].x);
        acc[0][i].y = fmaf(t.y, c0, acc[0][i].y);
        acc[2][i].x = fmaf(-t.y, d0, acc[2][i].x);
        acc[2][i].y = fmaf(t.x, d0, acc[2][i].y);
        acc[1][i].x = fmaf(t.x, c1, acc[1][i].x);
        acc[1][i].y = fmaf(t.y, c1, acc[1][i].y);
        acc[3][i].x = fmaf(-t.y, d1, acc[3][i].x);
        acc[3][i].y = fmaf(t.x, d1, acc[3][i].y);
      }
    } else {
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const float2 mq = cmul(tq, twn[jb[q] * kN1]);
        const float2 my = conj3 ? make_float2(-mq.x, -mq.y) : mq;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          acc[q][i].x = fmaf(v[i].x, mq.x, fmaf(-v[i].y, my.y, acc[q][i].x));
          acc[q][i].y = fmaf(v[i].x, mq.y, fmaf(v[i].y, my.x, acc[q][i].y));
        }
        jb[q] += blk[q];
        if (jb[q] >= n2) jb[q] -= n2;
      }
      if constexpr (!FIRST) {
        const float2 mx = cmul(tq, twn[jbx * kN1]);
        accx.x = fmaf(v[0].x, mx.x, fmaf(-v[0].y, mx.y, accx.x));
        accx.y = fmaf(v[0].x, mx.y, fmaf(v[0].y, mx.x, accx.y));
        jbx += blkx;
        if (jbx >= n2) jbx -= n2;
      }
    }
  };
  if constexpr (PIPE) {
    fwd_head(0);
    __syncthreads();
    for (int j2 = 0; j2 < n2; ++j2) {
      const float2* xb = xchg + (j2 & 1) * XB;
      float2 w[16];
#pragma unroll
      for (int ah = 0; ah < 16; ++ah) w[ah] = xb[lds_r1 + kR * CP * ah];
      if (j2 + 1 < n2) fwd_head(j2 + 1);    // writes the other buffer
      fwd_tail(j2, w);
      __syncthreads();                      // the other buffer is complete; this one may be overwritten
    }
  } else {
    for (int j2 = 0; j2 < n2; ++j2) {
      const float2* xb = xchg + (j2 & (NBUF - 1)) * XB;
      fwd_head(j2);
      __syncthreads();
      float2 w[16];
#pragma unroll
      for (int ah = 0; ah < 16; ++ah) w[ah] = xb[lds_r1 + kR * CP * ah];
      if (NBUF == 1) __syncthreads();       // single buffer: everyone has read before the next write
      fwd_tail(j2, w);
    }
  }

  // ================================================================ low-pass filter on the kept blocks
  // low block q pairs with high block n2-1-q at the mirrored m1 (and, for m1 = 0, with the m1 = 0
  // entry of high block n2-q, which this same thread holds).
  float2* xbuf = xchg;
  const float csg = cmode ? -1.f : 1.f;       // sign of the in-pair projector (see the header comment)
  // The filter's factors e^{i pi m/N} of this pass's modes (m0 <= m < min(rcut, m0 + Q*N1)): the
  // workgroup copies them into LDS with one coalesced read - into the second exchange buffer, which is
  // idle here, or, with one buffer, into a region of its own behind it when the launch found room
  // (ph_lds).  (Read from the table in memory, one entry at a time by every wave of every workgroup at
  // the same moment, the same few hundred cache lines cost 10 us per column group.)
  const int m0 = kN1 * q0;
  const float2* ph = phase + m0;              // indexed by m - m0
  if (NBUF == 2 || ph_lds) {
    if (NBUF == 2 && !PIPE) __syncthreads();  // (the unpipelined loop ends without one: a wave may still read its last step)
    float2* phl = xchg + XB;                  // NBUF = 2: the second buffer; NBUF = 1: the region behind the only one
    const int cnt = min(rcut, m0 + Q * kN1) - m0;
    for (int i = tid; i < cnt; i += NT) phl[i] = phase[m0 + i];
    ph = phl;                                 // (visible after the first barrier below)
  }
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    __syncthreads();
    if constexpr (PAIR) {                   // sum and difference of this pair -> its two blocks
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float2 p = acc[q][i], m = acc[Q + q][i];
        acc[q][i] = make_float2(0.5f * (p.x + m.x), 0.5f * (p.y + m.y));
        acc[Q + q][i] = make_float2(0.5f * (p.x - m.x), 0.5f * (p.y - m.y));
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) xbuf[(m1base + 16 * i) * CP + c2] = acc[Q + q][i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m1 = m1base + 16 * i;
      const int m = m1 + kN1 * (q0 + q);
      float2 w = acc[q][i], out = make_float2(0.f, 0.f);
      if (m == 0) {
        if (!cmode) out = w;
      } else if (m < rcut) {
        float2 wn;
        if (m1 != 0) wn = xbuf[(kN1 - m1) * CP + c2];
        else if (q > 0) wn = acc[Q + (q > 0 ? q - 1 : 0)][0];  // m1 == 0 implies i == 0
        else wn = accx;                                         // q == 0, q0 > 0
        const float2 t = cmul(wn, ph[m - m0]);
        out = make_float2(0.5f * fmaf(csg, t.x, w.x), 0.5f * fmaf(csg, t.y, w.y));
      }
      acc[q][i] = out;
    }
  }
  // energy of the kept DCT coefficients of this pass's blocks (Eq. 11 as written): for a column
  // pair |C_a[m]|^2 + |C_b[m]|^2 = alpha[m]^2 |W^[m]|^2, alpha^2 = 1/N for m = 0 and 2/N otherwise
  float elow_f = 0.f;
#pragma unroll
  for (int q = 0; q < Q; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float wgt = (m1base + 16 * i + kN1 * (q0 + q) == 0) ? 1.f : 2.f;
      elow_f = fmaf(wgt, fmaf(acc[q][i].x, acc[q][i].x, acc[q][i].y * acc[q][i].y), elow_f);
    }
  asm volatile("" : "+v"(elow_f));            // (summed here, while the filtered blocks are in registers)
  double elow = (double)elow_f;
  // the mirror of 1024*q0 (only the m1 = 0 thread has a meaningful value; zero elsewhere)
  accx = make_float2(0.f, 0.f);
  if (m1base == 0 && q0 > 0 && kN1 * q0 < rcut) {
    const float2 t = cmulc(acc[0][0], ph[0]);
    accx = make_float2(csg * t.x, csg * t.y);
  }
  // all low blocks are filtered before any high block is rebuilt from them
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) xbuf[(m1base + 16 * i) * CP + c2] = acc[q][i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m1 = m1base + 16 * i;
      float2 out = make_float2(0.f, 0.f);
      if (m1 != 0) {
        const int ml = (kN1 - m1) + kN1 * (q0 + q);             // the low mode this high entry mirrors
        if (ml < rcut) out = cmulc(xbuf[(kN1 - m1) * CP + c2], ph[ml - m0]);
      } else if (q + 1 < Q) {
        const int ml = kN1 * (q0 + q + 1);
        if (ml < rcut) out = cmulc(acc[q + 1][0], ph[ml - m0]);
      }
      acc[Q + q][i] = make_float2(csg * out.x, csg * out.y);
    }
  }
  __syncthreads();
  if constexpr (PAIR) {                     // the four blocks -> sums and differences of the conjugate pairs
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float2 lo = acc[q][i], hi = acc[2 + q][i];
        acc[q][i] = make_float2(lo.x + hi.x, lo.y + hi.y);
        acc[2 + q][i] = make_float2(lo.x - hi.x, lo.y - hi.y);
      }
  }

  // ================================================================ inverse stream + scoring
  // 1/N, times the sign the stage across lanes left on this thread's rows when it runs in its signed
  // form: rows a + kA*k come from the lanes with a_lo = a mod R, whose sign is uniform for the thread
  const float inv_n = ((kLaneSigned && (__popc(a & (kR - 1)) & 1)) ? -1.f : 1.f) / (float)n;
  set_row_pointers();
  float* part = partial + ((size_t)ut * slabs + slab) * (size_t)n;
  // jb[q] is back at n2*blk mod n2 = 0; each head below first moves it one step back.
  // Head: kept blocks -> radix-R across lanes -> twiddle -> radix-16 -> exchange buffer.  Tail:
  // exchange buffer -> twiddle -> radix-16 -> residual against the re-read rows (or the fp32 buffer
  // of a multi-pass cut-off).  Pipelined like the forward stream when there are two buffers.
  auto load_rows = [&](int j2) {
    // this step's rows, needed only where the residual is formed (with cmode the summed parts
    // are the residual itself: zero rows stand in for the input)
    if (SCORE && !cmode) {
#ifdef FC_FFT_NOLOAD
      if (j2 != n2 - 1) return;
#endif
      if (kStage) {
        const Raw* sstep = stage + (size_t)j2 * (kN1 * CP) + buf_t;
#pragma unroll
        for (int k = 0; k < 16; ++k) raw[k] = sstep[kA * CP * k];
      } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) raw[k] = *reinterpret_cast<const Raw*>(FC_ROW_PTR(k, j2));
      }
    }
  };
  if (SCORE && cmode) {                     // the zero rows are set once and never loaded over
#pragma unroll
    for (int k = 0; k < 16; ++k) raw[k] = RawPair<T>::zero();
  }
  auto inv_head = [&](int j2) {
    float2* xb = xchg + (j2 & (NBUF - 1)) * XB;
    float2 v[16];
    const float2 tq = cmul(kTeInLds ? te[16 * j2] : twn[j2 * e2], tf[kR * j2]);   // w_N^(j2*m1base)
    // factors that produce v.y (handed over negated on the lanes with conj3)
    const float2 tqy = conj3 ? make_float2(-tq.x, -tq.y) : tq;
    if constexpr (PAIR) {
      // W0 + W1 conj(s) + W-1 s + W-2 s^2 (s = u^2) = u * (W0 conj(u) + W-1 u + W1 conj(u^3) + W-2 u^3),
      // each pair = Re * sum - i Im * difference; the leading u joins conj(t): u conj(tq) = conj(tq conj(u))
      const float2 u1 = twn[j2 * (kN1 / 2)];
      const int j3 = 3 * j2 * (kN1 / 2);
      const float2 u3 = twn[j3 >= n ? j3 - n : j3];
      const float2 tp = cmulc(tq, u1), tpy = cmulc(tqy, u1);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float2 in;
        in.x = fmaf(u1.y, acc[2][i].y, u1.x * acc[0][i].x);
        in.y = fmaf(-u1.y, acc[2][i].x, u1.x * acc[0][i].y);
        in.x = fmaf(u3.x, acc[1][i].x, fmaf(u3.y, acc[3][i].y, in.x));
        in.y = fmaf(u3.x, acc[1][i].y, fmaf(-u3.y, acc[3][i].x, in.y));
        v[i].x = fmaf(in.x, tp.x, in.y * tp.y);
        v[i].y = fmaf(in.y, tpy.x, -in.x * tpy.y);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = make_float2(0.f, 0.f);
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        jb[q] -= blk[q];
        if (jb[q] < 0) jb[q] += n2;
        const float2 mq = cmul(tq, twn[jb[q] * kN1]);
        const float2 my = conj3 ? make_float2(-mq.x, -mq.y) : mq;
#pragma unroll
        for (int i = 0; i < 16; ++i) {                            // v += acc * conj(mq)
          v[i].x = fmaf(acc[q][i].x, mq.x, fmaf(acc[q][i].y, mq.y, v[i].x));
          v[i].y = fmaf(acc[q][i].y, my.x, fmaf(-acc[q][i].x, my.y, v[i].y));
        }
      }
      if constexpr (!FIRST) {
        jbx -= blkx;
        if (jbx < 0) jbx += n2;
        const float2 mx = cmul(tq, twn[jbx * kN1]);
        v[0].x = fmaf(accx.x, mx.x, fmaf(accx.y, mx.y, v[0].x));
        v[0].y = fmaf(accx.y, mx.x, fmaf(-accx.x, mx.y, v[0].y));
      }
    }
    lane_dft16<true, kLaneSigned>(v, lc);
    const float2* t2 = t2base + 16 * j2;
    fft16_tw<true, true, false, 1>(v, t2);  // conj(t2[bh]) * v[bh], folded into the transform
#pragma unroll
    for (int ah = 0; ah < 16; ++ah) xb[lds_r1 + kR * CP * ah] = v[ah];
  };
  auto inv_tail = [&](int j2, float2 (&v)[16], const float2 (&prev)[16]) {
    float2* bstep = buf + (size_t)j2 * (kN1 * CP) + buf_t;
    fft16_tw<true, true, false, 1>(v, t1);  // conj(t1[e]) * v[e], folded into the transform
    // v[k] = N * (this pass's part) at permuted position j = n2*(a + 64k) + j2, columns col, col+1
    if (MODE >= 2) {                        // sum of the parts so far
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        v[k].x = fmaf(v[k].x, inv_n, prev[k].x);
        v[k].y = fmaf(v[k].y, inv_n, prev[k].y);
      }
    } else if (MODE == 1) {
#pragma unroll
      for (int k = 0; k < 16; ++k) { v[k].x *= inv_n; v[k].y *= inv_n; }
    }
    if (!SCORE) {
#pragma unroll
      for (int k = 0; k < 16; ++k) bstep[kA * CP * k] = v[k];
    } else {
      float sq[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const float2 xv = RawPair<T>::unpack(raw[k]);
        const float dx = MODE == 0 ? fmaf(-v[k].x, inv_n, xv.x) : xv.x - v[k].x;
        const float dy = MODE == 0 ? fmaf(-v[k].y, inv_n, xv.y) : xv.y - v[k].y;
        sq[k] = fmaf(dx, dx, dy * dy);
      }
      if constexpr (CP == 8) {
        // Sum over the 8 lanes that hold a row's column pairs, as a transposing reduction: every
        // exchange halves the rows a lane still carries (34 instructions for the 16 rows, against 64
        // for 16 full reductions and the selection of the rows a lane stores).  Lanes c and 7-c first:
        // c < 4 keeps rows 0-7, c >= 4 rows 8-15 (two DPP adds per row pair, the second written by the
        // upper four lanes of every eight only); then the lanes 2 apart, then neighbours, after which
        // lane c holds rows 2c and 2c+1.
        float u[8];
        half_mirror_fold8(sq, u);
        const bool b1 = (c & 2) != 0, b0 = (c & 1) != 0;
        float w[4], z[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (b1 ? u[i + 4] : u[i]) + dpp_f<kQuadXor2>(b1 ? u[i] : u[i + 4]);
#pragma unroll
        for (int i = 0; i < 2; ++i) z[i] = (b0 ? w[i + 2] : w[i]) + dpp_f<kQuadXor1>(b0 ? w[i] : w[i + 2]);
        part[j2 * kN1 + a + kA * (2 * c)] = z[0];
        part[j2 * kN1 + a + kA * (2 * c + 1)] = z[1];
      } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          sq[k] = dpp_add<kQuadXor1>(sq[k]);
          if (CP >= 4) sq[k] = dpp_add<kQuadXor2>(sq[k]);   // sum over this workgroup's 2*CP columns, in every lane
        }
        // lane c stores rows k = c, c+CP, ...: all lanes take part in every store
#pragma unroll
        for (int g = 0; g < 16 / CP; ++g) {
          float val = sq[g * CP];
#pragma unroll
          for (int cc = 1; cc < CP; ++cc) val = (c == cc) ? sq[g * CP + cc] : val;
          part[j2 * kN1 + a + kA * (g * CP + c)] = val;
        }
      }
    }
  };
  // the parts of the earlier passes (MODE >= 2; their loads fly during the transform)
  auto load_prev = [&](int j2, float2 (&prev)[16]) {
    if (MODE >= 2) {
      const float2* bstep = buf + (size_t)j2 * (kN1 * CP) + buf_t;
#pragma unroll
      for (int k = 0; k < 16; ++k) prev[k] = bstep[kA * CP * k];
    }
  };
  if constexpr (PIPE) {
    load_rows(n2 - 1);
    inv_head(n2 - 1);
    __syncthreads();
    for (int j2 = n2 - 1; j2 >= 0; --j2) {
      const float2* xb = xchg + (j2 & 1) * XB;
      float2 w[16], prev[16];
      load_prev(j2, prev);
#pragma unroll
      for (int e = 0; e < 16; ++e) w[e] = xb[lds_w1 + e * S];
      if (j2 > 0) inv_head(j2 - 1);         // writes the other buffer
      inv_tail(j2, w, prev);
      if (j2 > 0) load_rows(j2 - 1);        // consumed by the next iteration's tail
      __syncthreads();
    }
  } else {
    for (int j2 = n2 - 1; j2 >= 0; --j2) {
      const float2* xb = xchg + (j2 & (NBUF - 1)) * XB;
      float2 w[16], prev[16];
      load_rows(j2);
      load_prev(j2, prev);
      inv_head(j2);
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 16; ++e) w[e] = xb[lds_w1 + e * S];
      if (NBUF == 1) __syncthreads();
      inv_tail(j2, w, prev);
    }
  }

#undef FC_ROW_PTR
  // total energy and kept-coefficient energy of this column group (fp64 sums in a fixed order of the
  // threads' fp32 shares)
  double etot = (double)etot_f;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    etot += __shfl_xor(etot, off, 64);
    elow += __shfl_xor(elow, off, 64);
  }
  __shared__ double red2[NT / 64];
  if ((tid & 63) == 0) { red[tid >> 6] = etot; red2[tid >> 6] = elow; }
  __syncthreads();
  if (tid == 0) {
    double s = 0.0, s2 = 0.0;
    for (int w = 0; w < NT / 64; ++w) { s += red[w]; s2 += red2[w]; }
    double* rec = etot_part + ((size_t)ut * slabs + slab) * 2;
    s2 /= (double)n;
    if (q0 == 0) { rec[0] = s; rec[1] = s2; }       // only the first pass sees the input itself
    else rec[1] += s2;                                 // later passes add their blocks (same owner)
  }
  }  // next column group of this workgroup
}

#if FC_FFT_R == 4
// ------------------------------------------------------------------ finalize
// Adds the per-column-group partial sums (fixed order), un-permutes them into scores and writes
// per-workgroup fp64 partials of the high-pass energies.  A workgroup owns 32 values of j1 below
// n1/2 (even tokens) and the mirrored 32 above (odd tokens), i.e. one contiguous span of 64*n2
// tokens: partial sums are read coalesced along j1, transposed through LDS, written coalesced.
// n1 = points of the register-resident transform the partial sums come from; grid.x = n1/64.
constexpr int kFinJ1 = 32;

__global__ __launch_bounds__(256) void fft_finalize_kernel(
    const float* __restrict__ partial, const double* __restrict__ etot_part, int n, int n1, int n2, int r,
    int d, int dtype, int slabs, WsHeader* hdr, float* __restrict__ scores, double* __restrict__ epart,
    UnitMap um) {
  extern __shared__ float span[];             // 64*n2 scores
  __shared__ double sm[2][256];
  if (ws_mismatch(hdr, FC_PATH_FFT, n, r, d, dtype)) return;
  const int tile = blockIdx.x, unit = blockIdx.y;
  const float* pk = partial + (size_t)(unit * 2 + 0) * slabs * n;
  const float* pv = partial + (size_t)(unit * 2 + 1) * slabs * n;
  const int t0 = 2 * kFinJ1 * n2 * tile;      // first token of the span
  const float inv_d = 1.0f / (float)d;
  double hk = 0.0, hv = 0.0;
  const int items = 2 * n2 * kFinJ1;
  // four neighbouring j1 per thread: 16-byte reads (the partial sums start 256-byte aligned and n, n1
  // and kFinJ1 are multiples of 4)
  constexpr int kQuads = kFinJ1 / 4;
  for (int it = threadIdx.x; it < items / 4; it += 256) {
    const int j1q = it % kQuads, j2 = (it / kQuads) % n2, half = it / (kQuads * n2);
    const int j1 = (half ? n1 - kFinJ1 * (tile + 1) : kFinJ1 * tile) + 4 * j1q;
    const size_t idx = (size_t)j2 * n1 + j1;
    float4 sk = make_float4(0.f, 0.f, 0.f, 0.f), sv = sk;
    for (int s = 0; s < slabs; ++s) {
      const float4 a = *reinterpret_cast<const float4*>(pk + (size_t)s * n + idx);
      const float4 b = *reinterpret_cast<const float4*>(pv + (size_t)s * n + idx);
      sk.x += a.x; sk.y += a.y; sk.z += a.z; sk.w += a.w;
      sv.x += b.x; sv.y += b.y; sv.z += b.z; sv.w += b.w;
    }
    const float ks[4] = {sk.x, sk.y, sk.z, sk.w}, vs[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = n2 * (j1 + e) + j2;
      const int tok = (2 * j < n) ? 2 * j : 2 * n - 2 * j - 1;
      span[tok - t0] = ks[e] * inv_d + vs[e] * inv_d;
      hk += (double)ks[e];
      hv += (double)vs[e];
    }
  }
  sm[0][threadIdx.x] = hk;
  sm[1][threadIdx.x] = hv;
  __syncthreads();
  float* sout = scores + out_unit(um, unit) * n + t0;
  for (int i = threadIdx.x; i < items; i += 256) sout[i] = span[i];
  for (int s = 128; s >= 1; s >>= 1) {
    if (threadIdx.x < s) {
      sm[0][threadIdx.x] += sm[0][threadIdx.x + s];
      sm[1][threadIdx.x] += sm[1][threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double* o = epart + ((size_t)unit * gridDim.x + tile) * 4;
    double tk = 0.0, tv = 0.0;
    if (tile == 0) {
      for (int s = 0; s < slabs; ++s) {
        tk += etot_part[((size_t)(unit * 2 + 0) * slabs + s) * 2];
        tv += etot_part[((size_t)(unit * 2 + 1) * slabs + s) * 2];
      }
    }
    o[0] = sm[0][0]; o[1] = sm[1][0]; o[2] = tk; o[3] = tv;
  }
}

// Geometry is a pure function of the shape and the cut-off.  Only a library built with
// -DFC_FFT_KNOBS (an experiment build, never the product) lets the environment override it, to time
// the variants the product does not pick: FLASHCACHE_FFT_CP=4 (4 column pairs per workgroup on the
// 1024-point kernel), FLASHCACHE_FFT_WIDE=0/1/2 (never a wider kernel / the 2048-point / the
// 4096-point kernel wherever it applies), FLASHCACHE_FFT_NBUF=1 (one exchange buffer).
#ifdef FC_FFT_KNOBS
int knob(const char* name) {
  const char* env = getenv(name);
  return (env && env[0] >= '0' && env[0] <= '9') ? env[0] - '0' : -1;
}
#else
constexpr int knob(const char*) { return -1; }
#endif

int pick_cp(const fc_kv_desc& d) {
  const int pairs = d.head_dim / 2;
  if (knob("FLASHCACHE_FFT_CP") == 4 && pairs % 4 == 0) return 4;
  return pairs % 8 == 0 ? 8 : 4;
}

// Lane radix by token count: multiples of 1024, of 512, of 256; 0 = no fast path.
int lane_radix(int n) { return n % 1024 == 0 ? 4 : (n % 512 == 0 ? 2 : (n % 256 == 0 ? 1 : 0)); }
int passes_for(int rcut, int n1) { return ((rcut + n1 - 1) / n1 + kMaxQ - 1) / kMaxQ; }

// Two exchange buffers (one barrier per FFT) while they fit beside the twiddle tables: 1024-point
// transforms with 8 column pairs up to 32768 tokens.  Otherwise one buffer: with 4 column pairs
// (35 KB) or the smaller transforms, so that several workgroups share a CU.
int exchange_buffers(int lr, int cp, int n) {
  if (knob("FLASHCACHE_FFT_NBUF") == 1) return 1;
  return (lr == 4 && cp == 8 && n <= 32 * 1024) ? 2 : 1;
}

#endif  // FC_FFT_R == 4

}  // namespace

#if FC_FFT_R == 4
// Dynamic LDS of the main kernel: exchange buffer(s), then the four twiddle tables.
size_t fft_lds_bytes(int lr, int cp, int nbuf, int n2) {
  const int a = 16 * lr, pad = cp < 8 ? 16 : 0, skew = lr == 16 ? 1 : 2;
  const int t1row = lr >= 8 ? 17 : 18;
  return ((size_t)nbuf * 16 * (a * cp + pad) + a * t1row + lr * (n2 * 16 + skew) +
          (lr >= 4 ? n2 * 16 : 0) + n2 * lr) * sizeof(float2);
}

// The 2048- and 4096-point transforms (lane radix 8 / 16, 4 / 2 column pairs per workgroup) cost
// about 1.4 / 2.15 passes of the 1024-point one (measured at 32768 tokens; the narrow column groups
// make their row loads expensive) and cover 2 / 4 times the modes: the geometry with the least
// estimated cost is taken (ties to the smaller transform).
static bool wide_applies(const fc_kv_desc& d, int lr) {
  const int n = d.n_tokens, n1 = 256 * lr, cp = 32 / lr;
  return n % n1 == 0 && (d.head_dim / 2) % cp == 0 && fft_lds_bytes(lr, cp, 1, n / n1) <= kLdsLimit &&
         (size_t)64 * (n / n1) * sizeof(float) <= 64 * 1024;
}

static inline int fft_cutoff(int n, int r, bool* complement);

// lane radix and column pairs per workgroup for this shape and cut-off; lr = 0: no fast path
static void fft_geometry(const fc_kv_desc& d, int32_t r, int* lr, int* cp) {
  bool cm;
  *lr = lane_radix(d.n_tokens);
  *cp = pick_cp(d);
  if (*lr < 4) *cp = (d.head_dim / 2) % 8 == 0 ? 8 : 4;     // (the experiment knob applies to R = 4 only)
  if (*lr != 4 || r < 1 || r > d.n_tokens) return;
  const int rcut = fft_cutoff(d.n_tokens, r, &cm);
  const int wide = knob("FLASHCACHE_FFT_WIDE");
  int pick = 4;
  if (wide == 0) {
  } else if (wide == 1) {
    if (wide_applies(d, 8)) pick = 8;
  } else if (wide == 2) {
    if (wide_applies(d, 16)) pick = 16;
  } else {
    int best = 100 * passes_for(rcut, 1024);
    if (wide_applies(d, 8) && 138 * passes_for(rcut, 2048) < best) { best = 138 * passes_for(rcut, 2048); pick = 8; }
    if (wide_applies(d, 16) && 215 * passes_for(rcut, 4096) < best) { best = 215 * passes_for(rcut, 4096); pick = 16; }
  }
  if (pick != 4) { *lr = pick; *cp = 32 / pick; }
}

bool fft_supported(const fc_kv_desc& d, int32_t r) {
  const int n = d.n_tokens;
  if (d.head_dim % 8 != 0) return false;
  int lr, cp;
  fft_geometry(d, r, &lr, &cp);
  if (lr == 0) return false;
  const int n2 = n / (256 * lr);
  if (lr < 4 && cp != 8) return false;              // the smaller transforms exist for 8 column pairs only
  if (fft_lds_bytes(lr, cp, exchange_buffers(lr, cp, n), n2) > kLdsLimit) return false;
  if ((size_t)64 * n2 * sizeof(float) > 64 * 1024) return false;   // span buffer of the finalize kernel
  // (cut-offs above N/2 run in complement mode with cut-off N-r+1 <= N/2, see fft_cutoff)
  if (r < 1 || r > n) return false;
  // the kernels index rows of one tensor with 32-bit byte offsets
  if (2 * (int64_t)n * d.stride_n * (d.dtype == FC_BF16 ? 2 : 4) >= ((int64_t)1 << 32)) return false;
  if (2 * (int64_t)n * d.head_dim * 4 >= ((int64_t)1 << 32)) return false;
  return true;
}

// The cut-off the kernel's filter works with, and whether it computes the dropped part (r > N/2)
// instead of the kept part.  Either way a mode and its mirror N-m are different frequencies.
static inline int fft_cutoff(int n, int r, bool* complement) {
  *complement = 2 * r > n;
  return *complement ? n - r + 1 : r;
}

FftLayout fft_layout(const fc_kv_desc& d, int32_t r) {
  FftLayout lay{};
  const size_t units = (size_t)d.batch * d.layers * d.kv_heads;
  int lr, cp;
  fft_geometry(d, r, &lr, &cp);
  lay.slabs = d.head_dim / 2 / cp;
  lay.lane_radix = lr;
  const int n1 = 256 * lay.lane_radix;
  lay.tiles = n1 / 2 / kFinJ1;
  bool cm;
  const int q = (fft_cutoff(d.n_tokens, r, &cm) + n1 - 1) / n1;
  lay.passes = (q + kMaxQ - 1) / kMaxQ;
  auto up = [](size_t x) { return (x + kWsAlign - 1) / kWsAlign * kWsAlign; };
  size_t off = sizeof(WsHeader);
  lay.twiddle = off; off = up(off + (size_t)d.n_tokens * sizeof(float2));
  lay.phase = off; off = up(off + (size_t)d.n_tokens * sizeof(float2));
  lay.partial = off; off = up(off + units * 2 * lay.slabs * d.n_tokens * sizeof(float));
  lay.etot = off; off = up(off + units * 2 * lay.slabs * 2 * sizeof(double));
  lay.epart = off; off = up(off + units * lay.tiles * 4 * sizeof(double));
  // for several passes: the fp32 sum of the passes' parts.  For a single pass of the 4096-point
  // kernel: a copy of the input in the kernel's own walking order (see kStage at the kernel)
  lay.resid = off;
  if (lay.passes > 1) off = up(off + units * 2 * (size_t)d.n_tokens * d.head_dim * sizeof(float));
#ifdef FC_FFT_STAGEREAD
  else if (lay.lane_radix >= 8)
#else
  else if (lay.lane_radix == 16)
#endif
    off = up(off + units * 2 * (size_t)d.n_tokens * d.head_dim * (d.dtype == FC_BF16 ? 2 : 4));
  lay.total = off;
  return lay;
}

// lowpass[unit][t] = sum over column groups of the kept-coefficient energies (fixed order)
// (in complement mode the kernels record the energy of the dropped coefficients, Eq. 12's
// numerator as written, and the kept energy is the total minus that)
__global__ void fft_lowpass_kernel(const double* __restrict__ epair, int slabs, int n_ut, int cmode,
                                   double* __restrict__ lowpass) {
  const int ut = blockIdx.x * blockDim.x + threadIdx.x;
  if (ut >= n_ut) return;
  double s = 0.0;
  for (int k = 0; k < slabs; ++k) {
    const double* rec = epair + ((size_t)ut * slabs + k) * 2;
    s += cmode ? rec[0] - rec[1] : rec[1];
  }
  lowpass[ut] = s;
}

hipError_t fft_lowpass(const fc_kv_desc& d, int32_t r, const FftLayout& lay, void* ws, double* lowpass,
                       hipStream_t s) {
  const int n_ut = d.batch * d.layers * d.kv_heads * 2;
  bool cm;
  fft_cutoff(d.n_tokens, r, &cm);
  ProfileScope ps("fft_lowpass_kernel", s);
  hipLaunchKernelGGL(fft_lowpass_kernel, dim3((n_ut + 255) / 256), dim3(256), 0, s,
                     reinterpret_cast<const double*>(static_cast<char*>(ws) + lay.etot), lay.slabs, n_ut,
                     cm ? 1 : 0, lowpass);
  return hipGetLastError();
}

hipError_t fft_prepare(const fc_kv_desc& d, int32_t r, const FftLayout& lay, void* ws, hipStream_t s) {
  char* base = static_cast<char*>(ws);
  const int n = d.n_tokens;
  hipLaunchKernelGGL(fft_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s,
                     reinterpret_cast<WsHeader*>(base), reinterpret_cast<float2*>(base + lay.twiddle),
                     reinterpret_cast<float2*>(base + lay.phase), n, r, d.head_dim, d.dtype);
  return hipGetLastError();
}

#endif  // FC_FFT_R == 4

namespace {

typedef FftPassArgs PassArgs;

template <typename T, int CP, int Q, int MODE, int NBUF>
hipError_t launch_pass(const PassArgs& a, hipStream_t s) {
  constexpr int PAD = (CP < 8) ? 16 : 0;
  size_t shmem = ((size_t)NBUF * 16 * (kA * CP + PAD) + kA * kT1Row + kR * (a.n2 * 16 + kT2Skew) +
                  (kTeInLds ? a.n2 * 16 : 0) + a.n2 * kR) * sizeof(float2);
  // workgroups a compute unit holds at once: registers allow two waves per SIMD, LDS is 160 KB
  constexpr int kWavesPerWg = kA * CP / 64;
  auto wgs_per_cu = [](size_t lds) {
    const int by_lds = (int)((160 * 1024) / (lds + 512));
    return std::max(1, std::min(by_lds, 8 / (kWavesPerWg > 0 ? kWavesPerWg : 1)));
  };
  // room for the filter's factors behind a single exchange buffer, if the compute unit's LDS has it
  // without costing a resident workgroup
  int ph_lds = 0;
  {
    const size_t with = shmem + (size_t)Q * kN1 * sizeof(float2);
    if (NBUF == 1 && with <= kLdsLimit && wgs_per_cu(with) == wgs_per_cu(shmem)) {
      ph_lds = Q * kN1;
      shmem = with;
    }
  }
  auto kern = fft_score_kernel<T, CP, Q, MODE, NBUF>;
  // raising the dynamic LDS limit is per kernel and per device, and idempotent: do it once for each
  static std::atomic<uint64_t> attr_done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
  const uint64_t bit = 1ull << (dev & 63);
  if (!(attr_done.load(std::memory_order_acquire) & bit)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256);
    if (e != hipSuccess) return e;
    attr_done.fetch_or(bit, std::memory_order_release);
  }
  // one workgroup per slot the device has, each walking its share of the n_items column groups; both
  // counts are multiples of 8
  const int n_items = (a.n_ut + 7) / 8 * 8 * a.slabs;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return hipErrorInvalidDevice;
  const int per_cu = wgs_per_cu(shmem);
  const int grid = std::min(n_items, (cus * per_cu + 7) / 8 * 8);
  ProfileScope ps(MODE == 0 || MODE == 3 ? "fft_score_kernel" : "fft_score_kernel(partial pass)", s);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kA * CP), shmem, s, static_cast<const T*>(a.K),
                     static_cast<const T*>(a.V), a.st, a.n, a.n2, a.r, a.rcut, a.cmode, a.d, a.dtype, a.q0,
                     a.n_ut, a.slabs, n_items, ph_lds, a.hdr, a.twn, a.phase, a.partial, a.etot, a.resid);
  return hipGetLastError();
}

template <typename T, int CP, int NBUF>
hipError_t launch_pass_q(const PassArgs& a, int q, int mode, hipStream_t s) {
#define FC_PASS(QV)                                                \
  switch (mode) {                                                  \
    case 0: return launch_pass<T, CP, QV, 0, NBUF>(a, s);          \
    case 1: return launch_pass<T, CP, QV, 1, NBUF>(a, s);          \
    case 2: return launch_pass<T, CP, QV, 2, NBUF>(a, s);          \
    default: return launch_pass<T, CP, QV, 3, NBUF>(a, s);         \
  }
  if (q == 1) { FC_PASS(1) }
  FC_PASS(2)
#undef FC_PASS
}

template <typename T>
hipError_t launch_pass_cp(const PassArgs& a, int cp, int q, int mode, hipStream_t s) {
#if FC_FFT_R == 16
  if (cp != 2 || a.nbuf != 1) return hipErrorInvalidValue;
  return launch_pass_q<T, 2, 1>(a, q, mode, s);
#elif FC_FFT_R == 8
  if (cp != 4 || a.nbuf != 1) return hipErrorInvalidValue;
  return launch_pass_q<T, 4, 1>(a, q, mode, s);
#else
#if FC_FFT_R == 4
  if (cp == 4) return launch_pass_q<T, 4, 1>(a, q, mode, s);
  if (a.nbuf == 2) return launch_pass_q<T, 8, 2>(a, q, mode, s);
#endif
  if (cp != 8 || a.nbuf != 1) return hipErrorInvalidValue;
  return launch_pass_q<T, 8, 1>(a, q, mode, s);
#endif
}

}  // namespace

// One pass of the transform kernel of this unit's lane radix (q = low blocks of the pass, mode as
// described at the kernel).
hipError_t FC_CAT(fft_launch_pass_r, FC_FFT_R)(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s) {
  return a.dtype == FC_BF16 ? launch_pass_cp<uint16_t>(a, cp, q, mode, s)
                            : launch_pass_cp<float>(a, cp, q, mode, s);
}

#if FC_FFT_R == 4

hipError_t fft_score(const void* K, const void* V, const fc_kv_desc& d, int32_t r, const FftLayout& lay,
                     float* scores, double* energy, void* ws, UnitMap um, hipStream_t s) {
  char* base = static_cast<char*>(ws);
  const int units = d.batch * d.layers * d.kv_heads;
  const int n = d.n_tokens, n1 = 256 * lay.lane_radix, n2 = n / n1;
  bool cm;
  const int rcut = fft_cutoff(n, r, &cm);
  const int q_total = (rcut + n1 - 1) / n1;
  const int cp = d.head_dim / 2 / lay.slabs;
  PassArgs a{};
  a.n = n; a.n2 = n2; a.r = r; a.rcut = rcut; a.cmode = cm ? 1 : 0; a.d = d.head_dim; a.dtype = d.dtype; a.n_ut = units * 2; a.slabs = lay.slabs;
  a.nbuf = exchange_buffers(lay.lane_radix, cp, n);
  a.hdr = reinterpret_cast<WsHeader*>(base);
  a.twn = reinterpret_cast<const float2*>(base + lay.twiddle);
  a.phase = reinterpret_cast<const float2*>(base + lay.phase);
  a.partial = reinterpret_cast<float*>(base + lay.partial);
  a.etot = reinterpret_cast<double*>(base + lay.etot);
  a.resid = reinterpret_cast<float*>(base + lay.resid);
  double* epart = reinterpret_cast<double*>(base + lay.epart);

  a.K = K; a.V = V; a.st = strides_of(d);
  for (int pass = 0; pass < lay.passes; ++pass) {
    a.q0 = pass * kMaxQ;
    const int q = q_total - a.q0 < kMaxQ ? q_total - a.q0 : kMaxQ;
    // 0: only pass; 1: first of several; 2: middle; 3: last
    const int mode = lay.passes == 1 ? 0 : (pass == 0 ? 1 : (pass + 1 < lay.passes ? 2 : 3));
    const hipError_t e = lay.lane_radix == 16  ? fft_launch_pass_r16(a, cp, q, mode, s)
                         : lay.lane_radix == 8 ? fft_launch_pass_r8(a, cp, q, mode, s)
                         : lay.lane_radix == 4 ? fft_launch_pass_r4(a, cp, q, mode, s)
                         : lay.lane_radix == 2 ? fft_launch_pass_r2(a, cp, q, mode, s)
                                               : fft_launch_pass_r1(a, cp, q, mode, s);
    if (e != hipSuccess) return e;
  }
  {
    ProfileScope ps("fft_finalize_kernel", s);
    hipLaunchKernelGGL(fft_finalize_kernel, dim3(lay.tiles, units), dim3(256), (size_t)64 * n2 * sizeof(float),
                       s, a.partial, a.etot, n, n1, n2, r, d.head_dim, d.dtype, lay.slabs, a.hdr, scores, epart,
                       um);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return energy_reduce_launch(epart, lay.tiles, units, energy, um, s);
}
#endif  // FC_FFT_R == 4

}  // namespace fc
