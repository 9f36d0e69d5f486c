// Device-side random stream of the ZGR perturbation: Philox4x32-10 counters
// (Salmon et al., SC'11) -> Box-Muller Gaussians, all in fp32 registers.
//
// The paper (Sec. 3.1 step 5, Algorithm 1) only requires that client and edge
// server regenerate the same perturbation from the shared seed; a counter-based
// generator makes every element a pure function of
// (seed, step, tensor id, stream, flat element index).
//
// Accuracy contract: each Gaussian is within 2 ulp (fp32) of
//   sqrt(-2 ln u) * {cos, sin}(2 pi v)
// evaluated exactly from the dyadic uniforms u, v.  The radius is computed to
// ~0.502 ulp (table-driven log with an exact argument reduction, compensated
// square root); cos/sin come out as hi+lo pairs good to ~0.4*2^-24 relative, so
// that the single product radius*trig loses at most ~1.9 ulp in the worst case.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zgr {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

struct u32x4 { uint32_t x, y, z, w; };

// a ^ b ^ c in one instruction (v_bitop3_b32 with the parity truth table): Philox has two of these per round.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
#else
  return a ^ b ^ c;
#endif
}

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
    const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += kPhiloxW0;   // uniform across the wave: scalar unit
    k1 += kPhiloxW1;
  }
  return {c0, c1, c2, c3};
}

// Counter of call q of one stream (0: isotropic G, 1: subspace coefficients R).
__device__ __forceinline__ u32x4 philox_call(uint64_t q, uint32_t id_stream, uint32_t step, uint32_t k0, uint32_t k1) {
  return philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), id_stream, step, k0, k1);
}

// ---------------------------------------------------------------------------
// Radius table: entry [E*64 + j] for the odd 24-bit integer N = 2n+1 with
// float exponent E (0..23) and top six mantissa bits j:
//   c   = short reciprocal of the bin centre (7 fractional bits) times 2^-E,
//         so that z = N*c - 1 is exact and |z| < 2^-6,
//   H+L = -2 ln(2^(E-24) / c_j) split in two floats.
// -2 ln(N 2^-24) = (H + L) - 2 log1p(z).
// ---------------------------------------------------------------------------
constexpr int kRadiusTabEntries = 24 * 64;
struct RadiusEntry { float H, L, C; };

// t = rho^2 = -2 ln(N * 2^-24) as hi + lo, then rho by one Newton step on rsq.
__device__ __forceinline__ float radius_from_odd24(uint32_t N, const RadiusEntry* __restrict__ tab) {
#pragma clang fp contract(off)   // the compensated steps below must not be re-fused
  const float Nf = (float)N;                                   // exact
  const int idx = (int)(__float_as_uint(Nf) >> 17) - (127 << 6);
  const RadiusEntry e = tab[idx];
  const float z = __builtin_fmaf(Nf, e.C, -1.0f);               // exact
  float q = __builtin_fmaf(z, -0.4f, 0.5f);
  q = __builtin_fmaf(z, q, -0.66666668653488159f);
  q = __builtin_fmaf(z, q, 1.0f);
  q = z * q;                                                    // z - 2/3 z^2 + 1/2 z^3 - 2/5 z^4
  float lo = __builtin_fmaf(z, q, e.L);                         // L + z^2 - ...
  float hi = __builtin_fmaf(-2.0f, z, e.H);
  const float err = __builtin_fmaf(-2.0f, z, e.H - hi);         // exact rounding error of hi
  lo += err;
  const float t = hi + lo;                                      // renormalise: |lo| <= ulp(t)/2
  lo = (hi - t) + lo;
  const float r = __builtin_amdgcn_rsqf(t);
  const float rho0 = t * r;
  const float d = __builtin_fmaf(-rho0, rho0, t) + lo;
  return __builtin_fmaf(d, 0.5f * r, rho0);
}

// cos(2 pi v), sin(2 pi v) for v = m * 2^-24 as (hi, lo) pairs, up to the common sign `sign`
// (0 or 0x80000000) that the caller folds into the radius.
struct TrigHL { float ch, cl, sh, sl; uint32_t sign; };

__device__ __forceinline__ TrigHL trig_from_u24(uint32_t m) {
#pragma clang fp contract(off)
  // exact reduction to the nearest quarter turn: y in [-1, 1) is the offset in units of 1/8 turn
  const uint32_t mp = m + 0x200000u;
  const float y = __builtin_fmaf((float)(mp & 0x3FFFFFu), 4.76837158203125e-07f, -1.0f);
  const float y2 = y * y;
  const float y2l = __builtin_fmaf(y, y, -y2);
  // sin(pi/4 y) = y (S0 + y^2 (S1 + y^2 (S2 + y^2 S3)))
  constexpr float S0h = 0.78539818525314331f, S0l = -2.1855694143368964e-08f;
  constexpr float S1 = -0.08074545115232468f, S2 = 0.002490044105798006f, S3 = -3.5975263017462566e-05f;
  float p = __builtin_fmaf(y2, S3, S2);
  p = __builtin_fmaf(y2, p, S1);
  p = __builtin_fmaf(y2, p, S0l);
  const float sh = y * S0h;
  const float sl = __builtin_fmaf(y, p, __builtin_fmaf(y, S0h, -sh));
  // cos(pi/4 y) = 1 + y^2 (C1 + y^2 (C2 + y^2 (C3 + y^2 C4))), C1 = -pi^2/32 as hi + lo
  constexpr float C1h = -0.3084251284599304f, C1l = -9.074112128359957e-09f;
  constexpr float C2 = 0.015854336321353912f, C3 = -0.00032595498487353325f, C4 = 3.5375171592022525e-06f;
  float g = __builtin_fmaf(y2, C4, C3);
  g = __builtin_fmaf(y2, g, C2);
  g = __builtin_fmaf(y2, g, C1l);
  g = __builtin_fmaf(y2, g, y2l * C1h);
  const float ch = __builtin_fmaf(y2, C1h, 1.0f);
  const float cl = __builtin_fmaf(y2, C1h, 1.0f - ch) + g;
  // quadrant q = bits 22..23 of mp: (cos, sin) = R(q * 90 deg) (c, s).  Odd q rotates by a quarter turn,
  // (c, s) -> (-s, c); q >= 2 negates both, which is left to the caller as one sign on the radius.
  const bool odd = (mp >> 22) & 1u;
  TrigHL o;
  o.ch = odd ? -sh : ch;  o.cl = odd ? -sl : cl;
  o.sh = odd ? ch : sh;   o.sl = odd ? cl : sl;
  o.sign = (mp << 8) & 0x80000000u;                // bit 23 -> bit 31
  return o;
}

// One Box-Muller pair from the odd 24-bit radius integer N (u = N 2^-24) and the 24-bit angle integer m.
__device__ __forceinline__ void box_muller(uint32_t N, uint32_t m, const RadiusEntry* __restrict__ tab, float& g_cos, float& g_sin) {
#pragma clang fp contract(off)
  const float rho = radius_from_odd24(N, tab);
  const TrigHL t = trig_from_u24(m);
  const float r = __uint_as_float(__float_as_uint(rho) ^ t.sign);
  g_cos = __builtin_fmaf(r, t.ch, r * t.cl);
  g_sin = __builtin_fmaf(r, t.sh, r * t.sl);
}

// Four Gaussians of one Philox call (32-bit mode): pairs from words (0,1) and (2,3).
// u = ((w >> 9) + 0.5) 2^-23 = ((w >> 8) | 1) 2^-24,  v = (w >> 8) 2^-24.
__device__ __forceinline__ void gauss4(const u32x4 w, const RadiusEntry* __restrict__ tab, float g[4]) {
  box_muller((w.x >> 8) | 1u, w.y >> 8, tab, g[0], g[1]);
  box_muller((w.z >> 8) | 1u, w.w >> 8, tab, g[2], g[3]);
}

// Eight Gaussians of one Philox call (16-bit mode): pair p from word p, low half radius, high half angle.
// u = (h + 0.5) 2^-16 = ((2h + 1) << 7) 2^-24,  v = h 2^-16 = (h << 8) 2^-24.
__device__ __forceinline__ void gauss8(const u32x4 w, const RadiusEntry* __restrict__ tab, float g[8]) {
  const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
  for (int p = 0; p < 4; ++p)
    box_muller((((ww[p] & 0xFFFFu) << 1) | 1u) << 7, (ww[p] >> 16) << 8, tab, g[2 * p], g[2 * p + 1]);
}

// Block-wide copy of the radius table from global memory into LDS.
__device__ __forceinline__ void load_radius_table(RadiusEntry* lds, const RadiusEntry* __restrict__ glob) {
  const float* s = reinterpret_cast<const float*>(glob);
  float* d = reinterpret_cast<float*>(lds);
  for (int i = threadIdx.x; i < kRadiusTabEntries * 3; i += blockDim.x) d[i] = s[i];
}

}  // namespace zgr
