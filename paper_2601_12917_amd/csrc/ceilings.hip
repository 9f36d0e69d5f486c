// Machine ceilings that the perturbation pass (Eq. (10), in-place theta + c Z) is rated against, measured
// rather than assumed:
//   - the bare in-place stream theta <- rnd(theta + c) over bf16 / fp32 data: what a read-modify-write pass
//     with no generator at all reaches on this chip, in 16-byte vectors like the real pass;
//   - the vector-ALU issue rate of the instruction kinds the generator is made of (fused multiply-add, xor,
//     three-input bit operation, 32 x 32 -> 64 multiply-add, conversions, v_rsq, ...), as cycles per wave64
//     instruction and SIMD, for 1..8 resident waves per SIMD and 1..4 independent chains per wave.  Two
//     clocks are read inside the kernel: the shader cycle counter and the constant 100 MHz real-time
//     counter, so the figures come in cycles and the clock the chip really ran at is known.
// Test / measurement exports only; nothing on the product path calls them.
#include "internal.h"

namespace zgr {

namespace {

struct bf16x8_t { uint32_t w[4]; };

template <bool BF16>
__global__ void __launch_bounds__(256) rmw_kernel(uint4* __restrict__ p, size_t n16, float c, int mode, uint4* __restrict__ sink) {
  uint4 keep = make_uint4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    uint4 v = mode == 2 ? make_uint4(0, 0, 0, 0) : p[i];
    uint32_t* w = reinterpret_cast<uint32_t*>(&v);
    if (mode != 1) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (BF16) {
          const float lo = __uint_as_float(w[j] << 16) + c, hi = __uint_as_float(w[j] & 0xFFFF0000u) + c;
          typedef float f2 __attribute__((ext_vector_type(2)));
          typedef __bf16 b2 __attribute__((ext_vector_type(2)));
          const b2 r = __builtin_convertvector(f2{lo, hi}, b2);
          w[j] = __builtin_bit_cast(uint32_t, r);
        } else {
          w[j] = __float_as_uint(__uint_as_float(w[j]) + c);
        }
      }
      p[i] = v;
    } else {
      keep.x ^= v.x; keep.y ^= v.y; keep.z ^= v.z; keep.w ^= v.w;
    }
  }
  if (mode == 1 && (keep.x ^ keep.y ^ keep.z ^ keep.w) == 0x9E3779B9u) sink[0] = keep;   // keeps the loads alive
}

// One wave runs iters x 64 instructions of kind OP in ILP independent dependent-chains and records the shader cycles
// it took and the real-time counter at its start and end.  The waves of a SIMD do not advance in step (the issue
// arbiter favours the oldest), so a rate comes from the span over all waves, first start to last end, not from the
// time of any one wave.
template <int OP, int ILP>
__global__ void __launch_bounds__(256) issue_kernel(int iters, unsigned long long* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t d[ILP], x[ILP], y[ILP];
  unsigned long long q[ILP];
#pragma unroll
  for (int i = 0; i < ILP; ++i) {
    d[i] = __float_as_uint(1.0f + 1e-3f * (float)(threadIdx.x + i));
    x[i] = __float_as_uint(1.0f + 1e-7f * (float)(threadIdx.x + 3 * i));
    y[i] = __float_as_uint(1e-9f * (float)(i + 1));
    q[i] = threadIdx.x + i;
  }
  const unsigned long long lane_mask = __builtin_amdgcn_ballot_w64((threadIdx.x * 2654435761u) & 0x10000u);   // a wave-uniform lane mask in an SGPR pair
  __builtin_amdgcn_s_barrier();
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 64 / ILP; ++r)
#pragma unroll
      for (int i = 0; i < ILP; ++i) {
        if (OP == 0) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(d[i]) : "v"(x[i]), "v"(y[i]));
        if (OP == 1) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 2) asm volatile("v_bitop3_b32 %0, %0, %1, %2 bitop3:0x96" : "+v"(d[i]) : "v"(x[i]), "v"(y[i]));
        if (OP == 3) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(q[i]) : "v"(x[i]), "v"(y[i]) : "vcc");
        if (OP == 4) asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 5) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 6) asm volatile("v_cvt_f32_u32 %0, %0" : "+v"(d[i]));
        if (OP == 7) asm volatile("v_rsq_f32 %0, %0" : "+v"(d[i]));
        if (OP == 8) asm volatile("v_add_u32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 9) asm volatile("v_lshrrev_b32 %0, 1, %0" : "+v"(d[i]));
        if (OP == 10) asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2" : "+v"(d[i]) : "v"(x[i]), "s"(lane_mask));
        if (OP == 11) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 12) asm volatile("v_add_f32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 13) asm volatile("v_log_f32 %0, %0" : "+v"(d[i]));
        if (OP == 14) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(d[i]) : "v"(x[i]));
        if (OP == 15) asm volatile("v_sqrt_f32 %0, %0" : "+v"(d[i]));
        if (OP == 16) asm volatile("v_mov_b32 %0, %1" : "+v"(d[i]) : "v"(x[i]));
      }
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < ILP; ++i) acc ^= d[i] ^ (uint32_t)q[i];
  if ((threadIdx.x & 63) == 0) {
    const size_t w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[4 * w] = c1 - c0;
    out[4 * w + 1] = r0;
    out[4 * w + 2] = r1;
    out[4 * w + 3] = acc;
  }
#endif
}

// The matrix core alone: every wave runs iters x 64 v_mfma_f32_32x32x16_bf16 (32768 flops each) on register
// operands, in ILP independent accumulators, and nothing else.  The operands are pseudo-random bf16 in (-2, 2): what
// the unit draws, and with it the clock the chip holds, depends on how many bits toggle.  out as for issue_kernel.
typedef __bf16 cbf16x8 __attribute__((ext_vector_type(8)));
typedef float cf32x16 __attribute__((ext_vector_type(16)));

template <int ILP>
__global__ void __launch_bounds__(256) mfma_kernel(int iters, unsigned long long* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
  union { uint32_t u[4]; cbf16x8 v; } a[ILP], b[ILP];
  cf32x16 acc[ILP];
  uint32_t h = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < ILP; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // two bf16 per word: random sign and mantissa, exponent of 1.0 or 0.5
      h = h * 1664525u + 1013904223u;  a[i].u[j] = (h & 0x80ff80ffu) | 0x3f003f00u;
      h = h * 1664525u + 1013904223u;  b[i].u[j] = (h & 0x80ff80ffu) | 0x3f003f00u;
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  }
  __builtin_amdgcn_s_barrier();
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 64 / ILP; ++r)
#pragma unroll
      for (int i = 0; i < ILP; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[i].v, acc[i], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float f = 0.f;
#pragma unroll
  for (int i = 0; i < ILP; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) f += acc[i][j];
  if ((threadIdx.x & 63) == 0) {
    const size_t w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[4 * w] = c1 - c0;
    out[4 * w + 1] = r0;
    out[4 * w + 2] = r1;
    out[4 * w + 3] = __float_as_uint(f);
  }
#endif
}

// The same for the fp32 matrix instruction, v_mfma_f32_32x32x2_f32 (4096 flops each), on random fp32 register operands.
// At least two waves per SIMD are allowed for, so that the accumulators stay in ordinary vector registers.
template <int ILP>
__global__ void __launch_bounds__(256, 2) mfma_f32_kernel(int iters, unsigned long long* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
  float a[ILP], b[ILP];
  cf32x16 acc[ILP];
  uint32_t h = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < ILP; ++i) {
    // random sign and mantissa, exponent of 1.0
    h = h * 1664525u + 1013904223u;  a[i] = __uint_as_float((h & 0x807fffffu) | 0x3f800000u);
    h = h * 1664525u + 1013904223u;  b[i] = __uint_as_float((h & 0x807fffffu) | 0x3f800000u);
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  }
  __builtin_amdgcn_s_barrier();
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 64 / ILP; ++r)
#pragma unroll
      for (int i = 0; i < ILP; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[i], acc[i], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float f = 0.f;
#pragma unroll
  for (int i = 0; i < ILP; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) f += acc[i][j];
  if ((threadIdx.x & 63) == 0) {
    const size_t w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[4 * w] = c1 - c0;
    out[4 * w + 1] = r0;
    out[4 * w + 2] = r1;
    out[4 * w + 3] = __float_as_uint(f);
  }
#endif
}

// The generator's own parts at full occupancy of the vector unit and nothing else: part 0 one Philox4x32-10 call,
// 1 two radii, 2 two (cos, sin) pairs, 3 two Box-Muller pairs (on cheap pseudo-random integers), 4 the whole
// generator of four Gaussians (Philox call + two Box-Muller pairs), 5 its two table look-ups alone.
template <int PART>
__global__ void __launch_bounds__(256) generator_kernel(int iters, uint32_t k0, uint32_t k1, const RadiusEntry* __restrict__ gtab,
                                                        unsigned long long* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ RadiusEntry tab[kRadiusTabEntries];
  load_radius_table(tab, gtab);
  __syncthreads();
  uint32_t acc = 0;
  float facc = 0.f;
  uint32_t q = blockIdx.x * 256 + threadIdx.x;
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
    const uint32_t a = q * 2654435761u, b = a ^ (a >> 13), c = b * 40503u, d = c ^ (a >> 7);
    if (PART == 0) {
      const u32x4 w = philox_call(q, 7, 3, k0, k1);
      acc ^= w.x ^ w.y ^ w.z ^ w.w;
    } else if (PART == 1) {
      facc += radius_from_odd24((a >> 8) | 1u, tab) + radius_from_odd24((b >> 8) | 1u, tab);
    } else if (PART == 2) {
      const TrigHL t = trig_from_u24(a >> 8), u = trig_from_u24(b >> 8);
      facc += t.ch + t.cl + t.sh + t.sl + u.ch + u.cl + u.sh + u.sl + __uint_as_float(t.sign ^ u.sign);
    } else if (PART == 3) {
      float g[4];
      box_muller((a >> 8) | 1u, b >> 8, tab, g[0], g[1]);
      box_muller((c >> 8) | 1u, d >> 8, tab, g[2], g[3]);
      facc += g[0] + g[1] + g[2] + g[3];
    } else if (PART == 4) {
      float g[4];
      gauss4(philox_call(q, 7, 3, k0, k1), tab, g);
      facc += g[0] + g[1] + g[2] + g[3];
    } else {
      const RadiusEntry e = tab[(a >> 8) & 1023], f = tab[(b >> 8) & 1023];
      facc += e.H + e.L + e.C + f.H + f.L + f.C;
    }
    q += gridDim.x * 256;
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  if ((threadIdx.x & 63) == 0) {
    const size_t w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[4 * w] = c1 - c0;
    out[4 * w + 1] = r0;
    out[4 * w + 2] = r1;
    out[4 * w + 3] = acc ^ __float_as_uint(facc);
  }
#endif
}

template <int OP>
hipError_t launch_issue_ilp(int ilp, int blocks, int iters, unsigned long long* out, hipStream_t s) {
  if (ilp == 1) hipLaunchKernelGGL((issue_kernel<OP, 1>), dim3(blocks), dim3(256), 0, s, iters, out);
  else if (ilp == 2) hipLaunchKernelGGL((issue_kernel<OP, 2>), dim3(blocks), dim3(256), 0, s, iters, out);
  else if (ilp == 4) hipLaunchKernelGGL((issue_kernel<OP, 4>), dim3(blocks), dim3(256), 0, s, iters, out);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_debug_rmw(void* p, size_t bytes, int dtype, float c, int mode, int blocks, void* sink, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (dtype == 1) hipLaunchKernelGGL(rmw_kernel<true>, dim3(blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(p), bytes / 16, c, mode, reinterpret_cast<uint4*>(sink));
  else            hipLaunchKernelGGL(rmw_kernel<false>, dim3(blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(p), bytes / 16, c, mode, reinterpret_cast<uint4*>(sink));
  return hipGetLastError();
}

hipError_t launch_debug_generator(int part, int blocks, int iters, unsigned long long* out, hipStream_t s) {
  const RadiusEntry* tab = nullptr;
  hipError_t e = ensure_radius_table(&tab, s);
  if (e != hipSuccess) return e;
  switch (part) {
#define ZGR_GEN_CASE(N) case N: hipLaunchKernelGGL((generator_kernel<N>), dim3(blocks), dim3(256), 0, s, iters, 42u, 0u, tab, out); break;
    ZGR_GEN_CASE(0) ZGR_GEN_CASE(1) ZGR_GEN_CASE(2) ZGR_GEN_CASE(3) ZGR_GEN_CASE(4) ZGR_GEN_CASE(5)
#undef ZGR_GEN_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_debug_issue(int op, int ilp, int blocks, int iters, unsigned long long* out, hipStream_t s) {
  if (op == 17) {
    if (ilp == 1) hipLaunchKernelGGL(mfma_kernel<1>, dim3(blocks), dim3(256), 0, s, iters, out);
    else if (ilp == 2) hipLaunchKernelGGL(mfma_kernel<2>, dim3(blocks), dim3(256), 0, s, iters, out);
    else if (ilp == 4) hipLaunchKernelGGL(mfma_kernel<4>, dim3(blocks), dim3(256), 0, s, iters, out);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  if (op == 18) {
    if (ilp == 1) hipLaunchKernelGGL(mfma_f32_kernel<1>, dim3(blocks), dim3(256), 0, s, iters, out);
    else if (ilp == 2) hipLaunchKernelGGL(mfma_f32_kernel<2>, dim3(blocks), dim3(256), 0, s, iters, out);
    else if (ilp == 4) hipLaunchKernelGGL(mfma_f32_kernel<4>, dim3(blocks), dim3(256), 0, s, iters, out);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  switch (op) {
#define ZGR_ISSUE_CASE(N) case N: return launch_issue_ilp<N>(ilp, blocks, iters, out, s);
    ZGR_ISSUE_CASE(0) ZGR_ISSUE_CASE(1) ZGR_ISSUE_CASE(2) ZGR_ISSUE_CASE(3) ZGR_ISSUE_CASE(4) ZGR_ISSUE_CASE(5)
    ZGR_ISSUE_CASE(6) ZGR_ISSUE_CASE(7) ZGR_ISSUE_CASE(8) ZGR_ISSUE_CASE(9) ZGR_ISSUE_CASE(10) ZGR_ISSUE_CASE(11)
    ZGR_ISSUE_CASE(12) ZGR_ISSUE_CASE(13) ZGR_ISSUE_CASE(14) ZGR_ISSUE_CASE(15) ZGR_ISSUE_CASE(16)
#undef ZGR_ISSUE_CASE
    default: return hipErrorInvalidValue;
  }
}

}  // namespace zgr
