// Forward pass L(W; x) for the two loss evaluations of the ZGR step (Sec. 3.2,
// Eq. (11); Sec. 3.1 workflow step 6): pre-LayerNorm transformer blocks with
// softmax attention and erf-GELU feed-forward, next-token cross-entropy through
// the tied embedding (decoder) or a classification head on the first token
// (encoder), and the least-squares loss of a single linear layer.
//
// Storage type T of weights and GEMM inputs is fp32 or bf16; accumulation, the
// residual stream, LayerNorm, softmax and the loss are fp32, the final mean fp64.
#include "forward.h"
#include <atomic>

namespace zgr {

namespace {

struct bf16_t { uint16_t bits; };
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }
__device__ __forceinline__ void from_f32(float x, float& o) { o = x; }
__device__ __forceinline__ void from_f32(float x, bf16_t& o) {     // round to nearest, ties to even (v_cvt_pk_bf16_f32)
  const __bf16 h = static_cast<__bf16>(x);
  o.bits = __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// block of 256 threads: reduce across the 4 waves through LDS
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E, const T* __restrict__ Pe,
                                                    float* __restrict__ x, int M, int seq, int d, int vocab) {
  const int m = blockIdx.x;
  int t = tok[m];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* e = E + (size_t)t * d;
  const T* p = Pe + (size_t)(m % seq) * d;
  for (int i = threadIdx.x; i < d; i += 256) x[(size_t)m * d + i] = to_f32(e[i]) + to_f32(p[i]);
}

// ------------------------------------------------------------------ LayerNorm (one block per row)
template <typename T>
__global__ void __launch_bounds__(256) layernorm_kernel(const float* x, const T* __restrict__ g, const T* __restrict__ b,
                                                        T* __restrict__ out, int d, float eps, float* xout) {
  __shared__ float red[4];
  const float* row = x + (size_t)blockIdx.x * d;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) s += row[i];
  const float mu = block_sum(s, red) / d;
  float v = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float t = row[i] - mu; v += t * t; }
  const float rstd = 1.0f / sqrtf(block_sum(v, red) / d + eps);
  T* o = out + (size_t)blockIdx.x * d;
  float* xo = xout ? xout + (size_t)blockIdx.x * d : nullptr;      // may be the row itself: an element is read, then written, by one thread
  for (int i = threadIdx.x; i < d; i += 256) {
    const float y = (row[i] - mu) * rstd * to_f32(g[i]) + to_f32(b[i]);
    from_f32(y, o[i]);
    if (xo) xo[i] = y;
  }
}

// Row held in registers (d % 4 == 0, d <= 8192): one read of x, float4 loads, packed stores.
template <typename T>
__global__ void __launch_bounds__(256) layernorm_reg_kernel(const float* x, const T* __restrict__ g, const T* __restrict__ b,
                                                            T* __restrict__ out, int d, float eps, float* xout) {
  __shared__ float red[4];
  constexpr int MAXV = 8;
  const float4* row = reinterpret_cast<const float4*>(x + (size_t)blockIdx.x * d);
  const int nv = d >> 2;
  float4 v[MAXV];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = threadIdx.x + 256 * j;
    v[j] = i < nv ? row[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  }
  const float mu = block_sum(s, red) / d;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = threadIdx.x + 256 * j;
    if (i < nv) {
      const float a0 = v[j].x - mu, a1 = v[j].y - mu, a2 = v[j].z - mu, a3 = v[j].w - mu;
      q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
  }
  const float rstd = 1.0f / sqrtf(block_sum(q, red) / d + eps);
  T* o = out + (size_t)blockIdx.x * d;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = threadIdx.x + 256 * j;
    if (i < nv) {
      struct alignas(sizeof(T) * 4) V4 { T e[4]; };
      const V4 gg = *reinterpret_cast<const V4*>(g + 4 * i), bb = *reinterpret_cast<const V4*>(b + 4 * i);
      V4 r;
      const float4 y = make_float4((v[j].x - mu) * rstd * to_f32(gg.e[0]) + to_f32(bb.e[0]), (v[j].y - mu) * rstd * to_f32(gg.e[1]) + to_f32(bb.e[1]),
                                   (v[j].z - mu) * rstd * to_f32(gg.e[2]) + to_f32(bb.e[2]), (v[j].w - mu) * rstd * to_f32(gg.e[3]) + to_f32(bb.e[3]));
      from_f32(y.x, r.e[0]); from_f32(y.y, r.e[1]); from_f32(y.z, r.e[2]); from_f32(y.w, r.e[3]);
      *reinterpret_cast<V4*>(o + 4 * i) = r;
      if (xout) reinterpret_cast<float4*>(xout + (size_t)blockIdx.x * d)[i] = y;      // the row is in registers: xout may be x
    }
  }
}

// One wave per row (d % 4 == 0, d <= 2048): the row sits in eight float4 per lane, eight 16-byte loads in flight per lane,
// and both reductions stay inside the wave: no LDS, no workgroup barrier.  Four rows per block.
template <typename T>
__global__ void __launch_bounds__(256) layernorm_wave_kernel(const float* x, const T* __restrict__ g, const T* __restrict__ b,
                                                             T* __restrict__ out, int M, int d, float eps, float* xout) {
  constexpr int MAXV = 8;
  const int lane = threadIdx.x & 63;
  const int row_i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row_i >= M) return;                                          // whole waves leave: no barrier below
  const float4* row = reinterpret_cast<const float4*>(x + (size_t)row_i * d);
  const int nv = d >> 2;
  float4 v[MAXV];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = lane + 64 * j;
    v[j] = i < nv ? row[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = lane + 64 * j;
    if (i < nv) {
      const float a0 = v[j].x - mu, a1 = v[j].y - mu, a2 = v[j].z - mu, a3 = v[j].w - mu;
      q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / d + eps);
  T* o = out + (size_t)row_i * d;
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int i = lane + 64 * j;
    if (i < nv) {
      struct alignas(sizeof(T) * 4) V4 { T e[4]; };
      const V4 gg = *reinterpret_cast<const V4*>(g + 4 * i), bb = *reinterpret_cast<const V4*>(b + 4 * i);
      V4 r;
      const float4 y = make_float4((v[j].x - mu) * rstd * to_f32(gg.e[0]) + to_f32(bb.e[0]), (v[j].y - mu) * rstd * to_f32(gg.e[1]) + to_f32(bb.e[1]),
                                   (v[j].z - mu) * rstd * to_f32(gg.e[2]) + to_f32(bb.e[2]), (v[j].w - mu) * rstd * to_f32(gg.e[3]) + to_f32(bb.e[3]));
      from_f32(y.x, r.e[0]); from_f32(y.y, r.e[1]); from_f32(y.z, r.e[2]); from_f32(y.w, r.e[3]);
      *reinterpret_cast<V4*>(o + 4 * i) = r;
      if (xout) reinterpret_cast<float4*>(xout + (size_t)row_i * d)[i] = y;          // the row is in registers: xout may be x
    }
  }
}

// ------------------------------------------------------------------ GEMM  C = A W^T (+bias) with epilogues
// A [M,K] and W [N,K] are K-contiguous.
//   EPI_STORE: out T [M,N] = acc + bias
//   EPI_GELU : out T [M,N] = gelu(acc + bias);  EPI_RELU: out T [M,N] = max(acc + bias, 0)
//   EPI_RESID: xres fp32 [M,N] += acc + bias
//   EPI_F32  : outf fp32 [M,N] = acc + bias (bias may be null)
struct GemmEpi { int mode; void* out; const void* bias; };

template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmEpi& ep, int m, int n, int N, float v) {
  if (ep.bias) v += to_f32(reinterpret_cast<const T*>(ep.bias)[n]);
  const size_t o = (size_t)m * N + n;
  switch (ep.mode) {
    case EPI_STORE: from_f32(v, reinterpret_cast<T*>(ep.out)[o]); break;
    case EPI_GELU:  from_f32(gelu_erf(v), reinterpret_cast<T*>(ep.out)[o]); break;
    case EPI_RELU:  from_f32(fmaxf(v, 0.f), reinterpret_cast<T*>(ep.out)[o]); break;
    case EPI_RESID: reinterpret_cast<float*>(ep.out)[o] += v; break;
    default:        reinterpret_cast<float*>(ep.out)[o] = v; break;
  }
}

// fp32 path: 64x64 tile, BK = 16, each thread 4x4 outputs; any M, N, K.
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W, int M, int N, int K, GemmEpi ep) {
  __shared__ float As[16][64 + 4], Ws[16][64 + 4];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i >> 4, kk = i & 15;
      As[kk][r] = (m0 + r < M && k0 + kk < K) ? A[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
      Ws[kk][r] = (n0 + r < N && k0 + kk < K) ? W[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; w[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) epilogue_store<float>(ep, m, n, N, acc[i][j]);
    }
}

// fp32 path on the matrix cores: v_mfma_f32_32x32x2_f32.  Block tile 64 F x 64 F (F = 1 or 2), BK = 16, four waves
// in 2 x 2, each owning F x F accumulator fragments of 32 x 32.  An fp32 MFMA keeps the matrix pipe busy for 64
// cycles with two floats per lane, so the operands are no bottleneck: the next k-tile travels global -> registers
// while the current one is multiplied and is written to the other LDS buffer afterwards, one barrier per k-tile.
// Four consecutive lanes fetch the 64 contiguous bytes a row contributes to a k-tile.  LDS keeps the rows as they
// are, [row][16 + 4 pad]; the contraction index is split so that a lane's eight values of a k-tile are contiguous
// (the half-wave h takes k = 8 h .. 8 h + 7, in both operands alike): two 16-byte reads per fragment and k-tile,
// conflict-free at a row stride of 20 floats.
// Any M, N; K % 4 == 0 and 16-byte aligned rows (the 64 x 64 kernel above takes what is left).
typedef float f32x16 __attribute__((ext_vector_type(16)));

// At least two waves per SIMD, i.e. at most 256 registers per lane: the accumulators then live in ordinary vector registers,
// which the MFMA reads and writes directly.  (Allowed 512, the compiler multiplies in the accumulation registers, carries
// the sums round the loop in vector registers and moves all 64 of them back and forth in every k-tile.)
template <int F, int BK>
__global__ void __launch_bounds__(256, 2) gemm_f32_mfma_kernel(const float* __restrict__ A, const float* __restrict__ W, int M, int N, int K, GemmEpi ep) {
  constexpr int BT = 64 * F, LD = BK + 4, KQ = BK / 4, NV = BT * KQ / 256, HK = BK / 2;
  __shared__ __attribute__((aligned(16))) float As[2][BT][LD], Ws[2][BT][LD];
  const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int wm = (wave >> 1) * 32 * F, wn = (wave & 1) * 32 * F;
  // a thread moves NV float4 of each operand per k-tile: row r = idx / KQ, k columns 4 (idx % KQ) .. + 3.  Rows past the
  // matrix are read from its last row (their products are never stored), so only the last, partial k-tile needs a mask.
  float4 ra[NV], rw[NV];
  const float* pa[NV];
  const float* pw[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int idx = tid + 256 * i, r = idx / KQ, kq = idx % KQ;
    pa[i] = A + (size_t)min(m0 + r, M - 1) * K + 4 * kq;
    pw[i] = W + (size_t)min(n0 + r, N - 1) * K + 4 * kq;
  }
  auto fetch = [&](int k0) {
    if (k0 + BK <= K) {
#pragma unroll
      for (int i = 0; i < NV; ++i) { ra[i] = *reinterpret_cast<const float4*>(pa[i] + k0); rw[i] = *reinterpret_cast<const float4*>(pw[i] + k0); }
    } else {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const bool kin = k0 + 4 * ((tid + 256 * i) % KQ) < K;
        ra[i] = kin ? *reinterpret_cast<const float4*>(pa[i] + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
        rw[i] = kin ? *reinterpret_cast<const float4*>(pw[i] + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int idx = tid + 256 * i, r = idx / KQ, kq = idx % KQ;
      *reinterpret_cast<float4*>(&As[buf][r][4 * kq]) = ra[i];
      *reinterpret_cast<float4*>(&Ws[buf][r][4 * kq]) = rw[i];
    }
  };
  f32x16 acc[F][F];
#pragma unroll
  for (int f = 0; f < F; ++f)
#pragma unroll
    for (int g = 0; g < F; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[f][g][v] = 0.f;
  // fragments of one k-tile: a lane's HK values of each of its F + F fragment rows
  auto read_frags = [&](int buf, float (&a)[F][HK], float (&w)[F][HK]) {
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
      for (int q = 0; q < HK / 4; ++q) {
        const float4 av = *reinterpret_cast<const float4*>(&As[buf][wm + 32 * f + l32][HK * half + 4 * q]);
        const float4 wv = *reinterpret_cast<const float4*>(&Ws[buf][wn + 32 * f + l32][HK * half + 4 * q]);
        a[f][4 * q] = av.x; a[f][4 * q + 1] = av.y; a[f][4 * q + 2] = av.z; a[f][4 * q + 3] = av.w;
        w[f][4 * q] = wv.x; w[f][4 * q + 1] = wv.y; w[f][4 * q + 2] = wv.z; w[f][4 * q + 3] = wv.w;
      }
  };
  auto multiply = [&](const float (&a)[F][HK], const float (&w)[F][HK], int ks0, int ks1) {
#pragma unroll
    for (int ks = ks0; ks < ks1; ++ks)
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int g = 0; g < F; ++g) acc[f][g] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[f][ks], w[g][ks], acc[f][g], 0, 0, 0);
  };
  // Three k-tiles are in flight: t in fragment registers (being multiplied), t + 1 in LDS (its fragments are read between
  // the two halves of t's MFMAs), t + 2 on its way from global memory (written to the buffer of t, which every wave left
  // before the previous barrier, behind t's MFMAs).  Everything but the MFMAs is issued in their shadow.
  const int ktiles = (K + BK - 1) / BK;
  float fa[2][F][HK], fw[2][F][HK];
  fetch(0);
  stage(0);
  if (ktiles > 1) fetch(BK);
  __syncthreads();
  read_frags(0, fa[0], fw[0]);
  if (ktiles > 1) stage(1);
  __syncthreads();
  auto step = [&](int kt, float (&ca)[F][HK], float (&cw)[F][HK], float (&na)[F][HK], float (&nw)[F][HK]) {
    if (kt + 2 < ktiles) fetch((kt + 2) * BK);
    multiply(ca, cw, 0, HK / 2);
    if (kt + 1 < ktiles) read_frags((kt + 1) & 1, na, nw);
    multiply(ca, cw, HK / 2, HK);
    if (kt + 2 < ktiles) stage(kt & 1);
    __syncthreads();
  };
  // The same step without its conditions, for k-tiles whose successors t + 1 and t + 2 exist and need no mask: one basic block,
  // in which the scheduler is told to put the global fetches between the first half's MFMAs and the fragment reads between the
  // second half's (a fetch or read blocks the wave's issue for tens of cycles; behind an MFMA of 64 cycles that costs nothing).
  auto fast_step = [&](int kt, float (&ca)[F][HK], float (&cw)[F][HK], float (&na)[F][HK], float (&nw)[F][HK]) {
#pragma unroll
    for (int i = 0; i < NV; ++i) { ra[i] = *reinterpret_cast<const float4*>(pa[i] + (kt + 2) * BK); rw[i] = *reinterpret_cast<const float4*>(pw[i] + (kt + 2) * BK); }
    multiply(ca, cw, 0, HK / 2);
    read_frags((kt + 1) & 1, na, nw);
    multiply(ca, cw, HK / 2, HK);
    stage(kt & 1);
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int MF = F * F * HK / 2;                    // MFMAs per half
#pragma unroll
    for (int i = 0; i < 2 * NV; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, MF / (2 * NV), 0);     // MFMA
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                 // one global fetch
    }
#pragma unroll
    for (int i = 0; i < F * HK / 2; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, MF / (F * HK / 2), 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                 // one fragment read
    }
#endif
    __syncthreads();
  };
  const int kfull = K / BK;                               // k-tiles that need no mask
  int kt = 0;
  for (; kt + 3 < kfull; kt += 2) {
    fast_step(kt, fa[0], fw[0], fa[1], fw[1]);
    fast_step(kt + 1, fa[1], fw[1], fa[0], fw[0]);
  }
  for (; kt < ktiles; kt += 2) {
    step(kt, fa[0], fw[0], fa[1], fw[1]);
    if (kt + 1 < ktiles) step(kt + 1, fa[1], fw[1], fa[0], fw[0]);
  }
  // lane (l32, half) holds column n = l32 of a fragment and its rows 8 (v / 4) + 4 half + v % 4
#pragma unroll
  for (int f = 0; f < F; ++f)
#pragma unroll
    for (int g = 0; g < F; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm + 32 * f + 8 * (v >> 2) + 4 * half + (v & 3), n = n0 + wn + 32 * g + l32;
        if (m < M && n < N) epilogue_store<float>(ep, m, n, N, acc[f][g][v]);
      }
}

// bf16 path: MFMA 32x32x16.  Block tile BM x BN, BK = 64, WM x WN waves, each owning (BM / WM) x (BN / WN) of
// the output as FM x FN accumulator fragments of 32 x 32.  Operands go from global memory straight into LDS
// (no register staging).  Two main loops: the ping-pong pipeline (PP = 1, eight waves, large tiles) and a plain
// multi-stage loop with one barrier per k-tile (PP = 0, the 128 x 128 tile of small problems).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int GB_K = 64;

__device__ __forceinline__ void wait_vmem() {   // all outstanding global -> LDS transfers of this wave have landed
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
}

// erf-GELU, x Phi(x) = max(x, 0) - |x|/2 erfc(|x| / sqrt 2), with erfc(|x| / sqrt 2) = exp2(q(|x|)): q is a
// degree-6 fit of log2 erfc on [0, 6] (beyond 6 the term is below 1e-8 and |x| is clamped).  Absolute error of
// the result <= 1e-7 for all x, relative error <= 2e-5 for |x| < 3: far below the bf16 rounding of the result.
// One transcendental (v_exp_f32) and nine full-rate operations.
__device__ __forceinline__ float gelu_fast(float x) {
  const float a = fminf(fabsf(x), 6.0f);
  float q = 3.1244733690982684e-05f;
  q = __builtin_fmaf(q, a, -0.0007523701642639935f);
  q = __builtin_fmaf(q, a, 0.008023424074053764f);
  q = __builtin_fmaf(q, a, -0.05332072451710701f);
  q = __builtin_fmaf(q, a, -0.4588412642478943f);
  q = __builtin_fmaf(q, a, -1.1511778831481934f);
  q = __builtin_fmaf(q, a, 4.343822638475103e-06f);
  const float e = __builtin_amdgcn_exp2f(q);
  return __builtin_fmaf(-fabsf(0.5f * x), e, fmaxf(x, 0.f));
}

template <int MODE>
__device__ __forceinline__ void epilogue_bf16(void* out, size_t o, float v) {
  if (MODE == EPI_STORE) from_f32(v, reinterpret_cast<bf16_t*>(out)[o]);
  else if (MODE == EPI_GELU) from_f32(gelu_fast(v), reinterpret_cast<bf16_t*>(out)[o]);
  else if (MODE == EPI_RELU) from_f32(fmaxf(v, 0.f), reinterpret_cast<bf16_t*>(out)[o]);
  else if (MODE == EPI_RESID) reinterpret_cast<float*>(out)[o] += v;
  else reinterpret_cast<float*>(out)[o] = v;
}

// Bare workgroup barrier.  __syncthreads() also fences memory, which makes the compiler drain every
// outstanding global -> LDS transfer (vmcnt(0)) and so serialises a multi-stage pipeline; the main loop
// orders its LDS traffic itself (wait_vmem_upto before the barrier, data-dependent waits on its own reads).
__device__ __forceinline__ void block_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_barrier();
#endif
}

template <int N> __device__ __forceinline__ void wait_vmem_upto() {   // at most N global -> LDS transfers of this wave still in flight
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}

template <int BM, int BN, int WM, int WN, int BK, int STAGES, int MODE, int PP = 0>
__global__ void __launch_bounds__(64 * WM * WN) gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, int M, int N, int K,
                                                                 void* __restrict__ out, const bf16_t* __restrict__ bias,
                                                                 const int32_t* __restrict__ targets, float* __restrict__ tlogit) {
  constexpr int NW = WM * WN;
  constexpr int FM = BM / (32 * WM), FN = BN / (32 * WN);      // 32x32 fragments per wave
  constexpr int CPR = BK / 8;                                  // 16-byte chunks per LDS row
  constexpr int RPI = 64 / CPR;                                // rows one global_load_lds instruction fills (1 KiB)
  constexpr int RPB = 256 / (BK * 2);                          // rows per 256 B of LDS (one sweep over all banks)
  constexpr int GA = BM / RPI / NW, GW = BN / RPI / NW;        // instructions per wave per k-tile
  static_assert(PP != 0 || (GA >= 1 && GW >= 1 && (STAGES - 2) * (GA + GW) < 64), "tile / stage configuration");
  // LDS: STAGES slabs of [BM + BN][BK] bf16, rows unpadded; the 16-byte chunk c of row r sits in slot
  // c ^ ((r / RPB) % CPR), which makes the MFMA operand reads conflict-free.  The slabs are written by
  // global_load_lds (global memory -> LDS without passing registers): one instruction fills RPI rows, lane L
  // supplying row L / CPR, slot L % CPR, i.e. it fetches the global chunk (L % CPR) ^ swizzle(row).
  extern __shared__ __attribute__((aligned(1024))) unsigned char gsm[];
  bf16_t* As = reinterpret_cast<bf16_t*>(gsm);                 // [STAGES][BM][BK]
  bf16_t* Ws = As + STAGES * BM * BK;                          // [STAGES][BN][BK]
  const int tid = threadIdx.x, lane = tid & 63;
#if defined(__HIP_DEVICE_COMPILE__)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: kept in a scalar register
#else
  const int wave = tid >> 6;
#endif
  const int wm = wave / WN, wn = wave % WN;
  // XCD-aware tile order.  Consecutive block ids go round-robin to the 8 XCDs, each with its own L2 and
  // about 32 blocks in flight.  Give XCD x the super-tiles x, x+8, ... of GM x GN = 4 x 8 tiles, walked in
  // order inside the XCD, so that the blocks resident in one L2 share 4 row panels of A and 8 of W.
  constexpr int GM = 4, GN = 8;
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int stn = (tiles_n + GN - 1) / GN;
  const int local = blockIdx.x >> 3, st = (local / (GM * GN)) * 8 + (blockIdx.x & 7), w = local % (GM * GN);
  const int tm = (st / stn) * GM + w / GN, tn = (st % stn) * GN + w % GN;
  if (tm >= tiles_m || tn >= tiles_n) return;
  const int m0 = tm * BM, n0 = tn * BN;
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // Residual epilogue on the smaller tiles: this lane's part of the residual stream is requested now, ahead of
  // every operand transfer (loads complete in order, so the vmcnt counts of the main loop still only see the
  // transfers), and has long arrived when the epilogue adds to it; only the write-back remains exposed there.
  constexpr bool PRE_RES = MODE == EPI_RESID && FM * FN <= 4;
  const bool pre_res = PRE_RES && m0 + BM <= M && n0 + BN <= N;
  float res[PRE_RES ? FM * FN * 16 : 1];
  if (PRE_RES && pre_res) {
    const float* rp = reinterpret_cast<const float*>(out) + (size_t)(m0 + wm * (BM / WM) + 4 * (lane >> 5)) * N + n0 + wn * (BN / WN) + (lane & 31);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) res[(i * FN + j) * 16 + v] = rp[(size_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * N + j * 32];
  }
  const int nk = K / BK;
  // reader: lane (l32, half) reads row l32 of each fragment, logical chunk 2*ks + half
  const int l32 = lane & 31, half = lane >> 5, swz = (l32 / RPB) % CPR;
  int koff[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) koff[ks] = ((2 * ks + half) ^ swz) << 3;
  if constexpr (PP != 0) {
    // Ping-pong pipeline.  Two groups of four waves (waves w and w + 4 share a SIMD) take turns: while one group
    // runs the MFMAs of half a k-tile (one wave per SIMD keeps the matrix pipe busy on its own: the products of
    // a half are independent), the other reads the operands of its next half from LDS and issues its share of
    // the global -> LDS transfers.  The groups run one phase apart (the second starts with an extra barrier,
    // the first ends with one) and every phase ends in a workgroup barrier, so a SIMD always holds one wave of
    // each kind and the transfers never wait behind a group that is issuing MFMAs.
    //
    // LDS is a ring of R units of 8 KiB: 64 rows of one operand over the BK = 64 columns of a k-tile (whole
    // 128-byte lines of the source).  One transfer
    // instruction per wave fills a unit (wave w supplies rows 8w .. 8w + 7).  K-tile kt owns the U = (BM + BN) / 64
    // units kt U .. kt U + U - 1 (A first), at ring positions taken modulo R.  Unit q may be overwritten by unit
    // q + R once k-tile q / U has been read by both groups, which is the case from the first memory phase of the
    // next k-tile on; so the two memory phases of k-tile kt issue the units R - U + kt U .. R + kt U - 1, i.e.
    // R - U units (one and a half k-tiles for 256 x 256 tiles) are in flight or landed ahead of the reader.
    // K-tile kt + 1 must have landed before the first group starts on it: the second group waits for its shares at
    // the end of its last memory phase of k-tile kt, the first at the end of its last MFMA phase, in both cases
    // with the R - 2U units of later k-tiles still in flight; the barrier that follows publishes them.
    static_assert(NW == 8 && BK == 64 && BM % 64 == 0 && BN % 64 == 0, "ping-pong configuration");
    constexpr int UA = BM / 64, U = (BM + BN) / 64, R = STAGES, Q0 = R - U;
    constexpr int UH0 = (U + 1) / 2;                             // units issued in the first memory phase of a k-tile
    static_assert(R >= 2 * U && R * 8192 <= 160 * 1024, "ring size");
    const int frow = wave * 8 + (lane >> 3);                     // row this lane supplies within a unit
    uint32_t uo[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool is_a = u < UA;
      const int rl = (is_a ? u : u - UA) * 64 + frow;
      int r = (is_a ? m0 : n0) + rl;
      const int lim = is_a ? M : N;
      r = r < lim ? r : lim - 1;
      uo[u] = ((uint32_t)r * (uint32_t)K + (((lane & 7) ^ ((frow >> 1) & 7)) << 3)) * 2;   // bytes
    }
#if defined(__HIP_DEVICE_COMPILE__)
    // buffer addressing: per-lane byte offset in a register, the k-tile's offset in a scalar, bounds-checked
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, (uint32_t)M * (uint32_t)K * 2u, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, (uint32_t)N * (uint32_t)K * 2u, 0x00020000);
#endif
    // Transfers are issued unconditionally, so that every wave's count of outstanding transfers is the same in
    // every k-tile: a unit past the last k-tile re-reads the last one into a ring slot nobody reads any more.
    auto issue_unit = [&](int u, int ktile, int pos) {           // u is a compile-time constant after unrolling
#if defined(__HIP_DEVICE_COMPILE__)
      const int kc = ktile < nk ? ktile : nk - 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(u < UA ? rsA : rsW, (__attribute__((address_space(3))) void*)(gsm + pos * 8192 + wave * 1024), 16, uo[u], kc * (BK * 2), 0, 0);
#endif
    };
    int wpos = 0;                                                // ring position of the next unit to issue
#pragma unroll
    for (int q = 0; q < Q0; ++q) {
      issue_unit(q % U, q / U, wpos);
      wpos = wpos + 1 == R ? 0 : wpos + 1;
    }
    wait_vmem_upto<Q0 - U>();
    block_barrier();
    int rbase = 0;                                               // ring position of unit 0 of k-tile kt
    const int rowA = wm * (BM / WM), rowW = wn * (BN / WN);      // this wave's first row of either operand
    const int grp = wave >> 2;
    if (grp) block_barrier();
    // LDS byte addresses of this lane's fragment reads in the coming memory phase.  They are worked out in the
    // MFMA phase before it, between the wave's own MFMAs: a vector instruction of the memory phase would queue
    // behind the other wave's MFMAs on the SIMD, so the memory phases hold LDS reads, transfers and scalar
    // bookkeeping only.
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte*)gsm;   // LDS address of the ring
    uint32_t lk[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) lk[ks] = lds0 + (uint32_t)(l32 * BK + koff[ks]) * 2u;
    uint32_t ra[2][FM], rb[2][FN];
    auto set_addrs = [&](int base, int h) {
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        int pos = base + (rowA + i * 32) / 64; pos = pos >= R ? pos - R : pos;
        const uint32_t sa = (uint32_t)(pos * 8192 + ((rowA + i * 32) % 64) * (BK * 2));
        ra[0][i] = sa + lk[2 * h]; ra[1][i] = sa + lk[2 * h + 1];
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        int pos = base + UA + (rowW + j * 32) / 64; pos = pos >= R ? pos - R : pos;
        const uint32_t sb = (uint32_t)(pos * 8192 + ((rowW + j * 32) % 64) * (BK * 2));
        rb[0][j] = sb + lk[2 * h]; rb[1][j] = sb + lk[2 * h + 1];
      }
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {                           // keep the additions where they are written
#pragma unroll
        for (int i = 0; i < FM; ++i) asm volatile("" : "+v"(ra[ks][i]));
#pragma unroll
        for (int j = 0; j < FN; ++j) asm volatile("" : "+v"(rb[ks][j]));
      }
#endif
    };
    set_addrs(0, 0);
    for (int kt = 0; kt < nk; ++kt) {
      int rnext = rbase + U; rnext = rnext >= R ? rnext - R : rnext;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        bf16x8 a[2][FM], b[2][FN];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
          for (int i = 0; i < FM; ++i) a[ks][i] = *(lds_bf16x8*)(uintptr_t)ra[ks][i];
#pragma unroll
          for (int j = 0; j < FN; ++j) b[ks][j] = *(lds_bf16x8*)(uintptr_t)rb[ks][j];
        }
#pragma unroll
        for (int t = 0; t < (h == 0 ? UH0 : U - UH0); ++t) {
          const int qq = Q0 + (h == 0 ? 0 : UH0) + t;             // unit number relative to kt U
          issue_unit(qq % U, kt + qq / U, wpos);
          wpos = wpos + 1 == R ? 0 : wpos + 1;
        }
        if (h == 1 && grp) wait_vmem_upto<Q0 - U>();
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
#endif
        set_addrs(h == 0 ? rbase : rnext, h == 0 ? 1 : 0);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i], b[ks][j], acc[i][j], 0, 0, 0);
        if (h == 1 && !grp) wait_vmem_upto<Q0 - U>();
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
#endif
      }
      rbase = rnext;
    }
    if (!grp) block_barrier();
  } else {
  // loader: this lane's source offsets (elements) for the row groups its wave owns
  const int lrow = lane / CPR, lslot = lane % CPR;
  uint32_t ao[GA], wo[GW];
#pragma unroll
  for (int g = 0; g < GA; ++g) {
    const int rl = (wave * GA + g) * RPI + lrow;               // row within the tile
    int r = m0 + rl; r = r < M ? r : M - 1;
    ao[g] = (uint32_t)r * (uint32_t)K + ((lslot ^ ((rl / RPB) % CPR)) << 3);
  }
#pragma unroll
  for (int g = 0; g < GW; ++g) {
    const int rl = (wave * GW + g) * RPI + lrow;
    int c = n0 + rl; c = c < N ? c : N - 1;
    wo[g] = (uint32_t)c * (uint32_t)K + ((lslot ^ ((rl / RPB) % CPR)) << 3);
  }
  auto issue = [&](int kt, int buf) {
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int g = 0; g < GA; ++g)
      __builtin_amdgcn_global_load_lds(A + ao[g] + kt * BK, As + (buf * BM + (wave * GA + g) * RPI) * BK, 16, 0, 0);
#pragma unroll
    for (int g = 0; g < GW; ++g)
      __builtin_amdgcn_global_load_lds(W + wo[g] + kt * BK, Ws + (buf * BN + (wave * GW + g) * RPI) * BK, 16, 0, 0);
#endif
  };
  // prologue: STAGES - 1 k-tiles in flight
#pragma unroll
  for (int p = 0; p < STAGES - 1; ++p)
    if (p < nk) issue(p, p);
  int buf = 0;
  for (int kt = 0; kt < nk; ++kt) {
    // k-tile kt has landed once at most the STAGES - 2 younger tiles are still in flight
    if (kt + STAGES - 2 < nk) wait_vmem_upto<(STAGES - 2) * (GA + GW)>(); else wait_vmem_upto<0>();
    block_barrier();                                           // ... for every wave; and slab (kt - 1) % STAGES is free
    if (kt + STAGES - 1 < nk) issue(kt + STAGES - 1, buf == 0 ? STAGES - 1 : buf - 1);
    const bf16_t* as = As + (buf * BM + wm * (BM / WM) + l32) * BK;
    const bf16_t* ws = Ws + (buf * BN + wn * (BN / WN) + l32) * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[FM], b[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * BK + koff[ks]);
#pragma unroll
      for (int j = 0; j < FN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(ws + j * 32 * BK + koff[ks]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    buf = buf + 1 == STAGES ? 0 : buf + 1;
  }
  }
  if (MODE == EPI_CE) {
    // Cross-entropy partials instead of logits.  The product is taken transposed (rows = vocabulary entries,
    // columns = tokens), so a lane holds one token per fragment column and FM x 16 vocabulary rows of it in
    // registers: the maximum and the sum of exp(logit - max) over the wave's BM / WM vocabulary rows reduce
    // over registers plus one exchange with the partner lane (lane ^ 32).  Written to out as
    // float2 [tokens][tiles_m * WM]; the lane that meets the target row stores its logit.
    float2* part = reinterpret_cast<float2*>(out);
    const int pstride = tiles_m * WM, pcol = tm * WM + wm;
    const int rbase = m0 + wm * (BM / WM) + 4 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int token = n0 + wn * (BN / WN) + j * 32 + l32;
      const int tgt = token < N ? targets[token] : -1;
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
          if (r < M) { mx = fmaxf(mx, acc[i][j][v]); if (r == tgt) tlogit[token] = acc[i][j][v]; }
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float msafe = mx == -INFINITY ? 0.f : mx;            // a strip entirely beyond the vocabulary contributes (-inf, 0)
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
          if (r < M) sum += __builtin_amdgcn_exp2f((acc[i][j][v] - msafe) * 1.44269504088896341f);
        }
      sum += __shfl_xor(sum, 32, 64);
      if (lane < 32 && token < N) part[(size_t)token * pstride + pcol] = make_float2(mx, sum);
    }
    return;
  }
  // epilogue: lane holds column l32, rows 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 fragment
  float bv[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int n = n0 + wn * (BN / WN) + j * 32 + l32;
    bv[j] = (bias && n < N) ? to_f32(bias[n]) : 0.f;
  }
  const int mbase = m0 + wm * (BM / WM) + 4 * (lane >> 5), nbase = n0 + wn * (BN / WN) + l32;
  if (PRE_RES && pre_res) {
    float* op = reinterpret_cast<float*>(out) + (size_t)mbase * N + nbase;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          op[(size_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * N + j * 32] = res[(i * FN + j) * 16 + v] + (acc[i][j][v] + bv[j]);
  } else if (m0 + BM <= M && n0 + BN <= N) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          epilogue_bf16<MODE>(out, (size_t)(mbase + i * 32 + 8 * (v >> 2) + (v & 3)) * N + nbase + j * 32, acc[i][j][v] + bv[j]);
  } else {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int n = nbase + j * 32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = mbase + i * 32 + 8 * (v >> 2) + (v & 3);
          if (m < M && n < N) epilogue_bf16<MODE>(out, (size_t)m * N + n, acc[i][j][v] + bv[j]);
        }
      }
  }
}

template <int BM, int BN, int WM, int WN, int BK, int STAGES, int PP = 0>
hipError_t launch_gemm_bf16_t(const bf16_t* A, const bf16_t* W, const bf16_t* bias, void* out, int epi, int M, int N, int K, hipStream_t s,
                              const int32_t* targets = nullptr, float* tlogit = nullptr) {
  const size_t lds = PP ? (size_t)STAGES * 8192 : (size_t)STAGES * (BM + BN) * BK * sizeof(bf16_t);   // ping-pong: STAGES counts 8 KiB ring units
  // super-tiles of 4 x 8 tiles, rounded up to a multiple of 8 super-tiles (one per XCD)
  const int stm = ((M + BM - 1) / BM + 3) / 4, stn = ((N + BN - 1) / BN + 7) / 8;
  const int grid = ((stm * stn + 7) / 8 * 8) * 32;
#define ZGR_GEMM_LAUNCH(MODE)                                                                                           \
  {                                                                                                                     \
    static std::atomic<bool> attr_set{false};   /* set twice by racing threads at worst: the call is idempotent */         \
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, BK, STAGES, MODE, PP>;                                                             \
    if (!attr_set) {                                                                                                    \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
      if (e != hipSuccess) return e;                                                                                    \
      attr_set = true;                                                                                                  \
    }                                                                                                                   \
    hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WM * WN), lds, s, A, W, M, N, K, out, bias, targets, tlogit);        \
  }
  switch (epi) {
    case EPI_STORE: ZGR_GEMM_LAUNCH(EPI_STORE) break;
    case EPI_GELU:  ZGR_GEMM_LAUNCH(EPI_GELU) break;
    case EPI_RELU:  ZGR_GEMM_LAUNCH(EPI_RELU) break;
    case EPI_RESID: ZGR_GEMM_LAUNCH(EPI_RESID) break;
    case EPI_CE:    ZGR_GEMM_LAUNCH(EPI_CE) break;
    default:        ZGR_GEMM_LAUNCH(EPI_F32) break;
  }
#undef ZGR_GEMM_LAUNCH
  return hipGetLastError();
}

// ------------------------------------------------------------------ attention
// One thread per query row, one block per (batch, head, 256-query chunk); keys/values
// stream through LDS in chunks of 32; online softmax in fp32.
template <typename T, int DH>
__global__ void __launch_bounds__(256) attention_kernel(const T* __restrict__ qkv, T* __restrict__ ctx, const int32_t* __restrict__ lengths,
                                                        int seq, int d, int n_head, int causal) {
  constexpr int KC = 32;
  __shared__ float Ks[KC][DH], Vs[KC][DH];
  const int chunks = (seq + 255) / 256;
  const int qc = blockIdx.x % chunks, h = (blockIdx.x / chunks) % n_head, b = blockIdx.x / (chunks * n_head);
  const int qi = qc * 256 + threadIdx.x;
  const bool active = qi < seq;
  const int len = lengths ? lengths[b] : seq;
  const size_t ld = (size_t)3 * d;
  const T* base = qkv + (size_t)b * seq * ld + (size_t)h * DH;
  float q[DH], acc[DH];
  const float scale = 1.0f / sqrtf((float)DH);
#pragma unroll
  for (int i = 0; i < DH; ++i) { q[i] = active ? to_f32(base[(size_t)qi * ld + i]) * scale : 0.f; acc[i] = 0.f; }
  float mx = -INFINITY, den = 0.f;
  int kend = len < seq ? len : seq;
  if (causal) { const int last = qc * 256 + 255; kend = kend < last + 1 ? kend : last + 1; }
  for (int k0 = 0; k0 < kend; k0 += KC) {
    __syncthreads();
    for (int i = threadIdx.x; i < KC * DH; i += 256) {
      const int r = i / DH, c = i - r * DH;
      const int kj = k0 + r;
      Ks[r][c] = kj < seq ? to_f32(base[(size_t)kj * ld + d + c]) : 0.f;
      Vs[r][c] = kj < seq ? to_f32(base[(size_t)kj * ld + 2 * d + c]) : 0.f;
    }
    __syncthreads();
    if (!active) continue;
    for (int r = 0; r < KC; ++r) {
      const int kj = k0 + r;
      if (kj >= kend || (causal && kj > qi)) break;
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < DH; ++i) s = __builtin_fmaf(q[i], Ks[r][i], s);
      const float nm = fmaxf(mx, s);
      const float corr = __expf(mx - nm), p = __expf(s - nm);
      den = den * corr + p;
#pragma unroll
      for (int i = 0; i < DH; ++i) acc[i] = __builtin_fmaf(p, Vs[r][i], acc[i] * corr);
      mx = nm;
    }
  }
  if (active) {
    T* o = ctx + ((size_t)b * seq + qi) * d + (size_t)h * DH;
    const float inv = den > 0.f ? 1.0f / den : 0.f;
#pragma unroll
    for (int i = 0; i < DH; ++i) from_f32(acc[i] * inv, o[i]);
  }
}

// MFMA attention for bf16 storage and head size 64.  One block = 128 queries of one (batch, head):
// K [keys][64] and V^T [64][keys] are staged in LDS (all keys at once up to AT_KCH of them, chunk after chunk of
// AT_KCH beyond: the online softmax carries over); each wave owns 32 queries and walks the keys in
// blocks of 32, computing S^T = K Q^T and O^T += V^T P^T with v_mfma_f32_32x32x16_bf16.  In the S^T
// result a lane holds one query column and 16 keys in registers, so the softmax reductions run over
// registers plus one exchange with the partner lane (lane ^ 32); P goes straight from the accumulator
// registers into the B operand of the second product (the contraction order of that product is the
// accumulator's key order, which the V^T operand is read in as well).
constexpr int AT_LDK = 64 + 8;          // K row stride (bf16): 144 B
constexpr int AT_KCH = 512;             // keys staged at a time: 72 KB of K rows + 65 KB of V^T
// NW waves per block, 32 queries each: with NW = 8 one block covers 256 queries of a head, so K and V^T of a
// 256-token sequence are staged once per head instead of once per 128 queries.
template <int DH, int NW>
__global__ void __launch_bounds__(64 * NW) attention_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx, const int32_t* __restrict__ lengths,
                                                                 int seq, int d, int n_head, int causal, int kpad) {
  static_assert(DH == 64, "head size 64");
  constexpr int QB = 32 * NW, NT = 64 * NW;                     // queries and threads per block
  extern __shared__ __attribute__((aligned(16))) unsigned char asm_[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(asm_);                 // [kpad][AT_LDK]
  bf16_t* Vt = Ks + (size_t)kpad * AT_LDK;                      // [DH][kpad + 8]
  const int ldv = kpad + 8;
  const int qblocks = (seq + QB - 1) / QB;
  // Under the causal mask a query block's work grows with its position: the blocks are handed out longest first (all heads'
  // last query blocks, then the ones before, ...), so that the short ones fill the gaps at the end of the launch.
  const int heads = gridDim.x / qblocks;
  const int qb = (causal && qblocks > 1) ? qblocks - 1 - (int)blockIdx.x / heads : (int)blockIdx.x % qblocks;
  const int bh = (causal && qblocks > 1) ? (int)blockIdx.x % heads : (int)blockIdx.x / qblocks;
  const int h = bh % n_head, b = bh / n_head;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int len = lengths ? min(lengths[b], seq) : seq;
  const size_t ld = (size_t)3 * d;
  const bf16_t* base = qkv + (size_t)b * seq * ld + (size_t)h * DH;
  // keys this block can need, rounded up to 32
  int kend = len;
  if (causal) kend = min(kend, qb * QB + QB);
  const int kblocks = (kend + 31) / 32;
  // this wave's queries: B operand of S^T = K Q^T, lane (query l32, k-group half) holds Q[q][16 s + 8 half .. +8]
  // Under the causal mask a wave's work grows with the position of its queries.  Waves w and w + 4 share a SIMD, so
  // with eight waves the upper four take their query groups in reverse order: every SIMD then holds the same total.
  const int qgroup = (NW == 8 && causal && wave >= 4) ? 11 - wave : wave;
  const int q0 = qb * QB + qgroup * 32;
  const int qi = q0 + l32;
  bf16x8 qf[DH / 16];
#pragma unroll
  for (int s4 = 0; s4 < DH / 16; ++s4) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (qi < seq) t = *reinterpret_cast<const uint4*>(base + (size_t)qi * ld + s4 * 16 + half * 8);
    qf[s4] = *reinterpret_cast<bf16x8*>(&t);
  }
  f32x16 o[DH / 32];
#pragma unroll
  for (int f = 0; f < DH / 32; ++f)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[f][v] = 0.f;
  float mx = -INFINITY, lsum = 0.f;
  const float scale_log2 = 1.44269504088896341f / sqrtf((float)DH);
  int wave_kblocks = kblocks;
  if (causal) wave_kblocks = min(kblocks, (q0 + 31) / 32 + 1);
  if (q0 >= seq) wave_kblocks = 0;
  for (int c0 = 0; c0 < kblocks; c0 += AT_KCH / 32) {                 // key chunks: the same trip count for every wave of the block
    const int c_end = min(kblocks, c0 + AT_KCH / 32);
    if (c0 > 0) __syncthreads();                                         // every wave is done with the previous chunk
    // stage K and V^T of key blocks [c0, c_end) (zero beyond seq so masked products stay finite)
    for (int i = tid; i < (c_end - c0) * 32 * 8; i += NT) {
      const int r = i >> 3, c = (i & 7) * 8, key = c0 * 32 + r;
      uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (key < seq) {
        kv = *reinterpret_cast<const uint4*>(base + (size_t)key * ld + d + c);
        vv = *reinterpret_cast<const uint4*>(base + (size_t)key * ld + 2 * d + c);
      }
      *reinterpret_cast<uint4*>(Ks + r * AT_LDK + c) = kv;
      const uint16_t* ve = reinterpret_cast<const uint16_t*>(&vv);
#pragma unroll
      for (int j = 0; j < 8; ++j) Vt[(c + j) * ldv + r].bits = ve[j];
    }
    __syncthreads();
    for (int kb = c0; kb < min(c_end, wave_kblocks); ++kb) {
      const int kl = (kb - c0) * 32;                                      // the block's first key within the staged chunk
      f32x16 sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
      for (int s4 = 0; s4 < DH / 16; ++s4) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + (kl + l32) * AT_LDK + s4 * 16 + half * 8);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s4], sacc, 0, 0, 0);
      }
      // lane: query qi, keys kb*32 + 8*(v/4) + 4*half + v%4; scores in log2 units
      float sv[16], mloc = -INFINITY;
      if (kb * 32 + 31 < len && (!causal || kb * 32 + 31 <= q0)) {      // every key of the block is visible to every query of the wave
#pragma unroll
        for (int v = 0; v < 16; ++v) { sv[v] = sacc[v] * scale_log2; mloc = fmaxf(mloc, sv[v]); }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = kb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
          const bool ok = key < len && (!causal || key <= qi);
          sv[v] = ok ? sacc[v] * scale_log2 : -INFINITY;
          mloc = fmaxf(mloc, sv[v]);
        }
      }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
      const float mnew = fmaxf(mx, mloc);
      const float msafe = mnew == -INFINITY ? 0.f : mnew;
      // v_exp_f32 directly: the arguments are <= 0 (or -inf, which gives 0), so the library routine's range handling is not needed
      const float corr = __builtin_amdgcn_exp2f(mx - msafe);            // mx = -inf -> 0
      float psum = 0.f;
      union { uint32_t w[4]; bf16x8 v; } pk[2];                          // P^T operand: two probabilities per conversion
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float p0 = __builtin_amdgcn_exp2f(sv[v] - msafe), p1 = __builtin_amdgcn_exp2f(sv[v + 1] - msafe);
        psum += p0 + p1;
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 pp = {p0, p1};
        pk[v >> 3].w[(v & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, bf16x2));
      }
      const bf16x8 pf[2] = {pk[0].v, pk[1].v};
      lsum = lsum * corr + psum;
      mx = mnew;
      if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {              // nothing to rescale while no lane's maximum moved
#pragma unroll
        for (int f = 0; f < DH / 32; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[f][v] *= corr;
      }
      // O^T += V^T P^T: A operand lane (dh row 32 f + l32, half) reads the keys in the accumulator's order
#pragma unroll
      for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int f = 0; f < DH / 32; ++f) {
          const bf16_t* vr = Vt + (f * 32 + l32) * ldv + kl + st * 16 + 4 * half;
          const uint2 lo = *reinterpret_cast<const uint2*>(vr), hi = *reinterpret_cast<const uint2*>(vr + 8);
          uint4 t = make_uint4(lo.x, lo.y, hi.x, hi.y);
          o[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&t), pf[st], o[f], 0, 0, 0);
        }
      }
    }
  }
  lsum += __shfl_xor(lsum, 32, 64);
  if (qi < seq) {
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16_t* orow = ctx + ((size_t)b * seq + qi) * d + (size_t)h * DH;
#pragma unroll
    for (int f = 0; f < DH / 32; ++f)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        uint16_t pk[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { bf16_t t; from_f32(o[f][v4 * 4 + i] * inv, t); pk[i] = t.bits; }
        *reinterpret_cast<uint2*>(orow + f * 32 + 8 * v4 + 4 * half) = *reinterpret_cast<uint2*>(pk);
      }
  }
}

// ------------------------------------------------------------------ losses
// Cross-entropy of one row of fp32 logits [n]: loss = logsumexp - logit[target]; target < 0: row skipped (loss 0).
__global__ void __launch_bounds__(256) ce_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ targets, float* __restrict__ row_loss,
                                                      int n, int vocab_clamp) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  int tgt = targets[m];
  if (tgt < 0) { if (threadIdx.x == 0) row_loss[m] = 0.f; return; }
  tgt = tgt >= vocab_clamp ? vocab_clamp - 1 : tgt;
  const float* row = logits + (size_t)m * n;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < n; i += 256) mx = fmaxf(mx, row[i]);
  mx = block_max(mx, red);
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += expf(row[i] - mx);
  s = block_sum(s, red);
  if (threadIdx.x == 0) row_loss[m] = logf(s) + mx - row[tgt];
}

// Combines the cross-entropy partials of one row: loss = log(sum_i s_i exp(m_i - M)) + M - logit[target].
__global__ void __launch_bounds__(256) ce_combine_kernel(const float2* __restrict__ part, int n_part, const int32_t* __restrict__ targets,
                                                         const float* __restrict__ tlogit, float* __restrict__ row_loss) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  if (targets[m] < 0) { if (threadIdx.x == 0) row_loss[m] = 0.f; return; }
  const float2* row = part + (size_t)m * n_part;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < n_part; i += 256) mx = fmaxf(mx, row[i].x);
  mx = block_max(mx, red);
  float s = 0.f;
  for (int i = threadIdx.x; i < n_part; i += 256) s += row[i].y * expf(row[i].x - mx);
  s = block_sum(s, red);
  if (threadIdx.x == 0) row_loss[m] = logf(s) + mx - tlogit[m];
}

// next-token targets: row m = b*seq + t predicts tok[m+1] for t < seq-1, else -1
__global__ void lm_targets_kernel(const int32_t* __restrict__ tok, int32_t* __restrict__ tgt, int M, int seq, int vocab) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= M) return;
  int t = -1;
  if ((m % seq) < seq - 1) { t = tok[m + 1]; t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t); }   // same clamp as the embedding
  tgt[m] = t;
}

// mean of n_rows losses (ignoring the skipped ones by dividing by `count`), accumulated in fp64
__global__ void __launch_bounds__(256) mean_f64_kernel(const float* __restrict__ v, int n, double inv_count, double* __restrict__ out) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += (double)v[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) { if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o]; __syncthreads(); }
  if (threadIdx.x == 0) *out = red[0] * inv_count;
}

// classification head on token 0 of every sequence: logits[b][c] = h[b*seq] . Wc[c] + bc[c]
template <typename T>
__global__ void __launch_bounds__(64) cls_head_kernel(const T* __restrict__ h, const T* __restrict__ Wc, const T* __restrict__ bc, float* __restrict__ logits,
                                                      int seq, int d, int n_class) {
  const int b = blockIdx.x / n_class, c = blockIdx.x % n_class;
  const T* x = h + (size_t)b * seq * d;
  const T* w = Wc + (size_t)c * d;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 64) s = __builtin_fmaf(to_f32(x[i]), to_f32(w[i]), s);
  s = wave_sum(s);
  if (threadIdx.x == 0) logits[b * n_class + c] = s + to_f32(bc[c]);
}

// least squares: row_loss[b] = sum_o (pred[b][o] - Y[b][o])^2 / 2
__global__ void __launch_bounds__(256) lsq_rows_kernel(const float* __restrict__ pred, const float* __restrict__ Y, float* __restrict__ row_loss, int n_out) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  float s = 0.f;
  for (int i = threadIdx.x; i < n_out; i += 256) { const float r = pred[(size_t)b * n_out + i] - Y[(size_t)b * n_out + i]; s = __builtin_fmaf(r, r, s); }
  s = block_sum(s, red);
  if (threadIdx.x == 0) row_loss[b] = 0.5f * s;
}

}  // namespace

// ------------------------------------------------------------------ host launchers
hipError_t launch_embed(int dtype, const int32_t* tok, const void* E, const void* Pe, float* x, int M, int seq, int d, int vocab, hipStream_t s) {
  if (dtype == 0) hipLaunchKernelGGL(embed_kernel<float>, dim3(M), dim3(256), 0, s, tok, (const float*)E, (const float*)Pe, x, M, seq, d, vocab);
  else            hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(M), dim3(256), 0, s, tok, (const bf16_t*)E, (const bf16_t*)Pe, x, M, seq, d, vocab);
  return hipGetLastError();
}

hipError_t launch_layernorm(int dtype, const float* x, const void* g, const void* b, void* out, int M, int d, float eps, hipStream_t s, float* xout) {
  if (d % 4 == 0 && d <= 2048 && (((uintptr_t)g | (uintptr_t)b | (uintptr_t)out | (uintptr_t)xout) & 15) == 0) {
    const dim3 grid((unsigned)((M + 3) / 4));
    if (dtype == 0) hipLaunchKernelGGL(layernorm_wave_kernel<float>, grid, dim3(256), 0, s, x, (const float*)g, (const float*)b, (float*)out, M, d, eps, xout);
    else            hipLaunchKernelGGL(layernorm_wave_kernel<bf16_t>, grid, dim3(256), 0, s, x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)out, M, d, eps, xout);
    return hipGetLastError();
  }
  if (d % 4 == 0 && d <= 8192 && (((uintptr_t)g | (uintptr_t)b | (uintptr_t)out | (uintptr_t)xout) & 15) == 0) {
    if (dtype == 0) hipLaunchKernelGGL(layernorm_reg_kernel<float>, dim3(M), dim3(256), 0, s, x, (const float*)g, (const float*)b, (float*)out, d, eps, xout);
    else            hipLaunchKernelGGL(layernorm_reg_kernel<bf16_t>, dim3(M), dim3(256), 0, s, x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)out, d, eps, xout);
    return hipGetLastError();
  }
  if (dtype == 0) hipLaunchKernelGGL(layernorm_kernel<float>, dim3(M), dim3(256), 0, s, x, (const float*)g, (const float*)b, (float*)out, d, eps, xout);
  else            hipLaunchKernelGGL(layernorm_kernel<bf16_t>, dim3(M), dim3(256), 0, s, x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)out, d, eps, xout);
  return hipGetLastError();
}

hipError_t launch_gemm(int dtype, const void* A, const void* W, const void* bias, void* out, int epi, int M, int N, int K, hipStream_t s) {
  GemmEpi ep{epi, out, bias};
  if (dtype == 0) {
    const bool mfma_ok = K % 4 == 0 && (((uintptr_t)A | (uintptr_t)W) & 15) == 0;
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (mfma_ok && t128 >= 512)   // enough 128 x 128 tiles for two blocks on every CU
      hipLaunchKernelGGL((gemm_f32_mfma_kernel<2, 16>), dim3((N + 127) / 128, (M + 127) / 128), dim3(256), 0, s, (const float*)A, (const float*)W, M, N, K, ep);
    else if (mfma_ok)
      hipLaunchKernelGGL((gemm_f32_mfma_kernel<1, 16>), dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, s, (const float*)A, (const float*)W, M, N, K, ep);
    else
      hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, s, (const float*)A, (const float*)W, M, N, K, ep);
  } else {
    if (K % GB_K != 0) return hipErrorInvalidValue;
    const bf16_t* a = (const bf16_t*)A; const bf16_t* w = (const bf16_t*)W; const bf16_t* b = (const bf16_t*)bias;
    // largest tile that still gives every CU a block
    const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256), t128x256 = (long)((M + 127) / 128) * ((N + 255) / 256);
    if ((size_t)M * K >= ((size_t)1 << 31) || (size_t)N * K >= ((size_t)1 << 31)) return hipErrorInvalidValue;   // 32-bit byte offsets
    // 256 x 256 tiles unless their count leaves the last round of 256 CUs less than ~85 % full and 256 x 192 tiles fill it better
    const long t192 = (long)((M + 255) / 256) * ((N + 191) / 192);
    auto fill = [](long t) { const long rounds = (t + 255) / 256; return (double)t / (double)(rounds * 256); };
    if (t256 >= 256 && (fill(t256) >= 0.85 || fill(t192) <= fill(t256))) return launch_gemm_bf16_t<256, 256, 2, 4, 64, 20, 1>(a, w, b, out, epi, M, N, K, s);
    if (t192 >= 256 && N % 192 == 0) return launch_gemm_bf16_t<256, 192, 4, 2, 64, 20, 1>(a, w, b, out, epi, M, N, K, s);
    if (t256 >= 256) return launch_gemm_bf16_t<256, 256, 2, 4, 64, 20, 1>(a, w, b, out, epi, M, N, K, s);
    if (t128x256 >= 200) return launch_gemm_bf16_t<128, 256, 2, 4, 64, 20, 1>(a, w, b, out, epi, M, N, K, s);
    // small problems.  More 128 x 128 tiles than CUs: the ping-pong loop on a short ring (64 KB, two blocks per CU, one block's
    // epilogue under the other's loop).  Fewer than half the CUs would get such a tile: 64 x 64 tiles with the plain loop
    // (four times the blocks, two of them per CU; 64 x 128 tiles were a few per cent slower).
    // In between (about one tile per CU): the ping-pong loop on the full ring.
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (t128 > 256) return launch_gemm_bf16_t<128, 128, 2, 4, 64, 8, 1>(a, w, b, out, epi, M, N, K, s);
    if (t128 <= 128) return launch_gemm_bf16_t<64, 64, 2, 2, 64, 4>(a, w, b, out, epi, M, N, K, s);
    return launch_gemm_bf16_t<128, 128, 2, 4, 64, 20, 1>(a, w, b, out, epi, M, N, K, s);
  }
  return hipGetLastError();
}

// Vocabulary projection fused with the row-wise cross-entropy (bf16 storage): logits are never stored.
// part: float2 scratch of ce_partials_per_row(N) entries per row; tlogit: float [M].
int ce_partials_per_row(int N) { return ((N + 255) / 256) * 2; }

hipError_t launch_gemm_ce_bf16(const void* A, const void* W, const int32_t* targets, void* part, float* tlogit, float* row_loss, int M, int N, int K, hipStream_t s) {
  if (K % GB_K != 0 || (size_t)M * K >= ((size_t)1 << 31) || (size_t)N * K >= ((size_t)1 << 31)) return hipErrorInvalidValue;
  // transposed product: the kernel's rows are the N vocabulary entries, its columns the M tokens
  hipError_t e = launch_gemm_bf16_t<256, 256, 2, 4, 64, 20, 1>((const bf16_t*)W, (const bf16_t*)A, nullptr, part, EPI_CE, N, M, K, s, targets, tlogit);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(ce_combine_kernel, dim3(M), dim3(256), 0, s, (const float2*)part, ce_partials_per_row(N), targets, tlogit, row_loss);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_attention_t(const T* qkv, T* ctx, const int32_t* lengths, int batch, int seq, int d, int n_head, int causal, hipStream_t s) {
  const int dh = d / n_head;
  const int grid = batch * n_head * ((seq + 255) / 256);
  switch (dh) {
    case 8:   hipLaunchKernelGGL((attention_kernel<T, 8>), dim3(grid), dim3(256), 0, s, qkv, ctx, lengths, seq, d, n_head, causal); break;
    case 16:  hipLaunchKernelGGL((attention_kernel<T, 16>), dim3(grid), dim3(256), 0, s, qkv, ctx, lengths, seq, d, n_head, causal); break;
    case 32:  hipLaunchKernelGGL((attention_kernel<T, 32>), dim3(grid), dim3(256), 0, s, qkv, ctx, lengths, seq, d, n_head, causal); break;
    case 64:  hipLaunchKernelGGL((attention_kernel<T, 64>), dim3(grid), dim3(256), 0, s, qkv, ctx, lengths, seq, d, n_head, causal); break;
    default:  return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_attention(int dtype, const void* qkv, void* ctx, const int32_t* lengths, int batch, int seq, int d, int n_head, int causal, hipStream_t s) {
  if (dtype == 1 && d / n_head == 64 && d % 8 == 0) {
    const int kpad = seq < AT_KCH ? (seq + 31) / 32 * 32 : AT_KCH;          // keys resident in LDS at a time
    const size_t lds = sizeof(bf16_t) * ((size_t)kpad * AT_LDK + (size_t)64 * (kpad + 8));
    static std::atomic<bool> attr_set{false};     // set twice by racing threads at worst: the calls are idempotent
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_kernel<64, 4>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_kernel<64, 8>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    if (seq > 128) {      // 256 queries per block: the keys of a head are staged once per 256 queries
      const int grid = batch * n_head * ((seq + 255) / 256);
      hipLaunchKernelGGL((attention_mfma_kernel<64, 8>), dim3(grid), dim3(512), lds, s, (const bf16_t*)qkv, (bf16_t*)ctx, lengths, seq, d, n_head, causal, kpad);
    } else {
      const int grid = batch * n_head * ((seq + 127) / 128);
      hipLaunchKernelGGL((attention_mfma_kernel<64, 4>), dim3(grid), dim3(256), lds, s, (const bf16_t*)qkv, (bf16_t*)ctx, lengths, seq, d, n_head, causal, kpad);
    }
    return hipGetLastError();
  }
  if (dtype == 0) return launch_attention_t<float>((const float*)qkv, (float*)ctx, lengths, batch, seq, d, n_head, causal, s);
  return launch_attention_t<bf16_t>((const bf16_t*)qkv, (bf16_t*)ctx, lengths, batch, seq, d, n_head, causal, s);
}

bool attention_head_dim_supported(int dh) { return dh == 8 || dh == 16 || dh == 32 || dh == 64; }

hipError_t launch_lm_targets(const int32_t* tok, int32_t* tgt, int M, int seq, int vocab, hipStream_t s) {
  hipLaunchKernelGGL(lm_targets_kernel, dim3((M + 255) / 256), dim3(256), 0, s, tok, tgt, M, seq, vocab);
  return hipGetLastError();
}

hipError_t launch_ce_rows(const float* logits, const int32_t* targets, float* row_loss, int M, int n, hipStream_t s) {
  hipLaunchKernelGGL(ce_rows_kernel, dim3(M), dim3(256), 0, s, logits, targets, row_loss, n, n);
  return hipGetLastError();
}

hipError_t launch_mean_f64(const float* v, int n, double inv_count, double* out, hipStream_t s) {
  hipLaunchKernelGGL(mean_f64_kernel, dim3(1), dim3(256), 0, s, v, n, inv_count, out);
  return hipGetLastError();
}

hipError_t launch_cls_head(int dtype, const void* h, const void* Wc, const void* bc, float* logits, int batch, int seq, int d, int n_class, hipStream_t s) {
  if (dtype == 0) hipLaunchKernelGGL(cls_head_kernel<float>, dim3(batch * n_class), dim3(64), 0, s, (const float*)h, (const float*)Wc, (const float*)bc, logits, seq, d, n_class);
  else            hipLaunchKernelGGL(cls_head_kernel<bf16_t>, dim3(batch * n_class), dim3(64), 0, s, (const bf16_t*)h, (const bf16_t*)Wc, (const bf16_t*)bc, logits, seq, d, n_class);
  return hipGetLastError();
}

hipError_t launch_lsq_rows(const float* pred, const float* Y, float* row_loss, int batch, int n_out, hipStream_t s) {
  hipLaunchKernelGGL(lsq_rows_kernel, dim3(batch), dim3(256), 0, s, pred, Y, row_loss, n_out);
  return hipGetLastError();
}

}  // namespace zgr
