// In-place perturbation pass theta <- rnd(theta + c Z), Z = a G + b U R (Eq. (10)),
// with G and R regenerated from the shared seed in registers / LDS and never
// stored (Sec. 3.1 step 5; Algorithm 1, client and edge-server blocks).  One
// pass reads and writes every parameter exactly once.
//
// Two persistent kernels per pass, each looping over a work list:
//   flat: tensors without a basis (embeddings, biases, LayerNorm, non-guided
//         rounds): one thread per Philox call, fully coalesced vector RMW;
//   tile: guided matrices: a block owns a [rows x 32P] column strip piece,
//         generates its slice of R once into LDS, stages U row blocks in LDS,
//         contracts U R in registers and fuses G, the mix and the axpy.
#include "internal.h"

#include <atomic>
#include <mutex>

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

template <typename T, int P> struct alignas(sizeof(T) * P <= 16 ? sizeof(T) * P : 16) Vec { T v[P]; };

// P fp32 results into the storage type: fp32 as they are, bf16 rounded two at a time (one v_cvt_pk_bf16_f32 per pair,
// which leaves the pair in the dword it is stored from).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <int P> __device__ __forceinline__ void round_into(Vec<float, P>& x, const float* f) {
#pragma unroll
  for (int j = 0; j < P; ++j) x.v[j] = f[j];
}
template <int P> __device__ __forceinline__ void round_into(Vec<bf16_t, P>& x, const float* f) {
#pragma unroll
  for (int j = 0; j < P; j += 2) {
    const bf16x2_t r = __builtin_convertvector(f32x2_t{f[j], f[j + 1]}, bf16x2_t);
    const uint32_t bits = __builtin_bit_cast(uint32_t, r);
    x.v[j].bits = (uint16_t)bits;
    x.v[j + 1].bits = (uint16_t)(bits >> 16);
  }
}

// theta pointers come out of descriptors in memory, so the compiler cannot know that they point to global
// memory and would emit FLAT accesses (which also tie up the LDS counter); say so explicitly.
template <typename V> __device__ __forceinline__ V load_global(const void* p) {
  typedef uint32_t R __attribute__((ext_vector_type(sizeof(V) / 4)));
  typedef const R __attribute__((address_space(1))) GR;
  const R r = *reinterpret_cast<GR*>(reinterpret_cast<uintptr_t>(p));
  V v;
  __builtin_memcpy(&v, &r, sizeof(V));
  return v;
}
template <> __device__ __forceinline__ float load_global<float>(const void* p) {
  typedef const float __attribute__((address_space(1))) GF;
  return *reinterpret_cast<GF*>(reinterpret_cast<uintptr_t>(p));
}
template <typename V> __device__ __forceinline__ void store_global(void* p, const V& v) {
  typedef uint32_t R __attribute__((ext_vector_type(sizeof(V) / 4)));
  typedef R __attribute__((address_space(1))) GR;
  R r;
  __builtin_memcpy(&r, &v, sizeof(V));
  *reinterpret_cast<GR*>(reinterpret_cast<uintptr_t>(p)) = r;
}

__device__ __forceinline__ float load_global_elem(const float* p) { return load_global<float>(p); }
__device__ __forceinline__ bf16_t load_global_elem(const bf16_t* p) {
  typedef const uint16_t __attribute__((address_space(1))) GH;
  bf16_t r; r.bits = *reinterpret_cast<GH*>(reinterpret_cast<uintptr_t>(p)); return r;
}
__device__ __forceinline__ void store_global_elem(float* p, float v) {
  typedef float __attribute__((address_space(1))) GF;
  *reinterpret_cast<GF*>(reinterpret_cast<uintptr_t>(p)) = v;
}
__device__ __forceinline__ void store_global_elem(bf16_t* p, bf16_t v) {
  typedef uint16_t __attribute__((address_space(1))) GH;
  *reinterpret_cast<GH*>(reinterpret_cast<uintptr_t>(p)) = v.bits;
}

// A descriptor or work-list entry read through the constant address space: these tables are never written by a
// kernel, and only a load the compiler knows to be invariant may use the scalar unit however many stores to theta
// surround it (as a vector load it would have to be waited for behind the stores issued just before it).
template <typename S> __device__ __forceinline__ S load_const(const S* p) {
  static_assert(sizeof(S) % 4 == 0, "whole words");
  typedef const uint32_t __attribute__((address_space(4))) CW;
  CW* w = reinterpret_cast<CW*>(reinterpret_cast<uintptr_t>(p));
  uint32_t buf[sizeof(S) / 4];
#pragma unroll
  for (size_t i = 0; i < sizeof(S) / 4; ++i) buf[i] = w[i];
  S s;
  __builtin_memcpy(&s, buf, sizeof(S));
  return s;
}

template <int P> __device__ __forceinline__ void gaussP(const u32x4 w, const RadiusEntry* tab, float* g);
template <> __device__ __forceinline__ void gaussP<4>(const u32x4 w, const RadiusEntry* tab, float* g) { gauss4(w, tab, g); }
template <> __device__ __forceinline__ void gaussP<8>(const u32x4 w, const RadiusEntry* tab, float* g) { gauss8(w, tab, g); }

// Element [row][l] of the basis: fp32 as stored, or restored from its 4-bit code as lambda (code - delta)
// (Sec. 3.4, first equation): the restore is fused into the operand load, the fp32 basis never exists in memory.
__device__ __forceinline__ float basis_at(const TensorDesc& d, int64_t row, int l) {
  if (d.Uq) {
    const uint32_t byte = d.Uq[row * d.ldu + (l >> 1)];
    const uint32_t code = (l & 1) ? (byte >> 4) : (byte & 15u);
    return d.qlambda * ((float)code - d.qdelta);
  }
  return load_global<float>(d.U + row * d.ldu + l);
}

// Layer pipeline (Sec. 3.3): a launch also fetches the basis data its successor will need, straight from pinned
// host memory into the staging slot the successor reads.  The last a.pull_blocks blocks of the grid do nothing
// else (a block that waited for the host link before computing would delay its share of the tiles by that long);
// the other blocks share the work list among themselves.  The kernel boundary makes the data visible.
__device__ __forceinline__ void pull_next_stage(const PerturbArgs& a, int part, int parts) {
  for (int t = 0; t < a.n_stage; ++t) {
    const StageCopy sc = a.stage[t];
    const uint64_t n16 = sc.bytes >> 4;
    const uint4* src = reinterpret_cast<const uint4*>(sc.src);
    uint4* dst = reinterpret_cast<uint4*>(sc.dst);
    for (uint64_t i = (uint64_t)part * blockDim.x + threadIdx.x; i < n16; i += (uint64_t)parts * blockDim.x) dst[i] = src[i];
    if (part == 0)
      for (uint64_t i = (n16 << 4) + threadIdx.x; i < sc.bytes; i += blockDim.x) sc.dst[i] = sc.src[i];
  }
}

__global__ void __launch_bounds__(256) stage_only_kernel(PerturbArgs a) { pull_next_stage(a, blockIdx.x, gridDim.x); }

// The P Gaussians of Philox call q of one stream.  BATCH: instead the combination sum_i qcoef[i] * (those of step
// qstep[i]), accumulated in the order of the list; since Z is linear in (G, R), a batched pass is the single
// pass with this combination in place of G and of R and the coefficient 1.
template <int P, bool BATCH>
__device__ __forceinline__ void draw(uint64_t q, uint32_t id_stream, const PerturbArgs& a, const RadiusEntry* tab, float* g) {
  if (!BATCH) {
    gaussP<P>(philox_call(q, id_stream, a.step, a.k0, a.k1), tab, g);
  } else {
#pragma unroll
    for (int j = 0; j < P; ++j) g[j] = 0.f;
    for (int i = 0; i < a.n_q; ++i) {
      float t[P];
      gaussP<P>(philox_call(q, id_stream, a.qstep[i], a.k0, a.k1), tab, t);
      const float ci = a.qcoef[i];
#pragma unroll
      for (int j = 0; j < P; ++j) g[j] = __builtin_fmaf(ci, t[j], g[j]);
    }
  }
}

// The work list and the tensor descriptors are separate __restrict__ kernel parameters (besides being members
// of PerturbArgs): only then can the compiler tell that the stores to theta do not change them, and fetch them
// with scalar loads.  Fetched through the struct they become vector loads behind an s_waitcnt vmcnt(0), which
// drains every outstanding load and store of the wave once per work item.
// ------------------------------------------------------------------ flat
// Materialiser of Z for the isotropic tensors (test boundary only): one thread per Philox call.
template <typename T, int P>
__global__ void __launch_bounds__(256) fill_flat_kernel(PerturbArgs a, const TensorDesc* __restrict__ descs, const WorkItem* __restrict__ items,
                                                        const RadiusEntry* __restrict__ gtab, float* __restrict__ zout) {
  __shared__ RadiusEntry tab[kRadiusTabEntries];
  load_radius_table(tab, gtab);
  __syncthreads();
  for (int w = blockIdx.x; w < a.n_flat; w += gridDim.x) {
    const WorkItem it = items[w];
    const TensorDesc d = descs[it.tensor];
    const int64_t n = d.rows * d.cols;
    for (int g = threadIdx.x; g < it.count; g += 256) {
      const int64_t q = it.first + g;
      float G[P];
      draw<P, false>((uint64_t)q, d.id, a, tab, G);
      for (int j = 0; j < P; ++j) if (q * P + j < n) zout[q * P + j] = G[j];
    }
  }
}

// The registers of v as inputs of an empty statement: whatever they are waiting for (a load issued long ago) is
// waited for HERE.  The compiler places the wait for an outstanding load in front of the first use of its
// registers, and that wait also covers every store issued before it; anchoring it in front of a store, at a point
// where the load is a whole work item old, keeps the write it would otherwise have to sit out behind it.
template <typename V> __device__ __forceinline__ void wait_here_for(const V& v) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t R __attribute__((ext_vector_type(sizeof(V) / 4 > 4 ? 4 : sizeof(V) / 4)));
  R r[sizeof(V) / sizeof(R)];
  __builtin_memcpy(r, &v, sizeof(V));
#pragma unroll
  for (size_t i = 0; i < sizeof(V) / sizeof(R); ++i) asm volatile("" ::"v"(r[i]));
#endif
}

// In-place pass over the isotropic tensors.  A work item is flat_groups_per_item Philox calls of one tensor; a
// thread owns the calls tid, tid + 256, ... of it (flat_slots of them, 64 bytes per lane).  The parameters of the NEXT item of the
// block are requested before the generator runs for the current one, so kFlatSlots vectors per lane are in
// flight under a whole item's arithmetic: the pass needs about 20 KB of reads in flight per compute unit to
// keep HBM busy, and one 8-byte request per lane at a time, waited for after one call, supplies less than that.
template <typename T, int P, bool BATCH>
__global__ void __launch_bounds__(256) perturb_flat_kernel(PerturbArgs a, const TensorDesc* __restrict__ descs, const WorkItem* __restrict__ items,
                                                           float c, const RadiusEntry* __restrict__ gtab) {
  __shared__ RadiusEntry tab[kRadiusTabEntries];
  constexpr int kFlatSlots = flat_slots((int)sizeof(T), P);
  const int nblk = (int)gridDim.x - a.pull_blocks;               // computing blocks
  if ((int)blockIdx.x >= nblk) { pull_next_stage(a, (int)blockIdx.x - nblk, a.pull_blocks); return; }
  load_radius_table(tab, gtab);
  __syncthreads();
  const int tid = threadIdx.x;
  // Requests the vectors of item w (the last item again once the list is exhausted).  A slot past the end of the
  // item or of the tensor re-reads the tensor's last whole vector, and a tensor shorter than one vector reads the
  // descriptor table instead: always in bounds, never used, and so the requests carry no condition at all (a
  // conditional request would make the compiler merge old and new registers behind it, with a wait).
  auto request = [&](int w, Vec<T, P>* buf) {
    const WorkItem it = load_const(items + (w < a.n_flat ? w : a.n_flat - 1));
    const TensorDesc d = load_const(descs + it.tensor);
    const int64_t n = d.rows * d.cols;
    const int64_t last = n >= P ? (n - P) / P * P : 0;
    const T* th = n >= P ? reinterpret_cast<const T*>(d.theta) : reinterpret_cast<const T*>(descs);
#pragma unroll
    for (int j = 0; j < kFlatSlots; ++j) {
      int64_t e0 = (it.first + tid + 256 * j) * P;
      e0 = e0 < last ? e0 : last;
      buf[j] = load_global<Vec<T, P>>(th + e0);
    }
  };
  Vec<T, P> cur[kFlatSlots], nxt[kFlatSlots];
  request(blockIdx.x, cur);
#pragma unroll
  for (int j = 0; j < kFlatSlots; ++j) wait_here_for(cur[j]);      // nothing outstanding on entry to the loop
  for (int w = blockIdx.x; w < a.n_flat; w += nblk) {
    request(w + nblk, nxt);
    const WorkItem it = load_const(items + w);
    const TensorDesc d = load_const(descs + it.tensor);
    const int64_t n = d.rows * d.cols;
    T* __restrict__ th = reinterpret_cast<T*>(d.theta);
#pragma unroll
    for (int j = 0; j < kFlatSlots; ++j) {
      const int g = tid + 256 * j;
      if (j == kFlatSlots - 1) {
        // the next item's vectors were requested a whole item ago and the youngest store is one call old: nothing to sit out
#pragma unroll
        for (int i = 0; i < kFlatSlots; ++i) wait_here_for(nxt[i]);
      }
      if (g < it.count) {
        const int64_t q = it.first + g, e0 = q * P;
        float G[P];
        draw<P, BATCH>((uint64_t)q, d.id, a, tab, G);
        if (e0 + P <= n) {
          Vec<T, P> x = cur[j];
          float f[P];
#pragma unroll
          for (int i = 0; i < P; ++i) f[i] = __builtin_fmaf(c, G[i], to_f32(x.v[i]));
          round_into<P>(x, f);
          store_global(th + e0, x);
        } else {
          // ragged end of a tensor: element by element
          for (int i = 0; i < P; ++i)
            if (e0 + i < n) {
              T x = load_global_elem(th + e0 + i);
              from_f32(__builtin_fmaf(c, G[i], to_f32(x)), x);
              store_global_elem(th + e0 + i, x);
            }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kFlatSlots; ++j) cur[j] = nxt[j];
  }
}

// ------------------------------------------------------------------ tile
typedef float f32x16 __attribute__((ext_vector_type(16)));

// One lane's P consecutive elements starting at flat index e0: G from the seed, Z = a G + (b U R), axpy.
template <typename T, int P, bool WRITE_Z, bool BATCH>
__device__ __forceinline__ void finish_row(const TensorDesc& d, T* __restrict__ th, float* __restrict__ zout, int64_t e0, const float* ur,
                                           float c, const PerturbArgs& a, const RadiusEntry* tab) {
  float G[P];
  draw<P, BATCH>((uint64_t)e0 / P, d.id, a, tab, G);
  if (WRITE_Z) {
#pragma unroll
    for (int j = 0; j < P; ++j) zout[e0 + j] = __builtin_fmaf(d.a, G[j], ur[j]);
  } else {
    Vec<T, P> x = load_global<Vec<T, P>>(th + e0);
    float f[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const float z = __builtin_fmaf(d.a, G[j], ur[j]);
      f[j] = __builtin_fmaf(c, z, to_f32(x.v[j]));
    }
    round_into<P>(x, f);
    store_global(th + e0, x);
  }
}

// Lane layout inside a wave's 32-row slab: column group cg = lane % 32 owns P
// consecutive columns; register v of the lane is row 8*(v/4) + 4*(lane/32) + v%4.
template <typename T, int P, bool WRITE_Z, bool BATCH>
__global__ void __launch_bounds__(256) perturb_tile_kernel(PerturbArgs a, const TensorDesc* __restrict__ descs, const WorkItem* __restrict__ items,
                                                           float c, const RadiusEntry* __restrict__ gtab, float* __restrict__ zout, int kp) {
  extern __shared__ float smem[];
  RadiusEntry* tab = reinterpret_cast<RadiusEntry*>(smem);
  float* Us = smem + kRadiusTabEntries * 3;          // [128][kp]
  float* Rs = Us + kTileRowsPerIter * kp;            // [kp][TC]
  constexpr int TC = 32 * P;
  constexpr int RB = (P == 4) ? 16 : 8;              // rows a lane holds at once
  const int nblk = (int)gridDim.x - a.pull_blocks;               // computing blocks
  if ((int)blockIdx.x >= nblk) { pull_next_stage(a, (int)blockIdx.x - nblk, a.pull_blocks); return; }
  load_radius_table(tab, gtab);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cg = lane & 31, rh = lane >> 5;

  // A block takes a contiguous run of the list; the list orders the row tiles of one column strip one after the
  // other, so the slice of R in LDS is regenerated only when the strip (or the tensor) changes.
  const int per_block = (a.n_tiles + nblk - 1) / nblk;
  const int w_end = min(a.n_tiles, ((int)blockIdx.x + 1) * per_block);
  int prev_tensor = -1;
  int64_t prev_col0 = -1;
  for (int w = (int)blockIdx.x * per_block; w < w_end; ++w) {
    const WorkItem it = items[w];
    const TensorDesc d = descs[it.tensor];
    const int64_t row0 = it.first >> 32, col0 = it.first & 0xFFFFFFFFll;
    const int nrows = it.count, k = d.k, kpt = (k + 7) & ~7;
    T* __restrict__ th = reinterpret_cast<T*>(d.theta);
    const bool same_strip = it.tensor == prev_tensor && col0 == prev_col0;
    prev_tensor = it.tensor; prev_col0 = col0;
    if (!same_strip) __syncthreads();                // table loaded / previous strip's readers of Rs done
    // this strip's slice of b*R: rows l < k, columns col0 .. col0+TC
    for (int idx = tid; idx < (same_strip ? 0 : kpt * 32); idx += 256) {
      const int l = idx >> 5, g = idx & 31;
      const int64_t col = col0 + (int64_t)g * P;
      float r[P];
#pragma unroll
      for (int j = 0; j < P; ++j) r[j] = 0.f;
      if (l < k && col < d.cols) {
        const uint64_t q = (uint64_t)((int64_t)l * d.cols + col) / P;
        draw<P, BATCH>(q, d.id | 0x80000000u, a, tab, r);
#pragma unroll
        for (int j = 0; j < P; ++j) r[j] *= d.b;
      }
#pragma unroll
      for (int j = 0; j < P; ++j) Rs[l * TC + g * P + j] = r[j];
    }
    for (int r0 = 0; r0 < nrows; r0 += kTileRowsPerIter) {
      __syncthreads();                               // Rs written / previous row block's readers of Us done
      for (int idx = tid; idx < kTileRowsPerIter * kpt; idx += 256) {
        const int r = idx / kpt, l = idx - r * kpt;
        const int64_t row = row0 + r0 + r;
        Us[r * kp + l] = (l < k && r0 + r < nrows && row < d.rows) ? basis_at(d, row, l) : 0.f;
      }
      __syncthreads();
      const int64_t col = col0 + (int64_t)cg * P;
#pragma unroll 1
      for (int vb = 0; vb < 16; vb += RB) {
        float acc[RB][P];
#pragma unroll
        for (int v = 0; v < RB; ++v)
#pragma unroll
          for (int j = 0; j < P; ++j) acc[v][j] = 0.f;
        for (int l0 = 0; l0 < kpt; l0 += 8) {
          float Rreg[8][P];
#pragma unroll
          for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < P; ++j) Rreg[i][j] = Rs[(l0 + i) * TC + cg * P + j];
#pragma unroll
          for (int v = 0; v < RB; ++v) {
            const int vv = vb + v;
            const int rloc = 32 * wave + 8 * (vv >> 2) + 4 * rh + (vv & 3);
            const float* u = Us + rloc * kp + l0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const float ui = u[i];
#pragma unroll
              for (int j = 0; j < P; ++j) acc[v][j] = __builtin_fmaf(ui, Rreg[i][j], acc[v][j]);
            }
          }
        }
        if (col < d.cols) {
#pragma unroll
          for (int v = 0; v < RB; ++v) {
            const int vv = vb + v;
            const int rloc = 32 * wave + 8 * (vv >> 2) + 4 * rh + (vv & 3);
            const int64_t row = row0 + r0 + rloc;
            if (r0 + rloc < nrows && row < d.rows) finish_row<T, P, WRITE_Z, BATCH>(d, th, zout, row * d.cols + col, acc[v], c, a, tab);
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------ tile, U R on the matrix cores (k >= 16)
// fp32 MFMA 16x16x4.  A wave covers 16 rows x 32P columns per step: lane (n = lane % 16, rg = lane / 16)
// ends up with rows 4 rg + v (v = 0..3) and, in each of the two column groups g, the P consecutive columns
// g*16P + P n + j -- one Philox call per (row, group) -- so Z never leaves registers and a lane needs only
// 2P x 4 accumulators.  The contraction index is l = rg * (kpt/4) + s: a lane reads kpt/4 consecutive floats
// of its row of U from global memory and one row of the R slice from LDS per step.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kTilePasses = 3;      // runs of the tile list per block of the matrix-core kernel

template <typename T, int P, bool WRITE_Z, bool BATCH, bool FULL>
__device__ __forceinline__ void mfma_row_block(const TensorDesc& d, const PerturbArgs& a, float c, const RadiusEntry* tab, const float* Rs,
                                               T* __restrict__ th, float* __restrict__ zout, int64_t row0, int64_t col0, int r0, int nrows,
                                               int k, int kq4, int wave, int n16, int rg) {
  constexpr int TC = 32 * P, GC = 16 * P;                     // tile columns, columns per group
  const int mrow = r0 + 16 * wave + n16;                      // A operand: this lane feeds row (lane % 16) of the slab
  const bool uvalid = FULL || (mrow < nrows && row0 + mrow < d.rows);
  const int64_t urow = row0 + mrow;
  const int ucol = rg * kq4;
  const int rbase = r0 + 16 * wave + 4 * rg;                  // first of this lane's 4 rows (tile-relative)
  const int64_t ebase = (row0 + rbase) * d.cols + col0 + (int64_t)P * n16;
  f32x4 acc[2 * P];
#pragma unroll
  for (int j = 0; j < 2 * P; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < kq4; s0 += 2) {
    float ua[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) ua[i] = (uvalid && ucol + s0 + i < k) ? basis_at(d, urow, ucol + s0 + i) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float* rrow = Rs + (rg * kq4 + s0 + i) * TC + P * n16;
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int j = 0; j < P; ++j)
          acc[g * P + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ua[i], rrow[g * GC + j], acc[g * P + j], 0, 0, 0);
    }
  }
  if (FULL && !WRITE_Z) {
    // Whole tile: the lane's eight vectors of theta are requested one generator call ahead.  The wait before a
    // vector is used is a full one (loads and stores share one counter, and with both kinds in flight it cannot
    // be a partial wait), so whatever was requested last sets its length: with the request a whole call old it
    // has landed, with the request placed a third of a call earlier, as the scheduler does by itself, it has not.
    Vec<T, P> xn = load_global<Vec<T, P>>(th + ebase);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int v = t >> 1, g = t & 1;
      const int64_t e0 = ebase + (int64_t)v * d.cols + g * GC;
      const Vec<T, P> xc = xn;
      if (t + 1 < 8) {
        xn = load_global<Vec<T, P>>(th + ebase + (int64_t)((t + 1) >> 1) * d.cols + ((t + 1) & 1) * GC);
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_barrier(0);
#endif
      }
      float G[P];
      draw<P, BATCH>((uint64_t)e0 / P, d.id, a, tab, G);
      Vec<T, P> xv = xc;
      float f[P];
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const float z = __builtin_fmaf(d.a, G[j], acc[g * P + j][v]);
        f[j] = __builtin_fmaf(c, z, to_f32(xv.v[j]));
      }
      round_into<P>(xv, f);
      store_global(th + e0, xv);
    }
    return;
  }
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int g = 0; g < 2; ++g)
      if (FULL || (rbase + v < nrows && row0 + rbase + v < d.rows && col0 + g * GC + P * n16 < d.cols)) {
        const int64_t e0 = ebase + (int64_t)v * d.cols + g * GC;
        Vec<T, P> xv;
        if (!WRITE_Z) xv = load_global<Vec<T, P>>(th + e0);
        float G[P];
        draw<P, BATCH>((uint64_t)e0 / P, d.id, a, tab, G);
        if (WRITE_Z) {
#pragma unroll
          for (int j = 0; j < P; ++j) zout[e0 + j] = __builtin_fmaf(d.a, G[j], acc[g * P + j][v]);
        } else {
          float f[P];
#pragma unroll
          for (int j = 0; j < P; ++j) {
            const float z = __builtin_fmaf(d.a, G[j], acc[g * P + j][v]);
            f[j] = __builtin_fmaf(c, z, to_f32(xv.v[j]));
          }
          round_into<P>(xv, f);
          store_global(th + e0, xv);
        }
      }
}

template <typename T, int P, bool WRITE_Z, bool BATCH>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8))) perturb_tile_mfma_kernel(PerturbArgs a, const TensorDesc* __restrict__ descs, const WorkItem* __restrict__ items,
                                                                float c, const RadiusEntry* __restrict__ gtab, float* __restrict__ zout, int kp) {
  extern __shared__ float smem[];
  RadiusEntry* tab = reinterpret_cast<RadiusEntry*>(smem);
  float* Rs = smem + kRadiusTabEntries * 3;          // [kp][TC]
  constexpr int TC = 32 * P;
  const int nblk = (int)gridDim.x - a.pull_blocks;               // computing blocks
  if ((int)blockIdx.x >= nblk) { pull_next_stage(a, (int)blockIdx.x - nblk, a.pull_blocks); return; }
  load_radius_table(tab, gtab);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, rg = lane >> 4;
  // Every block takes kTilePasses contiguous runs of the list; the R slice is regenerated only when the column strip
  // changes (see above).  Consecutive block ids go round-robin to the 8 XCDs, so the list is cut into 8 chunks, one
  // per XCD, and in pass i the blocks q = 0, 1, ... of an XCD take the neighbouring runs i n + q of its chunk: at any
  // time the blocks of one XCD work on neighbouring column strips of the same few matrices, walk the same rows and
  // find each other's rows of U in their common L2, and a block's next run lies in other matrices.
  const bool by_xcd = (nblk & 7) == 0;
  // (a run shorter than a strip of a 2048-row matrix, 16 tiles, would only regenerate R slices more often: short
  // launches, e.g. one pipeline stage of streamed bases, take fewer runs per block)
  const int by_len = a.n_tiles / (nblk * 16);
  const int n_pass = !by_xcd || by_len < 1 ? 1 : (by_len < kTilePasses ? by_len : kTilePasses);
  const int per_xcd = nblk >> 3;
  const int64_t n_runs = (int64_t)nblk * n_pass;          // run r is tiles [r n / R, (r + 1) n / R): lengths differ by at most one
  int prev_tensor = -1;
  int64_t prev_col0 = -1;
  for (int pass = 0; pass < n_pass; ++pass) {
    const int run = by_xcd ? (((int)blockIdx.x & 7) * n_pass + pass) * per_xcd + ((int)blockIdx.x >> 3) : (int)blockIdx.x;
    const int w_end = (int)(((int64_t)run + 1) * a.n_tiles / n_runs);
    for (int w = (int)((int64_t)run * a.n_tiles / n_runs); w < w_end; ++w) {
      const WorkItem it = items[w];
      const TensorDesc d = descs[it.tensor];
      const int64_t row0 = it.first >> 32, col0 = it.first & 0xFFFFFFFFll;
      const int nrows = it.count, k = d.k, kpt = (k + 7) & ~7, kq4 = kpt >> 2;
      T* __restrict__ th = reinterpret_cast<T*>(d.theta);
      const bool same_strip = it.tensor == prev_tensor && col0 == prev_col0;
      prev_tensor = it.tensor; prev_col0 = col0;
      if (!same_strip) __syncthreads();                // table loaded / previous strip's readers of Rs done
      for (int idx = tid; idx < (same_strip ? 0 : kpt * 32); idx += 256) {
        const int l = idx >> 5, g = idx & 31;
        const int64_t col = col0 + (int64_t)g * P;
        float r[P];
#pragma unroll
        for (int j = 0; j < P; ++j) r[j] = 0.f;
        if (l < k && col < d.cols) {
          draw<P, BATCH>((uint64_t)((int64_t)l * d.cols + col) / P, d.id | 0x80000000u, a, tab, r);
#pragma unroll
          for (int j = 0; j < P; ++j) r[j] *= d.b;
        }
#pragma unroll
        for (int j = 0; j < P; ++j) Rs[l * TC + g * P + j] = r[j];
      }
      if (!same_strip) __syncthreads();
      const bool full = (nrows % 64 == 0) && row0 + nrows <= d.rows && col0 + TC <= d.cols && k == kpt;
      for (int r0 = 0; r0 < nrows; r0 += 64) {
        if (full) mfma_row_block<T, P, WRITE_Z, BATCH, true>(d, a, c, tab, Rs, th, zout, row0, col0, r0, nrows, k, kq4, wave, n16, rg);
        else      mfma_row_block<T, P, WRITE_Z, BATCH, false>(d, a, c, tab, Rs, th, zout, row0, col0, r0, nrows, k, kq4, wave, n16, rg);
      }
    }
  }
}

// ------------------------------------------------------------------ affine quantiser of a basis (cloud side of Sec. 3.4)
// min / max as order-preserving integers, so that integer atomics reduce them
__device__ __forceinline__ int32_t float_order(float x) { const int32_t b = __float_as_int(x); return b >= 0 ? b : (int32_t)(0x80000000u - (uint32_t)b); }
__device__ __forceinline__ float order_float(int32_t o) { return __int_as_float(o >= 0 ? o : (int32_t)(0x80000000u - (uint32_t)o)); }

__global__ void basis_minmax_init_kernel(int32_t* mm) { mm[0] = 0x7FFFFFFF; mm[1] = (int32_t)0x80000000; }
__global__ void __launch_bounds__(256) basis_minmax_kernel(const float* __restrict__ U, int64_t rows, int k, int ldu, int32_t* __restrict__ mm) {
  int32_t lo = 0x7FFFFFFF, hi = (int32_t)0x80000000;
  const int64_t n = rows * k;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int32_t o = float_order(U[(i / k) * ldu + (i % k)]);
    lo = o < lo ? o : lo; hi = o > hi ? o : hi;
  }
  for (int off = 32; off > 0; off >>= 1) {
    const int32_t l2 = __shfl_xor(lo, off, 64), h2 = __shfl_xor(hi, off, 64);
    lo = l2 < lo ? l2 : lo; hi = h2 > hi ? h2 : hi;
  }
  if ((threadIdx.x & 63) == 0) { atomicMin(mm, lo); atomicMax(mm + 1, hi); }
}
__global__ void basis_minmax_finish_kernel(int32_t* mm) {
  float* f = reinterpret_cast<float*>(mm);
  const float lo = order_float(mm[0]), hi = order_float(mm[1]);
  f[0] = lo; f[1] = hi;
}
// one thread per output byte: codes of elements 2j and 2j + 1 of a row, round(x / lambda + delta) clipped to [0, 15]
__global__ void __launch_bounds__(256) basis_quantize_kernel(const float* __restrict__ U, int64_t rows, int k, int ldu, float lambda, float delta,
                                                             uint8_t* __restrict__ Uq, int ldq) {
#pragma clang fp contract(off)   // x / lambda is rounded before delta is added, as the definition has it
  const int kb = (k + 1) >> 1;
  const int64_t n = rows * kb;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / kb;
    const int j = (int)(i % kb);
    uint32_t byte = 0;
    for (int h = 0; h < 2; ++h) {
      const int l = 2 * j + h;
      if (l < k) {
        const float t = U[r * ldu + l] / lambda;
        float q = __builtin_rintf(t + delta);
        q = q < 0.f ? 0.f : (q > 15.f ? 15.f : q);
        byte |= (uint32_t)q << (4 * h);
      }
    }
    Uq[r * ldq + j] = (uint8_t)byte;
  }
}

// ------------------------------------------------------------------ debug kernels
__global__ void debug_philox_kernel(const uint32_t* __restrict__ ctr, uint32_t k0, uint32_t k1, uint32_t* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const u32x4 r = philox4x32_10(ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3], k0, k1);
  out[4 * i] = r.x; out[4 * i + 1] = r.y; out[4 * i + 2] = r.z; out[4 * i + 3] = r.w;
}

template <int P>
__global__ void __launch_bounds__(256) debug_gauss_kernel(uint32_t k0, uint32_t k1, uint32_t step, uint32_t id_stream, int64_t first,
                                                          int64_t n, const RadiusEntry* __restrict__ gtab, float* __restrict__ out) {
  __shared__ RadiusEntry tab[kRadiusTabEntries];
  load_radius_table(tab, gtab);
  __syncthreads();
  const int64_t q0 = first / P, q1 = (first + n + P - 1) / P;
  for (int64_t q = q0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < q1; q += (int64_t)gridDim.x * blockDim.x) {
    float G[P];
    gaussP<P>(philox_call((uint64_t)q, id_stream, step, k0, k1), tab, G);
    for (int j = 0; j < P; ++j) {
      const int64_t e = q * P + j;
      if (e >= first && e < first + n) out[e - first] = G[j];
    }
  }
}

// all radius uniforms: bits=32: N = 2n+1, n < 2^23; bits=16: N = (2h+1) << 7, h < 2^16
__global__ void __launch_bounds__(256) debug_radius_kernel(int bits, const RadiusEntry* __restrict__ gtab, float* __restrict__ out) {
  __shared__ RadiusEntry tab[kRadiusTabEntries];
  load_radius_table(tab, gtab);
  __syncthreads();
  const uint32_t total = bits == 32 ? (1u << 23) : (1u << 16);
  for (uint32_t n = blockIdx.x * blockDim.x + threadIdx.x; n < total; n += gridDim.x * blockDim.x) {
    const uint32_t N = bits == 32 ? ((n << 1) | 1u) : (((n << 1) | 1u) << 7);
    out[n] = radius_from_odd24(N, tab);
  }
}

__global__ void __launch_bounds__(256) debug_cossin_kernel(int bits, float* __restrict__ co, float* __restrict__ so) {
#pragma clang fp contract(off)
  const uint32_t total = bits == 32 ? (1u << 24) : (1u << 16);
  for (uint32_t n = blockIdx.x * blockDim.x + threadIdx.x; n < total; n += gridDim.x * blockDim.x) {
    const uint32_t m = bits == 32 ? n : (n << 8);
    const TrigHL t = trig_from_u24(m);
    // the fused kernel multiplies (hi, lo) by the radius; with radius 1 the product is the rounded sum
    const float one = __uint_as_float(0x3F800000u ^ t.sign);
    co[n] = __builtin_fmaf(one, t.ch, one * t.cl);
    so[n] = __builtin_fmaf(one, t.sh, one * t.sl);
  }
}

__global__ void __launch_bounds__(256) copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// The table lives in static device memory: the library allocates nothing.
__device__ RadiusEntry g_radius_table[kRadiusTabEntries];

}  // namespace

hipError_t ensure_radius_table(const RadiusEntry** dev_ptr, hipStream_t s) {
  static std::mutex mu;
  static const RadiusEntry* cached[64] = {};
  static RadiusEntry host[kRadiusTabEntries];
  static bool host_ready = false;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!cached[dev]) {
    if (!host_ready) {
      for (int E = 0; E < 24; ++E)
        for (int j = 0; j < 64; ++j) {
          const double cj = __builtin_rint(128.0 / (1.0 + (j + 0.5) / 64.0)) / 128.0;
          double hl = 2.0 * __builtin_log(cj) + 2.0 * (24.0 - E) * 0.69314718055994530942;
          if (E == 23 && j == 63) hl = 0.0;        // c = 1/2, N c 2^-23 -> exactly -2 log1p(z)
          RadiusEntry& r = host[E * 64 + j];
          r.H = (float)hl;
          r.L = (float)(hl - (double)r.H);
          r.C = (float)__builtin_ldexp(cj, -E);
        }
      host_ready = true;
    }
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_radius_table));
    if (e != hipSuccess) return e;
    // ordered with the caller's work: on its stream, complete before anything that follows this call is enqueued
    e = hipMemcpyAsync(p, host, sizeof(host), hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    cached[dev] = reinterpret_cast<const RadiusEntry*>(p);
  }
  *dev_ptr = cached[dev];
  return hipSuccess;
}

namespace {
// Resident blocks of 256 threads per CU for a persistent kernel: the grid is sized to what the register and
// LDS budget really admits, because a block that has to wait for a slot would start its share of the work
// list only after another block has finished all of its own.
template <typename K>
int resident_blocks_per_cu(K kern, size_t dyn_lds, int cap) {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 256, dyn_lds) != hipSuccess || nb < 1) nb = 1;
  return nb < cap ? nb : cap;
}

// Launch set-up of one tile-kernel variant: the dynamic-LDS limit (only ever raised, so that contexts with different
// ranks can take turns) and the occupancy at the LDS size asked for (the last answer is kept).
struct TileLaunchCache {
  size_t lds_limit = 0;       // what the kernel's attribute was last set to
  size_t lds = 0;
  int per_cu = 0;
};
template <typename K>
hipError_t tile_launch_setup(K kern, size_t lds, int cap, TileLaunchCache& cache, int* per_cu) {
  static std::mutex mu;                                  // the caches are shared by every context of the process
  std::lock_guard<std::mutex> lock(mu);
  if (lds > cache.lds_limit) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    cache.lds_limit = lds;
  }
  if (!(cache.per_cu > 0 && cache.lds == lds)) {
    cache.lds = lds;
    cache.per_cu = resident_blocks_per_cu(kern, lds, cap);
  }
  *per_cu = cache.per_cu;
  return hipSuccess;
}

// Grid of a persistent launch: as many computing blocks as there are items, at most the resident capacity, the
// last kPullBlocks of that capacity set aside for pulling the next stage's bases when there are any to pull.
int split_grid(PerturbArgs& a, int items, int capacity) {
  a.pull_blocks = a.n_stage > 0 ? kPullBlocks : 0;
  int compute = capacity - a.pull_blocks;
  if (compute < 1) compute = 1;
  if (compute > items) compute = items;
  return compute + a.pull_blocks;
}

template <typename T, int P>
hipError_t launch_flat_t(const PerturbArgs& a_in, float c, float* zout, hipStream_t s, int n_cu, const RadiusEntry* tab) {
  PerturbArgs a = a_in;
  if (zout) {
    const int grid = a.n_flat < n_cu * 8 ? a.n_flat : n_cu * 8;
    hipLaunchKernelGGL((fill_flat_kernel<T, P>), dim3(grid), dim3(256), 0, s, a, a.descs, a.flat, tab, zout);
    return hipGetLastError();
  }
  auto kern = a.n_q > 0 ? perturb_flat_kernel<T, P, true> : perturb_flat_kernel<T, P, false>;
  static std::atomic<int> per[2];                        // zero-initialised; racing threads compute the same value
  std::atomic<int>& slot = per[a.n_q > 0 ? 1 : 0];
  int nb = slot.load(std::memory_order_relaxed);
  if (nb == 0) { nb = resident_blocks_per_cu(kern, 0, 8); slot.store(nb, std::memory_order_relaxed); }
  const int grid = split_grid(a, a.n_flat, n_cu * nb);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, s, a, a.descs, a.flat, c, tab);
  return hipGetLastError();
}
template <typename T, int P>
hipError_t launch_tile_t(const PerturbArgs& a_in, float c, float* zout, hipStream_t s, int n_cu, const RadiusEntry* tab) {
  PerturbArgs a = a_in;
  const int kp = (a.max_k + 7) & ~7;
  const size_t lds = sizeof(float) * ((size_t)kRadiusTabEntries * 3 + (size_t)kTileRowsPerIter * kp + (size_t)kp * 32 * P);
  if (a.min_k >= kMfmaMinK) {
    const size_t lds_m = sizeof(float) * ((size_t)kRadiusTabEntries * 3 + (size_t)kp * 32 * P);
    const int variant = zout ? 1 : (a.n_q > 0 ? 2 : 0);
    auto km = zout ? perturb_tile_mfma_kernel<T, P, true, false> : (a.n_q > 0 ? perturb_tile_mfma_kernel<T, P, false, true> : perturb_tile_mfma_kernel<T, P, false, false>);
    static TileLaunchCache cache_m[3];
    int per_cu = 1;
    hipError_t e = tile_launch_setup(km, lds_m, 8, cache_m[variant], &per_cu);
    if (e != hipSuccess) return e;
    const int grid_m = split_grid(a, a.n_tiles, n_cu * per_cu);
    hipLaunchKernelGGL(km, dim3(grid_m), dim3(256), lds_m, s, a, a.descs, a.tiles, c, tab, zout, kp);
    return hipGetLastError();
  }
  const int variant = zout ? 1 : (a.n_q > 0 ? 2 : 0);
  auto kern = zout ? perturb_tile_kernel<T, P, true, false> : (a.n_q > 0 ? perturb_tile_kernel<T, P, false, true> : perturb_tile_kernel<T, P, false, false>);
  static TileLaunchCache cache_v[3];
  int per_cu = 1;
  hipError_t e = tile_launch_setup(kern, lds, 4, cache_v[variant], &per_cu);
  if (e != hipSuccess) return e;
  const int grid = split_grid(a, a.n_tiles, n_cu * per_cu);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, a, a.descs, a.tiles, c, tab, zout, kp);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_perturb_flat(const PerturbArgs& a, float c, float* zout, hipStream_t s, int n_cu) {
  if (a.n_flat <= 0) return hipSuccess;
  if (a.n_q < 0 || a.n_q > kMaxBatch || (a.n_q > 0 && zout)) return hipErrorInvalidValue;
  if (a.n_stage < 0 || a.n_stage > kMaxStage) return hipErrorInvalidValue;
  const RadiusEntry* tab = nullptr;
  hipError_t e = ensure_radius_table(&tab, s);
  if (e != hipSuccess) return e;
  if (a.dtype == 0) return a.bits == 32 ? launch_flat_t<float, 4>(a, c, zout, s, n_cu, tab) : launch_flat_t<float, 8>(a, c, zout, s, n_cu, tab);
  return a.bits == 32 ? launch_flat_t<bf16_t, 4>(a, c, zout, s, n_cu, tab) : launch_flat_t<bf16_t, 8>(a, c, zout, s, n_cu, tab);
}

hipError_t launch_perturb_tile(const PerturbArgs& a, float c, float* zout, hipStream_t s, int n_cu) {
  if (a.n_tiles <= 0) return hipSuccess;
  if (a.max_k < 1 || a.max_k > kMaxK) return hipErrorInvalidValue;
  if (a.n_q < 0 || a.n_q > kMaxBatch || (a.n_q > 0 && zout)) return hipErrorInvalidValue;
  if (a.n_stage < 0 || a.n_stage > kMaxStage) return hipErrorInvalidValue;
  if (a.n_stage < 0 || a.n_stage > kMaxStage) return hipErrorInvalidValue;
  const RadiusEntry* tab = nullptr;
  hipError_t e = ensure_radius_table(&tab, s);
  if (e != hipSuccess) return e;
  if (a.dtype == 0) return a.bits == 32 ? launch_tile_t<float, 4>(a, c, zout, s, n_cu, tab) : launch_tile_t<float, 8>(a, c, zout, s, n_cu, tab);
  return a.bits == 32 ? launch_tile_t<bf16_t, 4>(a, c, zout, s, n_cu, tab) : launch_tile_t<bf16_t, 8>(a, c, zout, s, n_cu, tab);
}

hipError_t launch_basis_minmax(const float* U, int64_t rows, int k, int ldu, float* minmax, hipStream_t s) {
  int32_t* mm = reinterpret_cast<int32_t*>(minmax);
  hipLaunchKernelGGL(basis_minmax_init_kernel, dim3(1), dim3(1), 0, s, mm);
  const int64_t n = rows * k;
  const int grid = (int)(n / 256 + 1 < 1024 ? n / 256 + 1 : 1024);
  hipLaunchKernelGGL(basis_minmax_kernel, dim3(grid), dim3(256), 0, s, U, rows, k, ldu, mm);
  hipLaunchKernelGGL(basis_minmax_finish_kernel, dim3(1), dim3(1), 0, s, mm);
  return hipGetLastError();
}

hipError_t launch_basis_quantize(const float* U, int64_t rows, int k, int ldu, float lambda, float delta, uint8_t* Uq, int ldq, hipStream_t s) {
  const int64_t n = rows * ((k + 1) / 2);
  const int grid = (int)(n / 256 + 1 < 1024 ? n / 256 + 1 : 1024);
  hipLaunchKernelGGL(basis_quantize_kernel, dim3(grid), dim3(256), 0, s, U, rows, k, ldu, lambda, delta, Uq, ldq);
  return hipGetLastError();
}

hipError_t launch_stage_only(const PerturbArgs& a, hipStream_t s) {
  if (a.n_stage <= 0) return hipSuccess;
  if (a.n_stage > kMaxStage) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stage_only_kernel, dim3(kPullBlocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_debug_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3(256 * 8), dim3(256), 0, s, reinterpret_cast<uint4*>(dst), reinterpret_cast<const uint4*>(src), bytes / 16);
  return hipGetLastError();
}

hipError_t launch_debug_philox(const uint32_t* ctr, uint32_t k0, uint32_t k1, uint32_t* out, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(debug_philox_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ctr, k0, k1, out, n);
  return hipGetLastError();
}

hipError_t launch_debug_gauss(uint32_t k0, uint32_t k1, uint32_t step, uint32_t id_stream, int bits, int64_t first, int64_t n,
                              float* out, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const RadiusEntry* tab = nullptr;
  hipError_t e = ensure_radius_table(&tab, s);
  if (e != hipSuccess) return e;
  const int P = bits == 32 ? 4 : 8;
  int64_t blocks = (n / P + 256) / 256;
  if (blocks > 4096) blocks = 4096;
  if (bits == 32) hipLaunchKernelGGL(debug_gauss_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, s, k0, k1, step, id_stream, first, n, tab, out);
  else            hipLaunchKernelGGL(debug_gauss_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, s, k0, k1, step, id_stream, first, n, tab, out);
  return hipGetLastError();
}

hipError_t launch_debug_radius_table(int bits, float* out, hipStream_t s) {
  const RadiusEntry* tab = nullptr;
  hipError_t e = ensure_radius_table(&tab, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(debug_radius_kernel, dim3(bits == 32 ? 2048 : 64), dim3(256), 0, s, bits, tab, out);
  return hipGetLastError();
}

hipError_t launch_debug_cossin_table(int bits, float* c, float* sn, hipStream_t s) {
  hipLaunchKernelGGL(debug_cossin_kernel, dim3(bits == 32 ? 4096 : 64), dim3(256), 0, s, bits, c, sn);
  return hipGetLastError();
}

}  // namespace zgr
