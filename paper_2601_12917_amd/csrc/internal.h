// Internal interfaces between the host runtime (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "rng.h"

namespace zgr {

// Device-visible description of one parameter tensor for the perturbation pass.
struct TensorDesc {
  void*        theta;
  const float* U;        // fp32 basis, or nullptr
  const uint8_t* Uq;     // 4-bit codes of the basis (two per byte, element l in byte l/2, low nibble first), or nullptr;
                         // U == nullptr && Uq == nullptr or k == 0: isotropic, Z = G
  float        qlambda, qdelta;   // U[r][l] = qlambda * (code - qdelta) when Uq is set
  int64_t      rows, cols;
  uint32_t     id;       // < 2^31
  int32_t      k, ldu;   // ldu: row stride of U in floats, of Uq in bytes
  float        a, b;     // Z = a G + b U R   (a = 1, b = 0 when isotropic)
  int32_t      dtype;    // 0 fp32, 1 bf16
};

// One unit of work of the perturbation kernels.
//  flat kernel: `first` = first Philox group of the chunk, `count` = groups in the chunk
//  tile kernel: `first` = row0 << 32 | col0, `count` = rows in the tile
struct WorkItem {
  int32_t tensor;
  int32_t count;
  int64_t first;
};

// Philox calls of a flat work item: 256 threads x as many vectors per thread as make 64 bytes per lane (what a lane
// keeps in flight while it works on the previous item): 8 for bf16 with 4 elements per call, down to 2 for fp32 with 8.
constexpr int flat_slots(int elem_bytes, int P) { return 64 / (elem_bytes * P) < 1 ? 1 : 64 / (elem_bytes * P); }
constexpr int flat_groups_per_item(int elem_bytes, int P) { return 256 * flat_slots(elem_bytes, P); }
constexpr int kTileRowsPerIter   = 128;    // rows one block covers per iteration (4 waves x 32)
constexpr int kMaxK              = 64;
constexpr int kMfmaMinK          = 16;     // from this rank on the U R contraction of a tile runs on the matrix cores
constexpr int kMaxBatch          = 8;      // perturbations summed in one pass (zgr_apply_updates)
constexpr int kMaxStage          = 16;     // tensors whose bases one launch may pull in for the next one
constexpr int kPullBlocks        = 32;     // blocks of such a launch that do the pulling

// One contiguous piece of basis data to copy from (pinned, device-visible) host memory into a staging slot.
struct StageCopy {
  const unsigned char* src;
  unsigned char*       dst;
  uint64_t             bytes;
};

struct PerturbArgs {
  const TensorDesc* descs;     // device
  const WorkItem*   flat;      // device
  const WorkItem*   tiles;     // device
  int32_t           n_flat, n_tiles;
  uint32_t          k0, k1;    // Philox key = seed
  uint32_t          step;
  int32_t           bits;      // 32 | 16
  int32_t           dtype;
  int32_t           max_k;     // largest k among tiled tensors
  int32_t           min_k;     // smallest k among tiled tensors
  // batched pass: theta += sum_i qcoef[i] Z(seed, qstep[i]); n_q == 0: the single pass theta += c Z(seed, step)
  int32_t           n_q;
  uint32_t          qstep[kMaxBatch];
  float             qcoef[kMaxBatch];
  // bases of the NEXT launch's tensors, pulled over the host link by this launch while it computes
  int32_t           n_stage;
  int32_t           pull_blocks;   // set by the launchers: the last pull_blocks blocks of the grid only copy, the others only compute
  StageCopy         stage[kMaxStage];
};

// theta += c * Z for everything in the flat / tile work list.  zout != nullptr:
// instead write Z of the single tensor in the list as fp32 [rows, cols].
hipError_t launch_perturb_flat(const PerturbArgs& a, float c, float* zout, hipStream_t s, int n_cu);
hipError_t launch_perturb_tile(const PerturbArgs& a, float c, float* zout, hipStream_t s, int n_cu);

// The radius table of the current device: filled once per process and device (thread-safe), by a copy on stream s
// that has completed when the call returns.
hipError_t ensure_radius_table(const RadiusEntry** dev_ptr, hipStream_t s);

hipError_t launch_debug_philox(const uint32_t* ctr, uint32_t k0, uint32_t k1, uint32_t* out, int64_t n, hipStream_t s);
hipError_t launch_debug_gauss(uint32_t k0, uint32_t k1, uint32_t step, uint32_t id_stream, int bits, int64_t first, int64_t n,
                              float* out, hipStream_t s);
hipError_t launch_debug_radius_table(int bits, float* out, hipStream_t s);
hipError_t launch_debug_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// only the staging copies of `a` (used when a pass has no other launch in front of its first streamed layer)
hipError_t launch_stage_only(const PerturbArgs& a, hipStream_t s);
// affine quantiser of a basis: min / max of U[rows, k] (row stride ldu) into minmax[2] (device), then the 4-bit codes
hipError_t launch_basis_minmax(const float* U, int64_t rows, int k, int ldu, float* minmax, hipStream_t s);
hipError_t launch_basis_quantize(const float* U, int64_t rows, int k, int ldu, float lambda, float delta, uint8_t* Uq, int ldq, hipStream_t s);
hipError_t launch_debug_cossin_table(int bits, float* c, float* sn, hipStream_t s);
// machine ceilings (ceilings.hip): bare in-place stream, vector-instruction issue rate
hipError_t launch_debug_rmw(void* p, size_t bytes, int dtype, float c, int mode, int blocks, void* sink, hipStream_t s);
hipError_t launch_debug_issue(int op, int ilp, int blocks, int iters, unsigned long long* out, hipStream_t s);
hipError_t launch_debug_generator(int part, int blocks, int iters, unsigned long long* out, hipStream_t s);

// cloud side (cloud.hip): tall-skinny products with the gradient snapshots, orthonormalisation, least-squares residual.
// part (optional scratch): the sum over the long dimension is split into up to kCloudMaxParts parts over more blocks and the
// parts are added in their order; kCloudMaxParts * cols * n floats for gt_q (needs ldt == n), kCloudMaxParts * rows * k for g_t.
constexpr int kCloudMaxParts = 16;
hipError_t launch_cloud_gt_q(const float* G, int64_t rows, int64_t cols, int64_t ldg, const float* Q, int n, int64_t ldq, float* T, int64_t ldt, float scale,
                             int accumulate, hipStream_t s, float* part = nullptr);
hipError_t launch_cloud_g_t(const float* G, int64_t rows, int64_t cols, const float* T, int k, float* Y, int accumulate, hipStream_t s, float* part = nullptr);
hipError_t launch_cloud_orth(float* Y, int64_t rows, int k, int* dependent, hipStream_t s);
hipError_t launch_cloud_copy_basis(const float* Q, int64_t rows, int k, float* U, int ldu, hipStream_t s);
hipError_t launch_cloud_residual(float* R, const float* Y, int64_t n, hipStream_t s);

}  // namespace zgr
