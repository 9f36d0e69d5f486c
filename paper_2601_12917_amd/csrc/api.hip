// Host runtime and C ABI of the ZGR step: tensor table, Philox work lists,
// workspace carving, launch sequencing on the caller's stream, HIP-event
// profiling.  Follows Algorithm 1 (client block: zgr_step; edge-server block:
// zgr_apply_update) with the estimator of Eq. (11).
#include "../../include/zgr.h"
#include "backward.h"
#include "forward.h"
#include "internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

using namespace zgr;

// Scratch of zgr_lsq_loss_static: the predictions X W^T (fp32, up to kStaticPredFloats of them) followed by the
// per-example losses (up to kStaticMaxBatch).  One copy per device, held until the process ends.  Host code never
// uses this name as an address: it asks the runtime for the device address (scratch_of_current_device below).
constexpr size_t kStaticPredFloats = (size_t)1 << 18;     // 1 MiB of predictions
constexpr size_t kStaticMaxBatch   = 4096;
constexpr size_t kStaticScratchBytes = (kStaticPredFloats + kStaticMaxBatch) * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

std::string g_init_error;   // message of the last failed zgr_init / context-free call

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

constexpr size_t kMinStageTiles = 8192;   // tiles that make a tile launch long enough to amortise its start-up and tail
constexpr int kSpcSlots = 2;   // layers' worth of streamed bases resident at once: the one in use and the one arriving

struct Layer {
  int ln1_g = -1, ln1_b = -1, wq = -1, bq = -1, wk = -1, bk = -1, wv = -1, bv = -1, wo = -1, bo = -1;
  int ln2_g = -1, ln2_b = -1, w1 = -1, b1 = -1, w2 = -1, b2 = -1;
};

struct Carve {                 // workspace layout (byte offsets)
  size_t descs = 0, flat = 0, tiles = 0, dbg = 0;
  size_t cap_flat = 0, cap_tiles = 0, cap_dbg = 0;   // capacities in items
  size_t x = 0, h = 0, qkv = 0, ctx = 0, ff = 0, logits = 0, row_loss = 0, targets = 0, loss = 0;
  size_t row_loss_stride = 0;                  // floats between the row losses of L+ (slot 0) and L- (slot 1)
  size_t spc[kSpcSlots] = {}, spc_bytes = 0;   // staging slots for the bases of one layer each (streamed bases)
  size_t total = 0;
};

struct Prof {
  bool on = false, paused = false;
  std::vector<hipEvent_t> ev;          // pairs
  std::vector<int> cls;
  size_t used = 0;                     // pairs in flight
  double ms[ZGR_K_COUNT] = {};
  int64_t n[ZGR_K_COUNT] = {};
};

}  // namespace

struct zgr_ctx {
  zgr_model model{};
  zgr_config cfg{};
  std::vector<zgr_tensor> t;
  struct QBasis { const uint8_t* q = nullptr; float lambda = 0.f, delta = 0.f; };
  std::vector<QBasis> qb;      // per tensor: 4-bit basis (then t[i].U is NULL, t[i].k its rank, t[i].ldu its row stride in bytes)
  // Bases that stay in HOST memory and are streamed layer by layer during a pass (t[i].U NULL, t[i].k the rank)
  struct HostBasis { const void* host = nullptr; const unsigned char* dev = nullptr; int bits = 0; float lambda = 0.f, delta = 0.f; size_t slot_off = 0; };
  std::vector<HostBasis> hb;
  // A run of the tile list served by one kernel: class 0 = ranks >= kMfmaMinK (matrix-core kernel), class 1 = smaller
  // ranks (vector kernel).  A context may mix both; each class gets its own launch.
  struct TileRange { size_t begin = 0, end = 0; int max_k = 0, min_k = kMaxK + 1; };
  struct Group { int layer = 0; std::vector<int> tensors; TileRange cls[2];
                 std::vector<StageCopy> copies; };   // host -> staging-slot pieces, contiguous runs merged
  std::vector<Group> groups;   // streamed groups in pass order; their tiles follow the resident ones in `tiles`
  TileRange res[2];            // tiles of the resident guided tensors, by class
  size_t min_stage_tiles = kMinStageTiles;   // consecutive layers share a stage until it holds this many tiles
  std::vector<TensorDesc> descs;
  std::vector<WorkItem> flat, tiles;
  bool lists_dirty = true;
  int max_k = 0, min_k = 0;
  int dtype = 0;
  std::vector<Layer> layers;
  int tok_emb = -1, pos_emb = -1, lnf_g = -1, lnf_b = -1, cls_w = -1, cls_b = -1, lsq_w = -1;
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  Carve cv;
  int max_batch = 0, max_seq = 0;
  hipStream_t stream = nullptr;
  int n_cu = 256;
  std::string err;
  Prof prof;
  int64_t last_rows = 0;       // rows of the last forward's row_loss
  int last_slot = 0;           // which of the two row-loss buffers the last forward wrote
  int64_t slot_rows[2] = {0, 0};
  double host_loss[2] = {0, 0};
};

namespace {

zgr_status fail(zgr_ctx* c, zgr_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_init_error = buf;
  return st;
}

#define HIP_TRY(ctx, expr)                                                                      \
  do {                                                                                          \
    hipError_t e__ = (expr);                                                                    \
    if (e__ != hipSuccess) return fail(ctx, ZGR_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

size_t elem_size(int dtype) { return dtype == ZGR_F32 ? 4 : 2; }

// (a, b) of Z = a G + b U R for one tensor; isotropic tensors get (1, 0).
void mix_coefficients(const zgr_config& cfg, const zgr_tensor& t, bool guided, float* a, float* b) {
  if (!guided) { *a = 1.f; *b = 0.f; return; }
  const double al = cfg.alpha, rows = (double)t.rows, cols = (double)t.cols, k = (double)t.k;
  if (cfg.scale_mode == ZGR_SCALE_UNIT) { *a = (float)std::sqrt(al); *b = (float)std::sqrt((1.0 - al) * rows / k); }
  else { *a = (float)std::sqrt(al / (rows * cols)); *b = (float)std::sqrt((1.0 - al) / (k * cols)); }
}

int group_size(int bits) { return bits == 32 ? 4 : 8; }

size_t flat_items_of(int64_t numel, int P, int dtype) {
  const int64_t groups = (numel + P - 1) / P, per = flat_groups_per_item((int)elem_size(dtype), P);
  return (size_t)((groups + per - 1) / per);
}
// Row tiles of 128 rows: fine enough that a launch over one layer's matrices (a stage of the layer pipeline) still
// gives every block several tiles; the slice of R is shared by the consecutive row tiles of a strip, so small tiles cost nothing.
int tile_rows_of(int64_t) { return kTileRowsPerIter; }
size_t tile_items_of(int64_t rows, int64_t cols, int P) {
  const int64_t tr = tile_rows_of(rows), tc = 32 * P;
  return (size_t)(((rows + tr - 1) / tr) * ((cols + tc - 1) / tc));
}

void append_items(const zgr_tensor& t, int index, bool guided, int P, std::vector<WorkItem>& flat, std::vector<WorkItem>& tiles) {
  if (!guided) {
    const int64_t groups = (t.rows * t.cols + P - 1) / P, per = flat_groups_per_item((int)elem_size(t.dtype), P);
    for (int64_t g0 = 0; g0 < groups; g0 += per)
      flat.push_back({index, (int32_t)std::min<int64_t>(per, groups - g0), g0});
  } else {
    const int64_t tr = tile_rows_of(t.rows), tc = 32 * P;
    // column strips outermost: the kernels keep a strip's slice of R in LDS across its consecutive row tiles
    for (int64_t c0 = 0; c0 < t.cols; c0 += tc)
      for (int64_t r0 = 0; r0 < t.rows; r0 += tr)
        tiles.push_back({index, (int32_t)std::min<int64_t>(tr, t.rows - r0), (r0 << 32) | c0});
  }
}

bool is_guided(const zgr_ctx* c, size_t i) {
  return (c->t[i].U != nullptr || (i < c->qb.size() && c->qb[i].q != nullptr) || (i < c->hb.size() && c->hb[i].host != nullptr)) && c->t[i].k > 0;
}
bool is_streamed(const zgr_ctx* c, size_t i) { return i < c->hb.size() && c->hb[i].host != nullptr && c->t[i].k > 0; }

// Host work lists + descriptors from the tensor table.
void build_lists(zgr_ctx* c) {
  const int P = group_size(c->cfg.gauss_bits);
  c->flat.clear(); c->tiles.clear(); c->descs.resize(c->t.size()); c->groups.clear();
  c->max_k = 0; c->min_k = kMaxK + 1;
  // Streamed tensors: layers in order of first appearance; consecutive layers are packed into one stage until the
  // stage holds min_stage_tiles tiles, as long as its bases fit a staging slot and its pieces one launch's list.
  struct LayerSet { int layer; std::vector<int> tensors; size_t bytes = 0, tiles = 0, pieces = 0; };
  std::vector<LayerSet> layers;
  for (size_t i = 0; i < c->t.size(); ++i) {
    if (!is_streamed(c, i)) continue;
    LayerSet* ls = nullptr;
    for (auto& l : layers) if (l.layer == c->t[i].layer) ls = &l;
    if (!ls) { layers.push_back({}); ls = &layers.back(); ls->layer = c->t[i].layer; }
    const size_t bytes = (size_t)c->t[i].rows * (c->hb[i].bits == 4 ? (size_t)(c->t[i].k + 1) / 2 : (size_t)c->t[i].k * 4);
    // a tensor continues the previous piece when it lies in host memory where the padded slot layout puts it
    bool continues = false;
    if (!ls->tensors.empty()) {
      const int pv = ls->tensors.back();
      const size_t pbytes = (size_t)c->t[pv].rows * (c->hb[pv].bits == 4 ? (size_t)(c->t[pv].k + 1) / 2 : (size_t)c->t[pv].k * 4);
      continues = c->hb[i].dev == c->hb[pv].dev + align_up(pbytes);
    }
    ls->tensors.push_back((int)i);
    ls->bytes += align_up(bytes);
    ls->tiles += tile_items_of(c->t[i].rows, c->t[i].cols, P);
    if (!continues) ls->pieces += 1;
  }
  {
    size_t bytes = 0, tiles = 0, pieces = 0;
    for (const LayerSet& l : layers) {
      const bool open = !c->groups.empty() && tiles > 0;
      if (!open || tiles >= c->min_stage_tiles || bytes + l.bytes > c->cv.spc_bytes || pieces + l.pieces > (size_t)kMaxStage) {
        c->groups.push_back({}); c->groups.back().layer = l.layer;
        bytes = tiles = pieces = 0;
      }
      for (int i : l.tensors) c->groups.back().tensors.push_back(i);
      bytes += l.bytes; tiles += l.tiles; pieces += l.pieces;
    }
  }
  for (size_t gi = 0; gi < c->groups.size(); ++gi) {
    size_t off = 0;
    for (int i : c->groups[gi].tensors) {
      c->hb[i].slot_off = off;
      const size_t row_bytes = c->hb[i].bits == 4 ? (size_t)(c->t[i].k + 1) / 2 : (size_t)c->t[i].k * 4;
      off += align_up((size_t)c->t[i].rows * row_bytes);
    }
  }
  for (size_t gi = 0; gi < c->groups.size(); ++gi) {
    // bases that lie in host memory as they lie in the slot (same order, same 256-byte padding) form one piece
    std::vector<StageCopy>& cp = c->groups[gi].copies;
    cp.clear();
    for (int i : c->groups[gi].tensors) {
      const size_t bytes = (size_t)c->t[i].rows * (c->hb[i].bits == 4 ? (size_t)(c->t[i].k + 1) / 2 : (size_t)c->t[i].k * 4);
      unsigned char* dst = c->ws + c->cv.spc[gi % kSpcSlots] + c->hb[i].slot_off;
      const unsigned char* src = c->hb[i].dev;
      if (!cp.empty() && dst - cp.back().dst == src - cp.back().src && (size_t)(dst - cp.back().dst) == align_up((size_t)cp.back().bytes))
        cp.back().bytes = (uint64_t)(dst - cp.back().dst) + bytes;     // the padding in between is copied along
      else
        cp.push_back(StageCopy{src, dst, (uint64_t)bytes});
    }
  }
  auto describe = [&](size_t i, int group_index) {
    const zgr_tensor& t = c->t[i];
    TensorDesc& d = c->descs[i];
    const bool guided = is_guided(c, i);
    const bool streamed = is_streamed(c, i);
    const bool q4 = guided && !streamed && t.U == nullptr;
    d.theta = t.theta; d.U = guided ? t.U : nullptr; d.rows = t.rows; d.cols = t.cols; d.id = t.tensor_id;
    d.Uq = q4 ? c->qb[i].q : nullptr; d.qlambda = q4 ? c->qb[i].lambda : 0.f; d.qdelta = q4 ? c->qb[i].delta : 0.f;
    d.k = guided ? t.k : 0; d.ldu = t.ldu; d.dtype = t.dtype;
    if (streamed) {
      // the basis of a streamed tensor is read from the staging slot its group rotates into, compact rows
      unsigned char* slot = c->ws + c->cv.spc[group_index % kSpcSlots] + c->hb[i].slot_off;
      if (c->hb[i].bits == 4) { d.U = nullptr; d.Uq = slot; d.qlambda = c->hb[i].lambda; d.qdelta = c->hb[i].delta; d.ldu = (t.k + 1) / 2; }
      else { d.U = reinterpret_cast<const float*>(slot); d.Uq = nullptr; d.ldu = t.k; }
    }
    mix_coefficients(c->cfg, t, guided, &d.a, &d.b);
    if (guided && t.k > c->max_k) c->max_k = t.k;
    if (guided && t.k < c->min_k) c->min_k = t.k;
  };
  // the tiles of a set of tensors, matrix-core class first, then the vector class
  auto tile_ranges = [&](const std::vector<int>& members, zgr_ctx::TileRange* cls) {
    for (int k_class = 0; k_class < 2; ++k_class) {
      cls[k_class] = zgr_ctx::TileRange{};
      cls[k_class].begin = c->tiles.size();
      for (int i : members) {
        if (!is_guided(c, (size_t)i) || (c->t[i].k >= kMfmaMinK ? 0 : 1) != k_class) continue;
        append_items(c->t[i], i, true, P, c->flat, c->tiles);
        cls[k_class].max_k = std::max(cls[k_class].max_k, c->t[i].k);
        cls[k_class].min_k = std::min(cls[k_class].min_k, c->t[i].k);
      }
      cls[k_class].end = c->tiles.size();
    }
  };
  std::vector<int> resident;
  for (size_t i = 0; i < c->t.size(); ++i) {
    if (is_streamed(c, i)) continue;
    describe(i, 0);
    if (is_guided(c, i)) resident.push_back((int)i);
    else append_items(c->t[i], (int)i, false, P, c->flat, c->tiles);
  }
  tile_ranges(resident, c->res);
  for (size_t gi = 0; gi < c->groups.size(); ++gi) {
    zgr_ctx::Group& g = c->groups[gi];
    for (int i : g.tensors) describe((size_t)i, (int)gi);
    tile_ranges(g.tensors, g.cls);
  }
  c->lists_dirty = true;
}

zgr_status check_tensor(zgr_ctx* c, const zgr_tensor& t, int i, int bits, bool need_ptrs) {
  if (need_ptrs && !t.theta) return fail(c, ZGR_ERR_NULL, "tensor %d: theta is NULL", i);
  if (t.rows < 1 || t.cols < 1 || t.rows > (int64_t)1 << 31 || t.cols > (int64_t)1 << 31) return fail(c, ZGR_ERR_SHAPE, "tensor %d: bad shape %lld x %lld", i, (long long)t.rows, (long long)t.cols);
  if (t.dtype != ZGR_F32 && t.dtype != ZGR_BF16) return fail(c, ZGR_ERR_DTYPE, "tensor %d: unknown dtype %d", i, t.dtype);
  if (t.tensor_id >= 0x80000000u) return fail(c, ZGR_ERR_CONFIG, "tensor %d: tensor_id must be < 2^31", i);
  if (need_ptrs && ((uintptr_t)t.theta & 15)) return fail(c, ZGR_ERR_SHAPE, "tensor %d: theta must be 16-byte aligned", i);
  if (t.k < 0) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k < 0", i);
  if ((t.U || !need_ptrs) && t.k > 0) {
    if (t.k > kMaxK) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds %d", i, t.k, kMaxK);
    if (t.k > t.rows) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds rows = %lld", i, t.k, (long long)t.rows);
    if (t.ldu < t.k) return fail(c, ZGR_ERR_SHAPE, "tensor %d: ldu = %d < k = %d", i, t.ldu, t.k);
    if (t.cols % group_size(bits)) return fail(c, ZGR_ERR_SHAPE, "tensor %d: a guided tensor needs cols %% %d == 0", i, group_size(bits));
  }
  return ZGR_OK;
}

zgr_status check_config(zgr_ctx* c, const zgr_config& cfg) {
  if (!(cfg.eps > 0.f) || !std::isfinite(cfg.eps)) return fail(c, ZGR_ERR_CONFIG, "eps must be positive and finite");
  if (!(cfg.alpha >= 0.f && cfg.alpha <= 1.f)) return fail(c, ZGR_ERR_CONFIG, "alpha must lie in [0, 1]");
  if (cfg.scale_mode != ZGR_SCALE_UNIT && cfg.scale_mode != ZGR_SCALE_PAPER) return fail(c, ZGR_ERR_CONFIG, "unknown scale_mode");
  if (cfg.gauss_bits != 32 && cfg.gauss_bits != 16) return fail(c, ZGR_ERR_CONFIG, "gauss_bits must be 32 or 16");
  if (cfg.fuse_restore_update != 0 && cfg.fuse_restore_update != 1) return fail(c, ZGR_ERR_CONFIG, "fuse_restore_update must be 0 or 1");
  if (cfg.fuse_restore_update && !std::isfinite(cfg.lr)) return fail(c, ZGR_ERR_CONFIG, "lr must be finite");
  return ZGR_OK;
}

bool is_transformer(int arch) { return arch == ZGR_ARCH_DECODER_LM || arch == ZGR_ARCH_ENCODER_CLS; }

zgr_status check_model(zgr_ctx* c, const zgr_model& m, int dtype) {
  if (m.arch != ZGR_ARCH_NONE && m.arch != ZGR_ARCH_LINEAR_LSQ && !is_transformer(m.arch)) return fail(c, ZGR_ERR_CONFIG, "unknown arch %d", m.arch);
  if (m.arch == ZGR_ARCH_LINEAR_LSQ && dtype != ZGR_F32) return fail(c, ZGR_ERR_DTYPE, "the least-squares model is fp32 only");
  if (!is_transformer(m.arch)) return ZGR_OK;
  if (m.n_layer < 1 || m.d_model < 1 || m.n_head < 1 || m.d_ff < 1 || m.vocab < 2 || m.max_pos < 1) return fail(c, ZGR_ERR_SHAPE, "bad transformer dimensions");
  if (m.d_model % m.n_head || !attention_head_dim_supported(m.d_model / m.n_head)) return fail(c, ZGR_ERR_SHAPE, "head size must be 8, 16, 32 or 64");
  if (dtype == ZGR_BF16 && (m.d_model % 64 || m.d_ff % 64)) return fail(c, ZGR_ERR_SHAPE, "bf16 storage needs d_model and d_ff to be multiples of 64");
  if (m.arch == ZGR_ARCH_ENCODER_CLS && m.n_class < 2) return fail(c, ZGR_ERR_SHAPE, "n_class must be >= 2");
  if (!(m.ln_eps > 0.f)) return fail(c, ZGR_ERR_CONFIG, "ln_eps must be positive");
  if (m.act != ZGR_ACT_GELU && m.act != ZGR_ACT_RELU) return fail(c, ZGR_ERR_CONFIG, "unknown activation %d", m.act);
  if (m.post_ln != 0 && m.post_ln != 1) return fail(c, ZGR_ERR_CONFIG, "post_ln must be 0 or 1");
  return ZGR_OK;
}

Carve carve(const zgr_model& m, const zgr_tensor* t, int n_t, int max_batch, int max_seq, int bits) {
  Carve cv;
  const int P = group_size(bits);
  size_t nf = 0, nt = 0, nd = 0;
  int dtype = n_t > 0 ? t[0].dtype : 0;
  for (int i = 0; i < n_t; ++i) {
    const size_t f = flat_items_of(t[i].rows * t[i].cols, P, t[i].dtype);
    const size_t tl = (t[i].cols % P == 0) ? tile_items_of(t[i].rows, t[i].cols, P) : 0;
    nf += f; nt += tl;
    nd = std::max(nd, std::max(f, tl));
  }
  cv.cap_flat = nf; cv.cap_tiles = nt; cv.cap_dbg = nd;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
  cv.descs = take(sizeof(TensorDesc) * (size_t)std::max(n_t, 1));
  cv.flat = take(sizeof(WorkItem) * std::max<size_t>(nf, 1));
  cv.tiles = take(sizeof(WorkItem) * std::max<size_t>(nt, 1));
  cv.dbg = take(sizeof(WorkItem) * std::max<size_t>(nd, 1));
  cv.loss = take(sizeof(double) * 2);
  {
    // A staging slot holds the fp32 bases (compact rows x k, ranks from the tensor table) of one stage: consecutive
    // layers packed until they hold kMinStageTiles tiles.  Sized as if every guidable tensor were streamed.
    struct PL { int layer; size_t bytes, tiles; };
    std::vector<PL> per_layer;
    for (int i = 0; i < n_t; ++i) {
      if (t[i].k <= 0 || t[i].cols % P) continue;
      const size_t bytes = align_up((size_t)t[i].rows * (size_t)t[i].k * 4);
      const size_t tl = tile_items_of(t[i].rows, t[i].cols, P);
      bool found = false;
      for (auto& pl : per_layer) if (pl.layer == t[i].layer) { pl.bytes += bytes; pl.tiles += tl; found = true; }
      if (!found) per_layer.push_back({t[i].layer, bytes, tl});
    }
    size_t bytes = 0, tiles = 0;
    for (const auto& pl : per_layer) {
      if (tiles >= kMinStageTiles) { bytes = 0; tiles = 0; }
      bytes += pl.bytes; tiles += pl.tiles;
      cv.spc_bytes = std::max(cv.spc_bytes, bytes);
    }
    for (int i = 0; i < kSpcSlots; ++i) cv.spc[i] = take(cv.spc_bytes);
  }
  const size_t es = elem_size(dtype);
  if (is_transformer(m.arch)) {
    const size_t M = (size_t)max_batch * max_seq, d = m.d_model;
    cv.x = take(M * d * 4);
    cv.h = take(M * d * es);
    cv.qkv = take(M * 3 * d * es);
    cv.ctx = take(M * d * es);
    cv.ff = take(M * (size_t)m.d_ff * es);
    // fp32 storage: full fp32 logits; bf16: only the softmax partials (float2 per 128-row strip of the vocabulary
    // and token) and the target logits of the fused cross-entropy
    const size_t lm_logits = dtype == ZGR_BF16 ? M * ((size_t)2 * ce_partials_per_row(m.vocab) + 1) * 4 : M * (size_t)m.vocab * 4;
    cv.logits = take(m.arch == ZGR_ARCH_DECODER_LM ? lm_logits : (size_t)max_batch * m.n_class * 4);
    cv.row_loss_stride = align_up(M * 4) / 4;
    cv.row_loss = take(2 * cv.row_loss_stride * 4);
    cv.targets = take(M * 4);
  } else if (m.arch == ZGR_ARCH_LINEAR_LSQ) {
    size_t out = 0;
    for (int i = 0; i < n_t; ++i) if (t[i].role == ZGR_ROLE_LSQ_W) out = (size_t)t[i].rows;
    cv.logits = take((size_t)max_batch * out * 4);
    cv.row_loss_stride = align_up((size_t)max_batch * 4) / 4;
    cv.row_loss = take(2 * cv.row_loss_stride * 4);
  }
  cv.total = off;
  return cv;
}

// ---------------------------------------------------------------- profiling
void prof_harvest(zgr_ctx* c) {
  Prof& p = c->prof;
  for (size_t i = 0; i < p.used; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]) == hipSuccess) { p.ms[p.cls[i]] += ms; p.n[p.cls[i]] += 1; }
  }
  p.used = 0;
}

struct ProfScope {
  zgr_ctx* c; bool live = false; size_t slot = 0;
  ProfScope(zgr_ctx* ctx, int cls) : c(ctx) {
    Prof& p = c->prof;
    if (!p.on || p.paused) return;
    if ((p.used + 1) * 2 > p.ev.size()) {
      if (p.ev.size() >= 16384) { (void)hipStreamSynchronize(c->stream); prof_harvest(c); }
      else {
        for (int i = 0; i < 512; ++i) { hipEvent_t e; if (hipEventCreate(&e) != hipSuccess) return; p.ev.push_back(e); }
        p.cls.resize(p.ev.size() / 2);
      }
    }
    slot = p.used++;
    p.cls[slot] = cls;
    live = hipEventRecord(p.ev[2 * slot], c->stream) == hipSuccess;
  }
  ~ProfScope() { if (live) (void)hipEventRecord(c->prof.ev[2 * slot + 1], c->stream); }
};

// ---------------------------------------------------------------- perturbation pass
zgr_status upload_lists(zgr_ctx* c) {
  if (!c->lists_dirty) return ZGR_OK;
  HIP_TRY(c, hipMemcpyAsync(c->ws + c->cv.descs, c->descs.data(), sizeof(TensorDesc) * c->descs.size(), hipMemcpyHostToDevice, c->stream));
  if (!c->flat.empty()) HIP_TRY(c, hipMemcpyAsync(c->ws + c->cv.flat, c->flat.data(), sizeof(WorkItem) * c->flat.size(), hipMemcpyHostToDevice, c->stream));
  if (!c->tiles.empty()) HIP_TRY(c, hipMemcpyAsync(c->ws + c->cv.tiles, c->tiles.data(), sizeof(WorkItem) * c->tiles.size(), hipMemcpyHostToDevice, c->stream));
  // the host vectors must outlive the copies
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->lists_dirty = false;
  return ZGR_OK;
}

PerturbArgs perturb_args(zgr_ctx* c, uint64_t step) {
  PerturbArgs a{};
  a.descs = reinterpret_cast<const TensorDesc*>(c->ws + c->cv.descs);
  a.flat = reinterpret_cast<const WorkItem*>(c->ws + c->cv.flat);
  a.tiles = reinterpret_cast<const WorkItem*>(c->ws + c->cv.tiles);
  a.n_flat = (int32_t)c->flat.size(); a.n_tiles = (int32_t)c->tiles.size();
  a.k0 = (uint32_t)c->cfg.seed; a.k1 = (uint32_t)(c->cfg.seed >> 32);
  a.step = (uint32_t)step; a.bits = c->cfg.gauss_bits; a.dtype = c->dtype; a.max_k = c->max_k; a.min_k = c->min_k;
  return a;
}

// The launch arguments `a` with the staging copies of streamed group gi attached (none past the last group).
PerturbArgs with_stage(const zgr_ctx* c, PerturbArgs a, size_t gi) {
  a.n_stage = 0;
  if (gi < c->groups.size()) {
    const std::vector<StageCopy>& cp = c->groups[gi].copies;
    a.n_stage = (int32_t)cp.size();
    for (size_t j = 0; j < cp.size(); ++j) a.stage[j] = cp[j];
  }
  return a;
}

// One pass over all parameters with the arguments `a` (single or batched) and coefficient coef: isotropic tensors
// and resident guided tensors in one launch each, then the streamed groups layer by layer (Sec. 3.3): the launch of
// layer l also pulls the bases of layer l + 1 out of host memory into the other staging slot, so the transfer runs
// under the arithmetic of layer l and needs no second stream; the first launch of the pass pulls layer 0.
zgr_status run_pass(zgr_ctx* c, PerturbArgs a, float coef) {
  const WorkItem* tiles = a.tiles;
  bool staged0 = c->groups.empty();
  if (a.n_flat > 0) {
    PerturbArgs af = staged0 ? a : with_stage(c, a, 0);
    af.n_tiles = 0;
    ProfScope ps(c, ZGR_K_PERTURB_FLAT);
    HIP_TRY(c, launch_perturb_flat(af, coef, nullptr, c->stream, c->n_cu));
    staged0 = true;
  }
  // one tile launch per rank class present; `first` carries the staging copies of streamed group `next`
  auto launch_ranges = [&](const zgr_ctx::TileRange* cls, bool& pending, size_t next) -> zgr_status {
    for (int k_class = 0; k_class < 2; ++k_class) {
      const zgr_ctx::TileRange& r = cls[k_class];
      if (r.end == r.begin) continue;
      PerturbArgs at = pending ? with_stage(c, a, next) : a;
      at.n_stage = pending ? at.n_stage : 0;
      at.tiles = tiles + r.begin; at.n_tiles = (int32_t)(r.end - r.begin); at.n_flat = 0; at.max_k = r.max_k; at.min_k = r.min_k;
      ProfScope ps(c, ZGR_K_PERTURB_TILE);
      HIP_TRY(c, launch_perturb_tile(at, coef, nullptr, c->stream, c->n_cu));
      pending = false;
    }
    return ZGR_OK;
  };
  bool pending = !staged0;
  zgr_status st = launch_ranges(c->res, pending, 0);
  if (st != ZGR_OK) return st;
  if (pending) HIP_TRY(c, launch_stage_only(with_stage(c, a, 0), c->stream));
  for (size_t gi = 0; gi < c->groups.size(); ++gi) {
    pending = gi + 1 < c->groups.size();
    const bool had = pending;
    if ((st = launch_ranges(c->groups[gi].cls, pending, gi + 1)) != ZGR_OK) return st;
    if (had && pending) HIP_TRY(c, launch_stage_only(with_stage(c, a, gi + 1), c->stream));   // a group without tiles still has to pull for its successor
  }
  return ZGR_OK;
}

zgr_status perturb_pass(zgr_ctx* c, uint64_t step, float coef) {
  if (step >> 32) return fail(c, ZGR_ERR_CONFIG, "step must be < 2^32");
  zgr_status st = upload_lists(c);
  if (st != ZGR_OK) return st;
  return run_pass(c, perturb_args(c, step), coef);
}

// One pass theta += sum_i coef[i] Z(seed, steps[i]), n <= kMaxBatch.
zgr_status perturb_pass_batched(zgr_ctx* c, int n, const uint64_t* steps, const float* coef) {
  zgr_status st = upload_lists(c);
  if (st != ZGR_OK) return st;
  PerturbArgs a = perturb_args(c, 0);
  a.n_q = n;
  for (int i = 0; i < n; ++i) { a.qstep[i] = (uint32_t)steps[i]; a.qcoef[i] = coef[i]; }
  return run_pass(c, a, 1.0f);
}

// ---------------------------------------------------------------- forward
const void* T(zgr_ctx* c, int idx) { return c->t[idx].theta; }

zgr_status forward_loss(zgr_ctx* c, const zgr_batch* b, int slot) {
  const zgr_model& m = c->model;
  hipStream_t s = c->stream;
  unsigned char* ws = c->ws;
  double* loss_dev = reinterpret_cast<double*>(ws + c->cv.loss) + slot;
  float* row_loss = reinterpret_cast<float*>(ws + c->cv.row_loss) + (size_t)slot * c->cv.row_loss_stride;
  float* logits = reinterpret_cast<float*>(ws + c->cv.logits);
  const int dt = c->dtype;
  if (m.arch == ZGR_ARCH_LINEAR_LSQ) {
    const zgr_tensor& w = c->t[c->lsq_w];
    { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(0, b->x, w.theta, nullptr, logits, EPI_F32, b->batch, (int)w.rows, (int)w.cols, s)); }
    { ProfScope ps(c, ZGR_K_LOSS);
      HIP_TRY(c, launch_lsq_rows(logits, reinterpret_cast<const float*>(b->y), row_loss, b->batch, (int)w.rows, s));
      HIP_TRY(c, launch_mean_f64(row_loss, b->batch, 1.0 / b->batch, loss_dev, s)); }
    c->last_rows = c->slot_rows[slot] = b->batch; c->last_slot = slot;
    return ZGR_OK;
  }
  const int M = b->batch * b->seq, d = m.d_model, ff = m.d_ff;
  float* x = reinterpret_cast<float*>(ws + c->cv.x);
  void* h = ws + c->cv.h; void* qkv = ws + c->cv.qkv; void* ctx = ws + c->cv.ctx; void* ffb = ws + c->cv.ff;
  const int32_t* tok = reinterpret_cast<const int32_t*>(b->x);
  const bool lm = m.arch == ZGR_ARCH_DECODER_LM;
  { ProfScope ps(c, ZGR_K_EMBED); HIP_TRY(c, launch_embed(dt, tok, T(c, c->tok_emb), T(c, c->pos_emb), x, M, b->seq, d, m.vocab, s)); }
  const int act_epi = m.act == ZGR_ACT_RELU ? EPI_RELU : EPI_GELU;
  // post_ln: the residual stream x is itself normalised after every sum (and after the embeddings), and h is its copy
  // in the storage type; otherwise h = LN(x) feeds each sublayer and x stays the raw sum.
  float* xn = m.post_ln ? x : nullptr;
  if (m.post_ln) { ProfScope ps(c, ZGR_K_NORM); HIP_TRY(c, launch_layernorm(dt, x, T(c, c->lnf_g), T(c, c->lnf_b), h, M, d, m.ln_eps, s, xn)); }
  for (int l = 0; l < m.n_layer; ++l) {
    const Layer& L = c->layers[l];
    if (!m.post_ln) { ProfScope ps(c, ZGR_K_NORM); HIP_TRY(c, launch_layernorm(dt, x, T(c, L.ln1_g), T(c, L.ln1_b), h, M, d, m.ln_eps, s)); }
    { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(dt, h, T(c, L.wq), T(c, L.bq), qkv, EPI_STORE, M, 3 * d, d, s)); }
    { ProfScope ps(c, ZGR_K_ATTN); HIP_TRY(c, launch_attention(dt, qkv, ctx, lm ? nullptr : b->lengths, b->batch, b->seq, d, m.n_head, lm ? 1 : 0, s)); }
    { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(dt, ctx, T(c, L.wo), T(c, L.bo), x, EPI_RESID, M, d, d, s)); }
    { ProfScope ps(c, ZGR_K_NORM);
      HIP_TRY(c, m.post_ln ? launch_layernorm(dt, x, T(c, L.ln1_g), T(c, L.ln1_b), h, M, d, m.ln_eps, s, xn)
                           : launch_layernorm(dt, x, T(c, L.ln2_g), T(c, L.ln2_b), h, M, d, m.ln_eps, s)); }
    { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(dt, h, T(c, L.w1), T(c, L.b1), ffb, act_epi, M, ff, d, s)); }
    { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(dt, ffb, T(c, L.w2), T(c, L.b2), x, EPI_RESID, M, d, ff, s)); }
    if (m.post_ln) { ProfScope ps(c, ZGR_K_NORM); HIP_TRY(c, launch_layernorm(dt, x, T(c, L.ln2_g), T(c, L.ln2_b), h, M, d, m.ln_eps, s, xn)); }
  }
  if (!m.post_ln) { ProfScope ps(c, ZGR_K_NORM); HIP_TRY(c, launch_layernorm(dt, x, T(c, c->lnf_g), T(c, c->lnf_b), h, M, d, m.ln_eps, s)); }
  if (lm) {
    int32_t* tgt = reinterpret_cast<int32_t*>(ws + c->cv.targets);
    { ProfScope ps(c, ZGR_K_LOSS); HIP_TRY(c, launch_lm_targets(tok, tgt, M, b->seq, m.vocab, s)); }
    if (dt == ZGR_BF16) {
      // the logits region holds the cross-entropy partials and, behind them, the target logits
      float* tlogit = logits + (size_t)2 * ce_partials_per_row(m.vocab) * M;
      ProfScope ps(c, ZGR_K_GEMM);
      HIP_TRY(c, launch_gemm_ce_bf16(h, T(c, c->tok_emb), tgt, logits, tlogit, row_loss, M, m.vocab, d, s));
    } else {
      { ProfScope ps(c, ZGR_K_GEMM); HIP_TRY(c, launch_gemm(dt, h, T(c, c->tok_emb), nullptr, logits, EPI_F32, M, m.vocab, d, s)); }
      ProfScope ps(c, ZGR_K_LOSS);
      HIP_TRY(c, launch_ce_rows(logits, tgt, row_loss, M, m.vocab, s));
    }
    { ProfScope ps(c, ZGR_K_LOSS);
      HIP_TRY(c, launch_mean_f64(row_loss, M, 1.0 / ((double)b->batch * (b->seq - 1)), loss_dev, s)); }
    c->last_rows = c->slot_rows[slot] = M; c->last_slot = slot;
  } else {
    { ProfScope ps(c, ZGR_K_LOSS);
      HIP_TRY(c, launch_cls_head(dt, h, T(c, c->cls_w), T(c, c->cls_b), logits, b->batch, b->seq, d, m.n_class, s));
      HIP_TRY(c, launch_ce_rows(logits, reinterpret_cast<const int32_t*>(b->y), row_loss, b->batch, m.n_class, s));
      HIP_TRY(c, launch_mean_f64(row_loss, b->batch, 1.0 / b->batch, loss_dev, s)); }
    c->last_rows = c->slot_rows[slot] = b->batch; c->last_slot = slot;
  }
  return ZGR_OK;
}

zgr_status check_batch(zgr_ctx* c, const zgr_batch* b) {
  if (!b || !b->x) return fail(c, ZGR_ERR_NULL, "batch or batch->x is NULL");
  const zgr_model& m = c->model;
  if (m.arch == ZGR_ARCH_NONE) return fail(c, ZGR_ERR_STATE, "this context has no model: it can only perturb and update");
  if (b->batch < 1 || b->batch > c->max_batch) return fail(c, ZGR_ERR_SHAPE, "batch = %d outside [1, %d]", b->batch, c->max_batch);
  if (m.arch == ZGR_ARCH_LINEAR_LSQ) { if (!b->y) return fail(c, ZGR_ERR_NULL, "batch->y is NULL"); return ZGR_OK; }
  const int min_seq = m.arch == ZGR_ARCH_DECODER_LM ? 2 : 1;      // a next-token target needs two tokens; a classifier reads the first
  if (b->seq < min_seq || b->seq > c->max_seq || b->seq > m.max_pos) return fail(c, ZGR_ERR_SHAPE, "seq = %d outside [%d, min(%d, %d)]", b->seq, min_seq, c->max_seq, m.max_pos);
  if (m.arch == ZGR_ARCH_ENCODER_CLS && (!b->y || !b->lengths)) return fail(c, ZGR_ERR_NULL, "the classifier needs labels and lengths");
  return ZGR_OK;
}

// Map roles to tensors and check shapes against the model.
zgr_status bind_model(zgr_ctx* c) {
  const zgr_model& m = c->model;
  if (m.arch == ZGR_ARCH_NONE) return ZGR_OK;
  auto shape_is = [&](int idx, int64_t r, int64_t cl) { return c->t[idx].rows == r && c->t[idx].cols == cl; };
  if (m.arch == ZGR_ARCH_LINEAR_LSQ) {
    for (size_t i = 0; i < c->t.size(); ++i) if (c->t[i].role == ZGR_ROLE_LSQ_W) { if (c->lsq_w >= 0) return fail(nullptr, ZGR_ERR_SHAPE, "more than one LSQ_W tensor"); c->lsq_w = (int)i; }
    if (c->lsq_w < 0) return fail(nullptr, ZGR_ERR_SHAPE, "the least-squares model needs one ZGR_ROLE_LSQ_W tensor");
    return ZGR_OK;
  }
  c->layers.assign(m.n_layer, Layer());
  const int d = m.d_model, ff = m.d_ff;
  for (size_t i = 0; i < c->t.size(); ++i) {
    const zgr_tensor& t = c->t[i];
    int* slot = nullptr; int64_t r = 1, cl = d;
    const bool in_layer = t.role >= ZGR_ROLE_LN1_G && t.role <= ZGR_ROLE_B2;
    if (in_layer && (t.layer < 0 || t.layer >= m.n_layer)) return fail(nullptr, ZGR_ERR_SHAPE, "tensor %zu: layer %d out of range", i, t.layer);
    Layer* L = in_layer ? &c->layers[t.layer] : nullptr;
    switch (t.role) {
      case ZGR_ROLE_TOK_EMB: slot = &c->tok_emb; r = m.vocab; break;
      case ZGR_ROLE_POS_EMB: slot = &c->pos_emb; r = m.max_pos; break;
      case ZGR_ROLE_LN1_G: slot = &L->ln1_g; break;  case ZGR_ROLE_LN1_B: slot = &L->ln1_b; break;
      case ZGR_ROLE_WQ: slot = &L->wq; r = d; break; case ZGR_ROLE_BQ: slot = &L->bq; break;
      case ZGR_ROLE_WK: slot = &L->wk; r = d; break; case ZGR_ROLE_BK: slot = &L->bk; break;
      case ZGR_ROLE_WV: slot = &L->wv; r = d; break; case ZGR_ROLE_BV: slot = &L->bv; break;
      case ZGR_ROLE_WO: slot = &L->wo; r = d; break; case ZGR_ROLE_BO: slot = &L->bo; break;
      case ZGR_ROLE_LN2_G: slot = &L->ln2_g; break;  case ZGR_ROLE_LN2_B: slot = &L->ln2_b; break;
      case ZGR_ROLE_W1: slot = &L->w1; r = ff; break; case ZGR_ROLE_B1: slot = &L->b1; cl = ff; break;
      case ZGR_ROLE_W2: slot = &L->w2; r = d; cl = ff; break; case ZGR_ROLE_B2: slot = &L->b2; break;
      case ZGR_ROLE_LNF_G: slot = &c->lnf_g; break;  case ZGR_ROLE_LNF_B: slot = &c->lnf_b; break;
      case ZGR_ROLE_CLS_W: slot = &c->cls_w; r = m.n_class; break;
      case ZGR_ROLE_CLS_B: slot = &c->cls_b; cl = m.n_class; break;
      default: return fail(nullptr, ZGR_ERR_SHAPE, "tensor %zu: role %d does not belong to a transformer", i, t.role);
    }
    if (*slot >= 0) return fail(nullptr, ZGR_ERR_SHAPE, "tensor %zu: role %d of layer %d given twice", i, t.role, t.layer);
    if (!shape_is((int)i, r, cl)) return fail(nullptr, ZGR_ERR_SHAPE, "tensor %zu (role %d): shape %lld x %lld, expected %lld x %lld", i, t.role, (long long)t.rows, (long long)t.cols, (long long)r, (long long)cl);
    *slot = (int)i;
  }
  if (c->tok_emb < 0 || c->pos_emb < 0 || c->lnf_g < 0 || c->lnf_b < 0) return fail(nullptr, ZGR_ERR_SHAPE, "embeddings or final LayerNorm missing");
  if (m.arch == ZGR_ARCH_ENCODER_CLS && (c->cls_w < 0 || c->cls_b < 0)) return fail(nullptr, ZGR_ERR_SHAPE, "classification head missing");
  const size_t es = elem_size(c->dtype);
  for (int l = 0; l < m.n_layer; ++l) {
    const Layer& L = c->layers[l];
    const int all[] = {L.ln1_g, L.ln1_b, L.wq, L.bq, L.wk, L.bk, L.wv, L.bv, L.wo, L.bo, L.ln2_g, L.ln2_b, L.w1, L.b1, L.w2, L.b2};
    for (int v : all) if (v < 0) return fail(nullptr, ZGR_ERR_SHAPE, "layer %d: a tensor is missing", l);
    const char* q = (const char*)c->t[L.wq].theta; const char* k = (const char*)c->t[L.wk].theta; const char* v = (const char*)c->t[L.wv].theta;
    if (k != q + (size_t)d * d * es || v != k + (size_t)d * d * es) return fail(nullptr, ZGR_ERR_SHAPE, "layer %d: Wq, Wk, Wv must be adjacent in memory", l);
    const char* bq = (const char*)c->t[L.bq].theta; const char* bk = (const char*)c->t[L.bk].theta; const char* bv = (const char*)c->t[L.bv].theta;
    if (bk != bq + (size_t)d * es || bv != bk + (size_t)d * es) return fail(nullptr, ZGR_ERR_SHAPE, "layer %d: bq, bk, bv must be adjacent in memory", l);
  }
  return ZGR_OK;
}

}  // namespace

// =============================================================================== C ABI
extern "C" {

size_t zgr_workspace_bytes(const zgr_model* model, const zgr_tensor* tensors, int32_t n_t, int32_t max_batch, int32_t max_seq) {
  if (!model || (n_t > 0 && !tensors) || n_t < 0 || max_batch < 0 || max_seq < 0) return 0;
  for (int i = 0; i < n_t; ++i) if (tensors[i].rows < 1 || tensors[i].cols < 1) return 0;
  // sized for the finer of the two Philox groupings so that either gauss_bits fits
  const size_t a = carve(*model, tensors, n_t, max_batch, max_seq, 32).total;
  const size_t b = carve(*model, tensors, n_t, max_batch, max_seq, 16).total;
  return std::max(a, b);
}

zgr_status zgr_init(zgr_ctx** out, const zgr_model* model, const zgr_tensor* tensors, int32_t n_t, const zgr_config* config,
                    void* workspace, size_t workspace_bytes, int32_t max_batch, int32_t max_seq, void* hip_stream) {
  if (!out) return fail(nullptr, ZGR_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!model || !tensors || !config) return fail(nullptr, ZGR_ERR_NULL, "model, tensors or config is NULL");
  if (n_t < 1) return fail(nullptr, ZGR_ERR_SHAPE, "n_t must be >= 1");
  zgr_status st = check_config(nullptr, *config);
  if (st != ZGR_OK) return st;
  for (int i = 0; i < n_t; ++i) {
    st = check_tensor(nullptr, tensors[i], i, config->gauss_bits, true);
    if (st != ZGR_OK) return st;
    if (tensors[i].dtype != tensors[0].dtype) return fail(nullptr, ZGR_ERR_DTYPE, "tensor %d: all tensors must share one dtype", i);
    for (int j = 0; j < i; ++j) if (tensors[j].tensor_id == tensors[i].tensor_id) return fail(nullptr, ZGR_ERR_CONFIG, "tensors %d and %d share tensor_id %u", j, i, tensors[i].tensor_id);
  }
  st = check_model(nullptr, *model, tensors[0].dtype);
  if (st != ZGR_OK) return st;
  if (model->arch != ZGR_ARCH_NONE && (max_batch < 1 || (is_transformer(model->arch) && max_seq < 2))) return fail(nullptr, ZGR_ERR_SHAPE, "max_batch / max_seq too small");
  if (!workspace) return fail(nullptr, ZGR_ERR_NULL, "workspace is NULL");
  if ((uintptr_t)workspace & 255) return fail(nullptr, ZGR_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  zgr_ctx* c = new (std::nothrow) zgr_ctx();
  if (!c) return fail(nullptr, ZGR_ERR_DEVICE, "out of host memory");
  c->model = *model; c->cfg = *config; c->t.assign(tensors, tensors + n_t); c->qb.assign((size_t)n_t, zgr_ctx::QBasis{}); c->hb.assign((size_t)n_t, zgr_ctx::HostBasis{}); c->dtype = tensors[0].dtype;
  c->max_batch = max_batch; c->max_seq = max_seq; c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->cv = carve(*model, tensors, n_t, max_batch, max_seq, config->gauss_bits);
  if (workspace_bytes < c->cv.total) {
    st = fail(nullptr, ZGR_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, c->cv.total);
    delete c; return st;
  }
  c->ws = reinterpret_cast<unsigned char*>(workspace); c->ws_bytes = workspace_bytes;
  st = bind_model(c);
  if (st != ZGR_OK) { delete c; return st; }
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
    delete c; return fail(nullptr, ZGR_ERR_DEVICE, "no usable HIP device");
  }
  c->n_cu = n_cu;
  const RadiusEntry* tab = nullptr;
  if (ensure_radius_table(&tab, c->stream) != hipSuccess) { delete c; return fail(nullptr, ZGR_ERR_DEVICE, "could not set up the device tables"); }
  build_lists(c);
  *out = c;
  return ZGR_OK;
}

zgr_status zgr_set_basis(zgr_ctx* c, int32_t idx, const float* U, int32_t k, int32_t ldu) {
  if (!c) return ZGR_ERR_NULL;
  if (idx < 0 || idx >= (int)c->t.size()) return fail(c, ZGR_ERR_SHAPE, "tensor_index %d out of range", idx);
  zgr_tensor t = c->t[idx];
  t.U = (U && k > 0) ? U : nullptr; t.k = (U && k > 0) ? k : 0; t.ldu = ldu;
  zgr_status st = check_tensor(c, t, idx, c->cfg.gauss_bits, true);
  if (st != ZGR_OK) return st;
  c->t[idx] = t;
  c->qb[idx] = zgr_ctx::QBasis{};
  c->hb[idx] = zgr_ctx::HostBasis{};
  build_lists(c);
  if (c->flat.size() > c->cv.cap_flat || c->tiles.size() > c->cv.cap_tiles) return fail(c, ZGR_ERR_WORKSPACE, "work lists outgrew the workspace");
  return ZGR_OK;
}

zgr_status zgr_set_basis_q4(zgr_ctx* c, int32_t idx, const uint8_t* Uq, int32_t k, int32_t ldq, float lambda, float delta) {
  if (!c) return ZGR_ERR_NULL;
  if (idx < 0 || idx >= (int)c->t.size()) return fail(c, ZGR_ERR_SHAPE, "tensor_index %d out of range", idx);
  if (!Uq) return fail(c, ZGR_ERR_NULL, "Uq is NULL");
  if (k < 1) return fail(c, ZGR_ERR_SHAPE, "k must be >= 1");
  if (ldq < (k + 1) / 2) return fail(c, ZGR_ERR_SHAPE, "ldq = %d bytes < (k + 1) / 2 = %d", ldq, (k + 1) / 2);
  if (!std::isfinite(lambda) || !(lambda > 0.f) || !std::isfinite(delta)) return fail(c, ZGR_ERR_CONFIG, "lambda must be positive and finite, delta finite");
  zgr_tensor t = c->t[idx];
  t.U = nullptr; t.k = k; t.ldu = ldq;
  if (t.k > kMaxK) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds %d", idx, t.k, kMaxK);
  if (t.k > t.rows) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds rows = %lld", idx, t.k, (long long)t.rows);
  if (t.cols % group_size(c->cfg.gauss_bits)) return fail(c, ZGR_ERR_SHAPE, "tensor %d: a guided tensor needs cols %% %d == 0", idx, group_size(c->cfg.gauss_bits));
  c->t[idx] = t;
  c->qb[idx].q = Uq; c->qb[idx].lambda = lambda; c->qb[idx].delta = delta;
  c->hb[idx] = zgr_ctx::HostBasis{};
  build_lists(c);
  if (c->flat.size() > c->cv.cap_flat || c->tiles.size() > c->cv.cap_tiles) return fail(c, ZGR_ERR_WORKSPACE, "work lists outgrew the workspace");
  return ZGR_OK;
}

zgr_status zgr_set_basis_host(zgr_ctx* c, int32_t idx, const void* U_host, int32_t k, int32_t bits, float lambda, float delta) {
  if (!c) return ZGR_ERR_NULL;
  if (idx < 0 || idx >= (int)c->t.size()) return fail(c, ZGR_ERR_SHAPE, "tensor_index %d out of range", idx);
  if (!U_host) return fail(c, ZGR_ERR_NULL, "U_host is NULL");
  if (bits != 32 && bits != 4) return fail(c, ZGR_ERR_CONFIG, "bits must be 32 (fp32 basis) or 4 (codes)");
  if (k < 1) return fail(c, ZGR_ERR_SHAPE, "k must be >= 1");
  if ((uintptr_t)U_host & 15) return fail(c, ZGR_ERR_SHAPE, "U_host must be 16-byte aligned");
  if (bits == 4 && (!std::isfinite(lambda) || !(lambda > 0.f) || !std::isfinite(delta))) return fail(c, ZGR_ERR_CONFIG, "lambda must be positive and finite, delta finite");
  zgr_tensor t = c->t[idx];
  if (k > kMaxK) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds %d", idx, k, kMaxK);
  if (k > t.rows) return fail(c, ZGR_ERR_SHAPE, "tensor %d: k = %d exceeds rows = %lld", idx, k, (long long)t.rows);
  if (t.cols % group_size(c->cfg.gauss_bits)) return fail(c, ZGR_ERR_SHAPE, "tensor %d: a guided tensor needs cols %% %d == 0", idx, group_size(c->cfg.gauss_bits));
  // the kernels read this memory themselves: it has to be pinned and mapped into the device's address space
  void* dev = nullptr;
  if (hipHostGetDevicePointer(&dev, const_cast<void*>(U_host), 0) != hipSuccess || !dev) {
    (void)hipGetLastError();
    return fail(c, ZGR_ERR_CONFIG, "U_host is not pinned host memory the device can read (allocate it with hipHostMalloc)");
  }
  const zgr_ctx::HostBasis old_hb = c->hb[idx];
  const zgr_tensor old_t = c->t[idx];
  const zgr_ctx::QBasis old_qb = c->qb[idx];
  t.U = nullptr; t.k = k; t.ldu = bits == 4 ? (k + 1) / 2 : k;
  c->t[idx] = t;
  c->qb[idx] = zgr_ctx::QBasis{};
  c->hb[idx].host = U_host; c->hb[idx].dev = static_cast<const unsigned char*>(dev); c->hb[idx].bits = bits;
  c->hb[idx].lambda = lambda; c->hb[idx].delta = delta;
  // the layer this tensor joins must still fit a staging slot and one launch's list of pieces
  size_t need = 0, members = 0;
  for (size_t i = 0; i < c->t.size(); ++i)
    if (is_streamed(c, i) && c->t[i].layer == t.layer) {
      need += align_up((size_t)c->t[i].rows * (c->hb[i].bits == 4 ? (size_t)(c->t[i].k + 1) / 2 : (size_t)c->t[i].k * 4));
      ++members;
    }
  if (need > c->cv.spc_bytes || members > (size_t)kMaxStage) {
    c->t[idx] = old_t; c->hb[idx] = old_hb; c->qb[idx] = old_qb;
    if (members > (size_t)kMaxStage) return fail(c, ZGR_ERR_SHAPE, "more than %d streamed tensors in layer %d", kMaxStage, t.layer);
    return fail(c, ZGR_ERR_WORKSPACE, "the bases of layer %d need %zu bytes of staging, the workspace holds %zu (sized from the ranks given to zgr_workspace_bytes)", t.layer, need, c->cv.spc_bytes);
  }
  build_lists(c);
  if (c->flat.size() > c->cv.cap_flat || c->tiles.size() > c->cv.cap_tiles) return fail(c, ZGR_ERR_WORKSPACE, "work lists outgrew the workspace");
  return ZGR_OK;
}

zgr_status zgr_dtc_omega(double data_bytes, double bandwidth_bytes_per_s, double t_cc_s, double restore_s_per_byte, double theta,
                         double* omega, int32_t* hidden) {
  if (!omega || !hidden) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if (!(data_bytes > 0) || !(bandwidth_bytes_per_s > 0) || !(t_cc_s >= 0) || !(restore_s_per_byte >= 0) || !(theta > 0 && theta < 1))
    return fail(nullptr, ZGR_ERR_CONFIG, "sizes and bandwidth must be positive, times non-negative, theta in (0, 1)");
  // transfer(w) - client(w) = (D/B - T) - w D ((1 - theta)/B + tau): linear and decreasing in w
  const double gap0 = data_bytes / bandwidth_bytes_per_s - t_cc_s;
  const double slope = data_bytes * ((1.0 - theta) / bandwidth_bytes_per_s + restore_s_per_byte);
  if (gap0 <= 0.0) { *omega = 0.0; *hidden = 1; return ZGR_OK; }
  const double w = gap0 / slope;
  if (w > 1.0) { *omega = 1.0; *hidden = 0; return ZGR_OK; }
  *omega = w; *hidden = 1;
  return ZGR_OK;
}

zgr_status zgr_dtc_memory_factor(int32_t n_layers, double omega, double theta, double* factor) {
  if (!factor) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if (n_layers < 1 || !(omega >= 0 && omega <= 1) || !(theta > 0 && theta < 1))
    return fail(nullptr, ZGR_ERR_CONFIG, "n_layers >= 1, omega in [0, 1], theta in (0, 1)");
  *factor = 1.0 + 2.0 / n_layers - omega * (1.0 - theta) / n_layers;
  return ZGR_OK;
}

zgr_status zgr_quantize_basis(const float* U, int64_t rows, int32_t k, int32_t ldu, uint8_t* Uq, int32_t ldq, float* minmax_dev,
                              float* lambda_out, float* delta_out, void* hip_stream) {
  if (!U || !Uq || !minmax_dev || !lambda_out || !delta_out) return fail(nullptr, ZGR_ERR_NULL, "a pointer is NULL");
  if (rows < 1 || k < 1 || k > kMaxK || ldu < k || ldq < (k + 1) / 2) return fail(nullptr, ZGR_ERR_SHAPE, "bad basis shape");
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  HIP_TRY(nullptr, launch_basis_minmax(U, rows, k, ldu, minmax_dev, s));
  float mm[2] = {0.f, 0.f};
  HIP_TRY(nullptr, hipMemcpyAsync(mm, minmax_dev, sizeof mm, hipMemcpyDeviceToHost, s));
  HIP_TRY(nullptr, hipStreamSynchronize(s));
  if (!std::isfinite(mm[0]) || !std::isfinite(mm[1])) return fail(nullptr, ZGR_ERR_NONFINITE, "the basis holds a non-finite value");
  // lambda = (max - min) / (2^4 - 1), delta = round(-min / lambda), all in fp32 (a constant basis gets lambda = 1)
  float lambda = (mm[1] - mm[0]) / 15.0f;
  if (!(lambda > 0.f)) lambda = 1.0f;
  const float delta = std::nearbyintf(-mm[0] / lambda);
  HIP_TRY(nullptr, launch_basis_quantize(U, rows, k, ldu, lambda, delta, Uq, ldq, s));
  *lambda_out = lambda; *delta_out = delta;
  return ZGR_OK;
}

size_t zgr_cloud_basis_workspace(int64_t rows, int64_t cols, int32_t k) {
  if (rows < 1 || cols < 1 || k < 1 || k > kMaxK) return 0;
  const size_t longer = (size_t)(rows > cols ? rows : cols);
  return 2 * align_up((size_t)rows * k * 4) + align_up((size_t)cols * k * 4) + 256 + align_up((size_t)kCloudMaxParts * longer * k * 4);
}

zgr_status zgr_cloud_basis(const float* const* snapshots, int32_t n_snap, int64_t rows, int64_t cols, int32_t k, const float* omega, int32_t n_iter,
                           float* U, int32_t ldu, int32_t* dependent_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!snapshots || !omega || !U || !workspace) return fail(nullptr, ZGR_ERR_NULL, "a pointer is NULL");
  if (n_snap < 1 || rows < 1 || cols < 1 || k < 1 || k > kMaxK || k > rows || ldu < k || n_iter < 0) return fail(nullptr, ZGR_ERR_SHAPE, "bad shape (1 <= k <= min(rows, 64), ldu >= k, n_iter >= 0)");
  for (int t = 0; t < n_snap; ++t) if (!snapshots[t]) return fail(nullptr, ZGR_ERR_NULL, "snapshot %d is NULL", t);
  if (workspace_bytes < zgr_cloud_basis_workspace(rows, cols, k) || ((uintptr_t)workspace & 255)) return fail(nullptr, ZGR_ERR_WORKSPACE, "workspace too small or not 256-byte aligned");
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  const size_t yb = align_up((size_t)rows * k * 4);
  float* Q = reinterpret_cast<float*>(ws);               // the current orthonormal block
  float* Y = reinterpret_cast<float*>(ws + yb);          // the block being built by a sweep
  float* T = reinterpret_cast<float*>(ws + 2 * yb);      // G_t^T Q of one snapshot
  int* dep = reinterpret_cast<int*>(ws + 2 * yb + align_up((size_t)cols * k * 4));
  float* part = reinterpret_cast<float*>(ws + 2 * yb + align_up((size_t)cols * k * 4) + 256);   // partial sums of the split products
  // Q = orth(sum_t G_t Omega)
  for (int t = 0; t < n_snap; ++t) HIP_TRY(nullptr, launch_cloud_g_t(snapshots[t], rows, cols, omega, k, Q, t > 0, s, part));
  HIP_TRY(nullptr, launch_cloud_orth(Q, rows, k, dep, s));
  // sweeps Q <- orth(sum_t G_t (G_t^T Q))
  for (int it = 0; it < n_iter; ++it) {
    for (int t = 0; t < n_snap; ++t) {
      HIP_TRY(nullptr, launch_cloud_gt_q(snapshots[t], rows, cols, cols, Q, k, k, T, k, 1.0f, 0, s, part));
      HIP_TRY(nullptr, launch_cloud_g_t(snapshots[t], rows, cols, T, k, Y, t > 0, s, part));
    }
    float* tmp = Q; Q = Y; Y = tmp;
    HIP_TRY(nullptr, launch_cloud_orth(Q, rows, k, dep, s));
  }
  HIP_TRY(nullptr, launch_cloud_copy_basis(Q, rows, k, U, ldu, s));
  if (dependent_out) {
    int h = 0;
    HIP_TRY(nullptr, hipMemcpyAsync(&h, dep, sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(nullptr, hipStreamSynchronize(s));
    *dependent_out = h;
  }
  return ZGR_OK;
}

zgr_status zgr_cloud_lsq_gradient(const float* W, const float* X, const float* Y, int32_t batch, int32_t n_out, int32_t n_in, float* G,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!W || !X || !Y || !G || !workspace) return fail(nullptr, ZGR_ERR_NULL, "a pointer is NULL");
  if (batch < 1 || n_out < 1 || n_in < 1) return fail(nullptr, ZGR_ERR_SHAPE, "batch, n_out and n_in must be positive");
  if (workspace_bytes < (size_t)batch * n_out * 4) return fail(nullptr, ZGR_ERR_WORKSPACE, "workspace must hold batch * n_out floats");
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  float* R = reinterpret_cast<float*>(workspace);
  HIP_TRY(nullptr, launch_gemm(0, X, W, nullptr, R, EPI_F32, batch, n_out, n_in, s));                     // X W^T
  HIP_TRY(nullptr, launch_cloud_residual(R, Y, (int64_t)batch * n_out, s));                                // - Y
  HIP_TRY(nullptr, launch_cloud_gt_q(R, batch, n_out, n_out, X, n_in, n_in, G, n_in, 1.0f / (float)batch, 0, s));   // R^T X / B
  return ZGR_OK;
}

}  // extern "C"

namespace {

// Workspace of one backward pass over a batch of `batch` sequences of `seq` tokens (byte offsets).
struct BwCarve {
  struct PerLayer { size_t xin, h1, qkv, ctx, xmid, h2, u, f, x1n, y2; };   // x1n, y2: post-LayerNorm models only
  size_t xout = 0;
  std::vector<PerLayer> layer;
  size_t xfin = 0, hf = 0, logits = 0, targets = 0, row_loss = 0, loss = 0;
  size_t dx = 0, dt = 0, dff = 0, dqkv = 0, P = 0, dS = 0, stats = 0;
  size_t part = 0;                   // chunk sums of the column reductions
  size_t tA = 0, tB = 0, tW = 0;     // bf16 operands of the matrix-core products (bf16 models with a token count that is a multiple of 64)
  bool mfma = false;
  size_t total = 0;
};

BwCarve bw_carve(const zgr_ctx* c, int batch, int seq) {
  BwCarve v;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
  const zgr_model& m = c->model;
  if (m.arch == ZGR_ARCH_LINEAR_LSQ) {
    v.logits = take((size_t)batch * (size_t)c->t[c->lsq_w].rows * 4);
    v.total = off;
    return v;
  }
  const size_t M = (size_t)batch * seq, d = m.d_model, ff = m.d_ff, es = elem_size(c->dtype);
  v.layer.resize(m.n_layer);
  for (int l = 0; l < m.n_layer; ++l) {
    BwCarve::PerLayer& L = v.layer[l];
    L.xin = take(M * d * 4);  L.h1 = take(M * d * es);  L.qkv = take(M * 3 * d * es);  L.ctx = take(M * d * es);
    L.xmid = take(M * d * 4); L.h2 = take(M * d * es);  L.u = take(M * ff * 4);        L.f = take(M * ff * es);
    L.x1n = L.y2 = 0;
    if (m.post_ln) { L.x1n = take(M * d * 4); L.y2 = take(M * d * 4); }
  }
  if (m.post_ln) v.xout = take(M * d * 4);
  v.xfin = take(M * d * 4);
  v.hf = take(M * d * es);
  v.logits = take(m.arch == ZGR_ARCH_DECODER_LM ? M * (size_t)m.vocab * 4 : (size_t)batch * m.n_class * 4);
  v.targets = take(M * 4);
  v.row_loss = take(M * 4);
  v.loss = take(sizeof(double));
  v.dx = take(M * d * 4);
  v.dt = take(M * d * 4);
  v.dff = take(M * ff * 4);
  v.dqkv = take(M * 3 * d * 4);
  v.P = take((size_t)batch * m.n_head * seq * seq * 4);
  v.dS = take((size_t)batch * m.n_head * seq * seq * 4);
  v.stats = take(M * 2 * 4);
  v.part = take(4 * bw_colsum_scratch_floats((int)std::max(std::max(ff, 3 * d), (size_t)m.n_class)));
  v.mfma = c->dtype == ZGR_BF16 && M % 64 == 0;
  if (v.mfma) {
    // widest contraction of a product: the feed-forward width, the three projections side by side, or (decoder) the
    // vocabulary, rounded up to the multiple of 64 the GEMM takes
    const size_t widest = std::max(std::max(ff, 3 * d), m.arch == ZGR_ARCH_DECODER_LM ? align_up((size_t)m.vocab, 64) : (size_t)0);
    v.tA = take(2 * M * widest);
    v.tB = take(2 * M * std::max(ff, d));
    v.tW = take(2 * d * widest);
  }
  v.total = off;
  return v;
}

}  // namespace

extern "C" {

size_t zgr_cloud_backward_workspace(const zgr_ctx* c, int32_t batch, int32_t seq) {
  if (!c || c->model.arch == ZGR_ARCH_NONE || batch < 1 || (c->model.arch != ZGR_ARCH_LINEAR_LSQ && seq < 1)) return 0;
  return bw_carve(c, batch, seq).total;
}

zgr_status zgr_cloud_backward(zgr_ctx* c, const zgr_batch* b, float* const* grads, int32_t n_grads, double* loss_out, void* workspace, size_t workspace_bytes) {
  if (!c) return ZGR_ERR_NULL;
  if (!grads || !loss_out || !workspace) return fail(c, ZGR_ERR_NULL, "grads, loss_out or workspace is NULL");
  zgr_status st = check_batch(c, b);
  if (st != ZGR_OK) return st;
  if (n_grads != (int32_t)c->t.size()) return fail(c, ZGR_ERR_SHAPE, "grads must hold one pointer per tensor (%zu), got %d", c->t.size(), n_grads);
  for (int32_t i = 0; i < n_grads; ++i) if (!grads[i]) return fail(c, ZGR_ERR_NULL, "grads[%d] is NULL", i);
  if ((uintptr_t)workspace & 255) return fail(c, ZGR_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  const zgr_model& m = c->model;
  hipStream_t s = c->stream;
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  const int dt = c->dtype;
  const BwCarve v = bw_carve(c, b->batch, m.arch == ZGR_ARCH_LINEAR_LSQ ? 1 : b->seq);
  if (workspace_bytes < v.total) return fail(c, ZGR_ERR_WORKSPACE, "workspace holds %zu bytes, the pass needs %zu", workspace_bytes, v.total);
  auto F = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  if (m.arch == ZGR_ARCH_LINEAR_LSQ) {
    // L = mean_b ||x_b W^T - y_b||^2 / 2: dW = (X W^T - Y)^T X / B
    const zgr_tensor& w = c->t[c->lsq_w];
    if ((st = forward_loss(c, b, 0)) != ZGR_OK) return st;
    float* R = F(v.logits);
    const float* X = reinterpret_cast<const float*>(b->x);
    HIP_TRY(c, launch_gemm(0, X, w.theta, nullptr, R, EPI_F32, b->batch, (int)w.rows, (int)w.cols, s));
    HIP_TRY(c, launch_cloud_residual(R, reinterpret_cast<const float*>(b->y), (int64_t)b->batch * w.rows, s));
    HIP_TRY(c, launch_cloud_gt_q(R, b->batch, w.rows, w.rows, X, (int)w.cols, w.cols, grads[c->lsq_w], w.cols, 1.0f / (float)b->batch, 0, s));
    HIP_TRY(c, hipMemcpyAsync(c->host_loss, c->ws + c->cv.loss, sizeof(double), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    *loss_out = c->host_loss[0];
    return std::isfinite(*loss_out) ? ZGR_OK : fail(c, ZGR_ERR_NONFINITE, "loss is not finite");
  }
  const int B = b->batch, Tn = b->seq, M = B * Tn, d = m.d_model, ff = m.d_ff, H = m.n_head;
  if (Tn > kBackwardMaxSeq) return fail(c, ZGR_ERR_SHAPE, "seq = %d is beyond the %d keys the backward softmax rule holds per row", Tn, kBackwardMaxSeq);
  if ((int64_t)B * H > 65535) return fail(c, ZGR_ERR_SHAPE, "batch x heads = %lld is beyond the 65535 heads one batched product of the backward attention takes", (long long)B * H);
  const bool lm = m.arch == ZGR_ARCH_DECODER_LM;
  const int32_t* tok = reinterpret_cast<const int32_t*>(b->x);
  const int32_t* lengths = lm ? nullptr : b->lengths;
  const size_t xbytes = (size_t)M * d * 4;
  // The products of the backward half.  fp32 models: the strided fp32 kernel on the operands as they lie.  bf16 models
  // (token count a multiple of 64): the forward pass's matrix-core GEMM, which contracts along the rows of both
  // operands, on bf16 copies written out with the contraction index innermost.
  unsigned char* tA = ws + v.tA; unsigned char* tB = ws + v.tB; unsigned char* tW = ws + v.tW;
  const void* tB_holds = nullptr;                       // the kept activation whose transpose tB holds
  // dA [M, Kp] = dY [M, Np] W [Np, Kp]
  auto input_grad = [&](const float* dy, int Np, const void* W, int Kp, float* out) -> zgr_status {
    const size_t lim = (size_t)1 << 31;                          // the GEMM addresses its operands with 32-bit offsets
    const int Npad = (Np + 63) & ~63;                            // zeros in both operands past Np
    if (v.mfma && (size_t)M * Npad < lim && (size_t)Kp * Npad < lim) {
      HIP_TRY(c, launch_bw_round_bf16(dy, M, Np, Np, tA, Npad, s));
      HIP_TRY(c, launch_bw_transpose_bf16(1, W, Np, Kp, Kp, tW, Npad, s));
      HIP_TRY(c, launch_gemm(ZGR_BF16, tA, tW, nullptr, out, EPI_F32, M, Kp, Npad, s));
    } else {
      HIP_TRY(c, launch_bw_gemm(dt, dy, Np, 1, W, Kp, 1, out, Kp, M, Kp, Np, 1.0f, 0, s));
    }
    return ZGR_OK;
  };
  // y = a W^T + bias with a [M, Kp] kept in the storage type and dy = columns of a row-major array with row stride ldy:
  // dW [Np, Kp] = dy^T a, dbias = column sums of dy
  auto param_grads = [&](const float* dy, int64_t ldy, const void* a, int Np, int Kp, float* dW, float* dbias) -> zgr_status {
    const size_t lim = (size_t)1 << 31;
    if (v.mfma && (size_t)Np * M < lim && (size_t)Kp * M < lim) {
      HIP_TRY(c, launch_bw_transpose_bf16(0, dy, M, Np, ldy, tA, M, s));
      if (tB_holds != a) { HIP_TRY(c, launch_bw_transpose_bf16(1, a, M, Kp, Kp, tB, M, s)); tB_holds = a; }
      HIP_TRY(c, launch_gemm(ZGR_BF16, tA, tB, nullptr, dW, EPI_F32, Np, Kp, M, s));
    } else {
      HIP_TRY(c, launch_bw_gemm(dt, dy, 1, ldy, a, Kp, 1, dW, Kp, Np, Kp, M, 1.0f, 0, s));
    }
    if (dbias) HIP_TRY(c, launch_bw_colsum(dy, M, Np, ldy, dbias, F(v.part), s));
    return ZGR_OK;
  };
  // ---- forward, every layer's intermediate results kept
  const int relu = m.act == ZGR_ACT_RELU ? 1 : 0;
  if (!m.post_ln) {
    HIP_TRY(c, launch_embed(dt, tok, T(c, c->tok_emb), T(c, c->pos_emb), F(v.layer[0].xin), M, Tn, d, m.vocab, s));
    for (int l = 0; l < m.n_layer; ++l) {
      const Layer& L = c->layers[l];
      const BwCarve::PerLayer& W = v.layer[l];
      float* xnext = F(l + 1 < m.n_layer ? v.layer[l + 1].xin : v.xfin);
      HIP_TRY(c, launch_layernorm(dt, F(W.xin), T(c, L.ln1_g), T(c, L.ln1_b), ws + W.h1, M, d, m.ln_eps, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.h1, T(c, L.wq), T(c, L.bq), ws + W.qkv, EPI_STORE, M, 3 * d, d, s));
      HIP_TRY(c, launch_attention(dt, ws + W.qkv, ws + W.ctx, lengths, B, Tn, d, H, lm ? 1 : 0, s));
      HIP_TRY(c, hipMemcpyAsync(F(W.xmid), F(W.xin), xbytes, hipMemcpyDeviceToDevice, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.ctx, T(c, L.wo), T(c, L.bo), F(W.xmid), EPI_RESID, M, d, d, s));
      HIP_TRY(c, launch_layernorm(dt, F(W.xmid), T(c, L.ln2_g), T(c, L.ln2_b), ws + W.h2, M, d, m.ln_eps, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.h2, T(c, L.w1), T(c, L.b1), F(W.u), EPI_F32, M, ff, d, s));
      HIP_TRY(c, launch_bw_act_forward(dt, relu, F(W.u), ws + W.f, (int64_t)M * ff, s));
      HIP_TRY(c, hipMemcpyAsync(xnext, F(W.xmid), xbytes, hipMemcpyDeviceToDevice, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.f, T(c, L.w2), T(c, L.b2), xnext, EPI_RESID, M, d, ff, s));
    }
    HIP_TRY(c, launch_layernorm(dt, F(v.xfin), T(c, c->lnf_g), T(c, c->lnf_b), ws + v.hf, M, d, m.ln_eps, s));
  } else {
    // post-LayerNorm blocks: xfin holds the raw embedding sum, a layer's xin / h1 its normalised input (fp32 / storage type),
    // xmid and y2 the raw sums in front of LN1 and LN2, x1n / h2 the output of LN1
    HIP_TRY(c, launch_embed(dt, tok, T(c, c->tok_emb), T(c, c->pos_emb), F(v.xfin), M, Tn, d, m.vocab, s));
    HIP_TRY(c, launch_layernorm(dt, F(v.xfin), T(c, c->lnf_g), T(c, c->lnf_b), ws + v.layer[0].h1, M, d, m.ln_eps, s, F(v.layer[0].xin)));
    for (int l = 0; l < m.n_layer; ++l) {
      const Layer& L = c->layers[l];
      const BwCarve::PerLayer& W = v.layer[l];
      const bool last = l + 1 == m.n_layer;
      HIP_TRY(c, launch_gemm(dt, ws + W.h1, T(c, L.wq), T(c, L.bq), ws + W.qkv, EPI_STORE, M, 3 * d, d, s));
      HIP_TRY(c, launch_attention(dt, ws + W.qkv, ws + W.ctx, lengths, B, Tn, d, H, lm ? 1 : 0, s));
      HIP_TRY(c, hipMemcpyAsync(F(W.xmid), F(W.xin), xbytes, hipMemcpyDeviceToDevice, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.ctx, T(c, L.wo), T(c, L.bo), F(W.xmid), EPI_RESID, M, d, d, s));
      HIP_TRY(c, launch_layernorm(dt, F(W.xmid), T(c, L.ln1_g), T(c, L.ln1_b), ws + W.h2, M, d, m.ln_eps, s, F(W.x1n)));
      HIP_TRY(c, launch_gemm(dt, ws + W.h2, T(c, L.w1), T(c, L.b1), F(W.u), EPI_F32, M, ff, d, s));
      HIP_TRY(c, launch_bw_act_forward(dt, relu, F(W.u), ws + W.f, (int64_t)M * ff, s));
      HIP_TRY(c, hipMemcpyAsync(F(W.y2), F(W.x1n), xbytes, hipMemcpyDeviceToDevice, s));
      HIP_TRY(c, launch_gemm(dt, ws + W.f, T(c, L.w2), T(c, L.b2), F(W.y2), EPI_RESID, M, d, ff, s));
      HIP_TRY(c, launch_layernorm(dt, F(W.y2), T(c, L.ln2_g), T(c, L.ln2_b), last ? ws + v.hf : ws + v.layer[l + 1].h1, M, d, m.ln_eps, s,
                                  F(last ? v.xout : v.layer[l + 1].xin)));
    }
  }
  // ---- the loss and its gradient with respect to the final hidden states (into dt), head parameters
  float* logits = F(v.logits);
  float* dx = F(v.dx);
  float* dtb = F(v.dt);
  double* loss_dev = reinterpret_cast<double*>(ws + v.loss);
  if (lm) {
    int32_t* tgt = reinterpret_cast<int32_t*>(ws + v.targets);
    const double inv_n = 1.0 / ((double)B * (Tn - 1));
    HIP_TRY(c, launch_lm_targets(tok, tgt, M, Tn, m.vocab, s));
    HIP_TRY(c, launch_gemm(dt, ws + v.hf, T(c, c->tok_emb), nullptr, logits, EPI_F32, M, m.vocab, d, s));
    HIP_TRY(c, launch_ce_rows(logits, tgt, F(v.row_loss), M, m.vocab, s));
    HIP_TRY(c, launch_mean_f64(F(v.row_loss), M, inv_n, loss_dev, s));
    HIP_TRY(c, launch_bw_cross_entropy(logits, tgt, M, m.vocab, (float)inv_n, s));
    // tied head: logits = hf E^T, so dE = dlogits^T hf (the embedding rule adds its share below), dhf = dlogits E
    if ((st = param_grads(logits, m.vocab, ws + v.hf, m.vocab, d, grads[c->tok_emb], nullptr)) != ZGR_OK) return st;
    if ((st = input_grad(logits, m.vocab, T(c, c->tok_emb), d, dtb)) != ZGR_OK) return st;
  } else {
    const int32_t* labels = reinterpret_cast<const int32_t*>(b->y);
    const int C = m.n_class;
    HIP_TRY(c, launch_cls_head(dt, ws + v.hf, T(c, c->cls_w), T(c, c->cls_b), logits, B, Tn, d, C, s));
    HIP_TRY(c, launch_ce_rows(logits, labels, F(v.row_loss), B, C, s));
    HIP_TRY(c, launch_mean_f64(F(v.row_loss), B, 1.0 / B, loss_dev, s));
    HIP_TRY(c, launch_bw_cross_entropy(logits, labels, B, C, 1.0f / (float)B, s));
    // the head reads the first token of each sequence: rows b T of hf
    HIP_TRY(c, launch_bw_gemm(dt, logits, 1, C, ws + v.hf, (int64_t)Tn * d, 1, grads[c->cls_w], d, C, d, B, 1.0f, 0, s));
    HIP_TRY(c, launch_bw_colsum(logits, B, C, C, grads[c->cls_b], F(v.part), s));
    HIP_TRY(c, launch_bw_fill(dtb, (int64_t)M * d, 0.f, s));
    HIP_TRY(c, launch_bw_gemm(dt, logits, C, 1, T(c, c->cls_w), d, 1, dtb, (int64_t)Tn * d, B, d, C, 1.0f, 0, s));
    HIP_TRY(c, launch_bw_fill(grads[c->tok_emb], (int64_t)m.vocab * d, 0.f, s));
  }
  // ---- the blocks in reverse; dx holds dL/d(residual stream) at the block's output
  const int64_t nx = (int64_t)M * d;
  if (m.post_ln) HIP_TRY(c, hipMemcpyAsync(dx, dtb, xbytes, hipMemcpyDeviceToDevice, s));       // the head reads the last LN2's output itself
  else HIP_TRY(c, launch_bw_layernorm(dt, F(v.xfin), T(c, c->lnf_g), dtb, nullptr, dx, F(v.stats), grads[c->lnf_g], grads[c->lnf_b], F(v.part), M, d, m.ln_eps, s));
  for (int l = m.n_layer - 1; l >= 0; --l) {
    const Layer& L = c->layers[l];
    const BwCarve::PerLayer& W = v.layer[l];
    float* dff = F(v.dff);
    float* dqkv = F(v.dqkv);
    // post-LN: x_out = LN2(y2), dx <- dL/dy2
    if (m.post_ln) HIP_TRY(c, launch_bw_layernorm(dt, F(W.y2), T(c, L.ln2_g), dx, nullptr, dx, F(v.stats), grads[L.ln2_g], grads[L.ln2_b], F(v.part), M, d, m.ln_eps, s));
    // x_out (or y2) = x_mid (or x1n) + f W2^T + b2
    if ((st = param_grads(dx, d, ws + W.f, d, ff, grads[L.w2], grads[L.b2])) != ZGR_OK) return st;
    if ((st = input_grad(dx, d, T(c, L.w2), ff, dff)) != ZGR_OK) return st;
    HIP_TRY(c, launch_bw_act(relu, F(W.u), dff, (int64_t)M * ff, s));
    // u = h2 W1^T + b1
    if ((st = param_grads(dff, ff, ws + W.h2, ff, d, grads[L.w1], grads[L.b1])) != ZGR_OK) return st;
    if ((st = input_grad(dff, ff, T(c, L.w1), d, dtb)) != ZGR_OK) return st;
    if (m.post_ln) {
      // h2 = x1n = LN1(y1): dL/dx1n = dx + dh2, then dx <- dL/dy1
      HIP_TRY(c, launch_bw_add(dtb, dx, nx, s));
      HIP_TRY(c, launch_bw_layernorm(dt, F(W.xmid), T(c, L.ln1_g), dtb, nullptr, dx, F(v.stats), grads[L.ln1_g], grads[L.ln1_b], F(v.part), M, d, m.ln_eps, s));
    } else {
      // h2 = LN2(x_mid): dx <- dx + LN2'(dh2)
      HIP_TRY(c, launch_bw_layernorm(dt, F(W.xmid), T(c, L.ln2_g), dtb, dx, dx, F(v.stats), grads[L.ln2_g], grads[L.ln2_b], F(v.part), M, d, m.ln_eps, s));
    }
    // x_mid (or y1) = x_in + ctx Wo^T + bo
    if ((st = param_grads(dx, d, ws + W.ctx, d, d, grads[L.wo], grads[L.bo])) != ZGR_OK) return st;
    if ((st = input_grad(dx, d, T(c, L.wo), d, dtb)) != ZGR_OK) return st;
    HIP_TRY(c, launch_bw_attention(dt, ws + W.qkv, dtb, lengths, B, Tn, d, H, lm ? 1 : 0, F(v.P), F(v.dS), dqkv, s));
    // q, k, v = h1 W{q,k,v}^T + b{q,k,v}: three column blocks of dqkv; Wq, Wk, Wv are adjacent, one [3 d, d] matrix
    const int wi[3] = {L.wq, L.wk, L.wv}, bi[3] = {L.bq, L.bk, L.bv};
    for (int p = 0; p < 3; ++p)
      if ((st = param_grads(dqkv + (size_t)p * d, 3 * d, ws + W.h1, d, d, grads[wi[p]], grads[bi[p]])) != ZGR_OK) return st;
    if ((st = input_grad(dqkv, 3 * d, T(c, L.wq), d, dtb)) != ZGR_OK) return st;
    if (m.post_ln) HIP_TRY(c, launch_bw_add(dx, dtb, nx, s));                                    // h1 = x_in
    else HIP_TRY(c, launch_bw_layernorm(dt, F(W.xin), T(c, L.ln1_g), dtb, dx, dx, F(v.stats), grads[L.ln1_g], grads[L.ln1_b], F(v.part), M, d, m.ln_eps, s));
  }
  // post-LN: x_0 = LNF(embedding sum)
  if (m.post_ln) HIP_TRY(c, launch_bw_layernorm(dt, F(v.xfin), T(c, c->lnf_g), dx, nullptr, dx, F(v.stats), grads[c->lnf_g], grads[c->lnf_b], F(v.part), M, d, m.ln_eps, s));
  HIP_TRY(c, launch_bw_embedding(tok, dx, M, Tn, d, m.vocab, grads[c->tok_emb], grads[c->pos_emb], m.max_pos, s));
  HIP_TRY(c, hipMemcpyAsync(c->host_loss, loss_dev, sizeof(double), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  *loss_out = c->host_loss[0];
  return std::isfinite(*loss_out) ? ZGR_OK : fail(c, ZGR_ERR_NONFINITE, "loss is not finite");
}

zgr_status zgr_perturb(zgr_ctx* c, uint64_t step, float coef) {
  if (!c) return ZGR_ERR_NULL;
  return perturb_pass(c, step, coef);
}

zgr_status zgr_loss(zgr_ctx* c, const zgr_batch* b, double* loss_out) {
  if (!c) return ZGR_ERR_NULL;
  if (!loss_out) return fail(c, ZGR_ERR_NULL, "loss_out is NULL");
  zgr_status st = check_batch(c, b);
  if (st != ZGR_OK) return st;
  st = forward_loss(c, b, 0);
  if (st != ZGR_OK) return st;
  HIP_TRY(c, hipMemcpyAsync(c->host_loss, c->ws + c->cv.loss, sizeof(double), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (c->prof.on) prof_harvest(c);
  *loss_out = c->host_loss[0];
  return std::isfinite(*loss_out) ? ZGR_OK : fail(c, ZGR_ERR_NONFINITE, "loss is not finite");
}

namespace {
// Device address of `scratch` on the current device, looked up once per device.
hipError_t scratch_of_current_device(unsigned char** out) {
  static std::mutex mu;
  static unsigned char* ptr_of[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    unsigned char* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    ptr_of[dev] = ptr;
  }
  *out = ptr_of[dev];
  return hipSuccess;
}
}  // namespace

zgr_status zgr_lsq_loss_static(const float* W, const float* X, const float* Y, int32_t batch, int32_t n_out, int32_t n_in,
                               double* loss_out, void* hip_stream) {
  if (!W || !X || !Y || !loss_out) return fail(nullptr, ZGR_ERR_NULL, "a pointer is NULL");
  if (batch < 1 || n_out < 1 || n_in < 1) return fail(nullptr, ZGR_ERR_SHAPE, "batch, n_out and n_in must be positive");
  if ((size_t)batch > kStaticMaxBatch || (size_t)batch * (size_t)n_out > kStaticPredFloats)
    return fail(nullptr, ZGR_ERR_WORKSPACE, "batch = %d, n_out = %d exceed the static scratch (batch <= %zu, batch * n_out <= %zu): use zgr_loss with a workspace",
                batch, n_out, kStaticMaxBatch, kStaticPredFloats);
  unsigned char* ptr = nullptr;
  HIP_TRY(nullptr, scratch_of_current_device(&ptr));
  float* pred = reinterpret_cast<float*>(ptr);
  float* row_loss = pred + kStaticPredFloats;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  // the three launches of zgr_loss for this model; every word of scratch they read they have written in this call
  HIP_TRY(nullptr, launch_gemm(0, X, W, nullptr, pred, EPI_F32, batch, n_out, n_in, s));
  HIP_TRY(nullptr, launch_lsq_rows(pred, Y, row_loss, batch, n_out, s));
  HIP_TRY(nullptr, launch_mean_f64(row_loss, batch, 1.0 / batch, loss_out, s));
  return ZGR_OK;
}

zgr_status zgr_step(zgr_ctx* c, uint64_t step, const zgr_batch* b, zgr_result* out) {
  if (!c) return ZGR_ERR_NULL;
  if (!out) return fail(c, ZGR_ERR_NULL, "out is NULL");
  zgr_status st = check_batch(c, b);
  if (st != ZGR_OK) return st;
  const float eps = c->cfg.eps;
  if ((st = perturb_pass(c, step, eps)) != ZGR_OK) return st;                 // W + eps Z
  st = forward_loss(c, b, 0);
  zgr_status st2 = perturb_pass(c, step, -2.0f * eps);                        // W - eps Z
  if (st == ZGR_OK && st2 == ZGR_OK) st = forward_loss(c, b, 1);
  const bool fuse = c->cfg.fuse_restore_update != 0;
  zgr_status st3 = ZGR_OK;
  if (!fuse || st != ZGR_OK || st2 != ZGR_OK) {
    st3 = perturb_pass(c, step, eps);                                         // restore
    if (st == ZGR_OK) st = st2 != ZGR_OK ? st2 : st3;
    if (st != ZGR_OK) return st;
  }
  HIP_TRY(c, hipMemcpyAsync(c->host_loss, c->ws + c->cv.loss, 2 * sizeof(double), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  out->loss_plus = c->host_loss[0];
  out->loss_minus = c->host_loss[1];
  out->g = (float)((out->loss_plus - out->loss_minus) / (2.0 * (double)eps));
  const bool finite = std::isfinite(out->loss_plus) && std::isfinite(out->loss_minus);
  if (fuse) {
    // restore and update in one pass: + eps Z - lr g Z; a non-finite loss only restores
    const float lg = c->cfg.lr * out->g;
    const float coef = finite ? eps - lg : eps;
    if ((st = perturb_pass(c, step, coef)) != ZGR_OK) return st;
    if (c->prof.on) HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  if (c->prof.on) prof_harvest(c);
  if (!finite) return fail(c, ZGR_ERR_NONFINITE, "a loss is not finite (L+ = %g, L- = %g)", out->loss_plus, out->loss_minus);
  return ZGR_OK;
}

zgr_status zgr_apply_update(zgr_ctx* c, uint64_t step, float g, float lr) {
  if (!c) return ZGR_ERR_NULL;
  if (!std::isfinite(g) || !std::isfinite(lr)) return fail(c, ZGR_ERR_NONFINITE, "g or lr is not finite");
  const float coef = -(lr * g);
  return perturb_pass(c, step, coef);
}

zgr_status zgr_apply_updates(zgr_ctx* c, int32_t n, const uint64_t* steps, const float* g, float lr) {
  if (!c) return ZGR_ERR_NULL;
  if (n < 0) return fail(c, ZGR_ERR_SHAPE, "n must be >= 0");
  if (n == 0) return ZGR_OK;
  if (!steps || !g) return fail(c, ZGR_ERR_NULL, "steps or g is NULL");
  if (!std::isfinite(lr)) return fail(c, ZGR_ERR_NONFINITE, "lr is not finite");
  for (int i = 0; i < n; ++i) {
    if (steps[i] >> 32) return fail(c, ZGR_ERR_CONFIG, "step must be < 2^32");
    if (!std::isfinite(g[i])) return fail(c, ZGR_ERR_NONFINITE, "g[%d] is not finite", i);
  }
  // kMaxBatch perturbations per pass over the parameters; each pass rounds to the storage type once
  for (int i0 = 0; i0 < n; i0 += kMaxBatch) {
    const int m = n - i0 < kMaxBatch ? n - i0 : kMaxBatch;
    float coef[kMaxBatch];
    for (int i = 0; i < m; ++i) coef[i] = -(lr * g[i0 + i]);
    zgr_status st = perturb_pass_batched(c, m, steps + i0, coef);
    if (st != ZGR_OK) return st;
  }
  return ZGR_OK;
}

void zgr_destroy(zgr_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->prof.ev) (void)hipEventDestroy(e);
  delete c;
}

const char* zgr_last_error(const zgr_ctx* c) { return c ? c->err.c_str() : g_init_error.c_str(); }

zgr_status zgr_profile_enable(zgr_ctx* c, int32_t on) {
  if (!c) return ZGR_ERR_NULL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->prof.used = 0;
  for (int i = 0; i < ZGR_K_COUNT; ++i) { c->prof.ms[i] = 0; c->prof.n[i] = 0; }
  c->prof.on = on != 0;
  c->prof.paused = false;
  return ZGR_OK;
}

zgr_status zgr_profile_pause(zgr_ctx* c, int32_t paused) {
  if (!c) return ZGR_ERR_NULL;
  c->prof.paused = paused != 0;
  return ZGR_OK;
}

zgr_status zgr_profile_read(zgr_ctx* c, double* ms, int64_t* launches) {
  if (!c) return ZGR_ERR_NULL;
  if (!ms || !launches) return fail(c, ZGR_ERR_NULL, "ms or launches is NULL");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  prof_harvest(c);
  for (int i = 0; i < ZGR_K_COUNT; ++i) { ms[i] = c->prof.ms[i]; launches[i] = c->prof.n[i]; }
  return ZGR_OK;
}

// ---------------------------------------------------------------- test-only exports
zgr_status zgr_debug_philox(const uint32_t* ctr, const uint32_t* key, uint32_t* out, int64_t n, void* hip_stream) {
  if (n < 0) return fail(nullptr, ZGR_ERR_SHAPE, "n < 0");
  if (n == 0) return ZGR_OK;
  if (!ctr || !key || !out) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  HIP_TRY(nullptr, launch_debug_philox(ctr, key[0], key[1], out, n, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_gauss(uint64_t seed, uint64_t step, uint32_t tensor_id, int32_t stream, int32_t gauss_bits, int64_t first, int64_t n,
                           float* out, void* hip_stream) {
  if (!out) return fail(nullptr, ZGR_ERR_NULL, "out is NULL");
  if ((gauss_bits != 32 && gauss_bits != 16) || first < 0 || n < 0 || tensor_id >= 0x80000000u || (stream != 0 && stream != 1) || (step >> 32))
    return fail(nullptr, ZGR_ERR_CONFIG, "bad argument");
  HIP_TRY(nullptr, launch_debug_gauss((uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, tensor_id | ((uint32_t)stream << 31), gauss_bits, first, n, out,
                                      reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_fill_z(zgr_ctx* c, int32_t idx, uint64_t step, float* Z) {
  if (!c) return ZGR_ERR_NULL;
  if (!Z) return fail(c, ZGR_ERR_NULL, "Z is NULL");
  if (idx < 0 || idx >= (int)c->t.size()) return fail(c, ZGR_ERR_SHAPE, "tensor_index %d out of range", idx);
  if (step >> 32) return fail(c, ZGR_ERR_CONFIG, "step must be < 2^32");
  zgr_status st = upload_lists(c);
  if (st != ZGR_OK) return st;
  std::vector<WorkItem> fl, tl;
  append_items(c->t[idx], idx, is_guided(c, (size_t)idx), group_size(c->cfg.gauss_bits), fl, tl);
  std::vector<WorkItem>& items = fl.empty() ? tl : fl;
  if (items.size() > c->cv.cap_dbg) return fail(c, ZGR_ERR_WORKSPACE, "debug list outgrew the workspace");
  HIP_TRY(c, hipMemcpyAsync(c->ws + c->cv.dbg, items.data(), sizeof(WorkItem) * items.size(), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  PerturbArgs a = perturb_args(c, step);
  const WorkItem* dbg = reinterpret_cast<const WorkItem*>(c->ws + c->cv.dbg);
  if (!fl.empty()) { a.flat = dbg; a.n_flat = (int32_t)fl.size(); a.n_tiles = 0; HIP_TRY(c, launch_perturb_flat(a, 0.f, Z, c->stream, c->n_cu)); }
  else {
    a.tiles = dbg; a.n_tiles = (int32_t)tl.size(); a.n_flat = 0; a.max_k = a.min_k = c->t[idx].k;
    if (is_streamed(c, (size_t)idx)) {
      // bring the bases of this tensor's layer into their staging slot first
      for (size_t gi = 0; gi < c->groups.size(); ++gi)
        for (int i : c->groups[gi].tensors)
          if (i == idx) HIP_TRY(c, launch_stage_only(with_stage(c, a, gi), c->stream));
    }
    a.n_stage = 0;
    HIP_TRY(c, launch_perturb_tile(a, 0.f, Z, c->stream, c->n_cu));
  }
  return ZGR_OK;
}

zgr_status zgr_debug_set_stage_tiles(zgr_ctx* c, int64_t min_tiles) {
  if (!c) return ZGR_ERR_NULL;
  if (min_tiles < 1) return fail(c, ZGR_ERR_CONFIG, "min_tiles must be >= 1");
  c->min_stage_tiles = (size_t)min_tiles;
  build_lists(c);
  return ZGR_OK;
}

zgr_status zgr_debug_last_row_losses(zgr_ctx* c, float* out, int64_t n) {
  if (!c) return ZGR_ERR_NULL;
  if (!out) return fail(c, ZGR_ERR_NULL, "out is NULL");
  if (c->model.arch == ZGR_ARCH_NONE || n != c->last_rows) return fail(c, ZGR_ERR_SHAPE, "n = %lld, the last forward produced %lld rows", (long long)n, (long long)c->last_rows);
  HIP_TRY(c, hipMemcpyAsync(out, c->ws + c->cv.row_loss + sizeof(float) * (size_t)c->last_slot * c->cv.row_loss_stride, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return ZGR_OK;
}

zgr_status zgr_debug_step_row_losses(zgr_ctx* c, int32_t which, float* out, int64_t n) {
  if (!c) return ZGR_ERR_NULL;
  if (!out) return fail(c, ZGR_ERR_NULL, "out is NULL");
  if (which != 0 && which != 1) return fail(c, ZGR_ERR_CONFIG, "which must be 0 (L+) or 1 (L-)");
  if (c->model.arch == ZGR_ARCH_NONE || n != c->slot_rows[which]) return fail(c, ZGR_ERR_SHAPE, "n = %lld, that forward produced %lld rows", (long long)n, (long long)c->slot_rows[which]);
  HIP_TRY(c, hipMemcpyAsync(out, c->ws + c->cv.row_loss + sizeof(float) * (size_t)which * c->cv.row_loss_stride, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return ZGR_OK;
}

zgr_status zgr_debug_radius_table(int32_t gauss_bits, float* out, void* hip_stream) {
  if (!out) return fail(nullptr, ZGR_ERR_NULL, "out is NULL");
  if (gauss_bits != 32 && gauss_bits != 16) return fail(nullptr, ZGR_ERR_CONFIG, "gauss_bits must be 32 or 16");
  HIP_TRY(nullptr, launch_debug_radius_table(gauss_bits, out, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_cossin_table(int32_t gauss_bits, float* cos_out, float* sin_out, void* hip_stream) {
  if (!cos_out || !sin_out) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if (gauss_bits != 32 && gauss_bits != 16) return fail(nullptr, ZGR_ERR_CONFIG, "gauss_bits must be 32 or 16");
  HIP_TRY(nullptr, launch_debug_cossin_table(gauss_bits, cos_out, sin_out, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_gemm(int32_t dtype, const void* A, const void* W, const void* bias, void* out, int32_t epilogue,
                          int32_t M, int32_t N, int32_t K, void* hip_stream) {
  if (!A || !W || !out) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if ((dtype != ZGR_F32 && dtype != ZGR_BF16) || epilogue < 0 || epilogue > 3) return fail(nullptr, ZGR_ERR_CONFIG, "bad dtype or epilogue");
  if (M < 1 || N < 1 || K < 1 || (dtype == ZGR_BF16 && K % 64)) return fail(nullptr, ZGR_ERR_SHAPE, "bad GEMM shape");
  HIP_TRY(nullptr, launch_gemm(dtype, A, W, bias, out, epilogue, M, N, K, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_rmw(void* buf, size_t bytes, int32_t dtype, float c, int32_t mode, int32_t blocks, void* sink16, void* hip_stream) {
  if (!buf || !sink16) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if (bytes % 16 || ((uintptr_t)buf & 15) || ((uintptr_t)sink16 & 15)) return fail(nullptr, ZGR_ERR_SHAPE, "size and pointers must be multiples of 16 bytes");
  if ((dtype != ZGR_F32 && dtype != ZGR_BF16) || mode < 0 || mode > 2 || blocks < 1 || blocks > (1 << 24)) return fail(nullptr, ZGR_ERR_CONFIG, "bad dtype, mode or grid");
  HIP_TRY(nullptr, launch_debug_rmw(buf, bytes, dtype, c, mode, blocks, sink16, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_issue_rate(int32_t op, int32_t ilp, int32_t blocks, int32_t iters, uint64_t* out, void* hip_stream) {
  if (!out) return fail(nullptr, ZGR_ERR_NULL, "out is NULL");
  if (op < 0 || op > 18 || (ilp != 1 && ilp != 2 && ilp != 4) || blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 20))
    return fail(nullptr, ZGR_ERR_CONFIG, "bad instruction kind, chain count, grid or iteration count");
  HIP_TRY(nullptr, launch_debug_issue(op, ilp, blocks, iters, reinterpret_cast<unsigned long long*>(out), reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_generator_rate(int32_t part, int32_t blocks, int32_t iters, uint64_t* out, void* hip_stream) {
  if (!out) return fail(nullptr, ZGR_ERR_NULL, "out is NULL");
  if (part < 0 || part > 5 || blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 20)) return fail(nullptr, ZGR_ERR_CONFIG, "bad part, grid or iteration count");
  HIP_TRY(nullptr, launch_debug_generator(part, blocks, iters, reinterpret_cast<unsigned long long*>(out), reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

zgr_status zgr_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src) return fail(nullptr, ZGR_ERR_NULL, "NULL argument");
  if (bytes % 16 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return fail(nullptr, ZGR_ERR_SHAPE, "size and pointers must be multiples of 16 bytes");
  HIP_TRY(nullptr, launch_debug_copy(dst, src, bytes, reinterpret_cast<hipStream_t>(hip_stream)));
  return ZGR_OK;
}

}  // extern "C"
